// Output projection Y(tok) = U~2 Z(tok) (the output-mode basis of the post-softmax tensor,
// Section "Tucker Attention" of the paper) for prefill-sized token counts.
//
// The contraction is only rt2 <= 128 long, so the product is bound by writing Y.  A workgroup
// therefore keeps its 128 token rows of Z in registers as MFMA operand fragments for its whole
// life and walks over tiles of output channels: the U~2 rows of the next tile are fetched while
// the current tile is multiplied, each wave turns its 32 tokens x TM channels of accumulators
// into whole output rows through a wave-private LDS patch, and the stores of one tile overlap
// the products of the next.  One barrier per channel tile.
#include "common.h"
#include "params.h"

namespace ta {

template <typename T, int KB, int TM> struct OutLds {
  static constexpr int kK = KB * 32;
  static constexpr int kARow = kK + 16 / sizeof(T);               // U~2 tile rows, padded by 16 bytes
  static constexpr int kAStage = TM * kARow;
  static constexpr int kPRow = TM + 16 / sizeof(T);               // patch rows: TM channels of one token
  static constexpr int kPatch = 32 * kPRow;
  static constexpr size_t kBytes = (2ul * kAStage + 4ul * kPatch) * sizeof(T);
};

template <typename T, int KB, int TM>
__global__ __launch_bounds__(256) void out_proj_kernel(GemmArgs g, int tiles_per_wg) {
  using L = OutLds<T, KB, TM>;
  constexpr int K = KB * 32, MB = TM / 32;
  constexpr int CE = 16 / sizeof(T);                              // elements per 16-byte chunk
  constexpr int CPR = K / CE;                                     // chunks per U~2 row
  constexpr int APT = TM * CPR / 256;                             // chunks per thread per tile
  static_assert((TM * CPR) % 256 == 0, "tile must fill all threads");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;
  const int TP = g.Bsz * g.Npad;
  const int t_wave = blockIdx.y * 128 + wave * 32;                // first padded token of this wave
  const int m_first = blockIdx.x * tiles_per_wg * TM;
  const int n_tiles = min(tiles_per_wg, (g.M - m_first + TM - 1) / TM);
  if (n_tiles <= 0) return;

  // Z fragments of this wave's 32 tokens (natural order in k); tokens past the end read as zero
  Frag<T> fb[KB];
  {
    const int tp = t_wave + lr;
    const T* Z = static_cast<const T*>(g.Bsrc) + (long)tp * g.ldb + 16 * h;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) fb[kb] = (tp < TP && kb * 32 < g.K) ? load_frag<T>(Z + kb * 32) : zero_frag<T>();
  }

  // U~2 tile rows through buffer loads whose range check supplies zeros for rows past M and for
  // contraction positions past K
  const T* A = static_cast<const T*>(g.A);
  u32x4 areg[APT];
  int arow[APT], acol[APT];
#pragma unroll
  for (int i = 0; i < APT; ++i) {
    const int ci = threadIdx.x + i * 256;
    arow[i] = ci / CPR;
    acol[i] = (ci % CPR) * CE;
  }
  auto a_load = [&](int tile) {
    const int m0 = m_first + tile * TM;
    const long bytes = (long)(g.M - m0) * g.lda * (long)sizeof(T);
    const long lim = 0x7fffffffl;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(A + (long)m0 * g.lda), 0, (int)(bytes < 0 ? 0 : (bytes > lim ? lim : bytes)), 0x00020000);
#pragma unroll
    for (int i = 0; i < APT; ++i) {
      const bool ok = acol[i] < g.K;
      const uint32_t off = ok ? (uint32_t)((arow[i] * g.lda + acol[i]) * (long)sizeof(T)) : 0x80000000u;
      areg[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
    }
  };
  auto a_store = [&](int stage) {
    T* as = smem + (long)stage * L::kAStage;
#pragma unroll
    for (int i = 0; i < APT; ++i) *reinterpret_cast<u32x4*>(as + arow[i] * L::kARow + acol[i]) = areg[i];
  };
  T* patch = smem + 2l * L::kAStage + (long)wave * L::kPatch;
  T* Y = static_cast<T*>(g.Out);

  a_load(0);
  a_store(0);
  __syncthreads();
  for (int tile = 0; tile < n_tiles; ++tile) {
    a_load(min(tile + 1, n_tiles - 1));                           // the last tile is fetched twice
    const T* as = smem + (long)(tile & 1) * L::kAStage + lr * L::kARow + 16 * h;
    f32x16 acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mb][e] = 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        Frag<T> fa = load_frag<T>(as + mb * 32 * L::kARow + kb * 32);
        mma32(acc[mb], fa, fb[kb]);
      }
    // accumulators -> [token][channel] patch -> 16-byte pieces of whole rows
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        store4(patch + lr * L::kPRow + mb * 32 + 8 * q + 4 * h, acc[mb][4 * q], acc[mb][4 * q + 1],
               acc[mb][4 * q + 2], acc[mb][4 * q + 3]);
    const int m0 = m_first + tile * TM;
    constexpr int PCR = TM / CE;                                  // chunks per patch row
#pragma unroll
    for (int it = 0; it < 32 * PCR / kWave; ++it) {
      const int ci = it * kWave + lane;
      const int row = ci / PCR, cc = ci % PCR;
      const int tp = t_wave + row, m = m0 + cc * CE;
      if (tp >= TP || m >= g.M) continue;
      const int b = tp / g.Npad, n = tp % g.Npad;
      if (n >= g.N) continue;
      const u32x4 v = *reinterpret_cast<const u32x4*>(patch + row * L::kPRow + cc * CE);
      *reinterpret_cast<u32x4*>(Y + ((long)b * g.N + n) * g.ldo + m) = v;
    }
    a_store((tile + 1) & 1);
    __syncthreads();
  }
}

template <typename T, int KB, int TM>
static hipError_t out_one(const GemmArgs& a, hipStream_t s) {
  const int TP = a.Bsz * a.Npad;
  const int t_tiles = (TP + 127) / 128, m_tiles = (a.M + TM - 1) / TM;
  // enough workgroups for every compute unit, but as many channel tiles per workgroup as that
  // allows: the Z fragments and the pipeline fill are paid once per workgroup
  int chunks = (256 + t_tiles - 1) / t_tiles;
  if (chunks > m_tiles) chunks = m_tiles;
  if (chunks < 1) chunks = 1;
  const int per = (m_tiles + chunks - 1) / chunks;
  dim3 grid((m_tiles + per - 1) / per, t_tiles);
  size_t smem = OutLds<T, KB, TM>::kBytes;
  auto kern = out_proj_kernel<T, KB, TM>;
  static LdsOnce lds_once;                                       // one per kernel instantiation
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, s, a, per);
  return hipGetLastError();
}

// Requires epi == 2, padded token source, K <= 128, M % (16 / element size) == 0 and 16-byte
// aligned rows; the caller falls back to the generic GEMM otherwise.
bool out_proj_supported(int dtype, const GemmArgs& a) {
  const int ce = dtype == 0 ? 4 : 8;
  return a.epi == 2 && a.src_padded == 1 && a.ksplit <= 1 && a.K <= 128 && a.K % 32 == 0 && a.ldb % ce == 0 &&
         a.lda % ce == 0 && a.M % ce == 0 && a.ldo % ce == 0 && (long)a.lda * 256 * 4 < 0x7fffffffl;
}

hipError_t launch_out_proj(int dtype, const GemmArgs& a, hipStream_t s) {
  const int kb = a.K / 32;
  if (dtype == 0) {
    switch (kb) {
      case 1: return out_one<float, 1, 64>(a, s);
      case 2: return out_one<float, 2, 64>(a, s);
      case 3: return out_one<float, 3, 64>(a, s);
      case 4: return out_one<float, 4, 64>(a, s);
    }
  } else {
    switch (kb) {
      case 1: return out_one<bf16, 1, 128>(a, s);
      case 2: return out_one<bf16, 2, 128>(a, s);
      case 3: return out_one<bf16, 3, 128>(a, s);
      case 4: return out_one<bf16, 4, 128>(a, s);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace ta
