// Products that contract over tokens, out[m][n] = sum_t A[t][m] B[t][n], for the weight gradients
// of the backward pass (dU = X^T dLatent, dU~2 = dY^T Z, dG = Qlat^T dQ, dG~ = dZ^T O: the
// derivatives of the factor projections and of the head-mixed cores of Definition "Tucker
// Attention").  Both operands are token-major, as the forward and backward kernels leave them, so
// the contraction index is the slow index in memory.  A slice of 64 tokens of each operand is staged
// row-major in LDS and the MFMA operand fragments, which want the contraction index inside a lane,
// are read with transposing LDS loads (see load_frag_tr in common.h): no token-minor copy of any
// operand is made.  Slices never straddle two sequences; rows of padding tokens read as zeros.
// The contraction is split over workgroups (blockIdx.z); partial tiles are summed, scaled and
// routed to their destinations by splitk_reduce_kernel through epilogue 3 of gemm.hip.
#include <type_traits>

#include "common.h"
#include "params.h"

namespace ta {

constexpr int kTS = 64;   // tokens per LDS stage

// [kTS tokens][COLS columns] slice of a token-major matrix: registers <- global, LDS <- registers
template <typename T, int COLS> struct TnStager {
  static constexpr int CE = 16 / sizeof(T);
  static constexpr int kCPR = COLS / CE;                         // chunks per row
  static constexpr int kChunks = kTS * kCPR;
  static constexpr int kPerThread = kChunks / 256;
  static_assert(kChunks % 256 == 0, "slice must fill all threads");
  // LDS row padded by 64 bytes: the four rows that one transposing read of 16 lanes touches (32
  // bytes each, and the 32 bytes next to them for the neighbouring 16 lanes) then fall into
  // disjoint banks
  static constexpr int kRow = COLS + 64 / (int)sizeof(T);
  static constexpr uint32_t kNone = 0x80000000u;
  struct Regs { u32x4 r[kPerThread]; };
  uint32_t off[kPerThread];                                      // byte offset inside a slice, or kNone
  const T* base; long ld; int padded, N, Npad, spp;              // spp: slices per sequence

  __device__ __forceinline__ void init(const T* mat, long ld_, int col0, int cols, int padded_, int N_, int Npad_) {
    base = mat + col0; ld = ld_; padded = padded_; N = N_; Npad = Npad_; spp = Npad_ / kTS;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int ci = threadIdx.x + i * 256;
      const int row = ci / kCPR, cc = ci % kCPR;
      off[i] = col0 + cc * CE < cols ? (uint32_t)((row * ld_ + cc * CE) * (long)sizeof(T)) : kNone;
    }
  }
  // slice s of the padded token axis: sequence s / spp, tokens (s % spp) * kTS .. + kTS - 1
  __device__ __forceinline__ void load(Regs& R, int s, int s_end) const {
    const int sc = min(s, s_end - 1);
    const int b = sc / spp, n0 = (sc % spp) * kTS;
    const long row0 = padded ? (long)b * Npad + n0 : (long)b * N + n0;
    // rows that exist from row0 on: the descriptor's size makes the others (and a slice past the
    // end of this workgroup's range) read as zeros
    int rows = padded ? kTS : max(0, min(kTS, N - n0));
    if (s >= s_end) rows = 0;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(base + row0 * ld), 0, (int)(rows * ld * (long)sizeof(T)), 0x00020000);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) R.r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off[i], 0, 0);
  }
  __device__ __forceinline__ void store(const Regs& R, T* lds) const {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int ci = threadIdx.x + i * 256;
      const int row = ci / kCPR, cc = ci % kCPR;
      *reinterpret_cast<u32x4*>(lds + row * kRow + cc * CE) = R.r[i];
    }
  }
};

template <typename T, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_tn_kernel(TnArgs a) {
  constexpr int MB = TM / 2 / 32, NB = TN / 2 / 32;
  using SA = TnStager<T, TM>;
  using SB = TnStager<T, TN>;
  constexpr int StageElems = kTS * (SA::kRow + SB::kRow);
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);
  auto stageA = [&](int s) { return smem + (long)s * StageElems; };
  auto stageB = [&](int s) { return smem + (long)s * StageElems + kTS * SA::kRow; };

  const int m_tile = blockIdx.x * TM, n_tile = blockIdx.y * TN;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int wm = wave % 2, wn = wave / 2;
  const int h = lane / 32, lr = lane % 32;

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // this workgroup's range of token slices
  const int n_slices = a.Bsz * (a.Npad / kTS);
  const int per = (n_slices + a.g.ksplit - 1) / a.g.ksplit;
  const int s0 = min((int)blockIdx.z * per, n_slices), s_end = min(n_slices, s0 + per);

  constexpr int PF = sizeof(T) == 2 ? 3 : 2;
  SA sa;
  SB sb;
  typename SA::Regs ra[PF];
  typename SB::Regs rb[PF];
  sa.init(static_cast<const T*>(a.At), a.lda, m_tile, a.g.M, a.a_padded, a.N, a.Npad);
  sb.init(static_cast<const T*>(a.Bt), a.ldb, n_tile, a.g.Npad, a.b_padded, a.N, a.Npad);
  if (s0 < s_end) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      sa.load(ra[u], s0 + u, s_end);
      sb.load(rb[u], s0 + u, s_end);
    }
    sa.store(ra[0], stageA(0));
    sb.store(rb[0], stageB(0));
    sa.load(ra[0], s0 + PF, s_end);
    sb.load(rb[0], s0 + PF, s_end);
    __syncthreads();
    // one slice: multiply from LDS, then move the next slice from its register slot to the other LDS
    // stage and refill that slot at once (a slot is never idle; past the end zeros are fetched)
    auto slice = [&](auto slot_c, int s) {
      constexpr int S1 = (decltype(slot_c)::value + 1) % PF;
      const int cur = (s - s0) & 1;
      const T* la = stageA(cur);
      const T* lb = stageB(cur);
#pragma unroll
      for (int kb = 0; kb < kTS / 32; ++kb) {
        Frag<T> fa[MB], fb[NB];
#pragma unroll
        for (int i = 0; i < MB; ++i) fa[i] = load_frag_tr(la, SA::kRow, kb * 32, (wm * MB + i) * 32, lane);
#pragma unroll
        for (int j = 0; j < NB; ++j) fb[j] = load_frag_tr(lb, SB::kRow, kb * 32, (wn * NB + j) * 32, lane);
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j) mma32(acc[i][j], fa[i], fb[j]);
      }
      sa.store(ra[S1], stageA(cur ^ 1));
      sb.store(rb[S1], stageB(cur ^ 1));
      sa.load(ra[S1], s + 1 + PF, s_end);
      sb.load(rb[S1], s + 1 + PF, s_end);
      __syncthreads();
    };
    int s = s0;
    for (; s + PF <= s_end; s += PF) {
      slice(std::integral_constant<int, 0>{}, s);
      if (PF > 1) slice(std::integral_constant<int, 1 % PF>{}, s + 1);
      if (PF > 2) slice(std::integral_constant<int, 2 % PF>{}, s + 2);
    }
    if (s < s_end) slice(std::integral_constant<int, 0>{}, s);
    if (PF > 2 && s + 1 < s_end) slice(std::integral_constant<int, 1 % PF>{}, s + 1);
  }

  // partial tile -> part[z][n][Mp] (the layout splitk_reduce_kernel sums)
  const int Mp = pad32(a.g.M), NC = a.g.Npad;
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int m0 = m_tile + (wm * MB + i) * 32;
      const int n = n_tile + (wn * NB + j) * 32 + lr;
      if (m0 >= Mp || n >= NC) continue;
      float* dst = a.g.part + ((long)blockIdx.z * NC + n) * Mp + m0 + 4 * h;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        store4(dst + 8 * q, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    }
}

template <typename T, int TM, int TN>
static hipError_t tn_one(const TnArgs& a, hipStream_t s) {
  dim3 grid((a.g.M + TM - 1) / TM, (a.g.Npad + TN - 1) / TN, a.g.ksplit);
  const size_t smem = 2ul * kTS * (TnStager<T, TM>::kRow + TnStager<T, TN>::kRow) * sizeof(T);
  auto kern = gemm_tn_kernel<T, TM, TN>;
  static LdsOnce lds_once;
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, s, a);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  return launch_splitk_reduce(sizeof(T) == 2 ? 1 : 0, a.g, s);
}

// a.g describes the output side as for epilogue 3 of launch_gemm: M rows, Bsz = 1, N = Npad = number
// of columns, ksplit >= 1 partial sums in part, out3 / out_scale / perm_m / perm_n.
hipError_t launch_gemm_tn(int dtype, const TnArgs& a, hipStream_t s) {
  const bool wide = a.g.Npad % 128 == 0;
  if (dtype == 0) return tn_one<float, 128, 64>(a, s);
  return wide ? tn_one<bf16, 128, 128>(a, s) : tn_one<bf16, 128, 64>(a, s);
}

}  // namespace ta
