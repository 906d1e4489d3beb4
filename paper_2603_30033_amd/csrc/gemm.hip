// Dense products of the Tucker-attention forward that are plain GEMMs, on bf16/fp32 MFMA:
//   projection   [Qlat | K | V](tok) = [U2 | U3 | U~3]^T x(tok)      (Qlat = X U2, K = X U3,
//                V = X U~3 of Section "KV Caching"), with latent RoPE on K in the epilogue
//                (Definition "Latent RoPE": the key rotation is computed once for all heads)
//   latent merge Z(tok) = sum_i G~_i O_i(tok)                          (head merge through the
//                post-softmax core, from the contraction of H1 and H2 over heads)
//   output       Y(tok) = U~2 Z(tok)                                   (output-mode basis; prefill-sized
//                calls with a short contraction use the dedicated kernel of out_proj.hip)
// With a shared key-value latent the projection has no V rows: the K block's accumulators are
// stored unrotated as V (and as the cache row) before they are rotated.
// All three compute acc[m][tok] = sum_k A[m][k] B[tok][k] with the weight side as MFMA rows
// and tokens as MFMA columns, so that an accumulator lane owns one token and four
// consecutive output channels per register quad.
//
// Tiling: workgroup = 4 waves, tile TM x TN (weights x tokens), contraction staged through
// LDS in slices of 64 elements, double buffered, fed from a ring of register slots that keeps
// three slices in flight; LDS rows are padded by 16 bytes so that the 16-byte fragment reads of
// 8 consecutive rows fall into distinct bank groups.  Token counts of a decode step run the same
// kernel with the contraction split over workgroups and a second kernel that sums the parts.
#include <type_traits>

#include "common.h"
#include "params.h"
#include "epilogue.h"

namespace ta {

constexpr int kKS = 64;   // contraction elements per LDS stage

template <typename T> struct Lds {
  static constexpr int kRowBytes = kKS * sizeof(T) + 16;
  static constexpr int kRowElems = kRowBytes / sizeof(T);
  static constexpr int kChunksPerRow = kKS * sizeof(T) / 16;
  static constexpr int kChunkElems = 16 / sizeof(T);
};

// Copy a [ROWS x kKS] slice of a row-major matrix into registers / from registers into LDS.
// Each thread moves ROWS*chunks/256 16-byte chunks.  Loads are buffer loads whose range check
// supplies the zeros: a chunk of a row that does not exist, or past the end of the contraction,
// gets an offset beyond the descriptor's size.  No load sits behind a branch, so the compiler
// can keep several slices in flight and wait for exactly the one it stores next.
template <typename T, int ROWS> struct Stager {
  static constexpr int kChunks = ROWS * Lds<T>::kChunksPerRow;
  static constexpr int kPerThread = (kChunks + 255) / 256;
  static_assert(kChunks % 256 == 0, "tile rows must fill all threads");
  static constexpr uint32_t kNone = 0x80000000u;              // offset no descriptor here reaches
  struct Regs { u32x4 r[kPerThread]; };                        // one slice in flight
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t roff[kPerThread];                                   // byte offset of the chunk at k = 0, or kNone
  int koff[kPerThread];

  // base: first row of the tile; bytes: extent of the matrix from there on; rowoff(row) gives the
  // element offset of tile row `row` from base, or -1 for a row of zeros
  template <class RowOff>
  __device__ __forceinline__ void init(const T* base, long bytes, RowOff rowoff) {
    const long lim = 0x7fffffffl;
    rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(base), 0, (int)(bytes < 0 ? 0 : (bytes > lim ? lim : bytes)),
                                             0x00020000);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      int ci = threadIdx.x + i * 256;
      int row = ci / Lds<T>::kChunksPerRow, cc = ci % Lds<T>::kChunksPerRow;
      koff[i] = cc * Lds<T>::kChunkElems;
      long ro = rowoff(row);
      roff[i] = ro < 0 ? kNone : (uint32_t)((ro + koff[i]) * (long)sizeof(T));
    }
  }
  __device__ __forceinline__ void load(Regs& R, int k0, int K) const {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const bool ok = roff[i] != kNone && k0 + koff[i] < K;
      const uint32_t off = ok ? roff[i] + (uint32_t)k0 * (uint32_t)sizeof(T) : kNone;
      R.r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
    }
  }
  __device__ __forceinline__ void store(const Regs& R, T* lds) const {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      int ci = threadIdx.x + i * 256;
      int row = ci / Lds<T>::kChunksPerRow, cc = ci % Lds<T>::kChunksPerRow;
      *reinterpret_cast<u32x4*>(lds + row * Lds<T>::kRowElems + cc * Lds<T>::kChunkElems) = R.r[i];
    }
  }
};

// Output tile of one wave written as whole rows: accumulators go to a wave-private LDS patch as
// [token][channel], then 16-byte chunks of consecutive channels are stored, eight rows per
// instruction (the accumulator layout itself would store 8-byte pieces 8 KB apart).
template <typename T, int MB, int NB>
__device__ __forceinline__ void store_rows_y(const GemmArgs& g, const f32x16 (&acc)[MB][NB], T* patch,
                                             int m_base, int t_base) {
  constexpr int CW = MB * 32;                                   // channels per patch row
  constexpr int PRE = CW + 16 / sizeof(T);                      // padded row, elements
  constexpr int CE = 16 / sizeof(T);
  constexpr int CPR = CW / CE;                                  // chunks per row
  const int lane = threadIdx.x % kWave, h = lane / 32, lr = lane % 32;
  const int TP = g.Bsz * g.Npad;
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        store4(patch + (j * 32 + lr) * PRE + i * 32 + 8 * q + 4 * h, acc[i][j][4 * q], acc[i][j][4 * q + 1],
               acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
  T* Y = static_cast<T*>(g.Out);
#pragma unroll
  for (int it = 0; it < NB * 32 * CPR / kWave; ++it) {
    const int ci = it * kWave + lane;
    const int row = ci / CPR, cc = ci % CPR;
    const int tp = t_base + row, m = m_base + cc * CE;
    if (tp >= TP || m >= g.M) continue;
    const int b = tp / g.Npad, n = tp % g.Npad;
    if (n >= g.N) continue;
    u32x4 v = *reinterpret_cast<const u32x4*>(patch + row * PRE + cc * CE);
    *reinterpret_cast<u32x4*>(Y + ((long)b * g.N + n) * g.ldo + m) = v;
  }
}

// TM x TN tile, WGM x WGN waves
template <typename T, int TM, int TN, int WGM, int WGN>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
  static_assert(WGM * WGN == 4, "four waves");
  constexpr int MB = TM / WGM / 32, NB = TN / WGN / 32;
  constexpr int RE = Lds<T>::kRowElems;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);
  // stage s: A rows [TM], then B rows [TN]
  auto stageA = [&](int s) { return smem + (long)s * (TM + TN) * RE; };
  auto stageB = [&](int s) { return smem + (long)s * (TM + TN) * RE + TM * RE; };

  // Workgroups go to the eight XCDs round-robin in dispatch order (x fastest).  Remap the index
  // so that each XCD works through one contiguous range of (token tile, weight tile) pairs: the
  // weight tiles of one token tile then run on the same XCD back to back, and the token rows
  // they share are fetched into that XCD's L2 once.
  int bx = blockIdx.x, by = blockIdx.y;
  {
    const int gx = gridDim.x, per = gridDim.x * gridDim.y / 8;
    const int lin = bx + gx * by;
    if (lin < per * 8) {
      const int logical = (lin % 8) * per + lin / 8;
      bx = logical % gx;
      by = logical / gx;
    }
  }
  const int m_tile = bx * TM, t_tile = by * TN;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int wm = wave % WGM, wn = wave / WGM;
  const int h = lane / 32, lr = lane % 32;
  const int TP = g.Bsz * g.Npad;

  const T* A = static_cast<const T*>(g.A);
  const T* Bs = static_cast<const T*>(g.Bsrc);
  // tile rows as offsets from the tile's first row; rows that do not exist read as zeros
  const T* baseA = A + (long)m_tile * g.lda;
  const long bytesA = (long)(g.M - m_tile) * g.lda * (long)sizeof(T);
  auto rowA = [&](int r) -> long { return m_tile + r < g.M ? (long)r * g.lda : -1l; };
  // token rows: the workspace copies are padded per sequence, the caller's X is not
  const long TR = g.src_padded ? (long)TP : (long)g.Bsz * g.N;  // rows the source holds
  auto src_row = [&](int tp) -> long {                          // source row of padded token tp, -1 if none
    if (tp >= TP) return -1l;
    if (g.src_padded) return tp;
    int b = tp / g.Npad, n = tp % g.Npad;
    return n < g.N ? (long)b * g.N + n : -1l;
  };
  long row0 = TR;                                               // first source row the tile touches
  {
    const int tp = t_tile < TP ? t_tile : TP;
    if (g.src_padded) row0 = tp;
    else if (tp < TP) row0 = (long)(tp / g.Npad) * g.N + min(tp % g.Npad, g.N);
  }
  const T* baseB = Bs + row0 * g.ldb;
  const long bytesB = (TR - row0) * g.ldb * (long)sizeof(T);
  auto rowB = [&](int r) -> long {
    long sr = src_row(t_tile + r);
    return sr < 0 ? -1l : (sr - row0) * g.ldb;
  };

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Slices of the contraction travel global -> registers -> LDS.  PF slices are in flight in
  // registers so that a round trip to memory is hidden behind PF-1 slices of MFMA work.
  constexpr int PF = sizeof(T) == 2 ? 3 : 2;
  Stager<T, TM> sa;
  Stager<T, TN> sb;
  typename Stager<T, TM>::Regs ra[PF];
  typename Stager<T, TN>::Regs rb[PF];
  const int nk_all = (g.K + kKS - 1) / kKS;
  const int per = (nk_all + g.ksplit - 1) / g.ksplit;
  const int ks0 = blockIdx.z * per;
  const int nk = min(nk_all, ks0 + per);
  const int klim = min(g.K, nk * kKS);                          // nothing is fetched past this split
  const int cnt = nk - ks0;
  auto kof = [&](int i) { return i < cnt ? (ks0 + i) * kKS : klim; };
  sa.init(baseA, bytesA, rowA);
  sb.init(baseB, bytesB, rowB);
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    sa.load(ra[u], kof(u), klim);
    sb.load(rb[u], kof(u), klim);
  }
  sa.store(ra[0], stageA(0));
  sb.store(rb[0], stageB(0));
  sa.load(ra[0], kof(PF), klim);
  sb.load(rb[0], kof(PF), klim);
  __syncthreads();

  // One slice: multiply from LDS, then move the next slice from its register slot to the other
  // LDS stage and refill that slot at once with the slice PF further on.  A slot is never idle,
  // so its registers are not handed to anything else while a load into them is in flight.
  auto slice = [&](auto slot_c, int ks) {
    constexpr int S1 = (decltype(slot_c)::value + 1) % PF;      // slot of slice ks + 1
    const int cur = (ks - ks0) & 1;
    const T* la = stageA(cur) + (wm * MB * 32 + lr) * RE + 16 * h;
    const T* lb = stageB(cur) + (wn * NB * 32 + lr) * RE + 16 * h;
#pragma unroll
    for (int kb = 0; kb < kKS / 32; ++kb) {
      Frag<T> fa[MB], fb[NB];
#pragma unroll
      for (int i = 0; i < MB; ++i) fa[i] = load_frag<T>(la + i * 32 * RE + kb * 32);
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[j] = load_frag<T>(lb + j * 32 * RE + kb * 32);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) mma32(acc[i][j], fa[i], fb[j]);
    }
    // (after the last slice this stages and fetches zeros: cheaper than a branch, behind which
    // the compiler would have to wait for every load in flight)
    sa.store(ra[S1], stageA(cur ^ 1));
    sb.store(rb[S1], stageB(cur ^ 1));
    sa.load(ra[S1], kof(ks - ks0 + 1 + PF), klim);
    sb.load(rb[S1], kof(ks - ks0 + 1 + PF), klim);
    __syncthreads();
  };
  // whole groups of PF slices run as one straight-line loop body; the remainder follows
  int ks = ks0;
  for (; ks + PF <= nk; ks += PF) {
    slice(std::integral_constant<int, 0>{}, ks);
    if (PF > 1) slice(std::integral_constant<int, 1 % PF>{}, ks + 1);
    if (PF > 2) slice(std::integral_constant<int, 2 % PF>{}, ks + 2);
  }
  if (ks < nk) slice(std::integral_constant<int, 0>{}, ks);
  if (PF > 2 && ks + 1 < nk) slice(std::integral_constant<int, 1 % PF>{}, ks + 1);

  if (g.epi == 2 && g.ksplit <= 1) {                            // Y: whole rows through LDS
    constexpr int PatchElems = NB * 32 * (MB * 32 + 16 / sizeof(T));
    store_rows_y<T, MB, NB>(g, acc, smem + wave * PatchElems, m_tile + wm * MB * 32, t_tile + wn * NB * 32);
    return;
  }

#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      int m0 = m_tile + (wm * MB + i) * 32;
      int tp = t_tile + (wn * NB + j) * 32 + lr;
      const int Mp = (g.epi == 0) ? g.R2 + (g.shared_kv ? 1 : 2) * g.D : pad32(g.M);
      if (m0 >= Mp) continue;
      if (g.ksplit > 1) {
        if (tp < TP) {
          float* dst = g.part + ((long)blockIdx.z * TP + tp) * Mp + m0 + 4 * h;
#pragma unroll
          for (int q = 0; q < 4; ++q)
            store4(dst + 8 * q, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        }
      } else {
        epilogue_block<T>(g, acc[i][j], m0, tp);
      }
    }
}

// sum of split-K partial tiles, then the ordinary epilogue; one wave per 32x32 block
template <typename T>
__global__ __launch_bounds__(64) void splitk_reduce_kernel(GemmArgs g) {
  const int lane = threadIdx.x, h = lane / 32, lr = lane % 32;
  const int TP = g.Bsz * g.Npad;
  const int Mp = (g.epi == 0) ? g.R2 + (g.shared_kv ? 1 : 2) * g.D : pad32(g.M);
  const int m0 = blockIdx.x * 32, tp = blockIdx.y * 32 + lr;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  if (tp < TP) {
    // eight splits at a time: their 32 loads are issued before the first add (a launch this small is all
    // round trips to memory), and the sums are still formed in split order
    constexpr int U = 8;
    for (int z0 = 0; z0 < g.ksplit; z0 += U) {
      f32x4 v[U][4];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int z = min(z0 + u, g.ksplit - 1);
        const float* src = g.part + ((long)z * TP + tp) * Mp + m0 + 4 * h;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[u][q] = *reinterpret_cast<const f32x4*>(src + 8 * q);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (z0 + u < g.ksplit)
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[4 * q + r] += v[u][q][r];
    }
  }
  epilogue_block<T>(g, acc, m0, tp);
}

template <typename T, int TM, int TN, int WGM, int WGN>
static hipError_t launch_one(const GemmArgs& a, int m_rows, hipStream_t s) {
  const int TP = a.Bsz * a.Npad;
  dim3 grid((m_rows + TM - 1) / TM, (TP + TN - 1) / TN, a.ksplit > 1 ? a.ksplit : 1);
  size_t smem = 2ul * (TM + TN) * Lds<T>::kRowBytes;
  auto kern = gemm_kernel<T, TM, TN, WGM, WGN>;
  static LdsOnce lds_once;                                       // one per kernel instantiation
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.ksplit <= 1 || a.defer_reduce) return e;
  dim3 rgrid((m_rows + 31) / 32, (TP + 31) / 32);
  hipLaunchKernelGGL(splitk_reduce_kernel<T>, rgrid, dim3(64), 0, s, a);
  return hipGetLastError();
}

// sum of a.ksplit partial tiles in a.part, then the epilogue (also used by the token-contracting
// products of gemm_tn.hip, which always go through partial tiles)
hipError_t launch_splitk_reduce(int dtype, const GemmArgs& a, hipStream_t s) {
  const int m_rows = (a.epi == 0) ? a.R2 + (a.shared_kv ? 1 : 2) * a.D : a.M;
  const int TP = a.Bsz * a.Npad;
  dim3 rgrid((m_rows + 31) / 32, (TP + 31) / 32);
  if (dtype == 0)
    hipLaunchKernelGGL(splitk_reduce_kernel<float>, rgrid, dim3(64), 0, s, a);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel<bf16>, rgrid, dim3(64), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_gemm(int dtype, const GemmArgs& a, int tile_n, hipStream_t s) {
  const int m_rows = (a.epi == 0) ? a.R2 + (a.shared_kv ? 1 : 2) * a.D : a.M;
  if (dtype == 0) {
    if (tile_n >= 128) return launch_one<float, 128, 128, 2, 2>(a, m_rows, s);
    if (tile_n >= 64) return launch_one<float, 128, 64, 2, 2>(a, m_rows, s);
    return launch_one<float, 128, 32, 4, 1>(a, m_rows, s);
  }
  // 129..192 weight rows (three 64-wide factor blocks): one 192-row tile instead of one full and one
  // half-empty 128-row tile, and the token rows are read once (only when the token tiles alone give
  // every compute unit two workgroups)
  if (tile_n == 64 && m_rows > 128 && m_rows <= 192 && ((long)a.Bsz * a.Npad + 63) / 64 >= 512)
    return launch_one<bf16, 192, 64, 2, 2>(a, m_rows, s);
  // An odd number of 128-row tiles that is a whole number of 96-row tiles (384 rows: query, key and value
  // factors of 128 each) leaves the compute units one and a half workgroups each.  96 x 128 tiles (every wave
  // 96 rows x 32 tokens) give 256 equal workgroups at 8192 tokens and move 224 instead of 256 (192 x 64 tiles)
  // or 288 (128 x 64) rows through LDS per 12288 outputs: 50.0 us against 53.9 (192 x 64) and 56 (128 x 64),
  // event-bracketed.  With fewer tokens than fill the chip that way, 192-row tiles still even out the count.
  if (tile_n == 64 && m_rows % 96 == 0 && (m_rows / 128) % 2 == 1) {
    const long tokens = (long)a.Bsz * a.Npad;
    if ((m_rows / 96) * ((tokens + 127) / 128) >= 256) return launch_one<bf16, 96, 128, 1, 4>(a, m_rows, s);
    if (m_rows % 192 == 0) return launch_one<bf16, 192, 64, 2, 2>(a, m_rows, s);
  }
  if (tile_n >= 128) return launch_one<bf16, 128, 128, 2, 2>(a, m_rows, s);
  if (tile_n >= 64) return launch_one<bf16, 128, 64, 2, 2>(a, m_rows, s);
  return launch_one<bf16, 128, 32, 4, 1>(a, m_rows, s);
}

}  // namespace ta
