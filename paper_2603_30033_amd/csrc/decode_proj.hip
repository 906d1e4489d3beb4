// Factor projection of a decode step (Section "KV Caching" of the paper: the new token's Qlat = x U2,
// K = x U3, V = x U~3) read straight from the caller's factor matrices, so that the step does not wait for
// transposed copies of them; the weight-preparation tiles that the rest of the step does need (the
// head-mixed cores) ride along as the first workgroups of the same launch.
//
// A factor matrix is [K][r] with r contiguous, and an MFMA operand wants the contraction index inside a
// lane: a wave stages a 64 (k) x 32 (columns) piece in LDS as it lies in memory and reads it back with
// transposing LDS loads, which hand a lane its 16 contraction elements in acc order; the token operand is
// fetched in the same order.  One workgroup = one 32-column block of [Qlat | K | V] x one split of the
// contraction; its four waves take the 64-wide slices of the split in turn and add up through LDS; the
// result is a split-K partial tile in the layout of the product kernel, which the query launch sums.
#include "common.h"
#include "params.h"
#include "prep_tile.h"

namespace ta {

template <typename T>
__global__ __launch_bounds__(256) void decode_proj_kernel(DecodeProjArgs a, PrepArgs prep) {
  constexpr int CE = 16 / (int)sizeof(T);
  constexpr int TS = 32 + CE;                                     // padded tile row, elements
  constexpr int CPRW = 32 / CE;                                   // 16-byte chunks per tile row
  constexpr size_t kTileBytes = 4ul * 64 * TS * sizeof(T);
  constexpr size_t kPrepBytes = sizeof(float) * kPrepTile * (kPrepTile + 1);
  constexpr size_t kRedBytes = 4ul * 16 * 64 * sizeof(float);
  constexpr size_t kBytes = kTileBytes > kPrepBytes ? (kTileBytes > kRedBytes ? kTileBytes : kRedBytes)
                                                    : (kPrepBytes > kRedBytes ? kPrepBytes : kRedBytes);
  __shared__ __attribute__((aligned(16))) unsigned char smem[kBytes];

  if ((int)blockIdx.x < prep.total_blocks) {                      // ---- a weight-preparation tile
    prep_tile<T>(prep, blockIdx.x, reinterpret_cast<float(*)[kPrepTile + 1]>(smem));
    return;
  }
  const int wg = blockIdx.x - prep.total_blocks;
  const int Mp = a.R2 + (a.shared_kv ? 1 : 2) * a.D;
  const int nmb = Mp / 32;
  const int mb = wg % nmb, z = wg / nmb;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;

  // the factor matrix this block of 32 product rows comes from, and its first column there
  const int m0 = mb * 32;
  const T* U;
  int col0, ncols;
  if (m0 < a.R2) { U = static_cast<const T*>(a.U2); col0 = m0; ncols = a.r2; }
  else if (m0 < a.R2 + a.D) { U = static_cast<const T*>(a.U3); col0 = m0 - a.R2; ncols = a.r3; }
  else { U = static_cast<const T*>(a.Ut3); col0 = m0 - a.R2 - a.D; ncols = a.rt3; }
  const T* X = static_cast<const T*>(a.X);

  const int nk_all = (a.K + 63) / 64;
  const int per = (nk_all + a.ksplit - 1) / a.ksplit;
  const int ks0 = z * per, nk = min(nk_all, ks0 + per);
  T* tile = reinterpret_cast<T*>(smem) + (long)wave * 64 * TS;    // this wave's 64 x 32 piece

  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  for (int ks = ks0 + wave; ks < nk; ks += 4) {
    const int k0 = ks * 64;
    // factor piece: rows k0.., 16-byte chunks; whatever lies outside the matrix is zero
    u32x4 uv[64 * CPRW / 64];
#pragma unroll
    for (int i = 0; i < 64 * CPRW / 64; ++i) {
      const int ci = lane + 64 * i, row = ci / CPRW, col = col0 + (ci % CPRW) * CE;
      const bool ok = k0 + row < a.K && col < ncols;
      uv[i] = ok ? *reinterpret_cast<const u32x4*>(U + (long)(k0 + row) * ncols + col) : u32x4{0u, 0u, 0u, 0u};
    }
    // token operand in acc order: lane (sequence lr, half h) holds k0 + 32 kb + 8q + 4h + r
    Frag<T> xf[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const T* src = X + (long)min(lr, a.Bsz - 1) * a.K + k0 + kb * 32 + 4 * h;
      const bool row_ok = lr < a.Bsz;
      if constexpr (sizeof(T) == 2) {
        u32x2 piece[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
          piece[q] = row_ok && k0 + kb * 32 + 8 * q + 4 * h < a.K ? *reinterpret_cast<const u32x2*>(src + 8 * q) : u32x2{0u, 0u};
        xf[kb].v[0] = __builtin_bit_cast(bf16x8, u32x4{piece[0][0], piece[0][1], piece[1][0], piece[1][1]});
        xf[kb].v[1] = __builtin_bit_cast(bf16x8, u32x4{piece[2][0], piece[2][1], piece[3][0], piece[3][1]});
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          xf[kb].v[q] = row_ok && k0 + kb * 32 + 8 * q + 4 * h < a.K ? *reinterpret_cast<const f32x4*>(src + 8 * q)
                                                                    : f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int i = 0; i < 64 * CPRW / 64; ++i) {
      const int ci = lane + 64 * i;
      *reinterpret_cast<u32x4*>(tile + (ci / CPRW) * TS + (ci % CPRW) * CE) = uv[i];
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) mma32(acc, load_frag_tr(tile, TS, kb * 32, 0, lane), xf[kb]);
  }
  __syncthreads();                                                // the pieces are done with: LDS becomes the adder

  float* red = reinterpret_cast<float*>(smem);                    // [4 waves][16 registers][64 lanes]
#pragma unroll
  for (int e = 0; e < 16; ++e) red[(wave * 16 + e) * 64 + lane] = acc[e];
  __syncthreads();
  if (wave == 0 && lr < a.Bsz) {
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] += red[(16 + e) * 64 + lane] + red[(32 + e) * 64 + lane] + red[(48 + e) * 64 + lane];
    float* dst = a.part + ((long)z * a.Bsz + lr) * Mp + m0 + 4 * h;
#pragma unroll
    for (int q = 0; q < 4; ++q) store4(dst + 8 * q, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
  }
}

hipError_t launch_decode_proj(int dtype, const DecodeProjArgs& a, const PrepArgs& prep, hipStream_t s) {
  const int Mp = a.R2 + (a.shared_kv ? 1 : 2) * a.D;
  const int blocks = prep.total_blocks + (Mp / 32) * a.ksplit;
  if (dtype == 0)
    hipLaunchKernelGGL(decode_proj_kernel<float>, dim3(blocks), dim3(256), 0, s, a, prep);
  else
    hipLaunchKernelGGL(decode_proj_kernel<bf16>, dim3(blocks), dim3(256), 0, s, a, prep);
  return hipGetLastError();
}

}  // namespace ta
