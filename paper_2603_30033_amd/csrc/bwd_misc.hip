// Small kernels of the backward pass: token-minor copies of token-major matrices (the weight
// gradients contract over tokens, and the MFMA operand fragments want the contraction index
// contiguous), and the gradients of the Tucker core and the head factor from the gradient of the
// head-mixed cores (G_i = sum_a U1[i,a] C[a], Definition "Tucker Attention").
#include "common.h"
#include "params.h"

namespace ta {

// natural index of the element stored at position p of an acc-ordered 32-block
__device__ __forceinline__ int acc_index(int p) { return 8 * ((p >> 2) & 3) + 4 * (p >> 4) + (p & 3); }

// Each thread moves one CE x CE block (CE = elements per 16 bytes) and transposes it in registers:
// CE loads of 16 bytes from CE consecutive token rows, CE stores of 16 bytes to CE consecutive
// output rows.  Lanes are arranged 8 (column chunks) x 8 (token blocks), so every load and every
// store instruction of a wave touches whole 128-byte lines; no LDS.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(TransposeArgs a) {
  constexpr int CE = 16 / sizeof(T);
  typedef T Vec __attribute__((ext_vector_type(CE)));
  const long TP = (long)a.Bsz * a.Npad;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int lc = lane % 8, lt = lane / 8;
  const int t0 = (blockIdx.x * 4 + wave) * 8 * CE + lt * CE;     // first token of this thread's block
  const int c0 = blockIdx.y * 8 * CE + lc * CE;                  // first source column
  if (t0 >= TP || c0 >= a.cols_pad) return;
  const T* src = static_cast<const T*>(a.src);
  Vec in[CE];
#pragma unroll
  for (int i = 0; i < CE; ++i) {
    const int tp = t0 + i;
    long row = tp;
    bool ok = c0 < a.cols;                                       // cols is a multiple of CE
    if (!a.src_padded) {
      const int b = tp / a.Npad, n = tp % a.Npad;
      ok = ok && n < a.N;
      row = (long)b * a.N + n;
    }
    Vec z;
#pragma unroll
    for (int k = 0; k < CE; ++k) z[k] = (T)0.f;
    in[i] = ok ? *reinterpret_cast<const Vec*>(src + row * a.ld + c0) : z;
  }
  T* dst = static_cast<T*>(a.dst);
#pragma unroll
  for (int k = 0; k < CE; ++k) {
    Vec out;
#pragma unroll
    for (int i = 0; i < CE; ++i) out[i] = in[i][k];
    const int col = c0 + k;
    const int c = a.unperm ? (col & ~31) + acc_index(col & 31) : col;
    *reinterpret_cast<Vec*>(dst + (long)c * TP + t0) = out;
  }
}

hipError_t launch_transpose(int dtype, const TransposeArgs& a, hipStream_t s) {
  const long TP = (long)a.Bsz * a.Npad;
  const int ce = dtype == 0 ? 4 : 8;
  dim3 grid((unsigned)((TP + 32 * ce - 1) / (32 * ce)), (unsigned)((a.cols_pad + 8 * ce - 1) / (8 * ce)));
  if (dtype == 0)
    hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(transpose_kernel<bf16>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

// blocks [0, nC): one (a, b) row of dC each, threads over c.  blocks [nC, nC + nH*r1): one dU1
// entry each, a block-wide sum over (b, c).
template <typename T>
__global__ __launch_bounds__(256) void core_grad_kernel(CoreGradArgs g) {
  const long ldg = (long)g.nH * g.D;
  const T* C = static_cast<const T*>(g.C);
  const T* U1 = static_cast<const T*>(g.U1);
  const int nC = g.r1 * g.r2;
  if ((int)blockIdx.x < nC) {
    const int a = blockIdx.x / g.r2, b = blockIdx.x % g.r2;
    for (int c = threadIdx.x; c < g.r3; c += 256) {
      // eight heads per round: their loads are all in flight before the first is used
      float acc = 0.f;
      for (int i0 = 0; i0 < g.nH; i0 += 8) {
        float u[8], v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int i = min(i0 + k, g.nH - 1);
          u[k] = to_f32(U1[(long)i * g.r1 + a]);
          v[k] = g.dG[(long)b * ldg + (long)i * g.D + c];
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) acc += i0 + k < g.nH ? u[k] * v[k] : 0.f;
      }
      g.dC[((long)a * g.r2 + b) * g.r3 + c] = g.scale * acc;
    }
    return;
  }
  const int e = blockIdx.x - nC;
  const int i = e / g.r1, a = e % g.r1;
  float acc = 0.f;
  const int n = g.r2 * g.r3;
  for (int j0 = threadIdx.x; j0 < n; j0 += 8 * 256) {
    float u[8], v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int j = min(j0 + k * 256, n - 1);
      const int b = j / g.r3, c = j % g.r3;
      u[k] = g.dG[(long)b * ldg + (long)i * g.D + c];
      v[k] = to_f32(C[((long)a * g.r2 + b) * g.r3 + c]);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += j0 + k * 256 < n ? u[k] * v[k] : 0.f;
  }
  __shared__ float red[256];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int sft = 128; sft > 0; sft >>= 1) {
    if ((int)threadIdx.x < sft) red[threadIdx.x] += red[threadIdx.x + sft];
    __syncthreads();
  }
  if (threadIdx.x == 0) g.dU1[(long)i * g.r1 + a] = g.scale * red[0];
}

hipError_t launch_core_grad(int dtype, const CoreGradArgs& a, hipStream_t s) {
  const int blocks = a.r1 * a.r2 + a.nH * a.r1;
  if (dtype == 0)
    hipLaunchKernelGGL(core_grad_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(core_grad_kernel<bf16>, dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ta
