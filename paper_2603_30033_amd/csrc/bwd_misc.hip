// Small kernels of the backward pass: token-minor copies of token-major matrices (the weight
// gradients contract over tokens, and the MFMA operand fragments want the contraction index
// contiguous), and the gradients of the Tucker core and the head factor from the gradient of the
// head-mixed cores (G_i = sum_a U1[i,a] C[a], Definition "Tucker Attention").
#include "common.h"
#include "params.h"

namespace ta {

// natural index of the element stored at position p of an acc-ordered 32-block
__device__ __forceinline__ int acc_index(int p) { return 8 * ((p >> 2) & 3) + 4 * (p >> 4) + (p & 3); }

template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(TransposeArgs a) {
  __shared__ float tile[32][33];
  const long TP = (long)a.Bsz * a.Npad;
  const int t0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
  const T* src = static_cast<const T*>(a.src);
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int tp = t0 + ty + 8 * rr;                            // < TP: TP is a multiple of 64
    long row = tp;
    bool ok = c0 + tx < a.cols;
    if (!a.src_padded) {
      const int b = tp / a.Npad, n = tp % a.Npad;
      ok = ok && n < a.N;
      row = (long)b * a.N + n;
    }
    tile[ty + 8 * rr][tx] = ok ? to_f32(src[row * a.ld + c0 + tx]) : 0.f;
  }
  __syncthreads();
  T* dst = static_cast<T*>(a.dst);
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int p = ty + 8 * rr;                                  // stored column position inside the block
    const int c = c0 + (a.unperm ? acc_index(p) : p);
    store1(dst + (long)c * TP + t0 + tx, tile[tx][p]);
  }
}

hipError_t launch_transpose(int dtype, const TransposeArgs& a, hipStream_t s) {
  const long TP = (long)a.Bsz * a.Npad;
  dim3 grid((unsigned)(TP / 32), (unsigned)(a.cols_pad / 32));
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
      float acc = 0.f;
      for (int i = 0; i < g.nH; ++i) acc += to_f32(U1[(long)i * g.r1 + a]) * g.dG[(long)b * ldg + (long)i * g.D + c];
      g.dC[((long)a * g.r2 + b) * g.r3 + c] = g.scale * acc;
    }
    return;
  }
  const int e = blockIdx.x - nC;
  const int i = e / g.r1, a = e % g.r1;
  float acc = 0.f;
  for (int j = threadIdx.x; j < g.r2 * g.r3; j += 256) {
    const int b = j / g.r3, c = j % g.r3;
    acc += g.dG[(long)b * ldg + (long)i * g.D + c] * to_f32(C[((long)a * g.r2 + b) * g.r3 + c]);
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
