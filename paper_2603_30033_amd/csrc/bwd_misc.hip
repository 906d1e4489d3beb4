// Gradients of the Tucker core and of the head factor from the gradient of the head-mixed cores
// (G_i = sum_a U1[i,a] C[a], Definition "Tucker Attention").
#include "common.h"
#include "params.h"

namespace ta {

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
