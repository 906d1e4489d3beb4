// Gradients of the Tucker core and of the head factor from the gradient of the head-mixed cores
// (G_i = sum_a U1[i,a] C[a], Definition "Tucker Attention").
#include "common.h"
#include "params.h"

namespace ta {

// GA core slices a0..a0+GA-1 per workgroup, so that an element of dG is fetched once per GA slices
// (GA grows with the head rank r1: few slices need the parallelism more than the reuse).  blocks [0, nC): rows (a-group, b) of dC, threads over c.  blocks [nC, nC + nH*groups):
// the dU1 entries (i, a-group), a block-wide sum over (b, c).
template <typename T, int GA>
__global__ __launch_bounds__(256) void core_grad_kernel(CoreGradArgs g) {
  constexpr int RD = GA >= 8 ? 4 : 8;                           // elements of dG in flight per thread
  const long ldg = (long)g.nH * g.D;
  const T* C = static_cast<const T*>(g.C);
  const T* U1 = static_cast<const T*>(g.U1);
  const int groups = (g.r1 + GA - 1) / GA;
  const int nC = groups * g.r2;
  if ((int)blockIdx.x < nC) {
    const int a0 = (blockIdx.x / g.r2) * GA, b = blockIdx.x % g.r2;
    for (int c = threadIdx.x; c < g.r3; c += 256) {
      float acc[GA];
#pragma unroll
      for (int u = 0; u < GA; ++u) acc[u] = 0.f;
      // RD heads per round: their loads are all in flight before the first is used
      for (int i0 = 0; i0 < g.nH; i0 += RD) {
        float v[RD], w[RD][GA];
#pragma unroll
        for (int k = 0; k < RD; ++k) {
          const int i = min(i0 + k, g.nH - 1);
          v[k] = i0 + k < g.nH ? g.dG[(long)b * ldg + (long)i * g.D + c] : 0.f;
#pragma unroll
          for (int u = 0; u < GA; ++u) w[k][u] = to_f32(U1[(long)i * g.r1 + min(a0 + u, g.r1 - 1)]);
        }
#pragma unroll
        for (int k = 0; k < RD; ++k)
#pragma unroll
          for (int u = 0; u < GA; ++u) acc[u] += w[k][u] * v[k];
      }
#pragma unroll
      for (int u = 0; u < GA; ++u)
        if (a0 + u < g.r1) g.dC[((long)(a0 + u) * g.r2 + b) * g.r3 + c] = g.scale * acc[u];
    }
    return;
  }
  const int e = blockIdx.x - nC;
  const int i = e / groups, a0 = (e % groups) * GA;
  float acc[GA];
#pragma unroll
  for (int u = 0; u < GA; ++u) acc[u] = 0.f;
  const int n = g.r2 * g.r3;
  for (int j0 = threadIdx.x; j0 < n; j0 += RD * 256) {
    float v[RD], w[RD][GA];
#pragma unroll
    for (int k = 0; k < RD; ++k) {
      const int j = min(j0 + k * 256, n - 1);
      const int b = j / g.r3, c = j % g.r3;
      v[k] = j0 + k * 256 < n ? g.dG[(long)b * ldg + (long)i * g.D + c] : 0.f;
#pragma unroll
      for (int u = 0; u < GA; ++u) w[k][u] = to_f32(C[(long)min(a0 + u, g.r1 - 1) * n + j]);
    }
#pragma unroll
    for (int k = 0; k < RD; ++k)
#pragma unroll
      for (int u = 0; u < GA; ++u) acc[u] += w[k][u] * v[k];
  }
  __shared__ float red[GA][256];
#pragma unroll
  for (int u = 0; u < GA; ++u) red[u][threadIdx.x] = acc[u];
  __syncthreads();
  for (int sft = 128; sft > 0; sft >>= 1) {
    if ((int)threadIdx.x < sft)
#pragma unroll
      for (int u = 0; u < GA; ++u) red[u][threadIdx.x] += red[u][threadIdx.x + sft];
    __syncthreads();
  }
  if (threadIdx.x < GA && a0 + (int)threadIdx.x < g.r1) g.dU1[(long)i * g.r1 + a0 + threadIdx.x] = g.scale * red[threadIdx.x][0];
}

template <typename T, int GA>
static hipError_t core_grad_one(const CoreGradArgs& a, hipStream_t s) {
  const int groups = (a.r1 + GA - 1) / GA;
  const int blocks = groups * a.r2 + a.nH * groups;
  hipLaunchKernelGGL((core_grad_kernel<T, GA>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_core_grad(int dtype, const CoreGradArgs& a, hipStream_t s) {
  if (dtype == 0) {
    if (a.r1 <= 16) return core_grad_one<float, 1>(a, s);
    return core_grad_one<float, 8>(a, s);
  }
  if (a.r1 <= 16) return core_grad_one<bf16, 1>(a, s);
  return core_grad_one<bf16, 8>(a, s);
}

}  // namespace ta
