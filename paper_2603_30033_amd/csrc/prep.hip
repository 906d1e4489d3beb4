// Weight preparation: the head-mixed cores G_i = sum_a U1[i,a] C[a] (the "x1 U1" of the
// paper's per-head query Qhat = C x1 U1 x2 (X U2)) and G~_i for the post-softmax tensor, and
// transposed / zero-padded copies of the factor matrices, in the operand layouts the MFMA
// kernels read.  One launch; every 32x32 tile of every output is one workgroup.
#include "common.h"
#include "params.h"

namespace ta {

template <typename T>
__global__ __launch_bounds__(256) void prep_kernel(PrepArgs args) {
  __shared__ float tile[32][33];
  int blk = blockIdx.x;
  int ji = 0;
#pragma unroll
  for (int j = 1; j < kMaxPrepJobs; ++j)
    if (j < args.n_jobs && blk >= args.job[j].first_block) ji = j;
  const PrepJob& jb = args.job[ji];
  int local = blk - jb.first_block;
  int tiles_r = jb.rows_pad / 32, tiles_c = jb.cols_pad / 32;
  int z = local / (tiles_r * tiles_c);
  int rem = local % (tiles_r * tiles_c);
  int r0 = (rem / tiles_c) * 32, c0 = (rem % tiles_c) * 32;
  int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
  const T* src = static_cast<const T*>(jb.src);
  const T* coef = static_cast<const T*>(jb.coef);
  T* out = static_cast<T*>(jb.out);

  // all loads of a batch of up to 8 core slices x 4 rows are issued before the first use, so a
  // workgroup pays for one round trip to memory per batch rather than one per slice
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const int col = c0 + tx;
  if (jb.A == 1) {                                              // plain (transposed) copy of one matrix
    const float w = coef ? to_f32(coef[z]) : 1.f;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int row = min(r0 + ty + 8 * rr, jb.rows - 1);
      acc[rr] = w * to_f32(src[(long)row * jb.cols + min(col, jb.cols - 1)]);
    }
  } else
  for (int a0 = 0; a0 < jb.A; a0 += 8) {
    T v[8][4];
    T cf[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int a = min(a0 + k, jb.A - 1);                      // clamped: slices past the end get weight 0
      cf[k] = coef ? coef[(long)z * jb.A + a] : (T)1.f;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int row = min(r0 + ty + 8 * rr, jb.rows - 1);
        v[k][rr] = src[((long)a * jb.rows + row) * jb.cols + min(col, jb.cols - 1)];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float w = a0 + k < jb.A ? to_f32(cf[k]) : 0.f;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) acc[rr] += w * to_f32(v[k][rr]);
    }
  }
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const bool inside = r0 + ty + 8 * rr < jb.rows && col < jb.cols;
    tile[ty + 8 * rr][tx] = inside ? acc[rr] * jb.scale : 0.f;
  }
  __syncthreads();
  int vpos = jb.perm ? acc_pos(tx) : tx;
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    int a = ty + 8 * rr;
    long u, v;
    float val;
    if (jb.transposed) {
      u = c0 + a; v = r0 + vpos; val = tile[tx][a];
    } else {
      u = r0 + a; v = c0 + vpos; val = tile[a][tx];
    }
    long off;
    if (jb.frag) {
      const int nvb = (jb.transposed ? jb.rows_pad : jb.cols_pad) / 32;
      off = ((u / 32) * nvb + v / 32) * kFragBlockElems + frag_major_offset<T>((int)(u % 32), (int)(v % 32));
    } else {
      off = u * jb.out_stride_u + v;
    }
    store1(out + (long)z * jb.out_stride_z + off, val);
  }
}

hipError_t launch_prep(int dtype, const PrepArgs& a, hipStream_t s) {
  if (a.total_blocks <= 0) return hipSuccess;
  if (dtype == 0)
    hipLaunchKernelGGL(prep_kernel<float>, dim3(a.total_blocks), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(prep_kernel<bf16>, dim3(a.total_blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ta
