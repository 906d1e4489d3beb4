// Weight preparation: the head-mixed cores G_i = sum_a U1[i,a] C[a] (the "x1 U1" of the
// paper's per-head query Qhat = C x1 U1 x2 (X U2)) and G~_i for the post-softmax tensor, and
// transposed / zero-padded copies of the factor matrices, in the operand layouts the MFMA
// kernels read.  One launch; every 64x64 tile of every output is one workgroup: the source is
// read with lanes along its rows (coalesced), summed over core slices in registers, turned
// through an fp32 LDS tile, and written as whole 16-byte chunks in whatever order the output
// layout asks for.
#include "common.h"
#include "params.h"
#include "prep_tile.h"

namespace ta {

template <typename T>
__global__ __launch_bounds__(256) void prep_kernel(PrepArgs args) {
  __shared__ float tile[kPrepTile][kPrepTile + 1];
  prep_tile<T>(args, blockIdx.x, tile);
}

// tiles of one job (the host's prefix sums over jobs use the same count)
int prep_job_blocks(const PrepJob& j) {
  return j.Z * ((j.rows_pad + kPrepTile - 1) / kPrepTile) * ((j.cols_pad + kPrepTile - 1) / kPrepTile);
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
