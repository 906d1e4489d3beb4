// Weight front-ends: classic attention weights -> Tucker-attention weights, on the device.
//   * GQA / MQA / MHA and MLA: the exact representations of the appendix "Tucker Representations
//     of MQA, GQA, and MLA" (selector cores; down-projections as bases, products of the
//     up-projections as core slices).
//   * MHA -> Tucker by a truncated higher-order SVD (appendix "Converting pretrained MHA
//     parameters to approximate attention parameters"), in fp64: Gram matrices of the mode
//     unfoldings from the dH-wide factors, eigenvectors by a one-sided Jacobi iteration, core by
//     contraction with the transposed factors.
#include "../../include/tucker_attn.h"
#include "../../include/tucker_convert.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "common.h"

namespace ta {
namespace {

// ---------------------------------------------------------------------------------------------
// element-wise builders of the exact representations
// ---------------------------------------------------------------------------------------------

template <typename T> __device__ __forceinline__ T from_f64(double v);
template <> __device__ __forceinline__ float from_f64<float>(double v) { return (float)v; }
template <> __device__ __forceinline__ bf16 from_f64<bf16>(double v) { return (bf16)(float)v; }

// C[i][row][col] = 1 iff row = (i,l) and col = (g(i),l); one pass over the whole core
template <typename T>
__global__ __launch_bounds__(256) void selector_core_kernel(T* C, int nH, int dH, int nG) {
  const long rows = (long)nH * dH, cols = (long)nG * dH;
  const long total = (long)nH * rows * cols;
  const int per = nH / nG;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
    const long col = e % cols, row = (e / cols) % rows, i = e / (cols * rows);
    const bool one = row / dH == i && col / dH == i / per && row % dH == col % dH;
    C[e] = from_f64<T>(one ? 1.0 : 0.0);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void identity_kernel(T* U, int n) {
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < (long)n * n; e += (long)gridDim.x * 256)
    U[e] = from_f64<T>(e / n == e % n ? 1.0 : 0.0);
}

// out[c][r] = in[r][c] through a 32x32 LDS tile; in is [rows, cols]
template <typename T>
__global__ __launch_bounds__(256) void transpose_copy_kernel(const T* in, T* out, int rows, int cols) {
  __shared__ T tile[32][33];
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int j = ty; j < 32; j += 8)
    if (r0 + j < rows && c0 + tx < cols) tile[j][tx] = in[(long)(r0 + j) * cols + c0 + tx];
  __syncthreads();
  for (int j = ty; j < 32; j += 8)
    if (c0 + j < cols && r0 + tx < rows) out[(long)(c0 + j) * rows + r0 + tx] = tile[tx][j];
}

// MLA pre-softmax core slice C[i][a][c] = sum_l WUQ[a][(i,l)] WUK[c][(i,l)]
template <typename T>
__global__ __launch_bounds__(256) void mla_core_kernel(const T* WUQ, const T* WUK, T* C, int nH, int dH, int dcQ, int dcK) {
  const long n = (long)nH * dH;
  const long total = (long)nH * dcQ * dcK;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
    const long c = e % dcK, a = (e / dcK) % dcQ, i = e / ((long)dcK * dcQ);
    const T* q = WUQ + a * n + i * dH;
    const T* k = WUK + c * n + i * dH;
    float acc = 0.f;
    for (int l = 0; l < dH; ++l) acc += to_f32(q[l]) * to_f32(k[l]);
    C[e] = from_f64<T>((double)acc);
  }
}

// MLA post-softmax core slice C~[i][(j,l)][c] = (j == i) ? WUV[c][(i,l)] : 0
template <typename T>
__global__ __launch_bounds__(256) void mla_post_core_kernel(const T* WUV, T* Ct, int nH, int dH, int dcK) {
  const long n = (long)nH * dH;
  const long total = (long)nH * n * dcK;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
    const long c = e % dcK, row = (e / dcK) % n, i = e / (dcK * n);
    Ct[e] = row / dH == i ? WUV[c * n + row] : from_f64<T>(0.0);
  }
}

// ---------------------------------------------------------------------------------------------
// fp64 pieces of the higher-order SVD
// ---------------------------------------------------------------------------------------------

// out[r][c] = in[r*sr + c*sc] as fp64, out row-major [rows, cols]
template <typename T>
__global__ __launch_bounds__(256) void to_f64_kernel(const T* in, long sr, long sc, double* out, int rows, int cols) {
  const long total = (long)rows * cols;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256)
    out[e] = (double)to_f32(in[(e / cols) * sr + (e % cols) * sc]);
}

template <typename T>
__global__ __launch_bounds__(256) void from_f64_kernel(const double* in, T* out, long total) {
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) out[e] = from_f64<T>(in[e]);
}

// C[m][n] = sum_k A(m,k) B(k,n) with element strides for every index (any transposition is a
// choice of strides) and a batch stride; 64x64 tile, 16-wide slices, 4x4 results per thread.
struct DgemmArgs {
  const double* A; long a_m, a_k, a_b;
  const double* B; long b_k, b_n, b_b;
  double* C; long c_m, c_n, c_b;
  int M, N, K;
};

__global__ __launch_bounds__(256) void dgemm_kernel(DgemmArgs g) {
  __shared__ double As[16][66], Bs[16][66];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const double* A = g.A + (long)blockIdx.z * g.a_b;
  const double* B = g.B + (long)blockIdx.z * g.b_b;
  double* C = g.C + (long)blockIdx.z * g.c_b;
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  for (int k0 = 0; k0 < g.K; k0 += 16) {
    double va[4], vb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {                       // lanes run along the contiguous index
      const int e = tid + 256 * j;
      const int ka = g.a_k == 1 ? (e & 15) : (e >> 6), ma = g.a_k == 1 ? (e >> 4) : (e & 63);
      const int kb = g.b_n == 1 ? (e >> 6) : (e & 15), nb = g.b_n == 1 ? (e & 63) : (e >> 4);
      va[j] = (m0 + ma < g.M && k0 + ka < g.K) ? A[(long)(m0 + ma) * g.a_m + (long)(k0 + ka) * g.a_k] : 0.0;
      vb[j] = (n0 + nb < g.N && k0 + kb < g.K) ? B[(long)(k0 + kb) * g.b_k + (long)(n0 + nb) * g.b_n] : 0.0;
    }
    __syncthreads();                                    // the previous slice has been consumed
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = tid + 256 * j;
      const int ka = g.a_k == 1 ? (e & 15) : (e >> 6), ma = g.a_k == 1 ? (e >> 4) : (e & 63);
      const int kb = g.b_n == 1 ? (e >> 6) : (e & 15), nb = g.b_n == 1 ? (e & 63) : (e >> 4);
      As[ka][ma] = va[j];
      Bs[kb][nb] = vb[j];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < g.M && n < g.N) C[(long)m * g.c_m + (long)n * g.c_n] = acc[i][j];
    }
}

// M1[i][j] = <W_i, W_j> = sum_{l,m} (A_i^T A_j)[l][m] (B_i^T B_j)[l][m]; GA = A^T A, GB = B^T B [n, n]
__global__ __launch_bounds__(256) void head_gram_kernel(const double* GA, const double* GB, double* M1, int nH, int dH) {
  const int i = blockIdx.y, j = blockIdx.x;
  const long n = (long)nH * dH;
  double s = 0.0;
  for (int e = threadIdx.x; e < dH * dH; e += 256) {
    const long at = ((long)i * dH + e / dH) * n + (long)j * dH + e % dH;
    s += GA[at] * GB[at];
  }
  __shared__ double red[256];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int sft = 128; sft > 0; sft >>= 1) {
    if ((int)threadIdx.x < sft) red[threadIdx.x] += red[threadIdx.x + sft];
    __syncthreads();
  }
  if (threadIdx.x == 0) M1[(long)i * nH + j] = red[0];
}

// sums of up to three doubles over the 256 threads of a block; every thread receives them
__device__ __forceinline__ void block_sum3(double& a, double& b, double& c, double (*red)[3]) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_down(a, o);
    b += __shfl_down(b, o);
    c += __shfl_down(c, o);
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[w][0] = a; red[w][1] = b; red[w][2] = c; }
  __syncthreads();
  a = red[0][0] + red[1][0] + red[2][0] + red[3][0];
  b = red[0][1] + red[1][1] + red[2][1] + red[3][1];
  c = red[0][2] + red[1][2] + red[2][2] + red[3][2];
}

typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

// One step of a blocked one-sided Jacobi sweep on the rows of G [m, len].  The rows are grouped in
// blocks of 8; workgroup k takes the k-th pair (P, Q) of round `step` of a round-robin tournament
// over the blocks (pairs of one round are disjoint, so workgroups touch disjoint rows) and
//   1. forms the 16 x 16 Gram matrix S = R R^T of its 16 rows with the fp64 matrix instruction
//      (D[16x16] += A[16x4] B[4x16]; lane l supplies A[l%16][l/16] and B[l/16][l%16], which for
//      B = A^T is the same register, and receives D[l/16 + 4i][l%16] in register i),
//   2. runs one cyclic sweep of two-sided Jacobi rotations on S in LDS (15 rounds of 8 disjoint
//      rotations, worked out once per round), accumulating them in V,
//   3. replaces the rows by V^T R, again with the matrix instruction.
// A rotation is applied only if the inner product exceeds tol times the product of the two norms (the
// relative test, which keeps the small rows accurate relative to their own size).  Rows whose squared
// norm is at most `tiny` are numerically zero and are left alone.  Rows >= m of the last block
// read as zero and are never written.  `rotations` counts the rotations applied.
template <int NW>   // waves per workgroup: they share the columns in steps 1 and 3; the first four run step 2
__global__ __launch_bounds__(64 * NW) void jacobi_block_kernel(double* G, int m, int len, int step, double tol, double tiny, int* rotations) {
  __shared__ double part[NW][16][17];                   // per-wave partial Gram matrices
  __shared__ double S[2][16][17];                       // double-buffered Gram matrix
  __shared__ double V[2][16][17];                       // accumulated rotations
  __shared__ int n_rot;
  const int nb = (m + 7) / 8, nbp = nb + (nb & 1), n1 = nbp - 1;
  const int k = blockIdx.x;
  const int P = k == 0 ? n1 : (step + k) % n1;
  const int Q = k == 0 ? step : (step - k + n1) % n1;
  // with an odd number of blocks one workgroup per round holds the bye (block index nb): its rows lie
  // beyond m and read as zero, so the workgroup still rotates the rows of its real block among themselves
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lq = lane >> 4;
  auto row_of = [&](int r) { return (r < 8 ? P * 8 : Q * 8 - 8) + r; };
  const int chunks = (len + 15) / 16;

  // 1. Gram matrix: lane (lr, lq) of a wave loads columns c0 + 4 lq .. + 3 of row lr of a 16-column chunk
  {
    const int grow = row_of(lr);
    const double* src = G + (long)grow * len;
    // four values of this lane's row at columns c .. c+3 (zero beyond the matrix)
    auto load4 = [&](int ch, double* x) __attribute__((always_inline)) {
      const int c = ch * 16 + 4 * lq;
      if (grow < m && c + 3 < len && (len & 1) == 0) {    // even rows start 16-byte aligned
        const f64x2 lo = *reinterpret_cast<const f64x2*>(src + c), hi = *reinterpret_cast<const f64x2*>(src + c + 2);
        x[0] = lo[0]; x[1] = lo[1]; x[2] = hi[0]; x[3] = hi[1];
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = (grow < m && ch < chunks && c + j < len) ? src[c + j] : 0.0;
      }
    };
    f64x4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
    for (int ch = wave; ch < chunks; ch += 2 * NW) {      // two chunks in flight, two accumulation chains
      double x0[4], x1[4];
      load4(ch, x0);
      load4(ch + NW, x1);                                 // a chunk index beyond the row loads zeros
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(x0[j], x0[j], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(x1[j], x1[j], acc1, 0, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) part[wave][lq + 4 * i][lr] = acc0[i] + acc1[i];
  }
  if (tid == 0) n_rot = 0;
  __syncthreads();
  const int ti = (tid >> 4) & 15, tj = tid & 15;        // this thread's element of S and V (threads 0..255)
  const bool solver = tid < 256;
  if (solver) {
    double sum = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += part[w][ti][tj];
    S[0][ti][tj] = sum;
    V[0][ti][tj] = ti == tj ? 1.0 : 0.0;
  }
  __syncthreads();

  // 2. one sweep over the 120 pairs of the 16 rows: 15 rounds of 8 disjoint rotations.  Eight threads work
  // out the rotations of a round (new_x = co[x] old_x + si[x] old_partner), then the 256 solver threads
  // update their elements of S and V; the other waves only keep the barriers company.
  __shared__ double co[16], si[16];
  int cur = 0;
  for (int s = 0; s < 15; ++s) {
    if (tid < 8) {
      const int x = tid == 0 ? 15 : (s + tid) % 15, y = tid == 0 ? s : (s - tid + 15) % 15;
      const int p = x < y ? x : y, q = x < y ? y : x;
      const double a = S[cur][p][p], b = S[cur][q][q], c = S[cur][p][q];
      double cs = 1.0, sn = 0.0;
      if (a > tiny && b > tiny && fabs(c) > tol * sqrt(a * b)) {
        const double zeta = (b - a) / (2.0 * c);
        const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        cs = 1.0 / sqrt(1.0 + t * t);
        sn = cs * t;
        atomicAdd(&n_rot, 1);
      }
      co[p] = cs; si[p] = -sn;                            // row p: cs p - sn q
      co[q] = cs; si[q] = sn;                             // row q: sn p + cs q
    }
    __syncthreads();
    if (solver) {
      const int pi = ti == 15 ? s : (ti == s ? 15 : (2 * s - ti + 30) % 15);
      const int pj = tj == 15 ? s : (tj == s ? 15 : (2 * s - tj + 30) % 15);
      const double ci = co[ti], zi = si[ti], cj = co[tj], zj = si[tj];
      const double snew = ci * (cj * S[cur][ti][tj] + zj * S[cur][ti][pj]) + zi * (cj * S[cur][pi][tj] + zj * S[cur][pi][pj]);
      const double vnew = cj * V[cur][ti][tj] + zj * V[cur][ti][pj];
      S[cur ^ 1][ti][tj] = snew;
      V[cur ^ 1][ti][tj] = vnew;
    }
    __syncthreads();
    cur ^= 1;
  }
  if (n_rot == 0) return;                               // uniform: read after the barrier
  if (tid == 0) atomicAdd(rotations, n_rot);

  // 3. rows <- V^T R, 16 columns at a time: A[r][k] = V[k][r], B[k][n] = R[k][c0 + n]
  double va[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) va[kk] = V[cur][4 * kk + lq][lr];
  for (int ch = wave; ch < chunks; ch += NW) {
    const int c = ch * 16 + lr;
    double xb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int grow = row_of(4 * kk + lq);
      xb[kk] = (grow < m && c < len) ? G[(long)grow * len + c] : 0.0;
    }
    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(va[kk], xb[kk], acc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int grow = row_of(lq + 4 * i);
      if (grow < m && c < len) G[(long)grow * len + c] = acc[i];
    }
  }
}

// norms2[row] = squared norm of row `row` of G [m, len]
__global__ __launch_bounds__(256) void row_norms_kernel(const double* G, int len, double* norms2) {
  __shared__ double red[4][3];
  const double* g = G + (long)blockIdx.x * len;
  double a = 0.0, b = 0.0, c = 0.0;
  for (int j = threadIdx.x; j < len; j += 256) a += g[j] * g[j];
  block_sum3(a, b, c, red);
  if (threadIdx.x == 0) norms2[blockIdx.x] = a;
}

// Factor column k = row idx[k] of G, normalised, signed so that its entry of largest magnitude
// (the first one on ties) is positive: U64 [len, r] fp64 and U [len, r] in the storage type.
template <typename T>
__global__ __launch_bounds__(256) void extract_factor_kernel(const double* G, int len, const int* idx, const double* norms2,
                                                             int r, double* U64, T* U) {
  __shared__ double best_v[256];
  __shared__ int best_j[256];
  const int k = blockIdx.x;
  const double* g = G + (long)idx[k] * len;
  double bv = -1.0;
  int bj = 0x7fffffff;
  for (int j = threadIdx.x; j < len; j += 256) {
    const double v = fabs(g[j]);
    if (v > bv) { bv = v; bj = j; }                     // j ascending: the first maximum of this thread
  }
  best_v[threadIdx.x] = bv;
  best_j[threadIdx.x] = bj;
  __syncthreads();
  for (int sft = 128; sft > 0; sft >>= 1) {
    if ((int)threadIdx.x < sft) {
      const double ov = best_v[threadIdx.x + sft];
      const int oj = best_j[threadIdx.x + sft];
      if (ov > best_v[threadIdx.x] || (ov == best_v[threadIdx.x] && oj < best_j[threadIdx.x])) {
        best_v[threadIdx.x] = ov;
        best_j[threadIdx.x] = oj;
      }
    }
    __syncthreads();
  }
  const double scale = (g[best_j[0]] < 0.0 ? -1.0 : 1.0) / sqrt(norms2[idx[k]]);
  for (int j = threadIdx.x; j < len; j += 256) {
    const double v = scale * g[j];
    U64[(long)j * r + k] = v;
    U[(long)j * r + k] = from_f64<T>(v);
  }
}

inline int blocks_for(long total) { return (int)std::min<long>((total + 255) / 256, 1 << 16); }

hipError_t dgemm(hipStream_t s, int batch, int M, int N, int K, const double* A, long a_m, long a_k, long a_b,
                 const double* B, long b_k, long b_n, long b_b, double* C, long c_m, long c_n, long c_b) {
  DgemmArgs g{A, a_m, a_k, a_b, B, b_k, b_n, b_b, C, c_m, c_n, c_b, M, N, K};
  hipLaunchKernelGGL(dgemm_kernel, dim3((N + 63) / 64, (M + 63) / 64, batch), dim3(256), 0, s, g);
  return hipGetLastError();
}

#define CK(expr)                                  \
  do {                                            \
    if ((expr) != hipSuccess) return TUCKER_ATTN_HIP_ERROR; \
  } while (0)

// Eigenvectors of the symmetric positive semi-definite G [m, m] (destroyed) with the r largest
// eigenvalues -> U64 / U [m, r]; sv (host, nullable) receives the square roots of all
// eigenvalues in decreasing order.  Synchronises the stream.
constexpr int kJacobiWaves = 16;

struct JacobiStats {
  int sweeps = 0;
  long launches = 0;
  double ms = 0.0;
};

template <typename T>
int leading_eigenvectors(hipStream_t s, double* G, int m, int r, double* norms2, int* idx, int* counter,
                         double* U64, T* U, double* sv, JacobiStats* stats) {
  std::vector<double> h(m);
  hipLaunchKernelGGL(row_norms_kernel, dim3(m), dim3(256), 0, s, G, m, norms2);
  CK(hipGetLastError());
  CK(hipMemcpyAsync(h.data(), norms2, sizeof(double) * m, hipMemcpyDeviceToHost, s));
  CK(hipStreamSynchronize(s));
  const double fro2 = std::accumulate(h.begin(), h.end(), 0.0);
  const double tiny = 1e-28 * m * fro2;                 // rows below the rounding noise of G's entries
  const double tol = std::max(2e-15, std::sqrt((double)m) * 2.3e-16);
  const int nb = (m + 7) / 8, nbp = nb + (nb & 1), n_steps = nbp - 1;   // rounds of the block tournament
  int rotated = 0;
  hipEvent_t ev[2] = {nullptr, nullptr};
  if (stats) {
    CK(hipEventCreate(&ev[0]));
    if (hipEventCreate(&ev[1]) != hipSuccess) {
      (void)hipEventDestroy(ev[0]);
      return TUCKER_ATTN_HIP_ERROR;
    }
    (void)hipEventRecord(ev[0], s);
  }
  struct EventGuard {
    hipEvent_t* e;
    ~EventGuard() {
      if (e[0]) (void)hipEventDestroy(e[0]);
      if (e[1]) (void)hipEventDestroy(e[1]);
    }
  } guard{ev};
  for (int sweep = 0; sweep < 60 && m > 1; ++sweep) {
    if (stats) {
      ++stats->sweeps;
      stats->launches += n_steps;
    }
    CK(hipMemsetAsync(counter, 0, sizeof(int), s));
    for (int step = 0; step < n_steps; ++step)
      hipLaunchKernelGGL((jacobi_block_kernel<kJacobiWaves>), dim3(nbp / 2), dim3(64 * kJacobiWaves), 0, s, G, m, m, step, tol,
                         tiny, counter);
    CK(hipGetLastError());
    CK(hipMemcpyAsync(&rotated, counter, sizeof(int), hipMemcpyDeviceToHost, s));
    CK(hipStreamSynchronize(s));
    if (rotated == 0) break;
  }
  if (stats) {
    float ms = 0.f;
    CK(hipEventRecord(ev[1], s));
    CK(hipEventSynchronize(ev[1]));
    CK(hipEventElapsedTime(&ms, ev[0], ev[1]));
    stats->ms += ms;
  }
  if (rotated != 0) return TUCKER_ATTN_UNSUPPORTED_SHAPE;   // no convergence within the sweep limit
  hipLaunchKernelGGL(row_norms_kernel, dim3(m), dim3(256), 0, s, G, m, norms2);
  CK(hipGetLastError());
  CK(hipMemcpyAsync(h.data(), norms2, sizeof(double) * m, hipMemcpyDeviceToHost, s));
  CK(hipStreamSynchronize(s));
  std::vector<int> order(m);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return h[x] > h[y]; });
  if (sv)
    for (int k = 0; k < m; ++k) sv[k] = std::sqrt(std::sqrt(h[order[k]]));   // row norm = eigenvalue = sigma^2
  if (!(h[order[r - 1]] > 1e8 * tiny) || !(h[order[r - 1]] > 0.0)) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  CK(hipMemcpyAsync(idx, order.data(), sizeof(int) * r, hipMemcpyHostToDevice, s));
  CK(hipStreamSynchronize(s));                          // `order` is pageable host memory
  hipLaunchKernelGGL((extract_factor_kernel<T>), dim3(r), dim3(256), 0, s, G, m, idx, norms2, r, U64, U);
  CK(hipGetLastError());
  return TUCKER_ATTN_OK;
}

struct HosvdWs {
  double *A, *B, *T, *M, *GA, *GB, *SA, *SB, *M1, *U1, *U2, *U3, *P, *Q, *H, *C, *norms2;
  int *idx, *counter;
  size_t bytes;
};

HosvdWs carve_hosvd(void* base, int d, int nH, int dH) {
  const size_t n = (size_t)nH * dH, D = d;
  const size_t rmax = std::min<size_t>(D, 512);         // the layer's own rank limit bounds P, Q, H, C
  size_t off = 0;
  auto take = [&](size_t elems, size_t size) {
    void* p = base ? static_cast<char*>(base) + off : nullptr;
    off += (elems * size + 255) / 256 * 256;
    return p;
  };
  HosvdWs w;
  w.A = (double*)take(D * n, 8);
  w.B = (double*)take(D * n, 8);
  w.T = (double*)take(D * n, 8);
  w.M = (double*)take(D * D, 8);
  w.GA = (double*)take(n * n, 8);
  w.GB = (double*)take(n * n, 8);
  w.SA = (double*)take(n * dH, 8);
  w.SB = (double*)take(n * dH, 8);
  w.M1 = (double*)take((size_t)nH * nH, 8);
  w.U1 = (double*)take((size_t)nH * nH, 8);
  w.U2 = (double*)take(D * rmax, 8);
  w.U3 = (double*)take(D * rmax, 8);
  w.P = (double*)take(rmax * n, 8);
  w.Q = (double*)take(rmax * n, 8);
  w.H = (double*)take((size_t)nH * rmax * rmax, 8);
  w.C = (double*)take((size_t)nH * rmax * rmax, 8);
  w.norms2 = (double*)take(D + nH, 8);
  w.idx = (int*)take(D + nH, 4);
  w.counter = (int*)take(64, 4);
  w.bytes = off;
  return w;
}

// One tensor (A_i B_i^T)_i, A and B [d, n] fp64 in the workspace: factors and core at the given
// ranks.  `given_U3`: the mode-3 factor is already in w.U3 (shared latent) and is not recomputed.
template <typename T>
int hosvd_one(hipStream_t s, const HosvdWs& w, int d, int nH, int dH, int r1, int r2, int r3, bool given_U3,
              T* C, T* U1, T* U2, T* U3, double* sv, JacobiStats* st3) {
  const long n = (long)nH * dH;
  // per-head dH x dH Gram matrices  SA_i = A_i^T A_i, SB_i = B_i^T B_i
  CK(dgemm(s, nH, dH, dH, d, w.A, 1, n, dH, w.A, n, 1, dH, w.SA, dH, 1, (long)dH * dH));
  CK(dgemm(s, nH, dH, dH, d, w.B, 1, n, dH, w.B, n, 1, dH, w.SB, dH, 1, (long)dH * dH));
  // mode 1: <W_i, W_j> from the full Gram matrices of the factors
  CK(dgemm(s, 1, (int)n, (int)n, d, w.A, 1, n, 0, w.A, n, 1, 0, w.GA, n, 1, 0));
  CK(dgemm(s, 1, (int)n, (int)n, d, w.B, 1, n, 0, w.B, n, 1, 0, w.GB, n, 1, 0));
  hipLaunchKernelGGL(head_gram_kernel, dim3(nH, nH), dim3(256), 0, s, w.GA, w.GB, w.M1, nH, dH);
  CK(hipGetLastError());
  int st = leading_eigenvectors<T>(s, w.M1, nH, r1, w.norms2, w.idx, w.counter, w.U1, U1, sv, st3 ? &st3[0] : nullptr);
  if (st != TUCKER_ATTN_OK) return st;
  // mode 2: sum_i W_i W_i^T = sum_i (A_i SB_i) A_i^T
  CK(dgemm(s, nH, d, dH, dH, w.A, n, 1, dH, w.SB, dH, 1, (long)dH * dH, w.T, n, 1, dH));
  CK(dgemm(s, 1, d, d, (int)n, w.T, n, 1, 0, w.A, 1, n, 0, w.M, d, 1, 0));
  st = leading_eigenvectors<T>(s, w.M, d, r2, w.norms2, w.idx, w.counter, w.U2, U2, sv ? sv + nH : nullptr,
                                st3 ? &st3[1] : nullptr);
  if (st != TUCKER_ATTN_OK) return st;
  // mode 3: sum_i W_i^T W_i = sum_i (B_i SA_i) B_i^T
  if (!given_U3) {
    CK(dgemm(s, nH, d, dH, dH, w.B, n, 1, dH, w.SA, dH, 1, (long)dH * dH, w.T, n, 1, dH));
    CK(dgemm(s, 1, d, d, (int)n, w.T, n, 1, 0, w.B, 1, n, 0, w.M, d, 1, 0));
    st = leading_eigenvectors<T>(s, w.M, d, r3, w.norms2, w.idx, w.counter, w.U3, U3, sv ? sv + nH + d : nullptr,
                                  st3 ? &st3[2] : nullptr);
    if (st != TUCKER_ATTN_OK) return st;
  } else if (sv) {
    for (int k = 0; k < d; ++k) sv[nH + d + k] = 0.0;
  }
  // core: C[a] = sum_i U1[i][a] (U2^T A_i)(U3^T B_i)^T
  CK(dgemm(s, 1, r2, (int)n, d, w.U2, 1, r2, 0, w.A, n, 1, 0, w.P, n, 1, 0));
  CK(dgemm(s, 1, r3, (int)n, d, w.U3, 1, r3, 0, w.B, n, 1, 0, w.Q, n, 1, 0));
  CK(dgemm(s, nH, r2, r3, dH, w.P, n, 1, dH, w.Q, 1, n, dH, w.H, r3, 1, (long)r2 * r3));
  CK(dgemm(s, 1, r1, r2 * r3, nH, w.U1, 1, r1, 0, w.H, (long)r2 * r3, 1, 0, w.C, (long)r2 * r3, 1, 0));
  const long total = (long)r1 * r2 * r3;
  hipLaunchKernelGGL((from_f64_kernel<T>), dim3(blocks_for(total)), dim3(256), 0, s, w.C, C, total);
  CK(hipGetLastError());
  return TUCKER_ATTN_OK;
}

template <typename T>
int from_gqa(int d, int nH, int dH, int nG, const T* WQ, const T* WK, const T* WV, const T* WO,
             const tucker_convert_weights_out& o, hipStream_t s) {
  const long n = (long)nH * dH, g = (long)nG * dH;
  const long core = (long)nH * n * g;
  hipLaunchKernelGGL((selector_core_kernel<T>), dim3(blocks_for(core)), dim3(256), 0, s, (T*)o.C, nH, dH, nG);
  hipLaunchKernelGGL((selector_core_kernel<T>), dim3(blocks_for(core)), dim3(256), 0, s, (T*)o.Ct, nH, dH, nG);
  hipLaunchKernelGGL((identity_kernel<T>), dim3(blocks_for((long)nH * nH)), dim3(256), 0, s, (T*)o.U1, nH);
  hipLaunchKernelGGL((identity_kernel<T>), dim3(blocks_for((long)nH * nH)), dim3(256), 0, s, (T*)o.Ut1, nH);
  hipLaunchKernelGGL((transpose_copy_kernel<T>), dim3((d + 31) / 32, (int)((n + 31) / 32)), dim3(256), 0, s, WO, (T*)o.Ut2, (int)n, d);
  CK(hipGetLastError());
  CK(hipMemcpyAsync(o.U2, WQ, sizeof(T) * d * n, hipMemcpyDeviceToDevice, s));
  CK(hipMemcpyAsync(o.U3, WK, sizeof(T) * d * g, hipMemcpyDeviceToDevice, s));
  CK(hipMemcpyAsync(o.Ut3, WV, sizeof(T) * d * g, hipMemcpyDeviceToDevice, s));
  return TUCKER_ATTN_OK;
}

template <typename T>
int from_mla(int d, int nH, int dH, int dcQ, int dcK, const T* WDQ, const T* WUQ, const T* WDKV, const T* WUK,
             const T* WDV, const T* WUV, const T* WO, const tucker_convert_weights_out& o, hipStream_t s) {
  const long n = (long)nH * dH;
  hipLaunchKernelGGL((mla_core_kernel<T>), dim3(blocks_for((long)nH * dcQ * dcK)), dim3(256), 0, s, WUQ, WUK, (T*)o.C, nH, dH, dcQ, dcK);
  hipLaunchKernelGGL((mla_post_core_kernel<T>), dim3(blocks_for((long)nH * n * dcK)), dim3(256), 0, s, WUV, (T*)o.Ct, nH, dH, dcK);
  hipLaunchKernelGGL((identity_kernel<T>), dim3(blocks_for((long)nH * nH)), dim3(256), 0, s, (T*)o.U1, nH);
  hipLaunchKernelGGL((identity_kernel<T>), dim3(blocks_for((long)nH * nH)), dim3(256), 0, s, (T*)o.Ut1, nH);
  hipLaunchKernelGGL((transpose_copy_kernel<T>), dim3((d + 31) / 32, (int)((n + 31) / 32)), dim3(256), 0, s, WO, (T*)o.Ut2, (int)n, d);
  CK(hipGetLastError());
  CK(hipMemcpyAsync(o.U2, WDQ, sizeof(T) * d * dcQ, hipMemcpyDeviceToDevice, s));
  CK(hipMemcpyAsync(o.U3, WDKV, sizeof(T) * d * dcK, hipMemcpyDeviceToDevice, s));
  if (WDV) CK(hipMemcpyAsync(o.Ut3, WDV, sizeof(T) * d * dcK, hipMemcpyDeviceToDevice, s));
  return TUCKER_ATTN_OK;
}

template <typename T>
int from_mha_hosvd(int d, int nH, int dH, const T* WQ, const T* WK, const T* WV, const T* WO, int r1, int r2, int r3,
                   int rt1, int rt2, int rt3, bool shared, const tucker_convert_weights_out& o, double* sv,
                   tucker_convert_hosvd_info* info, void* workspace, hipStream_t s) {
  JacobiStats stats[6];
  struct Report {                                       // filled on every return path
    tucker_convert_hosvd_info* info;
    const JacobiStats* st;
    int d;
    ~Report() {
      if (!info) return;
      info->jacobi_launches = 0;
      info->jacobi_ms = 0.0;
      for (int k = 0; k < 6; ++k) {
        info->sweeps[k] = st[k].sweeps;
        if (k % 3 != 0) {
          info->jacobi_launches += st[k].launches;
          info->jacobi_ms += st[k].ms;
        }
      }
      info->jacobi_bytes = 16.0 * d * d * (double)info->jacobi_launches;
    }
  } report{info, stats, d};
  const HosvdWs w = carve_hosvd(workspace, d, nH, dH);
  const long n = (long)nH * dH;
  const int cb = blocks_for((long)d * n);
  // pre-softmax tensor: A = WQ, B = WK
  hipLaunchKernelGGL((to_f64_kernel<T>), dim3(cb), dim3(256), 0, s, WQ, n, 1, w.A, d, (int)n);
  hipLaunchKernelGGL((to_f64_kernel<T>), dim3(cb), dim3(256), 0, s, WK, n, 1, w.B, d, (int)n);
  CK(hipGetLastError());
  int st = hosvd_one<T>(s, w, d, nH, dH, r1, r2, r3, false, (T*)o.C, (T*)o.U1, (T*)o.U2, (T*)o.U3, sv, info ? stats : nullptr);
  if (st != TUCKER_ATTN_OK) return st;
  // post-softmax tensor, output index first: A = WO^T, B = WV
  hipLaunchKernelGGL((to_f64_kernel<T>), dim3(cb), dim3(256), 0, s, WO, 1, (long)d, w.A, d, (int)n);
  hipLaunchKernelGGL((to_f64_kernel<T>), dim3(cb), dim3(256), 0, s, WV, n, 1, w.B, d, (int)n);
  CK(hipGetLastError());
  st = hosvd_one<T>(s, w, d, nH, dH, rt1, rt2, rt3, shared, (T*)o.Ct, (T*)o.Ut1, (T*)o.Ut2, (T*)o.Ut3,
                    sv ? sv + nH + 2 * d : nullptr, info ? stats + 3 : nullptr);
  if (st != TUCKER_ATTN_OK) return st;
  CK(hipStreamSynchronize(s));
  return TUCKER_ATTN_OK;
}

}  // namespace
}  // namespace ta

extern "C" {

int tucker_convert_from_gqa(int32_t dtype, int32_t d, int32_t nH, int32_t dH, int32_t nG, const void* WQ, const void* WK,
                            const void* WV, const void* WO, const tucker_convert_weights_out* out, void* hip_stream) {
  if (dtype != TUCKER_ATTN_F32 && dtype != TUCKER_ATTN_BF16) return TUCKER_ATTN_INVALID_ARG;
  if (d < 1 || nH < 1 || dH < 1 || nG < 1 || nH % nG != 0) return TUCKER_ATTN_INVALID_ARG;
  if (!WQ || !WK || !WV || !WO || !out) return TUCKER_ATTN_INVALID_ARG;
  if (!out->C || !out->U1 || !out->U2 || !out->U3 || !out->Ct || !out->Ut1 || !out->Ut2 || !out->Ut3)
    return TUCKER_ATTN_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (dtype == TUCKER_ATTN_F32)
    return ta::from_gqa<float>(d, nH, dH, nG, (const float*)WQ, (const float*)WK, (const float*)WV, (const float*)WO, *out, s);
  return ta::from_gqa<ta::bf16>(d, nH, dH, nG, (const ta::bf16*)WQ, (const ta::bf16*)WK, (const ta::bf16*)WV,
                                (const ta::bf16*)WO, *out, s);
}

int tucker_convert_from_mla(int32_t dtype, int32_t d, int32_t nH, int32_t dH, int32_t dcQ, int32_t dcK, const void* WDQ,
                            const void* WUQ, const void* WDKV, const void* WUK, const void* WDV, const void* WUV,
                            const void* WO, const tucker_convert_weights_out* out, void* hip_stream) {
  if (dtype != TUCKER_ATTN_F32 && dtype != TUCKER_ATTN_BF16) return TUCKER_ATTN_INVALID_ARG;
  if (d < 1 || nH < 1 || dH < 1 || dcQ < 1 || dcK < 1) return TUCKER_ATTN_INVALID_ARG;
  if (!WDQ || !WUQ || !WDKV || !WUK || !WUV || !WO || !out) return TUCKER_ATTN_INVALID_ARG;
  if (!out->C || !out->U1 || !out->U2 || !out->U3 || !out->Ct || !out->Ut1 || !out->Ut2) return TUCKER_ATTN_INVALID_ARG;
  if (WDV && !out->Ut3) return TUCKER_ATTN_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (dtype == TUCKER_ATTN_F32)
    return ta::from_mla<float>(d, nH, dH, dcQ, dcK, (const float*)WDQ, (const float*)WUQ, (const float*)WDKV,
                               (const float*)WUK, (const float*)WDV, (const float*)WUV, (const float*)WO, *out, s);
  return ta::from_mla<ta::bf16>(d, nH, dH, dcQ, dcK, (const ta::bf16*)WDQ, (const ta::bf16*)WUQ, (const ta::bf16*)WDKV,
                                (const ta::bf16*)WUK, (const ta::bf16*)WDV, (const ta::bf16*)WUV, (const ta::bf16*)WO, *out, s);
}

size_t tucker_convert_hosvd_workspace_bytes(int32_t d, int32_t nH, int32_t dH) {
  if (d < 1 || nH < 1 || dH < 1 || d > 8192 || nH > 256 || (long)nH * dH > 8192) return 0;
  return ta::carve_hosvd(nullptr, d, nH, dH).bytes;
}

int tucker_convert_from_mha_hosvd(int32_t dtype, int32_t d, int32_t nH, int32_t dH, const void* WQ, const void* WK,
                                  const void* WV, const void* WO, int32_t r1, int32_t r2, int32_t r3, int32_t rt1,
                                  int32_t rt2, int32_t rt3, int32_t shared_kv, const tucker_convert_weights_out* out,
                                  double* singular_values, tucker_convert_hosvd_info* info, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  if (dtype != TUCKER_ATTN_F32 && dtype != TUCKER_ATTN_BF16) return TUCKER_ATTN_INVALID_ARG;
  if (d < 1 || nH < 1 || dH < 1) return TUCKER_ATTN_INVALID_ARG;
  if (d > 8192 || nH > 256 || (long)nH * dH > 8192) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if (r1 < 1 || r2 < 1 || r3 < 1 || rt1 < 1 || rt2 < 1 || rt3 < 1) return TUCKER_ATTN_INVALID_ARG;
  if (r1 > nH || rt1 > nH || r2 > d || r3 > d || rt2 > d || rt3 > d) return TUCKER_ATTN_INVALID_ARG;
  if (r2 > 512 || r3 > 512 || rt2 > 512 || rt3 > 512) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if (shared_kv != 0 && shared_kv != 1) return TUCKER_ATTN_INVALID_ARG;
  if (shared_kv && rt3 != r3) return TUCKER_ATTN_INVALID_ARG;
  if (!WQ || !WK || !WV || !WO || !out || !workspace) return TUCKER_ATTN_INVALID_ARG;
  if (!out->C || !out->U1 || !out->U2 || !out->U3 || !out->Ct || !out->Ut1 || !out->Ut2) return TUCKER_ATTN_INVALID_ARG;
  if (!shared_kv && !out->Ut3) return TUCKER_ATTN_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return TUCKER_ATTN_INVALID_ARG;
  if (workspace_bytes < tucker_convert_hosvd_workspace_bytes(d, nH, dH)) return TUCKER_ATTN_WORKSPACE_TOO_SMALL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (dtype == TUCKER_ATTN_F32)
    return ta::from_mha_hosvd<float>(d, nH, dH, (const float*)WQ, (const float*)WK, (const float*)WV, (const float*)WO, r1,
                                     r2, r3, rt1, rt2, rt3, shared_kv != 0, *out, singular_values, info, workspace, s);
  return ta::from_mha_hosvd<ta::bf16>(d, nH, dH, (const ta::bf16*)WQ, (const ta::bf16*)WK, (const ta::bf16*)WV,
                                      (const ta::bf16*)WO, r1, r2, r3, rt1, rt2, rt3, shared_kv != 0, *out, singular_values,
                                      info, workspace, s);
}

}  // extern "C"
