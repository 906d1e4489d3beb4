// One 64x64 tile of the weight preparation (see prep.hip), as a device function: the preparation kernel runs
// one tile per workgroup, and a decode step lets the tiles ride along in the launch of its factor projection.
#pragma once
#include "common.h"
#include "params.h"

namespace ta {

constexpr int kPrepTile = 64;

// one tile (workgroup index blk over all jobs); `tile` is kPrepTile x (kPrepTile + 1) floats of LDS
template <typename T>
__device__ __forceinline__ void prep_tile(const PrepArgs& args, int blk, float (*tile)[kPrepTile + 1]) {
  constexpr int TS = kPrepTile, CE = 16 / (int)sizeof(T);
  int ji = 0;
#pragma unroll
  for (int j = 1; j < kMaxPrepJobs; ++j)
    if (j < args.n_jobs && blk >= args.job[j].first_block) ji = j;
  const PrepJob& jb = args.job[ji];
  const int local = blk - jb.first_block;
  const int tiles_r = (jb.rows_pad + TS - 1) / TS, tiles_c = (jb.cols_pad + TS - 1) / TS;
  const int z = local / (tiles_r * tiles_c);
  const int rem = local % (tiles_r * tiles_c);
  const int r0 = (rem / tiles_c) * TS, c0 = (rem % tiles_c) * TS;
  const T* src = static_cast<const T*>(jb.src);
  const T* coef = static_cast<const T*>(jb.coef);
  T* out = static_cast<T*>(jb.out) + (long)z * jb.out_stride_z;

  // ---- source tile (rows r0.., columns c0..) summed over the A slices -> LDS ------------------------
  // All loads of a batch of slices are issued before the first use.  Rows whose length and base keep every
  // 16-byte chunk aligned are read a chunk per load (thread = chunk tx of rows ty, ty+32); other shapes an
  // element per load (thread = column tx of rows ty, ty+4, ...).
  const bool chunked = jb.cols % CE == 0 && reinterpret_cast<uintptr_t>(src) % 16 == 0;
  if (chunked) {
    constexpr int CPR = TS / CE;                                  // chunks per tile row
    constexpr int RPT = TS * CPR / 256;                           // rows per thread
    const int tx = threadIdx.x % CPR, ty = threadIdx.x / CPR;
    const int col = c0 + tx * CE;
    const int colc = min(col, jb.cols - CE);                      // a chunk past the end re-reads the last one
    float acc[RPT][CE];
#pragma unroll
    for (int i = 0; i < RPT; ++i)
#pragma unroll
      for (int e = 0; e < CE; ++e) acc[i][e] = 0.f;
    for (int a0 = 0; a0 < jb.A; a0 += 8) {
      u32x4 v[8][RPT];
      float w[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int a = min(a0 + k, jb.A - 1);                      // slices past the end get weight 0
        w[k] = a0 + k < jb.A ? (coef ? to_f32(coef[(long)z * jb.A + a]) : 1.f) : 0.f;
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
          const int row = min(r0 + ty + (256 / CPR) * i, jb.rows - 1);
          v[k][i] = *reinterpret_cast<const u32x4*>(src + ((long)a * jb.rows + row) * jb.cols + colc);
        }
        if (jb.A == 1) break;
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
          if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              acc[i][2 * e] += w[k] * __uint_as_float(v[k][i][e] << 16);
              acc[i][2 * e + 1] += w[k] * __uint_as_float(v[k][i][e] & 0xffff0000u);
            }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][e] += w[k] * __uint_as_float(v[k][i][e]);
          }
        }
        if (jb.A == 1) break;
      }
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      const int r = ty + (256 / CPR) * i;
#pragma unroll
      for (int e = 0; e < CE; ++e) {
        const bool inside = r0 + r < jb.rows && col + e < jb.cols; // the padded part of the output is zero
        tile[r][tx * CE + e] = inside ? acc[i][e] * jb.scale : 0.f;
      }
    }
  } else {
    constexpr int RPT = TS / 4;                                   // rows per thread
    const int tx = threadIdx.x % TS, ty = threadIdx.x / TS;
    const int col = min(c0 + tx, jb.cols - 1);
    float acc[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) acc[i] = 0.f;
    for (int a0 = 0; a0 < jb.A; a0 += 4) {
      T v[4][RPT];
      float w[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int a = min(a0 + k, jb.A - 1);
        w[k] = a0 + k < jb.A ? (coef ? to_f32(coef[(long)z * jb.A + a]) : 1.f) : 0.f;
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
          const int row = min(r0 + ty + 4 * i, jb.rows - 1);
          v[k][i] = src[((long)a * jb.rows + row) * jb.cols + col];
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < RPT; ++i) acc[i] += w[k] * to_f32(v[k][i]);
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      const int r = ty + 4 * i;
      const bool inside = r0 + r < jb.rows && c0 + tx < jb.cols;
      tile[r][tx] = inside ? acc[i] * jb.scale : 0.f;
    }
  }
  __syncthreads();

  // ---- output chunks of CE consecutive stored positions -----------------------------------------------
  // (u, v) = (column, row) of the source when transposed, (row, column) otherwise; with perm the stored
  // position p of a 32-block holds natural index acc_index(p)
  const int u_ext = jb.transposed ? jb.cols_pad : jb.rows_pad, v_ext = jb.transposed ? jb.rows_pad : jb.cols_pad;
  const int u0 = jb.transposed ? c0 : r0, v0 = jb.transposed ? r0 : c0;
  constexpr int CPU = TS / CE;                                    // chunks per output row of the tile
  for (int ci = threadIdx.x; ci < TS * CPU; ci += 256) {
    // consecutive threads take consecutive chunks of one output row
    const int ul = ci / CPU, vc = (ci % CPU) * CE;
    const int u = u0 + ul, v = v0 + vc;
    if (u >= u_ext || v >= v_ext) continue;
    float x[CE];
#pragma unroll
    for (int e = 0; e < CE; ++e) {
      const int p = (v + e) % 32, vb = (v + e) - p;
      const int vn = vb + (jb.perm ? acc_index(p) : p) - v0;       // natural index inside the tile
      x[e] = jb.transposed ? tile[vn][ul] : tile[ul][vn];
    }
    long off;
    if (jb.frag) {
      const int nvb = v_ext / 32;
      off = ((long)(u / 32) * nvb + v / 32) * kFragBlockElems + frag_major_offset<T>(u % 32, v % 32);
    } else {
      off = (long)u * jb.out_stride_u + v;
    }
    if constexpr (sizeof(T) == 2) {
      u32x4 pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f32x2 two = {x[2 * e], x[2 * e + 1]};
        pk[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
      }
      *reinterpret_cast<u32x4*>(out + off) = pk;
    } else {
      *reinterpret_cast<f32x4*>(out + off) = f32x4{x[0], x[1], x[2], x[3]};
    }
  }
}

}  // namespace ta
