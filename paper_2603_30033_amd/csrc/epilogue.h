// Epilogues of the token-side products: what becomes of one 32x32 accumulator block.  Shared by the
// product kernel, the split-K reduction and the decode kernel that sums the projection's partial tiles itself.
#pragma once
#include "common.h"
#include "params.h"

namespace ta {

// ---- epilogues: one 32x32 accumulator block = 32 weight rows (m0..) x 32 tokens ----------
template <typename T>
__device__ __forceinline__ void epilogue_block(const GemmArgs& g, f32x16 acc, int m0, int tp) {
  const int lane = threadIdx.x % kWave;
  const int h = lane / 32;
  const int TP = g.Bsz * g.Npad;
  if (tp >= TP) return;
  const int b = tp / g.Npad, n = tp % g.Npad;
  const bool valid = n < g.N;

  if (g.epi == 0) {
    const int pos = g.decode ? g.kv_pos[b] : g.pos0 + n;
    if (m0 < g.R2) {                                            // ---- Qlat, acc order
      T* dst = static_cast<T*>(g.Qlat) + (long)tp * g.R2 + m0 + 16 * h;
      store_frag<T>(dst, to_frag<T>(acc));
    } else if (m0 < g.R2 + g.D) {                               // ---- K, rotated
      const int c0 = m0 - g.R2;
      if (g.shared_kv) {
        // shared key-value latent: the unrotated block is the value block and the cache row
        if (g.Vt != nullptr) {
          T* base = static_cast<T*>(g.Vt) + (long)b * g.D * g.Npad + (n & ~31) + acc_pos(n & 31);
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) store1(base + (long)(c0 + 8 * q + 4 * h + e) * g.Npad, acc[4 * q + e]);
        }
        if (g.Vr != nullptr) store_frag<T>(static_cast<T*>(g.Vr) + (long)tp * g.D + c0 + 16 * h, to_frag<T>(acc));
        if (g.Kcache != nullptr && valid) {
          T* row = static_cast<T*>(g.Kcache) + ((long)b * g.Lmax + pos) * g.r3;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            int c = c0 + 8 * q + 4 * h;
            if (c + 3 < g.r3 && (g.r3 % 4) == 0)
              store4(row + c, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
            else
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (c + e < g.r3) store1(row + c + e, acc[4 * q + e]);
          }
        }
      }
      if (g.rope != nullptr) {
        // (cos, sin) of two adjacent pairs per load, all four loads issued before the first use;
        // rows of padding tokens hold zeros, so any table row serves them
        const f32x4* tab = reinterpret_cast<const f32x4*>(g.rope) + (long)(c0 / 4 + h) * g.rope_ld + (valid ? pos : 0);
        f32x4 cs[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) cs[q] = tab[(long)2 * q * g.rope_ld];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; e += 2) {
            float x0 = acc[4 * q + e], x1 = acc[4 * q + e + 1];
            acc[4 * q + e] = x0 * cs[q][e] - x1 * cs[q][e + 1];
            acc[4 * q + e + 1] = x0 * cs[q][e + 1] + x1 * cs[q][e];
          }
      }
      if (g.Kr != nullptr) {
        T* dst = static_cast<T*>(g.Kr) + (long)tp * g.D + c0 + 16 * h;
        store_frag<T>(dst, to_frag<T>(acc));
      }
      if (g.Krt != nullptr) {
        T* base = static_cast<T*>(g.Krt) + (long)b * g.D * g.Npad + (n & ~31) + acc_pos(n & 31);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) store1(base + (long)(c0 + 8 * q + 4 * h + e) * g.Npad, acc[4 * q + e]);
      }
      if (g.Kcache != nullptr && valid && !g.shared_kv) {
        T* row = static_cast<T*>(g.Kcache) + ((long)b * g.Lmax + pos) * g.r3;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          int c = c0 + 8 * q + 4 * h;
          if (c + 3 < g.r3 && (g.r3 % 4) == 0)
            store4(row + c, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
          else
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (c + e < g.r3) store1(row + c + e, acc[4 * q + e]);
        }
      }
    } else {                                                    // ---- V
      const int c0 = m0 - g.R2 - g.D;
      if (g.Vr != nullptr) store_frag<T>(static_cast<T*>(g.Vr) + (long)tp * g.D + c0 + 16 * h, to_frag<T>(acc));
      if (g.Vt != nullptr) {
        // Vt[b][c][n], n stored at its acc-order position inside its 32-block
        T* base = static_cast<T*>(g.Vt) + (long)b * g.D * g.Npad + (n & ~31) + acc_pos(n & 31);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            int c = c0 + 8 * q + 4 * h + e;
            store1(base + (long)c * g.Npad, acc[4 * q + e]);
          }
      }
      if (g.Vcache != nullptr && valid) {
        T* row = static_cast<T*>(g.Vcache) + ((long)b * g.Lmax + pos) * g.rt3;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          int c = c0 + 8 * q + 4 * h;
          if (c + 3 < g.rt3 && (g.rt3 % 4) == 0)
            store4(row + c, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
          else
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (c + e < g.rt3) store1(row + c + e, acc[4 * q + e]);
        }
      }
    }
  } else if (g.epi == 1) {                                      // ---- Z, natural order, padded tokens
    T* row = static_cast<T*>(g.Out) + (long)tp * g.ldo;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int c = m0 + 8 * q + 4 * h;
      if (c < g.M) store4(row + c, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    }
  } else if (g.epi == 3) {                                      // ---- fp32 matrix, column ranges routed
    // a row or column that sits at an acc-order position of its 32-block is stored at its natural index
    const int nn = g.perm_n ? (tp & ~31) + acc_index(tp & 31) : tp;
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      const GemmArgs::Out3& o = g.out3[u];
      if (o.ptr == nullptr || nn < o.n0 || nn >= o.n1) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int mp = 8 * q + 4 * h + e;
          const int m = m0 + (g.perm_m ? acc_index(mp) : mp);
          if (m < g.M) o.ptr[(long)m * o.ld + (nn - o.n0)] = g.out_scale * acc[4 * q + e];
        }
    }
  } else {                                                      // ---- Y, caller's [B][N][d]
    if (!valid) return;
    T* row = static_cast<T*>(g.Out) + ((long)b * g.N + n) * g.ldo;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int c = m0 + 8 * q + 4 * h;
      if (c + 3 < g.M)
        store4(row + c, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
      else
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (c + e < g.M) store1(row + c + e, acc[4 * q + e]);
    }
  }
}

}  // namespace ta
