// Decode against the latent KV cache (Section "KV Caching" of the paper): one new query
// token per sequence attends the cached rotated keys and plain values, width r3, that all
// heads share.  The heads of a sequence are the MFMA column dimension, so one pass over a
// cache tile serves every head.
//
//   decode_qhat    Qhat_i = qscale * Qlat G_i, latent RoPE at position kv_len-1
//   decode_attn    split-KV: each workgroup streams a contiguous slice of one sequence's
//                  cache through LDS once and emits a partial (max, sum, O) per head
//   decode_merge_heads  log-sum-exp merge of the partials and the head merge, one workgroup per head
//   decode_out     output projection from the heads' contributions
#include "common.h"
#include "params.h"
#include "epilogue.h"

namespace ta {

// ---------------------------------------------------------------------------------------
// Qhat^T[c][tok] = sum_b Gt_i[c][b] Qlat[tok][b];  one workgroup per head slot, wave = c-block
// ---------------------------------------------------------------------------------------
// The launch also finishes the factor projection, whose product leaves split-K partial tiles
// ([split][sequence][R2 + D (+ D)] fp32): every head's workgroup sums the Qlat columns of all sequences into
// LDS itself (a few hundred KB that stay in L2; all loads of a thread issued together), and the workgroups
// behind the heads' sum one 32-column block of the key or value part each and run the projection's epilogue
// on it (rotation, cache rows).  With one split the product has run its epilogue already and Qlat is read
// from where it put it.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_qhat_kernel(DecodeArgs p, GemmArgs g) {
  constexpr int CB = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* Ql = reinterpret_cast<T*>(smem_raw);                         // [32][R2 + pad], acc order inside 32-blocks
  const int RE = p.R2 + 16 / (int)sizeof(T);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, tok = lane % 32;
  const int n_heads_wg = p.HB * 32;
  const int Mp = g.R2 + (g.shared_kv ? 1 : 2) * g.D;
  constexpr int U = 8;                                            // partial tiles whose loads are issued together

  if ((int)blockIdx.x >= n_heads_wg) {                            // ---- a key / value block of the projection
    if (wave != 0) return;
    const int m0 = g.R2 + ((int)blockIdx.x - n_heads_wg) * 32;
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    if (tok < p.Bsz) {
      for (int z0 = 0; z0 < g.ksplit; z0 += U) {
        f32x4 v[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const float* src = g.part + ((long)min(z0 + u, g.ksplit - 1) * p.Bsz + tok) * Mp + m0 + 4 * h;
#pragma unroll
          for (int q = 0; q < 4; ++q) v[u][q] = *reinterpret_cast<const f32x4*>(src + 8 * q);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (z0 + u < g.ksplit)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
              for (int r = 0; r < 4; ++r) acc[4 * q + r] += v[u][q][r];
      }
    }
    epilogue_block<T>(g, acc, m0, tok);
    return;
  }

  const int head = blockIdx.x;                                    // 0 .. HB*32-1
  // this wave's first block of core fragments is requested before the sum: the launch is a chain of round trips
  const int nbb = p.R2 / 32;
  const T* Gt = static_cast<const T*>(p.Gt) + (long)min(head, p.nH - 1) * D * p.R2;
  constexpr int PRE = 4;
  Frag<T> gf0[PRE];
#pragma unroll
  for (int bb = 0; bb < PRE; ++bb)
    gf0[bb] = load_frag_major<T>(Gt + (long)(min(wave, CB - 1) * nbb + min(bb, nbb - 1)) * kFragBlockElems, lane);

  // ---- Qlat [sequence][R2] in the storage type, acc order -> LDS ----
  for (int ci = threadIdx.x; ci < 32 * (p.R2 / 4); ci += 256) {
    const int t = ci / (p.R2 / 4), k = (ci % (p.R2 / 4)) * 4;     // four natural indices k..k+3 keep their order
    const int pos = (k & ~31) + acc_pos(k & 31);
    if (g.ksplit > 1) {
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      if (t < p.Bsz) {
        for (int z0 = 0; z0 < g.ksplit; z0 += 2 * U) {
          f32x4 v[2 * U];
#pragma unroll
          for (int u = 0; u < 2 * U; ++u)
            v[u] = *reinterpret_cast<const f32x4*>(g.part + ((long)min(z0 + u, g.ksplit - 1) * p.Bsz + t) * Mp + k);
#pragma unroll
          for (int u = 0; u < 2 * U; ++u)
            if (z0 + u < g.ksplit) sum += v[u];
        }
      }
      store4(Ql + t * RE + pos, sum[0], sum[1], sum[2], sum[3]);
    } else {
      const T* src = static_cast<const T*>(p.Qlat) + (long)t * p.R2 + pos;   // already in acc order
      if (t < p.Bsz) store4(Ql + t * RE + pos, to_f32(src[0]), to_f32(src[1]), to_f32(src[2]), to_f32(src[3]));
      else store4(Ql + t * RE + pos, 0.f, 0.f, 0.f, 0.f);
    }
  }
  __syncthreads();

  T* Qh = static_cast<T*>(p.Qh);
  for (int cb = wave; cb < CB; cb += 4) {
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    if (head < p.nH) {
#pragma unroll
      for (int bb = 0; bb < PRE; ++bb)
        if (bb < nbb) {
          const Frag<T> gf = cb == wave ? gf0[bb] : load_frag_major<T>(Gt + (long)(cb * nbb + bb) * kFragBlockElems, lane);
          mma32(acc, gf, load_frag<T>(Ql + tok * RE + bb * 32 + 16 * h));
        }
      for (int bb = PRE; bb < nbb; ++bb)
        mma32(acc, load_frag_major<T>(Gt + (long)(cb * nbb + bb) * kFragBlockElems, lane),
              load_frag<T>(Ql + tok * RE + bb * 32 + 16 * h));
      if (p.rope != nullptr && tok < p.Bsz) {
        const f32x4* tab = reinterpret_cast<const f32x4*>(p.rope) + (long)(cb * 8 + h) * p.rope_ld + (p.kv_len[tok] - 1);
        f32x4 cs[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) cs[q] = tab[(long)2 * q * p.rope_ld];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; e += 2) {
            float x0 = acc[4 * q + e], x1 = acc[4 * q + e + 1];
            acc[4 * q + e] = x0 * cs[q][e] - x1 * cs[q][e + 1];
            acc[4 * q + e + 1] = x0 * cs[q][e + 1] + x1 * cs[q][e];
          }
      }
    }
    if (tok < p.Bsz) {
      T* row = Qh + ((long)tok * p.HB * 32 + head) * D;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        store4(row + cb * 32 + 8 * q + 4 * h, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// split-KV attention over cache rows [first, last) of sequence b
// ---------------------------------------------------------------------------------------
template <typename T, int D, int BC> struct DecLds {
  static constexpr int kRowElems = D + 16 / sizeof(T);
  static constexpr int kTileElems = BC * kRowElems;
  static constexpr int kStageElems = 2 * kTileElems;              // K tile, V tile
  static constexpr size_t kBytes = 2ul * kStageElems * sizeof(T);
};


// SH: shared key-value latent (one unrotated cache; keys rotated as a tile is staged)
template <typename T, int D, int BC, int HB, bool SH>
__global__ __launch_bounds__(256) void decode_attn_kernel(DecodeArgs p) {
  constexpr int CB = D / 32, NB = BC / 32;
  constexpr int CE = 16 / sizeof(T);
  constexpr int CPR = D / CE;                                     // 16-byte chunks per tile row
  constexpr int PT = BC * CPR / 256;                              // chunks per thread per tile
  static_assert((BC * CPR) % 256 == 0, "tile must fill all threads");
  using L = DecLds<T, D, BC>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);

  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;
  const int b = blockIdx.y, split = blockIdx.x;
  const int Lb = p.kv_len[b];
  const int nt_all = (Lb + BC - 1) / BC;
  const int per = (nt_all + p.nsplit - 1) / p.nsplit;
  const int t_first = split * per, t_last = min(nt_all, t_first + per);
  const int HB32 = HB * 32;

  float* pm = p.part_m + ((long)b * p.nsplit + split) * HB32;
  float* pl = p.part_l + ((long)b * p.nsplit + split) * HB32;
  float* po = p.part_o + ((long)b * p.nsplit + split) * HB32 * D;

  // query fragments: lane = head, natural order in c
  Frag<T> qf[HB][CB];
  {
    const T* Qh = static_cast<const T*>(p.Qh) + (long)b * HB32 * D;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) qf[hb][cb] = load_frag<T>(Qh + (long)(hb * 32 + lr) * D + cb * 32 + 16 * h);
  }
  const bool has_c = wave < CB;                                   // this wave's value block
  const int cbw = has_c ? wave : 0;
  f32x16 oacc[HB];
  float m_run[HB], l_run[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    m_run[hb] = -INFINITY;
    l_run[hb] = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[hb][e] = 0.f;
  }

  // Cache rows travel global -> registers -> LDS.  Two register sets alternate, each filled two
  // tiles ahead of its use by buffer loads whose range check supplies the zeros (rows past
  // kv_len, channels past r3 / rt3, tiles past this split), so no load sits behind a branch and
  // two tiles per workgroup are always in flight.
  const T* Kc = static_cast<const T*>(p.Kcache) + (long)b * p.Lmax * p.r3;
  const T* Vc = static_cast<const T*>(p.Vcache) + (long)b * p.Lmax * p.rt3;
  const long lim = 0x7fffffffl;
  const long kbytes = (long)Lb * p.r3 * (long)sizeof(T), vbytes = (long)Lb * p.rt3 * (long)sizeof(T);
  __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(Kc), 0, (int)(kbytes > lim ? lim : kbytes), 0x00020000);
  __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(Vc), 0, (int)(vbytes > lim ? lim : vbytes), 0x00020000);
  struct Set { u32x4 k[PT], v[PT]; } ra, rb;
  int srow[PT], scol[PT];
#pragma unroll
  for (int i = 0; i < PT; ++i) {
    const int ci = threadIdx.x + i * 256;
    srow[i] = ci / CPR;
    scol[i] = (ci % CPR) * CE;
  }
  auto g_load = [&](Set& r, int tile) {
    const bool live = tile < t_last;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const long n = (long)tile * BC + srow[i];
      const uint32_t ko = (live && scol[i] < p.r3) ? (uint32_t)((n * p.r3 + scol[i]) * (long)sizeof(T)) : 0x80000000u;
      const uint32_t vo = (live && !SH && scol[i] < p.rt3) ? (uint32_t)((n * p.rt3 + scol[i]) * (long)sizeof(T)) : 0x80000000u;
      r.k[i] = __builtin_amdgcn_raw_buffer_load_b128(krs, ko, 0, 0);
      r.v[i] = __builtin_amdgcn_raw_buffer_load_b128(vrs, vo, 0, 0);
    }
  };
  // Shared key-value latent: the cache row is the value as it stands and becomes the key once
  // rotated to its position n = tile*BC + row.  The rotation by n is the rotation by tile*BC
  // followed by the rotation by row: the second is the same for every tile and is fetched once per
  // thread (its chunks sit at fixed rows and channels of a tile), the first is one table entry per
  // channel quad per tile.  Both come from the context's table.
  constexpr int QPC = CE / 4;                                     // table entries per 16-byte chunk
  const bool rotate_on_load = SH && p.rope != nullptr;
  f32x4 rot_row[PT][QPC], rot_tile[QPC];
  if (rotate_on_load) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const f32x4* tab = reinterpret_cast<const f32x4*>(p.rope) + (long)(scol[i] / 4) * p.rope_ld + min(srow[i], p.rope_ld - 1);
#pragma unroll
      for (int q = 0; q < QPC; ++q) rot_row[i][q] = tab[(long)q * p.rope_ld];
    }
  }
  auto rot_load = [&](int tile) {                                 // every chunk of a thread has the same channels
    if (!rotate_on_load) return;
    const f32x4* tab = reinterpret_cast<const f32x4*>(p.rope) + (long)(scol[0] / 4) * p.rope_ld +
                       min((long)tile * BC, (long)p.rope_ld - 1); // a dead tile holds zeros: any entry serves
#pragma unroll
    for (int q = 0; q < QPC; ++q) rot_tile[q] = tab[(long)q * p.rope_ld];
  };
  auto rotated = [&](const u32x4& raw, const f32x4 (&row)[QPC]) -> u32x4 {
    float x[CE];
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        x[2 * j] = __uint_as_float(raw[j] << 16);
        x[2 * j + 1] = __uint_as_float(raw[j] & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) x[j] = __uint_as_float(raw[j]);
    }
#pragma unroll
    for (int q = 0; q < QPC; ++q)
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        const float ca = row[q][e], sa = row[q][e + 1], cb = rot_tile[q][e], sb = rot_tile[q][e + 1];
        const float c = ca * cb - sa * sb, sn = sa * cb + ca * sb;   // angle addition
        const float x0 = x[4 * q + e], x1 = x[4 * q + e + 1];
        x[4 * q + e] = x0 * c - x1 * sn;
        x[4 * q + e + 1] = x0 * sn + x1 * c;
      }
    u32x4 out;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        f32x2 two = {x[2 * j], x[2 * j + 1]};
        out[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) out[j] = __float_as_uint(x[j]);
    }
    return out;
  };
  auto s_store = [&](const Set& r, int stage) {
    T* ks = smem + (long)stage * L::kStageElems;
    T* vs = ks + L::kTileElems;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const u32x4 kv = rotate_on_load ? rotated(r.k[i], rot_row[i]) : r.k[i];
      *reinterpret_cast<u32x4*>(ks + srow[i] * L::kRowElems + scol[i]) = kv;
      *reinterpret_cast<u32x4*>(vs + srow[i] * L::kRowElems + scol[i]) = SH ? r.k[i] : r.v[i];
    }
  };

  // one tile from LDS stage `cur`
  auto compute = [&](int tile, int cur) {
    const T* ks = smem + (long)cur * L::kStageElems;
    const T* vs = ks + L::kTileElems;
    const int n0 = tile * BC;

    f32x16 s[HB][NB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[hb][nb][e] = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        Frag<T> kf = load_frag<T>(ks + (nb * 32 + lr) * L::kRowElems + cb * 32 + 16 * h);
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) mma32(s[hb][nb], kf, qf[hb][cb]);
      }
    if (n0 + BC > Lb) {
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            int n = n0 + nb * 32 + 8 * (e / 4) + 4 * h + (e % 4);
            if (n >= Lb) s[hb][nb][e] = -INFINITY;
          }
    }
    Frag<T> pf[HB][NB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      float mx = -INFINITY;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[hb][nb][e]);
      mx = halves_max(mx);
      const float m_new = fmaxf(m_run[hb], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = fast_exp2(m_run[hb] - m_use);
      m_run[hb] = m_new;
      float rs = 0.f;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float pv = fast_exp2(s[hb][nb][e] - m_use);
          s[hb][nb][e] = pv;
          rs += pv;
        }
        pf[hb][nb] = to_frag<T>(s[hb][nb]);
      }
      l_run[hb] = l_run[hb] * alpha + rs;
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[hb][e] *= alpha;
    }
    // O^T[c][head] += V^T[c][n] P^T[n][head] for this wave's value block: lane = channel c,
    // half h takes keys 8q+4h+r of each 32-key block from the row-major V tile (transposing LDS loads)
    if (has_c) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const Frag<T> vf = load_frag_tr(vs, L::kRowElems, nb * 32, cbw * 32, lane);
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) mma32(oacc[hb], vf, pf[hb][nb]);
      }
    }
  };

  // The slices of different workgroups lie a power of two apart in memory; walking them in step
  // would keep all workgroups on the same memory channels.  Each workgroup therefore starts at
  // its own tile of its slice and wraps around (the online softmax does not care about order).
  const int cnt = max(t_last - t_first, 0);
  const int first = cnt > 0 ? (int)((split * 5u + b * 3u) % (unsigned)cnt) : 0;
  auto tile_at = [&](int j) {                                     // j-th tile in this workgroup's order
    int r = j + first;
    if (r >= cnt) r -= cnt;
    return j < cnt ? t_first + r : t_last;                        // past the end: a dead tile
  };
  g_load(ra, tile_at(0));
  g_load(rb, tile_at(1));
  rot_load(tile_at(0));
  s_store(ra, 0);
  g_load(ra, tile_at(2));
  __syncthreads();
  for (int j = 0; j < cnt; j += 2) {
    rot_load(tile_at(j + 1));
    compute(tile_at(j), 0);
    s_store(rb, 1);
    g_load(rb, tile_at(j + 3));
    __syncthreads();
    rot_load(tile_at(j + 2));
    if (j + 1 < cnt) compute(tile_at(j + 1), 1);
    s_store(ra, 0);
    g_load(ra, tile_at(j + 4));
    __syncthreads();
  }

  // partial results: natural order in c, un-normalised, with running max and sum (base-2 domain)
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    const float l_tot = halves_sum(l_run[hb]);
    if (wave == 0 && h == 0) {
      pm[hb * 32 + lr] = m_run[hb];
      pl[hb * 32 + lr] = l_tot;
    }
    if (has_c) {
      float* row = po + (long)(hb * 32 + lr) * D + cbw * 32;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        store4(row + 8 * q + 4 * h, oacc[hb][4 * q], oacc[hb][4 * q + 1], oacc[hb][4 * q + 2], oacc[hb][4 * q + 3]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// split-KV attention over a shared key-value latent, bf16, cache rows exactly D wide
// ---------------------------------------------------------------------------------------
// With one cache to read, a step has half the bytes to stream and the arithmetic per byte doubles: the
// kernel above (every wave computes every score of a tile) is then bound by its own instructions.  Here
// the slice of a workgroup is walked in rounds of 128 keys; wave w owns keys 32w .. 32w+31 of every round
// and does ALL the work for them: scores against every head, its own running softmax, and the product
// with the values for all D channels.  Nothing is shared between the waves while they stream, so there is
// no barrier in the loop and no score is computed twice; the four partial results are merged through LDS
// once at the end.  A wave moves its 32 cache rows from global memory straight into one of its two LDS
// stages (no registers in between), two rounds ahead.  The tile serves as value tile as it stands
// (transposing reads) and as key tile, its fragments being rotated in registers by the angle of
// (first key of the tile) + (row): the entries of the first come with the tile as one extra 1 KB piece of
// the rotation table (one 16-byte entry per channel quad), those of the second are the same for every tile
// and sit in an LDS table that all waves read.
template <int D, bool ROT> struct DecWaveLds {
  static constexpr int kTile = 32 * D;                            // elements of a 32-key tile
  static constexpr int kRot = ROT ? 512 : 0;                      // one 1 KB piece of table entries
  static constexpr int kStage = kTile + kRot;
  static constexpr size_t kStagesBytes = 4ul * 2 * kStage * sizeof(bf16);
  // ROT: behind the stages, the rotation of every tile row, [D/4 quads][32 rows] x 16 bytes
  static constexpr size_t kRowTabBytes = ROT ? (size_t)(D / 4) * 32 * 16 : 0;
  static constexpr size_t pipeline_bytes() { return kStagesBytes + kRowTabBytes; }
  static constexpr size_t merge_bytes(int HB) { return 4ul * HB * 32 * (D + 4 + 2) * sizeof(float); }
  static constexpr size_t bytes(int HB) { return pipeline_bytes() > merge_bytes(HB) ? pipeline_bytes() : merge_bytes(HB); }
};

// at most N vector-memory operations of this wave (loads, direct-to-LDS loads) still in flight
template <int N> __device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "six-bit counter");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
  asm volatile("" ::: "memory");
}
// every LDS read of this wave has returned
__device__ __forceinline__ void wait_lds() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xc07f);
  asm volatile("" ::: "memory");
}

// Up to 32 heads the kernel is held to 256 registers: with more, the compiler parks values in accumulation
// registers and pays a copy for every use by the vector unit.
template <int D, int HB, bool ROT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(HB == 1 ? 2 : 1, HB == 1 ? 2 : 1)))
void decode_attn_shared_kernel(DecodeArgs p) {
  using T = bf16;
  using L = DecWaveLds<D, ROT>;
  constexpr int CB = D / 32, CPR = D / 8;
  constexpr int PIECES = L::kTile / 512;                          // 1 KB pieces of a tile
  constexpr int HB32 = HB * 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int h = lane / 32, lr = lane % 32;
  const int b = blockIdx.y, split = blockIdx.x;
  const int Lb = p.kv_len[b];
  const int rounds_all = (Lb + kDecodeRoundWave - 1) / kDecodeRoundWave;
  const int per = (rounds_all + p.nsplit - 1) / p.nsplit;
  const int r_first = split * per, r_last = min(rounds_all, r_first + per);
  const int cnt = max(r_last - r_first, 0);                       // rounds of this workgroup

  f32x16 oacc[HB][CB];
  float m_run[HB], l_run[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    m_run[hb] = -INFINITY;
    l_run[hb] = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[hb][cb][e] = 0.f;
  }

  if (cnt > 0) {                                                  // (the same for the whole workgroup)
    T* wbase = reinterpret_cast<T*>(smem_raw) + (long)wave * 2 * L::kStage;
    const T* Lc = static_cast<const T*>(p.Kcache) + (long)b * p.Lmax * D;
    // The slices of different workgroups lie a power of two apart in memory: each workgroup starts at
    // its own round of its slice and wraps around (the online softmax does not care about order).
    const int first = (int)((split * 5u + b * 3u) % (unsigned)cnt);
    auto block_at = [&](int j) {                                  // this wave's 32-key block of round j
      int r = min(j, cnt - 1) + first;                            // past the end: the last round again (not used)
      if (r >= cnt) r -= cnt;
      return (r_first + r) * 4 + wave;
    };
    // Rows past the end of the sequence read its last row (they are masked below), so every address stays
    // inside the rows the sequence owns.
    auto issue = [&](int j, int st) {
      const int n0 = block_at(j) * 32;
      T* kt = wbase + (long)st * L::kStage;
#pragma unroll
      for (int q = 0; q < PIECES; ++q)
        dma_piece<T, CPR>(kt, q, lane, [&](int row) { return Lc + (long)min(n0 + row, Lb - 1) * D; });
      if constexpr (ROT) {
        const f32x4* tab = reinterpret_cast<const f32x4*>(p.rope) + (long)min(lane % 32, D / 4 - 1) * p.rope_ld +
                           min(n0, p.rope_ld - 1);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)tab,
                                         (__attribute__((address_space(3))) void*)(kt + L::kTile), 16, 0, 0);
      }
    };
    // direct-to-LDS loads of one stage; while a stage is read, at most the other one may still be in flight
    constexpr int OPS = PIECES + (ROT ? 1 : 0);

    // query fragments: lane = head, natural order in c
    Frag<T> qf[HB][CB];
    {
      const T* Qh = static_cast<const T*>(p.Qh) + (long)b * HB32 * D;
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) qf[hb][cb] = load_frag<T>(Qh + (long)(hb * 32 + lr) * D + cb * 32 + 16 * h);
    }
    f32x4* rowtab = reinterpret_cast<f32x4*>(smem_raw + L::kStagesBytes);
    if constexpr (ROT) {
      for (int i = threadIdx.x; i < (D / 4) * 32; i += 256)
        rowtab[i] = reinterpret_cast<const f32x4*>(p.rope)[(long)(i / 32) * p.rope_ld + min(i % 32, p.rope_ld - 1)];
    }
    wait_vm<0>();                                                 // plain loads out of the way of the counted ones
    if constexpr (ROT) __syncthreads();
    issue(0, 0);
    issue(1, 1);

    constexpr float kLazy = 8.f;
    const int xs = swz_x<CPR>(lr);
    auto round = [&](int j, int st) {
      const int n0 = block_at(j) * 32;
      const T* kt = wbase + (long)st * L::kStage;
      wait_vm<OPS>();
      f32x16 s[HB];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[hb][e] = 0.f;
      if constexpr (ROT) {
        // one 32-channel block at a time, the operands of the next one requested before this one is rotated:
        // key fragment, the tile's entries (angle of its first key) and the row's entries of 4 channel quads
        struct In { Frag<T> k; f32x4 t[4], a[4]; };
        const f32x4* rl = reinterpret_cast<const f32x4*>(kt + L::kTile);
        auto fetch = [&](int cb) {
          In in;
          in.k = load_frag_swz<T>(kt + lr * D, 4 * cb + 2 * h, xs);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            in.t[q] = rl[8 * cb + 4 * h + q];
            in.a[q] = rowtab[(8 * cb + 4 * h + q) * 32 + lr];
          }
          return in;
        };
        In cur = fetch(0);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          In nxt = cur;
          if (cb + 1 < CB) nxt = fetch(cb + 1);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            u32x4 raw = __builtin_bit_cast(u32x4, cur.k.v[i]);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              // dword d of chunk i: channel pair 4i+d of this lane's 8 pairs = quad 2i + d/2, entry (d%2)
              const f32x4 a = cur.a[2 * i + d / 2], t = cur.t[2 * i + d / 2];
              const int e = 2 * (d % 2);
              const float c = a[e] * t[e] - a[e + 1] * t[e + 1], sn = a[e + 1] * t[e] + a[e] * t[e + 1];
              const float x0 = __uint_as_float(raw[d] << 16), x1 = __uint_as_float(raw[d] & 0xffff0000u);
              f32x2 two = {x0 * c - x1 * sn, x0 * sn + x1 * c};
              raw[d] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
            }
            cur.k.v[i] = __builtin_bit_cast(bf16x8, raw);
          }
#pragma unroll
          for (int hb = 0; hb < HB; ++hb) mma32(s[hb], cur.k, qf[hb][cb]);
          __builtin_amdgcn_sched_barrier(0);
          cur = nxt;
        }
      } else {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          const Frag<T> kf = load_frag_swz<T>(kt + lr * D, 4 * cb + 2 * h, xs);
#pragma unroll
          for (int hb = 0; hb < HB; ++hb) mma32(s[hb], kf, qf[hb][cb]);
        }
      }
      // the value fragments (transposing reads of the same tile) are taken before the stage is refilled
      FragTrPending vp[CB];
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) vp[cb] = load_frag_tr_swz_start<CPR>(kt, 0, cb * 32, lane);
      wait_lds();
      issue(j + 2, st);
      Frag<T> vf[CB];
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) vf[cb] = load_frag_tr_finish(vp[cb]);

      if (n0 + 32 > Lb) {
#pragma unroll
        for (int hb = 0; hb < HB; ++hb)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (n0 + 8 * (e / 4) + 4 * h + (e % 4) >= Lb) s[hb][e] = -INFINITY;
      }
      // online softmax with a lazily raised reference: O and l are rescaled only when a block's maximum
      // exceeds the reference by more than kLazy (probabilities stay below 2^kLazy)
      Frag<T> pf[HB];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[hb][e]);
        mx = halves_max(mx);
        const bool upd = mx > m_run[hb] + kLazy;                  // -inf + kLazy = -inf: the first live block updates
        if (__builtin_amdgcn_ballot_w64(upd) != 0ull) {
          const float alpha = upd ? fast_exp2(m_run[hb] - mx) : 1.f;   // exp2(-inf) = 0: O and l are still zero
          if (upd) m_run[hb] = mx;
          l_run[hb] *= alpha;
#pragma unroll
          for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[hb][cb][e] *= alpha;
        }
        const float m_use = (m_run[hb] == -INFINITY) ? 0.f : m_run[hb];
        float rs = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          s[hb][e] = fast_exp2(s[hb][e] - m_use);
          rs += s[hb][e];
        }
        l_run[hb] += rs;
        pf[hb] = to_frag<T>(s[hb]);
      }
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) mma32(oacc[hb][cb], vf[cb], pf[hb]);
    };
    for (int j = 0; j < cnt; j += 2) {                            // the stage index is a constant in each call
      round(j, 0);
      if (j + 1 < cnt) round(j + 1, 1);
    }
    wait_vm<0>();                                                 // tiles requested past the end still land in LDS
  }
  __syncthreads();

  // ---- merge of the four waves' partial results through LDS -> one partial per workgroup ----
  // The lane index is formed afresh (from the execution mask, not from the thread index): every register the
  // loop above can have is in use, and an index kept across it would be spilled to scratch memory.
  const int lane_m = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int tid_m = wave * kWave + lane_m;
  const int h_m = lane_m / 32, lr_m = lane_m % 32;
  constexpr int RE = D + 4;                                       // padded row of a wave's O[head][c]
  float* mo = reinterpret_cast<float*>(smem_raw);                 // [4][HB32][RE]
  float* mm = mo + 4 * HB32 * RE;                                 // [4][HB32] references, then [4][HB32] sums
  float* ml = mm + 4 * HB32;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    const float l_tot = halves_sum(l_run[hb]);
    if (h_m == 0) {
      mm[wave * HB32 + hb * 32 + lr_m] = m_run[hb];
      ml[wave * HB32 + hb * 32 + lr_m] = l_tot;
    }
    float* row = mo + ((long)wave * HB32 + hb * 32 + lr_m) * RE;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<f32x4*>(row + cb * 32 + 8 * q + 4 * h_m) =
            f32x4{oacc[hb][cb][4 * q], oacc[hb][cb][4 * q + 1], oacc[hb][cb][4 * q + 2], oacc[hb][cb][4 * q + 3]};
  }
  __syncthreads();
  const long part = (long)blockIdx.y * p.nsplit + blockIdx.x;    // (formed here, not above: nothing to keep across the loop)
  float* pm = p.part_m + part * HB32;
  float* pl = p.part_l + part * HB32;
  float* po = p.part_o + part * HB32 * D;
  for (int idx = tid_m; idx < HB32 * D; idx += 256) {
    const int hd = idx / D, c = idx % D;
    float mw[4], mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      mw[w] = mm[w * HB32 + hd];
      mx = fmaxf(mx, mw[w]);
    }
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = mw[w] == -INFINITY ? 0.f : fast_exp2(mw[w] - mx);
      num += f * mo[((long)w * HB32 + hd) * RE + c];
      den += f * ml[w * HB32 + hd];
    }
    po[idx] = num;
    if (c == 0) {
      pm[hd] = mx;
      pl[hd] = den;
    }
  }
}

// ---------------------------------------------------------------------------------------
// merge of split partials and head merge in one launch: one workgroup per head
// ---------------------------------------------------------------------------------------
// The workgroup of head i merges the split partials of its head for every sequence (log-sum-exp, loads
// of 16 splits issued together), keeps the normalised O_i [sequence][c] in LDS in operand order, and multiplies it by the head's
// post-softmax core: Zpart_i^T[b][sequence] = sum_c G~_i[b][c] O_i[sequence][c].  The per-head
// contributions are written where a split-K product would put its partial tiles ([head][sequence][RT2],
// fp32), and the split-K reduction sums them over heads into Z.  This replaces two launches (the merge and
// a product that streams all heads' cores through a few workgroups) by one in which every head's 32 KB core
// block is read by its own workgroup.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_merge_heads_kernel(DecodeArgs p) {
  constexpr int CB = D / 32, CPT = D / 8;                         // channels per thread in the merge: 8 threads per row
  constexpr int RE = D + 16 / (int)sizeof(T);                     // padded LDS row
  __shared__ __attribute__((aligned(16))) T Ol[32 * RE];
  __shared__ float px[256 * (CPT + 2)];                           // partial merges of the thread groups of a sequence
  const int head = blockIdx.x;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;
  const int HB32 = p.HB * 32;
  const long ldg = (long)p.nH * D;

  // the first core block of this wave is requested before anything else: the launch is a chain of round trips
  const T* G = static_cast<const T*>(p.Gtil2) + (long)head * D;
  Frag<T> gf0[CB];
  if (wave < p.RT2 / 32) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) gf0[cb] = load_frag<T>(G + (long)(wave * 32 + lr) * ldg + cb * 32 + 16 * h);
  }

  // ---- merged, normalised O_i[tok][c] -> LDS (c stored in acc order inside each 32-block) ----
  // Eight threads share a sequence's D channels.  A sequence with more than 16 splits (few sequences, long caches)
  // gets S groups of such threads out of the 32 thread rows, as many as keep a group's share at 16 splits if the
  // batch leaves that many rows free: group sg merges the splits sg, sg + S, ..., and the S partial merges of a
  // sequence are combined through LDS in group order.  With 16 splits or fewer (S = 1) there is no exchange.  The
  // result does not depend on timing.
  {
    int Bp = 1;
    while (Bp < p.Bsz) Bp *= 2;                                   // batch rounded up to a power of two, 1 .. 32
    int S = 1;
    while (S * 16 < p.nsplit && 2 * S * Bp <= 32) S *= 2;
    const int row = threadIdx.x / 8, cg = threadIdx.x % 8, c0 = cg * CPT;
    const int tok = row % Bp, sg = row / Bp;
    float num[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) num[e] = 0.f;
    float mrun = -INFINITY, den = 0.f;
    if (tok < p.Bsz && sg < S) {
      constexpr int U = 16;                                       // splits whose loads are issued together (one
                                                                  // workgroup per compute unit: registers are plentiful)
      for (int s0 = sg; s0 < p.nsplit; s0 += U * S) {
        float mv[U], lv[U];
        f32x4 ov[U][CPT / 4];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const long ps = ((long)tok * p.nsplit + min(s0 + u * S, p.nsplit - 1)) * HB32 + head;
          mv[u] = p.part_m[ps];
          lv[u] = p.part_l[ps];
#pragma unroll
          for (int q = 0; q < CPT / 4; ++q) ov[u][q] = *reinterpret_cast<const f32x4*>(p.part_o + ps * D + c0 + 4 * q);
        }
        float mb = mrun;
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (s0 + u * S < p.nsplit) mb = fmaxf(mb, mv[u]);
        if (mb == -INFINITY) continue;                            // only empty splits so far
        const float a = fast_exp2(mrun - mb);                     // 0 while mrun is still -inf
        den *= a;
#pragma unroll
        for (int e = 0; e < CPT; ++e) num[e] *= a;
        mrun = mb;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const bool live = s0 + u * S < p.nsplit && mv[u] != -INFINITY;
          const float w = live ? fast_exp2(mv[u] - mb) : 0.f;
          den += w * lv[u];
#pragma unroll
          for (int q = 0; q < CPT / 4; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) num[4 * q + r] += w * ov[u][q][r];
        }
      }
    }
    if (S > 1) {                                                  // (the same for the whole workgroup)
      float* mine = px + (row * 8 + cg) * (CPT + 2);
#pragma unroll
      for (int e = 0; e < CPT; ++e) mine[e] = num[e];
      mine[CPT] = mrun;
      mine[CPT + 1] = den;
      __syncthreads();
      if (sg == 0 && tok < p.Bsz) {
        // reference = the largest of the groups' references; then the parts are scaled and added in group order
        float mall = mrun;
        for (int j = 1; j < S; ++j) mall = fmaxf(mall, px[((tok + j * Bp) * 8 + cg) * (CPT + 2) + CPT]);
        const float a0 = mrun == -INFINITY ? 0.f : fast_exp2(mrun - mall);   // (mall is finite: some split is not empty)
        den *= a0;
#pragma unroll
        for (int e = 0; e < CPT; ++e) num[e] *= a0;
        for (int j = 1; j < S; ++j) {
          const float* other = px + ((tok + j * Bp) * 8 + cg) * (CPT + 2);
          const float b = other[CPT] == -INFINITY ? 0.f : fast_exp2(other[CPT] - mall);
          den += other[CPT + 1] * b;
#pragma unroll
          for (int e = 0; e < CPT; ++e) num[e] += other[e] * b;
        }
      }
    }
    // thread row `row` writes LDS row `row`: a sequence's merged output from its group 0, zeros elsewhere
    const float inv = (sg == 0 && tok < p.Bsz) ? 1.f / den : 0.f;
#pragma unroll
    for (int q = 0; q < CPT / 4; ++q) {
      const int c = c0 + 4 * q;                                   // four consecutive channels keep their order
      store4(Ol + row * RE + (c & ~31) + acc_pos(c & 31), num[4 * q] * inv, num[4 * q + 1] * inv, num[4 * q + 2] * inv,
             num[4 * q + 3] * inv);
    }
  }
  __syncthreads();

  // ---- Zpart_i^T[b][tok]: wave w takes the 32-row blocks w, w+4, ... of the core ----
  for (int rb = wave; rb < p.RT2 / 32; rb += 4) {
    Frag<T> gf[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      gf[cb] = rb == wave ? gf0[cb] : load_frag<T>(G + (long)(rb * 32 + lr) * ldg + cb * 32 + 16 * h);
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) mma32(acc, gf[cb], load_frag<T>(Ol + lr * RE + cb * 32 + 16 * h));
    if (lr < p.Bsz) {
      float* dst = p.zpart + ((long)head * p.Bsz + lr) * p.RT2 + rb * 32 + 4 * h;
#pragma unroll
      for (int q = 0; q < 4; ++q) store4(dst + 8 * q, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// output projection of a decode step from the per-head contributions: Y = (sum_heads Zpart) U~2^T
// ---------------------------------------------------------------------------------------
// One workgroup per 128 output channels.  Every workgroup first sums the heads' contributions
// ([nH][Bsz][RT2] fp32, a few hundred KB that stay in L2) into Z [Bsz][RT2] in LDS, loads for 16 heads
// issued together, while its rows of the output factor are already on their way; then each wave multiplies
// its 32 factor rows by Z.  (The sum over heads is formed in head order by every workgroup alike.)
template <typename T>
__global__ __launch_bounds__(256) void decode_out_kernel(DecodeArgs p) {
  constexpr int PRE = 4;                                          // contraction blocks requested up front
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* Zl = reinterpret_cast<T*>(smem_raw);                         // [32][RT2 + pad]
  const int RE = p.RT2 + 16 / (int)sizeof(T);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;
  const int KB = p.RT2 / 32;
  const int m_row = blockIdx.x * 128 + wave * 32 + lr;            // this lane's factor row
  const bool row_ok = m_row < p.d_model;
  const T* urow = static_cast<const T*>(p.Ut2) + (long)(row_ok ? m_row : 0) * p.ut2_ld + 16 * h;
  Frag<T> uf[PRE];
#pragma unroll
  for (int kb = 0; kb < PRE; ++kb) uf[kb] = kb < KB && row_ok ? load_frag<T>(urow + kb * 32) : zero_frag<T>();

  // ---- Z = sum over heads, rounded to T as the stored Z of a prefill is ----
  {
    constexpr int U = 16;
    const int chunks = 32 * (p.RT2 / 4);                          // (sequence, 4 contraction indices)
    for (int ci = threadIdx.x; ci < chunks; ci += 256) {
      const int tok = ci / (p.RT2 / 4), k = (ci % (p.RT2 / 4)) * 4;
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      if (tok < p.Bsz) {
        for (int h0 = 0; h0 < p.nH; h0 += U) {
          f32x4 v[U];
#pragma unroll
          for (int u = 0; u < U; ++u)
            v[u] = *reinterpret_cast<const f32x4*>(p.zpart + ((long)min(h0 + u, p.nH - 1) * p.Bsz + tok) * p.RT2 + k);
#pragma unroll
          for (int u = 0; u < U; ++u)
            if (h0 + u < p.nH) sum += v[u];
        }
      }
      store4(Zl + tok * RE + k, sum[0], sum[1], sum[2], sum[3]);
    }
  }
  __syncthreads();

  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
  for (int kb = 0; kb < PRE; ++kb)
    if (kb < KB) mma32(acc, uf[kb], load_frag<T>(Zl + lr * RE + kb * 32 + 16 * h));
  for (int kb = PRE; kb < KB; ++kb) {
    const Frag<T> u = row_ok ? load_frag<T>(urow + kb * 32) : zero_frag<T>();
    mma32(acc, u, load_frag<T>(Zl + lr * RE + kb * 32 + 16 * h));
  }
  // lane = sequence, rows = output channels 8q+4h+r of this wave's block
  if (lr < p.Bsz) {
    T* yrow = static_cast<T*>(p.Y) + (long)lr * p.d_model + blockIdx.x * 128 + wave * 32 + 4 * h;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (blockIdx.x * 128 + wave * 32 + 8 * q + 4 * h < p.d_model)
        store4(yrow + 8 * q, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
  }
}

// ---------------------------------------------------------------------------------------
template <typename T, int D>
static hipError_t qhat_one(const DecodeArgs& a, const GemmArgs& proj, hipStream_t s) {
  const size_t smem = 32ul * (a.R2 + 16 / sizeof(T)) * sizeof(T);
  auto kern = decode_qhat_kernel<T, D>;
  static LdsOnce lds_once;                                       // one per kernel instantiation
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  // behind the heads' workgroups: one per 32-column block of the projection's key (and value) part
  const int kv_blocks = proj.ksplit > 1 ? (proj.shared_kv ? 1 : 2) * proj.D / 32 : 0;
  hipLaunchKernelGGL(kern, dim3(a.HB * 32 + kv_blocks), dim3(256), smem, s, a, proj);
  return hipGetLastError();
}
hipError_t launch_decode_qhat(int dtype, const DecodeArgs& a, const GemmArgs& proj, hipStream_t s) {
  if (dtype == 0) {
    switch (a.D) {
      case 32: return qhat_one<float, 32>(a, proj, s);
      case 64: return qhat_one<float, 64>(a, proj, s);
      case 128: return qhat_one<float, 128>(a, proj, s);
    }
  } else {
    switch (a.D) {
      case 32: return qhat_one<bf16, 32>(a, proj, s);
      case 64: return qhat_one<bf16, 64>(a, proj, s);
      case 128: return qhat_one<bf16, 128>(a, proj, s);
    }
  }
  return hipErrorInvalidValue;
}

template <typename T, int D, int BC, int HB, bool SH>
static hipError_t attn_one_sh(const DecodeArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  size_t smem = DecLds<T, D, BC>::kBytes;
  auto kern = decode_attn_kernel<T, D, BC, HB, SH>;
  static LdsOnce lds_once;                                       // one per kernel instantiation
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  if (k0 != nullptr && k1 != nullptr) hipExtLaunchKernelGGL(kern, dim3(a.nsplit, a.Bsz), dim3(256), (uint32_t)smem, s, k0, k1, 0, a);
  else hipLaunchKernelGGL(kern, dim3(a.nsplit, a.Bsz), dim3(256), smem, s, a);
  return hipGetLastError();
}
template <typename T, int D, int BC, int HB>
static hipError_t attn_one(const DecodeArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  return a.shared_kv ? attn_one_sh<T, D, BC, HB, true>(a, s, k0, k1) : attn_one_sh<T, D, BC, HB, false>(a, s, k0, k1);
}
template <typename T, int BC>
static hipError_t attn_dispatch(const DecodeArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  if (a.HB == 1) {
    switch (a.D) {
      case 32: return attn_one<T, 32, BC, 1>(a, s, k0, k1);
      case 64: return attn_one<T, 64, BC, 1>(a, s, k0, k1);
      case 128: return attn_one<T, 128, BC, 1>(a, s, k0, k1);
    }
  } else if (a.HB == 2) {
    switch (a.D) {
      case 32: return attn_one<T, 32, BC, 2>(a, s, k0, k1);
      case 64: return attn_one<T, 64, BC, 2>(a, s, k0, k1);
      case 128: return attn_one<T, 128, BC, 2>(a, s, k0, k1);
    }
  }
  return hipErrorInvalidValue;
}
template <int D, int HB, bool ROT>
static hipError_t shared_one(const DecodeArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  const size_t smem = DecWaveLds<D, ROT>::bytes(HB);
  auto kern = decode_attn_shared_kernel<D, HB, ROT>;
  static LdsOnce lds_once;                                       // one per kernel instantiation
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  if (k0 != nullptr && k1 != nullptr) hipExtLaunchKernelGGL(kern, dim3(a.nsplit, a.Bsz), dim3(256), (uint32_t)smem, s, k0, k1, 0, a);
  else hipLaunchKernelGGL(kern, dim3(a.nsplit, a.Bsz), dim3(256), smem, s, a);
  return hipGetLastError();
}
template <int D, int HB>
static hipError_t shared_variant(const DecodeArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  return a.rope != nullptr ? shared_one<D, HB, true>(a, s, k0, k1) : shared_one<D, HB, false>(a, s, k0, k1);
}
static hipError_t shared_dispatch(const DecodeArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  if (a.HB == 1) {
    switch (a.D) {
      case 32: return shared_variant<32, 1>(a, s, k0, k1);
      case 64: return shared_variant<64, 1>(a, s, k0, k1);
      case 128: return shared_variant<128, 1>(a, s, k0, k1);
    }
  } else if (a.HB == 2) {
    switch (a.D) {
      case 32: return shared_variant<32, 2>(a, s, k0, k1);
      case 64: return shared_variant<64, 2>(a, s, k0, k1);
      case 128: return shared_variant<128, 2>(a, s, k0, k1);
    }
  }
  return hipErrorInvalidValue;
}

hipError_t launch_decode_attn(int dtype, const DecodeArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  if (decode_wave_private(dtype, a.r3, a.D, a.shared_kv)) return shared_dispatch(a, s, k0, k1);
  return dtype == 0 ? attn_dispatch<float, 32>(a, s, k0, k1) : attn_dispatch<bf16, 64>(a, s, k0, k1);
}

template <typename T>
static hipError_t merge_heads_dispatch(const DecodeArgs& a, hipStream_t s) {
  switch (a.D) {
    case 32: hipLaunchKernelGGL((decode_merge_heads_kernel<T, 32>), dim3(a.nH), dim3(256), 0, s, a); break;
    case 64: hipLaunchKernelGGL((decode_merge_heads_kernel<T, 64>), dim3(a.nH), dim3(256), 0, s, a); break;
    case 128: hipLaunchKernelGGL((decode_merge_heads_kernel<T, 128>), dim3(a.nH), dim3(256), 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
hipError_t launch_decode_merge_heads(int dtype, const DecodeArgs& a, hipStream_t s) {
  return dtype == 0 ? merge_heads_dispatch<float>(a, s) : merge_heads_dispatch<bf16>(a, s);
}

template <typename T>
static hipError_t out_one(const DecodeArgs& a, hipStream_t s) {
  const size_t smem = 32ul * (a.RT2 + 16 / sizeof(T)) * sizeof(T);
  auto kern = decode_out_kernel<T>;
  static LdsOnce lds_once;                                       // one per kernel instantiation
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  hipLaunchKernelGGL(kern, dim3((a.d_model + 127) / 128), dim3(256), smem, s, a);
  return hipGetLastError();
}
hipError_t launch_decode_out(int dtype, const DecodeArgs& a, hipStream_t s) {
  return dtype == 0 ? out_one<float>(a, s) : out_one<bf16>(a, s);
}

}  // namespace ta
