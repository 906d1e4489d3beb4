// Fused prefill attention for Tucker attention (Sections "Rotary Position Embedding" and
// "Flash Attention" of the paper): per-head query Qhat_i = Qlat G_i built in a prologue,
// latent RoPE applied to it in fp32 registers, then online-softmax attention over the ONE
// latent K/V pair that all heads share, K/V tiles staged once in LDS per workgroup (loaded
// from global memory straight into LDS, no register stage) and reused by every head in it.
//
// Everything is computed transposed so that an accumulator lane owns one query:
//   Qhat^T[c][m] = sum_b Gt_i[c][b] Qlat[m][b]         rows c, columns m (queries)
//   S^T[n][m]    = sum_c K[n][c] Qhat[m][c]            rows n (keys),   columns m
//   O^T[c][m]   += sum_n V^T[c][n] P^T[n][m]           rows c (values), columns m
// A lane (column m, half h) then holds 16 keys of a 32-key block in registers, so the row
// maximum and row sum of the softmax are in-register reductions plus one exchange with the
// partner lane, and accumulators turn into the next product's operand without any
// cross-lane movement (see the fragment model in common.h).
//
// Workgroup = QW x HW waves = HW heads x (32*QB*QW) queries; K/V tile = BC keys, double buffered.
// Built as 8 waves: 4 heads x 2 query blocks of 32; waves w and w+4 share a SIMD.
#include <type_traits>

#include "common.h"
#include "params.h"

namespace ta {

template <typename T, int D, int BC> struct AttnLds {
  static constexpr int kKRowElems = D;                         // K tile rows: D channels, chunks swizzled
  static constexpr int kVRowElems = BC;                        // V^T tile rows: BC keys, chunks swizzled
  static constexpr int kKElems = BC * kKRowElems;
  static constexpr int kVElems = D * kVRowElems;
  static constexpr int kStageElems = kKElems + kVElems;
  static constexpr size_t kBytes = 2ul * kStageElems * sizeof(T);
};

template <typename T, int D, int QB, int BC, int QW, int HW>
__global__ __launch_bounds__(64 * QW * HW) void attn_prefill_kernel(AttnArgs p) {
  // QW x HW waves: wave (qw, hw) owns 32*QB queries of one head; the workgroup covers
  // TQ = 32*QB*QW consecutive tokens of HW heads
  constexpr int CB = D / 32, NB = BC / 32, TQ = 32 * QB * QW, NT = 64 * QW * HW;
  constexpr int CE = 16 / sizeof(T);                            // elements per 16-byte chunk
  using L = AttnLds<T, D, BC>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);

  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;
  const int n_qtiles = (p.N + TQ - 1) / TQ;
  // blockIdx.x = (head group, sequence) varies fastest, blockIdx.y = query tile: workgroups are
  // dispatched heavy (late causal tiles) first, and those running together read the same keys
  const int qt = n_qtiles - 1 - blockIdx.y;
  const int n_hg = (p.nH + HW - 1) / HW;
  // Workgroups are dealt to the 8 XCDs (each with its own L2) in turn.  The (sequence, head group) items of a
  // row are therefore re-indexed so that one XCD gets neighbouring items: it then sees the K/V of as few
  // sequences as possible, and those stay in its L2 for all the head groups and query tiles that read them.
  int item = blockIdx.x;
  if (gridDim.x % 8 == 0) item = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
  const int b = item / n_hg;
  const int head_raw = (item % n_hg) * HW + wave / QW;
  const bool head_ok = head_raw < p.nH;
  const int head = head_ok ? head_raw : p.nH - 1;
  const int t0 = qt * TQ;                                       // first token of the workgroup
  const int tw = t0 + (wave % QW) * 32 * QB;                    // first token of this wave
  const long tok_base = (long)b * p.Npad;

  // cooperative staging: K tile = BC rows x D, V^T tile = D rows x BC
  constexpr int KCH = BC * D / CE, VCH = D * BC / CE;           // 16-byte chunks
  constexpr int KCPR = D / CE, VCPR = BC / CE;                  // chunks per row
  const T* Kg = static_cast<const T*>(p.Kr) + tok_base * D;
  const T* Vg = static_cast<const T*>(p.Vt) + (long)b * D * p.Npad;
  // Tiles go from global memory straight into LDS (no registers): one instruction of a wave fills
  // 1 KB = 64 consecutive 16-byte chunks of the tile, lane l supplying the global address of the
  // chunk that belongs at position l.  Rows are not padded; instead chunk c of row r sits at
  // position c ^ ((r / W) & mask) of its row, which spreads the 16 rows that one fragment read
  // touches over all banks.
  constexpr int NWV = NT / 64;
  constexpr int WK = KCPR >= 16 ? 1 : 16 / KCPR, MK = (KCPR >= 16 ? 16 : KCPR) - 1;
  constexpr int WV = VCPR >= 16 ? 1 : 16 / VCPR, MV = (VCPR >= 16 ? 16 : VCPR) - 1;
  static_assert(KCH % 64 == 0 && VCH % 64 == 0, "whole 1 KB pieces");
  auto dma_load = [&](int ktile, int vtile, int stage) {
    T* ks = smem + (long)stage * L::kStageElems;
    T* vs = ks + L::kKElems;
#pragma unroll
    for (int i = 0; i < (KCH / 64 + NWV - 1) / NWV; ++i) {
      const int q = i * NWV + wave;                              // 1 KB piece of the K tile
      if (q < KCH / 64) {
        const int ci = q * 64 + lane, row = ci / KCPR, pos = ci % KCPR;
        const int c = pos ^ ((row / WK) & MK);
        const T* g = Kg + (long)(ktile * BC + row) * D + c * CE;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                         (__attribute__((address_space(3))) void*)(ks + q * 64 * CE), 16, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < (VCH / 64 + NWV - 1) / NWV; ++i) {
      const int q = i * NWV + wave;
      if (q < VCH / 64) {
        const int ci = q * 64 + lane, row = ci / VCPR, pos = ci % VCPR;
        const int c = pos ^ ((row / WV) & MV);
        const T* g = Vg + (long)row * p.Npad + vtile * BC + c * CE;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                         (__attribute__((address_space(3))) void*)(vs + q * 64 * CE), 16, 0, 0);
      }
    }
  };
  const int xk = (lr / WK) & MK, xv = (lr / WV) & MV;            // swizzle of this lane's fragment rows
  // fragment of row-chunks k0 .. (16 elements) of a swizzled row
  auto frag_swz = [&](const T* rowp, int k0, int x) -> Frag<T> {
    Frag<T> f;
    if constexpr (sizeof(T) == 2) {
      f.v[0] = *reinterpret_cast<const bf16x8*>(rowp + ((k0) ^ x) * CE);
      f.v[1] = *reinterpret_cast<const bf16x8*>(rowp + ((k0 + 1) ^ x) * CE);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) f.v[j] = *reinterpret_cast<const f32x4*>(rowp + ((k0 + j) ^ x) * CE);
    }
    return f;
  };

  dma_load(0, 0, 0);                                           // in flight during the prologue (the V part of stage 0 is never read)

  // ---- prologue: Qhat^T = Gt_i * Qlat^T, RoPE, -> B-operand fragments ---------------------
  // Operand fragments are fetched two contraction blocks ahead of their product; the rotation
  // table entries of this lane's token are fetched after the last product, into the registers
  // the operands leave free.
  Frag<T> qf[QB][CB];
  {
    f32x16 qa[QB][CB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) qa[qb][cb][e] = 0.f;
    // Gt_i is fragment-major: block (cb, bb) is one contiguous kilobyte-per-load piece
    const int nbb = p.R2 / 32;
    const T* Gt = static_cast<const T*>(p.Gt) + (long)head * D * p.R2;
    const T* Ql = static_cast<const T*>(p.Qlat) + (tok_base + tw + lr) * p.R2 + 16 * h;   // tw+lr < Npad
    // two register sets, filled alternately two contraction blocks ahead (no copies between
    // them); a block index past the end re-reads the last block, whose product is skipped
    struct Set { Frag<T> xq[QB], gf[CB]; } sa, sb;
    auto fetch = [&](Set& st, int bb) {
      const int bc = min(bb, nbb - 1);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) st.xq[qb] = load_frag<T>(Ql + (long)32 * qb * p.R2 + bc * 32);
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) st.gf[cb] = load_frag_major<T>(Gt + (long)(cb * nbb + bc) * kFragBlockElems, lane);
    };
    auto multiply = [&](const Set& st) {
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mma32(qa[qb][cb], st.gf[cb], st.xq[qb]);
    };
    constexpr bool kTwoSets = 2 * sizeof(Set) <= 96 * 4;        // else one set (wide fp32 fragments)
    fetch(sa, 0);
    if (kTwoSets) {
      fetch(sb, 1);
      for (int bb = 0; bb < nbb; bb += 2) {
        __builtin_amdgcn_sched_barrier(0);
        multiply(sa);
        __builtin_amdgcn_sched_barrier(0);
        fetch(sa, bb + 2);
        __builtin_amdgcn_sched_barrier(0);
        if (bb + 1 < nbb) multiply(sb);
        __builtin_amdgcn_sched_barrier(0);
        fetch(sb, bb + 3);
      }
    } else {
      for (int bb = 0; bb < nbb; ++bb) {
        multiply(sa);
        fetch(sa, bb + 1);
      }
    }
    __builtin_amdgcn_sched_barrier(0);                          // the table entries reuse the operand registers
    if (p.rope != nullptr) {
      f32x4 cs[QB][CB][4];                                      // (cos, sin) of channel pairs 8q+4h+{0,2}
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int m = min(tw + 32 * qb + lr, p.N - 1);          // padding tokens borrow the last row
        const f32x4* tab = reinterpret_cast<const f32x4*>(p.rope) + (long)h * p.rope_ld + p.pos0 + m;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
          for (int q = 0; q < 4; ++q) cs[qb][cb][q] = tab[(long)(cb * 8 + 2 * q) * p.rope_ld];
      }
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; e += 2) {
              float x0 = qa[qb][cb][4 * q + e], x1 = qa[qb][cb][4 * q + e + 1];
              qa[qb][cb][4 * q + e] = x0 * cs[qb][cb][q][e] - x1 * cs[qb][cb][q][e + 1];
              qa[qb][cb][4 * q + e + 1] = x0 * cs[qb][cb][q][e + 1] + x1 * cs[qb][cb][q][e];
            }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) qf[qb][cb] = to_frag<T>(qa[qb][cb]);
  }

  // ---- main loop over key tiles ----------------------------------------------------------
  // Online softmax with a lazily updated reference exponent: probabilities are formed as
  // exp2(s - m_ref) where m_ref is the row maximum seen when it was last refreshed; it is
  // refreshed (and O, l rescaled) only when a tile's maximum exceeds it by more than kLazy, so
  // the common tile does no rescaling.  The subtraction costs nothing: a score block is accumulated
  // on top of -m_ref.  Values stay below 2^kLazy; the final O / l is exact.
  constexpr float kLazy = 8.f;
  f32x16 oacc[QB][CB];
  float m_ref[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_ref[qb] = 0.f;
    l_run[qb] = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[qb][cb][e] = 0.f;
  }

  // keys needed: causal -> 0 .. t0+TQ-1 (clipped to N), else 0 .. N-1
  const int kv_end = p.causal ? min(p.N, t0 + TQ) : p.N;
  const int n_tiles = (kv_end + BC - 1) / BC;

  // The two waves that share a SIMD (waves w and w+4) go through a key tile in opposite order, so
  // that one is in its MFMA phase while the other is in its softmax (VALU) phase:
  //   interval t, waves 0..3:  O += V(t-1) P(t-1);  S = K(t) Qhat;  P(t) = softmax step of S
  //   interval t, waves 4..7:  P(t-1) = softmax step of S;  O += V(t-1) P(t-1);  S = K(t) Qhat
  // Both read K(t) and V(t-1) in interval t, so LDS stage t%2 holds exactly that pair, and the
  // pair of interval t+1 is staged meanwhile; one barrier per interval, n_tiles+1 intervals.
  f32x16 s[QB][NB];
  Frag<T> pf[QB][NB];
  f32x16 negm[QB];                                              // -reference in all 16 registers: start of a score block
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int e = 0; e < 16; ++e) negm[qb][e] = 0.f;
  // MFMA phase: O += V(tile-1) P(tile-1) (if PV) and then S = K(tile) Qhat (if SS), as ONE stream
  // of operand fragments read from LDS through a ring of kRing registers sets: the read of
  // fragment i+kRing-1 is issued before the product with fragment i, so a product never waits
  // for the read issued just before it.
  constexpr int kRing = sizeof(T) == 2 ? 4 : 2;                 // fp32 fragments are twice as large
  auto mfma_phase = [&](auto pv_c, auto ss_c, int tile) {
    constexpr bool PV = decltype(pv_c)::value, SS = decltype(ss_c)::value;
    constexpr int NPV = PV ? CB * NB : 0, NSS = SS ? NB * CB : 0, TOT = NPV + NSS;
    const T* st = smem + (long)(tile & 1) * L::kStageElems;    // K(tile) and V(tile-1) share a stage
    const T* kbase = st + lr * L::kKRowElems;
    const T* vbase = st + L::kKElems + lr * L::kVRowElems;
    constexpr int FC = 16 / CE;                                   // 16-byte chunks per fragment half-slice
    auto fetch = [&](int i) -> Frag<T> {
      if (i < NPV) return frag_swz(vbase + (i / NB) * 32 * L::kVRowElems, (i % NB) * 2 * FC + h * FC, xv);
      const int j = i - NPV;
      return frag_swz(kbase + (j / CB) * 32 * L::kKRowElems, (j % CB) * 2 * FC + h * FC, xk);
    };
    Frag<T> ring[kRing];
    // the partner wave of the SIMD is in its softmax or staging phase meanwhile: matrix work goes first
    // (268 against 273 us at 4096 tokens; the reverse assignment takes 282)
    __builtin_amdgcn_s_setprio(3);
#pragma unroll
    for (int i = 0; i < kRing - 1 && i < TOT; ++i) ring[i] = fetch(i);
#pragma unroll
    for (int i = 0; i < TOT; ++i) {
      if (i + kRing - 1 < TOT) ring[(i + kRing - 1) % kRing] = fetch(i + kRing - 1);
      __builtin_amdgcn_sched_barrier(0);                        // keep the read ahead of the products
      const Frag<T>& f = ring[i % kRing];
      if (i < NPV) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mma32(oacc[qb][i / NB], f, pf[qb][i % NB]);
      } else {
        const int j = i - NPV;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          // a score block starts from -reference, so the products form S - reference directly
          if (j % CB == 0) mma32_from(s[qb][j / CB], negm[qb], f, qf[qb][0]);
          else mma32(s[qb][j / CB], f, qf[qb][j % CB]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_setprio(0);
  };
  constexpr std::true_type kYes{};
  constexpr std::false_type kNo{};
  auto do_softmax = [&](int tile) {                             // s of `tile` -> pf, running sums
    const int n0 = tile * BC;
    // mask: keys beyond the sequence, and (causal) keys after the query
    const bool need_mask = (n0 + BC > p.N) || (p.causal && n0 + BC - 1 > t0);
    if (need_mask) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int m = tw + 32 * qb + lr;
        const int lim = p.causal ? min(m, p.N - 1) : p.N - 1;   // last visible key
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            int n = n0 + nb * 32 + 8 * (e / 4) + 4 * h + (e % 4);
            if (n > lim) s[qb][nb][e] = -INFINITY;
          }
      }
    }
    // online softmax (scores already carry log2(e)/sqrt(d_head))
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float mx = -INFINITY;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[qb][nb][e]);
      mx = halves_max(mx);                                      // relative to the reference in force
      const bool upd = (tile == 0 || mx > kLazy) && mx != -INFINITY;
      if (__builtin_amdgcn_ballot_w64(upd) != 0ull) {
        const float delta = upd ? mx : 0.f;                     // new reference = old + delta
        const float alpha = tile == 0 ? 1.f : fast_exp2(-delta); // tile 0: O and l are still zero
        m_ref[qb] += delta;
        l_run[qb] *= alpha;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[qb][cb][e] *= alpha;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int e = 0; e < 16; ++e) s[qb][nb][e] -= delta;
#pragma unroll
        for (int e = 0; e < 16; ++e) negm[qb][e] = -m_ref[qb];
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[qb][nb][e] = fast_exp2(s[qb][nb][e]);
        pf[qb][nb] = to_frag<T>(s[qb][nb]);
        // 128 channels keep the matrix pipe busy: keep the row sum off it
        if constexpr (D >= 128) l_run[qb] = block_sum(s[qb][nb], l_run[qb]);
        else l_run[qb] = frag_sum(pf[qb][nb], l_run[qb]);
      }
    }
  };

  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  const int last = n_tiles - 1;
  // interval t reads stage t&1 = {K(t), V(t-1)}; stage (t+1)&1 was last read in interval t-1, so the
  // pair of interval t+1 is fetched into it while interval t computes
  if (wave < NT / 128) {                                        // ---- MFMA phase first
    dma_load(min(1, last), 0, 1);
    mfma_phase(kNo, kYes, 0);
    do_softmax(0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int t = 1; t < n_tiles; ++t) {
      dma_load(min(t + 1, last), t, (t + 1) & 1);
      mfma_phase(kYes, kYes, t);
      do_softmax(t);
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
    }
    mfma_phase(kYes, kNo, n_tiles);
  } else {                                                      // ---- softmax phase first
    dma_load(min(1, last), 0, 1);
    mfma_phase(kNo, kYes, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int t = 1; t < n_tiles; ++t) {
      dma_load(min(t + 1, last), t, (t + 1) & 1);
      do_softmax(t - 1);
      mfma_phase(kYes, kYes, t);
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
    }
    do_softmax(last);
    mfma_phase(kYes, kNo, n_tiles);
  }

  // ---- epilogue: normalise, store O[tok][head][c] (acc order in c) -------------------------
  // Rows of padding tokens (N <= m < Npad) are written as zeros, and their log-sum-exp as +inf,
  // so that a pass over all padded rows (the backward kernels) sees no undefined values.
  if (head_ok) {
    T* O = static_cast<T*>(p.O);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int m = tw + 32 * qb + lr;                          // < Npad
      const float l_tot = halves_sum(l_run[qb]);
      const float inv = m < p.N ? 1.f / l_tot : 0.f;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        f32x16 o = oacc[qb][cb];
#pragma unroll
        for (int e = 0; e < 16; ++e) o[e] = m < p.N ? o[e] * inv : 0.f;
        store_frag<T>(O + ((tok_base + m) * p.nH + head) * D + cb * 32 + 16 * h, to_frag<T>(o));
      }
      if (p.lse != nullptr && h == 0)
        p.lse[((long)b * p.nH + head) * p.Npad + m] = m < p.N ? m_ref[qb] + log2f(l_tot) : INFINITY;
    }
  }
}

template <typename T, int D, int QB, int BC, int QW, int HW>
static hipError_t launch_one(const AttnArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  constexpr int TQ = 32 * QB * QW;
  dim3 grid(((a.nH + HW - 1) / HW) * a.Bsz, (a.N + TQ - 1) / TQ);
  size_t smem = AttnLds<T, D, BC>::kBytes;
  auto kern = attn_prefill_kernel<T, D, QB, BC, QW, HW>;
  static LdsOnce lds_once;                                       // one per kernel instantiation
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  if (k0 != nullptr && k1 != nullptr) hipExtLaunchKernelGGL(kern, grid, dim3(64 * QW * HW), (uint32_t)smem, s, k0, k1, 0, a);
  else hipLaunchKernelGGL(kern, grid, dim3(64 * QW * HW), smem, s, a);
  return hipGetLastError();
}

hipError_t launch_attn_prefill(int dtype, const AttnArgs& a, hipStream_t s, hipEvent_t k0, hipEvent_t k1) {
  if (dtype == 0) {
    switch (a.D) {
      case 32: return launch_one<float, 32, 1, 32, 2, 4>(a, s, k0, k1);
      case 64: return launch_one<float, 64, 1, 32, 2, 4>(a, s, k0, k1);
      case 128: return launch_one<float, 128, 1, 32, 2, 4>(a, s, k0, k1);
    }
  } else {
    switch (a.D) {
      case 32: return launch_one<bf16, 32, 1, 64, 2, 4>(a, s, k0, k1);
      case 64: return launch_one<bf16, 64, 1, 64, 2, 4>(a, s, k0, k1);
      case 128: return launch_one<bf16, 128, 1, 64, 2, 4>(a, s, k0, k1);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace ta
