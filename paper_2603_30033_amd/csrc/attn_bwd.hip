// Backward pass of the fused prefill attention (the paper trains the layer, Section
// "Experiments", and its timing tables carry a backward column; the gradient itself is the
// derivative of Definition "Latent RoPE for Tucker Attention" followed by softmax attention over
// the shared latent keys and values).  Flash-style: no N x N matrix is kept; probabilities are
// recomputed from the saved log-sum-exp.
//
// With P_i = softmax(S_i), S_i = Q_i K^T (Q_i the rotated, scaled per-head query; K the rotated
// latent keys), O_i = P_i V, and upstream dO_i = dZ G~_i:
//     delta_i = rowsum(dO_i * O_i)          dP_i = dO_i V^T        dS_i = P_i * (dP_i - delta_i)
//     dQ_i = dS_i K                         dK = sum_i dS_i^T Q_i  dV = sum_i P_i^T dO_i
// Two kernels, neither with atomics:
//   bwd_dq   one wave = 32 queries of one head, walks the key tiles like the forward kernel:
//            builds Q_i and dO_i in a prologue from the latent query and dZ (and leaves copies of
//            both for the second kernel), accumulates dQ_i, removes the rotation and stores it.
//   bwd_dkv  a pair of waves = 32 keys kept in registers as operands, walks (head, query block)
//            pairs staged in LDS; one wave of the pair accumulates dV^T, the other dK^T; heads are
//            split into groups over workgroups, each writing a partial sum that kv_reduce adds up
//            (and un-rotates).
// Products are computed in the orientation that keeps the contraction index inside a lane (see
// the fragment model in common.h): bwd_dq keeps queries as MFMA columns, bwd_dkv keeps keys.
#include <type_traits>

#include "common.h"
#include "params.h"

namespace ta {

namespace {

constexpr float kLn2 = 0.6931471805599453f;

// acc[cb] = (32 rows c of core block cb) x (this wave's 32 tokens): sum_b G[c][b] xrow[token][b].
// G: one head's fragment-major blocks [cb][bb]; xrow: this lane's token row + 16*h.
template <typename T, int CB>
__device__ __forceinline__ void core_product(f32x16 (&acc)[CB], const T* G, const T* xrow, int nbb, int lane) {
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[cb][e] = 0.f;
  for (int bb = 0; bb < nbb; ++bb) {
    const Frag<T> x = load_frag<T>(xrow + bb * 32);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const Frag<T> g = load_frag_major<T>(G + (long)(cb * nbb + bb) * kFragBlockElems, lane);
      mma32(acc[cb], g, x);
    }
  }
}

// rotate (sign = +1) or un-rotate (sign = -1) the channel pairs of accumulator blocks whose column
// (lane) sits at table position pos
template <int CB>
__device__ __forceinline__ void rotate_blocks(f32x16 (&a)[CB], const float4* rope, int rope_ld, int pos, int h,
                                              float sign) {
  const f32x4* tab = reinterpret_cast<const f32x4*>(rope) + (long)h * rope_ld + pos;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    f32x4 cs[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) cs[q] = tab[(long)(cb * 8 + 2 * q) * rope_ld];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        const float x0 = a[cb][4 * q + e], x1 = a[cb][4 * q + e + 1];
        const float c = cs[q][e], s = sign * cs[q][e + 1];
        a[cb][4 * q + e] = x0 * c - x1 * s;
        a[cb][4 * q + e + 1] = x0 * s + x1 * c;
      }
  }
}

// element e of a fragment (same index as the accumulator register it came from)
__device__ __forceinline__ float frag_elem(const Frag<float>& f, int e) { return f.v[e / 4][e % 4]; }
__device__ __forceinline__ float frag_elem(const Frag<bf16>& f, int e) { return (float)f.v[e / 8][e % 8]; }

}  // namespace

// ---- dQ ----------------------------------------------------------------------------------------------
template <typename T, int D, int BC> struct DqLds {
  static constexpr int kRow = D + 16 / sizeof(T);               // K / V tile rows
  static constexpr int kTRow = BC + 16 / sizeof(T);             // K^T tile rows
  static constexpr int kKElems = BC * kRow;
  static constexpr int kTElems = D * kTRow;
  static constexpr int kStage = 2 * kKElems + kTElems;
  static constexpr size_t kBytes = 2ul * kStage * sizeof(T);
};

// Workgroup = 8 waves = 4 heads x 2 blocks of 32 queries (waves w and w+4 share a SIMD); key tiles
// of BC keys are staged once per workgroup and walked in 32-key halves, so that only one half's
// scores live in registers at a time.
template <typename T, int D, int BC>
__global__ __launch_bounds__(512) void bwd_dq_kernel(BwdArgs p) {
  constexpr int CB = D / 32, NB = BC / 32, HW = 4, QW = 2, TQ = 32 * QW, NT = 64 * HW * QW;
  constexpr int CE = 16 / sizeof(T);
  using L = DqLds<T, D, BC>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);

  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;
  const int n_qtiles = p.Npad / TQ;
  const int qt = n_qtiles - 1 - blockIdx.y;                     // heavy (late causal) tiles first
  const int n_hg = (p.nH + HW - 1) / HW;
  // consecutive workgroups go to the 8 XCDs in turn: re-index the (sequence, head group) items of a row so
  // that one XCD, with its own L2, gets neighbouring items and sees the K/V of as few sequences as possible
  int item = blockIdx.x;
  if (gridDim.x % 8 == 0) item = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
  const int b = item / n_hg;
  const int head_raw = (item % n_hg) * HW + wave % HW;
  const bool head_ok = head_raw < p.nH;
  const int head = head_ok ? head_raw : p.nH - 1;
  const int t0 = qt * TQ;
  const int tw = t0 + (wave / HW) * 32;                         // first query of this wave
  const int m = tw + lr;                                        // this lane's query, < Npad
  const long tok_base = (long)b * p.Npad;
  const long TP = (long)p.Bsz * p.Npad;

  // staging of one key tile: K rows, V rows, K^T columns
  constexpr int RCH = BC * D / CE;                              // chunks of a row tile (and of the transposed one)
  constexpr int PT = (RCH + NT - 1) / NT;
  constexpr bool FULL = RCH % NT == 0;
  constexpr int RCPR = D / CE, TCPR = BC / CE;
  const T* Kg = static_cast<const T*>(p.Kr) + tok_base * D;
  const T* Vg = static_cast<const T*>(p.Vr) + tok_base * D;
  const T* Tg = static_cast<const T*>(p.Krt) + (long)b * D * p.Npad;
  u32x4 kreg[PT], vreg[PT], treg[PT];
  auto g_load = [&](int tile) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int ci = threadIdx.x + i * NT;
      if (!FULL && ci >= RCH) break;
      const int row = ci / RCPR, cc = ci % RCPR;
      kreg[i] = *reinterpret_cast<const u32x4*>(Kg + (long)(tile * BC + row) * D + cc * CE);
      vreg[i] = *reinterpret_cast<const u32x4*>(Vg + (long)(tile * BC + row) * D + cc * CE);
      const int trow = ci / TCPR, tc = ci % TCPR;
      treg[i] = *reinterpret_cast<const u32x4*>(Tg + (long)trow * p.Npad + tile * BC + tc * CE);
    }
  };
  auto s_store = [&](int stage) {
    T* ks = smem + (long)stage * L::kStage;
    T* vs = ks + L::kKElems;
    T* ts = vs + L::kKElems;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int ci = threadIdx.x + i * NT;
      if (!FULL && ci >= RCH) break;
      const int row = ci / RCPR, cc = ci % RCPR;
      *reinterpret_cast<u32x4*>(ks + row * L::kRow + cc * CE) = kreg[i];
      *reinterpret_cast<u32x4*>(vs + row * L::kRow + cc * CE) = vreg[i];
      const int trow = ci / TCPR, tc = ci % TCPR;
      *reinterpret_cast<u32x4*>(ts + trow * L::kTRow + tc * CE) = treg[i];
    }
  };

  g_load(0);

  // ---- prologue: Q_i^T and dO_i^T of this wave's 32 tokens, delta, copies for the dK/dV kernel ----
  Frag<T> qf[CB], dof[CB];
  f32x16 negl, negd;                                            // -log-sum-exp and -delta of this lane's query
  {
    f32x16 qa[CB], da[CB];
    const T* Gt = static_cast<const T*>(p.Gt) + (long)head * D * p.R2;
    const T* Ql = static_cast<const T*>(p.Qlat) + (tok_base + m) * p.R2 + 16 * h;
    core_product<T, CB>(qa, Gt, Ql, p.R2 / 32, lane);
    if (p.rope != nullptr) rotate_blocks<CB>(qa, p.rope, p.rope_ld, p.pos0 + min(m, p.N - 1), h, 1.f);
    const T* Gtt = static_cast<const T*>(p.Gtil_t) + (long)head * D * p.RT2;
    const T* dZ = static_cast<const T*>(p.dZ) + (tok_base + m) * p.RT2 + 16 * h;
    core_product<T, CB>(da, Gtt, dZ, p.RT2 / 32, lane);
    const T* Orow = static_cast<const T*>(p.O) + ((tok_base + m) * p.nH + head) * D + 16 * h;
    float dsum = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      qf[cb] = to_frag<T>(qa[cb]);
      dof[cb] = to_frag<T>(da[cb]);
      const Frag<T> of = load_frag<T>(Orow + cb * 32);
#pragma unroll
      for (int e = 0; e < 16; ++e) dsum += frag_elem(dof[cb], e) * frag_elem(of, e);   // the rounded dO that forms dP
    }
    const float delta = halves_sum(dsum);
    const float lse = p.lse[((long)b * p.nH + head) * p.Npad + m];    // +inf for padding tokens
#pragma unroll
    for (int e = 0; e < 16; ++e) { negl[e] = -lse; negd[e] = -delta; }
    if (head_ok) {
      if (h == 0) p.delta[((long)b * p.nH + head) * p.Npad + m] = delta;
      T* Qr = static_cast<T*>(p.Qr) + ((tok_base + m) * p.nH + head) * D + 16 * h;
      T* dOr = static_cast<T*>(p.dO) + ((tok_base + m) * p.nH + head) * D + 16 * h;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        store_frag<T>(Qr + cb * 32, qf[cb]);
        store_frag<T>(dOr + cb * 32, dof[cb]);
      }
    }
  }

  // ---- key tiles ------------------------------------------------------------------------------------
  f32x16 dq[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[cb][e] = 0.f;
  const int kv_end = p.causal ? min(p.N, t0 + TQ) : p.N;
  const int n_tiles = (kv_end + BC - 1) / BC;
  const int last = n_tiles - 1;
  const int lim = p.causal ? min(m, p.N - 1) : p.N - 1;         // last key visible to this lane's query
  s_store(0);
  __syncthreads();
  for (int t = 0; t < n_tiles; ++t) {
    g_load(min(t + 1, last));
    const T* st = smem + (long)(t & 1) * L::kStage;
    const T* kbase = st + lr * L::kRow + 16 * h;
    const T* vbase = kbase + L::kKElems;
    const T* tbase = st + 2 * L::kKElems + lr * L::kTRow + 16 * h;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n0 = t * BC + nb * 32;
      if (p.causal && n0 > tw + 31) continue;                   // every key of the half follows every query
      // scores start from -log-sum-exp and dP from -delta, so the products form S - lse and dP - delta
      f32x16 s, dp;
      mma32_from(s, negl, load_frag<T>(kbase + nb * 32 * L::kRow), qf[0]);
#pragma unroll
      for (int cb = 1; cb < CB; ++cb) mma32(s, load_frag<T>(kbase + nb * 32 * L::kRow + cb * 32), qf[cb]);
      mma32_from(dp, negd, load_frag<T>(vbase + nb * 32 * L::kRow), dof[0]);
#pragma unroll
      for (int cb = 1; cb < CB; ++cb) mma32(dp, load_frag<T>(vbase + nb * 32 * L::kRow + cb * 32), dof[cb]);
      if (n0 + 31 >= p.N || (p.causal && n0 + 31 > tw)) {       // a key past the sequence or after a query
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (n0 + 8 * (e / 4) + 4 * h + (e % 4) > lim) s[e] = -INFINITY;
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = fast_exp2(s[e]) * dp[e];
      const Frag<T> dsf = to_frag<T>(s);
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) mma32(dq[cb], load_frag<T>(tbase + cb * 32 * L::kTRow + nb * 32), dsf);
    }
    s_store((t + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: remove the rotation, store -----------------------------------------------------------
  if (p.rope != nullptr) rotate_blocks<CB>(dq, p.rope, p.rope_ld, p.pos0 + min(m, p.N - 1), h, -1.f);
  if (head_ok) {
    T* dQ = static_cast<T*>(p.dQ) + ((tok_base + m) * p.nH + head) * D + 16 * h;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) store_frag<T>(dQ + cb * 32, to_frag<T>(dq[cb]));
  }
}

// ---- dK, dV ------------------------------------------------------------------------------------------
template <typename T, int D, int TQ> struct DkvLds {
  static constexpr int kStages = 3;
  static constexpr int kRow = D;                                // Q / dO rows, unpadded, chunks swizzled
  static constexpr int kRElems = TQ * kRow;
  static constexpr int kStageElems = 2 * kRElems;
  static constexpr size_t kStageBytes = kStageElems * sizeof(T) + 2ul * TQ * sizeof(float);
  // probabilities handed from the dV^T waves to the dK^T waves: [2][4 key blocks][TQ/32] fragment blocks
  static constexpr size_t kPBytes = 2ul * 4 * (TQ / 32) * kFragBlockElems * sizeof(T);
  static constexpr size_t kBytes = kStages * kStageBytes + kPBytes;
};

// Workgroup = 8 waves over 128 keys: waves w and w+4 (one SIMD) own the same 32 keys.  Wave w holds
// the keys in registers as MFMA column operands, forms the probabilities P of a (head, query block)
// pair, leaves them in LDS and accumulates dV^T += dO^T P; wave w+4 holds the values, forms dP one
// interval later, takes P from LDS, and accumulates dK^T += Q^T (P (dP - delta)).  Two resident
// waves per SIMD let one wave's exponentials overlap the other's matrix products.  The Q and dO rows
// of a pair are staged once, row-major (straight from global memory into LDS, three stages, two pairs
// ahead); the transposed operands Q^T and dO^T are read from the same
// tiles with transposing LDS loads, so their rows (the channels) come out in the stored channel
// order of Q and dO (acc order within 32-blocks), which kv_reduce undoes.
template <typename T, int D, int TQ>
__global__ __launch_bounds__(512) void bwd_dkv_kernel(BwdArgs p) {
  constexpr int CB = D / 32, QBN = TQ / 32, KT = 128, NT = 512;
  constexpr int CE = 16 / sizeof(T);
  using L = DkvLds<T, D, TQ>;
  constexpr int NS = L::kStages;
  static_assert(L::kStageBytes % 16 == 0, "stages stay 16-byte aligned");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* pbuf = reinterpret_cast<T*>(smem_raw + NS * L::kStageBytes);

  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int h = lane / 32, lr = lane % 32;
  const bool k_role = wave >= 4;                                // dK^T wave (else dV^T wave)
  const int kb = wave % 4;                                      // key block of this wave
  const int b = blockIdx.x / p.n_hg, hg = blockIdx.x % p.n_hg;
  const int key0 = blockIdx.y * KT + 32 * kb;                   // first key of this wave
  const int nk = key0 + lr;                                     // this lane's key
  const bool key_ok = nk < p.Npad;
  const long tok_base = (long)b * p.Npad;
  const long TP = (long)p.Bsz * p.Npad;

  // column operand of this wave's keys for the whole kernel: the rotated keys in a dV^T wave (it
  // forms the scores), the values in a dK^T wave (it forms dP)
  Frag<T> kop[CB];
  {
    const long row = tok_base + (key_ok ? nk : 0);
    const T* src = static_cast<const T*>(k_role ? p.Vr : p.Kr) + row * D + 16 * h;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) kop[cb] = key_ok ? load_frag<T>(src + cb * 32) : zero_frag<T>();
  }
  f32x16 acc[CB];                                               // dV^T or dK^T of this wave's keys
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[cb][e] = 0.f;

  // (head, query block) pairs of this workgroup
  const int head0 = hg * p.hpg;
  const int n_heads = min(p.hpg, p.nH - head0);
  const int qb_first = p.causal ? (blockIdx.y * KT) / TQ : 0;
  const int n_qb = p.Npad / TQ - qb_first;                      // >= 1: the grid covers Npad
  const int n_it = n_heads * n_qb;
  // Query blocks are walked from the last one down: the workgroups of one (sequence, head group),
  // which run on the same XCD at the same time, then all read the same block at the same moment
  // (with causal masking their ranges start at different blocks but all end at the last).
  auto q_of = [&](int it) { return (qb_first + n_qb - 1 - it % n_qb) * TQ; };

  // The Q and dO rows of a pair go from global memory straight into LDS (see dma_piece in common.h),
  // into the stage that the lagging dK^T waves have just left, one interval before the dV^T waves
  // need them; only the two small per-query vectors pass through a register.  That register load is
  // issued last and waited for before it is stored, and loads return in order, so the tiles of a
  // pair have landed when its vectors are stored (and the barrier that follows publishes both).
  constexpr int CPR = D / CE;                                    // chunks per row
  constexpr int PIECES = TQ * CPR / 64;                          // 1 KB pieces per tensor
  constexpr int PF = 2;                                         // pairs in flight
  float stat[PF];
  auto g_load = [&](float& st_reg, int it_raw, int stage) {
    const int it = min(it_raw, n_it - 1);                       // past the end: the last pair again, never read
    const int head = head0 + it / n_qb, q0 = q_of(it);
    const T* Qg = static_cast<const T*>(p.Qr) + ((tok_base + q0) * p.nH + head) * D;
    const T* Og = static_cast<const T*>(p.dO) + ((tok_base + q0) * p.nH + head) * D;
    T* qs = reinterpret_cast<T*>(smem_raw + (size_t)stage * L::kStageBytes);
    T* os = qs + L::kRElems;
    const long rs = (long)p.nH * D;
#pragma unroll
    for (int i = 0; i < (PIECES + 7) / 8; ++i) {
      const int q = i * 8 + wave;
      if (q < PIECES) {
        dma_piece<T, CPR>(qs, q, lane, [&](int row) { return Qg + row * rs; });
        dma_piece<T, CPR>(os, q, lane, [&](int row) { return Og + row * rs; });
      }
    }
    // threads 0..255 fetch the log-sum-exp of the block's queries, threads 256.. their delta (TQ of
    // each are kept)
    const long so = ((long)b * p.nH + head) * p.Npad + q0 + threadIdx.x % TQ;
    st_reg = (threadIdx.x < 256 ? p.lse : p.delta)[so];
  };
  auto s_store = [&](float st_reg, int stage) {
    float* st = reinterpret_cast<float*>(smem_raw + (size_t)stage * L::kStageBytes + L::kStageElems * sizeof(T));
    // stored negated: a score block starts from -log-sum-exp, a dP block from -delta
    if (threadIdx.x < TQ) st[threadIdx.x] = -st_reg;
    else if (threadIdx.x >= 256 && threadIdx.x < 256 + TQ) st[TQ + threadIdx.x - 256] = -st_reg;
  };

  g_load(stat[0], 0, 0);
  g_load(stat[1], 1, 1);
  s_store(stat[0], 0);
  __syncthreads();
  // one interval: the dV^T waves work on pair t (stage t % 3), the dK^T waves on pair t-1; then the
  // vectors of pair t+1 are stored, and after the barrier pair t+2 is fetched into stage (t+2) % 3,
  // which held pair t-1.
  auto interval = [&](auto slot_c, int t) {
    constexpr int S1 = (decltype(slot_c)::value + 1) % PF;      // slot of pair t + 1
    const int it = k_role ? t - 1 : t;                          // pair this wave works on in this interval
    if (it >= 0 && it < n_it) {
      const unsigned char* sb = smem_raw + (size_t)(it % NS) * L::kStageBytes;
      const T* qs = reinterpret_cast<const T*>(sb);
      const T* os = qs + L::kRElems;
      const float* stat = reinterpret_cast<const float*>(os + L::kRElems);
      const int q0 = q_of(it);
#pragma unroll
      for (int qb = 0; qb < QBN; ++qb) {
        const int qfirst = q0 + 32 * qb;
        // all 32 keys of the wave lie after all 32 queries of the block: nothing to do
        if (p.causal && key0 > qfirst + 31) continue;
        T* pblk = pbuf + (long)(((it & 1) * 4 + kb) * QBN + qb) * kFragBlockElems;
        // rows of the block start from -log-sum-exp (scores) or -delta (dP)
        f32x16 a;
        const float* st4 = stat + (k_role ? TQ : 0) + qb * 32 + 4 * h;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v4 = *reinterpret_cast<const f32x4*>(st4 + 8 * q);
#pragma unroll
          for (int e = 0; e < 4; ++e) a[4 * q + e] = v4[e];
        }
        const T* rows = (k_role ? os : qs) + (qb * 32 + lr) * L::kRow;
        constexpr int FC = 16 / CE;                             // chunks per fragment half
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
          mma32(a, load_frag_swz<T>(rows, cb * 2 * FC + h * FC, swz_x<CPR>(qb * 32 + lr)), kop[cb]);
        Frag<T> bf;                                             // P (dV^T wave) or dS (dK^T wave), k = queries
        if (!k_role) {
          if (key0 + 31 >= p.N || (p.causal && key0 + 31 > qfirst)) {   // a key past the sequence or after a query
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int mq = qfirst + 8 * (e / 4) + 4 * h + (e % 4);    // query of this register
              if (nk >= p.N || (p.causal && nk > mq)) a[e] = -INFINITY;
            }
          }
#pragma unroll
          for (int e = 0; e < 16; ++e) a[e] = fast_exp2(a[e]);
          bf = to_frag<T>(a);
          store_frag_major<T>(pblk, lane, bf);
        } else {
          const Frag<T> pf = load_frag_major<T>(pblk, lane);
#pragma unroll
          for (int e = 0; e < 16; ++e) a[e] *= frag_elem(pf, e);
          bf = to_frag<T>(a);
        }
        const T* tile = k_role ? qs : os;                       // dK^T += Q^T dS,  dV^T += dO^T P
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) mma32(acc[cb], load_frag_tr_swz<CPR>(tile, qb * 32, cb * 32, lane), bf);
      }
    }
    s_store(stat[S1], (t + 1) % NS);
    __syncthreads();
    if (t + 2 < n_it) g_load(stat[decltype(slot_c)::value], t + 2, (t + 2) % NS);   // nothing is left in flight at the end
  };
  const int n_int = n_it + 1;
  int t = 0;
  for (; t + PF <= n_int; t += PF) {
    interval(std::integral_constant<int, 0>{}, t);
    interval(std::integral_constant<int, 1>{}, t + 1);
  }
  if (t < n_int) interval(std::integral_constant<int, 0>{}, t);

  // rows of the accumulators are stored channel positions: position 16h'+4q'+r of a 32-block
  if (key_ok) {
    float* dst = (k_role ? p.dKp : p.dVp) + ((long)hg * TP + tok_base + nk) * D + 4 * h;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        store4(dst + cb * 32 + 8 * q, acc[cb][4 * q], acc[cb][4 * q + 1], acc[cb][4 * q + 2], acc[cb][4 * q + 3]);
  }
}

// ---- sum of the head-group partials, rotation removed from the key part -----------------------------
// The scores carry a factor log2(e) (the per-head query is pre-scaled so that the softmax runs on
// exp2), so the key gradient formed from those queries is multiplied by ln 2 here.
template <typename T>
__global__ __launch_bounds__(256) void kv_reduce_kernel(KvReduceArgs a) {
  const long TP = (long)a.Bsz * a.Npad;
  const int quads = a.D / 4;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= TP * quads) return;
  const long tp = idx / quads;
  const int k = (int)(idx % quads);
  const int n = (int)(tp % a.Npad);
  f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
  // the partials hold channel quad k at its stored (acc-order) position inside its 32-block
  const int c32 = (4 * k) % 32;
  const int spos = (4 * k) / 32 * 32 + 16 * ((c32 / 4) % 2) + 4 * (c32 / 8);
  for (int g = 0; g < a.n_hg; ++g) {
    const long off = ((long)g * TP + tp) * a.D + spos;
    const f32x4 x = *reinterpret_cast<const f32x4*>(a.dKp + off);
    const f32x4 y = *reinterpret_cast<const f32x4*>(a.dVp + off);
#pragma unroll
    for (int e = 0; e < 4; ++e) { sk[e] += x[e]; sv[e] += y[e]; }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) sk[e] *= kLn2;
  if (a.rope != nullptr && n < a.N) {
    const f32x4 cs = reinterpret_cast<const f32x4*>(a.rope)[(long)k * a.rope_ld + a.pos0 + n];
#pragma unroll
    for (int e = 0; e < 4; e += 2) {
      const float x0 = sk[e], x1 = sk[e + 1];
      sk[e] = x0 * cs[e] + x1 * cs[e + 1];
      sk[e + 1] = -x0 * cs[e + 1] + x1 * cs[e];
    }
  }
  T* row = static_cast<T*>(a.dLat) + tp * a.ld;
  if (a.shared_kv) {
    store4(row + a.colK + 4 * k, sk[0] + sv[0], sk[1] + sv[1], sk[2] + sv[2], sk[3] + sv[3]);
  } else {
    store4(row + a.colK + 4 * k, sk[0], sk[1], sk[2], sk[3]);
    store4(row + a.colV + 4 * k, sv[0], sv[1], sv[2], sv[3]);
  }
}

// ---- launchers ---------------------------------------------------------------------------------------
template <typename T, int D, int BC>
static hipError_t dq_one(const BwdArgs& a, hipStream_t s) {
  dim3 grid(((a.nH + 3) / 4) * a.Bsz, a.Npad / 64);
  const size_t smem = DqLds<T, D, BC>::kBytes;
  auto kern = bwd_dq_kernel<T, D, BC>;
  static LdsOnce lds_once;
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  hipLaunchKernelGGL(kern, grid, dim3(512), smem, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dq(int dtype, const BwdArgs& a, hipStream_t s) {
  if (dtype == 0) {
    switch (a.D) {
      case 32: return dq_one<float, 32, 32>(a, s);
      case 64: return dq_one<float, 64, 32>(a, s);
      case 128: return dq_one<float, 128, 32>(a, s);
    }
  } else {
    switch (a.D) {
      case 32: return dq_one<bf16, 32, 64>(a, s);
      case 64: return dq_one<bf16, 64, 64>(a, s);
      case 128: return dq_one<bf16, 128, 64>(a, s);
    }
  }
  return hipErrorInvalidValue;
}

template <typename T, int D, int TQ>
static hipError_t dkv_one(const BwdArgs& a, hipStream_t s) {
  dim3 grid(a.n_hg * a.Bsz, (a.Npad + 127) / 128);
  const size_t smem = DkvLds<T, D, TQ>::kBytes;
  static_assert(DkvLds<T, D, TQ>::kBytes <= 160 * 1024, "fits the LDS of a compute unit");
  auto kern = bwd_dkv_kernel<T, D, TQ>;
  static LdsOnce lds_once;
  if (hipError_t ae = allow_dynamic_lds(lds_once, kern, smem); ae != hipSuccess) return ae;
  hipLaunchKernelGGL(kern, grid, dim3(512), smem, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dkv(int dtype, const BwdArgs& a, hipStream_t s) {
  if (dtype == 0) {
    switch (a.D) {
      case 32: return dkv_one<float, 32, 32>(a, s);
      case 64: return dkv_one<float, 64, 32>(a, s);
      case 128: return dkv_one<float, 128, 32>(a, s);
    }
  } else {
    switch (a.D) {
      case 32: return dkv_one<bf16, 32, 64>(a, s);
      case 64: return dkv_one<bf16, 64, 64>(a, s);
      case 128: return dkv_one<bf16, 128, 64>(a, s);
    }
  }
  return hipErrorInvalidValue;
}

hipError_t launch_kv_reduce(int dtype, const KvReduceArgs& a, hipStream_t s) {
  const long total = (long)a.Bsz * a.Npad * (a.D / 4);
  const int blocks = (int)((total + 255) / 256);
  if (dtype == 0)
    hipLaunchKernelGGL(kv_reduce_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(kv_reduce_kernel<bf16>, dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ta
