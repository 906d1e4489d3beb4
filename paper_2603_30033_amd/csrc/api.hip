// Host side of the C ABI: argument validation, workspace carving and kernel sequencing.
// Nothing here computes on the CPU except the rotation table built once in create.
#include "../../include/tucker_attn.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "common.h"
#include "params.h"

using namespace ta;

namespace {
constexpr int kMaxKernels = 40;
constexpr size_t kAlign = 256;
// Token tiles (32 padded tokens at the smallest) are the y dimension of the GEMM launches, which HIP
// limits to 65535: more padded tokens than this are refused before anything is enqueued.
constexpr long kMaxTokens = 65535l * 32;
constexpr int kDecodeChunk = 32;      // sequences per pass of the decode kernels (their per-sequence arguments)
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
}  // namespace

// Workspace of tucker_attn_decode_static: device memory that belongs to the loaded library, one copy on
// every GPU the library runs on, held until the process ends.  In host code the name is only a handle
// for hipGetSymbolAddress; the address kernels and copies use is the one static_scratch() returns.
constexpr size_t kStaticScratchBytes = 32ul << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct tucker_attn_ctx {
  tucker_attn_config cfg;
  int R2, RT2, D, dp;          // padded ranks, common K/V width, padded d
  int es;                      // bytes per stored element
  float4* rope;                // device [D/4][max_positions] (cos, sin, cos, sin) or null
  float qscale;                // log2(e) / sqrt(d_head), folded into the head-mixed core
  int n_cus;                   // compute units of the device current at create (256 if none could be asked)
  int profile;
  int n_kernels;
  const char* names[kMaxKernels];
  hipEvent_t ev[kMaxKernels + 1];
  hipEvent_t kev[2];           // start and end of the dominant kernel itself (attached to its dispatch)
  const char* kev_name;        // null until such a launch has been made with profiling on
  bool ev_created;
  // prepared weights (tucker_attn_prepare_weights): caller-owned buffer in the layout of
  // carve_weights, and the weight pointers it was made from
  void* prepared;
  tucker_attn_weights prepared_from;
};

namespace {

// Device address of `scratch` on the current device, looked up once per device.
hipError_t static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> ptrs[kMaxDevices];
  *out = nullptr;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = ptrs[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    ptrs[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return hipSuccess;
}

struct Carver {
  char* base;
  size_t off;
  template <typename P> P* take(size_t bytes) {
    P* p = reinterpret_cast<P*>(base + off);
    off += align_up(bytes);
    return p;
  }
};

struct PrefillWs {
  void *Gt, *Gtil2, *Wcat, *Ut2p, *Qlat, *Kr, *Vt, *O, *Z;
  size_t bytes;
};
struct DecodeWs {
  void *Gt, *Gtil2, *Wcat, *Ut2p, *Qlat, *Qh;
  float *pm, *pl, *po, *part;
  size_t bytes;
};

void carve_weights(const tucker_attn_ctx* c, Carver& cv, void*& Gt, void*& Gtil2, void*& Wcat, void*& Ut2p) {
  const tucker_attn_config& f = c->cfg;
  Gt = cv.take<char>((size_t)f.n_heads * c->D * c->R2 * c->es);
  Gtil2 = cv.take<char>((size_t)c->RT2 * f.n_heads * c->D * c->es);
  Wcat = cv.take<char>((size_t)(c->R2 + 2 * c->D) * c->dp * c->es);
  Ut2p = cv.take<char>((size_t)c->dp * c->RT2 * c->es);
}

size_t prepared_bytes(const tucker_attn_ctx* c) {
  Carver cv{nullptr, 0};
  void *a, *b, *d, *e;
  carve_weights(c, cv, a, b, d, e);
  return cv.off;
}

// The operand-layout copies of the weights: a piece of the call's workspace, or the caller's
// prepared buffer when one is registered (then no preparation kernel runs).
template <typename W> void use_prepared(const tucker_attn_ctx* c, W& w) {
  if (!c->prepared) return;
  Carver cv{static_cast<char*>(c->prepared), 0};
  carve_weights(c, cv, w.Gt, w.Gtil2, w.Wcat, w.Ut2p);
}

bool same_weights(const tucker_attn_weights& a, const tucker_attn_weights& b) {
  return a.C == b.C && a.U1 == b.U1 && a.U2 == b.U2 && a.U3 == b.U3 && a.Ct == b.Ct && a.Ut1 == b.Ut1 &&
         a.Ut2 == b.Ut2 && a.Ut3 == b.Ut3;
}

PrefillWs carve_prefill(const tucker_attn_ctx* c, void* ws, int B, int N) {
  const tucker_attn_config& f = c->cfg;
  const size_t Npad = pad64(N), TP = (size_t)B * Npad;
  Carver cv{static_cast<char*>(ws), 0};
  PrefillWs w;
  carve_weights(c, cv, w.Gt, w.Gtil2, w.Wcat, w.Ut2p);
  w.Qlat = cv.take<char>(TP * c->R2 * c->es);
  w.Kr = cv.take<char>(TP * c->D * c->es);
  w.Vt = cv.take<char>((size_t)B * c->D * Npad * c->es);
  w.O = cv.take<char>(TP * f.n_heads * c->D * c->es);
  w.Z = cv.take<char>(TP * c->RT2 * c->es);
  w.bytes = cv.off;
  return w;
}

struct BackwardWs {
  PrefillWs f;
  float *lse, *delta, *dKp, *dVp, *dG, *dGt, *part;
  void *Vr, *Krt, *Ut2T, *Gtil_t, *G2, *Wb, *dZ, *Qr, *dO, *dQ, *dLat;
  int LW;            // width of the latent-gradient rows: R2 + D (shared latent) or R2 + 2 D
  int hpg, n_hg;     // heads per group / number of groups of the key-value gradient kernel
  int ks_w, ks_u, ks_g;   // contraction splits of the weight-gradient products
  size_t bytes;
};

// contraction split of a token-contracted product with `tiles` output tiles and K tokens
int grad_ksplit(long tiles, long K) {
  long want = (512 + tiles - 1) / tiles;
  const long nk = (K + 63) / 64;
  if (want > 16) want = 16;
  if (want > nk) want = nk;
  return want < 1 ? 1 : (int)want;
}

BackwardWs carve_backward(const tucker_attn_ctx* c, void* ws, int B, int N) {
  const tucker_attn_config& f = c->cfg;
  const size_t Npad = pad64(N), TP = (size_t)B * Npad, es = c->es;
  const size_t nHD = (size_t)f.n_heads * c->D;
  BackwardWs w;
  w.f = carve_prefill(c, ws, B, N);
  Carver cv{static_cast<char*>(ws), w.f.bytes};
  w.LW = c->R2 + (f.shared_kv ? 1 : 2) * c->D;
  const long ktiles = (long)((Npad + 127) / 128) * B;
  int n_hg = (int)((1024 + ktiles - 1) / ktiles);
  if (n_hg > f.n_heads) n_hg = f.n_heads;
  if (n_hg < 1) n_hg = 1;
  w.hpg = (f.n_heads + n_hg - 1) / n_hg;
  w.n_hg = (f.n_heads + w.hpg - 1) / w.hpg;
  w.lse = cv.take<float>((size_t)B * f.n_heads * Npad * 4);
  w.delta = cv.take<float>((size_t)B * f.n_heads * Npad * 4);
  w.Vr = cv.take<char>(TP * c->D * es);
  w.Krt = cv.take<char>(TP * c->D * es);
  w.Ut2T = cv.take<char>((size_t)c->RT2 * c->dp * es);
  w.Gtil_t = cv.take<char>(nHD * c->RT2 * es);
  w.G2 = cv.take<char>((size_t)c->R2 * nHD * es);
  w.Wb = cv.take<char>((size_t)c->dp * w.LW * es);
  w.dZ = cv.take<char>(TP * c->RT2 * es);
  w.Qr = cv.take<char>(TP * nHD * es);
  w.dO = cv.take<char>(TP * nHD * es);
  w.dQ = cv.take<char>(TP * nHD * es);
  w.dKp = cv.take<float>((size_t)w.n_hg * TP * c->D * 4);
  w.dVp = cv.take<float>((size_t)w.n_hg * TP * c->D * 4);
  w.dLat = cv.take<char>(TP * w.LW * es);
  w.dG = cv.take<float>((size_t)c->R2 * nHD * 4);
  w.dGt = cv.take<float>((size_t)c->RT2 * nHD * 4);
  const long mt = (f.d_model + 127) / 128;
  auto col_tiles = [&](long cols) { return f.dtype == TUCKER_ATTN_BF16 && cols % 128 == 0 ? cols / 128 : (cols + 63) / 64; };
  w.ks_w = grad_ksplit(mt * col_tiles(w.LW), (long)TP);
  w.ks_u = grad_ksplit(mt * col_tiles(c->RT2), (long)TP);
  const int rmax = c->R2 > c->RT2 ? c->R2 : c->RT2;
  w.ks_g = grad_ksplit(((rmax + 127) / 128) * col_tiles((long)nHD), (long)TP);
  size_t part = (size_t)w.ks_w * w.LW * pad32(f.d_model);
  const size_t p2 = (size_t)w.ks_u * c->RT2 * pad32(f.d_model), p3 = (size_t)w.ks_g * nHD * rmax;
  if (p2 > part) part = p2;
  if (p3 > part) part = p3;
  w.part = cv.take<float>(part * 4);
  w.bytes = cv.off;
  return w;
}

// Workgroups per sequence of the split-KV decode attention.  Measured at 16 sequences x 32768 cached tokens on a
// board of 256 compute units: 256 workgroups in all (one per compute unit) 54 us, 512: 57 us, 128: 90 us, counts
// that are no multiple of the number of compute units (192, 320, 384): 64-79 us.  So one round over the compute
// units, and never more splits than the longest cache has 64-key tiles.  The shared-latent variant of that kernel
// rotates keys as it stages them and is bound by that arithmetic, not by HBM: it runs two rounds (52 us against 68
// with one); the wave-private shared-latent kernel holds one workgroup per compute unit and takes 128 keys at a
// time.  At most 256 splits (a single sequence on 256 compute units): the merge spreads a sequence's splits over
// thread groups, 16 at a time each.
int decode_nsplit(const tucker_attn_ctx* c, int B, int longest) {
  const tucker_attn_config& f = c->cfg;
  const bool wave_private = decode_wave_private(f.dtype, f.r3, c->D, f.shared_kv);
  int n = (f.shared_kv && !wave_private ? 2 : 1) * c->n_cus / B;
  const int step = wave_private ? kDecodeRoundWave : kDecodeTile;  // keys a workgroup takes at a time
  const long tiles = ((long)longest + step - 1) / step;
  if (n > 256) n = 256;
  if (n > tiles) n = (int)tiles;
  return n < 1 ? 1 : n;
}
int decode_ksplit(int K) {
  int nk = (K + 63) / 64;
  return nk < 16 ? (nk < 1 ? 1 : nk) : 16;
}
// the decode projection can read the factor matrices as they lie in memory when every row of them is a whole
// number of aligned 16-byte chunks
bool decode_direct_projection(const tucker_attn_ctx* c, const tucker_attn_weights* w) {
  const tucker_attn_config& f = c->cfg;
  auto chunked = [&](const void* p, int r) { return reinterpret_cast<uintptr_t>(p) % 16 == 0 && (r * c->es) % 16 == 0; };
  return chunked(w->U2, f.r2) && chunked(w->U3, f.r3) && (f.shared_kv || chunked(w->Ut3, f.rt3));
}

DecodeWs carve_decode(const tucker_attn_ctx* c, void* ws, int B) {
  const tucker_attn_config& f = c->cfg;
  const int HB32 = pad32(f.n_heads);
  const int ns = decode_nsplit(c, B, 1 << 30);                     // the most a call can use
  Carver cv{static_cast<char*>(ws), 0};
  DecodeWs w;
  carve_weights(c, cv, w.Gt, w.Gtil2, w.Wcat, w.Ut2p);
  w.Qlat = cv.take<char>((size_t)32 * c->R2 * c->es);
  w.Qh = cv.take<char>((size_t)B * HB32 * c->D * c->es);
  w.pm = cv.take<float>((size_t)B * ns * HB32 * 4);
  w.pl = cv.take<float>((size_t)B * ns * HB32 * 4);
  w.po = cv.take<float>((size_t)B * ns * HB32 * c->D * 4);
  const int ks1 = decode_ksplit(f.d_model) < 2 ? 2 : decode_ksplit(f.d_model);
  const size_t p1 = (size_t)ks1 * B * (c->R2 + 2 * c->D) * 4;
  const size_t p2 = (size_t)f.n_heads * B * c->RT2 * 4;            // one contribution to Z per head
  w.part = cv.take<float>(p1 > p2 ? p1 : p2);
  w.bytes = cv.off;
  return w;
}

void add_job(PrepArgs& pa, const void* src, const void* coef, void* out, int A, int rows, int cols, int Z,
             int rows_pad, int cols_pad, long sz, long su, int transposed, int perm, float scale, int frag = 0) {
  PrepJob& j = pa.job[pa.n_jobs++];
  j.src = src; j.coef = coef; j.out = out;
  j.A = A; j.rows = rows; j.cols = cols; j.Z = Z;
  j.rows_pad = rows_pad; j.cols_pad = cols_pad;
  j.out_stride_z = sz; j.out_stride_u = su;
  j.transposed = transposed; j.perm = perm; j.scale = scale; j.frag = frag;
  j.first_block = pa.total_blocks;
  pa.total_blocks += prep_job_blocks(j);
}

// head-mixed cores and factor matrices in MFMA operand layout; returns the output-factor pointer
PrepArgs make_prep(const tucker_attn_ctx* c, const tucker_attn_weights* w, void* Gt, void* Gtil2, void* Wcat,
                   void* Ut2p, const void** ut2_used, long* ut2_ld, bool with_wcat = true) {
  const tucker_attn_config& f = c->cfg;
  const int es = c->es;
  PrepArgs pa;
  std::memset(&pa, 0, sizeof(pa));
  const long nHD = (long)f.n_heads * c->D;
  // Gt[i][c][b] = qscale * sum_a U1[i,a] C[a,b,c], fragment-major 32x32 blocks of (c, b)
  add_job(pa, w->C, w->U1, Gt, f.r1, f.r2, f.r3, f.n_heads, c->R2, c->D, (long)c->D * c->R2, c->R2, 1, 1, c->qscale, 1);
  // Gtil2[b][i*D + c] = sum_a U~1[i,a] C~[a,b,c]
  add_job(pa, w->Ct, w->Ut1, Gtil2, f.rt1, f.rt2, f.rt3, f.n_heads, c->RT2, c->D, c->D, nHD, 0, 1, 1.f);
  // Wcat rows: U2^T | U3^T | U~3^T, each [rank_pad][dp]
  char* wc = static_cast<char*>(Wcat);
  if (with_wcat) {
    add_job(pa, w->U2, nullptr, wc, 1, f.d_model, f.r2, 1, c->dp, c->R2, 0, c->dp, 1, 0, 1.f);
    add_job(pa, w->U3, nullptr, wc + (size_t)c->R2 * c->dp * es, 1, f.d_model, f.r3, 1, c->dp, c->D, 0, c->dp, 1, 0, 1.f);
    if (!f.shared_kv)
      add_job(pa, w->Ut3, nullptr, wc + (size_t)(c->R2 + c->D) * c->dp * es, 1, f.d_model, f.rt3, 1, c->dp, c->D, 0,
              c->dp, 1, 0, 1.f);
  }
  if (f.rt2 != c->RT2) {
    add_job(pa, w->Ut2, nullptr, Ut2p, 1, f.d_model, f.rt2, 1, c->dp, c->RT2, 0, c->RT2, 0, 0, 1.f);
    *ut2_used = Ut2p;
  } else {
    *ut2_used = w->Ut2;
  }
  *ut2_ld = c->RT2;
  return pa;
}

// Token-tile width of a GEMM launch.  A 128-wide tile pays only where the contraction is long
// (operand re-reads dominate) and the grid still gives every compute unit two workgroups; short
// contractions are bound by their output stores and run best with more, smaller workgroups.
int pick_tile_n(int m_tiles, long TP, int K) {
  if (K >= 1024 && (long)m_tiles * ((TP + 127) / 128) >= 512) return 128;
  if ((long)m_tiles * ((TP + 63) / 64) >= 256) return 64;
  return 32;
}

struct Recorder {
  tucker_attn_ctx* c;
  hipStream_t s;
  bool on;
  hipError_t begin() {
    c->n_kernels = 0;
    if (!on) return hipSuccess;
    return hipEventRecord(c->ev[0], s);
  }
  hipError_t after(const char* name) {
    if (!on) return hipSuccess;
    if (c->n_kernels >= kMaxKernels) return hipSuccess;
    c->names[c->n_kernels] = name;
    ++c->n_kernels;
    return hipEventRecord(c->ev[c->n_kernels], s);
  }
};

bool weights_ok(const tucker_attn_ctx* c, const tucker_attn_weights* w) {
  return c && w && w->C && w->U1 && w->U2 && w->U3 && w->Ct && w->Ut1 && w->Ut2 && (w->Ut3 || c->cfg.shared_kv);
}

// prep, factor projection, attention and head merge of a prefill call: everything up to Z.  The
// backward pass calls it with buffers for the extra outputs it needs (value rows, transposed keys,
// log-sum-exp); the forward passes null for those.
int forward_core(tucker_attn_ctx* c, const tucker_attn_weights* w, const void* X, int B, int N, int pos0,
                 void* Kcache_out, void* Vcache_out, int Lmax, const PrefillWs& ws, void* Vr, void* Krt, float* lse,
                 hipStream_t s, Recorder& rec, const void** ut2_out, long* ut2_ld_out) {
  const tucker_attn_config& f = c->cfg;
  const int Npad = pad64(N);
  const long TP = (long)B * Npad;
  const void* ut2;
  long ut2_ld;
  PrepArgs pa = make_prep(c, w, ws.Gt, ws.Gtil2, ws.Wcat, ws.Ut2p, &ut2, &ut2_ld);
  if (!c->prepared) {
    if (launch_prep(f.dtype, pa, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("prep_weights");
  }

  GemmArgs g;
  std::memset(&g, 0, sizeof(g));
  g.A = ws.Wcat; g.lda = c->dp; g.M = c->R2 + (f.shared_kv ? 1 : 2) * c->D; g.shared_kv = f.shared_kv;
  g.Bsrc = X; g.ldb = f.d_model; g.K = f.d_model;
  g.Bsz = B; g.N = N; g.Npad = Npad; g.src_padded = 0;
  g.epi = 0;
  g.Qlat = ws.Qlat; g.R2 = c->R2; g.Kr = ws.Kr; g.D = c->D; g.Vt = ws.Vt; g.Vr = Vr; g.Krt = Krt;
  g.Kcache = Kcache_out; g.Vcache = Vcache_out; g.Lmax = Lmax; g.r3 = f.r3; g.rt3 = f.rt3;
  g.rope = c->rope; g.rope_ld = f.max_positions; g.pos0 = pos0; g.decode = 0; g.ksplit = 1;
  if (launch_gemm(f.dtype, g, pick_tile_n((g.M + 127) / 128, TP, g.K), s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  rec.after("factor_projection");

  AttnArgs a;
  std::memset(&a, 0, sizeof(a));
  a.Qlat = ws.Qlat; a.Gt = ws.Gt; a.Kr = ws.Kr; a.Vt = ws.Vt; a.O = ws.O; a.lse = lse;
  a.rope = c->rope; a.rope_ld = f.max_positions;
  a.Bsz = B; a.N = N; a.Npad = Npad; a.nH = f.n_heads; a.R2 = c->R2; a.r3 = f.r3; a.D = c->D;
  a.causal = f.causal; a.pos0 = pos0;
  if (launch_attn_prefill(f.dtype, a, s, rec.on ? c->kev[0] : nullptr, rec.on ? c->kev[1] : nullptr) != hipSuccess)
    return TUCKER_ATTN_HIP_ERROR;
  if (rec.on) c->kev_name = "attention_kernel";
  rec.after("attention");

  GemmArgs z;
  std::memset(&z, 0, sizeof(z));
  z.A = ws.Gtil2; z.lda = (long)f.n_heads * c->D; z.M = c->RT2;
  z.Bsrc = ws.O; z.ldb = (long)f.n_heads * c->D; z.K = f.n_heads * c->D;
  z.Bsz = B; z.N = N; z.Npad = Npad; z.src_padded = 1;
  z.epi = 1; z.Out = ws.Z; z.ldo = c->RT2; z.ksplit = 1; z.R2 = 0; z.D = 0;
  if (launch_gemm(f.dtype, z, pick_tile_n((z.M + 127) / 128, TP, z.K), s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  rec.after("latent_merge");
  *ut2_out = ut2;
  *ut2_ld_out = ut2_ld;
  return TUCKER_ATTN_OK;
}

// One decode step of B sequences inside `workspace`.  The kernels take their per-sequence arguments
// (cache length, position) by value for at most kDecodeChunk sequences, so a larger batch runs as
// consecutive passes over chunks of sequences on the same stream, sharing the workspace; the weight
// preparation runs once.
int decode_impl(tucker_attn_ctx* c, const tucker_attn_weights* w, const void* x, void* y, void* Kcache, void* Vcache,
                int32_t Lmax, const int32_t* kv_len, int32_t B, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
  if (!c || !weights_ok(c, w) || !x || !y || !Kcache || !kv_len || !workspace) return TUCKER_ATTN_INVALID_ARG;
  if (B < 1 || Lmax < 1) return TUCKER_ATTN_INVALID_ARG;
  const tucker_attn_config& f = c->cfg;
  if (f.shared_kv ? Vcache != nullptr : Vcache == nullptr) return TUCKER_ATTN_INVALID_ARG;
  const long row_bytes = (long)(f.r3 > f.rt3 ? f.r3 : f.rt3) * c->es;
  for (int b = 0; b < B; ++b) {
    if (kv_len[b] < 1 || kv_len[b] > Lmax) return TUCKER_ATTN_INVALID_ARG;
    if (f.use_rope && kv_len[b] > f.max_positions) return TUCKER_ATTN_INVALID_ARG;
    // the cache of one sequence is addressed through 32-bit byte offsets of a buffer descriptor
    if ((long)kv_len[b] * row_bytes >= (1l << 31)) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  }
  if (f.n_heads > 64) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if ((f.r3 * c->es) % 16 != 0 || (f.rt3 * c->es) % 16 != 0) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return TUCKER_ATTN_INVALID_ARG;
  if (c->prepared && !same_weights(*w, c->prepared_from)) return TUCKER_ATTN_INVALID_ARG;
  const int Bc_max = B < kDecodeChunk ? B : kDecodeChunk;
  if (workspace_bytes < carve_decode(c, nullptr, Bc_max).bytes) return TUCKER_ATTN_WORKSPACE_TOO_SMALL;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Recorder rec{c, s, c->profile != 0};
  if (rec.begin() != hipSuccess) return TUCKER_ATTN_HIP_ERROR;

  for (int b0 = 0; b0 < B; b0 += kDecodeChunk) {
    const int Bc = B - b0 < kDecodeChunk ? B - b0 : kDecodeChunk;
    DecodeWs ws = carve_decode(c, workspace, Bc);                  // the weight copies come first: same place in every pass
    use_prepared(c, ws);
    const char* xb = static_cast<const char*>(x) + (size_t)b0 * f.d_model * c->es;
    char* yb = static_cast<char*>(y) + (size_t)b0 * f.d_model * c->es;
    char* Kb = static_cast<char*>(Kcache) + (size_t)b0 * Lmax * f.r3 * c->es;
    char* Vb = Vcache ? static_cast<char*>(Vcache) + (size_t)b0 * Lmax * f.rt3 * c->es : nullptr;
    const int32_t* len = kv_len + b0;
    int longest = 1;
    for (int b = 0; b < Bc; ++b) longest = len[b] > longest ? len[b] : longest;

    // Factor matrices whose rows are whole 16-byte chunks are multiplied as they lie in memory, in a launch that
    // also carries the weight-preparation tiles; other shapes go through transposed copies and the product kernel.
    const bool direct = decode_direct_projection(c, w);
    const void* ut2;
    long ut2_ld;
    PrepArgs pa = make_prep(c, w, ws.Gt, ws.Gtil2, ws.Wcat, ws.Ut2p, &ut2, &ut2_ld, !direct);
    const bool prepare_now = !c->prepared && b0 == 0;
    if (prepare_now && !direct) {
      if (launch_prep(f.dtype, pa, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
      rec.after("prep_weights");
    }

    GemmArgs g;                                                   // the projection's epilogue and partial-tile layout
    std::memset(&g, 0, sizeof(g));
    g.A = ws.Wcat; g.lda = c->dp; g.M = c->R2 + (f.shared_kv ? 1 : 2) * c->D; g.shared_kv = f.shared_kv;
    g.Bsrc = xb; g.ldb = f.d_model; g.K = f.d_model;
    g.Bsz = Bc; g.N = 1; g.Npad = 1; g.src_padded = 0;
    g.epi = 0;
    g.Qlat = ws.Qlat; g.R2 = c->R2; g.Kr = nullptr; g.D = c->D; g.Vt = nullptr;
    g.Kcache = Kb; g.Vcache = Vb; g.Lmax = Lmax; g.r3 = f.r3; g.rt3 = f.rt3;
    g.rope = c->rope; g.rope_ld = f.max_positions; g.pos0 = 0; g.decode = 1;
    for (int b = 0; b < Bc; ++b) g.kv_pos[b] = len[b] - 1;
    g.ksplit = decode_ksplit(g.K); g.part = ws.part;
    g.defer_reduce = 1;                                           // the query launch sums the partial tiles
    if (direct) {
      if (g.ksplit < 2) g.ksplit = 2;                             // always partial tiles on this path
      DecodeProjArgs dp;
      std::memset(&dp, 0, sizeof(dp));
      dp.X = xb; dp.U2 = w->U2; dp.U3 = w->U3; dp.Ut3 = w->Ut3;
      dp.r2 = f.r2; dp.r3 = f.r3; dp.rt3 = f.rt3; dp.R2 = c->R2; dp.D = c->D;
      dp.K = f.d_model; dp.Bsz = Bc; dp.ksplit = g.ksplit; dp.shared_kv = f.shared_kv; dp.part = ws.part;
      PrepArgs none;
      std::memset(&none, 0, sizeof(none));
      if (launch_decode_proj(f.dtype, dp, prepare_now ? pa : none, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    } else {
      if (launch_gemm(f.dtype, g, 32, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    }
    rec.after("factor_projection");

    DecodeArgs d;
    std::memset(&d, 0, sizeof(d));
    d.Qlat = ws.Qlat; d.Gt = ws.Gt; d.Qh = ws.Qh; d.Kcache = Kb; d.Vcache = Vb;
    d.part_m = ws.pm; d.part_l = ws.pl; d.part_o = ws.po; d.rope = c->rope; d.rope_ld = f.max_positions;
    d.Bsz = Bc; d.nH = f.n_heads; d.HB = pad32(f.n_heads) / 32; d.R2 = c->R2; d.r3 = f.r3; d.rt3 = f.rt3;
    d.D = c->D; d.Lmax = Lmax; d.nsplit = decode_nsplit(c, Bc, longest); d.shared_kv = f.shared_kv;
    for (int b = 0; b < Bc; ++b) d.kv_len[b] = len[b];
    if (launch_decode_qhat(f.dtype, d, g, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("decode_query");
    if (launch_decode_attn(f.dtype, d, s, rec.on ? c->kev[0] : nullptr, rec.on ? c->kev[1] : nullptr) != hipSuccess)
      return TUCKER_ATTN_HIP_ERROR;
    if (rec.on) c->kev_name = "decode_attention_kernel";
    rec.after("decode_attention");
    // merge of the split partials and the head merge: one workgroup per head writes its contribution to Z
    d.Gtil2 = ws.Gtil2; d.zpart = ws.part; d.RT2 = c->RT2;
    if (launch_decode_merge_heads(f.dtype, d, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("decode_merge");
    // the output projection sums the heads' contributions itself
    d.Ut2 = ut2; d.ut2_ld = ut2_ld; d.Y = yb; d.d_model = f.d_model;
    if (launch_decode_out(f.dtype, d, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("output_projection");
  }
  return TUCKER_ATTN_OK;
}

}  // namespace

extern "C" {

int tucker_attn_create(const tucker_attn_config* cfg, tucker_attn_ctx** out) {
  if (!cfg || !out) return TUCKER_ATTN_INVALID_ARG;
  *out = nullptr;
  const tucker_attn_config& f = *cfg;
  if (f.d_model < 1 || f.n_heads < 1 || f.d_head < 1 || f.r1 < 1 || f.r2 < 1 || f.r3 < 1 || f.rt1 < 1 ||
      f.rt2 < 1 || f.rt3 < 1 || f.max_positions < 1)
    return TUCKER_ATTN_INVALID_ARG;
  if (f.dtype != TUCKER_ATTN_F32 && f.dtype != TUCKER_ATTN_BF16) return TUCKER_ATTN_INVALID_ARG;
  if ((f.causal != 0 && f.causal != 1) || (f.use_rope != 0 && f.use_rope != 1)) return TUCKER_ATTN_INVALID_ARG;
  if (f.shared_kv != 0 && f.shared_kv != 1) return TUCKER_ATTN_INVALID_ARG;
  if (f.save_for_backward != 0 && f.save_for_backward != 1) return TUCKER_ATTN_INVALID_ARG;
  if (f.shared_kv && f.rt3 != f.r3) return TUCKER_ATTN_INVALID_ARG;
  if (f.use_rope && !(f.rope_base > 0.f)) return TUCKER_ATTN_INVALID_ARG;
  if (f.r3 > 128 || f.rt3 > 128 || f.r2 > 512 || f.rt2 > 512 || f.r1 > 64 || f.rt1 > 64)
    return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if (f.d_model % 8 != 0) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if (f.use_rope && (f.r3 % 2) != 0) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if ((long)f.max_positions * f.r3 > (1l << 31)) return TUCKER_ATTN_UNSUPPORTED_SHAPE;

  tucker_attn_ctx* c = new (std::nothrow) tucker_attn_ctx;
  if (!c) return TUCKER_ATTN_HIP_ERROR;
  std::memset(c, 0, sizeof(*c));
  c->cfg = f;
  c->R2 = pad32(f.r2);
  c->RT2 = pad32(f.rt2);
  const int dk = pad32(f.r3), dv = pad32(f.rt3);
  int D = dk > dv ? dk : dv;
  if (D == 96) D = 128;
  c->D = D;
  c->dp = pad32(f.d_model);
  c->es = f.dtype == TUCKER_ATTN_F32 ? 4 : 2;
  c->qscale = (float)(1.4426950408889634 / std::sqrt((double)f.d_head));
  c->n_cus = 256;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      c->n_cus = cus;
    else
      (void)hipGetLastError();
  }
  c->rope = nullptr;
  if (f.use_rope) {
    // angle = position * base^(-2j/r3), evaluated in double precision, stored as fp32.  Entry
    // [k][p] holds (cos, sin) of pairs 2k and 2k+1 at position p; pairs beyond r3/2 belong to
    // padding channels and are the identity rotation, so the kernels never look at r3.
    const int half = f.r3 / 2, quads = D / 4;
    std::vector<float4> tab((size_t)quads * f.max_positions, make_float4(1.f, 0.f, 1.f, 0.f));
    for (int j = 0; j < half; ++j) {
      const double theta = std::pow((double)f.rope_base, -2.0 * j / (double)f.r3);
      for (int p = 0; p < f.max_positions; ++p) {
        const double a = (double)p * theta;
        float4& e = tab[(size_t)(j / 2) * f.max_positions + p];
        if (j % 2 == 0) { e.x = (float)std::cos(a); e.y = (float)std::sin(a); }
        else { e.z = (float)std::cos(a); e.w = (float)std::sin(a); }
      }
    }
    if (hipMalloc(&c->rope, tab.size() * sizeof(float4)) != hipSuccess) {
      delete c;
      return TUCKER_ATTN_HIP_ERROR;
    }
    if (hipMemcpy(c->rope, tab.data(), tab.size() * sizeof(float4), hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipFree(c->rope);
      delete c;
      return TUCKER_ATTN_HIP_ERROR;
    }
  }
  if (f.use_rope) {                                             // a device is current (the table was just copied to it):
    void* unused;                                               // look up this device's static scratch now rather than
    (void)static_scratch(&unused);                              // on the first tucker_attn_decode_static call
  }
  *out = c;
  return TUCKER_ATTN_OK;
}

void tucker_attn_destroy(tucker_attn_ctx* c) {
  if (!c) return;
  if (c->rope) (void)hipFree(c->rope);
  if (c->ev_created)
  {
    for (int i = 0; i <= kMaxKernels; ++i) (void)hipEventDestroy(c->ev[i]);
    for (int i = 0; i < 2; ++i) (void)hipEventDestroy(c->kev[i]);
  }
  delete c;
}

size_t tucker_attn_parameter_count(const tucker_attn_config* f) {
  if (!f) return 0;
  const size_t d = f->d_model, nH = f->n_heads;
  const size_t pre = nH * f->r1 + d * ((size_t)f->r2 + f->r3) + (size_t)f->r1 * f->r2 * f->r3;
  const size_t post = nH * f->rt1 + d * ((size_t)f->rt2 + (f->shared_kv ? 0 : f->rt3)) + (size_t)f->rt1 * f->rt2 * f->rt3;
  return pre + post;
}

size_t tucker_attn_cache_bytes(const tucker_attn_ctx* c, int32_t B, int32_t Lmax) {
  if (!c || B < 1 || Lmax < 1) return 0;
  const tucker_attn_config& f = c->cfg;
  return (size_t)B * Lmax * ((size_t)f.r3 + (f.shared_kv ? 0 : f.rt3)) * c->es;
}

size_t tucker_attn_workspace_bytes(const tucker_attn_ctx* c, int32_t B, int32_t N) {
  if (!c || B < 1 || N < 1) return 0;
  if (c->cfg.save_for_backward) return carve_backward(c, nullptr, B, N).bytes;
  return carve_prefill(c, nullptr, B, N).bytes;
}

size_t tucker_attn_decode_workspace_bytes(const tucker_attn_ctx* c, int32_t B) {
  if (!c || B < 1) return 0;
  return carve_decode(c, nullptr, B < kDecodeChunk ? B : kDecodeChunk).bytes;
}

int tucker_attn_forward(tucker_attn_ctx* c, const tucker_attn_weights* w, const void* X, void* Y, int32_t B,
                        int32_t N, int32_t pos0, void* Kcache_out, void* Vcache_out, int32_t Lmax, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  if (!c || !weights_ok(c, w) || !X || !Y || !workspace) return TUCKER_ATTN_INVALID_ARG;
  if (B < 1 || N < 1 || pos0 < 0) return TUCKER_ATTN_INVALID_ARG;
  const tucker_attn_config& f = c->cfg;
  if (f.shared_kv ? Vcache_out != nullptr : (Kcache_out == nullptr) != (Vcache_out == nullptr))
    return TUCKER_ATTN_INVALID_ARG;
  if (Kcache_out && (Lmax < 1 || (long)pos0 + N > Lmax)) return TUCKER_ATTN_INVALID_ARG;
  if (f.use_rope && (long)pos0 + N > f.max_positions) return TUCKER_ATTN_INVALID_ARG;
  if ((long)B * pad64(N) > kMaxTokens || B > 65535) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return TUCKER_ATTN_INVALID_ARG;
  if (c->prepared && !same_weights(*w, c->prepared_from)) return TUCKER_ATTN_INVALID_ARG;
  PrefillWs ws = carve_prefill(c, workspace, B, N);
  use_prepared(c, ws);
  void *Vr = nullptr, *Krt = nullptr;
  float* lse = nullptr;
  size_t need = ws.bytes;
  if (f.save_for_backward) {                                    // the backward layout, of which ws is the head
    const BackwardWs bw = carve_backward(c, workspace, B, N);
    Vr = bw.Vr; Krt = bw.Krt; lse = bw.lse; need = bw.bytes;
  }
  if (workspace_bytes < need) return TUCKER_ATTN_WORKSPACE_TOO_SMALL;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int Npad = pad64(N);
  const long TP = (long)B * Npad;
  Recorder rec{c, s, c->profile != 0};
  if (rec.begin() != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  const void* ut2;
  long ut2_ld;
  if (int st = forward_core(c, w, X, B, N, pos0, Kcache_out, Vcache_out, Lmax, ws, Vr, Krt, lse, s, rec,
                            &ut2, &ut2_ld);
      st != TUCKER_ATTN_OK)
    return st;

  GemmArgs y;
  std::memset(&y, 0, sizeof(y));
  y.A = ut2; y.lda = ut2_ld; y.M = f.d_model;
  y.Bsrc = ws.Z; y.ldb = c->RT2; y.K = c->RT2;
  y.Bsz = B; y.N = N; y.Npad = Npad; y.src_padded = 1;
  y.epi = 2; y.Out = Y; y.ldo = f.d_model; y.ksplit = 1;
  const hipError_t ye = out_proj_supported(f.dtype, y) ? launch_out_proj(f.dtype, y, s)
                                                       : launch_gemm(f.dtype, y, pick_tile_n((y.M + 127) / 128, TP, y.K), s);
  if (ye != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  rec.after("output_projection");
  return TUCKER_ATTN_OK;
}

size_t tucker_attn_backward_workspace_bytes(const tucker_attn_ctx* c, int32_t B, int32_t N) {
  if (!c || B < 1 || N < 1) return 0;
  return carve_backward(c, nullptr, B, N).bytes;
}

int tucker_attn_backward(tucker_attn_ctx* c, const tucker_attn_weights* w, const void* X, const void* dY, void* dX,
                         const tucker_attn_grads* gr, int32_t B, int32_t N, int32_t pos0, int32_t forward_state,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!c || !weights_ok(c, w) || !X || !dY || !dX || !gr || !workspace) return TUCKER_ATTN_INVALID_ARG;
  const tucker_attn_config& f = c->cfg;
  if (!gr->dC || !gr->dU1 || !gr->dU2 || !gr->dU3 || !gr->dCt || !gr->dUt1 || !gr->dUt2) return TUCKER_ATTN_INVALID_ARG;
  if (f.shared_kv ? gr->dUt3 != nullptr : gr->dUt3 == nullptr) return TUCKER_ATTN_INVALID_ARG;
  if (B < 1 || N < 1 || pos0 < 0) return TUCKER_ATTN_INVALID_ARG;
  if (forward_state != 0 && forward_state != 1) return TUCKER_ATTN_INVALID_ARG;
  if (forward_state && !f.save_for_backward) return TUCKER_ATTN_INVALID_ARG;
  if (f.use_rope && (long)pos0 + N > f.max_positions) return TUCKER_ATTN_INVALID_ARG;
  if ((long)B * pad64(N) > kMaxTokens || B > 65535) return TUCKER_ATTN_UNSUPPORTED_SHAPE;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return TUCKER_ATTN_INVALID_ARG;
  if (c->prepared && !same_weights(*w, c->prepared_from)) return TUCKER_ATTN_INVALID_ARG;
  BackwardWs ws = carve_backward(c, workspace, B, N);
  use_prepared(c, ws.f);
  if (workspace_bytes < ws.bytes) return TUCKER_ATTN_WORKSPACE_TOO_SMALL;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int Npad = pad64(N);
  const long TP = (long)B * Npad;
  const int nHD = f.n_heads * c->D, LW = ws.LW, es = c->es;
  Recorder rec{c, s, c->profile != 0};
  if (rec.begin() != hipSuccess) return TUCKER_ATTN_HIP_ERROR;

  // ---- forward intermediates: Qlat, K, V (three layouts), O, log-sum-exp, Z ----------------------------
  if (!forward_state) {
    const void* ut2;
    long ut2_ld;
    if (int st = forward_core(c, w, X, B, N, pos0, nullptr, nullptr, 0, ws.f, ws.Vr, ws.Krt, ws.lse, s, rec, &ut2, &ut2_ld);
        st != TUCKER_ATTN_OK)
      return st;
  }

  // ---- weights in the layouts of the backward products ------------------------------------------------------
  {
    PrepArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    // U~2^T [RT2][dp]
    add_job(pa, w->Ut2, nullptr, ws.Ut2T, 1, f.d_model, f.rt2, 1, c->dp, c->RT2, 0, c->dp, 1, 0, 1.f);
    // G~t[i][c][b] = G~_i[b][c], fragment-major blocks of (c, b), b in natural order
    add_job(pa, w->Ct, w->Ut1, ws.Gtil_t, f.rt1, f.rt2, f.rt3, f.n_heads, c->RT2, c->D, (long)c->D * c->RT2, c->RT2, 1, 0,
            1.f, 1);
    // G2[b][i*D + c] = G_i[b][c] / sqrt(d_head), c in acc order like the stored query gradient
    add_job(pa, w->C, w->U1, ws.G2, f.r1, f.r2, f.r3, f.n_heads, c->R2, c->D, c->D, nHD, 0, 1,
            (float)(1.0 / std::sqrt((double)f.d_head)));
    // Wb[j][.] = [U2 | U3 | U~3] rows, zero padded to the latent-gradient row layout
    char* wb = static_cast<char*>(ws.Wb);
    add_job(pa, w->U2, nullptr, wb, 1, f.d_model, f.r2, 1, c->dp, c->R2, 0, LW, 0, 0, 1.f);
    add_job(pa, w->U3, nullptr, wb + (size_t)c->R2 * es, 1, f.d_model, f.r3, 1, c->dp, c->D, 0, LW, 0, 0, 1.f);
    if (!f.shared_kv)
      add_job(pa, w->Ut3, nullptr, wb + (size_t)(c->R2 + c->D) * es, 1, f.d_model, f.rt3, 1, c->dp, c->D, 0, LW, 0, 0, 1.f);
    if (launch_prep(f.dtype, pa, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("prep_weights_bwd");
  }

  // ---- dZ = dY U~2 -----------------------------------------------------------------------------------------------
  {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A = ws.Ut2T; g.lda = c->dp; g.M = c->RT2;
    g.Bsrc = dY; g.ldb = f.d_model; g.K = f.d_model;
    g.Bsz = B; g.N = N; g.Npad = Npad; g.src_padded = 0;
    g.epi = 1; g.Out = ws.dZ; g.ldo = c->RT2; g.ksplit = 1;
    if (launch_gemm(f.dtype, g, pick_tile_n((g.M + 127) / 128, TP, g.K), s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_z");
  }

  // ---- attention backward -------------------------------------------------------------------------------------
  BwdArgs a;
  std::memset(&a, 0, sizeof(a));
  a.Qlat = ws.f.Qlat; a.Gt = ws.f.Gt; a.dZ = ws.dZ; a.Gtil_t = ws.Gtil_t; a.Kr = ws.f.Kr; a.Vr = ws.Vr; a.Krt = ws.Krt;
  a.O = ws.f.O; a.lse = ws.lse; a.delta = ws.delta; a.Qr = ws.Qr; a.dO = ws.dO;
  a.dQ = ws.dQ; a.dKp = ws.dKp; a.dVp = ws.dVp; a.rope = c->rope; a.rope_ld = f.max_positions;
  a.Bsz = B; a.N = N; a.Npad = Npad; a.nH = f.n_heads; a.R2 = c->R2; a.RT2 = c->RT2; a.D = c->D;
  a.causal = f.causal; a.pos0 = pos0; a.hpg = ws.hpg; a.n_hg = ws.n_hg;
  if (launch_bwd_dq(f.dtype, a, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  rec.after("attention_bwd_dq");
  if (launch_bwd_dkv(f.dtype, a, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  rec.after("attention_bwd_dkv");
  {
    KvReduceArgs k;
    std::memset(&k, 0, sizeof(k));
    k.dKp = ws.dKp; k.dVp = ws.dVp; k.dLat = ws.dLat; k.ld = LW; k.colK = c->R2; k.colV = c->R2 + c->D;
    k.rope = c->rope; k.rope_ld = f.max_positions;
    k.Bsz = B; k.N = N; k.Npad = Npad; k.D = c->D; k.n_hg = ws.n_hg; k.pos0 = pos0; k.shared_kv = f.shared_kv;
    if (launch_kv_reduce(f.dtype, k, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_kv_latent");
  }

  // ---- dQlat = sum_i dQ_i G_i^T / sqrt(d_head), into the first R2 columns of the latent-gradient rows ---------
  {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A = ws.G2; g.lda = nHD; g.M = c->R2;
    g.Bsrc = ws.dQ; g.ldb = nHD; g.K = nHD;
    g.Bsz = B; g.N = N; g.Npad = Npad; g.src_padded = 1;
    g.epi = 1; g.Out = ws.dLat; g.ldo = LW; g.ksplit = 1;
    if (launch_gemm(f.dtype, g, pick_tile_n((g.M + 127) / 128, TP, g.K), s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_q_latent");
  }

  // ---- dX = [dQlat | dKlat | dVlat] [U2 | U3 | U~3]^T ----------------------------------------------------------
  {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A = ws.Wb; g.lda = LW; g.M = f.d_model;
    g.Bsrc = ws.dLat; g.ldb = LW; g.K = LW;
    g.Bsz = B; g.N = N; g.Npad = Npad; g.src_padded = 1;
    g.epi = 2; g.Out = dX; g.ldo = f.d_model; g.ksplit = 1;
    if (launch_gemm(f.dtype, g, pick_tile_n((g.M + 127) / 128, TP, g.K), s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_x");
  }

  // ---- products over tokens: out[m][n] = sum_t A[t][m] B[t][n], operands token-major as they are -----------------
  auto over_tokens = [&](const void* At, long lda, int a_padded, int M, int perm_m, const void* Bt, long ldb, int cols,
                         int perm_n, int ksplit, const GemmArgs::Out3 (&outs)[3]) {
    TnArgs t;
    std::memset(&t, 0, sizeof(t));
    t.At = At; t.lda = lda; t.a_padded = a_padded; t.Bt = Bt; t.ldb = ldb; t.b_padded = 1;
    t.Bsz = B; t.N = N; t.Npad = Npad;
    t.g.M = M; t.g.Bsz = 1; t.g.N = cols; t.g.Npad = cols;
    t.g.epi = 3; t.g.ksplit = ksplit; t.g.part = ws.part; t.g.out_scale = 1.f;
    t.g.perm_m = perm_m; t.g.perm_n = perm_n;
    for (int u = 0; u < 3; ++u) t.g.out3[u] = outs[u];
    return launch_gemm_tn(f.dtype, t, s);
  };
  {
    const GemmArgs::Out3 o[3] = {{gr->dU2, 0, f.r2, f.r2},
                                 {gr->dU3, c->R2, c->R2 + f.r3, f.r3},
                                 {f.shared_kv ? nullptr : gr->dUt3, c->R2 + c->D, c->R2 + c->D + f.rt3, f.rt3}};
    if (over_tokens(X, f.d_model, 0, f.d_model, 0, ws.dLat, LW, LW, 0, ws.ks_w, o) != hipSuccess)
      return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_u2_u3_ut3");
  }
  {
    const GemmArgs::Out3 o[3] = {{gr->dUt2, 0, f.rt2, f.rt2}, {nullptr, 0, 0, 0}, {nullptr, 0, 0, 0}};
    if (over_tokens(dY, f.d_model, 0, f.d_model, 0, ws.f.Z, c->RT2, c->RT2, 0, ws.ks_u, o) != hipSuccess)
      return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_ut2");
  }
  {
    // Qlat holds its columns, and dQ / O their channels, in acc order: undone when the result is stored
    const GemmArgs::Out3 o[3] = {{ws.dG, 0, nHD, nHD}, {nullptr, 0, 0, 0}, {nullptr, 0, 0, 0}};
    if (over_tokens(ws.f.Qlat, c->R2, 1, c->R2, 1, ws.dQ, nHD, nHD, 1, ws.ks_g, o) != hipSuccess)
      return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_core_mixed");
  }
  {
    const GemmArgs::Out3 o[3] = {{ws.dGt, 0, nHD, nHD}, {nullptr, 0, 0, 0}, {nullptr, 0, 0, 0}};
    if (over_tokens(ws.dZ, c->RT2, 1, c->RT2, 0, ws.f.O, nHD, nHD, 1, ws.ks_g, o) != hipSuccess)
      return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_core_mixed_post");
  }

  // ---- G_i = sum_a U1[i,a] C[a]: gradients of the core and of the head factor ----------------------------------
  {
    CoreGradArgs k;
    std::memset(&k, 0, sizeof(k));
    k.dG = ws.dG; k.D = c->D; k.nH = f.n_heads; k.C = w->C; k.U1 = w->U1; k.r1 = f.r1; k.r2 = f.r2; k.r3 = f.r3;
    k.scale = (float)(1.0 / std::sqrt((double)f.d_head)); k.dC = gr->dC; k.dU1 = gr->dU1;
    if (launch_core_grad(f.dtype, k, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    k.dG = ws.dGt; k.C = w->Ct; k.U1 = w->Ut1; k.r1 = f.rt1; k.r2 = f.rt2; k.r3 = f.rt3;
    k.scale = 1.f; k.dC = gr->dCt; k.dU1 = gr->dUt1;
    if (launch_core_grad(f.dtype, k, s) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    rec.after("grad_core_and_head_factor");
  }
  return TUCKER_ATTN_OK;
}

int tucker_attn_decode(tucker_attn_ctx* c, const tucker_attn_weights* w, const void* x, void* y, void* Kcache,
                       void* Vcache, int32_t Lmax, const int32_t* kv_len, int32_t B, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  if (!workspace) return TUCKER_ATTN_INVALID_ARG;
  return decode_impl(c, w, x, y, Kcache, Vcache, Lmax, kv_len, B, workspace, workspace_bytes, hip_stream);
}

int tucker_attn_decode_static(tucker_attn_ctx* c, const tucker_attn_weights* w, const void* x, void* y, void* Kcache,
                              void* Vcache, int32_t Lmax, const int32_t* kv_len, int32_t B, void* hip_stream) {
  if (!c || B < 1) return TUCKER_ATTN_INVALID_ARG;
  if (carve_decode(c, nullptr, B < kDecodeChunk ? B : kDecodeChunk).bytes > kStaticScratchBytes)
    return TUCKER_ATTN_WORKSPACE_TOO_SMALL;
  void* ws = nullptr;
  if (static_scratch(&ws) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  return decode_impl(c, w, x, y, Kcache, Vcache, Lmax, kv_len, B, ws, kStaticScratchBytes, hip_stream);
}

size_t tucker_attn_prepared_weights_bytes(const tucker_attn_ctx* c) { return c ? prepared_bytes(c) : 0; }

int tucker_attn_prepare_weights(tucker_attn_ctx* c, const tucker_attn_weights* w, void* prepared, size_t bytes,
                                void* hip_stream) {
  if (!c || !weights_ok(c, w) || !prepared) return TUCKER_ATTN_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(prepared) % kAlign != 0) return TUCKER_ATTN_INVALID_ARG;
  if (bytes < prepared_bytes(c)) return TUCKER_ATTN_WORKSPACE_TOO_SMALL;
  Carver cv{static_cast<char*>(prepared), 0};
  void *Gt, *Gtil2, *Wcat, *Ut2p;
  carve_weights(c, cv, Gt, Gtil2, Wcat, Ut2p);
  const void* ut2;
  long ut2_ld;
  PrepArgs pa = make_prep(c, w, Gt, Gtil2, Wcat, Ut2p, &ut2, &ut2_ld);
  if (launch_prep(c->cfg.dtype, pa, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  c->prepared = prepared;
  c->prepared_from = *w;
  return TUCKER_ATTN_OK;
}

int tucker_attn_release_weights(tucker_attn_ctx* c) {
  if (!c) return TUCKER_ATTN_INVALID_ARG;
  c->prepared = nullptr;
  std::memset(&c->prepared_from, 0, sizeof(c->prepared_from));
  return TUCKER_ATTN_OK;
}

int tucker_attn_profile_enable(tucker_attn_ctx* c, int32_t on) {
  if (!c) return TUCKER_ATTN_INVALID_ARG;
  if (on && !c->ev_created) {
    for (int i = 0; i <= kMaxKernels; ++i)
      if (hipEventCreate(&c->ev[i]) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    for (int i = 0; i < 2; ++i)
      if (hipEventCreate(&c->kev[i]) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
    c->ev_created = true;
  }
  c->profile = on ? 1 : 0;
  c->n_kernels = 0;
  c->kev_name = nullptr;
  return TUCKER_ATTN_OK;
}

int tucker_attn_profile_read(tucker_attn_ctx* c, const char** names, float* ms, int32_t n_max) {
  if (!c || !c->ev_created) return TUCKER_ATTN_INVALID_ARG;
  const int n = c->n_kernels;
  if (n == 0) return 0;
  if (hipEventSynchronize(c->ev[n]) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  for (int i = 0; i < n && i < n_max; ++i) {
    if (names) names[i] = c->names[i];
    if (ms) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, c->ev[i], c->ev[i + 1]) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
      ms[i] = t;
    }
  }
  // one more entry: the dominant kernel alone, from the two events attached to its dispatch
  if (c->kev_name != nullptr && n < n_max) {
    if (names) names[n] = c->kev_name;
    if (ms) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, c->kev[0], c->kev[1]) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
      ms[n] = t;
    }
    return n + 1;
  }
  return n;
}

const char* tucker_attn_status_string(int status) {
  switch (status) {
    case TUCKER_ATTN_OK: return "ok";
    case TUCKER_ATTN_INVALID_ARG: return "invalid argument";
    case TUCKER_ATTN_UNSUPPORTED_SHAPE: return "unsupported shape";
    case TUCKER_ATTN_WORKSPACE_TOO_SMALL: return "workspace too small";
    case TUCKER_ATTN_HIP_ERROR: return "HIP runtime error";
    default: return "unknown status";
  }
}

}  // extern "C"
