// Kernel argument structures and launcher declarations shared by the host API and the
// device code.  All pointers are device pointers; all sizes are in elements unless a name
// says bytes.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

namespace ta {

// ---- weight preparation (head-mixed cores, transposed factor matrices) ------------------
// out[z][u][v] = scale * sum_a coef[z][a] * src[a][row][col]   with (u,v) = (col,row) when
// transposed, (row,col) otherwise; rows/cols beyond the source extents read as zero so the
// padded part of the output is written as zero.  perm: store column v of each 32-block at
// its acc-order position.  frag: the output is fragment-major (see common.h): 32x32 blocks of
// (u, v), block (u/32, v/32) at ((u/32) * n_vblocks + v/32) * 1024 from out + z*out_stride_z.
struct PrepJob {
  const void* src;      // [A][rows][cols]
  const void* coef;     // [Z][A] or null (A must be 1, coefficient 1)
  void* out;
  int A, rows, cols;    // source extents
  int Z;
  int rows_pad, cols_pad;   // padded extents covered by tiles (multiples of 32)
  long out_stride_z, out_stride_u;
  int transposed, perm, frag;
  float scale;
  int first_block;      // prefix sum of the jobs' workgroup counts (prep_job_blocks)
};
constexpr int kMaxPrepJobs = 8;
struct PrepArgs {
  PrepJob job[kMaxPrepJobs];
  int n_jobs;
  int total_blocks;
};

// ---- generic product  acc[m][tok] = sum_k A[m][k] * Btok[tok][k]  with three epilogues ---
struct GemmArgs {
  const void* A;        // [M][lda] weights side (rows beyond M read as zero)
  long lda;
  int M;
  const void* Bsrc;     // token side
  long ldb;
  int K;                // contraction length (elements beyond K read as zero)
  // token indexing: padded token tp = b*Npad + n ; source row exists iff n < N
  int Bsz, N, Npad;
  int src_padded;       // 1: Bsrc rows are indexed by tp; 0: by b*N+n (caller's X)
  // epilogue outputs
  int epi;              // 0 = projection, 1 = latent merge Z, 2 = output Y, 3 = fp32 matrix (gradients)
  // projection
  void* Qlat; int R2;           // [TP][R2] acc order
  void* Kr;   int D;            // [TP][D]  acc order, rotated
  void* Vt;                     // [B][D][Npad], n in acc order within 32-blocks; null in decode
  void* Vr;                     // nullable [TP][D] acc order: value rows (for the backward pass)
  void* Krt;                    // nullable [B][D][Npad] like Vt: rotated keys, transposed (backward pass)
  void* Kcache; void* Vcache;   // nullable [B][Lmax][r3]/[B][Lmax][rt3], natural order
  int Lmax, r3, rt3;
  // rotation table or null: [D/4][rope_ld positions] entries (cos, sin, cos, sin) of the channel
  // pairs (4k, 4k+1), (4k+2, 4k+3); identity beyond r3.  Positions are the fast index, so lanes
  // that hold consecutive tokens read consecutive entries.
  const float4* rope;
  int rope_ld;
  int pos0;
  int shared_kv;                // 1: no V rows in A; the K block also yields Vt, and the cache row, UNROTATED
  int decode;                   // 1: one token per sequence, position/cache row from kv_pos[b]
  int kv_pos[32];
  // Z / Y
  void* Out; long ldo;          // Z: [TP][ldo] natural order;  Y: [B][N][ldo] natural order
  // split-K (decode-sized token counts): ksplit > 1 writes fp32 partial tiles to part
  // [ksplit][TP][Mp] (Mp = weight rows padded to 32); a second kernel sums them and runs the
  // epilogue
  int ksplit;
  float* part;
  int defer_reduce;     // 1: no reduction launch here; the caller's next kernel sums the partial tiles
  // epi 3: out_scale * acc[m][n] as fp32; column range [n0, n1) of the product goes to
  // ptr[m * ld + (n - n0)] (up to three destinations; ptr null = unused)
  struct Out3 { float* ptr; int n0, n1; long ld; } out3[3];
  float out_scale;
  int perm_m, perm_n;   // 1: rows / columns of the product are in acc order within 32-blocks; stored natural
};

// out[m][n] = sum over tokens t of At[t][m] * Bt[t][n]; both operands token-major.  g carries the
// output side as for epilogue 3 (M, Bsz = 1, N = Npad = number of columns, ksplit, part, out3, ...).
struct TnArgs {
  GemmArgs g;
  const void* At; long lda; int a_padded;   // padded: row of token (b, n) is b*Npad + n, else b*N + n
  const void* Bt; long ldb; int b_padded;
  int Bsz, N, Npad;
};

// ---- prefill attention ---------------------------------------------------------------------
struct AttnArgs {
  const void* Qlat;   // [TP][R2] acc order
  const void* Gt;     // [nH] x fragment-major 32x32 blocks of Gt[i][c][b] = qscale * G_i[b][c], b in acc order
  const void* Kr;     // [TP][D]
  const void* Vt;     // [B][D][Npad]
  void* O;            // [TP][nH][D] acc order in c, normalised; rows of padding tokens are zero
  float* lse;         // nullable [B][nH][Npad]: log2 of the softmax denominator (+inf for padding tokens)
  const float4* rope; // [D/4][rope_ld] as in GemmArgs, or null
  int rope_ld;
  int Bsz, N, Npad, nH, R2, r3, D;   // D = padded common width of K and V (32, 64 or 128)
  int causal, pos0;
};

// ---- backward pass of prefill attention ---------------------------------------------------------
struct BwdArgs {
  const void* Qlat;    // [TP][R2] acc order
  const void* Gt;      // as AttnArgs
  const void* dZ;      // [TP][RT2] natural order (rows of padding tokens zero)
  const void* Gtil_t;  // [nH] x fragment-major blocks of G~t[i][c][b] = G~_i[b][c], b natural
  const void* Kr;      // [TP][D] rotated keys, acc order in c
  const void* Vr;      // [TP][D] values, acc order in c
  const void* Krt;     // [B][D][Npad] rotated keys transposed, n acc order
  const void* O;       // [TP][nH][D]
  const float* lse;    // [B][nH][Npad]
  float* delta;        // [B][nH][Npad]  sum_c dO O
  void* Qr;            // [TP][nH][D] rotated, scaled per-head queries (acc order in c)
  void* dO;            // [TP][nH][D] (acc order in c)
  void* dQ;            // [TP][nH][D] dS K with the rotation removed (the 1/sqrt(d_head) is applied later), acc order in c
  float* dKp;          // [n_hg][TP][D] per-head-group partial gradients of the rotated keys / values, channels at
                       // their stored (acc-order) positions
  float* dVp;
  const float4* rope;
  int rope_ld;
  int Bsz, N, Npad, nH, R2, RT2, D;
  int causal, pos0;
  int hpg, n_hg;       // heads per group and number of groups of the key/value gradient kernel
};

// dLat[tp][col0 + c] from the partial key/value gradients: keys un-rotated; with a shared latent
// the value part is added to the key part
struct KvReduceArgs {
  const float* dKp; const float* dVp;
  void* dLat; long ld; int colK, colV;
  const float4* rope; int rope_ld;
  int Bsz, N, Npad, D, n_hg, pos0, shared_kv;
};

// dC[a][b][c] = scale * sum_i U1[i][a] dG[b][i*D + c];  dU1[i][a] = scale * sum_bc dG[b][i*D+c] C[a][b][c]
struct CoreGradArgs {
  const float* dG; int D, nH;
  const void* C; const void* U1;
  int r1, r2, r3;
  float scale;
  float* dC; float* dU1;
};

// ---- decode ------------------------------------------------------------------------------
struct DecodeArgs {
  const void* Qlat;    // [32][R2] acc order (rows >= B are zero)
  const void* Gt;      // as above
  void* Qh;            // [B][HB*32][D] natural order, rotated, scaled (rows >= nH zero)
  const void* Kcache;  // [B][Lmax][r3]
  const void* Vcache;  // [B][Lmax][rt3]
  float* part_m;       // [B][nsplit][HB*32]
  float* part_l;
  float* part_o;       // [B][nsplit][HB*32][D]
  const float4* rope; // [D/4][rope_ld] as in GemmArgs, or null
  int rope_ld;
  int Bsz, nH, HB, R2, r3, rt3, D, Lmax, nsplit;
  int shared_kv;       // 1: Kcache holds the unrotated latent, which is also the value; Vcache is null
  const void* Gtil2;   // [RT2][nH*D] post-softmax head-mixed cores, c in acc order (head merge)
  float* zpart;        // [nH][Bsz][RT2] per-head contributions to Z, summed by the split-K reduction
  int RT2;
  const void* Ut2;     // [d_model][ut2_ld] output factor, k = RT2 contiguous (padded copy where rt2 is no multiple of 32)
  long ut2_ld;
  void* Y;             // [Bsz][d_model]
  int d_model;
  int kv_len[32];
};

// Which attention kernel a decode step runs.  A bf16 shared-latent cache whose rows are exactly D wide (a rank
// that is a multiple of 32) takes the wave-private kernel, which walks a slice in rounds of kDecodeRoundWave keys;
// any other configuration takes the workgroup-tile kernel (range-checked loads, tiles of kDecodeTile keys).
constexpr int kDecodeRoundWave = 128, kDecodeTile = 64;
inline bool decode_wave_private(int dtype, int r3, int D, int shared_kv) {
  return dtype == 1 && shared_kv && r3 == D;
}

// Raise a kernel's dynamic-LDS limit to `bytes`, once per kernel and device (the attribute belongs
// to the device's copy of the code object).  `once` is a static of the launcher of that one
// kernel instantiation.  Safe to call from several host threads.
struct LdsOnce {
  static constexpr int kMaxDevices = 64;
  std::atomic<unsigned char> done[kMaxDevices];
};
template <typename K>
inline hipError_t allow_dynamic_lds(LdsOnce& once, K kernel, size_t bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < LdsOnce::kMaxDevices;
  if (tracked && once.done[dev].load(std::memory_order_acquire)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && tracked) once.done[dev].store(1, std::memory_order_release);
  return e;
}

int prep_job_blocks(const PrepJob& j);     // workgroups (output tiles) of one job
hipError_t launch_prep(int dtype, const PrepArgs& a, hipStream_t s);
bool out_proj_supported(int dtype, const GemmArgs& a);
hipError_t launch_out_proj(int dtype, const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm(int dtype, const GemmArgs& a, int tile_n, hipStream_t s);
hipError_t launch_splitk_reduce(int dtype, const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm_tn(int dtype, const TnArgs& a, hipStream_t s);
// k0, k1 (both or neither): events that take the start and the end of the kernel itself (profiling)
hipError_t launch_attn_prefill(int dtype, const AttnArgs& a, hipStream_t s, hipEvent_t k0 = nullptr, hipEvent_t k1 = nullptr);
hipError_t launch_bwd_dq(int dtype, const BwdArgs& a, hipStream_t s);
hipError_t launch_bwd_dkv(int dtype, const BwdArgs& a, hipStream_t s);
hipError_t launch_kv_reduce(int dtype, const KvReduceArgs& a, hipStream_t s);
hipError_t launch_core_grad(int dtype, const CoreGradArgs& a, hipStream_t s);
// Factor projection of a decode step straight from the caller's factor matrices (no transposed copies):
// rows [0,R2) of the product are Qlat, [R2,R2+D) the key latent, [R2+D,R2+2D) the value latent; it leaves
// split-K partial tiles for the query launch to sum.  Needs factor rows that are whole 16-byte chunks.
struct DecodeProjArgs {
  const void* X;        // [Bsz][K]
  const void* U2;       // [K][r2]
  const void* U3;       // [K][r3]
  const void* Ut3;      // [K][rt3]; unused for a shared latent
  int r2, r3, rt3;
  int R2, D;
  int K, Bsz, ksplit, shared_kv;
  float* part;          // [ksplit][Bsz][Mp] fp32, Mp = R2 + (shared_kv ? 1 : 2) * D
};
// `prep` (possibly empty): weight-preparation tiles that ride along as the first workgroups of the launch
hipError_t launch_decode_proj(int dtype, const DecodeProjArgs& a, const PrepArgs& prep, hipStream_t s);
hipError_t launch_decode_qhat(int dtype, const DecodeArgs& a, const GemmArgs& proj, hipStream_t s);
hipError_t launch_decode_attn(int dtype, const DecodeArgs& a, hipStream_t s, hipEvent_t k0 = nullptr, hipEvent_t k1 = nullptr);
hipError_t launch_decode_merge_heads(int dtype, const DecodeArgs& a, hipStream_t s);
hipError_t launch_decode_out(int dtype, const DecodeArgs& a, hipStream_t s);

}  // namespace ta
