// Shared device helpers for the gfx950 Tucker-attention kernels: element types, 32x32 MFMA
// block products on "fragments", LDS/global fragment access.
//
// Fragment model.  Every product here is built from 32x32 output blocks with a 32-wide
// slice of the contraction index.  For such a slice a lane holds 16 elements of an operand:
// lane l serves operand row (or column) l%32 and the half h = l/32 of the slice.  Which 16
// of the 32 contraction indices half h holds is free as long as both operands agree:
//   natural order   half h holds indices 16h .. 16h+15           (both operands from memory)
//   acc order       half h holds indices 8q+4h+r, q,r in 0..3    (one operand converted in
//                   registers from an MFMA accumulator, whose lane (column l%32, half h)
//                   holds rows 8q+4h+r in register 4q+r)
// Buffers that feed the second kind are stored with each 32-block permuted so that the 16
// elements of a half are contiguous: index 8q+4h+r sits at position 16h+4q+r.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ta {

typedef __bf16 bf16;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__host__ __device__ constexpr int pad32(int x) { return (x + 31) / 32 * 32; }
__host__ __device__ constexpr int pad64(int x) { return (x + 63) / 64 * 64; }

// position of contraction index x (0..31) inside an acc-ordered 32-block
__host__ __device__ constexpr int acc_pos(int x) { return 16 * ((x >> 2) & 1) + 4 * (x >> 3) + (x & 3); }

// natural index of the element stored at position p of an acc-ordered 32-block (inverse of acc_pos)
__host__ __device__ constexpr int acc_index(int p) { return 8 * ((p >> 2) & 3) + 4 * (p >> 4) + (p & 3); }

template <typename T> struct Frag;
template <> struct Frag<float> { f32x4 v[4]; };      // 16 fp32
template <> struct Frag<bf16> { bf16x8 v[2]; };      // 16 bf16

// acc += A_frag * B_frag over one 32-slice.  Result lane (column = B lane % 32, half h) holds
// rows 8q+4h+r of the A operand in register 4q+r.
__device__ __forceinline__ void mma32(f32x16& acc, const Frag<bf16>& a, const Frag<bf16>& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v[0], b.v[0], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v[1], b.v[1], acc, 0, 0, 0);
}
__device__ __forceinline__ void mma32(f32x16& acc, const Frag<float>& a, const Frag<float>& b) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[i][j], b.v[i][j], acc, 0, 0, 0);
}

// out = c + A_frag * B_frag over one 32-slice (c is read, not overwritten: a block that starts
// from a constant need not be copied first)
__device__ __forceinline__ void mma32_from(f32x16& out, const f32x16& c, const Frag<bf16>& a, const Frag<bf16>& b) {
  out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v[0], b.v[0], c, 0, 0, 0);
  out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v[1], b.v[1], out, 0, 0, 0);
}
__device__ __forceinline__ void mma32_from(f32x16& out, const f32x16& c, const Frag<float>& a, const Frag<float>& b) {
  out = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[0][0], b.v[0][0], c, 0, 0, 0);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (i + j > 0) out = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[i][j], b.v[i][j], out, 0, 0, 0);
}

// accumulator block -> operand fragment (acc order), with rounding to T
__device__ __forceinline__ Frag<float> to_frag_f32(const f32x16& a) {
  Frag<float> f;
#pragma unroll
  for (int i = 0; i < 4; ++i) f.v[i] = f32x4{a[4 * i], a[4 * i + 1], a[4 * i + 2], a[4 * i + 3]};
  return f;
}
__device__ __forceinline__ Frag<bf16> to_frag_bf16(const f32x16& a) {
  Frag<bf16> f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f32x2 two = {a[8 * i + 2 * j], a[8 * i + 2 * j + 1]};
      bf16x2 pk = __builtin_convertvector(two, bf16x2);
      f.v[i][2 * j] = pk[0];
      f.v[i][2 * j + 1] = pk[1];
    }
  return f;
}
template <typename T> __device__ __forceinline__ Frag<T> to_frag(const f32x16& a);
template <> __device__ __forceinline__ Frag<float> to_frag<float>(const f32x16& a) { return to_frag_f32(a); }
template <> __device__ __forceinline__ Frag<bf16> to_frag<bf16>(const f32x16& a) { return to_frag_bf16(a); }

// 16 contiguous elements (32 or 64 bytes, 16-byte aligned) <-> fragment
template <typename T> __device__ __forceinline__ Frag<T> load_frag(const T* p);
template <> __device__ __forceinline__ Frag<float> load_frag<float>(const float* p) {
  Frag<float> f;
  const f32x4* q = reinterpret_cast<const f32x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) f.v[i] = q[i];
  return f;
}
template <> __device__ __forceinline__ Frag<bf16> load_frag<bf16>(const bf16* p) {
  Frag<bf16> f;
  const bf16x8* q = reinterpret_cast<const bf16x8*>(p);
  f.v[0] = q[0];
  f.v[1] = q[1];
  return f;
}
template <typename T> __device__ __forceinline__ Frag<T> zero_frag();
template <> __device__ __forceinline__ Frag<float> zero_frag<float>() {
  Frag<float> f;
#pragma unroll
  for (int i = 0; i < 4; ++i) f.v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  return f;
}
template <> __device__ __forceinline__ Frag<bf16> zero_frag<bf16>() {
  Frag<bf16> f;
  u32x4 z = {0u, 0u, 0u, 0u};
  f.v[0] = __builtin_bit_cast(bf16x8, z);
  f.v[1] = f.v[0];
  return f;
}
template <typename T> __device__ __forceinline__ void store_frag(T* p, const Frag<T>& f);
template <> __device__ __forceinline__ void store_frag<float>(float* p, const Frag<float>& f) {
  f32x4* q = reinterpret_cast<f32x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) q[i] = f.v[i];
}
template <> __device__ __forceinline__ void store_frag<bf16>(bf16* p, const Frag<bf16>& f) {
  bf16x8* q = reinterpret_cast<bf16x8*>(p);
  q[0] = f.v[0];
  q[1] = f.v[1];
}

// Fragment-major storage of an operand matrix: every 32 (rows) x 32 (contraction positions)
// block is kept as 1024 consecutive elements ordered [16-byte chunk j][lane][element], so
// that the j-th 16-byte load of all 64 lanes of a wave reads one contiguous kilobyte.
// Lane = 32*h + row, where half h owns stored positions 16h .. 16h+15 of the block.
constexpr int kFragBlockElems = 1024;
template <typename T> __host__ __device__ constexpr int frag_major_offset(int row, int pos) {
  constexpr int CE = 16 / (int)sizeof(T);
  const int lane = 32 * (pos / 16) + row, p16 = pos % 16;
  return ((p16 / CE) * 64 + lane) * CE + p16 % CE;
}
template <typename T> __device__ __forceinline__ Frag<T> load_frag_major(const T* block, int lane);
template <> __device__ __forceinline__ Frag<float> load_frag_major<float>(const float* block, int lane) {
  Frag<float> f;
  const f32x4* q = reinterpret_cast<const f32x4*>(block) + lane;
#pragma unroll
  for (int i = 0; i < 4; ++i) f.v[i] = q[64 * i];
  return f;
}
template <> __device__ __forceinline__ Frag<bf16> load_frag_major<bf16>(const bf16* block, int lane) {
  Frag<bf16> f;
  const bf16x8* q = reinterpret_cast<const bf16x8*>(block) + lane;
  f.v[0] = q[0];
  f.v[1] = q[64];
  return f;
}

template <typename T> __device__ __forceinline__ void store_frag_major(T* block, int lane, const Frag<T>& f);
template <> __device__ __forceinline__ void store_frag_major<float>(float* block, int lane, const Frag<float>& f) {
  f32x4* q = reinterpret_cast<f32x4*>(block) + lane;
#pragma unroll
  for (int i = 0; i < 4; ++i) q[64 * i] = f.v[i];
}
template <> __device__ __forceinline__ void store_frag_major<bf16>(bf16* block, int lane, const Frag<bf16>& f) {
  bf16x8* q = reinterpret_cast<bf16x8*>(block) + lane;
  q[0] = f.v[0];
  q[64] = f.v[1];
}

// Transposed fragment from a row-major LDS tile: the operand row of this lane is tile COLUMN
// col0 + lane%32, and its 16 contraction elements are tile rows row0 + 8q+4h+r (acc order, q and r
// in 0..3) of that column.  bf16: four transposing LDS reads (each hands a lane four consecutive
// rows of its column: within 16 lanes, lane i supplies the address of row i/4, columns 4(i%4)..+3,
// and receives column i of the four rows); fp32: sixteen 4-byte reads.  `stride` in elements.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ Frag<bf16> load_frag_tr(const bf16* tile, int stride, int row0, int col0, int lane) {
  const int h = lane / 32, i = lane % 16;
  const bf16* base = tile + (row0 + 4 * h + i / 4) * stride + col0 + (lane & 16) + 4 * (i % 4);
  Frag<bf16> f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    auto* lp = (__attribute__((address_space(3))) s16x4*)(base + 8 * q * stride);
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(lp);
    const bf16x4 b = __builtin_bit_cast(bf16x4, v);
#pragma unroll
    for (int r = 0; r < 4; ++r) f.v[q / 2][(q % 2) * 4 + r] = b[r];
  }
  return f;
}
__device__ __forceinline__ Frag<float> load_frag_tr(const float* tile, int stride, int row0, int col0, int lane) {
  const int h = lane / 32;
  const float* base = tile + (row0 + 4 * h) * stride + col0 + lane % 32;
  Frag<float> f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) f.v[q][r] = base[(8 * q + r) * stride];
  return f;
}

// ---- unpadded LDS tiles with swizzled 16-byte chunks ---------------------------------------------
// A tile row of CPR chunks is stored without padding; chunk c of row r sits at chunk position
// c ^ swz_x<CPR>(r).  The 16 consecutive rows that one fragment read touches then fall into
// different banks.  (This is the layout that direct global-to-LDS loads can produce: one such load
// of a wave fills 64 consecutive chunks, lane l choosing which global chunk lands at position l.)
template <int CPR> __host__ __device__ constexpr int swz_x(int row) {
  constexpr int W = CPR >= 16 ? 1 : 16 / CPR, M = (CPR >= 16 ? 16 : CPR) - 1;
  return (row / W) & M;
}
// 16 consecutive elements, starting at chunk k0, of a swizzled row (x = swz_x of that row)
template <typename T> __device__ __forceinline__ Frag<T> load_frag_swz(const T* rowp, int k0, int x);
template <> __device__ __forceinline__ Frag<bf16> load_frag_swz<bf16>(const bf16* rowp, int k0, int x) {
  Frag<bf16> f;
  f.v[0] = *reinterpret_cast<const bf16x8*>(rowp + ((k0) ^ x) * 8);
  f.v[1] = *reinterpret_cast<const bf16x8*>(rowp + ((k0 + 1) ^ x) * 8);
  return f;
}
template <> __device__ __forceinline__ Frag<float> load_frag_swz<float>(const float* rowp, int k0, int x) {
  Frag<float> f;
#pragma unroll
  for (int j = 0; j < 4; ++j) f.v[j] = *reinterpret_cast<const f32x4*>(rowp + ((k0 + j) ^ x) * 4);
  return f;
}
// load_frag_tr on a swizzled tile whose rows hold CPR chunks (stride = CPR * elements per chunk)
template <int CPR>
__device__ __forceinline__ Frag<bf16> load_frag_tr_swz(const bf16* tile, int row0, int col0, int lane) {
  const int h = lane / 32, i = lane % 16;
  const int col = col0 + (lane & 16) + 4 * (i % 4);              // 4 consecutive columns: half a chunk
  Frag<bf16> f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = row0 + 8 * q + 4 * h + i / 4;
    const bf16* src = tile + row * (CPR * 8) + (((col / 8) ^ swz_x<CPR>(row)) * 8) + col % 8;
    auto* lp = (__attribute__((address_space(3))) s16x4*)(src);
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(lp);
    const bf16x4 b = __builtin_bit_cast(bf16x4, v);
#pragma unroll
    for (int r = 0; r < 4; ++r) f.v[q / 2][(q % 2) * 4 + r] = b[r];
  }
  return f;
}
template <int CPR>
__device__ __forceinline__ Frag<float> load_frag_tr_swz(const float* tile, int row0, int col0, int lane) {
  const int h = lane / 32, col = col0 + lane % 32;
  Frag<float> f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = row0 + 8 * q + 4 * h + r;
      f.v[q][r] = tile[row * (CPR * 4) + (((col / 4) ^ swz_x<CPR>(row)) * 4) + col % 4];
    }
  return f;
}
// The same transposed fragment read in two steps, for loops that keep direct global-to-LDS loads in flight
// while they read: the compiler puts a wait for ALL outstanding direct-to-LDS loads in front of the
// transposing-read builtin.  `start` only issues the four reads (the compiler does not see them as LDS reads);
// `finish` waits until every LDS read of the wave has returned and hands the fragment over.  Nothing may touch
// the result of `start` except `finish`.
struct FragTrPending { u32x2 q[4]; };
template <int CPR>
__device__ __forceinline__ FragTrPending load_frag_tr_swz_start(const bf16* tile, int row0, int col0, int lane) {
  const int h = lane / 32, i = lane % 16;
  const int col = col0 + (lane & 16) + 4 * (i % 4);
  FragTrPending f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = row0 + 8 * q + 4 * h + i / 4;
    const bf16* src = tile + row * (CPR * 8) + (((col / 8) ^ swz_x<CPR>(row)) * 8) + col % 8;
    const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const bf16*)src;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.q[q]) : "v"(addr) : "memory");
  }
  return f;
}
__device__ __forceinline__ Frag<bf16> load_frag_tr_finish(FragTrPending& f) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.q[0]), "+v"(f.q[1]), "+v"(f.q[2]), "+v"(f.q[3]) : : "memory");
  Frag<bf16> r;
  r.v[0] = __builtin_bit_cast(bf16x8, u32x4{f.q[0][0], f.q[0][1], f.q[1][0], f.q[1][1]});
  r.v[1] = __builtin_bit_cast(bf16x8, u32x4{f.q[2][0], f.q[2][1], f.q[3][0], f.q[3][1]});
  return r;
}
// one direct global-to-LDS load of this wave: 64 consecutive chunks of a swizzled tile starting at
// chunk q*64; `row_ptr(row)` gives the global address of tile row `row`
template <typename T, int CPR, class RowPtr>
__device__ __forceinline__ void dma_piece(T* tile, int q, int lane, RowPtr row_ptr) {
  constexpr int CE = 16 / (int)sizeof(T);
  const int ci = q * 64 + lane, row = ci / CPR, pos = ci % CPR;
  const T* g = row_ptr(row) + (pos ^ swz_x<CPR>(row)) * CE;
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)(tile + q * 64 * CE), 16, 0, 0);
}

// four consecutive accumulator registers (rows 8q+4h .. +3) -> 4 elements of T at p (natural order)
__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d) {
  *reinterpret_cast<f32x4*>(p) = f32x4{a, b, c, d};
}
__device__ __forceinline__ void store4(bf16* p, float a, float b, float c, float d) {
  f32x4 v = {a, b, c, d};
  *reinterpret_cast<bf16x4*>(p) = __builtin_convertvector(v, bf16x4);
}
__device__ __forceinline__ void store1(float* p, float a) { *p = a; }
__device__ __forceinline__ void store1(bf16* p, float a) { *p = (bf16)a; }
__device__ __forceinline__ float to_f32(float a) { return a; }
__device__ __forceinline__ float to_f32(bf16 a) { return (float)a; }

// Row-sum pieces of the softmax: the 16 probabilities a lane holds of one 32x32 block, added to acc.
// block_sum: the unrounded fp32 values, pairwise, in plain v_add_f32.
// frag_sum (bf16): the rounded values, two per v_dot2c_f32_bf16 -- half the instructions, but that
// instruction runs on the matrix pipe: measured on gfx950, one of them between two MFMAs stretches the
// pair from 17 to 30 ns, and issued by the partner wave it waits behind every MFMA in flight.  It pays
// only where the matrix pipe has idle time (the 32- and 64-channel kernels); see the call site.
__device__ __forceinline__ float block_sum(const f32x16& a, float acc) {
  float t[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] = a[2 * i] + a[2 * i + 1];
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = t[2 * i] + t[2 * i + 1];
  return acc + ((t[0] + t[1]) + (t[2] + t[3]));
}
__device__ __forceinline__ float frag_sum(const Frag<float>& f, float acc) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc += f.v[i][j];
  return acc;
}
__device__ __forceinline__ float frag_sum(const Frag<bf16>& f, float acc) {
  const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x2 pr = {f.v[i][2 * j], f.v[i][2 * j + 1]};
      acc = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, acc, false);
    }
  return acc;
}

// 16-byte chunk of T elements
template <typename T> struct Chunk { static constexpr int kElems = 16 / sizeof(T); };

// value held by the partner lane (l ^ 32) combined with ours
__device__ __forceinline__ float halves_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace ta
