// Measured matrix-pipe ceiling of the device the library runs on, for reports that quote a fraction of the
// published peak: a loop of bf16 32x32x16 MFMAs on pseudo-random operands (the operand values matter: the board's
// power limit sets the clock, and all-zero operands draw far less power), eight waves per compute unit, either
// with both operands held in registers or with one operand fragment re-read from LDS for every pair of MFMAs,
// which is how the attention kernel is fed.
#include "../../include/tucker_attn.h"

#include <hip/hip_runtime.h>

#include "common.h"

using namespace ta;

// written only if a sum hits one particular value; external linkage, so the stores (and with them the loop) stay
__device__ float tucker_attn_ceiling_sink[64];

namespace {

constexpr int kCeilWaves = 8;          // waves per workgroup
constexpr int kCeilAcc = 4;            // independent accumulator blocks per wave

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// two bf16 values in (-1, 1) packed in a dword
__device__ __forceinline__ uint32_t rand_bf16x2(uint32_t s) {
  const uint32_t r = hash32(s);
  // sign and 7 mantissa bits from r, exponent 0x7e (values of magnitude in [0.5, 1))
  const uint32_t lo = ((r & 0x8000u) | 0x3f00u | (r & 0x7fu));
  const uint32_t hi = (((r >> 16) & 0x8000u) | 0x3f00u | ((r >> 16) & 0x7fu));
  return lo | (hi << 16);
}

template <bool FROM_LDS>
__global__ __launch_bounds__(64 * kCeilWaves) void mfma_ceiling_kernel(int iters) {
  __shared__ __attribute__((aligned(16))) uint32_t lds[kCeilWaves * kCeilAcc * 2 * 64 * 4];   // 2 KB fragment x 4 x 8 waves
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint32_t seed = (blockIdx.x * 512u + threadIdx.x) * 64u;
  Frag<bf16> a[kCeilAcc], b;
  u32x4 t;
#pragma unroll
  for (int i = 0; i < kCeilAcc; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) t[e] = rand_bf16x2(seed + 8 * i + 4 * j + e);
      a[i].v[j] = __builtin_bit_cast(bf16x8, t);
      if (FROM_LDS) *reinterpret_cast<u32x4*>(lds + (((wave * kCeilAcc + i) * 2 + j) * 64 + lane) * 4) = t;
    }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = rand_bf16x2(seed + 40 + 4 * j + e);
    b.v[j] = __builtin_bit_cast(bf16x8, t);
  }
  f32x16 acc[kCeilAcc];
#pragma unroll
  for (int i = 0; i < kCeilAcc; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  __syncthreads();
  // a fresh 2 KB fragment of this wave from LDS for every pair of MFMAs (conflict-free 16-byte reads), requested
  // one pair ahead of its use
  auto read = [&](int i) {
    const uint32_t* p = lds + ((wave * kCeilAcc + i) * 2 * 64 + lane) * 4;
    Frag<bf16> f;
    f.v[0] = *reinterpret_cast<const bf16x8*>(p);
    f.v[1] = *reinterpret_cast<const bf16x8*>(p + 64 * 4);
    asm volatile("" : "+v"(f.v[0]), "+v"(f.v[1]));                // the read is not hoisted out of the loop
    return f;
  };
  Frag<bf16> f[2];
  if (FROM_LDS) f[0] = read(0);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kCeilAcc; ++i) {
      if (FROM_LDS) {
        f[(i + 1) & 1] = read((i + 1) % kCeilAcc);
        mma32(acc[i], f[i & 1], b);
      } else {
        mma32(acc[i], a[i], b);
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kCeilAcc; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  if (s == 12345.678f) tucker_attn_ceiling_sink[lane] = s;                    // keeps the products alive; practically never taken
}

}  // namespace

extern "C" int tucker_attn_measure_mfma_ceiling(int32_t from_lds, int32_t iters, float* tflops_out) {
  if (!tflops_out || iters < 1 || (from_lds != 0 && from_lds != 1)) return TUCKER_ATTN_INVALID_ARG;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return TUCKER_ATTN_HIP_ERROR;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return TUCKER_ATTN_HIP_ERROR;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return TUCKER_ATTN_HIP_ERROR; }
  const dim3 grid(cus), block(64 * kCeilWaves);
  auto launch = [&](int n) {
    if (from_lds) hipLaunchKernelGGL(mfma_ceiling_kernel<true>, grid, block, 0, nullptr, n);
    else hipLaunchKernelGGL(mfma_ceiling_kernel<false>, grid, block, 0, nullptr, n);
  };
  int st = TUCKER_ATTN_OK;
  float best_ms = 0.f;
  launch(iters);                                                  // warm-up: code object, clocks
  launch(iters);
  for (int rep = 0; rep < 5 && st == TUCKER_ATTN_OK; ++rep) {
    float ms = 0.f;
    if (hipEventRecord(e0, nullptr) != hipSuccess) st = TUCKER_ATTN_HIP_ERROR;
    launch(iters);
    if (hipEventRecord(e1, nullptr) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess)
      st = TUCKER_ATTN_HIP_ERROR;
    if (rep == 0 || ms < best_ms) best_ms = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != TUCKER_ATTN_OK) return st;
  const double flops = (double)cus * kCeilWaves * (double)iters * kCeilAcc * 2.0 * 32768.0;
  *tflops_out = (float)(flops / (best_ms * 1e-3) / 1e12);
  return TUCKER_ATTN_OK;
}
