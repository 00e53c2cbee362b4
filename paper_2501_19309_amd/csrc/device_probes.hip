// Two measurements of the device itself, for reading the library's roofline fractions: what a loop of
// nothing but independent bf16 MFMAs sustains (the matrix cores at the clock the board grants them), and what a
// pure streaming read of a large buffer sustains (HBM).  Diagnostics behind the C ABI; the verification
// path does not use them.
#include "../../include/jd_verify.h"

#include <cstdint>
#include <cstdio>

#include <hip/hip_runtime.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeTiles = 24;  // independent accumulator tiles per wavefront: no MFMA waits for another

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4* p) {  // non-temporal 128-bit load
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int kProbeTiles32 = 6;  // independent 32 x 32 tiles (96 accumulator registers, as the 24 tiles of 16 x 16)

// Several wavefronts per SIMD (the kernel needs about 110 registers), each a loop of nothing but independent
// MFMAs that accumulate in place (inline assembly: left to the compiler the loop gets register copies and
// wait states between the MFMAs, and then measures those).  The loop has no memory traffic, so however the
// dispatcher places the workgroups, every SIMD's matrix pipeline always has an MFMA waiting.
// operand_mode 0: all-zero operands; 1: values spread like N(0,1) rounded to bf16, different per lane and
// element (what embeddings and weights look like to the matrix cores).
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* out, int iters, int operand_mode) {
  f32x4 acc[kProbeTiles];
#pragma unroll
  for (int i = 0; i < kProbeTiles; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
  auto value = [&](unsigned i) -> unsigned {  // bf16 bits of a sum of two uniforms, scaled to unit variance
    unsigned h = (threadIdx.x * 8u + i + blockIdx.x * 4099u) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    const float f = (((h & 0xffff) + ((h >> 16) & 0xffff)) * (1.0f / 65536.0f) - 1.0f) * 2.45f;
    return __float_as_uint(f) >> 16;
  };
  auto pair = [&](unsigned i) { return operand_mode == 0 ? 0u : (value(2 * i) | (value(2 * i + 1) << 16)); };
  const u32x4 a = {pair(0), pair(1), pair(2), pair(3)};
  const u32x4 b = {pair(4), pair(5), pair(6), pair(7)};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kProbeTiles; ++i)
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last MFMAs leave the pipeline before their tiles are read
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kProbeTiles; ++i) s += (acc[i][0] + acc[i][1]) + (acc[i][2] + acc[i][3]);
  if (s == 12345.678f) out[blockIdx.x * 256 + threadIdx.x] = s;  // keeps the loop alive; practically never taken
}

// The same loop on the other bf16 MFMA shape, v_mfma_f32_32x32x16_bf16 (twice the flops per instruction and per
// operand fragment, four times the accumulator registers per tile), N(0,1)-like operands: which of the two shapes
// the matrix cores sustain at the higher rate decides the tile shape of the large-row LM-head kernels.
__global__ __launch_bounds__(256) void mfma_rate_32x32_kernel(float* out, int iters) {
  f32x16 acc[kProbeTiles32];
#pragma unroll
  for (int i = 0; i < kProbeTiles32; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  auto value = [&](unsigned i) -> unsigned {
    unsigned h = (threadIdx.x * 8u + i + blockIdx.x * 4099u) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    const float f = (((h & 0xffff) + ((h >> 16) & 0xffff)) * (1.0f / 65536.0f) - 1.0f) * 2.45f;
    return __float_as_uint(f) >> 16;
  };
  auto pair = [&](unsigned i) { return value(2 * i) | (value(2 * i + 1) << 16); };
  const u32x4 a = {pair(0), pair(1), pair(2), pair(3)};
  const u32x4 b = {pair(4), pair(5), pair(6), pair(7)};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kProbeTiles32; ++i)
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kProbeTiles32; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[i][j];
  if (s == 12345.678f) out[blockIdx.x * 256 + threadIdx.x] = s;
}

// Streaming read: a wavefront reads 32 KiB of consecutive memory per turn as four batches of eight 128-bit
// non-temporal loads per lane (plain loads reach 6.0-6.2 TB/s where these reach 6.8-7.1), two batches in flight
// while a third is folded (straight-line code inside a turn, so the compiler's wait counts are exact); the
// wavefronts of the grid read consecutive pieces and the grid moves through the buffer as one window - the access
// pattern of the LM-head weight stream.  STREAM = false: the same with plain loads, for the comparison.
template <bool STREAM>
__global__ __launch_bounds__(256) void hbm_read_kernel(const uint4* __restrict__ src, size_t n_items, uint4* out) {
  auto ld = [](const uint4* q) -> uint4 {
    if constexpr (STREAM) return load_stream(q);
    else return *q;
  };
  const size_t lane = threadIdx.x & 63;
  const size_t n_chunks = n_items / 2048;                            // 2048 items = 32 KiB
  const size_t n_waves = (size_t)gridDim.x * 4;
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  auto fold = [&](const uint4 (&v)[8]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
  };
  for (size_t c = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6); c < n_chunks; c += n_waves) {
    const uint4* p = src + c * 2048 + lane;
    uint4 a[8], b[8], x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] = ld(p + u * 64);
#pragma unroll
    for (int u = 0; u < 8; ++u) b[u] = ld(p + 512 + u * 64);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = a[u];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] = ld(p + 1024 + u * 64);
    __builtin_amdgcn_sched_barrier(0);
    fold(x);
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = b[u];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 8; ++u) b[u] = ld(p + 1536 + u * 64);
    __builtin_amdgcn_sched_barrier(0);
    fold(x);
    fold(a);
    fold(b);
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) out[blockIdx.x * 256 + threadIdx.x] = acc;  // buffer is zero: never
}

int fail(hipError_t e) { (void)hipGetLastError(); return e == hipErrorOutOfMemory ? JD_ERR_OOM : JD_ERR_HIP; }

}  // namespace

#define JD_TRY(expr) do { const hipError_t e_ = (expr); if (e_ != hipSuccess) { rc = fail(e_); goto done; } } while (0)

extern "C" int jd_verify_probe_mfma_bf16(int32_t device, int32_t operand_mode, double* out_tflops) {
  if (!out_tflops || device < 0 || operand_mode < 0 || operand_mode > 2) return JD_ERR_INVALID_ARG;
  *out_tflops = 0.0;
  int rc = JD_OK;
  float* out = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipDeviceProp_t prop;
  int wgs = 0;
  const int iters = 4000;
  float ms = 0.f;
  JD_TRY(hipSetDevice(device));
  JD_TRY(hipGetDeviceProperties(&prop, device));
  wgs = 4 * prop.multiProcessorCount;  // 4 wavefronts each: several per SIMD, wherever the dispatcher puts them
  JD_TRY(hipMalloc(reinterpret_cast<void**>(&out), (size_t)wgs * 256 * sizeof(float)));
  JD_TRY(hipEventCreate(&e0));
  JD_TRY(hipEventCreate(&e1));
  // some launches first: the clock settles only after tens of milliseconds under this load
  for (int w = 0; w < 13; ++w) {
    if (w == 10) JD_TRY(hipEventRecord(e0, nullptr));  // the last three launches are the timed ones
    if (operand_mode == 2)
      hipLaunchKernelGGL(mfma_rate_32x32_kernel, dim3(wgs), dim3(256), 0, nullptr, out, iters);
    else
      hipLaunchKernelGGL(mfma_rate_kernel, dim3(wgs), dim3(256), 0, nullptr, out, iters, operand_mode);
  }
  JD_TRY(hipGetLastError());
  JD_TRY(hipEventRecord(e1, nullptr));
  JD_TRY(hipEventSynchronize(e1));
  JD_TRY(hipEventElapsedTime(&ms, e0, e1));
  {
    const double flops_per_wave_iter = operand_mode == 2 ? kProbeTiles32 * (2.0 * 32 * 32 * 16) : kProbeTiles * (2.0 * 16 * 16 * 32);
    *out_tflops = 3.0 * (double)wgs * 4 * iters * flops_per_wave_iter / ((double)ms * 1e-3) / 1e12;
  }
done:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (out) (void)hipFree(out);
  return rc;
}

static int probe_hbm_read(int32_t device, uint64_t bytes, bool stream, double* out_gbs) {
  if (!out_gbs || device < 0 || bytes < (1ull << 20) || bytes > (64ull << 30)) return JD_ERR_INVALID_ARG;
  *out_gbs = 0.0;
  int rc = JD_OK;
  uint4* buf = nullptr;
  uint4* out = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipDeviceProp_t prop;
  int wgs = 0;
  float ms = 0.f;
  const size_t n_items = bytes / sizeof(uint4);
  auto launch = [stream](int grid, const uint4* src, size_t n, uint4* dst) {
    if (stream) hipLaunchKernelGGL(hbm_read_kernel<true>, dim3(grid), dim3(256), 0, nullptr, src, n, dst);
    else hipLaunchKernelGGL(hbm_read_kernel<false>, dim3(grid), dim3(256), 0, nullptr, src, n, dst);
  };
  JD_TRY(hipSetDevice(device));
  JD_TRY(hipGetDeviceProperties(&prop, device));
  wgs = prop.multiProcessorCount * 8;
  JD_TRY(hipMalloc(reinterpret_cast<void**>(&buf), n_items * sizeof(uint4)));
  JD_TRY(hipMalloc(reinterpret_cast<void**>(&out), (size_t)wgs * 256 * sizeof(uint4)));
  JD_TRY(hipMemset(buf, 0, n_items * sizeof(uint4)));
  JD_TRY(hipEventCreate(&e0));
  JD_TRY(hipEventCreate(&e1));
  launch(wgs, buf, n_items, out);
  JD_TRY(hipGetLastError());
  JD_TRY(hipEventRecord(e0, nullptr));
  for (int w = 0; w < 3; ++w) launch(wgs, buf, n_items, out);
  JD_TRY(hipGetLastError());
  JD_TRY(hipEventRecord(e1, nullptr));
  JD_TRY(hipEventSynchronize(e1));
  JD_TRY(hipEventElapsedTime(&ms, e0, e1));
  *out_gbs = 3.0 * (double)((n_items / 2048) * 2048 * sizeof(uint4)) / ((double)ms * 1e-3) / 1e9;
done:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (buf) (void)hipFree(buf);
  if (out) (void)hipFree(out);
  return rc;
}

extern "C" int jd_verify_probe_hbm_read(int32_t device, uint64_t bytes, double* out_gbs) {
  return probe_hbm_read(device, bytes, true, out_gbs);
}
extern "C" int jd_verify_probe_hbm_read_plain(int32_t device, uint64_t bytes, double* out_gbs) {
  return probe_hbm_read(device, bytes, false, out_gbs);
}
