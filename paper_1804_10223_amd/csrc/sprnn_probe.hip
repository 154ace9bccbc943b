// Device microbenchmarks behind the stated roofline (see include/sprnn_probe.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <random>
#include <vector>

#include "sprnn_probe.h"

namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr int kAuxCoherent = 16;   // sc1
constexpr unsigned kBufWord3 = 0x00027000u;
constexpr int kGatherWords = 16;

#define PROBE_CHECK(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); return -3; } } while (0)

__device__ __forceinline__ uint32_t xcc_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)); }

template <int WIDTH>
__global__ __launch_bounds__(1024) void gather_kernel(const uint32_t* __restrict__ offs, int iters, int lds_bytes, float* out) {
  extern __shared__ __align__(16) unsigned char lds[];
  for (int i = threadIdx.x * 4; i < lds_bytes; i += blockDim.x * 4) *reinterpret_cast<float*>(lds + i) = 1.0f;
  uint32_t o[kGatherWords];
#pragma unroll
  for (int k = 0; k < kGatherWords; ++k) o[k] = offs[k * blockDim.x + threadIdx.x];
  __syncthreads();
  float a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kGatherWords; ++k) {
      if (WIDTH == 16) {
        const float4 v = *reinterpret_cast<const float4*>(lds + o[k]);
        a0 += v.x; a1 += v.y; a2 += v.z; a3 += v.w;
      } else if (WIDTH == 8) {
        const float2 v = *reinterpret_cast<const float2*>(lds + o[k]);
        a0 += v.x; a1 += v.y;
      } else {
        a0 += *reinterpret_cast<const float*>(lds + o[k]);
      }
    }
    asm volatile("" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3));   // keep the loads inside the loop
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3;
}

// The same 16-byte reads with nothing else in the loop (the results are only kept alive, not added up), so that the
// loop is bound by the LDS alone and not by the additions of gather_kernel.
template <int WIDTH>
__global__ __launch_bounds__(1024) void gather_raw_kernel(const uint32_t* __restrict__ offs, int iters, int lds_bytes, float* out) {
  extern __shared__ __align__(16) unsigned char lds[];
  for (int i = threadIdx.x * 4; i < lds_bytes; i += blockDim.x * 4) *reinterpret_cast<float*>(lds + i) = 1.0f;
  uint32_t o[kGatherWords];
  const uint32_t base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)lds;
#pragma unroll
  for (int k = 0; k < kGatherWords; ++k) o[k] = base + offs[k * blockDim.x + threadIdx.x];
  __syncthreads();
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  f32x4 v[kGatherWords];
#pragma unroll
  for (int k = 0; k < kGatherWords; ++k) v[k] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kGatherWords; ++k) {
      if constexpr (WIDTH == 16) asm volatile("ds_read_b128 %0, %1" : "=v"(v[k]) : "v"(o[k]));
      else if constexpr (WIDTH == 8) asm volatile("ds_read_b64 %0, %1" : "=v"(*reinterpret_cast<double*>(&v[k])) : "v"(o[k]));
      else asm volatile("ds_read_b32 %0, %1" : "=v"(v[k].x) : "v"(o[k]));
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  float a = 0.0f;
#pragma unroll
  for (int k = 0; k < kGatherWords; ++k) a += v[k].x + v[k].y + v[k].z + v[k].w;
  out[blockIdx.x * blockDim.x + threadIdx.x] = a;
}

__global__ void where_kernel(uint32_t* xcc) {
  if (threadIdx.x == 0) xcc[blockIdx.x] = xcc_id();
}

// Bounded ping-pong: workgroup a writes r, b answers r; every wait gives up after `limit` polls.
__global__ void pingpong_kernel(uint32_t* flags, int a, int b, int rounds, int limit, long long* out, int* fail) {
  if (threadIdx.x != 0) return;
  const int me = blockIdx.x;
  if (me != a && me != b) return;
  uint32_t* mine = flags + (me == a ? 0 : 64);
  uint32_t* theirs = flags + (me == a ? 64 : 0);
  const long long t0 = wall_clock64();
  for (int r = 1; r <= rounds; ++r) {
    if (me == a) __hip_atomic_store(mine, (uint32_t)r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int spins = 0;
    while (__hip_atomic_load(theirs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (uint32_t)r) {
      if (++spins > limit) { *fail = 1; return; }
    }
    if (me == b) __hip_atomic_store(mine, (uint32_t)r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  const long long t1 = wall_clock64();
  if (me == a) { out[0] = t1 - t0; out[1] = xcc_id(); } else { out[2] = xcc_id(); }
}

__global__ __launch_bounds__(1024) void fill_probe_kernel(int* buf, int n4, int rounds, long long* out, int* sink) {
  extern __shared__ __align__(16) unsigned char lds[];
  __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(buf, 0, n4 * 16, kBufWord3);
  const long long t0 = wall_clock64();
  for (int r = 0; r < rounds; ++r) {
    for (int base = threadIdx.x; base < n4; base += 4 * blockDim.x) {
      i32x4 v[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int ci = base + c * blockDim.x;
        if (ci < n4) v[c] = __builtin_amdgcn_raw_buffer_load_b128(rs, ci * 16, 0, kAuxCoherent);
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int ci = base + c * blockDim.x;
        if (ci < n4) *reinterpret_cast<i32x4*>(lds + ci * 16) = v[c];
      }
    }
    __syncthreads();
  }
  const long long t1 = wall_clock64();
  if (threadIdx.x == 0) { out[blockIdx.x] = t1 - t0; sink[blockIdx.x] = *reinterpret_cast<int*>(lds + 16); }
}

struct DevBuf {
  void* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
};

double wall_clock_hz(int device) {
  int khz = 0;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, device) != hipSuccess || khz <= 0) khz = 100000;
  return khz * 1e3;
}

}  // namespace

extern "C" {

static int run_gather(int device, int workgroups, int threads, int width_bytes, const std::vector<uint32_t>& offs, double* bytes_per_second,
                      bool raw = false) {
  PROBE_CHECK(hipSetDevice(device));
  const int lds_bytes = 64 * 1024;
  DevBuf d_offs, d_out;
  PROBE_CHECK(hipMalloc(&d_offs.p, offs.size() * 4));
  PROBE_CHECK(hipMalloc(&d_out.p, (size_t)workgroups * threads * 4));
  PROBE_CHECK(hipMemcpy(d_offs.p, offs.data(), offs.size() * 4, hipMemcpyHostToDevice));
  const void* fn = width_bytes == 16 ? (const void*)gather_kernel<16> : width_bytes == 8 ? (const void*)gather_kernel<8> : (const void*)gather_kernel<4>;
  if (raw) fn = width_bytes == 16 ? (const void*)gather_raw_kernel<16> : width_bytes == 8 ? (const void*)gather_raw_kernel<8> : (const void*)gather_raw_kernel<4>;
  PROBE_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));   // > half a CU: one workgroup per CU
  hipEvent_t e0, e1;
  PROBE_CHECK(hipEventCreate(&e0));
  PROBE_CHECK(hipEventCreate(&e1));
  double best = 0;
  for (int rep = 0; rep < 3; ++rep) {
    const int iters = rep == 0 ? 50 : 4000;
    const uint32_t* po = (const uint32_t*)d_offs.p; float* pout = (float*)d_out.p; int lb = lds_bytes; int it = iters;
    void* args[] = {&po, &it, &lb, &pout};
    PROBE_CHECK(hipEventRecord(e0, 0));
    PROBE_CHECK(hipLaunchKernel(fn, dim3(workgroups), dim3(threads), args, 96 * 1024, 0));
    PROBE_CHECK(hipEventRecord(e1, 0));
    PROBE_CHECK(hipEventSynchronize(e1));
    float ms = 0;
    PROBE_CHECK(hipEventElapsedTime(&ms, e0, e1));
    if (rep > 0) best = std::max(best, (double)iters * kGatherWords * threads * width_bytes * workgroups / (ms * 1e-3));
  }
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  *bytes_per_second = best;
  return 0;
}

int sprnn_probe_lds_gather(int device, int workgroups, int threads, int width_bytes, int pattern, double* bytes_per_second) {
  if (!bytes_per_second || workgroups < 1 || threads < 64 || threads > 1024 || threads % 64) return -1;
  if (width_bytes != 4 && width_bytes != 8 && width_bytes != 16) return -1;
  const int ncol = 64 * 1024 / width_bytes;
  std::vector<uint32_t> offs((size_t)kGatherWords * threads);
  std::mt19937 rng(1);
  for (int k = 0; k < kGatherWords; ++k)
    for (int t = 0; t < threads; ++t) {
      const uint32_t col = pattern == 1 ? (uint32_t)(rng() % ncol) : (uint32_t)(((t % 64) + 64 * k + 7 * (t / 64)) % ncol);
      offs[(size_t)k * threads + t] = col * width_bytes;
    }
  return run_gather(device, workgroups, threads, width_bytes, offs, bytes_per_second);
}

int sprnn_probe_lds_gather_offsets(int device, int workgroups, int threads, int width_bytes, int bare, const uint32_t* offsets,
                                   double* bytes_per_second) {
  if (!bytes_per_second || !offsets || workgroups < 1 || threads < 64 || threads > 1024 || threads % 64) return -1;
  if (width_bytes != 4 && width_bytes != 8 && width_bytes != 16) return -1;
  std::vector<uint32_t> offs(offsets, offsets + (size_t)kGatherWords * threads);
  for (uint32_t o : offs)
    if (o % width_bytes || o + width_bytes > 64u * 1024u) return -1;   // every read inside the 64 KB the kernel fills
  return run_gather(device, workgroups, threads, width_bytes, offs, bytes_per_second, bare != 0);
}

int sprnn_probe_handoff(int device, int same_xcd, int rounds, double* nanoseconds, int xcc[2]) {
  if (!nanoseconds || rounds < 1) return -1;
  PROBE_CHECK(hipSetDevice(device));
  const int G = 32;
  DevBuf d_x, d_flags, d_out, d_fail;
  PROBE_CHECK(hipMalloc(&d_x.p, G * 4));
  hipLaunchKernelGGL(where_kernel, dim3(G), dim3(64), 0, 0, (uint32_t*)d_x.p);
  PROBE_CHECK(hipDeviceSynchronize());
  std::vector<uint32_t> where(G);
  PROBE_CHECK(hipMemcpy(where.data(), d_x.p, G * 4, hipMemcpyDeviceToHost));
  int a = 0, b = -1;
  for (int i = 1; i < G && b < 0; ++i)
    if ((where[i] == where[0]) == (same_xcd != 0)) b = i;
  if (b < 0) return -2;   // the device has a single XCD (or placement is not what was asked for)
  PROBE_CHECK(hipMalloc(&d_flags.p, 1024));
  PROBE_CHECK(hipMalloc(&d_out.p, 64));
  PROBE_CHECK(hipMalloc(&d_fail.p, 4));
  double best = 1e30;
  long long o[3] = {0, 0, 0};
  for (int rep = 0; rep < 3; ++rep) {
    PROBE_CHECK(hipMemset(d_flags.p, 0, 1024));
    PROBE_CHECK(hipMemset(d_out.p, 0, 64));
    PROBE_CHECK(hipMemset(d_fail.p, 0, 4));
    hipLaunchKernelGGL(pingpong_kernel, dim3(G), dim3(64), 0, 0, (uint32_t*)d_flags.p, a, b, rounds, 1 << 20, (long long*)d_out.p, (int*)d_fail.p);
    PROBE_CHECK(hipDeviceSynchronize());
    int f = 0;
    PROBE_CHECK(hipMemcpy(o, d_out.p, 24, hipMemcpyDeviceToHost));
    PROBE_CHECK(hipMemcpy(&f, d_fail.p, 4, hipMemcpyDeviceToHost));
    if (f) return -4;
    best = std::min(best, (double)o[0] / wall_clock_hz(device) * 1e9 / rounds / 2.0);
  }
  *nanoseconds = best;
  if (xcc) { xcc[0] = (int)o[1]; xcc[1] = (int)o[2]; }
  return 0;
}

int sprnn_probe_fill(int device, int workgroups, int threads, int bytes, int rounds, double* seconds_per_copy) {
  if (!seconds_per_copy || workgroups < 1 || threads < 64 || threads > 1024 || threads % 64 || bytes < 16 || bytes % 16 || bytes > 80 * 1024 || rounds < 1)
    return -1;
  PROBE_CHECK(hipSetDevice(device));
  DevBuf d_buf, d_out, d_sink;
  PROBE_CHECK(hipMalloc(&d_buf.p, bytes));
  PROBE_CHECK(hipMalloc(&d_out.p, (size_t)workgroups * 8));
  PROBE_CHECK(hipMalloc(&d_sink.p, (size_t)workgroups * 4));
  PROBE_CHECK(hipMemset(d_buf.p, 0, bytes));
  PROBE_CHECK(hipFuncSetAttribute((const void*)fill_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
  double best = 1e30;
  std::vector<long long> o(workgroups);
  for (int rep = 0; rep < 3; ++rep) {
    int* pb = (int*)d_buf.p; int n4 = bytes / 16; int r = rounds; long long* po = (long long*)d_out.p; int* ps = (int*)d_sink.p;
    void* args[] = {&pb, &n4, &r, &po, &ps};
    PROBE_CHECK(hipLaunchKernel((const void*)fill_probe_kernel, dim3(workgroups), dim3(threads), args, 96 * 1024, 0));   // (96 KB of LDS: one workgroup per CU, all at once)
    PROBE_CHECK(hipDeviceSynchronize());
    PROBE_CHECK(hipMemcpy(o.data(), d_out.p, (size_t)workgroups * 8, hipMemcpyDeviceToHost));
    const long long mx = *std::max_element(o.begin(), o.end());
    best = std::min(best, (double)mx / wall_clock_hz(device) / rounds);
  }
  *seconds_per_copy = best;
  return 0;
}

}  // extern "C"
