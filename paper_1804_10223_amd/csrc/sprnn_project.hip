// Input projection b'[m][n] = sum_k x[m][k] * W[n][k] + bias[n] on the matrix cores of gfx950.
//
// Section 3.1 of the paper turns Eq. 1 into Eq. 2 by computing the input term W x_t + b for all timesteps
// ahead of the recurrence.  That term is one dense product over M = T * B input vectors; both operands are
// contiguous along k, so a wavefront's MFMA fragments (8 consecutive k of one row per lane) are 16-byte reads.
//
// Precision: W is binary16 (exact in the MFMA, subnormals included), x is binary32.  Each x is split once,
// while it is staged into LDS, into hi = fp16(x) (rounded toward zero) and lo = fp16((x - hi) * 2^11) (rounded to
// nearest); hi + lo / 2^11 reproduces x to 2^-21 relative.  The two halves go through v_mfma_f32_32x32x16_f16 with
// separate binary32 accumulators that are combined in the epilogue, so products are exact and every sum is
// binary32.  The scale keeps lo in the normal binary16 range whenever x is.  |x| must stay below the binary16
// maximum (65504).
//
// Tiling: a workgroup of eight wavefronts owns a 64 (m) x 64 NJ (n) tile of b' (NJ = 1, 2, 3) and walks k in slabs of
// 64; four wavefronts (2 x 2 over the tile, 32 x 32 NJ each: NJ 32x32 MFMA tiles, hi and lo accumulators each) multiply
// the lower 32 k of every slab, the other four the upper 32 k, and the two sets of sums meet through LDS at the end:
// two wavefronts per SIMD cover each other's LDS and issue latencies.  Two LDS stages: while slab
// s is multiplied out of one, slab s + 1 is converted and written into the other between the MFMAs, and slabs
// s + 2 and s + 3 are in flight from memory in two register sets; one workgroup barrier per slab.  LDS rows are
// padded by 16 bytes so that the eight lanes served in one LDS pass touch all banks.  Consecutive tiles of one n
// block (the same rows of W) are dealt to workgroups that share an XCD, hence an L2.
#include <cstdlib>

#include "sprnn_device.h"

namespace sprnn {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 64;                 // rows of x (time x batch) per workgroup tile
constexpr int kBK = 64;                 // k per slab
constexpr int kPitch = (kBK + 8) * 2;   // LDS row pitch in bytes: 144
constexpr int kThreads = 512;           // eight wavefronts: 2 (m) x 2 (n) x 2 (halves of a slab's k)
constexpr float kLoScale = 2048.0f;
constexpr int kAPlane = kBM * kPitch;   // bytes of the hi (or lo) plane of one stage
constexpr int stage_bytes(int nj) { return 2 * kAPlane + 64 * nj * kPitch; }

// NJ = 32-wide MFMA tiles per wavefront along n.
template <int NJ>
struct SlabRegs {
  float4 a[2];        // 2 x (4 consecutive k of one x row)
  uint4 b[NJ];        // NJ x (8 consecutive k of one W row, binary16 bits)
};

// Per-thread constants of the staging copies: chunk i of a thread is x row (tid / 16 + 32 i), k (tid % 16) * 4 and
// W row (tid / 8 + 64 i), k (tid % 8) * 8 of the slab.
template <int NJ>
struct Staging {
  uint32_t a_off[2];        // byte offset of the chunk from x + m0 * K + k0 (row clamped to M - 1)
  uint32_t b_off[NJ];       // byte offset from W + n0 * K + k0 (row clamped to N - 1)
};

// Full slab, rows 16-byte aligned: plain vector loads at precomputed offsets.
template <int NJ>
__device__ __forceinline__ void load_slab_fast(SlabRegs<NJ>& r, const Staging<NJ>& st, const char* xs, const char* ws) {
#pragma unroll
  for (int i = 0; i < 2; ++i) r.a[i] = *reinterpret_cast<const float4*>(xs + st.a_off[i]);
#pragma unroll
  for (int i = 0; i < NJ; ++i) r.b[i] = *reinterpret_cast<const uint4*>(ws + st.b_off[i]);
}

// Any slab: element-wise loads with zeros beyond K.
template <int NJ>
__device__ __forceinline__ void load_slab_any(SlabRegs<NJ>& r, const float* __restrict__ X, const uint16_t* __restrict__ W,
                                              int tid, int m0, int n0, int k0, int M, int N, int K) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = tid + kThreads * i;
    const int row = min(m0 + (c >> 4), M - 1);
    const int k = k0 + (c & 15) * 4;
    const float* src = X + (size_t)row * K + k;
    r.a[i].x = (k + 0 < K) ? src[0] : 0.0f;
    r.a[i].y = (k + 1 < K) ? src[1] : 0.0f;
    r.a[i].z = (k + 2 < K) ? src[2] : 0.0f;
    r.a[i].w = (k + 3 < K) ? src[3] : 0.0f;
  }
#pragma unroll
  for (int i = 0; i < NJ; ++i) {
    const int c = tid + kThreads * i;
    const int row = min(n0 + (c >> 3), N - 1);
    const int k = k0 + (c & 7) * 8;
    const uint16_t* src = W + (size_t)row * K + k;
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = (k + e < K) ? (uint32_t)src[e] : 0u;
    r.b[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
  }
}

// (x0, x1) -> packed hi halves and packed scaled lo halves.
__device__ __forceinline__ void split2(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  const auto h = __builtin_amdgcn_cvt_pkrtz(x0, x1);
  hi = __builtin_bit_cast(uint32_t, h);
  typedef _Float16 half2v __attribute__((ext_vector_type(2)));
  half2v l;
  l[0] = (_Float16)((x0 - (float)h[0]) * kLoScale);
  l[1] = (_Float16)((x1 - (float)h[1]) * kLoScale);
  lo = __builtin_bit_cast(uint32_t, l);
}

// Convert and write chunk i of x and chunks of W of a slab into one LDS stage.
template <int NJ>
__device__ __forceinline__ void store_a_chunk(const SlabRegs<NJ>& r, int i, char* stage, int a_at) {
  uint2 hi, lo;
  split2(r.a[i].x, r.a[i].y, hi.x, lo.x);
  split2(r.a[i].z, r.a[i].w, hi.y, lo.y);
  *reinterpret_cast<uint2*>(stage + a_at + i * 32 * kPitch) = hi;
  *reinterpret_cast<uint2*>(stage + kAPlane + a_at + i * 32 * kPitch) = lo;
}
template <int NJ>
__device__ __forceinline__ void store_b_chunk(const SlabRegs<NJ>& r, int i, char* stage, int b_at) {
  *reinterpret_cast<uint4*>(stage + 2 * kAPlane + b_at + i * 64 * kPitch) = r.b[i];
}

template <int NJ>
__global__ __launch_bounds__(kThreads) void project_kernel(const float* __restrict__ X, const uint16_t* __restrict__ W,
                                                           const float* __restrict__ bias, float* __restrict__ out,
                                                           int M, int N, int K, int tiles_m, int vec) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int kBN = 64 * NJ;
  constexpr int kStage = stage_bytes(NJ);

  // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles.
  const int nb = gridDim.x, bid = blockIdx.x;
  const int id = (nb % 8 == 0) ? (bid % 8) * (nb / 8) + bid / 8 : bid;
  const int m0 = (id % tiles_m) * kBM, n0 = (id / tiles_m) * kBN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kg = wave >> 2;                       // which half of a slab's k this wavefront multiplies
  const int wm = wave & 1, wn = (wave >> 1) & 1;
  const int r = lane & 31, kh = lane >> 5;
  const int a_frag = (wm * 32 + r) * kPitch + kh * 16;                       // within the hi plane
  const int b_frag = 2 * kAPlane + (wn * 32 * NJ + r) * kPitch + kh * 16;
  const int a_at = (tid >> 4) * kPitch + (tid & 15) * 8;
  const int b_at = (tid >> 3) * kPitch + (tid & 7) * 16;

  Staging<NJ> st;
#pragma unroll
  for (int i = 0; i < 2; ++i)
    st.a_off[i] = (uint32_t)(min(m0 + (tid >> 4) + 32 * i, M - 1) - m0) * (uint32_t)K * 4u + (uint32_t)(tid & 15) * 16u;
#pragma unroll
  for (int i = 0; i < NJ; ++i)
    st.b_off[i] = (uint32_t)(min(n0 + (tid >> 3) + 64 * i, N - 1) - n0) * (uint32_t)K * 2u + (uint32_t)(tid & 7) * 16u;
  const char* x_tile = reinterpret_cast<const char*>(X + (size_t)m0 * K);
  const char* w_tile = reinterpret_cast<const char*>(W + (size_t)n0 * K);

  floatx16 acc_hi[NJ], acc_lo[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc_hi[j][v] = 0.0f; acc_lo[j][v] = 0.0f; }

  // Fragments of 16 k of a slab: this lane's 8 k of one x row (hi and lo) and of NJ rows of W.
  struct Frags { half8 ah, al, b[NJ]; };
  auto read_frags = [&](Frags& f, const char* cur, int q) {
    f.ah = *reinterpret_cast<const half8*>(cur + a_frag + q * 32);
    f.al = *reinterpret_cast<const half8*>(cur + kAPlane + a_frag + q * 32);
#pragma unroll
    for (int j = 0; j < NJ; ++j) f.b[j] = *reinterpret_cast<const half8*>(cur + b_frag + j * 32 * kPitch + q * 32);
  };
  auto mfmas = [&](const Frags& f) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      acc_hi[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.ah, f.b[j], acc_hi[j], 0, 0, 0);
      acc_lo[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.al, f.b[j], acc_lo[j], 0, 0, 0);
    }
  };
  auto multiply = [&](const char* cur, int q) {
    Frags f;
    read_frags(f, cur, q);
    mfmas(f);
  };

  // Pipelined part: the full slabs of a problem whose rows are 16-byte aligned.
  const int nfast = vec ? K / kBK : 0;
  auto load = [&](SlabRegs<NJ>& regs, int s) {
    load_slab_fast<NJ>(regs, st, x_tile + (size_t)s * kBK * 4, w_tile + (size_t)s * kBK * 2);
  };
  // One slab: multiply slab s out of `cur` while `regs` (slab s + 1) is converted into `nxt` in the shadow of the
  // MFMAs (harmless when there is no slab s + 1), then refill `regs` with slab s + 3 (the last slab again near the end).  After the closing barrier
  // every wavefront is done with `cur` and `nxt` is complete.
  auto step = [&](char* cur, char* nxt, SlabRegs<NJ>& regs, int s) {
    Frags f[2];
    read_frags(f[0], cur, 2 * kg);
    read_frags(f[1], cur, 2 * kg + 1);
    mfmas(f[0]);
    store_a_chunk<NJ>(regs, 0, nxt, a_at);
#pragma unroll
    for (int i = 0; i < NJ; i += 2) store_b_chunk<NJ>(regs, i, nxt, b_at);
    mfmas(f[1]);
    store_a_chunk<NJ>(regs, 1, nxt, a_at);
#pragma unroll
    for (int i = 1; i < NJ; i += 2) store_b_chunk<NJ>(regs, i, nxt, b_at);
    load(regs, min(s + 3, nfast - 1));   // unconditional, so that the count of loads in flight is the same on every path
    __syncthreads();
  };
  if (nfast > 0) {
    SlabRegs<NJ> r0, r1;
    load(r0, 0);
    load(r1, nfast > 1 ? 1 : 0);
#pragma unroll
    for (int i = 0; i < 2; ++i) store_a_chunk<NJ>(r0, i, lds, a_at);
#pragma unroll
    for (int i = 0; i < NJ; ++i) store_b_chunk<NJ>(r0, i, lds, b_at);
    load(r0, min(2, nfast - 1));
    __syncthreads();
    int s = 0;
    for (; s + 2 <= nfast; s += 2) {
      step(lds, lds + kStage, r1, s);          // stage 0 holds slab s; r1 holds slab s + 1
      step(lds + kStage, lds, r0, s + 1);      // stage 1 holds slab s + 1; r0 holds slab s + 2
    }
    if (s < nfast) step(lds, lds + kStage, r1, s);
  }

  // The rest (a ragged last slab, or every slab of an unaligned problem): one slab at a time, guarded loads.
  const int slabs = (K + kBK - 1) / kBK;
  for (int s = nfast; s < slabs; ++s) {
    SlabRegs<NJ> regs;
    load_slab_any<NJ>(regs, X, W, tid, m0, n0, s * kBK, M, N, K);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) store_a_chunk<NJ>(regs, i, lds, a_at);
#pragma unroll
    for (int i = 0; i < NJ; ++i) store_b_chunk<NJ>(regs, i, lds, b_at);
    __syncthreads();
    multiply(lds, 2 * kg);
    multiply(lds, 2 * kg + 1);
  }

  // The two halves of k meet: the wavefronts of the upper half hand their sums over through LDS.
  __syncthreads();
  float* const handover = reinterpret_cast<float*>(lds) + (size_t)(wave & 3) * NJ * 16 * 64;
  if (kg == 1) {
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) handover[(j * 16 + v) * 64 + lane] = acc_hi[j][v] + acc_lo[j][v] * (1.0f / kLoScale);
  }
  __syncthreads();
  if (kg == 1) return;

  // Accumulator element v of lane (r, kh) is row 8 (v / 4) + 4 kh + v % 4, column r of its 32 x 32 tile.
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int n = n0 + wn * 32 * NJ + j * 32 + r;
    if (n >= N) continue;
    const float bn = bias ? bias[n] : 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = m0 + wm * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
      if (m < M) out[(size_t)m * N + n] = ((acc_hi[j][v] + acc_lo[j][v] * (1.0f / kLoScale)) + handover[(j * 16 + v) * 64 + lane]) + bn;
    }
  }
}

}  // namespace

hipError_t launch_project(const float* x, const uint16_t* w, const float* bias, float* out, int M, int N, int K,
                          hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
  if (K > (1 << 23)) return hipErrorInvalidValue;   // 32-bit byte offsets inside a tile
  const int vec = (K % 8 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (reinterpret_cast<uintptr_t>(w) % 16 == 0);
  const int tiles_m = (M + kBM - 1) / kBM;
  // Tile width 64 NJ (SPRNN_PROJECT_TILE=64|128|192 overrides the choice for experiments).
  static const int force = std::getenv("SPRNN_PROJECT_TILE") ? std::atoi(std::getenv("SPRNN_PROJECT_TILE")) : 0;
  int cus = 256;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  static int cu_count[64] = {};
  if (dev >= 0 && dev < 64) {
    if (!cu_count[dev]) {
      hipDeviceProp_t prop;
      if (hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0) cu_count[dev] = prop.multiProcessorCount;
      else cu_count[dev] = 256;
    }
    cus = cu_count[dev];
  }
  int nj = 2;
  if (force) {
    nj = force / 64;
  } else {
    // Measured on four layer shapes: 128-wide tiles are the best all-rounder; 192-wide ones win when the 128-wide
    // tiles are a little more than one per CU (every CU would otherwise wait for the few that carry two) and the
    // wider ones fit one per CU; 64-wide ones only serve outputs that are no wider.
    const long long t2 = (long long)tiles_m * ((N + 127) / 128), t3 = (long long)tiles_m * ((N + 191) / 192);
    if (N <= 64) nj = 1;
    else if (t2 > cus && 2 * t2 <= 3LL * cus && t3 <= cus) nj = 3;
  }
  if (nj < 1 || nj > 3) return hipErrorInvalidValue;
  const long long tiles = (long long)tiles_m * ((N + 64 * nj - 1) / (64 * nj));
  if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
  // Two LDS stages of the wider kernels exceed the 64 KB a launch may ask for by default: raise the limit once per device.
  static bool raised[64][4] = {};
  const void* kernels[4] = {nullptr, (const void*)project_kernel<1>, (const void*)project_kernel<2>, (const void*)project_kernel<3>};
  const int lds = 2 * stage_bytes(nj);
  if (lds > 65536 && dev >= 0 && dev < 64 && !raised[dev][nj]) {
    e = hipFuncSetAttribute(kernels[nj], hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    raised[dev][nj] = true;
  }
  void* args[] = {(void*)&x, (void*)&w, (void*)&bias, (void*)&out, (void*)&M, (void*)&N, (void*)&K, (void*)&tiles_m, (void*)&vec};
  e = hipLaunchKernel(kernels[nj], dim3((unsigned)tiles), dim3(kThreads), args, (size_t)lds, stream);
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace sprnn
