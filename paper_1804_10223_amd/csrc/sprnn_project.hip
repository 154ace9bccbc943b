// Input projection b'[m][n] = sum_k x[m][k] * W[n][k] + bias[n] on the matrix cores of gfx950.
//
// Section 3.1 of the paper turns Eq. 1 into Eq. 2 by computing the input term W x_t + b for all timesteps
// ahead of the recurrence.  That term is one dense product over M = T * B input vectors; both operands are
// contiguous along k, so a wavefront's MFMA fragments (8 consecutive k of one row per lane) are 16-byte reads.
//
// Precision: W is binary16 (exact in the MFMA), x is binary32.  Each x is split once, while it is staged into
// LDS, into hi = fp16(x) and lo = fp16((x - hi) * 2^11); hi + lo / 2^11 carries 22 significant bits of x.  The
// two halves go through v_mfma_f32_32x32x16_f16 with separate binary32 accumulators that are combined in the
// epilogue, so products are exact and every sum is binary32.  The scale keeps lo a normal binary16 number
// whenever x is, and hi is forced to zero where it would be subnormal, so the result does not depend on how
// the matrix cores treat subnormal inputs.  |x| must stay below the binary16 maximum (65504).
//
// Tiling: a workgroup of four wavefronts owns a 64 (m) x 128 (n) tile of b' and walks k in slabs of 64; each
// wavefront owns 32 x 64 of it (two 32x32 MFMA tiles, hi and lo accumulators each).  The next slab is fetched
// into registers while the current one is multiplied out of LDS.  LDS rows are padded by 16 bytes so that the
// eight lanes served in one LDS pass touch all banks.  Consecutive tiles of one n block (the same rows of W)
// are dealt to workgroups that share an XCD, hence an L2.
#include "sprnn_device.h"

namespace sprnn {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 64;                 // rows of x (time x batch) per workgroup tile
constexpr int kBN = 128;                // rows of W (outputs) per workgroup tile
constexpr int kBK = 64;                 // k per slab
constexpr int kRowHalfs = kBK + 8;      // LDS row pitch: 144 bytes
constexpr int kThreads = 256;
constexpr float kLoScale = 2048.0f;
constexpr float kMinNormalHalf = 6.103515625e-05f;

struct SlabRegs {
  float4 a[4];   // 4 x (4 consecutive k of one x row)
  uint4 b[4];    // 4 x (8 consecutive k of one W row, binary16 bits)
};

__device__ __forceinline__ void load_slab(SlabRegs& r, const float* __restrict__ X, const uint16_t* __restrict__ W, int tid,
                                          int m0, int n0, int k0, int M, int N, int K, bool a_vec, bool b_vec) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + kThreads * i;
    const int row = min(m0 + (c >> 4), M - 1);
    const int k = k0 + (c & 15) * 4;
    const float* src = X + (size_t)row * K + k;
    if (a_vec && k + 4 <= K) {
      r.a[i] = *reinterpret_cast<const float4*>(src);
    } else {
      r.a[i].x = (k + 0 < K) ? src[0] : 0.0f;
      r.a[i].y = (k + 1 < K) ? src[1] : 0.0f;
      r.a[i].z = (k + 2 < K) ? src[2] : 0.0f;
      r.a[i].w = (k + 3 < K) ? src[3] : 0.0f;
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + kThreads * i;
    const int row = min(n0 + (c >> 3), N - 1);
    const int k = k0 + (c & 7) * 8;
    const uint16_t* src = W + (size_t)row * K + k;
    if (b_vec && k + 8 <= K) {
      r.b[i] = *reinterpret_cast<const uint4*>(src);
    } else {
      uint32_t h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = (k + e < K) ? (uint32_t)src[e] : 0u;
      r.b[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
  }
}

__device__ __forceinline__ void split(float x, _Float16& hi, _Float16& lo) {
  hi = (fabsf(x) >= kMinNormalHalf) ? (_Float16)x : (_Float16)0.0f;
  lo = (_Float16)((x - (float)hi) * kLoScale);
}

__device__ __forceinline__ void store_slab(const SlabRegs& r, _Float16* a_hi, _Float16* a_lo, _Float16* b_s, int tid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + kThreads * i;
    const int at = (c >> 4) * kRowHalfs + (c & 15) * 4;
    half4 hi, lo;
    _Float16 h, l;
    split(r.a[i].x, h, l); hi[0] = h; lo[0] = l;
    split(r.a[i].y, h, l); hi[1] = h; lo[1] = l;
    split(r.a[i].z, h, l); hi[2] = h; lo[2] = l;
    split(r.a[i].w, h, l); hi[3] = h; lo[3] = l;
    *reinterpret_cast<half4*>(a_hi + at) = hi;
    *reinterpret_cast<half4*>(a_lo + at) = lo;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + kThreads * i;
    *reinterpret_cast<uint4*>(b_s + (c >> 3) * kRowHalfs + (c & 7) * 8) = r.b[i];
  }
}

__global__ __launch_bounds__(kThreads) void project_kernel(const float* __restrict__ X, const uint16_t* __restrict__ W,
                                                           const float* __restrict__ bias, float* __restrict__ out,
                                                           int M, int N, int K, int tiles_m, int a_vec, int b_vec) {
  __shared__ __attribute__((aligned(16))) _Float16 a_hi[kBM * kRowHalfs];
  __shared__ __attribute__((aligned(16))) _Float16 a_lo[kBM * kRowHalfs];
  __shared__ __attribute__((aligned(16))) _Float16 b_s[kBN * kRowHalfs];

  // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles.
  const int nb = gridDim.x, bid = blockIdx.x;
  const int id = (nb % 8 == 0) ? (bid % 8) * (nb / 8) + bid / 8 : bid;
  const int m0 = (id % tiles_m) * kBM, n0 = (id / tiles_m) * kBN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int r = lane & 31, kh = lane >> 5;
  const _Float16* a_hi_row = a_hi + (wm * 32 + r) * kRowHalfs + kh * 8;
  const _Float16* a_lo_row = a_lo + (wm * 32 + r) * kRowHalfs + kh * 8;
  const _Float16* b_row = b_s + (wn * 64 + r) * kRowHalfs + kh * 8;

  floatx16 acc_hi[2], acc_lo[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc_hi[j][v] = 0.0f; acc_lo[j][v] = 0.0f; }

  SlabRegs regs;
  const int slabs = (K + kBK - 1) / kBK;
  load_slab(regs, X, W, tid, m0, n0, 0, M, N, K, a_vec != 0, b_vec != 0);
  for (int s = 0; s < slabs; ++s) {
    __syncthreads();   // every wavefront is done with the previous slab
    store_slab(regs, a_hi, a_lo, b_s, tid);
    __syncthreads();
    if (s + 1 < slabs) load_slab(regs, X, W, tid, m0, n0, (s + 1) * kBK, M, N, K, a_vec != 0, b_vec != 0);
#pragma unroll
    for (int q = 0; q < kBK / 16; ++q) {
      const half8 ah = *reinterpret_cast<const half8*>(a_hi_row + q * 16);
      const half8 al = *reinterpret_cast<const half8*>(a_lo_row + q * 16);
      const half8 b0 = *reinterpret_cast<const half8*>(b_row + q * 16);
      const half8 b1 = *reinterpret_cast<const half8*>(b_row + 32 * kRowHalfs + q * 16);
      acc_hi[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, b0, acc_hi[0], 0, 0, 0);
      acc_hi[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, b1, acc_hi[1], 0, 0, 0);
      acc_lo[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, b0, acc_lo[0], 0, 0, 0);
      acc_lo[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, b1, acc_lo[1], 0, 0, 0);
    }
  }

  // Accumulator element v of lane (r, kh) is row 8 (v / 4) + 4 kh + v % 4, column r of its 32 x 32 tile.
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + j * 32 + r;
    if (n >= N) continue;
    const float bn = bias ? bias[n] : 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = m0 + wm * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
      if (m < M) out[(size_t)m * N + n] = (acc_hi[j][v] + acc_lo[j][v] * (1.0f / kLoScale)) + bn;
    }
  }
}

}  // namespace

hipError_t launch_project(const float* x, const uint16_t* w, const float* bias, float* out, int M, int N, int K,
                          hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  const long long tiles = (long long)tiles_m * tiles_n;
  if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
  const int a_vec = (K % 4 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
  const int b_vec = (K % 8 == 0) && (reinterpret_cast<uintptr_t>(w) % 16 == 0);
  hipLaunchKernelGGL(project_kernel, dim3((unsigned)tiles), dim3(kThreads), 0, stream, x, w, bias, out, M, N, K, tiles_m,
                     a_vec, b_vec);
  return hipGetLastError();
}

}  // namespace sprnn
