// Device code of libsprnn: the persistent sparse recurrent kernel and the per-timestep comparison kernel.
//
// Persistent kernel (paper, Section 3.3): every lane loads its packed <index,value> words into registers
// once; h_{t-1} lives in LDS; per timestep the pipeline is  load -> operate -> reduce -> hand-off.
//   load     every workgroup copies the whole h_{t-1} from the exchange ring into its LDS, polling until
//            every 32-bit element differs from the "not written" mark (-0.0f, Section 4.2's flag-free
//            Lamport scheme).  The ring has 4 slots; the slot index is the timestep tag (t mod 4).
//   operate  acc[b] += fp32(value) * h_lds[index][b], one wide LDS gather per word (Section 4.1)
//   reduce   lanes that share a row combine with DPP / swizzle butterflies (no LDS round trip)
//   hand-off the row's leader lane adds b'_t, applies g, publishes to the ring slot of step t with
//            agent-coherent stores, writes h_out, and re-arms its part of the slot two steps ahead.
// No grid barrier is needed in the tagged mode; SPRNN_SYNC_BARRIER keeps the paper's baseline
// (Section 3.2, "Synchronize") for comparison.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "sprnn_device.h"

namespace sprnn {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kAuxCoherent = 16;   // sc1: agent-scope coherent access (misses the per-CU vector cache)
constexpr unsigned kBufWord3 = 0x00027000u;

__device__ __forceinline__ float half_bits_to_float(uint32_t w) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
  return v + __builtin_bit_cast(float, moved);
}

// Sum over the L consecutive lanes (L a power of two, aligned) that share a row; every lane gets the total.
__device__ __forceinline__ float group_sum(float v, int L, int lane) {
  if (L >= 2) v = dpp_add<0xB1>(v);     // quad_perm [1,0,3,2]
  if (L >= 4) v = dpp_add<0x4E>(v);     // quad_perm [2,3,0,1]
  if (L >= 8) v = dpp_add<0x141>(v);    // row_half_mirror: the other quad of the octet
  if (L >= 16) v = dpp_add<0x140>(v);   // row_mirror: the other octet of the row of 16
  if (L >= 32) v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));  // lane ^ 16
  if (L >= 64) v += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, v)));
  return v;
}

__device__ __forceinline__ float activate(int act, float pre) {
  float h;
  if (act == SPRNN_ACT_RELU) h = fmaxf(pre, 0.0f);
  else if (act == SPRNN_ACT_TANH) h = tanhf(pre);
  else h = pre;
  return h + 0.0f;   // -0.0 -> +0.0: -0.0 is reserved as the "not written" mark
}

__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + expf(-z)); }

__device__ __forceinline__ bool all_written(i32x4 v) {
  return ((uint32_t)v.x != kSentinelBits) & ((uint32_t)v.y != kSentinelBits) & ((uint32_t)v.z != kSentinelBits) &
         ((uint32_t)v.w != kSentinelBits);
}

// LDS byte offset of h[col j][sample b]
template <int B>
__device__ __forceinline__ int lds_offset(int j, int b, int H) {
  if (B == 8) return (b >> 2) * H * 16 + j * 16 + (b & 3) * 4;
  return (j * B + b) * 4;
}

template <int B>
__device__ __forceinline__ void mac_word(float (&acc)[B], uint32_t w, const unsigned char* hb, int plane_bytes) {
  const uint32_t off = w >> 16;
  const float wv = half_bits_to_float(w);
  if constexpr (B == 1) {
    const float h = *reinterpret_cast<const float*>(hb + off);
    acc[0] = fmaf(wv, h, acc[0]);
  } else if constexpr (B == 2) {
    const f32x2 h = *reinterpret_cast<const f32x2*>(hb + off);
    acc[0] = fmaf(wv, h.x, acc[0]);
    acc[1] = fmaf(wv, h.y, acc[1]);
  } else if constexpr (B == 4) {
    const f32x4 h = *reinterpret_cast<const f32x4*>(hb + off);
    acc[0] = fmaf(wv, h.x, acc[0]);
    acc[1] = fmaf(wv, h.y, acc[1]);
    acc[2] = fmaf(wv, h.z, acc[2]);
    acc[3] = fmaf(wv, h.w, acc[3]);
  } else {
    const f32x4 h0 = *reinterpret_cast<const f32x4*>(hb + off);
    const f32x4 h1 = *reinterpret_cast<const f32x4*>(hb + plane_bytes + off);
    acc[0] = fmaf(wv, h0.x, acc[0]);
    acc[1] = fmaf(wv, h0.y, acc[1]);
    acc[2] = fmaf(wv, h0.z, acc[2]);
    acc[3] = fmaf(wv, h0.w, acc[3]);
    acc[4] = fmaf(wv, h1.x, acc[4]);
    acc[5] = fmaf(wv, h1.y, acc[5]);
    acc[6] = fmaf(wv, h1.z, acc[6]);
    acc[7] = fmaf(wv, h1.w, acc[7]);
  }
}

// Publish the B outputs of one row into a ring slot (same layout as the LDS copy of h).
template <int B>
__device__ __forceinline__ void ring_store(__amdgpu_buffer_rsrc_t ring, int slot_byte, int row, int H, const float (&v)[B]) {
  if constexpr (B == 1) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v[0]), ring, slot_byte + row * 4, 0, kAuxCoherent);
  } else if constexpr (B == 2) {
    i32x2 p = {__builtin_bit_cast(int, v[0]), __builtin_bit_cast(int, v[1])};
    __builtin_amdgcn_raw_buffer_store_b64(p, ring, slot_byte + row * 8, 0, kAuxCoherent);
  } else if constexpr (B == 4) {
    i32x4 p = {__builtin_bit_cast(int, v[0]), __builtin_bit_cast(int, v[1]), __builtin_bit_cast(int, v[2]), __builtin_bit_cast(int, v[3])};
    __builtin_amdgcn_raw_buffer_store_b128(p, ring, slot_byte + row * 16, 0, kAuxCoherent);
  } else {
    i32x4 p = {__builtin_bit_cast(int, v[0]), __builtin_bit_cast(int, v[1]), __builtin_bit_cast(int, v[2]), __builtin_bit_cast(int, v[3])};
    i32x4 q = {__builtin_bit_cast(int, v[4]), __builtin_bit_cast(int, v[5]), __builtin_bit_cast(int, v[6]), __builtin_bit_cast(int, v[7])};
    __builtin_amdgcn_raw_buffer_store_b128(p, ring, slot_byte + row * 16, 0, kAuxCoherent);
    __builtin_amdgcn_raw_buffer_store_b128(q, ring, slot_byte + H * 16 + row * 16, 0, kAuxCoherent);
  }
}

template <int B, int NW, bool LSTM>
__global__ __launch_bounds__(NW >= 48 ? 512 : 1024) void persistent_kernel(const KernelArgs p) {
  extern __shared__ __align__(16) unsigned char lds[];   // [h copy 0][h copy 1][abort flags]
  // abort flags, indexed by step parity so that a fast wave's next-step flag cannot be read one step early
  volatile int* s_abort = reinterpret_cast<volatile int*>(lds + 2 * p.h_bytes);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int block = blockDim.x, wg = blockIdx.x;
  const int H = p.hidden, L = p.lanes_per_row;
  const int R = LSTM ? 4 * H : H;
  const int plane_bytes = H * 16;   // used only for B == 8

  // ---- one-time weight load: NW register slots per lane, all of one row (Section 3.3)
  const int n_w = __builtin_amdgcn_readfirstlane(p.wave_words[wg * (block >> 6) + wave]);
  uint32_t w[NW];
#pragma unroll
  for (int k = 0; k < NW; ++k) w[k] = (k < n_w) ? p.words[((size_t)wg * NW + k) * block + tid] : 0u;
  const int row = p.lane_row[(size_t)wg * block + tid];
  const bool group_leader = row >= 0 && (lane & (L - 1)) == 0;
  const bool unit_leader = LSTM ? (row >= 0 && (lane & (4 * L - 1)) == 0) : group_leader;
  const int unit = LSTM ? (row >= 0 ? row % H : 0) : row;   // hidden-unit index of the row

  __amdgpu_buffer_rsrc_t ring = __builtin_amdgcn_make_buffer_rsrc(p.ring, 0, kRingSlotsDev * p.h_bytes, kBufWord3);
  __amdgpu_buffer_rsrc_t ctrl = __builtin_amdgcn_make_buffer_rsrc(p.ctrl, 0, 256, kBufWord3);

  // ---- h_0 into LDS copy 0, cell state into registers
  if (tid == 0) { s_abort[0] = 0; s_abort[1] = 0; }
  for (int e = tid; e < H * B; e += block) {
    const int j = e / B, b = e % B;
    const float v = p.h0 ? p.h0[(size_t)b * H + j] : 0.0f;
    *reinterpret_cast<float*>(lds + lds_offset<B>(j, b, H)) = v;
  }
  float c_state[B];
#pragma unroll
  for (int b = 0; b < B; ++b) c_state[b] = (LSTM && unit_leader && p.c0) ? p.c0[(size_t)b * H + unit] : 0.0f;
  __syncthreads();

  int cur = 0;
  bool failed = false;
  for (int t = 0; t < p.T; ++t) {
    const uint32_t g = p.step_base + (uint32_t)t;         // global step index: the slot number is the timestep tag
    const int slot_byte = (int)(g & (kRingSlotsDev - 1)) * p.h_bytes;
    const int rearm_byte = (int)((g + 2) & (kRingSlotsDev - 1)) * p.h_bytes;

    // b'_t of this row, fetched early so the loads overlap the operate stage
    float xv[B];
#pragma unroll
    for (int b = 0; b < B; ++b) xv[b] = group_leader ? p.x[((size_t)t * B + b) * R + row] : 0.0f;

    // ---- operate: n_w gathers, in groups of four so the LDS reads are issued back to back
    const unsigned char* hb = lds + cur * p.h_bytes;
    float acc[B];
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = 0.0f;
#pragma unroll
    for (int k = 0; k < NW; k += 4) {
      if (k + 4 <= n_w) {
        mac_word<B>(acc, w[k], hb, plane_bytes);
        mac_word<B>(acc, w[k + 1], hb, plane_bytes);
        mac_word<B>(acc, w[k + 2], hb, plane_bytes);
        mac_word<B>(acc, w[k + 3], hb, plane_bytes);
      } else if (k < n_w) {   // ragged tail of 1..3 words (no early exit: keeps every w[] index static)
        mac_word<B>(acc, w[k], hb, plane_bytes);
        if (k + 1 < n_w) mac_word<B>(acc, w[k + 1], hb, plane_bytes);
        if (k + 2 < n_w) mac_word<B>(acc, w[k + 2], hb, plane_bytes);
      }
    }

    // ---- reduce over the lanes of the row
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = group_sum(acc[b], L, lane);

    // ---- epilogue + hand-off
    float hv[B];
    if constexpr (LSTM) {
      float pg[4][B];
#pragma unroll
      for (int b = 0; b < B; ++b) {
        const float pre = acc[b] + xv[b];   // complete pre-activation sits in each gate's group leader
#pragma unroll
        for (int q = 0; q < 4; ++q)
          pg[q][b] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane + q * L) << 2, __builtin_bit_cast(int, pre)));
      }
#pragma unroll
      for (int b = 0; b < B; ++b) {
        const float c = sigmoidf_(pg[1][b]) * c_state[b] + sigmoidf_(pg[0][b]) * tanhf(pg[2][b]);
        c_state[b] = c;
        hv[b] = sigmoidf_(pg[3][b]) * tanhf(c) + 0.0f;
      }
    } else {
#pragma unroll
      for (int b = 0; b < B; ++b) hv[b] = activate(p.act, acc[b] + xv[b]);
    }
    if (unit_leader) {
      // the re-arm stores issued one step ago must be performed before this step's data can be seen
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      ring_store<B>(ring, slot_byte, unit, H, hv);
#pragma unroll
      for (int b = 0; b < B; ++b) {
        __builtin_nontemporal_store(hv[b], &p.h_out[((size_t)t * B + b) * H + unit]);
        if constexpr (LSTM) __builtin_nontemporal_store(c_state[b], &p.c_out[((size_t)t * B + b) * H + unit]);
      }
      if (p.sync == SPRNN_SYNC_TAGGED) {
        float mark[B];
#pragma unroll
        for (int b = 0; b < B; ++b) mark[b] = __builtin_bit_cast(float, kSentinelBits);
        ring_store<B>(ring, rearm_byte, unit, H, mark);
      }
    }
    if (t + 1 == p.T) break;

    // ---- load h_t for the next step into the other LDS copy
    unsigned char* dst = lds + (cur ^ 1) * p.h_bytes;
    const int n4 = p.h_bytes >> 4;
    if (p.sync == SPRNN_SYNC_BARRIER) {
      // grid barrier (Section 3.2): all stores performed, one arrival per workgroup, wait for everyone
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (tid == 0) {
        __hip_atomic_fetch_add(p.ctrl + kCtrlBarrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t target = p.barrier_base + (uint32_t)(t + 1) * (uint32_t)gridDim.x;
        int spins = 0;
        for (;;) {
          const uint32_t seen = __hip_atomic_load(p.ctrl + kCtrlBarrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if ((int)(seen - target) >= 0) break;
          if (++spins > p.spin_limit || ((spins & 1023) == 0 && __hip_atomic_load(p.ctrl + kCtrlStatus, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
            failed = true;
            break;
          }
        }
      }
      __syncthreads();
      for (int ci = tid; ci < n4; ci += block) {
        const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(ring, slot_byte + ci * 16, 0, kAuxCoherent);
        *reinterpret_cast<i32x4*>(dst + ci * 16) = v;
      }
    } else {
      for (int d = 0; d < p.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
      for (int base = tid; base < n4; base += 4 * block) {
        i32x4 v[4];
        bool ok[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int ci = base + c * block;
          ok[c] = ci >= n4;
          if (!ok[c]) v[c] = __builtin_amdgcn_raw_buffer_load_b128(ring, slot_byte + ci * 16, 0, kAuxCoherent);
        }
        int spins = 0;
        for (;;) {
          bool all = true;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if (!ok[c]) {
              if (all_written(v[c])) ok[c] = true;
              else all = false;
            }
          }
          if (all) break;
          ++spins;
          if (spins > p.spin_limit ||
              ((spins & 1023) == 0 && __builtin_amdgcn_raw_buffer_load_b32(ctrl, kCtrlStatus * 4, 0, kAuxCoherent) != 0)) {
            failed = true;
            break;
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int ci = base + c * block;
            if (!ok[c]) v[c] = __builtin_amdgcn_raw_buffer_load_b128(ring, slot_byte + ci * 16, 0, kAuxCoherent);
          }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int ci = base + c * block;
          if (ci < n4) *reinterpret_cast<i32x4*>(dst + ci * 16) = v[c];
        }
        if (failed) break;
      }
    }
    if (failed) {
      s_abort[t & 1] = 1;
      __hip_atomic_store(p.ctrl + kCtrlStatus, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (s_abort[t & 1]) break;   // every wave of the workgroup leaves together; other workgroups see the status word
    cur ^= 1;
  }
}

// ------------------------------------------------------------------------------------------------
// Per-timestep comparison kernel: one launch per step, CSR weights re-read from device memory,
// one wavefront per weight row (vanilla) or per hidden unit (LSTM: its four gate rows in turn).
template <int B, bool LSTM>
__global__ __launch_bounds__(256) void stepwise_kernel(const StepArgs p) {
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int H = p.hidden;
  if (unit >= H) return;
  constexpr int G = LSTM ? 4 : 1;
  float pre[G][B];
#pragma unroll
  for (int q = 0; q < G; ++q) {
    const int row = q * H + unit;
    float acc[B];
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = 0.0f;
    for (int k = p.row_ptr[row] + lane; k < p.row_ptr[row + 1]; k += 64) {
      const float wv = half_bits_to_float(p.val[k]);
      const int c = p.col[k];
#pragma unroll
      for (int b = 0; b < B; ++b) acc[b] = fmaf(wv, p.h_prev ? p.h_prev[(size_t)b * H + c] : 0.0f, acc[b]);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
      float v = acc[b];
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
      pre[q][b] = v + p.x_t[(size_t)b * (G * H) + row];
    }
  }
  if (lane != 0) return;
#pragma unroll
  for (int b = 0; b < B; ++b) {
    if constexpr (LSTM) {
      const float cp = p.c_prev ? p.c_prev[(size_t)b * H + unit] : 0.0f;
      const float c = sigmoidf_(pre[1][b]) * cp + sigmoidf_(pre[0][b]) * tanhf(pre[2][b]);
      p.c_cur[(size_t)b * H + unit] = c;
      p.h_cur[(size_t)b * H + unit] = sigmoidf_(pre[3][b]) * tanhf(c) + 0.0f;
    } else {
      p.h_cur[(size_t)b * H + unit] = activate(p.act, pre[0][b]);
    }
  }
}

// Fill a device buffer with one 32-bit pattern (used instead of a memset node so that callers may capture it).
__global__ void fill_kernel(uint32_t* dst, uint32_t value, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = value;
}

// ------------------------------------------------------------------------------------------------
template <int B, bool LSTM>
static const void* pick_nw(int nw) {
  switch (nw) {
    case 8: return (const void*)persistent_kernel<B, 8, LSTM>;
    case 16: return (const void*)persistent_kernel<B, 16, LSTM>;
    case 24: return (const void*)persistent_kernel<B, 24, LSTM>;
    case 32: return (const void*)persistent_kernel<B, 32, LSTM>;
    case 48: return (const void*)persistent_kernel<B, 48, LSTM>;
    case 64: return (const void*)persistent_kernel<B, 64, LSTM>;
    default: return nullptr;
  }
}

template <bool LSTM>
static const void* pick_b(int batch, int nw) {
  switch (batch) {
    case 1: return pick_nw<1, LSTM>(nw);
    case 2: return pick_nw<2, LSTM>(nw);
    case 4: return pick_nw<4, LSTM>(nw);
    case 8: return pick_nw<8, LSTM>(nw);
    default: return nullptr;
  }
}

const void* persistent_kernel_for(int batch, int template_words, bool lstm) {
  return lstm ? pick_b<true>(batch, template_words) : pick_b<false>(batch, template_words);
}

hipError_t launch_stepwise(int batch, bool lstm, const StepArgs& a, hipStream_t stream) {
  const int waves_per_block = 4;
  dim3 grid((a.hidden + waves_per_block - 1) / waves_per_block), block(waves_per_block * 64);
#define SPRNN_LAUNCH_STEP(BB)                                                                          \
  if (lstm) hipLaunchKernelGGL((stepwise_kernel<BB, true>), grid, block, 0, stream, a);              \
  else hipLaunchKernelGGL((stepwise_kernel<BB, false>), grid, block, 0, stream, a);
  switch (batch) {
    case 1: SPRNN_LAUNCH_STEP(1) break;
    case 2: SPRNN_LAUNCH_STEP(2) break;
    case 4: SPRNN_LAUNCH_STEP(4) break;
    case 8: SPRNN_LAUNCH_STEP(8) break;
    default: return hipErrorInvalidValue;
  }
#undef SPRNN_LAUNCH_STEP
  return hipGetLastError();
}

hipError_t launch_fill(uint32_t* dst, uint32_t value, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const int block = 256;
  const int grid = (int)((n + block - 1) / block < 1024 ? (n + block - 1) / block : 1024);
  hipLaunchKernelGGL(fill_kernel, dim3(grid), dim3(block), 0, stream, dst, value, n);
  return hipGetLastError();
}

}  // namespace sprnn
