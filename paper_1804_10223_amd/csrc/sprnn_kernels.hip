// Device code of libsprnn: the forward instantiations of the persistent kernel (sprnn_persistent.h), the weight
// gradient kernel, the per-timestep comparison kernel and small helpers.
#include <algorithm>

#include "sprnn_persistent.h"

namespace sprnn {

// ------------------------------------------------------------------------------------------------
// Weight gradient on the sparsity pattern (the non-recurrent half of the backward pass): the forward mapping
// turned around.  A lane keeps one ACCUMULATOR per nonzero it holds in the forward pass, resident in registers for
// all T steps; per step every workgroup brings h_{t-1} into LDS in the forward layout, a lane gathers the column of
// each of its nonzeros (the same wide reads, the same bank-aware order) and adds delta_t[b][row] * h_{t-1}[b][col].
// Workgroups do not talk to each other; the sums leave through the packer's word -> CSR position map.
template <int B, int NW>
__global__ __launch_bounds__(NW >= 48 ? 256 : 768) void weight_grad_kernel(const WGradArgs p) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int block = blockDim.x, wg = blockIdx.x, H = p.hidden;
  const int n_w = __builtin_amdgcn_readfirstlane(p.wave_words[wg * (block >> 6) + wave]);
  const int plane_bytes = H * 16;
  uint32_t w_off[NW];
  float acc[NW];
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    const uint32_t word = (k < n_w) ? p.words[((size_t)wg * NW + k) * block + tid] : 0u;
    w_off[k] = lds_address(lds) + ((word >> 16) << p.index_shift);
    acc[k] = 0.0f;
  }
  const int row = p.lane_row[(size_t)wg * block + tid];
  (void)lane;
  // [B][H] in memory -> [H][B] in LDS (two planes of four samples for B = 8): a lane assembles whole 16-byte LDS
  // chunks from four coalesced 4-byte loads each, sixteen loads in flight, and writes them as consecutive b128.
  // The first four chunks of a lane (all of them up to 16 KB x waves of h) and its delta values are fetched one step
  // ahead, while the gathers of the current step run.
  constexpr int bb = B < 4 ? B : 4, cpc = 4 / bb;
  const int per_plane = (H + cpc - 1) / cpc, chunks = (B == 8 ? 2 : 1) * per_plane;
  auto h_before = [&](int t) { return t ? p.h_fwd + (size_t)(t - 1) * B * H : p.h0; };
  // Element offsets of a lane's chunks are fixed for the whole launch: chunk c holds columns cc * cpc .. of samples
  // pl * 4 ..; element e of it sits (e % bb) rows of H and e / bb columns further.  When H is not a multiple of the
  // columns per chunk (batch 1 or 2 only) the last chunk is ragged and every element is checked instead.
  const bool whole_chunks = H % cpc == 0;
  auto chunk_offsets = [&](uint32_t (&goff)[4], uint32_t (&loff)[4], int c0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = min(c0 + i * block, chunks - 1);   // clamped: the last chunk may be copied twice
      const int pl = c / per_plane, cc = c % per_plane;
      goff[i] = (uint32_t)(pl * 4 * H + cc * cpc);
      loff[i] = (uint32_t)(pl * plane_bytes + cc * 16);
    }
  };
  auto load_chunks = [&](f32x4 (&v)[4], const float* hp, const uint32_t (&goff)[4]) {
    if (hp && !whole_chunks) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t at = goff[i] + (uint32_t)((e % bb) * H + e / bb);
          const int col = (int)(goff[i] % (uint32_t)H) + e / bb;     // goff = sample row * H + first column
          v[i][e] = col < H ? hp[at] : 0.0f;
        }
    } else if (hp) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float* he = hp + (size_t)(e % bb) * H + e / bb;   // wavefront-uniform base, per-lane 32-bit offset
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i][e] = he[goff[i]];
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
  };
  auto store_chunks = [&](const f32x4 (&v)[4], const uint32_t (&loff)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<f32x4*>(lds + loff[i]) = v[i];
  };
  auto load_delta = [&](float (&d)[B], int t) {
#pragma unroll
    for (int b = 0; b < B; ++b) d[b] = row >= 0 ? p.delta[((size_t)t * B + b) * p.rows + row] : 0.0f;
  };
  uint32_t goff0[4], loff0[4];
  chunk_offsets(goff0, loff0, tid);
  f32x4 ahead[4];
  float d_ahead[B];
  if (p.T > 0) {
    load_chunks(ahead, h_before(0), goff0);
    load_delta(d_ahead, 0);
  }
  for (int t = 0; t < p.T; ++t) {
    const float* hp = h_before(t);
    __syncthreads();   // the gathers of the previous step are done
    store_chunks(ahead, loff0);
    for (int c0 = tid + 4 * block; c0 < chunks; c0 += 4 * block) {   // long h: the rest, not fetched ahead
      uint32_t goff[4], loff[4];
      f32x4 v[4];
      chunk_offsets(goff, loff, c0);
      load_chunks(v, hp, goff);
      store_chunks(v, loff);
    }
    float d[B];
#pragma unroll
    for (int b = 0; b < B; ++b) d[b] = d_ahead[b];
    __syncthreads();
    if (t + 1 < p.T) {
      load_chunks(ahead, h_before(t + 1), goff0);
      load_delta(d_ahead, t + 1);
    }
#pragma unroll
    for (int k0 = 0; k0 < NW; k0 += 4) {
      if (k0 < n_w) {   // a group of four slots: slots past n_w read the first column and feed sums that are never stored
        Column<B> c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = gather_column<B>(w_off[k0 + j], plane_bytes);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float s = acc[k0 + j];
          s = fmaf(d[0], c[j].lo.x, s);
          if constexpr (B >= 2) s = fmaf(d[1], c[j].lo.y, s);
          if constexpr (B >= 4) { s = fmaf(d[2], c[j].lo.z, s); s = fmaf(d[3], c[j].lo.w, s); }
          if constexpr (B == 8) {
            s = fmaf(d[4], c[j].hi.x, s); s = fmaf(d[5], c[j].hi.y, s);
            s = fmaf(d[6], c[j].hi.z, s); s = fmaf(d[7], c[j].hi.w, s);
          }
          acc[k0 + j] = s;
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    if (k < n_w) {
      const int src = p.word_src[((size_t)wg * NW + k) * block + tid];
      if (src >= 0) p.dU[src] = acc[k];
    }
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
      const float c = sigmoidf_(pre[1][b]) * cp + sigmoidf_(pre[0][b]) * tanhf_(pre[2][b]);
      p.c_cur[(size_t)b * H + unit] = c;
      p.h_cur[(size_t)b * H + unit] = sigmoidf_(pre[3][b]) * tanhf_(c) + 0.0f;
    } else {
      p.h_cur[(size_t)b * H + unit] = activate(p.act, pre[0][b]);
    }
  }
}

// Fill a device buffer with one 32-bit pattern (used instead of a memset node so that callers may capture it).
__global__ void fill_kernel(uint32_t* dst, uint32_t value, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = value;
}

__global__ void exchange_reset_kernel(uint32_t* ring, size_t slot_words, size_t used_words, int slots, uint32_t* ctrl, int ctrl_words) {
  const size_t first = blockIdx.x * (size_t)blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = first; i < slot_words * (size_t)slots; i += stride) ring[i] = (i % slot_words) < used_words ? kSentinelBits : 0u;
  for (size_t i = first; i < (size_t)ctrl_words; i += stride) ctrl[i] = 0u;
}

// ------------------------------------------------------------------------------------------------
const void* persistent_kernel_for(int batch, int template_words, int cell, bool timeline) {
  const int kind = cell == SPRNN_CELL_LSTM ? 1 : (cell == SPRNN_CELL_GRU ? 2 : 0);
  const bool forward = cell >= SPRNN_ACT_RELU && cell <= SPRNN_CELL_GRU;
  if (timeline) {   // the phase timeline is built for the forward pass of the vanilla and LSTM cells only
    if (!forward || kind == 2) return nullptr;
    return persistent_timeline_kernel_for(batch, template_words, kind == 1);
  }
  if (cell == kCellBackward || cell == kCellBackwardGrad) return persistent_backward_kernel_for(batch, template_words, cell);
  if (!forward) return persistent_gated_backward_kernel_for(batch, template_words, cell);
  if (kind == 2) return pick_b<2, false>(batch, template_words);
  return kind == 1 ? pick_b<1, false>(batch, template_words) : pick_b<0, false>(batch, template_words);
}

template <int B>
static const void* pick_wgrad(int nw) {
  switch (nw) {
    case 8: return (const void*)weight_grad_kernel<B, 8>;
    case 16: return (const void*)weight_grad_kernel<B, 16>;
    case 24: return (const void*)weight_grad_kernel<B, 24>;
    case 32: return (const void*)weight_grad_kernel<B, 32>;
    case 48: return (const void*)weight_grad_kernel<B, 48>;
    case 64: return (const void*)weight_grad_kernel<B, 64>;
    default: return nullptr;
  }
}

const void* weight_grad_kernel_for(int batch, int template_words) {
  switch (batch) {
    case 1: return pick_wgrad<1>(template_words);
    case 2: return pick_wgrad<2>(template_words);
    case 4: return pick_wgrad<4>(template_words);
    case 8: return pick_wgrad<8>(template_words);
    default: return nullptr;
  }
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

hipError_t launch_exchange_reset(uint32_t* ring, size_t slot_words, size_t used_words, int slots, uint32_t* ctrl, int ctrl_words,
                                 hipStream_t stream) {
  const size_t n = std::max(slot_words * (size_t)slots, (size_t)ctrl_words);
  const int block = 256;
  const int grid = (int)std::min<size_t>((n + block - 1) / block, 256);
  hipLaunchKernelGGL(exchange_reset_kernel, dim3(std::max(grid, 1)), dim3(block), 0, stream, ring, slot_words, used_words, slots, ctrl, ctrl_words);
  return hipGetLastError();
}

}  // namespace sprnn
