// Device code of libsprnn: the persistent kernel for the lane-pool layout (vanilla cells: forward pass, backward pass
// through time, backward pass with the weight gradient fused in).
//
// Same method as sprnn_persistent.h (paper, Section 3.3: weights in registers for the whole sequence, h_{t-1} in LDS,
// load -> operate -> reduce -> hand-off per timestep; Section 4.1: wide loads over the batch, bank-aware order;
// Section 4.2: validity travels with the data), with the work of a workgroup divided differently:
//   * GATHERING wavefronts (4 or 7) form a pool of lanes.  A row owns whole groups of `B` lanes out of the pool, as many
//     as its nonzeros need, so a workgroup's nonzeros spread evenly over the SIMDs whatever the row lengths are.  These
//     wavefronts poll and copy h_{t-1} into LDS, gather, multiply-add, reduce inside each group (one sample per lane)
//     and leave the group sums in LDS.  Their only global memory operations are the polls.
//   * OUTPUT wavefronts own (row, sample) pairs: they add up the group sums of their row, add b'_t, apply g, publish to
//     the exchange ring, write h_out, re-arm, and fetch b' one step ahead.
// Why: a wavefront's vector memory operations complete in order, and a workgroup barrier that also orders global
// memory drains them all.  With every wavefront doing every stage, each poll of step t + 1 waited for the stores and the
// b' fetch that the same wavefront had issued at the end of step t (about 0.3 us per step).  Here polls queue behind
// nothing, the two barriers of a step order LDS traffic only, and one wavefront per SIMD carries the arithmetic, so the
// per-wavefront costs of a step (reduction, validity checks, address set-up) are paid 4 times per CU instead of 9.
#ifndef SPRNN_POOL_H_
#define SPRNN_POOL_H_

#include "sprnn_persistent.h"

namespace sprnn {

template <int B>
__device__ __forceinline__ void gather_unit(Column<B> (&c)[4], const uint32_t* off, int plane_bytes) {
#pragma unroll
  for (int j = 0; j < 4; ++j) c[j] = gather_column<B>(off[j], plane_bytes);
}

// The NW words of a lane in units of four, the gathers of two units ahead of the arithmetic in flight: with one gathering
// wavefront per SIMD nothing else hides the LDS latency.  Straight-line code on purpose: NW is the kernel's template
// argument (a multiple of four, the workgroups' largest need), slots a lane does not use hold zero-valued padding that
// points at a harmless column, and no branch depends on the wavefront's own word count, so the compiler's counters of
// outstanding LDS reads stay exact (with a branch per unit it waited for every read in flight before every unit).
// With GRAD every column also feeds the weight-gradient sum of its nonzero (see mac_words).
constexpr int kUnitsAhead = 2;
template <int B, int NW, bool GRAD, int NG>
__device__ __forceinline__ void operate_pipelined(float (&acc)[B], const uint32_t (&w_off)[NW], const float (&w_val)[NW],
                                                  int plane_bytes, float (&g)[NG], const float (&side)[B]) {
  static_assert(NW % 4 == 0, "register slots come in units of four");
  constexpr int U = NW / 4;
  Column<B> buf[kUnitsAhead + 1][4];
#pragma unroll
  for (int u = 0; u < kUnitsAhead && u < U; ++u) gather_unit<B>(buf[u], &w_off[4 * u], plane_bytes);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (u + kUnitsAhead < U) gather_unit<B>(buf[(u + kUnitsAhead) % (kUnitsAhead + 1)], &w_off[4 * (u + kUnitsAhead)], plane_bytes);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      mac_column<B>(acc, w_val[4 * u + j], buf[u % (kUnitsAhead + 1)][j]);
      if constexpr (GRAD) g[4 * u + j] = dot_column<B>(side, buf[u % (kUnitsAhead + 1)][j], g[4 * u + j]);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// D chunks of one lane (first, first + stride, ...; clamped to the last chunk) from a ring slot into the same offsets of
// LDS, all D loads in flight at once.  Every chunk goes to LDS as soon as it is there, checked or not (nobody reads h in
// LDS before the workgroup barrier behind the copy); if any of them still held the "not written" mark, the wavefront
// polls all D again (bounded by spin_limit; a tripped watchdog anywhere ends the wait).  Returns false when the wait was
// given up.
template <int D>
__device__ __forceinline__ bool copy_stream(__amdgpu_buffer_rsrc_t ring, int slot_byte, int first, int stride, int last_chunk,
                                            unsigned char* lds, const KernelArgs& p, unsigned long long& repolls) {
  int off[D];
#pragma unroll
  for (int c = 0; c < D; ++c) off[c] = min(first + c * stride, last_chunk) * 16;
  int spins = 0;
  for (;;) {
    i32x4 v[D];
#pragma unroll
    for (int c = 0; c < D; ++c) v[c] = __builtin_amdgcn_raw_buffer_load_b128(ring, off[c], slot_byte, kAuxCoherent);
    int low = 0x7fffffff;
#pragma unroll
    for (int c = 0; c < D; ++c) {
      low = min(low, min_word(v[c]));
      *reinterpret_cast<i32x4*>(lds + off[c]) = v[c];
    }
    if (__builtin_amdgcn_ballot_w64(low == (int)kSentinelBits) == 0) return true;
    ++spins;
    ++repolls;
    if (spins > p.spin_limit || ((spins & 1023) == 0 && __hip_atomic_load(p.ctrl + kCtrlStatus, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) return false;
  }
}

// `rounds` (1..16, wavefront-uniform) chunks per lane: one straight-line instantiation per count.
__device__ __forceinline__ bool copy_rounds(int rounds, __amdgpu_buffer_rsrc_t ring, int slot_byte, int first, int stride, int last_chunk,
                                            unsigned char* lds, const KernelArgs& p, unsigned long long& repolls) {
#define SPRNN_COPY_CASE(N) case N: return copy_stream<N>(ring, slot_byte, first, stride, last_chunk, lds, p, repolls);
  switch (rounds) {
    SPRNN_COPY_CASE(1) SPRNN_COPY_CASE(2) SPRNN_COPY_CASE(3) SPRNN_COPY_CASE(4) SPRNN_COPY_CASE(5) SPRNN_COPY_CASE(6)
    SPRNN_COPY_CASE(7) SPRNN_COPY_CASE(8) SPRNN_COPY_CASE(9) SPRNN_COPY_CASE(10) SPRNN_COPY_CASE(11) SPRNN_COPY_CASE(12)
    SPRNN_COPY_CASE(13) SPRNN_COPY_CASE(14) SPRNN_COPY_CASE(15)
    default: return copy_stream<16>(ring, slot_byte, first, stride, last_chunk, lds, p, repolls);
  }
#undef SPRNN_COPY_CASE
}

// CELL: 0 = forward pass of a vanilla cell, 3 = its backward pass through time on the transposed matrix, 4 = the same
// with the weight gradient fused in (meanings and arguments as in persistent_kernel).
// TL: phase timeline (sprnn_read_timeline) of gathering wavefront p.tl_wave and of the first output wavefront of every
// workgroup, in wall-clock ticks: [0] back-off, [1] poll + copy, [2] wait for the workgroup after the copy, [3] gathers and
// multiply-adds, [4] reduction inside the groups + group sums to LDS, [5] wait for the workgroup after that; output
// wavefront: [6] adding up the group sums, [7] b', g and the wait before the publish; [8] re-polls, [9] steps.
template <int B, int NW, int CELL, bool TL = false>
__global__ __launch_bounds__(512) void pool_kernel(const KernelArgs p) {
  constexpr bool BWD = CELL == 3 || CELL == 4;
  constexpr bool WGRAD = CELL == 4;
  constexpr int G = B;                               // lanes per group: after the in-group reduction a lane holds one sample
  const int steps = BWD ? p.T + ((p.dh0 || WGRAD) ? 1 : 0) : p.T;
  auto time_of = [&](int s) { return BWD ? p.T - 1 - s : s; };
  // LDS: [h][abort flags (+ unused timeline area)][group sums [B][groups of the pool] (+ 64 bytes that reads may run into)]
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* const lds_tail = lds + p.lds_h_bytes;
  const uint32_t s_abort = lds_address(lds_tail);   // LDS address of the two flags
  float* const qsum = reinterpret_cast<float*>(lds_tail + kLdsTailBytes);

  const int tid = threadIdx.x, lane = tid & 63;
  const int block = blockDim.x, wg = blockIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid) >> 6;
  const int gather_waves = p.gather_waves, pool = gather_waves * 64, pool_groups = pool / G;
  const bool output_wave = wave >= gather_waves;     // wavefront-uniform
  const int H = p.hidden;
  const int plane_bytes = H * 16;                    // distance of the two planes of a batch-8 layout

  // ---- one-time weight load (gathering wavefronts; the output wavefronts have no words)
  const int n_w = __builtin_amdgcn_readfirstlane(p.wave_words[wg * (block >> 6) + wave]);
  uint32_t w_off[NW];
  float w_val[NW];
  const uint32_t lds_base = lds_address(lds);
  const uint32_t pad_word = ((uint32_t)min((lane & 15) * 16, p.h_bytes - 16) >> p.index_shift) << 16;   // zero value
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    // (slots past n_w get a zero value and one of the first sixteen 16-byte pieces of h, a different one in every lane
    // of an LDS pass, so that their reads collide with nothing)
    const uint32_t word = (k < n_w) ? p.words[((size_t)wg * NW + k) * block + tid] : pad_word;
    w_off[k] = lds_base + ((word >> 16) << p.index_shift);
    w_val[k] = half_bits_to_float(word);
  }
  const int row = p.lane_row[(size_t)wg * block + tid];   // gathering lane: the row of its words; output lane: the row it owns
  const int my_sample = sample_of_lane<B>(lane);          // gathering lane: the sample whose group sum it holds after the reduction

  // ---- output lanes: lane e of the output wavefronts owns sample e % B of the workgroup's row e / B
  const bool owner = output_wave && row >= 0;
  const int sample = (tid - pool) % B;
  const int sum_info = output_wave ? p.lane_sum[(size_t)wg * block + tid] : 0;
  const int first_group = sum_info & 0xffff, n_groups = owner ? (sum_info >> 16) : 0;
  const float* const my_sums = qsum + (owner ? sample * pool_groups + first_group : 0);
  int most_groups = n_groups;                        // of any lane of this wavefront: trip count of its summation loop
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) most_groups = max(most_groups, __shfl_xor(most_groups, o));
  most_groups = __builtin_amdgcn_readfirstlane(most_groups);
  const int x_voff = owner ? (sample * H + row) * 4 : kOutOfRange;
  const int out_voff = x_voff;
  const int ring_voff = owner ? lds_offset<B>(row, sample, H) : kOutOfRange;
  const __amdgpu_buffer_rsrc_t ring = __builtin_amdgcn_make_buffer_rsrc(p.ring, 0, kRingSlotsDev * p.h_bytes, kBufWord3);
  const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.x), 0, p.T * B * H * 4, kBufWord3);
  const __amdgpu_buffer_rsrc_t hbuf = __builtin_amdgcn_make_buffer_rsrc(p.h_out, 0, p.T * B * H * 4, kBufWord3);
  const __amdgpu_buffer_rsrc_t abuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(BWD ? p.aux : p.x), 0, p.T * B * H * 4, kBufWord3);
  const __amdgpu_buffer_rsrc_t dbuf = __builtin_amdgcn_make_buffer_rsrc(BWD && p.dh0 ? p.dh0 : p.h_out, 0, B * H * 4, kBufWord3);

  // ---- the copy of h into LDS by the gathering lanes: lane tid copies the 16-byte chunks tid, tid + pool, ... (LDS mirrors
  // the ring slot; indices past the end are clamped to the last chunk, which a few lanes then copy twice)
  const int n4 = p.h_bytes >> 4, last_chunk = n4 - 1;
  const int chunk_rounds = (n4 + pool - 1) / pool;

  // ---- h_0 into LDS
  if (tid < 2) lds_store_int(s_abort + 4 * tid, 0);
  for (int e = tid; e < H * B; e += block) {
    const int j = e / B, b = e % B;
    *reinterpret_cast<float*>(lds + lds_offset<B>(j, b, H)) = p.h0 ? p.h0[(size_t)b * H + j] : 0.0f;
  }

  // b'_t (backward: e_t and the forward output h_t) of an output lane's element, fetched one step ahead
  float xn = 0.0f, an = 0.0f;
  if (output_wave) {
    xn = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, x_voff, time_of(0) * B * H * 4, 0));
    if constexpr (BWD) an = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(abuf, x_voff, time_of(0) * B * H * 4, 0));
  }
  // weight gradient: forward output of a gathering lane's own row for every sample (h_0 in the extra step), fetched one
  // step ahead, and one accumulator per word
  float side[B], gacc[WGRAD ? NW : 1];
  const int row_voff = (!output_wave && row >= 0) ? row * 4 : kOutOfRange;
  const __amdgpu_buffer_rsrc_t h0buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(WGRAD && p.bwd_h0 ? p.bwd_h0 : p.x), 0,
                                                                         (WGRAD && p.bwd_h0) ? B * H * 4 : 0, kBufWord3);
  auto load_side = [&](int s) {   // rows of step T come from h_0 (an empty buffer returns zeros)
#pragma unroll
    for (int b = 0; b < B; ++b)
      side[b] = __builtin_bit_cast(float, s < p.T ? __builtin_amdgcn_raw_buffer_load_b32(abuf, row_voff, (time_of(s) * B + b) * H * 4, 0)
                                                  : __builtin_amdgcn_raw_buffer_load_b32(h0buf, row_voff, b * H * 4, 0));
  };
  if constexpr (WGRAD) {
#pragma unroll
    for (int k = 0; k < NW; ++k) gacc[k] = 0.0f;
    load_side(0);
  }
  __syncthreads();

  const uint32_t wave_id = (uint32_t)(wg * (block >> 6) + wave);
  const bool tl_on = TL && p.timeline != nullptr && (wave == p.tl_wave || wave == gather_waves);
  unsigned long long tl_sum[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  for (int t = 0; t < steps; ++t) {
    const uint32_t g = p.step_base + (uint32_t)t;    // global step index: the slot number is the timestep tag
    unsigned long long repolls = 0;
    long long k0 = tick<TL>(tl_on), k1 = k0, k2 = k0, k3 = k0;

    // ---- load: h_{t-1}, published by the output wavefronts of every workgroup in step t-1
    if (t > 0) {
      const int slot_byte = (int)((g - 1) & (kRingSlotsDev - 1)) * p.h_bytes;
      bool failed = false;
      if (p.sync == SPRNN_SYNC_BARRIER) {
        // grid barrier (Section 3.2): every store of the workgroup performed, one arrival per workgroup, wait for all
        // (counters as in persistent_kernel)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        if (tid == 0) {
          const uint32_t n = p.barrier_base + (uint32_t)t;
          uint32_t target;
          if (gridDim.x < 64u) {
            __hip_atomic_fetch_add(p.ctrl + kCtrlBarrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            target = n * gridDim.x;
          } else {
            const uint32_t grp = (uint32_t)wg % 8u, members = gridDim.x / 8u + (grp < gridDim.x % 8u ? 1u : 0u);
            const uint32_t before = __hip_atomic_fetch_add(p.ctrl + kCtrlBarrier + 16 * (1 + grp), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (before + 1 == n * members) __hip_atomic_fetch_add(p.ctrl + kCtrlBarrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            target = n * 8u;
          }
          int spins = 0;
          for (;;) {
            const uint32_t seen = __hip_atomic_load(p.ctrl + kCtrlBarrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((int)(seen - target) >= 0) break;
            if (++spins > p.spin_limit || ((spins & 1023) == 0 && __hip_atomic_load(p.ctrl + kCtrlStatus, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
              lds_store_int(s_abort + 4 * (t & 1), 1);
              break;
            }
          }
        }
        lds_barrier();
        failed = __builtin_amdgcn_readfirstlane(lds_load_int(s_abort + 4 * (t & 1))) != 0;
      }
      if (!output_wave) {
        if (p.sync != SPRNN_SYNC_BARRIER) {
          // Polling a line before its producer wrote it installs a stale copy in this XCD's L2 that has to be invalidated
          // and fetched again, which costs more than waiting a little too long: back off first.  The wait counts from the
          // barrier behind the group sums; it covers the output wavefronts' work and the way of their stores.
          for (int d = 0; d < p.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
          jitter_pause(p.jitter, wave_id, g, 1);
        }
        k1 = tick<TL>(tl_on);
        if (!failed) {
          // all of a lane's chunks in flight at once, up to sixteen; longer copies in batches of sixteen
          for (int r0 = 0; r0 < chunk_rounds && !failed; r0 += 16)
            failed = !copy_rounds(min(chunk_rounds - r0, 16), ring, slot_byte, tid + r0 * pool, pool, last_chunk, lds, p, repolls);
        }
        jitter_pause(p.jitter, wave_id, g, 2);
        k2 = tick<TL>(tl_on);
        if (failed) {
          lds_store_int(s_abort + 4 * (t & 1), 1);
          __hip_atomic_store(p.ctrl + kCtrlStatus, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      lds_barrier();   // h_{t-1} is complete in LDS; the output wavefronts have read the group sums of step t-1
      // every wavefront of the workgroup leaves together; other workgroups see the status word
      if (__builtin_amdgcn_readfirstlane(lds_load_int(s_abort + 4 * (t & 1)))) break;
      k3 = tick<TL>(tl_on);
      if (TL && tl_on && !output_wave) { tl_sum[0] += k1 - k0; tl_sum[1] += k2 - k1; tl_sum[2] += k3 - k2; tl_sum[8] += repolls; }
    }
    k3 = tick<TL>(tl_on);

    // ---- operate and reduce inside each group: afterwards a lane holds its group's sum for sample my_sample
    if (!output_wave) {
      float acc[B];
#pragma unroll
      for (int b = 0; b < B; ++b) acc[b] = 0.0f;
      operate_pipelined<B, NW, WGRAD>(acc, w_off, w_val, plane_bytes, gacc, side);
      if constexpr (TL) {   // (waits for the sums so that the arithmetic is not billed to the reduction)
#pragma unroll
        for (int b = 0; b < B; ++b) asm volatile("" : "+v"(acc[b]));
      }
      const long long k4 = tick<TL>(tl_on);
      const float part = reduce_scatter<G, B>(acc, lane);
      qsum[my_sample * pool_groups + (tid / G)] = part;
      if (TL && tl_on) { const long long k5 = tick<TL>(tl_on); tl_sum[3] += k4 - k3; tl_sum[4] += k5 - k4; k3 = k5; }
      if constexpr (WGRAD) {
        if (t + 1 < steps) load_side(t + 1);
      }
    }
    lds_barrier();     // the group sums of step t are in LDS; every gather of step t is done (h may be overwritten)
    const long long k6 = tick<TL>(tl_on);
    if (TL && tl_on && !output_wave) { tl_sum[5] += k6 - k3; tl_sum[9] += 1; }

    // ---- epilogue and hand-off by the output wavefronts
    if (output_wave) {
      float sum = 0.0f;
      for (int i0 = 0; i0 < most_groups; i0 += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = my_sums[i0 + j];      // (may read past the row's groups: those values are dropped)
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += (i0 + j < n_groups) ? v[j] : 0.0f;
      }
      if constexpr (TL) asm volatile("" : "+v"(sum));
      const long long k7 = tick<TL>(tl_on);
      const float pre = sum + xn;
      float hval;
      if constexpr (BWD) {
        if (t < p.T) {
          const float slope = p.act == SPRNN_ACT_RELU ? (an > 0.0f ? 1.0f : 0.0f) : (p.act == SPRNN_ACT_TANH ? fmaf(-an, an, 1.0f) : 1.0f);
          hval = slope * pre + 0.0f;   // + 0.0f: 0 * negative is -0.0, the "not written" mark
        } else {
          hval = sum + 0.0f;           // the extra step: U^T delta_1, no e, no g'
        }
      } else {
        hval = activate(p.act, pre);
      }
      jitter_pause(p.jitter, wave_id, g, 3);
      const int slot_byte = (int)(g & (kRingSlotsDev - 1)) * p.h_bytes;
      const int rearm_byte = (int)((g + 2) & (kRingSlotsDev - 1)) * p.h_bytes;
      const int out_soff = time_of(t) * B * H * 4;
      // the re-arm stores issued one step ago must be performed before this step's data can be seen, hence the wait
      // (everything this wavefront has in flight was issued a whole step ago)
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (TL && tl_on) { const long long k8 = tick<TL>(tl_on); tl_sum[6] += k7 - k6; tl_sum[7] += k8 - k7; }
      __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), ring, ring_voff, slot_byte, kAuxCoherent);
      if (p.sync == SPRNN_SYNC_TAGGED) __builtin_amdgcn_raw_buffer_store_b32((int)kSentinelBits, ring, ring_voff, rearm_byte, kAuxCoherent);
      if (BWD && t == p.T) {
        if (p.dh0) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), dbuf, out_voff, 0, 0);
      } else {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), hbuf, out_voff, out_soff, 0);
      }
      if (t + 1 < p.T) {
        xn = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, x_voff, time_of(t + 1) * B * H * 4, 0));
        if constexpr (BWD) an = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(abuf, x_voff, time_of(t + 1) * B * H * 4, 0));
      }
    }
  }
  if constexpr (TL) {
    if (tl_on && lane == 0) {
      const int first = output_wave ? 6 : 0, last = output_wave ? 7 : 5;
      for (int i = first; i <= last; ++i) p.timeline[(size_t)wg * kTimelineSlots + i] += tl_sum[i];
      if (!output_wave) { p.timeline[(size_t)wg * kTimelineSlots + 8] += tl_sum[8]; p.timeline[(size_t)wg * kTimelineSlots + 9] += tl_sum[9]; }
    }
  }
  if constexpr (WGRAD) {   // the sums leave through the packer's word -> CSR position map (of the transposed matrix)
#pragma unroll
    for (int k = 0; k < NW; ++k) {
      if (k < n_w) {
        const int src = p.word_src[((size_t)wg * NW + k) * block + tid];
        if (src >= 0) p.dU[src] = gacc[k];
      }
    }
  }
}

// Instantiations: every multiple of four words per lane up to 64 (the arithmetic runs over all NW slots, so the menu is
// fine-grained), as far as everything stays in the 256 registers of a lane: the kernel with the weight gradient fused in
// keeps one more register per word and goes up to 32 words, 16 at batch 8; the others up to 64, 48 at batch 8.
template <int B, int CELL, bool TL = false>
static const void* pick_pool_nw(int nw) {
  constexpr int most = CELL == 4 ? (B == 8 ? 16 : 32) : (B == 8 ? 48 : 64);
#define SPRNN_POOL_CASE(N) case N: if constexpr (most >= N) return (const void*)pool_kernel<B, N, CELL, TL>; else return nullptr;
  switch (nw) {
    SPRNN_POOL_CASE(4) SPRNN_POOL_CASE(8) SPRNN_POOL_CASE(12) SPRNN_POOL_CASE(16) SPRNN_POOL_CASE(20) SPRNN_POOL_CASE(24)
    SPRNN_POOL_CASE(28) SPRNN_POOL_CASE(32) SPRNN_POOL_CASE(36) SPRNN_POOL_CASE(40) SPRNN_POOL_CASE(44) SPRNN_POOL_CASE(48)
    SPRNN_POOL_CASE(52) SPRNN_POOL_CASE(56) SPRNN_POOL_CASE(60) SPRNN_POOL_CASE(64)
    default: return nullptr;
  }
#undef SPRNN_POOL_CASE
}

template <int CELL>
static const void* pick_pool_b(int batch, int nw) {
  switch (batch) {
    case 1: return pick_pool_nw<1, CELL>(nw);
    case 2: return pick_pool_nw<2, CELL>(nw);
    case 4: return pick_pool_nw<4, CELL>(nw);
    case 8: return pick_pool_nw<8, CELL>(nw);
    default: return nullptr;
  }
}

}  // namespace sprnn
#endif
