// Device code of libsprnn: the persistent sparse recurrent kernel as a template.  Included by the translation units that
// instantiate it (forward cells, their timeline variants, vanilla backward, gated cells' backward), which are compiled
// side by side.
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
#ifndef SPRNN_PERSISTENT_H_
#define SPRNN_PERSISTENT_H_

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

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

// ---- reduction over the L lanes of a row, scattering the B samples over the lanes (reduce-scatter) -------------
// Every lane enters with B partial sums (one per sample).  The first log2(B) butterfly stages are halving
// exchanges: a lane keeps one half of its values and hands the other half to its partner, so after them a
// lane holds ONE value; the remaining stages are plain butterflies.  At the end every lane of the row holds
// the complete sum for sample  sample_of_lane<B>(lane)  and nothing else: about 2 B + log2(L) additions per
// lane instead of B log2(L), and the epilogue (b'_t, activation, stores) handles one value per lane.
// Partner of stage K is lane ^ (1 << K): quad permutes (K = 0, 1), masked row shifts (K = 2), a row rotation
// (K = 3) and the row-swap instructions of gfx950 (K = 4, 5).
template <int K>
__device__ __forceinline__ float from_partner(float give) {
  const int g = __builtin_bit_cast(int, give);
  if constexpr (K == 0) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, g, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
  if constexpr (K == 1) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, g, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
  if constexpr (K == 2) {   // lanes of quads 0, 2 read four lanes up, lanes of quads 1, 3 four lanes down
    const int up = __builtin_amdgcn_update_dpp(0, g, 0x104, 0xf, 0x5, false);     // row_shl:4, banks 0 and 2
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(up, g, 0x114, 0xf, 0xa, false));   // row_shr:4, banks 1 and 3
  }
  if constexpr (K == 3) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, g, 0x128, 0xf, 0xf, false));  // row_ror:8
  return 0.0f;
}

// Plain butterfly across rows of 16 lanes (K = 4) or halves of the wavefront (K = 5): copy, swap the odd rows of
// one copy with the even rows of the other, add.  (v_permlane16_swap / v_permlane32_swap: VALU, no LDS.)
template <int K>
__device__ __forceinline__ float cross_row_sum(float v) {
  float a = v, b;
  if constexpr (K == 4) asm volatile("v_mov_b32 %1, %0\n\ts_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "=&v"(b));
  else asm volatile("v_mov_b32 %1, %0\n\ts_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "=&v"(b));
  return a + b;
}

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }

// Sample whose sum a lane holds after reduce_scatter: stage K hands the upper half of the value list to the lanes
// with bit K set.
template <int B>
__device__ __forceinline__ int sample_of_lane(int lane) {
  int s = 0;
#pragma unroll
  for (int k = 0; k < ilog2(B); ++k) s += ((lane >> k) & 1) * (B >> (k + 1));
  return s;
}

template <int B, int N, int K>
__device__ __forceinline__ void halving_stage(float (&v)[B], int lane) {
  if constexpr (N > 1) {
    const bool upper = (lane >> K) & 1;
#pragma unroll
    for (int j = 0; j < N / 2; ++j) {
      const float keep = upper ? v[j + N / 2] : v[j];
      const float give = upper ? v[j] : v[j + N / 2];
      v[j] = keep + from_partner<K>(give);
    }
  }
}

template <int L, int B>
__device__ __forceinline__ float reduce_scatter(float (&v)[B], int lane) {
  static_assert(L >= B, "a row needs at least as many lanes as there are samples");
  constexpr int SPLITS = ilog2(B), STAGES = ilog2(L);
  if constexpr (SPLITS >= 1) halving_stage<B, B, 0>(v, lane);
  if constexpr (SPLITS >= 2) halving_stage<B, B / 2, 1>(v, lane);
  if constexpr (SPLITS >= 3) halving_stage<B, B / 4, 2>(v, lane);
  float t = v[0];
  if constexpr (SPLITS <= 0 && STAGES > 0) t += from_partner<0>(t);
  if constexpr (SPLITS <= 1 && STAGES > 1) t += from_partner<1>(t);
  if constexpr (SPLITS <= 2 && STAGES > 3) {
    // both in-row stages are plain: two rotations sum the four lanes that share lane % 4
    t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x124, 0xf, 0xf, false));   // row_ror:4
    t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x128, 0xf, 0xf, false));   // row_ror:8
  } else {
    if constexpr (SPLITS <= 2 && STAGES > 2) t += from_partner<2>(t);
    if constexpr (STAGES > 3) t += from_partner<3>(t);
  }
  if constexpr (STAGES > 4) t = cross_row_sum<4>(t);
  if constexpr (STAGES > 5) t = cross_row_sum<5>(t);
  return t;
}

// One jump on the (kernel-uniform) lanes-per-row, then straight-line code.
template <int B>
__device__ __forceinline__ float reduce_rows(float (&acc)[B], int L, int lane) {
  switch (L) {
    case 64: return reduce_scatter<64, B>(acc, lane);
    case 32: return reduce_scatter<32, B>(acc, lane);
    case 16: return reduce_scatter<16, B>(acc, lane);
    case 8: return reduce_scatter<8, B>(acc, lane);
    case 4: if constexpr (B <= 4) return reduce_scatter<4, B>(acc, lane); else break;
    case 2: if constexpr (B <= 2) return reduce_scatter<2, B>(acc, lane); else break;
    case 1: if constexpr (B <= 1) return acc[0]; else break;
    default: break;
  }
  return 0.0f;
}

// Logistic function and tanh from the hardware exp2 / reciprocal instructions (about 1 ulp each):
// absolute error of a few 1e-7, far inside the 1e-3 parity bound, at a handful of instructions.
__device__ __forceinline__ float sigmoidf_(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}
__device__ __forceinline__ float tanhf_(float z) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.8853900817779268f * z));
}

__device__ __forceinline__ float activate(int act, float pre) {
  float h;
  if (act == SPRNN_ACT_RELU) h = fmaxf(pre, 0.0f);
  else if (act == SPRNN_ACT_TANH) h = tanhf_(pre);
  else h = pre;
  return h + 0.0f;   // -0.0 -> +0.0: -0.0 is reserved as the "not written" mark
}

// The "not written" mark 0x80000000 is the smallest signed integer, so a chunk (or several) is completely
// written exactly when the signed minimum of its words is larger than that.
__device__ __forceinline__ int min_word(i32x4 v) { return min(min(v.x, v.y), min(v.z, v.w)); }
__device__ __forceinline__ bool all_written(i32x4 v) { return min_word(v) != (int)kSentinelBits; }

// LDS byte offset of h[col j][sample b]
template <int B>
__device__ __forceinline__ int lds_offset(int j, int b, int H) {
  if (B == 8) return (b >> 2) * H * 16 + j * 16 + (b & 3) * 4;
  return (j * B + b) * 4;
}

// One gathered column of h for all B samples (two planes of four samples when B == 8).
template <int B>
struct Column {
  f32x4 lo, hi;
};

// `addr` is an absolute LDS address (32 bits), so the read needs no address arithmetic.  (The host pass of the
// compiler sees a 32-bit integer turned into one of its 64-bit pointers here and would warn; it never runs this.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wint-to-pointer-cast"
#define SPRNN_LDS_PTR(T, addr) ((const __attribute__((address_space(3))) T*)(uint32_t)(addr))
__device__ __forceinline__ uint32_t lds_address(const void* generic) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)generic;
}

// Workgroup barrier that orders LDS traffic only: global loads and stores of the wavefront stay in flight across it.
// (__syncthreads() also waits for every outstanding global memory operation of the wavefront.)
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// The abort flags live in LDS and are read by every wavefront in every step: explicit LDS accesses.  (Through a
// generic volatile pointer the compiler emits system-scope flat instructions, which take the long way through the
// vector memory pipeline and make every wavefront drain its global loads and stores first.)
__device__ __forceinline__ void lds_store_int(uint32_t addr, int v) {
  *((volatile __attribute__((address_space(3))) int*)(uint32_t)addr) = v;
}
__device__ __forceinline__ int lds_load_int(uint32_t addr) {
  return *((volatile __attribute__((address_space(3))) int*)(uint32_t)addr);
}

// NARROW: one 4-byte read per sample instead of one wide read per column (batch 4 only): the rung below Section 4.1's
// wide loads in the ablation.  The four reads of a lane hit four different banks, but the lanes of a pass now spread
// over a quarter of the banks per read, and the LDS has four times the instructions to serve.
template <int B, bool NARROW = false>
__device__ __forceinline__ Column<B> gather_column(uint32_t addr, int plane_bytes) {
  Column<B> c;
  if constexpr (NARROW && B == 4) {
    c.lo.x = *SPRNN_LDS_PTR(float, addr);
    c.lo.y = *SPRNN_LDS_PTR(float, addr + 4);
    c.lo.z = *SPRNN_LDS_PTR(float, addr + 8);
    c.lo.w = *SPRNN_LDS_PTR(float, addr + 12);
  } else if constexpr (B == 1) {
    c.lo.x = *SPRNN_LDS_PTR(float, addr);
  } else if constexpr (B == 2) {
    const f32x2 v = *SPRNN_LDS_PTR(f32x2, addr);
    c.lo.x = v.x; c.lo.y = v.y;
  } else if constexpr (B == 4) {
    c.lo = *SPRNN_LDS_PTR(f32x4, addr);
  } else {
    c.lo = *SPRNN_LDS_PTR(f32x4, addr);
    c.hi = *SPRNN_LDS_PTR(f32x4, addr + (uint32_t)plane_bytes);
  }
  return c;
}
#pragma clang diagnostic pop

template <int B>
__device__ __forceinline__ void mac_column(float (&acc)[B], float wv, const Column<B>& c) {
  acc[0] = fmaf(wv, c.lo.x, acc[0]);
  if constexpr (B >= 2) acc[1] = fmaf(wv, c.lo.y, acc[1]);
  if constexpr (B >= 4) {
    acc[2] = fmaf(wv, c.lo.z, acc[2]);
    acc[3] = fmaf(wv, c.lo.w, acc[3]);
  }
  if constexpr (B == 8) {
    acc[4] = fmaf(wv, c.hi.x, acc[4]);
    acc[5] = fmaf(wv, c.hi.y, acc[5]);
    acc[6] = fmaf(wv, c.hi.z, acc[6]);
    acc[7] = fmaf(wv, c.hi.w, acc[7]);
  }
}

// N (1..4) words of one lane: all N gathers are issued back to back, then the multiply-adds follow.
// The scheduling barrier keeps the compiler from sinking a gather below the arithmetic of an earlier one,
// so a wavefront has N wide LDS reads in flight instead of one.
template <int B>
__device__ __forceinline__ float dot_column(const float (&s)[B], const Column<B>& c, float sum) {
  sum = fmaf(s[0], c.lo.x, sum);
  if constexpr (B >= 2) sum = fmaf(s[1], c.lo.y, sum);
  if constexpr (B >= 4) { sum = fmaf(s[2], c.lo.z, sum); sum = fmaf(s[3], c.lo.w, sum); }
  if constexpr (B == 8) {
    sum = fmaf(s[4], c.hi.x, sum); sum = fmaf(s[5], c.hi.y, sum);
    sum = fmaf(s[6], c.hi.z, sum); sum = fmaf(s[7], c.hi.w, sum);
  }
  return sum;
}

// With GRAD, the gathered column also feeds the weight gradient of its nonzero: g[j] += sum_b side[b] * column[b]
// (backward pass: the column is delta_{t+1} of the nonzero's column, side is the forward output of the lane's row).
template <int B, int N, bool GRAD = false, bool NARROW = false>
__device__ __forceinline__ void mac_words(float (&acc)[B], const uint32_t* off, const float* wv, int plane_bytes,
                                          float* g = nullptr, const float (*side)[B] = nullptr) {
  Column<B> c[N];
#pragma unroll
  for (int j = 0; j < N; ++j) c[j] = gather_column<B, NARROW>(off[j], plane_bytes);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < N; ++j) {
    mac_column<B>(acc, wv[j], c[j]);
    if constexpr (GRAD) g[j] = dot_column<B>(*side, c[j], g[j]);
  }
}

// binary16 activations (batch 4): a column of h is four binary16 values, one 8-byte read; products and sums stay
// binary32 (the conversion is exact, and the compiler folds it into a mixed-precision multiply-add).
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wint-to-pointer-cast"   // (the host pass sees a 32-bit LDS address become one of its pointers; it never runs this)
template <int N, int B>
__device__ __forceinline__ void mac_words_half(float (&acc)[B], const uint32_t* off, const float* wv) {
  static_assert(B == 4 || B == 8, "a column of binary16 activations is one 8- or 16-byte read");
  using column = typename std::conditional<B == 4, halfx4, halfx8>::type;
  column c[N];
#pragma unroll
  for (int j = 0; j < N; ++j) c[j] = *SPRNN_LDS_PTR(column, off[j]);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < N; ++j) {
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = fmaf(wv[j], (float)c[j][b], acc[b]);
  }
}
#pragma clang diagnostic pop
template <int NW, int B>
__device__ __forceinline__ void operate_half(float (&acc)[B], const uint32_t (&w_off)[NW], const float (&w_val)[NW], int n_w) {
#pragma unroll
  for (int k = 0; k < NW; k += 8) {
    if (k + 8 <= n_w) {
      mac_words_half<8, B>(acc, &w_off[k], &w_val[k]);
    } else if (k < n_w) {
      const int rem = n_w - k;
      if (rem >= 4) {
        mac_words_half<4, B>(acc, &w_off[k], &w_val[k]);
        if (rem == 7) mac_words_half<3, B>(acc, &w_off[k + 4], &w_val[k + 4]);
        else if (rem == 6) mac_words_half<2, B>(acc, &w_off[k + 4], &w_val[k + 4]);
        else if (rem == 5) mac_words_half<1, B>(acc, &w_off[k + 4], &w_val[k + 4]);
      } else if (rem == 3) mac_words_half<3, B>(acc, &w_off[k], &w_val[k]);
      else if (rem == 2) mac_words_half<2, B>(acc, &w_off[k], &w_val[k]);
      else mac_words_half<1, B>(acc, &w_off[k], &w_val[k]);
    }
  }
}
// A 32-bit word of the exchange ring holds two binary16 elements; "not written" is the mark in both halves.
constexpr uint32_t kSentinelHalfPair = 0x80008000u;
// smallest of the chunk's words after an exclusive-or with the mark pair: zero exactly when one of them is unwritten
__device__ __forceinline__ uint32_t unwritten_key_half(i32x4 v) {
  const uint32_t a = (uint32_t)v.x ^ kSentinelHalfPair, b = (uint32_t)v.y ^ kSentinelHalfPair;
  const uint32_t c = (uint32_t)v.z ^ kSentinelHalfPair, d = (uint32_t)v.w ^ kSentinelHalfPair;
  return min(min(a, b), min(c, d));
}
// binary32 -> binary16 bits, round to nearest even; -0.0 (the mark) becomes +0.0
__device__ __forceinline__ uint32_t half_bits_for_exchange(float v) {
  const _Float16 h = (_Float16)v;
  const uint32_t bits = (uint32_t)__builtin_bit_cast(unsigned short, h);
  return bits == 0x8000u ? 0u : bits;
}

constexpr int kOutOfRange = 0x7ffffff0;   // a byte offset beyond every buffer this kernel addresses

// The n_w (wavefront-uniform) packed words of a lane (w_off: absolute LDS addresses of their columns): gathers in
// groups of four so the LDS reads are issued back to back; no early exit, so every register index stays static.
// GS: words per group, 4 or 8 (see the kernel's choice).
template <int B, int NW, bool GRAD = false, int GS = 4, bool NARROW = false>
__device__ __forceinline__ void operate(float (&acc)[B], const uint32_t (&w_off)[NW], const float (&w_val)[NW], int n_w,
                                        int plane_bytes, float* g = nullptr, const float (*side)[B] = nullptr) {
#pragma unroll
  for (int k = 0; k < NW; k += GS) {
    float* gk = GRAD ? g + k : nullptr;
    if (k + GS <= n_w) {
      mac_words<B, GS, GRAD, NARROW>(acc, &w_off[k], &w_val[k], plane_bytes, gk, side);
    } else if (k < n_w) {   // ragged tail
      const int rem = n_w - k;
      if (GS == 8 && rem >= 4) {
        mac_words<B, 4, GRAD, NARROW>(acc, &w_off[k], &w_val[k], plane_bytes, gk, side);
        float* gk4 = GRAD ? gk + 4 : nullptr;   // the second half's sums belong to words k + 4 ..
        if (rem == 7) mac_words<B, 3, GRAD, NARROW>(acc, &w_off[k + 4], &w_val[k + 4], plane_bytes, gk4, side);
        else if (rem == 6) mac_words<B, 2, GRAD, NARROW>(acc, &w_off[k + 4], &w_val[k + 4], plane_bytes, gk4, side);
        else if (rem == 5) mac_words<B, 1, GRAD, NARROW>(acc, &w_off[k + 4], &w_val[k + 4], plane_bytes, gk4, side);
      } else if (rem == 3) mac_words<B, 3, GRAD, NARROW>(acc, &w_off[k], &w_val[k], plane_bytes, gk, side);
      else if (rem == 2) mac_words<B, 2, GRAD, NARROW>(acc, &w_off[k], &w_val[k], plane_bytes, gk, side);
      else mac_words<B, 1, GRAD, NARROW>(acc, &w_off[k], &w_val[k], plane_bytes, gk, side);
    }
  }
}

// Words [lo, hi) of a lane (wavefront-uniform bounds, lo a multiple of four): the two-part copy works through a lane's
// leading words while the rest of h is still arriving, and through the others afterwards.  Groups of eight gathers
// where a whole one lies inside the span, of four otherwise.
template <int B, int NW, int K>
__device__ __forceinline__ void span_four(float (&acc)[B], const uint32_t (&w_off)[NW], const float (&w_val)[NW], int lo, int hi, int plane_bytes) {
  if constexpr (K < NW) {   // (NW is a multiple of eight, so four slots from K on exist)
    if (K >= lo && K < hi) {
      const int rem = hi - K;
      if (rem >= 4) mac_words<B, 4>(acc, &w_off[K], &w_val[K], plane_bytes);
      else if (rem == 3) mac_words<B, 3>(acc, &w_off[K], &w_val[K], plane_bytes);
      else if (rem == 2) mac_words<B, 2>(acc, &w_off[K], &w_val[K], plane_bytes);
      else mac_words<B, 1>(acc, &w_off[K], &w_val[K], plane_bytes);
    }
  }
}
template <int B, int NW, int K = 0>
__device__ __forceinline__ void operate_span(float (&acc)[B], const uint32_t (&w_off)[NW], const float (&w_val)[NW], int lo, int hi,
                                             int plane_bytes) {
  if constexpr (K < NW) {
    if (K >= lo && K + 8 <= hi) {
      mac_words<B, 8>(acc, &w_off[K], &w_val[K], plane_bytes);
    } else {
      span_four<B, NW, K>(acc, w_off, w_val, lo, hi, plane_bytes);
      span_four<B, NW, K + 4>(acc, w_off, w_val, lo, hi, plane_bytes);
    }
    operate_span<B, NW, K + 8>(acc, w_off, w_val, lo, hi, plane_bytes);
  }
}

// The chunks of rounds [LO, HI) of a copy whose loads (v, from ring offsets `off`) are already in flight: wait until
// all of them are written (polling again where the "not written" mark is still there; bounded like copy_chunks), then
// put them into LDS at the same offsets.  Returns false when the wait was given up.  The bounds are compile-time values so
// that the wait for a load's data counts exactly the loads issued after it: the later rounds stay in flight.
template <int D, int LO, int HI>
__device__ __forceinline__ bool finish_chunks(__amdgpu_buffer_rsrc_t ring, int slot_byte, const int (&off)[D], i32x4 (&v)[D],
                                              unsigned char* dst, int spin_limit, const uint32_t* status_word, unsigned long long& repolls) {
  // The first check stands outside the polling loop: straight-line code after the loads were issued, where the wait
  // for round c's data is "all but the HI - 1 - c .. loads issued after it"; inside a loop the compiler has to assume
  // the worst of both ways into it and would wait for every load in flight.
  auto all_written_now = [&]() {
    int low = min_word(v[LO]);
#pragma unroll
    for (int c = LO + 1; c < HI; ++c) low = min(low, min_word(v[c]));
    return __builtin_amdgcn_ballot_w64(low == (int)kSentinelBits) == 0;
  };
  bool ok = true;
  if (!all_written_now()) {
    int spins = 0;
    for (;;) {
      ++spins;
      ++repolls;
      if (spins > spin_limit || ((spins & 1023) == 0 && __hip_atomic_load(status_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
        ok = false;
        break;
      }
#pragma unroll
      for (int c = LO; c < HI; ++c) v[c] = __builtin_amdgcn_raw_buffer_load_b128(ring, off[c], slot_byte, kAuxCoherent);
      if (all_written_now()) break;
    }
  }
#pragma unroll
  for (int c = LO; c < HI; ++c) *reinterpret_cast<i32x4*>(dst + off[c]) = v[c];
  return ok;
}

// Copy D 16-byte chunks per lane from a ring slot (byte offsets `off`) into LDS (byte offsets `to`), all D loads in
// flight at once.  With MAYSKIP an entry with to[c] < 0 is empty: its source offset lies out of range, so the load
// costs no memory traffic and returns zeros, and nothing is written.  A chunk that still holds the "not written" mark makes
// the whole wavefront poll again (bounded by spin_limit; a tripped watchdog anywhere ends the wait).  Returns false
// when the wait was given up.
template <int D, bool MAYSKIP, bool HALF = false>
__device__ __forceinline__ bool copy_chunks(__amdgpu_buffer_rsrc_t ring, int slot_byte, const int (&off)[D], const int (&to)[D],
                                            unsigned char* dst, int spin_limit, const uint32_t* status_word, unsigned long long& repolls) {
  i32x4 v[D];
  bool ok = true;
  int spins = 0;
  for (;;) {
#pragma unroll
    for (int c = 0; c < D; ++c) v[c] = __builtin_amdgcn_raw_buffer_load_b128(ring, off[c], slot_byte, kAuxCoherent);
    bool pending;
    if constexpr (HALF) {
      uint32_t key = unwritten_key_half(v[0]);
#pragma unroll
      for (int c = 1; c < D; ++c) key = min(key, unwritten_key_half(v[c]));
      pending = key == 0u;
    } else {
      int low = min_word(v[0]);
#pragma unroll
      for (int c = 1; c < D; ++c) low = min(low, min_word(v[c]));
      pending = low == (int)kSentinelBits;
    }
    if (__builtin_amdgcn_ballot_w64(pending) == 0) break;
    // some producer has not published yet
    ++spins;
    ++repolls;
    if (spins > spin_limit || ((spins & 1023) == 0 && __hip_atomic_load(status_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
      ok = false;
      break;
    }
  }
#pragma unroll
  for (int c = 0; c < D; ++c)
    if (!MAYSKIP || to[c] >= 0) *reinterpret_cast<i32x4*>(dst + to[c]) = v[c];
  return ok;
}

// Test aid: a pause of 0..15 x 64 clocks that differs per wavefront, step and call site (seed != 0 only).
__device__ __forceinline__ void jitter_pause(int seed, uint32_t wave_id, uint32_t step, uint32_t site) {
  if (seed == 0) return;
  uint32_t x = (uint32_t)seed * 0x9E3779B9u ^ (wave_id * 0x85EBCA6Bu) ^ (step * 0xC2B2AE35u) ^ (site * 0x27D4EB2Fu);
  x ^= x >> 15; x *= 0x2C1B3C6Du; x ^= x >> 12;
  const int n = (int)__builtin_amdgcn_readfirstlane(x & 15u);
  for (int i = 0; i < n; ++i) __builtin_amdgcn_s_sleep(1);
}

// Timestamps of the optional phase timeline (TL): wall-clock reads that vanish from the TL = false kernels.
template <bool TL>
__device__ __forceinline__ long long tick(bool on) {
  if constexpr (TL) return on ? (long long)wall_clock64() : 0;
  return 0;
}

// The load stage of the two-part copy for a copy of R rounds, the first R / 2 of them forming the first part: all R
// loads go out at once; the first part is checked, stored and, after a barrier that orders LDS traffic only (so the
// other loads stay in flight across it), every wavefront works through the `early` leading words of its lanes; then the
// second part is checked and stored.  A wavefront that gave up still meets the others at the barrier.
// (LDS mirrors the ring slot: round c of lane tid is the chunk tid + c * block, clamped to the last one.)
template <int B, int NW, int R, bool TL>
__device__ __forceinline__ bool copy_two_parts(__amdgpu_buffer_rsrc_t ring, int slot_byte, int tid, int block, int last_chunk, unsigned char* dst,
                                               int spin_limit, const uint32_t* status_word, unsigned long long& repolls, int jitter,
                                               uint32_t wave_id, uint32_t step, float (&acc)[B], const uint32_t (&w_off)[NW],
                                               const float (&w_val)[NW], int early, int plane_bytes, bool tl_on, long long& t_first) {
  constexpr int R0 = R / 2;
  int off[R];
  i32x4 v[R];
#pragma unroll
  for (int c = 0; c < R; ++c) off[c] = min(tid + c * block, last_chunk) * 16;
#pragma unroll
  for (int c = 0; c < R; ++c) v[c] = __builtin_amdgcn_raw_buffer_load_b128(ring, off[c], slot_byte, kAuxCoherent);
  bool ok = finish_chunks<R, 0, R0>(ring, slot_byte, off, v, dst, spin_limit, status_word, repolls);
  jitter_pause(jitter, wave_id, step, 4);
  lds_barrier();
  t_first = tick<TL>(tl_on);
  operate_span<B, NW>(acc, w_off, w_val, 0, early, plane_bytes);
  if (ok) ok = finish_chunks<R, R0, R>(ring, slot_byte, off, v, dst, spin_limit, status_word, repolls);
  return ok;
}

// CELL: 0 = vanilla cell (one row per unit), 1 = LSTM (four gate rows per unit), 2 = GRU (the LSTM's layout with an
// idle fourth row; a template value of its own so that the LSTM instantiations carry none of its code),
// 3 = backward pass through time of the vanilla cell: the handle holds the transposed matrix, time runs from T
// down to 1, the state that is exchanged is delta_t = g'(a_t) (e_t + U^T delta_{t+1}), with g' taken from the forward
// output h_t (p.aux) and e_t = p.x; one more step without g' and e gives dL/dh_0 = U^T delta_1 (p.dh0),
// 4 = the same with the weight gradient fused in (one more register per packed word, so the instantiations with 24
// and 32 words per lane are built for at most 512 threads): the column a lane gathers for a nonzero (i, j) of the transposed
// matrix is delta_{t+1}[.][i], exactly the factor that dL/dU[i][j] = sum_t sum_b delta_{t+1}[b][i] h_t[b][j] pairs with
// the forward output of the lane's own row j, so every gather also feeds one resident accumulator per nonzero.
// 5 = backward pass through time of the LSTM: the handle holds the transposed matrix, one row per hidden unit over
// the 4H gate gradients, so p.hidden (the length of the exchanged vector) is 4 * units and the vanilla layout applies.
// The owner lane of (unit, sample) turns dh_t = e_t + U^T dp_{t+1} into the unit's four gate gradients with the gate
// values (p.aux) and cell states (p.c_out, p.c0) of the forward pass, keeps dc_{t+1} f_{t+1} in a register, and
// publishes four elements of the exchanged vector instead of one; one more step gives dL/dh_0 (p.dh0),
// 6 = the same with the weight gradient fused in as in 4: the column gathered for a nonzero (j, g H + i) of the transposed
// matrix is dp_{t+1}[.][g H + i], the factor that dL/dU[g H + i][j] pairs with the forward output h_t[.][j] of the lane's row,
// 7 = backward pass through time of the GRU: as 5 with three elements per unit, v = (dp_r | dp_z | dq) over the transposed
// [H][3H] matrix; kept from the forward pass are r, z, n, q (p.aux, [T][B][4H]) and h_{t-1} (p.c_out, p.c0); the lane carries
// dh_{t+1} z_{t+1}; outputs dL/db' = (dp_r | dp_z | da) in p.h_out and v itself in p.gates_out (the weight gradient's factor),
// 8 = the same with the weight gradient fused in as in 4 and 6,
// 9 = the vanilla cell's forward pass with one 4-byte LDS read per sample instead of one wide read per column (batch 4
// only): the "no wide loads" rung of the ablation (options.gather),
// 10 = the vanilla cell's forward pass with the copy of h consumed in two parts (batch <= 4, no column compaction, at
// most eight copy rounds; options.overlap): every load of the copy goes out at once, the first p.seg_rounds rounds of
// it (the low columns) are stored first, and while the rest is still arriving every wavefront works through the leading
// words of its lanes, which the packer filled with nonzeros of those low columns only (Section 4.2's case for doing
// useful work during the load stage),
// 11 = the vanilla cell's forward pass with h exchanged and kept in LDS as binary16 (batch 4; options.activations;
// Section 6 names lower-precision activations as future work): one 8-byte gather per nonzero, products and sums in
// binary32, every h_t rounded to nearest once before it is published (h_out keeps the unrounded value),
// 12, 13, 14 = the forward passes 0, 1, 2 for a layer whose h takes at most three rounds of the copy (one 16-byte piece
// per lane and round): the copy issues exactly that many loads.  The general code always issues four (rounds past the
// end re-fetch the clamped last piece), which costs a small layer 0.1 us per surplus round; choosing between the two
// inside one kernel cost the four-round layers 3 %, hence separate instantiations.
template <int B, int NW, int CELLX, bool TL>
__global__ __launch_bounds__(NW >= 48 ? 256 : ((CELLX == 4 || CELLX == 6 || CELLX == 8) && NW >= 24 ? 512 : 768)) void persistent_kernel(const KernelArgs p) {
  constexpr bool kShort = CELLX >= 12 && CELLX <= 14;        // forward pass of cell CELLX - 12 for a short h (see the list above)
  constexpr int CELL = kShort ? CELLX - 12 : CELLX;
  constexpr bool LSTM = CELL == 1 || CELL == 2;   // gated cell: four row groups per unit, cell lanes
  constexpr bool LBWD = CELL >= 5 && CELL <= 8;                // backward pass of a gated cell
  constexpr bool GBWD = CELL == 7 || CELL == 8;                // ... of the GRU
  constexpr int NG = GBWD ? 3 : 4;                             // elements of the exchanged vector per hidden unit
  constexpr bool BWD = CELL == 3 || CELL == 4;
  constexpr bool WGRAD = CELL == 4 || CELL == 6 || CELL == 8;
  const int steps = (BWD || LBWD) ? p.T + ((p.dh0 || WGRAD) ? 1 : 0) : p.T;   // the last one pairs delta_1 (dp_1) with h_0
  auto time_of = [&](int s) { return (BWD || LBWD) ? p.T - 1 - s : s; };   // index into x / aux / outputs of step s
  // LDS: [h][abort flags][timeline sums][LSTM hand-over area].  A single workgroup (no exchange) keeps two copies of
  // h and writes h_t straight into the other one; otherwise one copy is enough, because the workgroup barrier
  // before a step's first poll also separates the last gather of step t from the first write of h_t.
  extern __shared__ __align__(16) unsigned char lds[];
  // One-XCD mode (small layers: at most 32 workgroups): the launch holds eight times the workgroups the mapping needs,
  // dealt over the eight XCDs by the dispatcher.  Every workgroup reports the XCD it runs on, waits until all have
  // reported, and the first XCD that received enough of them takes the work; its workgroups number themselves in the
  // order they arrived, all others leave.  The exchange then stays inside one L2: results are published with plain
  // stores (no write-through to the memory side) and read with loads that only miss the per-CU cache.  If no XCD got
  // enough workgroups the launch gives up and flags it in the status word.
  int grid_x = (int)gridDim.x, wg_index = (int)blockIdx.x;
  if (p.one_xcd) {
    grid_x = (int)gridDim.x / 8;
    const uint32_t flags = lds_address(lds);          // two words at the start of LDS, before anything else uses it
    if (threadIdx.x == 0) {
      uint32_t* const cnt = p.ctrl + kCtrlPlacement + 16 * (p.launch_epoch & 1u);
      const uint32_t xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7u;   // XCC_ID
      const uint32_t order = __hip_atomic_fetch_add(cnt + xcc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(cnt + 8, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      int rank = -1, spins = 0;
      bool all_here = true;
      while (__hip_atomic_load(cnt + 8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < gridDim.x) {
        if (++spins > p.spin_limit) { all_here = false; break; }
      }
      int chosen = -1;
      if (all_here) {
        for (int x = 7; x >= 0; --x)
          if (__hip_atomic_load(cnt + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (uint32_t)grid_x) chosen = x;
      }
      if (chosen == (int)xcc && order < (uint32_t)grid_x) rank = (int)order;
      if (chosen < 0 && blockIdx.x == 0) __hip_atomic_fetch_or(p.ctrl + kCtrlStatus, kStatusPlacement, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (blockIdx.x == 0) {   // the other set of counters belongs to the launch before (done) and the one after (not begun)
        uint32_t* const other = p.ctrl + kCtrlPlacement + 16 * ((p.launch_epoch + 1u) & 1u);
        for (int i = 0; i < 9; ++i) __hip_atomic_store(other + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      lds_store_int(flags, rank);
    }
    __syncthreads();
    wg_index = lds_load_int(flags);
    __syncthreads();                                   // (LDS is initialised only after everyone has read the flag)
    if (wg_index < 0) return;
  }
  const bool solo = grid_x == 1;   // no other workgroup to exchange with
  unsigned char* const lds_tail = lds + (solo ? 2 : 1) * p.lds_h_bytes;
  // abort flags, indexed by step parity so that a fast wave's next-step flag cannot be read one step early
  const uint32_t s_abort = lds_address(lds_tail);   // LDS address of the two flags
  unsigned long long* s_tl = reinterpret_cast<unsigned long long*>(lds_tail + 16);

  const int tid = threadIdx.x, lane = tid & 63;
  const int block = blockDim.x, wg = wg_index;
  const int wave = __builtin_amdgcn_readfirstlane(tid) >> 6;
  const int H = p.hidden, L = p.lanes_per_row;
  const int R = LSTM ? 4 * H : H;
  const bool compacted = p.fill_src != nullptr;   // LDS holds only the chunks of h that this workgroup's rows read
  // distance of the two planes of a batch-8 layout inside the LDS copy (the ring always uses H * 16)
  const int plane_bytes = (B == 8 && compacted) ? __builtin_amdgcn_readfirstlane(p.wg_plane[wg]) : H * 16;

  // ---- one-time weight load: NW register slots per lane, all of one row (Section 3.3).
  // Each word is unpacked once into an LDS byte offset and an fp32 value (two registers per nonzero): the
  // hot loop then spends its VALU issue slots on the multiply-adds only.
  const int n_w = __builtin_amdgcn_readfirstlane(p.wave_words[wg * (block >> 6) + wave]);
  // Two-part copy (vanilla forward pass, one plane): the first p.seg_rounds rounds of the copy bring the low columns of
  // h, and the first k_early words of every lane of this wavefront read only those.
  constexpr bool kTwoPart = CELL == 10;
  constexpr bool kHalf = CELL == 11;   // h travels and sits in LDS as binary16: [H][B] halves, 8 bytes per column at batch 4, 16 at batch 8
  static_assert(!kHalf || B == 4 || B == 8, "binary16 activations are built for batch 4 and 8");
  const int k_early = kTwoPart ? __builtin_amdgcn_readfirstlane(p.wave_early[wg * (block >> 6) + wave]) : 0;
  uint32_t w_off[NW];
  float w_val[NW];
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    const uint32_t word = (k < n_w) ? p.words[((size_t)wg * NW + k) * block + tid] : 0u;
    w_off[k] = lds_address(lds) + ((word >> 16) << p.index_shift);   // (the 16-bit index counts columns when byte offsets would not fit)
    w_val[k] = half_bits_to_float(word);
  }
  // After the reduction (reduce_scatter) the first B lanes of a row group each own one sample of the row: they
  // add b'_t and, for vanilla cells, apply g and store the result ("owner lanes").
  // LSTM: the four gate rows of a hidden unit sit in four consecutive groups; the owners hand their
  // pre-activation to "cell lanes" through a small per-wavefront LDS area, so that lane u * B + b owns sample b
  // of the wavefront's unit slot u: one cell update per lane.
  // Lanes that load or store nothing point out of range, where loads return zero and stores are dropped.
  // The GRU uses the same four-row layout with an empty fourth row: its b' has three blocks per sample, its
  // candidate row hands over the recurrent sum (+ b_hn) and b'_n separately (the reset gate multiplies only the
  // former), the latter in the fourth row's slot, and the cell lanes keep h_{t-1} where the LSTM keeps c.
  constexpr bool gru = CELL == 2;
  const int Hu = LBWD ? H / NG : H;            // hidden units (H is the length of the exchanged vector)
  const int Rx = gru ? 3 * H : (LBWD ? Hu : R);   // rows of b' (backward: of e) per sample
  const int row = p.lane_row[(size_t)wg * block + tid];
  const int sample = sample_of_lane<B>(lane);
  const bool owner = row >= 0 && (lane & (L - 1)) < B;
  const int x_voff = (owner && row < Rx) ? (sample * Rx + row) * 4 : kOutOfRange;
  const int gate = LSTM ? (lane / L) & 3 : 0;
  const float bhn = (gru && owner && gate == 2 && p.b_hn) ? p.b_hn[row - 2 * H] : 0.0f;
  int out_voff, ring_voff;
  int cell_unit = -1;
  if constexpr (LSTM) {
    const int cells = (64 / (4 * L)) * B;   // <= 64 because L >= B
    if (lane < cells) {
      const int r = p.lane_row[(size_t)wg * block + (tid & ~63) + (lane / B) * 4 * L];
      cell_unit = r >= 0 ? r % H : -1;
    }
    const int b = lane % B;
    out_voff = cell_unit >= 0 ? (b * H + cell_unit) * 4 : kOutOfRange;
    ring_voff = cell_unit >= 0 ? lds_offset<B>(cell_unit, b, H) : kOutOfRange;
  } else {
    out_voff = owner ? (sample * H + row) * 4 : kOutOfRange;
    // (binary16 activations: the owner of sample 0 stores the row's four elements as one 8-byte piece)
    ring_voff = kHalf ? ((owner && sample == 0) ? row * (B * 2) : kOutOfRange) : (owner ? lds_offset<B>(row, sample, H) : kOutOfRange);
  }
  const __amdgpu_buffer_rsrc_t ring = __builtin_amdgcn_make_buffer_rsrc(p.ring, 0, kRingSlotsDev * p.h_bytes, kBufWord3);
  const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.x), 0, p.T * B * Rx * 4, kBufWord3);
  const __amdgpu_buffer_rsrc_t hbuf = __builtin_amdgcn_make_buffer_rsrc(p.h_out, 0, p.T * B * H * 4, kBufWord3);
  const __amdgpu_buffer_rsrc_t abuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>((BWD || LBWD) ? p.aux : p.x), 0,
                                                                        p.T * B * (LBWD ? 4 * Hu : H) * 4, kBufWord3);
  const int gates_voff = (LBWD && owner) ? (sample * 4 * Hu + row) * 4 : kOutOfRange;   // this lane's first kept gate value
  const __amdgpu_buffer_rsrc_t dbuf = __builtin_amdgcn_make_buffer_rsrc((BWD || LBWD) && p.dh0 ? p.dh0 : p.h_out, 0, B * Hu * 4, kBufWord3);
  // LSTM backward: forward cell states [T][B][Hu], c_0 and dL/dc_0 [B][Hu] (an absent one is an empty buffer: loads
  // give zero, stores are dropped); this lane's element of them, and the distance of two gate blocks in the ring
  const __amdgpu_buffer_rsrc_t cfbuf = __builtin_amdgcn_make_buffer_rsrc(LBWD ? p.c_out : p.h_out, 0, LBWD ? p.T * B * Hu * 4 : 0, kBufWord3);
  const __amdgpu_buffer_rsrc_t c0buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(LBWD && p.c0 ? p.c0 : p.x), 0, (LBWD && p.c0) ? B * Hu * 4 : 0, kBufWord3);
  const __amdgpu_buffer_rsrc_t dc0buf = __builtin_amdgcn_make_buffer_rsrc(LBWD && p.dc0 ? p.dc0 : p.h_out, 0, (LBWD && p.dc0) ? B * Hu * 4 : 0, kBufWord3);
  const int unit_voff = (LBWD && owner) ? (sample * Hu + row) * 4 : kOutOfRange;
  const int gate_ring_bytes = Hu * (B < 4 ? B : 4) * 4;

  // ---- the copy of h into LDS: 16-byte chunks.  In round c a lane copies the chunk at ring offset src to LDS
  // offset dst.  Without compaction LDS mirrors the ring slot: chunk tid + c * block goes to the same offset, and
  // indices past the end are clamped to the last chunk (a few lanes then copy it twice), which keeps that path free
  // of per-lane branches.  With compaction the sources come from the workgroup's copy list, the destinations are
  // consecutive, and an entry past the end of the list is empty (src out of range, dst < 0).
  // The first four rounds have their sources in registers.
  const int n4 = p.h_bytes >> 4;               // 16-byte chunks in a ring slot
  const int last_chunk = n4 - 1;
  const int chunk_rounds = compacted ? p.fill_rows : (n4 + block - 1) / block;
  const uint32_t* const my_list = compacted ? p.fill_src + (size_t)wg * p.fill_rows * block + tid : nullptr;
  auto copy_src = [&](int c) -> int {          // source of round c
    if (compacted) return c < chunk_rounds ? (int)my_list[(size_t)c * block] : kOutOfRange;
    return min(tid + c * block, last_chunk) * 16;
  };
  auto copy_dst = [&](int c, int src) -> int { return compacted ? (src == kOutOfRange ? -1 : (tid + c * block) * 16) : src; };
  int fsrc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) fsrc[c] = copy_src(c);

  // ---- h_0 into LDS copy 0, cell state into registers
  if (tid < 2) lds_store_int(s_abort + 4 * tid, 0);
  if (TL && tid < kTimelineSlots) s_tl[tid] = 0ull;
  if (!compacted) {
    for (int e = tid; e < H * B; e += block) {
      const int j = e / B, b = e % B;
      const float v = p.h0 ? p.h0[(size_t)b * H + j] : 0.0f;
      if constexpr (kHalf) *reinterpret_cast<_Float16*>(lds + (j * B + b) * 2) = (_Float16)v;
      else *reinterpret_cast<float*>(lds + lds_offset<B>(j, b, H)) = v;
    }
  } else {
    // the same chunks the step loop will copy, taken from the caller's [B][H] array
    for (int c = 0; c < chunk_rounds; ++c) {
      const int src = copy_src(c), dst = copy_dst(c, src);
      if (dst < 0) continue;
      if constexpr (kHalf) {                       // eight binary16 elements of the [H][B] slot layout
        halfx8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int f = (src >> 1) + i, j = f / B, b = f % B;
          v[i] = (_Float16)((p.h0 && j < H) ? p.h0[(size_t)b * H + j] : 0.0f);
        }
        *reinterpret_cast<halfx8*>(lds + dst) = v;
        continue;
      }
      f32x4 v;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int f = (src >> 2) + i;             // element of the slot layout: [H][B], or [2][H][4] for batch 8
        const int j = B == 8 ? (f % (H * 4)) / 4 : f / B;
        const int b = B == 8 ? (f / (H * 4)) * 4 + (f & 3) : f % B;
        v[i] = (p.h0 && j < H) ? p.h0[(size_t)b * H + j] : 0.0f;
      }
      *reinterpret_cast<f32x4*>(lds + dst) = v;
    }
  }
  const float* const state0 = gru ? p.h0 : p.c0;
  float c_state = (LSTM && cell_unit >= 0 && state0) ? state0[(size_t)(lane % B) * H + cell_unit] : 0.0f;
  // hand-over area of this wavefront: [unit slot][sample][gate] floats, after the flags and the timeline sums
  float* const stage = reinterpret_cast<float*>(lds_tail + kLdsTailBytes) + (LSTM ? wave * (64 / (4 * L)) * B * 4 : 0);
  const int stage_write = ((lane / (4 * L)) * B + sample) * 4 + ((lane / L) & 3);   // [unit slot][sample][gate]
  const int stage_read = min(lane, (64 / (4 * L)) * B - 1) * 4;

  // b'_t of this row is fetched one step ahead: a first-touch read from HBM takes about as long as a
  // whole timestep, so the load for step t+1 is issued before step t's wait for h_t.
  // (scalar offsets select the timestep and the sample; the host keeps one launch below 1 GiB of x, so an
  // out-of-range lane offset stays out of range whatever scalar offset is added to it)
  float xn = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, x_voff, time_of(0) * B * Rx * 4, 0));
  float an = 0.0f;   // backward pass: forward output h_t of the same element
  if constexpr (BWD) an = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(abuf, x_voff, time_of(0) * B * H * 4, 0));
  // LSTM backward: gate values i, f, g, o and the cell states c_t, c_{t-1} of this lane's (unit, sample), fetched one
  // step ahead like e_t; carry = dc_{t+1} f_{t+1}
  float gn[4] = {0.0f, 0.0f, 0.0f, 0.0f}, c_cur = 0.0f, c_prev = 0.0f, carry = 0.0f;
  auto load_saved = [&](int time) {   // c_cur of this time is the c_prev of the step before
#pragma unroll
    for (int q = 0; q < 4; ++q)
      gn[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(abuf, gates_voff, (time * B * 4 + q) * Hu * 4, 0));
    c_prev = __builtin_bit_cast(float, time > 0 ? __builtin_amdgcn_raw_buffer_load_b32(cfbuf, unit_voff, (time - 1) * B * Hu * 4, 0)
                                                : __builtin_amdgcn_raw_buffer_load_b32(c0buf, unit_voff, 0, 0));
  };
  if constexpr (LBWD) {
    if (p.T > 0) {
      if constexpr (!GBWD) c_cur = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(cfbuf, unit_voff, time_of(0) * B * Hu * 4, 0));
      load_saved(time_of(0));
    }
  }
  // weight gradient: forward output of this lane's row for every sample (h_0 in the extra step), one accumulator per word
  float side[B], gacc[WGRAD ? NW : 1];
  const int row_voff = row >= 0 ? row * 4 : kOutOfRange;
  const __amdgpu_buffer_rsrc_t h0buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(WGRAD && p.bwd_h0 ? p.bwd_h0 : p.x), 0,
                                                                         (WGRAD && p.bwd_h0) ? B * Hu * 4 : 0, kBufWord3);
  // (the vanilla cell's g' and its weight gradient both read the forward outputs: one descriptor serves both)
  const __amdgpu_buffer_rsrc_t sbuf = CELL == 4 ? abuf
                                                : __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(WGRAD ? p.side_src : p.x), 0,
                                                                                    WGRAD ? p.T * B * Hu * 4 : 0, kBufWord3);
  auto load_side = [&](int s) {   // s: step index; rows of step T come from h_0 (an empty buffer returns zeros)
#pragma unroll
    for (int b = 0; b < B; ++b)
      side[b] = __builtin_bit_cast(float, s < p.T ? __builtin_amdgcn_raw_buffer_load_b32(sbuf, row_voff, (time_of(s) * B + b) * Hu * 4, 0)
                                                  : __builtin_amdgcn_raw_buffer_load_b32(h0buf, row_voff, b * Hu * 4, 0));
  };
  if constexpr (WGRAD) {
#pragma unroll
    for (int k = 0; k < NW; ++k) gacc[k] = 0.0f;
    load_side(0);
  }

  __syncthreads();

  const bool tl_on = TL && p.timeline != nullptr && wave == p.tl_wave;
  long long tl_launch_core = 0, tl_launch_wall = 0, tl_clock_cost = 0;
  if (TL && tl_on) {   // cost of reading the clock itself: 16 back-to-back reads
    const long long c0 = wall_clock64();
    long long c1 = c0;
#pragma unroll
    for (int i = 0; i < 15; ++i) c1 = wall_clock64();
    tl_clock_cost = c1 - c0;
    tl_launch_core = (long long)clock64();
    tl_launch_wall = (long long)wall_clock64();
  }

  const uint32_t wave_id = (uint32_t)(wg * (block >> 6) + wave);
  int cur = 0;   // LDS copy that holds h_{t-1}; stays 0 unless solo
  long long tl_prev = 0;
  for (int t = 0; t < steps; ++t) {
    const uint32_t g = p.step_base + (uint32_t)t;         // global step index: the slot number is the timestep tag
    long long ts0 = 0, ts1 = 0, ts2 = 0, ts3 = 0, ts4 = 0, ts5 = 0, ts6 = 0, ts7 = 0;
    unsigned long long repolls = 0;
    float acc[B];
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = 0.0f;
    int k_done = 0;   // words of this step's operate stage already worked through during the copy

    // ---- load: h_{t-1} (published by every workgroup in step t-1) into the other LDS copy
    if (solo) {
      // a single workgroup keeps h in LDS: the owners wrote h_{t-1} straight into the other copy
      if (t > 0) {
        __syncthreads();
        cur ^= 1;
        // the gather offsets follow the copy (only this mapping has two), so the hot loop adds no base
        const uint32_t delta = cur ? (uint32_t)p.lds_h_bytes : 0u - (uint32_t)p.lds_h_bytes;
#pragma unroll
        for (int k = 0; k < NW; ++k) w_off[k] += delta;
      }
    } else if (t > 0) {
      const int slot_byte = (int)((g - 1) & (kRingSlotsDev - 1)) * p.h_bytes;
      unsigned char* dst = lds;
      bool failed = false;
      if (p.sync == SPRNN_SYNC_BARRIER) {
        // grid barrier (Section 3.2): all stores performed, one arrival per workgroup, wait for everyone
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
          // Counters only grow: barrier number n (counted since the handle was created) is complete when its counter
          // reaches n * arrivals.  A small grid arrives at and waits on one counter.  A large one uses two levels, so
          // that no counter sees more than 32 arrivals: workgroup w belongs to group w % 8 (the XCD it is normally
          // dispatched to), the last arrival of a group reports to the top counter, and everybody waits for that.
          const uint32_t n = p.barrier_base + (uint32_t)t;
          uint32_t target;
          if (grid_x < 64) {
            __hip_atomic_fetch_add(p.ctrl + kCtrlBarrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            target = n * (uint32_t)grid_x;
          } else {
            const uint32_t grp = (uint32_t)wg % 8u, members = (uint32_t)grid_x / 8u + (grp < (uint32_t)grid_x % 8u ? 1u : 0u);
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
        __syncthreads();
        failed = __builtin_amdgcn_readfirstlane(lds_load_int(s_abort + 4 * (t & 1))) != 0;   // the same for every lane of the workgroup
      } else {
        // Polling a line before its producer wrote it installs a stale copy in this XCD's L2 that has to be
        // invalidated and fetched again, which costs more than waiting a little too long: back off first.
        // The wavefronts of a workgroup finish a step at different times; they wait for each other here, so that
        // the back-off counts from the moment the whole workgroup has published (the skew inside a workgroup would
        // otherwise have to be covered by a longer back-off in every workgroup).
        __syncthreads();
        for (int d = 0; d < p.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
        jitter_pause(p.jitter, wave_id, g, 1);
      }
      ts4 = tick<TL>(tl_on);
      if constexpr (kTwoPart) {
        if (!failed) {
          // (timeline: slot 5 = first part stored and seen by all, slot 6 = early words + second part)
          const int early = min(k_early, n_w);
#define SPRNN_TWO_PARTS(R)                                                                                                    \
  case R:                                                                                                                     \
    failed = !copy_two_parts<B, NW, R, TL>(ring, slot_byte, tid, block, last_chunk, dst, p.spin_limit, p.ctrl + kCtrlStatus,    \
                                           repolls, p.jitter, wave_id, g, acc, w_off, w_val, early, plane_bytes, tl_on, ts5);   \
    break;
          switch (chunk_rounds) {   // (the host selects this kernel only for 2..8 rounds)
            SPRNN_TWO_PARTS(2) SPRNN_TWO_PARTS(3) SPRNN_TWO_PARTS(4) SPRNN_TWO_PARTS(5)
            SPRNN_TWO_PARTS(6) SPRNN_TWO_PARTS(7) SPRNN_TWO_PARTS(8)
            default: failed = true; break;
          }
#undef SPRNN_TWO_PARTS
          k_done = k_early;
        } else {
          ts5 = ts4;
        }
      } else if (!failed) {   // (after a grid barrier every chunk is valid at the first load)
        if (chunk_rounds <= 4) {
          if (!compacted) {
            if constexpr (kShort) {   // (the host selects these instantiations only for one to three rounds)
              if (chunk_rounds <= 1) {
                const int one[1] = {fsrc[0]};
                failed = !copy_chunks<1, false>(ring, slot_byte, one, one, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
              } else if (chunk_rounds == 2) {
                const int two[2] = {fsrc[0], fsrc[1]};
                failed = !copy_chunks<2, false>(ring, slot_byte, two, two, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
              } else {
                const int three[3] = {fsrc[0], fsrc[1], fsrc[2]};
                failed = !copy_chunks<3, false>(ring, slot_byte, three, three, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
              }
            } else if (kHalf && chunk_rounds <= 2) {
              // half the bytes, half the rounds (see instantiations 12..14 for why the count is matched)
              const int two[2] = {fsrc[0], fsrc[1]};
              failed = !copy_chunks<2, false, kHalf>(ring, slot_byte, two, two, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
            } else {
              failed = !copy_chunks<4, false, kHalf>(ring, slot_byte, fsrc, fsrc, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
            }
          } else {
            int to[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) to[c] = copy_dst(c, fsrc[c]);
            failed = !copy_chunks<4, true, kHalf>(ring, slot_byte, fsrc, to, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
          }
        } else if (!compacted) {
          // a large h or a small workgroup: eight loads per lane in flight, as many rounds as it takes
          for (int r0 = 0; r0 < chunk_rounds && !failed; r0 += 8) {
            int off[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) off[c] = copy_src(r0 + c);
            failed = !copy_chunks<8, false, kHalf>(ring, slot_byte, off, off, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
          }
        } else {
          // the same with a copy list: the sources of the next eight rounds are fetched while this round's data is
          // on its way
          int off[8];
#pragma unroll
          for (int c = 0; c < 8; ++c) off[c] = copy_src(c);
          for (int r0 = 0; r0 < chunk_rounds && !failed; r0 += 8) {
            int to[8], next[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) to[c] = copy_dst(r0 + c, off[c]);
#pragma unroll
            for (int c = 0; c < 8; ++c) next[c] = (r0 + 8 < chunk_rounds) ? copy_src(r0 + 8 + c) : kOutOfRange;
            failed = !copy_chunks<8, true, kHalf>(ring, slot_byte, off, to, dst, p.spin_limit, p.ctrl + kCtrlStatus, repolls);
#pragma unroll
            for (int c = 0; c < 8; ++c) off[c] = next[c];
          }
        }
        ts5 = ts4;
      }
      jitter_pause(p.jitter, wave_id, g, 2);
      ts6 = tick<TL>(tl_on);
      if (failed) {
        lds_store_int(s_abort + 4 * (t & 1), 1);
        __hip_atomic_store(p.ctrl + kCtrlStatus, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();
      // every wave of the workgroup leaves together; other workgroups see the status word
      // (readfirstlane: the flag is the same for every lane, and a scalar exit keeps the loop counter scalar)
      if (__builtin_amdgcn_readfirstlane(lds_load_int(s_abort + 4 * (t & 1)))) break;
      ts7 = tick<TL>(tl_on);
    }
    ts0 = tick<TL>(tl_on);

    // ---- operate
    if constexpr (WGRAD) {
      operate<B, NW, true>(acc, w_off, w_val, n_w, plane_bytes, gacc, &side);
    } else if constexpr (kTwoPart) {
      operate_span<B, NW>(acc, w_off, w_val, k_done, n_w, plane_bytes);
    } else if constexpr (kHalf) {
      operate_half<NW, B>(acc, w_off, w_val, n_w);
    } else {
      // Groups of eight words for batch 4 in the one-row-per-unit layouts (eight gathers in flight, half as many
      // waits for the LDS: 2.5 % on the headline shape); four otherwise: eight would spill at batch 8, measured no
      // better at batch 2 and for vanilla cells at batch 1, 15-20 % slower for the gated cells at batch 1, and at
      // batch 4 a few per cent either way for them depending on the words per lane.
      operate<B, NW, false, (B == 4 && !LSTM) ? 8 : 4, CELL == 9>(acc, w_off, w_val, n_w, plane_bytes);
    }
    ts1 = tick<TL>(tl_on);

    // ---- reduce over the lanes of the row: every lane ends up with the sum of its own sample
    const float red = reduce_rows<B>(acc, L, lane);
    const float pre = red + xn;

    // ---- epilogue and hand-off: publish h_t, write the outputs (only the owners' stores land).
    // The re-arm stores issued one step ago must be performed before this step's data can be seen, hence the wait.
    const int slot_byte = (int)(g & (kRingSlotsDev - 1)) * p.h_bytes;
    const int rearm_byte = (int)((g + 2) & (kRingSlotsDev - 1)) * p.h_bytes;
    const int out_soff = time_of(t) * B * H * 4;
    float hval;
    float kept[4] = {0.0f, 0.0f, 0.0f, 0.0f}, c_new = 0.0f;   // gated cells: values stored after the publish
    if constexpr (LSTM) {
      if (gru) {
        if (owner && gate < 2) stage[stage_write] = pre;
        if (owner && gate == 2) { stage[stage_write] = red + bhn; stage[stage_write + 1] = xn; }
      } else if (owner) {
        stage[stage_write] = pre;
      }
      // LDS serves the operations of one wavefront in order: no hardware barrier between these writes and the
      // read, only a fence that keeps the compiler from moving one across the other
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      const f32x4 gates = *reinterpret_cast<const f32x4*>(stage + stage_read);   // i, f, g, o of this lane's sample
      if (gru) {                                                                 // GRU: p_r, p_z, U_n h + b_hn, b'_n
        const float r = sigmoidf_(gates.x), z = sigmoidf_(gates.y);
        const float n = tanhf_(fmaf(r, gates.z, gates.w));
        hval = fmaf(z, c_state - n, n) + 0.0f;                                   // (1 - z) n + z h_{t-1}
        c_state = hval;
        kept[0] = r; kept[1] = z; kept[2] = n; kept[3] = gates.z;               // r, z, n and q = U_n h + b_hn
      } else {
        const float gi = sigmoidf_(gates.x), gf = sigmoidf_(gates.y), gg = tanhf_(gates.z), go = sigmoidf_(gates.w);
        const float c = gf * c_state + gi * gg;
        c_state = c;
        hval = go * tanhf_(c) + 0.0f;   // + 0.0f: -0.0 -> +0.0 (-0.0 is the "not written" mark)
        c_new = c;
        kept[0] = gi; kept[1] = gf; kept[2] = gg; kept[3] = go;
      }
    } else if constexpr (LBWD) {
      float dp[NG], dx_n = 0.0f;       // dx_n: GRU, gradient of the candidate's pre-activation
#pragma unroll
      for (int q = 0; q < NG; ++q) dp[q] = 0.0f;
      hval = (GBWD ? red + carry : red) + 0.0f;   // the extra step: dL/dh_0 (the GRU adds the update gate's direct path)
      if (t < p.T) {
        if constexpr (GBWD) {
          const float gr = gn[0], gz = gn[1], gc = gn[2], gq = gn[3];
          const float dh = pre + carry;                                  // pre = e_t + U^T v_{t+1}
          dx_n = dh * (1.0f - gz) * fmaf(-gc, gc, 1.0f) + 0.0f;
          dp[0] = dx_n * gq * gr * (1.0f - gr) + 0.0f;                   // + 0.0f: never the "not written" mark
          dp[1] = dh * (c_prev - gc) * gz * (1.0f - gz) + 0.0f;          // c_prev holds h_{t-1}
          dp[2] = dx_n * gr + 0.0f;
          carry = dh * gz;
        } else {
          const float gi = gn[0], gf = gn[1], gg = gn[2], go = gn[3];
          const float tc = tanhf_(c_cur);
          const float dc = fmaf(pre * go, fmaf(-tc, tc, 1.0f), carry);   // pre = dh_t
          dp[0] = dc * gg * gi * (1.0f - gi) + 0.0f;
          dp[1] = dc * c_prev * gf * (1.0f - gf) + 0.0f;
          dp[2] = dc * gi * fmaf(-gg, gg, 1.0f) + 0.0f;
          dp[3] = pre * tc * go * (1.0f - go) + 0.0f;
          carry = dc * gf;
          c_cur = c_prev;
        }
      }
      jitter_pause(p.jitter, wave_id, g, 3);
      if (solo) {
        if (ring_voff != kOutOfRange) {
#pragma unroll
          for (int q = 0; q < NG; ++q) *reinterpret_cast<float*>(lds + (cur ^ 1) * p.lds_h_bytes + ring_voff + q * gate_ring_bytes) = dp[q];
        }
      } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int q = 0; q < NG; ++q)
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, dp[q]), ring, ring_voff, slot_byte + q * gate_ring_bytes, kAuxCoherent);
        if (p.sync == SPRNN_SYNC_TAGGED) {
#pragma unroll
          for (int q = 0; q < NG; ++q)
            __builtin_amdgcn_raw_buffer_store_b32((int)kSentinelBits, ring, ring_voff, rearm_byte + q * gate_ring_bytes, kAuxCoherent);
        }
      }
      if (t < p.T) {
        if constexpr (GBWD) {   // the recurrent sums' gradient for the weight gradient, then dL/db' with da in the third block
          const __amdgpu_buffer_rsrc_t vbuf = __builtin_amdgcn_make_buffer_rsrc(p.gates_out, 0, p.gates_out ? p.T * B * H * 4 : 0, kBufWord3);
#pragma unroll
          for (int q = 0; q < NG; ++q)
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, dp[q]), vbuf, out_voff, out_soff + q * Hu * 4, 0);
          dp[2] = dx_n;
        }
#pragma unroll
        for (int q = 0; q < NG; ++q)
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, dp[q]), hbuf, out_voff, out_soff + q * Hu * 4, 0);
        if (!GBWD && t == p.T - 1) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, carry), dc0buf, unit_voff, 0, 0);   // dL/dc_0 = dc_1 f_1
      } else if (p.dh0) {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), dbuf, unit_voff, 0, 0);
      }
      if (t + 1 < p.T) {
        xn = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, x_voff, time_of(t + 1) * B * Rx * 4, 0));
        load_saved(time_of(t + 1));
      }
    } else if constexpr (BWD) {
      if (t < p.T) {
        const float slope = p.act == SPRNN_ACT_RELU ? (an > 0.0f ? 1.0f : 0.0f) : (p.act == SPRNN_ACT_TANH ? fmaf(-an, an, 1.0f) : 1.0f);
        hval = slope * pre + 0.0f;   // + 0.0f: 0 * negative is -0.0, the "not written" mark
      } else {
        hval = red + 0.0f;           // the extra step: U^T delta_1, no e, no g'
      }
    } else {
      hval = activate(p.act, pre);
    }
    ts2 = tick<TL>(tl_on);
    if constexpr (!LBWD) {   // (the LSTM's backward pass has published its four elements above)
    jitter_pause(p.jitter, wave_id, g, 3);
    if constexpr (kHalf) {
      const int mine = (int)half_bits_for_exchange(hval);
      if constexpr (B == 4) {
        // the four owner lanes of a row are one aligned quad, and lane q of it holds sample sample_of_lane(q) = 0, 2, 1, 3:
        // the owner of sample 0 collects the four rounded values in sample order
        const int s2 = __builtin_amdgcn_update_dpp(0, mine, 0x55, 0xf, 0xf, false);   // quad_perm: lane 1 of the quad (sample 2)
        const int s1 = __builtin_amdgcn_update_dpp(0, mine, 0xAA, 0xf, 0xf, false);   // lane 2 (sample 1)
        const int s3 = __builtin_amdgcn_update_dpp(0, mine, 0xFF, 0xf, 0xf, false);   // lane 3 (sample 3)
        i32x2 pair;
        pair.x = mine | (s1 << 16);
        pair.y = s2 | (s3 << 16);
        if (solo) {
          if (ring_voff != kOutOfRange) *reinterpret_cast<i32x2*>(lds + (cur ^ 1) * p.lds_h_bytes + ring_voff) = pair;
        } else {
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          i32x2 mark;
          mark.x = (int)kSentinelHalfPair;
          mark.y = (int)kSentinelHalfPair;
          if (p.one_xcd) {
            __builtin_amdgcn_raw_buffer_store_b64(pair, ring, ring_voff, slot_byte, 0);
            if (p.sync == SPRNN_SYNC_TAGGED) __builtin_amdgcn_raw_buffer_store_b64(mark, ring, ring_voff, rearm_byte, 0);
          } else {
            __builtin_amdgcn_raw_buffer_store_b64(pair, ring, ring_voff, slot_byte, kAuxCoherent);
            if (p.sync == SPRNN_SYNC_TAGGED) __builtin_amdgcn_raw_buffer_store_b64(mark, ring, ring_voff, rearm_byte, kAuxCoherent);
          }
        }
      } else {
        // the eight owner lanes of a row are two aligned quads of one row of 16 lanes; lane q holds sample
        // sample_of_lane(q) = 0, 4, 2, 6 | 1, 5, 3, 7.  A lane of the first quad pairs its value with the one four lanes
        // up (samples s and s + 1), and the owner of sample 0 collects the four pairs in sample order.
        const int up = __builtin_amdgcn_update_dpp(0, mine, 0x104, 0xf, 0xf, false);   // row_shl:4: the value of lane + 4
        const int both = mine | (up << 16);
        i32x4 column;
        column.x = both;                                                                // samples 0, 1 (lanes 0 and 4)
        column.y = __builtin_amdgcn_update_dpp(0, both, 0xAA, 0xf, 0xf, false);          // lane 2 of the quad: samples 2, 3
        column.z = __builtin_amdgcn_update_dpp(0, both, 0x55, 0xf, 0xf, false);          // lane 1: samples 4, 5
        column.w = __builtin_amdgcn_update_dpp(0, both, 0xFF, 0xf, 0xf, false);          // lane 3: samples 6, 7
        if (solo) {
          if (ring_voff != kOutOfRange) *reinterpret_cast<i32x4*>(lds + (cur ^ 1) * p.lds_h_bytes + ring_voff) = column;
        } else {
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          i32x4 mark;
          mark.x = mark.y = mark.z = mark.w = (int)kSentinelHalfPair;
          if (p.one_xcd) {
            __builtin_amdgcn_raw_buffer_store_b128(column, ring, ring_voff, slot_byte, 0);
            if (p.sync == SPRNN_SYNC_TAGGED) __builtin_amdgcn_raw_buffer_store_b128(mark, ring, ring_voff, rearm_byte, 0);
          } else {
            __builtin_amdgcn_raw_buffer_store_b128(column, ring, ring_voff, slot_byte, kAuxCoherent);
            if (p.sync == SPRNN_SYNC_TAGGED) __builtin_amdgcn_raw_buffer_store_b128(mark, ring, ring_voff, rearm_byte, kAuxCoherent);
          }
        }
      }
    } else if (solo) {
      if (ring_voff != kOutOfRange) *reinterpret_cast<float*>(lds + (cur ^ 1) * p.lds_h_bytes + ring_voff) = hval;
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (p.one_xcd) {   // every workgroup shares one L2: plain stores reach it and need not go further
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), ring, ring_voff, slot_byte, 0);
        if (p.sync == SPRNN_SYNC_TAGGED) __builtin_amdgcn_raw_buffer_store_b32((int)kSentinelBits, ring, ring_voff, rearm_byte, 0);
      } else {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), ring, ring_voff, slot_byte, kAuxCoherent);
        if (p.sync == SPRNN_SYNC_TAGGED) __builtin_amdgcn_raw_buffer_store_b32((int)kSentinelBits, ring, ring_voff, rearm_byte, kAuxCoherent);
      }
    }
    if (BWD && t == p.T) {
      if (p.dh0) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), dbuf, out_voff, 0, 0);
    } else {
      __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, hval), hbuf, out_voff, out_soff, 0);
    }
    if constexpr (LSTM) {
      // The cell state and (training) the kept gate values leave after the publish: the publish waits for every
      // earlier store of the wavefront, and these would sit in front of it.
      if (!gru) {
        const __amdgpu_buffer_rsrc_t cbuf = __builtin_amdgcn_make_buffer_rsrc(p.c_out, 0, p.T * B * H * 4, kBufWord3);
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, c_new), cbuf, out_voff, out_soff, 0);
      }
      if (p.gates_out) {   // [T][B][4H]: i | f | g | o after their activations, or r | z | n | q for the GRU
        const __amdgpu_buffer_rsrc_t gbuf = __builtin_amdgcn_make_buffer_rsrc(p.gates_out, 0, p.T * B * H * 16, kBufWord3);
        const int gate_voff = cell_unit >= 0 ? ((lane % B) * 4 * H + cell_unit) * 4 : kOutOfRange;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, kept[q]), gbuf, gate_voff, out_soff * 4 + q * H * 4, 0);
      }
    }
    if (t + 1 < p.T) {
      xn = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, x_voff, time_of(t + 1) * B * Rx * 4, 0));
      if constexpr (BWD) an = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(abuf, x_voff, time_of(t + 1) * B * H * 4, 0));
    }
    }
    if constexpr (WGRAD) {
      if (t + 1 < steps) load_side(t + 1);
    }
    ts3 = tick<TL>(tl_on);

    if constexpr (TL) {
      if (tl_on && lane == 0) {
        if (t == (p.T >> 1)) {   // absolute times of one step, to compare workgroups with each other
          s_tl[13] = (unsigned long long)ts2;   // results ready, about to publish
          s_tl[14] = (unsigned long long)ts4;   // first poll issued
          s_tl[15] = (unsigned long long)ts7;   // h_{t-1} complete in LDS (after the workgroup barrier)
        }
        s_tl[0] += (unsigned long long)(ts1 - ts0);   // operate (issue)
        s_tl[1] += (unsigned long long)(ts2 - ts1);   // reduce + epilogue arithmetic
        s_tl[2] += (unsigned long long)(ts3 - ts2);   // publish, outputs, re-arm, next b' prefetch
        if (t > 0 && p.sync == SPRNN_SYNC_TAGGED) {
          s_tl[4] += (unsigned long long)(ts4 - tl_prev);   // back-off before the first poll
          s_tl[5] += (unsigned long long)(ts5 - ts4);       // first poll in flight
          s_tl[6] += (unsigned long long)(ts6 - ts5);       // re-polls until every chunk is valid, LDS writes
          s_tl[7] += (unsigned long long)(ts7 - ts6);       // wait for the other waves of the workgroup
          s_tl[8] += repolls;
        }
        s_tl[9] += 1ull;                                    // steps counted
      }
      tl_prev = ts3;
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
  if constexpr (TL) {
    if (tl_on && lane == 0) {
      s_tl[10] = (unsigned long long)tl_clock_cost;
      s_tl[11] = (unsigned long long)((long long)clock64() - tl_launch_core);
      s_tl[12] = (unsigned long long)((long long)wall_clock64() - tl_launch_wall);
#pragma unroll
      for (int i = 0; i < kTimelineSlots; ++i) {
        unsigned long long* dst = p.timeline + (size_t)wg * kTimelineSlots + i;
        *dst = (i >= 13) ? s_tl[i] : *dst + s_tl[i];
      }
    }
  }
}

// ---- instantiation tables: kernel for a batch size and a number of register slots per lane
template <int B, int CELL, bool TL>
static const void* pick_nw(int nw) {
  switch (nw) {
    case 8: return (const void*)persistent_kernel<B, 8, CELL, TL>;
    case 16: return (const void*)persistent_kernel<B, 16, CELL, TL>;
    case 24: return (const void*)persistent_kernel<B, 24, CELL, TL>;
    case 32: return (const void*)persistent_kernel<B, 32, CELL, TL>;
    case 48: return (const void*)persistent_kernel<B, 48, CELL, TL>;
    case 64:   // (with the weight gradient fused in, batch 8 and 64 words per lane no longer fit in registers: not built)
      if constexpr (B == 8 && (CELL == 4 || CELL == 6 || CELL == 8)) return nullptr;
      else return (const void*)persistent_kernel<B, 64, CELL, TL>;
    default: return nullptr;
  }
}

template <int CELL, bool TL>
static const void* pick_b(int batch, int nw) {
  switch (batch) {
    case 1: return pick_nw<1, CELL, TL>(nw);
    case 2: return pick_nw<2, CELL, TL>(nw);
    case 4: return pick_nw<4, CELL, TL>(nw);
    case 8: return pick_nw<8, CELL, TL>(nw);
    default: return nullptr;
  }
}

}  // namespace sprnn
#endif
