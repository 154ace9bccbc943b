// Declarations shared by the device code (sprnn_kernels.hip) and the C ABI (sprnn_api.hip).
#ifndef SPRNN_DEVICE_H_
#define SPRNN_DEVICE_H_

#include <hip/hip_runtime.h>

#include <cstdint>

#include "sprnn.h"

namespace sprnn {

constexpr int kRingSlotsDev = 4;                  // exchange ring depth (power of two)
constexpr uint32_t kSentinelBits = 0x80000000u;   // -0.0f marks a ring element that is not written yet
constexpr int kCtrlStatus = 0;                    // ctrl[0]: non-zero once a spin watchdog tripped
constexpr int kCtrlBarrier = 32;                  // grid-barrier mode: ctrl[32] top counter, ctrl[32 + 16 (1 + g)] counter of group g (64 bytes apart)
constexpr int kCtrlPlacement = kCtrlBarrier + 16 * 9;   // one-XCD mode: two sets (launch parity) of 16 words: workgroups seen per XCD [0..7], arrivals [8]
constexpr int kCtrlWords = kCtrlPlacement + 32;
constexpr uint32_t kStatusWatchdog = 1u, kStatusPlacement = 2u;   // bits of the status word
constexpr int kCellBackward = 100;                // persistent_kernel_for: backward pass of a vanilla cell
constexpr int kCellBackwardGrad = 101;            // the same with the weight gradient fused in
constexpr int kCellLstmBackwardGrad = 102;        // backward pass of the LSTM with the weight gradient fused in
constexpr int kCellGruBackwardGrad = 103;         // backward pass of the GRU with the weight gradient fused in
constexpr int kTimelineSlots = 16;                // 64-bit accumulators per workgroup in the phase timeline
constexpr int kLdsTailBytes = 16 + 8 * kTimelineSlots;   // LDS after h: abort flags, timeline sums

struct KernelArgs {
  const uint32_t* words;      // [grid][NW][block] packed <index,value> words
  const int32_t* lane_row;    // [grid][block]
  const int32_t* wave_words;  // [grid][waves]
  const uint32_t* fill_src;   // column compaction: [grid][fill_rows][block] copy list, or null
  const int32_t* wg_plane;    // column compaction: [grid] bytes of one plane of the workgroup's LDS copy
  const int32_t* wave_early;  // two-part copy: [grid][waves] leading slots of a wavefront's lanes that read only the first part, or null
  const int32_t* lane_sum;    // lane-pool layout: [grid][block] for an output lane: first group of its row | groups << 16
  uint32_t* ring;             // [4][h_bytes / 4]
  uint32_t* ctrl;             // [kCtrlWords]
  const float* x;             // [T][B][R]
  const float* h0;            // [B][H] or null
  const float* c0;            // [B][H] or null (LSTM)
  const float* b_hn;          // [H] or null (GRU: recurrent bias of the candidate)
  const float* aux;           // backward pass: forward outputs h_t, [T][B][H]; LSTM backward: gate values, [T][B][4H]
  float* dh0;                 // backward pass: dL/dh_0, [B][H], or null
  const float* bwd_h0;        // backward pass with weight gradient: h_0, [B][H], or null (zeros)
  const float* side_src;      // backward pass with weight gradient: forward outputs h_t, [T][B][H]
  const int32_t* word_src;    // backward pass with weight gradient: packed word -> CSR position (of the handle's matrix)
  float* dU;                  // backward pass with weight gradient: [nnz] sums, in the handle's CSR order
  float* h_out;               // [T][B][H]
  float* c_out;               // [T][B][H] (LSTM; its backward pass reads the forward cell states from here)
  float* gates_out;           // LSTM forward: [T][B][4H] gate values after their activations, or null (not kept)
  float* dc0;                 // LSTM backward: dL/dc_0, [B][H], or null
  unsigned long long* timeline;  // [grid][16] phase accumulators in wall-clock ticks, or null (off)
  int hidden, T, lanes_per_row, act, h_bytes, poll_delay, spin_limit, sync;
  int fill_rows;              // rounds in the copy list (column compaction)
  int lds_h_bytes;            // bytes of one LDS copy of h (= h_bytes without column compaction)
  int jitter;                 // test aid: seed of pseudo-random pauses (0 = none)
  int tl_wave;                // phase timeline: the wavefront of every workgroup that records it
  int one_xcd;                // 1: the launch has 8 x the workgroups, those of one XCD take the work (see persistent_kernel)
  uint32_t launch_epoch;      // launches of this handle so far (parity selects the placement counters)
  int seg_rounds;             // > 0: the copy of h is consumed in two parts, its first seg_rounds rounds first (see persistent_kernel)
  int gather_waves;           // lane-pool layout: wavefronts of a workgroup that hold weights (the others own the outputs)
  int index_shift;            // LDS byte offset of a packed word = (word >> 16) << index_shift
  uint32_t step_base;         // global index of the first step of this call (ring slot = index mod 4)
  uint32_t barrier_base;      // grid barriers completed before this call (step t waits at barrier number barrier_base + t)
};

// Weight gradient of a vanilla cell on the sparsity pattern: dU[k] = sum_t sum_b delta_t[b][row(k)] h_{t-1}[b][col(k)].
struct WGradArgs {
  const uint32_t* words;      // the handle's packed words (only the column offsets are used)
  const int32_t* lane_row;    // [grid][block]
  const int32_t* wave_words;  // [grid][waves]
  const int32_t* word_src;    // [grid][NW][block] CSR position of each packed word, -1 for padding
  const float* delta;         // [T][B][rows]
  const float* h_fwd;         // [T][B][H] forward outputs h_1..h_T
  const float* h0;            // [B][H] or null (zeros)
  float* dU;                  // [nnz] CSR order
  int hidden, T, index_shift;
  int rows;                   // rows of the matrix: hidden, or 4 * hidden for the LSTM
};

struct StepArgs {
  const int32_t* row_ptr;
  const int32_t* col;
  const uint16_t* val;
  const float* x_t;     // [B][R]
  const float* h_prev;  // [B][H] or null
  const float* c_prev;  // [B][H] or null
  float* h_cur;         // [B][H]
  float* c_cur;         // [B][H]
  int hidden, act;
};

const void* persistent_kernel_for(int batch, int template_words, int cell, bool timeline);   // cell: SPRNN_ACT_* / SPRNN_CELL_*
// (the instantiations live in four translation units; persistent_kernel_for forwards to these three)
const void* persistent_timeline_kernel_for(int batch, int template_words, bool lstm);        // forward pass with the phase timeline
const void* persistent_overlap_kernel_for(int batch, int template_words, bool timeline);     // vanilla forward with the copy of h consumed in two parts (batch <= 4; timeline: batch 4)
const void* persistent_short_kernel_for(int batch, int template_words, int cell);              // forward pass of a layer whose h takes at most three copy rounds
const void* persistent_half_kernel_for(int batch, int template_words);                       // vanilla forward with h exchanged as binary16 (batch 4, 8)
const void* persistent_narrow_kernel_for(int batch, int template_words);                     // vanilla forward, batch 4, 4-byte gathers (ablation)
const void* persistent_backward_kernel_for(int batch, int template_words, int cell);         // kCellBackward, kCellBackwardGrad
const void* persistent_gated_backward_kernel_for(int batch, int template_words, int cell);   // SPRNN_CELL_*_BACKWARD, kCell{Lstm,Gru}BackwardGrad
hipError_t launch_stepwise(int batch, bool lstm, const StepArgs& a, hipStream_t stream);
// b'[m][n] = sum_k x[m][k] W[n][k] + bias[n] (bias may be null); x [M][K] float32, w [N][K] binary16 bits, out [M][N] float32.
hipError_t launch_project(const float* x, const uint16_t* w, const float* bias, float* out, int M, int N, int K,
                          hipStream_t stream);
const void* pool_kernel_for(int batch, int template_words, int cell, bool timeline = false);                         // lane-pool layout: SPRNN_ACT_*, kCellBackward, kCellBackwardGrad
const void* weight_grad_kernel_for(int batch, int template_words);
hipError_t launch_fill(uint32_t* dst, uint32_t value, size_t n, hipStream_t stream);
// Put an exchange ring and its control words into the state a new handle starts from: the first `used_words` 32-bit
// elements of each of the `slots` slots (of `slot_words` each) carry the "not written" mark, the rest of a slot is
// zero, the control words are zero.
hipError_t launch_exchange_reset(uint32_t* ring, size_t slot_words, size_t used_words, int slots, uint32_t* ctrl, int ctrl_words,
                                 hipStream_t stream);

}  // namespace sprnn
#endif
