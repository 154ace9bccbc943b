// Host-side weight preparation for the persistent sparse recurrent kernel.
//
// Turns a CSR matrix into the per-lane register image the kernel loads once (paper, Section 3.3:
// every lane keeps n <index,value> pairs that all belong to one row; Section 4: rows padded with
// <index,0>; Section 4.1 / Appendix A: the pairs of a row are re-ordered so that the lanes served
// together by one LDS pass fall into different banks).  Pure host C++, no HIP.
#ifndef SPRNN_PACK_H_
#define SPRNN_PACK_H_

#include <cstdint>
#include <vector>

#include "sprnn.h"

namespace sprnn {

constexpr int kWave = 64;          // lanes per wavefront on gfx950
constexpr int kMaxWaves = 12;      // wavefronts per workgroup (768 threads: 168 registers per lane)
constexpr int kRingSlots = 4;      // exchange ring depth
constexpr int kLdsLimit = 160 * 1024;
constexpr uint32_t kSentinel = 0x80000000u;  // -0.0f: "not written yet" (Section 4.2)

// Register slots per lane for which a kernel instantiation exists.
constexpr int kTemplateWords[] = {8, 16, 24, 32, 48, 64};
constexpr int kNumTemplateWords = 6;

struct Mapping {
  int hidden = 0, rows = 0, batch = 0, cell = 0;
  int cols = 0;              // columns of the matrix = length of the exchanged vector (4 * hidden for the LSTM's backward pass, else hidden)
  int grid = 0, waves = 0, row_waves = 0, block = 0, lanes_per_row = 0;   // waves = all, row_waves = those owning rows
  int sync = SPRNN_SYNC_TAGGED, bank_aware = 1, balance = 2, poll_delay = 0, spin_limit = 0, timeline = 0;
  int cooperative = 0;       // 1: cooperative launch instead of an ordinary one
  int jitter = 0;            // test aid: seed of pseudo-random pauses in the hand-off (0 = none)
  int half = 0;              // 1: h is exchanged and kept in LDS as binary16 (options.activations = 2)
  int layout_batch = 0;      // samples' worth of 4-byte elements per column of the LDS copy: batch, or batch / 2 with binary16 activations
  int narrow = 0;            // 1: one 4-byte LDS read per sample instead of one wide read per column (ablation)
  int template_words = 0;    // NW of the kernel instantiation
  int words_max = 0;         // largest per-lane word count actually used
  int col_stride = 0;        // bytes between consecutive columns of h in LDS (4 * min(B, 4))
  int index_shift = 0;       // packed index = (col * col_stride) >> index_shift
  int h_bytes = 0;           // bytes of one copy of h in LDS / one ring slot (multiple of 16)
  int lds_bytes = 0;         // LDS taken by h: h_bytes, 2 * h_bytes for a single workgroup, less with column compaction
  int compact = 0;           // 1: a workgroup copies only the chunks of h that its rows read (see pack())
  int fill_rows = 0;         // compaction: rounds in the per-workgroup copy list
  int stage_bytes = 0;       // LSTM: per-workgroup LDS area through which gate sums reach the cell lanes; lane-pool layout: the group sums
  int seg_words = 0;         // two-part copy: least number of leading slots (over the wavefronts that hold weights) that read only the first part
  int seg_rounds = 0;        // > 0: the copy of h is consumed in two parts, the first seg_rounds rounds of it first (see pack())
  int layout = 0;            // 0: one power-of-two lane group per row; 1: lane pool (see pack_pool): row_waves gather, the others own the outputs
  int group = 0;             // lane pool: lanes per group (= batch); a row takes whole groups
  int64_t nnz = 0, padded_words = 0;
};

struct Packed {
  Mapping map;
  std::vector<uint32_t> words;      // [grid][template_words][block]
  std::vector<int32_t> lane_row;    // [grid][block]  row of W served by the lane, -1 if idle
  std::vector<int32_t> lane_words;  // [grid][block]  real (non-padding) words of the lane
  std::vector<int32_t> wave_words;  // [grid][waves]  loop trip count of each wavefront
  std::vector<int32_t> wave_early;  // two-part copy: [grid][waves] leading slots that only read columns of the first part
  std::vector<uint32_t> fill_src;   // compaction: [grid][fill_rows][block] ring byte offset of each copied chunk (out of range: none)
  std::vector<int32_t> wg_plane;    // compaction: [grid] bytes of one plane of the workgroup's LDS copy
  std::vector<int32_t> word_src;    // [grid][template_words][block] CSR position of the nonzero a packed word holds, -1 for padding
  std::vector<int32_t> lane_sum;    // lane pool: [grid][block] for an output lane: first group of its row | groups of the row << 16
};

// Returns SPRNN_OK or an error code; on success `out` holds the mapping and the image.
int pack(int hidden, int batch, int cell, const int32_t* row_ptr, const int32_t* col_idx,
         const uint16_t* val_bits, const sprnn_options_t* opt, int num_cus, Packed* out);

double lds_pass_factor(const Packed& P);

// CSR checks shared by create and pack_host: shape, monotone row_ptr, strictly increasing in-range
// columns, finite binary16 values.
int validate_csr(int hidden, int batch, int cell, const int32_t* row_ptr, const int32_t* col_idx,
                 const uint16_t* val_bits);

}  // namespace sprnn
#endif
