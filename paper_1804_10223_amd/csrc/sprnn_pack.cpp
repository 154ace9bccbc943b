// Host-side weight preparation: CSR -> per-lane register image (see sprnn_pack.h).
#include "sprnn_pack.h"

#include <algorithm>
#include <cstring>
#include <atomic>
#include <new>
#include <numeric>
#include <thread>

namespace sprnn {

static inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
static inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// Gate rows per hidden unit in the caller's matrix; the gated cells are laid out with four row groups per unit
// (the GRU leaves the fourth one empty).
static int visible_gates(int cell) { return cell == SPRNN_CELL_LSTM ? 4 : (cell == SPRNN_CELL_GRU ? 3 : 1); }
static bool gated(int cell) { return cell == SPRNN_CELL_LSTM || cell == SPRNN_CELL_GRU; }
// Columns of the matrix = length of the vector the workgroups exchange.  The backward pass of the LSTM holds the
// transposed matrix: one row per hidden unit over the 4H gate gradients (3H for the GRU).
static int exchange_cols(int cell, int hidden) {
  return cell == SPRNN_CELL_LSTM_BACKWARD ? 4 * hidden : (cell == SPRNN_CELL_GRU_BACKWARD ? 3 * hidden : hidden);
}

int validate_csr(int hidden, int batch, int cell, const int32_t* row_ptr, const int32_t* col_idx,
                 const uint16_t* val_bits) {
  if (hidden < 1) return SPRNN_ERR_INVALID;
  if (hidden > 65535) return SPRNN_ERR_UNSUPPORTED;
  if (exchange_cols(cell, hidden) > 65535) return SPRNN_ERR_UNSUPPORTED;   // 16-bit column indices
  if (!(batch == 1 || batch == 2 || batch == 4 || batch == 8)) return SPRNN_ERR_UNSUPPORTED;
  if (cell < SPRNN_ACT_RELU || cell > SPRNN_CELL_GRU_BACKWARD) return SPRNN_ERR_INVALID;
  if (!row_ptr) return SPRNN_ERR_INVALID;
  const int rows = hidden * visible_gates(cell), cols = exchange_cols(cell, hidden);
  if (row_ptr[0] != 0) return SPRNN_ERR_INVALID;
  for (int r = 0; r < rows; ++r) {
    if (row_ptr[r + 1] < row_ptr[r]) return SPRNN_ERR_INVALID;
    if (row_ptr[r + 1] - row_ptr[r] > cols) return SPRNN_ERR_INVALID;
  }
  const int64_t nnz = row_ptr[rows];
  if (nnz > 0 && (!col_idx || !val_bits)) return SPRNN_ERR_INVALID;
  for (int r = 0; r < rows; ++r) {
    int32_t prev = -1;
    for (int32_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      const int32_t c = col_idx[k];
      if (c <= prev || c >= cols) return SPRNN_ERR_INVALID;  // in range, strictly increasing, no duplicates
      prev = c;
      if ((val_bits[k] & 0x7C00u) == 0x7C00u) return SPRNN_ERR_INVALID;  // inf / NaN weight
    }
  }
  return SPRNN_OK;
}

// Which lanes of a wavefront the LDS of gfx950 serves together in one pass of a gather, and how many bank classes a
// gather of that width can fall into (64 banks x 4 bytes = 256 bytes per pass), as measured with pairs of lanes that
// read different addresses of one class (sprnn_probe_lds_gather_offsets):
//   16-byte reads: four passes of 16 lanes.  A half of the wavefront (32 lanes = 8 groups of four lanes) is served as the
//                  groups {0, 3, 5, 6} and then {1, 2, 4, 7}: the order in which 64 consecutive 16-byte pieces fall into
//                  all 64 banks twice over.  16 classes (column mod 16).
//   8-byte reads:  two passes, the lower and the upper 32 lanes; 32 classes.
//   4-byte reads:  the same two passes; 64 classes (a 4-byte gather runs at half the bytes per clock of the wider ones).
// Lanes of a pass that read different addresses of one class serialise; the same address is served once.
struct PassModel {
  int npass = 0, classes = 0;
  int pass_of[kWave];
  std::vector<int> lanes[4];
};
static PassModel make_pass_model(int batch) {
  PassModel pm;
  pm.npass = batch >= 4 ? 4 : 2;
  pm.classes = batch >= 4 ? 16 : (batch == 2 ? 32 : 64);
  for (int lane = 0; lane < kWave; ++lane) {
    int p = lane / 32;
    if (batch >= 4) {
      const int quad = (lane % 32) / 4;
      const bool first = quad == 0 || quad == 3 || quad == 5 || quad == 6;
      p = (lane / 32) * 2 + (first ? 0 : 1);
    }
    pm.pass_of[lane] = p;
    pm.lanes[p].push_back(lane);
  }
  return pm;
}

static int choose_mapping(int hidden, int batch, int cell, const std::vector<int>& row_nnz, const sprnn_options_t* opt,
                          int num_cus, Mapping* m) {
  const bool lstm = gated(cell);                 // four row groups per unit
  const int rows = hidden * (lstm ? 4 : 1);      // rows of the layout (row_nnz has this many entries)
  const int lmax = lstm ? 16 : kWave;
  int maxnnz = 1;
  int64_t nnz = 0;
  for (int r = 0; r < rows; ++r) { maxnnz = std::max(maxnnz, row_nnz[r]); nnz += row_nnz[r]; }
  if (num_cus < 1) return SPRNN_ERR_INVALID;

  auto total_waves = [&](int L) {
    const int groups_per_wave = kWave / L;
    const int units_per_wave = lstm ? groups_per_wave / 4 : groups_per_wave;
    return ceil_div(hidden, units_per_wave);   // a unit is one row (vanilla) or one hidden unit's 4 gate rows
  };

  // The reduction leaves one sample per lane, so a row needs at least `batch` lanes.
  const int lmin = batch;
  int L = opt ? opt->lanes_per_row : 0;
  if (L != 0) {
    if (!is_pow2(L) || L > lmax || L < lmin) return SPRNN_ERR_INVALID;
  } else {
    L = lmax;
    while (L > lmin && ceil_div(maxnnz, L) < 8) L /= 2;
    while (L > lmin && total_waves(L) > (int64_t)kMaxWaves * num_cus) L /= 2;
    while (L < lmax && ceil_div(maxnnz, L) > kTemplateWords[kNumTemplateWords - 1]) L *= 2;
  }
  const int need = ceil_div(maxnnz, L);
  if (need > kTemplateWords[kNumTemplateWords - 1]) return SPRNN_ERR_CAPACITY;
  int tw = 0;
  for (int i = 0; i < kNumTemplateWords; ++i) if (kTemplateWords[i] >= need) { tw = kTemplateWords[i]; break; }

  const int wt = total_waves(L);
  const int wave_cap = tw >= 48 ? 4 : kMaxWaves;   // the 48/64-slot kernels are built for at most 256 threads
  int waves = opt ? opt->waves : 0;
  int grid = opt ? opt->grid : 0;
  if (waves < 0 || waves > kMaxWaves || grid < 0) return SPRNN_ERR_INVALID;
  if (grid && !waves) waves = ceil_div(wt, grid);
  if (!waves) {
    // Eight wavefronts per workgroup copy h into LDS efficiently; but when the gathers of one step would keep a
    // CU's LDS busy for long (about 0.25 us: 600 clocks), spreading the rows over more CUs with four wavefronts
    // each is faster.  LDS clocks per step and CU ~ nonzeros * passes per gather / 64 lanes / workgroups.
    waves = std::min(wave_cap, std::max(ceil_div(wt, num_cus), std::min(8, wt)));
    if (!grid) {
      const int passes = (batch >= 4 ? 4 : batch) * (batch == 8 ? 2 : 1);
      auto lds_clocks = [&](int w) { return (double)nnz * passes * 1.3 / 64.0 / ceil_div(wt, w); };
      while (waves > 4 && ceil_div(wt, waves / 2) <= num_cus && lds_clocks(waves) > 600.0) waves /= 2;
    }
  }
  if (waves > wave_cap) return SPRNN_ERR_CAPACITY;
  if (!grid) grid = ceil_div(wt, waves);
  if ((int64_t)grid * waves < wt) return SPRNN_ERR_CAPACITY;

  m->hidden = hidden; m->rows = hidden * visible_gates(cell); m->batch = batch; m->cell = cell;
  m->cols = exchange_cols(cell, hidden);
  const int activations = opt ? opt->activations : 0;
  if (activations < 0 || activations > 2) return SPRNN_ERR_INVALID;
  m->half = activations == 2 ? 1 : 0;
  if (m->half && ((batch != 4 && batch != 8) || cell > SPRNN_ACT_IDENTITY)) return SPRNN_ERR_UNSUPPORTED;
  // binary16 activations: a column of h is batch x 2 bytes, which is the geometry of binary32 activations at half the batch
  const int lb = m->half ? batch / 2 : batch;
  m->layout_batch = lb;
  m->col_stride = 4 * std::min(lb, 4);
  const int64_t plane = (int64_t)m->cols * m->col_stride;         // batch 8 keeps two planes of 4 samples
  const int64_t hb = ((plane * (lb == 8 ? 2 : 1)) + 15) / 16 * 16;
  // Wavefronts beyond the ones that own rows only help with copying h into LDS (more loads in flight).  Where the
  // row owners alone would need more than four rounds of 16-byte loads for it, the workgroup is filled up to eight
  // wavefronts (measured on the LSTM shapes: 2.51 -> 2.37 us per step forward, 4.4 -> 3.5 backward; more than eight
  // lose again to the workgroup barriers).
  int total = waves;
  if (opt && opt->fill_waves > 0) {
    if (opt->fill_waves > wave_cap) return SPRNN_ERR_INVALID;
    total = std::max(waves, opt->fill_waves);
  } else if ((!opt || opt->waves == 0) && grid > 1 && waves < 8 && wave_cap >= 8 && hb / 16 > (int64_t)waves * kWave * 4) {
    total = 8;
  }
  m->grid = grid; m->row_waves = waves; m->waves = total; m->block = total * kWave; m->lanes_per_row = L;
  m->template_words = tw;
  m->stage_bytes = lstm ? total * (kWave / (4 * L)) * batch * 16 : 0;   // [wave][unit slot][sample][4 gates] floats
  if (hb * kRingSlots > ((int64_t)1 << 30)) return SPRNN_ERR_CAPACITY;
  m->h_bytes = (int)hb;       // the LDS footprint of h and the index scaling are settled by pack() (column compaction)
  int compact = opt ? opt->compact : 0;
  if (compact < 0 || compact > 2) return SPRNN_ERR_INVALID;
  m->compact = compact;       // still the request here: 0 auto, 1 on, 2 off
  m->nnz = nnz;
  m->sync = (opt && opt->sync) ? opt->sync : SPRNN_SYNC_TAGGED;
  if (m->sync != SPRNN_SYNC_TAGGED && m->sync != SPRNN_SYNC_BARRIER) return SPRNN_ERR_INVALID;
  m->bank_aware = (opt && opt->bank_aware) ? opt->bank_aware : 1;
  if (m->bank_aware != 1 && m->bank_aware != 2) return SPRNN_ERR_INVALID;
  int balance = opt ? opt->balance : 0;
  if (balance < 0 || balance > 2) return SPRNN_ERR_INVALID;
  // Contiguous rows publish whole cache lines per workgroup; dealing rows by nonzero count scatters a workgroup's
  // rows over the exchange ring.  On the measured shapes the scatter costs more than about 15 % of zero padding
  // saves, so rows are only dealt by count when the longest row exceeds the mean by more than a quarter.
  const int64_t real_rows = (int64_t)hidden * visible_gates(cell);   // the GRU's empty fourth rows do not count
  if (balance == 0) balance = ((int64_t)maxnnz * real_rows > nnz + nnz / 4 + real_rows) ? 1 : 2;
  m->balance = balance;
  m->poll_delay = opt ? opt->poll_delay : 0;
  m->spin_limit = (opt && opt->spin_limit > 0) ? opt->spin_limit : (1 << 22);
  m->timeline = (opt && opt->timeline) ? 1 : 0;
  if (opt && (opt->launch < 0 || opt->launch > 2)) return SPRNN_ERR_INVALID;
  m->cooperative = (opt && opt->launch == 2) ? 1 : 0;
  m->jitter = opt ? opt->jitter : 0;
  m->narrow = (opt && opt->gather == 2) ? 1 : 0;
  if (opt && (opt->gather < 0 || opt->gather > 2)) return SPRNN_ERR_INVALID;
  if (m->narrow && (batch != 4 || cell > SPRNN_ACT_IDENTITY || m->timeline)) return SPRNN_ERR_UNSUPPORTED;
  if (m->half && (m->narrow || m->timeline)) return SPRNN_ERR_UNSUPPORTED;
  return SPRNN_OK;
}

namespace {
struct Nz { int32_t col; uint16_t bits; };
}

struct RowGroup {
  int lane0 = 0;              // first lane of the group inside the wavefront
  int row = -1;               // weight row, -1 for an idle group
  std::vector<Nz> items;      // the row's nonzeros in CSR order
  std::vector<int> pos;       // [trip * L] position k * L + l -> index into items, -1 = filler
};

// Place the nonzeros of all rows of one wavefront into their lanes' register slots.
//
// Bank-aware ordering (Section 4.1; Appendix A gives one greedy way for 32 banks, this is another for the
// same goal on this LDS).  All the hardware cares about is which columns are read together in one LDS pass:
// a pass serves a fixed set of lanes of one gather instruction (= one slot k; see PassModel) and takes as many
// cycles as the largest number of different addresses that fall into one bank class (column mod classes).
// A nonzero may sit in any slot and any lane of its own row, so the nonzeros are dealt class by
// class (largest class first) to the pass, among those that contain lanes of the row and still have room,
// where they add no cycle, else to the emptiest one.  Surplus nonzeros of over-full classes thereby pile
// into the same few passes, and a row that owns whole passes reaches max(largest class, passes) cycles,
// the lower bound.  Rows that share a pass are scheduled against the same pass state.
// A run of lanes of one wavefront that holds (part of) one row.
namespace {
struct Seg {
  int lane0 = 0, n = 0;       // lanes [lane0, lane0 + n) of the wavefront
  int row = -1;
  int first = 0;              // CSR position of items[0]
  std::vector<Nz> items;      // the part of the row held by these lanes, in CSR order
  std::vector<int> pos;       // [trip * n] slot k, lane j -> index into items, -1 = filler
};
}  // namespace

// LDS cycles one wavefront needs for its `trip` gathers under the pass model.
static int64_t segs_cycles(const std::vector<Seg>& segs, int trip, const PassModel& pm) {
  int64_t total = 0;
  std::vector<std::vector<int32_t>> seen(pm.classes);
  for (int k = 0; k < trip; ++k)
    for (int p = 0; p < pm.npass; ++p) {
      for (auto& v : seen) v.clear();
      for (const Seg& q : segs)
        for (int j = 0; j < q.n; ++j) {
          if (pm.pass_of[q.lane0 + j] != p) continue;
          const int i = q.pos[(size_t)k * q.n + j];
          if (i < 0) continue;   // fillers are given a free bank class afterwards
          auto& v = seen[q.items[i].col % pm.classes];
          if (std::find(v.begin(), v.end(), q.items[i].col) == v.end()) v.push_back(q.items[i].col);
        }
      size_t worst = 1;
      for (auto& v : seen) worst = std::max(worst, v.size());
      total += (int64_t)worst;
    }
  return total;
}

static void order_segments(std::vector<Seg>& segs, int trip, const PassModel& pm, bool bank_aware) {
  for (auto& q : segs) {
    q.pos.assign((size_t)trip * q.n, -1);
    for (int i = 0; i < (int)q.items.size(); ++i) q.pos[i] = i;   // CSR order: item i -> lane i % n, slot i / n
  }
  if (!bank_aware || trip == 0) return;
  const int64_t csr_cycles = segs_cycles(segs, trip, pm);
  std::vector<std::vector<int>> csr_pos(segs.size());
  for (size_t q = 0; q < segs.size(); ++q) { csr_pos[q] = segs[q].pos; segs[q].pos.assign((size_t)trip * segs[q].n, -1); }
  const int classes = pm.classes, np = pm.npass;
  const int P = trip * np;                         // passes of this wavefront: index k * np + p
  std::vector<int> pass_cycles(P, 0), pass_load(P, 0), mult((size_t)P * classes, 0);
  std::vector<int64_t> class_total(classes, 0);
  std::vector<std::vector<std::vector<int>>> bucket(segs.size(), std::vector<std::vector<int>>(classes));
  std::vector<std::vector<int>> taken(segs.size());
  std::vector<std::vector<std::vector<int>>> mine(segs.size(), std::vector<std::vector<int>>(np));   // lanes of a segment (as offsets into it) per pass
  for (size_t q = 0; q < segs.size(); ++q) {
    taken[q].assign((size_t)trip * np, 0);
    for (int j = 0; j < segs[q].n; ++j) mine[q][pm.pass_of[segs[q].lane0 + j]].push_back(j);
    for (int i = (int)segs[q].items.size() - 1; i >= 0; --i) {
      bucket[q][segs[q].items[i].col % classes].push_back(i);
      class_total[segs[q].items[i].col % classes] += 1;
    }
  }
  std::vector<int> order(classes);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return class_total[a] > class_total[b]; });
  for (int g : order)
    for (size_t q = 0; q < segs.size(); ++q) {
      const Seg& sg = segs[q];
      while (!bucket[q][g].empty()) {
        int best_k = -1, best_p = 0, best_cost = 0, best_load = 0;
        for (int k = 0; k < trip; ++k)
          for (int p = 0; p < np; ++p) {
            if (taken[q][(size_t)k * np + p] >= (int)mine[q][p].size()) continue;
            const int at = k * np + p;
            const int cost = (mult[(size_t)at * classes + g] + 1 > pass_cycles[at]) ? 1 : 0;
            if (best_k < 0 || cost < best_cost || (cost == best_cost && pass_load[at] < best_load)) {
              best_k = k; best_p = p; best_cost = cost; best_load = pass_load[at];
            }
          }
        const int i = bucket[q][g].back();   // (a segment never holds more than trip * n nonzeros: a free lane exists)
        bucket[q][g].pop_back();
        const int at = best_k * np + best_p;
        int& used = taken[q][(size_t)best_k * np + best_p];
        segs[q].pos[(size_t)best_k * sg.n + mine[q][best_p][used]] = i;
        used += 1;
        pass_load[at] += 1;
        const int mcount = ++mult[(size_t)at * classes + g];
        pass_cycles[at] = std::max(pass_cycles[at], mcount);
      }
    }
  // the greedy deal is not optimal when many short rows share a pass: never do worse than CSR order
  if (segs_cycles(segs, trip, pm) > csr_cycles)
    for (size_t q = 0; q < segs.size(); ++q) segs[q].pos = csr_pos[q];
}

// Place the nonzeros of all rows of one wavefront of the one-group-per-row layout: every row group is one segment.
static void order_wave(std::vector<RowGroup>& rg, int L, int trip, const PassModel& pm, bool bank_aware) {
  std::vector<Seg> segs(rg.size());
  for (size_t q = 0; q < rg.size(); ++q) { segs[q].lane0 = rg[q].lane0; segs[q].n = L; segs[q].row = rg[q].row; segs[q].items = rg[q].items; }
  order_segments(segs, trip, pm, bank_aware);
  for (size_t q = 0; q < rg.size(); ++q) rg[q].pos = std::move(segs[q].pos);
}

// Two-phase order for the overlap of the copy with the gathers (Section 4.2 wants useful work while the load stage is
// still in flight): the columns below seg_col reach LDS first, and slots [0, k1) of every lane may only hold nonzeros
// of those columns (or fillers), so that a wavefront can work through them while the rest of h is still on its way.
// Largest k1 (a multiple of four, the gathers' group size) that needs no extra slot: what a row cannot place in the
// first k1 slots must fit into the other trip - k1.
static int phase_words(const std::vector<RowGroup>& rg, int L, int trip, int seg_col) {
  int k1 = trip / 4 * 4;
  for (const RowGroup& q : rg) {
    if (q.row < 0) continue;
    int n0 = 0;
    for (const Nz& z : q.items) n0 += z.col < seg_col ? 1 : 0;
    const int n = (int)q.items.size();
    while (k1 > 0 && n - std::min(n0, k1 * L) > (trip - k1) * L) k1 -= 4;
  }
  return k1;
}

static void order_wave_phased(std::vector<RowGroup>& rg, int L, int trip, int k1, int seg_col, const PassModel& pm, bool bank_aware) {
  std::vector<Seg> early(rg.size()), late(rg.size());
  std::vector<std::vector<int>> early_of(rg.size()), late_of(rg.size());   // index into the row's items
  for (size_t q = 0; q < rg.size(); ++q) {
    early[q].lane0 = late[q].lane0 = rg[q].lane0;
    early[q].n = late[q].n = L;
    early[q].row = late[q].row = rg[q].row;
    for (int i = 0; i < (int)rg[q].items.size(); ++i) {
      const bool first = rg[q].items[i].col < seg_col && (int)early_of[q].size() < k1 * L;
      (first ? early_of[q] : late_of[q]).push_back(i);
      (first ? early[q] : late[q]).items.push_back(rg[q].items[i]);
    }
  }
  order_segments(early, k1, pm, bank_aware);
  order_segments(late, trip - k1, pm, bank_aware);
  for (size_t q = 0; q < rg.size(); ++q) {
    rg[q].pos.assign((size_t)trip * L, -1);
    for (int k = 0; k < trip; ++k)
      for (int l = 0; l < L; ++l) {
        const int i = k < k1 ? early[q].pos[(size_t)k * L + l] : late[q].pos[(size_t)(k - k1) * L + l];
        if (i >= 0) rg[q].pos[(size_t)k * L + l] = k < k1 ? early_of[q][i] : late_of[q][i];
      }
  }
}

// Filler words should not add bank conflicts: give each one a column whose bank group is still free in
// its pass (or, failing that, an address that another lane of the pass already reads: a broadcast).
static void place_fillers(Packed& P, const std::vector<int>& wg_cols, const std::vector<char>& is_real_zero) {
  const Mapping& m = P.map;
  const int NW = m.template_words;
  const PassModel pm = make_pass_model(m.layout_batch ? m.layout_batch : m.batch);
  const int classes = pm.classes;
  for (int wg = 0; wg < m.grid; ++wg)
    for (int wave = 0; wave < m.waves; ++wave) {
      const int trip = P.wave_words[(size_t)wg * m.waves + wave];
      for (int k = 0; k < trip; ++k)
        for (int p = 0; p < pm.npass; ++p) {
          std::vector<char> used(classes, 0);
          const size_t base = ((size_t)wg * NW + k) * m.block + (size_t)wave * kWave;
          std::vector<int> fillers;
          uint32_t some_addr = 0; bool have_addr = false;
          for (int l : pm.lanes[p]) {
            const uint32_t w = P.words[base + l];
            if ((w & 0x7FFFu) == 0) { fillers.push_back(l); continue; }   // zero value: a filler, or a stored zero (kept below)
            used[((w >> 16) << m.index_shift) / m.col_stride % classes] = 1;
            some_addr = w >> 16; have_addr = true;
          }
          int g = 0;
          for (int l : fillers) {
            if (is_real_zero[base + l]) {
              used[((P.words[base + l] >> 16) << m.index_shift) / m.col_stride % classes] = 1;
              continue;
            }
            while (g < classes && (used[g] || g >= wg_cols[wg])) ++g;
            if (g < classes) {
              P.words[base + l] = (uint32_t)(((uint32_t)g * (uint32_t)m.col_stride) >> m.index_shift) << 16;
              used[g] = 1;
            } else {
              P.words[base + l] = have_addr ? (some_addr << 16) : 0u;
            }
          }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Lane-pool layout (vanilla cells, more than one workgroup).
//
// The gathering wavefronts of a workgroup form one pool of lanes.  A row takes as many GROUPS of `batch` lanes as its
// nonzeros need at NW words per lane, anywhere in the pool (groups of one row are consecutive and may straddle
// wavefronts); all words of a lane still belong to one row (Section 3.3), and a ragged matrix balances by itself
// because a longer row simply takes more groups (Section 6's load balancing by nonzero count, without sorting rows).
// The lanes of a group reduce among themselves (one sample per lane), the group sums meet in LDS, and OUTPUT lanes in
// separate wavefronts (lane e -> row e / batch of the workgroup, sample e % batch) add them up, add b', apply g and do
// every store.  The gathering wavefronts therefore issue no global memory operation but the polls of the exchange
// ring, so that no poll ever queues behind a store or a b' fetch of its own wavefront.
// Returns SPRNN_OK, or SPRNN_ERR_CAPACITY when the matrix does not suit this layout (the caller then uses the other one).
static int pack_pool(int hidden, int batch, int cell, const int32_t* row_ptr, const int32_t* col_idx,
                     const uint16_t* val_bits, const sprnn_options_t* opt, int num_cus, Packed* out) {
  const int rows = hidden, cols = hidden, G = batch;
  const int64_t nnz = row_ptr[rows];
  if (num_cus < 1) return SPRNN_ERR_INVALID;
  if (opt && (opt->compact == 1 || opt->lanes_per_row || opt->fill_waves || opt->balance == 1 || opt->gather == 2)) return SPRNN_ERR_CAPACITY;
  constexpr int kMaxWavesPool = 8;      // gathering + output wavefronts of one workgroup (512 threads: 256 registers per lane)
  constexpr int64_t kRowCost = 8;       // what an (even empty) row adds to a workgroup's share besides its nonzeros
  const int max_rows_wg = (kMaxWavesPool - 4) * kWave / batch;   // output lanes for them must fit beside four gathering wavefronts

  // --- workgroups: enough of them that the gathers of a step are short, few enough that every one has work
  int grid = opt ? opt->grid : 0;
  if (grid < 0) return SPRNN_ERR_INVALID;
  if (!grid) {
    const int64_t by_work = (nnz + 2047) / 2048;
    const int64_t by_rows = ((int64_t)rows + max_rows_wg / 2 - 1) / (max_rows_wg / 2);
    grid = (int)std::max<int64_t>(2, std::min<int64_t>(num_cus, std::max(by_work, by_rows)));
  }
  if (grid < 2 || grid > rows) return SPRNN_ERR_CAPACITY;
  // contiguous rows per workgroup (whole cache lines of the ring per producer), shares balanced by nonzero count
  std::vector<int> first_row(grid + 1, rows);
  {
    std::vector<int64_t> cum((size_t)rows + 1, 0);
    for (int r = 0; r < rows; ++r) cum[r + 1] = cum[r] + (row_ptr[r + 1] - row_ptr[r]) + kRowCost;
    first_row[0] = 0;
    for (int i = 1; i < grid; ++i) {
      const int64_t target = cum[rows] * i / grid;
      int r = (int)(std::lower_bound(cum.begin(), cum.end(), target) - cum.begin());   // smallest r with cum[r] >= target
      if (r > 0 && target - cum[r - 1] < cum[r] - target) --r;                          // ... or the boundary just below, if nearer
      r = std::max(r, first_row[i - 1] + 1);                                            // every workgroup owns a row
      r = std::min(r, rows - (grid - i));
      first_row[i] = r;
    }
  }
  int rows_wg_max = 0;
  for (int wg = 0; wg < grid; ++wg) rows_wg_max = std::max(rows_wg_max, first_row[wg + 1] - first_row[wg]);
  const int epi_waves = std::max(1, ceil_div((int64_t)rows_wg_max * batch, kWave));

  // --- gathering wavefronts and words per lane: the smallest NW per workgroup for which its rows' groups fit in the pool
  auto words_needed = [&](int wg, int W) -> int {   // 0 = does not fit at any NW
    const int pool_groups = W * kWave / G;
    int64_t wg_nnz = row_ptr[first_row[wg + 1]] - row_ptr[first_row[wg]];
    for (int nw = std::max<int64_t>(1, ceil_div(wg_nnz, (int64_t)W * kWave)); nw <= kTemplateWords[kNumTemplateWords - 1]; ++nw) {
      int64_t need = 0;
      for (int r = first_row[wg]; r < first_row[wg + 1] && need <= pool_groups; ++r) need += ceil_div(row_ptr[r + 1] - row_ptr[r], (int64_t)nw * G);
      if (need <= pool_groups) return nw;
    }
    return 0;
  };
  int W = 0, words_max = 0;
  std::vector<int> nw_wg(grid, 1);
  {
    int64_t best_cost = 0;
    const int forced = opt ? opt->waves : 0;
    for (int cand : {4, 7}) {
      if (forced && forced != cand) continue;
      if (cand + epi_waves > kMaxWavesPool) continue;
      int worst = 0;
      bool fits = true;
      std::vector<int> nws(grid);
      for (int wg = 0; wg < grid && fits; ++wg) { nws[wg] = words_needed(wg, cand); fits = nws[wg] > 0; worst = std::max(worst, nws[wg]); }
      if (!fits) continue;
      // multiply-add issue slots per SIMD and step ~ (wavefronts per SIMD) x words, plus what every wavefront spends around them
      const int64_t cost = (int64_t)(cand == 4 ? 1 : 2) * (4 * worst + 12);
      if (!W || cost < best_cost) { W = cand; best_cost = cost; nw_wg = nws; words_max = worst; }
    }
    if (forced && forced != 4 && forced != 7) return SPRNN_ERR_INVALID;
  }
  if (!W) return SPRNN_ERR_CAPACITY;
  const int tw = std::max(4, (words_max + 3) / 4 * 4);   // the lane-pool kernels are built for every multiple of four up to 64
  if (tw > 64) return SPRNN_ERR_CAPACITY;

  Mapping m;
  m.hidden = hidden; m.rows = rows; m.batch = batch; m.cell = cell; m.cols = cols;
  m.layout_batch = batch;
  m.col_stride = 4 * std::min(batch, 4);
  const int64_t plane = (int64_t)cols * m.col_stride;
  const int64_t hb = ((plane * (batch == 8 ? 2 : 1)) + 15) / 16 * 16;
  m.grid = grid; m.row_waves = W; m.waves = W + epi_waves; m.block = m.waves * kWave; m.lanes_per_row = G; m.group = G;
  m.layout = 1;
  m.template_words = tw;
  m.stage_bytes = batch * (W * kWave / G) * 4 + 64;   // group sums [sample][group] (+ room for reads past a short row)
  if (hb * kRingSlots > ((int64_t)1 << 30)) return SPRNN_ERR_CAPACITY;
  m.h_bytes = (int)hb;
  if (hb + 256 + m.stage_bytes > kLdsLimit) return SPRNN_ERR_CAPACITY;   // h has to fit in LDS whole (no column compaction here)
  m.lds_bytes = (int)hb;
  m.compact = 0; m.fill_rows = 0;
  m.index_shift = 0;
  if (plane > 65536) { while ((1 << m.index_shift) < m.col_stride) ++m.index_shift; }
  m.nnz = nnz;
  m.sync = (opt && opt->sync) ? opt->sync : SPRNN_SYNC_TAGGED;
  if (m.sync != SPRNN_SYNC_TAGGED && m.sync != SPRNN_SYNC_BARRIER) return SPRNN_ERR_INVALID;
  m.bank_aware = (opt && opt->bank_aware) ? opt->bank_aware : 1;
  if (m.bank_aware != 1 && m.bank_aware != 2) return SPRNN_ERR_INVALID;
  m.balance = 2;
  m.poll_delay = opt ? opt->poll_delay : 0;
  m.spin_limit = (opt && opt->spin_limit > 0) ? opt->spin_limit : (1 << 22);
  m.timeline = (opt && opt->timeline) ? 1 : 0;
  if (opt && (opt->launch < 0 || opt->launch > 2)) return SPRNN_ERR_INVALID;
  m.cooperative = (opt && opt->launch == 2) ? 1 : 0;
  m.jitter = opt ? opt->jitter : 0;

  Packed& P = *out;
  P = Packed();
  P.map = m;
  const int NW = tw;
  const size_t lanes = (size_t)grid * m.block;
  P.words.assign(lanes * NW, 0u);
  P.word_src.assign(lanes * NW, -1);
  P.lane_row.assign(lanes, -1);
  P.lane_words.assign(lanes, 0);
  P.lane_sum.assign(lanes, 0);
  P.wave_words.assign((size_t)grid * m.waves, 0);
  std::vector<char> is_real_zero(P.words.size(), 0);
  const PassModel pm = make_pass_model(batch);
  int64_t padded = 0;
  int used_words_max = 0;
  std::vector<std::vector<Seg>> wave_segs(W);
  for (int wg = 0; wg < grid; ++wg) {
    for (auto& v : wave_segs) v.clear();
    int lane = 0;                                   // next free lane of the pool
    for (int r = first_row[wg]; r < first_row[wg + 1]; ++r) {
      const int n = row_ptr[r + 1] - row_ptr[r];
      const int ng = ceil_div(n, (int64_t)nw_wg[wg] * G), nl = ng * G;
      const int e = (r - first_row[wg]) * batch;    // first output lane of the row
      for (int b = 0; b < batch; ++b) {
        const size_t at = (size_t)wg * m.block + (size_t)W * kWave + e + b;
        P.lane_row[at] = r;
        P.lane_sum[at] = (lane / G) | (ng << 16);
      }
      if (!nl) continue;
      const int wpl = ceil_div(n, nl);              // words per lane of this row (<= the workgroup's NW)
      int given = 0;
      for (int l0 = lane; l0 < lane + nl;) {        // one segment per wavefront the row touches
        const int wave = l0 / kWave, l1 = std::min(lane + nl, (wave + 1) * kWave);
        Seg q;
        q.lane0 = l0 % kWave; q.n = l1 - l0; q.row = r;
        const int take = std::min(n - given, q.n * wpl);
        q.first = row_ptr[r] + given;
        for (int i = 0; i < take; ++i) q.items.push_back({col_idx[q.first + i], val_bits[q.first + i]});
        given += take;
        wave_segs[wave].push_back(std::move(q));
        P.wave_words[(size_t)wg * m.waves + wave] = std::max(P.wave_words[(size_t)wg * m.waves + wave], wpl);
        l0 = l1;
      }
      lane += nl;
    }
    for (int wave = 0; wave < W; ++wave) {
      const int trip = P.wave_words[(size_t)wg * m.waves + wave];
      used_words_max = std::max(used_words_max, trip);
      padded += (int64_t)trip * kWave;
      order_segments(wave_segs[wave], trip, pm, m.bank_aware == 1);
      for (const Seg& q : wave_segs[wave]) {
        const size_t tid0 = (size_t)wg * m.block + (size_t)wave * kWave + q.lane0;
        for (int j = 0; j < q.n; ++j) P.lane_row[tid0 + j] = q.row;
        for (int k = 0; k < trip; ++k)
          for (int j = 0; j < q.n; ++j) {
            const size_t at = ((size_t)wg * NW + k) * m.block + (size_t)wave * kWave + q.lane0 + j;
            const int i = q.pos[(size_t)k * q.n + j];
            if (i < 0) continue;                   // stays a zero word; place_fillers gives it a harmless column
            const uint32_t idx = ((uint32_t)q.items[i].col * (uint32_t)m.col_stride) >> m.index_shift;
            P.words[at] = (idx << 16) | q.items[i].bits;
            P.word_src[at] = q.first + i;
            if ((q.items[i].bits & 0x7FFFu) == 0) is_real_zero[at] = 1;
            P.lane_words[tid0 + j] += 1;
          }
      }
    }
  }
  std::vector<int> wg_cols(grid, cols);
  place_fillers(P, wg_cols, is_real_zero);
  P.map.words_max = used_words_max;
  P.map.padded_words = padded;
  return SPRNN_OK;
}

int pack(int hidden, int batch, int cell, const int32_t* row_ptr, const int32_t* col_idx,
         const uint16_t* val_bits, const sprnn_options_t* opt, int num_cus, Packed* out) {
  int rc = validate_csr(hidden, batch, cell, row_ptr, col_idx, val_bits);
  if (rc != SPRNN_OK) return rc;
  const int layout = opt ? opt->layout : 0;
  if (layout < 0 || layout > 2) return SPRNN_ERR_INVALID;
  if (layout == 2 && cell > SPRNN_ACT_IDENTITY) return SPRNN_ERR_UNSUPPORTED;
  if (layout == 2 && opt && opt->activations == 2) return SPRNN_ERR_UNSUPPORTED;
  if (cell <= SPRNN_ACT_IDENTITY && layout == 2) {
    rc = pack_pool(hidden, batch, cell, row_ptr, col_idx, val_bits, opt, num_cus, out);
    if (rc != SPRNN_ERR_CAPACITY || layout == 2) return rc;   // (auto: a matrix that does not suit the pool takes the other layout)
  }
  const bool lstm = gated(cell);
  const int rows = hidden * (lstm ? 4 : 1);
  // the GRU's three row blocks become four with an empty last one
  std::vector<int32_t> padded_row_ptr;
  if (cell == SPRNN_CELL_GRU) {
    padded_row_ptr.assign(row_ptr, row_ptr + 3 * hidden + 1);
    padded_row_ptr.resize((size_t)rows + 1, row_ptr[3 * hidden]);
    row_ptr = padded_row_ptr.data();
  }
  std::vector<int> row_nnz(rows);
  for (int r = 0; r < rows; ++r) row_nnz[r] = row_ptr[r + 1] - row_ptr[r];
  Mapping m;
  rc = choose_mapping(hidden, batch, cell, row_nnz, opt, num_cus, &m);
  if (rc != SPRNN_OK) return rc;

  const int L = m.lanes_per_row;
  const int gpw = kWave / L;                      // row groups per wavefront
  const int upw = lstm ? gpw / 4 : gpw;           // units per wavefront
  const int gpu_ = lstm ? 4 : 1;                  // row groups per unit
  const int units = hidden;
  const int cols = m.cols;
  auto unit_row = [&](int u, int g) { return lstm ? g * hidden + u : u; };
  auto unit_cost = [&](int u) {
    int c = 0;
    for (int g = 0; g < gpu_; ++g) c = std::max(c, row_nnz[unit_row(u, g)]);
    return c;
  };

  // --- units -> (workgroup, wave, unit slot)
  const int total_waves = m.grid * m.waves;
  std::vector<int> wave_units((size_t)total_waves * upw, -1);   // unit id per (global wave, slot)
  if (m.balance == 1) {
    // deal by nonzero count: similar rows share a wavefront (little padding inside it), and wavefronts are
    // dealt to workgroups in serpentine order of their trip count so every workgroup gets the same load
    std::vector<int> order(units);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return unit_cost(a) > unit_cost(b); });
    const int nw = ceil_div(units, upw);
    for (int w = 0; w < nw; ++w) {
      const int round = w / m.grid, idx = w % m.grid;
      const int wg = (round & 1) ? (m.grid - 1 - idx) : idx;
      const int gw = wg * m.waves + round;        // round < row_waves because grid * row_waves >= nw
      for (int s = 0; s < upw; ++s) {
        const int i = w * upw + s;
        if (i < units) wave_units[(size_t)gw * upw + s] = order[i];
      }
    }
  } else {
    for (int u = 0; u < units; ++u) {           // contiguous rows: row-owning wavefront u / upw, slot u % upw
      const int cw = u / upw;
      const int gw = (cw / m.row_waves) * m.waves + cw % m.row_waves;
      wave_units[(size_t)gw * upw + u % upw] = u;
    }
  }

  // --- column compaction (Section 6 names the loading of activations as what dominates for very large, very
  // sparse layers, and proposes to give a block less than whole rows' worth of it): a workgroup only copies the 16-byte chunks of h that its rows read, into
  // consecutive LDS positions.  Used when the whole of h does not fit in LDS, or when every workgroup needs
  // less than half of it; otherwise LDS mirrors the ring slot.
  const int lb = m.layout_batch;                             // (batch / 2 with binary16 activations: twice the columns per chunk)
  const int cpc = lb >= 4 ? 1 : 4 / lb;                      // columns per 16-byte chunk
  const int planes = lb == 8 ? 2 : 1;
  const int chunks_per_plane = ceil_div(cols, cpc);
  // Flow control: the exchange ring is only safe because a workgroup cannot start step t before it has seen
  // something of step t-1 from EVERY workgroup (that is what keeps all of them within one step of each other and
  // lets a producer re-arm a slot two steps ahead).  Copying all of h gives that for free; a compacted copy must
  // keep it, so every workgroup's list also contains the chunk of the first unit of every workgroup.
  std::vector<int32_t> first_chunk_of_wg;
  for (int wg = 0; wg < m.grid; ++wg)
    for (int i = 0; i < m.waves * upw; ++i) {
      const int u = wave_units[(size_t)wg * m.waves * upw + i];
      if (u >= 0) { first_chunk_of_wg.push_back(u / cpc); break; }
    }
  std::vector<std::vector<int32_t>> wg_chunks(m.grid);         // sorted needed chunks (of one plane) per workgroup
  {
    std::vector<char> mark(chunks_per_plane);
    for (int wg = 0; wg < m.grid; ++wg) {
      std::fill(mark.begin(), mark.end(), 0);
      for (int32_t c : first_chunk_of_wg) mark[c] = 1;
      for (int wave = 0; wave < m.waves; ++wave)
        for (int s = 0; s < upw; ++s) {
          const int u = wave_units[((size_t)wg * m.waves + wave) * upw + s];
          if (u < 0) continue;
          for (int g = 0; g < gpu_; ++g) {
            const int r = unit_row(u, g);
            for (int32_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) mark[col_idx[k] / cpc] = 1;
          }
        }
      for (int c = 0; c < chunks_per_plane; ++c) if (mark[c]) wg_chunks[wg].push_back(c);
    }
  }
  size_t need_max = 1;
  for (auto& v : wg_chunks) need_max = std::max(need_max, v.size());
  const int copies = m.grid == 1 ? 2 : 1;   // a single workgroup double-buffers h in LDS, several exchange it through the ring
  const bool identity_fits = (int64_t)copies * m.h_bytes + 256 + m.stage_bytes <= kLdsLimit;
  // (scattered 16-byte reads cost more per byte than the contiguous copy: measured break-even near one half)
  bool compact = m.compact == 1 || (m.compact == 0 && (!identity_fits || need_max * 2 < (size_t)chunks_per_plane));
  if (m.grid == 1) compact = false;          // a single workgroup produces all of h itself
  if (!compact && !identity_fits) return SPRNN_ERR_CAPACITY;
  m.compact = compact ? 1 : 0;
  int64_t lds_plane;                          // bytes of one plane of the LDS copy (bounds the packed offsets)
  if (compact) {
    const int rounds = ceil_div((int64_t)planes * (int64_t)need_max, m.block);
    m.fill_rows = rounds;
    m.lds_bytes = rounds * m.block * 16;
    lds_plane = (int64_t)need_max * 16;
    if ((int64_t)m.lds_bytes + 256 + m.stage_bytes > kLdsLimit) return SPRNN_ERR_CAPACITY;
  } else {
    m.fill_rows = 0;
    m.lds_bytes = copies * m.h_bytes;
    lds_plane = (int64_t)cols * m.col_stride;
  }
  m.index_shift = 0;
  if (lds_plane > 65536) { while ((1 << m.index_shift) < m.col_stride) ++m.index_shift; }
  // LDS column position of a column for a workgroup

  // Overlap of the copy with the gathers: the first seg_rounds of the copy's rounds (a round = one 16-byte chunk per
  // lane of the workgroup) bring the columns below seg_col; see order_wave_phased.
  const int overlap = opt ? opt->overlap : 0;
  if (overlap < 0 || overlap > 2) return SPRNN_ERR_INVALID;
  const int copy_rounds = ceil_div(m.h_bytes / 16, m.block);
  const bool can_overlap = !compact && m.grid > 1 && planes == 1 && cell <= SPRNN_ACT_IDENTITY && m.sync == SPRNN_SYNC_TAGGED &&
                           copy_rounds >= 2 && copy_rounds <= 8 && !m.narrow && !m.half;
  if (overlap == 2 && !can_overlap) return SPRNN_ERR_UNSUPPORTED;
  m.seg_rounds = (overlap == 2 && can_overlap) ? copy_rounds / 2 : 0;
  const int seg_col = m.seg_rounds * m.block * cpc;

  Packed& P = *out;
  P.map = m;
  const int NW = m.template_words;
  if (compact) {
    // copy list: entry e = c * block + tid of a workgroup is the ring byte offset of the chunk that thread tid
    // copies in round c to LDS position e * 16, or an out-of-range offset past the end of the list.  Both planes
    // of a batch-8 layout follow each other, so plane 1 starts at (chunks) * 16 in LDS.
    constexpr uint32_t kEmptyEntry = 0x7ffffff0u;
    P.fill_src.assign((size_t)m.grid * m.fill_rows * m.block, kEmptyEntry);
    P.wg_plane.assign(m.grid, 0);
    for (int wg = 0; wg < m.grid; ++wg) {
      const auto& ch = wg_chunks[wg];
      const size_t n = ch.size();
      P.wg_plane[wg] = (int32_t)(n * 16);
      for (size_t e = 0; e < n * planes; ++e)
        P.fill_src[(size_t)wg * m.fill_rows * m.block + e] = (uint32_t)((e / n) * ((size_t)cols * 16) + (size_t)ch[e % n] * 16);
    }
  }

  const size_t lanes = (size_t)m.grid * m.block;
  P.words.assign(lanes * NW, 0u);
  P.word_src.assign(lanes * NW, -1);
  P.lane_row.assign(lanes, -1);
  P.lane_words.assign(lanes, 0);
  P.wave_words.assign(total_waves, 0);
  if (m.seg_rounds) P.wave_early.assign(total_waves, 0);

  const PassModel pm = make_pass_model(lb);
  auto pad_word = [&](int lane_in_wave, int k, int ncols) -> uint32_t {
    // zero-valued filler (place_fillers gives it a bank class that is free in its pass afterwards)
    int col = (lane_in_wave + k * L) % pm.classes;
    if (col >= ncols) col = 0;
    return (uint32_t)(((uint32_t)col * (uint32_t)m.col_stride) >> m.index_shift) << 16;
  };

  std::vector<char> is_real_zero(P.words.size(), 0);   // positions holding a stored (explicit) zero weight
  int words_max = 0;
  int64_t padded = 0;
  std::vector<int> wg_cols(m.grid, cols);     // LDS column positions a workgroup may address
  // The wavefronts are packed independently of each other (the bank-aware order is most of the time this function
  // takes), so the workgroups of a large matrix are dealt to a few host threads; each writes only its own workgroups'
  // parts of the arrays.
  std::atomic<bool> out_of_memory(false);
  auto pack_workgroups = [&](int wg_begin, int wg_end, int* words_max_out, int64_t* padded_out) {
    try {
      std::vector<int32_t> pos_of_chunk(compact ? (size_t)chunks_per_plane : 0);   // this thread's view of its current workgroup
      auto col_in_lds = [&](int col) { return compact ? pos_of_chunk[col / cpc] * cpc + col % cpc : col; };
      std::vector<RowGroup> rg;
      int local_max = 0;
      int64_t local_padded = 0;
      for (int wg = wg_begin; wg < wg_end; ++wg) {
        if (compact) {
          for (size_t i = 0; i < wg_chunks[wg].size(); ++i) pos_of_chunk[wg_chunks[wg][i]] = (int32_t)i;
          wg_cols[wg] = std::min<int64_t>((int64_t)wg_chunks[wg].size() * cpc, cols);
        }
        const int ncols = wg_cols[wg];
        for (int wave = 0; wave < m.waves; ++wave) {
          const int gw = wg * m.waves + wave;
          int trip = 0;
          for (int s = 0; s < upw; ++s) {
            const int u = wave_units[(size_t)gw * upw + s];
            if (u >= 0) trip = std::max(trip, ceil_div(unit_cost(u), L));
          }
          P.wave_words[gw] = trip;
          local_max = std::max(local_max, trip);
          local_padded += (int64_t)trip * kWave;
          rg.clear();
          for (int s = 0; s < upw; ++s) {
            const int u = wave_units[(size_t)gw * upw + s];
            for (int g = 0; g < gpu_; ++g) {
              RowGroup q;
              q.lane0 = (s * gpu_ + g) * L;
              if (u >= 0) {
                q.row = unit_row(u, g);
                for (int32_t k = row_ptr[q.row]; k < row_ptr[q.row + 1]; ++k) q.items.push_back({col_in_lds(col_idx[k]), val_bits[k]});   // bank classes follow LDS positions
              }
              rg.push_back(std::move(q));
            }
          }
          if (m.seg_rounds) {
            const int k1 = phase_words(rg, L, trip, seg_col);
            P.wave_early[gw] = k1;
            order_wave_phased(rg, L, trip, k1, seg_col, pm, m.bank_aware == 1);
          } else {
            order_wave(rg, L, trip, pm, m.bank_aware == 1);
          }
          for (const RowGroup& q : rg) {
            const size_t tid0 = (size_t)wg * m.block + (size_t)wave * kWave + q.lane0;
            for (int l = 0; l < L; ++l) P.lane_row[tid0 + l] = q.row < m.rows ? q.row : -1;   // the GRU's empty fourth row owns nothing
            for (int k = 0; k < trip; ++k)
              for (int l = 0; l < L; ++l) {
                const size_t at = ((size_t)wg * NW + k) * m.block + (size_t)wave * kWave + q.lane0 + l;
                const int i = q.pos[(size_t)k * L + l];
                if (i < 0) { P.words[at] = pad_word(q.lane0 + l, k, ncols); continue; }
                const uint32_t idx = ((uint32_t)q.items[i].col * (uint32_t)m.col_stride) >> m.index_shift;
                P.words[at] = (idx << 16) | q.items[i].bits;
                P.word_src[at] = row_ptr[q.row] + i;   // items are the row's nonzeros in CSR order
                if ((q.items[i].bits & 0x7FFFu) == 0) is_real_zero[at] = 1;
                P.lane_words[tid0 + l] += 1;
              }
          }
        }
      }
      *words_max_out = local_max;
      *padded_out = local_padded;
    } catch (const std::bad_alloc&) {
      out_of_memory = true;
    }
  };
  {
    const int hw = (int)std::thread::hardware_concurrency();
    const int nthreads = (m.nnz < 100000 || m.grid < 2) ? 1 : std::max(1, std::min(std::min(hw, 16), m.grid));
    std::vector<int> part_max(nthreads, 0);
    std::vector<int64_t> part_padded(nthreads, 0);
    std::vector<std::thread> workers;
    bool spawn_failed = false;
    for (int t = 1; t < nthreads && !spawn_failed; ++t) {
      const int b0 = (int)((int64_t)m.grid * t / nthreads), b1 = (int)((int64_t)m.grid * (t + 1) / nthreads);
      try {
        workers.emplace_back(pack_workgroups, b0, b1, &part_max[t], &part_padded[t]);
      } catch (...) {   // no more threads to be had: this thread does the rest
        spawn_failed = true;
        pack_workgroups(b0, m.grid, &part_max[t], &part_padded[t]);
      }
    }
    pack_workgroups(0, (int)((int64_t)m.grid / nthreads), &part_max[0], &part_padded[0]);
    for (auto& w : workers) w.join();
    if (out_of_memory) throw std::bad_alloc();
    for (int t = 0; t < nthreads; ++t) { words_max = std::max(words_max, part_max[t]); padded += part_padded[t]; }
  }
  place_fillers(P, wg_cols, is_real_zero);
  P.map.words_max = words_max;
  P.map.padded_words = padded;
  if (m.seg_rounds) {
    int least = -1;
    for (int gw = 0; gw < total_waves; ++gw)
      if (P.wave_words[gw] > 0 && (least < 0 || P.wave_early[gw] < least)) least = P.wave_early[gw];
    P.map.seg_words = std::max(least, 0);
  }
  return SPRNN_OK;
}

// LDS cycles needed by the packed gathers relative to a conflict-free layout, under the measured gfx950 model (see
// PassModel): lanes of a pass that read different addresses in the same bank class serialise, lanes that read the same
// address are served together.
double lds_pass_factor(const Packed& P) {
  const Mapping& m = P.map;
  const PassModel pm = make_pass_model(m.layout_batch ? m.layout_batch : m.batch);
  const int width = m.col_stride;
  int64_t passes = 0, ideal = 0;
  std::vector<std::vector<uint32_t>> seen(pm.classes);
  for (int wg = 0; wg < m.grid; ++wg)
    for (int wave = 0; wave < m.waves; ++wave) {
      const int trip = P.wave_words[(size_t)wg * m.waves + wave];
      for (int k = 0; k < trip; ++k)
        for (int p = 0; p < pm.npass; ++p) {
          for (auto& v : seen) v.clear();
          for (int l : pm.lanes[p]) {
            const uint32_t w = P.words[((size_t)wg * m.template_words + k) * m.block + (size_t)wave * kWave + l];
            const uint32_t byte = (w >> 16) << m.index_shift;
            auto& v = seen[(byte / width) % pm.classes];
            if (std::find(v.begin(), v.end(), byte) == v.end()) v.push_back(byte);
          }
          size_t worst = 1;
          for (auto& v : seen) worst = std::max(worst, v.size());
          passes += (int64_t)worst;
          ideal += 1;
        }
    }
  return ideal ? (double)passes / (double)ideal : 1.0;
}

}  // namespace sprnn
