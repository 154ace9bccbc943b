// Host-side weight preparation: CSR -> per-lane register image (see sprnn_pack.h).
#include "sprnn_pack.h"

#include <algorithm>
#include <cstring>
#include <numeric>

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

// Lanes that one LDS pass serves together, and the number of bank groups a gather of this width can
// hit, on gfx950: 64 banks x 4 B = 256 B per pass, so a 16-byte gather serves 16 lanes per pass over 16
// groups, an 8-byte gather 32 over 32, a 4-byte gather 64 over 64.
static int pass_lanes(int batch) { return batch >= 4 ? 16 : (batch == 2 ? 32 : 64); }

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
  m->col_stride = 4 * std::min(batch, 4);
  const int64_t plane = (int64_t)m->cols * m->col_stride;         // batch 8 keeps two planes of 4 samples
  const int64_t hb = ((plane * (batch == 8 ? 2 : 1)) + 15) / 16 * 16;
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
  m->plain_launch = (opt && opt->plain_launch) ? 1 : 0;
  m->jitter = opt ? opt->jitter : 0;
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
// a pass serves `groups` consecutive lanes of one gather instruction (= one slot k) and takes as many
// cycles as the largest number of different addresses that fall into one bank group (class = column mod
// groups).  A nonzero may sit in any slot and any lane of its own row, so the nonzeros are dealt class by
// class (largest class first) to the pass, among those that contain lanes of the row and still have room,
// where they add no cycle, else to the emptiest one.  Surplus nonzeros of over-full classes thereby pile
// into the same few passes, and a row that owns whole passes reaches max(largest class, passes) cycles,
// the lower bound.  Rows that share a pass (L < groups) are scheduled against the same pass state.
// LDS cycles one wavefront needs for its `trip` gathers under the pass model above.
static int64_t wave_cycles(const std::vector<RowGroup>& rg, int L, int trip, int groups) {
  int64_t total = 0;
  std::vector<std::vector<int32_t>> seen(groups);
  for (int k = 0; k < trip; ++k)
    for (int base = 0; base < kWave; base += groups) {
      for (auto& v : seen) v.clear();
      for (const RowGroup& q : rg)
        for (int l = 0; l < L; ++l) {
          if (q.lane0 + l < base || q.lane0 + l >= base + groups) continue;
          const int i = q.pos[(size_t)k * L + l];
          if (i < 0) continue;   // fillers are given a free bank group afterwards
          auto& v = seen[q.items[i].col % groups];
          if (std::find(v.begin(), v.end(), q.items[i].col) == v.end()) v.push_back(q.items[i].col);
        }
      size_t worst = 1;
      for (auto& v : seen) worst = std::max(worst, v.size());
      total += (int64_t)worst;
    }
  return total;
}

static void order_wave(std::vector<RowGroup>& rg, int L, int trip, int groups, bool bank_aware) {
  for (auto& g : rg) g.pos.assign((size_t)trip * L, -1);
  if (trip == 0) return;
  // CSR order: nonzero i -> lane i % L, slot i / L
  for (auto& g : rg)
    for (int i = 0; i < (int)g.items.size(); ++i) g.pos[i] = i;
  if (!bank_aware) return;
  const int64_t csr_cycles = wave_cycles(rg, L, trip, groups);
  std::vector<std::vector<int>> csr_pos(rg.size());
  for (size_t q = 0; q < rg.size(); ++q) { csr_pos[q] = rg[q].pos; rg[q].pos.assign((size_t)trip * L, -1); }
  const int pgs = kWave / groups;                  // pass groups per gather instruction
  const int P = trip * pgs;                        // passes of this wavefront: p = k * pgs + pg
  std::vector<int> pass_cycles(P, 0), pass_load(P, 0);
  std::vector<int> mult((size_t)P * groups, 0);
  const int sub = std::max(1, L / groups);         // pass groups one row spans
  const int cap = std::min(L, groups);             // lanes of one row inside one pass
  // per row and pass: how many of the row's lanes are already taken
  std::vector<std::vector<int>> taken(rg.size(), std::vector<int>((size_t)trip * sub, 0));
  std::vector<std::vector<std::vector<int>>> bucket(rg.size(), std::vector<std::vector<int>>(groups));
  std::vector<int64_t> class_total(groups, 0);
  for (size_t q = 0; q < rg.size(); ++q)
    for (int i = (int)rg[q].items.size() - 1; i >= 0; --i) {
      bucket[q][rg[q].items[i].col % groups].push_back(i);
      class_total[rg[q].items[i].col % groups] += 1;
    }
  std::vector<int> order(groups);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return class_total[a] > class_total[b]; });
  for (int g : order)
    for (size_t q = 0; q < rg.size(); ++q) {
      const int pg0 = rg[q].lane0 / groups;
      while (!bucket[q][g].empty()) {
        int best_k = -1, best_s = 0, best_cost = 0, best_load = 0;
        for (int k = 0; k < trip; ++k)
          for (int sidx = 0; sidx < sub; ++sidx) {
            if (taken[q][(size_t)k * sub + sidx] >= cap) continue;
            const int p = k * pgs + pg0 + sidx;
            const int cost = (mult[(size_t)p * groups + g] + 1 > pass_cycles[p]) ? 1 : 0;
            if (best_k < 0 || cost < best_cost || (cost == best_cost && pass_load[p] < best_load)) {
              best_k = k; best_s = sidx; best_cost = cost; best_load = pass_load[p];
            }
          }
        // the row has at most trip * L nonzeros, so a free lane always exists
        const int i = bucket[q][g].back();
        bucket[q][g].pop_back();
        const int p = best_k * pgs + pg0 + best_s;
        int& used = taken[q][(size_t)best_k * sub + best_s];
        rg[q].pos[(size_t)best_k * L + best_s * groups + used] = i;
        used += 1;
        pass_load[p] += 1;
        const int mcount = ++mult[(size_t)p * groups + g];
        pass_cycles[p] = std::max(pass_cycles[p], mcount);
      }
    }
  // the greedy deal is not optimal when many short rows share a pass: never do worse than CSR order
  if (wave_cycles(rg, L, trip, groups) > csr_cycles)
    for (size_t q = 0; q < rg.size(); ++q) rg[q].pos = csr_pos[q];
}

int pack(int hidden, int batch, int cell, const int32_t* row_ptr, const int32_t* col_idx,
         const uint16_t* val_bits, const sprnn_options_t* opt, int num_cus, Packed* out) {
  int rc = validate_csr(hidden, batch, cell, row_ptr, col_idx, val_bits);
  if (rc != SPRNN_OK) return rc;
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
  const int cpc = batch >= 4 ? 1 : 4 / batch;                 // columns per 16-byte chunk
  const int planes = batch == 8 ? 2 : 1;
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
  std::vector<int32_t> chunk_pos(compact ? (size_t)chunks_per_plane : 0);
  auto lds_col = [&](int col) { return compact ? chunk_pos[col / cpc] * cpc + col % cpc : col; };

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

  const int groups = pass_lanes(batch);
  auto pad_word = [&](int lane_in_wave, int k, int ncols) -> uint32_t {
    // zero-valued filler that reads the bank group this lane would ideally hit
    int col = (lane_in_wave + k * L) % groups;
    if (col >= ncols) col = 0;
    return (uint32_t)(((uint32_t)col * (uint32_t)m.col_stride) >> m.index_shift) << 16;
  };

  std::vector<char> is_real_zero(P.words.size(), 0);   // positions holding a stored (explicit) zero weight
  int words_max = 0;
  int64_t padded = 0;
  std::vector<RowGroup> rg;
  int pos_wg = -1;
  std::vector<int> wg_cols(m.grid, cols);     // LDS column positions a workgroup may address
  for (int gw = 0; gw < total_waves; ++gw) {
    const int wg = gw / m.waves, wave = gw % m.waves;
    if (compact && wg != pos_wg) {
      pos_wg = wg;
      for (size_t i = 0; i < wg_chunks[wg].size(); ++i) chunk_pos[wg_chunks[wg][i]] = (int32_t)i;
      wg_cols[wg] = std::min<int64_t>((int64_t)wg_chunks[wg].size() * cpc, cols);
    }
    const int ncols = wg_cols[wg];
    int trip = 0;
    for (int s = 0; s < upw; ++s) {
      const int u = wave_units[(size_t)gw * upw + s];
      if (u >= 0) trip = std::max(trip, ceil_div(unit_cost(u), L));
    }
    P.wave_words[gw] = trip;
    words_max = std::max(words_max, trip);
    padded += (int64_t)trip * kWave;
    rg.clear();
    for (int s = 0; s < upw; ++s) {
      const int u = wave_units[(size_t)gw * upw + s];
      for (int g = 0; g < gpu_; ++g) {
        RowGroup q;
        q.lane0 = (s * gpu_ + g) * L;
        if (u >= 0) {
          q.row = unit_row(u, g);
          for (int32_t k = row_ptr[q.row]; k < row_ptr[q.row + 1]; ++k) q.items.push_back({lds_col(col_idx[k]), val_bits[k]});   // bank classes follow LDS positions
        }
        rg.push_back(std::move(q));
      }
    }
    order_wave(rg, L, trip, groups, m.bank_aware == 1);
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
  // Filler words should not add bank conflicts: give each one a column whose bank group is still free in
  // its pass (or, failing that, an address that another lane of the pass already reads: a broadcast).
  for (int wg = 0; wg < m.grid; ++wg)
    for (int wave = 0; wave < m.waves; ++wave) {
      const int trip = P.wave_words[(size_t)wg * m.waves + wave];
      for (int k = 0; k < trip; ++k)
        for (int base = 0; base < kWave; base += groups) {
          std::vector<char> used(groups, 0);
          uint32_t* wp = &P.words[((size_t)wg * NW + k) * m.block + (size_t)wave * kWave + base];
          std::vector<int> fillers;
          uint32_t some_addr = 0; bool have_addr = false;
          for (int l = 0; l < groups; ++l) {
            const uint32_t w = wp[l];
            if ((w & 0x7FFFu) == 0) { fillers.push_back(l); continue; }   // zero value: a filler, or a stored zero (kept below)
            used[((w >> 16) << m.index_shift) / m.col_stride % groups] = 1;
            some_addr = w >> 16; have_addr = true;
          }
          int g = 0;
          for (int l : fillers) {
            if (is_real_zero[((size_t)wg * NW + k) * m.block + (size_t)wave * kWave + base + l]) {
              used[((wp[l] >> 16) << m.index_shift) / m.col_stride % groups] = 1;
              continue;
            }
            while (g < groups && (used[g] || g >= wg_cols[wg])) ++g;
            if (g < groups) {
              wp[l] = (uint32_t)(((uint32_t)g * (uint32_t)m.col_stride) >> m.index_shift) << 16;
              used[g] = 1;
            } else {
              wp[l] = have_addr ? (some_addr << 16) : 0u;
            }
          }
        }
    }
  P.map.words_max = words_max;
  P.map.padded_words = padded;
  return SPRNN_OK;
}

// LDS passes needed by the packed gathers relative to a conflict-free layout, under the measured gfx950
// model: a pass serves `groups` consecutive lanes; lanes that read different addresses in the same bank
// group serialise, lanes that read the same address are served together.
double lds_pass_factor(const Packed& P) {
  const Mapping& m = P.map;
  const int groups = pass_lanes(m.batch);
  const int width = m.col_stride;
  int64_t passes = 0, ideal = 0;
  std::vector<std::vector<uint32_t>> seen(groups);
  for (int wg = 0; wg < m.grid; ++wg)
    for (int wave = 0; wave < m.waves; ++wave) {
      const int trip = P.wave_words[(size_t)wg * m.waves + wave];
      for (int k = 0; k < trip; ++k)
        for (int base = 0; base < kWave; base += groups) {
          for (auto& v : seen) v.clear();
          for (int l = base; l < base + groups; ++l) {
            const uint32_t w = P.words[((size_t)wg * m.template_words + k) * m.block + (size_t)wave * kWave + l];
            const uint32_t byte = (w >> 16) << m.index_shift;
            auto& v = seen[(byte / width) % groups];
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
