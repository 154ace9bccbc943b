// C ABI of libsprnn (see include/sprnn.h): handle life cycle, launches, host-only packing entry point.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "sprnn.h"
#include "sprnn_device.h"
#include "sprnn_pack.h"

using namespace sprnn;

struct sprnn_handle_s {
  Mapping map;
  int device = 0;
  int num_cus = 0;
  int capacity = 0;
  int launch_lds = 0;            // dynamic LDS requested at launch (>= map.lds_bytes; large enough for one workgroup per CU)
  double pass_factor = 1.0;
  const void* kernel = nullptr;
  const void* kernel_bwd = nullptr;   // backward pass of a vanilla cell (same launch shape and LDS)
  const void* kernel_bwd_grad = nullptr;   // the same with the weight gradient fused in
  uint32_t* d_words = nullptr;
  int32_t* d_lane_row = nullptr;
  int32_t* d_wave_words = nullptr;
  int32_t* d_wave_early = nullptr;   // two-part copy only
  uint32_t* d_fill_src = nullptr;    // column compaction only
  int32_t* d_wg_plane = nullptr;
  int32_t* d_lane_sum = nullptr;     // lane-pool layout only
  int32_t* d_word_src = nullptr;     // vanilla cells without compaction: packed word -> CSR position (weight gradient)
  const void* kernel_wgrad = nullptr;
  uint32_t* d_ring = nullptr;
  uint32_t* d_ctrl = nullptr;
  unsigned long long* d_timeline = nullptr;   // [grid][16], only with options.timeline
  int32_t* d_row_ptr = nullptr;
  int32_t* d_col = nullptr;
  uint16_t* d_val = nullptr;
  uint32_t step_base = 0;        // global step index at which the next forward starts
  uint32_t barrier_base = 0;     // grid barriers completed so far (grid-barrier mode)
  uint32_t launch_epoch = 0;     // persistent launches so far (parity selects the placement counters of the one-XCD mode)
  bool one_xcd = false;          // launches hold 8 x grid workgroups and those of one XCD take the work
  bool poisoned = false;         // a watchdog trip was observed: the ring no longer holds a consistent state
  bool used_shared_exchange = false;   // sprnn_forward_noalloc ran on this handle: sprnn_check also reads its status word
  float calibrated_us = 0.0f;    // microseconds per step of the setting the calibration kept (0: not measured)
};

// ---- storage of sprnn_forward_noalloc: one array per device, alive as long as the library is loaded.
// Layout: [control words, kScratchCtrlBytes][exchange ring, 4 slots].  On the host the array's name is only a
// stand-in for the symbol; the address on each device comes from hipGetSymbolAddress and is kept in g_scratch.
constexpr size_t kScratchBytes = (size_t)1 << 20;
constexpr size_t kScratchCtrlBytes = 1024;
static_assert(kScratchCtrlBytes >= kCtrlWords * 4 && kScratchCtrlBytes % 256 == 0, "control words must fit in front of the ring");
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxScratchDevices = 64;
static unsigned char* g_scratch[kMaxScratchDevices];   // per device, null until looked up
static std::mutex g_scratch_mutex;

namespace {

// With SPRNN_DEBUG set in the environment, a failing HIP call is named on stderr.
bool hip_ok(hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  static const bool verbose = std::getenv("SPRNN_DEBUG") != nullptr;
  if (verbose) std::fprintf(stderr, "sprnn: %s failed: %s\n", what, hipGetErrorString(e));
  (void)hipGetLastError();
  return false;
}
#define SPRNN_HIP(call) hip_ok((call), #call)

struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int dev) {
    if (!SPRNN_HIP(hipGetDevice(&prev))) return;
    ok = (prev == dev) || SPRNN_HIP(hipSetDevice(dev));
    if (prev == dev) prev = -1;
  }
  ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

void fill_info(const Mapping& m, int capacity, double pass_factor, sprnn_info_t* info) {
  std::memset(info, 0, sizeof(*info));
  info->hidden = m.hidden; info->rows = m.rows; info->batch = m.batch; info->cell = m.cell;
  info->grid = m.grid; info->block = m.block; info->waves = m.waves; info->lanes_per_row = m.lanes_per_row;
  info->sync = m.sync; info->bank_aware = m.bank_aware; info->balance = m.balance; info->poll_delay = m.poll_delay;
  info->words_per_lane_max = m.words_max; info->template_words = m.template_words; info->lds_bytes = m.lds_bytes;
  info->resident_capacity = capacity;
  info->nnz = m.nnz; info->padded_words = m.padded_words;
  info->ring_bytes = (int64_t)kRingSlots * m.h_bytes;
  info->lds_pass_factor = pass_factor;
  info->compact = m.compact;
  info->layout = m.layout ? 2 : 1;
  info->gather_waves = m.row_waves;
  info->overlap_rounds = m.seg_rounds;
  info->overlap_words = m.seg_words;
  info->activations = m.half ? 2 : 1;
}
// (fill_info has no handle: the one-XCD flag is added by sprnn_get_info)

template <typename T>
hipError_t upload(T** dst, const T* src, size_t n) {
  *dst = nullptr;
  hipError_t e = hipMalloc((void**)dst, std::max<size_t>(n, 1) * sizeof(T));
  if (e != hipSuccess) return e;
  if (n) e = hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice);
  return e;
}

void release(sprnn_handle_s* h) {
  if (!h) return;
  (void)hipFree(h->d_words); (void)hipFree(h->d_lane_row); (void)hipFree(h->d_wave_words); (void)hipFree(h->d_wave_early);
  (void)hipFree(h->d_fill_src); (void)hipFree(h->d_wg_plane); (void)hipFree(h->d_word_src); (void)hipFree(h->d_lane_sum);
  (void)hipFree(h->d_ring); (void)hipFree(h->d_ctrl); (void)hipFree(h->d_timeline);
  (void)hipFree(h->d_row_ptr); (void)hipFree(h->d_col); (void)hipFree(h->d_val);
  delete h;
}

// Fallback back-off before a step's first poll (units of s_sleep(1) = 64 clocks) when the calibration at create
// time cannot run: the spread of the workgroups' publish times plus the time a store needs to reach the memory
// side, as measured on MI355X.
int default_poll_delay(const Mapping& m) { return m.grid > 1 ? 6 : 0; }

// Address of this device's copy of `scratch`; the device must be current.  Looked up once per device.
unsigned char* scratch_on_device(int device) {
  if (device < 0 || device >= kMaxScratchDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch[device]) {
    void* ptr = nullptr;
    if (!SPRNN_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)))) return nullptr;
    g_scratch[device] = static_cast<unsigned char*>(ptr);
  }
  return g_scratch[device];
}

}  // namespace

// What a launch of the persistent kernel takes beyond the forward pass's five buffers.
struct LaunchExtras {
  const float* b_hn = nullptr;       // GRU: recurrent bias of the candidate
  float* gates_out = nullptr;        // LSTM forward: gate values kept for the backward pass
  bool backward = false;             // time runs from T down to 1; one launch only
  const float* saved = nullptr;      // backward: forward outputs h_t (vanilla cells) or gate values (LSTM)
  float* dh0 = nullptr;              // backward: dL/dh_0 (adds one step)
  float* dc0 = nullptr;              // LSTM backward: dL/dc_0
  const float* wgrad_h_fwd = nullptr;   // backward with the weight gradient fused in: forward outputs h_t ...
  const float* wgrad_h0 = nullptr;      // ... h_0 ...
  float* dU = nullptr;                  // ... and the sums (selects the fused kernel; adds one step)
  bool shared_exchange = false;      // ring and control words in the device's static array instead of the handle's own
};
static int forward_persistent(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                              float* h_out, float* c_out, void* stream, const LaunchExtras& ex = LaunchExtras());
// Ordinary launches of kernels whose workgroups spin on each other: two of them must never hold compute units while
// waiting for the other's, so the library runs its persistent launches on a device one after the other.  Launches on
// one stream are in order already.  A launch on another stream than the one before waits for an event that lies
// behind that earlier launch.  A stream the caller created may be destroyed at any time, and a destroyed stream must
// not be handed to the runtime again, so the event is recorded right behind every launch on such a stream (a few
// microseconds per call); the default stream cannot go away, and a launch there is followed by the event only when
// the next launch turns out to use another stream.  Inside a stream capture nothing is recorded or waited for (an
// event from outside cannot be waited on there): a captured graph's order is the caller's.
struct LaunchOrder {
  std::mutex mutex;
  hipEvent_t done = nullptr;
  bool any = false;               // a persistent launch has been made on this device
  bool on_default = false;        // ... the latest one on the default stream, not yet followed by the event
  hipStream_t stream = nullptr;   // the stream of the latest launch: compared, never used
};
static LaunchOrder g_launch_order[kMaxScratchDevices];

static hipError_t launch_in_order(int device, const void* kernel, int grid, int block, void** args, unsigned lds, hipStream_t stream) {
  if (device < 0 || device >= kMaxScratchDevices) return hipErrorInvalidDevice;
  LaunchOrder& o = g_launch_order[device];
  std::lock_guard<std::mutex> lock(o.mutex);
  hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &capturing) != hipSuccess) { (void)hipGetLastError(); capturing = hipStreamCaptureStatusNone; }
  const bool ordered = capturing == hipStreamCaptureStatusNone;
  if (!o.done) {
    const hipError_t c = hipEventCreateWithFlags(&o.done, hipEventDisableTiming);
    if (c != hipSuccess) { o.done = nullptr; return c; }
  }
  if (ordered && o.any && o.stream != stream) {
    bool recorded = !o.on_default;
    if (o.on_default) {
      // (this fails while another stream is being captured in the global mode; nothing can be ordered against then)
      if (hipEventRecord(o.done, nullptr) == hipSuccess) { recorded = true; o.on_default = false; }
      else (void)hipGetLastError();
    }
    if (recorded) {
      const hipError_t w = hipStreamWaitEvent(stream, o.done, 0);
      if (w != hipSuccess) return w;
    }
  }
  const hipError_t e = hipLaunchKernel(kernel, dim3(grid), dim3(block), args, lds, stream);
  if (e != hipSuccess || !ordered) return e;
  o.any = true;
  o.stream = stream;
  if (stream == nullptr) {
    o.on_default = true;
  } else {
    o.on_default = false;
    const hipError_t r = hipEventRecord(o.done, stream);
    if (r != hipSuccess) return r;
  }
  return hipSuccess;
}

static int calibrate_poll_delay(sprnn_handle_s* h, bool try_one_xcd, bool long_runs);

extern "C" {

const char* sprnn_status_string(int code) {
  switch (code) {
    case SPRNN_OK: return "ok";
    case SPRNN_ERR_INVALID: return "invalid argument or malformed CSR";
    case SPRNN_ERR_CAPACITY: return "does not fit on chip or grid exceeds co-resident capacity";
    case SPRNN_ERR_HIP: return "HIP runtime call failed";
    case SPRNN_ERR_UNSUPPORTED: return "unsupported batch, hidden size or cell for this call";
    case SPRNN_ERR_STATE: return "spin watchdog tripped; handle unusable";
    default: return "unknown status";
  }
}

void sprnn_free_host(void* p) { std::free(p); }

int sprnn_pack_host(int hidden, int batch, int activation, const int32_t* row_ptr, const int32_t* col_idx,
                    const uint16_t* val_fp16_bits, const sprnn_options_t* opt, int num_cus,
                    uint32_t** words, int32_t** lane_row, int32_t** lane_words, sprnn_info_t* info) {
  if (!words || !lane_row || !lane_words || !info) return SPRNN_ERR_INVALID;
  *words = nullptr; *lane_row = nullptr; *lane_words = nullptr;
  Packed P;
  int rc;
  try {
    rc = pack(hidden, batch, activation, row_ptr, col_idx, val_fp16_bits, opt, num_cus, &P);
  } catch (const std::bad_alloc&) {
    return SPRNN_ERR_CAPACITY;
  }
  if (rc != SPRNN_OK) return rc;
  auto dup = [](const void* src, size_t bytes) -> void* {
    void* p = std::malloc(std::max<size_t>(bytes, 1));
    if (p && bytes) std::memcpy(p, src, bytes);
    return p;
  };
  *words = (uint32_t*)dup(P.words.data(), P.words.size() * 4);
  *lane_row = (int32_t*)dup(P.lane_row.data(), P.lane_row.size() * 4);
  *lane_words = (int32_t*)dup(P.lane_words.data(), P.lane_words.size() * 4);
  if (!*words || !*lane_row || !*lane_words) {
    std::free(*words); std::free(*lane_row); std::free(*lane_words);
    *words = nullptr; *lane_row = nullptr; *lane_words = nullptr;
    return SPRNN_ERR_CAPACITY;
  }
  fill_info(P.map, 0, lds_pass_factor(P), info);
  return SPRNN_OK;
}

// A second mapping worth measuring against the library's own choice (0 = none): fewer, larger workgroups that fit one
// XCD, or more wavefronts per workgroup so that the copy of h issues fewer surplus loads.
struct Alternative {
  int grid = 0;
  int fill_waves = 0;
};

// One handle for one set of options: mapping, packing, upload, kernel choice, calibration.  `long_runs` makes the
// calibration time runs long enough to be compared between two handles of different launch size.
static int create_one(sprnn_handle_t* out, int hidden, int batch, int activation, const int32_t* row_ptr,
                      const int32_t* col_idx, const uint16_t* val_fp16_bits, int device_id,
                      const sprnn_options_t* opt, const hipDeviceProp_t& prop, bool free_choice, bool long_runs,
                      Alternative* alternative) {
  Packed P;
  int rc;
  try {
    rc = pack(hidden, batch, activation, row_ptr, col_idx, val_fp16_bits, opt, prop.multiProcessorCount, &P);
  } catch (const std::bad_alloc&) {
    return SPRNN_ERR_CAPACITY;
  }
  if (rc != SPRNN_OK) return rc;
  if (P.map.layout == 1 && !pool_kernel_for(P.map.batch, P.map.template_words, P.map.cell, P.map.timeline != 0)) {
    // no lane-pool kernel is built for this many words per lane: the automatic choice takes the other layout
    if (opt && opt->layout == 2) return SPRNN_ERR_UNSUPPORTED;
    sprnn_options_t other = opt ? *opt : sprnn_options_t();
    if (!opt) std::memset(&other, 0, sizeof(other));
    other.layout = 1;
    try {
      rc = pack(hidden, batch, activation, row_ptr, col_idx, val_fp16_bits, &other, prop.multiProcessorCount, &P);
    } catch (const std::bad_alloc&) {
      return SPRNN_ERR_CAPACITY;
    }
    if (rc != SPRNN_OK) return rc;
  }

  (void)scratch_on_device(device_id);   // sprnn_forward_noalloc's array: address looked up once per device, here at set-up
  sprnn_handle_s* h = new (std::nothrow) sprnn_handle_s;
  if (!h) return SPRNN_ERR_CAPACITY;
  h->map = P.map;
  const bool calibrate = h->map.poll_delay == 0 && h->map.grid > 1 && h->map.sync == SPRNN_SYNC_TAGGED;
  if (h->map.poll_delay == 0) h->map.poll_delay = default_poll_delay(h->map);
  if (h->map.poll_delay < 0) h->map.poll_delay = 0;
  h->device = device_id;
  h->num_cus = prop.multiProcessorCount;
  h->pass_factor = lds_pass_factor(P);
  const Mapping& m = h->map;
  const bool pool = m.layout == 1;
  h->kernel = pool ? pool_kernel_for(m.batch, m.template_words, m.cell, m.timeline != 0)
                   : (m.narrow ? persistent_narrow_kernel_for(m.batch, m.template_words)
                               : (m.seg_rounds ? persistent_overlap_kernel_for(m.batch, m.template_words, m.timeline != 0)
                                  : (m.half ? persistent_half_kernel_for(m.batch, m.template_words)
                                            : persistent_kernel_for(m.batch, m.template_words, m.cell, m.timeline != 0))));
  // a short h (at most three rounds of the copy): the forward instantiation that issues exactly that many loads
  const int copy_rounds = (m.h_bytes / 16 + m.block - 1) / m.block;
  if (!pool && !m.narrow && !m.seg_rounds && !m.half && !m.timeline && !m.compact && m.grid > 1 && copy_rounds <= 3 &&
      m.cell <= SPRNN_CELL_GRU) {
    const void* k = persistent_short_kernel_for(m.batch, m.template_words, m.cell);
    if (k) h->kernel = k;
  }
  if (!h->kernel) { release(h); return SPRNN_ERR_UNSUPPORTED; }

  // One workgroup per CU: ask for more than half of a CU's LDS so that two can never share one.
  // (sharedMemPerMultiprocessor is not used: some runtime versions report the whole chip's LDS there.)
  const int lds_cu = prop.sharedMemPerBlockOptin > 0 ? (int)prop.sharedMemPerBlockOptin : (int)prop.sharedMemPerBlock;
  const int lds_need = m.lds_bytes + kLdsTailBytes + m.stage_bytes;      // h + the abort flags (+ the LSTM hand-over area)
  h->launch_lds = std::max(lds_need, lds_cu / 2 + 1024);
  if (h->launch_lds > lds_cu) { release(h); return SPRNN_ERR_CAPACITY; }
  // (the per-kernel limit on dynamic LDS is state shared by every handle that uses the same instantiation: it is
  // always raised to the device's maximum, never set to one handle's own request)
  if (!SPRNN_HIP(hipFuncSetAttribute(h->kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cu))) { release(h); return SPRNN_ERR_HIP; }
  if (m.cell <= SPRNN_ACT_IDENTITY && !m.timeline && !m.narrow && !m.half) {
    // the backward pass of a vanilla cell runs on a handle that holds the transposed matrix: same shape, same LDS
    h->kernel_bwd = pool ? pool_kernel_for(m.batch, m.template_words, kCellBackward) : persistent_kernel_for(m.batch, m.template_words, kCellBackward, false);
    if (h->kernel_bwd && !SPRNN_HIP(hipFuncSetAttribute(h->kernel_bwd, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cu))) { release(h); return SPRNN_ERR_HIP; }
    // it spins on its neighbours like the forward kernel: usable only if the same grid is co-resident with it
    int per_cu_bwd = 0;
    if (h->kernel_bwd && (!SPRNN_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_bwd, h->kernel_bwd, m.block, h->launch_lds)) ||
                          m.grid > per_cu_bwd * prop.multiProcessorCount)) h->kernel_bwd = nullptr;
  }
  int per_cu = 0;
  if (!SPRNN_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, h->kernel, m.block, h->launch_lds))) { release(h); return SPRNN_ERR_HIP; }
  h->capacity = per_cu * h->num_cus;
  if (m.grid > h->capacity) { release(h); return SPRNN_ERR_CAPACITY; }   // a spinning grid that is not co-resident would deadlock
  // One-XCD mode: small layers whose workgroups fit the CUs of one XCD (8 x grid workgroups must be co-resident)
  const int xcd_opt = opt ? opt->xcd : 0;
  if (xcd_opt < 0 || xcd_opt > 2) { release(h); return SPRNN_ERR_INVALID; }
  const bool xcd_eligible = !pool && m.grid >= 2 && m.grid * 8 <= h->capacity && m.grid <= prop.multiProcessorCount / 8 &&
                            m.cell != SPRNN_CELL_LSTM_BACKWARD && m.cell != SPRNN_CELL_GRU_BACKWARD && !m.timeline;
  if (xcd_opt == 2 && !xcd_eligible) { release(h); return SPRNN_ERR_UNSUPPORTED; }
  h->one_xcd = xcd_opt == 2;
  const bool try_one_xcd = xcd_opt == 0 && xcd_eligible && calibrate;

  const size_t ring_words = (size_t)kRingSlots * m.h_bytes / 4;
  // (binary16 activations: two elements per 32-bit word, each carrying the mark)
  std::vector<uint32_t> ring(ring_words, m.half ? (kSentinel >> 16 | kSentinel) : kSentinel);
  {
    // bytes of a slot beyond the last element of h are never written by a producer: mark them as present
    const size_t used = (size_t)m.cols * m.batch / (m.half ? 2 : 1);     // 32-bit words (both planes for batch 8)
    for (int s = 0; s < kRingSlots; ++s)
      for (size_t i = used; i < (size_t)m.h_bytes / 4; ++i) ring[(size_t)s * m.h_bytes / 4 + i] = 0u;
  }
  std::vector<uint32_t> ctrl(kCtrlWords, 0u);
  const int rows = m.rows;
  bool ok = SPRNN_HIP(upload(&h->d_words, P.words.data(), P.words.size())) &&
            SPRNN_HIP(upload(&h->d_lane_row, P.lane_row.data(), P.lane_row.size())) &&
            SPRNN_HIP(upload(&h->d_wave_words, P.wave_words.data(), P.wave_words.size())) &&
            (!m.compact || (SPRNN_HIP(upload(&h->d_fill_src, P.fill_src.data(), P.fill_src.size())) &&
                            SPRNN_HIP(upload(&h->d_wg_plane, P.wg_plane.data(), P.wg_plane.size())))) &&
            (!pool || SPRNN_HIP(upload(&h->d_lane_sum, P.lane_sum.data(), P.lane_sum.size()))) &&
            (!m.seg_rounds || SPRNN_HIP(upload(&h->d_wave_early, P.wave_early.data(), P.wave_early.size()))) &&
            SPRNN_HIP(upload(&h->d_ring, ring.data(), ring.size())) &&
            SPRNN_HIP(upload(&h->d_ctrl, ctrl.data(), ctrl.size())) &&
            SPRNN_HIP(upload(&h->d_row_ptr, row_ptr, (size_t)rows + 1)) &&
            SPRNN_HIP(upload(&h->d_col, col_idx, (size_t)m.nnz)) &&
            SPRNN_HIP(upload(&h->d_val, val_fp16_bits, (size_t)m.nnz));
  if (ok && (m.cell == SPRNN_CELL_LSTM_BACKWARD || m.cell == SPRNN_CELL_GRU_BACKWARD) && !m.compact) {
    // backward pass of a gated cell with the weight gradient fused in: needs the word -> CSR position map, co-residency
    // of the same grid with that kernel, and a kernel built for this many threads
    const void* k = persistent_kernel_for(m.batch, m.template_words,
                                          m.cell == SPRNN_CELL_LSTM_BACKWARD ? kCellLstmBackwardGrad : kCellGruBackwardGrad, false);
    int per_cu_g = 0;
    hipFuncAttributes fa;
    if (k && SPRNN_HIP(hipFuncGetAttributes(&fa, k)) && fa.maxThreadsPerBlock >= m.block &&
        SPRNN_HIP(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cu)) &&
        SPRNN_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_g, k, m.block, h->launch_lds)) &&
        m.grid <= per_cu_g * prop.multiProcessorCount) {
      ok = SPRNN_HIP(upload(&h->d_word_src, P.word_src.data(), P.word_src.size()));
      if (ok) h->kernel_bwd_grad = k;
    }
  }
  if (ok && (m.cell <= SPRNN_ACT_IDENTITY || m.cell == SPRNN_CELL_LSTM || m.cell == SPRNN_CELL_GRU) && !m.compact && !m.half) {
    // the weight gradient re-uses the forward mapping: one accumulator per packed word, left through this map
    // (built for the word counts of the one-group-per-row layout; a lane-pool mapping with another count has none:
    // sprnn_weight_gradient is then unsupported on this handle, the fused backward pass is the way)
    h->kernel_wgrad = weight_grad_kernel_for(m.batch, m.template_words);
    ok = SPRNN_HIP(upload(&h->d_word_src, P.word_src.data(), P.word_src.size())) &&
         (!h->kernel_wgrad || SPRNN_HIP(hipFuncSetAttribute(h->kernel_wgrad, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cu)));
    hipFuncAttributes wfa;   // (the instantiations with many words per lane are built for fewer threads than a lane-pool workgroup may have)
    if (ok && h->kernel_wgrad && (!SPRNN_HIP(hipFuncGetAttributes(&wfa, h->kernel_wgrad)) || wfa.maxThreadsPerBlock < m.block)) h->kernel_wgrad = nullptr;
    if (ok && h->kernel_bwd && !m.timeline && m.cell <= SPRNN_ACT_IDENTITY) {
      // backward pass with the weight gradient fused in: same co-residency requirement as the plain one
      const void* k = pool ? pool_kernel_for(m.batch, m.template_words, kCellBackwardGrad) : persistent_kernel_for(m.batch, m.template_words, kCellBackwardGrad, false);
      int per_cu_g = 0;
      hipFuncAttributes fa;
      if (k && SPRNN_HIP(hipFuncGetAttributes(&fa, k)) && fa.maxThreadsPerBlock >= m.block &&
          SPRNN_HIP(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cu)) &&
          SPRNN_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_g, k, m.block, h->launch_lds)) &&
          m.grid <= per_cu_g * prop.multiProcessorCount)
        h->kernel_bwd_grad = k;
    }
  }
  if (ok && m.timeline) {
    std::vector<unsigned long long> zeros((size_t)m.grid * kTimelineSlots, 0ull);
    ok = SPRNN_HIP(upload(&h->d_timeline, zeros.data(), zeros.size()));
  }
  if (!ok || !SPRNN_HIP(hipDeviceSynchronize())) { release(h); return SPRNN_ERR_HIP; }
  // Would the same rows fit the CUs of one XCD as fewer, larger workgroups?  (the caller then builds that mapping too)
  Alternative alt;
  if (free_choice && calibrate && !pool && !m.compact) {
    const int per_xcd = prop.multiProcessorCount / 8;
    const int units_per_wave = (kWave / m.lanes_per_row) / ((m.cell == SPRNN_CELL_LSTM || m.cell == SPRNN_CELL_GRU) ? 4 : 1);
    const int wt = (m.hidden + units_per_wave - 1) / units_per_wave;          // wavefronts that own rows
    const int wave_cap = m.template_words >= 48 ? 4 : kMaxWaves;
    const int waves2 = per_xcd > 0 ? (wt + per_xcd - 1) / per_xcd : 0;
    if (per_xcd >= 2 && m.grid > per_xcd && waves2 <= wave_cap &&
        m.cell != SPRNN_CELL_LSTM_BACKWARD && m.cell != SPRNN_CELL_GRU_BACKWARD) {
      alt.grid = (wt + waves2 - 1) / waves2;
    } else {
      // The copy of h issues its 16-byte loads in rounds of one per lane: exactly the rounds it needs up to three (in
      // the instantiations built for that), four up to four, and groups of eight beyond; a load past the end of h
      // fetches the last piece again and costs the CU's memory port as much as a useful one.  More wavefronts per
      // workgroup change the count: where some number of them would issue at least a tenth fewer loads per workgroup,
      // that mapping is measured as well.
      const int n4 = m.h_bytes / 16;
      auto issued = [&](int waves) {
        const int rounds = (n4 + waves * kWave - 1) / (waves * kWave);
        const int loads = rounds <= 3 && m.cell <= SPRNN_CELL_GRU ? rounds : (rounds <= 4 ? 4 : (rounds + 7) / 8 * 8);
        return (int64_t)loads * waves;
      };
      int best_waves = m.waves;
      for (int w2 = m.waves + 1; w2 <= wave_cap; ++w2)
        if (issued(w2) < issued(best_waves)) best_waves = w2;
      if (best_waves != m.waves && issued(best_waves) * 10 <= issued(m.waves) * 9) alt.fill_waves = best_waves;
    }
  }
  if (calibrate) {
    const int rc2 = calibrate_poll_delay(h, try_one_xcd, long_runs || alt.grid > 0 || alt.fill_waves > 0);
    if (rc2 != SPRNN_OK) { release(h); return rc2; }
  }
  if (alternative) *alternative = alt;
  *out = h;
  return SPRNN_OK;
}

int sprnn_create_ex(sprnn_handle_t* out, int hidden, int batch, int activation, const int32_t* row_ptr,
                    const int32_t* col_idx, const uint16_t* val_fp16_bits, int device_id,
                    const sprnn_options_t* opt) {
  if (!out) return SPRNN_ERR_INVALID;
  *out = nullptr;
  int ndev = 0;
  if (!SPRNN_HIP(hipGetDeviceCount(&ndev))) return SPRNN_ERR_HIP;
  if (device_id < 0 || device_id >= ndev) return SPRNN_ERR_INVALID;
  DeviceGuard guard(device_id);
  if (!guard.ok) return SPRNN_ERR_HIP;
  hipDeviceProp_t prop;
  if (!SPRNN_HIP(hipGetDeviceProperties(&prop, device_id))) return SPRNN_ERR_HIP;
  if (opt && opt->launch == 2 && !prop.cooperativeLaunch) return SPRNN_ERR_UNSUPPORTED;

  // A layer whose own mapping needs a few more workgroups than one XCD has CUs may run faster on fewer, larger
  // workgroups that fit one XCD (the exchange then stays inside one L2), and a layer with a large h on workgroups of
  // more wavefronts (see create_one).  Which is faster depends on the matrix, so when nothing about the mapping was
  // asked for, both are built and calibrated with runs of the same length, and the faster handle is kept.
  const bool free_choice = !opt || (opt->grid == 0 && opt->waves == 0 && opt->fill_waves == 0 && opt->lanes_per_row == 0 &&
                                    opt->layout == 0 && opt->poll_delay == 0 && opt->xcd == 0 && opt->sync == 0 &&
                                    opt->timeline == 0 && opt->gather == 0 && opt->overlap == 0 && opt->compact == 0);
  sprnn_handle_t first = nullptr;
  Alternative alt;
  const int rc = create_one(&first, hidden, batch, activation, row_ptr, col_idx, val_fp16_bits, device_id, opt, prop,
                            free_choice, free_choice, &alt);
  if (rc != SPRNN_OK) return rc;
  if (!free_choice || first->calibrated_us <= 0.0f) { *out = first; return SPRNN_OK; }
  sprnn_options_t base = opt ? *opt : sprnn_options_t();
  if (!opt) std::memset(&base, 0, sizeof(base));
  // builds the mapping `other` asks for, measures it like the first, and keeps the faster of the two in `first`
  auto contend = [&](const sprnn_options_t& other) {
    sprnn_handle_t second = nullptr;
    const int rc2 = create_one(&second, hidden, batch, activation, row_ptr, col_idx, val_fp16_bits, device_id, &other, prop,
                               false, true, nullptr);
    static const bool verbose = std::getenv("SPRNN_DEBUG") != nullptr;
    if (verbose)
      std::fprintf(stderr, "sprnn_create: contender (lanes %d, grid %d, fill %d) -> %s, %d x %d, %.3f us per step against %.3f\n",
                   other.lanes_per_row, other.grid, other.fill_waves, sprnn_status_string(rc2), rc2 == SPRNN_OK ? second->map.grid : 0,
                   rc2 == SPRNN_OK ? second->map.block : 0, rc2 == SPRNN_OK ? second->calibrated_us : 0.0f, first->calibrated_us);
    if (rc2 != SPRNN_OK) return;
    if (second->calibrated_us > 0.0f && second->calibrated_us < 0.98f * first->calibrated_us) {
      release(first);
      first = second;
    } else {
      release(second);
    }
  };
  // (1) fewer, larger workgroups on one XCD, or a wavefront count that copies h with fewer loads (see create_one)
  if (alt.grid > 0 || alt.fill_waves > 0) {
    sprnn_options_t other = base;
    other.grid = alt.grid;
    other.fill_waves = alt.fill_waves;
    contend(other);
  }
  // (2) The lanes a row is spread over: the packer's rule of thumb (at least eight nonzeros per lane) is not the best
  // for every shape; twice and half as many lanes are measured too, each with the mapping the packer picks for it.
  const int own_lanes = first->map.lanes_per_row;
  const bool gated_rows = first->map.cell == SPRNN_CELL_LSTM || first->map.cell == SPRNN_CELL_GRU;
  for (int pass = 0; pass < 2; ++pass) {
    const int lanes = pass == 0 ? own_lanes * 2 : own_lanes / 2;
    if (lanes < batch || lanes < 1 || lanes > (gated_rows ? 16 : kWave)) continue;
    sprnn_options_t other = base;
    other.lanes_per_row = lanes;
    contend(other);
  }
  *out = first;
  return SPRNN_OK;
}

int sprnn_create(sprnn_handle_t* out, int hidden, int batch, int activation, const int32_t* row_ptr,
                 const int32_t* col_idx, const uint16_t* val_fp16_bits, int device_id) {
  return sprnn_create_ex(out, hidden, batch, activation, row_ptr, col_idx, val_fp16_bits, device_id, nullptr);
}

static int forward_persistent(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                              float* h_out, float* c_out, void* stream, const LaunchExtras& ex) {
  if (h->poisoned) return SPRNN_ERR_STATE;
  if (T == 0) return SPRNN_OK;
  DeviceGuard guard(h->device);
  if (!guard.ok) return SPRNN_ERR_HIP;
  if (!ex.shared_exchange) {
    // A launch on the handle's own ring carries the handle's position in that ring in its arguments and moves it on: a
    // captured launch would be replayed with a position the ring has left behind, and would take the last replay's
    // values for its own.  Under capture only the entry point that starts every call from a fresh ring may be used.
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)stream, &capturing) != hipSuccess) { (void)hipGetLastError(); capturing = hipStreamCaptureStatusNone; }
    if (capturing != hipStreamCaptureStatusNone) return SPRNN_ERR_UNSUPPORTED;
  }
  const Mapping& m = h->map;
  // The kernel addresses x and the outputs with 32-bit byte offsets from the start of the call, so a very
  // long sequence is run as several launches, each continuing from the last state of the one before.
  const size_t step_bytes = (size_t)m.batch * std::max(std::max(m.rows, m.cols), m.cell > SPRNN_ACT_IDENTITY ? 4 * m.hidden : 0) * 4;
  const int t_max = (int)std::max<size_t>(1, ((size_t)1 << 30) / step_bytes);
  const size_t hb = (size_t)m.batch * m.hidden;
  if (ex.backward && T > t_max) return SPRNN_ERR_UNSUPPORTED;   // time runs backwards: one launch only
  uint32_t* ring = h->d_ring;
  uint32_t* ctrl = h->d_ctrl;
  if (ex.shared_exchange) {
    unsigned char* const base = scratch_on_device(h->device);
    if (!base) return SPRNN_ERR_HIP;
    ctrl = reinterpret_cast<uint32_t*>(base);
    ring = reinterpret_cast<uint32_t*>(base + kScratchCtrlBytes);
    h->used_shared_exchange = true;
  }
  for (int t0 = 0; t0 < T; t0 += t_max) {
    const int tn = std::min(t_max, T - t0);
    if (ex.shared_exchange) {
      // the array keeps whatever the last call on this device left: every launch starts from a freshly marked ring and
      // cleared control words, as a new handle would (a fill kernel, so that the call can be captured in a graph)
      if (!SPRNN_HIP(launch_exchange_reset(ring, (size_t)m.h_bytes / 4, (size_t)m.cols * m.batch, kRingSlots, ctrl, kCtrlWords,
                                           (hipStream_t)stream))) return SPRNN_ERR_HIP;
    }
    KernelArgs a;
    a.words = h->d_words; a.lane_row = h->d_lane_row; a.wave_words = h->d_wave_words;
    a.fill_src = h->d_fill_src; a.wg_plane = h->d_wg_plane; a.fill_rows = m.fill_rows;
    a.lane_sum = h->d_lane_sum; a.gather_waves = m.row_waves;
    a.wave_early = ex.backward ? nullptr : h->d_wave_early;   // (only the forward pass consumes h in two parts)
    a.seg_rounds = ex.backward ? 0 : m.seg_rounds;
    a.one_xcd = h->one_xcd ? 1 : 0;
    a.launch_epoch = ex.shared_exchange ? 0u : h->launch_epoch;
    a.lds_h_bytes = m.grid == 1 ? m.lds_bytes / 2 : m.lds_bytes;
    a.ring = ring; a.ctrl = ctrl;
    a.x = x + (size_t)t0 * m.batch * m.rows;
    a.h0 = t0 ? h_out + (size_t)(t0 - 1) * hb : h0;
    a.c0 = t0 ? (c_out ? c_out + (size_t)(t0 - 1) * hb : nullptr) : c0;
    a.h_out = h_out + (size_t)t0 * hb;
    a.c_out = c_out ? c_out + (size_t)t0 * hb : nullptr;
    a.gates_out = ex.gates_out ? ex.gates_out + (size_t)t0 * m.batch * 4 * m.hidden : nullptr;   // [T][B][4H] for both gated cells
    a.dc0 = ex.dc0;
    a.b_hn = ex.b_hn;
    a.aux = ex.saved; a.dh0 = ex.dh0; a.bwd_h0 = ex.wgrad_h0; a.word_src = h->d_word_src; a.dU = ex.dU;
    a.side_src = ex.wgrad_h_fwd;
    a.timeline = h->d_timeline;
    { const char* tw = std::getenv("SPRNN_TIMELINE_WAVE"); a.tl_wave = tw ? std::atoi(tw) : 0; }
    a.hidden = m.cols; a.T = tn; a.lanes_per_row = m.lanes_per_row; a.act = m.cell; a.h_bytes = m.h_bytes;
    a.index_shift = m.index_shift; a.jitter = m.jitter; a.poll_delay = m.poll_delay; a.spin_limit = m.spin_limit; a.sync = m.sync;
    a.step_base = ex.shared_exchange ? 0u : h->step_base;
    a.barrier_base = ex.shared_exchange ? 0u : h->barrier_base;
    void* args[] = {&a};
    const bool lstm_bwd = m.cell == SPRNN_CELL_LSTM_BACKWARD || m.cell == SPRNN_CELL_GRU_BACKWARD;   // the handle's own kernel is the backward pass
    const void* kernel = ex.backward ? (ex.dU ? h->kernel_bwd_grad : (lstm_bwd ? h->kernel : h->kernel_bwd)) : h->kernel;
    const int launch_grid = m.grid * (h->one_xcd ? 8 : 1);
    hipError_t e;
    if (m.cooperative && m.grid > 1) {
      e = hipLaunchCooperativeKernel(kernel, dim3(launch_grid), dim3(m.block), args, (unsigned)h->launch_lds, (hipStream_t)stream);
    } else if (m.grid == 1) {
      // a single workgroup waits for nobody
      e = hipLaunchKernel(kernel, dim3(launch_grid), dim3(m.block), args, (unsigned)h->launch_lds, (hipStream_t)stream);
    } else {
      e = launch_in_order(h->device, kernel, launch_grid, m.block, args, (unsigned)h->launch_lds, (hipStream_t)stream);
    }
    if (!hip_ok(e, "launch of the persistent kernel")) return e == hipErrorCooperativeLaunchTooLarge ? SPRNN_ERR_CAPACITY : SPRNN_ERR_HIP;
    if (ex.shared_exchange) continue;   // (the handle's own ring did not move)
    h->launch_epoch += 1;
    const int ran = tn + ((ex.backward && (ex.dh0 || ex.dU)) ? 1 : 0);   // the backward pass adds the step that pairs delta_1 with h_0
    h->step_base += (uint32_t)ran;
    h->barrier_base += (uint32_t)(ran - 1);   // one barrier before every step but the first
  }
  return SPRNN_OK;
}

// The best back-off depends on how far apart the workgroups of this matrix finish a step (row lengths, LDS bank
// conflicts, cell type).  Polling too early is far more expensive than polling late, and the sweet spot moves
// from 3 to 12 units between the measured shapes, so it is measured once per handle: a short run on zero input
// for a handful of candidates, keeping the fastest.  Timing does not depend on the data.
static int calibrate_poll_delay(sprnn_handle_s* h, bool try_one_xcd, bool long_runs) {
  const Mapping& m = h->map;
  // (a launch of the one-XCD mode holds eight times the workgroups and costs a few microseconds more to start: the
  // comparison of the two placements runs long enough for the per-step time to decide, as it does at real lengths)
  const int T = (try_one_xcd || long_runs) ? 160 : 48;
  // (the gated cells' backward passes read [T][B][4H] kept gate values from the zero buffer)
  const size_t xn = (size_t)T * m.batch * std::max(std::max(m.rows, m.cols), 4 * m.hidden), hn = (size_t)T * m.batch * m.cols;
  float *d_x = nullptr, *d_h = nullptr, *d_c = nullptr, *d_v = nullptr;
  const bool gru_bwd = m.cell == SPRNN_CELL_GRU_BACKWARD;   // (its second output costs stores in every step: measured with it)
  hipEvent_t e0 = nullptr, e1 = nullptr;
  const bool lstm = m.cell == SPRNN_CELL_LSTM;
  bool ok = SPRNN_HIP(hipMalloc((void**)&d_x, xn * 4)) && SPRNN_HIP(hipMemset(d_x, 0, xn * 4)) &&
            SPRNN_HIP(hipMalloc((void**)&d_h, hn * 4)) && (!lstm || SPRNN_HIP(hipMalloc((void**)&d_c, hn * 4))) &&
            (!gru_bwd || SPRNN_HIP(hipMalloc((void**)&d_v, hn * 4))) &&
            SPRNN_HIP(hipEventCreate(&e0)) && SPRNN_HIP(hipEventCreate(&e1));
  int best = h->map.poll_delay;
  bool best_one_xcd = h->one_xcd;
  float best_ms_kept = 0.0f;
  int rc = SPRNN_OK;
  if (ok) {
    // The exchange inside one XCD is shorter, so its candidates start lower; it is tried second, and dropped for good if
    // the dispatcher did not put enough workgroups on one XCD (the kernel flags that in the status word and leaves).
    static const int spread[] = {-1, 1, 2, 3, 4, 6, 8, 10, 12, 16};   // (-1: none; a wavefront's polls queue behind its own publish anyway)
    static const int local[] = {-1, 1, 2, 3, 4, 6};
    float best_ms = 0.0f;
    for (int mode = h->one_xcd ? 1 : 0; mode < ((try_one_xcd || h->one_xcd) ? 2 : 1) && ok && rc == SPRNN_OK; ++mode) {
      h->one_xcd = mode == 1;
      const int* cand = mode ? local : spread;
      const int ncand = mode ? (int)(sizeof(local) / sizeof(int)) : (int)(sizeof(spread) / sizeof(int));
      for (int ci = 0; ci < ncand; ++ci) {
        const int c = cand[ci];
        h->map.poll_delay = c < 0 ? 0 : c;
        float ms = 0.0f, best_of = 0.0f;
        for (int rep = 0; rep < 4 && rc == SPRNN_OK; ++rep) {   // the first run of a setting warms up, the fastest of three counts
          if (!SPRNN_HIP(hipEventRecord(e0, nullptr))) { ok = false; break; }
          // (the LSTM's backward pass reads e_t, the gate values and the cell states: all from the zero buffer)
          LaunchExtras ex;
          const bool gated_bwd = m.cell == SPRNN_CELL_LSTM_BACKWARD || m.cell == SPRNN_CELL_GRU_BACKWARD;
          if (gated_bwd) { ex.backward = true; ex.saved = d_x; ex.gates_out = d_v; }
          rc = forward_persistent(h, T, d_x, nullptr, nullptr, d_h, gated_bwd ? d_x : d_c, nullptr, ex);
          if (rc != SPRNN_OK) break;
          if (!SPRNN_HIP(hipEventRecord(e1, nullptr)) || !SPRNN_HIP(hipEventSynchronize(e1)) || !SPRNN_HIP(hipEventElapsedTime(&ms, e0, e1))) { ok = false; break; }
          if (rep > 0 && (best_of == 0.0f || ms < best_of)) best_of = ms;
        }
        ms = best_of;
        if (!ok || rc != SPRNN_OK) break;
        if (mode == 1) {
          uint32_t status = 0;
          if (!SPRNN_HIP(hipMemcpy(&status, h->d_ctrl + kCtrlStatus, 4, hipMemcpyDeviceToHost))) { ok = false; break; }
          if (status & kStatusPlacement) {   // not enough workgroups on any XCD: this mode is not for this device state
            status &= ~kStatusPlacement;
            if (!SPRNN_HIP(hipMemcpy(h->d_ctrl + kCtrlStatus, &status, 4, hipMemcpyHostToDevice))) ok = false;
            break;
          }
        }
        if (best_ms == 0.0f || ms < best_ms) { best_ms = ms; best = h->map.poll_delay; best_one_xcd = mode == 1; }
      }
    }
    best_ms_kept = best_ms;
    // A gated cell's backward handle serves two kernels, the plain pass and the one with the weight gradient fused in,
    // and a mapping that suits one may not suit the other: handles are compared by the sum of both.
    const bool gated_bwd_cell = m.cell == SPRNN_CELL_LSTM_BACKWARD || m.cell == SPRNN_CELL_GRU_BACKWARD;
    if (ok && rc == SPRNN_OK && gated_bwd_cell && h->kernel_bwd_grad && best_ms > 0.0f) {
      float* d_dU = nullptr;
      h->map.poll_delay = best;
      h->one_xcd = best_one_xcd;
      if (SPRNN_HIP(hipMalloc((void**)&d_dU, std::max<size_t>((size_t)m.nnz, 1) * 4))) {
        float fused = 0.0f;
        for (int rep = 0; rep < 3 && ok && rc == SPRNN_OK; ++rep) {
          float ms = 0.0f;
          LaunchExtras ex;
          ex.backward = true; ex.saved = d_x; ex.gates_out = d_v; ex.wgrad_h_fwd = d_x; ex.dU = d_dU;
          if (!SPRNN_HIP(hipEventRecord(e0, nullptr))) { ok = false; break; }
          rc = forward_persistent(h, T, d_x, nullptr, nullptr, d_h, d_x, nullptr, ex);
          if (rc != SPRNN_OK) break;
          if (!SPRNN_HIP(hipEventRecord(e1, nullptr)) || !SPRNN_HIP(hipEventSynchronize(e1)) || !SPRNN_HIP(hipEventElapsedTime(&ms, e0, e1))) { ok = false; break; }
          if (rep > 0 && (fused == 0.0f || ms < fused)) fused = ms;
        }
        if (ok && rc == SPRNN_OK) best_ms_kept += fused;
      }
      (void)hipFree(d_dU);
    }
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(d_x); (void)hipFree(d_h); (void)hipFree(d_c); (void)hipFree(d_v);
  h->one_xcd = (ok && rc == SPRNN_OK) ? best_one_xcd : false;
  h->map.poll_delay = (ok && rc == SPRNN_OK) ? best : default_poll_delay(h->map);
  h->calibrated_us = (ok && rc == SPRNN_OK) ? best_ms_kept * 1000.0f / (float)T : 0.0f;
  if (rc == SPRNN_OK && sprnn_check(h) != SPRNN_OK) rc = SPRNN_ERR_STATE;
  return rc;   // allocation or timing trouble is not fatal: the fallback value is used
}

int sprnn_forward(sprnn_handle_t h, int T, const float* x, const float* h0, float* h_out, void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell > SPRNN_ACT_IDENTITY) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!x || !h_out)) return SPRNN_ERR_INVALID;
  return forward_persistent(h, T, x, h0, nullptr, h_out, nullptr, stream);
}

int sprnn_forward_noalloc(sprnn_handle_t h, int T, const float* x, const float* h0, float* h_out, void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell > SPRNN_ACT_IDENTITY) return SPRNN_ERR_UNSUPPORTED;
  if (h->map.half) return SPRNN_ERR_UNSUPPORTED;   // (the per-launch reset marks binary32 elements)
  if (T > 0 && (!x || !h_out)) return SPRNN_ERR_INVALID;
  // the ring of this layer must fit behind the control words of the static array
  if ((size_t)kRingSlots * (size_t)h->map.h_bytes + kScratchCtrlBytes > kScratchBytes) {
    static const bool verbose = std::getenv("SPRNN_DEBUG") != nullptr;
    if (verbose) std::fprintf(stderr, "sprnn_forward_noalloc: exchange ring of %zu bytes exceeds the static limit of %zu bytes\n",
                              (size_t)kRingSlots * (size_t)h->map.h_bytes, kScratchBytes - kScratchCtrlBytes);
    return SPRNN_ERR_CAPACITY;
  }
  LaunchExtras ex;
  ex.shared_exchange = true;
  return forward_persistent(h, T, x, h0, nullptr, h_out, nullptr, stream, ex);
}

int sprnn_forward_lstm(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                       float* h_out, float* c_out, void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_LSTM) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!x || !h_out || !c_out)) return SPRNN_ERR_INVALID;
  return forward_persistent(h, T, x, h0, c0, h_out, c_out, stream);
}

int sprnn_forward_lstm_train(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                             float* h_out, float* c_out, float* gates_out, void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_LSTM) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!x || !h_out || !c_out || !gates_out)) return SPRNN_ERR_INVALID;
  LaunchExtras ex;
  ex.gates_out = gates_out;
  return forward_persistent(h, T, x, h0, c0, h_out, c_out, stream, ex);
}

int sprnn_backward_lstm(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates, const float* c_fwd,
                        const float* c0, float* d_bprime, float* dh0, float* dc0, void* stream) {
  sprnn_handle_t h = h_transposed;
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_LSTM_BACKWARD) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!dh_ext || !gates || !c_fwd || !d_bprime)) return SPRNN_ERR_INVALID;
  if (T == 0) {   // nothing flows back: both initial-state gradients are zero
    DeviceGuard guard(h->device);
    if (!guard.ok) return SPRNN_ERR_HIP;
    const size_t n = (size_t)h->map.batch * h->map.hidden;
    for (float* out : {dh0, dc0})
      if (out && !SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(out), 0u, n, (hipStream_t)stream))) return SPRNN_ERR_HIP;
    return SPRNN_OK;
  }
  // (the kernel only reads the cell states; they travel in the forward pass's output slot of the argument block)
  LaunchExtras ex;
  ex.backward = true; ex.saved = gates; ex.dh0 = dh0; ex.dc0 = dc0;
  return forward_persistent(h, T, dh_ext, nullptr, c0, d_bprime, const_cast<float*>(c_fwd), stream, ex);
}

int sprnn_backward_lstm_with_weights(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates,
                                     const float* c_fwd, const float* c0, const float* h_fwd, const float* h0, float* d_bprime,
                                     float* dh0, float* dc0, float* dU_transposed, void* stream) {
  sprnn_handle_t h = h_transposed;
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_LSTM_BACKWARD || !h->kernel_bwd_grad || !h->d_word_src) return SPRNN_ERR_UNSUPPORTED;
  if (!dU_transposed && h->map.nnz > 0) return SPRNN_ERR_INVALID;
  if (T > 0 && (!dh_ext || !gates || !c_fwd || !h_fwd || !d_bprime)) return SPRNN_ERR_INVALID;
  if (T == 0) {   // nothing to sum, nothing flows back
    DeviceGuard guard(h->device);
    if (!guard.ok) return SPRNN_ERR_HIP;
    const size_t n = (size_t)h->map.batch * h->map.hidden;
    for (float* out : {dh0, dc0})
      if (out && !SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(out), 0u, n, (hipStream_t)stream))) return SPRNN_ERR_HIP;
    if (h->map.nnz > 0 && !SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(dU_transposed), 0u, (size_t)h->map.nnz, (hipStream_t)stream))) return SPRNN_ERR_HIP;
    return SPRNN_OK;
  }
  LaunchExtras ex;
  ex.backward = true; ex.saved = gates; ex.dh0 = dh0; ex.dc0 = dc0;
  ex.wgrad_h_fwd = h_fwd; ex.wgrad_h0 = h0; ex.dU = dU_transposed;
  return forward_persistent(h, T, dh_ext, nullptr, c0, d_bprime, const_cast<float*>(c_fwd), stream, ex);
}

int sprnn_forward_gru(sprnn_handle_t h, int T, const float* x, const float* b_hn, const float* h0, float* h_out,
                      void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_GRU) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!x || !h_out)) return SPRNN_ERR_INVALID;
  LaunchExtras ex;
  ex.b_hn = b_hn;
  return forward_persistent(h, T, x, h0, nullptr, h_out, nullptr, stream, ex);
}

int sprnn_forward_gru_train(sprnn_handle_t h, int T, const float* x, const float* b_hn, const float* h0, float* h_out,
                            float* gates_out, void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_GRU) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!x || !h_out || !gates_out)) return SPRNN_ERR_INVALID;
  LaunchExtras ex;
  ex.b_hn = b_hn; ex.gates_out = gates_out;
  return forward_persistent(h, T, x, h0, nullptr, h_out, nullptr, stream, ex);
}

int sprnn_backward_gru(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates, const float* h_fwd,
                       const float* h0, float* d_bprime, float* d_recurrent, float* dh0, void* stream) {
  sprnn_handle_t h = h_transposed;
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_GRU_BACKWARD) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!dh_ext || !gates || !h_fwd || !d_bprime)) return SPRNN_ERR_INVALID;
  if (T == 0) {   // nothing flows back
    DeviceGuard guard(h->device);
    if (!guard.ok) return SPRNN_ERR_HIP;
    if (dh0 && !SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(dh0), 0u, (size_t)h->map.batch * h->map.hidden, (hipStream_t)stream))) return SPRNN_ERR_HIP;
    return SPRNN_OK;
  }
  // (h_{t-1} travels where the LSTM's backward pass has its cell states, the second output where the forward pass
  // keeps gate values)
  LaunchExtras ex;
  ex.backward = true; ex.saved = gates; ex.dh0 = dh0; ex.gates_out = d_recurrent;
  return forward_persistent(h, T, dh_ext, nullptr, h0, d_bprime, const_cast<float*>(h_fwd), stream, ex);
}

int sprnn_backward_gru_with_weights(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates,
                                    const float* h_fwd, const float* h0, float* d_bprime, float* d_recurrent, float* dh0,
                                    float* dU_transposed, void* stream) {
  sprnn_handle_t h = h_transposed;
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell != SPRNN_CELL_GRU_BACKWARD || !h->kernel_bwd_grad || !h->d_word_src) return SPRNN_ERR_UNSUPPORTED;
  if (!dU_transposed && h->map.nnz > 0) return SPRNN_ERR_INVALID;
  if (T > 0 && (!dh_ext || !gates || !h_fwd || !d_bprime)) return SPRNN_ERR_INVALID;
  if (T == 0) {   // nothing to sum, nothing flows back
    DeviceGuard guard(h->device);
    if (!guard.ok) return SPRNN_ERR_HIP;
    if (dh0 && !SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(dh0), 0u, (size_t)h->map.batch * h->map.hidden, (hipStream_t)stream))) return SPRNN_ERR_HIP;
    if (h->map.nnz > 0 && !SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(dU_transposed), 0u, (size_t)h->map.nnz, (hipStream_t)stream))) return SPRNN_ERR_HIP;
    return SPRNN_OK;
  }
  LaunchExtras ex;
  ex.backward = true; ex.saved = gates; ex.dh0 = dh0; ex.gates_out = d_recurrent;
  ex.wgrad_h_fwd = h_fwd; ex.wgrad_h0 = h0; ex.dU = dU_transposed;
  return forward_persistent(h, T, dh_ext, nullptr, h0, d_bprime, const_cast<float*>(h_fwd), stream, ex);
}

int sprnn_backward(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* h_fwd, float* d_bprime,
                   float* dh0, void* stream) {
  sprnn_handle_t h = h_transposed;
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell > SPRNN_ACT_IDENTITY || !h->kernel_bwd) return SPRNN_ERR_UNSUPPORTED;
  if (T > 0 && (!dh_ext || !h_fwd || !d_bprime)) return SPRNN_ERR_INVALID;
  if (T == 0) {   // nothing flows back
    if (!dh0) return SPRNN_OK;
    DeviceGuard guard(h->device);
    if (!guard.ok) return SPRNN_ERR_HIP;
    return SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(dh0), 0u, (size_t)h->map.batch * h->map.hidden, (hipStream_t)stream)) ? SPRNN_OK : SPRNN_ERR_HIP;
  }
  LaunchExtras ex;
  ex.backward = true; ex.saved = h_fwd; ex.dh0 = dh0;
  return forward_persistent(h, T, dh_ext, nullptr, nullptr, d_bprime, nullptr, stream, ex);
}

int sprnn_backward_with_weights(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* h_fwd, const float* h0,
                                float* d_bprime, float* dh0, float* dU_transposed, void* stream) {
  sprnn_handle_t h = h_transposed;
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell > SPRNN_ACT_IDENTITY || !h->kernel_bwd_grad || !h->d_word_src) return SPRNN_ERR_UNSUPPORTED;
  if (!dU_transposed && h->map.nnz > 0) return SPRNN_ERR_INVALID;
  if (T > 0 && (!dh_ext || !h_fwd || !d_bprime)) return SPRNN_ERR_INVALID;
  if (T == 0) {   // nothing to sum, nothing flows back
    DeviceGuard guard(h->device);
    if (!guard.ok) return SPRNN_ERR_HIP;
    if (dh0 && !SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(dh0), 0u, (size_t)h->map.batch * h->map.hidden, (hipStream_t)stream))) return SPRNN_ERR_HIP;
    if (h->map.nnz == 0) return SPRNN_OK;
    return SPRNN_HIP(launch_fill(reinterpret_cast<uint32_t*>(dU_transposed), 0u, (size_t)h->map.nnz, (hipStream_t)stream)) ? SPRNN_OK : SPRNN_ERR_HIP;
  }
  LaunchExtras ex;
  ex.backward = true; ex.saved = h_fwd; ex.dh0 = dh0;   // (vanilla cells: g' and the weight gradient both use h_t)
  ex.wgrad_h_fwd = h_fwd; ex.wgrad_h0 = h0; ex.dU = dU_transposed;
  return forward_persistent(h, T, dh_ext, nullptr, nullptr, d_bprime, nullptr, stream, ex);
}

int sprnn_weight_gradient(sprnn_handle_t h, int T, const float* d_bprime, const float* h_fwd, const float* h0, float* dU,
                          void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (!h->kernel_wgrad || !h->d_word_src) return SPRNN_ERR_UNSUPPORTED;   // gated cell, or column compaction in use
  if (!dU && h->map.nnz > 0) return SPRNN_ERR_INVALID;
  if (T > 0 && (!d_bprime || !h_fwd)) return SPRNN_ERR_INVALID;
  if (h->map.nnz == 0) return SPRNN_OK;
  DeviceGuard guard(h->device);
  if (!guard.ok) return SPRNN_ERR_HIP;
  const Mapping& m = h->map;
  WGradArgs a;
  a.words = h->d_words; a.lane_row = h->d_lane_row; a.wave_words = h->d_wave_words; a.word_src = h->d_word_src;
  a.delta = d_bprime; a.h_fwd = h_fwd; a.h0 = h0; a.dU = dU;
  a.hidden = m.hidden; a.T = T; a.index_shift = m.index_shift; a.rows = m.rows;
  void* args[] = {&a};
  // workgroups are independent here: an ordinary launch, one workgroup per CU by the same LDS request
  const hipError_t e = hipLaunchKernel(h->kernel_wgrad, dim3(m.grid), dim3(m.block), args, (unsigned)h->launch_lds, (hipStream_t)stream);
  return hip_ok(e, "hipLaunchKernel(weight gradient)") ? SPRNN_OK : SPRNN_ERR_HIP;
}

int sprnn_transpose_csr(int rows, int cols, const int32_t* row_ptr, const int32_t* col_idx, const uint16_t* val_fp16_bits,
                        int32_t* t_row_ptr, int32_t* t_col_idx, uint16_t* t_val_fp16_bits, int32_t* t_source) {
  if (rows < 0 || cols < 0 || !row_ptr || !t_row_ptr) return SPRNN_ERR_INVALID;
  const int64_t nnz = row_ptr[rows];
  if (nnz < 0 || (nnz > 0 && (!col_idx || !val_fp16_bits || !t_col_idx || !t_val_fp16_bits))) return SPRNN_ERR_INVALID;
  for (int c = 0; c <= cols; ++c) t_row_ptr[c] = 0;
  for (int64_t k = 0; k < nnz; ++k) {
    if (col_idx[k] < 0 || col_idx[k] >= cols) return SPRNN_ERR_INVALID;
    ++t_row_ptr[col_idx[k] + 1];
  }
  for (int c = 0; c < cols; ++c) t_row_ptr[c + 1] += t_row_ptr[c];
  std::vector<int32_t> next(t_row_ptr, t_row_ptr + cols);
  for (int r = 0; r < rows; ++r)   // rows in ascending order, so the columns of a transposed row come out ascending
    for (int32_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      const int32_t at = next[col_idx[k]]++;
      t_col_idx[at] = r;
      t_val_fp16_bits[at] = val_fp16_bits[k];
      if (t_source) t_source[at] = k;
    }
  return SPRNN_OK;
}

int sprnn_forward_stepwise(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                           float* h_out, float* c_out, void* stream) {
  if (!h || T < 0) return SPRNN_ERR_INVALID;
  if (h->map.cell == SPRNN_CELL_GRU || h->map.cell >= SPRNN_CELL_LSTM_BACKWARD) return SPRNN_ERR_UNSUPPORTED;
  const Mapping& m = h->map;
  const bool lstm = m.cell == SPRNN_CELL_LSTM;
  if (T > 0 && (!x || !h_out || (lstm && !c_out))) return SPRNN_ERR_INVALID;
  DeviceGuard guard(h->device);
  if (!guard.ok) return SPRNN_ERR_HIP;
  const size_t hb = (size_t)m.batch * m.hidden, xb = (size_t)m.batch * m.rows;
  for (int t = 0; t < T; ++t) {
    StepArgs a;
    a.row_ptr = h->d_row_ptr; a.col = h->d_col; a.val = h->d_val;
    a.x_t = x + (size_t)t * xb;
    a.h_prev = t ? h_out + (size_t)(t - 1) * hb : h0;
    a.c_prev = lstm ? (t ? c_out + (size_t)(t - 1) * hb : c0) : nullptr;
    a.h_cur = h_out + (size_t)t * hb;
    a.c_cur = lstm ? c_out + (size_t)t * hb : nullptr;
    a.hidden = m.hidden; a.act = m.cell;
    if (launch_stepwise(m.batch, lstm, a, (hipStream_t)stream) != hipSuccess) return SPRNN_ERR_HIP;
  }
  return SPRNN_OK;
}

int sprnn_project(sprnn_handle_t h, int T, int input_size, const float* x_in, const uint16_t* w_in_fp16_bits,
                  const float* bias, float* b_prime, void* stream) {
  if (!h || T < 0 || input_size <= 0) return SPRNN_ERR_INVALID;
  if (T > 0 && (!x_in || !w_in_fp16_bits || !b_prime)) return SPRNN_ERR_INVALID;
  if ((long long)T * h->map.batch > 0x7fffffffLL) return SPRNN_ERR_INVALID;
  if (h->map.cell >= SPRNN_CELL_LSTM_BACKWARD) return SPRNN_ERR_UNSUPPORTED;
  if (T == 0) return SPRNN_OK;
  DeviceGuard guard(h->device);
  if (!guard.ok) return SPRNN_ERR_HIP;
  const hipError_t e = launch_project(x_in, w_in_fp16_bits, bias, b_prime, T * h->map.batch, h->map.rows, input_size,
                                      static_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue) return SPRNN_ERR_INVALID;
  return SPRNN_HIP(e) ? SPRNN_OK : SPRNN_ERR_HIP;
}

int sprnn_read_timeline(sprnn_handle_t h, uint64_t* out, int capacity_words, double* ticks_per_second) {
  if (!h || !out) return SPRNN_ERR_INVALID;
  if (!h->d_timeline) return SPRNN_ERR_UNSUPPORTED;
  const size_t n = (size_t)h->map.grid * kTimelineSlots;
  if (capacity_words < (int)n) return SPRNN_ERR_INVALID;
  DeviceGuard guard(h->device);
  if (!guard.ok) return SPRNN_ERR_HIP;
  if (!SPRNN_HIP(hipDeviceSynchronize())) return SPRNN_ERR_HIP;
  if (!SPRNN_HIP(hipMemcpy(out, h->d_timeline, n * 8, hipMemcpyDeviceToHost))) return SPRNN_ERR_HIP;
  if (!SPRNN_HIP(hipMemset(h->d_timeline, 0, n * 8))) return SPRNN_ERR_HIP;
  if (ticks_per_second) {
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, h->device) != hipSuccess || khz <= 0) khz = 100000;
    *ticks_per_second = khz * 1e3;
  }
  return SPRNN_OK;
}

int sprnn_get_info(sprnn_handle_t h, sprnn_info_t* info) {
  if (!h || !info) return SPRNN_ERR_INVALID;
  fill_info(h->map, h->capacity, h->pass_factor, info);
  info->one_xcd = h->one_xcd ? 1 : 0;
  return SPRNN_OK;
}

int sprnn_check(sprnn_handle_t h) {
  if (!h) return SPRNN_ERR_INVALID;
  DeviceGuard guard(h->device);
  if (!guard.ok) return SPRNN_ERR_HIP;
  if (hipDeviceSynchronize() != hipSuccess) return SPRNN_ERR_HIP;
  uint32_t status = 0;
  if (hipMemcpy(&status, h->d_ctrl + kCtrlStatus, 4, hipMemcpyDeviceToHost) != hipSuccess) return SPRNN_ERR_HIP;
  if (!status && h->used_shared_exchange) {
    // sprnn_forward_noalloc keeps its status word in the device's static array (cleared by every such call)
    unsigned char* const base = scratch_on_device(h->device);
    if (!base || hipMemcpy(&status, reinterpret_cast<uint32_t*>(base) + kCtrlStatus, 4, hipMemcpyDeviceToHost) != hipSuccess) return SPRNN_ERR_HIP;
  }
  if (status) h->poisoned = true;
  return status ? SPRNN_ERR_STATE : SPRNN_OK;
}

int sprnn_destroy(sprnn_handle_t h) {
  if (!h) return SPRNN_OK;
  DeviceGuard guard(h->device);
  if (guard.ok) (void)hipDeviceSynchronize();
  release(h);
  return SPRNN_OK;
}

}  // extern "C"
