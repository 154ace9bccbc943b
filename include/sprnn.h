/*
 * sprnn — persistent sparse recurrent step for AMD MI355X (gfx950).
 *
 * C ABI of libsprnn.so.  Every function returns an SPRNN_* status code (0 = success, negative =
 * error); nothing throws or aborts across this boundary.  "host" pointers are ordinary CPU memory,
 * "device" pointers are HIP device memory on the GPU the handle was created for.  The library never
 * allocates inside a forward call: all device storage it needs (packed weights, exchange ring,
 * status word) is allocated by sprnn_create and released by sprnn_destroy.
 *
 * One HIP runtime per process: libsprnn.so links against libamdhip64.so.7 and uses whichever copy the process
 * has already mapped.  A process that also uses another HIP client that ships its own runtime (PyTorch does)
 * must load that client FIRST, so that the dynamic linker resolves libsprnn's dependency to the copy already
 * in the process; streams and device pointers of one runtime are invalid in another.  The Python binding
 * enforces this (it imports torch before loading the library and refuses to run with two runtimes mapped).
 *
 * Threads: different handles may be used from different host threads at the same time (the library's own per-device
 * state is guarded); calls on ONE handle must not overlap, on the host (each call advances the handle's position in
 * its exchange ring) or on the device (two launches of one handle share that ring: give them to one stream, or order
 * the streams yourself).
 *
 * What is computed (paper, Section 3.1, Eq. 2):  h_t = g(U_r h_{t-1} + b'_t)  for t = 1..T, with
 * U_r the pruned recurrent weight matrix held in on-chip storage for the whole sequence
 * (Section 3.3) and b'_t = W x_t + b computed by the caller ahead of time (Eq. 1 -> Eq. 2).
 * The LSTM variant (Appendix B, first paragraph) keeps four gate rows per hidden unit.
 */
#ifndef SPRNN_H_
#define SPRNN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sprnn_handle_s* sprnn_handle_t; /* opaque */

enum {
  SPRNN_OK = 0,
  SPRNN_ERR_INVALID = -1,     /* bad argument or malformed CSR                                   */
  SPRNN_ERR_CAPACITY = -2,    /* weights do not fit on chip, or grid exceeds co-resident capacity */
  SPRNN_ERR_HIP = -3,         /* a HIP runtime call failed                                        */
  SPRNN_ERR_UNSUPPORTED = -4, /* batch not in {1,2,4,8}, hidden > 65535, wrong cell for the call  */
  SPRNN_ERR_STATE = -5        /* a previous forward tripped the spin watchdog; handle unusable    */
};

/* Cell / activation g of Eq. 2.  SPRNN_CELL_LSTM selects the four-gate cell of Appendix B, SPRNN_CELL_GRU a
 * three-gate gated recurrent unit (Section 2 names it as a cell the approach extends to).
 * SPRNN_CELL_LSTM_BACKWARD makes a handle for the backward pass of an LSTM layer (sprnn_backward_lstm): it holds the
 * TRANSPOSE of the LSTM's [4H][H] matrix, H rows whose columns index the 4H gate rows; SPRNN_CELL_GRU_BACKWARD the
 * same for the GRU (sprnn_backward_gru, the transpose of its [3H][H] matrix). */
enum { SPRNN_ACT_RELU = 0, SPRNN_ACT_TANH = 1, SPRNN_ACT_IDENTITY = 2, SPRNN_CELL_LSTM = 3, SPRNN_CELL_GRU = 4,
       SPRNN_CELL_LSTM_BACKWARD = 5, SPRNN_CELL_GRU_BACKWARD = 6 };

/* Cross-workgroup hand-off of h_t (Section 4.2 discusses a global barrier versus Lamport timestamps). */
enum {
  SPRNN_SYNC_AUTO = 0,
  SPRNN_SYNC_TAGGED = 1, /* validity travels with the data; consumers spin on it (Lamport-style)  */
  SPRNN_SYNC_BARRIER = 2 /* one grid-wide barrier per timestep                                     */
};

/*
 * Optional tuning knobs for sprnn_create_ex; zero in any field means "choose automatically".
 * They change only where operands live and in which order they are visited, never the result
 * (Section 4.1: re-ordering the nonzeros of a row does not affect the final result).
 */
typedef struct sprnn_options_s {
  int grid;          /* number of persistent workgroups (<= co-resident capacity)                  */
  int waves;         /* wavefronts (64 lanes) per workgroup, 1..12                                 */
  int lanes_per_row; /* lanes that share one weight row: batch,...,32,64 (<= 16 for the gated cells) */
  int sync;          /* SPRNN_SYNC_*                                                               */
  int bank_aware;    /* 0 auto, 1 = bank-aware ordering of a row's nonzeros (Section 4.1, App. A),
                        2 = keep CSR order ("naive")                                               */
  int balance;       /* 0 auto, 1 = rows dealt to workgroups by nonzero count, 2 = contiguous rows */
  int poll_delay;    /* back-off before the first poll of a step, in units of 64 clocks; 0 = measured
                        at create time on a short zero-input run (a few ms), -1 none               */
  int spin_limit;    /* polls before the watchdog gives up (0 = default)                           */
  int timeline;      /* 1 = workgroup 0..grid-1 accumulate per-phase times (see sprnn_read_timeline) */
  int fill_waves;    /* total wavefronts per workgroup when larger than `waves`: the extra ones own no
                        rows and only help to copy h into LDS                                      */
  int launch;        /* how the persistent kernel is started: 0 or 1 = ordinary kernel launch, 2 = cooperative
                        launch.  The workgroups spin on each other and must all be resident at once.  The
                        library checks at create time that the grid fits the device, and it orders its own
                        persistent launches on a device one after the other, whatever streams they are given
                        to (an event behind every launch on a caller-made stream, a few microseconds per
                        call, and between the default stream and others when needed; not inside a stream
                        capture), so two of them never wait for each other's compute units.  Other kernels on
                        other streams only delay a launch.  What an ordinary launch cannot rule out is another
                        PROCESS spinning on the same device at the same time: every wait is bounded, so that
                        ends in SPRNN_ERR_STATE from sprnn_check, not in a hang.  A cooperative launch has the
                        runtime enforce exclusive residency instead; it costs about 16 us more per call, and
                        the HIP runtime grants cooperative launches to one process per device at a time
                        (another process gets SPRNN_ERR_HIP from sprnn_create)                         */
  int jitter;        /* test aid: non-zero seeds pseudo-random pauses (0..15 x 64 clocks) of every
                        wavefront before it publishes, before it polls and after it has copied h,
                        different in every step, to widen the windows of any race in the hand-off;
                        results must not change                                                   */
  int compact;       /* column compaction: a workgroup copies only the 16-byte pieces of h that its rows
                        read, into consecutive LDS positions.  0 auto (when all of h does not fit in
                        LDS, or every workgroup needs less than half of it), 1 on, 2 off            */
  int layout;        /* how the lanes of a workgroup are given to rows (vanilla cells, more than one workgroup):
                        0 auto, 1 = one power-of-two lane group per row, every wavefront does every stage,
                        2 = lane pool: a row takes as many groups of `batch` lanes as its nonzeros need out of a
                        pool of 4 or 7 gathering wavefronts, and separate wavefronts own b', g and the stores  */
  int gather;        /* 0 auto, 1 = one wide LDS read per nonzero fetches all samples of its column (Section 4.1's wide
                        loads), 2 = one 4-byte read per sample (the rung below it in the ablation; batch 4, vanilla
                        cells, layout 1, forward pass only)                                            */
  int xcd;           /* small layers (at most 32 workgroups; not the gated cells' backward passes): 0 auto = measured at
                        create time together with the back-off, 1 = workgroups spread over all XCDs, 2 = one XCD:
                        the launch holds eight times the workgroups, those that the dispatcher put on one XCD take
                        the work and exchange h through that XCD's L2 alone (if it put too few there, the launch
                        leaves without results and sprnn_check reports SPRNN_ERR_STATE)                       */
  int overlap;       /* copy of h into LDS overlapped with the gathers (vanilla cells, forward pass, batch <= 4, no column
                        compaction, 2..8 copy rounds): 0 auto, 1 off, 2 on = the columns of h are consumed in two
                        parts; a row's nonzeros of the first part sit in its lanes' leading slots and are worked
                        through while the second part is still arriving                                    */
  int activations;   /* precision in which h travels between workgroups and sits in LDS (vanilla cells, forward pass, batch 4
                        and 8, one lane group per row): 0 auto = 1 = binary32 (the default everywhere);
                        2 = binary16 (Section 6 names lower-precision activations as future work): every h_t is rounded
                        to nearest once before it is published, sums, b' and h_out stay binary32, so h_out[t] is the
                        unrounded value while step t + 1 reads the rounded one.  Half the exchange and LDS traffic;
                        the error against binary32 activations is a few 1e-4 of max|h|, inside the 1e-3 bound of the
                        tests but no longer far inside                                                        */
} sprnn_options_t;

/* Filled by sprnn_get_info: how the matrix was mapped onto the chip. */
typedef struct sprnn_info_s {
  int hidden, rows, batch, cell;
  int grid, block, waves, lanes_per_row, sync, bank_aware, balance, poll_delay;
  int words_per_lane_max;   /* largest number of packed nonzeros held by one lane                 */
  int template_words;       /* register slots per lane of the kernel instantiation in use         */
  int lds_bytes;            /* LDS bytes per workgroup for h (one copy; two when grid is 1; less
                               with column compaction)                                               */
  int resident_capacity;    /* co-resident workgroups the device can hold for this kernel         */
  int64_t nnz;              /* nonzeros in the CSR input                                           */
  int64_t padded_words;     /* packed words including zero padding                                 */
  int64_t ring_bytes;       /* size of the exchange ring in device memory                          */
  double lds_pass_factor;   /* LDS passes the packed gathers need / passes of a conflict-free layout
                               (1.0 = no bank conflicts), from the 64-bank, 256 B-per-pass model     */
  int compact;              /* 1 if column compaction is in use                                      */
  int layout;               /* 1 = one lane group per row, 2 = lane pool (see sprnn_options_t.layout)   */
  int gather_waves;         /* wavefronts per workgroup that hold weights (all of them for layout 1)    */
  int one_xcd;              /* 1 if the workgroups are confined to one XCD (see sprnn_options_t.xcd)     */
  int overlap_rounds;       /* > 0: copy rounds (one 16-byte piece per lane each) that make up the first part of h when
                               the copy is overlapped with the gathers (see sprnn_options_t.overlap)     */
  int overlap_words;        /* leading slots per lane that read only that first part: least over the wavefronts */
  int activations;          /* 1 = h is exchanged as binary32, 2 = as binary16 (see sprnn_options_t.activations)   */
  int reserved[1];
} sprnn_info_t;

/*
 * Validate, pack and upload a pruned recurrent matrix (the one-time weight preparation of
 * Sections 3.3 and 4.1: <index,value> pairs per row, zero padding, bank-aware ordering, all
 * nonzeros of a lane from one row).
 *
 *   hidden      H, 1..65535.
 *   batch       B in {1,2,4,8}: sequences advanced together (wide loads of Section 4.1).
 *   activation  SPRNN_ACT_* (R = H rows), SPRNN_CELL_LSTM (R = 4H rows, row blocks i|f|g|o),
 *               SPRNN_CELL_GRU (R = 3H rows, row blocks r|z|n), SPRNN_CELL_LSTM_BACKWARD (R = H rows with
 *               columns below 4H, H <= 16383: the transpose of an LSTM's matrix) or SPRNN_CELL_GRU_BACKWARD (R = H rows
 *               with columns below 3H, H <= 21845).
 *   row_ptr     host, R+1 entries, row_ptr[0] = 0, non-decreasing.
 *   col_idx     host, nnz = row_ptr[R] entries, 0 <= col < H (< 4H, < 3H for the two backward cells), strictly
 *               increasing inside a row.
 *   val_fp16_bits host, nnz IEEE binary16 bit patterns (finite).  The library rounds nothing.
 *   device_id   HIP device ordinal.
 *
 * The arrays are copied; the caller may free them on return.  On error *out is NULL.
 * Empty rows and an all-empty matrix are legal.
 */
int sprnn_create(sprnn_handle_t* out, int hidden, int batch, int activation, const int32_t* row_ptr,
                 const int32_t* col_idx, const uint16_t* val_fp16_bits, int device_id);

/* Same, with tuning knobs (opt may be NULL).  Unless opt fixes the back-off (poll_delay), creation runs a few short
 * launches on zero input on the device's default stream to measure it (and the XCD placement, if xcd is 0) and
 * synchronizes the device.  When opt fixes nothing about the mapping (grid, waves, fill_waves, lanes_per_row,
 * layout, poll_delay, xcd, sync, timeline, gather, overlap, compact all 0), up to three more mappings are built and
 * measured the same way, and the fastest is kept (sprnn_get_info reports the one in use): fewer, larger workgroups when
 * the layer needs only a few more than one XCD has compute units, or another number of wavefronts per workgroup when
 * that copies a large h with at least a tenth fewer loads; and twice and half the lanes per row.  Creation then takes
 * 0.05 to 0.25 s depending on the size of the matrix (the packing runs on several host threads).
 * Results are bit-for-bit the same from call to call on one handle, and between handles with the same lanes_per_row
 * (which fixes the order in which a row's products are added); a caller who needs that across handles passes the value
 * sprnn_get_info reported for the first. */
int sprnn_create_ex(sprnn_handle_t* out, int hidden, int batch, int activation, const int32_t* row_ptr,
                    const int32_t* col_idx, const uint16_t* val_fp16_bits, int device_id,
                    const sprnn_options_t* opt);

/*
 * Run T timesteps of Eq. 2 with one persistent kernel launch (the load / operate / reduce /
 * synchronize pipeline of Section 3.3).  Vanilla cells only.
 *
 *   x      device, float32 [T][B][H], H fastest: b'_t of Eq. 2.
 *   h0     device, float32 [B][H], or NULL for zeros.
 *   h_out  device, float32 [T][B][H]: every h_t; h_out[T-1] is the final state.  A result that
 *          would be -0.0 is written as +0.0 (Section 4.2 reserves -0.0 as the "not yet written" mark).
 *   stream hipStream_t cast to void* (NULL = default stream).
 *
 * Only enqueues work on `stream` and returns.  One forward per handle at a time, in stream order;
 * calls on different handles are independent.  T = 0 is a no-op.  All activations must be finite.
 * Not under stream capture (SPRNN_ERR_UNSUPPORTED): every call on a handle's own exchange ring, this one and all
 * the others except sprnn_forward_noalloc, carries the handle's position in that ring in its launch and moves it on,
 * so a replayed launch would not find the ring where it expects it.  sprnn_forward_noalloc may be captured.
 */
int sprnn_forward(sprnn_handle_t h, int T, const float* x, const float* h0, float* h_out, void* stream);

/*
 * sprnn_forward for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernels and results, but the exchange ring and the control words live in
 * one array of 1 MiB that the library holds in static device memory on every GPU it runs on (until the process ends)
 * instead of the handle's own allocations.  Calls no hipMalloc, hipFree or other allocating routine; enqueues one
 * small fill kernel (the array keeps the last call's contents, so ring marks and control words are set afresh) and the
 * persistent kernel.  Vanilla cells only; arguments as sprnn_forward.
 *   Limit: 4 ring slots of the layer (4 * 4 * B * H bytes, rounded up to 16 per slot) plus 1 KiB must fit in the
 *   array, i.e. B * H <= 65 472; larger layers get SPRNN_ERR_CAPACITY and nothing is enqueued.
 *   All calls on one GPU share that GPU's array: two such calls that overlap in time on one GPU (different streams,
 *   different handles) race and are not allowed; calls in stream order are fine.  sprnn_check on the handle also
 *   reports a watchdog trip of its most recent call here.
 */
int sprnn_forward_noalloc(sprnn_handle_t h, int T, const float* x, const float* h0, float* h_out, void* stream);

/*
 * LSTM cell (Appendix B): x is float32 [T][B][4H] with gate blocks i|f|g|o (biases folded in),
 * c0 / h0 are [B][H] or NULL, h_out and c_out are [T][B][H].
 *   c_t = sigmoid(p_f) c_{t-1} + sigmoid(p_i) tanh(p_g),  h_t = sigmoid(p_o) tanh(c_t).
 */
int sprnn_forward_lstm(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                       float* h_out, float* c_out, void* stream);

/*
 * sprnn_forward_lstm that also keeps what the backward pass needs: gates_out, device float32 [T][B][4H], receives the
 * gate values after their activations, blocks sigmoid(p_i) | sigmoid(p_f) | tanh(p_g) | sigmoid(p_o).
 */
int sprnn_forward_lstm_train(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                             float* h_out, float* c_out, float* gates_out, void* stream);

/*
 * GRU cell: x is float32 [T][B][3H] with gate blocks r|z|n (input projection and every bias except b_hn folded in),
 * b_hn is device float32 [H] or NULL (zeros): the recurrent bias of the candidate, which sits inside the reset
 * product; h0 is [B][H] or NULL, h_out is [T][B][H].
 *   r = sigmoid(p_r), z = sigmoid(p_z), n = tanh(x_n + r (U_n h_{t-1} + b_hn)),  h_t = (1 - z) n + z h_{t-1}.
 * Internally the unit keeps the four-row layout of the LSTM with the fourth row empty.
 */
int sprnn_forward_gru(sprnn_handle_t h, int T, const float* x, const float* b_hn, const float* h0, float* h_out,
                      void* stream);

/*
 * Backward pass through time of a vanilla cell with the pruned weights resident on chip (Appendix B.1: the pruned
 * weights are used for the computation of both passes).  For a loss L with e_t = dL/dh_t from outside the layer,
 *   delta_t = g'(a_t) (e_t + U_r^T delta_{t+1}),  delta_{T+1} = 0,   dL/db'_t = delta_t,   dL/dh_0 = U_r^T delta_1,
 * which is the forward recurrence on the transposed matrix with time reversed and g' (taken from the forward
 * output: ReLU h_t > 0, tanh 1 - h_t^2, identity 1) in place of g.  The handle must therefore have been created
 * from the TRANSPOSE of the forward matrix (sprnn_transpose_csr) with the forward pass's activation and batch.
 *
 *   dh_ext    device, float32 [T][B][H]: e_t.
 *   h_fwd     device, float32 [T][B][H]: the forward outputs h_1..h_T.
 *   d_bprime  device, float32 [T][B][H]: delta_t (the gradient of the input projection's output; the gradient of
 *             the recurrent weights follows from it without a recurrence: sprnn_weight_gradient).
 *   dh0       device, float32 [B][H], or NULL if not wanted.
 * One launch; T is limited to 2^30 / (4 B H) timesteps per call.  Same stream, state and error rules as sprnn_forward.
 */
int sprnn_backward(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* h_fwd, float* d_bprime,
                   float* dh0, void* stream);

/*
 * sprnn_backward with the gradient of the recurrent weights fused in.  The column of delta_{t+1} that a lane gathers
 * for a nonzero (j, i) of the transposed matrix is exactly the factor that dL/dU[i][j] pairs with the forward output
 * h_t[.][j] of the lane's own row, so every gather of the recurrence also feeds one accumulator per nonzero that
 * stays in a register for the whole sequence; the sums cost no extra pass over h.
 *   h0             device, float32 [B][H] or NULL (zeros): h_0 of the forward pass (pairs with delta_1).
 *   dU_transposed  device, float32 [nnz]: dL/dU in the order of the TRANSPOSED matrix's CSR arrays (entry p belongs to
 *                  the forward nonzero t_source[p] of sprnn_transpose_csr); overwritten.
 * Other arguments as sprnn_backward.  Not available with column compaction (SPRNN_ERR_UNSUPPORTED).
 */
int sprnn_backward_with_weights(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* h_fwd, const float* h0,
                                float* d_bprime, float* dh0, float* dU_transposed, void* stream);

/*
 * Gradient of the recurrent weights on their sparsity pattern, the non-recurrent half of the backward pass:
 *   dU[k] = sum_t sum_b delta_t[b][row(k)] * h_{t-1}[b][col(k)]      for every stored nonzero k, in CSR order.
 * Runs on the FORWARD handle (vanilla cells, the LSTM and the GRU, where h fits in LDS whole: no column compaction) and
 * re-uses its mapping: every lane keeps one accumulator per nonzero it holds in the forward pass, in registers, for
 * all T steps.
 *   d_bprime  device, float32 [T][B][R]: delta_t from sprnn_backward (R = H), dp_t from sprnn_backward_lstm (R = 4H),
 *             d_recurrent from sprnn_backward_gru (R = 3H).
 *   h_fwd     device, float32 [T][B][H]: forward outputs h_1..h_T;  h0: device [B][H] or NULL (zeros).
 *   dU        device, float32 [nnz]: overwritten (T = 0 writes zeros).
 * Sums are binary32, in time order.  Only enqueues work; allocates nothing.
 */
int sprnn_weight_gradient(sprnn_handle_t h, int T, const float* d_bprime, const float* h_fwd, const float* h0, float* dU,
                          void* stream);

/*
 * Backward pass through time of the LSTM cell (Appendix B: four gate rows per hidden unit; B.1: the pruned weights
 * serve both passes), weights resident on chip.  For a loss with e_t = dL/dh_t from outside the layer, going from
 * t = T down to 1 with everything beyond T zero:
 *   dh_t = e_t + U^T dp_{t+1},     dc_t = dc_{t+1} f_{t+1} + dh_t o_t (1 - tanh(c_t)^2),
 *   dp_i = dc_t g_t i_t (1 - i_t),  dp_f = dc_t c_{t-1} f_t (1 - f_t),  dp_g = dc_t i_t (1 - g_t^2),
 *   dp_o = dh_t tanh(c_t) o_t (1 - o_t);        dL/db'_t = dp_t,  dL/dh_0 = U^T dp_1,  dL/dc_0 = dc_1 f_1.
 * The recurrent product runs over the 4H gate gradients, so the handle holds the TRANSPOSE of the forward matrix
 * (sprnn_transpose_csr with rows = 4H, cols = H; created with SPRNN_CELL_LSTM_BACKWARD and the forward pass's batch):
 * one row per hidden unit, whose lanes gather from the exchanged vector dp_{t+1} of length 4H; the lane that owns
 * (unit, sample) keeps dc in a register and publishes the unit's four gate gradients.
 *
 *   dh_ext    device, float32 [T][B][H]: e_t.
 *   gates     device, float32 [T][B][4H]: gate values kept by sprnn_forward_lstm_train.
 *   c_fwd     device, float32 [T][B][H]: cell states c_1..c_T of the forward pass;  c0: [B][H] or NULL (zeros).
 *   d_bprime  device, float32 [T][B][4H]: dp_t (the gradient of the recurrent weights follows from it and the
 *             forward outputs without a recurrence: sprnn_weight_gradient on the forward LSTM handle).
 *   dh0, dc0  device, float32 [B][H], or NULL if not wanted.
 * One launch; T is limited to 2^30 / (16 B H) timesteps per call.  Same stream, state and error rules as sprnn_forward.
 */
int sprnn_backward_lstm(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates, const float* c_fwd,
                        const float* c0, float* d_bprime, float* dh0, float* dc0, void* stream);

/*
 * sprnn_forward_gru that also keeps what the backward pass needs: gates_out, device float32 [T][B][4H], receives the
 * blocks r | z | n | q with q = U_n h_{t-1} + b_hn, the factor the reset gate multiplies.
 */
int sprnn_forward_gru_train(sprnn_handle_t h, int T, const float* x, const float* b_hn, const float* h0, float* h_out,
                            float* gates_out, void* stream);

/*
 * Backward pass through time of the GRU cell of sprnn_forward_gru, weights resident on chip.  With e_t = dL/dh_t from
 * outside the layer, going from t = T down to 1 with everything beyond T zero:
 *   dh_t = e_t + dh_{t+1} z_{t+1} + U^T v_{t+1},      da = dh_t (1 - z_t) (1 - n_t^2),
 *   dp_r = da q_t r_t (1 - r_t),   dp_z = dh_t (h_{t-1} - n_t) z_t (1 - z_t),   dq = da r_t,   v_t = (dp_r | dp_z | dq);
 *   dL/db'_t = (dp_r | dp_z | da),   dL/dh_0 = dh_1 z_1 + U^T v_1.
 * The handle holds the TRANSPOSE of the forward matrix (sprnn_transpose_csr with rows = 3H, cols = H; created with
 * SPRNN_CELL_GRU_BACKWARD and the forward pass's batch): one row per hidden unit, whose lanes gather from the exchanged
 * vector v_{t+1} of length 3H; the lane that owns (unit, sample) keeps dh_{t+1} z_{t+1} in a register and publishes
 * the unit's three elements.
 *
 *   dh_ext       device, float32 [T][B][H]: e_t.
 *   gates        device, float32 [T][B][4H]: r | z | n | q kept by sprnn_forward_gru_train.
 *   h_fwd        device, float32 [T][B][H]: forward outputs h_1..h_T;  h0: [B][H] or NULL (zeros).
 *   d_bprime     device, float32 [T][B][3H]: dL/db'_t.
 *   d_recurrent  device, float32 [T][B][3H], or NULL if not wanted: v_t, the gradient of the three recurrent sums.  It
 *                is what sprnn_weight_gradient on the forward GRU handle takes as d_bprime (dL/dU[r][k] = sum_t sum_b
 *                v_t[b][r] h_{t-1}[b][k]), and the sum of its third block over t and b is dL/db_hn.
 *   dh0          device, float32 [B][H], or NULL if not wanted.
 * One launch; T is limited to 2^30 / (16 B H) timesteps per call.  Same stream, state and error rules as sprnn_forward.
 */
int sprnn_backward_gru(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates, const float* h_fwd,
                       const float* h0, float* d_bprime, float* d_recurrent, float* dh0, void* stream);

/*
 * sprnn_backward_gru with the gradient of the recurrent weights fused in, as in sprnn_backward_with_weights: the column
 * of v_{t+1} that a lane gathers for a nonzero (j, r) of the transposed matrix is the factor that dL/dU[r][j] pairs with
 * the forward output h_t[.][j] of the lane's own row.
 *   dU_transposed  device, float32 [nnz]: dL/dU in the order of the TRANSPOSED matrix's CSR arrays (entry p belongs to
 *                  the forward nonzero t_source[p] of sprnn_transpose_csr); overwritten.
 * Other arguments as sprnn_backward_gru.  Always runs T + 1 steps.  Not available with column compaction or where the
 * mapping needs more threads than the instantiation is built for (SPRNN_ERR_UNSUPPORTED: use the two separate calls).
 */
int sprnn_backward_gru_with_weights(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates,
                                    const float* h_fwd, const float* h0, float* d_bprime, float* d_recurrent, float* dh0,
                                    float* dU_transposed, void* stream);

/*
 * sprnn_backward_lstm with the gradient of the recurrent weights fused in, as in sprnn_backward_with_weights: the
 * column of dp_{t+1} that a lane gathers for a nonzero (j, r) of the transposed matrix is the factor that dL/dU[r][j]
 * pairs with the forward output h_t[.][j] of the lane's own row.
 *   h_fwd          device, float32 [T][B][H]: forward outputs h_1..h_T;  h0: [B][H] or NULL (zeros).
 *   dU_transposed  device, float32 [nnz]: dL/dU in the order of the TRANSPOSED matrix's CSR arrays (entry p belongs to
 *                  the forward nonzero t_source[p] of sprnn_transpose_csr); overwritten.
 * Other arguments as sprnn_backward_lstm.  Always runs T + 1 steps.  Not available with column compaction or where
 * the mapping needs more threads than the instantiation is built for (SPRNN_ERR_UNSUPPORTED: use the two separate calls).
 */
int sprnn_backward_lstm_with_weights(sprnn_handle_t h_transposed, int T, const float* dh_ext, const float* gates,
                                     const float* c_fwd, const float* c0, const float* h_fwd, const float* h0, float* d_bprime,
                                     float* dh0, float* dc0, float* dU_transposed, void* stream);

/*
 * Host helper: transpose a CSR matrix (rows x cols) of binary16 values.  t_row_ptr has cols + 1 entries, t_col_idx
 * and t_val_fp16_bits have row_ptr[rows] entries; the columns inside a transposed row come out ascending.
 * t_source (row_ptr[rows] entries, or NULL) receives, for every entry of the transpose, the position of the same
 * nonzero in the input arrays.
 */
int sprnn_transpose_csr(int rows, int cols, const int32_t* row_ptr, const int32_t* col_idx, const uint16_t* val_fp16_bits,
                        int32_t* t_row_ptr, int32_t* t_col_idx, uint16_t* t_val_fp16_bits, int32_t* t_source);

/*
 * The step before the recurrence (Section 3.1: Eq. 1's input term is computed for all timesteps ahead of
 * time and enters Eq. 2 as b'):  b'[t][b][r] = sum_k W[r][k] x_in[t][b][k] + bias[r]  as one dense product on
 * the matrix cores.  Its output is laid out as the `x` argument of the forward calls of the same handle, so a
 * whole layer runs as sprnn_project followed by sprnn_forward / sprnn_forward_lstm on one stream.
 *
 *   input_size      I >= 1, length of one input vector.
 *   x_in            device, float32 [T][B][I], I fastest; every |x| below 65504 (it is split into two
 *                   binary16 numbers that together reproduce it to 2^-21).
 *   w_in_fp16_bits  device, [R][I] IEEE binary16 bit patterns, row r = weights of output r (R = H, or 4H with
 *                   gate blocks i|f|g|o for the LSTM cell).  Read, never written; the caller keeps ownership.
 *   bias            device, float32 [R], or NULL for zeros.
 *   b_prime         device, float32 [T][B][R]; must not overlap the inputs.
 *   stream          hipStream_t cast to void* (NULL = default stream).
 *
 * Products are exact and sums are binary32; the result is within
 *   (I + 8) * 2^-24 * (sum_k |W[r][k] x[k]| + |bias[r]|) + 2^-26 * sum_k |W[r][k]|
 * of the exact value (the second term is the floor for inputs below 2^-14, the smallest normal binary16
 * number).  Only enqueues work and returns; allocates nothing.  T = 0 is a no-op.
 */
int sprnn_project(sprnn_handle_t h, int T, int input_size, const float* x_in, const uint16_t* w_in_fp16_bits,
                  const float* bias, float* b_prime, void* stream);

/*
 * Non-persistent comparison path: one kernel launch per timestep that re-reads the CSR weights
 * from device memory every step (the per-timestep sparse product the paper compares against in
 * Section 5.2).  Same arguments and results as the persistent calls; c0 / c_out are ignored for
 * vanilla cells.  Not offered for the GRU cell (SPRNN_ERR_UNSUPPORTED).
 */
int sprnn_forward_stepwise(sprnn_handle_t h, int T, const float* x, const float* h0, const float* c0,
                           float* h_out, float* c_out, void* stream);

/*
 * Phase timing of the persistent kernel (only for handles created with options.timeline = 1).
 * Copies grid x 16 accumulators to `out` (host, capacity in 64-bit words, >= grid * 16) and clears them:
 * per workgroup, wall-clock ticks (see `*ticks_per_second`) spent by its first wavefront in
 * [0] operate, [1] reduce + epilogue arithmetic, [2] publish + outputs + next b' prefetch, [3] unused, [4] back-off,
 * [5] first poll, [6] re-polls and LDS writes, [7] waiting for the workgroup's other wavefronts;
 * [8] = number of re-polls, [9] = timesteps counted, [10] = ticks of 16 back-to-back clock reads
 * (the cost of the instrumentation itself, summed over launches), [11] / [12] = shader-clock ticks and
 * wall-clock ticks over whole launches (their ratio is the shader clock delivered), [13..15] unused.
 * Synchronises with the device.
 */
int sprnn_read_timeline(sprnn_handle_t h, uint64_t* out, int capacity_words, double* ticks_per_second);

/* Describe the mapping chosen at create time. */
int sprnn_get_info(sprnn_handle_t h, sprnn_info_t* info);

/*
 * Synchronise with the handle's device and report whether any forward on this handle tripped the
 * spin watchdog (SPRNN_ERR_STATE) since creation.
 */
int sprnn_check(sprnn_handle_t h);

/*
 * Host-only packing (no GPU needed): run the same validation and weight preparation as
 * sprnn_create and return the packed image for inspection.
 *   *words        malloc'ed uint32 [grid][template_words][block]: (LDS byte offset >> shift) << 16 | fp16 bits
 *   *lane_row     malloc'ed int32 [grid][block]: weight row served by each lane, -1 for an idle lane
 *   *lane_words   malloc'ed int32 [grid][block]: number of real (non-padding) words in that lane
 * info receives the mapping.  Free the three arrays with sprnn_free_host.
 */
int sprnn_pack_host(int hidden, int batch, int activation, const int32_t* row_ptr, const int32_t* col_idx,
                    const uint16_t* val_fp16_bits, const sprnn_options_t* opt, int num_cus,
                    uint32_t** words, int32_t** lane_row, int32_t** lane_words, sprnn_info_t* info);
void sprnn_free_host(void* p);

const char* sprnn_status_string(int code);

/* Release everything the handle owns.  NULL is a no-op. */
int sprnn_destroy(sprnn_handle_t h);

#ifdef __cplusplus
}
#endif
#endif /* SPRNN_H_ */
