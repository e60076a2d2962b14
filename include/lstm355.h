/*
 * liblstm355 -- stacked (optionally bidirectional) LSTM inference forward pass with
 * sparsity masks, for one AMD MI355X (gfx950).  Plain C ABI: opaque handle, plain
 * pointers and sizes.  Every pointer below is marked HOST or DEVICE.
 *
 * What is computed (paper: Yin et al., "Hardware-Guided Symbiotic Training for Compact,
 * Accurate, yet Execution-Efficient LSTM", Section 4, cell equations, with zero hidden
 * layers inside each gate, i.e. the conventional cell used as the paper's baseline in
 * Section 5):
 *
 *     [f; i; o; g] = [sigmoid; sigmoid; sigmoid; tanh]( W . [x_t, h_{t-1}] + b )
 *     c_t = f (x) c_{t-1} + i (x) g          h_t = o (x) tanh(c_t)
 *
 * W is passed as its two column blocks W_x (acts on x_t) and W_h (acts on h_{t-1}).
 * Each weight matrix may carry a binary mask of the same shape (Section 4, "mask-based
 * approach"; effective weight = W (x) Msk).  Layers are stacked (Section 5.1); with two
 * directions (Section 5.2) the second one walks the sequence backwards and the two hidden
 * sequences are concatenated on the feature axis, forward half first.
 *
 * Symbols: L layers, Dn in {1,2} directions, D_0 = input_dim, D_l = Dn*H for l > 0,
 * H hidden width, T timesteps, B batch.
 *
 * All functions return LSTM_OK (0) or a negative LSTM_ERR_* code; none throws or aborts.
 * lstm_last_error() returns a human-readable description of the most recent failure.
 * A handle may be used from one host thread and one stream at a time.
 */
#ifndef LSTM355_H
#define LSTM355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lstm355 lstm_t; /* opaque; owned by the library */

/* arithmetic type of the matrix products */
enum {
    LSTM_F32 = 0, /* fp32 operands, fp32 accumulation */
    LSTM_BF16 = 1 /* bf16 weights, inputs and recurrent operand h; fp32 accumulation, fp32 cell state, fp32 outputs */
};

enum {
    LSTM_OK = 0,
    LSTM_ERR_ARG = -1,    /* NULL where a pointer is required, non-positive size, bad enum, mask byte not in {0,1} */
    LSTM_ERR_SHAPE = -2,  /* layer / direction index outside the model */
    LSTM_ERR_STATE = -3,  /* forward before every (layer, direction) has weights */
    LSTM_ERR_NOMEM = -4,  /* device allocation failed, or caller's workspace too small */
    LSTM_ERR_LAUNCH = -5, /* a HIP call or kernel launch failed */
    LSTM_ERR_TIMEOUT = -6 /* a bounded device-side wait expired (reported by the next synchronising call) */
};

/* storage format of one (layer, direction)'s matrices on the device */
enum {
    LSTM_FMT_AUTO = 0,          /* library chooses from the mask density: row-compressed up to 25 % kept (H-LSTM: 50 %);
                                   within 5 % of that the second direction of a layer follows the first */
    LSTM_FMT_DENSE_MASKED = 1,  /* dense matrix with +0 stored where Msk = 0 */
    LSTM_FMT_ROW_COMPRESSED = 2 /* per row: the kept positions only, ascending column order */
};

/* execution plan of the recurrence (debug / measurement override; AUTO is the product path) */
enum {
    LSTM_PLAN_AUTO = 0,
    LSTM_PLAN_STEPWISE = 1,  /* one fused kernel launch per timestep */
    LSTM_PLAN_PERSISTENT = 2 /* one launch per layer; the time loop runs on the device */
};

/*
 * Create a model.  layers >= 1, input_dim >= 1, hidden_dim >= 1, bidirectional in {0,1},
 * dtype LSTM_F32 or LSTM_BF16.  *out receives the handle.  Uses the current HIP device.
 */
int lstm_create(int layers, int input_dim, int hidden_dim, int bidirectional, int dtype, lstm_t** out);

/*
 * Create a model whose cells are H-LSTM cells (paper Section 4: the same equation block with hidden layers inside
 * the control gates; Sections 5.1 and 5.2: one hidden layer per gate, as wide as the hidden state, in the models
 * the paper reports).  One hidden layer H per gate with ReLU activation:
 *
 *     u_q = relu( W1_q . [x_t, h_{t-1}] + b1_q )     q in {f, i, o, g}; width gate_hidden_dim = G
 *     [f; i; o; g] = [sigmoid; sigmoid; sigmoid; tanh]( W2_q . u_q + b2_q )
 *     c_t = f (x) c_{t-1} + i (x) g          h_t = o (x) tanh(c_t)
 *
 * Each gate has its own hidden layer.  gate_hidden_dim >= 1; dtype must be LSTM_F32 (LSTM_ERR_ARG otherwise).
 * Everything else as lstm_create; weights are set with lstm_set_weights_h, all other calls are shared.
 */
int lstm_create_h(int layers, int input_dim, int hidden_dim, int gate_hidden_dim, int bidirectional, int dtype,
                  lstm_t** out);

/*
 * Create a stack whose layers have their own widths (paper Section 4, row/column growth and pruning: the dimensions
 * of the weight matrices shrink and grow layer by layer; Section 5.1 step (b): 1500/400 -> 1197/317): layer l has
 * hidden width hidden_dims[l] and input width D_l = input_dim for l = 0, Dn * hidden_dims[l-1] otherwise.
 * gate_hidden_dims = NULL: conventional cells; otherwise H-LSTM cells with gate hidden width gate_hidden_dims[l] in
 * layer l (dtype LSTM_F32 only).  Both arrays HOST, `layers` entries, every entry >= 1.
 * Weights are set per (layer, direction) with lstm_set_weights / lstm_set_weights_h using that layer's widths.
 * y is [T, B, Dn * hidden_dims[layers-1]].  The states h0, c0, hT, cT are sequences of blocks: block n = l*Dn + d
 * holds [B, hidden_dims[l]] values and the blocks follow each other in the order of n (with one width for all layers
 * this is the [L*Dn, B, H] array of lstm_forward).  Two consecutive unidirectional layers run in one launch at
 * batch 1 only where their widths are equal.
 */
int lstm_create_layers(int layers, int input_dim, const int* hidden_dims, const int* gate_hidden_dims, int bidirectional,
                       int dtype, lstm_t** out);

/* Frees the handle and every device buffer it owns.  NULL is accepted. */
int lstm_destroy(lstm_t* m);

/* Text of the most recent error on this handle (or of the last failed lstm_create when m is NULL).
 * The string is owned by the library and valid until the next call on the handle. */
const char* lstm_last_error(const lstm_t* m);

/*
 * Set the weights of one (layer, direction).  All pointers HOST, row-major, fp32.
 *   Wx[4H, D_l], Wh[4H, H], b[4H]; gate rows in the paper's order f, i, o, g:
 *   rows [0,H) forget, [H,2H) input, [2H,3H) output, [3H,4H) cell candidate.
 *   mask_x, mask_h: uint8 in {0,1} with the shape of Wx / Wh, or NULL for "keep everything".
 * The mask is applied as a selection: where the mask byte is 0 the stored value is never read into
 * the arithmetic, so NaN or Inf there is harmless.  The compressed form keeps exactly the positions
 * with mask byte 1 (a kept zero value stays a stored entry), columns ascending within a row.
 * With dtype LSTM_BF16 the matrices are rounded to bf16 (nearest, ties to even); b stays fp32.
 * The library copies everything; the caller may free its arrays on return.  Synchronous.
 * Device memory held per (layer, direction): the input-side matrix is always kept dense (4H * D_l values; in fp32
 * models a second time in the operand order of the matrix instruction, for products with at most 64 input rows) and,
 * when row-compressed, in the compressed forms as well; the recurrent matrix in the one form its kernels read.
 */
int lstm_set_weights(lstm_t* m, int layer, int direction,
                     const float* Wx, const uint8_t* mask_x,
                     const float* Wh, const uint8_t* mask_h,
                     const float* b, int format);

/*
 * Weights of one (layer, direction) of an H-LSTM model (handle from lstm_create_h; LSTM_ERR_STATE on a handle from
 * lstm_create, and lstm_set_weights returns LSTM_ERR_STATE on an H-LSTM handle).  All pointers HOST, row-major, fp32.
 *   W1x[4G, D_l], W1h[4G, H], b1[4G]: the hidden layers, gate-major rows: row q*G + g is hidden unit g of gate q
 *   W2[4H, G], b2[4H]: the gate outputs, row q*H + j is output j of gate q and multiplies the hidden layer of gate q
 *   mask_1x, mask_1h, mask_2: uint8 in {0,1} of the matrix's shape, or NULL for "keep everything"
 * Masks select, formats and copying as in lstm_set_weights.
 */
int lstm_set_weights_h(lstm_t* m, int layer, int direction,
                       const float* W1x, const uint8_t* mask_1x,
                       const float* W1h, const uint8_t* mask_1h, const float* b1,
                       const float* W2, const uint8_t* mask_2, const float* b2, int format);

/* Bytes of DEVICE workspace lstm_forward needs for (T, B); 0 on bad arguments. */
size_t lstm_workspace_bytes(const lstm_t* m, int T, int B);

/*
 * Forward pass of the whole stack.  All data pointers DEVICE, owned by the caller.
 *   x   [T, B, D_0]     fp32 for LSTM_F32, bf16 (raw uint16 bit patterns) for LSTM_BF16
 *   h0, c0 [L*Dn, B, H] fp32, index l*Dn + d; NULL = zeros
 *   y   [T, B, Dn*H]    fp32, hidden sequence of the last layer; the backward direction's state is
 *                       stored at the input position it was computed for
 *   hT, cT [L*Dn, B, H] fp32, state after the last step each (layer, direction) processed
 *                       (t = T-1 forward, t = 0 backward); NULL = not wanted
 *   workspace           at least lstm_workspace_bytes(m, T, B) bytes, 256-byte aligned
 *   stream              hipStream_t passed as void*; NULL = the default stream
 * Asynchronous on `stream`: no host synchronisation and no allocation inside.  T = 0 or B = 0 is a
 * no-op that returns LSTM_OK.  Two forwards on the same handle must not overlap in time.  The persistent kernels
 * (batch 1, small-batch row-compressed, and large-batch bf16) occupy every compute unit for the duration of a layer: forwards issued
 * on other streams at the same time wait for them (cooperative launch) or, with ordinary launches, may make the
 * bounded waits expire (LSTM_ERR_TIMEOUT from lstm_check).
 * Graph capture: a forward may be issued on a stream that is being captured (hipStreamBeginCapture); the library
 * notices and records a form that can be replayed any number of times, between eager forwards or other graphs of the
 * same handle: exchange state is cleared by fill kernels inside the graph (no memset nodes), the step tags of the
 * exchange start from zero in every replay, persistent kernels are recorded as ordinary launches whatever the launch
 * mode (a graph holds no cooperative launches; the residency condition of lstm_set_launch_mode applies to a replay),
 * and profiling records nothing.  Run one eager forward of the same (T, B) on the handle before capturing it, so
 * that one-time kernel attributes are set outside the capture.  A replay uses the pointers of the capture.
 */
int lstm_forward(lstm_t* m, int T, int B, const void* x, const float* h0, const float* c0,
                 float* y, float* hT, float* cT, void* workspace, size_t workspace_bytes, void* stream);

/* After the stream has been synchronised: LSTM_OK, or LSTM_ERR_TIMEOUT if a device-side bounded wait
 * expired during an earlier forward on this handle (its outputs are then invalid).  Clears the flag; exchange
 * state that the abandoned steps may have left half-written is cleared before the next forward uses it. */
int lstm_check(lstm_t* m);

/* Override the recurrence plan (LSTM_PLAN_*) and, for measurement, the number of waves per workgroup of
 * the persistent kernels (0 = library default). */
int lstm_set_plan(lstm_t* m, int plan, int waves_per_group);

/*
 * How the persistent kernels are launched.  Their workgroups exchange the hidden state among themselves, so all of
 * them must be resident for any of them to make progress.
 * cooperative = 0 (default): an ordinary launch.  The grid never exceeds one workgroup per compute unit, so every
 * workgroup is resident as soon as the device has room for it; on a device that runs nothing else at that moment
 * that is at once.  If other kernels hold compute units, the workgroups that are already running poll until the
 * others have started; every wait is bounded (2^22 polls, a few seconds; LSTM355_SPIN_LIMIT in the environment at
 * lstm_create overrides the count), and if a bound expires the kernel drains and lstm_check reports LSTM_ERR_TIMEOUT
 * (the outputs of that forward are invalid); nothing hangs.  Callers that share the device with long-running kernels
 * should call lstm_check after synchronising, or choose the cooperative mode.
 * cooperative = 1: hipLaunchCooperativeKernel, with which the runtime guarantees the residency, at the price of a
 * slower dispatch (about 18 microseconds per launch measured on MI355X).
 *
 * Environment read at lstm_create: LSTM355_L2_HANDOVER=0 makes every exchange store device-scope (the hand-over of the
 * hidden state through the L2 of one XCD, used where a group of workgroups has been verified to share an XCD, is
 * switched off; results are bit-identical, only slower; for A/B checks).
 * LSTM355_SPARSE_PROJ_MAX_DENSITY=<fraction>: the input projection W_x . x_t + b of an fp32 model with row-compressed
 * W_x and at least 64 input rows (T * B) runs over the kept entries only when at most this fraction of W_x is kept
 * (default 0.18; 0 sends every such product to the dense matrix-core kernel; for A/B checks -- both compute the sum
 * of the paper's Section 4 over the mask-selected weights, in different summation orders).
 */
int lstm_set_launch_mode(lstm_t* m, int cooperative);
/* Process-wide default that lstm_create gives to new handles (including those lstm_latency_sweep creates). */
int lstm_set_default_launch_mode(int cooperative);

/*
 * Kernel timing for measurement.  With profiling enabled every forward brackets each of its kernels (or, for
 * the stepwise plan, each run of per-step launches) with a pair of events on the caller's stream; this
 * perturbs the stream slightly, so end-to-end latency is quoted with profiling off.
 * lstm_get_profile synchronises on the recorded events and returns, accumulated since the last call:
 * total microseconds and launch count of the input-projection kernels (proj) and of the recurrence kernels
 * (rec).  All pointers HOST, each may be NULL.  Clears the accumulated records.
 */
int lstm_set_profiling(lstm_t* m, int enable);
int lstm_get_profile(lstm_t* m, double* proj_us, int* proj_launches, double* rec_us, int* rec_launches);

/* Writes a short description of the plan the last forward used ("l0.d0:proj=...,rec=...;...", one entry per layer and
 * direction) into buf.  In a recurrence entry "(s, u, b)" are the kernel's slot count, units per wave and batch columns
 * per workgroup, and "batch/N" says that the layer's batch columns were run as N launches over runs of columns (a layer
 * whose time-loop kernel would need more workgroups than the device has compute units is cut that way, and/or into one
 * launch per direction, before the library falls back to one launch per timestep). */
int lstm_describe_plan(const lstm_t* m, char* buf, size_t buf_bytes);

/*
 * Read back the row-compressed structure of one matrix as the library stores it, translated to the
 * ABI row order (row r = q*H + j).  which: 0 = W_x, 1 = W_h; on an H-LSTM handle 0 = W1x, 1 = W1h (rows
 * r = q*G + g, 4G+1 row_ptr entries), 2 = W2.  All pointers HOST.
 * Call with row_ptr = col = val = NULL to obtain *nnz only.  row_ptr has 4H+1 entries.
 * LSTM_ERR_STATE if that matrix is not held in compressed form.
 */
int lstm_get_compressed(const lstm_t* m, int layer, int direction, int which,
                        int64_t* nnz, int64_t* row_ptr, int32_t* col, float* val);

/*
 * Latency profile over the gate dimension (paper Section 3: latency is globally increasing in the
 * dimension but locally non-monotonic; Section 4: the flow profiles latency on the target hardware to
 * pick hardware-favoured dimensions).  For each H in Hs: a 1-layer unidirectional model with
 * input_dim = H, dense seeded weights ~ U(-0.1, 0.1), forget-gate bias 1, x ~ N(0,1); `warmup` untimed
 * and `iters` timed forwards on `stream`, each bracketed by events.  Writes per point the median, 10th
 * and 90th percentile latency in microseconds and is_lhp (see lstm_find_lhp, eps = 0).
 * All pointers HOST.  Allocates and frees its own device buffers; synchronises the stream.
 */
int lstm_latency_sweep(const int* Hs, int nH, int T, int B, int dtype, uint64_t seed,
                       int warmup, int iters, double* med_us, double* p10_us, double* p90_us,
                       uint8_t* is_lhp, void* stream);

/*
 * The same profile for a whole model family (paper Section 3, the model-level latency figure: latency against the
 * model size set by the hidden-state width at batch 16; Section 5.1 step (c): the hysteresis points are located on
 * the target device before the row/column growth).  Point i is a stack of `layers` layers, `bidirectional` in {0,1},
 * hidden width Hs[i], input width Ds[i] (Ds = NULL: input width = hidden width); gate_hidden = 1 makes the cells
 * H-LSTM cells whose gate hidden layers are as wide as the hidden state (fp32 only), 0 conventional cells.
 * keep in (0,1): every matrix gets a seeded Bernoulli mask of that density and LSTM_FMT_AUTO; 0 or 1: dense.
 * Weights ~ U(-0.1, 0.1), forget-gate output bias 1, x ~ N(0,1).  Outputs and timing protocol as
 * lstm_latency_sweep.  All pointers HOST.
 */
int lstm_latency_sweep_model(const int* Hs, const int* Ds, int n, int layers, int bidirectional, int gate_hidden,
                             double keep, int T, int B, int dtype, uint64_t seed, int warmup, int iters,
                             double* med_us, double* p10_us, double* p90_us, uint8_t* is_lhp, void* stream);

/*
 * Latency hysteresis points of a measured curve (paper Section 3).  A dimension is a latency
 * hysteresis point iff it is faster, by the relative margin eps, than every larger dimension:
 * lat[i] < (1 - eps) * lat[j] for all j with dims[j] > dims[i]; the largest dimension always is one.
 * redundancy_pct = (1 - #LHP / n) * 100 (caption of the paper's model-level latency figure).
 * All pointers HOST; dims need not be sorted.  No GPU needed.
 */
int lstm_find_lhp(const int* dims, const double* lat, int n, double eps, uint8_t* is_lhp, double* redundancy_pct);

/*
 * Growth target of the hardware-guided step (paper Section 4, row/column grow-and-prune: growth recovers the model
 * to its hysteresis point; Section 5.1 step (c): a layer pruned to 1197 is grown back to the 1200 the device
 * favours).  Among the measured dimensions, *target_dim receives the smallest latency hysteresis point (margin eps,
 * as lstm_find_lhp) that is >= from_dim; *latency_gain_pct (may be NULL) the latency reduction in percent against
 * the smallest measured dimension >= from_dim (from_dim itself when it was measured; 0 when that is the target).
 * LSTM_ERR_ARG when from_dim exceeds every measured dimension.  All pointers HOST.  No GPU needed.
 */
int lstm_grow_to_lhp(const int* dims, const double* lat, int n, double eps, int from_dim, int* target_dim,
                     double* latency_gain_pct);

/*
 * Mask updates of the pruning phases, on DEVICE arrays (paper Section 4).
 *
 * lstm_prune_weights: one iteration of magnitude-based weight pruning ("Msk(w) = 0 iff |w| <= the (100 p_w)-th
 * percentile of |W|").  W fp32 [count], mask uint8 [count] in {0,1}, updated in place; W is not changed.  The
 * percentile is taken over the connections that are still active (mask 1): with k = ceil(p_w * active), every active
 * entry whose magnitude is at or below the k-th smallest active magnitude is switched off (ties go together; k = 0
 * prunes nothing).  What lies under a zero mask byte is never looked at.  *kept_before / *kept_after (HOST, may be
 * NULL) receive the number of active entries before and after.  count < 2^32 - 1.
 *
 * lstm_prune_rows_cols: one iteration of the paper's row/column pruning algorithm on one matrix W [M, N] (row-major)
 * with its mask.  Importance of a row / column = sum of the magnitudes of its active entries.  Thresholds: the
 * ceil(p_r * M)-th smallest row sum and the ceil(p_c * N)-th smallest column sum, both of the matrix as passed in.
 * Rows at or below the row threshold are removed first (mask bytes and weights set to zero), then the columns whose
 * sum over the matrix as the row pass left it is at or below the column threshold.  A ratio of 0 removes nothing
 * along that axis.  (Because the column threshold is the one of the matrix as passed in, a call that removes many rows
 * lowers every column sum against it: on a matrix without structure, removing a fifth of the rows and asking for a fifth
 * of the columns in the same call removes all columns.  Use one call per axis for independent ratios.)
 * Every sum is accumulated in fp64 in index order (from +0, adding the entries of the row / column one after the
 * other), and sums are compared as fp64: the result does not depend on the launch shape.  *rows_removed / *cols_removed (HOST, may be NULL) receive how many
 * rows / columns this call zeroed.
 *
 * Both allocate and free their own scratch and synchronise the stream.  The packed form of a model is not touched:
 * pass the new masks to lstm_set_weights / lstm_set_weights_h to run the pruned model.
 */
int lstm_prune_weights(const float* W, uint8_t* mask, size_t count, double p_w, size_t* kept_before, size_t* kept_after,
                       void* stream);
int lstm_prune_rows_cols(float* W, uint8_t* mask, int M, int N, double p_r, double p_c, int* rows_removed,
                         int* cols_removed, void* stream);

/*
 * lstm_prune_rows_cols for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid it): the same iteration with the same kernels and the same result, bit for bit, but the
 * scratch (row and column sums, the two thresholds, two counters) lives in a fixed device array inside the library,
 * about 256 KiB, which every GPU the library runs on holds until the process ends.  Nothing is allocated or freed, and
 * the call does not synchronise: it is asynchronous on `stream`.
 *   W, mask, M, N, p_r, p_c as lstm_prune_rows_cols (DEVICE arrays, updated in place).
 *   M <= 16384 and N <= 16384, else LSTM_ERR_ARG (the scratch is fixed); M * N is not limited otherwise.
 *   removed: DEVICE int[2] or NULL; receives the number of rows and of columns this call zeroed, on the stream.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two host threads)
 * race and give undefined masks; calls on one stream, or ordered by events, are fine, and a call does not depend on
 * what an earlier one left in the array.  The first call on a device looks up that device's array (no allocation, but
 * make it outside a graph capture).
 */
int lstm_prune_rows_cols_static(float* W, uint8_t* mask, int M, int N, double p_r, double p_c, int* removed, void* stream);

/*
 * Dimension compaction after row/column pruning (paper Section 4, "Row/column growth & pruning": the pruning shrinks
 * the dimensions of the weight matrices; Section 5.1 step (b): each control-gate matrix goes from 1500/400 to
 * 1197/317, Section 5.2 step (b): from 800/800 to 626/626).  All array pointers DEVICE, owned by the caller.
 *
 *   W [gates*R, N] fp32 row-major, mask uint8 in {0,1} of the same shape (not NULL): `gates` blocks of R rows, row
 *   q*R + r is unit r of gate q (gates = 4 for a packed LSTM matrix, 1 for a plain matrix).
 *   A unit is kept iff at least one of its `gates` rows has an active connection (mask byte 1), a column iff at least
 *   one row has an active connection in it (the paper removes a neuron once all of its connections are pruned).
 *   row_index [R], col_index [N] int32: the kept units / columns, ascending, in the first *Rc / *Nc entries; the rest
 *   is set to -1.
 *   Wc: capacity gates*R*N floats; receives the compacted matrix [gates * *Rc, *Nc] row-major in its first elements
 *   (same block layout): the weight where the mask byte is 1, +0 where it is 0 - what lies under a zero mask byte is
 *   never read into the result.  mask_c: same capacity in bytes, receives the compacted mask; may be NULL.
 *   *Rc, *Nc HOST.  Either may come back 0 (nothing is written to Wc then).
 *
 * A dropped unit or column had no active connection, so every product with the kept part is unchanged and a second
 * call on the result keeps everything.  Whether a unit may also leave a *model* is the caller's to decide from the
 * matrices that consume it: a hidden unit of an LSTM layer can go without changing any kept output when its column in
 * the layer's own recurrent matrix and in the next layer's input matrices is dropped too; its bias entries and its
 * rows of every matrix of the layer then go with it (row_index names them).
 * The outputs must not overlap the inputs.  Allocates and frees its own scratch and synchronises the stream.
 * LSTM_ERR_ARG: NULL where required, a non-positive size, or gates*R*N > 2^31.
 */
int lstm_compact_rows_cols(const float* W, const uint8_t* mask, int gates, int R, int N, int32_t* row_index,
                           int32_t* col_index, float* Wc, uint8_t* mask_c, int* Rc, int* Nc, void* stream);

/* Measurement helpers (used by the benchmark to quote achievable peaks next to spec-sheet ones).
 * copy: device-to-device streaming copy of `bytes` bytes (a multiple of 16), `iters` times after one warm-up; 16-byte
 * loads, four in flight per thread, eight workgroups per compute unit, non-temporal stores.  *avg_us (HOST): average
 * microseconds per copy; bandwidth = 2 * bytes / time.  DEVICE pointers dst, src. */
int lstm_bench_copy(void* dst, const void* src, size_t bytes, int iters, double* avg_us, void* stream);

/*
 * Stand-alone product Y[batch, n] = X[batch, n] . (W (x) Msk)[n, n]^T with a dense input batch and a square weight
 * matrix (paper Section 3, the two matrix-multiplication latency figures: latency against the dimension for dense and
 * sparse operands).  format LSTM_FMT_DENSE_MASKED runs the library's dense projection (+0 stored where Msk = 0),
 * LSTM_FMT_ROW_COMPRESSED its row-compressed one (for batch <= 64 and n <= 5120 the kernel that splits a row's kept
 * entries over the lanes; otherwise the transpose of X plus the kernel that puts the input rows on the lanes).
 * Operands, all HOST, row-major:
 *   X_host [batch, n], W_host [n, n] fp32, mask_host [n, n] uint8 in {0,1} or NULL for "keep everything"; the mask
 *   selects (what lies under a zero byte is never read into the product); `keep` and `seed` are then ignored.
 *   X_host = W_host = mask_host = NULL: W ~ U(-0.1, 0.1), mask Bernoulli(keep), keep in (0, 1], X ~ N(0,1), all from
 *   `seed` with one fixed generator, so both formats see the same operands.
 * n a multiple of 4.  *avg_us: average over `iters` launches after 3 warm-up launches.  y_host (HOST, [batch, n],
 * may be NULL) receives the product.  Allocates and frees its own device buffers; synchronises the stream.
 */
int lstm_bench_matmul(int n, int batch, double keep, int format, uint64_t seed, int iters, const float* X_host,
                      const float* W_host, const uint8_t* mask_host, double* avg_us, float* y_host, void* stream);
/*
 * Matrix-instruction issue loop: every wave of two four-wave workgroups per compute unit issues `reps` rounds of eight
 * independent matrix instructions (dtype LSTM_BF16: 32x32x16 bf16, LSTM_F32: 32x32x2 fp32) on operands and
 * accumulators it holds in registers, so nothing but the matrix pipes, and the power they draw, limits it: the
 * achievable peak that the projection kernels' rates are quoted against, next to the spec-sheet one.
 * random_operands = 0: one constant operand pair (the highest clock the device holds under matrix load);
 * random_operands = 1: twelve operand fragments of random sign and mantissa, rotated every round, as a product of
 * real data presents them; the device then settles at a lower clock, and that rate is the ceiling of a product on
 * real data.  *tflops (HOST): 10^12 operations per second over `iters` launches after one warm-up; *clock_ghz (HOST,
 * may be NULL): the shader clock during the loop (cycle counter against the 100 MHz counter).  Allocates small
 * buffers; synchronises the stream.
 */
int lstm_bench_mfma(int dtype, int random_operands, int reps, int iters, double* tflops, double* clock_ghz, void* stream);
/*
 * Device-wide barrier with no data: `workgroups` (<= compute units, <= 256) workgroups of `waves` waves; in each of
 * `steps` rounds every workgroup raises one tagged 8-byte slot and waits until it has seen the slots of all of them
 * (the protocol of the recurrence kernels' exchange, carrying nothing).  The yardstick "same grid, T barriers, no
 * work" for the step time of the persistent kernels.  The poll of a round is tried unpaced and behind a short wait
 * (6, 10, 12, 16 times 64 clocks after the workgroup's own store, which lets the first polling round find the other
 * workgroups' stores visible); *avg_us_per_step (HOST) is the fastest of those.  Allocates its own buffers and
 * synchronises the stream; LSTM_ERR_TIMEOUT if a bounded wait expired.
 */
int lstm_bench_barrier(int workgroups, int waves, int steps, int iters, int cooperative, double* avg_us_per_step, void* stream);
/* exchange: `steps` rounds of the hidden-state exchange with no arithmetic, for `hidden` units (one tagged slot each,
 * all of them polled by every workgroup) and workgroups of `waves` waves (0: the library's choice); returns the
 * average microseconds per round for the fastest pacing of the poll (as lstm_bench_barrier). */
int lstm_bench_exchange(int hidden, int waves, int steps, int iters, int cooperative, double* avg_us_per_step, void* stream);
/*
 * The exchange inside groups of workgroups, with no arithmetic (yardstick of the kernels whose workgroups exchange only
 * inside one (direction, batch group), and the measurement behind the hand-over through one XCD's L2): `groups` groups
 * of `members` (<= 64) workgroups, each group passing `slots` (<= 16384) tagged 8-byte slots round among its members for
 * `steps` rounds; groups * members must not exceed the number of compute units.
 *   placed = 0: block ids in order, so a group's members are dealt over all XCDs; device-scope stores.
 *   placed = 1: a group's members take block ids of one residue modulo 8 (LSTM_ERR_ARG when an XCD's share of the groups
 *   does not fit its compute units); each group checks from the hardware's XCD ids that it shares an XCD, and only then,
 *   and only if workgroup_stores = 1, publishes with workgroup-scope stores.
 * *avg_us_per_round (HOST): average microseconds per round; *groups_verified (HOST, may be NULL): groups whose check
 * succeeded in the warm-up launch (0 when placed = 0).  Allocates its own buffers and synchronises the stream.
 */
int lstm_bench_group_exchange(int slots, int members, int groups, int placed, int workgroup_stores, int steps, int iters,
                              int cooperative, double* avg_us_per_round, int* groups_verified, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LSTM355_H */
