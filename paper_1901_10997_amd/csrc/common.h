// Internal declarations shared by the host code and the kernel launchers of liblstm355.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>
#include <string>
#include <vector>

namespace l355 {

// One weight matrix (W_x or W_h) of one (layer, direction), as held on the device.
// Row order is "packed": packed row 4*j + q holds gate q (0=f,1=i,2=o,3=g) of hidden unit j, so the
// four pre-activations a cell update needs are adjacent.
struct PackedMat {
    int rows = 0, cols = 0;
    bool compressed = false;
    void* dense = nullptr;       // [rows][cols], fp32 or bf16 bits; +0 where the mask is 0
    float* dense_frag16 = nullptr;  // fp32 input-side matrices: `dense` once more in the fragment order of the 16x16x4
                                    // matrix instruction (launch_proj_mfma), for products with at most 64 input rows
    int64_t nnz = 0;             // compressed: kept positions (== popcount of the mask)
    int32_t* row_ptr = nullptr;  // device [rows+1]
    uint16_t* col16 = nullptr;   // device [nnz]  (cols <= 65536)
    float* val = nullptr;        // device [nnz], fp32 (bf16-representable values in bf16 models)
    int max_row_nnz = 0;
    // register-resident slices for the persistent batch-1 kernel: [rows][slots][64] entries
    int slots = 0;               // ceil(max_row_nnz / 64)
    float* ell_val = nullptr;    // device [rows*slots*64]
    uint16_t* ell_col = nullptr; // device [rows*slots*64]
    // The same slices cut to fewer slots for the batch-1 kernel, when only a few rows are longer than the rest: rows
    // keep their first 64*slots_trim entries in the slices, the remainder of a unit's four rows (at most 64 entries
    // per unit) goes to a per-unit overflow list: entry = (gate << 16) | column.  slots_trim == 0: not built.
    int slots_trim = 0;
    float* ell_val_trim = nullptr;
    uint16_t* ell_col_trim = nullptr;
    int32_t* ovf_ptr = nullptr;   // device [rows/4 + 1]
    uint32_t* ovf_ent = nullptr;  // device [overflow entries]
    float* ovf_val = nullptr;
    std::vector<int32_t> h_ovf_ptr;   // host copy of ovf_ptr
    // Quarter-wave form for the small-batch kernel (recurrent matrices whose rows keep at most 256 entries): the four
    // gate rows of unit j share 64-lane slots, gate q on lanes 16q..16q+15, so that a slot is one gather for all four
    // gates and a row's partial sums stay inside a 16-lane row.  [rows/4][q16_slots][64]; q16_slots == 0: not built.
    int q16_slots = 0;            // even; 16 q16_slots entries of every row are in the slots
    float* q16_val = nullptr;
    uint16_t* q16_col = nullptr;
    // the few entries of rows longer than that (at most 6 in any eight consecutive units), per unit: entry = (gate << 16) | column; or nullptr
    int32_t* q16_ovf_ptr = nullptr;   // device [rows/4 + 1]
    uint32_t* q16_ovf_ent = nullptr;
    float* q16_ovf_val = nullptr;
    // host copy of the compressed structure in packed row order (for read-back)
    std::vector<int64_t> h_row_ptr;
    std::vector<int32_t> h_col;
    std::vector<float> h_val;
};

struct LayerDir {
    bool set = false;
    PackedMat wx, wh;
    float* bias = nullptr;  // device [4H], packed row order, fp32
    // H-LSTM cell: wx, wh and bias are the hidden layers of the four gates (W1x [4G][D], W1h [4G][H], b1 [4G],
    // packed row 4g+q = hidden unit g of gate q); w2 [4H][G] and bias2 [4H] are the gate outputs (packed row 4j+q)
    PackedMat w2;
    float* bias2 = nullptr;
    // batch-1 persistent kernel: the hidden-layer activations travel as 32-bit words stamped with the parity of the
    // step count of the array they live in, so every cell has arrays of its own: [0, 4G) for eager calls (u_epoch counts
    // their steps), [4G, 8G) for calls captured into a graph (cleared inside the graph, counted from zero)
    unsigned* u_slots = nullptr;
    unsigned u_epoch = 0;
    bool u_dirty = false;   // a wait expired while the array was in use: clear it before the next launch
};

// Number of compute units of the current device (cached; 256 if the query fails).  The persistent kernels need
// every workgroup resident at once, i.e. at most one per compute unit.
int device_num_cus();

// ---- kernel launchers (all asynchronous on `s`; return hipError_t of the launch) ----

// P[m][n] = bias[n] + sum_k X[m][k] * W[n][k];  X fp32 or bf16 (x_bf16), W fp32 or bf16 (w_bf16).
hipError_t launch_proj_dense(const void* X, bool x_bf16, int ldx, const void* W, bool w_bf16, const float* bias,
                             float* P, int M, int N, int K, hipStream_t s);
// Same product on the matrix cores (needs proj_mfma_supported); fp32 X with bf16 W is rounded to bf16 on load.
bool proj_mfma_supported(bool w_bf16, int K, int ldx);
// W_frag16 (fp32 models, may be null): the same W in the fragment order of the 16x16x4 matrix instruction
// ([ceil(N/16)][ceil(K/16)][64 lanes][4], lane l: row 16 nb + l % 16, k = 16 kb + 4 (l / 16) .. + 3, zero padded),
// used when X has at most 64 rows.
hipError_t launch_proj_mfma(const void* X, bool x_bf16, int ldx, const void* W, bool w_bf16, const float* bias, float* P,
                            int M, int N, int K, hipStream_t s, const float* W_frag16 = nullptr);
hipError_t launch_proj_mfma_f32_pair(const float* X, int ldx, const float* W0, const float* bias0, float* P0,
                                     const float* W1, const float* bias1, float* P1, int M, int N, int K, hipStream_t s);
// XT[k][m] = (float) X[m][k]   (optionally rounding fp32 -> bf16 -> fp32 on the way)
hipError_t launch_transpose_to_f32(const void* X, bool x_bf16, int ldx, float* XT, int M, int K, bool round_bf16,
                                   hipStream_t s);
// P[m][r] = bias[r] + sum_{i in row r} val[i] * XT[col[i]][m]
hipError_t launch_proj_csr(const float* XT, const int32_t* row_ptr, const uint16_t* col, const float* val,
                           const float* bias, float* P, int M, int rows, hipStream_t s);

// Row-compressed projection for M <= 64 input rows from the 64-lane slices (no transpose of X needed).
bool proj_ell_small_supported(int M, int rows, int K, int slots);
hipError_t launch_proj_ell_small(const void* X, bool x_bf16, int ldx, bool round_x_bf16, const float* ell_val,
                                 const uint16_t* ell_col, int slots, const float* bias, float* P, int M, int rows, int K,
                                 hipStream_t s);

struct StepArgs {
    const float* P;        // [T*B][4H] pre-activations from the input projection (bias included)
    const float* h_prev;   // h_{t-1}: element (b,k) at h_prev[b*h_prev_ld + k]; nullptr = zeros
    int h_prev_ld;
    float* c;              // [B][H] cell state, updated in place
    float* y_t;            // h_t goes to y_t[b*y_ld + j]
    int y_ld;
    float* hT;             // optional [B][H]: written when last != 0
    float* cT;
    int last;
    int t;                 // time index into P
    int B, H;
    int round_h_bf16;      // bf16 models: the recurrent operand h is rounded to bf16 when read
};
hipError_t launch_step_dense(const StepArgs& a, const void* Wh, bool w_bf16, hipStream_t s);
hipError_t launch_step_csr(const StepArgs& a, const int32_t* row_ptr, const uint16_t* col, const float* val,
                           hipStream_t s);

// H-LSTM, one timestep in two launches (any shape): hidden layers of the gates, then gate outputs + cell update.
struct HStage1Args {
    const float* P1;        // [T*B][4G] hidden-layer pre-activations from the input projection (b1 included)
    const float* h_prev;    // (b,k) at h_prev[b*h_prev_ld + k]; nullptr = zeros
    int h_prev_ld;
    const float* w_dense;   // W1h [4G][H] fp32 packed rows, or nullptr when row-compressed
    const int32_t* row_ptr; // row-compressed W1h
    const uint16_t* col;
    const float* val;
    float* u;               // [B][4G], packed: u[b][4g+q]
    int t, B, H, G;
};
struct HStage2Args {
    const float* u;         // [B][4G]
    const float* w_dense;   // W2 [4H][G] fp32 packed rows, or nullptr when row-compressed
    const int32_t* row_ptr;
    const uint16_t* col;
    const float* val;
    const float* bias2;     // [4H] packed
    float* c;               // [B][H] in place
    float* y_t;             // h_t -> y_t[b*y_ld + j]
    int y_ld;
    float* hT;
    float* cT;
    int last, B, H, G;
};
// Row-compressed H-LSTM step for small batches: both stages, one or both directions of a layer per launch pair.
// The hidden activations travel between the stages gate-major: u[b][q*G + g].
struct HStepDir {
    const float* P1;         // [T*B][4G] packed rows
    const float* h_prev;     // (b,k) at h_prev[b*h_prev_ld + k]; nullptr = zeros
    int h_prev_ld;
    float* u;                // [B][4G] gate-major scratch of this direction
    const float* ell_val_1h; // W1h [4G][slots_1h][64]
    const uint16_t* ell_col_1h;
    const float* ell_val_2;  // W2 [4H][slots_2][64]
    const uint16_t* ell_col_2;
    int slots_1h, slots_2;
    const float* bias2;      // [4H] packed
    float* c;                // [B][H]
    float* y_t;              // h_t -> y_t[b*y_ld + j]
    int y_ld;
    float* hT;
    float* cT;
    int t;
};
struct HStepPairArgs {
    HStepDir d[2];
    int B, H, G, last;
};
bool hstep_pair_supported(int H, int G, int slots_1h, int slots_2);
hipError_t launch_hstep_pair(const HStepPairArgs& p, int ndir, hipStream_t s);
hipError_t launch_hstage1(const HStage1Args& a, hipStream_t s);
hipError_t launch_hstage2(const HStage2Args& a, hipStream_t s);

// H-LSTM at batch 1, all three matrices row-compressed and register-resident, time loop on the device.
struct PersistHArgs {
    const float* ell_val_1x;    // W1x [4G][slots_1x][64]
    const uint16_t* ell_col_1x;
    const float* ell_val_1h;    // W1h [4G][slots_1h][64]
    const uint16_t* ell_col_1h;
    const float* ell_val_2;     // W2 [4H][slots_2][64], columns = hidden units of the row's own gate
    const uint16_t* ell_col_2;
    int slots_1x, slots_1h, slots_2;
    const float* bias1;         // [4G] packed
    const float* bias2;         // [4H] packed
    const float* x;             // input sequence [T][x_ld], fp32
    int x_ld, D;
    const float* h0;            // [H] or nullptr
    const float* c0;
    float* y;                   // h_t -> y[t*y_ld + j]
    int y_ld;
    float* hT;
    float* cT;
    int T, H, G, reverse;
    unsigned long long* xchg_h; // [H] tagged slots
    unsigned* xchg_u;           // [4G] 32-bit words, gate-major: u >= 0, so the sign bit carries the step's parity
    unsigned u_epoch;           // steps this array has seen before the launch: step s stamps (u_epoch + s + 1) & 1
    unsigned tag_base;          // step s publishes tag_base + s + 1 in xchg_h
    int* timeout_flag;
    unsigned spin_limit;
    int poll_pace_u;            // pace_poll units between the publication of the hidden activations and their poll
};
bool persist_b1_hlstm_supported(int H, int G, int D, int slots_1x, int slots_1h, int slots_2);
hipError_t launch_persist_b1_hlstm(const PersistHArgs& a, int cooperative, hipStream_t s);

// bf16 step on the matrix cores (large batch, dense W_h): recurrent product + fused cell update.
struct StepMfmaArgs {
    const float* P;            // [T*B][4H]
    const uint16_t* Wh;        // [4H][H] bf16, packed rows
    const uint16_t* hb_prev;   // h_{t-1} in bf16, (b,k) at hb_prev[b*hb_prev_ld + k]; nullptr = zeros
    int hb_prev_ld;
    float* c;                  // [B][H] fp32, in place
    float* y_t;                // h_t fp32 -> y_t[b*y_ld + j]
    int y_ld;
    uint16_t* hb_t;            // h_t bf16 -> hb_t[b*hb_ld + j]
    int hb_ld;
    float* hT;
    float* cT;
    int last, t, B, H;
};
bool step_mfma_supported(int B, int H);
hipError_t launch_step_mfma_bf16(const StepMfmaArgs& a, hipStream_t s);
hipError_t launch_f32_to_bf16(const float* src, int src_ld, uint16_t* dst, int dst_ld, int rows, int cols, hipStream_t s);

// bf16 dense recurrence at large batch with the time loop on the device (one launch per layer and direction).
struct PersistMfmaArgs {
    const float* P;            // [T*B][4H]
    const uint16_t* Wh;        // [4H][H] bf16, packed rows
    const float* c0;           // [B][H] or nullptr
    float* y;                  // h_t fp32 -> y[(t*B + b)*y_ld + j], or nullptr
    int y_ld;
    uint16_t* yb;              // h_t bf16 -> yb[(t*B + b)*yb_ld + j], or nullptr
    int yb_ld;
    float* hT;
    float* cT;
    uint16_t* hx;              // two exchange buffers of H * Bp bf16 each, Bp = B rounded up to 64
    unsigned* flags;           // one per tile, [row blocks][tiles of a row block]; every value below tag_base + 1
    unsigned long long* xcc_ids;  // [row blocks][64] tagged slots for the XCD ids of the tiles' workgroups, or nullptr
    int xcd_local;             // block ids grouped by XCD (set by the launcher)
    int device_scope_only;     // 1: publish with device-scope stores even where the group shares an XCD (A/B switch)
    unsigned tag_base;         // step s publishes tag_base + s + 1
    int* timeout_flag;
    unsigned spin_limit;
    int has_h0;                // exchange buffer 0 holds h0 (set by the launcher)
    int T, B, H, reverse;
};
bool persist_mfma_supported(int B, int H);
// fp32 dense recurrence at small and medium batch with the time loop on the device (all directions of a layer per launch)
struct PersistDenseDir {
    const float* P;            // [T*B][4H]
    const float* Wh;           // [4H][H] fp32, packed rows
    const float* c0;           // [B][H] or nullptr
    float* y;                  // h_t -> y[(t*B + b)*y_ld + j]
    int y_ld;
    float* hT;
    float* cT;
    int reverse;
    int has_h0;                // exchange buffer 0 holds h0 (set by the launcher)
};
struct PersistDenseArgs {
    PersistDenseDir d[2];
    float* hx;                 // per direction two exchange buffers of ceil(H/16) * Bp * 16 words (Bp: B rounded up to the
                               // row blocks), all zero at launch
    int* timeout_flag;
    unsigned spin_limit;
    int T, B, H, ndir;
    int Bld;                   // rows per timestep in P and y (>= B: the launch may cover a run of the batch's columns)
    int gm, gn;                // row blocks, workgroups per row block (set by the launcher)
    int poll_pace;             // pace_poll units in front of a step's first read of h (exchange.h)
    unsigned long long* xcc_ids;  // [ndir * row blocks][64] tagged slots for the XCD ids of a group's workgroups (zero or
                               // older tags only), or nullptr: no hand-over through one XCD's L2
    unsigned tag_base;         // the XCD ids of this launch carry tag_base + 1
    int xcd_local;             // block ids grouped by XCD (set by the launcher)
    int device_scope_only;     // 1: publish with device-scope stores even where a group shares an XCD (A/B switch)
};
size_t persist_dense_f32_ids_count();   // 8-byte slots behind xcc_ids
bool persist_dense_f32_supported(int B, int H, int ndir);
size_t persist_dense_f32_exchange_floats(int B, int H, int ndir);
// h0[d]: fp32 [B][H] of direction d or nullptr
hipError_t launch_persist_dense_f32(PersistDenseArgs& a, const float* const* h0, bool cooperative, hipStream_t s);
size_t persist_mfma_exchange_bytes(int B, int H);
size_t persist_mfma_flag_count(int B, int H);   // 32-bit words of flag storage, XCD id slots included
size_t persist_mfma_ids_offset(int B, int H);   // word offset of the XCD id slots inside it
hipError_t launch_persist_mfma_bf16(const PersistMfmaArgs& a, const float* h0, bool cooperative, hipStream_t s);

// Row-compressed step for small batches: one or both directions of a layer per launch (H <= 2048).
bool step_csr_pair_supported(int H, int slots);
hipError_t launch_step_csr_pair(const StepArgs* a, const float* const* ell_val, const uint16_t* const* ell_col,
                                const int* slots, int ndir, hipStream_t s);

struct PersistB1Args {
    // recurrent weights, dense packed rows [4H][H], fp32 or bf16 bits
    const void* Wh;
    int w_bf16;
    // input side: either P (projection done by a separate kernel, bias included) or, fused,
    // Wx [4H][D] + bias [4H] + the input sequence x [T][D]
    const float* P;        // [T][4H] or nullptr
    const void* Wx;        // nullptr = not fused
    const float* bias;
    const void* x;
    int x_bf16;            // x holds bf16 bits
    int round_x_bf16;      // x is fp32 but the operand is rounded to bf16 (bf16 model, layer > 0)
    int D;
    const float* h0;       // [H] or nullptr
    const float* c0;       // [H] or nullptr
    float* y;              // h_t -> y[t*y_ld + j]
    int y_ld;
    float* hT;             // [H] or nullptr
    float* cT;
    int T, H;
    int reverse;           // 1: walk t = T-1 .. 0
    int round_h_bf16;
    unsigned long long* xchg;  // [2][H] (value, tag) slots, library-owned
    unsigned long long* xcc_ids;  // [64] tagged slots for the XCD ids of the workgroups, library-owned
    int one_xcd;               // every workgroup on one XCD: only block ids = 0 mod 8 work (filled by the launcher)
    int device_scope_only;     // 1: publish with device-scope stores even on one XCD (A/B switch)
    unsigned tag_base;         // tags tag_base+1 .. tag_base+T are used by this launch
    int* timeout_flag;         // set to 1 if a bounded wait expired
    unsigned spin_limit;
};
hipError_t launch_persist_b1_dense(const PersistB1Args& a, int waves_per_group, int cooperative, hipStream_t s);
bool persist_b1_dense_supported(int H);
bool persist_b1_dense_fusable(int H, int D);

// Row-compressed batch-1 recurrence, one or two stacked layers per launch (unidirectional when two).
struct SparseLayerArgs {
    const float* ell_val_x;     // [4H][slots_x][64]
    const uint16_t* ell_col_x;
    const float* ell_val_h;     // [4H][slots_h][64]
    const uint16_t* ell_col_h;
    int slots_x, slots_h;
    // per-unit overflow lists of rows longer than 64*slots entries (nullptr: none); entry = (gate << 16) | column
    const int32_t* ovf_ptr_x;
    const uint32_t* ovf_ent_x;
    const float* ovf_val_x;
    const int32_t* ovf_ptr_h;
    const uint32_t* ovf_ent_h;
    const float* ovf_val_h;
    const float* bias;          // [4H] packed order
    const float* h0;            // [H] or nullptr
    const float* c0;
    float* y;                   // h_t -> y[t*y_ld + j]; nullptr = hidden sequence of this layer not wanted
    int y_ld;
    float* hT;
    float* cT;
};
struct SparseStackArgs {
    SparseLayerArgs layer[2];
    const void* x;              // input sequence of the first layer, [T][D0]
    int x_bf16, round_x_bf16;
    int D0;
    int T, H;
    int reverse;                // only with one layer
    int round_h_bf16;
    unsigned long long* xchg;   // [layers][2][H]
    unsigned tag_base;
    int* timeout_flag;
    unsigned spin_limit;
};
hipError_t launch_persist_b1_sparse(const SparseStackArgs& a, int layers, int waves_per_group, int cooperative, hipStream_t s);
bool persist_b1_sparse_supported(int H, int D0, int slots_x, int slots_h, int layers);

// Small-batch row-compressed recurrence with the time loop on the device (all directions of a layer per launch).
struct PersistBatchedDir {
    const float* P;            // [T*B][4H] projection incl. bias
    // W_h in the quarter-wave form [H][q16_slots][64]
    const float* q16_val;
    const uint16_t* q16_col;
    int q16_slots;
    const int32_t* q16_ovf_ptr;   // per-unit lists of the entries beyond 16 q16_slots of a row, or nullptr
    const uint32_t* q16_ovf_ent;  // (gate << 16) | column
    const float* q16_ovf_val;
    const float* h0;           // [B][H] or nullptr
    const float* c0;
    float* y;                  // h_t -> y[(t*B + b)*y_ld + j]  (already offset to this direction's columns)
    int y_ld;
    float* hT;                 // [B][H] or nullptr
    float* cT;
    int reverse;
};
struct PersistBatchedArgs {
    PersistBatchedDir d[2];
    int T, B, H;
    int Bld;                   // rows per timestep in P and y (>= B: the launch may cover a run of the batch's columns)
    int ug, bg;                // unit groups / batch groups per direction (filled by the launcher)
    int ndir, xcd_local;       // directions in the grid; block ids grouped by XCD (filled by the launcher)
    int device_scope_only;     // 1: publish with device-scope stores even where a group shares an XCD (A/B switch)
    int round_h_bf16;
    unsigned long long* xchg;  // slots, zero or older tags only: 2 (B + 3) H per direction, [2][batch group][H][columns of a group]
    unsigned long long* xcc_ids;  // [ndir * bg][64] tagged slots (XCD id of each unit group's workgroup), zero or older tags only
    unsigned tag_base;
    int* timeout_flag;
    unsigned spin_limit;
    int poll_pace;             // pace_poll units in front of the poll of h where the exchange is device-wide (set by the launcher)
};
// Input projection with W_x in the quarter-wave form, for many input rows (fp32): P[m][4H] = b + W_x . X[m]
struct ProjQ16Dir {
    const float* val;            // [H][slots][64]
    const uint16_t* col;
    int slots;
    const int32_t* ovf_ptr;      // entries outside the slots, per unit; or nullptr
    const uint32_t* ovf_ent;     // (gate << 16) | column
    const float* ovf_val;
    const float* bias;           // [4H] packed rows
    float* P;                    // [M][4H]
};
struct ProjQ16Args {
    ProjQ16Dir d[2];
    const float* X;              // [M][ldx], K columns used
    int ldx, M, K, H;
};
bool proj_q16_supported(int M, int H, int K, int slots);
hipError_t launch_proj_q16(const ProjQ16Args& a, int ndir, int slots, hipStream_t s);

// `slots` = the largest q16_slots of the directions (even, <= 16)
bool persist_batched_q16_plan(int B, int H, int slots, int ndir, int* upw, int* bw, int* ug, int* bg);
hipError_t launch_persist_batched_q16(PersistBatchedArgs& a, int ndir, int slots, int cooperative, hipStream_t s);

// H-LSTM at small batch (B >= 2), W1h and W2 row-compressed and register-resident, time loop on the device, every
// direction of a layer in one launch.
struct PersistBatchedHDir {
    const float* P1;            // [T*B][4G] packed rows (4g + q): b1 + W1x . x_t
    // W1h [G][slots_1h][64] and W2 [H][slots_2][64] in the quarter-wave form; W2's columns carry their gate's offset
    // q * G into the hidden-layer vector
    const float* q16_val_1h;
    const uint16_t* q16_col_1h;
    const float* q16_val_2;
    const uint16_t* q16_col_2;
    int slots_1h, slots_2;
    // per-unit lists of the few entries outside the slots (nullptr: none); entry = (gate << 16) | column (W2: the
    // column inside its gate's block); at most 6 in any eight consecutive units
    const int32_t* ovf_ptr_1h;
    const uint32_t* ovf_ent_1h;
    const float* ovf_val_1h;
    const int32_t* ovf_ptr_2;
    const uint32_t* ovf_ent_2;
    const float* ovf_val_2;
    const float* bias2;         // [4H] packed
    const float* h0;            // [B][H] or nullptr
    const float* c0;
    float* y;                   // h_t(b, j) -> y[(t*B + b)*y_ld + j]
    int y_ld;
    float* hT;                  // [B][H] or nullptr
    float* cT;
    int reverse;
};
struct PersistBatchedHArgs {
    PersistBatchedHDir d[2];
    int T, B, H, G;
    int Bld;                    // rows per timestep in P1 and y (>= B: the launch may cover a run of the batch's columns)
    int ug, bg;                 // unit groups / batch groups per direction (filled by the launcher)
    int ndir, xcd_local;        // directions in the grid; block ids grouped by XCD (filled by the launcher)
    int device_scope_only;      // 1: publish with device-scope stores even where a group shares an XCD (A/B switch)
    size_t h_stride, u_stride;  // elements per (direction, batch group) in xchg_h / xchg_u (filled by the launcher)
    unsigned long long* xchg_h; // tagged slots, zero or older tags only
    float* xchg_u;              // plain values
    unsigned* flags;            // [ndir * bg][64], zero or older tags only
    unsigned long long* xcc_ids; // [ndir * bg][64] tagged slots (XCD id of each unit group's workgroup), zero or older tags only
    unsigned tag_base;
    int* timeout_flag;
    unsigned spin_limit;
};
// `slots` = the largest slot count of the two matrices over the directions (even, <= 16)
bool persist_batched_h_plan(int B, int H, int G, int slots, int ndir, int* upw, int* bw, int* ug, int* bg);
hipError_t launch_persist_batched_h(PersistBatchedHArgs& a, int ndir, int slots, int cooperative, hipStream_t s);

// Pruning mask updates (device arrays; scratch supplied by the caller of the launcher).
size_t prune_state_bytes();
hipError_t launch_prune_weights(const float* W, uint8_t* mask, size_t count, double p_w, unsigned* keys, void* state,
                                unsigned long long* counters, hipStream_t s);
size_t prune_rows_cols_scratch_bytes(int M, int N);
hipError_t launch_prune_rows_cols(float* W, uint8_t* mask, int M, int N, unsigned k_rows, unsigned k_cols, void* scratch,
                                  int** removed_out, hipStream_t s);
int prune_rows_cols_static_max_lines();
hipError_t launch_prune_rows_cols_static(float* W, uint8_t* mask, int M, int N, unsigned k_rows, unsigned k_cols,
                                         int* removed_dev, hipStream_t s);
size_t compact_scratch_bytes(int gates, int R, int N);
hipError_t launch_compact_rows_cols(const float* W, const uint8_t* mask, int gates, int R, int N, int* row_index,
                                    int* col_index, float* Wc, uint8_t* mask_c, void* scratch, int** counts_out, hipStream_t s);
hipError_t launch_fill_u64(unsigned long long* p, size_t n, unsigned long long v, hipStream_t s);
// yardsticks
hipError_t launch_copy_stream(void* dst, const void* src, size_t bytes, hipStream_t s);
int mfma_issue_blocks();
hipError_t launch_mfma_issue(bool bf16, bool random, float* sink, long long* clocks, int reps, double* flops, hipStream_t s);
size_t mfma_issue_sink_floats();
hipError_t launch_barrier_only(unsigned long long* slots, unsigned tag_base, int groups, int waves, int steps,
                               int* timeout_flag, unsigned spin_limit, int poll_pace, int cooperative, hipStream_t s);
hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_exchange_only(unsigned long long* xchg, unsigned tag_base, int H, int waves, int steps,
                                int* timeout_flag, unsigned spin_limit, int poll_pace, int cooperative, hipStream_t s);
hipError_t launch_group_exchange(unsigned long long* slots, unsigned long long* ids, unsigned tag_base, int n, int members,
                                 int groups, int placed, int workgroup_stores, int steps, int* timeout_flag,
                                 unsigned spin_limit, int* verified, int cooperative, hipStream_t s);

}  // namespace l355
