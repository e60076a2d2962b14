// Host side of liblstm355: handle, weight packing, workspace carve-up, launch sequencing, latency sweep.
// The C ABI is declared and documented in include/lstm355.h.
#include "../../include/lstm355.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <string>
#include <vector>

#include "common.h"

using namespace l355;

struct lstm355 {
    int L = 0, D0 = 0, H = 0, Dn = 1, dtype = LSTM_F32;
    int G = 0;                 // > 0: H-LSTM cell, width of the hidden layer inside each gate
    int device = 0;
    std::vector<LayerDir> ld;  // index l*Dn + d
    mutable std::string err;
    unsigned long long* xchg = nullptr;  // [2][2][H] tagged exchange slots of the persistent batch-1 kernels
    unsigned tag_base = 0;               // tags <= tag_base have been used
    int* timeout_flag = nullptr;         // device int
    unsigned spin_limit = 1u << 22;
    int device_scope_only = 0;           // 1: no hand-over through an XCD's L2 (environment LSTM355_L2_HANDOVER=0)
    int poll_pace = -1;                  // pace_poll units where a kernel paces a poll; -1: each kernel's measured default (environment LSTM355_POLL_PACE)
    double sparse_proj_max_density = 0.18;   // projection over the kept entries up to this kept fraction (environment LSTM355_SPARSE_PROJ_MAX_DENSITY)
    int plan = LSTM_PLAN_AUTO;
    int waves_per_group = 0;
    int cooperative = 0;
    // set for the duration of a forward whose stream is being captured into a graph
    bool capturing = false;
    bool cap_cleared = false;            // the batch-1 exchange slots have been cleared inside this capture
    unsigned cap_tag = 0;                // tags <= cap_tag have been used inside this capture
    int launch_mode() const { return capturing ? 0 : cooperative; }   // a captured launch is an ordinary one
    std::string last_plan;
    bool profiling = false;
    struct Span { hipEvent_t e0, e1; int kind; };
    std::vector<Span> spans;             // recorded, not yet read
    std::vector<hipEvent_t> event_pool;  // idle events
    // widths per layer (H and G above hold the largest of them: sizes of shared buffers)
    std::vector<int> Hs, Gs;
    std::vector<size_t> state_off;       // state_off[l*Dn + d]: hidden units in front of that cell in h0/c0/hT/cT
    size_t xchg_slots = 0;               // 64-bit slots in xchg
    int hid(int l) const { return Hs[(size_t)l]; }
    int ghid(int l) const { return Gs[(size_t)l]; }
    int in_dim(int l) const { return l == 0 ? D0 : Dn * Hs[(size_t)l - 1]; }
    size_t soff(size_t n) const { return state_off[n]; }
};

static thread_local std::string g_create_error;
static int g_default_cooperative = 0;   // ordinary launches (see lstm_set_launch_mode in the header)

static int fail(const lstm_t* m, int code, const std::string& msg)
{
    if (m) m->err = msg; else g_create_error = msg;
    return code;
}
static int fail_hip(const lstm_t* m, hipError_t e, const char* what)
{
    return fail(m, e == hipErrorOutOfMemory ? LSTM_ERR_NOMEM : LSTM_ERR_LAUNCH,
                std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(m, call)                                   \
    do {                                                   \
        hipError_t e__ = (call);                           \
        if (e__ != hipSuccess) return fail_hip(m, e__, #call); \
    } while (0)

// RAII bracket: records an event pair around the launches issued during its lifetime (profiling only).
struct ProfSpan {
    lstm_t* m; hipStream_t s; int idx = -1;
    ProfSpan(lstm_t* m_, hipStream_t s_, int kind) : m(m_), s(s_)
    {
        if (!m->profiling || m->capturing) return;   // event pairs of a captured forward could not be read back
        hipEvent_t ev[2];
        for (auto& e : ev) {
            if (!m->event_pool.empty()) { e = m->event_pool.back(); m->event_pool.pop_back(); }
            else if (hipEventCreate(&e) != hipSuccess) return;
        }
        m->spans.push_back({ev[0], ev[1], kind});
        idx = (int)m->spans.size() - 1;
        (void)hipEventRecord(ev[0], s);
    }
    ~ProfSpan() { if (idx >= 0) (void)hipEventRecord(m->spans[idx].e1, s); }
};

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

static uint16_t host_f32_to_bf16(float f)
{
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x0040u);  // NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static float host_bf16_to_f32(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// How the recurrence of a layer is cut when its persistent kernel cannot take it in one launch (more workgroups than
// compute units): `passes` launches over the directions (1: all directions in one grid, 2: one launch each) times `chunks`
// runs of batch columns of nearly equal length (batch columns are independent).  The cut with the fewest launches that
// `fits(columns, directions)` accepts for its longest and shortest run wins; at most eight launches per layer.
// slots of the quarter-wave form the small-batch recurrences take (rows of up to 16 x 24 = 384 kept entries)
constexpr int kMaxRecurrentSlots = 24;
struct LaunchCut { int passes = 0, chunks = 0; };
template <class Fits>
static bool choose_cut(int B, int Dn, Fits fits, LaunchCut* out)
{
    for (int total = 1; total <= 8; ++total)
        for (int passes = 1; passes <= Dn; ++passes) {
            if (total % passes) continue;
            const int chunks = total / passes, nd = Dn / passes;
            const int lo = B / chunks, hi = (B + chunks - 1) / chunks;
            if (lo < 2) continue;
            if (fits(hi, nd) && (lo == hi || fits(lo, nd))) {
                out->passes = passes;
                out->chunks = chunks;
                return true;
            }
        }
    return false;
}
static inline int chunk_begin(int B, int chunks, int c) { return (int)((long long)c * B / chunks); }

// pace_poll units (64 clocks each) in front of a device-wide poll that follows the wave's own publication at once (exchange.h).
// Measured optima, both broad: batch-1 H-LSTM, poll of the hidden activations: 135.4 us per sequence unpaced, 121.6 at 8,
// 120.1 at 10, 121.0 at 12, 124.0 at 16; small-batch recurrence with a device-wide exchange (two 1500-wide layers, batch
// 20): 144.7 us per layer unpaced, 141.0 at 8, 143.4 at 12.  Every other persistent kernel was measured too and is left
// unpaced: a delay in front of its poll lengthens the step from the first unit on (its own work after the publication,
// or an exchange inside one XCD, already puts the first poll round where it succeeds).
constexpr int kPollPaceHlstmB1 = 10;
constexpr int kPollPaceBatchedDeviceWide = 8;
// dense fp32 recurrence at small and medium batch, first read of h in a step (its own stores just in front of it): layers of
// 256 to 1024 units at batch 4 to 64 are fastest between 16 and 24 (H = 800, both directions, batch 16: 1665 us per layer
// unpaced, 1567 at 16, 1453 at 24, 1503 at 32; H = 256, batch 16: 2.48 us per step unpaced, 2.31 at 16, 2.54 at 24)
constexpr int kPollPaceDenseNarrow = 16, kPollPaceDenseWide = 24;
// the yardsticks try these and report the fastest
static const int kYardstickPaces[] = {0, 6, 10, 12, 16};

static void free_mat(PackedMat& p)
{
    if (p.dense) (void)hipFree(p.dense);
    if (p.dense_frag16) (void)hipFree(p.dense_frag16);
    if (p.row_ptr) (void)hipFree(p.row_ptr);
    if (p.col16) (void)hipFree(p.col16);
    if (p.val) (void)hipFree(p.val);
    if (p.ell_val) (void)hipFree(p.ell_val);
    if (p.ell_col) (void)hipFree(p.ell_col);
    if (p.ell_val_trim) (void)hipFree(p.ell_val_trim);
    if (p.ell_col_trim) (void)hipFree(p.ell_col_trim);
    if (p.ovf_ptr) (void)hipFree(p.ovf_ptr);
    if (p.ovf_ent) (void)hipFree(p.ovf_ent);
    if (p.ovf_val) (void)hipFree(p.ovf_val);
    if (p.q16_val) (void)hipFree(p.q16_val);
    if (p.q16_col) (void)hipFree(p.q16_col);
    if (p.q16_ovf_ptr) (void)hipFree(p.q16_ovf_ptr);
    if (p.q16_ovf_ent) (void)hipFree(p.q16_ovf_ent);
    if (p.q16_ovf_val) (void)hipFree(p.q16_ovf_val);
    p = PackedMat();
}

template <typename T>
static hipError_t upload(T** dst, const std::vector<T>& src)
{
    *dst = nullptr;
    const size_t bytes = std::max<size_t>(src.size(), 1) * sizeof(T);
    hipError_t e = hipMalloc((void**)dst, bytes);
    if (e != hipSuccess) return e;
    if (!src.empty()) e = hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
    return e;
}

// Quarter-wave form for the small-batch kernel: slot s of unit j is one 64-lane gather that serves all four gate
// rows, gate q on lanes 16q..16q+15.  An 8-byte gather serves lanes 0..31 (gates 0, 1) and 32..63 (gates 2, 3) in
// separate passes whose 32 columns must differ modulo 32.  Within a pass bank b (= column mod 32) belongs to lane
// b mod 16 of one of the two rows: in slot s row q owns the banks of half (s + q) mod 2.  An entry goes to a
// position that owns its bank (S/2 slots per row and bank).  What does not fit there is placed in a free lane of a
// slot in which the OTHER row of the pass owns the entry's bank but has nothing to put there: that position's
// filler (value 0) is pointed at the entry's own column, the two lanes read one address, and nothing collides.  Among
// the free lanes one whose bits 2 and 3 differ in parity from the owner's is preferred, which keeps the 16-byte
// gather (four passes of 16 lanes, picked by lane bit 5 and the parity of bits 2..4) free of collisions as well.
// Only an entry for which no such slot exists takes any free position, from the end.
// force_slots > 0: that many slots (the other direction of the layer uses them: one launch serves both, and the
// kernel is built for the larger count) instead of the smallest count the rule below allows.  max_slots: the most the
// consuming kernel takes (24); nothing is built for longer rows.
// gather16: the consumer gathers 16 bytes per entry only (the projection: four input rows per tile).  Such a gather makes
// four passes of 16 lanes -- lane bit 5 and the parity of bits 2..4 pick the pass, so a pass holds eight lanes of each
// of two rows, with complementary parities of bits 2, 3 -- whose columns must differ modulo 16.  An entry then goes to
// lane (column mod 16) of its row in any slot (S places per row and lane instead of S/2 per row and bank), and one that
// does not fit goes to a free lane of the other parity class in a slot where the other row has nothing at lane
// (column mod 16), whose filler is pointed at the entry's column.
// gate_col_stride > 0 (the H-LSTM's gate-output matrix): row q of a unit reads block q of a vector of four blocks of
// that many elements; the stored column, and the bank it is placed by, is gate_col_stride * q + column.
// soft_slots > 0: the consumer loses its best configuration above that many slots (the H-LSTM kernel keeps two matrices
// in registers); a matrix that would need more is cut to soft_slots anyway as long as no eight consecutive units
// leave more than 48 entries outside (the kernels take at most 64 per wave).
static int build_quarter_wave(lstm_t* m, PackedMat& out, int force_slots, int max_slots, bool gather16 = false,
                              int gate_col_stride = 0, int soft_slots = 0)
{
    if (out.q16_val) (void)hipFree(out.q16_val);
    if (out.q16_col) (void)hipFree(out.q16_col);
    if (out.q16_ovf_ptr) (void)hipFree(out.q16_ovf_ptr);
    if (out.q16_ovf_ent) (void)hipFree(out.q16_ovf_ent);
    if (out.q16_ovf_val) (void)hipFree(out.q16_ovf_val);
    out.q16_val = nullptr; out.q16_col = nullptr; out.q16_ovf_ptr = nullptr; out.q16_ovf_ent = nullptr; out.q16_ovf_val = nullptr;
    out.q16_slots = 0;
    const int rows = out.rows, cols = out.cols, max_nnz = out.max_row_nnz;
    if (!out.compressed || max_slots < 2 || rows < 4 || cols + 3 * gate_col_stride > 16383) return LSTM_OK;
    {
        const int units = rows / 4;
        // The slot count is set by the longest row, and with random masks a handful of rows are a few entries longer
        // than all others.  Take the smallest (even) count that leaves at most 6 entries outside the slots in any eight
        // consecutive units (a wave owns at most eight): the owning wave adds those one at a time, which costs it about
        // as much per entry as a tenth of a slot, and the step waits for the slowest wave.
        int S = std::max(2, 2 * ((max_nnz + 31) / 32));
        if (force_slots > 0) S = std::max(2, std::min(S, force_slots + (force_slots & 1)));
        else {
            std::vector<int> per_unit((size_t)units);
            for (int St = 2; St < S; St += 2) {
                for (int u = 0; u < units; ++u) {
                    int64_t n = 0;
                    for (int q = 0; q < 4; ++q)
                        n += std::max<int64_t>(0, out.h_row_ptr[4 * u + q + 1] - out.h_row_ptr[4 * u + q] - (int64_t)16 * St);
                    per_unit[(size_t)u] = (int)std::min<int64_t>(n, 1 << 20);
                }
                int64_t window = 0, worst = 0;
                for (int u = 0; u < units; ++u) {
                    window += per_unit[(size_t)u];
                    if (u >= 8) window -= per_unit[(size_t)u - 8];
                    worst = std::max(worst, window);
                }
                if (worst <= 6 || (soft_slots > 0 && St >= soft_slots && worst <= 48)) { S = St; break; }
            }
        }
        if (S > max_slots) return LSTM_OK;   // rows too long for the kernels that use this form
        std::vector<float> qv((size_t)units * S * 64, 0.0f);
        std::vector<uint16_t> qc((size_t)units * S * 64, 0);
        std::vector<char> used((size_t)S * 64), aliased((size_t)S * 64);
        std::vector<int64_t> leftover[4];
        auto par23 = [](int j) { return ((j >> 2) ^ (j >> 3)) & 1; };
        for (int u = 0; u < units; ++u) {
            std::fill(used.begin(), used.end(), 0);
            std::fill(aliased.begin(), aliased.end(), 0);
            float* uv = qv.data() + (size_t)u * S * 64;
            uint16_t* uc = qc.data() + (size_t)u * S * 64;
            for (int sl = 0; sl < S; ++sl)
                for (int ln = 0; ln < 64; ++ln) {
                    const int c = (ln & 15) + (gather16 ? 0 : 16 * ((sl + (ln >> 4)) & 1));   // a column of the bank this position owns
                    uc[sl * 64 + ln] = (uint16_t)(c < cols ? c : 0);
                }
            for (int q = 0; q < 4; ++q) {
                const int rp = 4 * u + q;
                int fill[32] = {0};
                leftover[q].clear();
                const int64_t row_end = std::min<int64_t>(out.h_row_ptr[rp + 1], out.h_row_ptr[rp] + (int64_t)16 * S);
                for (int64_t e = out.h_row_ptr[rp]; e < row_end; ++e) {
                    const int ec = out.h_col[e] + q * gate_col_stride;   // the column as the kernel addresses it
                    const int bank = gather16 ? (ec & 15) : (ec & 31), j = bank & 15, hb = bank >> 4;
                    if (fill[bank] < (gather16 ? S : S / 2)) {
                        const int sl = gather16 ? fill[bank] : 2 * fill[bank] + ((hb + q) & 1);
                        ++fill[bank];
                        const int pos = sl * 64 + 16 * q + j;
                        used[pos] = 1;
                        uv[pos] = out.h_val[e];
                        uc[pos] = (uint16_t)ec;
                    } else {
                        leftover[q].push_back(e);
                    }
                }
            }
            for (int q = 0; q < 4; ++q) {
                for (int64_t e : leftover[q]) {
                    const int ec = out.h_col[e] + q * gate_col_stride;
                    const int bank = gather16 ? (ec & 15) : (ec & 31), j = bank & 15, hb = bank >> 4;
                    int best = -1, best_owner = -1;
                    // slots where the other row owns `bank` (every slot for 16-byte gathers, where only a lane of the other
                    // parity class shares a pass with the other row's lane j)
                    for (int sl = gather16 ? 0 : ((hb + (q ^ 1)) & 1); sl < S && best < 0; sl += gather16 ? 1 : 2) {
                        const int owner = sl * 64 + 16 * (q ^ 1) + j;
                        if (used[owner] || aliased[owner]) continue;
                        int any = -1;
                        for (int jj = 0; jj < 16; ++jj) {
                            const int pos = sl * 64 + 16 * q + jj;
                            if (used[pos] || aliased[pos]) continue;
                            if (par23(jj) != par23(j)) { best = pos; break; }
                            if (any < 0 && !gather16) any = pos;
                        }
                        if (best < 0) best = any;
                        if (best >= 0) best_owner = owner;
                    }
                    if (best >= 0) {
                        aliased[best_owner] = 1;
                        uc[best_owner] = (uint16_t)ec;
                    } else {
                        // no such slot: any free position of the row, from the end; a filler that serves the other row's
                        // entry is given up only when nothing else is left (the row holds at most 16 S entries)
                        for (int pass = 0; pass < 2 && best < 0; ++pass)
                            for (int t = S * 16 - 1; t >= 0 && best < 0; --t) {
                                const int pos = (t / 16) * 64 + 16 * q + (t & 15);
                                if (!used[pos] && (pass == 1 || !aliased[pos])) best = pos;
                            }
                        aliased[best] = 0;
                    }
                    used[best] = 1;
                    uv[best] = out.h_val[e];
                    uc[best] = (uint16_t)ec;
                }
            }
        }
        out.q16_slots = S;
        HIP_TRY(m, upload(&out.q16_val, qv));
        HIP_TRY(m, upload(&out.q16_col, qc));
        std::vector<int32_t> optr((size_t)units + 1, 0);
        std::vector<uint32_t> oe;
        std::vector<float> ov;
        for (int u = 0; u < units; ++u) {
            for (int q = 0; q < 4; ++q) {
                const int rp = 4 * u + q;
                for (int64_t e = out.h_row_ptr[rp] + (int64_t)16 * S; e < out.h_row_ptr[rp + 1]; ++e) {
                    oe.push_back(((uint32_t)q << 16) | (uint32_t)out.h_col[e]);
                    ov.push_back(out.h_val[e]);
                }
            }
            optr[(size_t)u + 1] = (int32_t)oe.size();
        }
        if (!oe.empty()) {
            HIP_TRY(m, upload(&out.q16_ovf_ptr, optr));
            HIP_TRY(m, upload(&out.q16_ovf_ent, oe));
            HIP_TRY(m, upload(&out.q16_ovf_val, ov));
        }
    }
    return LSTM_OK;
}

// A row-major fp32 matrix W[rows][cols] in the fragment order of the 16x16x4 matrix instruction: tile (nb, kb) is 64 lanes
// x 4 values, lane l holding W[16 nb + l % 16][16 kb + 4 (l / 16) .. + 3]; zero beyond the matrix (launch_proj_mfma).
static std::vector<float> to_frag16(const float* W, int rows, int cols)
{
    const int NB = (rows + 15) / 16, KB = (cols + 15) / 16;
    std::vector<float> out((size_t)NB * KB * 256, 0.0f);
    for (int nb = 0; nb < NB; ++nb)
        for (int kb = 0; kb < KB; ++kb) {
            float* tile = out.data() + ((size_t)nb * KB + kb) * 256;
            for (int l = 0; l < 64; ++l) {
                const int n = 16 * nb + (l & 15), k0 = 16 * kb + 4 * (l >> 4);
                if (n >= rows) continue;
                for (int c = 0; c < 4 && k0 + c < cols; ++c) tile[4 * l + c] = W[(size_t)n * cols + k0 + c];
            }
        }
    return out;
}

// Pack one matrix W[4H][cols] (ABI row order q*H + j) with its optional mask into device storage.
static int pack_matrix(lstm_t* m, PackedMat& out, const float* W, const uint8_t* mask, int H, int cols, bool compressed,
                       bool bf16, bool keep_dense, int quarter_slots = 0, int gate_col_stride = 0, int soft_slots = 0,
                       bool frag16 = false, bool q16_gather16 = false)
{
    free_mat(out);
    const int rows = 4 * H;
    out.rows = rows;
    out.cols = cols;
    out.compressed = compressed;
    auto abi_row = [H](int rp) { return (rp & 3) * H + (rp >> 2); };
    if (!compressed || keep_dense) {
        const size_t n = (size_t)rows * cols;
        if (bf16) {
            std::vector<uint16_t> buf(n);
            for (int rp = 0; rp < rows; ++rp) {
                const size_t src = (size_t)abi_row(rp) * cols, dst = (size_t)rp * cols;
                for (int k = 0; k < cols; ++k)
                    buf[dst + k] = (mask == nullptr || mask[src + k]) ? host_f32_to_bf16(W[src + k]) : (uint16_t)0;
            }
            uint16_t* d = nullptr;
            HIP_TRY(m, upload(&d, buf));
            out.dense = d;
        } else {
            std::vector<float> buf(n);
            for (int rp = 0; rp < rows; ++rp) {
                const size_t src = (size_t)abi_row(rp) * cols, dst = (size_t)rp * cols;
                for (int k = 0; k < cols; ++k) buf[dst + k] = (mask == nullptr || mask[src + k]) ? W[src + k] : 0.0f;
            }
            float* d = nullptr;
            HIP_TRY(m, upload(&d, buf));
            out.dense = d;
            if (frag16 && cols % 4 == 0) HIP_TRY(m, upload(&out.dense_frag16, to_frag16(buf.data(), rows, cols)));
        }
        if (!compressed) return LSTM_OK;
    }
    // row-compressed: structure = the mask (every position when there is no mask), columns ascending
    out.h_row_ptr.assign(rows + 1, 0);
    out.h_col.clear();
    out.h_val.clear();
    int max_nnz = 0;
    for (int rp = 0; rp < rows; ++rp) {
        const size_t src = (size_t)abi_row(rp) * cols;
        int cnt = 0;
        for (int k = 0; k < cols; ++k) {
            if (mask == nullptr || mask[src + k]) {
                float v = W[src + k];
                if (bf16) v = host_bf16_to_f32(host_f32_to_bf16(v));
                out.h_col.push_back(k);
                out.h_val.push_back(v);
                ++cnt;
            }
        }
        out.h_row_ptr[rp + 1] = (int64_t)out.h_col.size();
        max_nnz = std::max(max_nnz, cnt);
    }
    out.nnz = (int64_t)out.h_col.size();
    out.max_row_nnz = max_nnz;
    std::vector<int32_t> rp32(rows + 1);
    for (int i = 0; i <= rows; ++i) rp32[i] = (int32_t)out.h_row_ptr[i];
    std::vector<uint16_t> c16(out.h_col.size());
    for (size_t i = 0; i < c16.size(); ++i) c16[i] = (uint16_t)out.h_col[i];
    HIP_TRY(m, upload(&out.row_ptr, rp32));
    HIP_TRY(m, upload(&out.col16, c16));
    HIP_TRY(m, upload(&out.val, out.h_val));
    // 64-lane slices for the register-resident kernels.  The kernels gather h[col] from LDS (4 bytes per column at
    // batch 1, 8 or 16 bytes with two or four batch columns adjacent).  Measured on gfx950: a 4- or 8-byte read serves
    // lanes 0..31 and 32..63 in separate passes, and within a pass two lanes collide when their columns are congruent
    // modulo 32; a 16-byte read makes four passes of 16 lanes whose columns must differ modulo 16.  An entry with
    // column c is therefore placed, where room allows, in a lane congruent to c modulo 32, which is conflict-free for
    // all three widths.  (The order of the entries inside a row is free: it only fixes the order of a sum.)
    out.slots = std::max(1, (max_nnz + 63) / 64);
    // slices of S slots holding the first min(nnz, 64 S) entries of every row
    auto build_slices = [&](int S, std::vector<float>& ev, std::vector<uint16_t>& ec) {
        ev.assign((size_t)rows * S * 64, 0.0f);
        ec.assign((size_t)rows * S * 64, 0);
        // empty positions (value 0) point at the column of their own lane's bank: pointing all of them at column 0
        // would make them collide, in every pass, with the real entry of bank 0
        for (size_t pos = 0; pos < ec.size(); ++pos) {
            const int c = (int)(pos & 31);
            ec[pos] = (uint16_t)(c < cols ? c : 0);
        }
        std::vector<char> used((size_t)S * 64);
        std::vector<int64_t> leftover;
        for (int rp = 0; rp < rows; ++rp) {
            const int64_t beg = out.h_row_ptr[rp];
            const int64_t end = std::min<int64_t>(out.h_row_ptr[rp + 1], beg + (int64_t)64 * S);
            std::fill(used.begin(), used.end(), 0);
            leftover.clear();
            int fill[32] = {0};  // positions already taken in each bank's lanes (slot-major: lane b, lane b+32)
            for (int64_t e = beg; e < end; ++e) {
                const int bank = out.h_col[e] & 31;
                if (fill[bank] < 2 * S) {
                    const int slot = fill[bank] >> 1, lane = bank + 32 * (fill[bank] & 1);
                    ++fill[bank];
                    used[(size_t)slot * 64 + lane] = 1;
                    const size_t idx = ((size_t)rp * S + slot) * 64 + lane;
                    ev[idx] = out.h_val[e];
                    ec[idx] = (uint16_t)out.h_col[e];
                } else {
                    leftover.push_back(e);
                }
            }
            // An entry whose bank's lanes are full meets a bank that is taken in every pass, so it costs its pass one
            // more cycle wherever it goes; all of them go to the same pass (free positions taken from the end: the
            // last slot's upper half fills up last), so that a row pays that cycle once and not once per entry.
            size_t pos = (size_t)S * 64;
            for (int64_t e : leftover) {
                do { --pos; } while (used[pos]);
                used[pos] = 1;
                const size_t idx = (size_t)rp * S * 64 + pos;
                ev[idx] = out.h_val[e];
                ec[idx] = (uint16_t)out.h_col[e];
            }
        }
    };
    if (out.slots <= 8) {
        std::vector<float> ev;
        std::vector<uint16_t> ec;
        build_slices(out.slots, ev, ec);
        HIP_TRY(m, upload(&out.ell_val, ev));
        HIP_TRY(m, upload(&out.ell_col, ec));
    }
    // Trimmed form: the slot count is set by the longest row, and with random masks a handful of rows are a few
    // entries longer than all others.  Take the smallest slot count that leaves at most 64 overflow entries per unit
    // (one per lane: a wave then pays one extra gather per step, against four per slot saved).
    if (out.slots >= 2 && out.slots <= 9) {
        const int units = rows / 4;
        for (int S = 1; S < out.slots; ++S) {
            int64_t worst = 0;
            for (int u = 0; u < units; ++u) {
                int64_t per_unit = 0;
                for (int q = 0; q < 4; ++q)
                    per_unit += std::max<int64_t>(0, out.h_row_ptr[4 * u + q + 1] - out.h_row_ptr[4 * u + q] - (int64_t)64 * S);
                worst = std::max(worst, per_unit);
            }
            if (worst > 64) continue;
            std::vector<float> ev, ov;
            std::vector<uint16_t> ec;
            std::vector<int32_t> optr((size_t)units + 1, 0);
            std::vector<uint32_t> oe;
            build_slices(S, ev, ec);
            for (int u = 0; u < units; ++u) {
                for (int q = 0; q < 4; ++q) {
                    const int rp = 4 * u + q;
                    for (int64_t e = out.h_row_ptr[rp] + (int64_t)64 * S; e < out.h_row_ptr[rp + 1]; ++e) {
                        oe.push_back(((uint32_t)q << 16) | (uint32_t)out.h_col[e]);
                        ov.push_back(out.h_val[e]);
                    }
                }
                optr[(size_t)u + 1] = (int32_t)oe.size();
            }
            out.slots_trim = S;
            HIP_TRY(m, upload(&out.ell_val_trim, ev));
            HIP_TRY(m, upload(&out.ell_col_trim, ec));
            out.h_ovf_ptr = optr;
            HIP_TRY(m, upload(&out.ovf_ptr, optr));
            HIP_TRY(m, upload(&out.ovf_ent, oe));
            HIP_TRY(m, upload(&out.ovf_val, ov));
            break;
        }
    }
    if (quarter_slots > 0) return build_quarter_wave(m, out, 0, quarter_slots, q16_gather16, gate_col_stride, soft_slots);
    return LSTM_OK;
}

extern "C" {

static int create_model(int layers, int input_dim, const int* hidden_dims, const int* gate_hidden_dims, int bidirectional,
                        int dtype, lstm_t** out)
{
    if (!out) return fail(nullptr, LSTM_ERR_ARG, "lstm_create: out is NULL");
    *out = nullptr;
    if (layers < 1 || input_dim < 1 || !hidden_dims)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_create: layers, input_dim and hidden_dim must be >= 1");
    if (bidirectional != 0 && bidirectional != 1)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_create: bidirectional must be 0 or 1");
    if (dtype != LSTM_F32 && dtype != LSTM_BF16) return fail(nullptr, LSTM_ERR_ARG, "lstm_create: unknown dtype");
    if (input_dim > (1 << 28)) return fail(nullptr, LSTM_ERR_ARG, "lstm_create: dimension too large");
    for (int l = 0; l < layers; ++l) {
        if (hidden_dims[l] < 1) return fail(nullptr, LSTM_ERR_ARG, "lstm_create: layers, input_dim and hidden_dim must be >= 1");
        if ((long long)hidden_dims[l] * 4 > (1 << 28)) return fail(nullptr, LSTM_ERR_ARG, "lstm_create: dimension too large");
        if (gate_hidden_dims && (gate_hidden_dims[l] < 1 || (long long)gate_hidden_dims[l] * 4 > (1 << 28)))
            return fail(nullptr, LSTM_ERR_ARG, "lstm_create_h: gate_hidden_dim must be >= 1");
    }
    lstm_t* m = new (std::nothrow) lstm355();
    if (!m) return fail(nullptr, LSTM_ERR_NOMEM, "lstm_create: host allocation failed");
    m->L = layers;
    m->D0 = input_dim;
    m->Dn = bidirectional ? 2 : 1;
    m->dtype = dtype;
    m->Hs.assign(hidden_dims, hidden_dims + layers);
    m->Gs.assign((size_t)layers, 0);
    if (gate_hidden_dims) m->Gs.assign(gate_hidden_dims, gate_hidden_dims + layers);
    m->H = *std::max_element(m->Hs.begin(), m->Hs.end());
    m->G = *std::max_element(m->Gs.begin(), m->Gs.end());
    m->state_off.assign((size_t)m->L * m->Dn + 1, 0);
    for (size_t n = 0; n < (size_t)m->L * m->Dn; ++n) m->state_off[n + 1] = m->state_off[n] + (size_t)m->Hs[n / (size_t)m->Dn];
    m->ld.resize((size_t)m->L * m->Dn);
    m->cooperative = g_default_cooperative;
    if (const char* sl = std::getenv("LSTM355_SPIN_LIMIT")) {
        const long v = std::atol(sl);
        if (v > 0) m->spin_limit = (unsigned)v;
    }
    if (const char* l2 = std::getenv("LSTM355_L2_HANDOVER")) m->device_scope_only = (std::atoi(l2) == 0) ? 1 : 0;
    if (const char* sp = std::getenv("LSTM355_SPARSE_PROJ_MAX_DENSITY")) m->sparse_proj_max_density = std::atof(sp);
    if (const char* pp = std::getenv("LSTM355_POLL_PACE")) m->poll_pace = std::max(-1, std::min(255, std::atoi(pp)));
    hipError_t e = hipGetDevice(&m->device);
    // two cells (directions, or two stacked layers) x two parities; H-LSTM: h slots, then the 4G hidden-layer slots
    m->xchg_slots = (m->G > 0 ? (size_t)m->H + 4 * (size_t)m->G : (size_t)4 * m->H) + 64;   // + XCD ids of a launch's workgroups
    if (e == hipSuccess) e = hipMalloc((void**)&m->xchg, m->xchg_slots * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipMemset(m->xchg, 0, m->xchg_slots * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipMalloc((void**)&m->timeout_flag, sizeof(int));
    if (e == hipSuccess) e = hipMemset(m->timeout_flag, 0, sizeof(int));
    if (e != hipSuccess) {
        const int rc = fail_hip(nullptr, e, "lstm_create: device set-up");
        lstm_destroy(m);
        return rc;
    }
    *out = m;
    return LSTM_OK;
}

// Does a separate projection launch of this input-side matrix run as a dense product on the matrix cores (zeros included)?
// Measured on MI355X: with a few hundred input rows or more the dense product beats the compressed ones at 10-15 % kept
// weights (the projection over the kept entries, tried before this is asked, takes the large sparse cases); with at most
// 64 input rows the stream over the fragment-ordered dense copy beats the lanes-over-entries kernel down to 5 % kept at
// every width from 256 to 4096 (batch 16: 14.5 against 15.9 us at n = 4096, 4.2 against 7.1 us at n = 1024).
static bool proj_runs_dense(const PackedMat& wx, int M, int D, bool bf16)
{
    if (!wx.dense) return false;
    if (!wx.compressed) return true;
    if (!proj_mfma_supported(bf16, D, D)) return false;
    if (M >= 256) return true;
    return M <= 64 && wx.dense_frag16 != nullptr && (double)wx.nnz >= 0.04 * (double)wx.rows * (double)wx.cols;
}

int lstm_create(int layers, int input_dim, int hidden_dim, int bidirectional, int dtype, lstm_t** out)
{
    if (out) *out = nullptr;
    if (layers < 1 || layers > (1 << 16)) return fail(nullptr, LSTM_ERR_ARG, "lstm_create: layers, input_dim and hidden_dim must be >= 1");
    const std::vector<int> hs((size_t)layers, hidden_dim);
    return create_model(layers, input_dim, hs.data(), nullptr, bidirectional, dtype, out);
}

int lstm_create_h(int layers, int input_dim, int hidden_dim, int gate_hidden_dim, int bidirectional, int dtype, lstm_t** out)
{
    if (out) *out = nullptr;
    if (gate_hidden_dim < 1 || (long long)gate_hidden_dim * 4 > (1 << 28))
        return fail(nullptr, LSTM_ERR_ARG, "lstm_create_h: gate_hidden_dim must be >= 1");
    if (dtype != LSTM_F32) return fail(nullptr, LSTM_ERR_ARG, "lstm_create_h: the H-LSTM cell is implemented for LSTM_F32 only");
    if (layers < 1 || layers > (1 << 16)) return fail(nullptr, LSTM_ERR_ARG, "lstm_create: layers, input_dim and hidden_dim must be >= 1");
    const std::vector<int> hs((size_t)layers, hidden_dim), gs((size_t)layers, gate_hidden_dim);
    return create_model(layers, input_dim, hs.data(), gs.data(), bidirectional, dtype, out);
}

int lstm_create_layers(int layers, int input_dim, const int* hidden_dims, const int* gate_hidden_dims, int bidirectional,
                       int dtype, lstm_t** out)
{
    if (out) *out = nullptr;
    if (layers < 1 || layers > (1 << 16) || !hidden_dims)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_create_layers: layers >= 1 and hidden_dims are required");
    if (gate_hidden_dims && dtype != LSTM_F32)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_create_layers: the H-LSTM cell is implemented for LSTM_F32 only");
    return create_model(layers, input_dim, hidden_dims, gate_hidden_dims, bidirectional, dtype, out);
}

int lstm_destroy(lstm_t* m)
{
    if (!m) return LSTM_OK;
    for (auto& x : m->ld) {
        free_mat(x.wx);
        free_mat(x.wh);
        free_mat(x.w2);
        if (x.bias) (void)hipFree(x.bias);
        if (x.bias2) (void)hipFree(x.bias2);
        if (x.u_slots) (void)hipFree(x.u_slots);
    }
    for (auto& sp : m->spans) { (void)hipEventDestroy(sp.e0); (void)hipEventDestroy(sp.e1); }
    for (auto& e : m->event_pool) (void)hipEventDestroy(e);
    if (m->xchg) (void)hipFree(m->xchg);
    if (m->timeout_flag) (void)hipFree(m->timeout_flag);
    delete m;
    return LSTM_OK;
}

const char* lstm_last_error(const lstm_t* m) { return m ? m->err.c_str() : g_create_error.c_str(); }

// LSTM_FMT_AUTO: row-compressed when at most a quarter of the entries are kept (H-LSTM: half).  The kernels that run both
// directions of a layer in one launch need both in the same form, so close to the threshold (within 5 % of all entries)
// the direction set second follows the one set first instead of landing on the other side of it by a few entries.
static bool auto_compressed(const lstm_t* m, int layer, int direction, bool masked, size_t kept, size_t total)
{
    if (!masked) return false;
    // The H-LSTM has no matrix-core path for dense weights at small batch, and its row-compressed kernels beat the dense
    // ones up to half the entries kept (800/800, two directions, batch 16, 40 % kept: 135 us per step dense, 37 compressed
    // with a launch per stage, 21 with the time loop on the device).
    const double limit = m->G > 0 ? 0.50 : 0.25;
    const double density = (double)kept / (double)total;
    if (m->Dn == 2) {
        const LayerDir& o = m->ld[(size_t)layer * 2 + (size_t)(1 - direction)];
        if (o.set && density > limit - 0.05 && density < limit + 0.05) return o.wh.compressed;
    }
    return density <= limit;
}

int lstm_set_weights(lstm_t* m, int layer, int direction, const float* Wx, const uint8_t* mask_x, const float* Wh,
                     const uint8_t* mask_h, const float* b, int format)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_set_weights: handle is NULL");
    if (layer < 0 || layer >= m->L || direction < 0 || direction >= m->Dn)
        return fail(m, LSTM_ERR_SHAPE, "lstm_set_weights: layer/direction outside the model");
    if (m->G > 0) return fail(m, LSTM_ERR_STATE, "lstm_set_weights: this handle is an H-LSTM, use lstm_set_weights_h");
    if (!Wx || !Wh || !b) return fail(m, LSTM_ERR_ARG, "lstm_set_weights: Wx, Wh and b are required");
    if (format != LSTM_FMT_AUTO && format != LSTM_FMT_DENSE_MASKED && format != LSTM_FMT_ROW_COMPRESSED)
        return fail(m, LSTM_ERR_ARG, "lstm_set_weights: unknown format");
    const int H = m->hid(layer), D = m->in_dim(layer), rows = 4 * H;
    size_t kept = 0, total = (size_t)rows * D + (size_t)rows * H;
    for (int which = 0; which < 2; ++which) {
        const uint8_t* mk = which ? mask_h : mask_x;
        const size_t n = (size_t)rows * (which ? H : D);
        if (!mk) { kept += n; continue; }
        for (size_t i = 0; i < n; ++i) {
            if (mk[i] > 1) return fail(m, LSTM_ERR_ARG, "lstm_set_weights: mask bytes must be 0 or 1");
            kept += mk[i];
        }
    }
    bool compressed;
    if (format == LSTM_FMT_AUTO)
        compressed = auto_compressed(m, layer, direction, mask_x || mask_h, kept, total);
    else
        compressed = (format == LSTM_FMT_ROW_COMPRESSED);
    if (compressed && (D > 65536 || H > 65536))
        return fail(m, LSTM_ERR_ARG, "lstm_set_weights: row-compressed form needs dimensions <= 65536");
    HIP_TRY(m, hipSetDevice(m->device));
    LayerDir& x = m->ld[(size_t)layer * m->Dn + direction];
    x.set = false;
    const bool bf16 = (m->dtype == LSTM_BF16);
    // W_x is kept in both forms when compressed: large T*B projections run dense on the matrix cores
    int rc = pack_matrix(m, x.wx, Wx, mask_x, H, D, compressed, bf16, true, bf16 ? 0 : 24, 0, 0, !bf16, true);
    if (rc != LSTM_OK) return rc;
    rc = pack_matrix(m, x.wh, Wh, mask_h, H, H, compressed, bf16, false, kMaxRecurrentSlots);
    if (rc != LSTM_OK) return rc;
    std::vector<float> bp(rows);
    for (int rp = 0; rp < rows; ++rp) bp[rp] = b[(rp & 3) * H + (rp >> 2)];
    if (x.bias) { (void)hipFree(x.bias); x.bias = nullptr; }
    HIP_TRY(m, upload(&x.bias, bp));
    x.set = true;
    // One launch serves both directions of a layer and is built for the larger slot count: a direction trimmed further
    // than the other would pay for the other's slots and for its own entries outside them.
    if (m->Dn == 2) {
        LayerDir& o = m->ld[(size_t)layer * 2 + (size_t)(1 - direction)];
        if (o.set && x.wh.q16_slots > 0 && o.wh.q16_slots > 0 && x.wh.q16_slots != o.wh.q16_slots) {
            const int target = std::max(x.wh.q16_slots, o.wh.q16_slots);
            rc = build_quarter_wave(m, x.wh.q16_slots < target ? x.wh : o.wh, target, kMaxRecurrentSlots);
            if (rc != LSTM_OK) return rc;
        }
        if (o.set && x.wx.q16_slots > 0 && o.wx.q16_slots > 0 && x.wx.q16_slots != o.wx.q16_slots) {
            const int target = std::max(x.wx.q16_slots, o.wx.q16_slots);
            rc = build_quarter_wave(m, x.wx.q16_slots < target ? x.wx : o.wx, target, 24, true);
            if (rc != LSTM_OK) return rc;
        }
    }
    return LSTM_OK;
}

int lstm_set_weights_h(lstm_t* m, int layer, int direction, const float* W1x, const uint8_t* mask_1x, const float* W1h,
                       const uint8_t* mask_1h, const float* b1, const float* W2, const uint8_t* mask_2, const float* b2,
                       int format)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_set_weights_h: handle is NULL");
    if (m->G <= 0) return fail(m, LSTM_ERR_STATE, "lstm_set_weights_h: this handle is a conventional LSTM, use lstm_set_weights");
    if (layer < 0 || layer >= m->L || direction < 0 || direction >= m->Dn)
        return fail(m, LSTM_ERR_SHAPE, "lstm_set_weights_h: layer/direction outside the model");
    if (!W1x || !W1h || !b1 || !W2 || !b2) return fail(m, LSTM_ERR_ARG, "lstm_set_weights_h: W1x, W1h, b1, W2 and b2 are required");
    if (format != LSTM_FMT_AUTO && format != LSTM_FMT_DENSE_MASKED && format != LSTM_FMT_ROW_COMPRESSED)
        return fail(m, LSTM_ERR_ARG, "lstm_set_weights_h: unknown format");
    const int H = m->hid(layer), G = m->ghid(layer), D = m->in_dim(layer);
    const size_t sizes[3] = {(size_t)4 * G * D, (size_t)4 * G * H, (size_t)4 * H * G};
    const uint8_t* masks[3] = {mask_1x, mask_1h, mask_2};
    size_t kept = 0, total = 0;
    for (int i = 0; i < 3; ++i) {
        total += sizes[i];
        if (!masks[i]) { kept += sizes[i]; continue; }
        for (size_t e = 0; e < sizes[i]; ++e) {
            if (masks[i][e] > 1) return fail(m, LSTM_ERR_ARG, "lstm_set_weights_h: mask bytes must be 0 or 1");
            kept += masks[i][e];
        }
    }
    bool compressed;
    if (format == LSTM_FMT_AUTO)
        compressed = auto_compressed(m, layer, direction, mask_1x || mask_1h || mask_2, kept, total);
    else
        compressed = (format == LSTM_FMT_ROW_COMPRESSED);
    if (compressed && (D > 65536 || H > 65536 || G > 65536))
        return fail(m, LSTM_ERR_ARG, "lstm_set_weights_h: row-compressed form needs dimensions <= 65536");
    HIP_TRY(m, hipSetDevice(m->device));
    LayerDir& x = m->ld[(size_t)layer * m->Dn + direction];
    x.set = false;
    // hidden layers: 4G rows, packed row 4g+q; kept dense as well for the projection on the matrix cores
    int rc = pack_matrix(m, x.wx, W1x, mask_1x, G, D, compressed, false, true, 0, 0, 0, true);
    if (rc != LSTM_OK) return rc;
    rc = pack_matrix(m, x.wh, W1h, mask_1h, G, H, compressed, false, false, kMaxRecurrentSlots, 0, 12);
    if (rc != LSTM_OK) return rc;
    // gate outputs: 4H rows, packed row 4j+q, columns = hidden units of the row's own gate
    rc = pack_matrix(m, x.w2, W2, mask_2, H, G, compressed, false, false, kMaxRecurrentSlots, G, 12);
    if (rc != LSTM_OK) return rc;
    std::vector<float> bp1((size_t)4 * G), bp2((size_t)4 * H);
    for (int rp = 0; rp < 4 * G; ++rp) bp1[rp] = b1[(size_t)(rp & 3) * G + (rp >> 2)];
    for (int rp = 0; rp < 4 * H; ++rp) bp2[rp] = b2[(size_t)(rp & 3) * H + (rp >> 2)];
    if (x.bias) { (void)hipFree(x.bias); x.bias = nullptr; }
    if (x.bias2) { (void)hipFree(x.bias2); x.bias2 = nullptr; }
    HIP_TRY(m, upload(&x.bias, bp1));
    HIP_TRY(m, upload(&x.bias2, bp2));
    // stamped words of the batch-1 kernel's hidden-layer activations: [eager | captured], zero = stamp of an even count
    if (x.u_slots) { (void)hipFree(x.u_slots); x.u_slots = nullptr; }
    HIP_TRY(m, hipMalloc((void**)&x.u_slots, (size_t)8 * G * sizeof(unsigned)));
    HIP_TRY(m, hipMemset(x.u_slots, 0, (size_t)8 * G * sizeof(unsigned)));
    x.u_epoch = 0;
    x.u_dirty = false;
    x.set = true;
    // One launch serves both matrices of every direction of a layer and is built for the largest slot count: bring the
    // others up to it (a matrix trimmed further would pay for those slots and for its own entries outside them).
    {
        PackedMat* mats[4] = {&x.wh, &x.w2, nullptr, nullptr};
        int strides[4] = {0, G, 0, G};
        if (m->Dn == 2) {
            LayerDir& o = m->ld[(size_t)layer * 2 + (size_t)(1 - direction)];
            if (o.set) { mats[2] = &o.wh; mats[3] = &o.w2; }
        }
        int target = 0;
        bool all = true;
        for (PackedMat* p : mats)
            if (p) { all = all && p->q16_slots > 0; target = std::max(target, p->q16_slots); }
        for (int i = 0; i < 4 && all; ++i)
            if (mats[i] && mats[i]->q16_slots < target) {
                rc = build_quarter_wave(m, *mats[i], target, kMaxRecurrentSlots, false, strides[i]);
                if (rc != LSTM_OK) return rc;
            }
    }
    return LSTM_OK;
}

// ---- workspace carve-up --------------------------------------------------------------------------------
struct Workspace {
    size_t P_off[2], XT_off, Y_off[2], c_off[2], Yb_off[2], hb0_off, slot_off, slot_bytes, hx_off, mflag_off, U_off[2], total;
};
static Workspace carve(const lstm_t* m, int T, int B)
{
    Workspace w{};
    size_t off = 0;
    const size_t M = (size_t)T * B, H = m->H;
    const size_t prow = m->G > 0 ? (size_t)m->G : H;   // H-LSTM: the projection feeds the 4G hidden-layer rows
    for (int d = 0; d < 2; ++d) {
        w.P_off[d] = off;
        if (d < m->Dn) off += align256(M * 4 * prow * sizeof(float));
    }
    size_t Dmax = (size_t)m->D0;
    if (m->L > 1) Dmax = std::max(Dmax, (size_t)m->Dn * H);
    w.XT_off = off;
    off += align256(Dmax * M * sizeof(float));
    for (int i = 0; i < 2; ++i) {
        w.Y_off[i] = off;
        if (m->L > 1) off += align256(M * m->Dn * H * sizeof(float));
    }
    for (int d = 0; d < 2; ++d) {
        w.c_off[d] = off;
        if (d < m->Dn) off += align256((size_t)B * H * sizeof(float));
    }
    // bf16 models: bf16 copy of each layer's hidden sequence (matrix-core operand of the next step and of the
    // next layer's projection) and a bf16 copy of h0
    for (int i = 0; i < 2; ++i) {
        w.Yb_off[i] = off;
        if (m->dtype == LSTM_BF16) off += align256(M * m->Dn * H * sizeof(uint16_t));
    }
    w.hb0_off = off;
    if (m->dtype == LSTM_BF16) off += align256((size_t)m->Dn * B * H * sizeof(uint16_t));
    // tagged exchange slots of the small-batch persistent recurrence: per direction [2][batch groups][H][columns of a
    // group] (ragged last group filled up: at most B + 3 columns), then one slot per workgroup for the XCD ids, 64 per
    // batch group
    // (H-LSTM: h slots in [k][columns of a batch group] blocks padded to 256 bytes, ragged last group filled up,
    // then one flag per unit group, 64 per batch group, then the XCD id slots)
    w.slot_off = off;
    if (B >= 2) {
        const size_t groups = (size_t)B / 2 + 1;
        w.slot_bytes = m->G > 0 ? (size_t)m->Dn * (((size_t)B + 3) * H * sizeof(unsigned long long) + groups * 256 +
                                                   groups * 64 * (sizeof(unsigned) + sizeof(unsigned long long)))
                                : (size_t)m->Dn * (2 * ((size_t)B + 3) * H + groups * 64) * sizeof(unsigned long long);
        off += align256(w.slot_bytes);
    }
    // bf16 large-batch persistent recurrence: two exchange buffers of h_t and one flag per tile
    w.hx_off = off;
    w.mflag_off = off;
    if (m->dtype == LSTM_BF16) {
        // the widest requirement over the layers whose width the kernel takes
        size_t xbytes = 0, flags = 0;
        for (int l = 0; l < m->L; ++l)
            if (persist_mfma_supported(B, m->hid(l))) {
                xbytes = std::max(xbytes, persist_mfma_exchange_bytes(B, m->hid(l)));
                flags = std::max(flags, persist_mfma_flag_count(B, m->hid(l)));
            }
        if (xbytes > 0) {
            off += align256(xbytes);
            w.mflag_off = off;
            off += align256(flags * sizeof(unsigned));
        }
    } else if (m->G == 0) {
        // fp32 dense persistent recurrence at small and medium batch: the same two regions (whether a layer's recurrent
        // matrix is held dense is not known before its weights are set, so every width the kernel takes is provided for)
        size_t xfloats = 0;
        for (int l = 0; l < m->L; ++l) {
            const int Hl = m->hid(l);
            LaunchCut cut;
            if (choose_cut(B, m->Dn, [&](int b, int nd) { return persist_dense_f32_supported(b, Hl, nd); }, &cut))
                for (int b : {(B + cut.chunks - 1) / cut.chunks, B / cut.chunks})
                    xfloats = std::max(xfloats, persist_dense_f32_exchange_floats(b, Hl, m->Dn / cut.passes));
        }
        off += align256(xfloats * sizeof(float));
        w.mflag_off = off;
        if (xfloats > 0) off += align256(persist_dense_f32_ids_count() * sizeof(unsigned long long));
    }
    // H-LSTM: hidden-layer activations of the current step, [B][4G] per direction (stepwise paths); the small-batch
    // persistent kernel uses both directions' storage as one array of [k][columns of a batch group] blocks
    for (int d = 0; d < 2; ++d) {
        w.U_off[d] = off;
        if (m->G > 0 && d < m->Dn) off += align256(((size_t)B + 3) * 4 * m->G * sizeof(float) + ((size_t)B / 2 + 1) * 256);
    }
    w.total = off;
    return w;
}

size_t lstm_workspace_bytes(const lstm_t* m, int T, int B)
{
    if (!m || T < 0 || B < 0) return 0;
    if (T == 0 || B == 0) return 256;
    return carve(m, T, B).total;
}

int lstm_set_plan(lstm_t* m, int plan, int waves_per_group)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_set_plan: handle is NULL");
    if (plan != LSTM_PLAN_AUTO && plan != LSTM_PLAN_STEPWISE && plan != LSTM_PLAN_PERSISTENT)
        return fail(m, LSTM_ERR_ARG, "lstm_set_plan: unknown plan");
    if (waves_per_group < 0 || waves_per_group > 16)
        return fail(m, LSTM_ERR_ARG, "lstm_set_plan: waves_per_group must be in [0,16]");
    m->plan = plan;
    m->waves_per_group = waves_per_group;
    return LSTM_OK;
}

int lstm_set_launch_mode(lstm_t* m, int cooperative)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_set_launch_mode: handle is NULL");
    m->cooperative = cooperative ? 1 : 0;
    return LSTM_OK;
}

int lstm_set_default_launch_mode(int cooperative)
{
    g_default_cooperative = cooperative ? 1 : 0;
    return LSTM_OK;
}

int lstm_set_profiling(lstm_t* m, int enable)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_set_profiling: handle is NULL");
    m->profiling = enable != 0;
    return LSTM_OK;
}

int lstm_get_profile(lstm_t* m, double* proj_us, int* proj_launches, double* rec_us, int* rec_launches)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_get_profile: handle is NULL");
    double us[2] = {0.0, 0.0};
    int cnt[2] = {0, 0};
    int rc = LSTM_OK;
    for (auto& sp : m->spans) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(sp.e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, sp.e0, sp.e1);
        if (e != hipSuccess) rc = fail_hip(m, e, "lstm_get_profile");
        us[sp.kind] += (double)ms * 1000.0;
        cnt[sp.kind] += 1;
        m->event_pool.push_back(sp.e0);
        m->event_pool.push_back(sp.e1);
    }
    m->spans.clear();
    if (proj_us) *proj_us = us[0];
    if (proj_launches) *proj_launches = cnt[0];
    if (rec_us) *rec_us = us[1];
    if (rec_launches) *rec_launches = cnt[1];
    return rc;
}

int lstm_describe_plan(const lstm_t* m, char* buf, size_t buf_bytes)
{
    if (!m || !buf || buf_bytes == 0) return fail(m, LSTM_ERR_ARG, "lstm_describe_plan: bad arguments");
    std::snprintf(buf, buf_bytes, "%s", m->last_plan.c_str());
    return LSTM_OK;
}

// Step tags of the batch-1 exchange (slots owned by the handle): `n` fresh tags, the first one being *base + 1.
// An eager call draws them from a counter that lives in the handle, so the slots never need clearing between calls.
// A call that is being captured into a graph cannot do that - every replay would repeat the tags of the capture and
// match what the previous replay left in the slots - so it clears the slots inside the graph (a fill kernel, once per
// forward), counts from zero, and leaves the handle's counter above everything a replay will ever write, which keeps
// later eager calls from matching a replay's left-overs.
static int take_b1_tags(lstm_t* m, unsigned n, size_t slots, hipStream_t s, unsigned* base)
{
    if (m->capturing) {
        if (!m->cap_cleared) {
            HIP_TRY(m, launch_fill_u64(m->xchg, slots, 0ull, s));
            m->cap_cleared = true;
            m->cap_tag = 0;
        }
        *base = m->cap_tag;
        m->cap_tag += n;
        if (m->tag_base < m->cap_tag) m->tag_base = m->cap_tag;
        return LSTM_OK;
    }
    if (m->tag_base > 0xFFFFFFFFu - n - 2u) {
        // tag space exhausted: restart from a clean slate
        HIP_TRY(m, launch_fill_u64(m->xchg, slots, 0ull, s));
        m->tag_base = 0;
    }
    *base = m->tag_base;
    m->tag_base += n;
    return LSTM_OK;
}

// H-LSTM stack (fp32).  Per layer and direction: the hidden layers' input side for all timesteps as one projection
// (P1 = W1x.x + b1, 4G rows), then per step the hidden layers (stage 1) and the gate outputs with the cell update
// (stage 2).
static int forward_hlstm(lstm_t* m, int T, int B, const void* x, const float* h0, const float* c0, float* y, float* hT,
                         float* cT, const Workspace& ws, char* base, hipStream_t s)
{
    const int Dn = m->Dn, L = m->L;
    const int M = T * B;
    float* P[2] = {(float*)(base + ws.P_off[0]), (float*)(base + ws.P_off[1])};
    float* XT = (float*)(base + ws.XT_off);
    float* Ybuf[2] = {(float*)(base + ws.Y_off[0]), (float*)(base + ws.Y_off[1])};
    float* cbuf[2] = {(float*)(base + ws.c_off[0]), (float*)(base + ws.c_off[1])};
    float* U[2] = {(float*)(base + ws.U_off[0]), (float*)(base + ws.U_off[1])};
    char tag[96];
    bool hslots_clean = false;   // exchange slots and flags zeroed during this forward (tags then restart at 1)
    int hslots_H = 0, hslots_G = 0;   // widths of the layer the region was last laid out for
    unsigned htag = 0;
    for (int l = 0; l < L; ++l) {
        const int H = m->hid(l), G = m->ghid(l);
        const int D = m->in_dim(l);
        const void* X = (l == 0) ? x : (const void*)Ybuf[(l - 1) & 1];
        float* Yout = (l == L - 1) ? y : Ybuf[l & 1];
        const int y_ld = Dn * H;
        // batch 1 with all three matrices row-compressed and small enough for registers: time loop on the device
        bool persist[2] = {false, false};
        for (int d = 0; d < Dn; ++d) {
            const LayerDir& w = m->ld[(size_t)l * Dn + d];
            persist[d] = B == 1 && m->plan != LSTM_PLAN_STEPWISE && w.wx.compressed && w.wh.compressed && w.w2.compressed &&
                         w.wx.ell_val && w.wh.ell_val && w.w2.ell_val &&
                         persist_b1_hlstm_supported(H, G, D, w.wx.slots, w.wh.slots, w.w2.slots);
            if (m->plan == LSTM_PLAN_PERSISTENT && B == 1 && !persist[d])
                return fail(m, LSTM_ERR_ARG, "lstm_forward: persistent plan not available for this shape");
        }
        bool xt_ready = false;
        bool proj_dense[2] = {false, false};
        for (int d = 0; d < Dn; ++d) {
            if (persist[d]) continue;
            const LayerDir& w = m->ld[(size_t)l * Dn + d];
            ProfSpan span(m, s, 0);
            const bool dense_proj = proj_runs_dense(w.wx, M, D, false);
            proj_dense[d] = dense_proj;
            if (!dense_proj && w.wx.ell_val && proj_ell_small_supported(M, 4 * G, D, w.wx.slots)) {
                HIP_TRY(m, launch_proj_ell_small(X, false, D, false, w.wx.ell_val, w.wx.ell_col, w.wx.slots, w.bias, P[d], M,
                                                 4 * G, D, s));
            } else if (!dense_proj) {
                if (!xt_ready) {
                    HIP_TRY(m, launch_transpose_to_f32(X, false, D, XT, M, D, false, s));
                    xt_ready = true;
                }
                HIP_TRY(m, launch_proj_csr(XT, w.wx.row_ptr, w.wx.col16, w.wx.val, w.bias, P[d], M, 4 * G, s));
            } else if (proj_mfma_supported(false, D, D)) {
                HIP_TRY(m, launch_proj_mfma(X, false, D, w.wx.dense, false, w.bias, P[d], M, 4 * G, D, s, w.wx.dense_frag16));
            } else {
                HIP_TRY(m, launch_proj_dense(X, false, D, w.wx.dense, false, w.bias, P[d], M, 4 * G, D, s));
            }
        }
        // small batch, W1h and W2 of every direction row-compressed with rows of at most 256 kept entries (the
        // quarter-wave form): one launch per layer with the time loop on the device
        {
            int nz = 0, upw = 0, bw = 0, ug = 0, bg = 0;
            bool pb_ok = B >= 2 && m->plan != LSTM_PLAN_STEPWISE;
            bool any_extra = false;
            for (int d = 0; d < Dn && pb_ok; ++d) {
                const LayerDir& w = m->ld[(size_t)l * Dn + d];
                pb_ok = w.wh.compressed && w.w2.compressed && w.wh.q16_slots > 0 && w.w2.q16_slots > 0;
                nz = std::max(nz, std::max(w.wh.q16_slots, w.w2.q16_slots));
                any_extra = any_extra || w.wh.q16_ovf_ptr || w.w2.q16_ovf_ptr;
            }
            LaunchCut cut;
            pb_ok = pb_ok && choose_cut(B, Dn, [&](int b, int nd) { return persist_batched_h_plan(b, H, G, nz, nd, &upw, &bw, &ug, &bg); }, &cut);
            const bool trimmed = any_extra;
            if (m->plan == LSTM_PLAN_PERSISTENT && B >= 2 && !pb_ok)
                return fail(m, LSTM_ERR_ARG, "lstm_forward: persistent plan not available for this shape");
            if (pb_ok) {
                unsigned long long* hslots = (unsigned long long*)(base + ws.slot_off);
                const size_t groups = (size_t)B / 2 + 1;
                const size_t hslot_bytes = (size_t)Dn * (((size_t)B + 3) * H * sizeof(unsigned long long) + groups * 256);
                unsigned* hflags = (unsigned*)(base + ws.slot_off + hslot_bytes);
                unsigned long long* hxcc = (unsigned long long*)(hflags + (size_t)Dn * groups * 64);
                // (a layer of other widths lays the region out differently: what the previous layer left under the
                // new flag positions is not a tag, so the region starts from zero again)
                if (!hslots_clean || hslots_H != H || hslots_G != G) {
                    HIP_TRY(m, launch_fill_u64(hslots, align256(ws.slot_bytes) / sizeof(unsigned long long), 0ull, s));
                    hslots_clean = true;
                    hslots_H = H; hslots_G = G;
                    htag = 0;
                }
                for (int launch = 0; launch < cut.passes * cut.chunks; ++launch) {
                const int pass = launch / cut.chunks, chunk = launch % cut.chunks;
                const int nd = Dn / cut.passes, d_lo = pass * nd;
                const int b_lo = chunk_begin(B, cut.chunks, chunk), bn = chunk_begin(B, cut.chunks, chunk + 1) - b_lo;
                persist_batched_h_plan(bn, H, G, nz, nd, &upw, &bw, &ug, &bg);
                PersistBatchedHArgs a{};
                for (int d = d_lo; d < d_lo + nd; ++d) {
                    const LayerDir& w = m->ld[(size_t)l * Dn + d];
                    const size_t n = (size_t)l * Dn + d;
                    PersistBatchedHDir& q = a.d[d - d_lo];
                    q.P1 = P[d] + (size_t)b_lo * 4 * G;
                    q.q16_val_1h = w.wh.q16_val; q.q16_col_1h = w.wh.q16_col; q.slots_1h = w.wh.q16_slots;
                    q.ovf_ptr_1h = w.wh.q16_ovf_ptr; q.ovf_ent_1h = w.wh.q16_ovf_ent; q.ovf_val_1h = w.wh.q16_ovf_val;
                    q.q16_val_2 = w.w2.q16_val; q.q16_col_2 = w.w2.q16_col; q.slots_2 = w.w2.q16_slots;
                    q.ovf_ptr_2 = w.w2.q16_ovf_ptr; q.ovf_ent_2 = w.w2.q16_ovf_ent; q.ovf_val_2 = w.w2.q16_ovf_val;
                    q.bias2 = w.bias2;
                    const size_t so = m->soff(n) * B + (size_t)b_lo * H;
                    q.h0 = h0 ? h0 + so : nullptr;
                    q.c0 = c0 ? c0 + so : nullptr;
                    q.y = Yout + (size_t)b_lo * y_ld + (size_t)d * H; q.y_ld = y_ld;
                    q.hT = hT ? hT + so : nullptr;
                    q.cT = cT ? cT + so : nullptr;
                    q.reverse = d;
                    if (chunk == 0) {
                        char cuts[24] = "";
                        if (cut.chunks > 1) std::snprintf(cuts, sizeof cuts, ",batch/%d", cut.chunks);
                        std::snprintf(tag, sizeof tag, "l%d.d%d:proj=%s,rec=persist_batched-hlstm-csr%s(s%d,u%d,b%d%s);", l, d,
                                      proj_dense[d] ? "dense" : "csr", trimmed ? "+ovf" : "", nz, upw, bw, cuts);
                        m->last_plan += tag;
                    }
                }
                a.T = T; a.B = bn; a.Bld = B; a.H = H; a.G = G;
                a.xchg_h = hslots; a.xchg_u = U[0]; a.flags = hflags; a.xcc_ids = hxcc;
                a.tag_base = htag; a.timeout_flag = m->timeout_flag; a.spin_limit = m->spin_limit; a.device_scope_only = m->device_scope_only;
                htag += (unsigned)T + 1u;
                ProfSpan span(m, s, 1);
                HIP_TRY(m, launch_persist_batched_h(a, nd, nz, m->launch_mode(), s));
                }
                continue;
            }
        }
        // small batch, every direction row-compressed: both stages of a step for all directions in two launches
        bool pair_ok = B >= 1;
        {
            int nz1 = 1, nz2 = 1;
            for (int d = 0; d < Dn; ++d) {
                const LayerDir& w = m->ld[(size_t)l * Dn + d];
                pair_ok = pair_ok && !persist[d] && w.wh.compressed && w.w2.compressed && w.wh.ell_val && w.w2.ell_val;
                nz1 = std::max(nz1, w.wh.slots);
                nz2 = std::max(nz2, w.w2.slots);
            }
            pair_ok = pair_ok && hstep_pair_supported(H, G, nz1, nz2);
        }
        if (pair_ok) {
            ProfSpan span(m, s, 1);
            for (int d = 0; d < Dn; ++d) {
                const size_t n = (size_t)l * Dn + d;
                if (c0) HIP_TRY(m, hipMemcpyAsync(cbuf[d], c0 + m->soff(n) * B, (size_t)B * H * sizeof(float), hipMemcpyDeviceToDevice, s));
                else HIP_TRY(m, launch_fill_f32(cbuf[d], (size_t)B * H, 0.0f, s));
                std::snprintf(tag, sizeof tag, "l%d.d%d:proj=%s,rec=hlstm-stepwise-pair-csr;", l, d, proj_dense[d] ? "dense" : "csr");
                m->last_plan += tag;
            }
            for (int step = 0; step < T; ++step) {
                HStepPairArgs a{};
                for (int d = 0; d < Dn; ++d) {
                    const LayerDir& w = m->ld[(size_t)l * Dn + d];
                    const size_t n = (size_t)l * Dn + d;
                    const int t = d ? (T - 1 - step) : step;
                    HStepDir& q = a.d[d];
                    q.P1 = P[d];
                    if (step == 0) {
                        q.h_prev = h0 ? h0 + m->soff(n) * B : nullptr;
                        q.h_prev_ld = H;
                    } else {
                        const int tp = d ? t + 1 : t - 1;
                        q.h_prev = Yout + (size_t)tp * B * y_ld + (size_t)d * H;
                        q.h_prev_ld = y_ld;
                    }
                    q.u = U[d];
                    q.ell_val_1h = w.wh.ell_val; q.ell_col_1h = w.wh.ell_col; q.slots_1h = w.wh.slots;
                    q.ell_val_2 = w.w2.ell_val; q.ell_col_2 = w.w2.ell_col; q.slots_2 = w.w2.slots;
                    q.bias2 = w.bias2;
                    q.c = cbuf[d];
                    q.y_t = Yout + (size_t)t * B * y_ld + (size_t)d * H;
                    q.y_ld = y_ld;
                    q.hT = hT ? hT + m->soff(n) * B : nullptr;
                    q.cT = cT ? cT + m->soff(n) * B : nullptr;
                    q.t = t;
                }
                a.B = B; a.H = H; a.G = G; a.last = (step == T - 1);
                HIP_TRY(m, launch_hstep_pair(a, Dn, s));
            }
            continue;
        }
        for (int d = 0; d < Dn; ++d) {
            LayerDir& w = m->ld[(size_t)l * Dn + d];
            const size_t n = (size_t)l * Dn + d;
            ProfSpan span(m, s, 1);
            if (persist[d]) {
                unsigned tag0 = 0;
                const int trc = take_b1_tags(m, (unsigned)T + 1u, (size_t)m->H, s, &tag0);
                if (trc != LSTM_OK) return trc;
                // the stamped words: a captured launch clears its own array inside the graph and counts from zero (every
                // replay then starts from the same state); an eager launch goes on counting where the last one stopped
                unsigned* uarr = w.u_slots;
                unsigned uepoch = 0;
                if (m->capturing) {
                    uarr += (size_t)4 * G;
                    HIP_TRY(m, launch_fill_u64((unsigned long long*)uarr, (size_t)2 * G, 0ull, s));
                } else {
                    if (w.u_dirty || w.u_epoch > 0xFFFFFFFFu - (unsigned)T - 2u) {
                        HIP_TRY(m, launch_fill_u64((unsigned long long*)uarr, (size_t)2 * G, 0ull, s));
                        w.u_epoch = 0;
                        w.u_dirty = false;
                    }
                    uepoch = w.u_epoch;
                }
                PersistHArgs a{};
                a.ell_val_1x = w.wx.ell_val; a.ell_col_1x = w.wx.ell_col; a.slots_1x = w.wx.slots;
                a.ell_val_1h = w.wh.ell_val; a.ell_col_1h = w.wh.ell_col; a.slots_1h = w.wh.slots;
                a.ell_val_2 = w.w2.ell_val; a.ell_col_2 = w.w2.ell_col; a.slots_2 = w.w2.slots;
                a.bias1 = w.bias; a.bias2 = w.bias2;
                a.x = (const float*)X; a.x_ld = D; a.D = D;
                a.h0 = h0 ? h0 + m->soff(n) : nullptr;
                a.c0 = c0 ? c0 + m->soff(n) : nullptr;
                a.y = Yout + (size_t)d * H; a.y_ld = y_ld;
                a.hT = hT ? hT + m->soff(n) : nullptr;
                a.cT = cT ? cT + m->soff(n) : nullptr;
                a.T = T; a.H = H; a.G = G; a.reverse = d;
                a.xchg_h = m->xchg; a.xchg_u = uarr; a.u_epoch = uepoch;
                a.tag_base = tag0;
                a.timeout_flag = m->timeout_flag; a.spin_limit = m->spin_limit;
                a.poll_pace_u = m->poll_pace >= 0 ? m->poll_pace : kPollPaceHlstmB1;
                std::snprintf(tag, sizeof tag, "l%d.d%d:proj=fused,rec=persist_b1-hlstm-csr;", l, d);
                m->last_plan += tag;
                HIP_TRY(m, launch_persist_b1_hlstm(a, m->launch_mode(), s));
                if (!m->capturing) w.u_epoch += (unsigned)T;
                continue;
            }
            if (c0) HIP_TRY(m, hipMemcpyAsync(cbuf[d], c0 + m->soff(n) * B, (size_t)B * H * sizeof(float), hipMemcpyDeviceToDevice, s));
            else HIP_TRY(m, launch_fill_f32(cbuf[d], (size_t)B * H, 0.0f, s));
            std::snprintf(tag, sizeof tag, "l%d.d%d:proj=%s,rec=hlstm-stepwise-%s;", l, d,
                          proj_dense[d] ? "dense" : "csr", w.wh.compressed ? "csr" : "dense");
            m->last_plan += tag;
            for (int step = 0; step < T; ++step) {
                const int t = d ? (T - 1 - step) : step;
                HStage1Args a1{};
                a1.P1 = P[d];
                if (step == 0) {
                    a1.h_prev = h0 ? h0 + m->soff(n) * B : nullptr;
                    a1.h_prev_ld = H;
                } else {
                    const int tp = d ? t + 1 : t - 1;
                    a1.h_prev = Yout + (size_t)tp * B * y_ld + (size_t)d * H;
                    a1.h_prev_ld = y_ld;
                }
                if (w.wh.compressed) { a1.row_ptr = w.wh.row_ptr; a1.col = w.wh.col16; a1.val = w.wh.val; }
                else a1.w_dense = (const float*)w.wh.dense;
                a1.u = U[d];
                a1.t = t; a1.B = B; a1.H = H; a1.G = G;
                HIP_TRY(m, launch_hstage1(a1, s));
                HStage2Args a2{};
                a2.u = U[d];
                if (w.w2.compressed) { a2.row_ptr = w.w2.row_ptr; a2.col = w.w2.col16; a2.val = w.w2.val; }
                else a2.w_dense = (const float*)w.w2.dense;
                a2.bias2 = w.bias2;
                a2.c = cbuf[d];
                a2.y_t = Yout + (size_t)t * B * y_ld + (size_t)d * H;
                a2.y_ld = y_ld;
                a2.hT = hT ? hT + m->soff(n) * B : nullptr;
                a2.cT = cT ? cT + m->soff(n) * B : nullptr;
                a2.last = (step == T - 1);
                a2.B = B; a2.H = H; a2.G = G;
                HIP_TRY(m, launch_hstage2(a2, s));
            }
        }
    }
    return LSTM_OK;
}

static int run_forward(lstm_t* m, int T, int B, const void* x, const float* h0, const float* c0, float* y, float* hT,
                       float* cT, const Workspace& ws, char* base, hipStream_t s);

int lstm_forward(lstm_t* m, int T, int B, const void* x, const float* h0, const float* c0, float* y, float* hT,
                 float* cT, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_forward: handle is NULL");
    if (T < 0 || B < 0) return fail(m, LSTM_ERR_ARG, "lstm_forward: T and B must be >= 0");
    for (const auto& x_ : m->ld)
        if (!x_.set) return fail(m, LSTM_ERR_STATE, "lstm_forward: weights of some (layer, direction) not set");
    if (T == 0 || B == 0) return LSTM_OK;
    if (!x || !y) return fail(m, LSTM_ERR_ARG, "lstm_forward: x and y are required");
    if (!workspace) return fail(m, LSTM_ERR_ARG, "lstm_forward: workspace is NULL");
    if (((uintptr_t)workspace & 255) != 0) return fail(m, LSTM_ERR_ARG, "lstm_forward: workspace must be 256-byte aligned");
    if ((long long)T * B > (1ll << 30)) return fail(m, LSTM_ERR_ARG, "lstm_forward: T*B too large");
    const Workspace ws = carve(m, T, B);
    if (workspace_bytes < ws.total) return fail(m, LSTM_ERR_NOMEM, "lstm_forward: workspace too small");
    hipStream_t s = (hipStream_t)stream;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    HIP_TRY(m, hipStreamIsCapturing(s, &cap));
    m->capturing = (cap != hipStreamCaptureStatusNone);
    m->cap_cleared = false;
    m->cap_tag = 0;
    const int rc_run = run_forward(m, T, B, x, h0, c0, y, hT, cT, ws, (char*)workspace, s);
    m->capturing = false;
    return rc_run;
}

static int run_forward(lstm_t* m, int T, int B, const void* x, const float* h0, const float* c0, float* y, float* hT,
                       float* cT, const Workspace& ws, char* base, hipStream_t s)
{
    const int Dn = m->Dn, L = m->L;
    const int M = T * B;
    const bool bf16 = (m->dtype == LSTM_BF16);
    float* P[2] = {(float*)(base + ws.P_off[0]), (float*)(base + ws.P_off[1])};
    float* XT = (float*)(base + ws.XT_off);
    float* Ybuf[2] = {(float*)(base + ws.Y_off[0]), (float*)(base + ws.Y_off[1])};
    float* cbuf[2] = {(float*)(base + ws.c_off[0]), (float*)(base + ws.c_off[1])};
    uint16_t* Ybf[2] = {(uint16_t*)(base + ws.Yb_off[0]), (uint16_t*)(base + ws.Yb_off[1])};
    uint16_t* hb0 = (uint16_t*)(base + ws.hb0_off);
    unsigned long long* bslots = (unsigned long long*)(base + ws.slot_off);
    bool bslots_clean = false;   // zeroed during this forward (tags then restart at 1)
    int bslots_H = 0;            // width of the layer the region was last laid out for
    unsigned btag = 0;
    uint16_t* hx = (uint16_t*)(base + ws.hx_off);
    unsigned* mflags = (unsigned*)(base + ws.mflag_off);
    bool mflags_clean = false;   // zeroed during this forward (tags then restart at 1)
    int mflags_H = 0;            // width of the layer the flags were last laid out for
    unsigned mtag = 0;
    bool prev_has_bf16 = false;  // the layer below left a bf16 copy of its hidden sequence in Ybf[(l-1)&1]
    m->last_plan.clear();
    if (m->G > 0) return forward_hlstm(m, T, B, x, h0, c0, y, hT, cT, ws, base, s);

    unsigned tag0 = 0;   // base of the tags the next batch-1 launch uses
    auto take_tags = [&](int T_) -> int { return take_b1_tags(m, (unsigned)T_, m->xchg_slots, s, &tag0); };
    // slot count the batch-1 kernel will hold in registers: the trimmed slices where they exist
    auto b1_slots = [](const PackedMat& p) { return p.slots_trim > 0 ? p.slots_trim : p.slots; };
    auto sparse_ok = [&](const LayerDir& w, int H, int D_in, int nl) {
        return w.wx.compressed && w.wh.compressed && (w.wx.ell_val || w.wx.slots_trim) && (w.wh.ell_val || w.wh.slots_trim) &&
               persist_b1_sparse_supported(H, D_in, b1_slots(w.wx), b1_slots(w.wh), nl);
    };
    auto fill_sparse_layer = [&](SparseLayerArgs& a, const LayerDir& w, size_t n, float* yout, int y_ld) {
        if (w.wx.slots_trim > 0) {
            a.ell_val_x = w.wx.ell_val_trim; a.ell_col_x = w.wx.ell_col_trim; a.slots_x = w.wx.slots_trim;
            a.ovf_ptr_x = w.wx.ovf_ptr; a.ovf_ent_x = w.wx.ovf_ent; a.ovf_val_x = w.wx.ovf_val;
        } else {
            a.ell_val_x = w.wx.ell_val; a.ell_col_x = w.wx.ell_col; a.slots_x = w.wx.slots;
        }
        if (w.wh.slots_trim > 0) {
            a.ell_val_h = w.wh.ell_val_trim; a.ell_col_h = w.wh.ell_col_trim; a.slots_h = w.wh.slots_trim;
            a.ovf_ptr_h = w.wh.ovf_ptr; a.ovf_ent_h = w.wh.ovf_ent; a.ovf_val_h = w.wh.ovf_val;
        } else {
            a.ell_val_h = w.wh.ell_val; a.ell_col_h = w.wh.ell_col; a.slots_h = w.wh.slots;
        }
        a.bias = w.bias;
        a.h0 = h0 ? h0 + m->soff(n) : nullptr;   // B == 1 on this path
        a.c0 = c0 ? c0 + m->soff(n) : nullptr;
        a.y = yout; a.y_ld = y_ld;
        a.hT = hT ? hT + m->soff(n) : nullptr;
        a.cT = cT ? cT + m->soff(n) : nullptr;
    };

    for (int l = 0; l < L; ++l) {
        const int H = m->hid(l);
        const int D = m->in_dim(l);
        const void* X = (l == 0) ? x : (prev_has_bf16 ? (const void*)Ybf[(l - 1) & 1] : (const void*)Ybuf[(l - 1) & 1]);
        const bool x_is_bf16 = bf16 && (l == 0 || prev_has_bf16);
        prev_has_bf16 = false;
        float* Yout = (l == L - 1) ? y : Ybuf[l & 1];
        const int y_ld = Dn * H;
        const bool try_persist = (B == 1 && m->plan != LSTM_PLAN_STEPWISE);
        char tag[128];

        // ---- batch 1, row-compressed, two stacked unidirectional layers in one launch (diagonal wavefront)
        if (try_persist && Dn == 1 && l + 1 < L && m->hid(l + 1) == H && sparse_ok(m->ld[l], H, D, 2) &&
            sparse_ok(m->ld[l + 1], H, D, 2)) {
            ProfSpan span(m, s, 1);
            int rc = take_tags(T);
            if (rc != LSTM_OK) return rc;
            SparseStackArgs a{};
            float* Yout2 = (l + 1 == L - 1) ? y : Ybuf[(l + 1) & 1];
            fill_sparse_layer(a.layer[0], m->ld[l], (size_t)l, nullptr, H);
            fill_sparse_layer(a.layer[1], m->ld[l + 1], (size_t)l + 1, Yout2, H);
            a.x = X; a.x_bf16 = x_is_bf16; a.round_x_bf16 = (bf16 && !x_is_bf16); a.D0 = D;
            a.T = T; a.H = H; a.reverse = 0; a.round_h_bf16 = bf16;
            a.xchg = m->xchg; a.tag_base = tag0; a.timeout_flag = m->timeout_flag; a.spin_limit = m->spin_limit;
            HIP_TRY(m, launch_persist_b1_sparse(a, 2, m->waves_per_group, m->launch_mode(), s));
            const bool ovf = m->ld[l].wx.slots_trim || m->ld[l].wh.slots_trim || m->ld[l + 1].wx.slots_trim || m->ld[l + 1].wh.slots_trim;
            std::snprintf(tag, sizeof tag, "l%d+l%d.d0:proj=fused-csr,rec=persist_b1-csr-wavefront%s;", l, l + 1, ovf ? "+ovf" : "");
            m->last_plan += tag;
            ++l;
            continue;
        }

        // ---- decide per direction
        int mode[2] = {0, 0};  // 0 stepwise, 1 persistent sparse (fused), 2 persistent dense fused, 3 persistent dense + projection kernel
        for (int d = 0; d < Dn; ++d) {
            const LayerDir& w = m->ld[(size_t)l * Dn + d];
            if (try_persist) {
                if (w.wh.compressed) mode[d] = sparse_ok(w, H, D, 1) ? 1 : 0;
                else if (persist_b1_dense_fusable(H, D)) mode[d] = 2;
                else if (persist_b1_dense_supported(H)) mode[d] = 3;
            }
            if (m->plan == LSTM_PLAN_PERSISTENT && mode[d] == 0 && B == 1)
                return fail(m, LSTM_ERR_ARG, "lstm_forward: persistent plan not available for this shape");
        }
        // ---- input projection for every timestep (only the modes that need P)
        bool xt_ready = false;
        bool pair_done = false;
        bool proj_q16_used = false;
        {
            // Row-compressed W_x in the quarter-wave form, many input rows, few kept weights: gathers and vector
            // multiply-adds over the kept entries only.  (Bound by LDS bandwidth at 16 bytes per four multiply-adds;
            // the dense product on the matrix cores, which multiplies the zeros too, wins above about a fifth kept.)
            bool q16p = !bf16 && !x_is_bf16 && M >= 64;
            int pslots = 0;
            for (int d = 0; d < Dn && q16p; ++d) {
                const PackedMat& p = m->ld[(size_t)l * Dn + d].wx;
                q16p = mode[d] != 1 && mode[d] != 2 && p.compressed && p.q16_slots > 0 &&
                       (double)p.nnz <= m->sparse_proj_max_density * (double)p.rows * (double)p.cols;
                pslots = std::max(pslots, p.q16_slots);
            }
            if (q16p && proj_q16_supported(M, H, D, pslots)) {
                ProfSpan span(m, s, 0);
                ProjQ16Args a{};
                for (int d = 0; d < Dn; ++d) {
                    const LayerDir& w = m->ld[(size_t)l * Dn + d];
                    a.d[d] = ProjQ16Dir{w.wx.q16_val, w.wx.q16_col, w.wx.q16_slots, w.wx.q16_ovf_ptr, w.wx.q16_ovf_ent,
                                        w.wx.q16_ovf_val, w.bias, P[d]};
                }
                a.X = (const float*)X; a.ldx = D; a.M = M; a.K = D; a.H = H;
                HIP_TRY(m, launch_proj_q16(a, Dn, pslots, s));
                pair_done = true;
                proj_q16_used = true;
            }
        }
        if (!pair_done && Dn == 2 && !bf16 && M > 64 && mode[0] != 1 && mode[0] != 2 && mode[1] != 1 && mode[1] != 2) {
            // fp32, both directions dense on the matrix cores: one launch (they read the same X).  (At most 64 input rows:
            // one stream over the fragment-ordered weights per direction, below.)
            const LayerDir& w0 = m->ld[(size_t)l * Dn], & w1 = m->ld[(size_t)l * Dn + 1];
            auto dense_ok = [&](const LayerDir& w) {
                return w.wx.dense && (!w.wx.compressed || M >= 256) && proj_mfma_supported(false, D, D);
            };
            if (dense_ok(w0) && dense_ok(w1)) {
                ProfSpan span(m, s, 0);
                HIP_TRY(m, launch_proj_mfma_f32_pair((const float*)X, D, (const float*)w0.wx.dense, w0.bias, P[0],
                                                     (const float*)w1.wx.dense, w1.bias, P[1], M, 4 * H, D, s));
                pair_done = true;
            }
        }
        for (int d = 0; d < Dn && !pair_done; ++d) {
            if (mode[d] == 1 || mode[d] == 2) continue;
            const LayerDir& w = m->ld[(size_t)l * Dn + d];
            ProfSpan span(m, s, 0);
            const bool dense_proj = proj_runs_dense(w.wx, M, D, bf16);
            if (!dense_proj && w.wx.ell_val && proj_ell_small_supported(M, 4 * H, D, w.wx.slots)) {
                // few input rows: lanes over the kept entries of a row (no transpose of X)
                HIP_TRY(m, launch_proj_ell_small(X, x_is_bf16, D, bf16 && !x_is_bf16, w.wx.ell_val, w.wx.ell_col, w.wx.slots,
                                                 w.bias, P[d], M, 4 * H, D, s));
            } else if (!dense_proj) {
                if (!xt_ready) {
                    HIP_TRY(m, launch_transpose_to_f32(X, x_is_bf16, D, XT, M, D, bf16 && !x_is_bf16, s));
                    xt_ready = true;
                }
                HIP_TRY(m, launch_proj_csr(XT, w.wx.row_ptr, w.wx.col16, w.wx.val, w.bias, P[d], M, 4 * H, s));
            } else if (proj_mfma_supported(bf16, D, D)) {
                HIP_TRY(m, launch_proj_mfma(X, x_is_bf16, D, w.wx.dense, bf16, w.bias, P[d], M, 4 * H, D, s, bf16 ? nullptr : w.wx.dense_frag16));
            } else {
                HIP_TRY(m, launch_proj_dense(X, x_is_bf16, D, w.wx.dense, bf16, w.bias, P[d], M, 4 * H, D, s));
            }
        }
        // ---- recurrence, bf16 dense at large batch: one matrix-core launch per step with the cell update fused
        bool dense_bf16 = bf16;
        for (int d = 0; d < Dn; ++d) dense_bf16 = dense_bf16 && mode[d] == 0 && !m->ld[(size_t)l * Dn + d].wh.compressed;
        const bool mfma_ok = dense_bf16 && step_mfma_supported(B, H);
        if (dense_bf16 && m->plan != LSTM_PLAN_STEPWISE && persist_mfma_supported(B, H)) {
            // time loop on the device: W_h stays in registers, h_t travels through flagged exchange buffers
            uint16_t* Yb = Ybf[l & 1];
            if (!mflags_clean || mflags_H != H) {
                HIP_TRY(m, launch_fill_f32((float*)mflags, persist_mfma_flag_count(B, H), 0.0f, s));
                mflags_clean = true;
                mflags_H = H;
                mtag = 0;
            }
            for (int d = 0; d < Dn; ++d) {
                const LayerDir& w = m->ld[(size_t)l * Dn + d];
                const size_t n = (size_t)l * Dn + d;
                ProfSpan span(m, s, 1);
                PersistMfmaArgs a{};
                a.P = P[d];
                a.Wh = (const uint16_t*)w.wh.dense;
                a.c0 = c0 ? c0 + m->soff(n) * B : nullptr;
                // the layer above reads the bf16 copy; only the last layer's fp32 sequence leaves the library
                a.y = (l == L - 1) ? Yout + (size_t)d * H : nullptr;
                a.y_ld = y_ld;
                a.yb = (l == L - 1) ? nullptr : Yb + (size_t)d * H;
                a.yb_ld = y_ld;
                a.hT = hT ? hT + m->soff(n) * B : nullptr;
                a.cT = cT ? cT + m->soff(n) * B : nullptr;
                a.hx = hx;
                a.flags = mflags;
                a.xcc_ids = (unsigned long long*)(mflags + persist_mfma_ids_offset(B, H));
                a.tag_base = mtag;
                a.timeout_flag = m->timeout_flag;
                a.spin_limit = m->spin_limit; a.device_scope_only = m->device_scope_only;
                a.T = T; a.B = B; a.H = H; a.reverse = d;
                mtag += (unsigned)T;
                std::snprintf(tag, sizeof tag, "l%d.d%d:proj=dense,rec=persist-mfma-bf16;", l, d);
                m->last_plan += tag;
                HIP_TRY(m, launch_persist_mfma_bf16(a, h0 ? h0 + m->soff(n) * B : nullptr, m->launch_mode() != 0, s));
            }
            prev_has_bf16 = true;
            continue;
        }
        if (mfma_ok) {
            uint16_t* Yb = Ybf[l & 1];
            for (int d = 0; d < Dn; ++d) {
                const LayerDir& w = m->ld[(size_t)l * Dn + d];
                const size_t n = (size_t)l * Dn + d;
                ProfSpan span(m, s, 1);
                if (c0) HIP_TRY(m, hipMemcpyAsync(cbuf[d], c0 + m->soff(n) * B, (size_t)B * H * sizeof(float), hipMemcpyDeviceToDevice, s));
                else HIP_TRY(m, launch_fill_f32(cbuf[d], (size_t)B * H, 0.0f, s));
                uint16_t* hb0d = hb0 + (size_t)d * B * H;
                if (h0) HIP_TRY(m, launch_f32_to_bf16(h0 + m->soff(n) * B, H, hb0d, H, B, H, s));
                std::snprintf(tag, sizeof tag, "l%d.d%d:proj=dense,rec=stepwise-mfma-bf16;", l, d);
                m->last_plan += tag;
                for (int step = 0; step < T; ++step) {
                    const int t = d ? (T - 1 - step) : step;
                    StepMfmaArgs a{};
                    a.P = P[d];
                    a.Wh = (const uint16_t*)w.wh.dense;
                    if (step == 0) {
                        a.hb_prev = h0 ? hb0d : nullptr;
                        a.hb_prev_ld = H;
                    } else {
                        const int tp = d ? t + 1 : t - 1;
                        a.hb_prev = Yb + (size_t)tp * B * y_ld + (size_t)d * H;
                        a.hb_prev_ld = y_ld;
                    }
                    a.c = cbuf[d];
                    a.y_t = Yout + (size_t)t * B * y_ld + (size_t)d * H;
                    a.y_ld = y_ld;
                    a.hb_t = Yb + (size_t)t * B * y_ld + (size_t)d * H;
                    a.hb_ld = y_ld;
                    a.hT = hT ? hT + m->soff(n) * B : nullptr;
                    a.cT = cT ? cT + m->soff(n) * B : nullptr;
                    a.last = (step == T - 1);
                    a.t = t;
                    a.B = B;
                    a.H = H;
                    HIP_TRY(m, launch_step_mfma_bf16(a, s));
                }
            }
            prev_has_bf16 = true;
            continue;
        }
        // ---- recurrence, fp32 dense at small and medium batch, time loop on the device (all directions in one launch):
        // W_h as matrix-instruction operand fragments in registers, h_t through flagged exchange buffers
        {
            bool dense_f32 = !bf16 && B >= 2 && m->plan != LSTM_PLAN_STEPWISE;
            for (int d = 0; d < Dn; ++d) {
                const LayerDir& w = m->ld[(size_t)l * Dn + d];
                dense_f32 = dense_f32 && mode[d] == 0 && !w.wh.compressed && w.wh.dense;
            }
            LaunchCut cut;
            if (dense_f32 && choose_cut(B, Dn, [&](int b, int nd) { return persist_dense_f32_supported(b, H, nd); }, &cut)) {
                for (int launch = 0; launch < cut.passes * cut.chunks; ++launch) {
                    const int pass = launch / cut.chunks, chunk = launch % cut.chunks;
                    const int nd = Dn / cut.passes, d_lo = pass * nd;
                    const int b_lo = chunk_begin(B, cut.chunks, chunk), bn = chunk_begin(B, cut.chunks, chunk + 1) - b_lo;
                    // the exchange buffers start every launch with all stamps clear
                    HIP_TRY(m, launch_fill_f32((float*)hx, persist_dense_f32_exchange_floats(bn, H, nd), 0.0f, s));
                    PersistDenseArgs a{};
                    const float* h0d[2] = {nullptr, nullptr};
                    for (int d = d_lo; d < d_lo + nd; ++d) {
                        const LayerDir& w = m->ld[(size_t)l * Dn + d];
                        const size_t n = (size_t)l * Dn + d;
                        const size_t so = m->soff(n) * B + (size_t)b_lo * H;
                        PersistDenseDir& q = a.d[d - d_lo];
                        q.P = P[d] + (size_t)b_lo * 4 * H;
                        q.Wh = (const float*)w.wh.dense;
                        q.c0 = c0 ? c0 + so : nullptr;
                        q.y = Yout + (size_t)b_lo * y_ld + (size_t)d * H; q.y_ld = y_ld;
                        q.hT = hT ? hT + so : nullptr;
                        q.cT = cT ? cT + so : nullptr;
                        q.reverse = d;
                        h0d[d - d_lo] = h0 ? h0 + so : nullptr;
                        if (chunk == 0) {
                            char cuts[24] = "";
                            if (cut.chunks > 1) std::snprintf(cuts, sizeof cuts, "(batch/%d)", cut.chunks);
                            std::snprintf(tag, sizeof tag, "l%d.d%d:proj=%s,rec=persist-dense-f32%s;", l, d,
                                          proj_runs_dense(w.wx, M, D, bf16) ? "dense" : "csr", cuts);
                            m->last_plan += tag;
                        }
                    }
                    a.hx = (float*)hx;
                    if (!mflags_clean) {
                        HIP_TRY(m, launch_fill_u64((unsigned long long*)mflags, persist_dense_f32_ids_count(), 0ull, s));
                        mflags_clean = true;
                        mtag = 0;
                    }
                    a.xcc_ids = (unsigned long long*)mflags;
                    a.tag_base = mtag++;
                    a.device_scope_only = m->device_scope_only;
                    a.timeout_flag = m->timeout_flag; a.spin_limit = m->spin_limit;
                    a.T = T; a.B = bn; a.Bld = B; a.H = H; a.ndir = nd;
                    a.poll_pace = m->poll_pace >= 0 ? m->poll_pace : (H <= 512 ? kPollPaceDenseNarrow : kPollPaceDenseWide);
                    ProfSpan span(m, s, 1);
                    HIP_TRY(m, launch_persist_dense_f32(a, h0d, m->launch_mode() != 0, s));
                }
                continue;
            }
        }
        // ---- recurrence, small-batch row-compressed, time loop on the device (all directions in one launch): W_h in
        // the quarter-wave form (rows of at most 256 kept entries)
        {
            int upw = 0, bw = 0, ug = 0, bg = 0, q16 = 0;
            bool pb_ok = B >= 2 && m->plan != LSTM_PLAN_STEPWISE;
            for (int d = 0; d < Dn && pb_ok; ++d) {
                const PackedMat& p = m->ld[(size_t)l * Dn + d].wh;
                pb_ok = p.compressed && p.q16_slots > 0;
                q16 = std::max(q16, p.q16_slots);
            }
            LaunchCut cut;
            pb_ok = pb_ok && choose_cut(B, Dn, [&](int b, int nd) { return persist_batched_q16_plan(b, H, q16, nd, &upw, &bw, &ug, &bg); }, &cut);
            if (pb_ok) {
                if (!bslots_clean || bslots_H != H) {   // another width is another layout: start from zero again
                    HIP_TRY(m, launch_fill_u64(bslots, align256(ws.slot_bytes) / sizeof(unsigned long long), 0ull, s));
                    bslots_clean = true;
                    bslots_H = H;
                    btag = 0;
                }
                for (int launch = 0; launch < cut.passes * cut.chunks; ++launch) {
                const int pass = launch / cut.chunks, chunk = launch % cut.chunks;
                const int nd = Dn / cut.passes, d_lo = pass * nd;
                const int b_lo = chunk_begin(B, cut.chunks, chunk), bn = chunk_begin(B, cut.chunks, chunk + 1) - b_lo;
                persist_batched_q16_plan(bn, H, q16, nd, &upw, &bw, &ug, &bg);
                PersistBatchedArgs a{};
                for (int d = d_lo; d < d_lo + nd; ++d) {
                    const LayerDir& w = m->ld[(size_t)l * Dn + d];
                    const size_t n = (size_t)l * Dn + d;
                    PersistBatchedDir& q = a.d[d - d_lo];
                    q.P = P[d] + (size_t)b_lo * 4 * H;
                    q.q16_val = w.wh.q16_val; q.q16_col = w.wh.q16_col; q.q16_slots = w.wh.q16_slots;
                    q.q16_ovf_ptr = w.wh.q16_ovf_ptr; q.q16_ovf_ent = w.wh.q16_ovf_ent; q.q16_ovf_val = w.wh.q16_ovf_val;
                    const size_t so = m->soff(n) * B + (size_t)b_lo * H;
                    q.h0 = h0 ? h0 + so : nullptr;
                    q.c0 = c0 ? c0 + so : nullptr;
                    q.y = Yout + (size_t)b_lo * y_ld + (size_t)d * H; q.y_ld = y_ld;
                    q.hT = hT ? hT + so : nullptr;
                    q.cT = cT ? cT + so : nullptr;
                    q.reverse = d;
                    if (chunk == 0) {
                        char cuts[24] = "";
                        if (cut.chunks > 1) std::snprintf(cuts, sizeof cuts, ",batch/%d", cut.chunks);
                        std::snprintf(tag, sizeof tag, "l%d.d%d:proj=%s,rec=persist_batched-q16%s(s%d,u%d,b%d%s);", l, d,
                                      proj_q16_used ? "q16" : proj_runs_dense(w.wx, M, D, bf16) ? "dense" : "csr",
                                      w.wh.q16_ovf_ptr ? "+ovf" : "", q16, upw, bw, cuts);
                        m->last_plan += tag;
                    }
                }
                a.T = T; a.B = bn; a.Bld = B; a.H = H; a.round_h_bf16 = bf16;
                a.xchg = bslots; a.xcc_ids = bslots + (size_t)Dn * 2 * (B + 3) * H; a.tag_base = btag; a.timeout_flag = m->timeout_flag; a.spin_limit = m->spin_limit; a.device_scope_only = m->device_scope_only;
                a.poll_pace = m->poll_pace >= 0 ? m->poll_pace : kPollPaceBatchedDeviceWide;   // (the launcher clears it where the exchange stays inside XCDs)
                btag += (unsigned)T;
                ProfSpan span(m, s, 1);
                HIP_TRY(m, launch_persist_batched_q16(a, nd, q16, m->launch_mode(), s));
                }
                continue;
            }
        }
        // ---- recurrence, small-batch row-compressed: every direction of the layer advances in the same launch
        bool pair_ok = true;
        for (int d = 0; d < Dn; ++d) {
            const LayerDir& w = m->ld[(size_t)l * Dn + d];
            pair_ok = pair_ok && mode[d] == 0 && w.wh.compressed && w.wh.ell_val && step_csr_pair_supported(H, w.wh.slots);
        }
        if (pair_ok) {
            const float* ev[2] = {nullptr, nullptr};
            const uint16_t* ec[2] = {nullptr, nullptr};
            int sl[2] = {0, 0};
            ProfSpan span(m, s, 1);
            for (int d = 0; d < Dn; ++d) {
                const LayerDir& w = m->ld[(size_t)l * Dn + d];
                const size_t n = (size_t)l * Dn + d;
                ev[d] = w.wh.ell_val; ec[d] = w.wh.ell_col; sl[d] = w.wh.slots;
                if (c0) HIP_TRY(m, hipMemcpyAsync(cbuf[d], c0 + m->soff(n) * B, (size_t)B * H * sizeof(float), hipMemcpyDeviceToDevice, s));
                else HIP_TRY(m, launch_fill_f32(cbuf[d], (size_t)B * H, 0.0f, s));
                std::snprintf(tag, sizeof tag, "l%d.d%d:proj=%s,rec=stepwise-csr-paired;", l, d,
                              proj_q16_used ? "q16" : proj_runs_dense(w.wx, M, D, bf16) ? "dense" : "csr");
                m->last_plan += tag;
            }
            for (int step = 0; step < T; ++step) {
                StepArgs a[2] = {};
                for (int d = 0; d < Dn; ++d) {
                    const size_t n = (size_t)l * Dn + d;
                    const int t = d ? (T - 1 - step) : step;
                    a[d].P = P[d];
                    if (step == 0) {
                        a[d].h_prev = h0 ? h0 + m->soff(n) * B : nullptr;
                        a[d].h_prev_ld = H;
                    } else {
                        const int tp = d ? t + 1 : t - 1;
                        a[d].h_prev = Yout + (size_t)tp * B * y_ld + (size_t)d * H;
                        a[d].h_prev_ld = y_ld;
                    }
                    a[d].c = cbuf[d];
                    a[d].y_t = Yout + (size_t)t * B * y_ld + (size_t)d * H;
                    a[d].y_ld = y_ld;
                    a[d].hT = hT ? hT + m->soff(n) * B : nullptr;
                    a[d].cT = cT ? cT + m->soff(n) * B : nullptr;
                    a[d].last = (step == T - 1);
                    a[d].t = t;
                    a[d].B = B;
                    a[d].H = H;
                    a[d].round_h_bf16 = bf16 ? 1 : 0;
                }
                HIP_TRY(m, launch_step_csr_pair(a, ev, ec, sl, Dn, s));
            }
            continue;
        }
        // ---- recurrence
        for (int d = 0; d < Dn; ++d) {
            const LayerDir& w = m->ld[(size_t)l * Dn + d];
            const size_t n = (size_t)l * Dn + d;
            const float* h0n = h0 ? h0 + m->soff(n) * B : nullptr;
            const float* c0n = c0 ? c0 + m->soff(n) * B : nullptr;
            float* hTn = hT ? hT + m->soff(n) * B : nullptr;
            float* cTn = cT ? cT + m->soff(n) * B : nullptr;
            static const char* const names[4] = {"stepwise", "persist_b1", "persist_b1", "persist_b1"};
            std::snprintf(tag, sizeof tag, "l%d.d%d:proj=%s%s,rec=%s-%s%s;", l, d, (mode[d] == 1 || mode[d] == 2) ? "fused-" : "",
                          proj_q16_used ? "q16" : ((mode[d] == 1 || mode[d] == 2) ? !w.wx.compressed : proj_runs_dense(w.wx, M, D, bf16)) ? "dense" : "csr",
                          names[mode[d]], w.wh.compressed ? "csr" : "dense",
                          (mode[d] == 1 && (w.wx.slots_trim || w.wh.slots_trim)) ? "+ovf" : "");
            m->last_plan += tag;
            ProfSpan span(m, s, 1);
            if (mode[d] == 1) {
                int rc = take_tags(T);
                if (rc != LSTM_OK) return rc;
                SparseStackArgs a{};
                fill_sparse_layer(a.layer[0], w, n, Yout + (size_t)d * H, y_ld);
                a.x = X; a.x_bf16 = x_is_bf16; a.round_x_bf16 = (bf16 && !x_is_bf16); a.D0 = D;
                a.T = T; a.H = H; a.reverse = d; a.round_h_bf16 = bf16;
                a.xchg = m->xchg + (size_t)d * 2 * H; a.tag_base = tag0;
                a.timeout_flag = m->timeout_flag; a.spin_limit = m->spin_limit;
                HIP_TRY(m, launch_persist_b1_sparse(a, 1, m->waves_per_group, m->launch_mode(), s));
            } else if (mode[d] == 2 || mode[d] == 3) {
                int rc = take_tags(T);
                if (rc != LSTM_OK) return rc;
                PersistB1Args a{};
                a.Wh = w.wh.dense; a.w_bf16 = bf16;
                if (mode[d] == 2) {
                    a.Wx = w.wx.dense; a.bias = w.bias; a.x = X; a.x_bf16 = x_is_bf16;
                    a.round_x_bf16 = (bf16 && !x_is_bf16); a.D = D;
                } else {
                    a.P = P[d];
                }
                a.h0 = h0n; a.c0 = c0n;
                a.y = Yout + (size_t)d * H; a.y_ld = y_ld;
                a.hT = hTn; a.cT = cTn;
                a.T = T; a.H = H; a.reverse = d; a.round_h_bf16 = bf16;
                a.xchg = m->xchg + (size_t)d * 2 * H; a.xcc_ids = m->xchg + (size_t)4 * H; a.tag_base = tag0;
                a.timeout_flag = m->timeout_flag; a.spin_limit = m->spin_limit; a.device_scope_only = m->device_scope_only;
                HIP_TRY(m, launch_persist_b1_dense(a, m->waves_per_group, m->launch_mode(), s));
            } else {
                const size_t state_bytes = (size_t)B * H * sizeof(float);
                if (c0n)
                    HIP_TRY(m, hipMemcpyAsync(cbuf[d], c0n, state_bytes, hipMemcpyDeviceToDevice, s));
                else
                    HIP_TRY(m, launch_fill_f32(cbuf[d], (size_t)B * H, 0.0f, s));
                for (int step = 0; step < T; ++step) {
                    const int t = d ? (T - 1 - step) : step;
                    StepArgs a{};
                    a.P = P[d];
                    if (step == 0) {
                        a.h_prev = h0n;
                        a.h_prev_ld = H;
                    } else {
                        const int tp = d ? t + 1 : t - 1;
                        a.h_prev = Yout + (size_t)tp * B * y_ld + (size_t)d * H;
                        a.h_prev_ld = y_ld;
                    }
                    a.c = cbuf[d];
                    a.y_t = Yout + (size_t)t * B * y_ld + (size_t)d * H;
                    a.y_ld = y_ld;
                    a.hT = hTn;
                    a.cT = cTn;
                    a.last = (step == T - 1);
                    a.t = t;
                    a.B = B;
                    a.H = H;
                    a.round_h_bf16 = bf16 ? 1 : 0;
                    if (w.wh.compressed)
                        HIP_TRY(m, launch_step_csr(a, w.wh.row_ptr, w.wh.col16, w.wh.val, s));
                    else
                        HIP_TRY(m, launch_step_dense(a, w.wh.dense, bf16, s));
                }
            }
        }
    }
    return LSTM_OK;
}

int lstm_check(lstm_t* m)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_check: handle is NULL");
    int flag = 0;
    HIP_TRY(m, hipMemcpy(&flag, m->timeout_flag, sizeof(int), hipMemcpyDeviceToHost));
    if (flag) {
        HIP_TRY(m, hipMemset(m->timeout_flag, 0, sizeof(int)));
        for (auto& x : m->ld) x.u_dirty = true;   // steps were abandoned half-way: the stamped words hold either parity
        return fail(m, LSTM_ERR_TIMEOUT, "a bounded device-side wait expired; outputs of that forward are invalid");
    }
    return LSTM_OK;
}

int lstm_get_compressed(const lstm_t* m, int layer, int direction, int which, int64_t* nnz, int64_t* row_ptr,
                        int32_t* col, float* val)
{
    if (!m) return fail(nullptr, LSTM_ERR_ARG, "lstm_get_compressed: handle is NULL");
    if (layer < 0 || layer >= m->L || direction < 0 || direction >= m->Dn || which < 0 || which > (m->G > 0 ? 2 : 1))
        return fail(m, LSTM_ERR_SHAPE, "lstm_get_compressed: index outside the model");
    const LayerDir& x = m->ld[(size_t)layer * m->Dn + direction];
    const PackedMat& p = which == 2 ? x.w2 : (which ? x.wh : x.wx);
    if (!x.set || !p.compressed) return fail(m, LSTM_ERR_STATE, "lstm_get_compressed: matrix not held in compressed form");
    if (nnz) *nnz = p.nnz;
    if (!row_ptr && !col && !val) return LSTM_OK;
    if (!row_ptr || !col || !val) return fail(m, LSTM_ERR_ARG, "lstm_get_compressed: pass all of row_ptr, col, val or none");
    // translate packed row order (4j+q) back to the ABI order (q*H + j); the hidden layers of an H-LSTM have G units
    const int H = (m->G > 0 && which != 2) ? m->ghid(layer) : m->hid(layer);
    int64_t pos = 0;
    for (int r = 0; r < 4 * H; ++r) {
        const int rp = 4 * (r % H) + (r / H);
        row_ptr[r] = pos;
        for (int64_t e = p.h_row_ptr[rp]; e < p.h_row_ptr[rp + 1]; ++e, ++pos) {
            col[pos] = p.h_col[e];
            val[pos] = p.h_val[e];
        }
    }
    row_ptr[4 * H] = pos;
    return LSTM_OK;
}

int lstm_find_lhp(const int* dims, const double* lat, int n, double eps, uint8_t* is_lhp, double* redundancy_pct)
{
    if (n < 0 || (n > 0 && (!dims || !lat || !is_lhp)) || !(eps >= 0.0) || eps >= 1.0)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_find_lhp: bad arguments");
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return dims[a] > dims[b]; });
    // walk from the largest dimension down, carrying the best latency among strictly larger dimensions
    double best_larger = INFINITY;
    int count = 0;
    size_t i = 0;
    while (i < order.size()) {
        size_t jn = i;
        double group_best = INFINITY;
        while (jn < order.size() && dims[order[jn]] == dims[order[i]]) {
            const int idx = order[jn];
            const bool lhp = std::isinf(best_larger) ? true : (lat[idx] < (1.0 - eps) * best_larger);
            is_lhp[idx] = lhp ? 1 : 0;
            count += lhp ? 1 : 0;
            group_best = std::min(group_best, lat[idx]);
            ++jn;
        }
        best_larger = std::min(best_larger, group_best);
        i = jn;
    }
    if (redundancy_pct) *redundancy_pct = n ? (1.0 - (double)count / n) * 100.0 : 0.0;
    return LSTM_OK;
}

// ---- latency sweep -----------------------------------------------------------------------------------------
namespace {
struct SplitMix {
    uint64_t s;
    uint64_t next() { uint64_t z = (s += 0x9E3779B97F4A7C15ull); z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
                      z = (z ^ (z >> 27)) * 0x94D049BB133111EBull; return z ^ (z >> 31); }
    double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
    double normal() { double u1 = uniform(), u2 = uniform(); if (u1 < 1e-300) u1 = 1e-300;
                      return std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586 * u2); }
};
double percentile(std::vector<double> v, double p)
{
    std::sort(v.begin(), v.end());
    if (v.empty()) return 0.0;
    const double pos = p * (v.size() - 1);
    const size_t lo = (size_t)pos;
    const size_t hi = std::min(lo + 1, v.size() - 1);
    return v[lo] + (v[hi] - v[lo]) * (pos - lo);
}
}  // namespace

int lstm_latency_sweep_model(const int* Hs, const int* Ds, int n, int layers, int bidirectional, int gate_hidden,
                             double keep, int T, int B, int dtype, uint64_t seed, int warmup, int iters,
                             double* med_us, double* p10_us, double* p90_us, uint8_t* is_lhp, void* stream)
{
    if (n < 0 || (n > 0 && (!Hs || !med_us)) || layers < 1 || (bidirectional != 0 && bidirectional != 1) || T < 1 ||
        B < 1 || warmup < 0 || iters < 1 || !(keep >= 0.0) || keep > 1.0 || (gate_hidden != 0 && gate_hidden != 1))
        return fail(nullptr, LSTM_ERR_ARG, "lstm_latency_sweep_model: bad arguments");
    const bool masked = keep > 0.0 && keep < 1.0;
    const int Dn = bidirectional ? 2 : 1;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    HIP_TRY(nullptr, hipEventCreate(&e0));
    HIP_TRY(nullptr, hipEventCreate(&e1));
    int rc = LSTM_OK;
    for (int idx = 0; idx < n && rc == LSTM_OK; ++idx) {
        const int H = Hs[idx], D0 = Ds ? Ds[idx] : H, G = gate_hidden ? H : 0;
        lstm_t* m = nullptr;
        rc = G ? lstm_create_h(layers, D0, H, G, bidirectional, dtype, &m) : lstm_create(layers, D0, H, bidirectional, dtype, &m);
        if (rc != LSTM_OK) break;
        SplitMix rng{seed + 0x1000ull * (uint64_t)idx};
        auto draw = [&](std::vector<float>& W, std::vector<uint8_t>& M, size_t count) {
            W.resize(count);
            for (auto& v : W) v = (float)(0.2 * rng.uniform() - 0.1);
            M.clear();
            if (masked) {
                M.resize(count);
                for (auto& v : M) v = rng.uniform() < keep ? 1 : 0;
            }
        };
        std::vector<float> A, Bm, C, b1, b2;
        std::vector<uint8_t> MA, MB, MC;
        for (int l = 0; l < layers && rc == LSTM_OK; ++l) {
            const int D = l == 0 ? D0 : Dn * H;
            for (int d = 0; d < Dn && rc == LSTM_OK; ++d) {
                if (G) {
                    draw(A, MA, (size_t)4 * G * D);
                    draw(Bm, MB, (size_t)4 * G * H);
                    draw(C, MC, (size_t)4 * H * G);
                    b1.assign((size_t)4 * G, 0.0f);
                    b2.assign((size_t)4 * H, 0.0f);
                    for (int j = 0; j < H; ++j) b2[j] = 1.0f;
                    rc = lstm_set_weights_h(m, l, d, A.data(), masked ? MA.data() : nullptr, Bm.data(), masked ? MB.data() : nullptr,
                                            b1.data(), C.data(), masked ? MC.data() : nullptr, b2.data(), LSTM_FMT_AUTO);
                } else {
                    draw(A, MA, (size_t)4 * H * D);
                    draw(Bm, MB, (size_t)4 * H * H);
                    b1.assign((size_t)4 * H, 0.0f);
                    for (int j = 0; j < H; ++j) b1[j] = 1.0f;
                    rc = lstm_set_weights(m, l, d, A.data(), masked ? MA.data() : nullptr, Bm.data(), masked ? MB.data() : nullptr,
                                          b1.data(), masked ? LSTM_FMT_AUTO : LSTM_FMT_DENSE_MASKED);
                }
                if (rc != LSTM_OK) g_create_error = lstm_last_error(m);
            }
        }
        void *dx = nullptr, *dy = nullptr, *dws = nullptr;
        const size_t xelems = (size_t)T * B * D0, yelems = (size_t)T * B * Dn * H;
        const size_t wsb = rc == LSTM_OK ? lstm_workspace_bytes(m, T, B) : 0;
        hipError_t e = hipSuccess;
        if (rc == LSTM_OK) {
            std::vector<float> xf(xelems);
            for (auto& v : xf) v = (float)rng.normal();
            if (dtype == LSTM_BF16) {
                std::vector<uint16_t> xb(xelems);
                for (size_t i = 0; i < xelems; ++i) xb[i] = host_f32_to_bf16(xf[i]);
                e = hipMalloc(&dx, xelems * 2);
                if (e == hipSuccess) e = hipMemcpy(dx, xb.data(), xelems * 2, hipMemcpyHostToDevice);
            } else {
                e = hipMalloc(&dx, xelems * 4);
                if (e == hipSuccess) e = hipMemcpy(dx, xf.data(), xelems * 4, hipMemcpyHostToDevice);
            }
            if (e == hipSuccess) e = hipMalloc(&dy, yelems * 4);
            if (e == hipSuccess) e = hipMalloc(&dws, wsb);
            if (e != hipSuccess) rc = fail_hip(nullptr, e, "lstm_latency_sweep_model: device buffers");
        }
        std::vector<double> times;
        for (int it = 0; it < warmup + iters && rc == LSTM_OK; ++it) {
            e = hipEventRecord(e0, s);
            rc = lstm_forward(m, T, B, dx, nullptr, nullptr, (float*)dy, nullptr, nullptr, dws, wsb, s);
            if (rc != LSTM_OK) { g_create_error = lstm_last_error(m); break; }
            if (e == hipSuccess) e = hipEventRecord(e1, s);
            if (e == hipSuccess) e = hipEventSynchronize(e1);
            float ms = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
            if (e != hipSuccess) { rc = fail_hip(nullptr, e, "lstm_latency_sweep_model: timing"); break; }
            if (it >= warmup) times.push_back((double)ms * 1000.0);
        }
        if (rc == LSTM_OK) {
            rc = lstm_check(m);
            if (rc != LSTM_OK) g_create_error = lstm_last_error(m);
        }
        if (rc == LSTM_OK) {
            med_us[idx] = percentile(times, 0.5);
            if (p10_us) p10_us[idx] = percentile(times, 0.1);
            if (p90_us) p90_us[idx] = percentile(times, 0.9);
        }
        if (dx) (void)hipFree(dx);
        if (dy) (void)hipFree(dy);
        if (dws) (void)hipFree(dws);
        lstm_destroy(m);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == LSTM_OK && is_lhp && n > 0) rc = lstm_find_lhp(Hs, med_us, n, 0.0, is_lhp, nullptr);
    return rc;
}

int lstm_latency_sweep(const int* Hs, int nH, int T, int B, int dtype, uint64_t seed, int warmup, int iters,
                       double* med_us, double* p10_us, double* p90_us, uint8_t* is_lhp, void* stream)
{
    return lstm_latency_sweep_model(Hs, nullptr, nH, 1, 0, 0, 0.0, T, B, dtype, seed, warmup, iters, med_us, p10_us,
                                    p90_us, is_lhp, stream);
}

int lstm_grow_to_lhp(const int* dims, const double* lat, int n, double eps, int from_dim, int* target_dim,
                     double* latency_gain_pct)
{
    if (n < 1 || !dims || !lat || !target_dim || !(eps >= 0.0) || eps >= 1.0)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_grow_to_lhp: bad arguments");
    std::vector<uint8_t> flags((size_t)n);
    const int rc = lstm_find_lhp(dims, lat, n, eps, flags.data(), nullptr);
    if (rc != LSTM_OK) return rc;
    // the smallest measured hysteresis point that is not below from_dim
    int best = -1;
    for (int i = 0; i < n; ++i)
        if (flags[i] && dims[i] >= from_dim && (best < 0 || dims[i] < dims[best])) best = i;
    if (best < 0) return fail(nullptr, LSTM_ERR_ARG, "lstm_grow_to_lhp: from_dim is above every measured dimension");
    *target_dim = dims[best];
    if (latency_gain_pct) {
        // against the smallest measured dimension that is not below from_dim (from_dim itself when it was measured)
        int ref = -1;
        for (int i = 0; i < n; ++i)
            if (dims[i] >= from_dim && (ref < 0 || dims[i] < dims[ref])) ref = i;
        *latency_gain_pct = (1.0 - lat[best] / lat[ref]) * 100.0;
    }
    return LSTM_OK;
}

int lstm_prune_weights(const float* W, uint8_t* mask, size_t count, double p_w, size_t* kept_before, size_t* kept_after,
                       void* stream)
{
    if (!W || !mask || count == 0 || count > ((size_t)1 << 32) - 2 || !(p_w >= 0.0) || p_w > 1.0)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_prune_weights: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    unsigned* keys = nullptr;
    char* small = nullptr;   // state | two counters
    const size_t st_bytes = align256(prune_state_bytes());
    hipError_t e = hipMalloc((void**)&keys, count * sizeof(unsigned));
    if (e == hipSuccess) e = hipMalloc((void**)&small, st_bytes + 256);
    unsigned long long host_cnt[2] = {0, 0};
    if (e == hipSuccess) e = launch_prune_weights(W, mask, count, p_w, keys, small, (unsigned long long*)(small + st_bytes), s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipMemcpy(host_cnt, small + st_bytes, sizeof host_cnt, hipMemcpyDeviceToHost);
    if (keys) (void)hipFree(keys);
    if (small) (void)hipFree(small);
    if (e != hipSuccess) return fail_hip(nullptr, e, "lstm_prune_weights");
    if (kept_before) *kept_before = (size_t)host_cnt[0];
    if (kept_after) *kept_after = (size_t)host_cnt[1];
    return LSTM_OK;
}

int lstm_prune_rows_cols(float* W, uint8_t* mask, int M, int N, double p_r, double p_c, int* rows_removed,
                         int* cols_removed, void* stream)
{
    if (!W || !mask || M < 1 || N < 1 || (long long)M * N > (1ll << 31) || !(p_r >= 0.0) || p_r > 1.0 || !(p_c >= 0.0) ||
        p_c > 1.0)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_prune_rows_cols: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    const unsigned kr = (unsigned)std::min<double>(std::ceil(p_r * M), M), kc = (unsigned)std::min<double>(std::ceil(p_c * N), N);
    char* scratch = nullptr;
    int* removed = nullptr;
    int host_removed[2] = {0, 0};
    hipError_t e = hipMalloc((void**)&scratch, prune_rows_cols_scratch_bytes(M, N));
    if (e == hipSuccess) e = launch_prune_rows_cols(W, mask, M, N, kr, kc, scratch, &removed, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipMemcpy(host_removed, removed, sizeof host_removed, hipMemcpyDeviceToHost);
    if (scratch) (void)hipFree(scratch);
    if (e != hipSuccess) return fail_hip(nullptr, e, "lstm_prune_rows_cols");
    if (rows_removed) *rows_removed = host_removed[0];
    if (cols_removed) *cols_removed = host_removed[1];
    return LSTM_OK;
}

int lstm_prune_rows_cols_static(float* W, uint8_t* mask, int M, int N, double p_r, double p_c, int* removed, void* stream)
{
    if (!W || !mask || M < 1 || N < 1 || !(p_r >= 0.0) || p_r > 1.0 || !(p_c >= 0.0) || p_c > 1.0)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_prune_rows_cols_static: bad arguments");
    const int cap = prune_rows_cols_static_max_lines();
    if (M > cap || N > cap) {
        char msg[160];
        std::snprintf(msg, sizeof msg, "lstm_prune_rows_cols_static: M = %d, N = %d exceed the fixed scratch (at most %d rows and %d columns)",
                      M, N, cap, cap);
        return fail(nullptr, LSTM_ERR_ARG, msg);
    }
    const unsigned kr = (unsigned)std::min<double>(std::ceil(p_r * M), M), kc = (unsigned)std::min<double>(std::ceil(p_c * N), N);
    const hipError_t e = launch_prune_rows_cols_static(W, mask, M, N, kr, kc, removed, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(nullptr, e, "lstm_prune_rows_cols_static");
    return LSTM_OK;
}

int lstm_compact_rows_cols(const float* W, const uint8_t* mask, int gates, int R, int N, int32_t* row_index, int32_t* col_index,
                           float* Wc, uint8_t* mask_c, int* Rc, int* Nc, void* stream)
{
    if (!W || !mask || !row_index || !col_index || !Wc || !Rc || !Nc || gates < 1 || R < 1 || N < 1 ||
        (long long)gates * R > (1ll << 31) / N)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_compact_rows_cols: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    char* scratch = nullptr;
    int* counts = nullptr;
    int host_counts[2] = {0, 0};
    hipError_t e = hipMalloc((void**)&scratch, compact_scratch_bytes(gates, R, N));
    if (e == hipSuccess) e = launch_compact_rows_cols(W, mask, gates, R, N, row_index, col_index, Wc, mask_c, scratch, &counts, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipMemcpy(host_counts, counts, sizeof host_counts, hipMemcpyDeviceToHost);
    if (scratch) (void)hipFree(scratch);
    if (e != hipSuccess) return fail_hip(nullptr, e, "lstm_compact_rows_cols");
    *Rc = host_counts[0];
    *Nc = host_counts[1];
    return LSTM_OK;
}

int lstm_bench_matmul(int n, int batch, double keep, int format, uint64_t seed, int iters, const float* X_host,
                      const float* W_host, const uint8_t* mask_host, double* avg_us, float* y_host, void* stream)
{
    const bool given = X_host || W_host || mask_host;
    if (n < 4 || n > 65536 || (n & 3) || batch < 1 || batch > 4096 || iters < 1 || !avg_us ||
        (format != LSTM_FMT_DENSE_MASKED && format != LSTM_FMT_ROW_COMPRESSED) || (given && (!X_host || !W_host)) ||
        (!given && (!(keep > 0.0) || keep > 1.0)))
        return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_matmul: bad arguments (n must be a multiple of 4; X and W come together)");
    hipStream_t s = (hipStream_t)stream;
    SplitMix rng{seed};
    const size_t nn = (size_t)n * n;
    if (mask_host)
        for (size_t i = 0; i < nn; ++i)
            if (mask_host[i] > 1) return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_matmul: mask byte not in {0,1}");
    std::vector<float> W(nn), X((size_t)batch * n), bias((size_t)n, 0.0f);
    if (given) std::copy(X_host, X_host + X.size(), X.begin());
    else for (auto& v : X) v = (float)rng.normal();
    std::vector<int32_t> rp((size_t)n + 1, 0);
    std::vector<uint16_t> col;
    std::vector<float> val;
    for (int r = 0; r < n; ++r) {
        for (int k = 0; k < n; ++k) {
            float w;
            bool kept;
            if (given) {
                // the mask selects: what lies under a zero byte is never read into the product
                kept = !mask_host || mask_host[(size_t)r * n + k] != 0;
                w = kept ? W_host[(size_t)r * n + k] : 0.0f;
            } else {
                w = (float)(0.2 * rng.uniform() - 0.1);
                kept = keep >= 1.0 || rng.uniform() < keep;
            }
            W[(size_t)r * n + k] = kept ? w : 0.0f;
            if (kept && format == LSTM_FMT_ROW_COMPRESSED) { col.push_back((uint16_t)k); val.push_back(w); }
        }
        rp[(size_t)r + 1] = (int32_t)col.size();
    }
    // 64-lane slices of the kept entries (entry e of a row in slice e / 64, lane e % 64), used when the input batch is
    // small enough for the lanes-over-entries projection
    int slots = 1;
    for (int r = 0; r < n && format == LSTM_FMT_ROW_COMPRESSED; ++r) slots = std::max(slots, (rp[(size_t)r + 1] - rp[r] + 63) / 64);
    const bool use_ell = format == LSTM_FMT_ROW_COMPRESSED && proj_ell_small_supported(batch, n, n, slots);
    std::vector<float> ev;
    std::vector<uint16_t> ec;
    if (use_ell) {
        ev.assign((size_t)n * slots * 64, 0.0f);
        ec.assign((size_t)n * slots * 64, 0);
        for (int r = 0; r < n; ++r)
            for (int e = rp[r]; e < rp[(size_t)r + 1]; ++e) {
                ev[(size_t)r * slots * 64 + (size_t)(e - rp[r])] = val[(size_t)e];
                ec[(size_t)r * slots * 64 + (size_t)(e - rp[r])] = col[(size_t)e];
            }
    }
    float *dX = nullptr, *dW = nullptr, *dWf = nullptr, *dB = nullptr, *dY = nullptr, *dXT = nullptr, *dval = nullptr, *dev_ = nullptr;
    int32_t* drp = nullptr;
    uint16_t *dcol = nullptr, *dec = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = LSTM_OK;
    auto run = [&]() -> hipError_t {
        if (use_ell) return launch_proj_ell_small(dX, false, n, false, dev_, dec, slots, dB, dY, batch, n, n, s);
        if (format == LSTM_FMT_ROW_COMPRESSED) {
            hipError_t e = launch_transpose_to_f32(dX, false, n, dXT, batch, n, false, s);
            if (e != hipSuccess) return e;
            return launch_proj_csr(dXT, drp, dcol, dval, dB, dY, batch, n, s);
        }
        if (proj_mfma_supported(false, n, n)) return launch_proj_mfma(dX, false, n, dW, false, dB, dY, batch, n, n, s, dWf);
        return launch_proj_dense(dX, false, n, dW, false, dB, dY, batch, n, n, s);
    };
    hipError_t e = upload(&dX, X);
    if (e == hipSuccess) e = upload(&dB, bias);
    if (e == hipSuccess) e = hipMalloc((void**)&dY, (size_t)batch * n * sizeof(float));
    if (e == hipSuccess && use_ell) {
        e = upload(&dev_, ev);
        if (e == hipSuccess) e = upload(&dec, ec);
    } else if (e == hipSuccess && format == LSTM_FMT_ROW_COMPRESSED) {
        e = upload(&drp, rp);
        if (e == hipSuccess) e = upload(&dcol, col);
        if (e == hipSuccess) e = upload(&dval, val);
        if (e == hipSuccess) e = hipMalloc((void**)&dXT, (size_t)batch * n * sizeof(float));
    } else if (e == hipSuccess) {
        e = upload(&dW, W);
        // as lstm_set_weights stores an input-side matrix: once more in fragment order, for batches of at most 64 rows
        if (e == hipSuccess && batch <= 64) e = upload(&dWf, to_frag16(W.data(), n, n));
    }
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    for (int i = 0; i < 3 && e == hipSuccess; ++i) e = run();
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    for (int i = 0; i < iters && e == hipSuccess; ++i) e = run();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess && y_host) e = hipMemcpy(y_host, dY, (size_t)batch * n * sizeof(float), hipMemcpyDeviceToHost);
    if (e != hipSuccess) rc = fail_hip(nullptr, e, "lstm_bench_matmul");
    else *avg_us = (double)ms * 1000.0 / iters;
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    for (void* p_ : {(void*)dX, (void*)dW, (void*)dWf, (void*)dB, (void*)dY, (void*)dXT, (void*)dval, (void*)drp, (void*)dcol, (void*)dev_, (void*)dec})
        if (p_) (void)hipFree(p_);
    return rc;
}

int lstm_bench_copy(void* dst, const void* src, size_t bytes, int iters, double* avg_us, void* stream)
{
    if (!dst || !src || !avg_us || iters < 1 || bytes == 0 || (bytes & 15))
        return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_copy: bad arguments (bytes must be a multiple of 16)");
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    HIP_TRY(nullptr, hipEventCreate(&e0));
    HIP_TRY(nullptr, hipEventCreate(&e1));
    HIP_TRY(nullptr, launch_copy_stream(dst, src, bytes, s));
    HIP_TRY(nullptr, hipEventRecord(e0, s));
    for (int i = 0; i < iters; ++i) HIP_TRY(nullptr, launch_copy_stream(dst, src, bytes, s));
    HIP_TRY(nullptr, hipEventRecord(e1, s));
    HIP_TRY(nullptr, hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(nullptr, hipEventElapsedTime(&ms, e0, e1));
    *avg_us = (double)ms * 1000.0 / iters;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return LSTM_OK;
}

int lstm_bench_mfma(int dtype, int random_operands, int reps, int iters, double* tflops, double* clock_ghz, void* stream)
{
    if ((dtype != LSTM_F32 && dtype != LSTM_BF16) || reps < 1 || iters < 1 || !tflops ||
        (random_operands != 0 && random_operands != 1))
        return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_mfma: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    float* sink = nullptr;
    long long* clocks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    double flops = 0.0;
    const int blocks = mfma_issue_blocks();
    const bool bf16 = dtype == LSTM_BF16, rnd = random_operands != 0;
    hipError_t e = hipMalloc((void**)&sink, mfma_issue_sink_floats() * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&clocks, (size_t)blocks * 2 * sizeof(long long));
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) e = launch_mfma_issue(bf16, rnd, sink, clocks, reps, &flops, s);      // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    for (int i = 0; i < iters && e == hipSuccess; ++i) e = launch_mfma_issue(bf16, rnd, sink, clocks, reps, &flops, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    std::vector<long long> h((size_t)blocks * 2, 0);
    if (e == hipSuccess) e = hipMemcpy(h.data(), clocks, h.size() * sizeof(long long), hipMemcpyDeviceToHost);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (clocks) (void)hipFree(clocks);
    if (e != hipSuccess) return fail_hip(nullptr, e, "lstm_bench_mfma");
    *tflops = flops * iters / ((double)ms * 1e-3) / 1e12;
    if (clock_ghz) {
        double cyc = 0.0, ticks = 0.0;
        for (int i = 0; i < blocks; ++i) { cyc += (double)h[2 * (size_t)i]; ticks += (double)h[2 * (size_t)i + 1]; }
        *clock_ghz = ticks > 0.0 ? cyc / (ticks * 10.0) : 0.0;    // shader cycles per 10 ns tick of the 100 MHz counter
    }
    return LSTM_OK;
}

int lstm_bench_barrier(int workgroups, int waves, int steps, int iters, int cooperative, double* avg_us_per_step, void* stream)
{
    if (workgroups < 1 || workgroups > 256 || workgroups > device_num_cus() || waves < 1 || waves > 16 || steps < 2 ||
        iters < 1 || !avg_us_per_step)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_barrier: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    unsigned long long* slots = nullptr;
    int* flag = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipMalloc((void**)&slots, (size_t)2 * workgroups * 8);
    if (e == hipSuccess) e = hipMemset(slots, 0, (size_t)2 * workgroups * 8);
    if (e == hipSuccess) e = hipMalloc((void**)&flag, 4);
    if (e == hipSuccess) e = hipMemset(flag, 0, 4);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    unsigned tag = 0;
    int pace = 0;
    auto run = [&]() {
        const hipError_t r = launch_barrier_only(slots, tag, workgroups, waves, steps, flag, 1u << 22, pace, cooperative, s);
        tag += (unsigned)steps;
        return r;
    };
    float ms = 0.f;
    for (int p : kYardstickPaces) {   // the fastest pacing of the poll is the yardstick
        pace = p;
        if (e == hipSuccess) e = run();
        if (e == hipSuccess) e = hipEventRecord(e0, s);
        for (int i = 0; i < iters && e == hipSuccess; ++i) e = run();
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms1 = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms1, e0, e1);
        if (e == hipSuccess && (ms == 0.f || ms1 < ms)) ms = ms1;
    }
    int f = 0;
    if (e == hipSuccess) e = hipMemcpy(&f, flag, 4, hipMemcpyDeviceToHost);
    int rc = LSTM_OK;
    if (e != hipSuccess) rc = fail_hip(nullptr, e, "lstm_bench_barrier");
    else if (f) rc = fail(nullptr, LSTM_ERR_TIMEOUT, "lstm_bench_barrier: bounded wait expired");
    else *avg_us_per_step = (double)ms * 1000.0 / iters / steps;
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (slots) (void)hipFree(slots);
    if (flag) (void)hipFree(flag);
    return rc;
}

int lstm_bench_exchange(int hidden, int waves, int steps, int iters, int cooperative, double* avg_us_per_step, void* stream)
{
    if (hidden < 1 || hidden > 8192 || waves < 0 || waves > 16 || steps < 2 || iters < 1 || !avg_us_per_step)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_exchange: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    unsigned long long* xchg = nullptr;
    int* flag = nullptr;
    HIP_TRY(nullptr, hipMalloc((void**)&xchg, (size_t)2 * hidden * 8));
    HIP_TRY(nullptr, hipMemset(xchg, 0, (size_t)2 * hidden * 8));
    HIP_TRY(nullptr, hipMalloc((void**)&flag, 4));
    HIP_TRY(nullptr, hipMemset(flag, 0, 4));
    hipEvent_t e0, e1;
    HIP_TRY(nullptr, hipEventCreate(&e0));
    HIP_TRY(nullptr, hipEventCreate(&e1));
    unsigned tag = 0;
    int rc = LSTM_OK;
    hipError_t e = hipSuccess;
    float ms = 0.f;
    for (int pace : kYardstickPaces) {   // the fastest pacing of the poll is the yardstick
        if (e == hipSuccess) e = launch_exchange_only(xchg, tag, hidden, waves, steps, flag, 1u << 22, pace, cooperative, s);
        tag += (unsigned)steps;
        if (e == hipSuccess) e = hipEventRecord(e0, s);
        for (int i = 0; i < iters && e == hipSuccess; ++i) {
            e = launch_exchange_only(xchg, tag, hidden, waves, steps, flag, 1u << 22, pace, cooperative, s);
            tag += (unsigned)steps;
        }
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms1 = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms1, e0, e1);
        if (e == hipSuccess && (ms == 0.f || ms1 < ms)) ms = ms1;
    }
    int f = 0;
    if (e == hipSuccess) e = hipMemcpy(&f, flag, 4, hipMemcpyDeviceToHost);
    if (e != hipSuccess) rc = fail_hip(nullptr, e, "lstm_bench_exchange");
    else if (f) rc = fail(nullptr, LSTM_ERR_TIMEOUT, "lstm_bench_exchange: bounded wait expired");
    else *avg_us_per_step = (double)ms * 1000.0 / iters / steps;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(xchg);
    (void)hipFree(flag);
    return rc;
}

int lstm_bench_group_exchange(int slots, int members, int groups, int placed, int workgroup_stores, int steps, int iters,
                              int cooperative, double* avg_us_per_round, int* groups_verified, void* stream)
{
    if (slots < 1 || slots > 16384 || members < 1 || members > 64 || groups < 1 || groups > 64 || steps < 2 || iters < 1 ||
        !avg_us_per_round || (long long)groups * members > device_num_cus())
        return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_group_exchange: bad arguments");
    if (placed && ((groups + 7) / 8) * members > device_num_cus() / 8)
        return fail(nullptr, LSTM_ERR_ARG, "lstm_bench_group_exchange: the groups of one XCD do not fit its compute units");
    hipStream_t s = (hipStream_t)stream;
    const size_t nslot = (size_t)groups * 2 * slots + (size_t)groups * 64;
    unsigned long long* buf = nullptr;
    int* small = nullptr;   // timeout flag | verified count
    HIP_TRY(nullptr, hipMalloc((void**)&buf, nslot * 8));
    hipError_t e = hipMemset(buf, 0, nslot * 8);
    if (e == hipSuccess) e = hipMalloc((void**)&small, 8);
    if (e == hipSuccess) e = hipMemset(small, 0, 8);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    unsigned tag = 0;
    auto run = [&]() {
        hipError_t r = launch_group_exchange(buf, buf + (size_t)groups * 2 * slots, tag, slots, members, groups, placed,
                                             workgroup_stores, steps, small, 1u << 22, small + 1, cooperative, s);
        tag += (unsigned)steps + 1u;
        return r;
    };
    if (e == hipSuccess) e = run();                       // warm-up, also the one whose verified count is reported
    int host_small[2] = {0, 0};
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipMemcpy(host_small, small, 8, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    for (int i = 0; i < iters && e == hipSuccess; ++i) e = run();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    int f = 0;
    if (e == hipSuccess) e = hipMemcpy(&f, small, 4, hipMemcpyDeviceToHost);
    int rc = LSTM_OK;
    if (e != hipSuccess) rc = fail_hip(nullptr, e, "lstm_bench_group_exchange");
    else if (f) rc = fail(nullptr, LSTM_ERR_TIMEOUT, "lstm_bench_group_exchange: bounded wait expired");
    else {
        *avg_us_per_round = (double)ms * 1000.0 / iters / steps;
        if (groups_verified) *groups_verified = host_small[1];
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (buf) (void)hipFree(buf);
    if (small) (void)hipFree(small);
    return rc;
}

}  // extern "C"
