// LSTM / GRU inference over a sequence (Sec. 2.1) with CSB-pruned weights.
//
// Two device paths behind csb_rnn_forward:
//
//  * resident (batch 1, after csb_rnn_upload): ONE kernel launch runs all T steps of all
//    layers.  The pruned weights are read from HBM once and stay in registers (the paper
//    likewise loads weights on chip once before frames stream, Sec. 6.1); every
//    workgroup owns a range of hidden units with all their gate rows, so the gate
//    arithmetic needs no second pass.  A row's non-zeros are cut into equal slices of S
//    entries, one slice per lane (the equal-work split that Sec. 5.2 obtains from its
//    compiler), slices of a row are summed through LDS in a fixed order, and h_t travels
//    between workgroups as 64-bit (tag, value) words that readers poll, so no grid-wide
//    barrier and no cache flush sits on the step's critical path.
//
//  * streaming (any batch): per step and layer one CSB mat-vec launch plus one gate
//    kernel, all enqueued on the stream without host synchronisation.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "csb_internal.hpp"
#include "csb_kernels.hpp"

namespace csb {

constexpr int kRnnThreads = 1024;      // lanes per workgroup of the resident kernel
constexpr int kRnnSlotsMax = 48;       // weights one lane keeps in registers
constexpr int kRnnMaxLayers = 8;       // model layers of a resident layout (more: streaming path)
constexpr int kRnnWgsPerXcd = 28;      // workgroups placed on one XCD (32 CUs, one workgroup per CU, a few CUs spare)
constexpr int kRnnMaxWgs = 8 * kRnnWgsPerXcd;   // all workgroups must be co-resident
// Per-phase shader clocks of the resident kernel (a development aid): compiled in only on
// request, so that the time loop of the shipped kernel carries none of it.
#ifdef CSB_RNN_PHASE_CLOCKS
constexpr bool kPhaseClocks = true;
#else
constexpr bool kPhaseClocks = false;
#endif

// The resident kernel works on a stack of stages.  An LSTM / GRU layer is one stage (its
// units' gate rows); an LSTMP layer is two: the gate stage, whose output m_t is not state, and
// a linear stage (the projection r_t = Wp m_t), whose output is the layer's state h and the
// gate stage's recurrent input.  A layer of the GRU with the reset gate before the candidate's
// recurrent product is two as well: the reset stage (row r over [u ; h_(t-1)], output
// q_t = r h_(t-1)) and the gate stage (row z over [u ; h_(t-1)], row n over u and over q_t, which
// it takes from the reset stage at the same step as a third input; output h_t).
constexpr uint32_t kStageLstm = 0, kStageGru = 1, kStageLinear = 2, kStageLiGru = 3, kStageGruRbReset = 4, kStageGruRbGate = 5;
constexpr int kRnnReps = 3;              // z entries a thread stages: C <= kRnnReps * kRnnThreads
constexpr uint32_t kStageOwnRec = 1;     // flag: the recurrent input is this stage's own output
constexpr uint32_t kStageIsState = 2;    // flag: the output is the layer's h state (h0 / hT)
constexpr uint32_t kStageIsSeq = 4;      // flag: the output is the model's output sequence
constexpr uint32_t kNoStage = 0xffffffffu;

// One workgroup of the resident kernel.
struct RnnWgRec {
    uint32_t aux;             // owner-table offset of a third input stage (same step, behind the recurrent input), or kNoStage
    uint32_t u0, nu;          // units [u0, u0 + nu) of the stage
    uint32_t off_zpos;        // byte offset of the z permutation: u16 position in LDS of every input entry [C]
    uint32_t S;               // slots per lane
    uint32_t n_in, C;         // width of the input from below, C = n_in + width of the recurrent input (+ width of the third)
    uint32_t off_rows;        // byte offset of the lane table: 1024 words (segment position, flags, row slot)
    uint32_t off_w;           // byte offset of weights  [S][1024] float
    uint32_t off_z;           // byte offset of z indices [S][1024] u16
    uint32_t upre;            // units owned by the workgroups before this one (all stages)
    uint32_t kind;            // stage kind | model layer << 8 | flags << 16
    uint32_t below;           // owner-table offset of the stage below, kNoStage = the input sequence x
    uint32_t rec;             // owner-table offset of the stage the recurrent input comes from, or kNoStage
    uint32_t width;           // units of this stage
    uint32_t rec_width;       // units of the recurrent source (row length of h0 for it)
};
static_assert(sizeof(RnnWgRec) == 64, "RnnWgRec layout");

struct RnnPlan {
    bool valid = false;
    int n_wgs = 0, smax = 0;
    std::vector<uint8_t> image;
    size_t off_unit_wg = 0;    // u16 per unit of every stage: the workgroup that owns it
    size_t total_units = 0;    // units of all stages (exchange words per time step)
    size_t cmax = 0;           // largest C of any stage (LDS sizing)
    double slot_fill = 0;      // non-zeros / (1024 * S * workgroups): the useful share of issued multiply-adds
    double lanes_max_over_mean = 0;
    size_t total_nnz = 0;      // surviving weights of the whole model
    long lds_conflicts = 0;    // words that share an LDS bank with another word of the same 32-lane gather (all workgroups)
};

}  // namespace csb

struct csb_rnn {
    int32_t cell = 0, n_layers = 0, input = 0, hidden = 0;
    int32_t proj = 0;                      // LSTMP: width of the recurrent projection (the state h is this wide)
    std::vector<csb_matrix *> W;
    std::vector<csb_matrix *> Wp;          // LSTMP: projection matrices, proj x hidden
    int32_t state_width() const { return proj > 0 ? proj : hidden; }
    std::vector<const float *> d_bias;
    csb::RnnPlan plan;
    void *d_img = nullptr;
    bool uploaded = false;
    mutable const void *ws_seen = nullptr;
    mutable uint32_t ws_gen = 0xffffffffu;
    mutable size_t ws_words = 0;             // exchange words cleared there so far
    mutable int64_t ws_use = -1;             // batch and path of the last forward call (they fix what lies where)
    // tuning knobs, read from the environment once, when the handle is created
    int32_t knob_xcds = 0;                   // CSB_RNN_XCDS: use at least this many XCDs (0: as few as hold the model)
    // The launches of the last streaming call (batch 1, row-owned plans: kernel launches only) as a
    // HIP graph: a call that repeats its predecessor's arguments records them, later ones replay.
    mutable hipGraphExec_t fwd_exec = nullptr;
    mutable hipStream_t fwd_cap = nullptr;                       // the stream the launches are recorded on
    mutable std::vector<uint64_t> fwd_key, fwd_last;             // arguments the graph was made for / of the last call
    mutable bool fwd_failed = false;                             // recording did not work here once: not tried again
    bool knob_graph = true;                  // CSB_RNN_GRAPH=0: every call enqueues its launches itself
    int32_t knob_poll_delay = -1;            // CSB_RNN_POLL_DELAY: sleeps before the first poll of a step (-1: default)
    int32_t knob_batch_path = 0;             // CSB_RNN_BATCH_PATH: 1 resident, 2 batched, 0 by estimate
    uint32_t poll_limit = 1u << 24;          // polls of one exchange word before the resident kernel gives up
    double clock_mhz = 2400.0;               // shader clock of the device the handle was created on (the path estimate uses it)
    csb_rnn() {
        int dev = 0, khz = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) == hipSuccess && khz > 0)
            clock_mhz = khz / 1000.0;
        (void)hipGetLastError();             // (no device: the default stands)
        if (const char *e = getenv("CSB_RNN_XCDS")) knob_xcds = std::min(8, std::max(1, atoi(e)));
        if (const char *e = getenv("CSB_RNN_POLL_DELAY")) knob_poll_delay = std::max(0, atoi(e));
        if (const char *e = getenv("CSB_RNN_GRAPH")) knob_graph = atoi(e) != 0;
        if (const char *e = getenv("CSB_RNN_BATCH_PATH")) knob_batch_path = !strcmp(e, "resident") ? 1 : !strcmp(e, "batched") ? 2 : 0;
    }
    ~csb_rnn() {
        // (a recorded sequence may still be running for a caller who frees early: let it finish first)
        if (fwd_exec) { (void)hipDeviceSynchronize(); (void)hipGraphExecDestroy(fwd_exec); }
        if (fwd_cap) (void)hipStreamDestroy(fwd_cap);
    }
    csb_rnn(const csb_rnn &) = delete;
    csb_rnn &operator=(const csb_rnn &) = delete;
};

namespace csb {

// Row r of layer l as (column, value) pairs in column order, after the GRU relabelling:
// virtual row v in [0, 4H): LSTM v = row; GRU v < 2H = row, 2H..3H = n rows restricted to
// input columns, 3H..4H = n rows restricted to recurrent columns.
static void gather_rows(const csb_matrix *m, int cell, int H, int n_in,
                        std::vector<std::vector<std::pair<uint32_t, float>>> &rows) {
    rows.assign((size_t)4 * H, {});
    for (int32_t bi = 0; bi < m->nbr; ++bi)
        for (int32_t bj = 0; bj < m->nbc; ++bj) {
            const size_t b = (size_t)bi * m->nbc + bj;
            const int nr = m->nrows[b], nc = m->ncols[b];
            for (int a = 0; a < nr; ++a) {
                const int64_t gr = (int64_t)bi * m->br + m->rowidx[m->row_off[b] + a];
                for (int q = 0; q < nc; ++q) {
                    const int64_t gc = (int64_t)bj * m->bc + m->colidx[m->col_off[b] + q];
                    int64_t v = gr;
                    if (cell == CSB_CELL_GRU && gr >= 2 * (int64_t)H && gc >= n_in) v = gr + H;
                    rows[(size_t)v].emplace_back((uint32_t)gc, m->val[m->val_off[b] + (size_t)a * nc + q]);
                }
            }
        }
    // blocks are visited in block-column order per block-row, so each row is already sorted
}

// Places row segments (k lanes each, k <= 32) into 16-lane rows of a workgroup: a segment
// of at most 16 lanes lies inside one row; a longer one starts on an even row, fills it and
// continues on the odd row after it.  First-fit decreasing.  Returns the number of 16-lane
// rows used; place[i] = first lane of segment i (-1 for k = 0).
static int pack_segments(const std::vector<int> &k, std::vector<int> *place) {
    std::vector<int> order(k.size());
    for (size_t i = 0; i < k.size(); ++i) order[i] = (int)i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return k[a] > k[b]; });
    std::vector<int> fill;                               // lanes used per 16-lane row
    if (place) place->assign(k.size(), -1);
    for (int i : order) {
        const int ki = k[i];
        if (ki <= 0) continue;
        if (ki > 16) {
            if (fill.size() & 1) fill.push_back(0);      // start on an even row
            if (place) (*place)[i] = (int)fill.size() * 16;
            fill.push_back(16);
            fill.push_back(ki - 16);
        } else {
            size_t r = fill.size();
            for (size_t q = 0; q < fill.size(); ++q) if (fill[q] + ki <= 16) { r = q; break; }
            if (r == fill.size()) fill.push_back(0);
            if (place) (*place)[i] = (int)r * 16 + fill[r];
            fill[r] += ki;
        }
    }
    return (int)fill.size();
}

// Rows of a projection matrix (P x H) as a linear stage: unit u has the single row u.
static void gather_linear_rows(const csb_matrix *m, int width,
                               std::vector<std::vector<std::pair<uint32_t, float>>> &rows) {
    rows.assign((size_t)4 * width, {});
    for (int32_t bi = 0; bi < m->nbr; ++bi)
        for (int32_t bj = 0; bj < m->nbc; ++bj) {
            const size_t b = (size_t)bi * m->nbc + bj;
            const int nr = m->nrows[b], nc = m->ncols[b];
            for (int a = 0; a < nr; ++a) {
                const int64_t gr = (int64_t)bi * m->br + m->rowidx[m->row_off[b] + a];
                for (int q = 0; q < nc; ++q)
                    rows[(size_t)gr].emplace_back((uint32_t)((int64_t)bj * m->bc + m->colidx[m->col_off[b] + q]),
                                                  m->val[m->val_off[b] + (size_t)a * nc + q]);
            }
        }
}

// Rows [row0, row0 + nrows) of a matrix appended to rows[dst_row0 + (row - row0)], their columns
// shifted by col_shift (entries arrive in column order per call).
static void append_rows(const csb_matrix *m, int row0, int nrows, int dst_row0, int col_shift,
                        std::vector<std::vector<std::pair<uint32_t, float>>> &rows) {
    for (int32_t bi = 0; bi < m->nbr; ++bi)
        for (int32_t bj = 0; bj < m->nbc; ++bj) {
            const size_t b = (size_t)bi * m->nbc + bj;
            const int nr = m->nrows[b], nc = m->ncols[b];
            for (int a = 0; a < nr; ++a) {
                const int64_t gr = (int64_t)bi * m->br + m->rowidx[m->row_off[b] + a];
                if (gr < row0 || gr >= (int64_t)row0 + nrows) continue;
                for (int q = 0; q < nc; ++q)
                    rows[(size_t)(dst_row0 + gr - row0)].emplace_back(
                        (uint32_t)((int64_t)bj * m->bc + m->colidx[m->col_off[b] + q] + col_shift),
                        m->val[m->val_off[b] + (size_t)a * nc + q]);
            }
        }
}

// `slots` > 0: that many slots per lane in every stage; 0: per stage whatever the step-time
// model below favours for one sequence.
static int build_resident_plan(csb_rnn *r, int slots = 0) {
    RnnPlan &pl = r->plan;
    pl = RnnPlan{};
    const bool lstmp = r->cell == CSB_CELL_LSTMP, gru_rb = r->cell == CSB_CELL_GRU_RB;
    const int NL = r->n_layers, L = (lstmp || gru_rb) ? 2 * NL : NL;      // L stages
    if (NL > kRnnMaxLayers) return CSB_EUNSUPPORTED;                      // the kernel takes that many bias pointers
    struct LayerTmp {
        std::vector<std::vector<std::pair<uint32_t, float>>> rows;
        int n_in, C, S, P;
        int width;                  // units of the stage
        uint32_t kind, real, flags;
        int below, rec, aux = -1;   // stage indices, -1 = x / none
        std::vector<int> u_cut;     // unit ranges per workgroup
    };
    std::vector<LayerTmp> lt(L);
    size_t total_nnz = 0;
    for (int l = 0; l < L; ++l) {
        LayerTmp &t = lt[l];
        if (gru_rb) {
            const int lam = l / 2, H = r->hidden;
            t.width = H; t.real = (uint32_t)lam;
            t.n_in = lam == 0 ? r->input : H;
            t.below = lam == 0 ? -1 : 2 * lam - 1;           // the gate stage of the layer below
            t.rows.assign((size_t)4 * H, {});
            if ((l & 1) == 0) {                              // reset stage: row r
                t.kind = kStageGruRbReset;
                t.C = t.n_in + H; t.rec = l + 1; t.flags = 0;
                append_rows(r->W[lam], 0, H, 0, 0, t.rows);
            } else {                                         // gate stage: rows z and n
                t.kind = kStageGruRbGate;
                t.C = t.n_in + 2 * H; t.rec = l; t.aux = l - 1;
                t.flags = kStageOwnRec | kStageIsState | (l == L - 1 ? kStageIsSeq : 0u);
                append_rows(r->W[lam], H, 2 * H, 0, 0, t.rows);          // z, n (input side) -> rows 0..2H
                append_rows(r->Wp[lam], 0, H, H, t.n_in + H, t.rows);    // Un -> the n rows, columns behind h
            }
        } else if (!lstmp) {
            t.width = r->hidden; t.real = (uint32_t)l;
            t.kind = r->cell == CSB_CELL_LSTM ? kStageLstm : (r->cell == CSB_CELL_LIGRU ? kStageLiGru : kStageGru);
            t.n_in = l == 0 ? r->input : r->hidden;
            t.C = t.n_in + r->hidden;
            t.below = l - 1; t.rec = l;
            t.flags = kStageOwnRec | kStageIsState | (l == L - 1 ? kStageIsSeq : 0u);
            gather_rows(r->W[l], r->cell, r->hidden, t.n_in, t.rows);
        } else if ((l & 1) == 0) {                       // gate stage of model layer l / 2
            t.width = r->hidden; t.real = (uint32_t)(l / 2); t.kind = kStageLstm;
            t.n_in = l == 0 ? r->input : r->proj;
            t.C = t.n_in + r->proj;
            t.below = l - 1; t.rec = l + 1;
            t.flags = 0;
            gather_rows(r->W[l / 2], CSB_CELL_LSTM, r->hidden, t.n_in, t.rows);
        } else {                                         // projection stage
            t.width = r->proj; t.real = (uint32_t)(l / 2); t.kind = kStageLinear;
            t.n_in = r->hidden; t.C = r->hidden;
            t.below = l - 1; t.rec = -1;
            t.flags = kStageIsState | (l == L - 1 ? kStageIsSeq : 0u);
            gather_linear_rows(r->Wp[l / 2], r->proj, t.rows);
        }
        if (t.C > kRnnReps * kRnnThreads || t.n_in > 2 * kRnnThreads) return CSB_EUNSUPPORTED;   // z entries a thread stages
        pl.cmax = std::max<size_t>(pl.cmax, (size_t)t.C);
        for (auto &row : t.rows) total_nnz += row.size();
    }
    // Slots per lane S and workgroups per layer.  A row's non-zeros are cut into k slices of
    // S entries, one lane each; the k lanes sit inside one aligned 32-lane half of a wavefront
    // so that the row sum is a shift-and-add inside the wavefront (k <= 32 fixes the smallest S).  Units are
    // laid out one after another (their four rows in a row), workgroups take contiguous
    // unit ranges, and the largest number of 16-lane rows per workgroup is minimised.
    constexpr int kSeg = 32;                       // lanes one row's slices may span
    constexpr int kBins = kRnnThreads / 16;        // 16-lane rows per workgroup
    int s_lo = 4, s_hi = kRnnSlotsMax;
    if (const char *e = getenv("CSB_RNN_S")) s_lo = s_hi = std::max(4, std::min(kRnnSlotsMax, atoi(e) / 4 * 4));
    if (slots > 0) s_lo = s_hi = std::max(4, std::min(kRnnSlotsMax, slots / 4 * 4));
    int total_wgs = 0;
    for (int l = 0; l < L; ++l) {
        LayerTmp &t = lt[l];
        const int H = t.width;                    // units of this stage
        size_t max_nnz = 0;
        for (auto &row : t.rows) max_nnz = std::max(max_nnz, row.size());
        double best_cost = 1e30;
        for (int S = s_lo; S <= s_hi; S += 4) {
            if ((max_nnz + S - 1) / S > (size_t)kSeg) continue;
            auto kof = [&](int g, int u) { return (int)((t.rows[(size_t)g * H + u].size() + S - 1) / S); };
            // exact number of 16-lane rows of a unit range
            auto pack = [&](int u0, int u1, std::vector<int> *place) {
                std::vector<int> ks((size_t)4 * (u1 - u0));
                for (int u = u0; u < u1; ++u)
                    for (int g = 0; g < 4; ++g) ks[(size_t)g * (u1 - u0) + (u - u0)] = kof(g, u);
                return pack_segments(ks, place);
            };
            std::vector<long> pre(H + 1, 0);
            for (int u = 0; u < H; ++u) { pre[u + 1] = pre[u]; for (int g = 0; g < 4; ++g) pre[u + 1] += kof(g, u); }
            auto fill_wgs = [&](int cap, std::vector<int> *cut) {
                int used = 0, u = 0;
                if (cut) cut->assign(1, 0);
                while (u < H) {
                    ++used;
                    int u1 = u + 1;
                    while (u1 < H && u1 - u < kRnnThreads / 4 && pre[u1 + 1] - pre[u] <= (long)cap * 16) ++u1;
                    while (u1 > u + 1 && pack(u, u1, nullptr) > cap) --u1;
                    if (pack(u, u1, nullptr) > kBins) return 1 << 20;           // one unit alone does not fit
                    if (cut) cut->push_back(u1);
                    u = u1;
                }
                return used;
            };
            const int P = fill_wgs(kBins, nullptr);
            if (P > kRnnMaxWgs) continue;
            // step-time model (shader clocks): S gathers per lane at ~100 clocks each for a full
            // workgroup, plus the exchange of h_t when more than one workgroup takes part
            const double cost = 60.0 * S + (P > 1 || L > 1 ? 1700.0 : 0.0) + 6.0 * P;
            if (cost >= best_cost) continue;
            int lo = 1, hi = kBins;
            while (lo < hi) {
                const int mid = (lo + hi) / 2;
                if (fill_wgs(mid, nullptr) <= P) hi = mid; else lo = mid + 1;
            }
            fill_wgs(lo, &t.u_cut);
            t.S = S; t.P = (int)t.u_cut.size() - 1;
            best_cost = cost;
        }
        if (best_cost >= 1e30) return CSB_EUNSUPPORTED;
        total_wgs += t.P;
    }
    if (total_wgs > kRnnMaxWgs) return CSB_EUNSUPPORTED;

    // image: workgroup records, then per workgroup the lane table and the slot arrays
    std::vector<RnnWgRec> wgs;
    std::vector<uint8_t> body;
    auto align = [&](size_t a) { while (body.size() % a) body.push_back(0); };
    size_t slots_total = 0;
    uint32_t upre_run = 0;
    std::vector<size_t> uoff(L + 1, 0);                      // owner-table offset of every stage
    for (int l = 0; l < L; ++l) uoff[l + 1] = uoff[l] + (size_t)lt[l].width;
    std::vector<uint16_t> unit_wg(uoff[L], 0);
    pl.total_units = uoff[L];
    int smax = 0;
    long conflicts_total = 0;
    double lanes_max = 0, lanes_sum = 0;
    for (int l = 0; l < L; ++l) {
        const LayerTmp &t = lt[l];
        const int H = t.width;
        smax = std::max(smax, t.S);
        for (int p = 0; p < t.P; ++p) {
            RnnWgRec w{};
            w.aux = t.aux < 0 ? kNoStage : (uint32_t)uoff[t.aux]; w.u0 = (uint32_t)t.u_cut[p]; w.nu = (uint32_t)(t.u_cut[p + 1] - t.u_cut[p]);
            w.S = (uint32_t)t.S; w.n_in = (uint32_t)t.n_in; w.C = (uint32_t)t.C;
            w.upre = upre_run; upre_run += w.nu;
            w.kind = t.kind | t.real << 8 | t.flags << 16;
            w.below = t.below < 0 ? kNoStage : (uint32_t)uoff[t.below];
            w.rec = t.rec < 0 ? kNoStage : (uint32_t)uoff[t.rec];
            w.width = (uint32_t)t.width;
            w.rec_width = t.rec < 0 ? 0u : (uint32_t)lt[t.rec].width;
            for (uint32_t ui = 0; ui < w.nu; ++ui) unit_wg[uoff[l] + w.u0 + ui] = (uint16_t)wgs.size();
            // per lane: position in its row's segment (bits 0-4), last lane of the segment
            // (bit 5), lane in use (bit 6), row slot g*nu + unit (bits 8-19)
            std::vector<uint32_t> lanetab(kRnnThreads, 0);
            std::vector<float> wv((size_t)t.S * kRnnThreads, 0.0f);
            std::vector<uint16_t> zi((size_t)t.S * kRnnThreads, (uint16_t)t.C);   // index C = the zero slot
            uint32_t lane = 0, busy = 0;
            std::vector<std::vector<std::pair<uint32_t, float>>> lane_elems(kRnnThreads);
            // placement of the rows' segments into 16-lane rows
            {
                std::vector<int> ks((size_t)4 * w.nu), place;
                for (uint32_t ui = 0; ui < w.nu; ++ui)
                    for (int g = 0; g < 4; ++g)
                        ks[(size_t)g * w.nu + ui] = (int)((t.rows[(size_t)g * H + w.u0 + ui].size() + t.S - 1) / t.S);
                if (pack_segments(ks, &place) > kBins) { set_error("csb_rnn_create: internal: lane overflow"); return CSB_EINVAL; }
                for (size_t sl = 0; sl < ks.size(); ++sl) {
                    if (ks[sl] <= 0) continue;
                    const uint32_t l0 = (uint32_t)place[sl], k = (uint32_t)ks[sl];
                    const int g = (int)(sl / w.nu), ui = (int)(sl % w.nu);
                    const auto &row = t.rows[(size_t)g * H + w.u0 + ui];
                    for (uint32_t q = 0; q < k; ++q)
                        lanetab[l0 + q] = q | (q + 1 == k ? 32u : 0u) | 64u | ((uint32_t)sl << 8);
                    for (size_t e = 0; e < row.size(); ++e) lane_elems[l0 + (uint32_t)(e / t.S)].push_back(row[e]);
                    lane = std::max<uint32_t>(lane, l0 + k);
                    busy += k;
                }
            }
            // Which of a lane's S slots each of its entries takes is free (it only fixes the
            // order of the lane's sum), and so is the place of every input entry in the staged
            // vector (each workgroup stages its own copy).  The LDS serves 32 lanes at a time
            // from 32 banks of 4 bytes: choose slots and places so that, slot by slot, the 32
            // lanes of a half wavefront hit different banks, or the very same word, as far as
            // possible.  Slots are chosen greedily for given places, places (a bank per entry,
            // every bank filled to its share of [0, C)) greedily for given slots, in turn.
            std::vector<uint16_t> zpos((size_t)t.C);
            for (int e = 0; e < t.C; ++e) zpos[(size_t)e] = (uint16_t)e;
            std::vector<std::vector<int>> slot_of(kRnnThreads);          // per lane: slot of each of its entries
            auto assign_slots = [&](const std::vector<uint16_t> &pos) -> long {
                long cost_total = 0;
                for (uint32_t h0 = 0; h0 < (uint32_t)kRnnThreads; h0 += 32) {
                    std::vector<std::vector<uint32_t>> seen((size_t)t.S * 32);   // [slot][bank] -> distinct words
                    for (uint32_t ln = h0; ln < h0 + 32; ++ln) {
                        std::vector<char> used(t.S, 0);
                        slot_of[ln].assign(lane_elems[ln].size(), 0);
                        for (size_t k = 0; k < lane_elems[ln].size(); ++k) {
                            const uint32_t col = lane_elems[ln][k].first, bank = pos[col] & 31u;
                            int best = -1, best_cost = 1 << 30;
                            for (int sl = 0; sl < t.S; ++sl) {
                                if (used[sl]) continue;
                                auto &words = seen[(size_t)sl * 32 + bank];
                                int cost = (int)words.size() * 2;
                                for (uint32_t wd : words) if (wd == col) { cost = -1; break; }   // broadcast
                                if (cost < best_cost) { best_cost = cost; best = sl; }
                            }
                            used[best] = 1;
                            auto &words = seen[(size_t)best * 32 + bank];
                            if (std::find(words.begin(), words.end(), col) == words.end()) {
                                cost_total += (long)words.size() ? 1 : 0;             // one more word in an occupied bank
                                words.push_back(col);
                            }
                            slot_of[ln][k] = best;
                        }
                    }
                }
                return cost_total;
            };
            auto choose_places = [&](std::vector<uint16_t> &pos) {
                // groups = (half wavefront, slot); an entry should not share a bank with another
                // entry of any of its groups
                const size_t n_groups = (size_t)(kRnnThreads / 32) * t.S;
                std::vector<std::vector<uint32_t>> groups_of((size_t)t.C);
                for (uint32_t ln = 0; ln < (uint32_t)kRnnThreads; ++ln)
                    for (size_t k = 0; k < lane_elems[ln].size(); ++k) {
                        auto &gl = groups_of[lane_elems[ln][k].first];
                        const uint32_t gid = (ln / 32) * (uint32_t)t.S + (uint32_t)slot_of[ln][k];
                        if (std::find(gl.begin(), gl.end(), gid) == gl.end()) gl.push_back(gid);
                    }
                std::vector<int> order((size_t)t.C);
                for (int e = 0; e < t.C; ++e) order[(size_t)e] = e;
                std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return groups_of[(size_t)x].size() > groups_of[(size_t)y].size(); });
                std::vector<uint8_t> cnt(n_groups * 32, 0);                           // [group][bank] entries placed
                int cap[32], fill[32];
                for (int bk = 0; bk < 32; ++bk) { cap[bk] = (t.C - bk + 31) / 32; fill[bk] = 0; }
                for (int e : order) {
                    int best = -1;
                    long best_cost = 1L << 60;
                    for (int bk = 0; bk < 32; ++bk) {
                        if (fill[bk] >= cap[bk]) continue;
                        long c = 0;
                        for (uint32_t gid : groups_of[(size_t)e]) c += cnt[(size_t)gid * 32 + bk];
                        c = c * 64 + fill[bk];                                        // ties: the emptier bank
                        if (c < best_cost) { best_cost = c; best = bk; }
                    }
                    for (uint32_t gid : groups_of[(size_t)e]) if (cnt[(size_t)gid * 32 + best] < 255) ++cnt[(size_t)gid * 32 + best];
                    pos[(size_t)e] = (uint16_t)(best + 32 * fill[best]);
                    ++fill[best];
                }
            };
            long best_cost = assign_slots(zpos);
            const long first_cost = best_cost;
            for (int round = 0; round < 2 && best_cost > 0; ++round) {
                std::vector<uint16_t> trial = zpos;
                choose_places(trial);
                const long c = assign_slots(trial);
                if (c < best_cost) { best_cost = c; zpos = trial; } else { assign_slots(zpos); break; }
            }
            conflicts_total += best_cost;
            if (getenv("CSB_RNN_VERBOSE")) fprintf(stderr, "wg %zu: bank conflicts %ld -> %ld\n", wgs.size(), first_cost, best_cost);
            for (uint32_t ln = 0; ln < (uint32_t)kRnnThreads; ++ln)
                for (size_t k = 0; k < lane_elems[ln].size(); ++k) {
                    wv[(size_t)slot_of[ln][k] * kRnnThreads + ln] = lane_elems[ln][k].second;
                    zi[(size_t)slot_of[ln][k] * kRnnThreads + ln] = zpos[lane_elems[ln][k].first];
                }
            if (lane > (uint32_t)kRnnThreads) { set_error("csb_rnn_create: internal: lane overflow"); return CSB_EINVAL; }
            align(256);
            w.off_rows = (uint32_t)body.size();
            body.insert(body.end(), (uint8_t *)lanetab.data(), (uint8_t *)(lanetab.data() + lanetab.size()));
            align(256);
            w.off_w = (uint32_t)body.size();
            body.insert(body.end(), (uint8_t *)wv.data(), (uint8_t *)(wv.data() + wv.size()));
            align(256);
            w.off_z = (uint32_t)body.size();
            body.insert(body.end(), (uint8_t *)zi.data(), (uint8_t *)(zi.data() + zi.size()));
            align(256);
            w.off_zpos = (uint32_t)body.size();
            body.insert(body.end(), (uint8_t *)zpos.data(), (uint8_t *)(zpos.data() + zpos.size()));
            wgs.push_back(w);
            slots_total += (size_t)kRnnThreads * t.S;
            lanes_max = std::max<double>(lanes_max, busy);
            lanes_sum += busy;
        }
    }
    align(256);
    const size_t off_uw_body = body.size();
    body.insert(body.end(), (uint8_t *)unit_wg.data(), (uint8_t *)(unit_wg.data() + unit_wg.size()));
    align(256);
    const size_t hdr = (wgs.size() * sizeof(RnnWgRec) + 255) / 256 * 256;
    pl.off_unit_wg = hdr + off_uw_body;
    pl.image.assign(hdr + body.size() + 256, 0);
    for (auto &w : wgs) { w.off_rows += (uint32_t)hdr; w.off_w += (uint32_t)hdr; w.off_z += (uint32_t)hdr; w.off_zpos += (uint32_t)hdr; }
    std::memcpy(pl.image.data(), wgs.data(), wgs.size() * sizeof(RnnWgRec));
    std::memcpy(pl.image.data() + hdr, body.data(), body.size());
    pl.n_wgs = (int)wgs.size();
    pl.smax = smax;
    pl.total_nnz = total_nnz;
    pl.slot_fill = slots_total ? (double)total_nnz / (double)slots_total : 0.0;
    pl.lanes_max_over_mean = lanes_sum > 0 ? lanes_max / (lanes_sum / (double)wgs.size()) : 0.0;
    pl.lds_conflicts = conflicts_total;
    pl.valid = true;
    return CSB_OK;
}

// ------------------------------------------------------------------ device side

struct RnnArgs {
    const uint8_t *img;                 // resident image
    const float *x;                     // [T][I]
    const float *h0, *c0;               // [layers][state width], [layers][H] or null
    const float *bias[kRnnMaxLayers];   // per model layer, entries may be null
    float *hseq;                        // [T][state width] or null
    float *hT, *cT;                     // [layers][state width], [layers][H]; cT may be null
    unsigned long long *seq;            // tagged words: per workgroup [T][its units]
    uint32_t T, H, I, tag_base;         // H: hidden width (rows per gate, width of c)
    uint32_t off_unit_wg;               // byte offset in img of the owner table
    uint32_t poll_delay;                // s_sleep units before the first poll of a step (0 = none)
    uint32_t xcds, per_xcd, n_wgs, xcd_step;      // workgroup w runs as block (w % per_xcd) * 8 + w / per_xcd; other blocks exit at once
    // Independent sequences side by side: instance i runs the whole model on the XCDs
    // i % xcd_step places further on (a model that fills at most half an XCD: `share` instances
    // behind each other on the same XCD, i / xcd_step the place) over its own x, states, outputs
    // and exchange words, each this many elements behind the instance before.
    uint32_t n_inst, share;
    size_t s_x, s_h, s_c, s_hseq, s_seq;
    // x, the states and the outputs of a batch stay where the caller has them, [.][batch][width]:
    // consecutive steps (or layers) of one sequence lie `nb` rows apart (1 for a single sequence)
    uint32_t nb;
    unsigned long long *dbg;            // optional: per-phase shader clocks summed over the steps (workgroup 0)
    uint32_t *status;                   // device word: set to 1 when a poll gives up
    uint32_t poll_limit;                // polls of one exchange word before giving up
};

// Workgroup barrier that orders LDS traffic only: global loads and stores in flight (the
// prefetched next frame, the published h_t) are not waited for.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Value of the lane N places down in the same 16-lane row, kept where `mask` is all ones and
// dropped (0) where it is zero or there is no such lane.
template <int N>
__device__ __forceinline__ float masked_shr(float v, uint32_t mask) {
    const uint32_t t = (uint32_t)__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x110 + N, 0xf, 0xf, true);
    return __uint_as_float(t & mask);
}

// Poll a tagged word until it carries `tag`; bounded by `limit` polls.  If the bound is hit the
// result is NaN, *status is set (the host reads it with csb_rnn_status) and `limit` drops to
// zero, so that the lane's later polls give up at once and the kernel still ends promptly.
// `retried` is set if the first load did not already carry the tag.
__device__ __forceinline__ float poll_word(const unsigned long long *word, uint32_t tag, bool &retried, uint32_t &limit, uint32_t *status) {
    // (the words live in device memory: say so, or the loads are issued as generic ones)
    const __attribute__((address_space(1))) unsigned long long *p =
        (const __attribute__((address_space(1))) unsigned long long *)word;
    unsigned long long v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (uint32_t spin = 0; (uint32_t)(v >> 32) != tag && spin < limit; ++spin) {
        retried = true;
        v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if ((uint32_t)(v >> 32) == tag) return __uint_as_float((uint32_t)v);
    limit = 0u;
    __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_nanf("");
}

// PLAIN: every stage is an LSTM / GRU / Li-GRU layer (its own recurrent source, its output the
// layer's state) with inputs at most 2048 wide, so the stage-kind tests and the third z entry
// of the time loop fold away at compile time.
template <int SMAX, bool PLAIN>
__global__ __launch_bounds__(kRnnThreads) void rnn_resident_kernel(const RnnArgs A) {
    extern __shared__ float lds[];
    const uint32_t tid = threadIdx.x;
    // Blocks go to the 8 XCDs in turn (block b to XCD b % 8); the model's workgroups are packed
    // onto as few XCDs as hold them, consecutive ones on the same XCD: the exchange of h_t is
    // fastest between CUs that share an L2.
    const uint32_t xq = (blockIdx.x & 7u) / A.xcd_step, xr = (blockIdx.x & 7u) % A.xcd_step;
    const uint32_t sub = (blockIdx.x >> 3) / A.per_xcd, pos = (blockIdx.x >> 3) - sub * A.per_xcd;
    const uint32_t wgi = xq * A.per_xcd + pos;
    const uint32_t inst = sub * A.xcd_step + xr;
    if (inst >= A.n_inst || sub >= A.share || xq >= A.xcds || wgi >= A.n_wgs) return;
    const float *const x_in = A.x + (size_t)inst * A.s_x;
    const float *const h0 = A.h0 ? A.h0 + (size_t)inst * A.s_h : nullptr;
    const float *const c0 = A.c0 ? A.c0 + (size_t)inst * A.s_c : nullptr;
    float *const hseq = A.hseq ? A.hseq + (size_t)inst * A.s_hseq : nullptr;
    float *const hT = A.hT + (size_t)inst * A.s_h;
    float *const cT = A.cT ? A.cT + (size_t)inst * A.s_c : nullptr;
    unsigned long long *const seq = A.seq + (size_t)inst * A.s_seq;
    const RnnWgRec wg = ((const RnnWgRec *)A.img)[wgi];
    const uint32_t H = A.H, T = A.T, nu = wg.nu, n_in = wg.n_in, C = wg.C, S = wg.S;
    const size_t x_step = (size_t)A.I * A.nb, hseq_step = (size_t)wg.width * A.nb;
    // (the record is the same for every lane: keep what steers branches in scalar registers)
    const uint32_t kword = __builtin_amdgcn_readfirstlane(wg.kind);
    const uint32_t kind = kword & 0xffu, real = (kword >> 8) & 0xffu, flags = kword >> 16;
    const bool lstm = kind == kStageLstm, ligru = kind == kStageLiGru, linear = !PLAIN && kind == kStageLinear;
    const bool rb_reset = !PLAIN && kind == kStageGruRbReset, rb_gate = !PLAIN && kind == kStageGruRbGate;
    const bool from_x = __builtin_amdgcn_readfirstlane(wg.below) == kNoStage;
    const bool own_rec = PLAIN || (flags & kStageOwnRec) != 0, is_state = PLAIN || (flags & kStageIsState) != 0;
    float *z = lds;                       // [C + 1], z[C] = 0
    float *arow = lds + ((C + 1 + 63) & ~63u);   // [4 * nu] row sums
    // weights and LDS addresses of their inputs: registers for the whole sequence
    float w[SMAX];
    uint32_t za[SMAX];
    {
        const float *gw = (const float *)(A.img + wg.off_w);
        const uint16_t *gz = (const uint16_t *)(A.img + wg.off_z);
#pragma unroll
        for (int s = 0; s < SMAX; ++s) {
            const bool in = (uint32_t)s < S;
            w[s] = in ? gw[(size_t)s * kRnnThreads + tid] : 0.0f;
            za[s] = (in ? (uint32_t)gz[(size_t)s * kRnnThreads + tid] : C) * 4u;
        }
    }
    // unit state of this thread (threads 0 .. nu-1 each own one unit) and the lanes that hold
    // the slices of its rows
    const bool owner = tid < nu;
    // this lane's place in its row's segment of lanes
    const uint32_t ltab = ((const uint32_t *)(A.img + wg.off_rows))[tid];
    const uint32_t seg_pos = ltab & 31u, row_slot = ltab >> 8;
    const bool seg_last = (ltab & 32u) != 0;
    const uint32_t unit = wg.u0 + tid;
    // the last lane of a row's segment ends up with the row sum: it adds the bias and applies
    // the gate's non-linearity at once (LSTM rows i,f,o: sigmoid, g: tanh; GRU rows r,z:
    // sigmoid, the two halves of n: none yet; Li-GRU row z: sigmoid, c: none yet; a linear
    // stage: the bare sum)
    float row_bias = 0.0f;
    uint32_t act = 0;                       // 0 none, 1 sigmoid, 2 tanh
    if (seg_last && !linear) {
        const uint32_t g = row_slot / nu, ui = row_slot - g * nu;
        const float *b = A.bias[real];
        if (lstm) { act = g == 2 ? 2u : 1u; if (b) row_bias = b[g * H + wg.u0 + ui]; }
        else if (rb_reset) { act = 1u; if (b && g == 0) row_bias = b[wg.u0 + ui]; }                         // r
        else if (rb_gate) { act = g == 0 ? 1u : 0u; if (b && g < 2) row_bias = b[(g + 1) * H + wg.u0 + ui]; }  // z, n
        else if (ligru) { act = g == 0 ? 1u : 0u; if (b && g < 2) row_bias = b[g * H + wg.u0 + ui]; }
        else { act = g < 2 ? 1u : 0u; if (b && g < 3) row_bias = b[g * H + wg.u0 + ui]; }
    }
    const float act_k = act == 2 ? -2.0f * 1.44269504088896341f : -1.44269504088896341f;
    const float act_a = act == 2 ? 2.0f : 1.0f, act_b = act == 2 ? -1.0f : 0.0f;
    // row-sum scan: which lanes add the value 1, 2, 4, 8 lanes down / the total of the row before
    // (kept as bit masks in vector registers: one AND per level instead of a compare-select)
    uint32_t scan_m1 = (seg_pos & 15u) >= 1 ? ~0u : 0u, scan_m2 = (seg_pos & 15u) >= 2 ? ~0u : 0u;
    uint32_t scan_m4 = (seg_pos & 15u) >= 4 ? ~0u : 0u, scan_m8 = (seg_pos & 15u) >= 8 ? ~0u : 0u;
    uint32_t scan_mb = seg_pos >= 16 ? ~0u : 0u;
    asm volatile("" : "+v"(scan_m1), "+v"(scan_m2), "+v"(scan_m4), "+v"(scan_m8), "+v"(scan_mb));
    float c_state = 0.0f, h_state = 0.0f;
    // where this owner's unit sits in the staged vector's recurrent part (if that part is this stage's own or its state)
    const uint32_t zown = (owner && n_in + unit < C) ? ((const uint16_t *)(A.img + wg.off_zpos))[n_in + unit] : C;
    if (owner) {
        if (c0 && lstm) c_state = c0[(size_t)real * H * A.nb + unit];
        if (h0 && is_state) h_state = h0[(size_t)real * wg.width * A.nb + unit];
    }
    if (tid == 0) z[C] = 0.0f;
    // rows without survivors have no lane: their entry keeps the activation of the bare bias
    for (uint32_t i = tid; i < 4 * nu; i += kRnnThreads) {
        const uint32_t g = i / nu, ui = i - g * nu;
        const float *b = linear ? nullptr : A.bias[real];
        float v = 0.0f;
        if (lstm) { if (b) v = b[g * H + wg.u0 + ui]; v = g == 2 ? fast_tanh(v) : fast_sigmoid(v); }
        else if (rb_reset) { if (b && g == 0) v = b[wg.u0 + ui]; if (g == 0) v = fast_sigmoid(v); }
        else if (rb_gate) { if (b && g < 2) v = b[(g + 1) * H + wg.u0 + ui]; if (g == 0) v = fast_sigmoid(v); }
        else if (ligru) { if (b && g < 2) v = b[g * H + wg.u0 + ui]; if (g == 0) v = fast_sigmoid(v); }
        else if (!linear) { if (b && g < 3) v = b[g * H + wg.u0 + ui]; if (g < 2) v = fast_sigmoid(v); }
        arow[i] = v;
    }
    // Exchange words: every workgroup publishes the outputs of its units into a region of its
    // own, [t][unit of the workgroup]; the regions of different workgroups lie T * nu words
    // apart, which spreads the polling over the memory channels.
    unsigned long long *pub = seq + (size_t)T * wg.upre + tid;     // + t * nu
    const uint16_t *unit_wg = (const uint16_t *)(A.img + A.off_unit_wg);
    // z entries are staged from the top of the workgroup: thread tid handles entries
    // zt and zt + 1024.  The unit owners (low tids) publish with global stores, and a
    // wavefront's loads return behind its own earlier stores; this way the wavefronts that
    // fetch the next input frame are not the ones that store.
    const uint32_t zt = kRnnThreads - 1 - tid;
    // This thread's (at most two) z entries.  An entry below n_in comes from the stage below
    // at the same step (or from x), the others from the recurrent source one step back: they
    // start from h0, and a unit of this workgroup is written by its owner, not polled.  A
    // polled entry has the address of its word at step 0 (one step's stride back for a
    // recurrent one, whose first poll is at step 1), the words per step of the workgroup that
    // publishes it, and the tag it carries at step 0.
    const uint16_t *zpos = (const uint16_t *)(A.img + wg.off_zpos);       // where entry e lives in z
    uint32_t zp[kRnnReps] = {C, C, C};
    const unsigned long long *pp[kRnnReps] = {nullptr, nullptr, nullptr};
    uint32_t pstride[kRnnReps] = {0, 0, 0}, ptmin[kRnnReps] = {~0u, ~0u, ~0u}, ptag[kRnnReps] = {0, 0, 0};
    const uint32_t rec_end = n_in + wg.rec_width;      // entries behind it come from the third input (same step)
#pragma unroll
    for (int rep = 0; rep < kRnnReps; ++rep) {
        const uint32_t e = zt + rep * kRnnThreads;
        if (e >= C) continue;
        zp[rep] = zpos[e];
        const bool rec = e >= n_in && e < rec_end, third = e >= rec_end;
        const uint32_t us = third ? e - rec_end : (rec ? e - n_in : e);
        if (rec) z[zp[rep]] = h0 ? h0[(size_t)real * wg.rec_width * A.nb + us] : 0.0f;
        if (rec ? (own_rec && us - wg.u0 < nu) : (!third && from_x)) continue;
        const RnnWgRec *q = (const RnnWgRec *)A.img + unit_wg[(size_t)(third ? wg.aux : (rec ? wg.rec : wg.below)) + us];
        const uint32_t back = rec ? 1u : 0u;
        pp[rep] = seq + ((size_t)T * q->upre + (us - q->u0)) - (size_t)back * q->nu;
        pstride[rep] = q->nu;
        ptmin[rep] = back;
        ptag[rep] = A.tag_base - back;
    }
    // first frame of the input sequence (the first stage reads x directly, one step ahead)
    const bool xl0 = from_x && zt < n_in, xl1 = from_x && zt + kRnnThreads < n_in;
    float xnext0 = 0.0f, xnext1 = 0.0f;
    if (T > 0) {
        if (xl0) xnext0 = x_in[zt];
        if (xl1) xnext1 = x_in[zt + kRnnThreads];
    }
    // does this wavefront poll at all (any lane with a remote source)?
    const bool polls = __ballot(ptmin[0] != ~0u || ptmin[1] != ~0u || ptmin[2] != ~0u) != 0ull;
    const bool two = C > kRnnThreads, three = !PLAIN && C > 2 * kRnnThreads;           // second / third entries exist
    uint32_t delay = A.poll_delay, streak = 0;
    uint32_t poll_limit = A.poll_limit;                         // drops to zero once a poll of this lane has given up
    unsigned long long wave_arrive = 0, after_b = 0;
    unsigned long long ph0 = 0, ph1 = 0, ph2 = 0, ph3 = 0, c0_ = 0, c1_ = 0;
    const bool dbg = kPhaseClocks && A.dbg != nullptr && blockIdx.x == 0 && tid == 0;
    for (uint32_t t = 0; t < T; ++t) {
        const uint32_t tag_now = A.tag_base + t;
        if (dbg) c0_ = __builtin_readcyclecounter();
        // ---- z = [layer input ; h_{t-1}] into LDS -------------------------------------------
        // A load that samples memory just before h arrives costs a whole extra round trip, one
        // that samples it long after wastes the difference.  Steps repeat with the same timing,
        // so each wavefront waits `delay` sleeps before its first poll and tunes it: three more
        // after a step in which a first poll came back stale, one less after 16 clean steps.
        if (polls)
            for (uint32_t d = 0; d < delay; ++d) __builtin_amdgcn_s_sleep(1);
        bool retried = false;
        if (t >= ptmin[0]) z[zp[0]] = poll_word(pp[0] + (size_t)t * pstride[0], ptag[0] + t, retried, poll_limit, A.status);
        if (two && t >= ptmin[1]) z[zp[1]] = poll_word(pp[1] + (size_t)t * pstride[1], ptag[1] + t, retried, poll_limit, A.status);
        if (three && t >= ptmin[2]) z[zp[2]] = poll_word(pp[2] + (size_t)t * pstride[2], ptag[2] + t, retried, poll_limit, A.status);
        if (kPhaseClocks && A.dbg && blockIdx.x == 0 && (tid & 63u) == 0 && t > 0) wave_arrive += __builtin_readcyclecounter() - after_b;
        if (polls) {
            if (__ballot(retried) != 0ull) { delay += 3; streak = 0; }
            else if (++streak >= 16) { delay -= delay > 0 ? 1u : 0u; streak = 0; }
        }
        if (from_x) {
            if (xl0) z[zp[0]] = xnext0;
            if (xl1) z[zp[1]] = xnext1;
            if (t + 1 < T) {
                if (xl0) xnext0 = x_in[(size_t)(t + 1) * x_step + zt];
                if (xl1) xnext1 = x_in[(size_t)(t + 1) * x_step + zt + kRnnThreads];
            }
        }
        lds_barrier();
        if (dbg) { c1_ = __builtin_readcyclecounter(); ph0 += c1_ - c0_; c0_ = c1_; }
        // ---- this lane's slice of its row ----------------------------------------------------
        float acc = 0.0f;
        const uint8_t *zb = (const uint8_t *)z;
        // all gathers of a lane first, then its multiply-adds; with many slots in batches of 8,
        // or the gathered values alone would push the weights out of the register file
        constexpr int CH = SMAX > 24 ? 8 : SMAX;
#pragma unroll
        for (int s0 = 0; s0 < SMAX; s0 += CH) {
            float zv[CH];
#pragma unroll
            for (int s = 0; s < CH; ++s) zv[s] = *(const float *)(zb + za[s0 + s]);   // unused slots read the zero entry
#pragma unroll
            for (int s = 0; s < CH; ++s) acc = fmaf(w[s0 + s], zv[s], acc);
        }
        // ---- row sum: inclusive scan over the segment's lanes (inside a 32-lane half) ---------
        // (every lane executes the shifts; only the add is conditional).  A segment of up to
        // 16 lanes lies inside one 16-lane row; a longer one fills an even row and continues at
        // the start of the odd row after it, which then adds the even row's total.
        {
            acc += masked_shr<1>(acc, scan_m1);
            acc += masked_shr<2>(acc, scan_m2);
            acc += masked_shr<4>(acc, scan_m4);
            acc += masked_shr<8>(acc, scan_m8);
            // lane 15 of rows 0 and 2 to every lane of rows 1 and 3
            const uint32_t tb = (uint32_t)__builtin_amdgcn_update_dpp(0, __float_as_int(acc), 0x142, 0xa, 0xf, false);
            acc += __uint_as_float(tb & scan_mb);
        }
        {
            // one exponential and one reciprocal per lane: sigmoid(v) = 1 / (1 + 2^(-v log2 e)),
            // tanh(v) = 2 sigmoid(2v) - 1; the lane's constants select between them
            const float pre = acc + row_bias;
            const float sg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(pre * act_k));
            const float out = act == 0 ? pre : fmaf(act_a, sg, act_b);
            if (seg_last) arow[row_slot] = out;
        }
        lds_barrier();
        if (kPhaseClocks && A.dbg && blockIdx.x == 0 && (tid & 63u) == 0) after_b = __builtin_readcyclecounter();
        if (dbg) { c1_ = __builtin_readcyclecounter(); ph1 += c1_ - c0_; c0_ = c1_; }
        // ---- gates and state of the units this workgroup owns --------------------------------
        if (owner) {
            const float a0 = arow[tid], a1 = arow[nu + tid], a2 = arow[2 * nu + tid], a3 = arow[3 * nu + tid];
            // all four reads are issued here, before the branch on the stage kind (left to
            // itself the compiler sinks three of them into the branches, one latency later)
            if constexpr (!PLAIN) asm volatile("" ::"v"(a0), "v"(a1), "v"(a2), "v"(a3));
            float hn;
            if (linear) {                                // the row sum is the output
                hn = a0;
            } else if (rb_reset) {                       // r activated: hand on q = r h_(t-1)
                hn = a0 * z[zown];
            } else if (rb_gate) {                        // z activated; n: input side + Un q (+ bias)
                hn = (1.0f - a0) * fast_tanh(a1) + a0 * h_state;
            } else if (lstm) {                           // activated rows i, f, g, o
                const float cn = a1 * c_state + a0 * a2;
                hn = a3 * fast_tanh(cn);
                c_state = cn;
            } else if (ligru) {                          // z activated; the candidate's sum (+ bias)
                hn = a0 * h_state + (1.0f - a0) * fmaxf(a1, 0.0f);
            } else {                                     // r, z activated; n: input side (+ bias), recurrent side
                const float n = fast_tanh(a2 + a0 * a3);
                hn = (1.0f - a1) * n + a1 * h_state;
            }
            h_state = hn;
            if (own_rec) z[zown] = hn;               // next step's input, read only after the next barrier
            const unsigned long long pk = ((unsigned long long)tag_now << 32) | (unsigned long long)__float_as_uint(hn);
            __hip_atomic_store(pub + (size_t)t * nu, pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (hseq && (flags & kStageIsSeq)) hseq[(size_t)t * hseq_step + unit] = hn;
        }
        if (dbg) { c1_ = __builtin_readcyclecounter(); ph3 += c1_ - c0_; }
    }
    if (dbg) { A.dbg[0] = ph0; A.dbg[1] = ph1; A.dbg[2] = ph2; A.dbg[3] = ph3; }
    if (kPhaseClocks && A.dbg && blockIdx.x == 0 && (tid & 63u) == 0) A.dbg[8 + (tid >> 6)] = wave_arrive;
    if (kPhaseClocks && A.dbg && blockIdx.x == 0 && tid == 512) A.dbg[6] = delay;
    if (owner) {
        if (is_state) hT[(size_t)real * wg.width * A.nb + unit] = h_state;
        if (cT && lstm) cT[(size_t)real * H * A.nb + unit] = c_state;
    }
}

// ------------------------------------------------------------------ streaming path

// Batched element-wise parts: a is [rows][B], the state is kept as [H][B].  One launch serves
// the cells of up to kMaxJobsPerLaunch layers (blockIdx.y), whose products shared a launch too.
struct GateJobs {
    const float *a[kMaxJobsPerLaunch];
    const float *bias[kMaxJobsPerLaunch];
    const float *a2[kMaxJobsPerLaunch];   // reset-before GRU, gate part: the second product's sums
    float *c[kMaxJobsPerLaunch];       // LSTM, LSTMP
    float *h[kMaxJobsPerLaunch];
    float *m[kMaxJobsPerLaunch];       // LSTMP: cell output m_t; reset-before GRU, reset part: q = r h
    float *hseq[kMaxJobsPerLaunch];    // [B][H] of this step, or null
};
// what gates_batched_kernel computes: a cell (CSB_CELL_LSTM / _GRU / _LIGRU) or one of the
// element-wise parts of the cells with two products per step
constexpr int kEwLstmpCell = 100;   // c_t, m_t = o tanh(c_t) (the projection product follows)
constexpr int kEwRbReset = 101;     // q = sigmoid(a_r) h (the candidate's recurrent product follows)
constexpr int kEwRbGate = 102;      // h_t from the z and n rows of a, and a2
__global__ void gates_batched_kernel(const GateJobs J, const int cell, const int H, const int B) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= H * B) return;
    const int j = blockIdx.y;
    const float *__restrict__ a = J.a[j], *__restrict__ bias = J.bias[j];
    float *__restrict__ h = J.h[j];
    const int k = e / B, n = e - k * B;
    float hn;
    if (cell == kEwRbReset) {
        float ar = a[(size_t)k * B + n];
        if (bias) ar += bias[k];
        J.m[j][e] = fast_sigmoid(ar) * h[e];
        return;
    }
    if (cell == kEwRbGate) {
        float az = a[(size_t)(H + k) * B + n], an = a[(size_t)(2 * H + k) * B + n] + J.a2[j][e];
        if (bias) { az += bias[H + k]; an += bias[2 * H + k]; }
        const float z = fast_sigmoid(az);
        hn = (1.0f - z) * fast_tanh(an) + z * h[e];
    } else if (cell == CSB_CELL_LSTM || cell == kEwLstmpCell) {   // rows i, f, g, o
        float *__restrict__ c = J.c[j];
        float ai = a[(size_t)k * B + n], af = a[(size_t)(H + k) * B + n], ag = a[(size_t)(2 * H + k) * B + n],
              ao = a[(size_t)(3 * H + k) * B + n];
        if (bias) { ai += bias[k]; af += bias[H + k]; ag += bias[2 * H + k]; ao += bias[3 * H + k]; }
        const float cn = fast_sigmoid(af) * c[e] + fast_sigmoid(ai) * fast_tanh(ag);
        hn = fast_sigmoid(ao) * fast_tanh(cn);
        c[e] = cn;
        if (cell == kEwLstmpCell) { J.m[j][e] = hn; return; }      // m_t; the state is the projection's result
    } else if (cell == CSB_CELL_GRU) {                 // rows r, z, input side of n, recurrent side of n
        float ar = a[(size_t)k * B + n], az = a[(size_t)(H + k) * B + n], anx = a[(size_t)(2 * H + k) * B + n];
        const float anh = a[(size_t)(3 * H + k) * B + n];
        if (bias) { ar += bias[k]; az += bias[H + k]; anx += bias[2 * H + k]; }
        const float r = fast_sigmoid(ar), z = fast_sigmoid(az);
        hn = (1.0f - z) * fast_tanh(anx + r * anh) + z * h[e];
    } else {                                           // Li-GRU: rows z, candidate
        float az = a[(size_t)k * B + n], ac = a[(size_t)(H + k) * B + n];
        if (bias) { az += bias[k]; ac += bias[H + k]; }
        const float z = fast_sigmoid(az);
        hn = z * h[e] + (1.0f - z) * fmaxf(ac, 0.0f);
    }
    h[e] = hn;
    if (J.hseq[j]) J.hseq[j][(size_t)n * H + k] = hn;
}

// hseq[b][k] = h[k][b] for one step ([W][B] internal -> [B][W] caller's layout)
__global__ void seq_out_kernel(float *__restrict__ dst, const float *__restrict__ src, int W, int B) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= W * B) return;
    const int b = e / W, k = e - b * W;
    dst[e] = src[(size_t)k * B + b];
}

// [L][B][H] (caller's layout) <-> [L][H][B] (internal); src may be null (zeros).
__global__ void state_in_kernel(float *__restrict__ dst, const float *__restrict__ src, int L, int B, int H) {
    const size_t n = (size_t)L * B * H;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const size_t l = i / ((size_t)H * B), rem = i - l * H * B, k = rem / B, b = rem - k * B;
        dst[i] = src ? src[(l * B + b) * H + k] : 0.0f;
    }
}
__global__ void state_out_kernel(float *__restrict__ dst, const float *__restrict__ src, int L, int B, int H) {
    const size_t n = (size_t)L * B * H;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const size_t l = i / ((size_t)H * B), rem = i - l * H * B, b = rem / H, k = rem - b * H;
        dst[i] = src[(l * H + k) * B + b];
    }
}

// dst[l][k][b] = src[l][b][k] through a 32 x 32 tile in LDS, so that both sides move whole
// rows of 128 bytes: block (32, 8), grid (ceil(K / 32), ceil(B / 32), L).
__global__ __launch_bounds__(256) void frames_in_kernel(float *__restrict__ dst, const float *__restrict__ src, int B, int K) {
    __shared__ float tile[32][33];
    const size_t plane = (size_t)blockIdx.z * B * K;
    const int k0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
    for (int i = threadIdx.y; i < 32; i += 8) {
        const int b = b0 + i, k = k0 + threadIdx.x;
        if (b < B && k < K) tile[i][threadIdx.x] = src[plane + (size_t)b * K + k];
    }
    __syncthreads();
    for (int i = threadIdx.y; i < 32; i += 8) {
        const int k = k0 + i, b = b0 + threadIdx.x;
        if (b < B && k < K) dst[plane + (size_t)k * B + b] = tile[threadIdx.x][i];
    }
}

__global__ void fill_kernel(float *p, size_t n, float v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void copy_kernel(float *__restrict__ d, const float *__restrict__ s, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) d[i] = s[i];
}

__global__ void clear_tags_kernel(unsigned long long *p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ull;
}

static void init_state(float *dst, const float *src, size_t n, hipStream_t st) {
    const int blocks = (int)std::min<size_t>((n + 255) / 256, 1024);
    if (src) hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, st, dst, src, n);
    else hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, st, dst, n, 0.0f);
}

static size_t align256(size_t v) { return (v + 255) / 256 * 256; }

struct RnnWs {
    size_t off_a, off_a2, off_c, off_part, off_biasptr, off_seq, off_hint, off_cint, off_m, off_fa, off_fs, rows_out, part_stride, total;
    size_t off_xt;                     // batched: the input frames of `xt_steps` steps as [input][batch]
    int32_t xt_steps;
};

// XCDs one instance of the resident kernel occupies, and how many instances fit side by side
static uint32_t resident_xcds(const csb_rnn *r) {
    uint32_t xcds = ((uint32_t)r->plan.n_wgs + kRnnWgsPerXcd - 1) / kRnnWgsPerXcd;
    if (r->knob_xcds > 0) xcds = std::max(xcds, (uint32_t)r->knob_xcds);
    return xcds;
}
static int resident_instances(const csb_rnn *r, int32_t batch) {
    if (!r->plan.valid) return 1;
    const uint32_t xcds = resident_xcds(r);
    if (xcds > 8) return 1;
    // a model of at most half an XCD's workgroups: several instances on each XCD
    const uint32_t share = xcds == 1 ? std::max<uint32_t>(1u, (uint32_t)kRnnWgsPerXcd / (uint32_t)std::max(1, r->plan.n_wgs)) : 1u;
    return (int)std::min<uint32_t>(8u / xcds * share, (uint32_t)batch);
}

static RnnWs ws_layout(const csb_rnn *r, int32_t batch, int32_t T) {
    RnnWs w{};
    size_t off = 0;
    size_t rows_out = 0, part = 0;
    auto account = [&](const csb_matrix *m) {
        if (!m->plan.valid) return;
        rows_out = std::max<size_t>(rows_out, (size_t)m->plan.hdr.rows_out);
        part = std::max<size_t>(part, (size_t)m->plan.hdr.n_partial_slots * m->plan.hdr.br * 8);
    };
    for (auto *m : r->W) account(m);
    for (auto *m : r->Wp) account(m);
    const size_t HS = (size_t)r->state_width();
    // (batched: one buffer of gate sums per layer -- the products of different layers share launches)
    w.off_a = off; off = align256(off + rows_out * sizeof(float) * (size_t)batch * (batch > 1 ? (size_t)r->n_layers : 1));
    const bool two_products = r->cell == CSB_CELL_GRU_RB;          // second product's output, its operand
    const size_t per_layer = batch > 1 ? (size_t)r->n_layers : 1;
    w.off_a2 = off; off = align256(off + (two_products ? (size_t)batch * r->hidden * sizeof(float) * per_layer : 0));
    w.off_c = off; off = align256(off + (size_t)r->n_layers * batch * r->hidden * sizeof(float));
    // (batch 1: the mat-vecs of different layers share launches, so each layer's two matrices
    // have a region of merge words of their own)
    w.part_stride = align256(part);
    w.off_part = off; off = align256(off + w.part_stride * (batch == 1 ? 2 * (size_t)r->n_layers : 1));
    w.off_biasptr = off; off = align256(off + (size_t)r->n_layers * sizeof(void *));
    // exchange words of the resident kernel: one per unit of every stage and step
    // (a batch may run as several instances of the resident kernel side by side, each with
    // exchange words of its own)
    const size_t seq_units = r->plan.valid ? r->plan.total_units : 0;
    const size_t inst = batch > 1 ? (size_t)resident_instances(r, batch) : 1;
    w.off_seq = off; off = align256(off + (size_t)std::max(T, 1) * seq_units * 8 * inst);
    if (batch > 1) {
        w.off_hint = off; off = align256(off + (size_t)r->n_layers * batch * HS * sizeof(float));
        w.off_cint = off; off = align256(off + (size_t)r->n_layers * batch * r->hidden * sizeof(float));
        // the caller's frames are [batch][input]; the products read right-hand sides with the
        // batch index contiguous, so the frames are turned over a few steps at a time (8 MB)
        const size_t frame = (size_t)batch * r->input * sizeof(float);
        w.xt_steps = (int32_t)std::max<size_t>(1, std::min<size_t>({(size_t)std::max(T, 1), (size_t)1024, ((size_t)8 << 20) / std::max<size_t>(frame, 1)}));
        w.off_xt = off; off = align256(off + (size_t)w.xt_steps * frame);
    }
    // (LSTMP at batch 1 as well: every layer's m_t, between its gate launch and its projection launch)
    w.off_m = off; off = align256(off + ((r->proj > 0 || two_products) ? (size_t)batch * r->hidden * sizeof(float) * (r->proj > 0 ? (size_t)r->n_layers : per_layer) : 0));
    // streaming at batch 1: per layer two buffers of gate sums (plus the second product's sums of
    // the reset-before GRU) and two of (c, h), used alternately by even and odd steps
    const bool fused = batch == 1;
    w.rows_out = rows_out;
    w.off_fa = off; off = align256(off + (fused ? 2 * (size_t)r->n_layers * (rows_out + r->hidden) * sizeof(float) : 0));
    w.off_fs = off; off = align256(off + (fused ? 4 * (size_t)r->n_layers * std::max<size_t>(r->hidden, HS) * sizeof(float) : 0));
    off += 512;   // last 512 bytes: debug clocks of the resident kernel
    w.total = off;
    return w;
}

// One launch of the resident kernel: `n_inst` sequences side by side (instance i on the XCDs
// one place further on), their x / states / outputs `s_*` elements apart.
static int forward_resident(const csb_rnn *r, const float *d_x, const float *d_h0, const float *d_c0, float *d_hseq,
                            float *d_hT, float *d_cT, int32_t T, void *d_ws, const RnnWs &wl, hipStream_t st, int n_inst = 1,
                            size_t s_x = 0, size_t s_h = 0, size_t s_c = 0, size_t s_hseq = 0, size_t region_words = 0, uint32_t nb = 1) {
    const int L = r->n_layers, H = r->hidden;
    unsigned long long *seq = (unsigned long long *)((uint8_t *)d_ws + wl.off_seq);
    const size_t words_inst = r->plan.total_units * (size_t)T, words = words_inst * (size_t)n_inst;
    // Unique tags for this call's T steps; a workspace seen for the first time (or a new tag
    // generation) is cleared so that no stale word can carry a tag of this call.  The resident
    // kernel writes nothing but these words into the workspace, so a region that was cleared
    // once stays good while it does not grow (all rounds of a batch use the same region).
    const size_t region = region_words ? region_words : words;
    const bool other_size = region > r->ws_words;
    uint32_t gen = 0;
    const uint32_t tag_base = reserve_tags((uint32_t)T, &gen);
    if (r->ws_seen != (const void *)seq || r->ws_gen != gen || other_size) {
        hipLaunchKernelGGL(clear_tags_kernel, dim3((unsigned)std::min<size_t>((region + 255) / 256, 2048)), dim3(256), 0, st,
                           seq, region);
        r->ws_words = region;
        r->ws_seen = seq;
        r->ws_gen = gen;
    }
    RnnArgs A{};
    A.img = (const uint8_t *)r->d_img;
    A.x = d_x; A.h0 = d_h0; A.c0 = d_c0;
    for (int l = 0; l < L && l < kRnnMaxLayers; ++l) A.bias[l] = r->d_bias[l];
    A.hseq = d_hseq; A.hT = d_hT; A.cT = d_cT; A.seq = seq;
    A.T = (uint32_t)T; A.H = (uint32_t)H; A.I = (uint32_t)r->input;
    A.tag_base = tag_base;
    A.off_unit_wg = (uint32_t)r->plan.off_unit_wg;
    // at most kRnnWgsPerXcd workgroups per XCD (32 CUs each, one workgroup per CU, all resident)
    const uint32_t xcds = resident_xcds(r);
    if (xcds > 8) { set_error("csb_rnn_forward: resident layout has more workgroups than the device holds at once"); return CSB_EUNSUPPORTED; }
    A.xcds = xcds;
    A.per_xcd = ((uint32_t)r->plan.n_wgs + xcds - 1) / xcds;
    A.n_wgs = (uint32_t)r->plan.n_wgs;
    A.xcd_step = 8u / xcds;                       // the XCDs in use lie this far apart
    A.n_inst = (uint32_t)n_inst;
    A.share = ((uint32_t)n_inst + A.xcd_step - 1) / A.xcd_step;
    if (n_inst < 1 || (A.share > 1 && (xcds > 1 || A.share * A.per_xcd > (uint32_t)kRnnWgsPerXcd))) {
        set_error("csb_rnn_forward: more instances than the XCDs hold");
        return CSB_EINVAL;
    }
    A.s_x = s_x; A.s_h = s_h; A.s_c = s_c; A.s_hseq = s_hseq; A.s_seq = words_inst;
    A.nb = nb;
    A.poll_delay = r->plan.n_wgs > 1 ? 8u : 0u;   // fewer polls in flight while h_t cannot have arrived yet
    if (r->knob_poll_delay >= 0) A.poll_delay = (uint32_t)r->knob_poll_delay;
    A.poll_limit = r->poll_limit;
    A.status = (uint32_t *)((uint8_t *)r->d_img + r->plan.image.size() - 256);   // the image's last 256 bytes: uploaded as zeros
    if (kPhaseClocks && getenv("CSB_RNN_DEBUG")) A.dbg = (unsigned long long *)((uint8_t *)d_ws + wl.total - 512);
    const size_t cmax = r->plan.cmax;
    const size_t lds = (((cmax + 1 + 63) & ~(size_t)63) + kRnnThreads) * sizeof(float);
    auto go = [&](auto kern) -> hipError_t {
        hipError_t e = ensure_dynamic_lds((const void *)kern, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(A.per_xcd * A.share * 8u), dim3(kRnnThreads), lds, st, A);
        return hipGetLastError();
    };
    hipError_t e;
    const int smax = r->plan.smax;
    // one stage per layer and at most two entries per thread: the specialised form
    if (r->cell != CSB_CELL_LSTMP && r->cell != CSB_CELL_GRU_RB && cmax <= 2 * (size_t)kRnnThreads) {
        if (smax <= 4) e = go(rnn_resident_kernel<4, true>);
        else if (smax <= 8) e = go(rnn_resident_kernel<8, true>);
        else if (smax <= 12) e = go(rnn_resident_kernel<12, true>);
        else if (smax <= 16) e = go(rnn_resident_kernel<16, true>);
        else if (smax <= 24) e = go(rnn_resident_kernel<24, true>);
        else if (smax <= 32) e = go(rnn_resident_kernel<32, true>);
        else if (smax <= 40) e = go(rnn_resident_kernel<40, true>);
        else e = go(rnn_resident_kernel<kRnnSlotsMax, true>);
    } else {
        if (smax <= 4) e = go(rnn_resident_kernel<4, false>);
        else if (smax <= 8) e = go(rnn_resident_kernel<8, false>);
        else if (smax <= 12) e = go(rnn_resident_kernel<12, false>);
        else if (smax <= 16) e = go(rnn_resident_kernel<16, false>);
        else if (smax <= 24) e = go(rnn_resident_kernel<24, false>);
        else if (smax <= 32) e = go(rnn_resident_kernel<32, false>);
        else if (smax <= 40) e = go(rnn_resident_kernel<40, false>);
        else e = go(rnn_resident_kernel<kRnnSlotsMax, false>);
    }
    if (e != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

// A batch on the resident kernel: the sequences are independent, and a model that fills only
// some of the 8 XCDs leaves room for further instances of itself beside it.  Every launch runs
// as many sequences as instances fit, each on XCDs (or a share of one) of its own; x, the
// states and the outputs are read and written where the caller has them ([.][batch][width]:
// sequence b starts b rows in, its steps and layers lie `batch` rows apart).
static int forward_resident_batch(const csb_rnn *r, const float *d_x, const float *d_h0, const float *d_c0, float *d_hseq,
                                  float *d_hT, float *d_cT, int32_t T, int32_t batch, void *d_ws, hipStream_t st) {
    const RnnWs wl = ws_layout(r, batch, T);
    const size_t H = (size_t)r->hidden, HS = (size_t)r->state_width(), I = (size_t)r->input;
    const bool lstm = r->cell == CSB_CELL_LSTM || r->cell == CSB_CELL_LSTMP;
    const int R = resident_instances(r, batch);
    for (int32_t b0 = 0; b0 < batch; b0 += R) {
        const int n = std::min<int32_t>(R, batch - b0);
        const size_t b = (size_t)b0;
        int rc = forward_resident(r, d_x + b * I, d_h0 ? d_h0 + b * HS : nullptr, (d_c0 && lstm) ? d_c0 + b * H : nullptr,
                                  d_hseq ? d_hseq + b * HS : nullptr, d_hT + b * HS, (d_cT && lstm) ? d_cT + b * H : nullptr,
                                  T, d_ws, wl, st, n, I, HS, H, HS, (size_t)R * r->plan.total_units * (size_t)T, (uint32_t)batch);
        if (rc != CSB_OK) return rc;
    }
    return CSB_OK;
}

// Rough cost of one time step of a batch, in microseconds, on the two paths that can run it
// (fitted to measurements on MI355X).  Resident kernel: the planner's step model (60 clocks per
// slot, 1700 for the exchange of h_t between workgroups, 6 per workgroup; the forms above 32 slots spill and cost
// half as much again) times 1.3, plus 0.12 us per further XCD an instance spans, twice for the
// cells with two dependent products per step; the batch runs in rounds of as many sequences
// as instances fit.  Batched MFMA path: its launches per diagonal, plus the products at about
// 12 TFLOP/s.
static double resident_batch_us(const csb_rnn *r, int32_t batch) {
    const bool two = r->cell == CSB_CELL_LSTMP || r->cell == CSB_CELL_GRU_RB;
    const int R = resident_instances(r, batch);
    const double rounds = (double)((batch + R - 1) / R);
    const int S = r->plan.smax;
    const double clocks = (60.0 * S + (r->plan.n_wgs > 1 ? 1700.0 : 0.0) + 6.0 * r->plan.n_wgs) * (S > 32 ? 1.5 : 1.0);
    return rounds * (clocks / r->clock_mhz * 1.3 + 0.12 * (resident_xcds(r) - 1)) * (two ? 2.0 : 1.0);
}
static double batched_us(const csb_rnn *r, int32_t batch) {
    const bool two = r->cell == CSB_CELL_LSTMP || r->cell == CSB_CELL_GRU_RB;
    return (10.0 + 4.0 * r->n_layers) * (two ? 1.25 : 1.0) + 2.0 * (double)r->plan.total_nnz * batch / 12e6;
}
static bool batch_prefers_resident(const csb_rnn *r, int32_t batch) {
    if (r->knob_batch_path == 1) return true;
    if (r->knob_batch_path == 2) return false;
    return resident_batch_us(r, batch) * 1.1 < batched_us(r, batch);
}

}  // namespace csb

extern "C" int csb_rnn_create(int32_t cell, int32_t n_layers, int32_t input, int32_t hidden,
                              csb_matrix *const *W, const float *const *d_bias, csb_rnn **out) {
    using namespace csb;
    if (!W || !out) { set_error("csb_rnn_create: NULL pointer"); return CSB_EINVAL; }
    *out = nullptr;
    if (cell != CSB_CELL_LSTM && cell != CSB_CELL_GRU && cell != CSB_CELL_LIGRU) {
        set_error("csb_rnn_create: unknown cell (LSTMP and the reset-before GRU have create calls of their own)");
        return CSB_EINVAL;
    }
    if (n_layers <= 0 || input <= 0 || hidden <= 0) { set_error("csb_rnn_create: non-positive size"); return CSB_EINVAL; }
    const int G = cell == CSB_CELL_LSTM ? 4 : (cell == CSB_CELL_LIGRU ? 2 : 3);
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l]) { set_error("csb_rnn_create: NULL weight matrix"); return CSB_EINVAL; }
        const int64_t n_in = l == 0 ? input : hidden;
        if (W[l]->rows != (int64_t)G * hidden || W[l]->cols != n_in + hidden) {
            set_error("csb_rnn_create: weight matrix shape does not match (G*hidden) x (in + hidden)");
            return CSB_EINVAL;
        }
    }
    try {
        auto *r = new csb_rnn();
        r->cell = cell; r->n_layers = n_layers; r->input = input; r->hidden = hidden;
        for (int l = 0; l < n_layers; ++l) {
            SplitSpec sp{};
            if (cell == CSB_CELL_GRU) { sp.split_row = 2 * (int64_t)hidden; sp.split_col = l == 0 ? input : hidden; sp.shift = hidden; }
            if (!W[l]->plan.valid || !(W[l]->plan.split == sp)) {
                // (a plan the caller made keeps its workgroup count and mode)
                const bool had = W[l]->plan.valid;
                W[l]->stream_wg_limit = 256 / std::min(n_layers, kMaxJobsPerLaunch);   // the layers of a diagonal share a launch
                // A workgroup of the row-owned plan owns units with all their gate rows (r, z and the two
                // halves of n for the GRU), and the streaming step's launches finish their cells
                // themselves (the other form -- a cell computed where its output is consumed, by every
                // workgroup while its weights are on their way -- remains for plans the caller makes).
                // Measured in a loop over the same buffers (launches replayed from the handle's graph), us
                // per step, consumer-side / whole units: LSTM 64->128 3.81 / 3.62, 153->512 4.14 / 3.94,
                // 153->1024 4.45 / 4.29; GRU 256->1024 4.76 / 4.01; Li-GRU 256->1024 4.29 / 3.92; with
                // stacked layers, where a cell has two consumers, 12-17 % apart.  (Enqueued from the host
                // one call at a time, single layers were the other way round: 5.06 / 5.68 for 153->512.)
                W[l]->stream_cell_gates = cell == CSB_CELL_LIGRU ? 2 : 4;
                int rc = plan_matrix(W[l], had ? W[l]->plan.req_chunks : 0, 16, sp, nullptr, had ? W[l]->plan.req_mode : 0);
                if (rc != CSB_OK) { delete r; return rc; }
            }
            r->W.push_back(W[l]);
            r->d_bias.push_back(d_bias ? d_bias[l] : nullptr);
        }
        if (n_layers <= 8) build_resident_plan(r);     // stays invalid if the model does not fit on chip
        *out = r;
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        set_error("csb_rnn_create: out of host memory");
        return CSB_ENOMEM;
    }
}

extern "C" int csb_rnn_create_lstmp(int32_t n_layers, int32_t input, int32_t hidden, int32_t proj,
                                    csb_matrix *const *W, csb_matrix *const *Wp, const float *const *d_bias,
                                    csb_rnn **out) {
    using namespace csb;
    if (!W || !Wp || !out) { set_error("csb_rnn_create_lstmp: NULL pointer"); return CSB_EINVAL; }
    *out = nullptr;
    if (n_layers <= 0 || input <= 0 || hidden <= 0 || proj <= 0) { set_error("csb_rnn_create_lstmp: non-positive size"); return CSB_EINVAL; }
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l] || !Wp[l]) { set_error("csb_rnn_create_lstmp: NULL weight matrix"); return CSB_EINVAL; }
        const int64_t n_in = l == 0 ? input : proj;
        if (W[l]->rows != (int64_t)4 * hidden || W[l]->cols != n_in + proj || Wp[l]->rows != proj || Wp[l]->cols != hidden) {
            set_error("csb_rnn_create_lstmp: shapes must be (4*hidden) x (in + proj) and proj x hidden");
            return CSB_EINVAL;
        }
    }
    try {
        auto *r = new csb_rnn();
        r->cell = CSB_CELL_LSTMP; r->n_layers = n_layers; r->input = input; r->hidden = hidden; r->proj = proj;
        for (int l = 0; l < n_layers; ++l) {
            for (csb_matrix *m : {W[l], Wp[l]})
                if (!m->plan.valid || m->plan.split.active()) {
                    m->stream_wg_limit = 256 / std::min(n_layers, kMaxJobsPerLaunch);   // the layers of a diagonal share a launch
                    // (the gate matrix: workgroups own whole units, the launch of the gate product leaves
                    // m_t = o tanh(c_t) behind and the projection is a plain product of it; measured on the
                    // 153 -> 1024 -> 512 shape in a loop over the same buffers, us per frame, consumer-side /
                    // whole units: one layer 7.71 / 7.24)
                    m->stream_cell_gates = m == W[l] ? 4 : 0;
                    int rc = plan_matrix(m, 0, 16, SplitSpec{}, nullptr, 0);
                    if (rc != CSB_OK) { delete r; return rc; }
                }
            r->W.push_back(W[l]);
            r->Wp.push_back(Wp[l]);
            r->d_bias.push_back(d_bias ? d_bias[l] : nullptr);
        }
        if (n_layers <= 8) build_resident_plan(r);     // stays invalid if the model does not fit on chip
        *out = r;
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        set_error("csb_rnn_create_lstmp: out of host memory");
        return CSB_ENOMEM;
    }
}

extern "C" int csb_rnn_create_gru_rb(int32_t n_layers, int32_t input, int32_t hidden,
                                     csb_matrix *const *Wa, csb_matrix *const *Un, const float *const *d_bias,
                                     csb_rnn **out) {
    using namespace csb;
    if (!Wa || !Un || !out) { set_error("csb_rnn_create_gru_rb: NULL pointer"); return CSB_EINVAL; }
    *out = nullptr;
    if (n_layers <= 0 || input <= 0 || hidden <= 0) { set_error("csb_rnn_create_gru_rb: non-positive size"); return CSB_EINVAL; }
    for (int l = 0; l < n_layers; ++l) {
        if (!Wa[l] || !Un[l]) { set_error("csb_rnn_create_gru_rb: NULL weight matrix"); return CSB_EINVAL; }
        const csb_matrix *m = Wa[l];
        const int64_t n_in = l == 0 ? input : hidden;
        if (m->rows != (int64_t)3 * hidden || m->cols != n_in + hidden || Un[l]->rows != hidden || Un[l]->cols != hidden) {
            set_error("csb_rnn_create_gru_rb: shapes must be (3*hidden) x (in + hidden) and hidden x hidden");
            return CSB_EINVAL;
        }
        // the n rows of Wa hold input-side entries only
        for (int32_t bi = 0; bi < m->nbr; ++bi)
            for (int32_t bj = 0; bj < m->nbc; ++bj) {
                const size_t b = (size_t)bi * m->nbc + bj;
                const int nr = m->nrows[b], nc = m->ncols[b];
                for (int a = 0; a < nr; ++a) {
                    if ((int64_t)bi * m->br + m->rowidx[m->row_off[b] + a] < 2 * (int64_t)hidden) continue;
                    for (int q = 0; q < nc; ++q)
                        if ((int64_t)bj * m->bc + m->colidx[m->col_off[b] + q] >= n_in &&
                            m->val[m->val_off[b] + (size_t)a * nc + q] != 0.0f) {
                            set_error("csb_rnn_create_gru_rb: an n row of Wa has a recurrent-side entry (it belongs in Un)");
                            return CSB_EINVAL;
                        }
                }
            }
    }
    try {
        auto *r = new csb_rnn();
        r->cell = CSB_CELL_GRU_RB; r->n_layers = n_layers; r->input = input; r->hidden = hidden;
        for (int l = 0; l < n_layers; ++l) {
            for (csb_matrix *m : {Wa[l], Un[l]})
                if (!m->plan.valid || m->plan.split.active()) {
                    m->stream_wg_limit = 256 / std::min(n_layers, kMaxJobsPerLaunch);   // the layers of a diagonal share a launch
                    // (workgroups own whole units -- r, z, n rows of the first matrix, the one row of the second --
                    // and both launches of a step finish their part of the cell themselves; for this cell
                    // also with one layer: measured, us per step, consumer-side / whole units: 39 -> 1024
                    // 8.43 / 7.52, 153 -> 512 7.91 / 7.11, 64 -> 256 7.39 / 7.12)
                    m->stream_cell_gates = m == Wa[l] ? 3 : 1;
                    int rc = plan_matrix(m, 0, 16, SplitSpec{}, nullptr, 0);
                    if (rc != CSB_OK) { delete r; return rc; }
                }
            r->W.push_back(Wa[l]);
            r->Wp.push_back(Un[l]);
            r->d_bias.push_back(d_bias ? d_bias[l] : nullptr);
        }
        if (n_layers <= 8) build_resident_plan(r);     // stays invalid if the model does not fit on chip
        *out = r;
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        set_error("csb_rnn_create_gru_rb: out of host memory");
        return CSB_ENOMEM;
    }
}

extern "C" size_t csb_rnn_device_bytes(const csb_rnn *r) {
    return (r && r->plan.valid) ? r->plan.image.size() : 0;
}

extern "C" int csb_rnn_upload(csb_rnn *r, void *d_buf, size_t bytes, void *stream) {
    using namespace csb;
    if (!r || !d_buf) { set_error("csb_rnn_upload: NULL pointer"); return CSB_EINVAL; }
    if (!r->plan.valid) { set_error("csb_rnn_upload: this model has no resident layout"); return CSB_EUNSUPPORTED; }
    if (bytes < r->plan.image.size()) { set_error("csb_rnn_upload: device buffer too small"); return CSB_ENOMEM; }
    if ((uintptr_t)d_buf % 256) { set_error("csb_rnn_upload: device buffer not 256-byte aligned"); return CSB_EINVAL; }
    hipError_t e = hipMemcpyAsync(d_buf, r->plan.image.data(), r->plan.image.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) { set_error(std::string("csb_rnn_upload: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    r->d_img = d_buf;
    r->uploaded = true;
    return CSB_OK;
}

extern "C" int csb_rnn_set_poll_limit(csb_rnn *r, uint32_t polls) {
    if (!r) { csb::set_error("csb_rnn_set_poll_limit: NULL handle"); return CSB_EINVAL; }
    r->poll_limit = polls;
    return CSB_OK;
}

// Has a workgroup of the resident kernel given up waiting for another one's h_t since the last check?
extern "C" int csb_rnn_status(const csb_rnn *r, void *stream, int32_t *timed_out) {
    using namespace csb;
    if (!r || !timed_out) { set_error("csb_rnn_status: NULL pointer"); return CSB_EINVAL; }
    *timed_out = 0;
    if (!r->plan.valid || !r->uploaded || !r->d_img) return CSB_OK;
    uint32_t *d = (uint32_t *)((uint8_t *)r->d_img + r->plan.image.size() - 256);
    uint32_t v = 0;
    hipError_t e = hipMemcpyAsync(&v, d, 4, hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess && v) e = hipMemsetAsync(d, 0, 4, (hipStream_t)stream);
    if (e != hipSuccess) { set_error(std::string("csb_rnn_status: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    *timed_out = (int32_t)v;
    return CSB_OK;
}

extern "C" int csb_rnn_plan_resident(csb_rnn *r, int32_t batch) {
    using namespace csb;
    if (!r || batch <= 0) { set_error("csb_rnn_plan_resident: NULL handle or batch <= 0"); return CSB_EINVAL; }
    if (!r->plan.valid) { set_error("csb_rnn_plan_resident: this model has no resident layout"); return CSB_EUNSUPPORTED; }
    r->uploaded = false;
    r->d_img = nullptr;
    r->ws_seen = nullptr;
    try {
        // More slots per lane make an instance smaller (more of them per launch, fewer rounds)
        // and its step longer: take the slot count with the smallest estimate for this batch.
        int best = 0;
        double best_us = 1e300;
        if (batch > 1)
            for (int S : {8, 12, 16, 24, 32}) {       // (none fits: the layout of create, 0 below)
                if (build_resident_plan(r, S) != CSB_OK) continue;
                const double us = resident_batch_us(r, batch);
                if (us < best_us) { best_us = us; best = S; }
            }
        int rc = build_resident_plan(r, best);
        if (rc != CSB_OK) rc = build_resident_plan(r, 0);       // (the default layout existed before)
        if (rc != CSB_OK) { set_error("csb_rnn_plan_resident: the layout could not be rebuilt"); return rc; }
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        r->plan = RnnPlan{};
        set_error("csb_rnn_plan_resident: out of host memory");
        return CSB_ENOMEM;
    }
}

extern "C" int csb_rnn_stats(const csb_rnn *r, csb_rnn_plan_stats *out) {
    if (!r || !out) { csb::set_error("csb_rnn_stats: NULL pointer"); return CSB_EINVAL; }
    out->resident = r->plan.valid ? 1 : 0;
    out->n_workgroups = r->plan.n_wgs;
    out->slots_per_lane = r->plan.smax;
    out->slot_fill = r->plan.slot_fill;
    out->lanes_max_over_mean = r->plan.lanes_max_over_mean;
    out->reserved = (int32_t)std::min<long>(r->plan.lds_conflicts, 0x7fffffff);
    return CSB_OK;
}

extern "C" size_t csb_rnn_workspace_bytes(const csb_rnn *r, int32_t batch, int32_t T) {
    if (!r || batch <= 0 || T < 0) return 0;
    return csb::ws_layout(r, batch, T).total;
}

static int rnn_forward_enqueue(const csb_rnn *r, const float *d_x, const float *d_h0, const float *d_c0,
                               float *d_hseq, float *d_hT, float *d_cT, int32_t T, int32_t batch,
                               void *d_ws, void *stream) {
    using namespace csb;
    if (!r || !d_hT || !d_ws) { set_error("csb_rnn_forward: NULL pointer"); return CSB_EINVAL; }
    if ((uintptr_t)d_ws % 256) { set_error("csb_rnn_forward: workspace not 256-byte aligned"); return CSB_EINVAL; }
    if (batch <= 0 || T < 0) { set_error("csb_rnn_forward: batch <= 0 or T < 0"); return CSB_EINVAL; }
    if (T > 0 && !d_x) { set_error("csb_rnn_forward: NULL input sequence"); return CSB_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    const int L = r->n_layers, H = r->hidden, I = r->input;
    const bool lstmp = r->cell == CSB_CELL_LSTMP;
    const bool lstm = r->cell == CSB_CELL_LSTM || lstmp;        // has a cell state c
    const bool gru_rb = r->cell == CSB_CELL_GRU_RB;
    const int HS = r->state_width();                             // width of h (the projection's for LSTMP)
    const size_t nstate = (size_t)L * batch * HS, ncstate = (size_t)L * batch * H;
    if (T == 0) {                                  // hand the state through
        init_state(d_hT, d_h0, nstate, st);
        if (lstm && d_cT) init_state(d_cT, d_c0, ncstate, st);
        return CSB_OK;
    }
    bool streams_ready = true;
    for (auto *m : r->W) streams_ready = streams_ready && m->plan.valid && m->uploaded;
    for (auto *m : r->Wp) streams_ready = streams_ready && m->plan.valid && m->uploaded;
    const bool can_reside = r->plan.valid && r->uploaded && resident_xcds(r) <= 8;
    const bool resident = can_reside && (batch == 1 || !streams_ready || batch_prefers_resident(r, batch));
    if (!resident) {
        for (auto *m : r->W)
            if (!m->plan.valid || !m->uploaded) {
                set_error("csb_rnn_forward: neither the resident layout nor every weight matrix is uploaded");
                return CSB_ESTATE;
            }
        // the step kernels index the sums by the row layout csb_rnn_create planned (the GRU keeps the two
        // halves of its n rows apart): a matrix planned otherwise since then must not be used
        for (int l = 0; l < L; ++l) {
            SplitSpec sp{};
            if (r->cell == CSB_CELL_GRU) { sp.split_row = 2 * (int64_t)H; sp.split_col = l == 0 ? r->input : H; sp.shift = H; }
            if (!(r->W[l]->plan.split == sp)) {
                set_error("csb_rnn_forward: a weight matrix was planned again in another row layout after csb_rnn_create");
                return CSB_ESTATE;
            }
        }
        for (auto *m : r->Wp)
            if (!m->plan.valid || !m->uploaded) {
                set_error("csb_rnn_forward: a layer's second matrix (projection / candidate recurrence) is not uploaded");
                return CSB_ESTATE;
            }
    }
    // Another handle (or another kind of call) may have used this workspace since this one did:
    // whatever it left there must not be taken for tagged words of this call.
    if (d_ws && workspace_changed_hands(d_ws, r)) {
        r->ws_seen = nullptr;
        for (auto *m : r->W) m->ws_seen = nullptr;
        for (auto *m : r->Wp) m->ws_seen = nullptr;
    }
    // The paths lay the workspace out differently, and so do different batch sizes: what was a
    // float buffer of the last call may be tagged words of this one.
    const int64_t use = (int64_t)batch * 2 + (resident ? 1 : 0);
    if (r->ws_use != use) {
        r->ws_use = use;
        r->ws_seen = nullptr;
        for (auto *m : r->W) m->ws_seen = nullptr;
        for (auto *m : r->Wp) m->ws_seen = nullptr;
    }
    if (resident && batch == 1) return forward_resident(r, d_x, d_h0, d_c0, d_hseq, d_hT, d_cT, T, d_ws, ws_layout(r, 1, T), st);
    if (resident) return forward_resident_batch(r, d_x, d_h0, d_c0, d_hseq, d_hT, d_cT, T, batch, d_ws, st);

    const RnnWs wl = ws_layout(r, batch, T);
    float *a = (float *)((uint8_t *)d_ws + wl.off_a), *a2 = (float *)((uint8_t *)d_ws + wl.off_a2);
    if (batch > 1) {
        // batched: one MFMA mat-mat launch and one gate launch per step and layer; the state
        // lives as [H][B] so that the batch index is the contiguous one
        float *hi = (float *)((uint8_t *)d_ws + wl.off_hint), *ci = (float *)((uint8_t *)d_ws + wl.off_cint);
        float *mb = (float *)((uint8_t *)d_ws + wl.off_m);
        float *xt = (float *)((uint8_t *)d_ws + wl.off_xt);
        const int sblocks = (int)std::min<size_t>((std::max(nstate, ncstate) + 255) / 256, 2048);
        hipLaunchKernelGGL(state_in_kernel, dim3(sblocks), dim3(256), 0, st, hi, d_h0, L, batch, HS);
        if (lstm) hipLaunchKernelGGL(state_in_kernel, dim3(sblocks), dim3(256), 0, st, ci, d_c0, L, batch, H);
        const int gb = (H * batch + 255) / 256;
        // Layer l at step t needs layer l - 1 at step t and itself at step t - 1: everything on
        // the diagonal l + t = d is independent, so a diagonal takes ONE product launch and ONE
        // element-wise launch per phase (for up to kMaxJobsPerLaunch layers each) instead of one per
        // layer -- a single layer's product is too small to fill the GPU.  The states are updated
        // in place: within a diagonal every phase of all layers runs before the next phase.
        // LSTM / GRU / Li-GRU have one phase (product, gates); LSTMP has two (gate product, cell;
        // projection product into the state), the reset-before GRU too (first product, reset;
        // second product, gates).
        const size_t a_stride = wl.rows_out * (size_t)batch, hb = (size_t)H * batch;
        const bool two_phase = lstmp || gru_rb;
        for (int d = 0; d < T + L - 1; ++d) {
            const int lo = std::max(0, d - (T - 1)), hi_l = std::min(L - 1, d);
            auto for_groups = [&](auto body) -> int {           // body(first layer, layers in the group)
                for (int l0 = lo; l0 <= hi_l; l0 += kMaxJobsPerLaunch) {
                    int rc = body(l0, std::min(kMaxJobsPerLaunch, hi_l - l0 + 1));
                    if (rc != CSB_OK) return rc;
                }
                return CSB_OK;
            };
            auto ew = [&](int mode) {                            // one element-wise launch per group
                return for_groups([&](int l0, int n) {
                    GateJobs J{};
                    for (int i = 0; i < n; ++i) {
                        const int l = l0 + i, t = d - l;
                        J.a[i] = a + (size_t)l * a_stride;
                        J.a2[i] = a2 + (size_t)l * hb;
                        J.bias[i] = r->d_bias[l];
                        J.c[i] = lstm ? ci + (size_t)l * hb : nullptr;
                        J.h[i] = hi + (size_t)l * HS * batch;
                        J.m[i] = mb + (size_t)l * hb;
                        J.hseq[i] = (d_hseq && l == L - 1) ? d_hseq + (size_t)t * batch * HS : nullptr;
                    }
                    hipLaunchKernelGGL(gates_batched_kernel, dim3(gb, n), dim3(256), 0, st, J, mode, H, batch);
                    return (int)CSB_OK;
                });
            };
            // first (or only) product: W_l [input ; state]
            if (d < T && d % wl.xt_steps == 0) {                // the first layer is at step d: its next frames
                const int steps = std::min(wl.xt_steps, T - d);
                hipLaunchKernelGGL(frames_in_kernel, dim3((I + 31) / 32, (batch + 31) / 32, steps), dim3(32, 8), 0, st, xt,
                                   d_x + (size_t)d * batch * I, batch, I);
            }
            int rc = for_groups([&](int l0, int n) {
                SpmmCall calls[kMaxJobsPerLaunch];
                for (int i = 0; i < n; ++i) {
                    const int l = l0 + i, t = d - l;
                    float *hl = hi + (size_t)l * HS * batch;
                    if (l == 0)
                        calls[i] = SpmmCall{r->W[l], xt + (size_t)(t % wl.xt_steps) * batch * I, (uint32_t)I, batch, 1, hl, batch, 1,
                                            a + (size_t)l * a_stride, batch};
                    else
                        calls[i] = SpmmCall{r->W[l], hi + (size_t)(l - 1) * HS * batch, (uint32_t)HS, batch, 1, hl, batch, 1,
                                            a + (size_t)l * a_stride, batch};
                }
                return spmm_strided_multi(calls, n, batch, st);
            });
            if (rc != CSB_OK) return rc;
            if (!two_phase) {
                ew((int)r->cell);
                continue;
            }
            ew(lstmp ? kEwLstmpCell : kEwRbReset);               // m_t, or q = r h_(t-1)
            // second product: the projection r_t = Wp m_t straight into the state, or Un q
            rc = for_groups([&](int l0, int n) {
                SpmmCall calls[kMaxJobsPerLaunch];
                for (int i = 0; i < n; ++i) {
                    const int l = l0 + i;
                    float *ml = mb + (size_t)l * hb;
                    float *dst = lstmp ? hi + (size_t)l * HS * batch : a2 + (size_t)l * hb;
                    calls[i] = SpmmCall{r->Wp[l], ml, (uint32_t)H, batch, 1, ml, batch, 1, dst, batch};
                }
                return spmm_strided_multi(calls, n, batch, st);
            });
            if (rc != CSB_OK) return rc;
            if (gru_rb) ew(kEwRbGate);
            else if (d_hseq && d >= L - 1 && d - (L - 1) < T)    // the last layer is on this diagonal
                hipLaunchKernelGGL(seq_out_kernel, dim3((HS * batch + 255) / 256), dim3(256), 0, st,
                                   d_hseq + (size_t)(d - (L - 1)) * batch * HS, hi + (size_t)(L - 1) * HS * batch, HS, batch);
        }
        hipLaunchKernelGGL(state_out_kernel, dim3(sblocks), dim3(256), 0, st, d_hT, hi, L, batch, HS);
        if (lstm && d_cT) hipLaunchKernelGGL(state_out_kernel, dim3(sblocks), dim3(256), 0, st, d_cT, ci, L, batch, H);
        hipError_t eb = hipGetLastError();
        if (eb != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(eb)); return CSB_EDEVICE; }
        return CSB_OK;
    }
    // ---- streaming path, batch 1 -------------------------------------------------------------
    // The element-wise part of a cell (Sec. 2.1) is no launch of its own: the mat-vec launches
    // that consume a cell's output -- layer l + 1 at step t, layer l at step t + 1 -- compute it
    // from the gate sums while they stage their input (see GateSrc).  Sums and states of step t
    // live in buffer t & 1 of their layer (the initial state in buffer 1), so a launch never
    // writes what another workgroup of the same launch still reads.  And the steps run by
    // DIAGONALS: layer l at step t needs layer l - 1 at step t and itself at step t - 1, so
    // the pairs with l + t = d are independent and share one launch per product phase.
    uint8_t *part0 = (uint8_t *)d_ws + wl.off_part;
    auto part_of = [&](int l, int which) { return (void *)(part0 + ((size_t)l * 2 + (size_t)which) * wl.part_stride); };
    float *fa = (float *)((uint8_t *)d_ws + wl.off_fa), *fs = (float *)((uint8_t *)d_ws + wl.off_fs);
    const size_t SW = (size_t)std::max(H, HS);                   // room of one state vector
    auto sums = [&](int l, int t) { return fa + ((size_t)l * 2 + (size_t)(t & 1)) * (wl.rows_out + (size_t)H); };
    auto sums2 = [&](int l, int t) { return sums(l, t) + wl.rows_out; };       // reset-before GRU: Un q
    auto c_of = [&](int l, int t) { return fs + (((size_t)l * 2 + (size_t)(t & 1)) * 2) * SW; };
    auto h_buf = [&](int l, int t) { return c_of(l, t) + SW; };
    // Row-owned plans whose workgroups own whole units (what csb_rnn_create lays out for these
    // cells): a launch is the whole step of its layers -- product, then c_t and h_t by the workgroup
    // that has the unit's sums -- and its input is two vectors that are already in memory.
    bool whole_units = !lstmp && !gru_rb;
    for (auto *m : r->W)
        whole_units = whole_units && m->plan.stream.valid && m->plan.stream.cell_gates != 0 && m->plan.stream.val_fmt == r->W[0]->plan.stream.val_fmt &&
                      m->plan.hdr.cols <= (uint64_t)kMaxStageCols;
    // ... and then the first step reads the caller's initial state where it lies (or none: zeros) and the
    // last step writes the caller's final state: no launch besides the steps -- unless the caller's
    // initial and final states share memory
    auto overlap = [&](const float *a, const float *b) { const size_t n = (size_t)L * H; return a && b && a < b + n && b < a + n; };
    const bool direct = whole_units && !overlap(d_h0, d_hT) && !overlap(d_c0, d_cT) && !overlap(d_h0, d_cT) && !overlap(d_c0, d_hT);
    if (!direct)
        for (int l = 0; l < L; ++l) {
            init_state(h_buf(l, -1), d_h0 ? d_h0 + (size_t)l * HS : nullptr, (size_t)HS, st);
            if (lstm) init_state(c_of(l, -1), d_c0 ? d_c0 + (size_t)l * H : nullptr, (size_t)H, st);
        }
    // LSTMP: r_(l,t), the projected output, is a plain vector (the result of the layer's second
    // product); the last layer's goes straight into the output sequence when one is asked for
    auto r_of = [&](int l, int t) { return (t >= 0 && d_hseq && l == L - 1) ? d_hseq + (size_t)t * HS : h_buf(l, t); };
    // h_(l,t) of the other cells, still to be computed from the sums of step t
    auto cell_output = [&](int l, int t) {
        GateSrc g{};
        g.a = sums(l, t); g.a2 = sums2(l, t); g.bias = r->d_bias[l];
        g.c_in = lstm ? c_of(l, t - 1) : nullptr; g.h_in = h_buf(l, t - 1);
        g.c_out = lstm ? c_of(l, t) : nullptr; g.h_out = h_buf(l, t);
        g.hseq = (d_hseq && l == L - 1) ? d_hseq + (size_t)t * H : nullptr;
        g.kind = gru_rb ? kGateRbGate : 1u + (uint32_t)r->cell; g.H = (uint32_t)H;
        return g;
    };
    bool lstmp_units = lstmp;
    for (auto *m : r->W)
        lstmp_units = lstmp_units && m->plan.stream.valid && m->plan.stream.cell_gates == 4 && m->plan.stream.val_fmt == r->W[0]->plan.stream.val_fmt &&
                      m->plan.hdr.cols <= (uint64_t)kMaxStageCols;
    for (auto *m : r->Wp)
        lstmp_units = lstmp_units && m->plan.stream.valid && m->plan.stream.cell_gates == 0 && m->plan.stream.val_fmt == r->Wp[0]->plan.stream.val_fmt;
    bool rb_units = gru_rb;
    for (auto *m : r->W)
        rb_units = rb_units && m->plan.stream.valid && m->plan.stream.cell_gates == 3 && m->plan.stream.val_fmt == r->W[0]->plan.stream.val_fmt &&
                   m->plan.hdr.cols <= (uint64_t)kMaxStageCols;
    for (auto *m : r->Wp)
        rb_units = rb_units && m->plan.stream.valid && m->plan.stream.cell_gates == 1 && m->plan.stream.val_fmt == r->Wp[0]->plan.stream.val_fmt;
    if (rb_units) {
        // reset-before GRU on such plans: the first launch leaves q = r h_(t-1), z and the n row's sum (in the
        // layer's sums buffer), the second adds Un q and writes h_t
        for (int d = 0; d < T + L - 1; ++d) {
            const int lo = std::max(0, d - (T - 1)), hi_l = std::min(L - 1, d);
            for (int l0 = lo; l0 <= hi_l; l0 += kMaxJobsPerLaunch) {
                SpmvCellCall first[kMaxJobsPerLaunch], second[kMaxJobsPerLaunch];
                const int n = std::min(kMaxJobsPerLaunch, hi_l - l0 + 1);
                for (int i = 0; i < n; ++i) {
                    const int l = l0 + i, t = d - l;
                    float *zs = sums(l, t), *ns = zs + H, *q = zs + 2 * (size_t)H;
                    first[i] = SpmvCellCall{r->W[l], l == 0 ? d_x + (size_t)t * I : h_buf(l - 1, t), l == 0 ? (uint32_t)I : (uint32_t)H,
                                            h_buf(l, t - 1), kCellRbReset, r->d_bias[l], nullptr, zs, q, ns};
                    second[i] = SpmvCellCall{r->Wp[l], q, (uint32_t)H, q, kCellRbGate, nullptr, zs, nullptr, h_buf(l, t),
                                             (d_hseq && l == L - 1) ? d_hseq + (size_t)t * H : nullptr, h_buf(l, t - 1), ns};
                }
                int rc = spmv_rows_cell_multi(first, n, st);
                if (rc == CSB_OK) rc = spmv_rows_cell_multi(second, n, st);
                if (rc != CSB_OK) return rc;
            }
        }
        for (int l = 0; l < L; ++l) init_state(d_hT + (size_t)l * H, h_buf(l, T - 1), (size_t)H, st);
        hipError_t ec = hipGetLastError();
        if (ec != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(ec)); return CSB_EDEVICE; }
        return CSB_OK;
    }
    if (lstmp_units) {
        // LSTMP on such plans: the gate product's launch finishes the cell (c_t, m_t = o tanh(c_t)), the
        // projection r_t = Wp m_t is a plain product (the last layer's straight into the output sequence)
        float *mbuf = (float *)((uint8_t *)d_ws + wl.off_m);
        for (int d = 0; d < T + L - 1; ++d) {
            const int lo = std::max(0, d - (T - 1)), hi_l = std::min(L - 1, d);
            for (int l0 = lo; l0 <= hi_l; l0 += kMaxJobsPerLaunch) {
                SpmvCellCall calls[kMaxJobsPerLaunch];
                SpmvPlainCall proj[kMaxJobsPerLaunch];
                const int n = std::min(kMaxJobsPerLaunch, hi_l - l0 + 1);
                for (int i = 0; i < n; ++i) {
                    const int l = l0 + i, t = d - l;
                    float *ml = mbuf + (size_t)l * H;
                    calls[i] = SpmvCellCall{r->W[l], l == 0 ? d_x + (size_t)t * I : (const float *)r_of(l - 1, t), l == 0 ? (uint32_t)I : (uint32_t)HS,
                                            r_of(l, t - 1), CSB_CELL_LSTM, r->d_bias[l], c_of(l, t - 1), c_of(l, t), ml, nullptr};
                    proj[i] = SpmvPlainCall{r->Wp[l], ml, r_of(l, t)};
                }
                int rc = spmv_rows_cell_multi(calls, n, st);
                if (rc == CSB_OK) rc = spmv_rows_multi(proj, n, st);
                if (rc != CSB_OK) return rc;
            }
        }
        for (int l = 0; l < L; ++l) {
            init_state(d_hT + (size_t)l * HS, r_of(l, T - 1), (size_t)HS, st);
            if (d_cT) init_state(d_cT + (size_t)l * H, c_of(l, T - 1), (size_t)H, st);
        }
        hipError_t ec = hipGetLastError();
        if (ec != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(ec)); return CSB_EDEVICE; }
        return CSB_OK;
    }
    if (whole_units) {
        auto hs = [&](int l, int t) -> float * { return (direct && t == T - 1) ? d_hT + (size_t)l * H : h_buf(l, t); };
        auto h_before = [&](int l, int t) -> const float * {
            return (t > 0 || !direct) ? hs(l, t - 1) : d_h0 ? d_h0 + (size_t)l * H : nullptr;
        };
        auto c_before = [&](int l, int t) -> const float * {
            return (t > 0 || !direct) ? c_of(l, t - 1) : d_c0 ? d_c0 + (size_t)l * H : nullptr;
        };
        auto c_after = [&](int l, int t) -> float * { return (direct && t == T - 1 && d_cT) ? d_cT + (size_t)l * H : c_of(l, t); };
        for (int d = 0; d < T + L - 1; ++d) {
            const int lo = std::max(0, d - (T - 1)), hi_l = std::min(L - 1, d);
            for (int l0 = lo; l0 <= hi_l; l0 += kMaxJobsPerLaunch) {
                SpmvCellCall calls[kMaxJobsPerLaunch];
                const int n = std::min(kMaxJobsPerLaunch, hi_l - l0 + 1);
                for (int i = 0; i < n; ++i) {
                    const int l = l0 + i, t = d - l;
                    calls[i] = SpmvCellCall{r->W[l], l == 0 ? d_x + (size_t)t * I : hs(l - 1, t), l == 0 ? (uint32_t)I : (uint32_t)H,
                                            h_before(l, t), (int32_t)r->cell, r->d_bias[l], lstm ? c_before(l, t) : nullptr,
                                            lstm ? c_after(l, t) : nullptr, hs(l, t),
                                            (d_hseq && l == L - 1) ? d_hseq + (size_t)t * H : nullptr};
                }
                int rc = spmv_rows_cell_multi(calls, n, st);
                if (rc != CSB_OK) return rc;
            }
        }
        if (!direct)
            for (int l = 0; l < L; ++l) {
                init_state(d_hT + (size_t)l * H, h_buf(l, T - 1), (size_t)H, st);
                if (lstm && d_cT) init_state(d_cT + (size_t)l * H, c_of(l, T - 1), (size_t)H, st);
            }
        hipError_t ec = hipGetLastError();
        if (ec != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(ec)); return CSB_EDEVICE; }
        return CSB_OK;
    }
    for (int d = 0; d < T + L - 1; ++d) {
        const int lo = std::max(0, d - (T - 1)), hi_l = std::min(L - 1, d);
        // first (or only) product of every pair on the diagonal: W_l [input ; state]
        for (int l0 = lo; l0 <= hi_l; l0 += kMaxJobsPerLaunch) {
            SpmvGatedCall calls[kMaxJobsPerLaunch];
            const int n = std::min(kMaxJobsPerLaunch, hi_l - l0 + 1);
            for (int i = 0; i < n; ++i) {
                const int l = l0 + i, t = d - l;
                GateSrc below, back;
                if (lstmp) {
                    below = plain_src(l == 0 ? d_x + (size_t)t * I : (const float *)r_of(l - 1, t));
                    back = plain_src(r_of(l, t - 1));
                } else {
                    below = l == 0 ? plain_src(d_x + (size_t)t * I) : cell_output(l - 1, t);
                    back = t == 0 ? plain_src(h_buf(l, -1)) : cell_output(l, t - 1);
                }
                calls[i] = SpmvGatedCall{r->W[l], below, l == 0 ? (uint32_t)I : (uint32_t)HS, back, sums(l, t), part_of(l, 0)};
            }
            int rc = spmv_gated_multi(calls, n, st);
            if (rc != CSB_OK) return rc;
        }
        if (!lstmp && !gru_rb) continue;
        // second product: LSTMP r_t = Wp m_t with m_t = o tanh(c_t) computed on the way in; the
        // reset-before GRU's Un q with q = r h_(t-1) (h_(t-1) was stored by the launch above)
        for (int l0 = lo; l0 <= hi_l; l0 += kMaxJobsPerLaunch) {
            SpmvGatedCall calls[kMaxJobsPerLaunch];
            const int n = std::min(kMaxJobsPerLaunch, hi_l - l0 + 1);
            for (int i = 0; i < n; ++i) {
                const int l = l0 + i, t = d - l;
                GateSrc g{};
                g.a = sums(l, t); g.bias = r->d_bias[l]; g.H = (uint32_t)H;
                if (lstmp) { g.c_in = c_of(l, t - 1); g.c_out = c_of(l, t); g.kind = 1u + CSB_CELL_LSTM; }
                else { g.h_in = h_buf(l, t - 1); g.kind = kGateRbReset; }
                calls[i] = SpmvGatedCall{r->Wp[l], g, (uint32_t)H, plain_src(g.a), lstmp ? r_of(l, t) : sums2(l, t), part_of(l, 1)};
            }
            int rc = spmv_gated_multi(calls, n, st);
            if (rc != CSB_OK) return rc;
        }
    }
    // the last step's cells have no consumer: apply them here, into the caller's state arrays
    for (int l = 0; l < L; ++l) {
        if (lstmp) {
            init_state(d_hT + (size_t)l * HS, r_of(l, T - 1), (size_t)HS, st);
            if (d_cT) init_state(d_cT + (size_t)l * H, c_of(l, T - 1), (size_t)H, st);
            continue;
        }
        GateSrc g = cell_output(l, T - 1);
        g.h_out = d_hT + (size_t)l * H;
        g.c_out = (lstm && d_cT) ? d_cT + (size_t)l * H : nullptr;
        int rc = commit_gates(g, st);
        if (rc != CSB_OK) return rc;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

extern "C" int csb_rnn_forward(const csb_rnn *r, const float *d_x, const float *d_h0, const float *d_c0,
                               float *d_hseq, float *d_hT, float *d_cT, int32_t T, int32_t batch,
                               void *d_ws, void *stream) {
    using namespace csb;
    // The streaming path at batch 1 on row-owned plans is launch-bound, and every launch of it
    // follows from the arguments alone.  The second call in a row with the same arguments records
    // its launches into a HIP graph (on a stream of the handle's own), the calls after it replay
    // the graph on the caller's stream: a replayed launch costs less than an enqueued one.  The
    // buffers' contents are free to change between the calls; other arguments, a new upload of
    // a matrix, or a caller who is capturing `stream` himself, and the call enqueues as ever.
    hipStream_t st = (hipStream_t)stream;
    bool graphable = r && r->knob_graph && !r->fwd_failed && batch == 1 && T > 0 && d_x && d_hT && d_ws && (uintptr_t)d_ws % 256 == 0 &&
                     !(r->plan.valid && r->uploaded);
    if (graphable) {
        for (auto *m : r->W) graphable = graphable && m->plan.valid && m->uploaded && m->plan.stream.valid;
        for (auto *m : r->Wp) graphable = graphable && m->plan.valid && m->uploaded && m->plan.stream.valid;
    }
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (graphable && (hipStreamIsCapturing(st, &capturing) != hipSuccess || capturing != hipStreamCaptureStatusNone)) {
        (void)hipGetLastError();
        graphable = false;
    }
    if (!graphable) return rnn_forward_enqueue(r, d_x, d_h0, d_c0, d_hseq, d_hT, d_cT, T, batch, d_ws, stream);
    std::vector<uint64_t> key = {(uint64_t)(uintptr_t)d_x, (uint64_t)(uintptr_t)d_h0, (uint64_t)(uintptr_t)d_c0, (uint64_t)(uintptr_t)d_hseq,
                                 (uint64_t)(uintptr_t)d_hT, (uint64_t)(uintptr_t)d_cT, (uint64_t)(uintptr_t)d_ws, (uint64_t)T};
    for (auto *m : r->W) { key.push_back((uint64_t)(uintptr_t)m->d_buf); key.push_back(m->upload_serial); }
    for (auto *m : r->Wp) { key.push_back((uint64_t)(uintptr_t)m->d_buf); key.push_back(m->upload_serial); }
    if (r->fwd_exec && key == r->fwd_key) {
        workspace_changed_hands(d_ws, r);                    // (this handle is the workspace's user again)
        hipError_t e = hipGraphLaunch(r->fwd_exec, st);
        if (e != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
        return CSB_OK;
    }
    if (key != r->fwd_last) {                                // new arguments: an ordinary call, remembered
        r->fwd_last = key;
        return rnn_forward_enqueue(r, d_x, d_h0, d_c0, d_hseq, d_hT, d_cT, T, batch, d_ws, stream);
    }
    // the same arguments as the call before: record, then replay
    if (r->fwd_exec) { (void)hipGraphExecDestroy(r->fwd_exec); r->fwd_exec = nullptr; r->fwd_key.clear(); }
    if (!r->fwd_cap && hipStreamCreateWithFlags(&r->fwd_cap, hipStreamNonBlocking) != hipSuccess) {
        (void)hipGetLastError();
        r->fwd_cap = nullptr;
        return rnn_forward_enqueue(r, d_x, d_h0, d_c0, d_hseq, d_hT, d_cT, T, batch, d_ws, stream);
    }
    hipGraph_t graph = nullptr;
    int rc = CSB_EDEVICE;
    if (hipStreamBeginCapture(r->fwd_cap, hipStreamCaptureModeRelaxed) == hipSuccess) {
        rc = rnn_forward_enqueue(r, d_x, d_h0, d_c0, d_hseq, d_hT, d_cT, T, batch, d_ws, (void *)r->fwd_cap);
        if (hipStreamEndCapture(r->fwd_cap, &graph) != hipSuccess) { graph = nullptr; if (rc == CSB_OK) rc = CSB_EDEVICE; }
    }
    if (rc == CSB_OK && graph && hipGraphInstantiate(&r->fwd_exec, graph, nullptr, nullptr, 0) == hipSuccess) {
        (void)hipGraphDestroy(graph);
        r->fwd_key = key;
        hipError_t e = hipGraphLaunch(r->fwd_exec, st);
        if (e != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
        return CSB_OK;
    }
    // recording failed (or the call is in error, which the ordinary call below reports): nothing has run
    // yet; enqueue as ever, and this handle does not try again
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipGetLastError();
    r->fwd_exec = nullptr;
    r->fwd_failed = true;
    return rnn_forward_enqueue(r, d_x, d_h0, d_c0, d_hseq, d_hT, d_cT, T, batch, d_ws, stream);
}

extern "C" void csb_rnn_free(csb_rnn *r) { delete r; }
