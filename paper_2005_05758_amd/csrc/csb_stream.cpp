// Row-owned stream section of the device image (host only): the layout csb_spmv reads.
//
// Role in the method: Sec. 4.3.1's CSB-MVM sweeps the blocks, multiplies every kernel matrix
// with the inputs its column indices name and accumulates at its row indices; Sec. 5.2 asks
// that every parallel unit gets the same share of that uneven work.  Here a workgroup owns a
// range of output rows outright (so no sum ever crosses workgroups), the kernel-matrix rows
// that land in the range are sorted by column count, packed 64 to a group (one per lane) and
// the groups' column steps are cut into equal ranges, one per wavefront and round.  Every
// wavefront's share is written as one self-contained segment of fixed size, so that a launch
// can request all of its bytes at once from addresses that depend on nothing but the
// workgroup and wavefront numbers.
#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>

#include "csb_internal.hpp"

namespace csb {
namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Default size of a workgroup's share: four 64-lane groups, cut along their column steps into a
// piece per wavefront.  Small matrices spread over more compute units and their wavefronts get
// short runs (measured, us per launch warm, 1024 / 512 / 256 / 128 lanes per workgroup: 2048 x 665:
// 3.67 / 3.43 / 3.16 / 3.16; streaming LSTM step on it 5.15 / 4.87 / 4.57 / 4.53; LSTMP step
// 11.3 / 11.1 / 10.7 / 12.2); large matrices are capped at 256 workgroups anyway.
constexpr uint64_t kLanesPerWg = 256;

// One virtual block of a workgroup: kernel-matrix rows [a0, a1) of CSB block b.
// With a GRU row split (SplitSpec) a block below the split row comes as two: its columns in
// front of the split column (summed into the row itself) and those from it on (summed into
// row + shift); q0 is the first column position of the part inside the block's column list.
struct SVb {
    uint32_t b;
    uint16_t a0, a1;
    uint16_t c;       // columns of the part
    uint16_t q0;
    uint16_t hi;      // 1: the part that is summed into row + shift
    int32_t radj;     // local row of the workgroup = output row + radj
};

struct Lane {
    uint32_t vb;      // index into the workgroup's SVb list
    uint16_t a;       // kernel-matrix row inside the CSB block
    uint16_t rr;      // output row - row0
};

// A piece of a wavefront share: column steps [j0, j1) of group g (lanes [64 g, 64 g + 64) of the
// workgroup's sorted lane sequence); nl lanes of the group still have columns at step j0.
struct Piece {
    uint32_t g;
    uint16_t j0, j1;
    uint16_t nl;
};

struct Share {
    std::vector<Piece> pieces;
    uint32_t bytes = 0;
    double work = 0;
};

struct WgLayout {
    uint32_t row0 = 0, nrows = 0;
    std::vector<SVb> vbs;
    std::vector<Lane> lanes;                       // sorted by column count, descending
    std::vector<uint32_t> g_cmax;                  // column steps of every 64-lane group
    std::vector<Share> share;                      // [n_rounds * 16], round-major
    uint32_t kmax = 0;
};

struct SegSize {
    size_t groups = 0, vbs = 0, lane_bytes = 0, list_bytes = 0, steps = 0;
    size_t vbytes = 4;                                    // bytes of one kernel value (4, or 2 in a 16-bit format)
    size_t list_pos() const { return sizeof(StreamSegHdr) + groups * sizeof(StreamGroup) + vbs * 4 + lane_bytes; }
    size_t total() const { return align_up(list_pos() + list_bytes, 16) + steps * kWave * vbytes; }
};

// Walks the virtual blocks of one piece: f(vb index, first lane of the run inside the group, rows, columns kept).
template <typename F>
void for_piece_vbs(const WgLayout &w, const Piece &p, F f) {
    const uint32_t l0 = p.g * kWave;
    uint32_t l = l0;
    while (l < l0 + p.nl) {
        const uint32_t vb = w.lanes[l].vb;
        uint32_t e = l + 1;
        while (e < l0 + p.nl && w.lanes[e].vb == vb) ++e;
        const int ck = std::min<int>(w.vbs[vb].c, p.j1) - (int)p.j0;
        f(vb, l - l0, e - l, ck);
        l = e;
    }
}

SegSize piece_size(const WgLayout &w, const Piece &p, size_t vbytes) {
    SegSize s;
    s.vbytes = vbytes;
    s.groups = 1;
    s.steps = (size_t)(p.j1 - p.j0);
    const size_t list_len = align_up(s.steps, 4);        // every list is padded to the piece's steps
    for_piece_vbs(w, p, [&](uint32_t, uint32_t, uint32_t, int) {
        s.vbs += 1;
        s.list_bytes += list_len;
    });
    s.lane_bytes = align_up(2 * (size_t)p.nl, 4);
    return s;
}

}  // namespace

// Builds the stream section for `m` and appends it to the plan's image.  Returns CSB_OK and
// leaves plan.stream.valid false when the matrix does not fit the layout (the caller then
// keeps the tile-based sections for the mat-vec as well).
int plan_stream(csb_matrix *m, int32_t n_wg_req, int32_t rounds_min, csb_plan_stats *stats_out) {
    Plan &pl = m->plan;
    pl.stream = StreamPlan{};
    const SplitSpec split = pl.split;
    // (a split whose shifted rows do not start where the matrix ends would interleave them with others: not laid out here)
    if (split.active() && (split.split_row + split.shift != m->rows || split.split_row < 0 || split.split_row > m->rows)) return CSB_OK;
    const size_t vbytes = m->val_fmt == CSB_VAL_F32 ? 4 : 2;
    if (m->cols > kMaxStageCols || m->rows + (split.active() ? split.shift : 0) > 0x7fffffff) return CSB_OK;
    try {
        const int br = m->br;
        const int64_t R = m->rows + (split.active() ? split.shift : 0);    // output rows
        // cell mode: workgroups own units (with all their gate rows) instead of row ranges
        const int64_t G = m->stream_cell_gates > 0 && R % m->stream_cell_gates == 0 && kStreamMaxRows >= m->stream_cell_gates ? m->stream_cell_gates : 0;
        const int64_t U = G ? R / G : 0;                                    // units
        if (G && split.active() && (split.split_row % U != 0 || split.shift % U != 0)) return CSB_OK;   // (a gate's rows lie in one zone)
        // position of the split column in a block's column list (all of it without a split)
        auto split_pos = [&](size_t b, int32_t bj) {
            const int nc = m->ncols[b];
            if (!split.active()) return nc;
            const uint16_t *ci = m->colidx.data() + m->col_off[b];
            int qs = 0;
            while (qs < nc && (int64_t)bj * m->bc + ci[qs] < split.split_col) ++qs;
            return qs;
        };

        // ---- 1. bytes each output row brings along, lanes in all ---------------------------
        std::vector<uint32_t> roww((size_t)R, 0);
        uint64_t lanes_total = 0;
        for (int32_t bi = 0; bi < m->nbr; ++bi)
            for (int32_t bj = 0; bj < m->nbc; ++bj) {
                const size_t b = (size_t)bi * m->nbc + bj;
                const int nr = m->nrows[b], nc = m->ncols[b];
                if (nr == 0 || nc == 0) continue;
                const uint16_t *ri = m->rowidx.data() + m->row_off[b];
                const int qs = split_pos(b, bj);
                for (int a = 0; a < nr; ++a) {
                    const int64_t g = (int64_t)bi * br + ri[a];
                    if (!split.active() || g < split.split_row) {
                        roww[(size_t)g] += (uint32_t)nc + (uint32_t)kStreamGroupOverhead;
                        ++lanes_total;
                        continue;
                    }
                    if (qs > 0) { roww[(size_t)g] += (uint32_t)qs + (uint32_t)kStreamGroupOverhead; ++lanes_total; }
                    if (nc > qs) { roww[(size_t)(g + split.shift)] += (uint32_t)(nc - qs) + (uint32_t)kStreamGroupOverhead; ++lanes_total; }
                }
            }
        // Steps 2 to 4 run several times: first with the rows weighted by the work they bring
        // (column steps plus the per-piece overhead, per lane), then with corrected weights (below).
        std::vector<double> rw(roww.begin(), roww.end());
        std::vector<uint32_t> cut;      // row boundaries: workgroup k owns [cut[k], cut[k+1])
        std::vector<WgLayout> W;
        uint32_t nwg = 0, rows_max = 0, hdr_bytes = 0, tpr = 0;
        // (the cell form of the kernel keeps its row sums where the input vector was)
        const uint32_t x_bytes = std::max<uint32_t>((uint32_t)align_up((size_t)m->cols * 4, 16), G ? 4u * (uint32_t)kStreamMaxRows : 0u);
        StreamPlan sp{};
        bool found = false;
        uint32_t nr_start = 1;
        auto attempt = [&]() {
        double total_w = 0;
        for (double v : rw) total_w += v;

        // ---- 2. row ranges of the workgroups: nearly equal weight, cut at any row ----------
        // (cell mode: the same over units, a unit weighing what its gate rows weigh)
        const int64_t NI = G ? U : R;                                   // items that are cut: units or rows
        const int64_t max_items = G ? kStreamMaxRows / G : kStreamMaxRows;
        auto item_w = [&](int64_t i) {
            if (!G) return rw[(size_t)i];
            double v = 0;
            for (int64_t g = 0; g < G; ++g) v += rw[(size_t)(g * U + i)];
            return v;
        };
        int64_t n_wg = n_wg_req > 0 ? n_wg_req : (int64_t)std::min<uint64_t>((uint64_t)std::max(1, std::min(256, m->stream_wg_limit)), std::max<uint64_t>(1, (lanes_total + kLanesPerWg - 1) / kLanesPerWg));
        n_wg = std::max<int64_t>(n_wg, (NI + max_items - 1) / max_items);
        n_wg = std::min<int64_t>(n_wg, NI);
        cut.clear();
        cut.push_back(0);
        {
            double acc = 0;              // weight of the rows before `row`
            int64_t k = 0;               // workgroup being filled
            for (int64_t row = 0; row < NI; ++row) {
                const int64_t rows_here = row - (int64_t)cut.back();
                const double wrow = item_w(row);
                if (rows_here > 0) {
                    bool close = rows_here == max_items;
                    if (!close && k + 1 < n_wg) {
                        // the boundary in front of this row is nearer to the k-th target than the one behind it
                        const double target = total_w * (double)(k + 1) / (double)n_wg;
                        close = acc + wrow / 2 >= target;
                    }
                    if (close) { cut.push_back((uint32_t)row); ++k; }
                }
                acc += wrow;
            }
            cut.push_back((uint32_t)NI);
        }
        nwg = (uint32_t)cut.size() - 1;

        // ---- 3. per workgroup: virtual blocks and kernel-matrix rows by descending column count,
        //         64 to a group: the lanes of a group then have (nearly) the same column count ----
        W.assign(nwg, WgLayout{});
        rows_max = 0;
        for (uint32_t k = 0; k < nwg; ++k) {
            WgLayout &w = W[k];
            w.row0 = cut[k];
            w.nrows = (cut[k + 1] - cut[k]) * (uint32_t)(G ? G : 1);
            rows_max = std::max(rows_max, w.nrows);
            // the workgroup's output rows come from up to three zones of the matrix: rows in front
            // of the split row (all columns), rows from it on (their columns in front of the split
            // column), and the same rows once more, relabelled (their columns from it on); in cell
            // mode from as many per gate (local rows: gate-major)
            struct Zone { int64_t o0, o1, back; int part; int64_t loc; };      // output rows [o0, o1) = matrix rows - back; part 0 all, 1 low, 2 high; local row of o0
            std::vector<Zone> zones;
            auto add_range = [&](int64_t r0, int64_t r1, int64_t loc) {
                if (!split.active()) { zones.push_back(Zone{r0, r1, 0, 0, loc}); return; }
                const int64_t sr = split.split_row, mr = m->rows;
                if (r0 < std::min(r1, sr)) zones.push_back(Zone{r0, std::min(r1, sr), 0, 0, loc});
                if (std::max(r0, sr) < std::min(r1, mr)) zones.push_back(Zone{std::max(r0, sr), std::min(r1, mr), 0, 1, loc + std::max(r0, sr) - r0});
                if (std::max(r0, mr) < r1) zones.push_back(Zone{std::max(r0, mr), r1, split.shift, 2, loc + std::max(r0, mr) - r0});
            };
            if (!G) add_range(cut[k], cut[k + 1], 0);
            else {
                const int64_t nu = (int64_t)cut[k + 1] - cut[k];
                for (int64_t g = 0; g < G; ++g) add_range(g * U + cut[k], g * U + cut[k + 1], g * nu);
            }
            for (size_t zi = 0; zi < zones.size(); ++zi) {
                const Zone &z = zones[zi];
                const int64_t g0 = z.o0 - z.back, g1 = z.o1 - z.back;          // matrix rows
                for (int64_t bi = g0 / br; bi <= (g1 - 1) / br; ++bi)
                    for (int32_t bj = 0; bj < m->nbc; ++bj) {
                        const size_t b = (size_t)bi * m->nbc + bj;
                        const int nr = m->nrows[b], nc = m->ncols[b];
                        if (nr == 0 || nc == 0) continue;
                        const int qs = z.part == 0 ? nc : split_pos(b, bj);
                        const int q0 = z.part == 2 ? qs : 0, q1 = z.part == 1 ? qs : nc;
                        if (q1 <= q0) continue;
                        const uint16_t *ri = m->rowidx.data() + m->row_off[b];
                        int a0 = 0;
                        while (a0 < nr && bi * br + ri[a0] < g0) ++a0;
                        int a1 = a0;
                        while (a1 < nr && bi * br + ri[a1] < g1) ++a1;
                        if (a1 > a0) w.vbs.push_back(SVb{(uint32_t)b, (uint16_t)a0, (uint16_t)a1, (uint16_t)(q1 - q0), (uint16_t)q0, (uint16_t)(z.part == 2 ? 1 : 0), (int32_t)(z.loc - z.o0)});
                    }
            }
            std::stable_sort(w.vbs.begin(), w.vbs.end(), [](const SVb &x, const SVb &y) { return x.c > y.c; });
            for (uint32_t v = 0; v < w.vbs.size(); ++v) {
                const SVb &vb = w.vbs[v];
                const int64_t bi = vb.b / m->nbc;
                const uint16_t *ri = m->rowidx.data() + m->row_off[vb.b];
                for (int a = vb.a0; a < vb.a1; ++a)
                    w.lanes.push_back(Lane{v, (uint16_t)a, (uint16_t)(bi * br + ri[a] + (vb.hi ? split.shift : 0) + vb.radj)});
            }
            for (uint32_t l0 = 0; l0 < w.lanes.size(); l0 += kWave) w.g_cmax.push_back(w.vbs[w.lanes[l0].vb].c);
        }

        // ---- 4. rounds: the smallest count whose segments and partial sums fit the LDS ------
        hdr_bytes = (uint32_t)(sizeof(StreamRoundHdr) + align_up(4 * (size_t)rows_max, 16));
        uint32_t rows_pad = 1;
        while (rows_pad < rows_max) rows_pad <<= 1;
        tpr = std::min<uint32_t>(kWave, (uint32_t)kStreamThreads / rows_pad);
        sp = StreamPlan{};
        found = false;
        // room for one segment if the partial sums took what the lanes and some cut pieces need
        size_t lanes_max = 0;
        for (const WgLayout &w : W) lanes_max = std::max(lanes_max, w.lanes.size());
        const size_t fixed_lds = (size_t)x_bytes + hdr_bytes + 1024 + align_up(4 * (lanes_max + 24 * kWave), 16);
        const size_t seg_room = fixed_lds + 16 * 1024 < (size_t)kLdsBudget
            ? std::min<size_t>((size_t)kStreamMaxSegUnits * 1024, ((size_t)kLdsBudget - fixed_lds) / kStreamWaves / 16 * 16) : 1024;
        // trials: rounds from the smallest on; per round count, smaller and smaller pieces while the
        // largest piece is what keeps the segments from fitting
        uint32_t NR = std::max<uint32_t>(nr_start, (uint32_t)std::max(1, rounds_min)), shrink = 0;
        for (; NR <= 64 && !found;) {
            const uint32_t N = NR * kStreamWaves;
            uint32_t seg_max = 0, kmax = 0;
            size_t piece_max = 0;
            bool ok = true, list_ok = true;
            if (seg_room < 1024 + 512 * (size_t)shrink) break;
            const size_t kPieceCap = seg_room - 512 * (size_t)shrink - sizeof(StreamSegHdr) - 16;
            for (uint32_t k = 0; k < nwg && ok; ++k) {
                WgLayout &w = W[k];
                const uint32_t G = (uint32_t)w.g_cmax.size();
                // Equal work per wavefront: the groups' column steps are dealt to the 16 wavefronts, work
                // being steps plus a fixed overhead per piece of a group (a piece is at least two steps
                // long and its bytes fit one segment).  A wavefront is filled greedily up to a budget
                // S: a group that does not fit is cut where the budget ends and goes on with the next
                // wavefront; when a new group is started, the first one (in the order widest,
                // narrowest, second widest, ... so that wavefronts get a mix of long and short pieces)
                // that fills the rest of the budget exactly is taken, else the first that leaves room
                // for another piece or overflows (and is cut), and only then one that would leave a
                // rest too small to use.  S is the smallest budget with which everything is placed
                // (such a walk is not monotone in S: S goes up one by one from the lower bound).
                // The pieces of a wavefront are then dealt to its NR rounds in order, so that the
                // largest segment is as small as can be; segments are read up to their own length,
                // so their bytes need not be equal; the longest sets the LDS need.
                std::vector<uint32_t> order(G);
                for (uint32_t i = 0, lo = 0, hi = G; i < G; ++i) order[i] = (i & 1u) ? --hi : lo++;
                std::vector<uint8_t> done(G);
                constexpr uint64_t kOv = kStreamGroupOverhead;
                // lanes and virtual blocks of group g that still have columns at step j
                auto live = [&](uint32_t g, uint32_t j, uint32_t *nl_out, uint32_t *nvb_out) {
                    const uint32_t l0 = g * kWave, l1 = std::min<uint32_t>(l0 + kWave, (uint32_t)w.lanes.size());
                    uint32_t nl = 0, nvb = 0;
                    while (l0 + nl < l1 && w.vbs[w.lanes[l0 + nl].vb].c > j) {
                        if (nl == 0 || w.lanes[l0 + nl].vb != w.lanes[l0 + nl - 1].vb) ++nvb;
                        ++nl;
                    }
                    *nl_out = nl; *nvb_out = nvb;
                };
                std::vector<std::vector<Piece>> wave_pieces(kStreamWaves);
                auto walk = [&](uint64_t S, bool emit) {
                    uint32_t placed = 0, j = 0, used = 0, first_open = 0;
                    int64_t cur = -1;
                    std::fill(done.begin(), done.end(), (uint8_t)0);
                    if (emit) for (auto &v : wave_pieces) v.clear();
                    while (placed < G) {
                        if (used == (uint32_t)kStreamWaves) return false;
                        uint64_t budget = S;
                        while (placed < G) {
                            if (cur < 0) {
                                while (first_open < G && done[order[first_open]]) ++first_open;
                                int64_t exact = -1, roomy = -1, any = -1;
                                for (uint32_t i = first_open; i < G && exact < 0; ++i) {
                                    const uint32_t g = order[i];
                                    if (done[g]) continue;
                                    const uint64_t need = kOv + w.g_cmax[g];
                                    if (budget < kOv + std::min<uint32_t>(w.g_cmax[g], 2u)) continue;   // cannot even start it
                                    if (any < 0) any = g;
                                    if (need == budget) exact = g;
                                    else if (roomy < 0 && (need + kOv + 2 <= budget || (need > budget && need - budget >= 2))) roomy = g;
                                }
                                cur = exact >= 0 ? exact : roomy >= 0 ? roomy : any;
                                if (cur < 0) break;                              // nothing can start in what is left
                                j = 0;
                            }
                            const uint32_t g = (uint32_t)cur;
                            const uint32_t left = w.g_cmax[g] - j;
                            if (budget < kOv + std::min<uint32_t>(left, 2u)) break;
                            uint32_t nl, nvb;
                            live(g, j, &nl, &nvb);
                            // steps whose bytes (record, block words, lane words, padded lists, values) fit a segment
                            const size_t fixed = sizeof(StreamGroup) + 4 * (size_t)nvb + align_up(2 * (size_t)nl, 4) + 3 * (size_t)nvb;
                            const uint32_t fit = (uint32_t)((kPieceCap - std::min(kPieceCap, fixed)) / (kWave * vbytes + nvb));
                            if (fit < std::min<uint32_t>(left, 2u)) return false;
                            uint32_t take = (uint32_t)std::min<uint64_t>(std::min(left, fit), budget - kOv);
                            if (left - take == 1u) --take;                   // never leave a one-step piece behind
                            if (take < std::min<uint32_t>(left, 2u)) break;
                            if (emit) wave_pieces[used].push_back(Piece{g, (uint16_t)j, (uint16_t)(j + take), (uint16_t)nl});
                            budget -= kOv + take;
                            j += take;
                            if (j == w.g_cmax[g]) { done[g] = 1; ++placed; cur = -1; }
                        }
                        ++used;
                    }
                    return true;
                };
                uint64_t steps_all = 0;
                for (uint32_t g = 0; g < G; ++g) steps_all += w.g_cmax[g];
                uint64_t S = std::max<uint64_t>(kOv + 2, (steps_all + kOv * G + kStreamWaves - 1) / kStreamWaves);
                const uint64_t S_stop = steps_all + kOv * G + kOv * kStreamWaves + 64;    // one wavefront could take it all
                while (S <= S_stop && !walk(S, false)) ++S;
                if (S > S_stop) { ok = false; break; }
                walk(S, true);
                // deal every wavefront's pieces to its rounds: the smallest limit on a round's bytes
                // with which NR runs in order hold them all
                w.share.assign(N, Share{});
                for (uint32_t wv = 0; wv < (uint32_t)kStreamWaves; ++wv) {
                    const std::vector<Piece> &pc = wave_pieces[wv];
                    std::vector<size_t> pb(pc.size());
                    size_t lo = 0, hi = 0;
                    for (size_t i = 0; i < pc.size(); ++i) { pb[i] = piece_size(w, pc[i], vbytes).total(); lo = std::max(lo, pb[i]); hi += pb[i]; }
                    piece_max = std::max(piece_max, lo);
                    auto runs_needed = [&](size_t limit) {
                        uint32_t runs = 1; size_t acc = 0;
                        for (size_t v : pb) { if (acc + v > limit && acc > 0) { ++runs; acc = 0; } acc += v; }
                        return runs;
                    };
                    while (lo < hi) { const size_t mid = (lo + hi) / 2; if (runs_needed(mid) <= NR) hi = mid; else lo = mid + 1; }
                    uint32_t r = 0; size_t acc = 0;
                    for (size_t i = 0; i < pc.size(); ++i) {
                        if (acc + pb[i] > lo && acc > 0) { ++r; acc = 0; }
                        acc += pb[i];
                        Share &sh = w.share[(size_t)r * kStreamWaves + wv];
                        sh.pieces.push_back(pc[i]);
                        sh.work += (double)(kOv + (pc[i].j1 - pc[i].j0));
                    }
                }
                // sizes, and the number of partial sums (one per lane and piece)
                w.kmax = 0;                                     // here: partial sums of the workgroup
                for (uint32_t s = 0; s < N; ++s) {
                    Share &sh = w.share[s];
                    SegSize tot;
                    tot.vbytes = vbytes;
                    for (const Piece &p : sh.pieces) {
                        const SegSize ps = piece_size(w, p, vbytes);
                        tot.groups += ps.groups; tot.vbs += ps.vbs; tot.lane_bytes += ps.lane_bytes;
                        tot.list_bytes += ps.list_bytes; tot.steps += ps.steps;
                        w.kmax += p.nl;
                    }
                    sh.bytes = (uint32_t)align_up(tot.total(), 16);
                    seg_max = std::max(seg_max, sh.bytes);
                    if (tot.list_pos() + tot.list_bytes > (size_t)kStreamListLimit) list_ok = false;   // 10-bit list word index
                }
                kmax = std::max(kmax, w.kmax);
                if (w.kmax > 65535u) ok = false;                // a lane names its slot in 16 bits
            }
            const uint32_t kstride = std::max(1u, kmax);     // partial-sum slots of the fullest workgroup
            // (1 KiB of slack behind the segments: a padded list byte may name an input up to 255 floats past a block's first)
            const size_t lds = (size_t)x_bytes + hdr_bytes + align_up((size_t)kstride * 4, 16) + (size_t)kStreamWaves * seg_max + 1024;
            if (!ok) break;                                  // more rounds do not shrink what failed
            if (!list_ok || seg_max > (uint32_t)kStreamMaxSegUnits * 1024u || lds > (size_t)kLdsBudget) {
                // segments of one piece: smaller pieces help; else more rounds do
                if ((size_t)seg_max <= piece_max + sizeof(StreamSegHdr) + 16 && shrink < 10) ++shrink; else { ++NR; }
                continue;
            }
            sp.n_wg = nwg; sp.n_rounds = NR; sp.seg_bytes = seg_max; sp.hdr_bytes = hdr_bytes;
            sp.wg_bytes = (uint32_t)align_up((size_t)hdr_bytes + (size_t)N * seg_max, 256);
            sp.kmax = kstride; sp.rows_max = rows_max; sp.tpr = tpr; sp.lds_bytes = (uint32_t)lds;
            found = true;
        }
        };   // attempt

        // largest wavefront work of a workgroup
        auto wg_max = [&](const WgLayout &w) {
            double v = 0;
            for (uint32_t wv = 0; wv < (uint32_t)kStreamWaves; ++wv) {
                double ww = 0;
                for (uint32_t r = 0; r < sp.n_rounds; ++r) ww += w.share[(size_t)r * kStreamWaves + wv].work;
                v = std::max(v, ww);
            }
            return v;
        };
        attempt();
        if (!found) return CSB_OK;
        nr_start = sp.n_rounds;                                 // the later passes do not look below it
        if (nwg > 1) {
            // Feedback on the row cuts: a workgroup whose fullest wavefront is above the average gives
            // rows away (its rows weigh more in the next pass).  The best pass is kept: the one with
            // the smallest largest wavefront work, then the smallest sum of the workgroups' largest.
            std::vector<double> best_rw = rw;
            double best_max = 0, best_sum = 0;
            for (const WgLayout &w : W) { const double v = wg_max(w); best_max = std::max(best_max, v); best_sum += v; }
            bool last_is_best = true;
            for (int pass = 0; pass < 8 && best_max * nwg > best_sum * 1.02; ++pass) {
                double sum = 0;
                for (const WgLayout &w : W) sum += wg_max(w);
                const double target = sum / nwg;
                for (uint32_t k = 0; k < nwg; ++k) {
                    const double f = 1.0 + 0.7 * (wg_max(W[k]) / target - 1.0);
                    for (uint32_t r = cut[k]; r < cut[k + 1]; ++r)
                        for (int64_t g = 0; g < (G ? G : 1); ++g) rw[(size_t)(g * U + r)] *= f;
                }
                attempt();
                last_is_best = false;
                if (!found) break;
                double mx = 0, sm = 0;
                for (const WgLayout &w : W) { const double v = wg_max(w); mx = std::max(mx, v); sm += v; }
                if (mx < best_max || (mx == best_max && sm < best_sum)) { best_max = mx; best_sum = sm; best_rw = rw; last_is_best = true; }
            }
            if (!last_is_best) { rw = best_rw; attempt(); }
            if (!found) return CSB_OK;
        }

        // ---- 5. write the section -----------------------------------------------------------
        const size_t off = align_up(pl.image.size(), 256);
        const size_t bytes = (size_t)sp.n_wg * sp.wg_bytes;
        pl.image.resize(off + bytes, 0);
        sp.off = off; sp.bytes = bytes;
        uint32_t n_groups = 0;
        uint64_t fma_steps = 0, traffic = (uint64_t)nwg * sp.hdr_bytes;
        for (uint32_t k = 0; k < nwg; ++k) {
            const WgLayout &w = W[k];
            uint8_t *wb = pl.image.data() + off + (size_t)k * sp.wg_bytes;
            StreamRoundHdr rh{};
            rh.row0 = w.row0; rh.nrows = w.nrows;
            // partial sums: a row's slots are consecutive; (first slot, count) per row goes into the header
            std::vector<uint32_t> cnt(w.nrows, 0u), first(w.nrows, 0u), next(w.nrows, 0u);
            for (const Share &sh : w.share)
                for (const Piece &p : sh.pieces)
                    for (uint32_t l = 0; l < p.nl; ++l) ++cnt[w.lanes[p.g * kWave + l].rr];
            for (uint32_t i = 1; i < w.nrows; ++i) first[i] = first[i - 1] + cnt[i - 1];
            next = first;
            for (uint32_t s = 0; s < sp.n_rounds * (uint32_t)kStreamWaves; ++s) {
                const Share &sh = w.share[s];
                uint8_t *seg = wb + sp.hdr_bytes + (size_t)s * sp.seg_bytes;
                SegSize tot;
                for (const Piece &p : sh.pieces) {
                    const SegSize ps = piece_size(w, p, vbytes);
                    tot.groups += ps.groups; tot.vbs += ps.vbs; tot.lane_bytes += ps.lane_bytes; tot.list_bytes += ps.list_bytes;
                }
                StreamSegHdr hd{};
                hd.ng = (uint16_t)sh.pieces.size();
                const size_t off_groups = sizeof(StreamSegHdr);
                const size_t off_vbs = off_groups + sh.pieces.size() * sizeof(StreamGroup);
                size_t lane_pos = off_vbs + tot.vbs * 4;
                size_t list_pos = lane_pos + tot.lane_bytes;
                size_t val_pos = align_up(list_pos + tot.list_bytes, 16) / 4;    // float index
                hd.off_vbs = (uint16_t)off_vbs;
                hd.bytes16 = (uint16_t)(sh.bytes / 16);
                if (s + kStreamWaves < sp.n_rounds * (uint32_t)kStreamWaves) hd.next16 = (uint16_t)(w.share[s + kStreamWaves].bytes / 16);
                traffic += sh.bytes;
                std::memcpy(seg, &hd, sizeof(hd));
                uint32_t vb_idx = 0;
                for (size_t gi = 0; gi < sh.pieces.size(); ++gi) {
                    const Piece &p = sh.pieces[gi];
                    const uint32_t steps = (uint32_t)(p.j1 - p.j0), l0 = p.g * kWave;
                    const size_t list_len = align_up(steps, 4);
                    StreamGroup sg{};
                    sg.vb0 = (uint16_t)vb_idx;
                    sg.cmax_minus_1 = (uint8_t)(steps - 1);
                    sg.lane_off = (uint16_t)lane_pos;
                    sg.val_off = (uint16_t)val_pos;
                    sg.nlanes = (uint8_t)p.nl;
                    uint8_t *dst = seg + val_pos * 4;                  // [steps][64] values (32 or 16 bits), zero where a lane has no column
                    for_piece_vbs(w, p, [&](uint32_t v, uint32_t lane0, uint32_t rws, int ck) {
                        const SVb &vb = w.vbs[v];
                        sg.start_mask |= 1ull << lane0;
                        const uint32_t word = stream_vb_word((uint32_t)(list_pos / 4), (uint32_t)(ck - 1), vb.b % (uint32_t)m->nbc);
                        std::memcpy(seg + off_vbs + (size_t)vb_idx * 4, &word, 4);
                        ++vb_idx;
                        // column indices; behind them, up to the piece's steps, the slice's first column again:
                        // an input every row of the block multiplies anyway (so a non-finite input
                        // reaches only rows that use it), here with values stored as zeros
                        const uint16_t *ci = m->colidx.data() + m->col_off[vb.b] + vb.q0 + p.j0;
                        for (size_t j = 0; j < list_len; ++j) seg[list_pos + j] = (uint8_t)ci[j < (size_t)ck ? j : 0];
                        list_pos += list_len;
                        const float *kv = m->val.data() + m->val_off[vb.b];
                        for (uint32_t i = 0; i < rws; ++i) {
                            const Lane &ln = w.lanes[l0 + lane0 + i];
                            for (int j = 0; j < ck; ++j) {
                                const float v = kv[(size_t)ln.a * m->ncols[vb.b] + vb.q0 + p.j0 + j];
                                const size_t at = (size_t)j * kWave + lane0 + i;
                                if (vbytes == 4) std::memcpy(dst + at * 4, &v, 4);
                                else {
                                    const uint16_t b16 = m->val_fmt == CSB_VAL_F16 ? f32_to_f16_bits(v) : f32_to_bf16_bits(v);
                                    std::memcpy(dst + at * 2, &b16, 2);
                                }
                            }
                            const uint16_t lw = (uint16_t)next[ln.rr]++;
                            std::memcpy(seg + lane_pos + 2 * (size_t)(lane0 + i), &lw, 2);
                        }
                    });
                    val_pos += (size_t)steps * kWave * vbytes / 4;
                    lane_pos += align_up(2 * (size_t)p.nl, 4);
                    std::memcpy(seg + off_groups + gi * sizeof(StreamGroup), &sg, sizeof(sg));
                    ++n_groups;
                    fma_steps += steps;
                }
            }
            std::memcpy(wb, &rh, sizeof(rh));
            for (uint32_t i = 0; i < w.nrows; ++i) {
                const uint32_t oc = first[i] | (cnt[i] << 16);
                std::memcpy(wb + sizeof(rh) + 4 * (size_t)i, &oc, 4);
            }
        }
        sp.n_groups = n_groups;
        sp.val_fmt = (uint32_t)m->val_fmt;
        sp.cell_gates = (uint32_t)G; sp.cell_units = (uint32_t)U;
        sp.valid = true;
        pl.stream = sp;

        // ---- 6. statistics of the plan csb_spmv will run ------------------------------------
        csb_plan_stats st = pl.stats;
        st.n_chunks = (int32_t)sp.n_wg;
        st.waves_per_chunk = kStreamWaves;
        st.n_groups = (int32_t)n_groups;
        st.n_shared_tiles = 0;
        double wmax = 0, wsum = 0, cmax_ = 0, csum_ = 0;
        for (const WgLayout &w : W) {
            double cc = 0;
            for (uint32_t wv = 0; wv < (uint32_t)kStreamWaves; ++wv) {
                double ww = 0;
                for (uint32_t r = 0; r < sp.n_rounds; ++r) ww += w.share[(size_t)r * kStreamWaves + wv].work;
                wmax = std::max(wmax, ww); wsum += ww; cc += ww;
            }
            cmax_ = std::max(cmax_, cc); csum_ += cc;
        }
        st.work_max = wmax;
        st.work_mean = wsum / ((double)sp.n_wg * kStreamWaves);
        st.chunk_max_over_mean = csum_ > 0 ? cmax_ / (csum_ / sp.n_wg) : 0.0;
        st.lane_fill = fma_steps ? (double)m->val.size() / (64.0 * (double)fma_steps) : 0.0;
        st.whole_tiles = 1;
        st.row_owned = G ? 2 : 1;
        st.rounds = (int32_t)sp.n_rounds;
        st.matvec_bytes = (int64_t)traffic;          // segments are read up to their own length, not the stride
        pl.stats = st;
        if (stats_out) *stats_out = st;
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        pl.stream = StreamPlan{};
        set_error("csb_plan: out of host memory");
        return CSB_ENOMEM;
    }
}

// Walks the stream section the way the kernel does, with bounds checks on every access,
// rebuilds the (row, column) -> value map and compares it with the packed matrix.
int validate_stream(const csb_matrix *m) {
    const Plan &pl = m->plan;
    const StreamPlan &sp = pl.stream;
    auto fail = [&](const char *what) { set_error(std::string("csb_plan_validate (row-owned section): ") + what); return CSB_EINVAL; };
    const uint32_t N = sp.n_rounds * (uint32_t)kStreamWaves;
    if (sp.off + sp.bytes > pl.image.size() || sp.bytes != (size_t)sp.n_wg * sp.wg_bytes) return fail("section size");
    if (sp.seg_bytes % 16 || sp.hdr_bytes % 16 || (size_t)sp.wg_bytes < sp.hdr_bytes + (size_t)N * sp.seg_bytes) return fail("workgroup layout");
    if (sp.seg_bytes > (uint32_t)kStreamMaxSegUnits * 1024u || sp.rows_max > (uint32_t)kStreamMaxRows) return fail("limits");
    if (sp.hdr_bytes < sizeof(StreamRoundHdr) + 4 * (size_t)sp.rows_max) return fail("header size");
    if (sp.tpr == 0 || (sp.tpr & (sp.tpr - 1)) || sp.tpr > (uint32_t)kWave || sp.rows_max * sp.tpr > (uint32_t)kStreamThreads) return fail("threads per row");
    if (sp.val_fmt != (uint32_t)m->val_fmt) return fail("value format");
    const size_t vbytes = sp.val_fmt == CSB_VAL_F32 ? 4 : 2;
    // bits of the value of lane `lane` at step j of a piece whose values start at 4-byte word val_off, widened to float bits
    auto value_bits = [&](const uint8_t *seg, uint32_t val_off, uint32_t j, uint32_t lane) {
        const uint8_t *at = seg + (size_t)val_off * 4 + ((size_t)j * kWave + lane) * vbytes;
        uint32_t bits = 0;
        if (vbytes == 4) { std::memcpy(&bits, at, 4); return bits; }
        uint16_t b16;
        std::memcpy(&b16, at, 2);
        const float f = sp.val_fmt == CSB_VAL_F16 ? f16_bits_to_f32(b16) : bf16_bits_to_f32(b16);
        std::memcpy(&bits, &f, 4);
        return bits;
    };
    const SplitSpec &split = pl.split;
    const int64_t R = m->rows + (split.active() ? split.shift : 0), Ccols = m->cols;     // output rows
    std::vector<float> expect((size_t)R * Ccols, 0.0f), got((size_t)R * Ccols, 0.0f);
    std::vector<uint8_t> seen((size_t)R * Ccols, 0);
    if (csb_unpack(m, expect.data(), Ccols) != CSB_OK) return CSB_EINVAL;
    if (split.active()) {                                 // the relabelling: entries below the split row, from the split column on, move down by `shift` rows
        if (split.split_row + split.shift != m->rows) return fail("row split");
        for (int64_t g = split.split_row; g < m->rows; ++g)
            for (int64_t c = split.split_col; c < Ccols; ++c) {
                expect[(size_t)(g + split.shift) * Ccols + c] = expect[(size_t)g * Ccols + c];
                expect[(size_t)g * Ccols + c] = 0.0f;
            }
    }
    std::vector<uint8_t> row_done((size_t)R, 0);
    size_t vals_used = 0;
    for (uint32_t k = 0; k < sp.n_wg; ++k) {
        const uint8_t *wb = pl.image.data() + sp.off + (size_t)k * sp.wg_bytes;
        StreamRoundHdr rh;
        std::memcpy(&rh, wb, sizeof(rh));
        const uint32_t row0 = rh.row0, nrows = rh.nrows;
        const uint32_t CG = sp.cell_gates, nu = CG ? nrows / CG : 0;
        if (CG && (nrows % CG || (int64_t)sp.cell_units * CG != R || (int64_t)row0 + nu > sp.cell_units)) return fail("unit range");
        if (nrows > sp.rows_max || (!CG && (int64_t)row0 + nrows > R)) return fail("row range");
        auto out_row = [&](uint32_t rr) { return CG ? (size_t)(rr / nu) * sp.cell_units + row0 + rr % nu : (size_t)row0 + rr; };
        // (first slot, count) per row: consecutive, inside the table; every slot written exactly once
        std::vector<uint8_t> slot_used(sp.kmax, 0);
        std::vector<int32_t> slot_row(sp.kmax, -1);
        {
            uint32_t expect_first = 0;
            for (uint32_t i = 0; i < nrows; ++i) {
                uint32_t oc;
                std::memcpy(&oc, wb + sizeof(rh) + 4 * (size_t)i, 4);
                const uint32_t f = oc & 0xffffu, c = oc >> 16;
                if (f != expect_first || f + c > sp.kmax) return fail("row slots");
                for (uint32_t q = 0; q < c; ++q) slot_row[f + q] = (int32_t)i;
                expect_first = f + c;
            }
        }
        for (uint32_t sgi = 0; sgi < N; ++sgi) {
            const uint8_t *seg = wb + sp.hdr_bytes + (size_t)sgi * sp.seg_bytes;
            StreamSegHdr sh;
            std::memcpy(&sh, seg, sizeof(sh));
            if ((size_t)sh.bytes16 * 16 > sp.seg_bytes || sh.bytes16 == 0) return fail("segment length");
            {
                uint16_t nx = 0;
                if (sgi + kStreamWaves < N) std::memcpy(&nx, seg + (size_t)kStreamWaves * sp.seg_bytes + 4, 2);
                if (sh.next16 != nx) return fail("length of the next round's segment");
            }
            const size_t SB = (size_t)sh.bytes16 * 16;           // everything the kernel touches lies inside the segment's own length
            if (sizeof(sh) + (size_t)sh.ng * sizeof(StreamGroup) > SB) return fail("group records");
            for (uint32_t g = 0; g < sh.ng; ++g) {
                StreamGroup sg;
                std::memcpy(&sg, seg + sizeof(sh) + (size_t)g * sizeof(StreamGroup), sizeof(sg));
                const uint32_t steps = (uint32_t)sg.cmax_minus_1 + 1u, steps4 = (steps + 3u) & ~3u;
                if (sg.nlanes == 0 || sg.nlanes > kWave || !(sg.start_mask & 1ull)) return fail("group lanes");
                if (sg.nlanes < kWave && (sg.start_mask >> sg.nlanes)) return fail("start mask beyond the lanes");
                if ((size_t)sg.lane_off + 2u * sg.nlanes > SB || sg.lane_off % 2) return fail("lane words");
                if ((size_t)sg.val_off * 4 + (size_t)steps * kWave * vbytes > SB) return fail("value offset");
                for (uint32_t lane = 0; lane < (uint32_t)kWave; ++lane) {
                    if (lane >= sg.nlanes) {                       // lanes without a row: zeros only
                        for (uint32_t j = 0; j < steps; ++j)
                            if (value_bits(seg, sg.val_off, j, lane)) return fail("value behind the last lane not zero");
                        continue;
                    }
                    const uint64_t upto = lane == 63 ? ~0ull : ((2ull << lane) - 1ull);
                    const uint32_t slot = (uint32_t)__builtin_popcountll(sg.start_mask & upto) - 1u;
                    const size_t vpos = (size_t)sh.off_vbs + ((size_t)sg.vb0 + slot) * 4;
                    if (vpos + 4 > SB) return fail("block words");
                    uint32_t word;
                    std::memcpy(&word, seg + vpos, 4);
                    const uint32_t c = ((word >> 10) & 0xffu) + 1u, lw = (word & 0x3ffu) * 4u, bj = word >> 18;
                    if (c > steps) return fail("block wider than its piece");
                    if ((size_t)lw + steps4 > SB) return fail("column list");
                    uint16_t word16;
                    std::memcpy(&word16, seg + sg.lane_off + 2 * (size_t)lane, 2);
                    if (word16 >= sp.kmax || slot_row[word16] < 0 || slot_used[word16]) return fail("partial-sum slot");
                    slot_used[word16] = 1;
                    const uint32_t rr = (uint32_t)slot_row[word16];
                    // the kernel multiplies all of the piece's steps (in fours): what lies behind the
                    // lane's own columns must be a valid column with a zero value
                    for (uint32_t j = 0; j < steps4; ++j) {
                        const int64_t col = (int64_t)bj * m->bc + seg[lw + j];
                        if (col >= Ccols) return fail("column index");
                        if (j >= steps) continue;
                        const uint32_t bits = value_bits(seg, sg.val_off, j, lane);
                        if (j >= c) {
                            if (bits) return fail("padding value not zero");
                            if (seg[lw + j] != seg[lw]) return fail("padding column is not the block's first");
                            continue;
                        }
                        const size_t e = out_row(rr) * Ccols + col;
                        if (seen[e]) return fail("entry stored twice");
                        seen[e] = 1;
                        std::memcpy(&got[e], &bits, 4);
                        ++vals_used;
                    }
                }
            }
        }
        for (uint32_t q = 0; q < sp.kmax; ++q)
            if (slot_row[q] >= 0 && !slot_used[q]) return fail("partial-sum slot never written");
        for (uint32_t i = 0; i < nrows; ++i) {
            if (row_done[out_row(i)]) return fail("row owned twice");
            row_done[out_row(i)] = 1;
        }
    }
    for (int64_t i = 0; i < R; ++i) if (!row_done[i]) return fail("row without an owner");
    if (vals_used != m->val.size()) return fail("not every value referenced exactly once");
    if (std::memcmp(expect.data(), got.data(), expect.size() * sizeof(float)) != 0) return fail("section does not decode to the matrix");
    return CSB_OK;
}

}  // namespace csb
