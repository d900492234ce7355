// Host-side model of the paper's own engine schedule (Sec. 4.3.2, 5.2): K x L PEGroups of
// P x Q PEs work on K x L blocks per block iteration; a PEGroup may hand a regular part of
// its kernel matrix to its right neighbour (horizontal sharing) or to the one below (vertical
// sharing), torus-wise.  The model returns the PE utilisation ("hardware efficiency",
// Sec. 6.3.2) of a CSB matrix under no / horizontal / vertical / 2-D sharing, so that the
// prefix-sum partition of this library can be put next to the paper's scheme on the same
// matrix.  No device code; nothing on the compute path calls it.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "csb_internal.hpp"

namespace {

struct Dim { int m, n; };

// One PEGroup's choice: dnh columns (every row) go right, dmv rows go down; shape 0 gives
// the horizontal part the full height (the vertical part is then dmv x (n - dnh)), shape 1
// gives the vertical part the full width (the horizontal part is then (m - dmv) x dnh).
struct Opt { int dnh, dmv, shape; };

struct Model {
    int P, Q, K, L;
    int64_t cyc(int a, int b) const { return a <= 0 || b <= 0 ? 0 : (int64_t)((a + P - 1) / P) * ((b + Q - 1) / Q); }
    int64_t local(const Dim &d, const Opt &o) const { return cyc(d.m - o.dmv, d.n - o.dnh); }
    int64_t out_h(const Dim &d, const Opt &o) const { return o.shape == 0 ? cyc(d.m, o.dnh) : cyc(d.m - o.dmv, o.dnh); }
    int64_t out_v(const Dim &d, const Opt &o) const { return o.shape == 0 ? cyc(o.dmv, d.n - o.dnh) : cyc(o.dmv, d.n); }
};

// Smallest possible largest load of a ring of PEGroups that share in one direction only:
// exhaustive over every PEGroup's share (multiples of the PE count in that direction).
int64_t ring_best(const Model &M, const std::vector<Dim> &d, bool horizontal, std::vector<Opt> *best_opt) {
    const int n = (int)d.size();
    std::vector<std::vector<Opt>> opts(n);
    for (int i = 0; i < n; ++i) {
        if (horizontal) for (int s = 0; s <= d[i].n; s += M.Q) opts[i].push_back(Opt{s, 0, 0});
        else for (int s = 0; s <= d[i].m / 2; s += M.P) opts[i].push_back(Opt{0, s, 1});
    }
    std::vector<int> pick(n, 0);
    std::vector<Opt> cur(n);
    int64_t best = INT64_MAX;
    // depth-first with the loads that are already fixed as a bound
    std::vector<int> idx(n, 0);
    int depth = 0;
    idx[0] = -1;
    while (depth >= 0) {
        if (++idx[depth] >= (int)opts[depth].size()) { --depth; continue; }
        cur[depth] = opts[depth][idx[depth]];
        // loads known so far: PEGroup i (1 <= i <= depth) gets its own rest plus what i-1 hands over
        int64_t worst = 0;
        for (int i = 1; i <= depth; ++i) {
            const int64_t in = horizontal ? M.out_h(d[i - 1], cur[i - 1]) : M.out_v(d[i - 1], cur[i - 1]);
            worst = std::max(worst, M.local(d[i], cur[i]) + in);
        }
        if (worst >= best) continue;
        if (depth + 1 < n) { ++depth; idx[depth] = -1; continue; }
        const int64_t in0 = horizontal ? M.out_h(d[n - 1], cur[n - 1]) : M.out_v(d[n - 1], cur[n - 1]);
        worst = std::max(worst, M.local(d[0], cur[0]) + in0);
        if (worst < best) { best = worst; if (best_opt) *best_opt = cur; }
    }
    return best;
}

// Exact 2-D optimum for at most four PEGroups: depth-first over every PEGroup's shape and
// shares, cut as soon as a load that is already determined reaches the best time known
// (`bound`, a schedule's time found before, so the result is never above it).  Returns false
// without a result if the number of combinations exceeds `limit`.
bool grid_best_2d(const Model &M, const std::vector<Dim> &d, int64_t bound, int64_t limit, int64_t *best_out) {
    const int K = M.K, L = M.L, n = K * L;
    *best_out = bound;
    if (bound == 0) return true;
    std::vector<std::vector<Opt>> opts(n);
    double combos = 1.0;
    for (int i = 0; i < n; ++i) {
        for (int shape = 0; shape < 2; ++shape)
            for (int dnh = 0; dnh <= d[i].n; dnh += M.Q)
                for (int dmv = 0; dmv <= d[i].m / 2; dmv += M.P) {
                    if (shape == 1 && (dnh == 0 || dmv == 0)) continue;          // the same parts as shape 0
                    const Opt o{dnh, dmv, shape};
                    if (M.local(d[i], o) < bound) opts[i].push_back(o);
                }
        if (opts[i].empty()) return true;                          // nothing can beat the bound
        combos *= (double)opts[i].size();
    }
    if (combos > (double)limit) return false;
    std::vector<Opt> cur(n);
    std::vector<int> idx(n, -1);
    int64_t best = bound;
    int depth = 0;
    while (depth >= 0) {
        if (++idx[depth] >= (int)opts[depth].size()) { idx[depth] = -1; --depth; continue; }
        cur[depth] = opts[depth][idx[depth]];
        // loads whose three contributors (the PEGroup, its left and its upper neighbour) are chosen
        int64_t worst = 0;
        for (int g = 0; g <= depth; ++g) {
            const int k = g / L, l = g % L;
            const int left = k * L + (l + L - 1) % L, up = ((k + K - 1) % K) * L + l;
            if (left > depth || up > depth) continue;
            worst = std::max(worst, M.local(d[g], cur[g]) + M.out_h(d[left], cur[left]) + M.out_v(d[up], cur[up]));
        }
        if (worst >= best) continue;
        if (depth + 1 < n) { ++depth; continue; }
        best = worst;
    }
    *best_out = best;
    return true;
}

}  // namespace

extern "C" int csb_sharing_model(const csb_matrix *m, int32_t P, int32_t Q, int32_t K, int32_t L,
                                 csb_sharing_stats *out) {
    using namespace csb;
    if (!m || !out) { set_error("csb_sharing_model: NULL pointer"); return CSB_EINVAL; }
    if (P <= 0 || Q <= 0 || K <= 0 || L <= 0 || K > 8 || L > 8) { set_error("csb_sharing_model: P, Q >= 1 and 1 <= K, L <= 8"); return CSB_EINVAL; }
    const Model M{P, Q, K, L};
    int64_t work = 0, t_none = 0, t_h = 0, t_v = 0, t_2d = 0, iters = 0;
    bool exact = K * L <= 4;
    const int IK = (m->nbr + K - 1) / K, JL = (m->nbc + L - 1) / L;
    std::vector<Dim> d((size_t)K * L);
    std::vector<Opt> o((size_t)K * L), ring;
    for (int bi = 0; bi < IK; ++bi)
        for (int bj = 0; bj < JL; ++bj) {
            for (int k = 0; k < K; ++k)
                for (int l = 0; l < L; ++l) {
                    const int r = bi * K + k, c = bj * L + l;
                    Dim &x = d[(size_t)k * L + l];
                    x = Dim{0, 0};
                    if (r < m->nbr && c < m->nbc) { x.m = m->nrows[(size_t)r * m->nbc + c]; x.n = m->ncols[(size_t)r * m->nbc + c]; }
                    work += (int64_t)x.m * x.n;
                }
            ++iters;
            // no sharing
            int64_t tn = 0;
            for (const Dim &x : d) tn = std::max(tn, M.cyc(x.m, x.n));
            t_none += tn;
            // horizontal only: the rows of PEGroups are independent rings
            int64_t th = 0;
            std::vector<Opt> oh((size_t)K * L);
            for (int k = 0; k < K; ++k) {
                std::vector<Dim> row(d.begin() + (size_t)k * L, d.begin() + (size_t)(k + 1) * L);
                th = std::max(th, ring_best(M, row, true, &ring));
                for (int l = 0; l < L; ++l) oh[(size_t)k * L + l] = ring[l];
            }
            t_h += th;
            // vertical only: the columns are
            int64_t tv = 0;
            std::vector<Opt> ov((size_t)K * L);
            for (int l = 0; l < L; ++l) {
                std::vector<Dim> col(K);
                for (int k = 0; k < K; ++k) col[k] = d[(size_t)k * L + l];
                tv = std::max(tv, ring_best(M, col, false, &ring));
                for (int k = 0; k < K; ++k) ov[(size_t)k * L + l] = ring[k];
            }
            t_v += tv;
            // 2-D: start from the better one-directional schedule and improve one PEGroup's
            // choice at a time (every shape and share of it, the others held) while the
            // largest load, then the sum of squared loads, goes down.  An upper bound on the
            // best 2-D schedule's time, i.e. a lower bound on its efficiency.
            o = th <= tv ? oh : ov;
            auto load = [&](int k, int l) {
                const int kl = k * L + l, left = k * L + (l + L - 1) % L, up = ((k + K - 1) % K) * L + l;
                return M.local(d[kl], o[kl]) + M.out_h(d[left], o[left]) + M.out_v(d[up], o[up]);
            };
            auto score = [&](int64_t *worst, int64_t *sq) {
                *worst = 0; *sq = 0;
                for (int k = 0; k < K; ++k)
                    for (int l = 0; l < L; ++l) { const int64_t v = load(k, l); *worst = std::max(*worst, v); *sq += v * v; }
            };
            int64_t bw, bs;
            score(&bw, &bs);
            for (int sweep = 0; sweep < 8; ++sweep) {
                bool improved = false;
                for (int kl = 0; kl < K * L; ++kl) {
                    const Opt keep = o[kl];
                    Opt best = keep;
                    for (int shape = 0; shape < 2; ++shape)
                        for (int dnh = 0; dnh <= d[kl].n; dnh += Q)
                            for (int dmv = 0; dmv <= d[kl].m / 2; dmv += P) {
                                o[kl] = Opt{dnh, dmv, shape};
                                int64_t w, s;
                                score(&w, &s);
                                if (w < bw || (w == bw && s < bs)) { bw = w; bs = s; best = o[kl]; improved = true; }
                            }
                    o[kl] = best;
                }
                if (!improved) break;
            }
            // Small grids: replace the bound by the exact optimum (every combination).
            if (K * L <= 4 && exact) {
                int64_t ex;
                if (grid_best_2d(M, d, bw, (int64_t)1 << 27, &ex)) bw = ex; else exact = false;
            }
            t_2d += bw;
        }
    const double denom = (double)P * Q * K * L;
    out->work = work;
    out->iterations = iters;
    out->cycles_none = t_none; out->cycles_horizontal = t_h; out->cycles_vertical = t_v; out->cycles_2d = t_2d;
    out->eff_none = t_none ? work / (denom * t_none) : 0.0;
    out->eff_horizontal = t_h ? work / (denom * t_h) : 0.0;
    out->eff_vertical = t_v ? work / (denom * t_v) : 0.0;
    out->eff_2d = t_2d ? work / (denom * t_2d) : 0.0;
    out->exact_2d = exact ? 1 : 0;
    out->reserved = 0;
    return CSB_OK;
}
