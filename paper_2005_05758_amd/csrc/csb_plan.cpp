// Equal-work partition and device image builder (host only).
//
// Role in the method: the paper balances uneven kernel-matrix work across its PE groups
// with a compiler pass (Sec. 5.2: every unit should end up with the average work of the
// iteration).  Here the parallel unit is a 64-lane wavefront and the balance comes from a
// prefix sum over wavefront steps that is cut into equal ranges.
#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>

#include "csb_internal.hpp"

namespace csb {
namespace {

struct Vb {
    uint32_t tile;             // output tile (out_row / br)
    uint32_t b;                // source CSB block
    uint16_t bj;
    uint16_t q0, q1;           // column positions [q0, q1) of the block's column list
    std::vector<uint16_t> a;   // kernel-matrix row positions inside the block
    std::vector<uint8_t> slot; // out_row - tile * br for each of them
    int c() const { return q1 - q0; }
    int r() const { return (int)a.size(); }
};

struct Group {
    uint32_t tile;
    std::vector<uint32_t> vbs;  // indices into the Vb array, column counts descending
    int cmax = 0, nlanes = 0;
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Floats a group holds before column step j (every step is a run of 64).
uint32_t vals_before_step(const std::vector<Vb> &, const Group &, int j) { return (uint32_t)j * kWave; }

}  // namespace

int plan_matrix(csb_matrix *m, int32_t n_chunks_req, int32_t waves_per_chunk, const SplitSpec &split,
                csb_plan_stats *stats_out, int32_t mode) {
    if (!m) { set_error("csb_plan: NULL matrix"); return CSB_EINVAL; }
    if (n_chunks_req < 0) { set_error("csb_plan: n_chunks < 0"); return CSB_EINVAL; }
    // mode 4 (internal): as mode 0 but without the row-owned section (the caller builds it itself)
    if (mode < 0 || mode > 4 || mode == 3) { set_error("csb_plan: mode must be 0 (auto), 1 (whole tiles) or 2 (equal split)"); return CSB_EINVAL; }
    const bool with_rows = mode == 0;
    if (mode == 4) mode = 0;
    if (waves_per_chunk != 16) {
        set_error("csb_plan: waves_per_chunk must be 16");
        return CSB_EINVAL;
    }
    if (m->val.size() >= (1ull << 32) || m->cols > (int64_t)65535 * m->bc) {
        set_error("csb_plan: matrix too large for 32-bit device offsets");
        return CSB_EUNSUPPORTED;
    }
    try {
        const int br = m->br, bc = m->bc;
        const int64_t rows_out = split.active() ? m->rows + split.shift : m->rows;
        const uint32_t n_tiles = (uint32_t)((rows_out + br - 1) / br);

        // ---- 1. virtual blocks, bucketed by output tile --------------------------------
        std::vector<Vb> vbs;
        std::vector<std::vector<uint32_t>> by_tile(n_tiles);
        for (int32_t bi = 0; bi < m->nbr; ++bi)
            for (int32_t bj = 0; bj < m->nbc; ++bj) {
                const size_t b = (size_t)bi * m->nbc + bj;
                const int nr = m->nrows[b], nc = m->ncols[b];
                if (nr == 0 || nc == 0) continue;
                const uint16_t *ri = m->rowidx.data() + m->row_off[b];
                const uint16_t *ci = m->colidx.data() + m->col_off[b];
                int qs = nc;  // first column position at or past the split column
                if (split.active()) {
                    qs = 0;
                    while (qs < nc && (int64_t)bj * bc + ci[qs] < split.split_col) ++qs;
                }
                // parts: (q0, q1, shifted?) ; rows below split_row always take the full range
                struct Part { int q0, q1; bool lower, shifted; };
                Part parts[3] = {{0, nc, true, false}, {0, qs, false, false}, {qs, nc, false, true}};
                for (const Part &p : parts) {
                    if (p.q0 >= p.q1) continue;
                    Vb cur;
                    bool open = false;
                    auto flush = [&]() {
                        if (open && !cur.a.empty()) {
                            by_tile[cur.tile].push_back((uint32_t)vbs.size());
                            vbs.push_back(cur);
                        }
                        open = false;
                    };
                    for (int a = 0; a < nr; ++a) {
                        const int64_t gr = (int64_t)bi * br + ri[a];
                        const bool is_lower = !split.active() || gr < split.split_row;
                        if (is_lower != p.lower) continue;
                        const int64_t orow = gr + (p.shifted ? split.shift : 0);
                        const uint32_t tile = (uint32_t)(orow / br);
                        if (!open || cur.tile != tile || cur.r() == kWave) {
                            flush();
                            cur = Vb{};
                            cur.tile = tile; cur.b = (uint32_t)b; cur.bj = (uint16_t)bj;
                            cur.q0 = (uint16_t)p.q0; cur.q1 = (uint16_t)p.q1;
                            open = true;
                        }
                        cur.a.push_back((uint16_t)a);
                        cur.slot.push_back((uint8_t)(orow - (int64_t)tile * br));
                    }
                    flush();
                }
            }

        // ---- 2. 64-lane groups per tile -------------------------------------------------
        std::vector<Group> groups;
        std::vector<uint32_t> nz_tiles, zero_tiles, tile_rank(n_tiles, 0);
        for (uint32_t t = 0; t < n_tiles; ++t) {
            auto &lst = by_tile[t];
            if (lst.empty()) { zero_tiles.push_back(t); continue; }
            tile_rank[t] = (uint32_t)nz_tiles.size();
            nz_tiles.push_back(t);
            std::stable_sort(lst.begin(), lst.end(),
                             [&](uint32_t x, uint32_t y) { return vbs[x].c() > vbs[y].c(); });
            std::vector<char> used(lst.size(), 0);
            size_t head = 0;
            while (head < lst.size()) {
                if (used[head]) { ++head; continue; }
                Group g;
                g.tile = t;
                // fill with the next unused blocks that still fit (look a little ahead)
                for (size_t p = head; p < lst.size() && p < head + 256; ++p) {
                    if (used[p]) continue;
                    const Vb &v = vbs[lst[p]];
                    if (g.nlanes + v.r() > kWave) continue;
                    used[p] = 1;
                    g.vbs.push_back(lst[p]);
                    g.nlanes += v.r();
                    g.cmax = std::max(g.cmax, v.c());
                    if ((int)g.vbs.size() == kMaxVbPerGroup || g.nlanes == kWave) break;
                }
                g.cmax = (g.cmax + kStepQuantum - 1) / kStepQuantum * kStepQuantum;
                groups.push_back(std::move(g));
            }
        }
        const uint32_t n_groups = (uint32_t)groups.size();

        // ---- 3. streams (group order) ---------------------------------------------------
        std::vector<GroupRec> grecs(n_groups);
        std::vector<VbRec> vrecs;
        std::vector<uint8_t> idx;
        std::vector<float> vals;
        std::vector<uint32_t> idx_end(n_groups);   // end of each group's index bytes
        vals.reserve(m->val.size() + m->val.size() / 4);
        uint64_t fma_steps = 0;
        size_t nnz_placed = 0;
        for (uint32_t gi = 0; gi < n_groups; ++gi) {
            const Group &g = groups[gi];
            GroupRec &gr = grecs[gi];
            gr.val_off = (uint32_t)vals.size();
            while (idx.size() % 8) idx.push_back(0);
            gr.idx_off = (uint32_t)idx.size();
            gr.vb_off = (uint32_t)vrecs.size();
            gr.nzrank = tile_rank[g.tile];
            gr.cmax = (uint16_t)g.cmax;
            gr.nvb = (uint8_t)g.vbs.size();
            gr.nlanes = (uint8_t)g.nlanes;
            // lane descriptors, 4 bytes per lane: row slot; block number (low 4 bits) and scatter
            // round (high 4 bits); 16-bit byte offset of the block's input-offset list from idx_off
            // (filled in below).  Lanes of one round have distinct row slots, so a round adds its
            // row results to the accumulator without conflicts.
            const size_t desc_base = idx.size();
            {
                uint8_t seen_rows[CSB_MAX_BLOCK] = {0};
                int rounds = 0;
                for (size_t k = 0; k < g.vbs.size(); ++k)
                    for (uint8_t s : vbs[g.vbs[k]].slot) {
                        const int rank = seen_rows[s]++;
                        rounds = std::max(rounds, rank + 1);
                        idx.push_back(s); idx.push_back((uint8_t)(k | (size_t)rank << 4)); idx.push_back(0); idx.push_back(0);
                    }
                gr.nrounds = (uint16_t)rounds;
            }
            while (idx.size() % 8) idx.push_back(0);
            const int cpad = (g.cmax + 3) & ~3;            // list length: lists stay 8-byte aligned
            const uint16_t zero_off = (uint16_t)(m->cols * 4);   // byte offset of the zero entry behind the input vector
            int lane0 = 0;
            for (size_t k = 0; k < g.vbs.size(); ++k) {
                const Vb &v = vbs[g.vbs[k]];
                VbRec vr{};
                vr.r = (uint8_t)v.r(); vr.lane0 = (uint8_t)lane0; vr.c = (uint16_t)v.c();
                vr.val_off = gr.val_off; vr.desc_pos = gr.idx_off; vr.list_pos = (uint32_t)idx.size();
                const size_t list_off = idx.size() - gr.idx_off;
                if (list_off > 0xffff) { set_error("csb_plan: internal: list offset"); return CSB_EINVAL; }
                for (int q = 0; q < v.r(); ++q) {
                    idx[desc_base + 4 * (size_t)(lane0 + q) + 2] = (uint8_t)(list_off & 0xff);
                    idx[desc_base + 4 * (size_t)(lane0 + q) + 3] = (uint8_t)(list_off >> 8);
                }
                const uint16_t *ci = m->colidx.data() + m->col_off[v.b];
                // byte offsets of the block's inputs in the staged vector, then the zero entry
                for (int j = 0; j < cpad; ++j) {
                    const uint16_t o = j < v.c() ? (uint16_t)(((uint32_t)v.bj * (uint32_t)bc + ci[v.q0 + j]) * 4u) : zero_off;
                    idx.push_back((uint8_t)(o & 0xff));
                    idx.push_back((uint8_t)(o >> 8));
                }
                vrecs.push_back(vr);
                lane0 += v.r();
            }
            while (idx.size() % 8) idx.push_back(0);
            idx_end[gi] = (uint32_t)idx.size();
            // values: step j is a run of 64 floats, lane l at [j * 64 + l], zero where unused
            {
                const size_t base = vals.size();
                vals.resize(base + (size_t)g.cmax * kWave, 0.0f);
                int l0 = 0;
                for (uint32_t k : g.vbs) {
                    const Vb &v = vbs[k];
                    const int nc = m->ncols[v.b];
                    const float *src = m->val.data() + m->val_off[v.b];
                    if (v.c() > g.cmax) { set_error("csb_plan: internal: group step count"); return CSB_EINVAL; }
                    for (int j = 0; j < v.c(); ++j)
                        for (int q = 0; q < v.r(); ++q)
                            vals[base + (size_t)j * kWave + l0 + q] = src[(size_t)v.a[q] * nc + v.q0 + j];
                    l0 += v.r();
                    nnz_placed += (size_t)v.r() * v.c();
                }
            }
            fma_steps += (uint64_t)g.cmax;
        }
        if (nnz_placed != m->val.size()) { set_error("csb_plan: internal: value count mismatch"); return CSB_EINVAL; }
        if (vals.size() + kWave >= (1ull << 32)) { set_error("csb_plan: matrix too large for 32-bit device offsets"); return CSB_EUNSUPPORTED; }
        const size_t vals_end = vals.size();
        vals.resize(vals_end + 2 * kWave, 0.0f);   // a wavefront without work still issues one (unused) load of a step pair

        // ---- 4. cost axis, chunk and wave cuts -----------------------------------------
        // Group g occupies [P[g], P[g+1]) with P[g+1]-P[g] = overhead + cmax; a cut inside
        // the overhead part snaps to the group start.
        const int NW = waves_per_chunk;
        std::vector<uint64_t> P(n_groups + 1, 0);
        for (uint32_t g = 0; g < n_groups; ++g) P[g + 1] = P[g] + kGroupOverhead + groups[g].cmax;
        const uint64_t total = P[n_groups];
        // LDS sizing: input vector + per-wavefront value windows + records + accumulators
        const uint32_t acc_rows_cap = (uint32_t)std::max(kAccRowsMax, br);
        const size_t zbytes = align_up((size_t)m->cols + 1, 64) * 4;   // input vector + the zero entry
        if (m->cols > kMaxStageCols) {
            set_error("csb_plan: more columns than the LDS staging of the input vector covers");
            return CSB_EUNSUPPORTED;
        }
        int n_chunks = n_chunks_req;
        if (n_chunks == 0) {
            // default: one workgroup per CU of an MI355X (256) once every wavefront has a group's
            // worth of work: a launch costs several microseconds of dependent latencies whatever
            // its size, so a small matrix is spread over many workgroups rather than few
            // (measured on the batch-1 RNN matrices: 6 cost units per wavefront beat 14 by 8 % of
            // the launch's kernel time; below that nothing more is gained)
            const uint64_t per_wave_min = 6;
            uint64_t want = total / (per_wave_min * (uint64_t)NW);
            want = std::min<uint64_t>(std::max<uint64_t>(want, 1), 256);
            n_chunks = (int)want;
        }
        struct Pos { uint32_t g; uint32_t j; };
        auto locate = [&](uint64_t X) -> Pos {
            if (X >= total) return Pos{n_groups, 0};
            uint32_t g = (uint32_t)(std::upper_bound(P.begin(), P.end(), X) - P.begin() - 1);
            const uint64_t in = X - P[g];
            if (in <= (uint64_t)kGroupOverhead) return Pos{g, 0};
            return Pos{g, (uint32_t)(in - kGroupOverhead) / kStepQuantum * kStepQuantum};
        };
        auto abs_val = [&](Pos p) -> uint32_t {
            if (p.g >= n_groups) return (uint32_t)vals_end;
            return grecs[p.g].val_off + vals_before_step(vbs, groups[p.g], (int)p.j);
        };
        const uint32_t max_tiles_per_chunk = (uint32_t)std::max<uint32_t>(1, acc_rows_cap / br);
        std::vector<uint64_t> chunk_cut;
        std::vector<WaveRec> waves;
        std::vector<Pos> cpos_a, cpos_b;
        std::vector<double> wave_cost;
        // per non-empty tile: group range, cost, values, record bytes
        const size_t n_nz = nz_tiles.size();
        std::vector<uint32_t> tile_g0(n_nz + 1, n_groups);
        for (uint32_t g = n_groups; g-- > 0;) tile_g0[tile_rank[groups[g].tile]] = g;
        // record segments for the batched kernel: group ranges inside one tile whose records fit
        // the LDS window one workgroup stages at a time
        std::vector<uint32_t> seg_g0, tile_seg0(n_nz + 1, 0);
        for (size_t r = 0; r < n_nz; ++r) {
            tile_seg0[r] = (uint32_t)seg_g0.size();
            size_t bytes = 0, nv = 0;
            for (uint32_t g = tile_g0[r]; g < tile_g0[r + 1]; ++g) {
                const size_t gb = sizeof(GroupRec) + (size_t)grecs[g].nvb * sizeof(VbRec) + (idx_end[g] - grecs[g].idx_off);
                if (g == tile_g0[r] || bytes + gb + 64 > (size_t)kChunkMetaMax || nv + grecs[g].nvb > 2048) {
                    seg_g0.push_back(g);
                    bytes = 0; nv = 0;
                }
                bytes += gb; nv += grecs[g].nvb;
            }
        }
        tile_seg0[n_nz] = (uint32_t)seg_g0.size();
        seg_g0.push_back(n_groups);
        auto tile_meta = [&](size_t r) {
            const uint32_t ga = tile_g0[r], gb = tile_g0[r + 1] - 1;
            return (size_t)(gb - ga + 1) * sizeof(GroupRec) + (idx_end[gb] - grecs[ga].idx_off) + 64;
        };
        auto lds_for = [&](size_t meta, size_t ntile) {
            return zbytes + align_up(meta, 256) + (size_t)NW * kAccPlanes * ntile * br * 4 + 4 * (size_t)kAccRowsMax * 4;
        };
        // Whole-tile chunks: contiguous tile ranges, smallest possible largest cost for at most
        // n_target chunks.  No output tile is then shared between workgroups.
        bool whole_tiles = false;
        if (mode != 2 && n_nz > 0) {
            const size_t n_target = (size_t)std::max(1, n_chunks);
            auto fill_tiles = [&](uint64_t Tmax, std::vector<uint64_t> *cuts) -> long {
                long used = 0;
                size_t r = 0;
                if (cuts) cuts->assign(1, 0);
                while (r < n_nz) {
                    ++used;
                    uint64_t cost = 0;
                    size_t mb = 0, nt = 0;
                    while (r < n_nz) {
                        const uint64_t tc = P[tile_g0[r + 1]] - P[tile_g0[r]];
                        const size_t tm = tile_meta(r);
                        const bool fits = nt + 1 <= max_tiles_per_chunk && lds_for(mb + tm, nt + 1) <= (size_t)kLdsBudget &&
                                          mb + tm <= (size_t)kChunkMetaMax;
                        if (nt == 0 && !fits) return -1;            // a single tile does not fit
                        if (!fits || (nt > 0 && cost + tc > Tmax)) break;
                        cost += tc; mb += tm; ++nt; ++r;
                    }
                    if (cuts) cuts->push_back(r < n_nz ? P[tile_g0[r]] : total);
                }
                return used;
            };
            if (fill_tiles(total, nullptr) > 0 && (mode == 1 || 2 * n_nz >= n_target)) {   // merging shared tiles costs more than a moderate imbalance
                uint64_t lo = 1, hi = total;
                while (lo < hi) {
                    const uint64_t mid = (lo + hi) / 2;
                    if (fill_tiles(mid, nullptr) <= (long)n_target) hi = mid; else lo = mid + 1;
                }
                fill_tiles(lo, &chunk_cut);
                whole_tiles = true;
            } else if (mode == 1) {
                set_error("csb_plan: a row tile does not fit one workgroup's LDS; whole-tile mode impossible");
                return CSB_EUNSUPPORTED;
            }
        }
        for (int attempt = 0;; ++attempt) {
            if (attempt > 40) { set_error("csb_plan: internal: cannot fit the LDS windows"); return CSB_EINVAL; }
            if (!whole_tiles) {
            chunk_cut.assign(1, 0);
            uint64_t X = 0;
            int remaining = n_chunks;
            while (X < total) {
                if (remaining < 1) remaining = 1;
                const uint64_t target = (total - X + remaining - 1) / remaining;
                uint64_t end = std::min(total, X + std::max<uint64_t>(target, 1));
                // limits: output tiles and record bytes; walk groups from the first one touched
                const Pos a = locate(X);
                uint32_t g = a.g;
                const uint32_t first_rank = g < n_groups ? tile_rank[groups[g].tile] : 0;
                size_t meta = 0;
                while (g < n_groups && P[g] < end) {
                    const size_t gmeta = sizeof(GroupRec) + (idx_end[g] - grecs[g].idx_off);
                    if (tile_rank[groups[g].tile] - first_rank >= max_tiles_per_chunk ||
                        (g > a.g && meta + gmeta + 64 > (size_t)kChunkMetaMax)) { end = P[g]; break; }
                    meta += gmeta;
                    ++g;
                }
                if (end <= X) end = std::min(total, P[a.g + 1]);  // always advance
                chunk_cut.push_back(end);
                X = end;
                --remaining;
            }
            }
            while ((int)chunk_cut.size() - 1 < std::max(n_chunks_req, 1)) chunk_cut.push_back(total);  // empty chunks
            const int nc = (int)chunk_cut.size() - 1;
            waves.assign((size_t)nc * NW, WaveRec{});
            cpos_a.assign(nc, Pos{0, 0});
            cpos_b.assign(nc, Pos{0, 0});
            wave_cost.assign((size_t)nc * NW, 0.0);
            uint32_t tiles_max = 1;
            size_t meta_max = 64;
            auto before = [&](Pos p, Pos q) { return p.g < q.g || (p.g == q.g && p.j < q.j); };
            // Wavefront cuts inside [ca, cb): smallest share T such that a greedy fill (a
            // wavefront that resumes inside a group pays the group overhead again) needs at
            // most NW wavefronts.
            auto cut_waves = [&](Pos ca, Pos cb, WaveRec *out, double *cost_out) {
                auto fill = [&](uint64_t T, std::vector<Pos> *cuts) -> bool {
                    Pos p = ca;
                    int used = 0;
                    if (cuts) cuts->assign(1, ca);
                    while (before(p, cb)) {
                        if (++used > NW) return false;
                        uint64_t budget = T;
                        bool first = true;
                        while (before(p, cb)) {
                            const uint32_t lim = p.g == cb.g ? cb.j : (uint32_t)groups[p.g].cmax;
                            if (budget <= (uint64_t)kGroupOverhead && !first) break;
                            if (budget <= (uint64_t)kGroupOverhead) budget = kGroupOverhead + 1;   // always advance
                            budget -= kGroupOverhead;
                            const uint32_t rem = lim - p.j;
                            if (rem <= budget) {
                                budget -= rem;
                                if (p.g == cb.g) p = cb; else p = Pos{p.g + 1, 0};
                            } else {                       // rem > budget; both positions stay multiples of the quantum
                                p.j += std::max<uint32_t>((uint32_t)budget / kStepQuantum * kStepQuantum, kStepQuantum);
                                if (p.j >= lim) { if (p.g == cb.g) p = cb; else p = Pos{p.g + 1, 0}; }
                                budget = 0;
                            }
                            first = false;
                            if (budget == 0) break;
                        }
                        if (cuts) cuts->push_back(p);
                    }
                    return true;
                };
                uint64_t span = 2 * kGroupOverhead + 2;
                for (uint32_t g = ca.g; g <= cb.g && g < n_groups; ++g) span += kGroupOverhead + groups[g].cmax;
                uint64_t lo = 1, hi = span;
                while (lo < hi) {
                    const uint64_t mid = (lo + hi) / 2;
                    if (fill(mid, nullptr)) hi = mid; else lo = mid + 1;
                }
                std::vector<Pos> cuts;
                fill(lo, &cuts);
                while ((int)cuts.size() < NW + 1) cuts.push_back(cb);
                for (int w = 0; w < NW; ++w) {
                    const Pos a = cuts[w], b = cuts[w + 1];
                    WaveRec &wr = out[w];
                    wr.g_begin = a.g; wr.j_begin = (uint16_t)a.j;
                    wr.g_end = b.g; wr.j_end = (uint16_t)b.j;
                    wr.val_begin = a.j * kWave;
                    wr.v_begin = abs_val(a);
                    wr.v_end = abs_val(b);
                    double cost = 0;
                    for (uint32_t g = a.g; g <= b.g && g < n_groups; ++g) {
                        const int jlo = g == a.g ? (int)a.j : 0;
                        const int jhi = g == b.g ? (int)b.j : groups[g].cmax;
                        if (jhi > jlo) cost += kGroupOverhead + (jhi - jlo);
                    }
                    cost_out[w] += cost;
                }
            };
            for (int c = 0; c < nc; ++c) {
                const uint64_t Xa = chunk_cut[c], Xb = chunk_cut[c + 1];
                cpos_a[c] = locate(Xa);
                cpos_b[c] = locate(Xb);
                const Pos ca = cpos_a[c], cb = cpos_b[c];
                cut_waves(ca, cb, &waves[(size_t)c * NW], &wave_cost[(size_t)c * NW]);
                // record bytes and tiles of this chunk
                {
                    uint32_t ga = ca.g, gb = cb.g;
                    bool any = true;
                    if (cb.j == 0) { if (gb == 0 || gb <= ga) any = false; else --gb; }
                    if (ga >= n_groups) any = false;
                    if (any) {
                        const uint32_t i0 = grecs[ga].idx_off & ~15u;
                        const size_t mb = align_up((gb - ga + 1) * sizeof(GroupRec), 16) + align_up(idx_end[gb] - i0, 16);
                        meta_max = std::max(meta_max, mb);
                        tiles_max = std::max<uint32_t>(tiles_max, tile_rank[groups[gb].tile] - tile_rank[groups[ga].tile] + 1);
                    }
                }
            }
            const bool fits = lds_for(meta_max, tiles_max) <= (size_t)kLdsBudget && meta_max <= (size_t)kChunkMetaMax + 64;
            if (fits) { n_chunks = nc; break; }
            whole_tiles = false;
            if (n_chunks_req == 0) n_chunks = nc < 256 ? std::min(256, nc * 2) : (nc / 256 + 1) * 256;   // whole rounds of 256 CUs
            else n_chunks = std::max(nc, n_chunks) * 5 / 4 + 1;
        }
        std::vector<ChunkRec> chunks(n_chunks);

        // ---- 5. tiles per chunk, shared tiles -------------------------------------------
        // touched groups of chunk c: [ga, gb] with gb included only if its j > 0
        std::vector<int> tile_first_chunk(nz_tiles.size(), -1), tile_last_chunk(nz_tiles.size(), -1);
        std::vector<int> c_rank0(n_chunks, 0), c_ntiles(n_chunks, 0);
        std::vector<uint32_t> c_ga(n_chunks, 0), c_gb(n_chunks, 0);
        for (int c = 0; c < n_chunks; ++c) {
            uint32_t ga = cpos_a[c].g, gb = cpos_b[c].g;
            if (cpos_b[c].j == 0) { if (gb == 0 || gb <= ga) { c_ntiles[c] = 0; continue; } --gb; }
            if (ga >= n_groups) { c_ntiles[c] = 0; continue; }
            const uint32_t r0 = tile_rank[groups[ga].tile], r1 = tile_rank[groups[gb].tile];
            c_rank0[c] = (int)r0;
            c_ntiles[c] = (int)(r1 - r0 + 1);
            c_ga[c] = ga; c_gb[c] = gb;
            for (uint32_t r = r0; r <= r1; ++r) {
                if (tile_first_chunk[r] < 0) tile_first_chunk[r] = c;
                tile_last_chunk[r] = c;
            }
        }
        std::vector<SharedRec> shared;
        std::vector<int> tile_sid(nz_tiles.size(), -1);
        uint32_t n_partial_slots = 0;
        for (size_t r = 0; r < nz_tiles.size(); ++r) {
            if (tile_first_chunk[r] < 0) { set_error("csb_plan: internal: tile without a chunk"); return CSB_EINVAL; }
            if (tile_last_chunk[r] > tile_first_chunk[r]) {
                SharedRec s{};
                s.tile = nz_tiles[r];
                tile_sid[r] = (int)shared.size();
                shared.push_back(s);
            }
        }
        uint32_t meta_cap = 64;
        for (int c = 0; c < n_chunks; ++c) {
            ChunkRec &cr = chunks[c];
            cr = ChunkRec{};
            cr.nzrank0 = (uint32_t)c_rank0[c];
            cr.ntiles = (uint32_t)c_ntiles[c];
            cr.sid_first = cr.part_first = cr.sid_last = cr.part_last = -1;
            if (c_ntiles[c] == 0) continue;
            const int rf = c_rank0[c], rl = c_rank0[c] + c_ntiles[c] - 1;
            if (tile_sid[rf] >= 0) {
                cr.sid_first = tile_sid[rf];
                cr.part_first = (int32_t)shared[tile_sid[rf]].nparts++;
            }
            if (rl != rf && tile_sid[rl] >= 0) {
                cr.sid_last = tile_sid[rl];
                cr.part_last = (int32_t)shared[tile_sid[rl]].nparts++;
            }
            const uint32_t ga = c_ga[c], gb = c_gb[c];
            cr.g0 = ga; cr.ng = gb - ga + 1;
            cr.vb0 = grecs[ga].vb_off; cr.nvbs = grecs[gb].vb_off + grecs[gb].nvb - cr.vb0;
            cr.idx0 = grecs[ga].idx_off & ~15u;
            cr.idx_bytes = (uint32_t)align_up(idx_end[gb] - cr.idx0, 16);
            cr.v0 = abs_val(cpos_a[c]);
            cr.nv4 = (abs_val(cpos_b[c]) - cr.v0) >> 2;
            const uint32_t mb = (uint32_t)(align_up(cr.ng * sizeof(GroupRec), 16) + cr.idx_bytes);
            meta_cap = std::max(meta_cap, mb);
        }
        if (meta_cap > (uint32_t)kChunkMetaMax + 4096) { set_error("csb_plan: internal: record window overflow"); return CSB_EINVAL; }
        for (auto &s : shared) { s.partial_off = n_partial_slots; n_partial_slots += s.nparts; }

        // ---- 6. image -------------------------------------------------------------------
        DevHeader h{};
        h.magic = 0x4353424d49333535ull;  // "CSBMI355"
        h.n_chunks = (uint32_t)n_chunks; h.waves_per_chunk = (uint32_t)NW;
        h.n_groups = n_groups; h.n_vbs = (uint32_t)vrecs.size();
        h.n_shared = (uint32_t)shared.size(); h.n_zero_tiles = (uint32_t)zero_tiles.size();
        h.n_nz_tiles = (uint32_t)nz_tiles.size(); h.n_partial_slots = n_partial_slots;
        h.max_chunk_tiles = 1;
        h.meta_cap = (uint32_t)align_up(meta_cap, 256);
        for (const ChunkRec &cr : chunks) h.max_chunk_tiles = std::max(h.max_chunk_tiles, cr.ntiles);
        h.br = (uint32_t)br; h.bc = (uint32_t)bc; h.rows_out = (uint64_t)rows_out; h.cols = (uint64_t)m->cols;
        size_t off = align_up(sizeof(DevHeader), 256);
        auto place = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes + 64, 256); return o; };
        h.off_chunks = place(chunks.size() * sizeof(ChunkRec));
        h.off_waves = place(waves.size() * sizeof(WaveRec));
        h.off_groups = place(grecs.size() * sizeof(GroupRec));
        h.off_vbs = place(vrecs.size() * sizeof(VbRec));
        h.off_idx = place(idx.size());
        // 16-bit value stream: one 32-bit word per lane and PAIR of steps (groups start on even
        // steps and have an even number of them), the even step in the low half
        std::vector<uint32_t> vals16;
        if (m->val_fmt != CSB_VAL_F32) {
            vals16.resize(vals.size() / 2);
            for (size_t pr = 0; pr < vals.size() / (2 * kWave); ++pr)
                for (size_t l = 0; l < (size_t)kWave; ++l) {
                    const float lo = vals[(2 * pr) * kWave + l], hi = vals[(2 * pr + 1) * kWave + l];
                    const uint32_t a = m->val_fmt == CSB_VAL_F16 ? f32_to_f16_bits(lo) : f32_to_bf16_bits(lo);
                    const uint32_t b = m->val_fmt == CSB_VAL_F16 ? f32_to_f16_bits(hi) : f32_to_bf16_bits(hi);
                    vals16[pr * kWave + l] = a | (b << 16);
                }
        }
        h.val_fmt = (uint32_t)m->val_fmt;
        h.off_vals = place(vals16.empty() ? vals.size() * sizeof(float) : vals16.size() * sizeof(uint32_t));
        h.off_nz_tiles = place(nz_tiles.size() * 4);
        h.off_zero_tiles = place(zero_tiles.size() * 4);
        h.off_shared = place(shared.size() * sizeof(SharedRec));
        h.off_counters = place((shared.size() + 1) * 4);     // merge tickets, then one status word (a merge that gave up)
        h.off_tile_g0 = place(tile_g0.size() * 4);
        h.off_tile_seg0 = place(tile_seg0.size() * 4);
        std::vector<SegRec> segs(seg_g0.size() - 1);
        for (size_t i = 0; i + 1 < seg_g0.size(); ++i) {
            const uint32_t ga = seg_g0[i], gb = seg_g0[i + 1];
            SegRec &sr = segs[i];
            sr = SegRec{};
            sr.g0 = ga; sr.ng = gb - ga;
            sr.vb0 = grecs[ga].vb_off;
            sr.nvbs = grecs[gb - 1].vb_off + grecs[gb - 1].nvb - sr.vb0;
            sr.idx0 = grecs[ga].idx_off & ~15u;
            sr.idx_bytes = (uint32_t)align_up(idx_end[gb - 1] - sr.idx0, 16);
            // what the batched kernel stages of it: group records, block records, index bytes
            const size_t staged = align_up(sr.ng * sizeof(GroupRec), 16) + align_up(sr.nvbs * sizeof(VbRec), 16) + sr.idx_bytes;
            h.seg_meta = std::max<uint32_t>(h.seg_meta, (uint32_t)align_up(staged + 16, 256));
        }
        h.off_segs = place(segs.size() * sizeof(SegRec));
        h.n_segs = segs.size();
        h.idx_bytes = idx.size(); h.n_vals = vals_end; h.total_bytes = off;
        Plan &pl = m->plan;
        pl.image.assign(off, 0);
        uint8_t *im = pl.image.data();
        std::memcpy(im, &h, sizeof(h));
        auto put = [&](size_t o, const void *p, size_t n) { if (n) std::memcpy(im + o, p, n); };
        put(h.off_chunks, chunks.data(), chunks.size() * sizeof(ChunkRec));
        put(h.off_waves, waves.data(), waves.size() * sizeof(WaveRec));
        put(h.off_groups, grecs.data(), grecs.size() * sizeof(GroupRec));
        put(h.off_vbs, vrecs.data(), vrecs.size() * sizeof(VbRec));
        put(h.off_idx, idx.data(), idx.size());
        if (vals16.empty()) put(h.off_vals, vals.data(), vals.size() * sizeof(float));
        else put(h.off_vals, vals16.data(), vals16.size() * sizeof(uint32_t));
        put(h.off_nz_tiles, nz_tiles.data(), nz_tiles.size() * 4);
        put(h.off_zero_tiles, zero_tiles.data(), zero_tiles.size() * 4);
        put(h.off_shared, shared.data(), shared.size() * sizeof(SharedRec));
        put(h.off_tile_g0, tile_g0.data(), tile_g0.size() * 4);
        put(h.off_tile_seg0, tile_seg0.data(), tile_seg0.size() * 4);
        put(h.off_segs, segs.data(), segs.size() * sizeof(SegRec));
        pl.hdr = h;
        pl.split = split;
        pl.req_chunks = n_chunks_req;
        pl.req_mode = with_rows ? 0 : (mode == 0 ? 4 : mode);
        pl.valid = true;
        m->uploaded = false;
        m->d_buf = nullptr;

        // ---- 7. statistics --------------------------------------------------------------
        csb_plan_stats st{};
        st.n_chunks = n_chunks; st.waves_per_chunk = NW; st.n_groups = (int32_t)n_groups;
        st.n_shared_tiles = (int32_t)shared.size();
        double wmax = 0, wsum = 0;
        for (double c : wave_cost) { wmax = std::max(wmax, c); wsum += c; }
        st.work_max = wmax;
        st.work_mean = wave_cost.empty() ? 0 : wsum / (double)wave_cost.size();
        {
            double cmax_ = 0, csum_ = 0;
            for (int c = 0; c < n_chunks; ++c) {
                double cc = 0;
                for (int w = 0; w < NW; ++w) cc += wave_cost[(size_t)c * NW + w];
                cmax_ = std::max(cmax_, cc); csum_ += cc;
            }
            st.chunk_max_over_mean = csum_ > 0 ? cmax_ / (csum_ / n_chunks) : 0.0;
            st.whole_tiles = whole_tiles ? 1 : 0;
        }
        st.lane_fill = fma_steps ? (double)m->val.size() / (64.0 * (double)fma_steps) : 0.0;
        {
            const size_t nwt = wave_cost.size();
            std::vector<double> rr(nwt, 0.0);
            size_t k = 0;
            for (size_t b = 0; b < m->nrows.size(); ++b) {
                if (m->nrows[b] == 0 || m->ncols[b] == 0) continue;
                rr[k % nwt] += (double)m->nrows[b] * m->ncols[b];
                ++k;
            }
            double mx = 0, sm = 0;
            for (double v : rr) { mx = std::max(mx, v); sm += v; }
            st.nosplit_max_over_mean = sm > 0 ? mx / (sm / (double)nwt) : 0.0;
        }
        st.matvec_bytes = (int64_t)pl.image.size();
        pl.stats = st;
        pl.stream = StreamPlan{};
        if (stats_out) *stats_out = st;
        // the row-owned section for csb_spmv, when the matrix fits it
        if (with_rows) return plan_stream(m, n_chunks_req, 0, stats_out);
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        set_error("csb_plan: out of host memory");
        return CSB_ENOMEM;
    }
}

// Walk the image the way the kernels do, with bounds checks on every access, rebuild the
// (output row, column) -> value map and compare it with the packed matrix.
int validate_plan(const csb_matrix *m) {
    if (!m) { set_error("csb_plan_validate: NULL matrix"); return CSB_EINVAL; }
    if (!m->plan.valid) { set_error("csb_plan_validate: matrix not planned"); return CSB_ESTATE; }
    const Plan &pl = m->plan;
    const DevHeader &h = pl.hdr;
    const uint8_t *im = pl.image.data();
    auto fail = [&](const char *what) { set_error(std::string("csb_plan_validate: ") + what); return CSB_EINVAL; };
    if (h.total_bytes > pl.image.size() || (!pl.stream.valid && h.total_bytes != pl.image.size())) return fail("image size");
    const auto *chunks = (const ChunkRec *)(im + h.off_chunks);
    const auto *waves = (const WaveRec *)(im + h.off_waves);
    const auto *groups = (const GroupRec *)(im + h.off_groups);
    const auto *vbs = (const VbRec *)(im + h.off_vbs);
    const uint8_t *idx = im + h.off_idx;
    if (h.val_fmt != (uint32_t)m->val_fmt) return fail("value format");
    // value slot va of the stream, whatever its storage format
    auto val_at = [&](uint64_t va) -> float {
        if (h.val_fmt == CSB_VAL_F32) return ((const float *)(im + h.off_vals))[va];
        const uint64_t step = va / kWave, lane = va % kWave;
        const uint32_t w = ((const uint32_t *)(im + h.off_vals))[(step >> 1) * kWave + lane];
        const uint16_t bits = (uint16_t)((step & 1) ? w >> 16 : w & 0xffffu);
        return h.val_fmt == CSB_VAL_F16 ? f16_bits_to_f32(bits) : bf16_bits_to_f32(bits);
    };
    const auto *nz_tiles = (const uint32_t *)(im + h.off_nz_tiles);
    const auto *zero_tiles = (const uint32_t *)(im + h.off_zero_tiles);
    const auto *shared = (const SharedRec *)(im + h.off_shared);
    const auto *tile_g0v = (const uint32_t *)(im + h.off_tile_g0);
    const auto *tile_seg0v = (const uint32_t *)(im + h.off_tile_seg0);
    const auto *segsv = (const SegRec *)(im + h.off_segs);
    // record segments of the batched kernel: tile the tiles' group ranges, fit the LDS window
    for (uint32_t r = 0; r < h.n_nz_tiles; ++r) {
        if (tile_seg0v[r] > tile_seg0v[r + 1] || tile_seg0v[r + 1] > h.n_segs) return fail("tile segment range");
        uint32_t gexp = tile_g0v[r];
        for (uint32_t sgi = tile_seg0v[r]; sgi < tile_seg0v[r + 1]; ++sgi) {
            const SegRec &sr = segsv[sgi];
            const uint32_t ga = sr.g0, gb = sr.g0 + sr.ng;
            if (ga != gexp || sr.ng == 0 || gb > h.n_groups) return fail("segment group range");
            if (sr.vb0 != groups[ga].vb_off || sr.nvbs != groups[gb - 1].vb_off + groups[gb - 1].nvb - sr.vb0 ||
                (uint64_t)sr.vb0 + sr.nvbs > h.n_vbs) return fail("segment block records");
            const size_t iend = gb < h.n_groups ? groups[gb].idx_off : (size_t)h.idx_bytes;
            if (sr.idx0 != (groups[ga].idx_off & ~15u) || (sr.idx_bytes & 15u) || (size_t)sr.idx0 + sr.idx_bytes < iend ||
                (size_t)sr.idx0 + sr.idx_bytes > h.idx_bytes + 64) return fail("segment index bytes");
            if (align_up(sr.ng * sizeof(GroupRec), 16) + align_up(sr.nvbs * sizeof(VbRec), 16) + sr.idx_bytes > (size_t)kChunkMetaMax + 64 || sr.nvbs > 2048)
                return fail("segment larger than the batched kernel's LDS window");
            gexp = gb;
        }
        if (gexp != tile_g0v[r + 1]) return fail("segments do not cover the tile");
    }
    const int64_t rows_out = (int64_t)h.rows_out, cols = (int64_t)h.cols;
    const uint32_t br = h.br, bc = h.bc, NW = h.waves_per_chunk;
    const uint32_t n_tiles = (uint32_t)((rows_out + br - 1) / br);

    // expected map: dense rows_out x cols with the split relabelling applied
    std::vector<float> expect((size_t)rows_out * cols, 0.0f), got((size_t)rows_out * cols, 0.0f);
    std::vector<uint8_t> seen((size_t)rows_out * cols, 0);
    for (int32_t bi = 0; bi < m->nbr; ++bi)
        for (int32_t bj = 0; bj < m->nbc; ++bj) {
            const size_t b = (size_t)bi * m->nbc + bj;
            const int nr = m->nrows[b], nc = m->ncols[b];
            for (int a = 0; a < nr; ++a)
                for (int q = 0; q < nc; ++q) {
                    int64_t gr = (int64_t)bi * br + m->rowidx[m->row_off[b] + a];
                    const int64_t gc = (int64_t)bj * bc + m->colidx[m->col_off[b] + q];
                    if (pl.split.active() && gr >= pl.split.split_row && gc >= pl.split.split_col) gr += pl.split.shift;
                    expect[(size_t)gr * cols + gc] = m->val[m->val_off[b] + (size_t)a * nc + q];
                }
        }
    std::vector<uint8_t> tile_written(n_tiles, 0);
    std::vector<uint32_t> parts_seen(h.n_shared, 0);
    uint64_t vals_used = 0;
    for (uint32_t c = 0; c < h.n_chunks; ++c) {
        const ChunkRec &cr = chunks[c];
        if (cr.ntiles * br > (uint32_t)std::max<int>(kAccRowsMax, (int)br)) return fail("chunk tile span");
        if ((cr.v0 & 63u) || (cr.nv4 & 15u) || (uint64_t)cr.v0 + 4 * (uint64_t)cr.nv4 > h.n_vals) return fail("chunk value window");
        if ((uint64_t)cr.g0 + cr.ng > h.n_groups || (uint64_t)cr.vb0 + cr.nvbs > h.n_vbs ||
            (uint64_t)cr.idx0 + cr.idx_bytes > h.idx_bytes + 64) return fail("chunk record window");
        if (align_up(cr.ng * sizeof(GroupRec), 16) + cr.idx_bytes > h.meta_cap)
            return fail("chunk record window larger than its LDS space");
        if (cr.nzrank0 + cr.ntiles > h.n_nz_tiles) return fail("chunk tile rank");
        uint32_t v_expect = cr.v0;   // the wavefronts' value runs tile the chunk's run in order
        for (uint32_t sw = 0; sw < NW; ++sw) {
            const WaveRec &wr = waves[(size_t)c * NW + sw];
            const uint32_t half_lo = cr.v0, half_hi = cr.v0 + 4 * cr.nv4;
            if (wr.v_begin < wr.v_end) {
                if (wr.v_begin != v_expect || ((wr.v_end - wr.v_begin) & 63u)) return fail("wave value run");
                v_expect = wr.v_end;
            }
            if (wr.g_begin > h.n_groups || wr.g_end > h.n_groups || wr.g_begin > wr.g_end) return fail("wave range");
            if (wr.v_begin > wr.v_end || wr.v_end > h.n_vals) return fail("wave value range");
            if (wr.v_begin < wr.v_end && (wr.v_begin < half_lo || wr.v_end > half_hi)) return fail("wave values outside the chunk's run");
            if (wr.g_begin < h.n_groups && wr.v_begin != groups[wr.g_begin].val_off + wr.val_begin) return fail("wave v_begin");
            if (wr.val_begin != (uint32_t)wr.j_begin * kWave) return fail("wave val_begin");
            // the kernel walks (v_end - v_begin) / 64 steps from (g_begin, j_begin), moving to the
            // next group at each group's last step: that walk must end at (g_end, j_end)
            {
                uint64_t steps = 0;
                for (uint32_t g = wr.g_begin; g <= wr.g_end && g < h.n_groups; ++g) {
                    const int jlo = g == wr.g_begin ? wr.j_begin : 0;
                    const int jhi = g == wr.g_end ? wr.j_end : groups[g].cmax;
                    if (jhi < jlo) return fail("wave step range");
                    if (g != wr.g_begin && g != wr.g_end && groups[g].cmax == 0) return fail("empty group");
                    steps += (uint64_t)(jhi - jlo);
                }
                if (steps * kWave != (uint64_t)(wr.v_end - wr.v_begin)) return fail("wave step count");
                if (wr.g_begin < h.n_groups && wr.j_begin >= groups[wr.g_begin].cmax && steps) return fail("wave starts past its group's end");
            }
            for (uint32_t g = wr.g_begin; g <= wr.g_end && g < h.n_groups; ++g) {
                const GroupRec &gr = groups[g];
                const int jlo = g == wr.g_begin ? wr.j_begin : 0;
                const int jhi = g == wr.g_end ? wr.j_end : gr.cmax;
                if (jhi <= jlo) continue;
                if (jhi > gr.cmax) return fail("wave step range");
                if (gr.nzrank < cr.nzrank0 || gr.nzrank >= cr.nzrank0 + cr.ntiles) return fail("group tile outside chunk");
                if (gr.nlanes > kWave || gr.nvb > kMaxVbPerGroup || gr.nvb == 0) return fail("group size");
                if ((gr.val_off & 63u) || (uint64_t)gr.val_off + (uint64_t)gr.cmax * kWave > h.n_vals) return fail("group value run");
                {   // scatter rounds: (row slot, round) pairs are unique and rounds stay below nrounds
                    uint8_t used[CSB_MAX_BLOCK][2] = {{0}};
                    for (int lane = 0; lane < gr.nlanes; ++lane) {
                        const uint8_t slot = idx[gr.idx_off + 4 * lane], rk = idx[gr.idx_off + 4 * lane + 1] >> 4;
                        if (rk >= gr.nrounds) return fail("scatter round");
                        if (used[slot][rk >> 3] >> (rk & 7) & 1) return fail("two lanes of one scatter round share a row");
                        used[slot][rk >> 3] |= (uint8_t)(1u << (rk & 7));
                    }
                }
                if (g < cr.g0 || g >= cr.g0 + cr.ng) return fail("group outside the chunk's record window");
                if (gr.vb_off < cr.vb0 || gr.vb_off + gr.nvb > cr.vb0 + cr.nvbs) return fail("vb outside the chunk's record window");
                if (gr.idx_off < cr.idx0) return fail("index bytes before the chunk's window");
                if ((uint64_t)gr.vb_off + gr.nvb > h.n_vbs) return fail("vb range");
                const uint32_t tile = nz_tiles[gr.nzrank];
                const uint32_t tile_h = (uint32_t)std::min<int64_t>(br, rows_out - (int64_t)tile * br);
                const size_t col_base = (size_t)gr.idx_off + align_up(4 * (size_t)gr.nlanes, 8);
                const int cpad = (gr.cmax + 3) & ~3;
                if ((gr.idx_off & 7u) || gr.cmax % kStepQuantum || jlo % kStepQuantum || jhi % kStepQuantum) return fail("group alignment");
                // input-offset lists: the block's columns, then the zero entry up to the padded length
                for (int k = 0; k < gr.nvb; ++k) {
                    const VbRec &v = vbs[gr.vb_off + k];
                    if (v.c > gr.cmax || v.c == 0 || v.r == 0 || (uint32_t)v.lane0 + v.r > gr.nlanes) return fail("vb shape");
                    if (v.val_off != gr.val_off || v.desc_pos != gr.idx_off) return fail("vb group fields");
                    if ((v.list_pos & 7u) || v.list_pos < col_base || (size_t)v.list_pos + 2 * (size_t)cpad > h.idx_bytes) return fail("vb list position");
                    for (int j = jlo & ~3; j < ((jhi + 3) & ~3) && j < cpad; ++j) {
                        const size_t ia = (size_t)v.list_pos + 2 * (size_t)j;
                        if (ia + 1 >= h.idx_bytes || ia + 1 >= (size_t)cr.idx0 + cr.idx_bytes) return fail("input offset list position");
                        const uint32_t o = (uint32_t)idx[ia] | (uint32_t)idx[ia + 1] << 8;
                        if (j >= v.c) { if (o != (uint32_t)cols * 4u) return fail("input offset padding"); continue; }
                        if ((o & 3u) || o / 4 >= (uint32_t)cols) return fail("input offset");
                    }
                }
                for (int j = jlo; j < jhi; ++j) {
                    for (int lane = 0; lane < kWave; ++lane) {
                        const uint64_t va = (uint64_t)gr.val_off + (uint64_t)j * kWave + lane;
                        if (va >= h.n_vals) return fail("value offset");
                        if (va < wr.v_begin || va >= wr.v_end) return fail("value outside the wave's window");
                        if (lane >= gr.nlanes) { if (val_at(va) != 0.0f) return fail("value padding (lane)"); continue; }
                        if ((size_t)gr.idx_off + 4 * lane + 3 >= h.idx_bytes) return fail("lane descriptor offset");
                        const uint8_t slot = idx[gr.idx_off + 4 * lane], k = idx[gr.idx_off + 4 * lane + 1] & 15;
                        if (k >= gr.nvb) return fail("lane vb number");
                        const VbRec &v = vbs[gr.vb_off + k];
                        const size_t lo = (size_t)idx[gr.idx_off + 4 * lane + 2] | (size_t)idx[gr.idx_off + 4 * lane + 3] << 8;
                        if ((size_t)gr.idx_off + lo != (size_t)v.list_pos) return fail("lane list offset");
                        if (lane < v.lane0 || lane >= v.lane0 + v.r) return fail("lane outside its vb");
                        if (slot >= tile_h) return fail("row slot");
                        if (j >= v.c) { if (val_at(va) != 0.0f) return fail("value padding (step)"); continue; }
                        const size_t ia = (size_t)v.list_pos + 2 * (size_t)j;
                        const int64_t gc = ((uint32_t)idx[ia] | (uint32_t)idx[ia + 1] << 8) / 4;
                        const size_t cell = (size_t)((int64_t)tile * br + slot) * cols + gc;
                        if (seen[cell]) return fail("entry referenced twice");
                        seen[cell] = 1;
                        got[cell] = val_at(va);
                        ++vals_used;
                    }
                }
            }
        }
        if (v_expect != cr.v0 + 4 * cr.nv4 && cr.nv4) return fail("wave value runs do not cover the chunk's run");
        for (uint32_t s = 0; s < cr.ntiles; ++s) {
            const uint32_t tile = nz_tiles[cr.nzrank0 + s];
            int sid = -1, part = -1;
            if (s == 0 && cr.sid_first >= 0) { sid = cr.sid_first; part = cr.part_first; }
            else if (s == cr.ntiles - 1 && cr.sid_last >= 0) { sid = cr.sid_last; part = cr.part_last; }
            if (sid >= 0) {
                if ((uint32_t)sid >= h.n_shared || shared[sid].tile != tile) return fail("shared tile record");
                if ((uint32_t)part >= shared[sid].nparts) return fail("shared part number");
                if (shared[sid].nparts <= 32) {                // (the seen-mask covers tiles of up to 32 parts)
                    if (parts_seen[sid] >> part & 1u) return fail("shared part twice");
                    parts_seen[sid] |= 1u << part;
                }
                if (shared[sid].partial_off + shared[sid].nparts > h.n_partial_slots) return fail("partial slot");
                tile_written[tile] = 1;   // by the last part to arrive
            } else {
                if (tile_written[tile]) return fail("tile written twice");
                tile_written[tile] = 1;
            }
        }
    }
    for (uint32_t s = 0; s < h.n_shared; ++s)
        if (shared[s].nparts <= 32 && parts_seen[s] != (shared[s].nparts == 32 ? 0xffffffffu : (1u << shared[s].nparts) - 1))
            return fail("shared tile with a missing part");
    for (uint32_t z = 0; z < h.n_zero_tiles; ++z) {
        if (zero_tiles[z] >= n_tiles || tile_written[zero_tiles[z]]) return fail("zero tile");
        tile_written[zero_tiles[z]] = 1;
    }
    for (uint32_t t = 0; t < n_tiles; ++t) if (!tile_written[t]) return fail("tile never written");
    if (vals_used != m->val.size()) return fail("not every value referenced exactly once");
    if (std::memcmp(expect.data(), got.data(), expect.size() * sizeof(float)) != 0) return fail("image does not decode to the matrix");
    if (pl.stream.valid) return validate_stream(m);
    return CSB_OK;
}

}  // namespace csb

// A matrix that a GRU handle has planned keeps that row layout when it is planned again (also after
// csb_set_value_format made the plan invalid): the handle's step kernels depend on it.
// (A plan the caller asks for may take all 256 compute units again, whatever share of them an RNN
// handle had left the matrix.)
extern "C" int csb_plan(csb_matrix *m, int32_t n_chunks, csb_plan_stats *stats) {
    if (m) { m->stream_wg_limit = 256; m->stream_cell_gates = 0; }
    return csb::plan_matrix(m, n_chunks, 16, m ? m->plan.split : csb::SplitSpec{}, stats, 0);
}

extern "C" int csb_plan_ex(csb_matrix *m, int32_t n_chunks, int32_t mode, csb_plan_stats *stats) {
    if (mode == 3 || mode == 4) { csb::set_error("csb_plan: mode must be 0 (auto), 1 (whole tiles) or 2 (equal split)"); return CSB_EINVAL; }
    if (m) { m->stream_wg_limit = 256; m->stream_cell_gates = 0; }
    return csb::plan_matrix(m, n_chunks, 16, m ? m->plan.split : csb::SplitSpec{}, stats, mode);
}

extern "C" int csb_plan_stats_get(const csb_matrix *m, csb_plan_stats *stats) {
    if (!m || !stats) { csb::set_error("csb_plan_stats_get: NULL pointer"); return CSB_EINVAL; }
    if (!m->plan.valid) { csb::set_error("csb_plan_stats_get: matrix not planned"); return CSB_ESTATE; }
    *stats = m->plan.stats;
    return CSB_OK;
}

extern "C" int csb_plan_rows(csb_matrix *m, int32_t n_workgroups, int32_t min_rounds, csb_plan_stats *stats) {
    if (n_workgroups < 0 || min_rounds < 0) { csb::set_error("csb_plan_rows: negative parameter"); return CSB_EINVAL; }
    if (m) { m->stream_wg_limit = 256; m->stream_cell_gates = 0; }
    int rc = csb::plan_matrix(m, 0, 16, csb::SplitSpec{}, nullptr, 4);
    if (rc != CSB_OK) return rc;
    rc = csb::plan_stream(m, n_workgroups, min_rounds, stats);
    if (rc != CSB_OK) return rc;
    if (!m->plan.stream.valid) {
        m->plan.valid = false;
        csb::set_error("csb_plan_rows: the matrix does not fit the row-owned layout");
        return CSB_EUNSUPPORTED;
    }
    return CSB_OK;
}

extern "C" int csb_plan_validate(const csb_matrix *m) { return csb::validate_plan(m); }

extern "C" size_t csb_device_bytes(const csb_matrix *m) {
    return (m && m->plan.valid) ? m->plan.image.size() : 0;
}

extern "C" size_t csb_workspace_bytes(const csb_matrix *m, int32_t batch) {
    if (!m || !m->plan.valid || batch <= 0) return 0;
    // one 64-bit word (value, launch tag) per row of every partial tile sum
    return (size_t)m->plan.hdr.n_partial_slots * m->plan.hdr.br * 8 * (size_t)batch;
}
