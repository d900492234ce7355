// CSB-MVM (Sec. 4.3.1) for gfx950: y = A x from the planned device image.
//
// One workgroup per chunk, one contiguous range of group steps per wavefront.  Inside a
// group, lane l owns one kernel-matrix row of one virtual block (inner-block parallelism
// over rows, inter-block parallelism over the lanes' different blocks, as the two
// hierarchy levels of Sec. 4.3.1) and walks that block's columns; a step reads the active
// lanes' values as one contiguous run of the value stream.  Row results go to a
// per-wavefront accumulator in LDS (the role of NeuronAccumBuffer) and are summed over
// wavefronts in a fixed order; row tiles shared by several workgroups are merged by the
// last workgroup to arrive, again in a fixed order, so results are bitwise reproducible.
#include <hip/hip_runtime.h>

#include <atomic>
#include <map>
#include <mutex>
#include <type_traits>

#include "csbrnn_debug.h"
#include "csb_internal.hpp"
#include "csb_kernels.hpp"

namespace csb {

DevMat dev_mat(const csb_matrix *m) {
    const DevHeader &h = m->plan.hdr;
    uint8_t *b = (uint8_t *)m->d_buf;
    DevMat d{};
    d.chunks = (const ChunkRec *)(b + h.off_chunks);
    d.waves = (const WaveRec *)(b + h.off_waves);
    d.groups = (const GroupRec *)(b + h.off_groups);
    d.vbs = (const VbRec *)(b + h.off_vbs);
    d.idx = b + h.off_idx;
    d.vals = (const float *)(b + h.off_vals);
    d.nz_tiles = (const uint32_t *)(b + h.off_nz_tiles);
    d.zero_tiles = (const uint32_t *)(b + h.off_zero_tiles);
    d.shared = (const SharedRec *)(b + h.off_shared);
    d.counters = (uint32_t *)(b + h.off_counters);
    d.n_chunks = h.n_chunks; d.waves_per_chunk = h.waves_per_chunk;
    d.n_zero_tiles = h.n_zero_tiles; d.n_shared = h.n_shared;
    d.br = h.br; d.bc = h.bc;
    d.rows_out = (uint32_t)h.rows_out; d.cols = (uint32_t)h.cols;
    d.n_groups = h.n_groups;
    d.n_nz_tiles = h.n_nz_tiles;
    d.idx_bytes = (uint32_t)h.idx_bytes;
    d.val_fmt = h.val_fmt;
    d.seg_meta = h.seg_meta;
    d.vals_bytes = (uint32_t)std::min<uint64_t>(h.n_vals * (h.val_fmt == CSB_VAL_F32 ? 4u : 2u), 0x7fffff00u);
    d.tile_g0 = (const uint32_t *)(b + h.off_tile_g0);
    d.tile_seg0 = (const uint32_t *)(b + h.off_tile_seg0);
    d.segs = (const SegRec *)(b + h.off_segs);
    return d;
}

__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// LDS map of one workgroup (byte offsets from the start of dynamic LDS).
struct LdsMap {
    uint32_t zpad;        // floats of the staged input vector (with the zero entry behind it)
    uint32_t meta_off;    // bytes: group records | index bytes
    uint32_t acc_off;     // bytes: [NW][kAccPlanes][acc_rows] accumulators
    uint32_t red_off;     // bytes: [4][256] partial sums of the final reduction
};

// Uniform copies of the records (every field through a scalar register).
// The records a workgroup / wavefront starts from are read-only and their address is the same
// for every lane: read through the constant address space they come in over the scalar path,
// which answers sooner than a vector load and needs no lane to be picked afterwards.
#define CSB_CONST_AS __attribute__((address_space(4)))
__device__ __forceinline__ ChunkRec load_chunk(const ChunkRec *gp) {
    const CSB_CONST_AS ChunkRec *p = (const CSB_CONST_AS ChunkRec *)gp;
    ChunkRec c;
    c.nzrank0 = uni(p->nzrank0); c.ntiles = uni(p->ntiles);
    c.sid_first = (int32_t)uni((uint32_t)p->sid_first); c.part_first = (int32_t)uni((uint32_t)p->part_first);
    c.sid_last = (int32_t)uni((uint32_t)p->sid_last); c.part_last = (int32_t)uni((uint32_t)p->part_last);
    c.g0 = uni(p->g0); c.ng = uni(p->ng);
    c.idx0 = uni(p->idx0); c.idx_bytes = uni(p->idx_bytes);
    c.vb0 = c.nvbs = c.v0 = c.nv4 = 0;          // host-side bookkeeping, not needed here
    c.pad[0] = c.pad[1] = 0;
    return c;
}

__device__ __forceinline__ WaveRec load_wave(const WaveRec *gp) {
    const CSB_CONST_AS WaveRec *p = (const CSB_CONST_AS WaveRec *)gp;
    WaveRec w;
    w.g_begin = uni(p->g_begin); w.g_end = uni(p->g_end);
    w.j_begin = (uint16_t)uni(p->j_begin); w.j_end = (uint16_t)uni(p->j_end);
    w.val_begin = 0; w.v_begin = uni(p->v_begin); w.v_end = uni(p->v_end);
    w.pad[0] = w.pad[1] = 0;
    return w;
}

// Barrier that orders LDS traffic only: global loads still in flight stay in flight.
__device__ __forceinline__ void lds_only_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

constexpr int kSpmvWaves = 16;
constexpr int kSpmvThreads = kSpmvWaves * 64;
constexpr int kStampsPerChunk = 8 + 3 * kSpmvWaves;
constexpr int kStepsInFlight = 32;   // column steps of a wavefront whose values are loaded at once

// A guarded load into a named register (arrays of these end up in scratch memory).
#define CSB_LD4(name, src, idx, n) \
    float4 name = make_float4(0.f, 0.f, 0.f, 0.f); \
    { const uint32_t i_ = (idx); if (i_ < (n)) name = (src)[i_]; }
#define CSB_LD2(name, src, idx, n) \
    uint2 name = make_uint2(0u, 0u); \
    { const uint32_t i_ = (idx); if (i_ < (n)) name = (src)[i_]; }
#define CSB_ST(dst, idx, n, name) \
    { const uint32_t i_ = (idx); if (i_ < (n)) (dst)[i_] = name; }

// The two kernel values a word of a 16-bit value stream holds (even step low), widened.
template <int VF>
__device__ __forceinline__ void unpack_pair(uint32_t w, float &lo, float &hi) {
    if constexpr (VF == CSB_VAL_BF16) {
        lo = __uint_as_float(w << 16);
        hi = __uint_as_float(w & 0xffff0000u);
    } else {
        lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
        hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    }
}

__global__ void commit_gates_kernel(const GateSrc s) {
    const uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u < s.H) gate_value(s, u, true);
}

// One workgroup per chunk.  Records and the input vector go to LDS; the kernel values never
// do: a wavefront's steps are consecutive 64-float runs of the value stream, so lane l loads
// word l of every run straight into a register (one coalesced 256-byte read per step) and
// multiplies it there.  VF: storage format of the value stream (CSB_VAL_*); a 16-bit stream
// holds one word per lane and pair of steps, so a step pair is one coalesced 256-byte read.
// GATED: the two input segments are GateSrc records (cell outputs computed while staging);
// otherwise plain vectors, and the kernel takes only their pointers.
template <bool GATED> struct SpmvSrc { const float *a; };
template <> struct SpmvSrc<true> : GateSrc {};
template <int VF, bool GATED>
__device__ __forceinline__ void spmv_body(const DevMat &m, const SpmvSrc<GATED> &g0, const uint32_t n0,
                                          const SpmvSrc<GATED> &g1, float *__restrict__ y,
                                          unsigned long long *__restrict__ partials, const uint32_t epoch, const LdsMap &L,
                                          unsigned long long *__restrict__ stamps, const uint32_t c) {
    extern __shared__ float4 smem4[];
    __shared__ uint32_t s_last;
    uint8_t *smem = (uint8_t *)smem4;
    float *z = (float *)smem;                          // [zpad] input vector, z[cols] = 0
    uint8_t *meta = smem + L.meta_off;
    float *acc = (float *)(smem + L.acc_off);          // [NW][kAccPlanes][ntiles * br]
    float *red = (float *)(smem + L.red_off);          // [4][256]
    constexpr int NW = kSpmvWaves, NT = kSpmvThreads, CAP = kStepsInFlight, Q = kStepQuantum;
    const uint32_t tid = threadIdx.x;
    const int lane = tid & 63, wave = (int)uni(tid >> 6);
    static_assert(kMaxStageCols / 4 <= 4 * NT, "input vector loads");
    static_assert(kChunkMetaMax <= 3 * NT * 8, "record loads");
    static_assert(kChunkMetaMax + 16 <= 2 * NT * 16, "index byte loads");
    static_assert(kAccRowsMax <= 256 && NT == 1024 && (kAccPlanes & (kAccPlanes - 1)) == 0, "final reduction layout");
    static_assert(CAP % Q == 0 && Q % 2 == 0 && (CAP & (CAP - 1)) == 0, "step quantum / batch size");

    // optional clock stamps (debug): per workgroup 8 phase stamps, then per wavefront: begin,
    // values arrived, end
    unsigned long long *st = stamps ? stamps + (size_t)c * kStampsPerChunk : nullptr;
    if (st && tid == 0) st[0] = __builtin_readcyclecounter();

    // ---- issue every global load before waiting for any ---------------------------------
    // Loads return in issue order: first what the whole workgroup needs (records, input
    // vector), then this wavefront's values.
    const ChunkRec cr = load_chunk(m.chunks + c);
    const WaveRec wr = load_wave(m.waves + (size_t)c * NW + wave);
    // records: groups in 8-byte units, index bytes in 16-byte units
    const uint32_t gu = cr.ng * 3u, iu = cr.idx_bytes >> 4;
    const uint32_t ioff = (cr.ng * (uint32_t)sizeof(GroupRec) + 15u) & ~15u;
    const uint2 *gsrc8 = (const uint2 *)(m.groups + cr.g0);
    const float4 *isrc = (const float4 *)(m.idx + cr.idx0);
    CSB_LD2(rg0, gsrc8, tid, gu) CSB_LD2(rg1, gsrc8, tid + NT, gu) CSB_LD2(rg2, gsrc8, tid + 2 * NT, gu)
    CSB_LD4(ri0, isrc, tid, iu) CSB_LD4(ri1, isrc, tid + NT, iu)
    // input vector: aligned single-source fast path, else element-wise from two sources
    const float *x0 = g0.a;
    const bool zfast = !GATED && n0 >= m.cols && (m.cols & 3u) == 0 && ((uintptr_t)x0 & 15u) == 0;
    const uint32_t z4 = zfast ? (m.cols >> 2) : 0u;
    const float4 *zsrc = (const float4 *)x0;
    CSB_LD4(rz0, zsrc, tid, z4) CSB_LD4(rz1, zsrc, tid + NT, z4) CSB_LD4(rz2, zsrc, tid + 2 * NT, z4)
    CSB_LD4(rz3, zsrc, tid + 3 * NT, z4)
    if constexpr (GATED) {                       // two segments, either one possibly a cell output still to be computed
        const uint32_t na = min(n0, m.cols);
        stage_segment(z, g0, na, tid, NT, c == 0);
        stage_segment(z + na, g1, m.cols - na, tid, NT, c == 0);
    } else if (!zfast) {
        const float *x1 = g1.a;
        for (uint32_t i = tid; i < m.cols; i += NT) z[i] = i < n0 ? x0[i] : x1[i - n0];
    }
    // values of the wavefront's first CAP steps (steps past its last one repeat the last)
    const uint32_t nsteps = (wr.v_end - wr.v_begin) >> 6;
    const uint32_t last_step = nsteps ? nsteps - 1u : 0u;
    constexpr int NR = VF == CSB_VAL_F32 ? CAP : CAP / 2;     // registers that hold CAP steps' values
    using RegT = typename std::conditional<VF == CSB_VAL_F32, float, uint32_t>::type;
    const RegT *wv = (const RegT *)m.vals + (VF == CSB_VAL_F32 ? wr.v_begin : wr.v_begin >> 1) + lane;
    const uint32_t last_reg = VF == CSB_VAL_F32 ? last_step : last_step >> 1;
    RegT R[NR];
#pragma unroll
    for (int s = 0; s < NR; ++s) R[s] = wv[(size_t)min((uint32_t)s, last_reg) * kWave];

    if (st && tid == 0) st[1] = __builtin_readcyclecounter();
    // ---- independent work while the loads fly -------------------------------------------
    const uint32_t arows = cr.ntiles * m.br;
    for (uint32_t i = tid; i < NW * kAccPlanes * arows; i += NT) acc[i] = 0.0f;
    for (uint32_t q = c; q < m.n_zero_tiles; q += m.n_chunks) {   // output tiles nobody has work for
        const uint32_t r0 = m.zero_tiles[q] * m.br;
        for (uint32_t i = tid; i < m.br; i += NT)
            if (r0 + i < m.rows_out) y[r0 + i] = 0.0f;
    }

    // ---- records and input vector into LDS ----------------------------------------------
    {
        uint2 *gd = (uint2 *)meta;
        CSB_ST(gd, tid, gu, rg0) CSB_ST(gd, tid + NT, gu, rg1) CSB_ST(gd, tid + 2 * NT, gu, rg2)
        float4 *id = (float4 *)(meta + ioff);
        CSB_ST(id, tid, iu, ri0) CSB_ST(id, tid + NT, iu, ri1)
        float4 *zd = (float4 *)z;
        CSB_ST(zd, tid, z4, rz0) CSB_ST(zd, tid + NT, z4, rz1) CSB_ST(zd, tid + 2 * NT, z4, rz2)
        CSB_ST(zd, tid + 3 * NT, z4, rz3)
        if (tid == 0) z[m.cols] = 0.0f;          // what padded steps multiply their zero values with
    }
    lds_only_barrier();
    if (st && tid == 0) st[2] = __builtin_readcyclecounter();
    if (st && lane == 0) st[8 + 3 * wave] = __builtin_readcyclecounter();
    if (st) {                                    // debug only: separate the wait for the values from the arithmetic
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (lane == 0) st[9 + 3 * wave] = __builtin_readcyclecounter();
    }

    // ---- the wavefront's steps ------------------------------------------------------------
    // Lane l owns one kernel-matrix row of one virtual block of the current group (inner-
    // block parallelism over rows, inter-block parallelism over the lanes' different blocks)
    // and walks the block's list of input offsets.  Eight steps at a time: the gathers of all
    // eight, then the multiply-adds, with the next eight list entries already on their way.
    // The records of the next group are fetched while the current one is being worked on.
    {
        const uint8_t *lidx = meta + ioff;
        const uint8_t *zb = (const uint8_t *)z;
        float *myacc = acc + wave * (kAccPlanes * arows);
        const uint32_t g_last = cr.g0 + cr.ng - 1u;       // last group with records in LDS
        // a group's record words: {idx_off, nzrank} and {cmax | nvb << 16 | nlanes << 24, nrounds}
        auto rec_lo = [&](uint32_t g) { return *(const uint2 *)(meta + (min(g, g_last) - cr.g0) * (uint32_t)sizeof(GroupRec) + 8u); };
        auto rec_hi = [&](uint32_t g) { return *(const uint2 *)(meta + (min(g, g_last) - cr.g0) * (uint32_t)sizeof(GroupRec) + 16u); };
        // a lane's descriptor; lanes without a row use lane 0's list (their values are all zero)
        auto lane_word = [&](uint32_t idx_off, uint32_t nlanes) {
            return *(const uint32_t *)(lidx + (idx_off - cr.idx0) + 4u * ((uint32_t)lane < nlanes ? (uint32_t)lane : 0u));
        };
        uint32_t g = wr.g_begin, j = wr.j_begin;
        uint2 clo = make_uint2(cr.idx0, 0u), chi = make_uint2(0u, 0u);
        uint32_t cd = 0;
        if (nsteps) {
            clo = rec_lo(g); chi = rec_hi(g);
            cd = lane_word(uni(clo.x), uni(chi.x) >> 24);
        }
        for (uint32_t base = 0; base < nsteps; base += CAP) {
            if (base) {                          // a wavefront with more than CAP steps: next batch
#pragma unroll
                for (int s = 0; s < NR; ++s)
                    R[s] = wv[(size_t)min((VF == CSB_VAL_F32 ? base : base >> 1) + (uint32_t)s, last_reg) * kWave];
            }
            const uint32_t bsteps = min((uint32_t)CAP, nsteps - base);
            uint32_t s = 0;
            while (s < bsteps) {                                     // one run: steps of one group
                const uint32_t ib = uni(clo.x) - cr.idx0, nzrank = uni(clo.y), w2 = uni(chi.x);
                const uint32_t cmax = w2 & 0xffffu, nlanes = w2 >> 24;
                const uint32_t jhi = g == wr.g_end ? (uint32_t)wr.j_end : cmax;
                const uint32_t run = min(jhi - j, bsteps - s);
                const uint2 nlo = rec_lo(g + 1u), nhi = rec_hi(g + 1u);   // next group's records
                const bool act = (uint32_t)lane < nlanes;
                const uint32_t d = cd;
                const uint32_t *zw = (const uint32_t *)(lidx + ib + (d >> 16) + 2u * j);   // this lane's position in its block's list
                uint32_t w0 = zw[0], w1 = zw[1], w2_ = zw[2], w3 = zw[3];
                float a0 = 0.0f, a1 = 0.0f;
                for (uint32_t t = 0; t < run; t += 8) {
                    const uint32_t left = run - t, s0 = s + t;
                    const uint32_t c0 = w0, c1 = w1, c2 = w2_, c3 = w3;
                    zw += 4;
                    if (left > 8) { w0 = zw[0]; w1 = zw[1]; w2_ = zw[2]; w3 = zw[3]; }   // uniform
                    // pairs of steps past the end of the run are skipped (uniform branches)
                    float z0, z1, z2 = 0.0f, z3 = 0.0f, z4 = 0.0f, z5 = 0.0f, z6 = 0.0f, z7 = 0.0f;
                    z0 = *(const float *)(zb + (c0 & 0xffffu)); z1 = *(const float *)(zb + (c0 >> 16));
                    if (left > 2) { z2 = *(const float *)(zb + (c1 & 0xffffu)); z3 = *(const float *)(zb + (c1 >> 16)); }
                    if (left > 4) { z4 = *(const float *)(zb + (c2 & 0xffffu)); z5 = *(const float *)(zb + (c2 >> 16)); }
                    if (left > 6) { z6 = *(const float *)(zb + (c3 & 0xffffu)); z7 = *(const float *)(zb + (c3 >> 16)); }
                    // The value registers of steps s0 .. s0 + 7.  s0 is even and uniform: one of 16
                    // copies of the multiply-adds, each with its registers named outright, is
                    // branched to (indexing the register file with a run-time index costs five
                    // instructions per read).
                    auto mads = [&](auto pair0) {
                        constexpr int P0 = decltype(pair0)::value;      // first pair of steps of the block
                        if constexpr (VF == CSB_VAL_F32) {
                            a0 = fmaf(R[(2 * P0) & (CAP - 1)], z0, a0); a1 = fmaf(R[(2 * P0 + 1) & (CAP - 1)], z1, a1);
                            if (left > 2) { a0 = fmaf(R[(2 * P0 + 2) & (CAP - 1)], z2, a0); a1 = fmaf(R[(2 * P0 + 3) & (CAP - 1)], z3, a1); }
                            if (left > 4) { a0 = fmaf(R[(2 * P0 + 4) & (CAP - 1)], z4, a0); a1 = fmaf(R[(2 * P0 + 5) & (CAP - 1)], z5, a1); }
                            if (left > 6) { a0 = fmaf(R[(2 * P0 + 6) & (CAP - 1)], z6, a0); a1 = fmaf(R[(2 * P0 + 7) & (CAP - 1)], z7, a1); }
                        } else {                 // a pair of steps shares a word
                            float lo, hi;
                            unpack_pair<VF>(R[P0 & (NR - 1)], lo, hi); a0 = fmaf(lo, z0, a0); a1 = fmaf(hi, z1, a1);
                            if (left > 2) { unpack_pair<VF>(R[(P0 + 1) & (NR - 1)], lo, hi); a0 = fmaf(lo, z2, a0); a1 = fmaf(hi, z3, a1); }
                            if (left > 4) { unpack_pair<VF>(R[(P0 + 2) & (NR - 1)], lo, hi); a0 = fmaf(lo, z4, a0); a1 = fmaf(hi, z5, a1); }
                            if (left > 6) { unpack_pair<VF>(R[(P0 + 3) & (NR - 1)], lo, hi); a0 = fmaf(lo, z6, a0); a1 = fmaf(hi, z7, a1); }
                        }
                    };
                    static_assert(CAP == 32, "one case per pair of steps of a batch");
                    switch ((s0 >> 1) & 15u) {
                    case 0: mads(std::integral_constant<int, 0>{}); break;
                    case 1: mads(std::integral_constant<int, 1>{}); break;
                    case 2: mads(std::integral_constant<int, 2>{}); break;
                    case 3: mads(std::integral_constant<int, 3>{}); break;
                    case 4: mads(std::integral_constant<int, 4>{}); break;
                    case 5: mads(std::integral_constant<int, 5>{}); break;
                    case 6: mads(std::integral_constant<int, 6>{}); break;
                    case 7: mads(std::integral_constant<int, 7>{}); break;
                    case 8: mads(std::integral_constant<int, 8>{}); break;
                    case 9: mads(std::integral_constant<int, 9>{}); break;
                    case 10: mads(std::integral_constant<int, 10>{}); break;
                    case 11: mads(std::integral_constant<int, 11>{}); break;
                    case 12: mads(std::integral_constant<int, 12>{}); break;
                    case 13: mads(std::integral_constant<int, 13>{}); break;
                    case 14: mads(std::integral_constant<int, 14>{}); break;
                    default: mads(std::integral_constant<int, 15>{}); break;
                    }
                }
                // the next group's lane descriptors (its records have arrived by now)
                const uint32_t nd = lane_word(uni(nlo.x), uni(nhi.x) >> 24);
                // Row results into the wavefront's accumulator.  Lanes of different virtual blocks
                // may target the same row: the planner numbered the lanes of each row, and lane
                // number q of a row adds into accumulator copy q % kAccPlanes, so all lanes of a
                // round (q / kAccPlanes, nearly always the only one) hit different words and a
                // plain read-add-write does (LDS float atomics take a few clocks per lane).  A
                // wavefront's LDS operations execute in program order, which fixes the sum.
                {
                    const float asum = a0 + a1;
                    const uint32_t q = (d >> 12) & 15u;
                    float *dst = myacc + (q & (kAccPlanes - 1)) * arows + (nzrank - cr.nzrank0) * m.br + (d & 0xffu);
                    const uint32_t round = act ? q / kAccPlanes : 0xffffffffu;
                    const uint32_t nr = (uni(chi.y) & 0xffffu) + kAccPlanes - 1;
                    for (uint32_t rq = 0; rq < nr / kAccPlanes; ++rq)
                        if (round == rq) *dst += asum;
                }
                s += run;
                j += run;
                if (j == jhi) { ++g; j = 0; clo = nlo; chi = nhi; cd = nd; }
            }
        }
    }
    if (st && lane == 0) st[10 + 3 * wave] = __builtin_readcyclecounter();
    __syncthreads();
    if (st && tid == 0) st[3] = __builtin_readcyclecounter();

    // Sum of the NW * kAccPlanes accumulator copies, in a fixed order: four partial sums of a
    // quarter of the copies each, then their sum; store or hand over as a partial.
    {
        constexpr uint32_t C = NW * kAccPlanes;
        const uint32_t part = tid >> 8, i = tid & 255u;
        if (i < arows) {
            float p = 0.0f;
#pragma unroll
            for (uint32_t cpy = 0; cpy < C / 4; ++cpy) p += acc[(part * (C / 4) + cpy) * arows + i];
            red[part * 256u + i] = p;
        }
    }
    __syncthreads();
    for (uint32_t i = tid; i < arows; i += NT) {
        const float s = (red[i] + red[256u + i]) + (red[512u + i] + red[768u + i]);
        const uint32_t ts = i / m.br, ri_ = i - ts * m.br;
        const uint32_t row = m.nz_tiles[cr.nzrank0 + ts] * m.br + ri_;
        // a partial travels as one 64-bit word: launch tag in the high half, value in the low
        const unsigned long long pk = ((unsigned long long)epoch << 32) | (unsigned long long)__float_as_uint(s);
        if (ts == 0 && cr.sid_first >= 0)
            __hip_atomic_store(&partials[(size_t)(m.shared[cr.sid_first].partial_off + cr.part_first) * m.br + ri_], pk,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else if (ts == cr.ntiles - 1 && cr.sid_last >= 0)
            __hip_atomic_store(&partials[(size_t)(m.shared[cr.sid_last].partial_off + cr.part_last) * m.br + ri_], pk,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else if (row < m.rows_out)
            y[row] = s;
    }
    if (st && tid == 0) st[4] = __builtin_readcyclecounter();
    // Shared tiles: every workgroup publishes its partial, then takes a ticket; the one that
    // draws the last ticket adds the parts in part order.  Nothing here relies on the order
    // in which stores to different addresses become visible: a partial is valid only once
    // its word shows this launch's tag, and the reader polls for that (all writers have
    // issued their stores before taking their tickets, so the poll ends; it is bounded
    // anyway and poisons the row with NaN if the bound is ever hit).
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int32_t sid = e == 0 ? cr.sid_first : cr.sid_last;
        if (sid < 0) continue;               // uniform over the workgroup
        __syncthreads();
        const SharedRec sr = m.shared[sid];
        if (tid == 0) {
            const uint32_t t = __hip_atomic_fetch_add(&m.counters[sid], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (t + 1u) % sr.nparts == 0u ? 1u : 0u;
        }
        __syncthreads();
        if (s_last) {
            for (uint32_t i = tid; i < m.br; i += NT) {
                const uint32_t row = sr.tile * m.br + i;
                if (row >= m.rows_out) continue;
                float s = 0.0f;
                for (uint32_t p = 0; p < sr.nparts; ++p) {
                    const unsigned long long *src = &partials[(size_t)(sr.partial_off + p) * m.br + i];
                    unsigned long long v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    for (uint32_t spin = 0; (uint32_t)(v >> 32) != epoch && spin < (1u << 22); ++spin) {
                        __builtin_amdgcn_s_sleep(1);
                        v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if ((uint32_t)(v >> 32) == epoch) s += __uint_as_float((uint32_t)v);
                    else {                       // gave up: poison the row and tell the host (csb_status)
                        s = __builtin_nanf("");
                        __hip_atomic_store(&m.counters[m.n_shared], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
                y[row] = s;
            }
        }
        __syncthreads();
    }
    if (st && tid == 0) st[5] = __builtin_readcyclecounter();
}

template <int VF, bool GATED>
__global__ __launch_bounds__(kSpmvThreads) void spmv_kernel(const DevMat m, const SpmvSrc<GATED> g0,
                                                             const uint32_t n0, const SpmvSrc<GATED> g1,
                                                             float *__restrict__ y, unsigned long long *__restrict__ partials,
                                                             const uint32_t epoch, const LdsMap L,
                                                             unsigned long long *__restrict__ stamps) {
    spmv_body<VF, GATED>(m, g0, n0, g1, y, partials, epoch, L, stamps, blockIdx.x);
}

// Several independent mat-vecs in one launch (blockIdx.y picks one): the per-step products of
// different layers of a stacked model on the streaming path.
struct SpmvJobs {
    DevMat m[kMaxJobsPerLaunch];
    SpmvSrc<true> g0[kMaxJobsPerLaunch], g1[kMaxJobsPerLaunch];
    uint32_t n0[kMaxJobsPerLaunch], epoch[kMaxJobsPerLaunch];
    float *y[kMaxJobsPerLaunch];
    unsigned long long *partials[kMaxJobsPerLaunch];
    LdsMap L[kMaxJobsPerLaunch];
};
template <int VF>
__global__ __launch_bounds__(kSpmvThreads) void spmv_multi_kernel(const SpmvJobs J) {
    const uint32_t j = blockIdx.y;
    if (blockIdx.x >= J.m[j].n_chunks) return;              // the grid is as wide as the job with most chunks
    spmv_body<VF, true>(J.m[j], J.g0[j], J.n0[j], J.g1[j], J.y[j], J.partials[j], J.epoch[j], J.L[j], nullptr, blockIdx.x);
}

hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes) {
    static std::mutex mu;
    static std::map<std::pair<const void *, int>, size_t> have;   // (kernel, device) -> limit set so far
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    size_t &limit = have[{kernel, dev}];
    if (bytes <= limit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) limit = bytes;
    return e;
}

__global__ void clear_words_kernel(unsigned long long *p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ull;
}

// What a launch needs besides its operands: the LDS map, and the launch tag of the merge words
// (a workspace seen for the first time, or a wrapped tag, is cleared first so that no stale
// word can carry the tag; tags are unique per launch across the process -- workspaces may be
// shared between matrices -- and every 2^32 launches a new generation starts).
static size_t prepare_spmv(const csb_matrix *mat, unsigned long long *partials, hipStream_t stream, LdsMap *Lout,
                           uint32_t *epoch_out) {
    const DevHeader &h = mat->plan.hdr;
    LdsMap L{};
    L.zpad = ((uint32_t)h.cols + 1u + 63u) & ~63u;
    L.meta_off = L.zpad * 4u;
    L.acc_off = L.meta_off + h.meta_cap;
    L.red_off = L.acc_off + h.waves_per_chunk * kAccPlanes * h.max_chunk_tiles * h.br * (uint32_t)sizeof(float);
    uint32_t epoch = 0;
    if (h.n_partial_slots) {
        uint32_t gen = 0;
        epoch = reserve_tags(1, &gen);
        const size_t words = (size_t)h.n_partial_slots * h.br;
        if (mat->ws_seen != (const void *)partials || mat->epoch != gen) {
            hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)std::min<size_t>((words + 255) / 256, 1024)), dim3(256), 0,
                               stream, partials, words);
            mat->ws_seen = partials;
            mat->epoch = gen;
        }
    }
    *Lout = L;
    *epoch_out = epoch;
    return (size_t)L.red_off + 4 * 256 * sizeof(float);
}

template <bool GATED>
static hipError_t launch_spmv(const csb_matrix *mat, const SpmvSrc<GATED> &g0, uint32_t n0, const SpmvSrc<GATED> &g1, float *y,
                              unsigned long long *partials, hipStream_t stream, unsigned long long *stamps = nullptr) {
    const DevHeader &h = mat->plan.hdr;
    if (h.waves_per_chunk != (uint32_t)kSpmvWaves) return hipErrorInvalidValue;
    const DevMat dm = dev_mat(mat);
    LdsMap L;
    uint32_t epoch;
    const size_t lds = prepare_spmv(mat, partials, stream, &L, &epoch);
    auto go = [&](auto kern, int nw) -> hipError_t {
        hipError_t e = ensure_dynamic_lds((const void *)kern, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(h.n_chunks), dim3(nw * 64), lds, stream, dm, g0, n0, g1, y, partials, epoch, L, stamps);
        return hipGetLastError();
    };
    if (h.val_fmt == CSB_VAL_F16) return go(spmv_kernel<CSB_VAL_F16, GATED>, kSpmvWaves);
    if (h.val_fmt == CSB_VAL_BF16) return go(spmv_kernel<CSB_VAL_BF16, GATED>, kSpmvWaves);
    return go(spmv_kernel<CSB_VAL_F32, GATED>, kSpmvWaves);
}

int spmv_segments(const csb_matrix *m, const float *d_x0, uint32_t n0, const float *d_x1, float *d_y,
                  void *d_ws, void *stream, unsigned long long *d_stamps) {
    if (!m->plan.valid || !m->uploaded || !m->d_buf) { set_error("csb_spmv: matrix not planned and uploaded"); return CSB_ESTATE; }
    if (m->plan.hdr.cols > (uint64_t)kMaxStageCols) { set_error("csb_spmv: more columns than the LDS staging covers"); return CSB_EUNSUPPORTED; }
    if (m->plan.hdr.n_partial_slots && !d_ws) { set_error("csb_spmv: workspace is NULL"); return CSB_EINVAL; }
    if ((uintptr_t)d_ws % 256) { set_error("csb_spmv: workspace not 256-byte aligned"); return CSB_EINVAL; }
    hipError_t e = launch_spmv<false>(m, SpmvSrc<false>{d_x0}, n0, SpmvSrc<false>{d_x1}, d_y, (unsigned long long *)d_ws,
                                      (hipStream_t)stream, d_stamps);
    if (e != hipSuccess) { set_error(std::string("csb_spmv: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

int spmv_gated(const csb_matrix *m, const GateSrc &s0, uint32_t n0, const GateSrc &s1, float *d_y, void *d_ws, void *stream) {
    if (!m->plan.valid || !m->uploaded || !m->d_buf) { set_error("csb_spmv: matrix not planned and uploaded"); return CSB_ESTATE; }
    if (m->plan.hdr.cols > (uint64_t)kMaxStageCols) { set_error("csb_spmv: more columns than the LDS staging covers"); return CSB_EUNSUPPORTED; }
    // a computed segment has exactly one entry per unit of its cell
    if ((s0.kind && s0.H != n0) || (s1.kind && (uint64_t)s1.H + n0 != m->plan.hdr.cols)) {
        set_error("csb_spmv: a computed input segment does not match the matrix's column split");
        return CSB_EINVAL;
    }
    if (m->plan.stream.valid && !m->plan.stream.cell_gates) return spmv_rows_gated(m, s0, n0, s1, d_y, stream);      // row-owned layout: no workspace
    if (m->plan.hdr.n_partial_slots && !d_ws) { set_error("csb_spmv: workspace is NULL"); return CSB_EINVAL; }
    if ((uintptr_t)d_ws % 256) { set_error("csb_spmv: workspace not 256-byte aligned"); return CSB_EINVAL; }
    SpmvSrc<true> g0, g1;
    static_cast<GateSrc &>(g0) = s0;
    static_cast<GateSrc &>(g1) = s1;
    hipError_t e = launch_spmv<true>(m, g0, n0, g1, d_y, (unsigned long long *)d_ws, (hipStream_t)stream, nullptr);
    if (e != hipSuccess) { set_error(std::string("csb_spmv: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

// Up to kMaxJobsPerLaunch independent gated mat-vecs in ONE launch (same value format); otherwise,
// or for a single one, a launch each.
int spmv_gated_multi(const SpmvGatedCall *calls, int n, void *stream) {
    bool rows = n > 1 && n <= kMaxJobsPerLaunch;            // every product in the row-owned layout: one launch of that kernel
    for (int i = 0; i < n && rows; ++i) {
        const csb_matrix *m = calls[i].mat;
        rows = m->plan.valid && m->uploaded && m->d_buf && m->plan.stream.valid && !m->plan.stream.cell_gates && m->plan.hdr.cols <= (uint64_t)kMaxStageCols &&
               m->plan.stream.val_fmt == calls[0].mat->plan.stream.val_fmt &&
               !(calls[i].s0.kind && calls[i].s0.H != calls[i].n0) &&
               !(calls[i].s1.kind && (uint64_t)calls[i].s1.H + calls[i].n0 != m->plan.hdr.cols);
    }
    if (rows) return spmv_rows_gated_multi(calls, n, stream);
    bool together = n > 1 && n <= kMaxJobsPerLaunch;
    for (int i = 0; i < n && together; ++i) {
        const csb_matrix *m = calls[i].mat;
        together = m->plan.valid && m->uploaded && m->d_buf && m->plan.hdr.val_fmt == calls[0].mat->plan.hdr.val_fmt &&
                   m->plan.hdr.waves_per_chunk == (uint32_t)kSpmvWaves && m->plan.hdr.cols <= (uint64_t)kMaxStageCols &&
                   !(m->plan.hdr.n_partial_slots && !calls[i].ws);
    }
    if (!together) {
        for (int i = 0; i < n; ++i) {
            int rc = spmv_gated(calls[i].mat, calls[i].s0, calls[i].n0, calls[i].s1, calls[i].y, calls[i].ws, stream);
            if (rc != CSB_OK) return rc;
        }
        return CSB_OK;
    }
    SpmvJobs J{};
    size_t lds = 0;
    unsigned chunks = 0;
    for (int i = 0; i < n; ++i) {
        const SpmvGatedCall &c = calls[i];
        const DevHeader &h = c.mat->plan.hdr;
        if ((c.s0.kind && c.s0.H != c.n0) || (c.s1.kind && (uint64_t)c.s1.H + c.n0 != h.cols)) {
            set_error("csb_spmv: a computed input segment does not match the matrix's column split");
            return CSB_EINVAL;
        }
        J.m[i] = dev_mat(c.mat);
        static_cast<GateSrc &>(J.g0[i]) = c.s0;
        static_cast<GateSrc &>(J.g1[i]) = c.s1;
        J.n0[i] = c.n0;
        J.y[i] = c.y;
        J.partials[i] = (unsigned long long *)c.ws;
        lds = std::max(lds, prepare_spmv(c.mat, J.partials[i], (hipStream_t)stream, &J.L[i], &J.epoch[i]));
        chunks = std::max(chunks, (unsigned)h.n_chunks);
    }
    const uint32_t vf = calls[0].mat->plan.hdr.val_fmt;
    auto go = [&](auto kern) -> hipError_t {
        hipError_t e = ensure_dynamic_lds((const void *)kern, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(chunks, (unsigned)n), dim3(kSpmvThreads), lds, (hipStream_t)stream, J);
        return hipGetLastError();
    };
    const hipError_t e = vf == CSB_VAL_F16 ? go(spmv_multi_kernel<CSB_VAL_F16>)
                       : vf == CSB_VAL_BF16 ? go(spmv_multi_kernel<CSB_VAL_BF16>) : go(spmv_multi_kernel<CSB_VAL_F32>);
    if (e != hipSuccess) { set_error(std::string("csb_spmv: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

int commit_gates(const GateSrc &s, void *stream) {
    hipLaunchKernelGGL(commit_gates_kernel, dim3((s.H + 255) / 256), dim3(256), 0, (hipStream_t)stream, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

}  // namespace csb

extern "C" int csb_upload(csb_matrix *m, void *d_buf, size_t bytes, void *stream) {
    if (!m || !d_buf) { csb::set_error("csb_upload: NULL pointer"); return CSB_EINVAL; }
    if (!m->plan.valid) { csb::set_error("csb_upload: matrix not planned"); return CSB_ESTATE; }
    if (bytes < m->plan.image.size()) { csb::set_error("csb_upload: device buffer too small"); return CSB_ENOMEM; }
    if ((uintptr_t)d_buf % 256) { csb::set_error("csb_upload: device buffer not 256-byte aligned"); return CSB_EINVAL; }
    hipError_t e = hipMemcpyAsync(d_buf, m->plan.image.data(), m->plan.image.size(), hipMemcpyHostToDevice,
                                  (hipStream_t)stream);
    if (e != hipSuccess) { csb::set_error(std::string("csb_upload: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    static std::atomic<uint64_t> serial{0};
    m->d_buf = d_buf;
    m->uploaded = true;
    m->upload_serial = ++serial;
    return CSB_OK;
}

extern "C" int csb_spmv(const csb_matrix *m, const float *d_x, float *d_y, void *d_ws, void *stream) {
    if (!m || !d_x || !d_y) { csb::set_error("csb_spmv: NULL pointer"); return CSB_EINVAL; }
    if (m->plan.valid && m->plan.split.active()) { csb::set_error("csb_spmv: matrix is planned for a GRU step"); return CSB_ESTATE; }
    // (a section whose workgroups own the units of a recurrent cell is for that cell's steps: a plain product reads the tile sections)
    if (m->plan.valid && m->plan.stream.valid && !m->plan.stream.cell_gates) {            // the row-owned section: nothing is merged, no workspace
        if (!m->uploaded || !m->d_buf) { csb::set_error("csb_spmv: matrix not planned and uploaded"); return CSB_ESTATE; }
        return csb::spmv_rows(m, d_x, d_y, stream);
    }
    if (d_ws && csb::workspace_changed_hands(d_ws, m)) m->ws_seen = nullptr;   // merge words: clear again
    return csb::spmv_segments(m, d_x, (uint32_t)m->cols, d_x, d_y, d_ws, stream, nullptr);
}

// ---- csb_spmv without a caller's workspace ---------------------------------------------------
// The partial sums of row tiles that several workgroups share (tile-based equal-split plans)
// travel through device memory: csb_spmv takes that memory from the caller's workspace,
// csb_spmv_static from this array, which every GPU the library runs on holds until the process
// ends.  In host code the array's name is only a stand-in: the address on the current device
// comes from hipGetSymbolAddress, once per device, and is what the kernels get.
namespace csb {
constexpr size_t kStaticScratchBytes = 1u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Address of `scratch` on the current device (asked for once per device), or null with *err set.
static void *static_scratch(hipError_t *err) {
    static std::mutex mu;
    static std::map<int, void *> addr;
    int dev = 0;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    auto it = addr.find(dev);
    if (it != addr.end()) return it->second;
    void *ptr = nullptr;
    *err = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || !ptr) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
    addr[dev] = ptr;
    return ptr;
}
}  // namespace csb

// Has a merge of shared row tiles given up waiting since the last check?  Synchronises `stream`.
extern "C" int csb_status(const csb_matrix *m, void *stream, int32_t *timed_out) {
    if (!m || !timed_out) { csb::set_error("csb_status: NULL pointer"); return CSB_EINVAL; }
    *timed_out = 0;
    if (!m->plan.valid || !m->uploaded || !m->d_buf) return CSB_OK;
    uint32_t *d = (uint32_t *)((uint8_t *)m->d_buf + m->plan.hdr.off_counters) + m->plan.hdr.n_shared;
    uint32_t v = 0;
    hipError_t e = hipMemcpyAsync(&v, d, 4, hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess && v) e = hipMemsetAsync(d, 0, 4, (hipStream_t)stream);
    if (e != hipSuccess) { csb::set_error(std::string("csb_status: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    *timed_out = (int32_t)v;
    return CSB_OK;
}

extern "C" size_t csb_spmv_static_limit(void) { return csb::kStaticScratchBytes; }

extern "C" int csb_spmv_static(const csb_matrix *m, const float *d_x, float *d_y, void *stream) {
    if (!m || !d_x || !d_y) { csb::set_error("csb_spmv_static: NULL pointer"); return CSB_EINVAL; }
    if (m->plan.valid && m->plan.split.active()) { csb::set_error("csb_spmv_static: matrix is planned for a GRU step"); return CSB_ESTATE; }
    if (!m->plan.valid || !m->uploaded || !m->d_buf) { csb::set_error("csb_spmv_static: matrix not planned and uploaded"); return CSB_ESTATE; }
    if (m->plan.stream.valid && !m->plan.stream.cell_gates) return csb::spmv_rows(m, d_x, d_y, stream);      // row-owned layout: no partial sums in memory at all
    const size_t need = csb_workspace_bytes(m, 1);
    if (need > csb::kStaticScratchBytes) {
        csb::set_error("csb_spmv_static: the plan's shared row tiles need " + std::to_string(need) + " bytes of partial sums, the built-in buffer holds " +
                       std::to_string(csb::kStaticScratchBytes) + "; use csb_spmv with a workspace, or plan with fewer workgroups");
        return CSB_EUNSUPPORTED;
    }
    hipError_t e = hipSuccess;
    void *ws = csb::static_scratch(&e);
    if (!ws) { csb::set_error(std::string("csb_spmv_static: hipGetSymbolAddress: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    // the merge words are told from stale ones by their launch tag; whoever used the buffer last, another
    // matrix or this one, a first use clears them (a small fill kernel on `stream`, no memset node)
    if (csb::workspace_changed_hands(ws, m)) m->ws_seen = nullptr;
    return csb::spmv_segments(m, d_x, (uint32_t)m->cols, d_x, d_y, ws, stream, nullptr);
}

namespace csb {
// Plain streaming read: the measured bandwidth the mat-vec figures are put next to.  Every
// wavefront owns a contiguous range of 1-KiB units and keeps eight 16-byte non-temporal loads
// per lane in flight (the fastest of the plain forms measured on this machine at 25 MB,
// 100 MB and 1 GiB per launch).
__global__ __launch_bounds__(1024) void stream_read_kernel(const float4 *__restrict__ p, size_t n4, float *__restrict__ out) {
    typedef float f4v __attribute__((ext_vector_type(4)));
    constexpr int K = 8;
    const size_t nw = (size_t)gridDim.x * (blockDim.x >> 6);
    const size_t w = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const size_t units = n4 >> 6;
    const size_t u0 = units / nw * w + (w < units % nw ? w : units % nw);
    const size_t u1 = u0 + units / nw + (w < units % nw ? 1 : 0);
    float s = 0.0f;
    for (size_t u = u0; u < u1; u += K) {
        f4v r[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const size_t uu = u + k < u1 ? u + k : u1 - 1;            // the tail re-reads the last unit (cached)
            r[k] = __builtin_nontemporal_load((const f4v *)(p + (uu << 6) + lane));
        }
#pragma unroll
        for (int k = 0; k < K; ++k) s += (r[k].x + r[k].y) + (r[k].z + r[k].w);
    }
    if (w == 0 && (size_t)lane < (n4 & 63)) { const float4 a = p[(units << 6) + lane]; s += (a.x + a.y) + (a.z + a.w); }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}
constexpr int kStreamReadBlocks = 256;                   // one workgroup of 16 wavefronts per CU
}  // namespace csb

extern "C" size_t csb_debug_stream_read_out_floats(void) { return (size_t)csb::kStreamReadBlocks * 1024; }

extern "C" int csb_debug_stream_read(const void *d_buf, size_t bytes, float *d_out, void *stream) {
    if (!d_buf || !d_out) { csb::set_error("csb_debug_stream_read: NULL pointer"); return CSB_EINVAL; }
    if (bytes % 16 || (uintptr_t)d_buf % 16) { csb::set_error("csb_debug_stream_read: buffer not a multiple of 16 bytes"); return CSB_EINVAL; }
    hipLaunchKernelGGL(csb::stream_read_kernel, dim3(csb::kStreamReadBlocks), dim3(1024), 0, (hipStream_t)stream,
                       (const float4 *)d_buf, bytes / 16, d_out);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { csb::set_error(std::string("csb_debug_stream_read: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

extern "C" size_t csb_debug_stamp_count(const csb_matrix *m) {
    if (m && m->plan.valid && m->plan.stream.valid && !m->plan.stream.cell_gates) return (size_t)m->plan.stream.n_wg * csb::kStreamWaves * 8;
    return (m && m->plan.valid) ? (size_t)m->plan.hdr.n_chunks * csb::kStampsPerChunk : 0;
}

extern "C" int csb_debug_spmv_stamps(const csb_matrix *m, const float *d_x, float *d_y, void *d_ws,
                                     unsigned long long *d_stamps, void *stream) {
    if (!m || !d_x || !d_y || !d_stamps) { csb::set_error("csb_debug_spmv_stamps: NULL pointer"); return CSB_EINVAL; }
    if (m->plan.valid && m->plan.split.active()) { csb::set_error("csb_debug_spmv_stamps: matrix is planned for a GRU step"); return CSB_ESTATE; }
    if (m->plan.valid && m->plan.stream.valid && !m->plan.stream.cell_gates) {
        if (!m->uploaded || !m->d_buf) { csb::set_error("csb_debug_spmv_stamps: matrix not planned and uploaded"); return CSB_ESTATE; }
        return csb::spmv_rows(m, d_x, d_y, stream, d_stamps);
    }
    if (d_ws && csb::workspace_changed_hands(d_ws, m)) m->ws_seen = nullptr;
    return csb::spmv_segments(m, d_x, (uint32_t)m->cols, d_x, d_y, d_ws, stream, d_stamps);
}
