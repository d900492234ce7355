// CSB-MVM (Sec. 4.3.1) for gfx950 from the row-owned stream section: y = A x.
//
// One workgroup (16 wavefronts) per row range.  Every load address follows from the workgroup
// and wavefront numbers alone, so nothing ever waits for a record that has to arrive first:
// the input vector and a wavefront's segments go from global memory straight into LDS (16
// bytes per lane, the segment verbatim into the wavefront's own area), a few KiB ahead of the
// multiplication, and the wavefront starts on a group as soon as the bytes of that group have
// landed.  Lane l owns one kernel-matrix row of one virtual block of the current group
// (inner-block parallelism over rows, inter-block parallelism over the lanes' different
// blocks: the two hierarchy levels of Sec. 4.3.1), walks that block's column index bytes,
// gathers the inputs from the staged vector and multiplies with its values, which it finds at
// constant offsets (a column step is a run of 64 floats, zero where a lane has nothing left).
// A lane's sum goes to its own slot of its output row in a table (the role of
// NeuronAccumBuffer); after a barrier the threads of a row add the row's slots in a fixed
// order, so results are bitwise reproducible and nothing is ever merged across workgroups.
// A wavefront's later rounds are requested while it multiplies the current one (a unit of the
// segment area is requested again as soon as the multiplication has left it); the only
// barriers are the one behind the staging of the input vector and the one in front of the row
// sums.
#include <hip/hip_runtime.h>

#include "csb_internal.hpp"
#include "csb_kernels.hpp"

namespace csb {

namespace {

__device__ __forceinline__ uint32_t uni_(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

typedef float f4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

struct RowsArgs {
    const uint8_t *img;        // header of workgroup 0
    const float *x;
    float *y;
    uint32_t n_rounds, wg_bytes, hdr_bytes, seg_bytes;
    uint32_t cols, kmax, tpr_log2, x_fast;
    uint32_t off_hdr, off_part, off_seg, bc;     // LDS map (bytes); width of a block column
    unsigned long long *stamps;                  // optional clock stamps (debug): 8 per wavefront
    uint32_t n_wg, n0;                           // workgroups of this matrix; gated form: entries of the first input segment
    GateSrc g0, g1;                              // gated form: the two segments of the input vector
};

// The arguments of up to kMaxJobsPerLaunch independent products that share a launch (blockIdx.y).
struct RowsJobs {
    RowsArgs a[kMaxJobsPerLaunch];
};

// LDS accesses by LDS byte address.
__device__ __forceinline__ float lds_f32(uint32_t a) { return *(const __attribute__((address_space(3))) float *)(uintptr_t)a; }
__device__ __forceinline__ uint32_t lds_u32(uint32_t a) { return *(const __attribute__((address_space(3))) uint32_t *)(uintptr_t)a; }
typedef uint32_t u4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 lds_u128(uint32_t a) {
    const u4v t = *(const __attribute__((address_space(3))) u4v *)(uintptr_t)a;
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint32_t lds_u16(uint32_t a) { return *(const __attribute__((address_space(3))) uint16_t *)(uintptr_t)a; }

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Global memory straight into LDS, 16 bytes per lane: lane l's bytes land at lds_base + 16 l
// (lds_base the same for the whole wavefront).  The wavefront's counter of outstanding vector
// memory operations covers these like any load, and they complete in the order issued.
__device__ __forceinline__ void dma16_stream(const uint8_t *g, uint32_t lds_base) {     // read-once data
    __builtin_amdgcn_global_load_lds((glb_void_t *)g, (lds_void_t *)(uintptr_t)lds_base, 16, 0, 2);
}
__device__ __forceinline__ void dma4(const uint8_t *g, uint32_t lds_base) {      // 4 bytes per lane: lane l's land at lds_base + 4 l
    __builtin_amdgcn_global_load_lds((glb_void_t *)g, (lds_void_t *)(uintptr_t)lds_base, 4, 0, 0);
}
__device__ __forceinline__ void dma16(const uint8_t *g, uint32_t lds_base) {
    __builtin_amdgcn_global_load_lds((glb_void_t *)g, (lds_void_t *)(uintptr_t)lds_base, 16, 0, 0);
}

// The value of another lane by a data-parallel-primitive move (CTRL: which lane; lanes the move
// has no source for read zero).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xf, 0xf, true));
}

// Waits until at most N of the wavefront's vector memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wait_outstanding() {
    static_assert(N >= 0 && N <= 8, "wait count");
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if constexpr (N == 1) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
    else if constexpr (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else if constexpr (N == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
    else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if constexpr (N == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
    else if constexpr (N == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else if constexpr (N == 7) asm volatile("s_waitcnt vmcnt(7)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
}

// W: units of round 0 a wavefront requests ahead of its multiplication.  GATED: the input vector
// is two segments, either one possibly the output of a cell whose gate sums an earlier launch
// left behind (the streaming RNN step: the cell arithmetic of step t - 1 is done while step t
// stages its input, every workgroup for itself, workgroup 0 also storing the new state).
// VF: storage format of the kernel values (CSB_VAL_*); a column step is a run of 64 values.
template <int VF>
__device__ __forceinline__ float lds_val(uint32_t a) {
    if constexpr (VF == CSB_VAL_F32) return lds_f32(a);
    else if constexpr (VF == CSB_VAL_BF16) return __uint_as_float(lds_u16(a) << 16);
    else return (float)__builtin_bit_cast(_Float16, (uint16_t)lds_u16(a));
}

// FORM: which of the run-time cases the kernel is compiled for.  These kernels run for a few
// microseconds, every launch with a cold instruction cache, and their run time follows their
// code size (measured: about 0.4 us per KiB of code on the path), so the common cases get
// kernels of their own without the code of the others.
enum : int {
    kRowsOneRound = 0,     // one round, no clock stamps
    kRowsRounds = 1,       // several rounds, no stamps
    kRowsAny = 2,          // everything decided at run time
};

// CELL: the rows are the gate rows of a recurrent cell and the plan gives a workgroup all gate
// rows of its units (StreamPlan::cell_gates): the input is two plain segments ([layer input ;
// h_(t-1)]: A.g0.a, A.g1.a), and behind the row sums the workgroup applies the cell's element-wise
// part (Sec. 2.1) to its units and stores c_t, h_t -- the whole step of a layer in this one
// launch, the gates computed once, by the workgroup that has their sums.
template <int W, bool GATED, int VF, int FORM, bool CELL = false>
__device__ __forceinline__ void rows_body(const RowsArgs &A, const uint32_t wg) {
    const bool stamps = FORM == kRowsAny && A.stamps != nullptr;
    const bool x_fast = A.x_fast != 0u;
    const uint32_t n_rounds = FORM == kRowsOneRound ? 1u : A.n_rounds;
    constexpr uint32_t VB = VF == CSB_VAL_F32 ? 4u : 2u, SS = 64u * VB;      // bytes of a value, of a column step
    extern __shared__ float4 smem4[];
    uint8_t *smem = (uint8_t *)smem4;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = uni_(tid >> 6);
    const uint8_t *wb = A.img + (size_t)wg * A.wg_bytes;
    const uint32_t seg16 = A.seg_bytes >> 4, hdr16 = A.hdr_bytes >> 4;
    uint32_t NU = (A.seg_bytes + 1023u) >> 10;                // 1 KiB units of a segment (of the current one, once its header is in)
    uint32_t own16 = seg16;                                    // its length in 16-byte pieces
    // LDS byte addresses (the staged vector sits at the start of the dynamic LDS)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const uint32_t s0 = lds0 + A.off_seg + wave * A.seg_bytes;
    unsigned long long t_start = 0, t_x = 0, t_first = 0, t_done = 0, t_bar = 0;
    if (stamps) t_start = wall_clock64();

    // ---- requests: the input vector and the header first, then the whole segment of round 0 --
    if constexpr (CELL) {                                      // two plain segments, 4 bytes per lane (their joint lies anywhere)
        const uint8_t *p0 = (const uint8_t *)A.g0.a, *p1 = (const uint8_t *)A.g1.a;
        for (uint32_t u = wave; u * 64u < A.cols; u += kStreamWaves) {
            const uint32_t e = u * 64u + lane;
            if (e < A.cols) {
                if (e < A.n0 || p1) dma4(e < A.n0 ? p0 + 4u * e : p1 + 4u * (e - A.n0), lds0 + u * 256u);
                else ((float *)smem)[e] = 0.0f;                 // no second segment in memory: a state that starts at zero
            }
        }
    } else if constexpr (GATED) {
        // (the segment's first units are requested below, before the cell arithmetic, whose loads
        // come back behind them)
    } else if (x_fast) {                                     // every wavefront's first requests: they arrive first
        const uint32_t x16 = A.cols >> 2;                      // 16-byte pieces of the vector
        for (uint32_t u = wave; u * 64u < x16; u += kStreamWaves) {
            if (u * 64u + lane < x16) dma16((const uint8_t *)A.x + (size_t)u * 1024u + lane * 16u, lds0 + u * 1024u);
        }
    } else {                                                   // a vector that is not 16-byte aligned: 4 bytes per lane
        for (uint32_t u = wave; u * 64u < A.cols; u += kStreamWaves) {
            if (u * 64u + lane < A.cols) dma4((const uint8_t *)A.x + (size_t)u * 256u + lane * 4u, lds0 + u * 256u);
        }
    }
    uint32_t req = 0;                                          // units of round 0 requested so far
    auto request_unit = [&](uint32_t round, uint32_t u, uint32_t len16) {     // len16: the segment's length in 16-byte pieces
        const uint8_t *sp = wb + A.hdr_bytes + (size_t)(round * kStreamWaves + wave) * A.seg_bytes;
        if (u * 64u + lane < len16) dma16_stream(sp + (size_t)u * 1024u + lane * 16u, s0 + u * 1024u);
    };
    // Round 0 is requested W units ahead of the multiplication instead of all at once: the memory
    // system serves a compute unit's requests in the order issued, so with short windows the
    // sixteen wavefronts receive their segments side by side and multiply while the rest arrives.
    // Requests complete in the order issued, so "unit u has landed" is "at most W - 1 requests are
    // outstanding" while W - 1 later units have been requested, and "none" otherwise.
    auto want_unit = [&](uint32_t u) {                         // unit u of round 0 is needed next: request up to u + W - 1
        const uint32_t upto = min(NU, u + (uint32_t)W);
        while (req < upto) request_unit(0u, req++, own16);
    };
    auto wait_unit = [&](uint32_t u) {                         // (after want_unit(u))
        if (u + (uint32_t)W <= NU) wait_outstanding<W - 1>(); else wait_outstanding<0>();
    };
    want_unit(0u);
    if constexpr (GATED) {
        float *xl = (float *)smem;
        const uint32_t na = min(A.n0, A.cols);
        // (two inlined copies of the staging code on purpose: the compiler then has the loads of
        // both segments in flight together, which is worth more than the 1.5 KiB of code: passing
        // one copy twice makes an LSTM step 0.2-0.5 us slower, a Li-GRU step 0.8)
        stage_segment(xl, A.g0, na, tid, kStreamThreads, wg == 0u);
        stage_segment(xl + na, A.g1, A.cols - na, tid, kStreamThreads, wg == 0u);
    } else { if (NU >= (uint32_t)W) wait_outstanding<W>(); else wait_outstanding<0>(); }   // the wavefront's part of the vector has landed
    // (a plain barrier: the fence builtins would also wait for the segment, which is still on its way)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (stamps) t_x = wall_clock64();
    if (wave == 0u)                                            // the header: needed for the row sums only
        for (uint32_t u = 0; u * 64u < hdr16; ++u)
            if (u * 64u + lane < hdr16) dma16_stream(wb + (size_t)u * 1024u + lane * 16u, lds0 + A.off_hdr + u * 1024u);

    float *part = (float *)(smem + A.off_part);
    uint32_t have = 0;                                         // units of round 0 known to have landed

    // ---- the wavefront's rounds: no barrier between them ------------------------------------
    for (uint32_t r = 0; r < n_rounds; ++r) {
        const bool more = r + 1u < n_rounds;
        if (r == 0u) {                                         // the records sit in the first unit(s)
            wait_unit(0u);
            have = 1u;
            want_unit(1u);
        } else {
            wait_outstanding<0>();                             // requested while the previous round was multiplied
            have = NU;
        }
        if (stamps && r == 0u) t_first = wall_clock64();
        // header and the first group's record in one go (both lie at the start of the first unit;
        // the record is read whether there is a group or not: one LDS round trip less in front of
        // the first group)
        const uint4 hdr = lds_u128(s0);
        uint4 rec = lds_u128(s0 + (uint32_t)sizeof(StreamSegHdr));   // record of the current group; the next one is fetched while this one runs
        const uint32_t h0 = uni_(hdr.x);
        const uint32_t ng = h0 & 0xffffu, off_vbs = h0 >> 16;
        // the segment's own length: what lies behind it (up to the stride) is never requested
        const uint32_t h1 = uni_(hdr.y);
        own16 = h1 & 0xffffu;
        NU = (own16 + 63u) >> 6;
        const uint32_t next16 = h1 >> 16, NUn = (next16 + 63u) >> 6;      // this wavefront's segment of the next round
        // units that hold records stay until the round is over; units of values are requested again
        // (for the next round) as soon as the multiplication has left them
        uint32_t meta_units = NU, released = NU;
        if (ng) {
            const uint32_t v0 = uni_(rec.w) & 0xffffu;          // val_off of group 0
            // (records may spill past the first unit: wait for them)
            const uint32_t mu = (v0 * 4u + 1023u) >> 10;
            if (r == 0u && mu > have) { want_unit(mu - 1u); wait_unit(mu - 1u); have = mu; want_unit(mu); }
            meta_units = mu; released = mu;
        }
        for (uint32_t g = 0; g < ng; ++g) {
            const uint32_t mlo = uni_(rec.x), mhi = uni_(rec.y), w2 = uni_(rec.z), w3 = uni_(rec.w);
            if (g + 1u < ng) rec = lds_u128(s0 + (uint32_t)sizeof(StreamSegHdr) + (g + 1u) * (uint32_t)sizeof(StreamGroup));
            const uint32_t vb0 = w2 & 0xffffu, lane_off = w2 >> 16, val_off = w3 & 0xffffu;
            const uint32_t cmax = ((w3 >> 16) & 0xffu) + 1u, nlanes = w3 >> 24;
            const bool act = lane < nlanes;
            // the lane's virtual block: start bits at or below the lane, minus one
            const uint32_t below = __builtin_amdgcn_mbcnt_hi(mhi, __builtin_amdgcn_mbcnt_lo(mlo, 0u));
            const uint32_t own = lane < 32u ? (mlo >> lane) & 1u : (mhi >> (lane - 32u)) & 1u;
            const uint32_t slot = act ? below + own - 1u : 0u;
            const uint32_t vbw = lds_u32(s0 + off_vbs + (vb0 + slot) * 4u);
            const uint32_t word = lds_u16(s0 + lane_off + 2u * (act ? lane : 0u));
            const uint32_t la = s0 + (vbw & 0x3ffu) * 4u;                               // its block's column list
            const uint32_t xb = lds0 + (vbw >> 18) * A.bc * 4u;                         // the block's first input
            const uint32_t vb0a = s0 + val_off * 4u + lane * VB;                        // the lane's value of step 0
            if (r == 0u) {                                      // round 0: have the group's values landed?
                const uint32_t need = (val_off * 4u + cmax * SS + 1023u) >> 10;         // units up to its last step
                if (need > have) { want_unit(need - 1u); wait_unit(need - 1u); have = need; want_unit(need); }
            }
            float a0 = 0.0f, a1 = 0.0f;
            // Eight (then four) column steps at a time, all loads issued before the first use: the
            // values at constant offsets (a step is a run of 64 floats, zero where a lane has no
            // column left), the inputs where the list bytes point.  No predicates: a zero value times
            // the input a padded list byte names (the first column of the slice, one the row uses anyway) adds nothing.
            uint32_t j = 0;
            uint32_t cw = lds_u32(la);
            for (; j + 8u <= cmax; j += 8u) {
                const uint32_t vj = vb0a + j * SS;
                const uint32_t cw2 = lds_u32(la + j + 4u);
                const float v0 = lds_val<VF>(vj), v1 = lds_val<VF>(vj + SS), v2 = lds_val<VF>(vj + 2u * SS), v3 = lds_val<VF>(vj + 3u * SS);
                const float x0 = lds_f32(xb + (cw & 0xffu) * 4u), x1 = lds_f32(xb + ((cw >> 8) & 0xffu) * 4u);
                const float x2 = lds_f32(xb + ((cw >> 16) & 0xffu) * 4u), x3 = lds_f32(xb + (cw >> 24) * 4u);
                const float v4 = lds_val<VF>(vj + 4u * SS), v5 = lds_val<VF>(vj + 5u * SS), v6 = lds_val<VF>(vj + 6u * SS), v7 = lds_val<VF>(vj + 7u * SS);
                const float x4 = lds_f32(xb + (cw2 & 0xffu) * 4u), x5 = lds_f32(xb + ((cw2 >> 8) & 0xffu) * 4u);
                const float x6 = lds_f32(xb + ((cw2 >> 16) & 0xffu) * 4u), x7 = lds_f32(xb + (cw2 >> 24) * 4u);
                cw = lds_u32(la + j + 8u);                      // the next steps' list bytes
                a0 = fmaf(v0, x0, a0); a1 = fmaf(v1, x1, a1); a0 = fmaf(v2, x2, a0); a1 = fmaf(v3, x3, a1);
                a0 = fmaf(v4, x4, a0); a1 = fmaf(v5, x5, a1); a0 = fmaf(v6, x6, a0); a1 = fmaf(v7, x7, a1);
            }
            if (j + 4u <= cmax) {
                const uint32_t vj = vb0a + j * SS;
                const float v0 = lds_val<VF>(vj), v1 = lds_val<VF>(vj + SS), v2 = lds_val<VF>(vj + 2u * SS), v3 = lds_val<VF>(vj + 3u * SS);
                const float x0 = lds_f32(xb + (cw & 0xffu) * 4u), x1 = lds_f32(xb + ((cw >> 8) & 0xffu) * 4u);
                const float x2 = lds_f32(xb + ((cw >> 16) & 0xffu) * 4u), x3 = lds_f32(xb + (cw >> 24) * 4u);
                cw = lds_u32(la + j + 4u);
                a0 = fmaf(v0, x0, a0); a1 = fmaf(v1, x1, a1); a0 = fmaf(v2, x2, a0); a1 = fmaf(v3, x3, a1);
                j += 4u;
            }
            if (j < cmax) {                                     // one to three steps left
                const uint32_t vj = vb0a + j * SS;
                a0 = fmaf(lds_val<VF>(vj), lds_f32(xb + (cw & 0xffu) * 4u), a0);
                if (j + 1u < cmax) a1 = fmaf(lds_val<VF>(vj + SS), lds_f32(xb + ((cw >> 8) & 0xffu) * 4u), a1);
                if (j + 2u < cmax) a0 = fmaf(lds_val<VF>(vj + 2u * SS), lds_f32(xb + ((cw >> 16) & 0xffu) * 4u), a0);
            }
            if (act) part[word] = a0 + a1;
            if (more) {                                         // units behind us: request them for the next round
                const uint32_t cur = (val_off * 4u + cmax * SS) >> 10;
                if (released < cur && released < NUn) {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    while (released < cur && released < NUn) request_unit(r + 1u, released++, next16);
                }
            }
        }
        if (more) {                                            // the rest of the next round: last values, then the records
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            while (released < NUn) request_unit(r + 1u, released++, next16);
            for (uint32_t u = 0; u < meta_units && u < NUn; ++u) request_unit(r + 1u, u, next16);
        }
    }
    if (stamps) t_done = wall_clock64();
    wait_outstanding<0>();                                     // (wavefront 0: the header)
    lds_barrier();
    if (stamps) t_bar = wall_clock64();

    // ---- row sums: the threads of a row add its slots in a fixed order -----------------------
    {
        const uint8_t *hl = smem + A.off_hdr;
        const uint32_t tpr = 1u << A.tpr_log2;
        const uint32_t rr = tid >> A.tpr_log2, sub = tid & (tpr - 1u);
        const uint32_t row0 = ((const uint32_t *)hl)[0], nrows = ((const uint32_t *)hl)[1];
        float s = 0.0f;
        if (rr < nrows) {
            const uint32_t oc = ((const uint32_t *)hl)[4u + rr];      // first slot, count
            const float *pr = part + (oc & 0xffffu);
            for (uint32_t k = sub; k < (oc >> 16); k += tpr) s += pr[k];
        }
        // the row's threads are neighbours: the first of them collects the sum, a fixed tree of
        // cross-lane moves (inside a 16-lane row without going through the LDS crossbar)
        if (tpr >= 2u) s += dpp_f32<0xB1>(s);                  // lanes 1,0,3,2 of every four
        if (tpr >= 4u) s += dpp_f32<0x4E>(s);                  // lanes 2,3,0,1
        if (tpr >= 8u) s += dpp_f32<0x104>(s);                 // the lane four further on (zero past the row's end)
        if (tpr >= 16u) s += dpp_f32<0x108>(s);                // eight further on
        if (tpr >= 32u) s += __shfl_down(s, 16);
        if (tpr >= 64u) s += __shfl_down(s, 32);
        if constexpr (!CELL) {
            if (sub == 0u && rr < nrows) A.y[row0 + rr] = s;
        } else {
            // local row g * nu + j holds gate g of unit row0 + j: thread j finishes unit row0 + j
            const GateSrc &c = A.g1;
            const uint32_t G = A.g0.H, H = c.H, nu = nrows / G, u = row0 + tid;
            const bool mine = tid < nu;
            // (what the cell needs from memory is asked for before the sums change hands)
            float b0 = 0.0f, b1 = 0.0f, b2 = 0.0f, b3 = 0.0f, prev = 0.0f;
            if (mine) {
                if (c.kind == kGateRbGate) {                   // what the reset launch left: z, and the n row's sum with its bias
                    b0 = c.c_in[u]; b1 = c.a2[u];
                } else if (c.bias) {
                    b0 = c.bias[u]; b1 = c.bias[H + u];
                    if (c.kind != 1u + CSB_CELL_LIGRU) b2 = c.bias[2u * H + u];
                    if (c.kind == 1u + CSB_CELL_LSTM) b3 = c.bias[3u * H + u];
                }
                const float *pv = c.kind == 1u + CSB_CELL_LSTM ? c.c_in : c.h_in;
                if (pv) prev = pv[u];                          // (null: the state starts at zero)
            }
            float *rs = (float *)smem;                         // the staged vector is done with
            if (sub == 0u && rr < nrows) rs[rr] = s;
            lds_barrier();
            if (mine && c.kind == kGateRbGate) {               // reset-before GRU, second product: its one row per unit is Un q
                const float hn = (1.0f - b0) * fast_tanh(b1 + rs[tid]) + b0 * prev;
                c.h_out[u] = hn;
                if (c.hseq) c.hseq[u] = hn;
            } else if (mine && c.kind == kGateRbReset) {       // ... first product, rows r, z, n (input side): q = r h_(t-1) for the second
                c.h_out[u] = fast_sigmoid(rs[tid] + b0) * prev;
                c.c_out[u] = fast_sigmoid(rs[nu + tid] + b1);  // z, kept for the second launch
                c.hseq[u] = rs[2u * nu + tid] + b2;            // the n row's sum with its bias, likewise
            } else if (mine) {
                const float a0 = rs[tid] + b0, a1 = rs[nu + tid] + b1;
                float hn;
                if (c.kind == 1u + CSB_CELL_LSTM) {            // rows i, f, g, o
                    const float a2 = rs[2u * nu + tid] + b2, a3 = rs[3u * nu + tid] + b3;
                    const float cn = fast_sigmoid(a1) * prev + fast_sigmoid(a0) * fast_tanh(a2);
                    hn = fast_sigmoid(a3) * fast_tanh(cn);
                    c.c_out[u] = cn;
                } else if (c.kind == 1u + CSB_CELL_GRU) {      // rows r, z, input side of n, recurrent side of n
                    const float a2 = rs[2u * nu + tid] + b2, a3 = rs[3u * nu + tid];
                    const float r = fast_sigmoid(a0), z = fast_sigmoid(a1);
                    hn = (1.0f - z) * fast_tanh(a2 + r * a3) + z * prev;
                } else {                                       // Li-GRU: rows z, candidate
                    const float z = fast_sigmoid(a0);
                    hn = z * prev + (1.0f - z) * fmaxf(a1, 0.0f);
                }
                c.h_out[u] = hn;
                if (c.hseq) c.hseq[u] = hn;
            }
        }
    }
    if (stamps && lane == 0u) {
        unsigned long long *st = A.stamps + ((size_t)wg * kStreamWaves + wave) * 8;
        st[0] = t_start; st[1] = t_x; st[2] = t_first; st[3] = t_first; st[4] = t_done; st[5] = t_bar; st[6] = wall_clock64();
    }
}

template <int W, int VF, int FORM>
__global__ __launch_bounds__(kStreamThreads) void spmv_rows_kernel(const RowsArgs A) {
    rows_body<W, false, VF, FORM>(A, blockIdx.x);
}

template <int W, int VF, int FORM>
__global__ __launch_bounds__(kStreamThreads) void spmv_rows_gated_kernel(const RowsArgs A) {
    rows_body<W, true, VF, FORM>(A, blockIdx.x);
}

// blockIdx.y selects the product; the grid is as wide as the largest of them.
template <int W, int VF, int FORM>
__global__ __launch_bounds__(kStreamThreads) void spmv_rows_gated_multi_kernel(const RowsJobs J) {
    const RowsArgs &A = J.a[blockIdx.y];
    if (blockIdx.x >= A.n_wg) return;
    rows_body<W, true, VF, FORM>(A, blockIdx.x);
}

// Independent plain products in one launch (blockIdx.y).
template <int W, int VF, int FORM>
__global__ __launch_bounds__(kStreamThreads) void spmv_rows_multi_kernel(const RowsJobs J) {
    const RowsArgs &A = J.a[blockIdx.y];
    if (blockIdx.x >= A.n_wg) return;
    rows_body<W, false, VF, FORM>(A, blockIdx.x);
}

// The step of one recurrent layer whose plan gives its workgroups whole units (a launch of its own
// for a single layer: the host then hands over one product's arguments instead of four).
template <int W, int VF, int FORM>
__global__ __launch_bounds__(kStreamThreads) void spmv_rows_cell_kernel(const RowsArgs A) {
    rows_body<W, false, VF, FORM, true>(A, blockIdx.x);
}

// ... of up to kMaxJobsPerLaunch layers (blockIdx.y: the layer).
template <int W, int VF, int FORM>
__global__ __launch_bounds__(kStreamThreads) void spmv_rows_cell_multi_kernel(const RowsJobs J) {
    const RowsArgs &A = J.a[blockIdx.y];
    if (blockIdx.x >= A.n_wg) return;
    rows_body<W, false, VF, FORM, true>(A, blockIdx.x);
}

// Kernel arguments of one product and the dynamic LDS it needs (0 with the error set if it does not fit).
size_t rows_args(const csb_matrix *m, RowsArgs *out) {
    const StreamPlan &sp = m->plan.stream;
    RowsArgs A{};
    A.img = (const uint8_t *)m->d_buf + sp.off;
    A.n_rounds = sp.n_rounds; A.wg_bytes = sp.wg_bytes; A.hdr_bytes = sp.hdr_bytes; A.seg_bytes = sp.seg_bytes;
    A.cols = (uint32_t)m->cols; A.kmax = sp.kmax; A.bc = (uint32_t)m->bc;
    A.tpr_log2 = (uint32_t)__builtin_ctz(sp.tpr);
    A.n_wg = sp.n_wg;
    uint32_t x_bytes = (uint32_t)(((size_t)m->cols * 4 + 15) / 16 * 16);
    if (sp.cell_gates) x_bytes = std::max<uint32_t>(x_bytes, 4u * (uint32_t)kStreamMaxRows);   // (the cell form keeps its row sums there)
    const uint32_t part_bytes = (uint32_t)(((size_t)sp.kmax * 4 + 15) / 16 * 16);
    A.off_hdr = x_bytes;
    A.off_part = A.off_hdr + sp.hdr_bytes;
    A.off_seg = A.off_part + part_bytes;
    // 1 KiB of slack behind the last segment: lanes that are done keep reading a little further
    const size_t lds = (size_t)A.off_seg + (size_t)kStreamWaves * sp.seg_bytes + 1024;
    if (lds > (size_t)160 * 1024) { set_error("csb_spmv: row-owned layout does not fit the LDS"); return 0; }
    *out = A;
    return lds;
}

template <typename Kern, typename Arg>
int launch_rows(Kern kern, dim3 grid, size_t lds, void *stream, const Arg &arg) {
    hipError_t e = ensure_dynamic_lds((const void *)kern, lds);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(kern, grid, dim3(kStreamThreads), lds, (hipStream_t)stream, arg);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { set_error(std::string("csb_spmv: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

}  // namespace

// Launch of KERN<2, format, form>: two units ahead -- measured best on the 8192 x 8192 stress matrix
// (cold, us: 8.1 with two, 8.6 with three, 9.0 with four, 10.0 with six units ahead after the first):
// what a wavefront asks for far ahead delays what its neighbours need next.
#define CSB_ROWS_LAUNCH(KERN, vf, form, grid, lds, stream, arg)                                                  \
    ((vf) == CSB_VAL_F16    ? launch_rows(KERN<2, CSB_VAL_F16, form>, grid, lds, stream, arg)                    \
     : (vf) == CSB_VAL_BF16 ? launch_rows(KERN<2, CSB_VAL_BF16, form>, grid, lds, stream, arg)                   \
                            : launch_rows(KERN<2, CSB_VAL_F32, form>, grid, lds, stream, arg))

int spmv_rows(const csb_matrix *m, const float *d_x, float *d_y, void *stream, unsigned long long *d_stamps) {
    RowsArgs A;
    const size_t lds = rows_args(m, &A);
    if (!lds) return CSB_EUNSUPPORTED;
    A.x = d_x; A.y = d_y; A.stamps = d_stamps;
    A.x_fast = ((uintptr_t)d_x % 16 == 0 && m->cols % 4 == 0) ? 1u : 0u;
    const uint32_t vf = m->plan.stream.val_fmt;
    if (d_stamps) return CSB_ROWS_LAUNCH(spmv_rows_kernel, vf, kRowsAny, dim3(A.n_wg), lds, stream, A);
    if (A.n_rounds == 1u) return CSB_ROWS_LAUNCH(spmv_rows_kernel, vf, kRowsOneRound, dim3(A.n_wg), lds, stream, A);
    return CSB_ROWS_LAUNCH(spmv_rows_kernel, vf, kRowsRounds, dim3(A.n_wg), lds, stream, A);
}

int spmv_rows_gated(const csb_matrix *m, const GateSrc &s0, uint32_t n0, const GateSrc &s1, float *d_y, void *stream) {
    RowsArgs A;
    const size_t lds = rows_args(m, &A);
    if (!lds) return CSB_EUNSUPPORTED;
    A.y = d_y; A.g0 = s0; A.g1 = s1; A.n0 = n0;
    const uint32_t vf = m->plan.stream.val_fmt;
    if (A.n_rounds == 1u) return CSB_ROWS_LAUNCH(spmv_rows_gated_kernel, vf, kRowsOneRound, dim3(A.n_wg), lds, stream, A);
    return CSB_ROWS_LAUNCH(spmv_rows_gated_kernel, vf, kRowsRounds, dim3(A.n_wg), lds, stream, A);
}

int spmv_rows_gated_multi(const SpmvGatedCall *calls, int n, void *stream) {
    RowsJobs J{};
    size_t lds = 0;
    uint32_t wgs = 0, rounds = 1;
    for (int i = 0; i < n; ++i) {
        const size_t l = rows_args(calls[i].mat, &J.a[i]);
        if (!l) return CSB_EUNSUPPORTED;
        J.a[i].y = calls[i].y; J.a[i].g0 = calls[i].s0; J.a[i].g1 = calls[i].s1; J.a[i].n0 = calls[i].n0;
        lds = std::max(lds, l);
        wgs = std::max(wgs, J.a[i].n_wg);
        rounds = std::max(rounds, J.a[i].n_rounds);
    }
    const uint32_t vf = calls[0].mat->plan.stream.val_fmt;             // (the caller has checked: one format for all)
    const dim3 grid(wgs, (unsigned)n);
    if (rounds == 1u) return CSB_ROWS_LAUNCH(spmv_rows_gated_multi_kernel, vf, kRowsOneRound, grid, lds, stream, J);
    return CSB_ROWS_LAUNCH(spmv_rows_gated_multi_kernel, vf, kRowsRounds, grid, lds, stream, J);
}

int spmv_rows_multi(const SpmvPlainCall *calls, int n, void *stream) {
    RowsJobs J{};
    size_t lds = 0;
    uint32_t wgs = 0, rounds = 1;
    if (n < 1 || n > kMaxJobsPerLaunch) { set_error("csb_spmv: between one and four products share a launch"); return CSB_EINVAL; }
    for (int i = 0; i < n; ++i) {
        const csb_matrix *m = calls[i].mat;
        if (!m->plan.valid || !m->uploaded || !m->plan.stream.valid || m->plan.stream.cell_gates ||
            m->plan.stream.val_fmt != calls[0].mat->plan.stream.val_fmt) {
            set_error("csb_spmv: matrix is not in the plain row-owned layout");
            return CSB_ESTATE;
        }
        const size_t l = rows_args(m, &J.a[i]);
        if (!l) return CSB_EUNSUPPORTED;
        J.a[i].x = calls[i].x; J.a[i].y = calls[i].y;
        J.a[i].x_fast = ((uintptr_t)calls[i].x % 16 == 0 && m->cols % 4 == 0) ? 1u : 0u;
        lds = std::max(lds, l);
        wgs = std::max(wgs, J.a[i].n_wg);
        rounds = std::max(rounds, J.a[i].n_rounds);
    }
    const uint32_t vf = calls[0].mat->plan.stream.val_fmt;
    if (n == 1) {
        if (rounds == 1u) return CSB_ROWS_LAUNCH(spmv_rows_kernel, vf, kRowsOneRound, dim3(wgs), lds, stream, J.a[0]);
        return CSB_ROWS_LAUNCH(spmv_rows_kernel, vf, kRowsRounds, dim3(wgs), lds, stream, J.a[0]);
    }
    const dim3 grid(wgs, (unsigned)n);
    if (rounds == 1u) return CSB_ROWS_LAUNCH(spmv_rows_multi_kernel, vf, kRowsOneRound, grid, lds, stream, J);
    return CSB_ROWS_LAUNCH(spmv_rows_multi_kernel, vf, kRowsRounds, grid, lds, stream, J);
}

int spmv_rows_cell_multi(const SpmvCellCall *calls, int n, void *stream) {
    RowsJobs J{};
    size_t lds = 0;
    uint32_t wgs = 0, rounds = 1;
    if (n < 1 || n > kMaxJobsPerLaunch) { set_error("csb_spmv: between one and four products share a launch"); return CSB_EINVAL; }
    for (int i = 0; i < n; ++i) {
        const SpmvCellCall &c = calls[i];
        const StreamPlan &sp = c.mat->plan.stream;
        const uint32_t kind = c.cell == kCellRbReset ? kGateRbReset : c.cell == kCellRbGate ? kGateRbGate : 1u + (uint32_t)c.cell;
        const uint32_t G = kind == kGateRbGate ? 1u : kind == kGateRbReset ? 3u : c.cell == CSB_CELL_LIGRU ? 2u : 4u;
        const bool own_state = c.cell == CSB_CELL_GRU || c.cell == CSB_CELL_LIGRU || kind == kGateRbReset;   // the second segment is h_(t-1), H wide
        if (!c.mat->plan.valid || !c.mat->uploaded || !sp.valid || sp.cell_gates != G || sp.val_fmt != calls[0].mat->plan.stream.val_fmt ||
            (uint64_t)c.n0 > (uint64_t)c.mat->cols || (own_state && (uint64_t)c.n0 + sp.cell_units != (uint64_t)c.mat->cols)) {
            set_error("csb_spmv: matrix is not laid out for a cell of this kind");
            return CSB_ESTATE;
        }
        const size_t l = rows_args(c.mat, &J.a[i]);
        if (!l) return CSB_EUNSUPPORTED;
        RowsArgs &A = J.a[i];
        A.n0 = c.n0;
        A.g0 = plain_src(c.x0); A.g0.H = G;
        A.g1 = plain_src(c.h_prev);
        A.g1.H = sp.cell_units; A.g1.kind = kind; A.g1.bias = c.bias;
        A.g1.c_in = c.c_in; A.g1.h_in = c.h_state ? c.h_state : c.h_prev; A.g1.c_out = c.c_out; A.g1.h_out = c.h_out; A.g1.hseq = c.hseq;
        A.g1.a2 = c.aux;
        lds = std::max(lds, l);
        wgs = std::max(wgs, A.n_wg);
        rounds = std::max(rounds, A.n_rounds);
    }
    const uint32_t vf = calls[0].mat->plan.stream.val_fmt;
    if (n == 1) {
        if (rounds == 1u) return CSB_ROWS_LAUNCH(spmv_rows_cell_kernel, vf, kRowsOneRound, dim3(wgs), lds, stream, J.a[0]);
        return CSB_ROWS_LAUNCH(spmv_rows_cell_kernel, vf, kRowsRounds, dim3(wgs), lds, stream, J.a[0]);
    }
    const dim3 grid(wgs, (unsigned)n);
    if (rounds == 1u) return CSB_ROWS_LAUNCH(spmv_rows_cell_multi_kernel, vf, kRowsOneRound, grid, lds, stream, J);
    return CSB_ROWS_LAUNCH(spmv_rows_cell_multi_kernel, vf, kRowsRounds, grid, lds, stream, J);
}

#undef CSB_ROWS_LAUNCH

}  // namespace csb
