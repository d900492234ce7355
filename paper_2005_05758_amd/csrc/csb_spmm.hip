// Batched CSB-MVM for gfx950: Y = A X with fp32 MFMA.
//
// With B right-hand sides a kernel matrix K_b (r x c) meets a gathered c x B slab of X: a
// real dense product, so it goes to the matrix cores (v_mfma_f32_16x16x4_f32).  One
// workgroup owns one output row tile and one batch tile.  The tile's records (groups,
// virtual blocks, lane descriptors, input-offset lists) are staged in LDS one segment at a
// time; the wavefronts take the segment's virtual blocks round-robin, each as 16-row
// slices: per 4 columns one A operand (16 x 4 of the kernel) feeds one MFMA per 16 batch
// columns.  The operands of the next pass are loaded while the current one multiplies.
// The 16 x 16 results are added at the block's row indices into a per-wavefront
// accumulator tile in LDS (the role of NeuronAccumBuffer, Sec. 4.3.1); the wavefronts'
// tiles are summed in wavefront order, so the result does not depend on timing.  The
// paper's engine is batch 1 only; this is the batched extension the matrix cores make
// worthwhile.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "csb_internal.hpp"
#include "csb_kernels.hpp"

namespace csb {

typedef float floatx4 __attribute__((ext_vector_type(4)));


__device__ __forceinline__ uint32_t uni_(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Element (column j of A, right-hand side n) of the input, from one of two sources.  Element
// offsets fit 32 bits and the strides over j fit 24 bits (checked on the host).
struct XSrc {
    const float *p0;
    uint32_t n0;          // columns j < n0 come from p0, the rest from p1
    uint32_t sj0, sn0;    // strides over j and over n
    const float *p1;
    uint32_t sj1, sn1;
};

// One pass: 4 KS columns (KS MFMA k-steps; 8, or 4 in the wide form, whose operands take
// four times the registers per k-step) of one 16-row slice of one virtual block.
struct Pass {
    uint32_t k;           // virtual block, counted inside the segment
    uint32_t m0, kc;      // first row of the slice, first column of the pass
    uint32_t r, c, lane0; // the block's rows, columns, first lane
    uint32_t val_off;     // the group's values
    uint32_t desc;        // LDS byte offset of the group's lane descriptors
    uint32_t list;        // LDS byte offset of the block's input-offset list
    bool valid;
};

template <int NT, int KS>
struct Operands {
    float av[KS];
    float bv[KS][NT];
};

// WIDE (NT = 4, right-hand sides contiguous in memory, batch a multiple of 4): a lane reads
// four neighbouring right-hand sides of its input row with one 16-byte load and feeds one
// of them to each of four MFMA tiles, so tile t holds the right-hand sides 4 n + t; a
// lane's four results of one row are then neighbours again and go to the accumulator as one
// 16-byte word.  A quarter of the load and LDS instructions per multiply.
template <int NT, bool TWO, int NW, bool WIDE>
__device__ __forceinline__ void spmm_body(const DevMat &m, const XSrc &X, float *__restrict__ Y, const int64_t ldy,
                                          const uint32_t batch, const uint32_t block_x, const uint32_t block_y) {
    extern __shared__ float4 smem4[];
    constexpr int NB = 16 * NT;                    // batch columns per workgroup
    constexpr int KS = WIDE ? 4 : 8;               // k-steps per pass
    constexpr uint32_t NTHR = NW * 64;             // NW wavefronts
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = uni_(tid >> 6);
    const uint32_t bt0 = block_y * NB;
    const uint32_t br = m.br;
    if (block_x >= m.n_nz_tiles) {                 // a row tile without work: zeros
        const uint32_t tile = m.zero_tiles[block_x - m.n_nz_tiles];
        for (uint32_t e = tid; e < br * NB; e += NTHR) {
            const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
            if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = 0.0f;
        }
        return;
    }
    uint8_t *meta = (uint8_t *)smem4;                              // one record segment
    float *acc = (float *)(meta + m.seg_meta);                     // [waves][br][NB]
    float *myacc = acc + (size_t)wave * br * NB;
    for (uint32_t e = lane; e < br * NB; e += 64) myacc[e] = 0.0f;
    const uint32_t rank = block_x, tile = m.nz_tiles[rank];
    const uint32_t vf = uni_(m.val_fmt);                           // storage format of the value stream
    const uint32_t mrow = lane & 15u, kq = lane >> 4;              // A: row, column-in-4; B: column n, row-in-4
    static_assert(!WIDE || NT == 4, "the wide form feeds four tiles from one load");
    const uint32_t ncol = bt0 + (WIDE ? 4u * mrow : mrow);         // this lane's right-hand side (per 16: + 16 nt)
    uint32_t noff0[NT], noff1[NT];                                 // its byte offset in either source
    bool n_ok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const uint32_t n = WIDE ? ncol + (uint32_t)nt : ncol + 16u * nt;
        n_ok[nt] = n < batch;
        noff0[nt] = (n_ok[nt] ? n : 0u) * X.sn0 * 4u;              // bytes
        noff1[nt] = (n_ok[nt] ? n : 0u) * X.sn1 * 4u;
    }

    for (uint32_t sg = m.tile_seg0[rank]; sg < m.tile_seg0[rank + 1]; ++sg) {
        // ---- stage the segment's records ------------------------------------------------
        const SegRec *sp = m.segs + sg;
        const uint32_t ga = sp->g0, ng = sp->ng, vb0 = sp->vb0, nvbs = sp->nvbs, idx0 = sp->idx0, idx_bytes = sp->idx_bytes;
        const uint32_t voff = (ng * (uint32_t)sizeof(GroupRec) + 15u) & ~15u;
        const uint32_t ioff = voff + ((nvbs * (uint32_t)sizeof(VbRec) + 15u) & ~15u);
        __syncthreads();                                           // the previous segment is done with
        {
            const uint2 *gs = (const uint2 *)(m.groups + ga);
            uint2 *gd = (uint2 *)meta;
            for (uint32_t i = tid; i < ng * 3u; i += NTHR) gd[i] = gs[i];
            const float4 *vs = (const float4 *)(m.vbs + vb0);
            float4 *vd = (float4 *)(meta + voff);
            for (uint32_t i = tid; i < nvbs; i += NTHR) vd[i] = vs[i];
            const float4 *is = (const float4 *)(m.idx + idx0);
            float4 *id = (float4 *)(meta + ioff);
            for (uint32_t i = tid; i < idx_bytes >> 4; i += NTHR) id[i] = is[i];
        }
        __syncthreads();

        // ---- passes of this wavefront's virtual blocks ----------------------------------
        auto open_vb = [&](uint32_t k) -> Pass {
            Pass p{};
            p.k = k;
            p.valid = k < nvbs;
            if (!p.valid) return p;
            const uint4 v = *(const uint4 *)(meta + voff + k * (uint32_t)sizeof(VbRec));
            const uint32_t v0 = uni_(v.x);
            p.r = v0 & 0xffu; p.lane0 = (v0 >> 8) & 0xffu; p.c = v0 >> 16;
            p.val_off = uni_(v.y);
            p.desc = ioff + (uni_(v.z) - idx0);
            p.list = ioff + (uni_(v.w) - idx0);
            p.m0 = 0; p.kc = 0;
            return p;
        };
        auto next_pass = [&](const Pass &p) -> Pass {
            Pass q = p;
            q.kc += 4 * KS;
            if (q.kc < q.c) return q;
            q.kc = 0; q.m0 += 16;
            if (q.m0 < q.r) return q;
            return open_vb(p.k + NW);
        };
        // All loads of a pass are independent: kernel values and gathered inputs of up to 8
        // k-steps.  Out-of-range lanes load from clamped addresses; their operands are zeroed.
        auto load_pass = [&](const Pass &p, Operands<NT, KS> &o) {
            const float *gv = m.vals + p.val_off;
            const uint32_t *gv16 = (const uint32_t *)m.vals + (p.val_off >> 1);
            const uint16_t *colp = (const uint16_t *)(meta + p.list);
            const bool row_ok = p.m0 + mrow < p.r;
            const uint32_t arow = p.lane0 + p.m0 + (row_ok ? mrow : 0u);
#pragma unroll
            for (int s8 = 0; s8 < KS; ++s8) {
                if (p.kc + 4u * s8 >= p.c) break;                  // uniform: k-steps the block does not have
                const uint32_t jj = p.kc + 4u * s8 + kq;
                const bool ok = jj < p.c;
                const uint32_t jc = ok ? jj : 0u;
                float t;
                if (vf == CSB_VAL_F32) {                           // uniform
                    t = gv[jc * (uint32_t)kWave + arow];
                } else {                                           // one word per lane and pair of steps
                    const uint32_t w = gv16[(jc >> 1) * (uint32_t)kWave + arow];
                    const uint32_t bits = (jc & 1u) ? w >> 16 : w & 0xffffu;
                    t = vf == CSB_VAL_BF16 ? __uint_as_float(bits << 16) : (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
                }
                o.av[s8] = ok && row_ok ? t : 0.0f;
                // The input operand is not zeroed where the kernel operand is: a lane without a
                // column reads the block's first column (finite wherever the block's own rows
                // would be), one past the batch reads right-hand side 0, and its result column
                // is never stored.
                const uint32_t cb = colp[jc];                      // 4 * column: the list holds byte offsets
                const bool first = !TWO || cb < 4u * X.n0;
                const uint8_t *src = (const uint8_t *)(first ? X.p0 : X.p1);
                const uint32_t joff = first ? __umul24(cb, X.sj0) : __umul24(cb - 4u * X.n0, X.sj1);   // bytes
                if constexpr (WIDE) {                              // batch % 4 == 0: the four are in or out together
                    const float4 x4 = *(const float4 *)(src + joff + (first ? noff0[0] : noff1[0]));
                    o.bv[s8][0] = x4.x; o.bv[s8][1] = x4.y; o.bv[s8][2] = x4.z; o.bv[s8][3] = x4.w;
                } else {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        o.bv[s8][nt] = *(const float *)(src + joff + (first ? noff0[nt] : noff1[nt]));
                }
            }
        };
        floatx4 D[NT];
        const floatx4 zero4 = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) D[nt] = zero4;
        auto mult_pass = [&](const Pass &p, const Operands<NT, KS> &o) {
#pragma unroll
            for (int s8 = 0; s8 < KS; ++s8) {
                if (p.kc + 4u * s8 >= p.c) break;                  // uniform
                // a slice's first k-step starts from a zero operand: the accumulators need no clearing
                if (s8 == 0 && p.kc == 0) {                        // uniform
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        D[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(o.av[s8], o.bv[s8][nt], zero4, 0, 0, 0);
                } else {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        D[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(o.av[s8], o.bv[s8][nt], D[nt], 0, 0, 0);
                }
            }
            if (p.kc + 4 * KS < p.c) return;                       // the slice has more columns
            // lane holds rows 4*(lane/16)+i, column lane%16 of each 16 x 16 result; the rows of
            // a slice are distinct, so no two lanes meet in the accumulator: all reads, then
            // all writes
            uint32_t at[4];
            bool on[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t mr = p.m0 + 4u * kq + i;
                on[i] = mr < p.r;
                const uint32_t slot = meta[p.desc + 4u * (p.lane0 + (on[i] ? mr : 0u))];
                at[i] = slot * NB + (WIDE ? 4u * mrow : mrow);
            }
            if constexpr (WIDE) {
                float4 old4[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) old4[i] = *(const float4 *)(myacc + at[i]);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (on[i])
                        *(float4 *)(myacc + at[i]) = make_float4(old4[i].x + D[0][i], old4[i].y + D[1][i],
                                                                 old4[i].z + D[2][i], old4[i].w + D[3][i]);
                return;
            }
            float old[4][NT];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) old[i][nt] = myacc[at[i] + 16u * nt];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    if (on[i]) myacc[at[i] + 16u * nt] = old[i][nt] + D[nt][i];
        };
        auto nxt = [&](const Pass &p) -> Pass { return p.valid ? next_pass(p) : p; };
        if constexpr (WIDE) {
            // three passes in flight (their operands are small: 4 k-steps)
            Operands<NT, KS> oa, ob, oc;
            Pass pa = open_vb(wave), pb = nxt(pa), pc{};
            if (pa.valid) load_pass(pa, oa);
            if (pb.valid) load_pass(pb, ob);
            while (true) {
                pc = nxt(pb); if (pc.valid) load_pass(pc, oc);
                if (!pa.valid) break;
                mult_pass(pa, oa);
                pa = nxt(pc); if (pa.valid) load_pass(pa, oa);
                if (!pb.valid) break;
                mult_pass(pb, ob);
                pb = nxt(pa); if (pb.valid) load_pass(pb, ob);
                if (!pc.valid) break;
                mult_pass(pc, oc);
            }
        } else {
            Operands<NT, KS> oa, ob;
            Pass pa = open_vb(wave), pb{};
            if (pa.valid) load_pass(pa, oa);
            while (pa.valid) {
                pb = next_pass(pa);
                if (pb.valid) load_pass(pb, ob);
                mult_pass(pa, oa);
                if (!pb.valid) break;
                pa = next_pass(pb);
                if (pa.valid) load_pass(pa, oa);
                mult_pass(pb, ob);
            }
        }
    }
    __syncthreads();
    for (uint32_t e = tid; e < br * NB; e += NTHR) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += acc[(size_t)w * br * NB + e];
        const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
        if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = s;
    }
}

template <int NT, bool TWO, int NW, bool WIDE>
__global__ __launch_bounds__(NW * 64) void spmm_kernel(const DevMat m, const XSrc X, float *__restrict__ Y,
                                                             const int64_t ldy, const uint32_t batch) {
    spmm_body<NT, TWO, NW, WIDE>(m, X, Y, ldy, batch, blockIdx.x, blockIdx.y);
}

// ---------------------------------------------------------------------------------------
// bfloat16 operands (v_mfma_f32_16x16x16_bf16): the kernel values are stored as bfloat16
// (csb_set_value_format) and the right-hand sides arrive as bfloat16, [cols][ldx] with the
// batch contiguous; products are exact in binary32 and are accumulated in binary32.  One
// MFMA takes 16 columns of a block (four times the f32 instruction's) and the gather of X --
// what bounds the f32 kernel -- moves half the bytes.  Same tiling as the wide f32 form: a
// lane loads four neighbouring right-hand sides of an input row at once (8 bytes), tile t
// holds the right-hand sides 4 n + t.
// The same kernel serves binary16 (HALF: v_mfma_f32_16x16x16_f16, values and right-hand sides
// as binary16, whose products are exact in binary32 as well).
typedef short bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
template <bool HALF>
__device__ __forceinline__ floatx4 mfma_16bit(const uint2 a, const uint2 b, const floatx4 c) {
    if constexpr (HALF) return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4, a), __builtin_bit_cast(bf16x4, b), c, 0, 0, 0);
}

template <int KS>
struct OperandsBf {
    uint2 a[KS];          // four consecutive columns of this lane's row
    uint2 b[KS][4];       // per tile: the same four columns of its right-hand side
};

template <int NW, bool HALF>
__global__ __launch_bounds__(NW * 64) void spmm_bf16_kernel(const DevMat m, const uint16_t *__restrict__ Xb, const uint32_t ldx,
                                                           float *__restrict__ Y, const int64_t ldy, const uint32_t batch) {
    extern __shared__ float4 smem4[];
    constexpr int NT = 4, NB = 64, KS = 2;         // 64 batch columns per workgroup, 32 block columns per pass
    constexpr uint32_t NTHR = NW * 64;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = uni_(tid >> 6);
    const uint32_t bt0 = blockIdx.y * NB;
    const uint32_t br = m.br;
    if (blockIdx.x >= m.n_nz_tiles) {              // a row tile without work: zeros
        const uint32_t tile = m.zero_tiles[blockIdx.x - m.n_nz_tiles];
        for (uint32_t e = tid; e < br * NB; e += NTHR) {
            const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
            if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = 0.0f;
        }
        return;
    }
    uint8_t *meta = (uint8_t *)smem4;
    float *acc = (float *)(meta + m.seg_meta);     // [waves][br][NB]
    float *myacc = acc + (size_t)wave * br * NB;
    for (uint32_t e = lane; e < br * NB; e += 64) myacc[e] = 0.0f;
    const uint32_t rank = blockIdx.x, tile = m.nz_tiles[rank];
    const uint32_t mrow = lane & 15u, kq = lane >> 4;
    const uint32_t ncol = bt0 + 4u * mrow;         // first of this lane's four right-hand sides (batch % 4 == 0)
    const uint32_t noff = (ncol < batch ? ncol : 0u) * 2u;   // bytes; one past the batch reads 0..3, never stored

    for (uint32_t sg = m.tile_seg0[rank]; sg < m.tile_seg0[rank + 1]; ++sg) {
        const SegRec *sp = m.segs + sg;
        const uint32_t ga = sp->g0, ng = sp->ng, vb0 = sp->vb0, nvbs = sp->nvbs, idx0 = sp->idx0, idx_bytes = sp->idx_bytes;
        const uint32_t voff = (ng * (uint32_t)sizeof(GroupRec) + 15u) & ~15u;
        const uint32_t ioff = voff + ((nvbs * (uint32_t)sizeof(VbRec) + 15u) & ~15u);
        __syncthreads();
        {
            const uint2 *gs = (const uint2 *)(m.groups + ga);
            uint2 *gd = (uint2 *)meta;
            for (uint32_t i = tid; i < ng * 3u; i += NTHR) gd[i] = gs[i];
            const float4 *vs = (const float4 *)(m.vbs + vb0);
            float4 *vd = (float4 *)(meta + voff);
            for (uint32_t i = tid; i < nvbs; i += NTHR) vd[i] = vs[i];
            const float4 *is = (const float4 *)(m.idx + idx0);
            float4 *id = (float4 *)(meta + ioff);
            for (uint32_t i = tid; i < idx_bytes >> 4; i += NTHR) id[i] = is[i];
        }
        __syncthreads();

        auto open_vb = [&](uint32_t k) -> Pass {
            Pass p{};
            p.k = k;
            p.valid = k < nvbs;
            if (!p.valid) return p;
            const uint4 v = *(const uint4 *)(meta + voff + k * (uint32_t)sizeof(VbRec));
            const uint32_t v0 = uni_(v.x);
            p.r = v0 & 0xffu; p.lane0 = (v0 >> 8) & 0xffu; p.c = v0 >> 16;
            p.val_off = uni_(v.y);
            p.desc = ioff + (uni_(v.z) - idx0);
            p.list = ioff + (uni_(v.w) - idx0);
            p.m0 = 0; p.kc = 0;
            return p;
        };
        auto next_pass = [&](const Pass &p) -> Pass {
            Pass q = p;
            q.kc += 16 * KS;
            if (q.kc < q.c) return q;
            q.kc = 0; q.m0 += 16;
            if (q.m0 < q.r) return q;
            return open_vb(p.k + NW);
        };
        auto load_pass = [&](const Pass &p, OperandsBf<KS> &o) {
            // one word per lane and pair of columns, the even column in the low half; a block
            // with an odd number of columns has a zero in its last word's high half
            const uint32_t *gv16 = (const uint32_t *)m.vals + (p.val_off >> 1);
            const uint16_t *colp = (const uint16_t *)(meta + p.list);
            const bool row_ok = p.m0 + mrow < p.r;
            const uint32_t arow = p.lane0 + p.m0 + (row_ok ? mrow : 0u);
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                if (p.kc + 16u * s >= p.c) break;                  // uniform: columns the block does not have
                const uint32_t j0 = p.kc + 16u * s + 4u * kq;      // this lane's four columns
                const bool ok0 = j0 < p.c, ok1 = j0 + 2u < p.c;
                const uint32_t w0 = gv16[((ok0 ? j0 : 0u) >> 1) * (uint32_t)kWave + arow];
                const uint32_t w1 = gv16[((ok1 ? j0 + 2u : 0u) >> 1) * (uint32_t)kWave + arow];
                o.a[s] = make_uint2(ok0 && row_ok ? w0 : 0u, ok1 && row_ok ? w1 : 0u);
                // (a lane without a column reads the block's first one: finite, times a zero)
                uint2 x[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t jj = j0 + (uint32_t)i;
                    const uint32_t cb = colp[jj < p.c ? jj : 0u];  // 4 * column
                    x[i] = *(const uint2 *)((const uint8_t *)Xb + (__umul24(cb, ldx) >> 1) + noff);
                }
                // x[i] = right-hand sides 0..3 at column i; tile t wants columns 0..3 at right-hand side t
                o.b[s][0] = make_uint2((x[0].x & 0xffffu) | (x[1].x << 16), (x[2].x & 0xffffu) | (x[3].x << 16));
                o.b[s][1] = make_uint2((x[0].x >> 16) | (x[1].x & 0xffff0000u), (x[2].x >> 16) | (x[3].x & 0xffff0000u));
                o.b[s][2] = make_uint2((x[0].y & 0xffffu) | (x[1].y << 16), (x[2].y & 0xffffu) | (x[3].y << 16));
                o.b[s][3] = make_uint2((x[0].y >> 16) | (x[1].y & 0xffff0000u), (x[2].y >> 16) | (x[3].y & 0xffff0000u));
            }
        };
        floatx4 D[NT];
        const floatx4 zero4 = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) D[nt] = zero4;
        auto mult_pass = [&](const Pass &p, const OperandsBf<KS> &o) {
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                if (p.kc + 16u * s >= p.c) break;                  // uniform
                if (s == 0 && p.kc == 0) {                         // uniform: a slice starts from a zero operand
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) D[nt] = mfma_16bit<HALF>(o.a[s], o.b[s][nt], zero4);
                } else {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) D[nt] = mfma_16bit<HALF>(o.a[s], o.b[s][nt], D[nt]);
                }
            }
            if (p.kc + 16 * KS < p.c) return;                      // the slice has more columns
            // lane holds rows 4*(lane/16)+i, right-hand side group lane%16 of each result tile
            uint32_t at[4];
            bool on[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t mr = p.m0 + 4u * kq + i;
                on[i] = mr < p.r;
                const uint32_t slot = meta[p.desc + 4u * (p.lane0 + (on[i] ? mr : 0u))];
                at[i] = slot * NB + 4u * mrow;
            }
            float4 old4[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) old4[i] = *(const float4 *)(myacc + at[i]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (on[i])
                    *(float4 *)(myacc + at[i]) = make_float4(old4[i].x + D[0][i], old4[i].y + D[1][i],
                                                             old4[i].z + D[2][i], old4[i].w + D[3][i]);
        };
        auto nxt = [&](const Pass &p) -> Pass { return p.valid ? next_pass(p) : p; };
        OperandsBf<KS> oa, ob, oc;                                  // three passes in flight
        Pass pa = open_vb(wave), pb = nxt(pa), pc{};
        if (pa.valid) load_pass(pa, oa);
        if (pb.valid) load_pass(pb, ob);
        while (true) {
            pc = nxt(pb); if (pc.valid) load_pass(pc, oc);
            if (!pa.valid) break;
            mult_pass(pa, oa);
            pa = nxt(pc); if (pa.valid) load_pass(pa, oa);
            if (!pb.valid) break;
            mult_pass(pb, ob);
            pb = nxt(pa); if (pb.valid) load_pass(pb, ob);
            if (!pc.valid) break;
            mult_pass(pc, oc);
        }
    }
    __syncthreads();
    for (uint32_t e = tid; e < br * NB; e += NTHR) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += acc[(size_t)w * br * NB + e];
        const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
        if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = s;
    }
}

// ---------------------------------------------------------------------------------------
// The wide form for row tiles of 16 or 32 rows, with the results kept in registers (VF: storage
// format of the kernel values; 16-bit values come as one word per row and pair of columns and
// are unpacked to binary32 on their way into the MFMA).  Counters of the general kernel above on the 8192 x 8192 matrix with 128
// right-hand sides show what its launch time is made of: vector instructions other than MFMA
// keep every SIMD busy for 38 % of the launch (about 480 instructions per pass of at most 16
// MFMAs, among them the accumulate of every 16-row slice's 16 x 64 results into the wavefront's
// LDS tile: four 16-byte reads and four writes per lane), the matrix pipe a quarter, and
// pointing every gather at ONE row of X makes it only 7 % faster -- the gather is not the
// bound.  Here the kernel operand of an MFMA is not the block's kernel matrix but its
// rows ALREADY SCATTERED to their places in the row tile: for each 16-row part of the tile, lane
// (row, k) holds the block's value at that tile row, or zero if the block does not keep the
// row.  The 16 x 64 results of a part then add up in the SAME registers over all blocks the
// wavefront works on, and go to LDS once, at the end.  The price is matrix-pipe work for parts
// a block has few rows in (parts it has none in are skipped).  Which kernel row sits at a tile
// row comes from a 64-byte map per wavefront in LDS that the block's lanes fill from their row
// slots.  A pass ALWAYS issues 4 NH kernel-value loads and four 16-byte input loads (k-steps and
// parts a block does not have repeat a valid address and are not multiplied), so the loads of
// the NEXT pass are in flight while this pass multiplies and the compiler's counted waits hold.
// Same records, same value layout, same merge of the wavefronts' tiles as the general kernel.
template <int NH>
struct RegOps {
    float av[NH][4];
    float4 bv[4];
    uint32_t parts;              // bit h: the block has rows in part h (uniform)
};
// ... with 16-bit right-hand sides (X16): a pass is ONE 16-column MFMA step per part and tile; a
// lane's four columns of its tile row are two words of the value stream, its four right-hand
// sides of a column eight bytes of X.
template <int NH>
struct RegOps16 {
    uint32_t aw[NH][2];
    uint2 xv[4];
    uint32_t parts;
};
struct RegPass {
    uint32_t k, kc;              // virtual block (inside the segment), first column of the pass
    uint32_t r, c, lane0;        // the block's rows, columns, first lane
    uint32_t val_off, desc, list;
    bool valid;
};

template <bool TWO, int NW, int NH, int VF, bool X16 = false>
__device__ __forceinline__ void spmm_reg_body(const DevMat &m, const XSrc &X, float *__restrict__ Y, const int64_t ldy,
                                              const uint32_t batch, const uint32_t block_x, const uint32_t block_y) {
    extern __shared__ float4 smem4[];
    constexpr uint32_t NB = 64, NTHR = NW * 64;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = uni_(tid >> 6);
    const uint32_t bt0 = block_y * NB;
    const uint32_t br = m.br;                                      // == 16 NH
    if (block_x >= m.n_nz_tiles) {                 // a row tile without work: zeros
        const uint32_t tile = m.zero_tiles[block_x - m.n_nz_tiles];
        for (uint32_t e = tid; e < br * NB; e += NTHR) {
            const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
            if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = 0.0f;
        }
        return;
    }
    uint8_t *meta = (uint8_t *)smem4;                              // one record segment
    float *acc = (float *)(meta + m.seg_meta);                     // [waves][br][NB]
    float *myacc = acc + (size_t)wave * br * NB;
    uint8_t *inv = (uint8_t *)(acc + (size_t)NW * br * NB) + wave * 64u;   // tile row -> kernel row of the current block, 0xff: none
    const uint32_t rank = block_x, tile = m.nz_tiles[rank];
    const uint32_t mrow = lane & 15u, kq = lane >> 4;              // A: tile row in its part, column-in-4; B: right-hand sides 4 mrow .. + 3, row-in-4
    const uint32_t ncol = bt0 + 4u * mrow;
    const uint32_t nbyte = (ncol < batch ? ncol : 0u) * (X16 ? 2u : 4u);   // (batch is a multiple of 4: the four are in or out together)
    const uint8_t *const x0 = (const uint8_t *)X.p0 + nbyte, *const x1 = (const uint8_t *)X.p1 + nbyte;
    const uint32_t split4 = 4u * X.n0;
    floatx4 D[NH][4];
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) D[h][nt] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    for (uint32_t sg = m.tile_seg0[rank]; sg < m.tile_seg0[rank + 1]; ++sg) {
        // ---- stage the segment's records ------------------------------------------------
        const SegRec *sp = m.segs + sg;
        const uint32_t ga = sp->g0, ng = sp->ng, vb0 = sp->vb0, nvbs = sp->nvbs, idx0 = sp->idx0, idx_bytes = sp->idx_bytes;
        const uint32_t voff = (ng * (uint32_t)sizeof(GroupRec) + 15u) & ~15u;
        const uint32_t ioff = voff + ((nvbs * (uint32_t)sizeof(VbRec) + 15u) & ~15u);
        __syncthreads();                                           // the previous segment is done with
        {
            const uint2 *gs = (const uint2 *)(m.groups + ga);
            uint2 *gd = (uint2 *)meta;
            for (uint32_t i = tid; i < ng * 3u; i += NTHR) gd[i] = gs[i];
            const float4 *vs = (const float4 *)(m.vbs + vb0);
            float4 *vd = (float4 *)(meta + voff);
            for (uint32_t i = tid; i < nvbs; i += NTHR) vd[i] = vs[i];
            const float4 *is = (const float4 *)(m.idx + idx0);
            float4 *id = (float4 *)(meta + ioff);
            for (uint32_t i = tid; i < idx_bytes >> 4; i += NTHR) id[i] = is[i];
        }
        __syncthreads();
        if (wave >= nvbs) continue;                                // (uniform per wavefront; the barriers above are passed by all)

        // Kernel values come through a buffer descriptor over the value stream: a load whose offset lies
        // past the stream returns zero, which is what a lane without a row or a column gets (its offset
        // is pushed there), so no operand is ever masked after the load.
        const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc((void *)m.vals, 0, (int)m.vals_bytes, 0x00020000);
        uint32_t irow4[NH];                                        // byte offset of this lane's kernel row in the current block's values, per part (bit 31: none)
        uint32_t parts = 0;
        // Opens virtual block k < nvbs: its record, and the map from tile rows to its kernel rows.
        auto open_vb = [&](uint32_t k, RegPass &p) {
            const uint4 v = *(const uint4 *)(meta + voff + k * (uint32_t)sizeof(VbRec));
            const uint32_t v0 = uni_(v.x);
            p.k = k; p.valid = true; p.kc = 0;
            p.r = v0 & 0xffu; p.lane0 = (v0 >> 8) & 0xffu; p.c = v0 >> 16;
            p.val_off = uni_(v.y);
            p.desc = ioff + (uni_(v.z) - idx0);
            p.list = ioff + (uni_(v.w) - idx0);
            // the map: cleared, then every kernel row of the block enters itself at its tile row (the
            // wavefront's LDS operations execute in order)
            const uint32_t slot = meta[p.desc + 4u * (p.lane0 + (lane < p.r ? lane : 0u))];
            if (lane < 16u) ((uint32_t *)inv)[lane] = 0xffffffffu;
            if (lane < p.r) inv[slot] = (uint8_t)lane;
            parts = 0;
            // (16-bit formats: one 32-bit word per kernel row and PAIR of columns, the even column in the low half)
            const uint32_t base4 = ((VF == CSB_VAL_F32 ? p.val_off : p.val_off >> 1) + p.lane0) * 4u;
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const uint32_t ir = inv[16u * h + mrow];
                irow4[h] = ir != 0xffu ? base4 + ir * 4u : 0x80000000u;
                parts |= __ballot(ir != 0xffu) != 0ull ? 1u << h : 0u;
            }
        };
        // The pass after p.  Without a branch: the block is opened again even when the pass stays in it
        // (same record, same map), so that no path through here differs in the memory operations it
        // issues and the compiler's counted waits stay exact.  Past the wavefront's last pass the
        // fields stay (their loads are issued once more and dropped) and only `valid` goes off.
        auto advance = [&](const RegPass &p) -> RegPass {
            const bool same = p.kc + 16u < p.c, more = p.k + NW < nvbs;
            const uint32_t kc2 = same ? p.kc + 16u : (more ? 0u : p.kc);
            RegPass q;
            open_vb(same || !more ? p.k : p.k + NW, q);
            q.kc = kc2;
            q.valid = same || more;
            return q;
        };
        // 4 NH + 4 loads, always.  (Uses irow4 / parts of the block opened last: p's.)
        auto issue = [&](const RegPass &p, RegOps<NH> &o) {
            uint32_t cb[4], ja[4];
            o.parts = parts;
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const uint32_t jj = p.kc + 4u * s4 + kq;
                ja[s4] = jj < p.c ? jj : 0x7fffffu;                             // a column the block lacks: past the stream
                cb[s4] = *(const uint16_t *)(meta + p.list + 2u * min(jj, p.c - 1u));      // 4 * column
            }
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
#pragma unroll
                for (int h = 0; h < NH; ++h)
                    if constexpr (VF == CSB_VAL_F32) {
                        o.av[h][s4] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(vrsrc, (int)(ja[s4] * 256u + irow4[h]), 0, 0));
                    } else {                                        // (unpacked in multiply: the load's result is not waited for here)
                        o.av[h][s4] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(vrsrc, (int)((ja[s4] >> 1) * 256u + irow4[h]), 0, 0));
                    }
                if constexpr (TWO) {
                    const bool first = cb[s4] < split4;
                    const uint8_t *src = first ? x0 + __umul24(cb[s4], X.sj0) : x1 + __umul24(cb[s4] - split4, X.sj1);
                    o.bv[s4] = *(const float4 *)src;
                } else {
                    o.bv[s4] = *(const float4 *)((const uint8_t *)X.p0 + (size_t)(__umul24(cb[s4], X.sj0) + nbyte));
                }
            }
        };
        auto multiply = [&](const RegPass &p, const RegOps<NH> &o) {
            const uint32_t nk = min(4u, (p.c - p.kc + 3u) >> 2);      // k-steps the block has in this pass (uniform)
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                if (!((o.parts >> h) & 1u)) continue;              // (uniform) no row of the block in this part
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    if ((uint32_t)s4 >= nk) break;
                    float a = o.av[h][s4];
                    if constexpr (VF != CSB_VAL_F32) {              // this lane's column of the pair: kc is even, so its parity is kq's
                        const uint32_t w = __float_as_uint(a);
                        if constexpr (VF == CSB_VAL_BF16) a = __uint_as_float((kq & 1u) ? w & 0xffff0000u : w << 16);
                        else a = (float)__builtin_bit_cast(_Float16, (uint16_t)((kq & 1u) ? w >> 16 : w & 0xffffu));
                    }
                    D[h][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, o.bv[s4].x, D[h][0], 0, 0, 0);
                    D[h][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, o.bv[s4].y, D[h][1], 0, 0, 0);
                    D[h][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, o.bv[s4].z, D[h][2], 0, 0, 0);
                    D[h][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, o.bv[s4].w, D[h][3], 0, 0, 0);
                }
            }
        };
        // The same two steps with 16-bit right-hand sides (X.p0: their rows, X.sj0: elements per row):
        // 2 NH + 4 loads, always, and one 16-column MFMA per part and tile.
        auto issue16 = [&](const RegPass &p, RegOps16<NH> &o) {
            o.parts = parts;
            const uint32_t j0 = p.kc + 4u * kq;                                  // this lane's four columns
            const uint32_t w0 = j0 < p.c ? (j0 >> 1) * 256u : 0x3fffff00u;       // words of the pairs (j0, j0 + 1), (j0 + 2, j0 + 3);
            const uint32_t w1 = j0 + 2u < p.c ? (j0 >> 1) * 256u + 256u : 0x3fffff00u;   // a pair the block lacks: past the stream
            uint32_t cb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) cb[i] = *(const uint16_t *)(meta + p.list + 2u * min(j0 + (uint32_t)i, p.c - 1u));   // 4 * column
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                o.aw[h][0] = __builtin_amdgcn_raw_buffer_load_b32(vrsrc, (int)(w0 + irow4[h]), 0, 0);
                o.aw[h][1] = __builtin_amdgcn_raw_buffer_load_b32(vrsrc, (int)(w1 + irow4[h]), 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)      // (a column the block lacks reads its last one: finite, times a zero)
                o.xv[i] = *(const uint2 *)((const uint8_t *)X.p0 + (size_t)((__umul24(cb[i], X.sj0) >> 1) + nbyte));
        };
        auto multiply16 = [&](const RegOps16<NH> &o) {
            // xv[i] = right-hand sides 0..3 at column i; tile t wants columns 0..3 at right-hand side t
            const uint2 b0 = make_uint2((o.xv[0].x & 0xffffu) | (o.xv[1].x << 16), (o.xv[2].x & 0xffffu) | (o.xv[3].x << 16));
            const uint2 b1 = make_uint2((o.xv[0].x >> 16) | (o.xv[1].x & 0xffff0000u), (o.xv[2].x >> 16) | (o.xv[3].x & 0xffff0000u));
            const uint2 b2 = make_uint2((o.xv[0].y & 0xffffu) | (o.xv[1].y << 16), (o.xv[2].y & 0xffffu) | (o.xv[3].y << 16));
            const uint2 b3 = make_uint2((o.xv[0].y >> 16) | (o.xv[1].y & 0xffff0000u), (o.xv[2].y >> 16) | (o.xv[3].y & 0xffff0000u));
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                if (!((o.parts >> h) & 1u)) continue;              // (uniform) no row of the block in this part
                const uint2 a = make_uint2(o.aw[h][0], o.aw[h][1]);
                D[h][0] = mfma_16bit<VF == CSB_VAL_F16>(a, b0, D[h][0]);
                D[h][1] = mfma_16bit<VF == CSB_VAL_F16>(a, b1, D[h][1]);
                D[h][2] = mfma_16bit<VF == CSB_VAL_F16>(a, b2, D[h][2]);
                D[h][3] = mfma_16bit<VF == CSB_VAL_F16>(a, b3, D[h][3]);
            }
        };
        if constexpr (X16) {
            RegOps16<NH> oa, ob;
            RegPass pa, pb;
            open_vb(wave, pa);
            issue16(pa, oa);
            while (true) {
                pb = advance(pa);
                issue16(pb, ob);
                multiply16(oa);
                if (!pb.valid) break;
                pa = advance(pb);
                issue16(pa, oa);
                multiply16(ob);
                if (!pa.valid) break;
            }
            continue;                                              // (the next segment)
        }
        RegOps<NH> oa, ob;
        RegPass pa, pb;
        open_vb(wave, pa);
        issue(pa, oa);
        while (true) {
            pb = advance(pa);
            issue(pb, ob);
            multiply(pa, oa);
            if (!pb.valid) break;
            pa = advance(pb);
            issue(pa, oa);
            multiply(pb, ob);
            if (!pa.valid) break;
        }
    }
    // the wavefront's tile: lane holds rows 16 h + 4 kq + i, right-hand sides 4 mrow + t (tile t)
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *(float4 *)(myacc + (16u * h + 4u * kq + i) * NB + 4u * mrow) = make_float4(D[h][0][i], D[h][1][i], D[h][2][i], D[h][3][i]);
    __syncthreads();
    for (uint32_t e = tid; e < br * NB; e += NTHR) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += acc[(size_t)w * br * NB + e];
        const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
        if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = s;
    }
}

template <bool TWO, int NW, int NH, int VF>
__global__ __launch_bounds__(NW * 64) void spmm_reg_kernel(const DevMat m, const XSrc X, float *__restrict__ Y,
                                                           const int64_t ldy, const uint32_t batch) {
    spmm_reg_body<TWO, NW, NH, VF>(m, X, Y, ldy, batch, blockIdx.x, blockIdx.y);
}

// 16-bit kernel values times 16-bit right-hand sides (X.p0: the rows of X, X.sj0: elements per row).
template <int NW, int NH, int VF>
__global__ __launch_bounds__(NW * 64) void spmm_reg16_kernel(const DevMat m, const XSrc X, float *__restrict__ Y,
                                                             const int64_t ldy, const uint32_t batch) {
    static_assert(VF == CSB_VAL_F16 || VF == CSB_VAL_BF16, "16-bit formats only");
    spmm_reg_body<false, NW, NH, VF, true>(m, X, Y, ldy, batch, blockIdx.x, blockIdx.y);
}

// Several independent products in one launch (blockIdx.z picks the product): the per-step
// products of different layers of a batched recurrent model, each too small to fill the GPU.
struct SpmmJobs {
    DevMat m[kMaxJobsPerLaunch];
    XSrc X[kMaxJobsPerLaunch];
    float *Y[kMaxJobsPerLaunch];
    int64_t ldy[kMaxJobsPerLaunch];
};
template <int NT, bool TWO, int NW, bool WIDE>
__global__ __launch_bounds__(NW * 64) void spmm_multi_kernel(const SpmmJobs J, const uint32_t batch) {
    const uint32_t j = blockIdx.z;
    if (blockIdx.x >= J.m[j].n_nz_tiles + J.m[j].n_zero_tiles) return;      // the grid is as wide as the widest product
    spmm_body<NT, TWO, NW, WIDE>(J.m[j], J.X[j], J.Y[j], J.ldy[j], batch, blockIdx.x, blockIdx.y);
}

template <bool TWO, int NW, int NH, int VF>
__global__ __launch_bounds__(NW * 64) void spmm_reg_multi_kernel(const SpmmJobs J, const uint32_t batch) {
    const uint32_t j = blockIdx.z;
    if (blockIdx.x >= J.m[j].n_nz_tiles + J.m[j].n_zero_tiles) return;      // the grid is as wide as the widest product
    spmm_reg_body<TWO, NW, NH, VF>(J.m[j], J.X[j], J.Y[j], J.ldy[j], batch, blockIdx.x, blockIdx.y);
}

// Launch shape of one product: batch columns per workgroup (16 nt), wavefronts per workgroup.
struct SpmmShape {
    int nt, nw;
    bool two, wide;
    int reg_parts;          // wide form, row tiles of 16 or 32 rows: the kernel that keeps the results in
                            // registers, with this many 16-row parts (else 0; four parts do not fit the
                            // registers of a 16-wavefront workgroup)
    int vf;                 // storage format of the kernel values
    size_t lds;
    unsigned tiles, batch_tiles;
};

// Checks one product's operands and chooses its launch shape; `launch_wgs_factor` products of
// this size share the launch, which counts when the launch is sized against the GPU's 256 CUs.
static int spmm_shape(const SpmmCall &c, int32_t batch, size_t launch_wgs_factor, SpmmShape *out, XSrc *X) {
    const csb_matrix *mat = c.mat;
    if (!mat->plan.valid || !mat->uploaded || !mat->d_buf) { set_error("csb_spmm: matrix not planned and uploaded"); return CSB_ESTATE; }
    const DevHeader &h = mat->plan.hdr;
    // 32-bit element offsets, 24-bit multiplies
    const int64_t smax_j = std::max(c.sj0, c.sj1), smax_n = std::max(c.sn0, c.sn1);
    if (c.sj0 < 0 || c.sj1 < 0 || c.sn0 < 0 || c.sn1 < 0 || smax_j >= (1 << 24) || (int64_t)h.cols >= (1 << 24) ||
        (int64_t)h.cols * smax_j + (int64_t)batch * smax_n >= (1ll << 30)) {
        set_error("csb_spmm: strides or sizes beyond the kernel's 32-bit element offsets");
        return CSB_EUNSUPPORTED;
    }
    *X = XSrc{c.p0, c.n0, (uint32_t)c.sj0, (uint32_t)c.sn0, c.p1, (uint32_t)c.sj1, (uint32_t)c.sn1};
    const bool two = c.n0 < (uint32_t)h.cols;
    // the wide form: right-hand sides contiguous, rows of the input 16-byte aligned, batch in
    // fours, and eight wavefronts' accumulator tiles of 64 columns fit LDS
    const bool aligned = ((uintptr_t)c.p0 % 16 == 0) && c.sj0 % 4 == 0 && c.sn0 == 1 &&
                         (!two || (((uintptr_t)c.p1 % 16 == 0) && c.sj1 % 4 == 0 && c.sn1 == 1));
    const bool wide_ok = aligned && batch % 4 == 0 &&
                         (size_t)h.seg_meta + 8 * (size_t)h.br * 64 * sizeof(float) <= (size_t)kLdsBudget;
    // batch columns per workgroup: the widest form whose launch still gives every CU (256) a workgroup
    const size_t tiles = (size_t)h.n_nz_tiles + h.n_zero_tiles;
    auto wgs = [&](int n) { return tiles * (size_t)((batch + 16 * n - 1) / (16 * n)); };
    int nt = 1;
    if (h.br <= 128 && batch > 16 && wgs(2) * launch_wgs_factor >= 256) nt = 2;
    if (wide_ok && batch >= 48 && wgs(4) * launch_wgs_factor >= 256) nt = 4;
    const bool wide = nt == 4;
    // 16 wavefronts share a tile's blocks when their accumulator tiles fit LDS and the launch
    // alone would not give every CU of an MI355X (256) two workgroups; else 8
    const size_t acc_per_wave = (size_t)h.br * 16 * nt * sizeof(float);
    const bool fits16 = (size_t)h.seg_meta + 16 * acc_per_wave <= (size_t)kLdsBudget;
    const int nw = fits16 && (wide || wgs(nt) * launch_wgs_factor < 2 * 256) ? 16 : 8;
    // (its 32-bit byte offsets into the value stream must stay below the out-of-range marker)
    const int reg_parts = (wide && (h.br == 16 || h.br == 32) && h.n_vals * 4 < 0x7fffff00ull &&
                           (size_t)h.seg_meta + (size_t)nw * acc_per_wave + (size_t)nw * 64 <= (size_t)160 * 1024) ? (int)h.br / 16 : 0;
    *out = SpmmShape{nt, nw, two, wide, reg_parts, (int)h.val_fmt, (size_t)h.seg_meta + (size_t)nw * acc_per_wave + (reg_parts ? (size_t)nw * 64 : 0), (unsigned)tiles,
                     (unsigned)((batch + 16 * nt - 1) / (16 * nt))};
    return CSB_OK;
}

// The kernel instantiation for a launch shape (one product per launch, or several).
template <bool MULTI>
static const void *spmm_kernel_for(const SpmmShape &sh) {
#define CSB_SPMM_K(NT, TWO, NW, WIDE) \
    (MULTI ? (const void *)spmm_multi_kernel<NT, TWO, NW, WIDE> : (const void *)spmm_kernel<NT, TWO, NW, WIDE>)
    if (sh.reg_parts) {
#define CSB_SPMM_RV(TWO, NW, NH, VF) (MULTI ? (const void *)spmm_reg_multi_kernel<TWO, NW, NH, VF> : (const void *)spmm_reg_kernel<TWO, NW, NH, VF>)
#define CSB_SPMM_R(TWO, NW, NH) (sh.vf == CSB_VAL_F16 ? CSB_SPMM_RV(TWO, NW, NH, CSB_VAL_F16) : sh.vf == CSB_VAL_BF16 ? CSB_SPMM_RV(TWO, NW, NH, CSB_VAL_BF16) : CSB_SPMM_RV(TWO, NW, NH, CSB_VAL_F32))
#define CSB_SPMM_RN(NH) \
        if (sh.nw == 16) return sh.two ? CSB_SPMM_R(true, 16, NH) : CSB_SPMM_R(false, 16, NH); \
        return sh.two ? CSB_SPMM_R(true, 8, NH) : CSB_SPMM_R(false, 8, NH);
        if (sh.reg_parts == 1) { CSB_SPMM_RN(1) }
        CSB_SPMM_RN(2)
#undef CSB_SPMM_RN
#undef CSB_SPMM_R
#undef CSB_SPMM_RV
    }
    if (sh.wide) {
        if (sh.nw == 16) return sh.two ? CSB_SPMM_K(4, true, 16, true) : CSB_SPMM_K(4, false, 16, true);
        return sh.two ? CSB_SPMM_K(4, true, 8, true) : CSB_SPMM_K(4, false, 8, true);
    }
    if (sh.nw == 16) {
        if (sh.nt == 2) return sh.two ? CSB_SPMM_K(2, true, 16, false) : CSB_SPMM_K(2, false, 16, false);
        return sh.two ? CSB_SPMM_K(1, true, 16, false) : CSB_SPMM_K(1, false, 16, false);
    }
    if (sh.nt == 2) return sh.two ? CSB_SPMM_K(2, true, 8, false) : CSB_SPMM_K(2, false, 8, false);
    return sh.two ? CSB_SPMM_K(1, true, 8, false) : CSB_SPMM_K(1, false, 8, false);
#undef CSB_SPMM_K
}

int spmm_strided(const csb_matrix *mat, const float *p0, uint32_t n0, int64_t sj0, int64_t sn0, const float *p1,
                 int64_t sj1, int64_t sn1, float *d_Y, int64_t ldy, int32_t batch, void *stream) {
    const SpmmCall c{mat, p0, n0, sj0, sn0, p1, sj1, sn1, d_Y, ldy};
    SpmmShape sh;
    XSrc X;
    int rc = spmm_shape(c, batch, 1, &sh, &X);
    if (rc != CSB_OK) return rc;
    DevMat dm = dev_mat(mat);
    uint32_t b = (uint32_t)batch;
    int64_t ld = ldy;
    void *args[] = {&dm, &X, &d_Y, &ld, &b};
    const void *kern = spmm_kernel_for<false>(sh);
    hipError_t e = ensure_dynamic_lds(kern, sh.lds);
    if (e == hipSuccess)
        e = hipLaunchKernel(kern, dim3(sh.tiles, sh.batch_tiles), dim3(sh.nw * 64), args, sh.lds, (hipStream_t)stream);
    if (e != hipSuccess) { set_error(std::string("csb_spmm: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

// Up to kMaxJobsPerLaunch independent products in ONE launch when they agree on the launch shape
// (same-shaped layers do); otherwise one launch each.
int spmm_strided_multi(const SpmmCall *calls, int n, int32_t batch, void *stream) {
    if (n <= 0) return CSB_OK;
    SpmmShape sh[kMaxJobsPerLaunch];
    SpmmJobs J{};
    bool same = n <= kMaxJobsPerLaunch && n > 1;
    if (same) {
        size_t lds = 0;
        unsigned tiles = 0;
        for (int i = 0; i < n; ++i) {
            int rc = spmm_shape(calls[i], batch, (size_t)n, &sh[i], &J.X[i]);
            if (rc != CSB_OK) return rc;
            same = same && sh[i].nt == sh[0].nt && sh[i].nw == sh[0].nw && sh[i].two == sh[0].two && sh[i].wide == sh[0].wide && sh[i].reg_parts == sh[0].reg_parts && sh[i].vf == sh[0].vf;
            lds = std::max(lds, sh[i].lds);
            tiles = std::max(tiles, sh[i].tiles);
            J.m[i] = dev_mat(calls[i].mat);
            J.Y[i] = calls[i].Y;
            J.ldy[i] = calls[i].ldy;
        }
        if (same) {
            uint32_t b = (uint32_t)batch;
            void *args[] = {&J, &b};
            const void *kern = spmm_kernel_for<true>(sh[0]);
            hipError_t e = ensure_dynamic_lds(kern, lds);
            if (e == hipSuccess)
                e = hipLaunchKernel(kern, dim3(tiles, sh[0].batch_tiles, (unsigned)n), dim3(sh[0].nw * 64), args, lds, (hipStream_t)stream);
            if (e != hipSuccess) { set_error(std::string("csb_spmm: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
            return CSB_OK;
        }
    }
    for (int i = 0; i < n; ++i) {
        const SpmmCall &c = calls[i];
        int rc = spmm_strided(c.mat, c.p0, c.n0, c.sj0, c.sn0, c.p1, c.sj1, c.sn1, c.Y, c.ldy, batch, stream);
        if (rc != CSB_OK) return rc;
    }
    return CSB_OK;
}

}  // namespace csb

namespace csb {
// csb_spmm_bfloat / csb_spmm_half: both operands in the 16-bit format `fmt`
static int spmm_16bit(const char *who, int fmt, const csb_matrix *m, const uint16_t *d_X, int64_t ldx, float *d_Y, int64_t ldy,
                      int32_t batch, void *stream) {
    const std::string w(who);
    if (!m || !d_X || !d_Y) { set_error(w + ": NULL pointer"); return CSB_EINVAL; }
    if (batch <= 0 || ldx < batch || ldy < batch) { set_error(w + ": batch <= 0 or a leading dimension below batch"); return CSB_EINVAL; }
    if (!m->plan.valid || !m->uploaded || !m->d_buf) { set_error(w + ": matrix not planned and uploaded"); return CSB_ESTATE; }
    if (m->plan.split.active()) { set_error(w + ": matrix is planned for a GRU step"); return CSB_ESTATE; }
    const DevHeader &h = m->plan.hdr;
    if ((int)h.val_fmt != fmt) { set_error(w + ": the matrix does not store its values in this format (csb_set_value_format)"); return CSB_ESTATE; }
    // four right-hand sides per 8-byte load; 32-bit byte offsets and a 24-bit multiply
    if (batch % 4 != 0 || ldx % 4 != 0 || (uintptr_t)d_X % 8 != 0) {
        set_error(w + ": batch and ldx must be multiples of 4 and X 8-byte aligned");
        return CSB_EUNSUPPORTED;
    }
    if (ldx >= (1 << 24) || (int64_t)h.cols * ldx + batch >= (1ll << 30)) {
        set_error(w + ": sizes beyond the kernel's 32-bit offsets");
        return CSB_EUNSUPPORTED;
    }
    const size_t acc_per_wave = (size_t)h.br * 64 * sizeof(float);
    const bool fits16 = (size_t)h.seg_meta + 16 * acc_per_wave <= (size_t)kLdsBudget;
    if ((size_t)h.seg_meta + 8 * acc_per_wave > (size_t)kLdsBudget) {
        set_error(w + ": the block rows are too tall for the accumulator tiles");
        return CSB_EUNSUPPORTED;
    }
    const int nw = fits16 ? 16 : 8;
    DevMat dm = dev_mat(m);
    uint32_t b = (uint32_t)batch, ld = (uint32_t)ldx;
    int64_t ldy_ = ldy;
    const bool half = fmt == CSB_VAL_F16;
    // row tiles of 16 or 32 rows: the kernel that keeps its results in registers
    const size_t lds_reg = (size_t)h.seg_meta + (size_t)nw * acc_per_wave + (size_t)nw * 64;
    if ((h.br == 16 || h.br == 32) && h.n_vals * 4 < 0x7fffff00ull && lds_reg <= (size_t)160 * 1024) {
        XSrc X{(const float *)d_X, (uint32_t)h.cols, ld, 1u, (const float *)d_X, ld, 1u};
        void *rargs[] = {&dm, &X, &d_Y, &ldy_, &b};
        const void *kern;
#define CSB_R16(NW, NH) (half ? (const void *)spmm_reg16_kernel<NW, NH, CSB_VAL_F16> : (const void *)spmm_reg16_kernel<NW, NH, CSB_VAL_BF16>)
        if (nw == 16) kern = h.br == 16 ? CSB_R16(16, 1) : CSB_R16(16, 2);
        else kern = h.br == 16 ? CSB_R16(8, 1) : CSB_R16(8, 2);
#undef CSB_R16
        hipError_t e = ensure_dynamic_lds(kern, lds_reg);
        if (e == hipSuccess)
            e = hipLaunchKernel(kern, dim3((unsigned)(h.n_nz_tiles + h.n_zero_tiles), (unsigned)((batch + 63) / 64)), dim3(nw * 64), rargs, lds_reg,
                                (hipStream_t)stream);
        if (e != hipSuccess) { set_error(w + ": " + hipGetErrorString(e)); return CSB_EDEVICE; }
        return CSB_OK;
    }
    const size_t lds = (size_t)h.seg_meta + (size_t)nw * acc_per_wave;
    void *args[] = {&dm, &d_X, &ld, &d_Y, &ldy_, &b};
    const void *kern = nw == 16 ? (half ? (const void *)spmm_bf16_kernel<16, true> : (const void *)spmm_bf16_kernel<16, false>)
                                : (half ? (const void *)spmm_bf16_kernel<8, true> : (const void *)spmm_bf16_kernel<8, false>);
    hipError_t e = ensure_dynamic_lds(kern, lds);
    if (e == hipSuccess)
        e = hipLaunchKernel(kern, dim3((unsigned)(h.n_nz_tiles + h.n_zero_tiles), (unsigned)((batch + 63) / 64)), dim3(nw * 64), args, lds,
                            (hipStream_t)stream);
    if (e != hipSuccess) { set_error(w + ": " + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}
}  // namespace csb

extern "C" int csb_spmm_bfloat(const csb_matrix *m, const uint16_t *d_Xb, int64_t ldx, float *d_Y, int64_t ldy,
                               int32_t batch, void *stream) {
    return csb::spmm_16bit("csb_spmm_bfloat", CSB_VAL_BF16, m, d_Xb, ldx, d_Y, ldy, batch, stream);
}

extern "C" int csb_spmm_half(const csb_matrix *m, const uint16_t *d_Xh, int64_t ldx, float *d_Y, int64_t ldy,
                             int32_t batch, void *stream) {
    return csb::spmm_16bit("csb_spmm_half", CSB_VAL_F16, m, d_Xh, ldx, d_Y, ldy, batch, stream);
}

extern "C" int csb_spmm(const csb_matrix *m, const float *d_X, int64_t ldx, float *d_Y, int64_t ldy,
                        int32_t batch, void *d_ws, void *stream) {
    (void)d_ws;
    if (!m || !d_X || !d_Y) { csb::set_error("csb_spmm: NULL pointer"); return CSB_EINVAL; }
    if (batch <= 0 || ldx < batch || ldy < batch) { csb::set_error("csb_spmm: batch <= 0 or a leading dimension below batch"); return CSB_EINVAL; }
    if (m->plan.valid && m->plan.split.active()) { csb::set_error("csb_spmm: matrix is planned for a GRU step"); return CSB_ESTATE; }
    return csb::spmm_strided(m, d_X, (uint32_t)m->cols, ldx, 1, d_X, ldx, 1, d_Y, ldy, batch, stream);
}
