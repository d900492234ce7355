// Projection of a dense matrix onto the CSB pattern (the pruning step inside Algorithm 1,
// Sec. 3.2.2) for gfx950: RowPrune in every block-column, then ColumnPrune in every
// block-row on the row-pruned matrix, each zeroing the share 1 - sqrt(1 - PruneRate) of the
// segments with the smallest sums of squares.
//
// Five launches on one stream: sums of squares of the in-block row segments, selection per
// block-column, sums of squares of the in-block column segments of the row-pruned matrix,
// selection per block-row, and the masked copy.  The decisions are integers taken from
// float32 sums, so the sums use one fixed order (left to right / top to bottom, one fused
// multiply-add per element) and ties go by position: the result is the same bits on every
// run and on every machine that does the arithmetic this way.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "csb_internal.hpp"

namespace csb {

constexpr int kProjectMaxDim = 16384;     // segments ranked by one workgroup: 16 keys in each of 1024 threads

// Ranking key of a sum of squares: its bit pattern (sums are >= +0 or NaN, so the unsigned
// order of the bits is the numeric order); every NaN ranks on top.
__device__ __forceinline__ uint32_t rank_key(float s) {
    const uint32_t u = __float_as_uint(s);
    return s != s ? 0xffffffffu : u;
}

// keys[bj * R + i] for row segment (i, bj).  A workgroup takes TR rows x TS segments: it
// reads their columns coalesced into LDS (segment stride BC | 1 words, so that the lanes of
// the next phase hit different banks), then thread (r, sj) adds up its own segment from left
// to right.  DIV_SHIFT >= 0: BC is 1 << DIV_SHIFT.
template <int DIV_SHIFT>
__global__ __launch_bounds__(256) void row_segment_keys_kernel(const float *__restrict__ W, const int64_t ld,
                                                                 const uint32_t R, const uint32_t C, const uint32_t BC,
                                                                 const uint32_t NBC, const uint32_t TR, const uint32_t TS,
                                                                 uint32_t *__restrict__ keys) {
    extern __shared__ float tile[];
    const uint32_t tid = threadIdx.x;
    const uint32_t bj0 = blockIdx.x * TS, i0 = blockIdx.y * TR;
    const uint32_t c0 = bj0 * BC, c1 = min(C, (bj0 + TS) * BC), ncols = c1 - c0;
    const uint32_t BCp = BC | 1u;
    for (uint32_t r = 0; r < TR && i0 + r < R; ++r) {
        const float *p = W + (size_t)(i0 + r) * ld + c0;
        float *row = tile + (size_t)r * TS * BCp;
        for (uint32_t cb = tid; cb < ncols; cb += 1024) {           // four independent loads per pass
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = cb + 256u * u < ncols ? p[cb + 256u * u] : 0.0f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t cc = cb + 256u * u;
                if (cc < ncols) {
                    const uint32_t seg = DIV_SHIFT >= 0 ? cc >> (DIV_SHIFT >= 0 ? DIV_SHIFT : 0) : cc / BC;
                    row[seg * BCp + (cc - seg * BC)] = v[u];
                }
            }
        }
    }
    __syncthreads();
    const uint32_t r = tid / TS, sj = tid - r * TS;
    if (r < TR && i0 + r < R && bj0 + sj < NBC) {
        const uint32_t w = min(BC, C - (bj0 + sj) * BC);
        const float *q = tile + ((size_t)r * TS + sj) * BCp;
        float s = 0.0f;
        for (uint32_t c = 0; c < w; ++c) s = fmaf(q[c], q[c], s);
        keys[(size_t)(bj0 + sj) * R + i0 + r] = rank_key(s);
    }
}

// The same for BC = 4 Q columns per segment (Q = 4, 8, 16), C a multiple of BC and rows that
// start at multiples of 16 bytes.  A workgroup takes kRowKeyRows rows x 256 segments, a row at a
// time: 16-byte loads, all of a row's in flight at once (and the next row's while this one is
// added up, and the one after that); the row goes through LDS with the 16-byte words of segment s rotated by s, so
// that the threads of the second phase -- thread s owns segment s, as above, and adds from
// left to right -- read theirs without bank conflicts.  A thread's kRowKeyRows keys are
// neighbours in keys[]: they leave as 32-byte words.
constexpr int kRowKeyRows = 8;
typedef float vec4f __attribute__((ext_vector_type(4)));
template <int Q>
__global__ __launch_bounds__(256) void row_segment_keys_vec_kernel(const float *__restrict__ W, const int64_t ld,
                                                                     const uint32_t R, const uint32_t NBC,
                                                                     uint32_t *__restrict__ keys) {
    extern __shared__ vec4f tile4[];                // [256 segments][Q]
    const uint32_t tid = threadIdx.x;
    const uint32_t bj0 = blockIdx.x * 256u, i0 = blockIdx.y * kRowKeyRows;
    const uint32_t nseg = min(256u, NBC - bj0), nf = nseg * Q;
    const uint32_t nrows = min((uint32_t)kRowKeyRows, R - i0);
    const vec4f zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const float *const row0 = W + (size_t)i0 * ld + (size_t)bj0 * 4u * Q;
    vec4f v[2][Q];                                   // two rows ahead of the one being added up
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int u = 0; u < Q; ++u) {
            const uint32_t f = tid + 256u * u;
            v[a][u] = (uint32_t)a < nrows && f < nf ? ((const vec4f *)(row0 + (size_t)a * ld))[f] : zero4;
        }
    uint32_t mine[kRowKeyRows];
#pragma unroll
    for (int r = 0; r < kRowKeyRows; ++r) {
        mine[r] = 0u;
        if ((uint32_t)r >= nrows) continue;          // uniform
        if (r > 0) __syncthreads();                  // the previous row has been read
#pragma unroll
        for (int u = 0; u < Q; ++u) {
            const uint32_t f = tid + 256u * u, sg = f / Q, m = f % Q;
            tile4[sg * Q + ((m + sg) % Q)] = v[r & 1][u];
        }
        if ((uint32_t)r + 2 < nrows) {
            const vec4f *p = (const vec4f *)(row0 + (size_t)(r + 2) * ld);
#pragma unroll
            for (int u = 0; u < Q; ++u) {
                const uint32_t f = tid + 256u * u;
                v[r & 1][u] = f < nf ? p[f] : zero4;
            }
        }
        __syncthreads();
        float acc = 0.0f;
#pragma unroll
        for (int m = 0; m < Q; ++m) {
            const vec4f q = tile4[tid * Q + ((m + tid) % Q)];
            acc = fmaf(q.x, q.x, acc); acc = fmaf(q.y, q.y, acc); acc = fmaf(q.z, q.z, acc); acc = fmaf(q.w, q.w, acc);
        }
        mine[r] = rank_key(acc);
    }
    if (tid >= nseg) return;
    uint32_t *out = keys + (size_t)(bj0 + tid) * R + i0;
    if (nrows == kRowKeyRows && (R & 3u) == 0) {
#pragma unroll
        for (int r = 0; r < kRowKeyRows; r += 4) *(uint4 *)(out + r) = make_uint4(mine[r], mine[r + 1], mine[r + 2], mine[r + 3]);
    } else {
#pragma unroll
        for (int r = 0; r < kRowKeyRows; ++r)
            if ((uint32_t)r < nrows) out[r] = mine[r];
    }
}

// keys[bi * C + c] for column segment (bi, c) of the row-pruned matrix: thread per segment,
// c fastest (every row of the segment is read coalesced).
__global__ __launch_bounds__(256) void col_segment_keys_kernel(const float *__restrict__ W, const int64_t ld,
                                                                 const uint32_t R, const uint32_t C, const uint32_t BR,
                                                                 const uint32_t BC, const uint8_t *__restrict__ keep_r,
                                                                 uint32_t *__restrict__ keys) {
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x, bi = blockIdx.y;
    if (c >= C) return;
    const uint32_t r0 = bi * BR, r1 = min(R, r0 + BR);
    const uint8_t *kr = keep_r + (size_t)(c / BC) * R;
    float s = 0.0f;
    for (uint32_t i = r0; i < r1; ++i) {
        const float v = kr[i] ? W[(size_t)i * ld + c] : 0.0f;
        s = fmaf(v, v, s);
    }
    keys[(size_t)bi * C + c] = rank_key(s);
}

// The same for R and BR multiples of 8: the keep flags of eight rows come as one 8-byte word
// (the same word for all the lanes of a block-column), then the eight loads of the rows that
// survive are in flight together.  Row segments that were pruned are not read at all.
__global__ __launch_bounds__(256) void col_segment_keys_vec_kernel(const float *__restrict__ W, const int64_t ld,
                                                                     const uint32_t R, const uint32_t C, const uint32_t BR,
                                                                     const uint32_t BC, const uint8_t *__restrict__ keep_r,
                                                                     uint32_t *__restrict__ keys) {
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x, bi = blockIdx.y;
    if (c >= C) return;
    const uint32_t r0 = bi * BR, r1 = min(R, r0 + BR);
    const uint8_t *kr = keep_r + (size_t)(c / BC) * R;
    float s = 0.0f;
    uint32_t i = r0;
    for (; i + 32 <= r1; i += 32) {                          // 32 rows: their flags first, then all surviving loads at once
        const uint2 fa = *(const uint2 *)(kr + i), fb = *(const uint2 *)(kr + i + 8), fc = *(const uint2 *)(kr + i + 16),
                    fd = *(const uint2 *)(kr + i + 24);
        const uint32_t fw[8] = {fa.x, fa.y, fb.x, fb.y, fc.x, fc.y, fd.x, fd.y};
        float v[32];
#pragma unroll
        for (int q = 0; q < 32; ++q) v[q] = ((fw[q >> 2] >> (8 * (q & 3))) & 0xffu) ? W[(size_t)(i + q) * ld + c] : 0.0f;
#pragma unroll
        for (int q = 0; q < 32; ++q) s = fmaf(v[q], v[q], s);
    }
    for (; i < r1; i += 8) {
        const uint2 f = *(const uint2 *)(kr + i);
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t byte = ((q < 4 ? f.x : f.y) >> (8 * (q & 3))) & 0xffu;
            v[q] = byte ? W[(size_t)(i + q) * ld + c] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) s = fmaf(v[q], v[q], s);
    }
    keys[(size_t)bi * C + c] = rank_key(s);
}

// One workgroup ranks the n <= 16384 segments of one block-column (block-row) and marks the k
// weakest as pruned, "weaker" being the order of (key, position).  No sort: every thread keeps
// 16 consecutive keys in registers; the key T of the k-th weakest is found eight bits at a time
// from the highest bit on which the keys differ at all (a histogram of the digit over the keys
// that still match, by LDS atomics -- sums of squares of one block-column agree on their top
// exponent bits, and counting those would put every key into one bin -- then the digit whose
// bin holds the k-th); then a segment is pruned if its key is below T, or equal to T and fewer
// than (k - #below) equal keys lie at earlier positions.
constexpr int kSelPer = 16;          // keys per thread
__global__ __launch_bounds__(1024) void select_kernel(const uint32_t *__restrict__ keys, uint8_t *__restrict__ keep,
                                                       const uint32_t n, const uint32_t k) {
    __shared__ uint32_t wsum[3][16];
    __shared__ uint32_t hist[4][256];            // one histogram per digit
    __shared__ uint32_t pick[2];                 // the digit that holds the k-th, and k inside its bin
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const size_t base = (size_t)blockIdx.x * n;
    const uint32_t i0 = tid * kSelPer;
    if (k == 0 || k >= n) {                      // nothing / everything pruned
        for (uint32_t q = 0; q < kSelPer; ++q)
            if (i0 + q < n) keep[base + i0 + q] = k == 0 ? 1 : 0;
        return;
    }
    uint32_t key[kSelPer];
    bool valid[kSelPer];
    const bool vec = (n & 15u) == 0;             // 16-byte accesses: every thread's run is whole and aligned
#pragma unroll
    for (int q = 0; q < kSelPer; ++q) valid[q] = i0 + q < n;
    if (vec) {
        if (valid[0]) {
            const uint4 *src = (const uint4 *)(keys + base + i0);
#pragma unroll
            for (int v = 0; v < kSelPer / 4; ++v) {
                const uint4 w = src[v];
                key[4 * v] = w.x; key[4 * v + 1] = w.y; key[4 * v + 2] = w.z; key[4 * v + 3] = w.w;
            }
        } else {
#pragma unroll
            for (int q = 0; q < kSelPer; ++q) key[q] = 0u;
        }
    } else {
#pragma unroll
        for (int q = 0; q < kSelPer; ++q) key[q] = valid[q] ? keys[base + i0 + q] : 0u;
    }
    ((uint32_t *)hist)[tid] = 0u;                // 4 x 256 words, 1024 threads
    // bits on which every key agrees need no counting
    uint32_t all_and = 0xffffffffu, all_or = 0u;
#pragma unroll
    for (int q = 0; q < kSelPer; ++q)
        if (valid[q]) { all_and &= key[q]; all_or |= key[q]; }
    for (int d = 32; d > 0; d >>= 1) {
        all_and &= (uint32_t)__shfl_xor((int)all_and, d, 64);
        all_or |= (uint32_t)__shfl_xor((int)all_or, d, 64);
    }
    if (lane == 0) { wsum[1][wave] = all_and; wsum[2][wave] = all_or; }
    __syncthreads();
    for (int w = 0; w < 16; ++w) { all_and &= wsum[1][w]; all_or |= wsum[2][w]; }
    const uint32_t varying = all_and ^ all_or;
    const int top = varying ? 31 - __builtin_clz(varying) : -1;      // the highest bit on which keys differ
    // the kk-th weakest of the keys that match prefix on mask
    uint32_t mask = top < 0 ? 0xffffffffu : ~((2u << top) - 1u), prefix = all_and & mask, kk = k;
    int round = 0;
    for (int hi = top; hi >= 0; hi -= 8, ++round) {
        const int lo = hi >= 7 ? hi - 7 : 0;
        const uint32_t dmask = (2u << (hi - lo)) - 1u;
#pragma unroll
        for (int q = 0; q < kSelPer; ++q)
            if (valid[q] && (key[q] & mask) == prefix) atomicAdd(&hist[round][(key[q] >> lo) & dmask], 1u);
        __syncthreads();
        uint32_t h = 0, incl = 0;
        if (tid < 256) {                         // inclusive scan of the 256 bins
            h = hist[round][tid];
            incl = h;
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t up = (uint32_t)__shfl_up((int)incl, d, 64);
                if (lane >= (uint32_t)d) incl += up;
            }
            if (lane == 63) wsum[0][wave] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            for (uint32_t w = 0; w < wave; ++w) incl += wsum[0][w];
            const uint32_t excl = incl - h;
            if (excl < kk && kk <= incl) { pick[0] = tid; pick[1] = kk - excl; }
        }
        __syncthreads();                         // (pick and wsum[0] are next written behind two more barriers)
        prefix |= pick[0] << lo;
        mask |= dmask << lo;
        kk = pick[1];
    }
    // prefix is T; kk of the keys equal to T are pruned: the first ones by position
    uint32_t eq_wave = 0, eq_lower = 0;          // equal keys in the wavefront / in its lower lanes
#pragma unroll
    for (int q = 0; q < kSelPer; ++q) {
        const unsigned long long m = __ballot(valid[q] && key[q] == prefix);
        eq_wave += (uint32_t)__popcll(m);
        eq_lower += __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    }
    __syncthreads();                             // (wsum[0] is free: the scans' readers are behind their rounds' last barrier)
    if (lane == 0) wsum[0][wave] = eq_wave;
    __syncthreads();
    uint32_t rank = eq_lower;
    for (uint32_t w = 0; w < wave; ++w) rank += wsum[0][w];
    uint32_t flags[kSelPer / 4] = {};            // keep flags, one byte each
#pragma unroll
    for (int q = 0; q < kSelPer; ++q) {
        const bool eq = valid[q] && key[q] == prefix;
        const bool pruned = key[q] < prefix || (eq && rank < kk);
        rank += eq ? 1u : 0u;
        flags[q >> 2] |= (pruned ? 0u : 1u) << (8 * (q & 3));
        if (!vec && valid[q]) keep[base + i0 + q] = pruned ? 0 : 1;
    }
    if (vec && valid[0]) *(uint4 *)(keep + base + i0) = make_uint4(flags[0], flags[1], flags[2], flags[3]);
}

// Z = W where both its row segment and its column segment survive, else +0.  A thread takes
// four consecutive columns of one row (kMaskedCopyRows rows per workgroup).
constexpr int kMaskedCopyRows = 4;
__global__ __launch_bounds__(256) void masked_copy_kernel(const float *W, const int64_t ld, float *Z,
                                                            const int64_t ldz, const uint32_t R, const uint32_t C,
                                                            const uint32_t BR, const uint32_t BC,
                                                            const uint8_t *__restrict__ keep_r, const uint8_t *__restrict__ keep_c,
                                                            const bool vec4) {
    const uint32_t c = (blockIdx.x * 64u + (threadIdx.x & 63u)) * 4u;
    const uint32_t i = blockIdx.y * kMaskedCopyRows + (threadIdx.x >> 6);
    if (c >= C || i >= R) return;
    const uint8_t *kc = keep_c + (size_t)(i / BR) * C;
    if (vec4 && c + 3 < C) {
        const float4 w = *(const float4 *)(W + (size_t)i * ld + c);
        const uint32_t kc4 = *(const uint32_t *)(kc + c);           // four keep flags (C is a multiple of 4 here)
        float4 z;
        z.x = keep_r[(size_t)(c / BC) * R + i] && (kc4 & 0xffu) ? w.x : 0.0f;
        z.y = keep_r[(size_t)((c + 1) / BC) * R + i] && (kc4 & 0xff00u) ? w.y : 0.0f;
        z.z = keep_r[(size_t)((c + 2) / BC) * R + i] && (kc4 & 0xff0000u) ? w.z : 0.0f;
        z.w = keep_r[(size_t)((c + 3) / BC) * R + i] && (kc4 & 0xff000000u) ? w.w : 0.0f;
        *(float4 *)(Z + (size_t)i * ldz + c) = z;
    } else {
        for (uint32_t cc = c; cc < min(C, c + 4u); ++cc) {
            const bool on = keep_r[(size_t)(cc / BC) * R + i] && kc[cc];
            Z[(size_t)i * ldz + cc] = on ? W[(size_t)i * ld + cc] : 0.0f;
        }
    }
}

// The same for 16-byte aligned rows, C a multiple of 4 that BC divides into whole words (BC a
// multiple of 4), R and BR multiples of 8: a thread takes four columns of eight rows.  Its
// eight row flags are one 8-byte word, its four column flags one word; what does not survive
// is not read.
__global__ __launch_bounds__(256) void masked_copy_vec_kernel(const float *W, const int64_t ld, float *Z, const int64_t ldz,
                                                                const uint32_t R, const uint32_t C, const uint32_t BR,
                                                                const uint32_t BC, const uint8_t *__restrict__ keep_r,
                                                                const uint8_t *__restrict__ keep_c) {
    const uint32_t c = (blockIdx.x * 256u + threadIdx.x) * 4u;
    const uint32_t i0 = blockIdx.y * 8u;
    if (c >= C) return;
    const uint2 fr = *(const uint2 *)(keep_r + (size_t)(c / BC) * R + i0);
    const uint32_t kc4 = *(const uint32_t *)(keep_c + (size_t)(i0 / BR) * C + c);
    float4 w[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const uint32_t byte = ((q < 4 ? fr.x : fr.y) >> (8 * (q & 3))) & 0xffu;
        w[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (byte && kc4) w[q] = *(const float4 *)(W + (size_t)(i0 + q) * ld + c);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const uint32_t byte = ((q < 4 ? fr.x : fr.y) >> (8 * (q & 3))) & 0xffu;
        float4 z;
        z.x = byte && (kc4 & 0xffu) ? w[q].x : 0.0f;
        z.y = byte && (kc4 & 0xff00u) ? w[q].y : 0.0f;
        z.z = byte && (kc4 & 0xff0000u) ? w[q].z : 0.0f;
        z.w = byte && (kc4 & 0xff000000u) ? w[q].w : 0.0f;
        // (written once and not read again here: stores that do not stay behind in the caches -- with
        // ordinary stores the 256 MB of an 8192 x 8192 result were still on their way to memory when
        // the next call's first kernel read its input: 73 us for it instead of 45, and 56 instead of 43 here)
        __builtin_nontemporal_store(__builtin_bit_cast(vec4f, z), (vec4f *)(Z + (size_t)(i0 + q) * ldz + c));
    }
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct ProjectLayout {
    size_t keys_r, keep_r, keys_c, keep_c, total;
};

static ProjectLayout project_layout(int64_t R, int64_t C, int32_t br, int32_t bc) {
    const size_t nbr = (size_t)((R + br - 1) / br), nbc = (size_t)((C + bc - 1) / bc);
    ProjectLayout L{};
    size_t off = 0;
    L.keys_r = off; off = align256(off + nbc * (size_t)R * 4);
    L.keep_r = off; off = align256(off + nbc * (size_t)R);
    L.keys_c = off; off = align256(off + nbr * (size_t)C * 4);
    L.keep_c = off; off = align256(off + nbr * (size_t)C);
    L.total = off;
    return L;
}

// Segments zeroed among n at pruning rate `rate` x: floor(n (1 - rate^-1/2) + 1/2).
static uint32_t prune_count(int64_t n, double rate) {
    const double q = 1.0 - 1.0 / std::sqrt(rate);
    int64_t k = (int64_t)std::floor((double)n * q + 0.5);
    if (k < 0) k = 0;
    if (k > n) k = n;
    return (uint32_t)k;
}


}  // namespace csb

extern "C" size_t csb_project_workspace_bytes(int64_t rows, int64_t cols, int32_t br, int32_t bc) {
    if (rows <= 0 || cols <= 0 || br < 1 || bc < 1) return 0;
    return csb::project_layout(rows, cols, br, bc).total;
}

extern "C" int csb_project(const float *d_W, int64_t rows, int64_t cols, int64_t ld, int32_t br, int32_t bc,
                           double rate, float *d_Z, int64_t ldz, void *d_ws, void *stream) {
    using namespace csb;
    if (!d_W || !d_Z || !d_ws) { set_error("csb_project: NULL pointer"); return CSB_EINVAL; }
    if ((uintptr_t)d_ws % 256) { set_error("csb_project: workspace not 256-byte aligned"); return CSB_EINVAL; }
    if (rows <= 0 || cols <= 0 || ld < cols || ldz < cols) { set_error("csb_project: bad shape or leading dimension"); return CSB_EINVAL; }
    if (br < 1 || br > CSB_MAX_BLOCK || bc < 1 || bc > CSB_MAX_BLOCK) { set_error("csb_project: block size outside [1, 256]"); return CSB_EINVAL; }
    if (!(rate >= 1.0) || !std::isfinite(rate)) { set_error("csb_project: pruning rate must be a finite number >= 1"); return CSB_EINVAL; }
    if (rows > kProjectMaxDim || cols > kProjectMaxDim) {
        set_error("csb_project: more than 16384 rows or columns (one workgroup ranks a block-column in LDS)");
        return CSB_EUNSUPPORTED;
    }
    static const char project_user = 0;                    // this entry point as a user of workspaces
    workspace_changed_hands(d_ws, &project_user);
    const uint32_t R = (uint32_t)rows, C = (uint32_t)cols, BR = (uint32_t)br, BC = (uint32_t)bc;
    const uint32_t NBR = (R + BR - 1) / BR, NBC = (C + BC - 1) / BC;
    const ProjectLayout L = project_layout(rows, cols, br, bc);
    uint8_t *ws = (uint8_t *)d_ws;
    uint32_t *keys_r = (uint32_t *)(ws + L.keys_r), *keys_c = (uint32_t *)(ws + L.keys_c);
    uint8_t *keep_r = ws + L.keep_r, *keep_c = ws + L.keep_c;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    {
        // tile of the row-sum kernel: TS segments x TR rows, at most 256 threads and 48 KB of LDS
        const uint32_t BCp = BC | 1u;
        const uint32_t TS = std::max(1u, std::min({NBC, 256u, 12288u / BCp}));
        const uint32_t TR = std::max(1u, std::min({256u / TS, 12288u / (TS * BCp), R}));
        const size_t lds_rows = (size_t)TR * TS * BCp * sizeof(float);
        const dim3 grid_r((NBC + TS - 1) / TS, (R + TR - 1) / TR);
        // 16-byte accesses need 16-byte aligned rows on both sides (and flag words at multiples of 4)
        const bool vec4 = C % 4 == 0 && ld % 4 == 0 && ldz % 4 == 0 && (uintptr_t)d_W % 16 == 0 && (uintptr_t)d_Z % 16 == 0;
        const bool rows8 = R % 8 == 0 && BR % 8 == 0;
        int shift = -1;
        for (int b = 0; b < 9; ++b) if (BC == (1u << b)) shift = b;
        if (vec4 && C % BC == 0 && shift >= 4 && shift <= 6) {
            const dim3 grid_v((NBC + 255) / 256, (R + kRowKeyRows - 1) / kRowKeyRows);
            const size_t lds_v = (size_t)256 * BC * sizeof(float);
            switch (shift) {
                case 4: hipLaunchKernelGGL(row_segment_keys_vec_kernel<4>, grid_v, dim3(256), lds_v, st, d_W, ld, R, NBC, keys_r); break;
                case 5: hipLaunchKernelGGL(row_segment_keys_vec_kernel<8>, grid_v, dim3(256), lds_v, st, d_W, ld, R, NBC, keys_r); break;
                default: hipLaunchKernelGGL(row_segment_keys_vec_kernel<16>, grid_v, dim3(256), lds_v, st, d_W, ld, R, NBC, keys_r); break;
            }
        } else {
            switch (shift) {
                case 4: hipLaunchKernelGGL(row_segment_keys_kernel<4>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
                case 5: hipLaunchKernelGGL(row_segment_keys_kernel<5>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
                case 6: hipLaunchKernelGGL(row_segment_keys_kernel<6>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
                default: hipLaunchKernelGGL(row_segment_keys_kernel<-1>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
            }
        }
        hipLaunchKernelGGL(select_kernel, dim3(NBC), dim3(1024), 0, st, keys_r, keep_r, R, prune_count(rows, rate));
        if (rows8)
            hipLaunchKernelGGL(col_segment_keys_vec_kernel, dim3((C + 255) / 256, NBR), dim3(256), 0, st, d_W, ld, R, C, BR, BC, keep_r, keys_c);
        else
            hipLaunchKernelGGL(col_segment_keys_kernel, dim3((C + 255) / 256, NBR), dim3(256), 0, st, d_W, ld, R, C, BR, BC, keep_r, keys_c);
        hipLaunchKernelGGL(select_kernel, dim3(NBR), dim3(1024), 0, st, keys_c, keep_c, C, prune_count(cols, rate));
        if (vec4 && rows8 && BC % 4 == 0)
            hipLaunchKernelGGL(masked_copy_vec_kernel, dim3((C + 1023) / 1024, R / 8), dim3(256), 0, st,
                               d_W, ld, d_Z, ldz, R, C, BR, BC, keep_r, keep_c);
        else
            hipLaunchKernelGGL(masked_copy_kernel, dim3((C + 255) / 256, (R + kMaskedCopyRows - 1) / kMaskedCopyRows), dim3(256), 0, st,
                               d_W, ld, d_Z, ldz, R, C, BR, BC, keep_r, keep_c, vec4);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { set_error(std::string("csb_project: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}
