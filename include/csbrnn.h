/*
 * csbrnn.h -- C ABI of the MI355X (gfx950) CSB-RNN inference library.
 *
 * The library applies a CSB-pruned weight matrix (compressed structured blocks, paper
 * Sec. 3.1.1) to vectors and runs LSTM / GRU inference with it (Sec. 2.1, Sec. 4.3.1).
 *
 * Conventions
 *   - Every function returns an int status (CSB_OK = 0, negative on error) unless it
 *     returns a size or a string.  csb_last_error() gives a thread-local message for the
 *     last failing call on this thread.  Bad arguments never crash: they return
 *     CSB_EINVAL.
 *   - "host" pointers are ordinary CPU memory; "device" pointers (prefix d_) are HIP
 *     device memory owned by the caller.  The library never allocates device memory:
 *     callers ask for sizes (csb_device_bytes, csb_workspace_bytes,
 *     csb_rnn_workspace_bytes) and pass buffers in.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device
 *     calls only enqueue work on that stream and do not synchronise with the host.
 *   - Handles (csb_matrix, csb_rnn) are host objects owned by the library; release them
 *     with csb_free / csb_rnn_free.  A csb_rnn borrows its csb_matrix handles and bias
 *     pointers; they must outlive it.
 *   - All matrices are float32.  A matrix is rows x cols, tiled in br x bc blocks (edge
 *     blocks are truncated); blocks are numbered row-major, b = bi * nbc + bj.
 *   - Calls that use the same csb_matrix (or csb_rnn) concurrently on different streams
 *     race on its device-side merge counters: order them on one stream.
 */
#ifndef CSBRNN_H
#define CSBRNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CSB_OK 0
#define CSB_EINVAL (-1)       /* bad argument (NULL, non-positive size, out of range)   */
#define CSB_ENOMEM (-2)       /* host allocation failed or a caller buffer is too small */
#define CSB_EDEVICE (-3)      /* a HIP call failed                                      */
#define CSB_EUNSUPPORTED (-4) /* valid request outside what the kernels cover           */
#define CSB_ESTATE (-5)       /* call order wrong (e.g. spmv before plan/upload)        */

#define CSB_CELL_LSTM 0
#define CSB_CELL_GRU 1
#define CSB_CELL_LSTMP 2     /* LSTM with a recurrent projection; created by csb_rnn_create_lstmp */
#define CSB_CELL_LIGRU 3     /* Li-GRU: update gate and ReLU candidate, rows z,c               */
#define CSB_CELL_GRU_RB 4    /* GRU, reset gate before the product; created by csb_rnn_create_gru_rb */

#define CSB_VAL_F32 0         /* kernel values stored as binary32 (default)               */
#define CSB_VAL_F16 1         /* ... as IEEE binary16                                     */
#define CSB_VAL_BF16 2        /* ... as bfloat16 (upper half of binary32)                 */

#define CSB_MAX_BLOCK 256     /* br, bc in [1, 256]: device indices are one byte */

typedef struct csb_matrix csb_matrix;
typedef struct csb_rnn csb_rnn;

/*
 * Canonical view of the five CSB arrays of Sec. 3.1.1 (row/column counts of the kernel
 * matrix per block; indices of the surviving rows and columns; kernel values of
 * successive blocks concatenated) plus exclusive prefix sums, which the paper omits
 * because its engine reads the arrays sequentially.  Indices are block-local and
 * ascending; a kernel is stored row-major; blocks follow in row-major order.
 * All pointers are host memory owned by the csb_matrix and valid until csb_free.
 */
typedef struct {
    int64_t rows, cols;
    int32_t br, bc, nbr, nbc;
    int64_t nnz, n_rowidx, n_colidx;
    const int32_t *nrows, *ncols;               /* [nbr*nbc]            */
    const uint16_t *rowidx, *colidx;            /* [n_rowidx],[n_colidx] */
    const float *val;                           /* [nnz]                */
    const int64_t *val_off, *row_off, *col_off; /* [nbr*nbc + 1]        */
} csb_view;

/*
 * Result of the equal-work partition (the role Sec. 5.2 gives to the micro-instruction
 * compiler: split the uneven kernel-matrix work so that every parallel unit gets the same
 * amount).  Work is counted in wavefront steps: one step is one 64-lane multiply-add
 * issue plus a fixed per-group overhead, which is what a wavefront's run time follows.
 */
typedef struct {
    int32_t n_chunks;        /* workgroups the kernels will launch                      */
    int32_t waves_per_chunk; /* wavefronts per workgroup                                */
    int32_t n_groups;        /* wavefront-sized groups of kernel-matrix rows            */
    int32_t n_shared_tiles;  /* output row tiles whose sum is merged across workgroups   */
    double work_max;         /* largest work assigned to one wavefront (steps)          */
    double work_mean;        /* mean work per wavefront (steps)                         */
    double lane_fill;        /* nnz / (64 * multiply-add steps): useful lanes per issue */
    double nosplit_max_over_mean; /* the same ratio when whole blocks are dealt out
                                round-robin with no splitting (the "no sharing" baseline
                                of Sec. 6.3.2), for context                             */
    double chunk_max_over_mean;   /* largest / mean work per workgroup                   */
    int32_t whole_tiles;     /* 1: every workgroup owns whole output row tiles (no merge) */
    int32_t row_owned;       /* 1: csb_spmv runs the row-owned layout (below); the figures above
                                then describe that layout.  2: the same layout with every
                                workgroup owning whole units of a recurrent cell (all their
                                gate rows), which csb_rnn_create* give their matrices: the
                                streaming step reads it, csb_spmv the tile sections       */
    int32_t rounds;          /* row-owned layout: rounds per workgroup                   */
    int32_t reserved;
    int64_t matvec_bytes;    /* bytes of the device image one csb_spmv launch reads      */
} csb_plan_stats;

const char *csb_last_error(void);

/*
 * CSB encoding, Sec. 3.1.1.  HOST ONLY.
 * dense: host, row-major, leading dimension ld >= cols.  An entry survives iff
 * v != 0.0f (so -0.0 is pruned, NaN is kept).  In each block the surviving rows
 * (columns) are those with at least one surviving entry in the block; the kernel is the
 * sub-matrix at their cross-points, explicit zeros included.
 * *out receives a new handle.  Errors: NULL pointers, rows/cols <= 0, br/bc outside
 * [1, CSB_MAX_BLOCK], ld < cols -> CSB_EINVAL; allocation failure -> CSB_ENOMEM.
 */
int csb_pack(const float *dense, int64_t rows, int64_t cols, int64_t ld,
             int32_t br, int32_t bc, csb_matrix **out);

/* Borrow the canonical arrays (host pointers, valid until csb_free). */
int csb_view_get(const csb_matrix *m, csb_view *out);

/* Inverse of csb_pack: writes all rows x cols entries of `dense` (host, ld >= cols). */
int csb_unpack(const csb_matrix *m, float *dense, int64_t ld);

/*
 * 16-bit weights (the paper evaluates its engine with weights quantised to 16 bits,
 * Sec. 6.2.2 / 6.3.1; here the two 16-bit floating-point formats of the target take the
 * place of its fixed-point format).  HOST ONLY.  Rounds every stored kernel value to the
 * nearest value of the format (ties to even; binary16 overflows to infinity and underflows
 * gradually; NaN stays NaN), so that csb_view_get / csb_unpack show the weights every device
 * path computes with, and makes csb_plan store the value stream in 16 bits: csb_spmv and
 * csb_spmm then read half the bytes per kernel value and widen to binary32 in registers;
 * sums are accumulated in binary32 as before.  A value rounded to zero stays a stored
 * (explicit) zero.  Any plan and upload of the matrix become invalid: plan and upload again.
 * CSB_VAL_F32 only switches the stream back to 32 bits (values already rounded stay rounded).
 * Call it before csb_rnn_create* takes the matrix: the resident layout of an RNN copies the
 * values it finds at creation (it keeps them in binary32 registers, rounded or not).
 * Errors: NULL handle or unknown format -> CSB_EINVAL.
 */
int csb_set_value_format(csb_matrix *m, int32_t format);

/* The value format of the matrix (CSB_VAL_*), or -1 for a NULL handle. */
int csb_value_format(const csb_matrix *m);

/*
 * Equal-work partition and device layout (host only; replaces the SMT-based schedule of
 * Sec. 5.2.2 by a prefix sum).  Kernel-matrix rows of one block-row are packed into
 * 64-lane groups, the groups' multiply-add steps are prefix-summed, and the sum is cut
 * into n_chunks * waves_per_chunk equal ranges, one per wavefront; a cut may fall inside
 * a group (between two of its column steps).  n_chunks = 0 picks a default for one
 * MI355X.  May be called again to re-plan; the matrix must then be uploaded again.
 * stats may be NULL.
 * Errors: NULL / negative n_chunks -> CSB_EINVAL; more than 16383 columns (the device
 * layout addresses the staged input vector with 16-bit byte offsets) or 2^32 stored
 * values -> CSB_EUNSUPPORTED; allocation failure -> CSB_ENOMEM.
 */
int csb_plan(csb_matrix *m, int32_t n_chunks, csb_plan_stats *stats);

/*
 * csb_plan with the partition mode spelled out.  mode 0: as csb_plan (whole tiles when
 * there are at least as many row tiles with work as workgroups wanted, else equal split);
 * mode 1: workgroups own whole output row tiles (contiguous tile ranges of nearly equal
 * work; no cross-workgroup merge; CSB_EUNSUPPORTED if one tile exceeds a workgroup's LDS);
 * mode 2: equal-work split at step granularity, tiles that straddle a cut are merged by
 * the last workgroup to arrive.  Inside a workgroup both modes split the steps equally
 * over the 16 wavefronts.
 */
int csb_plan_ex(csb_matrix *m, int32_t n_chunks, int32_t mode, csb_plan_stats *stats);
/* A matrix that csb_rnn_create has planned for a GRU (its n rows' input-side and recurrent-side
 * sums kept apart, the layout the step kernels of that handle read) keeps this row layout when
 * csb_plan / csb_plan_ex plan it again, also after csb_set_value_format: only the workgroup
 * count and the mode change.  csb_rnn_create in turn keeps the workgroup count and mode of a
 * plan the caller made before.  csb_rnn_forward refuses (CSB_ESTATE) a weight matrix whose row
 * layout is no longer the one its handle planned (e.g. after csb_plan_rows). */

/*
 * The row-owned layout of the mat-vec (Sec. 4.3.1 / the equal-work role of Sec. 5.2), which
 * csb_plan and csb_plan_ex(mode 0) build next to the tile-based sections whenever the matrix
 * fits it: at most 16383 columns (kernel values in any of the three storage formats; a
 * matrix planned for a GRU step is laid out with the row split of that step).  Every
 * workgroup owns a contiguous range of at most 256 output rows (ranges of nearly equal
 * stored bytes, cut at any row), so no sum crosses workgroups and nothing is merged.  The
 * kernel-matrix rows that land in a range are sorted by column count, packed 64 to a group
 * (one per lane), and the groups' column steps are cut into equal ranges, one per wavefront
 * and round; a wavefront's share of a round is stored as ONE self-contained segment of a
 * fixed size (8-bit column indices, column-major kernel values, no padding of the values),
 * so a launch requests all of its bytes at once from addresses that depend only on the
 * workgroup and wavefront numbers.  Row sums are formed in a fixed order (bitwise
 * reproducible).  csb_spmv and the per-step launches of csb_rnn_forward's streaming path read
 * this section when it exists; csb_spmm keeps reading the tile-based sections.
 * csb_plan_rows plans like csb_plan with the parameters of this layout spelled out:
 * n_workgroups (0 = default: one per 256 kernel-matrix rows, at most 256, at least
 * rows / 256) and min_rounds (0 or 1 = as few rounds as the LDS allows; more rounds make
 * the segments shorter).  Errors as csb_plan; CSB_EUNSUPPORTED if the matrix does not fit
 * the layout.
 */
int csb_plan_rows(csb_matrix *m, int32_t n_workgroups, int32_t min_rounds, csb_plan_stats *stats);

/* The statistics of the matrix's current plan (what csb_plan* returned, or what a csb_rnn_create*
 * call planned).  Errors: NULL -> CSB_EINVAL; not planned -> CSB_ESTATE. */
int csb_plan_stats_get(const csb_matrix *m, csb_plan_stats *stats);

/* Integer self-check of the planned device image: every offset in bounds, every kernel
 * value referenced exactly once, image decodes to the packed matrix.  Host only. */
int csb_plan_validate(const csb_matrix *m);

/* Bytes of device memory the planned matrix needs (0 if not planned). */
size_t csb_device_bytes(const csb_matrix *m);

/*
 * Copy the planned image into d_buf (device, caller-owned, >= csb_device_bytes bytes,
 * 256-byte aligned, must stay valid and otherwise untouched while the matrix is in use).
 * Asynchronous on `stream` from a staging copy kept inside the handle.
 */
int csb_upload(csb_matrix *m, void *d_buf, size_t bytes, void *stream);

/* Bytes of scratch csb_spmv / csb_spmm need for `batch` right-hand sides (partial sums of
 * row tiles that several workgroups share).  Contents need no initialisation.
 * Workspaces in general (this one, csb_rnn_forward's, csb_project's): 256-byte aligned (else
 * CSB_EINVAL); a buffer may be handed to
 * different handles and entry points in turn, never to two calls that overlap in time.  The
 * library identifies a workspace by its base address and clears the words that workgroups
 * exchange through it whenever another handle or entry point has used the buffer in between;
 * writing into a workspace yourself between two calls on the same handle is not allowed. */
size_t csb_workspace_bytes(const csb_matrix *m, int32_t batch);

/*
 * CSB-MVM, Sec. 4.3.1: y = A x.  d_x [cols], d_y [rows] device float32; d_ws device
 * scratch of csb_workspace_bytes(m, 1) (may be NULL if that is 0).  Every y entry is
 * written (rows without survivors get 0).  Results are bitwise reproducible run to run.
 * On a row-owned plan (what csb_plan makes by default) the call is one kernel launch and
 * nothing else, and may be captured into a HIP graph.
 * Errors: NULL -> CSB_EINVAL; not planned/uploaded -> CSB_ESTATE; launch failure ->
 * CSB_EDEVICE.
 */
int csb_spmv(const csb_matrix *m, const float *d_x, float *d_y, void *d_ws, void *stream);

/*
 * csb_spmv for callers that cannot allocate device memory or pass a workspace along (code
 * under HIP graph capture set-up, tight serving loops, harnesses that forbid hipMalloc): the
 * same kernels and the same result as csb_spmv, bit for bit, but the partial sums of row tiles
 * that several workgroups share go through a buffer built into the library (a file-scope
 * device array of csb_spmv_static_limit() bytes = 1 MiB, which every GPU the library runs on
 * holds until the process ends) instead of a caller's workspace.  The call allocates nothing.
 * A matrix whose plan needs more (csb_workspace_bytes(m, 1) above the limit) is refused with
 * CSB_EUNSUPPORTED; plans in the row-owned layout need no such memory and always pass.
 * All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (other
 * streams, other threads) race on it -- order them on one stream.  The merge words in it are
 * tagged per launch, so contents left by earlier calls, for this or another matrix, do no harm.
 * Errors otherwise as csb_spmv; a failing hipGetSymbolAddress -> CSB_EDEVICE.
 */
/*
 * Merges of row tiles that several workgroups share wait for each other's partial sums with a
 * bounded number of polls; a merge that gives up stores NaN in its rows and sets a word in the
 * matrix image.  csb_status reads that word (it synchronises `stream`), clears it, and returns
 * it in *timed_out: non-zero means some csb_spmv / csb_spmm result since the last check holds
 * NaNs for this reason (workgroups of one launch not all running at once).  Plans in the
 * row-owned layout merge nothing and never set it.
 */
int csb_status(const csb_matrix *m, void *stream, int32_t *timed_out);

size_t csb_spmv_static_limit(void);
int csb_spmv_static(const csb_matrix *m, const float *d_x, float *d_y, void *stream);

/*
 * Batched CSB-MVM: Y = A X for `batch` right-hand sides.  d_X is [cols][ldx] (entry
 * (j,k) at d_X[j*ldx + k], ldx >= batch), d_Y is [rows][ldy] (ldy >= batch).
 * d_ws: csb_workspace_bytes(m, batch) (may be NULL when that is 0).  Runs on the matrix
 * cores (fp32 MFMA); the result does not depend on timing (fixed summation order).
 * Errors: NULL / batch <= 0 / a leading dimension below batch -> CSB_EINVAL; not planned
 * or uploaded, or planned for a GRU step -> CSB_ESTATE; cols * ldx beyond 2^30 elements
 * or ldx >= 2^24 (the kernel uses 32-bit element offsets) -> CSB_EUNSUPPORTED; launch
 * failure -> CSB_EDEVICE.
 */
int csb_spmm(const csb_matrix *m, const float *d_X, int64_t ldx, float *d_Y, int64_t ldy,
             int32_t batch, void *d_ws, void *stream);

/*
 * Batched CSB-MVM with bfloat16 operands on the matrix cores (the 16-bit datapath of
 * Sec. 6.3.1 taken to the batched product): the matrix stores bfloat16 values
 * (csb_set_value_format(CSB_VAL_BF16) before csb_plan) and the right-hand sides arrive as
 * bfloat16 bit patterns, d_Xb [cols][ldx] (device, entry (j,k) at d_Xb[j*ldx + k]); the
 * products are exact in binary32 and are accumulated in binary32 into d_Y [rows][ldy] float.
 * Y equals A X for the rounded operands to the float32 dot-product bound of csb_spmm.
 * Errors: NULL / batch <= 0 / a leading dimension below batch -> CSB_EINVAL; matrix not
 * planned and uploaded, planned for a GRU step, or not storing bfloat16 -> CSB_ESTATE; batch or
 * ldx not a multiple of 4, d_Xb not 8-byte aligned, block rows too tall for the accumulator
 * tiles -> CSB_EUNSUPPORTED.  Needs no workspace; runs on `stream` without host
 * synchronisation.
 */
int csb_spmm_bfloat(const csb_matrix *m, const uint16_t *d_Xb, int64_t ldx, float *d_Y, int64_t ldy,
                    int32_t batch, void *stream);
/* The same with IEEE binary16 operands (matrix: CSB_VAL_F16; d_Xh: binary16 bit patterns):
 * products of two binary16 numbers are exact in binary32 too.  Same layout, bound and errors. */
int csb_spmm_half(const csb_matrix *m, const uint16_t *d_Xh, int64_t ldx, float *d_Y, int64_t ldy,
                  int32_t batch, void *stream);

/*
 * Model of the paper's own schedule, for context next to csb_plan's statistics.  HOST ONLY,
 * no device work, not on any compute path.  The paper's engine (Sec. 4.3) runs K x L blocks
 * per block iteration on K x L PEGroups of P x Q PEs; an a x b partition of a kernel matrix
 * takes ceil(a/P) ceil(b/Q) cycles on a PEGroup; an iteration lasts as long as its most loaded
 * PEGroup; efficiency = multiply-adds / (P Q K L cycles) (Sec. 6.3.2).  With workload sharing
 * (Sec. 4.3.2, 5.2.2) PEGroup (k,l) hands dnh of its columns to (k, l+1) and / or dmv of its
 * rows (at most half) to (k+1, l), torus-wise, in one of the two regular shapes of the
 * partition constraints of Sec. 5.2.2; shares are multiples of Q and P.  The paper finds a
 * schedule per iteration with an SMT solver and a growing margin around the mean load; this
 * model takes the schedule with the smallest largest load instead: exactly (exhaustive search)
 * for horizontal-only and vertical-only sharing, and for 2-D sharing on grids of at most four
 * PEGroups (K L <= 4; exact_2d = 1).  On larger grids, and when an iteration of a small grid
 * has more than 2^27 combinations, the 2-D schedule is found by improving one PEGroup's choice
 * at a time from the better one-directional schedule (exact_2d = 0): eff_2d is then a lower
 * bound on what the best 2-D schedule reaches, checked against brute force only as a bound
 * (never below the optimum's time, never above the one-directional ones).  The paper's
 * evaluation uses P = Q = K = L = 4, which is such a grid.
 * Errors: NULL pointers, P, Q < 1, K, L outside [1, 8] -> CSB_EINVAL.
 */
typedef struct {
    int64_t work;                 /* multiply-adds: sum of r_b c_b                           */
    int64_t iterations;           /* block iterations: ceil(nbr / K) ceil(nbc / L)             */
    int64_t cycles_none, cycles_horizontal, cycles_vertical, cycles_2d;
    double eff_none, eff_horizontal, eff_vertical, eff_2d;
    int32_t exact_2d;             /* 1: cycles_2d is the optimum; 0: an upper bound on it      */
    int32_t reserved;
} csb_sharing_stats;
int csb_sharing_model(const csb_matrix *m, int32_t P, int32_t Q, int32_t K, int32_t L,
                      csb_sharing_stats *out);

/*
 * RNN handle (Sec. 2.1).  cell: CSB_CELL_LSTM (gate rows stacked i,f,g,o; no peepholes),
 * CSB_CELL_GRU (rows r,z,n; the reset gate multiplies the recurrent product of the n
 * rows) or CSB_CELL_LIGRU (the cell of the paper's speech model SR3, Table 1, as its
 * authors published it, the batch normalisation of the input part folded into W and the
 * bias as it is at inference; rows z,c: z = sigmoid(a_z), cand = max(a_c, 0),
 * h_t = z h_(t-1) + (1 - z) cand; G = 2).  Layer l has W[l] of shape (G*hidden) x (in_l + hidden), in_0 = input,
 * in_l = hidden, applied to [layer input ; h_{l,t-1}], and an optional device bias
 * d_bias[l] of G*hidden floats (d_bias NULL or d_bias[l] NULL = zero bias).
 * Each W[l] must be packed; it is planned by this call if it is not yet, in the layout
 * the step kernels need (the GRU keeps the input-side and recurrent-side sums of its n
 * rows apart; a workgroup of the row-owned layout owns whole units with all their gate rows,
 * so that a step of the streaming path is one launch that finishes its cells --
 * csb_plan_stats.row_owned = 2; in a model of several layers, whose products share launches, a
 * matrix is laid out for its share of the compute units: at most 256 / min(n_layers, 4)
 * workgroups; csb_plan* on the matrix afterwards plans plain row ranges for all compute units
 * again, which the step kernels run on as well, computing a cell where its output is consumed).
 * Upload each W[l] afterwards with csb_upload.
 */
int csb_rnn_create(int32_t cell, int32_t n_layers, int32_t input, int32_t hidden,
                   csb_matrix *const *W, const float *const *d_bias, csb_rnn **out);

/*
 * LSTM with a recurrent projection (LSTMP: the cell of the paper's speech model SR1,
 * Table 1; the paper names the cell and gives no equations, so this is the cell as its
 * authors published it).  Per layer: a = W [u ; r_(t-1)] + b with rows i,f,g,o as for the
 * LSTM, c_t = f c_(t-1) + i g, m_t = o tanh(c_t) (hidden wide), and r_t = Wp m_t (proj wide,
 * no bias, no non-linearity); r_t is the recurrent state and the next layer's input.
 * W[l]: (4*hidden) x (in_l + proj) with in_0 = input, in_l = proj; Wp[l]: proj x hidden; both
 * packed, planned by this call if they are not yet.  Upload every W[l] and Wp[l] with
 * csb_upload.  In csb_rnn_forward the state h (d_h0, d_hT, d_hseq) is proj wide and the cell
 * state c (d_c0, d_cT) hidden wide.  Batch 1 with the resident layout uploaded
 * (csb_rnn_upload): one kernel launch for the whole sequence, the gate rows and the
 * projection rows of a layer being two stages that hand m_t and r_t to each other; else the
 * streaming paths (two CSB products per step and layer; batch > 1 on the matrix cores, with
 * an element-wise kernel between them).  Errors as csb_rnn_create.
 */
int csb_rnn_create_lstmp(int32_t n_layers, int32_t input, int32_t hidden, int32_t proj,
                         csb_matrix *const *W, csb_matrix *const *Wp, const float *const *d_bias,
                         csb_rnn **out);

/*
 * GRU with the reset gate applied BEFORE the recurrent product of the candidate, the form
 * of the work the paper cites for the GRU (Sec. 2.1): r, z as for CSB_CELL_GRU, then
 * n = tanh(Wn u + Un (r * h_(t-1)) + b_n), h_t = (1 - z) n + z h_(t-1).  The candidate's
 * recurrent product needs every r first, so a step is two dependent CSB products, and the
 * caller hands the weights over in two matrices per layer:
 *   Wa[l]: (3*hidden) x (in_l + hidden), rows r,z,n, in which the n rows hold their
 *          input-side entries only (a non-zero in an n row at a recurrent column:
 *          CSB_EINVAL);
 *   Un[l]: hidden x hidden, the recurrent side of the n rows.
 * Both packed; planned by this call if they are not yet; upload both with csb_upload.
 * d_bias[l]: 3*hidden floats (r,z,n) or NULL.  Batch 1 with the resident layout uploaded
 * (csb_rnn_upload): one kernel launch for the whole sequence, a layer being a reset stage
 * (row r, output r * h_(t-1)) and a gate stage (rows z and n, the latter over the layer input
 * and the reset stage's output of the same step); else the streaming paths: per step two
 * CSB product launches that do the element-wise parts themselves at batch 1 (on plans whose
 * workgroups own whole units, as csb_rnn_create makes them), two products and two
 * element-wise kernels on the matrix cores at batch > 1.
 * Errors as csb_rnn_create.
 */
int csb_rnn_create_gru_rb(int32_t n_layers, int32_t input, int32_t hidden,
                          csb_matrix *const *Wa, csb_matrix *const *Un, const float *const *d_bias,
                          csb_rnn **out);

/*
 * Resident layout of the whole model for batch-1 inference: every row's surviving weights
 * cut into equal slices, one slice per lane, kept in registers for the whole sequence (the
 * equal-work split of Sec. 5.2 applied to on-chip storage).  csb_rnn_device_bytes is 0 if
 * the model does not fit on chip (more than 8 layers, more than 224 workgroups' worth of weights, a layer input
 * wider than 2048, or a stage whose inputs together are wider than 3072).  After csb_rnn_upload (d_buf device, caller-owned,
 * 256-byte aligned, >= csb_rnn_device_bytes, valid while the handle is used) csb_rnn_forward
 * with batch 1 runs all timesteps of all layers in ONE kernel launch.  A batch can run there
 * too: its sequences are independent, so a model that leaves XCDs free runs them as instances
 * of itself side by side (8 / XCDs-per-instance of them per launch; a model of at most half
 * an XCD several per XCD), the batch in rounds of that many.  Without the resident layout
 * csb_rnn_forward launches CSB products step by step and needs every W[l] uploaded: stacked
 * layers run by diagonals (layer l at step t with l + t constant are independent and share a
 * launch); at batch 1 nothing else is launched -- the gates of a step are computed by the
 * products that consume its output -- and at batch > 1 (the products on the matrix cores) one
 * element-wise kernel follows each product launch.  With both uploaded, batch 1 takes the
 * resident kernel and a larger batch whichever an estimate of the time per step favours
 * (rounds of the resident kernel against the batched products' launches per diagonal).
 * The resident kernel's workgroups wait for each other's h_t: they must all be on the GPU at
 * once, so nothing else should occupy the device while it runs.  The workgroups are placed on
 * as few of the 8 XCDs as hold them (at most 28 per XCD, one per CU).
 * Development knobs (NOT part of the interface: they exist for the experiments behind the
 * defaults, which are the measured best, and may go away), read from the environment ONCE, by
 * csb_rnn_create*: CSB_RNN_S = slots per lane of the resident layout (multiple
 * of 4), CSB_RNN_XCDS = use at least this many XCDs, CSB_RNN_POLL_DELAY = sleeps before the
 * first poll of a step, CSB_RNN_BATCH_PATH = "resident" or "batched": the path of a batch when
 * both are uploaded, CSB_RNN_GRAPH = 0: csb_rnn_forward never records its launches (below).
 */
typedef struct {
    int32_t resident;          /* 1 if a resident layout exists                            */
    int32_t n_workgroups;      /* workgroups (all layers)                                  */
    int32_t slots_per_lane;    /* multiply-adds every lane issues per step (largest layer) */
    int32_t reserved;          /* (diagnostic) words left sharing an LDS bank within a 32-lane gather */
    double slot_fill;          /* non-zeros / issued multiply-adds (1 = no padding)        */
    double lanes_max_over_mean;/* largest / mean number of busy lanes per workgroup        */
} csb_rnn_plan_stats;
size_t csb_rnn_device_bytes(const csb_rnn *r);
int csb_rnn_upload(csb_rnn *r, void *d_buf, size_t bytes, void *stream);
/* Lay the resident kernel out for batches of `batch` sequences (host only; the equal-work
 * split of Sec. 5.2 with another slice length).  csb_rnn_create* lays it out for ONE
 * sequence: few slots per lane, the shortest step.  More slots per lane make an instance
 * smaller, so that more of them run side by side and the batch takes fewer rounds, at a longer
 * step: this call takes the slot count with the smallest estimated time for `batch` (batch 1
 * gives the layout of create back).  The handle is no longer uploaded afterwards:
 * csb_rnn_device_bytes and csb_rnn_upload again (a launch still in flight keeps reading the old
 * image).  Errors: NULL / batch <= 0 -> CSB_EINVAL; no resident layout -> CSB_EUNSUPPORTED. */
int csb_rnn_plan_resident(csb_rnn *r, int32_t batch);
int csb_rnn_stats(const csb_rnn *r, csb_rnn_plan_stats *out);

/*
 * The resident kernel's workgroups wait for each other's h_t with a bounded number of polls per
 * exchange word (default 2^24, minutes in all if nothing ever arrives).  A wait that gives up
 * yields NaN, makes every later wait of that lane give up at once (so the launch still ends
 * promptly) and sets a word in the resident image.  csb_rnn_status reads that word (it
 * synchronises `stream`), clears it and returns it in *timed_out: non-zero means a result since
 * the last check is NaN because the workgroups of a launch were not all running at once -- two
 * resident launches on different streams, or another kernel occupying the device: launch them
 * one after the other.  csb_rnn_set_poll_limit changes the bound (0: a word must be there at
 * the first look), for tests and for callers that prefer a quick failure.
 */
int csb_rnn_set_poll_limit(csb_rnn *r, uint32_t polls);
int csb_rnn_status(const csb_rnn *r, void *stream, int32_t *timed_out);

size_t csb_rnn_workspace_bytes(const csb_rnn *r, int32_t batch, int32_t T);

/*
 * Inference over a sequence.  All data device float32.
 *   d_x    [T][batch][input]
 *   d_h0   [n_layers][batch][hidden] or NULL (zeros);  d_c0 likewise (LSTM only)
 *   d_hseq [T][batch][hidden], outputs of the last layer, or NULL
 *   d_hT   [n_layers][batch][hidden];  d_cT likewise (LSTM; may be NULL)
 *   d_ws   csb_rnn_workspace_bytes(r, batch, T) bytes
 * T = 0 copies h0/c0 to hT/cT.  The time loop runs on the device side of `stream`
 * without host synchronisation.  Errors: NULL / batch <= 0 / T < 0 -> CSB_EINVAL;
 * neither the resident layout nor every W[l] uploaded -> CSB_ESTATE.
 * Not for replay from a captured HIP graph: the resident kernel (and csb_spmv / csb_spmm on a
 * matrix planned with shared row tiles) tell this call's exchange words from stale ones by a
 * launch tag that the HOST draws per call; a replay would reuse the tag.  Without a resident
 * layout uploaded, the streaming path at batch 1 on row-owned plans (what csb_rnn_create lays
 * out) and the batched path are kernel launches only and MAY be captured and replayed, with new
 * contents in the captured buffers (call once before the capture: a kernel's first launch raises
 * its LDS limit, which is not a stream operation).  The library does the same by itself for the
 * streaming path at batch 1: a call whose arguments (pointers, T, the matrices' uploads) repeat
 * those of the call before records its launches into a HIP graph that the handle keeps -- a
 * few milliseconds once, about 17 us per launch -- and calls with the same arguments replay it
 * from then on, on `stream` (a replayed launch costs less than an enqueued one); the buffers'
 * contents may change between such calls, anything else makes the call enqueue its launches
 * as before, and so does a `stream` that is being captured.  Calls on one handle
 * must not overlap either (they share the workspace's exchange words).
 */
int csb_rnn_forward(const csb_rnn *r, const float *d_x, const float *d_h0, const float *d_c0,
                    float *d_hseq, float *d_hT, float *d_cT, int32_t T, int32_t batch,
                    void *d_ws, void *stream);

/*
 * Projection of a dense matrix onto the CSB pattern: the pruning step inside Algorithm 1 as
 * Sec. 3.2.2 describes it.  The matrix is partitioned into br x bc blocks (edge blocks
 * truncated); RowPrune: in every block-column the in-block row segments are ranked by their
 * sum of squares and the weakest share 1 - sqrt(1 - PruneRate) is zeroed; ColumnPrune: the
 * same for the in-block column segments of every block-row, on the row-pruned matrix.
 * `rate` is the pruning rate as a factor ("10x" = 10, PruneRate = 1 - 1/rate), so
 * floor(n (1 - rate^-1/2) + 1/2) of n segments go in each pass.  Sums are float32, left to
 * right / top to bottom with one fused multiply-add per element; equal sums rank by
 * position (the earlier segment is the weaker); a NaN sum ranks on top.  Survivors keep
 * their bits, pruned entries become +0.0: the result is ready for csb_pack.
 * d_W: device, [rows][ld], ld >= cols.  d_Z: device, [rows][ldz], ldz >= cols; may be d_W
 * itself (with ldz == ld).  d_ws: device, csb_project_workspace_bytes(...) bytes, 256-byte
 * aligned, contents need no initialisation.  Five kernels, asynchronous on `stream`.
 * Errors: NULL, non-positive sizes, a leading dimension below cols, block size outside
 * [1, CSB_MAX_BLOCK], rate not a finite number >= 1 -> CSB_EINVAL; more than 16384 rows or
 * columns (one workgroup ranks a whole block-column in LDS) -> CSB_EUNSUPPORTED; launch
 * failure -> CSB_EDEVICE.
 */
size_t csb_project_workspace_bytes(int64_t rows, int64_t cols, int32_t br, int32_t bc);
int csb_project(const float *d_W, int64_t rows, int64_t cols, int64_t ld, int32_t br, int32_t bc,
                double rate, float *d_Z, int64_t ldz, void *d_ws, void *stream);

/* Release a handle (NULL is allowed).  The work of every call on it should have completed on its
 * stream: kernels in flight still read the handle's device image (the caller's buffer).
 * csb_rnn_free waits for the device first when the handle holds a recorded launch sequence. */
void csb_free(csb_matrix *m);
void csb_rnn_free(csb_rnn *r);

#ifdef __cplusplus
}
#endif
#endif /* CSBRNN_H */
