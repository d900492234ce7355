// Internal definitions shared by the host packer/planner and the gfx950 kernels.
// Not part of the public ABI (that is include/csbrnn.h).
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "csbrnn.h"

namespace csb {

constexpr int kWave = 64;             // gfx950 wavefront width
constexpr int kMaxVbPerGroup = 16;    // virtual blocks packed into one 64-lane group
constexpr int kGroupOverhead = 8;     // per-group fixed cost in the work model (steps)
constexpr int kStepQuantum = 2;       // a group's column steps are padded to, and cut at, multiples of this
constexpr int kAccRowsMax = 256;      // output-row slots one workgroup accumulates in LDS
constexpr int kAccPlanes = 4;         // accumulator copies per wavefront: lanes that share a row use different copies
constexpr int kMaxStageCols = 16383;  // input vector floats staged in LDS; byte offsets fit 16 bits
constexpr int kChunkMetaMax = 24576;  // bytes of group/block/index records per workgroup
constexpr int kLdsBudget = 160 * 1024 - 2048;  // gfx950 LDS per workgroup, minus slack

// ---- device image records (plain structs, identical on host and device) ----------

// A group: up to 64 kernel-matrix rows of up to 16 virtual blocks of ONE output row
// tile, one row per lane.  Its values are stored step-major with a fixed stride: column
// step j is a run of 64 floats, lane l's value at [j * 64 + l], zero where the lane has no
// row or its block has no column j.  Every kernel value is stored once; the zeros are
// what keeps the inner loop free of address arithmetic and predicates.
struct GroupRec {
    uint32_t val_off;   // float index of (step 0, lane 0) in the value stream
    uint32_t vb_off;    // first VbRec of the group
    uint32_t idx_off;   // byte offset in the index stream: lane descriptors, input-offset lists
    uint32_t nzrank;    // rank of the group's output tile among tiles that have work
    uint16_t cmax;      // column steps of the group: largest column count, rounded up to kStepQuantum
    uint8_t nvb;        // virtual blocks
    uint8_t nlanes;     // kernel-matrix rows (lanes in use)
    uint16_t nrounds;   // the largest number of lanes that share one output row
    uint16_t pad;
};
static_assert(sizeof(GroupRec) == 24, "GroupRec layout");

// A virtual block: the kernel-matrix rows of one CSB block that fall into one output tile
// and one column part, at most 64 of them.  Only the batched kernel reads these records (the
// mat-vec kernel finds everything it needs in the lane descriptors).
struct VbRec {
    uint8_t r;          // rows (lanes)
    uint8_t lane0;      // first lane
    uint16_t c;         // columns
    uint32_t val_off;   // the group's val_off
    uint32_t desc_pos;  // the group's idx_off (lane descriptors)
    uint32_t list_pos;  // byte position of the block's input-offset list in the index stream
};
static_assert(sizeof(VbRec) == 16, "VbRec layout");

// Work of one wavefront: steps from (g_begin, j_begin) up to but excluding
// (g_end, j_end), groups in order; (g, cmax_g) is the same position as (g + 1, 0).
struct WaveRec {
    uint32_t g_begin, g_end;
    uint16_t j_begin, j_end;
    uint32_t val_begin;  // float offset inside group g_begin of step j_begin (j_begin * 64)
    uint32_t v_begin;    // absolute float index of the wavefront's first value; its steps are the
    uint32_t v_end;      // consecutive runs of 64 floats up to v_end
    uint32_t pad[2];
};
static_assert(sizeof(WaveRec) == 32, "WaveRec layout");

struct ChunkRec {
    uint32_t nzrank0;    // first non-empty tile rank the workgroup accumulates
    uint32_t ntiles;     // how many (LDS slots of br rows each)
    int32_t sid_first, part_first;  // shared-tile record / part of the first tile, or -1
    int32_t sid_last, part_last;    // same for the last tile (only if ntiles > 1), or -1
    uint32_t g0, ng;     // groups the workgroup touches: [g0, g0 + ng)
    uint32_t vb0, nvbs;  // their virtual-block records
    uint32_t idx0;       // their index bytes: start, rounded down to 16
    uint32_t idx_bytes;  // length from idx0, rounded up to 16
    uint32_t v0;         // first value of the workgroup's run of the value stream (float index, multiple of 64)
    uint32_t nv4;        // length of the run in float4
    uint32_t pad[2];
};
static_assert(sizeof(ChunkRec) == 64, "ChunkRec layout");

// A record segment of the batched kernel: a run of groups inside one row tile whose records
// fit the kernel's LDS window.
struct SegRec {
    uint32_t g0, ng;       // groups
    uint32_t vb0, nvbs;    // their virtual-block records
    uint32_t idx0;         // their index bytes: start, rounded down to 16
    uint32_t idx_bytes;    // length from idx0, rounded up to 16
    uint32_t pad[2];
};
static_assert(sizeof(SegRec) == 32, "SegRec layout");

struct SharedRec {
    uint32_t tile;         // output tile
    uint32_t nparts;       // workgroups that hold a partial sum of it
    uint32_t partial_off;  // first partial slot (each slot br floats per right-hand side)
    uint32_t pad;
};
static_assert(sizeof(SharedRec) == 16, "SharedRec layout");

struct DevHeader {
    uint64_t magic;
    uint32_t n_chunks, waves_per_chunk, n_groups, n_vbs;
    uint32_t n_shared, n_zero_tiles, n_nz_tiles, n_partial_slots;
    uint32_t br, bc;
    uint32_t max_chunk_tiles, seg_meta;        // LDS sizing: tiles per chunk; bytes of the largest record segment (batched kernel)
    uint32_t meta_cap, val_fmt;                // bytes of records per chunk; CSB_VAL_* of the value stream
    uint64_t rows_out, cols;
    uint64_t off_chunks, off_waves, off_groups, off_vbs, off_idx, off_vals;
    uint64_t off_nz_tiles, off_zero_tiles, off_shared, off_counters;
    uint64_t off_tile_g0;      // [n_nz_tiles + 1] first group of every row tile that has work
    uint64_t off_tile_seg0;    // [n_nz_tiles + 1] first record segment of every such tile
    uint64_t off_segs;         // [n_segs] record segments (never crossing tiles)
    uint64_t n_segs;
    uint64_t idx_bytes, n_vals, total_bytes;
};

// Device-side pointers resolved from the image base (kernel argument, by value).
struct DevMat {
    const ChunkRec *chunks;
    const WaveRec *waves;
    const GroupRec *groups;
    const VbRec *vbs;
    const uint8_t *idx;
    const float *vals;
    const uint32_t *nz_tiles;
    const uint32_t *zero_tiles;
    const uint32_t *tile_g0;
    const uint32_t *tile_seg0;
    const SegRec *segs;
    const SharedRec *shared;
    uint32_t *counters;
    uint32_t n_chunks, waves_per_chunk, n_zero_tiles, n_shared;
    uint32_t br, bc;
    uint32_t rows_out, cols;
    uint32_t n_groups, n_nz_tiles;
    uint32_t idx_bytes, val_fmt;   // val_fmt != 0: vals holds one 32-bit word per lane and PAIR of steps (even step low)
    uint32_t seg_meta, vals_bytes; // LDS bytes the batched kernel sets aside for one record segment; bytes of the value stream (saturated)
};

// How rows are relabelled when the image is built for a GRU: entries in rows >= split_row
// and columns >= split_col are summed into output row (row + shift) instead of row.
struct SplitSpec {
    int64_t split_row = -1, split_col = -1, shift = 0;
    bool active() const { return split_row >= 0; }
    bool operator==(const SplitSpec &o) const {
        return split_row == o.split_row && split_col == o.split_col && shift == o.shift;
    }
};

// ---- row-owned stream section (batch-1 mat-vec of csb_spmv) ---------------------------
// A second section of the device image, laid out so that a launch is ONE pass of loads whose
// addresses depend on nothing but the workgroup and wavefront numbers.  Every workgroup owns
// a contiguous range of output rows (at most kStreamMaxRows) and all kernel-matrix rows that
// land in them; its work is dealt to its 16 wavefronts in `n_rounds` rounds.  The section is
// n_wg runs of `wg_bytes` each: a header (`hdr_bytes`) followed by n_rounds * 16 wavefront
// segments of `seg_bytes`, round-major (wavefront w works on segments w, w + 16, ...).  A
// segment is self-describing (all offsets inside it are relative to its start), is copied
// verbatim into the wavefront's own LDS area, and holds its records in front of its values,
// the values in the order in which they are multiplied: a wavefront can start on a segment
// while the rest of it is still on its way.
constexpr int kStreamWaves = 16;
constexpr int kStreamThreads = kStreamWaves * kWave;
constexpr int kStreamMaxRows = 256;      // output rows of one workgroup (at least four threads add up a row)
constexpr int kStreamMaxSegUnits = 8;    // 1 KiB units of a wavefront segment (one 16-byte load per lane each)
constexpr int kStreamGroupOverhead = 8;  // fixed cost of a piece of a group in the work model (steps)
constexpr int kStreamListLimit = 4096;   // column lists start below this byte offset of their segment (10-bit word index)

// Workgroup header: what the row-sum pass needs.
struct StreamRoundHdr {
    uint32_t row0;       // first output row of the workgroup
    uint32_t nrows;      // its number of output rows
    uint32_t pad[2];
    // followed by uint32_t [rows_max]: first slot (low half) and number (high half) of each row's
    // partial sums in the workgroup's table, padded to 16 bytes
};
static_assert(sizeof(StreamRoundHdr) == 16, "StreamRoundHdr layout");

struct StreamSegHdr {
    uint16_t ng;         // groups in this segment
    uint16_t off_vbs;    // byte offset of the virtual-block words
    uint16_t bytes16;    // the segment's own length in 16-byte units (the rest of the stride is never read)
    uint16_t next16;     // the same of the wavefront's segment of the next round (0: none)
    uint16_t pad[4];
};
static_assert(sizeof(StreamSegHdr) == 16, "StreamSegHdr layout");

// A group: up to 64 kernel-matrix rows (one per lane) of consecutive virtual blocks, and a run
// of their column steps.  Bit l of start_mask is set when lane l is the first row of a virtual
// block: a lane's block is vb0 + popcount(start_mask & bits up to and including l) - 1.
// Values: step-major with a fixed stride -- step j is a run of 64 floats (lane l at [j * 64 + l]),
// zero where the lane has no row or its block has no column j, so the multiplication needs no
// predicates and reads its values at constant offsets.  The rows of a workgroup are sorted by
// column count before they are grouped, so few of the slots are zeros.
struct StreamGroup {
    uint64_t start_mask;
    uint16_t vb0;           // first virtual-block word of the group (index inside the segment)
    uint16_t lane_off;      // byte offset of the lanes' (row, slot) words
    uint16_t val_off;       // float index (inside the segment) of the value of step 0, lane 0
    uint8_t cmax_minus_1;   // column steps - 1
    uint8_t nlanes;
};
static_assert(sizeof(StreamGroup) == 16, "StreamGroup layout");

// A virtual block (consecutive kernel-matrix rows of one CSB block, a range of its columns) is
// one 32-bit word: bits 0-9 the 4-byte word index of its column index list inside the segment
// (bytes; padded with its first byte to the piece's steps rounded up to 4), bits 10-17 its column
// count - 1, bits 18-31 the block column of the CSB block (its first input is block column * bc).
constexpr uint32_t stream_vb_word(uint32_t list_word, uint32_t c_minus_1, uint32_t bj) { return list_word | (c_minus_1 << 10) | (bj << 18); }

struct StreamPlan {
    bool valid = false;
    uint32_t n_wg = 0, n_rounds = 0;
    uint32_t seg_bytes = 0;     // multiple of 16
    uint32_t hdr_bytes = 0;     // multiple of 16
    uint32_t wg_bytes = 0;      // hdr_bytes + n_rounds * 16 * seg_bytes rounded up to 256
    uint32_t kmax = 0;          // slots of the partial-sum table (the fullest workgroup's)
    uint32_t rows_max = 0;      // largest row count of a workgroup
    uint32_t tpr = 0;           // threads that share an output row in the row-sum pass (power of two)
    uint32_t lds_bytes = 0;
    uint32_t n_groups = 0;
    uint32_t val_fmt = 0;       // CSB_VAL_*: 32-bit values, or 16-bit ones (a column step is then a run of 64 half words)
    uint32_t cell_gates = 0;    // 0: a workgroup owns output rows [row0, row0 + nrows).  G > 0: it owns the units
                                // [row0, row0 + nrows / G) of a recurrent cell with all their G gate rows; its local row
                                // g * (nrows / G) + j is output row g * cell_units + row0 + j
    uint32_t cell_units = 0;    // units of the cell (output rows / G)
    uint64_t off = 0, bytes = 0;   // the section inside the image
};

struct Plan {
    bool valid = false;
    SplitSpec split;              // stays when the plan becomes invalid: csb_plan keeps the row layout of a matrix a GRU handle planned
    int32_t req_chunks = 0, req_mode = 0;   // what the plan was asked for
    std::vector<uint8_t> image;   // host staging copy of the device image
    DevHeader hdr{};
    StreamPlan stream;            // valid: csb_spmv reads this section instead of the sections above
    csb_plan_stats stats{};
};

void set_error(const std::string &msg);
// 16-bit value formats: nearest, ties to even
uint16_t f32_to_f16_bits(float f);
float f16_bits_to_f32(uint16_t h);
uint16_t f32_to_bf16_bits(float f);
inline float bf16_bits_to_f32(uint16_t h) { uint32_t u = (uint32_t)h << 16; float f; __builtin_memcpy(&f, &u, 4); return f; }
uint32_t reserve_tags(uint32_t count, uint32_t *generation);
// Records `user` as the last user of the caller's workspace `ws` (a workspace is identified by
// its base address) and tells whether somebody else has used it since `user` last did.  What
// that somebody wrote there may look like anything, a tagged word included, so the tagged words
// that `user` keeps in the workspace have to be cleared again before they are polled.
bool workspace_changed_hands(const void *ws, const void *user);

}  // namespace csb

struct csb_matrix {
    int64_t rows = 0, cols = 0;
    int32_t br = 0, bc = 0, nbr = 0, nbc = 0;
    std::vector<int32_t> nrows, ncols;
    std::vector<uint16_t> rowidx, colidx;
    std::vector<float> val;
    std::vector<int64_t> val_off, row_off, col_off;
    int32_t val_fmt = 0;          // CSB_VAL_*: how the device value stream is stored
    int32_t stream_wg_limit = 256;   // most workgroups a default row-owned plan takes (an RNN handle with stacked layers,
                                     // whose products share launches, leaves its matrices a share of the 256 CUs each)
    int32_t stream_cell_gates = 0;   // > 0: the rows are `gates` stacked groups of rows/gates units each, and a workgroup of
                                     // the row-owned plan is to own all gate rows of its units (set by an RNN handle, whose
                                     // mat-vec launches then finish their cells themselves; csb_plan* ask for plain ranges)
    csb::Plan plan;
    void *d_buf = nullptr;        // caller-owned device image, set by csb_upload
    bool uploaded = false;
    uint64_t upload_serial = 0;   // a number no other upload of any matrix has had (what a recorded launch sequence was made for)
    // launch bookkeeping for the cross-workgroup merge (mutable: csb_spmv takes a const handle)
    mutable uint32_t epoch = 0;          // tag generation in which ws_seen was cleared
    mutable const void *ws_seen = nullptr;  // workspace already cleared for this matrix
};

namespace csb {
int plan_matrix(csb_matrix *m, int32_t n_chunks, int32_t waves_per_chunk, const SplitSpec &split,
                csb_plan_stats *stats, int32_t mode);
int validate_plan(const csb_matrix *m);
int plan_stream(csb_matrix *m, int32_t n_wg_req, int32_t rounds_min, csb_plan_stats *stats);
int validate_stream(const csb_matrix *m);
DevMat dev_mat(const csb_matrix *m);
}  // namespace csb
