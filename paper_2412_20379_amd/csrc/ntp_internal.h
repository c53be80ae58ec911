// Internal structures of libntp: host-side graph, plan (bins, segments, chunks) and
// the argument block handed to the aggregation kernels.  Not part of the C boundary.
#pragma once

#include <cstdint>
#include <cstddef>
#include <string>
#include <vector>

#include "ntp.h"

namespace ntp {

// ---------------------------------------------------------------------------------------
// error reporting (thread-local text behind ntp_last_error)
void set_error(const char* fmt, ...);
const char* last_error();

// ---------------------------------------------------------------------------------------
// run fn(t, n_threads) on n_threads std::threads (t = 0..n_threads-1)
int host_threads();
void parallel_run(int n_threads, void (*fn)(int, int, void*), void* ctx);

template <class F>
inline void parallel_for_threads(int n_threads, F&& f) {
    struct Ctx { F* f; } ctx{&f};
    parallel_run(n_threads, [](int t, int nt, void* c) { (*static_cast<Ctx*>(c)->f)(t, nt); }, &ctx);
}

// ---------------------------------------------------------------------------------------
// One compressed form on the host.  colidx/val may live in pinned memory (owner decides).
struct HostSparse {
    int64_t n = 0;
    int64_t nnz = 0;
    std::vector<int64_t> rowptr;   // n + 1
    int32_t* colidx = nullptr;     // nnz
    float* val = nullptr;          // nnz
    bool pinned = false;           // colidx allocated with hipHostMalloc
    bool val_pinned = false;       // val allocated with hipHostMalloc (false: malloc)
    int64_t max_degree = 0;
};

struct BuiltGraph {
    int64_t n = 0;
    HostSparse csr;    // by destination
    HostSparse csc;    // by source (empty when symmetric: use csr)
    bool symmetric = false;
    bool has_csc = true;    // false: built with NTP_SCATTER_BWD and not symmetric (backward = scatter over csr)
    // How the stored weights follow from the structure, when they do (no caller weights):
    //   VAL_STORED: only the stored arrays know them
    //   VAL_GCN:    val(u -> v) = (float)(1 / sqrt((double)din[v] * (double)dout[u])), the formula they were built with
    //   VAL_ONES:   every weight is 1
    // din / dout: by-destination and by-source row lengths (empty unless VAL_GCN).
    int val_mode = 0;
    std::vector<int32_t> din, dout;
};
enum { VAL_STORED = 0, VAL_GCN = 1, VAL_ONES = 2 };

// allocator hooks so that graph_build.cpp stays free of HIP: returns nullptr on failure
struct EntryAllocator {
    void* (*alloc)(size_t bytes, void* ctx);            // column ids (and weights that have to travel)
    void* ctx;
    void* (*alloc_val)(size_t bytes, void* ctx);        // weights that never travel (rebuilt on the device)
};

// Build both compressed forms from an edge list (see ntp.h for the processing order).
// Returns NTP_OK or an error code (text set).
int build_host_graph(int64_t n, int64_t n_edges, const int32_t* src, const int32_t* dst,
                     const float* edge_weight, uint32_t flags, EntryAllocator alloc,
                     BuiltGraph* out);

// perm[p] (nnz entries, nnz < 2^31): where the edge at position p of the by-source form sits in
// the by-destination form
void build_edge_perm(const BuiltGraph& G, int32_t* perm);

// ---------------------------------------------------------------------------------------
// Plan: how the rows of one compressed form are mapped to wavefronts.
//
// Rows are binned by entry count d:  bin 0: d <= 1, bin k (1..NBINS-2): 2^(k-1) < d <= 2^k,
// last whole-row bin: everything up to split_threshold.  A row with more than
// split_threshold entries is cut into segments of about seg_len entries; each segment is
// summed by one wavefront into a partial-sum slot and a second small kernel adds the slots
// of a row in order.
constexpr int NBINS = 9;             // d<=1, 2, 3-4, 5-8, 9-16, 17-32, 33-64, 65-128, >128
constexpr int NGROUPS = NBINS + 1;   // + the segment group

struct Segment {        // one piece of a split row (device-visible, 24 bytes)
    int64_t e_begin;    // first entry (global offset into colidx/val)
    int32_t len;        // number of entries
    int32_t row;        // row the piece belongs to
    int32_t slot;       // partial-sum slot (global numbering within the form)
    int32_t pad;
};

struct ReduceItem {     // a split row whose last segment lies in this chunk (16 bytes)
    int32_t row;
    int32_t first_slot;
    int32_t n_slots;
    int32_t pad;
};

struct Chunk {
    int64_t row_begin = 0, row_end = 0;       // rows [row_begin, row_end)
    int64_t e_begin = 0, e_end = 0;           // entries [e_begin, e_end)
    bool partial_row = false;                  // chunk holds only pieces of one giant row
    // meta blob (host copy; same layout on the device): rowptr slice | bin rows | segments | reduce items
    std::vector<char> meta;
    size_t off_rowptr = 0;                     // int64[row_end - row_begin + 1]
    size_t off_rows = 0;                       // int32[n_bin_rows_total]
    size_t off_segs = 0;                       // Segment[n_segs]
    size_t off_reduce = 0;                     // ReduceItem[n_reduce]
    int32_t bin_count[NBINS] = {0};            // rows per bin
    int32_t bin_row_off[NBINS] = {0};          // offset of each bin's row list inside rows[]
    int32_t n_segs = 0;
    int32_t n_reduce = 0;
    int32_t max_split_len = 0;                 // entries of the longest split row that ends in this chunk
    bool block_rows = false;                   // split rows are summed by one block each (no segments, no partial sums)
    // device image layout: [meta | colidx | val], each part 256-byte aligned
    size_t img_off_colidx = 0, img_off_val = 0, img_bytes = 0;
    // residency
    int32_t* d_colidx_hub = nullptr;           // resident chunks of a form with a hub table: hub-encoded column ids
    char* d_image = nullptr;                   // device image if resident
    char* h_meta_pinned = nullptr;             // pinned copy of meta for streaming
};

struct Plan {
    // the most gathered columns of the form, most gathered first (at most agg_hub_slots(); empty: no
    // hub table): the aggregation keeps their feature rows in LDS (agg_kernels.hip)
    std::vector<int32_t> hub_cols;
    int64_t seg_len = 0;
    int64_t split_threshold = 0;
    int64_t chunk_edges = 0;
    int64_t n_slots = 0;                       // partial-sum slots of the whole form
    size_t max_img_bytes = 0;                  // largest chunk image (staging buffer size)
    std::vector<Chunk> chunks;
};

// Build the plan of one compressed form.  chunk_edges <= 0: a single chunk.
void make_plan(const HostSparse& m, int64_t chunk_edges, Plan* plan);

// The hub columns of a form: the up to max_slots columns with most entries, most first (ties by
// id), among those with at least min_count entries.  transposed (nullable): the other compressed
// form of the same matrix (this form itself if symmetric), whose row lengths are the column counts.
void pick_hub_columns(const HostSparse& m, const HostSparse* transposed, int max_slots, int64_t min_count,
                      std::vector<int32_t>* hub_cols);
// out[k] = 0x80000000 | slot for entries e_begin + k whose column is a hub, else the column id
void encode_hub_columns(const HostSparse& m, const std::vector<int32_t>& hub_cols, int64_t e_begin, int64_t e_end, int32_t* out);

// ---------------------------------------------------------------------------------------
// Argument block of the aggregation kernel (passed by value).
struct AggArgs {
    const int64_t* rowptr;     // chunk slice: rowptr[r - row_base]
    const int32_t* colidx;     // chunk slice: colidx[e - e_base]
    const float* val;
    const int32_t* rows;       // bin row lists (global row ids)
    const Segment* segs;
    const ReduceItem* split_rows;   // the chunk's split rows (block-per-row mode)
    const int32_t* colidx_hub; // chunk slice of the column ids with the hub columns replaced by 0x80000000 | slot
                               // (nullptr: the chunk has no hub table)
    const int32_t* hub_cols;   // [n_hub] vertex ids of the hub columns in slot order
    const void* X;
    void* Y;
    const void* M;             // epilogue mask source, rows indexed like Y (nullptr: the output itself)
    float* partial;            // [n_slots x fp] partial sums of split rows
    int64_t row_base;
    int64_t e_base;
    int64_t ldx, ldy, ldm;
    int32_t epilogue;          // 1: an output element is kept where its mask element (M, or itself) is > 0, else stored as 0
    int32_t f;                 // slice width
    int32_t fp;                // row stride of `partial` in floats: f rounded up to 8
    int32_t pass_lanes;        // vectors per feature row and column pass (0: widest shape)
    int32_t n_hub;             // hub columns (at most agg_hub_slots())
    int32_t n_groups;          // entries used in the tables below
    int32_t wave_start[NGROUPS + 1];   // first wavefront of each group; last = total
    int32_t item_off[NGROUPS];         // offset into rows[] (bins) or segs[] (segment group)
    int32_t item_count[NGROUPS];       // rows / segments in the group
    int32_t mode[NGROUPS];             // MODE_*
};
enum { MODE_GROUP_PER_ROW = 0, MODE_WAVE_PER_ROW = 1, MODE_SEGMENT = 2, MODE_BLOCK_PER_ROW = 3 };

struct ReduceArgs {
    const ReduceItem* items;
    const float* partial;
    void* Y;
    const void* M;             // epilogue mask source (see AggArgs)
    int64_t ldy, ldm;
    int32_t epilogue;
    int32_t f;
    int32_t fp;                // row stride of `partial` in floats
    int32_t n_items;
};

// kernels (agg_kernels.hip / nn_kernels.hip); stream is a hipStream_t
int launch_aggregate(const AggArgs& a, int dtype, void* stream);
int launch_reduce(const ReduceArgs& a, int dtype, void* stream);
int agg_hub_slots();               // lines of the LDS hub table
// does the launch of `a` (already holding X, Y, f, strides, pass_lanes) take the hub kernel?
bool agg_uses_hub(const AggArgs& a, int dtype);
// transposed product by scatter-add over the same rows: Y[colidx[k], :] += val[k] * X[row, :] (fp32 only)
int launch_scatter(const AggArgs& a, void* stream);
int scatter_lanes(int64_t f);      // lanes per feature row the scatter kernel uses for width f
// Y[0:n, 0:f] = 0 (row stride ld); a fill kernel, not a memset node
int launch_zero_rows(void* Y, int64_t n, int64_t f, int64_t ld, int dtype, void* stream);
// lanes per row chosen for (f, vec): exposed for tests of the host logic
void agg_shape(int64_t f, int vec, int pass_lanes, int* lanes_per_row, int* n_acc, int* n_passes);
int agg_pick_pass_lanes(const void* X, int64_t ldx, int dtype, int vec, double entries_per_row);
int agg_pick_vec(const void* X, const void* Y, int64_t f, int64_t ldx, int64_t ldy, int dtype, const void* M = nullptr, int64_t ldm = 0);

// edge attention weights (attention_kernels.hip)
struct AttArgs {
    const int64_t* rowptr;     // indexed by the global row id (a chunk's slice, shifted)
    const int32_t* colidx;     // indexed by the global entry offset (a chunk's slice, shifted)
    const int32_t* rows;       // bin row lists
    const float* p;            // per-vertex source score
    const float* q;            // per-vertex destination score
    float* st;                 // per destination, four floats (16-byte aligned): q, maximum score over its
                               // in-edges, 1 / sum of exp(score - maximum), 0
    float* alpha;              // output, entry order of the form
    float slope;               // LeakyReLU slope for negative scores
};
int launch_attention(const AttArgs& a, const int32_t* bin_row_off, const int32_t* bin_count,
                     const Segment* segs, int n_segs, const ReduceItem* split_rows, int n_split_rows,
                     float* seg_stats, bool transposed, int phase, void* stream);

struct AttBwdArgs {
    const int64_t* rowptr;     // indexed by the global row id
    const int32_t* colidx;     // indexed by the global entry offset
    const int32_t* rows;       // all rows below the split threshold (the bin lists, one after the other)
    const float* p;
    const float* q;
    const float* alpha;        // attention weights in this form's entry order
    const float* own;          // row vectors of this form's rows: dY (by destination) or Z (by source)
    const float* other;        // row vectors gathered by column id: Z (by destination) or dY (by source)
    int64_t ld_own, ld_other;
    float* t;                  // per destination, two floats (8-byte aligned): sum of alpha * dalpha, q
    float* park;               // [nnz] dalpha per entry (by-destination pass)
    float* out;                // dq (by destination) or dp (by source)
    float* slots;              // [n_slots] partial sums of the segments of split rows
    float slope;
    int32_t m;                 // feature width
    int32_t accumulate;        // add to out instead of overwriting it
    int32_t keep_w;            // by destination: leave (dalpha - t) * LeakyReLU' of every entry in park
};
// rows[0 .. n_group_rows): a lane group each; rows[n_group_rows .. + n_block_rows): a wavefront
// each (the bin lists are stored by increasing entry count); split rows: a block per segment
struct AttBwdRows {
    int n_group_rows;
    int n_block_rows;
    const Segment* segs;
    int n_segs;
    const ReduceItem* split_rows;      // rows whose last segment lies in this chunk
    int n_split_rows;
};
int launch_attention_bwd(const AttBwdArgs& a, const AttBwdRows& r, bool transposed, int phase, void* stream);

// per-vertex attention scores and their chain rule (attention_scores_kernels.hip)
int64_t attention_scores_max_width();
int64_t attention_scores_bwd_scratch_bytes(int64_t n, int64_t m);
int launch_attention_scores_fwd(const float* Z, const float* a_src, const float* a_dst, float* p, float* q,
                                int64_t n, int64_t m, int64_t ldz, void* stream);
int launch_attention_scores_bwd(const float* Z, const float* a_src, const float* a_dst, const float* dp, const float* dq,
                                float* dZ, float* da_src, float* da_dst, int64_t n, int64_t m, int64_t ldz, int64_t lddz,
                                float* scratch, void* stream);

// val[e] of a chunk's entries from the structure (VAL_GCN / VAL_ONES): rowptr is the chunk's slice
// (global entry offsets), colidx / val its entry arrays, deg_row / deg_col indexed by vertex id
int launch_rebuild_weights(const int64_t* rowptr, int64_t row_base, int64_t n_rows, int64_t e_base, int64_t n_entries,
                           const int32_t* colidx, float* val, const int32_t* deg_row, const int32_t* deg_col, int mode,
                           void* stream);

// a[i] += b[i]
int launch_vec_add(float* a, const float* b, int64_t n, void* stream);

int launch_softmax_xent(const float* Z, const int64_t* labels, float* dZ, float* loss, float* scratch,
                        int64_t n, int64_t c, int64_t ldz, int64_t lddz, void* stream);

int launch_nn_fwd(const void* A, const void* W, void* H, int64_t n, int64_t k, int64_t m,
                  int act, int dtype, void* stream);
int launch_nn_bwd(const void* A, const void* W, const void* H, const void* dH, void* dA, float* dW,
                  int64_t n, int64_t k, int64_t m, int act, int dtype,
                  void* workspace, int64_t workspace_bytes, void* stream);
int64_t nn_bwd_workspace_bytes(int64_t n, int64_t k, int64_t m);
int launch_relu(const void* dH, const void* H, void* out, int64_t n, int64_t f, int64_t ld, int dtype,
                bool backward, void* stream);

}  // namespace ntp
