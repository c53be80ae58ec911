// C boundary of libntp (see include/ntp.h): graph handle, device residency, the
// aggregation calls and the chunk streamer of Section 4.2.1.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>

#include "ntp_internal.h"

using namespace ntp;

#define HIP_TRY(expr)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) {                                                              \
            set_error("%s failed: %s", #expr, hipGetErrorString(e_));                        \
            return NTP_EHIP;                                                                 \
        }                                                                                    \
    } while (0)

struct Form {
    HostSparse* m = nullptr;
    Plan plan;
    bool all_resident = false;
    // forms of several chunks: the reduce items of all chunks that sum their split rows from
    // segments, in chunk order, on the device (one reduce_kernel launch per pass)
    ReduceItem* d_all_reduce = nullptr;
    int n_all_reduce = 0;
    int32_t* d_hub_cols = nullptr;      // the form's hub columns on the device (plan.hub_cols), when it has a hub table
    bool one_reduce() const { return d_all_reduce != nullptr; }
};

struct ntp_graph {
    BuiltGraph g;
    Form form[2];                  // NTP_CSR, NTP_CSC (unused when symmetric)
    bool host_only = false;
    bool pinned_entries = false;
    bool val_pinned = false;       // the weights are in pinned memory too (caller weights on a graph that may stream)
    // staging for streamed chunks
    char* stage[2] = {nullptr, nullptr};
    size_t stage_bytes = 0;
    hipEvent_t ev_ready[2] = {nullptr, nullptr};   // copy of the chunk finished
    hipEvent_t ev_free[2] = {nullptr, nullptr};    // kernels reading the buffer finished
    bool stage_used[2] = {false, false};
    int next_stage = 0;
    char* pinned_meta = nullptr;                    // metas of streamed chunks
    // partial sums of split rows
    float* partial = nullptr;
    size_t partial_bytes = 0;
    float* att_stats = nullptr;    // [4 n]: per-destination (q, maximum, 1 / sum, 0) of the last ntp_edge_softmax
    float* att_bwd = nullptr;      // scratch of ntp_edge_softmax_bwd: per-destination (t, q), per-segment partial sums, per-edge dalpha
    std::vector<int32_t> h_perm;   // NTP_EDGE_PERM: by-source entry -> by-destination entry
    int32_t* d_din = nullptr;      // by-destination / by-source row lengths on the device: weights of streamed
    int32_t* d_dout = nullptr;     // chunks are rebuilt from them (VAL_GCN graphs with streamed chunks only)
    int32_t* d_perm = nullptr;
    int64_t device_bytes = 0;

    // streamed chunks carry column ids only; their weights are rebuilt after the copy
    bool streams_without_weights() const { return g.val_mode == VAL_ONES || (g.val_mode == VAL_GCN && d_din != nullptr); }
    // the by-source product runs as a scatter over the by-destination form
    bool scatter_bwd() const { return !g.has_csc; }
    Form& f(int which) { return form[(which == NTP_CSC && !g.symmetric && g.has_csc) ? 1 : 0]; }
    const Form& f(int which) const { return form[(which == NTP_CSC && !g.symmetric && g.has_csc) ? 1 : 0]; }
};

// Scratch of ntp_aggregate_fwd_noalloc: partial sums of split rows, in the library's own image
// (every GPU the library is loaded on holds its own copy until the process ends).  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels get the resolved address.
// (No `used` attribute: with it the symbol stays local to the code object and the look-up aborts;
// the host-side reference alone makes the compiler export it.)
static __device__ __align__(256) float scratch[NTP_NOALLOC_SCRATCH_BYTES / sizeof(float)];

namespace {

// device address of `scratch` on the current device, resolved once per device
int static_scratch(float** out) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static float* ptr[MAX_DEVICES] = {nullptr};
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) { set_error("device ordinal %d outside 0..%d", dev, MAX_DEVICES - 1); return NTP_EUNSUPPORTED; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { set_error("hipGetSymbolAddress returned no address for the static scratch"); return NTP_EHIP; }
        ptr[dev] = static_cast<float*>(p);
    }
    *out = ptr[dev];
    return NTP_OK;
}

void* alloc_plain(size_t bytes, void*) { return malloc(bytes); }
void* alloc_pinned(size_t bytes, void*) {
    void* p = nullptr;
    if (hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) return nullptr;
    return p;
}

// colidx lives in pinned memory when chunks may be streamed; val only if it has to travel too
void free_entries(HostSparse& m, bool pinned, bool val_pinned) {
    if (m.colidx) { if (pinned) (void)hipHostFree(m.colidx); else free(m.colidx); }
    if (m.val) { if (val_pinned) (void)hipHostFree(m.val); else free(m.val); }
    m.colidx = nullptr;
    m.val = nullptr;
}

// with_val = false: the weights are rebuilt on the device after the copy (launch_rebuild_weights)
int upload_chunk(const HostSparse& m, Chunk& c, char* dst, hipStream_t st, bool async, const char* meta_src, bool with_val = true) {
    const size_t ne = (size_t)(c.e_end - c.e_begin);
    if (async) {
        HIP_TRY(hipMemcpyAsync(dst, meta_src, c.meta.size(), hipMemcpyHostToDevice, st));
        if (ne) {
            HIP_TRY(hipMemcpyAsync(dst + c.img_off_colidx, m.colidx + c.e_begin, ne * 4, hipMemcpyHostToDevice, st));
            if (with_val) HIP_TRY(hipMemcpyAsync(dst + c.img_off_val, m.val + c.e_begin, ne * 4, hipMemcpyHostToDevice, st));
        }
    } else {
        HIP_TRY(hipMemcpy(dst, meta_src, c.meta.size(), hipMemcpyHostToDevice));
        if (ne) {
            HIP_TRY(hipMemcpy(dst + c.img_off_colidx, m.colidx + c.e_begin, ne * 4, hipMemcpyHostToDevice));
            HIP_TRY(hipMemcpy(dst + c.img_off_val, m.val + c.e_begin, ne * 4, hipMemcpyHostToDevice));
        }
    }
    return NTP_OK;
}

// what the aggregation does to an output element on its way out (AggArgs::epilogue)
struct Epilogue {
    bool on = false;
    const void* M = nullptr;       // mask source (nullptr: the output itself, i.e. ReLU)
    int64_t ldm = 0;
};

inline int bin_max_degree(int b) { return b == 0 ? 1 : (b == NBINS - 1 ? INT_MAX : (1 << b)); }

// Enqueue the kernels of one chunk whose image lives at `img` on the device.
// scatter: Y[colidx[k], :] += val[k] * X[row, :] instead of Y[row, :] = sum val[k] * X[colidx[k], :]
// weights: caller's edge weights in the entry order of the form (nullptr: the stored ones)
int run_chunk(const Chunk& c, const char* img, const void* X, void* Y, float* partial,
              int64_t f, int64_t ldx, int64_t ldy, int dtype, hipStream_t st, bool scatter = false,
              const float* weights = nullptr, const int32_t* columns = nullptr, bool defer_reduce = false,
              const int32_t* hub_cols = nullptr, int n_hub = 0, const Epilogue& epi = Epilogue()) {
    AggArgs a;
    memset(&a, 0, sizeof a);
    a.rowptr = reinterpret_cast<const int64_t*>(img + c.off_rowptr);
    a.rows = reinterpret_cast<const int32_t*>(img + c.off_rows);
    a.segs = reinterpret_cast<const Segment*>(img + c.off_segs);
    a.colidx = columns ? columns + c.e_begin : reinterpret_cast<const int32_t*>(img + c.img_off_colidx);
    a.val = weights ? weights + c.e_begin : reinterpret_cast<const float*>(img + c.img_off_val);
    a.X = X;
    a.Y = Y;
    a.M = epi.M;
    a.ldm = epi.ldm;
    a.epilogue = epi.on ? 1 : 0;
    a.partial = partial;
    a.row_base = c.row_begin;
    a.e_base = c.e_begin;
    a.ldx = ldx;
    a.ldy = ldy;
    a.f = (int32_t)f;
    a.fp = (int32_t)((f + 7) / 8 * 8);

    int L, nacc = 1, passes = 1;
    if (scatter) {
        L = scatter_lanes(f);
    } else {
        const int vec = agg_pick_vec(X, Y, f, ldx, ldy, dtype, epi.M, epi.ldm);
        const int64_t rows = c.partial_row ? 1 : c.row_end - c.row_begin;
        a.pass_lanes = agg_pick_pass_lanes(X, ldx, dtype, vec, (double)(c.e_end - c.e_begin) / (double)std::max<int64_t>(1, rows));
        agg_shape(f, vec, a.pass_lanes, &L, &nacc, &passes);
    }
    const int R = 64 / L;
    bool hub = false;
    if (!scatter && !columns && c.d_colidx_hub && hub_cols) {
        a.colidx_hub = c.d_colidx_hub;
        a.hub_cols = hub_cols;
        a.n_hub = n_hub;
        hub = agg_uses_hub(a, dtype);
    }

    int ng = 0;
    int64_t waves = 0;
    auto add_group = [&](int mode, int off, int count, int64_t nw) {
        a.wave_start[ng] = (int32_t)waves;
        a.item_off[ng] = off;
        a.item_count[ng] = count;
        a.mode[ng] = mode;
        waves += nw;
        ++ng;
    };
    const bool block_rows = !scatter && !hub && c.block_rows;      // split rows summed by one block each (see make_plan)
    a.split_rows = reinterpret_cast<const ReduceItem*>(img + c.off_reduce);
    // heaviest work first: split rows, then bins from long rows to short rows
    if (block_rows) add_group(MODE_BLOCK_PER_ROW, 0, c.n_reduce, 4 * (int64_t)c.n_reduce);   // first: block-aligned
    else if (c.n_segs > 0) add_group(MODE_SEGMENT, 0, c.n_segs, c.n_segs);
    for (int b = NBINS - 1; b >= 0; --b) {
        const int cnt = c.bin_count[b];
        if (cnt == 0) continue;
        // rows of up to 32 entries: one lane group per row (measured best for every group count)
        const bool per_group = R > 1 && bin_max_degree(b) <= 32;
        if (per_group) add_group(MODE_GROUP_PER_ROW, c.bin_row_off[b], cnt, (cnt + R - 1) / R);
        else add_group(MODE_WAVE_PER_ROW, c.bin_row_off[b], cnt, cnt);
    }
    if (waves > INT_MAX - 8) { set_error("chunk too large for one launch (%lld wavefronts)", (long long)waves); return NTP_EUNSUPPORTED; }
    a.wave_start[ng] = (int32_t)waves;
    a.n_groups = ng;
    if (ng > 0) {
        const int rc = scatter ? launch_scatter(a, st) : launch_aggregate(a, dtype, st);
        if (rc != NTP_OK) return rc;
    }
    if (c.n_reduce > 0 && !scatter && !block_rows && !defer_reduce) {
        ReduceArgs r;
        r.items = reinterpret_cast<const ReduceItem*>(img + c.off_reduce);
        r.partial = partial;
        r.Y = Y;
        r.M = epi.M;
        r.ldm = epi.ldm;
        r.epilogue = epi.on ? 1 : 0;
        r.ldy = ldy;
        r.f = (int32_t)f;
        r.fp = (int32_t)((f + 7) / 8 * 8);
        r.n_items = c.n_reduce;
        const int rc = launch_reduce(r, dtype, st);
        if (rc != NTP_OK) return rc;
    }
    return NTP_OK;
}

// One reduce_kernel launch for the split rows of every chunk of a form (their items were
// gathered on the device at build time): replaces one launch per chunk when a form has several.
int reduce_all(const Form& F, float* partial, void* Y, int64_t f, int64_t ldy, int dtype, hipStream_t st, const Epilogue& epi = Epilogue()) {
    if (F.n_all_reduce == 0) return NTP_OK;
    ReduceArgs r;
    r.items = F.d_all_reduce;
    r.partial = partial;
    r.Y = Y;
    r.M = epi.M;
    r.ldm = epi.ldm;
    r.epilogue = epi.on ? 1 : 0;
    r.ldy = ldy;
    r.f = (int32_t)f;
    r.fp = (int32_t)((f + 7) / 8 * 8);
    r.n_items = F.n_all_reduce;
    return launch_reduce(r, dtype, st);
}

// floats of scratch one right-hand side needs for the partial sums of split rows
size_t partial_floats(const Form& F, int64_t f) { return (size_t)F.plan.n_slots * (size_t)((f + 7) / 8 * 8); }

int ensure_partial(ntp_graph* G, const Form& F, int64_t f, int n_rhs = 1) {
    const size_t need = partial_floats(F, f) * sizeof(float) * (size_t)n_rhs;
    if (need <= G->partial_bytes) return NTP_OK;
    if (G->partial) {
        HIP_TRY(hipDeviceSynchronize());       // earlier calls may still read the old buffer
        HIP_TRY(hipFree(G->partial));
        G->device_bytes -= (int64_t)G->partial_bytes;
        G->partial = nullptr;
        G->partial_bytes = 0;
    }
    void* p = nullptr;
    if (hipMalloc(&p, need) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu scratch bytes failed", need); return NTP_ENOMEM; }
    G->partial = (float*)p;
    G->partial_bytes = need;
    G->device_bytes += (int64_t)need;
    return NTP_OK;
}

// Do two row-major views of n rows x f elements (row strides lda, ldb in elements of es bytes)
// share a byte?  Each view is n intervals of f * es bytes.  Disjoint spans: no.  Equal strides: the
// intervals of both repeat with the same period, so they meet iff the two windows meet modulo the
// stride.  Different strides inside one span: not decided here, reported as overlapping.
bool views_overlap(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n, int64_t f, int64_t es) {
    if (n <= 0 || f <= 0) return false;
    const uintptr_t a = (uintptr_t)A, b = (uintptr_t)B;
    const uintptr_t wa = (uintptr_t)(f * es);
    const uintptr_t span_a = (uintptr_t)((n - 1) * lda * es) + wa, span_b = (uintptr_t)((n - 1) * ldb * es) + wa;
    if (a + span_a <= b || b + span_b <= a) return false;
    if (lda != ldb) return true;
    const uintptr_t period = (uintptr_t)(lda * es);
    const uintptr_t d = (b >= a ? b - a : a - b) % period;       // offset of one window inside the other's period
    return d < wa || period - d < wa;
}

int check_agg_args(const ntp_graph* g, const void* X, const void* Y, int64_t f, int64_t ldx, int64_t ldy, int dtype, bool need_device = true) {
    if (!g) { set_error("graph handle is NULL"); return NTP_EINVAL; }
    if (dtype != NTP_F32 && dtype != NTP_BF16) { set_error("unknown dtype %d", dtype); return NTP_EINVAL; }
    if (f < 1 || f > (1 << 20)) { set_error("slice width %lld out of range (1..2^20)", (long long)f); return NTP_EINVAL; }
    if (ldx < f || ldy < f) { set_error("row stride smaller than the slice width"); return NTP_EINVAL; }
    // the kernels form row addresses as vertex id x stride in bytes with a 32 x 32 -> 64-bit multiply
    if (ldx >= (1ll << 30) || ldy >= (1ll << 30)) { set_error("row stride of 2^30 elements or more"); return NTP_EINVAL; }
    if (g->g.n > 0 && (!X || !Y)) { set_error("X or Y is NULL"); return NTP_EINVAL; }
    if (g->g.n > 0 && views_overlap(X, ldx, Y, ldy, g->g.n, f, dtype == NTP_BF16 ? 2 : 4)) {
        set_error("input and output must not overlap");
        return NTP_EINVAL;
    }
    if (need_device && g->host_only) { set_error("graph was built with NTP_HOST_ONLY: nothing is on the device"); return NTP_EBUDGET; }
    return NTP_OK;
}

void destroy(ntp_graph* G) {
    if (!G) return;
    if (!G->host_only) (void)hipDeviceSynchronize();
    for (int k = 0; k < 2; ++k) {
        for (auto& c : G->form[k].plan.chunks)
            if (c.d_image) (void)hipFree(c.d_image);
        for (auto& c : G->form[k].plan.chunks)
            if (c.d_colidx_hub) (void)hipFree(c.d_colidx_hub);
        if (G->form[k].d_hub_cols) (void)hipFree(G->form[k].d_hub_cols);
        if (G->form[k].d_all_reduce) (void)hipFree(G->form[k].d_all_reduce);
        if (G->stage[k]) (void)hipFree(G->stage[k]);
        if (G->ev_ready[k]) (void)hipEventDestroy(G->ev_ready[k]);
        if (G->ev_free[k]) (void)hipEventDestroy(G->ev_free[k]);
    }
    if (G->partial) (void)hipFree(G->partial);
    if (G->att_stats) (void)hipFree(G->att_stats);
    if (G->att_bwd) (void)hipFree(G->att_bwd);
    if (G->d_perm) (void)hipFree(G->d_perm);
    if (G->d_din) (void)hipFree(G->d_din);
    if (G->d_dout && G->d_dout != G->d_din) (void)hipFree(G->d_dout);
    if (G->pinned_meta) (void)hipHostFree(G->pinned_meta);
    free_entries(G->g.csr, G->pinned_entries, G->val_pinned);
    free_entries(G->g.csc, G->pinned_entries, G->val_pinned);
    delete G;
}

}  // namespace

extern "C" {

const char* ntp_last_error(void) { return last_error(); }

static int graph_build_impl(int64_t n, int64_t n_edges, const int32_t* src, const int32_t* dst,
                            const float* edge_weight, uint32_t flags, int64_t budget, int64_t chunk_edges,
                            ntp_graph_t** out) {
    if (!out) { set_error("out is NULL"); return NTP_EINVAL; }
    *out = nullptr;
    if (n < 0 || n > INT_MAX - 1) { set_error("n_vertices %lld out of range", (long long)n); return NTP_EINVAL; }
    if (n_edges < 0 || (n_edges > 0 && (!src || !dst))) { set_error("edge list missing"); return NTP_EINVAL; }
    if (budget < 0 || chunk_edges < 0) { set_error("negative budget or chunk size"); return NTP_EINVAL; }
    if (chunk_edges > INT_MAX) { set_error("chunk_edges must be below 2^31"); return NTP_EINVAL; }
    const uint32_t known = NTP_SYMMETRISE | NTP_DEDUP | NTP_ADD_SELF_LOOPS | NTP_NORM_GCN_SYM | NTP_HOST_ONLY | NTP_FORCE_STREAM | NTP_SCATTER_BWD | NTP_EDGE_PERM;
    if (flags & ~known) { set_error("unknown flag bits 0x%x", flags & ~known); return NTP_EINVAL; }
    if ((flags & NTP_EDGE_PERM) && (flags & NTP_SCATTER_BWD)) { set_error("NTP_EDGE_PERM needs the by-source form that NTP_SCATTER_BWD leaves out"); return NTP_EINVAL; }

    ntp_graph* G = new (std::nothrow) ntp_graph();
    if (!G) { set_error("out of host memory"); return NTP_ENOMEM; }
    std::unique_ptr<ntp_graph, void (*)(ntp_graph*)> guard(G, destroy);   // frees everything on any early return
    G->host_only = flags & NTP_HOST_ONLY;
    const bool force_stream = flags & NTP_FORCE_STREAM;
    // entries go to pinned memory whenever chunks may have to be streamed
    G->pinned_entries = !G->host_only && (budget > 0 || force_stream);
    G->val_pinned = G->pinned_entries && edge_weight != nullptr;
    EntryAllocator alloc{G->pinned_entries ? alloc_pinned : alloc_plain, nullptr, alloc_plain};

    int rc = build_host_graph(n, n_edges, src, dst, edge_weight, flags, alloc, &G->g);
    if (rc != NTP_OK) { return rc; }
    if (G->g.symmetric && G->g.csc.colidx) { free_entries(G->g.csc, G->pinned_entries, G->val_pinned); G->g.csc = HostSparse(); }

    const int n_forms = (G->g.symmetric || !G->g.has_csc) ? 1 : 2;
    G->form[0].m = &G->g.csr;
    G->form[1].m = n_forms == 1 ? &G->g.csr : &G->g.csc;

    // chunk size: caller's, else one chunk if everything fits, else half of what the
    // budget leaves per staging buffer
    int64_t ce = chunk_edges;
    if (ce == 0 && (budget > 0 || force_stream)) {
        int64_t need = 0;
        for (int k = 0; k < n_forms; ++k) need += G->form[k].m->nnz * 8 + (n + 1) * 12 + 4096;
        if (force_stream || need > budget) {
            const int64_t per_buf = (budget > 0 ? budget : need) / 4;    // two buffers use half
            ce = std::max<int64_t>(1024, std::min<int64_t>((per_buf - 4096) / 20, INT_MAX / 2));
        }
    }
    if (flags & NTP_EDGE_PERM) {
        const int64_t nnz = G->g.csr.nnz;
        if (nnz > INT_MAX) { set_error("NTP_EDGE_PERM takes graphs of fewer than 2^31 stored entries"); return NTP_EUNSUPPORTED; }
        G->h_perm.resize((size_t)nnz);
        build_edge_perm(G->g, G->h_perm.data());
    }
    for (int k = 0; k < n_forms; ++k) make_plan(*G->form[k].m, ce, &G->form[k].plan);
    for (int k = 0; k < n_forms; ++k)
        for (auto& c : G->form[k].plan.chunks)
            if (c.e_end - c.e_begin > INT_MAX || G->form[k].plan.n_slots > INT_MAX / 2) {
                set_error("a chunk holds more than 2^31 entries: pass a chunk_edges below that");
                return NTP_EUNSUPPORTED;
            }

    if (!G->host_only) {
        size_t all = 0, max_img = 0;
        for (int k = 0; k < n_forms; ++k) {
            for (auto& c : G->form[k].plan.chunks) all += c.img_bytes;
            max_img = std::max(max_img, G->form[k].plan.max_img_bytes);
        }
        const bool fits = !force_stream && (budget == 0 || (int64_t)all <= budget);
        int64_t left = 0;
        if (!fits) {
            if (budget > 0 && (int64_t)(2 * max_img) > budget) {
                set_error("device budget %lld cannot hold two staging buffers of %zu bytes", (long long)budget, max_img);
                return NTP_EBUDGET;
            }
            G->stage_bytes = max_img;
            for (int b = 0; b < 2; ++b) {
                void* p = nullptr;
                if (hipMalloc(&p, max_img) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of a %zu-byte staging buffer failed", max_img); return NTP_ENOMEM; }
                G->stage[b] = (char*)p;
                G->device_bytes += (int64_t)max_img;
                if (hipEventCreateWithFlags(&G->ev_ready[b], hipEventDisableTiming) != hipSuccess ||
                    hipEventCreateWithFlags(&G->ev_free[b], hipEventDisableTiming) != hipSuccess) {
                    set_error("hipEventCreate failed"); return NTP_EHIP;
                }
            }
            left = force_stream ? 0 : budget - (int64_t)(2 * max_img);
        }
        // residency: everything if it fits, else chunks in round-robin order over the forms
        size_t max_chunks = 0;
        for (int k = 0; k < n_forms; ++k) max_chunks = std::max(max_chunks, G->form[k].plan.chunks.size());
        size_t pinned_meta_bytes = 0;
        for (size_t ci = 0; ci < max_chunks; ++ci)
            for (int k = 0; k < n_forms; ++k) {
                auto& chunks = G->form[k].plan.chunks;
                if (ci >= chunks.size()) continue;
                Chunk& c = chunks[ci];
                const bool resident = fits || (int64_t)c.img_bytes <= left;
                if (resident) {
                    void* p = nullptr;
                    if (hipMalloc(&p, c.img_bytes) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of a %zu-byte chunk failed", c.img_bytes); return NTP_ENOMEM; }
                    c.d_image = (char*)p;
                    G->device_bytes += (int64_t)c.img_bytes;
                    if (!fits) left -= (int64_t)c.img_bytes;
                    rc = upload_chunk(*G->form[k].m, c, c.d_image, nullptr, false, c.meta.data());
                    if (rc != NTP_OK) { return rc; }
                } else {
                    pinned_meta_bytes += c.meta.size();
                }
            }
        for (int k = 0; k < n_forms; ++k) {
            bool allr = true;
            for (auto& c : G->form[k].plan.chunks) allr = allr && c.d_image;
            G->form[k].all_resident = allr;
        }
        for (int k = 0; k < n_forms; ++k) {
            Form& F = G->form[k];
            if (F.plan.chunks.size() < 2) continue;
            std::vector<ReduceItem> all;
            for (auto& c : F.plan.chunks)
                if (c.n_reduce > 0 && !c.block_rows) {
                    const ReduceItem* it = reinterpret_cast<const ReduceItem*>(c.meta.data() + c.off_reduce);
                    all.insert(all.end(), it, it + c.n_reduce);
                }
            if (all.empty()) continue;
            void* p = nullptr;
            const size_t bytes = all.size() * sizeof(ReduceItem);
            if (hipMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu bytes for the split rows failed", bytes); return NTP_ENOMEM; }
            F.d_all_reduce = (ReduceItem*)p;
            F.n_all_reduce = (int)all.size();
            G->device_bytes += (int64_t)bytes;
            if (hipMemcpy(p, all.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) { (void)hipGetLastError(); set_error("upload of the split rows failed"); return NTP_EHIP; }
        }
        if (pinned_meta_bytes) {
            void* p = nullptr;
            if (hipHostMalloc(&p, pinned_meta_bytes, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); set_error("pinned allocation of %zu bytes failed", pinned_meta_bytes); return NTP_ENOMEM; }
            G->pinned_meta = (char*)p;
            size_t off = 0;
            for (int k = 0; k < n_forms; ++k)
                for (auto& c : G->form[k].plan.chunks)
                    if (!c.d_image) {
                        c.h_meta_pinned = G->pinned_meta + off;
                        memcpy(c.h_meta_pinned, c.meta.data(), c.meta.size());
                        off += c.meta.size();
                    }
        }
        // Hub tables (opt-in: NTP_AGG_HUB=1 in the environment of the build call; measured slower than
        // the plain kernel, see agg_kernels.hip): for a fully resident topology with room for 4 more
        // bytes per entry, the most gathered columns of each form get LDS slots and a second column-id
        // array names them.  A column is worth a slot when it is gathered more often than the table is
        // filled (once per compute unit and column pass): NTP_AGG_HUB_MIN_COUNT overrides the bound,
        // NTP_AGG_HUB_SLOTS the number of slots.
        const char* hub_env = getenv("NTP_AGG_HUB");
        if (fits && n > 0 && hub_env && hub_env[0] == '1') {
            int64_t min_count = 256;
            if (const char* e = getenv("NTP_AGG_HUB_MIN_COUNT")) min_count = std::max<int64_t>(1, atoll(e));
            int64_t extra = 0;
            for (int k = 0; k < n_forms; ++k) extra += G->form[k].m->nnz * 4;
            if (budget == 0 || (int64_t)all + extra <= budget) {
                for (int k = 0; k < n_forms; ++k) {
                    Form& F = G->form[k];
                    const HostSparse* transposed = k == 1 ? &G->g.csr : (G->g.symmetric ? &G->g.csr : (G->g.has_csc ? &G->g.csc : nullptr));
                    int slots = agg_hub_slots();
                    if (const char* e = getenv("NTP_AGG_HUB_SLOTS")) slots = std::max(1, std::min(slots, atoi(e)));
                    pick_hub_columns(*F.m, transposed, slots, min_count, &F.plan.hub_cols);
                    if (F.plan.hub_cols.empty()) continue;
                    void* p = nullptr;
                    const size_t hb = F.plan.hub_cols.size() * 4;
                    if (hipMalloc(&p, hb) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu bytes for the hub columns failed", hb); return NTP_ENOMEM; }
                    F.d_hub_cols = (int32_t*)p;
                    G->device_bytes += (int64_t)hb;
                    if (hipMemcpy(p, F.plan.hub_cols.data(), hb, hipMemcpyHostToDevice) != hipSuccess) { (void)hipGetLastError(); set_error("upload of the hub columns failed"); return NTP_EHIP; }
                    std::vector<int32_t> enc;
                    for (auto& c : F.plan.chunks) {
                        const size_t ne = (size_t)(c.e_end - c.e_begin);
                        if (ne == 0) continue;
                        enc.resize(ne);
                        encode_hub_columns(*F.m, F.plan.hub_cols, c.e_begin, c.e_end, enc.data());
                        if (hipMalloc(&p, ne * 4) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu bytes for the hub column ids failed", ne * 4); return NTP_ENOMEM; }
                        c.d_colidx_hub = (int32_t*)p;
                        G->device_bytes += (int64_t)(ne * 4);
                        if (hipMemcpy(p, enc.data(), ne * 4, hipMemcpyHostToDevice) != hipSuccess) { (void)hipGetLastError(); set_error("upload of the hub column ids failed"); return NTP_EHIP; }
                    }
                }
            }
        }
        bool any_streamed = false;
        for (int k = 0; k < n_forms; ++k) any_streamed = any_streamed || !G->form[k].all_resident;
        if (any_streamed && G->g.val_mode == VAL_GCN && n > 0) {
            // degrees on the device: a streamed chunk then travels without its weights
            const size_t bytes = (size_t)n * 4;
            const bool same = G->g.din == G->g.dout;
            for (int k = 0; k < (same ? 1 : 2); ++k) {
                void* p = nullptr;
                if (hipMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu bytes for the degrees failed", bytes); return NTP_ENOMEM; }
                (k == 0 ? G->d_din : G->d_dout) = (int32_t*)p;
                G->device_bytes += (int64_t)bytes;
                const std::vector<int32_t>& src_deg = k == 0 ? G->g.din : G->g.dout;
                if (hipMemcpy(p, src_deg.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) { (void)hipGetLastError(); set_error("upload of the degrees failed"); return NTP_EHIP; }
            }
            if (same) G->d_dout = G->d_din;
        }
        if (!G->h_perm.empty()) {
            void* p = nullptr;
            const size_t bytes = G->h_perm.size() * 4;
            if (hipMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu bytes for the edge permutation failed", bytes); return NTP_ENOMEM; }
            G->d_perm = (int32_t*)p;
            G->device_bytes += (int64_t)bytes;
            if (hipMemcpy(G->d_perm, G->h_perm.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) { (void)hipGetLastError(); set_error("upload of the edge permutation failed"); return NTP_EHIP; }
        }
        const hipError_t se = hipDeviceSynchronize();
        if (se != hipSuccess) { set_error("hipDeviceSynchronize failed: %s", hipGetErrorString(se)); return NTP_EHIP; }
        // partial sums of split rows: allocated here for slices of up to 256 columns, so that only a
        // call with a wider slice ever allocates (and synchronises) inside an aggregation
        for (int k = 0; k < n_forms; ++k)
            if (G->form[k].plan.n_slots > 0) {
                rc = ensure_partial(G, G->form[k], 256);
                if (rc != NTP_OK) return rc;
            }
        float* unused = nullptr;            // resolve the static scratch of this device at set-up
        rc = static_scratch(&unused);
        if (rc != NTP_OK) return rc;
    }
    *out = guard.release();
    return NTP_OK;
}

int ntp_graph_build(int64_t n, int64_t n_edges, const int32_t* src, const int32_t* dst,
                    const float* edge_weight, uint32_t flags, int64_t budget, int64_t chunk_edges,
                    ntp_graph_t** out) {
    try {       // no C++ exception may cross the C boundary
        return graph_build_impl(n, n_edges, src, dst, edge_weight, flags, budget, chunk_edges, out);
    } catch (const std::bad_alloc&) {
        set_error("out of host memory while building the graph");
        if (out) *out = nullptr;
        return NTP_ENOMEM;
    } catch (...) {
        set_error("unexpected failure while building the graph");
        if (out) *out = nullptr;
        return NTP_EINVAL;
    }
}

int ntp_graph_info(const ntp_graph_t* g, int64_t* n, int64_t* nnz, int32_t* n_chunks,
                   int32_t* is_symmetric, int64_t* max_degree) {
    if (!g) { set_error("graph handle is NULL"); return NTP_EINVAL; }
    if (n) *n = g->g.n;
    if (nnz) *nnz = g->g.csr.nnz;
    if (n_chunks) *n_chunks = (int32_t)g->form[0].plan.chunks.size();
    if (is_symmetric) *is_symmetric = g->g.symmetric ? 1 : 0;
    if (max_degree) *max_degree = g->g.csr.max_degree;
    return NTP_OK;
}

int ntp_graph_export(const ntp_graph_t* g, int which, int64_t* rowptr, int32_t* colidx, float* val) {
    if (!g) { set_error("graph handle is NULL"); return NTP_EINVAL; }
    if (which != NTP_CSR && which != NTP_CSC) { set_error("which must be NTP_CSR or NTP_CSC"); return NTP_EINVAL; }
    if (which == NTP_CSC && g->scatter_bwd()) { set_error("graph was built with NTP_SCATTER_BWD: no by-source form is stored"); return NTP_EUNSUPPORTED; }
    const HostSparse& m = *g->f(which).m;
    if (rowptr) memcpy(rowptr, m.rowptr.data(), (size_t)(m.n + 1) * 8);
    if (colidx && m.nnz) memcpy(colidx, m.colidx, (size_t)m.nnz * 4);
    if (val && m.nnz) memcpy(val, m.val, (size_t)m.nnz * 4);
    return NTP_OK;
}

int ntp_graph_export_perm(const ntp_graph_t* g, int32_t* perm) {
    if (!g || !perm) { set_error("NULL argument"); return NTP_EINVAL; }
    if (g->h_perm.empty() && g->g.csr.nnz > 0) { set_error("graph was built without NTP_EDGE_PERM"); return NTP_EUNSUPPORTED; }
    if (!g->h_perm.empty()) memcpy(perm, g->h_perm.data(), g->h_perm.size() * 4);
    return NTP_OK;
}

int ntp_graph_chunks(const ntp_graph_t* g, int which, int32_t* n_chunks, int64_t* row_begin,
                     int64_t* row_end, int64_t* entry_begin, int64_t* entry_end, int32_t* resident) {
    if (!g || !n_chunks) { set_error("graph handle or n_chunks is NULL"); return NTP_EINVAL; }
    if (which != NTP_CSR && which != NTP_CSC) { set_error("which must be NTP_CSR or NTP_CSC"); return NTP_EINVAL; }
    if (which == NTP_CSC && g->scatter_bwd()) { set_error("graph was built with NTP_SCATTER_BWD: no by-source form is stored"); return NTP_EUNSUPPORTED; }
    const auto& chunks = g->f(which).plan.chunks;
    *n_chunks = (int32_t)chunks.size();
    for (size_t i = 0; i < chunks.size(); ++i) {
        if (row_begin) row_begin[i] = chunks[i].row_begin;
        if (row_end) row_end[i] = chunks[i].row_end;
        if (entry_begin) entry_begin[i] = chunks[i].e_begin;
        if (entry_end) entry_end[i] = chunks[i].e_end;
        if (resident) resident[i] = chunks[i].d_image ? 1 : 0;
    }
    return NTP_OK;
}

int ntp_graph_stream_bytes(const ntp_graph_t* g, int which, int64_t* bytes) {
    if (!g || !bytes) { set_error("NULL argument"); return NTP_EINVAL; }
    if (which != NTP_CSR && which != NTP_CSC) { set_error("which must be NTP_CSR or NTP_CSC"); return NTP_EINVAL; }
    const Form& F = (which == NTP_CSC && g->scatter_bwd()) ? g->form[0] : g->f(which);
    const int64_t per_entry = g->streams_without_weights() ? 4 : 8;
    int64_t total = 0;
    if (!g->host_only)
        for (const Chunk& c : F.plan.chunks)
            if (!c.d_image) total += (int64_t)c.meta.size() + (c.e_end - c.e_begin) * per_entry;
    *bytes = total;
    return NTP_OK;
}

int ntp_graph_device_bytes(const ntp_graph_t* g, int64_t* bytes) {
    if (!g || !bytes) { set_error("NULL argument"); return NTP_EINVAL; }
    *bytes = g->device_bytes;
    return NTP_OK;
}

// static_partial: run on the library's static scratch instead of the handle's (no allocation)
static int aggregate_resident(ntp_graph_t* g, int which, const void* X, void* Y, int64_t f,
                              int64_t ldx, int64_t ldy, int dtype, void* stream, const float* weights = nullptr,
                              const int32_t* columns = nullptr, bool static_partial = false) {
    int rc = check_agg_args(g, X, Y, f, ldx, ldy, dtype);
    if (rc != NTP_OK) return rc;
    Form& F = g->f(which);
    const bool scatter = which == NTP_CSC && g->scatter_bwd();
    if (scatter && dtype != NTP_F32) { set_error("the scatter backward (NTP_SCATTER_BWD) takes fp32 buffers only"); return NTP_EUNSUPPORTED; }
    if (!F.all_resident) { set_error("topology is not fully device-resident: use ntp_chunked_aggregate"); return NTP_EBUDGET; }
    if (g->g.n == 0) return NTP_OK;
    float* partial = nullptr;
    if (static_partial) {
        const size_t need = partial_floats(F, f) * sizeof(float);
        if (need > (size_t)NTP_NOALLOC_SCRATCH_BYTES) {
            set_error("the split rows of this graph need %zu bytes of partial sums at width %lld: more than the %lld-byte static scratch "
                      "(use ntp_aggregate_fwd)", need, (long long)f, (long long)NTP_NOALLOC_SCRATCH_BYTES);
            return NTP_EUNSUPPORTED;
        }
        rc = static_scratch(&partial);
    } else if (scatter) {
        rc = launch_zero_rows(Y, g->g.n, f, ldy, dtype, stream);
    } else {
        rc = ensure_partial(g, F, f);
        partial = g->partial;
    }
    if (rc != NTP_OK) return rc;
    for (auto& c : F.plan.chunks) {
        rc = run_chunk(c, c.d_image, X, Y, partial, f, ldx, ldy, dtype, (hipStream_t)stream, scatter, weights, columns, F.one_reduce(),
                       F.d_hub_cols, (int)F.plan.hub_cols.size());
        if (rc != NTP_OK) return rc;
    }
    if (!scatter && F.one_reduce()) return reduce_all(F, partial, Y, f, ldy, dtype, (hipStream_t)stream);
    return NTP_OK;
}

int ntp_aggregate_fwd(ntp_graph_t* g, const void* X, void* Y, int64_t f, int64_t ldx, int64_t ldy,
                      int dtype, void* stream) {
    return aggregate_resident(g, NTP_CSR, X, Y, f, ldx, ldy, dtype, stream);
}

int ntp_aggregate_fwd_noalloc(ntp_graph_t* g, const void* X, void* Y, int64_t f, int64_t ldx, int64_t ldy,
                              int dtype, void* stream) {
    return aggregate_resident(g, NTP_CSR, X, Y, f, ldx, ldy, dtype, stream, nullptr, nullptr, true);
}

int ntp_aggregate_bwd(ntp_graph_t* g, const void* Gout, void* Gin, int64_t f, int64_t ldo, int64_t ldi,
                      int dtype, void* stream) {
    return aggregate_resident(g, NTP_CSC, Gout, Gin, f, ldo, ldi, dtype, stream);
}

static int chunked_multi(ntp_graph_t* g, int direction, int32_t n_rhs,
                         const void* const* X, void* const* Y, int64_t f,
                         int64_t ldx, int64_t ldy, int dtype, void* compute_stream, void* copy_stream, const Epilogue& epi) {
    if (n_rhs < 1 || n_rhs > 64) { set_error("n_rhs must be in 1..64"); return NTP_EINVAL; }
    if (!X || !Y) { set_error("X or Y is NULL"); return NTP_EINVAL; }
    int rc;
    for (int r = 0; r < n_rhs; ++r) {
        rc = check_agg_args(g, X[r], Y[r], f, ldx, ldy, dtype, false);
        if (rc != NTP_OK) return rc;
        const int64_t es = dtype == NTP_BF16 ? 2 : 4;
        for (int q = 0; q < n_rhs; ++q)
            if (q != r && views_overlap(X[q], ldx, Y[r], ldy, g->g.n, f, es)) { set_error("an output overlaps an input"); return NTP_EINVAL; }
        for (int q = 0; q < r; ++q)
            if (views_overlap(Y[q], ldy, Y[r], ldy, g->g.n, f, es)) { set_error("two outputs overlap"); return NTP_EINVAL; }
    }
    if (direction != NTP_FWD && direction != NTP_BWD) { set_error("direction must be NTP_FWD or NTP_BWD"); return NTP_EINVAL; }
    if (g->host_only) { set_error("graph was built with NTP_HOST_ONLY: nothing is on the device"); return NTP_EBUDGET; }
    Form& F = g->f(direction == NTP_FWD ? NTP_CSR : NTP_CSC);
    const bool scatter = direction == NTP_BWD && g->scatter_bwd();
    if (scatter && dtype != NTP_F32) { set_error("the scatter backward (NTP_SCATTER_BWD) takes fp32 buffers only"); return NTP_EUNSUPPORTED; }
    if (g->g.n == 0) return NTP_OK;
    hipStream_t cs = (hipStream_t)compute_stream, xs = (hipStream_t)copy_stream;
    if (!F.all_resident && cs == xs) { set_error("copy_stream must differ from compute_stream when chunks are streamed"); return NTP_EINVAL; }
    if (scatter) {
        for (int r = 0; r < n_rhs && rc == NTP_OK; ++r) rc = launch_zero_rows(Y[r], g->g.n, f, ldy, dtype, cs);
    } else {
        rc = ensure_partial(g, F, f, n_rhs);
    }
    if (rc != NTP_OK) return rc;
    const size_t pstride = scatter ? 0 : partial_floats(F, f);
    // every chunk is brought in once and applied to all right-hand sides before the next one
    auto run_all = [&](const Chunk& c, const char* img) -> int {
        for (int r = 0; r < n_rhs; ++r) {
            const int e = run_chunk(c, img, X[r], Y[r], scatter ? nullptr : g->partial + (size_t)r * pstride, f, ldx, ldy, dtype, cs, scatter,
                                    nullptr, nullptr, F.one_reduce(), F.d_hub_cols, (int)F.plan.hub_cols.size(), epi);
            if (e != NTP_OK) return e;
        }
        return NTP_OK;
    };
    for (auto& c : F.plan.chunks) {
        if (c.d_image) {
            rc = run_all(c, c.d_image);
            if (rc != NTP_OK) return rc;
            continue;
        }
        const int b = g->next_stage;
        g->next_stage ^= 1;
        // the buffer may still be read by the kernels of the chunk that used it last
        if (g->stage_used[b]) HIP_TRY(hipStreamWaitEvent(xs, g->ev_free[b], 0));
        const bool rebuild = g->streams_without_weights();
        rc = upload_chunk(*F.m, c, g->stage[b], xs, true, c.h_meta_pinned, !rebuild);
        if (rc != NTP_OK) return rc;
        HIP_TRY(hipEventRecord(g->ev_ready[b], xs));
        HIP_TRY(hipStreamWaitEvent(cs, g->ev_ready[b], 0));
        if (rebuild) {
            const bool by_source = &F == &g->form[1];          // rows are sources: row degree = dout, column degree = din
            char* img = g->stage[b];
            rc = launch_rebuild_weights(reinterpret_cast<const int64_t*>(img + c.off_rowptr), c.row_begin, c.row_end - c.row_begin,
                                        c.e_begin, c.e_end - c.e_begin, reinterpret_cast<const int32_t*>(img + c.img_off_colidx),
                                        reinterpret_cast<float*>(img + c.img_off_val), by_source ? g->d_dout : g->d_din,
                                        by_source ? g->d_din : g->d_dout, g->g.val_mode, cs);
            if (rc != NTP_OK) return rc;
        }
        rc = run_all(c, g->stage[b]);
        if (rc != NTP_OK) return rc;
        HIP_TRY(hipEventRecord(g->ev_free[b], cs));
        g->stage_used[b] = true;
    }
    if (!scatter && F.one_reduce())
        for (int r = 0; r < n_rhs; ++r) {
            rc = reduce_all(F, g->partial + (size_t)r * pstride, Y[r], f, ldy, dtype, cs, epi);
            if (rc != NTP_OK) return rc;
        }
    return NTP_OK;
}

int ntp_chunked_aggregate_multi(ntp_graph_t* g, int direction, int32_t n_rhs,
                                const void* const* X, void* const* Y, int64_t f,
                                int64_t ldx, int64_t ldy, int dtype, void* compute_stream, void* copy_stream) {
    return chunked_multi(g, direction, n_rhs, X, Y, f, ldx, ldy, dtype, compute_stream, copy_stream, Epilogue());
}

int ntp_aggregate_act(ntp_graph_t* g, int direction, const void* X, void* Y, int64_t f, int64_t ldx, int64_t ldy,
                      int dtype, int act, const void* M, int64_t ldm, void* compute_stream, void* copy_stream) {
    if (act != NTP_ACT_NONE && act != NTP_ACT_RELU) { set_error("unknown activation %d", act); return NTP_EINVAL; }
    Epilogue epi;
    if (act == NTP_ACT_RELU) {
        epi.on = true;
        epi.M = M;
        epi.ldm = M ? ldm : 0;
        if (M && ldm < f) { set_error("row stride of the mask smaller than the slice width"); return NTP_EINVAL; }
        if (M && g && g->g.n > 0 && views_overlap(M, ldm, Y, ldy, g->g.n, f, dtype == NTP_BF16 ? 2 : 4)) {
            set_error("the mask and the output must not overlap");
            return NTP_EINVAL;
        }
        if (g && direction == NTP_BWD && g->scatter_bwd()) {
            set_error("graph was built with NTP_SCATTER_BWD: the scatter-add backward has no epilogue (use ntp_relu_bwd)");
            return NTP_EUNSUPPORTED;
        }
    }
    return chunked_multi(g, direction, 1, &X, &Y, f, ldx, ldy, dtype, compute_stream, copy_stream, epi);
}

int ntp_chunked_aggregate(ntp_graph_t* g, int direction, const void* X, void* Y, int64_t f,
                          int64_t ldx, int64_t ldy, int dtype, void* compute_stream, void* copy_stream) {
    return ntp_chunked_aggregate_multi(g, direction, 1, &X, &Y, f, ldx, ldy, dtype, compute_stream, copy_stream);
}

int ntp_aggregate_weighted(ntp_graph_t* g, int direction, const float* weights, const void* X, void* Y,
                           int64_t f, int64_t ldx, int64_t ldy, int dtype, void* stream) {
    if (direction != NTP_FWD && direction != NTP_BWD) { set_error("direction must be NTP_FWD or NTP_BWD"); return NTP_EINVAL; }
    if (g && g->g.csr.nnz > 0 && !weights) { set_error("weights is NULL"); return NTP_EINVAL; }
    return aggregate_resident(g, direction == NTP_FWD ? NTP_CSR : NTP_CSC, X, Y, f, ldx, ldy, dtype, stream, weights);
}

int ntp_edge_softmax(ntp_graph_t* g, const float* p, const float* q, float negative_slope,
                     float* alpha_in, float* alpha_out, void* stream) {
    if (!g) { set_error("graph handle is NULL"); return NTP_EINVAL; }
    if (g->host_only) { set_error("graph was built with NTP_HOST_ONLY: nothing is on the device"); return NTP_EBUDGET; }
    if (!(negative_slope >= 0.f) || !(negative_slope <= 1.f)) { set_error("negative_slope must be in [0, 1]"); return NTP_EINVAL; }
    const int64_t n = g->g.n;
    if (n == 0) return NTP_OK;
    if (!p || !q || !alpha_in) { set_error("p, q or alpha_in is NULL"); return NTP_EINVAL; }
    if (alpha_out && g->scatter_bwd()) { set_error("graph was built with NTP_SCATTER_BWD: no by-source form is stored"); return NTP_EUNSUPPORTED; }
    Form& Fin = g->f(NTP_CSR);
    Form& Fout = g->f(NTP_CSC);
    if (!Fin.all_resident || (alpha_out && !Fout.all_resident)) {
        set_error("attention weights need every chunk of the topology device-resident");
        return NTP_EBUDGET;
    }
    // scratch kept by the handle: 16 bytes per vertex + 8 bytes per segment of a split row
    const int64_t seg_floats = 2 * Fin.plan.n_slots;
    if (!g->att_stats) {
        void* ptr = nullptr;
        const size_t bytes = (size_t)n * 16 + (size_t)seg_floats * 4 + 16;
        if (hipMalloc(&ptr, bytes) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu bytes failed", bytes); return NTP_ENOMEM; }
        g->att_stats = (float*)ptr;
        g->device_bytes += (int64_t)bytes;
    }
    float* seg_stats = g->att_stats + 4 * n;
    // chunk by chunk, phase by phase (a split row's segments may lie in several chunks)
    auto run = [&](const Form& F, float* out, bool transposed) -> int {
        for (int phase = transposed ? 2 : 0; phase < 3; ++phase)
            for (const Chunk& c : F.plan.chunks) {
                AttArgs a;
                a.rowptr = reinterpret_cast<const int64_t*>(c.d_image + c.off_rowptr) - c.row_begin;
                a.colidx = reinterpret_cast<const int32_t*>(c.d_image + c.img_off_colidx) - c.e_begin;
                a.rows = reinterpret_cast<const int32_t*>(c.d_image + c.off_rows);
                a.p = p; a.q = q;
                a.st = g->att_stats;
                a.alpha = out;
                a.slope = negative_slope;
                const int rc = launch_attention(a, c.bin_row_off, c.bin_count,
                                                reinterpret_cast<const Segment*>(c.d_image + c.off_segs), c.n_segs,
                                                reinterpret_cast<const ReduceItem*>(c.d_image + c.off_reduce), c.n_reduce,
                                                seg_stats, transposed, phase, stream);
                if (rc != NTP_OK) return rc;
            }
        return NTP_OK;
    };
    int rc = run(Fin, alpha_in, false);
    if (rc == NTP_OK && alpha_out) rc = run(Fout, alpha_out, true);
    return rc;
}

int ntp_edge_softmax_bwd(ntp_graph_t* g, const float* p, const float* q, float negative_slope,
                         const float* alpha_in, const float* alpha_out, const float* Z, const float* dY,
                         int64_t m, int64_t ldz, int64_t lddy, float* dp, float* dq, int accumulate, void* stream) {
    if (!g) { set_error("graph handle is NULL"); return NTP_EINVAL; }
    if (g->host_only) { set_error("graph was built with NTP_HOST_ONLY: nothing is on the device"); return NTP_EBUDGET; }
    if (!(negative_slope >= 0.f) || !(negative_slope <= 1.f)) { set_error("negative_slope must be in [0, 1]"); return NTP_EINVAL; }
    if (m < 1 || m > 1024 || ldz < m || lddy < m) { set_error("bad feature shape m=%lld ldz=%lld lddy=%lld (1 <= m <= 1024)", (long long)m, (long long)ldz, (long long)lddy); return NTP_EINVAL; }
    const int64_t n = g->g.n;
    if (n == 0) return NTP_OK;
    if (!p || !q || !alpha_in || !alpha_out || !Z || !dY || !dp || !dq) { set_error("NULL buffer"); return NTP_EINVAL; }
    if (g->scatter_bwd()) { set_error("graph was built with NTP_SCATTER_BWD: no by-source form is stored"); return NTP_EUNSUPPORTED; }
    Form& Fin = g->f(NTP_CSR);
    Form& Fout = g->f(NTP_CSC);
    if (!Fin.all_resident || !Fout.all_resident) {
        set_error("the attention gradient needs every chunk of the topology device-resident");
        return NTP_EBUDGET;
    }
    // scratch kept by the handle: (t, q) of every destination, one partial sum per segment of a
    // split row, one dp per vertex, dalpha of every edge
    const int64_t nnz = g->g.csr.nnz;
    const int64_t n_slots = std::max(Fin.plan.n_slots, Fout.plan.n_slots);
    if (!g->att_bwd) {
        void* ptr = nullptr;
        // the per-edge array is also read as a one-column feature matrix indexed by ids below n
        const size_t bytes = ((size_t)std::max(nnz, n) + 3 * (size_t)n + (size_t)n_slots) * 4 + 16;
        if (hipMalloc(&ptr, bytes) != hipSuccess) { (void)hipGetLastError(); set_error("device allocation of %zu bytes failed", bytes); return NTP_ENOMEM; }
        g->att_bwd = (float*)ptr;
        g->device_bytes += (int64_t)bytes;
    }
    float* t = g->att_bwd;              // (t, q) pairs
    float* slots = t + 2 * n;
    float* dp_round = slots + n_slots;  // [n] this call's dp when it is added to the caller's
    float* park = dp_round + n;
    const bool by_perm = g->d_perm != nullptr;
    // chunk by chunk, phase by phase (a split row's segments may lie in several chunks)
    auto run = [&](const Form& F, bool transposed) -> int {
        for (int phase = 0; phase < (transposed ? 2 : 4); ++phase)
            for (const Chunk& c : F.plan.chunks) {
                AttBwdArgs a;
                a.rowptr = reinterpret_cast<const int64_t*>(c.d_image + c.off_rowptr) - c.row_begin;
                a.colidx = reinterpret_cast<const int32_t*>(c.d_image + c.img_off_colidx) - c.e_begin;
                a.rows = reinterpret_cast<const int32_t*>(c.d_image + c.off_rows);
                a.p = p; a.q = q;
                a.alpha = transposed ? alpha_out : alpha_in;
                a.own = transposed ? Z : dY;
                a.ld_own = transposed ? ldz : lddy;
                a.other = transposed ? dY : Z;
                a.ld_other = transposed ? lddy : ldz;
                a.t = t;
                a.park = park;
                a.out = transposed ? dp : dq;
                a.slots = slots;
                a.slope = negative_slope;
                a.m = (int32_t)m;
                a.accumulate = accumulate ? 1 : 0;
                a.keep_w = by_perm ? 1 : 0;
                AttBwdRows r;
                r.n_group_rows = c.bin_row_off[NBINS - 1];
                r.n_block_rows = c.bin_count[NBINS - 1];
                r.segs = reinterpret_cast<const Segment*>(c.d_image + c.off_segs);
                r.n_segs = c.n_segs;
                r.split_rows = reinterpret_cast<const ReduceItem*>(c.d_image + c.off_reduce);
                r.n_split_rows = c.n_reduce;
                const int rc = launch_attention_bwd(a, r, transposed, phase, stream);
                if (rc != NTP_OK) return rc;
            }
        return NTP_OK;
    };
    int rc = run(Fin, false);           // dq and t first: the by-source pass reads t
    if (rc != NTP_OK) return rc;
    if (!by_perm) return run(Fout, true);
    // every edge's w = (dalpha - t) * LeakyReLU' now sits in park, in by-destination order:
    // dp[u] = sum over the out-edges of alpha w is a one-column aggregation over the by-source
    // form whose column ids are the edges' by-destination positions
    float* dst = accumulate ? dp_round : dp;
    rc = aggregate_resident(g, NTP_CSC, park, dst, 1, 1, 1, NTP_F32, stream, alpha_out, g->d_perm);
    if (rc == NTP_OK && accumulate) rc = launch_vec_add(dp, dp_round, n, stream);
    return rc;
}

int ntp_attention_scores_fwd(const float* Z, const float* a_src, const float* a_dst, float* p, float* q,
                             int64_t n, int64_t m, int64_t ldz, void* stream) {
    if (n < 0 || m < 1 || m > attention_scores_max_width() || ldz < m) {
        set_error("bad shape n=%lld m=%lld ldz=%lld (1 <= m <= %lld)", (long long)n, (long long)m, (long long)ldz, (long long)attention_scores_max_width());
        return NTP_EINVAL;
    }
    if (n == 0) return NTP_OK;
    if (!Z || !a_src || !a_dst || !p || !q) { set_error("NULL buffer"); return NTP_EINVAL; }
    return launch_attention_scores_fwd(Z, a_src, a_dst, p, q, n, m, ldz, stream);
}

int64_t ntp_attention_scores_bwd_scratch_bytes(int64_t n, int64_t m) { return attention_scores_bwd_scratch_bytes(n, m); }

int ntp_attention_scores_bwd(const float* Z, const float* a_src, const float* a_dst, const float* dp, const float* dq,
                             float* dZ, float* da_src, float* da_dst, int64_t n, int64_t m, int64_t ldz, int64_t lddz,
                             void* scratch, int64_t scratch_bytes, void* stream) {
    if (n < 0 || m < 1 || m > attention_scores_max_width() || ldz < m || lddz < m) {
        set_error("bad shape n=%lld m=%lld ldz=%lld lddz=%lld (1 <= m <= %lld)", (long long)n, (long long)m, (long long)ldz, (long long)lddz,
                  (long long)attention_scores_max_width());
        return NTP_EINVAL;
    }
    if (!a_src || !a_dst || !da_src || !da_dst) { set_error("NULL buffer"); return NTP_EINVAL; }
    if (n > 0 && (!Z || !dp || !dq || !dZ)) { set_error("NULL buffer"); return NTP_EINVAL; }
    if (n == 0) return launch_zero_rows(da_src, 1, m, m, NTP_F32, stream) || launch_zero_rows(da_dst, 1, m, m, NTP_F32, stream);
    const int64_t need = attention_scores_bwd_scratch_bytes(n, m);
    if (!scratch || scratch_bytes < need) { set_error("scratch too small: need %lld bytes", (long long)need); return NTP_EINVAL; }
    return launch_attention_scores_bwd(Z, a_src, a_dst, dp, dq, dZ, da_src, da_dst, n, m, ldz, lddz, (float*)scratch, stream);
}

int ntp_nn_fwd(const void* A, const void* W, void* H, int64_t n, int64_t k, int64_t m,
               int act, int dtype, void* stream) {
    if (n < 0 || k < 1 || m < 1 || k > 65536 || m > 65536) { set_error("bad transform shape n=%lld k=%lld m=%lld", (long long)n, (long long)k, (long long)m); return NTP_EINVAL; }
    if (n == 0) return NTP_OK;
    if (!A || !W || !H) { set_error("NULL buffer"); return NTP_EINVAL; }
    if (act != NTP_ACT_NONE && act != NTP_ACT_RELU) { set_error("unknown activation %d", act); return NTP_EINVAL; }
    if (dtype != NTP_F32 && dtype != NTP_BF16) { set_error("unknown dtype %d", dtype); return NTP_EINVAL; }
    return launch_nn_fwd(A, W, H, n, k, m, act, dtype, stream);
}

int ntp_nn_bwd(const void* A, const void* W, const void* H, const void* dH, void* dA, float* dW,
               int64_t n, int64_t k, int64_t m, int act, int dtype,
               void* workspace, int64_t workspace_bytes, void* stream) {
    if (n < 0 || k < 1 || m < 1 || k > 65536 || m > 65536) { set_error("bad transform shape n=%lld k=%lld m=%lld", (long long)n, (long long)k, (long long)m); return NTP_EINVAL; }
    if (!dW && !dA) { set_error("dW and dA are both NULL: nothing to compute"); return NTP_EINVAL; }
    if (n > 0 && (!A || !dH || (dA && !W) || (act == NTP_ACT_RELU && !H))) { set_error("NULL buffer"); return NTP_EINVAL; }
    if (act != NTP_ACT_NONE && act != NTP_ACT_RELU) { set_error("unknown activation %d", act); return NTP_EINVAL; }
    if (dtype != NTP_F32 && dtype != NTP_BF16) { set_error("unknown dtype %d", dtype); return NTP_EINVAL; }
    if (dW && (workspace_bytes < nn_bwd_workspace_bytes(n, k, m) || (!workspace && nn_bwd_workspace_bytes(n, k, m) > 0))) {
        set_error("workspace too small: need %lld bytes", (long long)nn_bwd_workspace_bytes(n, k, m));
        return NTP_EINVAL;
    }
    return launch_nn_bwd(A, W, H, dH, dA, dW, n, k, m, act, dtype, workspace, workspace_bytes, stream);
}

int64_t ntp_softmax_xent_scratch_bytes(int64_t n) { return n < 0 ? 0 : (n + 1024) * 4; }

int ntp_softmax_xent(const float* Z, const int64_t* labels, float* dZ, float* loss, void* scratch, int64_t scratch_bytes,
                     int64_t n, int64_t c, int64_t ldz, int64_t lddz, void* stream) {
    if (n < 1 || c < 1 || c > 65536 || ldz < c || lddz < c) { set_error("bad loss shape n=%lld c=%lld ldz=%lld lddz=%lld", (long long)n, (long long)c, (long long)ldz, (long long)lddz); return NTP_EINVAL; }
    if (!Z || !labels || !dZ || !loss) { set_error("NULL buffer"); return NTP_EINVAL; }
    if (!scratch || scratch_bytes < ntp_softmax_xent_scratch_bytes(n)) { set_error("scratch too small: need %lld bytes", (long long)ntp_softmax_xent_scratch_bytes(n)); return NTP_EINVAL; }
    return launch_softmax_xent(Z, labels, dZ, loss, static_cast<float*>(scratch), n, c, ldz, lddz, stream);
}

int ntp_relu_fwd(void* H, int64_t n, int64_t f, int64_t ld, int dtype, void* stream) {
    if (n < 0 || f < 1 || ld < f) { set_error("bad activation shape n=%lld f=%lld ld=%lld", (long long)n, (long long)f, (long long)ld); return NTP_EINVAL; }
    if (dtype != NTP_F32 && dtype != NTP_BF16) { set_error("unknown dtype %d", dtype); return NTP_EINVAL; }
    if (n > 0 && !H) { set_error("NULL buffer"); return NTP_EINVAL; }
    return launch_relu(nullptr, nullptr, H, n, f, ld, dtype, false, stream);
}

int ntp_relu_bwd(const void* dH, const void* H, void* dZ, int64_t n, int64_t f, int64_t ld, int dtype, void* stream) {
    if (n < 0 || f < 1 || ld < f) { set_error("bad activation shape n=%lld f=%lld ld=%lld", (long long)n, (long long)f, (long long)ld); return NTP_EINVAL; }
    if (dtype != NTP_F32 && dtype != NTP_BF16) { set_error("unknown dtype %d", dtype); return NTP_EINVAL; }
    if (n > 0 && (!dH || !H || !dZ)) { set_error("NULL buffer"); return NTP_EINVAL; }
    return launch_relu(dH, H, dZ, n, f, ld, dtype, true, stream);
}

int64_t ntp_nn_bwd_workspace_bytes(int64_t n, int64_t k, int64_t m) { return nn_bwd_workspace_bytes(n, k, m); }

void ntp_graph_free(ntp_graph_t* g) { destroy(g); }

}  // extern "C"
