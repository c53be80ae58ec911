// Host-side construction of the per-worker topology: the normalised adjacency of
// Section 4.1.3 in both compressed forms (by destination for eq. 1/3, by source for the
// backward pass of Section 4.2.1).  Pure C++, no device code.
//
// Processing order (fixed, so that the result is reproducible bit for bit):
//   input edges in input order; reversed copies after all originals (SYMMETRISE);
//   input self loops dropped and the first of equal (src,dst) kept (DEDUP);
//   one (v,v) entry of weight 1 per vertex appended last (ADD_SELF_LOOPS);
//   rows sorted by neighbour id, stable.
#include "ntp_internal.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <thread>

namespace ntp {

// ---------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}
const char* last_error() { return g_err; }

int host_threads() {
    unsigned hc = std::thread::hardware_concurrency();
    int t = hc ? (int)hc : 4;
    if (const char* e = getenv("NTP_HOST_THREADS")) t = atoi(e);
    return std::max(1, std::min(t, 32));
}

void parallel_run(int n_threads, void (*fn)(int, int, void*), void* ctx) {
    if (n_threads <= 1) { fn(0, 1, ctx); return; }
    std::vector<std::thread> th;
    th.reserve(n_threads - 1);
    for (int t = 1; t < n_threads; ++t) th.emplace_back(fn, t, n_threads, ctx);
    fn(0, n_threads, ctx);
    for (auto& x : th) x.join();
}

namespace {

struct Entry { int32_t nb; float w; };   // neighbour id + raw weight, in edge order within a row

// Exclusive prefix sum of counts into ptr[0..n]; returns the total.
int64_t prefix(const std::vector<int64_t>& cnt, std::vector<int64_t>& ptr) {
    int64_t s = 0;
    const size_t n = cnt.size();
    ptr.resize(n + 1);
    for (size_t i = 0; i < n; ++i) { ptr[i] = s; s += cnt[i]; }
    ptr[n] = s;
    return s;
}

// Walk the conceptual edge sequence (originals, then reversed copies) restricted to major
// ids in [lo, hi) and call f(major, minor, weight) in sequence order.  "major" is the
// destination for the by-destination form.
template <class F>
void for_edges_in_range(int64_t n_edges, const int32_t* src, const int32_t* dst, const float* w,
                        bool symmetrise, bool drop_loops, int64_t lo, int64_t hi, F&& f) {
    for (int64_t i = 0; i < n_edges; ++i) {
        const int32_t s = src[i], d = dst[i];
        if (d >= lo && d < hi && !(drop_loops && s == d)) f(d, s, w ? w[i] : 1.0f);
    }
    if (symmetrise)
        for (int64_t i = 0; i < n_edges; ++i) {
            const int32_t s = dst[i], d = src[i];   // reversed copy
            if (d >= lo && d < hi && !(drop_loops && s == d)) f(d, s, w ? w[i] : 1.0f);
        }
}

}  // namespace

int build_host_graph(int64_t n, int64_t n_edges, const int32_t* src, const int32_t* dst,
                     const float* edge_weight, uint32_t flags, EntryAllocator alloc,
                     BuiltGraph* out) {
    const bool symmetrise = flags & NTP_SYMMETRISE;
    const bool dedup = flags & NTP_DEDUP;
    const bool loops = flags & NTP_ADD_SELF_LOOPS;
    const bool norm = flags & NTP_NORM_GCN_SYM;
    const int T = host_threads();

    // ---- validate ids
    std::atomic<int64_t> bad{-1};
    parallel_for_threads(T, [&](int t, int nt) {
        const int64_t a = n_edges * t / nt, b = n_edges * (t + 1) / nt;
        for (int64_t i = a; i < b; ++i)
            if (src[i] < 0 || src[i] >= n || dst[i] < 0 || dst[i] >= n) { bad.store(i); break; }
    });
    if (bad.load() >= 0) {
        set_error("edge %lld has a vertex id outside [0, %lld)", (long long)bad.load(), (long long)n);
        return NTP_EINVAL;
    }

    // ---- pass 1: entries per destination row, in sequence order (threads own row ranges)
    std::vector<int64_t> cnt(n, 0), tptr;
    parallel_for_threads(T, [&](int t, int nt) {
        const int64_t lo = n * t / nt, hi = n * (t + 1) / nt;
        for_edges_in_range(n_edges, src, dst, nullptr, symmetrise, dedup, lo, hi,
                           [&](int32_t d, int32_t, float) { ++cnt[d]; });
    });
    const int64_t total_raw = prefix(cnt, tptr);
    std::vector<Entry> raw;
    try { raw.resize((size_t)total_raw); } catch (...) { set_error("out of host memory (%lld raw entries)", (long long)total_raw); return NTP_ENOMEM; }
    {
        std::vector<int64_t> fill(tptr.begin(), tptr.end() - 1);
        parallel_for_threads(T, [&](int t, int nt) {
            const int64_t lo = n * t / nt, hi = n * (t + 1) / nt;
            for_edges_in_range(n_edges, src, dst, edge_weight, symmetrise, dedup, lo, hi,
                               [&](int32_t d, int32_t s, float w) { raw[(size_t)fill[d]++] = Entry{s, w}; });
        });
    }

    // ---- pass 2: sort each row by neighbour (stable), dedup (keep first), count final lengths
    std::vector<int64_t> len(n, 0);
    std::atomic<int64_t> next{0};
    const int64_t grain = 1024;
    parallel_for_threads(T, [&](int, int) {
        for (;;) {
            const int64_t r0 = next.fetch_add(grain);
            if (r0 >= n) break;
            const int64_t r1 = std::min(n, r0 + grain);
            for (int64_t r = r0; r < r1; ++r) {
                Entry* a = raw.data() + tptr[r];
                Entry* b = raw.data() + tptr[r + 1];
                std::stable_sort(a, b, [](const Entry& x, const Entry& y) { return x.nb < y.nb; });
                if (dedup) b = std::unique(a, b, [](const Entry& x, const Entry& y) { return x.nb == y.nb; });
                len[r] = (b - a) + (loops ? 1 : 0);
            }
        }
    });

    HostSparse& R = out->csr;
    R.n = n;
    R.nnz = prefix(len, R.rowptr);
    R.colidx = (int32_t*)alloc.alloc(std::max<size_t>(4, (size_t)R.nnz * 4), alloc.ctx);
    // without caller weights the values follow from the structure and are rebuilt on the device for
    // streamed chunks: they need not sit in pinned memory
    auto alloc_val = edge_weight ? alloc.alloc : alloc.alloc_val;
    R.val = (float*)alloc_val(std::max<size_t>(4, (size_t)R.nnz * 4), alloc.ctx);
    if (!R.colidx || !R.val) { set_error("out of host memory for %lld entries", (long long)R.nnz); return NTP_ENOMEM; }

    // ---- pass 3: write the final rows; the self loop goes after every entry with id <= v
    next = 0;
    parallel_for_threads(T, [&](int, int) {
        for (;;) {
            const int64_t r0 = next.fetch_add(grain);
            if (r0 >= n) break;
            const int64_t r1 = std::min(n, r0 + grain);
            for (int64_t r = r0; r < r1; ++r) {
                const Entry* a = raw.data() + tptr[r];
                const int64_t m = len[r] - (loops ? 1 : 0);
                int64_t o = R.rowptr[r];
                bool placed = !loops;
                for (int64_t i = 0; i < m; ++i) {
                    if (!placed && a[i].nb > r) { R.colidx[o] = (int32_t)r; R.val[o] = 1.0f; ++o; placed = true; }
                    R.colidx[o] = a[i].nb; R.val[o] = a[i].w; ++o;
                }
                if (!placed) { R.colidx[o] = (int32_t)r; R.val[o] = 1.0f; ++o; }
            }
        }
    });
    raw.clear(); raw.shrink_to_fit();
    R.max_degree = 0;
    for (int64_t r = 0; r < n; ++r) R.max_degree = std::max(R.max_degree, len[r]);

    // With unit weights and SYMMETRISE the entry multiset is its own transpose and both
    // degree arrays coincide, so the by-source form equals the by-destination form.
    const bool known_symmetric = symmetrise && edge_weight == nullptr;

    // NTP_SCATTER_BWD: the backward pass scatters over the by-destination rows (Section 4.2.1),
    // so the by-source form is not stored; its row lengths are still needed for the weights.
    const bool want_csc = !(flags & NTP_SCATTER_BWD);
    HostSparse& C = out->csc;
    std::vector<int64_t> dout;          // by-source row lengths
    if (!known_symmetric && !want_csc) {
        dout.assign(n, 0);
        parallel_for_threads(T, [&](int t, int nt) {
            const int64_t lo = n * t / nt, hi = n * (t + 1) / nt;
            for (int64_t e = 0; e < R.nnz; ++e) { const int32_t u = R.colidx[e]; if (u >= lo && u < hi) ++dout[u]; }
        });
    }
    if (!known_symmetric && want_csc) {
        // ---- by-source form = transpose of the final entries, rows of C filled in CSR order
        std::vector<int64_t> ccnt(n, 0);
        parallel_for_threads(T, [&](int t, int nt) {
            const int64_t lo = n * t / nt, hi = n * (t + 1) / nt;
            for (int64_t e = 0; e < R.nnz; ++e) { const int32_t u = R.colidx[e]; if (u >= lo && u < hi) ++ccnt[u]; }
        });
        C.n = n;
        C.nnz = prefix(ccnt, C.rowptr);
        C.colidx = (int32_t*)alloc.alloc(std::max<size_t>(4, (size_t)C.nnz * 4), alloc.ctx);
        C.val = (float*)alloc_val(std::max<size_t>(4, (size_t)C.nnz * 4), alloc.ctx);
        if (!C.colidx || !C.val) { set_error("out of host memory for %lld entries", (long long)C.nnz); return NTP_ENOMEM; }
        std::vector<int64_t> fill(C.rowptr.begin(), C.rowptr.end() - 1);
        parallel_for_threads(T, [&](int t, int nt) {
            const int64_t lo = n * t / nt, hi = n * (t + 1) / nt;
            // rows v ascending, entries in order: each by-source row receives v ascending
            int64_t v = 0;
            for (int64_t e = 0; e < R.nnz; ++e) {
                while (R.rowptr[v + 1] <= e) ++v;
                const int32_t u = R.colidx[e];
                if (u >= lo && u < hi) { const int64_t p = fill[u]++; C.colidx[p] = (int32_t)v; C.val[p] = R.val[e]; }
            }
        });
        C.max_degree = 0;
        for (int64_t r = 0; r < n; ++r) C.max_degree = std::max(C.max_degree, ccnt[r]);
        dout.swap(ccnt);
    }

    // ---- weights: (float)((double)w * (1 / sqrt(din(v) * dout(u))))
    if (norm) {
        const std::vector<int64_t>& d_out = known_symmetric ? len : dout;
        auto scale_rows = [&](HostSparse& M, const std::vector<int64_t>& d_row, const std::vector<int64_t>& d_col) {
            next = 0;
            parallel_for_threads(T, [&](int, int) {
                for (;;) {
                    const int64_t r0 = next.fetch_add(grain);
                    if (r0 >= n) break;
                    const int64_t r1 = std::min(n, r0 + grain);
                    for (int64_t r = r0; r < r1; ++r)
                        for (int64_t e = M.rowptr[r]; e < M.rowptr[r + 1]; ++e) {
                            const double prod = (double)d_row[r] * (double)d_col[M.colidx[e]];
                            const double scale = 1.0 / std::sqrt(prod);
                            M.val[e] = (float)((double)M.val[e] * scale);
                        }
                }
            });
        };
        // CSR row v / column u: din(v) * dout(u);  CSC row u / column v: dout(u) * din(v)
        scale_rows(R, len, d_out);
        if (!known_symmetric && want_csc) scale_rows(C, dout, len);
    }

    // ---- symmetric detection (bitwise)
    bool sym = known_symmetric;
    if (!known_symmetric && want_csc) {
        sym = (C.nnz == R.nnz) && C.rowptr == R.rowptr &&
              memcmp(C.colidx, R.colidx, (size_t)R.nnz * 4) == 0 &&
              memcmp(C.val, R.val, (size_t)R.nnz * 4) == 0;
    }
    out->n = n;
    out->symmetric = sym;
    out->has_csc = sym || want_csc;
    // weights that follow from the structure alone need not travel with a streamed chunk
    out->val_mode = edge_weight ? VAL_STORED : (norm ? VAL_GCN : VAL_ONES);
    if (out->val_mode == VAL_GCN) {
        const std::vector<int64_t>& d_out = known_symmetric ? len : dout;
        out->din.resize((size_t)n);
        out->dout.resize((size_t)n);
        for (int64_t v = 0; v < n; ++v) { out->din[v] = (int32_t)len[v]; out->dout[v] = (int32_t)d_out[v]; }
    }
    return NTP_OK;
}

// perm[p] = position, in the by-destination form, of the edge stored at position p of the
// by-source form (the by-destination form itself when the graph is symmetric).  The rows of the
// by-source form were filled by walking the by-destination entries in order, so walking them
// again in that order meets the positions of every by-source row in increasing order.
void build_edge_perm(const BuiltGraph& G, int32_t* perm) {
    const HostSparse& R = G.csr;
    const HostSparse& S = G.symmetric ? G.csr : G.csc;
    const int64_t n = G.n;
    const int T = host_threads();
    std::vector<int64_t> fill(S.rowptr.begin(), S.rowptr.end() - 1);
    parallel_for_threads(T, [&](int t, int nt) {
        const int64_t lo = n * t / nt, hi = n * (t + 1) / nt;
        for (int64_t e = 0; e < R.nnz; ++e) {
            const int32_t u = R.colidx[e];
            if (u >= lo && u < hi) perm[fill[u]++] = (int32_t)e;
        }
    });
}

}  // namespace ntp
