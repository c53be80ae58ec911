// Stand-alone driver for the host side of libntp (graph_build.cpp + plan.cpp): builds graphs
// for every combination of the build flags, plans them with several chunk sizes and checks
// the structural invariants of the result.  It links no device code, so it can be compiled
// with the host sanitizers (tests/test_host_sanitizers.py builds it with
// -fsanitize=address,undefined and runs it); any invariant that fails, and anything a
// sanitizer finds, ends the process with a non-zero status.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "ntp_internal.h"

using namespace ntp;

namespace {

int failures = 0;
#define CHECK(cond, ...)                                                     \
    do {                                                                     \
        if (!(cond)) {                                                       \
            ++failures;                                                      \
            fprintf(stderr, "%s:%d: %s: ", __FILE__, __LINE__, #cond);       \
            fprintf(stderr, __VA_ARGS__);                                    \
            fprintf(stderr, "\n");                                           \
        }                                                                    \
    } while (0)

void* alloc_plain(size_t bytes, void*) { return malloc(bytes ? bytes : 1); }

struct Lcg {        // small seeded generator for the driver's own inputs
    uint64_t s;
    uint32_t next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(s >> 33); }
};

void free_graph(BuiltGraph& G) {
    free(G.csr.colidx); free(G.csr.val); free(G.csc.colidx); free(G.csc.val);
    G.csr.colidx = G.csc.colidx = nullptr;
    G.csr.val = G.csc.val = nullptr;
}

// rowptr monotone from 0 to nnz, columns inside [0, n) and ascending within a row
void check_form(const HostSparse& m, int64_t n, bool strictly, const char* what) {
    CHECK(m.n == n, "%s: n %" PRId64, what, m.n);
    CHECK((int64_t)m.rowptr.size() == n + 1 && m.rowptr[0] == 0 && m.rowptr[n] == m.nnz, "%s: rowptr ends", what);
    int64_t longest = 0;
    for (int64_t v = 0; v < n; ++v) {
        const int64_t b = m.rowptr[v], e = m.rowptr[v + 1];
        CHECK(e >= b, "%s: rowptr decreases at %" PRId64, what, v);
        longest = e - b > longest ? e - b : longest;
        for (int64_t k = b; k < e; ++k) {
            CHECK(m.colidx[k] >= 0 && m.colidx[k] < n, "%s: column out of range", what);
            if (k > b) CHECK(strictly ? m.colidx[k - 1] < m.colidx[k] : m.colidx[k - 1] <= m.colidx[k], "%s: row %" PRId64 " not ascending", what, v);
        }
    }
    CHECK(longest == m.max_degree, "%s: max_degree %" PRId64 " vs %" PRId64, what, m.max_degree, longest);
}

// every row of the form is covered exactly once: by a bin list or by the segments of a split row;
// chunks tile the entries in order; segment slots are consecutive per row
void check_plan(const HostSparse& m, const Plan& P, int64_t chunk_edges, const char* what) {
    const int64_t n = m.n;
    std::vector<int64_t> covered(n > 0 ? n : 0, 0);      // entries of each row accounted for
    int64_t e_next = 0, slots = 0;
    CHECK(!P.chunks.empty(), "%s: no chunk", what);
    for (const Chunk& c : P.chunks) {
        CHECK(c.e_begin == e_next, "%s: chunk starts at %" PRId64 ", expected %" PRId64, what, c.e_begin, e_next);
        CHECK(c.e_end >= c.e_begin, "%s: chunk entries", what);
        e_next = c.e_end;
        if (chunk_edges > 0 && !c.partial_row && c.row_end - c.row_begin > 1)
            CHECK(c.e_end - c.e_begin <= chunk_edges, "%s: chunk of %" PRId64 " entries over the limit %" PRId64, what, c.e_end - c.e_begin, chunk_edges);
        const int64_t* rp = reinterpret_cast<const int64_t*>(c.meta.data() + c.off_rowptr);
        const int32_t* rows = reinterpret_cast<const int32_t*>(c.meta.data() + c.off_rows);
        const Segment* segs = reinterpret_cast<const Segment*>(c.meta.data() + c.off_segs);
        const ReduceItem* red = reinterpret_cast<const ReduceItem*>(c.meta.data() + c.off_reduce);
        CHECK(c.meta.size() >= c.off_reduce + (size_t)c.n_reduce * sizeof(ReduceItem), "%s: meta too small", what);
        for (int64_t r = c.row_begin; r <= c.row_end && n > 0; ++r)
            CHECK(rp[r - c.row_begin] == m.rowptr[r], "%s: rowptr slice", what);
        int64_t nb = 0;
        for (int b = 0; b < NBINS; ++b) {
            CHECK(c.bin_row_off[b] == nb, "%s: bin offset", what);
            for (int i = 0; i < c.bin_count[b]; ++i) {
                const int32_t v = rows[nb + i];
                CHECK(v >= c.row_begin && v < c.row_end, "%s: bin row outside the chunk", what);
                const int64_t d = m.rowptr[v + 1] - m.rowptr[v];
                CHECK(d <= P.split_threshold, "%s: long row in a bin", what);
                CHECK(b == 0 ? d <= 1 : (b == NBINS - 1 ? d > (1 << (NBINS - 2)) : (d > (1 << (b - 1)) && d <= (1 << b))), "%s: row of %" PRId64 " entries in bin %d", what, d, b);
                covered[v] += d;
            }
            nb += c.bin_count[b];
        }
        for (int i = 0; i < c.n_segs; ++i) {
            const Segment& s = segs[i];
            CHECK(s.row >= c.row_begin && s.row < c.row_end, "%s: segment row", what);
            CHECK(s.e_begin >= c.e_begin && s.e_begin + s.len <= c.e_end, "%s: segment outside its chunk", what);
            CHECK(s.e_begin >= m.rowptr[s.row] && s.e_begin + s.len <= m.rowptr[s.row + 1], "%s: segment outside its row", what);
            CHECK(s.len > 0 && s.len <= 2 * P.seg_len, "%s: segment length %d", what, s.len);
            CHECK(s.slot == slots, "%s: slot %d, expected %" PRId64, what, s.slot, slots);
            ++slots;
            covered[s.row] += s.len;
        }
        for (int i = 0; i < c.n_reduce; ++i) {
            const ReduceItem& it = red[i];
            const int64_t d = m.rowptr[it.row + 1] - m.rowptr[it.row];
            CHECK(d > P.split_threshold || c.partial_row, "%s: short row split", what);
            CHECK(it.first_slot >= 0 && it.first_slot + it.n_slots <= slots, "%s: reduce item slots", what);
        }
        CHECK(c.img_bytes >= c.img_off_val && c.img_off_val >= c.img_off_colidx && c.img_off_colidx >= c.meta.size(), "%s: image layout", what);
        CHECK(c.img_bytes <= P.max_img_bytes, "%s: image larger than the staging size", what);
    }
    CHECK(e_next == m.nnz, "%s: chunks end at %" PRId64 " of %" PRId64, what, e_next, m.nnz);
    CHECK(slots == P.n_slots, "%s: %" PRId64 " slots, plan says %" PRId64, what, slots, P.n_slots);
    for (int64_t v = 0; v < n; ++v)
        CHECK(covered[v] == m.rowptr[v + 1] - m.rowptr[v], "%s: row %" PRId64 " covered %" PRId64 " of %" PRId64, what, v, covered[v], m.rowptr[v + 1] - m.rowptr[v]);
}

// hub columns: the most gathered ones, most first, none below the bound; the encoded ids decode back
void check_hubs(const HostSparse& m, const HostSparse* transposed, const char* what) {
    std::vector<int64_t> count((size_t)m.n, 0);
    for (int64_t k = 0; k < m.nnz; ++k) ++count[(size_t)m.colidx[k]];
    for (int slots : {1, 5, 1024})
        for (int64_t min_count : {(int64_t)1, (int64_t)3, (int64_t)1000000}) {
            std::vector<int32_t> hubs, counted;
            pick_hub_columns(m, transposed, slots, min_count, &hubs);
            pick_hub_columns(m, nullptr, slots, min_count, &counted);
            CHECK(hubs == counted, "%s: hub columns differ between the two ways of counting", what);
            CHECK((int)hubs.size() <= slots, "%s: %zu hubs for %d slots", what, hubs.size(), slots);
            std::vector<char> is_hub((size_t)m.n, 0);
            int64_t least = INT64_MAX;
            for (size_t i = 0; i < hubs.size(); ++i) {
                const int32_t c = hubs[i];
                CHECK(c >= 0 && c < m.n && !is_hub[(size_t)c], "%s: bad hub column", what);
                is_hub[(size_t)c] = 1;
                CHECK(count[(size_t)c] >= min_count, "%s: hub below the bound", what);
                if (i > 0) CHECK(count[(size_t)hubs[i - 1]] > count[(size_t)c] || (count[(size_t)hubs[i - 1]] == count[(size_t)c] && hubs[i - 1] < c), "%s: hub order", what);
                least = count[(size_t)c] < least ? count[(size_t)c] : least;
            }
            for (int64_t c = 0; c < m.n; ++c)
                if (!is_hub[(size_t)c] && count[(size_t)c] >= min_count)
                    CHECK((int)hubs.size() == slots && count[(size_t)c] <= least, "%s: column %" PRId64 " with %" PRId64 " entries left out", what, c, count[(size_t)c]);
            if (m.nnz == 0) continue;
            const int64_t e0 = m.nnz / 3, e1 = m.nnz - m.nnz / 5;
            std::vector<int32_t> enc((size_t)(e1 - e0));
            encode_hub_columns(m, hubs, e0, e1, enc.data());
            for (int64_t k = e0; k < e1; ++k) {
                const int32_t e = enc[(size_t)(k - e0)], c = m.colidx[k];
                if (is_hub[(size_t)c]) CHECK(e < 0 && (size_t)(e & 0x7fffffff) < hubs.size() && hubs[(size_t)(e & 0x7fffffff)] == c, "%s: hub entry encoded wrongly", what);
                else CHECK(e == c, "%s: plain entry changed", what);
            }
        }
}

void build_and_plan(int64_t n, const std::vector<int32_t>& src, const std::vector<int32_t>& dst, const float* w, uint32_t flags, const char* what) {
    BuiltGraph G;
    EntryAllocator alloc{alloc_plain, nullptr, alloc_plain};
    const int rc = build_host_graph(n, (int64_t)src.size(), src.data(), dst.data(), w, flags, alloc, &G);
    CHECK(rc == NTP_OK, "%s: build failed: %s", what, last_error());
    if (rc != NTP_OK) return;
    const bool strictly = flags & NTP_DEDUP;
    check_form(G.csr, n, strictly, what);
    if (G.has_csc && !G.symmetric) check_form(G.csc, n, strictly, what);
    if (G.has_csc && !G.symmetric) CHECK(G.csc.nnz == G.csr.nnz, "%s: forms differ in size", what);
    if (G.has_csc && !G.symmetric && G.csr.nnz < INT32_MAX) {
        std::vector<int32_t> perm((size_t)G.csr.nnz);
        build_edge_perm(G, perm.data());
        for (int64_t u = 0; u < n; ++u)
            for (int64_t k = G.csc.rowptr[u]; k < G.csc.rowptr[u + 1]; ++k) {
                const int32_t p = perm[(size_t)k];
                CHECK(p >= 0 && p < G.csr.nnz && G.csr.colidx[p] == u && G.csr.val[p] == G.csc.val[k], "%s: edge permutation", what);
            }
    }
    check_hubs(G.csr, G.symmetric ? &G.csr : (G.has_csc ? &G.csc : nullptr), what);
    if (G.has_csc && !G.symmetric) check_hubs(G.csc, &G.csr, what);
    for (int64_t ce : {(int64_t)0, (int64_t)1, (int64_t)7, (int64_t)100, (int64_t)5000}) {
        Plan P;
        make_plan(G.csr, ce, &P);
        check_plan(G.csr, P, ce, what);
        if (G.has_csc && !G.symmetric) {
            Plan Q;
            make_plan(G.csc, ce, &Q);
            check_plan(G.csc, Q, ce, what);
        }
    }
    free_graph(G);
}

}  // namespace

int main() {
    // 1. every flag combination, weighted and not, on random multigraphs with loops and repeats
    Lcg rng{12345};
    for (int64_t n : {(int64_t)0, (int64_t)1, (int64_t)2, (int64_t)57, (int64_t)900}) {
        std::vector<int32_t> src, dst;
        std::vector<float> w;
        const int64_t m = n == 0 ? 0 : 6 * n + 3;
        for (int64_t i = 0; i < m; ++i) {
            src.push_back((int32_t)(rng.next() % n));
            dst.push_back((int32_t)(rng.next() % (i % 3 == 0 ? (n < 4 ? n : 4) : n)));      // a few heavy destinations
            w.push_back(0.25f + (float)(rng.next() % 1000) / 500.f);
        }
        for (uint32_t flags = 0; flags < 16; ++flags)
            for (int weighted = 0; weighted < 2; ++weighted)
                for (uint32_t extra : {0u, (uint32_t)NTP_SCATTER_BWD}) {
                    char what[96];
                    snprintf(what, sizeof what, "n=%" PRId64 " flags=%u weighted=%d extra=%u", n, flags, weighted, extra);
                    build_and_plan(n, src, dst, weighted ? w.data() : nullptr, flags | extra, what);
                }
    }
    // 2. a star whose hub has far more entries than a chunk may hold: the hub's row is cut by entry range
    {
        const int64_t n = 20000;
        std::vector<int32_t> src, dst;
        for (int32_t v = 1; v < n; ++v) { src.push_back(v); dst.push_back(0); }
        BuiltGraph G;
        EntryAllocator alloc{alloc_plain, nullptr, alloc_plain};
        const int rc = build_host_graph(n, (int64_t)src.size(), src.data(), dst.data(), nullptr,
                                        NTP_DEDUP | NTP_ADD_SELF_LOOPS | NTP_NORM_GCN_SYM, alloc, &G);
        CHECK(rc == NTP_OK, "star: %s", last_error());
        if (rc == NTP_OK) {
            for (int64_t ce : {(int64_t)512, (int64_t)3000, (int64_t)19999, (int64_t)20000}) {
                Plan P;
                make_plan(G.csr, ce, &P);
                check_plan(G.csr, P, ce, "star, by destination");
                int partial = 0;
                for (const Chunk& c : P.chunks) partial += c.partial_row;
                CHECK((ce < 20000) == (partial > 1), "star: %d chunks of the hub row at chunk size %" PRId64, partial, ce);
                Plan Q;
                make_plan(G.csc, ce, &Q);
                check_plan(G.csc, Q, ce, "star, by source");
            }
            free_graph(G);
        }
    }
    // 3. a form whose entry offsets pass 2^31 (row pointers only: the plan never reads the entries):
    //    3,000 rows of 1,000,000 entries and one of 5, in chunks of 256 Mi entries
    {
        HostSparse m;
        m.n = 3001;
        m.rowptr.resize(m.n + 1);
        m.rowptr[0] = 0;
        for (int64_t v = 0; v < m.n; ++v) m.rowptr[v + 1] = m.rowptr[v] + (v == 1500 ? 5 : 1000000);
        m.nnz = m.rowptr[m.n];
        m.max_degree = 1000000;
        CHECK(m.nnz > (int64_t)INT32_MAX, "large form too small");
        for (int64_t ce : {(int64_t)0, (int64_t)(256 << 20), (int64_t)999999}) {
            Plan P;
            make_plan(m, ce, &P);
            check_plan(m, P, ce, "entry offsets beyond 2^31");
            if (ce == (256 << 20)) CHECK(P.chunks.size() == 12, "%zu chunks", P.chunks.size());
            int64_t far = 0;
            for (const Chunk& c : P.chunks)
                for (int i = 0; i < c.n_segs; ++i) {
                    const Segment& s = reinterpret_cast<const Segment*>(c.meta.data() + c.off_segs)[i];
                    far = s.e_begin > far ? s.e_begin : far;
                }
            CHECK(far > (int64_t)INT32_MAX, "no segment starts beyond 2^31");
        }
    }
    // 4. bad input is refused, not read
    {
        BuiltGraph G;
        EntryAllocator alloc{alloc_plain, nullptr, alloc_plain};
        const int32_t s[2] = {0, 9}, d[2] = {1, 2};
        CHECK(build_host_graph(3, 2, s, d, nullptr, NTP_DEDUP, alloc, &G) == NTP_EINVAL, "vertex id out of range accepted");
    }
    if (failures) { fprintf(stderr, "%d checks failed\n", failures); return 1; }
    printf("host checks passed\n");
    return 0;
}
