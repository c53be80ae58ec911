// Host-side planning of one compressed form: chunk boundaries (Section 4.2.1: contiguous
// destination ranges with all their entries, as large as allowed), degree bins that map
// rows to wavefronts, and the segments of rows too long for one wavefront.
#include "ntp_internal.h"

#include <algorithm>
#include <climits>
#include <cstring>

namespace ntp {

namespace {

inline int bin_of(int64_t d) {
    if (d <= 1) return 0;
    int b = 1;
    int64_t hi = 2;
    while (d > hi && b < NBINS - 1) { hi <<= 1; ++b; }
    return b;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct ChunkBuilder {
    const HostSparse& m;
    Plan& plan;
    std::vector<int32_t> bin_rows[NBINS];
    std::vector<Segment> segs;
    std::vector<ReduceItem> reduce;

    void reset() {
        for (auto& b : bin_rows) b.clear();
        segs.clear();
        reduce.clear();
    }

    void finish(Chunk& c) {
        const int64_t nrows = c.row_end - c.row_begin;
        size_t nbin = 0;
        for (int b = 0; b < NBINS; ++b) {
            c.bin_count[b] = (int32_t)bin_rows[b].size();
            c.bin_row_off[b] = (int32_t)nbin;
            nbin += bin_rows[b].size();
        }
        c.n_segs = (int32_t)segs.size();
        c.n_reduce = (int32_t)reduce.size();
        // Split rows.  While the chip is loaded a wavefront gets its share of the compute unit's
        // gather rate: one 8192nd of the chip's (256 compute units x up to 32 wavefronts).  A split
        // row handled by one block (four wavefronts, a quarter of the row each, sums combined through
        // LDS: no partial sums in memory, no second kernel) therefore lasts as long as a chunk of
        // 2048 x its length on the whole chip; it must stay well inside the column pass it belongs
        // to.  Longer rows go to wavefronts all over the chip as segments, and reduce_kernel adds
        // the pieces.  Measured on MI355X: 2.3 % faster on a 114 M-entry graph whose longest row has
        // 20 k entries; block rows of 10 k entries on a 2.5 M-entry graph cost 9 %.
        c.block_rows = c.n_reduce > 0 && !c.partial_row && (int64_t)c.max_split_len * 4096 <= c.e_end - c.e_begin;
        c.off_rowptr = 0;
        c.off_rows = align_up(c.off_rowptr + (size_t)(nrows + 1) * 8, 16);
        c.off_segs = align_up(c.off_rows + nbin * 4, 16);
        c.off_reduce = align_up(c.off_segs + segs.size() * sizeof(Segment), 16);
        const size_t meta_bytes = align_up(c.off_reduce + reduce.size() * sizeof(ReduceItem), 256);
        c.meta.assign(meta_bytes, 0);
        memcpy(c.meta.data() + c.off_rowptr, m.rowptr.data() + c.row_begin, (size_t)(nrows + 1) * 8);
        for (int b = 0; b < NBINS; ++b)
            if (!bin_rows[b].empty())
                memcpy(c.meta.data() + c.off_rows + (size_t)c.bin_row_off[b] * 4, bin_rows[b].data(), bin_rows[b].size() * 4);
        if (!segs.empty()) memcpy(c.meta.data() + c.off_segs, segs.data(), segs.size() * sizeof(Segment));
        if (!reduce.empty()) memcpy(c.meta.data() + c.off_reduce, reduce.data(), reduce.size() * sizeof(ReduceItem));
        const size_t ne = (size_t)(c.e_end - c.e_begin);
        c.img_off_colidx = meta_bytes;
        c.img_off_val = c.img_off_colidx + align_up(ne * 4, 256);
        c.img_bytes = c.img_off_val + align_up(ne * 4, 256);
        plan.max_img_bytes = std::max(plan.max_img_bytes, c.img_bytes);
    }
};

}  // namespace

void pick_hub_columns(const HostSparse& m, const HostSparse* transposed, int max_slots, int64_t min_count,
                      std::vector<int32_t>* hub_cols) {
    hub_cols->clear();
    if (m.n <= 0 || m.nnz <= 0 || max_slots <= 0) return;
    // entries per column: the row lengths of the transposed form when there is one, else counted
    std::vector<int32_t> counted;
    if (!transposed) {
        counted.assign((size_t)m.n, 0);
        for (int64_t k = 0; k < m.nnz; ++k) ++counted[(size_t)m.colidx[k]];
    }
    std::vector<std::pair<int64_t, int32_t>> cand;        // (-count, id): ascending = most gathered first, ties by id
    for (int64_t c = 0; c < m.n; ++c) {
        const int64_t total = transposed ? transposed->rowptr[(size_t)c + 1] - transposed->rowptr[(size_t)c] : counted[(size_t)c];
        if (total >= min_count) cand.emplace_back(-total, (int32_t)c);
    }
    const size_t k = std::min<size_t>((size_t)max_slots, cand.size());
    std::partial_sort(cand.begin(), cand.begin() + (std::ptrdiff_t)k, cand.end());
    for (size_t i = 0; i < k; ++i) hub_cols->push_back(cand[i].second);
}

void encode_hub_columns(const HostSparse& m, const std::vector<int32_t>& hub_cols, int64_t e_begin, int64_t e_end, int32_t* out) {
    std::vector<int32_t> slot_of((size_t)m.n, -1);
    for (size_t s = 0; s < hub_cols.size(); ++s) slot_of[(size_t)hub_cols[s]] = (int32_t)s;
    const int64_t ne = e_end - e_begin;
    const int T = std::max(1, std::min(host_threads(), (int)std::min<int64_t>(16, ne / (1 << 20) + 1)));
    parallel_for_threads(T, [&](int t, int nt) {
        const int64_t lo = e_begin + ne * t / nt, hi = e_begin + ne * (t + 1) / nt;
        for (int64_t k = lo; k < hi; ++k) {
            const int32_t c = m.colidx[k];
            const int32_t s = slot_of[(size_t)c];
            out[k - e_begin] = s >= 0 ? (int32_t)(0x80000000u | (uint32_t)s) : c;
        }
    });
}

void make_plan(const HostSparse& m, int64_t chunk_edges, Plan* plan) {
    Plan& P = *plan;
    P = Plan();
    const int64_t n = m.n;
    const bool chunked = chunk_edges > 0;
    P.chunk_edges = chunked ? chunk_edges : 0;

    // segment length: enough pieces to spread a hub over the chip, few enough that the
    // partial sums stay a small fraction of the traffic.  It follows the size of one launch
    // (a chunk): while the chip is loaded a wavefront works through some nine entries per
    // microsecond, so a piece must be short against the launch it belongs to or it outlives it
    // (measured: 9 chunks of 16 M entries with pieces of 4096 cost 5 % more than with 512).
    const int64_t launch_entries = chunked ? std::min(m.nnz, chunk_edges) : m.nnz;
    int64_t seg = 256;
    while (seg < 4096 && seg * 32768 < launch_entries) seg <<= 1;
    if (chunked) seg = std::min(seg, chunk_edges);
    seg = std::max<int64_t>(seg, 1);
    P.seg_len = seg;
    P.split_threshold = chunked ? std::min(2 * seg, chunk_edges) : 2 * seg;

    ChunkBuilder cb{m, P, {}, {}, {}};
    int32_t next_slot = 0;
    int64_t r = 0;
    while (r < n) {
        const int64_t e0 = m.rowptr[r];
        int64_t r1;
        if (!chunked) {
            r1 = n;
        } else {
            // last row boundary with at most chunk_edges entries since e0, at least one row
            const int64_t* b = std::upper_bound(m.rowptr.data() + r, m.rowptr.data() + n + 1, e0 + chunk_edges);
            r1 = std::max<int64_t>(r + 1, (b - m.rowptr.data()) - 1);
            r1 = std::min(r1, n);
        }
        const bool giant = chunked && (r1 == r + 1) && (m.rowptr[r + 1] - e0 > chunk_edges);
        if (!giant) {
            Chunk c;
            c.row_begin = r; c.row_end = r1; c.e_begin = e0; c.e_end = m.rowptr[r1];
            cb.reset();
            for (int64_t v = r; v < r1; ++v) {
                const int64_t d = m.rowptr[v + 1] - m.rowptr[v];
                if (d > P.split_threshold) {
                    const int64_t nseg = (d + seg - 1) / seg;
                    const int64_t base = d / nseg, extra = d % nseg;
                    int64_t e = m.rowptr[v];
                    cb.reduce.push_back(ReduceItem{(int32_t)v, next_slot, (int32_t)nseg, 0});
                    c.max_split_len = (int32_t)std::max<int64_t>(c.max_split_len, std::min<int64_t>(d, INT32_MAX));
                    for (int64_t i = 0; i < nseg; ++i) {
                        const int64_t l = base + (i < extra ? 1 : 0);
                        cb.segs.push_back(Segment{e, (int32_t)l, (int32_t)v, next_slot++, 0});
                        e += l;
                    }
                } else {
                    cb.bin_rows[bin_of(d)].push_back((int32_t)v);
                }
            }
            cb.finish(c);
            P.chunks.push_back(std::move(c));
        } else {
            // one row larger than a chunk: its segments are packed into chunks of their own
            const int64_t d = m.rowptr[r + 1] - e0;
            const int64_t nseg = (d + seg - 1) / seg;
            const int64_t base = d / nseg, extra = d % nseg;
            const int32_t first_slot = next_slot;
            int64_t e = e0;
            int64_t i = 0;
            while (i < nseg) {
                Chunk c;
                c.row_begin = r; c.row_end = r + 1; c.partial_row = true;
                c.e_begin = e;
                cb.reset();
                int64_t used = 0;
                while (i < nseg) {
                    const int64_t l = base + (i < extra ? 1 : 0);
                    if (used + l > chunk_edges && used > 0) break;
                    cb.segs.push_back(Segment{e, (int32_t)l, (int32_t)r, next_slot++, 0});
                    e += l; used += l; ++i;
                }
                c.e_end = e;
                if (i == nseg) cb.reduce.push_back(ReduceItem{(int32_t)r, first_slot, (int32_t)nseg, 0});
                cb.finish(c);
                P.chunks.push_back(std::move(c));
            }
        }
        r = r1;
    }
    if (n == 0) {   // an empty graph still has one (empty) chunk
        Chunk c;
        cb.reset();
        cb.finish(c);
        P.chunks.push_back(std::move(c));
    }
    P.n_slots = next_slot;
}

}  // namespace ntp
