// Edge attention weights of GAT-style aggregation (AGG of GAT, Section 2.1 of the paper;
// Section 4.1 computes them for all edges before the aggregation starts):
//   e(u -> v) = LeakyReLU(p[u] + q[v]),   alpha(u -> v) = exp(e(u -> v)) / sum over the
//   in-edges (u' -> v) of exp(e(u' -> v))
// with per-vertex scores p (source half of the mapping a^T [. || .]) and q (destination half).
//
// Rows of the by-destination form are softmax rows: a lane group (rows of up to 8 or 32
// entries) or a wavefront (longer rows) takes the row maximum, the sum of exponentials and
// writes the weights; rows beyond the split threshold go segment by segment (one block each,
// partial maxima and sums combined per row); all reductions in fixed trees
// (deterministic).  The score q, the maximum and the reciprocal sum of every destination are
// kept, so the same weights can be written in the entry order of the by-source form element
// by element, with the same arithmetic (bit-identical numbers for an edge in both orders).
#include <hip/hip_runtime.h>

#include <cmath>

#include "lane_util.h"
#include "ntp_internal.h"

namespace ntp {

namespace {

__device__ __forceinline__ float lrelu(float x, float slope) { return x > 0.f ? x : slope * x; }

template <int L> __device__ __forceinline__ float group_max(float v, int lane) {
#pragma unroll
    for (int off = 1; off < L; off <<= 1) v = fmaxf(v, bperm_f(lane ^ off, v));
    return v;
}
template <int L> __device__ __forceinline__ float group_sum(float v, int lane) {
#pragma unroll
    for (int off = 1; off < L; off <<= 1) v += bperm_f(lane ^ off, v);
    return v;
}

// Per destination v the by-destination pass leaves st[v] = (q[v], row maximum, 1 / row sum, 0):
// one 16-byte gather gives the by-source pass everything it needs about v.
//
// alpha = exp(e - maximum) * (1 / sum) in both passes, from the same stored numbers.
__device__ __forceinline__ float weight_of(float e, float mx, float rs) { return expf(e - mx) * rs; }

// One group of L lanes per row; rows taken from rows[0..n_rows).
// TRANSPOSED = false: rows are destinations v, columns sources u; writes alpha and st[v].
// TRANSPOSED = true : rows are sources u, columns destinations v; reads st[v].
// Entries are taken four per lane at a time so that four gathers are in flight.  A row longer
// than 4 L entries parks its scores in the output array after the first sweep, so the random
// gathers of p happen once and the later sweeps read consecutive memory.
template <int L, bool TRANSPOSED>
__global__ void __launch_bounds__(256) attention_rows_kernel(const AttArgs a, int first, int n_rows) {
    constexpr int R = 64 / L;
    const int lane = threadIdx.x & 63;
    const int g = lane / L, l = lane % L;
    const int64_t idx = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * R + g;
    const bool valid = idx < n_rows;
    int row = 0;
    int64_t beg = 0;
    int64_t d = 0;
    if (valid) {
        row = a.rows[first + idx];
        beg = a.rowptr[row];
        d = a.rowptr[row + 1] - beg;
    }
    const int32_t* ci = a.colidx + beg;
    float* out = a.alpha + beg;
    if constexpr (TRANSPOSED) {
        const float pu = valid ? a.p[row] : 0.f;
        for (int64_t k0 = l; k0 < d; k0 += 4 * L) {
            int c[4];
            float4 t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) c[u] = k0 + u * L < d ? ci[k0 + u * L] : row;
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = reinterpret_cast<const float4*>(a.st)[c[u]];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (k0 + u * L < d) out[k0 + u * L] = weight_of(lrelu(pu + t[u].x, a.slope), t[u].y, t[u].z);
        }
        return;
    }
    const float qv = valid ? a.q[row] : 0.f;
    // first sweep: scores of up to four entries per lane stay in registers
    float e[4];
    {
        int c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) c[u] = l + u * L < d ? ci[l + u * L] : row;
#pragma unroll
        for (int u = 0; u < 4; ++u) e[u] = l + u * L < d ? lrelu(a.p[c[u]] + qv, a.slope) : -INFINITY;
    }
    float m = fmaxf(fmaxf(e[0], e[1]), fmaxf(e[2], e[3]));
    const bool longer = __ballot(d > 4 * L) != 0;          // some row of the wavefront needs more sweeps
    if (longer) {
        for (int64_t k0 = l + 4 * L; k0 < d; k0 += 4 * L) {
            int c[4];
            float x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) c[u] = k0 + u * L < d ? ci[k0 + u * L] : row;
#pragma unroll
            for (int u = 0; u < 4; ++u) x[u] = lrelu(a.p[c[u]] + qv, a.slope);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (k0 + u * L < d) { out[k0 + u * L] = x[u]; m = fmaxf(m, x[u]); }
        }
    }
    m = group_max<L>(m, lane);
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) s += l + u * L < d ? expf(e[u] - m) : 0.f;
    if (longer)
        for (int64_t k = l + 4 * L; k < d; k += L) s += expf(out[k] - m);
    s = group_sum<L>(s, lane);
    const float rs = 1.f / s;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (l + u * L < d) out[l + u * L] = weight_of(e[u], m, rs);
    if (longer)
        for (int64_t k = l + 4 * L; k < d; k += L) out[k] = weight_of(out[k], m, rs);
    if (valid && l == 0) reinterpret_cast<float4*>(a.st)[row] = d > 0 ? make_float4(qv, m, rs, 0.f) : make_float4(qv, 0.f, 1.f, 0.f);
}

// ---- rows beyond the split threshold: one block per segment (the pieces the aggregation
// cuts such rows into), so that a hub row of 10^5 entries is spread over many blocks ---------
// pass 1: scores parked in the output array; per segment maximum and sum of exp(score - maximum)
__global__ void __launch_bounds__(256) attention_segment_stats_kernel(const AttArgs a, const Segment* segs, float2* seg_stats) {
    __shared__ float red[4];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const Segment sg = segs[blockIdx.x];
    const int32_t* ci = a.colidx + sg.e_begin;
    float* out = a.alpha + sg.e_begin;
    const float qv = a.q[sg.row];
    float m = -INFINITY;
    for (int k = threadIdx.x; k < sg.len; k += 256) {
        const float x = lrelu(a.p[ci[k]] + qv, a.slope);
        out[k] = x;
        m = fmaxf(m, x);
    }
    m = group_max<64>(m, lane);
    if (lane == 0) red[w] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float s = 0.f;
    for (int k = threadIdx.x; k < sg.len; k += 256) s += expf(out[k] - m);
    s = group_sum<64>(s, lane);
    if (lane == 0) red[w] = s;
    __syncthreads();
    if (threadIdx.x == 0) seg_stats[sg.slot] = make_float2(m, (red[0] + red[1]) + (red[2] + red[3]));
}

// pass 2: one wavefront per split row combines its segments: maximum of the maxima, sums
// rescaled to it and added in a fixed tree
__global__ void __launch_bounds__(64) attention_combine_kernel(const AttArgs a, const ReduceItem* items, const float2* seg_stats) {
    const int lane = threadIdx.x;
    const ReduceItem it = items[blockIdx.x];
    const float2* st = seg_stats + it.first_slot;
    float m = -INFINITY;
    for (int k = lane; k < it.n_slots; k += 64) m = fmaxf(m, st[k].x);
    m = group_max<64>(m, lane);
    float s = 0.f;
    for (int k = lane; k < it.n_slots; k += 64) s += st[k].y * expf(st[k].x - m);
    s = group_sum<64>(s, lane);
    if (lane == 0) reinterpret_cast<float4*>(a.st)[it.row] = make_float4(a.q[it.row], m, 1.f / s, 0.f);
}

// pass 3 (by destination): parked scores -> weights; by source: the element-wise form
template <bool TRANSPOSED>
__global__ void __launch_bounds__(256) attention_segment_write_kernel(const AttArgs a, const Segment* segs) {
    const Segment sg = segs[blockIdx.x];
    float* out = a.alpha + sg.e_begin;
    if constexpr (TRANSPOSED) {
        const int32_t* ci = a.colidx + sg.e_begin;
        const float pu = a.p[sg.row];
        for (int k = threadIdx.x; k < sg.len; k += 256) {
            const float4 t = reinterpret_cast<const float4*>(a.st)[ci[k]];
            out[k] = weight_of(lrelu(pu + t.x, a.slope), t.y, t.z);
        }
    } else {
        const float4 t = reinterpret_cast<const float4*>(a.st)[sg.row];
        for (int k = threadIdx.x; k < sg.len; k += 256) out[k] = weight_of(out[k], t.y, t.z);
    }
}

// ---- gradient of the scores through the attention weights --------------------------------------
// Given dY = dLoss/dY of Y[v,:] = sum_u alpha(u -> v) Z[u,:]:
//   dalpha(u -> v) = dY[v,:] . Z[u,:],  t[v] = sum_u alpha dalpha,  de = alpha (dalpha - t[v]),
//   ds = de * (1 if p[u] + q[v] > 0 else slope),  dq[v] = sum over in-edges of ds,
//   dp[u] = sum over out-edges of ds.
// By-destination pass (rows v, own = dY[v,:], gathered = Z[u,:]): dalpha of every entry (parked in
// scratch), t[v], dq[v].  By-source pass (rows u, own = Z[u,:], gathered = dY[v,:]): dalpha again
// in that order, with t[v] and alpha in by-source order: dp[u].  A group of L lanes (4, 8 or 16)
// forms one dot product at a time (L x VEC x NJ columns, xor tree over the group).  Rows of more
// than 128 entries take one block (its groups share the entries, partial sums combined through
// LDS in a fixed order; one wavefront per such row measured slower); rows beyond the split
// threshold one block per segment, the partial sums of the segments combined by a small kernel
// in segment order.  Where both sweeps run in one kernel each lane keeps the dalpha of its first
// entry in a register (short rows park nothing) and a parked dalpha is read back by the thread
// that wrote it.  Widest row: 1024 columns with 16-byte vectors, 256 otherwise.
template <int VEC, int NJ, int L>
struct DotRow {
    float own[NJ][VEC];
    int col[NJ];
    bool on[NJ];
    __device__ __forceinline__ void load_own(const float* row, int l, int m) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            col[j] = (j * L + l) * VEC;
            on[j] = col[j] < m;
#pragma unroll
            for (int i = 0; i < VEC; ++i) own[j][i] = 0.f;
            if (on[j]) {
                if constexpr (VEC == 4) { const float4 t = *reinterpret_cast<const float4*>(row + col[j]); own[j][0] = t.x; own[j][1] = t.y; own[j][2] = t.z; own[j][3] = t.w; }
                else own[j][0] = row[col[j]];
            }
        }
    }
    // this lane's share of own . other (columns outside the row contribute zero)
    __device__ __forceinline__ float partial(const float* other, bool live) const {
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (on[j] && live) {
                if constexpr (VEC == 4) {
                    const float4 t = *reinterpret_cast<const float4*>(other + col[j]);
                    acc = fmaf(own[j][0], t.x, acc); acc = fmaf(own[j][1], t.y, acc);
                    acc = fmaf(own[j][2], t.z, acc); acc = fmaf(own[j][3], t.w, acc);
                } else {
                    acc = fmaf(own[j][0], other[col[j]], acc);
                }
            }
        }
        return acc;
    }
};

// WORK_GROUP  : one row per group of L lanes, rows[first .. first + n_rows).
// WORK_BLOCK  : one row per block (its 256 / L groups take the entries in turn), rows[first + blockIdx.x].
// WORK_SEG    : one segment of a split row per block, segs[blockIdx.x]: the dot products of its
//               entries; the partial t (by destination) or partial dp (by source) goes to the
//               segment's slot.
// WORK_SEG_DS : by destination only, after the slots of t were combined: ds of the segment's
//               entries from the parked dalpha, partial dq to the slot.
enum { WORK_GROUP = 0, WORK_BLOCK = 1, WORK_SEG = 2, WORK_SEG_DS = 3 };

template <int VEC, int NJ, int L, bool TRANSPOSED, int WORK>
__global__ void __launch_bounds__(256) attention_bwd_kernel(const AttBwdArgs a, int first, int n_rows, const Segment* segs) {
    constexpr bool SEG = WORK == WORK_SEG || WORK == WORK_SEG_DS;
    constexpr int R = 64 / L;                                          // groups per wavefront
    constexpr int NG = 256 / L;                                        // groups per block
    constexpr int SHARE = WORK == WORK_GROUP ? 1 : NG;                  // groups on one row
    constexpr int U = 4;                                               // dot products in flight per group
    __shared__ float red[NG];
    const int lane = threadIdx.x & 63;
    const int l = lane % L;
    const int gi = SHARE == 1 ? 0 : (int)(threadIdx.x / L);            // group among those on the row
    int row = 0;
    int slot = 0;
    bool valid = true;
    int64_t beg = 0, d = 0;
    if constexpr (SEG) {
        const Segment sg = segs[blockIdx.x];
        row = sg.row; slot = sg.slot; beg = sg.e_begin; d = sg.len;
    } else {
        const int64_t idx = WORK == WORK_BLOCK ? (int64_t)blockIdx.x : ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * R + lane / L;
        valid = idx < n_rows;
        if (valid) { row = a.rows[first + idx]; beg = a.rowptr[row]; d = a.rowptr[row + 1] - beg; }
    }
    const int32_t* ci = a.colidx + beg;
    const float* al = a.alpha + beg;
    float* park = a.park + beg;
    // sum over the groups that share the row of a value all lanes of a group hold, in a fixed order
    auto share_sum = [&](float v) {
        if constexpr (SHARE == 1) {
            return v;
        } else {
            if (l == 0) red[gi] = v;
            __syncthreads();
            float s = 0.f;
            for (int i = 0; i < NG; ++i) s += red[i];
            __syncthreads();
            return s;
        }
    };
    const bool writer = SHARE == NG ? threadIdx.x == 0 : (valid && l == 0);
    if constexpr (WORK == WORK_SEG_DS) {
        const float t = a.t[2 * row];
        const float qv = a.q[row];
        float dqp = 0.f;
        for (int64_t k = threadIdx.x; k < d; k += 256) {
            const int cc = ci[k];
            const float wv = (park[k] - t) * (a.p[cc] + qv > 0.f ? 1.f : a.slope);
            if (a.keep_w) park[k] = wv;
            dqp += al[k] * wv;
        }
        dqp = share_sum(group_sum<L>(dqp, lane));
        if (writer) a.slots[slot] = dqp;
        return;
    }
    DotRow<VEC, NJ, L> dot;
    dot.load_own(a.own + (int64_t)row * a.ld_own, l, valid ? a.m : 0);
    bool in[U];
    int c[U], cn[U];
    float da[U];
    auto columns = [&](int64_t k, int (&cc)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) cc[u] = k + u * SHARE < d ? ci[k + u * SHARE] : row;
    };
    // dalpha of entries k, k + SHARE, ...: U gathers issued before the first xor tree; the
    // column ids of the next batch are fetched meanwhile
    auto dots = [&](int64_t k) {
#pragma unroll
        for (int u = 0; u < U; ++u) { in[u] = k + u * SHARE < d; c[u] = cn[u]; }
#pragma unroll
        for (int u = 0; u < U; ++u) da[u] = dot.partial(a.other + (int64_t)c[u] * a.ld_other, in[u]);
        columns(k + U * SHARE, cn);
#pragma unroll
        for (int u = 0; u < U; ++u) da[u] = group_sum<L>(da[u], lane);
    };
    columns(gi, cn);
    if constexpr (TRANSPOSED) {
        const float pu = valid ? a.p[row] : 0.f;
        float acc = 0.f;
        for (int64_t k = gi; __ballot(k < d) != 0; k += U * SHARE) {          // the wavefront stays together for the shuffles
            dots(k);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (in[u]) {
                    const float2 tq = reinterpret_cast<const float2*>(a.t)[c[u]];      // (t, q) of the destination
                    acc += al[k + u * SHARE] * (da[u] - tq.x) * (pu + tq.y > 0.f ? 1.f : a.slope);
                }
        }
        acc = share_sum(acc);
        if (writer) { if constexpr (SEG) a.slots[slot] = acc; else a.out[row] = a.accumulate ? a.out[row] + acc : acc; }
        return;
    }
    // by destination: sweep 1 = dalpha of every entry (parked by the lane that reads it back), t
    float t = 0.f;
    float mine = 0.f;
    for (int64_t k = gi; __ballot(k < d) != 0; k += U * SHARE) {
        dots(k);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (in[u]) {
                const int64_t ku = k + u * SHARE;             // ku % SHARE == gi
                t += al[ku] * da[u];
                if (l == (int)((ku / SHARE) % L)) {
                    if (!SEG && ku < SHARE * L) mine = da[u]; // the lane's first entry stays in a register
                    else park[ku] = da[u];
                }
            }
        }
    }
    t = share_sum(t);
    if constexpr (SEG) {
        if (writer) a.slots[slot] = t;
        return;
    }
    // sweep 2: ds of the entries this lane parked, summed over the row
    const float qv = valid ? a.q[row] : 0.f;
    float dqp = 0.f;
    for (int64_t k = gi + SHARE * l; k < d; k += SHARE * L) {                // k % SHARE == gi, (k / SHARE) % L == l
        const int cc = ci[k];
        const float dak = k < SHARE * L ? mine : park[k];
        const float wv = (dak - t) * (a.p[cc] + qv > 0.f ? 1.f : a.slope);
        if (a.keep_w) park[k] = wv;
        dqp += al[k] * wv;
    }
    dqp = share_sum(group_sum<L>(dqp, lane));
    if (writer) { a.out[row] = a.accumulate ? a.out[row] + dqp : dqp; reinterpret_cast<float2*>(a.t)[row] = make_float2(t, qv); }
}

// out[row] = sum of the row's slots, in segment order (added to out[row] when accumulate is set);
// with q: the pair (sum, q[row]) at out[2 row]
__global__ void __launch_bounds__(256) attention_bwd_combine_kernel(const ReduceItem* items, int n_items, const float* slots, float* out,
                                                                    const float* q, int accumulate) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_items) return;
    const ReduceItem it = items[i];
    float s = 0.f;
    for (int j = 0; j < it.n_slots; ++j) s += slots[it.first_slot + j];
    if (q) reinterpret_cast<float2*>(out)[it.row] = make_float2(s, q[it.row]);
    else out[it.row] = accumulate ? out[it.row] + s : s;
}

__global__ void __launch_bounds__(256) vec_add_kernel(float* __restrict__ a, const float* __restrict__ b, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) a[i] += b[i];
}

template <int VEC, int NJ, int L, bool T>
int launch_bwd_shape(const AttBwdArgs& a, const AttBwdRows& r, int phase, hipStream_t st) {
    const Segment* none = nullptr;
    constexpr int ROWS_PER_BLOCK = 4 * (64 / L);
    if (phase == 0) {
        if (r.n_segs > 0)
            hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, L, T, WORK_SEG>), dim3((unsigned)r.n_segs), dim3(256), 0, st, a, 0, 0, r.segs);
        if (r.n_block_rows > 0)
            hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, L, T, WORK_BLOCK>), dim3((unsigned)r.n_block_rows), dim3(256), 0, st, a,
                               r.n_group_rows, r.n_block_rows, none);
        if (r.n_group_rows > 0)
            hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, L, T, WORK_GROUP>), dim3((unsigned)((r.n_group_rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK)),
                               dim3(256), 0, st, a, 0, r.n_group_rows, none);
    } else if (phase == 2) {
        if constexpr (!T) {
            if (r.n_segs > 0)
                hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, L, false, WORK_SEG_DS>), dim3((unsigned)r.n_segs), dim3(256), 0, st, a, 0, 0, r.segs);
        }
    }
    return hipGetLastError() == hipSuccess ? NTP_OK : NTP_EHIP;
}

// lanes per group: the smallest of 4, 8, 16 whose vectors cover the row; wider rows take several
// vectors per lane
template <int VEC, bool T>
int launch_bwd_vec(const AttBwdArgs& a, const AttBwdRows& r, int phase, hipStream_t st) {
    const int nvec = (a.m + VEC - 1) / VEC;
    if (nvec <= 4) return launch_bwd_shape<VEC, 1, 4, T>(a, r, phase, st);
    if (nvec <= 8) return launch_bwd_shape<VEC, 1, 8, T>(a, r, phase, st);
    const int nj = (nvec + 15) / 16;
    if (nj <= 1) return launch_bwd_shape<VEC, 1, 16, T>(a, r, phase, st);
    if (nj <= 2) return launch_bwd_shape<VEC, 2, 16, T>(a, r, phase, st);
    if (nj <= 4) return launch_bwd_shape<VEC, 4, 16, T>(a, r, phase, st);
    if (nj <= 8) return launch_bwd_shape<VEC, 8, 16, T>(a, r, phase, st);
    if (nj <= 16) return launch_bwd_shape<VEC, 16, 16, T>(a, r, phase, st);
    set_error("feature width %d too large for the attention gradient (at most %d)", a.m, 256 * VEC);
    return NTP_EUNSUPPORTED;
}

template <int L, bool T>
int launch_rows(const AttArgs& a, int first, int n_rows, hipStream_t st) {
    if (n_rows <= 0) return NTP_OK;
    const int rows_per_block = 4 * (64 / L);
    hipLaunchKernelGGL((attention_rows_kernel<L, T>), dim3((unsigned)((n_rows + rows_per_block - 1) / rows_per_block)), dim3(256), 0, st, a, first, n_rows);
    return hipGetLastError() == hipSuccess ? NTP_OK : NTP_EHIP;
}

}  // namespace

// One chunk of a form, one phase at a time (a row beyond the split threshold may have its
// segments in several chunks, so the caller runs a phase over all chunks before the next):
//   phase 0: per-segment statistics of split rows (by-destination pass only)
//   phase 1: per-row combination of the segment statistics (by-destination pass only)
//   phase 2: weights of the split rows' segments and of all other rows
// bins: bin_row_off / bin_count describe rows[] (see Plan); bins 0..3 hold rows of up to 8
// entries, 4..5 up to 32, the rest up to the split threshold; split rows come as segments
// (segs, n_segs), their rows as reduce items; seg_stats: two floats per partial-sum slot.
int launch_attention(const AttArgs& a, const int32_t* bin_row_off, const int32_t* bin_count,
                     const Segment* segs, int n_segs, const ReduceItem* split_rows, int n_split_rows,
                     float* seg_stats, bool transposed, int phase, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    float2* ss = reinterpret_cast<float2*>(seg_stats);
    int rc = NTP_OK;
    if (phase == 0) {
        if (!transposed && n_segs > 0)
            hipLaunchKernelGGL(attention_segment_stats_kernel, dim3((unsigned)n_segs), dim3(256), 0, st, a, segs, ss);
    } else if (phase == 1) {
        if (!transposed && n_split_rows > 0)
            hipLaunchKernelGGL(attention_combine_kernel, dim3((unsigned)n_split_rows), dim3(64), 0, st, a, split_rows, ss);
    } else {
        auto span = [&](int b0, int b1, int& first, int& count) {
            first = bin_row_off[b0];
            count = 0;
            for (int b = b0; b <= b1; ++b) count += bin_count[b];
        };
        int first, count;
        // long rows first: they are the longest-running pieces
        if (n_segs > 0) {
            if (transposed) hipLaunchKernelGGL(attention_segment_write_kernel<true>, dim3((unsigned)n_segs), dim3(256), 0, st, a, segs);
            else hipLaunchKernelGGL(attention_segment_write_kernel<false>, dim3((unsigned)n_segs), dim3(256), 0, st, a, segs);
        }
        span(6, NBINS - 1, first, count);
        rc = transposed ? launch_rows<64, true>(a, first, count, st) : launch_rows<64, false>(a, first, count, st);
        if (rc == NTP_OK) {
            span(4, 5, first, count);
            rc = transposed ? launch_rows<32, true>(a, first, count, st) : launch_rows<32, false>(a, first, count, st);
        }
        if (rc == NTP_OK) {
            span(0, 3, first, count);
            rc = transposed ? launch_rows<8, true>(a, first, count, st) : launch_rows<8, false>(a, first, count, st);
        }
    }
    if (rc == NTP_OK && hipGetLastError() != hipSuccess) rc = NTP_EHIP;
    if (rc != NTP_OK) set_error("attention kernel launch failed");
    return rc;
}

int launch_vec_add(float* a, const float* b, int64_t n, void* stream) {
    if (n <= 0) return NTP_OK;
    hipLaunchKernelGGL(vec_add_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, a, b, n);
    if (hipGetLastError() != hipSuccess) { set_error("kernel launch failed"); return NTP_EHIP; }
    return NTP_OK;
}

// By destination: phase 0 = whole rows (dq, t) and the first sweep of the segments (partial t),
// 1 = t of the split rows from their slots, 2 = second sweep of the segments (partial dq),
// 3 = dq of the split rows.  By source: phase 0 = whole rows and segments (partial dp), 1 = dp of
// the split rows.  The caller runs each phase over every chunk before the next one.
int launch_attention_bwd(const AttBwdArgs& a, const AttBwdRows& r, bool transposed, int phase, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    if (phase == 1 || phase == 3) {
        if (r.n_split_rows == 0) return NTP_OK;
        const bool is_t = phase == 1 && !transposed;
        hipLaunchKernelGGL(attention_bwd_combine_kernel, dim3((unsigned)((r.n_split_rows + 255) / 256)), dim3(256), 0, st,
                           r.split_rows, r.n_split_rows, a.slots, is_t ? a.t : a.out, is_t ? a.q : (const float*)nullptr,
                           is_t ? 0 : a.accumulate);
        if (hipGetLastError() != hipSuccess) { set_error("attention gradient kernel launch failed"); return NTP_EHIP; }
        return NTP_OK;
    }
    const bool vec4 = a.m % 4 == 0 && a.ld_own % 4 == 0 && a.ld_other % 4 == 0 &&
                      (uintptr_t)a.own % 16 == 0 && (uintptr_t)a.other % 16 == 0;
    int rc;
    if (vec4) rc = transposed ? launch_bwd_vec<4, true>(a, r, phase, st)
                              : launch_bwd_vec<4, false>(a, r, phase, st);
    else rc = transposed ? launch_bwd_vec<1, true>(a, r, phase, st)
                         : launch_bwd_vec<1, false>(a, r, phase, st);
    if (rc == NTP_EHIP) set_error("attention gradient kernel launch failed");
    return rc;
}

}  // namespace ntp
