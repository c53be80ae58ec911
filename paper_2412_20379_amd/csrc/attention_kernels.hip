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

#include "ntp_internal.h"

namespace ntp {

namespace {

__device__ __forceinline__ float bperm_f(int src_lane, float v) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}
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
// in that order, with t[v] and alpha in by-source order: dp[u].  A group of 16 lanes forms one dot
// product at a time (16 x VEC x NJ columns, xor tree over the 16 lanes); rows beyond the split
// threshold take one block (16 groups over the entries, partial sums combined through LDS in a
// fixed order).  Every entry's parked dalpha is read back by the thread that wrote it.
template <int VEC, int NJ>
struct DotRow {
    float own[NJ][VEC];
    int col[NJ];
    bool on[NJ];
    __device__ __forceinline__ void load_own(const float* row, int l, int m) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            col[j] = (j * 16 + l) * VEC;
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
    __device__ __forceinline__ float partial(const float* other) const {
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (on[j]) {
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

// WORK_GROUP  : four rows per wavefront (one group each), rows[first .. first + n_rows).
// WORK_BLOCK  : one row per block of 16 groups, rows[first + blockIdx.x].
// WORK_SEG    : one segment of a split row per block, segs[blockIdx.x]: the dot products of its
//               entries; the partial t (by destination) or partial dp (by source) goes to the
//               segment's slot.
// WORK_SEG_DS : by destination only, after the slots of t were combined: ds of the segment's
//               entries from the parked dalpha, partial dq to the slot.
enum { WORK_GROUP = 0, WORK_BLOCK = 1, WORK_SEG = 2, WORK_SEG_DS = 3 };

template <int VEC, int NJ, bool TRANSPOSED, int WORK>
__global__ void __launch_bounds__(256) attention_bwd_kernel(const AttBwdArgs a, int first, int n_rows, const Segment* segs) {
    __shared__ float red[16];
    constexpr bool BLOCK = WORK != WORK_GROUP;
    constexpr bool SEG = WORK == WORK_SEG || WORK == WORK_SEG_DS;
    constexpr int U = 4;                                               // dot products in flight per group
    const int lane = threadIdx.x & 63;
    const int l = lane & 15;
    const int gi = BLOCK ? (int)(threadIdx.x >> 4) : (lane >> 4);      // group inside the block / wavefront
    constexpr int GSTRIDE = BLOCK ? 16 : 1;                            // groups sharing a row
    int row = 0;
    int slot = 0;
    bool valid = true;
    int64_t beg = 0, d = 0;
    if constexpr (SEG) {
        const Segment sg = segs[blockIdx.x];
        row = sg.row; slot = sg.slot; beg = sg.e_begin; d = sg.len;
    } else {
        if constexpr (BLOCK) {
            row = a.rows[first + blockIdx.x];
        } else {
            const int64_t idx = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 4 + gi;
            valid = idx < n_rows;
            if (valid) row = a.rows[first + idx];
        }
        if (valid) { beg = a.rowptr[row]; d = a.rowptr[row + 1] - beg; }
    }
    const int32_t* ci = a.colidx + beg;
    const float* al = a.alpha + beg;
    float* park = a.park + beg;
    // sum of one value per group over the block, in group order (every thread gets it)
    auto block_sum = [&](float v) {
        if (l == 0) red[gi] = v;
        __syncthreads();
        float s = 0.f;
        for (int i = 0; i < 16; ++i) s += red[i];
        __syncthreads();
        return s;
    };
    if constexpr (WORK == WORK_SEG_DS) {
        const float t = a.t[row];
        const float qv = a.q[row];
        float dqp = 0.f;
        for (int64_t k = threadIdx.x; k < d; k += 256) {
            const int cc = ci[k];
            dqp += al[k] * (park[k] - t) * (a.p[cc] + qv > 0.f ? 1.f : a.slope);
        }
        dqp = block_sum(group_sum<16>(dqp, lane));
        if (threadIdx.x == 0) a.slots[slot] = dqp;
        return;
    }
    DotRow<VEC, NJ> dot;
    dot.load_own(a.own + (int64_t)row * a.ld_own, l, valid ? a.m : 0);
    const int k_first = BLOCK ? gi : 0;
    // dalpha of entries k, k + GSTRIDE, ...: U gathers issued before the first xor tree
    auto dots = [&](int64_t k, bool (&in)[U], int (&c)[U], float (&da)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) { in[u] = k + u * GSTRIDE < d; c[u] = in[u] ? ci[k + u * GSTRIDE] : row; }
#pragma unroll
        for (int u = 0; u < U; ++u) da[u] = dot.partial(a.other + (int64_t)c[u] * a.ld_other);
#pragma unroll
        for (int u = 0; u < U; ++u) da[u] = group_sum<16>(da[u], lane);
    };
    bool in[U];
    int c[U];
    float da[U];
    if constexpr (TRANSPOSED) {
        const float pu = valid ? a.p[row] : 0.f;
        float acc = 0.f;
        for (int64_t k = k_first; __ballot(k < d) != 0; k += U * GSTRIDE) {   // the wavefront stays together for the shuffles
            dots(k, in, c, da);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (in[u]) acc += al[k + u * GSTRIDE] * (da[u] - a.t[c[u]]) * (pu + a.q[c[u]] > 0.f ? 1.f : a.slope);
        }
        if constexpr (BLOCK) {
            acc = block_sum(acc);
            if (threadIdx.x == 0) { if constexpr (SEG) a.slots[slot] = acc; else a.out[row] = acc; }
        } else {
            if (valid && l == 0) a.out[row] = acc;
        }
        return;
    }
    // by destination: sweep 1 = dalpha of every entry (parked by the lane that reads it back), t
    float t = 0.f;
    for (int64_t k = k_first; __ballot(k < d) != 0; k += U * GSTRIDE) {
        dots(k, in, c, da);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (in[u]) {
                const int64_t ku = k + u * GSTRIDE;
                t += al[ku] * da[u];
                const int owner = BLOCK ? (int)((ku / 16) & 15) : (int)(ku & 15);
                if (l == owner) park[ku] = da[u];
            }
        }
    }
    if constexpr (BLOCK) t = block_sum(t);
    if constexpr (SEG) {
        if (threadIdx.x == 0) a.slots[slot] = t;
        return;
    }
    // sweep 2: ds of the entries this lane parked, summed over the row
    const float qv = valid ? a.q[row] : 0.f;
    float dqp = 0.f;
    for (int64_t k = BLOCK ? gi + 16 * l : l; k < d; k += BLOCK ? 256 : 16) {   // BLOCK: k % 16 == gi, (k / 16) % 16 == l
        const int cc = ci[k];
        dqp += al[k] * (park[k] - t) * (a.p[cc] + qv > 0.f ? 1.f : a.slope);
    }
    dqp = group_sum<16>(dqp, lane);
    if constexpr (BLOCK) {
        dqp = block_sum(dqp);
        if (threadIdx.x == 0) { a.out[row] = dqp; a.t[row] = t; }
    } else {
        if (valid && l == 0) { a.out[row] = dqp; a.t[row] = t; }
    }
}

// out[row] = sum of the row's slots, in segment order
__global__ void __launch_bounds__(256) attention_bwd_combine_kernel(const ReduceItem* items, int n_items, const float* slots, float* out) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_items) return;
    const ReduceItem it = items[i];
    float s = 0.f;
    for (int j = 0; j < it.n_slots; ++j) s += slots[it.first_slot + j];
    out[it.row] = s;
}

template <int VEC, int NJ, bool T>
int launch_bwd_shape(const AttBwdArgs& a, const AttBwdRows& r, int phase, hipStream_t st) {
    const Segment* none = nullptr;
    if (phase == 0) {
        if (r.n_segs > 0)
            hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, T, WORK_SEG>), dim3((unsigned)r.n_segs), dim3(256), 0, st, a, 0, 0, r.segs);
        if (r.n_block_rows > 0)
            hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, T, WORK_BLOCK>), dim3((unsigned)r.n_block_rows), dim3(256), 0, st, a, r.n_group_rows, 0, none);
        if (r.n_group_rows > 0)
            hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, T, WORK_GROUP>), dim3((unsigned)((r.n_group_rows + 15) / 16)), dim3(256), 0, st, a, 0,
                               r.n_group_rows, none);
    } else if (phase == 2) {
        if constexpr (!T) {
            if (r.n_segs > 0)
                hipLaunchKernelGGL((attention_bwd_kernel<VEC, NJ, false, WORK_SEG_DS>), dim3((unsigned)r.n_segs), dim3(256), 0, st, a, 0, 0, r.segs);
        }
    }
    return hipGetLastError() == hipSuccess ? NTP_OK : NTP_EHIP;
}

template <int VEC, bool T>
int launch_bwd_vec(const AttBwdArgs& a, const AttBwdRows& r, int phase, hipStream_t st) {
    const int per = 16 * VEC;
    const int nj = (a.m + per - 1) / per;
    if (nj <= 1) return launch_bwd_shape<VEC, 1, T>(a, r, phase, st);
    if (nj <= 2) return launch_bwd_shape<VEC, 2, T>(a, r, phase, st);
    if (nj <= 4) return launch_bwd_shape<VEC, 4, T>(a, r, phase, st);
    if (nj <= 8) return launch_bwd_shape<VEC, 8, T>(a, r, phase, st);
    if (nj <= 16) return launch_bwd_shape<VEC, 16, T>(a, r, phase, st);
    set_error("feature width %d too large for the attention gradient (at most %d)", a.m, 16 * per);
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

// widest feature row the gradient kernels take: 1024 columns with 16-byte vectors, 256 otherwise
// By destination: phase 0 = whole rows (dq, t) and the first sweep of the segments (partial t),
// 1 = t of the split rows from their slots, 2 = second sweep of the segments (partial dq),
// 3 = dq of the split rows.  By source: phase 0 = whole rows and segments (partial dp), 1 = dp of
// the split rows.  The caller runs each phase over every chunk before the next one.
int launch_attention_bwd(const AttBwdArgs& a, const AttBwdRows& r, bool transposed, int phase, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    if (phase == 1 || phase == 3) {
        if (r.n_split_rows == 0) return NTP_OK;
        float* dst = (phase == 1 && !transposed) ? a.t : a.out;
        hipLaunchKernelGGL(attention_bwd_combine_kernel, dim3((unsigned)((r.n_split_rows + 255) / 256)), dim3(256), 0, st,
                           r.split_rows, r.n_split_rows, a.slots, dst);
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
