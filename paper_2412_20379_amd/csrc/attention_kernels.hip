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

}  // namespace ntp
