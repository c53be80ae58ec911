// The vertex-associated half of the GAT attention of Section 2.1: the mapping a^T [W h_u || W h_v]
// splits into two per-vertex scalars, p[v] = Z[v,:] . a_src and q[v] = Z[v,:] . a_dst (Z = the
// transformed embeddings), which the edge kernels combine per edge.  Forward: both dot products
// from one read of Z.  Backward (chain rule through the two products): the gradient of Z gains
// dp[v] a_src + dq[v] a_dst, and da_src = Z^T dp, da_dst = Z^T dq.
//
// Forward: a group of L lanes per vertex (L = 4..64 by the width), xor-tree sums.  Backward: a
// block owns a contiguous range of vertices; thread (ty, tx) walks the vertices ty, ty + TY, ...
// of the range for the columns tx, tx + TX, ...; the column sums of a block are combined over ty
// in a fixed order through LDS and those of the blocks by a second kernel in block order, so the
// result is deterministic.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "lane_util.h"
#include "ntp_internal.h"

namespace ntp {

namespace {

constexpr int MAXC = 4;            // column slots per thread in the backward kernel: widths up to 4 * 256
constexpr int MAX_BLOCKS = 512;    // partial column sums kept per call


template <int L>
__global__ void __launch_bounds__(256) scores_fwd_kernel(const float* __restrict__ Z, const float* __restrict__ a_src,
                                                         const float* __restrict__ a_dst, float* __restrict__ p,
                                                         float* __restrict__ q, int64_t n, int m, int64_t ldz) {
    constexpr int R = 64 / L;
    const int lane = threadIdx.x & 63;
    const int g = lane / L, l = lane % L;
    const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * R + g;
    const bool valid = row < n;
    const float* z = Z + (valid ? row : 0) * ldz;
    float sp = 0.f, sq = 0.f;
    if (valid)
        for (int j = l; j < m; j += L) {
            const float x = z[j];
            sp = fmaf(x, a_src[j], sp);
            sq = fmaf(x, a_dst[j], sq);
        }
#pragma unroll
    for (int off = 1; off < L; off <<= 1) {
        sp += bperm_f(lane ^ off, sp);
        sq += bperm_f(lane ^ off, sq);
    }
    if (valid && l == 0) { p[row] = sp; q[row] = sq; }
}

// TX columns x TY vertices per block step, TX * TY = 256
template <int TX>
__global__ void __launch_bounds__(256) scores_bwd_kernel(const float* __restrict__ Z, const float* __restrict__ a_src,
                                                         const float* __restrict__ a_dst, const float* __restrict__ dp,
                                                         const float* __restrict__ dq, float* __restrict__ dZ,
                                                         float* __restrict__ partial, int64_t n, int m, int64_t ldz,
                                                         int64_t lddz, int64_t rows_per_block) {
    constexpr int TY = 256 / TX;
    __shared__ float red[256];
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
    float as[MAXC], ad[MAXC], acc_s[MAXC], acc_d[MAXC];
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int c = tx + j * TX;
        as[j] = c < m ? a_src[c] : 0.f;
        ad[j] = c < m ? a_dst[c] : 0.f;
        acc_s[j] = 0.f;
        acc_d[j] = 0.f;
    }
    for (int64_t r = r0 + ty; r < r1; r += TY) {
        const float gp = dp[r], gq = dq[r];
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
            const int c = tx + j * TX;
            if (c < m) {
                const float z = Z[r * ldz + c];
                dZ[r * lddz + c] += gp * as[j] + gq * ad[j];
                acc_s[j] = fmaf(z, gp, acc_s[j]);
                acc_d[j] = fmaf(z, gq, acc_d[j]);
            }
        }
    }
    // column sums of the block: over ty in order, one slot and one vector at a time
    float* out = partial + (int64_t)blockIdx.x * 2 * m;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            red[threadIdx.x] = which ? acc_d[j] : acc_s[j];
            __syncthreads();
            const int c = tx + j * TX;
            if (ty == 0 && c < m) {
                float s = 0.f;
                for (int y = 0; y < TY; ++y) s += red[y * TX + tx];
                out[which * m + c] = s;
            }
            __syncthreads();
        }
    }
}

__global__ void __launch_bounds__(256) scores_bwd_final_kernel(const float* __restrict__ partial, float* __restrict__ da_src,
                                                               float* __restrict__ da_dst, int m, int n_blocks) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= m) return;
    float s = 0.f, d = 0.f;
    for (int b = 0; b < n_blocks; ++b) {
        s += partial[(int64_t)b * 2 * m + c];
        d += partial[(int64_t)b * 2 * m + m + c];
    }
    da_src[c] = s;
    da_dst[c] = d;
}

int bwd_tx(int64_t m) {
    int tx = 4;
    while (tx < 256 && tx < m) tx <<= 1;
    return tx;
}

int bwd_blocks(int64_t n, int64_t m) {
    const int ty = 256 / bwd_tx(m);
    const int64_t want = (n + (int64_t)ty * 16 - 1) / ((int64_t)ty * 16);       // about 16 vertices per thread
    return (int)std::max<int64_t>(1, std::min<int64_t>(want, MAX_BLOCKS));
}

}  // namespace

int64_t attention_scores_max_width() { return (int64_t)MAXC * 256; }

int64_t attention_scores_bwd_scratch_bytes(int64_t n, int64_t m) {
    if (n <= 0 || m <= 0) return 0;
    return (int64_t)bwd_blocks(n, m) * 2 * m * (int64_t)sizeof(float);
}

int launch_attention_scores_fwd(const float* Z, const float* a_src, const float* a_dst, float* p, float* q,
                                int64_t n, int64_t m, int64_t ldz, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    int L = 4;
    while (L < 64 && L < m) L <<= 1;
    const int64_t rows_per_block = 4 * (64 / L);
    const dim3 grid((unsigned)((n + rows_per_block - 1) / rows_per_block));
#define NTP_SCORES_FWD(LL) hipLaunchKernelGGL(scores_fwd_kernel<LL>, grid, dim3(256), 0, st, Z, a_src, a_dst, p, q, n, (int)m, ldz)
    switch (L) {
        case 4: NTP_SCORES_FWD(4); break;
        case 8: NTP_SCORES_FWD(8); break;
        case 16: NTP_SCORES_FWD(16); break;
        case 32: NTP_SCORES_FWD(32); break;
        default: NTP_SCORES_FWD(64); break;
    }
#undef NTP_SCORES_FWD
    if (hipGetLastError() != hipSuccess) { set_error("attention score kernel launch failed"); return NTP_EHIP; }
    return NTP_OK;
}

int launch_attention_scores_bwd(const float* Z, const float* a_src, const float* a_dst, const float* dp, const float* dq,
                                float* dZ, float* da_src, float* da_dst, int64_t n, int64_t m, int64_t ldz, int64_t lddz,
                                float* scratch, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    const int nb = bwd_blocks(n, m);
    const int64_t rows_per_block = (n + nb - 1) / nb;
#define NTP_SCORES_BWD(TX) hipLaunchKernelGGL(scores_bwd_kernel<TX>, dim3((unsigned)nb), dim3(256), 0, st, Z, a_src, a_dst, dp, dq, dZ, \
                                              scratch, n, (int)m, ldz, lddz, rows_per_block)
    switch (bwd_tx(m)) {
        case 4: NTP_SCORES_BWD(4); break;
        case 8: NTP_SCORES_BWD(8); break;
        case 16: NTP_SCORES_BWD(16); break;
        case 32: NTP_SCORES_BWD(32); break;
        case 64: NTP_SCORES_BWD(64); break;
        case 128: NTP_SCORES_BWD(128); break;
        default: NTP_SCORES_BWD(256); break;
    }
#undef NTP_SCORES_BWD
    hipLaunchKernelGGL(scores_bwd_final_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st, scratch, da_src, da_dst, (int)m, nb);
    if (hipGetLastError() != hipSuccess) { set_error("attention score gradient kernel launch failed"); return NTP_EHIP; }
    return NTP_OK;
}

}  // namespace ntp
