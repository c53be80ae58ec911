// Softmax cross-entropy of the vertex classification task that closes an epoch (the
// downstream task of Alg. 1): loss = mean over the vertices of -log softmax(Z[v,:])[label[v]],
// and its gradient dZ = (softmax(Z) - onehot(label)) / n, which starts the reverse loop.
//
// One group of L lanes per vertex (L = 8..64 by the number of classes, up to eight classes per lane); the row maximum, the
// sum of exponentials and the per-vertex loss come from fixed xor trees.  The mean is taken
// in fixed-order steps (one sum per block of the first kernel, then one block, with 1024 partial
// sums in between when there are many), so the loss is deterministic.
#include <hip/hip_runtime.h>

#include <cmath>

#include "lane_util.h"
#include "ntp_internal.h"

namespace ntp {

namespace {

// One group of L lanes per vertex.  With at most eight classes per lane (IN_REGS) the row is read
// once and kept in registers together with its exponentials.  The block adds up the losses of
// its vertices in a fixed order (xor tree over the wavefront, then (w0 + w1) + (w2 + w3)) and
// writes one partial sum.
template <int L, bool IN_REGS>
__global__ void __launch_bounds__(256) xent_rows_kernel(const float* __restrict__ Z, const int64_t* __restrict__ labels,
                                                        float* __restrict__ dZ, float* __restrict__ block_loss,
                                                        int64_t n, int c, int64_t ldz, int64_t lddz, float inv_n) {
    constexpr int R = 64 / L;
    __shared__ float wsum[4];
    const int lane = threadIdx.x & 63;
    const int g = lane / L, l = lane % L;
    const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * R + g;
    const bool valid = row < n;
    const float* z = Z + (valid ? row : 0) * ldz;
    float v[8];
    float m = -INFINITY;
    if constexpr (IN_REGS) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = l + i * L;
            v[i] = (valid && j < c) ? z[j] : -INFINITY;
            m = fmaxf(m, v[i]);
        }
    } else {
        if (valid)
            for (int j = l; j < c; j += L) m = fmaxf(m, z[j]);
    }
#pragma unroll
    for (int off = 1; off < L; off <<= 1) m = fmaxf(m, bperm_f(lane ^ off, m));
    float s = 0.f;
    if constexpr (IN_REGS) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            v[i] = (valid && l + i * L < c) ? expf(v[i] - m) : 0.f;
            s += v[i];
        }
    } else {
        if (valid)
            for (int j = l; j < c; j += L) s += expf(z[j] - m);
    }
#pragma unroll
    for (int off = 1; off < L; off <<= 1) s += bperm_f(lane ^ off, s);
    float rl = 0.f;
    if (valid) {
        const int lab = (int)labels[row];
        const float rs = 1.f / s;
        float* d = dZ + row * lddz;
        if constexpr (IN_REGS) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int j = l + i * L;
                if (j < c) d[j] = (v[i] * rs - (j == lab ? 1.f : 0.f)) * inv_n;
            }
        } else {
            for (int j = l; j < c; j += L) d[j] = (expf(z[j] - m) * rs - (j == lab ? 1.f : 0.f)) * inv_n;
        }
        if (l == 0 && lab >= 0 && lab < c) rl = -(z[lab] - m - logf(s));
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) rl += bperm_f(lane ^ off, rl);
    if (lane == 0) wsum[threadIdx.x >> 6] = rl;
    __syncthreads();
    if (threadIdx.x == 0) block_loss[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// partial[b] = sum of v over the b-th of 1024 contiguous ranges (fixed order inside a block)
__global__ void __launch_bounds__(256) xent_partial_kernel(const float* __restrict__ v, float* __restrict__ partial, int64_t n) {
    __shared__ float red[256];
    const int64_t per = (n + 1023) / 1024;
    const int64_t beg = (int64_t)blockIdx.x * per;
    const int64_t end = beg + per < n ? beg + per : n;
    float s = 0.f;
    for (int64_t i = beg + threadIdx.x; i < end; i += 256) s += v[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// loss = inv_n x sum of count partial sums: thread t adds t, t + 256, ... in ascending order, then a fixed tree
__global__ void __launch_bounds__(256) xent_final_kernel(const float* __restrict__ partial, int count, float* __restrict__ loss, float inv_n) {
    __shared__ float red[256];
    float s = 0.f;
    for (int i = threadIdx.x; i < count; i += 256) s += partial[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = red[0] * inv_n;
}

// returns the number of blocks (= partial sums written to block_loss)
template <int L>
int64_t launch_rows(const float* Z, const int64_t* labels, float* dZ, float* block_loss, int64_t n, int c,
                    int64_t ldz, int64_t lddz, hipStream_t st) {
    const int64_t rows_per_block = 4 * (64 / L);
    const int64_t blocks = (n + rows_per_block - 1) / rows_per_block;
    if (c <= 8 * L)
        hipLaunchKernelGGL((xent_rows_kernel<L, true>), dim3((unsigned)blocks), dim3(256), 0, st,
                           Z, labels, dZ, block_loss, n, c, ldz, lddz, 1.f / (float)n);
    else
        hipLaunchKernelGGL((xent_rows_kernel<L, false>), dim3((unsigned)blocks), dim3(256), 0, st,
                           Z, labels, dZ, block_loss, n, c, ldz, lddz, 1.f / (float)n);
    return blocks;
}

}  // namespace

// scratch: n + 1024 floats (the blocks' sums at the start, the 1024 partial sums from float n on)
int launch_softmax_xent(const float* Z, const int64_t* labels, float* dZ, float* loss, float* scratch,
                        int64_t n, int64_t c, int64_t ldz, int64_t lddz, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    // up to eight classes per lane: eight vertices per wavefront for the usual class counts
    int64_t nb;
    if (c <= 64) nb = launch_rows<8>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    else if (c <= 128) nb = launch_rows<16>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    else if (c <= 256) nb = launch_rows<32>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    else nb = launch_rows<64>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    // the blocks' sums (at most n / 4 + 1 of them, at the start of the scratch): one block adds
    // up to 16384 of them directly, more go through 1024 partial sums first
    if (nb <= 16384) {
        hipLaunchKernelGGL(xent_final_kernel, dim3(1), dim3(256), 0, st, scratch, (int)nb, loss, 1.f / (float)n);
    } else {
        hipLaunchKernelGGL(xent_partial_kernel, dim3(1024), dim3(256), 0, st, scratch, scratch + n, nb);
        hipLaunchKernelGGL(xent_final_kernel, dim3(1), dim3(256), 0, st, scratch + n, 1024, loss, 1.f / (float)n);
    }
    if (hipGetLastError() != hipSuccess) { set_error("loss kernel launch failed"); return NTP_EHIP; }
    return NTP_OK;
}

}  // namespace ntp
