// Softmax cross-entropy of the vertex classification task that closes an epoch (the
// downstream task of Alg. 1): loss = mean over the vertices of -log softmax(Z[v,:])[label[v]],
// and its gradient dZ = (softmax(Z) - onehot(label)) / n, which starts the reverse loop.
//
// One group of L lanes per vertex (L = 8..64 by the number of classes, up to eight classes per lane); the row maximum, the
// sum of exponentials and the per-vertex loss come from fixed xor trees.  The mean is taken
// in two fixed-order steps (1024 partial sums, then one block), so the loss is deterministic.
#include <hip/hip_runtime.h>

#include <cmath>

#include "lane_util.h"
#include "ntp_internal.h"

namespace ntp {

namespace {

template <int L>
__global__ void __launch_bounds__(256) xent_rows_kernel(const float* __restrict__ Z, const int64_t* __restrict__ labels,
                                                        float* __restrict__ dZ, float* __restrict__ row_loss,
                                                        int64_t n, int c, int64_t ldz, int64_t lddz, float inv_n) {
    constexpr int R = 64 / L;
    const int lane = threadIdx.x & 63;
    const int g = lane / L, l = lane % L;
    const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * R + g;
    const bool valid = row < n;
    const float* z = Z + (valid ? row : 0) * ldz;
    float m = -INFINITY;
    if (valid)
        for (int j = l; j < c; j += L) m = fmaxf(m, z[j]);
#pragma unroll
    for (int off = 1; off < L; off <<= 1) m = fmaxf(m, bperm_f(lane ^ off, m));
    float s = 0.f;
    if (valid)
        for (int j = l; j < c; j += L) s += expf(z[j] - m);
#pragma unroll
    for (int off = 1; off < L; off <<= 1) s += bperm_f(lane ^ off, s);
    if (!valid) return;
    const int lab = (int)labels[row];
    const float rs = 1.f / s;
    float* d = dZ + row * lddz;
    for (int j = l; j < c; j += L) d[j] = (expf(z[j] - m) * rs - (j == lab ? 1.f : 0.f)) * inv_n;
    if (l == 0) row_loss[row] = (lab >= 0 && lab < c) ? -(z[lab] - m - logf(s)) : 0.f;
}

// partial[b] = sum of row_loss over the b-th of 1024 contiguous ranges (fixed order inside a block)
__global__ void __launch_bounds__(256) xent_partial_kernel(const float* __restrict__ row_loss, float* __restrict__ partial, int64_t n) {
    __shared__ float red[256];
    const int64_t per = (n + 1023) / 1024;
    const int64_t beg = (int64_t)blockIdx.x * per;
    const int64_t end = beg + per < n ? beg + per : n;
    float s = 0.f;
    for (int64_t i = beg + threadIdx.x; i < end; i += 256) s += row_loss[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(256) xent_final_kernel(const float* __restrict__ partial, float* __restrict__ loss, float inv_n) {
    __shared__ float red[256];
    red[threadIdx.x] = (partial[threadIdx.x] + partial[threadIdx.x + 256]) + (partial[threadIdx.x + 512] + partial[threadIdx.x + 768]);
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = red[0] * inv_n;
}

template <int L>
void launch_rows(const float* Z, const int64_t* labels, float* dZ, float* row_loss, int64_t n, int c,
                 int64_t ldz, int64_t lddz, hipStream_t st) {
    const int64_t rows_per_block = 4 * (64 / L);
    hipLaunchKernelGGL((xent_rows_kernel<L>), dim3((unsigned)((n + rows_per_block - 1) / rows_per_block)), dim3(256), 0, st,
                       Z, labels, dZ, row_loss, n, c, ldz, lddz, 1.f / (float)n);
}

}  // namespace

// scratch: n + 1024 floats (per-vertex losses, then the partial sums)
int launch_softmax_xent(const float* Z, const int64_t* labels, float* dZ, float* loss, float* scratch,
                        int64_t n, int64_t c, int64_t ldz, int64_t lddz, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    // up to eight classes per lane: eight vertices per wavefront for the usual class counts
    if (c <= 64) launch_rows<8>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    else if (c <= 128) launch_rows<16>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    else if (c <= 256) launch_rows<32>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    else launch_rows<64>(Z, labels, dZ, scratch, n, (int)c, ldz, lddz, st);
    hipLaunchKernelGGL(xent_partial_kernel, dim3(1024), dim3(256), 0, st, scratch, scratch + n, n);
    hipLaunchKernelGGL(xent_final_kernel, dim3(1), dim3(256), 0, st, scratch + n, loss, 1.f / (float)n);
    if (hipGetLastError() != hipSuccess) { set_error("loss kernel launch failed"); return NTP_EHIP; }
    return NTP_OK;
}

}  // namespace ntp
