// Weights of a streamed chunk rebuilt on the device.  The chunk scheduling of Section 4.2.1 is
// bound by the host link when chunks do not stay resident; for a graph without caller weights the
// stored values follow from the structure alone (the GCN normalisation 1 / sqrt(din(v) dout(u)) of
// Section 4.1.3, or 1), so only the column ids travel and the values are recomputed after the
// copy: half the bytes per chunk.  The arithmetic is the host's, step for step in IEEE double
// (product of the two degrees, square root, reciprocal, one rounding to fp32), so the rebuilt
// values are the stored ones bit for bit.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "ntp_internal.h"

namespace ntp {

namespace {

constexpr int ENTRIES_PER_BLOCK = 256 * 16;

// largest r in [lo, hi] with rowptr[r] <= e  (rowptr[lo] <= e is given)
__device__ __forceinline__ int64_t row_of(const int64_t* __restrict__ rowptr, int64_t lo, int64_t hi, int64_t e) {
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (rowptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__global__ void __launch_bounds__(256) rebuild_weights_kernel(const int64_t* __restrict__ rowptr, int64_t row_base, int64_t n_rows,
                                                              int64_t e_base, int64_t n_entries, const int32_t* __restrict__ colidx,
                                                              float* __restrict__ val, const int32_t* __restrict__ deg_row,
                                                              const int32_t* __restrict__ deg_col, int mode) {
    __shared__ int64_t span[2];
    const int64_t first = (int64_t)blockIdx.x * ENTRIES_PER_BLOCK;
    const int64_t last = std::min<int64_t>(first + ENTRIES_PER_BLOCK, n_entries) - 1;
    if (mode == VAL_ONES) {
        for (int64_t i = first + threadIdx.x; i <= last; i += 256) val[i] = 1.0f;
        return;
    }
    // rows this block's entries lie in (entries are ordered by row); a chunk that holds part of
    // one row has n_rows = 1 and every entry belongs to that row
    if (threadIdx.x < 2) span[threadIdx.x] = row_of(rowptr, 0, n_rows - 1, e_base + (threadIdx.x == 0 ? first : last));
    __syncthreads();
    const int64_t r_lo = span[0], r_hi = span[1];
    for (int64_t i = first + threadIdx.x; i <= last; i += 256) {
        const int64_t r = row_of(rowptr, r_lo, r_hi, e_base + i);
        const double prod = (double)deg_row[row_base + r] * (double)deg_col[colidx[i]];
        const double scale = 1.0 / sqrt(prod);
        val[i] = (float)scale;
    }
}

}  // namespace

int launch_rebuild_weights(const int64_t* rowptr, int64_t row_base, int64_t n_rows, int64_t e_base, int64_t n_entries,
                           const int32_t* colidx, float* val, const int32_t* deg_row, const int32_t* deg_col, int mode,
                           void* stream) {
    if (n_entries <= 0) return NTP_OK;
    const int64_t blocks = (n_entries + ENTRIES_PER_BLOCK - 1) / ENTRIES_PER_BLOCK;
    hipLaunchKernelGGL(rebuild_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, rowptr, row_base, n_rows,
                       e_base, n_entries, colidx, val, deg_row, deg_col, mode);
    if (hipGetLastError() != hipSuccess) { set_error("weight rebuild kernel launch failed"); return NTP_EHIP; }
    return NTP_OK;
}

}  // namespace ntp
