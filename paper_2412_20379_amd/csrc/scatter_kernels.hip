// Backward aggregation as a scatter over the by-destination rows (Section 4.2.1 of the
// paper: the gradient of vertex v flows back along its in-edges to the sources):
//   Gin[colidx[k], :] += val[k] * Gout[v, :]   for every entry k of every row v.
// Used when the by-source form is not stored (NTP_SCATTER_BWD on a directed graph), which
// halves the topology held on the device and streamed from the host.  The additions are
// fp32 hardware atomics at the L2, so their order is not fixed: results agree with the
// gather form to rounding, not bit for bit.  fp32 buffers only.
//
// The work decomposition is the one of the gather kernel (same chunk image, same groups
// of wavefronts: lane group per short row, wavefront per long row, wavefront per segment
// of a split row); a segment needs no partial-sum slot here because every addition goes
// straight to its target row.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "lane_util.h"
#include "ntp_internal.h"

namespace ntp {

namespace {

// L lanes per feature row, lane l owns columns l, l + L, ... (NACC of them) of the pass
// blockIdx.y, so one atomic instruction of a lane group covers L consecutive floats of
// one target row.
template <int L, int NACC>
__global__ void __launch_bounds__(256) scatter_kernel(const AggArgs a) {
    constexpr int R = 64 / L;
    constexpr int PASS_W = L * NACC;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (wave >= a.wave_start[a.n_groups]) return;
    int grp = 0;
    while (grp + 1 < a.n_groups && wave >= a.wave_start[grp + 1]) ++grp;
    const int item0 = wave - a.wave_start[grp];
    const int mode = a.mode[grp];
    const int g = lane / L;
    const int l = lane % L;
    const int colbase = (int)blockIdx.y * PASS_W + l;

    const float* __restrict__ X = static_cast<const float*>(a.X);
    float* __restrict__ Y = static_cast<float*>(a.Y);
    bool on[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j) on[j] = colbase + j * L < a.f;

    float gv[NACC];
    auto load_row = [&](int row) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) gv[j] = on[j] ? X[(int64_t)row * a.ldx + colbase + j * L] : 0.f;
    };
    auto add_to = [&](int c, float w) {
        float* y = Y + (int64_t)c * a.ldy + colbase;
#pragma unroll
        for (int j = 0; j < NACC; ++j)
            if (on[j]) unsafeAtomicAdd(y + j * L, w * gv[j]);
    };

    if (mode == MODE_GROUP_PER_ROW) {
        const int idx = item0 * R + g;
        const bool valid = idx < a.item_count[grp];
        int row = 0;
        int64_t beg = a.e_base;
        int d = 0;
        if (valid) {
            row = a.rows[a.item_off[grp] + idx];
            beg = a.rowptr[row - a.row_base];
            d = (int)(a.rowptr[row - a.row_base + 1] - beg);
        }
#pragma unroll
        for (int j = 0; j < NACC; ++j) gv[j] = 0.f;
        if (valid) load_row(row);
        const int32_t* ci = a.colidx + (beg - a.e_base);
        const float* vv = a.val + (beg - a.e_base);
        for (int k0 = 0; __ballot(k0 < d) != 0; k0 += L) {
            int c = row;
            float w = 0.f;
            if (k0 + l < d) { c = __builtin_nontemporal_load(ci + k0 + l); w = __builtin_nontemporal_load(vv + k0 + l); }
            for (int j0 = 0; j0 < L; ++j0) {
                if (__ballot(k0 + j0 < d) == 0) break;
                const int cj = bperm_i(g * L + j0, c);
                const float wj = bperm_f(g * L + j0, w);
                if (k0 + j0 < d) add_to(cj, wj);
            }
        }
        return;
    }

    // one wavefront per row or per segment: all groups hold the same Gout row and take
    // every R-th entry
    int row;
    int64_t beg, end;
    if (mode == MODE_SEGMENT) {
        const Segment* sp = a.segs + a.item_off[grp] + item0;
        row = __builtin_amdgcn_readfirstlane(sp->row);
        beg = uniform64(sp->e_begin);
        end = beg + __builtin_amdgcn_readfirstlane(sp->len);
    } else {
        row = __builtin_amdgcn_readfirstlane(a.rows[a.item_off[grp] + item0]);
        beg = uniform64(a.rowptr[row - a.row_base]);
        end = uniform64(a.rowptr[row - a.row_base + 1]);
    }
    load_row(row);
    const int32_t* ci = a.colidx + (beg - a.e_base);
    const float* vv = a.val + (beg - a.e_base);
    const int64_t cnt = end - beg;
    for (int64_t base = 0; base < cnt; base += 64) {
        const int n = (int)(cnt - base < 64 ? cnt - base : 64);
        int c = row;
        float w = 0.f;
        if (lane < n) { c = __builtin_nontemporal_load(ci + base + lane); w = __builtin_nontemporal_load(vv + base + lane); }
        for (int j0 = 0; j0 * R < n; ++j0) {
            const int e = j0 * R + g;                  // < 64: j0 < L
            const int cj = bperm_i(e & 63, c);
            const float wj = bperm_f(e & 63, w);
            if (e < n) add_to(cj, wj);
        }
    }
}

template <class T>
__global__ void __launch_bounds__(256) zero_rows_kernel(T* Y, int64_t n, int64_t f, int64_t ld) {
    const int64_t total = n * f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / f, c = i - r * f;
        Y[r * ld + c] = (T)0;
    }
}

template <int L, int NACC>
int launch_scatter_one(const AggArgs& a, hipStream_t st) {
    const int total = a.wave_start[a.n_groups];
    if (total <= 0) return NTP_OK;
    const int passes = (a.f + L * NACC - 1) / (L * NACC);
    dim3 grid((unsigned)((total + 3) / 4), (unsigned)passes);
    hipLaunchKernelGGL((scatter_kernel<L, NACC>), grid, dim3(256), 0, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("scatter kernel launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    return NTP_OK;
}

}  // namespace

int scatter_lanes(int64_t f) {
    int L = 2;
    while (L < 64 && L < f) L <<= 1;
    return L;
}

int launch_scatter(const AggArgs& a, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    switch (scatter_lanes(a.f)) {
        case 2: return launch_scatter_one<2, 1>(a, st);
        case 4: return launch_scatter_one<4, 1>(a, st);
        case 8: return launch_scatter_one<8, 1>(a, st);
        case 16: return launch_scatter_one<16, 1>(a, st);
        case 32: return launch_scatter_one<32, 1>(a, st);
        default: break;
    }
    if (a.f <= 64) return launch_scatter_one<64, 1>(a, st);
    if (a.f <= 128) return launch_scatter_one<64, 2>(a, st);
    return launch_scatter_one<64, 4>(a, st);
}

int launch_zero_rows(void* Y, int64_t n, int64_t f, int64_t ld, int dtype, void* stream) {
    if (n <= 0 || f <= 0) return NTP_OK;
    hipStream_t st = (hipStream_t)stream;
    const int64_t total = n * f;
    const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 256 * 32);
    if (dtype == NTP_F32) hipLaunchKernelGGL(zero_rows_kernel<float>, dim3(blocks), dim3(256), 0, st, (float*)Y, n, f, ld);
    else hipLaunchKernelGGL(zero_rows_kernel<unsigned short>, dim3(blocks), dim3(256), 0, st, (unsigned short*)Y, n, f, ld);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("fill kernel launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    return NTP_OK;
}

}  // namespace ntp
