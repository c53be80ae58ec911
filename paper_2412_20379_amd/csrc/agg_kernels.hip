// Aggregation kernels for gfx950: Y[v,:] = sum_k val[k] * X[colidx[k],:] over the entries
// of row v (eq. 1/3 of the paper on one column slice; the same kernel runs the by-source
// rows for the backward pass of Section 4.2.1).
//
// Mapping.  A wavefront (64 lanes) is cut into R = 64/L groups of L lanes; the L lanes
// of a group cover one feature row with one 4/8/16-byte vector load each, so a gather of
// one neighbour row is one coalesced access.  Rows are binned by entry count on the host:
//   - rows of up to 32 entries: one group per row, R rows per wavefront (no cross-lane
//     reduction);
//   - longer rows: one wavefront per row; 64 (index, weight) pairs are fetched with one
//     coalesced load per lane, handed to the groups through the cross-lane network, the R
//     groups gather R neighbour rows at a time and their sums are combined by a butterfly;
//   - rows beyond the split threshold: cut into segments, one wavefront per segment, fp32
//     partial sums to a scratch slot; reduce_kernel adds the slots of a row in order.
// No atomics anywhere: the result is deterministic.
//
// Hub table (agg_hub_kernel).  Every gathered row misses the L1.  On a power-law graph a few columns take a large
// share of the gathers, so the graph build marks the most gathered columns ("hubs") in a second
// column-id array: a hub entry carries 0x80000000 | slot instead of its vertex id.  The hub
// kernel runs one persistent block of 16 wavefronts per compute unit, which first copies the hub
// rows of its column pass into an LDS table (one line of L x 16 bytes per slot) and then works
// through the launch's rows exactly as agg_kernel does, except that a hub entry's row comes from
// LDS.  No look-up and no branch: the sign of the id selects the source, the global load of a
// hub entry is pointed at the first hub's row (a line every wavefront keeps touching, so it
// stays in the L1), and the summation order is that of agg_kernel: same bits.
// Measured on MI355X it does not pay and is therefore opt-in (graphs built with NTP_AGG_HUB=1 in
// the environment): the L1-to-L2 requests fall by the hubs' share of the gathers (a third on a
// 2.5 M-entry R-MAT graph), but the persistent blocks run 20-35 % behind the plain kernel with
// one slot as with 1024, i.e. what the table saves never becomes the bottleneck: the launch time is
// set by the gathers that miss the L2 (random lines beyond it arrive at 53-56 G lines/s on this chip),
// and hub rows are the ones that hit it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

#include "lane_util.h"
#include "ntp_internal.h"

namespace ntp {

namespace {

__device__ __forceinline__ unsigned f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// ---- element access: VEC consecutive elements <-> VEC floats -------------------------
template <int VEC> struct IoF32 {
    static_assert(VEC == 1 || VEC == 2 || VEC == 4, "fp32 vectors of 1, 2 or 4 elements");
    using elem = float;
    static constexpr int kVec = VEC;
    static __device__ __forceinline__ void load(const float* p, float (&v)[VEC]) {
        if constexpr (VEC == 4) { const float4 t = *reinterpret_cast<const float4*>(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
        else if constexpr (VEC == 2) { const float2 t = *reinterpret_cast<const float2*>(p); v[0] = t.x; v[1] = t.y; }
        else { v[0] = *p; }
    }
    static __device__ __forceinline__ void store(float* p, const float (&v)[VEC]) {
        if constexpr (VEC == 4) {
            // written once and not read again by this kernel: a non-temporal store keeps the
            // output rows from displacing gathered rows in the L2 (measured: 1-5 % on the
            // low-degree config at 256 columns, nothing lost elsewhere)
            typedef float v4f __attribute__((ext_vector_type(4)));
            const v4f t = {v[0], v[1], v[2], v[3]};
            __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
        }
        else if constexpr (VEC == 2) { *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]); }
        else { *p = v[0]; }
    }
    static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
    // exact copy of loaded elements (for staging in LDS)
    static __device__ __forceinline__ void store_plain(float* p, const float (&v)[VEC]) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) p[i] = v[i];
    }
};

// VEC fp32 partial sums to scratch (VEC may be 8 for bf16 features)
template <int VEC>
__device__ __forceinline__ void store_partial(float* p, const float (&v)[VEC]) {
    if constexpr (VEC == 8) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
        IoF32<VEC>::store(p, v);
    }
}

template <int VEC> struct IoBf16 {
    static_assert(VEC == 1 || VEC == 2 || VEC == 4 || VEC == 8, "bf16 vectors of 1, 2, 4 or 8 elements");
    using elem = unsigned short;
    static constexpr int kVec = VEC;
    static __device__ __forceinline__ void unpack(unsigned w, float& lo, float& hi) {
        lo = __uint_as_float(w << 16);
        hi = __uint_as_float(w & 0xffff0000u);
    }
    static __device__ __forceinline__ void load(const unsigned short* p, float (&v)[VEC]) {
        if constexpr (VEC == 8) { const uint4 t = *reinterpret_cast<const uint4*>(p); unpack(t.x, v[0], v[1]); unpack(t.y, v[2], v[3]); unpack(t.z, v[4], v[5]); unpack(t.w, v[6], v[7]); }
        else if constexpr (VEC == 4) { const uint2 t = *reinterpret_cast<const uint2*>(p); unpack(t.x, v[0], v[1]); unpack(t.y, v[2], v[3]); }
        else if constexpr (VEC == 2) { const unsigned t = *reinterpret_cast<const unsigned*>(p); unpack(t, v[0], v[1]); }
        else { v[0] = __uint_as_float((unsigned)(*p) << 16); }
    }
    static __device__ __forceinline__ unsigned pack(float lo, float hi) {
        return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
    }
    static __device__ __forceinline__ void store(unsigned short* p, const float (&v)[VEC]) {
        if constexpr (VEC == 8) { *reinterpret_cast<uint4*>(p) = make_uint4(pack(v[0], v[1]), pack(v[2], v[3]), pack(v[4], v[5]), pack(v[6], v[7])); }
        else if constexpr (VEC == 4) { *reinterpret_cast<uint2*>(p) = make_uint2(pack(v[0], v[1]), pack(v[2], v[3])); }
        else if constexpr (VEC == 2) { *reinterpret_cast<unsigned*>(p) = pack(v[0], v[1]); }
        else { *p = (unsigned short)f32_to_bf16_rne(v[0]); }
    }
    static __device__ __forceinline__ void store1(unsigned short* p, float v) { *p = (unsigned short)f32_to_bf16_rne(v); }
    // exact copy of loaded elements (for staging in LDS): the floats hold bf16 values, truncation is exact
    static __device__ __forceinline__ void store_plain(unsigned short* p, const float (&v)[VEC]) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) p[i] = (unsigned short)(__float_as_uint(v[i]) >> 16);
    }
};

// Wavefronts per SIMD the register allocation must allow.  The gather loop lives on loads in
// flight across wavefronts: the line-wide fp32 shape (8 lanes x 16 bytes) fits 8 per SIMD in 59
// registers without spilling (67 and 7 per SIMD when left alone; measured 1.5-2.5 % faster on
// the low-degree config, 0.6 % on config 3); the other shapes keep the compiler's choice.
template <class IO, int L, int NACC>
constexpr int agg_min_waves() {
    if (sizeof(typename IO::elem) == 4 && IO::kVec == 4 && NACC == 1) {
        if (L == 8) return 8;
    }
    return 1;
}

// ---- the aggregation kernels ----------------------------------------------------------
constexpr int HUB_SLOTS = 1024;       // lines of the LDS hub table (128 KB at 128 bytes per line)

// One wavefront's unit of work (item `wave` of the launch: a row, R short rows, a segment, or a
// quarter of a block-per-row row) in column pass `pass`.  HUB: entries whose column id is negative
// take their row from `table`; MODE_BLOCK_PER_ROW is not available then.
template <class IO, int L, int NACC, bool HUB>
__device__ __forceinline__ void agg_item(const AggArgs& a, const int wave, const int pass,
                                         const typename IO::elem* table, float (*quarter)[L * IO::kVec * NACC]) {
    using T = typename IO::elem;
    constexpr int VEC = IO::kVec;
    constexpr int R = 64 / L;
    constexpr int PASS_W = L * VEC * NACC;
    // gathers kept in flight per lane.  Measured on MI355X: 1, 2 and 4 give the same
    // throughput (the gather rate is set by the L2's miss path, not by latency hiding in
    // the wavefront), so a small count is used to keep the register footprint low; 8 no longer
    // fits the 64 registers of the line-wide shape and halves its speed.
    constexpr int UMAX = NACC == 4 ? 2 : 4;
    constexpr int U = L < UMAX ? L : UMAX;

    const int lane = threadIdx.x & 63;
    int grp = 0;
    while (grp + 1 < a.n_groups && wave >= a.wave_start[grp + 1]) ++grp;
    const int item0 = wave - a.wave_start[grp];
    const int mode = a.mode[grp];
    const int g = lane / L;
    const int l = lane % L;
    const int colbase = pass * PASS_W + l * VEC;

    int nval[NACC];            // elements of vector j that lie inside the slice (0..VEC)
    int coff[NACC];            // column offset read by this lane
    // A lane whose vector lies outside the slice re-reads the first vector of its group's
    // 16*L-byte piece (or of the pass, if the whole piece is outside): an address the
    // active lanes fetch anyway, so it adds no cache line to the gather.
    const int passbase = pass * PASS_W;
#pragma unroll
    for (int j = 0; j < NACC; ++j) {
        const int c = colbase + j * L * VEC;
        const int c0 = passbase + j * L * VEC;
        nval[j] = a.f - c < 0 ? 0 : (a.f - c > VEC ? VEC : a.f - c);
        coff[j] = nval[j] > 0 ? c : (c0 < a.f ? c0 : passbase);
    }
    // a vector that straddles the end of the slice is read whole (the row stride is a
    // multiple of the vector width, so the read stays inside the row) and stored element
    // by element (store_row below)

    const T* __restrict__ X = static_cast<const T*>(a.X);
    const int64_t ldx = a.ldx;
    float acc[NACC][VEC];
#pragma unroll
    for (int j = 0; j < NACC; ++j)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[j][i] = 0.f;
    // epilogue (a.epilogue): an element is kept where its mask element is > 0, else stored as zero;
    // the mask element is the same position of row `row` of M, or the output itself (ReLU)
    auto store_row = [&](T* y, const int row) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) {
            if (a.epilogue && nval[j] > 0) {
                float m[VEC];
                if (a.M) IO::load(static_cast<const T*>(a.M) + (int64_t)row * a.ldm + colbase + j * L * VEC, m);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[j][i] = (a.M ? m[i] : acc[j][i]) > 0.f ? acc[j][i] : 0.f;
            }
            if (nval[j] == VEC) IO::store(y + j * L * VEC, acc[j]);
            else {
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    if (i < nval[j]) IO::store1(y + j * L * VEC + i, acc[j][i]);
            }
        }
    };

    // the feature-row vectors of entry c: from memory, or for a hub entry (HUB, c < 0) from the LDS
    // table; the global load of a hub entry goes to the first hub's row, which stays in the L1
    // Address of a gathered vector: one 32 x 32 -> 64-bit multiply-add per load (vertex id times the
    // row stride in bytes, which the host keeps below 2^32, plus this lane's own base pointer).  A
    // full 64-bit product of id and stride costs five more integer instructions per gathered row,
    // which is what the gather loop's issue slots go to.
    const uint32_t row_bytes = (uint32_t)(ldx * (int64_t)sizeof(T));
    const char* xl[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j) xl[j] = reinterpret_cast<const char*>(X + coff[j]);
    auto row_ptr = [&](const int j, const uint32_t c) {
        return reinterpret_cast<const T*>(xl[j] + (uint64_t)c * row_bytes);
    };
    const uint32_t hub0 = HUB ? (uint32_t)a.hub_cols[0] : 0u;
    auto load_row = [&](const int c, float (&x)[NACC][VEC]) {
        if constexpr (HUB) {
            const bool hub = c < 0;
            const T* xt = table + (hub ? (c & 0x7fffffff) : 0) * (L * VEC) + l * VEC;
            float t[VEC];
            IO::load(row_ptr(0, hub ? hub0 : (uint32_t)c), x[0]);
            IO::load(xt, t);
#pragma unroll
            for (int i = 0; i < VEC; ++i) x[0][i] = hub ? t[i] : x[0][i];
        } else {
#pragma unroll
            for (int j = 0; j < NACC; ++j) IO::load(row_ptr(j, (uint32_t)c), x[j]);
        }
    };
    // acc += sum over u < U of w[u] * X[c[u], columns of this lane]; all loads first
    auto gather_u = [&](const int (&c)[U], const float (&w)[U]) {
        float x[U][NACC][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) load_row(c[u], x[u]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < NACC; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[j][i] = fmaf(w[u], x[u][j][i], acc[j][i]);
    };
    // same with entries that may not exist: their loaded values count as zero
    auto gather_u_if = [&](const bool (&on)[U], const int (&c)[U], const float (&w)[U]) {
        float x[U][NACC][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) load_row(c[u], x[u]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < NACC; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[j][i] = fmaf(on[u] ? w[u] : 0.f, on[u] ? x[u][j][i] : 0.f, acc[j][i]);
    };
    const int32_t* const colidx = HUB ? a.colidx_hub : a.colidx;

    if (mode == MODE_GROUP_PER_ROW) {
        // ---- one group of L lanes per row ------------------------------------------
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
        const int32_t* ci = colidx + (beg - a.e_base);
        const float* vv = a.val + (beg - a.e_base);
        for (int k0 = 0; __ballot(k0 < d) != 0; k0 += L) {
            int c = row;
            float w = 0.f;
            if (k0 + l < d) { c = __builtin_nontemporal_load(ci + k0 + l); w = __builtin_nontemporal_load(vv + k0 + l); }
#pragma unroll
            for (int j0 = 0; j0 < L; j0 += U) {
                if (__ballot(k0 + j0 < d) == 0) break;
                int cj[U];
                float wj[U];
                bool on[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    cj[u] = bperm_i(g * L + j0 + u, c);      // lanes past the row's end hold (row, 0)
                    wj[u] = bperm_f(g * L + j0 + u, w);
                    on[u] = k0 + j0 + u < d;
                }
                gather_u_if(on, cj, wj);
            }
        }
        if (valid) store_row(static_cast<T*>(a.Y) + (int64_t)row * a.ldy + colbase, row);
        return;
    }

    // ---- one wavefront per row or per segment ------------------------------------------
    int row;
    int64_t beg, end;
    float* pout = nullptr;
    if (!HUB && mode == MODE_BLOCK_PER_ROW) {
        // the block's four wavefronts take a quarter of the row each; the group is the first of
        // the launch, so item0 / 4 is the block and item0 % 4 the wavefront inside it
        row = __builtin_amdgcn_readfirstlane(a.split_rows[a.item_off[grp] + (item0 >> 2)].row);
        const int64_t b0 = uniform64(a.rowptr[row - a.row_base]);
        const int64_t d = uniform64(a.rowptr[row - a.row_base + 1]) - b0;
        const int q = item0 & 3;
        beg = b0 + d * q / 4;
        end = b0 + d * (q + 1) / 4;
    } else if (mode == MODE_SEGMENT) {
        const Segment* sp = a.segs + a.item_off[grp] + item0;
        row = __builtin_amdgcn_readfirstlane(sp->row);
        beg = uniform64(sp->e_begin);
        end = beg + __builtin_amdgcn_readfirstlane(sp->len);
        pout = a.partial + (int64_t)__builtin_amdgcn_readfirstlane(sp->slot) * a.fp + colbase;
    } else {
        row = __builtin_amdgcn_readfirstlane(a.rows[a.item_off[grp] + item0]);
        beg = uniform64(a.rowptr[row - a.row_base]);
        end = uniform64(a.rowptr[row - a.row_base + 1]);
    }
    const int32_t* ci = colidx + (beg - a.e_base);
    const float* vv = a.val + (beg - a.e_base);
    const int64_t cnt = end - beg;

    int c = row;
    float w = 0.f;
    if (lane < cnt) { c = __builtin_nontemporal_load(ci + lane); w = __builtin_nontemporal_load(vv + lane); }
    for (int64_t base = 0; base < cnt; base += 64) {
        const int n = (int)(cnt - base < 64 ? cnt - base : 64);
        // fetch the next 64 pairs while this batch is gathered
        int cn = row;
        float wn = 0.f;
        if (base + 64 + lane < cnt) { cn = __builtin_nontemporal_load(ci + base + 64 + lane); wn = __builtin_nontemporal_load(vv + base + 64 + lane); }
        if (n == 64) {
            // group g takes entries g, g + R, ...: L entries per group, U at a time
#pragma unroll
            for (int j0 = 0; j0 < L; j0 += U) {
                int cj[U];
                float wj[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (R == 1) {
                        cj[u] = __builtin_amdgcn_readlane(c, j0 + u);
                        wj[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), j0 + u));
                    } else {
                        cj[u] = bperm_i((j0 + u) * R + g, c);
                        wj[u] = bperm_f((j0 + u) * R + g, w);
                    }
                }
                gather_u(cj, wj);
            }
        } else {
            for (int j0 = 0; j0 * R < n; j0 += U) {
                int cj[U];
                float wj[U];
                bool on[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = (j0 + u) * R + g;       // e < 64 always (j0 + u < L)
                    cj[u] = bperm_i(e & 63, c);            // lanes >= n hold (row, 0)
                    wj[u] = bperm_f(e & 63, w);
                    on[u] = e < n;
                }
                gather_u_if(on, cj, wj);
            }
        }
        c = cn;
        w = wn;
    }

    // butterfly over the R groups
#pragma unroll
    for (int off = L; off < 64; off <<= 1)
#pragma unroll
        for (int j = 0; j < NACC; ++j)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[j][i] += bperm_f(lane ^ off, acc[j][i]);

    if (!HUB && mode == MODE_BLOCK_PER_ROW) {
        // wavefronts 1..3 hand their sums to wavefront 0, which adds them in a fixed order
        const int q = item0 & 3;
        if (q > 0 && g == 0) {
#pragma unroll
            for (int j = 0; j < NACC; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) quarter[q - 1][(j * VEC + i) * L + l] = acc[j][i];
        }
        __syncthreads();
        if (q == 0 && g == 0) {
#pragma unroll
            for (int j = 0; j < NACC; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    const int s = (j * VEC + i) * L + l;
                    acc[j][i] = (acc[j][i] + quarter[0][s]) + (quarter[1][s] + quarter[2][s]);
                }
            store_row(static_cast<T*>(a.Y) + (int64_t)row * a.ldy + colbase, row);
        }
        return;
    }
    if (g == 0) {
        if (mode == MODE_SEGMENT) {     // scratch rows are padded to whole vectors
#pragma unroll
            for (int j = 0; j < NACC; ++j)
                if (nval[j] > 0) store_partial<VEC>(pout + j * L * VEC, acc[j]);
        } else {
            store_row(static_cast<T*>(a.Y) + (int64_t)row * a.ldy + colbase, row);
        }
    }
}

// L lanes per feature row, NACC vectors per lane (columns l*VEC + j*L*VEC), 4 wavefronts
// per block, every wavefront an independent unit of work.  blockIdx.y walks column passes
// when the slice is wider than L*VEC*NACC.
//
// Gathers are issued U at a time with no branch between them, so that U neighbour rows
// are in flight per lane before the first multiply-add waits.  To keep the loads free of
// branches every lane always loads from a valid address: a lane whose columns lie beyond
// the slice reads the first column of its pass, an entry that does not exist reads the row's own vertex, and
// what such a load returns is replaced by zero before it is used.
template <class IO, int L, int NACC>
__global__ void __launch_bounds__(256, (agg_min_waves<IO, L, NACC>())) agg_kernel(const AggArgs a) {
    __shared__ float quarter[3][L * IO::kVec * NACC];     // block-per-row mode: sums of wavefronts 1..3
    const int wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (wave >= a.wave_start[a.n_groups]) return;
    agg_item<IO, L, NACC, false>(a, wave, (int)blockIdx.y, nullptr, quarter);
}

// The same work with the hub rows of the column pass in LDS: one block of 16 wavefronts per
// compute unit; wavefront w of block b takes the items b*16 + w, + 16*gridDim.x, ... (the items are
// sorted heaviest first, so the shares come out even).
template <class IO, int L>
__global__ void __launch_bounds__(1024, 4) agg_hub_kernel(const AggArgs a) {
    using T = typename IO::elem;
    constexpr int VEC = IO::kVec;
    constexpr int LINE = L * VEC;
    __shared__ __align__(16) T table[HUB_SLOTS * LINE];
    {
        const int l = threadIdx.x % L;
        const int c = (int)blockIdx.y * LINE + l * VEC;
        const int coff = c < a.f ? c : (int)blockIdx.y * LINE;     // lanes beyond the slice re-read the pass's first vector
        const T* X = static_cast<const T*>(a.X);
        for (int s = threadIdx.x / L; s < a.n_hub; s += 1024 / L) {
            float v[VEC];
            IO::load(X + (int64_t)a.hub_cols[s] * a.ldx + coff, v);
            IO::store_plain(table + s * LINE + l * VEC, v);
        }
    }
    __syncthreads();
    const int total = a.wave_start[a.n_groups];
    const int w0 = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 16 + (threadIdx.x >> 6)));
    for (int wave = w0; wave < total; wave += 16 * (int)gridDim.x)
        agg_item<IO, L, 1, true>(a, wave, (int)blockIdx.y, table, nullptr);
}

// ---- second pass for split rows: Y[row,:] = sum of its partial-sum slots ---------------
// One block per split row and 64 columns.  Wavefront w adds the slots w, w+4, w+8, ... in ascending
// order (independent loads, four in flight), the four sums are combined through LDS as
// (s0 + s1) + (s2 + s3): a fixed order, so the result is deterministic.
template <class T>
__global__ void __launch_bounds__(256) reduce_kernel(const ReduceArgs a) {
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const ReduceItem it = a.items[blockIdx.x];
    {
        const int col = (int)blockIdx.y * 64 + lane;        // one block per split row and 64 columns
        float s = 0.f;
        if (col < a.f) {
            const float* p = a.partial + (int64_t)it.first_slot * a.fp + col;
            int k = w;
            for (; k + 12 < it.n_slots; k += 16) {
                const float t0 = p[(int64_t)k * a.fp], t1 = p[(int64_t)(k + 4) * a.fp];
                const float t2 = p[(int64_t)(k + 8) * a.fp], t3 = p[(int64_t)(k + 12) * a.fp];
                s += t0; s += t1; s += t2; s += t3;
            }
            for (; k < it.n_slots; k += 4) s += p[(int64_t)k * a.fp];
        }
        part[w][lane] = s;
        __syncthreads();
        if (w == 0 && col < a.f) {
            float r = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
            if (a.epilogue) {        // the aggregation's epilogue for rows summed here
                float m = r;
                if (a.M) {
                    const T mv = static_cast<const T*>(a.M)[(int64_t)it.row * a.ldm + col];
                    if constexpr (sizeof(T) == 4) m = mv;
                    else m = __uint_as_float((unsigned)mv << 16);
                }
                r = m > 0.f ? r : 0.f;
            }
            T* y = static_cast<T*>(a.Y) + (int64_t)it.row * a.ldy + col;
            if constexpr (sizeof(T) == 4) *y = r;
            else *y = (T)f32_to_bf16_rne(r);
        }
    }
}

template <class IO, int L, int NACC>
int launch_one(const AggArgs& a, int n_passes, hipStream_t st) {
    const int total = a.wave_start[a.n_groups];
    if (total <= 0) return NTP_OK;
    dim3 grid((unsigned)((total + 3) / 4), (unsigned)n_passes);
    hipLaunchKernelGGL((agg_kernel<IO, L, NACC>), grid, dim3(256), 0, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("aggregation kernel launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    return NTP_OK;
}

int compute_units() {
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        return n;
    }();
    return cus;
}

template <class IO, int L>
int launch_hub(const AggArgs& a, int n_passes, hipStream_t st) {
    const int total = a.wave_start[a.n_groups];
    if (total <= 0) return NTP_OK;
    const int blocks = std::min(compute_units(), (total + 15) / 16);
    hipLaunchKernelGGL((agg_hub_kernel<IO, L>), dim3((unsigned)blocks, (unsigned)n_passes), dim3(1024), 0, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("aggregation kernel (hub table) launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    return NTP_OK;
}

template <class IO>
int launch_by_shape(const AggArgs& a, int L, int nacc, int n_passes, hipStream_t st) {
    if (nacc == 1) {
        switch (L) {
            case 2: return launch_one<IO, 2, 1>(a, n_passes, st);
            case 4: return launch_one<IO, 4, 1>(a, n_passes, st);
            case 8: return launch_one<IO, 8, 1>(a, n_passes, st);
            case 16: return launch_one<IO, 16, 1>(a, n_passes, st);
            case 32: return launch_one<IO, 32, 1>(a, n_passes, st);
            case 64: return launch_one<IO, 64, 1>(a, n_passes, st);
        }
    } else if (L == 64 && nacc == 2) {
        return launch_one<IO, 64, 2>(a, n_passes, st);
    } else if (L == 64 && nacc == 4) {
        return launch_one<IO, 64, 4>(a, n_passes, st);
    }
    set_error("no aggregation kernel for lanes=%d acc=%d", L, nacc);
    return NTP_EUNSUPPORTED;
}

}  // namespace

// pass_lanes > 0: columns are walked in passes (blockIdx.y) of pass_lanes vectors per
// feature row instead of the widest shape that fits a wavefront.
void agg_shape(int64_t f, int vec, int pass_lanes, int* lanes_per_row, int* n_acc, int* n_passes) {
    const int64_t nv = (f + vec - 1) / vec;    // vectors per row
    int L = 2;
    while (L < 64 && L < nv) L <<= 1;
    int nacc = 1;
    if (pass_lanes > 0 && nv > pass_lanes) { L = pass_lanes; }
    else if (nv > 64) { nacc = nv > 128 ? 4 : 2; }
    *lanes_per_row = L;
    *n_acc = nacc;
    *n_passes = (int)((nv + (int64_t)L * nacc - 1) / ((int64_t)L * nacc));
}

// Column passes of one 128-byte line per feature row (8 lanes x 16 bytes): all wavefronts
// in flight then gather from the same 128-byte column of X, whose footprint (n x 128 B) is
// the smallest that still uses whole cache lines, so more of the repeatedly gathered rows
// stay in the L2 of each XCD.  Measured against one pass over the full width (fp32, widths
// 128..512): 1.6x faster at ~490 entries per row, 1.2x at ~50, 1.07x at ~15.  It needs
// rows that start on line boundaries (otherwise every 128-byte piece straddles two lines:
// measured 1.4-1.7x slower), and each pass re-reads the indices and redoes the per-row
// bookkeeping, which outweighs the gain for bf16 rows (half the gathered bytes) on graphs
// with few entries per row (measured 0.9x at ~15 entries per row).
// NTP_AGG_PASS_LANES (2..64, or 0 for full-width passes) overrides the choice.
int agg_pick_pass_lanes(const void* X, int64_t ldx, int dtype, int vec, double entries_per_row) {
    static const int forced = [] {
        const char* e = getenv("NTP_AGG_PASS_LANES");
        if (!e) return -1;
        const int x = atoi(e);
        if (x <= 0) return 0;
        int p = 2;
        while (p < 64 && p < x) p <<= 1;
        return p;
    }();
    if (forced >= 0) return forced;
    const int es = dtype == NTP_BF16 ? 2 : 4;
    if (vec * es != 16) return 0;
    if (((uintptr_t)X % 128) || ((ldx * es) % 128)) return 0;
    if (dtype == NTP_BF16 && entries_per_row < 24.0) return 0;
    return 8;
}

int agg_pick_vec(const void* X, const void* Y, int64_t f, int64_t ldx, int64_t ldy, int dtype, const void* M, int64_t ldm) {
    const int es = dtype == NTP_BF16 ? 2 : 4;
    int vec = 16 / es;
    const uintptr_t px = (uintptr_t)X, py = (uintptr_t)Y, pm = (uintptr_t)M;
    (void)f;   // the slice width need not be a multiple: a straddling vector is read whole, stored by element
    while (vec > 1 && (ldx % vec || ldy % vec || px % (uintptr_t)(vec * es) || py % (uintptr_t)(vec * es) ||
                       (M && (ldm % vec || pm % (uintptr_t)(vec * es))))) vec >>= 1;
    return vec;
}

int agg_hub_slots() { return HUB_SLOTS; }

// The hub kernel exists for rows walked in 16-byte vectors by 4 or 8 lanes (64- and 128-byte
// lines per pass), on graphs that were built with a hub table (NTP_AGG_HUB=1 at build time).
bool agg_uses_hub(const AggArgs& a, int dtype) {
    if (!a.colidx_hub || a.n_hub <= 0 || !a.hub_cols) return false;
    const int vec = agg_pick_vec(a.X, a.Y, a.f, a.ldx, a.ldy, dtype, a.M, a.ldm);
    if (vec * (dtype == NTP_BF16 ? 2 : 4) != 16) return false;
    int L, nacc, passes;
    agg_shape(a.f, vec, a.pass_lanes, &L, &nacc, &passes);
    return nacc == 1 && (L == 8 || L == 4);
}

int launch_aggregate(const AggArgs& a, int dtype, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    const int vec = agg_pick_vec(a.X, a.Y, a.f, a.ldx, a.ldy, dtype, a.M, a.ldm);
    int L, nacc, passes;
    agg_shape(a.f, vec, a.pass_lanes, &L, &nacc, &passes);
    if (agg_uses_hub(a, dtype)) {
        if (dtype == NTP_F32) return L == 8 ? launch_hub<IoF32<4>, 8>(a, passes, st) : launch_hub<IoF32<4>, 4>(a, passes, st);
        return L == 8 ? launch_hub<IoBf16<8>, 8>(a, passes, st) : launch_hub<IoBf16<8>, 4>(a, passes, st);
    }
    if (dtype == NTP_F32) {
        switch (vec) {
            case 4: return launch_by_shape<IoF32<4>>(a, L, nacc, passes, st);
            case 2: return launch_by_shape<IoF32<2>>(a, L, nacc, passes, st);
            case 1: return launch_by_shape<IoF32<1>>(a, L, nacc, passes, st);
        }
    } else if (dtype == NTP_BF16) {
        switch (vec) {
            case 8: return launch_by_shape<IoBf16<8>>(a, L, nacc, passes, st);
            case 4: return launch_by_shape<IoBf16<4>>(a, L, nacc, passes, st);
            case 2: return launch_by_shape<IoBf16<2>>(a, L, nacc, passes, st);
            case 1: return launch_by_shape<IoBf16<1>>(a, L, nacc, passes, st);
        }
    }
    set_error("unsupported dtype %d", dtype);
    return NTP_EUNSUPPORTED;
}

int launch_reduce(const ReduceArgs& a, int dtype, void* stream) {
    if (a.n_items <= 0) return NTP_OK;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)a.n_items, (unsigned)((a.f + 63) / 64));
    if (dtype == NTP_F32) hipLaunchKernelGGL(reduce_kernel<float>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(reduce_kernel<unsigned short>, grid, dim3(256), 0, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("reduce kernel launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    return NTP_OK;
}

}  // namespace ntp
