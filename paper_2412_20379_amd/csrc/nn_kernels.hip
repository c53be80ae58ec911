// Dense transform of eq. (4) on the matrix cores of gfx950: H = act(A W), and its
// gradients dW = A^T dZ, dA = dZ W^T with dZ = dH * 1[H > 0].
//
// One tiled kernel serves the three products.  A block of 256 threads (4 wavefronts)
// owns a BM x BN tile of the output; the contraction runs in steps of BK = 32 through
// LDS.  Both operands are kept in LDS as [kk][mn] (contraction index major), so a
// wavefront reads the fragments of v_mfma_f32_32x32x2_f32 (lane = 32*kk + mn) as 32
// consecutive floats per half wave, free of bank conflicts.  An operand whose memory
// layout is contraction-contiguous (A in the forward, dH and W in dA) is transposed on its
// way into LDS; the ReLU mask and the bf16 -> fp32 conversion are applied on the same way.
// The next tile is fetched into registers while the current one is multiplied.
// dW contracts over the vertices: the rows are split over blocks, each block writes an
// fp32 partial [K x M] to the caller's workspace and a second kernel adds them in order
// (deterministic, no atomics).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "ntp_internal.h"

namespace ntp {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;
constexpr int NTHREADS = 256;

struct GemmArgs {
    const void* A;       // first operand source
    const void* B;       // second operand source
    const void* maskA;   // same shape/stride as A (nullable): element used only where mask > 0
    const void* maskB;
    void* C;
    int64_t lda, ldb, ldc;
    int64_t Mdim, Ndim, Kdim;     // C is Mdim x Ndim, contraction length Kdim
    int64_t k_per_split;          // contraction range per blockIdx.z (multiple of BK)
    int64_t c_split_stride;       // elements between the outputs of consecutive splits
    int relu;
    // block id -> tile: blocks that read the same rows of the streamed operand ("major":
    // the row tile of C, or the split for dW) differ by 8 in block id, so the hardware's
    // round-robin puts them on the same XCD at about the same time and the second reader
    // finds the rows in that XCD's L2.
    int tiles_m, tiles_n, n_splits;
    int share_splits;             // 1: major = split (dW), 0: major = row tile of C
};

__device__ __forceinline__ float elem_to_f32(float v) { return v; }
__device__ __forceinline__ float elem_to_f32(unsigned short v) { return __uint_as_float((unsigned)v << 16); }

__device__ __forceinline__ unsigned f32_to_bf16_bits(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(unsigned short* p, float v) { *p = (unsigned short)f32_to_bf16_bits(v); }

// four consecutive elements starting at p (aligned for the vector path), as floats
__device__ __forceinline__ void load4(const float* p, float (&v)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load4(const unsigned short* p, float (&v)[4]) {
    const uint2 t = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}

// Fetch this thread's share of a tile into registers.
//   KCONTIG: tile element (mn, kk) at src[(mn0+mn)*ld + k0+kk]  (rows = mn, 4 consecutive kk per vector)
//   else   : tile element (mn, kk) at src[(k0+kk)*ld + mn0+mn]  (rows = kk, 4 consecutive mn per vector)
// Elements outside [0,mn_lim) x [0,k_lim) read as zero.  With a mask, an element is kept
// only where the mask element is > 0.
template <class T, bool KCONTIG, bool MASK, int TILE_MN>
__device__ __forceinline__ void fetch_tile(const T* __restrict__ src, const T* __restrict__ mask, int64_t ld,
                                           int64_t mn0, int64_t k0, int64_t mn_lim, int64_t k_lim, bool vec_ok,
                                           float (&regs)[TILE_MN * BK / 4 / NTHREADS][4]) {
    constexpr int NV = TILE_MN * BK / 4 / NTHREADS;
    constexpr int VPR = KCONTIG ? BK / 4 : TILE_MN / 4;     // vectors per tile row
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int idx = threadIdx.x + NTHREADS * v;
        const int r = idx / VPR, c4 = (idx % VPR) * 4;
        const int64_t row = (KCONTIG ? mn0 : k0) + r;
        const int64_t col = (KCONTIG ? k0 : mn0) + c4;
        const int64_t row_lim = KCONTIG ? mn_lim : k_lim;
        const int64_t col_lim = KCONTIG ? k_lim : mn_lim;
        float x[4] = {0.f, 0.f, 0.f, 0.f};
        if (row < row_lim && col < col_lim) {
            const T* p = src + row * ld + col;
            if (vec_ok && col + 3 < col_lim) {
                load4(p, x);
                if constexpr (MASK) {
                    float m[4];
                    load4(mask + row * ld + col, m);
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = m[e] > 0.f ? x[e] : 0.f;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < col_lim) {
                        float t = elem_to_f32(p[e]);
                        if constexpr (MASK) t = elem_to_f32(mask[row * ld + col + e]) > 0.f ? t : 0.f;
                        x[e] = t;
                    }
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) regs[v][e] = x[e];
    }
}

// Put the registers into LDS as dst[kk][mn] with row stride LD.
template <bool KCONTIG, int TILE_MN, int LD>
__device__ __forceinline__ void stash_tile(float* __restrict__ dst, const float (&regs)[TILE_MN * BK / 4 / NTHREADS][4]) {
    constexpr int NV = TILE_MN * BK / 4 / NTHREADS;
    constexpr int VPR = KCONTIG ? BK / 4 : TILE_MN / 4;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int idx = threadIdx.x + NTHREADS * v;
        const int r = idx / VPR, c4 = (idx % VPR) * 4;
        if constexpr (KCONTIG) {          // r = mn, c4 = kk: transpose
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[(c4 + e) * LD + r] = regs[v][e];
        } else {                          // r = kk, c4 = mn
            *reinterpret_cast<float4*>(dst + r * LD + c4) = make_float4(regs[v][0], regs[v][1], regs[v][2], regs[v][3]);
        }
    }
}

template <bool KCONTIG, int TILE_MN> struct LdsStride {
    // transposed stores: stride = 1 mod 8 keeps the 32 lanes of a half wave on 32 banks;
    // vector stores: stride multiple of 4 (16-byte rows) and not a multiple of 32
    static constexpr int value = KCONTIG ? TILE_MN + 1 : TILE_MN + 4;
};

// C[Mdim x Ndim] (+split) = Aop * Bop, tiles BM x BN, WM x WN wavefronts.
template <class TA, class TB, class TC, bool A_KCONTIG, bool B_KCONTIG, bool MASK_A, bool MASK_B,
          int BM, int BN, int WM, int WN>
__global__ void __launch_bounds__(NTHREADS) gemm_kernel(const GemmArgs g) {
    static_assert(WM * WN == 4, "four wavefronts per block");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int LDA_S = LdsStride<A_KCONTIG, BM>::value;
    constexpr int LDB_S = LdsStride<B_KCONTIG, BN>::value;
    __shared__ __attribute__((aligned(16))) float As[BK * LDA_S];
    __shared__ __attribute__((aligned(16))) float Bs[BK * LDB_S];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave % WN;
    int bx, by, bz;
    {
        const int n_major = g.share_splits ? g.n_splits : g.tiles_m;
        const int n_minor = g.share_splits ? g.tiles_m * g.tiles_n : g.tiles_n;
        const int id = (int)blockIdx.x;
        const int grp = id / (8 * n_minor), r = id % (8 * n_minor);
        const int minor = r / 8, major = grp * 8 + r % 8;
        if (major >= n_major) return;              // padding of the last group of eight
        if (g.share_splits) { bz = major; bx = minor % g.tiles_m; by = minor / g.tiles_m; }
        else { bz = 0; bx = major; by = minor; }
    }
    const int64_t m0 = (int64_t)bx * BM;
    const int64_t n0 = (int64_t)by * BN;
    const int64_t kbeg = (int64_t)bz * g.k_per_split;
    const int64_t kend = kbeg + g.k_per_split < g.Kdim ? kbeg + g.k_per_split : g.Kdim;

    const TA* A = static_cast<const TA*>(g.A);
    const TB* B = static_cast<const TB*>(g.B);
    const TA* mA = static_cast<const TA*>(g.maskA);
    const TB* mB = static_cast<const TB*>(g.maskB);
    const bool a_vec = (g.lda % 4 == 0) && ((uintptr_t)A % (4 * sizeof(TA)) == 0) && (!MASK_A || (uintptr_t)mA % (4 * sizeof(TA)) == 0);
    const bool b_vec = (g.ldb % 4 == 0) && ((uintptr_t)B % (4 * sizeof(TB)) == 0) && (!MASK_B || (uintptr_t)mB % (4 * sizeof(TB)) == 0);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    float ra[BM * BK / 4 / NTHREADS][4];
    float rb[BN * BK / 4 / NTHREADS][4];
    if (kbeg < kend) {
        fetch_tile<TA, A_KCONTIG, MASK_A, BM>(A, mA, g.lda, m0, kbeg, g.Mdim, kend, a_vec, ra);
        fetch_tile<TB, B_KCONTIG, MASK_B, BN>(B, mB, g.ldb, n0, kbeg, g.Ndim, kend, b_vec, rb);
    }
    for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();                       // previous tile fully consumed
        stash_tile<A_KCONTIG, BM, LDA_S>(As, ra);
        stash_tile<B_KCONTIG, BN, LDB_S>(Bs, rb);
        __syncthreads();
        if (k0 + BK < kend) {                  // fetch the next tile while this one is multiplied
            fetch_tile<TA, A_KCONTIG, MASK_A, BM>(A, mA, g.lda, m0, k0 + BK, g.Mdim, kend, a_vec, ra);
            fetch_tile<TB, B_KCONTIG, MASK_B, BN>(B, mB, g.ldb, n0, k0 + BK, g.Ndim, kend, b_vec, rb);
        }
        const float* as = As + (lane >> 5) * LDA_S + wm * (TM * 32) + (lane & 31);
        const float* bs = Bs + (lane >> 5) * LDB_S + wn * (TN * 32) + (lane & 31);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = as[kk * LDA_S + i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = bs[kk * LDB_S + j * 32];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }

    // epilogue: element e of a 32x32 accumulator sits at row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
    TC* C = static_cast<TC*>(g.C) + (int64_t)bz * g.c_split_stride;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = n0 + wn * (TN * 32) + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t row = m0 + wm * (TM * 32) + i * 32 + 8 * (e / 4) + 4 * (lane >> 5) + (e % 4);
                if (row < g.Mdim && col < g.Ndim) {
                    float v = acc[i][j][e];
                    if (g.relu) v = v > 0.f ? v : 0.f;
                    store_elem(C + row * g.ldc + col, v);
                }
            }
        }
}

// out[i] = sum over the splits of part[s * stride + i].  A block owns 64 consecutive
// elements; wavefront w adds the splits w, w+4, ... in ascending order and the four sums
// are combined as (s0 + s1) + (s2 + s3): fixed order, deterministic.
__global__ void __launch_bounds__(256) sum_splits_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                         int64_t count, int64_t stride, int n_splits) {
    __shared__ float tmp[4][64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + lane;
    float s = 0.f;
    if (i < count) {
        const float* p = part + i;
        int k = w;
        for (; k + 12 < n_splits; k += 16) {
            const float t0 = p[(int64_t)k * stride], t1 = p[(int64_t)(k + 4) * stride];
            const float t2 = p[(int64_t)(k + 8) * stride], t3 = p[(int64_t)(k + 12) * stride];
            s += t0; s += t1; s += t2; s += t3;
        }
        for (; k < n_splits; k += 4) s += p[(int64_t)k * stride];
    }
    tmp[w][lane] = s;
    __syncthreads();
    if (w == 0 && i < count) out[i] = (tmp[0][lane] + tmp[1][lane]) + (tmp[2][lane] + tmp[3][lane]);
}

// ---- activation alone (for layers evaluated as act(A_hat (H W)): the activation follows the
// aggregation, so it cannot ride on the transform's epilogue) ----------------------------
// FWD: h = max(h, 0) in place.  BWD: dz = dh where h > 0, else 0.  Rows of f elements, stride ld.
template <class T, bool BWD>
__global__ void __launch_bounds__(256) relu_kernel(const T* __restrict__ dh, T* __restrict__ h_or_dz,
                                                   const T* __restrict__ h, int64_t n, int64_t f, int64_t ld) {
    const int64_t total = n * f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / f, c = i - r * f;
        const int64_t o = r * ld + c;
        if constexpr (BWD) {
            h_or_dz[o] = elem_to_f32(h[o]) > 0.f ? dh[o] : (T)0;
        } else {
            if (!(elem_to_f32(h_or_dz[o]) > 0.f)) h_or_dz[o] = (T)0;      // NaN becomes 0 as well, like max(x, 0)
        }
    }
}

template <class TA, class TB, class TC, bool AK, bool BKC, bool MA, bool MB, int BM, int BN, int WM, int WN>
void launch_tiles(GemmArgs g, int n_splits, hipStream_t st) {
    g.tiles_m = (int)((g.Mdim + BM - 1) / BM);
    g.tiles_n = (int)((g.Ndim + BN - 1) / BN);
    g.n_splits = n_splits;
    g.share_splits = n_splits > 1 ? 1 : 0;
    const int64_t n_major = g.share_splits ? n_splits : g.tiles_m;
    const int64_t n_minor = g.share_splits ? (int64_t)g.tiles_m * g.tiles_n : g.tiles_n;
    const int64_t blocks = (n_major + 7) / 8 * 8 * n_minor;
    hipLaunchKernelGGL((gemm_kernel<TA, TB, TC, AK, BKC, MA, MB, BM, BN, WM, WN>), dim3((unsigned)blocks), dim3(NTHREADS), 0, st, g);
}

template <class TA, class TB, class TC, bool AK, bool BKC, bool MA, bool MB>
int launch_gemm(const GemmArgs& g, int n_splits, hipStream_t st) {
    hipError_t e;
    if (g.Ndim > 64) {
        launch_tiles<TA, TB, TC, AK, BKC, MA, MB, 128, 128, 2, 2>(g, n_splits, st);
    } else if (g.Ndim > 32) {
        launch_tiles<TA, TB, TC, AK, BKC, MA, MB, 256, 64, 4, 1>(g, n_splits, st);
    } else if ((g.Mdim + 255) / 256 * n_splits >= 256) {
        launch_tiles<TA, TB, TC, AK, BKC, MA, MB, 256, 32, 4, 1>(g, n_splits, st);
    } else {     // few rows: smaller tiles so that more compute units get a block
        launch_tiles<TA, TB, TC, AK, BKC, MA, MB, 128, 32, 4, 1>(g, n_splits, st);
    }
    e = hipGetLastError();
    if (e != hipSuccess) { set_error("transform kernel launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    return NTP_OK;
}

// number of row splits for dW = A^T dZ
int dw_splits(int64_t n, int64_t k, int64_t m) {
    const int64_t bm = m > 64 ? 128 : 256;
    const int64_t bn = m > 64 ? 128 : (m > 32 ? 64 : 32);
    const int64_t tiles = ((k + bm - 1) / bm) * ((m + bn - 1) / bn);
    // one round of blocks at three blocks per compute unit (256 CUs): no partial last round
    int64_t s = std::max<int64_t>(1, 768 / tiles);
    const int64_t max_s = std::max<int64_t>(1, n / (BK * 8));
    s = std::max<int64_t>(1, std::min(s, max_s));
    return (int)std::min<int64_t>(s, 1024);
}

template <class T>
int nn_fwd_t(const void* A, const void* W, void* H, int64_t n, int64_t k, int64_t m, int act, hipStream_t st) {
    GemmArgs g{};
    g.A = A; g.B = W; g.C = H;
    g.lda = k; g.ldb = m; g.ldc = m;
    g.Mdim = n; g.Ndim = m; g.Kdim = k;
    g.k_per_split = (k + BK - 1) / BK * BK;
    g.relu = act == NTP_ACT_RELU;
    return launch_gemm<T, T, T, true, false, false, false>(g, 1, st);
}

template <class T>
int nn_bwd_t(const void* A, const void* W, const void* H, const void* dH, void* dA, float* dW,
             int64_t n, int64_t k, int64_t m, int act, void* ws, hipStream_t st) {
    const bool relu = act == NTP_ACT_RELU;
    int rc;
    if (dA && n > 0) {
        // dA[n x k] = dZ[n x m] * W^T : contraction over m; W is read as (kk=m, j=k) = W[j*m + kk]
        GemmArgs g{};
        g.A = dH; g.maskA = H; g.B = W; g.C = dA;
        g.lda = m; g.ldb = m; g.ldc = k;
        g.Mdim = n; g.Ndim = k; g.Kdim = m;
        g.k_per_split = (m + BK - 1) / BK * BK;
        rc = relu ? launch_gemm<T, T, T, true, true, true, false>(g, 1, st)
                  : launch_gemm<T, T, T, true, true, false, false>(g, 1, st);
        if (rc != NTP_OK) return rc;
    }
    // dW[k x m] = A^T[k x n] * dZ[n x m] : contraction over the vertices, split over blocks
    const int S = dw_splits(n, k, m);
    GemmArgs g{};
    g.A = A; g.B = dH; g.maskB = H;
    g.lda = k; g.ldb = m; g.ldc = m;
    g.Mdim = k; g.Ndim = m; g.Kdim = n;
    const int64_t per = (n + S - 1) / S;
    g.k_per_split = std::max<int64_t>(BK, (per + BK - 1) / BK * BK);
    g.c_split_stride = k * m;
    g.C = S > 1 ? ws : (void*)dW;
    rc = relu ? launch_gemm<T, T, float, false, false, false, true>(g, S, st)
              : launch_gemm<T, T, float, false, false, false, false>(g, S, st);
    if (rc != NTP_OK) return rc;
    if (S > 1) {
        const int64_t count = k * m;
        hipLaunchKernelGGL(sum_splits_kernel, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, st,
                           (const float*)ws, dW, count, count, S);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) { set_error("split reduction launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    }
    return NTP_OK;
}

}  // namespace

int64_t nn_bwd_workspace_bytes(int64_t n, int64_t k, int64_t m) {
    const int S = dw_splits(n, k, m);
    return S > 1 ? (int64_t)S * k * m * 4 : 0;
}

int launch_relu(const void* dH, const void* H, void* out, int64_t n, int64_t f, int64_t ld, int dtype,
                bool backward, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    const int64_t total = n * f;
    if (total == 0) return NTP_OK;
    const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 256 * 32);
    if (dtype == NTP_BF16) {
        using T = unsigned short;
        if (backward) hipLaunchKernelGGL((relu_kernel<T, true>), dim3(blocks), dim3(256), 0, st, (const T*)dH, (T*)out, (const T*)H, n, f, ld);
        else hipLaunchKernelGGL((relu_kernel<T, false>), dim3(blocks), dim3(256), 0, st, (const T*)nullptr, (T*)out, (const T*)nullptr, n, f, ld);
    } else {
        using T = float;
        if (backward) hipLaunchKernelGGL((relu_kernel<T, true>), dim3(blocks), dim3(256), 0, st, (const T*)dH, (T*)out, (const T*)H, n, f, ld);
        else hipLaunchKernelGGL((relu_kernel<T, false>), dim3(blocks), dim3(256), 0, st, (const T*)nullptr, (T*)out, (const T*)nullptr, n, f, ld);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("activation kernel launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
    return NTP_OK;
}

int launch_nn_fwd(const void* A, const void* W, void* H, int64_t n, int64_t k, int64_t m,
                  int act, int dtype, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    return dtype == NTP_BF16 ? nn_fwd_t<unsigned short>(A, W, H, n, k, m, act, st)
                             : nn_fwd_t<float>(A, W, H, n, k, m, act, st);
}

int launch_nn_bwd(const void* A, const void* W, const void* H, const void* dH, void* dA, float* dW,
                  int64_t n, int64_t k, int64_t m, int act, int dtype,
                  void* workspace, int64_t, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) {   // nothing to contract over: dW = 0 (a fill kernel, not a memset node)
        const int64_t count = k * m;
        hipLaunchKernelGGL(sum_splits_kernel, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, st,
                           (const float*)nullptr, dW, count, count, 0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) { set_error("fill launch failed: %s", hipGetErrorString(e)); return NTP_EHIP; }
        return NTP_OK;
    }
    return dtype == NTP_BF16 ? nn_bwd_t<unsigned short>(A, W, H, dH, dA, dW, n, k, m, act, workspace, st)
                             : nn_bwd_t<float>(A, W, H, dH, dA, dW, n, k, m, act, workspace, st);
}

}  // namespace ntp
