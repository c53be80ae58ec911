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
//
// Two multiply cores share that skeleton:
//   * fp32 MFMA (v_mfma_f32_32x32x2_f32), the plain form;
//   * split bf16 MFMA (v_mfma_f32_32x32x16_bf16), the default: every fp32 operand element
//     is cut into three bf16 pieces hi + mid + lo = x (exact: 3 x 8 significant bits, by
//     truncation) on its way into LDS, and a product a*b is formed as the six piece
//     products of weight >= 2^-16 (hi*hi, hi*mid, mid*hi, mid*mid, hi*lo, lo*hi), each exact
//     in the fp32 accumulator's input; the dropped pieces are below 2^-23 |a b|.  Six bf16
//     instructions cost 6 x 32 cycles per 32x32x16 block against 8 x 64 for fp32, and
//     operands that are bf16 in memory need one piece only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

#include "ntp_internal.h"

namespace ntp {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// pieces an element of type T is cut into for the bf16 core
template <class T> struct Pieces { static constexpr int n = 3; };
template <> struct Pieces<unsigned short> { static constexpr int n = 1; };

// x = sum of NP bf16 values, each returned as an fp32 bit pattern whose low half is zero
// (NP = 1: x is a bf16 value already)
template <int NP>
__device__ __forceinline__ void split_bf16(float x, unsigned (&piece)[NP]) {
    if constexpr (NP == 1) {
        piece[0] = __float_as_uint(x);
    } else {
        const unsigned hi = __float_as_uint(x) & 0xffff0000u;
        const float r1 = x - __uint_as_float(hi);                 // exact: at most 16 significant bits left
        const unsigned mid = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(mid);               // exact: at most 8 significant bits left
        piece[0] = hi; piece[1] = mid; piece[2] = __float_as_uint(r2);
    }
}
// bf16 pair in one dword: low half = piece of the even contraction index, high half = odd
__device__ __forceinline__ unsigned pack_pair(unsigned even, unsigned odd) {
    return __builtin_amdgcn_perm(odd, even, 0x07060302u);
}

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

// Four consecutive elements of row `row` starting at column `col` of a row-major source,
// as floats; elements outside [0,row_lim) x [0,col_lim) read as zero.  With a mask, an
// element is kept only where the mask element is > 0.
template <class T, bool MASK>
__device__ __forceinline__ void load_vec4(const T* __restrict__ src, const T* __restrict__ mask, int64_t ld,
                                          int64_t row, int64_t col, int64_t row_lim, int64_t col_lim, bool vec_ok,
                                          float (&out)[4]) {
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
    for (int e = 0; e < 4; ++e) out[e] = x[e];
}

// Fetch this thread's share of a tile into registers.
//   KCONTIG: tile element (mn, kk) at src[(mn0+mn)*ld + k0+kk]  (rows = mn, 4 consecutive kk per vector)
//   else   : tile element (mn, kk) at src[(k0+kk)*ld + mn0+mn]  (rows = kk, 4 consecutive mn per vector)
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
        load_vec4<T, MASK>(src, mask, ld, (KCONTIG ? mn0 : k0) + r, (KCONTIG ? k0 : mn0) + c4,
                           KCONTIG ? mn_lim : k_lim, KCONTIG ? k_lim : mn_lim, vec_ok, regs[v]);
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

// block id -> (row tile, column tile, split); false for the padding blocks of the last group
__device__ __forceinline__ bool block_to_tile(const GemmArgs& g, int& bx, int& by, int& bz) {
    const int n_major = g.share_splits ? g.n_splits : g.tiles_m;
    const int n_minor = g.share_splits ? g.tiles_m * g.tiles_n : g.tiles_n;
    const int id = (int)blockIdx.x;
    const int grp = id / (8 * n_minor), r = id % (8 * n_minor);
    const int minor = r / 8, major = grp * 8 + r % 8;
    if (major >= n_major) return false;
    if (g.share_splits) { bz = major; bx = minor % g.tiles_m; by = minor / g.tiles_m; }
    else { bz = 0; bx = major; by = minor; }
    return true;
}

// epilogue: element e of a 32x32 accumulator sits at row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
// One pointer per 32x32 block walks down the rows; the row test is a 32-bit compare against the
// rows left below the block's first row, and a wavefront whose whole tile lies inside the matrix
// stores without tests.
template <class TC, int TM, int TN>
__device__ __forceinline__ void store_tile(const GemmArgs& g, const f32x16 (&acc)[TM][TN], int bz,
                                           int64_t row0, int64_t col0, int lane) {
    TC* C = static_cast<TC*>(g.C) + (int64_t)bz * g.c_split_stride;
    const bool inside = row0 + TM * 32 <= g.Mdim && col0 + TN * 32 <= g.Ndim;      // uniform over the wavefront
    const int64_t ldc = g.ldc;
    const bool relu = g.relu != 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = col0 + j * 32 + (lane & 31);
            const int64_t rbase = row0 + i * 32 + 4 * (lane >> 5);
            const int64_t left64 = g.Mdim - rbase;
            const int rows_left = inside ? 32 : (col < g.Ndim ? (left64 > 32 ? 32 : (left64 < 0 ? 0 : (int)left64)) : 0);
            TC* p = C + rbase * ldc + col;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = 8 * (e / 4) + (e % 4);          // row offset inside the block, compile time
                float v = acc[i][j][e];
                if (relu) v = v > 0.f ? v : 0.f;
                if (r < rows_left) store_elem(p, v);
                p += (e % 4 == 3) ? 5 * ldc : ldc;             // next row: +1, or +5 to the next group of four
            }
        }
}

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
    if (!block_to_tile(g, bx, by, bz)) return;     // padding of the last group of eight
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

    store_tile<TC, TM, TN>(g, acc, bz, m0 + wm * (TM * 32), n0 + wn * (TN * 32), lane);
}

// ---- the split-bf16 core -----------------------------------------------------------------
// LDS holds, per operand and piece, P[g][mn] = four dwords = the eight bf16 of contraction
// indices 8g .. 8g+7 of tile row/column mn (g = 0..BK/8-1).  A lane of the 32x32x16
// instruction (mn = lane % 32, h = lane / 32) needs exactly such a 16-byte group
// (g = 2c + h in chunk c), so a fragment is one ds_read_b128 and consecutive lanes read
// consecutive 16 bytes.
//
// Operand loaders.  Each thread owns whole items of the tile:
//   contraction-contiguous source (memory rows run along k): an item = 4 consecutive k of
//     one row mn = half a group, written with one 8-byte LDS store per piece;
//   otherwise (memory rows run along mn): an item = 8 contraction rows x 2 adjacent mn =
//     two whole groups, loaded with eight 8-byte reads that are contiguous across the lanes.
// fetch<true> is the interior form: no bounds checks and no branches (rows/columns beyond
// the matrix are clamped to the last valid ones: what they produce lands only in output
// rows/columns that are never stored), so the loads of two tiles can be in flight with
// exact wait counts.  fetch<false> checks every element and reads zero outside.
template <class T, bool KCONTIG, bool MASK, int TILE_MN> struct Loader;

template <class T, bool MASK, int TILE_MN>
struct Loader<T, true, MASK, TILE_MN> {
    static constexpr int NI = TILE_MN * BK / 4 / NTHREADS;     // items per thread (all threads busy)
    static constexpr int REGS = 4;
    using Regs = float[NI][REGS];
    static __device__ __forceinline__ bool can_be_fast(const void* src, const void* mask, int64_t ld, int64_t mn_lim) {
        return mn_lim > 0 && ld % 4 == 0 && (uintptr_t)src % (4 * sizeof(T)) == 0 && (!MASK || (uintptr_t)mask % (4 * sizeof(T)) == 0);
    }
    template <bool FAST>
    static __device__ __forceinline__ void fetch(const T* __restrict__ src, const T* __restrict__ mask, int64_t ld,
                                                 int64_t mn0, int64_t k0, int64_t mn_lim, int64_t k_lim, Regs& regs) {
#pragma unroll
        for (int v = 0; v < NI; ++v) {
            const int idx = threadIdx.x + NTHREADS * v;
            const int r = idx / (BK / 4), c4 = (idx % (BK / 4)) * 4;
            if constexpr (FAST) {
                int64_t row = mn0 + r;
                row = row < mn_lim ? row : mn_lim - 1;
                const int64_t off = row * ld + k0 + c4;
                load4(src + off, regs[v]);
                if constexpr (MASK) {
                    float m[4];
                    load4(mask + off, m);
#pragma unroll
                    for (int e = 0; e < 4; ++e) regs[v][e] = m[e] > 0.f ? regs[v][e] : 0.f;
                }
            } else {
                const bool vec_ok = ld % 4 == 0 && (uintptr_t)src % (4 * sizeof(T)) == 0 && (!MASK || (uintptr_t)mask % (4 * sizeof(T)) == 0);
                load_vec4<T, MASK>(src, mask, ld, mn0 + r, k0 + c4, mn_lim, k_lim, vec_ok, regs[v]);
            }
        }
    }
    template <int NP, int LD>
    static __device__ __forceinline__ void stash(uint4 (*dst)[BK / 8][LD], const Regs& regs) {
#pragma unroll
        for (int v = 0; v < NI; ++v) {
            const int idx = threadIdx.x + NTHREADS * v;
            const int r = idx / (BK / 4), q = idx % (BK / 4);       // q-th group of four k: half of group q/2
            unsigned x[4][NP];
#pragma unroll
            for (int e = 0; e < 4; ++e) split_bf16<NP>(regs[v][e], x[e]);
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                unsigned* g4 = reinterpret_cast<unsigned*>(&dst[p][q / 2][r]);
                *reinterpret_cast<uint2*>(g4 + 2 * (q % 2)) = make_uint2(pack_pair(x[0][p], x[1][p]), pack_pair(x[2][p], x[3][p]));
            }
        }
    }
};

template <class T, bool MASK, int TILE_MN>
struct Loader<T, false, MASK, TILE_MN> {
    static constexpr int ITEMS = (BK / 8) * (TILE_MN / 2);
    static constexpr int NI = (ITEMS + NTHREADS - 1) / NTHREADS;
    static constexpr bool ALL = ITEMS % NTHREADS == 0;
    static constexpr int REGS = 16;                               // [8 contraction rows][2 mn]
    using Regs = float[NI][REGS];
    static __device__ __forceinline__ bool can_be_fast(const void* src, const void* mask, int64_t ld, int64_t mn_lim) {
        return mn_lim >= 2 && mn_lim % 2 == 0 && ld % 2 == 0 && (uintptr_t)src % (2 * sizeof(T)) == 0 &&
               (!MASK || (uintptr_t)mask % (2 * sizeof(T)) == 0);
    }
    static __device__ __forceinline__ void load2(const float* p, float& a, float& b) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        a = t.x; b = t.y;
    }
    static __device__ __forceinline__ void load2(const unsigned short* p, float& a, float& b) {
        const unsigned t = *reinterpret_cast<const unsigned*>(p);
        a = __uint_as_float(t << 16); b = __uint_as_float(t & 0xffff0000u);
    }
    template <bool FAST>
    static __device__ __forceinline__ void fetch(const T* __restrict__ src, const T* __restrict__ mask, int64_t ld,
                                                 int64_t mn0, int64_t k0, int64_t mn_lim, int64_t k_lim, Regs& regs) {
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int idx = threadIdx.x + NTHREADS * u;
            const int g = idx / (TILE_MN / 2), m2 = (idx % (TILE_MN / 2)) * 2;
            if (ALL || idx < ITEMS) {
                if constexpr (FAST) {
                    int64_t col = mn0 + m2;
                    col = col < mn_lim ? col : mn_lim - 2;
                    const T* p = src + (k0 + 8 * g) * ld + col;
                    const T* pm = MASK ? mask + (k0 + 8 * g) * ld + col : nullptr;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        load2(p + j * ld, regs[u][2 * j], regs[u][2 * j + 1]);
                        if constexpr (MASK) {
                            float ma, mb;
                            load2(pm + j * ld, ma, mb);
                            regs[u][2 * j] = ma > 0.f ? regs[u][2 * j] : 0.f;
                            regs[u][2 * j + 1] = mb > 0.f ? regs[u][2 * j + 1] : 0.f;
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            const int64_t row = k0 + 8 * g + j, col = mn0 + m2 + e;
                            float t = 0.f;
                            if (row < k_lim && col < mn_lim) {
                                t = elem_to_f32(src[row * ld + col]);
                                if constexpr (MASK) t = elem_to_f32(mask[row * ld + col]) > 0.f ? t : 0.f;
                            }
                            regs[u][2 * j + e] = t;
                        }
                }
            }
        }
    }
    template <int NP, int LD>
    static __device__ __forceinline__ void stash(uint4 (*dst)[BK / 8][LD], const Regs& regs) {
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int idx = threadIdx.x + NTHREADS * u;
            const int g = idx / (TILE_MN / 2), m2 = (idx % (TILE_MN / 2)) * 2;
            if (ALL || idx < ITEMS) {
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    unsigned x[8][NP];
#pragma unroll
                    for (int j = 0; j < 8; ++j) split_bf16<NP>(regs[u][2 * j + e], x[j]);
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        dst[p][g][m2 + e] = make_uint4(pack_pair(x[0][p], x[1][p]), pack_pair(x[2][p], x[3][p]),
                                                       pack_pair(x[4][p], x[5][p]), pack_pair(x[6][p], x[7][p]));
                }
            }
        }
    }
};

// Scheduling hint for one pipelined step: after the first fragment reads, every matrix
// instruction is followed by a few vector instructions of the stash (and now and then an LDS
// write or a fragment read of the next chunk), so that the matrix pipe runs while the vector
// pipe cuts the next tile into pieces.
template <int N, int VALU_PER_MFMA, int DS_READS_FIRST>
__device__ __forceinline__ void interleave_hint() {
    if constexpr (N > 0) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);               // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);   // vector ALU
        if constexpr (N % 2 == 0) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // an LDS write
        if constexpr (N % 2 == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // an LDS read
        interleave_hint<N - 1, VALU_PER_MFMA, DS_READS_FIRST>();
    }
}

// LDS bytes of the split kernel: two buffers of (pieces x BK/8 groups x padded tile) 16-byte groups
template <class TA, class TB, int BM, int BN>
constexpr int split_lds_bytes() {
    return 2 * (BK / 8) * 16 * (Pieces<TA>::n * (BM + 4) + Pieces<TB>::n * (BN + 4));
}

// Two schedules of the same step (fetch a tile to registers, cut it into pieces and write it
// to LDS, multiply it):
//   OCC >= 2 (the default for fp32 operands): one LDS buffer (50-63 KB), OCC blocks per compute
//     unit.  A block stores tile s, multiplies it while tile s+1 is on its way from memory, and
//     meets a barrier on either side of the store; what overlaps the cutting, the LDS traffic
//     and the waiting of one block is the other block on the same compute unit.  Measured
//     against the schedule below (169,343 rows): forward 128->256 0.132 -> 0.103 ms, 256->256
//     0.202 -> 0.183 ms, dA 0.242 -> 0.190 ms, dW (with twice the row splits) 0.228 -> 0.208 ms.
//   OCC == 1: two LDS buffers (100-126 KB for fp32 operands), one block per compute unit.  In
//     step s a wavefront multiplies the tile in buffer s%2 while it cuts tile s+1 (already in
//     registers) into pieces and writes it to the other buffer, and tile s+2 is on its way from
//     memory: the three tiles overlap inside every wavefront, with one barrier per step.  Kept
//     for bf16 operands with narrow outputs, where it measured faster (dW 256x40: 0.047 against
//     0.074 ms).
template <class TA, class TB, class TC, bool A_KCONTIG, bool B_KCONTIG, bool MASK_A, bool MASK_B,
          int BM, int BN, int WM, int WN, int OCC = 1>
__global__ void __launch_bounds__(NTHREADS, OCC) gemm_split_kernel(const GemmArgs g) {
    constexpr bool ONEBUF = OCC > 1;      // one LDS buffer, OCC blocks per compute unit
    static_assert(WM * WN == 4, "four wavefronts per block");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int NPA = Pieces<TA>::n, NPB = Pieces<TB>::n;
    // row stride in 16-byte groups: 4 mod 16 spreads the 8-byte stores of a contraction-
    // contiguous source (4 rows x 4 groups x 2 halves per 32 lanes) over all banks
    constexpr int LDA_S = BM + 4, LDB_S = BN + 4;
    extern __shared__ uint4 smem[];
    typedef uint4 (*TileA)[BK / 8][LDA_S];
    typedef uint4 (*TileB)[BK / 8][LDB_S];
    // two buffers: [A0 | A1 | B0 | B1]; one buffer: [A0 | B0]
    const TileA As0 = reinterpret_cast<TileA>(smem), As1 = As0 + NPA;
    const TileB Bs0 = reinterpret_cast<TileB>(ONEBUF ? As1 : As1 + NPA), Bs1 = Bs0 + NPB;
    using LA = Loader<TA, A_KCONTIG, MASK_A, BM>;
    using LB = Loader<TB, B_KCONTIG, MASK_B, BN>;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave % WN;
    int bx, by, bz;
    if (!block_to_tile(g, bx, by, bz)) return;     // padding of the last group of eight
    const int64_t m0 = (int64_t)bx * BM;
    const int64_t n0 = (int64_t)by * BN;
    const int64_t kbeg = (int64_t)bz * g.k_per_split;
    const int64_t kend = kbeg + g.k_per_split < g.Kdim ? kbeg + g.k_per_split : g.Kdim;

    const TA* A = static_cast<const TA*>(g.A);
    const TB* B = static_cast<const TB*>(g.B);
    const TA* mA = static_cast<const TA*>(g.maskA);
    const TB* mB = static_cast<const TB*>(g.maskB);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int mn_a = wm * (TM * 32) + (lane & 31);
    const int mn_b = wn * (TN * 32) + (lane & 31);
    const int h = lane >> 5;
    // multiply the tile held in (as, bs) into the accumulators
    auto multiply = [&](TileA as, TileB bs) {
#pragma unroll
        for (int c = 0; c < BK / 16; ++c) {
            uint4 a[TM][NPA], b[TN][NPB];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int p = 0; p < NPA; ++p) a[i][p] = as[p][2 * c + h][mn_a + i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int p = 0; p < NPB; ++p) b[j][p] = bs[p][2 * c + h][mn_b + j * 32];
            // piece products of weight 2^-8w, small ones first; consecutive instructions go to
            // different accumulators so that none waits for its predecessor
#pragma unroll
            for (int w = 2; w >= 0; --w)
#pragma unroll
                for (int pa = 0; pa <= w; ++pa)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const int pb = w - pa;
                            if (pa < NPA && pb < NPB)
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                    __builtin_bit_cast(bf16x8, a[i][pa < NPA ? pa : 0]), __builtin_bit_cast(bf16x8, b[j][pb < NPB ? pb : 0]), acc[i][j], 0, 0, 0);
                        }
        }
    };
    auto stash = [&](TileA as, TileB bs, const typename LA::Regs& ra, const typename LB::Regs& rb) {
        LA::template stash<NPA, LDA_S>(as, ra);
        LB::template stash<NPB, LDB_S>(bs, rb);
    };

    int64_t k0 = kbeg;
    const bool fast = LA::can_be_fast(A, mA, g.lda, g.Mdim) && LB::can_be_fast(B, mB, g.ldb, g.Ndim);
    if (!ONEBUF && fast && kend - kbeg >= 2 * BK) {
        // An even number of whole steps.  Every fetch is issued unconditionally (past the end
        // it re-reads a tile already taken, and what is stashed from it is never multiplied)
        // so that the number of loads in flight is known at compile time and a stash waits
        // only for its own tile; the scheduling fences keep the loads in program order, which
        // the wait counts rely on.
        const int64_t npipe = (kend - kbeg) / BK / 2 * 2;
        constexpr int N_PROD = NPA == 3 && NPB == 3 ? 6 : (NPA == 1 && NPB == 1 ? 1 : 3);
        constexpr int N_MFMA = (BK / 16) * TM * TN * N_PROD;           // matrix instructions per step
        constexpr int FIRST_READS = TM * NPA + TN * NPB;               // fragment reads of the first chunk
        constexpr int VALU_PER_MFMA = (LA::NI * LA::REGS * (4 * NPA - 2) + LB::NI * LB::REGS * (4 * NPB - 2)) / N_MFMA + 1;
        typename LA::Regs ra0, ra1;
        typename LB::Regs rb0, rb1;
        auto fetch = [&](int64_t s, typename LA::Regs& ra, typename LB::Regs& rb) {
            LA::template fetch<true>(A, mA, g.lda, m0, kbeg + s * BK, g.Mdim, kend, ra);
            LB::template fetch<true>(B, mB, g.ldb, n0, kbeg + s * BK, g.Ndim, kend, rb);
        };
        fetch(0, ra0, rb0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(1, ra1, rb1);
        __builtin_amdgcn_sched_barrier(0);
        stash(As0, Bs0, ra0, rb0);
        __syncthreads();
        for (int64_t s = 0; s < npipe; s += 2) {
            fetch(s + 2 < npipe ? s + 2 : s, ra0, rb0);
            __builtin_amdgcn_sched_barrier(0);
            multiply(As0, Bs0);                 // tile s
            stash(As1, Bs1, ra1, rb1);          // tile s+1
            __builtin_amdgcn_sched_group_barrier(0x100, FIRST_READS, 0);
            interleave_hint<N_MFMA, VALU_PER_MFMA, FIRST_READS>();
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            fetch(s + 3 < npipe ? s + 3 : s + 1, ra1, rb1);
            __builtin_amdgcn_sched_barrier(0);
            multiply(As1, Bs1);                 // tile s+1
            stash(As0, Bs0, ra0, rb0);          // tile s+2 (not used after the last step)
            __builtin_amdgcn_sched_group_barrier(0x100, FIRST_READS, 0);
            interleave_hint<N_MFMA, VALU_PER_MFMA, FIRST_READS>();
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        }
        k0 = kbeg + npipe * BK;
    }
    // what is left (an odd whole step, a partial last step, or everything when the operands
    // are not aligned for the interior form): checked loads, one buffer, next tile fetched
    // while this one is multiplied
    if (k0 < kend) {
        typename LA::Regs ra;
        typename LB::Regs rb;
        auto fetch1 = [&](int64_t k) {
            if (ONEBUF && fast && k + BK <= kend) {
                LA::template fetch<true>(A, mA, g.lda, m0, k, g.Mdim, kend, ra);
                LB::template fetch<true>(B, mB, g.ldb, n0, k, g.Ndim, kend, rb);
            } else {
                LA::template fetch<false>(A, mA, g.lda, m0, k, g.Mdim, kend, ra);
                LB::template fetch<false>(B, mB, g.ldb, n0, k, g.Ndim, kend, rb);
            }
        };
        fetch1(k0);
        for (; k0 < kend; k0 += BK) {
            __syncthreads();
            stash(As0, Bs0, ra, rb);
            __syncthreads();
            if (k0 + BK < kend) fetch1(k0 + BK);
            multiply(As0, Bs0);
        }
    }

    store_tile<TC, TM, TN>(g, acc, bz, m0 + wm * (TM * 32), n0 + wn * (TN * 32), lane);
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
        for (; k + 28 < n_splits; k += 32) {       // eight loads in flight, added in ascending order
            float t[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = p[(int64_t)(k + 4 * j) * stride];
#pragma unroll
            for (int j = 0; j < 8; ++j) s += t[j];
        }
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

// NTP_NN_CORE=fp32 selects the plain fp32 MFMA core (for comparison); default is the split-bf16 core
bool use_split_core() {
    static const bool v = [] {
        const char* e = getenv("NTP_NN_CORE");
        return !(e && e[0] == 'f');
    }();
    return v;
}

// NTP_NN_SCHEDULE=1 / 2 forces the two-buffer / one-buffer schedule of the split core (for comparison)
int split_schedule() {
    static const int v = [] {
        const char* e = getenv("NTP_NN_SCHEDULE");
        return e ? atoi(e) : 0;
    }();
    return v;
}

// launch a split-core kernel with LDS bytes of dynamic LDS (more than the 64 KB a kernel may use
// without asking, so the limit is raised once per kernel and device)
template <auto kernel, int LDS>
void launch_split(int64_t blocks, hipStream_t st, const GemmArgs& g) {
    static bool allowed[64] = {};              // one table per kernel instantiation
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev >= 0 && dev < 64 && !allowed[dev])
        allowed[dev] = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, LDS) == hipSuccess;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(NTHREADS), LDS, st, g);
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
    // The split core pays off from two contraction steps per block on and for output tiles of at
    // least 64 columns; shorter contractions and narrower outputs (memory bound) stay on the plain
    // core.  bf16 operands need one piece product only and always take the bf16 instructions.
    const int64_t k_len = std::min<int64_t>(g.k_per_split, g.Kdim);
    const bool split_pays = sizeof(TA) == 2 || (k_len >= 2 * BK && BN >= 64);
    // fp32 operands: one LDS buffer and two blocks per compute unit; bf16 operands (one piece,
    // small tiles in LDS either way): the same for wide outputs, the two-buffer schedule otherwise
    const bool one_buffer = split_schedule() == 0 ? (sizeof(TA) == 4 || BN >= 128) : split_schedule() == 2;
    if (use_split_core() && split_pays && one_buffer) {
        constexpr int lds = split_lds_bytes<TA, TB, BM, BN>() / 2;
        launch_split<gemm_split_kernel<TA, TB, TC, AK, BKC, MA, MB, BM, BN, WM, WN, 2>, lds>(blocks, st, g);
    } else if (use_split_core() && split_pays) {
        constexpr int lds = split_lds_bytes<TA, TB, BM, BN>();
        launch_split<gemm_split_kernel<TA, TB, TC, AK, BKC, MA, MB, BM, BN, WM, WN, 1>, lds>(blocks, st, g);
    } else
        hipLaunchKernelGGL((gemm_kernel<TA, TB, TC, AK, BKC, MA, MB, BM, BN, WM, WN>), dim3((unsigned)blocks), dim3(NTHREADS), 0, st, g);
}

template <class TA, class TB, class TC, bool AK, bool BKC, bool MA, bool MB>
int launch_gemm(const GemmArgs& g, int n_splits, hipStream_t st) {
    hipError_t e;
    if (g.Ndim > 64) {
        launch_tiles<TA, TB, TC, AK, BKC, MA, MB, 128, 128, 2, 2>(g, n_splits, st);
    } else if (g.Ndim > 32) {
        // two blocks per compute unit run at a time (512 on 256 CUs): take the tile height whose
        // last round of blocks is fuller (169,343 rows: 662 blocks of 256 rows fill 65 % of two
        // rounds, 1,323 blocks of 128 rows 86 % of three)
        auto fill = [&](int64_t bm) {
            const int64_t b = (g.Mdim + bm - 1) / bm * n_splits;
            return (double)b / (double)((b + 511) / 512 * 512);
        };
        if (fill(128) > fill(256) + 0.1) launch_tiles<TA, TB, TC, AK, BKC, MA, MB, 128, 64, 4, 1>(g, n_splits, st);
        else launch_tiles<TA, TB, TC, AK, BKC, MA, MB, 256, 64, 4, 1>(g, n_splits, st);
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
    // one round of blocks with two blocks per compute unit (256 CUs), each block with at least
    // eight contraction steps
    const int64_t target = 512;
    int64_t s = std::max<int64_t>(1, target / tiles);
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
    if (!dW) return NTP_OK;
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
        if (!dW) return NTP_OK;
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
