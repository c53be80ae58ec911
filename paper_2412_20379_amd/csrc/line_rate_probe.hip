// line_rate_probe - how many 128-byte lines per second an MI355X delivers to its compute units, as a
// function of where the lines live (L2, Infinity Cache, HBM) and of how the addresses are produced.
// A measurement aid for the aggregation kernel (eq. 1/3 of the paper: every stored entry gathers one
// feature row): it gives the rate the memory system sustains for the kernel's access pattern with
// none of the kernel's other work, so the kernel's own line rate can be read against it.
//
// Every group of 8 lanes reads one 128-byte line per load (16 bytes per lane), 8 lines per wavefront
// instruction, 4 loads in flight per lane, 8 wavefronts per SIMD: the shape of the aggregation
// kernel's line-wide fp32 pass.  Variants:
//   seq      consecutive lines
//   hash     pseudo-random lines, ids computed in registers (no index stream, no dependent load)
//   gather   random ids read from memory, 64 per wavefront load, handed to the lane groups through the
//            cross-lane network, a weight per id, multiply-add: the aggregation kernel's inner loop
// Usage: line_rate_probe            (prints one line per buffer size: seq, hash, gather)
//        line_rate_probe --quick    (the gather variant at 128 MB and 1 GB only, one line:
//                                    "quick <G lines/s at 128 MB> <G lines/s at 1 GB>")
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <random>
#include <string>
#include <vector>

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                            \
        }                                                                            \
    } while (0)

namespace {

enum { SEQ = 0, HASH = 1, GATHER = 2 };
constexpr int WAVES = 256 * 8 * 4 * 4;      // four rounds of 8 blocks of 4 wavefronts on each of 256 compute units
constexpr int BATCHES = 32;                 // batches of 64 lines per wavefront: 67 M lines per launch

__device__ __forceinline__ int bperm_i(int src_lane, int v) { return __builtin_amdgcn_ds_bpermute(src_lane << 2, v); }
__device__ __forceinline__ float bperm_f(int src_lane, float v) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}
__device__ __forceinline__ unsigned mix(unsigned h) {     // integer finaliser: a pseudo-random 32-bit value per item
    h ^= h >> 16; h *= 0x85ebca6bu; h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    return h;
}

// x: `line_mask + 1` lines of 8 float4; idx, wts: WAVES * BATCHES * 64 entries, ids <= line_mask
template <int MODE>
__global__ __launch_bounds__(256, 8) void probe(const float4* __restrict__ x, const int* __restrict__ idx,
                                                const float* __restrict__ wts, float* __restrict__ out,
                                                unsigned line_mask) {
    const int lane = threadIdx.x & 63;
    const unsigned wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int g = lane >> 3, r = lane & 7;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    const unsigned e0 = wave * (unsigned)(BATCHES * 64);
    int c = 0;
    float w = 1.f;
    if (MODE == GATHER) { c = __builtin_nontemporal_load(idx + e0 + lane); w = __builtin_nontemporal_load(wts + e0 + lane); }
    for (int b = 0; b < BATCHES; ++b) {
        int cn = 0;
        float wn = 1.f;
        if (MODE == GATHER && b + 1 < BATCHES) {
            cn = __builtin_nontemporal_load(idx + e0 + (b + 1) * 64 + lane);
            wn = __builtin_nontemporal_load(wts + e0 + (b + 1) * 64 + lane);
        }
#pragma unroll
        for (int j0 = 0; j0 < 8; j0 += 4) {
            unsigned cj[4];
            float wj[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned item = e0 + b * 64 + (j0 + u) * 8 + g;
                if (MODE == SEQ) { cj[u] = item & line_mask; wj[u] = 1.f; }
                else if (MODE == HASH) { cj[u] = mix(item) & line_mask; wj[u] = 1.f; }
                else { cj[u] = (unsigned)bperm_i((j0 + u) * 8 + g, c); wj[u] = bperm_f((j0 + u) * 8 + g, w); }
            }
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = x[(size_t)cj[u] * 8 + r];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc.x = fmaf(wj[u], v[u].x, acc.x);
                acc.y = fmaf(wj[u], v[u].y, acc.y);
                acc.z = fmaf(wj[u], v[u].z, acc.z);
                acc.w = fmaf(wj[u], v[u].w, acc.w);
            }
        }
        c = cn;
        w = wn;
    }
    const float s = acc.x + acc.y + acc.z + acc.w;
    if (s == 123.456f) out[wave] = s;       // the buffers hold zeros: never taken, keeps the loads alive
}

int* d_idx;
float* d_w;
float4* d_x;
float* d_out;

template <int MODE>
double run(size_t bytes) {
    const unsigned lines = (unsigned)(bytes / 128);
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    for (int i = 0; i < 2; ++i) probe<MODE><<<WAVES / 4, 256>>>(d_x, d_idx, d_w, d_out, lines - 1);
    CK(hipDeviceSynchronize());
    const int reps = 5;
    CK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) probe<MODE><<<WAVES / 4, 256>>>(d_x, d_idx, d_w, d_out, lines - 1);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return (double)WAVES * BATCHES * 64 / (ms / reps) / 1e6;      // G lines/s
}

}  // namespace

int main(int argc, char** argv) {
    const bool quick = argc > 1 && std::string(argv[1]) == "--quick";
    const size_t n = (size_t)WAVES * BATCHES * 64;
    const size_t sizes[] = {(size_t)1 << 20, (size_t)4 << 20, (size_t)32 << 20, (size_t)128 << 20, (size_t)1 << 30};
    const size_t maxb = (size_t)1 << 30;
    CK(hipMalloc(&d_x, maxb));
    CK(hipMemset(d_x, 0, maxb));
    CK(hipMalloc(&d_idx, n * 4));
    CK(hipMalloc(&d_w, n * 4));
    CK(hipMemset(d_w, 0, n * 4));
    CK(hipMalloc(&d_out, (size_t)WAVES * 4));
    CK(hipMemset(d_out, 0, (size_t)WAVES * 4));
    std::vector<int> h(n);
    if (quick) {
        double rate[2];
        const size_t qs[2] = {(size_t)128 << 20, (size_t)1 << 30};
        for (int q = 0; q < 2; ++q) {
            std::mt19937 rng(1);
            const unsigned lines = (unsigned)(qs[q] / 128);
            for (size_t i = 0; i < n; ++i) h[i] = (int)(rng() % lines);
            CK(hipMemcpy(d_idx, h.data(), n * 4, hipMemcpyHostToDevice));
            rate[q] = run<GATHER>(qs[q]);
        }
        std::printf("quick %.1f %.1f\n", rate[0], rate[1]);
        return 0;
    }
    std::printf("%10s %14s %14s %14s   (G lines/s of 128 bytes; x 0.128 = TB/s)\n", "buffer", "seq", "hash", "gather");
    for (size_t b : sizes) {
        std::mt19937 rng(1);
        const unsigned lines = (unsigned)(b / 128);
        for (size_t i = 0; i < n; ++i) h[i] = (int)(rng() % lines);        // ids < lines: every access inside the buffer
        CK(hipMemcpy(d_idx, h.data(), n * 4, hipMemcpyHostToDevice));
        const double s = run<SEQ>(b), r = run<HASH>(b), k = run<GATHER>(b);
        std::printf("%7.0f MB %14.1f %14.1f %14.1f\n", b / 1048576.0, s, r, k);
        std::fflush(stdout);
    }
    CK(hipFree(d_x));
    CK(hipFree(d_idx));
    CK(hipFree(d_w));
    CK(hipFree(d_out));
    return 0;
}
