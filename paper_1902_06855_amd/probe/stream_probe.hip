// Stand-alone probe: what this GPU's memory system sustains for the access mixes
// of the gradient-aggregation kernels, with nothing else in the way.  It shares
// no code with the library; bench.py prints its figures beside the library's so
// that "fraction of the 8 TB/s peak" can be read against what a bare kernel of
// the same shape reaches on the same chip.
//
// Patterns (all through buffer descriptors, 128-bit accesses, streaming cache
// policy, 256 threads x 8 vectors per 8192-element tile, tiles dealt to the
// XCDs in runs of 2^grp):
//   read      sum of a            (4 B read per element)
//   inplace   r += g              (8 B read, 4 B written: the accumulate pass)
//   cast      h = fp16(g)         (4 B read, 2 B written elsewhere: the dense cast)
//   fold8     out = x0 + ... + x7 (eight fp16 streams read at the same offset, one
//                                  written: the ring fold of eight workers)
// Output: one JSON object on stdout.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                              \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            std::fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                                  \
        }                                                                                  \
    } while (0)

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

constexpr int AUX = 19;          // sc0 sc1 nt
constexpr int NT = 256, U = 8;
constexpr long TILE = static_cast<long>(NT) * U * 4;

enum { READ = 0, INPLACE = 1, CAST = 2 };

__device__ inline long xcd_order(long b, long total, int grp)
{
    const long span = 8L << grp;
    if (b >= total / span * span) return b;
    const long x = b % 8, i = b / 8;
    return ((i >> grp) * span) + (x << grp) + (i & ((1L << grp) - 1));
}

template <int PAT, int WPE>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void k_probe(const float *g, float *r, uint16_t *h, float *sink, long n_tiles, int grp)
{
    const long tile = xcd_order(blockIdx.x, n_tiles, grp);
    const __amdgpu_buffer_rsrc_t gd = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(g) + tile * TILE, 0, static_cast<int>(TILE * 4), 0x00020000);
    const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(r + tile * TILE, 0, static_cast<int>(TILE * 4), 0x00020000);
    const __amdgpu_buffer_rsrc_t hd = __builtin_amdgcn_make_buffer_rsrc(h + tile * TILE, 0, static_cast<int>(TILE * 2), 0x00020000);
    const int t = threadIdx.x;
    u4 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        a[u] = __builtin_amdgcn_raw_buffer_load_b128(gd, (t + u * NT) * 16, 0, AUX);
        if (PAT == INPLACE) b[u] = __builtin_amdgcn_raw_buffer_load_b128(rd, (t + u * NT) * 16, 0, AUX);
    }
    f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const f4 x = __builtin_bit_cast(f4, a[u]);
        if (PAT == READ) acc += x;
        if (PAT == INPLACE) {
            const f4 s = x + __builtin_bit_cast(f4, b[u]);
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, s), rd, (t + u * NT) * 16, 0, AUX);
        }
        if (PAT == CAST) {
            const _Float16 h0 = static_cast<_Float16>(x.x), h1 = static_cast<_Float16>(x.y);
            const _Float16 h2 = static_cast<_Float16>(x.z), h3 = static_cast<_Float16>(x.w);
            u2 o;
            o.x = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h0)) | (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h1)) << 16);
            o.y = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h2)) | (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h3)) << 16);
            __builtin_amdgcn_raw_buffer_store_b64(o, hd, (t + u * NT) * 8, 0, AUX);
        }
    }
    if (PAT == READ) {
        const float s = acc.x + acc.y + acc.z + acc.w;
        if (s == 12345.678f) sink[0] = s;          // keeps the loads alive
    }
}

typedef _Float16 h2v __attribute__((ext_vector_type(2)));
__device__ inline uint32_t add_h2(uint32_t a, uint32_t b)
{
    const h2v s = __builtin_bit_cast(h2v, a) + __builtin_bit_cast(h2v, b);
    return __builtin_bit_cast(uint32_t, s);
}

constexpr int FOLD_P = 8, FOLD_NT = 512;

// 512 threads, 16 bytes of every stream per thread: all eight loads in flight, then the fold.
__global__ __launch_bounds__(FOLD_NT) void k_fold(const uint16_t *const *streams, uint16_t *out, long n_blocks, int grp)
{
    const long blk = xcd_order(blockIdx.x, n_blocks, grp);
    const long e0 = blk * FOLD_NT * 8;
    u4 x[FOLD_P];
#pragma unroll
    for (int q = 0; q < FOLD_P; ++q) {
        const __amdgpu_buffer_rsrc_t d = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(streams[q]) + e0, 0, FOLD_NT * 16, 0x00020000);
        x[q] = __builtin_amdgcn_raw_buffer_load_b128(d, threadIdx.x * 16, 0, AUX);
    }
    u4 v = x[0];
#pragma unroll
    for (int q = 1; q < FOLD_P; ++q) {
        v.x = add_h2(v.x, x[q].x); v.y = add_h2(v.y, x[q].y); v.z = add_h2(v.z, x[q].z); v.w = add_h2(v.w, x[q].w);
    }
    const __amdgpu_buffer_rsrc_t od = __builtin_amdgcn_make_buffer_rsrc(out + e0, 0, FOLD_NT * 16, 0x00020000);
    __builtin_amdgcn_raw_buffer_store_b128(v, od, threadIdx.x * 16, 0, 0);
}

__global__ void k_fill_h(uint16_t *x, long n, unsigned seed)
{
    long i = blockIdx.x * static_cast<long>(blockDim.x) + threadIdx.x;
    const long stride = static_cast<long>(gridDim.x) * blockDim.x;
    for (; i < n; i += stride) {
        unsigned v = static_cast<unsigned>(i) * 2654435761u + seed;
        v ^= v >> 15; v *= 2246822519u; v ^= v >> 13;
        x[i] = static_cast<uint16_t>(0x2000u + (v & 0x0fffu));      // small positive halves
    }
}

// pseudo-random finite floats: the memory system is not timed on zeros
__global__ void k_fill(float *x, long n, unsigned seed)
{
    long i = blockIdx.x * static_cast<long>(blockDim.x) + threadIdx.x;
    const long stride = static_cast<long>(gridDim.x) * blockDim.x;
    for (; i < n; i += stride) {
        unsigned v = static_cast<unsigned>(i) * 2654435761u + seed;
        v ^= v >> 15; v *= 2246822519u; v ^= v >> 13;
        x[i] = (static_cast<int>(v & 0xffff) - 32768) * 1e-6f;
    }
}

template <typename F>
static double time_ms(F launch, int reps)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch(); launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) launch();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipGetLastError());
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms / reps;
}

int main(int argc, char **argv)
{
    // elements per array: default 2^29 (2 GiB of fp32), a multiple of the tile
    long n = argc > 1 ? std::atol(argv[1]) : (1L << 29);
    n = n / TILE * TILE;
    if (n < TILE) { std::fprintf(stderr, "stream_probe: at least %ld elements\n", TILE); return 2; }
    const long n_tiles = n / TILE;
    float *g, *r, *sink;
    uint16_t *h;
    CK(hipMalloc(&g, n * 4));
    CK(hipMalloc(&r, n * 4));
    CK(hipMalloc(&h, n * 2));
    CK(hipMalloc(&sink, 256));
    hipLaunchKernelGGL(k_fill, dim3(4096), dim3(256), 0, 0, g, n, 1u);
    hipLaunchKernelGGL(k_fill, dim3(4096), dim3(256), 0, 0, r, n, 2u);
    CK(hipDeviceSynchronize());
    const dim3 grid(static_cast<unsigned>(n_tiles)), block(NT);
    const int reps = 10;
    double best[3] = {0, 0, 0};
    int best_grp[3] = {0, 0, 0}, best_wpe[3] = {0, 0, 0};
    const double bytes[3] = {4.0 * n, 12.0 * n, 6.0 * n};
    for (int grp = 3; grp <= 5; grp += 2) {
        for (int wpe = 1; wpe <= 2; ++wpe) {
            double ms[3];
            if (wpe == 1) {
                ms[READ] = time_ms([&] { hipLaunchKernelGGL((k_probe<READ, 1>), grid, block, 0, 0, g, r, h, sink, n_tiles, grp); }, reps);
                ms[INPLACE] = time_ms([&] { hipLaunchKernelGGL((k_probe<INPLACE, 1>), grid, block, 0, 0, g, r, h, sink, n_tiles, grp); }, reps);
                ms[CAST] = time_ms([&] { hipLaunchKernelGGL((k_probe<CAST, 1>), grid, block, 0, 0, g, r, h, sink, n_tiles, grp); }, reps);
            } else {
                ms[READ] = time_ms([&] { hipLaunchKernelGGL((k_probe<READ, 2>), grid, block, 0, 0, g, r, h, sink, n_tiles, grp); }, reps);
                ms[INPLACE] = time_ms([&] { hipLaunchKernelGGL((k_probe<INPLACE, 2>), grid, block, 0, 0, g, r, h, sink, n_tiles, grp); }, reps);
                ms[CAST] = time_ms([&] { hipLaunchKernelGGL((k_probe<CAST, 2>), grid, block, 0, 0, g, r, h, sink, n_tiles, grp); }, reps);
            }
            for (int p = 0; p < 3; ++p) {
                const double gbs = bytes[p] / ms[p] / 1e6;
                if (gbs > best[p]) { best[p] = gbs; best_grp[p] = grp; best_wpe[p] = wpe; }
            }
        }
    }
    // eight separately allocated fp16 streams of n / 8 elements each, one output
    const long nh = n / 8 / (FOLD_NT * 8 * 64) * (FOLD_NT * 8 * 64);
    const uint16_t *hs[FOLD_P];
    for (int q = 0; q < FOLD_P; ++q) {
        uint16_t *p;
        CK(hipMalloc(&p, nh * 2));
        hipLaunchKernelGGL(k_fill_h, dim3(2048), dim3(256), 0, 0, p, nh, 11u + q);
        hs[q] = p;
    }
    const uint16_t **d_hs;
    uint16_t *fold_out;
    CK(hipMalloc(&d_hs, sizeof(hs)));
    CK(hipMalloc(&fold_out, nh * 2));
    CK(hipMemcpy(d_hs, hs, sizeof(hs), hipMemcpyHostToDevice));
    CK(hipDeviceSynchronize());
    const long fold_blocks = nh / (FOLD_NT * 8);
    double fold_best = 0;
    int fold_grp = 0;
    for (int grp = 0; grp <= 6; grp += 2) {
        const double ms = time_ms([&] { hipLaunchKernelGGL(k_fold, dim3(static_cast<unsigned>(fold_blocks)), dim3(FOLD_NT), 0, 0, d_hs, fold_out, fold_blocks, grp); }, reps);
        const double gbs = 2.0 * nh * (FOLD_P + 1) / ms / 1e6;
        if (gbs > fold_best) { fold_best = gbs; fold_grp = grp; }
    }
    std::printf("{\"elements\": %ld, \"tile\": %ld, \"unit\": \"GB/s\", "
                "\"fold8\": %.1f, \"fold8_shape\": \"8 fp16 streams of %ld elements, runs of %d blocks per XCD\", ",
                n, TILE, fold_best, nh, 1 << fold_grp);
    std::printf("\"read\": %.1f, \"read_shape\": \"runs of %d tiles per XCD, %d waves per SIMD\", "
                "\"inplace\": %.1f, \"inplace_shape\": \"runs of %d tiles per XCD, %d waves per SIMD\", "
                "\"cast\": %.1f, \"cast_shape\": \"runs of %d tiles per XCD, %d waves per SIMD\"}\n",
                best[READ], 1 << best_grp[READ], best_wpe[READ],
                best[INPLACE], 1 << best_grp[INPLACE], best_wpe[INPLACE],
                best[CAST], 1 << best_grp[CAST], best_wpe[CAST]);
    return 0;
}
