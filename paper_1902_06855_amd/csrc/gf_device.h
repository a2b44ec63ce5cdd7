// Device-side helpers for the gfx950 kernels: wire-type conversion, 128-bit
// accesses, deterministic wave/workgroup reductions and scans.
#ifndef GF_DEVICE_H
#define GF_DEVICE_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "gf_internal.h"

// ---- global address space ---------------------------------------------------
// Data pointers reach the kernels through pointer tables, so the compiler sees
// generic (flat) addresses.  Everything they point to is device global memory;
// saying so selects global_load / global_store instead of flat accesses.
#define GF_GLOBAL __attribute__((address_space(1)))

template <typename T>
__device__ __forceinline__ GF_GLOBAL T *gf_global(T *p)
{
    return (GF_GLOBAL T *)p;
}

// Plain clang vector types (HIP's float4 / uint4 classes cannot live behind an
// address-space qualified pointer).
typedef float gf_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t gf_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t gf_u32x4 __attribute__((ext_vector_type(4)));

// Streaming accesses: data that is touched once per iteration bypasses the
// caches (nontemporal), which on this part is worth several percent of HBM
// bandwidth for mixed read/write streams.
template <typename T>
__device__ __forceinline__ T gf_ld_stream(const GF_GLOBAL T *p)
{
    return __builtin_nontemporal_load(p);
}
template <typename T>
__device__ __forceinline__ void gf_st_stream(T v, GF_GLOBAL T *p)
{
    __builtin_nontemporal_store(v, p);
}

// Buffer (resource-descriptor) accesses for the streaming kernels.  On this
// part a stream of buffer_load/store_dwordx4 with the cache policy "sc0 sc1 nt"
// sustains about 10 % more HBM bandwidth than the same stream through
// global_load/store ... nt (measured: in-place a += b at 6.5 vs 5.9 TB/s).  The
// descriptor also bounds every access to the run it was made for: loads beyond
// it return zero and stores are dropped.
constexpr int GF_AUX_STREAM = 19;   // sc0 | nt | sc1: touched once, keep it out of the caches
constexpr int GF_AUX_CACHED = 0;    // default policy: data that is read again soon

__device__ __forceinline__ __amdgpu_buffer_rsrc_t gf_make_buf(const GF_GLOBAL void *base, uint32_t bytes)
{
    // Base and size are the same in every lane of a workgroup; saying so keeps the descriptor
    // in scalar registers (otherwise each access is wrapped in a per-lane uniformity loop).
    const uint64_t a = reinterpret_cast<uint64_t>(base);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
    const uint64_t u = (static_cast<uint64_t>(hi) << 32) | lo;
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(u), 0,
                                             static_cast<int>(__builtin_amdgcn_readfirstlane(bytes)), 0x00020000);
}
template <int AUX>
__device__ __forceinline__ gf_f32x4 gf_buf_ld128(__amdgpu_buffer_rsrc_t r, int byte_off)
{
    return __builtin_bit_cast(gf_f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, AUX));
}
template <int AUX>
__device__ __forceinline__ gf_u32x4 gf_buf_ld128u(__amdgpu_buffer_rsrc_t r, int byte_off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, AUX);
}
template <int AUX>
__device__ __forceinline__ gf_u32x2 gf_buf_ld64u(__amdgpu_buffer_rsrc_t r, int byte_off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, AUX);
}
template <int AUX>
__device__ __forceinline__ void gf_buf_st(gf_f32x4 v, __amdgpu_buffer_rsrc_t r, int byte_off)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(gf_u32x4, v), r, byte_off, 0, AUX);
}
template <int AUX>
__device__ __forceinline__ void gf_buf_st(gf_u32x4 v, __amdgpu_buffer_rsrc_t r, int byte_off)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, AUX);
}
template <int AUX>
__device__ __forceinline__ void gf_buf_st(gf_u32x2 v, __amdgpu_buffer_rsrc_t r, int byte_off)
{
    __builtin_amdgcn_raw_buffer_store_b64(v, r, byte_off, 0, AUX);
}

// ---- fp16 wire values travel as raw 16-bit patterns -------------------------
// The conversions below compile to the hardware's cvt instructions, which round
// to nearest even and keep subnormals under the default float mode of HIP
// kernels (no flush-to-zero is requested anywhere in this library).

// Plain conversion.  The compiler may merge it with the arithmetic that made x
// (for the sum of two halves that is the exact native half add).
__device__ __forceinline__ uint16_t gf_f32_to_h_mergeable(float x)
{
    const _Float16 h = static_cast<_Float16>(x);
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ uint16_t gf_f32_to_h(float x)
{
    // The empty asm keeps the conversion an instruction of its own.  Folded into
    // a preceding fp32 multiply (the mixed-precision fma) the exact product
    // would be rounded once, straight to fp16; the value that travels is the
    // fp32 product, rounded, then converted (two roundings, like any fp32 value).
    asm("" : "+v"(x));
    const _Float16 h = static_cast<_Float16>(x);
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float gf_h_to_f32(uint16_t b)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, b));
}

// One ring hop on a pair of halves packed in a 32-bit word: fp32 sum rounded
// back to half (Section 2.5: the message is fp16, so every partial sum is).
// 24 >= 2*11 + 2 significand bits make the two roundings equal to one, so the
// native half add the compiler may pick instead gives the same bits.
__device__ __forceinline__ uint32_t gf_hop_add_h2(uint32_t a, uint32_t b)
{
    const float s0 = gf_h_to_f32(static_cast<uint16_t>(a)) + gf_h_to_f32(static_cast<uint16_t>(b));
    const float s1 = gf_h_to_f32(static_cast<uint16_t>(a >> 16)) + gf_h_to_f32(static_cast<uint16_t>(b >> 16));
    return static_cast<uint32_t>(gf_f32_to_h_mergeable(s0)) |
           (static_cast<uint32_t>(gf_f32_to_h_mergeable(s1)) << 16);
}

__device__ __forceinline__ uint16_t gf_hop_add(uint16_t a, uint16_t b)
{
    return gf_f32_to_h_mergeable(gf_h_to_f32(a) + gf_h_to_f32(b));
}

__device__ __forceinline__ float gf_hop_add(float a, float b) { return a + b; }

// Wire element from an fp32 value.
template <typename W> __device__ __forceinline__ W gf_to_wire(float x);
template <> __device__ __forceinline__ uint16_t gf_to_wire<uint16_t>(float x) { return gf_f32_to_h(x); }
template <> __device__ __forceinline__ float gf_to_wire<float>(float x) { return x; }

template <typename W> __device__ __forceinline__ float gf_from_wire(W x);
template <> __device__ __forceinline__ float gf_from_wire<uint16_t>(uint16_t x) { return gf_h_to_f32(x); }
template <> __device__ __forceinline__ float gf_from_wire<float>(float x) { return x; }

// Four wire elements as one naturally aligned vector.
template <typename W> struct gf_wire4;
template <> struct gf_wire4<uint16_t> { using type = gf_u32x2; };
template <> struct gf_wire4<float> { using type = gf_f32x4; };

__device__ __forceinline__ gf_u32x2 gf_pack4(uint16_t a, uint16_t b, uint16_t c, uint16_t d)
{
    gf_u32x2 r;
    r.x = static_cast<uint32_t>(a) | (static_cast<uint32_t>(b) << 16);
    r.y = static_cast<uint32_t>(c) | (static_cast<uint32_t>(d) << 16);
    return r;
}
__device__ __forceinline__ gf_f32x4 gf_pack4(float a, float b, float c, float d)
{
    gf_f32x4 r = {a, b, c, d};
    return r;
}

__device__ __forceinline__ void gf_unpack4(gf_u32x2 v, float &a, float &b, float &c, float &d)
{
    a = gf_h_to_f32(static_cast<uint16_t>(v.x)); b = gf_h_to_f32(static_cast<uint16_t>(v.x >> 16));
    c = gf_h_to_f32(static_cast<uint16_t>(v.y)); d = gf_h_to_f32(static_cast<uint16_t>(v.y >> 16));
}
__device__ __forceinline__ void gf_unpack4(gf_f32x4 v, float &a, float &b, float &c, float &d)
{
    a = v.x; b = v.y; c = v.z; d = v.w;
}

__device__ __forceinline__ bool gf_aligned(const void *p, unsigned bytes)
{
    return (reinterpret_cast<uintptr_t>(p) & (bytes - 1u)) == 0;
}
__device__ __forceinline__ bool gf_aligned(const GF_GLOBAL void *p, unsigned bytes)
{
    return (reinterpret_cast<uintptr_t>(p) & (bytes - 1u)) == 0;
}

// ---- reductions -------------------------------------------------------------
// Fixed trees: the result depends only on the values, never on scheduling.

__device__ __forceinline__ double gf_wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;   // complete in lane 0
}

// Sum over a workgroup of NT threads (NT a multiple of 64); valid in thread 0.
template <int NT>
__device__ __forceinline__ double gf_block_sum(double v)
{
    __shared__ double part[NT / 64];
    v = gf_wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) part[wave] = v;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) s += part[w];
    }
    __syncthreads();
    return s;
}

// Work item of a workgroup.  The hardware hands workgroup b to XCD b mod 8, and
// each XCD has its own L2: streaming kernels go faster when one XCD sweeps a few
// hundred contiguous KB than when neighbouring 8-32 KB pieces land on different
// XCDs.  Item numbers are therefore dealt in runs of 2^grp_shift per XCD.  A
// permutation of [0, total).
constexpr int GF_N_XCD = 8;
__device__ __forceinline__ uint32_t gf_xcd_order(uint32_t b, uint32_t total, int grp_shift)
{
    const uint32_t span = static_cast<uint32_t>(GF_N_XCD) << grp_shift;
    if (b >= total / span * span) return b;                 // ragged end: identity
    const uint32_t x = b % GF_N_XCD, i = b / GF_N_XCD;
    return ((i >> grp_shift) * span) + (x << grp_shift) + (i & ((1u << grp_shift) - 1u));
}

#endif  // GF_DEVICE_H
