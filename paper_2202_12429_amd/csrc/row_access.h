// Row-granular access shared by the cache, forward and backward kernels.
//
// A row is moved as 16-byte pieces, one piece per lane.  A row of `lpr` pieces (lanes per row) is
// handled by a group of GW consecutive lanes, GW the next power of two >= lpr (so four D=48 fp32
// rows, 12 pieces each, share a wavefront); lanes with piece index >= lpr idle.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "common.h"

namespace bp {

constexpr int kRowBlock = 256;   // threads per workgroup of the row kernels

inline int group_width(int lpr) {
    int gw = 1;
    while (gw < lpr) gw <<= 1;
    return gw;
}

// bf16 <-> fp32, round-to-nearest-even on the way down (NaN stays NaN)
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// One 16-byte piece of a weight row as fp32 values: 4 for fp32 storage, 8 for bf16 storage.
template <bool BF16>
struct Piece {
    static constexpr int N = BF16 ? 8 : 4;
    float v[N];
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = 0.f;
    }
    __device__ __forceinline__ void decode(const uint4& raw) {
        if constexpr (BF16) {
            const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[2 * i] = bf16_bits_to_f32(r[i] & 0xffffu);
                v[2 * i + 1] = bf16_bits_to_f32(r[i] >> 16);
            }
        } else {
            v[0] = __uint_as_float(raw.x);
            v[1] = __uint_as_float(raw.y);
            v[2] = __uint_as_float(raw.z);
            v[3] = __uint_as_float(raw.w);
        }
    }
    __device__ __forceinline__ uint4 encode() const {
        uint4 raw;
        if constexpr (BF16) {
            uint32_t r[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = f32_to_bf16_bits(v[2 * i]) | (f32_to_bf16_bits(v[2 * i + 1]) << 16);
            raw = make_uint4(r[0], r[1], r[2], r[3]);
        } else {
            raw = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
        }
        return raw;
    }
    // fp32 [.. D] array (pooled output, upstream gradient, Adagrad state, partial sums): the piece of lane c
    // starts at element c * N of the row.
    __device__ __forceinline__ void load_f32(const float* row, int c) {
        const float4* p = reinterpret_cast<const float4*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const float4 t = p[i];
            v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
        }
    }
    __device__ __forceinline__ void store_f32(float* row, int c) const {
        float4* p = reinterpret_cast<float4*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N / 4; ++i) p[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
    }
    // Streaming variants for data touched once (pooled output, upstream gradient of one-hot bags): non-temporal
    // accesses leave the cache lines to the table rows that are reused.
    __device__ __forceinline__ void load_f32_stream(const float* row, int c) {
        typedef float vec4 __attribute__((ext_vector_type(4)));
        const vec4* p = reinterpret_cast<const vec4*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const vec4 t = __builtin_nontemporal_load(p + i);
            v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
        }
    }
    __device__ __forceinline__ void store_f32_stream(float* row, int c) const {
        typedef float vec4 __attribute__((ext_vector_type(4)));
        vec4* p = reinterpret_cast<vec4*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            vec4 t;
            t.x = v[4 * i]; t.y = v[4 * i + 1]; t.z = v[4 * i + 2]; t.w = v[4 * i + 3];
            __builtin_nontemporal_store(t, p + i);
        }
    }
    __device__ __forceinline__ void add(const Piece& o) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += o.v[i];
    }
};

// Calls f.template run<GW, BF16>() for the group width and storage type of a configuration.
template <typename F>
int dispatch_row(int lpr, bool bf16, F&& f) {
    const int gw = group_width(lpr);
#define BP_CASE(W)                                         \
    case W:                                                \
        return bf16 ? f.template run<W, true>() : f.template run<W, false>();
    switch (gw) {
        BP_CASE(1) BP_CASE(2) BP_CASE(4) BP_CASE(8) BP_CASE(16) BP_CASE(32) BP_CASE(64)
        default: return fail(BP_ERR_UNSUPPORTED, "row of %d 16-byte pieces is wider than 1024 bytes", lpr);
    }
#undef BP_CASE
}

}  // namespace bp
