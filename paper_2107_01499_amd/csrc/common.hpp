// Device-side building blocks shared by the gfx950 kernels of this library.
//
// Data layout used by every chunked kernel: a chunk of C elements (C a multiple of 256) is cut
// into "rows" of 256 consecutive elements.  One 64-lane wavefront reads or writes a row with a
// single 128-bit access per lane (lane l owns elements 4l..4l+3 of the row), which is the widest
// coalesced access the memory pipeline offers.  A wavefront keeps ROWS_PER_WAVE rows in registers,
// so a chunk is read from HBM exactly once: statistics and quantisation both work on registers.
// A workgroup is the ceil(rows / ROWS_PER_WAVE) wavefronts of one chunk; their partial statistics
// meet in LDS behind a single barrier.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include "bagua_hip.h"

namespace bagua {

constexpr int kWave = 64;
constexpr int kRow = 256;      // elements per wave-wide 128-bit access
constexpr int kMaxWaves = 16;  // waves per workgroup (1024 threads)

struct PtrTable {
    const void* p[BAGUA_MAX_WORKERS];
};
struct MutPtrTable {
    void* p[BAGUA_MAX_WORKERS];
};

// ---------------------------------------------------------------- wave-level reductions
__device__ __forceinline__ float wave_min(float v)
{
#pragma unroll
    for (int s = 1; s < kWave; s <<= 1) v = fminf(v, __shfl_xor(v, s, kWave));
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int s = 1; s < kWave; s <<= 1) v = fmaxf(v, __shfl_xor(v, s, kWave));
    return v;
}
// acc[l] <- acc[l] + acc[l xor s], s = 1,2,...,32: the fixed summation tree of the sign codec.
__device__ __forceinline__ float wave_butterfly_sum(float v)
{
#pragma unroll
    for (int s = 1; s < kWave; s <<= 1) v = v + __shfl_xor(v, s, kWave);
    return v;
}

// ---------------------------------------------------------------- row accessors with ragged tails
// `remain` = number of valid elements counted from the start of the row (wave-uniform, may be <= 0
// for an absent row or >= 256 for a full one).  Absent elements read as `fill`.
__device__ __forceinline__ float4 load_row(const float* __restrict__ row, int lane, long remain, float fill)
{
    float4 r;
    if (remain >= kRow) {
        r = reinterpret_cast<const float4*>(row)[lane];
    } else {
        const int e = lane * 4;
        r.x = (e + 0 < remain) ? row[e + 0] : fill;
        r.y = (e + 1 < remain) ? row[e + 1] : fill;
        r.z = (e + 2 < remain) ? row[e + 2] : fill;
        r.w = (e + 3 < remain) ? row[e + 3] : fill;
    }
    return r;
}
__device__ __forceinline__ void store_row(float* __restrict__ row, int lane, long remain, float4 v)
{
    if (remain >= kRow) {
        reinterpret_cast<float4*>(row)[lane] = v;
    } else {
        const int e = lane * 4;
        if (e + 0 < remain) row[e + 0] = v.x;
        if (e + 1 < remain) row[e + 1] = v.y;
        if (e + 2 < remain) row[e + 2] = v.z;
        if (e + 3 < remain) row[e + 3] = v.w;
    }
}
// Four u8 codes per lane, little-endian in one dword.
__device__ __forceinline__ uint32_t load_codes_row(const uint8_t* __restrict__ row, int lane, long remain)
{
    if (remain >= kRow) return reinterpret_cast<const uint32_t*>(row)[lane];
    uint32_t w = 0;
    const int e = lane * 4;
#pragma unroll
    for (int t = 0; t < 4; ++t)
        if (e + t < remain) w |= static_cast<uint32_t>(row[e + t]) << (8 * t);
    return w;
}
__device__ __forceinline__ void store_codes_row(uint8_t* __restrict__ row, int lane, long remain, uint32_t w)
{
    if (remain >= kRow) {
        reinterpret_cast<uint32_t*>(row)[lane] = w;
    } else {
        const int e = lane * 4;
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (e + t < remain) row[e + t] = static_cast<uint8_t>(w >> (8 * t));
    }
}

__device__ __forceinline__ float byte_to_float(uint32_t w, int b) { return static_cast<float>((w >> (8 * b)) & 0xffu); }

// Quantisation step of a chunk from its stored statistics: fl(fl(mx - mn) / 255), 0 for a flat chunk.
__device__ __forceinline__ float minmax_step(float mn, float mx)
{
    const float r = mx - mn;
    return (r == 0.0f) ? 0.0f : r / 255.0f;
}

// ---------------------------------------------------------------- host-side argument checks
inline bool chunk_ok(size_t chunk) { return chunk >= 256 && chunk <= 16384 && chunk % 256 == 0; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t num_chunks(size_t n, size_t chunk) { return (n + chunk - 1) / chunk; }
constexpr size_t kMaxGrid = 0x7fffffffu;

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? BAGUA_OK : BAGUA_ERR_LAUNCH;
}

}  // namespace bagua
