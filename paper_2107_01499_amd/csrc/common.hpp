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

#include <algorithm>
#include <stddef.h>
#include <stdint.h>

#include "bagua_hip.h"

namespace bagua {

// 128-bit lane payload as a native clang vector (the nontemporal builtins need one).
typedef float f4 __attribute__((ext_vector_type(4)));

// Streaming accesses: every bucket byte is touched once per kernel, so loads and stores carry the
// nontemporal hint and do not displace each other in L2 / Infinity Cache.
#ifndef BAGUA_NT
#define BAGUA_NT 1
#endif
template <typename T>
__device__ __forceinline__ T ld_stream(const T* p)
{
#if BAGUA_NT
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename T>
__device__ __forceinline__ void st_stream(T* p, T v)
{
#if BAGUA_NT
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// Preferred rows (of 256 elements) per wave for each chunked kernel (compile-time tuning knobs).
// Measured on MI355X: two rows per wave (512 elements, 8 waves for a 4096-element chunk) stream
// fastest in the worker-side kernels, the fused ring kernel and the sign codec's server kernel; the MinMax
// server kernel and the top-K kernels prefer four.  Larger values are used only when a chunk would need more than 16 waves.
#ifndef BAGUA_RPW_COMPRESS
#define BAGUA_RPW_COMPRESS 2
#endif
#ifndef BAGUA_RPW_DRR
#define BAGUA_RPW_DRR 4
#endif
#ifndef BAGUA_RPW_SIGN
#define BAGUA_RPW_SIGN 2
#endif
#ifndef BAGUA_RPW_DRR_SIGN
#define BAGUA_RPW_DRR_SIGN 2
#endif
#ifndef BAGUA_RPW_TOPK
#define BAGUA_RPW_TOPK 4
#endif
#ifndef BAGUA_RPW_DRR_TOPK
#define BAGUA_RPW_DRR_TOPK 4
#endif
#ifndef BAGUA_RPW_LP
#define BAGUA_RPW_LP 2
#endif
// Peers whose statistics share one barrier in the fused ring kernel.
#ifndef BAGUA_LP_GROUP
#define BAGUA_LP_GROUP 1
#endif
// Workers whose code loads are issued together in the server-side kernels.
#ifndef BAGUA_DRR_NJ
#define BAGUA_DRR_NJ 1
#endif
#ifndef BAGUA_DRR_SIGN_NJ
#define BAGUA_DRR_SIGN_NJ 8
#endif

constexpr int kWave = 64;
constexpr int kRow = 256;      // elements per wave-wide 128-bit access
constexpr int kMaxWaves = 16;  // waves per workgroup (1024 threads)
// Rows (one wavefront each) per workgroup of the kernels that stream row by row without a chunk statistic (decode,
// optimizer steps, peer averaging, the probes).  Measured: two waves per workgroup are 0.5-3 % faster than four and than one.
#ifndef BAGUA_ROW_WAVES
#define BAGUA_ROW_WAVES 2
#endif
constexpr int kRowWaves = BAGUA_ROW_WAVES;

// Upper bound on the workgroup size of a chunked kernel that keeps RPW rows per wave: chunks have at most
// 64 rows, and pick_rpw never asks for more than kMaxWaves waves.
constexpr int wg_threads_max(int rpw)
{
    return kWave * (((64 + rpw - 1) / rpw) < kMaxWaves ? ((64 + rpw - 1) / rpw) : kMaxWaves);
}
static_assert(wg_threads_max(1) <= 1024 && wg_threads_max(2) <= 1024 && wg_threads_max(8) == 512, "launch bound");

struct PtrTable {
    const void* p[BAGUA_MAX_WORKERS];
};
struct MutPtrTable {
    void* p[BAGUA_MAX_WORKERS];
};

// Pacing of a wave's streaming loads in the worker-side kernels.  In a very large launch the memory system is
// saturated and latency is mostly queueing: a wave that waits for each row before it requests the next keeps the
// queues shorter, which the DRAM scheduler rewards (+3 % for the batched sign compression over 229 buckets of
// 1.5 G elements, +0.5-1 % for the unbatched launches in an A/B on the same buffers); in a small launch the longer
// chain of dependent requests costs 3 %.  The launchers pace from 2^28 elements per launch on.
__device__ __forceinline__ void pace_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
inline int pace_for(size_t elements_per_launch) { return elements_per_launch >= (static_cast<size_t>(1) << 28) ? 1 : 0; }

// Index of this wavefront in its workgroup, as a scalar.  The compiler cannot tell that threadIdx.x >> 6 is the same
// in all 64 lanes and would carry every row offset and tail test derived from it through 64-bit vector arithmetic
// and exec-mask branches; read from the first lane it lives in scalar registers.
__device__ __forceinline__ int wave_index()
{
    return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
}

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
__device__ __forceinline__ f4 load_row(const float* __restrict__ row, int lane, int remain, float fill)
{
    f4 r;
    if (remain >= kRow) {
        r = ld_stream(reinterpret_cast<const f4*>(row) + lane);
    } else {
        const int e = lane * 4;
        r.x = (e + 0 < remain) ? row[e + 0] : fill;
        r.y = (e + 1 < remain) ? row[e + 1] : fill;
        r.z = (e + 2 < remain) ? row[e + 2] : fill;
        r.w = (e + 3 < remain) ? row[e + 3] : fill;
    }
    return r;
}
__device__ __forceinline__ void store_row(float* __restrict__ row, int lane, int remain, f4 v)
{
    if (remain >= kRow) {
        st_stream(reinterpret_cast<f4*>(row) + lane, v);
    } else {
        const int e = lane * 4;
        if (e + 0 < remain) row[e + 0] = v.x;
        if (e + 1 < remain) row[e + 1] = v.y;
        if (e + 2 < remain) row[e + 2] = v.z;
        if (e + 3 < remain) row[e + 3] = v.w;
    }
}
// Four u8 codes per lane, little-endian in one dword.
__device__ __forceinline__ uint32_t load_codes_row(const uint8_t* __restrict__ row, int lane, int remain)
{
    if (remain >= kRow) return ld_stream(reinterpret_cast<const uint32_t*>(row) + lane);
    uint32_t w = 0;
    const int e = lane * 4;
#pragma unroll
    for (int t = 0; t < 4; ++t)
        if (e + t < remain) w |= static_cast<uint32_t>(row[e + t]) << (8 * t);
    return w;
}
__device__ __forceinline__ void store_codes_row(uint8_t* __restrict__ row, int lane, int remain, uint32_t w)
{
    if (remain >= kRow) {
        st_stream(reinterpret_cast<uint32_t*>(row) + lane, w);
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
// Per-chunk metadata and top-K entry arrays are accessed element by element: natural alignment suffices, so a
// partition's slice of them (any whole number of chunks) can be passed as it is.
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
inline bool aligned2(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 1u) == 0; }
inline size_t num_chunks(size_t n, size_t chunk) { return (n + chunk - 1) / chunk; }
constexpr size_t kMaxGrid = 0x7fffffffu;

// Aliasing rule of every entry point: a buffer the call writes must not overlap, by byte range, any
// other buffer of the same call (buffers that are only read may overlap each other).
struct RangeCheck {
    struct Item {
        uintptr_t lo, hi;  // [lo, hi)
        bool written;
    };
    Item item[6 * BAGUA_MAX_WORKERS + 12];
    int count = 0;
    void add(const void* p, size_t bytes, bool written)
    {
        if (!p || bytes == 0) return;
        const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
        item[count++] = Item{lo, lo + bytes, written};
    }
    void writes(const void* p, size_t bytes) { add(p, bytes, true); }
    void reads(const void* p, size_t bytes) { add(p, bytes, false); }
    // Sweep over the ranges in address order: a written range must start at or after the end of every
    // earlier range, a read-only range at or after the end of every earlier written range.
    bool disjoint()
    {
        std::sort(item, item + count, [](const Item& a, const Item& b) { return a.lo < b.lo; });
        uintptr_t end_any = 0, end_written = 0;
        for (int i = 0; i < count; ++i) {
            const Item& r = item[i];
            if (r.lo < (r.written ? end_any : end_written)) return false;
            if (r.hi > end_any) end_any = r.hi;
            if (r.written && r.hi > end_written) end_written = r.hi;
        }
        return true;
    }
};

// Rows per wave actually used: the preferred value, doubled until the chunk fits kMaxWaves waves.
inline int pick_rpw(int rows, int preferred)
{
    int rpw = preferred;
    while (rpw < 8 && (rows + rpw - 1) / rpw > kMaxWaves) rpw *= 2;
    return rpw;
}

// Worker-side kernels (compress with error feedback, both codecs), one launch over one contiguous buffer: two rows
// per wave stream fastest, except for chunks of 6 to 8 rows (1536..2048 elements), where that gives a workgroup of
// three or four waves -- measured slowest at every chunk size -- and one row per wave (six to eight waves) is
// 1-4 % faster.  Not used by the batched launches: there every wave first looks up its bucket, and with half the
// bytes per wave that latency is no longer hidden (11 % slower).
inline int pick_rpw_worker(int rows, int preferred)
{
    return pick_rpw(rows, (preferred == 2 && rows >= 6 && rows <= 8) ? 1 : preferred);
}

// Expands `stmt` with a constexpr RPW equal to the runtime value rpw (2, 4 or 8).
#define BAGUA_DISPATCH_RPW(rpw, stmt)                    \
    switch (rpw) {                                        \
        case 2: { constexpr int RPW = 2; stmt; } break;  \
        case 4: { constexpr int RPW = 4; stmt; } break;  \
        default: { constexpr int RPW = 8; stmt; } break; \
    }

// The same for the worker-side kernels, which also come with one row per wave.
#define BAGUA_DISPATCH_RPW_WORKER(rpw, stmt)             \
    switch (rpw) {                                        \
        case 1: { constexpr int RPW = 1; stmt; } break;  \
        case 2: { constexpr int RPW = 2; stmt; } break;  \
        case 4: { constexpr int RPW = 4; stmt; } break;  \
        default: { constexpr int RPW = 8; stmt; } break; \
    }

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? BAGUA_OK : BAGUA_ERR_LAUNCH;
}

}  // namespace bagua
