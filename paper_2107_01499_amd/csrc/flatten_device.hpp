// Tensor table of a planned bucket (see bagua_flatten_plan) and the device-side lookups on it.
#pragma once
#include "common.hpp"

namespace bagua {

struct TensorDesc {
    const float* src;
    size_t numel;
    size_t dst;  // element offset in the bucket
};

// The tensor's pointer as read from the table on the device.  Cast through the global address space: a pointer loaded
// from memory is otherwise a generic one, and every access through it a "flat" instruction that counts against both
// wait counters and cannot stay in flight past LDS or scalar-memory waits.
__device__ __forceinline__ const float* tensor_ptr(const TensorDesc& d)
{
    typedef __attribute__((address_space(1))) const float* global_ptr;
    return (const float*)reinterpret_cast<global_ptr>(reinterpret_cast<uintptr_t>(d.src));
}

#ifndef BAGUA_FLATTEN_TILE
#define BAGUA_FLATTEN_TILE 1024
#endif
constexpr int kTile = BAGUA_FLATTEN_TILE;  // bucket elements per workgroup (256 lanes x kTile/1024 groups of four)
static_assert(kTile % 1024 == 0, "a tile is a whole number of 256-lane groups of four elements");

inline size_t align16_up(size_t b) { return (b + 15) & ~static_cast<size_t>(15); }
inline size_t num_tiles(size_t bucket_numel) { return (bucket_numel + kTile - 1) / kTile; }

// Value of bucket element e, starting the search at tensor t (the first tensor whose end is > some e' <= e).
__device__ __forceinline__ float element_at(const TensorDesc* __restrict__ desc, uint32_t& t, uint32_t T, size_t e)
{
    while (t < T && desc[t].dst + desc[t].numel <= e) ++t;
    if (t < T && desc[t].dst <= e) return tensor_ptr(desc[t])[e - desc[t].dst];
    return 0.0f;
}


// 256 consecutive floats starting at s, where s is only 4-byte aligned: lane l receives s[4l .. 4l+3] with ONE
// 128-bit load whose declared alignment is 4 bytes (the memory pipeline splits the accesses that straddle a 16-byte
// boundary; one request per lane instead of four).  All 256 elements must be readable.
typedef float f4_a4 __attribute__((ext_vector_type(4), aligned(4)));
__device__ __forceinline__ f4 load_row_shifted(const float* __restrict__ s, int lane)
{
    const f4_a4 v = __builtin_nontemporal_load(reinterpret_cast<const f4_a4*>(s) + lane);
    return f4{v.x, v.y, v.z, v.w};
}

// The planned workspace: T descriptors, then (tiles + 1) "first tensor" indices.
struct FlattenPlanView {
    const TensorDesc* desc;
    const uint32_t* tile_first;
};
inline FlattenPlanView plan_view(const void* workspace, size_t T)
{
    const size_t desc_bytes = align16_up((T ? T : 1) * sizeof(TensorDesc));
    return FlattenPlanView{static_cast<const TensorDesc*>(workspace),
                           reinterpret_cast<const uint32_t*>(static_cast<const unsigned char*>(workspace) + desc_bytes)};
}

// One 256-element row of the (virtual) bucket starting at element e0 (a multiple of 256), gathered
// straight from the layer tensors: lane l receives elements e0+4l .. e0+4l+3; elements beyond
// `remain` or not covered by a tensor read as +0.0f.
__device__ __forceinline__ f4 gather_row(const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ tile_first,
                                         uint32_t T, size_t e0, int lane, int remain)
{
    const size_t tile = e0 / kTile;
    uint32_t lo = tile_first[tile];
    const uint32_t hi = tile_first[tile + 1];
    // first tensor whose end lies beyond e0 (wave-uniform search)
    while (lo < hi && desc[lo].dst + desc[lo].numel <= e0) ++lo;
    if (lo < T && remain >= kRow) {
        const TensorDesc d = desc[lo];
        if (d.dst <= e0 && e0 + kRow <= d.dst + d.numel) {
            const float* s = tensor_ptr(d) + (e0 - d.dst);
            if ((reinterpret_cast<uintptr_t>(s) & 15u) == 0) return ld_stream(reinterpret_cast<const f4*>(s) + lane);
            return load_row_shifted(s, lane);
        }
    }
    uint32_t t = lo;
    const size_t e = e0 + lane * 4;
    const int l4 = lane * 4;
    f4 v;
    v.x = (l4 + 0 < remain) ? element_at(desc, t, T, e + 0) : 0.0f;
    v.y = (l4 + 1 < remain) ? element_at(desc, t, T, e + 1) : 0.0f;
    v.z = (l4 + 2 < remain) ? element_at(desc, t, T, e + 2) : 0.0f;
    v.w = (l4 + 3 < remain) ? element_at(desc, t, T, e + 3) : 0.0f;
    return v;
}

}  // namespace bagua
