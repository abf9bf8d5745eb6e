// Bucket flatten (Section 3.1 "Flattening", Section 3.5 "Tensor Bucketing and Memory Flattening"):
// gather T layer tensors into one contiguous fp32 bucket, zero-filling what no tensor covers.
//
// The copy is driven from the destination side: each lane owns 16-byte aligned groups of four
// bucket elements and looks up which tensor covers them, so every bucket byte is written exactly
// once with 128-bit stores (8 bytes of traffic per element).  A host-built table in the
// caller's workspace gives, for every tile of the bucket, the first tensor that can intersect it.
#include <mutex>
#include <vector>

#include "batch.hpp"
#include "flatten_device.hpp"

#pragma clang fp contract(off)

namespace bagua {

// Workgroups are single wavefronts: a plain copy streams 3-4 % faster that way than with four waves per workgroup
// (a wave's slot is free again as soon as its own stores are out).  kTileWaves of them share one tile of the table.
constexpr int kTileWaves = kTile / kRow;
static_assert(kTile == 1024 && kTileWaves == 4, "the tile body below moves 16 bytes per lane of 256 lanes");

// One tile (kTile elements) of one bucket; `tile` = index of the tile in its bucket, `tid` = 0..255 = this lane's
// place among the tile's 256 lanes.
__device__ __forceinline__ void flatten_tile(const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ tile_first,
                                             uint32_t T, float* __restrict__ bucket, size_t bucket_numel, size_t tile,
                                             uint32_t tid)
{
    const size_t tile0 = tile * kTile;
    const uint32_t lo0 = tile_first[tile], hi0 = tile_first[tile + 1];

    // Fast path (almost every tile of a large tensor): the whole tile lies inside one tensor whose
    // source is 16-byte congruent with the bucket -> a plain streaming copy with a uniform base pointer.
    if (lo0 < T && tile0 + kTile <= bucket_numel) {
        const TensorDesc d = desc[lo0];   // uniform: scalar loads
        if (d.dst <= tile0 && tile0 + kTile <= d.dst + d.numel) {
            const float* s = tensor_ptr(d) + (tile0 - d.dst);
            if ((reinterpret_cast<uintptr_t>(s) & 15u) == 0) {
                const f4* s4 = reinterpret_cast<const f4*>(s);
                f4* b4 = reinterpret_cast<f4*>(bucket + tile0);
                f4 v[kTile / 1024];
#pragma unroll
                for (int g = 0; g < kTile / 1024; ++g) v[g] = ld_stream(s4 + g * 256 + tid);
#pragma unroll
                for (int g = 0; g < kTile / 1024; ++g) st_stream(b4 + g * 256 + tid, v[g]);
                return;
            }
            // same, source only 4-byte aligned: 128-bit loads with 4-byte declared alignment, aligned 128-bit stores
            f4* b4 = reinterpret_cast<f4*>(bucket + tile0);
#pragma unroll
            for (int g = 0; g < kTile / 1024; ++g)
                st_stream(b4 + g * 256 + tid, load_row_shifted(s + g * 1024, tid));
            return;
        }
    }

#pragma unroll
    for (int g = 0; g < kTile / 1024; ++g) {
        const size_t e = tile0 + static_cast<size_t>(g) * 1024 + tid * 4;
        if (e >= bucket_numel) continue;
        // first tensor whose end lies beyond e, searched in [lo0, hi0]
        uint32_t lo = lo0, hi = hi0;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (desc[mid].dst + desc[mid].numel <= e) lo = mid + 1;
            else hi = mid;
        }
        uint32_t t = lo;
        f4 v;
        bool done = false;
        if (t < T) {
            const TensorDesc d = desc[t];
            if (d.dst <= e && e + 4 <= d.dst + d.numel) {
                const float* s = tensor_ptr(d) + (e - d.dst);
                const f4_a4 u = __builtin_nontemporal_load(reinterpret_cast<const f4_a4*>(s));   // any 4-byte alignment
                v = f4{u.x, u.y, u.z, u.w};
                done = true;
            }
        }
        if (!done) {
            v.x = (e + 0 < bucket_numel) ? element_at(desc, t, T, e + 0) : 0.0f;
            v.y = (e + 1 < bucket_numel) ? element_at(desc, t, T, e + 1) : 0.0f;
            v.z = (e + 2 < bucket_numel) ? element_at(desc, t, T, e + 2) : 0.0f;
            v.w = (e + 3 < bucket_numel) ? element_at(desc, t, T, e + 3) : 0.0f;
        }
        if (e + 4 <= bucket_numel) {
            st_stream(reinterpret_cast<f4*>(bucket + e), v);
        } else {
            bucket[e] = v.x;
            if (e + 1 < bucket_numel) bucket[e + 1] = v.y;
            if (e + 2 < bucket_numel) bucket[e + 2] = v.z;
        }
    }
}

__global__ void __launch_bounds__(kWave)
k_flatten(const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ tile_first, uint32_t T,
          float* __restrict__ bucket, size_t bucket_numel)
{
    flatten_tile(desc, tile_first, T, bucket, bucket_numel, blockIdx.x / kTileWaves,
                 (blockIdx.x % kTileWaves) * kWave + threadIdx.x);
}

// Batched: entry = [planned workspace, T, bucket, bucket_numel]; unit = tile.
__global__ void __launch_bounds__(kWave)
k_flatten_batched(BatchView bv)
{
    const uint32_t unit = blockIdx.x / kTileWaves;
    const uint32_t b = batch_find(bv, unit);
    const uint64_t* e = bv.entries + static_cast<size_t>(b) * bv.entry_words;
    const size_t T = e[1];
    const unsigned char* ws = table_ptr<const unsigned char>(e[0]);
    const size_t desc_bytes = ((T ? T : 1) * sizeof(TensorDesc) + 15) & ~static_cast<size_t>(15);
    flatten_tile(reinterpret_cast<const TensorDesc*>(ws), reinterpret_cast<const uint32_t*>(ws + desc_bytes),
                 static_cast<uint32_t>(T), table_ptr<float>(e[2]), e[3], unit - bv.first_unit[b],
                 (blockIdx.x % kTileWaves) * kWave + threadIdx.x);
}

// Inverse scatter: copy every tensor's range of the bucket back into the tensor (same table as the
// flatten; bucket elements no tensor covers are skipped).  The tensors' pointers in the table are
// written through, so the table must have been planned with writable tensors.
__global__ void __launch_bounds__(kWave)
k_unflatten(const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ tile_first, uint32_t T,
            const float* __restrict__ bucket, size_t bucket_numel)
{
    const size_t tile = blockIdx.x / kTileWaves;                                  // single-wave workgroups, as in k_flatten
    const uint32_t tid = (blockIdx.x % kTileWaves) * kWave + threadIdx.x;
    const size_t tile0 = tile * kTile;
    const uint32_t lo0 = tile_first[tile], hi0 = tile_first[tile + 1];
    if (lo0 < T && tile0 + kTile <= bucket_numel) {
        const TensorDesc d = desc[lo0];
        if (d.dst <= tile0 && tile0 + kTile <= d.dst + d.numel) {
            float* s = const_cast<float*>(tensor_ptr(d)) + (tile0 - d.dst);
            if ((reinterpret_cast<uintptr_t>(s) & 15u) == 0) {
                f4* s4 = reinterpret_cast<f4*>(s);
                const f4* b4 = reinterpret_cast<const f4*>(bucket + tile0);
                f4 v[kTile / 1024];
#pragma unroll
                for (int g = 0; g < kTile / 1024; ++g) v[g] = ld_stream(b4 + g * 256 + tid);
#pragma unroll
                for (int g = 0; g < kTile / 1024; ++g) st_stream(s4 + g * 256 + tid, v[g]);
                return;
            }
            // same, tensor only 4-byte aligned: 128-bit stores with 4-byte declared alignment
            const f4* b4 = reinterpret_cast<const f4*>(bucket + tile0);
            f4_a4* s4 = reinterpret_cast<f4_a4*>(s);
#pragma unroll
            for (int g = 0; g < kTile / 1024; ++g) {
                const f4 v = ld_stream(b4 + g * 256 + tid);
                __builtin_nontemporal_store(f4_a4{v.x, v.y, v.z, v.w}, s4 + g * 256 + tid);
            }
            return;
        }
    }
#pragma unroll
    for (int g = 0; g < kTile / 1024; ++g) {
        const size_t e = tile0 + static_cast<size_t>(g) * 1024 + tid * 4;
        if (e >= bucket_numel) continue;
        uint32_t lo = lo0, hi = hi0;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (desc[mid].dst + desc[mid].numel <= e) lo = mid + 1;
            else hi = mid;
        }
        uint32_t t = lo;
        if (t < T && e + 4 <= bucket_numel) {
            const TensorDesc d = desc[t];
            if (d.dst <= e && e + 4 <= d.dst + d.numel) {
                float* s = const_cast<float*>(tensor_ptr(d)) + (e - d.dst);
                const f4 v = ld_stream(reinterpret_cast<const f4*>(bucket + e));
                __builtin_nontemporal_store(f4_a4{v.x, v.y, v.z, v.w}, reinterpret_cast<f4_a4*>(s));   // any 4-byte alignment
                continue;
            }
        }
        for (int q = 0; q < 4; ++q) {
            const size_t eq = e + q;
            if (eq >= bucket_numel) break;
            while (t < T && desc[t].dst + desc[t].numel <= eq) ++t;
            if (t < T && desc[t].dst <= eq) const_cast<float*>(tensor_ptr(desc[t]))[eq - desc[t].dst] = bucket[eq];
        }
    }
}

// Decode fused into the inverse scatter: the decoded value of every bucket element goes straight to the layer tensor
// that covers it (nothing is written for uncovered elements), so the decoded bucket never exists in memory.
// CODEC 0: MinMax-u8 (codes u8[n], meta = (min, max) pairs); CODEC 1: sign (codes = sign words, meta = scales).
constexpr int kDecodeTiles = 4;   // tiles per workgroup of the decode + scatter kernel
template <int CODEC>
__global__ void __launch_bounds__(256)
k_decompress_unflatten(const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ tile_first, uint32_t T,
                       const void* __restrict__ codes, const float* __restrict__ meta, size_t n, uint32_t chunk)
{
    static_assert(kTile == 1024, "one 256-element row per wave and tile");
    const int wave = wave_index(), lane = threadIdx.x & 63;
    const size_t ntiles = (n + kTile - 1) / kTile;
    const size_t first = static_cast<size_t>(blockIdx.x) * kDecodeTiles;

    // 1. everything that does not depend on the tensor table: codes and per-chunk metadata of this wave's rows
    uint32_t w[kDecodeTiles];
    float m0[kDecodeTiles], m1[kDecodeTiles];
#pragma unroll
    for (int i = 0; i < kDecodeTiles; ++i) {
        const size_t e0 = (first + i) * kTile + wave * kRow;   // this wave's row of tile i
        w[i] = 0;
        m0[i] = m1[i] = 0.0f;
        if (e0 >= n) continue;
        const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
        const size_t c = e0 / chunk;                            // a row never straddles chunks
        if (CODEC == 0) {
            m0[i] = meta[2 * c];
            m1[i] = meta[2 * c + 1];
            w[i] = load_codes_row(static_cast<const uint8_t*>(codes) + e0, lane, remain);
        } else {
            m0[i] = meta[c];
            if (static_cast<int>(lane >> 3) * 32 < remain) w[i] = static_cast<const uint32_t*>(codes)[(e0 >> 5) + (lane >> 3)];
        }
    }
    // 2. the table: almost every tile lies inside one tensor, whose base pointer is then uniform
    float* tile_dst[kDecodeTiles];
    uint32_t lo0[kDecodeTiles], hi0[kDecodeTiles];
#pragma unroll
    for (int i = 0; i < kDecodeTiles; ++i) {
        const size_t tile = first + i;
        tile_dst[i] = nullptr;
        lo0[i] = hi0[i] = T;
        if (tile >= ntiles) continue;
        lo0[i] = tile_first[tile];
        hi0[i] = tile_first[tile + 1];
        const size_t tile0 = tile * kTile;
        if (lo0[i] < T && tile0 + kTile <= n) {
            const TensorDesc d = desc[lo0[i]];
            if (d.dst <= tile0 && tile0 + kTile <= d.dst + d.numel) tile_dst[i] = const_cast<float*>(tensor_ptr(d)) + (tile0 - d.dst);
        }
    }
    // 3. decode and scatter
#pragma unroll
    for (int i = 0; i < kDecodeTiles; ++i) {
        const size_t tile0 = (first + i) * kTile;
        const size_t e0 = tile0 + wave * kRow;
        if (e0 >= n) continue;
        f4 v;
        if (CODEC == 0) {
            const float mn = m0[i], step = minmax_step(mn, m1[i]);
            v.x = mn + byte_to_float(w[i], 0) * step;
            v.y = mn + byte_to_float(w[i], 1) * step;
            v.z = mn + byte_to_float(w[i], 2) * step;
            v.w = mn + byte_to_float(w[i], 3) * step;
        } else {
            const float sc = m0[i], neg = -sc;
            const uint32_t nib = w[i] >> (4 * (lane & 7));
            v.x = (nib & 1u) ? sc : neg;
            v.y = (nib & 2u) ? sc : neg;
            v.z = (nib & 4u) ? sc : neg;
            v.w = (nib & 8u) ? sc : neg;
        }
        const size_t e = e0 + lane * 4;
        if (tile_dst[i]) {
            typedef __attribute__((address_space(1))) float* global_ptr;     // tile_dst[i] came from the tensor table
            float* gd = (float*)reinterpret_cast<global_ptr>(reinterpret_cast<uintptr_t>(tile_dst[i]));
            __builtin_nontemporal_store(f4_a4{v.x, v.y, v.z, v.w}, reinterpret_cast<f4_a4*>(gd + (e - tile0)));
            continue;
        }
        if (e >= n) continue;
        // first tensor whose end lies beyond e, searched in [lo0, hi0]
        uint32_t lo = lo0[i], hi = hi0[i];
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (desc[mid].dst + desc[mid].numel <= e) lo = mid + 1;
            else hi = mid;
        }
        uint32_t t = lo;
        if (t < T && e + 4 <= n) {
            const TensorDesc d = desc[t];
            if (d.dst <= e && e + 4 <= d.dst + d.numel) {
                float* s = const_cast<float*>(tensor_ptr(d)) + (e - d.dst);
                __builtin_nontemporal_store(f4_a4{v.x, v.y, v.z, v.w}, reinterpret_cast<f4_a4*>(s));
                continue;
            }
        }
        const float q[4] = {v.x, v.y, v.z, v.w};
        for (int r = 0; r < 4; ++r) {
            const size_t eq = e + r;
            if (eq >= n) break;
            while (t < T && desc[t].dst + desc[t].numel <= eq) ++t;
            if (t < T && desc[t].dst <= eq) const_cast<float*>(tensor_ptr(desc[t]))[eq - desc[t].dst] = q[r];
        }
    }
}

}  // namespace bagua

using namespace bagua;

extern "C" size_t bagua_flatten_workspace_bytes(size_t T, size_t bucket_numel)
{
    return align16_up((T ? T : 1) * sizeof(TensorDesc)) + align16_up((num_tiles(bucket_numel) + 1) * sizeof(uint32_t));
}

extern "C" int bagua_flatten_plan(const void* const* src, const size_t* numel, const size_t* dst_offset, size_t T,
                                  size_t bucket_numel, void* workspace, size_t workspace_bytes, void* stream)
{
    if (bucket_numel == 0 || !workspace || (T && (!src || !numel || !dst_offset))) return BAGUA_ERR_INVALID_ARG;
    if (T > 0xfffffff0u || num_tiles(bucket_numel) > kMaxGrid / kTileWaves) return BAGUA_ERR_UNSUPPORTED;
    if (workspace_bytes < bagua_flatten_workspace_bytes(T, bucket_numel)) return BAGUA_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return BAGUA_ERR_ALIGNMENT;
    size_t prev_end = 0;
    for (size_t t = 0; t < T; ++t) {
        if (numel[t] && !src[t]) return BAGUA_ERR_INVALID_ARG;
        if (dst_offset[t] < prev_end) return BAGUA_ERR_INVALID_ARG;                 // ascending, no overlap
        if (numel[t] > bucket_numel || dst_offset[t] > bucket_numel - numel[t]) return BAGUA_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(src[t]) & 3u) return BAGUA_ERR_ALIGNMENT;
        prev_end = dst_offset[t] + numel[t];
    }
    const size_t desc_bytes = align16_up((T ? T : 1) * sizeof(TensorDesc));
    const size_t tiles = num_tiles(bucket_numel);
    std::vector<unsigned char> host(bagua_flatten_workspace_bytes(T, bucket_numel), 0);
    TensorDesc* d = reinterpret_cast<TensorDesc*>(host.data());
    uint32_t* first = reinterpret_cast<uint32_t*>(host.data() + desc_bytes);
    for (size_t t = 0; t < T; ++t) d[t] = TensorDesc{static_cast<const float*>(src[t]), numel[t], dst_offset[t]};
    // first[i] = first tensor whose end lies beyond the start of tile i (T if none); first[tiles] = same for the end
    size_t t = 0;
    for (size_t i = 0; i <= tiles; ++i) {
        const size_t e = i * static_cast<size_t>(kTile);
        while (t < T && dst_offset[t] + numel[t] <= e) ++t;
        first[i] = static_cast<uint32_t>(t);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(workspace, host.data(), host.size(), hipMemcpyHostToDevice, s) != hipSuccess) return BAGUA_ERR_LAUNCH;
    if (hipStreamSynchronize(s) != hipSuccess) return BAGUA_ERR_LAUNCH;   // `host` dies at return
    return BAGUA_OK;
}

extern "C" int bagua_bucket_flatten_run(const void* workspace, size_t T, float* bucket, size_t bucket_numel, void* stream)
{
    if (!workspace || !bucket || bucket_numel == 0) return BAGUA_ERR_INVALID_ARG;
    if (T > 0xfffffff0u || num_tiles(bucket_numel) > kMaxGrid / kTileWaves) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(workspace) || !aligned16(bucket)) return BAGUA_ERR_ALIGNMENT;
    const FlattenPlanView pv = plan_view(workspace, T);
    hipLaunchKernelGGL(k_flatten, dim3(static_cast<unsigned>(num_tiles(bucket_numel) * kTileWaves)), dim3(kWave), 0,
                       static_cast<hipStream_t>(stream), pv.desc, pv.tile_first, static_cast<uint32_t>(T), bucket, bucket_numel);
    return launch_status();
}

extern "C" int bagua_bucket_flatten(const void* const* src, const size_t* numel, const size_t* dst_offset, size_t T,
                                    float* bucket, size_t bucket_numel, void* workspace, size_t workspace_bytes,
                                    void* stream)
{
    if (!bucket) return BAGUA_ERR_INVALID_ARG;
    if (!aligned16(bucket)) return BAGUA_ERR_ALIGNMENT;
    const int rc = bagua_flatten_plan(src, numel, dst_offset, T, bucket_numel, workspace, workspace_bytes, stream);
    if (rc != BAGUA_OK) return rc;
    return bagua_bucket_flatten_run(workspace, T, bucket, bucket_numel, stream);
}

extern "C" int bagua_bucket_flatten_batched_run(const void* const* plans, const size_t* T, float* const* bucket,
                                                const size_t* bucket_numel, size_t B, void* workspace,
                                                size_t workspace_bytes, void* stream)
{
    if (!plans || !T || !bucket || !bucket_numel || !workspace || B == 0 || B > 0xffffffffu) return BAGUA_ERR_INVALID_ARG;
    if (workspace_bytes < bagua_batch_workspace_bytes(B, 0)) return BAGUA_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return BAGUA_ERR_ALIGNMENT;
    const size_t ew = batch_entry_words_for(0);
    std::vector<uint64_t> table(batch_table_words(B, ew), 0);
    uint64_t* entries = table.data() + batch_first_words(B);
    RangeList rl;
    size_t total = 0;
    for (size_t b = 0; b < B; ++b) {
        if (!plans[b] || !bucket[b] || bucket_numel[b] == 0) return BAGUA_ERR_INVALID_ARG;
        if (T[b] > 0xfffffff0u) return BAGUA_ERR_UNSUPPORTED;
        if (!aligned16(plans[b]) || !aligned16(bucket[b])) return BAGUA_ERR_ALIGNMENT;
        rl.reads(plans[b], bagua_flatten_workspace_bytes(T[b], bucket_numel[b]));
        rl.writes(bucket[b], bucket_numel[b] * sizeof(float));
        table[b] = total;
        uint64_t* e = entries + b * ew;
        e[0] = reinterpret_cast<uintptr_t>(plans[b]);
        e[1] = T[b];
        e[2] = reinterpret_cast<uintptr_t>(bucket[b]);
        e[3] = bucket_numel[b];
        total += num_tiles(bucket_numel[b]);
    }
    table[B] = total;
    batch_fill_lut(table.data(), B, ew);
    rl.writes(workspace, table.size() * sizeof(uint64_t));
    if (!rl.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (total > kMaxGrid / kTileWaves) return BAGUA_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (batch_upload(table.data(), table.size(), static_cast<uint64_t*>(workspace), s) != BAGUA_OK) return BAGUA_ERR_LAUNCH;
    hipLaunchKernelGGL(k_flatten_batched, dim3(static_cast<unsigned>(total * kTileWaves)), dim3(kWave), 0, s,
                       batch_view(workspace, B, ew, total));
    return launch_status();
}

extern "C" int bagua_decompress_unflatten(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                                          const void* workspace, size_t T, void* stream)
{
    if (codec != BAGUA_CODEC_MINMAX_U8 && codec != BAGUA_CODEC_SIGN1) return BAGUA_ERR_INVALID_ARG;
    if (!codes || !meta || !workspace || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    if (T > 0xfffffff0u || num_tiles(n) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(codes) || !aligned4(meta) || !aligned16(workspace)) return BAGUA_ERR_ALIGNMENT;
    const FlattenPlanView pv = plan_view(workspace, T);
    dim3 grid(static_cast<unsigned>((num_tiles(n) + kDecodeTiles - 1) / kDecodeTiles)), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (codec == BAGUA_CODEC_MINMAX_U8)
        hipLaunchKernelGGL((k_decompress_unflatten<0>), grid, block, 0, s, pv.desc, pv.tile_first, static_cast<uint32_t>(T),
                           codes, meta, n, static_cast<uint32_t>(chunk));
    else
        hipLaunchKernelGGL((k_decompress_unflatten<1>), grid, block, 0, s, pv.desc, pv.tile_first, static_cast<uint32_t>(T),
                           codes, meta, n, static_cast<uint32_t>(chunk));
    return launch_status();
}

// ------------------------------------------------------------------------------------------ no allocation
// bagua_bucket_flatten_static: the tensor table lives in a fixed device array of this library instead of a
// caller-provided workspace, and is built on the device from kernel arguments, so the call allocates
// nothing, copies nothing from host memory and never synchronises.
namespace bagua {

constexpr size_t kStaticMaxT = BAGUA_FLATTEN_STATIC_MAX_TENSORS;
constexpr size_t kStaticMaxNumel = BAGUA_FLATTEN_STATIC_MAX_NUMEL;
constexpr size_t kStaticDescBytes = kStaticMaxT * sizeof(TensorDesc);
constexpr size_t kStaticTileBytes = (kStaticMaxNumel / kTile + 2) * sizeof(uint32_t);
static_assert(kStaticDescBytes % 16 == 0, "the tile table starts 16-byte aligned");

// One copy of this array exists on every GPU the library runs on.  In host code the name is only a handle:
// the device address is looked up once per device (static_scratch_ptr) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[kStaticDescBytes + kStaticTileBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // per device, nullptr until looked up
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (nullptr on error).
static unsigned char* static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return static_cast<unsigned char*>(g_scratch_ptr[dev]);
}

// Up to kDescPerLaunch descriptors travel as kernel arguments and are written into the table.
constexpr int kDescPerLaunch = 64;
struct DescBatch {
    TensorDesc d[kDescPerLaunch];
};
__global__ void __launch_bounds__(kDescPerLaunch)
k_table_desc(DescBatch batch, uint32_t count, TensorDesc* __restrict__ desc)
{
    if (threadIdx.x < count) desc[threadIdx.x] = batch.d[threadIdx.x];
}

// tile_first[i] = first tensor whose end lies beyond the start of tile i (T if none), i in [0, tiles]:
// the ends are ascending, so a binary search gives what the host loop of bagua_flatten_plan gives.
__global__ void __launch_bounds__(256)
k_table_tiles(const TensorDesc* __restrict__ desc, uint32_t T, uint32_t* __restrict__ tile_first, size_t tiles)
{
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i > tiles) return;
    const size_t e = i * static_cast<size_t>(kTile);
    uint32_t lo = 0, hi = T;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (desc[mid].dst + desc[mid].numel <= e) lo = mid + 1;
        else hi = mid;
    }
    tile_first[i] = lo;
}

}  // namespace bagua

extern "C" int bagua_bucket_flatten_static(const void* const* src, const size_t* numel, const size_t* dst_offset,
                                           size_t T, float* bucket, size_t bucket_numel, void* stream)
{
    if (!bucket || bucket_numel == 0 || (T && (!src || !numel || !dst_offset))) return BAGUA_ERR_INVALID_ARG;
    if (T > kStaticMaxT || bucket_numel > kStaticMaxNumel) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(bucket)) return BAGUA_ERR_ALIGNMENT;
    size_t prev_end = 0;
    for (size_t t = 0; t < T; ++t) {
        if (numel[t] && !src[t]) return BAGUA_ERR_INVALID_ARG;
        if (dst_offset[t] < prev_end) return BAGUA_ERR_INVALID_ARG;
        if (numel[t] > bucket_numel || dst_offset[t] > bucket_numel - numel[t]) return BAGUA_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(src[t]) & 3u) return BAGUA_ERR_ALIGNMENT;
        prev_end = dst_offset[t] + numel[t];
    }
    {
        // the bucket is written, the tensors are read: none may overlap it
        const uintptr_t blo = reinterpret_cast<uintptr_t>(bucket), bhi = blo + bucket_numel * sizeof(float);
        for (size_t t = 0; t < T; ++t) {
            const uintptr_t lo = reinterpret_cast<uintptr_t>(src[t]), hi = lo + numel[t] * sizeof(float);
            if (numel[t] && lo < bhi && blo < hi) return BAGUA_ERR_INVALID_ARG;
        }
    }
    unsigned char* table = static_scratch_ptr();
    if (!table) return BAGUA_ERR_LAUNCH;
    TensorDesc* desc = reinterpret_cast<TensorDesc*>(table);
    uint32_t* tile_first = reinterpret_cast<uint32_t*>(table + kStaticDescBytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (size_t t0 = 0; t0 < T; t0 += kDescPerLaunch) {
        DescBatch batch{};
        const uint32_t count = static_cast<uint32_t>(std::min<size_t>(kDescPerLaunch, T - t0));
        for (uint32_t i = 0; i < count; ++i)
            batch.d[i] = TensorDesc{static_cast<const float*>(src[t0 + i]), numel[t0 + i], dst_offset[t0 + i]};
        hipLaunchKernelGGL(k_table_desc, dim3(1), dim3(kDescPerLaunch), 0, s, batch, count, desc + t0);
    }
    const size_t tiles = num_tiles(bucket_numel);
    hipLaunchKernelGGL(k_table_tiles, dim3(static_cast<unsigned>((tiles + 1 + 255) / 256)), dim3(256), 0, s, desc,
                       static_cast<uint32_t>(T), tile_first, tiles);
    hipLaunchKernelGGL(k_flatten, dim3(static_cast<unsigned>(tiles * kTileWaves)), dim3(kWave), 0, s, desc, tile_first,
                       static_cast<uint32_t>(T), bucket, bucket_numel);
    return launch_status();
}

extern "C" int bagua_bucket_unflatten_run(const void* workspace, size_t T, const float* bucket, size_t bucket_numel,
                                          void* stream)
{
    if (!workspace || !bucket || bucket_numel == 0) return BAGUA_ERR_INVALID_ARG;
    if (T > 0xfffffff0u || num_tiles(bucket_numel) > kMaxGrid / kTileWaves) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(workspace) || !aligned16(bucket)) return BAGUA_ERR_ALIGNMENT;
    const FlattenPlanView pv = plan_view(workspace, T);
    hipLaunchKernelGGL(k_unflatten, dim3(static_cast<unsigned>(num_tiles(bucket_numel) * kTileWaves)), dim3(kWave), 0,
                       static_cast<hipStream_t>(stream), pv.desc, pv.tile_first, static_cast<uint32_t>(T), bucket, bucket_numel);
    return launch_status();
}
