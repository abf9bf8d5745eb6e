// Flatten fused into the worker-side MinMax-u8 compression: the rows of a chunk are gathered
// straight from the layer tensors (through the planned tensor table), so the flattened bucket is
// never written to and re-read from HBM.  Result = bagua_bucket_flatten followed by
// bagua_compress_minmax_u8, bit for bit; traffic = that of the compression alone.
#include "flatten_device.hpp"
#include "launchers.hpp"
#include "minmax_device.hpp"
#include "sign_device.hpp"

#pragma clang fp contract(off)

namespace bagua {

template <int RPW, bool EF, bool WB>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_flatten_compress_minmax(const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ tile_first, uint32_t T,
                          float* __restrict__ residual, size_t n, uint32_t chunk, uint8_t* __restrict__ codes,
                          float* __restrict__ minmax, float* __restrict__ bucket_out)
{
    __shared__ float s_red[2 * kMaxWaves];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    // the error state does not depend on the table lookups: get its loads going first
    f4 d[RPW];
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            d[i] = f4{0.f, 0.f, 0.f, 0.f};
            if (remain > 0) d[i] = load_row(residual + base + off, lane, remain, 0.0f);
        }
    }
    f4 v[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (remain > 0) {
            v[i] = gather_row(desc, tile_first, T, base + off, lane, remain);
            if (WB) store_row(bucket_out + base + off, lane, remain, v[i]);
        }
    }
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            v[i].x = v[i].x + d[i].x;
            v[i].y = v[i].y + d[i].y;
            v[i].z = v[i].z + d[i].z;
            v[i].w = v[i].w + d[i].w;
        }
    }
    minmax_encode_chunk<RPW, EF, false>(v, len, wave, lane, nwaves, EF ? residual + base : nullptr,
                                        codes + base, minmax + 2 * c, nullptr, s_red);
}

// The same gather in front of the 1-bit sign codec: bagua_bucket_flatten followed by bagua_sign_compress_ef.
template <int RPW, bool EF, bool WB>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_flatten_sign_compress(const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ tile_first, uint32_t T,
                        float* __restrict__ residual, size_t n, uint32_t chunk, uint32_t* __restrict__ bits,
                        float* __restrict__ scale, float* __restrict__ bucket_out)
{
    extern __shared__ float s_q[];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    f4 d[RPW];
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            d[i] = f4{0.f, 0.f, 0.f, 0.f};
            if (remain > 0) d[i] = load_row(residual + base + off, lane, remain, 0.0f);
        }
    }
    f4 v[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (remain > 0) {
            v[i] = gather_row(desc, tile_first, T, base + off, lane, remain);
            if (WB) store_row(bucket_out + base + off, lane, remain, v[i]);
        }
    }
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            v[i].x = v[i].x + d[i].x;
            v[i].y = v[i].y + d[i].y;
            v[i].z = v[i].z + d[i].z;
            v[i].w = v[i].w + d[i].w;
        }
    }
    sign_encode_chunk<RPW, EF, false>(v, len, chunk, wave, lane, nwaves, EF ? residual + base : nullptr,
                                      bits + (base >> 5), scale + c, nullptr, s_q);
}

// Intra-node stage of hierarchical C_LP_S (Section 3.5): the k_local workers' uncompressed buckets are
// averaged (ascending order, one multiply by inv_k) and the leader compresses the average with its
// error state.  4*k_local + 9 bytes per element, one pass.
template <int RPW, bool EF>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_reduce_compress_minmax(PtrTable xs, int k_local, float inv_k, float* __restrict__ residual, size_t n, uint32_t chunk,
                         uint8_t* __restrict__ codes, float* __restrict__ minmax)
{
    __shared__ float s_red[2 * kMaxWaves];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    f4 v[RPW];
    for (int j = 0; j < k_local; ++j) {
        const float* xj = static_cast<const float*>(xs.p[j]) + base;
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            f4 d = f4{0.f, 0.f, 0.f, 0.f};
            if (remain > 0) d = load_row(xj + off, lane, remain, 0.0f);
            if (j == 0) {
                v[i] = d;
            } else {
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        v[i].x = v[i].x * inv_k;
        v[i].y = v[i].y * inv_k;
        v[i].z = v[i].z * inv_k;
        v[i].w = v[i].w * inv_k;
    }
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            if (remain > 0) {
                const f4 d = load_row(residual + base + off, lane, remain, 0.0f);
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    }
    minmax_encode_chunk<RPW, EF, false>(v, len, wave, lane, nwaves, EF ? residual + base : nullptr,
                                        codes + base, minmax + 2 * c, nullptr, s_red);
}

// The same intra-node stage in front of the 1-bit sign codec.
template <int RPW, bool EF>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_reduce_compress_sign(PtrTable xs, int k_local, float inv_k, float* __restrict__ residual, size_t n, uint32_t chunk,
                       uint32_t* __restrict__ bits, float* __restrict__ scale)
{
    extern __shared__ float s_q[];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    f4 v[RPW];
    for (int j = 0; j < k_local; ++j) {
        const float* xj = static_cast<const float*>(xs.p[j]) + base;
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            f4 d = f4{0.f, 0.f, 0.f, 0.f};
            if (remain > 0) d = load_row(xj + off, lane, remain, 0.0f);
            if (j == 0) {
                v[i] = d;
            } else {
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        v[i].x = v[i].x * inv_k;
        v[i].y = v[i].y * inv_k;
        v[i].z = v[i].z * inv_k;
        v[i].w = v[i].w * inv_k;
    }
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            if (remain > 0) {
                const f4 d = load_row(residual + base + off, lane, remain, 0.0f);
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    }
    sign_encode_chunk<RPW, EF, false>(v, len, chunk, wave, lane, nwaves, EF ? residual + base : nullptr,
                                      bits + (base >> 5), scale + c, nullptr, s_q);
}

}  // namespace bagua

using namespace bagua;

extern "C" int bagua_flatten_compress_minmax_u8(const void* workspace, size_t T, float* residual, size_t bucket_numel,
                                                size_t chunk, uint8_t* codes, float* minmax, float* bucket_out,
                                                void* stream)
{
    if (!workspace || !codes || !minmax || bucket_numel == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    RangeCheck rc;
    rc.writes(residual, bucket_numel * sizeof(float));
    rc.writes(codes, bucket_numel);
    rc.writes(minmax, 2 * num_chunks(bucket_numel, chunk) * sizeof(float));
    rc.writes(bucket_out, bucket_numel * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (T > 0xfffffff0u || num_chunks(bucket_numel, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(workspace) || !aligned16(residual) || !aligned16(codes) || !aligned4(minmax) ||
        !aligned16(bucket_out))
        return BAGUA_ERR_ALIGNMENT;
    const FlattenPlanView pv = plan_view(workspace, T);
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw_worker(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(num_chunks(bucket_numel, chunk))), block(64 * ((rows + rpw - 1) / rpw));
    const uint32_t ch = static_cast<uint32_t>(chunk), t32 = static_cast<uint32_t>(T);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define BAGUA_FC(EFv, WBv)                                                                                       \
    BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_flatten_compress_minmax<RPW, EFv, WBv>), grid, block, 0, s,    \
                                               pv.desc, pv.tile_first, t32, residual, bucket_numel, ch, codes,  \
                                               minmax, bucket_out))
    if (residual && bucket_out) { BAGUA_FC(true, true) }
    else if (residual) { BAGUA_FC(true, false) }
    else if (bucket_out) { BAGUA_FC(false, true) }
    else { BAGUA_FC(false, false) }
#undef BAGUA_FC
    return launch_status();
}

extern "C" int bagua_flatten_sign_compress_ef(const void* workspace, size_t T, float* residual, size_t bucket_numel,
                                              size_t chunk, uint32_t* bits, float* scale, float* bucket_out,
                                              void* stream)
{
    if (!workspace || !bits || !scale || bucket_numel == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    RangeCheck rc;
    rc.writes(residual, bucket_numel * sizeof(float));
    rc.writes(bits, ((bucket_numel + 31) / 32) * sizeof(uint32_t));
    rc.writes(scale, num_chunks(bucket_numel, chunk) * sizeof(float));
    rc.writes(bucket_out, bucket_numel * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (T > 0xfffffff0u || num_chunks(bucket_numel, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(workspace) || !aligned16(residual) || !aligned16(bits) || !aligned4(scale) || !aligned16(bucket_out))
        return BAGUA_ERR_ALIGNMENT;
    const FlattenPlanView pv = plan_view(workspace, T);
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw_worker(rows, BAGUA_RPW_SIGN);
    const int waves = (rows + rpw - 1) / rpw;
    dim3 grid(static_cast<unsigned>(num_chunks(bucket_numel, chunk))), block(64 * waves);
    const size_t lds = waves > 1 ? static_cast<size_t>(rows) * kWave * sizeof(float) : 0;
    const uint32_t ch = static_cast<uint32_t>(chunk), t32 = static_cast<uint32_t>(T);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define BAGUA_FS(EFv, WBv)                                                                                       \
    BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_flatten_sign_compress<RPW, EFv, WBv>), grid, block, lds, s,    \
                                               pv.desc, pv.tile_first, t32, residual, bucket_numel, ch, bits,   \
                                               scale, bucket_out))
    if (residual && bucket_out) { BAGUA_FS(true, true) }
    else if (residual) { BAGUA_FS(true, false) }
    else if (bucket_out) { BAGUA_FS(false, true) }
    else { BAGUA_FS(false, false) }
#undef BAGUA_FS
    return launch_status();
}

extern "C" int bagua_reduce_compress_minmax_u8(const float* const* x, int k_local, float* residual, size_t n,
                                               size_t chunk, uint8_t* codes, float* minmax, void* stream)
{
    if (!x || k_local < 1 || k_local > BAGUA_MAX_WORKERS || !codes || !minmax || n == 0 || !chunk_ok(chunk))
        return BAGUA_ERR_INVALID_ARG;
    RangeCheck rc;
    for (int j = 0; j < k_local; ++j) {
        if (!x[j]) return BAGUA_ERR_INVALID_ARG;
        rc.reads(x[j], n * sizeof(float));
    }
    rc.writes(residual, n * sizeof(float));
    rc.writes(codes, n);
    rc.writes(minmax, 2 * num_chunks(n, chunk) * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    for (int j = 0; j < k_local; ++j)
        if (!aligned16(x[j])) return BAGUA_ERR_ALIGNMENT;
    if (!aligned16(residual) || !aligned16(codes) || !aligned4(minmax)) return BAGUA_ERR_ALIGNMENT;
    PtrTable xt{};
    for (int j = 0; j < k_local; ++j) xt.p[j] = x[j];
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw_worker(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(num_chunks(n, chunk))), block(64 * ((rows + rpw - 1) / rpw));
    const float inv_k = 1.0f / static_cast<float>(k_local);
    const uint32_t ch = static_cast<uint32_t>(chunk);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (residual) {
        BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_reduce_compress_minmax<RPW, true>), grid, block, 0, s, xt, k_local,
                                                   inv_k, residual, n, ch, codes, minmax))
    } else {
        BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_reduce_compress_minmax<RPW, false>), grid, block, 0, s, xt, k_local,
                                                   inv_k, residual, n, ch, codes, minmax))
    }
    return launch_status();
}

extern "C" int bagua_reduce_compress_sign_ef(const float* const* x, int k_local, float* residual, size_t n, size_t chunk,
                                             uint32_t* bits, float* scale, void* stream)
{
    if (!x || k_local < 1 || k_local > BAGUA_MAX_WORKERS || !bits || !scale || n == 0 || !chunk_ok(chunk))
        return BAGUA_ERR_INVALID_ARG;
    RangeCheck rc;
    for (int j = 0; j < k_local; ++j) {
        if (!x[j]) return BAGUA_ERR_INVALID_ARG;
        rc.reads(x[j], n * sizeof(float));
    }
    rc.writes(residual, n * sizeof(float));
    rc.writes(bits, ((n + 31) / 32) * sizeof(uint32_t));
    rc.writes(scale, num_chunks(n, chunk) * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    for (int j = 0; j < k_local; ++j)
        if (!aligned16(x[j])) return BAGUA_ERR_ALIGNMENT;
    if (!aligned16(residual) || !aligned16(bits) || !aligned4(scale)) return BAGUA_ERR_ALIGNMENT;
    PtrTable xt{};
    for (int j = 0; j < k_local; ++j) xt.p[j] = x[j];
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw_worker(rows, BAGUA_RPW_SIGN);
    const int waves = (rows + rpw - 1) / rpw;
    dim3 grid(static_cast<unsigned>(num_chunks(n, chunk))), block(64 * waves);
    const size_t lds = waves > 1 ? static_cast<size_t>(rows) * kWave * sizeof(float) : 0;
    const float inv_k = 1.0f / static_cast<float>(k_local);
    const uint32_t ch = static_cast<uint32_t>(chunk);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (residual) {
        BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_reduce_compress_sign<RPW, true>), grid, block, lds, s, xt, k_local,
                                                   inv_k, residual, n, ch, bits, scale))
    } else {
        BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_reduce_compress_sign<RPW, false>), grid, block, lds, s, xt, k_local,
                                                   inv_k, residual, n, ch, bits, scale))
    }
    return launch_status();
}
