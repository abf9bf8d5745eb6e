// MinMax-u8 codec kernels: worker-side compress with error feedback, server-side
// decompress-average-recompress, and plain decompress (C_LP_S, Section 3.2 of the paper).
//
// All three are single-pass streaming kernels bound by HBM bandwidth: a chunk lives in
// registers between the statistics phase and the quantisation phase.
#include "batch.hpp"
#include "launchers.hpp"
#include "minmax_device.hpp"

#pragma clang fp contract(off)

namespace bagua {

// ------------------------------------------------------------------------------------------
// Worker side: v = x (+ residual); codes = Q(v); residual <- v - decode.
// One workgroup per chunk, block = 64 * ceil(rows / RPW); c = index of the chunk in its bucket.
template <int RPW, bool EF>
__device__ __forceinline__ void compress_minmax_chunk(const float* __restrict__ x, float* __restrict__ residual, size_t n,
                                                      uint32_t chunk, uint8_t* __restrict__ codes,
                                                      float* __restrict__ minmax, size_t c, float* s_red, int pace)
{
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    f4 v[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (remain > 0) v[i] = load_row(x + base + off, lane, remain, 0.0f);
        if (pace) pace_loads();
    }
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            if (remain > 0) {
                const f4 d = load_row(residual + base + off, lane, remain, 0.0f);
                if (pace) pace_loads();
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

template <int RPW, bool EF>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_compress_minmax(const float* __restrict__ x, float* __restrict__ residual, size_t n, uint32_t chunk,
                  uint8_t* __restrict__ codes, float* __restrict__ minmax, int pace)
{
    __shared__ float s_red[2 * kMaxWaves];
    compress_minmax_chunk<RPW, EF>(x, residual, n, chunk, codes, minmax, blockIdx.x, s_red, pace);
}

// Batched: entry = [x, residual, codes, minmax, n]; unit = chunk.
template <int RPW, bool EF>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_compress_minmax_batched(BatchView bv, uint32_t chunk, int pace)
{
    __shared__ float s_red[2 * kMaxWaves];
    const uint32_t b = batch_find(bv, blockIdx.x);
    const uint64_t* e = bv.entries + static_cast<size_t>(b) * bv.entry_words;
    compress_minmax_chunk<RPW, EF>(table_ptr<const float>(e[0]), table_ptr<float>(e[1]), e[4], chunk,
                                   table_ptr<uint8_t>(e[2]), table_ptr<float>(e[3]),
                                   blockIdx.x - bv.first_unit[b], s_red, pace);
}

// ------------------------------------------------------------------------------------------
// Server side: a = (sum_j decode_j) * inv_k in ascending j; w = a (+ epsilon); then as above.
// SRC names the workers' inputs: code(j) -> u8 codes of worker j, meta(j) -> its (min, max) pairs.
struct DrrTableSrc {   // pointers in the kernel arguments
    const PtrTable& codes;
    const PtrTable& metas;
    __device__ __forceinline__ const void* code(int j) const { return codes.p[j]; }
    __device__ __forceinline__ const float* meta(int j) const { return static_cast<const float*>(metas.p[j]); }
};
struct DrrEntrySrc {   // pointers in a batch entry: [eps, codes_out, meta_out, out, n, code[0..k), meta[0..k)]
    const uint64_t* e;
    int k;
    __device__ __forceinline__ const void* code(int j) const { return table_ptr<const void>(e[5 + j]); }
    __device__ __forceinline__ const float* meta(int j) const { return table_ptr<const float>(e[5 + k + j]); }
};

template <int RPW, bool EF, bool OUT, typename SRC>
__device__ __forceinline__ void drr_minmax_chunk(const SRC& src, int k, float inv_k, float* __restrict__ eps, size_t n,
                                                 uint32_t chunk, uint8_t* __restrict__ codes_out,
                                                 float* __restrict__ minmax_out, float* __restrict__ out, size_t c,
                                                 float* s_red, float* s_mn, float* s_step)
{
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    // per-worker (min, step) of this chunk: one lane per worker, so the k divisions run side by side
    if (static_cast<int>(threadIdx.x) < k) {
        const float* m = src.meta(threadIdx.x);
        const float mn = m[2 * c], mx = m[2 * c + 1];
        s_mn[threadIdx.x] = mn;
        s_step[threadIdx.x] = minmax_step(mn, mx);
    }
    __syncthreads();

    f4 v[RPW];
    // Workers are summed in ascending order; the code loads of NJ workers are issued together so
    // that NJ*RPW dword loads are in flight per wave before the first is consumed.
    constexpr int NJ = BAGUA_DRR_NJ;
    auto accumulate = [&](int j, uint32_t (&w)[RPW]) {
        const float mn = s_mn[j], step = s_step[j];
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            f4 d;
            d.x = mn + byte_to_float(w[i], 0) * step;
            d.y = mn + byte_to_float(w[i], 1) * step;
            d.z = mn + byte_to_float(w[i], 2) * step;
            d.w = mn + byte_to_float(w[i], 3) * step;
            if (j == 0) {
                v[i] = d;
            } else {
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    };
    auto fetch = [&](int j, uint32_t (&w)[RPW]) {
        const uint8_t* cj = static_cast<const uint8_t*>(src.code(j)) + base;
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            w[i] = 0;
            if (remain > 0) w[i] = load_codes_row(cj + off, lane, remain);
        }
    };
    int j = 0;
    for (; j + NJ <= k; j += NJ) {
        uint32_t w[NJ][RPW];
#pragma unroll
        for (int u = 0; u < NJ; ++u) fetch(j + u, w[u]);
#pragma unroll
        for (int u = 0; u < NJ; ++u) accumulate(j + u, w[u]);
    }
    for (; j < k; ++j) {
        uint32_t w[RPW];
        fetch(j, w);
        accumulate(j, w);
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
                const f4 d = load_row(eps + base + off, lane, remain, 0.0f);
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    }
    minmax_encode_chunk<RPW, EF, OUT>(v, len, wave, lane, nwaves, EF ? eps + base : nullptr,
                                      codes_out + base, minmax_out + 2 * c, OUT ? out + base : nullptr, s_red);
}

template <int RPW, bool EF, bool OUT>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_drr_minmax(PtrTable codes_in, PtrTable meta_in, int k, float inv_k, float* __restrict__ eps, size_t n,
             uint32_t chunk, uint8_t* __restrict__ codes_out, float* __restrict__ minmax_out,
             float* __restrict__ out)
{
    __shared__ float s_red[2 * kMaxWaves];
    __shared__ float s_mn[BAGUA_MAX_WORKERS], s_step[BAGUA_MAX_WORKERS];
    drr_minmax_chunk<RPW, EF, OUT>(DrrTableSrc{codes_in, meta_in}, k, inv_k, eps, n, chunk, codes_out, minmax_out, out,
                                   blockIdx.x, s_red, s_mn, s_step);
}

template <int RPW, bool EF, bool OUT>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_drr_minmax_batched(BatchView bv, int k, float inv_k, uint32_t chunk)
{
    __shared__ float s_red[2 * kMaxWaves];
    __shared__ float s_mn[BAGUA_MAX_WORKERS], s_step[BAGUA_MAX_WORKERS];
    const uint32_t b = batch_find(bv, blockIdx.x);
    const uint64_t* e = bv.entries + static_cast<size_t>(b) * bv.entry_words;
    drr_minmax_chunk<RPW, EF, OUT>(DrrEntrySrc{e, k}, k, inv_k, table_ptr<float>(e[0]), e[4], chunk,
                                   table_ptr<uint8_t>(e[1]), table_ptr<float>(e[2]),
                                   table_ptr<float>(e[3]), blockIdx.x - bv.first_unit[b], s_red, s_mn, s_step);
}

// ------------------------------------------------------------------------------------------
// Decode: out = mn + code * step.  One wave per row, 4 rows per workgroup.
__global__ void __launch_bounds__(kWave * kRowWaves)
k_decompress_minmax(const uint8_t* __restrict__ codes, const float* __restrict__ minmax, size_t n,
                    uint32_t chunk, float* __restrict__ out)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const size_t c = e0 / chunk;
    const float mn = minmax[2 * c], step = minmax_step(mn, minmax[2 * c + 1]);
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    const uint32_t w = load_codes_row(codes + e0, lane, remain);
    f4 d;
    d.x = mn + byte_to_float(w, 0) * step;
    d.y = mn + byte_to_float(w, 1) * step;
    d.z = mn + byte_to_float(w, 2) * step;
    d.w = mn + byte_to_float(w, 3) * step;
    store_row(out + e0, lane, remain, d);
}

// ------------------------------------------------------------------------------------------ host
int launch_compress_minmax(const float* x, float* residual, size_t n, size_t chunk, uint8_t* codes,
                           float* minmax, hipStream_t stream)
{
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw_worker(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(num_chunks(n, chunk))), block(64 * ((rows + rpw - 1) / rpw));
    const uint32_t ch = static_cast<uint32_t>(chunk);
    if (residual) {
        BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_compress_minmax<RPW, true>), grid, block, 0, stream, x,
                                                          residual, n, ch, codes, minmax, pace_for(n)))
    } else {
        BAGUA_DISPATCH_RPW_WORKER(rpw, hipLaunchKernelGGL((k_compress_minmax<RPW, false>), grid, block, 0, stream, x,
                                                          residual, n, ch, codes, minmax, pace_for(n)))
    }
    return launch_status();
}

int launch_drr_minmax(const void* const* codes_in, const float* const* meta_in, int k, float* eps, size_t n,
                      size_t chunk, uint8_t* codes_out, float* minmax_out, float* out, hipStream_t stream)
{
    PtrTable ct{}, mt{};
    for (int j = 0; j < k; ++j) {
        ct.p[j] = codes_in[j];
        mt.p[j] = meta_in[j];
    }
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_DRR);
    dim3 grid(static_cast<unsigned>(num_chunks(n, chunk))), block(64 * ((rows + rpw - 1) / rpw));
    const float inv_k = 1.0f / static_cast<float>(k);
    const uint32_t ch = static_cast<uint32_t>(chunk);
#define BAGUA_DRR(EFv, OUTv)                                                                                   \
    BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_drr_minmax<RPW, EFv, OUTv>), grid, block, 0, stream, ct, mt, \
                                               k, inv_k, eps, n, ch, codes_out, minmax_out, out))
    if (eps && out) { BAGUA_DRR(true, true) }
    else if (eps) { BAGUA_DRR(true, false) }
    else if (out) { BAGUA_DRR(false, true) }
    else { BAGUA_DRR(false, false) }
#undef BAGUA_DRR
    return launch_status();
}

int launch_drr_minmax_batched(const void* workspace, size_t B, int k, size_t total_chunks, size_t chunk, bool ef,
                              bool with_out, hipStream_t stream)
{
    const BatchView bv = batch_view(workspace, B, 5 + 2 * static_cast<size_t>(k), total_chunks);
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_DRR);
    dim3 grid(static_cast<unsigned>(total_chunks)), block(64 * ((rows + rpw - 1) / rpw));
    const float inv_k = 1.0f / static_cast<float>(k);
    const uint32_t ch = static_cast<uint32_t>(chunk);
#define BAGUA_DRR(EFv, OUTv)                                                                                       \
    BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_drr_minmax_batched<RPW, EFv, OUTv>), grid, block, 0, stream, bv, \
                                               k, inv_k, ch))
    if (ef && with_out) { BAGUA_DRR(true, true) }
    else if (ef) { BAGUA_DRR(true, false) }
    else if (with_out) { BAGUA_DRR(false, true) }
    else { BAGUA_DRR(false, false) }
#undef BAGUA_DRR
    return launch_status();
}

int launch_decompress_minmax(const uint8_t* codes, const float* minmax, size_t n, size_t chunk, float* out,
                             hipStream_t stream)
{
    const size_t rows = (n + kRow - 1) / kRow;
    dim3 grid(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves)), block(kWave * kRowWaves);
    hipLaunchKernelGGL(k_decompress_minmax, grid, block, 0, stream, codes, minmax, n,
                       static_cast<uint32_t>(chunk), out);
    return launch_status();
}

}  // namespace bagua

using namespace bagua;

extern "C" int bagua_compress_minmax_u8(const float* x, float* residual, size_t n, size_t chunk,
                                        uint8_t* codes, float* minmax, void* stream)
{
    if (!x || !codes || !minmax || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    RangeCheck rc;
    rc.reads(x, n * sizeof(float));
    rc.writes(residual, n * sizeof(float));
    rc.writes(codes, n);
    rc.writes(minmax, 2 * num_chunks(n, chunk) * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(residual) || !aligned16(codes) || !aligned4(minmax)) return BAGUA_ERR_ALIGNMENT;
    return launch_compress_minmax(x, residual, n, chunk, codes, minmax, static_cast<hipStream_t>(stream));
}

extern "C" int bagua_compress_minmax_u8_batched(const float* const* x, float* const* residual, const size_t* n, size_t B,
                                                size_t chunk, uint8_t* const* codes, float* const* minmax,
                                                void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !n || !codes || !minmax || !workspace || B == 0 || B > 0xffffffffu || !chunk_ok(chunk))
        return BAGUA_ERR_INVALID_ARG;
    if (workspace_bytes < bagua_batch_workspace_bytes(B, 0)) return BAGUA_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return BAGUA_ERR_ALIGNMENT;
    const bool ef = residual != nullptr;
    const size_t ew = batch_entry_words_for(0);
    std::vector<uint64_t> table(batch_table_words(B, ew), 0);
    uint64_t* entries = table.data() + batch_first_words(B);
    RangeList rl;
    size_t total = 0;
    for (size_t b = 0; b < B; ++b) {
        if (!x[b] || !codes[b] || !minmax[b] || n[b] == 0 || (ef && !residual[b])) return BAGUA_ERR_INVALID_ARG;
        float* r = ef ? residual[b] : nullptr;
        if (!aligned16(x[b]) || !aligned16(r) || !aligned16(codes[b]) || !aligned4(minmax[b])) return BAGUA_ERR_ALIGNMENT;
        const size_t nc = num_chunks(n[b], chunk);
        rl.reads(x[b], n[b] * sizeof(float));
        rl.writes(r, n[b] * sizeof(float));
        rl.writes(codes[b], n[b]);
        rl.writes(minmax[b], 2 * nc * sizeof(float));
        table[b] = total;
        uint64_t* e = entries + b * ew;
        e[0] = reinterpret_cast<uintptr_t>(x[b]);
        e[1] = reinterpret_cast<uintptr_t>(r);
        e[2] = reinterpret_cast<uintptr_t>(codes[b]);
        e[3] = reinterpret_cast<uintptr_t>(minmax[b]);
        e[4] = n[b];
        total += nc;
    }
    table[B] = total;
    batch_fill_lut(table.data(), B, ew);
    rl.writes(workspace, table.size() * sizeof(uint64_t));
    if (!rl.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (total > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (batch_upload(table.data(), table.size(), static_cast<uint64_t*>(workspace), s) != BAGUA_OK) return BAGUA_ERR_LAUNCH;
    const BatchView bv = batch_view(workspace, B, ew, total);
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(total)), block(64 * ((rows + rpw - 1) / rpw));
    const uint32_t ch = static_cast<uint32_t>(chunk);
    if (ef) {
        BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_compress_minmax_batched<RPW, true>), grid, block, 0, s, bv, ch, pace_for(total * chunk)))
    } else {
        BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_compress_minmax_batched<RPW, false>), grid, block, 0, s, bv, ch, pace_for(total * chunk)))
    }
    return launch_status();
}
