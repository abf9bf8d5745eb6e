// Per-chunk top-K sparsification as a third compression function Q of C_LP_S (the aggressive
// compression the paper names when it motivates error compensation, Section 3.2): worker-side
// compress with error feedback, server-side decompress-average-recompress, and decompress.
//
// Selection of the K largest |v| of a chunk (ties: lower index) without sorting: the chunk stays in
// registers; a 4-pass radix select over the IEEE bit pattern of |v| (256-bin histograms in LDS,
// integer atomics only, so the result does not depend on execution order) finds the K-th largest
// magnitude T and how many elements equal to T are still needed; one packed prefix count in index
// order (wave shuffles + one LDS exchange) then gives every kept element its output slot.
#include "launchers.hpp"

#pragma clang fp contract(off)

namespace bagua {

constexpr int kTopkLdsWords = 4 * 256 + kMaxWaves;  // four histograms + per-wave totals

__device__ __forceinline__ uint32_t mag_key(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// All lanes of a wave: D = largest digit whose suffix count sum_{d >= D} h[d] reaches `need`,
// above = sum_{d > D} h[d].  Requires 1 <= need <= sum of all bins.
__device__ __forceinline__ void find_digit(const uint32_t* h, int lane, uint32_t need, uint32_t& D, uint32_t& above)
{
    const uint32_t h0 = h[4 * lane], h1 = h[4 * lane + 1], h2 = h[4 * lane + 2], h3 = h[4 * lane + 3];
    const uint32_t c = h0 + h1 + h2 + h3;
    uint32_t s = c;  // inclusive suffix sum over lanes
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t t = __shfl_down(s, d, kWave);
        if (lane + d < kWave) s += t;
    }
    const unsigned long long ok = __ballot(s >= need);  // lanes 0..L (suffix sums do not increase with the lane)
    const int L = 63 - __builtin_clzll(ok);
    uint32_t t = __shfl(s, L, kWave) - __shfl(c, L, kWave);  // everything above lane L's four bins
    const uint32_t b3 = __shfl(h3, L, kWave), b2 = __shfl(h2, L, kWave), b1 = __shfl(h1, L, kWave);
    if (t + b3 >= need) {
        D = 4 * L + 3;
    } else {
        t += b3;
        if (t + b2 >= need) {
            D = 4 * L + 2;
        } else {
            t += b2;
            if (t + b1 >= need) {
                D = 4 * L + 1;
            } else {
                t += b1;
                D = 4 * L;
            }
        }
    }
    above = t;
}

// Encode the chunk held in v (absent elements are ignored).  idx_c/val_c point at the chunk's `keep`
// output slots, residual/out at the chunk's first element (nullptr = not wanted).
// smem: kTopkLdsWords words of LDS; the function starts with a barrier-protected clear of it.
template <int RPW>
__device__ __forceinline__ void topk_encode_chunk(const f4 (&v)[RPW], long len, uint32_t keep, int wave, int lane,
                                                  int nwaves, float* __restrict__ residual,
                                                  uint16_t* __restrict__ idx_c, float* __restrict__ val_c,
                                                  float* __restrict__ out, uint32_t* smem)
{
    uint32_t* hist = smem;
    uint32_t* tot = smem + 4 * 256;
    const uint32_t keff = (static_cast<long>(keep) < len) ? keep : static_cast<uint32_t>(len);
    for (int t = threadIdx.x; t < 4 * 256; t += blockDim.x) hist[t] = 0;
    __syncthreads();

    // ---- radix select: threshold key T and the number R of elements equal to T that are kept
    uint32_t prefix = 0, need = keff;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        const uint32_t himask = (pass == 0) ? 0u : (0xffffffffu << (shift + 8));
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const long e0 = static_cast<long>(wave * RPW + i) * kRow + lane * 4;
            const float el[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t key = mag_key(el[e]);
                if (e0 + e < len && (key & himask) == prefix) atomicAdd(&hist[pass * 256 + ((key >> shift) & 255u)], 1u);
            }
        }
        __syncthreads();
        uint32_t D, above;
        find_digit(hist + pass * 256, lane, need, D, above);
        need -= above;
        prefix |= D << shift;
    }
    const uint32_t T = prefix, R = need;

    // ---- packed prefix counts in index order: low half = elements > T, high half = elements == T
    uint32_t cnt[RPW], lane_excl[RPW];
    uint32_t run = 0;
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const long e0 = static_cast<long>(wave * RPW + i) * kRow + lane * 4;
        const float el[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        uint32_t c = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t key = mag_key(el[e]);
            if (e0 + e < len) c += (key > T ? 1u : 0u) + (key == T ? 0x10000u : 0u);
        }
        cnt[i] = c;
        uint32_t inc = c;  // inclusive prefix over lanes
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const uint32_t t = __shfl_up(inc, d, kWave);
            if (lane >= d) inc += t;
        }
        lane_excl[i] = run + inc - c;
        run += __shfl(inc, kWave - 1, kWave);
    }
    if (lane == 0) tot[wave] = run;
    __syncthreads();
    uint32_t before_wave = 0;
    for (int w = 0; w < wave; ++w) before_wave += tot[w];

    // ---- emit
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const long off = static_cast<long>(wave * RPW + i) * kRow;
        const long remain = len - off;
        if (remain <= 0) continue;
        const long e0 = off + lane * 4;
        const float el[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        float res[4], dec[4];
        uint32_t before = before_wave + lane_excl[i];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t key = mag_key(el[e]);
            const bool valid = e0 + e < len;
            const uint32_t bgt = before & 0xffffu, beq = before >> 16;
            const bool gt = valid && key > T, eq = valid && key == T;
            const bool sel = gt || (eq && beq < R);
            const float stored = el[e] + 0.0f;  // -0 is stored as +0
            if (sel) {
                const uint32_t pos = bgt + (beq < R ? beq : R);
                idx_c[pos] = static_cast<uint16_t>(e0 + e);
                val_c[pos] = stored;
            }
            res[e] = sel ? 0.0f : el[e];
            dec[e] = sel ? stored : 0.0f;
            before += (gt ? 1u : 0u) + (eq ? 0x10000u : 0u);
        }
        if (residual) store_row(residual + off, lane, remain, f4{res[0], res[1], res[2], res[3]});
        if (out) store_row(out + off, lane, remain, f4{dec[0], dec[1], dec[2], dec[3]});
    }
    for (uint32_t t = keff + threadIdx.x; t < keep; t += blockDim.x) {  // unused slots of a short last chunk
        idx_c[t] = 0xFFFFu;
        val_c[t] = 0.0f;
    }
}

// ------------------------------------------------------------------------------------------ worker side
template <int RPW, bool EF>
__global__ void __launch_bounds__(64 * ((64 + RPW - 1) / RPW))
k_compress_topk(const float* __restrict__ x, float* __restrict__ residual, size_t n, uint32_t chunk, uint32_t keep,
                uint16_t* __restrict__ idx, float* __restrict__ val)
{
    extern __shared__ uint32_t smem[];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const long len = static_cast<long>((n - base < chunk) ? (n - base) : chunk);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    f4 v[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const long off = static_cast<long>(wave * RPW + i) * kRow;
        const long remain = len - off;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (remain > 0) {
            v[i] = load_row(x + base + off, lane, remain, 0.0f);
            if (EF) {
                const f4 d = load_row(residual + base + off, lane, remain, 0.0f);
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    }
    topk_encode_chunk<RPW>(v, len, keep, wave, lane, nwaves, EF ? residual + base : nullptr, idx + c * keep,
                           val + c * keep, nullptr, smem);
}

// ------------------------------------------------------------------------------------------ server side
// The k sparse chunks are summed into a dense LDS copy of the chunk, one worker after the other
// (ascending order; a worker's indices are unique, so its adds never collide), then averaged,
// the server error state is added and the result is sparsified again.
template <int RPW, bool EF, bool OUT>
__global__ void __launch_bounds__(64 * ((64 + RPW - 1) / RPW))
k_drr_topk(PtrTable idx_in, PtrTable val_in, int k, float inv_k, uint32_t keep, float* __restrict__ eps, size_t n,
           uint32_t chunk, uint16_t* __restrict__ idx_out, float* __restrict__ val_out, float* __restrict__ out)
{
    extern __shared__ uint32_t smem[];
    float* dense = reinterpret_cast<float*>(smem);
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const long len = static_cast<long>((n - base < chunk) ? (n - base) : chunk);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    for (uint32_t t = threadIdx.x; t < chunk; t += blockDim.x) dense[t] = 0.0f;
    __syncthreads();
    for (int j = 0; j < k; ++j) {
        const uint16_t* ij = static_cast<const uint16_t*>(idx_in.p[j]) + c * keep;
        const float* vj = static_cast<const float*>(val_in.p[j]) + c * keep;
        for (uint32_t t = threadIdx.x; t < keep; t += blockDim.x) {
            const uint32_t p = ij[t];
            if (static_cast<long>(p) < len) dense[p] = dense[p] + vj[t];
        }
        __syncthreads();
    }
    f4 v[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const long off = static_cast<long>(wave * RPW + i) * kRow;
        const long remain = len - off;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (remain > 0) {
            const f4 a = *reinterpret_cast<const f4*>(dense + off + lane * 4);
            v[i].x = a.x * inv_k;
            v[i].y = a.y * inv_k;
            v[i].z = a.z * inv_k;
            v[i].w = a.w * inv_k;
            if (EF) {
                const f4 d = load_row(eps + base + off, lane, remain, 0.0f);
                v[i].x = v[i].x + d.x;
                v[i].y = v[i].y + d.y;
                v[i].z = v[i].z + d.z;
                v[i].w = v[i].w + d.w;
            }
        }
    }
    __syncthreads();  // the dense copy is dead: its LDS is reused by the selection
    topk_encode_chunk<RPW>(v, len, keep, wave, lane, nwaves, EF ? eps + base : nullptr, idx_out + c * keep,
                           val_out + c * keep, OUT ? out + base : nullptr, smem);
}

// ------------------------------------------------------------------------------------------ decode
// Dense chunk assembled in LDS, written out with coalesced 128-bit stores.
__global__ void __launch_bounds__(256)
k_decompress_topk(const uint16_t* __restrict__ idx, const float* __restrict__ val, size_t n, uint32_t chunk,
                  uint32_t keep, float* __restrict__ out)
{
    extern __shared__ uint32_t smem[];
    float* dense = reinterpret_cast<float*>(smem);
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const long len = static_cast<long>((n - base < chunk) ? (n - base) : chunk);
    for (uint32_t t = threadIdx.x; t < chunk; t += blockDim.x) dense[t] = 0.0f;
    __syncthreads();
    for (uint32_t t = threadIdx.x; t < keep; t += blockDim.x) {
        const uint32_t p = idx[c * keep + t];
        if (static_cast<long>(p) < len) dense[p] = val[c * keep + t];
    }
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (long off = static_cast<long>(wave) * kRow; off < len; off += 4 * kRow)
        store_row(out + base + off, lane, len - off, *reinterpret_cast<const f4*>(dense + off + lane * 4));
}

}  // namespace bagua

using namespace bagua;

static bool topk_args_ok(size_t n, size_t chunk, size_t keep) { return n != 0 && chunk_ok(chunk) && keep >= 1 && keep <= chunk; }

extern "C" int bagua_compress_topk_ef(const float* x, float* residual, size_t n, size_t chunk, size_t keep,
                                      uint16_t* idx, float* val, void* stream)
{
    if (!x || !idx || !val || !topk_args_ok(n, chunk, keep)) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(residual) || !aligned16(idx) || !aligned16(val)) return BAGUA_ERR_ALIGNMENT;
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(num_chunks(n, chunk))), block(64 * ((rows + rpw - 1) / rpw));
    const size_t lds = kTopkLdsWords * sizeof(uint32_t);
    const uint32_t ch = static_cast<uint32_t>(chunk), kp = static_cast<uint32_t>(keep);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (residual) {
        BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_compress_topk<RPW, true>), grid, block, lds, s, x, residual, n, ch, kp,
                                                   idx, val))
    } else {
        BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_compress_topk<RPW, false>), grid, block, lds, s, x, residual, n, ch, kp,
                                                   idx, val))
    }
    return launch_status();
}

extern "C" int bagua_decompress_reduce_recompress_topk(const uint16_t* const* idx_in, const float* const* val_in, int k,
                                                       size_t keep, float* server_residual, size_t n, size_t chunk,
                                                       uint16_t* idx_out, float* val_out, float* out_fp32, void* stream)
{
    if (!idx_in || !val_in || k < 1 || k > BAGUA_MAX_WORKERS || !idx_out || !val_out || !topk_args_ok(n, chunk, keep))
        return BAGUA_ERR_INVALID_ARG;
    for (int j = 0; j < k; ++j) {
        if (!idx_in[j] || !val_in[j] || idx_in[j] == idx_out || val_in[j] == val_out) return BAGUA_ERR_INVALID_ARG;
    }
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    for (int j = 0; j < k; ++j)
        if (!aligned16(idx_in[j]) || !aligned16(val_in[j])) return BAGUA_ERR_ALIGNMENT;
    if (!aligned16(server_residual) || !aligned16(idx_out) || !aligned16(val_out) || !aligned16(out_fp32))
        return BAGUA_ERR_ALIGNMENT;
    PtrTable it{}, vt{};
    for (int j = 0; j < k; ++j) {
        it.p[j] = idx_in[j];
        vt.p[j] = val_in[j];
    }
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(num_chunks(n, chunk))), block(64 * ((rows + rpw - 1) / rpw));
    size_t lds = chunk * sizeof(float);
    if (lds < kTopkLdsWords * sizeof(uint32_t)) lds = kTopkLdsWords * sizeof(uint32_t);
    const float inv_k = 1.0f / static_cast<float>(k);
    const uint32_t ch = static_cast<uint32_t>(chunk), kp = static_cast<uint32_t>(keep);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define BAGUA_DRR(EFv, OUTv)                                                                                      \
    BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_drr_topk<RPW, EFv, OUTv>), grid, block, lds, s, it, vt, k, inv_k, \
                                               kp, server_residual, n, ch, idx_out, val_out, out_fp32))
    if (server_residual && out_fp32) { BAGUA_DRR(true, true) }
    else if (server_residual) { BAGUA_DRR(true, false) }
    else if (out_fp32) { BAGUA_DRR(false, true) }
    else { BAGUA_DRR(false, false) }
#undef BAGUA_DRR
    return launch_status();
}

extern "C" int bagua_decompress_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep,
                                     float* out, void* stream)
{
    if (!idx || !val || !out || !topk_args_ok(n, chunk, keep)) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(idx) || !aligned16(val) || !aligned16(out)) return BAGUA_ERR_ALIGNMENT;
    hipLaunchKernelGGL(k_decompress_topk, dim3(static_cast<unsigned>(num_chunks(n, chunk))), dim3(256),
                       chunk * sizeof(float), static_cast<hipStream_t>(stream), idx, val, n, static_cast<uint32_t>(chunk),
                       static_cast<uint32_t>(keep), out);
    return launch_status();
}
