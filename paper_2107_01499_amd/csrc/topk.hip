// Per-chunk top-K sparsification as a third compression function Q of C_LP_S (the aggressive
// compression the paper names when it motivates error compensation, Section 3.2): worker-side
// compress with error feedback, server-side decompress-average-recompress, and decompress.
//
// Selection of the K largest |v| of a chunk (ties: lower index) without sorting: the chunk stays in
// registers; a 4-pass radix select over the IEEE bit pattern of |v| (256-bin histograms in LDS,
// integer atomics only, so the result does not depend on execution order) finds the K-th largest
// magnitude T and how many elements equal to T are still needed; one packed prefix count in index
// order (DPP scans on the vector ALU + one LDS exchange between waves) then gives every kept element
// its output slot.  The first digit is the sign-stripped exponent, which takes only a handful of
// values inside a chunk: its counters are replicated 16 times, interleaved over the LDS banks, so that
// equal digits from the lanes of one wave do not serialise on one address.
#include "launchers.hpp"

#pragma clang fp contract(off)

namespace bagua {

#ifndef BAGUA_TOPK_COPIES
#define BAGUA_TOPK_COPIES 16
#endif
constexpr int kCopies = BAGUA_TOPK_COPIES;  // interleaved copies of the first-pass histogram (spreads equal digits over banks)
constexpr int kTopkLdsWords = 256 * kCopies + 4 * 256 + kMaxWaves;

__device__ __forceinline__ uint32_t mag_key(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// Inclusive prefix sum over the 64 lanes on the vector ALU only: DPP row shifts inside each row of
// 16 lanes, then the totals of the lower rows are added from lanes 15, 31 and 47.
__device__ __forceinline__ uint32_t wave_prefix_incl(uint32_t x, int lane)
{
    x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x111, 0xf, 0xf, true));  // row_shr:1
    x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x112, 0xf, 0xf, true));  // row_shr:2
    x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x114, 0xf, 0xf, true));  // row_shr:4
    x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x118, 0xf, 0xf, true));  // row_shr:8
    const uint32_t t0 = __builtin_amdgcn_readlane(static_cast<int>(x), 15);
    const uint32_t t1 = __builtin_amdgcn_readlane(static_cast<int>(x), 31);
    const uint32_t t2 = __builtin_amdgcn_readlane(static_cast<int>(x), 47);
    const int row = lane >> 4;
    return x + (row >= 1 ? t0 : 0u) + (row >= 2 ? t1 : 0u) + (row >= 3 ? t2 : 0u);
}

// All lanes of a wave: D = largest digit whose suffix count sum_{d >= D} h[d] reaches `need`,
// above = sum_{d > D} h[d].  Requires 1 <= need <= sum of all bins.
__device__ __forceinline__ void find_digit(const uint32_t* h, int lane, uint32_t need, uint32_t& D, uint32_t& above)
{
    const uint4 hb = *reinterpret_cast<const uint4*>(h + 4 * lane);
    const uint32_t c = hb.x + hb.y + hb.z + hb.w;
    const uint32_t pre = wave_prefix_incl(c, lane);
    const uint32_t total = __builtin_amdgcn_readlane(static_cast<int>(pre), 63);
    const uint32_t suffix = total - pre + c;             // sum over lanes >= this one
    const unsigned long long ok = __ballot(suffix >= need);  // lanes 0..L (suffix sums do not increase with the lane)
    const int L = 63 - __builtin_clzll(ok);
    uint32_t t = __builtin_amdgcn_readlane(static_cast<int>(suffix - c), L);  // everything above lane L's four bins
    const uint32_t b3 = __builtin_amdgcn_readlane(static_cast<int>(hb.w), L);
    const uint32_t b2 = __builtin_amdgcn_readlane(static_cast<int>(hb.z), L);
    const uint32_t b1 = __builtin_amdgcn_readlane(static_cast<int>(hb.y), L);
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

// Zero the histograms (128-bit LDS stores) and synchronise.  Called while the chunk's global loads are
// still in flight, so the clear costs no extra latency.
__device__ __forceinline__ void topk_clear_lds(uint32_t* smem)
{
    static_assert((256 * kCopies + 4 * 256) % 4 == 0, "histogram words come in groups of four");
    uint4* q = reinterpret_cast<uint4*>(smem);
    for (int t = threadIdx.x; t < (256 * kCopies + 4 * 256) / 4; t += blockDim.x) q[t] = uint4{0u, 0u, 0u, 0u};
    __syncthreads();
}

// Encode the chunk held in v (absent elements are ignored).  idx_c/val_c point at the chunk's `keep`
// output slots, residual/out at the chunk's first element (nullptr = not wanted).
// smem: kTopkLdsWords words of LDS, cleared by topk_clear_lds (all waves must have passed its barrier).
// FULL: every row of every wave of the workgroup is complete (len == RPW * 256 * nwaves), so no element needs a validity
// test.
template <int RPW, bool FULL>
__device__ __forceinline__ void topk_encode_rows(const f4 (&v)[RPW], int len, uint32_t keep, int wave, int lane,
                                                  int nwaves, float* __restrict__ residual,
                                                  uint16_t* __restrict__ idx_c, float* __restrict__ val_c,
                                                  float* __restrict__ out, uint32_t* smem)
{
    uint32_t* copies = smem;                  // [256][kCopies], first pass only
    uint32_t* hist = smem + 256 * kCopies;    // [4][256]
    uint32_t* tot = hist + 4 * 256;
    const uint32_t keff = (static_cast<int>(keep) < len) ? keep : static_cast<uint32_t>(len);

    uint32_t key[RPW][4];
    bool valid[RPW][4];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int e0 = static_cast<int>(wave * RPW + i) * kRow + lane * 4;
        const float el[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            key[i][e] = mag_key(el[e]);
            valid[i][e] = FULL || e0 + e < len;
        }
    }

    // ---- radix select: threshold key T and the number R of elements equal to T that are kept.
    // First digit (sign-stripped exponent): values of one chunk share a handful of exponents, so equal
    // digits are spread over kCopies interleaved counters to keep the LDS atomics from serialising.
    uint32_t prefix = 0, need = keff;
#pragma unroll
    for (int i = 0; i < RPW; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (valid[i][e]) atomicAdd(&copies[(key[i][e] >> 24) * kCopies + (lane & (kCopies - 1))], 1u);
    __syncthreads();
    for (int b = threadIdx.x; b < 256; b += blockDim.x) {
        uint32_t sum = 0;
#pragma unroll
        for (int q = 0; q < kCopies; q += 4) {
            const uint4 part = *reinterpret_cast<const uint4*>(copies + b * kCopies + q);
            sum += part.x + part.y + part.z + part.w;
        }
        hist[b] = sum;
    }
    __syncthreads();
    {
        uint32_t D, above;
        find_digit(hist, lane, need, D, above);
        need -= above;
        prefix = D << 24;
    }
#pragma unroll
    for (int pass = 1; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        const uint32_t himask = 0xffffffffu << (shift + 8);
        bool cand[RPW][4];
        bool any = false;
#pragma unroll
        for (int i = 0; i < RPW; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                cand[i][e] = valid[i][e] && (key[i][e] & himask) == prefix;
                any = any || cand[i][e];
            }
        if (__ballot(any) != 0) {  // after the first pass most waves hold no candidate at all
#pragma unroll
            for (int i = 0; i < RPW; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (cand[i][e]) atomicAdd(&hist[pass * 256 + ((key[i][e] >> shift) & 255u)], 1u);
        }
        __syncthreads();
        uint32_t D, above;
        find_digit(hist + pass * 256, lane, need, D, above);
        need -= above;
        prefix |= D << shift;
    }
    const uint32_t T = prefix, R = need;

    // ---- packed prefix counts in index order: low half = elements > T, high half = elements == T
    uint32_t lane_excl[RPW];
    uint32_t run = 0;
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        uint32_t c = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (valid[i][e]) c += (key[i][e] > T ? 1u : 0u) + (key[i][e] == T ? 0x10000u : 0u);
        const uint32_t inc = wave_prefix_incl(c, lane);
        lane_excl[i] = run + inc - c;
        run += __builtin_amdgcn_readlane(static_cast<int>(inc), 63);
    }
    if (lane == 0) tot[wave] = run;
    __syncthreads();
    uint32_t before_wave = 0;
    for (int w = 0; w < wave; ++w) before_wave += tot[w];

    // ---- emit
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        if (remain <= 0) continue;
        const int e0 = off + lane * 4;
        const float el[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        float res[4], dec[4];
        uint32_t before = before_wave + lane_excl[i];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t bgt = before & 0xffffu, beq = before >> 16;
            const bool gt = valid[i][e] && key[i][e] > T, eq = valid[i][e] && key[i][e] == T;
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

template <int RPW>
__device__ __forceinline__ void topk_encode_chunk(const f4 (&v)[RPW], int len, uint32_t keep, int wave, int lane,
                                                  int nwaves, float* __restrict__ residual,
                                                  uint16_t* __restrict__ idx_c, float* __restrict__ val_c,
                                                  float* __restrict__ out, uint32_t* smem)
{
    // the same branch for every wave of the workgroup (the barriers inside are reached by all of them either way)
    if (len == RPW * kRow * nwaves) topk_encode_rows<RPW, true>(v, len, keep, wave, lane, nwaves, residual, idx_c, val_c, out, smem);
    else topk_encode_rows<RPW, false>(v, len, keep, wave, lane, nwaves, residual, idx_c, val_c, out, smem);
}

// ------------------------------------------------------------------------------------------ worker side
template <int RPW, bool EF>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_compress_topk(const float* __restrict__ x, float* __restrict__ residual, size_t n, uint32_t chunk, uint32_t keep,
                uint16_t* __restrict__ idx, float* __restrict__ val)
{
    extern __shared__ uint32_t smem[];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    f4 v[RPW], d[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        d[i] = v[i];
        if (remain > 0) {
            v[i] = load_row(x + base + off, lane, remain, 0.0f);
            if (EF) d[i] = load_row(residual + base + off, lane, remain, 0.0f);
        }
    }
    topk_clear_lds(smem);
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            v[i].x = v[i].x + d[i].x;
            v[i].y = v[i].y + d[i].y;
            v[i].z = v[i].z + d[i].z;
            v[i].w = v[i].w + d[i].w;
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
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_drr_topk(PtrTable idx_in, PtrTable val_in, int k, float inv_k, uint32_t keep, float* __restrict__ eps, size_t n,
           uint32_t chunk, uint16_t* __restrict__ idx_out, float* __restrict__ val_out, float* __restrict__ out)
{
    extern __shared__ uint32_t smem[];
    float* dense = reinterpret_cast<float*>(smem);
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    // The error state of this wave's rows is requested first: it is not needed before the sparse sums are done.
    f4 e[RPW];
    if (EF) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            e[i] = f4{0.f, 0.f, 0.f, 0.f};
            if (remain > 0) e[i] = load_row(eps + base + off, lane, remain, 0.0f);
        }
    }
    for (uint32_t t = threadIdx.x; t < chunk / 4; t += blockDim.x) reinterpret_cast<f4*>(dense)[t] = f4{0.f, 0.f, 0.f, 0.f};
    if (keep <= blockDim.x) {
        // one entry per thread and worker: the entries of up to eight workers are fetched together, so the
        // chain of k dependent steps pays one memory latency per group instead of one per worker
        constexpr int G = 8;
        const uint32_t t = threadIdx.x;
        for (int j0 = 0; j0 < k; j0 += G) {
            uint32_t p[G];
            float a[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                p[g] = 0xFFFFu;
                a[g] = 0.0f;
                if (j0 + g < k && t < keep) {
                    p[g] = static_cast<const uint16_t*>(idx_in.p[j0 + g])[c * keep + t];
                    a[g] = static_cast<const float*>(val_in.p[j0 + g])[c * keep + t];
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (j0 + g >= k) break;
                __syncthreads();  // the previous worker's sums (or the clear) are complete
                if (static_cast<int>(p[g]) < len) dense[p[g]] = dense[p[g]] + a[g];
            }
        }
        __syncthreads();
    } else {
        __syncthreads();
        for (int j = 0; j < k; ++j) {
            const uint16_t* ij = static_cast<const uint16_t*>(idx_in.p[j]) + c * keep;
            const float* vj = static_cast<const float*>(val_in.p[j]) + c * keep;
            for (uint32_t t = threadIdx.x; t < keep; t += blockDim.x) {
                const uint32_t p = ij[t];
                if (static_cast<int>(p) < len) dense[p] = dense[p] + vj[t];
            }
            __syncthreads();
        }
    }
    f4 v[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (remain > 0) {
            const f4 a = *reinterpret_cast<const f4*>(dense + off + lane * 4);
            v[i].x = a.x * inv_k;
            v[i].y = a.y * inv_k;
            v[i].z = a.z * inv_k;
            v[i].w = a.w * inv_k;
            if (EF) {
                v[i].x = v[i].x + e[i].x;
                v[i].y = v[i].y + e[i].y;
                v[i].z = v[i].z + e[i].z;
                v[i].w = v[i].w + e[i].w;
            }
        }
    }
    __syncthreads();  // the dense copy is dead: its LDS is reused by the selection
    topk_clear_lds(smem);
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
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    for (uint32_t t = threadIdx.x; t < chunk; t += blockDim.x) dense[t] = 0.0f;
    __syncthreads();
    for (uint32_t t = threadIdx.x; t < keep; t += blockDim.x) {
        const uint32_t p = idx[c * keep + t];
        if (static_cast<int>(p) < len) dense[p] = val[c * keep + t];
    }
    __syncthreads();
    const int wave = wave_index(), lane = threadIdx.x & 63;
    for (int off = static_cast<int>(wave) * kRow; off < len; off += 4 * kRow)
        store_row(out + base + off, lane, len - off, *reinterpret_cast<const f4*>(dense + off + lane * 4));
}

}  // namespace bagua

using namespace bagua;

static bool topk_args_ok(size_t n, size_t chunk, size_t keep) { return n != 0 && chunk_ok(chunk) && keep >= 1 && keep <= chunk; }

extern "C" int bagua_compress_topk_ef(const float* x, float* residual, size_t n, size_t chunk, size_t keep,
                                      uint16_t* idx, float* val, void* stream)
{
    if (!x || !idx || !val || !topk_args_ok(n, chunk, keep)) return BAGUA_ERR_INVALID_ARG;
    {
        const size_t slots = num_chunks(n, chunk) * keep;
        RangeCheck rc;
        rc.reads(x, n * sizeof(float));
        rc.writes(residual, n * sizeof(float));
        rc.writes(idx, slots * sizeof(uint16_t));
        rc.writes(val, slots * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(residual) || !aligned2(idx) || !aligned4(val)) return BAGUA_ERR_ALIGNMENT;
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_TOPK);
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
    {
        const size_t slots = num_chunks(n, chunk) * keep;
        RangeCheck rc;
        for (int j = 0; j < k; ++j) {
            if (!idx_in[j] || !val_in[j]) return BAGUA_ERR_INVALID_ARG;
            rc.reads(idx_in[j], slots * sizeof(uint16_t));
            rc.reads(val_in[j], slots * sizeof(float));
        }
        rc.writes(server_residual, n * sizeof(float));
        rc.writes(idx_out, slots * sizeof(uint16_t));
        rc.writes(val_out, slots * sizeof(float));
        rc.writes(out_fp32, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    for (int j = 0; j < k; ++j)
        if (!aligned2(idx_in[j]) || !aligned4(val_in[j])) return BAGUA_ERR_ALIGNMENT;
    if (!aligned16(server_residual) || !aligned2(idx_out) || !aligned4(val_out) || !aligned16(out_fp32))
        return BAGUA_ERR_ALIGNMENT;
    PtrTable it{}, vt{};
    for (int j = 0; j < k; ++j) {
        it.p[j] = idx_in[j];
        vt.p[j] = val_in[j];
    }
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_DRR_TOPK);
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
    {
        const size_t slots = num_chunks(n, chunk) * keep;
        RangeCheck rc;
        rc.reads(idx, slots * sizeof(uint16_t));
        rc.reads(val, slots * sizeof(float));
        rc.writes(out, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned2(idx) || !aligned4(val) || !aligned16(out)) return BAGUA_ERR_ALIGNMENT;
    hipLaunchKernelGGL(k_decompress_topk, dim3(static_cast<unsigned>(num_chunks(n, chunk))), dim3(256),
                       chunk * sizeof(float), static_cast<hipStream_t>(stream), idx, val, n, static_cast<uint32_t>(chunk),
                       static_cast<uint32_t>(keep), out);
    return launch_status();
}
