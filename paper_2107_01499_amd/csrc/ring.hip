// Decentralised averaging on a ring (D_FP_S / D_LP_S, Section 3.2; ring peers, Section 3.4).
//
// Full precision: one thread owns the same four elements of all k replicas, so every replica is
// read once and written once (8 bytes per element per peer) although each output has three inputs.
// Low precision: one workgroup owns one chunk of all k peers.  The per-peer difference is
// quantised, the public copies xhat are advanced and the three-neighbour mix is formed while x and
// the new xhat of every peer are still in registers: 17 bytes per element per peer, one pass.
#include "launchers.hpp"
#include "minmax_device.hpp"

#pragma clang fp contract(off)

namespace bagua {

__device__ __forceinline__ f4 add4(f4 a, f4 b) { return f4{a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w}; }
__device__ __forceinline__ f4 sub4(f4 a, f4 b) { return f4{a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w}; }
__device__ __forceinline__ f4 mul4(f4 a, float s) { return f4{a.x * s, a.y * s, a.z * s, a.w * s}; }

// ------------------------------------------------------------------------------------------ FP
// One wave per 256-element row; K replicas held in registers.  kFpWaves rows per workgroup: measured at 8 peers x
// 110 M elements, 1 and 8 waves per workgroup stream 3-5 % faster than 2, 4 or 16.
#ifndef BAGUA_FP_WAVES
#define BAGUA_FP_WAVES 8
#endif
constexpr int kFpWaves = BAGUA_FP_WAVES;
template <int K>
__global__ void __launch_bounds__(64 * kFpWaves)
k_ring_avg_fp(PtrTable xin, MutPtrTable xout, size_t n, float third)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kFpWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    f4 x[K];
#pragma unroll
    for (int i = 0; i < K; ++i) x[i] = load_row(static_cast<const float*>(xin.p[i]) + e0, lane, remain, 0.0f);
#pragma unroll
    for (int i = 0; i < K; ++i) {
        const f4 s = add4(add4(x[(i + K - 1) % K], x[i]), x[(i + 1) % K]);
        store_row(static_cast<float*>(xout.p[i]) + e0, lane, remain, mul4(s, third));
    }
}

// Any k: rolling window over the peers (fewer loads in flight; used above the templated range).
__global__ void __launch_bounds__(kWave * kRowWaves)
k_ring_avg_fp_any(PtrTable xin, MutPtrTable xout, int k, size_t n, float third)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    const f4 first = load_row(static_cast<const float*>(xin.p[0]) + e0, lane, remain, 0.0f);
    f4 prev = load_row(static_cast<const float*>(xin.p[k - 1]) + e0, lane, remain, 0.0f);
    f4 cur = first;
    for (int i = 0; i < k; ++i) {
        const f4 next = (i + 1 < k) ? load_row(static_cast<const float*>(xin.p[i + 1]) + e0, lane, remain, 0.0f) : first;
        const f4 s = add4(add4(prev, cur), next);
        store_row(static_cast<float*>(xout.p[i]) + e0, lane, remain, mul4(s, third));
        prev = cur;
        cur = next;
    }
}

// ------------------------------------------------------------------------------------------ LP, fused
// Workgroup = one chunk of all K peers; wave w holds rows [w*RPW, (w+1)*RPW) of every peer.
// Peers are processed in order; peer p's output is formed as soon as the new public copies of
// p-1, p, p+1 exist, so only a short window of peers is live in registers at any time.
template <int K, int RPW>
__global__ void __launch_bounds__(64 * ((16 + RPW - 1) / RPW))
k_ring_avg_lp(PtrTable xin, MutPtrTable xout, MutPtrTable xhat, MutPtrTable codes, MutPtrTable minmax, size_t n,
              uint32_t chunk, float third)
{
    __shared__ float s_red[K][2 * kMaxWaves];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    f4 h[K][RPW];    // new public copy xhat' of every peer
    f4 own[K][RPW];  // x - xhat' of every peer
    auto finalize = [&](int p) {
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int off = static_cast<int>(wave * RPW + r) * kRow;
            const int remain = len - off;
            const f4 s = add4(add4(h[(p + K - 1) % K][r], h[p][r]), h[(p + 1) % K][r]);
            const f4 o = add4(mul4(s, third), own[p][r]);
            if (remain > 0) store_row(static_cast<float*>(xout.p[p]) + base + off, lane, remain, o);
        }
    };
    // Peers are taken in groups of G: the statistics of a whole group sit behind one barrier.
    constexpr int G = BAGUA_LP_GROUP;
#pragma unroll
    for (int g0 = 0; g0 < K; g0 += G) {
        f4 x[G][RPW], d[G][RPW];
        float mn[G], mx[G];
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const int i = g0 + gi;
            if (i >= K) continue;
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int off = static_cast<int>(wave * RPW + r) * kRow;
                const int remain = len - off;
                x[gi][r] = f4{0.f, 0.f, 0.f, 0.f};
                h[i][r] = f4{0.f, 0.f, 0.f, 0.f};
                if (remain > 0) {
                    x[gi][r] = load_row(static_cast<const float*>(xin.p[i]) + base + off, lane, remain, 0.0f);
                    h[i][r] = load_row(static_cast<const float*>(xhat.p[i]) + base + off, lane, remain, 0.0f);
                }
                d[gi][r] = sub4(x[gi][r], h[i][r]);
            }
            chunk_minmax_partial<RPW>(d[gi], len, wave, lane, nwaves, s_red[i], mn[gi], mx[gi]);
        }
        if (nwaves > 1) __syncthreads();
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const int i = g0 + gi;
            if (i >= K) continue;
            chunk_minmax_finish(nwaves, s_red[i], mn[gi], mx[gi]);
            // d <- decode(Q(d)); codes and (min,max) of peer i are written on the way
            minmax_quantise_chunk<RPW, false, false, true>(d[gi], mn[gi], mx[gi], len, wave, lane, nullptr,
                                                           static_cast<uint8_t*>(codes.p[i]) + base,
                                                           static_cast<float*>(minmax.p[i]) + 2 * c, nullptr);
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int off = static_cast<int>(wave * RPW + r) * kRow;
                const int remain = len - off;
                h[i][r] = add4(h[i][r], d[gi][r]);
                own[i][r] = sub4(x[gi][r], h[i][r]);
                if (remain > 0) store_row(static_cast<float*>(xhat.p[i]) + base + off, lane, remain, h[i][r]);
            }
            if (i >= 2) finalize(i - 1);
        }
    }
    finalize(K - 1);
    if (K > 1) finalize(0);
}

// ------------------------------------------------------------------------------------------ LP, two-pass fallback
// Pass 1 (per peer): d = x - xhat; codes, minmax = Q(d); xhat <- xhat + decode.
template <int RPW>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_lp_encode(const float* __restrict__ x, float* __restrict__ xhat, size_t n, uint32_t chunk,
            uint8_t* __restrict__ codes, float* __restrict__ minmax)
{
    __shared__ float s_red[2 * kMaxWaves];
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    f4 h[RPW], d[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int off = static_cast<int>(wave * RPW + r) * kRow;
        const int remain = len - off;
        h[r] = f4{0.f, 0.f, 0.f, 0.f};
        d[r] = h[r];
        if (remain > 0) {
            h[r] = load_row(xhat + base + off, lane, remain, 0.0f);
            d[r] = sub4(load_row(x + base + off, lane, remain, 0.0f), h[r]);
        }
    }
    minmax_encode_chunk<RPW, false, false, true>(d, len, wave, lane, nwaves, nullptr, codes + base,
                                                 minmax + 2 * c, nullptr, s_red);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int off = static_cast<int>(wave * RPW + r) * kRow;
        const int remain = len - off;
        if (remain > 0) store_row(xhat + base + off, lane, remain, add4(h[r], d[r]));
    }
}

// Pass 2: x_out[i] = ((xhat[i-1] + xhat[i]) + xhat[i+1]) * third + (x[i] - xhat[i]), rolling over peers.
__global__ void __launch_bounds__(kWave * kRowWaves)
k_lp_mix(PtrTable xin, MutPtrTable xout, MutPtrTable xhat, int k, size_t n, float third)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    const f4 first = load_row(static_cast<const float*>(xhat.p[0]) + e0, lane, remain, 0.0f);
    f4 prev = load_row(static_cast<const float*>(xhat.p[k - 1]) + e0, lane, remain, 0.0f);
    f4 cur = first;
    for (int i = 0; i < k; ++i) {
        const f4 next = (i + 1 < k) ? load_row(static_cast<const float*>(xhat.p[i + 1]) + e0, lane, remain, 0.0f) : first;
        const f4 xi = load_row(static_cast<const float*>(xin.p[i]) + e0, lane, remain, 0.0f);
        const f4 s = add4(add4(prev, cur), next);
        store_row(static_cast<float*>(xout.p[i]) + e0, lane, remain, add4(mul4(s, third), sub4(xi, cur)));
        prev = cur;
        cur = next;
    }
}

// ------------------------------------------------------------------------------------------ host
template <int K>
static void launch_fp_k(const PtrTable& in, const MutPtrTable& out, size_t n, float third, dim3 grid, hipStream_t s)
{
    const size_t rows = (n + kRow - 1) / kRow;
    hipLaunchKernelGGL((k_ring_avg_fp<K>), dim3(static_cast<unsigned>((rows + kFpWaves - 1) / kFpWaves)),
                       dim3(64 * kFpWaves), 0, s, in, out, n, third);
}

static int launch_ring_fp(const float* const* x_in, float* const* x_out, int k, size_t n, hipStream_t stream)
{
    PtrTable in{};
    MutPtrTable out{};
    for (int i = 0; i < k; ++i) {
        in.p[i] = x_in[i];
        out.p[i] = x_out[i];
    }
    const size_t rows = (n + kRow - 1) / kRow;
    dim3 grid(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves));
    const float third = 1.0f / 3.0f;
    switch (k) {
#define BAGUA_FP_CASE(K) case K: launch_fp_k<K>(in, out, n, third, grid, stream); break;
        BAGUA_FP_CASE(1) BAGUA_FP_CASE(2) BAGUA_FP_CASE(3) BAGUA_FP_CASE(4) BAGUA_FP_CASE(5) BAGUA_FP_CASE(6)
        BAGUA_FP_CASE(7) BAGUA_FP_CASE(8) BAGUA_FP_CASE(9) BAGUA_FP_CASE(10) BAGUA_FP_CASE(11) BAGUA_FP_CASE(12)
        BAGUA_FP_CASE(13) BAGUA_FP_CASE(14) BAGUA_FP_CASE(15) BAGUA_FP_CASE(16)
#undef BAGUA_FP_CASE
        default:
            hipLaunchKernelGGL(k_ring_avg_fp_any, grid, dim3(kWave * kRowWaves), 0, stream, in, out, k, n, third);
    }
    return launch_status();
}

template <int K>
static void launch_lp_k(const PtrTable& in, const MutPtrTable& out, const MutPtrTable& hat, const MutPtrTable& cd,
                        const MutPtrTable& mm, size_t n, uint32_t chunk, float third, dim3 grid, dim3 block,
                        hipStream_t s)
{
    hipLaunchKernelGGL((k_ring_avg_lp<K, BAGUA_RPW_LP>), grid, block, 0, s, in, out, hat, cd, mm, n, chunk, third);
}

static int launch_ring_lp(const float* const* x_in, float* const* x_out, float* const* xhat, uint8_t* const* codes,
                          float* const* minmax, int k, size_t n, size_t chunk, hipStream_t stream)
{
    PtrTable in{};
    MutPtrTable out{}, hat{}, cd{}, mm{};
    for (int i = 0; i < k; ++i) {
        in.p[i] = x_in[i];
        out.p[i] = x_out[i];
        hat.p[i] = xhat[i];
        cd.p[i] = codes[i];
        mm.p[i] = minmax[i];
    }
    const float third = 1.0f / 3.0f;
    const size_t nc = num_chunks(n, chunk);
    const int rows = static_cast<int>(chunk / kRow);
    if (k <= 8 && rows <= 16) {
        dim3 grid(static_cast<unsigned>(nc)), block(64 * ((rows + BAGUA_RPW_LP - 1) / BAGUA_RPW_LP));
        const uint32_t ch = static_cast<uint32_t>(chunk);
        switch (k) {
#define BAGUA_LP_CASE(K) case K: launch_lp_k<K>(in, out, hat, cd, mm, n, ch, third, grid, block, stream); break;
            BAGUA_LP_CASE(1) BAGUA_LP_CASE(2) BAGUA_LP_CASE(3) BAGUA_LP_CASE(4) BAGUA_LP_CASE(5) BAGUA_LP_CASE(6)
            BAGUA_LP_CASE(7) BAGUA_LP_CASE(8)
#undef BAGUA_LP_CASE
        }
        return launch_status();
    }
    // larger k or chunk: the chunk of all peers does not fit one workgroup's registers
    const int rpw = pick_rpw(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(nc)), block(64 * ((rows + rpw - 1) / rpw));
    for (int i = 0; i < k; ++i) {
        BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_lp_encode<RPW>), grid, block, 0, stream, x_in[i], xhat[i], n,
                                                   static_cast<uint32_t>(chunk), codes[i], minmax[i]))
    }
    const size_t nrows = (n + kRow - 1) / kRow;
    hipLaunchKernelGGL(k_lp_mix, dim3(static_cast<unsigned>((nrows + kRowWaves - 1) / kRowWaves)), dim3(kWave * kRowWaves), 0, stream, in, out, hat, k, n,
                       third);
    return launch_status();
}

}  // namespace bagua

using namespace bagua;

extern "C" int bagua_decentralized_avg(int mode, const float* const* x_in, float* const* x_out, float* const* xhat,
                                       uint8_t* const* codes, float* const* minmax, int k, size_t n, size_t chunk,
                                       void* stream)
{
    if (mode != BAGUA_AVG_FP && mode != BAGUA_AVG_LP_MINMAX_U8) return BAGUA_ERR_INVALID_ARG;
    if (!x_in || !x_out || k < 1 || k > BAGUA_MAX_WORKERS || n == 0) return BAGUA_ERR_INVALID_ARG;
    const bool lp = mode == BAGUA_AVG_LP_MINMAX_U8;
    if (lp && (!xhat || !codes || !minmax || !chunk_ok(chunk))) return BAGUA_ERR_INVALID_ARG;
    for (int i = 0; i < k; ++i) {
        if (!x_in[i] || !x_out[i]) return BAGUA_ERR_INVALID_ARG;
        if (lp && (!xhat[i] || !codes[i] || !minmax[i])) return BAGUA_ERR_INVALID_ARG;
    }
    {
        const size_t bytes = n * sizeof(float);
        RangeCheck rc;
        for (int i = 0; i < k; ++i) {
            rc.reads(x_in[i], bytes);
            rc.writes(x_out[i], bytes);
            if (lp) {
                rc.writes(xhat[i], bytes);
                rc.writes(codes[i], n);
                rc.writes(minmax[i], 2 * num_chunks(n, chunk) * sizeof(float));
            }
        }
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    for (int i = 0; i < k; ++i) {
        if (!aligned16(x_in[i]) || !aligned16(x_out[i])) return BAGUA_ERR_ALIGNMENT;
        if (lp && (!aligned16(xhat[i]) || !aligned16(codes[i]) || !aligned4(minmax[i]))) return BAGUA_ERR_ALIGNMENT;
    }
    const size_t rows = (n + kRow - 1) / kRow;
    if ((rows + kRowWaves - 1) / kRowWaves > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!lp) return launch_ring_fp(x_in, x_out, k, n, s);
    return launch_ring_lp(x_in, x_out, xhat, codes, minmax, k, n, chunk, s);
}

// ------------------------------------------------------------------------------------------ chosen peers
// x_out[i] = (x_in[i] + x_in[peer[i]]) * 0.5.  The host turns the peer map into "jobs": a matched
// pair (a, b) is one job that reads both replicas once and writes the same bits to both outputs
// (8 bytes per element per peer); any other worker is a job of its own that reads its two inputs.
namespace bagua {

struct PeerJobs {
    const float* a[BAGUA_MAX_WORKERS];
    const float* b[BAGUA_MAX_WORKERS];
    float* out_a[BAGUA_MAX_WORKERS];
    float* out_b[BAGUA_MAX_WORKERS];  // nullptr for a single-output job
};

__global__ void __launch_bounds__(kWave * kRowWaves)
k_peer_avg_fp(PeerJobs jobs, size_t n)
{
    const int job = blockIdx.y;
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    const f4 xa = load_row(jobs.a[job] + e0, lane, remain, 0.0f);
    const f4 xb = load_row(jobs.b[job] + e0, lane, remain, 0.0f);
    const f4 o = mul4(add4(xa, xb), 0.5f);
    store_row(jobs.out_a[job] + e0, lane, remain, o);
    if (jobs.out_b[job]) store_row(jobs.out_b[job] + e0, lane, remain, o);
}

}  // namespace bagua

extern "C" int bagua_decentralized_avg_peers(const float* const* x_in, float* const* x_out, const int* peer, int k,
                                             size_t n, void* stream)
{
    if (!x_in || !x_out || !peer || k < 1 || k > BAGUA_MAX_WORKERS || n == 0) return BAGUA_ERR_INVALID_ARG;
    for (int i = 0; i < k; ++i)
        if (!x_in[i] || !x_out[i] || peer[i] < 0 || peer[i] >= k) return BAGUA_ERR_INVALID_ARG;
    {
        RangeCheck rc;
        for (int i = 0; i < k; ++i) {
            rc.reads(x_in[i], n * sizeof(float));
            rc.writes(x_out[i], n * sizeof(float));
        }
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    for (int i = 0; i < k; ++i)
        if (!aligned16(x_in[i]) || !aligned16(x_out[i])) return BAGUA_ERR_ALIGNMENT;
    const size_t rows = (n + kRow - 1) / kRow;
    if ((rows + kRowWaves - 1) / kRowWaves > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    PeerJobs jobs{};
    int nj = 0;
    for (int i = 0; i < k; ++i) {
        const int p = peer[i];
        const bool matched = p != i && peer[p] == i;
        if (matched && p < i) continue;  // written by the partner's job
        jobs.a[nj] = x_in[i];
        jobs.b[nj] = x_in[p];
        jobs.out_a[nj] = x_out[i];
        jobs.out_b[nj] = matched ? x_out[p] : nullptr;
        ++nj;
    }
    hipLaunchKernelGGL(k_peer_avg_fp, dim3(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves), nj), dim3(kWave * kRowWaves), 0,
                       static_cast<hipStream_t>(stream), jobs, n);
    return launch_status();
}

// ------------------------------------------------------------------------------------------ C_FP_S
// Centralised full-precision average of k replicas: out = (x_0 + x_1 + ...) * inv_k, ascending order.
// One wave per row; the loads of four workers are in flight together.
namespace bagua {

__global__ void __launch_bounds__(kWave * kRowWaves)
k_centralized_avg_fp(PtrTable xs, int k, float inv_k, size_t n, float* __restrict__ out)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    f4 s = load_row(static_cast<const float*>(xs.p[0]) + e0, lane, remain, 0.0f);
    int j = 1;
    for (; j + 4 <= k; j += 4) {
        f4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = load_row(static_cast<const float*>(xs.p[j + u]) + e0, lane, remain, 0.0f);
#pragma unroll
        for (int u = 0; u < 4; ++u) s = add4(s, v[u]);
    }
    for (; j < k; ++j) s = add4(s, load_row(static_cast<const float*>(xs.p[j]) + e0, lane, remain, 0.0f));
    store_row(out + e0, lane, remain, mul4(s, inv_k));
}

}  // namespace bagua

extern "C" int bagua_centralized_avg_fp(const float* const* x, int k, size_t n, float* out, void* stream)
{
    if (!x || k < 1 || k > BAGUA_MAX_WORKERS || n == 0 || !out) return BAGUA_ERR_INVALID_ARG;
    {
        RangeCheck rc;
        for (int j = 0; j < k; ++j) {
            if (!x[j]) return BAGUA_ERR_INVALID_ARG;
            rc.reads(x[j], n * sizeof(float));
        }
        rc.writes(out, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    for (int j = 0; j < k; ++j)
        if (!aligned16(x[j])) return BAGUA_ERR_ALIGNMENT;
    if (!aligned16(out)) return BAGUA_ERR_ALIGNMENT;
    const size_t rows = (n + kRow - 1) / kRow;
    if ((rows + kRowWaves - 1) / kRowWaves > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    PtrTable xt{};
    for (int j = 0; j < k; ++j) xt.p[j] = x[j];
    hipLaunchKernelGGL(k_centralized_avg_fp, dim3(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves)), dim3(kWave * kRowWaves), 0,
                       static_cast<hipStream_t>(stream), xt, k, 1.0f / static_cast<float>(k), n, out);
    return launch_status();
}

// ------------------------------------------------------------------------------------------ chosen peers, LP
// D_LP_S with one chosen peer per worker (Sections 3.2 and 3.4): every worker publishes Q(x - xhat),
// all holders advance xhat, then x_out[i] = (xhat[i] + xhat[peer[i]]) * 0.5 + (x[i] - xhat[i]).
// A matched pair is one fused job: a workgroup owns one chunk of both partners, so x and xhat of
// each are read once and out, xhat, codes written once (17 bytes per element per peer).  Any other
// peer map takes two passes: k_lp_encode per worker, then a mix over the advanced public copies.
namespace bagua {

struct PeerLpJobs {
    const float* x[2][BAGUA_MAX_WORKERS / 2];
    float* out[2][BAGUA_MAX_WORKERS / 2];
    float* hat[2][BAGUA_MAX_WORKERS / 2];
    uint8_t* codes[2][BAGUA_MAX_WORKERS / 2];
    float* minmax[2][BAGUA_MAX_WORKERS / 2];
};

template <int RPW>
__global__ void __launch_bounds__(64 * ((16 + RPW - 1) / RPW))
k_peer_avg_lp(PeerLpJobs jobs, size_t n, uint32_t chunk)
{
    __shared__ float s_red[2][2 * kMaxWaves];
    const int job = blockIdx.y;
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;

    f4 h[2][RPW], own[2][RPW];
#pragma unroll
    for (int sd = 0; sd < 2; ++sd) {
        const float* __restrict__ xp = jobs.x[sd][job];
        float* __restrict__ hp = jobs.hat[sd][job];
        f4 x[RPW], d[RPW];
        float mn, mx;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int off = static_cast<int>(wave * RPW + r) * kRow;
            const int remain = len - off;
            x[r] = f4{0.f, 0.f, 0.f, 0.f};
            h[sd][r] = x[r];
            if (remain > 0) {
                x[r] = load_row(xp + base + off, lane, remain, 0.0f);
                h[sd][r] = load_row(hp + base + off, lane, remain, 0.0f);
            }
            d[r] = sub4(x[r], h[sd][r]);
        }
        chunk_minmax_partial<RPW>(d, len, wave, lane, nwaves, s_red[sd], mn, mx);
        if (nwaves > 1) __syncthreads();
        chunk_minmax_finish(nwaves, s_red[sd], mn, mx);
        minmax_quantise_chunk<RPW, false, false, true>(d, mn, mx, len, wave, lane, nullptr, jobs.codes[sd][job] + base,
                                                       jobs.minmax[sd][job] + 2 * c, nullptr);
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int off = static_cast<int>(wave * RPW + r) * kRow;
            const int remain = len - off;
            h[sd][r] = add4(h[sd][r], d[r]);
            own[sd][r] = sub4(x[r], h[sd][r]);
            if (remain > 0) store_row(hp + base + off, lane, remain, h[sd][r]);
        }
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int off = static_cast<int>(wave * RPW + r) * kRow;
        const int remain = len - off;
        if (remain <= 0) continue;
        const f4 avg = mul4(add4(h[0][r], h[1][r]), 0.5f);
        store_row(jobs.out[0][job] + base + off, lane, remain, add4(avg, own[0][r]));
        store_row(jobs.out[1][job] + base + off, lane, remain, add4(avg, own[1][r]));
    }
}

// Second pass of the general case: worker i = blockIdx.y reads the advanced xhat of itself and of its peer.
struct PeerMixJobs {
    const float* x[BAGUA_MAX_WORKERS];
    const float* hat_own[BAGUA_MAX_WORKERS];
    const float* hat_peer[BAGUA_MAX_WORKERS];
    float* out[BAGUA_MAX_WORKERS];
};

__global__ void __launch_bounds__(kWave * kRowWaves)
k_peer_mix_lp(PeerMixJobs jobs, size_t n)
{
    const int i = blockIdx.y;
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    const f4 a = load_row(jobs.hat_own[i] + e0, lane, remain, 0.0f);
    const f4 b = load_row(jobs.hat_peer[i] + e0, lane, remain, 0.0f);
    const f4 xi = load_row(jobs.x[i] + e0, lane, remain, 0.0f);
    store_row(jobs.out[i] + e0, lane, remain, add4(mul4(add4(a, b), 0.5f), sub4(xi, a)));
}

}  // namespace bagua

extern "C" int bagua_decentralized_avg_peers_lp(const float* const* x_in, float* const* x_out, float* const* xhat,
                                                uint8_t* const* codes, float* const* minmax, const int* peer, int k,
                                                size_t n, size_t chunk, void* stream)
{
    if (!x_in || !x_out || !xhat || !codes || !minmax || !peer || k < 1 || k > BAGUA_MAX_WORKERS || n == 0 ||
        !chunk_ok(chunk))
        return BAGUA_ERR_INVALID_ARG;
    for (int i = 0; i < k; ++i)
        if (!x_in[i] || !x_out[i] || !xhat[i] || !codes[i] || !minmax[i] || peer[i] < 0 || peer[i] >= k)
            return BAGUA_ERR_INVALID_ARG;
    {
        const size_t bytes = n * sizeof(float);
        RangeCheck rc;
        for (int i = 0; i < k; ++i) {
            rc.reads(x_in[i], bytes);
            rc.writes(x_out[i], bytes);
            rc.writes(xhat[i], bytes);
            rc.writes(codes[i], n);
            rc.writes(minmax[i], 2 * num_chunks(n, chunk) * sizeof(float));
        }
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    for (int i = 0; i < k; ++i)
        if (!aligned16(x_in[i]) || !aligned16(x_out[i]) || !aligned16(xhat[i]) || !aligned16(codes[i]) ||
            !aligned4(minmax[i]))
            return BAGUA_ERR_ALIGNMENT;
    const size_t nrows = (n + kRow - 1) / kRow;
    if ((nrows + 3) / 4 > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t nc = num_chunks(n, chunk);
    const int rows = static_cast<int>(chunk / kRow);
    const uint32_t ch = static_cast<uint32_t>(chunk);

    bool matching = true;  // every worker is in a pair with a distinct partner
    for (int i = 0; i < k; ++i) matching = matching && peer[i] != i && peer[peer[i]] == i;
    if (matching && rows <= 16) {
        PeerLpJobs jobs{};
        int nj = 0;
        for (int i = 0; i < k; ++i) {
            const int p = peer[i];
            if (p < i) continue;
            const int side[2] = {i, p};
            for (int sd = 0; sd < 2; ++sd) {
                jobs.x[sd][nj] = x_in[side[sd]];
                jobs.out[sd][nj] = x_out[side[sd]];
                jobs.hat[sd][nj] = xhat[side[sd]];
                jobs.codes[sd][nj] = codes[side[sd]];
                jobs.minmax[sd][nj] = minmax[side[sd]];
            }
            ++nj;
        }
        dim3 grid(static_cast<unsigned>(nc), nj), block(64 * ((rows + BAGUA_RPW_LP - 1) / BAGUA_RPW_LP));
        hipLaunchKernelGGL((k_peer_avg_lp<BAGUA_RPW_LP>), grid, block, 0, s, jobs, n, ch);
        return launch_status();
    }
    const int rpw = pick_rpw(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(nc)), block(64 * ((rows + rpw - 1) / rpw));
    for (int i = 0; i < k; ++i) {
        BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_lp_encode<RPW>), grid, block, 0, s, x_in[i], xhat[i], n, ch,
                                                   codes[i], minmax[i]))
    }
    PeerMixJobs mix{};
    for (int i = 0; i < k; ++i) {
        mix.x[i] = x_in[i];
        mix.hat_own[i] = xhat[i];
        mix.hat_peer[i] = xhat[peer[i]];
        mix.out[i] = x_out[i];
    }
    hipLaunchKernelGGL(k_peer_mix_lp, dim3(static_cast<unsigned>((nrows + kRowWaves - 1) / kRowWaves), k), dim3(kWave * kRowWaves), 0, s, mix, n);
    return launch_status();
}

// ------------------------------------------------------------------------------------------ one peer's share of D_LP_S
// What a single GPU does in a sharded run of the low-precision ring (Sections 3.2 and 3.4): it encodes
// its own difference and advances its own public copy (k_lp_encode, 13 bytes per element), receives the
// two neighbours' codes, advances its copies of their public replicas and forms its own new replica
// (k_lp_apply_mix, 30 bytes per element).  The arithmetic is that of the all-peers kernel above.
namespace bagua {

// APPLY_L / APPLY_R: that neighbour's codes are decoded into its copy (otherwise the copy is current).
// SAME: both neighbours are one peer (ring of two): one copy, advanced once, counted twice.
template <bool APPLY_L, bool APPLY_R, bool SAME>
__global__ void __launch_bounds__(kWave * kRowWaves)
k_lp_apply_mix(const float* __restrict__ x, const float* __restrict__ h_own, float* h_left, float* h_right,
               const uint8_t* __restrict__ c_left, const float* __restrict__ m_left,
               const uint8_t* __restrict__ c_right, const float* __restrict__ m_right, size_t n, uint32_t chunk,
               float third, float* __restrict__ x_out)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const size_t c = e0 / chunk;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    const f4 xi = load_row(x + e0, lane, remain, 0.0f);
    const f4 ho = load_row(h_own + e0, lane, remain, 0.0f);
    auto advanced = [&](float* h, const uint8_t* codes, const float* mm, bool apply) {
        f4 v = load_row(h + e0, lane, remain, 0.0f);
        if (apply) {
            const float mn = mm[2 * c], step = minmax_step(mn, mm[2 * c + 1]);
            const uint32_t w = load_codes_row(codes + e0, lane, remain);
            v.x = v.x + (mn + byte_to_float(w, 0) * step);
            v.y = v.y + (mn + byte_to_float(w, 1) * step);
            v.z = v.z + (mn + byte_to_float(w, 2) * step);
            v.w = v.w + (mn + byte_to_float(w, 3) * step);
            store_row(h + e0, lane, remain, v);
        }
        return v;
    };
    const f4 hl = advanced(h_left, c_left, m_left, APPLY_L);
    const f4 hr = SAME ? hl : advanced(h_right, c_right, m_right, APPLY_R);
    const f4 s = add4(add4(hl, ho), hr);
    store_row(x_out + e0, lane, remain, add4(mul4(s, third), sub4(xi, ho)));
}

}  // namespace bagua

extern "C" int bagua_lp_encode(const float* x, float* xhat, size_t n, size_t chunk, uint8_t* codes, float* minmax,
                               void* stream)
{
    if (!x || !xhat || !codes || !minmax || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    RangeCheck rc;
    rc.reads(x, n * sizeof(float));
    rc.writes(xhat, n * sizeof(float));
    rc.writes(codes, n);
    rc.writes(minmax, 2 * num_chunks(n, chunk) * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(xhat) || !aligned16(codes) || !aligned4(minmax)) return BAGUA_ERR_ALIGNMENT;
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, BAGUA_RPW_COMPRESS);
    dim3 grid(static_cast<unsigned>(num_chunks(n, chunk))), block(64 * ((rows + rpw - 1) / rpw));
    BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_lp_encode<RPW>), grid, block, 0, static_cast<hipStream_t>(stream), x, xhat,
                                               n, static_cast<uint32_t>(chunk), codes, minmax))
    return launch_status();
}

extern "C" int bagua_lp_apply_mix(const float* x, const float* xhat_own, float* xhat_left, float* xhat_right,
                                  const uint8_t* codes_left, const float* minmax_left, const uint8_t* codes_right,
                                  const float* minmax_right, size_t n, size_t chunk, float* x_out, void* stream)
{
    if (!x || !xhat_own || !xhat_left || !xhat_right || !x_out || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    if ((codes_left == nullptr) != (minmax_left == nullptr) || (codes_right == nullptr) != (minmax_right == nullptr))
        return BAGUA_ERR_INVALID_ARG;
    const bool same = xhat_left == xhat_right;
    if (same && codes_right) return BAGUA_ERR_INVALID_ARG;  // one copy is advanced once, through codes_left
    const size_t bytes = n * sizeof(float), mbytes = 2 * num_chunks(n, chunk) * sizeof(float);
    RangeCheck rc;
    rc.reads(x, bytes);
    rc.reads(codes_left, n);
    rc.reads(minmax_left, mbytes);
    rc.reads(codes_right, n);
    rc.reads(minmax_right, mbytes);
    rc.writes(x_out, bytes);
    // a neighbour copy that is not advanced is only read (on a ring of one it is the peer's own copy)
    if (codes_left) rc.writes(xhat_left, bytes); else rc.reads(xhat_left, bytes);
    if (!same) { if (codes_right) rc.writes(xhat_right, bytes); else rc.reads(xhat_right, bytes); }
    rc.reads(xhat_own, bytes);
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    const size_t rows = (n + kRow - 1) / kRow;
    if ((rows + kRowWaves - 1) / kRowWaves > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(xhat_own) || !aligned16(xhat_left) || !aligned16(xhat_right) || !aligned16(codes_left) ||
        !aligned16(codes_right) || !aligned4(minmax_left) || !aligned4(minmax_right) || !aligned16(x_out))
        return BAGUA_ERR_ALIGNMENT;
    dim3 grid(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves)), block(kWave * kRowWaves);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t ch = static_cast<uint32_t>(chunk);
    const float third = 1.0f / 3.0f;
#define BAGUA_MIX(L, R, S)                                                                                            \
    hipLaunchKernelGGL((k_lp_apply_mix<L, R, S>), grid, block, 0, s, x, xhat_own, xhat_left, xhat_right, codes_left, \
                       minmax_left, codes_right, minmax_right, n, ch, third, x_out)
    const bool al = codes_left != nullptr, ar = codes_right != nullptr;
    if (same) { if (al) BAGUA_MIX(true, false, true); else BAGUA_MIX(false, false, true); }
    else if (al && ar) BAGUA_MIX(true, true, false);
    else if (al) BAGUA_MIX(true, false, false);
    else if (ar) BAGUA_MIX(false, true, false);
    else BAGUA_MIX(false, false, false);
#undef BAGUA_MIX
    return launch_status();
}
