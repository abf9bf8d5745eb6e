// 1-bit sign codec kernels: worker-side compress with error feedback, server-side
// decompress-average-recompress, and decompress (C_LP_S with the compression of "1-bit Adam",
// Sections 3.2 and 4.1 of the paper).
//
// Lane l of a wave owns elements 4l..4l+3 of every 256-element row, so the group of four that the
// fixed |v| summation order is defined on is exactly one lane's 128-bit load, accumulator m mod 64
// is lane m mod 64, and the final xor butterfly is a wave-level shuffle reduction.
#include "batch.hpp"
#include "launchers.hpp"
#include "sign_device.hpp"

#pragma clang fp contract(off)

namespace bagua {

// ------------------------------------------------------------------------------------------
// MOM: the compressed tensor is the local momentum beta1*m + omb1*x of the compression stage of
// 1-bit Adam (x is then the gradient; m is read only).
template <int RPW, bool EF, bool MOM>
__device__ __forceinline__ void sign_compress_chunk(const float* __restrict__ x, float* __restrict__ residual, size_t n,
                                                    uint32_t chunk, uint32_t* __restrict__ bits,
                                                    float* __restrict__ scale, const float* __restrict__ mom,
                                                    float beta1, float omb1, size_t c, float* s_q, int pace)
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
    if (MOM) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            if (remain > 0) {
                const f4 m = load_row(mom + base + off, lane, remain, 0.0f);
                v[i].x = beta1 * m.x + omb1 * v[i].x;
                v[i].y = beta1 * m.y + omb1 * v[i].y;
                v[i].z = beta1 * m.z + omb1 * v[i].z;
                v[i].w = beta1 * m.w + omb1 * v[i].w;
            }
        }
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
    sign_encode_chunk<RPW, EF, false>(v, len, chunk, wave, lane, nwaves, EF ? residual + base : nullptr,
                                      bits + (base >> 5), scale + c, nullptr, s_q);
}

template <int RPW, bool EF, bool MOM = false>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_sign_compress(const float* __restrict__ x, float* __restrict__ residual, size_t n, uint32_t chunk,
                uint32_t* __restrict__ bits, float* __restrict__ scale, const float* __restrict__ mom, float beta1,
                float omb1, int pace)
{
    extern __shared__ float s_q[];
    sign_compress_chunk<RPW, EF, MOM>(x, residual, n, chunk, bits, scale, mom, beta1, omb1, blockIdx.x, s_q, pace);
}

// Batched: entry = [x, residual, bits, scale, n]; unit = chunk.
template <int RPW, bool EF>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_sign_compress_batched(BatchView bv, uint32_t chunk, int pace)
{
    extern __shared__ float s_q[];
    const uint32_t b = batch_find(bv, blockIdx.x);
    const uint64_t* e = bv.entries + static_cast<size_t>(b) * bv.entry_words;
    sign_compress_chunk<RPW, EF, false>(table_ptr<const float>(e[0]), table_ptr<float>(e[1]), e[4], chunk,
                                        table_ptr<uint32_t>(e[2]), table_ptr<float>(e[3]), nullptr, 0.0f,
                                        0.0f, blockIdx.x - bv.first_unit[b], s_q, pace);
}

// Server side with the sign codec: a = (sum_j +-scale_j) * inv_k in ascending j; w = a (+ eps).
// SRC names the workers' inputs: code(j) -> sign words of worker j, meta(j) -> its per-chunk scales.
struct SignTableSrc {   // pointers in the kernel arguments
    const PtrTable& bits;
    const PtrTable& scales;
    __device__ __forceinline__ const void* code(int j) const { return bits.p[j]; }
    __device__ __forceinline__ const float* meta(int j) const { return static_cast<const float*>(scales.p[j]); }
};
struct SignEntrySrc {   // pointers in a batch entry: [eps, bits_out, scale_out, out, n, bits[0..k), scale[0..k)]
    const uint64_t* e;
    int k;
    __device__ __forceinline__ const void* code(int j) const { return table_ptr<const void>(e[5 + j]); }
    __device__ __forceinline__ const float* meta(int j) const { return table_ptr<const float>(e[5 + k + j]); }
};

template <int RPW, bool EF, bool OUT, typename SRC>
__device__ __forceinline__ void drr_sign_chunk(const SRC& src, int k, float inv_k, float* __restrict__ eps, size_t n,
                                               uint32_t chunk, uint32_t* __restrict__ bits_out,
                                               float* __restrict__ scale_out, float* __restrict__ out, size_t c,
                                               float* s_q)
{
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    const int sh = 4 * (lane & 7);

    // Scales of this chunk: lane j fetches worker j's (one memory round trip for all workers instead of a chain
    // of k dependent ones), broadcast below with readlane.
    float lane_scale = 0.0f;
    if (lane < k) lane_scale = src.meta(lane)[c];

    f4 v[RPW];
    constexpr int NJ = BAGUA_DRR_SIGN_NJ;   // workers whose sign words are fetched together
    // Workers are summed in ascending order; worker 0 starts the sum (s = d_0, not 0 + d_0).
    // The one row of a bucket's last chunk that is cut short (if any) is the only one that needs per-element tail
    // tests; a wave that does not own it sees complete rows and, past the chunk's end, absent ones.
    const int rows = static_cast<int>(len / kRow);   // complete rows of this chunk
    const int ragged_row = (len % kRow) ? rows : -1;
    if (rows > 0 && (ragged_row < wave * RPW || ragged_row >= wave * RPW + RPW)) {
        // ---- complete (or absent) rows only, wave-uniform: no tail tests, uniform row addresses, one shift + one
        // three-input bit operation + one add per element and worker.  An absent row re-reads row 0 of the chunk
        // (complete, since rows > 0) and is cleared afterwards.
        int row_of[RPW];
#pragma unroll
        for (int i = 0; i < RPW; ++i) row_of[i] = (wave * RPW + i < rows) ? wave * RPW + i : 0;
        f4 e[RPW];
        if (EF) {
#pragma unroll
            for (int i = 0; i < RPW; ++i)
                e[i] = ld_stream(reinterpret_cast<const f4*>(eps + base + static_cast<size_t>(row_of[i]) * kRow) + lane);
        }
        const uint32_t word = static_cast<uint32_t>(lane >> 3);
        const uint32_t s0 = 31u - sh, s1 = 30u - sh, s2 = 29u - sh, s3 = 28u - sh;   // element's bit -> bit 31
        auto fetch = [&](int j, uint32_t (&w)[RPW]) {
            const uint32_t* bj = static_cast<const uint32_t*>(src.code(j)) + (base >> 5);
#pragma unroll
            for (int i = 0; i < RPW; ++i) w[i] = bj[row_of[i] * (kRow / 32) + word];
        };
        auto decode = [&](int j, const uint32_t (&w)[RPW], bool first) {
            const uint32_t sc = __builtin_amdgcn_readlane(__float_as_uint(lane_scale), j);
            const uint32_t neg = sc ^ 0x80000000u;
#pragma unroll
            for (int i = 0; i < RPW; ++i) {
                f4 d;
                d.x = sign_select(w[i] << s0, sc, neg);
                d.y = sign_select(w[i] << s1, sc, neg);
                d.z = sign_select(w[i] << s2, sc, neg);
                d.w = sign_select(w[i] << s3, sc, neg);
                if (first) {
                    v[i] = d;
                } else {
                    v[i].x = v[i].x + d.x;
                    v[i].y = v[i].y + d.y;
                    v[i].z = v[i].z + d.z;
                    v[i].w = v[i].w + d.w;
                }
            }
        };
        int j = 0;
        if (k >= NJ) {
            uint32_t w[NJ][RPW];
#pragma unroll
            for (int u = 0; u < NJ; ++u) fetch(u, w[u]);
            decode(0, w[0], true);
#pragma unroll
            for (int u = 1; u < NJ; ++u) decode(u, w[u], false);
            j = NJ;
        } else {
            uint32_t w[RPW];
            fetch(0, w);
            decode(0, w, true);
            j = 1;
        }
        for (; j + NJ <= k; j += NJ) {
            uint32_t w[NJ][RPW];
#pragma unroll
            for (int u = 0; u < NJ; ++u) fetch(j + u, w[u]);
#pragma unroll
            for (int u = 0; u < NJ; ++u) decode(j + u, w[u], false);
        }
        for (; j < k; ++j) {
            uint32_t w[RPW];
            fetch(j, w);
            decode(j, w, false);
        }
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            v[i].x = v[i].x * inv_k;
            v[i].y = v[i].y * inv_k;
            v[i].z = v[i].z * inv_k;
            v[i].w = v[i].w * inv_k;
            if (EF) {
                v[i].x = v[i].x + e[i].x;
                v[i].y = v[i].y + e[i].y;
                v[i].z = v[i].z + e[i].z;
                v[i].w = v[i].w + e[i].w;
            }
            if (wave * RPW + i >= rows) v[i] = f4{0.f, 0.f, 0.f, 0.f};   // absent row: +0 in the |v| sum, nothing stored
        }
    } else {
        // ---- the wave that owns the ragged row of a bucket's last chunk
        auto accumulate = [&](int j, uint32_t (&w)[RPW]) {
            const float sc = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(lane_scale), j));
            const float neg = -sc;
#pragma unroll
            for (int i = 0; i < RPW; ++i) {
                const uint32_t nib = w[i] >> sh;
                f4 d;
                d.x = (nib & 1u) ? sc : neg;
                d.y = (nib & 2u) ? sc : neg;
                d.z = (nib & 4u) ? sc : neg;
                d.w = (nib & 8u) ? sc : neg;
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
        for (int j = 0; j < k; ++j) {
            const uint32_t* bj = static_cast<const uint32_t*>(src.code(j)) + (base >> 5);
            uint32_t w[RPW];
#pragma unroll
            for (int i = 0; i < RPW; ++i) {
                const int off = static_cast<int>(wave * RPW + i) * kRow;
                const int remain = len - off;
                w[i] = 0;
                if (static_cast<int>(lane >> 3) * 32 < remain) w[i] = bj[(off >> 5) + (lane >> 3)];
            }
            accumulate(j, w);
        }
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int off = static_cast<int>(wave * RPW + i) * kRow;
            const int remain = len - off;
            const int e = lane * 4;
            // elements beyond the chunk must enter the |v| sum as +0.0f
            v[i].x = (e + 0 < remain) ? v[i].x * inv_k : 0.0f;
            v[i].y = (e + 1 < remain) ? v[i].y * inv_k : 0.0f;
            v[i].z = (e + 2 < remain) ? v[i].z * inv_k : 0.0f;
            v[i].w = (e + 3 < remain) ? v[i].w * inv_k : 0.0f;
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
    }
    sign_encode_chunk<RPW, EF, OUT>(v, len, chunk, wave, lane, nwaves, EF ? eps + base : nullptr,
                                    bits_out + (base >> 5), scale_out + c, OUT ? out + base : nullptr, s_q);
}

template <int RPW, bool EF, bool OUT>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_drr_sign(PtrTable bits_in, PtrTable scale_in, int k, float inv_k, float* __restrict__ eps, size_t n,
           uint32_t chunk, uint32_t* __restrict__ bits_out, float* __restrict__ scale_out,
           float* __restrict__ out)
{
    extern __shared__ float s_q[];
    drr_sign_chunk<RPW, EF, OUT>(SignTableSrc{bits_in, scale_in}, k, inv_k, eps, n, chunk, bits_out, scale_out, out,
                                 blockIdx.x, s_q);
}

template <int RPW, bool EF, bool OUT>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_drr_sign_batched(BatchView bv, int k, float inv_k, uint32_t chunk)
{
    extern __shared__ float s_q[];
    const uint32_t b = batch_find(bv, blockIdx.x);
    const uint64_t* e = bv.entries + static_cast<size_t>(b) * bv.entry_words;
    drr_sign_chunk<RPW, EF, OUT>(SignEntrySrc{e, k}, k, inv_k, table_ptr<float>(e[0]), e[4], chunk,
                                 table_ptr<uint32_t>(e[1]), table_ptr<float>(e[2]),
                                 table_ptr<float>(e[3]), blockIdx.x - bv.first_unit[b], s_q);
}

__global__ void __launch_bounds__(kWave * kRowWaves)
k_decompress_sign(const uint32_t* __restrict__ bits, const float* __restrict__ scale, size_t n, uint32_t chunk,
                  float* __restrict__ out)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const float sc = scale[e0 / chunk];
    const float neg = -sc;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);
    uint32_t w = 0;
    if (static_cast<int>(lane >> 3) * 32 < remain) w = bits[(e0 >> 5) + (lane >> 3)];
    const uint32_t nib = w >> (4 * (lane & 7));
    f4 d;
    d.x = (nib & 1u) ? sc : neg;
    d.y = (nib & 2u) ? sc : neg;
    d.z = (nib & 4u) ? sc : neg;
    d.w = (nib & 8u) ? sc : neg;
    store_row(out + e0, lane, remain, d);
}

// ------------------------------------------------------------------------------------------ host
struct SignGeometry {
    dim3 grid, block;
    size_t lds;
    int rpw;
};
static SignGeometry sign_geometry(size_t n, size_t chunk, int preferred, bool worker_side)
{
    SignGeometry g;
    const int rows = static_cast<int>(chunk / kRow);
    g.rpw = worker_side ? pick_rpw_worker(rows, preferred) : pick_rpw(rows, preferred);
    const int waves = (rows + g.rpw - 1) / g.rpw;
    g.grid = dim3(static_cast<unsigned>(num_chunks(n, chunk)));
    g.block = dim3(64 * waves);
    g.lds = waves > 1 ? static_cast<size_t>(rows) * kWave * sizeof(float) : 0;
    return g;
}

int launch_sign_compress(const float* x, float* residual, size_t n, size_t chunk, uint32_t* bits, float* scale,
                         hipStream_t stream)
{
    const SignGeometry g = sign_geometry(n, chunk, BAGUA_RPW_SIGN, true);
    const uint32_t ch = static_cast<uint32_t>(chunk);
    if (residual) {
        BAGUA_DISPATCH_RPW_WORKER(g.rpw, hipLaunchKernelGGL((k_sign_compress<RPW, true>), g.grid, g.block, g.lds, stream, x,
                                                     residual, n, ch, bits, scale, nullptr, 0.0f, 0.0f, pace_for(n)))
    } else {
        BAGUA_DISPATCH_RPW_WORKER(g.rpw, hipLaunchKernelGGL((k_sign_compress<RPW, false>), g.grid, g.block, g.lds, stream, x,
                                                     residual, n, ch, bits, scale, nullptr, 0.0f, 0.0f, pace_for(n)))
    }
    return launch_status();
}

int launch_drr_sign(const void* const* bits_in, const float* const* scale_in, int k, float* eps, size_t n,
                    size_t chunk, uint32_t* bits_out, float* scale_out, float* out, hipStream_t stream)
{
    PtrTable bt{}, st{};
    for (int j = 0; j < k; ++j) {
        bt.p[j] = bits_in[j];
        st.p[j] = scale_in[j];
    }
    const SignGeometry g = sign_geometry(n, chunk, BAGUA_RPW_DRR_SIGN, false);
    const float inv_k = 1.0f / static_cast<float>(k);
    const uint32_t ch = static_cast<uint32_t>(chunk);
#define BAGUA_DRR(EFv, OUTv)                                                                                      \
    BAGUA_DISPATCH_RPW(g.rpw, hipLaunchKernelGGL((k_drr_sign<RPW, EFv, OUTv>), g.grid, g.block, g.lds, stream, bt, \
                                                 st, k, inv_k, eps, n, ch, bits_out, scale_out, out))
    if (eps && out) { BAGUA_DRR(true, true) }
    else if (eps) { BAGUA_DRR(true, false) }
    else if (out) { BAGUA_DRR(false, true) }
    else { BAGUA_DRR(false, false) }
#undef BAGUA_DRR
    return launch_status();
}

int launch_drr_sign_batched(const void* workspace, size_t B, int k, size_t total_chunks, size_t chunk, bool ef,
                            bool with_out, hipStream_t stream)
{
    const BatchView bv = batch_view(workspace, B, 5 + 2 * static_cast<size_t>(k), total_chunks);
    SignGeometry g = sign_geometry(chunk, chunk, BAGUA_RPW_DRR_SIGN, false);
    g.grid = dim3(static_cast<unsigned>(total_chunks));
    const float inv_k = 1.0f / static_cast<float>(k);
    const uint32_t ch = static_cast<uint32_t>(chunk);
#define BAGUA_DRR(EFv, OUTv)                                                                                           \
    BAGUA_DISPATCH_RPW(g.rpw, hipLaunchKernelGGL((k_drr_sign_batched<RPW, EFv, OUTv>), g.grid, g.block, g.lds, stream, \
                                                 bv, k, inv_k, ch))
    if (ef && with_out) { BAGUA_DRR(true, true) }
    else if (ef) { BAGUA_DRR(true, false) }
    else if (with_out) { BAGUA_DRR(false, true) }
    else { BAGUA_DRR(false, false) }
#undef BAGUA_DRR
    return launch_status();
}

int launch_decompress_sign(const uint32_t* bits, const float* scale, size_t n, size_t chunk, float* out,
                           hipStream_t stream)
{
    const size_t rows = (n + kRow - 1) / kRow;
    dim3 grid(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves)), block(kWave * kRowWaves);
    hipLaunchKernelGGL(k_decompress_sign, grid, block, 0, stream, bits, scale, n, static_cast<uint32_t>(chunk), out);
    return launch_status();
}

}  // namespace bagua

using namespace bagua;

extern "C" int bagua_sign_compress_ef(const float* x, float* residual, size_t n, size_t chunk, uint32_t* bits,
                                      float* scale, void* stream)
{
    if (!x || !bits || !scale || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    RangeCheck rc;
    rc.reads(x, n * sizeof(float));
    rc.writes(residual, n * sizeof(float));
    rc.writes(bits, ((n + 31) / 32) * sizeof(uint32_t));
    rc.writes(scale, num_chunks(n, chunk) * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(residual) || !aligned16(bits) || !aligned4(scale)) return BAGUA_ERR_ALIGNMENT;
    return launch_sign_compress(x, residual, n, chunk, bits, scale, static_cast<hipStream_t>(stream));
}

extern "C" int bagua_momentum_sign_compress_ef(const float* g, const float* m, float beta1, float* residual, size_t n,
                                               size_t chunk, uint32_t* bits, float* scale, void* stream)
{
    if (!g || !m || !bits || !scale || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    RangeCheck rc;
    rc.reads(g, n * sizeof(float));
    rc.reads(m, n * sizeof(float));
    rc.writes(residual, n * sizeof(float));
    rc.writes(bits, ((n + 31) / 32) * sizeof(uint32_t));
    rc.writes(scale, num_chunks(n, chunk) * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (!aligned16(g) || !aligned16(m) || !aligned16(residual) || !aligned16(bits) || !aligned4(scale))
        return BAGUA_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const SignGeometry geo = sign_geometry(n, chunk, BAGUA_RPW_SIGN, true);
    const uint32_t ch = static_cast<uint32_t>(chunk);
    const float omb1 = 1.0f - beta1;
    if (residual) {
        BAGUA_DISPATCH_RPW_WORKER(geo.rpw, hipLaunchKernelGGL((k_sign_compress<RPW, true, true>), geo.grid, geo.block, geo.lds,
                                                       s, g, residual, n, ch, bits, scale, m, beta1, omb1, pace_for(n)))
    } else {
        BAGUA_DISPATCH_RPW_WORKER(geo.rpw, hipLaunchKernelGGL((k_sign_compress<RPW, false, true>), geo.grid, geo.block, geo.lds,
                                                       s, g, residual, n, ch, bits, scale, m, beta1, omb1, pace_for(n)))
    }
    return launch_status();
}

extern "C" int bagua_sign_compress_ef_batched(const float* const* x, float* const* residual, const size_t* n, size_t B,
                                              size_t chunk, uint32_t* const* bits, float* const* scale, void* workspace,
                                              size_t workspace_bytes, void* stream)
{
    if (!x || !n || !bits || !scale || !workspace || B == 0 || B > 0xffffffffu || !chunk_ok(chunk))
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
        if (!x[b] || !bits[b] || !scale[b] || n[b] == 0 || (ef && !residual[b])) return BAGUA_ERR_INVALID_ARG;
        float* r = ef ? residual[b] : nullptr;
        if (!aligned16(x[b]) || !aligned16(r) || !aligned16(bits[b]) || !aligned4(scale[b])) return BAGUA_ERR_ALIGNMENT;
        const size_t nc = num_chunks(n[b], chunk);
        rl.reads(x[b], n[b] * sizeof(float));
        rl.writes(r, n[b] * sizeof(float));
        rl.writes(bits[b], ((n[b] + 31) / 32) * sizeof(uint32_t));
        rl.writes(scale[b], nc * sizeof(float));
        table[b] = total;
        uint64_t* e = entries + b * ew;
        e[0] = reinterpret_cast<uintptr_t>(x[b]);
        e[1] = reinterpret_cast<uintptr_t>(r);
        e[2] = reinterpret_cast<uintptr_t>(bits[b]);
        e[3] = reinterpret_cast<uintptr_t>(scale[b]);
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
    SignGeometry g = sign_geometry(chunk, chunk, BAGUA_RPW_SIGN, false);
    g.grid = dim3(static_cast<unsigned>(total));
    const uint32_t ch = static_cast<uint32_t>(chunk);
    if (ef) {
        BAGUA_DISPATCH_RPW(g.rpw, hipLaunchKernelGGL((k_sign_compress_batched<RPW, true>), g.grid, g.block, g.lds, s, bv, ch, pace_for(total * chunk)))
    } else {
        BAGUA_DISPATCH_RPW(g.rpw, hipLaunchKernelGGL((k_sign_compress_batched<RPW, false>), g.grid, g.block, g.lds, s, bv, ch, pace_for(total * chunk)))
    }
    return launch_status();
}
