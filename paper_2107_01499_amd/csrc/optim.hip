// Decode fused into the bucket-level optimizer step: the last step of C_LP_S on every worker
// (decode the tensor the server sent back) and the update of the flattened bucket (Section 3.5 of
// the paper) in one pass.  The decoded tensor is never written to memory.  SGD: 1 (or 1/8) + 8
// (+ 8 with momentum) bytes per element; Adam: 1 + 24 (full), 1/8 + 16 (frozen variance).
#include <cmath>

#include "launchers.hpp"

#pragma clang fp contract(off)

namespace bagua {

// Decoded values of the row starting at element e0 (chunk c): four per lane.
template <int CODEC>
__device__ __forceinline__ f4 decode_row(const void* __restrict__ codes, const float* __restrict__ meta, size_t e0,
                                         size_t c, int lane, int remain)
{
    f4 g;
    if (CODEC == BAGUA_CODEC_MINMAX_U8) {
        const float mn = meta[2 * c], step = minmax_step(mn, meta[2 * c + 1]);
        const uint32_t w = load_codes_row(static_cast<const uint8_t*>(codes) + e0, lane, remain);
        g.x = mn + byte_to_float(w, 0) * step;
        g.y = mn + byte_to_float(w, 1) * step;
        g.z = mn + byte_to_float(w, 2) * step;
        g.w = mn + byte_to_float(w, 3) * step;
    } else {
        const float sc = meta[c];
        const float neg = -sc;
        uint32_t w = 0;
        if (static_cast<int>(lane >> 3) * 32 < remain) w = static_cast<const uint32_t*>(codes)[(e0 >> 5) + (lane >> 3)];
        const uint32_t nib = w >> (4 * (lane & 7));
        g.x = (nib & 1u) ? sc : neg;
        g.y = (nib & 2u) ? sc : neg;
        g.z = (nib & 4u) ? sc : neg;
        g.w = (nib & 8u) ? sc : neg;
    }
    return g;
}

// One wave per 256-element row, four rows per workgroup.
template <int CODEC, bool MOM, bool WD>
__global__ void __launch_bounds__(kWave * kRowWaves)
k_decompress_sgd(const void* __restrict__ codes, const float* __restrict__ meta, size_t n, uint32_t chunk,
                 float* __restrict__ param, float* __restrict__ mbuf, float lr, float mu, float wd)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const size_t c = e0 / chunk;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);

    f4 p = load_row(param + e0, lane, remain, 0.0f);
    f4 m = f4{0.f, 0.f, 0.f, 0.f};
    if (MOM) m = load_row(mbuf + e0, lane, remain, 0.0f);

    f4 g = decode_row<CODEC>(codes, meta, e0, c, lane, remain);
    if (WD) {
        g.x = g.x + wd * p.x;
        g.y = g.y + wd * p.y;
        g.z = g.z + wd * p.z;
        g.w = g.w + wd * p.w;
    }
    f4 u = g;
    if (MOM) {
        m.x = mu * m.x + g.x;
        m.y = mu * m.y + g.y;
        m.z = mu * m.z + g.z;
        m.w = mu * m.w + g.w;
        store_row(mbuf + e0, lane, remain, m);
        u = m;
    }
    p.x = p.x - lr * u.x;
    p.y = p.y - lr * u.y;
    p.z = p.z - lr * u.z;
    p.w = p.w - lr * u.w;
    store_row(param + e0, lane, remain, p);
}

// Adam-type update (no bias correction).  FROZEN: the decoded tensor is the averaged momentum of the
// compression stage of 1-bit Adam: it replaces m, and v is only read.
template <int CODEC, bool FROZEN, bool WD>
__global__ void __launch_bounds__(kWave * kRowWaves)
k_decompress_adam(const void* __restrict__ codes, const float* __restrict__ meta, size_t n, uint32_t chunk,
                  float* __restrict__ param, float* __restrict__ mbuf, float* __restrict__ vbuf, float lr, float beta1,
                  float omb1, float beta2, float omb2, float eps, float wd)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * kRowWaves + wave_index();
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    const size_t c = e0 / chunk;
    const int remain = static_cast<int>((n - e0 < static_cast<size_t>(kRow)) ? (n - e0) : kRow);

    f4 p = load_row(param + e0, lane, remain, 0.0f);
    f4 v = load_row(vbuf + e0, lane, remain, 1.0f);
    const f4 d = decode_row<CODEC>(codes, meta, e0, c, lane, remain);
    f4 m = d;
    if (!FROZEN) {
        const f4 mo = load_row(mbuf + e0, lane, remain, 0.0f);
        m.x = beta1 * mo.x + omb1 * d.x;
        m.y = beta1 * mo.y + omb1 * d.y;
        m.z = beta1 * mo.z + omb1 * d.z;
        m.w = beta1 * mo.w + omb1 * d.w;
        v.x = beta2 * v.x + omb2 * (d.x * d.x);
        v.y = beta2 * v.y + omb2 * (d.y * d.y);
        v.z = beta2 * v.z + omb2 * (d.z * d.z);
        v.w = beta2 * v.w + omb2 * (d.w * d.w);
        store_row(vbuf + e0, lane, remain, v);
    }
    store_row(mbuf + e0, lane, remain, m);
    f4 u;
    u.x = m.x / (sqrtf(v.x) + eps);
    u.y = m.y / (sqrtf(v.y) + eps);
    u.z = m.z / (sqrtf(v.z) + eps);
    u.w = m.w / (sqrtf(v.w) + eps);
    if (WD) {
        u.x = u.x + wd * p.x;
        u.y = u.y + wd * p.y;
        u.z = u.z + wd * p.z;
        u.w = u.w + wd * p.w;
    }
    p.x = p.x - lr * u.x;
    p.y = p.y - lr * u.y;
    p.z = p.z - lr * u.z;
    p.w = p.w - lr * u.w;
    store_row(param + e0, lane, remain, p);
}

// ------------------------------------------------------------------------------------------ top-K codec
// Without momentum and weight decay (and lr >= +0, finite) only the kept entries change: p - fl(lr * +0) = p bit for
// bit.  One thread per (chunk, slot) entry.
__global__ void __launch_bounds__(256)
k_sgd_topk_sparse(const uint16_t* __restrict__ idx, const float* __restrict__ val, size_t entries, uint32_t chunk,
                  uint32_t keep, size_t n, float* __restrict__ param, float lr)
{
    const size_t e = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= entries) return;
    const uint32_t q = idx[e];
    if (q == 0xFFFFu) return;
    const size_t i = (e / keep) * chunk + q;
    if (i < n) param[i] = param[i] - lr * val[e];
}

// General case: the chunk's decoded gradient is built in LDS (+0 everywhere, then the kept entries), and every
// element is updated as in k_decompress_sgd.  One workgroup per chunk, RPW rows per wave.
template <int RPW, bool MOM, bool WD>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_decompress_sgd_topk(const uint16_t* __restrict__ idx, const float* __restrict__ val, size_t n, uint32_t chunk,
                      uint32_t keep, float* __restrict__ param, float* __restrict__ mbuf, float lr, float mu, float wd)
{
    extern __shared__ float s_g[];   // chunk floats
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63;

    // parameters (and momentum) do not depend on the decode: request them first
    f4 p[RPW], m[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        p[i] = f4{0.f, 0.f, 0.f, 0.f};
        m[i] = p[i];
        if (remain > 0) {
            p[i] = load_row(param + base + off, lane, remain, 0.0f);
            if (MOM) m[i] = load_row(mbuf + base + off, lane, remain, 0.0f);
        }
    }
    for (uint32_t e = threadIdx.x * 4; e < chunk; e += blockDim.x * 4)
        *reinterpret_cast<f4*>(s_g + e) = f4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    for (uint32_t s = threadIdx.x; s < keep; s += blockDim.x) {
        const uint32_t q = idx[c * keep + s];
        if (q != 0xFFFFu && q < chunk) s_g[q] = val[c * keep + s];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        if (remain <= 0) continue;
        f4 g = *reinterpret_cast<const f4*>(s_g + off + lane * 4);
        if (WD) {
            g.x = g.x + wd * p[i].x;
            g.y = g.y + wd * p[i].y;
            g.z = g.z + wd * p[i].z;
            g.w = g.w + wd * p[i].w;
        }
        f4 u = g;
        if (MOM) {
            m[i].x = mu * m[i].x + g.x;
            m[i].y = mu * m[i].y + g.y;
            m[i].z = mu * m[i].z + g.z;
            m[i].w = mu * m[i].w + g.w;
            store_row(mbuf + base + off, lane, remain, m[i]);
            u = m[i];
        }
        p[i].x = p[i].x - lr * u.x;
        p[i].y = p[i].y - lr * u.y;
        p[i].z = p[i].z - lr * u.z;
        p[i].w = p[i].w - lr * u.w;
        store_row(param + base + off, lane, remain, p[i]);
    }
}

// Adam-type update after a top-K round: the chunk's decoded tensor is built in LDS as above, then every element is
// updated as in k_decompress_adam.
template <int RPW, bool FROZEN, bool WD>
__global__ void __launch_bounds__(wg_threads_max(RPW))
k_decompress_adam_topk(const uint16_t* __restrict__ idx, const float* __restrict__ val, size_t n, uint32_t chunk,
                       uint32_t keep, float* __restrict__ param, float* __restrict__ mbuf, float* __restrict__ vbuf,
                       float lr, float beta1, float omb1, float beta2, float omb2, float eps, float wd)
{
    extern __shared__ float s_g[];   // chunk floats
    const size_t c = blockIdx.x;
    const size_t base = c * static_cast<size_t>(chunk);
    const int len = static_cast<int>((n - base < chunk) ? (n - base) : chunk);
    const int wave = wave_index(), lane = threadIdx.x & 63;

    // parameters and optimizer state do not depend on the decode: request them first
    f4 p[RPW], m[RPW], v[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        p[i] = f4{0.f, 0.f, 0.f, 0.f};
        m[i] = p[i];
        v[i] = f4{1.f, 1.f, 1.f, 1.f};
        if (remain > 0) {
            p[i] = load_row(param + base + off, lane, remain, 0.0f);
            v[i] = load_row(vbuf + base + off, lane, remain, 1.0f);
            if (!FROZEN) m[i] = load_row(mbuf + base + off, lane, remain, 0.0f);
        }
    }
    for (uint32_t e = threadIdx.x * 4; e < chunk; e += blockDim.x * 4)
        *reinterpret_cast<f4*>(s_g + e) = f4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    for (uint32_t s = threadIdx.x; s < keep; s += blockDim.x) {
        const uint32_t q = idx[c * keep + s];
        if (q != 0xFFFFu && q < chunk) s_g[q] = val[c * keep + s];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        if (remain <= 0) continue;
        const f4 d = *reinterpret_cast<const f4*>(s_g + off + lane * 4);
        f4 mi = d;
        if (!FROZEN) {
            mi.x = beta1 * m[i].x + omb1 * d.x;
            mi.y = beta1 * m[i].y + omb1 * d.y;
            mi.z = beta1 * m[i].z + omb1 * d.z;
            mi.w = beta1 * m[i].w + omb1 * d.w;
            v[i].x = beta2 * v[i].x + omb2 * (d.x * d.x);
            v[i].y = beta2 * v[i].y + omb2 * (d.y * d.y);
            v[i].z = beta2 * v[i].z + omb2 * (d.z * d.z);
            v[i].w = beta2 * v[i].w + omb2 * (d.w * d.w);
            store_row(vbuf + base + off, lane, remain, v[i]);
        }
        store_row(mbuf + base + off, lane, remain, mi);
        f4 u;
        u.x = mi.x / (sqrtf(v[i].x) + eps);
        u.y = mi.y / (sqrtf(v[i].y) + eps);
        u.z = mi.z / (sqrtf(v[i].z) + eps);
        u.w = mi.w / (sqrtf(v[i].w) + eps);
        if (WD) {
            u.x = u.x + wd * p[i].x;
            u.y = u.y + wd * p[i].y;
            u.z = u.z + wd * p[i].z;
            u.w = u.w + wd * p[i].w;
        }
        p[i].x = p[i].x - lr * u.x;
        p[i].y = p[i].y - lr * u.y;
        p[i].z = p[i].z - lr * u.z;
        p[i].w = p[i].w - lr * u.w;
        store_row(param + base + off, lane, remain, p[i]);
    }
}

}  // namespace bagua

using namespace bagua;

extern "C" int bagua_decompress_sgd_step(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                                         float* param, float* momentum_buf, float lr, float momentum,
                                         float weight_decay, void* stream)
{
    if (codec != BAGUA_CODEC_MINMAX_U8 && codec != BAGUA_CODEC_SIGN1) return BAGUA_ERR_INVALID_ARG;
    if (!codes || !meta || !param || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    {
        const size_t nc = num_chunks(n, chunk);
        RangeCheck rc;
        rc.reads(codes, codec == BAGUA_CODEC_MINMAX_U8 ? n : ((n + 31) / 32) * sizeof(uint32_t));
        rc.reads(meta, (codec == BAGUA_CODEC_MINMAX_U8 ? 2 * nc : nc) * sizeof(float));
        rc.writes(param, n * sizeof(float));
        rc.writes(momentum_buf, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    const size_t rows = (n + kRow - 1) / kRow;
    if ((rows + kRowWaves - 1) / kRowWaves > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(codes) || !aligned4(meta) || !aligned16(param) || !aligned16(momentum_buf)) return BAGUA_ERR_ALIGNMENT;
    dim3 grid(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves)), block(kWave * kRowWaves);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t ch = static_cast<uint32_t>(chunk);
    const bool mom = momentum_buf != nullptr, wd = weight_decay != 0.0f;
#define BAGUA_SGD(CODEC, MOMv, WDv)                                                                          \
    hipLaunchKernelGGL((k_decompress_sgd<CODEC, MOMv, WDv>), grid, block, 0, s, codes, meta, n, ch, param, \
                       momentum_buf, lr, momentum, weight_decay)
#define BAGUA_SGD_CODEC(CODEC)                       \
    if (mom && wd) BAGUA_SGD(CODEC, true, true);     \
    else if (mom) BAGUA_SGD(CODEC, true, false);     \
    else if (wd) BAGUA_SGD(CODEC, false, true);      \
    else BAGUA_SGD(CODEC, false, false);
    if (codec == BAGUA_CODEC_MINMAX_U8) { BAGUA_SGD_CODEC(BAGUA_CODEC_MINMAX_U8) }
    else { BAGUA_SGD_CODEC(BAGUA_CODEC_SIGN1) }
#undef BAGUA_SGD_CODEC
#undef BAGUA_SGD
    return launch_status();
}

extern "C" int bagua_decompress_adam_step(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                                          float* param, float* m, float* v, float lr, float beta1, float beta2,
                                          float eps, float weight_decay, int variance_frozen, void* stream)
{
    if (codec != BAGUA_CODEC_MINMAX_U8 && codec != BAGUA_CODEC_SIGN1) return BAGUA_ERR_INVALID_ARG;
    if (!codes || !meta || !param || !m || !v || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    {
        const size_t nc = num_chunks(n, chunk);
        RangeCheck rc;
        rc.reads(codes, codec == BAGUA_CODEC_MINMAX_U8 ? n : ((n + 31) / 32) * sizeof(uint32_t));
        rc.reads(meta, (codec == BAGUA_CODEC_MINMAX_U8 ? 2 * nc : nc) * sizeof(float));
        rc.writes(param, n * sizeof(float));
        rc.writes(m, n * sizeof(float));
        rc.writes(v, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    const size_t rows = (n + kRow - 1) / kRow;
    if ((rows + kRowWaves - 1) / kRowWaves > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(codes) || !aligned4(meta) || !aligned16(param) || !aligned16(m) || !aligned16(v))
        return BAGUA_ERR_ALIGNMENT;
    dim3 grid(static_cast<unsigned>((rows + kRowWaves - 1) / kRowWaves)), block(kWave * kRowWaves);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t ch = static_cast<uint32_t>(chunk);
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    const bool frozen = variance_frozen != 0, wd = weight_decay != 0.0f;
#define BAGUA_ADAM(CODEC, FRv, WDv)                                                                            \
    hipLaunchKernelGGL((k_decompress_adam<CODEC, FRv, WDv>), grid, block, 0, s, codes, meta, n, ch, param, m, \
                       v, lr, beta1, omb1, beta2, omb2, eps, weight_decay)
#define BAGUA_ADAM_CODEC(CODEC)                        \
    if (frozen && wd) BAGUA_ADAM(CODEC, true, true);   \
    else if (frozen) BAGUA_ADAM(CODEC, true, false);   \
    else if (wd) BAGUA_ADAM(CODEC, false, true);       \
    else BAGUA_ADAM(CODEC, false, false);
    if (codec == BAGUA_CODEC_MINMAX_U8) { BAGUA_ADAM_CODEC(BAGUA_CODEC_MINMAX_U8) }
    else { BAGUA_ADAM_CODEC(BAGUA_CODEC_SIGN1) }
#undef BAGUA_ADAM_CODEC
#undef BAGUA_ADAM
    return launch_status();
}

extern "C" int bagua_decompress_sgd_step_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep,
                                              float* param, float* momentum_buf, float lr, float momentum,
                                              float weight_decay, void* stream)
{
    if (!idx || !val || !param || n == 0 || !chunk_ok(chunk) || keep < 1 || keep > chunk) return BAGUA_ERR_INVALID_ARG;
    const size_t nc = num_chunks(n, chunk);
    {
        RangeCheck rc;
        rc.reads(idx, nc * keep * sizeof(uint16_t));
        rc.reads(val, nc * keep * sizeof(float));
        rc.writes(param, n * sizeof(float));
        rc.writes(momentum_buf, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    if (nc > kMaxGrid || (nc * keep + 255) / 256 > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned2(idx) || !aligned4(val) || !aligned16(param) || !aligned16(momentum_buf)) return BAGUA_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t ch = static_cast<uint32_t>(chunk), kp = static_cast<uint32_t>(keep);
    const bool mom = momentum_buf != nullptr, wd = weight_decay != 0.0f;
    // lr * (+0) must be +0 for the sparse form to equal the dense update: lr finite with a clear sign bit
    if (!mom && !wd && std::isfinite(lr) && !std::signbit(lr)) {
        const size_t entries = nc * keep;
        hipLaunchKernelGGL(k_sgd_topk_sparse, dim3(static_cast<unsigned>((entries + 255) / 256)), dim3(256), 0, s, idx, val,
                           entries, ch, kp, n, param, lr);
        return launch_status();
    }
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, 2);
    dim3 grid(static_cast<unsigned>(nc)), block(64 * ((rows + rpw - 1) / rpw));
    const size_t lds = chunk * sizeof(float);
#define BAGUA_TS(MOMv, WDv)                                                                                      \
    BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_decompress_sgd_topk<RPW, MOMv, WDv>), grid, block, lds, s, idx, \
                                               val, n, ch, kp, param, momentum_buf, lr, momentum, weight_decay))
    if (mom && wd) { BAGUA_TS(true, true) }
    else if (mom) { BAGUA_TS(true, false) }
    else if (wd) { BAGUA_TS(false, true) }
    else { BAGUA_TS(false, false) }
#undef BAGUA_TS
    return launch_status();
}

extern "C" int bagua_decompress_adam_step_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep,
                                               float* param, float* m, float* v, float lr, float beta1, float beta2,
                                               float eps, float weight_decay, int variance_frozen, void* stream)
{
    if (!idx || !val || !param || !m || !v || n == 0 || !chunk_ok(chunk) || keep < 1 || keep > chunk)
        return BAGUA_ERR_INVALID_ARG;
    const size_t nc = num_chunks(n, chunk);
    {
        RangeCheck rc;
        rc.reads(idx, nc * keep * sizeof(uint16_t));
        rc.reads(val, nc * keep * sizeof(float));
        rc.writes(param, n * sizeof(float));
        rc.writes(m, n * sizeof(float));
        rc.writes(v, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    if (nc > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned2(idx) || !aligned4(val) || !aligned16(param) || !aligned16(m) || !aligned16(v)) return BAGUA_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t ch = static_cast<uint32_t>(chunk), kp = static_cast<uint32_t>(keep);
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    const bool frozen = variance_frozen != 0, wd = weight_decay != 0.0f;
    const int rows = static_cast<int>(chunk / kRow);
    const int rpw = pick_rpw(rows, 2);
    dim3 grid(static_cast<unsigned>(nc)), block(64 * ((rows + rpw - 1) / rpw));
    const size_t lds = chunk * sizeof(float);
#define BAGUA_TA(FRv, WDv)                                                                                         \
    BAGUA_DISPATCH_RPW(rpw, hipLaunchKernelGGL((k_decompress_adam_topk<RPW, FRv, WDv>), grid, block, lds, s, idx,  \
                                               val, n, ch, kp, param, m, v, lr, beta1, omb1, beta2, omb2, eps,     \
                                               weight_decay))
    if (frozen && wd) { BAGUA_TA(true, true) }
    else if (frozen) { BAGUA_TA(true, false) }
    else if (wd) { BAGUA_TA(false, true) }
    else { BAGUA_TA(false, false) }
#undef BAGUA_TA
    return launch_status();
}
