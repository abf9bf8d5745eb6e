// Statistics + quantisation of one chunk held in registers (MinMax-u8 codec).
#pragma once
#include "common.hpp"

#pragma clang fp contract(off)

namespace bagua {

// Chunk-wide (min, max) of the values held by the waves of one workgroup, in two phases so that a
// caller can put the statistics of several chunks behind one barrier.
// Phase 1: this wave's (min, max) over its valid elements (`len` = valid elements of the chunk; rows
// beyond it are ignored); with several waves the pair is also parked in s_red (2*kMaxWaves floats).
template <int RPW>
__device__ __forceinline__ void chunk_minmax_partial(const f4 (&v)[RPW], int len, int wave, int lane, int nwaves,
                                                     float* s_red, float& mn_out, float& mx_out)
{
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int remain = len - static_cast<int>(wave * RPW + i) * kRow;
        if (remain >= kRow) {
            mn = fminf(fminf(mn, v[i].x), fminf(v[i].y, fminf(v[i].z, v[i].w)));
            mx = fmaxf(fmaxf(mx, v[i].x), fmaxf(v[i].y, fmaxf(v[i].z, v[i].w)));
        } else if (remain > 0) {
            const int e = lane * 4;
            if (e + 0 < remain) { mn = fminf(mn, v[i].x); mx = fmaxf(mx, v[i].x); }
            if (e + 1 < remain) { mn = fminf(mn, v[i].y); mx = fmaxf(mx, v[i].y); }
            if (e + 2 < remain) { mn = fminf(mn, v[i].z); mx = fmaxf(mx, v[i].z); }
            if (e + 3 < remain) { mn = fminf(mn, v[i].w); mx = fmaxf(mx, v[i].w); }
        }
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if (nwaves > 1 && lane == 0) {
        s_red[wave] = mn;
        s_red[kMaxWaves + wave] = mx;
    }
    mn_out = mn;
    mx_out = mx;
}
// Phase 2 (after a barrier when nwaves > 1): combine the waves' pairs; result canonicalised (-0 -> +0).
__device__ __forceinline__ void chunk_minmax_finish(int nwaves, const float* s_red, float& mn, float& mx)
{
    if (nwaves > 1) {
        for (int w = 0; w < nwaves; ++w) {
            mn = fminf(mn, s_red[w]);
            mx = fmaxf(mx, s_red[kMaxWaves + w]);
        }
    }
    mn = mn + 0.0f;
    mx = mx + 0.0f;
}
template <int RPW>
__device__ __forceinline__ void chunk_minmax(const f4 (&v)[RPW], int len, int wave, int lane, int nwaves,
                                             float* s_red, float& mn_out, float& mx_out)
{
    chunk_minmax_partial<RPW>(v, len, wave, lane, nwaves, s_red, mn_out, mx_out);
    if (nwaves > 1) __syncthreads();
    chunk_minmax_finish(nwaves, s_red, mn_out, mx_out);
}

// One quantised element: q = clamp(rint((v - mn) * inv), 0, 255) as a float, deq = mn + q * step.
__device__ __forceinline__ float quantise(float v, float mn, float inv)
{
    const float d = v - mn;
    const float t = d * inv;
    float q = rintf(t);
    q = (q >= 0.0f) ? q : 0.0f;  // also sends NaN to 0
    q = (q > 255.0f) ? 255.0f : q;
    return q;
}

__device__ __forceinline__ uint32_t pack_codes(float q0, float q1, float q2, float q3)
{
    // q are integer-valued floats in [0,255]: the conversion is exact whatever its rounding
    uint32_t w = 0;
    w = __builtin_amdgcn_cvt_pk_u8_f32(q0, 0, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(q1, 1, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(q2, 2, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(q3, 3, w);
    return w;
}

template <int RPW, bool EF, bool OUT, bool DEQ_BACK>
__device__ __forceinline__ void minmax_quantise_chunk(f4 (&v)[RPW], float mn, float mx, int len, int wave, int lane,
                                                      float* __restrict__ residual, uint8_t* __restrict__ codes,
                                                      float* __restrict__ minmax_c, float* __restrict__ out);

// Encode the chunk held in v: writes codes, (min,max), and optionally the updated residual
// (v - decode) and the decoded values.  Pointers are already offset to the start of the chunk.
// If DEQ_BACK, v is overwritten with the decoded values (used by the decentralised LP kernel).
template <int RPW, bool EF, bool OUT, bool DEQ_BACK = false>
__device__ __forceinline__ void minmax_encode_chunk(f4 (&v)[RPW], int len, int wave, int lane, int nwaves,
                                                    float* __restrict__ residual, uint8_t* __restrict__ codes,
                                                    float* __restrict__ minmax_c, float* __restrict__ out,
                                                    float* s_red)
{
    float mn, mx;
    chunk_minmax<RPW>(v, len, wave, lane, nwaves, s_red, mn, mx);
    minmax_quantise_chunk<RPW, EF, OUT, DEQ_BACK>(v, mn, mx, len, wave, lane, residual, codes, minmax_c, out);
}

// Quantise the chunk held in v given its canonical (min, max): writes codes, (min,max), and optionally the
// updated residual (v - decode) and the decoded values; if DEQ_BACK, v is overwritten with the decoded values.
template <int RPW, bool EF, bool OUT, bool DEQ_BACK>
__device__ __forceinline__ void minmax_quantise_chunk(f4 (&v)[RPW], float mn, float mx, int len, int wave, int lane,
                                                      float* __restrict__ residual, uint8_t* __restrict__ codes,
                                                      float* __restrict__ minmax_c, float* __restrict__ out)
{
    const float r = mx - mn;
    const float step = (r == 0.0f) ? 0.0f : r / 255.0f;
    const float inv = (r == 0.0f) ? 0.0f : 255.0f / r;  // flat chunk: (v - mn) * 0 = 0 -> code 0
    if (threadIdx.x == 0) {
        minmax_c[0] = mn;
        minmax_c[1] = mx;
    }
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        if (remain <= 0) continue;
        const float q0 = quantise(v[i].x, mn, inv), q1 = quantise(v[i].y, mn, inv);
        const float q2 = quantise(v[i].z, mn, inv), q3 = quantise(v[i].w, mn, inv);
        store_codes_row(codes + off, lane, remain, pack_codes(q0, q1, q2, q3));
        if (EF || OUT || DEQ_BACK) {
            f4 deq;
            deq.x = mn + q0 * step;
            deq.y = mn + q1 * step;
            deq.z = mn + q2 * step;
            deq.w = mn + q3 * step;
            if (EF) {
                f4 e;
                e.x = v[i].x - deq.x;
                e.y = v[i].y - deq.y;
                e.z = v[i].z - deq.z;
                e.w = v[i].w - deq.w;
                store_row(residual + off, lane, remain, e);
            }
            if (OUT) store_row(out + off, lane, remain, deq);
            if (DEQ_BACK) v[i] = deq;
        }
    }
}

}  // namespace bagua
