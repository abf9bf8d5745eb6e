// Statistics + encoding of one chunk held in registers (1-bit sign codec): the fixed-order |v| sum, the nibble
// gather into 32-bit sign words, and the error-state / decoded-value stores.
#pragma once
#include "common.hpp"

#pragma clang fp contract(off)

namespace bagua {

// Sum of |v| over the chunk in the fixed order (see bagua_sign_compress_ef in the header).
// s_q: LDS, rows*64 floats, used only when the chunk is spread over several waves.
template <int RPW>
__device__ __forceinline__ float chunk_abs_sum(const f4 (&v)[RPW], int rows, int wave, int lane, int nwaves,
                                               float* s_q)
{
    float acc = 0.0f;
    if (nwaves == 1) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            if (i < rows) {
                const float p = fabsf(v[i].x) + fabsf(v[i].y);
                const float q = fabsf(v[i].z) + fabsf(v[i].w);
                acc = acc + (p + q);
            }
        }
    } else {
        // rows are accumulated in row order, which crosses waves: park the per-row group sums in LDS
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int row = wave * RPW + i;
            if (row < rows) {
                const float p = fabsf(v[i].x) + fabsf(v[i].y);
                const float q = fabsf(v[i].z) + fabsf(v[i].w);
                s_q[row * kWave + lane] = p + q;
            }
        }
        __syncthreads();
        for (int row = 0; row < rows; ++row) acc = acc + s_q[row * kWave + lane];
    }
    return wave_butterfly_sum(acc);
}

// OR of the 4-bit nibbles of the 8 lanes that share one 32-bit sign word.
__device__ __forceinline__ uint32_t gather_word(uint32_t nib, int lane)
{
    uint32_t w = nib << (4 * (lane & 7));
    w |= __shfl_xor(w, 1, kWave);
    w |= __shfl_xor(w, 2, kWave);
    w |= __shfl_xor(w, 4, kWave);
    return w;
}

// bit ? sc : -sc for a sign bit that has been shifted to bit 31 of t; the bits of t below bit 31 are arbitrary.
// sc and -sc differ in the sign bit only, so selecting sc's bits where t is set and (-sc)'s elsewhere gives exactly
// the two-way choice (one bit-field insert instead of test + compare + select).
__device__ __forceinline__ float sign_select(uint32_t t, uint32_t sc_bits, uint32_t neg_bits)
{
    return __uint_as_float((t & sc_bits) | (~t & neg_bits));
}

// Encode the chunk held in v (absent elements must be +0.0f).  `bits` points at the word of the
// chunk's first element; residual/out point at the chunk's first element.
template <int RPW, bool EF, bool OUT>
__device__ __forceinline__ void sign_encode_chunk(f4 (&v)[RPW], int len, uint32_t chunk, int wave, int lane,
                                                  int nwaves, float* __restrict__ residual,
                                                  uint32_t* __restrict__ bits, float* __restrict__ scale_c,
                                                  float* __restrict__ out, float* s_q)
{
    const int rows = static_cast<int>((len + kRow - 1) / kRow);
    const float sum = chunk_abs_sum<RPW>(v, rows, wave, lane, nwaves, s_q);
    const bool pow2 = (chunk & (chunk - 1)) == 0;
    float scale;
    if (len == static_cast<int>(chunk) && pow2) scale = sum * (1.0f / static_cast<float>(chunk));
    else scale = sum / static_cast<float>(len);
    if (threadIdx.x == 0) *scale_c = scale;
    const float neg = -scale;
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int off = static_cast<int>(wave * RPW + i) * kRow;
        const int remain = len - off;
        if (remain <= 0) continue;
        const bool full = remain >= kRow;   // wave-uniform: a complete row needs no per-element tail tests
        bool b0 = v[i].x >= 0.0f, b1 = v[i].y >= 0.0f, b2 = v[i].z >= 0.0f, b3 = v[i].w >= 0.0f;
        if (!full) {
            const int e = lane * 4;
            b0 = b0 && (e + 0 < remain);
            b1 = b1 && (e + 1 < remain);
            b2 = b2 && (e + 2 < remain);
            b3 = b3 && (e + 3 < remain);
        }
        const uint32_t nib = (b0 ? 1u : 0u) | (b1 ? 2u : 0u) | (b2 ? 4u : 0u) | (b3 ? 8u : 0u);
        const uint32_t w = gather_word(nib, lane);
        if ((lane & 7) == 0 && (full || static_cast<int>(lane >> 3) * 32 < remain)) bits[(off >> 5) + (lane >> 3)] = w;
        if (EF || OUT) {
            f4 deq;
            deq.x = b0 ? scale : neg;
            deq.y = b1 ? scale : neg;
            deq.z = b2 ? scale : neg;
            deq.w = b3 ? scale : neg;
            if (EF) {
                f4 r;
                r.x = v[i].x - deq.x;
                r.y = v[i].y - deq.y;
                r.z = v[i].z - deq.z;
                r.w = v[i].w - deq.w;
                store_row(residual + off, lane, full ? kRow : remain, r);
            }
            if (OUT) store_row(out + off, lane, full ? kRow : remain, deq);
        }
    }
}

}  // namespace bagua
