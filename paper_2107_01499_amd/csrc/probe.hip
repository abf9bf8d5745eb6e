// Measurement utilities for the benchmark: what this GPU's memory system delivers for plain access patterns of
// the same shape as the primitives' traffic (ceilings quoted next to the roofline; no arithmetic of the method).
#include "common.hpp"

namespace bagua {

// Read-only reduction: a wave sums kProbeRows consecutive 256-element rows (one 128-bit load per lane and row, all in
// flight together); the four waves of a workgroup combine their sums in LDS and one lane writes the workgroup's sum.
constexpr int kProbeRows = 4;
constexpr int kProbeTile = 4 * kProbeRows * kRow;   // elements per workgroup
__global__ void __launch_bounds__(256)
k_probe_read(const float* __restrict__ x, size_t n, float* __restrict__ tile_sums)
{
    __shared__ float s_part[4];
    const int wave = wave_index(), lane = threadIdx.x & 63;
    const size_t e0 = (static_cast<size_t>(blockIdx.x) * 4 + wave) * kProbeRows * kRow;
    f4 v[kProbeRows];
#pragma unroll
    for (int r = 0; r < kProbeRows; ++r) {
        const size_t e = e0 + static_cast<size_t>(r) * kRow;
        v[r] = f4{0.f, 0.f, 0.f, 0.f};
        if (e < n) v[r] = load_row(x + e, lane, static_cast<int>((n - e < static_cast<size_t>(kRow)) ? (n - e) : kRow), 0.0f);
    }
    float s = 0.0f;
#pragma unroll
    for (int r = 0; r < kProbeRows; ++r) s = s + ((v[r].x + v[r].y) + (v[r].z + v[r].w));
    s = wave_butterfly_sum(s);
    if (lane == 0) s_part[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
}

// Stream mix: a wave owns one row and visits `seq` groups of streams one after another; in each group it reads
// the row from NR fp32 streams, then writes it to NW fp32 streams and NB byte streams (one dword per lane).
// PW waves per workgroup: one for a single group (the copy-like shapes: measured at 1.5 G elements per launch,
// 1R+1W 0.84 of peak with one wave per workgroup, 0.78 with two, 0.82 with four; 2R+1W in place 0.78-0.80 / 0.73-0.75 /
// 0.78), two when a wave visits several groups (the ring kernels' shape, where two measured fastest).  `pace` as in
// the worker-side kernels: wait for each load before the next is requested.
template <int NR, int NW, int NB, int PW>
__global__ void __launch_bounds__(kWave * PW)
k_probe_streams(PtrTable in, MutPtrTable out, MutPtrTable bout, int seq, size_t n, int pace)
{
    const size_t row = static_cast<size_t>(blockIdx.x) * PW + (PW > 1 ? wave_index() : 0);
    const int lane = threadIdx.x & 63;
    const size_t e0 = row * kRow;
    if (e0 >= n) return;
    f4 carry = f4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < seq; ++s) {
        f4 v[NR];
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            v[i] = ld_stream(reinterpret_cast<const f4*>(static_cast<const float*>(in.p[s * NR + i]) + e0) + lane);
            if (pace) pace_loads();
        }
        f4 acc = carry;
#pragma unroll
        for (int i = 0; i < NR; ++i) acc = acc + v[i];
#pragma unroll
        for (int i = 0; i < NW; ++i)
            st_stream(reinterpret_cast<f4*>(static_cast<float*>(out.p[s * NW + i]) + e0) + lane, acc);
#pragma unroll
        for (int i = 0; i < NB; ++i)
            st_stream(reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(bout.p[s * NB + i]) + e0) + lane,
                      __float_as_uint(acc.x));
        carry = v[0];
    }
}

}  // namespace bagua

using namespace bagua;

extern "C" int bagua_probe_read(const float* x, size_t n, float* tile_sums, void* stream)
{
    if (!x || !tile_sums || n == 0) return BAGUA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned4(tile_sums)) return BAGUA_ERR_ALIGNMENT;
    const size_t tiles = (n + kProbeTile - 1) / kProbeTile;
    if (tiles > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_probe_read, dim3(static_cast<unsigned>(tiles)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), x, n, tile_sums);
    return launch_status();
}

extern "C" int bagua_probe_streams(const float* const* in, float* const* out, uint8_t* const* bout, int nr, int nw,
                                   int nb, int seq, size_t n, void* stream)
{
    if (seq < 1 || nr < 1 || nw < 0 || nb < 0 || n == 0 || n % kRow != 0) return BAGUA_ERR_INVALID_ARG;
    if (seq * nr > BAGUA_MAX_WORKERS || seq * nw > BAGUA_MAX_WORKERS || seq * nb > BAGUA_MAX_WORKERS)
        return BAGUA_ERR_INVALID_ARG;
    if (!in || (nw && !out) || (nb && !bout)) return BAGUA_ERR_INVALID_ARG;
    PtrTable it{};
    MutPtrTable ot{}, bt{};
    for (int i = 0; i < seq * nr; ++i) {
        if (!in[i]) return BAGUA_ERR_INVALID_ARG;
        if (!aligned16(in[i])) return BAGUA_ERR_ALIGNMENT;
        it.p[i] = in[i];
    }
    for (int i = 0; i < seq * nw; ++i) {
        if (!out[i]) return BAGUA_ERR_INVALID_ARG;
        if (!aligned16(out[i])) return BAGUA_ERR_ALIGNMENT;
        ot.p[i] = out[i];
    }
    for (int i = 0; i < seq * nb; ++i) {
        if (!bout[i]) return BAGUA_ERR_INVALID_ARG;
        if (!aligned16(bout[i])) return BAGUA_ERR_ALIGNMENT;
        bt.p[i] = bout[i];
    }
    const size_t rows = n / kRow;
    const int pw = seq == 1 ? 1 : kRowWaves;
    const size_t groups = (rows + pw - 1) / pw;
    if (groups > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    dim3 grid(static_cast<unsigned>(groups)), block(kWave * pw);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int pace = pace_for(n);
#define BAGUA_PROBE(NR, NW, NB)                                                                                    \
    if (nr == NR && nw == NW && nb == NB) {                                                                        \
        if (pw == 1) hipLaunchKernelGGL((k_probe_streams<NR, NW, NB, 1>), grid, block, 0, s, it, ot, bt, seq, n, pace); \
        else hipLaunchKernelGGL((k_probe_streams<NR, NW, NB, kRowWaves>), grid, block, 0, s, it, ot, bt, seq, n, pace); \
        return launch_status();                                                                                    \
    }
    BAGUA_PROBE(1, 1, 0) BAGUA_PROBE(2, 1, 0) BAGUA_PROBE(2, 1, 1) BAGUA_PROBE(2, 2, 1) BAGUA_PROBE(4, 4, 0) BAGUA_PROBE(8, 8, 0)
    BAGUA_PROBE(1, 8, 0) BAGUA_PROBE(8, 1, 0)
#undef BAGUA_PROBE
    return BAGUA_ERR_UNSUPPORTED;
}
