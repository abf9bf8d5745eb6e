// Internal host-side launch functions, one per kernel family.  Arguments are already validated.
#pragma once
#include "common.hpp"

namespace bagua {

int launch_compress_minmax(const float* x, float* residual, size_t n, size_t chunk, uint8_t* codes,
                           float* minmax, hipStream_t stream);
int launch_drr_minmax(const void* const* codes_in, const float* const* meta_in, int k, float* eps, size_t n,
                      size_t chunk, uint8_t* codes_out, float* minmax_out, float* out, hipStream_t stream);
int launch_drr_minmax_batched(const void* workspace, size_t B, int k, size_t total_chunks, size_t chunk, bool ef,
                              bool with_out, hipStream_t stream);
int launch_drr_sign_batched(const void* workspace, size_t B, int k, size_t total_chunks, size_t chunk, bool ef,
                            bool with_out, hipStream_t stream);
int launch_decompress_minmax(const uint8_t* codes, const float* minmax, size_t n, size_t chunk, float* out,
                             hipStream_t stream);

int launch_sign_compress(const float* x, float* residual, size_t n, size_t chunk, uint32_t* bits, float* scale,
                         hipStream_t stream);
int launch_drr_sign(const void* const* bits_in, const float* const* scale_in, int k, float* eps, size_t n,
                    size_t chunk, uint32_t* bits_out, float* scale_out, float* out, hipStream_t stream);
int launch_decompress_sign(const uint32_t* bits, const float* scale, size_t n, size_t chunk, float* out,
                           hipStream_t stream);

}  // namespace bagua
