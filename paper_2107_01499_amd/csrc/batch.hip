// Table upload for the batched entry points (see batch.hpp) and the workspace size query.
#include "batch.hpp"

namespace bagua {

__global__ void __launch_bounds__(kUploadWords)
k_upload_words(UploadBlob blob, uint32_t words, uint64_t* __restrict__ dst)
{
    if (threadIdx.x < words) dst[threadIdx.x] = blob.w[threadIdx.x];
}

int batch_upload(const uint64_t* host, size_t words, uint64_t* dst, hipStream_t stream)
{
    for (size_t w0 = 0; w0 < words; w0 += kUploadWords) {
        UploadBlob blob;
        const uint32_t count = static_cast<uint32_t>(std::min<size_t>(kUploadWords, words - w0));
        for (uint32_t i = 0; i < count; ++i) blob.w[i] = host[w0 + i];
        for (uint32_t i = count; i < kUploadWords; ++i) blob.w[i] = 0;
        hipLaunchKernelGGL(k_upload_words, dim3(1), dim3(kUploadWords), 0, stream, blob, count, dst + w0);
    }
    return launch_status();
}

}  // namespace bagua

using namespace bagua;

extern "C" size_t bagua_batch_workspace_bytes(size_t B, int k)
{
    if (k < 0 || k > BAGUA_MAX_WORKERS) return 0;
    return batch_table_words(B, batch_entry_words_for(k)) * sizeof(uint64_t);
}
