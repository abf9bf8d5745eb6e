// C-ABI entry points that dispatch over the codec (see include/bagua_hip.h), and status strings.
#include "batch.hpp"
#include "launchers.hpp"

using namespace bagua;

extern "C" const char* bagua_status_string(int status)
{
    switch (status) {
        case BAGUA_OK: return "BAGUA_OK";
        case BAGUA_ERR_INVALID_ARG: return "BAGUA_ERR_INVALID_ARG";
        case BAGUA_ERR_ALIGNMENT: return "BAGUA_ERR_ALIGNMENT";
        case BAGUA_ERR_LAUNCH: return "BAGUA_ERR_LAUNCH";
        case BAGUA_ERR_UNSUPPORTED: return "BAGUA_ERR_UNSUPPORTED";
        default: return "BAGUA_ERR_UNKNOWN";
    }
}

extern "C" int bagua_decompress_reduce_recompress(int codec, const void* const* codes_in, const float* const* meta_in,
                                                  int k, float* server_residual, size_t n, size_t chunk,
                                                  void* codes_out, float* meta_out, float* out_fp32, void* stream)
{
    if (codec != BAGUA_CODEC_MINMAX_U8 && codec != BAGUA_CODEC_SIGN1) return BAGUA_ERR_INVALID_ARG;
    if (!codes_in || !meta_in || k < 1 || k > BAGUA_MAX_WORKERS || !codes_out || !meta_out || n == 0 ||
        !chunk_ok(chunk))
        return BAGUA_ERR_INVALID_ARG;
    for (int j = 0; j < k; ++j) {
        if (!codes_in[j] || !meta_in[j]) return BAGUA_ERR_INVALID_ARG;
    }
    const size_t nc = num_chunks(n, chunk);
    const size_t code_bytes = codec == BAGUA_CODEC_MINMAX_U8 ? n : ((n + 31) / 32) * sizeof(uint32_t);
    const size_t meta_bytes = (codec == BAGUA_CODEC_MINMAX_U8 ? 2 * nc : nc) * sizeof(float);
    RangeCheck rc;
    for (int j = 0; j < k; ++j) {
        rc.reads(codes_in[j], code_bytes);
        rc.reads(meta_in[j], meta_bytes);
    }
    rc.writes(server_residual, n * sizeof(float));
    rc.writes(codes_out, code_bytes);
    rc.writes(meta_out, meta_bytes);
    rc.writes(out_fp32, n * sizeof(float));
    if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    if (num_chunks(n, chunk) > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    for (int j = 0; j < k; ++j)
        if (!aligned16(codes_in[j]) || !aligned4(meta_in[j])) return BAGUA_ERR_ALIGNMENT;
    if (!aligned16(server_residual) || !aligned16(codes_out) || !aligned4(meta_out) || !aligned16(out_fp32))
        return BAGUA_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (codec == BAGUA_CODEC_MINMAX_U8)
        return launch_drr_minmax(codes_in, meta_in, k, server_residual, n, chunk, static_cast<uint8_t*>(codes_out),
                                 meta_out, out_fp32, s);
    return launch_drr_sign(codes_in, meta_in, k, server_residual, n, chunk, static_cast<uint32_t*>(codes_out),
                           meta_out, out_fp32, s);
}

extern "C" int bagua_decompress_reduce_recompress_batched(int codec, const void* const* codes_in,
                                                          const float* const* meta_in, int k,
                                                          float* const* server_residual, const size_t* n, size_t B,
                                                          size_t chunk, void* const* codes_out, float* const* meta_out,
                                                          float* const* out_fp32, void* workspace,
                                                          size_t workspace_bytes, void* stream)
{
    if (codec != BAGUA_CODEC_MINMAX_U8 && codec != BAGUA_CODEC_SIGN1) return BAGUA_ERR_INVALID_ARG;
    if (!codes_in || !meta_in || k < 1 || k > BAGUA_MAX_WORKERS || !n || !codes_out || !meta_out || !workspace ||
        B == 0 || B > 0xffffffffu || !chunk_ok(chunk))
        return BAGUA_ERR_INVALID_ARG;
    if (workspace_bytes < bagua_batch_workspace_bytes(B, k)) return BAGUA_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return BAGUA_ERR_ALIGNMENT;
    const bool minmax = codec == BAGUA_CODEC_MINMAX_U8;
    const bool ef = server_residual != nullptr, with_out = out_fp32 != nullptr;
    const size_t ew = 5 + 2 * static_cast<size_t>(k);   // <= batch_entry_words_for(k)
    std::vector<uint64_t> table(batch_table_words(B, ew), 0);
    uint64_t* entries = table.data() + batch_first_words(B);
    RangeList rl;
    size_t total = 0;
    for (size_t b = 0; b < B; ++b) {
        if (n[b] == 0 || !codes_out[b] || !meta_out[b] || (ef && !server_residual[b]) || (with_out && !out_fp32[b]))
            return BAGUA_ERR_INVALID_ARG;
        const size_t nc = num_chunks(n[b], chunk);
        const size_t code_bytes = minmax ? n[b] : ((n[b] + 31) / 32) * sizeof(uint32_t);
        const size_t meta_bytes = (minmax ? 2 * nc : nc) * sizeof(float);
        float* eps = ef ? server_residual[b] : nullptr;
        float* out = with_out ? out_fp32[b] : nullptr;
        if (!aligned16(eps) || !aligned16(codes_out[b]) || !aligned4(meta_out[b]) || !aligned16(out)) return BAGUA_ERR_ALIGNMENT;
        uint64_t* e = entries + b * ew;
        for (int j = 0; j < k; ++j) {
            const void* cj = codes_in[b * k + j];
            const float* mj = meta_in[b * k + j];
            if (!cj || !mj) return BAGUA_ERR_INVALID_ARG;
            if (!aligned16(cj) || !aligned4(mj)) return BAGUA_ERR_ALIGNMENT;
            rl.reads(cj, code_bytes);
            rl.reads(mj, meta_bytes);
            e[5 + j] = reinterpret_cast<uintptr_t>(cj);
            e[5 + k + j] = reinterpret_cast<uintptr_t>(mj);
        }
        rl.writes(eps, n[b] * sizeof(float));
        rl.writes(codes_out[b], code_bytes);
        rl.writes(meta_out[b], meta_bytes);
        rl.writes(out, n[b] * sizeof(float));
        table[b] = total;
        e[0] = reinterpret_cast<uintptr_t>(eps);
        e[1] = reinterpret_cast<uintptr_t>(codes_out[b]);
        e[2] = reinterpret_cast<uintptr_t>(meta_out[b]);
        e[3] = reinterpret_cast<uintptr_t>(out);
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
    if (minmax) return launch_drr_minmax_batched(workspace, B, k, total, chunk, ef, with_out, s);
    return launch_drr_sign_batched(workspace, B, k, total, chunk, ef, with_out, s);
}

extern "C" int bagua_decompress(int codec, const void* codes, const float* meta, size_t n, size_t chunk, float* out,
                                void* stream)
{
    if (codec != BAGUA_CODEC_MINMAX_U8 && codec != BAGUA_CODEC_SIGN1) return BAGUA_ERR_INVALID_ARG;
    if (!codes || !meta || !out || n == 0 || !chunk_ok(chunk)) return BAGUA_ERR_INVALID_ARG;
    {
        const size_t nc = num_chunks(n, chunk);
        RangeCheck rc;
        rc.reads(codes, codec == BAGUA_CODEC_MINMAX_U8 ? n : ((n + 31) / 32) * sizeof(uint32_t));
        rc.reads(meta, (codec == BAGUA_CODEC_MINMAX_U8 ? 2 * nc : nc) * sizeof(float));
        rc.writes(out, n * sizeof(float));
        if (!rc.disjoint()) return BAGUA_ERR_INVALID_ARG;
    }
    if (((n + kRow - 1) / kRow + 3) / 4 > kMaxGrid) return BAGUA_ERR_UNSUPPORTED;
    if (!aligned16(codes) || !aligned4(meta) || !aligned16(out)) return BAGUA_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (codec == BAGUA_CODEC_MINMAX_U8)
        return launch_decompress_minmax(static_cast<const uint8_t*>(codes), meta, n, chunk, out, s);
    return launch_decompress_sign(static_cast<const uint32_t*>(codes), meta, n, chunk, out, s);
}
