/*
 * Memory-safety self-test of the CPU oracle (test infrastructure): every oracle function is run on
 * ragged sizes with heap buffers of exactly the documented size, so that AddressSanitizer /
 * UndefinedBehaviorSanitizer (the test builds this file with -fsanitize=address,undefined) flag any
 * out-of-bounds access, misuse or undefined arithmetic.  Prints "oracle selftest ok" on success.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_compress_minmax_u8(const float*, float*, size_t, size_t, uint8_t*, float*);
int oracle_decompress_minmax_u8(const uint8_t*, const float*, size_t, size_t, float*);
int oracle_drr_minmax_u8(const uint8_t* const*, const float* const*, int, float*, size_t, size_t, uint8_t*, float*, float*);
int oracle_ring_avg_fp(const float* const*, float* const*, int, size_t);
int oracle_ring_avg_lp(const float* const*, float* const*, float* const*, uint8_t* const*, float* const*, int, size_t, size_t);
int oracle_sign_compress_ef(const float*, float*, size_t, size_t, uint32_t*, float*);
int oracle_decompress_sign(const uint32_t*, const float*, size_t, size_t, float*);
int oracle_drr_sign(const uint32_t* const*, const float* const*, int, float*, size_t, size_t, uint32_t*, float*, float*);
int oracle_bucket_flatten(const float* const*, const size_t*, const size_t*, size_t, float*, size_t);
int oracle_decompress_sgd_step(int, const void*, const float*, size_t, size_t, float*, float*, float, float, float);
int oracle_peer_avg_fp(const float* const*, float* const*, const int*, int, size_t);
int oracle_reduce_compress_minmax_u8(const float* const*, int, float*, size_t, size_t, uint8_t*, float*);
void oracle_set_threads(int);

static uint32_t rng_state = 12345u;
static float rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((float)(rng_state >> 8) / 16777216.0f - 0.5f) * 2e-3f;
}
static float* fbuf(size_t n)
{
    float* p = (float*)malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
#define CHECK(x) do { if ((x) != 0) { printf("FAILED %s line %d\n", #x, __LINE__); return 1; } } while (0)

static int run(size_t n, size_t C, int k)
{
    size_t nc = (n + C - 1) / C, nw = (n + 31) / 32;
    float *x[8], *res[8], *mm[8], *sc[8], *xo[8], *hat[8];
    uint8_t* codes[8];
    uint32_t* bits[8];
    for (int j = 0; j < k; ++j) {
        x[j] = fbuf(n); res[j] = fbuf(n); xo[j] = fbuf(n); hat[j] = fbuf(n);
        mm[j] = (float*)malloc(2 * nc * sizeof(float)); sc[j] = (float*)malloc(nc * sizeof(float));
        codes[j] = (uint8_t*)malloc(n); bits[j] = (uint32_t*)malloc(nw * sizeof(uint32_t));
        CHECK(oracle_compress_minmax_u8(x[j], res[j], n, C, codes[j], mm[j]));
        CHECK(oracle_compress_minmax_u8(x[j], NULL, n, C, codes[j], mm[j]));
        CHECK(oracle_sign_compress_ef(x[j], res[j], n, C, bits[j], sc[j]));
    }
    float *eps = fbuf(n), *out = fbuf(n), *mo = (float*)malloc(2 * nc * sizeof(float)), *so = (float*)malloc(nc * sizeof(float));
    uint8_t* co = (uint8_t*)malloc(n);
    uint32_t* bo = (uint32_t*)malloc(nw * sizeof(uint32_t));
    CHECK(oracle_drr_minmax_u8((const uint8_t* const*)codes, (const float* const*)mm, k, eps, n, C, co, mo, out));
    CHECK(oracle_drr_minmax_u8((const uint8_t* const*)codes, (const float* const*)mm, k, NULL, n, C, co, mo, NULL));
    CHECK(oracle_decompress_minmax_u8(co, mo, n, C, out));
    CHECK(oracle_drr_sign((const uint32_t* const*)bits, (const float* const*)sc, k, eps, n, C, bo, so, out));
    CHECK(oracle_decompress_sign(bo, so, n, C, out));
    CHECK(oracle_ring_avg_fp((const float* const*)x, xo, k, n));
    CHECK(oracle_ring_avg_lp((const float* const*)x, xo, hat, codes, mm, k, n, C));
    CHECK(oracle_decompress_sgd_step(0, co, mo, n, C, x[0], res[0], 0.1f, 0.9f, 0.01f));
    CHECK(oracle_decompress_sgd_step(1, bo, so, n, C, x[0], NULL, 0.1f, 0.0f, 0.0f));
    int peer[8];
    for (int j = 0; j < k; ++j) peer[j] = (j ^ 1) < k ? (j ^ 1) : j;
    CHECK(oracle_peer_avg_fp((const float* const*)x, xo, peer, k, n));
    CHECK(oracle_reduce_compress_minmax_u8((const float* const*)x, k, res[0], n, C, co, mo));
    /* flatten: the k buffers as tensors with one-element gaps */
    size_t numel[8], offs[8], pos = 0;
    for (int j = 0; j < k; ++j) { numel[j] = n / (size_t)(j + 1); offs[j] = pos + (size_t)(j % 2); pos = offs[j] + numel[j]; }
    float* bucket = (float*)malloc((pos + 3) * sizeof(float));
    CHECK(oracle_bucket_flatten((const float* const*)x, numel, offs, (size_t)k, bucket, pos + 3));
    free(bucket); free(eps); free(out); free(mo); free(so); free(co); free(bo);
    for (int j = 0; j < k; ++j) { free(x[j]); free(res[j]); free(xo[j]); free(hat[j]); free(mm[j]); free(sc[j]); free(codes[j]); free(bits[j]); }
    return 0;
}

int main(void)
{
    const size_t sizes[] = {1, 31, 33, 255, 256, 257, 1023, 4095, 4097, 2 * 4096 + 7};
    const size_t chunks[] = {256, 768, 4096};
    for (int threads = 1; threads <= 4; threads += 3) {
        oracle_set_threads(threads);
        for (size_t a = 0; a < sizeof(sizes) / sizeof(sizes[0]); ++a)
            for (size_t b = 0; b < sizeof(chunks) / sizeof(chunks[0]); ++b)
                for (int k = 1; k <= 8; k += 3)
                    if (run(sizes[a], chunks[b], k)) return 1;
    }
    printf("oracle selftest ok\n");
    return 0;
}
