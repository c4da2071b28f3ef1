/* A C caller of the CPU oracle for runs under AddressSanitizer / UndefinedBehaviorSanitizer (host code only):
 * every buffer is allocated at exactly the size the oracle's comments promise, so a read or write one
 * element too far is a heap overflow the sanitizer reports.  Built and run by tests/test_oracle_sanitizers.py.
 * Cases: the ragged and degenerate sizes (n = 0, 1, 7, 9, 4097, odd n with its nibble tail), cluster-major
 * codes with a short last group, one group per tensor (G = 0), a table map, both element widths. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t oracle_encode_sparse(const uint16_t *, const uint16_t *, int64_t, uint8_t *, uint16_t *);
int64_t oracle_encode_sparse_naive(const uint16_t *, const uint16_t *, int64_t, uint8_t *, uint16_t *);
void oracle_tile_offsets(const uint8_t *, int64_t, int64_t, uint64_t *);
void oracle_decode_sparse(const uint16_t *, const uint8_t *, const uint16_t *, int64_t, uint16_t *);
int64_t oracle_encode_sparse_ex(const uint16_t *, const uint16_t *, int64_t, int, uint8_t *, uint16_t *, uint16_t *);
void oracle_decode_sparse_ex(const uint16_t *, const uint8_t *, const uint16_t *, int64_t, int, uint16_t *);
int64_t oracle_encode_sparse32_ex(const uint32_t *, const uint32_t *, int64_t, int, uint8_t *, uint32_t *, uint32_t *);
void oracle_decode_sparse32_ex(const uint32_t *, const uint8_t *, const uint32_t *, int64_t, int, uint32_t *);
void oracle_quantize_cluster(const float *, int64_t, int64_t, int, const float *, uint8_t *, uint8_t *, float *, float *);
void oracle_dequantize_cluster(const uint8_t *, const uint8_t *, const float *, int64_t, int64_t, int, float *);
void oracle_quantize_cluster_ex(const float *, int64_t, int64_t, int, const float *, const float *, int, uint8_t *,
                                uint8_t *, float *, float *);
void oracle_dequantize_cluster_ex(const uint8_t *, const uint8_t *, const float *, int64_t, int64_t, int, const float *,
                                  int, float *);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void)
{
    state ^= state << 13, state ^= state >> 7, state ^= state << 17;
    return (uint32_t)(state >> 32);
}
static void *exact(size_t bytes) { return malloc(bytes ? bytes : 1); }  /* malloc(0) may return NULL */
static int failures = 0;
#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) {                                                     \
            printf("FAILED %s (line %d)\n", #c, __LINE__);              \
            failures += 1;                                              \
        }                                                               \
    } while (0)

static void sparse_case(int64_t n, unsigned changed_per_256)
{
    uint16_t *cur = exact((size_t)n * 2), *base = exact((size_t)n * 2), *payload = exact((size_t)n * 2),
             *out = exact((size_t)n * 2), *nb = exact((size_t)n * 2);
    uint8_t *mask = exact((size_t)((n + 7) / 8)), *flags = exact((size_t)n);
    int64_t want = 0;
    for (int64_t i = 0; i < n; ++i) {
        base[i] = (uint16_t)next_u32();
        const int ch = (next_u32() & 255u) < changed_per_256;
        cur[i] = ch ? (uint16_t)(base[i] ^ (1u + next_u32() % 65535u)) : base[i];
        want += ch;
    }
    CHECK(oracle_encode_sparse(cur, base, n, mask, payload) == want);
    oracle_decode_sparse(base, mask, payload, n, out);
    CHECK(memcmp(out, cur, (size_t)n * 2) == 0);
    CHECK(oracle_encode_sparse_naive(cur, base, n, flags, payload) == want);
    const int64_t tile = 8, tiles = (n + tile - 1) / tile;
    uint64_t *off = exact((size_t)(tiles + 1) * 8);  /* ceil(n/tile) + 1 entries: the last one is n_c */
    oracle_tile_offsets(mask, n, tile, off);
    CHECK((int64_t)off[tiles] == want);
    for (int delta = 0; delta < 2; ++delta) {
        CHECK(oracle_encode_sparse_ex(cur, base, n, delta, mask, payload, nb) == want);
        CHECK(memcmp(nb, cur, (size_t)n * 2) == 0);
        oracle_decode_sparse_ex(base, mask, payload, n, delta, out);
        CHECK(memcmp(out, cur, (size_t)n * 2) == 0);
    }
    /* the base array itself as the new base */
    memcpy(nb, base, (size_t)n * 2);
    CHECK(oracle_encode_sparse_ex(cur, nb, n, 0, mask, payload, nb) == want);
    CHECK(memcmp(nb, cur, (size_t)n * 2) == 0);
    free(cur), free(base), free(payload), free(out), free(nb), free(mask), free(flags), free(off);

    uint32_t *c32 = exact((size_t)n * 4), *b32 = exact((size_t)n * 4), *p32 = exact((size_t)n * 4), *o32 = exact((size_t)n * 4);
    uint8_t *m32 = exact((size_t)((n + 7) / 8));
    want = 0;
    for (int64_t i = 0; i < n; ++i) {
        b32[i] = next_u32();
        const int ch = (next_u32() & 255u) < changed_per_256;
        c32[i] = ch ? b32[i] ^ (1u << (next_u32() & 31u)) : b32[i];
        want += ch;
    }
    for (int delta = 0; delta < 2; ++delta) {
        CHECK(oracle_encode_sparse32_ex(c32, b32, n, delta, m32, p32, NULL) == want);
        oracle_decode_sparse32_ex(b32, m32, p32, n, delta, o32);
        CHECK(memcmp(o32, c32, (size_t)n * 4) == 0);
    }
    free(c32), free(b32), free(p32), free(o32), free(m32);
}

static float gauss(void)
{
    const double u1 = (next_u32() + 1.0) / 4294967297.0, u2 = next_u32() / 4294967296.0;
    return (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2));
}

static void cluster_case(int64_t n, int64_t G, int m, int use_table, int major)
{
    const int64_t groups = n <= 0 ? 0 : (G <= 0 || G >= n ? 1 : (n + G - 1) / G);
    float *x = exact((size_t)n * 4), *out = exact((size_t)n * 4), *params = exact((size_t)groups * m * 2 * 4),
          *fit = exact((size_t)groups * (2 + m - 1) * 4), *fit_in = exact((size_t)groups * 2 * 4), qmap[256];
    uint8_t *codes = exact((size_t)n), *labels = exact((size_t)((n + 1) / 2));
    for (int64_t i = 0; i < n; ++i)
        x[i] = 1e-3f * gauss() + (i % 97 == 0 ? 0.5f : 0.0f);
    for (int j = 0; j < 256; ++j)
        qmap[j] = (float)(j * j) / (255.0f * 255.0f);
    oracle_quantize_cluster(x, n, G, m, NULL, codes, labels, params, fit);
    oracle_dequantize_cluster(codes, labels, params, n, G, m, out);
    for (int64_t g = 0; g < groups; ++g)
        fit_in[2 * g] = fit[g * (2 + m - 1)], fit_in[2 * g + 1] = fit[g * (2 + m - 1) + 1];
    oracle_quantize_cluster(x, n, G, m, fit_in, codes, labels, params, NULL);
    oracle_quantize_cluster_ex(x, n, G, m, NULL, use_table ? qmap : NULL, major, codes, labels, params, fit);
    oracle_dequantize_cluster_ex(codes, labels, params, n, G, m, use_table ? qmap : NULL, major, out);
    for (int64_t i = 0; i < n; ++i)
        CHECK(isfinite(out[i]));
    free(x), free(out), free(params), free(fit), free(fit_in), free(codes), free(labels);
}

int main(void)
{
    const int64_t sizes[] = {0, 1, 7, 8, 9, 63, 65, 4095, 4097, 12345};
    for (size_t k = 0; k < sizeof sizes / sizeof sizes[0]; ++k) {
        sparse_case(sizes[k], 0), sparse_case(sizes[k], 16), sparse_case(sizes[k], 256);
        for (int opt = 0; opt < 4; ++opt) {
            cluster_case(sizes[k], 4096, 16, opt & 1, opt >> 1);
            cluster_case(sizes[k], 256, 5, opt & 1, opt >> 1);
            cluster_case(sizes[k], 0, 16, opt & 1, opt >> 1);   /* one group per tensor: the group buffer is malloc'ed */
            cluster_case(sizes[k], 1024, 1, opt & 1, opt >> 1);
        }
    }
    printf(failures ? "oracle_sanitize: %d check(s) failed\n" : "oracle_sanitize: ok\n", failures);
    return failures ? 1 : 0;
}
