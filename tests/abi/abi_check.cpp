// A caller of libbitsnap that is not Python: plain HIP runtime calls for memory, the C ABI for
// the codecs, and the CPU oracle (linked in as C) to check every output bit for bit.
// Built by __graft_entry__.build(); run by tests/test_gpu_abi.py.  Exit status 0 = all checks passed.
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/bitsnap.h"

extern "C" {
int64_t oracle_encode_sparse(const uint16_t *cur, const uint16_t *base, int64_t n, uint8_t *mask, uint16_t *payload);
void oracle_quantize_cluster(const float *x, int64_t n, int64_t G, int m, const float *fit_in, uint8_t *codes,
                             uint8_t *labels, float *params, float *fit_out);
void oracle_dequantize_cluster(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n, int64_t G,
                               int m, float *out);
}

#define CHECK_HIP(call)                                                          \
    do {                                                                         \
        hipError_t e_ = (call);                                                  \
        if (e_ != hipSuccess) {                                                  \
            fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));           \
            return 2;                                                            \
        }                                                                        \
    } while (0)
#define CHECK_RC(call)                                                           \
    do {                                                                         \
        int rc_ = (call);                                                        \
        if (rc_ != BITSNAP_OK) {                                                 \
            fprintf(stderr, "%s: %s\n", #call, bitsnap_error_string(rc_));       \
            return 3;                                                            \
        }                                                                        \
    } while (0)
#define REQUIRE(cond)                                                            \
    do {                                                                         \
        if (!(cond)) {                                                           \
            fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__);    \
            return 1;                                                            \
        }                                                                        \
    } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13, rng_state ^= rng_state >> 7, rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}

int main(void)
{
    const int64_t n = 5 * 32768 + 4321;  // several tiles / groups and a ragged end
    const int64_t G = 4096;
    const int m = 16;
    printf("abi_check: library version %d, n = %lld\n", bitsnap_version(), (long long)n);
    fflush(stdout);

    // ---- sparse pair
    uint16_t *cur = (uint16_t *)malloc(n * 2), *base = (uint16_t *)malloc(n * 2), *back = (uint16_t *)malloc(n * 2);
    for (int64_t i = 0; i < n; ++i) {
        base[i] = (uint16_t)rnd();
        cur[i] = (rnd() % 100 < 30) ? (uint16_t)(base[i] ^ (1u + rnd() % 65535u)) : base[i];
    }
    const size_t mask_bytes = bitsnap_sparse_mask_bytes(n), ws_bytes = bitsnap_sparse_workspace_bytes(n);
    void *d_cur, *d_base, *d_mask, *d_pay, *d_out, *d_ws, *d_cnt;
    CHECK_HIP(hipMalloc(&d_cur, n * 2));
    CHECK_HIP(hipMalloc(&d_base, n * 2));
    CHECK_HIP(hipMalloc(&d_mask, mask_bytes));
    CHECK_HIP(hipMalloc(&d_pay, n * 2));
    CHECK_HIP(hipMalloc(&d_out, n * 2));
    CHECK_HIP(hipMalloc(&d_ws, ws_bytes));
    CHECK_HIP(hipMalloc(&d_cnt, 8));
    CHECK_HIP(hipMemset(d_ws, 0, ws_bytes));  // once; the library keeps it usable afterwards
    CHECK_HIP(hipMemcpy(d_cur, cur, n * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_base, base, n * 2, hipMemcpyHostToDevice));
    CHECK_RC(bitsnap_encode_sparse(d_cur, d_base, n, 2, (uint8_t *)d_mask, d_pay, n, NULL, (uint64_t *)d_cnt, d_ws, ws_bytes,
                                   NULL));
    CHECK_RC(bitsnap_decode_sparse(d_base, (const uint8_t *)d_mask, d_pay, n, n, 2, d_out, NULL, d_ws, ws_bytes, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    uint64_t n_changed = 0;
    uint8_t *mask = (uint8_t *)malloc(mask_bytes), *o_mask = (uint8_t *)malloc(mask_bytes);
    uint16_t *pay = (uint16_t *)malloc(n * 2), *o_pay = (uint16_t *)malloc(n * 2);
    CHECK_HIP(hipMemcpy(&n_changed, d_cnt, 8, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(mask, d_mask, mask_bytes, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(pay, d_pay, n * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(back, d_out, n * 2, hipMemcpyDeviceToHost));
    const int64_t o_nc = oracle_encode_sparse(cur, base, n, o_mask, o_pay);
    REQUIRE((int64_t)n_changed == o_nc);
    REQUIRE(memcmp(mask, o_mask, (size_t)((n + 7) / 8)) == 0);
    REQUIRE(memcmp(pay, o_pay, (size_t)o_nc * 2) == 0);
    REQUIRE(memcmp(back, cur, (size_t)n * 2) == 0);
    printf("abi_check: sparse pair ok (%lld of %lld changed)\n", (long long)o_nc, (long long)n);
    fflush(stdout);

    // ---- cluster pair
    const size_t groups = bitsnap_cluster_groups(n, G);
    float *x = (float *)malloc(n * 4), *xh = (float *)malloc(n * 4), *o_xh = (float *)malloc(n * 4);
    for (int64_t i = 0; i < n; ++i) {  // a sum of uniforms: bell-shaped, like optimizer states
        float s = 0.0f;
        for (int k = 0; k < 6; ++k)
            s += (float)(rnd() >> 8) * (1.0f / 16777216.0f);
        x[i] = (s - 3.0f) * 1e-3f;
    }
    const size_t label_bytes = bitsnap_cluster_label_bytes(n), param_bytes = bitsnap_cluster_param_bytes(n, G, m);
    const size_t fit_floats = bitsnap_cluster_fit_floats(n, G, m);
    void *d_x, *d_codes, *d_labels, *d_params, *d_fit, *d_xh;
    CHECK_HIP(hipMalloc(&d_x, n * 4));
    CHECK_HIP(hipMalloc(&d_codes, n));
    CHECK_HIP(hipMalloc(&d_labels, label_bytes));
    CHECK_HIP(hipMalloc(&d_params, param_bytes));
    CHECK_HIP(hipMalloc(&d_fit, fit_floats * 4));
    CHECK_HIP(hipMalloc(&d_xh, n * 4));
    CHECK_HIP(hipMemcpy(d_x, x, n * 4, hipMemcpyHostToDevice));
    CHECK_RC(bitsnap_quantize_cluster((const float *)d_x, n, G, m, (uint8_t *)d_codes, (uint8_t *)d_labels, (float *)d_params,
                                      (float *)d_fit, NULL, NULL, NULL, 0, NULL));
    CHECK_RC(bitsnap_dequantize_cluster((const uint8_t *)d_codes, (const uint8_t *)d_labels, (const float *)d_params, n, G, m,
                                        (float *)d_xh, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    uint8_t *codes = (uint8_t *)malloc(n), *labels = (uint8_t *)malloc(label_bytes);
    uint8_t *o_codes = (uint8_t *)malloc(n), *o_labels = (uint8_t *)malloc(label_bytes);
    float *params = (float *)malloc(param_bytes), *o_params = (float *)malloc(param_bytes);
    float *fit = (float *)malloc(fit_floats * 4), *o_fit = (float *)malloc(fit_floats * 4), *fit_in = (float *)malloc(groups * 8);
    CHECK_HIP(hipMemcpy(codes, d_codes, n, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(labels, d_labels, label_bytes, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(params, d_params, param_bytes, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(fit, d_fit, fit_floats * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(xh, d_xh, n * 4, hipMemcpyDeviceToHost));
    for (size_t g = 0; g < groups; ++g) {  // the oracle takes the library's (mu, sigma): a floating reduction's order may differ
        fit_in[2 * g] = fit[g * (m + 1)];
        fit_in[2 * g + 1] = fit[g * (m + 1) + 1];
    }
    oracle_quantize_cluster(x, n, G, m, fit_in, o_codes, o_labels, o_params, o_fit);
    oracle_dequantize_cluster(o_codes, o_labels, o_params, n, G, m, o_xh);
    REQUIRE(memcmp(codes, o_codes, (size_t)n) == 0);
    REQUIRE(memcmp(labels, o_labels, label_bytes) == 0);
    REQUIRE(memcmp(params, o_params, param_bytes) == 0);
    REQUIRE(memcmp(fit, o_fit, fit_floats * 4) == 0);
    REQUIRE(memcmp(xh, o_xh, (size_t)n * 4) == 0);
    printf("abi_check: cluster pair ok (%zu groups)\n", groups);

    // ---- a rejected call touches nothing and says why
    REQUIRE(bitsnap_quantize_cluster((const float *)d_x, n, G, 17, (uint8_t *)d_codes, (uint8_t *)d_labels, (float *)d_params, NULL,
                                     NULL, NULL, NULL, 0, NULL) == BITSNAP_E_SIZE);
    REQUIRE(bitsnap_encode_sparse(d_cur, d_base, n, 2, (uint8_t *)d_mask, d_pay, n, NULL, (uint64_t *)d_cnt, NULL, 0, NULL) ==
            BITSNAP_E_NULL);
    printf("abi_check: all checks passed\n");
    return 0;
}
