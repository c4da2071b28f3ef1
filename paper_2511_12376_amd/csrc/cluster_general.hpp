// Host entry points of the multi-pass cluster path (any even group length, or one group per tensor).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace bitsnap {

bool cluster_general_supported(int64_t n, int64_t group);
size_t cluster_general_workspace_bytes(int64_t n, int64_t group);
int cluster_general_quantize(const float *x, int64_t n, int64_t group, int m, uint8_t *codes, uint8_t *labels,
                             float *params, float *fit_out, const float *fit_in, uint32_t *status, void *workspace,
                             hipStream_t s);
int cluster_general_dequantize(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                               int64_t group, int m, float *out, hipStream_t s);

}  // namespace bitsnap
