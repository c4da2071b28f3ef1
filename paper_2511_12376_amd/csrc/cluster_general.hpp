// Host entry points of the multi-pass cluster path (any even group length, or one group per tensor).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/bitsnap.h"

namespace bitsnap {

bool cluster_general_supported(int64_t n, int64_t group);
size_t cluster_general_workspace_bytes(int64_t n, int64_t group);
int cluster_general_quantize(const float *x, int64_t n, int64_t group, int m, uint8_t *codes, uint8_t *labels,
                             float *params, float *fit_out, const float *fit_in, uint32_t *status, void *workspace,
                             hipStream_t s);
int cluster_general_dequantize(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                               int64_t group, int m, float *out, hipStream_t s);

// The same with the format options (a table for the quantisation map, cluster-major codes); with
// `major` the workspace also holds the per-chunk cluster counts, and dequantisation needs it too.
size_t cluster_general_workspace_bytes_ex(int64_t n, int64_t group, bool major);
int cluster_general_quantize_ex(const float *x, int64_t n, int64_t group, int m, bool major, const float *qmap,
                                uint8_t *codes, uint8_t *labels, float *params, float *fit_out, const float *fit_in,
                                uint32_t *status, void *workspace, hipStream_t s);
int cluster_general_dequantize_ex(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                                  int64_t group, int m, bool major, const float *qmap, float *out, void *workspace,
                                  hipStream_t s);

// A list of tensors with one group each (the batched form of group = 0): items[i].first_group
// counts the 4096-element chunks of all earlier items, total_chunks all of them.
size_t cluster_list_workspace_bytes(int64_t total_chunks, int64_t count, bool major);
int cluster_list_quantize(const bitsnap_cluster_item *items, int64_t count, int64_t total_chunks, int m, bool major,
                          const float *qmap, uint32_t *status, void *workspace, hipStream_t s);
int cluster_list_dequantize(const bitsnap_cluster_item *items, int64_t count, int64_t total_chunks, int m, bool major,
                            const float *qmap, void *workspace, hipStream_t s);

// K (float4 per lane) of the one-wave-per-group kernels for a group length, or 0 when the length
// needs the multi-pass path.
inline int one_wave_group_k(int64_t group)
{
    switch (group) {
    case 256: return 1;
    case 512: return 2;
    case 1024: return 4;
    case 2048: return 8;
    case 4096: return 16;
    default: return 0;
    }
}

}  // namespace bitsnap
