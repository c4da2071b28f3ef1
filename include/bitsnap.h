/*
 * bitsnap.h - C ABI of libbitsnap: the per-tensor checkpoint codecs of BitSnap
 * (arXiv 2511.12376) as hand-written HIP kernels for gfx950 (MI355X).
 *
 *   encode_sparse / decode_sparse          bitmask-based delta sparsification of 16-bit model
 *                                          states (or 32-bit ones) against a base checkpoint
 *                                          (lossless)
 *   quantize_cluster / dequantize_cluster  cluster-based 8-bit quantisation of fp32 optimizer
 *                                          states (lossy, error bounded per cluster)
 *
 * Conventions for every call
 *   - Pointers are DEVICE pointers unless a parameter says "host".  The caller owns all
 *     buffers; the library never allocates or frees device memory.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream)
 *     and the call returns without waiting.  Outputs are valid once the stream has passed it.
 *   - Return value: BITSNAP_OK or a negative BITSNAP_E_* code.  Errors are found on the host
 *     before anything is launched; a rejected call has touched no buffer.
 *   - Tensors are flat and contiguous.  Pointers named below as "aligned" must be multiples
 *     of 16 bytes.  Input buffers that are aligned (cur, base, mask, payload, codes, labels, x) are
 *     read in whole 16-byte pieces: a buffer whose length is not a multiple of 16 bytes is read up
 *     to the next 16-byte boundary past its last element (never beyond that, and what lies there
 *     does not influence any output).  Any allocator that hands out 16-byte granules - hipMalloc,
 *     torch - satisfies this; a sub-buffer carved out of a larger one must leave those bytes
 *     readable.
 *   - Two calls that share a workspace must not overlap in time.
 */
#ifndef BITSNAP_H
#define BITSNAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *bitsnap_stream_t;

enum {
    BITSNAP_OK = 0,
    BITSNAP_E_NULL = -1,        /* a required pointer is NULL                              */
    BITSNAP_E_SIZE = -2,        /* n < 0, unsupported elem_bytes / m / group, n too large  */
    BITSNAP_E_ALIGN = -3,       /* a pointer that must be 16-byte aligned is not           */
    BITSNAP_E_WORKSPACE = -4,   /* workspace missing or smaller than *_workspace_bytes()   */
    BITSNAP_E_OFFSETS = -5,     /* tile_offsets requested but n >= 2^32                    */
    BITSNAP_E_LAUNCH = -6,      /* the HIP runtime refused the launch                      */
    BITSNAP_E_STATIC_LIMIT = -7 /* bitsnap_encode_sparse_static: more tiles than
                                   BITSNAP_STATIC_MAX_TILES                                */
};

/* Library version, major*10000 + minor*100 + patch. */
int bitsnap_version(void);

/* Static, NUL-terminated text for a return code (host pointer, never freed). */
const char *bitsnap_error_string(int code);

/* The bitsnap_debug_* entry points are measurement and test aids, not part of the codec's surface:
 * they may change or disappear between versions. */

/* Diagnostic: a plain 16-byte-per-lane streaming copy of `bytes` (a multiple of 16) from src to
 * dst, both aligned.  It moves exactly `bytes` in and `bytes` out, which makes it the yardstick
 * for HBM byte counters and for what a kernel without dependencies sustains on the same device. */
int bitsnap_debug_stream_copy(void *dst, const void *src, int64_t bytes, bitsnap_stream_t stream);

/* Diagnostic: streaming traffic with the byte mix and access pattern of the cluster codecs and
 * next to no arithmetic, i.e. what the memory system leaves to win for those kernels.
 *   wide [n] fp32, bytes [n], halves [n/2]: device buffers, aligned; n a multiple of 4096
 *   to_small != 0: reads wide, writes bytes and halves (quantize_cluster's 4 : 1.5 traffic)
 *   to_small == 0: reads bytes and halves, writes wide (dequantize_cluster's 1.5 : 4 traffic)
 * The values written are meaningless. */
int bitsnap_debug_stream_mix(void *wide, void *bytes, void *halves, int64_t n, int to_small,
                             bitsnap_stream_t stream);

/* ------------------------------------------------------------------------------------------
 * Sparse path.  Paper: "Bitmask Based Sparsification for Model States" (improved bitmask,
 * space n/8 + 2 n_c, Eq. improved-bitmask) and Algorithm 1.
 *
 * Format of one encoded tensor of n elements of 2 bytes (fp16 and bf16 are the same to the codec)
 * or 4 bytes:
 *   mask     bit i (byte i/8, bit position i%8, least significant first) is 1 iff the bit
 *            pattern of cur[i] differs from base[i]; padding bits are 0.  ceil(n/8) bytes count
 *            as stored data.
 *   payload  the changed elements of cur (the new values, not differences), in index order:
 *            n_c elements of 2 bytes.
 * ---------------------------------------------------------------------------------------- */

/* Number of elements covered by one entry of `tile_offsets`: 32768 two-byte elements ... */
size_t bitsnap_sparse_tile_elems(void);
/* ... or 16384 four-byte ones (a tile is 64 KB of input either way); 0 for any other width. */
size_t bitsnap_sparse_tile_elems_for(int elem_bytes);

/* Bytes the caller must provide for `mask`: ceil(n/8) rounded up to a multiple of 16.  The
 * bytes after ceil(n/8) are written as 0. */
size_t bitsnap_sparse_mask_bytes(int64_t n);

/* Bytes of workspace encode_sparse / decode_sparse need for a tensor of n elements (256 bytes
 * plus 128 per tile).  encode keeps its cross-workgroup scan state there (a count word and an
 * answer word per tile, the latter on a 64-byte slot of its own); decode the payload offset and
 * count of every tile.  It must contain zeros the first time it is used (any means:
 * hipMemset, torch.zeros); afterwards the kernels leave it ready for the next call, encode or
 * decode, of any size that fits, so one workspace serves a whole checkpoint. */
size_t bitsnap_sparse_workspace_bytes(int64_t n);
/* The same for elements of elem_bytes (2 or 4) bytes; bitsnap_sparse_workspace_bytes is the 2-byte case. */
size_t bitsnap_sparse_workspace_bytes_for(int64_t n, int elem_bytes);

/* Algorithm 1, steps 1-5, for one tensor.
 *   cur, base        [n] elements of elem_bytes bytes, aligned
 *   elem_bytes       2 (fp16 / bf16 model states, the paper's case) or 4 (fp32 states: the same
 *                    scheme with 4-byte values, n/8 + 4 n_c bytes stored); the element is changed
 *                    iff its whole bit pattern differs
 *   mask             [bitsnap_sparse_mask_bytes(n)] out, aligned
 *   payload          [payload_capacity_elems] elements out, aligned.  If more than
 *                    payload_capacity_elems elements changed, only the first
 *                    payload_capacity_elems are written; mask and n_changed are still complete,
 *                    so the caller can see the overflow (n_changed > capacity) and keep the
 *                    full tensor instead - the paper's own rule once n_c >= 15n/16.
 *   tile_offsets     nullable; [ceil(n/tile_elems)] out: number of changed elements before
 *                    each tile (the compaction offset of the tile)
 *   n_changed        [1] out, 8-byte aligned: n_c.  UINT64_MAX reports that the scan gave up
 *                    waiting (see bitsnap_debug_set_spin_limit); outputs are then unspecified
 *                    but every access stayed in bounds and the workspace is reusable.
 *   workspace        see bitsnap_sparse_workspace_bytes
 * n == 0 is legal and writes n_changed = 0. */
int bitsnap_encode_sparse(const void *cur, const void *base, int64_t n, int elem_bytes,
                          uint8_t *mask, void *payload, int64_t payload_capacity_elems,
                          uint32_t *tile_offsets, uint64_t *n_changed,
                          void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);

/* Inverse of encode_sparse: out[i] = bit i of mask ? next payload element : base[i].
 *   base             [n] elements of elem_bytes (2 or 4) bytes, aligned
 *   mask             [ceil(n/8)] bytes, aligned; bits at or beyond n are ignored
 *   payload          [payload_elems] elements, aligned.  Never read at or beyond payload_elems;
 *                    if the mask has more set bits than that, the surplus elements decode to 0.
 *   out              [n] elements, aligned; may be the same buffer as base (in-place patch)
 *   n_changed        nullable, [1] out: the number of set mask bits below n
 * Three launches: set bits per tile, payload offset per tile, then the merge, which has no
 * dependency between workgroups (nothing in decode waits, so it cannot give up); a tensor of at
 * most 8 tiles is decoded by one launch, in which every wavefront counts the mask before its part,
 * and one of at most 4096 tiles by two (the merge adds up the tile counts itself). */
int bitsnap_decode_sparse(const void *base, const uint8_t *mask, const void *payload,
                          int64_t payload_elems, int64_t n, int elem_bytes, void *out,
                          uint64_t *n_changed,
                          void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);

/* Options of the extended sparse entry points (flags). */
#define BITSNAP_SPARSE_DELTA 1u   /* the payload holds cur XOR base, not cur (see below) */
#define BITSNAP_SPARSE_OFFSETS 2u /* batched decode: every item carries the encoder's tile_offsets */

/* bitsnap_encode_sparse with two options.
 *   flags & BITSNAP_SPARSE_DELTA   the payload holds the non-zero elements of the delta states
 *                    themselves (the literal reading of what the section "Bitmask Based
 *                    Sparsification for Model States" stores beside the mask), with the delta of two
 *                    bit patterns taken bitwise, cur XOR base, which keeps the scheme lossless.  Mask, n_changed,
 *                    tile_offsets and the order of the payload do not depend on the flag.
 *   new_base         nullable; [n] elements out, aligned: receives a copy of cur, for the checkpoint that
 *                    becomes the base of the following delta checkpoints (the paper's interval
 *                    between base checkpoints).  May be the buffer `base` itself; must not overlap
 *                    cur, mask or payload.
 * flags == 0 and new_base == NULL is bitsnap_encode_sparse. */
int bitsnap_encode_sparse_ex(const void *cur, const void *base, int64_t n, int elem_bytes, uint32_t flags,
                             uint8_t *mask, void *payload, int64_t payload_capacity_elems,
                             uint32_t *tile_offsets, uint64_t *n_changed, void *new_base,
                             void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);

/* bitsnap_decode_sparse for a payload written with the same flags:
 * out[i] = bit i of mask ? (DELTA ? base[i] XOR next payload element : next payload element) : base[i].
 *   tile_offsets  nullable; [ceil(n / tile_elems)] uint32 in: the array the encoder wrote for this
 *                 tensor.  With it the decoder need not count the mask first (one launch instead of
 *                 two or three; it does so for tensors of up to 2048 tiles, where that is faster,
 *                 and counts as usual beyond); n must be below 2^32, and payload_elems must not be
 *                 below the number of changed elements.  Offsets that do not belong to the mask give unspecified output
 *                 values, inside out[0..n). */
int bitsnap_decode_sparse_ex(const void *base, const uint8_t *mask, const void *payload,
                             int64_t payload_elems, int64_t n, int elem_bytes, uint32_t flags,
                             const uint32_t *tile_offsets, void *out, uint64_t *n_changed,
                             void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);

/* bitsnap_encode_sparse for callers that cannot allocate device memory, not even a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * outputs and errors as bitsnap_encode_sparse, without the workspace: the scan state lives in a
 * device array inside the library (256 bytes + 128 per tile = 2 MiB + 256 bytes on every GPU the
 * call has run on, held until the process ends).  The call allocates and frees nothing.
 *   - a tensor of more than BITSNAP_STATIC_MAX_TILES tiles (536,870,912 two-byte or 268,435,456
 *     four-byte elements) is rejected with BITSNAP_E_STATIC_LIMIT before anything is launched;
 *   - all calls on one GPU share the one array: two of them that overlap in time (different
 *     streams, different threads) race, exactly like two calls that share a workspace;
 *   - the first call on a GPU also enqueues a small kernel that clears the array. */
#define BITSNAP_STATIC_MAX_TILES 16384
int bitsnap_encode_sparse_static(const void *cur, const void *base, int64_t n, int elem_bytes,
                                 uint8_t *mask, void *payload, int64_t payload_capacity_elems,
                                 uint32_t *tile_offsets, uint64_t *n_changed, bitsnap_stream_t stream);

/* Host-side knob for tests of the give-up path: the number of polls a workgroup spends waiting
 * for its tile's place in the payload (and the scanning wave for a tile's count) before it
 * reports failure through n_changed.  0 restores the
 * default (large enough never to trigger in normal operation).  The value is PROCESS-GLOBAL (one
 * atomic word, read by every later encode call on any thread, stream or device when it launches):
 * a test aid, not to be called by code that encodes concurrently on other threads.  The call does
 * nothing unless the environment variable BITSNAP_DEBUG_KNOBS is "1" when it is made. */
void bitsnap_debug_set_spin_limit(uint32_t polls);

/* ------------------------------------------------------------------------------------------
 * Cluster path.  Paper: "Cluster Based Quantization for Optimizer States" (Eq. qmap-distance,
 * S = max - min and b = min per cluster, Eq. decluster, size analysis) and Algorithm 2.
 *
 * The flat fp32 tensor is cut into groups of `group` consecutive elements (the last one may be
 * short); group == 0 means one group spanning the tensor, the paper's own formulation.  Each
 * group gets its own fit: mean and standard deviation -> m clusters bounded by the normal
 * quantiles mu + sigma * Phi^-1(k/m) -> label (uint4) per element -> per-cluster (S, b) ->
 * uint8 code = nearest of the 256 levels b + j*S/255.
 *
 *   codes   [n] uint8, element order
 *   labels  [ceil(n/2)] bytes, element 2i in the low nibble of byte i, element 2i+1 in the high
 *   params  [groups][m][2] fp32: (S, b) per cluster; (0, 0) for a cluster without members
 *   fit     [groups][2 + (m-1)] fp32: mu, sigma, e_1 .. e_{m-1}
 * Stored size per group: group + group/2 + 8m bytes (1.5 n + 128 per 4096 elements at m = 16).
 * ---------------------------------------------------------------------------------------- */

size_t bitsnap_cluster_groups(int64_t n, int64_t group);
size_t bitsnap_cluster_param_bytes(int64_t n, int64_t group, int m);
size_t bitsnap_cluster_label_bytes(int64_t n);
size_t bitsnap_cluster_fit_floats(int64_t n, int64_t group, int m);
size_t bitsnap_cluster_workspace_bytes(int64_t n, int64_t group, int m);

/* Host: the standard-normal quantile Phi^-1(k/m) the kernels use for edge k (0 < k < m <= 16);
 * 0.0 outside that range. */
double bitsnap_cluster_z(int k, int m);

/* Algorithm 2 for one tensor.
 *   x          [n] fp32, aligned
 *   group      0 (whole tensor) or the group length
 *   m          clusters, 1..16
 *   codes      [n] out, aligned;  labels [ceil(n/2)] out, aligned;  params out, aligned
 *   fit_out    nullable, [bitsnap_cluster_fit_floats] out
 *   fit_in     nullable, [groups][2]: use these (mu, sigma) instead of computing them
 *              (everything after step 1 of Algorithm 2 is a function of these two numbers)
 *   status     nullable, [1] uint32: bit 0 is OR-ed in when a group's mean or deviation is not
 *              finite (NaN/Inf in the input); that group's output is unspecified, in bounds
 *   workspace  [bitsnap_cluster_workspace_bytes]; may be NULL when that size is 0
 */
int bitsnap_quantize_cluster(const float *x, int64_t n, int64_t group, int m,
                             uint8_t *codes, uint8_t *labels, float *params,
                             float *fit_out, const float *fit_in, uint32_t *status,
                             void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);

/* Dequantisation and "decluster": out[i] = (codes[i] * (S/255)) + b with (S, b) of the cluster
 * labels[i] names in element i's group; values return to their original positions because
 * codes are kept in element order.   out [n] fp32, aligned. */
int bitsnap_dequantize_cluster(const uint8_t *codes, const uint8_t *labels, const float *params,
                               int64_t n, int64_t group, int m, float *out,
                               bitsnap_stream_t stream);

/* ------------------------------------------------------------------------------------------
 * Format variants of the cluster pair.
 *
 * qmap   nullable, DEVICE [256] fp32, 4-byte aligned: the map Q^map of Eq. qmap-distance as a
 *        table.  It must be non-decreasing (its contents cannot be checked on the host; with any
 *        other table the codes are unspecified, still 0..255).  code = the index of the entry
 *        nearest to t = (x-b)/S, the lowest such index where several are equally near, decided
 *        in fp32: t = fl32(fl32(x-b) * fl32(1/S)), distance fl32(|Q_j - t|); a cluster whose
 *        range cannot be coded (S = 0, or 1/S not finite) gets code 0.  Dequantisation maps the code
 *        back through the table, scales by S and adds b (the section's dequantisation formula):
 *        out = fl32(fl32(Q[code] * S) + b).  NULL = the linear map of
 *        the plain entry points (levels j/255, S/255 folded into one factor).
 * flags  BITSNAP_CLUSTER_MAJOR: the codes of a group are stored cluster by cluster - all of
 *        cluster 0, then cluster 1, ... - and inside a cluster in element order: the T_{C_i k}
 *        of Eq. decluster, which dequantisation undoes through the labels (V_j = T_{C_i k} with
 *        i = L_j, k = the number of earlier elements of the group with label i).  Labels stay in
 *        element order; params, fit and status are those of bitsnap_quantize_cluster.
 * group  as in the plain calls: 0 = the whole tensor is one group (the paper's formulation:
 *        one fit, and with BITSNAP_CLUSTER_MAJOR one cluster-major arrangement, per tensor).
 * workspace  [bitsnap_cluster_workspace_bytes_ex(n, group, m, flags)] bytes, 16-byte aligned;
 *        may be NULL when that is 0 (the group lengths 256 .. 4096).  Dequantisation uses it only
 *        with BITSNAP_CLUSTER_MAJOR, where it needs n < 2^32 (as does quantisation).
 * With qmap == NULL and flags == 0 these are the plain entry points.
 * ---------------------------------------------------------------------------------------- */
#define BITSNAP_CLUSTER_MAJOR 1u

size_t bitsnap_cluster_workspace_bytes_ex(int64_t n, int64_t group, int m, uint32_t flags);

int bitsnap_quantize_cluster_ex(const float *x, int64_t n, int64_t group, int m, uint32_t flags,
                                const float *qmap, uint8_t *codes, uint8_t *labels, float *params,
                                float *fit_out, const float *fit_in, uint32_t *status, void *workspace,
                                size_t workspace_bytes, bitsnap_stream_t stream);
int bitsnap_dequantize_cluster_ex(const uint8_t *codes, const uint8_t *labels, const float *params,
                                  int64_t n, int64_t group, int m, uint32_t flags, const float *qmap,
                                  float *out, void *workspace, size_t workspace_bytes,
                                  bitsnap_stream_t stream);

/* ------------------------------------------------------------------------------------------
 * Batched forms: one launch for a whole list of tensors.  The paper compresses an entire
 * state_dict per checkpoint (section "Details of Modifications"); a
 * launch per tensor leaves the device ramping up and draining a few thousand groups at a time.
 * Results are identical to calling the single-tensor entry point on every item.
 *
 * `items` is a DEVICE array written by the caller; its contents cannot be checked on the host:
 * every pointer in an item must meet the requirements of the single-tensor call, n must be > 0,
 * and first_group must be the number of groups, ceil(n/group), of all earlier items.
 * ---------------------------------------------------------------------------------------- */

typedef struct bitsnap_cluster_item {
    void *values;          /* quantize: const float* x [n] in;   dequantize: float* out [n]        */
    uint8_t *codes;        /* [n]          quantize: out, dequantize: in                            */
    uint8_t *labels;       /* [ceil(n/2)]  quantize: out, dequantize: in                            */
    float *params;         /* [groups][m][2]  quantize: out, dequantize: in                         */
    float *fit_out;        /* quantize only, nullable: [groups][m+1]                                */
    const float *fit_in;   /* quantize only, nullable: [groups][2]                                  */
    int64_t n;             /* elements                                                              */
    int64_t first_group;   /* index of this tensor's first group in the list-wide numbering         */
} bitsnap_cluster_item;

typedef struct bitsnap_sparse_item {
    const void *src;         /* encode: cur [n] in;                 decode: unused                      */
    const void *base;        /* [n] in                                                                  */
    uint8_t *mask;           /* encode: [bitsnap_sparse_mask_bytes(n)] out;   decode: [ceil(n/8)] in    */
    void *payload;           /* encode: [capacity] out;             decode: [capacity] in               */
    void *out;               /* decode: [n] out (may equal base);   encode: unused (_ex: new_base)      */
    uint64_t *n_changed;     /* [1] out; required for encode, nullable for decode                       */
    uint32_t *tile_offsets;  /* encode: nullable, [ceil(n/tile_elems)] out;   decode (_ex, OFFSETS): in */
    int64_t n;               /* elements, > 0                                                           */
    int64_t capacity;        /* encode: payload capacity in elements;   decode: payload elements        */
    int64_t first_tile;      /* sum of ceil(n/tile_elems) over all earlier items                        */
} bitsnap_sparse_item;

/* Workspace for a batched sparse call over total_tiles = sum of ceil(n/tile_elems); same rules as
 * bitsnap_sparse_workspace_bytes (zero once, then self-maintaining; a workspace of this size
 * also serves single-tensor calls of up to total_tiles tiles). */
size_t bitsnap_sparse_batch_workspace_bytes(int64_t total_tiles);

/* The scan restarts at every tensor: each item gets its own mask, payload and n_changed exactly
 * as from the single-tensor call.  If encode's scan gives up, every item's n_changed reads
 * UINT64_MAX. */
int bitsnap_encode_sparse_batched(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                  void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);
int bitsnap_decode_sparse_batched(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                  void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);

/* The batched calls with the options of bitsnap_encode_sparse_ex / bitsnap_decode_sparse_ex and the
 * element width (2 or 4; first_tile and total_tiles count tiles of bitsnap_sparse_tile_elems_for(elem_bytes)
 * elements).  In the encoder an item's `out`, where not NULL, is that tensor's new_base.  The decoder
 * takes BITSNAP_SPARSE_OFFSETS: every item's tile_offsets is the array the encoder wrote (every
 * n < 2^32; the caller sees to that), and a list of up to 2048 tiles is decoded in one launch (a longer
 * one is faster with the counting launches, and its offsets are left unused). */
int bitsnap_encode_sparse_batched_ex(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                     int elem_bytes, uint32_t flags, void *workspace, size_t workspace_bytes,
                                     bitsnap_stream_t stream);
int bitsnap_decode_sparse_batched_ex(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                     int elem_bytes, uint32_t flags, void *workspace, size_t workspace_bytes,
                                     bitsnap_stream_t stream);

/* group must be one of 256, 512, 1024, 2048, 4096; total_groups = sum of ceil(n/group). */
int bitsnap_quantize_cluster_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                     int64_t group, int m, uint32_t *status, bitsnap_stream_t stream);
int bitsnap_dequantize_cluster_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                       int64_t group, int m, bitsnap_stream_t stream);

/* The batched cluster calls with the options of bitsnap_quantize_cluster_ex /
 * bitsnap_dequantize_cluster_ex (flags and qmap apply to every item), and with group = 0: one
 * group per tensor for the whole list (the paper's formulation, a checkpoint pass at a time).
 *   group   one of 256 .. 4096, or 0.
 *           With 0, groups are not the unit of the list-wide numbering (every tensor has one);
 *           chunks of bitsnap_cluster_chunk_elems() elements are: an item's first_group is the sum
 *           of ceil(n / chunk_elems) over all earlier items and total_groups that sum over all
 *           items; params holds [m][2] and fit_out [m+1] floats per tensor.
 *   workspace  [bitsnap_cluster_batch_workspace_bytes(total_groups, count, group, flags)], 16-byte
 *           aligned; 0 bytes (may be NULL) unless group = 0.  Dequantisation uses it only with
 *           BITSNAP_CLUSTER_MAJOR, which needs every n < 2^32 when group = 0. */
size_t bitsnap_cluster_chunk_elems(void);
size_t bitsnap_cluster_batch_workspace_bytes(int64_t total_groups, int64_t count, int64_t group, uint32_t flags);
int bitsnap_quantize_cluster_batched_ex(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                        int64_t group, int m, uint32_t flags, const float *qmap, uint32_t *status,
                                        void *workspace, size_t workspace_bytes, bitsnap_stream_t stream);
int bitsnap_dequantize_cluster_batched_ex(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                          int64_t group, int m, uint32_t flags, const float *qmap, void *workspace,
                                          size_t workspace_bytes, bitsnap_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* BITSNAP_H */
