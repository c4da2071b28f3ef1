/*
 * CPU oracle for the BitSnap per-tensor codecs.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the HIP library is checked against.  It shares
 * no code, header, table or helper with the HIP tree, and nothing in the product path may call
 * it: only tests/, the smoke check and the benchmark's cpu_baseline leg load it.
 *
 * Everything is a scalar loop in the order the paper states the steps.  Floating point follows
 * IEEE-754 with no contraction (build with -ffp-contract=off, no -ffast-math).
 *
 * Parity pins (tests/test_oracle_*.py): every function below is pinned; none is "parity
 * unpinned".  The MSE/MRE tables of the paper's evaluation depend on trained optimizer states
 * and are not reproduced anywhere.
 *
 * Sparse path  - paper section "Bitmask Based Sparsification for Model States"
 *                (naive and improved bitmask, space formulas) and Algorithm 1.
 * Cluster path - paper section "Cluster Based Quantization for Optimizer States"
 *                (Eq. qmap-distance, the S/b definition, Eq. decluster, the size analysis)
 *                and Algorithm 2.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------
 * Sparse path
 * ---------------------------------------------------------------------------------------- */

/* Algorithm 1 steps 1-5 for one flattened tensor of 16-bit elements.
 *   step 1-2: an element is "changed" iff its 16-bit pattern differs from the base's
 *             (a bitwise test is the only one that keeps the scheme lossless for -0 and NaN);
 *   step 3-4: bit i of the mask goes to byte i/8, bit position i%8 (least significant first),
 *             padding bits of the last byte are 0;
 *   step 5  : the changed values (the new values themselves) are stored in index order.
 * mask has ceil(n/8) bytes, payload room for n elements.  Returns n_c. */
int64_t oracle_encode_sparse(const uint16_t *cur, const uint16_t *base, int64_t n,
                             uint8_t *mask, uint16_t *payload)
{
    int64_t nc = 0;
    int64_t nbytes = (n + 7) / 8;
    for (int64_t j = 0; j < nbytes; ++j)
        mask[j] = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (cur[i] != base[i]) {
            mask[i >> 3] = (uint8_t)(mask[i >> 3] | (1u << (i & 7)));
            payload[nc] = cur[i];
            nc += 1;
        }
    }
    return nc;
}

/* The naive variant of the same section: one uint8 (0 or 1) per element.  Kept only so the
 * space formula n + 2 n_c of Eq. bitmask-required-space can be checked on real buffers. */
int64_t oracle_encode_sparse_naive(const uint16_t *cur, const uint16_t *base, int64_t n,
                                   uint8_t *flags, uint16_t *payload)
{
    int64_t nc = 0;
    for (int64_t i = 0; i < n; ++i) {
        flags[i] = (uint8_t)(cur[i] != base[i]);
        if (flags[i]) {
            payload[nc] = cur[i];
            nc += 1;
        }
    }
    return nc;
}

/* off[t] = number of set mask bits among elements [0, t*tile), t = 0 .. ceil(n/tile)
 * (the last entry is n_c).  This is the compaction offset of each tile. */
void oracle_tile_offsets(const uint8_t *mask, int64_t n, int64_t tile, uint64_t *off)
{
    int64_t ntiles = (n + tile - 1) / tile;
    uint64_t run = 0;
    for (int64_t t = 0; t < ntiles; ++t) {
        off[t] = run;
        int64_t hi = (t + 1) * tile;
        if (hi > n)
            hi = n;
        for (int64_t i = t * tile; i < hi; ++i)
            run += (mask[i >> 3] >> (i & 7)) & 1u;
    }
    off[ntiles] = run;
}

/* Inverse of oracle_encode_sparse: out[i] = changed ? next payload value : base[i]. */
void oracle_decode_sparse(const uint16_t *base, const uint8_t *mask, const uint16_t *payload,
                          int64_t n, uint16_t *out)
{
    int64_t r = 0;
    for (int64_t i = 0; i < n; ++i) {
        if ((mask[i >> 3] >> (i & 7)) & 1u) {
            out[i] = payload[r];
            r += 1;
        } else {
            out[i] = base[i];
        }
    }
}

/* The same codec with the two options of the extended entry points.
 *   delta != 0   the payload holds the non-zero elements of the delta states themselves, with
 *                the delta of two 16-bit patterns taken as their bitwise difference cur XOR base
 *                (what the section stores beside the mask, read literally;
 *                an arithmetic fp16/bf16 difference would not reconstruct bit for bit);
 *                delta == 0 stores the new values, as oracle_encode_sparse does.
 *   new_base     if not NULL, receives a copy of cur: the tensor becomes the base of the next
 *                delta checkpoints.  It may be the very array `base` (each element is compared
 *                before it is overwritten).
 * Mask, count and order of the payload are those of oracle_encode_sparse. */
int64_t oracle_encode_sparse_ex(const uint16_t *cur, const uint16_t *base, int64_t n, int delta,
                                uint8_t *mask, uint16_t *payload, uint16_t *new_base)
{
    int64_t nc = 0;
    int64_t nbytes = (n + 7) / 8;
    for (int64_t j = 0; j < nbytes; ++j)
        mask[j] = 0;
    for (int64_t i = 0; i < n; ++i) {
        const uint16_t c = cur[i], b = base[i];
        if (c != b) {
            mask[i >> 3] = (uint8_t)(mask[i >> 3] | (1u << (i & 7)));
            payload[nc] = delta ? (uint16_t)(c ^ b) : c;
            nc += 1;
        }
        if (new_base)
            new_base[i] = c;
    }
    return nc;
}

/* Inverse: out[i] = changed ? (delta ? base[i] XOR next payload element : next payload element)
 * : base[i]. */
void oracle_decode_sparse_ex(const uint16_t *base, const uint8_t *mask, const uint16_t *payload,
                             int64_t n, int delta, uint16_t *out)
{
    int64_t r = 0;
    for (int64_t i = 0; i < n; ++i) {
        if ((mask[i >> 3] >> (i & 7)) & 1u) {
            out[i] = delta ? (uint16_t)(base[i] ^ payload[r]) : payload[r];
            r += 1;
        } else {
            out[i] = base[i];
        }
    }
}

/* The same codec for tensors of 32-bit elements (fp32 model states): the element is "changed" iff
 * its 32-bit pattern differs; the mask has one bit per element as before; the payload holds 32-bit
 * values (the new ones, or cur XOR base with delta != 0).  Stored size: n/8 + 4 n_c bytes. */
int64_t oracle_encode_sparse32_ex(const uint32_t *cur, const uint32_t *base, int64_t n, int delta,
                                  uint8_t *mask, uint32_t *payload, uint32_t *new_base)
{
    int64_t nc = 0;
    int64_t nbytes = (n + 7) / 8;
    for (int64_t j = 0; j < nbytes; ++j)
        mask[j] = 0;
    for (int64_t i = 0; i < n; ++i) {
        const uint32_t c = cur[i], b = base[i];
        if (c != b) {
            mask[i >> 3] = (uint8_t)(mask[i >> 3] | (1u << (i & 7)));
            payload[nc] = delta ? (c ^ b) : c;
            nc += 1;
        }
        if (new_base)
            new_base[i] = c;
    }
    return nc;
}

void oracle_decode_sparse32_ex(const uint32_t *base, const uint8_t *mask, const uint32_t *payload,
                               int64_t n, int delta, uint32_t *out)
{
    int64_t r = 0;
    for (int64_t i = 0; i < n; ++i) {
        if ((mask[i >> 3] >> (i & 7)) & 1u) {
            out[i] = delta ? (base[i] ^ payload[r]) : payload[r];
            r += 1;
        } else {
            out[i] = base[i];
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Cluster path
 * ---------------------------------------------------------------------------------------- */

/* z = Phi^{-1}(k/m): the standard-normal quantile that cuts the line into m parts of equal
 * probability (Algorithm 2 step 2: clusters laid out like a normal distribution, so that each
 * holds about the same number of elements).  Found by bisection on the normal CDF written with
 * erfc, in long double; symmetric by construction. */
double oracle_norm_quantile(int k, int m)
{
    if (m < 1 || k <= 0 || k >= m)
        return 0.0;
    if (2 * k == m)
        return 0.0;
    if (2 * k > m)
        return -oracle_norm_quantile(m - k, m);
    long double p = (long double)k / (long double)m; /* p < 1/2, so z < 0 */
    long double lo = -40.0L, hi = 0.0L;
    for (int it = 0; it < 200; ++it) {
        long double mid = 0.5L * (lo + hi);
        long double cdf = 0.5L * erfcl(-mid / sqrtl(2.0L));
        if (cdf < p)
            lo = mid;
        else
            hi = mid;
    }
    return (double)(0.5L * (lo + hi));
}

/* Algorithm 2 step 1 for one group: mean and (population) standard deviation, accumulated in
 * fp64 in index order, each rounded once to fp32. */
void oracle_cluster_fit(const float *x, int64_t len, float *mu, float *sigma)
{
    if (len <= 0) {
        *mu = 0.0f;
        *sigma = 0.0f;
        return;
    }
    double s = 0.0;
    for (int64_t i = 0; i < len; ++i)
        s += (double)x[i];
    double mean = s / (double)len;
    double q = 0.0;
    for (int64_t i = 0; i < len; ++i) {
        double d = (double)x[i] - mean;
        q += d * d;
    }
    *mu = (float)mean;
    *sigma = (float)sqrt(q / (double)len);
}

/* Algorithm 2 step 2: the m-1 interior cluster edges e_k = mu + sigma * z_k, k = 1..m-1,
 * evaluated in fp64 (product rounded, then sum rounded) and rounded to fp32.
 * edges[k-1] = e_k. */
void oracle_cluster_edges(float mu, float sigma, int m, float *edges)
{
    for (int k = 1; k < m; ++k) {
        double prod = (double)sigma * oracle_norm_quantile(k, m);
        double e = (double)mu + prod;
        edges[k - 1] = (float)e;
    }
}

/* Algorithm 2 step 3: label = number of edges that are <= x (fp32 compares).
 * Cluster 0 is (-inf, e_1), cluster m-1 is [e_{m-1}, +inf). */
static int label_of(float x, const float *edges, int m)
{
    int l = 0;
    for (int k = 1; k < m; ++k)
        if (edges[k - 1] <= x)
            l += 1;
    return l;
}

/* Eq. qmap-distance with the linear map Q_j = j/255, in closed form: the code is the integer
 * nearest to (x-b)/S*255.  inv = fl32(255/S); y = fl32(fl32(x-b)*inv); ties to even.
 * S == 0, or S so small that 255/S is not finite, codes everything as 0. */
static uint8_t code_of(float x, float b, float S)
{
    if (!(S > 0.0f))
        return 0;
    float inv = 255.0f / S;
    if (!isfinite(inv))
        return 0;
    float d = x - b;
    float y = d * inv;
    float r = rintf(y); /* default rounding mode: nearest, ties to even */
    if (r < 0.0f)
        r = 0.0f;
    if (r > 255.0f)
        r = 255.0f;
    return (uint8_t)r;
}

/* Algorithm 2 for a flattened fp32 tensor cut into groups of G consecutive elements (G <= 0 or
 * G >= n: the whole tensor is one group, which is the paper's own formulation).
 *
 *   fit_in  (nullable) [groups][2]     : use these (mu, sigma) instead of computing them
 *   codes              [n]             : uint8 code per element, element order
 *   labels             [ceil(n/2)]     : uint4 label per element, even index in the low nibble
 *   params             [groups][m][2]  : (S, b) per cluster; empty cluster -> (0, 0)
 *   fit_out (nullable) [groups][2+m-1] : mu, sigma, e_1 .. e_{m-1}
 */
void oracle_quantize_cluster(const float *x, int64_t n, int64_t G, int m, const float *fit_in,
                             uint8_t *codes, uint8_t *labels, float *params, float *fit_out)
{
    if (n <= 0)
        return;
    if (G <= 0 || G > n)
        G = n;
    int64_t groups = (n + G - 1) / G;
    memset(labels, 0, (size_t)((n + 1) / 2));
    for (int64_t g = 0; g < groups; ++g) {
        int64_t lo = g * G;
        int64_t len = (lo + G <= n) ? G : (n - lo);
        const float *xg = x + lo;
        float mu, sigma;
        if (fit_in) {
            mu = fit_in[2 * g];
            sigma = fit_in[2 * g + 1];
        } else {
            oracle_cluster_fit(xg, len, &mu, &sigma);
        }
        float edges[16];
        oracle_cluster_edges(mu, sigma, m, edges);
        if (fit_out) {
            float *f = fit_out + g * (2 + (m - 1));
            f[0] = mu;
            f[1] = sigma;
            for (int k = 1; k < m; ++k)
                f[1 + k] = edges[k - 1];
        }
        /* step 3: labels; step 4: per-cluster min and max */
        float mn[16], mx[16];
        int seen[16];
        for (int c = 0; c < m; ++c) {
            seen[c] = 0;
            mn[c] = 0.0f;
            mx[c] = 0.0f;
        }
        for (int64_t i = 0; i < len; ++i) {
            int l = label_of(xg[i], edges, m);
            int64_t idx = lo + i;
            labels[idx >> 1] = (uint8_t)(labels[idx >> 1] | (l << ((idx & 1) * 4)));
            if (!seen[l]) {
                seen[l] = 1;
                mn[l] = xg[i];
                mx[l] = xg[i];
            } else {
                if (xg[i] < mn[l])
                    mn[l] = xg[i];
                if (xg[i] > mx[l])
                    mx[l] = xg[i];
            }
        }
        float *pg = params + g * (int64_t)m * 2;
        for (int c = 0; c < m; ++c) {
            pg[2 * c + 0] = seen[c] ? (mx[c] - mn[c]) : 0.0f; /* S = max - min */
            pg[2 * c + 1] = seen[c] ? mn[c] : 0.0f;           /* b = min       */
        }
        /* steps 5-6: normalise inside the cluster, nearest uint8 */
        for (int64_t i = 0; i < len; ++i) {
            int64_t idx = lo + i;
            int l = (labels[idx >> 1] >> ((idx & 1) * 4)) & 15;
            codes[idx] = code_of(xg[i], pg[2 * l + 1], pg[2 * l + 0]);
        }
    }
}

/* Dequantization: T^D = Q(T^Q) * S + b with Q(j) = j/255, evaluated as
 * fl32(fl32(q * fl32(S/255)) + b); Eq. decluster (values go back to the positions their labels
 * came from) is the identity here because codes are kept in element order. */
void oracle_dequantize_cluster(const uint8_t *codes, const uint8_t *labels, const float *params,
                               int64_t n, int64_t G, int m, float *out)
{
    if (n <= 0)
        return;
    if (G <= 0 || G > n)
        G = n;
    for (int64_t i = 0; i < n; ++i) {
        int64_t g = i / G;
        int l = (labels[i >> 1] >> ((i & 1) * 4)) & 15;
        const float *pg = params + g * (int64_t)m * 2;
        float S = pg[2 * l + 0];
        float b = pg[2 * l + 1];
        float step = S / 255.0f;
        float t = (float)codes[i] * step;
        out[i] = t + b;
    }
}

/* ------------------------------------------------------------------------------------------
 * Format variants of the cluster path: a general (non-linear) map Q^map, and the cluster-major
 * arrangement of the codes that Eq. decluster describes.
 * ---------------------------------------------------------------------------------------- */

/* Eq. qmap-distance with a table of 256 reals: t = (x-b)/S, code = the j that minimises
 * |Q_j - t|, the lowest such j when several do.  The decision is taken in fp32, the precision
 * of the data: t = fl32(fl32(x-b) * fl32(1/S)), distance = fl32(|Q_j - t|).  S == 0, or S so
 * small that 1/S is not finite, codes everything as 0 (as with the linear map). */
static uint8_t code_of_qmap(float x, float b, float S, const float *qmap)
{
    if (!(S > 0.0f))
        return 0;
    float inv = 1.0f / S;
    if (!isfinite(inv))
        return 0;
    float d = x - b;
    float t = d * inv;
    int best = 0;
    float bd = INFINITY;
    for (int j = 0; j < 256; ++j) {
        float dist = fabsf(qmap[j] - t);
        if (dist < bd) {
            bd = dist;
            best = j;
        }
    }
    return (uint8_t)best;
}

/* Algorithm 2 with the two format options.
 *   qmap          (nullable) [256]: Q^map; NULL = the linear map, exactly oracle_quantize_cluster
 *   cluster_major 0: codes in element order
 *                 1: inside every group the codes of cluster 0 come first, then those of cluster
 *                    1, ...; inside a cluster in the order of the elements (the T_{C_i k} of
 *                    Eq. decluster: k counts the members of cluster i in element order)
 * labels, params and fit_out are those of oracle_quantize_cluster in either case. */
void oracle_quantize_cluster_ex(const float *x, int64_t n, int64_t G, int m, const float *fit_in,
                                const float *qmap, int cluster_major, uint8_t *codes,
                                uint8_t *labels, float *params, float *fit_out)
{
    if (n <= 0)
        return;
    if (G <= 0 || G > n)
        G = n;
    /* steps 1-4 and the linear codes */
    oracle_quantize_cluster(x, n, G, m, fit_in, codes, labels, params, fit_out);
    int64_t groups = (n + G - 1) / G;
    if (qmap) {
        for (int64_t i = 0; i < n; ++i) {
            int64_t g = i / G;
            int l = (labels[i >> 1] >> ((i & 1) * 4)) & 15;
            const float *pg = params + g * (int64_t)m * 2;
            codes[i] = code_of_qmap(x[i], pg[2 * l + 1], pg[2 * l + 0], qmap);
        }
    }
    if (cluster_major) {
        uint8_t *tmp = (uint8_t *)malloc((size_t)G);
        for (int64_t g = 0; g < groups; ++g) {
            int64_t lo = g * G;
            int64_t len = (lo + G <= n) ? G : (n - lo);
            int64_t k = 0;
            for (int c = 0; c < m; ++c)
                for (int64_t i = 0; i < len; ++i) {
                    int64_t idx = lo + i;
                    int l = (labels[idx >> 1] >> ((idx & 1) * 4)) & 15;
                    if (l == c)
                        tmp[k++] = codes[idx];
                }
            memcpy(codes + lo, tmp, (size_t)len);
        }
        free(tmp);
    }
}

/* The inverse: T^D = Q^map(T^Q) * S + b, evaluated as fl32(fl32(Q_q * S) + b) with a table
 * (with qmap == NULL: the linear map as in oracle_dequantize_cluster), and Eq. decluster:
 * V_j = T_{C_i k} with i = L_j and k = the number of earlier elements of the group that carry
 * label i. */
void oracle_dequantize_cluster_ex(const uint8_t *codes, const uint8_t *labels, const float *params,
                                  int64_t n, int64_t G, int m, const float *qmap, int cluster_major,
                                  float *out)
{
    if (n <= 0)
        return;
    if (G <= 0 || G > n)
        G = n;
    int64_t groups = (n + G - 1) / G;
    for (int64_t g = 0; g < groups; ++g) {
        int64_t lo = g * G;
        int64_t len = (lo + G <= n) ? G : (n - lo);
        const float *pg = params + g * (int64_t)m * 2;
        int64_t start[16], seen[16];
        for (int c = 0; c < 16; ++c)
            start[c] = seen[c] = 0;
        if (cluster_major) {
            int64_t count[16] = {0};
            for (int64_t i = 0; i < len; ++i) {
                int64_t idx = lo + i;
                count[(labels[idx >> 1] >> ((idx & 1) * 4)) & 15] += 1;
            }
            for (int c = 1; c < 16; ++c)
                start[c] = start[c - 1] + count[c - 1];
        }
        for (int64_t i = 0; i < len; ++i) {
            int64_t idx = lo + i;
            int l = (labels[idx >> 1] >> ((idx & 1) * 4)) & 15;
            uint8_t q = cluster_major ? codes[lo + start[l] + seen[l]] : codes[idx];
            seen[l] += 1;
            float S = pg[2 * l + 0];
            float b = pg[2 * l + 1];
            float t;
            if (qmap) {
                t = qmap[q] * S;
            } else {
                float step = S / 255.0f;
                t = (float)q * step;
            }
            out[idx] = t + b;
        }
    }
}

/* Eq. qmap-distance with a table, for one element, in long double (64-bit significand: far
 * finer than the fp32 decision above): the minimiser of |Q_j - (x-b)/S|, lowest j on ties, and
 * the gap to the runner-up, so that a test can set near-ties aside. */
int oracle_code_qmap_bruteforce(float x, float b, float S, const float *qmap, double *gap)
{
    if (!(S > 0.0f)) {
        if (gap)
            *gap = 1.0;
        return 0;
    }
    long double t = ((long double)x - (long double)b) / (long double)S;
    int best = 0;
    long double bd = 1e300L, second = 1e300L;
    for (int j = 0; j < 256; ++j) {
        long double d = fabsl((long double)qmap[j] - t);
        if (d < bd) {
            second = bd;
            bd = d;
            best = j;
        } else if (d < second) {
            second = d;
        }
    }
    if (gap)
        *gap = (double)(second - bd);
    return best;
}

/* Brute-force form of Eq. qmap-distance for one element: the j in [0,255] minimising
 * |j/255 - (x-b)/S| in fp64, lowest j on exact ties.  Also reports the gap between the best
 * and the second-best distance so a test can tell a near-tie from a real disagreement. */
int oracle_code_bruteforce(float x, float b, float S, double *gap)
{
    if (!(S > 0.0f)) {
        if (gap)
            *gap = 1.0;
        return 0;
    }
    double t = ((double)x - (double)b) / (double)S;
    int best = 0;
    double bd = 1e300, second = 1e300;
    for (int j = 0; j < 256; ++j) {
        double d = fabs((double)j / 255.0 - t);
        if (d < bd) {
            second = bd;
            bd = d;
            best = j;
        } else if (d < second) {
            second = d;
        }
    }
    if (gap)
        *gap = second - bd;
    return best;
}
