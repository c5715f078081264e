/*
 * CPU oracle for one rank's share of a multi-colour Allreduce step followed by SGD.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain, slow, obviously-correct definition that
 * the GPU library is checked against.  Only the tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it; the product never does.  It shares no code, header,
 * table or helper with the HIP implementation.
 *
 * What it computes, and where the paper defines it:
 *   - The gradient that every worker ends up with is the plain elementwise sum of all
 *     contributions: first over the GPUs of a node, then over the nodes (Section 3,
 *     Algorithm 1, the two summation lines).
 *   - The payload is one flat buffer split into k chunks ("colours"); each chunk is summed
 *     independently of the others along its own tree, with no synchronisation between
 *     colours (Section 4.2, first two paragraphs).
 *   - A rank that is root or non-leaf for a colour adds the buffers that arrived from its
 *     children to the local contributions of its GPUs (Section 4.2, last paragraph).
 *   - After the sum every GPU performs an SGD step (Section 3, Algorithm 1, last line).
 *
 * The method is an exact re-scheduling of a sum, not an approximation, so the oracle is
 * that definition written out.  In binary32 the order of additions is part of the result;
 * the readings taken where the paper is silent are:
 *   - flat payload = dense concatenation of the per-layer tensors in the given order;
 *   - chunk size = ceil(N/k) rounded up to 256 elements, chunks contiguous, last one short,
 *     trailing chunks may be empty;
 *   - inside colour c the contributions are added strictly left to right in the sequence
 *     order[c][0], order[c][1], ... starting FROM the first term (not from 0.0f);
 *   - the update is heavy-ball momentum with L2 decay folded into the gradient,
 *       d = g + wd*w ;  v' = mu*v + d ;  w' = w - lr*v'
 *     with every operation rounded separately to binary32 (no fused multiply-add).
 *
 * Build:  gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -shared -fPIC
 * (x86-64 SSE arithmetic: binary32 operations are rounded once, denormals are kept).
 */
#include <stdint.h>
#include <stddef.h>

#define MCO_COLOUR_ALIGN 256

/* Flat offsets of the tensors and the k+1 colour bounds.  off has n+1 entries, bounds k+1.
 * Returns 0, or -1 on an invalid argument. */
int mco_layout(const int64_t *numel, int32_t n, int32_t k, int64_t *off, int64_t *bounds)
{
    if (!numel || !off || !bounds || n < 1 || k < 1) return -1;
    off[0] = 0;
    for (int32_t t = 0; t < n; ++t) {
        if (numel[t] < 0) return -1;
        off[t + 1] = off[t] + numel[t];
    }
    const int64_t N = off[n];
    int64_t chunk = (N + k - 1) / k;                                   /* ceil(N / k)      */
    chunk = (chunk + MCO_COLOUR_ALIGN - 1) / MCO_COLOUR_ALIGN * MCO_COLOUR_ALIGN;
    for (int32_t c = 0; c <= k; ++c)          /* b_c = min(N, c * chunk), written so that  */
        bounds[c] = (chunk == 0 || c > N / chunk) ? N : c * chunk;   /* it cannot overflow */
    return 0;
}

/* flat[off[t] + j] = tensors[t][j]  -- a bit copy (moved as 32-bit words, never as floats). */
void mco_pack(const int64_t *off, int32_t n, const uint32_t *const *tensors, uint32_t *flat)
{
    for (int32_t t = 0; t < n; ++t)
        for (int64_t j = 0; j < off[t + 1] - off[t]; ++j)
            flat[off[t] + j] = tensors[t][j];
}

/* tensors[t][j] = flat[off[t] + j]  -- the inverse bit copy. */
void mco_unpack(const int64_t *off, int32_t n, const uint32_t *flat, uint32_t *const *tensors)
{
    for (int32_t t = 0; t < n; ++t)
        for (int64_t j = 0; j < off[t + 1] - off[t]; ++j)
            tensors[t][j] = flat[off[t] + j];
}

/* One colour: elements [lo, hi).  seq[0..P) is the order in which this colour's
 * contributions are added.  g may be NULL (the reduced gradient is then not stored). */
void mco_reduce_update_colour(int64_t lo, int64_t hi, const float *const *x, int32_t P,
                              const int32_t *seq, float *g, float *w, float *v,
                              float lr, float mu, float wd)
{
    for (int64_t i = lo; i < hi; ++i) {
        float acc = x[seq[0]][i];
        for (int32_t q = 1; q < P; ++q)
            acc = acc + x[seq[q]][i];
        if (g) g[i] = acc;
        const float decay = wd * w[i];
        const float d = acc + decay;
        const float mv = mu * v[i];
        const float vn = mv + d;
        const float step = lr * vn;
        w[i] = w[i] - step;
        v[i] = vn;
    }
}

/* The same with the Nesterov look-ahead step (the paper names no variant of "SGD"; the Torch
 * ResNet recipe it builds on uses this one): d and v' as above, then
 *   w' = w - lr * (d + mu * v')
 * again with every operation rounded separately. */
void mco_reduce_update_colour_nesterov(int64_t lo, int64_t hi, const float *const *x, int32_t P,
                                       const int32_t *seq, float *g, float *w, float *v,
                                       float lr, float mu, float wd)
{
    for (int64_t i = lo; i < hi; ++i) {
        float acc = x[seq[0]][i];
        for (int32_t q = 1; q < P; ++q)
            acc = acc + x[seq[q]][i];
        if (g) g[i] = acc;
        const float decay = wd * w[i];
        const float d = acc + decay;
        const float mv = mu * v[i];
        const float vn = mv + d;
        const float look = mu * vn;
        const float dir = d + look;
        const float step = lr * dir;
        w[i] = w[i] - step;
        v[i] = vn;
    }
}

/* One colour, sum only: what a leaf or inner node of the colour's tree produces (its partial
 * sum, handed to the parent).  The SGD step needs the complete sum, which only the root has
 * (Section 4.2: roots and non-leaf nodes sum, leaves only send; the result is broadcast from
 * the roots afterwards). */
void mco_reduce_colour(int64_t lo, int64_t hi, const float *const *x, int32_t n_terms,
                       const int32_t *seq, float *g)
{
    for (int64_t i = lo; i < hi; ++i) {
        float acc = x[seq[0]][i];
        for (int32_t q = 1; q < n_terms; ++q)
            acc = acc + x[seq[q]][i];
        g[i] = acc;
    }
}

/* Per-colour roles: colour c adds the first n_terms[c] entries of its sequence (0 = the
 * colour is skipped, nothing of its range is touched); where do_update[c] is non-zero the
 * SGD step follows (this rank holds the colour's complete sum), elsewhere only g is written.
 * order as in mco_reduce_update (NULL = identity).  Returns 0 or -1. */
int mco_reduce_update_roles(const int64_t *bounds, int32_t k, const float *const *x, int32_t P,
                            const int32_t *order, const int32_t *n_terms,
                            const uint8_t *do_update, float *g, float *w, float *v,
                            float lr, float mu, float wd)
{
    if (!bounds || !x || !n_terms || !do_update || k < 1 || P < 1 || P > 64) return -1;
    int32_t ident[64];
    for (int32_t q = 0; q < P; ++q) ident[q] = q;
    for (int32_t c = 0; c < k; ++c) {
        if (n_terms[c] < 0 || n_terms[c] > P) return -1;
        if (n_terms[c] == 0) continue;
        const int32_t *seq = order ? order + (size_t)c * (size_t)P : ident;
        if (do_update[c]) {
            if (!w || !v) return -1;
            mco_reduce_update_colour(bounds[c], bounds[c + 1], x, n_terms[c], seq, g, w, v, lr, mu, wd);
        } else {
            if (!g) return -1;
            mco_reduce_colour(bounds[c], bounds[c + 1], x, n_terms[c], seq, g);
        }
    }
    return 0;
}

/* All colours, in index order.  order is k*P row-major (row c = sequence of colour c) or
 * NULL for the identity sequence 0,1,..,P-1 in every colour.  Returns 0 or -1. */
int mco_reduce_update(const int64_t *bounds, int32_t k, const float *const *x, int32_t P,
                      const int32_t *order, float *g, float *w, float *v,
                      float lr, float mu, float wd)
{
    if (!bounds || !x || !w || !v || k < 1 || P < 1 || P > 64) return -1;
    int32_t ident[64];
    for (int32_t q = 0; q < P; ++q) ident[q] = q;
    for (int32_t c = 0; c < k; ++c) {
        const int32_t *seq = order ? order + (size_t)c * (size_t)P : ident;
        mco_reduce_update_colour(bounds[c], bounds[c + 1], x, P, seq, g, w, v, lr, mu, wd);
    }
    return 0;
}
