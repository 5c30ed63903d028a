/*
 * CPU oracle for the Linear-Layouts hot path (arXiv 2505.23819).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, written from the paper's definitions.
 * It shares no code with the HIP library: nothing here is included, linked or
 * imported by the product path, and nothing here includes product headers.
 *
 * Conventions (paper Sec. 4.1, the worked Layout A example and its footnote):
 *   - A layout with d_in input bits is stored as its matrix COLUMNS:
 *     bases[k] is the image of input bit k, written as a flattened output
 *     index.  Input bits are ordered register bits first, then lane (thread)
 *     bits, then wave (warp) bits; least-significant bit first.
 *   - The flattened output index puts the LAST logical dimension in the lowest
 *     bits (the fastest moving one), e.g. for a rows x cols tile
 *     flat = col | row << log2(cols).
 *   - L(h) is the XOR of the columns selected by the set bits of h
 *     (matrix-vector product over F2, Sec. 2.4).
 *
 * Functions and the passage each follows:
 *   oracle_apply            Sec. 4.1  w = A v over F2
 *   oracle_compose          Def. Composition (label-wise matrix product), with
 *                           the product written out as c_ij = XOR_k a_ik b_kj
 *   oracle_inverse_table    Def. Right Inverse, restricted to bijective
 *                           layouts: the inverse is found by tabulating L(h)
 *                           for every h (no elimination)
 *   oracle_right_inverse_table  Def. Right Inverse / Sec. 5.4 rule 2 for surjective
 *                           layouts that are not injective (broadcasting): the
 *                           solution with all free variables zero, built by
 *                           growing the span column by column (no elimination)
 *   oracle_convert_general  Sec. 5.4 with broadcasting: every destination unit
 *                           reads the value of its logical element from the
 *                           canonical source unit
 *   oracle_convert          Sec. 5.4: the conversion is B^-1 o A; element by
 *                           element on images (see below)
 *   oracle_convert_table    same result; the composed map is tabulated once
 *                           and tiles are processed by all host threads
 *   oracle_gather           Sec. 5.5: out[.., i, ..] = in[.., idx[.., i, ..], ..]
 *                           along `axis`, all three tensors under layout L
 *   oracle_convert_affine,
 *   oracle_gather_affine    Conclusions: affine layouts y = A x xor b (flips, slices)
 *   oracle_wavefronts       Sec. 5.4 "Optimal Swizzling" + the wavefront lemma
 *                           of the appendix: exhaustive enumeration of the
 *                           shared-memory (LDS) wavefronts an access needs
 *
 * Images.  A tensor tile held "under layout L" is stored as an array indexed
 * by the hardware index h = reg | lane << nreg | wave << (nreg+nlane): element
 * h of tile t sits at buf[t * 2^d + h] and is the logical element L(h).
 *
 * Pins: tests/test_oracle_pins.py (values the paper prints for Layout A,
 * closed forms, textbook transpose / take_along_axis, brute force).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG 1
#define ORACLE_ERR_NOT_BIJECTIVE 2
#define ORACLE_ERR_AXIS 3
#define ORACLE_ERR_ALLOC 4

/* w = L v : XOR of the columns picked by the set bits of v (Sec. 4.1). */
uint64_t oracle_apply(const uint64_t *bases, int d_in, uint64_t h)
{
    uint64_t x = 0;
    for (int k = 0; k < d_in; ++k)
        if ((h >> k) & 1u)
            x ^= bases[k];
    return x;
}

/*
 * Composition outer o inner (Def. Composition): the matrix product over F2,
 * entry by entry: c_ij = XOR_k a_ik * b_kj  (Sec. 2.4).
 * inner: d_in columns, each a d_mid-bit vector; outer: d_mid columns.
 */
int oracle_compose(const uint64_t *outer, int d_mid, int d_out,
                   const uint64_t *inner, int d_in, uint64_t *result)
{
    if (!outer || !inner || !result || d_mid < 0 || d_mid > 63 || d_out > 63)
        return ORACLE_ERR_ARG;
    for (int j = 0; j < d_in; ++j) {
        uint64_t col = 0;
        for (int i = 0; i < d_out; ++i) {
            unsigned c = 0;
            for (int k = 0; k < d_mid; ++k) {
                unsigned a_ik = (unsigned)((outer[k] >> i) & 1u); /* row i, col k of outer */
                unsigned b_kj = (unsigned)((inner[j] >> k) & 1u); /* row k, col j of inner */
                c ^= (a_ik & b_kj);
            }
            col |= (uint64_t)c << i;
        }
        result[j] = col;
    }
    return ORACLE_OK;
}

/*
 * Inverse of a bijective layout on d bits by tabulation: table[L(h)] = h.
 * Fails unless every output index is hit exactly once (this is the
 * bijectivity check of the oracle).
 */
int oracle_inverse_table(const uint64_t *bases, int d, uint32_t *table)
{
    if (!bases || !table || d < 0 || d > 30)
        return ORACLE_ERR_ARG;
    const uint64_t n = 1ull << d;
    for (uint64_t x = 0; x < n; ++x)
        table[x] = 0xFFFFFFFFu;
    for (uint64_t h = 0; h < n; ++h) {
        uint64_t x = oracle_apply(bases, d, h);
        if (x >= n || table[x] != 0xFFFFFFFFu)
            return ORACLE_ERR_NOT_BIJECTIVE;
        table[x] = (uint32_t)h;
    }
    return ORACLE_OK;
}

/*
 * Right inverse of a surjective layout with d_in >= d_out input bits
 * (Def. Right Inverse; Sec. 5.4 rule 2: "set the slack variables to zero").
 * Columns are visited in input order (register bits first).  A column that is
 * not yet in the span of the earlier ones is a pivot: it doubles the span, and
 * every new element x ^ col gets the representative table[x] | 1 << k.  A
 * column already in the span is a free variable and is never used.  Hence
 * table[x] is the unique h with L(h) = x whose free variables are all zero.
 */
int oracle_right_inverse_table(const uint64_t *bases, int d_in, int d_out, uint32_t *table)
{
    if (!bases || !table || d_in < 0 || d_in > 30 || d_out < 0 || d_out > 30)
        return ORACLE_ERR_ARG;
    const uint64_t n = 1ull << d_out;
    for (uint64_t x = 0; x < n; ++x)
        table[x] = 0xFFFFFFFFu;
    table[0] = 0;
    uint64_t *members = (uint64_t *)malloc(n * sizeof(uint64_t));   /* elements of the span so far */
    if (!members) return ORACLE_ERR_ALLOC;
    uint64_t count = 1;
    members[0] = 0;
    for (int k = 0; k < d_in; ++k) {
        const uint64_t col = bases[k];
        if (col >= n) { free(members); return ORACLE_ERR_ARG; }
        if (table[col] != 0xFFFFFFFFu)
            continue;                           /* dependent column: a free variable, left at zero */
        for (uint64_t i = 0; i < count; ++i) {
            const uint64_t x = members[i] ^ col;
            table[x] = table[members[i]] | (1u << k);
            members[count + i] = x;
        }
        count *= 2;
    }
    free(members);
    return count == n ? ORACLE_OK : ORACLE_ERR_NOT_BIJECTIVE;      /* not surjective */
}

/*
 * Conversion with broadcasting (Sec. 5.4: B^-1 o A with rule 2; Sec. 5.1
 * "Broadcasting").  A has dA input bits, B has dB, both map onto the same d_out
 * logical bits and both are surjective.  For every tile t and every destination
 * hardware index hB:
 *     x  = B(hB)                 (the logical element unit hB must hold)
 *     hA = A^+(x)                (canonical source unit: free variables zero)
 *     dst[t*2^dB + hB] = src[t*2^dA + hA]
 */
int oracle_convert_general(const uint64_t *basesA, int dA, const uint64_t *basesB, int dB, int d_out,
                           int elem_bytes, const void *src, void *dst, int64_t ntiles)
{
    if (!basesA || !basesB || dA < 0 || dA > 30 || dB < 0 || dB > 30 || d_out < 0 || d_out > 30 ||
        elem_bytes <= 0 || ntiles < 0)
        return ORACLE_ERR_ARG;
    if (ntiles > 0 && (!src || !dst))
        return ORACLE_ERR_ARG;
    uint32_t *invA = (uint32_t *)malloc((1ull << d_out) * sizeof(uint32_t));
    uint32_t *invB = (uint32_t *)malloc((1ull << d_out) * sizeof(uint32_t));
    if (!invA || !invB) { free(invA); free(invB); return ORACLE_ERR_ALLOC; }
    int rc = oracle_right_inverse_table(basesA, dA, d_out, invA);
    if (rc == ORACLE_OK)
        rc = oracle_right_inverse_table(basesB, dB, d_out, invB);   /* only to check that B is surjective */
    if (rc != ORACLE_OK) { free(invA); free(invB); return rc; }
    const unsigned char *s = (const unsigned char *)src;
    unsigned char *o = (unsigned char *)dst;
    const uint64_t nA = 1ull << dA, nB = 1ull << dB;
    for (int64_t t = 0; t < ntiles; ++t) {
        for (uint64_t hB = 0; hB < nB; ++hB) {
            const uint64_t x = oracle_apply(basesB, dB, hB);
            const uint64_t hA = invA[x];
            memcpy(o + ((uint64_t)t * nB + hB) * (uint64_t)elem_bytes,
                   s + ((uint64_t)t * nA + hA) * (uint64_t)elem_bytes, (size_t)elem_bytes);
        }
    }
    free(invA);
    free(invB);
    return ORACLE_OK;
}

/*
 * Same result as oracle_convert_general.  The pull map hB -> A^+(B(hB)) does not
 * depend on the tile: it is tabulated once with the very statements of the plain
 * function, and the tile loop runs on all host threads.  For checking whole
 * full-size images, where the plain function would take minutes.
 */
int oracle_convert_general_table(const uint64_t *basesA, int dA, const uint64_t *basesB, int dB, int d_out,
                                 int elem_bytes, const void *src, void *dst, int64_t ntiles)
{
    if (!basesA || !basesB || dA < 0 || dA > 30 || dB < 0 || dB > 30 || d_out < 0 || d_out > 30 ||
        elem_bytes <= 0 || ntiles < 0)
        return ORACLE_ERR_ARG;
    if (ntiles > 0 && (!src || !dst))
        return ORACLE_ERR_ARG;
    const uint64_t nA = 1ull << dA, nB = 1ull << dB;
    uint32_t *invA = (uint32_t *)malloc((1ull << d_out) * sizeof(uint32_t));
    uint32_t *invB = (uint32_t *)malloc((1ull << d_out) * sizeof(uint32_t));
    uint32_t *pull = (uint32_t *)malloc(nB * sizeof(uint32_t));
    if (!invA || !invB || !pull) { free(invA); free(invB); free(pull); return ORACLE_ERR_ALLOC; }
    int rc = oracle_right_inverse_table(basesA, dA, d_out, invA);
    if (rc == ORACLE_OK)
        rc = oracle_right_inverse_table(basesB, dB, d_out, invB);   /* only to check that B is surjective */
    if (rc != ORACLE_OK) { free(invA); free(invB); free(pull); return rc; }
    for (uint64_t hB = 0; hB < nB; ++hB) {
        const uint64_t x = oracle_apply(basesB, dB, hB);
        pull[hB] = invA[x];
    }
    const unsigned char *s = (const unsigned char *)src;
    unsigned char *o = (unsigned char *)dst;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t t = 0; t < ntiles; ++t) {
        for (uint64_t hB = 0; hB < nB; ++hB)
            memcpy(o + ((uint64_t)t * nB + hB) * (uint64_t)elem_bytes,
                   s + ((uint64_t)t * nA + pull[hB]) * (uint64_t)elem_bytes, (size_t)elem_bytes);
    }
    free(invA);
    free(invB);
    free(pull);
    return ORACLE_OK;
}

/*
 * The same with affine layouts (Conclusions: y = A x xor b): slot hA of the
 * source holds the logical element A(hA) xor offA, slot hB of the destination
 * must hold B(hB) xor offB; the canonical source slot of a logical element x is
 * A^+(x xor offA).
 */
int oracle_convert_general_affine(const uint64_t *basesA, uint64_t offA, int dA, const uint64_t *basesB,
                                  uint64_t offB, int dB, int d_out, int elem_bytes, const void *src,
                                  void *dst, int64_t ntiles)
{
    if (!basesA || !basesB || dA < 0 || dA > 30 || dB < 0 || dB > 30 || d_out < 0 || d_out > 30 ||
        elem_bytes <= 0 || ntiles < 0 || (offA >> d_out) || (offB >> d_out))
        return ORACLE_ERR_ARG;
    if (ntiles > 0 && (!src || !dst))
        return ORACLE_ERR_ARG;
    uint32_t *invA = (uint32_t *)malloc((1ull << d_out) * sizeof(uint32_t));
    uint32_t *invB = (uint32_t *)malloc((1ull << d_out) * sizeof(uint32_t));
    if (!invA || !invB) { free(invA); free(invB); return ORACLE_ERR_ALLOC; }
    int rc = oracle_right_inverse_table(basesA, dA, d_out, invA);
    if (rc == ORACLE_OK)
        rc = oracle_right_inverse_table(basesB, dB, d_out, invB);   /* only to check that B is surjective */
    if (rc != ORACLE_OK) { free(invA); free(invB); return rc; }
    const unsigned char *s = (const unsigned char *)src;
    unsigned char *o = (unsigned char *)dst;
    const uint64_t nA = 1ull << dA, nB = 1ull << dB;
    for (int64_t t = 0; t < ntiles; ++t) {
        for (uint64_t hB = 0; hB < nB; ++hB) {
            const uint64_t x = oracle_apply(basesB, dB, hB) ^ offB;     /* logical element of slot hB */
            const uint64_t hA = invA[x ^ offA];                          /* A(hA) xor offA = x */
            memcpy(o + ((uint64_t)t * nB + hB) * (uint64_t)elem_bytes,
                   s + ((uint64_t)t * nA + hA) * (uint64_t)elem_bytes, (size_t)elem_bytes);
        }
    }
    free(invA);
    free(invB);
    return ORACLE_OK;
}

/*
 * Layout conversion A -> B on images (Sec. 5.4: the conversion is B^-1 o A).
 * For every tile t and every source hardware index hA:
 *     x  = A(hA)                      (logical element held at hA)
 *     hB = the unique index with B(hB) = x
 *     dst[t*2^d + hB] = src[t*2^d + hA]      (bytes copied verbatim)
 */
int oracle_convert(const uint64_t *basesA, const uint64_t *basesB, int d,
                   int elem_bytes, const void *src, void *dst, int64_t ntiles)
{
    if (!basesA || !basesB || d < 0 || d > 30 || elem_bytes <= 0 || ntiles < 0)
        return ORACLE_ERR_ARG;
    if (ntiles > 0 && (!src || !dst))
        return ORACLE_ERR_ARG;
    const uint64_t n = 1ull << d;
    uint32_t *invB = (uint32_t *)malloc(n * sizeof(uint32_t));
    uint32_t *invA = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!invB || !invA) { free(invB); free(invA); return ORACLE_ERR_ALLOC; }
    int rc = oracle_inverse_table(basesB, d, invB);
    if (rc == ORACLE_OK)
        rc = oracle_inverse_table(basesA, d, invA); /* A must be bijective too */
    if (rc != ORACLE_OK) { free(invB); free(invA); return rc; }
    const unsigned char *s = (const unsigned char *)src;
    unsigned char *o = (unsigned char *)dst;
    for (int64_t t = 0; t < ntiles; ++t) {
        for (uint64_t hA = 0; hA < n; ++hA) {
            uint64_t x = oracle_apply(basesA, d, hA);
            uint64_t hB = invB[x];
            memcpy(o + ((uint64_t)t * n + hB) * (uint64_t)elem_bytes,
                   s + ((uint64_t)t * n + hA) * (uint64_t)elem_bytes,
                   (size_t)elem_bytes);
        }
    }
    free(invB);
    free(invA);
    return ORACLE_OK;
}

/*
 * Same result as oracle_convert.  The composed map hA -> hB is tabulated once
 * (it does not depend on the tile) and the tile loop runs on all host threads.
 * Returns the number of threads used through *threads_used (may be NULL).
 */
#ifdef _OPENMP
#include <omp.h>
#endif
int oracle_convert_table(const uint64_t *basesA, const uint64_t *basesB, int d,
                         int elem_bytes, const void *src, void *dst,
                         int64_t ntiles, int *threads_used)
{
    if (!basesA || !basesB || d < 0 || d > 30 || elem_bytes <= 0 || ntiles < 0)
        return ORACLE_ERR_ARG;
    if (ntiles > 0 && (!src || !dst))
        return ORACLE_ERR_ARG;
    const uint64_t n = 1ull << d;
    uint32_t *invB = (uint32_t *)malloc(n * sizeof(uint32_t));
    uint32_t *pmap = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!invB || !pmap) { free(invB); free(pmap); return ORACLE_ERR_ALLOC; }
    int rc = oracle_inverse_table(basesB, d, invB);
    if (rc == ORACLE_OK) {
        /* A bijective <=> the composed map is a permutation of [0, 2^d) */
        unsigned char *seen = (unsigned char *)calloc(n, 1);
        if (!seen) { free(invB); free(pmap); return ORACLE_ERR_ALLOC; }
        for (uint64_t hA = 0; hA < n && rc == ORACLE_OK; ++hA) {
            uint64_t x = oracle_apply(basesA, d, hA);
            if (x >= n) { rc = ORACLE_ERR_NOT_BIJECTIVE; break; }
            pmap[hA] = invB[x];
            if (seen[pmap[hA]]) rc = ORACLE_ERR_NOT_BIJECTIVE;
            seen[pmap[hA]] = 1;
        }
        free(seen);
    }
    if (rc != ORACLE_OK) { free(invB); free(pmap); return rc; }
    const unsigned char *s = (const unsigned char *)src;
    unsigned char *o = (unsigned char *)dst;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(static)
#endif
    for (int64_t t = 0; t < ntiles; ++t) {
        const unsigned char *st = s + (uint64_t)t * n * (uint64_t)elem_bytes;
        unsigned char *ot = o + (uint64_t)t * n * (uint64_t)elem_bytes;
        for (uint64_t hA = 0; hA < n; ++hA)
            memcpy(ot + (uint64_t)pmap[hA] * (uint64_t)elem_bytes,
                   st + hA * (uint64_t)elem_bytes, (size_t)elem_bytes);
    }
    if (threads_used) *threads_used = nthreads;
    free(invB);
    free(pmap);
    return ORACLE_OK;
}

/*
 * Gather along `axis` (Sec. 5.5), all three tensors under the same bijective
 * layout L on d bits.  out_dim_bits[k] is log2 of logical dimension k, slowest
 * dimension first (the last one is the fastest, in the low bits of the
 * flattened index).  For every tile and every hardware index h:
 *     x = L(h); split x into coordinates; s = idx_img[h] & (len(axis) - 1);
 *     x' = x with the axis coordinate replaced by s;
 *     out_img[h] = in_img[L^-1(x')].
 * Out-of-range indices are reduced modulo the axis length (a power of two).
 */
int oracle_gather(const uint64_t *basesL, int d, const int32_t *out_dim_bits,
                  int n_out_dims, int axis, int elem_bytes, const void *in,
                  const int32_t *idx, void *out, int64_t ntiles)
{
    if (!basesL || !out_dim_bits || d < 0 || d > 30 || elem_bytes <= 0 ||
        ntiles < 0 || n_out_dims <= 0)
        return ORACLE_ERR_ARG;
    if (axis < 0 || axis >= n_out_dims)
        return ORACLE_ERR_AXIS;
    if (ntiles > 0 && (!in || !idx || !out))
        return ORACLE_ERR_ARG;
    int total = 0, axis_shift = 0;
    for (int k = n_out_dims - 1; k >= 0; --k) { /* last dim sits lowest */
        if (k == axis) axis_shift = total;
        total += out_dim_bits[k];
    }
    if (total != d)
        return ORACLE_ERR_ARG;
    const int axis_bits = out_dim_bits[axis];
    const uint64_t axis_len_mask = (1ull << axis_bits) - 1;
    const uint64_t n = 1ull << d;
    uint32_t *invL = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!invL) return ORACLE_ERR_ALLOC;
    int rc = oracle_inverse_table(basesL, d, invL);
    if (rc != ORACLE_OK) { free(invL); return rc; }
    const unsigned char *pi = (const unsigned char *)in;
    unsigned char *po = (unsigned char *)out;
    for (int64_t t = 0; t < ntiles; ++t) {
        const uint64_t base = (uint64_t)t * n;
        for (uint64_t h = 0; h < n; ++h) {
            uint64_t x = oracle_apply(basesL, d, h);
            uint64_t s = (uint64_t)(uint32_t)idx[base + h] & axis_len_mask;
            uint64_t xs = (x & ~(axis_len_mask << axis_shift)) | (s << axis_shift);
            uint64_t hs = invL[xs];
            memcpy(po + (base + h) * (uint64_t)elem_bytes,
                   pi + (base + hs) * (uint64_t)elem_bytes, (size_t)elem_bytes);
        }
    }
    free(invL);
    return ORACLE_OK;
}

/*
 * Same result as oracle_gather.  L(h) and L^-1 are tabulated once (L(h) with the
 * very statement of the plain function) and the tile loop runs on all host
 * threads.  For checking whole full-size images.
 */
int oracle_gather_table(const uint64_t *basesL, int d, const int32_t *out_dim_bits,
                        int n_out_dims, int axis, int elem_bytes, const void *in,
                        const int32_t *idx, void *out, int64_t ntiles)
{
    if (!basesL || !out_dim_bits || d < 0 || d > 30 || elem_bytes <= 0 ||
        ntiles < 0 || n_out_dims <= 0)
        return ORACLE_ERR_ARG;
    if (axis < 0 || axis >= n_out_dims)
        return ORACLE_ERR_AXIS;
    if (ntiles > 0 && (!in || !idx || !out))
        return ORACLE_ERR_ARG;
    int total = 0, axis_shift = 0;
    for (int k = n_out_dims - 1; k >= 0; --k) { /* last dim sits lowest */
        if (k == axis) axis_shift = total;
        total += out_dim_bits[k];
    }
    if (total != d)
        return ORACLE_ERR_ARG;
    const int axis_bits = out_dim_bits[axis];
    const uint64_t axis_len_mask = (1ull << axis_bits) - 1;
    const uint64_t n = 1ull << d;
    uint32_t *invL = (uint32_t *)malloc(n * sizeof(uint32_t));
    uint32_t *fwdL = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!invL || !fwdL) { free(invL); free(fwdL); return ORACLE_ERR_ALLOC; }
    int rc = oracle_inverse_table(basesL, d, invL);
    if (rc != ORACLE_OK) { free(invL); free(fwdL); return rc; }
    for (uint64_t h = 0; h < n; ++h)
        fwdL[h] = (uint32_t)oracle_apply(basesL, d, h);
    const unsigned char *pi = (const unsigned char *)in;
    unsigned char *po = (unsigned char *)out;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t t = 0; t < ntiles; ++t) {
        const uint64_t base = (uint64_t)t * n;
        for (uint64_t h = 0; h < n; ++h) {
            uint64_t x = fwdL[h];
            uint64_t s = (uint64_t)(uint32_t)idx[base + h] & axis_len_mask;
            uint64_t xs = (x & ~(axis_len_mask << axis_shift)) | (s << axis_shift);
            uint64_t hs = invL[xs];
            memcpy(po + (base + h) * (uint64_t)elem_bytes,
                   pi + (base + hs) * (uint64_t)elem_bytes, (size_t)elem_bytes);
        }
    }
    free(invL);
    free(fwdL);
    return ORACLE_OK;
}

/*
 * Affine layouts (Conclusions: flips and slices are y = A x xor b).  An affine
 * layout is a bijective linear layout A on d bits plus a constant b < 2^d:
 * hardware index h holds the logical element A h xor b.
 *
 * Conversion between two affine layouts, by the definition on images: the
 * element at source index h is the logical element x = A h xor a; it goes to
 * the destination index h' with B h' xor b = x.  The inverse of the affine map
 * of the destination is tabulated (table[B h' xor b] = h'), never solved for.
 */
int oracle_convert_affine(const uint64_t *basesA, uint64_t offA, const uint64_t *basesB, uint64_t offB,
                          int d, int elem_bytes, const void *src, void *dst, int64_t ntiles)
{
    if (!basesA || !basesB || d < 0 || d > 30 || elem_bytes <= 0 || ntiles < 0)
        return ORACLE_ERR_ARG;
    if (ntiles > 0 && (!src || !dst))
        return ORACLE_ERR_ARG;
    const uint64_t n = 1ull << d;
    if (offA >= n || offB >= n) return ORACLE_ERR_ARG;
    uint32_t *where = (uint32_t *)malloc(n * sizeof(uint32_t));      /* logical x -> destination index */
    unsigned char *seen = (unsigned char *)calloc(n, 1);
    if (!where || !seen) { free(where); free(seen); return ORACLE_ERR_ALLOC; }
    int rc = ORACLE_OK;
    for (uint64_t h = 0; h < n; ++h) {
        uint64_t x = oracle_apply(basesB, d, h) ^ offB;
        if (x >= n || seen[x]) { rc = ORACLE_ERR_NOT_BIJECTIVE; break; }
        seen[x] = 1;
        where[x] = (uint32_t)h;
    }
    if (rc == ORACLE_OK) {
        memset(seen, 0, n);
        for (uint64_t h = 0; h < n; ++h) {                             /* A must be a bijection as well */
            uint64_t x = oracle_apply(basesA, d, h) ^ offA;
            if (x >= n || seen[x]) { rc = ORACLE_ERR_NOT_BIJECTIVE; break; }
            seen[x] = 1;
        }
    }
    if (rc == ORACLE_OK) {
        const unsigned char *s = (const unsigned char *)src;
        unsigned char *o = (unsigned char *)dst;
        for (int64_t t = 0; t < ntiles; ++t)
            for (uint64_t h = 0; h < n; ++h) {
                uint64_t x = oracle_apply(basesA, d, h) ^ offA;
                uint64_t to = where[x];
                memcpy(o + ((uint64_t)t * n + to) * (uint64_t)elem_bytes,
                       s + ((uint64_t)t * n + h) * (uint64_t)elem_bytes, (size_t)elem_bytes);
            }
    }
    free(where);
    free(seen);
    return rc;
}

/*
 * Gather along `axis` (Sec. 5.5) with all three tensors under the same affine
 * layout h -> L h xor off: for every hardware index h the logical position is
 * x = L h xor off; its axis coordinate is replaced by the index; the source is
 * the hardware index that holds that logical position (tabulated).
 */
int oracle_gather_affine(const uint64_t *basesL, uint64_t off, int d, const int32_t *out_dim_bits,
                         int n_out_dims, int axis, int elem_bytes, const void *in,
                         const int32_t *idx, void *out, int64_t ntiles)
{
    if (!basesL || !out_dim_bits || d < 0 || d > 30 || elem_bytes <= 0 || ntiles < 0 || n_out_dims <= 0)
        return ORACLE_ERR_ARG;
    if (axis < 0 || axis >= n_out_dims) return ORACLE_ERR_AXIS;
    if (ntiles > 0 && (!in || !idx || !out)) return ORACLE_ERR_ARG;
    int total = 0, axis_shift = 0;
    for (int k = n_out_dims - 1; k >= 0; --k) {
        if (k == axis) axis_shift = total;
        total += out_dim_bits[k];
    }
    if (total != d) return ORACLE_ERR_ARG;
    const uint64_t n = 1ull << d;
    if (off >= n) return ORACLE_ERR_ARG;
    const uint64_t axis_len_mask = (1ull << out_dim_bits[axis]) - 1;
    uint32_t *where = (uint32_t *)malloc(n * sizeof(uint32_t));
    unsigned char *seen = (unsigned char *)calloc(n, 1);
    if (!where || !seen) { free(where); free(seen); return ORACLE_ERR_ALLOC; }
    int rc = ORACLE_OK;
    for (uint64_t h = 0; h < n; ++h) {
        uint64_t x = oracle_apply(basesL, d, h) ^ off;
        if (x >= n || seen[x]) { rc = ORACLE_ERR_NOT_BIJECTIVE; break; }
        seen[x] = 1;
        where[x] = (uint32_t)h;
    }
    if (rc == ORACLE_OK) {
        const unsigned char *pi = (const unsigned char *)in;
        unsigned char *po = (unsigned char *)out;
        for (int64_t t = 0; t < ntiles; ++t) {
            const uint64_t base = (uint64_t)t * n;
            for (uint64_t h = 0; h < n; ++h) {
                uint64_t x = oracle_apply(basesL, d, h) ^ off;
                uint64_t s = (uint64_t)(uint32_t)idx[base + h] & axis_len_mask;
                uint64_t xs = (x & ~(axis_len_mask << axis_shift)) | (s << axis_shift);
                memcpy(po + (base + h) * (uint64_t)elem_bytes,
                       pi + (base + where[xs]) * (uint64_t)elem_bytes, (size_t)elem_bytes);
            }
        }
    }
    free(where);
    free(seen);
    return rc;
}

/*
 * Exhaustive wavefront (bank-conflict) count of one shared-memory access
 * pattern (Sec. 5.4 "Optimal Swizzling"; appendix lemma on wavefronts).
 *
 *   mem_bases   memory layout M on d bits: offset (in elements) -> logical
 *   dist_bases  distributed layout L on d bits: hardware index -> logical,
 *               input bits ordered reg (nreg), lane (nlane), then the rest
 *   elem_bytes  w
 *   vec_bits    v: one instruction moves the 2^v elements of registers
 *               r0 .. r0 + 2^v - 1 (r0 a multiple of 2^v) of a lane
 *   nbanks      number of 4-byte banks
 *   phase_of_lane[l]  lanes with the same value are served together
 *
 * For every wave (all settings of the bits above the lane bits), every vector
 * slot r0 and every phase: gather the 4-byte words the lanes of the phase
 * touch at offsets M^-1(L(h)); the phase needs max over banks of the number
 * of DISTINCT words that fall in that bank (same word twice is a broadcast).
 *
 * Results: *max_wavefronts = largest count over all phases;
 *          *total_wavefronts = sum over all phases;
 *          *total_phases = number of (wave, slot, phase) triples that touch
 *          at least one word (the conflict-free total).
 */
int oracle_wavefronts(const uint64_t *mem_bases, const uint64_t *dist_bases,
                      int d, int nreg, int nlane, int elem_bytes, int vec_bits,
                      int nbanks, const int32_t *phase_of_lane,
                      int64_t *max_wavefronts, int64_t *total_wavefronts,
                      int64_t *total_phases)
{
    if (!mem_bases || !dist_bases || !phase_of_lane || d < 0 || d > 26 ||
        nreg < 0 || nlane < 0 || nreg + nlane > d || vec_bits < 0 ||
        vec_bits > nreg || nbanks <= 0 || elem_bytes <= 0)
        return ORACLE_ERR_ARG;
    const uint64_t n = 1ull << d;
    const int nlanes = 1 << nlane;
    uint32_t *invM = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!invM) return ORACLE_ERR_ALLOC;
    int rc = oracle_inverse_table(mem_bases, d, invM);
    if (rc != ORACLE_OK) { free(invM); return rc; }
    int nphases = 0;
    for (int l = 0; l < nlanes; ++l)
        if (phase_of_lane[l] + 1 > nphases) nphases = phase_of_lane[l] + 1;
    const int vec = 1 << vec_bits;
    const int max_words = nlanes * vec * ((elem_bytes + 3) / 4 + 1);
    uint64_t *words = (uint64_t *)malloc((size_t)max_words * sizeof(uint64_t));
    int *bank_count = (int *)malloc((size_t)nbanks * sizeof(int));
    if (!words || !bank_count) { free(invM); free(words); free(bank_count); return ORACLE_ERR_ALLOC; }
    int64_t maxw = 0, totw = 0, totp = 0;
    const uint64_t nwaves = n >> (nreg + nlane);
    for (uint64_t wv = 0; wv < nwaves; ++wv) {
        for (int r0 = 0; r0 < (1 << nreg); r0 += vec) {
            for (int ph = 0; ph < nphases; ++ph) {
                int nw = 0;
                for (int l = 0; l < nlanes; ++l) {
                    if (phase_of_lane[l] != ph) continue;
                    for (int e = 0; e < vec; ++e) {
                        uint64_t h = (uint64_t)(r0 + e) | ((uint64_t)l << nreg) |
                                     (wv << (nreg + nlane));
                        uint64_t off = invM[oracle_apply(dist_bases, d, h)];
                        uint64_t b0 = off * (uint64_t)elem_bytes;
                        uint64_t b1 = b0 + (uint64_t)elem_bytes - 1;
                        for (uint64_t wd = b0 / 4; wd <= b1 / 4; ++wd) {
                            int dup = 0;
                            for (int q = 0; q < nw; ++q)
                                if (words[q] == wd) { dup = 1; break; }
                            if (!dup) words[nw++] = wd;
                        }
                    }
                }
                if (nw == 0) continue;
                memset(bank_count, 0, (size_t)nbanks * sizeof(int));
                int worst = 0;
                for (int q = 0; q < nw; ++q) {
                    int b = (int)(words[q] % (uint64_t)nbanks);
                    if (++bank_count[b] > worst) worst = bank_count[b];
                }
                if (worst > maxw) maxw = worst;
                totw += worst;
                totp += 1;
            }
        }
    }
    if (max_wavefronts) *max_wavefronts = maxw;
    if (total_wavefronts) *total_wavefronts = totw;
    if (total_phases) *total_phases = totp;
    free(invM); free(words); free(bank_count);
    return ORACLE_OK;
}
