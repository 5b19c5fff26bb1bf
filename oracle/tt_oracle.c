/*
 * CPU oracle for the out-of-place rank-n dense tensor transpose.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is
 * compared against.  It shares no code, header, table or helper with the HIP
 * path, and nothing in the product path may call it.
 *
 * Conventions (0-based restatement of the notation of Section 2 of the paper):
 *   dims[0] is the stride-1 dimension, later dimensions are more senior.
 *   perm[j] is the input dimension that sits at output position j (the
 *   paper's w_{j+1} - 1), so the output extents are odims[j] = dims[perm[j]].
 *   sI[z] = prod_{t<z} dims[t]          -- cumulative volume c(z, I)
 *   sO[j] = prod_{t<j} dims[perm[t]]    -- cumulative volume c(perm[j], O)
 *
 * Everything is written the slow, obvious way: one element at a time, every
 * coordinate recovered by an integer division and a modulo (the inverse of
 * the scalar position, Section 2), every offset re-summed from scratch.  No
 * blocking, no incremental index updates.  Elements are moved as raw bytes so
 * NaN payloads, -0.0 and denormals survive.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define TTO_MAX_RANK 32

enum { TTO_OK = 0, TTO_BAD_RANK = 1, TTO_BAD_DIMS = 2, TTO_BAD_PERM = 3, TTO_BAD_ELEM = 4 };

/* Argument check: rank in range, extents positive, perm a permutation. */
static int tto_check(int rank, const int64_t *dims, const int *perm, size_t elem)
{
    int seen[TTO_MAX_RANK];
    if (rank < 1 || rank > TTO_MAX_RANK) return TTO_BAD_RANK;
    if (elem < 1) return TTO_BAD_ELEM;
    for (int z = 0; z < rank; ++z) {
        if (dims[z] < 1) return TTO_BAD_DIMS;
        seen[z] = 0;
    }
    for (int j = 0; j < rank; ++j) {
        if (perm[j] < 0 || perm[j] >= rank || seen[perm[j]]) return TTO_BAD_PERM;
        seen[perm[j]] = 1;
    }
    return TTO_OK;
}

/* Cumulative volumes of the input layout I = {0,1,..} and of the output layout
 * O = {perm[0], perm[1], ..} (definition of c(z,{w}) in Section 2). */
static void tto_strides(int rank, const int64_t *dims, const int *perm,
                        int64_t *sI, int64_t *sO)
{
    for (int z = 0; z < rank; ++z) {
        int64_t c = 1;
        for (int t = 0; t < z; ++t) c *= dims[t];
        sI[z] = c;
    }
    for (int j = 0; j < rank; ++j) {
        int64_t c = 1;
        for (int t = 0; t < j; ++t) c *= dims[perm[t]];
        sO[j] = c;
    }
}

int64_t tto_volume(int rank, const int64_t *dims)
{
    int64_t v = 1;
    for (int z = 0; z < rank; ++z) v *= dims[z];
    return v;
}

/*
 * Scalar position in the input of the element that lands at output scalar
 * position o.  The output coordinates are recovered with the inverse of the
 * scalar-position map (x_j = floor(o / sO[j]) mod odims[j]); coordinate j of
 * the output is coordinate perm[j] of the input, so the input position is
 * sum_j x_j * sI[perm[j]].  Returns -1 on bad arguments.
 */
int64_t tto_input_position(int rank, const int64_t *dims, const int *perm, int64_t o)
{
    int64_t sI[TTO_MAX_RANK], sO[TTO_MAX_RANK];
    if (tto_check(rank, dims, perm, 1) != TTO_OK) return -1;
    tto_strides(rank, dims, perm, sI, sO);
    int64_t p = 0;
    for (int j = 0; j < rank; ++j) {
        int64_t x = (o / sO[j]) % dims[perm[j]];
        p += x * sI[perm[j]];
    }
    return p;
}

/*
 * Gather form: for every output scalar position o, copy the element found at
 * the matching input scalar position.  Iterations are independent, so the
 * loop is handed to OpenMP as it stands (nthreads <= 0: library default).
 */
int tto_transpose_gather(int rank, const int64_t *dims, const int *perm, size_t elem,
                         const void *in, void *out, int nthreads)
{
    int64_t sI[TTO_MAX_RANK], sO[TTO_MAX_RANK];
    int rc = tto_check(rank, dims, perm, elem);
    if (rc != TTO_OK) return rc;
    tto_strides(rank, dims, perm, sI, sO);
    const int64_t vol = tto_volume(rank, dims);
    const unsigned char *src = (const unsigned char *)in;
    unsigned char *dst = (unsigned char *)out;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t o = 0; o < vol; ++o) {
        int64_t p = 0;
        for (int j = 0; j < rank; ++j) {
            int64_t x = (o / sO[j]) % dims[perm[j]];
            p += x * sI[perm[j]];
        }
        memcpy(dst + (size_t)o * elem, src + (size_t)p * elem, elem);
    }
    return TTO_OK;
}

/*
 * Accumulating form (the mode of the paper's third benchmark set, Section 3.3: read input,
 * read output, accumulate, write output): out[o] = out[o] + in[p(o)], one IEEE addition
 * per output element, in binary32 for 4-byte and binary64 for 8-byte elements.
 */
int tto_transpose_accumulate(int rank, const int64_t *dims, const int *perm, size_t elem,
                             const void *in, void *out)
{
    int64_t sI[TTO_MAX_RANK], sO[TTO_MAX_RANK];
    int rc = tto_check(rank, dims, perm, elem);
    if (rc != TTO_OK) return rc;
    if (elem != 4 && elem != 8) return TTO_BAD_ELEM;
    tto_strides(rank, dims, perm, sI, sO);
    const int64_t vol = tto_volume(rank, dims);
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < vol; ++o) {
        int64_t p = 0;
        for (int j = 0; j < rank; ++j) {
            int64_t x = (o / sO[j]) % dims[perm[j]];
            p += x * sI[perm[j]];
        }
        if (elem == 8) {
            volatile double s = ((double *)out)[o] + ((const double *)in)[p];
            ((double *)out)[o] = s;
        } else {
            volatile float s = ((float *)out)[o] + ((const float *)in)[p];
            ((float *)out)[o] = s;
        }
    }
    return TTO_OK;
}

/*
 * Scatter form, Eq. (1): walk the input linearly; recover the input
 * coordinate y_z of every dimension z from the input scalar position and
 * multiply it by the cumulative volume of that same dimension z in the output
 * layout.  (The printed equation pairs coordinate i with the stride of w_i;
 * that only holds for involutions.  The reading taken here -- stride of the
 * dimension whose coordinate it is -- is the one Eqs. (2)-(5) use.)
 */
int tto_transpose_scatter(int rank, const int64_t *dims, const int *perm, size_t elem,
                          const void *in, void *out)
{
    int64_t sI[TTO_MAX_RANK], sO[TTO_MAX_RANK], cO[TTO_MAX_RANK];
    int rc = tto_check(rank, dims, perm, elem);
    if (rc != TTO_OK) return rc;
    tto_strides(rank, dims, perm, sI, sO);
    /* cO[z] = c(z, O): stride in the output of input dimension z. */
    for (int j = 0; j < rank; ++j) cO[perm[j]] = sO[j];
    const int64_t vol = tto_volume(rank, dims);
    const unsigned char *src = (const unsigned char *)in;
    unsigned char *dst = (unsigned char *)out;
    for (int64_t p = 0; p < vol; ++p) {
        int64_t q = 0;
        for (int z = 0; z < rank; ++z) {
            int64_t y = (p / sI[z]) % dims[z];
            q += y * cO[z];
        }
        memcpy(dst + (size_t)q * elem, src + (size_t)p * elem, elem);
    }
    return TTO_OK;
}

/*
 * Sampled outputs: vals[i] = element at output scalar position pos[i], taken
 * straight from the input.  Lets a test check a huge GPU result at chosen
 * positions without building the whole expected tensor.
 */
int tto_sample(int rank, const int64_t *dims, const int *perm, size_t elem,
               const void *in, int64_t n, const int64_t *pos, void *vals)
{
    int rc = tto_check(rank, dims, perm, elem);
    if (rc != TTO_OK) return rc;
    const int64_t vol = tto_volume(rank, dims);
    const unsigned char *src = (const unsigned char *)in;
    unsigned char *dst = (unsigned char *)vals;
    for (int64_t i = 0; i < n; ++i) {
        if (pos[i] < 0 || pos[i] >= vol) return TTO_BAD_DIMS;
        int64_t p = tto_input_position(rank, dims, perm, pos[i]);
        memcpy(dst + (size_t)i * elem, src + (size_t)p * elem, elem);
    }
    return TTO_OK;
}

/*
 * Binary tensor contraction D = D + L * R (the operation of Section 3.4, written as the
 * direct loop nest that Section 1 calls the direct approach): every element of D receives the
 * sum, over all values of the contracted labels, of the product of the matching elements of L
 * and R.
 *
 * Labels are numbered 0..nlab-1 with extents ext[].  Each tensor is a flat buffer whose
 * dimensions are the labels listed in dl / ll / rl, first one = stride-1 dimension.  Labels
 * that occur in both ll and rl and not in dl are summed over; the products of one output
 * element are added in double precision in a fixed order (summed labels in the order they
 * appear in ll, the first of them running fastest), then that sum is added to D once.
 * elem = 8: buffers are double; elem = 4: buffers are float, widened for the arithmetic and
 * rounded to float once at the end.  No blocking, no reordering, one output element at a time.
 */
int tto_contract(int nlab, const int64_t *ext, int nd, const int *dl, int nl, const int *ll,
                 int nr, const int *rl, size_t elem, const void *l, const void *r, void *d)
{
    int in_d[TTO_MAX_RANK], in_l[TTO_MAX_RANK], in_r[TTO_MAX_RANK];
    int64_t sl[TTO_MAX_RANK], sr[TTO_MAX_RANK];   /* stride of a label in L / R, 0 if absent */
    int summed[TTO_MAX_RANK], ns = 0;
    if (nlab < 1 || nlab > TTO_MAX_RANK || nd < 1 || nl < 1 || nr < 1) return TTO_BAD_RANK;
    if (nd > nlab || nl > nlab || nr > nlab) return TTO_BAD_RANK;
    if (elem != 4 && elem != 8) return TTO_BAD_ELEM;
    for (int a = 0; a < nlab; ++a) {
        if (ext[a] < 1) return TTO_BAD_DIMS;
        in_d[a] = in_l[a] = in_r[a] = 0;
        sl[a] = sr[a] = 0;
    }
    for (int j = 0; j < nd; ++j) {   /* D is walked by its own scalar position o: no strides needed */
        if (dl[j] < 0 || dl[j] >= nlab || in_d[dl[j]]) return TTO_BAD_PERM;
        in_d[dl[j]] = 1;
    }
    int64_t c = 1;
    for (int j = 0; j < nl; ++j) {
        if (ll[j] < 0 || ll[j] >= nlab || in_l[ll[j]]) return TTO_BAD_PERM;
        in_l[ll[j]] = 1; sl[ll[j]] = c; c *= ext[ll[j]];
    }
    c = 1;
    for (int j = 0; j < nr; ++j) {
        if (rl[j] < 0 || rl[j] >= nlab || in_r[rl[j]]) return TTO_BAD_PERM;
        in_r[rl[j]] = 1; sr[rl[j]] = c; c *= ext[rl[j]];
    }
    /* every label: either summed (in L and R, not in D) or free (in D and exactly one input) */
    for (int a = 0; a < nlab; ++a) {
        const int s = in_l[a] && in_r[a] && !in_d[a];
        const int f = in_d[a] && (in_l[a] != in_r[a]);
        if (!s && !f) return TTO_BAD_PERM;
    }
    for (int j = 0; j < nl; ++j)
        if (in_r[ll[j]]) summed[ns++] = ll[j];
    int64_t vol_d = 1, vol_s = 1;
    for (int j = 0; j < nd; ++j) vol_d *= ext[dl[j]];
    for (int j = 0; j < ns; ++j) vol_s *= ext[summed[j]];
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < vol_d; ++o) {
        int64_t coord[TTO_MAX_RANK];
        int64_t rem = o;
        for (int j = 0; j < nd; ++j) {          /* coordinates of the free labels from o */
            coord[dl[j]] = rem % ext[dl[j]];
            rem /= ext[dl[j]];
        }
        double acc = 0.0;
        for (int64_t q = 0; q < vol_s; ++q) {
            int64_t t = q;
            for (int j = 0; j < ns; ++j) {      /* coordinates of the summed labels from q */
                coord[summed[j]] = t % ext[summed[j]];
                t /= ext[summed[j]];
            }
            int64_t pl = 0, pr = 0;
            for (int a = 0; a < nlab; ++a) {
                if (in_l[a]) pl += coord[a] * sl[a];
                if (in_r[a]) pr += coord[a] * sr[a];
            }
            const double x = elem == 8 ? ((const double *)l)[pl] : (double)((const float *)l)[pl];
            const double y = elem == 8 ? ((const double *)r)[pr] : (double)((const float *)r)[pr];
            volatile double prod = x * y;       /* a rounded product, then a rounded sum */
            acc = acc + prod;
        }
        if (elem == 8) ((double *)d)[o] = ((double *)d)[o] + acc;
        else ((float *)d)[o] = (float)((double)((float *)d)[o] + acc);
    }
    return TTO_OK;
}

int tto_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
