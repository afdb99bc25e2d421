/*
 * CPU oracle for the sparse-convolution hot path of fVDB (arXiv 2407.01781).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
 * path is checked against.  It shares no code with the HIP path and must never be
 * called from it: only tests, the smoke check and the benchmark's CPU-baseline leg
 * load this library.
 *
 * What it computes, and the passage each part follows:
 *
 *  O1  index grid  -- Sec. 3.2 (IndexGrid: only active voxels get a linear index
 *      into side-car arrays), Listing 1 (leaf record: mOffset, mPrefixSum,
 *      mBitMask[8], off = (i&7)<<6|(j&7)<<3|k&7), Listing 2 (lower/upper node
 *      offsets) and Sec. 3.3 steps 2-9 (voxels ordered by root-tile key, then by
 *      upper, lower and leaf offsets; node counts = numbers of distinct key
 *      prefixes).  The build algorithm of Sec. 3.3 reaches exactly one result, a
 *      total order of the distinct voxels, so the oracle is that order written out:
 *      a hash set for de-duplication and a comparison sort on the 12 fields
 *      (tile i,j,k signed; upper i,j,k; lower i,j,k; leaf i,j,k).  No tree is built.
 *      Sec. 3.6 (GridBatch = grids stored one after the other; JaggedTensor jdata /
 *      joffsets [B,2]) fixes the batch convention: grid b's voxels take the indices
 *      base_b .. base_b + N_b - 1, base_b = sum of the earlier grids' voxel counts.
 *
 *  O2  kernel map  -- Sec. 3.5 (stencil "spokes"; scenario 3(c): input/output index
 *      pairs linked by an offset; scenario 1: neighbour indices come from the tree's
 *      index lookup).  nbmap[o][kappa] = index of the input voxel at
 *      stride*p_o + delta_kappa, or -1.  Found here with the hash map only.
 *
 *  O3  convolution -- Sec. 3.6.2 (convolution takes G_in, kernel K, features Z_in and
 *      gives G_out, Z_out) and Sec. 4.1.3 (effective FLOPs count only stencil taps
 *      whose input voxel is active):
 *          out[o,:] = sum over kappa with an active input of  in[nb(o,kappa),:] . W[kappa]
 *      accumulated in double, looping voxel -> offset -> C_in -> C_out, neighbours
 *      found through this file's own hash map (not through O2's output).
 *
 *  O4  backward pass -- Sec. 3.6 / 3.6.2 call the operators differentiable and Sec. 4.1.3
 *      speaks of the gradient with respect to the filter coefficients; no formula is
 *      printed, so the oracle is the derivative of O3's formula written out.  With
 *      L any scalar function of out and gout = dL/dout:
 *          gin[i,:]      = sum over pairs (o,kappa) with nb(o,kappa) = i of  W[kappa] . gout[o,:]
 *          gw[kappa,:,:] = sum over outputs o with an active input of  in[nb(o,kappa),:]^T gout[o,:]
 *      both accumulated in double by walking the same voxel -> offset loop as O3 and
 *      adding each pair's contribution where it belongs.
 *
 *  O5  transposed convolution, pooling, upsampling -- Sec. 3.6.2 lists, beside the
 *      convolution, average and max pooling on a GridBatch / JaggedTensor pair and an
 *      operator that upsamples a grid and its features by subdivision and nearest-
 *      neighbour sampling; Sec. 4.1.4's encoder-decoder network goes back up to the fine
 *      resolution.  No formula is printed.  With nb(o,kappa) the map of a convolution
 *      from a fine grid (inputs i) to a coarser one (outputs o):
 *          transposed convolution  out[i,:] = sum over pairs (o,kappa) with nb(o,kappa) = i
 *                                             of  z[o,:] . W[kappa]        (z lives on the outputs o;
 *                                             the adjoint of O3 in the features for the weights
 *                                             W[kappa]^T, i.e. O4's input gradient with W read as
 *                                             [c_in, c_out] of the new direction)
 *          pooling, factor 2       out[o,c] = max / mean over the active children i of o (the
 *                                             voxels with floor(ijk_i / 2) = ijk_o) of z[i,c]
 *          upsampling, factor 2    fine grid = all 8 children 2*ijk + {0,1}^3 of every coarse voxel
 *                                  (fo_grid_subdivide2), or any given fine grid; out[i,:] = z[parent(i),:],
 *                                  zero where the parent is not active
 *      All are written as plain loops over voxels with this file's hash map.
 *      Their gradients (Sec. 3.6: the operators are differentiable) are the derivatives of those sums:
 *          mean pooling   gin[i,c] = gout[o,c] / n(o)      o the parent of i, n(o) its active children
 *          max pooling    gin[i,c] = gout[o,c] for the child i that attains the maximum of channel c --
 *                         the first one in offset order when several are equal, the one the forward
 *                         pass keeps -- and 0 for the others
 *          upsampling     gin[o,c] = sum over the active children i of o of gout[i,c]
 *
 *  O7  padded grid -- Sec. 3.6.2 lists padding beside coarsening and subdivision among the ways to
 *      make a grid from another; Sec. 3.3 names morphological dilation as the case that changes
 *      topology.  No formula is printed; the reading taken: padding by r >= 0 voxels activates
 *      every voxel within Chebyshev distance r of an active one, per grid of the batch,
 *          S' = { p + d : p in S, d in {-r..r}^3 }
 *      (r = 1: the voxels a 3x3x3 stencil centred on them reaches S from -- the output set of a
 *      convolution that is not restricted to the input's voxels).  Written as that union.
 *
 *  O6  voxel coordinates of points -- Sec. 3.6.2 and Sec. 4.1.1: a grid can be built from
 *      xyz point coordinates as well as from ijk.  No formula is printed; the reading taken:
 *      voxel (i,j,k) is the half-open cell [origin + i*s, origin + (i+1)*s) per axis, so
 *          ijk = floor((xyz - origin) / voxel_size)
 *      evaluated in IEEE single precision (one rounded subtraction, one rounded division,
 *      floorf), the precision of the input; a point is invalid if the quotient is not finite
 *      or its floor lies outside [-2^30, 2^30).  The grid of a point cloud is O1 applied to
 *      these coordinates.
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - exported indices are 0-based rows of jdata, -1 means inactive (the paper's
 *     in-tree index 0 is its background value);
 *   - offsets: K odd -> delta in {-(K-1)/2..(K-1)/2}^3, K even -> {0..K-1}^3;
 *     kappa = (di-dmin)*K*K + (dj-dmin)*K + (dk-dmin), i slowest as in Listing 1;
 *   - weights W[kappa][c_in][c_out]; cross-correlation, no flip, no bias;
 *   - stride 1: output voxel set = input set; stride 2: output set = distinct
 *     floor(ijk/2) (arithmetic shift), indexed by O1 applied to those coordinates;
 *   - average pooling divides by the number of ACTIVE children, not by 8 (inactive voxels
 *     carry no value in an IndexGrid; a dense average would mix in the background);
 *   - prefix field w (bits 9w..9w+8, w = 0..6) of mPrefixSum = popcount of mask
 *     words 0..w, as the prose under Listing 1 states.
 *
 * Pins: tests/test_oracle_*.py (closed forms of Listings 1-2, dense special cases,
 * counting identities of Sec. 3.3, brute-force neighbour search, dense masked 3-D
 * correlation, K=1 per-voxel GEMM, identity-weight and all-ones exact cases; for O4 the
 * gradients a library's autograd gives for the dense masked correlation, the adjoint
 * identities against O3, and central differences of O3; for O6 exact dyadic cases, points on
 * cell faces, and containment of every point in its cell checked in exact rational arithmetic).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t b, i, j, k; } fo_vox;

typedef struct {
    int64_t  offset;     /* index of the leaf's first active voxel (0-based, batch-global) */
    uint64_t prefix;     /* 7 x 9-bit inclusive popcount prefixes of mask words 0..6       */
    uint64_t mask[8];    /* word = i&7, bit = (j&7)<<3 | (k&7)                             */
    int32_t  origin[3];  /* 8*(i>>3), 8*(j>>3), 8*(k>>3)                                   */
    int32_t  batch;
} fo_leaf;               /* 96 bytes; the first 80 are the record of Listing 1             */

typedef struct fo_grid {
    int32_t  B;
    int64_t  N;          /* total active voxels                    */
    fo_vox  *vox;        /* [N] in index order                     */
    int64_t *base;       /* [B+1] first index of each grid         */
    /* hash map (b,i,j,k) -> index */
    uint64_t cap;        /* power of two                           */
    int64_t *slot;       /* [cap] index into vox or -1             */
    /* leaf table */
    int64_t  n_leaf, n_lower, n_upper;
    fo_leaf *leaf;
} fo_grid;

/* ------------------------------------------------------------------ hash map */
static uint64_t fo_hash(int32_t b, int32_t i, int32_t j, int32_t k) {
    uint64_t h = 0x9E3779B97F4A7C15ull;
    uint32_t v[4] = { (uint32_t)b, (uint32_t)i, (uint32_t)j, (uint32_t)k };
    for (int t = 0; t < 4; ++t) {
        h ^= v[t];
        h *= 0xBF58476D1CE4E5B9ull;
        h ^= h >> 29;
    }
    return h;
}

static int64_t fo_find(const fo_grid *g, int32_t b, int32_t i, int32_t j, int32_t k) {
    if (g->cap == 0) return -1;
    uint64_t h = fo_hash(b, i, j, k) & (g->cap - 1);
    for (;;) {
        int64_t s = g->slot[h];
        if (s < 0) return -1;
        const fo_vox *v = &g->vox[s];
        if (v->b == b && v->i == i && v->j == j && v->k == k) return s;
        h = (h + 1) & (g->cap - 1);
    }
}

/* insert index s (vox[s] must be set); returns existing index if the key is present */
static int64_t fo_insert(fo_grid *g, int64_t s) {
    const fo_vox *n = &g->vox[s];
    uint64_t h = fo_hash(n->b, n->i, n->j, n->k) & (g->cap - 1);
    for (;;) {
        int64_t t = g->slot[h];
        if (t < 0) { g->slot[h] = s; return s; }
        const fo_vox *v = &g->vox[t];
        if (v->b == n->b && v->i == n->i && v->j == n->j && v->k == n->k) return t;
        h = (h + 1) & (g->cap - 1);
    }
}

/* ------------------------------------------------------------------ VDB order */
/* Lexicographic order of (batch; tile i,j,k = coord>>12, signed; upper i,j,k =
 * (coord>>7)&31; lower i,j,k = (coord>>3)&15; leaf i,j,k = coord&7): the order that
 * sorting by key a and then key b of Sec. 3.3 produces, with Listing 2's offsets. */
static int fo_cmp_vdb(const void *pa, const void *pb) {
    const fo_vox *x = (const fo_vox *)pa, *y = (const fo_vox *)pb;
    if (x->b != y->b) return x->b < y->b ? -1 : 1;
    int32_t fx[12] = { x->i >> 12, x->j >> 12, x->k >> 12,
                       (x->i >> 7) & 31, (x->j >> 7) & 31, (x->k >> 7) & 31,
                       (x->i >> 3) & 15, (x->j >> 3) & 15, (x->k >> 3) & 15,
                       x->i & 7, x->j & 7, x->k & 7 };
    int32_t fy[12] = { y->i >> 12, y->j >> 12, y->k >> 12,
                       (y->i >> 7) & 31, (y->j >> 7) & 31, (y->k >> 7) & 31,
                       (y->i >> 3) & 15, (y->j >> 3) & 15, (y->k >> 3) & 15,
                       y->i & 7, y->j & 7, y->k & 7 };
    for (int t = 0; t < 12; ++t)
        if (fx[t] != fy[t]) return fx[t] < fy[t] ? -1 : 1;
    return 0;
}

static int fo_popcount64(uint64_t w) {
    int c = 0;
    while (w) { w &= w - 1; ++c; }
    return c;
}

/* ------------------------------------------------------------------ O1 */
void fo_grid_destroy(fo_grid *g) {
    if (!g) return;
    free(g->vox); free(g->base); free(g->slot); free(g->leaf); free(g);
}

/* ijk: [n_rows,3] int32; joffsets: [B,2] int64 (start,end) rows of each grid. */
fo_grid *fo_grid_create(const int32_t *ijk, const int64_t *joffsets, int32_t B) {
    fo_grid *g = (fo_grid *)calloc(1, sizeof(fo_grid));
    if (!g) return NULL;
    g->B = B;
    int64_t n_in = 0;
    for (int32_t b = 0; b < B; ++b) n_in += joffsets[2 * b + 1] - joffsets[2 * b];
    g->base = (int64_t *)calloc((size_t)B + 1, sizeof(int64_t));
    g->vox = (fo_vox *)malloc(sizeof(fo_vox) * (size_t)(n_in > 0 ? n_in : 1));
    uint64_t cap = 16;
    while (cap < (uint64_t)n_in * 2u) cap <<= 1;
    g->cap = cap;
    g->slot = (int64_t *)malloc(sizeof(int64_t) * cap);
    for (uint64_t t = 0; t < cap; ++t) g->slot[t] = -1;

    /* distinct voxels of every grid (duplicates collapse) */
    int64_t n = 0;
    for (int32_t b = 0; b < B; ++b) {
        for (int64_t r = joffsets[2 * b]; r < joffsets[2 * b + 1]; ++r) {
            g->vox[n].b = b;
            g->vox[n].i = ijk[3 * r + 0];
            g->vox[n].j = ijk[3 * r + 1];
            g->vox[n].k = ijk[3 * r + 2];
            if (fo_insert(g, n) == n) ++n;
        }
    }
    g->N = n;
    /* rank in VDB order = linear index */
    qsort(g->vox, (size_t)n, sizeof(fo_vox), fo_cmp_vdb);
    for (uint64_t t = 0; t < cap; ++t) g->slot[t] = -1;
    for (int64_t s = 0; s < n; ++s) fo_insert(g, s);
    for (int64_t s = 0; s < n; ++s) g->base[g->vox[s].b + 1] += 1;
    for (int32_t b = 0; b < B; ++b) g->base[b + 1] += g->base[b];

    /* leaf table and node counts by grouping the ordered list */
    g->leaf = (fo_leaf *)calloc((size_t)(n > 0 ? n : 1), sizeof(fo_leaf));
    int64_t L = 0;
    for (int64_t s = 0; s < n; ++s) {
        const fo_vox *v = &g->vox[s];
        int new_leaf = 1, new_lower = 1, new_upper = 1;
        if (s > 0) {
            const fo_vox *u = &g->vox[s - 1];
            int same_b = (u->b == v->b);
            new_upper = !(same_b && (u->i >> 12) == (v->i >> 12) && (u->j >> 12) == (v->j >> 12) &&
                          (u->k >> 12) == (v->k >> 12));
            new_lower = !(same_b && (u->i >> 7) == (v->i >> 7) && (u->j >> 7) == (v->j >> 7) &&
                          (u->k >> 7) == (v->k >> 7));
            new_leaf = !(same_b && (u->i >> 3) == (v->i >> 3) && (u->j >> 3) == (v->j >> 3) &&
                         (u->k >> 3) == (v->k >> 3));
        }
        g->n_upper += new_upper;
        g->n_lower += new_lower;
        if (new_leaf) {
            fo_leaf *lf = &g->leaf[L++];
            lf->offset = s;
            lf->origin[0] = (v->i >> 3) * 8;
            lf->origin[1] = (v->j >> 3) * 8;
            lf->origin[2] = (v->k >> 3) * 8;
            lf->batch = v->b;
        }
        g->leaf[L - 1].mask[v->i & 7] |= 1ull << (((v->j & 7) << 3) | (v->k & 7));
    }
    g->n_leaf = L;
    for (int64_t l = 0; l < L; ++l) {
        uint64_t acc = 0, pre = 0;
        for (int w = 0; w < 7; ++w) {
            acc += (uint64_t)fo_popcount64(g->leaf[l].mask[w]);
            pre |= acc << (9 * w);
        }
        g->leaf[l].prefix = pre;
    }
    return g;
}

int64_t fo_grid_num_voxels(const fo_grid *g) { return g->N; }
int32_t fo_grid_batch_size(const fo_grid *g) { return g->B; }
int64_t fo_grid_num_leaves(const fo_grid *g) { return g->n_leaf; }

void fo_grid_counts(const fo_grid *g, int64_t counts[3]) {
    counts[0] = g->n_leaf; counts[1] = g->n_lower; counts[2] = g->n_upper;
}

void fo_grid_voxel_joffsets(const fo_grid *g, int64_t *out /* [B,2] */) {
    for (int32_t b = 0; b < g->B; ++b) { out[2 * b] = g->base[b]; out[2 * b + 1] = g->base[b + 1]; }
}

void fo_grid_ijk(const fo_grid *g, int32_t *out /* [N,3] */, int32_t *jidx /* [N] or NULL */) {
    for (int64_t s = 0; s < g->N; ++s) {
        out[3 * s + 0] = g->vox[s].i; out[3 * s + 1] = g->vox[s].j; out[3 * s + 2] = g->vox[s].k;
        if (jidx) jidx[s] = g->vox[s].b;
    }
}

void fo_grid_leaf_table(const fo_grid *g, fo_leaf *out /* [n_leaf] */) {
    memcpy(out, g->leaf, sizeof(fo_leaf) * (size_t)g->n_leaf);
}

/* index of (jidx[r]; ijk[r]) or -1; jidx NULL means grid 0 */
void fo_grid_lookup(const fo_grid *g, const int32_t *ijk, const int32_t *jidx, int64_t n,
                    int64_t *out) {
    for (int64_t r = 0; r < n; ++r)
        out[r] = fo_find(g, jidx ? jidx[r] : 0, ijk[3 * r], ijk[3 * r + 1], ijk[3 * r + 2]);
}

/* output grid of a stride-2 operator: distinct floor(ijk/2) per grid */
fo_grid *fo_grid_coarsen2(const fo_grid *g) {
    int32_t *c = (int32_t *)malloc(sizeof(int32_t) * 3 * (size_t)(g->N > 0 ? g->N : 1));
    int64_t *jo = (int64_t *)malloc(sizeof(int64_t) * 2 * (size_t)(g->B > 0 ? g->B : 1));
    for (int64_t s = 0; s < g->N; ++s) {
        c[3 * s + 0] = g->vox[s].i >> 1; c[3 * s + 1] = g->vox[s].j >> 1; c[3 * s + 2] = g->vox[s].k >> 1;
    }
    for (int32_t b = 0; b < g->B; ++b) { jo[2 * b] = g->base[b]; jo[2 * b + 1] = g->base[b + 1]; }
    fo_grid *o = fo_grid_create(c, jo, g->B);
    free(c); free(jo);
    return o;
}

/* ------------------------------------------------------------------ O2 */
static int fo_delta_min(int K) { return (K & 1) ? -(K - 1) / 2 : 0; }

/* nbmap: [N_out, K^3] int64.  Returns the number of active pairs, or -1 on bad args. */
int64_t fo_kernel_map(const fo_grid *gin, const fo_grid *gout, int K, int stride, int64_t *nbmap) {
    if (K < 1 || stride < 1 || gin->B != gout->B) return -1;
    const int d0 = fo_delta_min(K);
    const int K3 = K * K * K;
    int64_t pairs = 0;
    for (int64_t o = 0; o < gout->N; ++o) {
        const fo_vox *p = &gout->vox[o];
        for (int a = 0; a < K; ++a)
            for (int b = 0; b < K; ++b)
                for (int c = 0; c < K; ++c) {
                    int kappa = (a * K + b) * K + c;
                    int64_t in = fo_find(gin, p->b, stride * p->i + d0 + a, stride * p->j + d0 + b,
                                         stride * p->k + d0 + c);
                    nbmap[o * K3 + kappa] = in;
                    pairs += (in >= 0);
                }
    }
    return pairs;
}

/* ------------------------------------------------------------------ O3 */
/* feat [N_in, C_in], w [K^3, C_in, C_out], out [N_out, C_out] (rows o_begin..o_end-1
 * are written, the rest untouched); all double.  Returns active pairs in the range. */
int64_t fo_conv(const fo_grid *gin, const fo_grid *gout, int K, int stride,
                const double *feat, const double *w, int C_in, int C_out,
                double *out, int64_t o_begin, int64_t o_end) {
    if (K < 1 || stride < 1 || gin->B != gout->B) return -1;
    const int d0 = fo_delta_min(K);
    int64_t pairs = 0;
    if (o_begin < 0) o_begin = 0;
    if (o_end > gout->N) o_end = gout->N;
    for (int64_t o = o_begin; o < o_end; ++o) {
        const fo_vox *p = &gout->vox[o];
        double *y = out + o * (int64_t)C_out;
        for (int co = 0; co < C_out; ++co) y[co] = 0.0;
        for (int a = 0; a < K; ++a)
            for (int b = 0; b < K; ++b)
                for (int c = 0; c < K; ++c) {
                    int64_t in = fo_find(gin, p->b, stride * p->i + d0 + a, stride * p->j + d0 + b,
                                         stride * p->k + d0 + c);
                    if (in < 0) continue;
                    ++pairs;
                    const double *x = feat + in * (int64_t)C_in;
                    const double *wk = w + (int64_t)((a * K + b) * K + c) * C_in * C_out;
                    for (int ci = 0; ci < C_in; ++ci) {
                        const double xv = x[ci];
                        const double *wr = wk + (int64_t)ci * C_out;
                        for (int co = 0; co < C_out; ++co) y[co] += xv * wr[co];
                    }
                }
    }
    return pairs;
}

/* ------------------------------------------------------------------ O4 */
/* gout [N_out, C_out], w [K^3, C_in, C_out], gin [N_in, C_in] (overwritten); all double.
 * Only the outputs in [o_begin, o_end) contribute (the whole gradient is the sum over disjoint
 * ranges).  Returns the active pairs, or -1 on bad args. */
int64_t fo_conv_bwd_data(const fo_grid *gin_grid, const fo_grid *gout_grid, int K, int stride,
                         const double *gout, const double *w, int C_in, int C_out, double *gin,
                         int64_t o_begin, int64_t o_end) {
    if (K < 1 || stride < 1 || gin_grid->B != gout_grid->B) return -1;
    const int d0 = fo_delta_min(K);
    int64_t pairs = 0;
    for (int64_t e = 0; e < gin_grid->N * (int64_t)C_in; ++e) gin[e] = 0.0;
    if (o_begin < 0) o_begin = 0;
    if (o_end > gout_grid->N) o_end = gout_grid->N;
    for (int64_t o = o_begin; o < o_end; ++o) {
        const fo_vox *p = &gout_grid->vox[o];
        const double *gy = gout + o * (int64_t)C_out;
        for (int a = 0; a < K; ++a)
            for (int b = 0; b < K; ++b)
                for (int c = 0; c < K; ++c) {
                    int64_t in = fo_find(gin_grid, p->b, stride * p->i + d0 + a, stride * p->j + d0 + b,
                                         stride * p->k + d0 + c);
                    if (in < 0) continue;
                    ++pairs;
                    double *gx = gin + in * (int64_t)C_in;
                    const double *wk = w + (int64_t)((a * K + b) * K + c) * C_in * C_out;
                    for (int ci = 0; ci < C_in; ++ci) {
                        const double *wr = wk + (int64_t)ci * C_out;
                        double s = 0.0;
                        for (int co = 0; co < C_out; ++co) s += wr[co] * gy[co];
                        gx[ci] += s;
                    }
                }
    }
    return pairs;
}

/* feat [N_in, C_in], gout [N_out, C_out], gw [K^3, C_in, C_out] (overwritten); all double.
 * Only outputs o_begin..o_end-1 contribute.  Returns their active pairs, or -1 on bad args. */
int64_t fo_conv_bwd_weight(const fo_grid *gin_grid, const fo_grid *gout_grid, int K, int stride,
                           const double *feat, const double *gout, int C_in, int C_out, double *gw,
                           int64_t o_begin, int64_t o_end) {
    if (K < 1 || stride < 1 || gin_grid->B != gout_grid->B) return -1;
    const int d0 = fo_delta_min(K);
    int64_t pairs = 0;
    for (int64_t e = 0; e < (int64_t)K * K * K * C_in * C_out; ++e) gw[e] = 0.0;
    if (o_begin < 0) o_begin = 0;
    if (o_end > gout_grid->N) o_end = gout_grid->N;
    for (int64_t o = o_begin; o < o_end; ++o) {
        const fo_vox *p = &gout_grid->vox[o];
        const double *gy = gout + o * (int64_t)C_out;
        for (int a = 0; a < K; ++a)
            for (int b = 0; b < K; ++b)
                for (int c = 0; c < K; ++c) {
                    int64_t in = fo_find(gin_grid, p->b, stride * p->i + d0 + a, stride * p->j + d0 + b,
                                         stride * p->k + d0 + c);
                    if (in < 0) continue;
                    ++pairs;
                    const double *x = feat + in * (int64_t)C_in;
                    double *gk = gw + (int64_t)((a * K + b) * K + c) * C_in * C_out;
                    for (int ci = 0; ci < C_in; ++ci) {
                        const double xv = x[ci];
                        double *gr = gk + (int64_t)ci * C_out;
                        for (int co = 0; co < C_out; ++co) gr[co] += xv * gy[co];
                    }
                }
    }
    return pairs;
}

/* ------------------------------------------------------------------ O5 */
/* z [N_out, C_in] on the outputs of the map (gin_grid, gout_grid, K, stride), w [K^3, C_in, C_out],
 * out [N_in, C_out] (overwritten); all double.  Returns the active pairs, or -1 on bad args. */
int64_t fo_conv_transpose(const fo_grid *gin_grid, const fo_grid *gout_grid, int K, int stride,
                          const double *z, const double *w, int C_in, int C_out, double *out) {
    if (K < 1 || stride < 1 || gin_grid->B != gout_grid->B) return -1;
    const int d0 = fo_delta_min(K);
    int64_t pairs = 0;
    for (int64_t e = 0; e < gin_grid->N * (int64_t)C_out; ++e) out[e] = 0.0;
    for (int64_t o = 0; o < gout_grid->N; ++o) {
        const fo_vox *p = &gout_grid->vox[o];
        const double *x = z + o * (int64_t)C_in;
        for (int a = 0; a < K; ++a)
            for (int b = 0; b < K; ++b)
                for (int c = 0; c < K; ++c) {
                    int64_t in = fo_find(gin_grid, p->b, stride * p->i + d0 + a, stride * p->j + d0 + b,
                                         stride * p->k + d0 + c);
                    if (in < 0) continue;
                    ++pairs;
                    double *y = out + in * (int64_t)C_out;
                    const double *wk = w + (int64_t)((a * K + b) * K + c) * C_in * C_out;
                    for (int ci = 0; ci < C_in; ++ci) {
                        const double xv = x[ci];
                        const double *wr = wk + (int64_t)ci * C_out;
                        for (int co = 0; co < C_out; ++co) y[co] += xv * wr[co];
                    }
                }
    }
    return pairs;
}

/* z [N_fine, C] -> out [N_coarse, C] (overwritten); mode 0 = max, 1 = mean over the active children.
 * Returns the number of (coarse voxel, child) pairs, or -1 on bad args. */
int64_t fo_pool2(const fo_grid *fine, const fo_grid *coarse, int mode, const double *z, int C, double *out) {
    if (fine->B != coarse->B || (mode != 0 && mode != 1)) return -1;
    int64_t pairs = 0;
    for (int64_t o = 0; o < coarse->N; ++o) {
        const fo_vox *p = &coarse->vox[o];
        double *y = out + o * (int64_t)C;
        int n = 0;
        for (int a = 0; a < 2; ++a)
            for (int b = 0; b < 2; ++b)
                for (int c = 0; c < 2; ++c) {
                    int64_t in = fo_find(fine, p->b, 2 * p->i + a, 2 * p->j + b, 2 * p->k + c);
                    if (in < 0) continue;
                    const double *x = z + in * (int64_t)C;
                    for (int ch = 0; ch < C; ++ch) {
                        if (n == 0) y[ch] = x[ch];
                        else if (mode == 0) y[ch] = x[ch] > y[ch] ? x[ch] : y[ch];
                        else y[ch] += x[ch];
                    }
                    ++n;
                }
        if (n == 0) for (int ch = 0; ch < C; ++ch) y[ch] = 0.0;
        if (mode == 1 && n > 1) for (int ch = 0; ch < C; ++ch) y[ch] /= (double)n;
        pairs += n;
    }
    return pairs;
}

/* z [N_coarse, C] -> out [N_fine, C] (overwritten): every fine voxel takes its parent's row. */
int64_t fo_upsample2(const fo_grid *fine, const fo_grid *coarse, const double *z, int C, double *out) {
    if (fine->B != coarse->B) return -1;
    int64_t found = 0;
    for (int64_t i = 0; i < fine->N; ++i) {
        const fo_vox *p = &fine->vox[i];
        int64_t o = fo_find(coarse, p->b, p->i >> 1, p->j >> 1, p->k >> 1);
        double *y = out + i * (int64_t)C;
        for (int ch = 0; ch < C; ++ch) y[ch] = o >= 0 ? z[o * (int64_t)C + ch] : 0.0;
        found += o >= 0;
    }
    return found;
}

/* the grid of all 8 children of every voxel */
fo_grid *fo_grid_subdivide2(const fo_grid *g) {
    int32_t *c = (int32_t *)malloc(sizeof(int32_t) * 3 * 8 * (size_t)(g->N > 0 ? g->N : 1));
    int64_t *jo = (int64_t *)malloc(sizeof(int64_t) * 2 * (size_t)(g->B > 0 ? g->B : 1));
    for (int64_t s = 0; s < g->N; ++s)
        for (int d = 0; d < 8; ++d) {
            int32_t *q = c + 3 * (8 * s + d);
            q[0] = 2 * g->vox[s].i + ((d >> 2) & 1); q[1] = 2 * g->vox[s].j + ((d >> 1) & 1); q[2] = 2 * g->vox[s].k + (d & 1);
        }
    for (int32_t b = 0; b < g->B; ++b) { jo[2 * b] = 8 * g->base[b]; jo[2 * b + 1] = 8 * g->base[b + 1]; }
    fo_grid *o = fo_grid_create(c, jo, g->B);
    free(c); free(jo);
    return o;
}

/* O7: the grid of all voxels within Chebyshev distance r of an active voxel; NULL if r < 0 */
fo_grid *fo_grid_pad(const fo_grid *g, int r) {
    if (r < 0) return NULL;
    const int64_t w = 2 * (int64_t)r + 1, w3 = w * w * w;
    int32_t *c = (int32_t *)malloc(sizeof(int32_t) * 3 * (size_t)(g->N > 0 ? g->N * w3 : 1));
    int64_t *jo = (int64_t *)malloc(sizeof(int64_t) * 2 * (size_t)(g->B > 0 ? g->B : 1));
    int64_t n = 0;
    for (int64_t s = 0; s < g->N; ++s)
        for (int a = -r; a <= r; ++a)
            for (int b = -r; b <= r; ++b)
                for (int d = -r; d <= r; ++d) {
                    c[3 * n] = g->vox[s].i + a; c[3 * n + 1] = g->vox[s].j + b; c[3 * n + 2] = g->vox[s].k + d;
                    ++n;
                }
    for (int32_t b = 0; b < g->B; ++b) { jo[2 * b] = w3 * g->base[b]; jo[2 * b + 1] = w3 * g->base[b + 1]; }
    fo_grid *o = fo_grid_create(c, jo, g->B);
    free(c); free(jo);
    return o;
}

/* O6: xyz [n,3] float -> ijk [n,3] int32 (rows of invalid points are set to 0,0,0); returns the
 * number of invalid points. */
int64_t fo_points_to_ijk(const float *xyz, int64_t n, const float origin[3], const float voxel_size[3],
                         int32_t *ijk) {
    int64_t invalid = 0;
    for (int64_t p = 0; p < n; ++p) {
        int ok = 1;
        int32_t c[3];
        for (int a = 0; a < 3; ++a) {
            volatile float d = xyz[3 * p + a] - origin[a];   /* volatile: each step rounded to float */
            volatile float t = d / voxel_size[a];
            float fl = floorf(t);
            if (!isfinite(fl) || fl < -1073741824.0f || fl >= 1073741824.0f) { ok = 0; c[a] = 0; }
            else c[a] = (int32_t)fl;
        }
        if (!ok) { c[0] = c[1] = c[2] = 0; ++invalid; }
        ijk[3 * p] = c[0]; ijk[3 * p + 1] = c[1]; ijk[3 * p + 2] = c[2];
    }
    return invalid;
}

/* O5, gradients.  mode 0 max (needs the forward input z), 1 mean.  gout [N_coarse, C] -> gin [N_fine, C]
 * (overwritten; every fine voxel has exactly one parent in the coarse grid of a factor-2 pooling). */
int64_t fo_pool2_bwd(const fo_grid *fine, const fo_grid *coarse, int mode, const double *z, const double *gout, int C,
                     double *gin) {
    if (fine->B != coarse->B || (mode != 0 && mode != 1) || (mode == 0 && !z)) return -1;
    for (int64_t e = 0; e < fine->N * (int64_t)C; ++e) gin[e] = 0.0;
    int64_t pairs = 0;
    for (int64_t o = 0; o < coarse->N; ++o) {
        const fo_vox *p = &coarse->vox[o];
        int64_t child[8];
        int n = 0;
        for (int a = 0; a < 2; ++a)
            for (int b = 0; b < 2; ++b)
                for (int c = 0; c < 2; ++c) {
                    int64_t in = fo_find(fine, p->b, 2 * p->i + a, 2 * p->j + b, 2 * p->k + c);
                    if (in >= 0) child[n++] = in;            /* offset order */
                }
        for (int ch = 0; ch < C; ++ch) {
            const double g = gout[o * (int64_t)C + ch];
            if (mode == 1) {
                for (int q = 0; q < n; ++q) gin[child[q] * (int64_t)C + ch] = g / (double)n;
            } else if (n > 0) {
                int best = 0;
                for (int q = 1; q < n; ++q)
                    if (z[child[q] * (int64_t)C + ch] > z[child[best] * (int64_t)C + ch]) best = q;
                gin[child[best] * (int64_t)C + ch] = g;
            }
        }
        pairs += n;
    }
    return pairs;
}

/* gout [N_fine, C] -> gin [N_coarse, C] (overwritten): the sum over the active children. */
int64_t fo_upsample2_bwd(const fo_grid *fine, const fo_grid *coarse, const double *gout, int C, double *gin) {
    if (fine->B != coarse->B) return -1;
    int64_t pairs = 0;
    for (int64_t o = 0; o < coarse->N; ++o) {
        const fo_vox *p = &coarse->vox[o];
        double *y = gin + o * (int64_t)C;
        for (int ch = 0; ch < C; ++ch) y[ch] = 0.0;
        for (int a = 0; a < 2; ++a)
            for (int b = 0; b < 2; ++b)
                for (int c = 0; c < 2; ++c) {
                    int64_t in = fo_find(fine, p->b, 2 * p->i + a, 2 * p->j + b, 2 * p->k + c);
                    if (in < 0) continue;
                    for (int ch = 0; ch < C; ++ch) y[ch] += gout[in * (int64_t)C + ch];
                    ++pairs;
                }
    }
    return pairs;
}
