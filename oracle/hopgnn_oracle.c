/*
 * CPU oracle for the micrograph hot path of HopGNN (arxiv 2409.00657).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP sources; nothing in the product path
 * may call it.  Everything here runs on host arrays.
 *
 * The paper defines the steps only at the level of "sample a k-hop
 * computation graph per root vertex (a micrograph), merge the vertex sets of
 * the micrographs a worker will train and drop duplicates (pre-gathering),
 * collect the feature vector of every vertex, then aggregate neighbour
 * features and apply a neural transform per layer" (paper sections 2, 4 and
 * 5.2).  It names no hash, no ordering and no layer formula; the concrete
 * readings taken here are:
 *
 *   - sampling is with replacement, child = row[hash64(key,root,v,h,j) mod deg]
 *     where the hash is a three-round chain of the SplitMix64 output finaliser;
 *   - a micrograph is a fixed-shape tree of slots stored level-major;
 *   - the pre-gather set is the ascending, duplicate-free list of valid IDs;
 *   - the layer is GraphSAGE-mean:  act(x_self W_self + mean(nbrs) W_neigh + b);
 *     the GCN-style and attention layers the evaluation also trains are defined at
 *     orc_gcn_fwd and orc_gat_fwd.
 *
 * All floating point is done in double; the caller decides how a result is
 * rounded for storage (orc_round_store does one round-to-nearest-even step).
 *
 * Pin status: every function below is pinned by tests that do not call back
 * into it (published SplitMix64 outputs, closed-form graphs, brute-force
 * enumeration, algebraic special cases, the paper's worked pre-gather example).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2, ORC_F64 = 3 };

/* ------------------------------------------------------------------ hash -- */

/* SplitMix64 output finaliser (Steele, Lea, Flood, OOPSLA 2014). */
uint64_t orc_mix(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

#define ORC_GOLDEN 0x9E3779B97F4A7C15ULL

/* hash64(key, root, v, h, j): absorb the key, then (root,v), then (h,j);
 * each absorption is "xor the word in, add the golden-ratio increment, mix". */
uint64_t orc_hash64(uint64_t key, uint32_t root, uint32_t v, uint32_t h, uint32_t j)
{
    uint64_t w0 = ((uint64_t)root << 32) | (uint64_t)v;
    uint64_t w1 = ((uint64_t)h << 32) | (uint64_t)j;
    uint64_t x = orc_mix(key + ORC_GOLDEN);
    x = orc_mix((x ^ w0) + ORC_GOLDEN);
    x = orc_mix((x ^ w1) + ORC_GOLDEN);
    return x;
}

/* -------------------------------------------------------------- sampling -- */

/* T_seed = sum_{h=0..L} P_h with P_0 = 1, P_h = f_1 ... f_h.  -1 on bad input. */
int64_t orc_slots_per_seed(const int32_t *fanouts, int32_t n_layers)
{
    if (!fanouts || n_layers < 1) return -1;
    int64_t p = 1, t = 1;
    for (int32_t h = 0; h < n_layers; ++h) {
        if (fanouts[h] < 1) return -1;
        p *= fanouts[h];
        t += p;
    }
    return t;
}

static int64_t off_at(const void *offsets, int off64, int64_t v)
{
    return off64 ? ((const int64_t *)offsets)[v] : (int64_t)((const int32_t *)offsets)[v];
}

/*
 * Micrograph sampling (paper section 2 "sampling", section 4 "micrograph
 * definition": one k-hop computation graph per root vertex of the batch).
 *
 * ids is level-major.  Level h (0..L) holds B*P_h slots starting at
 * S_{h-1} = B * sum_{i<h} P_i; inside a level the slot of micrograph m and
 * path p is m*P_h + p.  The children of the slot with level-local index q
 * at level h-1 are the f_h slots q*f_h .. q*f_h+f_h-1 of level h.
 * A slot holding v<0 or a vertex of degree 0 has only invalid (-1) children.
 *
 * indptr (optional) has one entry per non-leaf slot plus one: the position,
 * counted from the first level-1 slot, where that slot's children start.
 */
int orc_sample(const void *offsets, int offsets_i64, const int32_t *indices,
               int64_t n_vertices, const int32_t *seeds, int32_t n_seeds,
               const int32_t *fanouts, int32_t n_layers, uint64_t key,
               int32_t *ids, int32_t *indptr)
{
    if (orc_slots_per_seed(fanouts, n_layers) < 0 || n_seeds < 0) return 1;
    const int64_t B = n_seeds;
    for (int64_t m = 0; m < B; ++m) {
        if (seeds[m] < 0 || seeds[m] >= n_vertices) return 3;
        ids[m] = seeds[m];
    }
    int64_t prev_base = 0;      /* S_{h-2}: first slot of level h-1 */
    int64_t prev_P = 1;         /* P_{h-1} */
    int64_t cur_base = B;       /* S_{h-1}: first slot of level h   */
    for (int32_t h = 1; h <= n_layers; ++h) {
        const int64_t f = fanouts[h - 1];
        for (int64_t q = 0; q < B * prev_P; ++q) {
            const int64_t m = q / prev_P;
            const int32_t v = ids[prev_base + q];
            const int64_t child0 = cur_base + q * f;
            if (indptr) indptr[prev_base + q] = (int32_t)(child0 - B);
            int64_t o0 = 0, deg = 0;
            if (v >= 0) {
                o0 = off_at(offsets, offsets_i64, v);
                deg = off_at(offsets, offsets_i64, (int64_t)v + 1) - o0;
            }
            for (int64_t j = 0; j < f; ++j) {
                if (v < 0 || deg <= 0) {
                    ids[child0 + j] = -1;
                } else {
                    uint64_t x = orc_hash64(key, (uint32_t)seeds[m], (uint32_t)v,
                                            (uint32_t)h, (uint32_t)j);
                    ids[child0 + j] = indices[o0 + (int64_t)(x % (uint64_t)deg)];
                }
            }
        }
        prev_base = cur_base;
        cur_base += B * prev_P * f;
        prev_P *= f;
    }
    /* prev_base is now S_{L-1} (first leaf slot), cur_base is T */
    if (indptr) indptr[prev_base] = (int32_t)(cur_base - B);
    return 0;
}

/* ------------------------------------------------------------ pre-gather -- */

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Pre-gathering (paper section 5.2: fetch the features needed by all the
 * micrographs of one iteration in a single batch, each vertex once; the
 * implementation section says duplicates are detected and removed from the
 * stored list of micrographs).
 *
 * uniq  = ascending duplicate-free list of the non-negative entries of ids
 * remap = for every slot the position of its id in uniq, -1 for invalid slots
 * returns U = |uniq|, or -1 on allocation failure.
 */
int64_t orc_pregather(const int32_t *ids, int64_t n_ids, int32_t *uniq, int32_t *remap)
{
    int32_t *tmp = (int32_t *)malloc((size_t)(n_ids > 0 ? n_ids : 1) * sizeof(int32_t));
    if (!tmp) return -1;
    int64_t n = 0;
    for (int64_t i = 0; i < n_ids; ++i)
        if (ids[i] >= 0) tmp[n++] = ids[i];
    qsort(tmp, (size_t)n, sizeof(int32_t), cmp_i32);
    int64_t U = 0;
    for (int64_t i = 0; i < n; ++i)
        if (i == 0 || tmp[i] != tmp[i - 1]) uniq[U++] = tmp[i];
    free(tmp);
    for (int64_t i = 0; i < n_ids; ++i) {
        if (ids[i] < 0) { remap[i] = -1; continue; }
        int64_t lo = 0, hi = U - 1;
        while (lo < hi) {
            int64_t mid = lo + (hi - lo) / 2;
            if (uniq[mid] < ids[i]) lo = mid + 1; else hi = mid;
        }
        remap[i] = (int32_t)lo;
    }
    return U;
}

/* -------------------------------------------------------------- locality -- */

/*
 * Data locality of micrographs (paper section 4, "data locality in micrographs"
 * and the text under the locality table): for each micrograph, N_total = number
 * of distinct vertices in it, N_colocated = number of distinct NON-ROOT vertices
 * whose home server equals the root's home server; R_micro = N_colocated/N_total.
 * (The worked example of the same section counts the root as local too - 3 of 4
 * for micrograph 6 - which is N_colocated + 1 over N_total.)
 * owner[v] = home server of vertex v.  A micrograph whose root is its only vertex
 * has N_total = 1, N_colocated = 0.
 */
int orc_micrograph_locality(const int32_t *ids, int32_t n_seeds, const int32_t *fanouts,
                            int32_t n_layers, const int32_t *owner, int32_t *n_total,
                            int32_t *n_coloc)
{
    const int64_t t_seed = orc_slots_per_seed(fanouts, n_layers);
    if (t_seed < 0 || n_seeds < 0) return 1;
    int32_t *tmp = (int32_t *)malloc((size_t)t_seed * sizeof(int32_t));
    if (!tmp) return 2;
    for (int64_t m = 0; m < n_seeds; ++m) {
        int64_t n = 0, base = 0, P = 1;
        for (int32_t h = 0; h <= n_layers; ++h) {
            for (int64_t p = 0; p < P; ++p) {
                int32_t v = ids[base + m * P + p];
                if (v >= 0) tmp[n++] = v;
            }
            base += (int64_t)n_seeds * P;
            if (h < n_layers) P *= fanouts[h];
        }
        const int32_t root = ids[m];
        qsort(tmp, (size_t)n, sizeof(int32_t), cmp_i32);
        int32_t tot = 0, col = 0;
        for (int64_t i = 0; i < n; ++i) {
            if (i > 0 && tmp[i] == tmp[i - 1]) continue;
            ++tot;
            if (tmp[i] != root && owner[tmp[i]] == owner[root]) ++col;
        }
        n_total[m] = tot;
        n_coloc[m] = col;
    }
    free(tmp);
    return 0;
}

/*
 * Owner split of a pre-gathered ID set (paper section 5.2: only the vertices that
 * are NOT stored on the worker's own server are fetched; section 7.3 reports the
 * miss rate of feature gathering = non-local requests / all requests).
 * remote = the entries of uniq whose owner differs from `server`, in order;
 * returns their number.  miss rate = return value / n_uniq.
 */
int64_t orc_split_by_owner(const int32_t *uniq, int64_t n_uniq, const int32_t *owner, int32_t server,
                           int32_t *remote)
{
    int64_t n = 0;
    for (int64_t i = 0; i < n_uniq; ++i)
        if (owner[uniq[i]] != server) remote[n++] = uniq[i];
    return n;
}

/* ---------------------------------------------------------------- gather -- */

/* Gathering (paper section 2): Xu[i,:] = X[uniq[i],:], a copy of row bytes.
 * ld_bytes is the distance between rows of X; Xu is packed. */
int orc_gather(const void *X, int64_t n_rows, int64_t row_bytes, int64_t ld_bytes,
               const int32_t *uniq, int64_t n_uniq, void *Xu)
{
    for (int64_t i = 0; i < n_uniq; ++i) {
        if (uniq[i] < 0 || uniq[i] >= n_rows) return 3;
        memcpy((char *)Xu + i * row_bytes, (const char *)X + (int64_t)uniq[i] * ld_bytes,
               (size_t)row_bytes);
    }
    return 0;
}

/* -------------------------------------------------- storage conversions -- */

static double half_to_double(uint16_t hbits)
{
    int sign = hbits >> 15, e = (hbits >> 10) & 31, m = hbits & 1023;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double load_elem(const void *p, int dtype, int64_t i)
{
    switch (dtype) {
    case ORC_F32: return (double)((const float *)p)[i];
    case ORC_BF16: return bf16_to_double(((const uint16_t *)p)[i]);
    case ORC_F16: return half_to_double(((const uint16_t *)p)[i]);
    default: return ((const double *)p)[i];
    }
}

/* One round-to-nearest-even step from double to a binary format with
 * `sig` significand bits (hidden bit included), smallest quantum 2^qmin and
 * largest finite value maxv; the result is returned as a double that is
 * exactly representable in the target format (or +-inf on overflow). */
static double round_to_format(double x, int sig, int qmin, double maxv)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);              /* |x| = m * 2^e, m in [0.5, 1) */
    int q = e - sig;                 /* quantum of a normal number    */
    if (q < qmin) q = qmin;
    double r = ldexp(rint(ldexp(x, -q)), q);   /* rint: ties to even */
    if (fabs(r) > maxv) r = x > 0 ? INFINITY : -INFINITY;
    return r;
}

/* Round n doubles once to `dtype` and store them (fp32 / bf16 / fp16 / fp64). */
void orc_round_store(const double *src, int64_t n, int dtype, void *dst)
{
    for (int64_t i = 0; i < n; ++i) {
        double x = src[i];
        if (dtype == ORC_F64) {
            ((double *)dst)[i] = x;
        } else if (dtype == ORC_F32) {
            ((float *)dst)[i] = (float)x;      /* IEEE default rounding: nearest even */
        } else if (dtype == ORC_BF16) {
            /* 8 significand bits, float exponent range: min quantum 2^-133 */
            double r = round_to_format(x, 8, -133, ldexp(255.0, 120));
            float f = (float)r;                /* exact */
            uint32_t u;
            memcpy(&u, &f, 4);
            ((uint16_t *)dst)[i] = (uint16_t)(u >> 16);
        } else {
            /* fp16: 11 significand bits, min quantum 2^-24, max 65504 */
            double r = round_to_format(x, 11, -24, 65504.0);
            uint16_t s = (uint16_t)(signbit(r) ? 0x8000 : 0), out;
            double a = fabs(r);
            if (isnan(r)) out = 0x7E00;
            else if (isinf(r)) out = (uint16_t)(s | 0x7C00);
            else if (a == 0.0) out = s;
            else if (a < ldexp(1.0, -14)) out = (uint16_t)(s | (uint16_t)ldexp(a, 24));
            else {
                int e;
                double m = frexp(a, &e);       /* a = m 2^e, m in [0.5,1) */
                out = (uint16_t)(s | ((e + 14) << 10) | ((uint16_t)ldexp(m, 11) - 1024));
            }
            ((uint16_t *)dst)[i] = out;
        }
    }
}

/* Convert n stored elements of `dtype` to double (exact). */
void orc_load_f64(const void *src, int64_t n, int dtype, double *dst)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = load_elem(src, dtype, i);
}

/* -------------------------------------------------------- GraphSAGE-mean -- */

/*
 * One layer: for destination row r
 *   c   = number of e in [indptr[r], indptr[r+1]) with idx[e] >= 0
 *   m   = (sum of Hsrc[idx[e], :] over those e, in order) / c, or 0 if c == 0
 *   out = x_self W_self + m W_neigh + b,  x_self = Hsrc[self_idx[r]] (identity
 *         if self_idx is NULL; a negative self index gives a zero row)
 *   out = max(out, 0) if relu
 * (paper section 2 "computation": aggregate the neighbouring features, then a
 * neural-network transform; mean aggregator of GraphSAGE).
 *
 * Hsrc and the weights are stored in `dtype`; everything is converted to
 * double first; out is double [n_dst x d_out], unrounded.
 */
int orc_sage_fwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in,
                 const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                 int64_t n_dst, const void *W_self, const void *W_neigh,
                 const void *bias, int32_t d_out, int32_t relu, double *out)
{
    double *xs = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *mn = (double *)malloc(sizeof(double) * (size_t)d_in);
    if (!xs || !mn) { free(xs); free(mn); return 2; }
    int rc = 0;
    for (int64_t r = 0; r < n_dst && !rc; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        if (s >= n_src) { rc = 3; break; }
        for (int32_t k = 0; k < d_in; ++k)
            xs[k] = s < 0 ? 0.0 : load_elem(Hsrc, dtype, s * d_in + k);
        for (int32_t k = 0; k < d_in; ++k) mn[k] = 0.0;
        int64_t c = 0;
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e) {
            int64_t u = idx[e];
            if (u < 0) continue;
            if (u >= n_src) { rc = 3; break; }
            for (int32_t k = 0; k < d_in; ++k) mn[k] += load_elem(Hsrc, dtype, u * d_in + k);
            ++c;
        }
        if (rc) break;
        if (c > 0)
            for (int32_t k = 0; k < d_in; ++k) mn[k] /= (double)c;
        for (int32_t n = 0; n < d_out; ++n) {
            double acc = bias ? load_elem(bias, dtype, n) : 0.0;
            for (int32_t k = 0; k < d_in; ++k)
                acc += xs[k] * load_elem(W_self, dtype, (int64_t)k * d_out + n);
            for (int32_t k = 0; k < d_in; ++k)
                acc += mn[k] * load_elem(W_neigh, dtype, (int64_t)k * d_out + n);
            if (relu && acc < 0.0) acc = 0.0;
            out[r * d_out + n] = acc;
        }
    }
    free(xs);
    free(mn);
    return rc;
}

/*
 * The GraphSAGE layer with another neighbour aggregator (the paper's discussion of generality
 * names sum and max next to the mean):
 *   agg 0  mean of the valid neighbour rows            (orc_sage_fwd)
 *   agg 1  their sum
 *   agg 2  their element-wise maximum
 * an empty segment aggregates to 0 in every case;  out = act(x_self W_self + a W_neigh + b).
 */
int orc_sage_agg_fwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in,
                     const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                     int64_t n_dst, const void *W_self, const void *W_neigh,
                     const void *bias, int32_t d_out, int32_t agg, int32_t relu, double *out)
{
    if (agg < 0 || agg > 2) return 1;
    double *xs = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *a = (double *)malloc(sizeof(double) * (size_t)d_in);
    if (!xs || !a) { free(xs); free(a); return 2; }
    int rc = 0;
    for (int64_t r = 0; r < n_dst && !rc; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        if (s >= n_src) { rc = 3; break; }
        for (int32_t k = 0; k < d_in; ++k) {
            xs[k] = s < 0 ? 0.0 : load_elem(Hsrc, dtype, s * d_in + k);
            a[k] = 0.0;
        }
        int64_t c = 0;
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e) {
            int64_t u = idx[e];
            if (u < 0) continue;
            if (u >= n_src) { rc = 3; break; }
            for (int32_t k = 0; k < d_in; ++k) {
                double v = load_elem(Hsrc, dtype, u * d_in + k);
                if (agg == 2) a[k] = (c == 0 || v > a[k]) ? v : a[k];
                else a[k] += v;
            }
            ++c;
        }
        if (rc) break;
        if (agg == 0 && c > 0)
            for (int32_t k = 0; k < d_in; ++k) a[k] /= (double)c;
        for (int32_t n = 0; n < d_out; ++n) {
            double acc = bias ? load_elem(bias, dtype, n) : 0.0;
            for (int32_t k = 0; k < d_in; ++k)
                acc += xs[k] * load_elem(W_self, dtype, (int64_t)k * d_out + n);
            for (int32_t k = 0; k < d_in; ++k)
                acc += a[k] * load_elem(W_neigh, dtype, (int64_t)k * d_out + n);
            if (relu && acc < 0.0) acc = 0.0;
            out[r * d_out + n] = acc;
        }
    }
    free(xs);
    free(a);
    return rc;
}

/*
 * GCN-style layer (the paper's evaluation trains GCN next to GraphSAGE and GAT and
 * describes a layer only as "aggregation (like addition or averaging) over the
 * neighbouring features, then a neural transform", section 2).  Reading: one weight
 * matrix applied to the aggregate of the vertex itself and its sampled neighbours,
 *   a   = x_self + sum of Hsrc[idx[e], :] over the valid entries e     (norm 0: sum)
 *   a   = that sum / (c + [self is valid])                              (norm 1: mean)
 *   out = act(a W + b)
 * i.e. (A + I) H W and D^-1 (A + I) H W on the sampled block, parallel edges counted.
 * A negative self index contributes nothing (and is not counted); no terms -> a = 0.
 */
int orc_gcn_fwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in,
                const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                int64_t n_dst, const void *W, const void *bias, int32_t d_out,
                int32_t norm, int32_t relu, double *out)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)d_in);
    if (!a) return 2;
    int rc = 0;
    for (int64_t r = 0; r < n_dst && !rc; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        if (s >= n_src) { rc = 3; break; }
        int64_t terms = 0;
        for (int32_t k = 0; k < d_in; ++k) a[k] = 0.0;
        if (s >= 0) {
            for (int32_t k = 0; k < d_in; ++k) a[k] += load_elem(Hsrc, dtype, s * d_in + k);
            ++terms;
        }
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e) {
            int64_t u = idx[e];
            if (u < 0) continue;
            if (u >= n_src) { rc = 3; break; }
            for (int32_t k = 0; k < d_in; ++k) a[k] += load_elem(Hsrc, dtype, u * d_in + k);
            ++terms;
        }
        if (rc) break;
        if (norm && terms > 0)
            for (int32_t k = 0; k < d_in; ++k) a[k] /= (double)terms;
        for (int32_t n = 0; n < d_out; ++n) {
            double acc = bias ? load_elem(bias, dtype, n) : 0.0;
            for (int32_t k = 0; k < d_in; ++k) acc += a[k] * load_elem(W, dtype, (int64_t)k * d_out + n);
            if (relu && acc < 0.0) acc = 0.0;
            out[r * d_out + n] = acc;
        }
    }
    free(a);
    return rc;
}

/*
 * Graph-attention layer (GAT, Velickovic et al. 2018, the third model of the paper's
 * evaluation).  n_heads heads of width d_head = d_out / n_heads, outputs concatenated:
 *   z_u        = Hsrc[u] W                                   (d_out values, head-major)
 *   s_src[u,h] = <z_u[h], a_src[h]>,  s_dst[u,h] = <z_u[h], a_dst[h]>
 * For destination row r with self row s the attended entries are s itself (if s >= 0)
 * followed by the valid idx entries of its segment, parallel edges kept:
 *   e[u,h]     = LeakyReLU_0.2( s_dst[s,h] + s_src[u,h] )   (s_dst term 0 if s < 0)
 *   alpha      = softmax of e over the entries, per head
 *   out[r,h]   = act( sum alpha[u,h] z_u[h] + b[h] );  no entries -> act(b)
 */
int orc_gat_fwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in,
                const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                int64_t n_dst, const void *W, const void *a_src, const void *a_dst,
                const void *bias, int32_t d_out, int32_t n_heads, int32_t relu, double *out)
{
    if (n_heads < 1 || d_out % n_heads != 0) return 1;
    const int32_t dh = d_out / n_heads;
    double *Z = (double *)malloc(sizeof(double) * (size_t)(n_src > 0 ? n_src : 1) * (size_t)d_out);
    double *ss = (double *)malloc(sizeof(double) * (size_t)(n_src > 0 ? n_src : 1) * (size_t)n_heads);
    double *sd = (double *)malloc(sizeof(double) * (size_t)(n_src > 0 ? n_src : 1) * (size_t)n_heads);
    if (!Z || !ss || !sd) { free(Z); free(ss); free(sd); return 2; }
    for (int64_t u = 0; u < n_src; ++u) {
        for (int32_t n = 0; n < d_out; ++n) {
            double acc = 0.0;
            for (int32_t k = 0; k < d_in; ++k)
                acc += load_elem(Hsrc, dtype, u * d_in + k) * load_elem(W, dtype, (int64_t)k * d_out + n);
            Z[u * d_out + n] = acc;
        }
        for (int32_t h = 0; h < n_heads; ++h) {
            double ps = 0.0, pd = 0.0;
            for (int32_t j = 0; j < dh; ++j) {
                ps += Z[u * d_out + h * dh + j] * load_elem(a_src, dtype, h * dh + j);
                pd += Z[u * d_out + h * dh + j] * load_elem(a_dst, dtype, h * dh + j);
            }
            ss[u * n_heads + h] = ps;
            sd[u * n_heads + h] = pd;
        }
    }
    int rc = 0;
    for (int64_t r = 0; r < n_dst && !rc; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        if (s >= n_src) { rc = 3; break; }
        int64_t seg = indptr[r + 1] - indptr[r];
        int64_t *ent = (int64_t *)malloc(sizeof(int64_t) * (size_t)(seg + 1));
        double *w = (double *)malloc(sizeof(double) * (size_t)(seg + 1));
        if (!ent || !w) { free(ent); free(w); rc = 2; break; }
        int64_t m = 0;
        if (s >= 0) ent[m++] = s;
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e) {
            if (idx[e] < 0) continue;
            if (idx[e] >= n_src) { rc = 3; break; }
            ent[m++] = idx[e];
        }
        for (int32_t h = 0; h < n_heads && !rc; ++h) {
            double mx = -INFINITY, den = 0.0;
            for (int64_t i = 0; i < m; ++i) {
                double e = (s >= 0 ? sd[s * n_heads + h] : 0.0) + ss[ent[i] * n_heads + h];
                w[i] = e > 0.0 ? e : 0.2 * e;
                if (w[i] > mx) mx = w[i];
            }
            for (int64_t i = 0; i < m; ++i) { w[i] = exp(w[i] - mx); den += w[i]; }
            for (int32_t j = 0; j < dh; ++j) {
                double acc = 0.0;
                for (int64_t i = 0; i < m; ++i) acc += (w[i] / den) * Z[ent[i] * d_out + h * dh + j];
                acc += bias ? load_elem(bias, dtype, h * dh + j) : 0.0;
                if (relu && acc < 0.0) acc = 0.0;
                out[r * d_out + h * dh + j] = acc;
            }
        }
        free(ent);
        free(w);
    }
    free(Z); free(ss); free(sd);
    return rc;
}

/*
 * Backward of one GraphSAGE-mean layer (paper section 5.1, steps 3-4: each micrograph
 * batch runs forward and backward on the server it sits on and the gradients are
 * accumulated until the whole subgraph is done; the discussion section says the
 * accumulated partial gradients are updated in place).
 *
 * With out = act(x_self W_self + m W_neigh + b) and dOut = dL/d out:
 *   dZ        = dOut where the activation passes (relu: where out_fwd > 0), else 0
 *   gW_self  += x_self^T dZ        gW_neigh += m^T dZ        gbias += column sums of dZ
 *   dHsrc[self_idx[r]] += dZ[r] W_self^T
 *   dHsrc[idx[e]]      += (dZ[r] W_neigh^T) / c_r   for every valid entry e of row r
 * out_fwd is the stored forward output that decides the ReLU mask (so that both sides of a
 * comparison take that decision on the same numbers); it may be NULL when relu == 0.
 * All accumulators are double and are ADDED to; dHsrc may be NULL.
 */
int orc_sage_bwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in, const int32_t *self_idx,
                 const int32_t *indptr, const int32_t *idx, int64_t n_dst, const void *W_self,
                 const void *W_neigh, const void *out_fwd, int32_t relu, const double *dOut,
                 int32_t d_out, double *gW_self, double *gW_neigh, double *gbias, double *dHsrc)
{
    (void)n_src;
    double *xs = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *mn = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *dz = (double *)malloc(sizeof(double) * (size_t)d_out);
    if (!xs || !mn || !dz) { free(xs); free(mn); free(dz); return 2; }
    for (int64_t r = 0; r < n_dst; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        for (int32_t k = 0; k < d_in; ++k) {
            xs[k] = s < 0 ? 0.0 : load_elem(Hsrc, dtype, s * d_in + k);
            mn[k] = 0.0;
        }
        int64_t c = 0;
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e) {
            if (idx[e] < 0) continue;
            for (int32_t k = 0; k < d_in; ++k) mn[k] += load_elem(Hsrc, dtype, (int64_t)idx[e] * d_in + k);
            ++c;
        }
        if (c > 0)
            for (int32_t k = 0; k < d_in; ++k) mn[k] /= (double)c;
        for (int32_t n = 0; n < d_out; ++n) {
            int pass = !relu || load_elem(out_fwd, dtype, r * d_out + n) > 0.0;
            dz[n] = pass ? dOut[r * d_out + n] : 0.0;
            if (gbias) gbias[n] += dz[n];
        }
        for (int32_t k = 0; k < d_in; ++k)
            for (int32_t n = 0; n < d_out; ++n) {
                gW_self[(int64_t)k * d_out + n] += xs[k] * dz[n];
                gW_neigh[(int64_t)k * d_out + n] += mn[k] * dz[n];
            }
        if (dHsrc) {
            for (int32_t k = 0; k < d_in; ++k) {
                double gs = 0.0, gm = 0.0;
                for (int32_t n = 0; n < d_out; ++n) {
                    gs += dz[n] * load_elem(W_self, dtype, (int64_t)k * d_out + n);
                    gm += dz[n] * load_elem(W_neigh, dtype, (int64_t)k * d_out + n);
                }
                if (s >= 0) dHsrc[s * d_in + k] += gs;
                if (c > 0)
                    for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e)
                        if (idx[e] >= 0) dHsrc[(int64_t)idx[e] * d_in + k] += gm / (double)c;
            }
        }
    }
    free(xs);
    free(mn);
    free(dz);
    return 0;
}

/*
 * Backward of the GraphSAGE layer with the sum or max aggregator (the aggregators the paper's
 * discussion of generality names next to the mean), same conventions as orc_sage_bwd:
 *   out = act(x_self W_self + a W_neigh + b),   a = aggregate of the valid neighbour rows
 *   dZ  = dOut where the activation passes;  gW_self += x_self^T dZ, gW_neigh += a^T dZ,
 *   gbias += column sums of dZ;  dHsrc[self] += dZ W_self^T;  with g = dZ[r] W_neigh^T:
 *   agg 0 (mean): dHsrc[u] += g / c_r for every valid entry u of row r
 *   agg 1 (sum):  dHsrc[u] += g
 *   agg 2 (max):  per column k only the entry that supplied the maximum receives g[k]: the first
 *                 one in entry order among equals (the forward pass replaces the running maximum
 *                 only by a strictly larger value, so that entry is the one it kept).
 */
int orc_sage_agg_bwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in, const int32_t *self_idx,
                     const int32_t *indptr, const int32_t *idx, int64_t n_dst, const void *W_self,
                     const void *W_neigh, const void *out_fwd, int32_t agg, int32_t relu,
                     const double *dOut, int32_t d_out, double *gW_self, double *gW_neigh,
                     double *gbias, double *dHsrc)
{
    (void)n_src;
    if (agg < 0 || agg > 2) return 1;
    double *xs = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *a = (double *)malloc(sizeof(double) * (size_t)d_in);
    int64_t *arg = (int64_t *)malloc(sizeof(int64_t) * (size_t)d_in);
    double *dz = (double *)malloc(sizeof(double) * (size_t)d_out);
    if (!xs || !a || !arg || !dz) { free(xs); free(a); free(arg); free(dz); return 2; }
    for (int64_t r = 0; r < n_dst; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        for (int32_t k = 0; k < d_in; ++k) {
            xs[k] = s < 0 ? 0.0 : load_elem(Hsrc, dtype, s * d_in + k);
            a[k] = 0.0;
            arg[k] = -1;
        }
        int64_t c = 0;
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e) {
            int64_t u = idx[e];
            if (u < 0) continue;
            for (int32_t k = 0; k < d_in; ++k) {
                double v = load_elem(Hsrc, dtype, u * d_in + k);
                if (agg == 2) {
                    if (c == 0 || v > a[k]) { a[k] = v; arg[k] = u; }
                } else {
                    a[k] += v;
                }
            }
            ++c;
        }
        if (agg == 0 && c > 0)
            for (int32_t k = 0; k < d_in; ++k) a[k] /= (double)c;
        for (int32_t n = 0; n < d_out; ++n) {
            int pass = !relu || load_elem(out_fwd, dtype, r * d_out + n) > 0.0;
            dz[n] = pass ? dOut[r * d_out + n] : 0.0;
            if (gbias) gbias[n] += dz[n];
        }
        for (int32_t k = 0; k < d_in; ++k)
            for (int32_t n = 0; n < d_out; ++n) {
                gW_self[(int64_t)k * d_out + n] += xs[k] * dz[n];
                gW_neigh[(int64_t)k * d_out + n] += a[k] * dz[n];
            }
        if (dHsrc) {
            for (int32_t k = 0; k < d_in; ++k) {
                double gs = 0.0, ga = 0.0;
                for (int32_t n = 0; n < d_out; ++n) {
                    gs += dz[n] * load_elem(W_self, dtype, (int64_t)k * d_out + n);
                    ga += dz[n] * load_elem(W_neigh, dtype, (int64_t)k * d_out + n);
                }
                if (s >= 0) dHsrc[s * d_in + k] += gs;
                if (c == 0) continue;
                if (agg == 2) {
                    dHsrc[arg[k] * d_in + k] += ga;
                } else {
                    const double share = agg == 0 ? ga / (double)c : ga;
                    for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e)
                        if (idx[e] >= 0) dHsrc[(int64_t)idx[e] * d_in + k] += share;
                }
            }
        }
    }
    free(xs); free(a); free(arg); free(dz);
    return 0;
}

/*
 * Backward of the GCN-style layer of orc_gcn_fwd:
 *   a = (x_self + sum of the valid neighbour rows) / t,  t = number of terms (norm 1) or 1 (norm 0)
 *   out = act(a W + b);  dZ = dOut where the activation passes
 *   gW += a^T dZ;  gbias += column sums of dZ;  every term's source row receives (dZ[r] W^T) / t
 * (a row that occurs several times among the terms receives it once per occurrence).
 */
int orc_gcn_bwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in, const int32_t *self_idx,
                const int32_t *indptr, const int32_t *idx, int64_t n_dst, const void *W,
                const void *out_fwd, int32_t norm, int32_t relu, const double *dOut, int32_t d_out,
                double *gW, double *gbias, double *dHsrc)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *dz = (double *)malloc(sizeof(double) * (size_t)d_out);
    if (!a || !dz) { free(a); free(dz); return 2; }
    for (int64_t r = 0; r < n_dst; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        int64_t terms = 0;
        for (int32_t k = 0; k < d_in; ++k) a[k] = 0.0;
        if (s >= 0) {
            for (int32_t k = 0; k < d_in; ++k) a[k] += load_elem(Hsrc, dtype, s * d_in + k);
            ++terms;
        }
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e) {
            if (idx[e] < 0) continue;
            for (int32_t k = 0; k < d_in; ++k) a[k] += load_elem(Hsrc, dtype, (int64_t)idx[e] * d_in + k);
            ++terms;
        }
        const double t = norm && terms > 0 ? (double)terms : 1.0;
        for (int32_t k = 0; k < d_in; ++k) a[k] /= t;
        for (int32_t n = 0; n < d_out; ++n) {
            int pass = !relu || load_elem(out_fwd, dtype, r * d_out + n) > 0.0;
            dz[n] = pass ? dOut[r * d_out + n] : 0.0;
            if (gbias) gbias[n] += dz[n];
        }
        for (int32_t k = 0; k < d_in; ++k)
            for (int32_t n = 0; n < d_out; ++n) gW[(int64_t)k * d_out + n] += a[k] * dz[n];
        if (dHsrc) {
            for (int32_t k = 0; k < d_in; ++k) {
                double ga = 0.0;
                for (int32_t n = 0; n < d_out; ++n) ga += dz[n] * load_elem(W, dtype, (int64_t)k * d_out + n);
                ga /= t;
                if (s >= 0) dHsrc[s * d_in + k] += ga;
                for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e)
                    if (idx[e] >= 0) dHsrc[(int64_t)idx[e] * d_in + k] += ga;
            }
        }
    }
    free(a); free(dz);
    (void)n_src;
    return 0;
}

/*
 * Backward of the graph-attention layer of orc_gat_fwd (the chain rule written out; the layer is
 * Velickovic et al. 2018).  With y[r,h] = sum_i alpha_i z_{u_i}[h] + b[h], out = act(y) and
 * dY = dOut where the activation passes, per destination row r and head h over its entries
 * u_0..u_{m-1} (self first, then the valid neighbours):
 *   gbias[h]    += dY[r,h]
 *   dalpha_i     = <dY[r,h], z_{u_i}[h]>              dz_{u_i}[h] += alpha_i dY[r,h]
 *   dl_i         = alpha_i (dalpha_i - sum_j alpha_j dalpha_j)            (softmax)
 *   de_i         = dl_i * (e_i > 0 ? 1 : 0.2)                             (LeakyReLU_0.2)
 *   ds_src[u_i,h] += de_i;   ds_dst[s,h] += sum_i de_i   (only if the self row exists)
 * and then per source row u:
 *   dz_u[h]     += ds_src[u,h] a_src[h] + ds_dst[u,h] a_dst[h]
 *   ga_src[h]   += ds_src[u,h] z_u[h];   ga_dst[h] += ds_dst[u,h] z_u[h]
 *   gW          += Hsrc[u]^T dz_u;       dHsrc[u] += dz_u W^T
 * Accumulators are double and ADDED to; gbias and dHsrc may be NULL.
 */
int orc_gat_bwd(const void *Hsrc, int dtype, int64_t n_src, int32_t d_in, const int32_t *self_idx,
                const int32_t *indptr, const int32_t *idx, int64_t n_dst, const void *W,
                const void *a_src, const void *a_dst, const void *out_fwd, int32_t relu,
                const double *dOut, int32_t d_out, int32_t n_heads, double *gW, double *ga_src,
                double *ga_dst, double *gbias, double *dHsrc)
{
    if (n_heads < 1 || d_out % n_heads != 0) return 1;
    const int32_t dh = d_out / n_heads;
    const size_t ns = (size_t)(n_src > 0 ? n_src : 1);
    double *Z = (double *)malloc(sizeof(double) * ns * (size_t)d_out);
    double *dZ = (double *)calloc(ns * (size_t)d_out, sizeof(double));
    double *ss = (double *)malloc(sizeof(double) * ns * (size_t)n_heads);
    double *sd = (double *)malloc(sizeof(double) * ns * (size_t)n_heads);
    double *dss = (double *)calloc(ns * (size_t)n_heads, sizeof(double));
    double *dsd = (double *)calloc(ns * (size_t)n_heads, sizeof(double));
    if (!Z || !dZ || !ss || !sd || !dss || !dsd) { free(Z); free(dZ); free(ss); free(sd); free(dss); free(dsd); return 2; }
    for (int64_t u = 0; u < n_src; ++u) {
        for (int32_t n = 0; n < d_out; ++n) {
            double acc = 0.0;
            for (int32_t k = 0; k < d_in; ++k)
                acc += load_elem(Hsrc, dtype, u * d_in + k) * load_elem(W, dtype, (int64_t)k * d_out + n);
            Z[u * d_out + n] = acc;
        }
        for (int32_t h = 0; h < n_heads; ++h) {
            double ps = 0.0, pd = 0.0;
            for (int32_t j = 0; j < dh; ++j) {
                ps += Z[u * d_out + h * dh + j] * load_elem(a_src, dtype, h * dh + j);
                pd += Z[u * d_out + h * dh + j] * load_elem(a_dst, dtype, h * dh + j);
            }
            ss[u * n_heads + h] = ps;
            sd[u * n_heads + h] = pd;
        }
    }
    int rc = 0;
    for (int64_t r = 0; r < n_dst && !rc; ++r) {
        int64_t s = self_idx ? self_idx[r] : r;
        int64_t seg = indptr[r + 1] - indptr[r];
        int64_t *ent = (int64_t *)malloc(sizeof(int64_t) * (size_t)(seg + 1));
        double *al = (double *)malloc(sizeof(double) * (size_t)(seg + 1));
        double *ev = (double *)malloc(sizeof(double) * (size_t)(seg + 1));
        double *da = (double *)malloc(sizeof(double) * (size_t)(seg + 1));
        if (!ent || !al || !ev || !da) { free(ent); free(al); free(ev); free(da); rc = 2; break; }
        int64_t m = 0;
        if (s >= 0) ent[m++] = s;
        for (int64_t e = indptr[r]; e < indptr[r + 1]; ++e)
            if (idx[e] >= 0) ent[m++] = idx[e];
        for (int32_t h = 0; h < n_heads; ++h) {
            /* dY of this row and head */
            for (int32_t j = 0; j < dh; ++j) {
                int64_t o = r * d_out + h * dh + j;
                int pass = !relu || load_elem(out_fwd, dtype, o) > 0.0;
                double g = pass ? dOut[o] : 0.0;
                if (gbias) gbias[h * dh + j] += g;
            }
            if (m == 0) continue;
            double mx = -INFINITY, den = 0.0;
            for (int64_t i = 0; i < m; ++i) {
                ev[i] = (s >= 0 ? sd[s * n_heads + h] : 0.0) + ss[ent[i] * n_heads + h];
                al[i] = ev[i] > 0.0 ? ev[i] : 0.2 * ev[i];
                if (al[i] > mx) mx = al[i];
            }
            for (int64_t i = 0; i < m; ++i) { al[i] = exp(al[i] - mx); den += al[i]; }
            double dot = 0.0;
            for (int64_t i = 0; i < m; ++i) {
                al[i] /= den;
                double d = 0.0;
                for (int32_t j = 0; j < dh; ++j) {
                    int64_t o = r * d_out + h * dh + j;
                    int pass = !relu || load_elem(out_fwd, dtype, o) > 0.0;
                    double g = pass ? dOut[o] : 0.0;
                    d += g * Z[ent[i] * d_out + h * dh + j];
                    dZ[ent[i] * d_out + h * dh + j] += al[i] * g;
                }
                da[i] = d;
                dot += al[i] * d;
            }
            for (int64_t i = 0; i < m; ++i) {
                double de = al[i] * (da[i] - dot) * (ev[i] > 0.0 ? 1.0 : 0.2);
                dss[ent[i] * n_heads + h] += de;
                if (s >= 0) dsd[s * n_heads + h] += de;
            }
        }
        free(ent); free(al); free(ev); free(da);
    }
    for (int64_t u = 0; u < n_src && !rc; ++u) {
        for (int32_t h = 0; h < n_heads; ++h)
            for (int32_t j = 0; j < dh; ++j) {
                int64_t o = u * d_out + h * dh + j;
                ga_src[h * dh + j] += dss[u * n_heads + h] * Z[o];
                ga_dst[h * dh + j] += dsd[u * n_heads + h] * Z[o];
                dZ[o] += dss[u * n_heads + h] * load_elem(a_src, dtype, h * dh + j) +
                         dsd[u * n_heads + h] * load_elem(a_dst, dtype, h * dh + j);
            }
        for (int32_t k = 0; k < d_in; ++k) {
            double x = load_elem(Hsrc, dtype, u * d_in + k), g = 0.0;
            for (int32_t n = 0; n < d_out; ++n) {
                gW[(int64_t)k * d_out + n] += x * dZ[u * d_out + n];
                g += dZ[u * d_out + n] * load_elem(W, dtype, (int64_t)k * d_out + n);
            }
            if (dHsrc) dHsrc[u * d_in + k] += g;
        }
    }
    free(Z); free(dZ); free(ss); free(sd); free(dss); free(dsd);
    return rc;
}
