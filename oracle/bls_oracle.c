/*
 * CPU oracle for the distributed embedding-lookup path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C that states what the path computes, written from
 * the paper's description of the problem and sharing nothing with the HIP library.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call it;
 * the product never does.
 *
 * What the paper fixes (section / listing cited at each function):
 *   - every rank owns a contiguous block of the global batch (Introduction: row-block
 *     partition of the batch into mini-batches) and a share of the embedding tables
 *     (the partitioning strategy is a given, not part of the method);
 *   - each rank works out which vectors it needs from which rank and fetches them
 *     with an alltoallv (Introduction);
 *   - the lookup itself is an EmbeddingBag over (offsets, indices) per table and the
 *     alltoallv moves the pooled vectors, sized by the number of tables per rank
 *     (Listing 1: apply_emb, then alltoall(ly, n_emb_per_rank));
 *   - with bound k = 0 the exchange is semantically MPI_Alltoallv (A zero-bound
 *     parameter), and for any k the results are unchanged (Abstract; Related Work:
 *     the retrieved vectors are never approximated);
 *   - completion copies the receive region of the iteration's ring slot to the
 *     caller's buffer (Alltoallv completion).
 * Where the paper is silent the reading taken is stated beside the code and listed in
 * the design notes: sum pooling without weights; a single fp32 accumulator starting
 * at +0.0f with terms added in bag order; stable (input-order) placement inside every
 * bucket; row-wise block shards of ceil(rows/P) rows; the first B mod P ranks get one
 * extra sample.
 *
 * Notation: P ranks, T tables, B global batch, D vector length, bag g = t*B + b,
 * lookup l in [offsets[g], offsets[g+1]); requester s(b); owner d(t, idx); F = 1 for
 * table-wise partition and P for row-wise.
 *
 * Every function returns 0, or a negative code: -1 bad argument, -2 index or offset
 * out of range, -3 out of memory.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ERANGE (-2)
#define ORC_ENOMEM (-3)

/* ---- partition helpers -------------------------------------------------------- */

/* Mini-batch of rank s: samples [first(s), first(s+1)).  The first B mod P ranks hold
 * one sample more (reading; every benchmark workload divides evenly). */
static int64_t batch_first(int64_t B, int P, int s)
{
    int64_t q = B / P, r = B % P;
    return (int64_t)s * q + (s < r ? s : r);
}

static int requester_of(int64_t B, int P, int64_t b)
{
    int s;
    for (s = 0; s < P; ++s)
        if (b < batch_first(B, P, s + 1)) return s;
    return P - 1;
}

/* Rows per shard for the row-wise block partition: ceil(rows / P); the last shards may
 * be short or empty. */
static int64_t rows_per_shard(int64_t rows, int P) { return (rows + P - 1) / P; }

/* n_loc[d]: number of tables rank d serves; loc[t]: position of t among its owner's
 * tables in increasing t.  Row-wise: every rank serves a shard of every table. */
static void local_tables(int P, int T, int part_kind, const int32_t *owner, int *n_loc, int *loc)
{
    int t, d;
    for (d = 0; d < P; ++d) n_loc[d] = 0;
    for (t = 0; t < T; ++t) {
        if (part_kind == 1) { loc[t] = t; }
        else { loc[t] = n_loc[owner[t]]; n_loc[owner[t]] += 1; }
    }
    if (part_kind == 1) for (d = 0; d < P; ++d) n_loc[d] = T;
}

/* Segment index of (owner d, requester s, local table t_loc, local sample b_loc): the
 * order in which owner-side lookups are stored, d-major, then s, then table, then
 * sample.  Also the order of pooled vectors in the send regions. */
static int64_t segment_index(int P, int64_t B, const int *n_loc, int d, int s, int t_loc, int64_t b_loc)
{
    int64_t base = 0;
    int dd;
    for (dd = 0; dd < d; ++dd) base += (int64_t)n_loc[dd] * B;
    base += (int64_t)n_loc[d] * batch_first(B, P, s);
    return base + (int64_t)t_loc * (batch_first(B, P, s + 1) - batch_first(B, P, s)) + b_loc;
}

static int check_partition(int P, int T, int part_kind, const int64_t *rows, const int32_t *owner)
{
    int t;
    if (P < 1 || T < 1 || (part_kind != 0 && part_kind != 1)) return ORC_EINVAL;
    for (t = 0; t < T; ++t) {
        if (rows[t] < 1) return ORC_EINVAL;
        if (part_kind == 0 && (owner[t] < 0 || owner[t] >= P)) return ORC_EINVAL;
    }
    return ORC_OK;
}

/* ---- index bucketing: counts, displacements, stable placement ------------------- */

/*
 * Introduction (every process works out which vectors it needs from which other
 * process and fetches them with an alltoallv): for every lookup l, in
 * increasing l, the requester s, the owner d and the row r inside the owner's shard.
 * sendcounts[s][d] = number of lookups rank s asks of rank d; recvcounts is its
 * transpose; displacements are running sums (the MPI_Alltoallv convention the
 * paper's benchmark signature uses); lookups keep their input order inside a bucket.
 *
 * Outputs: sendcounts, sdispls [P*P] row-major [s][d]; recvcounts, rdispls [P*P]
 * row-major [d][s]; ridx[nnz] local rows in owner-side order (d, then s, then l);
 * segoff[F*T*B+1] start of every (d, s, t_loc, b_loc) segment in ridx; perm[nnz]
 * (nullable) requester-side position of lookup l (s, then d, then l).
 */
int orc_plan_weighted(int P, int T, int64_t B, int part_kind, const int64_t *rows, const int32_t *owner,
                      const int64_t *indices, const int64_t *offsets, const float *weights,
                      int64_t *sendcounts, int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls,
                      int64_t *ridx, float *rweights, int64_t *segoff, int64_t *perm);

int orc_plan(int P, int T, int64_t B, int part_kind, const int64_t *rows, const int32_t *owner,
             const int64_t *indices, const int64_t *offsets,
             int64_t *sendcounts, int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls,
             int64_t *ridx, int64_t *segoff, int64_t *perm)
{
    return orc_plan_weighted(P, T, B, part_kind, rows, owner, indices, offsets, NULL, sendcounts, sdispls,
                             recvcounts, rdispls, ridx, NULL, segoff, perm);
}

/* The same with per-sample weights (Listing 1 passes them to apply_emb as v_W_l): the weight
 * of lookup l travels with it, rweights[.] is in the same owner order as ridx[.]. */
int orc_plan_weighted(int P, int T, int64_t B, int part_kind, const int64_t *rows, const int32_t *owner,
                      const int64_t *indices, const int64_t *offsets, const float *weights,
                      int64_t *sendcounts, int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls,
                      int64_t *ridx, float *rweights, int64_t *segoff, int64_t *perm)
{
    int rc = check_partition(P, T, part_kind, rows, owner);
    int s, d, t;
    int64_t b, l, g, nseg, i;
    int F = part_kind == 1 ? P : 1;
    int *n_loc, *loc;
    int64_t *sbase, *rbase, *cursor, *seglen;
    if (rc) return rc;
    if (B < 1) return ORC_EINVAL;
    nseg = (int64_t)F * T * B;
    n_loc = (int *)malloc(sizeof(int) * P);
    loc = (int *)malloc(sizeof(int) * T);
    sbase = (int64_t *)malloc(sizeof(int64_t) * P);
    rbase = (int64_t *)malloc(sizeof(int64_t) * P);
    cursor = (int64_t *)malloc(sizeof(int64_t) * P * P);
    seglen = (int64_t *)calloc((size_t)nseg, sizeof(int64_t));
    if (!n_loc || !loc || !sbase || !rbase || !cursor || !seglen) { rc = ORC_ENOMEM; goto done; }
    local_tables(P, T, part_kind, owner, n_loc, loc);

    if (offsets[0] != 0) { rc = ORC_ERANGE; goto done; }
    for (g = 0; g < (int64_t)T * B; ++g)
        if (offsets[g + 1] < offsets[g]) { rc = ORC_ERANGE; goto done; }

    /* pass 1: count */
    for (i = 0; i < (int64_t)P * P; ++i) sendcounts[i] = 0;
    for (t = 0; t < T; ++t) {
        for (b = 0; b < B; ++b) {
            g = (int64_t)t * B + b;
            s = requester_of(B, P, b);
            for (l = offsets[g]; l < offsets[g + 1]; ++l) {
                int64_t idx = indices[l];
                if (idx < 0 || idx >= rows[t]) { rc = ORC_ERANGE; goto done; }
                d = part_kind == 1 ? (int)(idx / rows_per_shard(rows[t], P)) : owner[t];
                sendcounts[s * P + d] += 1;
                seglen[segment_index(P, B, n_loc, d, s, loc[t], b - batch_first(B, P, s))] += 1;
            }
        }
    }
    /* transpose and running sums */
    for (s = 0; s < P; ++s)
        for (d = 0; d < P; ++d) recvcounts[d * P + s] = sendcounts[s * P + d];
    for (s = 0; s < P; ++s) {
        int64_t run = 0;
        for (d = 0; d < P; ++d) { sdispls[s * P + d] = run; run += sendcounts[s * P + d]; }
    }
    for (d = 0; d < P; ++d) {
        int64_t run = 0;
        for (s = 0; s < P; ++s) { rdispls[d * P + s] = run; run += recvcounts[d * P + s]; }
    }
    {   /* region bases: rank regions laid one after another */
        int64_t run = 0;
        for (s = 0; s < P; ++s) {
            sbase[s] = run;
            for (d = 0; d < P; ++d) run += sendcounts[s * P + d];
        }
        run = 0;
        for (d = 0; d < P; ++d) {
            rbase[d] = run;
            for (s = 0; s < P; ++s) run += recvcounts[d * P + s];
        }
    }
    segoff[0] = 0;
    for (i = 0; i < nseg; ++i) segoff[i + 1] = segoff[i] + seglen[i];

    /* pass 2: stable placement, one cursor per (s, d) bucket */
    for (i = 0; i < (int64_t)P * P; ++i) cursor[i] = 0;
    for (t = 0; t < T; ++t) {
        for (b = 0; b < B; ++b) {
            g = (int64_t)t * B + b;
            s = requester_of(B, P, b);
            for (l = offsets[g]; l < offsets[g + 1]; ++l) {
                int64_t idx = indices[l], r, rank;
                if (part_kind == 1) {
                    int64_t rps = rows_per_shard(rows[t], P);
                    d = (int)(idx / rps);
                    r = idx - (int64_t)d * rps;
                } else {
                    d = owner[t];
                    r = idx;
                }
                rank = cursor[s * P + d]++;
                ridx[rbase[d] + rdispls[d * P + s] + rank] = r;
                if (weights && rweights) rweights[rbase[d] + rdispls[d * P + s] + rank] = weights[l];
                if (perm) perm[l] = sbase[s] + sdispls[s * P + d] + rank;
            }
        }
    }
done:
    free(n_loc); free(loc); free(sbase); free(rbase); free(cursor); free(seglen);
    return rc;
}

/* ---- EmbeddingBag --------------------------------------------------------------- */

/* IEEE binary16 -> binary32, exact. */
static float half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1Fu, m = h & 0x3FFu, bits;
    float f;
    if (e == 0) {
        if (m == 0) bits = sign;
        else {                       /* subnormal: normalise */
            int sh = 0;
            while (!(m & 0x400u)) { m <<= 1; ++sh; }
            m &= 0x3FFu;
            bits = sign | ((uint32_t)(127 - 15 - sh + 1) << 23) | (m << 13);
        }
    } else if (e == 31) bits = sign | 0x7F800000u | (m << 13);
    else bits = sign | ((e + 127 - 15) << 23) | (m << 13);
    memcpy(&f, &bits, 4);
    return f;
}

/* Bytes from one row of a row-quantised table (dtype 2) to the next: D one-byte codes, the
 * row's fp32 scale, its fp32 bias, padded to a multiple of 16. */
static int64_t rowq_stride(int D) { return ((int64_t)D + 8 + 15) / 16 * 16; }

/* 8-bit float E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, the
 * all-ones exponent-and-mantissa pattern is NaN, subnormals at exponent 0) -> binary32, exact. */
static float e4m3_to_float(uint8_t v)
{
    int e = (v >> 3) & 15, m = v & 7;
    float mag;
    if (e == 15 && m == 7) { uint32_t nan = 0x7FC00000u | ((uint32_t)(v & 0x80u) << 24); float f; memcpy(&f, &nan, 4); return f; }
    if (e == 0) mag = (float)m * 0.001953125f;                      /* m * 2^-9 */
    else {
        uint32_t bits = ((uint32_t)(e + 120) << 23) | ((uint32_t)m << 20);   /* 2^(e-7) * (1 + m/8) */
        memcpy(&mag, &bits, 4);
    }
    return (v & 0x80u) ? -mag : mag;
}

/* Element (row, c) of a table as the fp32 number it stands for.  dtype 0: fp32; 1: binary16
 * (conversion exact); 2 and 3: 8-bit codes with one scale and one bias per row (an extension
 * the paper does not describe; reading: value = code * scale + bias evaluated in fp32, the
 * product rounded, then the sum rounded - the usual row-wise 8-bit embedding format), the code
 * an unsigned integer (2) or an E4M3 float (3). */
static float elem(const void *table, int dtype, int D, int64_t row, int c)
{
    if (dtype == 2 || dtype == 3) {
        const uint8_t *p = (const uint8_t *)table + row * rowq_stride(D);
        float scale, bias, prod;
        memcpy(&scale, p + D, 4);
        memcpy(&bias, p + D + 4, 4);
        prod = (dtype == 2 ? (float)p[c] : e4m3_to_float(p[c])) * scale;
        return prod + bias;
    }
    return dtype == 1 ? half_to_float(((const uint16_t *)table)[row * D + c]) : ((const float *)table)[row * D + c];
}

/*
 * Listing 1, apply_emb: the plain definition of the whole path's result.
 *   Out[b][t][c] = sum over l in bag (t,b) of W_t[indices[l]][c]
 * computed in double precision (out64, nullable) and with one fp32 accumulator that
 * starts at +0.0f and adds the terms in increasing l (out32, nullable).  tables[t] is
 * table t with global row numbering, dtype 0 = fp32, 1 = fp16, 2 / 3 = row-quantised 8-bit storage
 * (integer / E4M3 codes).
 */
int orc_embbag_plain_ex(int T, int D, int64_t B, int dtype, const int64_t *rows, const void *const *tables,
                        const int64_t *indices, const int64_t *offsets, const float *weights, int mean,
                        double *out64, float *out32);

int orc_embbag_plain(int T, int D, int64_t B, int dtype, const int64_t *rows, const void *const *tables,
                     const int64_t *indices, const int64_t *offsets, double *out64, float *out32)
{
    return orc_embbag_plain_ex(T, D, B, dtype, rows, tables, indices, offsets, NULL, 0, out64, out32);
}

/* EmbeddingBag with per-sample weights (sum of w_l * row_l) or mean pooling (sum / bag length,
 * an empty bag gives +0).  fp32 variant: every product and every sum rounded separately, the
 * mean by one fp32 division at the end. */
int orc_embbag_plain_ex(int T, int D, int64_t B, int dtype, const int64_t *rows, const void *const *tables,
                        const int64_t *indices, const int64_t *offsets, const float *weights, int mean,
                        double *out64, float *out32)
{
    int t, c;
    int64_t b, l;
    for (t = 0; t < T; ++t)
        for (b = 0; b < B; ++b) {
            int64_t g = (int64_t)t * B + b;
            for (l = offsets[g]; l < offsets[g + 1]; ++l)
                if (indices[l] < 0 || indices[l] >= rows[t]) return ORC_ERANGE;
            for (c = 0; c < D; ++c) {
                double a64 = 0.0;
                float a32 = 0.0f;
                for (l = offsets[g]; l < offsets[g + 1]; ++l) {
                    float x = elem(tables[t], dtype, D, indices[l], c);
                    if (weights) {
                        float term = weights[l] * x;
                        a64 += (double)weights[l] * (double)x;
                        a32 += term;
                    } else {
                        a64 += (double)x;
                        a32 += x;
                    }
                }
                if (mean && offsets[g + 1] > offsets[g]) {
                    a64 /= (double)(offsets[g + 1] - offsets[g]);
                    a32 /= (float)(offsets[g + 1] - offsets[g]);
                }
                if (out64) out64[((int64_t)b * T + t) * D + c] = a64;
                if (out32) out32[((int64_t)b * T + t) * D + c] = a32;
            }
        }
    return ORC_OK;
}

/* Sum of the absolute values of a bag's terms, in double: the scale the fp32
 * tolerance is relative to.  Same layout as orc_embbag_plain's outputs. */
int orc_embbag_absmass(int T, int D, int64_t B, int dtype, const void *const *tables,
                       const int64_t *indices, const int64_t *offsets, double *mass)
{
    int t, c;
    int64_t b, l;
    for (t = 0; t < T; ++t)
        for (b = 0; b < B; ++b)
            for (c = 0; c < D; ++c) {
                int64_t g = (int64_t)t * B + b;
                double a = 0.0;
                for (l = offsets[g]; l < offsets[g + 1]; ++l) {
                    double x = (double)elem(tables[t], dtype, D, indices[l], c);
                    a += x < 0 ? -x : x;
                }
                mass[((int64_t)b * T + t) * D + c] = a;
            }
    return ORC_OK;
}

/*
 * Owner-side pooling (Listing 1, apply_emb on each rank's local tables / shards).
 * For owner d, local table t_loc, sample b = first(s) + b_loc:
 *   Y_d[t_loc][b][:] = sum over the segment's rows of W_{t,d}[ridx[.]][:]
 * fp32 accumulator from +0.0f, terms in segment order.  Y is the concatenation of
 * Y_0 .. Y_{P-1}, each [n_loc(d)][B][D].  Row-wise shard d of table t is rows
 * [d*rps, min((d+1)*rps, rows_t)) of the global table.
 */
int orc_pool_weighted(int P, int T, int D, int64_t B, int part_kind, const int64_t *rows, const int32_t *owner,
                      int dtype, const void *const *tables, const int64_t *ridx, const float *rweights,
                      const int64_t *segoff, float *Y);

int orc_pool(int P, int T, int D, int64_t B, int part_kind, const int64_t *rows, const int32_t *owner,
             int dtype, const void *const *tables, const int64_t *ridx, const int64_t *segoff, float *Y)
{
    return orc_pool_weighted(P, T, D, B, part_kind, rows, owner, dtype, tables, ridx, NULL, segoff, Y);
}

/* rweights (nullable): weight of every lookup in owner order; each term w * x is rounded to
 * fp32 before it is added. */
int orc_pool_weighted(int P, int T, int D, int64_t B, int part_kind, const int64_t *rows, const int32_t *owner,
                      int dtype, const void *const *tables, const int64_t *ridx, const float *rweights,
                      const int64_t *segoff, float *Y)
{
    int rc = check_partition(P, T, part_kind, rows, owner);
    int *n_loc, *loc, d, s, t, c;
    int64_t ybase = 0;
    if (rc) return rc;
    n_loc = (int *)malloc(sizeof(int) * P);
    loc = (int *)malloc(sizeof(int) * T);
    if (!n_loc || !loc) { free(n_loc); free(loc); return ORC_ENOMEM; }
    local_tables(P, T, part_kind, owner, n_loc, loc);
    for (d = 0; d < P; ++d) {
        for (t = 0; t < T; ++t) {
            int64_t shard_first, shard_rows;
            if (part_kind == 0 && owner[t] != d) continue;
            if (part_kind == 1) {
                int64_t rps = rows_per_shard(rows[t], P);
                shard_first = (int64_t)d * rps;
                shard_rows = rows[t] - shard_first;
                if (shard_rows > rps) shard_rows = rps;
                if (shard_rows < 0) shard_rows = 0;
            } else { shard_first = 0; shard_rows = rows[t]; }
            for (s = 0; s < P; ++s) {
                int64_t f = batch_first(B, P, s), n = batch_first(B, P, s + 1) - f, b_loc, j;
                for (b_loc = 0; b_loc < n; ++b_loc) {
                    int64_t sg = segment_index(P, B, n_loc, d, s, loc[t], b_loc);
                    float *y = Y + ybase + ((int64_t)loc[t] * B + f + b_loc) * D;
                    for (j = segoff[sg]; j < segoff[sg + 1]; ++j)
                        if (ridx[j] < 0 || ridx[j] >= shard_rows) { rc = ORC_ERANGE; goto done; }
                    for (c = 0; c < D; ++c) {
                        float acc = 0.0f;
                        for (j = segoff[sg]; j < segoff[sg + 1]; ++j) {
                            float x = elem(tables[t], dtype, D, shard_first + ridx[j], c);
                            if (rweights) { float term = rweights[j] * x; acc += term; }
                            else acc += x;
                        }
                        y[c] = acc;
                    }
                }
            }
        }
        ybase += (int64_t)n_loc[d] * B * D;
    }
done:
    free(n_loc); free(loc);
    return rc;
}

/* ---- pooled-vector exchange ----------------------------------------------------- */

/*
 * Listing 1, alltoall(ly, n_emb_per_rank): counts of the pooled exchange in fp32
 * elements.  Owner d sends requester s its n_loc(d) local tables for s's mini-batch:
 * pcount[d][s] = n_loc(d) * B_loc(s) * D.  Displacements are running sums; region
 * bases lay the ranks' send (resp. receive) regions one after another.
 * Outputs [P*P]: pcount, psdispl row-major [d][s]; prcount, prdispl row-major [s][d];
 * [P]: psbase, prbase.
 */
int orc_pooled_counts(int P, int T, int D, int64_t B, int part_kind, const int32_t *owner,
                      int64_t *pcount, int64_t *psdispl, int64_t *prcount, int64_t *prdispl,
                      int64_t *psbase, int64_t *prbase)
{
    int *n_loc = (int *)malloc(sizeof(int) * P), *loc = (int *)malloc(sizeof(int) * T), d, s;
    int64_t run;
    if (!n_loc || !loc) { free(n_loc); free(loc); return ORC_ENOMEM; }
    local_tables(P, T, part_kind, owner, n_loc, loc);
    for (d = 0; d < P; ++d)
        for (s = 0; s < P; ++s) {
            int64_t n = batch_first(B, P, s + 1) - batch_first(B, P, s);
            pcount[d * P + s] = (int64_t)n_loc[d] * n * D;
            prcount[s * P + d] = pcount[d * P + s];
        }
    for (d = 0, run = 0; d < P; ++d) {
        int64_t in = 0;
        psbase[d] = run;
        for (s = 0; s < P; ++s) { psdispl[d * P + s] = in; in += pcount[d * P + s]; }
        run += in;
    }
    for (s = 0, run = 0; s < P; ++s) {
        int64_t in = 0;
        prbase[s] = run;
        for (d = 0; d < P; ++d) { prdispl[s * P + d] = in; in += prcount[s * P + d]; }
        run += in;
    }
    free(n_loc); free(loc);
    return ORC_OK;
}

/* S(p), the send buffer of Fig. 5: owner d lays its pooled vectors out by destination,
 * S_d[s][t_loc][b_loc][:] = Y_d[t_loc][first(s) + b_loc][:]. */
int orc_pack(int P, int T, int D, int64_t B, int part_kind, const int32_t *owner, const float *Y, float *S)
{
    int *n_loc = (int *)malloc(sizeof(int) * P), *loc = (int *)malloc(sizeof(int) * T), d, s, tl;
    int64_t ybase = 0;
    if (!n_loc || !loc) { free(n_loc); free(loc); return ORC_ENOMEM; }
    local_tables(P, T, part_kind, owner, n_loc, loc);
    for (d = 0; d < P; ++d) {
        for (s = 0; s < P; ++s) {
            int64_t f = batch_first(B, P, s), n = batch_first(B, P, s + 1) - f, b_loc;
            for (tl = 0; tl < n_loc[d]; ++tl)
                for (b_loc = 0; b_loc < n; ++b_loc)
                    memcpy(S + segment_index(P, B, n_loc, d, s, tl, b_loc) * D,
                           Y + ybase + ((int64_t)tl * B + f + b_loc) * D, sizeof(float) * D);
        }
        ybase += (int64_t)n_loc[d] * B * D;
    }
    free(n_loc); free(loc);
    return ORC_OK;
}

/*
 * MPI_Alltoallv as the textbook defines it (A zero-bound parameter: with k = 0 the
 * collective is semantically MPI_Alltoallv): for every source and destination rank,
 *   recv[dst][rdispls[dst][src] ..] = send[src][sdispls[src][dst] ..], sendcounts[src][dst] items.
 * Rank regions are concatenated: rank p's send region starts at sbase[p], its receive
 * region at rbase[p].  Alltoallv initiation writes these blocks into R(dst, slot); on
 * one device that write is this copy.
 */
int orc_alltoallv_f32(int P, const float *send, const int64_t *sbase, const int64_t *sendcounts,
                      const int64_t *sdispls, float *recv, const int64_t *rbase,
                      const int64_t *recvcounts, const int64_t *rdispls)
{
    int src, dst;
    for (src = 0; src < P; ++src)
        for (dst = 0; dst < P; ++dst) {
            if (recvcounts[dst * P + src] != sendcounts[src * P + dst]) return ORC_EINVAL;
            memcpy(recv + rbase[dst] + rdispls[dst * P + src],
                   send + sbase[src] + sdispls[src * P + dst],
                   sizeof(float) * (size_t)sendcounts[src * P + dst]);
        }
    return ORC_OK;
}

/*
 * Alltoallv completion: copy the receive region out into the caller's tensor,
 * Out[b][t][:] for b in the requester's mini-batch.  Table-wise: the one block that
 * holds table t.  Row-wise: every owner sent a partial sum for (t, b); add them from
 * +0.0f in increasing owner rank (reading: the paper never shards a table by rows).
 * R is the concatenation of the requesters' receive regions, each [d][t_loc][b_loc][D].
 */
int orc_unpack_mean(int P, int T, int D, int64_t B, int part_kind, const int32_t *owner, const float *R,
                    const int64_t *offsets, float *Out);

int orc_unpack(int P, int T, int D, int64_t B, int part_kind, const int32_t *owner, const float *R, float *Out)
{
    return orc_unpack_mean(P, T, D, B, part_kind, owner, R, NULL, Out);
}

/* offsets (nullable): mean pooling - after the copy-out (and, row-wise, the sum of the
 * partials) every vector of a non-empty bag is divided by the bag's length in fp32. */
int orc_unpack_mean(int P, int T, int D, int64_t B, int part_kind, const int32_t *owner, const float *R,
                    const int64_t *offsets, float *Out)
{
    int *n_loc = (int *)malloc(sizeof(int) * P), *loc = (int *)malloc(sizeof(int) * T), d, s, t, c;
    int64_t rbase = 0;
    if (!n_loc || !loc) { free(n_loc); free(loc); return ORC_ENOMEM; }
    local_tables(P, T, part_kind, owner, n_loc, loc);
    for (s = 0; s < P; ++s) {
        int64_t f = batch_first(B, P, s), n = batch_first(B, P, s + 1) - f, b_loc, total = 0;
        for (b_loc = 0; b_loc < n; ++b_loc)
            for (t = 0; t < T; ++t) {
                float *o = Out + ((f + b_loc) * T + t) * D;
                for (c = 0; c < D; ++c) o[c] = 0.0f;
                {
                    int64_t blk = 0;           /* start of owner d's block inside R_s */
                    for (d = 0; d < P; ++d) {
                        if (part_kind == 1 || owner[t] == d) {
                            const float *r = R + rbase + blk + ((int64_t)loc[t] * n + b_loc) * D;
                            if (part_kind == 1) for (c = 0; c < D; ++c) o[c] += r[c];
                            else memcpy(o, r, sizeof(float) * D);
                        }
                        blk += (int64_t)n_loc[d] * n * D;
                    }
                }
                if (offsets) {
                    int64_t g = (int64_t)t * B + f + b_loc, len = offsets[g + 1] - offsets[g];
                    if (len > 0) for (c = 0; c < D; ++c) o[c] /= (float)len;
                }
            }
        for (d = 0; d < P; ++d) total += (int64_t)n_loc[d] * n * D;
        rbase += total;
    }
    free(n_loc); free(loc);
    return ORC_OK;
}

/* Ordered fp32 sum and fp64 sum of n rows of length D given directly (for checking
 * single bags of workloads too large to hold on the host). */
int orc_bag_sum(int D, int64_t n, const float *rows_nd, float *out32, double *out64)
{
    int c;
    int64_t j;
    for (c = 0; c < D; ++c) {
        float a32 = 0.0f;
        double a64 = 0.0;
        for (j = 0; j < n; ++j) { a32 += rows_nd[j * D + c]; a64 += (double)rows_nd[j * D + c]; }
        if (out32) out32[c] = a32;
        if (out64) out64[c] = a64;
    }
    return ORC_OK;
}

/* ---- dense part of the model around the lookup ------------------------------------- */

#include <math.h>

#define ORC_U32 5.9604644775390625e-08 /* 2^-24, unit roundoff of fp32 */

/*
 * One layer of apply_mlp (Listings 1 and 2; the model overview in the Introduction: a
 * bottom MLP on the dense features, a top MLP that produces the prediction):
 *   y[m][n] = act( bias[n] + sum_k x[m][k] * W[n][k] ),  W stored [N][K] as a linear layer's
 * weight, act 0 = identity, 1 = ReLU, 2 = logistic sigmoid.  Everything in double.
 * The paper does not give layer sizes or activations; reading: the reference model's ReLU
 * layers with a sigmoid on the last top layer.
 *
 * err_in (nullable, [M][K]) bounds how far an fp32 implementation's input may be from x;
 * err_out (nullable, [M][N]) receives a bound for its output: the input error carried
 * through |W|, plus (K + 3) roundings of relative size 2^-24 on the sum of magnitudes, plus
 * a few units for the activation (ReLU and the sigmoid do not amplify).
 */
int orc_mlp_layer(int64_t M, int K, int N, const double *x, const float *W, const float *bias, int act,
                  const double *err_in, double *y, double *err_out)
{
    int64_t m;
    int n, k;
    if (M < 0 || K < 1 || N < 1 || act < 0 || act > 2) return ORC_EINVAL;
    for (m = 0; m < M; ++m)
        for (n = 0; n < N; ++n) {
            double acc = bias ? (double)bias[n] : 0.0;
            double mass = bias ? fabs((double)bias[n]) : 0.0, carried = 0.0, v, e;
            for (k = 0; k < K; ++k) {
                double w = (double)W[(int64_t)n * K + k], xv = x[m * K + k];
                acc += xv * w;
                mass += fabs(xv * w);
                if (err_in) { carried += fabs(w) * err_in[m * K + k]; mass += fabs(w) * err_in[m * K + k]; }
            }
            e = carried + (double)(K + 3) * ORC_U32 * mass;
            if (act == 1) v = acc > 0.0 ? acc : 0.0;
            else if (act == 2) { v = 1.0 / (1.0 + exp(-acc)); e = 0.25 * e + 8.0 * ORC_U32; }
            else v = acc;
            y[m * N + n] = v;
            if (err_out) err_out[m * N + n] = e;
        }
    return ORC_OK;
}

/*
 * interact_features (Listings 1 and 2; Introduction: the vectors are combined by a dot-product interaction layer):
 * per sample the D-vector x from the bottom MLP and the T pooled embedding vectors form
 * Z = [x; e_0; ...; e_{T-1}] ((T+1) x D); the output is x followed by the dot products
 * Z_i . Z_j for every pair i > j, ordered by i, then j (the reference model's order; the
 * diagonal is left out).  z is [B][D + T(T+1)/2], everything in double.
 * err_x / err_z as in orc_mlp_layer; the embedding vectors are taken as exact.
 */
int orc_interact(int64_t B, int T, int D, const double *x, const float *emb, const double *err_x,
                 double *z, double *err_z)
{
    int64_t b, W = (int64_t)D + (int64_t)T * (T + 1) / 2;
    int i, j, c;
    if (B < 0 || T < 1 || D < 1) return ORC_EINVAL;
    for (b = 0; b < B; ++b) {
        int64_t at = D;
        for (c = 0; c < D; ++c) {
            z[b * W + c] = x[b * D + c];
            if (err_z) err_z[b * W + c] = err_x ? err_x[b * D + c] : 0.0;
        }
        for (i = 1; i <= T; ++i)
            for (j = 0; j < i; ++j) {
                const float *ei = emb + (b * T + (i - 1)) * D;
                double dot = 0.0, mass = 0.0, carried = 0.0;
                for (c = 0; c < D; ++c) {
                    double u = (double)ei[c];
                    double v = j == 0 ? x[b * D + c] : (double)emb[(b * T + (j - 1)) * D + c];
                    dot += u * v;
                    mass += fabs(u * v);
                    if (j == 0 && err_x) { carried += fabs(u) * err_x[b * D + c]; mass += fabs(u) * err_x[b * D + c]; }
                }
                z[b * W + at] = dot;
                if (err_z) err_z[b * W + at] = carried + (double)(D + 2) * ORC_U32 * mass;
                ++at;
            }
    }
    return ORC_OK;
}


/* The 256 E4M3 codes as binary32 (for pinning the decoder on its own). */
int orc_e4m3_table(float *out256)
{
    int v;
    for (v = 0; v < 256; ++v) out256[v] = e4m3_to_float((uint8_t)v);
    return ORC_OK;
}
