// Host side of libbls: context, configuration checks, sizes, descriptor upload, the ring
// of receive buffers and the C entry points.  Kernels live in bls_plan.hip, bls_pool.hip,
// bls_permute.hip and bls_dense.hip.  Nothing here throws across the C boundary: the two places
// that allocate host containers catch and report BLS_EINVAL.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "bls_internal.h"

int bls_fail(bls_ctx *ctx, int code, const char *what)
{
    if (ctx) ctx->err = what;
    return code;
}

int bls_fail_hip(bls_ctx *ctx, hipError_t e, const char *what)
{
    if (ctx) ctx->err = std::string(what) + ": " + hipGetErrorString(e);
    return BLS_EHIP;
}

static int64_t first_of(int64_t B, int P, int s)
{
    const int64_t q = B / P, r = B % P;
    return (int64_t)s * q + std::min<int64_t>(s, r);
}

extern "C" int bls_create(const bls_config *cfg, bls_ctx **out)
{
    if (!cfg || !out) return BLS_EINVAL;
    *out = nullptr;
    if (cfg->P < 1 || cfg->P > 64 || cfg->T < 1 || cfg->D < 1 || cfg->k < 0) return BLS_EINVAL;
    if (cfg->B < cfg->P || cfg->B > 0x7fffffffLL) return BLS_EINVAL;
    if (cfg->table_dtype != BLS_FP32 && cfg->table_dtype != BLS_FP16 && cfg->table_dtype != BLS_U8_ROWQ &&
        cfg->table_dtype != BLS_F8_ROWQ)
        return BLS_EINVAL;
    if (cfg->part_kind != BLS_TABLE_WISE && cfg->part_kind != BLS_ROW_WISE) return BLS_EINVAL;
    if (!cfg->rows || (cfg->part_kind == BLS_TABLE_WISE && !cfg->table_owner)) return BLS_EINVAL;
    const int P = cfg->P, T = cfg->T;
    const int F = cfg->part_kind == BLS_ROW_WISE ? P : 1;
    if ((int64_t)F * T > 65535) return BLS_EINVAL;   // one grid row per (owner, local table)
    for (int t = 0; t < T; ++t) {
        if (cfg->rows[t] < 1) return BLS_EINVAL;
        if (cfg->part_kind == BLS_TABLE_WISE && (cfg->table_owner[t] < 0 || cfg->table_owner[t] >= P)) return BLS_EINVAL;
    }
    bls_ctx *c = new (std::nothrow) bls_ctx();
    if (!c) return BLS_EINVAL;
    try {
    c->P = P; c->T = T; c->D = cfg->D; c->k = cfg->k; c->K = std::max(cfg->k, 1); c->F = F; c->Q = F * T;
    c->dtype = cfg->table_dtype; c->part_kind = cfg->part_kind; c->B = cfg->B;
    c->rows.assign(cfg->rows, cfg->rows + T);
    c->owner.assign(T, 0);
    if (cfg->part_kind == BLS_TABLE_WISE) c->owner.assign(cfg->table_owner, cfg->table_owner + T);
    c->first.resize(P + 1);
    for (int s = 0; s <= P; ++s) c->first[s] = first_of(c->B, P, s);
    c->n_loc.assign(P, 0); c->nsum.assign(P + 1, 0); c->t_loc.assign(T, 0); c->t_q.assign(T, 0); c->rps.assign(T, 0);
    for (int t = 0; t < T; ++t) {
        if (c->part_kind == BLS_TABLE_WISE) { c->t_loc[t] = c->n_loc[c->owner[t]]++; c->rps[t] = c->rows[t]; }
        else { c->t_loc[t] = t; c->rps[t] = (c->rows[t] + P - 1) / P; }
    }
    if (c->part_kind == BLS_ROW_WISE) c->n_loc.assign(P, T);
    for (int d = 0; d < P; ++d) c->nsum[d + 1] = c->nsum[d] + c->n_loc[d];
    c->q_t.assign(c->Q, 0); c->q_d.assign(c->Q, 0); c->q_rows.assign(c->Q, 0);
    c->q_base.assign(c->Q, nullptr); c->q_set.assign(c->Q, 0); c->q_hot.assign(c->Q, std::vector<uint32_t>());
    for (int t = 0; t < T; ++t) {
        if (c->part_kind == BLS_TABLE_WISE) {
            const int q = c->nsum[c->owner[t]] + c->t_loc[t];
            c->t_q[t] = q; c->q_t[q] = t; c->q_d[q] = c->owner[t]; c->q_rows[q] = c->rows[t];
        } else {
            c->t_q[t] = t;
            for (int d = 0; d < P; ++d) {
                const int q = d * T + t;
                const int64_t lo = (int64_t)d * c->rps[t];
                c->q_t[q] = t; c->q_d[q] = d;
                c->q_rows[q] = std::max<int64_t>(0, std::min<int64_t>(c->rps[t], c->rows[t] - lo));
                if (c->q_rows[q] == 0) c->q_set[q] = 1;   // an empty shard needs no storage
            }
        }
    }
    c->nseg = c->nvec = (int64_t)c->Q * c->B;
    c->slot_bytes = (size_t)c->nvec * c->D * sizeof(float);
    c->ring.resize(c->K);
    } catch (...) {                                            // out of host memory
        delete c;
        return BLS_EINVAL;
    }
    *out = c;
    return BLS_OK;
}

extern "C" int bls_destroy(bls_ctx *ctx)
{
    if (!ctx) return BLS_EINVAL;
    if (ctx->device >= 0) {
        int cur = -1;
        if (hipGetDevice(&cur) == hipSuccess) {
            if (cur != ctx->device) (void)hipSetDevice(ctx->device);
            for (auto &r : ctx->ring) {
                if (r.filled) (void)hipEventDestroy(r.filled);
                if (r.released) (void)hipEventDestroy(r.released);
            }
            for (auto e : ctx->rr.arrived) if (e) (void)hipEventDestroy(e);
            for (auto e : ctx->rr.released) if (e) (void)hipEventDestroy(e);
            if (cur != ctx->device) (void)hipSetDevice(cur);
        }
    }
    delete ctx;
    return BLS_OK;
}

extern "C" int bls_set_shard(bls_ctx *ctx, int32_t t, int32_t rank, const void *d_rows, int64_t rows_in_shard)
{
    if (!ctx) return BLS_EINVAL;
    if (t < 0 || t >= ctx->T || rank < 0 || rank >= ctx->P) return bls_fail(ctx, BLS_EINVAL, "bls_set_shard: table or rank out of range");
    int q;
    if (ctx->part_kind == BLS_TABLE_WISE) {
        if (rank != ctx->owner[t]) return bls_fail(ctx, BLS_EINVAL, "bls_set_shard: rank is not the table's owner");
        q = ctx->t_q[t];
    } else q = rank * ctx->T + t;
    if (rows_in_shard != ctx->q_rows[q]) return bls_fail(ctx, BLS_EINVAL, "bls_set_shard: rows_in_shard does not match the partition");
    if (rows_in_shard > 0 && !d_rows) return bls_fail(ctx, BLS_EINVAL, "bls_set_shard: NULL storage for a non-empty shard");
    if (((uintptr_t)d_rows & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_set_shard: storage must be 16-byte aligned");
    if (rows_in_shard >= 0xffffffffLL) return bls_fail(ctx, BLS_EINVAL, "bls_set_shard: shard too large");
    ctx->q_base[q] = d_rows;
    ctx->q_set[q] = 1;
    ctx->dirty = true;
    return BLS_OK;
}

extern "C" int bls_shard_range(const bls_ctx *ctx, int32_t t, int32_t rank, int64_t *first_row, int64_t *rows_in_shard)
{
    if (!ctx || t < 0 || t >= ctx->T || rank < 0 || rank >= ctx->P) return BLS_EINVAL;
    int64_t lo = 0, n = 0;
    if (ctx->part_kind == BLS_TABLE_WISE) {
        if (rank == ctx->owner[t]) n = ctx->rows[t];
    } else {
        lo = std::min<int64_t>((int64_t)rank * ctx->rps[t], ctx->rows[t]);
        n = ctx->q_rows[rank * ctx->T + t];
    }
    if (first_row) *first_row = lo;
    if (rows_in_shard) *rows_in_shard = n;
    return BLS_OK;
}

extern "C" int bls_set_hot_rows(bls_ctx *ctx, int32_t t, int32_t rank, const int64_t *rows, int32_t n)
{
    if (!ctx) return BLS_EINVAL;
    if (t < 0 || t >= ctx->T || rank < 0 || rank >= ctx->P) return bls_fail(ctx, BLS_EINVAL, "bls_set_hot_rows: table or rank out of range");
    if (n < 0 || (n > 0 && !rows)) return bls_fail(ctx, BLS_EINVAL, "bls_set_hot_rows: bad list");
    int q;
    if (ctx->part_kind == BLS_TABLE_WISE) {
        if (rank != ctx->owner[t]) return bls_fail(ctx, BLS_EINVAL, "bls_set_hot_rows: rank is not the table's owner");
        q = ctx->t_q[t];
    } else q = rank * ctx->T + t;
    try {
        std::vector<uint32_t> keep;
        for (int32_t i = 0; i < n && keep.size() < (size_t)BLS_HOT_ROWS_MAX; ++i) {
            if (rows[i] < 0 || rows[i] >= ctx->q_rows[q]) return bls_fail(ctx, BLS_EINVAL, "bls_set_hot_rows: a row outside the shard");
            if (std::find(keep.begin(), keep.end(), (uint32_t)rows[i]) == keep.end()) keep.push_back((uint32_t)rows[i]);
        }
        ctx->q_hot[q].swap(keep);
    } catch (...) {
        return bls_fail(ctx, BLS_EINVAL, "out of host memory");
    }
    ctx->dirty = true;
    return BLS_OK;
}

extern "C" int bls_set_pool_tuning(bls_ctx *ctx, int32_t lane_bytes, int32_t segments_per_group, int32_t xcd_map, int32_t wide_positions)
{
    if (!ctx) return BLS_EINVAL;
    if (lane_bytes != 0 && lane_bytes != 4 && lane_bytes != 8 && lane_bytes != 16)
        return bls_fail(ctx, BLS_EINVAL, "bls_set_pool_tuning: lane_bytes must be 0, 4, 8 or 16");
    if (segments_per_group < 0 || segments_per_group > 63 || xcd_map < -1 || xcd_map > 1 || wide_positions < -1 || wide_positions > 1)
        return bls_fail(ctx, BLS_EINVAL, "bls_set_pool_tuning: value out of range");
    ctx->tune_lane_bytes = lane_bytes;
    ctx->tune_segs = segments_per_group;
    ctx->tune_xcd = xcd_map;
    ctx->tune_wide = wide_positions;
    return BLS_OK;
}

extern "C" int bls_set_plan_tuning(bls_ctx *ctx, int32_t scan_while_placing)
{
    if (!ctx) return BLS_EINVAL;
    if (scan_while_placing < -1 || scan_while_placing > 1) return bls_fail(ctx, BLS_EINVAL, "bls_set_plan_tuning: value out of range");
    ctx->tune_plan_scan = scan_while_placing;
    return BLS_OK;
}

extern "C" int bls_sizes(const bls_ctx *ctx, int64_t max_nnz, size_t *plan_ws_bytes, size_t *pooled_bytes,
                         size_t *send_bytes, size_t *slot_bytes)
{
    if (!ctx || max_nnz < 0) return BLS_EINVAL;
    if (plan_ws_bytes) *plan_ws_bytes = bls_plan_ws_bytes(ctx);
    if (pooled_bytes) *pooled_bytes = ctx->slot_bytes;
    if (send_bytes) *send_bytes = ctx->slot_bytes;
    if (slot_bytes) *slot_bytes = ctx->slot_bytes;
    return BLS_OK;
}

extern "C" int bls_pooled_counts(const bls_ctx *ctx, int64_t *pcount, int64_t *psdispl, int64_t *prcount, int64_t *prdispl)
{
    if (!ctx) return BLS_EINVAL;
    const int P = ctx->P;
    for (int d = 0; d < P; ++d) {
        int64_t run = 0;
        for (int s = 0; s < P; ++s) {
            const int64_t n = (int64_t)ctx->n_loc[d] * (ctx->first[s + 1] - ctx->first[s]) * ctx->D;
            if (pcount) pcount[d * P + s] = n;
            if (psdispl) psdispl[d * P + s] = run;
            if (prcount) prcount[s * P + d] = n;
            run += n;
        }
    }
    if (prdispl)
        for (int s = 0; s < P; ++s) {
            int64_t run = 0;
            for (int d = 0; d < P; ++d) {
                prdispl[s * P + d] = run;
                run += (int64_t)ctx->n_loc[d] * (ctx->first[s + 1] - ctx->first[s]) * ctx->D;
            }
        }
    return BLS_OK;
}

// ---- descriptor tables ---------------------------------------------------------------
// The kernels read a few small tables (mini-batch starts, tables per rank, shard pointers and
// sizes).  They live in device memory the caller provides (bls_desc_bytes / bls_commit): the
// library allocates none.  Layout: 16 bytes for the error flag, then the arrays, each on a
// 16-byte boundary.

namespace {
constexpr size_t kFlagBytes = 16;

struct BlobLayout {
    size_t first, n_loc, nsum, rows, rps, t_q, q_t, q_d, q_base, q_rows, q_deal, hot_n, hot_off, hot_rows, total;
};

size_t put(size_t &at, size_t bytes)
{
    const size_t here = (at + 15) & ~size_t(15);
    at = here + bytes;
    return here;
}

BlobLayout blob_layout(const bls_ctx *c)
{
    BlobLayout L;
    size_t at = kFlagBytes;
    const size_t P = (size_t)c->P, T = (size_t)c->T, Q = (size_t)c->Q;
    L.first = put(at, (P + 1) * sizeof(int64_t));
    L.n_loc = put(at, P * sizeof(int32_t));
    L.nsum = put(at, (P + 1) * sizeof(int32_t));
    L.rows = put(at, T * sizeof(int64_t));
    L.rps = put(at, T * sizeof(int64_t));
    L.t_q = put(at, T * sizeof(int32_t));
    L.q_t = put(at, Q * sizeof(int32_t));
    L.q_d = put(at, Q * sizeof(int32_t));
    L.q_base = put(at, Q * sizeof(void *));
    L.q_rows = put(at, Q * sizeof(int64_t));
    L.q_deal = put(at, Q * sizeof(int32_t));
    size_t hot = 0;
    for (const auto &h : c->q_hot) hot += h.size();
    L.hot_n = put(at, Q * sizeof(int32_t));
    L.hot_off = put(at, Q * sizeof(int32_t));
    L.hot_rows = put(at, hot * sizeof(uint32_t));
    L.total = (at + 15) & ~size_t(15);
    return L;
}

template <class V> void fill(std::vector<char> &blob, size_t at, const std::vector<V> &v)
{
    if (!v.empty()) memcpy(blob.data() + at, v.data(), v.size() * sizeof(V));
}
}  // namespace

size_t bls_desc_size(const bls_ctx *ctx) { return blob_layout(ctx).total; }

extern "C" int bls_desc_bytes(const bls_ctx *ctx, size_t *bytes)
{
    if (!ctx || !bytes) return BLS_EINVAL;
    *bytes = bls_desc_size(ctx);
    return BLS_OK;
}

extern "C" int bls_commit(bls_ctx *ctx, void *d_desc, size_t bytes, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    for (int q = 0; q < ctx->Q; ++q)
        if (!ctx->q_set[q]) return bls_fail(ctx, BLS_EINVAL, "bls_commit: a table shard has not been set (bls_set_shard)");
    if (!d_desc || ((uintptr_t)d_desc & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_commit: NULL or misaligned descriptor buffer");
    const BlobLayout L = blob_layout(ctx);
    if (bytes < L.total) return bls_fail(ctx, BLS_ENOSPC, "bls_commit: descriptor buffer smaller than bls_desc_bytes");
    if (ctx->head != ctx->tail) return bls_fail(ctx, BLS_EORDER, "bls_commit: iterations in flight");
    int dev = -1;
    BLS_HIP(ctx, hipGetDevice(&dev));
    if (ctx->device >= 0 && dev != ctx->device) return bls_fail(ctx, BLS_EINVAL, "context used on a different device than before");
    // a second upload: kernels of earlier calls may still read the old tables, and the earlier copy its source
    if (ctx->blob) BLS_HIP(ctx, hipDeviceSynchronize());
    try {
        ctx->host_blob.assign(L.total, 0);
    } catch (...) {
        return bls_fail(ctx, BLS_EINVAL, "out of host memory");
    }
    std::vector<char> &h = ctx->host_blob;
    fill(h, L.first, ctx->first); fill(h, L.n_loc, ctx->n_loc); fill(h, L.nsum, ctx->nsum);
    fill(h, L.rows, ctx->rows); fill(h, L.rps, ctx->rps); fill(h, L.t_q, ctx->t_q);
    fill(h, L.q_t, ctx->q_t); fill(h, L.q_d, ctx->q_d); fill(h, L.q_base, ctx->q_base); fill(h, L.q_rows, ctx->q_rows);
    {
        // The order in which a pooling launch over all shards deals them to the XCDs (position i goes to XCD
        // i % 8 in round i / 8).  By size, largest first, every other round backwards, so that no XCD collects
        // the largest shard of every round (the large ones are those whose rows miss the caches); and every XCD
        // starts at another place of its list, so that the XCDs are not all at their largest shard at once.
        std::vector<int32_t> by_size(ctx->Q), deal(ctx->Q);
        for (int q = 0; q < ctx->Q; ++q) by_size[q] = q;
        std::stable_sort(by_size.begin(), by_size.end(), [&](int32_t a, int32_t b) { return ctx->q_rows[a] > ctx->q_rows[b]; });
        std::vector<std::vector<int32_t>> mine(8);
        for (int i = 0; i < ctx->Q; ++i) {
            const int round = i / 8, j = i % 8, in_round = std::min(8, ctx->Q - round * 8);
            mine[round % 2 ? in_round - 1 - j : j].push_back(by_size[i]);
        }
        for (int x = 0; x < 8; ++x) {
            const int n = (int)mine[x].size();
            for (int k = 0; k < n; ++k) deal[k * 8 + x] = mine[x][(k + x) % n];
        }
        fill(h, L.q_deal, deal);
    }
    {
        std::vector<int32_t> hn(ctx->Q, 0), ho(ctx->Q, 0);
        size_t at = 0;
        for (int q = 0; q < ctx->Q; ++q) {
            hn[q] = (int32_t)ctx->q_hot[q].size();
            ho[q] = (int32_t)at;
            if (hn[q]) memcpy(h.data() + L.hot_rows + at * sizeof(uint32_t), ctx->q_hot[q].data(), hn[q] * sizeof(uint32_t));
            at += ctx->q_hot[q].size();
        }
        fill(h, L.hot_n, hn); fill(h, L.hot_off, ho);
    }
    BLS_HIP(ctx, hipDeviceGetAttribute(&ctx->compute_units, hipDeviceAttributeMultiprocessorCount, dev));
    // a buffer seen for the first time gets a cleared error flag; a re-upload into the same buffer
    // (a shard was replaced) leaves the flag as the kernels set it
    const size_t skip = d_desc == ctx->blob ? kFlagBytes : 0;
    BLS_HIP(ctx, hipMemcpyAsync((char *)d_desc + skip, h.data() + skip, L.total - skip, hipMemcpyHostToDevice,
                                (hipStream_t)hip_stream));
    ctx->blob = d_desc;
    ctx->device = dev;
    char *b = (char *)d_desc;
    DevDesc &d = ctx->desc;
    d.P = ctx->P; d.T = ctx->T; d.D = ctx->D; d.F = ctx->F; d.Q = ctx->Q; d.part_kind = ctx->part_kind; d.dtype = ctx->dtype;
    d.pad0 = 0; d.B = ctx->B; d.Bq = (uint32_t)(ctx->B / ctx->P); d.Br = (uint32_t)(ctx->B % ctx->P); d.nseg = ctx->nseg;
    d.err = (int32_t *)b;
    d.first = (const int64_t *)(b + L.first); d.n_loc = (const int32_t *)(b + L.n_loc); d.nsum = (const int32_t *)(b + L.nsum);
    d.rows = (const int64_t *)(b + L.rows); d.rps = (const int64_t *)(b + L.rps); d.t_q = (const int32_t *)(b + L.t_q);
    d.q_t = (const int32_t *)(b + L.q_t); d.q_d = (const int32_t *)(b + L.q_d);
    d.q_base = (const void *const *)(b + L.q_base); d.q_rows = (const int64_t *)(b + L.q_rows);
    d.q_deal = (const int32_t *)(b + L.q_deal);
    d.hot_n = (const int32_t *)(b + L.hot_n); d.hot_off = (const int32_t *)(b + L.hot_off);
    d.hot_rows = (const uint32_t *)(b + L.hot_rows);
    ctx->dirty = false;
    return BLS_OK;
}

int bls_ready(bls_ctx *ctx)
{
    if (!ctx->blob || ctx->dirty)
        return bls_fail(ctx, BLS_EINVAL, "descriptor tables not on the device: call bls_commit after the last bls_set_shard");
    return BLS_OK;
}

// ---- entry points that launch kernels -------------------------------------------------

static int plan_common(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, const float *d_weights, int64_t nnz,
                       int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts, int64_t *d_rdispls,
                       int64_t *d_ridx, float *d_rweights, int64_t *d_segoff, int64_t *d_perm, void *d_ws, size_t ws_bytes,
                       void *hip_stream)
{
    if (nnz < 0 || !d_offsets || !d_sendcounts || !d_sdispls || !d_recvcounts || !d_rdispls || !d_segoff || !d_ws)
        return bls_fail(ctx, BLS_EINVAL, "bls_plan: NULL argument or negative nnz");
    if (nnz > 0 && (!d_indices || !d_ridx)) return bls_fail(ctx, BLS_EINVAL, "bls_plan: NULL indices or ridx with nnz > 0");
    if (ws_bytes < bls_plan_ws_bytes(ctx)) return bls_fail(ctx, BLS_ENOSPC, "bls_plan: workspace too small");
    if (((uintptr_t)d_ws & 7u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_plan: workspace must be 8-byte aligned");
    int rc = bls_ready(ctx);
    if (rc) return rc;
    return bls_launch_plan(ctx, d_indices, d_offsets, nnz, d_sendcounts, d_sdispls, d_recvcounts, d_rdispls, d_ridx,
                           d_segoff, d_perm, d_weights, d_rweights, d_ws, ws_bytes, (hipStream_t)hip_stream);
}

extern "C" int bls_plan(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, int64_t nnz,
                        int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts, int64_t *d_rdispls,
                        int64_t *d_ridx, int64_t *d_segoff, int64_t *d_perm, void *d_ws, size_t ws_bytes, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    return plan_common(ctx, d_indices, d_offsets, nullptr, nnz, d_sendcounts, d_sdispls, d_recvcounts, d_rdispls, d_ridx,
                       nullptr, d_segoff, d_perm, d_ws, ws_bytes, hip_stream);
}

// ---- bls_plan without a caller workspace ---------------------------------------------------
// For callers that cannot allocate device memory: the plan's scratch (block sums of the scan, bucket
// starts) lives in a file-scope device array.  Every GPU the library runs on holds its own copy of
// the array at its own address, so the address is asked for once per device, with that device
// current, and host code only ever uses that address - never the array's name, which on the host
// is a stand-in and not a device pointer.
namespace {
constexpr size_t kStaticWsBytes = size_t(1) << 20;            // 1 MiB per device, held until the process ends
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];
void *g_scratch_ptr[kMaxDevices];                             // device address of `scratch` on device i, once known
std::mutex g_scratch_mutex;

int static_workspace(bls_ctx *ctx, void **out)
{
    int dev = -1;
    BLS_HIP(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return bls_fail(ctx, BLS_EINVAL, "bls_plan_noalloc: device number out of range");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        BLS_HIP(ctx, hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return bls_fail(ctx, BLS_EHIP, "bls_plan_noalloc: no device address for the static workspace");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return BLS_OK;
}
}  // namespace

extern "C" int bls_plan_noalloc(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, int64_t nnz,
                                int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts, int64_t *d_rdispls,
                                int64_t *d_ridx, int64_t *d_segoff, int64_t *d_perm, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (bls_plan_ws_bytes(ctx) > kStaticWsBytes)
        return bls_fail(ctx, BLS_ENOSPC, "bls_plan_noalloc: this problem needs more than the 1 MiB static workspace; use bls_plan");
    void *ws = nullptr;
    const int rc = static_workspace(ctx, &ws);
    if (rc) return rc;
    return plan_common(ctx, d_indices, d_offsets, nullptr, nnz, d_sendcounts, d_sdispls, d_recvcounts, d_rdispls, d_ridx,
                       nullptr, d_segoff, d_perm, ws, kStaticWsBytes, hip_stream);
}

extern "C" int bls_plan_weighted(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, const float *d_weights,
                                 int64_t nnz, int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts,
                                 int64_t *d_rdispls, int64_t *d_ridx, float *d_rweights, int64_t *d_segoff, int64_t *d_perm,
                                 void *d_ws, size_t ws_bytes, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (nnz > 0 && (!d_weights || !d_rweights)) return bls_fail(ctx, BLS_EINVAL, "bls_plan_weighted: NULL weights");
    return plan_common(ctx, d_indices, d_offsets, d_weights, nnz, d_sendcounts, d_sdispls, d_recvcounts, d_rdispls, d_ridx,
                       d_rweights, d_segoff, d_perm, d_ws, ws_bytes, hip_stream);
}

static int pool_common(bls_ctx *ctx, const int64_t *d_ridx, const float *d_rweights, const int64_t *d_segoff, int64_t nnz,
                       float *d_pooled, void *hip_stream)
{
    if (nnz < 0 || !d_segoff || !d_pooled || (nnz > 0 && !d_ridx)) return bls_fail(ctx, BLS_EINVAL, "bls_embbag_pool: NULL argument");
    if (((uintptr_t)d_pooled & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_embbag_pool: output must be 16-byte aligned");
    int rc = bls_ready(ctx);
    if (rc) return rc;
    return bls_launch_pool(ctx, d_ridx, d_rweights, d_segoff, nnz, d_pooled, 0, 0, ctx->Q, (hipStream_t)hip_stream);
}

extern "C" int bls_embbag_pool(bls_ctx *ctx, const int64_t *d_ridx, const int64_t *d_segoff, int64_t nnz,
                               float *d_pooled, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    return pool_common(ctx, d_ridx, nullptr, d_segoff, nnz, d_pooled, hip_stream);
}

extern "C" int bls_embbag_pool_weighted(bls_ctx *ctx, const int64_t *d_ridx, const float *d_rweights, const int64_t *d_segoff,
                                        int64_t nnz, float *d_pooled, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (nnz > 0 && !d_rweights) return bls_fail(ctx, BLS_EINVAL, "bls_embbag_pool_weighted: NULL weights");
    return pool_common(ctx, d_ridx, nnz > 0 ? d_rweights : nullptr, d_segoff, nnz, d_pooled, hip_stream);
}

extern "C" int bls_pack(bls_ctx *ctx, const float *d_pooled, float *d_send, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (!d_pooled || !d_send || d_pooled == d_send) return bls_fail(ctx, BLS_EINVAL, "bls_pack: NULL or aliased buffers");
    if ((((uintptr_t)d_pooled | (uintptr_t)d_send) & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_pack: buffers must be 16-byte aligned");
    int rc = bls_ready(ctx);
    if (rc) return rc;
    return bls_launch_pack(ctx, d_pooled, d_send, (hipStream_t)hip_stream);
}

// ---- ring -------------------------------------------------------------------------------

extern "C" int bls_set_ring(bls_ctx *ctx, void *d_slots, size_t bytes)
{
    if (!ctx) return BLS_EINVAL;
    if (!d_slots || ((uintptr_t)d_slots & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_set_ring: NULL or misaligned ring");
    if (bytes < (size_t)ctx->K * ctx->slot_bytes) return bls_fail(ctx, BLS_ENOSPC, "bls_set_ring: ring smaller than K slots");
    if (ctx->head != ctx->tail) return bls_fail(ctx, BLS_EORDER, "bls_set_ring: iterations in flight");
    ctx->slots = (char *)d_slots;
    return BLS_OK;
}

extern "C" int bls_ring_state(const bls_ctx *ctx, int64_t *head, int64_t *tail, int32_t *K)
{
    if (!ctx) return BLS_EINVAL;
    if (head) *head = ctx->head;
    if (tail) *tail = ctx->tail;
    if (K) *K = ctx->K;
    return BLS_OK;
}

extern "C" int bls_ring_advance(bls_ctx *ctx, int64_t *iter_out, int32_t *slot_out, void *hip_stream)
{
    if (!ctx || !iter_out || !slot_out) return BLS_EINVAL;
    if (ctx->head - ctx->tail >= ctx->K) return bls_fail(ctx, BLS_ERING_FULL, "bls_ring_advance: K iterations in flight");
    for (int r = 0; r < (int)ctx->rr.put_next.size(); ++r)
        if (ctx->rr.put_next[r] != ctx->rr.done_next[r] || ctx->rr.put_next[r] != ctx->rr.put_next[0])
            return bls_fail(ctx, BLS_EORDER, "bls_ring_advance: per-rank iterations are in flight on this context");
    const int64_t j = ctx->head;
    const int slot = (int)(j % ctx->K);
    RingSlot &r = ctx->ring[slot];
    if (r.has_released && r.released_on != (hipStream_t)hip_stream)   // the stream that refills the slot must see the earlier copy-out finished
        BLS_HIP(ctx, hipStreamWaitEvent((hipStream_t)hip_stream, r.released, 0));
    r.state = 1;
    r.iter = j;
    ctx->head = j + 1;
    *iter_out = j;
    *slot_out = slot;
    return BLS_OK;
}


static int ensure_events(bls_ctx *ctx, RingSlot &r)
{
    if (!r.filled) BLS_HIP(ctx, hipEventCreateWithFlags(&r.filled, hipEventDisableTiming));
    if (!r.released) BLS_HIP(ctx, hipEventCreateWithFlags(&r.released, hipEventDisableTiming));
    return BLS_OK;
}

// The slot must be the one handed out by the latest bls_ring_advance and still be empty.
static int slot_to_fill(bls_ctx *ctx, int32_t slot, const char *who, RingSlot **out)
{
    if (!ctx->slots) return bls_fail(ctx, BLS_EINVAL, "no ring (bls_set_ring)");
    if (slot < 0 || slot >= ctx->K) return bls_fail(ctx, BLS_EINVAL, "slot out of range");
    RingSlot &r = ctx->ring[slot];
    if (r.state != 1 || r.iter != ctx->head - 1) {
        ctx->err = std::string(who) + ": slot does not belong to the iteration just started";
        return BLS_EORDER;
    }
    int rc = bls_ready(ctx);
    if (rc) return rc;
    rc = ensure_events(ctx, r);
    if (rc) return rc;
    *out = &r;
    return BLS_OK;
}

extern "C" int bls_alltoallv_local(bls_ctx *ctx, const float *d_send, int32_t slot, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (!d_send || ((uintptr_t)d_send & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_alltoallv_local: NULL or misaligned send buffer");
    RingSlot *r = nullptr;
    int rc = slot_to_fill(ctx, slot, "bls_alltoallv_local", &r);
    if (rc) return rc;
    rc = bls_launch_exchange(ctx, d_send, (float *)(ctx->slots + (size_t)slot * ctx->slot_bytes), (hipStream_t)hip_stream);
    if (rc) return rc;
    BLS_HIP(ctx, hipEventRecord(r->filled, (hipStream_t)hip_stream));
    r->filled_on = (hipStream_t)hip_stream;
    r->state = 2;
    return BLS_OK;
}

static int put_common(bls_ctx *ctx, const int64_t *d_ridx, const float *d_rweights, const int64_t *d_segoff, int64_t nnz,
                      int32_t slot, void *hip_stream)
{
    if (nnz < 0 || !d_segoff || (nnz > 0 && !d_ridx)) return bls_fail(ctx, BLS_EINVAL, "bls_embbag_pool_put: NULL argument");
    RingSlot *r = nullptr;
    int rc = slot_to_fill(ctx, slot, "bls_embbag_pool_put", &r);
    if (rc) return rc;
    rc = bls_launch_pool(ctx, d_ridx, d_rweights, d_segoff, nnz, (float *)(ctx->slots + (size_t)slot * ctx->slot_bytes), 1,
                         0, ctx->Q, (hipStream_t)hip_stream);
    if (rc) return rc;
    BLS_HIP(ctx, hipEventRecord(r->filled, (hipStream_t)hip_stream));
    r->filled_on = (hipStream_t)hip_stream;
    r->state = 2;
    return BLS_OK;
}

extern "C" int bls_embbag_pool_put(bls_ctx *ctx, const int64_t *d_ridx, const int64_t *d_segoff, int64_t nnz,
                                   int32_t slot, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    return put_common(ctx, d_ridx, nullptr, d_segoff, nnz, slot, hip_stream);
}

extern "C" int bls_embbag_pool_put_weighted(bls_ctx *ctx, const int64_t *d_ridx, const float *d_rweights,
                                            const int64_t *d_segoff, int64_t nnz, int32_t slot, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (nnz > 0 && !d_rweights) return bls_fail(ctx, BLS_EINVAL, "bls_embbag_pool_put_weighted: NULL weights");
    return put_common(ctx, d_ridx, nnz > 0 ? d_rweights : nullptr, d_segoff, nnz, slot, hip_stream);
}

static int unpack_common(bls_ctx *ctx, int64_t iter, const int64_t *mean_off, float *d_out, void *hip_stream)
{
    if (ctx->head == ctx->tail) return bls_fail(ctx, BLS_ERING_EMPTY, "bls_unpack: nothing in flight");
    if (iter != ctx->tail) return bls_fail(ctx, BLS_EORDER, "bls_unpack: not the oldest iteration in flight");
    if (!d_out || ((uintptr_t)d_out & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_unpack: NULL or misaligned output");
    const int slot = (int)(iter % ctx->K);
    RingSlot &r = ctx->ring[slot];
    if (r.state != 2) return bls_fail(ctx, BLS_EORDER, "bls_unpack: the iteration's exchange has not been issued");
    int rc = bls_ready(ctx);
    if (rc) return rc;
    if (r.filled_on != (hipStream_t)hip_stream) BLS_HIP(ctx, hipStreamWaitEvent((hipStream_t)hip_stream, r.filled, 0));
    rc = bls_launch_unpack(ctx, (const float *)(ctx->slots + (size_t)slot * ctx->slot_bytes), d_out, mean_off, 0u,
                           (uint32_t)ctx->B, (hipStream_t)hip_stream);
    if (rc) return rc;
    BLS_HIP(ctx, hipEventRecord(r.released, (hipStream_t)hip_stream));
    r.released_on = (hipStream_t)hip_stream;
    r.has_released = true;
    r.state = 0;
    ctx->tail = iter + 1;
    return BLS_OK;
}

extern "C" int bls_unpack(bls_ctx *ctx, int64_t iter, float *d_out, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    return unpack_common(ctx, iter, nullptr, d_out, hip_stream);
}

extern "C" int bls_unpack_mean(bls_ctx *ctx, int64_t iter, const int64_t *d_offsets, float *d_out, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (!d_offsets) return bls_fail(ctx, BLS_EINVAL, "bls_unpack_mean: NULL offsets");
    return unpack_common(ctx, iter, d_offsets, d_out, hip_stream);
}

// ---- a whole synchronous iteration in one launch (table-wise partitions) ------------------------

extern "C" int bls_step_tablewise(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, int64_t nnz,
                                  int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts, int64_t *d_rdispls,
                                  int64_t *d_ridx, int64_t *d_segoff, int64_t *d_perm, float *d_pooled, float *d_send,
                                  float *d_out, int64_t *iter_out, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (nnz < 0 || !d_offsets || !d_sendcounts || !d_sdispls || !d_recvcounts || !d_rdispls || !d_segoff || !d_pooled ||
        !d_send || !d_out || (nnz > 0 && (!d_indices || !d_ridx)))
        return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: NULL argument or negative nnz");
    if ((((uintptr_t)d_pooled | (uintptr_t)d_send | (uintptr_t)d_out) & 15u) != 0)
        return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: vector buffers must be 16-byte aligned");
    if (d_pooled == d_send || d_pooled == d_out || d_send == d_out) return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: aliased buffers");
    if (!ctx->slots) return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: no ring (bls_set_ring)");
    if (ctx->head != ctx->tail) return bls_fail(ctx, BLS_EORDER, "bls_step_tablewise: iterations in flight");
    for (int r = 0; r < (int)ctx->rr.put_next.size(); ++r)
        if (ctx->rr.put_next[r] != ctx->rr.done_next[r] || ctx->rr.put_next[r] != ctx->rr.put_next[0])
            return bls_fail(ctx, BLS_EORDER, "bls_step_tablewise: per-rank iterations are in flight on this context");
    int rc = bls_ready(ctx);
    if (rc) return rc;
    const int64_t j = ctx->head;
    const int slot = (int)(j % ctx->K);
    RingSlot &r = ctx->ring[slot];
    rc = ensure_events(ctx, r);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    if (r.has_released && r.released_on != st) BLS_HIP(ctx, hipStreamWaitEvent(st, r.released, 0));
    rc = bls_launch_step_tablewise(ctx, d_indices, d_offsets, nnz, d_sendcounts, d_sdispls, d_recvcounts, d_rdispls, d_ridx,
                                   d_segoff, d_perm, d_pooled, d_send, (float *)(ctx->slots + (size_t)slot * ctx->slot_bytes),
                                   d_out, st);
    if (rc) return rc;
    BLS_HIP(ctx, hipEventRecord(r.released, st));             // the slot is free again once this launch has run
    r.released_on = st;
    r.has_released = true;
    r.state = 0;
    r.iter = j;
    ctx->head = ctx->tail = j + 1;
    if (iter_out) *iter_out = j;
    return BLS_OK;
}

// ---- per-rank issue and completion -----------------------------------------------------------

static int rank_ring_init(bls_ctx *ctx)
{
    RankRing &rr = ctx->rr;
    if (!rr.arrived.empty()) return BLS_OK;
    const size_t n = (size_t)ctx->K * ctx->P;
    try {
        rr.put_next.assign(ctx->P, 0);
        rr.done_next.assign(ctx->P, 0);
        rr.has_arrived.assign(n, 0);
        rr.has_released.assign(n, 0);
        rr.arrived_on.assign(n, nullptr);
        rr.released_on.assign(n, nullptr);
        rr.released.assign(n, nullptr);
        rr.arrived.assign(n, nullptr);                         // last: its size marks the ring as set up
    } catch (...) {
        rr.arrived.clear();
        return bls_fail(ctx, BLS_EINVAL, "out of host memory");
    }
    for (size_t i = 0; i < n; ++i) {
        BLS_HIP(ctx, hipEventCreateWithFlags(&rr.arrived[i], hipEventDisableTiming));
        BLS_HIP(ctx, hipEventCreateWithFlags(&rr.released[i], hipEventDisableTiming));
    }
    return BLS_OK;
}

extern "C" int bls_rank_put(bls_ctx *ctx, int32_t rank, const int64_t *d_ridx, const float *d_rweights,
                            const int64_t *d_segoff, int64_t nnz, int64_t iter, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (rank < 0 || rank >= ctx->P) return bls_fail(ctx, BLS_EINVAL, "bls_rank_put: rank out of range");
    if (nnz < 0 || !d_segoff || (nnz > 0 && !d_ridx)) return bls_fail(ctx, BLS_EINVAL, "bls_rank_put: NULL argument");
    if (!ctx->slots) return bls_fail(ctx, BLS_EINVAL, "bls_rank_put: no ring (bls_set_ring)");
    if (ctx->head != ctx->tail) return bls_fail(ctx, BLS_EORDER, "bls_rank_put: whole-batch iterations are in flight on this context");
    int rc = bls_ready(ctx);
    if (rc) return rc;
    rc = rank_ring_init(ctx);
    if (rc) return rc;
    RankRing &rr = ctx->rr;
    if (iter != rr.put_next[rank]) return bls_fail(ctx, BLS_EORDER, "bls_rank_put: not this rank's next iteration");
    // the slot is free again only when every requester has copied iteration iter - K out of it
    for (int s = 0; s < ctx->P; ++s)
        if (iter - rr.done_next[s] >= ctx->K) return bls_fail(ctx, BLS_ERING_FULL, "bls_rank_put: a requester still holds the slot");
    const int slot = (int)(iter % ctx->K);
    hipStream_t st = (hipStream_t)hip_stream;
    for (int s = 0; s < ctx->P; ++s)
        if (rr.has_released[(size_t)slot * ctx->P + s] && rr.released_on[(size_t)slot * ctx->P + s] != st)
            BLS_HIP(ctx, hipStreamWaitEvent(st, rr.released[(size_t)slot * ctx->P + s], 0));
    rc = bls_launch_pool(ctx, d_ridx, nnz > 0 ? d_rweights : nullptr, d_segoff, nnz,
                         (float *)(ctx->slots + (size_t)slot * ctx->slot_bytes), 1, ctx->nsum[rank], ctx->n_loc[rank], st);
    if (rc) return rc;
    BLS_HIP(ctx, hipEventRecord(rr.arrived[(size_t)slot * ctx->P + rank], st));
    rr.has_arrived[(size_t)slot * ctx->P + rank] = 1;
    rr.arrived_on[(size_t)slot * ctx->P + rank] = st;
    rr.put_next[rank] = iter + 1;
    return BLS_OK;
}

extern "C" int bls_rank_complete(bls_ctx *ctx, int32_t rank, int64_t iter, const int64_t *d_mean_offsets, float *d_out,
                                 void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (rank < 0 || rank >= ctx->P) return bls_fail(ctx, BLS_EINVAL, "bls_rank_complete: rank out of range");
    if (!d_out || ((uintptr_t)d_out & 15u) != 0) return bls_fail(ctx, BLS_EINVAL, "bls_rank_complete: NULL or misaligned output");
    RankRing &rr = ctx->rr;
    if (rr.arrived.empty()) return bls_fail(ctx, BLS_ERING_EMPTY, "bls_rank_complete: nothing in flight");
    if (iter != rr.done_next[rank]) return bls_fail(ctx, BLS_EORDER, "bls_rank_complete: not this rank's oldest iteration");
    for (int d = 0; d < ctx->P; ++d)
        if (rr.put_next[d] <= iter)
            return bls_fail(ctx, BLS_EORDER, "bls_rank_complete: an owner has not issued this iteration yet");
    const int slot = (int)(iter % ctx->K);
    hipStream_t st = (hipStream_t)hip_stream;
    // completion = the blocks of all P owners have arrived (the paper polls a tag counter for this)
    for (int d = 0; d < ctx->P; ++d)
        if (rr.arrived_on[(size_t)slot * ctx->P + d] != st) BLS_HIP(ctx, hipStreamWaitEvent(st, rr.arrived[(size_t)slot * ctx->P + d], 0));
    int rc = bls_launch_unpack(ctx, (const float *)(ctx->slots + (size_t)slot * ctx->slot_bytes), d_out, d_mean_offsets,
                               (uint32_t)ctx->first[rank], (uint32_t)(ctx->first[rank + 1] - ctx->first[rank]), st);
    if (rc) return rc;
    BLS_HIP(ctx, hipEventRecord(rr.released[(size_t)slot * ctx->P + rank], st));
    rr.has_released[(size_t)slot * ctx->P + rank] = 1;
    rr.released_on[(size_t)slot * ctx->P + rank] = st;
    rr.done_next[rank] = iter + 1;
    return BLS_OK;
}

extern "C" int bls_rank_delay(bls_ctx *ctx, uint32_t microseconds, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (microseconds > 1000000u) return bls_fail(ctx, BLS_EINVAL, "bls_rank_delay: at most one second");
    return bls_launch_delay(ctx, microseconds, (hipStream_t)hip_stream);
}

extern "C" int bls_mlp_layer(bls_ctx *ctx, const float *d_x, int64_t M, int32_t K, const float *d_W, const float *d_bias,
                             int32_t N, int32_t act, float *d_y, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (M < 0 || K < 1 || N < 1 || K > 0x7fffffff / 128 || N > 0x7fffffff / 128)
        return bls_fail(ctx, BLS_EINVAL, "bls_mlp_layer: bad shape");
    if (act != BLS_ACT_NONE && act != BLS_ACT_RELU && act != BLS_ACT_SIGMOID)
        return bls_fail(ctx, BLS_EINVAL, "bls_mlp_layer: unknown activation");
    if (M > 0 && (!d_x || !d_W || !d_y)) return bls_fail(ctx, BLS_EINVAL, "bls_mlp_layer: NULL array");
    return bls_launch_mlp_layer(ctx, d_x, M, K, d_W, d_bias, N, act, d_y, (hipStream_t)hip_stream);
}

extern "C" int bls_interact(bls_ctx *ctx, const float *d_x, const float *d_emb, float *d_z, int64_t b0, int64_t bn,
                            void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (b0 < 0 || bn < 0 || b0 + bn > ctx->B) return bls_fail(ctx, BLS_EINVAL, "bls_interact: samples outside the batch");
    if (bls_interact_lds_bytes(ctx->T, ctx->D) > 64 * 1024)
        return bls_fail(ctx, BLS_EINVAL, "bls_interact: the pooled vectors of one sample do not fit in 64 KB of LDS");
    if (bn > 0 && (!d_x || !d_emb || !d_z)) return bls_fail(ctx, BLS_EINVAL, "bls_interact: NULL array");
    return bls_launch_interact(ctx, d_x, d_emb, 0, d_z, (uint32_t)b0, (uint32_t)bn, (hipStream_t)hip_stream);
}

extern "C" int bls_unpack_interact(bls_ctx *ctx, int64_t iter, const float *d_x, float *d_z, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    if (ctx->head == ctx->tail) return bls_fail(ctx, BLS_ERING_EMPTY, "bls_unpack_interact: nothing in flight");
    if (iter != ctx->tail) return bls_fail(ctx, BLS_EORDER, "bls_unpack_interact: not the oldest iteration in flight");
    if (!d_x || !d_z) return bls_fail(ctx, BLS_EINVAL, "bls_unpack_interact: NULL array");
    if (bls_interact_lds_bytes(ctx->T, ctx->D) > 64 * 1024)
        return bls_fail(ctx, BLS_EINVAL, "bls_unpack_interact: the pooled vectors of one sample do not fit in 64 KB of LDS");
    const int slot = (int)(iter % ctx->K);
    RingSlot &r = ctx->ring[slot];
    if (r.state != 2) return bls_fail(ctx, BLS_EORDER, "bls_unpack_interact: the iteration's exchange has not been issued");
    int rc = bls_ready(ctx);
    if (rc) return rc;
    if (r.filled_on != (hipStream_t)hip_stream) BLS_HIP(ctx, hipStreamWaitEvent((hipStream_t)hip_stream, r.filled, 0));
    rc = bls_launch_interact(ctx, d_x, (const float *)(ctx->slots + (size_t)slot * ctx->slot_bytes), 1, d_z, 0u, (uint32_t)ctx->B,
                             (hipStream_t)hip_stream);
    if (rc) return rc;
    BLS_HIP(ctx, hipEventRecord(r.released, (hipStream_t)hip_stream));
    r.released_on = (hipStream_t)hip_stream;
    r.has_released = true;
    r.state = 0;
    ctx->tail = iter + 1;
    return BLS_OK;
}

extern "C" int bls_check(bls_ctx *ctx, void *hip_stream)
{
    if (!ctx) return BLS_EINVAL;
    BLS_HIP(ctx, hipStreamSynchronize((hipStream_t)hip_stream));
    if (!ctx->blob) return BLS_OK;
    int32_t flag = 0;
    BLS_HIP(ctx, hipMemcpy(&flag, ctx->desc.err, sizeof(flag), hipMemcpyDeviceToHost));
    if (flag) {
        int32_t zero = 0;
        BLS_HIP(ctx, hipMemcpy(ctx->desc.err, &zero, sizeof(zero), hipMemcpyHostToDevice));
        return bls_fail(ctx, BLS_ERANGE, "a kernel skipped an out-of-range index, offset or segment");
    }
    return BLS_OK;
}

extern "C" const char *bls_last_error(const bls_ctx *ctx)
{
    return ctx ? ctx->err.c_str() : "NULL context";
}
