// bls_step_tablewise: a whole synchronous iteration of a table-wise partition in one launch.
//
// Small batches spend their time in the hand-over between the seven to ten dependent kernels of
// the staged calls, not in the kernels.  With whole tables per rank nothing in the path depends on
// a pass over all lookups: a run (q, s) - the bags of one table in one rank's mini-batch - keeps
// its input order on the owner's side, so its place there follows from the run lengths alone, and
// those are differences of the offsets at the run edges.  Every workgroup reads the run edges for
// itself (a few hundred values out of L2), scans them in LDS, and then works on its own bags:
// segment start, the lookups' places in ridx and perm, the pooled vector, and that vector stored
// four times - pooled buffer, send region, receive region of the ring slot, output - each at its
// closed-form address.  Bit for bit what bls_plan, bls_embbag_pool, bls_pack, bls_alltoallv_local
// and bls_unpack leave behind.
#include <algorithm>

#include "bls_internal.h"
#include "bls_rows.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxRuns = 2048;                 // runs (q, s) whose starts one workgroup scans in LDS
constexpr int kPerThread = kMaxRuns / kThreads;
constexpr int kU = 8;                          // independent row loads per lane before the first add

__device__ __forceinline__ void flag_error(const DevDesc &dd) { atomicOr(dd.err, 1); }

__device__ __forceinline__ int64_t wave_inclusive_scan(int64_t v, int lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int64_t u = __shfl_up(v, o, 64);
        if (lane >= o) v += u;
    }
    return v;
}

// Position of run (q, s) in owner order (d, s, local table): the order of the owner-side blocks.
__device__ __forceinline__ int run_entry(const DevDesc &dd, int q, int s)
{
    const int d = dd.q_d[q];
    return dd.nsum[d] * dd.P + s * dd.n_loc[d] + (q - dd.nsum[d]);
}

// grid: x over (requester s, chunk of its mini-batch), y = q.  G lanes per bag, 16 bytes of a row per lane.
template <int G, int DT>
__global__ __launch_bounds__(kThreads) void step_tablewise(DevDesc dd, const int64_t *__restrict__ idx,
                                                           const int64_t *__restrict__ off, int64_t nnz,
                                                           int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                           int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                           int64_t *__restrict__ ridx, int64_t *__restrict__ segoff,
                                                           int64_t *__restrict__ perm, float *__restrict__ Y,
                                                           float *__restrict__ S, float *__restrict__ R,
                                                           float *__restrict__ out, uint32_t chunks)
{
    using A = Acc<DT, 16>;
    __shared__ int64_t rb[kMaxRuns + 1];       // run lengths in owner order, then their exclusive scan
    __shared__ int64_t part[kWaves];
    __shared__ int64_t red[kWaves];
    const int P = dd.P, nruns = dd.Q * P;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;

    // 1. run lengths from the offsets at the run edges, scanned in owner order
    for (int i = threadIdx.x; i < kMaxRuns + 1; i += kThreads) rb[i] = 0;
    __syncthreads();
    bool bad_edges = false;
    for (int i = threadIdx.x; i < nruns; i += kThreads) {
        const int q = i / P, s = i - q * P;
        const int64_t g0 = (int64_t)dd.q_t[q] * dd.B;
        const int64_t lo = off[g0 + dd.first[s]], hi = off[g0 + dd.first[s + 1]];
        int64_t len = hi - lo;
        if (lo < 0 || hi > nnz || len < 0) { bad_edges = true; len = 0; }
        rb[run_entry(dd, q, s)] = len;
    }
    if (bad_edges) flag_error(dd);
    __syncthreads();
    {
        int64_t x[kPerThread], run = 0;
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) { x[k] = run; run += rb[threadIdx.x * kPerThread + k]; }
        const int64_t inc = wave_inclusive_scan(run, lane);
        if (lane == 63) part[wv] = inc;
        __syncthreads();
        int64_t before = inc - run;
        for (int w = 0; w < wv; ++w) before += part[w];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) rb[threadIdx.x * kPerThread + k] = x[k] + before;
        if (threadIdx.x == kThreads - 1) rb[kMaxRuns] = before + run;
    }
    __syncthreads();
    const int64_t placed = rb[kMaxRuns];                      // runs past nruns are empty: this is the total
    auto edge = [&](int d, int s) -> int64_t {                // start of the owner-side block (d, s); (P, 0) is the end
        return d >= P ? placed : rb[dd.nsum[d] * P + s * dd.n_loc[d]];
    };
    auto count = [&](int s, int d) -> int64_t {               // lookups rank s asks of rank d
        return (s + 1 < P ? edge(d, s + 1) : edge(d + 1, 0)) - edge(d, s);
    };

    // 2. the alltoallv counts and displacements, by the first workgroup
    if (blockIdx.x == 0 && blockIdx.y == 0) {
        for (int e = threadIdx.x; e < P * P; e += kThreads) {
            const int d = e / P, s = e - d * P;
            recvcounts[d * P + s] = count(s, d);
            sendcounts[s * P + d] = count(s, d);
            rdispls[d * P + s] = edge(d, s) - edge(d, 0);
            int64_t run = 0;
            for (int dd2 = 0; dd2 < d; ++dd2) run += count(s, dd2);
            sdispls[s * P + d] = run;
        }
        if (threadIdx.x == 0) segoff[dd.nseg] = placed;
    }

    // 3. this workgroup's bags: samples of requester s, table q
    const int q = blockIdx.y;
    const int s = (int)(blockIdx.x / chunks);
    const uint32_t chunk = blockIdx.x - (uint32_t)s * chunks;
    const int t = dd.q_t[q], d = dd.q_d[q];
    const int64_t f = dd.first[s], n = dd.first[s + 1] - f;
    const int64_t g0 = (int64_t)t * dd.B + f;
    int64_t lo_run = off[g0], hi_run = off[g0 + n];
    if (lo_run < 0 || hi_run > nnz || hi_run < lo_run) lo_run = hi_run = 0;   // flagged above; the run counts as empty
    const int64_t dst = rb[run_entry(dd, q, s)];
    // owner-side place -> requester-side place of the run's lookups: start of bucket (s, d) in requester
    // order minus its start in owner order.  The requester-side start adds up every count of an
    // earlier requester and this requester's counts for earlier owners.
    int64_t to_send = 0;
    if (perm) {
        int64_t a = 0;
        for (int e = threadIdx.x; e < P * P; e += kThreads) {
            const int sp = e / P, dp = e - sp * P;
            if (sp < s || (sp == s && dp < d)) a += count(sp, dp);
        }
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) a += __shfl_xor(a, sh, 64);
        if (lane == 0) red[wv] = a;
        __syncthreads();
        for (int w = 0; w < kWaves; ++w) to_send += red[w];
        to_send -= edge(d, s);
    }

    const int li = threadIdx.x & (G - 1);
    const int gbase = lane & ~(G - 1);
    const int64_t b_loc = (int64_t)chunk * (kThreads / G) + threadIdx.x / G;
    const bool live = b_loc < n;
    const uint32_t row_bytes = (uint32_t)payload_bytes(DT, dd.D), row_stride = (uint32_t)stride_bytes(DT, dd.D);
    const bool col_ok = (uint32_t)li * 16 < row_bytes;        // lanes past the row's end idle
    const char *__restrict__ base = (const char *)dd.q_base[q] + (col_ok ? (uint32_t)li * 16 : 0u);
    const int tail = (int)row_bytes - (col_ok ? li * 16 : 0);
    const int64_t rows = dd.q_rows[q], run_len = hi_run - lo_run;

    int64_t beg = 0, len = 0, place = 0;
    if (live) {
        beg = off[g0 + b_loc];
        const int64_t end = off[g0 + b_loc + 1];
        len = end - beg;
        int64_t at = beg - lo_run;
        if (at < 0 || at > run_len || len < 0 || at + len > run_len) {   // a bag outside its run: treated as empty
            if (li == 0) flag_error(dd);
            at = at < 0 ? 0 : (at > run_len ? run_len : at);
            len = 0;
        }
        place = dst + at;
        const int64_t sg = (int64_t)dd.nsum[d] * dd.B + (int64_t)dd.n_loc[d] * f + (int64_t)(q - dd.nsum[d]) * n + b_loc;
        if (li == 0) segoff[sg] = place;
        if (place < 0 || place + len > nnz) { if (li == 0) flag_error(dd); len = 0; }
    }

    A acc;
    acc.zero();
    int64_t ahead = li < len ? idx[beg + li] : -1;            // a block's row numbers are asked for one block early
    for (int64_t c0 = 0; __any(c0 < len); c0 += G) {
        const int64_t left = len - c0;
        const int rem = left < 0 ? 0 : (left > G ? G : (int)left);
        int64_t mine = -1;
        const int64_t got = ahead;
        ahead = c0 + G + li < len ? idx[beg + c0 + G + li] : -1;
        if (li < rem) {
            mine = got;
            if (mine < 0 || mine >= rows) { flag_error(dd); mine = -1; }       // adds nothing to the bag
            ridx[place + c0 + li] = mine;
            if (perm) perm[beg + c0 + li] = place + c0 + li + to_send;
        }
        for (int j = 0; __any(j < rem); j += kU) {
            int64_t r[kU];
            typename A::Raw v[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) r[u] = __shfl(mine, gbase + ((j + u) & (G - 1)), 64);
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                v[u] = A::none();
                if (j + u < rem && r[u] >= 0) v[u] = A::load(base + (uint64_t)r[u] * row_stride, tail);
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) acc.add(v[u]);       // adding +0 for the rows not there changes nothing
        }
    }
    if (live && col_ok) {
        const int64_t b = f + b_loc;
        const int64_t sg = (int64_t)dd.nsum[d] * dd.B + (int64_t)dd.n_loc[d] * f + (int64_t)(q - dd.nsum[d]) * n + b_loc;
        const int64_t rho = (int64_t)dd.Q * f + (int64_t)q * n + b_loc;
        acc.store(Y + ((int64_t)q * dd.B + b) * dd.D + li * A::NV);
        acc.store(S + sg * dd.D + li * A::NV);
        acc.store(R + rho * dd.D + li * A::NV);
        acc.store(out + (b * dd.T + t) * dd.D + li * A::NV);
    }
}

template <int DT>
bool dispatch(const bls_ctx *ctx, int lanes, dim3 grid, hipStream_t st, const int64_t *idx, const int64_t *off, int64_t nnz,
              int64_t *sc, int64_t *sd, int64_t *rc, int64_t *rd, int64_t *ridx, int64_t *segoff, int64_t *perm, float *Y,
              float *S, float *R, float *out, uint32_t chunks)
{
    switch (lanes) {
    case 1: step_tablewise<1, DT><<<grid, kThreads, 0, st>>>(ctx->desc, idx, off, nnz, sc, sd, rc, rd, ridx, segoff, perm, Y, S, R, out, chunks); return true;
    case 2: step_tablewise<2, DT><<<grid, kThreads, 0, st>>>(ctx->desc, idx, off, nnz, sc, sd, rc, rd, ridx, segoff, perm, Y, S, R, out, chunks); return true;
    case 4: step_tablewise<4, DT><<<grid, kThreads, 0, st>>>(ctx->desc, idx, off, nnz, sc, sd, rc, rd, ridx, segoff, perm, Y, S, R, out, chunks); return true;
    case 8: step_tablewise<8, DT><<<grid, kThreads, 0, st>>>(ctx->desc, idx, off, nnz, sc, sd, rc, rd, ridx, segoff, perm, Y, S, R, out, chunks); return true;
    case 16: step_tablewise<16, DT><<<grid, kThreads, 0, st>>>(ctx->desc, idx, off, nnz, sc, sd, rc, rd, ridx, segoff, perm, Y, S, R, out, chunks); return true;
    case 32: step_tablewise<32, DT><<<grid, kThreads, 0, st>>>(ctx->desc, idx, off, nnz, sc, sd, rc, rd, ridx, segoff, perm, Y, S, R, out, chunks); return true;
    case 64: step_tablewise<64, DT><<<grid, kThreads, 0, st>>>(ctx->desc, idx, off, nnz, sc, sd, rc, rd, ridx, segoff, perm, Y, S, R, out, chunks); return true;
    }
    return false;
}

}  // namespace

// BLS_EINVAL (and nothing launched) when the problem is not one this kernel takes: a row-wise
// partition, rows that 64 lanes of 16 bytes do not cover evenly, more than kMaxRuns runs.
int bls_launch_step_tablewise(bls_ctx *ctx, const int64_t *idx, const int64_t *off, int64_t nnz, int64_t *sendcounts,
                              int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls, int64_t *ridx, int64_t *segoff,
                              int64_t *perm, float *Y, float *S, float *R, float *out, hipStream_t st)
{
    if (ctx->part_kind != BLS_TABLE_WISE) return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: the partition is row-wise");
    const int64_t row_bytes = payload_bytes(ctx->dtype, ctx->D);
    if (row_bytes % 16 != 0 || row_bytes > 64 * 16 || (int64_t)ctx->Q * ctx->P > kMaxRuns)
        return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: row length or number of runs outside what one launch takes; use the staged calls");
    int lanes = 1;
    while ((int64_t)lanes * 16 < row_bytes) lanes <<= 1;
    const uint32_t per_block = (uint32_t)(kThreads / lanes);
    const int64_t n_max = ctx->B / ctx->P + (ctx->B % ctx->P ? 1 : 0);
    const uint32_t chunks = (uint32_t)((n_max + per_block - 1) / per_block);
    const uint64_t gx = (uint64_t)chunks * ctx->P;
    if (gx > 0x7fffffffull) return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: batch too large for one launch");
    const dim3 grid((unsigned)gx, (unsigned)ctx->Q);
    bool ok;
    switch (ctx->dtype) {
    case BLS_FP16: ok = dispatch<BLS_FP16>(ctx, lanes, grid, st, idx, off, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, segoff, perm, Y, S, R, out, chunks); break;
    case BLS_U8_ROWQ: ok = dispatch<BLS_U8_ROWQ>(ctx, lanes, grid, st, idx, off, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, segoff, perm, Y, S, R, out, chunks); break;
    case BLS_F8_ROWQ: ok = dispatch<BLS_F8_ROWQ>(ctx, lanes, grid, st, idx, off, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, segoff, perm, Y, S, R, out, chunks); break;
    default: ok = dispatch<BLS_FP32>(ctx, lanes, grid, st, idx, off, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, segoff, perm, Y, S, R, out, chunks); break;
    }
    if (!ok) return bls_fail(ctx, BLS_EINVAL, "bls_step_tablewise: unsupported row length");
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
