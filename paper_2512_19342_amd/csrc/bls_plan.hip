// bls_plan: index bucketing by owning rank.
//
// Owner-side order is (owner d, requester s, local table, local sample, position in the bag).
// All bags of one table in one rank's mini-batch - a run (t, s) - are contiguous in the input,
// and inside the run the order of the lookups an owner receives is their input order.  So the
// owner-side place of a lookup is
//      start of block (d, s, t)  +  number of earlier lookups of the run that go to the same owner,
// i.e. a stable split of every run's lookup stream by owner, and the start of a segment
// (d, s, t, b) is the same expression evaluated at the bag's first lookup.  Three launches:
//   1. count   - runs are cut into tiles of consecutive bags; every tile counts its lookups per
//                owner (table-wise: one tile per run, its length read off the offsets),
//   2. scan    - exclusive scan of the tile counts in owner order (d, s, t, tile) gives every
//                tile's start per owner; the alltoallv counts and displacements are differences
//                of that scan at the (d, s) block edges - no atomics, no separate histogram,
//   3. place   - every tile streams its lookups once more, ranks them per owner with a scan of
//                packed per-owner counters over the workgroup (running counts carried from chunk
//                to chunk) and writes ridx, perm and the weights; the segment starts fall out of
//                the same running counts.
// Row-wise with at most eight ranks there is no scan launch: the tiles are fewer and larger, and
// every placing workgroup adds the count array up for itself (plan_place_tiles_scan).
#include <algorithm>

#include "bls_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kItems = 16;                       // scan items per thread
constexpr int kChunk = kThreads * kItems;        // scan items per block
constexpr int kWideThreads = 1024;               // the one-workgroup scan
constexpr int kWideChunk = kWideThreads * kItems;
constexpr int kSmallScanTiles = 8;               // up to this many scan tiles one workgroup scans alone
constexpr int kRounds = 8;                       // place: lookups per thread and chunk
constexpr int kStream = kThreads * kRounds;      // place: lookups per chunk of a tile's stream
constexpr int kOwnersPerPass = 8;                // owners ranked together (packed counters)

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

// Geometry of the row-wise tiles: a run (t, s) is cut into `tiles` tiles of `cb` bags.
struct Tiles {
    uint32_t cb, tiles;
};

// Entry of (owner d, requester s, table t, tile c) in the count array: owner order.
__device__ __forceinline__ int64_t tile_entry(const DevDesc &dd, const Tiles &tg, int d, int s, int t, uint32_t c)
{
    return (((int64_t)d * dd.P + s) * dd.T + t) * tg.tiles + c;
}

// Owner and local row of a global row number under the block partition of ceil(rows / P) rows
// per shard.  The owner is below 64, so a single-precision estimate of the quotient (two 32-bit
// halves converted and combined, times the reciprocal) is off by less than one; the remainder is
// taken exactly in integers and corrects it.  In place of a 64-bit division.
__device__ __forceinline__ void owner_and_row(int64_t ix, int64_t rps, float inv, int &d, int64_t &r)
{
    const float x = fmaf((float)(uint32_t)((uint64_t)ix >> 32), 4294967296.f, (float)(uint32_t)ix);
    d = (int)(x * inv);
    r = ix - (int64_t)d * rps;
    if (r < 0) { --d; r += rps; }
    else if (r >= rps) { ++d; r -= rps; }
}

// The lookups [lo, hi) of the bags [g0, g0 + nb); empty (and flagged) if the offsets are not usable.
__device__ __forceinline__ void tile_range(const DevDesc &dd, const int64_t *__restrict__ off, int64_t g0, uint32_t nb,
                                           int64_t nnz, int64_t &lo, int64_t &hi)
{
    lo = off[g0];
    hi = off[g0 + nb];
    if (lo < 0 || hi > nnz || hi < lo) {
        if (threadIdx.x == 0) flag_error(dd);
        lo = hi = 0;
    }
}

// ---- 1. count ------------------------------------------------------------------------

// Table-wise: one entry per run (q, s) in owner order, its number of lookups.
__global__ __launch_bounds__(kThreads) void plan_count_runs(DevDesc dd, const int64_t *__restrict__ off, int64_t nnz,
                                                            int64_t *__restrict__ cnt)
{
    const int64_t run = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (run >= (int64_t)dd.Q * dd.P) return;
    const int q = (int)(run / dd.P), s = (int)(run - (int64_t)q * dd.P);
    const int t = dd.q_t[q], d = dd.q_d[q];
    const int64_t lo = off[(int64_t)t * dd.B + dd.first[s]], hi = off[(int64_t)t * dd.B + dd.first[s + 1]];
    int64_t len = hi - lo;
    if (lo < 0 || hi > nnz || len < 0) { flag_error(dd); len = 0; }
    cnt[(int64_t)dd.nsum[d] * dd.P + (int64_t)s * dd.n_loc[d] + (q - dd.nsum[d])] = len;
}

// Row-wise: every tile streams its lookups (coalesced, several loads in flight) and counts them
// per owner.  Up to eight owners are counted in two registers of four 16-bit fields; more owners
// in a histogram in LDS.
__global__ __launch_bounds__(kThreads) void plan_count_tiles(DevDesc dd, Tiles tg, const int64_t *__restrict__ idx,
                                                             const int64_t *__restrict__ off, int64_t nnz,
                                                             int64_t *__restrict__ cnt)
{
    __shared__ unsigned long long hist[64];
    const int t = blockIdx.y / dd.P, s = blockIdx.y - t * dd.P;
    const uint32_t c = blockIdx.x;
    const int64_t f = bls_first(dd, s), n = bls_first(dd, s + 1) - f;   // no table look-up: the offsets can be asked for at once
    const int64_t rows = dd.rows[t], rps = dd.rps[t];
    const int64_t b0 = (int64_t)c * tg.cb;
    if (threadIdx.x < 64) hist[threadIdx.x] = 0ull;
    __syncthreads();
    if (b0 < n) {                                             // uniform over the workgroup
        const uint32_t nb = (uint32_t)(n - b0 < tg.cb ? n - b0 : tg.cb);
        int64_t lo, hi;
        tile_range(dd, off, (int64_t)t * dd.B + f + b0, nb, nnz, lo, hi);
        const float inv = 1.f / (float)rps;
        constexpr int kLoads = 8;                              // independent loads per thread in flight
        constexpr int64_t kEpoch = (int64_t)kThreads * 32768;  // no 16-bit field can overflow within one epoch
        for (int64_t e0 = lo; e0 < hi; e0 += kEpoch) {
            const int64_t e1 = e0 + kEpoch < hi ? e0 + kEpoch : hi;
            unsigned long long pk0 = 0ull, pk1 = 0ull;
            for (int64_t i0 = e0 + threadIdx.x; i0 < e1; i0 += (int64_t)kThreads * kLoads) {
                int64_t ix[kLoads];
#pragma unroll
                for (int k = 0; k < kLoads; ++k) ix[k] = i0 + k * kThreads < e1 ? idx[i0 + k * kThreads] : -1;
#pragma unroll
                for (int k = 0; k < kLoads; ++k) {
                    if (i0 + k * kThreads >= e1) continue;
                    if (ix[k] < 0 || ix[k] >= rows) { flag_error(dd); continue; }
                    int d; int64_t r;
                    owner_and_row(ix[k], rps, inv, d, r);
                    if (dd.P <= 8) {
                        if (d < 4) pk0 += 1ull << (16 * d);
                        else pk1 += 1ull << (16 * (d - 4));
                    } else {
                        atomicAdd(&hist[d], 1ull);
                    }
                }
            }
            if (dd.P <= 8) {
#pragma unroll
                for (int o = 0; o < 8; ++o) {
                    unsigned int v = (unsigned int)(((o < 4 ? pk0 : pk1) >> (16 * (o & 3))) & 0xffffull);
#pragma unroll
                    for (int sh = 32; sh >= 1; sh >>= 1) v += __shfl_xor(v, sh, 64);
                    if ((threadIdx.x & 63) == 0 && v) atomicAdd(&hist[o], (unsigned long long)v);
                }
            }
        }
    }
    __syncthreads();
    if (threadIdx.x < dd.P) cnt[tile_entry(dd, tg, threadIdx.x, s, t, c)] = (int64_t)hist[threadIdx.x];
}

// ---- 2. scan ---------------------------------------------------------------------------
// From the counts C[0 .. n) to their exclusive scan X[0 .. n]: X[i] = sum of the counts before entry i,
// X[0] = 0, X[n] = the total (the inclusive scan of C, written one place up).

__global__ __launch_bounds__(kThreads) void scan_block_sums(const int64_t *__restrict__ v, int64_t n,
                                                            int64_t *__restrict__ sums)
{
    __shared__ int64_t part[kWaves];
    const int64_t base = (int64_t)blockIdx.x * kChunk;
    int64_t a = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int64_t i = base + k * kThreads + threadIdx.x;
        if (i < n) a += v[i];
    }
    const int lane = threadIdx.x & 63;
    a = wave_inclusive_scan(a, lane);
    if (lane == 63) part[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t tot = 0;
        for (int w = 0; w < kWaves; ++w) tot += part[w];
        sums[blockIdx.x] = tot;
    }
}

// One block: exclusive scan of the block sums, in place.
__global__ __launch_bounds__(kThreads) void scan_spine(int64_t *__restrict__ sums, int64_t nblk)
{
    __shared__ int64_t part[kWaves];
    __shared__ int64_t carry_s;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < nblk; base += kThreads) {
        const int64_t i = base + threadIdx.x;
        const int64_t x = i < nblk ? sums[i] : 0;
        int64_t inc = wave_inclusive_scan(x, lane);
        if (lane == 63) part[wv] = inc;
        __syncthreads();
        int64_t before = carry_s;
        for (int w = 0; w < wv; ++w) before += part[w];
        if (i < nblk) sums[i] = before + inc - x;
        __syncthreads();
        if (threadIdx.x == kThreads - 1) carry_s = before + inc;
        __syncthreads();
    }
}

// Inclusive scan of one tile src[base .. base + kChunk) into v, offset by `carry`; returns
// carry + the tile's total (the same value in every thread).  Items are staged in LDS so that
// global accesses stay coalesced while every thread owns a contiguous run; one padding word
// per run keeps the per-thread walks off one bank.
__device__ __forceinline__ int64_t scan_tile(const int64_t *__restrict__ src, int64_t *__restrict__ v, int64_t n, int64_t base,
                                             int64_t carry, int64_t *tile, int64_t *part)
{
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int e = k * kThreads + threadIdx.x;
        const int64_t i = base + e;
        tile[e + e / kItems] = i < n ? src[i] : 0;
    }
    __syncthreads();
    const int mine = threadIdx.x * (kItems + 1);
    int64_t run = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k) { run += tile[mine + k]; tile[mine + k] = run; }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t inc = wave_inclusive_scan(run, lane);
    if (lane == 63) part[wv] = inc;
    __syncthreads();
    int64_t before = carry + inc - run, total = carry;
    for (int w = 0; w < kWaves; ++w) {
        if (w < wv) before += part[w];
        total += part[w];
    }
#pragma unroll
    for (int k = 0; k < kItems; ++k) tile[mine + k] += before;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int e = k * kThreads + threadIdx.x;
        const int64_t i = base + e;
        if (i < n) v[i] = tile[e + e / kItems];
    }
    __syncthreads();                                  // tile and part may be reused by the caller
    return total;
}

__global__ __launch_bounds__(kThreads) void scan_apply(const int64_t *__restrict__ src, int64_t *__restrict__ v, int64_t n,
                                                       const int64_t *__restrict__ sums, int64_t *__restrict__ head)
{
    __shared__ int64_t tile[kChunk + kThreads];
    __shared__ int64_t part[kWaves];
    if (blockIdx.x == 0 && threadIdx.x == 0) *head = 0;
    scan_tile(src, v, n, (int64_t)blockIdx.x * kChunk, sums[blockIdx.x], tile, part);
}

// First entry of block (d, s) in the scanned array X (owner order); block (P, 0) is the end.
__device__ __forceinline__ int64_t block_edge(const DevDesc &dd, uint32_t tiles, int d, int s)
{
    if (dd.part_kind == BLS_ROW_WISE) return ((int64_t)d * dd.P + s) * dd.T * tiles;
    if (d >= dd.P) return (int64_t)dd.Q * dd.P;
    return (int64_t)dd.nsum[d] * dd.P + (int64_t)s * dd.n_loc[d];
}

// Counts and displacements from the scan X at the (d, s) block edges, by one workgroup; also the
// last segment start, segoff[nseg] = number of lookups placed.  Called by every thread of the workgroup.
// sabs[s][d] / rabs[d][s]: absolute start of bucket (s, d) in requester / owner order.
__device__ __forceinline__ void finish_counts(const DevDesc &dd, uint32_t tiles, const int64_t *__restrict__ X,
                                              int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                              int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                              int64_t *__restrict__ sabs, int64_t *__restrict__ rabs,
                                              int64_t *__restrict__ segoff_end, int64_t *sc, int64_t *rowtot)
{
    const int P = dd.P;
    for (int e = threadIdx.x; e < P * P; e += blockDim.x) {
        const int d = e / P, s = e - d * P;
        const int64_t lo = X[block_edge(dd, tiles, d, s)];
        const int64_t hi = X[s + 1 < P ? block_edge(dd, tiles, d, s + 1) : block_edge(dd, tiles, d + 1, 0)];
        recvcounts[d * P + s] = hi - lo;
        rdispls[d * P + s] = lo - X[block_edge(dd, tiles, d, 0)];
        rabs[d * P + s] = lo;
        sendcounts[s * P + d] = hi - lo;
        sc[s * P + d] = hi - lo;                      // a copy in LDS for the running sums below
    }
    if (threadIdx.x == 0) *segoff_end = X[block_edge(dd, tiles, P, 0)];
    __syncthreads();
    if (threadIdx.x < P) {
        const int s = threadIdx.x;
        int64_t run = 0;
        for (int d = 0; d < P; ++d) run += sc[s * P + d];
        rowtot[s] = run;
    }
    __syncthreads();
    if (threadIdx.x < P) {
        const int s = threadIdx.x;
        int64_t run = 0;
        for (int r = 0; r < s; ++r) run += rowtot[r];
        const int64_t sbase = run;
        for (int d = 0; d < P; ++d) {
            sdispls[s * P + d] = run - sbase;
            sabs[s * P + d] = run;
            run += sc[s * P + d];
        }
    }
}

__global__ __launch_bounds__(kThreads) void plan_finish(DevDesc dd, uint32_t tiles, const int64_t *__restrict__ X,
                                                        int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                        int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                        int64_t *__restrict__ sabs, int64_t *__restrict__ rabs,
                                                        int64_t *__restrict__ segoff_end)
{
    __shared__ int64_t sc[64 * 64];
    __shared__ int64_t rowtot[64];
    finish_counts(dd, tiles, X, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs, segoff_end, sc, rowtot);
}

// Up to kSmallScanTiles * kChunk counts: one workgroup scans them and derives the alltoallv counts,
// in place of the three scan kernels and plan_finish.
__global__ __launch_bounds__(kThreads) void plan_scan_small(DevDesc dd, uint32_t tiles, const int64_t *__restrict__ C,
                                                            int64_t *__restrict__ X, int64_t n,
                                                            int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                            int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                            int64_t *__restrict__ sabs, int64_t *__restrict__ rabs,
                                                            int64_t *__restrict__ segoff_end)
{
    __shared__ int64_t tile[kChunk + kThreads];
    __shared__ int64_t part[kWaves];
    __shared__ int64_t rowtot[64];
    if (threadIdx.x == 0) X[0] = 0;
    int64_t carry = 0;
    for (int64_t base = 0; base < n; base += kChunk) carry = scan_tile(C, X + 1, n, base, carry, tile, part);
    __syncthreads();                                  // every entry written by this workgroup is visible to it
    finish_counts(dd, tiles, X, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs, segoff_end, tile, rowtot);
}

// Row-wise, few ranks: one workgroup per block (d, s) of the count array.  Every workgroup adds up
// the whole array for itself (it is small and sits in L2), keeping apart what lies before its block,
// what belongs to its owner, to its requester and to earlier requesters; that gives the block's
// start and its row of the counts and displacements without waiting for any other workgroup.  Then
// it scans its own T * tiles entries.  One launch in place of the scan kernels and plan_finish.
__global__ __launch_bounds__(kWideThreads) void plan_scan_blocks(DevDesc dd, uint32_t tiles, const int64_t *__restrict__ cnt,
                                                                 int64_t *__restrict__ X, int64_t n,
                                                                 int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                                 int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                                 int64_t *__restrict__ sabs, int64_t *__restrict__ rabs,
                                                                 int64_t *__restrict__ segoff_end)
{
    constexpr int kW = kWideThreads / 64;
    constexpr int kSums = 6;          // before the block; same owner, earlier requesters; same requester, earlier owners;
                                      // earlier requesters, any owner; the block itself; everything
    __shared__ int64_t part[kW][kSums];
    __shared__ int64_t scanpart[kW];
    const int P = dd.P;
    const int d = blockIdx.x / P, s = blockIdx.x - d * P;
    const uint32_t per_block = (uint32_t)dd.T * tiles;        // entries per (d, s) block
    const int64_t e0 = (int64_t)blockIdx.x * per_block;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    // n is below 2^22 here: entry numbers are exact in single precision, and a quotient estimated
    // with the reciprocal is off by one at most
    const float inv_block = 1.f / (float)per_block, inv_p = 1.f / (float)P;

    int64_t acc[kSums] = {0, 0, 0, 0, 0, 0};
    for (int64_t base = 0; base < n; base += (int64_t)kWideThreads * kItems) {
        int64_t x[kItems];
#pragma unroll
        for (int k = 0; k < kItems; ++k) {                    // consecutive threads read consecutive entries
            const int64_t e = base + (int64_t)k * kWideThreads + threadIdx.x;
            x[k] = e < n ? cnt[e] : 0;
        }
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            const uint32_t e = (uint32_t)(base + (int64_t)k * kWideThreads + threadIdx.x);
            uint32_t b = (uint32_t)((float)e * inv_block);
            if (b * per_block > e) --b;
            else if ((b + 1u) * per_block <= e) ++b;
            uint32_t dp = (uint32_t)((float)b * inv_p);
            if (dp * (uint32_t)P > b) --dp;
            else if ((dp + 1u) * (uint32_t)P <= b) ++dp;
            const int sp = (int)(b - dp * (uint32_t)P);
            if (b < blockIdx.x) acc[0] += x[k];
            if ((int)dp == d && sp < s) acc[1] += x[k];
            if (sp == s && (int)dp < d) acc[2] += x[k];
            if (sp < s) acc[3] += x[k];
            if (b == blockIdx.x) acc[4] += x[k];
            acc[5] += x[k];
        }
    }
#pragma unroll
    for (int a = 0; a < kSums; ++a) {
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) acc[a] += __shfl_xor(acc[a], sh, 64);
        if (lane == 0) part[wv][a] = acc[a];
    }
    __syncthreads();
    int64_t mine[kSums] = {0, 0, 0, 0, 0, 0};
    for (int w = 0; w < kW; ++w)
#pragma unroll
        for (int a = 0; a < kSums; ++a) mine[a] += part[w][a];
    if (threadIdx.x == 0) {
        recvcounts[d * P + s] = mine[4];
        sendcounts[s * P + d] = mine[4];
        rdispls[d * P + s] = mine[1];
        sdispls[s * P + d] = mine[2];
        rabs[d * P + s] = mine[0];
        sabs[s * P + d] = mine[3] + mine[2];
        if ((int)blockIdx.x == P * P - 1) { X[n] = mine[5]; *segoff_end = mine[5]; }
    }
    int64_t carry = mine[0];
    // the block's own entries: X[e] = start of the block + the counts before e inside it
    for (int64_t base = 0; base < per_block; base += kWideChunk) {
        const int64_t at = base + (int64_t)threadIdx.x * kItems;
        int64_t x[kItems];
#pragma unroll
        for (int k = 0; k < kItems; ++k) x[k] = at + k < per_block ? cnt[e0 + at + k] : 0;
        int64_t run = 0;
#pragma unroll
        for (int k = 0; k < kItems; ++k) { const int64_t v = x[k]; x[k] = run; run += v; }
        const int64_t inc = wave_inclusive_scan(run, lane);
        __syncthreads();                              // scanpart is free again
        if (lane == 63) scanpart[wv] = inc;
        __syncthreads();
        int64_t before = carry + inc - run, total = carry;
        for (int w = 0; w < kW; ++w) {
            if (w < wv) before += scanpart[w];
            total += scanpart[w];
        }
#pragma unroll
        for (int k = 0; k < kItems; ++k)
            if (at + k < per_block) X[e0 + at + k] = x[k] + before;
        carry = total;
    }
}

// ---- 3. place --------------------------------------------------------------------------

// Table-wise: a run (q, s) is contiguous both in input order and in owner order, so placing is
// Q*P block copies of index lists, and a segment starts as far into the owner-side block as its
// bag starts into the run.  grid: x strides over a run, y strides over the runs.
__global__ __launch_bounds__(kThreads) void plan_place_runs(DevDesc dd, const int64_t *__restrict__ idx,
                                                            const int64_t *__restrict__ off, int64_t nnz,
                                                            const int64_t *__restrict__ X, int64_t *__restrict__ segoff,
                                                            int64_t *__restrict__ ridx, int64_t *__restrict__ perm,
                                                            const int64_t *__restrict__ sabs,
                                                            const int64_t *__restrict__ rabs,
                                                            const float *__restrict__ w_in, float *__restrict__ w_out)
{
    constexpr int kPer = 4;
    for (int run = blockIdx.y; run < dd.Q * dd.P; run += gridDim.y) {
        const int q = run / dd.P, s = run - q * dd.P;
        const int t = dd.q_t[q], d = dd.q_d[q];
        const int64_t f = dd.first[s], n = dd.first[s + 1] - f;
        const int64_t g0 = (int64_t)t * dd.B + f;
        int64_t lo = off[g0], hi = off[g0 + n];
        if (lo < 0 || hi > nnz || hi < lo) lo = hi = 0;       // flagged by the count kernel; the run counts as empty
        const int64_t len = hi - lo;
        const int64_t dst = X[(int64_t)dd.nsum[d] * dd.P + (int64_t)s * dd.n_loc[d] + (q - dd.nsum[d])];
        // segment starts of the run's bags
        const int64_t sg0 = (int64_t)dd.nsum[d] * dd.B + (int64_t)dd.n_loc[d] * f + (int64_t)(q - dd.nsum[d]) * n;
        for (int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x; b < n; b += (int64_t)gridDim.x * kThreads) {
            int64_t at = off[g0 + b] - lo;
            const int64_t nxt = off[g0 + b + 1] - lo;
            if (at < 0 || at > len || nxt < at) { flag_error(dd); at = at < 0 ? 0 : (at > len ? len : at); }
            segoff[sg0 + b] = dst + at;
        }
        if (len <= 0) continue;
        if (dst < 0 || dst + len > nnz) { if (threadIdx.x == 0 && blockIdx.x == 0) flag_error(dd); continue; }
        const int64_t rows = dd.rows[t];
        const int64_t to_send = perm ? sabs[s * dd.P + d] - rabs[d * dd.P + s] : 0;
        const int64_t stride = (int64_t)gridDim.x * kThreads * kPer;
        for (int64_t i0 = (int64_t)blockIdx.x * kThreads * kPer + threadIdx.x; i0 < len; i0 += stride) {
            int64_t v[kPer];
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int64_t i = i0 + k * kThreads;
                v[k] = i < len ? idx[lo + i] : 0;
            }
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int64_t i = i0 + k * kThreads;
                if (i < len) {
                    if (v[k] < 0 || v[k] >= rows) { flag_error(dd); v[k] = -1; }   // the pool skips negative rows
                    ridx[dst + i] = v[k];
                    if (w_in) w_out[dst + i] = w_in[lo + i];
                    if (perm) perm[lo + i] = dst + i + to_send;
                }
            }
        }
    }
}

// Table-wise with up to kMaxRuns runs: count, scan and place in one launch.  A run's place on the
// owner's side follows from the run lengths alone, and those are differences of the offsets at
// the run edges: every workgroup reads the edges for itself (a few hundred values out of L2),
// scans the lengths in owner order in LDS, and then copies its runs as plan_place_runs does; the
// first workgroup also writes the counts and displacements.
constexpr int kMaxRuns = 2048;
constexpr int kRunsPerThread = kMaxRuns / kThreads;
__global__ __launch_bounds__(kThreads) void plan_runs_one_launch(DevDesc dd, const int64_t *__restrict__ idx,
                                                                 const int64_t *__restrict__ off, int64_t nnz,
                                                                 int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                                 int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                                 int64_t *__restrict__ segoff, int64_t *__restrict__ ridx,
                                                                 int64_t *__restrict__ perm, const float *__restrict__ w_in,
                                                                 float *__restrict__ w_out)
{
    constexpr int kPer = 4;
    __shared__ int64_t rb[kMaxRuns + 1];       // run lengths in owner order, then their exclusive scan
    __shared__ int64_t part[kWaves];
    __shared__ int64_t req_before[65];         // lookups of the requesters before s
    const int P = dd.P, nruns = dd.Q * P;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    auto entry = [&](int q, int s) -> int {    // position of run (q, s) in owner order (d, s, local table)
        const int d = dd.q_d[q];
        return dd.nsum[d] * P + s * dd.n_loc[d] + (q - dd.nsum[d]);
    };

    for (int i = threadIdx.x; i < kMaxRuns + 1; i += kThreads) rb[i] = 0;
    __syncthreads();
    bool bad_edges = false;
    for (int i = threadIdx.x; i < nruns; i += kThreads) {
        const int q = i / P, s = i - q * P;
        const int64_t g0 = (int64_t)dd.q_t[q] * dd.B;
        const int64_t lo = off[g0 + dd.first[s]], hi = off[g0 + dd.first[s + 1]];
        int64_t len = hi - lo;
        if (lo < 0 || hi > nnz || len < 0) { bad_edges = true; len = 0; }
        rb[entry(q, s)] = len;
    }
    if (bad_edges && blockIdx.x == 0 && blockIdx.y == 0) flag_error(dd);
    __syncthreads();
    {
        int64_t x[kRunsPerThread], run = 0;
#pragma unroll
        for (int k = 0; k < kRunsPerThread; ++k) { x[k] = run; run += rb[threadIdx.x * kRunsPerThread + k]; }
        const int64_t inc = wave_inclusive_scan(run, lane);
        if (lane == 63) part[wv] = inc;
        __syncthreads();
        int64_t before = inc - run;
        for (int w = 0; w < wv; ++w) before += part[w];
#pragma unroll
        for (int k = 0; k < kRunsPerThread; ++k) rb[threadIdx.x * kRunsPerThread + k] = x[k] + before;
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
    if (threadIdx.x < P) {                                    // lookups per requester, then those of earlier requesters
        int64_t run = 0;
        for (int d = 0; d < P; ++d) run += count(threadIdx.x, d);
        req_before[threadIdx.x + 1] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        req_before[0] = 0;
        for (int s = 0; s < P; ++s) req_before[s + 1] += req_before[s];
    }
    __syncthreads();

    if (blockIdx.x == 0 && blockIdx.y == 0) {
        for (int e = threadIdx.x; e < P * P; e += kThreads) {
            const int d = e / P, s = e - d * P;
            recvcounts[d * P + s] = count(s, d);
            sendcounts[s * P + d] = count(s, d);
            rdispls[d * P + s] = edge(d, s) - edge(d, 0);
            int64_t run = 0;
            for (int o = 0; o < d; ++o) run += count(s, o);
            sdispls[s * P + d] = run;
        }
        if (threadIdx.x == 0) segoff[dd.nseg] = placed;
    }

    for (int run = blockIdx.y; run < nruns; run += gridDim.y) {
        const int q = run / P, s = run - q * P;
        const int t = dd.q_t[q], d = dd.q_d[q];
        const int64_t f = dd.first[s], n = dd.first[s + 1] - f;
        const int64_t g0 = (int64_t)t * dd.B + f;
        int64_t lo = off[g0], hi = off[g0 + n];
        if (lo < 0 || hi > nnz || hi < lo) lo = hi = 0;       // flagged above; the run counts as empty
        const int64_t len = hi - lo;
        const int64_t dst = rb[entry(q, s)];
        const int64_t sg0 = (int64_t)dd.nsum[d] * dd.B + (int64_t)dd.n_loc[d] * f + (int64_t)(q - dd.nsum[d]) * n;
        for (int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x; b < n; b += (int64_t)gridDim.x * kThreads) {
            int64_t at = off[g0 + b] - lo;
            const int64_t nxt = off[g0 + b + 1] - lo;
            if (at < 0 || at > len || nxt < at) { flag_error(dd); at = at < 0 ? 0 : (at > len ? len : at); }
            segoff[sg0 + b] = dst + at;
        }
        if (len <= 0) continue;
        if (dst < 0 || dst + len > nnz) { if (threadIdx.x == 0 && blockIdx.x == 0) flag_error(dd); continue; }
        const int64_t rows = dd.rows[t];
        // owner-side place -> requester-side place: start of bucket (s, d) in requester order (the lookups of
        // earlier requesters, and this requester's for earlier owners) minus its start in owner order
        int64_t to_send = 0;
        if (perm) {
            to_send = req_before[s] - edge(d, s);
            for (int o = 0; o < d; ++o) to_send += count(s, o);
        }
        const int64_t stride = (int64_t)gridDim.x * kThreads * kPer;
        for (int64_t i0 = (int64_t)blockIdx.x * kThreads * kPer + threadIdx.x; i0 < len; i0 += stride) {
            int64_t v[kPer];
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int64_t i = i0 + k * kThreads;
                v[k] = i < len ? idx[lo + i] : 0;
            }
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int64_t i = i0 + k * kThreads;
                if (i < len) {
                    if (v[k] < 0 || v[k] >= rows) { flag_error(dd); v[k] = -1; }   // the pool skips negative rows
                    ridx[dst + i] = v[k];
                    if (w_in) w_out[dst + i] = w_in[lo + i];
                    if (perm) perm[lo + i] = dst + i + to_send;
                }
            }
        }
    }
}

// Four bytes spread to four 16-bit fields of a 64-bit word.
__device__ __forceinline__ unsigned long long spread4(uint32_t x)
{
    unsigned long long v = x;
    v = (v | (v << 16)) & 0x0000ffff0000ffffull;
    v = (v | (v << 8)) & 0x00ff00ff00ff00ffull;
    return v;
}

// Field o (0..7) of a pair of words with four 16-bit fields each.
__device__ __forceinline__ uint32_t field16(unsigned long long w0, unsigned long long w1, int o)
{
    return (uint32_t)(((o < 4 ? w0 : w1) >> (16 * (o & 3))) & 0xffffull);
}

// Row-wise: a tile streams its lookups in chunks of kStream.  They are loaded coalesced (lookup e
// of the chunk by thread e % 256), which gives owner and local row; the owners go to LDS, one byte
// each, and are ranked in blocks: thread i reads the owners of lookups 8i .. 8i+7, counts them per
// owner in byte fields, and an exclusive scan of those counts over the workgroup (16-bit fields,
// up to eight owners in two words, more owners eight at a time) gives every lookup its rank among
// the chunk's lookups of the same owner.  The ranks return through LDS to the threads that hold
// the rows; running totals carry the rank from chunk to chunk.  The start of segment (d, bag) is
// the same count taken at the bag's first lookup.
// LDS of one placing workgroup.
struct PlaceLds {
    unsigned long long ownb[kThreads];             // owners of the chunk's lookups, a byte each (0xff: none)
    unsigned long long excl[kThreads][2];          // per thread: same-owner lookups before its first one
    __attribute__((aligned(16))) unsigned short rk[kStream];   // rank of every lookup among its owner's
    unsigned long long wtot[kWaves][2];            // per wavefront: its lookups per owner
    int64_t start[64];                             // owner's next free place: tile start + running count
    int64_t shift[64];                             // owner-side place -> requester-side place
};

// Places the lookups [lo, lo + len) of a tile of run (t, s): the nb bags from bag b0 of the run's n.
// L.start and L.shift are set by the caller (threads below P) before the call; no barrier is needed
// in between.
template <bool PERM, bool WGT>
__device__ __forceinline__ void place_tile(const DevDesc &dd, PlaceLds &L, const int64_t *__restrict__ idx,
                                           const int64_t *__restrict__ off, int64_t nnz, int64_t *__restrict__ segoff,
                                           int64_t *__restrict__ ridx, int64_t *__restrict__ perm,
                                           const float *__restrict__ w_in, float *__restrict__ w_out, int t, int s,
                                           int64_t n, int64_t b0, uint32_t nb, int64_t lo, int64_t len)
{
    auto &ownb = L.ownb;
    auto &excl = L.excl;
    auto &rk = L.rk;
    auto &wtot = L.wtot;
    auto &start = L.start;
    auto &shift = L.shift;
    const int64_t rows = dd.rows[t], rps = dd.rps[t];
    const int64_t g0 = (int64_t)t * dd.B + bls_first(dd, s) + b0;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const float inv = 1.f / (float)rps;
    const int passes = (dd.P + kOwnersPerPass - 1) / kOwnersPerPass;

    // where bag b of the tile starts in the tile's stream, clamped into it (bad offsets are flagged once)
    auto bag_start = [&](uint32_t b, bool report) -> int64_t {
        int64_t at = off[g0 + b] - lo;
        if (at < 0 || at > len || off[g0 + b + 1] - lo < at) {
            if (report) flag_error(dd);
            at = at < 0 ? 0 : (at > len ? len : at);
        }
        return at;
    };
    const int64_t at_first = threadIdx.x < nb ? bag_start(threadIdx.x, true) : -1;   // bag b = threadIdx.x
    for (uint32_t b = threadIdx.x + kThreads; b < nb; b += kThreads) (void)bag_start(b, true);

    for (int64_t c0 = 0; c0 < len || c0 == 0; c0 += kStream) {
        const bool last = c0 + kStream >= len;
        // this thread's lookups of the chunk: owner (a byte each, 0xff: none or a bad index) and local
        // row (below 2^32: no shard has more rows)
        unsigned long long owns = ~0ull;
        uint32_t row[kRounds];
        {
            int64_t ix[kRounds];
#pragma unroll
            for (int k = 0; k < kRounds; ++k) {
                const int64_t i = c0 + k * kThreads + threadIdx.x;
                ix[k] = i < len ? idx[lo + i] : -1;
            }
#pragma unroll
            for (int k = 0; k < kRounds; ++k) {
                uint32_t o = 0xffu;
                row[k] = 0u;
                if (c0 + k * kThreads + threadIdx.x < len) {
                    if (ix[k] < 0 || ix[k] >= rows) flag_error(dd);
                    else { int d; int64_t r; owner_and_row(ix[k], rps, inv, d, r); o = (uint32_t)d; row[k] = (uint32_t)r; }
                }
                owns = (owns & ~(0xffull << (8 * k))) | ((unsigned long long)o << (8 * k));
                reinterpret_cast<unsigned char *>(ownb)[k * kThreads + threadIdx.x] = (unsigned char)o;
            }
        }
        __syncthreads();                                      // the owners are in LDS; start[] is up to date
        for (int pass = 0; pass < passes; ++pass) {
            const uint32_t o0 = (uint32_t)(pass * kOwnersPerPass);
            // blocked: lookups 8i .. 8i+7 of the chunk
            const unsigned long long own8 = ownb[threadIdx.x];
            unsigned long long pk8 = 0ull;                     // lookups per owner among this thread's eight, byte fields
            uint32_t lr = 0u;                                  // rank of each of the eight inside the thread, 4 bits each
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t o = (uint32_t)((own8 >> (8 * j)) & 0xffull) - o0;
                const bool mine = o < (uint32_t)kOwnersPerPass;
                const int sh = mine ? (int)(8 * o) : 0;
                lr |= (uint32_t)((pk8 >> sh) & 0xfull) << (4 * j);
                if (mine) pk8 += 1ull << sh;
            }
            const unsigned long long e0 = spread4((uint32_t)pk8), e1 = spread4((uint32_t)(pk8 >> 32));
            const unsigned long long i0 = (unsigned long long)wave_inclusive_scan((int64_t)e0, lane);
            const unsigned long long i1 = (unsigned long long)wave_inclusive_scan((int64_t)e1, lane);
            if (lane == 63) { wtot[wv][0] = i0; wtot[wv][1] = i1; }
            __syncthreads();
            unsigned long long x0 = i0 - e0, x1 = i1 - e1, t0 = 0ull, t1 = 0ull;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                if (w < wv) { x0 += wtot[w][0]; x1 += wtot[w][1]; }
                t0 += wtot[w][0]; t1 += wtot[w][1];
            }
            excl[threadIdx.x][0] = x0;
            excl[threadIdx.x][1] = x1;
            {
                unsigned long long r0 = 0ull, r1 = 0ull;       // eight 16-bit ranks
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t o = (uint32_t)((own8 >> (8 * j)) & 0xffull) - o0;
                    const unsigned long long v = o < (uint32_t)kOwnersPerPass ? (unsigned long long)(field16(x0, x1, (int)o) + ((lr >> (4 * j)) & 0xfu)) : 0ull;
                    if (j < 4) r0 |= v << (16 * j);
                    else r1 |= v << (16 * (j - 4));
                }
                unsigned long long *dst = reinterpret_cast<unsigned long long *>(rk + 8 * threadIdx.x);
                dst[0] = r0;
                dst[1] = r1;
            }
            __syncthreads();
            // back to the threads that hold the rows
#pragma unroll
            for (int k = 0; k < kRounds; ++k) {
                const uint32_t d = (uint32_t)((owns >> (8 * k)) & 0xffull);
                if (d - o0 < (uint32_t)kOwnersPerPass) {
                    const int64_t place = start[d] + rk[k * kThreads + threadIdx.x];
                    if (place >= 0 && place < nnz) {
                        const int64_t l = lo + c0 + k * kThreads + threadIdx.x;
                        ridx[place] = (int64_t)row[k];
                        if constexpr (WGT) w_out[place] = w_in[l];
                        if constexpr (PERM) perm[l] = place + shift[d];
                    } else flag_error(dd);
                }
            }
            // segments that start inside this chunk; one that starts where the chunk's last lookup ends
            // can only be at the end of the tile's stream and takes the chunk's totals
            for (uint32_t b = threadIdx.x; b < nb; b += kThreads) {
                const int64_t at = b < (uint32_t)kThreads ? at_first : bag_start(b, false);
                if (at < c0 || at > c0 + kStream || (at == c0 + kStream && !last)) continue;
                const int e = (int)(at - c0);
                unsigned long long w0 = t0, w1 = t1, before8 = 0ull;
                if (e < kStream) {
                    const int th = e >> 3, j = e & 7;
                    w0 = excl[th][0];
                    w1 = excl[th][1];
                    const unsigned long long o8 = ownb[th];
#pragma unroll
                    for (int jj = 0; jj < 7; ++jj) {
                        const uint32_t o = (uint32_t)((o8 >> (8 * jj)) & 0xffull) - o0;
                        if (jj < j && o < (uint32_t)kOwnersPerPass) before8 += 1ull << (8 * o);
                    }
                }
                // segments (owner, bag) of consecutive owners lie B*T entries apart
                int64_t *so = segoff + bls_sigma_rowwise(dd, (int)o0, t, s, (uint32_t)(b0 + b), (uint32_t)n);
                const int64_t per_owner = dd.B * dd.T;
#pragma unroll 1
                for (uint32_t o = 0; o < (uint32_t)kOwnersPerPass && o0 + o < (uint32_t)dd.P; ++o, so += per_owner)
                    *so = start[o0 + o] + field16(w0, w1, (int)o) + (uint32_t)((before8 >> (8 * o)) & 0xffull);
            }
            __syncthreads();
            if (threadIdx.x < kOwnersPerPass && o0 + threadIdx.x < (uint32_t)dd.P)
                start[o0 + threadIdx.x] += field16(t0, t1, (int)threadIdx.x);
        }
        __syncthreads();                                      // start[] is final before the next chunk reads it; LDS is free
    }
}

template <bool PERM, bool WGT>
__global__ __launch_bounds__(kThreads) void plan_place_tiles(DevDesc dd, Tiles tg, const int64_t *__restrict__ idx,
                                                             const int64_t *__restrict__ off, int64_t nnz,
                                                             const int64_t *__restrict__ X, int64_t *__restrict__ segoff,
                                                             int64_t *__restrict__ ridx, int64_t *__restrict__ perm,
                                                             const int64_t *__restrict__ sabs,
                                                             const int64_t *__restrict__ rabs,
                                                             const float *__restrict__ w_in, float *__restrict__ w_out)
{
    __shared__ PlaceLds L;
    const int t = blockIdx.y / dd.P, s = blockIdx.y - t * dd.P;
    const uint32_t c = blockIdx.x;
    const int64_t f = bls_first(dd, s), n = bls_first(dd, s + 1) - f;
    const int64_t b0 = (int64_t)c * tg.cb;
    if (b0 >= n) return;                                      // uniform over the workgroup: no bags in this tile
    const uint32_t nb = (uint32_t)(n - b0 < tg.cb ? n - b0 : tg.cb);
    int64_t lo, hi;
    tile_range(dd, off, (int64_t)t * dd.B + f + b0, nb, nnz, lo, hi);
    if (threadIdx.x < dd.P) {
        L.start[threadIdx.x] = X[tile_entry(dd, tg, threadIdx.x, s, t, c)];
        L.shift[threadIdx.x] = PERM ? sabs[s * dd.P + threadIdx.x] - rabs[threadIdx.x * dd.P + s] : 0;
    }
    place_tile<PERM, WGT>(dd, L, idx, off, nnz, segoff, ridx, perm, w_in, w_out, t, s, n, b0, nb, lo, hi - lo);
}

// Row-wise with at most eight ranks: placing without a scan launch.  A tile's start for owner d is the
// sum of all counts before entry (d, s, t, c) in owner order; an owner's entries are a row of P*T*tiles
// counts, so the eight starts are the totals of the earlier rows plus a prefix of the own row.  Every
// workgroup adds the count array up for itself (it is small and sits in L2): 32 threads per owner,
// keeping apart what lies before this tile, what belongs to earlier requesters and to this requester
// (the last two place the buckets in requester order, for perm).  The first workgroup also derives
// the alltoallv counts and displacements.  Sums are kept in 32 bits: for batches below 2^32 lookups.
template <bool PERM, bool WGT>
__global__ __launch_bounds__(kThreads) void plan_place_tiles_scan(DevDesc dd, Tiles tg, const int64_t *__restrict__ idx,
                                                                  const int64_t *__restrict__ off, int64_t nnz,
                                                                  const int64_t *__restrict__ C,
                                                                  int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                                  int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                                  int64_t *__restrict__ segoff, int64_t *__restrict__ ridx,
                                                                  int64_t *__restrict__ perm, const float *__restrict__ w_in,
                                                                  float *__restrict__ w_out)
{
    __shared__ PlaceLds L;
    __shared__ uint32_t part[8][4];                   // per owner: total, earlier requesters, this requester, before this tile
    __shared__ int64_t blk[64], rowtot[8];            // the first workgroup: lookups per (owner, requester) block

    const int P = dd.P;
    const int t = blockIdx.y / P, s = blockIdx.y - t * P;
    const uint32_t c = blockIdx.x;
    const int64_t f = bls_first(dd, s), n = bls_first(dd, s + 1) - f;
    const int64_t b0 = (int64_t)c * tg.cb;
    const bool first_wg = blockIdx.x == 0 && blockIdx.y == 0;
    if (b0 >= n && !first_wg) return;                 // uniform over the workgroup: no bags in this tile

    const uint32_t per_req = (uint32_t)dd.T * tg.tiles, rowlen = (uint32_t)P * per_req;
    {
        const int d = threadIdx.x >> 5, l = threadIdx.x & 31;
        const uint32_t a0 = (uint32_t)s * per_req, a1 = a0 + per_req, at = a0 + (uint32_t)t * tg.tiles + c;
        uint32_t tot = 0, early = 0, same = 0, before = 0;
        if (d < P) {
            const int64_t *row = C + (int64_t)d * rowlen;
            constexpr int kAhead = 8;                 // independent loads in flight
            for (uint32_t j0 = l; j0 < rowlen; j0 += 32 * kAhead) {
                uint32_t x[kAhead];
#pragma unroll
                for (int k = 0; k < kAhead; ++k) x[k] = j0 + 32 * k < rowlen ? (uint32_t)row[j0 + 32 * k] : 0u;
#pragma unroll
                for (int k = 0; k < kAhead; ++k) {
                    const uint32_t j = j0 + 32 * k;
                    tot += x[k];
                    if (j < a0) early += x[k];
                    else if (j < a1) same += x[k];
                    if (j < at) before += x[k];
                }
            }
        }
#pragma unroll
        for (int sh = 16; sh >= 1; sh >>= 1) {
            tot += __shfl_xor(tot, sh, 64);
            early += __shfl_xor(early, sh, 64);
            same += __shfl_xor(same, sh, 64);
            before += __shfl_xor(before, sh, 64);
        }
        if (l == 0) { part[d][0] = tot; part[d][1] = early; part[d][2] = same; part[d][3] = before; }
    }
    __syncthreads();
    if (threadIdx.x < P) {
        const int d = threadIdx.x;
        int64_t owners_before = 0, early_all = 0, same_before = 0;
        for (int o = 0; o < P; ++o) {
            if (o < d) { owners_before += part[o][0]; same_before += part[o][2]; }
            early_all += part[o][1];
        }
        L.start[d] = owners_before + part[d][3];
        // bucket (s, d) starts at early_all + same_before in requester order, at owners_before + early(d) in owner order
        L.shift[d] = PERM ? (early_all + same_before) - (owners_before + (int64_t)part[d][1]) : 0;
    }

    if (first_wg) {
        const int e = threadIdx.x >> 2, l = threadIdx.x & 3;  // block e = d * P + s', four threads each
        uint32_t sum = 0;
        if (e < P * P)
            for (uint32_t j = l; j < per_req; j += 4) sum += (uint32_t)C[(int64_t)e * per_req + j];
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        if (l == 0 && e < P * P) blk[e] = sum;
        __syncthreads();
        if (threadIdx.x < P) {                            // lookups per requester
            int64_t run = 0;
            for (int d = 0; d < P; ++d) run += blk[d * P + threadIdx.x];
            rowtot[threadIdx.x] = run;
        }
        __syncthreads();
        if (threadIdx.x < P * P) {
            const int d = threadIdx.x / P, sp = threadIdx.x - d * P;
            int64_t rd = 0, sd = 0;
            for (int r = 0; r < sp; ++r) rd += blk[d * P + r];
            for (int o = 0; o < d; ++o) sd += blk[o * P + sp];
            recvcounts[d * P + sp] = blk[d * P + sp];
            rdispls[d * P + sp] = rd;
            sendcounts[sp * P + d] = blk[d * P + sp];
            sdispls[sp * P + d] = sd;
        }
        if (threadIdx.x == 0) {
            int64_t all = 0;
            for (int r = 0; r < P; ++r) all += rowtot[r];
            segoff[dd.nseg] = all;
        }
        if (b0 >= n) return;
    }

    const uint32_t nb = (uint32_t)(n - b0 < tg.cb ? n - b0 : tg.cb);
    int64_t lo, hi;
    tile_range(dd, off, (int64_t)t * dd.B + f + b0, nb, nnz, lo, hi);
    place_tile<PERM, WGT>(dd, L, idx, off, nnz, segoff, ridx, perm, w_in, w_out, t, s, n, b0, nb, lo, hi - lo);
}

int64_t scan_blocks(int64_t n) { return (n + kChunk - 1) / kChunk; }

uint32_t pow2_at_least(int64_t x)
{
    uint32_t p = 1;
    while ((int64_t)p < x && p < (1u << 30)) p <<= 1;
    return p;
}

// Row-wise tiles: about kTilesWanted tiles in all, none below `min_bags` bags.
constexpr int64_t kTilesWanted = 2048;
uint32_t bags_per_tile(const bls_ctx *ctx, int64_t min_bags, int64_t tiles_wanted = kTilesWanted)
{
    const int64_t n_max = ctx->B / ctx->P + (ctx->B % ctx->P ? 1 : 0);
    const int64_t runs = (int64_t)ctx->T * ctx->P;
    const int64_t for_count = (n_max * runs + tiles_wanted - 1) / tiles_wanted;
    return pow2_at_least(std::max<int64_t>({for_count, min_bags, 32}));
}

// Entries of the count array: runs (table-wise), or owners * runs * tiles per run.
int64_t count_entries(const bls_ctx *ctx, uint32_t cb)
{
    if (ctx->part_kind == BLS_TABLE_WISE) return (int64_t)ctx->Q * ctx->P;
    const int64_t n_max = ctx->B / ctx->P + (ctx->B % ctx->P ? 1 : 0);
    return (int64_t)ctx->P * ctx->P * ctx->T * ((n_max + cb - 1) / cb);
}

}  // namespace

// Workspace: the count array, its scan (one more entry for the total), the scan's block sums, the
// bucket starts in requester and in owner order.  The smallest tiles any call may choose bound the size.
size_t bls_plan_ws_bytes(const bls_ctx *ctx)
{
    const int64_t n = count_entries(ctx, bags_per_tile(ctx, 0));
    return (size_t)(2 * n + 1 + scan_blocks(n) + 2 * ctx->P * ctx->P + 2) * sizeof(int64_t);
}

int bls_launch_plan(bls_ctx *ctx, const int64_t *idx, const int64_t *off, int64_t nnz, int64_t *sendcounts,
                    int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls, int64_t *ridx, int64_t *segoff,
                    int64_t *perm, const float *w_in, float *w_out, void *ws, size_t ws_bytes, hipStream_t st)
{
    (void)ws_bytes;
    const DevDesc &dd = ctx->desc;
    const bool rowwise = ctx->part_kind == BLS_ROW_WISE;
    // tiles of about a thousand lookups or more, going by the batch's mean bag length
    const int64_t mean = nnz / std::max<int64_t>(1, (int64_t)ctx->T * ctx->B) + 1;
    const int64_t n_max = ctx->B / ctx->P + (ctx->B % ctx->P ? 1 : 0);
    // row-wise with few ranks and a count array small enough for every workgroup to read (with many
    // tables the runs alone outnumber that): the placing workgroups add the counts up themselves, on
    // fewer and larger tiles, and there is no scan launch
    constexpr int64_t kOwnScanEntries = 16384;
    bool own_scan = rowwise && ctx->P <= 8 && nnz < ((int64_t)1 << 32) && ctx->tune_plan_scan != 0;
    Tiles tg;
    tg.cb = rowwise ? bags_per_tile(ctx, 1024 / mean, own_scan ? 1024 : kTilesWanted) : 1u;
    if (own_scan && count_entries(ctx, tg.cb) > kOwnScanEntries) {
        own_scan = false;
        tg.cb = bags_per_tile(ctx, 1024 / mean);
    }
    tg.tiles = rowwise ? (uint32_t)((n_max + tg.cb - 1) / tg.cb) : 1u;
    const int64_t n = count_entries(ctx, tg.cb), nblk = scan_blocks(n);
    int64_t *C = (int64_t *)ws;                       // n counts
    int64_t *X = C + n;                               // n + 1 entries: their exclusive scan
    int64_t *sums = X + n + 1;
    int64_t *sabs = sums + nblk, *rabs = sabs + ctx->P * ctx->P;
    int64_t *segoff_end = segoff + ctx->nseg;
    const dim3 tgrid(tg.tiles, (unsigned)(ctx->T * ctx->P));

    // small table-wise batches (large ones are a copy of hundreds of megabytes, which three launches do faster:
    // workload 4, 34 M lookups, 0.121 ms against 0.145)
    if (!rowwise && (int64_t)ctx->Q * ctx->P <= kMaxRuns && nnz <= ((int64_t)1 << 22) && ctx->tune_plan_scan != 0) {
        const int64_t runs = (int64_t)ctx->Q * ctx->P;
        // every workgroup pays for the scan of the run edges: about four thousand workgroups in all, none
        // with less than 2048 lookups or bags to work on
        const int64_t per_run = std::max<int64_t>(nnz / runs, n_max) + 1;
        const int64_t want = (4096 + runs - 1) / runs;
        const unsigned gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>(want, (per_run + 2047) / 2048));
        plan_runs_one_launch<<<dim3(gx, (unsigned)runs), kThreads, 0, st>>>(dd, idx, off, nnz, sendcounts, sdispls, recvcounts, rdispls,
                                                                             segoff, ridx, perm, w_in, w_out);
        BLS_HIP(ctx, hipGetLastError());
        return BLS_OK;
    }
    if (rowwise) plan_count_tiles<<<tgrid, kThreads, 0, st>>>(dd, tg, idx, off, nnz, C);
    else plan_count_runs<<<dim3((unsigned)((n + kThreads - 1) / kThreads)), kThreads, 0, st>>>(dd, off, nnz, C);
    if (own_scan) {
        // no launch
    } else if (rowwise && (int64_t)ctx->P * ctx->P * n <= (int64_t)1 << 22) {
        plan_scan_blocks<<<dim3((unsigned)(ctx->P * ctx->P)), kWideThreads, 0, st>>>(dd, tg.tiles, C, X, n, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs, segoff_end);
    } else if (nblk <= kSmallScanTiles) {
        plan_scan_small<<<1, kThreads, 0, st>>>(dd, tg.tiles, C, X, n, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs, segoff_end);
    } else {
        scan_block_sums<<<dim3((unsigned)nblk), kThreads, 0, st>>>(C, n, sums);
        scan_spine<<<1, kThreads, 0, st>>>(sums, nblk);
        scan_apply<<<dim3((unsigned)nblk), kThreads, 0, st>>>(C, X + 1, n, sums, X);
        plan_finish<<<1, kThreads, 0, st>>>(dd, tg.tiles, X, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs, segoff_end);
    }
    if (own_scan) {
#define BLS_PLACE_SCAN(PERM, WGT) plan_place_tiles_scan<PERM, WGT><<<tgrid, kThreads, 0, st>>>(dd, tg, idx, off, nnz, C, sendcounts, sdispls, recvcounts, rdispls, segoff, ridx, perm, w_in, w_out)
        if (perm && w_in) BLS_PLACE_SCAN(true, true);
        else if (perm) BLS_PLACE_SCAN(true, false);
        else if (w_in) BLS_PLACE_SCAN(false, true);
        else BLS_PLACE_SCAN(false, false);
#undef BLS_PLACE_SCAN
    } else if (rowwise) {
        if (perm && w_in) plan_place_tiles<true, true><<<tgrid, kThreads, 0, st>>>(dd, tg, idx, off, nnz, X, segoff, ridx, perm, sabs, rabs, w_in, w_out);
        else if (perm) plan_place_tiles<true, false><<<tgrid, kThreads, 0, st>>>(dd, tg, idx, off, nnz, X, segoff, ridx, perm, sabs, rabs, w_in, w_out);
        else if (w_in) plan_place_tiles<false, true><<<tgrid, kThreads, 0, st>>>(dd, tg, idx, off, nnz, X, segoff, ridx, perm, sabs, rabs, w_in, w_out);
        else plan_place_tiles<false, false><<<tgrid, kThreads, 0, st>>>(dd, tg, idx, off, nnz, X, segoff, ridx, perm, sabs, rabs, w_in, w_out);
    } else {
        const int64_t runs = (int64_t)ctx->Q * ctx->P;
        const int64_t per_run = std::max<int64_t>(nnz / runs, n_max) + 1;
        const unsigned gx = (unsigned)std::min<int64_t>(256, std::max<int64_t>(1, (per_run + 2047) / 2048));
        dim3 grid(gx, (unsigned)std::min<int64_t>(runs, 65535));
        plan_place_runs<<<grid, kThreads, 0, st>>>(dd, idx, off, nnz, X, segoff, ridx, perm, sabs, rabs, w_in, w_out);
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
