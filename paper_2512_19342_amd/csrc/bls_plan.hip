// bls_plan: index bucketing by owning rank.
//
// Every lookup belongs to exactly one segment (owner d, requester s, local table, local
// sample), and segments are numbered in owner order, so
//   1. count   - the length of every segment (table-wise: the bag length; row-wise: a
//                group of lanes per bag splits its lookups over the P owners: packed byte
//                counters summed over the lanes for P <= 8, one ballot per owner otherwise),
//   2. scan    - an exclusive scan of the segment lengths (LDS-staged, three phases) gives
//                segoff, and the alltoallv counts and displacements are differences of
//                segoff at the (d, s) block edges - no atomics, no separate histogram,
//   3. scatter - every lookup is written to segoff[segment] + its rank among the
//                segment's earlier lookups (lane prefix counts), which is the stable order.
#include <algorithm>

#include "bls_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 16;                       // scan items per thread
constexpr int kChunk = kThreads * kItems;        // scan items per block
constexpr int kSmallScanTiles = 2;               // up to this many tiles one workgroup scans alone
constexpr int kAhead = 4;                        // row-wise kernels: chunks of a bag's indices loaded ahead

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

// ---- 1. count ------------------------------------------------------------------------

// Table-wise: one thread per (q, b); the segment is the whole bag.
__global__ __launch_bounds__(kThreads) void plan_count_tablewise(DevDesc dd, const int64_t *__restrict__ off,
                                                                 int64_t nnz, int64_t *__restrict__ seglen)
{
    const int q = blockIdx.y;
    const uint32_t b = blockIdx.x * kThreads + threadIdx.x;
    if (b >= (uint32_t)dd.B) return;
    const int64_t g = (int64_t)dd.q_t[q] * dd.B + b;
    const int64_t lo = off[g], hi = off[g + 1];
    int64_t len = hi - lo;
    if (lo < 0 || hi > nnz || len < 0) { flag_error(dd); len = 0; }
    int s; uint32_t b_loc, n;
    bls_split_sample(dd, b, s, b_loc, n);
    seglen[bls_sigma(dd, q, s, b_loc, n)] = len;
}

__device__ __forceinline__ int owner_of_row(int64_t ix, int64_t rps)
{
    return rps <= 0xffffffffLL && ix <= 0xffffffffLL ? (int)((uint32_t)ix / (uint32_t)rps) : (int)(ix / rps);
}

// Row-wise: a group of G >= P lanes per bag (t, b), several bags per wavefront.  One ballot
// per owner tells every group how many of its lookups fall in that owner's block of rows;
// lane o of the group accumulates owner o's count.
template <int G>
__global__ __launch_bounds__(kThreads) void plan_count_rowwise(DevDesc dd, const int64_t *__restrict__ idx,
                                                               const int64_t *__restrict__ off, int64_t nnz,
                                                               int64_t *__restrict__ seglen)
{
    const int lane = threadIdx.x & 63;
    const int li = lane & (G - 1), gbase = lane & ~(G - 1);
    const unsigned long long gmask = G == 64 ? ~0ull : (1ull << (G & 63)) - 1ull;
    const int t = blockIdx.y;
    const uint32_t b = blockIdx.x * (kThreads / G) + threadIdx.x / G;
    const bool live = b < (uint32_t)dd.B;
    int64_t lo = 0, len = 0;
    if (live) {
        const int64_t g = (int64_t)t * dd.B + b;
        lo = off[g];
        const int64_t hi = off[g + 1];
        len = hi - lo;
        if (lo < 0 || hi > nnz || len < 0) { if (li == 0) flag_error(dd); len = 0; }
    }
    const int64_t rows = dd.rows[t], rps = dd.rps[t];
    int64_t cnt = 0;
    // a bag is a handful of chunks and every chunk a dependent round trip: the indices of the next
    // kAhead chunks are always in flight while the current one is counted
    int64_t nx[kAhead];
#pragma unroll
    for (int a = 0; a < kAhead; ++a) nx[a] = a * G + li < len ? idx[lo + a * G + li] : 0;
    for (int64_t c = 0; __any(c < len); c += G) {
        const int64_t j = c + li;
        const int64_t ix = nx[0];
#pragma unroll
        for (int a = 0; a + 1 < kAhead; ++a) nx[a] = nx[a + 1];
        nx[kAhead - 1] = j + kAhead * G < len ? idx[lo + j + kAhead * G] : 0;
        int d = -1;
        if (j < len) {
            if (ix < 0 || ix >= rows) flag_error(dd);
            else d = owner_of_row(ix, rps);
        }
        if (dd.P <= 8) {
            // up to eight owners: one byte per owner in a 64-bit word, summed over the group's lanes
            unsigned long long pk = d >= 0 ? 1ull << (8 * d) : 0ull;
#pragma unroll
            for (int o = G / 2; o >= 1; o >>= 1) pk += __shfl_xor(pk, o, 64);
            cnt += (int64_t)((pk >> (8 * (li & 7))) & 0xffull);
        } else {
            for (int o = 0; o < dd.P; ++o) {
                const unsigned long long m = (__ballot(d == o) >> gbase) & gmask;
                if (li == o) cnt += __popcll(m);
            }
        }
    }
    if (live && li < dd.P) {
        int s; uint32_t b_loc, n;
        bls_split_sample(dd, b, s, b_loc, n);
        seglen[bls_sigma_rowwise(dd, li, t, s, b_loc, n)] = cnt;
    }
}

// ---- 2. scan ---------------------------------------------------------------------------
// In-place inclusive scan of v[0..n) (v = segoff + 1, holding segment lengths), so that
// segoff becomes the exclusive scan with segoff[nseg] = total.

__global__ __launch_bounds__(kThreads) void scan_block_sums(const int64_t *__restrict__ v, int64_t n,
                                                            int64_t *__restrict__ sums)
{
    __shared__ int64_t part[kThreads / 64];
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
        for (int w = 0; w < kThreads / 64; ++w) tot += part[w];
        sums[blockIdx.x] = tot;
    }
}

// One block: exclusive scan of the block sums, in place.
__global__ __launch_bounds__(kThreads) void scan_spine(int64_t *__restrict__ sums, int64_t nblk)
{
    __shared__ int64_t part[kThreads / 64];
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

// Inclusive scan of one tile v[base .. base + kChunk) in place, offset by `carry`; returns
// carry + the tile's total (the same value in every thread).  Items are staged in LDS so that
// global accesses stay coalesced while every thread owns a contiguous run; one padding word
// per run keeps the per-thread walks off one bank.
__device__ __forceinline__ int64_t scan_tile(int64_t *__restrict__ v, int64_t n, int64_t base, int64_t carry,
                                             int64_t *tile, int64_t *part)
{
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int e = k * kThreads + threadIdx.x;
        const int64_t i = base + e;
        tile[e + e / kItems] = i < n ? v[i] : 0;
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
    for (int w = 0; w < kThreads / 64; ++w) {
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

__global__ __launch_bounds__(kThreads) void scan_apply(int64_t *__restrict__ v, int64_t n,
                                                       const int64_t *__restrict__ sums, int64_t *__restrict__ head)
{
    __shared__ int64_t tile[kChunk + kThreads];
    __shared__ int64_t part[kThreads / 64];
    if (blockIdx.x == 0 && threadIdx.x == 0) *head = 0;   // segoff[0]
    scan_tile(v, n, (int64_t)blockIdx.x * kChunk, sums[blockIdx.x], tile, part);
}

// Counts and displacements from segoff at the (d, s) block edges, by one workgroup.
// sabs[s][d] / rabs[d][s]: absolute start of bucket (s, d) in requester / owner order.
__device__ __forceinline__ void finish_counts(const DevDesc &dd, const int64_t *__restrict__ segoff,
                                              int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                              int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                              int64_t *__restrict__ sabs, int64_t *__restrict__ rabs, int64_t *rowtot)
{
    const int P = dd.P;
    for (int e = threadIdx.x; e < P * P; e += kThreads) {
        const int d = e / P, s = e - d * P;
        const int64_t edge0 = (int64_t)dd.nsum[d] * dd.B;
        const int64_t lo = segoff[edge0 + (int64_t)dd.n_loc[d] * dd.first[s]];
        const int64_t hi = segoff[edge0 + (int64_t)dd.n_loc[d] * dd.first[s + 1]];
        recvcounts[d * P + s] = hi - lo;
        rdispls[d * P + s] = lo - segoff[edge0];
        rabs[d * P + s] = lo;
        sendcounts[s * P + d] = hi - lo;
    }
    __syncthreads();
    if (threadIdx.x < P) {
        const int s = threadIdx.x;
        int64_t run = 0;
        for (int d = 0; d < P; ++d) { sdispls[s * P + d] = run; run += sendcounts[s * P + d]; }
        rowtot[s] = run;
    }
    __syncthreads();
    if (threadIdx.x < P) {
        const int s = threadIdx.x;
        int64_t sbase = 0;
        for (int r = 0; r < s; ++r) sbase += rowtot[r];
        for (int d = 0; d < P; ++d) sabs[s * P + d] = sbase + sdispls[s * P + d];
    }
}

__global__ __launch_bounds__(kThreads) void plan_finish(DevDesc dd, const int64_t *__restrict__ segoff,
                                                        int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                        int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                        int64_t *__restrict__ sabs, int64_t *__restrict__ rabs)
{
    __shared__ int64_t rowtot[64];
    finish_counts(dd, segoff, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs, rowtot);
}

// Small problems are bound by the number of launches: one workgroup scans all tiles in turn and
// derives the counts, in place of the three scan kernels and plan_finish.
__global__ __launch_bounds__(kThreads) void plan_scan_small(DevDesc dd, int64_t *__restrict__ segoff, int64_t n,
                                                            int64_t *__restrict__ sendcounts, int64_t *__restrict__ sdispls,
                                                            int64_t *__restrict__ recvcounts, int64_t *__restrict__ rdispls,
                                                            int64_t *__restrict__ sabs, int64_t *__restrict__ rabs)
{
    __shared__ int64_t tile[kChunk + kThreads];
    __shared__ int64_t part[kThreads / 64];
    __shared__ int64_t rowtot[64];
    if (threadIdx.x == 0) segoff[0] = 0;
    int64_t carry = 0;
    for (int64_t base = 0; base < n; base += kChunk) carry = scan_tile(segoff + 1, n, base, carry, tile, part);
    __syncthreads();                                  // every segoff entry written by this workgroup is visible to it
    finish_counts(dd, segoff, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs, rowtot);
}

// ---- 3. scatter ------------------------------------------------------------------------

// Table-wise: all bags of one table in one rank's mini-batch - a run (q, s) - are contiguous
// both in input order and in owner order, so the scatter is Q*P block copies of index
// lists.  grid: x strides over a run, y strides over the runs.
__global__ __launch_bounds__(kThreads) void plan_scatter_runs(DevDesc dd, const int64_t *__restrict__ idx,
                                                              const int64_t *__restrict__ off, int64_t nnz,
                                                              const int64_t *__restrict__ segoff,
                                                              int64_t *__restrict__ ridx, int64_t *__restrict__ perm,
                                                              const int64_t *__restrict__ sabs,
                                                              const int64_t *__restrict__ rabs,
                                                              const float *__restrict__ w_in, float *__restrict__ w_out)
{
    constexpr int kPer = 4;
    for (int run = blockIdx.y; run < dd.Q * dd.P; run += gridDim.y) {
        const int q = run / dd.P, s = run - q * dd.P;
        const int t = dd.q_t[q], d = dd.q_d[q];
        const int64_t lo = off[(int64_t)t * dd.B + dd.first[s]], hi = off[(int64_t)t * dd.B + dd.first[s + 1]];
        const int64_t len = hi - lo;
        if (lo < 0 || hi > nnz || len <= 0) continue;        // bad offsets are flagged by the count kernel
        const int64_t n = dd.first[s + 1] - dd.first[s];
        const int64_t dst = segoff[(int64_t)dd.nsum[d] * dd.B + (int64_t)dd.n_loc[d] * dd.first[s] + (int64_t)(q - dd.nsum[d]) * n];
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

// Row-wise: a group of G >= P lanes per bag.  Lane o of the group holds the start of owner
// o's segment and how many of the bag's lookups it has already received; a lookup's place is
// that start plus the number of earlier lanes of the group with the same owner.
template <int G>
__global__ __launch_bounds__(kThreads) void plan_scatter_rowwise(DevDesc dd, const int64_t *__restrict__ idx,
                                                                 const int64_t *__restrict__ off, int64_t nnz,
                                                                 const int64_t *__restrict__ segoff,
                                                                 int64_t *__restrict__ ridx, int64_t *__restrict__ perm,
                                                                 const int64_t *__restrict__ sabs,
                                                                 const int64_t *__restrict__ rabs,
                                                                 const float *__restrict__ w_in, float *__restrict__ w_out)
{
    const int lane = threadIdx.x & 63;
    const int li = lane & (G - 1), gbase = lane & ~(G - 1);
    const unsigned long long gmask = G == 64 ? ~0ull : (1ull << (G & 63)) - 1ull;
    const unsigned long long below = (1ull << li) - 1ull;
    const int t = blockIdx.y;
    const uint32_t b = blockIdx.x * (kThreads / G) + threadIdx.x / G;
    const bool live = b < (uint32_t)dd.B;
    int64_t lo = 0, len = 0;
    int64_t next = 0, to_send = 0;                        // lane o: next free place of owner o
    if (live) {
        const int64_t g = (int64_t)t * dd.B + b;
        lo = off[g];
        const int64_t hi = off[g + 1];
        len = hi - lo;
        if (lo < 0 || hi > nnz || len < 0) len = 0;       // flagged by the count kernel
        if (li < dd.P) {
            int s; uint32_t b_loc, n;
            bls_split_sample(dd, b, s, b_loc, n);
            next = segoff[bls_sigma_rowwise(dd, li, t, s, b_loc, n)];
            if (perm) to_send = sabs[s * dd.P + li] - rabs[li * dd.P + s];
        }
    }
    const int64_t rows = dd.rows[t], rps = dd.rps[t];
    // a bag is a handful of chunks and every chunk a dependent round trip: the indices of the next
    // kAhead chunks are always in flight while the current one is placed
    int64_t nx[kAhead];
#pragma unroll
    for (int a = 0; a < kAhead; ++a) nx[a] = a * G + li < len ? idx[lo + a * G + li] : 0;
    for (int64_t c = 0; __any(c < len); c += G) {
        const int64_t j = c + li;
        const int64_t ix = nx[0];
#pragma unroll
        for (int a = 0; a + 1 < kAhead; ++a) nx[a] = nx[a + 1];
        nx[kAhead - 1] = j + kAhead * G < len ? idx[lo + j + kAhead * G] : 0;
        int d = -1;
        int64_t r = 0;
        if (j < len) {
            if (ix >= 0 && ix < rows) { d = owner_of_row(ix, rps); r = ix - (int64_t)d * rps; }
        }
        int rank = 0, add = 0;
        if (dd.P <= 8) {
            // one byte per owner: a prefix sum over the group's lanes gives every lookup its rank among
            // the earlier ones of the same owner, the last lane's sum the chunk's count per owner
            const unsigned long long pk = d >= 0 ? 1ull << (8 * d) : 0ull;
            unsigned long long pre = pk;
#pragma unroll
            for (int o = 1; o < G; o <<= 1) {
                const unsigned long long v = __shfl_up(pre, o, G);
                if (li >= o) pre += v;
            }
            if (d >= 0) rank = (int)(((pre - pk) >> (8 * d)) & 0xffull);
            const unsigned long long total = __shfl(pre, gbase + G - 1, 64);
            add = (int)((total >> (8 * (li & 7))) & 0xffull);
        } else {
            for (int o = 0; o < dd.P; ++o) {
                const unsigned long long m = (__ballot(d == o) >> gbase) & gmask;
                if (d == o) rank = __popcll(m & below);
                if (li == o) add = __popcll(m);
            }
        }
        const int src = gbase + (d < 0 ? 0 : d);
        const int64_t place = __shfl(next, src, 64) + rank;
        const int64_t shift = __shfl(to_send, src, 64);
        if (d >= 0) {
            if (place >= 0 && place < nnz) {
                ridx[place] = r;
                if (w_in) w_out[place] = w_in[lo + j];
                if (perm) perm[lo + j] = place + shift;
            } else flag_error(dd);
        }
        next += add;
    }
}

int64_t scan_blocks(int64_t n) { return (n + kChunk - 1) / kChunk; }

}  // namespace

size_t bls_plan_ws_bytes(const bls_ctx *ctx)
{
    return (size_t)(scan_blocks(ctx->nseg) + 2 * ctx->P * ctx->P + 2) * sizeof(int64_t);
}

int bls_launch_plan(bls_ctx *ctx, const int64_t *idx, const int64_t *off, int64_t nnz, int64_t *sendcounts,
                    int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls, int64_t *ridx, int64_t *segoff,
                    int64_t *perm, const float *w_in, float *w_out, void *ws, size_t ws_bytes, hipStream_t st)
{
    (void)ws_bytes;
    const DevDesc &dd = ctx->desc;
    const int64_t nseg = ctx->nseg, nblk = scan_blocks(nseg);
    int64_t *sums = (int64_t *)ws;
    int64_t *sabs = sums + nblk, *rabs = sabs + ctx->P * ctx->P;
    const uint32_t B = (uint32_t)ctx->B;
    const bool rowwise = ctx->part_kind == BLS_ROW_WISE;

    // lanes per bag for row-wise partitions: at least P (lane o keeps owner o's counters)
    const int rg = ctx->P <= 8 ? 8 : ctx->P <= 16 ? 16 : ctx->P <= 32 ? 32 : 64;
    const dim3 rgrid((B + kThreads / rg - 1) / (kThreads / rg), ctx->T);
    if (rowwise) {
        switch (rg) {
        case 8: plan_count_rowwise<8><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff + 1); break;
        case 16: plan_count_rowwise<16><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff + 1); break;
        case 32: plan_count_rowwise<32><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff + 1); break;
        default: plan_count_rowwise<64><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff + 1); break;
        }
    } else {
        dim3 grid((B + kThreads - 1) / kThreads, ctx->Q);
        plan_count_tablewise<<<grid, kThreads, 0, st>>>(dd, off, nnz, segoff + 1);
    }
    if (nblk <= kSmallScanTiles) {
        plan_scan_small<<<1, kThreads, 0, st>>>(dd, segoff, nseg, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs);
    } else {
        scan_block_sums<<<dim3((unsigned)nblk), kThreads, 0, st>>>(segoff + 1, nseg, sums);
        scan_spine<<<1, kThreads, 0, st>>>(sums, nblk);
        scan_apply<<<dim3((unsigned)nblk), kThreads, 0, st>>>(segoff + 1, nseg, sums, segoff);
        plan_finish<<<1, kThreads, 0, st>>>(dd, segoff, sendcounts, sdispls, recvcounts, rdispls, sabs, rabs);
    }
    if (nnz > 0) {
        if (rowwise) {
            switch (rg) {
            case 8: plan_scatter_rowwise<8><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff, ridx, perm, sabs, rabs, w_in, w_out); break;
            case 16: plan_scatter_rowwise<16><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff, ridx, perm, sabs, rabs, w_in, w_out); break;
            case 32: plan_scatter_rowwise<32><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff, ridx, perm, sabs, rabs, w_in, w_out); break;
            default: plan_scatter_rowwise<64><<<rgrid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff, ridx, perm, sabs, rabs, w_in, w_out); break;
            }
        } else {
            const int64_t runs = (int64_t)ctx->Q * ctx->P;
            const int64_t per_run = nnz / runs + 1;
            const unsigned gx = (unsigned)std::min<int64_t>(256, std::max<int64_t>(1, (per_run + 2047) / 2048));
            dim3 grid(gx, (unsigned)std::min<int64_t>(runs, 65535));
            plan_scatter_runs<<<grid, kThreads, 0, st>>>(dd, idx, off, nnz, segoff, ridx, perm, sabs, rabs, w_in, w_out);
        }
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
