// bls_pack, bls_alltoallv_local, bls_unpack: pooled vectors moved between the pooled
// buffer Y, the per-destination send regions S, the receive regions R of a ring slot and
// the output.  All three are permutations of whole D-vectors (plus, for row-wise
// partitions, the sum of the P partial vectors in unpack), so a group of lanes moves one
// vector with 128-bit accesses and the only arithmetic is the address of the vector in
// each layout (y, sigma, rho in bls_internal.h).
//
// Workgroups are numbered so that one side of every move is walked front to back as a single
// stream (measured: 5.7-6.1 TB/s of read + write traffic, against 4.6-5.0 when both sides are
// eight interleaved streams): pack reads Y in order, the exchange writes the slot in order,
// unpack reads the slot in order.
#include <stdlib.h>

#include <algorithm>

#include "bls_internal.h"

namespace {

constexpr int kThreads = 256;

// log2 of the lanes per vector: a power of two, 1..64, covering D / VEC columns where it can
inline int lanes_log2(int64_t cols)
{
    int lg = 0;
    while ((1 << lg) < cols && lg < 6) ++lg;
    return lg;
}

__device__ __forceinline__ void vdiv(float4 &a, float x) { a.x /= x; a.y /= x; a.z /= x; a.w /= x; }
__device__ __forceinline__ void vdiv(float &a, float x) { a /= x; }
__device__ __forceinline__ void vadd(float4 &a, const float4 &x) { a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w; }
__device__ __forceinline__ void vadd(float &a, const float &x) { a += x; }
__device__ __forceinline__ void vzero(float4 &a) { a = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void vzero(float &a) { a = 0.f; }

// Length of bag (t, b) as a float divisor for mean pooling; 1 for an empty or malformed bag.
__device__ __forceinline__ float bag_divisor(const DevDesc &dd, const int64_t *off, int t, uint32_t b)
{
    const int64_t g = (int64_t)t * dd.B + b;
    const int64_t len = off[g + 1] - off[g];
    return len > 0 ? (float)len : 1.f;
}

// Pack: Y (read front to back) -> send regions.  Grid: x over groups of samples, y = q.
template <class V>
__global__ __launch_bounds__(kThreads) void pack_vectors(DevDesc dd, const float *__restrict__ Y, float *__restrict__ S, int lg)
{
    constexpr int VEC = sizeof(V) / sizeof(float);
    const int G = 1 << lg;
    const int q = blockIdx.y;
    const int li = threadIdx.x & (G - 1);
    const uint32_t b = blockIdx.x * (uint32_t)(kThreads >> lg) + (threadIdx.x >> lg);
    if (b >= (uint32_t)dd.B) return;
    int s; uint32_t b_loc, n;
    bls_split_sample(dd, b, s, b_loc, n);
    const V *__restrict__ ps = reinterpret_cast<const V *>(Y + ((int64_t)q * dd.B + b) * dd.D);
    V *__restrict__ pd = reinterpret_cast<V *>(S + bls_sigma(dd, q, s, b_loc, n) * dd.D);
    const int cols = dd.D / VEC;
    for (int c = li; c < cols; c += G) pd[c] = ps[c];
}

// Position of a workgroup in receive order: requester s = s0 + ..., then `rows` rows (the Q
// (owner, table) pairs, or the T tables), then chunks of the mini-batch.
struct RecvPos { int s, row; uint32_t b_loc, n; bool live; };

__device__ __forceinline__ RecvPos recv_position(const DevDesc &dd, int lg, uint32_t chunks, uint32_t rows, int s0,
                                                 uint32_t b0, uint32_t bn)
{
    RecvPos p;
    const uint32_t chunk = blockIdx.x % chunks, sr = blockIdx.x / chunks;
    p.row = (int)(sr % rows);
    p.s = s0 + (int)(sr / rows);
    const int64_t f = dd.first[p.s];
    p.n = (uint32_t)(dd.first[p.s + 1] - f);
    p.b_loc = chunk * (uint32_t)(kThreads >> lg) + (threadIdx.x >> lg);
    const int64_t b = f + p.b_loc;
    p.live = p.b_loc < p.n && b >= (int64_t)b0 && b < (int64_t)b0 + bn;   // samples b0 .. b0+bn-1 only
    return p;
}

// Exchange: send regions -> the slot, written front to back.  Grid: x over (s, q, chunk).
template <class V>
__global__ __launch_bounds__(kThreads) void exchange_vectors(DevDesc dd, const float *__restrict__ S, float *__restrict__ R,
                                                             int lg, uint32_t chunks)
{
    constexpr int VEC = sizeof(V) / sizeof(float);
    const int G = 1 << lg;
    const int li = threadIdx.x & (G - 1);
    const RecvPos p = recv_position(dd, lg, chunks, (uint32_t)dd.Q, 0, 0u, (uint32_t)dd.B);
    if (!p.live) return;
    const V *__restrict__ ps = reinterpret_cast<const V *>(S + bls_sigma(dd, p.row, p.s, p.b_loc, p.n) * dd.D);
    V *__restrict__ pd = reinterpret_cast<V *>(R + bls_rho(dd, p.row, p.s, p.b_loc, p.n) * dd.D);
    const int cols = dd.D / VEC;
    for (int c = li; c < cols; c += G) pd[c] = ps[c];
}

// Table-wise completion: the slot, read front to back -> Out[b][t].  Grid: x over (s, q, chunk).
template <class V>
__global__ __launch_bounds__(kThreads) void unpack_tablewise(DevDesc dd, const float *__restrict__ R, float *__restrict__ out,
                                                             int lg, uint32_t chunks, int s0,
                                                             const int64_t *__restrict__ mean_off, uint32_t b0, uint32_t bn)
{
    constexpr int VEC = sizeof(V) / sizeof(float);
    const int G = 1 << lg;
    const int li = threadIdx.x & (G - 1);
    const RecvPos p = recv_position(dd, lg, chunks, (uint32_t)dd.Q, s0, b0, bn);
    if (!p.live) return;
    const int t = dd.q_t[p.row];
    const int64_t b = dd.first[p.s] + p.b_loc;
    const V *__restrict__ ps = reinterpret_cast<const V *>(R + bls_rho(dd, p.row, p.s, p.b_loc, p.n) * dd.D);
    V *__restrict__ pd = reinterpret_cast<V *>(out + (b * dd.T + t) * dd.D);
    const int cols = dd.D / VEC;
    if (mean_off) {
        const float div = bag_divisor(dd, mean_off, t, (uint32_t)b);
        for (int c = li; c < cols; c += G) { V x = ps[c]; vdiv(x, div); pd[c] = x; }
    } else {
        for (int c = li; c < cols; c += G) pd[c] = ps[c];
    }
}

// Row-wise completion: Out[b][t] = sum over owners d = 0..P-1 (in that order, from +0) of the
// partial vector rank d sent for (t, b).  Grid: x over (s, t, chunk): every owner's region of the
// slot is read front to back.
template <class V>
__global__ __launch_bounds__(kThreads) void unpack_rowwise(DevDesc dd, const float *__restrict__ R, float *__restrict__ out,
                                                           int lg, uint32_t chunks, int s0,
                                                           const int64_t *__restrict__ mean_off, uint32_t b0, uint32_t bn)
{
    constexpr int VEC = sizeof(V) / sizeof(float);
    const int G = 1 << lg;
    const int li = threadIdx.x & (G - 1);
    const RecvPos p = recv_position(dd, lg, chunks, (uint32_t)dd.T, s0, b0, bn);
    if (!p.live) return;
    const int t = p.row;
    const int64_t b = dd.first[p.s] + p.b_loc;
    V *__restrict__ pd = reinterpret_cast<V *>(out + (b * dd.T + t) * dd.D);
    const int cols = dd.D / VEC;
    const float div = mean_off ? bag_divisor(dd, mean_off, t, (uint32_t)b) : 1.f;
    for (int c = li; c < cols; c += G) {
        V acc;
        vzero(acc);
        for (int d = 0; d < dd.P; ++d) {
            const V *__restrict__ ps = reinterpret_cast<const V *>(R + bls_rho(dd, d * dd.T + t, p.s, p.b_loc, p.n) * dd.D);
            vadd(acc, ps[c]);
        }
        if (mean_off) vdiv(acc, div);
        pd[c] = acc;
    }
}

// Keeps a stream busy for about `ticks` of the constant-rate wall clock (a modelled straggler).
// One lane sleeps in short naps; the loop is bounded, so the kernel always ends.
__global__ void delay_kernel(unsigned long long ticks, unsigned int max_naps)
{
    const unsigned long long t0 = wall_clock64();
    for (unsigned int i = 0; i < max_naps && wall_clock64() - t0 < ticks; ++i) __builtin_amdgcn_s_sleep(16);
}

}  // namespace

int bls_launch_delay(bls_ctx *ctx, uint32_t microseconds, hipStream_t st)
{
    int dev = 0, khz = 0;
    BLS_HIP(ctx, hipGetDevice(&dev));
    BLS_HIP(ctx, hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) khz = 100000;                               // 100 MHz
    const unsigned long long ticks = (unsigned long long)microseconds * (unsigned long long)khz / 1000ull;
    // a nap is at least 16 * 64 clocks; 64 naps per microsecond asked for is far more than needed
    delay_kernel<<<1, 1, 0, st>>>(ticks, microseconds * 64u + 1024u);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

int bls_launch_pack(bls_ctx *ctx, const float *Y, float *S, hipStream_t st)
{
    const bool vec = ctx->D % 4 == 0;
    const int lg = lanes_log2(vec ? ctx->D / 4 : ctx->D);
    const uint32_t per_block = kThreads >> lg;
    const dim3 grid((unsigned)((ctx->B + per_block - 1) / per_block), (unsigned)ctx->Q);
    if (vec) pack_vectors<float4><<<grid, kThreads, 0, st>>>(ctx->desc, Y, S, lg);
    else pack_vectors<float><<<grid, kThreads, 0, st>>>(ctx->desc, Y, S, lg);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

// workgroups for `rows` rows of the requesters s0 .. s1, every mini-batch cut into chunks
static int recv_grid(bls_ctx *ctx, int lg, uint32_t rows, int s0, int s1, uint32_t *chunks, dim3 *grid)
{
    const uint32_t per_block = kThreads >> lg;
    const int64_t n_max = (ctx->B + ctx->P - 1) / ctx->P;
    *chunks = (uint32_t)((n_max + per_block - 1) / per_block);
    const uint64_t blocks = (uint64_t)*chunks * rows * (uint64_t)(s1 - s0 + 1);
    if (blocks > 0x7fffffffull) return bls_fail(ctx, BLS_EINVAL, "too many vectors for one launch");
    *grid = dim3((unsigned)blocks);
    return BLS_OK;
}

int bls_launch_exchange(bls_ctx *ctx, const float *S, float *R, hipStream_t st)
{
    const bool vec = ctx->D % 4 == 0;
    const int lg = lanes_log2(vec ? ctx->D / 4 : ctx->D);
    uint32_t chunks;
    dim3 grid;
    const int rc = recv_grid(ctx, lg, (uint32_t)ctx->Q, 0, ctx->P - 1, &chunks, &grid);
    if (rc) return rc;
    if (vec) exchange_vectors<float4><<<grid, kThreads, 0, st>>>(ctx->desc, S, R, lg, chunks);
    else exchange_vectors<float><<<grid, kThreads, 0, st>>>(ctx->desc, S, R, lg, chunks);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

int bls_launch_unpack(bls_ctx *ctx, const float *R, float *out, const int64_t *mean_off, uint32_t b0, uint32_t bn,
                      hipStream_t st)
{
    if (bn == 0) return BLS_OK;
    const bool vec = ctx->D % 4 == 0;
    const int lg = lanes_log2(vec ? ctx->D / 4 : ctx->D);
    // requesters whose mini-batches meet samples b0 .. b0+bn-1
    int s0 = 0, s1 = ctx->P - 1;
    while (ctx->first[s0 + 1] <= (int64_t)b0) ++s0;
    while (ctx->first[s1] >= (int64_t)b0 + bn) --s1;
    const bool rowwise = ctx->part_kind == BLS_ROW_WISE;
    uint32_t chunks;
    dim3 grid;
    const int rc = recv_grid(ctx, lg, (uint32_t)(rowwise ? ctx->T : ctx->Q), s0, s1, &chunks, &grid);
    if (rc) return rc;
    if (rowwise) {
        if (vec) unpack_rowwise<float4><<<grid, kThreads, 0, st>>>(ctx->desc, R, out, lg, chunks, s0, mean_off, b0, bn);
        else unpack_rowwise<float><<<grid, kThreads, 0, st>>>(ctx->desc, R, out, lg, chunks, s0, mean_off, b0, bn);
    } else {
        if (vec) unpack_tablewise<float4><<<grid, kThreads, 0, st>>>(ctx->desc, R, out, lg, chunks, s0, mean_off, b0, bn);
        else unpack_tablewise<float><<<grid, kThreads, 0, st>>>(ctx->desc, R, out, lg, chunks, s0, mean_off, b0, bn);
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
