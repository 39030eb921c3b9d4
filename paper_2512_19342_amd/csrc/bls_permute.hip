// bls_pack, bls_alltoallv_local, bls_unpack: pooled vectors moved between the pooled
// buffer Y, the per-destination send regions S, the receive regions R of a ring slot and
// the output.  All three are permutations of whole D-vectors (plus, for row-wise
// partitions, the sum of the P partial vectors in unpack), so a group of lanes moves one
// vector with 128-bit accesses and the only arithmetic is the address of the vector in
// each layout (y, sigma, rho in bls_internal.h).  Grid: x over samples, y = q.
#include "bls_internal.h"

namespace {

constexpr int kThreads = 256;

enum { kPack = 0, kExchange = 1, kUnpackTable = 2 };

// lanes per vector: power of two, 1..64, covering D / VEC columns where it can
inline int lanes_for(int64_t cols)
{
    int g = 1;
    while (g < cols && g < 64) g <<= 1;
    return g;
}

__device__ __forceinline__ void vdiv(float4 &a, float x) { a.x /= x; a.y /= x; a.z /= x; a.w /= x; }
__device__ __forceinline__ void vdiv(float &a, float x) { a /= x; }

// Length of bag (t, b) as a float divisor for mean pooling; 1 for an empty or malformed bag.
__device__ __forceinline__ float bag_divisor(const DevDesc &dd, const int64_t *off, int t, uint32_t b)
{
    const int64_t g = (int64_t)t * dd.B + b;
    const int64_t len = off[g + 1] - off[g];
    return len > 0 ? (float)len : 1.f;
}

template <int MODE, class V>
__global__ __launch_bounds__(kThreads) void move_vectors(DevDesc dd, const float *__restrict__ src,
                                                         float *__restrict__ dst, int lg,
                                                         const int64_t *__restrict__ mean_off, uint32_t b0, uint32_t bn)
{
    constexpr int VEC = sizeof(V) / sizeof(float);
    const int G = 1 << lg;
    const int q = blockIdx.y;
    const int li = threadIdx.x & (G - 1);
    const uint32_t b = b0 + blockIdx.x * (uint32_t)(kThreads >> lg) + (threadIdx.x >> lg);   // samples b0 .. b0+bn-1
    if (b >= b0 + bn) return;
    int s; uint32_t b_loc, n;
    bls_split_sample(dd, b, s, b_loc, n);
    int64_t from, to;
    if (MODE == kPack) {
        from = (int64_t)q * dd.B + b;
        to = bls_sigma(dd, q, s, b_loc, n);
    } else if (MODE == kExchange) {
        from = bls_sigma(dd, q, s, b_loc, n);
        to = bls_rho(dd, q, s, b_loc, n);
    } else {
        from = bls_rho(dd, q, s, b_loc, n);
        to = (int64_t)b * dd.T + dd.q_t[q];
    }
    const V *__restrict__ ps = reinterpret_cast<const V *>(src + from * dd.D);
    V *__restrict__ pd = reinterpret_cast<V *>(dst + to * dd.D);
    const int cols = dd.D / VEC;
    if (MODE == kUnpackTable && mean_off) {
        const float div = bag_divisor(dd, mean_off, dd.q_t[q], b);
        for (int c = li; c < cols; c += G) { V x = ps[c]; vdiv(x, div); pd[c] = x; }
    } else {
        for (int c = li; c < cols; c += G) pd[c] = ps[c];
    }
}

__device__ __forceinline__ void vadd(float4 &a, const float4 &x) { a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w; }
__device__ __forceinline__ void vadd(float &a, const float &x) { a += x; }
__device__ __forceinline__ void vzero(float4 &a) { a = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void vzero(float &a) { a = 0.f; }

// Row-wise completion: Out[b][t] = sum over owners d = 0..P-1 (in that order, from +0) of the
// partial vector rank d sent for (t, b).  Grid y = t.
template <class V>
__global__ __launch_bounds__(kThreads) void unpack_rowwise(DevDesc dd, const float *__restrict__ R,
                                                           float *__restrict__ out, int lg,
                                                           const int64_t *__restrict__ mean_off, uint32_t b0, uint32_t bn)
{
    constexpr int VEC = sizeof(V) / sizeof(float);
    const int G = 1 << lg;
    const int t = blockIdx.y;
    const int li = threadIdx.x & (G - 1);
    const uint32_t b = b0 + blockIdx.x * (uint32_t)(kThreads >> lg) + (threadIdx.x >> lg);
    if (b >= b0 + bn) return;
    int s; uint32_t b_loc, n;
    bls_split_sample(dd, b, s, b_loc, n);
    V *__restrict__ pd = reinterpret_cast<V *>(out + ((int64_t)b * dd.T + t) * dd.D);
    const int cols = dd.D / VEC;
    const float div = mean_off ? bag_divisor(dd, mean_off, t, b) : 1.f;
    for (int c = li; c < cols; c += G) {
        V acc;
        vzero(acc);
        for (int d = 0; d < dd.P; ++d) {
            const V *__restrict__ ps = reinterpret_cast<const V *>(R + bls_rho(dd, d * dd.T + t, s, b_loc, n) * dd.D);
            vadd(acc, ps[c]);
        }
        if (mean_off) vdiv(acc, div);
        pd[c] = acc;
    }
}

template <int MODE>
int launch_move(bls_ctx *ctx, const float *src, float *dst, const int64_t *mean_off, uint32_t b0, uint32_t bn, hipStream_t st)
{
    if (bn == 0) return BLS_OK;
    const bool vec = ctx->D % 4 == 0;
    const int g = lanes_for(vec ? ctx->D / 4 : ctx->D);
    int lg = 0;
    while ((1 << lg) < g) ++lg;
    const uint32_t per_block = kThreads >> lg;
    dim3 grid((unsigned)((bn + per_block - 1) / per_block), ctx->Q);
    if (vec) move_vectors<MODE, float4><<<grid, kThreads, 0, st>>>(ctx->desc, src, dst, lg, mean_off, b0, bn);
    else move_vectors<MODE, float><<<grid, kThreads, 0, st>>>(ctx->desc, src, dst, lg, mean_off, b0, bn);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
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

int bls_launch_pack(bls_ctx *ctx, const float *Y, float *S, hipStream_t st) { return launch_move<kPack>(ctx, Y, S, nullptr, 0u, (uint32_t)ctx->B, st); }

int bls_launch_exchange(bls_ctx *ctx, const float *S, float *R, hipStream_t st)
{
    return launch_move<kExchange>(ctx, S, R, nullptr, 0u, (uint32_t)ctx->B, st);
}

int bls_launch_unpack(bls_ctx *ctx, const float *R, float *out, const int64_t *mean_off, uint32_t b0, uint32_t bn,
                      hipStream_t st)
{
    if (bn == 0) return BLS_OK;
    if (ctx->part_kind == BLS_TABLE_WISE) return launch_move<kUnpackTable>(ctx, R, out, mean_off, b0, bn, st);
    const bool vec = ctx->D % 4 == 0;
    const int g = lanes_for(vec ? ctx->D / 4 : ctx->D);
    int lg = 0;
    while ((1 << lg) < g) ++lg;
    const uint32_t per_block = kThreads >> lg;
    dim3 grid((unsigned)((bn + per_block - 1) / per_block), ctx->T);
    if (vec) unpack_rowwise<float4><<<grid, kThreads, 0, st>>>(ctx->desc, R, out, lg, mean_off, b0, bn);
    else unpack_rowwise<float><<<grid, kThreads, 0, st>>>(ctx->desc, R, out, lg, mean_off, b0, bn);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
