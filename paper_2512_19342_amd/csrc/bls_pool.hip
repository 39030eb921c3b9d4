// bls_embbag_pool: EmbeddingBag sum over HBM-resident table shards.
//
// A group of G lanes owns one segment (one bag's lookups at one owner); lane i of the
// group holds columns [i*V, (i+1)*V) of the pooled vector in registers, V = 16 bytes of
// table storage (4 fp32 or 8 fp16 values), so a row is fetched with one 128-bit load per
// lane and consecutive lanes read consecutive addresses.  G = row bytes / 16 rounded up to
// a power of two: a 512-byte row takes half a wavefront and a wavefront works on two bags
// at once, a 256-byte row takes a quarter.  The group first loads up to G of its row
// numbers with one coalesced load, then walks them U at a time: U independent row loads
// are issued before the first add so that many rows are in flight per lane, and the adds
// follow in segment order, which keeps the fp32 result identical to a sequential sum.
#include "bls_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr uint32_t kBadRow = 0xffffffffu;

__device__ __forceinline__ void flag_error(const DevDesc &dd) { atomicOr(dd.err, 1); }

template <int DT> struct Acc;

template <> struct Acc<BLS_FP32> {
    static constexpr int V = 4;
    float4 a;
    __device__ __forceinline__ void zero() { a = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void add(const uint4 &x)
    {
        a.x += __uint_as_float(x.x); a.y += __uint_as_float(x.y);
        a.z += __uint_as_float(x.z); a.w += __uint_as_float(x.w);
    }
    __device__ __forceinline__ void store(float *p) const { *reinterpret_cast<float4 *>(p) = a; }
};

// IEEE binary16 -> binary32 (exact; one v_cvt_f32_f16 each)
__device__ __forceinline__ float half_bits(unsigned short h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ __forceinline__ float half_lo(uint32_t w) { return half_bits((unsigned short)(w & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t w) { return half_bits((unsigned short)(w >> 16)); }

template <> struct Acc<BLS_FP16> {
    static constexpr int V = 8;
    float4 a, b;
    __device__ __forceinline__ void zero() { a = make_float4(0.f, 0.f, 0.f, 0.f); b = a; }
    __device__ __forceinline__ void add(const uint4 &x)
    {
        a.x += half_lo(x.x); a.y += half_hi(x.x); a.z += half_lo(x.y); a.w += half_hi(x.y);
        b.x += half_lo(x.z); b.y += half_hi(x.z); b.z += half_lo(x.w); b.w += half_hi(x.w);
    }
    __device__ __forceinline__ void store(float *p) const
    {
        reinterpret_cast<float4 *>(p)[0] = a;
        reinterpret_cast<float4 *>(p)[1] = b;
    }
};

// grid: x over groups of samples, y = q (owner, local table).
template <int G, int DT, int U>
__global__ __launch_bounds__(kThreads) void pool_rows(DevDesc dd, const int64_t *__restrict__ ridx,
                                                      const int64_t *__restrict__ segoff, int64_t nnz,
                                                      float *__restrict__ Y)
{
    using A = Acc<DT>;
    const int q = blockIdx.y;
    const int li = threadIdx.x & (G - 1);
    const int gbase = (threadIdx.x & 63) & ~(G - 1);
    const uint32_t b = blockIdx.x * (kThreads / G) + threadIdx.x / G;
    const bool live = b < (uint32_t)dd.B;
    const uint32_t row_bytes = (uint32_t)dd.D * (DT == BLS_FP16 ? 2u : 4u);
    const bool col_ok = (uint32_t)li * 16u < row_bytes;      // lanes past the row's end idle
    const char *__restrict__ base = (const char *)dd.q_base[q];
    const int64_t shard_rows = dd.q_rows[q];

    int64_t beg = 0, len = 0;
    if (live) {
        int s; uint32_t b_loc, n;
        bls_split_sample(dd, b, s, b_loc, n);
        const int64_t sg = bls_sigma(dd, q, s, b_loc, n);
        beg = segoff[sg];
        const int64_t end = segoff[sg + 1];
        len = end - beg;
        if (beg < 0 || len < 0 || end > nnz) { if (li == 0) flag_error(dd); len = 0; }
    }

    A acc;
    acc.zero();
    for (int64_t c0 = 0; __any(c0 < len); c0 += G) {
        const int64_t left = len - c0;
        const int rem = left < 0 ? 0 : (left > G ? G : (int)left);
        uint32_t mine = kBadRow;
        if (li < rem) {
            const int64_t r = ridx[beg + c0 + li];
            if (r < 0 || r >= shard_rows) flag_error(dd);
            else mine = (uint32_t)r;
        }
        for (int j = 0; __any(j < rem); j += U) {
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t r = (uint32_t)__shfl((int)mine, gbase + ((j + u) & (G - 1)), 64);
                v[u] = make_uint4(0u, 0u, 0u, 0u);
                if (j + u < rem && r != kBadRow && col_ok)
                    v[u] = *reinterpret_cast<const uint4 *>(base + (uint64_t)r * row_bytes + (uint32_t)li * 16u);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) acc.add(v[u]);      // adding +0 for skipped rows changes nothing
        }
    }
    if (live && col_ok) acc.store(Y + ((int64_t)q * dd.B + b) * dd.D + li * A::V);
}

// Any D (odd lengths, rows longer than 1 KB): one wavefront per segment, lanes stride the
// columns, scalar loads.
template <int DT>
__global__ __launch_bounds__(kThreads) void pool_rows_generic(DevDesc dd, const int64_t *__restrict__ ridx,
                                                              const int64_t *__restrict__ segoff, int64_t nnz,
                                                              float *__restrict__ Y)
{
    const int q = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const uint32_t b = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (b >= (uint32_t)dd.B) return;
    int s; uint32_t b_loc, n;
    bls_split_sample(dd, b, s, b_loc, n);
    const int64_t sg = bls_sigma(dd, q, s, b_loc, n);
    int64_t beg = segoff[sg], end = segoff[sg + 1];
    if (beg < 0 || end < beg || end > nnz) { if (lane == 0) flag_error(dd); end = beg = 0; }
    const int64_t shard_rows = dd.q_rows[q];
    const void *base = dd.q_base[q];
    float *y = Y + ((int64_t)q * dd.B + b) * dd.D;
    for (int c = lane; c < dd.D; c += 64) {
        float acc = 0.f;
        for (int64_t j = beg; j < end; ++j) {
            const int64_t r = ridx[j];
            if (r < 0 || r >= shard_rows) { if (c == 0) flag_error(dd); continue; }
            const int64_t e = r * dd.D + c;
            acc += DT == BLS_FP16 ? half_bits(((const unsigned short *)base)[e]) : ((const float *)base)[e];
        }
        y[c] = acc;
    }
}

template <int G, int DT>
void launch_rows(const bls_ctx *ctx, const int64_t *ridx, const int64_t *segoff, int64_t nnz, float *Y, hipStream_t st)
{
    constexpr int U = DT == BLS_FP16 ? 4 : 8;
    const uint32_t per_block = kThreads / G;
    dim3 grid((unsigned)((ctx->B + per_block - 1) / per_block), ctx->Q);
    pool_rows<G, DT, (U < G ? U : G)><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, segoff, nnz, Y);
}

template <int DT>
bool dispatch_rows(const bls_ctx *ctx, int lanes, const int64_t *ridx, const int64_t *segoff, int64_t nnz, float *Y,
                   hipStream_t st)
{
    switch (lanes) {
    case 1: launch_rows<1, DT>(ctx, ridx, segoff, nnz, Y, st); return true;
    case 2: launch_rows<2, DT>(ctx, ridx, segoff, nnz, Y, st); return true;
    case 4: launch_rows<4, DT>(ctx, ridx, segoff, nnz, Y, st); return true;
    case 8: launch_rows<8, DT>(ctx, ridx, segoff, nnz, Y, st); return true;
    case 16: launch_rows<16, DT>(ctx, ridx, segoff, nnz, Y, st); return true;
    case 32: launch_rows<32, DT>(ctx, ridx, segoff, nnz, Y, st); return true;
    case 64: launch_rows<64, DT>(ctx, ridx, segoff, nnz, Y, st); return true;
    }
    return false;
}

}  // namespace

int bls_launch_pool(bls_ctx *ctx, const int64_t *ridx, const int64_t *segoff, int64_t nnz, float *Y, hipStream_t st)
{
    const int64_t row_bytes = (int64_t)ctx->D * (ctx->dtype == BLS_FP16 ? 2 : 4);
    bool done = false;
    if (row_bytes % 16 == 0 && row_bytes <= 1024) {
        int lanes = 1;
        while (lanes * 16 < row_bytes) lanes <<= 1;
        done = ctx->dtype == BLS_FP16 ? dispatch_rows<BLS_FP16>(ctx, lanes, ridx, segoff, nnz, Y, st)
                                      : dispatch_rows<BLS_FP32>(ctx, lanes, ridx, segoff, nnz, Y, st);
    }
    if (!done) {
        dim3 grid((unsigned)((ctx->B + kThreads / 64 - 1) / (kThreads / 64)), ctx->Q);
        if (ctx->dtype == BLS_FP16) pool_rows_generic<BLS_FP16><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, segoff, nnz, Y);
        else pool_rows_generic<BLS_FP32><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, segoff, nnz, Y);
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
