// bls_embbag_pool: EmbeddingBag sum over HBM-resident table shards.
//
// A group of G lanes owns one segment (one bag's lookups at one owner); lane i of the
// group keeps the columns stored in bytes [i*VB, (i+1)*VB) of a row in registers, so a row
// is fetched with one load per lane and consecutive lanes read consecutive addresses.
// G*VB covers the row: a 512-byte row is read by a whole wavefront with 8 bytes per lane
// or by half a wavefront with 16.  The group first loads up to G of its row numbers with
// one coalesced load, then walks them U at a time: U independent row loads are issued
// before the first add so that many rows are in flight per lane, and the adds follow in
// segment order, which keeps the fp32 result identical to a sequential sum.
//
// Bags are short (tens of rows), so a group does not stop at one: it streams the rows of
// several consecutive segments - they are contiguous in ridx - and stores and clears its
// accumulator whenever the stream crosses a segment boundary.  That amortises the
// dependent loads at the start (segment offsets, then row numbers, then rows), lets the
// next block of row numbers be fetched while the current one is consumed, and evens out
// the lengths of the streams that share a wavefront.
#include <algorithm>
#include <type_traits>

#include "bls_internal.h"
#include "bls_rows.h"

namespace {

constexpr int kThreads = 256;
constexpr uint32_t kBadRow = 0xffffffffu;
#ifndef BLS_POOL_U
#define BLS_POOL_U 8
#endif
constexpr int kRowsInFlight = BLS_POOL_U;   // U: independent row loads issued per lane before the first add
#ifndef BLS_POOL_UQ
#define BLS_POOL_UQ 4
#endif
// row-quantised rows are four times shorter, so a load instruction carries four times as many rows:
// fewer per lane keep as many rows in flight with fewer registers (more wavefronts per SIMD)
constexpr int kRowsInFlightQuantised = BLS_POOL_UQ;

__device__ __forceinline__ void flag_error(const DevDesc &dd) { atomicOr(dd.err, 1); }

// 64-bit value of lane (gbase + k), k uniform.  A whole-wavefront group reads it into scalar
// registers; narrower groups use the lane permute network (two ds_bpermute, no vector ALU
// work beyond the address), which pipelines when several are issued back to back.
template <int G>
__device__ __forceinline__ uint32_t group_broadcast32(uint32_t v, int gbase4, int k)
{
    if constexpr (G == 64) return (uint32_t)__builtin_amdgcn_readlane((int)v, k);
    else return (uint32_t)__builtin_amdgcn_ds_bpermute(gbase4 + 4 * k, (int)v);
}

template <int G>
__device__ __forceinline__ uint64_t group_broadcast64(uint64_t v, int gbase4, int k)
{
    if constexpr (G == 64) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, k);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), k);
        return ((uint64_t)hi << 32) | lo;
    } else {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute(gbase4 + 4 * k, (int)(uint32_t)v);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute(gbase4 + 4 * k, (int)(uint32_t)(v >> 32));
        return ((uint64_t)hi << 32) | lo;
    }
}

// One segment per group of G lanes (used for G < 4, rows of 16 or 32 bytes).
// grid: x over groups of samples, y = q (owner, local table).
template <int G, int DT, int VB, int U>
__global__ __launch_bounds__(kThreads) void pool_rows(DevDesc dd, const int64_t *__restrict__ ridx,
                                                      const float *__restrict__ rw,
                                                      const int64_t *__restrict__ segoff, int64_t nnz,
                                                      float *__restrict__ Y, int to_slot, int q0)
{
    using A = Acc<DT, VB>;
    const int q = q0 + blockIdx.y;
    const int li = threadIdx.x & (G - 1);
    const int gbase = (threadIdx.x & 63) & ~(G - 1);
    const uint32_t b = blockIdx.x * (kThreads / G) + threadIdx.x / G;
    const bool live = b < (uint32_t)dd.B;
    const uint32_t row_bytes = (uint32_t)payload_bytes(DT, dd.D), row_stride = (uint32_t)stride_bytes(DT, dd.D);
    const bool col_ok = (uint32_t)li * VB < row_bytes;       // lanes past the row's end idle
    const char *__restrict__ base = (const char *)dd.q_base[q] + (uint32_t)li * VB;
    const int tail = (int)row_bytes - li * VB;               // from this lane's bytes to the row's scale and bias
    const int64_t shard_rows = dd.q_rows[q];

    int64_t beg = 0, len = 0, out = 0;
    if (live) {
        int s; uint32_t b_loc, n;
        bls_split_sample(dd, b, s, b_loc, n);
        const int64_t sg = bls_sigma(dd, q, s, b_loc, n);
        out = to_slot ? bls_rho(dd, q, s, b_loc, n) : (int64_t)q * dd.B + b;
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
        float wmine = 0.f;
        if (li < rem) {
            const int64_t r = ridx[beg + c0 + li];
            if (r < 0 || r >= shard_rows) flag_error(dd);
            else mine = (uint32_t)r;
            if (rw) wmine = rw[beg + c0 + li];
        }
        for (int j = 0; __any(j < rem); j += U) {
            uint32_t r[U];
            float wt[U];
            typename A::Raw v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                r[u] = (uint32_t)__shfl((int)mine, gbase + ((j + u) & (G - 1)), 64);
                wt[u] = __shfl(wmine, gbase + ((j + u) & (G - 1)), 64);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                v[u] = A::none();
                if (j + u < rem && r[u] != kBadRow && col_ok) v[u] = A::load(base + (uint64_t)r[u] * row_stride, tail);
                else wt[u] = 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {                   // adding +0 for skipped rows changes nothing
                if (rw) acc.add_weighted(v[u], wt[u]);
                else acc.add(v[u]);
            }
        }
    }
    if (live && col_ok) acc.store(Y + out * dd.D + li * A::NV);
}

// The popular rows of the table a workgroup is working on, copied to LDS (pool_stream_hot), and
// an open-addressing table from row number to the row's place there.
constexpr uint32_t kHotBit = 0x80000000u;      // a row position with this bit set is a place in LDS
constexpr int kHotHash = 1024;                 // slots of the row -> place table (a power of two)
constexpr uint32_t kHotEmpty = 0xffffffffu;
struct HotRows {
    const unsigned char *data;                 // LDS: the rows, row_stride bytes each
    const uint32_t *keys;                      // LDS: row number per slot, or kHotEmpty
    const unsigned short *vals;                // LDS: the row's place
    int n;                                     // rows held (0: none)
};
__device__ __forceinline__ uint32_t hot_hash(uint32_t row) { return (row * 2654435761u) >> 22; }   // 10 bits

// One lane group's work: G >= 4 lanes stream up to nb_max (< G) consecutive segments of (q, s)
// block number gx / chunks_per_s, chunk gx % chunks_per_s.  HOT: rows found in `hot` are read from
// LDS instead of global memory.
template <int G, int DT, int VB, int U, bool WIDE, bool WGT, bool HOT>
__device__ __forceinline__ void stream_group(const DevDesc &dd, int q, uint32_t gx, const int64_t *__restrict__ ridx,
                                             const float *__restrict__ rw, const int64_t *__restrict__ segoff, int64_t nnz,
                                             float *__restrict__ Y, int to_slot, int nb_max, uint32_t chunks_per_s,
                                             const HotRows &hot)
{
    using A = Acc<DT, VB>;
    const int lane = threadIdx.x & 63;
    const int li = lane & (G - 1);
    const int gbase = lane & ~(G - 1);
    const uint32_t s = gx / chunks_per_s;
    const uint32_t chunk = gx - s * chunks_per_s;
    const uint32_t row_bytes = (uint32_t)payload_bytes(DT, dd.D), row_stride = (uint32_t)stride_bytes(DT, dd.D);
    const bool col_ok = (uint32_t)li * VB < row_bytes;       // lanes past the row's end idle:
    // idle lanes re-read the row's first bytes (in bounds, same cache line) and never store
    const char *__restrict__ base = (const char *)dd.q_base[q] + (col_ok ? (uint32_t)li * VB : 0u);
    const int tail = (int)row_bytes - (col_ok ? li * VB : 0);   // to the row's scale and bias
    const int64_t shard_rows = dd.q_rows[q];

    // this group's segments: samples [b0, b0 + nb) of mini-batch s
    int nb = 0;
    int64_t sg0 = 0, out0 = 0;                                // first segment, its vector in the output
    if (s < (uint32_t)dd.P) {
        const int64_t f = dd.first[s], n = dd.first[s + 1] - f;
        const int64_t bl0 = (int64_t)chunk * nb_max;
        if (bl0 < n) {
            nb = n - bl0 < nb_max ? (int)(n - bl0) : nb_max;
            const int d = dd.q_d[q];
            sg0 = (int64_t)dd.nsum[d] * dd.B + (int64_t)dd.n_loc[d] * f + (int64_t)(q - dd.nsum[d]) * n + bl0;
            out0 = to_slot ? (int64_t)dd.Q * f + (int64_t)q * n + bl0 : (int64_t)q * dd.B + f + bl0;
        }
    }
    // lane i of the group holds the start of segment i (i <= nb); all must be in order
    int64_t seg = 0;
    if (nb > 0 && li <= nb) seg = segoff[sg0 + li];
    const int64_t seg_next = __shfl_down(seg, 1, G);
    const int64_t beg = __shfl(seg, gbase, 64);
    const int64_t end = __shfl(seg, gbase + nb, 64);
    const bool bad = nb > 0 && ((li < nb && seg_next < seg) || beg < 0 || end > nnz || end - beg > 0x7fffffffLL);
    const unsigned long long gmask = G == 64 ? ~0ull : ((1ull << (G & 63)) - 1ull) << gbase;
    if (__ballot(bad) & gmask) { if (bad) flag_error(dd); nb = 0; }
    const int rel = (int)(seg - beg);                        // segment starts relative to the stream
    const int total = nb > 0 ? (int)(end - beg) : 0;

    int cur = 0;                                             // segment being summed
    int cur_end = nb > 0 ? (int)__shfl(rel, gbase + 1, 64) : -1;
    A acc;
    acc.zero();

    // Store finished segments (also empty ones) once `pos` rows of the stream are consumed.  The
    // test is one compare against a uniform value; the rest runs only when some group of the
    // wavefront is at a boundary.  Every lane takes part in the lane exchange, the updates are
    // per group.  cur_end is -1 when the group has no segment left, which no position equals.
    auto flush = [&](int pos) {
        if (!__any(cur_end == pos)) return;
        do {
            const int nxt = __shfl(rel, gbase + (cur + 2 < G ? cur + 2 : G - 1), 64);
            if (cur_end == pos) {
                if (col_ok) acc.store(Y + (out0 + cur) * dd.D + li * A::NV);
                acc.zero();
                ++cur;
                cur_end = cur < nb ? nxt : -1;
            }
        } while (__any(cur_end == pos));
    };
    flush(0);

    // this lane's row of block c0 as a position in the shard (all ones: none or out of range)
    using pos_t = typename std::conditional<WIDE, uint64_t, uint32_t>::type;
    constexpr pos_t kNone = (pos_t)~(pos_t)0;
    const uint32_t row_units = WIDE ? row_stride : row_stride / VB;
    auto fetch = [&](int c0) -> pos_t {
        pos_t m = kNone;
        if (c0 + li < total) {
            const int64_t r = ridx[beg + c0 + li];
            if (r < 0 || r >= shard_rows) flag_error(dd);
            else {
                m = (pos_t)((pos_t)r * row_units);
                if constexpr (HOT) {
                    if (hot.n > 0) {                          // the table is never full: the walk ends at an empty slot
                        for (uint32_t h = hot_hash((uint32_t)r);; h = (h + 1u) & (kHotHash - 1)) {
                            const uint32_t key = hot.keys[h];
                            if (key == (uint32_t)r) { m = (pos_t)(kHotBit | hot.vals[h]); break; }
                            if (key == kHotEmpty) break;
                        }
                    }
                }
            }
        }
        return m;
    };
    auto is_row = [&](pos_t p) -> bool {
        if constexpr (WIDE) return (uint32_t)(p >> 32) != 0xffffffffu;
        else return p != kNone;
    };
    auto fetch_weight = [&](int c0) -> float {
        if constexpr (WGT) return c0 + li < total ? rw[beg + c0 + li] : 0.f;
        else return 0.f;
    };
    pos_t mine = fetch(0);
    float wmine = fetch_weight(0);
    typename A::Raw v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = A::none();
    for (int c0 = 0; __any(c0 < total); c0 += G) {
        const pos_t ahead = fetch(c0 + G);                   // next block of row numbers, in flight
        const float wahead = fetch_weight(c0 + G);
        const int left = total - c0;
        const int rem = left < 0 ? 0 : (left > G ? G : left);
        for (int j = 0; __any(j < rem); j += U) {
            pos_t off[U];
            float wt[WGT ? U : 1];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (WIDE) off[u] = group_broadcast64<G>(mine, gbase * 4, j + u);
                else off[u] = group_broadcast32<G>(mine, gbase * 4, j + u);
                if constexpr (WGT) wt[u] = __uint_as_float(group_broadcast32<G>(__float_as_uint(wmine), gbase * 4, j + u));
            }
            // lanes without a row keep stale registers and skip the add: nothing to clear
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (HOT) {
                    if (is_row(off[u])) {
                        if ((uint32_t)off[u] & kHotBit) v[u] = A::load_lds(hot.data + ((uint32_t)off[u] & ~kHotBit) * row_stride + (col_ok ? li * VB : 0), tail);
                        else v[u] = A::load(base + (uint64_t)off[u] * VB, tail);
                    }
                } else {
                    if (is_row(off[u])) v[u] = A::load(base + (WIDE ? (uint64_t)off[u] : (uint64_t)off[u] * VB), tail);
                }
            }
            // every load of the batch has landed before the first add: said once, here, so that
            // no wait is placed between the conditional loads of the next batch
            __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
            const int at = c0 + j;                           // stream position of the batch (uniform)
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (is_row(off[u])) {
                    if constexpr (WGT) acc.add_weighted(v[u], wt[u]);
                    else acc.add(v[u]);
                }
                flush(at + u + 1);                           // positions past the stream's end match nothing
            }
        }
        mine = ahead;
        wmine = wahead;
    }
}

// grid: x over groups (s-major, then chunks of nb_max samples), y = q.
// WIDE: row positions as 64-bit byte offsets; otherwise 32-bit, in units of VB bytes (shards
// below 2^32 * VB bytes), which halves the lane exchanges and the registers they occupy.
// WGT: per-sample weights rw[] (in ridx order) multiply every row before it is added.
template <int G, int DT, int VB, int U, bool WIDE, bool WGT>
__global__ __launch_bounds__(kThreads) void pool_stream(DevDesc dd, const int64_t *__restrict__ ridx,
                                                        const float *__restrict__ rw,
                                                        const int64_t *__restrict__ segoff, int64_t nnz,
                                                        float *__restrict__ Y, int to_slot, int nb_max, uint32_t chunks_per_s, uint32_t wgx,
                                                        int q0, int qn)
{
    // wgx = 0: grid y = q.  Otherwise a flat grid dealt out so that the workgroups an XCD receives
    // (every eighth one) all belong to the same few tables: q = 8 * (round of tables) + XCD.
    // Only the (owner, table) pairs q0 .. q0+qn-1 are worked on (all of them, or one owner's); all of them
    // are taken in the order dd.q_deal, which spreads the large shards evenly over the XCDs.
    uint32_t bx = blockIdx.x;
    int q = q0 + blockIdx.y;
    if (wgx) {
        const uint32_t xcd = blockIdx.x & 7u, r = blockIdx.x >> 3;
        const int pos = (int)((r / wgx) * 8u + xcd);
        bx = r % wgx;
        if (pos >= qn) return;
        q = qn == dd.Q ? dd.q_deal[pos] : q0 + pos;           // all shards: in the balanced order
    }
    const HotRows none{nullptr, nullptr, nullptr, 0};
    stream_group<G, DT, VB, U, WIDE, WGT, false>(dd, q, bx * (kThreads / G) + threadIdx.x / G, ridx, rw, segoff, nnz, Y, to_slot,
                                                 nb_max, chunks_per_s, none);
}

// The same work by workgroups that stay: one workgroup of 1024 threads per compute unit, XCD x
// (workgroups x, x + 8, ...) takes the tables q0 + x, q0 + x + 8, ... one after the other, and its
// workgroups share a table's lane-group streams.  Before a table's first stream a workgroup copies
// the rows the caller named as popular (bls_set_hot_rows) to LDS and builds the row -> place table;
// lookups of those rows are then served from LDS, which takes them off the vector L1 path that
// bounds the kernel when a few rows receive most of the lookups.  Same adds in the same order.
constexpr int kHotThreads = 1024;
constexpr size_t kHotLdsBytes = 128 * 1024;     // LDS for the rows themselves (of 160 KB per compute unit)
template <int G, int DT, int VB, int U, bool WGT>
__global__ __launch_bounds__(kHotThreads) void pool_stream_hot(DevDesc dd, const int64_t *__restrict__ ridx,
                                                               const float *__restrict__ rw,
                                                               const int64_t *__restrict__ segoff, int64_t nnz,
                                                               float *__restrict__ Y, int to_slot, int nb_max,
                                                               uint32_t chunks_per_s, int q0, int qn, int cap_rows)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const uint32_t row_stride = (uint32_t)stride_bytes(DT, dd.D);
    unsigned char *data = lds;
    uint32_t *keys = reinterpret_cast<uint32_t *>(lds + (size_t)cap_rows * row_stride);
    unsigned short *vals = reinterpret_cast<unsigned short *>(keys + kHotHash);
    const uint32_t xcd = blockIdx.x & 7u, j = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
    const uint32_t groups = chunks_per_s * (uint32_t)dd.P, per_wg = kHotThreads / G;
    const uint32_t blocks = (groups + per_wg - 1) / per_wg;
    for (int q = q0 + (int)xcd; q < q0 + qn; q += 8) {
        __syncthreads();                                      // the previous table's rows are no longer read
        const int n_hot = dd.hot_n[q] < cap_rows ? dd.hot_n[q] : cap_rows;
        if (n_hot > 0) {
            for (int i = threadIdx.x; i < kHotHash; i += kHotThreads) keys[i] = kHotEmpty;
            const uint32_t *rows = dd.hot_rows + dd.hot_off[q];
            const unsigned char *src = (const unsigned char *)dd.q_base[q];
            const uint32_t per_row = row_stride / 16;         // 16-byte pieces per row
            for (uint32_t i = threadIdx.x; i < (uint32_t)n_hot * per_row; i += kHotThreads) {
                const uint32_t r = i / per_row, piece = i - r * per_row;
                *reinterpret_cast<u32x4 *>(data + (size_t)r * row_stride + piece * 16) =
                    *reinterpret_cast<const u32x4 *>(src + (uint64_t)rows[r] * row_stride + piece * 16);
            }
            __syncthreads();                                  // the table is empty before anyone inserts
            for (int i = threadIdx.x; i < n_hot; i += kHotThreads) {
                const uint32_t row = rows[i];
                for (uint32_t h = hot_hash(row);; h = (h + 1u) & (kHotHash - 1)) {
                    const uint32_t seen = atomicCAS(&keys[h], kHotEmpty, row);
                    if (seen == kHotEmpty) { vals[h] = (unsigned short)i; break; }
                    if (seen == row) break;                   // named twice: the first copy serves
                }
            }
        }
        __syncthreads();
        const HotRows hot{data, keys, vals, n_hot};
        for (uint32_t blk = j; blk < blocks; blk += per_xcd)
            stream_group<G, DT, VB, U, false, WGT, true>(dd, q, blk * per_wg + threadIdx.x / G, ridx, rw, segoff, nnz, Y, to_slot,
                                                         nb_max, chunks_per_s, hot);
    }
}

// Any D (odd lengths, rows longer than 1 KB): one wavefront per segment, lanes stride the
// columns, scalar loads.
template <int DT>
__global__ __launch_bounds__(kThreads) void pool_rows_generic(DevDesc dd, const int64_t *__restrict__ ridx,
                                                              const float *__restrict__ rw,
                                                              const int64_t *__restrict__ segoff, int64_t nnz,
                                                              float *__restrict__ Y, int to_slot, int q0)
{
    const int q = q0 + blockIdx.y;
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
    float *y = Y + (to_slot ? bls_rho(dd, q, s, b_loc, n) : (int64_t)q * dd.B + b) * dd.D;
    for (int c = lane; c < dd.D; c += 64) {
        float acc = 0.f;
        for (int64_t j = beg; j < end; ++j) {
            const int64_t r = ridx[j];
            if (r < 0 || r >= shard_rows) { if (c == 0) flag_error(dd); continue; }
            float x;
            if constexpr (is_rowq(DT)) {
                const unsigned char *row = (const unsigned char *)base + r * stride_bytes(DT, dd.D);
                float scale, bias;                              // any D: no alignment to rely on
                __builtin_memcpy(&scale, row + dd.D, 4);
                __builtin_memcpy(&bias, row + dd.D + 4, 4);
                const float code = DT == BLS_F8_ROWQ ? __builtin_amdgcn_cvt_f32_fp8((int)row[c], 0) : (float)row[c];
                const float prod = code * scale;
                x = prod + bias;
            } else {
                const int64_t e = r * dd.D + c;
                x = DT == BLS_FP16 ? half_bits(((const unsigned short *)base)[e]) : ((const float *)base)[e];
            }
            if (rw) { const float term = rw[j] * x; acc += term; }
            else acc += x;
        }
        y[c] = acc;
    }
}

template <int G, int DT, int VB, int U>
void launch_rows(const bls_ctx *ctx, const int64_t *ridx, const float *rw, const int64_t *segoff, int64_t nnz, float *Y, int to_slot, int q0, int qn, hipStream_t st)
{
    constexpr int UU = U < G ? U : G;
    const uint32_t per_block = kThreads / G;
    if constexpr (G >= 4) {
        // segments per group: aim at a stream of two to three hundred rows (the lane groups of a wavefront finish
        // at different times, and the longer the streams the smaller the share of loads only one of them uses;
        // much longer streams lose again)
        const int64_t mean = nnz / std::max<int64_t>(1, ctx->nseg) + 1;
        int nb = 1;
        while (nb * 2 < G && nb * 2 <= 16 && nb * mean < 192) nb *= 2;
        // ... but a small batch takes shorter streams (down to some sixty rows) rather than fewer than two
        // workgroups per compute unit
        const int64_t room = 2 * (int64_t)std::max(ctx->compute_units, 1);
        while (nb > 1 && nb * mean >= 64 && (int64_t)qn * ((ctx->B + nb - 1) / nb) < room * per_block) nb /= 2;
        if (ctx->tune_segs > 0) nb = ctx->tune_segs;
        nb = std::max(1, std::min(nb, G - 1));
        const int64_t n_max = ctx->B / ctx->P + (ctx->B % ctx->P ? 1 : 0);
        const uint32_t chunks = (uint32_t)((n_max + nb - 1) / nb);
        const int64_t groups = (int64_t)chunks * ctx->P;
        const uint32_t wgx = (uint32_t)((groups + per_block - 1) / per_block);
        const bool xcd = ctx->tune_xcd != 0;
        const dim3 grid = xcd ? dim3((unsigned)((uint64_t)((qn + 7) / 8) * 8u * wgx)) : dim3(wgx, qn);
        const uint32_t deal = xcd ? wgx : 0u;
        // 32-bit row positions unless some shard is too large for them
        const int64_t row_stride = stride_bytes(DT, ctx->D);
        bool wide = ctx->tune_wide == 1;
        for (int q = q0; q < q0 + qn; ++q) wide = wide || ctx->q_rows[q] * (row_stride / VB) >= 0xffffffffLL;
        // popular rows named for some shard of this launch: the staying workgroups that keep them in LDS,
        // if every row position leaves the top bit free for the "in LDS" mark
        bool hot = VB == 16 && !wide && ctx->tune_hot != 0 && ctx->compute_units >= 8;
        bool any_hot = false;
        for (int q = q0; q < q0 + qn; ++q) {
            any_hot = any_hot || !ctx->q_hot[q].empty();
            hot = hot && ctx->q_rows[q] * (row_stride / VB) < (int64_t)kHotBit;
        }
        if constexpr (VB == 16) {
            if (hot && any_hot) {
                const int cap = (int)std::min<int64_t>(BLS_HOT_ROWS_MAX, (int64_t)kHotLdsBytes / row_stride);
                const size_t lds = (size_t)cap * row_stride + kHotHash * (sizeof(uint32_t) + sizeof(unsigned short));
                const dim3 hgrid((unsigned)(ctx->compute_units / 8 * 8));
                auto launch = [&](auto kernel) -> hipError_t {
                    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                    if (e != hipSuccess) return e;
                    kernel<<<hgrid, kHotThreads, lds, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, nb, chunks, q0, qn, cap);
                    return hipSuccess;
                };
                if (cap > 0 && (rw ? launch(pool_stream_hot<G, DT, VB, UU, true>) : launch(pool_stream_hot<G, DT, VB, UU, false>)) == hipSuccess)
                    return;
            }
        }
        if (rw) {
            if (wide) pool_stream<G, DT, VB, UU, true, true><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, nb, chunks, deal, q0, qn);
            else pool_stream<G, DT, VB, UU, false, true><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, nb, chunks, deal, q0, qn);
        } else {
            if (wide) pool_stream<G, DT, VB, UU, true, false><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, nb, chunks, deal, q0, qn);
            else pool_stream<G, DT, VB, UU, false, false><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, nb, chunks, deal, q0, qn);
        }
    } else {
        dim3 grid((unsigned)((ctx->B + per_block - 1) / per_block), qn);
        pool_rows<G, DT, VB, UU><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, q0);
    }
}

template <int DT, int VB, int U>
bool dispatch_lanes(const bls_ctx *ctx, int lanes, const int64_t *ridx, const float *rw, const int64_t *segoff, int64_t nnz,
                    float *Y, int to_slot, int q0, int qn, hipStream_t st)
{
    switch (lanes) {
    case 1: if constexpr (VB == 16) { launch_rows<1, DT, VB, U>(ctx, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st); return true; } break;
    case 2: if constexpr (VB == 16) { launch_rows<2, DT, VB, U>(ctx, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st); return true; } break;
    case 4: if constexpr (VB == 16) { launch_rows<4, DT, VB, U>(ctx, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st); return true; } break;
    case 8: if constexpr (VB == 16) { launch_rows<8, DT, VB, U>(ctx, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st); return true; } break;
    case 16: if constexpr (VB >= 8) { launch_rows<16, DT, VB, U>(ctx, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st); return true; } break;
    case 32: launch_rows<32, DT, VB, U>(ctx, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st); return true;
    case 64: launch_rows<64, DT, VB, U>(ctx, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st); return true;
    }
    return false;
}

template <int DT>
bool dispatch_rows(const bls_ctx *ctx, int vb, int lanes, const int64_t *ridx, const float *rw,
                   const int64_t *segoff, int64_t nnz, float *Y, int to_slot, int q0, int qn, hipStream_t st)
{
    switch (vb) {
    case 16: return dispatch_lanes<DT, 16, (is_rowq(DT) ? kRowsInFlightQuantised : kRowsInFlight)>(ctx, lanes, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st);
    case 8: return dispatch_lanes<DT, 8, kRowsInFlight>(ctx, lanes, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st);
    case 4: return dispatch_lanes<DT, 4, kRowsInFlight>(ctx, lanes, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st);
    }
    return false;
}


}  // namespace

int bls_launch_pool(bls_ctx *ctx, const int64_t *ridx, const float *rw, const int64_t *segoff, int64_t nnz, float *Y, int to_slot, int q0, int qn, hipStream_t st)
{
    const int64_t row_bytes = payload_bytes(ctx->dtype, ctx->D);
    // bytes per lane and row: 16 when the row length allows, unless bls_set_pool_tuning says otherwise
    int vb = ctx->tune_lane_bytes ? ctx->tune_lane_bytes : 16;
    while (vb > 4 && row_bytes % vb != 0) vb >>= 1;          // lanes must split the row evenly
    while (vb < 16 && row_bytes > 64 * (int64_t)vb) vb <<= 1; // and 64 of them must cover it
    bool done = false;
    if (row_bytes % vb == 0 && row_bytes <= 64 * (int64_t)vb) {
        int lanes = 1;
        while ((int64_t)lanes * vb < row_bytes) lanes <<= 1;
        done = ctx->dtype == BLS_U8_ROWQ ? dispatch_rows<BLS_U8_ROWQ>(ctx, vb, lanes, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st)
             : ctx->dtype == BLS_F8_ROWQ ? dispatch_rows<BLS_F8_ROWQ>(ctx, vb, lanes, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st)
             : ctx->dtype == BLS_FP16  ? dispatch_rows<BLS_FP16>(ctx, vb, lanes, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st)
                                       : dispatch_rows<BLS_FP32>(ctx, vb, lanes, ridx, rw, segoff, nnz, Y, to_slot, q0, qn, st);
    }
    if (!done) {
        dim3 grid((unsigned)((ctx->B + kThreads / 64 - 1) / (kThreads / 64)), qn);
        if (ctx->dtype == BLS_U8_ROWQ) pool_rows_generic<BLS_U8_ROWQ><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, q0);
        else if (ctx->dtype == BLS_F8_ROWQ) pool_rows_generic<BLS_F8_ROWQ><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, q0);
        else if (ctx->dtype == BLS_FP16) pool_rows_generic<BLS_FP16><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, q0);
        else pool_rows_generic<BLS_FP32><<<grid, kThreads, 0, st>>>(ctx->desc, ridx, rw, segoff, nnz, Y, to_slot, q0);
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
