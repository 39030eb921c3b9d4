// Internal declarations shared by the libbls translation units (host context,
// device-side descriptor, launch helpers).  Not part of the public interface.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "bls.h"

// Device-side view of the problem.  Passed to kernels by value; the arrays live in the
// caller's descriptor buffer (bls_commit).
//
// q numbers the (owner, local table) pairs in owner-major order, q = nsum[d] + t_loc,
// 0 <= q < Q = F*T.  Pooled vector (q, b) sits at vector index
//   y(q,b)     = q*B + b                                        in the pooled buffer Y,
//   sigma(q,b) = nsum[d]*B + n_loc[d]*first[s] + t_loc*n + b_loc in segment / send order,
//   rho(q,b)   = Q*first[s] + q*n + b_loc                        in receive order,
// with s the requester of b, n its mini-batch size and b_loc = b - first[s].
struct DevDesc {
    int32_t P, T, D, F, Q, part_kind, dtype, pad0;
    int64_t B;
    uint32_t Bq, Br;             // B / P and B % P
    int64_t nseg;                // F*T*B
    const int64_t *first;        // [P+1] first sample of every mini-batch
    const int32_t *n_loc;        // [P]
    const int32_t *nsum;         // [P+1] exclusive running sum of n_loc
    const int64_t *rows;         // [T]
    const int64_t *rps;          // [T] rows per shard (row-wise); rows (table-wise)
    const int32_t *t_q;          // [T] q of table t at its owner (table-wise); t (row-wise, add d*T)
    const int32_t *q_t;          // [Q]
    const int32_t *q_d;          // [Q]
    const void *const *q_base;   // [Q] shard storage
    const int64_t *q_rows;       // [Q] rows in the shard
    const int32_t *q_deal;       // [Q] the shards in the order a pooling launch over all of them deals them to the XCDs
    const int32_t *hot_n;        // [Q] popular rows named for the shard (bls_set_hot_rows), 0 if none
    const int32_t *hot_off;      // [Q] where the shard's list starts in hot_rows
    const uint32_t *hot_rows;    // the lists, local row numbers, most popular first
    int32_t *err;                // error flag, set to 1 by kernels that skip a bad item
};

// Per-rank issue and completion (bls_rank_put / bls_rank_complete): every rank has its own
// iteration counters, and every slot one arrival event per owner and one release event per
// requester - the arrival events play the part of the paper's per-iteration tag counters.
struct RankRing {
    std::vector<int64_t> put_next, done_next;     // [P] next iteration rank r puts / completes
    std::vector<hipEvent_t> arrived, released;    // [K*P] slot-major
    std::vector<uint8_t> has_arrived, has_released;
    std::vector<hipStream_t> arrived_on, released_on;   // stream of the last record: same-stream waits are skipped
};

struct RingSlot {
    int state = 0;               // 0 free, 1 acquired (exchange not yet enqueued), 2 filled
    int64_t iter = -1;
    hipEvent_t filled = nullptr;   // recorded after the exchange into the slot
    hipEvent_t released = nullptr; // recorded after the slot was copied out
    bool has_released = false;
    // streams the two events were last recorded on: a wait from the same stream is implied by
    // stream order and is not enqueued
    hipStream_t filled_on = nullptr, released_on = nullptr;
};

struct bls_ctx {
    // configuration (host copies)
    int32_t P = 0, T = 0, D = 0, k = 0, K = 1, F = 1, Q = 0, dtype = 0, part_kind = 0;
    int64_t B = 0;
    std::vector<int64_t> rows, rps, first, q_rows;
    std::vector<int32_t> owner, n_loc, nsum, t_loc, t_q, q_t, q_d;
    std::vector<const void *> q_base;
    std::vector<uint8_t> q_set;
    std::vector<std::vector<uint32_t>> q_hot;   // [Q] popular rows of the shard, most popular first (may be empty)
    int compute_units = 0;        // of the device the tables were committed on
    int64_t nseg = 0, nvec = 0;   // nvec = nseg = F*T*B pooled vectors per iteration

    // device side
    int device = -1;
    void *blob = nullptr;         // caller's descriptor buffer: error flag, then the arrays
    std::vector<char> host_blob;  // what was last uploaded there (kept: the upload is asynchronous)
    bool dirty = true;            // host tables changed since the last upload
    DevDesc desc{};

    // pool launch shape overrides (bls_set_pool_tuning); 0 / -1 = the library's choice
    int tune_lane_bytes = 0, tune_segs = 0, tune_xcd = -1, tune_wide = -1, tune_hot = -1;
    int tune_plan_scan = -1;      // row-wise plan: 0 = always a scan launch, otherwise the placing workgroups scan where they can

    // ring
    char *slots = nullptr;
    size_t slot_bytes = 0;
    int64_t head = 0, tail = 0;   // next iteration to start, oldest in flight
    std::vector<RingSlot> ring;
    RankRing rr;

    std::string err;
};

// ---- helpers shared by the translation units -------------------------------------
int bls_fail(bls_ctx *ctx, int code, const char *what);
int bls_fail_hip(bls_ctx *ctx, hipError_t e, const char *what);
int bls_ready(bls_ctx *ctx);    // BLS_OK when the descriptor tables on the device are current (bls_commit)
size_t bls_desc_size(const bls_ctx *ctx);

#define BLS_HIP(ctx, call)                                         \
    do {                                                           \
        hipError_t e_ = (call);                                    \
        if (e_ != hipSuccess) return bls_fail_hip(ctx, e_, #call); \
    } while (0)

// launches, defined next to their kernels
int bls_launch_plan(bls_ctx *ctx, const int64_t *idx, const int64_t *off, int64_t nnz, int64_t *sendcounts,
                    int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls, int64_t *ridx, int64_t *segoff,
                    int64_t *perm, const float *w_in, float *w_out, void *ws, size_t ws_bytes, hipStream_t st);
size_t bls_plan_ws_bytes(const bls_ctx *ctx);
// to_slot = 0: Y in pooled order (y); 1: Y is a ring slot, vectors go to receive order (rho)
// rw: weight of every lookup in ridx order, or NULL; (owner, table) pairs q0 .. q0+qn-1 only
int bls_launch_pool(bls_ctx *ctx, const int64_t *ridx, const float *rw, const int64_t *segoff, int64_t nnz, float *Y,
                    int to_slot, int q0, int qn, hipStream_t st);
int bls_launch_step_tablewise(bls_ctx *ctx, const int64_t *idx, const int64_t *off, int64_t nnz, int64_t *sendcounts,
                              int64_t *sdispls, int64_t *recvcounts, int64_t *rdispls, int64_t *ridx, int64_t *segoff,
                              int64_t *perm, float *Y, float *S, float *R, float *out, hipStream_t st);
int bls_launch_pack(bls_ctx *ctx, const float *Y, float *S, hipStream_t st);
int bls_launch_exchange(bls_ctx *ctx, const float *S, float *R, hipStream_t st);
// mean_off: the batch's offsets for mean pooling (divide by the bag length), or NULL; samples b0 .. b0+bn-1 only
int bls_launch_unpack(bls_ctx *ctx, const float *R, float *out, const int64_t *mean_off, uint32_t b0, uint32_t bn,
                      hipStream_t st);
int bls_launch_delay(bls_ctx *ctx, uint32_t microseconds, hipStream_t st);
int bls_launch_mlp_layer(bls_ctx *ctx, const float *x, int64_t M, int K, const float *W, const float *bias, int N,
                         int act, float *y, hipStream_t st);
size_t bls_interact_lds_bytes(int T, int D);
// from_slot = 0: emb is [B][T][D]; 1: emb is a ring slot in receive order (the copy-out is folded in)
int bls_launch_interact(bls_ctx *ctx, const float *x, const float *emb, int from_slot, float *z, uint32_t b0, uint32_t bn,
                        hipStream_t st);

// ---- device helpers ----------------------------------------------------------------
#ifdef __HIPCC__
// Requester s of sample b, its position b_loc inside the mini-batch and the
// mini-batch size n.  The first Br ranks hold Bq+1 samples, the rest Bq.
__device__ __forceinline__ void bls_split_sample(const DevDesc &dd, uint32_t b, int &s, uint32_t &b_loc, uint32_t &n)
{
    const uint32_t big = dd.Br * (dd.Bq + 1u);
    if (b < big) {
        s = (int)(b / (dd.Bq + 1u));
        b_loc = b - (uint32_t)s * (dd.Bq + 1u);
        n = dd.Bq + 1u;
    } else {
        const uint32_t r = b - big;
        const uint32_t q = r / dd.Bq;
        s = (int)(dd.Br + q);
        b_loc = r - q * dd.Bq;
        n = dd.Bq;
    }
}

// First sample of rank s's mini-batch (s = P gives B): the first Br ranks hold one sample more.
__device__ __forceinline__ int64_t bls_first(const DevDesc &dd, int s)
{
    return (int64_t)s * dd.Bq + ((uint32_t)s < dd.Br ? (uint32_t)s : dd.Br);
}

__device__ __forceinline__ int64_t bls_sigma(const DevDesc &dd, int q, int s, uint32_t b_loc, uint32_t n)
{
    const int d = dd.q_d[q];
    const int64_t ns = dd.nsum[d];
    return ns * dd.B + (int64_t)dd.n_loc[d] * dd.first[s] + (int64_t)(q - ns) * n + b_loc;
}

// sigma for a row-wise partition, where every rank serves all T tables: q = d*T + t, nsum(d) = d*T,
// n_loc = T and first(s) = s*Bq + min(s, Br) - no table look-ups.
__device__ __forceinline__ int64_t bls_sigma_rowwise(const DevDesc &dd, int d, int t, int s, uint32_t b_loc, uint32_t n)
{
    const int64_t first_s = (int64_t)s * dd.Bq + ((uint32_t)s < dd.Br ? (uint32_t)s : dd.Br);
    return ((int64_t)d * dd.B + first_s) * dd.T + (int64_t)t * n + b_loc;
}

__device__ __forceinline__ int64_t bls_rho(const DevDesc &dd, int q, int s, uint32_t b_loc, uint32_t n)
{
    return (int64_t)dd.Q * dd.first[s] + (int64_t)q * n + b_loc;
}
#endif
