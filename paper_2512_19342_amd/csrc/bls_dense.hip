// bls_mlp_layer and bls_interact: the dense part of the model around the lookup (apply_mlp and
// interact_features of Listings 1 and 2), in fp32 on the matrix cores.
//
// Both are dense contractions, so both run on v_mfma_f32_32x32x2_f32: one instruction multiplies
// a 32x2 by a 2x32 fp32 block into a 32x32 fp32 accumulator held in 16 registers per lane.
// Operand layout: lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32]; accumulator register
// v of lane l is element (8 * (v / 4) + 4 * (l / 32) + v % 4, l % 32).
#include <stdint.h>

#include "bls_internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

template <int ACT>
__device__ __forceinline__ float activate(float v)
{
    if constexpr (ACT == BLS_ACT_RELU) return v > 0.f ? v : 0.f;
    else if constexpr (ACT == BLS_ACT_SIGMOID) return 1.f / (1.f + expf(-v));
    else return v;
}

// ---- one layer: Y[M][N] = act(X[M][K] * W[N][K]^T + bias[N]) ---------------------------------
//
// A workgroup of four wavefronts owns a 128 x 128 tile of Y; each wavefront a 64 x 64 quarter
// (2 x 2 accumulators).  X and W tiles of 16 columns of K are staged through LDS, transposed
// to k-major so that the 32 lanes of a half-wavefront read 32 consecutive floats for one k, and
// double-buffered: the loads of the next tile are in flight while the current one is multiplied.
// Workgroups are numbered so that the eight that share rows of X follow each other on one XCD
// (one L2), N-tile fastest.
#ifndef BLS_GEMM_BK
#define BLS_GEMM_BK 16
#endif
constexpr int BM = 128, BN = 128, BK = BLS_GEMM_BK, LDT = BM + 4;

template <bool VEC, int ACT>
__global__ __launch_bounds__(kThreads) void mlp_gemm(const float *__restrict__ X, const float *__restrict__ W,
                                                     const float *__restrict__ bias, float *__restrict__ Y,
                                                     int64_t M, int N, int K, uint32_t n_tiles, uint32_t tiles)
{
    __shared__ float As[2][BK][LDT];
    __shared__ float Bs[2][BK][LDT];

    // XCD x gets the tiles [x * per, (x + 1) * per) in launch order
    const uint32_t per = (tiles + 7u) / 8u;
    const uint32_t tile = (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per || tile >= tiles) return;
    const int64_t m0 = (int64_t)(tile / n_tiles) * BM;
    const int n0 = (int)(tile % n_tiles) * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int half = lane >> 5, l32 = lane & 31;

    // staging registers for one tile of X and one of W
    constexpr int NLD = VEC ? BM * BK / 4 / kThreads : BM * BK / kThreads;
    float4 xa[VEC ? NLD : 1], wa[VEC ? NLD : 1];
    float xs[VEC ? 1 : NLD], ws[VEC ? 1 : NLD];

    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = tid + i * kThreads;
            if constexpr (VEC) {
                const int row = idx / (BK / 4), kq = (idx % (BK / 4)) * 4;
                const bool kin = k0 + kq < K;                 // K % 4 == 0: a whole float4 is in or out
                xa[i] = (kin && m0 + row < M) ? *reinterpret_cast<const float4 *>(X + (m0 + row) * K + k0 + kq)
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
                wa[i] = (kin && n0 + row < N) ? *reinterpret_cast<const float4 *>(W + (int64_t)(n0 + row) * K + k0 + kq)
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                const int row = idx / BK, k = idx % BK;
                const bool kin = k0 + k < K;
                xs[i] = (kin && m0 + row < M) ? X[(m0 + row) * K + k0 + k] : 0.f;
                ws[i] = (kin && n0 + row < N) ? W[(int64_t)(n0 + row) * K + k0 + k] : 0.f;
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = tid + i * kThreads;
            if constexpr (VEC) {
                const int row = idx / (BK / 4), kq = (idx % (BK / 4)) * 4;
                As[buf][kq + 0][row] = xa[i].x; As[buf][kq + 1][row] = xa[i].y;
                As[buf][kq + 2][row] = xa[i].z; As[buf][kq + 3][row] = xa[i].w;
                Bs[buf][kq + 0][row] = wa[i].x; Bs[buf][kq + 1][row] = wa[i].y;
                Bs[buf][kq + 2][row] = wa[i].z; Bs[buf][kq + 3][row] = wa[i].w;
            } else {
                const int row = idx / BK, k = idx % BK;
                As[buf][k][row] = xs[i];
                Bs[buf][k][row] = ws[i];
            }
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // operands of the next pair of k are read from LDS before the four multiplies of the current
    // pair are issued, so their latency passes while the matrix pipe is busy
    auto multiply = [&](int buf) {
        const float *pa = &As[buf][half][wm + l32], *pb = &Bs[buf][half][wn + l32];
        float a0 = pa[0], a1 = pa[32], b0 = pb[0], b1 = pb[32];
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
            if (kk + 2 < BK) {
                na0 = pa[(kk + 2) * LDT]; na1 = pa[(kk + 2) * LDT + 32];
                nb0 = pb[(kk + 2) * LDT]; nb1 = pb[(kk + 2) * LDT + 32];
            }
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
            // keep that order in the schedule: the LDS reads of the pair, then its four multiplies
            if (kk + 2 < BK) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        }
    };

    fetch(0);
    stage(0);
    __syncthreads();
    const int steps = (K + BK - 1) / BK;
    int buf = 0;
    for (int t = 1; t < steps; ++t) {
        fetch(t * BK);                                        // in flight during the multiplies below
        multiply(buf);
        stage(buf ^ 1);                                       // the other buffer: nobody reads it now
        __syncthreads();
        buf ^= 1;
    }
    multiply(buf);

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn + j * 32 + l32;
            if (col >= N) continue;
            const float bv = bias ? bias[col] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (row < M) Y[row * N + col] = activate<ACT>(acc[i][j][v] + bv);
            }
        }
}

// ---- dot interaction ---------------------------------------------------------------------------
//
// One workgroup per sample.  The sample's T pooled vectors are copied to LDS (rows padded to a
// multiple of 32 with zeros, row stride odd so that 32 rows at one column fall in 32 banks); the
// 32 x 32 tiles on and below the diagonal of their Gram matrix are dealt to the wavefronts, each
// tile one accumulator over D / 2 matrix instructions; the last wavefront also takes the T
// products with the dense vector x.  Output row: x, then for i = 1..T the products of pooled
// vector i-1 with x and with pooled vectors 0..i-2.
// SLOT = false: emb is the completed lookup [B][T][D].  SLOT = true: emb is a ring slot in receive
// order and the copy to LDS is the completion itself - vector (b, t) is read where its owner put
// it, and for a row-wise partition the P partial vectors are added in increasing owner rank from
// +0, exactly as the copy-out kernel does.
template <bool SLOT>
__global__ __launch_bounds__(kThreads) void interact_gram(DevDesc dd, const float *__restrict__ x, const float *__restrict__ emb,
                                                          float *__restrict__ z, int T, int D, int TP, int LD,
                                                          uint32_t b0, int vec4)
{
    extern __shared__ float lds[];
    float *Es = lds;                                          // [TP][LD]
    float *xsh = lds + (size_t)TP * LD;                       // [D]
    const int64_t b = (int64_t)b0 + blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t Wz = (int64_t)D + (int64_t)T * (T + 1) / 2;
    const float *__restrict__ e = emb + b * T * D;               // SLOT = false only
    float *__restrict__ zb = z + b * Wz;
    int64_t slot_base = 0, slot_step = 0;                        // vector (q, b) of the slot: slot_base + q * slot_step
    if constexpr (SLOT) {
        int s; uint32_t b_loc, n;
        bls_split_sample(dd, (uint32_t)b, s, b_loc, n);
        slot_base = (int64_t)dd.Q * dd.first[s] + b_loc;
        slot_step = n;
    }
    // start of the d-th partial (d < F; F = 1 table-wise) of pooled vector t of this sample
    auto partial = [&](uint32_t t, int d) -> const float * {
        return emb + (slot_base + (int64_t)(dd.t_q[t] + d * dd.T) * slot_step) * D;
    };

    // zeros: the padding columns behind every vector and the padding rows behind the last one
    const int padc = LD - D;
    for (int i = tid; i < T * padc; i += kThreads) Es[(i / padc) * LD + D + i % padc] = 0.f;
    for (int i = T * LD + tid; i < TP * LD; i += kThreads) Es[i] = 0.f;
    // the vectors themselves: eight independent loads per lane in flight, then the LDS writes
    constexpr int kFill = 8;
    if (vec4) {
        const float4 *__restrict__ e4 = reinterpret_cast<const float4 *>(e);
        const uint32_t n4 = (uint32_t)T * (uint32_t)D / 4u, c4n = (uint32_t)D / 4u;
        for (uint32_t base = 0; base < n4; base += kThreads * kFill) {
            float4 v[kFill];
#pragma unroll
            for (int u = 0; u < kFill; ++u) {
                const uint32_t i = base + u * kThreads + tid;
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if constexpr (SLOT) {
                    if (i < n4) {
                        const uint32_t r = i / c4n, c = (i - r * c4n) * 4u;
                        for (int d = 0; d < dd.F; ++d) {
                            const float4 part = *reinterpret_cast<const float4 *>(partial(r, d) + c);
                            v[u].x += part.x; v[u].y += part.y; v[u].z += part.z; v[u].w += part.w;
                        }
                    }
                } else if (i < n4) {
                    v[u] = e4[i];
                }
            }
#pragma unroll
            for (int u = 0; u < kFill; ++u) {
                const uint32_t i = base + u * kThreads + tid;
                if (i < n4) {
                    const uint32_t r = i / c4n, c = (i - r * c4n) * 4u;
                    float *d = Es + r * LD + c;
                    d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
                }
            }
        }
    } else {
        const uint32_t n1 = (uint32_t)T * (uint32_t)D;
        for (uint32_t base = 0; base < n1; base += kThreads * kFill) {
            float v[kFill];
#pragma unroll
            for (int u = 0; u < kFill; ++u) {
                const uint32_t i = base + u * kThreads + tid;
                v[u] = 0.f;
                if constexpr (SLOT) {
                    if (i < n1) {
                        const uint32_t r = i / (uint32_t)D, c = i - r * (uint32_t)D;
                        for (int d = 0; d < dd.F; ++d) v[u] += partial(r, d)[c];
                    }
                } else if (i < n1) {
                    v[u] = e[i];
                }
            }
#pragma unroll
            for (int u = 0; u < kFill; ++u) {
                const uint32_t i = base + u * kThreads + tid;
                if (i < n1) { const uint32_t r = i / (uint32_t)D; Es[r * LD + (i - r * (uint32_t)D)] = v[u]; }
            }
        }
    }
    for (int c = tid; c < D; c += kThreads) {
        const float v = x[b * D + c];
        xsh[c] = v;
        zb[c] = v;
    }
    __syncthreads();

    const int half = lane >> 5, l32 = lane & 31;
    const int nt = TP / 32;
    int tile = 0;
    for (int ti = 0; ti < nt; ++ti)
        for (int tj = 0; tj <= ti; ++tj, ++tile) {
            if ((tile & 3) != wave) continue;
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const float *pa = Es + (ti * 32 + l32) * LD + half;
            const float *pb = Es + (tj * 32 + l32) * LD + half;
            for (int k = 0; k < D; k += 2)                    // column D of an odd D is a zero
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[k], pb[k], acc, 0, 0, 0);
            const int col = tj * 32 + l32;                    // the lower-numbered vector of the pair
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = ti * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (row < T && col < row) zb[D + (int64_t)(row + 1) * row / 2 + col + 1] = acc[v];
            }
        }
    if (wave == 3) {
        for (int t = lane; t < T; t += 64) {
            float dot = 0.f;
            for (int c = 0; c < D; ++c) dot += Es[t * LD + c] * xsh[c];
            zb[D + (int64_t)(t + 1) * t / 2] = dot;
        }
    }
}

}  // namespace

int bls_launch_mlp_layer(bls_ctx *ctx, const float *x, int64_t M, int K, const float *W, const float *bias, int N,
                         int act, float *y, hipStream_t st)
{
    if (M == 0) return BLS_OK;
    const uint64_t m_tiles = (uint64_t)((M + BM - 1) / BM), n_tiles = (uint64_t)((N + BN - 1) / BN);
    if (m_tiles * n_tiles > 0x7fffffffull - 8) return bls_fail(ctx, BLS_EINVAL, "bls_mlp_layer: too many tiles");
    const uint32_t tiles = (uint32_t)(m_tiles * n_tiles);
    const dim3 grid((tiles + 7u) / 8u * 8u);
    const bool vec = K % 4 == 0 && (((uintptr_t)x | (uintptr_t)W) & 15u) == 0;
#define BLS_GEMM(V, A) mlp_gemm<V, A><<<grid, kThreads, 0, st>>>(x, W, bias, y, M, N, K, (uint32_t)n_tiles, tiles)
    if (vec) {
        if (act == BLS_ACT_RELU) BLS_GEMM(true, BLS_ACT_RELU);
        else if (act == BLS_ACT_SIGMOID) BLS_GEMM(true, BLS_ACT_SIGMOID);
        else BLS_GEMM(true, BLS_ACT_NONE);
    } else {
        if (act == BLS_ACT_RELU) BLS_GEMM(false, BLS_ACT_RELU);
        else if (act == BLS_ACT_SIGMOID) BLS_GEMM(false, BLS_ACT_SIGMOID);
        else BLS_GEMM(false, BLS_ACT_NONE);
    }
#undef BLS_GEMM
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

size_t bls_interact_lds_bytes(int T, int D)
{
    const int TP = (T + 31) / 32 * 32, LD = ((D + 1) & ~1) + 1;
    return ((size_t)TP * LD + (size_t)D) * sizeof(float);
}

int bls_launch_interact(bls_ctx *ctx, const float *x, const float *emb, int from_slot, float *z, uint32_t b0, uint32_t bn,
                        hipStream_t st)
{
    if (bn == 0) return BLS_OK;
    const int T = ctx->T, D = ctx->D;
    const int TP = (T + 31) / 32 * 32, LD = ((D + 1) & ~1) + 1;
    const int vec4 = D % 4 == 0 && ((uintptr_t)emb & 15u) == 0;   // every vector then starts 16-byte aligned
    const size_t lds = bls_interact_lds_bytes(T, D);
    if (from_slot) interact_gram<true><<<dim3(bn), kThreads, lds, st>>>(ctx->desc, x, emb, z, T, D, TP, LD, b0, vec4);
    else interact_gram<false><<<dim3(bn), kThreads, lds, st>>>(ctx->desc, x, emb, z, T, D, TP, LD, b0, vec4);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
