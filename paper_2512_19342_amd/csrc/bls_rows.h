// Table rows as the pooling kernels read them: bytes per row for every storage type, and a
// per-lane accumulator that loads its bytes of a row (from global memory or LDS), turns them into
// fp32 values and adds them.  Shared by the translation units with pooling kernels; everything is
// in an unnamed namespace, so every unit gets its own copy.
#pragma once

#include "bls_internal.h"

namespace {

// IEEE binary16 -> binary32 (exact; one v_cvt_f32_f16 each)
__device__ __forceinline__ float half_bits(unsigned short h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ __forceinline__ float half_lo(uint32_t w) { return half_bits((unsigned short)(w & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t w) { return half_bits((unsigned short)(w >> 16)); }

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_a4 __attribute__((aligned(4)));   // a row's scale and bias sit on a 4-byte boundary

// Bytes of a row that hold its elements, and bytes from one row to the next.
__host__ __device__ constexpr bool is_rowq(int dtype) { return dtype == BLS_U8_ROWQ || dtype == BLS_F8_ROWQ; }
__host__ __device__ __forceinline__ int64_t payload_bytes(int dtype, int D)
{
    return is_rowq(dtype) ? (int64_t)D : (int64_t)D * (dtype == BLS_FP16 ? 2 : 4);
}
__host__ __device__ __forceinline__ int64_t stride_bytes(int dtype, int D)
{
    return is_rowq(dtype) ? ((int64_t)D + 8 + 15) / 16 * 16 : payload_bytes(dtype, D);
}

// Per-lane accumulator: VB bytes of table storage per lane and row, NV values in them.
// Row-quantised rows also bring their scale and bias (8 bytes behind the codes, the same
// address for every lane of the group), and a value is code * scale + bias with the product
// and the sum each rounded to fp32.
template <int DT, int VB> struct Acc {
    static constexpr int NW = VB / 4;                              // 32-bit words loaded per row
    static constexpr int NV = is_rowq(DT) ? VB : DT == BLS_FP16 ? VB / 2 : VB / 4;   // fp32 values accumulated
    static constexpr int NX = is_rowq(DT) ? 2 : 0;                  // scale, bias
    struct Raw { uint32_t w[NW + NX]; };
    float a[NV];

    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) a[i] = 0.f;
    }
    static __device__ __forceinline__ Raw none()
    {
        Raw r;
#pragma unroll
        for (int i = 0; i < NW + NX; ++i) r.w[i] = 0u;
        return r;
    }
    // tables live in global memory: say so, or the loads are emitted as flat accesses.
    // p: this lane's bytes of the row; p + tail: the row's scale and bias (row-quantised only)
    static __device__ __forceinline__ Raw load(const char *p, int tail)
    {
        Raw r;
        if constexpr (NX == 2) {
            const u32x2 sb = *(const __attribute__((address_space(1))) u32x2_a4 *)(p + tail);
            r.w[NW] = sb.x; r.w[NW + 1] = sb.y;
        }
        if constexpr (NW == 4) {
            const u32x4 v = *(const __attribute__((address_space(1))) u32x4 *)p;
            r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
        } else if constexpr (NW == 2) {
            const u32x2 v = *(const __attribute__((address_space(1))) u32x2 *)p;
            r.w[0] = v.x; r.w[1] = v.y;
        } else {
            r.w[0] = *(const __attribute__((address_space(1))) uint32_t *)p;
        }
        return r;
    }
    // the same from LDS (a row copied there whole, scale and bias included)
    static __device__ __forceinline__ Raw load_lds(const unsigned char *p, int tail)
    {
        Raw r;
        if constexpr (NX == 2) {
            const u32x2 sb = *(const __attribute__((address_space(3))) u32x2_a4 *)(p + tail);
            r.w[NW] = sb.x; r.w[NW + 1] = sb.y;
        }
        if constexpr (NW == 4) {
            const u32x4 v = *(const __attribute__((address_space(3))) u32x4 *)p;
            r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
        } else if constexpr (NW == 2) {
            const u32x2 v = *(const __attribute__((address_space(3))) u32x2 *)p;
            r.w[0] = v.x; r.w[1] = v.y;
        } else {
            r.w[0] = *(const __attribute__((address_space(3))) uint32_t *)p;
        }
        return r;
    }
    // byte k of a word of codes as the number the row format gives it: an unsigned integer, or an
    // E4M3 float (v_cvt_f32_fp8, exact), times the scale, plus the bias
    template <int K>
    static __device__ __forceinline__ float decode(uint32_t word, float scale, float bias)
    {
        float code;
        if constexpr (DT == BLS_F8_ROWQ) code = __builtin_amdgcn_cvt_f32_fp8((int)word, K);
        else code = (float)((word >> (8 * K)) & 0xffu);
        const float prod = code * scale;
        return prod + bias;
    }
    __device__ __forceinline__ void add(const Raw &r)
    {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            if constexpr (is_rowq(DT)) {
                const float sc = __uint_as_float(r.w[NW]), bi = __uint_as_float(r.w[NW + 1]);
                a[4 * i + 0] += decode<0>(r.w[i], sc, bi); a[4 * i + 1] += decode<1>(r.w[i], sc, bi);
                a[4 * i + 2] += decode<2>(r.w[i], sc, bi); a[4 * i + 3] += decode<3>(r.w[i], sc, bi);
            } else if constexpr (DT == BLS_FP16) { a[2 * i] += half_lo(r.w[i]); a[2 * i + 1] += half_hi(r.w[i]); }
            else a[i] += __uint_as_float(r.w[i]);
        }
    }
    // per-sample weight: the product is rounded to fp32, then added (no fused multiply-add)
    __device__ __forceinline__ void add_weighted(const Raw &r, float w)
    {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            if constexpr (is_rowq(DT)) {
                const float sc = __uint_as_float(r.w[NW]), bi = __uint_as_float(r.w[NW + 1]);
                const float t0 = w * decode<0>(r.w[i], sc, bi), t1 = w * decode<1>(r.w[i], sc, bi);
                const float t2 = w * decode<2>(r.w[i], sc, bi), t3 = w * decode<3>(r.w[i], sc, bi);
                a[4 * i + 0] += t0; a[4 * i + 1] += t1; a[4 * i + 2] += t2; a[4 * i + 3] += t3;
            } else if constexpr (DT == BLS_FP16) {
                const float p0 = w * half_lo(r.w[i]), p1 = w * half_hi(r.w[i]);
                a[2 * i] += p0; a[2 * i + 1] += p1;
            } else {
                const float p0 = w * __uint_as_float(r.w[i]);
                a[i] += p0;
            }
        }
    }
    __device__ __forceinline__ void store(float *p) const
    {
        if constexpr (NV % 4 == 0) {
#pragma unroll
            for (int i = 0; i < NV / 4; ++i)
                reinterpret_cast<float4 *>(p)[i] = make_float4(a[4 * i], a[4 * i + 1], a[4 * i + 2], a[4 * i + 3]);
        } else if constexpr (NV == 2) {
            *reinterpret_cast<float2 *>(p) = make_float2(a[0], a[1]);
        } else {
            p[0] = a[0];
        }
    }
};

}  // namespace
