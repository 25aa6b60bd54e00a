// Device helpers shared by the gfx950 kernels: 16-bit operand packing, MFMA wrappers,
// input widening and the 3-axis rotary rotation of eight consecutive channels.
#pragma once
#include "dit_attn_internal.h"

namespace dit {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 mk4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) {
    u32x4 r = {x, y, z, w};
    return r;
}

// Two fp32 values -> one dword of two 16-bit operands, round to nearest even (low half = a).
template <int OP>
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    f32x2 f = {a, b};
    if constexpr (OP == OP_F16) {
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
    } else {
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
    }
}

// acc + lo + hi of one packed operand pair, summed in fp32 (one v_dot2c against (1, 1)).  Used for bf16
// probabilities only: the instruction does not overlap with a running MFMA.
template <int OP>
__device__ __forceinline__ float sum2(uint32_t packed, float acc) {
    if constexpr (OP == OP_F16) {
        const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, packed), one, acc, false);
    } else {
        const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), one, acc, false);
    }
}

// fp16 operands saturate: a value beyond the largest finite fp16 number becomes +-65504 instead of an
// infinity that would turn the products into NaN (bf16 inputs can hold such values).  NaN stays NaN.
constexpr float kF16Max = 65504.0f;
__device__ __forceinline__ float sat_f16(float x) { return x > kF16Max ? kF16Max : (x < -kF16Max ? -kF16Max : x); }

// Eight fp32 values -> four dwords of 16-bit operands, saturating for fp16.  Used where q', k' and v are
// rounded (prologue, pre-pack pass), never in the key loop: probabilities cannot overflow.
template <int OP>
__device__ __forceinline__ u32x4 pack8(const float x[8]) {
    if constexpr (OP == OP_F16) {
        return mk4(pack2<OP>(sat_f16(x[0]), sat_f16(x[1])), pack2<OP>(sat_f16(x[2]), sat_f16(x[3])),
                   pack2<OP>(sat_f16(x[4]), sat_f16(x[5])), pack2<OP>(sat_f16(x[6]), sat_f16(x[7])));
    } else {
        return mk4(pack2<OP>(x[0], x[1]), pack2<OP>(x[2], x[3]), pack2<OP>(x[4], x[5]), pack2<OP>(x[6], x[7]));
    }
}

// D(32x32, fp32) += A(32x16) * B(16x32).  Lane l supplies row (l % 32) of A and column
// (l % 32) of B, eight contraction indices each (group l / 32); it receives column (l % 32)
// of D, rows 8*(r/4) + 4*(l/32) + r%4 for r = 0..15.
template <int OP>
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
    if constexpr (OP == OP_F16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
}

// ---- 8-bit (OCP e4m3) score operands ----
typedef int i32x8 __attribute__((ext_vector_type(8)));

// Exponent e such that amax * 2^e lies in [128, 256), inside e4m3's normal range (largest finite
// value 448); 0 for an all-zero row.  Clamped so that 127 - e stays a valid 8-bit scale code.
__device__ __forceinline__ int fp8_row_exponent(float amax) {
    const int be = (int)((__float_as_uint(amax) >> 23) & 255u);  // amax in [2^(be-127), 2^(be-126))
    if (be == 0) return 0;
    const int e = 134 - be;
    return e > 100 ? 100 : (e < -100 ? -100 : e);
}
__device__ __forceinline__ float pow2i(int e) { return __uint_as_float((uint32_t)(e + 127) << 23); }

// Eight fp32 values -> eight e4m3 bytes (round to nearest even), byte i = x[i].
__device__ __forceinline__ uint2 pack8_fp8(const float x[8]) {
    int lo = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], 0, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], lo, true);
    int hi = __builtin_amdgcn_cvt_pk_fp8_f32(x[4], x[5], 0, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(x[6], x[7], hi, true);
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

// 16x16x32 form of the same instructions (half the issue time per instruction, same flops per cycle): lane
// 16 g + i supplies, for both operands, row i and contraction indices 8g .. 8g+7; result: column i, rows 4g .. 4g+3.
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int OP>
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
    if constexpr (OP == OP_F16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                      0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                       0, 0);
    }
}

// D(32x32, fp32) += 2^(sa-127) A(32x64, e4m3) * 2^(sb-127) B(64x32, e4m3).  Lane l supplies 32
// contraction indices of row (l % 32) of A and of column (l % 32) of B, the same 32 indices on
// both sides (group l / 32); sa and sb are the lane's own 8-bit scale codes for that row resp.
// column, and the two lanes of a row must carry the same code.  Result layout as mfma32.
__device__ __forceinline__ f32x16 mfma32_fp8(i32x8 a, i32x8 b, f32x16 c, int sa, int sb) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, sa, 0, sb);
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ void widen8(u32x4 u, float x[8]) {
    x[0] = bf16_lo(u.x); x[1] = bf16_hi(u.x);
    x[2] = bf16_lo(u.y); x[3] = bf16_hi(u.y);
    x[4] = bf16_lo(u.z); x[5] = bf16_hi(u.z);
    x[6] = bf16_lo(u.w); x[7] = bf16_hi(u.w);
}

// Eight consecutive channels starting at element offset `off` (a multiple of 8) as fp32.
__device__ __forceinline__ void load8(const void* base, int64_t off, int in_f32, float x[8]) {
    if (in_f32) {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + off);
        float4 lo = p[0], hi = p[1];
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
        x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
    } else {
        widen8(*reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + off), x);
    }
}

// Multiplier 1/sqrt(mean(x^2) + eps) of one q row.  The row's D channels are read by the lane
// pair (lane, lane ^ 32), lane half `half` taking chunks 2*ks + half; `base` is the element
// offset of the row's head, `stat` the row's index in the per-token table (mode 2).
template <int D>
__device__ __forceinline__ float q_row_rstd(const NormArgs& n, const void* q, int64_t base, int in_f32, int half,
                                            int64_t stat) {
    if (n.mode == 2) return n.rstd[stat];
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        float x[8];
        load8(q, base + 8 * (2 * ks + half), in_f32, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
    }
    ss += __shfl_xor(ss, 32);
    return 1.0f / sqrtf(ss * (1.0f / D) + n.eps);
}

// x[0..8) = channels [8c, 8c+8) of head h: times the row multiplier and the channel weights
__device__ __forceinline__ void norm8(float x[8], const NormArgs& n, float rs, int h, int D, int c) {
    if (n.gamma) {
        const float4* g = reinterpret_cast<const float4*>(n.gamma + (int64_t)h * D + 8 * c);
        const float4 g0 = g[0], g1 = g[1];
        x[0] *= rs * g0.x; x[1] *= rs * g0.y; x[2] *= rs * g0.z; x[3] *= rs * g0.w;
        x[4] *= rs * g1.x; x[5] *= rs * g1.y; x[6] *= rs * g1.z; x[7] *= rs * g1.w;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] *= rs;
    }
}

// Token index -> position indices along (t, h, w), counted from the grid origin.
__device__ __forceinline__ void token_pos(int n, const RopeGeom& rg, int& pt, int& ph, int& pw) {
    const int hw = rg.Hg * rg.Wg;
    pt = n / hw;
    const int rem = n - pt * hw;
    ph = rem / rg.Wg;
    pw = rem - ph * rg.Wg;
}

// Rotate channels [8c, 8c+8) = pairs 4c..4c+3 of a token at position indices (pt, ph, pw).
// A pair (x0, x1) becomes (x0 cos - x1 sin, x0 sin + x1 cos); all in fp32.
__device__ __forceinline__ void rope8(float x[8], int c, const RopeGeom& rg, const float2* tab,
                                      int pt, int ph, int pw) {
#pragma unroll
    for (int pp = 0; pp < 4; ++pp) {
        const int ip = 4 * c + pp;
        int idx;
        if (ip < rg.hd[0]) {
            idx = rg.off[0] + pt * rg.hd[0] + ip;
        } else if (ip < rg.hd[0] + rg.hd[1]) {
            idx = rg.off[1] + ph * rg.hd[1] + (ip - rg.hd[0]);
        } else {
            idx = rg.off[2] + pw * rg.hd[2] + (ip - rg.hd[0] - rg.hd[1]);
        }
        const float2 cs = tab[idx];
        const float x0 = x[2 * pp], x1 = x[2 * pp + 1];
        x[2 * pp] = x0 * cs.x - x1 * cs.y;
        x[2 * pp + 1] = x0 * cs.y + x1 * cs.x;
    }
}

}  // namespace dit
