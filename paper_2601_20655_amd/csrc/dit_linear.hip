// Dense projection of token rows on the matrix cores: y[M, N] = x[M, K] w[N, K]^T + bias[N]
// (the q/k/v and output projections either side of attention in a transformer block of the Diffusion
// stage, Sec. 2.4; weights stored [out, in] as the model's linear layers keep them).
//
// One workgroup of 8 wavefronts owns a 256-token x 256-feature tile of y and walks K in steps of 64.
// Both operand tiles of a step (256 rows x 64 contraction indices, 16-bit) are copied from global
// memory straight into LDS by the load-to-LDS DMA, 1 KiB per wavefront instruction, two stages deep:
// the copies of step j+1 fly while step j is multiplied.  The DMA fills LDS densely in lane order,
// so the bank spreading is done by choosing WHICH 16-byte piece of a row each lane fetches: piece p
// of row r lives in slot p ^ ((r >> 1) & 7) of the row's 128 bytes, which makes the 16 rows a quarter
// wavefront reads with one ds_read_b128 fall into 16 distinct bank groups.
//
// MFMA roles: w rows ride the A operand (the M axis of v_mfma_f32_32x32x16_bf16), token rows the
// B operand, so a lane ends up with four CONSECUTIVE features of one token per register quad and
// stores them with one instruction.  Wavefront (wt, wf) of the 2 x 4 grid computes 128 tokens x 64
// features: 8 accumulators, 6 fragment reads per 8 MFMAs.
#include "dit_attn_device.h"
#include "dit_attn_internal.h"

namespace dit {

namespace {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int kLinStage = (kLinBM + kLinBN) * kLinBK * 2;  // bytes of one stage: x tile, then w tile
constexpr int kLinXBytes = kLinBM * kLinBK * 2;
constexpr int kLinGroup = 8;  // token tiles per group of the workgroup order

template <bool OUT_F32>
__global__ void __launch_bounds__(512, 1) linear_kernel(const LinearArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wt = wave & 1, wf = wave >> 1;

    // Workgroup order.  Workgroups are dealt to the 8 XCDs round-robin; each XCD is given a contiguous
    // range of logical ids, and logical ids run feature tile by feature tile through groups of 8
    // token tiles, so the 32 workgroups an XCD holds at a time share 8 x tiles and 4 w tiles in its L2.
    int tm, tn;
    {
        const int nblk = gridDim.x, bid = blockIdx.x;
        const int xcd = bid & 7, idx = bid >> 3;
        const int chunk = nblk >> 3, rem = nblk & 7;
        const int logical = xcd * chunk + (xcd < rem ? xcd : rem) + idx;
        const int per_group = kLinGroup * a.nTN;
        const int group = logical / per_group, within = logical - group * per_group;
        const int first = group * kLinGroup;
        const int gsz = a.nTM - first < kLinGroup ? a.nTM - first : kLinGroup;
        tm = first + within % gsz;
        tn = within / gsz;
    }

    // ---- DMA sources: wavefront w moves 1 KiB chunks w, w+8, w+16, w+24 of both tiles; a chunk is 8
    // rows.  Rows past the end of x or w are clamped to the last one (their products are never stored).
    const uint16_t* xsrc[4];
    const uint16_t* wsrc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 8 * (wave + 8 * i) + (lane >> 3);
        const int p = (lane & 7) ^ ((r >> 1) & 7);
        int xr = tm * kLinBM + r, wr = tn * kLinBN + r;
        xr = xr < a.M ? xr : a.M - 1;
        wr = wr < a.N ? wr : a.N - 1;
        xsrc[i] = a.x + (int64_t)xr * a.ldx + 8 * p;
        wsrc[i] = a.w + (int64_t)wr * a.ldw + 8 * p;
    }
    auto dma = [&](int kt, int st) {
        uint8_t* const xd = smem + st * kLinStage + wave * 1024;
        uint8_t* const wd = xd + kLinXBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __builtin_amdgcn_global_load_lds((gptr_t)(xsrc[i] + kt * kLinBK), (lptr_t)(xd + i * 8192), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(wsrc[i] + kt * kLinBK), (lptr_t)(wd + i * 8192), 16, 0, 0);
        }
    };

    // ---- fragment addresses: row base + swizzled piece of contraction step ks ----
    const int sw = (l32 >> 1) & 7;
    int koff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) koff[ks] = ((2 * ks + half) ^ sw) * 16;
    const int xread = (wt * 128 + l32) * 128;
    const int wread = kLinXBytes + (wf * 64 + l32) * 128;

    f32x16 acc[2][4];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fb][tb][r] = 0.f;

    const int nK = a.K / kLinBK;
    dma(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int kt = 0; kt < nK; ++kt) {
        const int st = kt & 1;
        // stage st^1 was last read in step kt-1, which every wavefront left through the barrier
        if (kt + 1 < nK) dma(kt + 1, st ^ 1);
        const uint8_t* const xs = smem + st * kLinStage + xread;
        const uint8_t* const ws = smem + st * kLinStage + wread;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 wfrag[2], xfrag[4];
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) wfrag[fb] = *reinterpret_cast<const u32x4*>(ws + fb * 4096 + koff[ks]);
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) xfrag[tb] = *reinterpret_cast<const u32x4*>(xs + tb * 4096 + koff[ks]);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                for (int tb = 0; tb < 4; ++tb) acc[fb][tb] = mfma32<OP_BF16>(wfrag[fb], xfrag[tb], acc[fb][tb]);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- epilogue: lane holds token (column l32 of block tb), features 32*fb + 8*g + 4*half + e ----
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n0 = tn * kLinBN + wf * 64 + fb * 32 + 8 * g + 4 * half;
            if (n0 >= a.N) continue;  // N is a multiple of 8: a quad is inside or outside as a whole
            float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
            if (a.bias) {
                const uint2 bb = *reinterpret_cast<const uint2*>(a.bias + n0);
                b0 = __uint_as_float(bb.x << 16);
                b1 = __uint_as_float(bb.x & 0xffff0000u);
                b2 = __uint_as_float(bb.y << 16);
                b3 = __uint_as_float(bb.y & 0xffff0000u);
            }
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                const int m = tm * kLinBM + wt * 128 + tb * 32 + l32;
                if (m >= a.M) continue;
                const float y0 = acc[fb][tb][4 * g + 0] + b0, y1 = acc[fb][tb][4 * g + 1] + b1;
                const float y2 = acc[fb][tb][4 * g + 2] + b2, y3 = acc[fb][tb][4 * g + 3] + b3;
                const int64_t o = (int64_t)m * a.ldy + n0;
                if constexpr (OUT_F32) {
                    *reinterpret_cast<float4*>(static_cast<float*>(a.y) + o) = make_float4(y0, y1, y2, y3);
                } else {
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.y) + o) =
                        make_uint2(pack2<OP_BF16>(y0, y1), pack2<OP_BF16>(y2, y3));
                }
            }
        }
}

template <bool OUT_F32>
hipError_t launch_linear_inst(const LinearArgs& a, hipStream_t s) {
    auto kern = linear_kernel<OUT_F32>;
    constexpr int smem = 2 * kLinStage;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((int64_t)a.nTM * a.nTN)), dim3(512), smem, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(const LinearArgs& a, hipStream_t s) {
    return a.out_f32 ? launch_linear_inst<true>(a, s) : launch_linear_inst<false>(a, s);
}

}  // namespace dit
