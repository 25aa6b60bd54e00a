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

#ifndef DIT_LIN_BK
#define DIT_LIN_BK 64
#endif
#ifndef DIT_LIN_STAGES
#define DIT_LIN_STAGES 2
#endif
#ifndef DIT_LIN_WAVES
#define DIT_LIN_WAVES 8
#endif
constexpr int kLinGroup = 8;  // token tiles per group of the workgroup order

// BK contraction indices per step (32 or 64), S stages of LDS, NW wavefronts (8: 128 tokens x 64
// features each, two per SIMD; 4: 128 x 128 each, one per SIMD with the accumulators in the AGPRs).
template <int BK, int S, int NW, bool OUT_F32>
__global__ void __launch_bounds__(64 * NW, 1) linear_kernel(const LinearArgs a) {
    static_assert(kLinBM == 256 && kLinBN == 256 && (BK == 32 || BK == 64) && S >= 2, "tile shape");
    static_assert(NW == 4 || NW == 8, "wavefronts per workgroup");
    constexpr int FB = 16 / NW;  // 32-feature blocks per wavefront
    constexpr int kLinStage = (kLinBM + kLinBN) * BK * 2;  // bytes of one stage: x tile, then w tile
    constexpr int kLinXBytes = kLinBM * BK * 2;
    constexpr int PPR = BK / 8;         // 16-byte pieces per row
    constexpr int RPC = 64 / PPR;       // rows per 1 KiB chunk
    constexpr int RP = 256 / (BK * 2);  // rows per 256 bytes (one sweep of the banks)
    constexpr int NCH = BK / 2 / NW;    // chunks per wavefront and tile
    constexpr int ROWB = BK * 2;        // bytes per row
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

    // ---- DMA sources: wavefront w moves 1 KiB chunks w, w+NW, ... of both tiles; a chunk is RPC rows.
    // Rows past the end of x or w are clamped to the last one (their products are never stored).
    const uint16_t* xsrc[NCH];
    const uint16_t* wsrc[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int r = RPC * (wave + NW * i) + lane / PPR;
        const int p = (lane % PPR) ^ ((r / RP) % PPR);
        int xr = tm * kLinBM + r, wr = tn * kLinBN + r;
        xr = xr < a.M ? xr : a.M - 1;
        wr = wr < a.N ? wr : a.N - 1;
        xsrc[i] = a.x + (int64_t)xr * a.ldx + 8 * p;
        wsrc[i] = a.w + (int64_t)wr * a.ldw + 8 * p;
    }
    const int nK = a.K / BK;
    // (a tile number past the end fetches the last tile again, into a stage nobody reads any more:
    // every step then has the same number of loads in flight, which the counted wait relies on)
    auto dma = [&](int kt, int st) {
        kt = kt < nK ? kt : nK - 1;
        uint8_t* const xd = smem + st * kLinStage + wave * 1024;
        uint8_t* const wd = xd + kLinXBytes;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            __builtin_amdgcn_global_load_lds((gptr_t)(xsrc[i] + kt * BK), (lptr_t)(xd + i * NW * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(wsrc[i] + kt * BK), (lptr_t)(wd + i * NW * 1024), 16, 0, 0);
        }
    };

    // ---- fragment addresses: row base + swizzled piece of contraction step ks ----
    const int sw = (l32 / RP) % PPR;
    int koff[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) koff[ks] = ((2 * ks + half) ^ sw) * 16;
    const int xread = (wt * 128 + l32) * ROWB;
    const int wread = kLinXBytes + (wf * 32 * FB + l32) * ROWB;

    f32x16 acc[FB][4];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fb][tb][r] = 0.f;

    // Operand fragments of one 16-index slice: 2 of w, 4 of x.  Two sets alternate, so the reads of
    // the next slice are in flight while the MFMAs of the current one issue.
    struct Frag {
        u32x4 w[FB], x[4];
    };
    constexpr int NKS = BK / 16;
    Frag F[2];
    auto read_frags = [&](Frag& f, int stage, int ks) {
        const uint8_t* const xs = smem + stage * kLinStage + xread + koff[ks];
        const uint8_t* const ws = smem + stage * kLinStage + wread + koff[ks];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) f.w[fb] = *reinterpret_cast<const u32x4*>(ws + fb * 32 * ROWB);
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) f.x[tb] = *reinterpret_cast<const u32x4*>(xs + tb * 32 * ROWB);
    };
    auto mfma_row = [&](const Frag& f, int fb) {
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) acc[fb][tb] = mfma32<OP_BF16>(f.w[fb], f.x[tb], acc[fb][tb]);
    };
    // Tiles kt+1 .. kt+S-2 may still be in flight when tile kt is needed; the counted wait leaves
    // exactly their loads outstanding, and the barrier then says that every wavefront's share of the
    // tile has landed AND that every wavefront has read all it needs of the previous tile, whose stage
    // the next loads overwrite.
    auto next_tile = [&](int kt_next, int st_next) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * 2 * NCH) : "memory");
        __syncthreads();
        dma(kt_next + S - 1, st_next == 0 ? S - 1 : st_next - 1);
    };
#pragma unroll
    for (int j = 0; j < S - 1; ++j) dma(j, j);
    next_tile(0, 0);
    read_frags(F[0], 0, 0);
    int st = 0;
    for (int kt = 0; kt < nK; ++kt) {
        const int st_next = st + 1 == S ? 0 : st + 1;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            // Half of the slice's MFMAs, then the reads of the next slice, then the other half: a
            // fragment is asked for 8 MFMAs of this SIMD (its two wavefronts take turns) before its use.
            // When the next slice belongs to the next tile the barrier comes first: by then this
            // wavefront has read every fragment of the present tile, so the present stage may be
            // refilled behind the barrier.  (A read-ahead of two slices with counted waits, the
            // wavefronts of a SIMD at different priorities, the loads spread over the step, 4
            // wavefronts of 128 x 128: all measured the same or slower.)
#pragma unroll
            for (int fb = 0; fb < FB / 2; ++fb) mfma_row(F[ks & 1], fb);
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 1 < NKS) {
                read_frags(F[(ks + 1) & 1], st, ks + 1);
            } else {
                // (after the last tile this fetches and reads a stage nobody uses: uniform control flow)
                next_tile(kt + 1, st_next);
                read_frags(F[0], st_next, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int fb = FB / 2; fb < FB; ++fb) mfma_row(F[ks & 1], fb);
            __builtin_amdgcn_sched_barrier(0);
        }
        st = st_next;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus loads of the last steps

    // ---- epilogue: lane holds token (column l32 of block tb), features 32*fb + 8*g + 4*half + e ----
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n0 = tn * kLinBN + wf * 32 * FB + fb * 32 + 8 * g + 4 * half;
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
    auto kern = linear_kernel<DIT_LIN_BK, DIT_LIN_STAGES, DIT_LIN_WAVES, OUT_F32>;
    constexpr int smem = DIT_LIN_STAGES * (kLinBM + kLinBN) * DIT_LIN_BK * 2;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((int64_t)a.nTM * a.nTN)), dim3(64 * DIT_LIN_WAVES), smem, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(const LinearArgs& a, hipStream_t s) {
    return a.out_f32 ? launch_linear_inst<true>(a, s) : launch_linear_inst<false>(a, s);
}

}  // namespace dit
