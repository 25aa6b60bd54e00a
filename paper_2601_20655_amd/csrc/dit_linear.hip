// Dense projection of token rows on the matrix cores: y[M, N] = x[M, K] w[N, K]^T + bias[N]
// (the q/k/v and output projections either side of attention in a transformer block of the Diffusion
// stage, Sec. 2.4; weights stored [out, in] as the model's linear layers keep them).
//
// One workgroup of 8 wavefronts owns a 256-token x 256-feature tile of y and walks K in steps of 64.
// Both operand tiles of a step (256 rows x 64 contraction indices, 16-bit: one 128-byte line per row)
// are copied from global memory straight into LDS by the load-to-LDS DMA, 1 KiB per wavefront
// instruction.  The DMA fills LDS densely in lane order, so the bank spreading is done by choosing
// WHICH 16-byte piece of a row each lane fetches: piece p of row r lives in slot p ^ ((r >> 1) & 7) of
// the row's 128 bytes, which makes the 16 rows a quarter wavefront reads with one ds_read_b128 fall
// into 16 distinct bank groups (measured: no bank conflicts).
//
// Buffering: all 160 KiB of LDS are used, SX = 3 buffers for the x tile (fetched two steps ahead) and
// SW = 2 for the w tile (one step ahead).  The loads of a step are issued one or two at a time between
// groups of MFMAs, never in a burst, and the one barrier per step sits where every wavefront still
// has MFMAs in flight.
//
// MFMA roles: w rows ride the A operand (the M axis of v_mfma_f32_32x32x16_bf16), token rows the
// B operand, so a lane ends up with four CONSECUTIVE features of one token per register quad and
// stores them with one instruction.  With 8 wavefronts, wavefront (wt, wf) of the 2 x 4 grid computes
// 128 tokens x 64 features (8 accumulators, 6 fragment reads per 8 MFMAs, two wavefronts per SIMD);
// with 4 wavefronts 128 x 128 (16 accumulators in the AGPRs, one wavefront per SIMD).  The two forms
// measure the same (1,250 TFLOP/s at M = 32,760, N = K = 5,120); the 8-wavefront form is the default.
// Bursts against spread loads, a two-slice read-ahead, 384-token tiles (17 % less L2 traffic), loads
// staggered between even and odd wavefronts and wavefront priorities all stayed within 2 %.
#include <type_traits>

#include "dit_attn_device.h"
#include "dit_attn_internal.h"

namespace dit {

namespace {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

#ifndef DIT_LIN_PRIO
#define DIT_LIN_PRIO 0
#endif
constexpr int kLinGroup = 8;  // token tiles per group of the workgroup order
constexpr int kLinTileBytes = 256 * kLinBK * 2;  // one operand tile of one step
constexpr int kLinSX = 3, kLinSW = 2;  // LDS buffers of x tiles (fetched two steps ahead) and of w tiles (one ahead)
constexpr int kLinWaves = 8;

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>());
        static_for<I + 1, N>(f);
    }
}

template <bool OUT_F32>
__global__ void __launch_bounds__(64 * kLinWaves, 1) linear_kernel(const LinearArgs a) {
    static_assert(kLinBM == 256 && kLinBN == 256 && kLinBK == 64, "tile shape");
    constexpr int SX = kLinSX, SW = kLinSW, NW = kLinWaves;
    constexpr int BR = 16;       // rows of an MFMA block
    constexpr int FB = 4;        // 16-feature blocks per wavefront
    constexpr int TB = 8;        // 16-token blocks per wavefront
    constexpr int NCH = 32 / NW;  // 1 KiB chunks (8 rows) per wavefront and tile
    constexpr int ROWB = 128;  // bytes per row of a tile
    constexpr int NKS = 2;     // contraction slices (32 indices) per step
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // LDS map: the x buffers, then the w buffers
    constexpr int kWBase = SX * kLinTileBytes;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 15, lg = lane >> 4;  // row of a block, 16-byte piece of a slice
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
    // Per lane: 32-bit byte offsets from the tile's first row (the host checks that a tile's extent
    // fits 32 bits); the tile base and the step's column offset are wavefront-uniform.
    uint32_t xoff[NCH], woff[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int r = 8 * (wave + NW * i) + (lane >> 3);
        const int p = (lane & 7) ^ ((r >> 1) & 7);
        int xr = tm * kLinBM + r, wr = tn * kLinBN + r;
        xr = (xr < a.M ? xr : a.M - 1) - tm * kLinBM;
        wr = (wr < a.N ? wr : a.N - 1) - tn * kLinBN;
        xoff[i] = (uint32_t)xr * (uint32_t)(a.ldx * 2) + 16 * p;
        woff[i] = (uint32_t)wr * (uint32_t)(a.ldw * 2) + 16 * p;
    }
    const uint8_t* const xtile = reinterpret_cast<const uint8_t*>(a.x + (int64_t)tm * kLinBM * a.ldx);
    const uint8_t* const wtile = reinterpret_cast<const uint8_t*>(a.w + (int64_t)tn * kLinBN * a.ldw);
    const int nK = a.K / kLinBK;
    // (a tile number past the end fetches the last tile again, into a buffer nobody reads any more:
    // every step then has the same number of loads in flight, which the counted wait relies on; the
    // empty asm keeps the compiler from folding base + offset into per-lane 64-bit pointers ahead of
    // the loop, which would cost two registers per load)
    auto dma_chunk = [&](const uint8_t* tile, uint32_t o, int kt, int lds_byte, int i) {
        kt = kt < nK ? kt : nK - 1;
        asm volatile("" : "+v"(o));
        __builtin_amdgcn_global_load_lds((gptr_t)(tile + kt * (kLinBK * 2) + o),
                                         (lptr_t)(smem + lds_byte + (wave + i * NW) * 1024), 16, 0, 0);
    };
    auto dma_x = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) dma_chunk(xtile, xoff[i], kt, buf * kLinTileBytes, i);
    };
    auto dma_w = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) dma_chunk(wtile, woff[i], kt, kWBase + buf * kLinTileBytes, i);
    };

    // ---- fragment addresses: row base + swizzled piece of contraction slice ks.  The same swizzle serves
    // this read pattern: the LDS serves a 128-bit read in four cycles of 16 lanes (lane quads {0,3,5,6},
    // {1,2,4,7}, {8,11,13,14}, {9,10,12,15}), and with piece (4 ks + lg) ^ ((row >> 1) & 7) each of those
    // cycles touches 16 different 16-byte bank groups.
    const int sw = (lr >> 1) & 7;
    int koff[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) koff[ks] = ((4 * ks + lg) ^ sw) * 16;
    const int xread = (wt * BR * TB + lr) * ROWB;
    const int wread = kWBase + (wf * BR * FB + lr) * ROWB;

    f32x4 acc[FB][TB];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[fb][tb][r] = 0.f;

    // Operand fragments.  A slice (32 contraction indices) takes FB fragments of w and TB of x and feeds
    // FB x TB MFMAs, walked token block by token block.  The w fragments are double-buffered and requested
    // a slice ahead; an x fragment is used by the FB MFMAs of its token block and refilled IN PLACE one
    // block later (an LDS return into registers whose MFMAs have issued is safe), so only one set is held.
    // The reads are inline assembly so that the waits can be counted: LDS returns in order, and the number
    // of reads issued behind the one a block needs is a constant of the block's place in the step, so a
    // fragment is asked for 5 to 10 reads (2 to 9 token blocks) before its use.  The compiler itself waits
    // for LDS reads with lgkmcnt(0), which would drain that queue at every use.
    //
    // Everything that is not an MFMA -- one or two LDS reads, at most one load, their address arithmetic --
    // is placed BETWEEN the four MFMAs of a token block (scheduling barriers pin the order), so that it
    // issues while the matrix pipe works on the MFMA in front of it: a wavefront issues in order, and four
    // MFMAs back to back followed by the rest leave the pipe idle for as long as the rest takes to issue.
    u32x4 W[2][FB], X[TB];
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    auto read_w = [&](u32x4& w, auto fb, int buf, int ks) {
        const uint32_t wa = lds0 + buf * kLinTileBytes + wread + koff[ks];
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(w) : "v"(wa), "n"(decltype(fb)::value * BR * ROWB));
    };
    auto read_x = [&](u32x4& x, auto tb, int buf, int ks) {
        const uint32_t xa = lds0 + buf * kLinTileBytes + xread + koff[ks];
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(x) : "v"(xa), "n"(decltype(tb)::value * BR * ROWB));
    };
    // The barrier that opens step k sits in the last slice of step k-1, in its second token block: by then
    // every wavefront has asked for all fragments of step k-1 (the wait in front of the barrier completes
    // the reads), so behind it the buffers of step k-1 may be refilled and the tiles of step k, which every
    // wavefront has waited for, may be read.  The loads of one barrier period go out one per token block:
    // the w tile of step k+1 in the first four blocks behind the barrier, the x tile of step k+2 in the
    // first four blocks of the next step.  The counted wait in front of the barrier leaves exactly that
    // youngest x tile in flight.
    // (the bare barrier instruction: __syncthreads() is a fence too, for which the compiler drains every
    // load in flight -- vmcnt(0) -- in front of the barrier, and the x tile that is meant to stay in
    // flight across it would be waited for after all)
    auto sync_point = [&]() {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NCH) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // Prologue: tiles x(0), w(0), x(1) in a burst; the first barrier; then what a last slice would
    // have sent behind it (the w tile of step 1); the loop sends the rest.
    dma_x(0, 0);
    dma_w(0, 0);
    dma_x(1, 1);
    sync_point();
    dma_w(1, 1);
    int xb = 0, wb = 0;  // buffers of the step being multiplied
    static_for<0, FB>([&](auto fb) { read_w(W[0][decltype(fb)::value], fb, wb, 0); });
    static_for<0, TB - 1>([&](auto tb) { read_x(X[decltype(tb)::value], tb, xb, 0); });
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    for (int kt = 0; kt < nK; ++kt) {
        const int xb_next = xb + 1 == SX ? 0 : xb + 1, wb_next = wb ^ 1;
        const int xb_prev = xb == 0 ? SX - 1 : xb - 1, wb_prev = wb ^ 1;
        auto block = [&](auto ksc, auto tbc) {
            constexpr int ks = decltype(ksc)::value, T = decltype(tbc)::value;
            constexpr bool last = ks + 1 == NKS;
            constexpr int cur = ks & 1, nxt = cur ^ 1;
            // fragments of the next slice come from this step's buffers, or from the next step's
            const int nxb = last ? xb_next : xb, nwb = last ? wb_next : wb;
            constexpr int nks = last ? 0 : ks + 1;
            // reads issued behind the youngest fragment this block needs (its x fragment; in the first
            // block of a slice the slice's last w fragment), from the issue order below
            constexpr int YOUNGER = last ? (T < 2 ? 6 : T == 2 ? 8 : 10) : (T == 0 ? 5 : 10);
            if constexpr (DIT_LIN_PRIO == 1) {
                if constexpr (T % 2 == 0) __builtin_amdgcn_s_setprio((T & 2) ? 0 : 1);
            }
            if constexpr (T == 0) {
                asm volatile("s_waitcnt lgkmcnt(%5)"
                             : "+v"(W[cur][0]), "+v"(W[cur][1]), "+v"(W[cur][2]), "+v"(W[cur][3]), "+v"(X[T])
                             : "n"(YOUNGER));
            } else {
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(X[T]) : "n"(YOUNGER));
            }
            acc[0][T] = mfma16<OP_BF16>(W[cur][0], X[T], acc[0][T]);
            __builtin_amdgcn_sched_barrier(0);
            // (after the last tile the loads and reads behind this barrier go to buffers nobody uses:
            // uniform control flow)
            if constexpr (last && T == 1) sync_point();
            // the x fragment of the block before: its MFMAs have issued
            if constexpr (T == 0) read_x(X[TB - 1], std::integral_constant<int, TB - 1>(), xb, ks);
            else read_x(X[T - 1], std::integral_constant<int, T - 1>(), nxb, nks);
            __builtin_amdgcn_sched_barrier(0);
            acc[1][T] = mfma16<OP_BF16>(W[cur][1], X[T], acc[1][T]);
            __builtin_amdgcn_sched_barrier(0);
            // this block's share of the loads (q = token blocks since the barrier)
            constexpr int q = last ? T - 1 : TB - 1 + T;
            if constexpr (q >= 0 && q < NCH) {
                dma_chunk(wtile, woff[q], kt + SW, kWBase + wb * kLinTileBytes, q);
            } else if constexpr (q >= TB - 1 && q - (TB - 1) < NCH) {
                dma_chunk(xtile, xoff[q - (TB - 1)], kt + SX - 1, xb_prev * kLinTileBytes, q - (TB - 1));
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[2][T] = mfma16<OP_BF16>(W[cur][2], X[T], acc[2][T]);
            __builtin_amdgcn_sched_barrier(0);
            // the next slice's w fragments, two per block (behind the barrier in the last slice)
            constexpr int wi = last ? T - 1 : T;
            if constexpr (wi == 0 || wi == 1) {
                read_w(W[nxt][2 * wi], std::integral_constant<int, 2 * wi>(), nwb, nks);
                read_w(W[nxt][2 * wi + 1], std::integral_constant<int, 2 * wi + 1>(), nwb, nks);
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[3][T] = mfma16<OP_BF16>(W[cur][3], X[T], acc[3][T]);
            __builtin_amdgcn_sched_barrier(0);
        };
        static_for<0, NKS>([&](auto ksc) { static_for<0, TB>([&](auto tbc) { block(ksc, tbc); }); });
        xb = xb_next;
        wb = wb_next;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus loads of the last steps

    // ---- epilogue: lane holds token (column lr of block tb) and four consecutive features per accumulator:
    // 16 fb + 4 lg + e of its wavefront's share.
    // All bias values are fetched before the first store: a load waited for behind stores would wait
    // for the stores too (one counter tracks both), several round trips in a row.
    auto feature0 = [&](int fb) { return tn * kLinBN + wf * BR * FB + fb * BR + 4 * lg; };
    uint2 bb[FB];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) {
        const int n0 = feature0(fb);
        bb[fb] = make_uint2(0u, 0u);
        if (a.bias && n0 < a.N) bb[fb] = *reinterpret_cast<const uint2*>(a.bias + n0);
    }
    // (the wait for them happens here, once: the empty statement reads every value)
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) asm volatile("" : "+v"(bb[fb].x), "+v"(bb[fb].y));
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) {
        const int n0 = feature0(fb);
        if (n0 >= a.N) continue;  // N is a multiple of 8: a quad is inside or outside as a whole
        const float b0 = __uint_as_float(bb[fb].x << 16), b1 = __uint_as_float(bb[fb].x & 0xffff0000u);
        const float b2 = __uint_as_float(bb[fb].y << 16), b3 = __uint_as_float(bb[fb].y & 0xffff0000u);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const int m = tm * kLinBM + wt * BR * TB + tb * BR + lr;
            if (m >= a.M) continue;
            const float y0 = acc[fb][tb][0] + b0, y1 = acc[fb][tb][1] + b1;
            const float y2 = acc[fb][tb][2] + b2, y3 = acc[fb][tb][3] + b3;
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
    constexpr int smem = (kLinSX + kLinSW) * kLinTileBytes;
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((int64_t)a.nTM * a.nTN)), dim3(64 * kLinWaves), smem, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(const LinearArgs& a, hipStream_t s) {
    return a.out_f32 ? launch_linear_inst<true>(a, s) : launch_linear_inst<false>(a, s);
}

}  // namespace dit
