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

#ifndef DIT_LIN_SX
#define DIT_LIN_SX 3
#endif
#ifndef DIT_LIN_SW
#define DIT_LIN_SW 2
#endif
#ifndef DIT_LIN_WAVES
#define DIT_LIN_WAVES 8
#endif
constexpr int kLinGroup = 8;  // token tiles per group of the workgroup order
constexpr int kLinTileBytes = 256 * kLinBK * 2;  // one operand tile of one step

// SX buffers for x tiles, SW for w tiles (SX = SW or SX = SW + 1).
template <int SX, int SW, int NW, bool OUT_F32>
__global__ void __launch_bounds__(64 * NW, 1) linear_kernel(const LinearArgs a) {
    static_assert(kLinBM == 256 && kLinBN == 256 && kLinBK == 64, "tile shape");
    static_assert(SW >= 2 && (SX == SW || SX == SW + 1), "buffering");
    static_assert(NW == 4 || NW == 8, "wavefronts: 2 (tokens) x NW/2 (features)");
    constexpr int FB = 16 / NW;  // 32-feature blocks per wavefront
    constexpr int TB = 4;        // 32-token blocks per wavefront
    constexpr int NCH = 32 / NW;  // 1 KiB chunks (8 rows) per wavefront and tile
    constexpr int ROWB = 128;  // bytes per row of a tile
    constexpr int NKS = kLinBK / 16;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // LDS map: the x buffers, then the w buffers
    constexpr int kWBase = SX * kLinTileBytes;
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

    // ---- fragment addresses: row base + swizzled piece of contraction slice ks ----
    const int sw = (l32 >> 1) & 7;
    int koff[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) koff[ks] = ((2 * ks + half) ^ sw) * 16;
    const int xread = (wt * 32 * TB + l32) * ROWB;
    const int wread = kWBase + (wf * 32 * FB + l32) * ROWB;

    f32x16 acc[FB][TB];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fb][tb][r] = 0.f;

    // Operand fragments.  A slice (16 contraction indices) takes FB fragments of w and TB of x.  The w
    // fragments are double-buffered and requested a whole slice ahead; an x fragment is used by the FB
    // MFMAs of its token block and then refilled IN PLACE with the next slice's fragment (an LDS
    // return into registers whose MFMAs have issued is safe), so only one set of them is held.
    // The reads are inline assembly so that the waits can be counted: LDS returns in order, and at
    // every use exactly FB + TB - 1 younger reads are in flight (the rest of this slice's x
    // fragments, the next w set, the refills already issued), so one constant serves every wait and a
    // fragment is asked for about 2 (TB - 1) + FB MFMAs of this wavefront before its use.  The compiler
    // itself waits for LDS reads with lgkmcnt(0), which would drain that queue at every use.
    constexpr int YOUNGER = FB + TB - 1;
    u32x4 W[2][FB], X[TB];
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    auto read_w = [&](u32x4 (&w)[FB], int buf, int ks) {
        const uint32_t wa = lds0 + buf * kLinTileBytes + wread + koff[ks];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(w[fb]) : "v"(wa), "n"(fb * 32 * ROWB));
    };
    auto read_x = [&](u32x4& x, auto tb, int buf, int ks) {
        const uint32_t xa = lds0 + buf * kLinTileBytes + xread + koff[ks];
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(x) : "v"(xa), "n"(decltype(tb)::value * 32 * ROWB));
    };
    // The barrier that opens step k sits in the last slice of step k-1, after the MFMAs of its first
    // token block: by then every wavefront has asked for all fragments of step k-1 (the wait completes
    // the reads; the last of them were requested a block earlier), so behind the barrier the buffers of
    // step k-1 may be refilled.  The loads of one barrier period go out between the MFMA groups, never
    // in a burst: the w tile of step k+SW-1 over the first four token blocks after the barrier, the x
    // tile of step k+SX-1 over the two slices before the next barrier.  The counted wait in front of
    // the barrier leaves exactly the youngest x tile in flight.
    static_assert(SX == 3 && SW == 2, "the load schedule below is written for 3 x and 2 w buffers");
    // (the bare barrier instruction: __syncthreads() is a fence too, for which the compiler drains every
    // load in flight -- vmcnt(0) -- in front of the barrier, and the x tile that is meant to stay in
    // flight across it would be waited for after all)
    auto sync_point = [&]() {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NCH) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    constexpr int WPB = NCH / 4;  // w chunks per token block
    // Prologue: tiles x(0), w(0), x(1) in a burst; the first barrier; then what a last slice would
    // have sent behind it (three token blocks' worth of w(1)); the loop sends the rest.
    dma_x(0, 0);
    dma_w(0, 0);
    dma_x(1, 1);
    sync_point();
#pragma unroll
    for (int i = 0; i < 3 * WPB; ++i) dma_chunk(wtile, woff[i], 1, kWBase + kLinTileBytes, i);
    int xb = 0, wb = 0;  // buffers of the step being multiplied
    read_w(W[0], wb, 0);
    read_x(X[0], std::integral_constant<int, 0>(), xb, 0);
    read_x(X[1], std::integral_constant<int, 1>(), xb, 0);
    read_x(X[2], std::integral_constant<int, 2>(), xb, 0);
    read_x(X[3], std::integral_constant<int, 3>(), xb, 0);
    for (int kt = 0; kt < nK; ++kt) {
        const int xb_next = xb + 1 == SX ? 0 : xb + 1, wb_next = wb ^ 1;
        const int xb_prev = xb == 0 ? SX - 1 : xb - 1, wb_prev = wb ^ 1;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bool last = ks + 1 == NKS;
            // fragments of the next slice come from this step's buffers, or from the next step's
            const int nxb = last ? xb_next : xb, nwb = last ? wb_next : wb;
            const int nks = last ? 0 : ks + 1;
            if (!last) read_w(W[(ks + 1) & 1], nwb, nks);
            auto block = [&](auto tb) {
                constexpr int T = decltype(tb)::value;
                // younger reads in flight at this use: the rest of the slice's x fragments, the next
                // w set and the refills already issued (the next w set is late in the last slice)
                if (last && T == 0) {
                    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(TB - 1));
                }
                if constexpr (FB == 2) {
                    asm volatile("s_waitcnt lgkmcnt(%3)"
                                 : "+v"(W[ks & 1][0]), "+v"(W[ks & 1][1]), "+v"(X[T])
                                 : "n"(YOUNGER));
                } else {
                    asm volatile("s_waitcnt lgkmcnt(%5)"
                                 : "+v"(W[ks & 1][0]), "+v"(W[ks & 1][1]), "+v"(W[ks & 1][2]), "+v"(W[ks & 1][3]),
                                   "+v"(X[T])
                                 : "n"(YOUNGER));
                }
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) acc[fb][T] = mfma32<OP_BF16>(W[ks & 1][fb], X[T], acc[fb][T]);
                if (last && T == 0) {
                    // (after the last tile the loads and reads behind this barrier go to buffers nobody
                    // uses: uniform control flow)
                    sync_point();
                    read_w(W[(ks + 1) & 1], nwb, nks);
                }
                read_x(X[T], tb, nxb, nks);
                // this block's share of the loads (q = token blocks since the barrier)
                const int q = last ? T - 1 : 3 + 4 * ks + T;
                if (q >= 0 && q < 4) {
#pragma unroll
                    for (int i = 0; i < WPB; ++i) {
                        const int c = q * WPB + i;
                        if (last) dma_chunk(wtile, woff[c], kt + SW, kWBase + wb * kLinTileBytes, c);
                        else dma_chunk(wtile, woff[c], kt + SW - 1, kWBase + wb_prev * kLinTileBytes, c);
                    }
                } else if (q >= 7 && q - 7 < NCH) {
                    dma_chunk(xtile, xoff[q - 7], kt + SX - 1, xb_prev * kLinTileBytes, q - 7);
                }
            };
            block(std::integral_constant<int, 0>());
            block(std::integral_constant<int, 1>());
            block(std::integral_constant<int, 2>());
            block(std::integral_constant<int, 3>());
        }
        xb = xb_next;
        wb = wb_next;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus loads of the last steps

    // ---- epilogue: lane holds token (column l32 of block tb), features 32*fb + 8*g + 4*half + e.
    // All bias values are fetched before the first store: a load waited for behind stores would wait
    // for the stores too (one counter tracks both), eight round trips in a row.
    uint2 bb[FB][4];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n0 = tn * kLinBN + wf * 32 * FB + fb * 32 + 8 * g + 4 * half;
            bb[fb][g] = make_uint2(0u, 0u);
            if (a.bias && n0 < a.N) bb[fb][g] = *reinterpret_cast<const uint2*>(a.bias + n0);
        }
    // (the wait for them happens here, once: the empty statement reads every value)
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int g = 0; g < 4; ++g) asm volatile("" : "+v"(bb[fb][g].x), "+v"(bb[fb][g].y));
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n0 = tn * kLinBN + wf * 32 * FB + fb * 32 + 8 * g + 4 * half;
            if (n0 >= a.N) continue;  // N is a multiple of 8: a quad is inside or outside as a whole
            const float b0 = __uint_as_float(bb[fb][g].x << 16), b1 = __uint_as_float(bb[fb][g].x & 0xffff0000u);
            const float b2 = __uint_as_float(bb[fb][g].y << 16), b3 = __uint_as_float(bb[fb][g].y & 0xffff0000u);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const int m = tm * kLinBM + wt * 32 * TB + tb * 32 + l32;
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
    auto kern = linear_kernel<DIT_LIN_SX, DIT_LIN_SW, DIT_LIN_WAVES, OUT_F32>;
    constexpr int smem = (DIT_LIN_SX + DIT_LIN_SW) * kLinTileBytes;
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((int64_t)a.nTM * a.nTN)), dim3(64 * DIT_LIN_WAVES), smem, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(const LinearArgs& a, hipStream_t s) {
    return a.out_f32 ? launch_linear_inst<true>(a, s) : launch_linear_inst<false>(a, s);
}

}  // namespace dit
