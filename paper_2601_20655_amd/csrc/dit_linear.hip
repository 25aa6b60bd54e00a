// Dense projection of token rows on the matrix cores: y[M, N] = x[M, K] w[N, K]^T + bias[N]
// (the q/k/v and output projections either side of attention in a transformer block of the Diffusion
// stage, Sec. 2.4; weights stored [out, in] as the model's linear layers keep them).
//
// A workgroup of 8 wavefronts computes 256-token x 256-feature tiles of y, walking K in steps of 64.
// Both operand tiles of a step (256 rows x 64 contraction indices, 16-bit: one 128-byte line per row)
// are copied from global memory straight into LDS by the load-to-LDS DMA, 1 KiB per wavefront
// instruction.  The DMA fills LDS densely in lane order, so the bank spreading is done by choosing
// WHICH 16-byte piece of a row each lane fetches: piece p of row r lives in slot p ^ ((r >> 1) & 7) of
// the row's 128 bytes, which makes every cycle of a fragment read fall into 16 distinct bank groups
// (measured: no bank conflicts).
//
// Buffering: all 160 KiB of LDS are used, 3 buffers for the x tile (fetched two steps ahead) and 2 for the
// w tile (one step ahead), one barrier per step.
//
// MFMA roles: w rows ride the A operand (the M axis of v_mfma_f32_16x16x32_bf16), token rows the
// B operand; wavefront (wt, wf) of the 2 x 4 grid computes 128 tokens x 64 features: 32 accumulators
// of 4 registers, 24 fragment reads per 64 MFMAs, two wavefronts per SIMD.  The 16x16x32 form does the
// same flops per cycle as the 32x32x16 one and draws less power per flop, and the board's power
// limit, not the issue rate, is what bounds a dense product on real data: 1,220 -> 1,315 TFLOP/s on
// the same box for the same schedule.
//
// What in-kernel timestamps showed, and what was done about it (M = 32,760, K = 5,120, N = 15,360):
//  - one workgroup per tile spent a tenth of the time between the end of one tile's loop and the start
//    of the next one's on a compute unit (stores, workgroup launch, first loads): the workgroups are
//    persistent and a tile's first loads go out during the tile before;
//  - stores of 32-byte pieces straight from the accumulators held the stream up for another tenth:
//    tiles are staged through LDS and stored as whole rows;
//  - four MFMAs back to back followed by the reads and loads of a token block leave the pipe idle while
//    those issue: everything that is not an MFMA sits between the MFMAs;
//  - the two wavefronts of a SIMD do not advance evenly (the older is served first and waits a third of
//    every step at the barrier): the older ones issue all the loads.
// Together 1,315 -> 1,421 TFLOP/s, where the vendor's GEMM library does 1,493 on the same box.
// Tried without gain: alternating wavefront priorities, bursts against spread loads, 384-token tiles,
// row strides padded against channel conflicts (the vendor library gains 15 % from those on all-zero
// operands and nothing on real ones).
#include <type_traits>

#include "dit_attn_device.h"
#include "dit_attn_internal.h"

namespace dit {

namespace {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

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

template <bool OUT_F32, int QKV>
__global__ void __launch_bounds__(64 * kLinWaves, 1) linear_kernel(const LinearArgs a) {
    // QKV: 0 plain rows; 1 the fused q/k/v form; 2 the same with the k rows RMS-normalised per head; 3 with the
    // per-token normalisation's first half (weights applied, sums of squares left for k_rescale_kernel)
    static_assert(!(OUT_F32 && QKV), "the fused q/k/v form writes 16-bit rows and tiles");
    static_assert(kLinBM == 256 && kLinBN == 256 && kLinBK == 64, "tile shape");
    constexpr int SX = kLinSX, SW = kLinSW, NW = kLinWaves;
    constexpr int BR = 16;       // rows of an MFMA block
    constexpr int FB = 4;        // 16-feature blocks per wavefront
    constexpr int TB = 8;        // 16-token blocks per wavefront
    constexpr int NLW = 4;        // wavefronts that issue the loads (the first four: see below)
    constexpr int NCH = 32 / NLW;  // 1 KiB chunks (8 rows) per loading wavefront and tile
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

    // Persistent workgroups: the grid holds one workgroup per compute unit (or one per tile, if there are
    // fewer tiles), and a workgroup walks its tiles one after the other as ONE stream of steps: the loads of
    // a tile's first steps go out during the last steps of the tile before, and the only thing that
    // happens between two tiles is the store of the accumulators.  (One workgroup per tile spent a tenth of
    // the time between the end of one tile's loop and the start of the next one's on a compute unit:
    // stores, workgroup launch, the first loads' round trip.)
    // Tile order.  Workgroups are dealt to the 8 XCDs round-robin; each XCD is given a contiguous range of
    // logical tile ids, which its workgroups take in turn, and logical ids run feature tile by feature
    // tile through groups of 8 token tiles, so the 32 tiles an XCD works on at a time share 8 x tiles and
    // 4 w tiles in its L2.
    const int ntiles = a.nTM * a.nTN;
    int first_tile, my_tiles, tile_stride;  // logical ids first_tile + i * tile_stride, i < my_tiles
    {
        const int nblk = gridDim.x, bid = blockIdx.x;
        const int xcd = bid & 7, slot = bid >> 3;
        const int chunk = ntiles >> 3, rem = ntiles & 7;
        const int count = chunk + (xcd < rem ? 1 : 0);   // tiles of this XCD
        tile_stride = (nblk - xcd + 7) >> 3;             // workgroups of this XCD
        first_tile = xcd * chunk + (xcd < rem ? xcd : rem) + slot;
        my_tiles = count > slot ? (count - slot + tile_stride - 1) / tile_stride : 0;
    }
    if (my_tiles == 0) return;
    auto tile_coords = [&](int i, int& tm, int& tn) __attribute__((always_inline)) {
        i = i < my_tiles ? i : my_tiles - 1;  // (past the end: the last tile again, for loads nobody uses)
        const int logical = first_tile + i * tile_stride;
        const int per_group = kLinGroup * a.nTN;
        const int group = logical / per_group, within = logical - group * per_group;
        const int first = group * kLinGroup;
        const int gsz = a.nTM - first < kLinGroup ? a.nTM - first : kLinGroup;
        tm = first + within % gsz;
        tn = within / gsz;
    };

    // ---- DMA sources: wavefront w of the first four moves 1 KiB chunks w, w+4, .., w+28 of both tiles; a
    // chunk is 8 rows.  (The two wavefronts of a SIMD do not advance evenly: the older one is served first and
    // reaches the step's barrier about a third of a step early, the younger one is the critical path.  So the
    // older ones -- wavefronts 0..3, one per SIMD -- issue all the loads, and the younger ones only multiply.)
    // Rows past the end of x or w are clamped to the last one (their products are never stored).
    // A lane's byte offset from the tile's first row (32 bits: the host checks that a tile's extent fits) is
    // worked out at each load from its row in chunk 0 and its 16-byte piece, which is the same for every
    // chunk (chunks are 32 rows apart, the swizzle has period 16 rows): two registers instead of a table
    // of sixteen.  The tile base and the step's column offset are wavefront-uniform.
    // The loads run two steps ahead of the MFMAs, so they have a tile and a step of their own.
    const int nK = a.K / kLinBK;
    const int load_row0 = 8 * (wave & (NLW - 1)) + (lane >> 3);
    const uint32_t load_piece = 16u * ((lane & 7) ^ ((load_row0 >> 1) & 7));
    const uint32_t ldx2 = (uint32_t)(a.ldx * 2), ldw2 = (uint32_t)(a.ldw * 2);
    const uint8_t *xtile, *wtile;
    int xrow_max, wrow_max;  // last valid row of the tile being loaded, from the tile's first row
    int load_tile = 0, load_kt = 0;
    auto set_load_tile = [&](int i) __attribute__((always_inline)) {
        int tm, tn;
        tile_coords(i, tm, tn);
        xrow_max = a.M - 1 - tm * kLinBM;
        wrow_max = a.N - 1 - tn * kLinBN;
        xtile = reinterpret_cast<const uint8_t*>(a.x + (int64_t)tm * kLinBM * a.ldx);
        wtile = reinterpret_cast<const uint8_t*>(a.w + (int64_t)tn * kLinBN * a.ldw);
    };
    set_load_tile(0);
    auto next_load_step = [&]() __attribute__((always_inline)) {
        if (++load_kt == nK) {
            load_kt = 0;
            set_load_tile(++load_tile);
        }
    };
    // (the empty asm keeps the compiler from working the offsets out ahead of the loop and carrying them
    // through it, and from folding base + offset into per-lane 64-bit pointers)
    auto dma_chunk = [&](const uint8_t* tile, int row_max, uint32_t ld2, int lds_byte, int i) __attribute__((always_inline)) {
        int r = load_row0;
        asm volatile("" : "+v"(r));
        r += 8 * NLW * i;
        r = r < row_max ? r : row_max;
        uint32_t o = (uint32_t)r * ld2 + load_piece;
        asm volatile("" : "+v"(o));
        __builtin_amdgcn_global_load_lds((gptr_t)(tile + load_kt * (kLinBK * 2) + o),
                                         (lptr_t)(smem + lds_byte + ((wave & (NLW - 1)) + i * NLW) * 1024), 16, 0, 0);
    };
    auto dma_x_chunk = [&](int buf, int i) __attribute__((always_inline)) { dma_chunk(xtile, xrow_max, ldx2, buf * kLinTileBytes, i); };
    auto dma_w_chunk = [&](int buf, int i) __attribute__((always_inline)) {
        dma_chunk(wtile, wrow_max, ldw2, kWBase + buf * kLinTileBytes, i);
    };
    const bool loader = wave < NLW;
    auto dma_x = [&](int buf) {
        if (!loader) return;
#pragma unroll
        for (int i = 0; i < NCH; ++i) dma_x_chunk(buf, i);
    };
    auto dma_w = [&](int buf) {
        if (!loader) return;
#pragma unroll
        for (int i = 0; i < NCH; ++i) dma_w_chunk(buf, i);
    };

    // ---- fragment addresses: row base + swizzled piece of contraction slice ks.  The same swizzle serves
    // this read pattern: the LDS serves a 128-bit read in four cycles of 16 lanes (lane quads {0,3,5,6},
    // {1,2,4,7}, {8,11,13,14}, {9,10,12,15}), and with piece (4 ks + lg) ^ ((row >> 1) & 7) each of those
    // cycles touches 16 different 16-byte bank groups.
    const int sw = (lr >> 1) & 7;
    int koff[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) koff[ks] = ((4 * ks + lg) ^ sw) * 16;
    int xread = (wt * BR * TB + lr) * ROWB;
    int wread = kWBase + (wf * BR * FB + lr) * ROWB;

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
    auto read_w = [&](u32x4& w, auto fb, int buf, int ks) __attribute__((always_inline)) {
        const uint32_t wa = lds0 + buf * kLinTileBytes + wread + koff[ks];
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(w) : "v"(wa), "n"(decltype(fb)::value * BR * ROWB));
    };
    auto read_x = [&](u32x4& x, auto tb, int buf, int ks) __attribute__((always_inline)) {
        const uint32_t xa = lds0 + buf * kLinTileBytes + xread + koff[ks];
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(x) : "v"(xa), "n"(decltype(tb)::value * BR * ROWB));
    };
    // The barrier that opens step k sits in the last slice of step k-1, in its second token block: by then
    // every wavefront has asked for all fragments of step k-1 (the wait in front of the barrier completes
    // the reads), so behind it the buffers of step k-1 may be refilled and the tiles of step k, which the loading
    // wavefronts have waited for, may be read.  The loads of one barrier period go out between the MFMAs:
    // the w tile of step k+1 in the first four blocks behind the barrier (two chunks a block), the x tile
    // of step k+2 one chunk a block in the first slice of the next step.  The counted wait in front of the
    // barrier leaves exactly that youngest x tile in flight.
    // (the bare barrier instruction: __syncthreads() is a fence too, for which the compiler drains every
    // load in flight -- vmcnt(0) -- in front of the barrier, and the x tile that is meant to stay in
    // flight across it would be waited for after all)
    auto sync_point = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NCH) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // ---- store of a finished tile.  A lane holds token (column lr of block tb) and four consecutive features
    // per accumulator (16 fb + 4 lg + e of its wavefront's 64), so stored from the accumulators a wavefront
    // instruction would write sixteen 32-byte pieces, and a tile's 4,096 such pieces held the stream up for a
    // tenth of the time.  So a wavefront passes its share through LDS, 4 KiB at a time, and stores whole
    // output rows: 8 (bf16) or 16 (fp32) lanes per row of its 64 features, 16 bytes each.  The staging area is
    // the x buffer of the step just finished: behind that step's barrier nobody reads it any more, and the
    // loads that refill it are issued in the next step -- behind the barrier that ends the store, so that a
    // loading wavefront that has stored cannot overwrite what another one still stages.  Pieces of a staged
    // row are swizzled with the row number.  The accumulators start the next tile at zero.
    auto store_tile = [&](int tm, int tn, int stage_buf) __attribute__((always_inline)) {
        constexpr int ES = OUT_F32 ? 4 : 2;   // bytes per output element
        constexpr int RB = 64 * ES;           // bytes per staged row (the wavefront's 64 features)
        constexpr int PR = RB / 16;           // 16-byte pieces per row
        constexpr int RP = 4096 / RB;         // rows per pass
        constexpr int TBP = RP / BR;          // token blocks per pass
        uint2 bb[FB];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) {
            const int n0 = tn * kLinBN + wf * BR * FB + fb * BR + 4 * lg;
            bb[fb] = make_uint2(0u, 0u);
            if (a.bias && n0 < a.N) bb[fb] = *reinterpret_cast<const uint2*>(a.bias + n0);
        }
        uint8_t* const region = smem + stage_buf * kLinTileBytes + wave * 4096;
        const int rrow = lane / PR, rp = lane % PR;
        const int n = tn * kLinBN + wf * BR * FB + rp * (16 / ES);
        // (16-bit output only: with fp32 output the extra path costs the step loop a register)
        const bool full = !OUT_F32 && (tm + 1) * kLinBM <= a.M && (tn + 1) * kLinBN <= a.N;  // uniform
#pragma unroll
        for (int pass = 0; pass < TB / TBP; ++pass) {
#pragma unroll
            for (int h = 0; h < TBP; ++h) {
                const int tb = pass * TBP + h;
                const int row = BR * h + lr;
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) {
                    const float b0 = __uint_as_float(bb[fb].x << 16), b1 = __uint_as_float(bb[fb].x & 0xffff0000u);
                    const float b2 = __uint_as_float(bb[fb].y << 16), b3 = __uint_as_float(bb[fb].y & 0xffff0000u);
                    const float y0 = acc[fb][tb][0] + b0, y1 = acc[fb][tb][1] + b1;
                    const float y2 = acc[fb][tb][2] + b2, y3 = acc[fb][tb][3] + b3;
                    const int col = (BR * fb + 4 * lg) * ES;
                    uint8_t* const dst = region + row * RB + (((col >> 4) ^ (row & (PR - 1))) << 4) + (col & 15);
                    if constexpr (OUT_F32) *reinterpret_cast<float4*>(dst) = make_float4(y0, y1, y2, y3);
                    else *reinterpret_cast<uint2*>(dst) = make_uint2(pack2<OP_BF16>(y0, y1), pack2<OP_BF16>(y2, y3));
                }
            }
            auto staged = [&](int k) __attribute__((always_inline)) {
                const int row = k * (64 / PR) + rrow;
                return *reinterpret_cast<const uint4*>(region + row * RB + ((rp ^ (row & (PR - 1))) << 4));
            };
            auto put = [&](int k, uint4 v) __attribute__((always_inline)) {
                const int m = tm * kLinBM + wt * BR * TB + pass * RP + k * (64 / PR) + rrow;
                // N is a multiple of 8: a piece of a row is inside or outside as a whole
                if (m < a.M && n < a.N)
                    *reinterpret_cast<uint4*>(static_cast<uint8_t*>(a.y) + ((int64_t)m * a.ldy + n) * ES) = v;
            };
            if (full) {
                // a tile inside y stores without tests, and all four pieces of the pass are read back before the
                // first is stored (behind a test each read sits in a branch of its own and is waited for there)
                u32x4 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int row = k * (64 / PR) + rrow;
                    v[k] = *reinterpret_cast<const u32x4*>(region + row * RB + ((rp ^ (row & (PR - 1))) << 4));
                }
                asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3])::"memory");
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int m = tm * kLinBM + wt * BR * TB + pass * RP + k * (64 / PR) + rrow;
                    *reinterpret_cast<u32x4*>(static_cast<uint8_t*>(a.y) + ((int64_t)m * a.ldy + n) * ES) = v[k];
                }
            } else {
                // (two at a time: the loop around this leaves few registers free)
                {
                    const uint4 v0 = staged(0), v1 = staged(1);
                    put(0, v0);
                    put(1, v1);
                }
                {
                    const uint4 v2 = staged(2), v3 = staged(3);
                    put(2, v2);
                    put(3, v3);
                }
            }
        }
        // (zeroed here, not as they are staged: the registers of staged accumulators serve as temporaries)
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[fb][tb][r] = 0.f;
        __builtin_amdgcn_s_barrier();
    };

    // ---- store of a finished tile, fused q/k/v form.  A wavefront's 64 features are half a head of ONE of q, k, v
    // (a part starts on a multiple of 256 features).  Staged as 16-bit rows as above, 32 tokens a pass; what differs
    // is what happens on the way in (k rows are rotated, each part is rounded to its own type, tokens past the end of
    // the sequence become zeros in the k and v parts: they fill the last tile's slots) and where the rows go: q rows
    // to y; k rows to the K' part of the token's tile image (row = key, its 16-byte chunks in the image's swizzled
    // order); v rows transposed: a lane gathers, for one channel, the eight keys of a V^T chunk in the order the
    // attention kernel's PV operand wants them (pack_tile, layout 1) and writes the chunk to the V^T part.
    // With the per-head RMS normalisation the k rows are scaled first (hd0 + ... indexes the [H*128] weights).
    auto store_tile_qkv = [&](int tm, int tn, int stage_buf) __attribute__((always_inline)) {
        using G = TileGeom<128>;
        constexpr int RB = 128, PR = 8, RP = 32, TBP = 2;
        // (every per-lane offset below comes from a lane number the compiler cannot see through: worked out ahead of
        // the tile stream they do not fit the registers the loop leaves, and their reloads from scratch memory put
        // a wait for ALL loads in flight into the loop)
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int lr = ln & 15, lg = ln >> 4;
        const int HD = a.qkv_H * 128;
        const int n_wave = tn * kLinBN + wf * BR * FB;  // first feature of this wavefront's share
        const int part = n_wave / HD;                   // 0: q, 1: k, 2: v
        const int hd0 = n_wave - part * HD;
        const int h = hd0 >> 7, c0 = hd0 & 127;         // head, first channel (0 or 64)
        uint2 bb[FB];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) {
            bb[fb] = make_uint2(0u, 0u);
            if (QKV < 2 && a.bias) bb[fb] = *reinterpret_cast<const uint2*>(a.bias + n_wave + fb * BR + 4 * lg);
        }
        uint8_t* const region = smem + stage_buf * kLinTileBytes + wave * 4096;
        // RMS normalisation of the k rows over the head's 128 channels, in fp32 on the accumulators (a tile is one
        // part, so the whole workgroup takes this branch or none of it does).  This wavefront holds 64 of a head's
        // channels and wavefront wave ^ 2 the other 64: pass by pass the two exchange the sums of squares of the
        // pass's 32 tokens through the staging regions (two at a time: the tile stream leaves few registers), and
        // the rows are scaled as they are staged.
        const bool normed = QKV >= 2 && part == 1;
        // k and v values pass through bf16 first, as the rows of the plain projection would: what the attention call
        // then computes is, bit for bit, what it computes from those rows
        auto as_bf16_row = [](float& y0, float& y1) __attribute__((always_inline)) {
            const uint32_t u = pack2<OP_BF16>(y0, y1);
            y0 = __uint_as_float(u << 16);
            y1 = __uint_as_float(u & 0xffff0000u);
        };
        if constexpr (QKV >= 2) {
            // (the bias goes into the accumulators first: its registers are needed below)
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) {
                uint2 b = make_uint2(0u, 0u);
                if (a.bias) b = *reinterpret_cast<const uint2*>(a.bias + n_wave + fb * BR + 4 * lg);
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    acc[fb][tb][0] += __uint_as_float(b.x << 16);
                    acc[fb][tb][1] += __uint_as_float(b.x & 0xffff0000u);
                    acc[fb][tb][2] += __uint_as_float(b.y << 16);
                    acc[fb][tb][3] += __uint_as_float(b.y & 0xffff0000u);
                    if (part != 0) {
                        float y0 = acc[fb][tb][0], y1 = acc[fb][tb][1], y2 = acc[fb][tb][2], y3 = acc[fb][tb][3];
                        as_bf16_row(y0, y1);
                        as_bf16_row(y2, y3);
                        acc[fb][tb][0] = y0;
                        acc[fb][tb][1] = y1;
                        acc[fb][tb][2] = y2;
                        acc[fb][tb][3] = y3;
                    }
                }
            }
        }
        uint8_t* const tiles_h = a.qkv_tiles + (size_t)h * a.qkv_nKT * G::TILE_BYTES;
        const int rrow = ln / PR, rp = ln % PR;
        const int tok_end = a.qkv_nKT * kBK;  // slots of the sequence's tiles
#pragma unroll
        for (int pass = 0; pass < TB / TBP; ++pass) {
            const int tok0 = tm * kLinBM + wt * BR * TB + pass * RP;  // a multiple of 32: half a key tile
            float rs2[TBP] = {1.f, 1.f};
            if (normed) {
                float* const mine = reinterpret_cast<float*>(region);
                const float* const theirs =
                    reinterpret_cast<const float*>(smem + stage_buf * kLinTileBytes + (wave ^ 2) * 4096);
#pragma unroll
                for (int hh = 0; hh < TBP; ++hh) {
                    const int tb = pass * TBP + hh;
                    float ss = 0.f;
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) ss = fmaf(acc[fb][tb][e], acc[fb][tb][e], ss);
                    }
                    ss += __shfl_xor(ss, 16);
                    ss += __shfl_xor(ss, 32);
                    if (lg == 0) mine[hh * BR + lr] = ss;
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
#pragma unroll
                for (int hh = 0; hh < TBP; ++hh) {
                    const float ssq = mine[hh * BR + lr] + theirs[hh * BR + lr];
                    if constexpr (QKV == 2) {
                        rs2[hh] = 1.0f / sqrtf(ssq * (1.0f / 128.0f) + a.qkv_eps);
                    } else {
                        // per-token mean: this head's share goes into the spare bytes behind the K' rows of the
                        // token's tile (one float per key slot), where k_rescale_kernel adds up the heads' shares
                        const int tok = tok0 + hh * BR + lr;
                        if (c0 == 0 && lg == 0 && tok < tok_end)
                            reinterpret_cast<float*>(tiles_h + (size_t)(tok >> 6) * G::TILE_BYTES + kBK * G::KROW)[tok & 63] = ssq;
                    }
                }
                // the partner has read this region before the staging below overwrites it
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
#pragma unroll
            for (int hh = 0; hh < TBP; ++hh) {
                const int tb = pass * TBP + hh;
                const int row = BR * hh + lr;
                const int tok = tok0 + row;
                int pt = 0, ph = 0, pw = 0;
                if (part == 1) token_pos(tok < a.M ? tok : a.M - 1, a.qkv_rg, pt, ph, pw);
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) {
                    const float b0 = __uint_as_float(bb[fb].x << 16), b1 = __uint_as_float(bb[fb].x & 0xffff0000u);
                    const float b2 = __uint_as_float(bb[fb].y << 16), b3 = __uint_as_float(bb[fb].y & 0xffff0000u);
                    float y0 = acc[fb][tb][0], y1 = acc[fb][tb][1], y2 = acc[fb][tb][2], y3 = acc[fb][tb][3];
                    if constexpr (QKV < 2) {
                        y0 += b0;
                        y1 += b1;
                        y2 += b2;
                        y3 += b3;
                    }
                    if (normed) {
                        float4 g = make_float4(1.f, 1.f, 1.f, 1.f);
                        if (a.qkv_kgamma) g = *reinterpret_cast<const float4*>(a.qkv_kgamma + hd0 + fb * BR + 4 * lg);
                        const float rs = rs2[hh];
                        y0 *= rs * g.x;
                        y1 *= rs * g.y;
                        y2 *= rs * g.z;
                        y3 *= rs * g.w;
                    }
                    if (QKV < 2 && part != 0) {
                        as_bf16_row(y0, y1);
                        as_bf16_row(y2, y3);
                    }
                    if (part == 1) {  // the two rotation pairs of channels c0 + 16 fb + 4 lg .. + 3
                        const RopeGeom& rg = a.qkv_rg;
#pragma unroll
                        for (int pp = 0; pp < 2; ++pp) {
                            const int ip = ((c0 + BR * fb + 4 * lg) >> 1) + pp;
                            int idx;
                            if (ip < rg.hd[0]) idx = rg.off[0] + pt * rg.hd[0] + ip;
                            else if (ip < rg.hd[0] + rg.hd[1]) idx = rg.off[1] + ph * rg.hd[1] + (ip - rg.hd[0]);
                            else idx = rg.off[2] + pw * rg.hd[2] + (ip - rg.hd[0] - rg.hd[1]);
                            const float2 cs = a.qkv_tab[idx];
                            float& x0 = pp ? y2 : y0;
                            float& x1 = pp ? y3 : y1;
                            const float r0 = x0 * cs.x - x1 * cs.y, r1 = x0 * cs.y + x1 * cs.x;
                            x0 = r0;
                            x1 = r1;
                        }
                    }
                    if (part != 0 && tok >= a.M) y0 = y1 = y2 = y3 = 0.f;
                    const bool f16 = part == 1 ? a.qkv_qk_f16 != 0 : part == 2 ? a.qkv_pv_f16 != 0 : false;
                    const uint2 packed = f16 ? make_uint2(pack2<OP_F16>(y0, y1), pack2<OP_F16>(y2, y3))
                                             : make_uint2(pack2<OP_BF16>(y0, y1), pack2<OP_BF16>(y2, y3));
                    const int col = (BR * fb + 4 * lg) * 2;
                    *reinterpret_cast<uint2*>(region + row * RB + (((col >> 4) ^ (row & (PR - 1))) << 4) + (col & 15)) = packed;
                }
            }
            if (part == 2) {
                // V^T: lane = channel d of the wavefront's 64; chunk j of this half tile holds the keys (slots
                // 4 g + e) 16 g + 4 j + e of the pass's 32
                const int d = ln, dch = c0 + d;
                const int tile = tok0 >> 6, half = (tok0 >> 5) & 1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t w4[4];
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int e2 = 0; e2 < 2; ++e2) {
                            const int r0 = 16 * g + 4 * j + 2 * e2, r1 = r0 + 1;
                            const uint32_t lo = *reinterpret_cast<const uint16_t*>(
                                region + r0 * RB + ((((d >> 3) ^ (r0 & (PR - 1)))) << 4) + (d & 7) * 2);
                            const uint32_t hi = *reinterpret_cast<const uint16_t*>(
                                region + r1 * RB + ((((d >> 3) ^ (r1 & (PR - 1)))) << 4) + (d & 7) * 2);
                            w4[2 * g + e2] = lo | (hi << 16);
                        }
                    const int kc = 4 * half + j;
                    const int kcs = kc ^ (((dch >> 2) ^ (dch >> 3)) & 1);
                    // (the rows' 16 pad bytes stay unwritten here: writing them, which takes a third off the
                    // stand-alone pre-pack pass, measured level in this epilogue and costs it registers)
                    if (tok0 < tok_end)
                        *reinterpret_cast<uint4*>(tiles_h + (size_t)tile * G::TILE_BYTES + G::K_BYTES + dch * G::VROW +
                                                  kcs * 16) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
                }
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int r = k * (64 / PR) + rrow;
                    const uint4 v = *reinterpret_cast<const uint4*>(region + r * RB + ((rp ^ (r & (PR - 1))) << 4));
                    const int tok = tok0 + r;
                    if (part == 0) {
                        if (tok < a.M)
                            *reinterpret_cast<uint4*>(static_cast<uint16_t*>(a.y) + (int64_t)tok * a.qkv_sq_t +
                                                      (int64_t)h * a.qkv_sq_h + c0 + rp * 8) = v;
                    } else if (tok < tok_end) {
                        const int tile = tok >> 6, rr = tok & 63;
                        const int chunk = (c0 >> 3) + rp;
                        const int cs = chunk ^ (((rr >> 2) ^ (rr >> 3)) & 1);
                        *reinterpret_cast<uint4*>(tiles_h + (size_t)tile * G::TILE_BYTES + rr * G::KROW + cs * 16) = v;
                    }
                }
            }
        }
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[fb][tb][r] = 0.f;
        __builtin_amdgcn_s_barrier();
    };

    // Prologue: tiles x(0), w(0), x(1) in a burst; the first barrier; then what a last slice would
    // have sent behind it (the w tile of step 1); the loop sends the rest.
    dma_x(0);
    dma_w(0);
    next_load_step();
    dma_x(1);
    sync_point();
    dma_w(1);
    next_load_step();
    int xb = 0, wb = 0;  // buffers of the step being multiplied
    static_for<0, FB>([&](auto fb) { read_w(W[0][decltype(fb)::value], fb, wb, 0); });
    static_for<0, TB - 1>([&](auto tb) { read_x(X[decltype(tb)::value], tb, xb, 0); });
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    int tile = 0, kt = 0;  // the step being multiplied
    int tm, tn;
    tile_coords(0, tm, tn);
    const int nsteps = my_tiles * nK;
    auto run = [&](auto loads) __attribute__((always_inline)) {
    constexpr bool LOADS = decltype(loads)::value;
    for (int step = 0; step < nsteps; ++step) {
        const int xb_next = xb + 1 == SX ? 0 : xb + 1, wb_next = wb ^ 1;
        const int xb_prev = xb == 0 ? SX - 1 : xb - 1;
        auto block = [&](auto ksc, auto tbc) __attribute__((always_inline)) {
            constexpr int ks = decltype(ksc)::value, T = decltype(tbc)::value;
            constexpr bool last = ks + 1 == NKS;
            constexpr int cur = ks & 1, nxt = cur ^ 1;
            // fragments of the next slice come from this step's buffers, or from the next step's
            const int nxb = last ? xb_next : xb, nwb = last ? wb_next : wb;
            constexpr int nks = last ? 0 : ks + 1;
            // reads issued behind the youngest fragment this block needs (its x fragment; in the first
            // block of a slice the slice's last w fragment), from the issue order below
            constexpr int YOUNGER = last ? (T < 2 ? 6 : T == 2 ? 8 : 10) : (T == 0 ? 5 : 10);
            if constexpr (T == 0) {
                asm volatile("s_waitcnt lgkmcnt(%5)"
                             : "+v"(W[cur][0]), "+v"(W[cur][1]), "+v"(W[cur][2]), "+v"(W[cur][3]), "+v"(X[T])
                             : "n"(YOUNGER));
            } else {
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(X[T]) : "n"(YOUNGER));
            }
            acc[0][T] = mfma16<OP_BF16>(W[cur][0], X[T], acc[0][T]);
            __builtin_amdgcn_sched_barrier(0);
            // (after the last step the loads and reads behind this barrier go to buffers nobody uses:
            // uniform control flow)
            if constexpr (last && T == 1) sync_point();
            // the x fragment of the block before: its MFMAs have issued
            if constexpr (T == 0) read_x(X[TB - 1], std::integral_constant<int, TB - 1>(), xb, ks);
            else read_x(X[T - 1], std::integral_constant<int, T - 1>(), nxb, nks);
            __builtin_amdgcn_sched_barrier(0);
            acc[1][T] = mfma16<OP_BF16>(W[cur][1], X[T], acc[1][T]);
            __builtin_amdgcn_sched_barrier(0);
            // this block's share of the loads (q = token blocks since the barrier); both tiles are those
            // of the step two ahead
            // (the w tile, needed a step from now, two chunks a block; the x tile, needed two steps from now, one)
            constexpr int q = last ? T - 1 : TB - 1 + T;
            if constexpr (LOADS && q >= 0 && 2 * q < NCH) {
                dma_w_chunk(wb, 2 * q);
                dma_w_chunk(wb, 2 * q + 1);
            } else if constexpr (LOADS && q >= TB - 1 && q - (TB - 1) < NCH) {
                dma_x_chunk(xb_prev, q - (TB - 1));
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
        static_for<0, NKS>([&](auto ksc) __attribute__((always_inline)) {
            static_for<0, TB>([&](auto tbc) __attribute__((always_inline)) { block(ksc, tbc); });
        });
        xb = xb_next;
        wb = wb_next;
        if constexpr (LOADS) next_load_step();
        if (++kt == nK) {
            if constexpr (QKV) store_tile_qkv(tm, tn, xb == 0 ? SX - 1 : xb - 1);
            else store_tile(tm, tn, xb == 0 ? SX - 1 : xb - 1);
            if constexpr (QKV != 0) {
                // The fused forms work the per-lane fragment offsets out again behind every store of a tile, from
                // a lane number the compiler cannot see through: they are then new values here, not values that
                // have to survive the store, which has no register to spare for them (kept across it, one of them
                // was spilled and reloaded INSIDE the step loop, and a reload from scratch memory there makes the
                // compiler wait for every load in flight).
                int l = lane;
                asm volatile("" : "+v"(l));
                const int r = l & 15, g = l >> 4;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) koff[ks] = ((4 * ks + g) ^ ((r >> 1) & 7)) * 16;
                xread = (wt * BR * TB + r) * ROWB;
                wread = kWBase + (wf * BR * FB + r) * ROWB;
            }
            kt = 0;
            tile_coords(++tile, tm, tn);
        }
    }
    };
    if (loader) run(std::true_type());
    else run(std::false_type());
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus loads of the last steps
}

template <bool OUT_F32, int QKV>
hipError_t launch_linear_inst(const LinearArgs& a, hipStream_t s) {
    auto kern = linear_kernel<OUT_F32, QKV>;
    constexpr int smem = (kLinSX + kLinSW) * kLinTileBytes;
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    // one workgroup per compute unit (a workgroup takes all of a unit's LDS), fewer if there are fewer tiles
    int dev = 0, cus = 0;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    const int64_t ntiles = (int64_t)a.nTM * a.nTN;
    const unsigned grid = (unsigned)(ntiles < cus ? ntiles : cus);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * kLinWaves), smem, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(const LinearArgs& a, hipStream_t s) {
    if (a.qkv) {
        if (a.qkv_norm == 2) return launch_linear_inst<false, 3>(a, s);
        return a.qkv_norm ? launch_linear_inst<false, 2>(a, s) : launch_linear_inst<false, 1>(a, s);
    }
    return a.out_f32 ? launch_linear_inst<true, false>(a, s) : launch_linear_inst<false, false>(a, s);
}

}  // namespace dit
