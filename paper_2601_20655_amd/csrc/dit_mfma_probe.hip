// Measurement utility: what the matrix cores of this board sustain when they do nothing else.
// Every SIMD runs two wavefronts (the occupancy of the attention kernel) that issue 32x32x16 MFMAs back
// to back from registers: no memory traffic, no LDS, no vector arithmetic.  With constant operands the
// rate is bound by instruction issue and the clock; with random operands (significand bits toggling from
// one MFMA to the next) the board reaches its power limit and lowers the clock, which is the ceiling an
// attention kernel on real data lives under -- and that ceiling moves with the number of significand bits
// the data carries.  bench.py reports these rates beside the published peak.
#include "../../include/dit_attn.h"
#include "dit_attn_device.h"

namespace dit {
namespace {

constexpr int kProbeUnroll = 16;  // MFMAs per loop iteration: 4 A operands x 4 B operands, 4 accumulators in turn

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// One dword = two 16-bit floats +-(1.m) * 2^e with random sign, random significand of `bits` significant bits
// (the leading one included; the low stored bits are zero) and e in [-3, 0]: magnitudes like unit-variance
// activations, every kept significand bit equally likely to be set.
template <int OP>
__device__ __forceinline__ uint32_t random_pair(uint32_t h, int bits) {
    constexpr int STORED = OP == OP_F16 ? 10 : 7;
    const int keep = bits - 1 < 0 ? 0 : (bits - 1 > STORED ? STORED : bits - 1);
    const uint32_t mant_mask = ((1u << STORED) - 1u) & ~((1u << (STORED - keep)) - 1u);
    uint32_t r = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t b16 = (h >> (16 * i)) & 0xffffu;
        const uint32_t sign = b16 >> 15, e = (b16 >> 13) & 3u;
        uint32_t v;
        if constexpr (OP == OP_F16) v = (sign << 15) | ((12u + e) << 10) | (b16 & mant_mask);   // bias 15
        else v = (sign << 15) | ((124u + e) << 7) | (b16 & mant_mask);                            // bias 127
        r |= v << (16 * i);
    }
    return r;
}

template <int OP>
__global__ void __launch_bounds__(256, 2) mfma_probe_kernel(float* sink, long long iters, int bits_a, int bits_b) {
    u32x4 a[4], b[4];
    const uint32_t id = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t wa[4], wb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t ha = mix32(id * 64u + i * 8u + j), hb = mix32(id * 64u + i * 8u + j + 4u);
            // constant operands: 0.5 everywhere (both formats have it: 0x3800 / 0x3f00)
            const uint32_t half = OP == OP_F16 ? 0x38003800u : 0x3f003f00u;
            wa[j] = bits_a > 0 ? random_pair<OP>(ha, bits_a) : half;
            wb[j] = bits_b > 0 ? random_pair<OP>(hb, bits_b) : half;
        }
        a[i] = mk4(wa[0], wa[1], wa[2], wa[3]);
        b[i] = mk4(wb[0], wb[1], wb[2], wb[3]);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (long long it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc[u & 3] = mfma32<OP>(a[u >> 2], b[u & 3], acc[u & 3]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[id] = s;
}

}  // namespace
}  // namespace dit

extern "C" dit_status dit_mfma_probe(int32_t operand_dtype, int32_t bits_a, int32_t bits_b, int64_t mfma_per_wavefront,
                                     float* sink, size_t sink_bytes, double* flops, void* stream) {
    if (!sink || !flops || mfma_per_wavefront < 1 || bits_a < 0 || bits_b < 0) return DIT_ERR_INVALID_ARG;
    if (operand_dtype != DIT_PROBE_BF16 && operand_dtype != DIT_PROBE_F16) return DIT_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(sink) & 3u) return DIT_ERR_ALIGNMENT;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return static_cast<dit_status>(dit::report_hip_error(e, "hipDeviceGetAttribute"));
    // two workgroups of four wavefronts per compute unit: two wavefronts on each of its four SIMDs
    const int blocks = 2 * cus;
    if (sink_bytes < (size_t)blocks * 256 * sizeof(float)) return DIT_ERR_WORKSPACE;
    const long long iters = (mfma_per_wavefront + dit::kProbeUnroll - 1) / dit::kProbeUnroll;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (operand_dtype == DIT_PROBE_F16)
        hipLaunchKernelGGL(dit::mfma_probe_kernel<dit::OP_F16>, dim3(blocks), dim3(256), 0, s, sink, iters, bits_a, bits_b);
    else
        hipLaunchKernelGGL(dit::mfma_probe_kernel<dit::OP_BF16>, dim3(blocks), dim3(256), 0, s, sink, iters, bits_a, bits_b);
    e = hipGetLastError();
    if (e != hipSuccess) return static_cast<dit_status>(dit::report_hip_error(e, "mfma_probe_kernel"));
    // 32x32x16 multiply-adds, two flops each
    *flops = (double)blocks * 4.0 * (double)iters * dit::kProbeUnroll * 32768.0;
    return DIT_OK;
}
