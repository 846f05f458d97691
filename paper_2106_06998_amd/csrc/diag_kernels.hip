// Matrix-instruction issue loop: what rate the matrix cores of this chip sustain at the clock it holds under
// them, as a reference next to the published peak that the roofline fractions are stated against.  Every wave
// keeps four independent 32x32 accumulators busy with operands that are neither zero nor constant (the power
// a multiply draws, and with it the clock, depends on the bits that toggle); two workgroups of four waves per
// compute unit, so each SIMD always has a second wave to issue from.
#include "common.h"
#include "launch.h"

namespace xc {

namespace {

typedef float f32x16d __attribute__((ext_vector_type(16)));

__device__ inline uint32_t diag_bits(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

}  // namespace

template <int DT>
__global__ __launch_bounds__(kThreads, 2) void mfma_rate_kernel(float *__restrict__ out, int iters)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    f32x16d acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    const uint32_t h = diag_bits((uint32_t)(blockIdx.x * kThreads + tid) + 1u);
    if constexpr (DT == XCONV_F32) {
        // magnitudes in [0.5, 1), random signs
        const float a = __uint_as_float(0x3f000000u | (h & 0x007fffffu) | ((h & 0x00800000u) << 8));
        const float b = __uint_as_float(0x3f000000u | ((h >> 9) & 0x007fffffu) | ((h & 1u) << 31));
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
        }
    } else {
        // eight 16-bit values per operand: exponent of 0.5 (fp16 0x3800, bf16 0x3f00), random mantissa and sign
        const uint32_t e16 = DT == XCONV_F16 ? 0x38003800u : 0x3f003f00u;
        const uint32_t m16 = DT == XCONV_F16 ? 0x83ff83ffu : 0x807f807fu;
        uint4 a, b;
        a.x = e16 | (diag_bits(h + 1) & m16); a.y = e16 | (diag_bits(h + 2) & m16);
        a.z = e16 | (diag_bits(h + 3) & m16); a.w = e16 | (diag_bits(h + 4) & m16);
        b.x = e16 | (diag_bits(h + 5) & m16); b.y = e16 | (diag_bits(h + 6) & m16);
        b.z = e16 | (diag_bits(h + 7) & m16); b.w = e16 | (diag_bits(h + 8) & m16);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (DT == XCONV_BF16)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc[i], 0, 0, 0);
                else
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc[i], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    // one value per wave keeps the loop alive
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d);
    if (lane == 0) out[blockIdx.x * (kThreads / 64) + wave] = s;
}

// floating-point operations of one launch
double mfma_rate_flops(int dtype, int iters)
{
    const double per_instr = dtype == XCONV_F32 ? 2.0 * 32 * 32 * 2 : 2.0 * 32 * 32 * 16;
    return (double)kMfmaRateGrid * (kThreads / 64) * (double)iters * 4.0 * per_instr;
}

hipError_t launch_mfma_rate(int dtype, float *out, int iters, hipStream_t st)
{
    if (dtype == XCONV_F32) hipLaunchKernelGGL(mfma_rate_kernel<XCONV_F32>, dim3(kMfmaRateGrid), dim3(kThreads), 0, st, out, iters);
    else if (dtype == XCONV_BF16) hipLaunchKernelGGL(mfma_rate_kernel<XCONV_BF16>, dim3(kMfmaRateGrid), dim3(kThreads), 0, st, out, iters);
    else hipLaunchKernelGGL(mfma_rate_kernel<XCONV_F16>, dim3(kMfmaRateGrid), dim3(kThreads), 0, st, out, iters);
    return hipGetLastError();
}

}  // namespace xc
