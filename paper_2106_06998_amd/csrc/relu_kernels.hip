// ReLU that keeps only the signs of its input for the backward pass (Sec. 5, "Overall effective memory savings":
// a ReLU used to rely on the next convolution to store its output; that convolution now stores the probe output
// only, so the ReLU keeps one bit per element instead).
//     forward   Y = max(X, 0), bit i%64 of 64-bit word i/64 = (X[i] > 0)
//     backward  dX[i] = bit ? dY[i] : 0
// Both are plain streaming kernels: a lane handles one 16-byte vector (4 fp32 or 8 16-bit values), the lanes that
// share a 64-bit mask word (16 or 8 neighbours) combine their bits with an OR over the group, and the group's first
// lane stores the word.
#include "common.h"
#include "launch.h"

namespace xc {

namespace {

template <int DT> struct Elems {
    static constexpr int V = DT == XCONV_F32 ? 4 : 8;   // values per 16-byte vector
};

template <int DT> __device__ inline float value_of(uint32_t bits, int half)
{
    if constexpr (DT == XCONV_F32) {
        (void)half;
        return __uint_as_float(bits);
    } else {
        return st16_to_f32<DT>(half ? (uint16_t)(bits >> 16) : (uint16_t)(bits & 0xffffu));
    }
}
// the sign bit that is stored, and whether max(x, 0) keeps x (a NaN is kept but has no positive sign)
__device__ inline bool positive(float x) { return x > 0.0f; }
__device__ inline bool kept(float x) { return !(x <= 0.0f); }

// one vector per lane; `nvec` whole vectors, then `tail` single values handled by the last lanes one by one
template <int DT>
__global__ __launch_bounds__(kThreads) void relu_sign_fwd_kernel(const uint4 *X, uint4 *Y, unsigned long long *__restrict__ words,
                                                                 long long n)   // Y may be X (in place)
{
    constexpr int V = Elems<DT>::V, G = 64 / V;          // lanes per mask word
    const long long vec = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long e0 = vec * V;
    unsigned long long mine = 0;
    if (e0 + V <= n) {
        const uint4 v = X[vec];
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t bits = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (DT == XCONV_F32) {
                const float x = value_of<DT>(w[q], 0);
                bits |= (positive(x) ? 1u : 0u) << q;
                w[q] = kept(x) ? w[q] : 0u;
            } else {
                const float x0 = value_of<DT>(w[q], 0), x1 = value_of<DT>(w[q], 1);
                bits |= ((positive(x0) ? 1u : 0u) | (positive(x1) ? 2u : 0u)) << (2 * q);
                w[q] = (kept(x0) ? (w[q] & 0xffffu) : 0u) | (kept(x1) ? (w[q] & 0xffff0000u) : 0u);
            }
        }
        Y[vec] = uint4{w[0], w[1], w[2], w[3]};
        mine = (unsigned long long)bits << (V * (threadIdx.x % G));
    } else if (e0 < n) {
        // ragged end: value by value
        uint32_t bits = 0;
        for (int q = 0; q < (int)(n - e0); ++q) {
            if constexpr (DT == XCONV_F32) {
                const float x = reinterpret_cast<const float *>(X)[e0 + q];
                reinterpret_cast<float *>(Y)[e0 + q] = kept(x) ? x : 0.0f;
                bits |= (positive(x) ? 1u : 0u) << q;
            } else {
                const uint16_t h = reinterpret_cast<const uint16_t *>(X)[e0 + q];
                const float x = st16_to_f32<DT>(h);
                reinterpret_cast<uint16_t *>(Y)[e0 + q] = kept(x) ? h : (uint16_t)0;
                bits |= (positive(x) ? 1u : 0u) << q;
            }
        }
        mine = (unsigned long long)bits << (V * (threadIdx.x % G));
    }
    // OR over the G lanes of a word (all 64 lanes take part; lanes past the end contribute zero)
#pragma unroll
    for (int d = 1; d < G; d <<= 1) mine |= __shfl_xor(mine, d, 64);
    const long long word = vec / G;
    if (threadIdx.x % G == 0 && word * 64 < n) words[word] = mine;
}

template <int DT>
__global__ __launch_bounds__(kThreads) void relu_sign_bwd_kernel(const uint4 *dY, const unsigned long long *__restrict__ words, uint4 *dX,
                                                                 long long n)   // dX may be dY (in place)
{
    constexpr int V = Elems<DT>::V, G = 64 / V;
    const long long vec = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long e0 = vec * V;
    if (e0 >= n) return;
    const uint32_t bits = (uint32_t)(words[vec / G] >> (V * (threadIdx.x % G)));
    if (e0 + V <= n) {
        const uint4 v = dY[vec];
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (DT == XCONV_F32) w[q] = ((bits >> q) & 1u) ? w[q] : 0u;
            else w[q] = (((bits >> (2 * q)) & 1u) ? (w[q] & 0xffffu) : 0u) | (((bits >> (2 * q + 1)) & 1u) ? (w[q] & 0xffff0000u) : 0u);
        }
        dX[vec] = uint4{w[0], w[1], w[2], w[3]};
    } else {
        for (int q = 0; q < (int)(n - e0); ++q) {
            const bool p = (bits >> q) & 1u;
            if constexpr (DT == XCONV_F32) {
                const float g = reinterpret_cast<const float *>(dY)[e0 + q];
                reinterpret_cast<float *>(dX)[e0 + q] = p ? g : 0.0f;
            } else {
                const uint16_t g = reinterpret_cast<const uint16_t *>(dY)[e0 + q];
                reinterpret_cast<uint16_t *>(dX)[e0 + q] = p ? g : (uint16_t)0;
            }
        }
    }
}

}  // namespace

hipError_t launch_relu_sign_fwd(int dtype, const void *X, void *Y, void *words, long long n, hipStream_t st)
{
    const int V = dtype == XCONV_F32 ? 4 : 8;
    const long long nvec = (n + V - 1) / V;
    const dim3 grid((unsigned)((nvec + kThreads - 1) / kThreads));
    const uint4 *x = static_cast<const uint4 *>(X);
    uint4 *y = static_cast<uint4 *>(Y);
    unsigned long long *w = static_cast<unsigned long long *>(words);
    if (dtype == XCONV_F32) hipLaunchKernelGGL(relu_sign_fwd_kernel<XCONV_F32>, grid, dim3(kThreads), 0, st, x, y, w, n);
    else if (dtype == XCONV_BF16) hipLaunchKernelGGL(relu_sign_fwd_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, x, y, w, n);
    else hipLaunchKernelGGL(relu_sign_fwd_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, x, y, w, n);
    return hipGetLastError();
}

hipError_t launch_relu_sign_bwd(int dtype, const void *dY, const void *words, void *dX, long long n, hipStream_t st)
{
    const int V = dtype == XCONV_F32 ? 4 : 8;
    const long long nvec = (n + V - 1) / V;
    const dim3 grid((unsigned)((nvec + kThreads - 1) / kThreads));
    const uint4 *g = static_cast<const uint4 *>(dY);
    uint4 *x = static_cast<uint4 *>(dX);
    const unsigned long long *w = static_cast<const unsigned long long *>(words);
    if (dtype == XCONV_F32) hipLaunchKernelGGL(relu_sign_bwd_kernel<XCONV_F32>, grid, dim3(kThreads), 0, st, g, w, x, n);
    else if (dtype == XCONV_BF16) hipLaunchKernelGGL(relu_sign_bwd_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, g, w, x, n);
    else hipLaunchKernelGGL(relu_sign_bwd_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, g, w, x, n);
    return hipGetLastError();
}

}  // namespace xc
