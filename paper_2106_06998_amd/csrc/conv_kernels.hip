// Forward convolution and exact input gradient of the layer (Sec. 2: XConv leaves the forward pass and
// the backpropagation through the layer exact; Algorithm 1 forward step 1 and the gradient with respect
// to the input):
//
//   forward      Y[b,m,oy,ox]  = sum_{n,ky,kx} W[m,n,ky,kx] X[b,n, oy*sh+ky-ph, ox*sw+kx-pw]
//   input grad   dX[b,n,iy,ix] = sum_{m,ky,kx} W[m,n,ky,kx] dY[b,m,oy,ox],  oy*sh+ky-ph = iy, ox*sw+kx-pw = ix
//
// Both are the implicit GEMM  out[co, p] = sum_{(o, ci)} Wv[co, ci, o] * in[ci, src(p, o)]  over output
// pixels p = (b, y, x), kernel offsets o and contraction channels ci, with zero for a source pixel outside
// the tensor (or, for the input gradient, between the strides).  One kernel does both: the host hands it
// the strides of the three tensors and the rule for src.  A workgroup owns TM output channels x 64 output
// pixels; for every offset it walks the contraction channels in chunks that are staged through LDS in the
// operand form of the matrix instruction (16x16x16 with four consecutive channels per lane for 16-bit
// storage, 16x16x4 for fp32), sums in fp32 and rounds once to the storage type.  LDS use is small (a few KB)
// so that several workgroups share a compute unit and hide each other's staging.
#include "common.h"
#include "launch.h"

namespace xc {

namespace {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

template <int DT> struct ConvTraits;
template <> struct ConvTraits<XCONV_F32> {
    typedef float elem_t;
    typedef float unit_t;                // one channel per lane
    static constexpr int KP = 1, KC = 16;
};
template <> struct ConvTraits<XCONV_F16> {
    typedef uint16_t elem_t;
    typedef uint2 unit_t;                // four consecutive channels per lane
    static constexpr int KP = 4, KC = 32;
};
template <> struct ConvTraits<XCONV_BF16> {
    typedef uint16_t elem_t;
    typedef uint2 unit_t;
    static constexpr int KP = 4, KC = 32;
};

template <int DT> __device__ inline f32x4 conv_mfma(const typename ConvTraits<DT>::unit_t &a, const typename ConvTraits<DT>::unit_t &b, f32x4 c)
{
    if constexpr (DT == XCONV_F32) return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    else if constexpr (DT == XCONV_F16)
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
}

template <int DT> __device__ inline typename ConvTraits<DT>::unit_t conv_pack(const typename ConvTraits<DT>::elem_t (&v)[ConvTraits<DT>::KP])
{
    if constexpr (DT == XCONV_F32) return v[0];
    else return uint2{(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16)};
}

}  // namespace

// MT: 16-row tiles of output channels per wave (TM = 32 * MT output channels per workgroup)
template <int DT, int MT>
__global__ __launch_bounds__(kThreads) void conv_gemm_kernel(const ConvGemmParams P)
{
    typedef ConvTraits<DT> T;
    typedef typename T::elem_t elem_t;
    typedef typename T::unit_t unit_t;
    constexpr int KP = T::KP, KC = T::KC, NU = KC / KP;   // units (lane operands) per chunk along the contraction
    constexpr int TM = 32 * MT, TP = 64;
    constexpr int UPT = NU / 4;                           // units per staging thread and tile row
    constexpr int NAW = TM * KC / kThreads;               // weight elements per staging thread and chunk
    __shared__ unit_t As[NU][TM];
    __shared__ unit_t Bs[NU][TP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int wm = wave & 1, wp = wave >> 1;
    const int co0 = blockIdx.y * TM;
    const long long p0 = (long long)blockIdx.x * TP;
    const elem_t *in = static_cast<const elem_t *>(P.in);
    const elem_t *wv = static_cast<const elem_t *>(P.w);
    const int HoWo = P.Ho * P.Wo;
    const int K2 = P.kH * P.kW;
    const bool w_along_ci = P.w_sci < P.w_sco;

    // staging roles for `in`: pixel tid % 64, units kg, kg + 4, ...
    const int sl = tid & 63, kg = tid >> 6;
    const long long sp = p0 + sl;
    const bool p_ok = sp < P.npix;
    const long long spc = p_ok ? sp : 0;
    const int sb = (int)(spc / HoWo);
    const int srem = (int)(spc - (long long)sb * HoWo);
    const int soy = srem / P.Wo, sox = srem - soy * P.Wo;
    const elem_t *in_b = in + (size_t)sb * P.in_sb;

    f32x4 acc[MT][2];
#pragma unroll
    for (int tm = 0; tm < MT; ++tm)
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) acc[tm][tp] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- in[ci, src(p, o)] and Wv[co, ci, o] of step (o, c0) -> registers (zero beyond the tensors).  The lanes of a weight
    // load run along whichever of the two channel indices has the smaller stride in [C_out, C_in, kH, kW] (values 18 or 36
    // bytes apart for a 3x3 kernel: a few cache lines per instruction; along the other index it would be one line per lane).
    unit_t bu[UPT];
    elem_t aw[NAW];
    auto load_step = [&](int o, int c0) {
        const int ky = o / P.kW, kx = o - ky * P.kW;
        // source pixel of my staging pixel for this offset
        int sy, sx;
        bool ok = p_ok;
        if (P.transposed) {
            const int ty = soy + P.ph - ky, tx = sox + P.pw - kx;
            ok = ok && ty >= 0 && tx >= 0 && ty % P.sh == 0 && tx % P.sw == 0;
            sy = ty / P.sh;
            sx = tx / P.sw;
        } else {
            sy = soy * P.sh + ky - P.ph;
            sx = sox * P.sw + kx - P.pw;
        }
        ok = ok && (unsigned)sy < (unsigned)P.Hi && (unsigned)sx < (unsigned)P.Wi;
        const elem_t *src = in_b + (size_t)(ok ? sy : 0) * P.in_sy + (size_t)(ok ? sx : 0) * P.in_sx;
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = kg + 4 * i;
            elem_t v[KP];
#pragma unroll
            for (int e = 0; e < KP; ++e) {
                const int c = c0 + u * KP + e;
                v[e] = (ok && c < P.Cin) ? src[(size_t)c * P.in_sc] : elem_t(0);
            }
            bu[i] = conv_pack<DT>(v);
        }
#pragma unroll
        for (int i = 0; i < NAW; ++i) {
            const int idx = tid + kThreads * i;
            const int cl = w_along_ci ? idx % KC : idx / TM, col = w_along_ci ? idx / KC : idx % TM;
            const int c = c0 + cl, co = co0 + col;
            aw[i] = (co < P.Cout && c < P.Cin) ? wv[(size_t)co * P.w_sco + (size_t)c * P.w_sci + o] : elem_t(0);
        }
    };

    // Steps (offset, chunk of contraction channels) in turn: the loads of the next step are issued before the matrix
    // instructions of the current one, whose operands are in LDS by then.
    int o = 0, c0 = 0;
    load_step(0, 0);
    while (o < K2) {
        __syncthreads();   // the previous step's fragments have been read
#pragma unroll
        for (int i = 0; i < UPT; ++i) Bs[kg + 4 * i][sl] = bu[i];
#pragma unroll
        for (int i = 0; i < NAW; ++i) {
            const int idx = tid + kThreads * i;
            const int cl = w_along_ci ? idx % KC : idx / TM, col = w_along_ci ? idx / KC : idx % TM;
            reinterpret_cast<elem_t *>(&As[0][0])[((cl / KP) * TM + col) * KP + cl % KP] = aw[i];
        }
        __syncthreads();
        c0 += KC;
        if (c0 >= P.Cin) { c0 = 0; ++o; }
        if (o < K2) load_step(o, c0);
#pragma unroll
        for (int kk = 0; kk < NU / 4; ++kk) {
            unit_t a[MT], b[2];
#pragma unroll
            for (int tm = 0; tm < MT; ++tm) a[tm] = As[kk * 4 + g][wm * (16 * MT) + tm * 16 + l16];
#pragma unroll
            for (int tp = 0; tp < 2; ++tp) b[tp] = Bs[kk * 4 + g][wp * 32 + tp * 16 + l16];
#pragma unroll
            for (int tm = 0; tm < MT; ++tm)
#pragma unroll
                for (int tp = 0; tp < 2; ++tp) acc[tm][tp] = conv_mfma<DT>(a[tm], b[tp], acc[tm][tp]);
        }
    }

    // ---- D tile: lane (l16, g) holds output channels 4g .. 4g+3 of pixel l16; one rounding to the storage type
    elem_t *out = static_cast<elem_t *>(P.out);
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
        const long long p = p0 + wp * 32 + tp * 16 + l16;
        if (p >= P.npix) continue;
        const int b = (int)(p / HoWo);
        const int rem = (int)(p - (long long)b * HoWo);
        const int oy = rem / P.Wo, ox = rem - oy * P.Wo;
        elem_t *dst = out + (size_t)b * P.out_sb + (size_t)oy * P.out_sy + (size_t)ox * P.out_sx;
#pragma unroll
        for (int tm = 0; tm < MT; ++tm)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int co = co0 + wm * (16 * MT) + tm * 16 + 4 * g + v;
                if (co < P.Cout) {
                    if constexpr (DT == XCONV_F32) dst[(size_t)co * P.out_sc] = acc[tm][tp][v];
                    else dst[(size_t)co * P.out_sc] = f32_to_st16<DT>(acc[tm][tp][v]);
                }
            }
    }
}

template <int DT> static hipError_t launch_conv_dt(const ConvGemmParams &P, hipStream_t st)
{
    const long long tiles = (P.npix + 63) / 64;
    // tiles of 128, 64 or 32 output channels: the smallest that covers the channels with the fewest empty rows
    if (P.Cout > 64 && (P.Cout % 128 == 0 || P.Cout % 128 > 64)) {
        hipLaunchKernelGGL((conv_gemm_kernel<DT, 4>), dim3((unsigned)tiles, (unsigned)ceil_div(P.Cout, 128)), dim3(kThreads), 0, st, P);
    } else if (P.Cout > 32) {
        hipLaunchKernelGGL((conv_gemm_kernel<DT, 2>), dim3((unsigned)tiles, (unsigned)ceil_div(P.Cout, 64)), dim3(kThreads), 0, st, P);
    } else {
        hipLaunchKernelGGL((conv_gemm_kernel<DT, 1>), dim3((unsigned)tiles, (unsigned)ceil_div(P.Cout, 32)), dim3(kThreads), 0, st, P);
    }
    return hipGetLastError();
}

hipError_t launch_conv_gemm(int dtype, const ConvGemmParams &P, hipStream_t st)
{
    if (dtype == XCONV_F32) return launch_conv_dt<XCONV_F32>(P, st);
    if (dtype == XCONV_BF16) return launch_conv_dt<XCONV_BF16>(P, st);
    return launch_conv_dt<XCONV_F16>(P, st);
}

}  // namespace xc
