// Forward product of the estimator with probing vectors over pixels and channels (Sec. 3 multi-channel
// case, Eq. (6) step (i); Algorithm 1 forward step 3):
//     Xbar[b, j] = sum_k Z[k, j] X[b, k],   k = (channel, pixel) over K = C_in * H * W values,
// a skinny product (r x B outputs, K terms each) that is bound by reading X once.  Both operands are
// K-contiguous (X row b; probing vector j as an image of K storage values), which is the order the
// matrix instructions want their reduction index in, so fragments go from global memory straight into
// the MFMA operands: rows = probing vectors, columns = images, a lane supplies 8 (16-bit) or 4 (fp32)
// consecutive k.  K is split over the workgroups; partial products go to scratch and are summed in a
// fixed order by reduce_partials_kernel.
#include <cstdlib>

#include "common.h"
#include "launch.h"

namespace xc {

namespace {

constexpr int kPfThreads = 256;

// Every wave is a worker of its own: TM column tiles of 16 images x TN row tiles of 16 probing vectors,
// one slice of the k range.  A stage is VPL consecutive 16-byte vectors per lane and tile (a lane group
// g reads VPL * 16 bytes in a row, so a row of X is read in bursts of 4 * VPL * 16 bytes); D stages of
// loads are in flight.  The k a lane supplies to an MFMA only has to be the same on both operands.
template <int DT, int TM, int TN>
__global__ __launch_bounds__(kPfThreads, 2) void pixel_fwd_kernel(const void *__restrict__ Xv, const void *__restrict__ Zv,
                                                              float *__restrict__ part, long long K, long long ld, int B,
                                                              int r_img, int CSt, int NM, int S, int nbb, int njb)
{
    constexpr int ES = DT == XCONV_F32 ? 4 : 2;
    constexpr int VE = 16 / ES;                          // k per vector
    constexpr int VPL = (TM + TN >= 5) ? 2 : 4;          // vectors per lane, tile and stage
    constexpr int D = (32 / (VPL * (TM + TN))) < 2 ? 2 : (32 / (VPL * (TM + TN)));
    constexpr int KM = 4 * VPL * VE;                     // k per stage ("macro step")
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    // worker -> (image block, k slice, probing vector block), image blocks fastest: the waves of a workgroup then read the
    // same slice of the probing vectors at about the same time, and all but the first find it in the caches of their
    // compute unit and die (C5: 49.2 -> 47.6 us against slices fastest)
    const long long w = (long long)blockIdx.x * 4 + wave;
    if (w >= (long long)S * nbb * njb) return;           // (no barrier in this kernel)
    const int bb = (int)(w % nbb);
    const int s = (int)((w / nbb) % S), jb = (int)(w / ((long long)S * nbb));
    const int b0 = bb * (16 * TM), j0 = jb * (16 * TN);
    const int q = NM / S, rem = NM % S;
    const int step0 = s * q + (s < rem ? s : rem);
    const int nstep = q + (s < rem ? 1 : 0);

    // blockIdx.y: independent probing, one product per input channel over its own K values of every row (rows are
    // `ld` values apart); a single product has ld = K and one grid row
    const char *X = static_cast<const char *>(Xv) + (size_t)blockIdx.y * (size_t)K * ES;
    const char *Z = static_cast<const char *>(Zv) + (size_t)blockIdx.y * (size_t)K * ES;
    part += (size_t)blockIdx.y * (size_t)S * B * CSt;
    // rows of this lane: image b0 + 16 tm + l16 and probing vector j0 + 16 tn + l16; past the end the
    // last one is read again and its products are not stored
    const char *xrow[TM];
    const char *zrow[TN];
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        int b = b0 + 16 * t + l16;
        b = b < B ? b : B - 1;
        xrow[t] = X + (size_t)b * (size_t)ld * ES;
    }
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        int j = j0 + 16 * t + l16;
        j = j < r_img ? j : r_img - 1;
        zrow[t] = Z + (size_t)j * (size_t)ld * ES;
    }

    f32x4 acc[TN][TM];   // [row tile of probing vectors][column tile of images]
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};

    struct Stage {
        uint4 x[TM][VPL], z[TN][VPL];
    };
    auto load = [&](Stage &sg, int step) {
        const long long kbase = (long long)step * KM + (long long)g * (VPL * VE);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            // K is a whole number of vectors: a vector is inside or outside
            const long long k = kbase + v * VE;
            const bool in = k < K;
            const size_t off = in ? (size_t)k * ES : 0;   // (past the end: a valid address, the value is dropped)
#pragma unroll
            for (int t = 0; t < TM; ++t) {
                const uint4 xv = *reinterpret_cast<const uint4 *>(xrow[t] + off);
                sg.x[t][v] = in ? xv : uint4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                const uint4 zv = *reinterpret_cast<const uint4 *>(zrow[t] + off);
                sg.z[t][v] = in ? zv : uint4{0u, 0u, 0u, 0u};
            }
        }
    };
    auto mma = [&](const Stage &sg) {
#pragma unroll
        for (int v = 0; v < VPL; ++v)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    if constexpr (DT == XCONV_F32) {
                        // MFMA u multiplies element u of both vectors
                        const float za[4] = {__uint_as_float(sg.z[tn][v].x), __uint_as_float(sg.z[tn][v].y),
                                             __uint_as_float(sg.z[tn][v].z), __uint_as_float(sg.z[tn][v].w)};
                        const float xa[4] = {__uint_as_float(sg.x[tm][v].x), __uint_as_float(sg.x[tm][v].y),
                                             __uint_as_float(sg.x[tm][v].z), __uint_as_float(sg.x[tm][v].w)};
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x4f32(za[u], xa[u], acc[tn][tm], 0, 0, 0);
                    } else {
                        acc[tn][tm] = mfma16<DT>(sg.z[tn][v], sg.x[tm][v], acc[tn][tm]);
                    }
                }
    };

    Stage ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < nstep) load(ring[d], step0 + d);
    int i = 0;
    for (; i + D <= nstep; i += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            mma(ring[d]);
            if (i + d + D < nstep) load(ring[d], step0 + i + d + D);
        }
    }
#pragma unroll
    for (int d = 0; d < D - 1; ++d)
        if (i + d < nstep) mma(ring[d]);

    // lane (l16, g) holds probing vectors 16 tn + 4 g .. + 3 of image 16 tm + l16: part[s][b][j..j+3]
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int b = b0 + 16 * tm + l16;
        if (b >= B) continue;
        float *dst = part + ((size_t)s * B + b) * CSt + j0 + 4 * g;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
            if (j0 + 16 * tn < CSt) *reinterpret_cast<f32x4 *>(dst + 16 * tn) = acc[tn][tm];
    }
}

// Xbar[b, j] = T[b, j] for j < r (T has rows of CSt >= r values)
__global__ __launch_bounds__(kPfThreads) void pixel_xbar_compact_kernel(const float *__restrict__ T, float *__restrict__ Xbar, int B,
                                                                        int CSt, int r)
{
    const int i = blockIdx.x * kPfThreads + threadIdx.x;
    if (i >= B * r) return;
    const int b = i / r, j = i - b * r;
    Xbar[i] = T[(size_t)b * CSt + j];
}

// Independent probing: Xbar[b, c, j] = T[c, b, j] for j < r (T has one [B, CSt] block per input channel)
__global__ __launch_bounds__(kPfThreads) void pixel_xbar_indep_kernel(const float *__restrict__ T, float *__restrict__ Xbar, int B,
                                                                      int C, int CSt, int r)
{
    const long long i = (long long)blockIdx.x * kPfThreads + threadIdx.x;
    if (i >= (long long)B * C * r) return;
    const int j = (int)(i % r);
    const long long bc = i / r;
    const int c = (int)(bc % C), b = (int)(bc / C);
    Xbar[i] = T[((size_t)c * B + b) * CSt + j];
}

}  // namespace

// The product takes X and the probing vectors as rows of K values each in whole 16-byte vectors.
bool pixel_fwd_ok(int dtype, long long K, const void *X)
{
    const int ve = dtype == XCONV_F32 ? 4 : 8;
    return K % ve == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0;
}

// Tiles per wave, k per stage and k slices of the launch
struct PixelFwdPlan {
    int TM, TN, KM, NM, S, nbb, njb;
};
static PixelFwdPlan pixel_fwd_plan(int dtype, long long K, int B, int r)
{
    PixelFwdPlan p;
    const int CSt = round_up(r, 16);
    p.TM = B > 32 ? 4 : (B > 16 ? 2 : 1);
    p.TN = CSt > 32 ? 4 : (CSt > 16 ? 2 : 1);
    if (const char *v = getenv("XCONV_PIXEL_TM")) {   // sweeps
        if (*v == '1' || *v == '2' || *v == '4') p.TM = *v - '0';
    }
    const int ve = dtype == XCONV_F32 ? 4 : 8;
    const int vpl = (p.TM + p.TN >= 5) ? 2 : 4;
    p.KM = 4 * vpl * ve;
    p.NM = (int)((K + p.KM - 1) / p.KM);
    p.nbb = ceil_div(B, 16 * p.TM);
    p.njb = ceil_div(CSt, 16 * p.TN);
    // four waves per compute unit over all (image block, probing vector block) pairs (a wave keeps 16 to 32 KB of
    // loads in flight), at least 4 stages per slice, partial sums below a sixth of the bytes of X; then a whole
    // number of waves per compute unit (an uneven spread costs a whole extra wave's time)
    const long long nb = (long long)p.nbb * p.njb;
    long long S = 1024 / nb;
    if (S > p.NM / 4) S = p.NM / 4;
    const long long cap = K * (dtype == XCONV_F32 ? 4 : 2) / ((long long)CSt * 4 * 6);
    if (S > cap) S = cap;
    if (S * nb > 256) S = (S * nb / 256) * 256 / nb;
    if (const char *v = getenv("XCONV_PIXEL_SPLITS")) {   // sweeps
        if (*v) S = atoi(v);
        if (S > p.NM) S = p.NM;
    }
    if (S < 1) S = 1;
    p.S = (int)S;
    return p;
}

// partial sums [S, B, CSt] and the reduced [B, CSt]
size_t pixel_fwd_partial_bytes(int dtype, long long K, int B, int r)
{
    return ((size_t)pixel_fwd_plan(dtype, K, B, r).S + 1) * B * round_up(r, 16) * sizeof(float);
}

template <int DT, int TM, int TN>
static void pixel_fwd_launch(const PixelFwdPlan &p, const void *X, const void *Zimg, float *part, long long K, long long ld,
                             int nprod, int B, int r, hipStream_t st)
{
    const long long workers = (long long)p.S * p.nbb * p.njb;
    hipLaunchKernelGGL((pixel_fwd_kernel<DT, TM, TN>), dim3((unsigned)((workers + 3) / 4), nprod), dim3(kPfThreads), 0, st, X, Zimg,
                       part, K, ld, B, r, round_up(r, 16), p.NM, p.S, p.nbb, p.njb);
}

template <int DT>
static void pixel_fwd_dt(const PixelFwdPlan &p, const void *X, const void *Zimg, float *part, long long K, long long ld, int nprod,
                         int B, int r, hipStream_t st)
{
#define XC_PF(TM_, TN_) \
    if (p.TM == TM_ && p.TN == TN_) return pixel_fwd_launch<DT, TM_, TN_>(p, X, Zimg, part, K, ld, nprod, B, r, st);
    XC_PF(1, 1) XC_PF(1, 2) XC_PF(1, 4) XC_PF(2, 1) XC_PF(2, 2) XC_PF(2, 4) XC_PF(4, 1) XC_PF(4, 2) XC_PF(4, 4)
#undef XC_PF
}

// Zimg: r images of K storage values (launch_gen_zimg, row order); part: pixel_fwd_partial_bytes() of scratch
hipError_t launch_pixel_fwd(int dtype, const void *X, const void *Zimg, float *part, float *Xbar, long long K, int B, int r,
                            hipStream_t st)
{
    const PixelFwdPlan p = pixel_fwd_plan(dtype, K, B, r);
    if (dtype == XCONV_F32) pixel_fwd_dt<XCONV_F32>(p, X, Zimg, part, K, K, 1, B, r, st);
    else if (dtype == XCONV_BF16) pixel_fwd_dt<XCONV_BF16>(p, X, Zimg, part, K, K, 1, B, r, st);
    else pixel_fwd_dt<XCONV_F16>(p, X, Zimg, part, K, K, 1, B, r, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int CSt = round_up(r, 16);
    // straight into Xbar when its rows need no compaction and it takes 16-byte stores
    const bool direct = r == CSt && (reinterpret_cast<uintptr_t>(Xbar) & 15u) == 0;
    float *T = direct ? Xbar : part + (size_t)p.S * B * CSt;
    e = launch_reduce_raw(part, T, p.S, B * CSt / 4, st);
    if (e != hipSuccess || direct) return e;
    hipLaunchKernelGGL(pixel_xbar_compact_kernel, dim3(ceil_div(B * r, kPfThreads)), dim3(kPfThreads), 0, st, T, Xbar, B, CSt, r);
    return hipGetLastError();
}

// Independent probing on NCHW rows: one product per input channel, Xbar[b, c, j] = sum_q X[b, c, q] Z[c*N + q, j], from the
// same r images of K = C*N values (the rows of channel c of Z are the probing vectors of channel c).  N values per
// channel in whole 16-byte vectors.  part: pixel_fwd_indep_partial_bytes() of scratch.
size_t pixel_fwd_indep_partial_bytes(int dtype, long long N, int C, int B, int r)
{
    return (size_t)C * ((size_t)pixel_fwd_plan(dtype, N, B, r).S + 1) * B * round_up(r, 16) * sizeof(float);
}

hipError_t launch_pixel_fwd_indep(int dtype, const void *X, const void *Zimg, float *part, float *Xbar, long long N, int C, int B,
                                  int r, hipStream_t st)
{
    const PixelFwdPlan p = pixel_fwd_plan(dtype, N, B, r);
    const long long K = N * C;
    if (dtype == XCONV_F32) pixel_fwd_dt<XCONV_F32>(p, X, Zimg, part, N, K, C, B, r, st);
    else if (dtype == XCONV_BF16) pixel_fwd_dt<XCONV_BF16>(p, X, Zimg, part, N, K, C, B, r, st);
    else pixel_fwd_dt<XCONV_F16>(p, X, Zimg, part, N, K, C, B, r, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int CSt = round_up(r, 16);
    float *T = part + (size_t)C * p.S * B * CSt;
    e = launch_reduce_raw(part, T, p.S, B * CSt / 4, st, C);
    if (e != hipSuccess) return e;
    const long long total = (long long)B * C * r;
    hipLaunchKernelGGL(pixel_xbar_indep_kernel, dim3((unsigned)((total + kPfThreads - 1) / kPfThreads)), dim3(kPfThreads), 0, st, T,
                       Xbar, B, C, CSt, r);
    return hipGetLastError();
}

}  // namespace xc
