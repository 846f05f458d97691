// Host-side launch wrappers implemented next to their kernels.
#pragma once
#include "common.h"

namespace xc {

// probe_kernels.hip
void host_probe_matrix(int dist, uint64_t seed, int n, float *Z);
hipError_t launch_gen_z(float *Z, int n, int dist, uint64_t seed, hipStream_t st);
// nhwc: X is channels-last [B, H, W, C_in] instead of [B, C_in, H, W]
bool probe_fast_path_ok(int dtype, int C_in, int HW, bool nhwc);
// the 16-bit probe kernel draws this matrix from (dist, seed) itself, from one generator word per 64 entries
bool probe_draws_words(int C_in, int r, int dist);
size_t zpack_bytes(int dtype, int C_in, int r, bool z_exact16);
hipError_t launch_pack_z(int dtype, const float *Z, void *out, int C_in, int r, bool z_exact16, int dist, uint64_t seed,
                         bool nhwc, hipStream_t st, float zmul = 1.0f);
// sm: where the output goes in Xt (SliceMap{} = plain order; volumetric layers: depth slices in slot order)
// Z == nullptr and zpack == nullptr: every workgroup draws its fragments of Z from (dist, seed) itself
hipError_t launch_probe(int dtype, const void *X, const float *Z, const void *zpack, void *Xt, int B, int C_in, int HW, int r,
                        int CS, bool z_exact16, bool nhwc, SliceMap sm, int dist, uint64_t seed, hipStream_t st);
hipError_t launch_probe_generic(int dtype, const void *X, const float *Z, void *Xt, int B, int C_in, int HW, int r, int CS,
                                bool nhwc, SliceMap sm, hipStream_t st);
// volumetric layers: zero the slots of Xt without image data; X -> channels-last slices in slot order;
// stored probe output -> fp32 [B, r, D, HWs];
// dY [B, C, Do, n] -> slice-major planes [B*period, C, pitch] with zero slices Do..period-1 behind every image
hipError_t launch_zero_gap_slices(void *Xt, size_t slice_bytes, int B, SliceMap sm, hipStream_t st);
hipError_t launch_to_slices(int dtype, const void *X, void *out, int B, int C, int CS, SliceMap sm, hipStream_t st);
// channels-last volumes: X [B, D, HWs, C] -> slices in slot order; dY [B, Do, n, C] -> slice-major planes
hipError_t launch_x_slices_nhwc(int dtype, const void *X, void *out, int B, int C, int CS, SliceMap sm, hipStream_t st);
hipError_t launch_dy_slices_nhwc(int dtype, const void *src, void *dst, int B, int C, int Do, int period, int n, int pitch,
                                 hipStream_t st);
hipError_t launch_unpack_slices(int dtype, const void *Xt, float *out, int B, int r, int CS, SliceMap sm, hipStream_t st);
hipError_t launch_dy_slices(int dtype, const void *src, void *dst, int B, int C, int Do, int period, int n, int pitch, hipStream_t st);
// probing vectors over pixels and channels as `nimg` images of K storage values (entry (k, j) = word k*r + j; images >= r zero);
// cl_cs > 0: each image channels-last [pixel][cl_cs] (k = channel * pixels + pixel), zero columns C_in..cl_cs-1;
// indep != 0: nch*r vectors over the channel window [n0, n0+nch), vector nl*r + j = column j of Z on the rows of channel
// n0+nl, zero elsewhere (n0 = 0, nch = C_in: all channels); with cl_cs > 0 the channel slots are the window's channels
hipError_t launch_gen_zimg(int dtype, void *out, long long K, int r, int nimg, int dist, uint64_t seed, int C_in, int cl_cs,
                           int indep, int n0, int nch, hipStream_t st);
hipError_t launch_scale(const float *in, float *out, int n, float f, hipStream_t st);
hipError_t launch_scale_cols(const float *in, float *out, int rows, int ld, int c0, int ncol, float f, hipStream_t st);
hipError_t launch_scatter_channels(const float *part, float *dW, int C_out, int C_in, int K2, int n0, int nch, hipStream_t st);
// ReLU that keeps one sign bit per element (64-bit words, bit i%64 of word i/64); Y may be X, dX may be dY
hipError_t launch_relu_sign_fwd(int dtype, const void *X, void *Y, void *words, long long n, hipStream_t st);
hipError_t launch_relu_sign_bwd(int dtype, const void *dY, const void *words, void *dX, long long n, hipStream_t st);
// dW[:, n] *= r / (kept blocks of channel n), or 0 without any (block-sparse probes over pixels and channels, Eq. (8))
hipError_t launch_nnz_rescale(float *dW, int C_out, int C_in, int K2, int r, int dist, uint64_t seed, hipStream_t st);
hipError_t launch_unpack(int dtype, const void *Xt, float *out, int B, int HW, int r, int CS, hipStream_t st);
hipError_t launch_to_nhwc(int dtype, const void *X, void *out, int B, int C, int HW, int CS, hipStream_t st);
// channels-last [B, HW, C] -> planes [B, C, pitch], zero tail
hipError_t launch_to_nchw(int dtype, const void *src, void *out, int B, int C, int HW, int pitch, hipStream_t st);
// channels-last [npix, C] -> [npix, CS], zero columns C..CS-1
hipError_t launch_pad_channels(int dtype, const void *src, void *out, long long npix, int C, int CS, hipStream_t st);

// corr_kernels.hip
// Fills every field of P except the three pointers.  Q is the number of
// probe/activation columns that carry data (r, or C_in on the exact path), CS
// their padded stride.  Returns false when no launch shape fits the device.
bool plan_corr(CorrParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw,
               int CS, bool dy_aligned);
size_t corr_partial_bytes(const CorrParams &P);
size_t corr_lds_bytes(int dtype, const CorrParams &P);
hipError_t launch_corr(int dtype, const CorrParams &P, hipStream_t st);
hipError_t launch_repack_planes(int dtype, const void *src, void *dst, long long nplanes, int n, int pitch, hipStream_t st);
// T[o,j,m] = sum_s part[s,o,j,m]; T lives behind the S partial buffers.  Zout != nullptr: the same
// launch also draws Z[s] (nz = C_in * r entries) from (dist, seed) into Zout.
// T != nullptr: the reduced tile goes there instead.  nsets > 1: that many sets of S partial buffers, back to back
// from P.part on, are reduced into as many tiles from T on (volumetric layers: one set per kernel-depth offset).
hipError_t launch_reduce(const CorrParams &P, hipStream_t st, float *Zout = nullptr, int nz = 0, int dist = 0, uint64_t seed = 0,
                         float *T = nullptr, int nsets = 1);
hipError_t launch_reduce_raw(const float *part, float *T, int S, int E4, hipStream_t st, int nsets = 1);
// The second pass in one launch: fixed-order sum of the S partial tiles and the expansion by Z / r or, for the exact
// gradient, the transposed store, straight into dW [C_out, C_in, nsets*K2].  reduce_expand_fused says whether this launch applies (otherwise launch_reduce
// followed by launch_expand do the same in two).
bool reduce_expand_fused(const CorrParams &P, bool have_z, bool exact, int C_in, int r, int dist, int nsets = 1);
hipError_t launch_reduce_expand(const CorrParams &P, const float *Z, bool exact, float *dW, int C_in, int r, bool nnz_norm, int dist,
                                uint64_t seed, int nsets, hipStream_t st);
// dW[m,n,o] = (1/r) * sum_j Z[n,j] * T[o,j,m]   (Z != nullptr)
// dW[m,n,o] = T[o,n,m]                          (Z == nullptr, exact path)
// T != nullptr: K2 tiles [K2, JP, MP] are read from there (volumetric layers: kD * kH * kW offsets).
hipError_t launch_expand(const CorrParams &P, const float *Z, float *dW, int C_in, int r, hipStream_t st, bool nnz_norm = false,
                         const float *T = nullptr, int K2 = 0);


// corr_ws_kernels.hip: producer/consumer variant for 16-bit storage.  plan_corr_ws returns
// false when the layer does not fit it (the caller then uses plan_corr / launch_corr).
bool plan_corr_ws(WsParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw, int CS);
size_t corr_ws_lds_bytes(const WsParams &P);
hipError_t launch_corr_ws(int dtype, const WsParams &P, hipStream_t st);

// corr_row_kernels.hip: producer/consumer kernel for 16-bit storage, 3x3 kernels at unit stride and short output rows
// (a multiple of 4 columns, as many as the ring of staged rows leaves room for in LDS: 28 with 64 probe columns) that a workgroup sweeps whole; plan_corr_row returns false for everything else
bool plan_corr_row(WsParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw, int CS);
size_t corr_row_lds_bytes(const WsParams &P);
hipError_t launch_corr_row(int dtype, const WsParams &P, hipStream_t st);

// corr_ws32_kernels.hip: the producer/consumer kernel for fp32 storage (same plan structure)
bool plan_corr_ws32(WsParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw, int CS);
size_t corr_ws32_lds_bytes(const WsParams &P);
hipError_t launch_corr_ws32(const WsParams &P, hipStream_t st);

// conv_kernels.hip: forward convolution and exact input gradient (one implicit-GEMM kernel, see ConvGemmParams)
hipError_t launch_conv_gemm(int dtype, const ConvGemmParams &P, hipStream_t st);

// pixel_kernels.hip: Xbar[b, j] = sum_k X[b, k] Zimg[j, k] (forward product of the pixel x channel probes)
bool pixel_fwd_ok(int dtype, long long K, const void *X);
size_t pixel_fwd_partial_bytes(int dtype, long long K, int B, int r);
// independent probing on NCHW rows: one product per input channel over its N = H*W values (whole 16-byte vectors)
size_t pixel_fwd_indep_partial_bytes(int dtype, long long N, int C, int B, int r);
hipError_t launch_pixel_fwd_indep(int dtype, const void *X, const void *Zimg, float *part, float *Xbar, long long N, int C, int B,
                                  int r, hipStream_t st);
hipError_t launch_pixel_fwd(int dtype, const void *X, const void *Zimg, float *part, float *Xbar, long long K, int B, int r,
                            hipStream_t st);

// diag_kernels.hip: matrix-instruction issue loop (two workgroups per compute unit), one float per wave into `out`
constexpr int kMfmaRateGrid = 512;
double mfma_rate_flops(int dtype, int iters);
hipError_t launch_mfma_rate(int dtype, float *out, int iters, hipStream_t st);

}  // namespace xc
