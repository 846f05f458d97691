// Internal definitions shared by the HIP translation units of libxconv.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/xconv.h"

namespace xc {

constexpr int kThreads = 256;  // every kernel runs 4 wavefronts of 64 lanes per workgroup
constexpr int kMaxGridZ = 65535;  // largest third extent of a grid: launches over more images go in pieces

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

enum KernelId {
    K_GEN_Z = 0,
    K_PROBE = 1,
    K_PROBE_GENERIC = 2,
    K_CORR = 3,
    K_REDUCE = 4,
    K_TO_NHWC = 5,
    K_UNPACK = 6,
    K_EXPAND = 7,
    K_REPACK = 8,
    K_PACK_Z = 9,
    K_ZERO_GAPS = 10,
    K_GEN_ZIMG = 11,
    K_SCALE = 12,
    K_PIXEL_FWD = 13,
    K_RELU = 14,
    K_CONV = 15,
    K_PASS2 = 16,
    K_DIAG = 17,
    K_COUNT = 18
};

// Where the probe output of a voxel goes in Xt.  sd == 0: plain order, pixel `first` of the
// input is pixel `first` of Xt.  Volumetric layers (sd = depth stride >= 1): Xt is sd runs of
// `run` depth slices; slice z of image `img` is slot (z + pd) / sd of the image's `period`
// slots in run (z + pd) % sd, so that kernel-depth offset kz pairs output slice oz with slot
// oz + kz / sd of run kz % sd.
struct SliceMap {
    int HWs, D, pd, sd, period;
    long long run;
    __host__ __device__ long long slice_of(long long img, int z) const
    {
        const int t = z + pd;
        return (long long)(t % sd) * run + img * period + t / sd;
    }
    // HW = D * HWs pixels per image
    __host__ __device__ long long out_pixel(long long first, int HW) const
    {
        if (sd == 0) return first;
        const long long img = first / HW;
        const int rem = (int)(first - img * HW);
        const int z = rem / HWs;
        return slice_of(img, z) * HWs + (rem - z * HWs);
    }
};

__host__ __device__ inline int round_up(int a, int b) { return (a + b - 1) / b * b; }
__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Layout of one fp32 tile of correlation sums (a K-split's partial tile, or the reduced tile): [K2][MP/4][JP][4].
// Four consecutive output channels of one (offset, column) are a 16-byte element, and the JP columns of such a
// channel quad are contiguous: the lanes of a matrix-instruction result (one column each, four rows per register
// group) store runs of 16-byte elements, and the second pass reads a quad's columns as one run.
__host__ __device__ inline size_t tile_index(int o, int j, int m, int JP, int MP)
{
    return ((((size_t)o * (size_t)(MP >> 2) + (size_t)(m >> 2)) * (size_t)JP + (size_t)j) << 2) + (size_t)(m & 3);
}

// ---- storage-type conversions (device) ------------------------------------
__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ inline uint16_t f32_to_f16_rne(float f)
{
    _Float16 h = (_Float16)f;  // v_cvt_f16_f32: round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}
__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ inline float f16_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

template <int DT> __device__ inline uint16_t f32_to_st16(float f)
{
    if constexpr (DT == XCONV_BF16) return f32_to_bf16_rne(f);
    else return f32_to_f16_rne(f);
}
template <int DT> __device__ inline float st16_to_f32(uint16_t h)
{
    if constexpr (DT == XCONV_BF16) return bf16_to_f32(h);
    else return f16_to_f32(h);
}

// 16x16x32 MFMA on eight 16-bit values per lane (passed as the raw 16 bytes).
template <int DT> __device__ inline f32x4 mfma16(const uint4 &a, const uint4 &b, f32x4 c)
{
    if constexpr (DT == XCONV_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// In-register transpose of an 8 (rows q) x 2*NW (16-bit columns) block held as
// rows[q][w] (two columns per 32-bit word) into per-column vectors: column t
// gets the eight row values packed in q order.
template <int NW> __device__ inline void transpose_rows8(const uint32_t (&rows)[8][NW], uint4 (&cols)[2 * NW])
{
    // One byte-permute per output word: v_perm_b32 picks its four bytes from the pair {second, first} operand
    // (selector values 0-3: bytes of the second operand, 4-7: bytes of the first).
    constexpr uint32_t kLow = 0x05040100u;    // low halves:  a.b0 a.b1 b.b0 b.b1
    constexpr uint32_t kHigh = 0x07060302u;   // high halves: a.b2 a.b3 b.b2 b.b3
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        // even column: low halves of each row pair; odd column: high halves
        cols[2 * w].x = __builtin_amdgcn_perm(rows[1][w], rows[0][w], kLow);
        cols[2 * w].y = __builtin_amdgcn_perm(rows[3][w], rows[2][w], kLow);
        cols[2 * w].z = __builtin_amdgcn_perm(rows[5][w], rows[4][w], kLow);
        cols[2 * w].w = __builtin_amdgcn_perm(rows[7][w], rows[6][w], kLow);
        cols[2 * w + 1].x = __builtin_amdgcn_perm(rows[1][w], rows[0][w], kHigh);
        cols[2 * w + 1].y = __builtin_amdgcn_perm(rows[3][w], rows[2][w], kHigh);
        cols[2 * w + 1].z = __builtin_amdgcn_perm(rows[5][w], rows[4][w], kHigh);
        cols[2 * w + 1].w = __builtin_amdgcn_perm(rows[7][w], rows[6][w], kHigh);
    }
}

// Quotient and remainder of small non-negative integers (n, d < 2^22) through one float
// multiplication and a correction step: a handful of instructions where the integer division
// of the instruction set takes some thirty.  rd = frcp(d).
__device__ inline float frcp(int d) { return __builtin_amdgcn_rcpf((float)d); }
__device__ inline void fast_divmod(int n, int d, float rd, int &q, int &r)
{
    q = (int)((float)n * rd);
    r = n - q * d;
    if (r < 0) {
        r += d;
        --q;
    } else if (r >= d) {
        r -= d;
        ++q;
    }
}

// ---------------------------------------------------------------------------
// Z[s]: SplitMix64 in counter form.  Word ctr of the stream of `seed` is
// fin(key + gamma*(ctr+1)) with key = fin(seed + gamma).
// ---------------------------------------------------------------------------
__host__ __device__ inline uint64_t mix_fin(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__host__ __device__ inline uint64_t stream_word(uint64_t key, uint64_t ctr)
{
    return mix_fin(key + 0x9E3779B97F4A7C15ull * (ctr + 1ull));
}
// `dist` carries the distribution in its low byte and, above it, keep_q15: 0 for dense probes,
// else entry idx is kept with probability keep_q15 / 32768 and zero otherwise (block-sparse
// probing vectors, Eq. (7)); the keep decision compares the top 15 bits of word idx of a
// second stream (seed xor kMaskStream), so kept entries equal those of the dense matrix.
constexpr uint64_t kMaskStream = 0x5851F42D4C957F2Dull;
struct ProbeGen {
    int dist, keep_q15;
    uint64_t key, mkey;
};
__host__ __device__ inline ProbeGen probe_gen(int dist, uint64_t seed)
{
    ProbeGen g;
    g.dist = dist & 0xff;
    g.keep_q15 = dist >> 8;
    g.key = mix_fin(seed + 0x9E3779B97F4A7C15ull);
    g.mkey = mix_fin((seed ^ kMaskStream) + 0x9E3779B97F4A7C15ull);
    return g;
}
// keep decision `block` of block-sparse probing vectors (Eq. (7)); always true for dense probes
__host__ __device__ inline bool probe_keep(const ProbeGen &g, uint64_t block)
{
    return g.keep_q15 == 0 || (int)(stream_word(g.mkey, block) >> 49) < g.keep_q15;
}
__host__ __device__ inline float probe_value(const ProbeGen &g, uint64_t idx);
// entry idx of Z; with block-sparse probes it is zero unless its own keep decision says keep
__host__ __device__ inline float probe_entry(const ProbeGen &g, uint64_t idx)
{
    return probe_keep(g, idx) ? probe_value(g, idx) : 0.0f;
}
__host__ __device__ inline float probe_value(const ProbeGen &g, uint64_t idx)
{
    // +-1: entry idx is bit idx % 64 of word idx / 64 (the bits of a SplitMix64 output are independent fair bits), so one
    // generator word serves 64 entries and a workgroup can draw a whole matrix from a few hundred words
    if (g.dist == XCONV_RADEMACHER) return ((stream_word(g.key, idx >> 6) >> (idx & 63)) & 1ull) ? -1.0f : 1.0f;
    // Box-Muller in double on two 53-bit uniforms, u1 in (0,1], u2 in [0,1)
    const double u1 = ((double)(stream_word(g.key, 2ull * idx) >> 11) + 1.0) * 0x1.0p-53;
    const double u2 = (double)(stream_word(g.key, 2ull * idx + 1ull) >> 11) * 0x1.0p-53;
    return (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2));
}

// ---- launch plan of the correlation kernel (host fills, kernel reads) ------
struct CorrParams {
    const void *dY;    // [B, C_out, Ho, Wo] storage dtype
    const void *A;     // channels-last activation-like tensor [B, H, W, CS] storage dtype (Xt, or X for the exact path)
    float *part;       // [S] partial tiles of fp32 sums, each in the layout of tile_index()
    int B, C_out, H, W, Ho, Wo;
    int kH, kW, sh, sw, ph, pw;
    int CS;            // channel stride of A (multiple of 16)
    int NBG;           // batch groups (BI images each)
    int RB, CW, CWp;   // output rows and columns per step; CWp = CW rounded up to 4
    int NSTRIP, NBAND; // steps per batch group = NSTRIP * NBAND
    int NR, NOLD, NNEW;  // rows of A per step: NR = (RB-1)*sh + kH; NOLD kept from the previous step, NNEW loaded
    int BWc;           // columns of A staged per row = (CWp-1)*sw + kW
    int WM, WJ, WK;    // wave arrangement inside a workgroup (product 4)
    int M_WG, J_WG;    // workgroup tile: output channels and probe columns
    int ASTR, BSTR;    // LDS strides (units) per pixel slot / per staged column
    int NCHR;          // vector chunks of dY staged per row and output channel
    int NTM, NTJ;      // tiles along C_out and along the probe columns
    int S, NS;         // K-splits and total steps
    int SQ, SR;        // NS / S and NS % S (set at launch): workgroup x takes SQ steps, one more if x < SR
    int K2, NOG;       // kernel offsets and offset groups of <= 9
    int MP, JP;        // padded extents of the partial buffer
    int dy_plane;      // elements between consecutive (image, channel) planes of dY as the kernel reads it (whole 16-byte vectors)
    int a_units, b_units;  // LDS units of the two staging tiles
    int AL;            // every staged row segment of dY starts on a 16-byte vector
    // Z[s] for the expansion that follows (Alg. 1 backward step 2): when zout is set, the launch's workgroups
    // each draw a slice of its nz entries from (zdist, zseed) before they start on the correlation
    float *zout;
    int nz, zdist;
    uint64_t zseed;
};


// ---- launch plan of the producer/consumer correlation kernel (16-bit storage) ----
struct WsParams {
    const void *dY;    // [B, C_out, Ho, Wo] storage dtype
    const void *A;     // channels-last [B, H, W, CS] storage dtype
    float *part;       // [S] partial tiles of fp32 sums, each in the layout of tile_index()
    int B, C_out, H, W, Ho, Wo;
    int kH, kW, sh, sw, ph, pw;
    int CS, NBG;            // channel stride of A; groups of 8 images
    int CW, NSTRIP;         // output columns per strip, strips per output row
    int CWs, NSUB;          // output columns per sub-step (multiple of 4), sub-steps per row-step
    int BWc, NRING;         // staged columns per ring row; ring rows (kH + sh)
    int WM, WJ, M_WG, J_WG, NTM, NTJ;
    int S, NS;              // K-splits, row-steps in total (NBG * NSTRIP * Ho)
    int SQ, SR;             // NS / S and NS % S (set at launch): workgroup x takes SQ row-steps, one more if x < SR
    int K2, NOG, MP, JP;
    int a_units;            // LDS units of one dY buffer (CWs * M_WG)
    int b_row_units, BSTR;  // LDS units per ring row, per staged column (J_WG + 1)
    int NA, NA_pad;         // dY tasks per sub-step and the same rounded up to whole waves
    int TS, TB;             // A tasks per sub-step slice, per row-step (sh * BWc * J_WG/8)
    int MT, NTASK;          // 16-row tiles per consumer wave; tasks per producer thread
    // Volumetric layers read dY [Bv, C_out, Do, Ho*Wo] in place: image i of the kernel's batch is depth
    // slot i % vol_period of volume i / vol_period, a zero image when the slot is >= vol_Do.  0: plain dY.
    int vol_period, vol_Do;
    uint32_t vol_bytes;     // bytes of the whole dY tensor (below 2^30)
    // Z[s] for the expansion that follows, drawn by this launch (see CorrParams)
    float *zout;
    int nz, zdist;
    uint64_t zseed;
};

// Entries wg*threads + tid, + (workgroups * threads), ... of Z[s], drawn by the calling thread (Alg. 1 backward
// step 2: the probing matrix is regenerated from the seed, never stored between the passes).
__device__ inline void draw_z_slice(float *zout, int nz, int dist, uint64_t seed)
{
    if (!zout) return;
    const int nwg = gridDim.x * gridDim.y * gridDim.z;
    const int wg = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const ProbeGen gen = probe_gen(dist, seed);
    for (int i = wg * (int)blockDim.x + (int)threadIdx.x; i < nz; i += nwg * (int)blockDim.x) zout[i] = probe_entry(gen, (uint64_t)i);
}

// Workgroups are handed to the chip's 8 dies in turn (workgroup b runs on die b % 8, each with an L2 of
// its own).  With a grid whose first extent is a multiple of 8 this gives the workgroups of one die neighbouring
// pieces of work (tiles of the probe, K-splits of the correlation: consecutive output rows of one group of images),
// so that a cache line which straddles two pieces (planes and rows are not line-aligned) is fetched from memory
// once, by one L2, instead of once by each of two.
__device__ inline int xcd_block(int b, int grid)
{
    return (grid & 7) == 0 ? (b & 7) * (grid >> 3) + (b >> 3) : b;
}

// ---- forward convolution / exact input gradient as one implicit GEMM (conv_kernels.hip) ----
struct ConvGemmParams {
    const void *in;    // activation-like tensor the contraction runs over (X, or dY for the input gradient)
    const void *w;     // weights [C_out, C_in, kH, kW] in the storage type
    void *out;         // Y, or dX
    int Cin, Cout;     // contraction channels and output channels of this product
    int Hi, Wi;        // extent of `in`
    int Ho, Wo;        // extent of `out`
    int kH, kW, sh, sw, ph, pw;
    int transposed;    // 0: src = (y*sh + ky - ph, x*sw + kx - pw); 1: src = ((y + ph - ky) / sh, ...) where that divides
    long long npix;    // B * Ho * Wo
    long long in_sb, out_sb;                              // element strides: image,
    int in_sc, in_sy, in_sx, out_sc, out_sy, out_sx;      // channel, row, column
    int w_sco, w_sci;                                     // weights: output channel of the product, contraction channel
};

}  // namespace xc
