// Probe-side kernels: regeneration of Z[s] from the seed, the forward channel
// probe Xt = Z^T X (Algorithm 1, forward step 3; Eq. (6) step (i) restricted to
// the channel axis), and the layout helpers around it.
//
// The probe is a skinny contraction: per image it is the product
//   Xt_b^T [r x HW] = Z^T [r x C_in] * X_b [C_in x HW],
// read C_in*HW, write r*HW, so it is bound by HBM bandwidth.  It still runs on
// the matrix cores: at 16-bit storage its arithmetic intensity is above what the
// vector ALUs deliver at HBM speed.  X is read straight from global memory into
// the MFMA B operand (pixels are the MFMA columns, so NCHW rows load coalesced),
// Z^T lives in LDS already arranged as A-operand fragments, and the rows of each
// 16-row MFMA tile are assigned to probe indices so that a lane ends up holding
// consecutive probe columns of one pixel, which makes the channels-last store a
// run of 16-byte vectors.
#include <type_traits>

#include "common.h"
#include "launch.h"

namespace xc {

// X is read once and never again: where a wave's piece of a channel plane is whole cache lines, its loads carry the
// non-temporal hint, so that the lines do not displace what the caches could keep.  Measured event-timed per probe
// launch: C4 34.2 -> 31.3 us, C3 20.8 -> 17.2, C2 13.4 -> 12.0.  Planes that are not whole lines (C5: 1568 bytes) share
// lines between neighbouring tiles, and a hinted line is fetched again by the neighbour (113-120 MB read instead of 104):
// there the hint made the kernel 1 us faster at first and, once the workgroups drew Z themselves and started less evenly,
// 1.3 us slower, so the 16-bit kernel loads such planes without it (`nt` = 0; the fp32 kernel always hints: a run-time
// choice cost it 0.5 us on C2 and C4).  The
// stores of Xt never carry it: the correlation reads them next (with the hint on the stores the correlation got slower);
// nor do the correlation's loads of dY, whose rows share cache lines with the rows of the next row-step (with the hint
// the C5 correlation took 69.7 instead of 62.9 us).
template <bool NT> __device__ inline uint4 load_x16(const void *p)
{
    if constexpr (NT) {
        typedef unsigned int u32x4nt __attribute__((ext_vector_type(4)));
        const u32x4nt v = __builtin_nontemporal_load(static_cast<const u32x4nt *>(p));
        return uint4{v.x, v.y, v.z, v.w};
    } else {
        return *static_cast<const uint4 *>(p);
    }
}
template <bool NT> __device__ inline uint2 load_x8(const void *p)
{
    if constexpr (NT) {
        typedef unsigned int u32x2nt __attribute__((ext_vector_type(2)));
        const u32x2nt v = __builtin_nontemporal_load(static_cast<const u32x2nt *>(p));
        return uint2{v.x, v.y};
    } else {
        return *static_cast<const uint2 *>(p);
    }
}
// whether the planes of an NCHW tensor (pitch bytes apart) are whole cache lines; channels-last rows always take the hint
static int probe_nt(bool nhwc, long long pitch_bytes) { return (nhwc || pitch_bytes % 128 == 0) ? 1 : 0; }

void host_probe_matrix(int dist, uint64_t seed, int n, float *Z)
{
    const ProbeGen g = probe_gen(dist, seed);
    for (int i = 0; i < n; ++i) Z[i] = probe_entry(g, (uint64_t)i);
}

__global__ __launch_bounds__(kThreads) void gen_z_kernel(float *__restrict__ Z, int n, int dist, uint64_t seed)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    Z[i] = probe_entry(probe_gen(dist, seed), (uint64_t)i);
}

// Tile number `it` (0, 1, ...) of wave w out of NW waves, or ntiles when the wave is done.  Every wave takes
// ntiles / NW tiles, and the remaining ones go to waves spread evenly over the grid (not to the first so many), so that every
// compute unit, which holds the same number of waves, moves the same number of bytes to within a tile.
__device__ inline int wave_tile(int w, int it, int NW, int ntiles)
{
    const int Q = ntiles / NW, R = ntiles - Q * NW;
    if (it < Q) return it * NW + w;
    if (it == Q) {
        const int a = (int)((long long)w * R / NW), b = (int)((long long)(w + 1) * R / NW);
        if (b > a) return Q * NW + a;
    }
    return ntiles;
}

// Row i of MFMA tile jt holds probe column j0 + jmap: lane group g = i/4 then
// owns the 4*JT consecutive columns g*4*JT .. (g+1)*4*JT-1 of the 16*JT block.
__device__ inline int jmap(int jt, int i, int JT) { return (i >> 2) * (4 * JT) + jt * 4 + (i & 3); }

// ---------------------------------------------------------------------------
// Z in MFMA A-operand order, written once per call so that every workgroup of the probe
// kernels fills its LDS copy with a straight vector copy.  Probe columns are handled in
// blocks of 64 (four 16-row tiles, fewer in the last block).  Z == nullptr draws the entries
// from the seed (Alg. 1 forward step 2).
//   fp32:   block bi at float offset bi*KQ4*4*64, entry (kq, jt, lane) = Z[4kq + lane/16][j],
//           KQ4 = channel quads rounded up to a multiple of 4, zero beyond C_in and r.
//   16-bit: block bi at uint4 offset bi*KK*4*64*(split ? 2 : 1), entry (kk, jt, lane) = the 8
//           channels 32kk + 8(lane/16) .. +7 of column j; with `split` the rounding residue
//           z - hi follows nfrag entries later.
// ---------------------------------------------------------------------------
// channel that lane group g of fragment kq stands for.  NCHW: 4kq + g.  Channels-last input: a
// lane loads 4 consecutive channels and MFMA u takes element u, so within a block of 16
// channels fragment u holds channel 4g + u.
__device__ inline int f32_frag_channel(int kq, int g, bool nhwc) { return nhwc ? 16 * (kq >> 2) + 4 * g + (kq & 3) : 4 * kq + g; }

__global__ __launch_bounds__(kThreads) void pack_z_f32_kernel(const float *__restrict__ Z, float *__restrict__ out, int C_in, int r,
                                                              int NTJ, int KQ4, int dist, uint64_t seed, int nhwc, float zmul)
{
    const int e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= KQ4 * NTJ * 64) return;
    const int l = e & 63, tj = (e >> 6) % NTJ, kq = (e >> 6) / NTJ;
    const int bi = tj >> 2, jt = tj & 3, JTb = (NTJ - 4 * bi) < 4 ? (NTJ - 4 * bi) : 4;
    const int c = f32_frag_channel(kq, l >> 4, nhwc != 0), j = 64 * bi + jmap(jt, l & 15, JTb);
    float z = 0.0f;
    if (c < C_in && j < r) {
        const size_t idx = (size_t)c * r + j;
        z = Z ? Z[idx] * zmul : probe_entry(probe_gen(dist, seed), (uint64_t)idx);
    }
    out[(size_t)bi * KQ4 * 4 * 64 + (kq * JTb + jt) * 64 + l] = z;
}

template <int DT>
__global__ __launch_bounds__(kThreads) void pack_z_16_kernel(const float *__restrict__ Z, uint4 *__restrict__ out, int C_in, int r,
                                                             int NTJ, int KK, int split, int dist, uint64_t seed, float zmul)
{
    const int e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= KK * NTJ * 64) return;
    const int l = e & 63, tj = (e >> 6) % NTJ, kk = (e >> 6) / NTJ;
    const int bi = tj >> 2, jt = tj & 3, JTb = (NTJ - 4 * bi) < 4 ? (NTJ - 4 * bi) : 4;
    const int j = 64 * bi + jmap(jt, l & 15, JTb);
    const ProbeGen gen = probe_gen(dist, seed);
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int q = 0; q < 8; q += 2) {
        float z[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int c = kk * 32 + 8 * (l >> 4) + q + u;
            z[u] = 0.0f;
            if (c < C_in && j < r) {
                const size_t idx = (size_t)c * r + j;
                z[u] = Z ? Z[idx] * zmul : probe_entry(gen, (uint64_t)idx);
            }
        }
        const uint16_t h0 = f32_to_st16<DT>(z[0]), h1 = f32_to_st16<DT>(z[1]);
        hi[q >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        const uint16_t w0 = f32_to_st16<DT>(z[0] - st16_to_f32<DT>(h0)), w1 = f32_to_st16<DT>(z[1] - st16_to_f32<DT>(h1));
        lo[q >> 1] = (uint32_t)w0 | ((uint32_t)w1 << 16);
    }
    const size_t nfrag = (size_t)KK * JTb * 64;
    const size_t at = (size_t)bi * KK * 4 * 64 * (split ? 2 : 1) + (kk * JTb + jt) * 64 + l;
    out[at] = uint4{hi[0], hi[1], hi[2], hi[3]};
    if (split) out[at + nfrag] = uint4{lo[0], lo[1], lo[2], lo[3]};
}

// ---------------------------------------------------------------------------
// fp32 probe.  v_mfma_f32_16x16x4_f32: A = Z^T tile (16 probe rows x 4
// channels), B = X tile (4 channels x 16 pixel columns).  Each lane loads four
// consecutive pixels (16 bytes) of one channel; MFMA t uses element t, so MFMA
// column n stands for pixel 4n+t of the wave's 64-pixel tile.
// ---------------------------------------------------------------------------
// NHWC: X is [pixels, C_in]; a lane then loads four consecutive channels (16 bytes) of one pixel,
// MFMA u uses element u of every lane (see f32_frag_channel), and the wave's tile is four
// sub-tiles of 16 pixels; `ngroups` is the number of pixels.
template <int JT, bool NHWC>
__global__ __launch_bounds__(kThreads, (JT == 1 ? 4 : 2)) void probe_f32_kernel(const float *__restrict__ X, const float *__restrict__ Z,
                                                             const float *__restrict__ zpack, float *__restrict__ Xt, int C_in,
                                                             int HW, int r, int CS, int j0, long long ngroups, int ntiles,
                                                             SliceMap sm, int dist, uint64_t seed)
{
    extern __shared__ float zs[];  // [KQ4][JT][64] A-operand fragments, zero beyond C_in
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int KQ4 = ((C_in + 15) >> 4) << 2;
    const int nfrag = KQ4 * JT * 64;
    auto stage_z = [&]() {
        if (zpack) {
            for (int e = tid; e < nfrag / 4; e += kThreads)
                reinterpret_cast<float4 *>(zs)[e] = reinterpret_cast<const float4 *>(zpack)[e];
        } else {
            for (int e = tid; e < nfrag; e += kThreads) {
                const int l = e & 63, jt = (e >> 6) % JT, kq = (e >> 6) / JT;
                const int c = f32_frag_channel(kq, l >> 4, NHWC);
                const int j = j0 + jmap(jt, l & 15, JT);
                // without a Z in memory the entries are drawn here (small seed-defined Z: no launch of their own)
                zs[e] = (c < C_in && j < r) ? (Z ? Z[(size_t)c * r + j] : probe_entry(probe_gen(dist, seed), (uint64_t)c * r + j)) : 0.0f;
            }
        }
    };

    constexpr int D = JT == 1 ? 3 : 4;  // groups of 16 channels a wave keeps in flight (16 registers each)
    constexpr int NP = NHWC ? 4 : 1;
    const int n = lane & 15, g = lane >> 4;
    const long long last_group = ngroups - 1;
    const int KK = (C_in + 15) >> 4;

    // pixel (or group of 4 pixels) of this lane; lanes past the end redo the last one and store nothing
    struct Tile {
        const float *xb[NP];
        long long first[NP];
        long long out[NP];  // pixel index in Xt
        bool valid[NP];
    };
    auto locate = [&](Tile &tl, int tile) {
        if constexpr (NHWC) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const long long pp = (long long)tile * 64 + 16 * t + n;
                tl.valid[t] = pp < ngroups;
                tl.first[t] = tl.valid[t] ? pp : last_group;
                tl.xb[t] = X + (size_t)tl.first[t] * C_in;
                tl.out[t] = sm.out_pixel(tl.first[t], HW);
            }
        } else {
            const long long pg_raw = (long long)tile * 16 + n;
            tl.valid[0] = pg_raw < ngroups;
            tl.first[0] = (tl.valid[0] ? pg_raw : last_group) * 4;
            const long long img = tl.first[0] / HW;
            tl.xb[0] = X + (size_t)img * C_in * HW + (int)(tl.first[0] % HW);
            tl.out[0] = sm.out_pixel(tl.first[0], HW);
        }
    };
    // Channels past the end re-read the last channels against zero fragment entries.
    struct Staged {
        float4 v[4];
    };
    auto load16 = [&](Staged &sg, const Tile &tl, int kk) {
        const int c0 = kk * 16;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (NHWC) {
                int c = c0 + 4 * g;
                c = c < C_in ? c : C_in - 4;
                sg.v[u] = __builtin_bit_cast(float4, load_x16<true>(tl.xb[u] + c));
            } else {
                int c = c0 + 4 * u + g;
                c = c < C_in ? c : C_in - 1;
                sg.v[u] = __builtin_bit_cast(float4, load_x16<true>(tl.xb[0] + (size_t)c * HW));
            }
        }
    };
    auto prefetch = [&](Staged (&rg)[D], const Tile &tl) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < KK) load16(rg[d], tl, d);
    };

    // The first tile's loads are in flight while the Z fragments are staged.
    const int wv = xcd_block(blockIdx.x, gridDim.x) * 4 + wave, NWV = gridDim.x * 4;
    int it = 0;
    int tile = wave_tile(wv, 0, NWV, ntiles);
    Tile cur;
    Staged rg[D];
    if (tile < ntiles) {
        locate(cur, tile);
        prefetch(rg, cur);
    }
    stage_z();
    __syncthreads();

    while (tile < ntiles) {
        f32x4 acc[JT][4];
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[jt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto process = [&](const Staged &sg, int kk) {
            const float4(&v)[4] = sg.v;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int kq = kk * 4 + u;
#pragma unroll
                for (int jt = 0; jt < JT; ++jt) {
                    const float a = zs[(kq * JT + jt) * 64 + lane];
                    if constexpr (NHWC) {
                        // fragment u multiplies element u of the four pixels' channel vectors
                        const float e0 = u == 0 ? v[0].x : u == 1 ? v[0].y : u == 2 ? v[0].z : v[0].w;
                        const float e1 = u == 0 ? v[1].x : u == 1 ? v[1].y : u == 2 ? v[1].z : v[1].w;
                        const float e2 = u == 0 ? v[2].x : u == 1 ? v[2].y : u == 2 ? v[2].z : v[2].w;
                        const float e3 = u == 0 ? v[3].x : u == 1 ? v[3].y : u == 2 ? v[3].z : v[3].w;
                        acc[jt][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, e0, acc[jt][0], 0, 0, 0);
                        acc[jt][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, e1, acc[jt][1], 0, 0, 0);
                        acc[jt][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, e2, acc[jt][2], 0, 0, 0);
                        acc[jt][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, e3, acc[jt][3], 0, 0, 0);
                    } else {
                        acc[jt][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, v[u].x, acc[jt][0], 0, 0, 0);
                        acc[jt][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, v[u].y, acc[jt][1], 0, 0, 0);
                        acc[jt][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, v[u].z, acc[jt][2], 0, 0, 0);
                        acc[jt][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, v[u].w, acc[jt][3], 0, 0, 0);
                    }
                }
            }
        };
        int kk = 0;
        for (; kk + D <= KK; kk += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                process(rg[d], kk + d);
                if (kk + d + D < KK) load16(rg[d], cur, kk + d + D);
            }
        }
#pragma unroll
        for (int d = 0; d < D - 1; ++d)
            if (kk + d < KK) process(rg[d], kk + d);

        // the next tile's first loads go out before this tile's stores
        const Tile done = cur;
        tile = wave_tile(wv, ++it, NWV, ntiles);
        if (tile < ntiles) {
            locate(cur, tile);
            prefetch(rg, cur);
        }
        // lane (n, g) holds rows 4g..4g+3 of every tile = probe columns j0 + g*4*JT + jt*4 + v
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (!done.valid[NHWC ? t : 0]) continue;
            float *out = Xt + (size_t)(NHWC ? done.out[NHWC ? t : 0] : done.out[0] + t) * CS + j0 + g * (4 * JT);
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) *reinterpret_cast<f32x4 *>(out + jt * 4) = acc[jt][t];
        }
    }
}

// ---------------------------------------------------------------------------
// 16-bit probe.  v_mfma_f32_16x16x32_{f16,bf16}: a lane supplies 8 consecutive
// k (channels) of one row/column.  In NCHW the 8 channels of a pixel are HW
// elements apart, so each lane loads PT consecutive pixels from 8 channel rows
// and transposes the 8 x PT block in registers; MFMA t then uses pixel t of
// every lane.  SPLIT: Z is not exactly representable in the storage type
// (Gaussian or user Z), so it is used as hi + lo (two MFMAs); +-1 needs one.
// ---------------------------------------------------------------------------
// NHWC: X is [pixels, C_in]; the 8 channels a lane supplies are then one 16-byte load, no
// transpose; the wave's tile is PT sub-tiles of 16 pixels and `ngroups` is the number of pixels.
template <int DT, int JT, int PT, bool SPLIT, bool NHWC>
__global__ __launch_bounds__(kThreads, 2) void probe_16_kernel(const uint16_t *__restrict__ X, const float *__restrict__ Z,
                                                            const uint4 *__restrict__ zpack, uint16_t *__restrict__ Xt, int C_in,
                                                            int HW, int r, int CS, int j0, long long ngroups, int ntiles,
                                                            SliceMap sm, int dist, uint64_t seed, int nword, int nt)
{
    extern __shared__ uint4 zf[];  // [SPLIT?2:1][KK][JT][64] A-operand fragments, then (nword > 0) the generator words of a +-1 matrix
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int KK = (C_in + 31) >> 5;
    const int nfrag = KK * JT * 64;
    auto stage_z = [&]() {
        if (zpack) {
            for (int e = tid; e < nfrag * (SPLIT ? 2 : 1); e += kThreads) zf[e] = zpack[e];
        } else if (nword > 0) {
            // dense +-1 matrix from the seed (Alg. 1 forward step 2): entry i is bit i % 64 of generator word i / 64, so the
            // workgroup draws the nword words once into LDS and every fragment entry is a bit of one of them
            const ProbeGen gen = probe_gen(dist, seed);
            uint64_t *words = reinterpret_cast<uint64_t *>(zf + nfrag * (SPLIT ? 2 : 1));
            for (int w = tid; w < nword; w += kThreads) words[w] = stream_word(gen.key, (uint64_t)w);
            __syncthreads();
            constexpr uint32_t one = DT == XCONV_F16 ? 0x3c00u : 0x3f80u;   // 1.0 in the storage type; the sign bit makes it -1.0
            // (the table holds at most 2^17 entries: 32-bit entry numbers; bit i % 64 of word i / 64 is bit i % 32 of the
            // 32-bit half i / 32 of the table)
            const uint32_t *half = reinterpret_cast<const uint32_t *>(words);
            for (int e = tid; e < nfrag; e += kThreads) {
                const int l = e & 63, jt = (e >> 6) % JT, kk = (e >> 6) / JT;
                const int j = j0 + jmap(jt, l & 15, JT);
                const int c0 = kk * 32 + 8 * (l >> 4);
                uint32_t i = (uint32_t)c0 * (uint32_t)r + (uint32_t)j;
                uint32_t h[8];
#pragma unroll
                for (int q = 0; q < 8; ++q, i += (uint32_t)r) {
                    const bool on = j < r && c0 + q < C_in;
                    const uint32_t bit = (half[on ? (i >> 5) : 0u] >> (i & 31u)) & 1u;
                    h[q] = on ? (one | (bit << 15)) : 0u;
                }
                zf[e] = uint4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                if constexpr (SPLIT) zf[nfrag + e] = uint4{0u, 0u, 0u, 0u};   // (+-1 is exact in 16 bits: no residue)
            }
        } else {
            // Z fragments: four entries (32 scalar loads) per thread in flight at a time
            for (int base = 0; base < nfrag; base += 4 * kThreads) {
                float z[4][8];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int e = base + k * kThreads + tid;
                    const int l = e & 63, jt = (e >> 6) % JT, kk = (e >> 6) / JT;
                    const int j = j0 + jmap(jt, l & 15, JT);
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const int c = kk * 32 + 8 * (l >> 4) + q;
                        z[k][q] = (e < nfrag && c < C_in && j < r)
                                      ? (Z ? Z[(size_t)c * r + j] : probe_entry(probe_gen(dist, seed), (uint64_t)c * r + j))
                                      : 0.0f;
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int e = base + k * kThreads + tid;
                    uint32_t hi[4], lo[4];
#pragma unroll
                    for (int q = 0; q < 8; q += 2) {
                        const uint16_t h0 = f32_to_st16<DT>(z[k][q]), h1 = f32_to_st16<DT>(z[k][q + 1]);
                        hi[q >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                        if constexpr (SPLIT) {
                            const uint16_t w0 = f32_to_st16<DT>(z[k][q] - st16_to_f32<DT>(h0));
                            const uint16_t w1 = f32_to_st16<DT>(z[k][q + 1] - st16_to_f32<DT>(h1));
                            lo[q >> 1] = (uint32_t)w0 | ((uint32_t)w1 << 16);
                        }
                    }
                    if (e < nfrag) {
                        zf[e] = uint4{hi[0], hi[1], hi[2], hi[3]};
                        if constexpr (SPLIT) zf[nfrag + e] = uint4{lo[0], lo[1], lo[2], lo[3]};
                    }
                }
            }
        }
    };

    constexpr int NW = PT / 2;
    // K-steps of loads a wave keeps in flight (16 or 32 registers each)
    constexpr int D = (!NHWC && PT == 8) ? 2 : 4;
    constexpr int NP = NHWC ? PT : 1;
    const int n = lane & 15, g = lane >> 4;
    const long long last_group = ngroups - 1;

    // pixel (NHWC) or group of PT pixels (NCHW) of this lane; lanes past the end redo the last one and store nothing
    struct Tile {
        const uint16_t *xb[NP];
        long long first[NP];
        long long out[NP];  // pixel index in Xt
        bool valid[NP];
    };
    auto locate = [&](Tile &tl, int tile) {
        if constexpr (NHWC) {
#pragma unroll
            for (int t = 0; t < PT; ++t) {
                const long long pp = (long long)tile * (16 * PT) + 16 * t + n;
                tl.valid[t] = pp < ngroups;
                tl.first[t] = tl.valid[t] ? pp : last_group;
                tl.xb[t] = X + (size_t)tl.first[t] * C_in;
                tl.out[t] = sm.out_pixel(tl.first[t], HW);
            }
        } else {
            const long long pg_raw = (long long)tile * 16 + n;
            tl.valid[0] = pg_raw < ngroups;
            tl.first[0] = (tl.valid[0] ? pg_raw : last_group) * PT;
            const long long img = tl.first[0] / HW;
            tl.xb[0] = X + (size_t)img * C_in * HW + (int)(tl.first[0] % HW);
            tl.out[0] = sm.out_pixel(tl.first[0], HW);
        }
    };
    // MFMA operands of one K-step: cols[t] = the 8 channels 32kk + 8g .. +7 of pixel t.
    // Channels past the end re-read the last channels, whose Z fragment entries are zero.
    struct Staged {
        uint32_t rows[NHWC ? 1 : 8][NHWC ? 1 : NW];  // NCHW: 8 channel rows of PT pixels
        uint4 cols[NHWC ? PT : 1];                   // NHWC: ready-made operands
    };
    auto load_step = [&](Staged &sg, const Tile &tl, int kk) {
        if constexpr (NHWC) {
            int c = kk * 32 + 8 * g;
            c = c < C_in ? c : C_in - 8;
#pragma unroll
            for (int t = 0; t < PT; ++t) sg.cols[t] = load_x16<true>(tl.xb[t] + c);
        } else {
            auto rows8 = [&](auto ntc) {
                constexpr bool NT = decltype(ntc)::value;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    int c = kk * 32 + 8 * g + q;
                    c = c < C_in ? c : C_in - 1;
                    if constexpr (PT == 8) {
                        const uint4 v = load_x16<NT>(tl.xb[0] + (size_t)c * HW);
                        sg.rows[q][0] = v.x; sg.rows[q][1] = v.y; sg.rows[q][2] = v.z; sg.rows[q][3] = v.w;
                    } else {
                        const uint2 v = load_x8<NT>(tl.xb[0] + (size_t)c * HW);
                        sg.rows[q][0] = v.x; sg.rows[q][1] = v.y;
                    }
                }
            };
            if (nt) rows8(std::true_type{});
            else rows8(std::false_type{});
        }
    };
    auto prefetch = [&](Staged (&rg)[D], const Tile &tl) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < KK) load_step(rg[d], tl, d);
    };

    // The first tile's loads are in flight while the Z fragments are staged.
    const int wv = xcd_block(blockIdx.x, gridDim.x) * 4 + wave, NWV = gridDim.x * 4;
    int it = 0;
    int tile = wave_tile(wv, 0, NWV, ntiles);
    Tile cur;
    Staged rg[D];
    if (tile < ntiles) {
        locate(cur, tile);
        prefetch(rg, cur);
    }
    stage_z();
    __syncthreads();

    while (tile < ntiles) {
        f32x4 acc[JT][PT];
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int t = 0; t < PT; ++t) acc[jt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto process = [&](const Staged &sg, int kk) {
            uint4 cols[PT];
            if constexpr (NHWC) {
#pragma unroll
                for (int t = 0; t < PT; ++t) cols[t] = sg.cols[t];
            } else {
                transpose_rows8<NW>(sg.rows, cols);
            }
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                const uint4 ah = zf[(kk * JT + jt) * 64 + lane];
#pragma unroll
                for (int t = 0; t < PT; ++t) acc[jt][t] = mfma16<DT>(ah, cols[t], acc[jt][t]);
                if constexpr (SPLIT) {
                    const uint4 al = zf[nfrag + (kk * JT + jt) * 64 + lane];
#pragma unroll
                    for (int t = 0; t < PT; ++t) acc[jt][t] = mfma16<DT>(al, cols[t], acc[jt][t]);
                }
            }
        };
        int kk = 0;
        for (; kk + D <= KK; kk += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                process(rg[d], kk + d);
                if (kk + d + D < KK) load_step(rg[d], cur, kk + d + D);
            }
        }
#pragma unroll
        for (int d = 0; d < D - 1; ++d)
            if (kk + d < KK) process(rg[d], kk + d);

        // the next tile's first loads go out before this tile's stores
        const Tile done = cur;
        tile = wave_tile(wv, ++it, NWV, ntiles);
        if (tile < ntiles) {
            locate(cur, tile);
            prefetch(rg, cur);
        }
        // lane (n, g) holds probe columns j0 + g*4*JT .. +4*JT-1 of pixel t: one run of 8*JT bytes
#pragma unroll
        for (int t = 0; t < PT; ++t) {
            if (!done.valid[NHWC ? t : 0]) continue;
            uint32_t w[2 * JT];
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                w[2 * jt] = (uint32_t)f32_to_st16<DT>(acc[jt][t][0]) | ((uint32_t)f32_to_st16<DT>(acc[jt][t][1]) << 16);
                w[2 * jt + 1] = (uint32_t)f32_to_st16<DT>(acc[jt][t][2]) | ((uint32_t)f32_to_st16<DT>(acc[jt][t][3]) << 16);
            }
            uint16_t *o = Xt + (size_t)(NHWC ? done.out[NHWC ? t : 0] : done.out[0] + t) * CS + j0 + g * (4 * JT);
            if constexpr (JT % 2 == 0) {
#pragma unroll
                for (int k = 0; k < JT / 2; ++k)
                    *reinterpret_cast<uint4 *>(o + 8 * k) = uint4{w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]};
            } else {
#pragma unroll
                for (int k = 0; k < JT; ++k) *reinterpret_cast<uint2 *>(o + 4 * k) = uint2{w[2 * k], w[2 * k + 1]};
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Any-shape probe on the vector ALUs (used when image planes are not a
// multiple of the vector width, so the MFMA path's aligned loads do not apply).
// One thread per (pixel, block of 16 probe columns).
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kThreads) void probe_generic_kernel(const void *__restrict__ Xv, const float *__restrict__ Z,
                                                                 void *__restrict__ Xtv, int C_in, int HW, int r, int CS,
                                                                 long long npix, int nhwc, SliceMap sm)
{
    const long long flat = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (flat >= npix) return;
    const int jb = blockIdx.y * 16;
    const int b = (int)(flat / HW), p = (int)(flat % HW);
    float acc[16];
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) acc[jj] = 0.f;
    for (int c = 0; c < C_in; ++c) {
        const size_t xi = nhwc ? (size_t)flat * C_in + c : ((size_t)b * C_in + c) * HW + p;
        float x;
        if constexpr (DT == XCONV_F32) x = static_cast<const float *>(Xv)[xi];
        else x = st16_to_f32<DT>(static_cast<const uint16_t *>(Xv)[xi]);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int j = jb + jj;
            const float z = (j < r) ? Z[(size_t)c * r + j] : 0.f;
            acc[jj] = fmaf(z, x, acc[jj]);
        }
    }
    const size_t oi = (size_t)sm.out_pixel(flat, HW) * CS + jb;
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
        if constexpr (DT == XCONV_F32) static_cast<float *>(Xtv)[oi + jj] = acc[jj];
        else static_cast<uint16_t *>(Xtv)[oi + jj] = f32_to_st16<DT>(acc[jj]);
    }
}

// Stored Xt [B, HW, CS] -> plain fp32 [B, r, HW] (test helper).
template <int DT>
__global__ __launch_bounds__(kThreads) void unpack_kernel(const void *__restrict__ Xtv, float *__restrict__ out, int HW, int r,
                                                          int CS, long long total)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int p = (int)(i % HW);
    const long long bj = i / HW;
    const int j = (int)(bj % r);
    const long long b = bj / r;
    const size_t src = ((size_t)b * HW + p) * CS + j;
    if constexpr (DT == XCONV_F32) out[i] = static_cast<const float *>(Xtv)[src];
    else out[i] = st16_to_f32<DT>(static_cast<const uint16_t *>(Xtv)[src]);
}

// X [B, C, HW] -> channels-last [B, HW, CS] with zero columns C..CS-1 (input of
// the correlation kernel on the exact-gradient path).  32x32 tiles through LDS.
template <typename T>
__global__ __launch_bounds__(kThreads) void to_nhwc_kernel(const T *__restrict__ X, T *__restrict__ out, int C, int HW, int CS, int z0)
{
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int p0 = blockIdx.x * 32, c0 = blockIdx.y * 32, b = z0 + blockIdx.z;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = c0 + ty + 8 * k, p = p0 + tx;
        tile[ty + 8 * k][tx] = (c < C && p < HW) ? X[((size_t)b * C + c) * HW + p] : T(0);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int p = p0 + ty + 8 * k, c = c0 + tx;
        if (p < HW && c < CS) out[((size_t)b * HW + p) * CS + c] = tile[tx][ty + 8 * k];
    }
}

// Channels-last [B, HW, C] -> planes [B, C, pitch] with a zero tail HW..pitch-1 (a channels-last
// dY in the plane form the correlation kernels read).  32x32 tiles through LDS.
template <typename T>
__global__ __launch_bounds__(kThreads) void to_nchw_kernel(const T *__restrict__ src, T *__restrict__ out, int C, int HW, int pitch, int z0)
{
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int p0 = blockIdx.x * 32, c0 = blockIdx.y * 32, b = z0 + blockIdx.z;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int p = p0 + ty + 8 * k, c = c0 + tx;
        tile[ty + 8 * k][tx] = (c < C && p < HW) ? src[((size_t)b * HW + p) * C + c] : T(0);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = c0 + ty + 8 * k, p = p0 + tx;
        if (c < C && p < pitch) out[((size_t)b * C + c) * pitch + p] = tile[tx][ty + 8 * k];
    }
}

// The same for C a multiple of the 16-byte vector (VE = 8 or 4 elements), without LDS: a thread
// loads VE pixels x VE channels (one vector per pixel), transposes the block in registers and
// stores one vector of VE pixels per channel.  Lanes run over 8 channel vectors (128 contiguous
// bytes of a pixel on the way in) and 8 pixel blocks (128 contiguous bytes of a plane on the way
// out).  Planes whose pitch is not a multiple of VE are stored element by element.
template <typename T>
__global__ __launch_bounds__(kThreads) void to_nchw_vec_kernel(const T *__restrict__ src, T *__restrict__ out, int C, int HW,
                                                               int pitch, int z0)
{
    constexpr int VE = 16 / sizeof(T);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cx = lane & 7, pb = lane >> 3;
    const int c = blockIdx.y * (8 * VE) + cx * VE;
    const int p0 = (blockIdx.x * 4 + wave) * (8 * VE) + pb * VE;
    const int b = z0 + blockIdx.z;
    if (c >= C || p0 >= pitch) return;
    uint32_t rows[VE][4];
#pragma unroll
    for (int q = 0; q < VE; ++q) {
        uint4 v = uint4{0u, 0u, 0u, 0u};
        if (p0 + q < HW) v = *reinterpret_cast<const uint4 *>(src + ((size_t)b * HW + p0 + q) * C + c);
        rows[q][0] = v.x; rows[q][1] = v.y; rows[q][2] = v.z; rows[q][3] = v.w;
    }
    uint4 cols[VE];
    if constexpr (VE == 8) {
        transpose_rows8<4>(rows, cols);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) cols[e] = uint4{rows[0][e], rows[1][e], rows[2][e], rows[3][e]};
    }
    const bool vec = (pitch % VE) == 0;  // then p0 + VE <= pitch and every plane starts on a vector
#pragma unroll
    for (int e = 0; e < VE; ++e) {
        T *dst = out + ((size_t)b * C + c + e) * pitch + p0;
        if (vec) {
            *reinterpret_cast<uint4 *>(dst) = cols[e];
        } else {
            const T *vals = reinterpret_cast<const T *>(&cols[e]);
#pragma unroll
            for (int q = 0; q < VE; ++q)
                if (p0 + q < pitch) dst[q] = vals[q];
        }
    }
}

// Channels-last [npix, C] -> [npix, CS] with zero columns C..CS-1.
template <typename T>
__global__ __launch_bounds__(kThreads) void pad_channels_kernel(const T *__restrict__ src, T *__restrict__ out, int C, int CS,
                                                                long long total)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const long long pix = i / CS;
    const int c = (int)(i - pix * CS);
    out[i] = c < C ? src[pix * C + c] : T(0);
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
hipError_t launch_gen_z(float *Z, int n, int dist, uint64_t seed, hipStream_t st)
{
    hipLaunchKernelGGL(gen_z_kernel, dim3(ceil_div(n, kThreads)), dim3(kThreads), 0, st, Z, n, dist, seed);
    return hipGetLastError();
}

template <typename K> static hipError_t set_lds(K kernel, size_t bytes)
{
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// 4 tiles (one per wave) per workgroup pass.  The grid is what is resident at once (256 compute
// units x `wgs_per_cu`), or fewer workgroups when there are fewer tiles; wave_tile hands the tiles out so that every
// compute unit gets the same number to within one.  A multiple of 8 (see xcd_block).
static int probe_grid(int ntiles, int wgs_per_cu)
{
    const int want = round_up(ceil_div(ntiles, 4), 8);
    const int slots = 256 * wgs_per_cu;
    return want < slots ? want : slots;
}

template <int JT, bool NHWC>
static hipError_t launch_probe_f32_jt(const float *X, const float *Z, const float *zpack, float *Xt, int C_in, int HW, int r, int CS,
                                      int j0, long long npix, SliceMap sm, int dist, uint64_t seed, hipStream_t st)
{
    // a lane owns 4 consecutive pixels of a plane (NCHW) or one pixel of each of 4 sub-tiles (NHWC)
    const long long ngroups = NHWC ? npix : npix / 4;
    const int ntiles = (int)(NHWC ? (npix + 63) / 64 : (ngroups + 15) / 16);
    const size_t lds = (size_t)ceil_div(C_in, 16) * 4 * JT * 64 * sizeof(float);
    hipError_t e = set_lds(probe_f32_kernel<JT, NHWC>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((probe_f32_kernel<JT, NHWC>), dim3(probe_grid(ntiles, JT == 1 ? 4 : 2)), dim3(kThreads), lds, st, X, Z, zpack, Xt, C_in, HW, r,
                       CS, j0, ngroups, ntiles, sm, dist, seed);
    return hipGetLastError();
}

template <int DT, int JT, int PT, bool SPLIT, bool NHWC>
static hipError_t launch_probe_16_cfg(const uint16_t *X, const float *Z, const uint4 *zpack, uint16_t *Xt, int C_in, int HW, int r,
                                      int CS, int j0, long long npix, SliceMap sm, int dist, uint64_t seed, hipStream_t st)
{
    const long long ngroups = NHWC ? npix : npix / PT;
    const int ntiles = (int)(NHWC ? (npix + 16 * PT - 1) / (16 * PT) : (ngroups + 15) / 16);
    // a dense +-1 matrix that comes from the seed and has no fragments in scratch is drawn by the workgroups from its generator words
    const int nword = (!Z && !zpack && probe_draws_words(C_in, r, dist)) ? (int)(((long long)C_in * r + 63) / 64) : 0;
    const size_t lds = (size_t)(SPLIT ? 2 : 1) * ceil_div(C_in, 32) * JT * 64 * sizeof(uint4) + (size_t)round_up(nword, 2) * 8;
    hipError_t e = set_lds(probe_16_kernel<DT, JT, PT, SPLIT, NHWC>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((probe_16_kernel<DT, JT, PT, SPLIT, NHWC>), dim3(probe_grid(ntiles, 2)), dim3(kThreads), lds, st, X, Z, zpack,
                       Xt, C_in, HW, r, CS, j0, ngroups, ntiles, sm, dist, seed, nword, probe_nt(NHWC, 2LL * (sm.sd ? sm.HWs : HW)));
    return hipGetLastError();
}

template <int DT, int JT>
static hipError_t launch_probe_16_jt(const uint16_t *X, const float *Z, const uint4 *zpack, uint16_t *Xt, int C_in, int HW, int r,
                                     int CS, int j0, long long npix, bool split, bool nhwc, SliceMap sm, int dist, uint64_t seed, hipStream_t st)
{
    if (nhwc) {
        if (split) return launch_probe_16_cfg<DT, JT, 4, true, true>(X, Z, zpack, Xt, C_in, HW, r, CS, j0, npix, sm, dist, seed, st);
        return launch_probe_16_cfg<DT, JT, 4, false, true>(X, Z, zpack, Xt, C_in, HW, r, CS, j0, npix, sm, dist, seed, st);
    }
    // 8 pixels per lane when the accumulators stay small, 4 for wide probe blocks
    if constexpr (JT <= 2) {
        if ((sm.sd ? sm.HWs : HW) % 8 == 0) {
            if (split) return launch_probe_16_cfg<DT, JT, 8, true, false>(X, Z, zpack, Xt, C_in, HW, r, CS, j0, npix, sm, dist, seed, st);
            return launch_probe_16_cfg<DT, JT, 8, false, false>(X, Z, zpack, Xt, C_in, HW, r, CS, j0, npix, sm, dist, seed, st);
        }
    }
    if (split) return launch_probe_16_cfg<DT, JT, 4, true, false>(X, Z, zpack, Xt, C_in, HW, r, CS, j0, npix, sm, dist, seed, st);
    return launch_probe_16_cfg<DT, JT, 4, false, false>(X, Z, zpack, Xt, C_in, HW, r, CS, j0, npix, sm, dist, seed, st);
}

// Dense +-1 matrices whose generator words (one per 64 entries) fit 16 KB of LDS next to the fragments: the 16-bit probe
// kernel draws them itself, whatever their size, and no fragment launch is needed.
bool probe_draws_words(int C_in, int r, int dist)
{
    return (dist & 0xff) == XCONV_RADEMACHER && (dist >> 8) == 0 && ((long long)C_in * r + 63) / 64 <= 2048;
}

bool probe_fast_path_ok(int dtype, int C_in, int HW, bool nhwc)
{
    // aligned vector loads: 4 pixels (16 bytes fp32, 8 bytes 16-bit) per channel row, or (NHWC)
    // 16 bytes of consecutive channels per pixel; LDS for the Z fragments (worst case JT = 4,
    // split) must fit
    if (nhwc ? (C_in % (dtype == XCONV_F32 ? 4 : 8) != 0) : (HW % 4 != 0)) return false;
    const size_t lds = dtype == XCONV_F32 ? (size_t)ceil_div(C_in, 16) * 4 * 4 * 64 * 4 : (size_t)2 * ceil_div(C_in, 32) * 4 * 64 * 16;
    return lds <= 128 * 1024;
}

// Bytes of Z in fragment order (pack_z_*_kernel) for all column blocks.
size_t zpack_bytes(int dtype, int C_in, int r, bool z_exact16)
{
    const size_t ntj = (size_t)ceil_div(r, 16);
    if (dtype == XCONV_F32) return (size_t)ceil_div(C_in, 16) * 4 * ntj * 64 * sizeof(float);
    return (size_t)(z_exact16 ? 1 : 2) * ceil_div(C_in, 32) * ntj * 64 * sizeof(uint4);
}

// zmul: factor on the entries of a given Z (1 leaves them as they are)
hipError_t launch_pack_z(int dtype, const float *Z, void *out, int C_in, int r, bool z_exact16, int dist, uint64_t seed,
                         bool nhwc, hipStream_t st, float zmul)
{
    const int ntj = ceil_div(r, 16);
    if (dtype == XCONV_F32) {
        const int KQ4 = ceil_div(C_in, 16) * 4;
        hipLaunchKernelGGL(pack_z_f32_kernel, dim3(ceil_div(KQ4 * ntj * 64, kThreads)), dim3(kThreads), 0, st, Z,
                           static_cast<float *>(out), C_in, r, ntj, KQ4, dist, seed, nhwc ? 1 : 0, zmul);
    } else {
        const int KK = ceil_div(C_in, 32);
        const dim3 grid(ceil_div(KK * ntj * 64, kThreads));
        if (dtype == XCONV_BF16)
            hipLaunchKernelGGL(pack_z_16_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, Z, static_cast<uint4 *>(out), C_in, r, ntj,
                               KK, z_exact16 ? 0 : 1, dist, seed, zmul);
        else
            hipLaunchKernelGGL(pack_z_16_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, Z, static_cast<uint4 *>(out), C_in, r, ntj,
                               KK, z_exact16 ? 0 : 1, dist, seed, zmul);
    }
    return hipGetLastError();
}

// zpack: Z in fragment order (launch_pack_z) or nullptr, in which case every workgroup gathers
// its fragments from Z itself.
hipError_t launch_probe(int dtype, const void *X, const float *Z, const void *zpack, void *Xt, int B, int C_in, int HW, int r,
                        int CS, bool z_exact16, bool nhwc, SliceMap sm, int dist, uint64_t seed, hipStream_t st)
{
    const long long npix = (long long)B * HW;
    const int ntj = CS / 16;
    hipError_t e = hipSuccess;
    for (int t0 = 0; t0 < ntj && e == hipSuccess; t0 += 4) {
        const int jt = (ntj - t0) < 4 ? (ntj - t0) : 4;
        const int j0 = t0 * 16;
        const size_t bi = (size_t)(t0 / 4);
        if (dtype == XCONV_F32) {
            const float *x = static_cast<const float *>(X);
            float *o = static_cast<float *>(Xt);
            const float *zp = zpack ? static_cast<const float *>(zpack) + bi * ceil_div(C_in, 16) * 4 * 4 * 64 : nullptr;
#define XC_P32(NH)                                                                                  \
    switch (jt) {                                                                                   \
    case 1: e = launch_probe_f32_jt<1, NH>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, sm, dist, seed, st); break;      \
    case 2: e = launch_probe_f32_jt<2, NH>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, sm, dist, seed, st); break;      \
    case 3: e = launch_probe_f32_jt<3, NH>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, sm, dist, seed, st); break;      \
    default: e = launch_probe_f32_jt<4, NH>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, sm, dist, seed, st); break;     \
    }
            if (nhwc) { XC_P32(true) } else { XC_P32(false) }
#undef XC_P32
        } else {
            const uint16_t *x = static_cast<const uint16_t *>(X);
            uint16_t *o = static_cast<uint16_t *>(Xt);
            const bool split = !z_exact16;
            const uint4 *zp = zpack ? static_cast<const uint4 *>(zpack) + bi * ceil_div(C_in, 32) * 4 * 64 * (split ? 2 : 1) : nullptr;
#define XC_P16(DT)                                                                                            \
    switch (jt) {                                                                                             \
    case 1: e = launch_probe_16_jt<DT, 1>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, split, nhwc, sm, dist, seed, st); break;          \
    case 2: e = launch_probe_16_jt<DT, 2>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, split, nhwc, sm, dist, seed, st); break;          \
    case 3: e = launch_probe_16_jt<DT, 3>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, split, nhwc, sm, dist, seed, st); break;          \
    default: e = launch_probe_16_jt<DT, 4>(x, Z, zp, o, C_in, HW, r, CS, j0, npix, split, nhwc, sm, dist, seed, st); break;         \
    }
            if (dtype == XCONV_BF16) { XC_P16(XCONV_BF16) } else { XC_P16(XCONV_F16) }
#undef XC_P16
        }
    }
    return e;
}

hipError_t launch_probe_generic(int dtype, const void *X, const float *Z, void *Xt, int B, int C_in, int HW, int r, int CS,
                                bool nhwc, SliceMap sm, hipStream_t st)
{
    const long long npix = (long long)B * HW;
    dim3 grid((unsigned)((npix + kThreads - 1) / kThreads), CS / 16);
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(probe_generic_kernel<XCONV_F32>, grid, dim3(kThreads), 0, st, X, Z, Xt, C_in, HW, r, CS, npix, nhwc ? 1 : 0, sm);
    else if (dtype == XCONV_BF16)
        hipLaunchKernelGGL(probe_generic_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, X, Z, Xt, C_in, HW, r, CS, npix, nhwc ? 1 : 0, sm);
    else
        hipLaunchKernelGGL(probe_generic_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, X, Z, Xt, C_in, HW, r, CS, npix, nhwc ? 1 : 0, sm);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Volumetric layers (3-D convolution) run the 2-D kernels on depth slices: Xt (in the order of
// the slice map, see SliceMap) and a copy of dY are laid out as runs of slices with the same
// number of slots per image, so that the slice a kernel-depth offset pairs with an output slice
// is always a constant number of slots away and is a zero slice whenever it falls outside the
// image.
// ---------------------------------------------------------------------------
// Zeroes the slices of Xt that hold no image data (slots of the slice map without a depth
// slice of the image behind them, and the `run - B * period` slices at the end of every run).
// `slice16` = 16-byte vectors per slice.
__global__ __launch_bounds__(kThreads) void zero_gap_slices_kernel(uint4 *__restrict__ Xt, long long slice16, int B, SliceMap sm,
                                                                   long long total16)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total16) return;
    const long long s = i / slice16;
    const int rho = (int)(s / sm.run);
    const long long w = s - (long long)rho * sm.run;
    bool data = false;
    if (w < (long long)B * sm.period) {
        const int q = (int)(w % sm.period);
        const int z = q * sm.sd + rho - sm.pd;
        data = z >= 0 && z < sm.D;
    }
    if (!data) Xt[i] = uint4{0u, 0u, 0u, 0u};
}

hipError_t launch_zero_gap_slices(void *Xt, size_t slice_bytes, int B, SliceMap sm, hipStream_t st)
{
    const long long slice16 = (long long)(slice_bytes / 16);
    const long long total16 = (long long)sm.sd * sm.run * slice16;
    hipLaunchKernelGGL(zero_gap_slices_kernel, dim3((unsigned)((total16 + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                       static_cast<uint4 *>(Xt), slice16, B, sm, total16);
    return hipGetLastError();
}

// X [B, C, D, HWs] -> channels-last depth slices [slot][HWs][CS] in the slice map's order, zero
// columns C..CS-1 (the exact gradient of a volumetric layer reads X like a stored probe
// output).  32x32 tiles through LDS; z0 + blockIdx.z = image * D + z.
template <typename T>
__global__ __launch_bounds__(kThreads) void to_slices_kernel(const T *__restrict__ X, T *__restrict__ out, int C, int CS, SliceMap sm,
                                                             int z0)
{
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int p0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const int b = (z0 + blockIdx.z) / sm.D, z = (z0 + blockIdx.z) % sm.D;
    const int HWs = sm.HWs;
    const T *src = X + ((size_t)b * C * sm.D + z) * HWs;
    T *dst = out + (size_t)sm.slice_of(b, z) * HWs * CS;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = c0 + ty + 8 * k, p = p0 + tx;
        tile[ty + 8 * k][tx] = (c < C && p < HWs) ? src[(size_t)c * sm.D * HWs + p] : T(0);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int p = p0 + ty + 8 * k, c = c0 + tx;
        if (p < HWs && c < CS) dst[(size_t)p * CS + c] = tile[tx][ty + 8 * k];
    }
}

hipError_t launch_to_slices(int dtype, const void *X, void *out, int B, int C, int CS, SliceMap sm, hipStream_t st)
{
    const long long nz = (long long)B * sm.D;
    for (long long z0 = 0; z0 < nz; z0 += kMaxGridZ) {   // a grid's third extent is 16 bits
        dim3 grid(ceil_div(sm.HWs, 32), ceil_div(CS, 32), (unsigned)(nz - z0 < kMaxGridZ ? nz - z0 : kMaxGridZ));
        if (dtype == XCONV_F32)
            hipLaunchKernelGGL(to_slices_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(X),
                               static_cast<float *>(out), C, CS, sm, (int)z0);
        else
            hipLaunchKernelGGL(to_slices_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(X),
                               static_cast<uint16_t *>(out), C, CS, sm, (int)z0);
    }
    return hipGetLastError();
}

// Channels-last volumes.  X [B, D, HWs, C] -> the same voxels as depth slices [slot][HWs][CS] in the slice map's
// order with zero columns C..CS-1 (one thread per element of the output).
template <typename T>
__global__ __launch_bounds__(kThreads) void x_slices_nhwc_kernel(const T *__restrict__ X, T *__restrict__ out, int C, int CS, SliceMap sm,
                                                                 long long total)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % CS);
    long long t = i / CS;
    const int p = (int)(t % sm.HWs);
    t /= sm.HWs;
    const int z = (int)(t % sm.D);
    const long long b = t / sm.D;
    const T v = c < C ? X[(((size_t)b * sm.D + z) * sm.HWs + p) * C + c] : T(0);
    out[((size_t)sm.slice_of(b, z) * sm.HWs + p) * CS + c] = v;
}

hipError_t launch_x_slices_nhwc(int dtype, const void *X, void *out, int B, int C, int CS, SliceMap sm, hipStream_t st)
{
    const long long total = (long long)B * sm.D * sm.HWs * CS;
    dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(x_slices_nhwc_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(X),
                           static_cast<float *>(out), C, CS, sm, total);
    else
        hipLaunchKernelGGL(x_slices_nhwc_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(X),
                           static_cast<uint16_t *>(out), C, CS, sm, total);
    return hipGetLastError();
}

// dY [B, Do, n, C] (channels-last) -> slice-major planes [B*period, C, pitch], zero tails and zero slots
// Do..period-1 behind every image.  32x32 tiles through LDS; z0 + blockIdx.z = image * period + slot.
template <typename T>
__global__ __launch_bounds__(kThreads) void dy_slices_nhwc_kernel(const T *__restrict__ src, T *__restrict__ dst, int C, int Do,
                                                                  int period, int n, int pitch, int z0)
{
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int p0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const int slot = z0 + blockIdx.z;
    const int b = slot / period, z = slot % period;
    const bool real = z < Do;
    const T *s = src + ((size_t)b * Do + (real ? z : 0)) * n * C;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int p = p0 + ty + 8 * k, c = c0 + tx;
        tile[ty + 8 * k][tx] = (real && p < n && c < C) ? s[(size_t)p * C + c] : T(0);
    }
    __syncthreads();
    T *d = dst + (size_t)slot * C * pitch;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = c0 + ty + 8 * k, p = p0 + tx;
        if (c < C && p < pitch) d[(size_t)c * pitch + p] = tile[tx][ty + 8 * k];
    }
}

hipError_t launch_dy_slices_nhwc(int dtype, const void *src, void *dst, int B, int C, int Do, int period, int n, int pitch,
                                 hipStream_t st)
{
    const long long nz = (long long)B * period;
    for (long long z0 = 0; z0 < nz; z0 += kMaxGridZ) {
        dim3 grid(ceil_div(pitch, 32), ceil_div(C, 32), (unsigned)(nz - z0 < kMaxGridZ ? nz - z0 : kMaxGridZ));
        if (dtype == XCONV_F32)
            hipLaunchKernelGGL(dy_slices_nhwc_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(src),
                               static_cast<float *>(dst), C, Do, period, n, pitch, (int)z0);
        else
            hipLaunchKernelGGL(dy_slices_nhwc_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                               static_cast<uint16_t *>(dst), C, Do, period, n, pitch, (int)z0);
    }
    return hipGetLastError();
}

// Test helper: the stored probe output of a volumetric layer as plain fp32 [B, r, D, HWs].
template <int DT>
__global__ __launch_bounds__(kThreads) void unpack_slices_kernel(const void *__restrict__ Xtv, float *__restrict__ out, int r, int CS,
                                                                 SliceMap sm, long long total)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int p = (int)(i % sm.HWs);
    long long t = i / sm.HWs;
    const int z = (int)(t % sm.D);
    t /= sm.D;
    const int j = (int)(t % r);
    const long long b = t / r;
    const size_t at = ((size_t)sm.slice_of(b, z) * sm.HWs + p) * CS + j;
    if constexpr (DT == XCONV_F32) out[i] = static_cast<const float *>(Xtv)[at];
    else out[i] = st16_to_f32<DT>(static_cast<const uint16_t *>(Xtv)[at]);
}

hipError_t launch_unpack_slices(int dtype, const void *Xt, float *out, int B, int r, int CS, SliceMap sm, hipStream_t st)
{
    const long long total = (long long)B * r * sm.D * sm.HWs;
    dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(unpack_slices_kernel<XCONV_F32>, grid, dim3(kThreads), 0, st, Xt, out, r, CS, sm, total);
    else if (dtype == XCONV_BF16)
        hipLaunchKernelGGL(unpack_slices_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, Xt, out, r, CS, sm, total);
    else
        hipLaunchKernelGGL(unpack_slices_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, Xt, out, r, CS, sm, total);
    return hipGetLastError();
}

// dY [B, C, Do, n] (planes of n = H'*W' values) -> [B*period, C, pitch]: slice-major planes of
// `pitch` >= n elements with zero tails; slices Do..period-1 of every image are zero.
template <typename T>
__global__ __launch_bounds__(kThreads) void dy_slices_kernel(const T *__restrict__ src, T *__restrict__ dst, int C, int Do, int period,
                                                             int n, int pitch, long long total)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int e = (int)(i % pitch);
    const long long pl = i / pitch;
    const int c = (int)(pl % C);
    const long long sl = pl / C;
    const int z = (int)(sl % period);
    const long long b = sl / period;
    dst[i] = (z < Do && e < n) ? src[(((size_t)b * C + c) * Do + z) * n + e] : T{};
}

hipError_t launch_dy_slices(int dtype, const void *src, void *dst, int B, int C, int Do, int period, int n, int pitch, hipStream_t st)
{
    const int es = dtype == XCONV_F32 ? 4 : 2;
    const int vec = 16 / es;
    if (n % vec == 0 && pitch % vec == 0 && (reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
        // whole 16-byte vectors: the same index arithmetic once per vector
        const long long total = (long long)B * period * C * (pitch / vec);
        hipLaunchKernelGGL(dy_slices_kernel<uint4>, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                           static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), C, Do, period, n / vec, pitch / vec, total);
        return hipGetLastError();
    }
    const long long total = (long long)B * period * C * pitch;
    dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(dy_slices_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(src),
                           static_cast<float *>(dst), C, Do, period, n, pitch, total);
    else
        hipLaunchKernelGGL(dy_slices_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                           static_cast<uint16_t *>(dst), C, Do, period, n, pitch, total);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Probing vectors over the stacked pixel x channel axis (Eq. (6) as stated): Z is [K, r] with
// K = C_in * H * W rows, entry (k, j) = generator word k * r + j.  It is laid out as `nimg`
// images of K values in the storage type, image j = probing vector j (images r..nimg-1 are
// zero), which is the form the probe and correlation kernels read an activation in.
// ---------------------------------------------------------------------------
// Block-sparse probes (Eq. (7)): block (n, j), the pixels of channel n in vector j, is zero unless keep decision
// n * r + j of the generator says keep.
// cl_cs == 0: image j holds its K values in row order (k fastest).  cl_cs > 0: channels-last,
// value (n, q) of image j at (j * N + q) * cl_cs + n with zero columns C_in..cl_cs-1 (N = K / C_in
// pixels), the form the correlation kernels read an activation in.
// indep != 0: independent probing over the channel window [n0, n0 + nch): nch * r images; image nl * r + j is probing
// vector j of channel n0 + nl, the values of column j of Z on the rows of that channel and zero on every other channel.
// With cl_cs > 0 the cl_cs channel slots of an image are the channels of the window (slot = channel - n0).
template <int DT>
__global__ __launch_bounds__(kThreads) void gen_zimg_kernel(void *__restrict__ out, long long K, int r, int nimg, int dist,
                                                            uint64_t seed, int C_in, int cl_cs, int indep, int n0, int nch)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long N = K / C_in;
    const int ncol = indep ? nch * r : r;
    float z = 0.0f;
    int j;
    long long k, nl;   // nl: channel relative to the window
    if (cl_cs == 0) {
        if (i >= K * nimg) return;
        j = (int)(i / K);
        k = i - (long long)j * K;
        nl = k / N - n0;
    } else {
        if (i >= N * nimg * cl_cs) return;
        nl = i % cl_cs;
        const long long jq = i / cl_cs;
        j = (int)(jq / N);
        k = (n0 + nl) * N + (jq - (long long)j * N);
    }
    if (j < ncol && nl >= 0 && nl < nch) {
        const ProbeGen gen = probe_gen(dist, seed);
        const long long n = n0 + nl;
        if (indep) {
            if (j / r == nl) z = probe_value(gen, (uint64_t)k * (uint64_t)r + (uint64_t)(j % r));
        } else if (probe_keep(gen, (uint64_t)n * (uint64_t)r + (uint64_t)j)) {
            z = probe_value(gen, (uint64_t)k * (uint64_t)r + (uint64_t)j);
        }
    }
    if constexpr (DT == XCONV_F32) static_cast<float *>(out)[i] = z;
    else static_cast<uint16_t *>(out)[i] = f32_to_st16<DT>(z);
}

// The same images for dense +-1 vectors over all channels (indep == 0, n0 == 0), where entry i of Z is bit i % 64 of
// generator word i / 64: a thread owns 8 consecutive values of an image (16 bytes of 16-bit storage; rows of Z that are
// r entries apart) and walks the images j0 .. j0 + nj - 1, in which the entries of a row are consecutive bits, so that it
// draws a word only when a row's bit position crosses into the next one: C5 8 + 8 words for 128 values where the kernel
// above draws one per value.  LINE = 8 consecutive k (cl_cs == 0; K a multiple of 8) or the 8 channel slots 8s .. 8s + 7 of
// one pixel (cl_cs > 0, a multiple of 8; slots from C_in on are zero).
template <int DT>
__global__ __launch_bounds__(kThreads) void gen_zimg_pm1_kernel(void *__restrict__ out, long long K, int r, int nimg, uint64_t seed,
                                                                int C_in, int cl_cs, int nj)
{
    const long long N = K / C_in;
    const long long t = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long nline = cl_cs == 0 ? K / 8 : N * (cl_cs / 8);
    if (t >= nline) return;
    const int j0 = blockIdx.y * nj;
    const ProbeGen gen = probe_gen(XCONV_RADEMACHER, seed);
    uint64_t row[8];    // entry number of (k_q, 0), or ~0 for a slot without a channel
    long long pix = 0;
    int slot0 = 0;
    if (cl_cs == 0) {
#pragma unroll
        for (int q = 0; q < 8; ++q) row[q] = (uint64_t)(8 * t + q) * (uint64_t)r;
    } else {
        const int spp = cl_cs / 8;
        pix = t / spp;
        slot0 = (int)(t - pix * spp) * 8;
#pragma unroll
        for (int q = 0; q < 8; ++q) row[q] = slot0 + q < C_in ? (uint64_t)((long long)(slot0 + q) * N + pix) * (uint64_t)r : ~0ull;
    }
    uint64_t word[8], have[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { have[q] = ~0ull; word[q] = 0; }
    constexpr uint32_t one16 = DT == XCONV_F16 ? 0x3c00u : 0x3f80u;
    for (int j = j0; j < j0 + nj && j < nimg; ++j) {
        uint32_t v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            v[q] = 0u;
            if (j < r && row[q] != ~0ull) {
                const uint64_t i = row[q] + (uint64_t)j;
                if ((i >> 6) != have[q]) { have[q] = i >> 6; word[q] = stream_word(gen.key, have[q]); }
                const uint32_t bit = (uint32_t)(word[q] >> (i & 63)) & 1u;
                v[q] = DT == XCONV_F32 ? (0x3f800000u | (bit << 31)) : (one16 | (bit << 15));
            }
        }
        const long long at = cl_cs == 0 ? (long long)j * K + 8 * t : ((long long)j * N + pix) * cl_cs + slot0;
        if constexpr (DT == XCONV_F32) {
            uint4 *o = reinterpret_cast<uint4 *>(static_cast<float *>(out) + at);
            o[0] = uint4{v[0], v[1], v[2], v[3]};
            o[1] = uint4{v[4], v[5], v[6], v[7]};
        } else {
            *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(out) + at) =
                uint4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
        }
    }
}

// n0, nch: channel window of the images (0, C_in for all channels); with cl_cs > 0 an image has cl_cs channel slots
// for the channels n0 .. n0 + nch - 1 and N = K / C_in pixels
hipError_t launch_gen_zimg(int dtype, void *out, long long K, int r, int nimg, int dist, uint64_t seed, int C_in, int cl_cs,
                           int indep, int n0, int nch, hipStream_t st)
{
    // dense +-1 vectors over all channels, whole 16-byte lines: one generator word per 64 entries
    if ((dist & 0xff) == XCONV_RADEMACHER && (dist >> 8) == 0 && !indep && n0 == 0 && nch == C_in &&
        (cl_cs == 0 ? K % 8 == 0 : cl_cs % 8 == 0) && (reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
        const long long nline = cl_cs == 0 ? K / 8 : (K / C_in) * (cl_cs / 8);
        const int nj = 8;    // images per thread: enough threads for the chip, few redrawn words (C5, 64 images: 13.4 us; 15.0 with 16, 15.4 with 2)
        dim3 grid((unsigned)((nline + kThreads - 1) / kThreads), (unsigned)ceil_div(nimg, nj));
        if (dtype == XCONV_F32)
            hipLaunchKernelGGL(gen_zimg_pm1_kernel<XCONV_F32>, grid, dim3(kThreads), 0, st, out, K, r, nimg, seed, C_in, cl_cs, nj);
        else if (dtype == XCONV_BF16)
            hipLaunchKernelGGL(gen_zimg_pm1_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, out, K, r, nimg, seed, C_in, cl_cs, nj);
        else
            hipLaunchKernelGGL(gen_zimg_pm1_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, out, K, r, nimg, seed, C_in, cl_cs, nj);
        return hipGetLastError();
    }
    const long long total = cl_cs ? (K / C_in) * nimg * cl_cs : K * nimg;
    dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(gen_zimg_kernel<XCONV_F32>, grid, dim3(kThreads), 0, st, out, K, r, nimg, dist, seed, C_in, cl_cs, indep, n0, nch);
    else if (dtype == XCONV_BF16)
        hipLaunchKernelGGL(gen_zimg_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, out, K, r, nimg, dist, seed, C_in, cl_cs, indep, n0, nch);
    else
        hipLaunchKernelGGL(gen_zimg_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, out, K, r, nimg, dist, seed, C_in, cl_cs, indep, n0, nch);
    return hipGetLastError();
}

// Eq. (8) for probes over pixels and channels: the estimate of input channel n, which carries the factor 1/r,
// is rescaled to 1/nnz(Z_n), nnz(Z_n) = kept blocks of channel n; a channel without any gives zeros.
// One workgroup per input channel.
__global__ __launch_bounds__(kThreads) void nnz_rescale_kernel(float *__restrict__ dW, int C_out, int C_in, int K2, int r, int dist,
                                                               uint64_t seed)
{
    const int n = blockIdx.x;
    const ProbeGen gen = probe_gen(dist, seed);
    int mine = 0;
    for (int j = threadIdx.x; j < r; j += kThreads) mine += probe_keep(gen, (uint64_t)n * (uint64_t)r + (uint64_t)j) ? 1 : 0;
    __shared__ int total;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    if (mine) atomicAdd(&total, mine);
    __syncthreads();
    const float f = total > 0 ? (float)r / (float)total : 0.0f;
    for (int i = threadIdx.x; i < C_out * K2; i += kThreads) {
        const int m = i / K2, o = i - m * K2;
        dW[((size_t)m * C_in + n) * K2 + o] *= f;
    }
}

hipError_t launch_nnz_rescale(float *dW, int C_out, int C_in, int K2, int r, int dist, uint64_t seed, hipStream_t st)
{
    hipLaunchKernelGGL(nnz_rescale_kernel, dim3(C_in), dim3(kThreads), 0, st, dW, C_out, C_in, K2, r, dist, seed);
    return hipGetLastError();
}

__global__ __launch_bounds__(kThreads) void scale_kernel(const float *__restrict__ in, float *__restrict__ out, int n, float f)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) out[i] = in[i] * f;
}

hipError_t launch_scale(const float *in, float *out, int n, float f, hipStream_t st)
{
    hipLaunchKernelGGL(scale_kernel, dim3(ceil_div(n, kThreads)), dim3(kThreads), 0, st, in, out, n, f);
    return hipGetLastError();
}

// out[b, c] = in[b, c0 + c] * f for c < ncol (rows of `ld` values in, of `ncol` values out)
__global__ __launch_bounds__(kThreads) void scale_cols_kernel(const float *__restrict__ in, float *__restrict__ out, int rows, int ld,
                                                              int c0, int ncol, float f)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= rows * ncol) return;
    const int b = i / ncol, c = i - b * ncol;
    out[i] = in[(size_t)b * ld + c0 + c] * f;
}

hipError_t launch_scale_cols(const float *in, float *out, int rows, int ld, int c0, int ncol, float f, hipStream_t st)
{
    hipLaunchKernelGGL(scale_cols_kernel, dim3(ceil_div(rows * ncol, kThreads)), dim3(kThreads), 0, st, in, out, rows, ld, c0, ncol, f);
    return hipGetLastError();
}

// dW[m, n0 + nl, o] = part[m, nl, o]: the gradient of a window of nch input channels into its place in [C_out, C_in, K2]
__global__ __launch_bounds__(kThreads) void scatter_channels_kernel(const float *__restrict__ part, float *__restrict__ dW, int C_out,
                                                                    int C_in, int K2, int n0, int nch)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= C_out * nch * K2) return;
    const int o = i % K2, nl = (i / K2) % nch, m = i / (K2 * nch);
    dW[((size_t)m * C_in + n0 + nl) * K2 + o] = part[i];
}

hipError_t launch_scatter_channels(const float *part, float *dW, int C_out, int C_in, int K2, int n0, int nch, hipStream_t st)
{
    hipLaunchKernelGGL(scatter_channels_kernel, dim3(ceil_div(C_out * nch * K2, kThreads)), dim3(kThreads), 0, st, part, dW, C_out, C_in,
                       K2, n0, nch);
    return hipGetLastError();
}

hipError_t launch_unpack(int dtype, const void *Xt, float *out, int B, int HW, int r, int CS, hipStream_t st)
{
    const long long total = (long long)B * r * HW;
    dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(unpack_kernel<XCONV_F32>, grid, dim3(kThreads), 0, st, Xt, out, HW, r, CS, total);
    else if (dtype == XCONV_BF16)
        hipLaunchKernelGGL(unpack_kernel<XCONV_BF16>, grid, dim3(kThreads), 0, st, Xt, out, HW, r, CS, total);
    else
        hipLaunchKernelGGL(unpack_kernel<XCONV_F16>, grid, dim3(kThreads), 0, st, Xt, out, HW, r, CS, total);
    return hipGetLastError();
}

hipError_t launch_to_nhwc(int dtype, const void *X, void *out, int B, int C, int HW, int CS, hipStream_t st)
{
    for (int z0 = 0; z0 < B; z0 += kMaxGridZ) {   // a grid's third extent is 16 bits
        dim3 grid(ceil_div(HW, 32), ceil_div(CS, 32), B - z0 < kMaxGridZ ? B - z0 : kMaxGridZ);
        if (dtype == XCONV_F32)
            hipLaunchKernelGGL(to_nhwc_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(X),
                               static_cast<float *>(out), C, HW, CS, z0);
        else
            hipLaunchKernelGGL(to_nhwc_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(X),
                               static_cast<uint16_t *>(out), C, HW, CS, z0);
    }
    return hipGetLastError();
}

hipError_t launch_to_nchw(int dtype, const void *src, void *out, int B, int C, int HW, int pitch, hipStream_t st)
{
    const int VE = dtype == XCONV_F32 ? 4 : 8;
    if (C % VE == 0 && (reinterpret_cast<uintptr_t>(src) & 15u) == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
        for (int z0 = 0; z0 < B; z0 += kMaxGridZ) {
            dim3 vgrid(ceil_div(pitch, 32 * VE), ceil_div(C, 8 * VE), B - z0 < kMaxGridZ ? B - z0 : kMaxGridZ);
            if (dtype == XCONV_F32)
                hipLaunchKernelGGL(to_nchw_vec_kernel<float>, vgrid, dim3(kThreads), 0, st, static_cast<const float *>(src),
                                   static_cast<float *>(out), C, HW, pitch, z0);
            else
                hipLaunchKernelGGL(to_nchw_vec_kernel<uint16_t>, vgrid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                                   static_cast<uint16_t *>(out), C, HW, pitch, z0);
        }
        return hipGetLastError();
    }
    for (int z0 = 0; z0 < B; z0 += kMaxGridZ) {
        dim3 grid(ceil_div(pitch, 32), ceil_div(C, 32), B - z0 < kMaxGridZ ? B - z0 : kMaxGridZ);
        if (dtype == XCONV_F32)
            hipLaunchKernelGGL(to_nchw_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(src),
                               static_cast<float *>(out), C, HW, pitch, z0);
        else
            hipLaunchKernelGGL(to_nchw_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                               static_cast<uint16_t *>(out), C, HW, pitch, z0);
    }
    return hipGetLastError();
}

hipError_t launch_pad_channels(int dtype, const void *src, void *out, long long npix, int C, int CS, hipStream_t st)
{
    const long long total = npix * CS;
    dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(pad_channels_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(src),
                           static_cast<float *>(out), C, CS, total);
    else
        hipLaunchKernelGGL(pad_channels_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                           static_cast<uint16_t *>(out), C, CS, total);
    return hipGetLastError();
}

}  // namespace xc
