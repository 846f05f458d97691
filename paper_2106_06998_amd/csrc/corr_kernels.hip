// Offset-wise correlation of the residual with a channels-last activation-like
// tensor (Algorithm 1, backward step 3 combined with the shift of step 4):
//
//   G[m,j,ky,kx] = sum_{b,oy,ox} dY[b,m,oy,ox] * A[b, oy*sh+ky-ph, ox*sw+kx-pw, j]
//
// and the final reduction + left multiplication with Z/r (backward step 4,
// Eq. (6) step (iii)).  With A = Xt this is the XConv estimate, with A = X in
// channels-last form it is the exact gradient of Eq. (2)/(5).
//
// Shape of the work: an implicit GEMM with M = C_out, N = (columns of A) x kH*kW
// and a very long reduction K = B*Ho*Wo.  Only a handful of output tiles exist,
// so the reduction is split over workgroups (deterministic two-pass reduction:
// partial tiles to scratch, then reduce_partials_kernel and expand_kernel).
//
// Mapping to the matrix cores.  The reduction index is (image, pixel); the MFMA
// needs several consecutive k per lane for the 16-bit types, and the +-1 pixel
// shifts of the kernel offsets would break the alignment of any vector taken
// along x or y.  The kernel therefore packs the *batch*: for 16-bit storage one
// LDS unit is the 8 values of 8 consecutive images at one (pixel, channel), so a
// kernel offset or a stride only changes which unit a lane reads.  dY (NCHW) and
// A (channels-last) are both brought into that form while they are staged into
// LDS, by an 8x8 transpose in registers.  For fp32 storage the MFMA takes one k
// per lane and a unit is a single float of a single image.
//
// One MFMA k-step covers 4 pixel slots (lane group g = lane/16 takes slot g):
//   A operand  lane (m = lane%16, g):  dY unit of pixel slot g, output channel m
//   B operand  lane (j = lane%16, g):  A  unit of the shifted pixel, column j
//   D          16x16 tile of G for one kernel offset
// A wave owns MT*16 output channels x 16 columns x up to 9 offsets (MT*9
// accumulator tiles) and walks over pixels; a workgroup is WM x WJ x WK waves
// (output channels x columns x a split of the k-steps).
//
// Staging.  A step is RB output rows x CW output columns of BI images.  The rows
// of A it needs live in an LDS ring, so consecutive steps of one image reload
// only the new rows.  Global loads for step t+1 are issued into registers before
// the MFMA loop of step t and written to LDS after it.
#include <type_traits>

#include "common.h"
#include "launch.h"

// Timing experiments only (never defined in the shipped build): bit 5 leaves time stamps of the first thread in the partial tile.
#ifndef XCONV_CORR_DBG
#define XCONV_CORR_DBG 0
#endif

namespace xc {

constexpr int kMaxOff = 9;

template <int Q, int N, class F> __device__ inline void ws_for(F &&f)
{
    if constexpr (Q < N) {
        f(std::integral_constant<int, Q>{});
        ws_for<Q + 1, N>(f);
    }
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load of the wave (its release fence drains vmcnt), which would expose
// the latency of the prefetch issued before the barrier; the kernel exchanges data through
// LDS only, so waiting for the LDS counter is sufficient.
// Compiler-only fence.  The prefetch loads of the next step have no use until the following
// loop iteration, so the optimiser would otherwise sink them below the MFMA loop (shorter
// live ranges) and expose their whole latency; a memory clobber keeps them where they are
// issued without making anything wait.
__device__ inline void pin_issued_loads()
{
    asm volatile("" ::: "memory");
}

__device__ inline void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Position of a step: batch group, first output row, first output column.
struct StepPos {
    int bg, band, strip, oy0, x0;
};

// Step positions are the same for every lane; readfirstlane says so to the compiler, which
// otherwise may treat values that went through loop-carried structs as divergent (vector ALU
// index math, and a lane-by-lane loop around every buffer load whose resource depends on them).
__device__ inline StepPos uniform_pos(StepPos s)
{
    s.bg = __builtin_amdgcn_readfirstlane(s.bg);
    s.band = __builtin_amdgcn_readfirstlane(s.band);
    s.strip = __builtin_amdgcn_readfirstlane(s.strip);
    s.oy0 = __builtin_amdgcn_readfirstlane(s.oy0);
    s.x0 = __builtin_amdgcn_readfirstlane(s.x0);
    return s;
}

__device__ inline StepPos decode_step(const CorrParams &P, int t)
{
    StepPos s;
    if (t < (1 << 22)) {
        int q;
        fast_divmod(t, P.NBAND, frcp(P.NBAND), q, s.band);
        fast_divmod(q, P.NSTRIP, frcp(P.NSTRIP), s.bg, s.strip);
    } else {
        s.band = t % P.NBAND;
        t /= P.NBAND;
        s.strip = t % P.NSTRIP;
        s.bg = t / P.NSTRIP;
    }
    s.oy0 = s.band * P.RB;
    s.x0 = s.strip * P.CW;
    return uniform_pos(s);
}
__device__ inline StepPos next_step(const CorrParams &P, StepPos s)
{
    if (++s.band == P.NBAND) {
        s.band = 0;
        if (++s.strip == P.NSTRIP) {
            s.strip = 0;
            ++s.bg;
        }
    }
    s.oy0 = s.band * P.RB;
    s.x0 = s.strip * P.CW;
    return uniform_pos(s);
}

// NOFF: kernel offsets a workgroup accumulates (9, or 1 for 1x1 kernels).  A
// last group with fewer offsets recomputes its first offset in the spare slots
// and does not write them.
// AL: every row segment of dY that a step stages starts on a 16-byte vector (W' and the
// strip width are multiples of the vector length); the staging of dY then has fixed LDS
// addresses per thread and needs no per-element predicates.
template <int DT, int MT, int NA, int NB, int NOFF, bool AL>
__global__ __launch_bounds__(kThreads, ((DT == XCONV_F32 && MT <= 2) ? 2 : 1)) void corr_kernel(const CorrParams P)
{
    draw_z_slice(P.zout, P.nz, P.zdist, P.zseed);
    constexpr bool F32 = (DT == XCONV_F32);
    constexpr int BI = F32 ? 1 : 8;   // images per LDS unit
    constexpr int EPV = F32 ? 4 : 8;  // elements per 16-byte global vector
    using unit_t = typename std::conditional<F32, float, uint4>::type;
    using elem_t = typename std::conditional<F32, float, uint16_t>::type;

#define XC_TRACE()
    unsigned long long ts_[8];
    if constexpr (XCONV_CORR_DBG & 32) { ts_[0] = __builtin_amdgcn_s_memrealtime(); ts_[1] = __builtin_readcyclecounter(); }
    __builtin_amdgcn_s_setprio(2);
    extern __shared__ uint4 lds_raw[];
    unit_t *lds_a0 = reinterpret_cast<unit_t *>(lds_raw);          // dY tile
    unit_t *lds_b = lds_a0 + P.a_units;                            // ring of A rows

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the k-step bookkeeping scalar
    const int jl = lane & 15, g = lane >> 4;
    // WM, WJ, WK are powers of two
    const int wm_shift = __builtin_ctz((unsigned)P.WM), wj_shift = __builtin_ctz((unsigned)P.WJ);
    const int wm = wave & (P.WM - 1), wj = (wave >> wm_shift) & (P.WJ - 1), wk = wave >> (wm_shift + wj_shift);

    int tm, tj;
    fast_divmod((int)blockIdx.y, P.NTM, frcp(P.NTM), tj, tm);
    const int m0 = tm * P.M_WG;   // first output channel of the workgroup tile
    const int jb = tj * P.J_WG;   // first column of A of the workgroup tile
    const int o_first = blockIdx.z * NOFF;
    const int noff = (P.K2 - o_first) < NOFF ? (P.K2 - o_first) : NOFF;

    const elem_t *dY = static_cast<const elem_t *>(P.dY);
    const elem_t *Ag = static_cast<const elem_t *>(P.A);

    // my share of the steps
    const int bx = xcd_block(blockIdx.x, gridDim.x);   // K-split of this workgroup: neighbouring splits on one die (C3: 32.0 -> 29.3 us: the rows of dY, 56 bytes, share cache lines with the rows of the neighbouring splits)
    const int t_begin = bx * P.SQ + (bx < P.SR ? bx : P.SR);
    const int t_end = t_begin + P.SQ + (bx < P.SR ? 1 : 0);

    // ---- per-thread staging tasks, decoded once -------------------------------
    // Global reads go through raw buffer loads: one resource per batch group whose
    // size is the bytes of the images that exist, so that images past the end of
    // the batch (and every offset marked invalid below) read as zero in hardware.
    constexpr uint32_t ES = sizeof(elem_t);
    constexpr uint32_t kOOR = 0x80000000u;  // beyond any resource: the plan keeps a batch group within 2^30 bytes, and no offset added to kOOR wraps
    constexpr int LOG_EPV = F32 ? 2 : 3;
    const uint32_t dy_img_bytes = (uint32_t)P.C_out * (uint32_t)P.dy_plane * ES;  // planes padded to whole 16-byte vectors
    const uint32_t a_img_bytes = (uint32_t)P.H * (uint32_t)P.W * (uint32_t)P.CS * ES;

    // dY task: (rb, ml, cc) = output row in the band, channel in the tile, vector chunk in the row
    const int ntask_a = P.RB * P.M_WG * P.NCHR;
    const float rcp_nchr = frcp(P.NCHR), rcp_mwg = frcp(P.M_WG);
    // Threads without a task get an encoding that fails every predicate (chunk 255 / column
    // 65535 are never real) and an out-of-range load offset, so that the staging code below is
    // free of divergent early-outs: waits for the prefetched registers then sit in
    // unconditional code, where the compiler can count outstanding loads exactly.
    uint32_t a_goff[NA];   // byte offset inside an image without the step's part, or kOOR
    int a_rbcc[NA];        // rb << 8 | cc
    int a_lds[NA];         // LDS unit of (rb, ml) at slot 0; AL: of the task's first slot
    bool a_st[NA];         // AL: the task has a place in the tile
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int task = tid + i * kThreads;
        int cc, ml, rb, q;
        fast_divmod(task, P.NCHR, rcp_nchr, q, cc);
        fast_divmod(q, P.M_WG, rcp_mwg, rb, ml);
        const bool has = task < ntask_a;
        a_rbcc[i] = has ? ((rb << 8) | cc) : 255;
        a_goff[i] = (has && m0 + ml < P.C_out) ? ((uint32_t)(m0 + ml) * (uint32_t)P.dy_plane + (uint32_t)cc * EPV) * ES : kOOR;
        a_lds[i] = has ? (F32 ? (ml * P.ASTR + rb * P.CWp) : (rb * P.CWp * P.ASTR + ml)) : 0;
        a_st[i] = has;
        if constexpr (AL) {
            if (has) a_goff[i] += (uint32_t)(rb * P.Wo) * ES;  // kOOR stays out of range
            a_lds[i] += F32 ? cc * EPV : cc * EPV * P.ASTR;
        }
    }
    // A task: (rr, c, jc) = row among the rows to load, staged column, vector of EPV channels
    const int JC = P.J_WG >> LOG_EPV;
    const int ntask_b = P.NNEW * P.BWc * JC;
    const int jc_shift = __builtin_ctz((unsigned)JC);
    const float rcp_bwc = frcp(P.BWc), rcp_nr = frcp(P.NR);
    const int rotmul = 8 >> __builtin_ctz((unsigned)(P.J_WG >> 4));  // 16-bit layout: rotation of each 16-column group (see b_store_task)
    int b_rr[NB], b_c[NB];   // c = 65535 for a thread without a task: fails every column test
    uint32_t b_goff[NB];     // byte offset of (row rr, column c, vector jc) from the step's first row and column
    int b_lds[NB];           // LDS unit of (slot 0, column c, vector jc)
    int b_rot[NB];           // 16-bit: first unit, inside the 16-column group, of the task's 8 columns
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int task = tid + i * kThreads;
        const int jc = task & (JC - 1);  // J_WG is 16, 32 or 64 and a vector is 4 or 8 columns: JC is a power of two
        int c, rr;
        fast_divmod(task >> jc_shift, P.BWc, rcp_bwc, rr, c);
        const bool has = task < ntask_b;
        b_rr[i] = has ? rr : 0;
        b_c[i] = has ? c : 0xffff;
        b_goff[i] = ((uint32_t)(rr * P.W + c) * (uint32_t)P.CS + (uint32_t)(jb + jc * EPV)) * ES;
        b_lds[i] = F32 ? (c * P.BSTR + jc * 4) : (c * P.BSTR + 16 * (jc >> 1));
        b_rot[i] = F32 ? 0 : (((jc & 1) * 8 + (jc >> 1) * rotmul) & 15);
    }

    uint4 ra[NA][BI];
    uint4 rbv[NB][BI];

    // `live` false (the step does not exist): a resource of size zero, every load reads as zero.
    // Prefetches are issued unconditionally with such a resource instead of being skipped by a
    // branch, which would leave a merge of "loaded" and "old" register values for the compiler
    // to copy (and to wait for) right after the loads are issued.
    auto rsrc_of = [&](const elem_t *base, int bg, uint32_t img_bytes, bool live) {
        bg = __builtin_amdgcn_readfirstlane(bg);
        int left = P.B - bg * BI;
        left = left < BI ? left : BI;
        left = (live && left > 0) ? left : 0;
        left = __builtin_amdgcn_readfirstlane(left);
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<elem_t *>(base + (size_t)bg * BI * (img_bytes / ES)), 0,
                                                 (uint32_t)left * img_bytes, 0x00020000);
    };
    auto buf16 = [](__amdgpu_buffer_rsrc_t r, uint32_t voff) {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
        return uint4{v.x, v.y, v.z, v.w};
    };

    // ---- dY: global -> registers ----------------------------------------------
    auto a_load = [&](const StepPos &sp, bool live) {
        const int fs = sp.oy0 * P.Wo + sp.x0;  // flat index of the step's first pixel
        const __amdgpu_buffer_rsrc_t rs = rsrc_of(dY, sp.bg, dy_img_bytes, live);
        const int rows_left = P.Ho - sp.oy0;
        const int cw_eff = (P.Wo - sp.x0) < P.CW ? (P.Wo - sp.x0) : P.CW;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int rb = a_rbcc[i] >> 8;
            uint32_t voff;
            if constexpr (AL) {
                // chunks past the strip's last column read as zero: they are the tile's zero tail
                voff = a_goff[i] + (uint32_t)fs * ES;
                voff = (rb < rows_left && (a_rbcc[i] & 0xff) * EPV < cw_eff) ? voff : kOOR;
            } else {
                const uint32_t f0 = (uint32_t)(fs + rb * P.Wo);
                voff = a_goff[i] + ((f0 >> LOG_EPV) << 4);
                voff = (rb < rows_left) ? voff : kOOR;
            }
#pragma unroll
            for (int img = 0; img < BI; ++img) ra[i][img] = buf16(rs, voff + (uint32_t)img * dy_img_bytes);
        }
    };

    // ---- dY: registers -> LDS.  16-bit: units [slot][m]; fp32: floats [m][slot].
    auto a_store = [&](const StepPos &sp, unit_t *lds_a) {
        const int cw_eff = (P.Wo - sp.x0) < P.CW ? (P.Wo - sp.x0) : P.CW;
        const int fs = sp.oy0 * P.Wo + sp.x0;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if constexpr (AL) {
                if constexpr (F32) {
                    asm volatile("" : "+v"(ra[i][0].x), "+v"(ra[i][0].y), "+v"(ra[i][0].z), "+v"(ra[i][0].w));
                    if (a_st[i]) *reinterpret_cast<uint4 *>(lds_a + a_lds[i]) = ra[i][0];
                } else {
                    uint32_t rows[8][4];
#pragma unroll
                    for (int q = 0; q < 8; ++q) { rows[q][0] = ra[i][q].x; rows[q][1] = ra[i][q].y; rows[q][2] = ra[i][q].z; rows[q][3] = ra[i][q].w; }
                    uint4 cols[8];
                    transpose_rows8<4>(rows, cols);
                    uint4 *dst = lds_a + a_lds[i];
                    if (a_st[i]) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) dst[e * P.ASTR] = cols[e];
                    }
                }
                continue;
            }
            const int rb = a_rbcc[i] >> 8, cc = a_rbcc[i] & 0xff;
            const int xs0 = cc * EPV - ((fs + rb * P.Wo) & (EPV - 1));  // slot of the chunk's first pixel (may be negative)
            if constexpr (F32) {
                asm volatile("" : "+v"(ra[i][0].x), "+v"(ra[i][0].y), "+v"(ra[i][0].z), "+v"(ra[i][0].w));  // data arrives here, not inside a branch
                float *dst = lds_a + a_lds[i];
                if (xs0 >= 0 && xs0 + 4 <= cw_eff && (xs0 & 3) == 0) {
                    *reinterpret_cast<uint4 *>(dst + xs0) = ra[i][0];
                } else {
                    const uint32_t w[4] = {ra[i][0].x, ra[i][0].y, ra[i][0].z, ra[i][0].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if ((unsigned)(xs0 + e) < (unsigned)cw_eff) dst[xs0 + e] = __uint_as_float(w[e]);
                }
            } else {
                uint32_t rows[8][4];
#pragma unroll
                for (int q = 0; q < 8; ++q) { rows[q][0] = ra[i][q].x; rows[q][1] = ra[i][q].y; rows[q][2] = ra[i][q].z; rows[q][3] = ra[i][q].w; }
                uint4 cols[8];
                transpose_rows8<4>(rows, cols);
                uint4 *dst = lds_a + a_lds[i];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if ((unsigned)(xs0 + e) < (unsigned)cw_eff) dst[(xs0 + e) * P.ASTR] = cols[e];
            }
        }
        // pixel slots past the strip's last column (up to CWp) take part in the MFMAs: keep them zero
        const int ntail = AL ? 0 : P.CWp - cw_eff;
        if (ntail > 0) {
            for (int t = tid; t < P.RB * ntail * P.M_WG; t += kThreads) {
                const int ml = t % P.M_WG, q = t / P.M_WG;
                const int xs = cw_eff + q % ntail, rb = q / ntail;
                if constexpr (F32) lds_a[ml * P.ASTR + rb * P.CWp + xs] = 0.0f;
                else lds_a[(size_t)(rb * P.CWp + xs) * P.ASTR + ml] = uint4{0u, 0u, 0u, 0u};
            }
        }
    };

    // ---- A rows: global -> registers.  Rows are in padded coordinates (iy + ph).
    // iy0, ix0: input row and column of the task grid's origin (may be negative: padding)
    auto b_load_task = [&](__amdgpu_buffer_rsrc_t rs, int iy0, int ix0, int rr, int c, uint32_t goff, uint4 (&dst)[BI]) {
        const bool ok = (unsigned)(iy0 + rr) < (unsigned)P.H && (unsigned)(ix0 + c) < (unsigned)P.W;
        const uint32_t base = (uint32_t)(iy0 * P.W + ix0) * ((uint32_t)P.CS * ES);  // wraps when negative; exact for every in-range pixel
        const uint32_t voff = ok ? base + goff : kOOR;
#pragma unroll
        for (int img = 0; img < BI; ++img) dst[img] = buf16(rs, voff + (uint32_t)img * a_img_bytes);
    };
    // 16-bit LDS unit of (staged pixel, column j): pixel stride J_WG+1 units; inside a pixel
    // the 16-column group G sits at 16G and is rotated by G*rotmul.  Fragment reads
    // (16 consecutive columns of one pixel) and staging writes (8 columns per lane,
    // lanes running over column chunks then pixels) are then both free of bank conflicts.
    auto b_store_task = [&](int slot, int c, int lds0, int rot, const uint4 (&src)[BI]) {
        if constexpr (F32) {
            uint4 v = src[0];
            asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));  // data arrives here, not inside a branch
            float *dst = lds_b + slot * (P.BWc * P.BSTR) + lds0;
            if (c < P.BWc) *reinterpret_cast<uint4 *>(dst) = v;
        } else {
            uint32_t rows[8][4];
#pragma unroll
            for (int q = 0; q < 8; ++q) { rows[q][0] = src[q].x; rows[q][1] = src[q].y; rows[q][2] = src[q].z; rows[q][3] = src[q].w; }
            uint4 cols[8];
            transpose_rows8<4>(rows, cols);
            uint4 *dst = lds_b + slot * (P.BWc * P.BSTR) + lds0;
            if (c < P.BWc) {
#pragma unroll
                for (int e = 0; e < 8; ++e) dst[(rot + e) & 15] = cols[e];
            }
        }
    };
    // rows the step loads in steady state: [oy0*sh + NOLD, oy0*sh + NR)
    auto b_load = [&](const StepPos &sp, bool live) {
        const __amdgpu_buffer_rsrc_t rs = rsrc_of(Ag, sp.bg, a_img_bytes, live);
        const int iy0 = sp.oy0 * P.sh + P.NOLD - P.ph;
        const int ix0 = sp.x0 * P.sw - P.pw;
#pragma unroll
        for (int i = 0; i < NB; ++i) b_load_task(rs, iy0, ix0, b_rr[i], b_c[i], b_goff[i], rbv[i]);
    };
    auto b_store = [&](const StepPos &sp) {
        int rowmod, qd_;
        fast_divmod(sp.oy0 * P.sh + P.NOLD, P.NR, rcp_nr, qd_, rowmod);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            int slot = rowmod + b_rr[i];
            slot = slot >= P.NR ? slot - P.NR : slot;
            b_store_task(slot, b_c[i], b_lds[i], b_rot[i], rbv[i]);
        }
    };
    // rows [oy0*sh, oy0*sh + NOLD) that a step normally inherits from its predecessor
    auto b_fill_old = [&](const StepPos &sp) {
        const __amdgpu_buffer_rsrc_t rs = rsrc_of(Ag, sp.bg, a_img_bytes, true);
        const int row_first = sp.oy0 * P.sh;
        const int ix0 = sp.x0 * P.sw - P.pw;
        const int ntask = P.NOLD * P.BWc * JC;
        for (int task = tid; task < ntask; task += kThreads) {
            const int jc = task & (JC - 1);
            int c, rr;
            fast_divmod(task >> jc_shift, P.BWc, rcp_bwc, rr, c);
            const uint32_t goff = ((uint32_t)(rr * P.W + c) * (uint32_t)P.CS + (uint32_t)(jb + jc * EPV)) * ES;
            const int lds0 = F32 ? (c * P.BSTR + jc * 4) : (c * P.BSTR + 16 * (jc >> 1));
            const int rot = F32 ? 0 : (((jc & 1) * 8 + (jc >> 1) * rotmul) & 15);
            uint4 tmp[BI];
            b_load_task(rs, row_first - P.ph, ix0, rr, c, goff, tmp);
            int slot, qd_;
            fast_divmod(row_first + rr, P.NR, rcp_nr, qd_, slot);
            b_store_task(slot, c, lds0, rot, tmp);
        }
    };

    // ---- accumulators -----------------------------------------------------------
    f32x4 acc[MT][NOFF];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int o = 0; o < NOFF; ++o) acc[mt][o] = f32x4{0.f, 0.f, 0.f, 0.f};

    int off_ky[NOFF], off_kx[NOFF];
    const float rcp_kw = frcp(P.kW);
#pragma unroll
    for (int o = 0; o < NOFF; ++o) {
        const int oo = (o < noff) ? (o_first + o) : o_first;
        fast_divmod(oo, P.kW, rcp_kw, off_ky[o], off_kx[o]);
    }

    // ---- MFMA loop over the k-steps of a staged step -----------------------------
    // A k-step is 4 consecutive pixel slots of one output row.  Wave wk takes
    // k-steps wk, wk+WK, ...  All of the bookkeeping below is wave-uniform.
    const int NXQ = P.CWp >> 2;          // k-steps per output row
    // fp32 dY tile is [m][slot] (row stride ASTR floats), 16-bit tile is [slot][m] (slot stride ASTR units)
    const int a_lane = F32 ? (((wm * MT) * 16 + jl) * P.ASTR + g) : (g * P.ASTR + (wm * MT) * 16 + jl);
    const int a_mt = F32 ? 16 * P.ASTR : 16;  // LDS units between the M tiles of a wave
    const int b_lane = F32 ? (g * P.sw * P.BSTR + wj * 16 + jl) : (g * P.sw * P.BSTR + wj * 16 + ((jl + wj * rotmul) & 15));
    const int b_xq = 4 * P.sw * P.BSTR;  // LDS units between k-steps of a row

    // Fragment reads are issued as opaque instructions and waited for by hand.  Left to the
    // compiler, the reads of a k-step end up right in front of the MFMAs that use them (it
    // folds the double buffer into one set of registers), and the matrix cores idle for an LDS
    // round trip per k-step.  Here the fragments of k-step i+1 are requested during the MFMAs
    // of k-step i, each B fragment into the registers that the MFMAs of the previous offset
    // have just read; LDS returns in order, so counting the younger requests tells when a
    // fragment has arrived.
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    using frag_t = typename std::conditional<F32, float, u32x4>::type;
    constexpr uint32_t US = sizeof(unit_t);
    auto lds_read = [](frag_t &dst, uint32_t addr) {
        if constexpr (F32) asm volatile("ds_read_b32 %0, %1" : "=v"(dst) : "v"(addr) : "memory");
        else asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr) : "memory");
    };
    const uint32_t lds0 = __builtin_amdgcn_groupstaticsize();  // the dynamic allocation starts behind the static one
    const uint32_t a_base = lds0 + (uint32_t)a_lane * US;
    const uint32_t b_base = lds0 + (uint32_t)(P.a_units + b_lane) * US;
    const uint32_t a_slot_bytes = F32 ? 4u : (uint32_t)P.ASTR * 16u;
    const uint32_t a_mt_bytes = (uint32_t)a_mt * US;
    const uint32_t step_a = (uint32_t)(4 * P.WK) * a_slot_bytes;   // bytes between two k-steps of this wave in a row
    const uint32_t step_b = (uint32_t)(P.WK * b_xq) * US;
    const int n_row = (NXQ - wk + P.WK - 1) >> __builtin_ctz((unsigned)P.WK);                // k-steps of this wave in every output row: xq = wk, wk + WK, ...
    int sh_mod, qs_;
    fast_divmod(P.sh, P.NR, rcp_nr, qs_, sh_mod);
    const int kRB = P.RB, kNR = P.NR, kCWp = P.CWp, kBWc = P.BWc, kBSTR = P.BSTR;  // loop constants, read once

    // ---- main loop ---------------------------------------------------------------
    // MFMA loop of one staged step
    auto compute_step = [&](const StepPos &spc) {
        if (n_row <= 0) return;
        const int total = kRB * n_row;
        int rowmod, qd_;   // ring slot of the first row that output row rb needs
        fast_divmod(spc.oy0 * P.sh, kNR, rcp_nr, qd_, rowmod);
        uint32_t pa[MT], pb[NOFF];
        auto set_row = [&](int rb) {
            const uint32_t a0 = a_base + (uint32_t)(rb * kCWp + 4 * wk) * a_slot_bytes;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) pa[mt] = a0 + (uint32_t)mt * a_mt_bytes;
#pragma unroll
            for (int o = 0; o < NOFF; ++o) {
                int slot = rowmod + off_ky[o];
                slot = slot >= kNR ? slot - kNR : slot;
                const int u = __builtin_amdgcn_readfirstlane(wk * b_xq + (slot * kBWc + off_kx[o]) * kBSTR);
                pb[o] = b_base + (uint32_t)u * US;
            }
        };
        // A wait names the registers it guards as operands, and no fragment is ever copied: the A fragments
        // alternate between two register sets (k-step i multiplies from set i & 1 and requests the next one into
        // the other set).  A copy "a = a_next" behind the wait would be the compiler's to place, and it has been seen
        // in front of the wait, reading registers whose data had not arrived yet.
        frag_t a2[2][MT], b[NOFF];
        auto a_arrived = [&](auto parc) {  // the A fragments are the oldest of the MT + NOFF requests of a k-step
            constexpr int par = decltype(parc)::value;
            if constexpr (MT == 1)
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a2[par][0]) : "n"(NOFF) : "memory");
            else if constexpr (MT == 2)
                asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a2[par][0]), "+v"(a2[par][1]) : "n"(NOFF) : "memory");
            else
                asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a2[par][0]), "+v"(a2[par][1]), "+v"(a2[par][2]), "+v"(a2[par][3]) : "n"(NOFF) : "memory");
            static_assert(MT == 1 || MT == 2 || MT == 4, "a_arrived names MT registers");
        };
        set_row(0);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) lds_read(a2[0][mt], pa[mt]);
#pragma unroll
        for (int o = 0; o < NOFF; ++o) lds_read(b[o], pb[o]);
        a_arrived(std::integral_constant<int, 0>{});

        // One k-step: its MFMAs and the requests for the fragments at (pa, pb).  Requests in
        // issue order: A (MT), then B of offset o-1 right after the MFMAs of offset o, B of the
        // last offset at the end.  Before the MFMAs of offsets o..o+2 (o = 0, 3, 6) the previous
        // k-step's requests up to offset o+2 must be done: at that point the younger ones are
        // the rest of the previous k-step, this k-step's A and its B up to offset o-2.
        constexpr int WG3 = (NOFF % 3 == 0) ? 3 : 1;
        auto kstep = [&](auto parc) {
            constexpr int par = decltype(parc)::value;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) lds_read(a2[par ^ 1][mt], pa[mt]);
            ws_for<0, NOFF>([&](auto oc) {
                constexpr int o = decltype(oc)::value;
                if constexpr (o % WG3 == 0) {
                    constexpr int younger = (NOFF - WG3 - o) + MT + (o >= 2 ? o - 1 : 0);
                    if constexpr (WG3 == 3)
                        asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(b[o]), "+v"(b[o + WG3 - 2]), "+v"(b[o + WG3 - 1]) : "n"(younger) : "memory");
                    else
                        asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(b[o]) : "n"(younger) : "memory");
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if constexpr (F32) acc[mt][o] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[par][mt], b[o], acc[mt][o], 0, 0, 0);
                    else acc[mt][o] = mfma16<DT>(__builtin_bit_cast(uint4, a2[par][mt]), __builtin_bit_cast(uint4, b[o]), acc[mt][o]);
                }
                if constexpr (o >= 1) lds_read(b[o - 1], pb[o - 1]);
            });
            lds_read(b[NOFF - 1], pb[NOFF - 1]);
            a_arrived(std::integral_constant<int, par ^ 1>{});
            __builtin_amdgcn_sched_barrier(0);
        };

        int i_row = 0, rb = 0;
        // addresses of the k-step after the current one (after the last one: unchanged, the requests repeat)
        auto advance = [&]() {
            if (++i_row == n_row) {
                i_row = 0;
                ++rb;
                rowmod += sh_mod;
                rowmod = rowmod >= kNR ? rowmod - kNR : rowmod;
                if (rb < kRB) set_row(rb);
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) pa[mt] += step_a;
#pragma unroll
                for (int o = 0; o < NOFF; ++o) pb[o] += step_b;
            }
        };
        int i = 0;
        for (; i + 1 < total; i += 2) {
            advance();
            kstep(std::integral_constant<int, 0>{});
            advance();
            kstep(std::integral_constant<int, 1>{});
        }
        if (i < total) {
            advance();
            kstep(std::integral_constant<int, 0>{});
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };
    auto contiguous = [&](const StepPos &a, const StepPos &b) { return b.bg == a.bg && b.x0 == a.x0 && b.oy0 == a.oy0 + P.RB; };

    StepPos sp = decode_step(P, t_begin);
    // Stage step t between two barriers, prefetch t+1 into registers, then run the MFMA loop
    // of t while those loads are in flight.  The prefetch is issued unconditionally (a step that
    // does not exist reads zeros through an empty resource): a branch around it would leave a
    // merge of loaded and old register values that the compiler resolves with copies, and so
    // with a wait for the loads right after issuing them.
    a_load(sp, t_begin < t_end);
    b_load(sp, t_begin < t_end);
    StepPos prev = sp;
    prev.bg = -1;
    for (int step = t_begin; step < t_end; ++step) {
        lds_barrier();  // everyone is done reading the tiles of the previous step
        if (P.NOLD > 0 && !contiguous(prev, sp)) b_fill_old(sp);
        a_store(sp, lds_a0);
        b_store(sp);
        lds_barrier();
        const StepPos spn = next_step(P, sp);
        a_load(spn, step + 1 < t_end);
        b_load(spn, step + 1 < t_end);
        pin_issued_loads();
        // A wave that issues MFMAs back to back is always ready, and the issue arbiter then
        // starves the vector, LDS and load instructions of the other waves on its SIMD (those of
        // the second workgroup on the CU, which is staging while this one multiplies).  Everything
        // but the MFMA loop runs at a raised priority so that staging slips in between MFMAs.
        if constexpr (XCONV_CORR_DBG & 32) { if (step == t_begin) { ts_[2] = __builtin_amdgcn_s_memrealtime(); ts_[3] = __builtin_readcyclecounter(); } }
        __builtin_amdgcn_s_setprio(0);
        compute_step(sp);
        __builtin_amdgcn_s_setprio(2);
        prev = sp;
        sp = spn;
    }
    lds_barrier();
    if constexpr (XCONV_CORR_DBG & 32) { ts_[4] = __builtin_amdgcn_s_memrealtime(); ts_[5] = __builtin_readcyclecounter(); }

    // ---- reduce the WK k-split waves through LDS, then write the partial tile --
    // One buffer per (wm, wj) group; waves wk = 1..WK-1 hand their tiles to wave
    // wk = 0 one after the other, so the summation order is fixed.
    f32x4 *red = reinterpret_cast<f32x4 *>(lds_raw) + ((size_t)(wm + P.WM * wj) * MT * NOFF) * 64 + lane;
    for (int k = 1; k < P.WK; ++k) {
        lds_barrier();
        if (wk == k) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int o = 0; o < NOFF; ++o) red[(mt * NOFF + o) * 64] = acc[mt][o];
        }
        lds_barrier();
        if (wk == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int o = 0; o < NOFF; ++o) acc[mt][o] += red[(mt * NOFF + o) * 64];
        }
    }
    if (wk == 0) {
        // D tile: lane (jl, g) holds rows 4g..4g+3 (output channels) of column jl
        const int jcol = jb + wj * 16 + jl;
#pragma unroll
        for (int o = 0; o < NOFF; ++o) {
            if (o < noff) {
                float *dst = P.part + (size_t)bx * P.K2 * P.JP * P.MP + tile_index(o_first + o, jcol, m0 + (wm * MT) * 16 + 4 * g, P.JP, P.MP);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) *reinterpret_cast<f32x4 *>(dst + (size_t)16 * mt * P.JP) = acc[mt][o];   // 16 rows = four channel quads
            }
        }
    }
    if constexpr (XCONV_CORR_DBG & 32) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        ts_[6] = __builtin_amdgcn_s_memrealtime(); ts_[7] = __builtin_readcyclecounter();
        if (tid == 0 && t_begin < t_end) {
            unsigned long long *d = reinterpret_cast<unsigned long long *>(P.part + (size_t)bx * P.K2 * P.JP * P.MP + tile_index(o_first, jb, m0, P.JP, P.MP));
            for (int q = 0; q < 8; ++q) d[q] = ts_[q];
        }
    }
}

// ---------------------------------------------------------------------------
// Second pass, part 1: T[e] = sum_s part[s][e] over the S partial buffers, in a
// fixed order.  16 consecutive float4 elements x 16 groups of s per workgroup.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(const f32x4 *__restrict__ part, f32x4 *__restrict__ T,
                                                                   int S, int E4, float *__restrict__ Zout, int nz, int zblocks,
                                                                   int dist, uint64_t seed)
{
    // The first `zblocks` workgroups redraw Z[s] for the expansion that follows (Alg. 1 backward
    // step 2) instead of a kernel launch of its own; the rest reduce.
    if ((int)blockIdx.x < zblocks) {
        const int i = blockIdx.x * kThreads + threadIdx.x;
        if (blockIdx.y == 0 && i < nz) Zout[i] = probe_entry(probe_gen(dist, seed), (uint64_t)i);
        return;
    }
    // blockIdx.y: one set of S partial buffers and one reduced tile per correlation launch
    // (volumetric layers: one per kernel-depth offset), stored back to back
    part += (size_t)blockIdx.y * S * E4;
    T += (size_t)blockIdx.y * E4;
    __shared__ f32x4 red[16][17];
    const int ve = threadIdx.x & 15, sg = threadIdx.x >> 4;
    const int e4 = ((int)blockIdx.x - zblocks) * 16 + ve;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0, s2 = s0, s3 = s0;
    if (e4 < E4) {
        const f32x4 *p = part + e4;
        int k = sg;
        for (; k + 48 < S; k += 64) {
            const f32x4 v0 = p[(size_t)k * E4], v1 = p[(size_t)(k + 16) * E4];
            const f32x4 v2 = p[(size_t)(k + 32) * E4], v3 = p[(size_t)(k + 48) * E4];
            s0 += v0; s1 += v1; s2 += v2; s3 += v3;
        }
        for (; k < S; k += 16) s0 += p[(size_t)k * E4];
    }
    red[sg][ve] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (sg == 0 && e4 < E4) {
        f32x4 t = red[0][ve];
#pragma unroll
        for (int q = 1; q < 16; ++q) t += red[q][ve];
        T[e4] = t;
    }
}

// ---------------------------------------------------------------------------
// Second pass, part 2 (Algorithm 1 backward step 4, Eq. (6) step (iii)):
//   dW[m,n,o] = (1/r) sum_j Z[n,j] T[o,j,m],
// one small fp32 GEMM per offset (rows m, columns n, contraction over the r probes) on the
// 16x16x4 matrix instruction.  One wave owns a 16 x 16 tile of (m, n) and OG consecutive
// offsets: the A operand (T, in the layout of tile_index) and the B operand (Z rows) are read straight
// from global memory, and a lane ends up with all OG offsets of its (m, n) pairs, which are
// adjacent in dW.
// ---------------------------------------------------------------------------
// nnz_norm: rows are scaled by 1 / nnz(Z_n), the number of non-zero entries of row n of Z (Eq. (8),
// block-sparse probing vectors), instead of 1 / r; a row without any gives zeros.
template <int OG>
__global__ __launch_bounds__(64) void expand_kernel(const float *__restrict__ T, const float *__restrict__ Z,
                                                    float *__restrict__ dW, int K2, int JP, int MP, int C_out, int C_in, int r,
                                                    int NTN, int nnz_norm)
{
    const int lane = threadIdx.x, l16 = lane & 15, g = lane >> 4;
    const int nt = blockIdx.x % NTN, mt = blockIdx.x / NTN;
    const int o0 = blockIdx.y * OG;
    const int ncol = nt * 16 + l16;
    const float *zrow = Z + (size_t)(ncol < C_in ? ncol : C_in - 1) * r;
    const float *tcol[OG];
#pragma unroll
    for (int o = 0; o < OG; ++o) {
        const int oo = (o0 + o < K2) ? o0 + o : K2 - 1;  // offsets past the end repeat the last one and are not stored
        tcol[o] = T + tile_index(oo, 0, mt * 16 + l16, JP, MP);
    }
    f32x4 acc[OG];
#pragma unroll
    for (int o = 0; o < OG; ++o) acc[o] = f32x4{0.f, 0.f, 0.f, 0.f};
    // NU k-steps (4 probes each) per trip, all loads issued before the first use: with few offsets per wave a trip
    // covers 64 probes, so that a wave waits for memory once; probes past r are clamped to the last one and enter
    // with a zero B operand
    constexpr int NU = OG >= 9 ? 4 : 16;
    for (int j0 = 0; j0 < r; j0 += 4 * NU) {
        float bv[NU], av[NU][OG];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int j = j0 + 4 * u + g;
            const int jc = j < r ? j : r - 1;
            const float zv = zrow[jc];
            bv[u] = j < r ? zv : 0.f;
#pragma unroll
            for (int o = 0; o < OG; ++o) av[u][o] = tcol[o][(size_t)jc * 4];
        }
#pragma unroll
        for (int u = 0; u < NU; ++u)
#pragma unroll
            for (int o = 0; o < OG; ++o) acc[o] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][o], bv[u], acc[o], 0, 0, 0);
    }
    float inv_r = 1.0f / (float)r;
    if (nnz_norm) {
        int cnt = 0;
        for (int j = 0; j < r; ++j) cnt += zrow[j] != 0.0f ? 1 : 0;
        inv_r = cnt > 0 ? 1.0f / (float)cnt : 0.0f;
    }
    if (ncol < C_in) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int m = mt * 16 + 4 * g + v;
            if (m < C_out) {
                float *dst = dW + ((size_t)m * C_in + ncol) * K2 + o0;
#pragma unroll
                for (int o = 0; o < OG; ++o)
                    if (o0 + o < K2) dst[o] = acc[o][v] * inv_r;
            }
        }
    }
}

// Fixed-order sum of the tiles first, first + step, ... < S of one 16-byte element (p points at the element in
// tile 0, tiles are `tile` elements apart): NC interleaved chains (NC loads in flight per thread: the tiles were
// written by other compute units and come from beyond the L2), combined in a fixed tree.
// A partial tile is read once: non-temporal, so that it does not stay in the caches in place of what the next launches
// read (the second pass itself takes the same time; the correlation of the next step was 0.6-1.6 us faster on C5 and C3).
__device__ inline f32x4 load_part(const f32x4 *p) { return __builtin_nontemporal_load(p); }

template <int NC> __device__ inline f32x4 chain_sum(const f32x4 *p, int first, int step, int S, size_t tile)
{
    f32x4 c[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) c[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    int k = first;
    for (; k + (NC - 1) * step < S; k += NC * step) {   // NC tiles per trip, every load issued before the first sum
        f32x4 v[NC];
#pragma unroll
        for (int i = 0; i < NC; ++i) v[i] = load_part(p + (size_t)(k + i * step) * tile);
#pragma unroll
        for (int i = 0; i < NC; ++i) c[i] += v[i];
    }
    if (k < S) {   // the last, shorter trip (chain i keeps taking tile k + i * step)
        f32x4 v[NC];
#pragma unroll
        for (int i = 0; i < NC; ++i) v[i] = (k + i * step < S) ? load_part(p + (size_t)(k + i * step) * tile) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NC; ++i) c[i] += v[i];
    }
#pragma unroll
    for (int w = NC / 2; w >= 1; w >>= 1)
#pragma unroll
        for (int i = 0; i < w; ++i) c[i] += c[i + w];
    return c[0];
}

// The same for an element with at most NC tiles to take: one trip, no running sums
template <int NC> __device__ inline f32x4 once_sum(const f32x4 *p, int first, int step, int S, size_t tile)
{
    f32x4 v[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) v[i] = (first + i * step < S) ? load_part(p + (size_t)(first + i * step) * tile) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = NC / 2; w >= 1; w >>= 1)
#pragma unroll
        for (int i = 0; i < w; ++i) v[i] += v[i + w];
    return v[0];
}

// ---------------------------------------------------------------------------
// Second pass of the exact gradient in one launch: a workgroup owns four consecutive output channels (one
// 16-byte element per column) of one kernel offset and JC input channels.  It sums the S partial tiles of its
// slab T[og, j0 .. j0+JC, 4mq .. 4mq+3] in a fixed order (16 interleaved chains per thread, chains and thread
// groups combined in a fixed tree: the result does not depend on timing) into LDS; the slab of a tile is one
// run of JC elements, so a wave reads whole cache lines.  Then dW[m,n,og] = T[og,n,m], a transposed store.
// Offsets are counted over `nsets` sets of partial tiles stored back to back (volumetric layers: one set per
// kernel-depth offset), og = set * K2 + o, K2T = nsets * K2.  The grid's first extent is a multiple of 8, so
// the workgroups that write the K2T offsets of one (m, n) run of dW share an L2, which merges their 4-byte stores.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void pass2_exact_kernel(const f32x4 *__restrict__ part, float *__restrict__ dW, int S, int K2,
                                                               int K2T, int JP, int MQ, int JC, int C_out, int C_in)
{
    extern __shared__ f32x4 p2_lds[];   // slab [JC], then the thread groups' sums [NG][NE] (few-element slabs only)
    const int tid = threadIdx.x;
    const int mq = blockIdx.x;
    if (mq >= MQ) return;   // (the grid is padded to a multiple of 8 workgroups per offset)
    const int og = blockIdx.y, set = og / K2, o = og - set * K2;
    const int j0 = blockIdx.z * JC;
    const int NE = JC;
    const size_t tile = (size_t)K2 * MQ * JP;   // 16-byte elements of one partial tile
    const f32x4 *base = part + (size_t)set * S * tile + ((size_t)o * MQ + mq) * JP + j0;
    const int NG = NE >= kThreads ? 1 : kThreads / NE;   // groups of threads that share the tiles of an element
    f32x4 *red = p2_lds + NE;

    if (NG == 1) {
        for (int e = tid; e < NE; e += kThreads) p2_lds[e] = chain_sum<16>(base + e, 0, 1, S, tile);
    } else {
        const int gi = tid / NE, e = tid - gi * NE;
        if (gi < NG) red[gi * NE + e] = chain_sum<16>(base + e, gi, NG, S, tile);
        __syncthreads();
        if (tid < NE) {
            f32x4 t = red[tid];
            for (int q = 1; q < NG; ++q) t += red[q * NE + tid];
            p2_lds[tid] = t;
        }
    }
    __syncthreads();
    const float *slab = reinterpret_cast<const float *>(p2_lds);   // [JC][4]: dW[4mq .. 4mq+3, j0.., og] transposed
    for (int e = tid; e < JC * 4; e += kThreads) {
        const int mi = e & 3, j = e >> 2;
        const int m = 4 * mq + mi, n = j0 + j;
        if (m < C_out && n < C_in) dW[((size_t)m * C_in + n) * K2T + og] = slab[e];
    }
}

// ---------------------------------------------------------------------------
// Second pass of the estimate in one launch, expansion on the matrix cores: a workgroup of 16 waves owns QW
// consecutive quads of output channels of one kernel offset.  Its threads request a block of rows of Z (whole
// rows, consecutive lanes consecutive 16 bytes), sum the S partial tiles of the slab
// T[og, :, 4 QW mg .. + 4 QW - 1] in a fixed order (chain_sum<8>: with 1024 threads that is 128 KB in flight per
// compute unit; the QW quads are one run of QW * JP elements of a tile) into LDS, put the rows of Z into LDS
// (row pitch = 4 * odd words: the 64 lanes of a B operand, 16 rows x 4 consecutive probes, fall on distinct
// banks), and each wave multiplies the slab (A operand of the 16x16x4 instruction, rows = output channels,
// 16 - 4 QW of them zero) with its tiles of 16 input channels:
//   dW[m,n,og] = (1/r) sum_j Z[n,j] T[og,j,m]      (or 1 / nnz(Z_n), Eq. (8))
// A lane ends up with 4 output channels of one input channel.  Layers with more input channels than one block
// of rows holds (NR rows, at most 4 x 16 bytes per thread) take further blocks in turn.  Grid: (quad groups
// padded to a multiple of 8, offsets): the workgroups that write the K2T offsets of one (m, n) run of dW then
// share an L2, which merges their 4-byte stores.
// ---------------------------------------------------------------------------
constexpr int kP2Threads = 1024;

template <int QW>
__global__ __launch_bounds__(kP2Threads) void pass2_mfma_kernel(const f32x4 *__restrict__ part, const float *__restrict__ Z,
                                                                float *__restrict__ dW, int S, int K2, int K2T, int JP, int MQ,
                                                                int C_out, int C_in, int r, int nnz_norm, int z_vec, int NR, int ZS)
{
    extern __shared__ f32x4 p2_lds[];   // slab [QW][JP], then the thread groups' sums [NG][NE] (few-element slabs only) and, after them, rows of Z [NR][ZS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, q4 = lane >> 4;
    const int mg = blockIdx.x;
    if (mg * QW >= MQ) return;   // (padding of the grid)
    const int og = blockIdx.y, set = og / K2, o = og - set * K2;
    const int NE = QW * JP;
    const size_t tile = (size_t)K2 * MQ * JP;   // 16-byte elements of one partial tile
    const f32x4 *base = part + (size_t)set * S * tile + ((size_t)o * MQ + (size_t)mg * QW) * JP;
    const int NG = NE >= kP2Threads ? 1 : kP2Threads / NE;
    f32x4 *red = p2_lds + NE;
    float *zs = reinterpret_cast<float *>(red);   // (the groups' sums are dead by then)
    const int r4 = (r + 3) >> 2;   // 16-byte elements of a row of Z

    // ---- rows n0 .. n0 + NR - 1 of Z -> registers -> LDS; entries past C_in or r are zero
    f32x4 zr[4];
    auto load_z = [&](int n0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = q * kP2Threads + tid;
            const int row = e / r4, j = (e - row * r4) * 4;
            const int n = n0 + row;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (row < NR && n < C_in) {
                const float *src = Z + (size_t)n * r + j;
                if (z_vec && j + 3 < r) {
                    v = *reinterpret_cast<const f32x4 *>(src);
                } else {
                    if (j < r) v[0] = src[0];
                    if (j + 1 < r) v[1] = src[1];
                    if (j + 2 < r) v[2] = src[2];
                    if (j + 3 < r) v[3] = src[3];
                }
            }
            zr[q] = v;
        }
    };
    auto store_z = [&]() {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = q * kP2Threads + tid;
            const int row = e / r4, j = (e - row * r4) * 4;
            if (row < NR) *reinterpret_cast<f32x4 *>(zs + row * ZS + j) = zr[q];
        }
    };
    load_z(0);   // in flight while the partial tiles are summed

    const bool once = (S + NG - 1) / NG <= 16;   // every thread's tiles fit one trip
    if (NG == 1) {
        for (int e = tid; e < NE; e += kP2Threads)
            p2_lds[e] = once ? once_sum<16>(base + e, 0, 1, S, tile) : chain_sum<8>(base + e, 0, 1, S, tile);
    } else {
        const int gi = tid / NE, e = tid - gi * NE;
        if (gi < NG) red[gi * NE + e] = once ? once_sum<16>(base + e, gi, NG, S, tile) : chain_sum<8>(base + e, gi, NG, S, tile);
        __syncthreads();
        if (tid < NE) {
            f32x4 t = red[tid];
            for (int q = 1; q < NG; ++q) t += red[q * NE + tid];
            p2_lds[tid] = t;
        }
        __syncthreads();   // the rows of Z go where the groups' sums were
    }
    store_z();
    __syncthreads();
    const float *slab = reinterpret_cast<const float *>(p2_lds);   // [QW][JP][4]

    const bool a_on = l16 < 4 * QW;                                       // A operand: output channel l16 of the group
    const int arow = ((a_on ? l16 >> 2 : 0) * JP) * 4 + (l16 & 3);
    for (int n0 = 0; n0 < C_in; n0 += NR) {
        if (n0 > 0) {
            load_z(n0);
            __syncthreads();   // every wave is done with the rows before
            store_z();
            __syncthreads();
        }
        for (int t = wave; t * 16 < NR && n0 + t * 16 < C_in; t += kP2Threads / 64) {
            const float *zrow = zs + (t * 16 + l16) * ZS;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            int cnt = 0;
            for (int jc = 0; jc < r; jc += 64) {
                float at[16], bz[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int j = jc + 4 * k + q4;
                    at[k] = (a_on && j < JP) ? slab[arow + j * 4] : 0.f;
                    bz[k] = j < 4 * r4 ? zrow[j] : 0.f;
                }
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(at[k], bz[k], acc, 0, 0, 0);
                    cnt += bz[k] != 0.0f ? 1 : 0;
                }
            }
            // D tile: lane (n, g) holds output channels 4g .. 4g+3 of the group for input channel n
            const int n = n0 + t * 16 + l16;
            float inv_r = 1.0f / (float)r;
            if (nnz_norm) {   // non-zero entries of row n: the four lanes that share l16 hold a quarter of the row each
                int c = cnt;
                c += __shfl_xor(c, 16);
                c += __shfl_xor(c, 32);
                inv_r = c > 0 ? 1.0f / (float)c : 0.0f;
            }
            if (n < C_in && q4 < QW) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = 4 * (mg * QW + q4) + v;
                    if (m < C_out) dW[((size_t)m * C_in + n) * K2T + og] = acc[v] * inv_r;
                }
            }
        }
    }
}

// Exact path: dW[m,n,o] = T[o,n,m] (a transpose of the reduced tile).
__global__ __launch_bounds__(kThreads) void untile_kernel(const float *__restrict__ T, float *__restrict__ dW, int K2, int JP,
                                                          int MP, int C_out, int C_in)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long total = (long long)C_out * C_in * K2;
    if (i >= total) return;
    const int o = (int)(i % K2);
    const long long mn = i / K2;
    const int n = (int)(mn % C_in), m = (int)(mn / C_in);
    dW[i] = T[tile_index(o, n, m, JP, MP)];
}

// dY planes whose size is not a whole number of 16-byte vectors are copied once into planes
// of pitch `pitch` elements (zero tail), so that the correlation kernel only ever issues
// aligned vector loads.
template <typename T>
__global__ __launch_bounds__(kThreads) void repack_planes_kernel(const T *__restrict__ src, T *__restrict__ dst, long long nplanes,
                                                                 int n, int pitch)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nplanes * pitch) return;
    const long long pl = i / pitch;
    const int e = (int)(i - pl * pitch);
    dst[i] = e < n ? src[pl * n + e] : T(0);
}

hipError_t launch_repack_planes(int dtype, const void *src, void *dst, long long nplanes, int n, int pitch, hipStream_t st)
{
    const long long total = nplanes * pitch;
    dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    if (dtype == XCONV_F32)
        hipLaunchKernelGGL(repack_planes_kernel<float>, grid, dim3(kThreads), 0, st, static_cast<const float *>(src),
                           static_cast<float *>(dst), nplanes, n, pitch);
    else
        hipLaunchKernelGGL(repack_planes_kernel<uint16_t>, grid, dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                           static_cast<uint16_t *>(dst), nplanes, n, pitch);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// host: launch plan
// ---------------------------------------------------------------------------
static int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

static const size_t kLdsLimit = 160 * 1024;


static void fill_geometry(CorrParams &P, int dtype, int RB, int CW)
{
    const bool f32 = dtype == XCONV_F32;
    const int EPV = f32 ? 4 : 8;
    P.RB = RB;
    P.CW = CW;
    P.CWp = round_up(CW, 4);
    P.NSTRIP = ceil_div(P.Wo, CW);
    P.NBAND = ceil_div(P.Ho, RB);
    P.NR = (RB - 1) * P.sh + P.kH;
    P.NOLD = P.kH > P.sh ? P.kH - P.sh : 0;
    P.NNEW = P.NR - P.NOLD;
    P.BWc = (P.CWp - 1) * P.sw + P.kW;
    // vector chunks of EPV pixels that can intersect a row segment of CWp slots,
    // over all alignments of the segment start (periodic in the row and strip index)
    int nch = 1;
    for (int oy = 0; oy < P.Ho && oy < 8; ++oy)
        for (int s = 0; s < P.NSTRIP && s < 8; ++s) {
            const int f0 = oy * P.Wo + s * CW;
            const int need = ceil_div(f0 % EPV + P.CWp, EPV);
            if (need > nch) nch = need;
        }
    P.NCHR = nch;
    P.AL = (P.Wo % EPV == 0 && CW % EPV == 0) ? 1 : 0;
    if (f32) {
        // dY tile [m][slot]: row stride = 4 mod 64 floats, so that the 16 rows x 4 slots of a
        // fragment read fall into 64 different banks; A tile [col][j]: column stride = 16 mod 64
        const int ps = RB * P.CWp;
        P.ASTR = ps + (68 - ps % 64) % 64;
        P.BSTR = P.J_WG + (80 - P.J_WG % 64) % 64;
        P.a_units = round_up(P.M_WG * P.ASTR, 4);
    } else {
        P.ASTR = P.M_WG + 1;
        P.BSTR = P.J_WG + 1;
        P.a_units = RB * P.CWp * P.ASTR;
    }
    P.b_units = P.NR * P.BWc * P.BSTR;
    P.NS = P.NBG * P.NSTRIP * P.NBAND;
}

static size_t lds_bytes_of(const CorrParams &P, int dtype, int MT)
{
    const size_t unit = dtype == XCONV_F32 ? 4 : 16;
    const size_t stage = ((size_t)P.a_units + P.b_units) * unit;
    const size_t red = P.WK > 1 ? (size_t)P.WM * P.WJ * MT * kMaxOff * 64 * 16 : 0;
    return stage > red ? stage : red;
}

// output-channel tiles (of 16) per wave: fp32 keeps the accumulator file small enough for two workgroups per CU
static int corr_mt(int dtype, int C_out)
{
    return C_out <= 16 ? 1 : (dtype == XCONV_F32 ? 2 : 4);
}

static bool geometry_fits(const CorrParams &P, int dtype, int MT)
{
    const bool f32 = dtype == XCONV_F32;
    const int EPV = f32 ? 4 : 8;
    const int na_max = f32 ? 8 : 2, nb_max = f32 ? 4 : 2;
    if (lds_bytes_of(P, dtype, MT) > kLdsLimit) return false;
    if (P.RB * P.M_WG * P.NCHR > kThreads * na_max) return false;
    if (P.NNEW * P.BWc * (P.J_WG / EPV) > kThreads * nb_max) return false;
    if (P.NCHR > 255 || P.BWc > 65535 || P.M_WG > 16383 || P.RB > 255) return false;
    return true;
}

bool plan_corr(CorrParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw,
               int CS, bool dy_aligned)
{
    const bool f32 = dtype == XCONV_F32;
    const int BI = f32 ? 1 : 8, EPV = f32 ? 4 : 8;
    P.B = B; P.C_out = C_out; P.H = H; P.W = W;
    P.kH = kH; P.kW = kW; P.sh = sh; P.sw = sw; P.ph = ph; P.pw = pw;
    P.Ho = (H + 2 * ph - kH) / sh + 1;
    P.Wo = (W + 2 * pw - kW) / sw + 1;
    P.CS = CS;
    P.NBG = ceil_div(B, BI);
    P.K2 = kH * kW;
    P.NOG = ceil_div(P.K2, P.K2 == 1 ? 1 : kMaxOff);
    P.dy_plane = round_up(P.Ho * P.Wo, EPV);  // the kernel reads dY planes of this pitch (repacked by the caller if needed)
    (void)dy_aligned;

    // the kernel addresses a batch group (BI images) with 32-bit byte offsets
    const long long es = f32 ? 4 : 2;
    if ((long long)BI * C_out * round_up(P.Ho * P.Wo, EPV) * es > (1LL << 30) || (long long)BI * H * W * CS * es > (1LL << 30)) return false;

    const int MT = corr_mt(dtype, C_out);
    const int nwm = ceil_div(C_out, 16 * MT), nwj = CS / 16;
    // waves along the A columns share dY through LDS, so prefer them; WJ must divide the column tiles
    int WJ = env_int("XCONV_CORR_WJ", 0);
    if (WJ != 1 && WJ != 2 && WJ != 4) WJ = (nwj % 4 == 0) ? 4 : (nwj % 2 == 0) ? 2 : 1;
    if (nwj % WJ != 0) WJ = 1;
    int WM = env_int("XCONV_CORR_WM", 0);
    if (WM != 1 && WM != 2 && WM != 4) WM = nwm >= 4 ? 4 : nwm >= 2 ? 2 : 1;
    while (WM * WJ > 4) WM >>= 1;
    P.WM = WM; P.WJ = WJ; P.WK = 4 / (WM * WJ);
    P.M_WG = WM * MT * 16;
    P.J_WG = WJ * 16;
    P.NTM = ceil_div(C_out, P.M_WG);
    P.NTJ = CS / P.J_WG;
    P.MP = P.NTM * P.M_WG;
    P.JP = CS;

    // Step shape: the widest strip that fits, then the tallest band under the slot cap.
    const int slots_cap = env_int("XCONV_CORR_SLOTS", f32 ? 128 : 64);
    int bestRB = env_int("XCONV_CORR_RB", 0), bestCW = env_int("XCONV_CORR_CW", 0);
    if (bestRB <= 0 || bestCW <= 0) {
        bestRB = bestCW = 0;
        int prevCW = -1;
        for (int nstrip = 1; nstrip <= P.Wo && bestRB == 0; nstrip = nstrip < 4 ? nstrip + 1 : nstrip + nstrip / 2) {
            int CW = nstrip == 1 ? P.Wo : round_up(ceil_div(P.Wo, nstrip), 4);
            if (CW > P.Wo) CW = P.Wo;
            if (CW == prevCW) continue;
            prevCW = CW;
            if (round_up(CW, 4) > slots_cap && CW > 4) continue;
            long long best_score = -1;
            for (int RB = 1; RB <= P.Ho && RB <= 32; ++RB) {
                fill_geometry(P, dtype, RB, CW);
                if (RB > 1 && RB * P.CWp > slots_cap) break;
                if (!geometry_fits(P, dtype, MT)) break;
                const long long useful = (long long)P.Ho * P.Wo;
                const long long padded = (long long)P.NBAND * RB * P.NSTRIP * P.CWp;
                const long long score = (long long)RB * P.CWp * 1000 * useful / padded;
                if (score > best_score) { best_score = score; bestRB = RB; bestCW = CW; }
            }
        }
        if (bestRB == 0) {  // last resort: one row, four columns
            bestRB = 1;
            bestCW = P.Wo < 4 ? P.Wo : 4;
        }
    }
    fill_geometry(P, dtype, bestRB, bestCW);
    if (!geometry_fits(P, dtype, MT)) return false;

    // K-split: fill the 256 compute units (two workgroups each when LDS allows)
    const size_t lds = lds_bytes_of(P, dtype, MT);
    const int per_cu = env_int("XCONV_CORR_WGS_PER_CU", lds <= 72 * 1024 ? 2 : 1);
    const int ny = P.NTM * P.NTJ * P.NOG;
    int target = env_int("XCONV_CORR_SPLITS", 0);
    if (target <= 0) {
        target = (256 * per_cu) / ny;
        if (target < 1) target = 1;
        if (target > P.NS) target = P.NS;
        // prefer a split count that divides the steps evenly
        int bestS = target;
        double best_eff = 0.0;
        for (int S = target; S >= 1 && S >= target * 3 / 4; --S) {
            const double eff = (double)P.NS / ((double)S * ceil_div(P.NS, S)) * ((double)S / target);
            if (eff > best_eff - 1e-9) { best_eff = eff > best_eff ? eff : best_eff; bestS = S; }   // (ties go to the smaller count: as many steps per workgroup, fewer partial tiles)
        }
        target = bestS;
    }
    if (target > P.NS) target = P.NS;
    if (target < 1) target = 1;
    P.S = target;
    return true;
}

size_t corr_lds_bytes(int dtype, const CorrParams &P) { return lds_bytes_of(P, dtype, corr_mt(dtype, P.C_out)); }

size_t corr_partial_bytes(const CorrParams &P)
{
    // S partial buffers followed by the reduced buffer T, each [K2, JP, MP] fp32
    return ((size_t)P.S + 1) * P.K2 * P.JP * P.MP * sizeof(float);
}

template <int DT, int MT, int NA, int NB, int NOFF, bool AL>
static hipError_t launch_corr_cfg(const CorrParams &P, size_t lds, hipStream_t st)
{
    if (lds > 64 * 1024) {
        static bool done = false;  // per instantiation: the attribute sticks to the function
        static size_t done_bytes = 0;
        if (!done || lds > done_bytes) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(corr_kernel<DT, MT, NA, NB, NOFF, AL>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
            if (e != hipSuccess) return e;
            done = true;
            done_bytes = kLdsLimit;
        }
    }
    CorrParams Q = P;
    Q.SQ = P.NS / P.S;
    Q.SR = P.NS % P.S;
    hipLaunchKernelGGL((corr_kernel<DT, MT, NA, NB, NOFF, AL>), dim3(P.S, P.NTM * P.NTJ, P.NOG), dim3(kThreads), lds, st, Q);
    return hipGetLastError();
}

template <int DT, int MT, int NA, int NB> static hipError_t launch_corr_noff(const CorrParams &P, size_t lds, hipStream_t st)
{
    if (P.AL) {
        if (P.K2 == 1) return launch_corr_cfg<DT, MT, NA, NB, 1, true>(P, lds, st);
        return launch_corr_cfg<DT, MT, NA, NB, kMaxOff, true>(P, lds, st);
    }
    if (P.K2 == 1) return launch_corr_cfg<DT, MT, NA, NB, 1, false>(P, lds, st);
    return launch_corr_cfg<DT, MT, NA, NB, kMaxOff, false>(P, lds, st);
}

template <int DT, int MT> static hipError_t launch_corr_16(const CorrParams &P, size_t lds, hipStream_t st)
{
    const int na = ceil_div(P.RB * P.M_WG * P.NCHR, kThreads), nb = ceil_div(P.NNEW * P.BWc * (P.J_WG / 8), kThreads);
    if (na <= 1 && nb <= 1) return launch_corr_noff<DT, MT, 1, 1>(P, lds, st);
    if (na <= 1) return launch_corr_noff<DT, MT, 1, 2>(P, lds, st);
    if (nb <= 1) return launch_corr_noff<DT, MT, 2, 1>(P, lds, st);
    return launch_corr_noff<DT, MT, 2, 2>(P, lds, st);
}

hipError_t launch_corr(int dtype, const CorrParams &P, hipStream_t st)
{
    const int MT = corr_mt(dtype, P.C_out);
    const size_t lds = lds_bytes_of(P, dtype, MT);
    if (dtype == XCONV_F32) {
        if (MT == 2) return launch_corr_noff<XCONV_F32, 2, 8, 4>(P, lds, st);
        return launch_corr_noff<XCONV_F32, 1, 8, 4>(P, lds, st);
    }
    if (dtype == XCONV_BF16) {
        if (MT == 4) return launch_corr_16<XCONV_BF16, 4>(P, lds, st);
        return launch_corr_16<XCONV_BF16, 1>(P, lds, st);
    }
    if (MT == 4) return launch_corr_16<XCONV_F16, 4>(P, lds, st);
    return launch_corr_16<XCONV_F16, 1>(P, lds, st);
}

static float *reduced_tile(const CorrParams &P) { return P.part + (size_t)P.S * P.K2 * P.JP * P.MP; }

hipError_t launch_reduce(const CorrParams &P, hipStream_t st, float *Zout, int nz, int dist, uint64_t seed, float *T, int nsets)
{
    const int E4 = (int)(((size_t)P.K2 * P.JP * P.MP) / 4);
    const int zblocks = Zout ? ceil_div(nz, kThreads) : 0;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(zblocks + ceil_div(E4, 16), nsets), dim3(kThreads), 0, st,
                       reinterpret_cast<const f32x4 *>(P.part), reinterpret_cast<f32x4 *>(T ? T : reduced_tile(P)), P.S, E4, Zout, nz,
                       zblocks, dist, seed);
    return hipGetLastError();
}

// T[e] = sum_s part[s][e] for E4 float4 elements (the same fixed-order kernel, for other callers' partial sums);
// nsets such sums stored back to back
hipError_t launch_reduce_raw(const float *part, float *T, int S, int E4, hipStream_t st, int nsets)
{
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(ceil_div(E4, 16), nsets), dim3(kThreads), 0, st, reinterpret_cast<const f32x4 *>(part),
                       reinterpret_cast<f32x4 *>(T), S, E4, nullptr, 0, 0, 0, (uint64_t)0);
    return hipGetLastError();
}

// Quads of output channels per workgroup of pass2_mfma_kernel: as many (of 4, 2, 1) as still leave half of the compute
// units a workgroup (a workgroup reads the whole of Z; a compute unit holds one workgroup of 16 waves at a time)
static int pass2_quads(int MQ, int K2T)
{
    for (int q = 4; q > 1; q >>= 1)
        if (MQ % q == 0 && (long long)K2T * (MQ / q) >= 128) return q;
    return 1;
}

bool reduce_expand_fused(const CorrParams &P, bool have_z, bool exact, int C_in, int r, int dist, int nsets)
{
    const int mode = env_int("XCONV_FUSED_PASS2", -1);   // tests: 0 takes the two-launch route (launch_reduce, launch_expand)
    if (mode == 0) return false;
    if (P.MP % 4 != 0) return false;
    if (!exact && P.JP > 1024) return false;   // (the slab of all probe columns sits in LDS)
    if (mode == 1) return true;
    // One round of workgroups: a compute unit turns memory requests around at a limited rate, so with more workgroups
    // than compute units the busiest unit sets the time and the two launches, whose many small workgroups spread
    // evenly, win (measured on 576 workgroups: 25 us against 19 us).
    const int MQ = P.MP / 4, K2T = nsets * P.K2;
    return (long long)K2T * (MQ / (exact ? 1 : pass2_quads(MQ, K2T))) <= 256;
}

hipError_t launch_reduce_expand(const CorrParams &P, const float *Z, bool exact, float *dW, int C_in, int r, bool nnz_norm, int dist,
                                uint64_t seed, int nsets, hipStream_t st)
{
    const int MQ = P.MP / 4;
    const int K2T = nsets * P.K2;
    const f32x4 *part = reinterpret_cast<const f32x4 *>(P.part);
    if (exact) {
        // slab of JC input channels x 4 output channels per workgroup: chunks of at most 256 input channels that
        // divide the padded channel count (a multiple of 16)
        int JC = P.JP < 256 ? P.JP : 256;
        for (; P.JP % JC != 0; JC -= 16) {}
        const int NE = JC;
        const int NG = NE >= kThreads ? 1 : kThreads / NE;
        const size_t lds = (size_t)NE * 16 + (NG > 1 ? (size_t)NG * NE * 16 : 0);
        const dim3 grid((unsigned)round_up(MQ, 8), (unsigned)K2T, (unsigned)(P.JP / JC));
        hipLaunchKernelGGL(pass2_exact_kernel, grid, dim3(kThreads), lds, st, part, dW, P.S, P.K2, K2T, P.JP, MQ, JC, P.C_out, C_in);
    } else {
        int QW = env_int("XCONV_PASS2_QW", pass2_quads(MQ, K2T));
        if ((QW != 1 && QW != 2 && QW != 4) || MQ % QW != 0) QW = 1;
        const int r4 = ceil_div(r, 4);
        const int ZS = 4 * (r4 + (r4 % 2 == 0 ? 1 : 2));         // words per staged row of Z: 4 * odd
        int NR = (4 * kP2Threads / r4) & ~15;                      // rows per block: 4 x 16 bytes per thread
        if (NR > round_up(C_in, 16)) NR = round_up(C_in, 16);
        const int NE = QW * P.JP, NG = NE >= kP2Threads ? 1 : kP2Threads / NE;
        const size_t red = NG > 1 ? (size_t)NG * NE * 16 : 0, zs = (size_t)NR * ZS * sizeof(float);
        const size_t lds = (size_t)NE * 16 + (red > zs ? red : zs);
        // rows of Z are read 16 bytes at a time where every row starts on such a boundary
        const int z_vec = (r % 4 == 0 && (reinterpret_cast<uintptr_t>(Z) & 15u) == 0) ? 1 : 0;
        const dim3 grid((unsigned)round_up(MQ / QW, 8), (unsigned)K2T);
#define XC_P2M(Q)                                                                                                        \
    {                                                                                                                    \
        static bool done = false;                                                                                        \
        if (!done) {                                                                                                     \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pass2_mfma_kernel<Q>),                      \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);                  \
            if (e != hipSuccess) return e;                                                                               \
            done = true;                                                                                                 \
        }                                                                                                                \
        hipLaunchKernelGGL(pass2_mfma_kernel<Q>, grid, dim3(kP2Threads), lds, st, part, Z, dW, P.S, P.K2, K2T, P.JP, MQ, \
                           P.C_out, C_in, r, nnz_norm ? 1 : 0, z_vec, NR, ZS);                                           \
    }
        if (QW == 4) XC_P2M(4) else if (QW == 2) XC_P2M(2) else XC_P2M(1)
#undef XC_P2M
    }
    return hipGetLastError();
}

hipError_t launch_expand(const CorrParams &P, const float *Z, float *dW, int C_in, int r, hipStream_t st, bool nnz_norm,
                         const float *Tin, int K2in)
{
    const int nn = nnz_norm ? 1 : 0;
    const int K2 = K2in > 0 ? K2in : P.K2;
    const float *T = Tin ? Tin : reduced_tile(P);
    if (Z) {
        // few tiles: split the offsets over more waves; many tiles: a lane writes whole runs of offsets
        const int NTM16 = ceil_div(P.C_out, 16), NTN = ceil_div(C_in, 16);
        const long long tiles = (long long)NTM16 * NTN;
        int og = K2 == 1 ? 1 : (tiles * ceil_div(K2, 9) >= 2048 ? 9 : (tiles * ceil_div(K2, 3) >= 512 ? 3 : 1));
        og = env_int("XCONV_EXPAND_OG", og);
        const dim3 grid((unsigned)tiles, (unsigned)ceil_div(K2, og));
        if (og == 9)
            hipLaunchKernelGGL(expand_kernel<9>, grid, dim3(64), 0, st, T, Z, dW, K2, P.JP, P.MP, P.C_out, C_in, r, NTN, nn);
        else if (og == 3)
            hipLaunchKernelGGL(expand_kernel<3>, grid, dim3(64), 0, st, T, Z, dW, K2, P.JP, P.MP, P.C_out, C_in, r, NTN, nn);
        else
            hipLaunchKernelGGL(expand_kernel<1>, dim3((unsigned)tiles, (unsigned)K2), dim3(64), 0, st, T, Z, dW, K2, P.JP, P.MP,
                               P.C_out, C_in, r, NTN, nn);
    } else {
        const long long total = (long long)P.C_out * C_in * K2;
        hipLaunchKernelGGL(untile_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, T, dW, K2,
                           P.JP, P.MP, P.C_out, C_in);
    }
    return hipGetLastError();
}

}  // namespace xc
