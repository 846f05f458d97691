// Offset-wise correlation (Algorithm 1, backward step 3 with the shift of step 4) for 16-bit
// storage, 3x3 kernels at unit stride and output rows that one workgroup sweeps whole:
//
//   G[m,j,ky,kx] = sum_{b,oy,ox} dY[b,m,oy,ox] * A[b, oy+ky-ph, ox+kx-pw, j]
//
// Same roles and LDS unit form as corr_ws_kernel (corr_ws_kernels.hip): one 16-byte unit holds the
// 8 images of one (pixel, channel); waves 0-3 (consumers) read fragments and issue
// v_mfma_f32_32x32x16, waves 4-7 (producers) bring dY and A from global memory, transpose 8x8
// blocks in registers and write units.  What differs is the walk through a row:
//
//   * The two lane groups of the matrix instruction (its reduction index is 8 images x 2 pixel
//     slots) sweep the two halves of an output row: at k-step q group g is at column g*Qr + q,
//     Qr = W'/2.  The fragments of A for kernel column kx at k-step q are those of column 0 at
//     k-step q + kx, so a window of three fragments per kernel row slides along the whole row:
//     Qr - 1 k-steps request 1 + 3 fragments and only the last one of the row, which moves the
//     window to the next row, requests 1 + 9.  A row may be cut into two sub-steps (two dY tiles
//     in LDS, one barrier each); the window does not notice.
//   * dY of a whole row is requested at once, the pieces of one (image, channel) row by
//     neighbouring lanes: the memory pipeline sends one request per cache line, and the rate of
//     such requests (at most 64 outstanding per compute unit) is what bounds the producers.
//     The lanes that hold the second sub-step's pieces keep them, already transposed, until
//     that sub-step's tile is written.
//   * The dY fragment alternates between three register sets with the window position, so no
//     k-step copies a fragment into registers that matrix instructions in flight still read.
#include <type_traits>

#include "common.h"
#include "launch.h"
#include "ws_pos.h"

// Timing experiments only (never defined in the shipped build): bit 0 consumers issue no MFMA, bit 1 no
// fragment reads, bit 3 producers issue no global loads, bit 4 no LDS writes or transposes, bit 5 the first
// consumer wave and the first producer thread leave time stamps in the partial tile.
#ifndef XCONV_ROW_DBG
#define XCONV_ROW_DBG 0
#endif
// wave priorities of the two roles (measured on C5: consumers above producers and equal priorities give the same loop,
// producers above consumers a loop 18 % longer)
#ifndef XCONV_ROW_CPRIO
#define XCONV_ROW_CPRIO 3
#endif
#ifndef XCONV_ROW_PPRIO
#define XCONV_ROW_PPRIO 0
#endif
// wave priorities of the two roles
#ifndef XCONV_ROW_CPRIO
#define XCONV_ROW_CPRIO 3
#endif
#ifndef XCONV_ROW_PPRIO
#define XCONV_ROW_PPRIO 0
#endif

namespace xc {

namespace {

typedef float f32x16r __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4r __attribute__((ext_vector_type(4)));
typedef int i32x4r __attribute__((ext_vector_type(4)));

template <int DT> __device__ inline f32x16r mfma32r(const u32x4r &a, const u32x4r &b, f32x16r c)
{
    if constexpr (DT == XCONV_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <int N> using IC = std::integral_constant<int, N>;

}  // namespace

// REM = (Qr - 1) % 3: window position at which the last k-step of a row starts.
// CB  = bytes of one staged column of A (BSTR * 16): the three columns of the window are immediates.
template <int DT, int REM, int CB>
__global__ __launch_bounds__(kWsThreads) void corr_row_kernel(const WsParams P)
{
    draw_z_slice(P.zout, P.nz, P.zdist, P.zseed);
    extern __shared__ uint4 row_lds[];
    uint4 *lds_a = row_lds;                    // two dY tiles [lane group][slot][M_WG]
    uint4 *lds_b = row_lds + 2 * P.a_units;    // ring of A rows [slot][column][BSTR]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned long long ts_[8];
    if constexpr (XCONV_ROW_DBG & 32) { ts_[0] = __builtin_amdgcn_s_memrealtime(); ts_[1] = __builtin_readcyclecounter(); }
    int tm, tj;
    fast_divmod((int)blockIdx.y, P.NTM, frcp(P.NTM), tj, tm);
    const int m0 = tm * P.M_WG;
    const int jb = tj * P.J_WG;

    const int bx = xcd_block(blockIdx.x, gridDim.x);   // K-split of this workgroup: neighbouring splits on one die (C5: no change)
    const int t_begin = bx * P.SQ + (bx < P.SR ? bx : P.SR);
    const int t_end = t_begin + P.SQ + (bx < P.SR ? 1 : 0);
    const int NI = (t_end - t_begin) * P.NSUB;  // sub-steps of this workgroup
    const int Qr = P.Wo >> 1;                   // k-steps of a row
    const int Q0 = P.CWs >> 1;                  // k-steps of the first sub-step of a row
    const int Q1 = Qr - Q0;                     // ... of the second one (0 when NSUB == 1)
    const int rotmul = 8 >> __builtin_ctz((unsigned)P.WJ);  // see corr_ws_kernel: rotation between the column groups of a pixel

    if (wave < 4) {
        // =========================== consumers ===========================
        __builtin_amdgcn_s_setprio(XCONV_ROW_CPRIO);
        const int l32 = lane & 31, g = lane >> 5;
        const int wm = wave & (P.WM - 1), wj = wave >> __builtin_ctz((unsigned)P.WM);
        const int G = 2 * wj + (l32 >> 4);  // 16-column group of this lane's column

        f32x16r acc[9];
#pragma unroll
        for (int o = 0; o < 9; ++o)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[o][e] = 0.f;

        if (NI > 0) {
            WsPos pc = ws_pos_of(P, t_begin);
            const uint32_t lds0 = __builtin_amdgcn_groupstaticsize();
            const uint32_t a_wave = lds0 + (uint32_t)(wm * 32 + l32) * 16u;
            // column 0 of this lane group's half of the row, in ring slot 0
            const uint32_t b_wave = lds0 + (uint32_t)(2 * P.a_units + G * 16 + (((l32 & 15) + wj * rotmul) & 15) + g * Qr * P.BSTR) * 16u;
            const uint32_t step_a = (uint32_t)P.M_WG * 16u;  // one pixel slot per k-step
            // first slot of this lane group in dY tile `buf` of a sub-step of Qu k-steps
            auto a_addr = [&](int buf, int Qu) { return a_wave + (uint32_t)(buf * P.a_units + g * Qu * P.M_WG) * 16u; };
            // window column 0 of kernel row ky for the row-step at ring position rowmod
            auto b_addr = [&](int rowmod, int ky) {
                int slot = rowmod + ky;
                slot = slot >= P.NRING ? slot - P.NRING : slot;
                return b_wave + (uint32_t)__builtin_amdgcn_readfirstlane(slot * P.b_row_units) * 16u;
            };
            auto lds_read = [](u32x4r &dst, uint32_t addr, auto off) {
                if constexpr (XCONV_ROW_DBG & 2) return;
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(decltype(off)::value) : "memory");
            };
            // requests return in order: at most N younger ones may be in flight behind x, y, z
            auto arrived3 = [](auto nc, u32x4r &x, u32x4r &y, u32x4r &z) {
                asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(x), "+v"(y), "+v"(z) : "n"(decltype(nc)::value) : "memory");
            };
            auto arrived1 = [](auto nc, u32x4r &x) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(decltype(nc)::value) : "memory"); };

            u32x4r af[3], b[9];   // af[ph]: dY fragment of a k-step at window position ph; b[3*ky + w]: window register w of kernel row ky
            uint32_t pa, pb3[3];
            auto mma = [&](auto phc, auto oc, const u32x4r &bf) {
                constexpr int o = decltype(oc)::value;
                if constexpr (XCONV_ROW_DBG & 1) return;
                acc[o] = mfma32r<DT>(af[decltype(phc)::value], bf, acc[o]);
            };

            pa = a_addr(0, Q0);
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) pb3[ky] = b_addr(pc.rowmod, ky);
            ws_barrier();  // the first dY tile and the rows of the first row-step are in LDS
            if constexpr (XCONV_ROW_DBG & 32) { ts_[2] = __builtin_amdgcn_s_memrealtime(); ts_[3] = __builtin_readcyclecounter(); }
            lds_read(af[0], pa, IC<0>{});
            ws_static_for<0, 9>([&](auto oc) {   // window register w <- column w, kernel rows inside
                constexpr int o = decltype(oc)::value;
                lds_read(b[3 * (o % 3) + o / 3], pb3[o % 3], IC<(o / 3) * CB>{});
            });
            arrived1(IC<9>{}, af[0]);
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) pb3[ky] += 3u * CB;   // the column that k-step 0 requests

            // One k-step at window position ph: window register (ph + kx) % 3 holds the column of
            // kernel column kx.  It requests the dY fragment of the next k-step (at pa) into the
            // next register set and the column three ahead into the registers whose last use was
            // issued an MFMA earlier.  In flight at the start: the three requests of the k-step
            // before, or the nine of a window refill; counted from the youngest, what a kernel
            // column needs is followed by at most 7 / 6 / 4 requests.
            auto inner = [&](auto phc) {
                constexpr int w0 = decltype(phc)::value, w1 = (w0 + 1) % 3, w2 = (w0 + 2) % 3;
                __builtin_amdgcn_sched_barrier(0);
                lds_read(af[w1], pa, IC<0>{});
                arrived3(IC<7>{}, b[w0], b[3 + w0], b[6 + w0]);
                mma(phc, IC<0>{}, b[w0]);
                mma(phc, IC<3>{}, b[3 + w0]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[w0], pb3[0], IC<0>{});
                __builtin_amdgcn_sched_barrier(0);
                mma(phc, IC<6>{}, b[6 + w0]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[3 + w0], pb3[1], IC<0>{});
                __builtin_amdgcn_sched_barrier(0);
                arrived3(IC<6>{}, b[w1], b[3 + w1], b[6 + w1]);
                mma(phc, IC<1>{}, b[w1]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[6 + w0], pb3[2], IC<0>{});
                __builtin_amdgcn_sched_barrier(0);
                mma(phc, IC<4>{}, b[3 + w1]);
                mma(phc, IC<7>{}, b[6 + w1]);
                __builtin_amdgcn_sched_barrier(0);
                arrived3(IC<4>{}, b[w2], b[3 + w2], b[6 + w2]);
                mma(phc, IC<2>{}, b[w2]);
                mma(phc, IC<5>{}, b[3 + w2]);
                mma(phc, IC<8>{}, b[6 + w2]);
                __builtin_amdgcn_sched_barrier(0);
                arrived1(IC<3>{}, af[w1]);
                __builtin_amdgcn_sched_barrier(0);
            };
            // The last k-step of a row, entered at window position REM: it multiplies the window
            // registers in the order 0, 1, 2 (register w holds kernel column (w - REM) mod 3) and
            // refills each, right after the MFMAs that read it, with column w of the next row-step
            // (pbn), so that the next row starts at position 0; the dY fragment of the next row's
            // first k-step (pa_n) goes to register set 0.
            auto cross = [&](uint32_t pa_n, const uint32_t (&pbn)[3]) {
                constexpr int k0 = (3 - REM) % 3, k1 = (4 - REM) % 3, k2 = (5 - REM) % 3;   // kernel column in window register 0, 1, 2
                constexpr int AN = REM == 0 ? 1 : 0;   // (at position 0 set 0 is in use: the fragment is moved there at the end)
                // The window register that the k-step before refilled (register (REM + 2) % 3, its requests are the
                // youngest but for the fragment just requested) must be waited for exactly; the others arrived long ago.
                constexpr int W0 = REM == 1 ? 1 : 7, W1 = REM == 2 ? 3 : 6;
                using PH = IC<REM>;
                __builtin_amdgcn_sched_barrier(0);
                lds_read(af[AN], pa_n, IC<0>{});
                arrived3(IC<W0>{}, b[0], b[3], b[6]);
                mma(PH{}, IC<k0>{}, b[0]);
                mma(PH{}, IC<3 + k0>{}, b[3]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[0], pbn[0], IC<0>{});
                __builtin_amdgcn_sched_barrier(0);
                mma(PH{}, IC<6 + k0>{}, b[6]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[3], pbn[1], IC<0>{});
                __builtin_amdgcn_sched_barrier(0);
                arrived3(IC<W1>{}, b[1], b[4], b[7]);
                mma(PH{}, IC<k1>{}, b[1]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[6], pbn[2], IC<0>{});
                __builtin_amdgcn_sched_barrier(0);
                mma(PH{}, IC<3 + k1>{}, b[4]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[1], pbn[0], IC<CB>{});
                __builtin_amdgcn_sched_barrier(0);
                mma(PH{}, IC<6 + k1>{}, b[7]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[4], pbn[1], IC<CB>{});
                __builtin_amdgcn_sched_barrier(0);
                arrived3(IC<6>{}, b[2], b[5], b[8]);
                mma(PH{}, IC<k2>{}, b[2]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[7], pbn[2], IC<CB>{});
                __builtin_amdgcn_sched_barrier(0);
                mma(PH{}, IC<3 + k2>{}, b[5]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[2], pbn[0], IC<2 * CB>{});
                __builtin_amdgcn_sched_barrier(0);
                mma(PH{}, IC<6 + k2>{}, b[8]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[5], pbn[1], IC<2 * CB>{});
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[8], pbn[2], IC<2 * CB>{});
                __builtin_amdgcn_sched_barrier(0);
                arrived1(IC<9>{}, af[AN]);
                if constexpr (REM == 0) af[0] = af[1];
                __builtin_amdgcn_sched_barrier(0);
            };

            // Before the last k-step of a sub-step the consumers no longer read that sub-step's dY
            // tile (its last fragment is in registers): they pass the barrier that hands the tile
            // back, and the fragment that k-step requests is the first one of the next tile.
            const int nrows = t_end - t_begin;
            int sub = 0;   // dY tile (row * NSUB + sub-step) being read
            uint32_t pbn[3];
            for (int row = 0; row < nrows; ++row) {
                // k-steps 0 .. Qr-2 of the row; the tile changes in front of k-step Q0 (two sub-steps)
                auto step = [&](int q, auto phc) {
                    if (P.NSUB == 2 && q == Q0 - 1) {
                        ws_barrier();
                        ++sub;
                        pa = a_addr(sub & 1, Q1);
                    } else {
                        pa += step_a;
                    }
                    inner(phc);
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pb3[ky] += (uint32_t)CB;
                };
                int q = 0;
                for (; q + 3 <= Qr - 1; q += 3) {
                    step(q, IC<0>{});
                    step(q + 1, IC<1>{});
                    step(q + 2, IC<2>{});
                }
                if constexpr (REM >= 1) step(q, IC<0>{});
                if constexpr (REM == 2) step(q + 1, IC<1>{});
                // the row's last k-step moves on to the next row-step
                uint32_t pa_n;
                if (row + 1 < nrows) {
                    WsPos pn = pc;
                    pn.u = P.NSUB - 1;
                    pn = ws_advance(P, pn);
                    if (pn.y == 0) ws_barrier();  // run boundary: the producers refill the whole ring first
                    ws_barrier();
                    ++sub;
                    pa_n = a_addr(sub & 1, Q0);
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pbn[ky] = b_addr(pn.rowmod, ky);
                    pc = pn;
                } else {
                    // after the very last row the requests repeat addresses of this one
                    pa_n = pa;
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pbn[ky] = b_addr(pc.rowmod, ky);
                }
                cross(pa_n, pbn);
                pa = pa_n;
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) pb3[ky] = pbn[ky] + 3u * CB;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        if constexpr (XCONV_ROW_DBG & 32) { ts_[4] = __builtin_amdgcn_s_memrealtime(); ts_[5] = __builtin_readcyclecounter(); }

        // D tile: lane (l32, g) holds column l32 and rows 8v + 4g .. 8v + 4g + 3 (v = 0..3)
        const int jcol = jb + wj * 32 + l32;
#pragma unroll
        for (int o = 0; o < 9; ++o) {
            float *dst = P.part + (size_t)bx * P.K2 * P.JP * P.MP + tile_index(o, jcol, m0 + wm * 32 + 4 * g, P.JP, P.MP);
#pragma unroll
            for (int v = 0; v < 4; ++v)   // rows 8v + 4g ..: two channel quads further on
                *reinterpret_cast<f32x4 *>(dst + (size_t)8 * v * P.JP) = f32x4{acc[o][4 * v], acc[o][4 * v + 1], acc[o][4 * v + 2], acc[o][4 * v + 3]};
        }
        if constexpr (XCONV_ROW_DBG & 32) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            ts_[6] = __builtin_amdgcn_s_memrealtime(); ts_[7] = __builtin_readcyclecounter();
            if (wave == 0 && lane == 0) {
                unsigned long long *d = reinterpret_cast<unsigned long long *>(P.part + (size_t)bx * P.K2 * P.JP * P.MP + tile_index(0, jb, m0, P.JP, P.MP));
                for (int q = 0; q < 8; ++q) d[q] = ts_[q];
                const unsigned long long *l = reinterpret_cast<const unsigned long long *>(row_lds + 2 * P.a_units + P.NRING * P.b_row_units);
                for (int q = 2; q < 7; ++q) d[8 + q] = l[q];   // cycle counter: producers' first loads issued .. first barrier passed
            }
        }
    } else {
        // =========================== producers ===========================
        __builtin_amdgcn_s_setprio(XCONV_ROW_PPRIO);
        const int p = tid - kProducers;
        const uint16_t *dY = static_cast<const uint16_t *>(P.dY);
        const uint16_t *Ag = static_cast<const uint16_t *>(P.A);
        const int HoWo = P.Ho * P.Wo;
        const uint32_t dy_plane_bytes = (uint32_t)HoWo * 2u;
        const uint32_t dy_img_bytes = (uint32_t)P.C_out * (uint32_t)HoWo * 2u;
        const uint32_t a_img_bytes = (uint32_t)P.H * (uint32_t)P.W * (uint32_t)P.CS * 2u;
        const int JC = P.J_WG >> 3;
        const int jc_shift = __builtin_ctz((unsigned)JC);  // J_WG is 32, 64 or 128

        // dY task of this thread: piece (lane group g, sub-step u) of the row of output channel m,
        // 8 columns (16 bytes) from column g*Qr + u*Q0 on.  The 2*NSUB pieces of a row sit in
        // neighbouring lanes and go out with one instruction per image.
        const int LPM = 2 * P.NSUB;
        int dm, didx;
        fast_divmod(p, LPM, frcp(LPM), dm, didx);
        const int dg = didx >= P.NSUB ? 1 : 0;
        const int du = didx - dg * P.NSUB;
        const bool d_on = dm < P.M_WG;
        const int dQu = du == 0 ? Q0 : Q1;          // columns of the piece that exist
        const uint32_t d_goff = (d_on && m0 + dm < P.C_out) ? (uint32_t)(m0 + dm) * dy_plane_bytes + (uint32_t)(dg * Qr + du * Q0) * 2u : kOOR;
        const int d_lds = dg * dQu * P.M_WG + dm;  // unit of the piece's first column inside a tile

        // A task of this thread: staged column c of the row a row-step adds, 8-column vector jc
        const int xjc = p & (JC - 1), xc = p >> jc_shift;
        const bool x_on = xc < P.BWc;
        const uint32_t x_goff = ((uint32_t)xc * (uint32_t)P.CS + (uint32_t)(jb + 8 * xjc)) * 2u;
        const int x_lds = xc * P.BSTR + 16 * (xjc >> 1);
        const int x_rot = ((xjc & 1) * 8 + (xjc >> 2) * rotmul) & 15;

        auto rsrc_of = [&](const uint16_t *base, int bg, uint32_t img_bytes, bool live) {
            bg = __builtin_amdgcn_readfirstlane(bg);
            int left = P.B - bg * 8;
            left = left < 8 ? left : 8;
            left = (live && left > 0) ? left : 0;
            const uint64_t addr = reinterpret_cast<uint64_t>(base + (size_t)bg * 8 * (img_bytes / 2));
            i32x4r r;
            r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
            r.y = __builtin_amdgcn_readfirstlane((int)(uint32_t)((addr >> 32) & 0xffffu));
            r.z = __builtin_amdgcn_readfirstlane((int)((uint32_t)left * img_bytes));
            r.w = 0x00020000;
            return r;
        };
        // loads are opaque to the compiler and waited for by hand (see corr_ws_kernel)
        auto buf16_async = [](u32x4r &dst, i32x4r r, uint32_t voff) {
            if constexpr (XCONV_ROW_DBG & 8) return;
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(r) : "memory");
        };
        auto wait8 = [](auto nc, u32x4r (&r)[8]) {
            asm volatile("s_waitcnt vmcnt(%8)"
                         : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                         : "n"(decltype(nc)::value)
                         : "memory");
        };
        // 8 images x 8 columns -> 8 units, in place
        auto transpose = [](u32x4r (&r)[8]) {
            if constexpr (XCONV_ROW_DBG & 16) return;
            uint32_t rows[8][4];
#pragma unroll
            for (int q = 0; q < 8; ++q) { rows[q][0] = r[q].x; rows[q][1] = r[q].y; rows[q][2] = r[q].z; rows[q][3] = r[q].w; }
            uint4 cols[8];
            transpose_rows8<4>(rows, cols);
#pragma unroll
            for (int q = 0; q < 8; ++q) r[q] = u32x4r{cols[q].x, cols[q].y, cols[q].z, cols[q].w};
        };

        // ---- dY of row-step ps -> registers (all pieces of the row at once)
        auto issue_dy = [&](const WsPos &ps, bool live, u32x4r (&r)[8]) {
            const i32x4r rs = rsrc_of(dY, ps.bg, dy_img_bytes, live);
            const uint32_t voff = d_goff != kOOR ? d_goff + (uint32_t)(ps.y * P.Wo) * 2u : kOOR;
#pragma unroll
            for (int img = 0; img < 8; ++img) buf16_async(r[img], rs, voff + (uint32_t)img * dy_img_bytes);
        };
        // ---- the row of A that row-step ps adds to the ring -> registers.  Nothing when the row-step
        // starts a run (a new group of images: its whole window is loaded by prime()).
        auto issue_xt = [&](const WsPos &ps, bool live, u32x4r (&r)[8]) {
            const bool on = live && ps.y > 0;
            const i32x4r rs = rsrc_of(Ag, ps.bg, a_img_bytes, on);
            const int iy = ps.y + P.kH - 1 - P.ph, ix = xc - P.pw;
            const bool in = x_on && (unsigned)iy < (unsigned)P.H && (unsigned)ix < (unsigned)P.W;
            // (the origin may lie in the padding: the sum wraps and is exact for every pixel inside the image)
            const uint32_t origin = (uint32_t)(iy * P.W - P.pw) * ((uint32_t)P.CS * 2u);
            const uint32_t voff = in ? origin + x_goff : kOOR;
#pragma unroll
            for (int img = 0; img < 8; ++img) buf16_async(r[img], rs, voff + (uint32_t)img * a_img_bytes);
        };
        // ---- the pieces of sub-step u of a row (transposed registers) -> dY tile `buf`
        auto write_dy = [&](int u, int buf, const u32x4r (&r)[8]) {
            if constexpr (XCONV_ROW_DBG & 16) return;
            if (d_on && du == u) {
                uint4 *dst = lds_a + buf * P.a_units + d_lds;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e < dQu) dst[e * P.M_WG] = uint4{r[e].x, r[e].y, r[e].z, r[e].w};
            }
        };
        // ---- the added row of row-step ps (transposed registers) -> its ring slot
        auto write_xt = [&](const WsPos &ps, const u32x4r (&r)[8]) {
            if constexpr (XCONV_ROW_DBG & 16) return;
            if (x_on && ps.y > 0) {
                int slot = ps.rowmod + P.kH - 1;
                slot = slot >= P.NRING ? slot - P.NRING : slot;
                uint4 *dst = lds_b + slot * P.b_row_units + x_lds;
#pragma unroll
                for (int e = 0; e < 8; ++e) dst[(x_rot + e) & 15] = uint4{r[e].x, r[e].y, r[e].z, r[e].w};
            }
        };
        // ---- every row of the window of row-step ps, loaded and written at once (start of a run)
        auto prime = [&](const WsPos &ps, auto npc) {
            const i32x4r rsB = rsrc_of(Ag, ps.bg, a_img_bytes, true);
            const int total = P.kH * P.BWc * JC;
            constexpr int NP = decltype(npc)::value;
            for (int base = 0; base < total; base += NP * kProducers) {
                u32x4r r[NP][8];
                int lds[NP], rot[NP];
#pragma unroll
                for (int u = 0; u < NP; ++u) {
                    const int idx = base + u * kProducers + p;
                    const int jc = idx & (JC - 1);
                    int c = idx >> jc_shift, rr = 0;
#pragma unroll
                    for (int q = 1; q < 3; ++q) {
                        const bool wrap = c >= P.BWc;
                        c = wrap ? c - P.BWc : c;
                        rr = wrap ? rr + 1 : rr;
                    }
                    const int iy = ps.y + rr - P.ph, ix = c - P.pw;
                    const bool in = idx < total && (unsigned)iy < (unsigned)P.H && (unsigned)ix < (unsigned)P.W;
                    int slot = ps.rowmod + rr;
                    slot = slot >= P.NRING ? slot - P.NRING : slot;
                    const uint32_t voff = in ? ((uint32_t)(iy * P.W + ix) * (uint32_t)P.CS + (uint32_t)(jb + 8 * jc)) * 2u : kOOR;
                    lds[u] = slot * P.b_row_units + c * P.BSTR + 16 * (jc >> 1);
                    rot[u] = ((jc & 1) * 8 + (jc >> 2) * rotmul) & 15;
#pragma unroll
                    for (int img = 0; img < 8; ++img) buf16_async(r[u][img], rsB, voff + (uint32_t)img * a_img_bytes);
                }
#pragma unroll
                for (int u = 0; u < NP; ++u) {
                    // needed right away; the loads of task u are older than those of the tasks after it
                    asm volatile("s_waitcnt vmcnt(%8)"
                                 : "+v"(r[u][0]), "+v"(r[u][1]), "+v"(r[u][2]), "+v"(r[u][3]), "+v"(r[u][4]), "+v"(r[u][5]),
                                   "+v"(r[u][6]), "+v"(r[u][7])
                                 : "n"((NP - 1 - u) * 8)
                                 : "memory");
                    transpose(r[u]);
                    if (base + u * kProducers + p < total) {
                        uint4 *dst = lds_b + lds[u];
#pragma unroll
                        for (int e = 0; e < 8; ++e) dst[(rot[u] + e) & 15] = uint4{r[u][e].x, r[u][e].y, r[u][e].z, r[u][e].w};
                    }
                }
            }
        };

        if (NI > 0) {
            const int nrows = t_end - t_begin;
            // At the top of a row-step r (steady state) dY of row r sits transposed in set r & 1, and the loads in flight
            // per thread are, oldest first, A of row r + 1 and dY of row r + 1 (set (r + 1) & 1).  After the row's first
            // barrier the second sub-step's tile is written, then the added row of row-step r + 1, then dY of row r + 1 is
            // transposed in its registers; behind the row's second barrier A and dY of row r + 2 go out.
            u32x4r sdy[2][8], sxt[8];
            WsPos pr = ws_pos_of(P, t_begin);   // row-step whose tiles are written next
            pr.u = P.NSUB - 1;                  // (ws_advance then moves on to the next row)
            WsPos p1 = ws_advance(P, pr);       // the row-step after it
            if constexpr (XCONV_ROW_DBG & 32) { ts_[2] = __builtin_readcyclecounter(); }
            issue_dy(pr, true, sdy[0]);
            if constexpr (XCONV_ROW_DBG & 32) { ts_[3] = __builtin_readcyclecounter(); }
            prime(pr, IC<3>{});
            if constexpr (XCONV_ROW_DBG & 32) { ts_[4] = __builtin_readcyclecounter(); }
            issue_xt(p1, nrows > 1, sxt);
            issue_dy(p1, nrows > 1, sdy[1]);
            wait8(IC<16>{}, sdy[0]);
            if constexpr (XCONV_ROW_DBG & 32) { ts_[5] = __builtin_readcyclecounter(); }
            transpose(sdy[0]);
            // One barrier per dY tile: it hands tile (row, u) and whatever was written to the ring meanwhile to the
            // consumers, who pass it one k-step before they finish the tile before.  The two register sets of dY take
            // turns row by row; the loop body is written out once per set so that which registers a load lands in
            // never depends on a run-time choice (a copy between its issue and its wait would read them too early).
            auto row_step = [&](int row, u32x4r (&sd)[8], u32x4r (&sn)[8]) {
                const int tile = row * P.NSUB;
                if (row > 0 && pr.y == 0) {
                    ws_barrier();  // the consumers have left the previous run: its ring rows are free
                    prime(pr, IC<1>{});
                }
                // first tile of the row (its dY is in `sd`, transposed half a row-step ago)
                write_dy(0, tile & 1, sd);
                ws_barrier();
                if constexpr (XCONV_ROW_DBG & 32) {
                    if (row == 0 && p == 0) {   // producer stamps go through spare LDS words to the consumer that writes them out
                        ts_[6] = __builtin_readcyclecounter();
                        unsigned long long *l = reinterpret_cast<unsigned long long *>(row_lds + 2 * P.a_units + P.NRING * P.b_row_units);
                        for (int q = 2; q < 7; ++q) l[q] = ts_[q];
                    }
                }
                if (P.NSUB == 2) write_dy(1, (tile + 1) & 1, sd);
                // the row that the next row-step adds to the ring (its slot was last read by the row-step before
                // this one), then the loads two row-steps ahead into the registers that just became free
                WsPos p2 = p1;
                p2.u = P.NSUB - 1;
                p2 = ws_advance(P, p2);
                wait8(IC<8>{}, sxt);
                transpose(sxt);
                if (row + 1 < nrows) write_xt(p1, sxt);
                // dY of the next row-step (the last load in flight): transposed here, in the longer half of the row-step,
                // so that the path to the next row's first barrier is short
                wait8(IC<0>{}, sn);
                transpose(sn);
                // The barrier of the row's second tile, then the loads two row-steps ahead.  Measured on the C5 layer,
                // loop cycles per workgroup: loads issued in front of this barrier and dY transposed at the top of its own
                // row-step 85.7K, loads behind the barrier 83.5K, that and the early transpose 81.9K; the barrier
                // right behind write_dy(1) 93.4K, the A loads in front of it and the dY loads behind 83.8K.
                if (P.NSUB == 2) ws_barrier();
                issue_xt(p2, row + 2 < nrows, sxt);
                issue_dy(p2, row + 2 < nrows, sd);
                pr = p1;
                p1 = p2;
            };
            for (int row = 0; row < nrows; row += 2) {
                row_step(row, sdy[0], sdy[1]);
                if (row + 1 < nrows) row_step(row + 1, sdy[1], sdy[0]);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the last (empty) prefetches
        }
    }
}

// ---------------------------------------------------------------------------
// host: launch plan
// ---------------------------------------------------------------------------
static int row_env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

static const size_t kRowLdsLimit = 160 * 1024;

size_t corr_row_lds_bytes(const WsParams &P)
{
    return ((size_t)2 * P.a_units + (size_t)P.NRING * P.b_row_units) * 16 + ((XCONV_ROW_DBG & 32) ? 64 : 0);
}

bool plan_corr_row(WsParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw, int CS)
{
    if (dtype == XCONV_F32) return false;
    if (row_env_int("XCONV_CORR_ROW", 1) == 0) return false;
    if (kH != 3 || kW != 3 || sh != 1 || sw != 1) return false;
    P = WsParams{};
    P.B = B; P.C_out = C_out; P.H = H; P.W = W;
    P.kH = kH; P.kW = kW; P.sh = sh; P.sw = sw; P.ph = ph; P.pw = pw;
    P.Ho = H + 2 * ph - 2;
    P.Wo = W + 2 * pw - 2;
    P.CS = CS;
    P.NBG = ceil_div(B, 8);
    P.K2 = 9;
    P.NOG = 1;
    if (P.Wo % 4 != 0) return false;   // two lane groups, each with its half of the row; the halves of dY rows start 4-byte aligned
    // a group of 8 images is addressed with 32-bit byte offsets
    if ((long long)8 * C_out * P.Ho * P.Wo * 2 > (1LL << 30) || (long long)8 * H * W * CS * 2 > (1LL << 30)) return false;
    if (CS % 32 != 0) return false;
    const int nwj = CS / 32;
    int WJ = (nwj % 2 == 0) ? 2 : 1;
    if (C_out <= 32 && nwj % 4 == 0) WJ = 4;
    WJ = row_env_int("XCONV_ROW_WJ", WJ);
    if (WJ != 1 && WJ != 2 && WJ != 4) return false;
    if (nwj % WJ != 0) return false;
    P.WM = 4 / WJ; P.WJ = WJ; P.MT = 1;
    P.M_WG = P.WM * 32;
    P.J_WG = WJ * 32;
    P.NTM = ceil_div(C_out, P.M_WG);
    P.NTJ = CS / P.J_WG;
    P.MP = P.NTM * P.M_WG;
    P.JP = CS;

    // a row in one or two sub-steps; a piece of a lane group's half in a sub-step is one 16-byte load
    const int Qr = P.Wo / 2;
    P.CW = P.Wo;
    P.NSTRIP = 1;
    P.NSUB = Qr <= 8 ? 1 : 2;
    P.NSUB = row_env_int("XCONV_ROW_NSUB", P.NSUB);
    if (P.NSUB != 1 && P.NSUB != 2) return false;
    const int Q0 = P.NSUB == 1 ? Qr : round_up(ceil_div(Qr, 2), 2);   // (the second sub-step's pieces start 4-byte aligned too)
    if (Q0 > 8 || (P.NSUB == 2 && (Qr - Q0 < 1 || Qr - Q0 > 8))) return false;
    P.CWs = 2 * Q0;
    P.BWc = P.Wo + 2;
    P.NRING = 4;
    P.a_units = 2 * Q0 * P.M_WG;
    P.BSTR = P.J_WG;
    P.b_row_units = P.BWc * P.BSTR;
    // one dY task and one A task per producer thread
    if (P.M_WG * 2 * P.NSUB > kProducers) return false;
    if (P.BWc * (P.J_WG / 8) > kProducers) return false;
    P.NA = P.M_WG * 2 * P.NSUB;
    P.NA_pad = round_up(P.NA, 64);
    P.TB = P.BWc * (P.J_WG / 8);
    P.TS = P.TB;
    P.NTASK = 1;
    P.NS = P.NBG * P.Ho;
    if (corr_row_lds_bytes(P) > kRowLdsLimit) return false;

    // K-split: one workgroup per compute unit
    const int ny = P.NTM * P.NTJ;
    int target = row_env_int("XCONV_ROW_SPLITS", 0);
    if (target <= 0) {
        target = 256 / ny;
        if (target < 1) target = 1;
        if (target > P.NS) target = P.NS;
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

template <int DT, int REM, int CB> static hipError_t launch_row_cfg(const WsParams &P, hipStream_t st)
{
    const size_t lds = corr_row_lds_bytes(P);
    static bool done = false;  // per instantiation: the attribute sticks to the function
    if (!done && lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(corr_row_kernel<DT, REM, CB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRowLdsLimit);
        if (e != hipSuccess) return e;
        done = true;
    }
    WsParams Q = P;
    Q.SQ = P.NS / P.S;
    Q.SR = P.NS % P.S;
    hipLaunchKernelGGL((corr_row_kernel<DT, REM, CB>), dim3(P.S, P.NTM * P.NTJ, 1), dim3(kWsThreads), lds, st, Q);
    return hipGetLastError();
}

template <int DT, int CB> static hipError_t launch_row_rem(const WsParams &P, hipStream_t st)
{
    switch ((P.Wo / 2 - 1) % 3) {
    case 0: return launch_row_cfg<DT, 0, CB>(P, st);
    case 1: return launch_row_cfg<DT, 1, CB>(P, st);
    default: return launch_row_cfg<DT, 2, CB>(P, st);
    }
}

template <int DT> static hipError_t launch_row_dt(const WsParams &P, hipStream_t st)
{
    switch (P.BSTR) {
    case 32: return launch_row_rem<DT, 32 * 16>(P, st);
    case 64: return launch_row_rem<DT, 64 * 16>(P, st);
    default: return launch_row_rem<DT, 128 * 16>(P, st);
    }
}

hipError_t launch_corr_row(int dtype, const WsParams &P, hipStream_t st)
{
    if (dtype == XCONV_BF16) return launch_row_dt<XCONV_BF16>(P, st);
    return launch_row_dt<XCONV_F16>(P, st);
}

}  // namespace xc
