// Offset-wise correlation G[m,j,ky,kx] = sum_{b,oy,ox} dY[b,m,oy,ox] * A[b, oy*sh+ky-ph, ox*sw+kx-pw, j]
// (Algorithm 1, backward step 3 with the shift of step 4; Eq. (2)/(5) when A = X) for fp32
// storage, as a producer/consumer kernel.  Same division of labour as the 16-bit kernel:
//
//   waves 0-3 (consumers)  read fragments from LDS and issue v_mfma_f32_16x16x4_f32 only.  Each
//                          owns a 16 (output channels) x 16 (columns of A) x 9 offsets block.
//   waves 4-7 (producers)  bring dY (NCHW) and A (channels-last) from global memory into LDS,
//                          three steps ahead of the consumers, the loads waiting in registers.
//
// The 16-byte LDS unit holds the 4 images of one (pixel, channel): the MFMA reduction index is
// the pixel slot (4 per MFMA, lane group g = lane / 16 takes slot 4q + g), and the four images
// of a unit go through four MFMAs.  As in the 16-bit kernel a kernel offset or a stride only
// changes which unit a lane reads.  A step is one output row of one strip of 4 images; the
// rows of A it needs live in a ring of kH + sh rows, so each row is loaded once per pass of a
// workgroup; dY row pieces are double-buffered.  One barrier per step, which the consumers run
// one k-step early (the fragments of their last k-step are in registers by then).
#include <type_traits>

#include "common.h"
#include "launch.h"
#include "ws_pos.h"

namespace xc {

// NOFF: kernel offsets a workgroup accumulates (9; a last group with fewer recomputes its first
// offset in the spare slots and does not write them).  NTASK: staging tasks per producer thread
// and step.  D: steps whose loads are in flight.
// OCC: workgroups per compute unit the register budget allows for (2: two consumer waves per SIMD,
// which the fp32 MFMA needs to issue at its full rate).
// VOL: dY is read in place as the depth slots of volumes (WsParams::vol_*)
template <int NOFF, int NTASK, int D, int OCC, bool VOL>
__global__ __launch_bounds__(kWsThreads, 2 * OCC) void corr_ws32_kernel(const WsParams P)
{
    draw_z_slice(P.zout, P.nz, P.zdist, P.zseed);
    extern __shared__ uint4 ws32_lds[];
    uint4 *lds_a = ws32_lds;                    // two dY tiles [slot][M_WG]
    uint4 *lds_b = ws32_lds + 2 * P.a_units;    // ring of A rows [slot][column][BSTR]
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    typedef int i32x4 __attribute__((ext_vector_type(4)));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int tm, tj;
    fast_divmod((int)blockIdx.y, P.NTM, frcp(P.NTM), tj, tm);
    const int m0 = tm * P.M_WG;
    const int jb = tj * P.J_WG;
    const int o_first = blockIdx.z * NOFF;
    const int noff = (P.K2 - o_first) < NOFF ? (P.K2 - o_first) : NOFF;

    // K-split of this workgroup: neighbouring splits on one die (C4: 97.5 -> 95.5 us), except for volumes read in place, whose
    // channel planes can lie a power of two apart: there neighbours on one die crowd the same L2 channels (V1: 105.7 -> 109 us)
    const int bx = VOL ? (int)blockIdx.x : xcd_block(blockIdx.x, gridDim.x);
    const int t_begin = bx * P.SQ + (bx < P.SR ? bx : P.SR);
    const int t_end = t_begin + P.SQ + (bx < P.SR ? 1 : 0);
    const int NI = t_end - t_begin;  // steps of this workgroup

    if (wave < 4) {
        // =========================== consumers ===========================
        __builtin_amdgcn_s_setprio(3);
        const int i16 = lane & 15, g = lane >> 4;
        const int wm = wave & (P.WM - 1), wj = wave >> __builtin_ctz((unsigned)P.WM);  // WM is 1, 2 or 4

        f32x4 acc[NOFF];
#pragma unroll
        for (int o = 0; o < NOFF; ++o) acc[o] = f32x4{0.f, 0.f, 0.f, 0.f};

        int off_ky[NOFF], off_kx[NOFF];
#pragma unroll
        for (int o = 0; o < NOFF; ++o) {
            const int oo = (o < noff) ? (o_first + o) : o_first;
            fast_divmod(oo, P.kW, frcp(P.kW), off_ky[o], off_kx[o]);
        }
        int brow[NOFF];  // LDS unit of (ring slot of the offset's row, column kx)
        auto set_brow = [&](const WsPos &p) {
#pragma unroll
            for (int o = 0; o < NOFF; ++o) {
                int slot = p.rowmod + off_ky[o];
                slot = slot >= P.NRING ? slot - P.NRING : slot;
                brow[o] = __builtin_amdgcn_readfirstlane(slot * P.b_row_units + off_kx[o] * P.BSTR);
            }
        };

        if (NI > 0) {
            WsPos pc = ws_pos_of(P, t_begin);
            set_brow(pc);
            const uint32_t lds0 = __builtin_amdgcn_groupstaticsize();
            const uint32_t a_base = lds0 + (uint32_t)(g * P.M_WG + wm * 16 + i16) * 16u;
            const uint32_t b_base = lds0 + (uint32_t)(2 * P.a_units + g * P.sw * P.BSTR + wj * 16 + i16) * 16u;
            const uint32_t step_a = (uint32_t)(4 * P.M_WG) * 16u;            // bytes between k-steps
            const uint32_t step_b = (uint32_t)(4 * P.sw * P.BSTR) * 16u;

            // Fragment reads are opaque instructions waited for by hand (see the 16-bit kernel):
            // requests return in order, so counting the younger ones tells when a fragment is here.
            auto lds_read = [](u32x4 &dst, uint32_t addr) {
                asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr) : "memory");
            };
            u32x4 a, an, b[NOFF];
            uint32_t pa = a_base, pb[NOFF];
            auto set_pb = [&]() {
#pragma unroll
                for (int o = 0; o < NOFF; ++o) pb[o] = b_base + (uint32_t)brow[o] * 16u;
            };
            set_pb();

            ws_barrier();  // the first dY tile and the rows of the first step are in LDS

            lds_read(a, pa);
            ws_static_for<0, NOFF>([&](auto oc) { lds_read(b[decltype(oc)::value], pb[decltype(oc)::value]); });
            asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(NOFF) : "memory");

            // One k-step: 4 pixel slots x 4 images x NOFF offsets.  Image e of every offset before
            // image e + 1 (MFMAs into one accumulator are then NOFF instructions apart).  The
            // requests for the next k-step: A at the start, the B fragment of offset o - 1 right
            // after the last MFMA (image 3) of offset o.  Before the first MFMAs of offsets
            // o..o+2 the previous k-step's requests up to o + 2 must be done; the younger ones
            // are then the rest of those and this k-step's A.
            constexpr int WG3 = (NOFF % 3 == 0) ? 3 : 1;
            auto kstep = [&]() {
                __builtin_amdgcn_sched_barrier(0);
                lds_read(an, pa);
                ws_static_for<0, 4>([&](auto ec) {
                    constexpr int e = decltype(ec)::value;
                    ws_static_for<0, NOFF>([&](auto oc) {
                        constexpr int o = decltype(oc)::value;
                        if constexpr (e == 0 && o % WG3 == 0) {
                            constexpr int younger = NOFF - WG3 - o + 1;
                            __builtin_amdgcn_sched_barrier(0);
                            if constexpr (WG3 == 3)
                                asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(b[o]), "+v"(b[o + 1]), "+v"(b[o + 2]) : "n"(younger) : "memory");
                            else
                                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(b[o]) : "n"(younger) : "memory");
                        }
                        // (element first, then the reinterpretation: a bit cast applied to a vector
                        // element expression reads element 0 whatever the index)
                        const unsigned int au = a[e], bu = b[o][e];
                        acc[o] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(au), __uint_as_float(bu), acc[o], 0, 0, 0);
                        if constexpr (e == 3 && o >= 1) {
                            __builtin_amdgcn_sched_barrier(0);
                            lds_read(b[o - 1], pb[o - 1]);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    });
                });
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[NOFF - 1], pb[NOFF - 1]);
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(an) : "n"(NOFF) : "memory");
                a = an;
                __builtin_amdgcn_sched_barrier(0);
            };

            for (int i = 0; i < NI; ++i) {
                const int nkq = ws_cw_sub(P, pc) >> 2;
                for (int q = 0; q + 1 < nkq; ++q) {
                    pa += step_a;
#pragma unroll
                    for (int o = 0; o < NOFF; ++o) pb[o] += step_b;
                    kstep();
                }
                // The last k-step of the step.  Its fragments were requested a whole k-step ago;
                // once they are here the consumers no longer read step i, so its buffer and the
                // ring rows it alone used go back to the producers now, and the fragments
                // requested during this k-step are those of the next step.
                if (i + 1 < NI) {
                    const WsPos pn = ws_advance(P, pc);
                    set_brow(pn);
                    pa = a_base + (uint32_t)(((i + 1) & 1) * P.a_units) * 16u;
                    set_pb();
                    if (pn.y == 0) ws_barrier();  // run boundary: the producers refill the whole ring first
                    ws_barrier();
                    pc = pn;
                }
                // (after the very last step the requests repeat the current addresses)
                kstep();
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }

        // D tile: lane (i16, g) holds column i16 and rows 4g .. 4g + 3
        const int jcol = jb + wj * 16 + i16;
#pragma unroll
        for (int o = 0; o < NOFF; ++o) {
            if (o < noff) {
                float *dst = P.part + (size_t)bx * P.K2 * P.JP * P.MP + tile_index(o_first + o, jcol, m0 + wm * 16 + 4 * g, P.JP, P.MP);
                *reinterpret_cast<f32x4 *>(dst) = acc[o];
            }
        }
    } else {
        // =========================== producers ===========================
        __builtin_amdgcn_s_setprio(0);
        const int p = tid - kProducers;
        const float *dY = static_cast<const float *>(P.dY);
        const float *Ag = static_cast<const float *>(P.A);
        const int HoWo = P.Ho * P.Wo;
        constexpr bool vol = VOL;
        // bytes between the planes of consecutive channels and between consecutive images of the batch
        const uint32_t dy_plane_bytes = (uint32_t)HoWo * 4u * (vol ? (uint32_t)P.vol_Do : 1u);
        const uint32_t dy_img_bytes = vol ? (uint32_t)HoWo * 4u : (uint32_t)P.C_out * (uint32_t)HoWo * 4u;
        const float rcp_period = frcp(vol ? P.vol_period : 1);
        const uint32_t a_img_bytes = (uint32_t)P.H * (uint32_t)P.W * (uint32_t)P.CS * 4u;
        const int JC = P.J_WG >> 2;                                      // 4-column vectors per staged pixel
        const int jc_shift = __builtin_ctz((unsigned)JC);                // J_WG is 16, 32 or 64
        const int rows_new = P.sh < P.kH ? P.sh : P.kH;                  // rows a step adds to the ring
        const int rows_old = P.kH - rows_new;                            // rows it inherits from its predecessor
        const float rcp_bwc = frcp(P.BWc);

        // Task slots of this thread.  Slots below NA_pad (whole waves) stage dY: chunk of 4 columns
        // fastest (neighbouring lanes read neighbouring 16-byte pieces of one (image, channel)
        // row).  The remaining slots stage the rows of A the step adds: column vector fastest.
        bool is_a[NTASK];
        uint32_t t_goff[NTASK];    // byte offset inside an image without the step's part, or kOOR
        int t_lds[NTASK], t_aux[NTASK];
        const int nch = P.CWs >> 2;
        const float rcp_nch = frcp(nch);
#pragma unroll
        for (int k = 0; k < NTASK; ++k) {
            const int s = p + kProducers * k;
            is_a[k] = __builtin_amdgcn_readfirstlane((int)(s < P.NA_pad)) != 0;
            if (is_a[k]) {
                int ch, m;
                fast_divmod(s, nch, rcp_nch, m, ch);
                t_goff[k] = (s < P.NA && m0 + m < P.C_out) ? (uint32_t)(m0 + m) * dy_plane_bytes + 16u * ch : kOOR;
                t_lds[k] = 4 * ch * P.M_WG + m;
                t_aux[k] = 4 * ch;          // first column of the chunk
            } else {
                const int w = s - P.NA_pad;
                const int jc = w & (JC - 1);
                int c, rr;
                fast_divmod(w >> jc_shift, P.BWc, rcp_bwc, rr, c);
                const bool has = w < P.TB;
                t_goff[k] = has ? ((uint32_t)(rr * P.W + c) * (uint32_t)P.CS + (uint32_t)(jb + 4 * jc)) * 4u : kOOR;
                t_lds[k] = c * P.BSTR + 4 * jc;
                t_aux[k] = c | (rr << 16);
            }
        }

        // Buffer resources built by hand (base, size, flags): a group with fewer than 4 images, or a
        // step that does not exist, gets a smaller (or empty) resource: reads past it return zero.
        auto rsrc_of = [&](const float *base, int bg, uint32_t img_bytes, bool live) {
            bg = __builtin_amdgcn_readfirstlane(bg);
            int left = P.B - bg * 4;
            left = left < 4 ? left : 4;
            left = (live && left > 0) ? left : 0;
            const uint64_t addr = reinterpret_cast<uint64_t>(base + (size_t)bg * 4 * (img_bytes / 4));
            i32x4 r;
            r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
            r.y = __builtin_amdgcn_readfirstlane((int)(uint32_t)((addr >> 32) & 0xffffu));
            r.z = __builtin_amdgcn_readfirstlane((int)((uint32_t)left * img_bytes));
            r.w = 0x00020000;
            return r;
        };
        // Loads of the software pipeline: opaque instructions, waited for by hand (stage_wait);
        // nothing reads a stage between its loads and its wait.
        auto buf16_async = [](u32x4 &dst, i32x4 r, uint32_t voff) {
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(r) : "memory");
        };
        // the 4 images x 4 values of a task as 4 units (value e of every image)
        auto store_units = [&](uint4 *dst, int stride, const u32x4 (&r)[4], bool (&keep)[4]) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                dst[e * stride] = keep[e] ? uint4{r[0][e], r[1][e], r[2][e], r[3][e]} : uint4{0u, 0u, 0u, 0u};
        };

        // ---- loads of step ps: its dY row piece and the rows it adds to the ring
        auto issue = [&](const WsPos &ps, bool live, u32x4 (&r)[NTASK][4]) {
            const int cw = ws_cw_sub(P, ps);
            const uint32_t fs = (uint32_t)(ps.y * P.Wo + ps.strip * P.CW) * 4u;
            // dY: byte offset of each of the group's 4 images, or kOOR for one that does not exist
            i32x4 rsA;
            uint32_t doff[4] = {0u, 0u, 0u, 0u};
            if constexpr (!vol) {
                rsA = rsrc_of(dY, ps.bg, dy_img_bytes, live);
            } else {
                // the whole tensor behind one resource; image -> (volume, depth slot), empty slots read as zero
                const uint64_t addr = reinterpret_cast<uint64_t>(dY);
                rsA.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
                rsA.y = __builtin_amdgcn_readfirstlane((int)(uint32_t)((addr >> 32) & 0xffffu));
                rsA.z = __builtin_amdgcn_readfirstlane((int)(live ? P.vol_bytes : 0u));
                rsA.w = 0x00020000;
                const uint32_t vol_stride = (uint32_t)P.C_out * dy_plane_bytes;
#pragma unroll
                for (int img = 0; img < 4; ++img) {
                    const int i = __builtin_amdgcn_readfirstlane(ps.bg) * 4 + img;
                    int bv, z;
                    fast_divmod(i, P.vol_period, rcp_period, bv, z);
                    doff[img] = (uint32_t)__builtin_amdgcn_readfirstlane(
                        (int)((i < P.B && z < P.vol_Do) ? (uint32_t)bv * vol_stride + (uint32_t)z * dy_img_bytes : kOOR));
                }
            }
            const i32x4 rsB = rsrc_of(Ag, ps.bg, a_img_bytes, live);
            const int iy0 = ps.y * P.sh + rows_old - P.ph;   // input row of the first added row
            const int ix0 = ps.strip * P.CW * P.sw - P.pw;
            const uint32_t origin = (uint32_t)(iy0 * P.W + ix0) * ((uint32_t)P.CS * 4u);  // wraps when negative; exact for every in-range pixel
#pragma unroll
            for (int k = 0; k < NTASK; ++k) {
                if (is_a[k]) {
                    const uint32_t voff = (t_goff[k] != kOOR && t_aux[k] < cw) ? t_goff[k] + fs : kOOR;
#pragma unroll
                    for (int img = 0; img < 4; ++img) {
                        if constexpr (!vol) buf16_async(r[k][img], rsA, voff + (uint32_t)img * dy_img_bytes);
                        else buf16_async(r[k][img], rsA, (voff != kOOR && doff[img] != kOOR) ? voff + doff[img] : kOOR);
                    }
                } else {
                    const int c = t_aux[k] & 0xffff, rr = t_aux[k] >> 16;
                    const bool in = t_goff[k] != kOOR && (unsigned)(iy0 + rr) < (unsigned)P.H && (unsigned)(ix0 + c) < (unsigned)P.W;
                    const uint32_t voff = in ? origin + t_goff[k] : kOOR;
#pragma unroll
                    for (int img = 0; img < 4; ++img) buf16_async(r[k][img], rsB, voff + (uint32_t)img * a_img_bytes);
                }
            }
        };
        // the loads of a stage are followed by those of D - 1 younger stages
        auto stage_wait = [&](u32x4 (&r)[NTASK][4]) {
            constexpr int kYounger = (D - 1) * NTASK * 4;
#pragma unroll
            for (int k = 0; k < NTASK; ++k)
                asm volatile("s_waitcnt vmcnt(%4)" : "+v"(r[k][0]), "+v"(r[k][1]), "+v"(r[k][2]), "+v"(r[k][3]) : "n"(kYounger) : "memory");
        };
        // ---- registers -> LDS
        auto write = [&](const WsPos &ps, int buf, const u32x4 (&r)[NTASK][4]) {
            const int cw = ws_cw_sub(P, ps);
            int slot0 = ps.rowmod + rows_old;   // ring slot of the first added row
            slot0 = slot0 >= P.NRING ? slot0 - P.NRING : slot0;
#pragma unroll
            for (int k = 0; k < NTASK; ++k) {
                if (is_a[k]) {
                    // columns past the end of the row take part in the MFMAs: they must be zero
                    bool keep[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) keep[e] = t_aux[k] + e < cw;
                    if (p + kProducers * k < P.NA) store_units(lds_a + buf * P.a_units + t_lds[k], P.M_WG, r[k], keep);
                } else if (t_goff[k] != kOOR) {
                    int slot = slot0 + (t_aux[k] >> 16);
                    slot = slot >= P.NRING ? slot - P.NRING : slot;
                    bool keep[4] = {true, true, true, true};
                    store_units(lds_b + slot * P.b_row_units + t_lds[k], 1, r[k], keep);
                }
            }
        };
        // ---- the rows a step inherits, loaded and written at once (start of a run)
        auto prime = [&](const WsPos &ps) {
            const i32x4 rsB = rsrc_of(Ag, ps.bg, a_img_bytes, true);
            const int total = rows_old * P.BWc * JC;
            const int iy0 = ps.y * P.sh - P.ph, ix0 = ps.strip * P.CW * P.sw - P.pw;
            constexpr int NP = 2;  // tasks in flight per thread
            for (int base = 0; base < total; base += NP * kProducers) {
                u32x4 r[NP][4];
                int lds[NP];
                bool has[NP];
#pragma unroll
                for (int u = 0; u < NP; ++u) {
                    const int idx = base + u * kProducers + p;
                    const int jc = idx & (JC - 1);
                    int c, rr;
                    fast_divmod(idx >> jc_shift, P.BWc, rcp_bwc, rr, c);
                    has[u] = idx < total;
                    const int iy = iy0 + rr, ix = ix0 + c;
                    const bool in = has[u] && (unsigned)iy < (unsigned)P.H && (unsigned)ix < (unsigned)P.W;
                    const uint32_t voff = in ? ((uint32_t)(iy * P.W + ix) * (uint32_t)P.CS + (uint32_t)(jb + 4 * jc)) * 4u : kOOR;
                    int slot = ps.rowmod + rr;
                    slot = slot >= P.NRING ? slot - P.NRING : slot;
                    lds[u] = slot * P.b_row_units + c * P.BSTR + 4 * jc;
#pragma unroll
                    for (int img = 0; img < 4; ++img) buf16_async(r[u][img], rsB, voff + (uint32_t)img * a_img_bytes);
                }
#pragma unroll
                for (int u = 0; u < NP; ++u) {
                    // needed right away; the loads of task u are older than those of the tasks after it
                    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(r[u][0]), "+v"(r[u][1]), "+v"(r[u][2]), "+v"(r[u][3]) : "n"((NP - 1 - u) * 4) : "memory");
                    bool keep[4] = {true, true, true, true};
                    if (has[u]) store_units(lds_b + lds[u], 1, r[u], keep);
                }
            }
        };

        if (NI > 0) {
            WsPos pw = ws_pos_of(P, t_begin);  // step whose data is written next
            WsPos pi = pw;                     // step whose loads are issued next
            u32x4 st[D][NTASK][4];
            // The loads of the first step go out first and stay in flight during the round trip of
            // the rows it inherits (their waits also cover these older loads).
            issue(pi, true, st[0]);
            pi = ws_advance(P, pi);
            prime(pw);
#pragma unroll
            for (int d = 1; d < D; ++d) {
                issue(pi, d < NI, st[d]);
                pi = ws_advance(P, pi);
            }
            for (int i0 = 0; i0 < NI; i0 += D) {
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const int i = i0 + d;
                    if (i < NI) {
                        if (i > 0 && pw.y == 0) {
                            ws_barrier();  // the consumers have left the previous run: its ring rows are free
                            // the younger stages' loads are in flight: drain them with the window's
                            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                            prime(pw);
                        }
                        stage_wait(st[d]);
                        write(pw, i & 1, st[d]);
                        issue(pi, i + D < NI, st[d]);
                        pw = ws_advance(P, pw);
                        pi = ws_advance(P, pi);
                        ws_barrier();
                    }
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the last (empty) prefetches
        }
    }
}

// ---------------------------------------------------------------------------
// host: launch plan
// ---------------------------------------------------------------------------
static int ws32_env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

static const size_t kWs32LdsLimit = 160 * 1024;

size_t corr_ws32_lds_bytes(const WsParams &P)
{
    return ((size_t)2 * P.a_units + (size_t)P.NRING * P.b_row_units) * 16;
}

bool plan_corr_ws32(WsParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw, int CS)
{
    if (dtype != XCONV_F32) return false;
    if (ws32_env_int("XCONV_CORR_WS32", 1) == 0) return false;
    P.B = B; P.C_out = C_out; P.H = H; P.W = W;
    P.kH = kH; P.kW = kW; P.sh = sh; P.sw = sw; P.ph = ph; P.pw = pw;
    P.Ho = (H + 2 * ph - kH) / sh + 1;
    P.Wo = (W + 2 * pw - kW) / sw + 1;
    P.CS = CS;
    P.K2 = kH * kW;
    if (P.K2 == 1) return false;           // 1x1: the generic kernel keeps whole images in flight instead
    if (P.Wo % 4 != 0) return false;       // rows of dY are read and multiplied in whole vectors of 4 columns
    if (kH > 8 || sh > 8) return false;
    P.NBG = ceil_div(B, 4);
    P.NOG = ceil_div(P.K2, 9);
    // a group of 4 images is addressed with 32-bit byte offsets
    if ((long long)4 * C_out * P.Ho * P.Wo * 4 > (1LL << 30) || (long long)4 * H * W * CS * 4 > (1LL << 30)) return false;

    // consumer waves: 16 output channels x 16 columns each; along the columns of A first
    const int nwj = CS / 16;
    int WJ = (nwj % 4 == 0 && C_out <= 16) ? 4 : (nwj % 2 == 0 && C_out <= 32) ? 2 : 1;
    WJ = ws32_env_int("XCONV_WS32_WJ", WJ);
    if (WJ != 1 && WJ != 2 && WJ != 4) return false;
    if (nwj % WJ != 0) return false;
    const int WM = 4 / WJ;
    P.WM = WM; P.WJ = WJ;
    P.M_WG = 16 * WM; P.J_WG = 16 * WJ;
    P.NTM = ceil_div(C_out, P.M_WG);
    P.NTJ = CS / P.J_WG;
    P.MP = P.NTM * P.M_WG;
    P.JP = CS;
    P.MT = 1;
    P.NSUB = 1;
    P.NRING = kH + sh;
    P.BSTR = P.J_WG;
    const int rows_new = sh < kH ? sh : kH;

    // Strip width: a multiple of 4.  First choice: two workgroups per compute unit (half the LDS,
    // at most two tasks per producer thread: see launch_corr_ws32), which gives every SIMD two
    // consumer waves; else one workgroup with up to three tasks.  Among the widths that fit, the
    // one that wastes the fewest columns in the last strip, then the widest.
    auto geometry = [&](int cw) {
        P.CW = cw; P.CWs = cw;
        P.NSTRIP = ceil_div(P.Wo, cw);
        P.BWc = (cw - 1) * sw + kW;
        P.a_units = cw * P.M_WG;
        P.b_row_units = P.BWc * P.BSTR;
        P.NA = P.M_WG * (cw / 4);
        P.NA_pad = round_up(P.NA, 64);
        P.TB = rows_new * P.BWc * (P.J_WG / 4);
        P.TS = P.TB;
        P.NTASK = ceil_div(P.NA_pad + P.TB, kProducers);
    };
    const int cw_max = ws32_env_int("XCONV_WS32_CW", 64);
    int best = 0, per_cu = 1;
    for (int occ = ws32_env_int("XCONV_WS32_OCC", 2); occ >= 1 && best == 0; --occ) {
        int best_waste = 1 << 30;
        for (int cw = (P.Wo < cw_max ? P.Wo : cw_max) & ~3; cw >= 4; cw -= 4) {
            geometry(cw);
            if (occ * corr_ws32_lds_bytes(P) > kWs32LdsLimit || P.NTASK > (occ == 2 ? 2 : 3)) continue;
            const int waste = P.NSTRIP * cw - P.Wo;
            if (waste < best_waste) { best_waste = waste; best = cw; }
        }
        if (best) per_cu = occ;
    }
    if (best == 0) return false;
    geometry(best);
    P.NS = P.NBG * P.NSTRIP * P.Ho;

    // K-split: one workgroup per compute unit
    const int ny = P.NTM * P.NTJ * P.NOG;
    int target = ws32_env_int("XCONV_WS32_SPLITS", 0);
    if (target <= 0) {
        target = 256 * per_cu / ny;
        // Two workgroups per compute unit overlap one's start with the other's loop, but with fewer than 8 steps each the
        // starts and the partial tiles are most of the work: then one workgroup per unit with twice the steps
        // (C2, 2048 steps: 512 splits 33.1 + 10.7 us for correlation + second pass, 256 splits 32.3 + 9.7 us;
        // C4, 8192 steps: 95.2 against 103.7 us)
        if (per_cu == 2 && target >= 2 && P.NS / target < 8) target /= 2;
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

template <int NTASK, int D, int OCC, bool VOL> static hipError_t launch_ws32_vol(const WsParams &P, hipStream_t st)
{
    const size_t lds = corr_ws32_lds_bytes(P);
    static bool done = false;  // per instantiation: the attribute sticks to the function
    if (!done && lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(corr_ws32_kernel<9, NTASK, D, OCC, VOL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kWs32LdsLimit);
        if (e != hipSuccess) return e;
        done = true;
    }
    WsParams Q = P;
    Q.SQ = P.NS / P.S;
    Q.SR = P.NS % P.S;
    hipLaunchKernelGGL((corr_ws32_kernel<9, NTASK, D, OCC, VOL>), dim3(P.S, P.NTM * P.NTJ, P.NOG), dim3(kWsThreads), lds, st, Q);
    return hipGetLastError();
}

template <int NTASK, int D, int OCC> static hipError_t launch_ws32_cfg(const WsParams &P, hipStream_t st)
{
    if (P.vol_period != 0) return launch_ws32_vol<NTASK, D, OCC, true>(P, st);
    return launch_ws32_vol<NTASK, D, OCC, false>(P, st);
}

hipError_t launch_corr_ws32(const WsParams &P, hipStream_t st)
{
    // two workgroups per compute unit when LDS and the staging registers (two stages of at most
    // two tasks) allow it
    if (P.NTASK <= 2 && 2 * corr_ws32_lds_bytes(P) <= kWs32LdsLimit) {
        if (P.NTASK == 1) return launch_ws32_cfg<1, 2, 2>(P, st);
        return launch_ws32_cfg<2, 2, 2>(P, st);
    }
    switch (P.NTASK) {
    case 1: return launch_ws32_cfg<1, 3, 1>(P, st);
    case 2: return launch_ws32_cfg<2, 3, 1>(P, st);
    default: return launch_ws32_cfg<3, 3, 1>(P, st);
    }
}

}  // namespace xc
