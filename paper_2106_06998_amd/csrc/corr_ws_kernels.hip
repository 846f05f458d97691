// Offset-wise correlation (Algorithm 1, backward step 3 with the shift of step 4) for 16-bit
// storage, as a producer/consumer kernel:
//
//   G[m,j,ky,kx] = sum_{b,oy,ox} dY[b,m,oy,ox] * A[b, oy*sh+ky-ph, ox*sw+kx-pw, j]
//
// As in corr_kernel (corr_kernels.hip) the reduction index is packed along the batch: one LDS
// unit (16 bytes) holds the 8 images of one (pixel, channel), so kernel offsets and strides
// only select which unit a lane reads.  Here the matrix instruction is v_mfma_f32_32x32x16
// (reduction = 8 images x 2 neighbouring pixel slots): measured on MI355X it reaches the full
// matrix-core rate from one wave per SIMD, the 16x16x32 shape only half of it.  Work is split
// by role:
//
//   waves 0-3 (consumers)  only read fragments from LDS and issue MFMAs.  Each owns
//                          32 output channels x 32 columns x NOFF offsets (NOFF 32x32 tiles).
//   waves 4-7 (producers)  bring dY (NCHW) and A (channels-last) from global memory into the
//                          unit form: eight 16-byte loads (one per image), an 8x8 transpose in
//                          registers, eight LDS writes.  Loads run D sub-steps ahead of the
//                          consumers and wait in registers, so HBM latency is covered by
//                          several sub-steps of MFMA work instead of one.
//
// A row-step is one output row of one strip of 8 images; it is cut into NSUB sub-steps of CWs
// output columns.  dY tiles are double-buffered per sub-step; the rows of A live in a ring of
// kH + sh row slots, so the rows a row-step adds are written while the previous rows are
// still being read.  One workgroup barrier per sub-step hands a dY buffer (and the ring rows
// written meanwhile) from the producers to the consumers and the previous buffer back.  The
// consumers run that barrier one k-step early: the fragments of the last k-step of a sub-step
// are already in registers, so its MFMAs overlap the barrier and the first fragment reads of
// the next sub-step.
#include <type_traits>

#include "common.h"
#include "launch.h"
#include "ws_pos.h"

namespace xc {


typedef float f32x16 __attribute__((ext_vector_type(16)));

// 32x32x16 MFMA on eight 16-bit values per lane.  This shape runs at the full matrix-core rate
// from a single wave per SIMD; the 16x16x32 shape needs twice the issue slots per flop.
template <int DT> __device__ inline f32x16 mfma32(const uint4 &a, const uint4 &b, f32x16 c)
{
    if constexpr (DT == XCONV_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// CB > 0: 3x3 offsets and the bytes of one staged column of A (BSTR * 16) known at compile time:
// the three column offsets of a kernel row are then immediates of one address register.
// VOL: dY is read in place as the depth slots of volumes (WsParams::vol_*)
template <int DT, int NOFF, int NTASK, int D, int CB, bool RU, bool VOL>
__global__ __launch_bounds__(kWsThreads) void corr_ws_kernel(const WsParams P)
{
    draw_z_slice(P.zout, P.nz, P.zdist, P.zseed);
    extern __shared__ uint4 ws_lds[];
    uint4 *lds_a = ws_lds;                    // two dY tiles [slot][M_WG]
    uint4 *lds_b = ws_lds + 2 * P.a_units;    // ring of A rows [slot][column][BSTR]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int tm, tj;
    fast_divmod((int)blockIdx.y, P.NTM, frcp(P.NTM), tj, tm);
    const int m0 = tm * P.M_WG;
    const int jb = tj * P.J_WG;
    const int o_first = blockIdx.z * NOFF;
    const int noff = (P.K2 - o_first) < NOFF ? (P.K2 - o_first) : NOFF;

    const int bx = xcd_block(blockIdx.x, gridDim.x);   // K-split of this workgroup: neighbouring splits on one die (V2: 37.2 -> 34.0 us per launch)
    const int t_begin = bx * P.SQ + (bx < P.SR ? bx : P.SR);
    const int t_end = t_begin + P.SQ + (bx < P.SR ? 1 : 0);
    const int NI = (t_end - t_begin) * P.NSUB;  // sub-steps of this workgroup
    // Units of one staged pixel: the 16-column group G sits at 16G, rotated by (G/2)*rotmul.  Both
    // groups that a consumer wave reads together (G = 2wj, 2wj+1) have the same rotation, which
    // ds_read_b128 needs to stay free of bank conflicts; the rotation between waves' groups spreads
    // the producers' writes (8 columns per lane, lanes running over the column vectors) over banks.
    const int rotmul = 8 >> __builtin_ctz((unsigned)P.WJ);  // WJ is 1, 2 or 4

    if (wave < 4) {
        // =========================== consumers ===========================
        // MFMA operands: A = dY units, lane (m = lane % 32, g = lane / 32) takes pixel slot 2q+g;
        // B = A-tensor units, lane (j = lane % 32, g) takes the shifted pixel; D is 32 x 32.
        // the MFMA stream goes first; the producers' vector and LDS instructions fill the gaps
        __builtin_amdgcn_s_setprio(3);
        const int l32 = lane & 31, g = lane >> 5;
        const int wm = wave & (P.WM - 1), wj = wave >> __builtin_ctz((unsigned)P.WM);  // WM is 1, 2 or 4
        const int a_lane = g * P.M_WG + wm * 32 + l32;
        const int G = 2 * wj + (l32 >> 4);  // 16-column group of this lane's column
        const int b_lane = g * P.sw * P.BSTR + G * 16 + (((l32 & 15) + wj * rotmul) & 15);

        f32x16 acc[NOFF];
#pragma unroll
        for (int o = 0; o < NOFF; ++o)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[o][e] = 0.f;

        int off_ky[NOFF], off_kx[NOFF];
#pragma unroll
        for (int o = 0; o < NOFF; ++o) {
            const int oo = (o < noff) ? (o_first + o) : o_first;  // spare slots redo the first offset and are not written
            fast_divmod(oo, P.kW, frcp(P.kW), off_ky[o], off_kx[o]);
        }
        auto set_brow = [&](const WsPos &p, int (&brow)[NOFF]) {
#pragma unroll
            for (int o = 0; o < NOFF; ++o) {
                int slot = p.rowmod + off_ky[o];
                slot = slot >= P.NRING ? slot - P.NRING : slot;
                brow[o] = __builtin_amdgcn_readfirstlane(slot * P.b_row_units + off_kx[o] * P.BSTR);
            }
        };

        if (NI > 0) {
          if constexpr (RU) {
            // ---- 3x3, unit stride: the fragments of one staged pixel serve three k-steps ----
            // Lane group g takes pixel slot q + g*Q of a sub-step of 2Q slots (not 2q + g), so the
            // B fragment of kernel column kx at k-step q is the one of column 0 at k-step q + kx:
            // per kernel row a window of three fragments slides along the staged row, and a
            // k-step requests 1 + 3 fragments instead of 1 + 9.  The three window registers of a
            // kernel row are used in rotation: k-steps come in groups of three (one variant of the
            // code per position in the group), each requesting the new column into the registers
            // whose last use was issued an MFMA earlier.  The k-steps left over at the end of a
            // sub-step, and its last one, refill the whole window instead (nine requests).
            typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
            WsPos pc = ws_pos_of(P, t_begin);
            int brow[NOFF];
            set_brow(pc, brow);
            const uint32_t lds0 = __builtin_amdgcn_groupstaticsize();
            const uint32_t a_wave = lds0 + (uint32_t)(wm * 32 + l32) * 16u;
            const uint32_t b_wave = lds0 + (uint32_t)(2 * P.a_units + G * 16 + (((l32 & 15) + wj * rotmul) & 15)) * 16u;
            const uint32_t step_a = (uint32_t)P.M_WG * 16u;  // one pixel slot per k-step
            auto a_addr = [&](int buf, int Q) { return a_wave + (uint32_t)(buf * P.a_units + g * Q * P.M_WG) * 16u; };
            // column 0 of kernel row ky for the lane's half of the sub-step
            auto b_addr = [&](const WsPos &p, int Q, int ky) {
                return b_wave + (uint32_t)(brow[3 * ky] + (p.u * P.CWs + g * Q) * P.BSTR) * 16u;
            };
            auto lds_read = [](u32x4 &dst, uint32_t addr, auto off) {
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(decltype(off)::value) : "memory");
            };
            // requests return in order: at most N younger ones may be in flight behind x, y, z
            auto arrived3 = [](auto nc, u32x4 &x, u32x4 &y, u32x4 &z) {
                asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(x), "+v"(y), "+v"(z) : "n"(decltype(nc)::value) : "memory");
            };
            auto arrived1 = [](auto nc, u32x4 &x) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(decltype(nc)::value) : "memory"); };
            using I0 = std::integral_constant<int, 0>;
            using C1 = std::integral_constant<int, CB>;
            using C2 = std::integral_constant<int, 2 * CB>;
            using O0 = std::integral_constant<int, 0>; using O1 = std::integral_constant<int, 1>; using O2 = std::integral_constant<int, 2>;
            using O3 = std::integral_constant<int, 3>; using O4 = std::integral_constant<int, 4>; using O5 = std::integral_constant<int, 5>;
            using O6 = std::integral_constant<int, 6>; using O7 = std::integral_constant<int, 7>; using O8 = std::integral_constant<int, 8>;
            u32x4 a, an, b[9];   // b[3*ky + w]: window register w of kernel row ky
            uint32_t pa, pb3[3];
            auto mma = [&](auto oc, const u32x4 &bf) {
                constexpr int o = decltype(oc)::value;
                acc[o] = mfma32<DT>(__builtin_bit_cast(uint4, a), __builtin_bit_cast(uint4, bf), acc[o]);
            };

            int Q = ws_cw_sub(P, pc) >> 1;
            pa = a_addr(0, Q);
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) pb3[ky] = b_addr(pc, Q, ky);
            ws_barrier();  // the first dY tile and the rows of the first row-step are in LDS
            lds_read(an, pa, I0{});
            ws_static_for<0, 9>([&](auto oc) {   // window register w <- column w, kernel rows inside
                constexpr int o = decltype(oc)::value;
                lds_read(b[3 * (o % 3) + o / 3], pb3[o % 3], std::integral_constant<int, (o / 3) * CB>{});
            });
            arrived1(std::integral_constant<int, 9>{}, an);
            a = an;
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) pb3[ky] += 3u * CB;   // the column that k-step 0 requests

            // Position `ph` of a group of three k-steps: window register (ph + kx) % 3 holds the
            // column of kernel column kx.  In flight at the start: the three requests of the k-step
            // before, or the nine of a window refill; counted from the youngest, what a kernel
            // column needs is followed by at most 7 / 6 / 4 requests, and in the steady state the
            // first two waits fall through.
            auto inner = [&](auto phc) {
                constexpr int w0 = decltype(phc)::value, w1 = (w0 + 1) % 3, w2 = (w0 + 2) % 3;
                __builtin_amdgcn_sched_barrier(0);
                lds_read(an, pa, I0{});
                arrived3(std::integral_constant<int, 7>{}, b[w0], b[3 + w0], b[6 + w0]);
                mma(O0{}, b[w0]);
                mma(O3{}, b[3 + w0]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[w0], pb3[0], I0{});
                __builtin_amdgcn_sched_barrier(0);
                mma(O6{}, b[6 + w0]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[3 + w0], pb3[1], I0{});
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_sched_barrier(0);
                arrived3(std::integral_constant<int, 6>{}, b[w1], b[3 + w1], b[6 + w1]);
                mma(O1{}, b[w1]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[6 + w0], pb3[2], I0{});
                __builtin_amdgcn_sched_barrier(0);
                mma(O4{}, b[3 + w1]);
                mma(O7{}, b[6 + w1]);
                __builtin_amdgcn_sched_barrier(0);
                arrived3(std::integral_constant<int, 4>{}, b[w2], b[3 + w2], b[6 + w2]);
                mma(O2{}, b[w2]);
                mma(O5{}, b[3 + w2]);
                mma(O8{}, b[6 + w2]);
                __builtin_amdgcn_sched_barrier(0);
                arrived1(std::integral_constant<int, 3>{}, an);
                a = an;
                __builtin_amdgcn_sched_barrier(0);
            };
            // A k-step at position 0 that refills the whole window (and A) from (pa_n, pbn): column
            // kx into window register kx right after the MFMAs that read it.  Used for the last
            // k-step of a sub-step (the addresses are then those of the next sub-step) and for
            // k-steps that do not fill a group of three.
            auto refill = [&](uint32_t pa_n, const uint32_t (&pbn)[3]) {
                __builtin_amdgcn_sched_barrier(0);
                lds_read(an, pa_n, I0{});
                arrived3(std::integral_constant<int, 7>{}, b[0], b[3], b[6]);
                mma(O0{}, b[0]);
                mma(O3{}, b[3]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[0], pbn[0], I0{});
                __builtin_amdgcn_sched_barrier(0);
                mma(O6{}, b[6]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[3], pbn[1], I0{});
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_sched_barrier(0);
                arrived3(std::integral_constant<int, 6>{}, b[1], b[4], b[7]);
                mma(O1{}, b[1]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[6], pbn[2], I0{});
                __builtin_amdgcn_sched_barrier(0);
                mma(O4{}, b[4]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[1], pbn[0], C1{});
                __builtin_amdgcn_sched_barrier(0);
                mma(O7{}, b[7]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[4], pbn[1], C1{});
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_sched_barrier(0);
                arrived3(std::integral_constant<int, 6>{}, b[2], b[5], b[8]);
                mma(O2{}, b[2]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[7], pbn[2], C1{});
                __builtin_amdgcn_sched_barrier(0);
                mma(O5{}, b[5]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[2], pbn[0], C2{});
                __builtin_amdgcn_sched_barrier(0);
                mma(O8{}, b[8]);
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[5], pbn[1], C2{});
                __builtin_amdgcn_sched_barrier(0);
                lds_read(b[8], pbn[2], C2{});
                __builtin_amdgcn_sched_barrier(0);
                arrived1(std::integral_constant<int, 9>{}, an);
                a = an;
                __builtin_amdgcn_sched_barrier(0);
            };

            uint32_t pbn[3];
            for (int i = 0; i < NI; ++i) {
                const int n_in = Q - 1;                        // k-steps before the last one
                const int n3 = (n_in * 0xAAAB) >> 17;          // n_in / 3
                for (int t = 0; t < n3; ++t) {
                    pa += step_a;
                    inner(std::integral_constant<int, 0>{});
                    pa += step_a;
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pb3[ky] += (uint32_t)CB;
                    inner(std::integral_constant<int, 1>{});
                    pa += step_a;
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pb3[ky] += (uint32_t)CB;
                    inner(std::integral_constant<int, 2>{});
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pb3[ky] += (uint32_t)CB;
                }
                for (int t = 3 * n3; t < n_in; ++t) {
                    // pb3 is the column three ahead of the current one: the next k-step starts two before it
                    pa += step_a;
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pbn[ky] = pb3[ky] - 2u * CB;
                    refill(pa, pbn);
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pb3[ky] += (uint32_t)CB;
                }
                // The last k-step of the sub-step.  Its fragments were requested during the k-step
                // before; once they are here the consumers no longer read sub-step i, so its buffer
                // and the ring rows it alone used go back to the producers now.
                uint32_t pa_n = pa;
                int Qn = Q;
                if (i + 1 < NI) {
                    const WsPos pn = ws_advance(P, pc);
                    if (pn.t != pc.t) set_brow(pn, brow);
                    Qn = ws_cw_sub(P, pn) >> 1;
                    pa_n = a_addr((i + 1) & 1, Qn);
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pbn[ky] = b_addr(pn, Qn, ky);
                    if (pn.u == 0 && pn.y == 0) ws_barrier();  // run boundary: the producers refill the whole ring first
                    ws_barrier();
                    pc = pn;
                } else {
                    // after the very last sub-step the requests repeat addresses of this one
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) pbn[ky] = b_addr(pc, Q, ky);
                }
                refill(pa_n, pbn);
                pa = pa_n;
                Q = Qn;
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) pb3[ky] = pbn[ky] + 3u * CB;
            }
          } else {
            typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
            WsPos pc = ws_pos_of(P, t_begin);
            int brow[NOFF];
            set_brow(pc, brow);
            // LDS byte addresses (the dynamic allocation starts behind the static one)
            const uint32_t lds0 = __builtin_amdgcn_groupstaticsize();
            const uint32_t a_base = lds0 + (uint32_t)a_lane * 16u;
            const uint32_t b_base = lds0 + (uint32_t)(2 * P.a_units + b_lane) * 16u;
            const uint32_t step_a = (uint32_t)(2 * P.M_WG) * 16u;            // bytes between k-steps
            const uint32_t step_b = (uint32_t)(2 * P.sw * P.BSTR) * 16u;

            // Fragment reads are issued as opaque instructions and waited for by hand.  Left to the
            // compiler, every loop back-edge and branch between two k-steps gets a wait for all
            // outstanding LDS reads, i.e. for the ones issued a few cycles earlier, and the matrix
            // cores idle for an LDS round trip per k-step.  The requests of a k-step are issued in
            // a fixed order (A of the next k-step, then after the MFMA of offset o the B fragment of
            // offset o for the next k-step), LDS returns in order, so just before the MFMA of any
            // offset at most NOFF younger requests may still be in flight (NOFF - 1 with the reads
            // issued one MFMA late, see kstep).
            auto lds_read = [](u32x4 &dst, uint32_t addr, auto off) {
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(decltype(off)::value) : "memory");
            };
            // address registers of the B fragments: one per offset, or (CB > 0) one per kernel row
            constexpr int NPB = CB > 0 ? 3 : NOFF;
            u32x4 a, an, b[NOFF];
            uint32_t pa = a_base, pbo[NPB];
            auto set_pbo = [&](const WsPos &p) {
                const uint32_t pb = b_base + (uint32_t)((p.u * P.CWs * P.sw) * P.BSTR) * 16u;
#pragma unroll
                for (int q = 0; q < NPB; ++q) pbo[q] = pb + (uint32_t)brow[CB > 0 ? 3 * q : q] * 16u;
            };
            auto read_b = [&](auto oc) {
                constexpr int o = decltype(oc)::value;
                if constexpr (CB > 0) lds_read(b[o], pbo[o / 3], std::integral_constant<int, (o % 3) * CB>{});
                else lds_read(b[o], pbo[o], std::integral_constant<int, 0>{});
            };
            set_pbo(pc);

            ws_barrier();  // the first dY tile and the rows of the first row-step are in LDS

            lds_read(a, pa, std::integral_constant<int, 0>{});
            ws_static_for<0, NOFF>([&](auto oc) { read_b(oc); });

            // One k-step: its MFMAs and the requests for the fragments at (pa, pbo).  The fragment
            // of offset o-1 is replaced one MFMA late (a load into registers that the MFMA just
            // issued still reads would be held back until that MFMA is done), and the waits come
            // once per three MFMAs: before the MFMA of offset o = 0, 3, 6 the fragment of offset
            // o+2 must be there, after which at most 6 younger requests are in flight.
            constexpr int WG3 = (NOFF % 3 == 0) ? 3 : 1;   // MFMAs per wait
            constexpr int WN = WG3 == 3 ? 6 : (NOFF > 1 ? NOFF - 1 : 1);
            auto kstep = [&]() {
                __builtin_amdgcn_sched_barrier(0);
                lds_read(an, pa, std::integral_constant<int, 0>{});
                ws_static_for<0, NOFF>([&](auto oc) {
                    constexpr int o = decltype(oc)::value;
                    if constexpr (o % WG3 == 0) {
                        if constexpr (WG3 == 3)
                            asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b[o]), "+v"(b[o + 1]), "+v"(b[o + 2]) : "n"(WN) : "memory");
                        else
                            asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b[o]) : "n"(WN) : "memory");
                    }
                    acc[o] = mfma32<DT>(__builtin_bit_cast(uint4, a), __builtin_bit_cast(uint4, b[o]), acc[o]);
                    if constexpr (o >= 1) read_b(std::integral_constant<int, o - 1>{});
                });
                read_b(std::integral_constant<int, NOFF - 1>{});
                // the A fragment of the next k-step is the oldest of the NOFF + 1 requests just issued
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(an) : "n"(NOFF) : "memory");
                a = an;
                __builtin_amdgcn_sched_barrier(0);
            };

            for (int i = 0; i < NI; ++i) {
                const int nkq = (ws_cw_sub(P, pc) + 1) >> 1;
                // k-steps whose successor lies in the same sub-step: constant address steps
                for (int q = 0; q + 1 < nkq; ++q) {
                    pa += step_a;
#pragma unroll
                    for (int o = 0; o < NPB; ++o) pbo[o] += step_b;
                    kstep();
                }
                // The last k-step of the sub-step.  Its fragments were requested a whole k-step
                // ago; once they are here the consumers no longer read sub-step i, so its buffer and
                // the ring rows it alone used go back to the producers now, and the fragments
                // requested during this k-step are those of the next sub-step.
                if (i + 1 < NI) {
                    const WsPos pn = ws_advance(P, pc);
                    if (pn.t != pc.t) set_brow(pn, brow);
                    pa = a_base + (uint32_t)(((i + 1) & 1) * P.a_units) * 16u;
                    set_pbo(pn);
                    if (pn.u == 0 && pn.y == 0) ws_barrier();  // run boundary: the producers refill the whole ring first
                    ws_barrier();
                    pc = pn;
                }
                // (after the very last sub-step the requests repeat the current addresses)
                kstep();
            }
          }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }


        // D tile: lane (l32, g) holds column l32 and rows 8v + 4g .. 8v + 4g + 3 (v = 0..3)
        const int jcol = jb + wj * 32 + l32;
#pragma unroll
        for (int o = 0; o < NOFF; ++o) {
            if (o < noff) {
                float *dst = P.part + (size_t)bx * P.K2 * P.JP * P.MP + tile_index(o_first + o, jcol, m0 + wm * 32 + 4 * g, P.JP, P.MP);
#pragma unroll
                for (int v = 0; v < 4; ++v)   // rows 8v + 4g ..: two channel quads further on
                    *reinterpret_cast<f32x4 *>(dst + (size_t)8 * v * P.JP) = f32x4{acc[o][4 * v], acc[o][4 * v + 1], acc[o][4 * v + 2], acc[o][4 * v + 3]};
            }
        }
    } else {
        // =========================== producers ===========================
        __builtin_amdgcn_s_setprio(0);
        const int p = tid - kProducers;
        const uint16_t *dY = static_cast<const uint16_t *>(P.dY);
        const uint16_t *Ag = static_cast<const uint16_t *>(P.A);
        const int HoWo = P.Ho * P.Wo;
        constexpr bool vol = VOL;
        // bytes between the planes of consecutive channels and between consecutive images of the batch
        const uint32_t dy_plane_bytes = (uint32_t)HoWo * 2u * (vol ? (uint32_t)P.vol_Do : 1u);
        const uint32_t dy_img_bytes = vol ? (uint32_t)HoWo * 2u : (uint32_t)P.C_out * (uint32_t)HoWo * 2u;
        const float rcp_period = frcp(vol ? P.vol_period : 1);
        const uint32_t a_img_bytes = (uint32_t)P.H * (uint32_t)P.W * (uint32_t)P.CS * 2u;
        const int JC = P.J_WG >> 3;
        const int jc_shift = __builtin_ctz((unsigned)JC);  // J_WG is 32, 64 or 128

        // Task slots of this thread.  Slots below NA_pad (whole waves) stage dY: output channel
        // m = slot % M_WG, chunk of 8 columns slot / M_WG, so that the 64 lanes of a wave write
        // 64 consecutive units of one pixel slot.  The remaining slots stage A.
        bool is_a[NTASK];
        uint32_t a_goff[NTASK];
        int a_lds[NTASK], a_c8[NTASK], b_w[NTASK];
#pragma unroll
        for (int k = 0; k < NTASK; ++k) {
            const int s = p + kProducers * k;
            is_a[k] = __builtin_amdgcn_readfirstlane((int)(s < P.NA_pad)) != 0;
            // chunk index fastest: neighbouring lanes read neighbouring 16-byte pieces of one
            // (image, channel) row, which the memory pipeline merges into one request
            const int nch = (P.CWs + 7) >> 3;
            int ch, m;
            fast_divmod(s, nch, frcp(nch), m, ch);
            a_goff[k] = (s < P.NA && m0 + m < P.C_out) ? (uint32_t)(m0 + m) * dy_plane_bytes + 16u * ch : kOOR;
            a_lds[k] = 8 * ch * P.M_WG + m;
            a_c8[k] = 8 * ch;
            b_w[k] = s - P.NA_pad;
        }

        // Buffer resources are built by hand (base, size, flags) so that they can be handed to the
        // load instruction below.  A group with fewer than 8 images, or a sub-step that does not
        // exist, gets a smaller (or empty) resource: reads past it return zero in hardware.
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        auto rsrc_of = [&](const uint16_t *base, int bg, uint32_t img_bytes, bool live) {
            bg = __builtin_amdgcn_readfirstlane(bg);
            int left = P.B - bg * 8;
            left = left < 8 ? left : 8;
            left = (live && left > 0) ? left : 0;
            const uint64_t addr = reinterpret_cast<uint64_t>(base + (size_t)bg * 8 * (img_bytes / 2));
            i32x4 r;
            r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
            r.y = __builtin_amdgcn_readfirstlane((int)(uint32_t)((addr >> 32) & 0xffffu));
            r.z = __builtin_amdgcn_readfirstlane((int)((uint32_t)left * img_bytes));
            r.w = 0x00020000;
            return r;
        };
        // Loads of the software pipeline.  They are issued as opaque instructions: the compiler
        // places its own waits for loads it knows about right before the first use and, across
        // this kernel's loops and branches, falls back to waiting for (nearly) all outstanding
        // loads, which would undo the prefetch distance.  The pipeline waits by hand instead
        // (stage_wait below); nothing reads a stage between its loads and its wait.
        auto buf16_async = [](u32x4 &dst, i32x4 r, uint32_t voff) {
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(r) : "memory");
        };

        // A task `idx` of a row window: staged column c, row rr of the rows being added, 8-column
        // vector jc.  pr0/slot0: padded input row and ring slot of rr = 0.
        struct XtTask {
            uint32_t voff;  // byte offset inside an image, or kOOR
            int lds;        // LDS unit of the task's first column, before the rotation
            int rot;
        };
        auto xt_task = [&](int idx, bool ok, int pr0, int slot0, int ix0) {
            const int jc = idx & (JC - 1);
            int c = idx >> jc_shift, rr = 0;
#pragma unroll
            for (int q = 1; q < 8; ++q) {  // at most 8 rows are added per row-step (plan_corr_ws)
                const bool wrap = c >= P.BWc;
                c = wrap ? c - P.BWc : c;
                rr = wrap ? rr + 1 : rr;
            }
            const int iy = pr0 + rr - P.ph, ix = ix0 + c;
            const bool in = ok && (unsigned)iy < (unsigned)P.H && (unsigned)ix < (unsigned)P.W;
            int slot = slot0 + rr;
            slot = slot >= P.NRING ? slot - P.NRING : slot;
            slot = slot >= P.NRING ? slot - P.NRING : slot;
            XtTask t;
            t.voff = in ? ((uint32_t)(iy * P.W + ix) * (uint32_t)P.CS + (uint32_t)(jb + 8 * jc)) * 2u : kOOR;
            t.lds = slot * P.b_row_units + c * P.BSTR + 16 * (jc >> 1);
            t.rot = ((jc & 1) * 8 + (jc >> 2) * rotmul) & 15;
            return t;
        };
        auto xt_store = [&](const XtTask &t, const uint4 (&src)[8]) {
            uint32_t rows[8][4];
#pragma unroll
            for (int q = 0; q < 8; ++q) { rows[q][0] = src[q].x; rows[q][1] = src[q].y; rows[q][2] = src[q].z; rows[q][3] = src[q].w; }
            uint4 cols[8];
            transpose_rows8<4>(rows, cols);
            uint4 *dst = lds_b + t.lds;
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[(t.rot + e) & 15] = cols[e];
        };

        // The A tasks of this thread, decoded once for each of the (at most two) slices: byte
        // offset of (row rr, column c, column vector jc) from the first added row and first
        // staged column, or kOOR for a thread without a task in that slice; LDS unit inside a ring
        // row; c, rr and the rotation packed into one word.
        uint32_t x_goff[NTASK][2];
        int x_lds[NTASK][2], x_crr[NTASK][2];
#pragma unroll
        for (int k = 0; k < NTASK; ++k)
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const int idx = v * P.TS + b_w[k];
                const bool ok = !is_a[k] && v < P.NSUB && b_w[k] >= 0 && b_w[k] < P.TS && idx < P.TB;
                const int jc = idx & (JC - 1);
                int c = idx >> jc_shift, rr = 0;
#pragma unroll
                for (int q = 1; q < 8; ++q) {
                    const bool wrap = c >= P.BWc;
                    c = wrap ? c - P.BWc : c;
                    rr = wrap ? rr + 1 : rr;
                }
                x_goff[k][v] = ok ? ((uint32_t)(rr * P.W + c) * (uint32_t)P.CS + (uint32_t)(jb + 8 * jc)) * 2u : kOOR;
                x_lds[k][v] = c * P.BSTR + 16 * (jc >> 1);
                x_crr[k][v] = c | (rr << 16) | ((((jc & 1) * 8 + (jc >> 2) * rotmul) & 15) << 24);
            }

        // The rows of A that sub-step `ps` brings in, as (row-step they belong to, slice).
        // One slice per sub-step: with a single sub-step per row-step the row-step's own new
        // rows; otherwise sub-step 0 brings the last slice of its own row-step and sub-step
        // u >= 1 slice u-1 of the next row-step (which reads them one row-step later).
        struct XtPlan {
            bool on;
            int slice, pr0, slot0, ix0;
        };
        auto xt_plan = [&](const WsPos &ps) {
            XtPlan x;
            int y = ps.y, rowmod = ps.rowmod;
            x.on = true;
            x.slice = 0;
            if (P.NSUB > 1) {
                if (ps.u == 0) {
                    x.slice = P.NSUB - 1;
                } else {
                    x.slice = ps.u - 1;
                    x.on = (ps.y + 1 < P.Ho) && (ps.t + 1 < t_end);
                    y = ps.y + 1;
                    rowmod += P.sh;
                    while (rowmod >= P.NRING) rowmod -= P.NRING;
                }
            }
            x.pr0 = y * P.sh + P.kH - P.sh;  // first of the sh rows that this row-step adds (kH <= sh: all of them start at 0)
            int slot0 = rowmod + P.kH - P.sh;
            if (P.kH < P.sh) { x.pr0 = y * P.sh; slot0 = rowmod; }
            while (slot0 >= P.NRING) slot0 -= P.NRING;
            x.slot0 = slot0;
            x.ix0 = ps.strip * P.CW * P.sw - P.pw;
            x.on = __builtin_amdgcn_readfirstlane((int)x.on) != 0;
            x.slice = __builtin_amdgcn_readfirstlane(x.slice);
            x.pr0 = __builtin_amdgcn_readfirstlane(x.pr0);
            x.slot0 = __builtin_amdgcn_readfirstlane(x.slot0);
            x.ix0 = __builtin_amdgcn_readfirstlane(x.ix0);
            return x;
        };

        // ---- global -> registers for sub-step ps --------------------------------------
        auto issue = [&](const WsPos &ps, bool live, u32x4 (&r)[NTASK][8]) {
            const int cw_sub = ws_cw_sub(P, ps);
            const uint32_t fs = (uint32_t)(ps.y * P.Wo + ps.strip * P.CW + ps.u * P.CWs) * 2u;
            // dY: byte offset of each of the group's 8 images, or kOOR for one that does not exist
            i32x4 rsA;
            uint32_t doff[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
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
                for (int img = 0; img < 8; ++img) {
                    const int i = __builtin_amdgcn_readfirstlane(ps.bg) * 8 + img;
                    int bv, z;
                    fast_divmod(i, P.vol_period, rcp_period, bv, z);
                    doff[img] = (uint32_t)__builtin_amdgcn_readfirstlane(
                        (int)((i < P.B && z < P.vol_Do) ? (uint32_t)bv * vol_stride + (uint32_t)z * dy_img_bytes : kOOR));
                }
            }
            const XtPlan x = xt_plan(ps);
            const i32x4 rsB = rsrc_of(Ag, ps.bg, a_img_bytes, live && x.on);
#pragma unroll
            for (int k = 0; k < NTASK; ++k) {
                if (is_a[k]) {
                    const uint32_t voff = (a_goff[k] != kOOR && a_c8[k] < cw_sub) ? a_goff[k] + fs : kOOR;
#pragma unroll
                    for (int img = 0; img < 8; ++img) {
                        if constexpr (!vol) buf16_async(r[k][img], rsA, voff + (uint32_t)img * dy_img_bytes);
                        else buf16_async(r[k][img], rsA, (voff != kOOR && doff[img] != kOOR) ? voff + doff[img] : kOOR);
                    }
                } else {
                    const uint32_t goff = x.slice ? x_goff[k][1] : x_goff[k][0];
                    const int crr = x.slice ? x_crr[k][1] : x_crr[k][0];
                    const int iy = x.pr0 - P.ph + ((crr >> 16) & 0xff), ix = x.ix0 + (crr & 0xffff);
                    const bool in = goff != kOOR && (unsigned)iy < (unsigned)P.H && (unsigned)ix < (unsigned)P.W;
                    // (the origin may lie in the padding: the sum wraps and is exact for every pixel inside the image)
                    const uint32_t origin = (uint32_t)((x.pr0 - P.ph) * P.W + x.ix0) * ((uint32_t)P.CS * 2u);
                    const uint32_t voff = in ? origin + goff : kOOR;
#pragma unroll
                    for (int img = 0; img < 8; ++img) buf16_async(r[k][img], rsB, voff + (uint32_t)img * a_img_bytes);
                }
            }
        };
        // Waits until the loads of a stage have arrived: they are the oldest outstanding ones and
        // loads return in order, so it is enough that at most the (D-1) younger stages are still
        // in flight.  (Loads that the compiler issues in between only make this wait longer.)  The
        // stage's registers are operands so that every use of them stays behind the wait.
        auto stage_wait = [&](u32x4 (&r)[NTASK][8]) {
            constexpr int kYounger = (D - 1) * NTASK * 8;
            static_assert(kYounger <= 63, "vmcnt field");
#pragma unroll
            for (int k = 0; k < NTASK; ++k)
                asm volatile("s_waitcnt vmcnt(%8)"
                             : "+v"(r[k][0]), "+v"(r[k][1]), "+v"(r[k][2]), "+v"(r[k][3]), "+v"(r[k][4]), "+v"(r[k][5]),
                               "+v"(r[k][6]), "+v"(r[k][7])
                             : "n"(kYounger)
                             : "memory");
        };
        // ---- registers -> LDS for sub-step ps (buffer `buf` of the dY tiles) ------------
        auto write = [&](const WsPos &ps, int buf, const u32x4 (&r)[NTASK][8]) {
            const int cw_sub = ws_cw_sub(P, ps);
            const XtPlan x = xt_plan(ps);
#pragma unroll
            for (int k = 0; k < NTASK; ++k) {
                uint4 src[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) src[q] = uint4{r[k][q].x, r[k][q].y, r[k][q].z, r[k][q].w};
                uint32_t rows[8][4];
#pragma unroll
                for (int q = 0; q < 8; ++q) { rows[q][0] = src[q].x; rows[q][1] = src[q].y; rows[q][2] = src[q].z; rows[q][3] = src[q].w; }
                uint4 cols[8];
                transpose_rows8<4>(rows, cols);
                if (is_a[k]) {
                    uint4 *dst = lds_a + buf * P.a_units + a_lds[k];
                    if (cw_sub >= ((P.CWs + 7) & ~7)) {  // every slot of every chunk is a real column
#pragma unroll
                        for (int e = 0; e < 8; ++e) dst[e * P.M_WG] = cols[e];
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            // columns past the end of the row take part in the MFMAs: they must be zero
                            // (the tile has whole chunks of 8 slots, so every store has a place)
                            const bool in = a_c8[k] + e < cw_sub;
                            dst[e * P.M_WG] = uint4{in ? cols[e].x : 0u, in ? cols[e].y : 0u, in ? cols[e].z : 0u, in ? cols[e].w : 0u};
                        }
                    }
                } else if (x.on) {
                    const uint32_t goff = x.slice ? x_goff[k][1] : x_goff[k][0];
                    if (goff != kOOR) {
                        const int crr = x.slice ? x_crr[k][1] : x_crr[k][0];
                        int slot = x.slot0 + ((crr >> 16) & 0xff);
                        slot = slot >= P.NRING ? slot - P.NRING : slot;
                        slot = slot >= P.NRING ? slot - P.NRING : slot;
                        uint4 *dst = lds_b + slot * P.b_row_units + (x.slice ? x_lds[k][1] : x_lds[k][0]);
                        const int rot = (crr >> 24) & 15;
#pragma unroll
                        for (int e = 0; e < 8; ++e) dst[(rot + e) & 15] = cols[e];
                    }
                }
            }
        };
        // ---- every row of the window of row-step ps, loaded and written at once (start of a run)
        auto prime = [&](const WsPos &ps, auto npc) {
            const i32x4 rsB = rsrc_of(Ag, ps.bg, a_img_bytes, true);
            const int total = P.kH * P.BWc * JC;
            const int pr0 = ps.y * P.sh, slot0 = ps.rowmod, ix0 = ps.strip * P.CW * P.sw - P.pw;
            // tasks in flight per thread: with 3, one round trip to memory covers 768 tasks (start of
            // the kernel, when the registers of the stages are still free); 1 inside the pipeline
            constexpr int NP = decltype(npc)::value;
            for (int base = 0; base < total; base += NP * kProducers) {
                u32x4 r[NP][8];
                XtTask t[NP];
#pragma unroll
                for (int u = 0; u < NP; ++u) {
                    const int idx = base + u * kProducers + p;
                    t[u] = xt_task(idx, idx < total, pr0, slot0, ix0);
#pragma unroll
                    for (int img = 0; img < 8; ++img) buf16_async(r[u][img], rsB, t[u].voff + (uint32_t)img * a_img_bytes);
                }
#pragma unroll
                for (int u = 0; u < NP; ++u) {
                    // needed right away; the loads of task u are older than those of the tasks after it
                    asm volatile("s_waitcnt vmcnt(%8)"
                                 : "+v"(r[u][0]), "+v"(r[u][1]), "+v"(r[u][2]), "+v"(r[u][3]), "+v"(r[u][4]), "+v"(r[u][5]),
                                   "+v"(r[u][6]), "+v"(r[u][7])
                                 : "n"((NP - 1 - u) * 8)
                                 : "memory");
                    uint4 src[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) src[q] = uint4{r[u][q].x, r[u][q].y, r[u][q].z, r[u][q].w};
                    if (base + u * kProducers + p < total) xt_store(t[u], src);
                }
            }
        };

        if (NI > 0) {
            WsPos pw = ws_pos_of(P, t_begin);  // sub-step whose data is written next
            WsPos pi = pw;                     // sub-step whose loads are issued next
            u32x4 st[D][NTASK][8];
            // The loads of the first sub-step go out first and stay in flight during the window's
            // round trip (one trip to memory instead of two before the first MFMA); the other stages
            // are issued after it, their registers being used by the window's loads meanwhile.
            issue(pi, true, st[0]);
            pi = ws_advance(P, pi);
            prime(pw, std::integral_constant<int, 3>{});
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
                        if (i > 0 && pw.u == 0 && pw.y == 0) {
                            ws_barrier();  // the consumers have left the previous run: its ring rows are free
                            prime(pw, std::integral_constant<int, 1>{});
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
static int ws_env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

static const size_t kWsLdsLimit = 160 * 1024;

size_t corr_ws_lds_bytes(const WsParams &P)
{
    return ((size_t)2 * P.a_units + (size_t)P.NRING * P.b_row_units) * 16;
}

// Fills the step geometry for a strip width CW cut into NSUB sub-steps; false if it does not fit.
static bool ws_geometry(WsParams &P, int CW, int NSUB)
{
    P.CW = CW;
    P.NSTRIP = ceil_div(P.Wo, CW);
    P.NSUB = NSUB;
    P.CWs = round_up(ceil_div(CW, NSUB), 4);
    if ((NSUB - 1) * P.CWs >= CW) return false;  // an empty last sub-step
    if (NSUB > 1 && P.NSTRIP > 1) return false;  // sub-steps only for whole rows
    P.BWc = (round_up(CW, 4) - 1) * P.sw + P.kW;
    P.NRING = P.kH + P.sh;
    P.a_units = round_up(P.CWs, 8) * P.M_WG;  // whole chunks of 8 slots: the producers store every slot of a chunk
    P.BSTR = P.J_WG;  // pixel stride = whole 256-byte bank rows: the four pixel slots of a fragment read then fall on the same banks, which is what ds_read_b128 wants
    P.b_row_units = P.BWc * P.BSTR;
    P.NA = P.M_WG * ceil_div(P.CWs, 8);
    P.NA_pad = round_up(P.NA, 64);
    const int rows_new = P.sh < P.kH ? P.sh : P.kH;
    P.TB = rows_new * P.BWc * (P.J_WG / 8);
    P.TS = ceil_div(P.TB, NSUB);
    P.NTASK = ceil_div(P.NA_pad + P.TS, kProducers);
    P.NS = P.NBG * P.NSTRIP * P.Ho;
    if (corr_ws_lds_bytes(P) > kWsLdsLimit) return false;
    // More than one task per producer thread does not fit the register file next to the
    // consumers' accumulators (the staged loads of D sub-steps live in registers).
    if (P.NTASK > 1) return false;
    return true;
}

bool plan_corr_ws(WsParams &P, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw, int CS)
{
    if (dtype == XCONV_F32) return false;
    if (ws_env_int("XCONV_CORR_WS", 1) == 0) return false;
    P = WsParams{};
    P.B = B; P.C_out = C_out; P.H = H; P.W = W;
    P.kH = kH; P.kW = kW; P.sh = sh; P.sw = sw; P.ph = ph; P.pw = pw;
    P.Ho = (H + 2 * ph - kH) / sh + 1;
    P.Wo = (W + 2 * pw - kW) / sw + 1;
    P.CS = CS;
    P.NBG = ceil_div(B, 8);
    P.K2 = kH * kW;
    if (P.K2 == 1) return false;          // 1x1 kernels have no halo to share: corr_kernel handles them
    if (kH > 8 || sh > 8) return false;    // rows added per row-step and rows of a window (xt_task)
    if (P.Wo % 2 != 0) return false;      // row starts of dY must be 4-byte aligned
    P.NOG = ceil_div(P.K2, 9);
    // a group of 8 images is addressed with 32-bit byte offsets
    if ((long long)8 * C_out * P.Ho * P.Wo * 2 > (1LL << 30) || (long long)8 * H * W * CS * 2 > (1LL << 30)) return false;

    // consumer waves: each owns 32 output channels x 32 columns; along the columns of A first
    // (those waves share the dY tile), WM * WJ = 4
    if (CS % 32 != 0) return false;
    const int nwj = CS / 32;
    int WJ = (nwj % 2 == 0) ? 2 : 1;
    if (C_out <= 32 && nwj % 4 == 0) WJ = 4;
    WJ = ws_env_int("XCONV_WS_WJ", WJ);
    if (WJ != 1 && WJ != 2 && WJ != 4) return false;
    if (nwj % WJ != 0) return false;
    const int WM = 4 / WJ;
    P.WM = WM; P.WJ = WJ; P.MT = 1;
    P.M_WG = WM * 32;
    P.J_WG = WJ * 32;
    P.NTM = ceil_div(C_out, P.M_WG);
    P.NTJ = CS / P.J_WG;
    P.MP = P.NTM * P.M_WG;
    P.JP = CS;

    // whole rows cut into sub-steps if the ring fits, else column strips
    bool found = false;
    const int fCW = ws_env_int("XCONV_WS_CW", 0), fNSUB = ws_env_int("XCONV_WS_NSUB", 0);
    if (fCW > 0 && fNSUB > 0 && fNSUB <= 2) {
        found = ws_geometry(P, fCW, fNSUB);
    } else {
        WsParams best = P;
        int best_ntask = 99, best_cws = 0;
        for (int nsub = 1; nsub <= 2; ++nsub) {  // the producers keep per-slice constants for two slices
            WsParams Q = P;
            if (!ws_geometry(Q, P.Wo, nsub)) continue;
            if (Q.CWs > 32) continue;
            if (Q.NTASK < best_ntask || (Q.NTASK == best_ntask && Q.CWs > best_cws)) { best = Q; best_ntask = Q.NTASK; best_cws = Q.CWs; found = true; }
        }
        if (!found) {
            for (int cw = 32; cw >= 8; cw -= 4) {
                if (cw >= P.Wo) continue;
                WsParams Q = P;
                if (!ws_geometry(Q, cw, 1)) continue;
                // prefer few tasks per thread, then little padding in the last strip, then wide strips
                const int waste = Q.NSTRIP * round_up(cw, 4) - P.Wo;
                const int score = Q.NTASK * 1000 + waste * 10 - cw / 4;
                if (!found || score < best_ntask) { best = Q; best_ntask = score; found = true; }
            }
        }
        if (found) P = best;
    }
    if (!found) return false;

    // K-split: one workgroup per compute unit
    const int ny = P.NTM * P.NTJ * P.NOG;
    int target = ws_env_int("XCONV_WS_SPLITS", 0);
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

template <int DT, int NTASK, int D, int CB, bool RU, bool VOL>
static hipError_t launch_ws_vol(const WsParams &P, hipStream_t st)
{
    const size_t lds = corr_ws_lds_bytes(P);
    static bool done = false;  // per instantiation: the attribute sticks to the function
    if (!done && lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(corr_ws_kernel<DT, 9, NTASK, D, CB, RU, VOL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kWsLdsLimit);
        if (e != hipSuccess) return e;
        done = true;
    }
    WsParams Q = P;
    Q.SQ = P.NS / P.S;
    Q.SR = P.NS % P.S;
    hipLaunchKernelGGL((corr_ws_kernel<DT, 9, NTASK, D, CB, RU, VOL>), dim3(P.S, P.NTM * P.NTJ, P.NOG), dim3(kWsThreads), lds, st, Q);
    return hipGetLastError();
}

template <int DT, int NTASK, int D, int CB, bool RU>
static hipError_t launch_ws_cfg(const WsParams &P, hipStream_t st)
{
    if (P.vol_period != 0) return launch_ws_vol<DT, NTASK, D, CB, RU, true>(P, st);
    return launch_ws_vol<DT, NTASK, D, CB, RU, false>(P, st);
}

template <int DT> static hipError_t launch_ws_dt(const WsParams &P, hipStream_t st)
{
    // (plan_corr_ws only accepts plans with one task per producer thread)
    static const bool generic = ws_env_int("XCONV_WS_GENERIC", 0) != 0;
    if (!generic && P.K2 == 9 && P.kW == 3) {
        // unit stride: fragments are reused along the staged row
        static const bool reuse = ws_env_int("XCONV_WS_REUSE", 1) != 0;
        if (reuse && P.sw == 1 && P.kH == 3) {
            switch (P.BSTR) {
            case 32: return launch_ws_cfg<DT, 1, 3, 32 * 16, true>(P, st);
            case 64: return launch_ws_cfg<DT, 1, 3, 64 * 16, true>(P, st);
            case 128: return launch_ws_cfg<DT, 1, 3, 128 * 16, true>(P, st);
            default: break;
            }
        }
        switch (P.BSTR) {
        case 32: return launch_ws_cfg<DT, 1, 3, 32 * 16, false>(P, st);
        case 64: return launch_ws_cfg<DT, 1, 3, 64 * 16, false>(P, st);
        case 128: return launch_ws_cfg<DT, 1, 3, 128 * 16, false>(P, st);
        default: break;
        }
    }
    return launch_ws_cfg<DT, 1, 3, 0, false>(P, st);
}

hipError_t launch_corr_ws(int dtype, const WsParams &P, hipStream_t st)
{
    if (dtype == XCONV_BF16) return launch_ws_dt<XCONV_BF16>(P, st);
    return launch_ws_dt<XCONV_F16>(P, st);
}

}  // namespace xc
