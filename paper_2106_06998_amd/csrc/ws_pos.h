// Shared by the producer/consumer correlation kernels: positions of the steps a workgroup walks
// through (wave-uniform), the barrier that orders LDS traffic only, small compile-time helpers.
#pragma once
#include <type_traits>

#include "common.h"

namespace xc {
namespace {

constexpr int kWsThreads = 512;
constexpr int kProducers = 256;
constexpr uint32_t kOOR = 0x80000000u;  // beyond any buffer resource (a group of 8 images stays below 2^30 bytes)

__device__ inline void ws_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Position of a sub-step; every field is wave-uniform.
struct WsPos {
    int u;       // sub-step inside the row-step
    int y;       // output row
    int strip;   // column strip
    int bg;      // group of 8 images
    int rowmod;  // (y * sh) mod NRING: ring slot of the first input row of the window
    int t;       // row-step index
};

__device__ inline WsPos ws_uniform(WsPos p)
{
    p.u = __builtin_amdgcn_readfirstlane(p.u);
    p.y = __builtin_amdgcn_readfirstlane(p.y);
    p.strip = __builtin_amdgcn_readfirstlane(p.strip);
    p.bg = __builtin_amdgcn_readfirstlane(p.bg);
    p.rowmod = __builtin_amdgcn_readfirstlane(p.rowmod);
    p.t = __builtin_amdgcn_readfirstlane(p.t);
    return p;
}

__device__ inline WsPos ws_pos_of(const WsParams &P, int t)
{
    WsPos p;
    p.t = t;
    p.u = 0;
    if (t < (1 << 22)) {
        int q;
        fast_divmod(t, P.Ho, frcp(P.Ho), q, p.y);
        fast_divmod(q, P.NSTRIP, frcp(P.NSTRIP), p.bg, p.strip);
    } else {
        p.y = t % P.Ho;
        const int q = t / P.Ho;
        p.strip = q % P.NSTRIP;
        p.bg = q / P.NSTRIP;
    }
    int qr;
    fast_divmod(p.y * P.sh, P.NRING, frcp(P.NRING), qr, p.rowmod);
    return ws_uniform(p);
}

__device__ inline WsPos ws_next_row(const WsParams &P, WsPos p)
{
    ++p.t;
    p.rowmod += P.sh;
    while (p.rowmod >= P.NRING) p.rowmod -= P.NRING;
    if (++p.y == P.Ho) {
        p.y = 0;
        p.rowmod = 0;
        if (++p.strip == P.NSTRIP) {
            p.strip = 0;
            ++p.bg;
        }
    }
    return p;
}

__device__ inline WsPos ws_advance(const WsParams &P, WsPos p)
{
    if (++p.u == P.NSUB) {
        p.u = 0;
        p = ws_next_row(P, p);
    }
    return ws_uniform(p);
}

// output columns of the sub-step that exist (the rest of its CWs slots is zero padding)
__device__ inline int ws_cw_sub(const WsParams &P, const WsPos &p)
{
    const int x0 = p.strip * P.CW;
    int cw = P.Wo - x0;
    cw = cw < P.CW ? cw : P.CW;
    cw -= p.u * P.CWs;
    return cw < P.CWs ? cw : P.CWs;
}

template <int Q, int N, class F> __device__ inline void ws_static_for(F &&f)
{
    if constexpr (Q < N) {
        f(std::integral_constant<int, Q>{});
        ws_static_for<Q + 1, N>(f);
    }
}

}  // namespace
}  // namespace xc
