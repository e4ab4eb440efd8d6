// Epilogue shared by the split-K kernels: from the four waves' partial tiles in LDS to Y.
//
// With one slab (S == 1) the workgroup scales and stores its tile.  With S > 1 every slab writes
// its partial B tile and partial A (sums of squares) through to memory with device-scope stores,
// (16 bytes per lane, whole cache lines per wave), waits for them, and bumps the tile's arrival counter; the last workgroup to arrive adds the S
// partials in slab order -- so the sum does not depend on arrival order and a launch shape is
// bit-reproducible -- applies 1/sqrt(A/K + eps), rounds once and stores.  The counter is left at
// zero for the next call.  No float atomics, no cache-wide write-back or invalidate.
#pragma once
#include <type_traits>
#include "common.hpp"

namespace rmsnl {

constexpr int kSumsqStride = 64;     // floats per (tile, slab) in ws_sumsq: room for 64 rows

struct TailArgs {
    u16* Y;          // (floats behind it when the kernel's type is float)
    int M, N;        // N: columns of W (= row length of the partial workspace, and of Y unless gated)
    int n_live;      // columns of the tile that belong to it (<= N_TILE)
    int half;        // gated block: the tile's first `half` columns are gate columns hn0.., the next `half` the
    int H;           //   up columns of the same outputs, and Y [M][H] gets SiLU(gate) * up; half = 0: plain block
    int G;           // gated block: where those columns lie in W, see gated_col()
    float eps, inv_K;
    int S;
    float* ws_partial; float* ws_sumsq; unsigned* counter;
    unsigned long long* trace; int trace_groups;
};

// NW waves per workgroup (4 or 8).  red: [NW][MT][N_TILE] fp32 in LDS (one copy per wave), complete
// and visible (barrier passed); s_sumsq: [NW][MT] per-wave partial sums of squares; s_rinv: [MT]
// scratch; s_last: 1 int scratch.
template <typename T, int MT, int N_TILE, bool FUSED, int NW = 4, bool GATED = false>
__device__ __forceinline__ void splitk_tail(const TailArgs& a, const float* red, const float* s_sumsq,
                                            float* s_rinv, int* s_last_p, int tile, int slab, int n0)
{
    // n0: first W column of the tile (plain), or first column hn0 of the tile inside each half (gated)
    const int tid = threadIdx.x;
    constexpr int NT = 64 * NW;              // threads
    constexpr int QUADS = MT * N_TILE / 4;   // groups of 4 columns in the tile, the threads share them
    constexpr int QPT = (QUADS + NT - 1) / NT; // quads per thread
    constexpr int WSTR = MT * N_TILE / 4;    // float4 stride between the waves' copies in red
    constexpr int kDev = 16;                 // buffer cache policy sc1: device scope, across XCDs
    float asum = 0.f;
    typedef Arith<T> Ar;                     // fp32 for the floating types; pairs over two fields for Ff
    if (FUSED && tid < MT) {
        asum = Ar::add(Ar::add(s_sumsq[tid], s_sumsq[MT + tid]), Ar::add(s_sumsq[2 * MT + tid], s_sumsq[3 * MT + tid]));
        if (NW == 8)
            asum = Ar::add(asum, Ar::add(Ar::add(s_sumsq[4 * MT + tid], s_sumsq[5 * MT + tid]),
                                         Ar::add(s_sumsq[6 * MT + tid], s_sumsq[7 * MT + tid])));
    }

    // sum of the waves' copies of a quad of the tile, in a fixed order
    auto wg_sum = [&](int m, int c) {
        const float4_t* q = (const float4_t*)(red + m * N_TILE + c);
        float4_t v = Ar::add4(Ar::add4(q[0], q[WSTR]), Ar::add4(q[2 * WSTR], q[3 * WSTR]));
        if (NW == 8) v = Ar::add4(v, Ar::add4(Ar::add4(q[4 * WSTR], q[5 * WSTR]), Ar::add4(q[6 * WSTR], q[7 * WSTR])));
        return v;
    };
    // tile-local quad (m, c): is it inside the problem, and where are its columns in W
    auto live = [&](int m, int c) {
        if (GATED) return m < a.M && c < 2 * a.half && n0 + (c < a.half ? c : c - a.half) < a.H;
        return m < a.M && c < a.n_live && n0 + c < a.N;
    };
    auto wcol = [&](int c) {
        if (GATED) return gated_col(n0 + (c < a.half ? c : c - a.half), c >= a.half, a.H, a.G);
        return n0 + c;
    };
    // plain block: Y = B * rinv.  Gated block: the quad is a gate quad, u the up quad of the same
    // outputs; Y = SiLU(gate * rinv) * (up * rinv), Y's rows are H long.
    auto store_y = [&](int m, int c, float4_t v, float4_t u, float ri) {
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = GATED ? Ar::out_gated(v[e], u[e], ri, a.eps) : Ar::out(v[e], ri, a.eps);
        if constexpr (std::is_same<T, float>::value) {      // 4-byte elements: Y points at floats
            *(float4_t*)((float*)a.Y + size_t(m) * (GATED ? a.H : a.N) + n0 + c) = float4_t{y[0], y[1], y[2], y[3]};
        } else {
            uint2_t o = {Elem<T>::pack(y[0], y[1]), Elem<T>::pack(y[2], y[3])};
            *(uint2_t*)(a.Y + size_t(m) * (GATED ? a.H : a.N) + n0 + c) = o;
        }
    };
    const float4_t kZero4 = {0.f, 0.f, 0.f, 0.f};

    if (a.S == 1) {
        if (tid < MT) s_rinv[tid] = FUSED ? Ar::rinv(asum, a.inv_K, a.eps) : Ar::one();
        __syncthreads();
        if (GATED && 2 * a.half == N_TILE) {
            // full-width gated tile: one thread per output quad, so that no thread sits out on an up quad
            constexpr int HQ = N_TILE / 8;   // output quads per row
#pragma unroll
            for (int qi = 0; qi < (QPT + 1) / 2; ++qi) {
                const int p = tid + qi * NT;
                const int m = p / HQ, c = (p % HQ) * 4;
                if (p < MT * HQ && live(m, c)) store_y(m, c, wg_sum(m, c), wg_sum(m, c + a.half), s_rinv[m]);
            }
            return;
        }
#pragma unroll
        for (int qi = 0; qi < QPT; ++qi) {
            const int p = tid + qi * NT;
            const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
            if (p < QUADS && live(m, c) && (!GATED || c < a.half))
                store_y(m, c, wg_sum(m, c), GATED ? wg_sum(m, c + a.half) : kZero4, s_rinv[m]);
        }
        return;
    }

    // ---- split-K.  Partials go out as 16-byte device-scope stores (written through, whole lines
    // per wave; no cache-wide write-back is needed to publish them); every wave waits for its own
    // stores, the workgroup meets at a barrier, and only then one thread bumps the tile's counter.
    const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(
        a.ws_partial, 0, int(size_t(a.S) * a.M * a.N * 4), 0x00020000);
    const int slab_bytes = a.M * a.N * 4;
    if (FUSED && tid < MT) st_dev(a.ws_sumsq + (tile * a.S + slab) * kSumsqStride + tid, asum);
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) {
        const int p = tid + qi * NT;
        const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
        if (p < QUADS && live(m, c)) {
            const float4_t v = wg_sum(m, c);
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4_t, v), prs,
                                                   slab * slab_bytes + (m * a.N + wcol(c)) * 4, 0, kDev);
        }
    }
    __builtin_amdgcn_s_waitcnt(0);           // this wave's stores have been acknowledged
    __syncthreads();
    trace_stamp(a.trace, a.trace_groups, 4);         // partials published
    if (tid == 0) {
        unsigned prev = __hip_atomic_fetch_add(a.counter + tile * kCounterStride, 1u, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
        *s_last_p = (prev == unsigned(a.S - 1));
    }
    __syncthreads();
    trace_stamp(a.trace, a.trace_groups, 5);         // counter bumped
    if (!*s_last_p) return;

    // ---- last arriver: device-scope loads see what the other slabs wrote through.  A round trip
    // to the memory side of the fabric costs microseconds here, so every thread asks for all the
    // slabs' shares of its quads, and of its rows' sums of squares, before it uses any of them, and
    // adds them in slab order once they are in.  No barrier, no LDS in this part.  (Gated block: a
    // thread whose quad is a gate quad also fetches the up quad of the same outputs; threads on
    // up quads have nothing to store.)
    constexpr int NQ = GATED ? 2 : 1;
    constexpr int SB = (QPT >= 8 ? 4 : QPT >= 4 ? 8 : 16) / NQ;   // slabs per batch: QPT * NQ * SB <= 32 loads of each kind in flight
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(
        a.ws_sumsq + size_t(tile) * a.S * kSumsqStride, 0, a.S * kSumsqStride * 4, 0x00020000);
    constexpr int kNowhere = 0x7ffffff0;     // beyond either resource: reads as zero
    float4_t yv[QPT][NQ];
    float asq[QPT];
    int poff[QPT][NQ], soff[QPT];            // byte offsets; kNowhere plus any slab offset stays out of range (sizes < 2^31)
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) {
        const int p = tid + qi * NT;
        const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
        const bool ok = p < QUADS && live(m, c) && (!GATED || c < a.half);
        poff[qi][0] = ok ? (m * a.N + wcol(c)) * 4 : kNowhere;
        if (GATED) poff[qi][1] = ok ? (m * a.N + wcol(c + a.half)) * 4 : kNowhere;
        soff[qi] = ok ? m * 4 : kNowhere;
#pragma unroll
        for (int h = 0; h < NQ; ++h) yv[qi][h] = kZero4;
        asq[qi] = 0.f;
    }
    // B slabs per batch (slabs at or beyond S are out of range and read as zero, but every load still
    // takes its turn in the address unit: a batch no longer than the slab count needs, and none at all
    // in a wave without a live quad)
    auto gather = [&](auto batch) {
        constexpr int B = decltype(batch)::value;
        for (int s0 = 0; s0 < a.S; s0 += B) {
            uint4_t q[QPT][NQ][B];
            float u[QPT][B];
#pragma unroll
            for (int qi = 0; qi < QPT; ++qi)
#pragma unroll
                for (int j = 0; j < B; ++j) {
                    // the whole offset goes through the range check (a scalar offset would not)
#pragma unroll
                    for (int h = 0; h < NQ; ++h)
                        q[qi][h][j] = __builtin_amdgcn_raw_buffer_load_b128(
                            prs, int(unsigned(poff[qi][h]) + unsigned((s0 + j) * slab_bytes)), 0, kDev);
                    if (FUSED)
                        u[qi][j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                            srs, int(unsigned(soff[qi]) + unsigned((s0 + j) * kSumsqStride * 4)), 0, kDev));
                }
#pragma unroll
            for (int qi = 0; qi < QPT; ++qi)
#pragma unroll
                for (int j = 0; j < B; ++j) {
#pragma unroll
                    for (int h = 0; h < NQ; ++h) yv[qi][h] = Ar::add4(yv[qi][h], __builtin_bit_cast(float4_t, q[qi][h][j]));
                    if (FUSED) asq[qi] = Ar::add(asq[qi], u[qi][j]);
                }
        }
    };
    bool live_here = false;
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) live_here |= poff[qi][0] != kNowhere;
    if (__builtin_amdgcn_ballot_w64(live_here) != 0) {   // uniform over the wave
        bool done = false;
        if constexpr (SB > 2) if (!done && a.S <= 2) { gather(std::integral_constant<int, 2>{}); done = true; }
        if constexpr (SB > 4) if (!done && a.S <= 4) { gather(std::integral_constant<int, 4>{}); done = true; }
        if constexpr (SB > 8) if (!done && a.S <= 8) { gather(std::integral_constant<int, 8>{}); done = true; }
        if (!done) gather(std::integral_constant<int, SB>{});
    }
    trace_stamp(a.trace, a.trace_groups, 6);         // all slabs' partials read
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) {
        const int p = tid + qi * NT;
        const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
        if (poff[qi][0] != kNowhere)
            store_y(m, c, yv[qi][0], yv[qi][NQ - 1], FUSED ? Ar::rinv(asq[qi], a.inv_K, a.eps) : Ar::one());
    }
    trace_stamp(a.trace, a.trace_groups, 7);         // Y stored
    if (tid == 0)                            // ready for the next call on this stream
        __hip_atomic_store(a.counter + tile * kCounterStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace rmsnl
