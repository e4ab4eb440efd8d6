// Epilogue shared by the split-K kernels: from the four waves' partial tiles in LDS to Y.
//
// With one slab (S == 1) the workgroup scales and stores its tile.  With S > 1 every slab writes
// its partial B tile and partial A (sums of squares) through to memory with device-scope stores,
// (16 bytes per lane, whole cache lines per wave), waits for them, and bumps the tile's arrival counter; the last workgroup to arrive adds the S
// partials in slab order -- so the sum does not depend on arrival order and a launch shape is
// bit-reproducible -- applies 1/sqrt(A/K + eps), rounds once and stores.  The counter is left at
// zero for the next call.  No float atomics, no cache-wide write-back or invalidate.
#pragma once
#include "common.hpp"

namespace rmsnl {

constexpr int kSumsqStride = 64;     // floats per (tile, slab) in ws_sumsq: room for 64 rows

struct TailArgs {
    u16* Y;
    int M, N;
    int n_live;      // columns of the tile that belong to it (<= N_TILE)
    float eps, inv_K;
    int S;
    float* ws_partial; float* ws_sumsq; unsigned* counter;
    unsigned long long* trace; int trace_groups;
};

// red: [4][MT][N_TILE] fp32 in LDS (one copy per wave), complete and visible (barrier passed);
// s_sumsq: [4][MT] per-wave partial sums of squares; s_rinv: [MT] scratch; s_last: 1 int scratch.
template <typename T, int MT, int N_TILE, bool FUSED>
__device__ __forceinline__ void splitk_tail(const TailArgs& a, const float* red, const float* s_sumsq,
                                            float* s_rinv, int* s_last_p, int tile, int slab, int n0)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int QUADS = MT * N_TILE / 4;   // groups of 4 columns in the tile, 256 threads share them
    constexpr int QPT = (QUADS + 255) / 256; // quads per thread
    constexpr int WSTR = MT * N_TILE / 4;    // float4 stride between the waves' copies in red
    constexpr int kDev = 16;                 // buffer cache policy sc1: device scope, across XCDs
    float asum = 0.f;
    if (FUSED && tid < MT) asum = (s_sumsq[tid] + s_sumsq[MT + tid]) + (s_sumsq[2 * MT + tid] + s_sumsq[3 * MT + tid]);

    // sum of the four waves' copies of quad p of the tile
    auto wg_sum = [&](int m, int c) {
        const float4_t* q = (const float4_t*)(red + m * N_TILE + c);
        return (q[0] + q[WSTR]) + (q[2 * WSTR] + q[3 * WSTR]);
    };
    auto store_y = [&](int m, int c, float4_t v, float ri) {
        uint2_t o = {Elem<T>::pack(v[0] * ri, v[1] * ri), Elem<T>::pack(v[2] * ri, v[3] * ri)};
        *(uint2_t*)(a.Y + size_t(m) * a.N + n0 + c) = o;
    };

    if (a.S == 1) {
        if (tid < MT) s_rinv[tid] = FUSED ? row_scale(asum, a.inv_K, a.eps) : 1.f;
        __syncthreads();
#pragma unroll
        for (int qi = 0; qi < QPT; ++qi) {
            const int p = tid + qi * 256;
            const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
            if (p < QUADS && m < a.M && c < a.n_live && n0 + c < a.N) store_y(m, c, wg_sum(m, c), s_rinv[m]);
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
        const int p = tid + qi * 256;
        const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
        if (p < QUADS && m < a.M && c < a.n_live && n0 + c < a.N) {
            const float4_t v = wg_sum(m, c);
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4_t, v), prs,
                                                   slab * slab_bytes + (m * a.N + n0 + c) * 4, 0, kDev);
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

    // ---- last arriver: device-scope loads see what the other slabs wrote through.
    // A_i: lane m of wave 3 reads row m's S partial sums of squares (consecutive lanes read
    // consecutive floats), sixteen loads in flight, and adds them in slab order.
    if (wave == 3 && lane < MT) {
        float t = 0.f;
        if (FUSED) {
            const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(
                a.ws_sumsq + size_t(tile) * a.S * kSumsqStride, 0, a.S * kSumsqStride * 4, 0x00020000);
            for (int s0 = 0; s0 < a.S; s0 += 16) {
                float u[16];
#pragma unroll
                for (int j = 0; j < 16; ++j)         // slabs at or beyond S are out of range: zero
                    u[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(srs, ((s0 + j) * kSumsqStride + lane) * 4, 0, kDev));
#pragma unroll
                for (int j = 0; j < 16; ++j) t += u[j];
            }
        }
        s_rinv[lane] = FUSED ? row_scale(t, a.inv_K, a.eps) : 1.f;
    }
    float4_t yv[QPT];
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) {
        const int p = tid + qi * 256;
        const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
        float4_t v = {0.f, 0.f, 0.f, 0.f};
        if (p < QUADS && m < a.M && c < a.n_live && n0 + c < a.N) {
            const int off = (m * a.N + n0 + c) * 4;
            for (int s0 = 0; s0 < a.S; s0 += 8) {    // eight loads in flight, added in slab order
                uint4_t q[8];
#pragma unroll
                for (int j = 0; j < 8; ++j)          // slabs at or beyond S are out of range: zero
                    q[j] = __builtin_amdgcn_raw_buffer_load_b128(prs, (s0 + j) * slab_bytes + off, 0, kDev);
#pragma unroll
                for (int j = 0; j < 8; ++j) v += __builtin_bit_cast(float4_t, q[j]);
            }
        }
        yv[qi] = v;
    }
    __syncthreads();                         // s_rinv is ready
    trace_stamp(a.trace, a.trace_groups, 6);         // all slabs' partials read
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) {
        const int p = tid + qi * 256;
        const int m = p / (N_TILE / 4), c = (p % (N_TILE / 4)) * 4;
        if (p < QUADS && m < a.M && c < a.n_live && n0 + c < a.N) store_y(m, c, yv[qi], s_rinv[m]);
    }
    trace_stamp(a.trace, a.trace_groups, 7);         // Y stored
    if (tid == 0)                            // ready for the next call on this stream
        __hip_atomic_store(a.counter + tile * kCounterStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace rmsnl
