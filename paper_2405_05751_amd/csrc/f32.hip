// The fp32 path of the fused block on the matrix cores (v_mfma_f32_16x16x4_f32: fp32 products, fp32
// sums), for every M: the case study's Fig. 2b again -- A_i = sum_k X_ik^2 and B_in = sum_k (X_ik g_k)
// W_kn in one K loop, the division by the root mean square after it -- on 4-byte elements.
//
// A workgroup (4 waves) owns 16 MB rows (MB = 1..4) x 64 columns of Y over one K slab; its waves
// take the slab's 16-row runs of W in turn.  fp32 matrix instructions are slow enough (64 flops
// per clock and SIMD) that operands straight from the caches keep them fed: nothing is staged
// through LDS in the K loop.
//   W: lane (c, q) = (lane % 16, lane / 16) loads rows k + 4 q + t, t = 0..3, columns n0 + 4 c .. + 3:
//      four loads of 4 rows x 256 contiguous bytes;
//   X: the same lane loads row 16 mb + c, elements k + 4 q .. + 3 (and g's), 16 bytes;
//   step t feeds element t of the X registers and, for j = 0..3, element j of W load t into the
//   instruction for columns n0 + 4 c' + j: the k of a lane group is k + 4 q + t on both sides.
// Sums: a matrix accumulator takes 128 k (8 runs) and is then added into a second accumulator, and
// so are the squares, so that the rounding error grows with sqrt(128) + sqrt(K / 512) ulps and not
// with sqrt(K); the waves' tiles are added in LDS, K slabs through the workspace by the last
// workgroup to arrive, in slab order (the epilogue the 16-bit split-K kernels use).
// M > 64: a row block per 64 rows in the same launch; workgroups that read the same rows of X or
// columns of W are neighbours on one XCD.
#include <algorithm>
#include "splitk.hpp"

namespace rmsnl {

constexpr int kF32Tile = 64;          // columns of W per workgroup
constexpr int kF32Chunk = 8;          // runs per first-level accumulator
// runs in flight per wave: 3, and 4 from 33 rows on (a unit's loads are then the scarcer side: 2 runs measured
// 20 % slower than 3 at 64 rows, 4 another 3.5 % faster; with 1 to 16 rows 4 is no gain)
constexpr int f32_ring(int MB) { return MB >= 3 ? 4 : 3; }
constexpr int kF32Out = -16;          // as a byte offset 0xfffffff0, beyond every buffer resource: reads zero
constexpr int kF32Flags = 0x00020000;

struct F32Args {
    const float* X; const float* g; const float* W; float* Y;
    int M, K, N;
    float eps, inv_K;
    int k_slab, S, n_tiles, RB;       // rows of W per slab (a multiple of 64), slabs, column tiles, row blocks
    int H, G;                         // gated block: outputs (N = 2 H) and the layout of W, see gated_col()
    float* ws_partial; float* ws_sumsq; unsigned* counter;
};

// GATED (the GatedMLP block on top): the tile's first 32 columns are the gate columns of 32 outputs, the
// next 32 their up columns; the epilogue forms SiLU(gate) * up.  Only the column a lane fetches changes.
template <int MB, bool FUSED, bool GATED>
__global__ __launch_bounds__(256) void f32_kernel(F32Args a)
{
    constexpr int MT = 16 * MB, D = f32_ring(MB);
    extern __shared__ __attribute__((aligned(16))) float smem[];      // red [4][MT][64]
    __shared__ float s_sumsq[4][MT];
    __shared__ float s_rinv[MT];
    __shared__ int s_last;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, q = lane >> 4;

    // consecutive workgroups go to the 8 XCDs in turn: renumber so that an XCD sees a run of
    // consecutive numbers, and number the workgroups in panels of 4 column tiles, inside a panel the
    // tile fastest, then the row block, then the slab: the 32 workgroups an XCD runs together are
    // 8 row blocks x 4 column tiles, which share their rows of X and columns of W in its L2
    int bid = blockIdx.x;
    const int G = gridDim.x;
    if ((G & 7) == 0) bid = (bid & 7) * (G >> 3) + (bid >> 3);
    const int per_panel = 4 * a.RB * a.S;
    const int panel = bid / per_panel;
    int idx = bid - panel * per_panel;
    const int pw = min(4, a.n_tiles - 4 * panel);       // the last panel may be narrower
    const int tile = 4 * panel + idx % pw;
    idx /= pw;
    const int rb = idx % a.RB;
    const int slab = idx / a.RB;
    const int n0 = tile * (GATED ? kF32Tile / 2 : kF32Tile), m0 = rb * 64;   // gated: first output of the tile
    const int Mh = min(a.M - m0, 64);                   // rows of this row block
    const int k0 = slab * a.k_slab, Kend = min(a.K, k0 + a.k_slab);
    const int nIter = (Kend - k0 + 63) >> 6;            // uniform: runs per wave

    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(a.X + size_t(m0) * a.K), 0, int(unsigned(Mh) * unsigned(a.K) * 4u), kF32Flags);
    const __amdgpu_buffer_rsrc_t grs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(FUSED ? a.g : a.X), 0, a.K * 4, kF32Flags);
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(a.W), 0, int(unsigned(Kend) * unsigned(a.N) * 4u), kF32Flags);
    // N % 4 == 0 (gated: H % 4 == 0): a lane's four columns lie inside together, next to each other in W
    const bool up = GATED && 4 * c >= kF32Tile / 2;
    const int hcol = n0 + (up ? 4 * c - kF32Tile / 2 : 4 * c);
    const bool col_ok = hcol < (GATED ? a.H : a.N);
    const int wcol = GATED ? gated_col(hcol, up, a.H, a.G) : hcol;
    unsigned xrow[MB];                                  // byte offset of the lane's row inside the row block
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) xrow[mb] = unsigned(16 * mb + c) * unsigned(a.K) * 4u;

    float4_t wv[D][4], xv[D][MB], gv[D];
    // Every load is issued whether or not its run exists (k at or beyond the slab's end: the
    // offset that reads zero, at no memory traffic), in a pinned order, so that the compiler can
    // count the loads younger than the one it waits for.
    auto issue = [&](int it, int r) {
        const int kk = k0 + 64 * it + 16 * wave + 4 * q;
        const bool kin = kk < Kend;                     // K % 4 == 0: the lane's four k lie inside together
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const unsigned off = (unsigned(kk + t) * unsigned(a.N) + unsigned(wcol)) * 4u;
            wv[r][t] = __builtin_bit_cast(float4_t, __builtin_amdgcn_raw_buffer_load_b128(
                wrs, kin && col_ok ? int(off) : kF32Out, 0, 0));
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            xv[r][mb] = __builtin_bit_cast(float4_t, __builtin_amdgcn_raw_buffer_load_b128(
                xrs, kin ? int(xrow[mb] + unsigned(kk) * 4u) : kF32Out, 0, 0));
        if (FUSED)
            gv[r] = __builtin_bit_cast(float4_t, __builtin_amdgcn_raw_buffer_load_b128(grs, kin ? kk * 4 : kF32Out, 0, 0));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };

    float4_t acc[MB][4], tot[MB][4];
    float ss[MB], ss_tot[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        ss[mb] = ss_tot[mb] = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[mb][j] = tot[mb][j] = float4_t{0.f, 0.f, 0.f, 0.f};
    }
    auto fold = [&]() {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            ss_tot[mb] += ss[mb];
            ss[mb] = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) { tot[mb][j] += acc[mb][j]; acc[mb][j] = float4_t{0.f, 0.f, 0.f, 0.f}; }
        }
    };
    auto consume = [&](int r) {
        float4_t xh[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const float4_t x = xv[r][mb];
            if (FUSED) {
#pragma unroll
                for (int t = 0; t < 4; ++t) ss[mb] = __fmaf_rn(x[t], x[t], ss[mb]);
                xh[mb] = x * gv[r];
            } else {
                xh[mb] = x;
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[mb][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(xh[mb][t], wv[r][t][j], acc[mb][j], 0, 0, 0);
    };

#pragma unroll
    for (int r = 0; r < D; ++r) issue(r, r);
    int in_chunk = 0;
    for (int i0 = 0; i0 < nIter; i0 += D) {
#pragma unroll
        for (int r = 0; r < D; ++r) {
            if (i0 + r < nIter) {                       // uniform; only the arithmetic is skipped
                consume(r);
                if (++in_chunk == kF32Chunk) { fold(); in_chunk = 0; }
            }
            issue(i0 + r + D, r);
        }
    }
    fold();

    // ---- A_i: add the four k groups of the wave (lanes c, c + 16, c + 32, c + 48 hold row c's shares)
    if (FUSED) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float v = ss_tot[mb];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (q == 0) s_sumsq[wave][mb * 16 + c] = v;
        }
    }
    // ---- B: element i of accumulator (mb, j) is row 16 mb + 4 q + i, column 4 c + j of the tile
    float* red = smem;                                  // [4][MT][64]
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *(float4_t*)(red + (wave * MT + mb * 16 + q * 4 + i) * kF32Tile + 4 * c) =
                float4_t{tot[mb][0][i], tot[mb][1][i], tot[mb][2][i], tot[mb][3][i]};
    __syncthreads();

    // every row block is a problem of its own to the epilogue: its rows of Y, its share of the workspace
    TailArgs ta{(u16*)(a.Y + size_t(m0) * (GATED ? a.H : a.N)), Mh, a.N, kF32Tile, GATED ? kF32Tile / 2 : 0, a.H, a.G,
                a.eps, a.inv_K, a.S,
                a.ws_partial ? a.ws_partial + size_t(rb) * a.S * 64 * a.N : nullptr,
                a.ws_sumsq ? a.ws_sumsq + size_t(rb) * a.n_tiles * a.S * kSumsqStride : nullptr,
                a.counter ? a.counter + size_t(rb) * a.n_tiles * kCounterStride : nullptr, nullptr, 0};
    splitk_tail<float, MT, kF32Tile, FUSED, 4, GATED>(ta, red, &s_sumsq[0][0], s_rinv, &s_last, tile, slab, n0);
}

// ------------------------------------------------------------------------------------------- host
struct F32Plan { int MB, RB, S, k_slab, n_tiles; size_t lds; bool ok; const char* why; };

static F32Plan f32_plan(const Problem& p)
{
    F32Plan pl{};
    pl.ok = false;
    if (p.dt != F32) { pl.why = "the fp32 matrix-core variant handles fp32 only"; return pl; }
    if (p.gated && (!p.fused || p.N % 8 != 0)) { pl.why = "gated block: the fp32 matrix-core variant needs H % 4 == 0"; return pl; }
    if (p.rscale) { pl.why = "the fp32 matrix-core variant takes no row factors"; return pl; }
    if (p.N % 4 != 0 || p.K % 4 != 0) { pl.why = "the fp32 matrix-core variant needs N % 4 == 0 and K % 4 == 0"; return pl; }
    if (p.n_tile != 0 && p.n_tile != kF32Tile) { pl.why = "the fp32 matrix-core variant has 64-column tiles"; return pl; }
    if (p.k_split < 0 || p.k_split > 16) { pl.why = "the fp32 matrix-core variant takes 1 to 16 K slabs"; return pl; }
    // byte offsets are 32-bit: all of W, and 64 rows of X, below 4 GiB
    if (int64_t(p.K) * p.N * 4 >= (int64_t(1) << 32) - 256 || int64_t(p.K) * 64 * 4 >= (int64_t(1) << 32) - 256) {
        pl.why = "the fp32 matrix-core variant needs K N < 2^30 and K < 2^24";
        return pl;
    }
    pl.RB = (p.M + 63) / 64;
    pl.MB = pl.RB > 1 ? 4 : (p.M + 15) / 16;
    pl.n_tiles = p.gated ? (p.N / 2 + kF32Tile / 2 - 1) / (kF32Tile / 2) : (p.N + kF32Tile - 1) / kF32Tile;
    const int runs = (p.K + 63) / 64;                    // 64 rows of W: one run for each wave
    const int Mb = std::min(p.M, 64);
    int S = p.k_split;
    if (S == 0) {
        // as many slabs as still give every workgroup a compute unit of its own (a sweep of 1 to 16 slabs over 14
        // shapes, M 1 to 128: the best count was the largest with at most 256 workgroups, or within 8 % of it; a
        // second round of workgroups cost 10 to 40 %), while a slab keeps at least 4 runs per wave and the
        // partials fit the library's workspace
        const int64_t wgs = int64_t(pl.n_tiles) * pl.RB;
        S = int(std::min<int64_t>(16, std::max<int64_t>(1, 256 / wgs)));
        S = std::min(S, std::max(1, runs / 4));
        while (S > 1 && int64_t(S) * pl.RB * Mb * p.N * 4 > (int64_t(48) << 20)) --S;
    }
    S = std::min(S, runs);
    // arrival counters and partial sums of squares exist per (row block, column tile): a launch with more of
    // them than the workspace head holds runs unsplit (a forced split is refused)
    const bool head_fits = int64_t(pl.n_tiles) * pl.RB <= kMaxCounters &&
                           int64_t(pl.n_tiles) * pl.RB * S * kSumsqStride <= kMaxSumsqFloats;
    if (S > 1 && !head_fits) {
        if (p.k_split > 1) { pl.why = "too many tiles for a split over K"; return pl; }
        S = 1;
    }
    pl.k_slab = 64 * ((runs + S - 1) / S);
    S = (runs * 64 + pl.k_slab - 1) / pl.k_slab;         // no empty slab
    pl.S = S;
    if (int64_t(S + 16) * Mb * p.N * 4 >= (int64_t(1) << 31)) { pl.why = "split-K partials too large"; return pl; }
    if (int64_t(pl.n_tiles) * pl.RB * S >= (int64_t(1) << 31)) { pl.why = "too many workgroups"; return pl; }
    pl.lds = size_t(4) * 16 * pl.MB * kF32Tile * 4;
    pl.ok = true;
    return pl;
}

size_t f32_workspace_bytes(const Problem& p)
{
    F32Plan pl = f32_plan(p);
    if (!pl.ok || pl.S <= 1) return 0;
    return size_t(pl.RB) * pl.S * std::min(p.M, 64) * p.N * 4;    // [row block][slab][rows][N]
}

template <int MB>
static hipError_t f32_go(const F32Args& a, bool fused, bool gated, const F32Plan& pl, hipStream_t s)
{
    dim3 grid(unsigned(pl.n_tiles) * pl.S * pl.RB);
    static LdsOnce once;                                 // 64 KiB of dynamic LDS at MB = 4
    hipError_t e = raise_lds_once(once, {(const void*)f32_kernel<MB, true, false>, (const void*)f32_kernel<MB, false, false>,
                                         (const void*)f32_kernel<MB, true, true>}, 80 * 1024);
    if (e != hipSuccess) return e;
    if (gated)      f32_kernel<MB, true, true><<<grid, 256, pl.lds, s>>>(a);
    else if (fused) f32_kernel<MB, true, false><<<grid, 256, pl.lds, s>>>(a);
    else            f32_kernel<MB, false, false><<<grid, 256, pl.lds, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_f32(const Problem& p, hipStream_t s, const char** why)
{
    F32Plan pl = f32_plan(p);
    if (!pl.ok) { if (why) *why = pl.why; return hipErrorInvalidValue; }
    if (pl.S > 1 && (!p.ws_partial || !p.ws_sumsq || !p.ws_counter)) {
        if (why) *why = "split-K needs the workspace";
        return hipErrorInvalidValue;
    }
    if (p.plan) { p.plan[0] = kF32Tile; p.plan[1] = pl.S; p.plan[2] = pl.n_tiles * pl.S * pl.RB; }
    F32Args a;
    a.X = (const float*)p.X; a.g = (const float*)p.g; a.W = (const float*)p.W; a.Y = (float*)p.Y;
    a.M = p.M; a.K = p.K; a.N = p.N; a.eps = p.eps; a.inv_K = 1.0f / float(p.K);
    a.k_slab = pl.k_slab; a.S = pl.S; a.n_tiles = pl.n_tiles; a.RB = pl.RB;
    a.H = p.gated ? p.N / 2 : 0; a.G = p.gate_group;
    a.ws_partial = p.ws_partial; a.ws_sumsq = p.ws_sumsq; a.counter = p.ws_counter;
    const bool fused = p.fused != 0, gated = p.gated != 0;
    switch (pl.MB) {
    case 1:  return f32_go<1>(a, fused, gated, pl, s);
    case 2:  return f32_go<2>(a, fused, gated, pl, s);
    case 3:  return f32_go<3>(a, fused, gated, pl, s);
    default: return f32_go<4>(a, fused, gated, pl, s);
    }
}

}  // namespace rmsnl
