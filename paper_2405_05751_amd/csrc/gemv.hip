// Split-K GEMV variant of the fused RMSNorm + MatMul for decode shapes (M <= 16), without matrix
// cores.  The block is bound by streaming W once from HBM and, at these sizes, by the length of
// the chain of dependent memory round trips, so the design keeps many 16-byte loads in flight per
// lane from the first instruction on and touches every W byte exactly once:
//
//   * a workgroup (4 waves) owns N_TILE = 8*LPR columns and one K slab.  A wave is cut into
//     RPI = 64/LPR lane groups; each of the workgroup's 4*RPI groups owns a run of consecutive W
//     rows, a lane owns 8 columns, so a wave-wide dwordx4 load covers RPI rows of 16*LPR
//     contiguous bytes.  Loads are raw buffer loads: rows beyond the slab read as zero with no
//     branch, and D batches of 8 rows per lane are in flight at any time.  Up to 4 rows of X the
//     batches land in an LDS ring by direct loads (each lane reads back the 16 bytes it asked
//     for: the ring is a queue, not a shared tile), which frees the registers a deep queue would
//     take and lets two workgroups share a compute unit; above that they land in registers;
//   * X-hat = X (.) g (fp32).  For M <= 4 a lane group loads the 8 X and g values of its batch
//     straight into registers next to the W batch (no LDS, no barrier); for M = 8, 16 the slab's
//     X-hat is staged once in LDS as [m][k].  Either way the same pass adds up the slab's share of
//     A_i = sum_k X_ik^2: the two accumulations of the paper's fused kernel share one K loop;
//   * B partials are reduced across the lane groups of a wave by shuffles, across waves through
//     LDS, and across K slabs through an fp32 workspace: every slab writes its partial B and
//     partial A through to memory, the last workgroup to arrive at the tile's counter adds the S
//     partials in slab order (so the result does not depend on arrival order), scales by
//     1/sqrt(A/K + eps), rounds once and stores.
#include <algorithm>
#include <cstring>
#include "common.hpp"
#include "splitk.hpp"

namespace rmsnl {

struct GemvArgs {
    const u16* X; const u16* g; const uint4_t* W; u16* Y;
    int M, K, N;
    float eps, inv_K;
    int k_slab;      // rows of W per slab (multiple of 8 * number of lane groups)
    int S;           // number of slabs
    int n_tiles;
    int H;           // gated block: N = 2H, a tile is N_TILE/2 gate columns and the same outputs' up columns; else 0
    int G;           // gated block: layout of W, see gated_col()
    float* ws_partial; float* ws_sumsq; unsigned* counter;
    unsigned long long* trace; int trace_groups;
};

constexpr int kWAux = 2;             // cache policy of the W loads: nt (streamed once)
constexpr int kOut = 0x7ffffff0;     // a byte offset beyond any buffer resource: reads as zero
constexpr int kRsrcFlags = 0x00020000;

// batches of 8 rows in flight per lane.  Up to four rows of X (the automatic choice's range) W goes
// through LDS, two batches deep: a compute unit keeps about 32 KiB of loads in flight whatever the
// kernel asks for, so a deeper queue buys nothing, and 64 KiB of ring lets two workgroups share a unit.
constexpr bool gemv_w_lds(int MT) { return MT <= 4; }
constexpr int gemv_depth(int MT) { return 2; }
constexpr int kGemvBatchBytes = 8 * 1024;     // 8 wave-wide loads of 1 KiB

// s_waitcnt for the vector-memory counter alone (n <= 63)
#define RL_GEMV_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))
// waves per workgroup (8, in half as many workgroups, measured 6 % slower at the decode projection)
constexpr int gemv_waves(int MT) { return 4; }

// What the first loads need comes as leading scalar arguments: the dispatcher preloads up to 14
// dwords of those into registers before the wave starts, so the first loads of W do not wait for
// a fetch of the argument block (a round trip to memory at the head of every launch).  The rest
// rides in a struct behind them and is fetched while the loads are in flight.
struct GemvCold {
    u16* Y;
    float eps, inv_K;
    int H, G;
    float* ws_partial; float* ws_sumsq; unsigned* counter;
    unsigned long long* trace; int trace_groups;
};

template <typename T, int MT, int LPR, bool FUSED, bool GATED>
__global__ __launch_bounds__(64 * gemv_waves(MT)) void gemv_splitk_kernel(
    const uint4_t* W, const u16* X, const u16* g, int M, int K, int N, int k_slab, int S, int n_tiles, GemvCold cold)
{
    GemvArgs a;
    a.X = X; a.g = g; a.W = W; a.Y = cold.Y;
    a.M = M; a.K = K; a.N = N; a.eps = cold.eps; a.inv_K = cold.inv_K;
    a.k_slab = k_slab; a.S = S; a.n_tiles = n_tiles; a.H = cold.H; a.G = cold.G;
    a.ws_partial = cold.ws_partial; a.ws_sumsq = cold.ws_sumsq; a.counter = cold.counter;
    a.trace = cold.trace; a.trace_groups = cold.trace_groups;
    constexpr int NW = gemv_waves(MT);
    constexpr int N_TILE = LPR * 8;
    constexpr int RPI = 64 / LPR;            // lane groups per wave = W rows per wave-wide load
    constexpr int NG = NW * RPI;             // lane groups per workgroup
    constexpr int D = gemv_depth(MT);
    constexpr bool XLDS = MT > 4;            // X-hat through LDS instead of registers
    constexpr bool WLDS = gemv_w_lds(MT);    // W through LDS (direct loads) instead of registers
    constexpr int RING = WLDS ? NW * D * kGemvBatchBytes : 0;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];   // WLDS: the W ring first
    float* smem = reinterpret_cast<float*>(smem_raw + RING);                   // XLDS: xs [MT][k_slab]; later red [NW][MT][N_TILE]
    __shared__ float s_sumsq[NW][MT];
    __shared__ float s_rinv[MT];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = lane / LPR, col8 = lane % LPR;
    trace_stamp(a.trace, a.trace_groups, 0);         // start

    // workgroups are dealt round-robin to the 8 XCDs; renumber so that the slabs of one tile share
    // an XCD (a locality hint only: nothing below depends on where a workgroup runs)
    int b = blockIdx.x;
    const int total = a.n_tiles * a.S;
    if ((total & 7) == 0) b = (b & 7) * (total >> 3) + (b >> 3);
    const int tile = b / a.S, slab = b % a.S;
    // plain: the tile's W columns start at n0.  Gated: the tile is N_TILE/2 gate columns from n0 and
    // the up columns of the same outputs, H further on; lane chunk col8 is one or the other.
    const int n0 = GATED ? tile * (N_TILE / 2) : tile * N_TILE;
    const int ccol = GATED ? gated_col(n0 + (col8 % (LPR / 2)) * 8, col8 >= LPR / 2, a.H, a.G) : n0 + col8 * 8;
    const int k0 = slab * a.k_slab;
    const int klen = min(a.k_slab, a.K - k0);
    const int R = a.k_slab / NG;             // rows per lane group, a multiple of 8
    const int gi = wave * RPI + grp;
    const int r0 = gi * R;                   // first row of this group inside the slab
    const int nB = R >> 3;                   // batches of 8 rows per group (uniform; rows past klen are zero)

    // The slab of W as a buffer resource: rows at or beyond klen read as zero.  Columns at or
    // beyond N (ragged last tile) wrap into the next row; those lanes' sums are never stored.
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4_t*>(a.W + size_t(k0) * (a.N >> 3)), 0, klen * a.N * 2, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(a.X), 0, a.M * a.K * 2, kRsrcFlags);        // rows >= M read as zero
    const __amdgpu_buffer_rsrc_t grs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(FUSED ? a.g : a.X), 0, a.K * 2, kRsrcFlags);
    const int wrow = a.N * 2;
    const int voff0 = (r0 * a.N + ccol) * 2;

    // W through LDS: a direct load writes lane l's 16 bytes at byte 16 l of its KiB, so batch slot d
    // of this wave is [8 loads][64 lanes][16 bytes] and every lane reads back exactly what it
    // asked for.  Measured against loads into registers on the same access shape: the stream of a
    // 1 x 4096 x 4096 launch ends 2 us earlier (data that lands in LDS does not queue for the
    // register file's write port).  The compiler cannot see these loads, so the wait for a batch
    // is placed by hand: loads complete in order, and the count passed to s_waitcnt is the
    // number of loads issued after the batch's last one.
    const uint32_t ring = uint32_t(uintptr_t(smem_raw)) + uint32_t(wave) * (D * kGemvBatchBytes);
    const uint4_t wdesc = {uint32_t(uintptr_t(a.W + size_t(k0) * (a.N >> 3))), uint32_t(uintptr_t(a.W + size_t(k0) * (a.N >> 3)) >> 32),
                           uint32_t(klen * a.N * 2), uint32_t(kRsrcFlags)};
    auto load_w_lds = [&](uint32_t dst, int v) {
        const uint4_t desc = wdesc;
        uint32_t keep;                       // M0 carries the LDS address; whatever it held is put back
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                     "buffer_load_dwordx4 %2, %3, 0 offen nt lds\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep) : "s"(dst), "v"(v), "s"(desc) : "memory");
    };
    uint4_t w[WLDS ? 1 : D][8];
    uint4_t xq[D][XLDS ? 1 : MT], gq[D];
    auto issue = [&](int bi, int d) {        // batch bi of this group into register set (or ring slot) d
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (WLDS) load_w_lds(__builtin_amdgcn_readfirstlane(ring + d * kGemvBatchBytes + j * 1024), voff0 + (bi * 8 + j) * wrow);
            else w[d][j] = __builtin_amdgcn_raw_buffer_load_b128(wrs, voff0 + (bi * 8 + j) * wrow, 0, kWAux);
        }
        if (!XLDS) {
            const int koff = (r0 + bi * 8 < klen) ? (k0 + r0 + bi * 8) * 2 : kOut;
            if (FUSED) gq[d] = __builtin_amdgcn_raw_buffer_load_b128(grs, koff, 0, 0);
#pragma unroll
            for (int m = 0; m < MT; ++m)
                xq[d][m] = __builtin_amdgcn_raw_buffer_load_b128(
                    xrs, (r0 + bi * 8 < klen) ? koff + m * a.K * 2 : kOut, 0, 0);
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < nB) issue(d, d);             // the queue is full before anything else happens
    trace_stamp(a.trace, a.trace_groups, 1);         // first loads issued

    float ss[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) ss[m] = 0.f;

    float* xs = smem;
    if (XLDS) {
        // X-hat of the whole slab into LDS as [m][k]; thread t converts 8 consecutive k per step
        for (int c = tid; c < (a.k_slab >> 3); c += 64 * NW) {
            const int kk = c * 8;
            const int koff = kk < klen ? (k0 + kk) * 2 : kOut;
            uint4_t gv = uint4_t{0, 0, 0, 0};
            if (FUSED) gv = __builtin_amdgcn_raw_buffer_load_b128(grs, koff, 0, 0);
            uint4_t xv[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m)
                xv[m] = __builtin_amdgcn_raw_buffer_load_b128(xrs, kk < klen ? koff + m * a.K * 2 : kOut, 0, 0);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float h[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x0 = Elem<T>::lo(xv[m][e]), x1 = Elem<T>::hi(xv[m][e]);
                    h[2 * e] = x0; h[2 * e + 1] = x1;
                    if (FUSED) {
                        ss[m] = Arith<T>::fma(x0, x0, ss[m]);
                        ss[m] = Arith<T>::fma(x1, x1, ss[m]);
                        h[2 * e] = Arith<T>::mul(x0, Elem<T>::lo(gv[e]));
                        h[2 * e + 1] = Arith<T>::mul(x1, Elem<T>::hi(gv[e]));
                    }
                }
                float4_t* dst = (float4_t*)(xs + m * a.k_slab + kk);
                dst[0] = float4_t{h[0], h[1], h[2], h[3]};
                dst[1] = float4_t{h[4], h[5], h[6], h[7]};
            }
        }
        __syncthreads();
    }

    // ---- main loop: acc[m][8 columns] += xhat[m][k] * W[k][8 columns]
    float acc[MT][8];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[m][e] = 0.f;

    // loads issued per batch after its W loads: g (fused only) and the rows of X
    constexpr int kAfterW = (XLDS ? 0 : MT) + ((FUSED && !XLDS) ? 1 : 0);
    auto consume = [&](int bi, int d) {
        constexpr int WS = WLDS ? 0 : 1;     // (register mode indexes w by slot, LDS mode has one set)
        if (WLDS) {
            // batches bi .. min(bi + D - 1, nB - 1) are in flight; D = 2
            if (bi + 1 < nB) RL_GEMV_WAIT_VM(kAfterW + 8 + kAfterW);
            else RL_GEMV_WAIT_VM(kAfterW);
            asm volatile("" ::: "memory");
            const unsigned char* slot = smem_raw + wave * (D * kGemvBatchBytes) + d * kGemvBatchBytes + lane * 16;
#pragma unroll
            for (int j = 0; j < 8; ++j) w[0][j] = *reinterpret_cast<const uint4_t*>(slot + j * 1024);
            // the slot may be refilled once these reads have returned
            __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0)
            asm volatile("" ::: "memory");
        }
        float h[MT][8];
        if (XLDS) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const float4_t* src = (const float4_t*)(xs + m * a.k_slab + r0 + bi * 8);
                const float4_t lo = src[0], hi = src[1];
                h[m][0] = lo[0]; h[m][1] = lo[1]; h[m][2] = lo[2]; h[m][3] = lo[3];
                h[m][4] = hi[0]; h[m][5] = hi[1]; h[m][6] = hi[2]; h[m][7] = hi[3];
            }
        } else {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x0 = Elem<T>::lo(xq[d][m][e]), x1 = Elem<T>::hi(xq[d][m][e]);
                    h[m][2 * e] = x0; h[m][2 * e + 1] = x1;
                    if (FUSED) {
                        ss[m] = Arith<T>::fma(x0, x0, ss[m]);
                        ss[m] = Arith<T>::fma(x1, x1, ss[m]);
                        h[m][2 * e] = Arith<T>::mul(x0, Elem<T>::lo(gq[d][e]));
                        h[m][2 * e + 1] = Arith<T>::mul(x1, Elem<T>::hi(gq[d][e]));
                    }
                }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float wf[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                wf[2 * e] = Elem<T>::lo(w[WS * d][j][e]);
                wf[2 * e + 1] = Elem<T>::hi(w[WS * d][j][e]);
            }
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[m][e] = Arith<T>::fma(h[m][j], wf[e], acc[m][e]);
        }
    };

    for (int b0 = 0; b0 < nB; b0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int bi = b0 + d;
            if (bi < nB) {                   // uniform over the workgroup
                consume(bi, d);
                if (bi + D < nB) issue(bi + D, d);
            }
        }
    }

    trace_stamp(a.trace, a.trace_groups, 2);         // K loop done (all W consumed by wave 0)
    // ---- reduce over the lane groups of the wave, then over the four waves through LDS.
    // In register mode every lane of a group carries the same ss, so the group sum over lanes
    // col8 == 0 is what the shuffles over the group index produce.
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[m][e] = Arith<T>::add(acc[m][e], __shfl_xor(acc[m][e], off, 64));
        if (FUSED && !XLDS) {
#pragma unroll
            for (int m = 0; m < MT; ++m) ss[m] = Arith<T>::add(ss[m], __shfl_xor(ss[m], off, 64));
        }
    }
    if (FUSED) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            float v = ss[m];
            if (XLDS) {
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) v = Arith<T>::add(v, __shfl_xor(v, off, 64));
            }
            if (lane == 0) s_sumsq[wave][m] = v;
        }
    }

    if (XLDS) __syncthreads();               // everyone is done reading xs
    float* red = smem;                       // [NW][MT][N_TILE]
    if (grp == 0) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            float4_t* dst = (float4_t*)(red + (wave * MT + m) * N_TILE + col8 * 8);
            dst[0] = float4_t{acc[m][0], acc[m][1], acc[m][2], acc[m][3]};
            dst[1] = float4_t{acc[m][4], acc[m][5], acc[m][6], acc[m][7]};
        }
    }
    __syncthreads();

    trace_stamp(a.trace, a.trace_groups, 3);         // workgroup partial in LDS
    TailArgs ta{a.Y, a.M, a.N, N_TILE, GATED ? N_TILE / 2 : 0, a.H, a.G, a.eps, a.inv_K, a.S, a.ws_partial, a.ws_sumsq, a.counter,
                a.trace, a.trace_groups};
    splitk_tail<T, MT, N_TILE, FUSED, NW, GATED>(ta, red, &s_sumsq[0][0], s_rinv, &s_last, tile, slab, n0);
}

// ------------------------------------------------------------------------------------------- host
struct GemvPlan { int MT, LPR, S, k_slab, n_tiles; size_t lds; bool ok; const char* why; };

static GemvPlan gemv_plan(const Problem& p)
{
    GemvPlan pl{};
    pl.ok = false;
    if (p.dt == F32) { pl.why = "gemv variant handles 16-bit types only"; return pl; }
    if (p.gated && (p.N % 16 != 0 || !p.fused)) { pl.why = "gated block: gemv variant needs H % 8 == 0"; return pl; }
    if (p.M > 16) { pl.why = "gemv variant needs M <= 16"; return pl; }
    if (p.N % 8 != 0 || p.K % 8 != 0) { pl.why = "gemv variant needs N % 8 == 0 and K % 8 == 0"; return pl; }
    if (int64_t(p.M) * p.K * 2 >= (int64_t(1) << 31)) { pl.why = "gemv variant needs M*K < 2^30"; return pl; }
    pl.MT = p.M <= 1 ? 1 : p.M <= 2 ? 2 : p.M <= 4 ? 4 : p.M <= 8 ? 8 : 16;
    int n_tile = p.n_tile ? p.n_tile : 128;
    if (n_tile != 64 && n_tile != 128 && n_tile != 256 && n_tile != 512) {
        pl.why = "gemv n_tile must be 64, 128, 256 or 512";
        return pl;
    }
    if (pl.MT * n_tile > 4096) n_tile = 4096 / pl.MT;          // cross-wave reduction buffer <= 64 KiB
    pl.LPR = n_tile / 8;
    pl.n_tiles = p.gated ? (p.N / 2 + n_tile / 2 - 1) / (n_tile / 2) : (p.N + n_tile - 1) / n_tile;
    const int nw = gemv_waves(pl.MT);
    const int gran = 8 * nw * (64 / pl.LPR);                   // 8 rows per batch and lane group
    int S = p.k_split;
    if (S <= 0) {
        // about 512 waves' worth of workgroups per 64 compute units, but no slab shorter than one batch per
        // lane group (two batches measured 8-10 % slower at 2048 x 2048 and 1024 x 4096)
        S = (2048 / nw + pl.n_tiles - 1) / pl.n_tiles;
        const int s_max = std::min(32, (p.K + gran - 1) / gran);     // (64 slabs of 8192 x 1024: 9.3 against 8.4 us)
        if (S > s_max) S = s_max;
        if (S < 1) S = 1;
    }
    int k_slab = (p.K + S - 1) / S;
    k_slab = (k_slab + gran - 1) / gran * gran;
    while (int64_t(k_slab) * p.N * 2 >= (int64_t(1) << 31)) k_slab = (k_slab / 2 + gran - 1) / gran * gran;
    if (pl.MT > 4) {                                           // xs [MT][k_slab] fp32 <= 64 KiB
        const int k_max = (64 * 1024) / (4 * pl.MT) / gran * gran;
        if (k_slab > k_max) k_slab = k_max;
    }
    S = (p.K + k_slab - 1) / k_slab;
    pl.S = S;
    pl.k_slab = k_slab;
    if (pl.n_tiles > kMaxCounters) { pl.why = "too many column tiles"; return pl; }
    if (int64_t(pl.n_tiles) * S * kSumsqStride > kMaxSumsqFloats) { pl.why = "too many K slabs"; return pl; }
    if (int64_t(S + 16) * p.M * p.N * 4 >= (int64_t(1) << 31)) { pl.why = "split-K partials too large"; return pl; }
    const size_t xs = pl.MT > 4 ? size_t(k_slab) * pl.MT * 4 : 0;
    const size_t red = size_t(nw) * pl.MT * n_tile * 4;
    const size_t ring = gemv_w_lds(pl.MT) ? size_t(nw) * gemv_depth(pl.MT) * kGemvBatchBytes : 0;
    pl.lds = ring + (xs > red ? xs : red);
    pl.ok = true;
    return pl;
}

size_t gemv_workspace_bytes(const Problem& p)
{
    GemvPlan pl = gemv_plan(p);
    if (!pl.ok || pl.S <= 1) return 0;
    return size_t(pl.S) * p.M * p.N * 4;
}

template <typename T, int MT, int LPR>
static hipError_t gemv_go(const GemvArgs& a, bool fused, bool gated, const GemvPlan& pl, hipStream_t s)
{
    dim3 grid(pl.n_tiles * pl.S);
    static LdsOnce once;                     // allow more than 64 KiB of dynamic LDS
    hipError_t e = raise_lds_once(once, {(const void*)gemv_splitk_kernel<T, MT, LPR, true, false>,
                                         (const void*)gemv_splitk_kernel<T, MT, LPR, false, false>,
                                         (const void*)gemv_splitk_kernel<T, MT, LPR, true, true>}, 128 * 1024);
    if (e != hipSuccess) return e;
    const int nt = 64 * gemv_waves(MT);
    const GemvCold c{a.Y, a.eps, a.inv_K, a.H, a.G, a.ws_partial, a.ws_sumsq, a.counter, a.trace, a.trace_groups};
#define RL_GEMV_ARGS a.W, a.X, a.g, a.M, a.K, a.N, a.k_slab, a.S, a.n_tiles, c
    if (gated)      gemv_splitk_kernel<T, MT, LPR, true, true><<<grid, nt, pl.lds, s>>>(RL_GEMV_ARGS);
    else if (fused) gemv_splitk_kernel<T, MT, LPR, true, false><<<grid, nt, pl.lds, s>>>(RL_GEMV_ARGS);
    else            gemv_splitk_kernel<T, MT, LPR, false, false><<<grid, nt, pl.lds, s>>>(RL_GEMV_ARGS);
#undef RL_GEMV_ARGS
    return hipGetLastError();
}

template <typename T, int MT>
static hipError_t gemv_lpr(const GemvArgs& a, bool fused, bool gated, const GemvPlan& pl, hipStream_t s)
{
    if constexpr (MT * 512 <= 4096) { if (pl.LPR == 64) return gemv_go<T, MT, 64>(a, fused, gated, pl, s); }
    if constexpr (MT * 256 <= 4096) { if (pl.LPR == 32) return gemv_go<T, MT, 32>(a, fused, gated, pl, s); }
    if (pl.LPR == 16) return gemv_go<T, MT, 16>(a, fused, gated, pl, s);
    if (pl.LPR == 8) return gemv_go<T, MT, 8>(a, fused, gated, pl, s);
    return hipErrorInvalidValue;
}

template <typename T>
static hipError_t gemv_mt(const GemvArgs& a, bool fused, bool gated, const GemvPlan& pl, hipStream_t s)
{
    switch (pl.MT) {
    case 1:  return gemv_lpr<T, 1>(a, fused, gated, pl, s);
    case 2:  return gemv_lpr<T, 2>(a, fused, gated, pl, s);
    case 4:  return gemv_lpr<T, 4>(a, fused, gated, pl, s);
    case 8:  return gemv_lpr<T, 8>(a, fused, gated, pl, s);
    default: return gemv_lpr<T, 16>(a, fused, gated, pl, s);
    }
}

// ---- the same kernel on pairs over Z_227 x Z_113 (the paper's random tests over finite fields): the
// schedule that ships -- column tiles, K slabs, lane groups, the reduction through LDS, partials in the
// workspace, the last arriver adding them in slab order, the pairing of gate and up columns -- with the
// arithmetic of Table 3 in place of fp32.  128 columns per workgroup (the automatic choice); W through
// LDS up to four rows, as for the floating types.
template <int MT>
static hipError_t gemv_go_ff(const GemvArgs& a, bool gated, const GemvPlan& pl, hipStream_t s)
{
    dim3 grid(pl.n_tiles * pl.S);
    static LdsOnce once;
    hipError_t e = raise_lds_once(once, {(const void*)gemv_splitk_kernel<Ff, MT, 16, true, false>,
                                         (const void*)gemv_splitk_kernel<Ff, MT, 16, true, true>}, 128 * 1024);
    if (e != hipSuccess) return e;
    const int nt = 64 * gemv_waves(MT);
    const GemvCold c{a.Y, a.eps, a.inv_K, a.H, a.G, a.ws_partial, a.ws_sumsq, a.counter, a.trace, a.trace_groups};
    if (gated) gemv_splitk_kernel<Ff, MT, 16, true, true><<<grid, nt, pl.lds, s>>>(a.W, a.X, a.g, a.M, a.K, a.N, a.k_slab, a.S, a.n_tiles, c);
    else       gemv_splitk_kernel<Ff, MT, 16, true, false><<<grid, nt, pl.lds, s>>>(a.W, a.X, a.g, a.M, a.K, a.N, a.k_slab, a.S, a.n_tiles, c);
    return hipGetLastError();
}

static uint32_t host_pow_mod(uint32_t b, uint32_t e, uint32_t m)
{
    uint64_t r = 1, x = b % m;
    while (e) { if (e & 1) r = r * x % m; x = x * x % m; e >>= 1; }
    return uint32_t(r);
}

// p: the problem as for the 16-bit floating types (dt is ignored); omega: a 113th root of unity of Z_227
hipError_t launch_gemv_ff(const Problem& p, uint32_t omega, hipStream_t s, const char** why)
{
    Problem q = p;
    q.dt = BF16;
    q.n_tile = 128;
    GemvPlan pl = gemv_plan(q);
    if (!pl.ok) { if (why) *why = pl.why; return hipErrorInvalidValue; }
    if (pl.LPR != 16) { if (why) *why = "field instantiation of the gemv kernel runs 128 columns per workgroup"; return hipErrorInvalidValue; }
    if (pl.S > 1 && (!p.ws_partial || !p.ws_sumsq || !p.ws_counter)) {
        if (why) *why = "split-K needs the workspace";
        return hipErrorInvalidValue;
    }
    if (p.plan) { p.plan[0] = 128; p.plan[1] = pl.S; p.plan[2] = pl.n_tiles * pl.S; }
    GemvArgs a;
    a.X = (const u16*)p.X; a.g = (const u16*)p.g; a.W = (const uint4_t*)p.W; a.Y = (u16*)p.Y;
    a.M = p.M; a.K = p.K; a.N = p.N;
    // the two float fields carry field constants as bits: omega, and the pair (1/K mod p, 1/K mod q)
    const uint32_t inv_k = host_pow_mod(uint32_t(p.K % int(kFfP)), kFfP - 2, kFfP) | (host_pow_mod(uint32_t(p.K % int(kFfQ)), kFfQ - 2, kFfQ) << 16);
    memcpy(&a.eps, &omega, 4);
    memcpy(&a.inv_K, &inv_k, 4);
    a.k_slab = pl.k_slab; a.S = pl.S; a.n_tiles = pl.n_tiles;
    a.H = p.gated ? p.N / 2 : 0;
    a.G = p.gate_group;
    a.ws_partial = p.ws_partial; a.ws_sumsq = p.ws_sumsq; a.counter = p.ws_counter;
    a.trace = p.trace; a.trace_groups = p.trace_groups;
    const bool gated = p.gated != 0;
    switch (pl.MT) {
    case 1:  return gemv_go_ff<1>(a, gated, pl, s);
    case 2:  return gemv_go_ff<2>(a, gated, pl, s);
    case 4:  return gemv_go_ff<4>(a, gated, pl, s);
    case 8:  return gemv_go_ff<8>(a, gated, pl, s);
    default: return gemv_go_ff<16>(a, gated, pl, s);
    }
}

hipError_t launch_gemv(const Problem& p, hipStream_t s, const char** why)
{
    GemvPlan pl = gemv_plan(p);
    if (!pl.ok) { if (why) *why = pl.why; return hipErrorInvalidValue; }
    if (pl.S > 1 && (!p.ws_partial || !p.ws_sumsq || !p.ws_counter)) {
        if (why) *why = "split-K needs the workspace";
        return hipErrorInvalidValue;
    }
    if (p.plan) { p.plan[0] = pl.LPR * 8; p.plan[1] = pl.S; p.plan[2] = pl.n_tiles * pl.S; }
    GemvArgs a;
    a.X = (const u16*)p.X; a.g = (const u16*)p.g; a.W = (const uint4_t*)p.W; a.Y = (u16*)p.Y;
    a.M = p.M; a.K = p.K; a.N = p.N; a.eps = p.eps; a.inv_K = 1.0f / float(p.K);
    a.k_slab = pl.k_slab; a.S = pl.S; a.n_tiles = pl.n_tiles;
    a.H = p.gated ? p.N / 2 : 0;
    a.G = p.gate_group;
    a.ws_partial = p.ws_partial; a.ws_sumsq = p.ws_sumsq; a.counter = p.ws_counter;
    a.trace = p.trace; a.trace_groups = p.trace_groups;
    const bool fused = p.fused != 0, gated = p.gated != 0;
    return p.dt == F16 ? gemv_mt<Fp16>(a, fused, gated, pl, s) : gemv_mt<Bf16>(a, fused, gated, pl, s);
}

}  // namespace rmsnl
