// Matrix-core variant of the fused RMSNorm + MatMul for small M (64 rows per workgroup; more rows
// as further row blocks in the same launch): still bound by streaming
// W once from HBM, but each W element now meets up to 64 rows of X-hat, which plain FMAs could not
// keep up with.  One v_mfma_f32_16x16x32 per 16 rows x 16 columns x 32 k.
//
// W never passes through LDS.  The matrix instruction wants, per lane, 8 consecutive k of ONE
// column, while W [K][N] offers 8 consecutive columns of one k per 16-byte load.  The k index
// inside an instruction is only a label, so the lanes are laid out as i = lane % 16 (column
// chunk) and q = lane / 16 (k group): lane (i, q) loads the 8x8 block
// W[kb + 8q .. +7][n0 + 8i .. +7] with eight coalesced dwordx4 loads (a wave-wide load covers 4
// rows of 256 contiguous bytes).  For each of the 8 columns c of the block, the B operand of MFMA
// #c is the column of that register block -- four v_perm_b32 pick it out -- and MFMA #c as a whole
// computes the 16 strided columns {n0 + 8i + c}.  The A operand of lane (m, q) is
// X-hat[m][kb + 8q .. +7]: X times g, rounded once to the 16-bit type; the squares of the raw X
// feed A_i in the same pass (the paper's two accumulators in one K loop).  X itself is loaded as
// whole 128-byte lines and turned into that layout through the wave's own piece of LDS (see the
// kernel).
//
// A workgroup owns 128 columns and one K slab; its NW waves take alternate 64-row runs of the
// slab, two 32-row steps each, so nothing in the K loop needs a barrier.  The waves' fp32 tiles
// meet in LDS, and the common split-K epilogue finishes (see splitk.hpp).
#include <algorithm>
#include "common.hpp"
#include "splitk.hpp"

namespace rmsnl {

struct SkinnyArgs {
    const u16* X; const u16* g; const uint4_t* W; u16* Y;
    int M, K, N;
    float eps, inv_K;
    int k_slab;      // most rows of W in a slab (a multiple of 64): slab s takes the 64-row runs
                     // [s R / S, (s + 1) R / S) of the R = ceil(K / 64) runs, so slabs differ by at most one run
    int S;
    int n_tiles;
    int n_tile;      // live columns per workgroup: a multiple of 8, at most kSkinnyTile
    int H;           // gated block: N = 2H, a tile is n_tile/2 gate columns and the same up columns; else 0
    int G;           // gated block: layout of W, see gated_col()
    int RB;          // row blocks of 64 rows in this launch (M > 64): workgroup (row block, tile, slab)
    float* ws_partial; float* ws_sumsq; unsigned* counter;
    unsigned long long* trace; int trace_groups;
};

#ifndef RL_SKINNY_TWO_PART
#define RL_SKINNY_TWO_PART 1
#endif
#ifndef RL_SKINNY_X_LDS
#define RL_SKINNY_X_LDS 1
#endif
#ifndef RL_SKINNY_TWO_MAX_MB
#define RL_SKINNY_TWO_MAX_MB 2
#endif
constexpr int kSkinnyTile = 128;     // most columns per workgroup (16 lanes x 8)
constexpr int kSkAux = 2;            // W loads: nt
constexpr int kSkOut = 0x7ffffff0;
constexpr int kSkFlags = 0x00020000;

template <typename T> struct Mfma16;
template <> struct Mfma16<Bf16> {
    static __device__ __forceinline__ float4_t run(uint4_t a, uint4_t b, float4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma16<Fp16> {
    static __device__ __forceinline__ float4_t run(uint4_t a, uint4_t b, float4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
};

// steps (8 W loads per lane each) kept in flight per wave; X is fetched one run ahead (two runs
// ahead measured 1 % slower at M <= 16)
constexpr int skinny_depth(int MB) { return MB == 1 ? 4 : 3; }
constexpr int skinny_waves(int MB) { return 4; }    // 8 (two waves per SIMD at MB = 1) measured equal or up to 20 % slower

// Leading scalar arguments are preloaded into registers by the dispatcher (see the GEMV kernel);
// what the first loads do not need follows in a struct.
struct SkinnyCold {
    u16* Y;
    float eps, inv_K;
    int H, G;
    float* ws_partial; float* ws_sumsq; unsigned* counter;
    unsigned long long* trace; int trace_groups;
};

// MULTI: the launch holds several row blocks of 64 rows (M > 64; MB = 4 then).
template <typename T, int MB, bool FUSED, bool GATED, bool MULTI = false>
__global__ __launch_bounds__(64 * skinny_waves(MB)) void skinny_kernel(
    const uint4_t* W, const u16* X, const u16* g, int M, int K, int N, int k_slab, int S, int n_tiles, int n_tile,
    int RB, SkinnyCold cold)
{
    SkinnyArgs a;
    a.X = X; a.g = g; a.W = W; a.Y = cold.Y;
    a.M = M; a.K = K; a.N = N; a.eps = cold.eps; a.inv_K = cold.inv_K;
    a.k_slab = k_slab; a.S = S; a.n_tiles = n_tiles; a.n_tile = n_tile; a.H = cold.H; a.G = cold.G; a.RB = RB;
    a.ws_partial = cold.ws_partial; a.ws_sumsq = cold.ws_sumsq; a.counter = cold.counter;
    a.trace = cold.trace; a.trace_groups = cold.trace_groups;
    constexpr int NW = skinny_waves(MB);
    constexpr int MT = 16 * MB;
    constexpr int N_TILE = kSkinnyTile;
    constexpr int D = skinny_depth(MB);
    extern __shared__ __align__(16) float smem[];   // red [NW][MT][N_TILE]
    __shared__ float s_sumsq[NW][MT];
    __shared__ float s_rinv[MT];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, q = lane >> 4;
    trace_stamp(a.trace, a.trace_groups, 0);

    // Workgroups are dealt round-robin to the 8 XCDs; renumber so that the slabs of a tile, and the
    // row blocks that stream the same part of W, share an XCD and start together: W then comes
    // from HBM once and from that XCD's L2 for the other row blocks (a hint, nothing depends on it).
    int b = blockIdx.x, rb = 0;
    const int total = a.n_tiles * a.S;
    if (!MULTI) {
        if ((total & 7) == 0) b = (b & 7) * (total >> 3) + (b >> 3);
    } else if ((total & 7) == 0) {
        const int j = b >> 3;
        rb = j % a.RB;
        b = (b & 7) * (total >> 3) + j / a.RB;
    } else {
        rb = b % a.RB;
        b /= a.RB;
    }
    const int tile = b / a.S, slab = b % a.S;
    const int Mh = MULTI ? min(a.M - 64 * rb, 64) : a.M;   // rows of this row block
    const u16* Xb = MULTI ? a.X + size_t(rb) * 64 * a.K : a.X;
    // plain: the tile's W columns start at n0.  Gated: the tile is half = n_tile/2 gate columns from
    // hn0 and the up columns of the same outputs, H further on; lane chunk i is one or the other.
    const int half = a.n_tile >> 1;
    const int n0 = GATED ? tile * half : tile * a.n_tile;
    const int ccol = GATED ? gated_col(n0 + (i * 8 < half ? i * 8 : i * 8 - half), i * 8 >= half, a.H, a.G) : n0 + i * 8;
    const bool live = i * 8 < a.n_tile;      // narrower tiles leave the last column chunks idle
    const int runs = (a.K + 63) >> 6;        // 64-row runs of W in all
    const int run0 = int(int64_t(slab) * runs / a.S), run1 = int(int64_t(slab + 1) * runs / a.S);
    const int k0 = run0 * 64;
    const int klen = min(run1 * 64, a.K) - k0;
    // runs of this wave: wave w takes runs w, w + NW, ... of the slab (the waves of a workgroup may
    // differ by one; nothing in the K loop is shared between them)
    const int nPairs = (run1 - run0 - wave + NW - 1) / NW;

    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4_t*>(a.W + size_t(k0) * (a.N >> 3)), 0, klen * a.N * 2, kSkFlags);
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(Xb), 0, Mh * a.K * 2, kSkFlags);
    const __amdgpu_buffer_rsrc_t grs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(FUSED ? a.g : a.X), 0, a.K * 2, kSkFlags);
    const int wrow = a.N * 2;
    // Run t of this wave is the 64 slab rows from (NW t + wave)*64, taken as two 32-row steps:
    // lane (i, q) owns rows 16q + 8h .. +7 of the run in step h.
    // idle lanes start at 2^31: their offsets stay beyond every resource (sizes are below 2^31) and read zero
    const unsigned woff0 = live ? unsigned(((wave * 64 + q * 16) * a.N + ccol) * 2) : 0x80000000u;
    const int wpair = 64 * NW * a.N * 2;     // bytes of W between two runs

    // X is fetched as whole 128-byte lines, each exactly once: load j of a run has lane (r8, c8)
    // take 16 bytes c8 of row 8j + r8 (64 k = 128 bytes per row), the wave passes the run through
    // its own corner of LDS, and lane (i, q) reads back chunk 2q + h of row 16mb + i, which is the
    // A operand layout.  (Loading in operand layout touches every line in both steps, half of it
    // each time, and by the second touch the line has left the vector cache again.)  The 16-byte
    // chunk index is XORed with (row / 2) % 8 so that writes and reads are free of bank conflicts.
    // g rides along as one more row.
    const int r8 = lane >> 3, c8 = lane & 7;
    char* stage = reinterpret_cast<char*>(smem) + wave * (MT * N_TILE * 4);   // inside this wave's part of red
    const int st_w0 = r8 * 128 + ((c8 ^ (r8 >> 1)) << 4);            // even j (+ 1024 j)
    const int st_w1 = r8 * 128 + ((c8 ^ (r8 >> 1) ^ 4) << 4);        // odd j
    const int st_r0 = i * 128 + (((2 * q) ^ (i >> 1)) << 4);         // step 0 (+ 2048 mb); step 1 is ^ 16
    const int st_g = MT * 128;
    // XLDS: the lines of X (and g) go straight from memory into that corner of LDS (direct loads; data
    // that lands in LDS does not queue for the register file, and a line from L2 arrives at 99
    // instead of 68 GB/s per compute unit).  A direct load writes lane l's 16 bytes at byte 16 l of its
    // KiB, so lane l = (r8, c8) of load j fetches the chunk that belongs in slot c8 of row 8j + r8:
    // chunk c8 ^ ((row / 2) % 8).  Two stage buffers, one per parity of the run; the wait for a run
    // is placed by hand (the 16 loads of W of the run before it were issued after it).
    constexpr bool XLDS = RL_SKINNY_X_LDS != 0;
    constexpr int STG = MT * 128 + 1024;     // a run of X, and the KiB that g's load writes (128 bytes of it used)
    static_assert(2 * STG <= MT * N_TILE * 4, "two stage buffers fit the wave's part of the reduction buffer");
    const uint32_t stage_lds = __builtin_amdgcn_readfirstlane(uint32_t(uintptr_t(stage)));
    const uint4_t xdesc = {uint32_t(uintptr_t(Xb)), uint32_t(uintptr_t(Xb) >> 32), uint32_t(Mh * a.K * 2), uint32_t(kSkFlags)};
    const uint4_t gdesc = {uint32_t(uintptr_t(FUSED ? a.g : a.X)), uint32_t(uintptr_t(FUSED ? a.g : a.X) >> 32),
                           uint32_t(a.K * 2), uint32_t(kSkFlags)};
    auto load_lds = [&](const uint4_t& rsrc, uint32_t dst, int v) {
        const uint4_t desc = rsrc;
        uint32_t keep;                       // M0 carries the LDS address; whatever it held is put back
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                     "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep) : "s"(dst), "v"(v), "s"(desc) : "memory");
    };

    uint4_t w[D][8];                         // D steps of W in flight
    uint4_t xr[XLDS ? 1 : 2 * MB], gr;       // register mode: the next run of X (and g), as lines
    // Load j of a run takes row 8j + r8 of X.  Where there is no such row (8 j >= rlim) it takes the
    // last row again: the repeated line costs nothing, nothing computed from those rows is ever
    // stored, and no instruction has part of its lanes out of range (measured the same as reading
    // zeros there).
    const int rlim = Mh - r8;
    const int xlane = r8 * a.K * 2;          // used only where r8 < M
    const int xlast = (Mh - 1) * a.K * 2;
    auto issue_x = [&](int t) {
        if constexpr (XLDS) {
            const uint32_t sb = stage_lds + uint32_t(t & 1) * STG;
            const int krun = (NW * t + wave) * 64;                  // slab-relative k of the run
            if (FUSED) {
                const int kr = krun + c8 * 8;
                load_lds(gdesc, sb + st_g, (r8 == 0 && kr < klen) ? (k0 + kr) * 2 : kSkOut);
            }
#pragma unroll
            for (int j = 0; j < 2 * MB; ++j) {
                const int kr = krun + ((c8 ^ (r8 >> 1) ^ (4 * (j & 1))) << 3);   // the chunk that belongs in this lane's slot
                load_lds(xdesc, sb + 1024 * j,
                         kr < klen ? (k0 + kr) * 2 + (8 * j < rlim ? xlane + 8 * j * a.K * 2 : xlast) : kSkOut);
            }
        } else {
        const int kr = (NW * t + wave) * 64 + c8 * 8;               // slab-relative k of this lane's chunk
        const int koff = (k0 + kr) * 2;
        const bool kin = kr < klen;
        if (FUSED) gr = __builtin_amdgcn_raw_buffer_load_b128(grs, (r8 == 0 && kin) ? koff : kSkOut, 0, 0);
#pragma unroll
        for (int j = 0; j < 2 * MB; ++j)
            xr[j] = __builtin_amdgcn_raw_buffer_load_b128(
                xrs, kin ? koff + (8 * j < rlim ? xlane + 8 * j * a.K * 2 : xlast) : kSkOut, 0, 0);
        }
    };
    auto issue_w = [&](int s, int d) {
        const int t = s >> 1, h = s & 1;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            w[d][j] = __builtin_amdgcn_raw_buffer_load_b128(     // (the uniform part is kept out of the lane's registers)
                wrs, int(woff0 + unsigned(__builtin_amdgcn_readfirstlane(int(unsigned(t) * unsigned(wpair) + unsigned((8 * h + j) * wrow))))), 0, kSkAux);
    };
    // Every load below is issued whether or not its step exists (a step past the slab reads zeros
    // through the range check): the compiler then knows exactly how many loads are younger than
    // the one it waits for, and the waits leave the rest of the ring in flight.
    __builtin_amdgcn_sched_barrier(0);       // (the order of issue is the order the waits count in)
    issue_w(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    issue_x(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = 1; d < D; ++d) {
        issue_w(d, d);
        __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("" ::: "memory");
    trace_stamp(a.trace, a.trace_groups, 1);

    float4_t acc[MB][8];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[mb][c] = float4_t{0.f, 0.f, 0.f, 0.f};
    float ss[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) ss[mb] = 0.f;

    // X-hat = X (.) g is exact in fp32 (two 16-bit significands), but the matrix cores take 16-bit
    // operands.  Up to 32 rows this kernel has matrix-core time to spare, so X-hat goes in as two
    // operands, its rounded value and the rounding's remainder (hi + lo, each exact in the storage
    // type, together good to 16 more bits), at two matrix instructions per step: the result then
    // carries no rounding of X-hat at all, only the final one of Y.  From 33 rows on the second
    // instruction is not free any more (64 x 4096 x 28672: +5 %; several row blocks: +20 %), and
    // X-hat is rounded once, as the tile kernels round it.
    constexpr bool TWO = FUSED && RL_SKINNY_TWO_PART && MB <= RL_SKINNY_TWO_MAX_MB;
    auto consume = [&](int d, int h, const char* stage) {     // stage: the buffer that holds this run of X
        // A operands: X-hat = X (.) g in the storage type (see above); squares of the raw X
        uint4_t aop[MB], alo[TWO ? MB : 1], gq;
        if (FUSED) gq = *reinterpret_cast<const uint4_t*>(stage + st_g + ((2 * q + h) << 4));
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const uint4_t xq = *reinterpret_cast<const uint4_t*>(stage + ((st_r0 ^ (h << 4)) + 2048 * mb));
            if (FUSED) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x0 = Elem<T>::lo(xq[e]), x1 = Elem<T>::hi(xq[e]);
                    ss[mb] = __fmaf_rn(x0, x0, ss[mb]);
                    ss[mb] = __fmaf_rn(x1, x1, ss[mb]);
                    const float p0 = x0 * Elem<T>::lo(gq[e]), p1 = x1 * Elem<T>::hi(gq[e]);
                    aop[mb][e] = Elem<T>::pack(p0, p1);
                    if (TWO) alo[mb][e] = Elem<T>::pack(p0 - Elem<T>::lo(aop[mb][e]), p1 - Elem<T>::hi(aop[mb][e]));
                }
            } else {
                aop[mb] = xq;
            }
        }
        // B operands: column c of the lane's 8x8 block, rows paired (2t, 2t+1)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            uint4_t bop;
#pragma unroll
            for (int t = 0; t < 4; ++t)
                bop[t] = __builtin_amdgcn_perm(w[d][2 * t + 1][c >> 1], w[d][2 * t][c >> 1],
                                               (c & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[mb][c] = Mfma16<T>::run(aop[mb], bop, acc[mb][c]);
            if (TWO) {                       // (after all the first parts: no instruction waits for the one before it)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[mb][c] = Mfma16<T>::run(alo[mb], bop, acc[mb][c]);
            }
        }
    };

    constexpr int PU = (D % 2 == 0) ? D / 2 : D;    // runs per trip: ring slots repeat every 2 PU steps
    for (int t0 = 0; t0 < nPairs; t0 += PU) {
#pragma unroll
        for (int p = 0; p < PU; ++p) {
            const int t = t0 + p;
            const bool there = t < nPairs;   // uniform over the workgroup; only the arithmetic is skipped
            const char* stg = stage + (XLDS ? (t & 1) * STG : 0);
            if (XLDS) {
                // this run's X was asked for a run ago; the 16 loads of W issued since are younger
                __builtin_amdgcn_s_waitcnt((16 & 15) | ((16 >> 4) << 14) | (7 << 4) | (15 << 8));
                asm volatile("" ::: "memory");
            } else if (there) {
                // the wave's LDS operations execute in order: these writes land after the previous
                // run's reads and before the reads below
#pragma unroll
                for (int j = 0; j < 2 * MB; ++j)
                    *reinterpret_cast<uint4_t*>(stage + ((j & 1) ? st_w1 : st_w0) + 1024 * j) = xr[XLDS ? 0 : j];
                if (FUSED && r8 == 0) *reinterpret_cast<uint4_t*>(stage + st_g + (c8 << 4)) = gr;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            __builtin_amdgcn_sched_barrier(0);
            issue_x(t + 1);
            asm volatile("" ::: "memory");   // pins the loads here: nothing may carry them down to their first use
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (there) consume((2 * p + h) % D, h, stg);
                __builtin_amdgcn_sched_barrier(0);
                issue_w(2 * t + h + D, (2 * p + h) % D);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    trace_stamp(a.trace, a.trace_groups, 2);
    if (XLDS) {
        // the loads issued for the run past the end still write (zeros) into this wave's stage buffers,
        // which the reduction buffer below lies over: nothing may be in flight any more
        __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
        asm volatile("" ::: "memory");
    }

    // ---- A_i: add the four k groups of the wave (lanes i, i+16, i+32, i+48 hold row i's shares)
    if (FUSED) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float v = ss[mb];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (q == 0) s_sumsq[wave][mb * 16 + i] = v;
        }
    }
    // ---- B: lane (i, q) holds rows 16mb + 4q + r, columns n0 + 8i + c of its wave's partial tile
    float* red = smem;                       // [NW][MT][N_TILE]
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float4_t* dst = (float4_t*)(red + ((wave * MT) + mb * 16 + q * 4 + r) * N_TILE + i * 8);
            dst[0] = float4_t{acc[mb][0][r], acc[mb][1][r], acc[mb][2][r], acc[mb][3][r]};
            dst[1] = float4_t{acc[mb][4][r], acc[mb][5][r], acc[mb][6][r], acc[mb][7][r]};
        }
    __syncthreads();
    trace_stamp(a.trace, a.trace_groups, 3);

    // every row block is a problem of its own to the epilogue: its rows of Y, its share of the workspace
    TailArgs ta{a.Y, Mh, a.N, a.n_tile, GATED ? half : 0, a.H, a.G, a.eps, a.inv_K, a.S,
                a.ws_partial, a.ws_sumsq, a.counter, a.trace, a.trace_groups};
    if (MULTI) {
        ta.Y += size_t(rb) * 64 * (GATED ? a.H : a.N);
        ta.ws_partial += size_t(rb) * a.S * 64 * a.N;
        ta.ws_sumsq += size_t(rb) * total * kSumsqStride;
        ta.counter += size_t(rb) * a.n_tiles * kCounterStride;
    }
    splitk_tail<T, MT, N_TILE, FUSED, NW, GATED>(ta, red, &s_sumsq[0][0], s_rinv, &s_last, tile, slab, n0);
}

// ------------------------------------------------------------------------------------------- host
constexpr int kSkinnyMaxM = 1024;
struct SkinnyPlan { int MB, RB, S, k_slab, n_tiles, n_tile; size_t lds; bool ok; const char* why; };

static SkinnyPlan skinny_plan(const Problem& p)
{
    SkinnyPlan pl{};
    pl.ok = false;
    if (p.dt == F32) { pl.why = "skinny variant handles 16-bit types only"; return pl; }
    if (p.M > kSkinnyMaxM) { pl.why = "skinny variant needs M <= 1024"; return pl; }
    if (p.N % 8 != 0 || p.K % 8 != 0) { pl.why = "skinny variant needs N % 8 == 0 and K % 8 == 0"; return pl; }
    if (int64_t(p.M) * p.K * 2 >= (int64_t(1) << 31)) { pl.why = "skinny variant needs M*K < 2^30"; return pl; }
    if (p.n_tile != 0 && (p.n_tile % 8 != 0 || p.n_tile < 8 || p.n_tile > kSkinnyTile)) {
        pl.why = "skinny n_tile must be a multiple of 8 in [8, 128]";
        return pl;
    }
    if (p.gated && (p.N % 16 != 0 || p.n_tile % 16 != 0 || !p.fused)) {
        pl.why = "gated block: skinny variant needs H % 8 == 0 and n_tile % 16 == 0";
        return pl;
    }
    pl.RB = (p.M + 63) / 64;                 // row blocks of 64 rows, all in one launch
    pl.MB = pl.RB > 1 ? 4 : (p.M + 15) / 16;
    const int Mb = std::min(p.M, 64);        // rows per workgroup
    const int runs = (p.K + 63) / 64;        // 64-row runs of W; a slab is a whole number of them
    const int nw = skinny_waves(pl.MB);
    int n_tile = p.n_tile, S = p.k_split;
    if (n_tile == 0 || S <= 0) {
        // Pick the slab count with a small cost model, fitted to a sweep of every slab count over 65
        // shapes (M 2 to 64; W from 1024 x 4096 to 28672 x 8192): the pick is within 1.5 % of the best
        // slab count on average, 9 % at worst.  W streams at the HBM rate unless the compute units
        // holding workgroups cannot pull their share of W plus their slab of X that fast (a unit
        // takes in about 45 GB/s; with more workgroups than units some units hold several, one
        // after the other as far as the stream is concerned: a launch of just over 256 workgroups
        // measured up to 30 % slower than one of just under); every extra slab costs a write and a
        // read of an fp32 partial tile set on top of the epilogue's fixed latency.
        double best = 1e30;
        int best_nt = kSkinnyTile, best_s = 1;
        // (narrower tiles measured slower: their row segments stop being whole 128-byte lines, so
        // the width stays at 128 unless the caller asks otherwise)
        for (int nt = (p.n_tile ? p.n_tile : kSkinnyTile); nt >= (p.n_tile ? p.n_tile : kSkinnyTile); nt -= 8) {
            const int tiles = (p.N + nt - 1) / nt;
            for (int s = (p.k_split > 0 ? p.k_split : 1); s <= (p.k_split > 0 ? p.k_split : 16); ++s) {
                if (s > 1 && s * nw > runs) break;                                           // at least one run per wave
                if (int64_t(tiles) * pl.RB > kMaxCounters || int64_t(tiles) * pl.RB * s * kSumsqStride > kMaxSumsqFloats) continue;
                if (s > 1 && int64_t(s) * pl.RB * 64 * p.N * 4 > (int64_t(48) << 20)) continue;   // fits the library workspace
                const double wgs = double(tiles) * s * pl.RB;
                const double slab_rows = 64.0 * ((runs + s - 1) / s);                        // the longest slab
                const double wg_bytes = slab_rows * (nt * 2.0 + Mb * 2.0);                   // its W and its X
                double t;
                if (pl.RB == 1) {
                    const double hbm_us = double(p.K) * p.N * 2.0 / 6.5e6;                   // W comes from HBM once
                    const double unit_us = double((int64_t(wgs) + 255) / 256) * wg_bytes / 45.0e3;
                    const double stream_us = std::max(hbm_us, unit_us) + 0.15 * std::min(hbm_us, unit_us);
                    const double tail_us = s > 1 ? 2.0 + 0.05 * s + 0.35 * s * double(p.M) * p.N * 8.0 / 1.0e6 : 0.0;
                    t = stream_us + tail_us;
                } else {
                    // several row blocks (M > 64): the first model, which the choice between this
                    // kernel and the tile kernels was measured with
                    const double per_unit = double((int64_t(wgs) + 255) / 256) * wg_bytes / 36.0e3;
                    const double stream_us = std::max(double(p.K) * p.N * 2.0 / 5.7e6, per_unit);
                    const double tail_us = s > 1 ? 3.0 + 2.0 * s * double(p.M) * p.N * 4.0 / 2.0e6 : 0.5;
                    t = stream_us + tail_us;
                }
                if (t < best) { best = t; best_nt = nt; best_s = s; }
            }
        }
        n_tile = best_nt;
        S = best_s;
        // a launch that would fill at most half the chip runs 64-column tiles instead, twice the
        // workgroups: 4 to 10 % faster on 13 small shapes (8 x 512 x 512 to 16 x 4096 x 1024), while
        // a W that fills the chip streams faster in 256-byte row segments
        if (p.n_tile == 0 && pl.RB == 1 && int64_t((p.N + kSkinnyTile - 1) / kSkinnyTile) * S <= 128 && p.N >= 128) n_tile = 64;
    }
    pl.n_tile = n_tile;
    pl.n_tiles = p.gated ? (p.N / 2 + n_tile / 2 - 1) / (n_tile / 2) : (p.N + n_tile - 1) / n_tile;
    if (S > runs) S = runs;
    // the ring runs a few steps past the slab, and those offsets must stay below 2^31 as well
    const int64_t past = 2048;               // rows: more than PU + D / 2 + 1 runs of every wave
    while ((int64_t(64) * ((runs + S - 1) / S) + past) * p.N * 2 >= (int64_t(1) << 31) && S < runs) ++S;
    const int k_slab = 64 * ((runs + S - 1) / S);
    if ((int64_t(k_slab) + past) * p.N * 2 >= (int64_t(1) << 31)) { pl.why = "skinny variant needs N < 2^20"; return pl; }
    pl.S = S;
    pl.k_slab = k_slab;
    if (int64_t(pl.n_tiles) * pl.RB > kMaxCounters) { pl.why = "too many column tiles"; return pl; }
    if (int64_t(pl.n_tiles) * pl.RB * S * kSumsqStride > kMaxSumsqFloats) { pl.why = "too many K slabs"; return pl; }
    if (int64_t(S + 16) * Mb * p.N * 4 >= (int64_t(1) << 31)) { pl.why = "split-K partials too large"; return pl; }
    pl.lds = size_t(skinny_waves(pl.MB)) * 16 * pl.MB * kSkinnyTile * 4;
    pl.ok = true;
    return pl;
}

size_t skinny_workspace_bytes(const Problem& p)
{
    SkinnyPlan pl = skinny_plan(p);
    if (!pl.ok || pl.S <= 1) return 0;
    return size_t(pl.RB) * pl.S * std::min(p.M, 64) * p.N * 4;    // [row block][slab][rows][N]
}

template <typename T, int MB, bool MULTI>
static hipError_t skinny_go(const SkinnyArgs& a, bool fused, bool gated, const SkinnyPlan& pl, hipStream_t s)
{
    dim3 grid(pl.n_tiles * pl.S * pl.RB);
    static LdsOnce once;                     // 128 KiB of dynamic LDS at MB = 4
    hipError_t e = raise_lds_once(once, {(const void*)skinny_kernel<T, MB, true, false, MULTI>,
                                         (const void*)skinny_kernel<T, MB, false, false, MULTI>,
                                         (const void*)skinny_kernel<T, MB, true, true, MULTI>}, 144 * 1024);
    if (e != hipSuccess) return e;
    const int nt = 64 * skinny_waves(MB);
    const SkinnyCold c{a.Y, a.eps, a.inv_K, a.H, a.G, a.ws_partial, a.ws_sumsq, a.counter, a.trace, a.trace_groups};
#define RL_SKINNY_ARGS a.W, a.X, a.g, a.M, a.K, a.N, a.k_slab, a.S, a.n_tiles, a.n_tile, a.RB, c
    if (gated)      skinny_kernel<T, MB, true, true, MULTI><<<grid, nt, pl.lds, s>>>(RL_SKINNY_ARGS);
    else if (fused) skinny_kernel<T, MB, true, false, MULTI><<<grid, nt, pl.lds, s>>>(RL_SKINNY_ARGS);
    else            skinny_kernel<T, MB, false, false, MULTI><<<grid, nt, pl.lds, s>>>(RL_SKINNY_ARGS);
#undef RL_SKINNY_ARGS
    return hipGetLastError();
}

template <typename T>
static hipError_t skinny_mb(const SkinnyArgs& a, bool fused, bool gated, const SkinnyPlan& pl, hipStream_t s)
{
    if (pl.RB > 1) return skinny_go<T, 4, true>(a, fused, gated, pl, s);
    switch (pl.MB) {
    case 1:  return skinny_go<T, 1, false>(a, fused, gated, pl, s);
    case 2:  return skinny_go<T, 2, false>(a, fused, gated, pl, s);
    case 3:  return skinny_go<T, 3, false>(a, fused, gated, pl, s);
    default: return skinny_go<T, 4, false>(a, fused, gated, pl, s);
    }
}

// M <= 64: one row block.  M up to 1024: a row block per 64 rows, all in one launch, the row
// blocks that read the same part of W side by side on one XCD (see the kernel).
hipError_t launch_skinny(const Problem& p, hipStream_t s, const char** why)
{
    SkinnyPlan pl = skinny_plan(p);
    if (!pl.ok) { if (why) *why = pl.why; return hipErrorInvalidValue; }
    if (pl.S > 1 && (!p.ws_partial || !p.ws_sumsq || !p.ws_counter)) {
        if (why) *why = "split-K needs the workspace";
        return hipErrorInvalidValue;
    }
    if (p.plan) { p.plan[0] = pl.n_tile; p.plan[1] = pl.S; p.plan[2] = pl.n_tiles * pl.S * pl.RB; }
    SkinnyArgs a;
    a.X = (const u16*)p.X; a.g = (const u16*)p.g; a.W = (const uint4_t*)p.W; a.Y = (u16*)p.Y;
    a.M = p.M; a.K = p.K; a.N = p.N; a.eps = p.eps; a.inv_K = 1.0f / float(p.K);
    a.k_slab = pl.k_slab; a.S = pl.S; a.n_tiles = pl.n_tiles; a.n_tile = pl.n_tile;
    a.H = p.gated ? p.N / 2 : 0;
    a.G = p.gate_group;
    a.RB = pl.RB;
    a.ws_partial = p.ws_partial; a.ws_sumsq = p.ws_sumsq; a.counter = p.ws_counter;
    a.trace = p.trace; a.trace_groups = p.trace_groups;
    const bool fused = p.fused != 0, gated = p.gated != 0;
    return p.dt == F16 ? skinny_mb<Fp16>(a, fused, gated, pl, s) : skinny_mb<Bf16>(a, fused, gated, pl, s);
}

}  // namespace rmsnl
