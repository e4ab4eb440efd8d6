// Matrix-core variant of the fused RMSNorm + MatMul for large M (prefill): bound by the dense
// contraction, so the design is a 256x256 output tile per workgroup on v_mfma_f32_32x32x16.
//
//   * 8 waves, two per SIMD, in a 2x4 arrangement, each owning 128x64 of the tile = 4x2 MFMA tiles,
//     128 fp32 accumulators per lane (the B accumulator of the paper's fused kernel); 4 waves of
//     128x128 and a 128x512 tile are selectable and measured slower;
//   * K advances in steps of 64 through two LDS buffers.  X goes global -> registers -> LDS, and on
//     the way it is multiplied by g, rounded once to the 16-bit type (X-hat), and its raw squares
//     are added to a per-row running sum (the A accumulator): the two accumulations share the K
//     loop and the work is done once per workgroup, at staging, not per wave on fragments;
//   * W goes straight from global memory into LDS as it lies in memory ([k][n], n contiguous).  The
//     matrix instruction wants 8 consecutive k of one column per lane, so the B fragments are
//     fetched with the transposing LDS read (ds_read_b64_tr_b16): within 16 lanes, lane j supplies
//     the address of 4 columns of row j/4 and receives the 4 rows of column j;
//   * LDS rows are unpadded and their 16-byte chunks swizzled (X-hat: chunk c of row r at
//     c ^ ((r/2) & 7); W: at c ^ 4 (r & 3)), so that the 16-byte fragment reads and the transposing
//     reads fall on distinct banks and a direct load can fill whole rows;
//   * epilogue: rinv_i = 1/sqrt(A_i/K + eps) per row, Y = B * rinv in fp32, one rounding, store.
//
// Out-of-range rows of X and W read as zero through buffer resources; ragged M, N and K % 64 are
// handled by those reads and by guarded stores (N % 8 == 0 and K % 8 == 0 are required).
#include <algorithm>
#include "common.hpp"
#include <type_traits>

namespace rmsnl {

struct TileArgs {
    const u16* X; const u16* g; const u16* W; u16* Y;
    int M, K, N;
    float eps, inv_K;
    int tiles_m, tiles_n;
    int H;           // gated block: N = 2H, a tile is 128 gate columns and the up columns of the same outputs; else 0
    int G;           // gated block: layout of W, see gated_col()
    const float* rscale;   // plain product: per-row factor applied in the epilogue, or null
    // SPLIT kernels: workgroup (tile, slab) covers k in [slab * k_slab, +k_slab) and stores its
    // fp32 tile to part [slab][M][N]; tiles_m * tiles_n workgroups per slab
    int k_slab;
    float* part;
    // A launch may cover only tiles tile_base .. tile_base + tiles_here - 1 of the order below
    // (tiles_here = 0: all of them).  SPLIT launches of such a range store compact partial tiles,
    // part [slab][tile - tile_base][256][256].
    int tile_base, tiles_here;
};

// position b of the tile order -> tile row and column.  Workgroups are dealt round-robin to the 8
// XCDs, each with its own L2, and a compute unit holds one workgroup, so the 32 workgroups with
// positions 8 i + x, i in a run of 32, are what XCD x runs together; they should share few X and W
// panels.  When the tile rows divide into 8 bands of a multiple of 4 rows, XCD x works through band
// x, four rows at a time (4 x 8 tiles together).  Otherwise the tiles are listed panel by panel of
// 4 tile rows, column by column inside a panel, and that list is cut into runs of 32 which are
// dealt to the XCDs in turn: again blocks of 4 x 8 tiles, whatever the shape of the grid
// (2048 x 8192 x 8192: 3-5 % faster than row by row).  Positions beyond the last full round of 256
// are dealt in equal consecutive shares when they divide by 8, else one by one.
__device__ __host__ __forceinline__ void tile_at(int b, int tiles_m, int tiles_n, int* tm, int* tn)
{
    if ((tiles_m & 31) == 0) {
        const int band = tiles_m >> 3;               // tile rows per XCD
        const int x = b & 7, idx = b >> 3;           // idx in [0, band * tiles_n)
        const int per_grp = 4 * tiles_n;
        const int grp = idx / per_grp, in = idx % per_grp;
        *tm = x * band + grp * 4 + in % 4;
        *tn = in / 4;
        return;
    }
    const int tiles = tiles_m * tiles_n;
    const int base = tiles & ~255;
    int l = b;
    if (b < base) {
        const int x = b & 7, idx = b >> 3;
        l = (((idx >> 5) << 3) + x) * 32 + (idx & 31);
    } else if (((tiles - base) & 7) == 0) {
        const int r = b - base;
        l = base + (r & 7) * ((tiles - base) >> 3) + (r >> 3);
    }
    const int per_panel = 4 * tiles_n;
    const int panel = l / per_panel, in = l - panel * per_panel;
    const int left = tiles_m - 4 * panel;
    const int rows = left < 4 ? left : 4;
    *tm = 4 * panel + in % rows;
    *tn = in / rows;
}

void tile_order_at(int b, int tiles_m, int tiles_n, int* tm, int* tn) { tile_at(b, tiles_m, tiles_n, tm, tn); }

// Tile shapes: 0 = 256 rows x 256 columns (2 x NW/2 waves), 1 = 128 rows x 512 columns (1 x NW waves).
// The second halves the X-hat staging work per matrix instruction (an X tile then meets 512
// columns) for a quarter more traffic out of L2; at 8192^3 it measured 1-2 % slower with the
// operands in the last-level cache and 5 % slower with them in HBM, so the first is the default.
constexpr int BK = 64;
constexpr int tile_bm(int shape) { return shape ? 128 : 256; }
constexpr int tile_bn(int shape) { return shape ? 512 : 256; }
constexpr int LDA = BK;              // X-hat rows in LDS are unpadded (128 bytes), chunks swizzled
constexpr int kTileOut = 0x7ffffff0;
constexpr int kTileFlags = 0x00020000;
constexpr int kTileDefaultWaves = 8;
constexpr size_t tile_lds(int shape) { return size_t(2) * (tile_bm(shape) * LDA + BK * tile_bn(shape)) * 2; }
constexpr int kTileDefaultShape = 0;

template <typename T> struct Mfma32;
template <> struct Mfma32<Bf16> {
    static __device__ __forceinline__ float16_t run(uint4_t a, uint4_t b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma32<Fp16> {
    static __device__ __forceinline__ float16_t run(uint4_t a, uint4_t b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
};

typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((address_space(3))) short4_t* lds_short4_ptr;

// transposing LDS read of 4 x 16-bit values (see the header comment)
__device__ __forceinline__ uint2_t lds_read_tr(const u16* p) {
    short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p));
    return __builtin_bit_cast(uint2_t, v);
}

// sum of the squares of a packed pair of 16-bit values, added to acc (one v_dot2c instead of two
// unpacks and two fused multiply-adds)
template <typename T> struct SqPair;
template <> struct SqPair<Bf16> {
    static __device__ __forceinline__ float add(uint32_t p, float acc) {
        const bf16x2_t v = __builtin_bit_cast(bf16x2_t, p);
        return __builtin_amdgcn_fdot2_f32_bf16(v, v, acc, false);
    }
};
template <> struct SqPair<Fp16> {
    static __device__ __forceinline__ float add(uint32_t p, float acc) {
        const f16x2_t v = __builtin_bit_cast(f16x2_t, p);
        return __builtin_amdgcn_fdot2(v, v, acc, false);
    }
};

// s_waitcnt that waits only for the vector-memory counter to drop to n (n <= 63)
#define RL_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// NW waves per workgroup: 4 (128x128 per wave, one wave per SIMD) or 8 (128x64 per wave, two waves
// per SIMD that cover each other's stalls); SHAPE: the tile shape, see tile_bm / tile_bn.
//
// GATED (the GatedMLP block on top): the tile's 256 columns are 128 outputs' gate and up columns,
// laid out so that MFMA tiles j and j + TN/2 of a wave are gate and up of the same 32 outputs; the
// epilogue then forms SiLU(gate) * up in registers.  Only the column a lane fetches changes.
// SPLIT (plain product only): the K range is split over workgroups, which leave fp32 partial tiles
// for tile_reduce_kernel to add up, for shapes with too few tiles to fill the chip.
template <typename T, bool FUSED, int NW, bool GATED, int SHAPE, bool SPLIT = false, bool BIGW = false>
__global__ __launch_bounds__(64 * NW, NW / 4) void tile_kernel(TileArgs a)
{
    static_assert(!SPLIT || (!FUSED && !GATED), "split-K runs the plain product");
    constexpr int BM = tile_bm(SHAPE), BN = tile_bn(SHAPE);
    constexpr int NT = 64 * NW;                  // threads
    constexpr int WM = SHAPE ? 1 : 2;            // waves along M
    constexpr int WN = NW / WM;                  // waves along N
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // MFMA tiles per wave along M (4) and N
    constexpr int NJ = BM * 8 / NT;              // 16-byte chunks of X a thread stages per K tile
    constexpr int XR = NT / 8;                   // row stride between a thread's X chunks
    constexpr int RPL = 512 / BN;                // rows of the W tile in one 1 KiB direct load (2 or 1)
    constexpr int NP = BK / RPL / NW;            // direct-to-LDS loads of W per wave and K tile
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    u16* As = (u16*)lds_raw;                             // [2][BM][LDA], chunks swizzled
    u16* Bs = As + 2 * BM * LDA;                         // [2][BK][BN], chunks swizzled
    float* s_ss = (float*)lds_raw;                       // [BM] sums of squares: over As once the K loop is done
    float* s_rinv = s_ss + BM;                           // [BM]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    int tm, tn;
    const int n_tiles = a.tiles_here ? a.tiles_here : a.tiles_m * a.tiles_n;   // tiles of this launch
    const int slab = SPLIT ? int(blockIdx.x) / n_tiles : 0;
    const int kb = SPLIT ? slab * a.k_slab : 0;                     // first k of this workgroup
    const int Kend = SPLIT ? min(a.K, kb + a.k_slab) : a.K;         // k at or beyond it reads as zero
    const int t_local = SPLIT ? int(blockIdx.x) % n_tiles : int(blockIdx.x);
    tile_at(t_local + a.tile_base, a.tiles_m, a.tiles_n, &tm, &tn);
    const int m0 = tm * BM, n0 = GATED ? tn * (BN / 2) : tn * BN;   // gated: first output column of the tile
    const int rows_here = min(BM, a.M - m0);

    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(a.X + size_t(m0) * a.K), 0, rows_here * a.K * 2, kTileFlags);
    const __amdgpu_buffer_rsrc_t grs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(FUSED ? a.g : a.X), 0, a.K * 2, kTileFlags);

    // ---- X staging role: chunk j of this thread is row ar + XR j, the 8 k from ac.  Byte offsets
    // inside the tile's rows; a row at or beyond rows_here lies beyond the resource and reads zero.
    const int ar = tid >> 3, ac = (tid & 7) * 8;
    int xoff[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) xoff[j] = ((ar + XR * j) * a.K + ac) * 2;

    // ---- W role: load p of this wave brings RPL rows of the K tile, from row RPL (wave + NW p),
    // = 1 KiB, straight into LDS.  A direct load writes lane l's 16 bytes at byte 16 l of that KiB,
    // so lane l fetches the chunk that belongs there: row l / (64 / RPL), and, with the swizzle
    // "chunk c of row r sits at chunk c ^ 4 (r & 3)", chunk (l % (64 / RPL)) ^ 4 (r & 3).
    // (RPL NW p is a multiple of 4, so r & 3 does not depend on p.)
    const int wrow = RPL * wave + lane / (64 / RPL);
    const int wchunk = (lane % (64 / RPL)) ^ (4 * (wrow & 3));
    int wcol = n0 + 8 * wchunk;
    bool wcol_ok = wcol < a.N;
    if (GATED) {
        // tile column 8 wchunk belongs to wave column wc, MFMA tile jn, lane column jj of it
        const int wc = (8 * wchunk) / (BN / WN), within = (8 * wchunk) % (BN / WN);
        const int jn = within / 32, jj = within % 32;
        const int hc = wc * (BN / WN / 2) + (jn % (TN / 2)) * 32 + jj;       // output column inside the tile
        wcol = gated_col(n0 + hc, jn >= TN / 2, a.H, a.G);
        wcol_ok = n0 + hc < a.H;
    }
    const int woff = wcol_ok ? (wrow * a.N + wcol) * 2 : kTileOut;

    uint4_t xa[NJ], gv;
    // Global loads of tile k0.  Unchecked form (the whole tile lies inside K): per-thread offsets
    // never change, the tile's position rides in the scalar offset.  Checked form: everything goes
    // through the vector offset, which is what the range check looks at, so that k at or beyond K
    // reads zero (ragged last tile, and the prefetches that run past the end).
    auto load_x = [&](auto checked, int k0, int j) {
        k0 += kb;
        if constexpr (decltype(checked)::value) {
            const bool kin = k0 + ac < Kend;
            if (FUSED && j == 0) gv = __builtin_amdgcn_raw_buffer_load_b128(grs, kin ? (k0 + ac) * 2 : kTileOut, 0, 0);
            xa[j] = __builtin_amdgcn_raw_buffer_load_b128(xrs, kin ? xoff[j] + k0 * 2 : kTileOut, 0, 0);
        } else {
            if (FUSED && j == 0) gv = __builtin_amdgcn_raw_buffer_load_b128(grs, ac * 2, k0 * 2, 0);
            xa[j] = __builtin_amdgcn_raw_buffer_load_b128(xrs, xoff[j], k0 * 2, 0);
        }
    };
    // The direct load is written in assembly: as a builtin, the compiler takes every later LDS read
    // for a possible reader of the bytes in flight and waits for all outstanding loads first.  The
    // waits for these loads are therefore placed by hand (RL_WAIT_VM before the barriers).
    // (rows of W at or beyond Kend lie beyond the resource)
    uint4_t wdesc = {uint32_t(uintptr_t(a.W)), uint32_t(uintptr_t(a.W) >> 32), uint32_t(BIGW ? 0 : Kend * a.N * 2),
                           uint32_t(kTileFlags)};
    // BIGW (K x N x 2 bytes >= 2^31, W may exceed 4 GiB): the resource of a load starts at the first row
    // the load brings, so byte offsets inside it stay small; it ends with the slab's last row (rows at
    // or beyond Kend read zero), or 2 GiB further on, whichever comes first; kTileOut lies beyond
    // either.  Costs 1-2 % at 8192^3 (a 64-bit product per load), so only large W takes it.
    const uint64_t wbase = uint64_t(uintptr_t(a.W));
    const uint64_t wrow_bytes = uint64_t(a.N) * 2u;
    uint32_t bs_base = uint32_t(uintptr_t(Bs)) + uint32_t(wave) * 1024;         // LDS byte address of this wave's first KiB
    auto load_w = [&](auto checked, int buf, int k0, int p) {
        if constexpr (BIGW) {
            const uint32_t dst = bs_base + uint32_t(buf * BK * BN * 2 + NW * p * 1024);
            const int krow = kb + k0 + RPL * NW * p;             // first row of W this load brings
            const uint64_t base = wbase + uint64_t(krow) * wrow_bytes;
            const int64_t left = int64_t(Kend - krow) * int64_t(wrow_bytes);
            const uint32_t nrec = left <= 0 ? 0u : left > 0x7fffffe0 ? 0x7fffffe0u : uint32_t(left);
            const uint4_t desc = {uint32_t(base), uint32_t(base >> 32), nrec, uint32_t(kTileFlags)};
            const int v = woff;
            uint32_t keep;                       // M0 carries the LDS address; whatever it held is put back
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                         "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                         : "=&s"(keep) : "s"(dst), "v"(v), "s"(desc) : "memory");
        } else {
            const uint32_t dst = bs_base + uint32_t(buf * BK * BN * 2 + NW * p * 1024);
            const unsigned rowoff = unsigned(kb + k0 + RPL * NW * p) * unsigned(a.N) * 2u;
            int v = woff, so = int(rowoff);
            if constexpr (decltype(checked)::value) {
                v = woff == kTileOut ? kTileOut : int(unsigned(woff) + rowoff);
                so = 0;
            }
            const uint4_t desc = wdesc;          // (operands of an asm inside a generic lambda must be its own locals)
            uint32_t keep;                       // M0 carries the LDS address; whatever it held is put back
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                         "buffer_load_dwordx4 %2, %3, %4 offen lds\n\ts_mov_b32 m0, %0"
                         : "=&s"(keep) : "s"(dst), "v"(v), "s"(desc), "s"(so) : "memory");
        }
    };

    float ssq[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) ssq[j] = 0.f;

    // one staged X chunk: squares of the raw values, times g, one rounding, into LDS
    float gf[8];
    auto unpack_g = [&]() {
        if (FUSED) {
#pragma unroll
            for (int e = 0; e < 4; ++e) { gf[2 * e] = Elem<T>::lo(gv[e]); gf[2 * e + 1] = Elem<T>::hi(gv[e]); }
        }
    };
    // (three-operand dot products against a masked g, which need no unpacking, were tried for
    // the products: fewer instructions, same time)
    auto stage = [&](int buf, int j) {
        uint4_t o = xa[j];
        if (FUSED) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ssq[j] = SqPair<T>::add(o[e], ssq[j]);
                o[e] = Elem<T>::pack(Elem<T>::lo(o[e]) * gf[2 * e], Elem<T>::hi(o[e]) * gf[2 * e + 1]);
            }
        }
        // chunk c of row r sits at chunk c ^ ((r / 2) & 7) of the row's 128 bytes ((XR j) / 2 is a multiple of 8)
        *(uint4_t*)(As + buf * BM * LDA + (ar + XR * j) * LDA + (ac ^ (8 * ((ar >> 1) & 7)))) = o;
    };

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // fragment addresses.  A: row wm*(BM/WM) + i*32 + lane%32, k chunk 2 ks + lane/32 of the K tile, at
    // its swizzled place (32 i rows further on the swizzle is the same).  B: 16-lane block blk, lane
    // jj in it: row 8*(blk/2) + jj/4 (+4 for the second read), columns 16*(blk%2) + 4*(jj%4) of MFMA
    // tile i, at the swizzled place of that row.
    const int a_row = wm * (BM / WM) + (lane & 31);
    int a_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) a_off[ks] = a_row * LDA + 8 * ((2 * ks + (lane >> 5)) ^ ((a_row >> 1) & 7));
    const int blk = lane >> 4, jj = lane & 15;
    const int b_row = 8 * (blk >> 1) + (jj >> 2);
    int b_off[TN];
#pragma unroll
    for (int i = 0; i < TN; ++i)
        b_off[i] = b_row * BN + ((wn * (BN / WN) + i * 32 + 16 * (blk & 1)) ^ (32 * (b_row & 3))) + 4 * (jj & 3);

    // Two sets of fragments: while the matrix cores work on one 16-deep K step, the LDS reads of
    // the next step land in the other set.
    uint4_t af[2][TM], bf[2][TN];
    auto read_frag = [&](int set, int buf, int ks, int i) {      // A fragment i and B fragment i of step ks
        const u16* Ab = As + buf * BM * LDA + a_off[ks];
        const u16* Bb = Bs + buf * BK * BN + (ks * 16) * BN;
        af[set][i] = *(const uint4_t*)(Ab + i * 32 * LDA);
        if (i < TN) {
            const uint2_t lo = lds_read_tr(Bb + b_off[i]);
            const uint2_t hi = lds_read_tr(Bb + b_off[i] + 4 * BN);
            bf[set][i] = uint4_t{lo[0], lo[1], hi[0], hi[1]};
        }
    };
    auto mfma_row = [&](int set, int i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = Mfma32<T>::run(af[set][i], bf[set][j], acc[i][j]);
    };
    // the staging work that belongs to group i (of 4) of a step
    auto for_pieces = [&](int n, int i, auto fn) {
#pragma unroll
        for (int p = 0; p < n; ++p)
            if (p * 4 / n == i) fn(p);
    };
#define RL_SB() __builtin_amdgcn_sched_barrier(0)
    const std::integral_constant<bool, true> checked_c;
    const std::integral_constant<bool, false> unchecked_c;

    // ---- prologue: tile 0 into LDS buffer 0, its first fragments into set 0, tile 1 on its way
    const int nk = (Kend - kb + BK - 1) / BK;
#pragma unroll
    for (int p = 0; p < NP; ++p) load_w(checked_c, 0, 0, p);
#pragma unroll
    for (int j = 0; j < NJ; ++j) load_x(checked_c, 0, j);
    unpack_g();
#pragma unroll
    for (int j = 0; j < NJ; ++j) stage(0, j);
    RL_WAIT_VM(0);                                       // this wave's part of W tile 0 is in LDS
    __syncthreads();
#pragma unroll
    for (int p = 0; p < NP; ++p) load_w(checked_c, 1, BK, p);
#pragma unroll
    for (int j = 0; j < NJ; ++j) load_x(checked_c, BK, j);
#pragma unroll
    for (int i = 0; i < 4; ++i) read_frag(0, 0, 0, i);

    // ---- main loop, branch free: beyond the last tile the loads return zeros and the extra LDS
    // traffic touches only the buffer nobody reads any more.  At entry of iteration kt: LDS buffer
    // cur holds tile kt, fragment set 0 its first step, the X registers tile kt+1 (on its way),
    // and the direct loads of W tile kt+1 into buffer nxt are on their way.
    //   step 0: MFMA on set 0 | read step 1 -> set 1
    //   step 1: MFMA on set 1 | read step 2 -> set 0 | stage the first half of X tile kt+1, reload
    //   step 2: MFMA on set 0 | read step 3 -> set 1 | stage the second half, reload
    //   wait for this wave's W loads of tile kt+1, barrier (tile kt+1 complete in nxt; all of
    //   this tile's fragments are in registers)
    //   step 3: MFMA on set 1 | read next tile's step 0 -> set 0 | W tile kt+2 -> buffer cur
    // (In the plain product X could take W's road straight into LDS; measured 1 % slower at 8192^3
    // and 7 % slower at 256 x 8192 x 8192 than going through registers two tiles ahead.)
    // An X register is reloaded, for tile kt+2, in the very group that has just stored it: every
    // global load then has a whole K tile of matrix work to arrive in, and the loads stay spread
    // out one or two per group of MFMAs.
    auto iteration = [&](auto chk, int kt) {
        const int cur = kt & 1, nxt = cur ^ 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) { read_frag(1, cur, 1, i); mfma_row(0, i); RL_SB(); }
        unpack_g();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            read_frag(0, cur, 2, i);
            mfma_row(1, i);
            for_pieces(NJ / 2, i, [&](int p) { stage(nxt, p); load_x(chk, (kt + 2) * BK, p); });
            RL_SB();
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            read_frag(1, cur, 3, i);
            mfma_row(0, i);
            for_pieces(NJ / 2, i, [&](int p) { stage(nxt, NJ / 2 + p); load_x(chk, (kt + 2) * BK, NJ / 2 + p); });
            RL_SB();
        }
        // the W loads of tile kt+1 are older than this iteration's NJ + 1 reloads (the g chunk rides with X chunk 0)
        RL_WAIT_VM(FUSED ? NJ + 1 : NJ);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            read_frag(0, nxt, 0, i);
            mfma_row(1, i);
            for_pieces(NP, i, [&](int p) { load_w(chk, cur, (kt + 2) * BK, p); });
            RL_SB();
        }
    };
    // iterations whose prefetches (tile kt+2) lie wholly inside K take the unchecked loads
    const int n_fast = max(0, (Kend - kb) / BK - 2);
    for (int kt = 0; kt < n_fast; ++kt) iteration(unchecked_c, kt);
    for (int kt = n_fast; kt < nk; ++kt) iteration(checked_c, kt);
#undef RL_SB
    RL_WAIT_VM(0);                                       // nothing may still be writing LDS past this point

    // ---- A_i: the 8 threads that share a row (tid & 7) add their shares (s_ss lies over the X-hat
    // buffers, which nobody needs any more once every wave has left the K loop)
    if (FUSED) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float v = ssq[j];
            v += __shfl_xor(v, 1, 64);
            v += __shfl_xor(v, 2, 64);
            v += __shfl_xor(v, 4, 64);
            if ((tid & 7) == 0) s_ss[ar + XR * j] = v;
        }
        __syncthreads();
        if (tid < BM) s_rinv[tid] = row_scale(s_ss[tid], a.inv_K, a.eps);
        __syncthreads();
    } else if (a.rscale) {                               // uniform: the rows' factors come from the caller
        __syncthreads();
        if (tid < BM) s_rinv[tid] = m0 + tid < a.M ? a.rscale[m0 + tid] : 0.f;
        __syncthreads();
    }
    const bool scaled = FUSED || a.rscale != nullptr;

    // ---- epilogue: D register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its tile.
    // Y is stored with the non-temporal hint: nothing reads it again here, and the L2 keeps the operand
    // panels instead (4096 x 4096 x 28672: 813 -> 791 us, 4096^3: 127 -> 125 us, 8192^3: no change).
    const int col_l = lane & 31, rowq = 4 * (lane >> 5);
    if constexpr (SPLIT) {
        const bool compact = a.tiles_here != 0;          // [slab][tile][BM][BN] instead of [slab][M][N]
        float* base = compact ? a.part + (size_t(slab) * n_tiles + t_local) * (BM * BN)
                              : a.part + size_t(slab) * a.M * a.N;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * (BM / WM) + i * 32 + 8 * (r >> 2) + rowq + (r & 3);
                if (m0 + row < a.M) {
                    const int ct = wn * (BN / WN) + col_l;       // column inside the tile
                    float* prow = compact ? base + row * BN + ct : base + size_t(m0 + row) * a.N + n0 + ct;
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        if (n0 + ct + j * 32 < a.N) prow[j * 32] = acc[i][j][r];
                }
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = wm * (BM / WM) + i * 32 + 8 * (r >> 2) + rowq + (r & 3);
            const float ri = scaled ? s_rinv[row] : 1.f;
            if (m0 + row < a.M) {
                if (GATED) {
                    const int c0 = n0 + wn * (BN / WN / 2) + col_l;
                    u16* yrow = a.Y + size_t(m0 + row) * a.H + c0;
#pragma unroll
                    for (int j = 0; j < TN / 2; ++j)
                        if (c0 + j * 32 < a.H)
                            __builtin_nontemporal_store(Elem<T>::from_f32(silu(acc[i][j][r] * ri) * (acc[i][j + TN / 2][r] * ri)), &yrow[j * 32]);
                } else {
                    const int c0 = n0 + wn * (BN / WN) + col_l;
                    u16* yrow = a.Y + size_t(m0 + row) * a.N + c0;
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        if (c0 + j * 32 < a.N) __builtin_nontemporal_store(Elem<T>::from_f32(acc[i][j][r] * ri), &yrow[j * 32]);
                }
            }
        }
}

// ------------------------------------------------------------------------------------------- host
template <typename T, bool FUSED, int NW, bool GATED, int SHAPE, bool BIGW = false>
static hipError_t tile_go(const TileArgs& a, dim3 grid, hipStream_t s)
{
    static LdsOnce once;
    hipError_t e = raise_lds_once(once, {(const void*)tile_kernel<T, FUSED, NW, GATED, SHAPE, false, BIGW>}, int(tile_lds(SHAPE)));
    if (e != hipSuccess) return e;
    tile_kernel<T, FUSED, NW, GATED, SHAPE, false, BIGW><<<grid, 64 * NW, tile_lds(SHAPE), s>>>(a);
    return hipGetLastError();
}

// W of 2 GiB or more: addressed row by row (see the kernel); the default tile shape only
static bool tile_big_w(const Problem& p) { return int64_t(p.K) * p.N * 2 >= (int64_t(1) << 31); }

template <typename T, bool FUSED, bool GATED>
static hipError_t tile_nw(const TileArgs& a, dim3 grid, int nw, int shape, bool big, hipStream_t s)
{
    if (big) return tile_go<T, FUSED, 8, GATED, 0, true>(a, grid, s);
    if (shape) return nw == 8 ? tile_go<T, FUSED, 8, GATED, 1>(a, grid, s) : tile_go<T, FUSED, 4, GATED, 1>(a, grid, s);
    return nw == 8 ? tile_go<T, FUSED, 8, GATED, 0>(a, grid, s) : tile_go<T, FUSED, 4, GATED, 0>(a, grid, s);
}

hipError_t launch_tile(const Problem& p, hipStream_t s, const char** why)
{
    if (p.dt == F32) { if (why) *why = "tile variant handles 16-bit types only"; return hipErrorInvalidValue; }
    if (p.N % 8 != 0 || p.K % 8 != 0) {
        if (why) *why = "tile variant needs N % 8 == 0 and K % 8 == 0";
        return hipErrorInvalidValue;
    }
    if (int64_t(256) * p.K * 2 >= (int64_t(1) << 31) || p.N >= (1 << 25)) {
        if (why) *why = "tile variant needs K < 2^22 and N < 2^25";
        return hipErrorInvalidValue;
    }
    const bool big = tile_big_w(p);
    if (big && ((p.k_split != 0 && p.k_split != 8) || (p.n_tile != 0 && p.n_tile != 256))) {
        if (why) *why = "tile variant: a W of 2 GiB or more runs 256x256 tiles with 8 waves only";
        return hipErrorInvalidValue;
    }
    // tuning: k_split carries the waves per workgroup for this variant (0 = default)
    if (p.k_split != 0 && p.k_split != 4 && p.k_split != 8) {
        if (why) *why = "tile variant: k_split selects 4 or 8 waves per workgroup";
        return hipErrorInvalidValue;
    }
    const int nw = p.k_split ? p.k_split : kTileDefaultWaves;
    // tuning: n_tile carries the tile shape for this variant (0 = default, 256 = 256x256, 512 = 128x512)
    if (p.n_tile != 0 && p.n_tile != 256 && p.n_tile != 512) {
        if (why) *why = "tile variant: n_tile selects 256 (256x256 tiles) or 512 (128x512 tiles)";
        return hipErrorInvalidValue;
    }
    const int shape = p.n_tile ? (p.n_tile == 512) : kTileDefaultShape;
    const int BM = tile_bm(shape), BN = tile_bn(shape);
    TileArgs a;
    a.X = (const u16*)p.X; a.g = (const u16*)p.g; a.W = (const u16*)p.W; a.Y = (u16*)p.Y;
    a.M = p.M; a.K = p.K; a.N = p.N; a.eps = p.eps; a.inv_K = 1.0f / float(p.K);
    if (p.gated && (p.N % 16 != 0 || (!p.fused && !p.rscale))) {
        if (why) *why = "gated block: tile variant needs H % 8 == 0";
        return hipErrorInvalidValue;
    }
    a.H = p.gated ? p.N / 2 : 0;
    a.G = p.gate_group;
    a.rscale = p.fused ? nullptr : p.rscale;
    a.k_slab = 0; a.part = nullptr; a.tile_base = 0; a.tiles_here = 0;
    a.tiles_m = (p.M + BM - 1) / BM;
    a.tiles_n = p.gated ? (a.H + BN / 2 - 1) / (BN / 2) : (p.N + BN - 1) / BN;
    if (int64_t(a.tiles_m) * a.tiles_n >= (int64_t(1) << 31)) {
        if (why) *why = "too many tiles";
        return hipErrorInvalidValue;
    }
    if (p.tile_limit < 0 || p.tile_limit > a.tiles_m * a.tiles_n) { if (why) *why = "bad tile range"; return hipErrorInvalidValue; }
    a.tiles_here = p.tile_limit;
    dim3 grid(p.tile_limit ? p.tile_limit : a.tiles_m * a.tiles_n);
    if (p.plan) { p.plan[0] = BN; p.plan[1] = nw; p.plan[2] = int(grid.x); }
    const bool fused = p.fused != 0;
    if (p.gated && !fused)                  // gate over a product of a materialised X-hat, scaled per row
        return p.dt == F16 ? tile_nw<Fp16, false, true>(a, grid, nw, shape, big, s) : tile_nw<Bf16, false, true>(a, grid, nw, shape, big, s);
    if (p.gated)
        return p.dt == F16 ? tile_nw<Fp16, true, true>(a, grid, nw, shape, big, s) : tile_nw<Bf16, true, true>(a, grid, nw, shape, big, s);
    if (p.dt == F16)
        return fused ? tile_nw<Fp16, true, false>(a, grid, nw, shape, big, s) : tile_nw<Fp16, false, false>(a, grid, nw, shape, big, s);
    return fused ? tile_nw<Bf16, true, false>(a, grid, nw, shape, big, s) : tile_nw<Bf16, false, false>(a, grid, nw, shape, big, s);
}

// --------------------------------------------------------- split-K product for shapes with few tiles
// part [S][M][N] fp32 -> Y: slabs added in order, rows scaled, one rounding (and, for the gated block,
// column h paired with column H + h).  One thread per four output columns.
template <typename T, bool GATED>
__global__ __launch_bounds__(256) void tile_reduce_kernel(const float* __restrict__ part, const float* __restrict__ rscale,
                                                          u16* __restrict__ Y, int M, int N, int S, int G)
{
    const int H = N / 2;
    const int cols4 = (GATED ? H : N) / 4;               // groups of four output columns per row
    const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= int64_t(M) * cols4) return;
    const int row = int(idx / cols4), c = int(idx % cols4) * 4;
    const size_t slab = size_t(M) * N;
    const float* src = part + size_t(row) * N + (GATED ? gated_col(c, false, H, G) : c);
    const int up = GATED ? gated_col(c, true, H, G) - gated_col(c, false, H, G) : 0;   // from the gate quad to the up quad
    float4_t v = *(const float4_t*)src, u = float4_t{0.f, 0.f, 0.f, 0.f};
    if (GATED) u = *(const float4_t*)(src + up);
    for (int s = 1; s < S; ++s) {
        const float4_t t = *(const float4_t*)(src + s * slab);
        v += t;
        if (GATED) u += *(const float4_t*)(src + s * slab + up);
    }
    const float ri = rscale ? rscale[row] : 1.f;
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = GATED ? silu(v[e] * ri) * (u[e] * ri) : v[e] * ri;
    uint2_t out = {Elem<T>::pack(o[0], o[1]), Elem<T>::pack(o[2], o[3])};
    *(uint2_t*)(Y + size_t(row) * (GATED ? H : N) + c) = out;
}

// slabs for a plain product whose 256x256 tiles number `tiles`: enough to give every compute unit a
// workgroup, each slab a multiple of 64 rows and at least 256 of them
static void tile_split_plan(int K, int64_t tiles, int* S, int* k_slab)
{
    int s = int(std::min<int64_t>(16, 256 / std::max<int64_t>(tiles, 1)));
    s = std::min(s, std::max(1, K / 256));
    if (s < 2) { *S = 1; *k_slab = K; return; }
    int ks = ((K + s - 1) / s + BK - 1) / BK * BK;
    *S = (K + ks - 1) / ks;
    *k_slab = ks;
}

// the product of a materialised X-hat in S slabs + the reduction; part has room for [S][M][N] fp32
static hipError_t launch_tile_split(const Problem& q, int S, int k_slab, float* part, hipStream_t s)
{
    TileArgs a;
    a.X = (const u16*)q.X; a.g = nullptr; a.W = (const u16*)q.W; a.Y = (u16*)q.Y;
    a.M = q.M; a.K = q.K; a.N = q.N; a.eps = 0.f; a.inv_K = 0.f;
    a.H = 0; a.G = 0; a.rscale = nullptr; a.k_slab = k_slab; a.part = part; a.tile_base = 0; a.tiles_here = 0;
    a.tiles_m = (q.M + 255) / 256;
    a.tiles_n = (q.N + 255) / 256;
    dim3 grid(a.tiles_m * a.tiles_n * S);
    static LdsOnce once;
    hipError_t e = raise_lds_once(once, {(const void*)tile_kernel<Fp16, false, 8, false, 0, true>,
                                         (const void*)tile_kernel<Bf16, false, 8, false, 0, true>}, int(tile_lds(0)));
    if (e != hipSuccess) return e;
    if (q.dt == F16) tile_kernel<Fp16, false, 8, false, 0, true><<<grid, 512, tile_lds(0), s>>>(a);
    else             tile_kernel<Bf16, false, 8, false, 0, true><<<grid, 512, tile_lds(0), s>>>(a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t groups = int64_t(q.M) * ((q.gated ? q.N / 2 : q.N) / 4);
    dim3 rgrid((unsigned)((groups + 255) / 256));
    u16* Y = (u16*)q.Y;
    if (q.dt == F16) {
        if (q.gated) tile_reduce_kernel<Fp16, true><<<rgrid, 256, 0, s>>>(part, q.rscale, Y, q.M, q.N, S, q.gate_group);
        else         tile_reduce_kernel<Fp16, false><<<rgrid, 256, 0, s>>>(part, q.rscale, Y, q.M, q.N, S, 0);
    } else {
        if (q.gated) tile_reduce_kernel<Bf16, true><<<rgrid, 256, 0, s>>>(part, q.rscale, Y, q.M, q.N, S, q.gate_group);
        else         tile_reduce_kernel<Bf16, false><<<rgrid, 256, 0, s>>>(part, q.rscale, Y, q.M, q.N, S, 0);
    }
    return hipGetLastError();
}

// ---------------------------------------------------- the last, partial round of tiles split over K
// A grid of t tiles runs in ceil(t / 256) rounds on 256 compute units, however little the last round
// holds.  When the last round holds few tiles (at most 128), the full rounds run unsplit and the
// remaining tiles are split over K so that they fill one short round, with compact fp32 partial tiles
// and a reduction over just those tiles.
template <typename T>
__global__ __launch_bounds__(256) void tile_reduce_rem_kernel(const float* __restrict__ part, const float* __restrict__ rscale,
                                                              u16* __restrict__ Y, int M, int N, int S,
                                                              int tiles_m, int tiles_n, int tile_base, int rem)
{
    const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;      // one thread per four columns of a tile row
    const int t = int(idx / (256 * 64));
    if (t >= rem) return;
    const int r = int(idx % (256 * 64)) / 64, c = (int(idx) & 63) * 4;
    int tm, tn;
    tile_at(tile_base + t, tiles_m, tiles_n, &tm, &tn);
    const int m = tm * 256 + r, n = tn * 256 + c;
    if (m >= M || n >= N) return;
    const float* src = part + (size_t(t) * 256 + r) * 256 + c;
    const size_t slab = size_t(rem) * 256 * 256;
    float4_t v = *(const float4_t*)src;
    for (int s = 1; s < S; ++s) v += *(const float4_t*)(src + s * slab);
    const float ri = rscale ? rscale[m] : 1.f;
    uint2_t out = {Elem<T>::pack(v[0] * ri, v[1] * ri), Elem<T>::pack(v[2] * ri, v[3] * ri)};
    *(uint2_t*)(Y + size_t(m) * N + n) = out;
}

// full rounds, remainder and its slabs for a plain product (rem = 0: no such split)
static void tile_rem_plan(const Problem& p, int* full, int* rem, int* S, int* k_slab)
{
    const int64_t tiles = int64_t((p.M + 255) / 256) * ((p.N + 255) / 256);
    *full = int(tiles / 256 * 256);
    *rem = 0; *S = 1; *k_slab = p.K;
    if (p.gated || tiles <= 256 || tiles > (int64_t(1) << 24) || tile_big_w(p)) return;
    const int r = int(tiles - *full);
    int s = r ? std::min(16, 256 / r) : 1;
    s = std::min(s, std::max(1, p.K / 256));
    if (p.n_tile == 2) s = (p.k_split >= 1 && p.k_split <= 16) ? p.k_split : 1;   // tuning override of this split only
    if (r == 0 || s < 2) return;
    const int ks = ((p.K + s - 1) / s + BK - 1) / BK * BK;
    *rem = r; *S = (p.K + ks - 1) / ks; *k_slab = ks;
    if (*S < 2) { *rem = 0; *S = 1; *k_slab = p.K; }
}

// q: the plain product (X-hat materialised or a plain matmul).  Tiles [0, full) unsplit, the rest in S slabs.
static hipError_t launch_tile_rem(const Problem& q, int full, int rem, int S, int k_slab, float* part, hipStream_t s,
                                  const char** why)
{
    Problem head = q;
    head.tile_limit = full;
    head.n_tile = 0; head.k_split = 0;
    hipError_t e = launch_tile(head, s, why);
    if (e != hipSuccess) return e;
    TileArgs a;
    a.X = (const u16*)q.X; a.g = nullptr; a.W = (const u16*)q.W; a.Y = (u16*)q.Y;
    a.M = q.M; a.K = q.K; a.N = q.N; a.eps = 0.f; a.inv_K = 0.f;
    a.H = 0; a.G = 0; a.rscale = nullptr; a.k_slab = k_slab; a.part = part; a.tile_base = full; a.tiles_here = rem;
    a.tiles_m = (q.M + 255) / 256;
    a.tiles_n = (q.N + 255) / 256;
    dim3 grid(rem * S);
    static LdsOnce once;
    e = raise_lds_once(once, {(const void*)tile_kernel<Fp16, false, 8, false, 0, true>,
                              (const void*)tile_kernel<Bf16, false, 8, false, 0, true>}, int(tile_lds(0)));
    if (e != hipSuccess) return e;
    if (q.dt == F16) tile_kernel<Fp16, false, 8, false, 0, true><<<grid, 512, tile_lds(0), s>>>(a);
    else             tile_kernel<Bf16, false, 8, false, 0, true><<<grid, 512, tile_lds(0), s>>>(a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 rgrid((unsigned)(rem * 64));        // 256 x 64 threads per tile
    if (q.dt == F16) tile_reduce_rem_kernel<Fp16><<<rgrid, 256, 0, s>>>(part, q.rscale, (u16*)q.Y, q.M, q.N, S, a.tiles_m, a.tiles_n, full, rem);
    else             tile_reduce_rem_kernel<Bf16><<<rgrid, 256, 0, s>>>(part, q.rscale, (u16*)q.Y, q.M, q.N, S, a.tiles_m, a.tiles_n, full, rem);
    return hipGetLastError();
}

// ------------------------------------------------------------------- two-kernel form for large M
// The fused tile kernel converts its 256 rows of X to X-hat once per workgroup, so a problem with
// N / 256 workgroup columns repeats that conversion N / 256 times, on the same vector units that
// have to feed the matrix cores.  For large M and N it is cheaper to write X-hat (rounded once, as in
// the fused kernel) and 1 / rms per row to device memory in a first, memory-bound kernel and to run
// the tile kernel as a plain product whose epilogue applies the row factors (Fig. 2b's division after
// the product, with the normalised input materialised as in Fig. 2a).
// One workgroup per row.  PER > 0: the row has at most 256 * PER 16-byte chunks and a thread's
// loads are all issued before the first is used; PER = 0: any K, one chunk at a time.
template <typename T, int PER>
__global__ __launch_bounds__(256) void xhat_rows_kernel(const uint4_t* __restrict__ X, const uint4_t* __restrict__ g,
                                                        uint4_t* __restrict__ Xh, float* __restrict__ rscale,
                                                        int K8, float eps, float inv_K)
{
    __shared__ float part[4];
    const size_t row = size_t(blockIdx.x) * K8;
    float ss = 0.f;
    auto one = [&](uint4_t xv, uint4_t gv) {
        uint4_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x0 = Elem<T>::lo(xv[e]), x1 = Elem<T>::hi(xv[e]);
            ss = __fmaf_rn(x0, x0, ss);
            ss = __fmaf_rn(x1, x1, ss);
            o[e] = Elem<T>::pack(x0 * Elem<T>::lo(gv[e]), x1 * Elem<T>::hi(gv[e]));
        }
        return o;
    };
    if constexpr (PER > 0) {
        uint4_t xv[PER], gv[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int c = threadIdx.x + j * 256;
            xv[j] = c < K8 ? X[row + c] : uint4_t{0, 0, 0, 0};
            gv[j] = c < K8 ? g[c] : uint4_t{0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int c = threadIdx.x + j * 256;
            const uint4_t o = one(xv[j], gv[j]);
            if (c < K8) Xh[row + c] = o;
        }
    } else {
        for (int c = threadIdx.x; c < K8; c += 256) Xh[row + c] = one(X[row + c], g[c]);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) rscale[blockIdx.x] = row_scale((part[0] + part[1]) + (part[2] + part[3]), inv_K, eps);
}

template <typename T>
static void xhat_rows_go(const Problem& p, uint4_t* Xh, float* rscale, hipStream_t s)
{
    const int K8 = p.K / 8;
    const float inv_K = 1.0f / float(p.K);
    const uint4_t* X = (const uint4_t*)p.X;
    const uint4_t* g = (const uint4_t*)p.g;
    if (K8 <= 256)       xhat_rows_kernel<T, 1><<<p.M, 256, 0, s>>>(X, g, Xh, rscale, K8, p.eps, inv_K);
    else if (K8 <= 512)  xhat_rows_kernel<T, 2><<<p.M, 256, 0, s>>>(X, g, Xh, rscale, K8, p.eps, inv_K);
    else if (K8 <= 1024) xhat_rows_kernel<T, 4><<<p.M, 256, 0, s>>>(X, g, Xh, rscale, K8, p.eps, inv_K);
    else if (K8 <= 2048) xhat_rows_kernel<T, 8><<<p.M, 256, 0, s>>>(X, g, Xh, rscale, K8, p.eps, inv_K);
    else                 xhat_rows_kernel<T, 0><<<p.M, 256, 0, s>>>(X, g, Xh, rscale, K8, p.eps, inv_K);
}

static size_t xhat_bytes(const Problem& p) { return (size_t(p.M) * p.K * 2 + 255) / 256 * 256; }

static size_t rscale_bytes(const Problem& p) { return (size_t(p.M) * 4 + 255) / 256 * 256; }

// slabs of the product (1 = no split): forced by k_split = 1..16 when n_tile is 1 (a tuning
// override of this variant only), else from the tile count
static void tile_pre_split(const Problem& p, int* S, int* k_slab)
{
    const int64_t tiles = int64_t((p.M + 255) / 256) * ((p.N + 255) / 256);
    tile_split_plan(p.K, tiles, S, k_slab);
    if (p.n_tile == 1 && p.k_split >= 1 && p.k_split <= 16) {
        if (p.k_split == 1) { *S = 1; *k_slab = p.K; return; }
        const int ks = ((p.K + p.k_split - 1) / p.k_split + BK - 1) / BK * BK;
        *S = (p.K + ks - 1) / ks;
        *k_slab = ks;
    }
    if (p.N % 8 != 0 || (p.gated && p.N % 16 != 0) || tile_big_w(p)) { *S = 1; *k_slab = p.K; }
}

size_t tile_pre_workspace_bytes(const Problem& p)
{
    int S, k_slab;
    tile_pre_split(p, &S, &k_slab);
    int full, rem, RS, rks;
    tile_rem_plan(p, &full, &rem, &RS, &rks);
    const size_t part = S > 1 ? size_t(S) * p.M * p.N * 4 : rem ? size_t(RS) * rem * 256 * 256 * 4 : 0;
    return (p.fused ? xhat_bytes(p) + rscale_bytes(p) : 0) + part;
}

hipError_t launch_tile_pre(const Problem& p, hipStream_t s, const char** why)
{
    if (p.gated && (p.N % 16 != 0 || !p.fused)) { if (why) *why = "gated block: tile variant needs H % 8 == 0"; return hipErrorInvalidValue; }
    if (p.dt == F32 || p.N % 8 != 0 || p.K % 8 != 0) {
        if (why) *why = "tile variants need a 16-bit type, N % 8 == 0 and K % 8 == 0";
        return hipErrorInvalidValue;
    }
    // check that the later kernels can run before the first is launched: all or none
    if (int64_t(256) * p.K * 2 >= (int64_t(1) << 31) || p.N >= (1 << 25)) {
        if (why) *why = "tile variant needs K < 2^22 and N < 2^25";
        return hipErrorInvalidValue;
    }
    int S, k_slab;
    tile_pre_split(p, &S, &k_slab);
    {
        int full, rem, RS, rks;
        tile_rem_plan(p, &full, &rem, &RS, &rks);
        if (rem && !p.ws_partial) { if (why) *why = "two-kernel tile variant needs the workspace"; return hipErrorInvalidValue; }
    }
    if ((p.fused || S > 1) && !p.ws_partial) { if (why) *why = "two-kernel tile variant needs the workspace"; return hipErrorInvalidValue; }
    Problem q = p;                           // the product, scaled per row if it is the fused block's
    float* part = p.ws_partial;
    if (p.fused) {
        uint4_t* Xh = reinterpret_cast<uint4_t*>(p.ws_partial);
        float* rscale = reinterpret_cast<float*>(reinterpret_cast<char*>(p.ws_partial) + xhat_bytes(p));
        part = reinterpret_cast<float*>(reinterpret_cast<char*>(rscale) + rscale_bytes(p));
        q.X = Xh; q.g = nullptr; q.fused = 0; q.rscale = rscale;
        if (p.dt == F16) xhat_rows_go<Fp16>(p, Xh, rscale, s);
        else             xhat_rows_go<Bf16>(p, Xh, rscale, s);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else {
        q.rscale = nullptr;                  // the plain product (matmul): no first kernel, only the split
    }
    if (S > 1) {
        if (p.plan) { p.plan[0] = 256; p.plan[1] = S; p.plan[2] = ((p.M + 255) / 256) * ((p.N + 255) / 256) * S; }
        q.plan = nullptr;
        return launch_tile_split(q, S, k_slab, part, s);
    }
    int full, rem, RS, rks;
    tile_rem_plan(p, &full, &rem, &RS, &rks);
    if (rem) return launch_tile_rem(q, full, rem, RS, rks, part, s, why);
    if (p.n_tile == 1 || p.n_tile == 2) { q.n_tile = 0; q.k_split = 0; }   // the override was for the splits only
    const char* w2 = nullptr;
    hipError_t e = launch_tile(q, s, &w2);
    if (e != hipSuccess && why && w2) *why = w2;
    return e;
}

}  // namespace rmsnl
