// Split-K GEMV variant of the fused RMSNorm + MatMul for decode shapes (M <= 16), without matrix
// cores.  The block is bound by streaming W once from HBM, so the design is about keeping many
// 16-byte loads in flight per lane and touching every W byte exactly once:
//
//   * a workgroup (4 waves) owns N_TILE = 8*LPR columns and one K slab; a wave-wide dwordx4 load
//     covers 64/LPR consecutive W rows of that column strip, i.e. 1 KiB of contiguous-per-row data;
//   * X-hat = X (.) g for the slab is formed once in fp32 and kept in LDS as [k][MT] (a lane reads the
//     MT values of its row with one broadcast read), while the same pass adds up the slab's share of
//     A_i = sum_k X_ik^2 -- the two accumulations of the paper's fused kernel share the K loop;
//   * B partials are reduced across the row groups of a wave by shuffles, across waves through LDS,
//     and across K slabs through an fp32 workspace: every slab writes its partial B and partial A,
//     the last workgroup to arrive at the tile's counter adds the S partials in slab order (so the
//     result does not depend on arrival order), scales by 1/sqrt(A/K + eps), rounds once and stores.
#include "common.hpp"

namespace rmsnl {

struct GemvArgs {
    const u16* X; const u16* g; const uint4_t* W; u16* Y;
    int M, K, N;
    float eps, inv_K;
    int k_slab;      // rows of W per slab (multiple of 8)
    int S;           // number of slabs
    int n_tiles;
    float* ws_partial; float* ws_sumsq; unsigned* counter;
};

constexpr int kGemvU = 8;            // 16-byte loads in flight per lane and buffer
constexpr int kSumsqStride = 16;     // floats per slab in ws_sumsq

template <typename T, int MT, int LPR, bool FUSED>
__global__ __launch_bounds__(256) void gemv_splitk_kernel(GemvArgs a)
{
    constexpr int N_TILE = LPR * 8;
    constexpr int RPI = 64 / LPR;            // W rows per wave-wide load
    constexpr int ROWS_IT = 4 * RPI;         // W rows per workgroup-wide load
    constexpr int U = kGemvU;
    extern __shared__ float smem[];          // max(xs, red): see gemv_lds_bytes()
    __shared__ float s_sumsq[4][MT];
    __shared__ float s_rinv[MT];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = lane / LPR, col8 = lane % LPR;

    // workgroups are dealt round-robin to the 8 XCDs; renumber so that the slabs of one tile share
    // an XCD (their partials and the counter then meet in one L2)
    int b = blockIdx.x;
    const int total = a.n_tiles * a.S;
    if ((total & 7) == 0) b = (b & 7) * (total >> 3) + (b >> 3);
    const int tile = b / a.S, slab = b % a.S;
    const int n0 = tile * N_TILE;
    const int k0 = slab * a.k_slab;
    const int klen = min(a.k_slab, a.K - k0);
    const int N8 = a.N >> 3;
    const bool colvalid = n0 + col8 * 8 < a.N;
    const uint4_t* Wp = a.W + size_t(k0) * N8 + (n0 >> 3) + col8;
    const int nIt = (klen + ROWS_IT - 1) / ROWS_IT;
    const int rbase = wave * RPI + grp;

    auto load_batch = [&](uint4_t (&w)[U], int it0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = (it0 + u) * ROWS_IT + rbase;
            w[u] = (colvalid && r < klen) ? __builtin_nontemporal_load(Wp + size_t(r) * N8)
                                          : uint4_t{0, 0, 0, 0};
        }
    };

    uint4_t wa[U], wb[U];
    load_batch(wa, 0);                      // first W loads go out before anything else

    // ---- X-hat for this slab into LDS as [k][MT] fp32, and this slab's share of A_i
    float* xs = smem;
    {
        float ss[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) ss[m] = 0.f;
        const int kpad = nIt * ROWS_IT;      // rows the main loop may index
        for (int kk = tid; kk < kpad; kk += 256) {
            const bool kin = kk < klen;
            float gk = 1.f;
            if (FUSED) gk = kin ? Elem<T>::to_f32(a.g[k0 + kk]) : 0.f;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float x = (kin && m < a.M) ? Elem<T>::to_f32(a.X[size_t(m) * a.K + k0 + kk]) : 0.f;
                if (FUSED) ss[m] = __fmaf_rn(x, x, ss[m]);
                xs[kk * MT + m] = FUSED ? x * gk : x;
            }
        }
        if (FUSED) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float v = wave_sum(ss[m]);
                if (lane == 0) s_sumsq[wave][m] = v;
            }
        }
    }
    __syncthreads();

    // ---- main loop: acc[m][8 columns] += xhat[m][k] * W[k][8 columns]
    float acc[MT][8];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[m][e] = 0.f;

    auto consume = [&](const uint4_t (&w)[U], int it0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = (it0 + u) * ROWS_IT + rbase;
            if ((it0 + u) < nIt) {           // uniform over the wave
                const float* xr = xs + r * MT;
                float wf[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wf[2 * e] = Elem<T>::lo(w[u][e]);
                    wf[2 * e + 1] = Elem<T>::hi(w[u][e]);
                }
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    const float xm = xr[m];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[m][e] = __fmaf_rn(xm, wf[e], acc[m][e]);
                }
            }
        }
    };

    for (int it0 = 0; it0 < nIt; it0 += 2 * U) {
        if (it0 + U < nIt) load_batch(wb, it0 + U);
        consume(wa, it0);
        if (it0 + 2 * U < nIt) load_batch(wa, it0 + 2 * U);
        if (it0 + U < nIt) consume(wb, it0 + U);
    }

    // ---- reduce over the row groups of the wave, then over the four waves through LDS
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[m][e] += __shfl_xor(acc[m][e], off, 64);

    __syncthreads();                         // everyone is done reading xs
    float* red = smem;                       // [4][MT][N_TILE]
    if (grp == 0) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            float4_t* dst = (float4_t*)(red + (wave * MT + m) * N_TILE + col8 * 8);
            dst[0] = float4_t{acc[m][0], acc[m][1], acc[m][2], acc[m][3]};
            dst[1] = float4_t{acc[m][4], acc[m][5], acc[m][6], acc[m][7]};
        }
    }
    __syncthreads();

    constexpr int PAIRS = MT * N_TILE / 2;   // column pairs of the tile, 256 threads share them
    const bool split = a.S > 1;
    float asum = 0.f;
    if (FUSED && tid < MT) asum = (s_sumsq[0][tid] + s_sumsq[1][tid]) + (s_sumsq[2][tid] + s_sumsq[3][tid]);

    if (!split) {
        if (tid < MT) s_rinv[tid] = FUSED ? row_scale(asum, a.inv_K, a.eps) : 1.f;
        __syncthreads();
        for (int p = tid; p < PAIRS; p += 256) {
            const int m = p / (N_TILE / 2), c = (p % (N_TILE / 2)) * 2;
            if (m < a.M && n0 + c < a.N) {
                const float2_t* r0 = (const float2_t*)(red + m * N_TILE + c);
                float2_t v = (r0[0] + r0[MT * N_TILE / 2]) + (r0[2 * MT * N_TILE / 2] + r0[3 * MT * N_TILE / 2]);
                const float ri = s_rinv[m];
                *(uint32_t*)(a.Y + size_t(m) * a.N + n0 + c) = Elem<T>::pack(v[0] * ri, v[1] * ri);
            }
        }
        return;
    }

    // ---- split-K: publish this slab's partial B and partial A
    if (FUSED && tid < MT) a.ws_sumsq[slab * kSumsqStride + tid] = asum;
    for (int p = tid; p < PAIRS; p += 256) {
        const int m = p / (N_TILE / 2), c = (p % (N_TILE / 2)) * 2;
        if (m < a.M && n0 + c < a.N) {
            const float2_t* r0 = (const float2_t*)(red + m * N_TILE + c);
            float2_t v = (r0[0] + r0[MT * N_TILE / 2]) + (r0[2 * MT * N_TILE / 2] + r0[3 * MT * N_TILE / 2]);
            *(float2_t*)(a.ws_partial + (size_t(slab) * a.M + m) * a.N + n0 + c) = v;
        }
    }
    __threadfence();                         // release: partials visible device-wide before the count
    __syncthreads();
    if (tid == 0) {
        unsigned prev = __hip_atomic_fetch_add(a.counter + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == unsigned(a.S - 1));
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();                         // acquire: see every slab's partials

    if (tid < MT) {
        float t = 0.f;
        if (FUSED) {
            for (int s = 0; s < a.S; ++s)
                t += __builtin_nontemporal_load(a.ws_sumsq + s * kSumsqStride + tid);
        }
        s_rinv[tid] = FUSED ? row_scale(t, a.inv_K, a.eps) : 1.f;
    }
    __syncthreads();
    for (int p = tid; p < PAIRS; p += 256) {
        const int m = p / (N_TILE / 2), c = (p % (N_TILE / 2)) * 2;
        if (m < a.M && n0 + c < a.N) {
            const float* src = a.ws_partial + size_t(m) * a.N + n0 + c;
            const size_t sstride = size_t(a.M) * a.N;
            float2_t v = {0.f, 0.f};
            int s = 0;
            for (; s + 4 <= a.S; s += 4) {   // four loads in flight, added in slab order
                float2_t p0 = __builtin_nontemporal_load((const float2_t*)(src + (s + 0) * sstride));
                float2_t p1 = __builtin_nontemporal_load((const float2_t*)(src + (s + 1) * sstride));
                float2_t p2 = __builtin_nontemporal_load((const float2_t*)(src + (s + 2) * sstride));
                float2_t p3 = __builtin_nontemporal_load((const float2_t*)(src + (s + 3) * sstride));
                v += p0; v += p1; v += p2; v += p3;
            }
            for (; s < a.S; ++s) v += __builtin_nontemporal_load((const float2_t*)(src + s * sstride));
            const float ri = s_rinv[m];
            *(uint32_t*)(a.Y + size_t(m) * a.N + n0 + c) = Elem<T>::pack(v[0] * ri, v[1] * ri);
        }
    }
    if (tid == 0) a.counter[tile] = 0;       // ready for the next call on this stream
}

// ------------------------------------------------------------------------------------------- host
struct GemvPlan { int MT, LPR, S, k_slab, n_tiles; size_t lds; bool ok; const char* why; };

static GemvPlan gemv_plan(const Problem& p)
{
    GemvPlan pl{};
    pl.ok = false;
    if (p.dt == F32) { pl.why = "gemv variant handles 16-bit types only"; return pl; }
    if (p.M > 16) { pl.why = "gemv variant needs M <= 16"; return pl; }
    if (p.N % 8 != 0) { pl.why = "gemv variant needs N % 8 == 0"; return pl; }
    pl.MT = p.M <= 1 ? 1 : p.M <= 2 ? 2 : p.M <= 4 ? 4 : p.M <= 8 ? 8 : 16;
    int n_tile = p.n_tile ? p.n_tile : 256;
    if (n_tile != 128 && n_tile != 256 && n_tile != 512) { pl.why = "gemv n_tile must be 128, 256 or 512"; return pl; }
    if (pl.MT * n_tile > 4096) n_tile = 4096 / pl.MT;          // cross-wave reduction buffer <= 64 KiB
    pl.LPR = n_tile / 8;
    pl.n_tiles = (p.N + n_tile - 1) / n_tile;
    const int rows_it = 4 * (64 / pl.LPR);
    // slab length: as requested, else aim at about 512 workgroups
    int S = p.k_split;
    if (S <= 0) {
        S = (512 + pl.n_tiles - 1) / pl.n_tiles;
        const int smax = (p.K + 63) / 64;                      // at least 64 rows per slab
        if (S > smax) S = smax;
        if (S < 1) S = 1;
    }
    int k_slab = (p.K + S - 1) / S;
    k_slab = (k_slab + rows_it - 1) / rows_it * rows_it;
    const int k_max = (64 * 1024) / (4 * pl.MT) / rows_it * rows_it;   // xs <= 64 KiB
    if (k_slab > k_max) k_slab = k_max;
    S = (p.K + k_slab - 1) / k_slab;
    pl.S = S;
    pl.k_slab = k_slab;
    if (pl.n_tiles > kMaxCounters) { pl.why = "too many column tiles"; return pl; }
    if (S * kSumsqStride > kMaxSumsqFloats) { pl.why = "too many K slabs"; return pl; }
    const size_t xs = size_t(k_slab + rows_it) * pl.MT * 4;
    const size_t red = size_t(4) * pl.MT * n_tile * 4;
    pl.lds = xs > red ? xs : red;
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
static hipError_t gemv_go(const GemvArgs& a, bool fused, const GemvPlan& pl, hipStream_t s)
{
    dim3 grid(pl.n_tiles * pl.S);
    static bool lds_raised = false;          // allow more than 64 KiB of dynamic LDS, once
    if (!lds_raised) {
        hipError_t e = hipFuncSetAttribute((const void*)gemv_splitk_kernel<T, MT, LPR, true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)gemv_splitk_kernel<T, MT, LPR, false>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e != hipSuccess) return e;
        lds_raised = true;
    }
    if (fused) gemv_splitk_kernel<T, MT, LPR, true><<<grid, 256, pl.lds, s>>>(a);
    else       gemv_splitk_kernel<T, MT, LPR, false><<<grid, 256, pl.lds, s>>>(a);
    return hipGetLastError();
}

template <typename T, int MT>
static hipError_t gemv_lpr(const GemvArgs& a, bool fused, const GemvPlan& pl, hipStream_t s)
{
    if constexpr (MT * 512 <= 4096) { if (pl.LPR == 64) return gemv_go<T, MT, 64>(a, fused, pl, s); }
    if constexpr (MT * 256 <= 4096) { if (pl.LPR == 32) return gemv_go<T, MT, 32>(a, fused, pl, s); }
    if (pl.LPR == 16) return gemv_go<T, MT, 16>(a, fused, pl, s);
    return hipErrorInvalidValue;
}

template <typename T>
static hipError_t gemv_mt(const GemvArgs& a, bool fused, const GemvPlan& pl, hipStream_t s)
{
    switch (pl.MT) {
    case 1:  return gemv_lpr<T, 1>(a, fused, pl, s);
    case 2:  return gemv_lpr<T, 2>(a, fused, pl, s);
    case 4:  return gemv_lpr<T, 4>(a, fused, pl, s);
    case 8:  return gemv_lpr<T, 8>(a, fused, pl, s);
    default: return gemv_lpr<T, 16>(a, fused, pl, s);
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
    GemvArgs a;
    a.X = (const u16*)p.X; a.g = (const u16*)p.g; a.W = (const uint4_t*)p.W; a.Y = (u16*)p.Y;
    a.M = p.M; a.K = p.K; a.N = p.N; a.eps = p.eps; a.inv_K = 1.0f / float(p.K);
    a.k_slab = pl.k_slab; a.S = pl.S; a.n_tiles = pl.n_tiles;
    a.ws_partial = p.ws_partial; a.ws_sumsq = p.ws_sumsq; a.counter = p.ws_counter;
    return p.dt == F16 ? gemv_mt<Fp16>(a, p.fused != 0, pl, s) : gemv_mt<Bf16>(a, p.fused != 0, pl, s);
}

}  // namespace rmsnl
