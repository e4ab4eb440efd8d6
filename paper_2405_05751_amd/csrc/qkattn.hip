// QKNorm in front of attention, decode form (the paper's QKNorm benchmark: layer normalisation of
// the query and key vectors before attention, fused with the attention itself so that the normalised
// keys never exist in memory): one query per (sample, head) against a key-value cache of S positions.
//
//   qn = LayerNorm(q; gq, bq),  kn_t = LayerNorm(k_t; gk, bk),  s_t = qn . kn_t / sqrt(D),
//   p = softmax_t(s),  o = sum_t p_t v_t.
//
// The same move as in the RMSNorm block: the key's normalisation is taken out of the dot product,
//   qn . kn_t = (sum_d qn_d gk_d (k_td - mu_t)) / sigma_t + qn . bk,
// so a key is read once, raw, and its mean, variance and dot product with qn (.) gk come out of the
// same registers.  The kernel is bound by streaming K and V once.
//
// Fast path (D = 64, 128 or 256, 16-bit types): D / 8 lanes share a key (8 elements each; a wave-wide
// load is 8, 4 or 2 consecutive keys, 1 KiB contiguous), the three sums over D are exchanges inside
// that lane group (DPP and, for D = 256, a swap of 16-lane rows: no LDS), every group keeps its own running
// maximum, denominator and 8 output sums (online softmax), and the groups, the waves and
// the splits of the sequence (by the last of them to arrive, through the workspace) are merged at
// the end.  Any other D or type: a slow plain kernel.
#include <algorithm>
#include "common.hpp"

namespace rmsnl {

constexpr int kQkOut = 0x7ffffff0;
constexpr int kQkFlags = 0x00020000;
constexpr int kQkRing = 6;           // iterations (one K and one V load per lane each) in flight
constexpr float kLog2e = 1.4426950408889634f;

struct QkArgs {
    const u16* Q; const u16* K; const u16* V;
    const u16* gq; const u16* bq; const u16* gk; const u16* bk;
    u16* O;
    float* part;                     // [B*H][SP][D + 2] when SP > 1
    unsigned* counter;               // one arrival counter per (sample, head), zero between calls; or null:
                                     // then a second kernel merges the splits
    float eps, scale_log2e;          // scores are kept in units of log2: s * log2(e) / sqrt(D)
    int S, SP, chunk;                // positions, splits, positions per split (a multiple of 32)
};

// sum over a group of LPK = 8, 16 or 32 consecutive lanes (aligned to LPK), in every lane of the group
template <int LPK>
__device__ __forceinline__ float group_sum(float v)
{
#define RL_DPP(ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), (ctrl), 0xf, 0xf, false))
    if constexpr (LPK == 8) {
        v += RL_DPP(0xB1);                   // lanes 1 0 3 2 of each four
        v += RL_DPP(0x4E);                   // lanes 2 3 0 1 of each four: the four now agree
        v += RL_DPP(0x141);                  // lane 7 - i of each eight: the other four's sum
    } else {
        v += RL_DPP(0x128);                  // rotations inside a row of 16 lanes
        v += RL_DPP(0x124);
        v += RL_DPP(0x122);
        v += RL_DPP(0x121);
        if constexpr (LPK == 32) {
            // v_permlane16_swap exchanges rows 1 and 3 (of 16 lanes) of its first operand with rows 0 and 2 of
            // its second: with v in both they become (row 0, row 0, row 2, row 2) and (row 1, row 1, row 3,
            // row 3), whose sum is the sum over each pair of rows.  Written out, waits included, because the
            // compiler's builtin adds the first result to itself.
            float t;
            asm volatile("v_mov_b32 %1, %0\n\ts_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1\n\tv_add_f32 %0, %0, %1"
                         : "+v"(v), "=&v"(t));
        }
    }
#undef RL_DPP
    return v;
}

template <typename T>
__device__ __forceinline__ void unpack8(uint4_t p, float* x)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[2 * e] = Elem<T>::lo(p[e]); x[2 * e + 1] = Elem<T>::hi(p[e]); }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void qkattn_kernel(QkArgs a)
{
    constexpr int R = kQkRing;
    constexpr int LPK = D / 8;               // lanes that share a key
    constexpr int KPW = 64 / LPK;            // keys in a wave-wide load
    constexpr int PPI = 4 * KPW;             // positions the workgroup takes per iteration (4 KiB of K and of V)
    __shared__ float s_m[4], s_l[4];
    __shared__ float s_acc[4][D];
    __shared__ int s_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kq = lane / LPK, c = lane % LPK;
    const int bh = blockIdx.x / a.SP, sp = blockIdx.x % a.SP;
    const int t0 = sp * a.chunk, t1 = min(a.S, t0 + a.chunk);

    // ---- the query: LayerNorm, then folded with the keys' gain and bias
    float qg[8], qb;
    {
        float q[8], g[8], b[8], gk8[8], bk8[8];
        unpack8<T>(*(const uint4_t*)(a.Q + size_t(bh) * D + 8 * c), q);
        unpack8<T>(*(const uint4_t*)(a.gq + 8 * c), g);
        unpack8<T>(*(const uint4_t*)(a.bq + 8 * c), b);
        unpack8<T>(*(const uint4_t*)(a.gk + 8 * c), gk8);
        unpack8<T>(*(const uint4_t*)(a.bk + 8 * c), bk8);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += q[e];
        const float mu = group_sum<LPK>(s) * (1.0f / D);
        float v = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { q[e] -= mu; v = __fmaf_rn(q[e], q[e], v); }
        const float rinv = 1.0f / __fsqrt_rn(group_sum<LPK>(v) * (1.0f / D) + a.eps);
        float t = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float qn = __fmaf_rn(q[e] * rinv, g[e], b[e]);
            qg[e] = qn * gk8[e];
            t = __fmaf_rn(qn, bk8[e], t);
        }
        qb = group_sum<LPK>(t);
    }

    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(a.K + size_t(bh) * a.S * D), 0, a.S * D * 2, kQkFlags);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16*>(a.V + size_t(bh) * a.S * D), 0, a.S * D * 2, kQkFlags);
    // iteration i of this wave: position t0 + PPI i + KPW wave + kq (the workgroup reads 4 KiB of K
    // and of V, contiguous, per iteration); a position outside the split is not fetched
    const int nIter = (t1 - t0 + PPI - 1) / PPI;   // uniform
    const int tl = t0 + KPW * wave + kq;
    const int off0 = (tl * D + 8 * c) * 2;

    uint4_t kx[R], vx[R];
    // Every load is issued whether or not its iteration exists (one past the split reads zeros
    // through the range check, at no memory traffic) and the issues are pinned in program order, so that the compiler
    // can count the loads younger than the one it waits for.
    auto issue = [&](int i, int r) {
        const int t = tl + PPI * i;
        const int off = t < t1 ? off0 + i * (PPI * D * 2) : kQkOut;
        __builtin_amdgcn_sched_barrier(0);
        kx[r] = __builtin_amdgcn_raw_buffer_load_b128(krs, off, 0, 2);
        vx[r] = __builtin_amdgcn_raw_buffer_load_b128(vrs, off, 0, 2);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
#pragma unroll
    for (int r = 0; r < R; ++r) issue(r, r);

    float m = -1.0e30f, l = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    auto consume = [&](int i, int r) {
        float x[8], v[8];
        unpack8<T>(kx[r], x);
        float s1 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s1 += x[e];
        const float mu = group_sum<LPK>(s1) * (1.0f / D);
        float s2 = 0.f, dot = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            x[e] -= mu;
            s2 = __fmaf_rn(x[e], x[e], s2);
            dot = __fmaf_rn(qg[e], x[e], dot);
        }
        s2 = group_sum<LPK>(s2);
        dot = group_sum<LPK>(dot);
        const float rinv = 1.0f / __fsqrt_rn(s2 * (1.0f / D) + a.eps);
        const float s = __fmaf_rn(dot, rinv, qb) * a.scale_log2e;
        const bool valid = tl + PPI * i < t1;
        const float m_new = valid ? fmaxf(m, s) : m;
        const float corr = __builtin_amdgcn_exp2f(m - m_new);
        const float p = valid ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
        m = m_new;
        l = __fmaf_rn(l, corr, p);
        unpack8<T>(vx[r], v);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = __fmaf_rn(acc[e], corr, p * v[e]);
    };

    for (int i0 = 0; i0 < nIter; i0 += R) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (i0 + r < nIter) consume(i0 + r, r);      // uniform; only the arithmetic is skipped
            issue(i0 + r + R, r);
        }
    }

    // ---- merge the key groups of the wave (lanes l, l ^ LPK, l ^ 2 LPK, ...)
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
        const float m_o = __shfl_xor(m, off, 64), l_o = __shfl_xor(l, off, 64);
        const float m_n = fmaxf(m, m_o);
        const float w_s = __builtin_amdgcn_exp2f(m - m_n), w_o = __builtin_amdgcn_exp2f(m_o - m_n);
        l = l * w_s + l_o * w_o;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * w_s + __shfl_xor(acc[e], off, 64) * w_o;
        m = m_n;
    }
    if (kq == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s_acc[wave][8 * c + e] = acc[e];
        if (c == 0) { s_m[wave] = m; s_l[wave] = l; }
    }
    __syncthreads();
    // ---- merge the four waves; thread j < D owns output dimension j
    if (tid < D) {
        const float mm = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
        float o = 0.f, ll = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float ws = __builtin_amdgcn_exp2f(s_m[w] - mm);
            o = __fmaf_rn(s_acc[w][tid], ws, o);
            ll = __fmaf_rn(s_l[w], ws, ll);
        }
        if (a.SP == 1) {
            a.O[size_t(bh) * D + tid] = Elem<T>::from_f32(o / ll);
        } else {                             // written through: another workgroup will read them
            float* dst = a.part + (size_t(bh) * a.SP + sp) * (D + 2);
            st_dev(dst + tid, o);
            if (tid == 0) { st_dev(dst + D, mm); st_dev(dst + D + 1, ll); }
        }
    }
    if (a.SP == 1 || !a.counter) return;     // uniform

    // ---- the last split of this (sample, head) to arrive merges them all
    __builtin_amdgcn_s_waitcnt(0);           // this wave's stores have been acknowledged
    __syncthreads();
    if (tid == 0) {
        const unsigned prev = __hip_atomic_fetch_add(a.counter + bh * kCounterStride, 1u, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == unsigned(a.SP - 1));
    }
    __syncthreads();
    if (!s_last) return;
    if (tid < D) {
        const float* src = a.part + size_t(bh) * a.SP * (D + 2);
        float mm = -1.0e30f, o = 0.f, ll = 0.f;
        for (int s0 = 0; s0 < a.SP; s0 += 16) {      // 16 splits per round trip, all loads before any use
            float pm[16], pl[16], po[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float* e = src + size_t(min(s0 + j, a.SP - 1)) * (D + 2);
                pm[j] = ld_dev(e + D); pl[j] = ld_dev(e + D + 1); po[j] = ld_dev(e + tid);
            }
            float bm = mm;
#pragma unroll
            for (int j = 0; j < 16; ++j) if (s0 + j < a.SP) bm = fmaxf(bm, pm[j]);
            const float w0 = __builtin_amdgcn_exp2f(mm - bm);
            o *= w0; ll *= w0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float ws = s0 + j < a.SP ? __builtin_amdgcn_exp2f(pm[j] - bm) : 0.f;
                o = __fmaf_rn(po[j], ws, o);
                ll = __fmaf_rn(pl[j], ws, ll);
            }
            mm = bm;
        }
        a.O[size_t(bh) * D + tid] = Elem<T>::from_f32(o / ll);
    }
    if (tid == 0)                            // ready for the next call on this stream
        __hip_atomic_store(a.counter + bh * kCounterStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// splits of one (sample, head) -> O; thread j owns output dimension j
template <typename T, int D>
__global__ __launch_bounds__(D) void qkattn_combine_kernel(const float* __restrict__ part, u16* __restrict__ O, int SP)
{
    const float* src = part + size_t(blockIdx.x) * SP * (D + 2);
    float mm = -1.0e30f;
    for (int s = 0; s < SP; ++s) mm = fmaxf(mm, src[s * (D + 2) + D]);
    float o = 0.f, ll = 0.f;
    for (int s = 0; s < SP; ++s) {
        const float ws = __builtin_amdgcn_exp2f(src[s * (D + 2) + D] - mm);
        o = __fmaf_rn(src[s * (D + 2) + threadIdx.x], ws, o);
        ll = __fmaf_rn(src[s * (D + 2) + D + 1], ws, ll);
    }
    O[size_t(blockIdx.x) * D + threadIdx.x] = Elem<T>::from_f32(o / ll);
}

// ---------------------------------------------------------------------------------- any D, any type
// One workgroup per (sample, head), fp32 arithmetic, the definition step by step: scores into the
// workspace, their maximum, the exponentials and their sum, then one thread per output dimension.
template <typename T>
__global__ __launch_bounds__(256) void qkattn_plain_kernel(const typename Elem<T>::store_t* __restrict__ Q,
    const typename Elem<T>::store_t* __restrict__ K, const typename Elem<T>::store_t* __restrict__ V,
    const typename Elem<T>::store_t* __restrict__ gq, const typename Elem<T>::store_t* __restrict__ bq,
    const typename Elem<T>::store_t* __restrict__ gk, const typename Elem<T>::store_t* __restrict__ bk,
    typename Elem<T>::store_t* __restrict__ O, float* __restrict__ scores, float eps, int S, int D)
{
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const size_t bh = blockIdx.x;
    auto ld = [](const typename Elem<T>::store_t* p, size_t i) { return Elem<T>::to_f32(p[i]); };
    auto block_reduce = [&](float v, bool is_max) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float o = __shfl_xor(v, off, 64);
            v = is_max ? fmaxf(v, o) : v + o;
        }
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = v;
        __syncthreads();
        return is_max ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) : (red[0] + red[1]) + (red[2] + red[3]);
    };
    // statistics of the query (every thread computes them: D is small)
    const typename Elem<T>::store_t* q = Q + bh * D;
    float qmu = 0.f;
    for (int j = 0; j < D; ++j) qmu += ld(q, j);
    qmu /= float(D);
    float qvar = 0.f;
    for (int j = 0; j < D; ++j) { const float d = ld(q, j) - qmu; qvar = __fmaf_rn(d, d, qvar); }
    const float qr = 1.0f / __fsqrt_rn(qvar / float(D) + eps);
    const float scale = 1.0f / __fsqrt_rn(float(D));
    float top = -INFINITY;
    for (int t = tid; t < S; t += 256) {
        const typename Elem<T>::store_t* k = K + (bh * S + t) * D;
        float mu = 0.f;
        for (int j = 0; j < D; ++j) mu += ld(k, j);
        mu /= float(D);
        float var = 0.f;
        for (int j = 0; j < D; ++j) { const float d = ld(k, j) - mu; var = __fmaf_rn(d, d, var); }
        const float r = 1.0f / __fsqrt_rn(var / float(D) + eps);
        float dot = 0.f;
        for (int j = 0; j < D; ++j) {
            const float qn = __fmaf_rn((ld(q, j) - qmu) * qr, ld(gq, j), ld(bq, j));
            const float kn = __fmaf_rn((ld(k, j) - mu) * r, ld(gk, j), ld(bk, j));
            dot = __fmaf_rn(qn, kn, dot);
        }
        const float s = dot * scale;
        scores[bh * S + t] = s;
        top = fmaxf(top, s);
    }
    top = block_reduce(top, true);
    float sum = 0.f;
    for (int t = tid; t < S; t += 256) {
        const float p = expf(scores[bh * S + t] - top);
        scores[bh * S + t] = p;
        sum += p;
    }
    sum = block_reduce(sum, false);      // (its barriers also order the scores written above)
    for (int j = tid; j < D; j += 256) {
        float o = 0.f;
        for (int t = 0; t < S; ++t) o = __fmaf_rn(scores[bh * S + t], ld(V, (bh * S + t) * D + j), o);
        O[bh * D + j] = Elem<T>::from_f32(o / sum);
    }
}

// ------------------------------------------------------------------------------------------- host
static void qk_plan(int64_t BH, int S, int force, int* SP, int* chunk)
{
    // one workgroup per compute unit, at least 256 positions each: more splits measured slower
    // (32 heads x 4096 positions: 8 splits 19.2 us, 16 splits 23.9 us, 32 splits 30.2 us);
    // force > 0: that many splits, at least 64 positions each
    int64_t sp = std::max<int64_t>(1, (256 + BH - 1) / BH);
    sp = std::min<int64_t>(sp, std::max(1, S / 256));
    if (force > 0) sp = std::min<int64_t>(force, std::max(1, S / 64));
    sp = std::min<int64_t>(sp, 64);
    int ch = int(((S + sp - 1) / sp + 31) / 32 * 32);
    *chunk = ch;
    *SP = (S + ch - 1) / ch;
}

// the fast kernel: 16-bit types, D of 64, 128 or 256, and a (sample, head)'s keys short of the byte
// offset that stands for "not fetched"
static bool qk_fast(int64_t S, int64_t D, DType dt)
{
    return dt != F32 && (D == 64 || D == 128 || D == 256) && S * D * 2 < kQkOut;
}

int qkattn_splits(int64_t B, int64_t H, int64_t S, int64_t D, DType dt, int splits)
{
    if (!qk_fast(S, D, dt)) return 0;
    int SP, chunk;
    qk_plan(B * H, int(S), splits, &SP, &chunk);
    return SP;
}

size_t qkattn_workspace_bytes(int64_t B, int64_t H, int64_t S, int64_t D, DType dt)
{
    if (!qk_fast(S, D, dt)) return size_t(B) * H * S * 4;           // the plain kernel's scores
    return size_t(B) * H * 64 * (D + 2) * 4;                         // room for the most splits there can be
}

template <typename T>
static hipError_t qk_plain_go(const void* Q, const void* K, const void* V, const void* gq, const void* bq,
                              const void* gk, const void* bk, void* O, float* ws, float eps,
                              int64_t BH, int S, int D, hipStream_t s)
{
    typedef typename Elem<T>::store_t E;
    qkattn_plain_kernel<T><<<dim3((unsigned)BH), 256, 0, s>>>((const E*)Q, (const E*)K, (const E*)V, (const E*)gq,
                                                               (const E*)bq, (const E*)gk, (const E*)bk, (E*)O, ws, eps, S, D);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t qk_fast_go(const QkArgs& a, int64_t BH, hipStream_t s)
{
    qkattn_kernel<T, D><<<dim3((unsigned)(BH * a.SP)), 256, 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.SP == 1 || a.counter) return e;
    qkattn_combine_kernel<T, D><<<dim3((unsigned)BH), D, 0, s>>>(a.part, a.O, a.SP);
    return hipGetLastError();
}

hipError_t launch_qkattn(const void* Q, const void* K, const void* V, const void* gq, const void* bq,
                         const void* gk, const void* bk, float eps, void* O,
                         int64_t B, int64_t H, int64_t S, int64_t D, DType dt, float* ws, unsigned* counters,
                         int splits, hipStream_t s)
{
    const int64_t BH = B * H;
    if (!qk_fast(S, D, dt)) {
        if (dt == F32) return qk_plain_go<float>(Q, K, V, gq, bq, gk, bk, O, ws, eps, BH, int(S), int(D), s);
        if (dt == F16) return qk_plain_go<Fp16>(Q, K, V, gq, bq, gk, bk, O, ws, eps, BH, int(S), int(D), s);
        return qk_plain_go<Bf16>(Q, K, V, gq, bq, gk, bk, O, ws, eps, BH, int(S), int(D), s);
    }
    QkArgs a;
    a.Q = (const u16*)Q; a.K = (const u16*)K; a.V = (const u16*)V;
    a.gq = (const u16*)gq; a.bq = (const u16*)bq; a.gk = (const u16*)gk; a.bk = (const u16*)bk;
    a.O = (u16*)O; a.part = ws; a.eps = eps;
    a.scale_log2e = kLog2e / sqrtf(float(D));
    a.S = int(S);
    qk_plan(BH, int(S), splits, &a.SP, &a.chunk);
    a.counter = (BH <= kMaxCounters) ? counters : nullptr;
    if (dt == F16) return D == 64 ? qk_fast_go<Fp16, 64>(a, BH, s) : D == 128 ? qk_fast_go<Fp16, 128>(a, BH, s) : qk_fast_go<Fp16, 256>(a, BH, s);
    return D == 64 ? qk_fast_go<Bf16, 64>(a, BH, s) : D == 128 ? qk_fast_go<Bf16, 128>(a, BH, s) : qk_fast_go<Bf16, 256>(a, BH, s);
}

}  // namespace rmsnl
