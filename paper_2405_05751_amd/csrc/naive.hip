// Reference-grade kernels of the library: the any-shape fp32-arithmetic fallback for the fused
// block, the stand-alone RMSNorm of the unfused A/B pair, and the measurement probes.
#include "../../include/rmsnl.h"
#include "common.hpp"
#include <type_traits>

namespace rmsnl {

// ---------------------------------------------------------------------------------------------
// Fallback: one workgroup = one row i and 64 consecutive columns; the K range is dealt to the four
// waves (k = wave, wave+4, ...), so every thread carries two running sums -- A_i and B_in, the two
// accumulators of the fused kernel -- and the four partials meet in LDS.  Works for every M, K, N
// (rows and column tiles share grid.x).  The 16-bit types accumulate in fp32 like the fast kernels;
// the fp32 type, which exists for its 1e-5 bar and is served by this kernel alone, accumulates in
// fp64, so that the bar holds for any K.
// ---------------------------------------------------------------------------------------------
template <typename T, bool FUSED, bool GATED>
__global__ __launch_bounds__(256) void naive_kernel(const typename Elem<T>::store_t* __restrict__ X,
                                                    const typename Elem<T>::store_t* __restrict__ g,
                                                    const typename Elem<T>::store_t* __restrict__ W,
                                                    typename Elem<T>::store_t* __restrict__ Y,
                                                    int M, int K, int N, float eps, float inv_K, int G)
{
    // GATED: N = 2H; output column n < H needs its gate and its up column of W (gated_col)
    typedef typename std::conditional<std::is_same<T, float>::value, double, float>::type acc_t;
    const int NO = GATED ? N / 2 : N;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int tiles_n = (NO + 63) / 64;
    const int i = blockIdx.x / tiles_n;
    const int n = (blockIdx.x % tiles_n) * 64 + lane;
    const bool live = n < NO;
    const size_t xrow = size_t(i) * K;

    acc_t B = 0, U = 0, A = 0;
    for (int k = wave; k < K; k += 4) {
        const acc_t x = Elem<T>::to_f32(X[xrow + k]);
        acc_t xg = x;
        if (FUSED) {
            A = fma(x, x, A);
            xg = x * acc_t(Elem<T>::to_f32(g[k]));
        }
        const acc_t w = live ? Elem<T>::to_f32(W[size_t(k) * N + (GATED ? gated_col(n, false, NO, G) : n)]) : 0.f;
        B = fma(xg, w, B);
        if (GATED) {
            const acc_t wu = live ? Elem<T>::to_f32(W[size_t(k) * N + gated_col(n, true, NO, G)]) : 0.f;
            U = fma(xg, wu, U);
        }
    }
    __shared__ acc_t sB[4][64];
    __shared__ acc_t sU[4][64];
    __shared__ acc_t sA[4];
    sB[wave][lane] = B;
    if (GATED) sU[wave][lane] = U;
    if (lane == 0) sA[wave] = A;
    __syncthreads();
    if (wave == 0 && live) {
        float b = float((sB[0][lane] + sB[1][lane]) + (sB[2][lane] + sB[3][lane]));
        float u = GATED ? float((sU[0][lane] + sU[1][lane]) + (sU[2][lane] + sU[3][lane])) : 0.f;
        if (FUSED) {
            const acc_t a = (sA[0] + sA[1]) + (sA[2] + sA[3]);
            if (std::is_same<T, float>::value) {
                // one rounding of the whole quotient instead of a rounded factor times a rounded sum
                const double ri = 1.0 / sqrt(double(a) * (1.0 / double(K)) + double(eps));
                b = float(double((sB[0][lane] + sB[1][lane]) + (sB[2][lane] + sB[3][lane])) * ri);
                u = GATED ? float(double((sU[0][lane] + sU[1][lane]) + (sU[2][lane] + sU[3][lane])) * ri) : 0.f;
            } else {
                const float ri = row_scale(float(a), inv_K, eps);
                b *= ri;
                u *= ri;
            }
        }
        if (GATED) b = silu(b) * u;
        Y[size_t(i) * NO + n] = Elem<T>::from_f32(b);
    }
}

template <typename T, bool GATED>
static hipError_t launch_naive_g(const Problem& p, hipStream_t s)
{
    typedef typename Elem<T>::store_t S;
    dim3 grid(unsigned(int64_t(((GATED ? p.N / 2 : p.N) + 63) / 64) * p.M));
    if (p.fused)
        naive_kernel<T, true, GATED><<<grid, 256, 0, s>>>((const S*)p.X, (const S*)p.g, (const S*)p.W, (S*)p.Y,
                                                          p.M, p.K, p.N, p.eps, 1.0f / float(p.K), p.gate_group);
    else
        naive_kernel<T, false, GATED><<<grid, 256, 0, s>>>((const S*)p.X, nullptr, (const S*)p.W, (S*)p.Y,
                                                           p.M, p.K, p.N, 0.f, 0.f, p.gate_group);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_naive_t(const Problem& p, hipStream_t s)
{
    return p.gated ? launch_naive_g<T, true>(p, s) : launch_naive_g<T, false>(p, s);
}

// Y[i][h] = SiLU(Z[i][h]) * Z[i][H + h]: the separate activation kernel of the unfused GatedMLP
template <typename T>
__global__ __launch_bounds__(256) void silu_mul_kernel(const typename Elem<T>::store_t* __restrict__ Z,
                                                       typename Elem<T>::store_t* __restrict__ Y, int H)
{
    const size_t i = blockIdx.y;
    const int h = blockIdx.x * 256 + threadIdx.x;
    if (h < H) {
        const float gt = Elem<T>::to_f32(Z[i * 2 * H + h]), up = Elem<T>::to_f32(Z[i * 2 * H + H + h]);
        Y[i * H + h] = Elem<T>::from_f32(silu(gt) * up);
    }
}

hipError_t launch_silu_mul(const void* Z, void* Y, int M, int H, DType dt, hipStream_t s)
{
    if (M > 65535) return hipErrorInvalidValue;
    dim3 grid((H + 255) / 256, M);
    switch (dt) {
    case F16:  silu_mul_kernel<Fp16><<<grid, 256, 0, s>>>((const u16*)Z, (u16*)Y, H); break;
    case BF16: silu_mul_kernel<Bf16><<<grid, 256, 0, s>>>((const u16*)Z, (u16*)Y, H); break;
    default:   silu_mul_kernel<float><<<grid, 256, 0, s>>>((const float*)Z, (float*)Y, H); break;
    }
    return hipGetLastError();
}

// W [K][2H] = [gate | up] -> Wi with groups of 64 gate columns alternating with the 64 up columns of the
// same outputs (gated_col with G = 64).  One thread per 16 bytes; H % 64 == 0.
__global__ __launch_bounds__(256) void interleave_gate_up_kernel(const uint4_t* __restrict__ W, uint4_t* __restrict__ Wi,
                                                                 int64_t chunks, int row_chunks, int per16, int H)
{
    const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= chunks) return;
    const int64_t k = idx / row_chunks;
    const int c = int(idx % row_chunks) * per16;         // first source column of the chunk
    const bool up = c >= H;
    const int dst = gated_col(up ? c - H : c, up, H, 64);
    Wi[k * row_chunks + dst / per16] = W[idx];
}

hipError_t launch_interleave_gate_up(const void* W, void* Wi, int64_t K, int H, DType dt, hipStream_t s)
{
    const int per16 = dt == F32 ? 4 : 8;                 // columns in 16 bytes
    const int row_chunks = 2 * H / per16;
    const int64_t chunks = K * row_chunks;
    if ((chunks + 255) / 256 >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    interleave_gate_up_kernel<<<dim3((unsigned)((chunks + 255) / 256)), 256, 0, s>>>((const uint4_t*)W, (uint4_t*)Wi, chunks,
                                                                                     row_chunks, per16, H);
    return hipGetLastError();
}

hipError_t launch_naive(const Problem& p, hipStream_t s, const char** why)
{
    if (int64_t(((p.gated ? p.N / 2 : p.N) + 63) / 64) * p.M >= (int64_t(1) << 31)) {
        if (why) *why = "naive variant supports ceil(N / 64) * M < 2^31 workgroups";
        return hipErrorInvalidValue;
    }
    switch (p.dt) {
    case F16:  return launch_naive_t<Fp16>(p, s);
    case BF16: return launch_naive_t<Bf16>(p, s);
    default:   return launch_naive_t<float>(p, s);
    }
}

// ---------------------------------------------------------------------------------------------
// Stand-alone RMSNorm (Eq. 1): one workgroup per row; first pass sums the squares, second pass
// re-reads the row (it is still in cache) and writes x * g * rinv rounded to the storage type.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const typename Elem<T>::store_t* __restrict__ X,
                                                      const typename Elem<T>::store_t* __restrict__ g,
                                                      typename Elem<T>::store_t* __restrict__ Xn,
                                                      int K, float eps, float inv_K)
{
    const size_t row = size_t(blockIdx.x) * K;
    float a = 0.f;
    for (int k = threadIdx.x; k < K; k += 256) {
        float x = Elem<T>::to_f32(X[row + k]);
        a = __fmaf_rn(x, x, a);
    }
    a = wave_sum(a);
    __shared__ float sA[4];
    if ((threadIdx.x & 63) == 0) sA[threadIdx.x >> 6] = a;
    __syncthreads();
    const float rinv = row_scale((sA[0] + sA[1]) + (sA[2] + sA[3]), inv_K, eps);
    for (int k = threadIdx.x; k < K; k += 256) {
        float x = Elem<T>::to_f32(X[row + k]);
        Xn[row + k] = Elem<T>::from_f32(x * Elem<T>::to_f32(g[k]) * rinv);
    }
}

// 16-bit rows with K % 8 == 0: 16-byte loads and stores, the row stays in registers when it fits
template <typename T, int PER_THREAD>
__global__ __launch_bounds__(256) void rmsnorm_vec_kernel(const uint4_t* __restrict__ X,
                                                          const uint4_t* __restrict__ g,
                                                          uint4_t* __restrict__ Xn,
                                                          int K8, float eps, float inv_K)
{
    const size_t row = size_t(blockIdx.x) * K8;
    uint4_t x[PER_THREAD];
    float a = 0.f;
#pragma unroll
    for (int j = 0; j < PER_THREAD; ++j) {
        int c = threadIdx.x + j * 256;
        x[j] = c < K8 ? X[row + c] : uint4_t{0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float lo = Elem<T>::lo(x[j][e]), hi = Elem<T>::hi(x[j][e]);
            a = __fmaf_rn(lo, lo, a);
            a = __fmaf_rn(hi, hi, a);
        }
    }
    a = wave_sum(a);
    __shared__ float sA[4];
    if ((threadIdx.x & 63) == 0) sA[threadIdx.x >> 6] = a;
    __syncthreads();
    const float rinv = row_scale((sA[0] + sA[1]) + (sA[2] + sA[3]), inv_K, eps);
#pragma unroll
    for (int j = 0; j < PER_THREAD; ++j) {
        int c = threadIdx.x + j * 256;
        if (c < K8) {
            uint4_t gg = g[c], o;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = Elem<T>::pack(Elem<T>::lo(x[j][e]) * Elem<T>::lo(gg[e]) * rinv,
                                     Elem<T>::hi(x[j][e]) * Elem<T>::hi(gg[e]) * rinv);
            Xn[row + c] = o;
        }
    }
}

template <typename T>
static hipError_t launch_rmsnorm_t(const void* X, const void* g, float eps, void* Xn, int M, int K,
                                   hipStream_t s)
{
    typedef typename Elem<T>::store_t S;
    const float inv_K = 1.0f / float(K);
    if constexpr (sizeof(S) == 2) {
        if (K % 8 == 0 && K <= 8 * 256 * 8) {
            const int K8 = K / 8;
            const int per = (K8 + 255) / 256;
            const uint4_t* x = (const uint4_t*)X;
            const uint4_t* gg = (const uint4_t*)g;
            uint4_t* o = (uint4_t*)Xn;
            if (per <= 1)      rmsnorm_vec_kernel<T, 1><<<M, 256, 0, s>>>(x, gg, o, K8, eps, inv_K);
            else if (per <= 2) rmsnorm_vec_kernel<T, 2><<<M, 256, 0, s>>>(x, gg, o, K8, eps, inv_K);
            else if (per <= 4) rmsnorm_vec_kernel<T, 4><<<M, 256, 0, s>>>(x, gg, o, K8, eps, inv_K);
            else               rmsnorm_vec_kernel<T, 8><<<M, 256, 0, s>>>(x, gg, o, K8, eps, inv_K);
            return hipGetLastError();
        }
    }
    rmsnorm_kernel<T><<<M, 256, 0, s>>>((const S*)X, (const S*)g, (S*)Xn, K, eps, inv_K);
    return hipGetLastError();
}

hipError_t launch_rmsnorm(const void* X, const void* g, float eps, void* Xn, int M, int K, DType dt,
                          hipStream_t s)
{
    switch (dt) {
    case F16:  return launch_rmsnorm_t<Fp16>(X, g, eps, Xn, M, K, s);
    case BF16: return launch_rmsnorm_t<Bf16>(X, g, eps, Xn, M, K, s);
    default:   return launch_rmsnorm_t<float>(X, g, eps, Xn, M, K, s);
    }
}

// ---------------------------------------------------------------------------------------------
// The block over Z_p (random tests over finite fields): one thread per output, modular arithmetic
// one operation at a time, in the order of the graph it stands for.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t ff_pow(uint32_t b, uint32_t e, uint32_t p)
{
    uint32_t r = 1;
    b %= p;
    while (e) {
        if (e & 1) r = r * b % p;
        b = b * b % p;
        e >>= 1;
    }
    return r;
}

// canonical root: the smallest y with y^2 = x, or, for a non-residue, with y^2 = x n (n the least non-residue)
__device__ uint32_t ff_sqrt(uint32_t x, uint32_t p)
{
    for (uint32_t y = 0; y < p; ++y)
        if (y * y % p == x) return y;
    uint32_t n = 2;
    while (ff_pow(n, (p - 1) / 2, p) == 1) ++n;      // Euler's criterion: first n that is no square
    const uint32_t t = x * n % p;
    for (uint32_t y = 0; y < p; ++y)
        if (y * y % p == t) return y;
    return 0;
}

__global__ __launch_bounds__(256) void ff_block_kernel(const uint32_t* __restrict__ X, const uint32_t* __restrict__ g,
                                                       const uint32_t* __restrict__ W, uint32_t* __restrict__ Y,
                                                       int M, int K, int N, uint32_t p, int reordered)
{
    const int n = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y;
    if (n >= N) return;
    const uint32_t* xi = X + size_t(i) * K;
    uint32_t a = 0;
    for (int k = 0; k < K; ++k) a = (a + xi[k] * xi[k]) % p;
    const uint32_t r = ff_sqrt(a * ff_pow(uint32_t(K) % p, p - 2, p) % p, p);
    uint32_t y = 0;
    if (r != 0) {
        const uint32_t rinv = ff_pow(r, p - 2, p);
        uint32_t acc = 0;
        for (int k = 0; k < K; ++k) {
            uint32_t t = xi[k] * g[k] % p;
            if (!reordered) t = t * rinv % p;            // Eq. 1 first: normalise, then multiply by W
            acc = (acc + t * W[size_t(k) * N + n]) % p;
        }
        y = reordered ? acc * rinv % p : acc;            // rewritten graph: divide after the product
    }
    Y[size_t(i) * N + n] = y;
}

hipError_t launch_ff_block(const void* X, const void* g, const void* W, void* Y, int M, int K, int N,
                           uint32_t p, int reordered, hipStream_t s)
{
    dim3 grid((N + 255) / 256, M);
    ff_block_kernel<<<grid, 256, 0, s>>>((const uint32_t*)X, (const uint32_t*)g, (const uint32_t*)W, (uint32_t*)Y,
                                         M, K, N, p, reordered);
    return hipGetLastError();
}

// The block and the gated block on pairs over Z_227 x Z_113 (Table 3 in full, with the Exp row), in the
// graph form the paper starts from: Eq. 1 first (every X-hat divided by the root), then the product,
// then the activation as a step of its own.  One thread per output; elements are x_p | x_q << 8.
__global__ __launch_bounds__(256) void ff_pairs_ref_kernel(const u16* __restrict__ X, const u16* __restrict__ g,
                                                           const u16* __restrict__ W, u16* __restrict__ Y,
                                                           int M, int K, int N, uint32_t omega, int gated)
{
    typedef Arith<Ff> Ar;
    const int NO = gated ? N / 2 : N;
    const int n = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y;
    if (n >= NO) return;
    const u16* xi = X + size_t(i) * K;
    float a = Ar::make(0, 0);
    for (int k = 0; k < K; ++k) { const float x = Elem<Ff>::widen(xi[k]); a = Ar::fma(x, x, a); }
    const float inv_k = Ar::make(ff_pow_mod(uint32_t(K) % kFfP, kFfP - 2, kFfP), ff_pow_mod(uint32_t(K) % kFfQ, kFfQ - 2, kFfQ));
    const float ri = Ar::rinv(a, inv_k, 0.f);
    float z = Ar::make(0, 0), u = Ar::make(0, 0);
    for (int k = 0; k < K; ++k) {
        const float t = Ar::mul(Ar::mul(Elem<Ff>::widen(xi[k]), Elem<Ff>::widen(g[k])), ri);   // Eq. 1
        z = Ar::fma(t, Elem<Ff>::widen(W[size_t(k) * N + n]), z);
        if (gated) u = Ar::fma(t, Elem<Ff>::widen(W[size_t(k) * N + NO + n]), u);
    }
    const float one = Ar::make(1, 1);
    const float y = gated ? Ar::out_gated(z, u, one, __uint_as_float(omega)) : z;
    Y[size_t(i) * NO + n] = u16(Elem<Ff>::narrow(y));
}

hipError_t launch_ff_pairs_ref(const void* X, const void* g, const void* W, void* Y, int M, int K, int N,
                               uint32_t omega, int gated, hipStream_t s)
{
    dim3 grid(((gated ? N / 2 : N) + 255) / 256, M);
    ff_pairs_ref_kernel<<<grid, 256, 0, s>>>((const u16*)X, (const u16*)g, (const u16*)W, (u16*)Y, M, K, N, omega, gated);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Probes
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void probe_copy_kernel(uint4_t* __restrict__ dst,
                                                         const uint4_t* __restrict__ src, size_t n16)
{
    size_t i = size_t(blockIdx.x) * 256 * 8 + threadIdx.x;
    uint4_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (i + j * 256 < n16) ? src[i + j * 256] : uint4_t{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (i + j * 256 < n16) dst[i + j * 256] = v[j];
}

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4_t* __restrict__ src, size_t n16,
                                                         uint32_t* __restrict__ sink)
{
    size_t i = size_t(blockIdx.x) * 256 * 16 + threadIdx.x;
    uint4_t v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = (i + j * 256 < n16) ? src[i + j * 256] : uint4_t{0, 0, 0, 0};
    uint32_t acc = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc ^= v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
    if (acc == 0x9e3779b9u) sink[0] = acc;       // practically never taken; keeps the loads alive
}

hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t s)
{
    size_t n16 = bytes / 16;
    unsigned blocks = unsigned((n16 + 2047) / 2048);
    probe_copy_kernel<<<blocks, 256, 0, s>>>((uint4_t*)dst, (const uint4_t*)src, n16);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t s)
{
    size_t n16 = bytes / 16;
    unsigned blocks = unsigned((n16 + 4095) / 4096);
    probe_read_kernel<<<blocks, 256, 0, s>>>((const uint4_t*)src, n16, (uint32_t*)sink);
    return hipGetLastError();
}

// Streaming-read probes with the launch shapes of the small-M kernels, for a measured ceiling beside
// their figures.  Strips: the matrix [rows][row_bytes] is cut into strips of 256 bytes (128 16-bit
// columns, what a workgroup of the GEMV and skinny kernels owns) and `parts` row ranges; workgroup
// (strip, part) reads its rows with the kernels' own access shape (a wave-wide 16-byte load covers
// 4 rows of 256 bytes), two batches of 8 loads per wave in flight, streaming cache policy, through a
// range-checked buffer resource.  Flat: workgroup b of G reads the b-th contiguous share of the
// buffer, 1 KiB per wave-wide load.
__global__ __launch_bounds__(256) void probe_strips_kernel(const char* __restrict__ src, int rows, int row_bytes,
                                                           int strips, int parts, uint32_t* __restrict__ sink,
                                                           unsigned long long* trace, int trace_groups)
{
    trace_stamp(trace, trace_groups, 0);                 // start (stage trace, if one is registered)
    int b = blockIdx.x;
    const int total = strips * parts;
    if ((total & 7) == 0) b = (b & 7) * (total >> 3) + (b >> 3);       // the parts of a strip share an XCD
    const int strip = b / parts, part = b % parts;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int prow = (rows + parts - 1) / parts;                        // rows per part
    const int r0 = part * prow;
    const int here = min(prow, rows - r0);
    if (here <= 0) return;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(src) + size_t(r0) * row_bytes, 0, here * row_bytes, 0x00020000);
    const int voff = strip * 256 + (lane & 15) * 16 + (lane >> 4) * row_bytes;
    const int nchunks = (here + 127) / 128;                             // chunks of 32 rows per wave; rows past `here` read zero
    uint4_t r[2][8];
    uint4_t acc = {0, 0, 0, 0};
    auto issue = [&](int c, int d) {
        const int base = voff + ((c * 4 + wave) * 32) * row_bytes;
#pragma unroll
        for (int j = 0; j < 8; ++j) r[d][j] = __builtin_amdgcn_raw_buffer_load_b128(rs, base + j * 4 * row_bytes, 0, 2);
    };
    issue(0, 0);
    if (nchunks > 1) issue(1, 1);
    for (int c0 = 0; c0 < nchunks; c0 += 2) {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            if (c0 + d < nchunks) {
#pragma unroll
                for (int j = 0; j < 8; ++j) acc ^= r[d][j];
                if (c0 + d + 2 < nchunks) issue(c0 + d + 2, d);
            }
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;   // practically never taken; keeps the loads alive
    __syncthreads();
    trace_stamp(trace, trace_groups, 2);                 // all of the workgroup's rows have arrived
}

__global__ __launch_bounds__(256) void probe_flat_kernel(const uint4_t* __restrict__ src, size_t n16, size_t share16,
                                                         uint32_t* __restrict__ sink)
{
    const size_t lo = size_t(blockIdx.x) * share16;
    const size_t hi = min(n16, lo + share16);
    uint4_t acc = {0, 0, 0, 0};
    // a wave takes alternate runs of 8 KiB (8 loads of 1 KiB), two runs in flight
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4_t r[2][8];
    auto issue = [&](size_t run, int d) {
        const size_t base = lo + (run * 4 + wave) * 512 + lane;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            r[d][j] = base + j * 64 < hi ? __builtin_nontemporal_load(src + base + j * 64) : uint4_t{0, 0, 0, 0};
    };
    const size_t nruns = (hi > lo ? hi - lo + 2047 : 0) / 2048;
    if (nruns == 0) return;
    issue(0, 0);
    if (nruns > 1) issue(1, 1);
    for (size_t c0 = 0; c0 < nruns; c0 += 2) {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            if (c0 + d < nruns) {
#pragma unroll
                for (int j = 0; j < 8; ++j) acc ^= r[d][j];
                if (c0 + d + 2 < nruns) issue(c0 + d + 2, d);
            }
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;
}

hipError_t launch_probe_strips(const void* src, int rows, int row_bytes, int parts, void* sink,
                               unsigned long long* trace, int trace_groups, hipStream_t s)
{
    probe_strips_kernel<<<(row_bytes / 256) * parts, 256, 0, s>>>((const char*)src, rows, row_bytes, row_bytes / 256, parts,
                                                                  (uint32_t*)sink, trace, trace_groups);
    return hipGetLastError();
}

hipError_t launch_probe_flat(const void* src, size_t bytes, int workgroups, void* sink, hipStream_t s)
{
    const size_t n16 = bytes / 16;
    const size_t share16 = ((n16 + workgroups - 1) / workgroups + 2047) / 2048 * 2048;   // whole 32 KiB rounds per workgroup
    probe_flat_kernel<<<workgroups, 256, 0, s>>>((const uint4_t*)src, n16, share16, (uint32_t*)sink);
    return hipGetLastError();
}

// register-only MFMA loop: 4 independent 32x32x16 accumulators per wave, 4 waves per workgroup,
// 4 workgroups per CU's worth of grid; flops = grid * 4 waves * iters * 4 * 32*32*16*2
constexpr int kProbeBlocks = 1024;
template <typename V>
__device__ __forceinline__ float16_t mfma32(V a, V b, float16_t c);
template <> __device__ __forceinline__ float16_t mfma32<bf16x8_t>(bf16x8_t a, bf16x8_t b, float16_t c)
{ return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
template <> __device__ __forceinline__ float16_t mfma32<f16x8_t>(f16x8_t a, f16x8_t b, float16_t c)
{ return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }

template <typename V>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ sink, int iters, int zero)
{
    // operands: pseudo-random values in (-2, 2), different per lane, element and accumulator, so the
    // datapath toggles like it does on real activations (constant operands draw less power and clock higher)
    typedef __attribute__((ext_vector_type(8))) float float8_t;
    V a[4], b[4];
    for (int j = 0; j < 4; ++j) {
        float8_t af, bf;
        for (int e = 0; e < 8; ++e) {
            uint32_t h = (threadIdx.x * 8u + e) * 2654435761u + j * 0x9e3779b9u + blockIdx.x * 40503u;
            h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
            af[e] = zero ? 0.f : float(int(h & 0xffff) - 32768) * (1.0f / 16384.0f);
            bf[e] = zero ? 0.f : float(int(h >> 16) - 32768) * (1.0f / 16384.0f);
        }
        a[j] = __builtin_convertvector(af, V);
        b[j] = __builtin_convertvector(bf, V);
    }
    float16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
        c0 = mfma32<V>(a[0], b[0], c0);
        c1 = mfma32<V>(a[1], b[1], c1);
        c2 = mfma32<V>(a[2], b[2], c2);
        c3 = mfma32<V>(a[3], b[3], c3);
    }
    float r = 0.f;
    for (int e = 0; e < 16; ++e) r += c0[e] + c1[e] + c2[e] + c3[e];
    sink[size_t(blockIdx.x) * 256 + threadIdx.x] = r;
}

hipError_t launch_probe_mfma(void* sink, int iters, DType dt, int zero, hipStream_t s)
{
    if (dt == F16) probe_mfma_kernel<f16x8_t><<<kProbeBlocks, 256, 0, s>>>((float*)sink, iters, zero);
    else           probe_mfma_kernel<bf16x8_t><<<kProbeBlocks, 256, 0, s>>>((float*)sink, iters, zero);
    return hipGetLastError();
}

}  // namespace rmsnl

extern "C" size_t rl_probe_mfma_sink_floats(void) { return size_t(rmsnl::kProbeBlocks) * 256; }
extern "C" double rl_probe_mfma_flops(int iters)
{
    return double(rmsnl::kProbeBlocks) * 4.0 * double(iters) * 4.0 * (32.0 * 32.0 * 16.0 * 2.0);
}
