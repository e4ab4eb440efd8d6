// Shared declarations of the rmsnl HIP sources (gfx950 only).
//
// Notation follows the paper's case study: X [M][K] activations, g [K] gain, W [K][N]
// weight, A_i = sum_k X_ik^2, B_in = sum_k X_ik g_k W_kn, Y_in = B_in / sqrt(A_i/K + eps).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <initializer_list>

namespace rmsnl {

enum DType : int { F16 = 0, BF16 = 1, F32 = 2 };

// One call, as the launchers see it.  Pointers are device pointers.
struct Problem {
    const void* X;        // [M][K]; for the plain matmul this is the left operand
    const void* g;        // [K]; unused when fused == 0
    const void* W;        // [K][N]
    void* Y;              // [M][N]
    int M, K, N;
    float eps;
    int fused;            // 1: RMSNorm prologue + row scaling, 0: plain product
    int gated;            // 1: W is [K][N] = [gate | up] with N = 2H, Y is [M][H] = SiLU(Z_gate) * Z_up
    int gate_group;       // gated: 0 = W's halves are gate and up; 64 = groups of 64 gate columns alternate with
                          // the 64 up columns of the same outputs (H % 64 == 0)
    const float* rscale;  // plain product only: Y rows scaled by rscale[i] in the epilogue, or null
    int tile_limit;       // tile kernel only: run the first tile_limit tiles of its order (0 = all)
    DType dt;
    // split-K workspace (may be null when the chosen launch needs none)
    float* ws_partial;    // [S][M][N] partial B
    float* ws_sumsq;      // [tiles][S][Mpad] partial A
    unsigned* ws_counter; // one arrival counter per N tile, zero between calls
    // launch-shape overrides, 0 = automatic
    int n_tile;
    int k_split;
    // where a launcher reports the launch shape it used (columns per workgroup or tile shape, K slabs or
    // waves, workgroups of the main kernel), or null
    int* plan;
    // optional stage trace: kTraceSlots 64-bit time stamps per workgroup, or null
    unsigned long long* trace;
    int trace_groups;     // workgroups the trace buffer has room for
};

constexpr int kTraceSlots = 16;

// Launchers: return hipSuccess/err of the launch; `why` (optional) gets a static string when
// the variant cannot run the shape (then nothing was launched and the return is hipErrorInvalidValue).
hipError_t launch_naive(const Problem& p, hipStream_t s, const char** why);
hipError_t launch_rmsnorm(const void* X, const void* g, float eps, void* Xn, int M, int K, DType dt,
                          hipStream_t s);
hipError_t launch_gemv(const Problem& p, hipStream_t s, const char** why);
hipError_t launch_skinny(const Problem& p, hipStream_t s, const char** why);
hipError_t launch_tile(const Problem& p, hipStream_t s, const char** why);
hipError_t launch_f32(const Problem& p, hipStream_t s, const char** why);
// two kernels: X-hat and 1/rms per row into the workspace (at ws_partial), then the tile kernel as a
// plain product of X-hat scaled per row
hipError_t launch_tile_pre(const Problem& p, hipStream_t s, const char** why);
size_t tile_pre_workspace_bytes(const Problem& p);
// tile of the workgroup at position b of the tile kernels' order over tiles_m x tiles_n tiles (host)
void tile_order_at(int b, int tiles_m, int tiles_n, int* tm, int* tn);
// bytes of partial-B workspace the launch of this problem would use (0 = no split)
size_t gemv_workspace_bytes(const Problem& p);
size_t skinny_workspace_bytes(const Problem& p);
size_t f32_workspace_bytes(const Problem& p);

// Kernels that use more than 64 KiB of dynamic LDS have the limit raised once per device (the
// attribute belongs to the device's copy of the kernel); one LdsOnce per group of kernels.
struct LdsOnce { std::atomic<unsigned> devices{0}; };
inline hipError_t raise_lds_once(LdsOnce& once, std::initializer_list<const void*> kernels, int bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned bit = 1u << (dev & 31);
    if (once.devices.load(std::memory_order_acquire) & bit) return hipSuccess;
    for (const void* k : kernels) {
        e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
    }
    once.devices.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
}

// QKNorm in front of attention, one query per (sample, head); ws: qkattn_workspace_bytes() of device memory;
// splits > 0 forces the number of sequence splits (tuning), 0 = automatic
hipError_t launch_qkattn(const void* Q, const void* K, const void* V, const void* gq, const void* bq,
                         const void* gk, const void* bk, float eps, void* O,
                         int64_t B, int64_t H, int64_t S, int64_t D, DType dt, float* ws, unsigned* counters,
                         int splits, hipStream_t s);
size_t qkattn_workspace_bytes(int64_t B, int64_t H, int64_t S, int64_t D, DType dt);
// sequence splits the fast kernel would launch for `splits` (0 = automatic); 0 where the plain kernel runs
int qkattn_splits(int64_t B, int64_t H, int64_t S, int64_t D, DType dt, int splits);
hipError_t launch_silu_mul(const void* Z, void* Y, int M, int H, DType dt, hipStream_t s);
hipError_t launch_interleave_gate_up(const void* W, void* Wi, int64_t K, int H, DType dt, hipStream_t s);

hipError_t launch_ntrans(const void* X, const void* Hh, const void* A, float eps, void* Y, int M, int D, DType dt,
                         hipStream_t s);
hipError_t launch_ff_block(const void* X, const void* g, const void* W, void* Y, int M, int K, int N,
                           uint32_t p, int reordered, hipStream_t s);

// the GEMV split-K kernel on pairs over Z_227 x Z_113 (X, g, W, Y: 16-bit elements x_p | x_q << 8)
hipError_t launch_gemv_ff(const Problem& p, uint32_t omega, hipStream_t s, const char** why);
// reference evaluation of the same graphs on pairs, one thread per output, Eq. 1 first
hipError_t launch_ff_pairs_ref(const void* X, const void* g, const void* W, void* Y, int M, int K, int N,
                               uint32_t omega, int gated, hipStream_t s);

hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t s);
hipError_t launch_probe_mfma(void* sink, int iters, DType dt, int zero, hipStream_t s);
hipError_t launch_probe_strips(const void* src, int rows, int row_bytes, int parts, void* sink,
                               unsigned long long* trace, int trace_groups, hipStream_t s);
hipError_t launch_probe_flat(const void* src, size_t bytes, int workgroups, void* sink, hipStream_t s);

// workspace head: arrival counters, then the per-slab partial sums of squares; partial B follows
// Counters sit one per 128-byte line so that the tiles' atomics spread over memory channels.
constexpr size_t kCounterBytes = 256 * 1024;
constexpr size_t kSumsqBytes = 1024 * 1024;
constexpr size_t kHeadBytes = kCounterBytes + kSumsqBytes;
constexpr int kCounterStride = 32;                         // unsigneds between two counters
constexpr int kMaxCounters = int(kCounterBytes / sizeof(unsigned)) / kCounterStride;
constexpr int kMaxSumsqFloats = int(kSumsqBytes / sizeof(float));

// ------------------------------------------------------------------ device helpers
#if defined(__HIPCC__)

typedef uint16_t u16;
typedef __attribute__((ext_vector_type(2))) float float2_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(16))) float float16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t uint4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t uint2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;

struct Bf16 {};   // tag types for the 16-bit storage formats
struct Fp16 {};

template <typename T> struct Elem;

template <> struct Elem<Bf16> {
    typedef u16 store_t;
    static __device__ __forceinline__ float to_f32(u16 b) { return __uint_as_float(uint32_t(b) << 16); }
    // low / high half of a packed pair
    static __device__ __forceinline__ float lo(uint32_t p) { return __uint_as_float(p << 16); }
    static __device__ __forceinline__ float hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
    static __device__ __forceinline__ u16 from_f32(float f) {
        __bf16 h = (__bf16)f;                        // v_cvt_pk_bf16_f32, nearest-even
        return __builtin_bit_cast(u16, h);
    }
    static __device__ __forceinline__ uint32_t pack(float a, float b) {
        float2_t v = {a, b};
        bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
        return __builtin_bit_cast(uint32_t, h);
    }
};

template <> struct Elem<Fp16> {
    typedef u16 store_t;
    static __device__ __forceinline__ float to_f32(u16 b) { return (float)__builtin_bit_cast(_Float16, b); }
    static __device__ __forceinline__ float lo(uint32_t p) { return to_f32(u16(p & 0xffffu)); }
    static __device__ __forceinline__ float hi(uint32_t p) { return to_f32(u16(p >> 16)); }
    static __device__ __forceinline__ u16 from_f32(float f) {
        _Float16 h = (_Float16)f;                    // v_cvt_f16_f32, nearest-even
        return __builtin_bit_cast(u16, h);
    }
    static __device__ __forceinline__ uint32_t pack(float a, float b) {
        return uint32_t(from_f32(a)) | (uint32_t(from_f32(b)) << 16);
    }
};

template <> struct Elem<float> {
    typedef float store_t;
    static __device__ __forceinline__ float to_f32(float f) { return f; }
    static __device__ __forceinline__ float from_f32(float f) { return f; }
};

// ---- the paper's random tests over finite fields (Table 3), as an element type of the kernels.
// A value is a pair (x_p, x_q) from Z_p x Z_q with the primes the paper's implementation uses,
// p = 227 and q = 113 (q divides p - 1; the pair fits 16 bits).  Stored as x_p | x_q << 8 in the
// 16 bits a bf16 element takes, so a kernel instantiated on this type moves exactly the bytes it
// moves for bf16; in registers a pair rides in the 32 bits of a float as x_p | x_q << 16 (never
// touched by floating-point arithmetic: moves, shuffles and LDS keep bits as they are).
struct Ff {};
constexpr uint32_t kFfP = 227, kFfQ = 113;

template <> struct Elem<Ff> {
    typedef u16 store_t;
    static __device__ __forceinline__ float widen(uint32_t e) { return __uint_as_float((e & 0xffu) | ((e >> 8 & 0xffu) << 16)); }
    static __device__ __forceinline__ float lo(uint32_t p) { return widen(p & 0xffffu); }
    static __device__ __forceinline__ float hi(uint32_t p) { return widen(p >> 16); }
    static __device__ __forceinline__ uint32_t narrow(float f) {
        const uint32_t u = __float_as_uint(f);
        return (u & 0xffu) | ((u >> 16 & 0xffu) << 8);
    }
    static __device__ __forceinline__ uint32_t pack(float a, float b) { return narrow(a) | (narrow(b) << 16); }
};

__device__ __forceinline__ uint32_t ff_pow_mod(uint32_t b, uint32_t e, uint32_t m) {
    uint32_t r = 1;
    b %= m;
    while (e) { if (e & 1) r = r * b % m; b = b * b % m; e >>= 1; }
    return r;
}
// canonical root: the smallest y with y^2 = x; for a non-residue x, the smallest y with y^2 = x n, n the least non-residue
__device__ __forceinline__ uint32_t ff_root_mod(uint32_t x, uint32_t m) {
    for (int pass = 0; pass < 2; ++pass) {
        for (uint32_t y = 0; y < m; ++y)
            if (y * y % m == x) return y;
        uint32_t n = 2;
        for (;; ++n) { bool res = false; for (uint32_t y = 1; y < m && !res; ++y) res = y * y % m == n; if (!res) break; }
        x = x * n % m;
    }
    return 0;
}

// The arithmetic of a kernel instantiation: fp32 for the 16-bit floating types, pairs for Ff.
// rinv: the row factor from the sum of squares (inv_K and eps as the kernels carry them: for Ff,
// inv_K holds the pair (1/K mod p, 1/K mod q) and eps holds omega, the sampled q-th root of unity,
// both as bits).  out: one output from its accumulated product(s) and the row factor.
template <typename T> struct Arith {
    static __device__ __forceinline__ float add(float a, float b) { return a + b; }
    static __device__ __forceinline__ float mul(float a, float b) { return a * b; }
    static __device__ __forceinline__ float fma(float a, float b, float c) { return __fmaf_rn(a, b, c); }
    static __device__ __forceinline__ float4_t add4(float4_t a, float4_t b) { return a + b; }
    static __device__ __forceinline__ float rinv(float sumsq, float inv_K, float eps) {
        return 1.0f / __fsqrt_rn(__fmaf_rn(sumsq, inv_K, eps));
    }
    static __device__ __forceinline__ float out(float v, float ri, float) { return v * ri; }
    static __device__ __forceinline__ float out_gated(float v, float u, float ri, float) {
        const float gt = v * ri;
        return gt / (1.0f + __expf(-gt)) * (u * ri);
    }
    static __device__ __forceinline__ float one() { return 1.f; }
};

template <> struct Arith<Ff> {
    static __device__ __forceinline__ uint32_t P(float f) { return __float_as_uint(f) & 0xffffu; }
    static __device__ __forceinline__ uint32_t Q(float f) { return __float_as_uint(f) >> 16; }
    static __device__ __forceinline__ float make(uint32_t xp, uint32_t xq) { return __uint_as_float(xp | (xq << 16)); }
    static __device__ __forceinline__ float add(float a, float b) { return make((P(a) + P(b)) % kFfP, (Q(a) + Q(b)) % kFfQ); }
    static __device__ __forceinline__ float mul(float a, float b) { return make(P(a) * P(b) % kFfP, Q(a) * Q(b) % kFfQ); }
    static __device__ __forceinline__ float fma(float a, float b, float c) {
        return make((P(a) * P(b) + P(c)) % kFfP, (Q(a) * Q(b) + Q(c)) % kFfQ);
    }
    static __device__ __forceinline__ float4_t add4(float4_t a, float4_t b) {
        return float4_t{add(a[0], b[0]), add(a[1], b[1]), add(a[2], b[2]), add(a[3], b[3])};
    }
    // 1 / sqrt(A / K) in each field (Div and Sqrt rows); a mean square of 0 has no inverse root: factor 0
    static __device__ __forceinline__ float rinv(float sumsq, float inv_K, float) {
        const uint32_t rp = ff_root_mod(P(sumsq) * P(inv_K) % kFfP, kFfP), rq = ff_root_mod(Q(sumsq) * Q(inv_K) % kFfQ, kFfQ);
        return make(rp ? ff_pow_mod(rp, kFfP - 2, kFfP) : 0, rq ? ff_pow_mod(rq, kFfQ - 2, kFfQ) : 0);
    }
    static __device__ __forceinline__ float out(float v, float ri, float) { return mul(v, ri); }
    // SiLU(G) * U = G / (1 + exp(-G)) * U: the exponential takes the q component (Exp row), the rest is Z_p
    static __device__ __forceinline__ float out_gated(float v, float u, float ri, float omega) {
        const float gt = mul(v, ri), up = mul(u, ri);
        const uint32_t e = ff_pow_mod(__float_as_uint(omega), (kFfQ - Q(gt)) % kFfQ, kFfP);
        const uint32_t den = (1 + e) % kFfP;
        return make(den ? P(gt) * ff_pow_mod(den, kFfP - 2, kFfP) % kFfP * P(up) % kFfP : 0, 0);
    }
    static __device__ __forceinline__ float one() { return make(1, 1); }
};

// rinv = 1 / sqrt(A / K + eps), correctly rounded division and root (not the fast approximations)
__device__ __forceinline__ float row_scale(float sumsq, float inv_K, float eps) {
    return 1.0f / __fsqrt_rn(__fmaf_rn(sumsq, inv_K, eps));
}

// Gated block: the W column that feeds the gate (up = false) or the up (up = true) input of output h.
// G = 0: W = [gate | up], two halves of H columns.  G = 64: columns 128 j .. 128 j + 63 are the gate
// columns of outputs 64 j .. 64 j + 63 and the next 64 their up columns (8 consecutive outputs from a
// multiple of 8 stay 8 consecutive columns either way).
__device__ __forceinline__ int gated_col(int h, bool up, int H, int G) {
    return G ? ((h >> 6) << 7) + (h & 63) + (up ? 64 : 0) : h + (up ? H : 0);
}

// SiLU(v) = v / (1 + exp(-v)) in fp32 (the activation of the paper's GatedMLP block)
__device__ __forceinline__ float silu(float v) { return v / (1.0f + __expf(-v)); }

// sum over the 64 lanes of a wave, result in every lane
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Device-scope (all XCDs) relaxed stores and loads: written through to / read from memory that
// every XCD's L2 agrees on.  Used for the split-K partials, which cross XCDs.
__device__ __forceinline__ void st_dev(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev2(float* p, float2_t v) {
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), __builtin_bit_cast(uint64_t, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2_t ld_dev2(const float* p) {
    uint64_t u = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(float2_t, u);
}

// Stage trace: thread 0 of a workgroup stores the constant-rate (100 MHz) clock into its slot.
__device__ __forceinline__ void trace_stamp(unsigned long long* trace, int groups, int slot) {
    if (trace && threadIdx.x == 0 && int(blockIdx.x) < groups)
        trace[size_t(blockIdx.x) * kTraceSlots + slot] = wall_clock64();
}

#endif  // __HIPCC__

}  // namespace rmsnl
