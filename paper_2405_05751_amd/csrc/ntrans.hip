// Normalised-Transformer chain (the paper's nTrans benchmark) in one kernel:
//     y = Norm(x + alpha (.) Norm(h - x)),   Norm(v) = v / sqrt(mean(v^2) + eps)   per row
// x, h, y [M][D], alpha [D].  Three kernels in existing systems (two norms around an elementwise
// step); here a row is read once, lives in registers, and is written once.  The paper's kernel
// keeps the intermediates in shared memory and notes that staging light kernels through it can
// dominate their run time; nothing here goes through LDS except the two row sums.
//
// One workgroup per row: thread t holds 16-byte chunks t, t + 256, ... of the row (whole 128-byte
// lines per 8 lanes), so the row is streamed with fully coalesced loads; fp32 arithmetic, one
// rounding to the storage type.  Rows that do not fit the registers, fp32 storage and D % 8 != 0
// take the scalar three-pass kernel.
#include "common.hpp"

namespace rmsnl {

__device__ __forceinline__ float block_sum(float v, float* scratch /* [4] */)
{
    v = wave_sum(v);
    __syncthreads();                                    // scratch may still be read from the last use
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    return (scratch[0] + scratch[1]) + (scratch[2] + scratch[3]);
}

template <typename T, int PER>
__global__ __launch_bounds__(256) void ntrans_vec_kernel(const uint4_t* __restrict__ X, const uint4_t* __restrict__ Hh,
                                                         const uint4_t* __restrict__ A, uint4_t* __restrict__ Y,
                                                         int D8, float eps, float inv_D)
{
    __shared__ float scratch[4];
    const size_t row = size_t(blockIdx.x) * D8;
    float x[PER][8], d[PER][8];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int c = threadIdx.x + j * 256;
        // streamed once: non-temporal loads and stores (6 % faster than the default policy at 16384 x 2048)
        const uint4_t xv = c < D8 ? __builtin_nontemporal_load(&X[row + c]) : uint4_t{0, 0, 0, 0};
        const uint4_t hv = c < D8 ? __builtin_nontemporal_load(&Hh[row + c]) : uint4_t{0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[j][2 * e] = Elem<T>::lo(xv[e]); x[j][2 * e + 1] = Elem<T>::hi(xv[e]);
            d[j][2 * e] = Elem<T>::lo(hv[e]) - x[j][2 * e];
            d[j][2 * e + 1] = Elem<T>::hi(hv[e]) - x[j][2 * e + 1];
            s = __fmaf_rn(d[j][2 * e], d[j][2 * e], s);
            s = __fmaf_rn(d[j][2 * e + 1], d[j][2 * e + 1], s);
        }
    }
    const float r1 = row_scale(block_sum(s, scratch), inv_D, eps);       // 1 / sqrt(mean (h-x)^2 + eps)
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int c = threadIdx.x + j * 256;
        const uint4_t av = c < D8 ? A[c] : uint4_t{0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[j][2 * e] = __fmaf_rn(Elem<T>::lo(av[e]), d[j][2 * e] * r1, x[j][2 * e]);          // u = x + alpha * Norm(h - x)
            x[j][2 * e + 1] = __fmaf_rn(Elem<T>::hi(av[e]), d[j][2 * e + 1] * r1, x[j][2 * e + 1]);
            t = __fmaf_rn(x[j][2 * e], x[j][2 * e], t);
            t = __fmaf_rn(x[j][2 * e + 1], x[j][2 * e + 1], t);
        }
    }
    const float r2 = row_scale(block_sum(t, scratch), inv_D, eps);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int c = threadIdx.x + j * 256;
        if (c < D8) {
            uint4_t o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = Elem<T>::pack(x[j][2 * e] * r2, x[j][2 * e + 1] * r2);
            __builtin_nontemporal_store(o, &Y[row + c]);
        }
    }
}

// any D, any type: three passes over the row (it stays in cache)
template <typename T>
__global__ __launch_bounds__(256) void ntrans_kernel(const typename Elem<T>::store_t* __restrict__ X,
                                                     const typename Elem<T>::store_t* __restrict__ Hh,
                                                     const typename Elem<T>::store_t* __restrict__ A,
                                                     typename Elem<T>::store_t* __restrict__ Y,
                                                     int D, float eps, float inv_D)
{
    __shared__ float scratch[4];
    const size_t row = size_t(blockIdx.x) * D;
    float s = 0.f;
    for (int j = threadIdx.x; j < D; j += 256) {
        const float dd = Elem<T>::to_f32(Hh[row + j]) - Elem<T>::to_f32(X[row + j]);
        s = __fmaf_rn(dd, dd, s);
    }
    const float r1 = row_scale(block_sum(s, scratch), inv_D, eps);
    float t = 0.f;
    for (int j = threadIdx.x; j < D; j += 256) {
        const float xx = Elem<T>::to_f32(X[row + j]);
        const float u = __fmaf_rn(Elem<T>::to_f32(A[j]), (Elem<T>::to_f32(Hh[row + j]) - xx) * r1, xx);
        t = __fmaf_rn(u, u, t);
    }
    const float r2 = row_scale(block_sum(t, scratch), inv_D, eps);
    for (int j = threadIdx.x; j < D; j += 256) {
        const float xx = Elem<T>::to_f32(X[row + j]);
        const float u = __fmaf_rn(Elem<T>::to_f32(A[j]), (Elem<T>::to_f32(Hh[row + j]) - xx) * r1, xx);
        Y[row + j] = Elem<T>::from_f32(u * r2);
    }
}

template <typename T>
static hipError_t launch_ntrans_t(const void* X, const void* Hh, const void* A, float eps, void* Y, int M, int D,
                                  hipStream_t s)
{
    typedef typename Elem<T>::store_t S;
    const float inv_D = 1.0f / float(D);
    if constexpr (sizeof(S) == 2) {
        if (D % 8 == 0 && D <= 8 * 256 * 4) {
            const int D8 = D / 8, per = (D8 + 255) / 256;
            const uint4_t* x = (const uint4_t*)X; const uint4_t* h = (const uint4_t*)Hh; const uint4_t* a = (const uint4_t*)A;
            uint4_t* y = (uint4_t*)Y;
            if (per <= 1)      ntrans_vec_kernel<T, 1><<<M, 256, 0, s>>>(x, h, a, y, D8, eps, inv_D);
            else if (per <= 2) ntrans_vec_kernel<T, 2><<<M, 256, 0, s>>>(x, h, a, y, D8, eps, inv_D);
            else               ntrans_vec_kernel<T, 4><<<M, 256, 0, s>>>(x, h, a, y, D8, eps, inv_D);
            return hipGetLastError();
        }
    }
    ntrans_kernel<T><<<M, 256, 0, s>>>((const S*)X, (const S*)Hh, (const S*)A, (S*)Y, D, eps, inv_D);
    return hipGetLastError();
}

hipError_t launch_ntrans(const void* X, const void* Hh, const void* A, float eps, void* Y, int M, int D, DType dt,
                         hipStream_t s)
{
    switch (dt) {
    case F16:  return launch_ntrans_t<Fp16>(X, Hh, A, eps, Y, M, D, s);
    case BF16: return launch_ntrans_t<Bf16>(X, Hh, A, eps, Y, M, D, s);
    default:   return launch_ntrans_t<float>(X, Hh, A, eps, Y, M, D, s);
    }
}

}  // namespace rmsnl
