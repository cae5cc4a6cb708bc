// Shared device-side types and small helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

namespace amdp {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int WAVE = 64;

// Host side: raises the dynamic-LDS limit of kernel Kern to `bytes` on the
// current device, once per device (a kernel attribute belongs to the device's
// copy of the code object). Threads that race here both set the same value.
template <auto Kern>
inline hipError_t allow_dynamic_lds(int bytes) {
    static std::atomic<uint64_t> done{0};          // one bit per device ordinal
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute((const void*)Kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

template <class T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v) { return (T)v; }   // bf16: RNE

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

// Exact (erf) GELU and its derivative, fp32.
__device__ __forceinline__ float gelu_f(float u) {
    return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f));
}
__device__ __forceinline__ float gelu_grad_f(float u) {
    const float cdf = 0.5f * (1.0f + erff(u * 0.70710678118654752f));
    const float pdf = 0.39894228040143268f * __expf(-0.5f * u * u);
    return cdf + u * pdf;
}

// Epilogue applied to every GEMM output element, in this order:
//   v = alpha*acc (+ bias[n]) (* gelu'(gelu_u[m,n])) (+ res[m,n]);  C[m,n] = v
//   (aux_out[m,n] = gelu(v) when aux_out is set)
struct Epilogue {
    const void* bias = nullptr;     // stage dtype [N]
    const void* res = nullptr;      // stage dtype [M, ldr]
    const void* gelu_u = nullptr;   // stage dtype [M, ldu]
    void* aux_out = nullptr;        // stage dtype [M, ldc]
    long ldr = 0, ldu = 0;
    float alpha = 1.0f;
    int out_f32 = 0;                // C is float instead of the stage dtype
    int accumulate = 0;             // with out_f32: C[m,n] += v instead of C[m,n] = v
};

template <class T>
__device__ __forceinline__ void epilogue_store(const Epilogue& e, void* C, long ldc, long m, long n,
                                               float acc) {
    float v = acc * e.alpha;
    if (e.bias) v += to_f32(((const T*)e.bias)[n]);
    if (e.gelu_u) v *= gelu_grad_f(to_f32(((const T*)e.gelu_u)[m * e.ldu + n]));
    if (e.res) v += to_f32(((const T*)e.res)[m * e.ldr + n]);
    if (e.out_f32) {
        float* p = (float*)C + m * ldc + n;
        *p = e.accumulate ? *p + v : v;
    }
    else ((T*)C)[m * ldc + n] = from_f32<T>(v);
    if (e.aux_out) ((T*)e.aux_out)[m * ldc + n] = from_f32<T>(gelu_f(v));
}

// Cheaper GELU terms for the bf16 epilogues, where they are a visible share of
// a launch (the d/du GELU epilogue of configuration 2's FFN1 backward carried 12
// other vector instructions per matrix instruction with erff): erf from the
// five-term rational-exponential form of Abramowitz & Stegun 7.1.26 (absolute
// error below 1.5e-7, a bf16 result keeps 8 bits), sharing its exp(-u^2/2) with
// the density. cdf = Phi(u), pdf = phi(u).
__device__ __forceinline__ void gelu_terms_fast(float u, float& cdf, float& pdf) {
    const float x = fabsf(u) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    const float e = __builtin_amdgcn_exp2f(-0.72134752044448170f * u * u);    // exp(-u*u/2)
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float erf_abs = fmaf(-p * t, e, 1.0f);                             // erf(|u|/sqrt 2)
    cdf = fmaf(0.5f, copysignf(erf_abs, u), 0.5f);
    pdf = 0.39894228040143268f * e;
}
__device__ __forceinline__ float gelu_fast(float u) {
    float cdf, pdf;
    gelu_terms_fast(u, cdf, pdf);
    return u * cdf;
}
__device__ __forceinline__ float gelu_grad_fast(float u) {
    float cdf, pdf;
    gelu_terms_fast(u, cdf, pdf);
    return fmaf(u, pdf, cdf);
}

// Same epilogue for 8 consecutive columns n..n+7 of row m (bf16 stage dtype);
// every pointer involved is 16-byte aligned at these columns.
__device__ __forceinline__ void epilogue_store8(const Epilogue& e, void* C, long ldc, long m, long n,
                                                float (&v)[8]) {
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] *= e.alpha;
    if (e.bias) {
        const bf16x8 b = *(const bf16x8*)((const bf16*)e.bias + n);
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] += (float)b[k];
    }
    if (e.gelu_u) {
        const bf16x8 u = *(const bf16x8*)((const bf16*)e.gelu_u + m * e.ldu + n);
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] *= gelu_grad_fast((float)u[k]);
    }
    if (e.res) {
        const bf16x8 r = *(const bf16x8*)((const bf16*)e.res + m * e.ldr + n);
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] += (float)r[k];
    }
    if (e.out_f32) {
        float* p = (float*)C + m * ldc + n;
        f32x4 lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
        if (e.accumulate) {
            lo += *(const f32x4*)p;
            hi += *(const f32x4*)(p + 4);
        }
        *(f32x4*)p = lo;
        *(f32x4*)(p + 4) = hi;
    } else {
        bf16x8 o;
#pragma unroll
        for (int k = 0; k < 8; ++k) o[k] = (bf16)v[k];
        *(bf16x8*)((bf16*)C + m * ldc + n) = o;
    }
    if (e.aux_out) {
        bf16x8 o;
#pragma unroll
        for (int k = 0; k < 8; ++k) o[k] = (bf16)gelu_fast(v[k]);
        *(bf16x8*)((bf16*)e.aux_out + m * ldc + n) = o;
    }
}

// fp32 output written, not accumulated, without bias / residual / GELU terms (the
// weight-gradient products into the staging buffer): four consecutive columns
// n..n+3 of row m. The callers give consecutive lanes consecutive column quads of
// one row, so that one store instruction writes whole contiguous row segments;
// with eight columns per lane as two 16-byte stores every instruction touches
// every 128-byte line of the segment half-way. Measured on configuration 5's four
// products: +3.7 to +5.7 %. (With C += the eight-column form, whose lane reads and
// writes 32 contiguous bytes, measured 2-3 % faster and is kept.)
__device__ __forceinline__ void epilogue_store4_f32(const Epilogue& e, void* C, long ldc, long m, long n, f32x4 v) {
    *(f32x4*)((float*)C + m * ldc + n) = v * e.alpha;
}
__device__ __forceinline__ bool epilogue_is_plain_f32(const Epilogue& e) {
    return e.out_f32 && !e.accumulate && !e.bias && !e.res && !e.gelu_u && !e.aux_out;
}

// One GEMM problem, possibly batched over (outer, inner) = (sequence, head).
//   C[m,n] = sum_k A(m,k) * B(k,n)
//   A(m,k) = A[m*a_rs + k*a_cs], B(k,n) = B[k*b_rs + n*b_cs]   (element strides)
// causal: 0 none;
//   1 output tiles entirely above the diagonal (n > m) are not computed/written;
//   2 contraction limited to k <= m (row block's upper bound);
//   3 contraction limited to k >= m (row block's lower bound).
struct GemmArgs {
    const void* A; const void* B; void* C;
    int M, N, K;
    long a_rs, a_cs, b_rs, b_cs, ldc;
    int batch = 1, batch_inner = 1;
    long a_bo = 0, a_bi = 0, b_bo = 0, b_bi = 0, c_bo = 0, c_bi = 0;
    int causal = 0;
    Epilogue epi;
};

}  // namespace amdp
