// Shared device helpers for the gfx950 shard-GEMM kernels: vector types, bf16 conversion,
// epilogue math.  Wave size is 64 everywhere.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace axo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

typedef uint16_t bf16_t;  // bf16 bit pattern in memory

// Operand layouts of C[i,j] = sum_r A(i,r) * B(j,r):
//   KC: the reduction index r is contiguous in memory   (element (i,r) at i*ld + r)
//   MC: the output index i (or j) is contiguous         (element (i,r) at r*ld + i)
enum Layout { KC = 0, MC = 1 };

// What happens to the fp32 accumulator on its way out.  1-3 belong to the forward product, 4-5
// to dgrad (multiply by the activation's derivative at the pre-activation `aux`), 6 to wgrad
// (add into an fp32 matrix instead of rounding to bf16).
enum Epilogue {
    EPI_NONE = 0, EPI_BIAS = 1, EPI_BIAS_GELU_TANH = 2, EPI_BIAS_GELU_ERF = 3,
    EPI_MUL_DGELU_TANH = 4, EPI_MUL_DGELU_ERF = 5, EPI_ACC_F32 = 6
};

// One GEMM as the kernels see it.
struct GemmArgs {
    const bf16_t* A; int64_t lda;
    const bf16_t* B; int64_t ldb;
    bf16_t* C;       int64_t ldc;   // EPI_ACC_F32: C points to fp32 and ldc counts fp32 elements
    const bf16_t* bias;  // [No] or nullptr
    const bf16_t* aux; int64_t ldaux;  // [Mo x No] pre-activation for EPI_MUL_DGELU_*, else nullptr
    int Mo, No, R;       // output rows, output cols, reduction length
    int epilogue;        // Epilogue
    int add_bias;        // 0: bias pointer ignored (shard is not at K-coordinate 0)
};

__device__ __forceinline__ float bf16_bits_to_f32(bf16_t b) {
    return __uint_as_float(((uint32_t)b) << 16);
}

// fp32 -> bf16 bits, round to nearest, ties to even; NaN stays NaN (quiet).
__device__ __forceinline__ bf16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Two fp32 values -> packed bf16 pair (low half = a), round to nearest even, NaN stays NaN: the
// gfx950 packed conversion instruction.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    const f32x2 v = {a, b};
    const bf16x2 r = __builtin_convertvector(v, bf16x2);
    union { bf16x2 v; uint32_t u; } u;
    u.v = r;
    return u.u;
}

// GELU, tanh form: 0.5 v (1 + tanh(z)) = v * sigmoid(2 z), z = sqrt(2/pi) (v + 0.044715 v^3).
// The sigmoid form has no cancellation for large negative v.
__device__ __forceinline__ float gelu_tanh(float v) {
    // -2 z log2(e) = v (k1 + k3 v^2); one exp2 and one reciprocal (1 ulp each: far inside the bf16
    // rounding that follows; a true division would cost ten more instructions per element)
    const float k1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    const float k3 = k1 * 0.044715f;
    const float t = v * __builtin_fmaf(k3, v * v, k1);
    return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

// GELU, erf form: 0.5 v (1 + erf(v / sqrt 2)) = 0.5 v erfc(-v / sqrt 2)  (no cancellation).
__device__ __forceinline__ float gelu_erf(float v) {
    return 0.5f * v * erfcf(-v * 0.7071067811865475f);
}

// d/dv of the tanh-form GELU.  With s = sigmoid(2 z): 0.5 (1 + tanh z) = s and 1 - tanh^2 z = 4 s (1 - s),
// so the derivative is s (1 + 2 v (1 - s) z'), z' = sqrt(2/pi) (1 + 3 * 0.044715 v^2).
__device__ __forceinline__ float dgelu_tanh(float v) {
    const float c = 0.7978845608028654f;
    const float k1 = -2.0f * c * 1.4426950408889634f, k3 = k1 * 0.044715f;
    const float v2 = v * v;
    const float s = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * __builtin_fmaf(k3, v2, k1)));
    const float dz = c * __builtin_fmaf(3.0f * 0.044715f, v2, 1.0f);
    return s * __builtin_fmaf(2.0f * v * (1.0f - s), dz, 1.0f);
}

// d/dv of the exact GELU: Phi(v) + v phi(v).
__device__ __forceinline__ float dgelu_erf(float v) {
    const float phi = 0.3989422804014327f * __expf(-0.5f * v * v);
    return 0.5f * erfcf(-v * 0.7071067811865475f) + v * phi;
}

__device__ __forceinline__ float apply_epilogue(float acc, float b, int epi) {
    float v = acc + b;
    if (epi == EPI_BIAS_GELU_TANH) v = gelu_tanh(v);
    else if (epi == EPI_BIAS_GELU_ERF) v = gelu_erf(v);
    return v;
}

// dgrad through an activation: accumulator times the activation's derivative at pre-activation p
__device__ __forceinline__ float apply_dact(float acc, float p, int epi) {
    return acc * (epi == EPI_MUL_DGELU_TANH ? dgelu_tanh(p) : dgelu_erf(p));
}

}  // namespace axo
