// Device-side vocabulary shared by the HIP kernels: vector types, bf16 conversion, small helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lrd {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }

template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

// Two floats -> packed bf16 pair (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    f32x2 v = {a, b};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

// GELU in its erf form, z * Phi(z), and its derivative Phi(z) + z * phi(z).
// Phi(z) = (1 + erf(z / sqrt 2)) / 2 with erf from the rational approximation 7.1.26 of Abramowitz &
// Stegun (|error| <= 1.5e-7, far below bf16 and the fp32 path's 1e-4 tolerance); it needs
// exp(-z^2 / 2), the same exponential the density phi(z) needs, one reciprocal and a degree-5
// polynomial: ~15 VALU instructions instead of the ~45 of the library erff, which made the GELU
// passes VALU-bound.
__device__ __forceinline__ void gelu_terms(float z, float& Phi, float& phi)
{
    const float x = fabsf(z) * 0.70710678118654752f;
    const float e = __expf(-x * x);                       // = exp(-z^2 / 2)
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float half_erfc = 0.5f * poly * t * e;           // (1 - erf(x)) / 2 for x >= 0
    Phi = z >= 0.f ? 1.f - half_erfc : half_erfc;
    phi = 0.39894228040143268f * e;
}

__device__ __forceinline__ float gelu_f(float z)
{
    float Phi, phi;
    gelu_terms(z, Phi, phi);
    return z * Phi;
}

__device__ __forceinline__ float gelu_grad_f(float z)
{
    float Phi, phi;
    gelu_terms(z, Phi, phi);
    return fmaf(z, phi, Phi);
}

// The same two functions for results that are rounded to bf16 (8 bits of mantissa): odd polynomials in
// the clamped argument, Phi(z) ~ 1/2 + c Q6(c^2) with c = clamp(z, +-4) (|error| <= 1.2e-4) and
// gelu'(z) ~ 1/2 + c R8(c^2) with c = clamp(z, +-4.5) (|error| <= 2.6e-4), least-squares fits on
// Chebyshev nodes.  No exponential and no reciprocal: 10-12 full-rate instructions per element against
// ~25 for the form above.  An epilogue that applies the activation to every element of a wide result
// spends most of its instructions here (20-25 vector instructions per matrix instruction in the fused
// kernels), so this is what the fused epilogues and the bf16 elementwise passes use.
__device__ __forceinline__ float gelu_bf16_f(float z)
{
    const float c = __builtin_amdgcn_fmed3f(z, -4.0f, 4.0f);
    const float s = c * c;
    float q = fmaf(2.804369359e-08f, s, -1.888105544e-06f);
    q = fmaf(q, s, 5.417549619e-05f);
    q = fmaf(q, s, -8.796401089e-04f);
    q = fmaf(q, s, 9.121535346e-03f);
    q = fmaf(q, s, -6.542359293e-02f);
    q = fmaf(q, s, 3.985679448e-01f);
    return z * fmaf(c, q, 0.5f);
}

__device__ __forceinline__ float gelu_grad_bf16_f(float z)
{
    const float c = __builtin_amdgcn_fmed3f(z, -4.5f, 4.5f);
    const float s = c * c;
    float q = fmaf(4.164355527e-10f, s, -4.259615949e-08f);
    q = fmaf(q, s, 1.884581820e-06f);
    q = fmaf(q, s, -4.748817082e-05f);
    q = fmaf(q, s, 7.562761311e-04f);
    q = fmaf(q, s, -7.982769981e-03f);
    q = fmaf(q, s, 5.659934506e-02f);
    q = fmaf(q, s, -2.627864778e-01f);
    q = fmaf(q, s, 7.970107198e-01f);
    return fmaf(c, q, 0.5f);
}

// MFMA operand fragment (v_mfma_f32_32x32x16_bf16: lane L holds row (L & 31), k = 8 * (L >> 5) + 0..7)
// out of a k-major LDS tile [k][row] with LDM elements between consecutive k: two transposing reads.
// Within a block of 16 lanes, ds_read_b64_tr_b16 hands lane l the element (l & 3) of the 8-byte words
// addressed by lanes (l >> 2) + 4e, e = 0..3.  Pointing lane s at [k = kb + (s >> 2)][row = rb + 4 * (s & 3)]
// therefore gives lane l the four values k = kb..kb+3 of row rb + l.
template <int LDM>
__device__ __forceinline__ bf16x8 km_frag(const bf16_t* tile, int row_block, int kk, int lane)
{
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const int blk = lane >> 4, s = lane & 15;
    const int rb = row_block * 32 + 16 * (blk & 1) + 4 * (s & 3);
    const int kb = kk * 16 + 8 * (blk >> 1) + (s >> 2);
    const bf16_t* p = tile + kb * LDM + rb;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 4 * LDM));
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}

__host__ __device__ __forceinline__ constexpr int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Geometry of a k x k convolution on NHWC data, as the kernels see it.
struct ConvShape {
    int N, H, W;     // input batch / height / width
    int Ho, Wo;      // output height / width
    int I, O;        // input / output channels of THIS convolution
    int k, stride, pad;
    // Data gradient of a strided convolution, one parity class at a time: with cls set, the rows of
    // the product are the input pixels with y = cy, x = cx (mod stride) only, and its K runs over
    // the taps that can reach such a pixel (class_taps), not over all k * k.
    int cls = 0, cy = 0, cx = 0;
};

// Taps u = first + stride * t, t = 0 .. count - 1, through which an input coordinate congruent to c
// (mod stride) receives from an output coordinate: u = c + pad - stride * (output coordinate).
struct ClassTaps { int first, count; };
__host__ __device__ __forceinline__ ClassTaps class_taps(int c, int pad, int stride, int k)
{
    const int f = (c + pad) % stride;
    return {f, f < k ? (k - 1 - f) / stride + 1 : 0};
}
// Input coordinates congruent to c (mod stride) below extent.
__host__ __device__ __forceinline__ int class_extent(int extent, int c, int stride) { return extent > c ? (extent - c + stride - 1) / stride : 0; }

}  // namespace lrd
