// Device-side helpers shared by the gfx950 kernels of libmbconv.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mbk {

constexpr int kWave = 64;

struct bf16_t {
    uint16_t bits;
};

// ---- storage <-> fp32 --------------------------------------------------------------

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even by the hardware conversion (v_cvt_pk_bf16_f32, one instruction per
// pair instead of five integer operations per value); NaN stays NaN
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
// two values rounded to bf16 and packed, lo in bits 0-15
__device__ __forceinline__ uint32_t bf16_pack2(float lo, float hi)
{
    typedef float float2v __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
    const float2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}

// v where the mask is all ones, +0 where it is zero (one v_and_b32, never a branch)
__device__ __forceinline__ float and_mask(float v, uint32_t mask)
{
    return __uint_as_float(__float_as_uint(v) & mask);
}

template <typename T>
__device__ __forceinline__ float ld(const T *p, size_t i);
template <>
__device__ __forceinline__ float ld<float>(const float *p, size_t i)
{
    return p[i];
}
template <>
__device__ __forceinline__ float ld<bf16_t>(const bf16_t *p, size_t i)
{
    return bf16_bits_to_float(p[i].bits);
}

template <typename T>
__device__ __forceinline__ void st(T *p, size_t i, float v);
template <>
__device__ __forceinline__ void st<float>(float *p, size_t i, float v)
{
    p[i] = v;
}
template <>
__device__ __forceinline__ void st<bf16_t>(bf16_t *p, size_t i, float v)
{
    p[i].bits = float_to_bf16_bits(v);
}

// The value a tensor of type T holds after storing v.
template <typename T>
__device__ __forceinline__ float as_stored(float v);
template <>
__device__ __forceinline__ float as_stored<float>(float v)
{
    return v;
}
template <>
__device__ __forceinline__ float as_stored<bf16_t>(float v)
{
    return bf16_bits_to_float(float_to_bf16_bits(v));
}

// ---- activation ----------------------------------------------------------------------

__device__ __forceinline__ float sigmoidf_fast(float t)
{
    // 1/(1+2^(-t*log2 e)) with the hardware v_exp_f32 and v_rcp_f32, each accurate to about
    // 1 ulp (a correctly rounded division would cost ten more instructions per element)
    return __builtin_amdgcn_rcpf(1.0f + __expf(-t));
}

__device__ __forceinline__ float swishf(float t) { return t * sigmoidf_fast(t); }

// Swish(t) and its derivative sigma*(1+t*(1-sigma)) from one sigmoid evaluation.
__device__ __forceinline__ void swish_both(float t, float &val, float &grad)
{
    float s = sigmoidf_fast(t);
    val = t * s;
    grad = s * (1.0f + t * (1.0f - s));
}

// The block's activation after BN1 and BN2, fixed at compile time: Swish (EfficientNet MBConv),
// or ReLU6 when the translation unit is built with MBK_ACT_RELU6 (MobileNet-V2 inverted
// residual; the whole kernel set is compiled a second time into its own namespace).  The
// squeeze-and-excitation stage keeps swishf / sigmoidf_fast in both builds.
//   act_aux(y)        what is worth keeping of y for a later derivative (sigmoid(y) for Swish)
//   act_val(y, aux)   the activation
//   act_grad(y, aux)  its derivative; ReLU6: 1 strictly inside (0, 6), 0 elsewhere
#ifdef MBK_ACT_RELU6
__device__ __forceinline__ float act_aux(float y) { return y; }
__device__ __forceinline__ float act_val(float y, float) { return fminf(fmaxf(y, 0.0f), 6.0f); }
__device__ __forceinline__ float act_grad(float y, float) { return (y > 0.0f && y < 6.0f) ? 1.0f : 0.0f; }
#else
__device__ __forceinline__ float act_aux(float y) { return sigmoidf_fast(y); }
__device__ __forceinline__ float act_val(float y, float aux) { return y * aux; }
__device__ __forceinline__ float act_grad(float y, float aux) { return aux * (1.0f + y * (1.0f - aux)); }
#endif
__device__ __forceinline__ float actf(float y) { return act_val(y, act_aux(y)); }
__device__ __forceinline__ void act_both(float y, float &val, float &grad)
{
    const float aux = act_aux(y);
    val = act_val(y, aux);
    grad = act_grad(y, aux);
}

// ---- integer division by a per-launch constant ------------------------------------------
// Exact for every 32-bit numerator (the round-up multiply-shift scheme of Granlund and
// Montgomery): with l = ceil(log2 d) and m = floor(2^32*(2^l-d)/d)+1,
//   t = mulhi(m, n);  n/d = (t + ((n-t) >> min(l,1))) >> max(l-1,0).
struct FastDiv {
    uint32_t d, m, sh1, sh2;
};
inline FastDiv make_div(uint32_t d)
{
    FastDiv f;
    uint32_t l = 0;
    while ((1ull << l) < d)
        ++l;
    f.d = d;
    f.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1ull);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 1 ? l - 1 : 0;
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t n, FastDiv f)
{
    const uint32_t t = __umulhi(f.m, n);
    return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// ---- reductions ------------------------------------------------------------------------

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, false)); // row_ror:8
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xf, 0xf, false)); // row_ror:4
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x122, 0xf, 0xf, false)); // row_ror:2
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x121, 0xf, 0xf, false)); // row_ror:1
    return v;
}

// Sum over the 64 lanes of the wavefront with DPP only (no LDS crossbar traffic, unlike a
// butterfly of __shfl_xor, which costs a ds_bpermute per step): four rotations inside each row
// of 16 lanes, then lane 15 of rows 0 and 2 is added into rows 1 and 3 (row_bcast:15) and lane 31
// into rows 2 and 3 (row_bcast:31).  Lanes 48..63 end with the total.  Every lane of the
// wavefront must be active.
__device__ __forceinline__ float wave_sum_lane63(float v)
{
    v = row16_sum(v);
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xa, 0xf, false)); // row_bcast:15
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xc, 0xf, false)); // row_bcast:31
    return v;
}
// The same, with the total broadcast to every lane (v_readlane of lane 63).
__device__ __forceinline__ float wave_sum(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_sum_lane63(v)), 63));
}

// Sum over the 32 lanes that share lane/32, by DPP row rotations plus one cross-row exchange.
__device__ __forceinline__ float half_wave_sum_dpp(float v)
{
    v = row16_sum(v);
    return v + __shfl_xor(v, 16, kWave);
}

// sum over the 32 lanes that share lane/32
__device__ __forceinline__ float half_wave_sum(float v)
{
#pragma unroll
    for (int o = 16; o > 0; o >>= 1)
        v += __shfl_xor(v, o, kWave);
    return v;
}

// Sum of NV per-thread values over a group of TPP consecutive threads of the block
// (TPP = 16 or a multiple of 64, groups aligned).  `red` is LDS scratch of at least
// (blockDim/64)*NV floats.  The result is valid in the first wavefront of every group (callers
// use it in the group's first thread).  All threads of the block must call it (it synchronises
// the block when TPP > 64).
template <int NV, int TPP>
__device__ __forceinline__ void group_sum(float (&v)[NV], float *red)
{
    if (TPP == 16) { // a DPP row per group: four rotations, no LDS, no cross-lane permute
#pragma unroll
        for (int i = 0; i < NV; ++i)
            v[i] = row16_sum(v[i]);
        return;
    }
    if (TPP == kWave) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
            v[i] = wave_sum(v[i]);
        return;
    }
    // several wavefronts per group: lane 63 of each leaves its wavefront's totals in LDS and the
    // group's first wavefront adds them in wavefront order
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    constexpr int WPG = TPP / kWave;
#pragma unroll
    for (int i = 0; i < NV; ++i)
        v[i] = wave_sum_lane63(v[i]);
    __syncthreads();
    if (lane == kWave - 1) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
            red[wave * NV + i] = v[i];
    }
    __syncthreads();
    if (wave % WPG == 0) { // uniform over the wavefront
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            float s = 0.f;
            for (int w = 0; w < WPG; ++w)
                s += red[(wave + w) * NV + i];
            v[i] = s;
        }
    }
}

} // namespace mbk
