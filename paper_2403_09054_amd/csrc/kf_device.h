// Device-side helpers shared by the Keyformer kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kf {

// bf16 storage type: the upper half of an fp32.
struct bf16_t {
    uint16_t bits;
};

// IEEE half storage type.
struct f16_t {
    uint16_t bits;
};

constexpr int kWave = 64;

// Mean and standard deviation of the standard Gumbel pdf as the paper prints
// them (Sec. 4.4.3); used by its Gaussian and constant ablation variants.
constexpr float kAdjMean = 0.5772f;
constexpr float kAdjStd = 1.2825f;

enum Noise : int { kNoiseNone = 0, kNoiseGumbel = 1, kNoiseGaussian = 2, kNoiseConstant = 3 };

// ---------------------------------------------------------------- elements
template <typename T>
struct ElemTraits;
template <>
struct ElemTraits<float> {
    static constexpr int kPerVec = 4;  // elements in a 16-byte vector
};
template <>
struct ElemTraits<bf16_t> {
    static constexpr int kPerVec = 8;
};
template <>
struct ElemTraits<f16_t> {
    static constexpr int kPerVec = 8;
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Expands one 16-byte vector of T into floats.
template <typename T>
__device__ __forceinline__ void unpack16(const uint4& r, float* f);
template <>
__device__ __forceinline__ void unpack16<float>(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x);
    f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z);
    f[3] = __uint_as_float(r.w);
}
template <>
__device__ __forceinline__ void unpack16<bf16_t>(const uint4& r, float* f) {
    f[0] = bf16_lo(r.x);
    f[1] = bf16_hi(r.x);
    f[2] = bf16_lo(r.y);
    f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z);
    f[5] = bf16_hi(r.z);
    f[6] = bf16_lo(r.w);
    f[7] = bf16_hi(r.w);
}

__device__ __forceinline__ float f16_lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu)); }
__device__ __forceinline__ float f16_hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
template <>
__device__ __forceinline__ void unpack16<f16_t>(const uint4& r, float* f) {
    f[0] = f16_lo(r.x);
    f[1] = f16_hi(r.x);
    f[2] = f16_lo(r.y);
    f[3] = f16_hi(r.y);
    f[4] = f16_lo(r.z);
    f[5] = f16_hi(r.z);
    f[6] = f16_lo(r.w);
    f[7] = f16_hi(r.w);
}

// ---------------------------------------------------------------- streaming access
// 16-byte loads / stores of data that is touched once per launch (K and V rows):
// marked non-temporal so that they stream through the caches instead of
// displacing lines.  On MI355X the decode kernel reads 6.1-6.3 TB/s this way
// against 5.7 TB/s with ordinary loads.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store(uint4* p, const uint4& v) {
    u32x4_t t;
    t.x = v.x;
    t.y = v.y;
    t.z = v.z;
    t.w = v.w;
    __builtin_nontemporal_store(t, (u32x4_t*)p);
}

// ---------------------------------------------------------------- noise hash
// Counter-based generator keyed by (seed, layer, head, query position, key's
// original position).  The paper only names the distribution of the logit
// adjustment (Eq. 4, Eq. 7); the generator is this library's own.
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 32;
    z *= 0x6A09E667F3BCC909ull;
    z ^= z >> 29;
    z *= 0xBB67AE8584CAA73Bull;
    z ^= z >> 32;
    return z;
}

__host__ __device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x6A09E667u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

constexpr uint32_t kQposMul = 0x9E3779B9u;
constexpr uint32_t kKposMul = 0x243F6A89u;

// Per-unit key, constant for a (sequence seed, layer, head).
__host__ __device__ __forceinline__ uint64_t unit_key(uint64_t seed, uint32_t layer, uint32_t head) {
    return mix64(mix64(seed + 0x9E3779B97F4A7C15ull) + (((uint64_t)layer << 32) | (uint64_t)head));
}

// Per-query-row key: constant along a row of logits (one decode step).
__host__ __device__ __forceinline__ uint32_t row_key(uint64_t ukey, uint32_t q_pos) {
    const uint32_t ka = (uint32_t)ukey, kb = (uint32_t)(ukey >> 32);
    return mix32(mix32(ka ^ (q_pos * kQposMul)) + kb);
}

// The 32 random bits of one logit.
__host__ __device__ __forceinline__ uint32_t logit_bits(uint32_t rkey, uint32_t k_pos) {
    return mix32(rkey ^ (k_pos * kKposMul));
}

// ---------------------------------------------------------------- base-2 transcendentals
// The hardware log2 / exp2 (v_log_f32, v_exp_f32).  Measured on gfx950 over all
// 2^23 uniforms the generator can produce: -log2(u) is within 1.2e-7 relative,
// also where u is next to 1; exp2 is within 8.3e-8 relative on [-40, 20].
__device__ __forceinline__ float hw_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// Temperature schedule (Eq. 12) in fp32: one multiplication, one addition, each
// rounded on its own.  Host and device must produce the same bits, so the
// compiler may not contract the pair into a fused multiply-add.
__host__ __device__ inline float schedule_tau(float tau_init, float dtau, int t) {
#pragma clang fp contract(off)
    const float ramp = (float)t * dtau;
    return tau_init + ramp;
}

constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;
constexpr float kLog2Ln2 = -0.52876637294489779f;  // log2(ln 2)

// u = (2*(bits >> 9) + 1) / 2^24, an odd multiple of 2^-24 in (0,1), in two instructions: the 23 bits
// become the mantissa of a float in [1,2) (one funnel shift puts them behind the exponent of 1.0), and
// subtracting 1 - 2^-24 leaves exactly u (the difference has at most 24 significant bits, so the
// subtraction does not round; checked on the host for all 2^23 values).
__device__ __forceinline__ float uniform_of(uint32_t bits) {
    return __uint_as_float(__builtin_amdgcn_alignbit(0x7Fu, bits, 9)) - 0x0.FFFFFFp0f;
}

// t = -log2(u) > 0.
__device__ __forceinline__ float neg_log2_uniform(uint32_t bits) { return -hw_log2(uniform_of(bits)); }

// Standard Gumbel variate (inverse CDF of Eq. 7) times log2(e):
//   zeta = -ln(-ln u), -ln u = t*ln2  =>  log2(e)*zeta = -(log2(t) + log2(ln 2)).
__device__ __forceinline__ float gumbel_log2e(uint32_t bits) {
    return -(hw_log2(neg_log2_uniform(bits)) + kLog2Ln2);
}

// Logit adjustment zeta (Eq. 4) for one (query, key) pair, times log2(e).
__device__ __forceinline__ float zeta_log2e(int noise, uint32_t rkey, uint32_t k_pos) {
    switch (noise) {
        case kNoiseGumbel:
            return gumbel_log2e(logit_bits(rkey, k_pos));
        case kNoiseGaussian: {  // Eq. 5 via Box-Muller on two draws
            const float l1 = neg_log2_uniform(logit_bits(rkey, k_pos)) * kLn2;  // -ln u1
            const float u2 = uniform_of(logit_bits(rkey, k_pos ^ 0x80000000u));
            return (kAdjMean + kAdjStd * (sqrtf(2.0f * l1) * cospif(2.0f * u2))) * kLog2e;
        }
        case kNoiseConstant:
            return kAdjMean * kLog2e;
        default:
            return 0.0f;
    }
}

// ---------------------------------------------------------------- reductions
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Block-wide reductions through a small LDS array (>= NT/64 floats).  Every
// thread of the block must call them; the result is returned to all.
template <int NT>
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) r = fmaxf(r, red[i]);
    return r;
}
template <int NT>
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) r += red[i];
    return r;
}

// Order-preserving map from fp32 to uint32 (larger float <=> larger key).
__device__ __forceinline__ uint32_t float_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

}  // namespace kf
