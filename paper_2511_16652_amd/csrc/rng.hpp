// Counter-based noise for EGGROLL on gfx950: Threefry-2x32-20 (Salmon et al., SC'11 -- the generator
// family the paper cites for on-demand noise reconstruction, Sec. 1 and Alg. 1) and the maps from
// 32-bit words to Gaussian / bounded-integer factor entries.
//
// Everything here is integer ALU work plus four transcendental ops per Box-Muller pair; the stream
// key is wave-uniform, so the key schedule lives in scalar registers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace egg {

struct StreamKey {  // derived key of one (seed, step, layer, which) stream, with its parity word
    uint32_t k0, k1, k2;
};

__host__ __device__ __forceinline__ uint32_t rotl(uint32_t v, int s) { return (v << s) | (v >> (32 - s)); }

// one Threefry-2x32-20 block: (c0, c1) under key (k0, k1); k2 = k0 ^ k1 ^ 0x1BD11BDA
__host__ __device__ __forceinline__ void threefry2x32_20(uint32_t k0, uint32_t k1, uint32_t k2, uint32_t c0,
                                                         uint32_t c1, uint32_t& o0, uint32_t& o1)
{
    uint32_t x0 = c0 + k0, x1 = c1 + k1;
#define EGG_TF_MIX(R) x0 += x1; x1 = rotl(x1, R); x1 ^= x0;
    EGG_TF_MIX(13) EGG_TF_MIX(15) EGG_TF_MIX(26) EGG_TF_MIX(6)
    x0 += k1; x1 += k2 + 1u;
    EGG_TF_MIX(17) EGG_TF_MIX(29) EGG_TF_MIX(16) EGG_TF_MIX(24)
    x0 += k2; x1 += k0 + 2u;
    EGG_TF_MIX(13) EGG_TF_MIX(15) EGG_TF_MIX(26) EGG_TF_MIX(6)
    x0 += k0; x1 += k1 + 3u;
    EGG_TF_MIX(17) EGG_TF_MIX(29) EGG_TF_MIX(16) EGG_TF_MIX(24)
    x0 += k1; x1 += k2 + 4u;
    EGG_TF_MIX(13) EGG_TF_MIX(15) EGG_TF_MIX(26) EGG_TF_MIX(6)
    x0 += k2; x1 += k0 + 5u;
#undef EGG_TF_MIX
    o0 = x0;
    o1 = x1;
}

// host side: key of the stream named by (seed, step, layer, which)
inline StreamKey make_stream_key(uint64_t seed, uint32_t step, uint32_t layer, int which)
{
    const uint32_t s0 = (uint32_t)seed, s1 = (uint32_t)(seed >> 32);
    StreamKey k;
    threefry2x32_20(s0, s1, s0 ^ s1 ^ 0x1BD11BDAu, step, (layer & 0x7FFFFFFFu) | ((uint32_t)(which & 1) << 31),
                    k.k0, k.k1);
    k.k2 = k.k0 ^ k.k1 ^ 0x1BD11BDAu;
    return k;
}

// words 2*block, 2*block+1 of member's vector
__device__ __forceinline__ void noise_words(const StreamKey& k, uint32_t member, uint32_t block, uint32_t& w0,
                                            uint32_t& w1)
{
    threefry2x32_20(k.k0, k.k1, k.k2, block, member, w0, w1);
}

// u = ((w >> 9) + 1/2) * 2^-23, exact in fp32 (24 significant bits)
__device__ __forceinline__ float word_to_unit(uint32_t w)
{
    return (float)((w >> 9) * 2u + 1u) * 5.9604644775390625e-08f;  // (2k+1) * 2^-24
}

// Box-Muller pair from one block.  PRECISE: library log/sincospi (few-ulp), used where the factors
// stay fp32; otherwise the hardware log2/sin/cos/sqrt approximations, whose error is far below the
// bf16 rounding applied to the result.
template <bool PRECISE>
__device__ __forceinline__ void normal_pair(uint32_t w0, uint32_t w1, float& z0, float& z1)
{
    const float u1 = word_to_unit(w0);
    const float u2 = word_to_unit(w1);
    if constexpr (PRECISE) {
        const float rho = sqrtf(-2.0f * logf(u1));
        float s, c;
        sincospif(2.0f * u2, &s, &c);
        z0 = rho * c;
        z1 = rho * s;
    } else {
        // -2 ln u = -2 ln2 * log2 u ; v_sin/v_cos take their argument in revolutions
        const float rho = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1));
        z0 = rho * __builtin_amdgcn_cosf(u2);
        z1 = rho * __builtin_amdgcn_sinf(u2);
    }
}

// byte -> integer on {-b..b}: m = 2b+1, q = 256/m; byte < q*m ? byte/q - b : 0.
// qm = q*m and the reciprocal multiplier are precomputed on the host (see IntMap).
struct IntMap {
    int bound;
    uint32_t q, qm, magic;  // byte / q == (byte * magic) >> 16 for byte < 256
};

inline IntMap make_int_map(int bound)
{
    IntMap m;
    m.bound = bound;
    const uint32_t mm = 2u * (uint32_t)bound + 1u;
    m.q = 256u / mm;
    m.qm = m.q * mm;
    m.magic = (65536u + m.q - 1u) / m.q;  // ceil(2^16 / q): exact for all byte < 256 (checked on the host)
    return m;
}

__host__ __device__ __forceinline__ int int_from_byte(const IntMap& m, uint32_t byte)
{
    return byte < m.qm ? (int)((byte * m.magic) >> 16) - m.bound : 0;
}

// four packed int8 values from one word
__device__ __forceinline__ uint32_t int4_from_word(const IntMap& m, uint32_t w)
{
    uint32_t out = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) out |= ((uint32_t)int_from_byte(m, (w >> (8 * b)) & 0xFFu) & 0xFFu) << (8 * b);
    return out;
}

// fp32 -> bf16, round to nearest even, through the gfx950 packed conversion instruction
typedef __bf16 egg_bf16x2 __attribute__((ext_vector_type(2)));
typedef float egg_f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const egg_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, egg_bf16x2));
}

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) { return (uint16_t)(pack_bf16x2(f, 0.f) & 0xFFFFu); }

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

// round an fp32 value to the nearest bf16 and return it as fp32
__device__ __forceinline__ float round_bf16(float f) { return bf16_lo(pack_bf16x2(f, 0.f)); }

}  // namespace egg
