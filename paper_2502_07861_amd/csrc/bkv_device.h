// Device-side building blocks shared by the BalanceKV kernels (gfx950 / CDNA4 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/balancekv.h"

namespace bkv {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------------
// Counter-based draws for "eta_j = +1 with probability p_j" (Alg. 2 line 9): two rounds of the
// SplitMix64 output mixer over (seed, stream, counter); the top 24 bits give u = bits * 2^-24.
// Integer-only, so host and device agree bit for bit.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}
__host__ __device__ inline uint64_t stream_key(uint64_t seed, uint64_t stream) {
    return mix64(seed + 0x9E3779B97F4A7C15ull * (stream + 1));
}
__host__ __device__ inline uint32_t draw_bits_keyed(uint64_t key, uint64_t ctr) {
    return (uint32_t)(mix64(key + 0x9E3779B97F4A7C15ull * (ctr + 1)) >> 40);
}
__host__ __device__ inline uint32_t draw_bits(uint64_t seed, uint64_t stream, uint64_t ctr) {
    return draw_bits_keyed(stream_key(seed, stream), ctr);
}

// ---------------------------------------------------------------------------------------------
// Element traits: 16-byte operand fragments and the MFMA step that consumes one pair of them.
// A fragment is what one lane contributes to a 32-row (or 32-column) operand for one "k-group"
// of 32 bytes per row: lane (n = lane%32, h = lane/32) holds bytes [32g + 16h, 32g + 16h + 16)
// of row n.  Both operands of the Gram use the same mapping, so the contraction visits every
// column of K exactly once whatever order the hardware pairs the sub-elements in.
// ---------------------------------------------------------------------------------------------
template <typename T> struct Elem;

template <> struct Elem<__bf16> {
    typedef bf16x8_t Frag;
    static constexpr int kPerFrag = 8;                 // elements in 16 bytes
    static __device__ __forceinline__ void mma(floatx16& acc, Frag a, Frag b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
    // the same product on top of c, into a result of its own (c stays intact: several accumulators can start from it)
    static __device__ __forceinline__ floatx16 mma_from(Frag a, Frag b, const floatx16& c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ void unpack(const uintx4& raw, float (&f)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(raw[i] << 16);
            f[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
        }
    }
    // part[e] += element e of the slice, e = 0..7: one v_dot2c_f32_bf16 per element (the pair times (1, 0) or (0, 1): the
    // product with 1 is exact, the one with 0 adds nothing for finite inputs) instead of a shift or mask and an add
    static __device__ __forceinline__ void accumulate(float (&part)[8], const uintx4& raw) {
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        // (1, 0) and (0, 1) as bf16 pairs, kept in registers: written as literals the compiler folds them into an inline
        // operand of the packed instruction that selects the wrong half (both calls then add the high element)
        unsigned int lo_one = 0x00003f80u, hi_one = 0x3f800000u;
        asm volatile("" : "+v"(lo_one), "+v"(hi_one));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned int ri = raw[i];
            part[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, ri), __builtin_bit_cast(bf16x2_t, lo_one), part[2 * i], false);
            part[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, ri), __builtin_bit_cast(bf16x2_t, hi_one), part[2 * i + 1], false);
        }
    }
    // dot product of two 16-byte slices (8 bf16 each), fp32 accumulation: v_dot2c_f32_bf16
    static __device__ __forceinline__ float dot(const uintx4& a, const uintx4& b) {
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned int ai = a[i], bi = b[i];      // scalars first: bit-casting a vector element directly picks element 0
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, ai), __builtin_bit_cast(bf16x2_t, bi), acc, false);
        }
        return acc;
    }
};

template <> struct Elem<float> {
    typedef floatx4 Frag;
    static constexpr int kPerFrag = 4;
    static __device__ __forceinline__ void mma(floatx16& acc, Frag a, Frag b) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], acc, 0, 0, 0);
    }
    static __device__ __forceinline__ floatx16 mma_from(Frag a, Frag b, const floatx16& c) {
        floatx16 acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
#pragma unroll
        for (int e = 1; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], acc, 0, 0, 0);
        return acc;
    }
    static __device__ __forceinline__ void unpack(const uintx4& raw, float (&f)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(raw[i]);
    }
    static __device__ __forceinline__ void accumulate(float (&part)[4], const uintx4& raw) {
#pragma unroll
        for (int i = 0; i < 4; ++i) part[i] += __uint_as_float(raw[i]);
    }
    static __device__ __forceinline__ float dot(const uintx4& a, const uintx4& b) {
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = fmaf(__uint_as_float(a[i]), __uint_as_float(b[i]), acc);
        return acc;
    }
};

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ unsigned int f32_to_bf16_bits(float x) {
    unsigned int u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// all-reduce (sum) over SL consecutive lanes, SL in {8,16,32}: DPP adds inside a row of 16 lanes
template <int SL> __device__ __forceinline__ float group_sum(float x) {
    // all-reduce over SL consecutive lanes (SL in {8,16,32}) with DPP adds
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // row_half_mirror
    if (SL >= 16)
        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));  // row_mirror
    if (SL >= 32) x += __shfl_xor(x, 16);
    return x;
}

// Sixteen values per lane, summed over the 16 lanes of a row: lane s of the row returns the total of x[s].  Each step
// halves the values a lane carries (it keeps the half its own lane bit selects and hands the other half to its
// partner), so the sixteen sums take 15 exchanges instead of 64.
__device__ __forceinline__ float row16_transpose_sum(const float (&x)[16], int s) {
    const bool b3 = (s & 8) != 0, b2 = (s & 4) != 0, b1 = (s & 2) != 0, b0 = (s & 1) != 0;
    float y[8], z[4], u[2];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float mine = b3 ? x[j + 8] : x[j], send = b3 ? x[j] : x[j + 8];
        y[j] = mine + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0x140, 0xF, 0xF, true));   // row_mirror
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float mine = b2 ? y[j + 4] : y[j], send = b2 ? y[j] : y[j + 4];
        z[j] = mine + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0x141, 0xF, 0xF, true));   // row_half_mirror
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float mine = b1 ? z[j + 2] : z[j], send = b1 ? z[j] : z[j + 2];
        u[j] = mine + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    }
    const float mine = b0 ? u[1] : u[0], send = b0 ? u[0] : u[1];
    return mine + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));        // quad_perm [1,0,3,2]
}

}  // namespace bkv
