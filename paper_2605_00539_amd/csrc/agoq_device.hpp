#ifndef AGOQ_DEVICE_HPP
#define AGOQ_DEVICE_HPP
// Device and host helpers shared by the kernel files of the AGoQ quantization hot path
// for gfx950 (MI355X): tuning constants, cache-hinted loads and stores, the cross-lane
// abs-max, the group scale, and the encoders / decoders of every code width.
//
// Every kernel here is a streaming pass: read a tensor once, write its encoded
// (or decoded) form once.  The bound is HBM bandwidth, so the design goals are
//   * 16-byte loads, several in flight per lane, issued before any use;
//   * one quantization group per DPP row (16 lanes) or half row, so the
//     abs-max reduction is a few cross-lane VALU ops and never touches LDS;
//   * codes packed in registers and stored as whole dwords / 16-byte vectors.
// No MFMA: nothing on this path is a contraction.
//
// Arithmetic contract (identical for all kernels): IEEE binary32, round to
// nearest even, no contraction.  scale = amax / qmax and inv = qmax / amax are
// true divisions; code = rint(x * inv).  rint is realised by adding 1.5 * 2^23:
// for |t| <= 2^22 the sum lies in [2^23, 2^24) where the spacing of binary32 is
// exactly 1, so the addition itself rounds t to the nearest integer, ties to
// even, and the low mantissa bits hold the integer in two's complement.
// Because |x| <= amax, |x * inv| <= qmax * (1 + 2^-22), whose nearest integer
// is at most qmax: the codes need no clamp.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <tuple>
#include <type_traits>

#include "agoq.h"
namespace {

typedef uint32_t u32;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- launch shapes, per kernel (measured on MI355X) ------------------------------------
// Block = lanes per workgroup, Unroll = 16-byte vectors (or dwords of codes) per lane.
// Every streaming load and store carries the non-temporal hint except the loads of scales in
// the dequantize kernels (a scale is read by up to 16 lanes).
constexpr int kAqBlock = 128, kAqUnroll = 2;     // activation quantize
constexpr int kDqBlock = 512;                    // activation dequantize (unroll chosen per launch)
constexpr int kGqBlock = 256, kGqUnroll = 1;     // gradient quantize and fp32-addend accumulate
constexpr int kGbBlock = 128, kGbUnroll = 2;     // accumulate, bf16 addend
constexpr int kGdBlock = 512, kGdUnroll = 2;     // gradient dequantize
constexpr int kSiBlock = 256, kSiBlockNarrow = 128, kSiUnroll = 2;   // SiLU & Multiply recompute (8-bit; below)
// Occupancy caps: dynamic LDS (bytes per workgroup, never touched by the kernel) that limits
// how many workgroups share a compute unit's 160 KB.  Measured per kernel: kernels that read
// or write several streams at once run faster with fewer wavefronts in flight than the
// registers allow; single-stream kernels have no cap.
constexpr size_t kCapGa = 26 * 1024;    // accumulate, fp32 addend: 6 workgroups of 256
constexpr size_t kCapSf = 20 * 1024;    // SiLU & Multiply forward + quantize: 8 workgroups of 128
constexpr size_t kCapLdq = 48 * 1024;   // layer dequantize: 3 workgroups of 512
constexpr size_t kCapDq8 = 48 * 1024;   // dequantize of 8-bit codes, tensors beyond one round: 3 of 512
constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23
constexpr u32 kAmaxMinBits = 0x0D800000u;   // 2^-100: groups below it are stored as zeros
constexpr u32 kInfBits = 0x7F800000u;       // magnitudes from here up are Inf or NaN
constexpr u32 kQuietNanBits = 0x7FC00000u;  // the scale of a group that holds one

__device__ __forceinline__ float as_f32(u32 u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ u32 as_u32(float f) { return __builtin_bit_cast(u32, f); }

// Streaming loads and stores: every byte is touched once, so the caches may drop it early.
template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T v)
{
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// DPP controls (row = 16 lanes)
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i within 8 lanes
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i within 16 lanes

template <int CTRL>
__device__ __forceinline__ u32 dpp_max_u32(u32 v)
{
    u32 o = (u32)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
    return v > o ? v : o;
}

// Maximum over the LANES consecutive lanes (4, 8 or 16, aligned) that share a group.
// Operates on magnitude bit patterns: for non-negative finite floats the unsigned
// integer order of the bits is the order of the values.
template <int LANES>
__device__ __forceinline__ u32 group_max_bits(u32 m)
{
    m = dpp_max_u32<kDppXor1>(m);
    m = dpp_max_u32<kDppXor2>(m);
    if (LANES >= 8) m = dpp_max_u32<kDppHalfMirror>(m);
    if (LANES >= 16) m = dpp_max_u32<kDppMirror>(m);
    return m;
}

__device__ __forceinline__ u32 umax(u32 a, u32 b) { return a > b ? a : b; }

// scale and inv of a group from the bits of its abs-max (integer order of the magnitude
// bits: Inf and every NaN sort above all finite values).  Returns whether the group keeps
// its codes: not a dead group (abs-max below 2^-100: scale 0) and not one that holds an Inf
// or a NaN (scale = quiet NaN, so the whole group reads back as NaN).  Otherwise inv = 0 and
// the caller stores zeros for the codes (x * 0 is not zero for a non-finite x).
template <int QMAX>
__device__ __forceinline__ bool scale_and_inv(u32 amax_bits, float& scale, float& inv)
{
    const float amax = as_f32(amax_bits);
    const bool finite = amax_bits < kInfBits;
    const bool keep = amax_bits >= kAmaxMinBits && finite;
    const float den = keep ? amax : 1.0f;
    const float s = __fdiv_rn(amax, (float)QMAX);
    const float r = __fdiv_rn((float)QMAX, den);
    scale = keep ? s : finite ? 0.0f : as_f32(kQuietNanBits);
    inv = keep ? r : 0.0f;
    return keep;
}

// round(x * inv) as the low bits of the returned word (two's complement).
__device__ __forceinline__ u32 code_bits(float x, float inv)
{
    return as_u32(__fadd_rn(__fmul_rn(x, inv), kRoundMagic));
}

// ---- stochastic rounding (optional variant; the paper itself rounds to nearest) ---------
// code = max(floor(x * inv + u), -qmax) with u = B / 256, B one byte of a 32-bit hash word
// that the four consecutive elements 4b .. 4b+3 share (byte 0, the least significant, is
// element 4b's):
//     key  = mix(seed ^ (high 32 bits of b) * 0x9E3779B9)
//     word = mix((low 32 bits of b) ^ key)
// mix() is the 32-bit finalizer of MurmurHash3.  x * inv + u is ONE binary32 addition of the
// rounded product and u (here an fma with the exact factor 2^-8, which rounds the same
// sum).  The sum stays below qmax + 1, so only the lower clamp can ever act (x = -amax can
// come out a hair below -qmax).
__device__ __forceinline__ u32 sr_mix(u32 h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

__device__ __forceinline__ u32 sr_word(u32 seed, int64_t block)
{
    const u32 lo = (u32)block, hi = (u32)((uint64_t)block >> 32);
    u32 key = sr_mix(seed);                      // the same for every lane: scalar work
    if (hi != 0) key = sr_mix(seed ^ (hi * 0x9E3779B9u));   // tensors beyond 2^34 elements
    return sr_mix(lo ^ key);
}

template <int K>
__device__ __forceinline__ float ubyte_to_f32(u32 w);     // (defined with the decoders below)

// The stochastic code of x under byte K of `word`, as the low bits of the returned word.
template <int K, int QMAX>
__device__ __forceinline__ u32 sr_code_bits(float x, float inv, u32 word)
{
    const float shifted = __fmaf_rn(ubyte_to_f32<K>(word), 0.00390625f, __fmul_rn(x, inv));
    const float r = fmaxf(__builtin_floorf(shifted), -(float)QMAX);
    return (u32)(int)r;
}

// The codes of the four elements 4*block .. 4*block+3 (low bits of c[0..3], two's complement).
template <bool SR, int QMAX>
__device__ __forceinline__ void codes4(float x0, float x1, float x2, float x3, float inv, u32 seed,
                                       int64_t block, u32 (&c)[4])
{
    if constexpr (SR) {
        const u32 word = sr_word(seed, block);
        c[0] = sr_code_bits<0, QMAX>(x0, inv, word);
        c[1] = sr_code_bits<1, QMAX>(x1, inv, word);
        c[2] = sr_code_bits<2, QMAX>(x2, inv, word);
        c[3] = sr_code_bits<3, QMAX>(x3, inv, word);
    } else {
        c[0] = code_bits(x0, inv);
        c[1] = code_bits(x1, inv);
        c[2] = code_bits(x2, inv);
        c[3] = code_bits(x3, inv);
    }
}

__device__ __forceinline__ u32 push_nibble(u32 packed, u32 code)
{
    // shifts the pair {code, packed} right by 4: the new nibble enters at the top, so
    // after eight pushes the first element sits in bits 0-3
    return __builtin_amdgcn_alignbit(code, packed, 4);
}

__device__ __forceinline__ u32 push_byte(u32 packed, u32 code)
{
    return __builtin_amdgcn_alignbit(code, packed, 8);
}

// Signed byte j of a word as a float: one conversion with a sign-extending byte select.
__device__ __forceinline__ float byte_to_f32(u32 w, int j)
{
    return (float)(int8_t)((w >> (8 * j)) & 0xFFu);
}

// ---- floating-point code books (E2M1 nibbles, OCP E4M3 bytes) ----------------------
// gfx950's conversion instructions round to nearest, ties to the even mantissa, saturate
// at the largest magnitude and keep the sign of a zero -- the semantics of the code books
// here.  fp4 conversions take a power-of-two scale operand; it is always 1.

// Four fp32 values times inv -> one word of 8-bit codes, element 0 in the low byte.  The
// four are the tensor elements 4*block .. 4*block+3 (which matters to stochastic rounding only).
template <bool FP, bool SR = false>
__device__ __forceinline__ u32 encode4_bytes(float x0, float x1, float x2, float x3, float inv,
                                             u32 seed = 0, int64_t block = 0)
{
    static_assert(!(FP && SR), "stochastic rounding is defined for the integer grids");
    if constexpr (FP) {
        int w = 0;
        w = __builtin_amdgcn_cvt_pk_fp8_f32(__fmul_rn(x0, inv), __fmul_rn(x1, inv), w, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(__fmul_rn(x2, inv), __fmul_rn(x3, inv), w, true);
        return (u32)w;
    } else {
        u32 c[4];
        codes4<SR, 127>(x0, x1, x2, x3, inv, seed, block, c);
        u32 w = 0;
        w = push_byte(w, c[0]);
        w = push_byte(w, c[1]);
        w = push_byte(w, c[2]);
        w = push_byte(w, c[3]);
        return w;
    }
}

// The four 8-bit codes of a word as fp32 values.
template <bool FP>
__device__ __forceinline__ void decode4_bytes(u32 w, float (&q)[4])
{
    if (FP) {
        q[0] = __builtin_amdgcn_cvt_f32_fp8((int)w, 0);
        q[1] = __builtin_amdgcn_cvt_f32_fp8((int)w, 1);
        q[2] = __builtin_amdgcn_cvt_f32_fp8((int)w, 2);
        q[3] = __builtin_amdgcn_cvt_f32_fp8((int)w, 3);
    } else {
        q[0] = byte_to_f32(w, 0);
        q[1] = byte_to_f32(w, 1);
        q[2] = byte_to_f32(w, 2);
        q[3] = byte_to_f32(w, 3);
    }
}

// Eight fp32 values times inv -> one word of E2M1 nibbles, element 0 in bits 0-3.
__device__ __forceinline__ u32 encode8_e2m1(const float (&f)[8], float inv)
{
    u32 p = 0;
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __fmul_rn(f[0], inv), __fmul_rn(f[1], inv), 1.0f, 0);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __fmul_rn(f[2], inv), __fmul_rn(f[3], inv), 1.0f, 1);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __fmul_rn(f[4], inv), __fmul_rn(f[5], inv), 1.0f, 2);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __fmul_rn(f[6], inv), __fmul_rn(f[7], inv), 1.0f, 3);
    return p;
}

// The eight E2M1 nibbles of a word as fp32 values.
__device__ __forceinline__ void decode8_e2m1(u32 w, float (&q)[8])
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 0);
    const f32x2 b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 1);
    const f32x2 c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 2);
    const f32x2 d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 3);
    q[0] = a[0]; q[1] = a[1]; q[2] = b[0]; q[3] = b[1];
    q[4] = c[0]; q[5] = c[1]; q[6] = d[0]; q[7] = d[1];
}

__device__ __forceinline__ u32 pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);   // round to nearest even
    return __builtin_bit_cast(u32, h);
}


// A 16-byte vector of 8 bf16 values -> fp32; returns the bit pattern of the largest magnitude.
__device__ __forceinline__ u32 unpack8_bf16(const u32x4& v, float (&f)[8])
{
    u32 m = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const u32 w = v[j];
        f[2 * j] = as_f32(w << 16);
        f[2 * j + 1] = as_f32(w & 0xFFFF0000u);
        m = umax(m, umax((w << 16) & 0x7FFFFFFFu, w & 0x7FFF0000u));
    }
    return m;
}

// Quantize the 8 elements a lane owns and store them.  amax_bits is the abs-max of the
// lane's whole group (already reduced across its GROUP/8 lanes); vi is the lane's vector
// index in the tensor of n_vec vectors.  Every lane must call this (the caller reduces
// across lanes first); `valid` gates the stores.
template <int BITS, int GROUP, bool FP, bool NTS, bool SR = false>
__device__ __forceinline__ void quantize_store8(const float (&f)[8], u32 amax_bits, int64_t vi,
                                                int64_t n_vec, bool valid, void* codes,
                                                float* scales, u32 seed = 0)
{
    static_assert(!FP || BITS == 4, "the floating-point activation code book is E2M1");
    static_assert(!(FP && SR), "stochastic rounding is defined for the integer grids");
    constexpr int LANES = GROUP / 8;
    constexpr int QMAX = FP ? 6 : (1 << (BITS - 1)) - 1;   // largest code magnitude
    float scale, inv;
    const bool keep = scale_and_inv<QMAX>(amax_bits, scale, inv);
    if (!valid) return;
    if constexpr (FP) {
        const u32 p = encode8_e2m1(f, inv);
        st<NTS>((u32*)codes + vi, keep ? p : 0u);   // no signed zeros left in a zeroed group
    } else {
        // the lane's elements are 8*vi .. 8*vi+7: two blocks of four
        u32 c[8];
        {
            u32 lo[4], hi[4];
            codes4<SR, QMAX>(f[0], f[1], f[2], f[3], inv, seed, 2 * vi, lo);
            codes4<SR, QMAX>(f[4], f[5], f[6], f[7], inv, seed, 2 * vi + 1, hi);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = lo[j];
                c[4 + j] = hi[j];
            }
        }
        if constexpr (BITS == 4) {
            u32 p = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) p = push_nibble(p, c[j]);
            st<NTS>((u32*)codes + vi, keep ? p : 0u);
        } else if constexpr (BITS == 5 || BITS == 6) {
            u32 p = 0, h = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                p = push_nibble(p, c[j]);
                h = __builtin_amdgcn_alignbit(c[j] >> 4, h, BITS - 4);  // bits 4.. of the code
            }
            h = keep ? h : 0u;
            st<NTS>((u32*)codes + vi, keep ? p : 0u);
            uint8_t* high = (uint8_t*)codes + n_vec * 4;
            if constexpr (BITS == 5)
                st<NTS>(high + vi, (uint8_t)(h >> 24));
            else
                st<NTS>((uint16_t*)high + vi, (uint16_t)(h >> 16));
        } else {
            u32 p0 = 0, p1 = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) p0 = push_byte(p0, c[j]);
#pragma unroll
            for (int j = 4; j < 8; ++j) p1 = push_byte(p1, c[j]);
            st<NTS>((u32x2*)codes + vi, u32x2{keep ? p0 : 0u, keep ? p1 : 0u});
        }
    }
    if ((vi & (LANES - 1)) == 0) st<NTS>(scales + vi / LANES, scale);
}

// The stored codes of the 8 elements a lane owns, as loaded.  4/5/6-bit: lo = the nibble
// word, hi = the lane's field of high bits.  8-bit: the two code words, kept as the one
// 64-bit integer the load fills (copying its halves out right after the load, or keeping
// it as a two-element vector that the compiler splits, makes the lane wait for the data
// before it can issue its next load).
// The high-bit field keeps the width it is loaded with: widening it to 32 bits where it is
// loaded is an operation on the loaded value, which the compiler places right behind the
// load -- and the lane then waits there for the data instead of where it decodes them.
template <int BITS>
struct Codes8 {
    u32 lo = 0;
};
template <>
struct Codes8<5> {
    u32 lo = 0;
    uint8_t hi = 0;
};
template <>
struct Codes8<6> {
    u32 lo = 0;
    uint16_t hi = 0;
};
template <>
struct Codes8<8> {
    uint64_t w = 0;
};

// Marks a point where a loaded value must have arrived: the compiler places the wait for
// its load before this point (an empty statement that takes the value in a register).
__device__ __forceinline__ void need_now(float v) { asm volatile("" ::"v"(v)); }
__device__ __forceinline__ void need_now(u32 v) { asm volatile("" ::"v"(v)); }
__device__ __forceinline__ void need_now(uint64_t v) { asm volatile("" ::"v"(v)); }
__device__ __forceinline__ void need_now(const u32x4& v) { asm volatile("" ::"v"(v)); }
template <int BITS>
__device__ __forceinline__ void need_now(const Codes8<BITS>& c)
{
    if constexpr (BITS == 8) {
        asm volatile("" ::"v"(c.w));
    } else {
        asm volatile("" ::"v"(c.lo));
        if constexpr (BITS != 4) asm volatile("" ::"v"((u32)c.hi));
    }
}

template <int BITS, bool NT>
__device__ __forceinline__ Codes8<BITS> load_codes8(const void* codes, int64_t n_vec, int64_t vi)
{
    Codes8<BITS> c;
    if constexpr (BITS == 8) {
        c.w = ld<NT>((const uint64_t*)codes + vi);
    } else {
        c.lo = ld<NT>((const u32*)codes + vi);
        const uint8_t* high = (const uint8_t*)codes + n_vec * 4;
        if constexpr (BITS == 5) c.hi = ld<NT>(high + vi);
        if constexpr (BITS == 6) c.hi = ld<NT>((const uint16_t*)high + vi);
    }
    return c;
}

template <int BITS>
__device__ __forceinline__ float decode8(const Codes8<BITS>& c, int j)
{
    if constexpr (BITS == 8) {
        return byte_to_f32(j < 4 ? (u32)c.w : (u32)(c.w >> 32), j & 3);
    } else if constexpr (BITS == 4) {
        return (float)(int)__builtin_amdgcn_sbfe((int)c.lo, 4 * j, 4);
    } else {
        const int h = (int)__builtin_amdgcn_sbfe((int)(u32)c.hi, (BITS - 4) * j, BITS - 4);
        return (float)(int)(((u32)h << 4) | __builtin_amdgcn_ubfe(c.lo, 4 * j, 4));
    }
}

// The lane's eight 4-, 5- or 6-bit codes as unsigned bytes code + 2^(BITS-1), the even
// elements in the four bytes of `even`, the odd ones in `odd`: a handful of word-wide
// operations instead of two to four per element, after which v_cvt_f32_ubyte<k> turns a byte
// into a float in one operation.
//   4 bits: flipping the top bit of every nibble adds 8 to the two's-complement code.
//   5 bits: the high-bit byte is flipped the same way, then its even (odd) bits are spread to
//           bit 4 of the four bytes by one 24-bit multiply: bit 2k times
//           2^4 + 2^10 + 2^16 + 2^22 puts a copy at 8k + 4; the other copies and the carries of
//           colliding copies land on bits the mask removes.
//   6 bits: the two high bits per element are spread by two shift-or-mask steps
//           (4-bit spacing -> 8-bit spacing), then shifted above the nibble.
template <int BITS>
__device__ __forceinline__ void biased_code_bytes(const Codes8<BITS>& c, u32& even, u32& odd)
{
    static_assert(BITS == 4 || BITS == 5 || BITS == 6, "8-bit codes are bytes already");
    if constexpr (BITS == 4) {
        const u32 w = c.lo ^ 0x88888888u;
        even = w & 0x0F0F0F0Fu;
        odd = (w >> 4) & 0x0F0F0F0Fu;
    } else if constexpr (BITS == 5) {
        const u32 h = (u32)c.hi ^ 0xFFu;
        const u32 he = __umul24(h & 0x55u, 0x410410u);   // bits 0,2,4,6 -> 4,12,20,28
        const u32 ho = __umul24(h & 0xAAu, 0x208208u);   // bits 1,3,5,7 -> 4,12,20,28
        even = (he & 0x10101010u) | (c.lo & 0x0F0F0F0Fu);
        odd = (ho & 0x10101010u) | ((c.lo >> 4) & 0x0F0F0F0Fu);
    } else {
        const u32 h = (u32)c.hi ^ 0xAAAAu;
        u32 he = h & 0x3333u, ho = (h >> 2) & 0x3333u;                   // fields 4 bits apart
        he = (he | (he << 8)) & 0x00FF00FFu;
        ho = (ho | (ho << 8)) & 0x00FF00FFu;
        he = (he | (he << 4)) & 0x03030303u;                             // fields 8 bits apart
        ho = (ho | (ho << 4)) & 0x03030303u;
        even = (he << 4) | (c.lo & 0x0F0F0F0Fu);
        odd = (ho << 4) | ((c.lo >> 4) & 0x0F0F0F0Fu);
    }
}

// Unsigned byte K of a word as a float (the compiler selects v_cvt_f32_ubyte<K>).
template <int K>
__device__ __forceinline__ float ubyte_to_f32(u32 w)
{
    return (float)((w >> (8 * K)) & 0xFFu);
}

// x' = bf16(code * scale) for the lane's 8 elements, as four words of two bf16 each
// (element 2k in the low half of word k).  FP: the codes are E2M1 nibbles.
// 5- and 6-bit codes go through their biased bytes u = code + 2^(BITS-1):
// fma(u, scale, -2^(BITS-1) * scale) rounds the exact value code * scale once, like the
// product itself (the subtrahend is exact, a power of two times the scale), so x' is the
// bit pattern agoq_act_dequant produces -- except that a zero scale yields +0 where the
// product of a negative code would be -0, which no consumer of these helpers can tell apart
// (sums of squares, and layer outputs compared by magnitude).
template <int BITS, bool FP = false>
__device__ __forceinline__ void dequant8_packed(const Codes8<BITS>& c, float scale, u32 (&w)[4])
{
    static_assert(!FP || BITS == 4, "the floating-point activation code book is E2M1");
    float x[8];
    if constexpr (FP) {
        float q[8];
        decode8_e2m1(c.lo, q);
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = __fmul_rn(q[j], scale);
    } else if constexpr (BITS == 8 || BITS == 4) {
        // one or two operations per element already (sign-extending byte select; bit-field
        // extract + convert): the byte route measured no shorter for 4-bit codes
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = __fmul_rn(decode8<BITS>(c, j), scale);
    } else {
        u32 even, odd;
        biased_code_bytes<BITS>(c, even, odd);
        const float off = __fmul_rn(-(float)(1 << (BITS - 1)), scale);
        x[0] = __fmaf_rn(ubyte_to_f32<0>(even), scale, off);
        x[1] = __fmaf_rn(ubyte_to_f32<0>(odd), scale, off);
        x[2] = __fmaf_rn(ubyte_to_f32<1>(even), scale, off);
        x[3] = __fmaf_rn(ubyte_to_f32<1>(odd), scale, off);
        x[4] = __fmaf_rn(ubyte_to_f32<2>(even), scale, off);
        x[5] = __fmaf_rn(ubyte_to_f32<2>(odd), scale, off);
        x[6] = __fmaf_rn(ubyte_to_f32<3>(even), scale, off);
        x[7] = __fmaf_rn(ubyte_to_f32<3>(odd), scale, off);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = pack_bf16x2(x[2 * k], x[2 * k + 1]);
}

// The same as fp32 values.
template <int BITS, bool FP = false>
__device__ __forceinline__ void dequant8_bf16(const Codes8<BITS>& c, float scale, float (&x)[8])
{
    u32 w[4];
    dequant8_packed<BITS, FP>(c, scale, w);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        x[2 * k] = as_f32(w[k] << 16);
        x[2 * k + 1] = as_f32(w[k] & 0xFFFF0000u);
    }
}

// Sum over the wavefront, result in every lane: DPP within rows of 16, then the
// row-swap and half-swap lane permutes.
__device__ __forceinline__ float wave_sum(float v)
{
    v += as_f32((u32)__builtin_amdgcn_update_dpp(0, (int)as_u32(v), kDppXor1, 0xF, 0xF, false));
    v += as_f32((u32)__builtin_amdgcn_update_dpp(0, (int)as_u32(v), kDppXor2, 0xF, 0xF, false));
    v += as_f32((u32)__builtin_amdgcn_update_dpp(0, (int)as_u32(v), kDppHalfMirror, 0xF, 0xF, false));
    v += as_f32((u32)__builtin_amdgcn_update_dpp(0, (int)as_u32(v), kDppMirror, 0xF, 0xF, false));
    auto a = __builtin_amdgcn_permlane16_swap(as_u32(v), as_u32(v), false, false);
    v = as_f32(a[0]) + as_f32(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(as_u32(v), as_u32(v), false, false);
    return as_f32(b[0]) + as_f32(b[1]);
}

// ---- host side ------------------------------------------------------------------------

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline int check_common(int64_t numel, int group)
{
    if (group != 64 && group != 128) return AGOQ_ERR_GROUP;
    if (numel <= 0 || numel % group != 0) return AGOQ_ERR_SHAPE;
    return AGOQ_OK;
}

// Enqueue one kernel and report THIS launch's status: the return value of the launch call
// itself.  An error that an earlier, unrelated HIP call of the caller left behind in the
// runtime's per-thread state is neither reported as this call's nor cleared.
template <typename... Params, typename... Args>
inline int launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                  Args... args)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<std::remove_cv_t<Params>...> held(static_cast<std::remove_cv_t<Params>>(args)...);
    return std::apply(
        [&](auto&... value) {
            void* slots[] = {static_cast<void*>(&value)...};
            return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, slots, lds_bytes,
                                   stream) == hipSuccess
                       ? AGOQ_OK
                       : AGOQ_ERR_HIP;
        },
        held);
}

// Calls f(std::integral_constant<int, BITS>, std::integral_constant<int, GROUP>) for the
// run-time pair (bits in {4, 5, 6, 8} and group in {64, 128}, already validated).
template <typename F>
inline int dispatch_bits_group(int bits, int group, F&& f)
{
    auto with_group = [&](auto b) {
        return group == 128 ? f(b, std::integral_constant<int, 128>{}) : f(b, std::integral_constant<int, 64>{});
    };
    switch (bits) {
    case 4: return with_group(std::integral_constant<int, 4>{});
    case 5: return with_group(std::integral_constant<int, 5>{});
    case 6: return with_group(std::integral_constant<int, 6>{});
    default: return with_group(std::integral_constant<int, 8>{});
    }
}

inline unsigned blocks_for(int64_t items, int per_block)
{
    return (unsigned)((items + per_block - 1) / per_block);
}

// Compute units of the current device (cached per device ordinal; threads that race on
// the first call all store the same value).
inline int compute_units()
{
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int cus = cached[dev].load(std::memory_order_relaxed);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            cus = 256;
        cached[dev].store(cus, std::memory_order_relaxed);
    }
    return cus;
}

// True when a one-shot grid of `block`-thread workgroups with `unroll` vectors per lane needs
// at most num/den rounds of the chip (2048 lanes resident per compute unit for these
// small-register kernels); 1/1 = the whole grid is resident at once.
inline bool fits_rounds(int64_t n_vec, int block, int unroll, int num, int den)
{
    const int64_t capacity = (int64_t)compute_units() * (2048 / block);
    const int64_t blocks = (n_vec + (int64_t)block * unroll - 1) / ((int64_t)block * unroll);
    return blocks * den <= capacity * num;
}

}  // namespace

#endif  // AGOQ_DEVICE_HPP
