// HIP kernels and C ABI of the AGoQ quantization hot path for gfx950 (MI355X).
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

#include "agoq.h"

namespace {

typedef uint32_t u32;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- launch shapes and cache hints, per kernel (measured on MI355X) ------------------
// Each macro can be overridden on the compiler command line for tuning sweeps.
#ifndef AGOQ_AQ_BLOCK          // activation quantize
#define AGOQ_AQ_BLOCK 128
#endif
#ifndef AGOQ_AQ_UNROLL         // 16-byte vectors per lane: 1, 2 or 4
#define AGOQ_AQ_UNROLL 2
#endif
#ifndef AGOQ_AQ_NTL
#define AGOQ_AQ_NTL 1
#endif
#ifndef AGOQ_AQ_NTS
#define AGOQ_AQ_NTS 1
#endif
#ifndef AGOQ_DQ_BLOCK          // activation dequantize
#define AGOQ_DQ_BLOCK 512
#endif
#ifndef AGOQ_DQ_FORCE_UNROLL   // 0 = chosen per launch; else 1, 2 or 4
#define AGOQ_DQ_FORCE_UNROLL 0
#endif
#ifndef AGOQ_DQ_NTC            // code loads
#define AGOQ_DQ_NTC 1
#endif
#ifndef AGOQ_DQ_NTSC           // scale loads
#define AGOQ_DQ_NTSC 0
#endif
#ifndef AGOQ_DQ_NTS
#define AGOQ_DQ_NTS 1
#endif
#ifndef AGOQ_GQ_BLOCK          // gradient quantize
#define AGOQ_GQ_BLOCK 256
#endif
#ifndef AGOQ_GQ_UNROLL
#define AGOQ_GQ_UNROLL 1
#endif
#ifndef AGOQ_GQ_NTL
#define AGOQ_GQ_NTL 1
#endif
#ifndef AGOQ_GQ_NTS
#define AGOQ_GQ_NTS 1
#endif
#ifndef AGOQ_RD_BLOCK          // reduce + requantize
#define AGOQ_RD_BLOCK 512
#endif
#ifndef AGOQ_RD_NTC
#define AGOQ_RD_NTC 1
#endif
#ifndef AGOQ_RD_NTSC
#define AGOQ_RD_NTSC 1
#endif
#ifndef AGOQ_RD_NTS
#define AGOQ_RD_NTS 1
#endif

#ifndef AGOQ_GD_BLOCK          // gradient dequantize
#define AGOQ_GD_BLOCK 512
#endif
#ifndef AGOQ_GD_UNROLL
#define AGOQ_GD_UNROLL 1
#endif
#ifndef AGOQ_GD_NTS
#define AGOQ_GD_NTS 1
#endif

constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23
constexpr u32 kAmaxMinBits = 0x0D800000u;   // 2^-100: groups below it are stored as zeros

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

// scale and inv of a group from the bits of its abs-max.
template <int QMAX>
__device__ __forceinline__ void scale_and_inv(u32 amax_bits, float& scale, float& inv)
{
    const float amax = as_f32(amax_bits);
    const bool live = amax_bits >= kAmaxMinBits;
    const float den = live ? amax : 1.0f;
    const float s = __fdiv_rn(amax, (float)QMAX);
    const float r = __fdiv_rn((float)QMAX, den);
    scale = live ? s : 0.0f;
    inv = live ? r : 0.0f;
}

// round(x * inv) as the low bits of the returned word (two's complement).
__device__ __forceinline__ u32 code_bits(float x, float inv)
{
    return as_u32(__fadd_rn(__fmul_rn(x, inv), kRoundMagic));
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

// Four fp32 values times inv -> one word of 8-bit codes, element 0 in the low byte.
template <bool FP>
__device__ __forceinline__ u32 encode4_bytes(float x0, float x1, float x2, float x3, float inv)
{
    if (FP) {
        int w = 0;
        w = __builtin_amdgcn_cvt_pk_fp8_f32(__fmul_rn(x0, inv), __fmul_rn(x1, inv), w, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(__fmul_rn(x2, inv), __fmul_rn(x3, inv), w, true);
        return (u32)w;
    }
    u32 w = 0;
    w = push_byte(w, code_bits(x0, inv));
    w = push_byte(w, code_bits(x1, inv));
    w = push_byte(w, code_bits(x2, inv));
    w = push_byte(w, code_bits(x3, inv));
    return w;
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

// ---------------------------------------------------------------------------
// Activation quantize: bf16 -> 4-, 5-, 6- or 8-bit codes + fp32 scale per group.
// One lane owns 8 consecutive elements (one 16-byte load) of a group;
// GROUP/8 consecutive lanes own a group.  5- and 6-bit codes go to two planes:
// the low nibbles exactly where 4-bit codes would go, the remaining high bits
// (one byte or two bytes per lane) to a second plane that starts n_vec*4 bytes in.
// ---------------------------------------------------------------------------
template <int BITS, int GROUP, int UNROLL, bool FP = false>
__global__ __launch_bounds__(AGOQ_AQ_BLOCK) void act_quant_kernel(const u32x4* __restrict__ x,
                                                           int64_t n_vec, void* __restrict__ codes,
                                                           float* __restrict__ scales)
{
    static_assert(!FP || BITS == 4, "the floating-point activation code book is E2M1");
    constexpr int LANES = GROUP / 8;
    constexpr int QMAX = FP ? 6 : (1 << (BITS - 1)) - 1;   // largest code magnitude
    constexpr int kBlock = AGOQ_AQ_BLOCK;
    constexpr bool NTL = AGOQ_AQ_NTL, NTS = AGOQ_AQ_NTS;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;

    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        v[u] = u32x4{0, 0, 0, 0};
        if (vi < n_vec) v[u] = ld<NTL>(x + vi);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        float f[8];
        u32 m = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32 w = v[u][j];
            f[2 * j] = as_f32(w << 16);
            f[2 * j + 1] = as_f32(w & 0xFFFF0000u);
            m = umax(m, umax((w << 16) & 0x7FFFFFFFu, w & 0x7FFF0000u));
        }
        m = group_max_bits<LANES>(m);
        float scale, inv;
        scale_and_inv<QMAX>(m, scale, inv);
        if (vi < n_vec) {
            if (FP) {
                const u32 p = encode8_e2m1(f, inv);
                st<NTS>((u32*)codes + vi, scale != 0.0f ? p : 0u);   // dead group: no signed zeros
            } else if (BITS == 4) {
                u32 p = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) p = push_nibble(p, code_bits(f[j], inv));
                st<NTS>((u32*)codes + vi, p);
            } else if (BITS == 5 || BITS == 6) {
                u32 p = 0, h = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const u32 c = code_bits(f[j], inv);
                    p = push_nibble(p, c);
                    h = __builtin_amdgcn_alignbit(c >> 4, h, BITS - 4);  // bits 4.. of the code
                }
                st<NTS>((u32*)codes + vi, p);
                uint8_t* high = (uint8_t*)codes + n_vec * 4;
                if (BITS == 5)
                    st<NTS>(high + vi, (uint8_t)(h >> 24));
                else
                    st<NTS>((uint16_t*)high + vi, (uint16_t)(h >> 16));
            } else {
                u32 p0 = 0, p1 = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) p0 = push_byte(p0, code_bits(f[j], inv));
#pragma unroll
                for (int j = 4; j < 8; ++j) p1 = push_byte(p1, code_bits(f[j], inv));
                st<NTS>((u32x2*)codes + vi, u32x2{p0, p1});
            }
            if ((threadIdx.x & (LANES - 1)) == 0) st<NTS>(scales + vi / LANES, scale);
        }
    }
}

// ---------------------------------------------------------------------------
// Activation dequantize: codes + scales -> bf16.  One lane produces 8 elements
// (one 16-byte store).
// ---------------------------------------------------------------------------
template <int BITS, int GROUP, int UNROLL, bool FP = false>
__global__ __launch_bounds__(AGOQ_DQ_BLOCK) void act_dequant_kernel(const void* __restrict__ codes,
                                                             const float* __restrict__ scales,
                                                             int64_t n_vec, u32x4* __restrict__ y)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = AGOQ_DQ_BLOCK;
    constexpr bool NTC = AGOQ_DQ_NTC, NTSC = AGOQ_DQ_NTSC, NTS = AGOQ_DQ_NTS;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;

    u32x2 c[UNROLL];    // 8-bit: both words are codes; 5/6-bit: [0] nibbles, [1] high bits
    float s[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        c[u] = u32x2{0, 0};
        s[u] = 0.0f;
        if (vi < n_vec) {
            if (BITS == 8) {
                c[u] = ld<NTC>((const u32x2*)codes + vi);
            } else {
                c[u][0] = ld<NTC>((const u32*)codes + vi);
                const uint8_t* high = (const uint8_t*)codes + n_vec * 4;
                if (BITS == 5) c[u][1] = ld<NTC>(high + vi);
                if (BITS == 6) c[u][1] = ld<NTC>((const uint16_t*)high + vi);
            }
            s[u] = ld<NTSC>(scales + vi / LANES);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        float f[8];
        float fpq[8];
        if (FP) decode8_e2m1(c[u][0], fpq);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float q;
            if (FP) {
                q = fpq[j];
            } else if (BITS == 4) {
                q = (float)(int)__builtin_amdgcn_sbfe((int)c[u][0], 4 * j, 4);  // the builtin returns unsigned
            } else if (BITS == 8) {
                q = byte_to_f32(c[u][j >> 2], j & 3);
            } else {
                // signed high field * 16 + unsigned low nibble
                const int hi = (int)__builtin_amdgcn_sbfe((int)c[u][1], (BITS - 4) * j, BITS - 4);
                const u32 lo = __builtin_amdgcn_ubfe(c[u][0], 4 * j, 4);
                q = (float)(int)(((u32)hi << 4) | lo);
            }
            f[j] = __fmul_rn(q, s[u]);
        }
        if (vi < n_vec)
            st<NTS>(y + vi, u32x4{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                                  pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7])});
    }
}

// ---------------------------------------------------------------------------
// Gradient quantize: fp32 -> int8 codes + fp32 scale per group.
// 16 lanes (one DPP row) own a group; a lane holds VPL 16-byte vectors of it,
// vector p of lane l being elements [p*64 + 4l, p*64 + 4l + 4) of the group, so
// each load instruction reads whole 256-byte runs.
// ---------------------------------------------------------------------------
template <int GROUP, int UNROLL, bool FP = false>
__global__ __launch_bounds__(AGOQ_GQ_BLOCK) void grad_quant_kernel(const f32x4* __restrict__ g,
                                                            int64_t n_groups,
                                                            u32* __restrict__ codes,
                                                            float* __restrict__ scales)
{
    constexpr int VPL = GROUP / 64;   // vectors per lane: 1 (group 64) or 2 (group 128)
    constexpr int VPG = GROUP / 4;    // vectors per group
    constexpr int kBlock = AGOQ_GQ_BLOCK;
    constexpr bool NTL = AGOQ_GQ_NTL, NTS = AGOQ_GQ_NTS;
    const int lane16 = threadIdx.x & 15;
    const int64_t slot = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;

    f32x4 v[UNROLL][VPL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t grp = (slot + (int64_t)u * kBlock) >> 4;
#pragma unroll
        for (int p = 0; p < VPL; ++p) {
            v[u][p] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (grp < n_groups) v[u][p] = ld<NTL>(g + grp * VPG + p * 16 + lane16);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t grp = (slot + (int64_t)u * kBlock) >> 4;
        u32 m = 0;
#pragma unroll
        for (int p = 0; p < VPL; ++p)
#pragma unroll
            for (int j = 0; j < 4; ++j) m = umax(m, as_u32(v[u][p][j]) & 0x7FFFFFFFu);
        m = group_max_bits<16>(m);
        float scale, inv;
        scale_and_inv<FP ? 448 : 127>(m, scale, inv);
        if (grp < n_groups) {
#pragma unroll
            for (int p = 0; p < VPL; ++p) {
                u32 w = encode4_bytes<FP>(v[u][p][0], v[u][p][1], v[u][p][2], v[u][p][3], inv);
                if (FP && scale == 0.0f) w = 0;               // dead group: no signed zeros
                st<NTS>(codes + grp * VPG + p * 16 + lane16, w);
            }
            if (lane16 == 0) st<NTS>(scales + grp, scale);
        }
    }
}

// ---------------------------------------------------------------------------
// Local reduce of K int8 chunks + requantize.  One lane owns 16 consecutive
// elements (one 16-byte load per chunk, one 16-byte store); GROUP/16 lanes own
// a group.  acc = fma(code_k, scale_k, acc) for k = 0..K-1 in that order.
// KT > 0: K known at compile time (all loads hoisted); KT == 0: run-time K.
// ---------------------------------------------------------------------------
template <int GROUP, bool FP = false>
__device__ __forceinline__ void reduce_finish(const float (&acc)[16], int64_t vi,
                                              bool valid, u32x4* __restrict__ out_codes,
                                              float* __restrict__ out_scales)
{
    constexpr int LANES = GROUP / 16;
    u32 m = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) m = umax(m, as_u32(acc[j]) & 0x7FFFFFFFu);
    m = group_max_bits<LANES>(m);
    float scale, inv;
    scale_and_inv<FP ? 448 : 127>(m, scale, inv);
    if (valid) {
        u32x4 w = {0, 0, 0, 0};
#pragma unroll
        for (int d = 0; d < 4; ++d)
            w[d] = encode4_bytes<FP>(acc[4 * d], acc[4 * d + 1], acc[4 * d + 2], acc[4 * d + 3], inv);
        if (FP && scale == 0.0f) w = u32x4{0, 0, 0, 0};       // dead group: no signed zeros
        st<AGOQ_RD_NTS>(out_codes + vi, w);
        if ((threadIdx.x & (LANES - 1)) == 0) st<AGOQ_RD_NTS>(out_scales + vi / LANES, scale);
    }
}

template <bool FP = false>
__device__ __forceinline__ void reduce_term(float (&acc)[16], const u32x4& c, float s)
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        float q[4];
        decode4_bytes<FP>(c[d], q);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[4 * d + j] = __fmaf_rn(q[j], s, acc[4 * d + j]);
    }
}

template <int GROUP, int KT, bool FP = false>
__global__ __launch_bounds__(AGOQ_RD_BLOCK) void grad_reduce_kernel(const int8_t* __restrict__ in_codes,
                                                             int64_t stride_codes,
                                                             const float* __restrict__ in_scales,
                                                             int64_t stride_scales, int K,
                                                             int64_t n_vec,
                                                             u32x4* __restrict__ out_codes,
                                                             float* __restrict__ out_scales)
{
    constexpr int LANES = GROUP / 16;
    constexpr int kBlock = AGOQ_RD_BLOCK;
    constexpr bool NTC = AGOQ_RD_NTC, NTSC = AGOQ_RD_NTSC;
    const int64_t vi = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool valid = vi < n_vec;
    const int64_t vc = valid ? vi : 0;      // out-of-range lanes read element 0, store nothing
    const int64_t grp = vc / LANES;
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0f;

    if (KT > 0) {
        u32x4 c[KT > 0 ? KT : 1];
        float s[KT > 0 ? KT : 1];
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            c[k] = ld<NTC>((const u32x4*)(in_codes + (int64_t)k * stride_codes) + vc);
            s[k] = ld<NTSC>(in_scales + (int64_t)k * stride_scales + grp);
        }
#pragma unroll
        for (int k = 0; k < KT; ++k) reduce_term<FP>(acc, c[k], s[k]);
    } else {
        int k = 0;
        for (; k + 4 <= K; k += 4) {
            u32x4 c[4];
            float s[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                c[t] = ld<NTC>((const u32x4*)(in_codes + (int64_t)(k + t) * stride_codes) + vc);
                s[t] = ld<NTSC>(in_scales + (int64_t)(k + t) * stride_scales + grp);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) reduce_term<FP>(acc, c[t], s[t]);
        }
        for (; k < K; ++k) {
            const u32x4 c = ld<NTC>((const u32x4*)(in_codes + (int64_t)k * stride_codes) + vc);
            const float s = ld<NTSC>(in_scales + (int64_t)k * stride_scales + grp);
            reduce_term<FP>(acc, c, s);
        }
    }
    reduce_finish<GROUP, FP>(acc, vi, valid, out_codes, out_scales);
}

// ---------------------------------------------------------------------------
// Local gradient accumulation: stored int8 gradient (+ scales) plus a new
// micro-batch gradient -> int8 (+ scales).  acc = fma(code, scale, g_new) in fp32,
// then the group is quantized to 8 bits.  May run in place: a group is read in
// full by the lanes that own it before any of them stores, and no other lane
// touches it, so the output may alias the stored gradient.
//   fp32 addend: lane layout of grad_quant_kernel (one DPP row per group).
//   bf16 addend: lane layout of act_quant_kernel (8 elements per lane).
// ---------------------------------------------------------------------------
template <int GROUP, int UNROLL>
__global__ __launch_bounds__(AGOQ_GQ_BLOCK) void grad_accumulate_f32_kernel(
    const u32* main_codes, const float* main_scales, const f32x4* __restrict__ g_new,
    int64_t n_groups, u32* out_codes, float* out_scales)
{
    constexpr int VPL = GROUP / 64;
    constexpr int VPG = GROUP / 4;
    constexpr int kBlock = AGOQ_GQ_BLOCK;
    const int lane16 = threadIdx.x & 15;
    const int64_t slot = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;

    f32x4 v[UNROLL][VPL];
    u32 c[UNROLL][VPL];
    float s[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t grp = (slot + (int64_t)u * kBlock) >> 4;
        s[u] = 0.0f;
        if (grp < n_groups) s[u] = ld<true>(main_scales + grp);
#pragma unroll
        for (int p = 0; p < VPL; ++p) {
            v[u][p] = f32x4{0.f, 0.f, 0.f, 0.f};
            c[u][p] = 0;
            if (grp < n_groups) {
                v[u][p] = ld<true>(g_new + grp * VPG + p * 16 + lane16);
                c[u][p] = ld<true>(main_codes + grp * VPG + p * 16 + lane16);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t grp = (slot + (int64_t)u * kBlock) >> 4;
        float acc[VPL][4];
        u32 m = 0;
#pragma unroll
        for (int p = 0; p < VPL; ++p)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[p][j] = __fmaf_rn(byte_to_f32(c[u][p], j), s[u], v[u][p][j]);
                m = umax(m, as_u32(acc[p][j]) & 0x7FFFFFFFu);
            }
        m = group_max_bits<16>(m);
        float scale, inv;
        scale_and_inv<127>(m, scale, inv);
        if (grp < n_groups) {
#pragma unroll
            for (int p = 0; p < VPL; ++p) {
                u32 w = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) w = push_byte(w, code_bits(acc[p][j], inv));
                st<true>(out_codes + grp * VPG + p * 16 + lane16, w);
            }
            if (lane16 == 0) st<true>(out_scales + grp, scale);
        }
    }
}

template <int GROUP, int UNROLL>
__global__ __launch_bounds__(AGOQ_AQ_BLOCK) void grad_accumulate_bf16_kernel(
    const u32x2* main_codes, const float* main_scales, const u32x4* __restrict__ g_new,
    int64_t n_vec, u32x2* out_codes, float* out_scales)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = AGOQ_AQ_BLOCK;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;

    u32x4 v[UNROLL];
    u32x2 c[UNROLL];
    float s[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        v[u] = u32x4{0, 0, 0, 0};
        c[u] = u32x2{0, 0};
        s[u] = 0.0f;
        if (vi < n_vec) {
            v[u] = ld<true>(g_new + vi);
            c[u] = ld<true>(main_codes + vi);
            s[u] = ld<true>(main_scales + vi / LANES);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        float acc[8];
        u32 m = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const u32 w = v[u][j >> 1];
            const float g = as_f32((j & 1) ? (w & 0xFFFF0000u) : (w << 16));
            acc[j] = __fmaf_rn(byte_to_f32(c[u][j >> 2], j & 3), s[u], g);
            m = umax(m, as_u32(acc[j]) & 0x7FFFFFFFu);
        }
        m = group_max_bits<LANES>(m);
        float scale, inv;
        scale_and_inv<127>(m, scale, inv);
        if (vi < n_vec) {
            u32 p0 = 0, p1 = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) p0 = push_byte(p0, code_bits(acc[j], inv));
#pragma unroll
            for (int j = 4; j < 8; ++j) p1 = push_byte(p1, code_bits(acc[j], inv));
            st<true>(out_codes + vi, u32x2{p0, p1});
            if ((threadIdx.x & (LANES - 1)) == 0) st<true>(out_scales + vi / LANES, scale);
        }
    }
}

// ---------------------------------------------------------------------------
// Gradient dequantize: int8 codes + scales -> fp32 (what an optimizer step reads).
// One lane: 4 codes (one dword) -> one 16-byte store.
// ---------------------------------------------------------------------------
template <int GROUP, int UNROLL, bool FP = false>
__global__ __launch_bounds__(AGOQ_GD_BLOCK) void grad_dequant_kernel(const u32* __restrict__ codes,
                                                                     const float* __restrict__ scales,
                                                                     int64_t n_vec,
                                                                     f32x4* __restrict__ out)
{
    constexpr int LANES = GROUP / 4;      // lanes per group
    constexpr int kBlock = AGOQ_GD_BLOCK;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;
    u32 c[UNROLL];
    float s[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        c[u] = 0;
        s[u] = 0.0f;
        if (vi < n_vec) {
            c[u] = ld<true>(codes + vi);
            s[u] = ld<false>(scales + vi / LANES);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        f32x4 o;
        float q[4];
        decode4_bytes<FP>(c[u], q);
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = __fmul_rn(q[j], s[u]);
        if (vi < n_vec) st<AGOQ_GD_NTS>(out + vi, o);
    }
}

// ---------------------------------------------------------------------------
// Dequantize fused with the recomputation of the layer's forward (the stored tensor is
// the layer's INPUT; what the backward pass needs is recomputed from its dequantized
// value instead of being written to memory and read again).
// ---------------------------------------------------------------------------

// The stored codes of the 8 elements a lane owns.  4/5/6-bit: lo = the nibble word,
// hi = the lane's field of high bits.  8-bit: lo, hi = the two code words.
template <int BITS, bool NT>
__device__ __forceinline__ void load_codes8(const void* codes, int64_t n_vec, int64_t vi, u32& lo,
                                            u32& hi)
{
    if (BITS == 8) {
        const u32x2 c = ld<NT>((const u32x2*)codes + vi);
        lo = c[0];
        hi = c[1];
    } else {
        lo = ld<NT>((const u32*)codes + vi);
        hi = 0;
        const uint8_t* high = (const uint8_t*)codes + n_vec * 4;
        if (BITS == 5) hi = ld<NT>(high + vi);
        if (BITS == 6) hi = ld<NT>((const uint16_t*)high + vi);
    }
}

template <int BITS>
__device__ __forceinline__ float decode8(u32 lo, u32 hi, int j)
{
    if (BITS == 4) return (float)(int)__builtin_amdgcn_sbfe((int)lo, 4 * j, 4);
    if (BITS == 8) return byte_to_f32(j < 4 ? lo : hi, j & 3);
    const int h = (int)__builtin_amdgcn_sbfe((int)hi, (BITS - 4) * j, BITS - 4);
    return (float)(int)(((u32)h << 4) | __builtin_amdgcn_ubfe(lo, 4 * j, 4));
}

// x' = bf16(code * scale) for the lane's 8 elements, returned as fp32 values.
template <int BITS>
__device__ __forceinline__ void dequant8_bf16(u32 lo, u32 hi, float scale, float (&x)[8])
{
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
        const u32 w = pack_bf16x2(__fmul_rn(decode8<BITS>(lo, hi, j), scale),
                                  __fmul_rn(decode8<BITS>(lo, hi, j + 1), scale));
        x[j] = as_f32(w << 16);
        x[j + 1] = as_f32(w & 0xFFFF0000u);
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

// RMSNorm recompute: one workgroup of 256 lanes per row of `cols` elements
// (cols <= 2048 * VPT); the row stays in registers between the two phases.
//   r = sqrt(mean(x'^2) + eps);  y = bf16(x' * (1/r) * gamma)
constexpr int kNormBlock = 256;
template <int BITS, int GROUP, int VPT>
__global__ __launch_bounds__(kNormBlock) void act_dequant_rmsnorm_kernel(
    const void* __restrict__ codes, const float* __restrict__ scales, int64_t n_vec_total,
    int vecs_per_row, const f32x4* __restrict__ gamma, float eps, float inv_cols,
    u32x4* __restrict__ y, float* __restrict__ r_out)
{
    constexpr int LANES = GROUP / 8;
    __shared__ float wave_part[kNormBlock / 64];
    const int64_t row_vec0 = (int64_t)blockIdx.x * vecs_per_row;
    float x[VPT][8];
    float ss = 0.0f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int v = threadIdx.x + u * kNormBlock;
        u32 lo = 0, hi = 0;
        float sc = 0.0f;
        if (v < vecs_per_row) {
            const int64_t vi = row_vec0 + v;
            load_codes8<BITS, true>(codes, n_vec_total, vi, lo, hi);
            sc = ld<false>(scales + vi / LANES);
        }
        dequant8_bf16<BITS>(lo, hi, sc, x[u]);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss = __fmaf_rn(x[u][j], x[u][j], ss);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float total = 0.0f;
#pragma unroll
    for (int w = 0; w < kNormBlock / 64; ++w) total += wave_part[w];
    const float r = __fsqrt_rn(__fmaf_rn(total, inv_cols, eps));
    const float rinv = __fdiv_rn(1.0f, r);
    if (threadIdx.x == 0) r_out[blockIdx.x] = r;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int v = threadIdx.x + u * kNormBlock;
        if (v < vecs_per_row) {
            const f32x4 g0 = gamma[2 * v], g1 = gamma[2 * v + 1];
            float o[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[j] = __fmul_rn(__fmul_rn(x[u][j], rinv), g0[j]);
                o[4 + j] = __fmul_rn(__fmul_rn(x[u][4 + j], rinv), g1[j]);
            }
            st<true>(y + row_vec0 + v, u32x4{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]),
                                             pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])});
        }
    }
}

// Narrow rows (cols <= 512 * VPT, i.e. up to 4096): one wavefront per row, four rows per
// workgroup, every load of the row in flight at once, no LDS and no barrier.
template <int BITS, int GROUP, int VPT>
__global__ __launch_bounds__(kNormBlock) void act_dequant_rmsnorm_wave_kernel(
    const void* __restrict__ codes, const float* __restrict__ scales, int64_t n_vec_total,
    int64_t rows, int vecs_per_row, const f32x4* __restrict__ gamma, float eps, float inv_cols,
    u32x4* __restrict__ y, float* __restrict__ r_out)
{
    constexpr int LANES = GROUP / 8;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (kNormBlock / 64) + (threadIdx.x >> 6);
    if (row >= rows) return;                      // whole wavefronts leave together
    const int64_t row_vec0 = row * vecs_per_row;
    u32 lo[VPT], hi[VPT];
    float sc[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int v = lane + u * 64;
        lo[u] = hi[u] = 0;
        sc[u] = 0.0f;
        if (v < vecs_per_row) {
            const int64_t vi = row_vec0 + v;
            load_codes8<BITS, true>(codes, n_vec_total, vi, lo[u], hi[u]);
            sc[u] = ld<false>(scales + vi / LANES);
        }
    }
    float x[VPT][8];
    float ss = 0.0f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        dequant8_bf16<BITS>(lo[u], hi[u], sc[u], x[u]);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss = __fmaf_rn(x[u][j], x[u][j], ss);
    }
    const float total = wave_sum(ss);
    const float r = __fsqrt_rn(__fmaf_rn(total, inv_cols, eps));
    const float rinv = __fdiv_rn(1.0f, r);
    if (lane == 0) r_out[row] = r;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int v = lane + u * 64;
        if (v < vecs_per_row) {
            const f32x4 g0 = gamma[2 * v], g1 = gamma[2 * v + 1];
            float o[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[j] = __fmul_rn(__fmul_rn(x[u][j], rinv), g0[j]);
                o[4 + j] = __fmul_rn(__fmul_rn(x[u][4 + j], rinv), g1[j]);
            }
            st<true>(y + row_vec0 + v, u32x4{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]),
                                             pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])});
        }
    }
}

// SiLU & Multiply recompute: z = bf16(u' * g' * sigmoid(g')), elementwise over the two
// stored tensors (which may have different code widths).
template <int BITS_G, int BITS_U, int GROUP, int UNROLL>
__global__ __launch_bounds__(AGOQ_DQ_BLOCK) void act_dequant_silu_mul_kernel(
    const void* __restrict__ gate_codes, const float* __restrict__ gate_scales,
    const void* __restrict__ up_codes, const float* __restrict__ up_scales, int64_t n_vec,
    u32x4* __restrict__ z)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = AGOQ_DQ_BLOCK;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;
    u32 glo[UNROLL], ghi[UNROLL], ulo[UNROLL], uhi[UNROLL];
    float gs[UNROLL], us[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        glo[u] = ghi[u] = ulo[u] = uhi[u] = 0;
        gs[u] = us[u] = 0.0f;
        if (vi < n_vec) {
            load_codes8<BITS_G, true>(gate_codes, n_vec, vi, glo[u], ghi[u]);
            load_codes8<BITS_U, true>(up_codes, n_vec, vi, ulo[u], uhi[u]);
            gs[u] = ld<false>(gate_scales + vi / LANES);
            us[u] = ld<false>(up_scales + vi / LANES);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        float g[8], up[8], o[8];
        dequant8_bf16<BITS_G>(glo[u], ghi[u], gs[u], g);
        dequant8_bf16<BITS_U>(ulo[u], uhi[u], us[u], up);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float e = __expf(-g[j]);                          // may be +inf: 1/(1+inf) = 0
            const float sig = __builtin_amdgcn_rcpf(1.0f + e);
            o[j] = __fmul_rn(__fmul_rn(up[j], g[j]), sig);
        }
        if (vi < n_vec)
            st<true>(z + vi, u32x4{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]),
                                   pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])});
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline int check_common(int64_t numel, int group)
{
    if (group != 64 && group != 128) return AGOQ_ERR_GROUP;
    if (numel <= 0 || numel % group != 0) return AGOQ_ERR_SHAPE;
    return AGOQ_OK;
}

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? AGOQ_OK : AGOQ_ERR_HIP;
}

inline unsigned blocks_for(int64_t items, int per_block)
{
    return (unsigned)((items + per_block - 1) / per_block);
}

// Compute units of the current device (cached per device ordinal).
inline int compute_units()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}

// True when a one-shot grid of `block`-thread workgroups with `unroll` vectors per lane is
// resident on the chip all at once (2048 threads per compute unit for these small-register
// kernels).
inline bool fits_one_round(int64_t n_vec, int block, int unroll)
{
    const int64_t capacity = (int64_t)compute_units() * (2048 / block);
    return (n_vec + (int64_t)block * unroll - 1) / ((int64_t)block * unroll) <= capacity;
}

}  // namespace

extern "C" {

int agoq_act_quant(const void* x_bf16, int64_t numel, int group, int bits, void* codes,
                   float* scales, void* stream)
{
    if (!x_bf16 || !codes || !scales) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    const int unroll = AGOQ_AQ_UNROLL;
    const dim3 grid(blocks_for(n_vec, AGOQ_AQ_BLOCK * unroll)), block(AGOQ_AQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    const u32x4* x = (const u32x4*)x_bf16;
#define AGOQ_LAUNCH_AQ(B, G)                                                                     \
    switch (unroll) {                                                                            \
    case 4: act_quant_kernel<B, G, 4><<<grid, block, 0, st>>>(x, n_vec, codes, scales); break;   \
    case 2: act_quant_kernel<B, G, 2><<<grid, block, 0, st>>>(x, n_vec, codes, scales); break;   \
    default: act_quant_kernel<B, G, 1><<<grid, block, 0, st>>>(x, n_vec, codes, scales); break;  \
    }
    if (group == 128) {
        switch (bits) {
        case 4: AGOQ_LAUNCH_AQ(4, 128) break;
        case 5: AGOQ_LAUNCH_AQ(5, 128) break;
        case 6: AGOQ_LAUNCH_AQ(6, 128) break;
        default: AGOQ_LAUNCH_AQ(8, 128) break;
        }
    } else {
        switch (bits) {
        case 4: AGOQ_LAUNCH_AQ(4, 64) break;
        case 5: AGOQ_LAUNCH_AQ(5, 64) break;
        case 6: AGOQ_LAUNCH_AQ(6, 64) break;
        default: AGOQ_LAUNCH_AQ(8, 64) break;
        }
    }
#undef AGOQ_LAUNCH_AQ
    return launch_status();
}

int agoq_act_dequant(const void* codes, const float* scales, int64_t numel, int group, int bits,
                     void* y_bf16, void* stream)
{
    if (!codes || !scales || !y_bf16) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(codes) || misaligned(scales) || misaligned(y_bf16)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    // measured: 4-bit codes run best with four vectors per lane at every size; 8-bit codes
    // with four when the whole grid is resident at once and with one otherwise
    int unroll = AGOQ_DQ_FORCE_UNROLL;
    if (unroll == 0) unroll = (bits != 8 || fits_one_round(n_vec, AGOQ_DQ_BLOCK, 4)) ? 4 : 1;
    const dim3 grid(blocks_for(n_vec, AGOQ_DQ_BLOCK * unroll)), block(AGOQ_DQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    u32x4* y = (u32x4*)y_bf16;
#define AGOQ_LAUNCH_DQ(B, G)                                                                      \
    switch (unroll) {                                                                             \
    case 4: act_dequant_kernel<B, G, 4><<<grid, block, 0, st>>>(codes, scales, n_vec, y); break;  \
    case 2: act_dequant_kernel<B, G, 2><<<grid, block, 0, st>>>(codes, scales, n_vec, y); break;  \
    default: act_dequant_kernel<B, G, 1><<<grid, block, 0, st>>>(codes, scales, n_vec, y); break; \
    }
    if (group == 128) {
        switch (bits) {
        case 4: AGOQ_LAUNCH_DQ(4, 128) break;
        case 5: AGOQ_LAUNCH_DQ(5, 128) break;
        case 6: AGOQ_LAUNCH_DQ(6, 128) break;
        default: AGOQ_LAUNCH_DQ(8, 128) break;
        }
    } else {
        switch (bits) {
        case 4: AGOQ_LAUNCH_DQ(4, 64) break;
        case 5: AGOQ_LAUNCH_DQ(5, 64) break;
        case 6: AGOQ_LAUNCH_DQ(6, 64) break;
        default: AGOQ_LAUNCH_DQ(8, 64) break;
        }
    }
#undef AGOQ_LAUNCH_DQ
    return launch_status();
}

int agoq_grad_quant(const float* grad, int64_t numel, int group, int8_t* codes, float* scales,
                    void* stream)
{
    if (!grad || !codes || !scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(grad) || misaligned(codes) || misaligned(scales)) return AGOQ_ERR_ALIGN;
    const int64_t n_groups = numel / group;
    constexpr int U = AGOQ_GQ_UNROLL;
    const dim3 grid(blocks_for(n_groups * 16, AGOQ_GQ_BLOCK * U)), block(AGOQ_GQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    if (group == 128)
        grad_quant_kernel<128, U><<<grid, block, 0, st>>>((const f32x4*)grad, n_groups, (u32*)codes,
                                                          scales);
    else
        grad_quant_kernel<64, U><<<grid, block, 0, st>>>((const f32x4*)grad, n_groups, (u32*)codes,
                                                         scales);
    return launch_status();
}

int agoq_grad_reduce_requant(const int8_t* in_codes, int64_t chunk_stride_codes,
                             const float* in_scales, int64_t chunk_stride_scales, int K,
                             int64_t numel, int group, int8_t* out_codes, float* out_scales,
                             void* stream)
{
    if (!in_codes || !in_scales || !out_codes || !out_scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (K < 1 || K > 64) return AGOQ_ERR_K;
    if (chunk_stride_codes < numel || chunk_stride_scales < numel / group) return AGOQ_ERR_SHAPE;
    if (misaligned(in_codes) || misaligned(in_scales) || misaligned(out_codes) ||
        misaligned(out_scales) || (chunk_stride_codes & 15) != 0)
        return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 16;
    const dim3 grid(blocks_for(n_vec, AGOQ_RD_BLOCK)), block(AGOQ_RD_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    u32x4* oc = (u32x4*)out_codes;
#define AGOQ_LAUNCH_REDUCE(G, KT)                                                              \
    grad_reduce_kernel<G, KT><<<grid, block, 0, st>>>(in_codes, chunk_stride_codes, in_scales, \
                                                      chunk_stride_scales, K, n_vec, oc, out_scales)
    if (group == 128) {
        switch (K) {
        case 4: AGOQ_LAUNCH_REDUCE(128, 4); break;
        case 8: AGOQ_LAUNCH_REDUCE(128, 8); break;
        case 16: AGOQ_LAUNCH_REDUCE(128, 16); break;
        default: AGOQ_LAUNCH_REDUCE(128, 0); break;
        }
    } else {
        switch (K) {
        case 4: AGOQ_LAUNCH_REDUCE(64, 4); break;
        case 8: AGOQ_LAUNCH_REDUCE(64, 8); break;
        case 16: AGOQ_LAUNCH_REDUCE(64, 16); break;
        default: AGOQ_LAUNCH_REDUCE(64, 0); break;
        }
    }
#undef AGOQ_LAUNCH_REDUCE
    return launch_status();
}

int agoq_grad_accumulate(const int8_t* main_codes, const float* main_scales, const void* g_new,
                         int g_new_is_bf16, int64_t numel, int group, int8_t* out_codes,
                         float* out_scales, void* stream)
{
    if (!main_codes || !main_scales || !g_new || !out_codes || !out_scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(main_codes) || misaligned(main_scales) || misaligned(g_new) ||
        misaligned(out_codes) || misaligned(out_scales))
        return AGOQ_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (g_new_is_bf16) {
        const int64_t n_vec = numel / 8;
        constexpr int U = AGOQ_AQ_UNROLL;
        const dim3 grid(blocks_for(n_vec, AGOQ_AQ_BLOCK * U)), block(AGOQ_AQ_BLOCK);
        if (group == 128)
            grad_accumulate_bf16_kernel<128, U><<<grid, block, 0, st>>>(
                (const u32x2*)main_codes, main_scales, (const u32x4*)g_new, n_vec,
                (u32x2*)out_codes, out_scales);
        else
            grad_accumulate_bf16_kernel<64, U><<<grid, block, 0, st>>>(
                (const u32x2*)main_codes, main_scales, (const u32x4*)g_new, n_vec,
                (u32x2*)out_codes, out_scales);
    } else {
        const int64_t n_groups = numel / group;
        constexpr int U = AGOQ_GQ_UNROLL;
        const dim3 grid(blocks_for(n_groups * 16, AGOQ_GQ_BLOCK * U)), block(AGOQ_GQ_BLOCK);
        if (group == 128)
            grad_accumulate_f32_kernel<128, U><<<grid, block, 0, st>>>(
                (const u32*)main_codes, main_scales, (const f32x4*)g_new, n_groups,
                (u32*)out_codes, out_scales);
        else
            grad_accumulate_f32_kernel<64, U><<<grid, block, 0, st>>>(
                (const u32*)main_codes, main_scales, (const f32x4*)g_new, n_groups,
                (u32*)out_codes, out_scales);
    }
    return launch_status();
}

int agoq_grad_dequant(const int8_t* codes, const float* scales, int64_t numel, int group,
                      float* out, void* stream)
{
    if (!codes || !scales || !out) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(codes) || misaligned(scales) || misaligned(out)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 4;
    constexpr int U = AGOQ_GD_UNROLL;
    const dim3 grid(blocks_for(n_vec, AGOQ_GD_BLOCK * U)), block(AGOQ_GD_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    if (group == 128)
        grad_dequant_kernel<128, U><<<grid, block, 0, st>>>((const u32*)codes, scales, n_vec,
                                                            (f32x4*)out);
    else
        grad_dequant_kernel<64, U><<<grid, block, 0, st>>>((const u32*)codes, scales, n_vec,
                                                           (f32x4*)out);
    return launch_status();
}

int agoq_act_dequant_rmsnorm(const void* codes, const float* scales, int64_t rows, int64_t cols,
                             int group, int bits, const float* gamma, float eps, void* y_bf16,
                             float* r_out, void* stream)
{
    if (!codes || !scales || !gamma || !y_bf16 || !r_out) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (group != 64 && group != 128) return AGOQ_ERR_GROUP;
    if (rows <= 0 || rows > 0x7FFFFFFF || cols <= 0 || cols % group != 0 ||
        cols > (int64_t)kNormBlock * 8 * 8)
        return AGOQ_ERR_SHAPE;
    if (misaligned(codes) || misaligned(scales) || misaligned(gamma) || misaligned(y_bf16))
        return AGOQ_ERR_ALIGN;
    const int vecs_per_row = (int)(cols / 8);
    const int64_t n_vec_total = rows * vecs_per_row;
    const float inv_cols = 1.0f / (float)cols;
    hipStream_t st = (hipStream_t)stream;
    const f32x4* gm = (const f32x4*)gamma;
    u32x4* y = (u32x4*)y_bf16;
    if (vecs_per_row <= 64 * 8 && bits != 8) {
        // one wavefront per row (measured faster for the narrow codes; 8-bit codes need too many
        // registers per lane for it and keep the workgroup-per-row form)
        const int wvpt = vecs_per_row <= 64 * 4 ? 4 : 8;
        const dim3 wgrid((unsigned)((rows + kNormBlock / 64 - 1) / (kNormBlock / 64))), wblock(kNormBlock);
#define AGOQ_LAUNCH_NORM_WAVE(B, G)                                                               \
    if (wvpt == 4)                                                                                \
        act_dequant_rmsnorm_wave_kernel<B, G, 4><<<wgrid, wblock, 0, st>>>(codes, scales, n_vec_total, rows, vecs_per_row, gm, eps, inv_cols, y, r_out); \
    else                                                                                          \
        act_dequant_rmsnorm_wave_kernel<B, G, 8><<<wgrid, wblock, 0, st>>>(codes, scales, n_vec_total, rows, vecs_per_row, gm, eps, inv_cols, y, r_out);
        if (group == 128) {
            switch (bits) {
            case 4: AGOQ_LAUNCH_NORM_WAVE(4, 128) break;
            case 5: AGOQ_LAUNCH_NORM_WAVE(5, 128) break;
            case 6: AGOQ_LAUNCH_NORM_WAVE(6, 128) break;
            default: AGOQ_LAUNCH_NORM_WAVE(8, 128) break;
            }
        } else {
            switch (bits) {
            case 4: AGOQ_LAUNCH_NORM_WAVE(4, 64) break;
            case 5: AGOQ_LAUNCH_NORM_WAVE(5, 64) break;
            case 6: AGOQ_LAUNCH_NORM_WAVE(6, 64) break;
            default: AGOQ_LAUNCH_NORM_WAVE(8, 64) break;
            }
        }
#undef AGOQ_LAUNCH_NORM_WAVE
        return launch_status();
    }
    int vpt = 1;
    while (kNormBlock * vpt < vecs_per_row) vpt *= 2;
    const dim3 grid((unsigned)rows), block(kNormBlock);
#define AGOQ_LAUNCH_NORM(B, G)                                                                    \
    switch (vpt) {                                                                                \
    case 1: act_dequant_rmsnorm_kernel<B, G, 1><<<grid, block, 0, st>>>(codes, scales, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out); break; \
    case 2: act_dequant_rmsnorm_kernel<B, G, 2><<<grid, block, 0, st>>>(codes, scales, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out); break; \
    case 4: act_dequant_rmsnorm_kernel<B, G, 4><<<grid, block, 0, st>>>(codes, scales, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out); break; \
    default: act_dequant_rmsnorm_kernel<B, G, 8><<<grid, block, 0, st>>>(codes, scales, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out); break; \
    }
    if (group == 128) {
        switch (bits) {
        case 4: AGOQ_LAUNCH_NORM(4, 128) break;
        case 5: AGOQ_LAUNCH_NORM(5, 128) break;
        case 6: AGOQ_LAUNCH_NORM(6, 128) break;
        default: AGOQ_LAUNCH_NORM(8, 128) break;
        }
    } else {
        switch (bits) {
        case 4: AGOQ_LAUNCH_NORM(4, 64) break;
        case 5: AGOQ_LAUNCH_NORM(5, 64) break;
        case 6: AGOQ_LAUNCH_NORM(6, 64) break;
        default: AGOQ_LAUNCH_NORM(8, 64) break;
        }
    }
#undef AGOQ_LAUNCH_NORM
    return launch_status();
}

int agoq_act_dequant_silu_mul(const void* gate_codes, const float* gate_scales, int gate_bits,
                              const void* up_codes, const float* up_scales, int up_bits,
                              int64_t numel, int group, void* z_bf16, void* stream)
{
    if (!gate_codes || !gate_scales || !up_codes || !up_scales || !z_bf16) return AGOQ_ERR_NULL;
    if ((gate_bits != 4 && gate_bits != 5 && gate_bits != 6 && gate_bits != 8) ||
        (up_bits != 4 && up_bits != 5 && up_bits != 6 && up_bits != 8))
        return AGOQ_ERR_BITS;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(gate_codes) || misaligned(gate_scales) || misaligned(up_codes) ||
        misaligned(up_scales) || misaligned(z_bf16))
        return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    constexpr int U = 2;
    const dim3 grid(blocks_for(n_vec, AGOQ_DQ_BLOCK * U)), block(AGOQ_DQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    u32x4* z = (u32x4*)z_bf16;
#define AGOQ_LAUNCH_SILU(BG, BU)                                                                  \
    if (group == 128)                                                                             \
        act_dequant_silu_mul_kernel<BG, BU, 128, U><<<grid, block, 0, st>>>(gate_codes, gate_scales, up_codes, up_scales, n_vec, z); \
    else                                                                                          \
        act_dequant_silu_mul_kernel<BG, BU, 64, U><<<grid, block, 0, st>>>(gate_codes, gate_scales, up_codes, up_scales, n_vec, z);
#define AGOQ_SILU_UP(BG)                                                                          \
    switch (up_bits) {                                                                            \
    case 4: AGOQ_LAUNCH_SILU(BG, 4) break;                                                        \
    case 5: AGOQ_LAUNCH_SILU(BG, 5) break;                                                        \
    case 6: AGOQ_LAUNCH_SILU(BG, 6) break;                                                        \
    default: AGOQ_LAUNCH_SILU(BG, 8) break;                                                       \
    }
    switch (gate_bits) {
    case 4: AGOQ_SILU_UP(4) break;
    case 5: AGOQ_SILU_UP(5) break;
    case 6: AGOQ_SILU_UP(6) break;
    default: AGOQ_SILU_UP(8) break;
    }
#undef AGOQ_SILU_UP
#undef AGOQ_LAUNCH_SILU
    return launch_status();
}

// ---- floating-point code books ---------------------------------------------------------

int agoq_fp4_act_quant(const void* x_bf16, int64_t numel, int group, void* codes, float* scales,
                       void* stream)
{
    if (!x_bf16 || !codes || !scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    constexpr int U = AGOQ_AQ_UNROLL;
    const dim3 grid(blocks_for(n_vec, AGOQ_AQ_BLOCK * U)), block(AGOQ_AQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    const u32x4* x = (const u32x4*)x_bf16;
    if (group == 128)
        act_quant_kernel<4, 128, U, true><<<grid, block, 0, st>>>(x, n_vec, codes, scales);
    else
        act_quant_kernel<4, 64, U, true><<<grid, block, 0, st>>>(x, n_vec, codes, scales);
    return launch_status();
}

int agoq_fp4_act_dequant(const void* codes, const float* scales, int64_t numel, int group,
                         void* y_bf16, void* stream)
{
    if (!codes || !scales || !y_bf16) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(codes) || misaligned(scales) || misaligned(y_bf16)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    constexpr int U = 4;
    const dim3 grid(blocks_for(n_vec, AGOQ_DQ_BLOCK * U)), block(AGOQ_DQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    u32x4* y = (u32x4*)y_bf16;
    if (group == 128)
        act_dequant_kernel<4, 128, U, true><<<grid, block, 0, st>>>(codes, scales, n_vec, y);
    else
        act_dequant_kernel<4, 64, U, true><<<grid, block, 0, st>>>(codes, scales, n_vec, y);
    return launch_status();
}

int agoq_fp8_grad_quant(const float* grad, int64_t numel, int group, uint8_t* codes, float* scales,
                        void* stream)
{
    if (!grad || !codes || !scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(grad) || misaligned(codes) || misaligned(scales)) return AGOQ_ERR_ALIGN;
    const int64_t n_groups = numel / group;
    constexpr int U = AGOQ_GQ_UNROLL;
    const dim3 grid(blocks_for(n_groups * 16, AGOQ_GQ_BLOCK * U)), block(AGOQ_GQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    if (group == 128)
        grad_quant_kernel<128, U, true><<<grid, block, 0, st>>>((const f32x4*)grad, n_groups,
                                                                (u32*)codes, scales);
    else
        grad_quant_kernel<64, U, true><<<grid, block, 0, st>>>((const f32x4*)grad, n_groups,
                                                               (u32*)codes, scales);
    return launch_status();
}

int agoq_fp8_grad_dequant(const uint8_t* codes, const float* scales, int64_t numel, int group,
                          float* out, void* stream)
{
    if (!codes || !scales || !out) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(codes) || misaligned(scales) || misaligned(out)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 4;
    constexpr int U = AGOQ_GD_UNROLL;
    const dim3 grid(blocks_for(n_vec, AGOQ_GD_BLOCK * U)), block(AGOQ_GD_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    if (group == 128)
        grad_dequant_kernel<128, U, true><<<grid, block, 0, st>>>((const u32*)codes, scales, n_vec,
                                                                  (f32x4*)out);
    else
        grad_dequant_kernel<64, U, true><<<grid, block, 0, st>>>((const u32*)codes, scales, n_vec,
                                                                 (f32x4*)out);
    return launch_status();
}

int agoq_fp8_grad_reduce_requant(const uint8_t* in_codes, int64_t chunk_stride_codes,
                                 const float* in_scales, int64_t chunk_stride_scales, int K,
                                 int64_t numel, int group, uint8_t* out_codes, float* out_scales,
                                 void* stream)
{
    if (!in_codes || !in_scales || !out_codes || !out_scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (K < 1 || K > 64) return AGOQ_ERR_K;
    if (chunk_stride_codes < numel || chunk_stride_scales < numel / group) return AGOQ_ERR_SHAPE;
    if (misaligned(in_codes) || misaligned(in_scales) || misaligned(out_codes) ||
        misaligned(out_scales) || (chunk_stride_codes & 15) != 0)
        return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 16;
    const dim3 grid(blocks_for(n_vec, AGOQ_RD_BLOCK)), block(AGOQ_RD_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    u32x4* oc = (u32x4*)out_codes;
    const int8_t* ic = (const int8_t*)in_codes;
#define AGOQ_LAUNCH_REDUCE_FP(G, KT)                                                           \
    grad_reduce_kernel<G, KT, true><<<grid, block, 0, st>>>(ic, chunk_stride_codes, in_scales, \
                                                            chunk_stride_scales, K, n_vec, oc, out_scales)
    if (group == 128) {
        switch (K) {
        case 4: AGOQ_LAUNCH_REDUCE_FP(128, 4); break;
        case 8: AGOQ_LAUNCH_REDUCE_FP(128, 8); break;
        case 16: AGOQ_LAUNCH_REDUCE_FP(128, 16); break;
        default: AGOQ_LAUNCH_REDUCE_FP(128, 0); break;
        }
    } else {
        switch (K) {
        case 4: AGOQ_LAUNCH_REDUCE_FP(64, 4); break;
        case 8: AGOQ_LAUNCH_REDUCE_FP(64, 8); break;
        case 16: AGOQ_LAUNCH_REDUCE_FP(64, 16); break;
        default: AGOQ_LAUNCH_REDUCE_FP(64, 0); break;
        }
    }
#undef AGOQ_LAUNCH_REDUCE_FP
    return launch_status();
}

}  // extern "C"
