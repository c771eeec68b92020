/*
 * agoq_ref.c -- CPU oracle for the AGoQ quantization hot path.
 *
 * THIS FILE IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is the slow, plain
 * definition that the HIP kernels are checked against.  It shares nothing
 * with the GPU library (no header, no helper, no table) and only the tests,
 * the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What it computes (paper: "System Overview" -- activations are stored as
 * block-wise low-bit codes and dequantized to BF16 before the backward pass;
 * "Layer-Aware Activation Quantization / Other Operations" -- block size 128;
 * "Precision-Preserved Gradient Quantization" -- gradients kept as 8-bit
 * block-wise codes, and the local step of the 8-bit All-Reduce dequantizes
 * the chunks received from the peers to FP32, sums them, and quantizes the
 * sum again; "Dynamic Bit-width Compensation", Eq. (dynamic) -- per-stage
 * bit-width).
 *
 * The paper names the scheme but prints no arithmetic.  The reading used
 * here (every line of it is a reading, listed in the design notes):
 *   - uniform symmetric integer grid, qmax = 2^(b-1) - 1, no zero point;
 *   - blocks ("groups") are G contiguous elements of the flat buffer;
 *   - all arithmetic is IEEE binary32, round-to-nearest-even, no fused
 *     multiply-add except the one fmaf written out in the reduce;
 *   - amax  = max |x_j| over the group;
 *   - amax < 2^-100 (includes 0): scale = 0 and every code = 0;
 *   - scale = amax / qmax,  inv = qmax / amax   (two separate divisions);
 *   - code  = clamp(rint(x_j * inv), -qmax, +qmax)   (rint = ties to even);
 *   - codes are two's-complement fields of b bits.  b = 8: int8, one byte per
 *     element.  b = 4: byte m holds element 2m in bits 0-3 and element 2m+1
 *     in bits 4-7.  b = 5 and b = 6: two planes over the whole tensor; the
 *     low four bits of every code form a 4-bit plane laid out exactly like
 *     b = 4 (numel/2 bytes), and the remaining high bits follow at byte
 *     offset numel/2: for b = 5, bit j of byte m is the high bit of element
 *     8m+j; for b = 6, bits 2j..2j+1 of byte m are the two high bits of
 *     element 4m+j;
 *   - dequantize: v = (float)code * scale; activations return bf16(v) with
 *     round-to-nearest-even;
 *   - reduce: acc = 0; for k = 0..K-1 in that order: acc = fmaf(code_k,
 *     scale_k, acc); then the group of acc values is quantized with b = 8.
 *
 * Parity status of each function:
 *   act_quant / act_dequant / grad_quant / grad_reduce_requant /
 *   grad_accumulate / grad_dequant / act_dequant_rmsnorm / act_dequant_silu_mul /
 *   dbca_bits:  pinned by tests/test_oracle_*.py
 *   (exact-arithmetic brute force over all bf16 patterns, closed forms on
 *   power-of-two scales, tie cases, byte-level packing fixtures, the
 *   round-trip bound, library cross-checks and the values the paper prints
 *   for the four-stage pipeline).
 *   Non-finite inputs (the paper is silent; reading): they propagate at group
 *   granularity.  A group that holds +-Inf or a NaN -- in the tensor being
 *   quantized, or in the fp32 sums of the reduce and of the accumulation, so
 *   also when a sum overflows or an incoming scale is not finite -- stores the
 *   scale quiet-NaN (bits 0x7FC00000) and all-zero codes; every element of it
 *   then dequantizes to a NaN (0 * NaN).  A NaN converts to bf16 as a NaN whose
 *   payload is not specified.  Pinned by tests/test_oracle_nonfinite_pins.py.
 *
 *   Stochastic rounding (the *_sr functions): the paper never uses it; it is
 *   the optional variant the task statement allows ("driven by a counter-based
 *   hash").  Reading: code = clamp(floor(x*inv + u)), u = B/256 with B one byte
 *   of a 32-bit hash of (seed, element index / 4); the hash is the 32-bit
 *   finalizer of MurmurHash3 (A. Appleby, public domain) applied to the counter
 *   xor a per-seed key.  Pinned by tests/test_oracle_sr_pins.py (published
 *   hash vectors, u = 0 gives floor, grid values unchanged, |code - t| < 1,
 *   the mean over many seeds, exact rational re-evaluation, byte statistics).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * Parallelism is over groups only; a group is always handled by one thread
 * from start to end, so results do not depend on the thread count.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_ERR_NULL 1
#define REF_ERR_BITS 2
#define REF_ERR_GROUP 3
#define REF_ERR_SHAPE 4
#define REF_ERR_K 6

/* Groups whose largest magnitude is below this are stored as all-zero. */
static const float REF_AMAX_MIN = 0x1p-100f;

/* ---- bf16 <-> fp32 ------------------------------------------------------ */

static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16; /* bf16 is the top half of a binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round a binary32 to bf16, nearest, ties to even (an infinity stays one; a NaN becomes
   the quiet NaN 0x7FC0: which NaN is not part of the contract). */
static uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u;
    if (isnan(f))
        return 0x7FC0u;
    memcpy(&u, &f, sizeof u);
    uint32_t lsb = (u >> 16) & 1u; /* parity of the bit that survives */
    u += 0x7FFFu + lsb;            /* > half rounds up; == half rounds to even */
    return (uint16_t)(u >> 16);
}

/* exported so that the tests can pin the conversion on its own */
float agoq_ref_bf16_to_f32(uint16_t h) { return bf16_bits_to_f32(h); }
uint16_t agoq_ref_f32_to_bf16(float f) { return f32_to_bf16_bits(f); }

/* ---- the group quantizer ------------------------------------------------ */

static int qmax_of_bits(int bits) { return (1 << (bits - 1)) - 1; }

static int bits_supported(int bits)
{
    return bits == 4 || bits == 5 || bits == 6 || bits == 8;
}

/* The scale of a group that holds a non-finite value. */
static float quiet_nan(void)
{
    const uint32_t u = 0x7FC00000u;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static int group_is_finite(const float *x, int G)
{
    for (int j = 0; j < G; ++j)
        if (!isfinite(x[j]))
            return 0;
    return 1;
}

/*
 * Stochastic rounding.  The random variate of element i under `seed` is one
 * byte of a 32-bit word that four consecutive elements share:
 *     block = i / 4                                   (64-bit)
 *     key   = mix(seed ^ (high 32 bits of block) * 0x9E3779B9)
 *     word  = mix((low 32 bits of block) ^ key)
 *     B     = byte (i mod 4) of word, byte 0 the least significant
 *     u     = B / 256                                 (exact in binary32)
 * mix() is the 32-bit finalizer of MurmurHash3 (xor-shift 16, multiply by
 * 0x85EBCA6B, xor-shift 13, multiply by 0xC2B2AE35, xor-shift 16).
 */
static uint32_t sr_mix(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

static uint32_t sr_word(uint32_t seed, uint64_t block)
{
    const uint32_t lo = (uint32_t)block;
    const uint32_t hi = (uint32_t)(block >> 32);
    const uint32_t key = sr_mix(seed ^ (hi * 0x9E3779B9u));
    return sr_mix(lo ^ key);
}

static float sr_u(uint32_t seed, int64_t i)
{
    const uint32_t word = sr_word(seed, (uint64_t)i >> 2);
    const uint32_t byte = (word >> (8 * (int)(i & 3))) & 0xFFu;
    return (float)byte / 256.0f;
}

uint32_t agoq_ref_sr_word(uint32_t seed, uint64_t block) { return sr_word(seed, block); }
float agoq_ref_sr_u(uint32_t seed, int64_t i) { return sr_u(seed, i); }

/* How t = x * inv becomes an integer: to nearest (ties to even), or stochastically. */
struct rounding {
    int stochastic;
    uint32_t seed;
};
static const struct rounding ROUND_NEAREST = {0, 0};

/* Quantize G fp32 values to integer codes in [-qmax, qmax]; returns scale.
   first_index is the tensor index of x[0] (the stochastic variate depends on it). */
static float quantize_group(const float *x, int G, int qmax, int *q, struct rounding mode,
                            int64_t first_index)
{
    if (!group_is_finite(x, G)) { /* Inf or NaN anywhere: the whole group reads back as NaN */
        for (int j = 0; j < G; ++j)
            q[j] = 0;
        return quiet_nan();
    }
    float amax = 0.0f;
    for (int j = 0; j < G; ++j) {
        float a = fabsf(x[j]);
        if (a > amax)
            amax = a;
    }
    if (amax < REF_AMAX_MIN) {
        for (int j = 0; j < G; ++j)
            q[j] = 0;
        return 0.0f;
    }
    const float fq = (float)qmax;
    const float scale = amax / fq;
    const float inv = fq / amax;
    for (int j = 0; j < G; ++j) {
        float t = x[j] * inv;
        float r;
        if (mode.stochastic) {
            float shifted = t + sr_u(mode.seed, first_index + j); /* one binary32 addition */
            r = floorf(shifted);
        } else {
            r = rintf(t); /* default rounding mode: ties to even */
        }
        if (r > fq)
            r = fq;
        if (r < -fq)
            r = -fq;
        q[j] = (int)r;
    }
    return scale;
}

/* ---- code layout: element i of a tensor of numel elements --------------- */

static void put_code(uint8_t *codes, int64_t numel, int64_t i, int bits, int q)
{
    const uint32_t field = (uint32_t)q & ((1u << bits) - 1u); /* two's complement */
    if (bits == 8) {
        codes[i] = (uint8_t)field;
        return;
    }
    /* low nibble plane (all of a 4-bit code) */
    {
        uint8_t *byte = codes + i / 2;
        const uint32_t lo = field & 0xFu;
        if (i % 2 == 0)
            *byte = (uint8_t)((*byte & 0xF0u) | lo);
        else
            *byte = (uint8_t)((*byte & 0x0Fu) | (lo << 4));
    }
    if (bits == 4)
        return;
    /* high plane, after the numel/2 bytes of the nibble plane */
    {
        uint8_t *high = codes + numel / 2;
        const uint32_t hi = field >> 4; /* 1 bit (b = 5) or 2 bits (b = 6) */
        if (bits == 5) {
            uint8_t *byte = high + i / 8;
            const int sh = (int)(i % 8);
            *byte = (uint8_t)((*byte & ~(1u << sh)) | (hi << sh));
        } else {
            uint8_t *byte = high + i / 4;
            const int sh = 2 * (int)(i % 4);
            *byte = (uint8_t)((*byte & ~(3u << sh)) | (hi << sh));
        }
    }
}

static int get_code(const uint8_t *codes, int64_t numel, int64_t i, int bits)
{
    uint32_t field;
    if (bits == 8) {
        field = codes[i];
    } else {
        const uint8_t byte = codes[i / 2];
        field = (i % 2 == 0) ? (byte & 0xFu) : (uint32_t)(byte >> 4);
        if (bits == 5)
            field |= (uint32_t)((codes[numel / 2 + i / 8] >> (i % 8)) & 1u) << 4;
        else if (bits == 6)
            field |= (uint32_t)((codes[numel / 2 + i / 4] >> (2 * (i % 4))) & 3u) << 4;
    }
    if (field & (1u << (bits - 1))) /* sign bit of the field */
        return (int)field - (1 << bits);
    return (int)field;
}

/* ---- argument checks ---------------------------------------------------- */

static int check_shape(int64_t numel, int group, int bits)
{
    if (!bits_supported(bits))
        return REF_ERR_BITS;
    if (group < 1 || group > 4096)
        return REF_ERR_GROUP;
    if (numel <= 0 || numel % group != 0)
        return REF_ERR_SHAPE;
    if (group % 8 != 0 && bits != 8) /* every plane of a group is a whole number of bytes */
        return REF_ERR_GROUP;
    return REF_OK;
}

/* ---- activations -------------------------------------------------------- */

static int act_quant_any(const uint16_t *x, int64_t numel, int group, int bits, struct rounding mode,
                         uint8_t *codes, float *scales)
{
    if (!x || !codes || !scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, bits);
    if (rc)
        return rc;
    const int qmax = qmax_of_bits(bits);
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        float xf[4096];
        int q[4096];
        const uint16_t *xg = x + g * group;
        for (int j = 0; j < group; ++j)
            xf[j] = bf16_bits_to_f32(xg[j]);
        scales[g] = quantize_group(xf, group, qmax, q, mode, g * group);
        /* a group's bytes in every plane belong to that group alone */
        for (int j = 0; j < group; ++j)
            put_code(codes, numel, g * group + j, bits, q[j]);
    }
    return REF_OK;
}

/* x: numel bf16 bit patterns.  codes: numel*bits/8 bytes.  scales: numel/group. */
int agoq_ref_act_quant(const uint16_t *x, int64_t numel, int group, int bits,
                       uint8_t *codes, float *scales)
{
    return act_quant_any(x, numel, group, bits, ROUND_NEAREST, codes, scales);
}

/* The same with stochastic rounding of the codes (scales are unchanged by the mode). */
int agoq_ref_act_quant_sr(const uint16_t *x, int64_t numel, int group, int bits, uint32_t seed,
                          uint8_t *codes, float *scales)
{
    const struct rounding mode = {1, seed};
    return act_quant_any(x, numel, group, bits, mode, codes, scales);
}

int agoq_ref_act_dequant(const uint8_t *codes, const float *scales, int64_t numel,
                         int group, int bits, uint16_t *y)
{
    if (!codes || !scales || !y)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, bits);
    if (rc)
        return rc;
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        const float s = scales[g];
        for (int j = 0; j < group; ++j) {
            float v = (float)get_code(codes, numel, g * group + j, bits) * s;
            y[g * group + j] = f32_to_bf16_bits(v);
        }
    }
    return REF_OK;
}

/* ---- dequantize fused with the recomputation of the layer's forward ------ */

/*
 * Case-1 recomputation for RMSNorm ("Error Analysis of Activation Quantization /
 * RMSNorm"; Eq. (rmsnorm)): only the quantized input X is stored; r and the
 * normalized output are recomputed from the dequantized X' in the backward pass.
 *   x'_ij = bf16(code_ij * scale)                      (exactly act_dequant's output)
 *   r_i   = sqrt( (1/d) * sum_j x'_ij^2 + eps )        (d = cols), in binary64
 *   y_ij  = bf16( gamma_j * x'_ij / r_i )
 * This is the plain definition in binary64; the GPU computes in binary32, so parity
 * for y is "equal, or one bf16 step apart where the exact value sits at a rounding
 * boundary", and relative 2e-6 for r.
 */
int agoq_ref_act_dequant_rmsnorm(const uint8_t *codes, const float *scales, int64_t rows,
                                 int64_t cols, int group, int bits, const float *gamma,
                                 float eps, uint16_t *y, float *r_out)
{
    if (!codes || !scales || !gamma || !y || !r_out)
        return REF_ERR_NULL;
    if (rows <= 0 || cols <= 0 || cols % group != 0)
        return REF_ERR_SHAPE;
    const int64_t numel = rows * cols;
    int rc = check_shape(numel, group, bits);
    if (rc)
        return rc;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double ss = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            const int64_t e = i * cols + j;
            float v = (float)get_code(codes, numel, e, bits) * scales[e / group];
            double x = (double)bf16_bits_to_f32(f32_to_bf16_bits(v));
            ss += x * x;
        }
        const double r = sqrt(ss / (double)cols + (double)eps);
        r_out[i] = (float)r;
        for (int64_t j = 0; j < cols; ++j) {
            const int64_t e = i * cols + j;
            float v = (float)get_code(codes, numel, e, bits) * scales[e / group];
            double x = (double)bf16_bits_to_f32(f32_to_bf16_bits(v));
            y[e] = f32_to_bf16_bits((float)((double)gamma[j] * x / r));
        }
    }
    return REF_OK;
}

/*
 * Case-1 recomputation for SiLU & Multiply (appendix "SiLU & Multiply": z = x * y *
 * sigma(y)): the stored inputs are the gate (through SiLU) and the up projection; the
 * input of the second FFN GEMM is recomputed from their dequantized values.
 *   g' = bf16(code_g * scale_g), u' = bf16(code_u * scale_u)
 *   z  = bf16( u' * g' / (1 + exp(-g')) )              in binary64
 */
int agoq_ref_act_dequant_silu_mul(const uint8_t *gate_codes, const float *gate_scales,
                                  int gate_bits, const uint8_t *up_codes,
                                  const float *up_scales, int up_bits, int64_t numel, int group,
                                  uint16_t *z)
{
    if (!gate_codes || !gate_scales || !up_codes || !up_scales || !z)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, gate_bits);
    if (rc)
        return rc;
    rc = check_shape(numel, group, up_bits);
    if (rc)
        return rc;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < numel; ++e) {
        float gv = (float)get_code(gate_codes, numel, e, gate_bits) * gate_scales[e / group];
        float uv = (float)get_code(up_codes, numel, e, up_bits) * up_scales[e / group];
        double g = (double)bf16_bits_to_f32(f32_to_bf16_bits(gv));
        double u = (double)bf16_bits_to_f32(f32_to_bf16_bits(uv));
        z[e] = f32_to_bf16_bits((float)(u * g / (1.0 + exp(-g))));
    }
    return REF_OK;
}

/*
 * The forward side of the same two layers, for the fused "compute the layer and store its
 * quantized input in one pass" kernels: plain binary64 definitions on the ORIGINAL bf16
 * inputs (the stored codes are act_quant's, unchanged).
 *   rmsnorm_fwd : r_i = sqrt(mean_j x_ij^2 + eps),  y_ij = bf16(gamma_j * x_ij / r_i)
 *   silu_mul_fwd: z = bf16(u * g / (1 + exp(-g)))
 */
int agoq_ref_rmsnorm_fwd(const uint16_t *x, int64_t rows, int64_t cols, const float *gamma,
                         float eps, uint16_t *y, float *r_out)
{
    if (!x || !gamma || !y || !r_out)
        return REF_ERR_NULL;
    if (rows <= 0 || cols <= 0)
        return REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double sumsq = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            const double v = (double)bf16_bits_to_f32(x[i * cols + j]);
            sumsq += v * v;
        }
        const double rms = sqrt(sumsq / (double)cols + (double)eps);
        r_out[i] = (float)rms;
        for (int64_t j = 0; j < cols; ++j) {
            const double v = (double)bf16_bits_to_f32(x[i * cols + j]);
            y[i * cols + j] = f32_to_bf16_bits((float)((double)gamma[j] * v / rms));
        }
    }
    return REF_OK;
}

int agoq_ref_silu_mul_fwd(const uint16_t *gate, const uint16_t *up, int64_t numel, uint16_t *z)
{
    if (!gate || !up || !z)
        return REF_ERR_NULL;
    if (numel <= 0)
        return REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < numel; ++e) {
        const double gate_v = (double)bf16_bits_to_f32(gate[e]);
        const double up_v = (double)bf16_bits_to_f32(up[e]);
        z[e] = f32_to_bf16_bits((float)(up_v * gate_v / (1.0 + exp(-gate_v))));
    }
    return REF_OK;
}

/* ---- gradients ---------------------------------------------------------- */

static int grad_quant_any(const float *grad, int64_t numel, int group, struct rounding mode,
                          int8_t *codes, float *scales)
{
    if (!grad || !codes || !scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        int q[4096];
        scales[g] = quantize_group(grad + g * group, group, 127, q, mode, g * group);
        for (int j = 0; j < group; ++j)
            codes[g * group + j] = (int8_t)q[j];
    }
    return REF_OK;
}

int agoq_ref_grad_quant(const float *grad, int64_t numel, int group, int8_t *codes,
                        float *scales)
{
    return grad_quant_any(grad, numel, group, ROUND_NEAREST, codes, scales);
}

int agoq_ref_grad_quant_sr(const float *grad, int64_t numel, int group, uint32_t seed,
                           int8_t *codes, float *scales)
{
    const struct rounding mode = {1, seed};
    return grad_quant_any(grad, numel, group, mode, codes, scales);
}

/* int8 codes + scales -> fp32 values (what an optimizer would read). */
int agoq_ref_grad_dequant(const int8_t *codes, const float *scales, int64_t numel,
                          int group, float *out)
{
    if (!codes || !scales || !out)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g)
        for (int j = 0; j < group; ++j)
            out[g * group + j] = (float)codes[g * group + j] * scales[g];
    return REF_OK;
}

/*
 * Local step of the 8-bit All-Reduce.  Chunk k starts at in_codes +
 * k*stride_codes (numel int8) and in_scales + k*stride_scales (numel/group
 * fp32).  Summation order is the chunk index, one fmaf per term.
 */
static int grad_reduce_any(const int8_t *in_codes, int64_t stride_codes, const float *in_scales,
                           int64_t stride_scales, int K, int64_t numel, int group,
                           struct rounding mode, int8_t *out_codes, float *out_scales)
{
    if (!in_codes || !in_scales || !out_codes || !out_scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    if (K < 1 || K > 64)
        return REF_ERR_K;
    const int64_t n_groups = numel / group;
    if (stride_codes < numel || stride_scales < n_groups)
        return REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        float acc[4096];
        int q[4096];
        for (int j = 0; j < group; ++j) {
            float a = 0.0f;
            for (int k = 0; k < K; ++k) {
                float c = (float)in_codes[k * stride_codes + g * group + j];
                float s = in_scales[k * stride_scales + g];
                a = fmaf(c, s, a);
            }
            acc[j] = a;
        }
        out_scales[g] = quantize_group(acc, group, 127, q, mode, g * group);
        for (int j = 0; j < group; ++j)
            out_codes[g * group + j] = (int8_t)q[j];
    }
    return REF_OK;
}

int agoq_ref_grad_reduce_requant(const int8_t *in_codes, int64_t stride_codes,
                                 const float *in_scales, int64_t stride_scales, int K,
                                 int64_t numel, int group, int8_t *out_codes,
                                 float *out_scales)
{
    return grad_reduce_any(in_codes, stride_codes, in_scales, stride_scales, K, numel, group,
                           ROUND_NEAREST, out_codes, out_scales);
}

/* The sums as above; the requantization rounds stochastically (variate of OUTPUT element i). */
int agoq_ref_grad_reduce_requant_sr(const int8_t *in_codes, int64_t stride_codes,
                                    const float *in_scales, int64_t stride_scales, int K,
                                    int64_t numel, int group, uint32_t seed, int8_t *out_codes,
                                    float *out_scales)
{
    const struct rounding mode = {1, seed};
    return grad_reduce_any(in_codes, stride_codes, in_scales, stride_scales, K, numel, group, mode,
                           out_codes, out_scales);
}

/*
 * The same sums in binary64, in the same order, without requantizing: the
 * yardstick for "how far is the fp32 accumulation from the exact sum".
 * abs_sum receives sum_k |code_k * scale_k| (may be NULL).
 */
int agoq_ref_grad_reduce_f64(const int8_t *in_codes, int64_t stride_codes,
                             const float *in_scales, int64_t stride_scales, int K,
                             int64_t numel, int group, double *sum, double *abs_sum)
{
    if (!in_codes || !in_scales || !sum)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    if (K < 1 || K > 64)
        return REF_ERR_K;
    for (int64_t i = 0; i < numel; ++i) {
        double a = 0.0, b = 0.0;
        for (int k = 0; k < K; ++k) {
            double term = (double)in_codes[k * stride_codes + i] *
                          (double)in_scales[k * stride_scales + i / group];
            a += term;
            b += fabs(term);
        }
        sum[i] = a;
        if (abs_sum)
            abs_sum[i] = b;
    }
    return REF_OK;
}

/*
 * Local gradient accumulation: the stored 8-bit main gradient is dequantized,
 * the new micro-batch gradient is added in fp32 (one rounding:
 * acc = fmaf(code, scale, g_new)), and the sum is quantized back to 8 bits.
 * g_new is fp32 (new_is_bf16 = 0) or bf16 bit patterns (new_is_bf16 = 1).
 */
static int grad_accumulate_any(const int8_t *main_codes, const float *main_scales, const void *g_new,
                               int new_is_bf16, int64_t numel, int group, struct rounding mode,
                               int8_t *out_codes, float *out_scales)
{
    if (!main_codes || !main_scales || !g_new || !out_codes || !out_scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        float acc[4096];
        int q[4096];
        const float s = main_scales[g];
        for (int j = 0; j < group; ++j) {
            int64_t i = g * group + j;
            float add = new_is_bf16 ? bf16_bits_to_f32(((const uint16_t *)g_new)[i])
                                    : ((const float *)g_new)[i];
            acc[j] = fmaf((float)main_codes[i], s, add);
        }
        out_scales[g] = quantize_group(acc, group, 127, q, mode, g * group);
        for (int j = 0; j < group; ++j)
            out_codes[g * group + j] = (int8_t)q[j];
    }
    return REF_OK;
}

int agoq_ref_grad_accumulate(const int8_t *main_codes, const float *main_scales,
                             const void *g_new, int new_is_bf16, int64_t numel, int group,
                             int8_t *out_codes, float *out_scales)
{
    return grad_accumulate_any(main_codes, main_scales, g_new, new_is_bf16, numel, group,
                               ROUND_NEAREST, out_codes, out_scales);
}

/* The same with stochastic rounding of the stored sum (variate of element i). */
int agoq_ref_grad_accumulate_sr(const int8_t *main_codes, const float *main_scales,
                                const void *g_new, int new_is_bf16, int64_t numel, int group,
                                uint32_t seed, int8_t *out_codes, float *out_scales)
{
    const struct rounding mode = {1, seed};
    return grad_accumulate_any(main_codes, main_scales, g_new, new_is_bf16, numel, group, mode,
                               out_codes, out_scales);
}

/* ======================================================================= */
/* Floating-point code books: the formats the paper names ("block-wise FP4  */
/* quantization" for activations, "FP8" for gradients), read as E2M1 and     */
/* OCP E4M3 (no infinities), block-wise abs-max scaled like the integer      */
/* grids above:                                                              */
/*     scale = amax / vmax,  inv = vmax / amax,  code = nearest(x * inv)     */
/* with vmax = 6 (E2M1) or 448 (E4M3), nearest = round to the nearest        */
/* representable value, ties to the code with an even mantissa, the sign bit */
/* of the code being the sign bit of x * inv.  Groups with amax < 2^-100     */
/* store scale 0 and all-zero codes.                                          */
/* ======================================================================= */

/* magnitude of E2M1 code index 0..7: exponent field e = idx >> 1, mantissa m = idx & 1;
   e == 0: m * 0.5 (subnormal);  else (1 + m/2) * 2^(e-1) */
static float e2m1_magnitude(int idx)
{
    const int e = idx >> 1, m = idx & 1;
    if (e == 0)
        return 0.5f * (float)m;
    return ldexpf(1.0f + 0.5f * (float)m, e - 1);
}

/* magnitude of E4M3 code index 0..126 (index 127 is NaN): e = idx >> 3, m = idx & 7, bias 7;
   e == 0: m * 2^-9;  else (1 + m/8) * 2^(e-7) */
static float e4m3_magnitude(int idx)
{
    const int e = idx >> 3, m = idx & 7;
    if (e == 0)
        return ldexpf((float)m, -9);
    return ldexpf(1.0f + (float)m / 8.0f, e - 7);
}

/* index of the representable magnitude nearest to a >= 0 among n_values (increasing),
   ties to the even index, beyond the last value: the last value (saturation) */
static int nearest_index(float a, int n_values, float (*magnitude)(int))
{
    int best = 0;
    double best_d = fabs((double)a - (double)magnitude(0));
    for (int i = 1; i < n_values; ++i) {
        const double d = fabs((double)a - (double)magnitude(i));
        if (d < best_d || (d == best_d && (i % 2 == 0))) {
            best = i;
            best_d = d;
        }
    }
    return best;
}

static uint8_t e2m1_encode(float t)
{
    const int idx = nearest_index(fabsf(t), 8, e2m1_magnitude);
    return (uint8_t)((signbit(t) ? 8 : 0) | idx);
}

static float e2m1_decode(uint8_t code)
{
    const float v = e2m1_magnitude(code & 7);
    return (code & 8) ? -v : v;
}

static uint8_t e4m3_encode(float t)
{
    const int idx = nearest_index(fabsf(t), 127, e4m3_magnitude);
    return (uint8_t)((signbit(t) ? 0x80 : 0) | idx);
}

static float e4m3_decode(uint8_t code)
{
    if ((code & 0x7F) == 0x7F) /* the format's NaN; the quantizer never produces it */
        return quiet_nan();
    const float v = e4m3_magnitude(code & 0x7F);
    return (code & 0x80) ? -v : v;
}

uint8_t agoq_ref_e2m1_encode(float t) { return e2m1_encode(t); }
float agoq_ref_e2m1_decode(uint8_t c) { return e2m1_decode(c); }
uint8_t agoq_ref_e4m3_encode(float t) { return e4m3_encode(t); }
float agoq_ref_e4m3_decode(uint8_t c) { return e4m3_decode(c); }

/* scale, inv of a group for a code book with largest magnitude vmax; returns 0 for a group
   whose codes are all zero (a dead group, or one that holds a non-finite value) */
static int fp_group_scale(const float *x, int G, float vmax, float *scale, float *inv)
{
    if (!group_is_finite(x, G)) {
        *scale = quiet_nan();
        *inv = 0.0f;
        return 0;
    }
    float amax = 0.0f;
    for (int j = 0; j < G; ++j) {
        const float mag = fabsf(x[j]);
        if (mag > amax)
            amax = mag;
    }
    if (amax < REF_AMAX_MIN) {
        *scale = 0.0f;
        *inv = 0.0f;
        return 0;
    }
    *scale = amax / vmax;
    *inv = vmax / amax;
    return 1;
}

/* activations: bf16 -> E2M1 codes (nibbles, even element low) + fp32 scales */
int agoq_ref_fp4_act_quant(const uint16_t *x, int64_t numel, int group, uint8_t *codes,
                           float *scales)
{
    if (!x || !codes || !scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 4);
    if (rc)
        return rc;
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        float xf[4096];
        for (int j = 0; j < group; ++j)
            xf[j] = bf16_bits_to_f32(x[g * group + j]);
        float scale, inv;
        const int live = fp_group_scale(xf, group, 6.0f, &scale, &inv);
        scales[g] = scale;
        for (int j = 0; j < group; j += 2) {
            const uint8_t lo = live ? e2m1_encode(xf[j] * inv) : 0;
            const uint8_t hi = live ? e2m1_encode(xf[j + 1] * inv) : 0;
            codes[(g * group + j) / 2] = (uint8_t)(lo | (hi << 4));
        }
    }
    return REF_OK;
}

int agoq_ref_fp4_act_dequant(const uint8_t *codes, const float *scales, int64_t numel, int group,
                             uint16_t *y)
{
    if (!codes || !scales || !y)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 4);
    if (rc)
        return rc;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < numel; ++e) {
        const uint8_t byte = codes[e / 2];
        const uint8_t code = (e % 2 == 0) ? (byte & 0xF) : (uint8_t)(byte >> 4);
        y[e] = f32_to_bf16_bits(e2m1_decode(code) * scales[e / group]);
    }
    return REF_OK;
}

/* gradients: fp32 -> E4M3 codes (one byte each) + fp32 scales */
int agoq_ref_fp8_grad_quant(const float *grad, int64_t numel, int group, uint8_t *codes,
                            float *scales)
{
    if (!grad || !codes || !scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        float scale, inv;
        const int live = fp_group_scale(grad + g * group, group, 448.0f, &scale, &inv);
        scales[g] = scale;
        for (int j = 0; j < group; ++j)
            codes[g * group + j] = live ? e4m3_encode(grad[g * group + j] * inv) : 0;
    }
    return REF_OK;
}

int agoq_ref_fp8_grad_dequant(const uint8_t *codes, const float *scales, int64_t numel, int group,
                              float *out)
{
    if (!codes || !scales || !out)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < numel; ++e)
        out[e] = e4m3_decode(codes[e]) * scales[e / group];
    return REF_OK;
}

/* local step of the All-Reduce on E4M3 chunks: fp32 fma chain in chunk order, requantize */
int agoq_ref_fp8_grad_reduce_requant(const uint8_t *in_codes, int64_t stride_codes,
                                     const float *in_scales, int64_t stride_scales, int K,
                                     int64_t numel, int group, uint8_t *out_codes,
                                     float *out_scales)
{
    if (!in_codes || !in_scales || !out_codes || !out_scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    if (K < 1 || K > 64)
        return REF_ERR_K;
    const int64_t n_groups = numel / group;
    if (stride_codes < numel || stride_scales < n_groups)
        return REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        float acc[4096];
        for (int j = 0; j < group; ++j) {
            const int64_t e = g * group + j;
            float a = 0.0f;
            for (int k = 0; k < K; ++k) {
                const float v = e4m3_decode(in_codes[k * stride_codes + e]);
                a = fmaf(v, in_scales[k * stride_scales + g], a);
            }
            acc[j] = a;
        }
        float scale, inv;
        const int live = fp_group_scale(acc, group, 448.0f, &scale, &inv);
        out_scales[g] = scale;
        for (int j = 0; j < group; ++j)
            out_codes[g * group + j] = live ? e4m3_encode(acc[j] * inv) : 0;
    }
    return REF_OK;
}

/* local accumulation on E4M3 codes: acc = fma(decode(code), scale, g_new), requantize */
int agoq_ref_fp8_grad_accumulate(const uint8_t *main_codes, const float *main_scales,
                                 const void *g_new, int new_is_bf16, int64_t numel, int group,
                                 uint8_t *out_codes, float *out_scales)
{
    if (!main_codes || !main_scales || !g_new || !out_codes || !out_scales)
        return REF_ERR_NULL;
    int rc = check_shape(numel, group, 8);
    if (rc)
        return rc;
    const int64_t n_groups = numel / group;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < n_groups; ++g) {
        float acc[4096];
        for (int j = 0; j < group; ++j) {
            const int64_t i = g * group + j;
            const float addend = new_is_bf16 ? bf16_bits_to_f32(((const uint16_t *)g_new)[i])
                                             : ((const float *)g_new)[i];
            acc[j] = fmaf(e4m3_decode(main_codes[i]), main_scales[g], addend);
        }
        float scale, inv;
        const int live = fp_group_scale(acc, group, 448.0f, &scale, &inv);
        out_scales[g] = scale;
        for (int j = 0; j < group; ++j)
            out_codes[g * group + j] = live ? e4m3_encode(acc[j] * inv) : 0;
    }
    return REF_OK;
}

/* ---- Dynamic Bit-width Compensation (Eq. "dynamic") --------------------- */

/*
 * Interleaved 1F1B with n stages: stage i (1-based) holds N_i = 3n - 2i + 1
 * micro-batches of activations at its peak (first stage the most: the text
 * gives 11, 9, 7, 5 for n = 4; the printed formula has the index reversed).
 * B_i = 4 * N_1 / N_i, rounded to the nearest integer (halves up), at least
 * 4 and at most 8.
 */
int agoq_ref_dbca_stored_microbatches(int n_stages, int stage)
{
    if (n_stages < 1 || stage < 1 || stage > n_stages)
        return -1;
    return 3 * n_stages - 2 * stage + 1;
}

int agoq_ref_dbca_bits(int n_stages, int stage, int *bits_out)
{
    if (!bits_out)
        return REF_ERR_NULL;
    if (n_stages < 1 || stage < 1 || stage > n_stages)
        return REF_ERR_SHAPE;
    int n1 = agoq_ref_dbca_stored_microbatches(n_stages, 1);
    int ni = agoq_ref_dbca_stored_microbatches(n_stages, stage);
    double b = 4.0 * (double)n1 / (double)ni;
    int r = (int)floor(b + 0.5);
    if (r < 4)
        r = 4;
    if (r > 8)
        r = 8;
    *bits_out = r;
    return REF_OK;
}

/* ---- thread control for the timed baseline ------------------------------ */

int agoq_ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void agoq_ref_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}
