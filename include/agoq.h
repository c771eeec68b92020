/*
 * agoq.h -- C ABI of the AGoQ quantization hot path for AMD MI355X (gfx950).
 *
 * The library implements the storage side of AGoQ's training-memory scheme:
 * block-wise low-bit storage of activations between forward and backward,
 * 8-bit storage of gradients, and the local, precision-preserving step of the
 * 8-bit All-Reduce.  Each entry point below names the passage of the paper
 * that defines the operation.
 *
 * Conventions shared by every device entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The
 *     library never allocates, frees, copies to the host or synchronizes.
 *   - A call enqueues its kernel(s) on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) of the CURRENT device and returns at
 *     once.  Outputs are complete when the stream reaches that point.
 *   - Return value: AGOQ_OK (0) or a positive AGOQ_ERR_* code.  On error
 *     nothing has been enqueued and no output byte has been touched.
 *   - `group` (block size) is 64 or 128 elements; groups are runs of `group`
 *     consecutive elements of the flat buffer, so a row-major [rows, cols]
 *     tensor with cols % group == 0 is quantized along its last dimension.
 *     `numel` must be a positive multiple of `group` (the paper defines no
 *     partial block).
 *   - Every tensor pointer must be 16-byte aligned.  Input and output
 *     buffers must not overlap unless an entry point says otherwise.
 *   - Arithmetic is IEEE binary32 with round-to-nearest-even throughout; for
 *     a group with largest magnitude amax and qmax = 2^(bits-1) - 1:
 *         amax <  2^-100 :  scale = 0, every code 0
 *         otherwise      :  scale = amax / qmax,  inv = qmax / amax
 *                           code  = rint(x * inv)   (ties to even; |code| <= qmax)
 *     and dequantization is value = (float)code * scale.
 *   - Non-finite values propagate per group (the paper does not say; this is
 *     the library's rule): a group that holds +-Inf or a NaN -- in the tensor
 *     being quantized, or in the fp32 sums of the reduce and the accumulation,
 *     so also when such a sum overflows or an incoming scale is not finite --
 *     is stored with scale = quiet NaN (bits 0x7FC00000) and all-zero codes,
 *     and therefore dequantizes to NaN in every element.  Which NaN a bf16
 *     output holds is unspecified.
 *   - Code layout: codes are two's-complement fields of `bits` bits.  8-bit
 *     codes are int8, one per element.  4-bit codes: byte m holds element 2m
 *     in bits 0-3 and element 2m+1 in bits 4-7.  5- and 6-bit codes occupy
 *     two planes over the whole tensor: the low four bits of every code form
 *     a plane laid out exactly like 4-bit codes (numel/2 bytes); the high
 *     bits follow at byte offset numel/2: for 5 bits, bit j of byte m is the
 *     high bit of element 8m+j; for 6 bits, bits 2j..2j+1 of byte m are the
 *     two high bits of element 4m+j.  Scales are fp32, one per group, in
 *     group order.
 */
#ifndef AGOQ_H
#define AGOQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    AGOQ_OK = 0,
    AGOQ_ERR_NULL = 1,  /* a required pointer is NULL */
    AGOQ_ERR_BITS = 2,  /* bits is not 4, 5, 6 or 8 */
    AGOQ_ERR_GROUP = 3, /* group is not 64 or 128 */
    AGOQ_ERR_SHAPE = 4, /* numel <= 0, numel % group != 0, or a stride below its extent */
    AGOQ_ERR_ALIGN = 5, /* a pointer (or a chunk stride) breaks 16-byte alignment */
    AGOQ_ERR_K = 6,     /* K outside 1..64 */
    AGOQ_ERR_HIP = 7,   /* the HIP runtime refused this launch (the launch call's own status) */
    AGOQ_ERR_COUNT = 8  /* a layer call with fewer than 1 or more than AGOQ_MAX_LAYER_SLOTS tensors */
};

/*
 * Quantize and pack an activation for storage until the backward pass
 * (paper: "System Overview", activations are stored at about 4 bits after the
 * forward pass; "Layer-Aware Activation Quantization / Other Operations",
 * block-wise quantization with block size 128; "Dynamic Bit-width
 * Compensation", later pipeline stages use wider codes).
 *   x_bf16 : in,  numel bf16 values
 *   bits   : 4, 5, 6 or 8, the width the bit map assigns to this tensor
 *   codes  : out, numel*bits/8 bytes
 *   scales : out, numel/group fp32
 */
int agoq_act_quant(const void *x_bf16, int64_t numel, int group, int bits, void *codes,
                   float *scales, void *stream);

/*
 * Unpack and dequantize a stored activation to bf16 for the backward pass
 * (paper: "System Overview": quantized activations are dequantized to
 * BF16 before gradient computation).  y = bf16(code * scale), the product
 * rounded to fp32 first and then to bf16, both to nearest-even.
 *   codes, scales : in, as written by agoq_act_quant (any codes are legal,
 *                   including -8 / -128)
 *   y_bf16        : out, numel bf16 values
 */
int agoq_act_dequant(const void *codes, const float *scales, int64_t numel, int group, int bits,
                     void *y_bf16, void *stream);

/*
 * All stored tensors of one layer in one launch (paper: "Layer-Aware Activation
 * Quantization", each stored tensor of a layer has the bit-width that the bit map gives
 * its layer type; "Dynamic Bit-width Compensation", the map changes with the pipeline
 * stage).  The result in every buffer is exactly that of agoq_act_quant /
 * agoq_act_dequant called once per tensor; one launch instead of `count` saves the fixed
 * cost of a launch, which is a third of the run time of a 32 MiB tensor.
 *   slots : in, HOST array of `count` descriptors, read before the call returns (the
 *           caller may free or reuse it at once); every pointer inside is a device
 *           pointer with the meaning, size, alignment and ownership of the matching
 *           single-tensor argument: for quantize `bf16` is the input and `codes`, `scales`
 *           are written; for dequantize `codes`, `scales` are the inputs and `bf16` is
 *           written
 *   count : 1..AGOQ_MAX_LAYER_SLOTS, else AGOQ_ERR_COUNT
 *   group : one group size for the whole call
 * Tensors must not overlap each other.  Any invalid slot fails the whole call with the
 * error the single-tensor call would give, and nothing is enqueued.
 */
enum { AGOQ_MAX_LAYER_SLOTS = 8 };
typedef struct agoq_act_slot {
    void *bf16;     /* numel bf16 values */
    void *codes;    /* numel*bits/8 bytes */
    float *scales;  /* numel/group fp32 */
    int64_t numel;
    int bits;       /* 4, 5, 6 or 8 */
} agoq_act_slot;
int agoq_act_quant_layer(const agoq_act_slot *slots, int count, int group, void *stream);
int agoq_act_dequant_layer(const agoq_act_slot *slots, int count, int group, void *stream);

/*
 * Dequantize a stored RMSNorm input and recompute the layer's forward from it (paper:
 * "Error Analysis of Activation Quantization / RMSNorm", Case 1, with Eq. (rmsnorm):
 * only the quantized input is stored; r and the normalized output are recomputed in the
 * backward pass).  For each row i of the [rows, cols] tensor:
 *     x' = bf16(code * scale)                 (what agoq_act_dequant would write)
 *     r_i = sqrt(mean_j x'_ij^2 + eps),   y_ij = bf16(gamma_j * x'_ij / r_i)
 * computed in fp32 (results are within one bf16 step of the exact value, r within 2e-6
 * relative).  Nothing but y and r is written: the dequantized tensor never goes to memory.
 *   cols   : multiple of group, at most 16384
 *   gamma  : in, cols fp32
 *   y_bf16 : out, rows*cols bf16 (the recomputed input of the next GEMM)
 *   r_out  : out, rows fp32 (for the norm's own backward)
 */
int agoq_act_dequant_rmsnorm(const void *codes, const float *scales, int64_t rows, int64_t cols,
                             int group, int bits, const float *gamma, float eps, void *y_bf16,
                             float *r_out, void *stream);

/*
 * Dequantize the two stored inputs of SiLU & Multiply and recompute its output (paper:
 * appendix "SiLU & Multiply", z = x * y * sigma(y), Case 1: only the quantized inputs are
 * stored and the input of the second FFN GEMM is recomputed in the backward pass).
 *     g' = bf16(gate code * scale), u' = bf16(up code * scale), z = bf16(u' * g' * sigmoid(g'))
 * computed in fp32 (within one bf16 step of the exact value; magnitudes below 2^-100 may
 * come out as zero).  The two tensors may have
 * different code widths (4, 5, 6 or 8 each) and share numel and group.
 */
int agoq_act_dequant_silu_mul(const void *gate_codes, const float *gate_scales, int gate_bits,
                              const void *up_codes, const float *up_scales, int up_bits,
                              int64_t numel, int group, void *z_bf16, void *stream);

/*
 * Forward-side counterparts: compute the layer and store its quantized input in the same
 * pass (paper: "Kernel Fusion of Quantization/Dequantization and GEMM" motivates fusing
 * the element-wise quantization into a neighbouring kernel; here the neighbour is the
 * element-wise / row-wise layer that produces the next GEMM's input, so the input tensor
 * is read once instead of twice).  codes/scales are exactly what agoq_act_quant writes
 * for the same input; y / z are within one bf16 step of the exact value.
 *   agoq_rmsnorm_fwd_quant : y = bf16(gamma * x / r), r = sqrt(mean(x^2) + eps) per row
 *                            (r_out may be NULL); cols a multiple of group, <= 16384
 *   agoq_silu_mul_fwd_quant: z = bf16(up * gate * sigmoid(gate)); the two inputs may be
 *                            stored at different widths
 */
int agoq_rmsnorm_fwd_quant(const void *x_bf16, int64_t rows, int64_t cols, const float *gamma,
                           float eps, int group, int bits, void *y_bf16, float *r_out, void *codes,
                           float *scales, void *stream);
int agoq_silu_mul_fwd_quant(const void *gate_bf16, const void *up_bf16, int64_t numel, int group,
                            int gate_bits, int up_bits, void *z_bf16, void *gate_codes,
                            float *gate_scales, void *up_codes, float *up_scales, void *stream);

/*
 * Store a gradient as 8-bit block-wise codes (paper: "Precision-Preserved
 * Gradient Quantization": the main gradient is kept in 8 bits).
 *   grad   : in,  numel fp32
 *   codes  : out, numel int8
 *   scales : out, numel/group fp32
 */
int agoq_grad_quant(const float *grad, int64_t numel, int group, int8_t *codes, float *scales,
                    void *stream);

/*
 * Local step of the 8-bit All-Reduce (paper: "Precision-Preserved Gradient
 * Quantization": after the All-to-All each device dequantizes the chunks it
 * received to FP32, reduces them locally and quantizes the result again for
 * the All-Gather).  The K chunks are this device's shard as sent by K peers,
 * laid out as one receive buffer: chunk k starts at in_codes +
 * k*chunk_stride_codes and in_scales + k*chunk_stride_scales.
 *   for each element i of group g:
 *       acc = 0;  for k = 0 .. K-1 (in this order):  acc = fma(code_k[i], scale_k[g], acc)
 *   then the group of acc values is quantized to 8 bits as in agoq_grad_quant.
 *   The summation order is fixed, so the result is bit-reproducible.
 *   chunk_stride_codes  : elements between chunks, >= numel, multiple of 16
 *   chunk_stride_scales : elements between chunks, >= numel/group
 *   K : 1..64
 */
int agoq_grad_reduce_requant(const int8_t *in_codes, int64_t chunk_stride_codes,
                             const float *in_scales, int64_t chunk_stride_scales, int K,
                             int64_t numel, int group, int8_t *out_codes, float *out_scales,
                             void *stream);

/*
 * Local gradient accumulation (paper: "System Overview" and "Precision-Preserved
 * Gradient Quantization", first overflow issue: the stored 8-bit main gradient is
 * dequantized, the new micro-batch gradient is added in high precision, and the sum is
 * quantized back to 8 bits and written over the stored gradient).
 *   for each element i of group g:  acc = fma(code[i], scale[g], g_new[i])   (fp32)
 *   then the group of acc values is quantized to 8 bits as in agoq_grad_quant.
 *   g_new         : in, numel values: fp32 (g_new_is_bf16 == 0) or bf16 (!= 0)
 *   out_codes, out_scales : may be the same buffers as main_codes, main_scales
 *                   (in-place update); any other overlap is undefined.
 */
int agoq_grad_accumulate(const int8_t *main_codes, const float *main_scales, const void *g_new,
                         int g_new_is_bf16, int64_t numel, int group, int8_t *out_codes,
                         float *out_scales, void *stream);

/*
 * Dequantize a stored 8-bit gradient to fp32 (paper: "Precision-Preserved Gradient
 * Quantization": quantized gradients are dequantized before they are used in high
 * precision).  out[i] = (float)code[i] * scale[g], one fp32 rounding.
 * For a bf16 result (that product rounded once more, to nearest even) call
 * agoq_act_dequant with bits = 8 on the same buffers: int8 gradient codes and 8-bit
 * activation codes share one layout.
 */
int agoq_grad_dequant(const int8_t *codes, const float *scales, int64_t numel, int group,
                      float *out, void *stream);

/* ---- the same path with floating-point code books ------------------------
 *
 * The paper words its formats as "block-wise FP4 quantization" (activations) and "FP8"
 * (gradients).  These entry points are the calls above with the integer grid replaced by
 * a floating-point code book, everything else unchanged (groups, fp32 scales, layouts,
 * error codes, the 2^-100 rule, fixed summation order):
 *     scale = amax / vmax,  inv = vmax / amax,  code = nearest(x * inv)
 *   FP4 = E2M1 (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6; vmax = 6), one nibble per element,
 *         sign in bit 3, even element in bits 0-3 of the byte;
 *   FP8 = OCP E4M3 (no infinities; vmax = 448), one byte per element, sign in bit 7.
 * nearest = round to the nearest representable value, ties to the even mantissa; the
 * code's sign bit is the sign bit of x * inv (negative values that round to zero give
 * -0), except that a group stored as zeros has all-zero codes.  The NaN code of E4M3 is
 * never produced; on input it decodes as NaN.
 */
int agoq_fp4_act_quant(const void *x_bf16, int64_t numel, int group, void *codes, float *scales,
                       void *stream);
int agoq_fp4_act_dequant(const void *codes, const float *scales, int64_t numel, int group,
                         void *y_bf16, void *stream);
/* The four calls fused with RMSNorm and SiLU & Multiply, on E2M1 codes (arguments as in the
 * integer forms above, without the `bits` arguments; same limits, same error codes). */
int agoq_fp4_act_dequant_rmsnorm(const void *codes, const float *scales, int64_t rows, int64_t cols,
                                 int group, const float *gamma, float eps, void *y_bf16,
                                 float *r_out, void *stream);
int agoq_fp4_act_dequant_silu_mul(const void *gate_codes, const float *gate_scales,
                                  const void *up_codes, const float *up_scales, int64_t numel,
                                  int group, void *z_bf16, void *stream);
int agoq_fp4_rmsnorm_fwd_quant(const void *x_bf16, int64_t rows, int64_t cols, const float *gamma,
                               float eps, int group, void *y_bf16, float *r_out, void *codes,
                               float *scales, void *stream);
int agoq_fp4_silu_mul_fwd_quant(const void *gate_bf16, const void *up_bf16, int64_t numel, int group,
                                void *z_bf16, void *gate_codes, float *gate_scales, void *up_codes,
                                float *up_scales, void *stream);
int agoq_fp8_grad_quant(const float *grad, int64_t numel, int group, uint8_t *codes, float *scales,
                        void *stream);
int agoq_fp8_grad_dequant(const uint8_t *codes, const float *scales, int64_t numel, int group,
                          float *out, void *stream);
int agoq_fp8_grad_reduce_requant(const uint8_t *in_codes, int64_t chunk_stride_codes,
                                 const float *in_scales, int64_t chunk_stride_scales, int K,
                                 int64_t numel, int group, uint8_t *out_codes, float *out_scales,
                                 void *stream);
int agoq_fp8_grad_accumulate(const uint8_t *main_codes, const float *main_scales, const void *g_new,
                             int g_new_is_bf16, int64_t numel, int group, uint8_t *out_codes,
                             float *out_scales, void *stream);

/* ---- host-only helpers: pure functions, no device access ---------------- */

/* Bytes of packed codes for numel elements at `bits` per element; -1 if bits is unsupported. */
int64_t agoq_codes_bytes(int64_t numel, int bits);

/* Number of scales (groups); -1 if numel is not a positive multiple of group. */
int64_t agoq_num_groups(int64_t numel, int group);

/*
 * Dynamic Bit-width Compensation (paper: "Dynamic Bit-width Compensation",
 * Eq. (dynamic)).  Under interleaved 1F1B with n_stages pipeline stages,
 * stage i (1-based) holds N_i = 3*n_stages - 2*i + 1 micro-batches of
 * activations at its peak (11, 9, 7, 5 for four stages), and is given
 * B_i = 4*N_1/N_i bits, rounded to the nearest integer, at least 4 and at
 * most 8 (4, 5, 6, 8 for four stages).
 * agoq_dbca_stored_microbatches returns N_i, or -1 for bad arguments.
 * agoq_dbca_bits writes B_i to *bits_out; AGOQ_ERR_SHAPE for bad arguments.
 */
int agoq_dbca_stored_microbatches(int n_stages, int stage_1based);
int agoq_dbca_bits(int n_stages, int stage_1based, int *bits_out);

/*
 * Bit map of one decoder layer (paper: Table "memory_comparison", row AGoQ,
 * and "Other Operations": the stored tensors are the inputs of the two
 * RMSNorms, the input of the attention output projection, and the two inputs
 * of SiLU & Multiply; attention's own tensors stay in bf16).  The slots of
 * bits_out are, in order: norm1 input, out-proj input, norm2 input, gate, up.
 * agoq_layer_bitmap_native gives every stored tensor the stage's own width
 * B (4..8, from agoq_dbca_bits; there are no 7-bit codes, B=7 is stored at 6).
 * agoq_layer_bitmap realizes B with 4- and 8-bit codes only, as a mix: B=4 all
 * 4-bit; B=5 both norm inputs 8-bit; B=6 and B=7 norm inputs and gate 8-bit;
 * B=8 all 8-bit.
 */
enum { AGOQ_SLOT_NORM1_IN = 0, AGOQ_SLOT_OPROJ_IN = 1, AGOQ_SLOT_NORM2_IN = 2,
       AGOQ_SLOT_GATE = 3, AGOQ_SLOT_UP = 4, AGOQ_LAYER_SLOTS = 5 };
int agoq_layer_bitmap(int target_bits, int bits_out[AGOQ_LAYER_SLOTS]);
int agoq_layer_bitmap_native(int target_bits, int bits_out[AGOQ_LAYER_SLOTS]);

/*
 * Bytes that one layer's five stored tensors occupy under a bit map
 * (codes plus, if with_scales != 0, 4 bytes per group), for `tokens` rows,
 * model width `hidden` and MLP width `ffn`.  -1 for bad arguments.
 */
int64_t agoq_layer_stored_bytes(int64_t tokens, int64_t hidden, int64_t ffn, int group,
                                const int bits[AGOQ_LAYER_SLOTS], int with_scales);

/* Static string for a status code. */
const char *agoq_strerror(int status);

/*
 * Stochastic rounding -- an optional variant of the four integer-grid quantizers above.
 * The paper itself never uses it (its quantizers round to nearest); the variant exists for
 * callers that want the stored value to be unbiased, e.g. when a gradient is re-quantized at
 * every accumulation step.  Same arguments and layouts as the calls without the suffix, plus
 * `seed`; scales are identical to theirs, only the codes differ:
 *     code = max(floor(x * inv + u), -qmax),       u = B / 256
 * where x * inv is the rounded binary32 product, the sum is one binary32 addition, and B is
 * one byte of a 32-bit hash word shared by the four consecutive elements 4b .. 4b+3 of the
 * tensor being written (byte 0, the least significant, belongs to element 4b):
 *     key  = mix(seed ^ (high 32 bits of b) * 0x9E3779B9),   word = mix((low 32 bits of b) ^ key)
 * with mix() the 32-bit finalizer of MurmurHash3 (h ^= h >> 16; h *= 0x85EBCA6B;
 * h ^= h >> 13; h *= 0xC2B2AE35; h ^= h >> 16).  For the reduce and the accumulation the
 * element index is that of the OUTPUT element.  A call is a pure function of its inputs and
 * the seed: the same seed gives the same codes on every run and launch shape.  Dead and
 * non-finite groups follow the rule of the nearest-rounding calls.  Integer grids only.
 */
int agoq_act_quant_sr(const void *x_bf16, int64_t numel, int group, int bits, uint32_t seed, void *codes,
                      float *scales, void *stream);
int agoq_grad_quant_sr(const float *grad, int64_t numel, int group, uint32_t seed, int8_t *codes,
                       float *scales, void *stream);
int agoq_grad_reduce_requant_sr(const int8_t *in_codes, int64_t chunk_stride_codes, const float *in_scales,
                                int64_t chunk_stride_scales, int K, int64_t numel, int group,
                                uint32_t seed, int8_t *out_codes, float *out_scales, void *stream);
int agoq_grad_accumulate_sr(const int8_t *main_codes, const float *main_scales, const void *g_new,
                            int g_new_is_bf16, int64_t numel, int group, uint32_t seed,
                            int8_t *out_codes, float *out_scales, void *stream);

/*
 * Measurement aid (no passage of the paper: this is not part of the method).  A streaming
 * kernel with the memory traffic of an encode or decode kernel and none of its arithmetic:
 * lane item i loads load_bytes bytes from src + i*load_bytes and stores store_bytes bytes to
 * dst + i*store_bytes.  Its run time on a tensor's footprint is the floor that a single
 * launch with this access pattern can reach at all (ramp and drain of a launch and the
 * memory system's read/write mix included); the benchmark reports it beside the real
 * kernels on tensors small enough for that fixed cost to matter.
 *   load_bytes  : 4, 8 or 16            store_bytes : 0 (read only), 4, 8 or 16
 *   src : in,  items*load_bytes bytes   dst : out, items*store_bytes bytes (at least 4)
 *   (16 B -> 4 B is the traffic of the 4-bit quantize, 4 B -> 16 B of the 4-bit dequantize)
 * Errors: AGOQ_ERR_BITS for an unsupported width, AGOQ_ERR_SHAPE for items outside 1..2^36.
 */
int agoq_probe_stream(const void *src, int load_bytes, void *dst, int store_bytes, int64_t items,
                      void *stream);

/* Library version: major*10000 + minor*100 + patch. */
int agoq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AGOQ_H */
