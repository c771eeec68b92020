// Host-only helpers of the AGoQ C ABI: sizes, the Dynamic Bit-width Compensation rule,
// the per-layer bit map and its memory accounting.  Pure functions, no device access.

#include <stdint.h>

#include "agoq.h"

extern "C" {

int64_t agoq_codes_bytes(int64_t numel, int bits)
{
    if (numel < 0 || (bits != 4 && bits != 5 && bits != 6 && bits != 8)) return -1;
    return numel * bits / 8;
}

int64_t agoq_num_groups(int64_t numel, int group)
{
    if (group <= 0 || numel <= 0 || numel % group != 0) return -1;
    return numel / group;
}

// Paper, "Dynamic Bit-width Compensation": with four stages the devices hold 11, 9, 7, 5
// micro-batches, i.e. the first stage the most; N_i = n + 2(n - i) + 1.  (The formula as
// printed, n + 2i - 1, runs the other way and contradicts the numbers next to it.)
int agoq_dbca_stored_microbatches(int n_stages, int stage_1based)
{
    if (n_stages < 1 || stage_1based < 1 || stage_1based > n_stages) return -1;
    return n_stages + 2 * (n_stages - stage_1based) + 1;
}

// Eq. (dynamic): B_i = 4 N_1 / N_i, to the nearest integer (halves up), within [4, 8].
// Integer arithmetic: round(4 N_1 / N_i) = floor((8 N_1 + N_i) / (2 N_i)).
int agoq_dbca_bits(int n_stages, int stage_1based, int* bits_out)
{
    if (!bits_out) return AGOQ_ERR_NULL;
    const int ni = agoq_dbca_stored_microbatches(n_stages, stage_1based);
    if (ni < 0) return AGOQ_ERR_SHAPE;
    const int n1 = agoq_dbca_stored_microbatches(n_stages, 1);
    int b = (8 * n1 + ni) / (2 * ni);
    if (b < 4) b = 4;
    if (b > 8) b = 8;
    *bits_out = b;
    return AGOQ_OK;
}

int agoq_layer_bitmap(int target_bits, int bits_out[AGOQ_LAYER_SLOTS])
{
    if (!bits_out) return AGOQ_ERR_NULL;
    if (target_bits < 4 || target_bits > 8) return AGOQ_ERR_BITS;
    for (int s = 0; s < AGOQ_LAYER_SLOTS; ++s) bits_out[s] = target_bits == 8 ? 8 : 4;
    if (target_bits >= 5 && target_bits < 8) {
        bits_out[AGOQ_SLOT_NORM1_IN] = 8;
        bits_out[AGOQ_SLOT_NORM2_IN] = 8;
    }
    if (target_bits >= 6 && target_bits < 8) bits_out[AGOQ_SLOT_GATE] = 8;
    return AGOQ_OK;
}

int agoq_layer_bitmap_native(int target_bits, int bits_out[AGOQ_LAYER_SLOTS])
{
    if (!bits_out) return AGOQ_ERR_NULL;
    if (target_bits < 4 || target_bits > 8) return AGOQ_ERR_BITS;
    const int b = target_bits == 7 ? 6 : target_bits;   // no 7-bit codes: stay under the budget
    for (int s = 0; s < AGOQ_LAYER_SLOTS; ++s) bits_out[s] = b;
    return AGOQ_OK;
}

int64_t agoq_layer_stored_bytes(int64_t tokens, int64_t hidden, int64_t ffn, int group,
                                const int bits[AGOQ_LAYER_SLOTS], int with_scales)
{
    if (!bits || tokens <= 0 || hidden <= 0 || ffn <= 0 || group <= 0) return -1;
    if (hidden % group != 0 || ffn % group != 0) return -1;
    int64_t total = 0;
    for (int s = 0; s < AGOQ_LAYER_SLOTS; ++s) {
        const int64_t cols = (s == AGOQ_SLOT_GATE || s == AGOQ_SLOT_UP) ? ffn : hidden;
        const int64_t numel = tokens * cols;
        const int64_t code_bytes = agoq_codes_bytes(numel, bits[s]);
        if (code_bytes < 0) return -1;
        total += code_bytes;
        if (with_scales) total += 4 * (numel / group);
    }
    return total;
}

const char* agoq_strerror(int status)
{
    switch (status) {
    case AGOQ_OK: return "ok";
    case AGOQ_ERR_NULL: return "null pointer";
    case AGOQ_ERR_BITS: return "unsupported bit-width (4, 5, 6 or 8)";
    case AGOQ_ERR_GROUP: return "unsupported group size (64 or 128)";
    case AGOQ_ERR_SHAPE: return "numel must be a positive multiple of group; strides must cover the extents";
    case AGOQ_ERR_ALIGN: return "pointers and chunk strides must be 16-byte aligned";
    case AGOQ_ERR_K: return "K must be in 1..64";
    case AGOQ_ERR_HIP: return "HIP runtime error at launch";
    case AGOQ_ERR_COUNT: return "layer call: tensor count outside 1..8";
    default: return "unknown status";
    }
}

int agoq_version(void) { return 200; }

}  // extern "C"
