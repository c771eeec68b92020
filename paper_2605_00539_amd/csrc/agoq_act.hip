// Activation storage kernels: bf16 -> packed codes + fp32 scales (quantize), and back
// (dequantize), for 4-, 5-, 6- and 8-bit integer codes and the E2M1 code book.
#include "agoq_device.hpp"

namespace {

// ---------------------------------------------------------------------------
// Activation quantize: bf16 -> 4-, 5-, 6- or 8-bit codes + fp32 scale per group.
// One lane owns 8 consecutive elements (one 16-byte load) of a group;
// GROUP/8 consecutive lanes own a group.  5- and 6-bit codes go to two planes:
// the low nibbles exactly where 4-bit codes would go, the remaining high bits
// (one byte or two bytes per lane) to a second plane that starts n_vec*4 bytes in.
// ---------------------------------------------------------------------------
// A tile runs in three phases with nothing moved across their borders: every load of the
// lane; then everything that needs the loaded data; then the encoding and the stores.  A
// load that is waited for after a store has been issued would also wait for that store to
// be acknowledged (one counter orders both), which costs more than the load itself.
// FULL: the whole tile lies inside the tensor and the code has no bounds test at all (with
// one, the compiler sinks loads and arithmetic into the guarded store blocks and the
// phases are gone).  Otherwise -- the one workgroup that straddles the end -- a lane past
// the end re-reads the last vector, which is always in bounds, and its stores are masked;
// lanes of one group are all inside or all outside.
template <int BITS, int GROUP, int UNROLL, bool FP, bool FULL, bool SR>
__device__ __forceinline__ void act_quant_body(const u32x4* __restrict__ x, int64_t n_vec,
                                               void* __restrict__ codes, float* __restrict__ scales,
                                               unsigned block, u32 seed)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = kAqBlock;
    constexpr bool NTL = true, NTS = true;
    const int64_t base = (int64_t)block * (kBlock * UNROLL) + threadIdx.x;

    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        v[u] = ld<NTL>(x + (FULL || vi < n_vec ? vi : n_vec - 1));
    }
    float f[UNROLL][8];
    u32 m[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) m[u] = group_max_bits<LANES>(unpack8_bf16(v[u], f[u]));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        quantize_store8<BITS, GROUP, FP, NTS, SR>(f[u], m[u], vi, n_vec, FULL || vi < n_vec, codes, scales, seed);
    }
}

template <int BITS, int GROUP, int UNROLL, bool FP, bool SR = false>
__device__ __forceinline__ void act_quant_tile(const u32x4* __restrict__ x, int64_t n_vec,
                                               void* __restrict__ codes, float* __restrict__ scales,
                                               unsigned block, u32 seed = 0)
{
    if (((int64_t)block + 1) * (kAqBlock * UNROLL) <= n_vec)
        act_quant_body<BITS, GROUP, UNROLL, FP, true, SR>(x, n_vec, codes, scales, block, seed);
    else
        act_quant_body<BITS, GROUP, UNROLL, FP, false, SR>(x, n_vec, codes, scales, block, seed);
}

// SR: the codes are rounded stochastically under `seed` (optional variant; else seed is unused).
template <int BITS, int GROUP, int UNROLL, bool FP = false, bool SR = false>
__global__ __launch_bounds__(kAqBlock) void act_quant_kernel(const u32x4* __restrict__ x,
                                                           int64_t n_vec, void* __restrict__ codes,
                                                           float* __restrict__ scales, u32 seed)
{
    act_quant_tile<BITS, GROUP, UNROLL, FP, SR>(x, n_vec, codes, scales, blockIdx.x, seed);
}

// ---------------------------------------------------------------------------
// Activation dequantize: codes + scales -> bf16.  One lane produces 8 elements
// (one 16-byte store).
// ---------------------------------------------------------------------------
// PACE: a lane waits for each store to be acknowledged before it starts on its next vector.
// Measured to help in one case only, 8-bit codes of a tensor small enough for the whole
// grid to be resident at once, where it keeps the burst of stores at the end of the single
// generation of wavefronts from piling up.
template <int BITS, int GROUP, int UNROLL, bool FP, bool FULL, bool PACE>
__device__ __forceinline__ void act_dequant_body(const void* __restrict__ codes,
                                                 const float* __restrict__ scales, int64_t n_vec,
                                                 u32x4* __restrict__ y, unsigned block)
{
    static_assert(!FP || BITS == 4, "the floating-point activation code book is E2M1");
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = kDqBlock;
    constexpr bool NTC = true, NTSC = false, NTS = true;
    const int64_t base = (int64_t)block * (kBlock * UNROLL) + threadIdx.x;

    // loads; decode (uses every loaded value); pack and store -- see act_quant_body
    Codes8<BITS> c[UNROLL];
    float s[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        const int64_t vc = FULL || vi < n_vec ? vi : n_vec - 1;
        c[u] = load_codes8<BITS, NTC>(codes, n_vec, vc);
        s[u] = ld<NTSC>(scales + vc / LANES);
    }
    // phase border: every loaded register is needed here, so every wait happens here
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        need_now(c[u]);
        need_now(s[u]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        float q[8], f[8];
        if constexpr (FP) {
            decode8_e2m1(c[u].lo, q);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = decode8<BITS>(c[u], j);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] = __fmul_rn(q[j], s[u]);
        if (FULL || vi < n_vec)
            st<NTS>(y + vi, u32x4{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                                  pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7])});
        if (PACE && u + 1 < UNROLL) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);   // the next vector's arithmetic stays behind this store
    }
}

template <int BITS, int GROUP, int UNROLL, bool FP, bool PACE = false>
__device__ __forceinline__ void act_dequant_tile(const void* __restrict__ codes,
                                                 const float* __restrict__ scales, int64_t n_vec,
                                                 u32x4* __restrict__ y, unsigned block)
{
    if (((int64_t)block + 1) * (kDqBlock * UNROLL) <= n_vec)
        act_dequant_body<BITS, GROUP, UNROLL, FP, true, PACE>(codes, scales, n_vec, y, block);
    else
        act_dequant_body<BITS, GROUP, UNROLL, FP, false, PACE>(codes, scales, n_vec, y, block);
}

template <int BITS, int GROUP, int UNROLL, bool FP = false, bool PACE = false>
__global__ __launch_bounds__(kDqBlock) void act_dequant_kernel(const void* __restrict__ codes,
                                                             const float* __restrict__ scales,
                                                             int64_t n_vec, u32x4* __restrict__ y)
{
    act_dequant_tile<BITS, GROUP, UNROLL, FP, PACE>(codes, scales, n_vec, y, blockIdx.x);
}

// ---------------------------------------------------------------------------
// The stored tensors of one layer in one launch.  Consecutive ranges of workgroups serve
// consecutive tensors, each at its own code width; a workgroup finds its tensor from the
// table of first workgroup indices (all scalar work) and then runs the single-tensor tile.
// A launch costs a few microseconds of ramp and drain whatever its size, which is a third
// of the run time of a 32 MiB tensor: one launch per layer pays it once.
// ---------------------------------------------------------------------------
struct LayerArgs {
    const void* src[AGOQ_MAX_LAYER_SLOTS];   // quantize: bf16 input; dequantize: codes
    void* dst[AGOQ_MAX_LAYER_SLOTS];         // quantize: codes; dequantize: bf16 output
    float* scales[AGOQ_MAX_LAYER_SLOTS];
    int64_t n_vec[AGOQ_MAX_LAYER_SLOTS];
    unsigned first_block[AGOQ_MAX_LAYER_SLOTS];  // unused entries hold 0xFFFFFFFF
    int bits[AGOQ_MAX_LAYER_SLOTS];
};

__device__ __forceinline__ int layer_slot_of(const LayerArgs& a, unsigned block)
{
    int t = 0;
#pragma unroll
    for (int i = 1; i < AGOQ_MAX_LAYER_SLOTS; ++i) t += block >= a.first_block[i] ? 1 : 0;
    return t;
}

// Vectors per lane in the layer dequantize (measured on 8B-shaped layers at seq 4096 and
// 8192 under every stage map: two for every width is best or within 1% of best).
constexpr int kLayerDqUnroll8 = 2;   // 8-bit codes
constexpr int kLayerDqUnroll = 2;    // 4-, 5- and 6-bit codes

template <int GROUP>
__global__ __launch_bounds__(kAqBlock) void act_quant_layer_kernel(const LayerArgs a)
{
    const int t = layer_slot_of(a, blockIdx.x);
    const unsigned block = blockIdx.x - a.first_block[t];
    const u32x4* x = (const u32x4*)a.src[t];
    void* codes = a.dst[t];
    float* scales = a.scales[t];
    const int64_t n_vec = a.n_vec[t];
    switch (a.bits[t]) {
    case 4: act_quant_tile<4, GROUP, kAqUnroll, false>(x, n_vec, codes, scales, block); break;
    case 5: act_quant_tile<5, GROUP, kAqUnroll, false>(x, n_vec, codes, scales, block); break;
    case 6: act_quant_tile<6, GROUP, kAqUnroll, false>(x, n_vec, codes, scales, block); break;
    default: act_quant_tile<8, GROUP, kAqUnroll, false>(x, n_vec, codes, scales, block); break;
    }
}

template <int GROUP>
__global__ __launch_bounds__(kDqBlock) void act_dequant_layer_kernel(const LayerArgs a)
{
    const int t = layer_slot_of(a, blockIdx.x);
    const unsigned block = blockIdx.x - a.first_block[t];
    const void* codes = a.src[t];
    const float* scales = a.scales[t];
    u32x4* y = (u32x4*)a.dst[t];
    const int64_t n_vec = a.n_vec[t];
    switch (a.bits[t]) {
    case 4: act_dequant_tile<4, GROUP, kLayerDqUnroll, false>(codes, scales, n_vec, y, block); break;
    case 5: act_dequant_tile<5, GROUP, kLayerDqUnroll, false>(codes, scales, n_vec, y, block); break;
    case 6: act_dequant_tile<6, GROUP, kLayerDqUnroll, false>(codes, scales, n_vec, y, block); break;
    default: act_dequant_tile<8, GROUP, kLayerDqUnroll8, false>(codes, scales, n_vec, y, block); break;
    }
}

// Validates the slots of a layer call and lays out the workgroup ranges.
int layer_args(const agoq_act_slot* slots, int count, int group, bool quantize, LayerArgs& a,
               unsigned& total_blocks)
{
    if (!slots) return AGOQ_ERR_NULL;
    if (count < 1 || count > AGOQ_MAX_LAYER_SLOTS) return AGOQ_ERR_COUNT;
    if (group != 64 && group != 128) return AGOQ_ERR_GROUP;
    uint64_t blocks = 0;
    for (int i = 0; i < AGOQ_MAX_LAYER_SLOTS; ++i) {
        a.src[i] = nullptr;
        a.dst[i] = nullptr;
        a.scales[i] = nullptr;
        a.n_vec[i] = 0;
        a.first_block[i] = 0xFFFFFFFFu;
        a.bits[i] = 8;
    }
    for (int i = 0; i < count; ++i) {
        const agoq_act_slot& s = slots[i];
        if (!s.bf16 || !s.codes || !s.scales) return AGOQ_ERR_NULL;
        if (s.bits != 4 && s.bits != 5 && s.bits != 6 && s.bits != 8) return AGOQ_ERR_BITS;
        if (int rc = check_common(s.numel, group)) return rc;
        if (misaligned(s.bf16) || misaligned(s.codes) || misaligned(s.scales)) return AGOQ_ERR_ALIGN;
        const int64_t n_vec = s.numel / 8;
        const int per_block = quantize ? kAqBlock * kAqUnroll
                                       : kDqBlock * (s.bits == 8 ? kLayerDqUnroll8 : kLayerDqUnroll);
        a.src[i] = quantize ? (const void*)s.bf16 : (const void*)s.codes;
        a.dst[i] = quantize ? s.codes : s.bf16;
        a.scales[i] = s.scales;
        a.n_vec[i] = n_vec;
        a.bits[i] = s.bits;
        a.first_block[i] = (unsigned)blocks;
        blocks += (uint64_t)((n_vec + per_block - 1) / per_block);
        if (blocks > 0x7FFFFFFFull) return AGOQ_ERR_SHAPE;
    }
    total_blocks = (unsigned)blocks;
    return AGOQ_OK;
}

}  // namespace

extern "C" {

}  // extern "C"

namespace {

template <bool SR>
int launch_act_quant(const void* x_bf16, int64_t numel, int group, int bits, u32 seed, void* codes,
                     float* scales, void* stream)
{
    if (!x_bf16 || !codes || !scales) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    const dim3 grid(blocks_for(n_vec, kAqBlock * kAqUnroll)), block(kAqBlock);
    return dispatch_bits_group(bits, group, [&](auto b, auto g) {
        return launch(act_quant_kernel<decltype(b)::value, decltype(g)::value, kAqUnroll, false, SR>, grid,
                      block, 0, (hipStream_t)stream, (const u32x4*)x_bf16, n_vec, codes, scales, seed);
    });
}

}  // namespace

extern "C" {

int agoq_act_quant(const void* x_bf16, int64_t numel, int group, int bits, void* codes,
                   float* scales, void* stream)
{
    return launch_act_quant<false>(x_bf16, numel, group, bits, 0, codes, scales, stream);
}

int agoq_act_quant_sr(const void* x_bf16, int64_t numel, int group, int bits, uint32_t seed, void* codes,
                      float* scales, void* stream)
{
    return launch_act_quant<true>(x_bf16, numel, group, bits, seed, codes, scales, stream);
}

int agoq_act_dequant(const void* codes, const float* scales, int64_t numel, int group, int bits,
                     void* y_bf16, void* stream)
{
    if (!codes || !scales || !y_bf16) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(codes) || misaligned(scales) || misaligned(y_bf16)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    // measured: a tensor small enough for (about) the whole grid to be resident at once runs
    // best with four vectors per lane, 8-bit codes then with paced stores; larger tensors
    // with two
    // ("about": up to one and a half rounds; for 8-bit codes exactly one).  5- and 6-bit
    // codes, with three loads per vector, stay at two vectors per lane at every size
    // (+2 to +5 % on 8M to 21M elements, nothing from 33M on).
    const bool small = bits == 8   ? fits_rounds(n_vec, kDqBlock, 4, 1, 1)
                       : bits == 4 ? fits_rounds(n_vec, kDqBlock, 4, 3, 2)
                                   : false;
    const int unroll = small ? 4 : 2;
    const dim3 grid(blocks_for(n_vec, kDqBlock * unroll)), block(kDqBlock);
    const size_t cap = (bits == 8 && !small) ? kCapDq8 : 0;
    hipStream_t st = (hipStream_t)stream;
    u32x4* y = (u32x4*)y_bf16;
    return dispatch_bits_group(bits, group, [&](auto b, auto g) {
        constexpr int B = decltype(b)::value, G = decltype(g)::value;
        if (small && B == 8)
            return launch(act_dequant_kernel<B, G, 4, false, B == 8>, grid, block, cap, st, codes, scales, n_vec, y);
        if (small) return launch(act_dequant_kernel<B, G, 4>, grid, block, cap, st, codes, scales, n_vec, y);
        return launch(act_dequant_kernel<B, G, 2>, grid, block, cap, st, codes, scales, n_vec, y);
    });
}

int agoq_fp4_act_quant(const void* x_bf16, int64_t numel, int group, void* codes, float* scales,
                       void* stream)
{
    if (!x_bf16 || !codes || !scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    const dim3 grid(blocks_for(n_vec, kAqBlock * kAqUnroll)), block(kAqBlock);
    hipStream_t st = (hipStream_t)stream;
    const u32x4* x = (const u32x4*)x_bf16;
    if (group == 128)
        return launch(act_quant_kernel<4, 128, kAqUnroll, true>, grid, block, 0, st, x, n_vec, codes, scales, 0u);
    return launch(act_quant_kernel<4, 64, kAqUnroll, true>, grid, block, 0, st, x, n_vec, codes, scales, 0u);
}

int agoq_fp4_act_dequant(const void* codes, const float* scales, int64_t numel, int group,
                         void* y_bf16, void* stream)
{
    if (!codes || !scales || !y_bf16) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(codes) || misaligned(scales) || misaligned(y_bf16)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    const bool small = fits_rounds(n_vec, kDqBlock, 4, 3, 2);   // as for 4-bit integer codes
    const dim3 grid(blocks_for(n_vec, kDqBlock * (small ? 4 : 2))), block(kDqBlock);
    hipStream_t st = (hipStream_t)stream;
    u32x4* y = (u32x4*)y_bf16;
    if (group == 128) {
        if (small) return launch(act_dequant_kernel<4, 128, 4, true>, grid, block, 0, st, codes, scales, n_vec, y);
        return launch(act_dequant_kernel<4, 128, 2, true>, grid, block, 0, st, codes, scales, n_vec, y);
    }
    if (small) return launch(act_dequant_kernel<4, 64, 4, true>, grid, block, 0, st, codes, scales, n_vec, y);
    return launch(act_dequant_kernel<4, 64, 2, true>, grid, block, 0, st, codes, scales, n_vec, y);
}

int agoq_act_quant_layer(const agoq_act_slot* slots, int count, int group, void* stream)
{
    LayerArgs a;
    unsigned blocks = 0;
    if (int rc = layer_args(slots, count, group, true, a, blocks)) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (group == 128) return launch(act_quant_layer_kernel<128>, dim3(blocks), dim3(kAqBlock), 0, st, a);
    return launch(act_quant_layer_kernel<64>, dim3(blocks), dim3(kAqBlock), 0, st, a);
}

int agoq_act_dequant_layer(const agoq_act_slot* slots, int count, int group, void* stream)
{
    LayerArgs a;
    unsigned blocks = 0;
    if (int rc = layer_args(slots, count, group, false, a, blocks)) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (group == 128) return launch(act_dequant_layer_kernel<128>, dim3(blocks), dim3(kDqBlock), kCapLdq, st, a);
    return launch(act_dequant_layer_kernel<64>, dim3(blocks), dim3(kDqBlock), kCapLdq, st, a);
}

}  // extern "C"
