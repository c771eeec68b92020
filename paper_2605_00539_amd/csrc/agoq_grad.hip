// Gradient kernels: 8-bit store, dequantize, local accumulation, and the local
// dequantize -> fp32 sum -> requantize step of the 8-bit All-Reduce, for int8 codes and
// the E4M3 code book.
#include "agoq_device.hpp"

namespace {

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
        const bool keep = scale_and_inv<FP ? 448 : 127>(m, scale, inv);
        if (grp < n_groups) {
#pragma unroll
            for (int p = 0; p < VPL; ++p) {
                u32 w = encode4_bytes<FP>(v[u][p][0], v[u][p][1], v[u][p][2], v[u][p][3], inv);
                if (!keep) w = 0;   // dead group: no signed zeros; non-finite group: no codes
                st<NTS>(codes + grp * VPG + p * 16 + lane16, w);
            }
            if (lane16 == 0) st<NTS && AGOQ_SCALE_NT>(scales + grp, scale);
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
    const bool keep = scale_and_inv<FP ? 448 : 127>(m, scale, inv);
    if (valid) {
        u32x4 w = {0, 0, 0, 0};
#pragma unroll
        for (int d = 0; d < 4; ++d)
            w[d] = encode4_bytes<FP>(acc[4 * d], acc[4 * d + 1], acc[4 * d + 2], acc[4 * d + 3], inv);
        if (!keep) w = u32x4{0, 0, 0, 0};   // dead group: no signed zeros; non-finite: no codes
        st<AGOQ_RD_NTS>(out_codes + vi, w);
        if ((threadIdx.x & (LANES - 1)) == 0) st<AGOQ_RD_NTS && AGOQ_SCALE_NT>(out_scales + vi / LANES, scale);
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

// K known at compile time (4, 8, 16): RU 16-byte vectors per lane, all RU*K code loads and
// scale loads of the lane issued before the first is needed, then one vector after the
// other is summed, requantized and stored.
#ifndef AGOQ_RD_PRIO_FROM_K     // chunk count from which the loads are issued at raised priority; 0 = never
#define AGOQ_RD_PRIO_FROM_K 16
#endif
template <int GROUP, int KT, bool FP, int BLOCK, int RU>
__global__ __launch_bounds__(BLOCK) void grad_reduce_kernel(const int8_t* __restrict__ in_codes,
                                                     int64_t stride_codes,
                                                     const float* __restrict__ in_scales,
                                                     int64_t stride_scales, int64_t n_vec,
                                                     u32x4* __restrict__ out_codes,
                                                     float* __restrict__ out_scales)
{
    constexpr int LANES = GROUP / 16;
    constexpr bool NTC = AGOQ_RD_NTC, NTSC = AGOQ_RD_NTSC;
    const int64_t base = (int64_t)blockIdx.x * (BLOCK * RU) + threadIdx.x;
    u32x4 c[RU][KT];
    float s[RU][KT];
    // With 16 chunks and two vectors per lane a wavefront issues 64 loads; at raised priority
    // it issues them in one go instead of taking turns with the wavefront that is summing
    // (measured: +4 % at K = 16, nothing at K = 8, -1 % on the one-vector shape).
    constexpr bool kLoadsFirst = AGOQ_RD_PRIO_FROM_K > 0 && RU > 1 && KT >= AGOQ_RD_PRIO_FROM_K;
    if (kLoadsFirst) __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int64_t vi = base + (int64_t)u * BLOCK;
        const int64_t vc = vi < n_vec ? vi : 0;   // out-of-range lanes read vector 0, store nothing
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            c[u][k] = ld<NTC>((const u32x4*)(in_codes + (int64_t)k * stride_codes) + vc);
            s[u][k] = ld<NTSC>(in_scales + (int64_t)k * stride_scales + vc / LANES);
        }
    }
    if (kLoadsFirst) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
    }
    if (RU > 1) {
        // no load may be waited for after the first store has been issued
#pragma unroll
        for (int u = 0; u < RU; ++u)
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                need_now(c[u][k]);
                need_now(s[u][k]);
            }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int64_t vi = base + (int64_t)u * BLOCK;
        float acc[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int k = 0; k < KT; ++k) reduce_term<FP>(acc, c[u][k], s[u][k]);
        reduce_finish<GROUP, FP>(acc, vi, vi < n_vec, out_codes, out_scales);
    }
}

// Any other K (1..64): chunks four at a time, then the rest.
template <int GROUP, bool FP>
__global__ __launch_bounds__(AGOQ_RD_BLOCK) void grad_reduce_anyk_kernel(
    const int8_t* __restrict__ in_codes, int64_t stride_codes, const float* __restrict__ in_scales,
    int64_t stride_scales, int K, int64_t n_vec, u32x4* __restrict__ out_codes,
    float* __restrict__ out_scales)
{
    constexpr int LANES = GROUP / 16;
    constexpr bool NTC = AGOQ_RD_NTC, NTSC = AGOQ_RD_NTSC;
    const int64_t vi = (int64_t)blockIdx.x * AGOQ_RD_BLOCK + threadIdx.x;
    const bool valid = vi < n_vec;
    const int64_t vc = valid ? vi : 0;      // out-of-range lanes read vector 0, store nothing
    const int64_t grp = vc / LANES;
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
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
    reduce_finish<GROUP, FP>(acc, vi, valid, out_codes, out_scales);
}

// Launch of the reduce for either code book (arguments already checked).
// Measured on K = 8 and 16 streams of 7M to 218M elements: the kernel is fastest with
// FEWER wavefronts in flight than the registers allow -- two workgroups per compute unit
// (K = 8 on 218M elements: 6.5 TB/s against 5.8 at full occupancy) -- presumably because
// every resident wavefront keeps K DRAM pages open.  The cap is a dynamic LDS allocation
// that no kernel touches: 64 KB per workgroup lets two share a compute unit's 160 KB.
// From 40M elements on the two workgroups are of 256 lanes with two vectors per lane, below
// that of 512 lanes with one (+2 % at 27M elements, +10 % at 7M, -6 % at 218M).
constexpr size_t kTwoPerCuLds = 64 * 1024;
constexpr int64_t kReduceTwoVectorsFrom = 2500000;    // 16-element vectors
template <bool FP>
int launch_reduce(const int8_t* in_codes, int64_t stride_codes, const float* in_scales,
                  int64_t stride_scales, int K, int64_t n_vec, int group, u32x4* oc,
                  float* out_scales, hipStream_t st)
{
    const bool two = n_vec >= kReduceTwoVectorsFrom;
#ifndef AGOQ_RD1_BLOCK         // the small-tensor shape of the compile-time-K reduce
#define AGOQ_RD1_BLOCK 512
#endif
#ifndef AGOQ_RD1_RU
#define AGOQ_RD1_RU 1
#endif
#ifndef AGOQ_RD1_CAP_KB
#define AGOQ_RD1_CAP_KB 64
#endif
#ifndef AGOQ_RD2_BLOCK         // the large-tensor shape of the compile-time-K reduce
#define AGOQ_RD2_BLOCK 256
#endif
#ifndef AGOQ_RD2_RU
#define AGOQ_RD2_RU 2
#endif
#ifndef AGOQ_RD2_CAP_KB
#define AGOQ_RD2_CAP_KB 64
#endif
#define AGOQ_LAUNCH_REDUCE(G, KT)                                                               \
    if (two)                                                                                    \
        grad_reduce_kernel<G, KT, FP, AGOQ_RD2_BLOCK, AGOQ_RD2_RU><<<dim3(blocks_for(n_vec, AGOQ_RD2_BLOCK * AGOQ_RD2_RU)), dim3(AGOQ_RD2_BLOCK), (size_t)AGOQ_RD2_CAP_KB * 1024, st>>>( \
            in_codes, stride_codes, in_scales, stride_scales, n_vec, oc, out_scales);           \
    else                                                                                        \
        grad_reduce_kernel<G, KT, FP, AGOQ_RD1_BLOCK, AGOQ_RD1_RU><<<dim3(blocks_for(n_vec, AGOQ_RD1_BLOCK * AGOQ_RD1_RU)), dim3(AGOQ_RD1_BLOCK), (size_t)AGOQ_RD1_CAP_KB * 1024, st>>>( \
            in_codes, stride_codes, in_scales, stride_scales, n_vec, oc, out_scales)
#ifndef AGOQ_RD_SMALLK_BLOCK
#define AGOQ_RD_SMALLK_BLOCK 256
#endif
#ifndef AGOQ_RD_SMALLK_RU
#define AGOQ_RD_SMALLK_RU 2
#endif
#ifndef AGOQ_RD_SMALLK_CAP_KB
#define AGOQ_RD_SMALLK_CAP_KB 0
#endif
    // K = 1, 2 (and 3 in the run-time-K kernel): too few loads per vector to fill the memory
    // pipes under a cap; two vectors per lane and full occupancy instead (K = 1: 5.5 TB/s
    // against 3.9 capped, K = 2: 5.8 against 4.5, K = 3: 6.1 against 4.8)
#define AGOQ_LAUNCH_REDUCE_SMALLK(G, KT)                                                        \
    grad_reduce_kernel<G, KT, FP, AGOQ_RD_SMALLK_BLOCK, AGOQ_RD_SMALLK_RU>                      \
        <<<dim3(blocks_for(n_vec, AGOQ_RD_SMALLK_BLOCK * AGOQ_RD_SMALLK_RU)), dim3(AGOQ_RD_SMALLK_BLOCK), (size_t)AGOQ_RD_SMALLK_CAP_KB * 1024, st>>>( \
            in_codes, stride_codes, in_scales, stride_scales, n_vec, oc, out_scales)
#define AGOQ_LAUNCH_REDUCE_G(G)                                                                 \
    switch (K) {                                                                                \
    case 1: AGOQ_LAUNCH_REDUCE_SMALLK(G, 1); break;                                             \
    case 2: AGOQ_LAUNCH_REDUCE_SMALLK(G, 2); break;                                             \
    case 4: AGOQ_LAUNCH_REDUCE(G, 4); break;                                                    \
    case 8: AGOQ_LAUNCH_REDUCE(G, 8); break;                                                    \
    case 16: AGOQ_LAUNCH_REDUCE(G, 16); break;                                                  \
    default:                                                                                    \
        grad_reduce_anyk_kernel<G, FP><<<dim3(blocks_for(n_vec, AGOQ_RD_BLOCK)), dim3(AGOQ_RD_BLOCK), K < 4 ? 0 : kTwoPerCuLds, st>>>( \
            in_codes, stride_codes, in_scales, stride_scales, K, n_vec, oc, out_scales);        \
        break;                                                                                  \
    }
    if (group == 128) {
        AGOQ_LAUNCH_REDUCE_G(128)
    } else {
        AGOQ_LAUNCH_REDUCE_G(64)
    }
#undef AGOQ_LAUNCH_REDUCE_G
#undef AGOQ_LAUNCH_REDUCE_SMALLK
#undef AGOQ_LAUNCH_REDUCE
    return launch_status();
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
template <int GROUP, int UNROLL, bool FP = false>
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
    // Loads are unconditional (lanes past the end re-read the last group; only their stores
    // are masked): under a branch each, the compiler waits for the first loads before it
    // issues the last.
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t grp = (slot + (int64_t)u * kBlock) >> 4;
        const int64_t gc = grp < n_groups ? grp : n_groups - 1;
        s[u] = ld<true>(main_scales + gc);
#pragma unroll
        for (int p = 0; p < VPL; ++p) {
            v[u][p] = ld<true>(g_new + gc * VPG + p * 16 + lane16);
            c[u][p] = ld<true>(main_codes + gc * VPG + p * 16 + lane16);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t grp = (slot + (int64_t)u * kBlock) >> 4;
        float acc[VPL][4];
        u32 m = 0;
#pragma unroll
        for (int p = 0; p < VPL; ++p) {
            float q[4];
            decode4_bytes<FP>(c[u][p], q);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[p][j] = __fmaf_rn(q[j], s[u], v[u][p][j]);
                m = umax(m, as_u32(acc[p][j]) & 0x7FFFFFFFu);
            }
        }
        m = group_max_bits<16>(m);
        float scale, inv;
        const bool keep = scale_and_inv<FP ? 448 : 127>(m, scale, inv);
        if (grp < n_groups) {
#pragma unroll
            for (int p = 0; p < VPL; ++p) {
                u32 w = encode4_bytes<FP>(acc[p][0], acc[p][1], acc[p][2], acc[p][3], inv);
                if (!keep) w = 0;   // dead group: no signed zeros; non-finite group: no codes
                st<true>(out_codes + grp * VPG + p * 16 + lane16, w);
            }
            if (lane16 == 0) st<AGOQ_SCALE_NT>(out_scales + grp, scale);
        }
    }
}

template <int GROUP, int UNROLL, bool FP = false>
__global__ __launch_bounds__(AGOQ_GB_BLOCK) void grad_accumulate_bf16_kernel(
    const u32x2* main_codes, const float* main_scales, const u32x4* __restrict__ g_new,
    int64_t n_vec, u32x2* out_codes, float* out_scales)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = AGOQ_GB_BLOCK;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;

    // (Measured: this kernel is fastest as first written, each vector's three loads under
    // its bounds test, which the compiler turns into two batches of loads with a wait
    // between them; all six loads at once cost 3 %.)
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
        float acc[8], g[8], q0[4], q1[4];
        unpack8_bf16(v[u], g);
        decode4_bytes<FP>(c[u][0], q0);
        decode4_bytes<FP>(c[u][1], q1);
        u32 m = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[j] = __fmaf_rn(q0[j], s[u], g[j]);
            acc[4 + j] = __fmaf_rn(q1[j], s[u], g[4 + j]);
            m = umax(m, umax(as_u32(acc[j]) & 0x7FFFFFFFu, as_u32(acc[4 + j]) & 0x7FFFFFFFu));
        }
        m = group_max_bits<LANES>(m);
        float scale, inv;
        const bool keep = scale_and_inv<FP ? 448 : 127>(m, scale, inv);
        if (vi < n_vec) {
            u32 p0 = encode4_bytes<FP>(acc[0], acc[1], acc[2], acc[3], inv);
            u32 p1 = encode4_bytes<FP>(acc[4], acc[5], acc[6], acc[7], inv);
            if (!keep) p0 = p1 = 0;   // dead group: no signed zeros; non-finite group: no codes
            st<true>(out_codes + vi, u32x2{p0, p1});
            if ((threadIdx.x & (LANES - 1)) == 0) st<AGOQ_SCALE_NT>(out_scales + vi / LANES, scale);
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
    // loads (unconditional: a lane past the end re-reads the last vector and stores nothing),
    // one point where all of them are waited for, then arithmetic and stores vector by vector
    u32 c[UNROLL];
    float s[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        const int64_t vc = vi < n_vec ? vi : n_vec - 1;
        c[u] = ld<true>(codes + vc);
        s[u] = ld<false>(scales + vc / LANES);
    }
    if (UNROLL > 1) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            need_now(c[u]);
            need_now(s[u]);
        }
        __builtin_amdgcn_sched_barrier(0);
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
        if (UNROLL > 1) __builtin_amdgcn_sched_barrier(0);
    }
}

// Validation and launch shared by the int8 and E4M3 forms of the local accumulation.
template <bool FP>
int launch_accumulate(const void* main_codes, const float* main_scales, const void* g_new,
                      int g_new_is_bf16, int64_t numel, int group, void* out_codes,
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
        constexpr int U = AGOQ_GB_UNROLL;
        const dim3 grid(blocks_for(n_vec, AGOQ_GB_BLOCK * U)), block(AGOQ_GB_BLOCK);
        if (group == 128)
            grad_accumulate_bf16_kernel<128, U, FP><<<grid, block, kCapLds, st>>>(
                (const u32x2*)main_codes, main_scales, (const u32x4*)g_new, n_vec,
                (u32x2*)out_codes, out_scales);
        else
            grad_accumulate_bf16_kernel<64, U, FP><<<grid, block, kCapLds, st>>>(
                (const u32x2*)main_codes, main_scales, (const u32x4*)g_new, n_vec,
                (u32x2*)out_codes, out_scales);
    } else {
        const int64_t n_groups = numel / group;
        constexpr int U = AGOQ_GQ_UNROLL;
        const dim3 grid(blocks_for(n_groups * 16, AGOQ_GQ_BLOCK * U)), block(AGOQ_GQ_BLOCK);
        if (group == 128)
            grad_accumulate_f32_kernel<128, U, FP><<<grid, block, kCapGa, st>>>(
                (const u32*)main_codes, main_scales, (const f32x4*)g_new, n_groups,
                (u32*)out_codes, out_scales);
        else
            grad_accumulate_f32_kernel<64, U, FP><<<grid, block, kCapGa, st>>>(
                (const u32*)main_codes, main_scales, (const f32x4*)g_new, n_groups,
                (u32*)out_codes, out_scales);
    }
    return launch_status();
}

}  // namespace

extern "C" {

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
        grad_quant_kernel<128, U><<<grid, block, kCapLds, st>>>((const f32x4*)grad, n_groups, (u32*)codes,
                                                          scales);
    else
        grad_quant_kernel<64, U><<<grid, block, kCapLds, st>>>((const f32x4*)grad, n_groups, (u32*)codes,
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
    return launch_reduce<false>(in_codes, chunk_stride_codes, in_scales, chunk_stride_scales, K,
                                numel / 16, group, (u32x4*)out_codes, out_scales,
                                (hipStream_t)stream);
}

int agoq_grad_accumulate(const int8_t* main_codes, const float* main_scales, const void* g_new,
                         int g_new_is_bf16, int64_t numel, int group, int8_t* out_codes,
                         float* out_scales, void* stream)
{
    return launch_accumulate<false>(main_codes, main_scales, g_new, g_new_is_bf16, numel, group,
                                    out_codes, out_scales, stream);
}

int agoq_fp8_grad_accumulate(const uint8_t* main_codes, const float* main_scales, const void* g_new,
                             int g_new_is_bf16, int64_t numel, int group, uint8_t* out_codes,
                             float* out_scales, void* stream)
{
    return launch_accumulate<true>(main_codes, main_scales, g_new, g_new_is_bf16, numel, group,
                                   out_codes, out_scales, stream);
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
        grad_dequant_kernel<128, U><<<grid, block, kCapGd, st>>>((const u32*)codes, scales, n_vec,
                                                            (f32x4*)out);
    else
        grad_dequant_kernel<64, U><<<grid, block, kCapGd, st>>>((const u32*)codes, scales, n_vec,
                                                           (f32x4*)out);
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
        grad_quant_kernel<128, U, true><<<grid, block, kCapLds, st>>>((const f32x4*)grad, n_groups,
                                                                (u32*)codes, scales);
    else
        grad_quant_kernel<64, U, true><<<grid, block, kCapLds, st>>>((const f32x4*)grad, n_groups,
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
        grad_dequant_kernel<128, U, true><<<grid, block, kCapGd, st>>>((const u32*)codes, scales, n_vec,
                                                                  (f32x4*)out);
    else
        grad_dequant_kernel<64, U, true><<<grid, block, kCapGd, st>>>((const u32*)codes, scales, n_vec,
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
    return launch_reduce<true>((const int8_t*)in_codes, chunk_stride_codes, in_scales,
                               chunk_stride_scales, K, numel / 16, group, (u32x4*)out_codes,
                               out_scales, (hipStream_t)stream);
}

}  // extern "C"
