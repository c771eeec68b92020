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
template <int GROUP, int UNROLL, bool FP = false, bool SR = false>
__global__ __launch_bounds__(kGqBlock) void grad_quant_kernel(const f32x4* __restrict__ g,
                                                            int64_t n_groups,
                                                            u32* __restrict__ codes,
                                                            float* __restrict__ scales, u32 seed)
{
    constexpr int VPL = GROUP / 64;   // vectors per lane: 1 (group 64) or 2 (group 128)
    constexpr int VPG = GROUP / 4;    // vectors per group
    constexpr int kBlock = kGqBlock;
    constexpr bool NTL = true, NTS = true;
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
                // the vector's four elements are 4 * (its index) ..: its index is their block
                const int64_t vec = grp * VPG + p * 16 + lane16;
                u32 w = encode4_bytes<FP, SR>(v[u][p][0], v[u][p][1], v[u][p][2], v[u][p][3], inv, seed, vec);
                if (!keep) w = 0;   // dead group: no signed zeros; non-finite group: no codes
                st<NTS>(codes + vec, w);
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
template <int GROUP, bool FP = false, bool SR = false>
__device__ __forceinline__ void reduce_finish(const float (&acc)[16], int64_t vi,
                                              bool valid, u32x4* __restrict__ out_codes,
                                              float* __restrict__ out_scales, u32 seed = 0)
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
            w[d] = encode4_bytes<FP, SR>(acc[4 * d], acc[4 * d + 1], acc[4 * d + 2], acc[4 * d + 3], inv, seed,
                                         4 * vi + d);   // the lane's elements are 16 * vi ..: four blocks
        if (!keep) w = u32x4{0, 0, 0, 0};   // dead group: no signed zeros; non-finite: no codes
        st<true>(out_codes + vi, w);
        if ((threadIdx.x & (LANES - 1)) == 0) st<true>(out_scales + vi / LANES, scale);
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

// K known at compile time: RU 16-byte vectors per lane, all RU*K code loads and scale loads
// of the lane issued before the first is needed, then one vector after the other is summed,
// requantized and stored.
constexpr int kReducePrioFromK = 16;   // chunk count from which the loads are issued at raised priority
template <int GROUP, int KT, bool FP, int BLOCK, int RU, bool SR = false>
__global__ __launch_bounds__(BLOCK) void grad_reduce_kernel(const int8_t* __restrict__ in_codes,
                                                     int64_t stride_codes,
                                                     const float* __restrict__ in_scales,
                                                     int64_t stride_scales, int64_t n_vec,
                                                     u32x4* __restrict__ out_codes,
                                                     float* __restrict__ out_scales, u32 seed)
{
    constexpr int LANES = GROUP / 16;
    const int64_t base = (int64_t)blockIdx.x * (BLOCK * RU) + threadIdx.x;
    u32x4 c[RU][KT];
    float s[RU][KT];
    // With 16 chunks and two vectors per lane a wavefront issues 64 loads; at raised priority
    // it issues them in one go instead of taking turns with the wavefront that is summing
    // (measured: +4 % at K = 16, nothing at K = 8, -1 % on the one-vector shape).
    constexpr bool kLoadsFirst = RU > 1 && KT >= kReducePrioFromK;
    if (kLoadsFirst) __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int64_t vi = base + (int64_t)u * BLOCK;
        const int64_t vc = vi < n_vec ? vi : 0;   // out-of-range lanes read vector 0, store nothing
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            c[u][k] = ld<true>((const u32x4*)(in_codes + (int64_t)k * stride_codes) + vc);
            s[u][k] = ld<true>(in_scales + (int64_t)k * stride_scales + vc / LANES);
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
        reduce_finish<GROUP, FP, SR>(acc, vi, vi < n_vec, out_codes, out_scales, seed);
    }
}

// Any K (1..64) at run time: chunks k .. k+N-1 of the lane's vector, loads first, then the
// N terms in chunk order.
template <int N, bool FP, int LANES>
__device__ __forceinline__ void reduce_batch(float (&acc)[16], const int8_t* __restrict__ in_codes,
                                             int64_t stride_codes, const float* __restrict__ in_scales,
                                             int64_t stride_scales, int k, int64_t vc)
{
    u32x4 c[N];
    float s[N];
#pragma unroll
    for (int t = 0; t < N; ++t) {
        c[t] = ld<true>((const u32x4*)(in_codes + (int64_t)(k + t) * stride_codes) + vc);
        s[t] = ld<true>(in_scales + (int64_t)(k + t) * stride_scales + vc / LANES);
    }
#pragma unroll
    for (int t = 0; t < N; ++t) reduce_term<FP>(acc, c[t], s[t]);
}

// Four chunks at a time, then the remaining one to three together (one at a time they would
// each wait a full memory latency).
constexpr int kAnyKBlock = 512;
template <int GROUP, bool FP, bool SR = false>
__global__ __launch_bounds__(kAnyKBlock) void grad_reduce_anyk_kernel(
    const int8_t* __restrict__ in_codes, int64_t stride_codes, const float* __restrict__ in_scales,
    int64_t stride_scales, int K, int64_t n_vec, u32x4* __restrict__ out_codes,
    float* __restrict__ out_scales, u32 seed)
{
    constexpr int LANES = GROUP / 16;
    const int64_t vi = (int64_t)blockIdx.x * kAnyKBlock + threadIdx.x;
    const bool valid = vi < n_vec;
    const int64_t vc = valid ? vi : 0;      // out-of-range lanes read vector 0, store nothing
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
    int k = 0;
    for (; k + 4 <= K; k += 4)
        reduce_batch<4, FP, LANES>(acc, in_codes, stride_codes, in_scales, stride_scales, k, vc);
    switch (K - k) {
    case 3: reduce_batch<3, FP, LANES>(acc, in_codes, stride_codes, in_scales, stride_scales, k, vc); break;
    case 2: reduce_batch<2, FP, LANES>(acc, in_codes, stride_codes, in_scales, stride_scales, k, vc); break;
    case 1: reduce_batch<1, FP, LANES>(acc, in_codes, stride_codes, in_scales, stride_scales, k, vc); break;
    default: break;
    }
    reduce_finish<GROUP, FP, SR>(acc, vi, valid, out_codes, out_scales, seed);
}

// Launch of the reduce for either code book (arguments already checked).  Measured on
// 13M to 218M elements per chunk, K = 1..64:
//   * Large tensors (from 40M elements) with a chunk count that has a compile-time kernel
//     (5, 6, 7, 8, 12, 16) are fastest with FEWER wavefronts in flight than the registers
//     allow -- two workgroups of 256 lanes per compute unit, two vectors per lane (K = 8 on
//     218M elements: 6.5 TB/s against 5.8 at full occupancy) -- presumably because every
//     resident wavefront keeps K DRAM pages open.  The cap is a dynamic LDS allocation that no
//     kernel touches: 64 KB per workgroup lets two share a compute unit's 160 KB.
//   * K = 8 below that size: the same cap, workgroups of 512 lanes with one vector each.
//   * K = 1, 2: too few loads per vector to fill the memory pipes under a cap; two vectors
//     per lane at full occupancy.
//   * K = 3, 4, 5 below that size: compile-time kernels at full occupancy, one vector per
//     lane (1-3 % ahead of the run-time-K kernel on 13M and 27M elements).
//   * Everything else runs the run-time-K kernel at full occupancy: 73-77 % of peak for
//     K = 6..64 on a 27M-element shard, 76-81 % for K = 3, 4 on 218M elements (where the
//     capped compile-time kernels for K = 4 measured 76 %).
constexpr size_t kTwoPerCuLds = 64 * 1024;
constexpr int64_t kReduceTwoVectorsFrom = 2500000;    // 16-element vectors
struct ReduceArgs {
    const int8_t* in_codes;
    int64_t stride_codes;
    const float* in_scales;
    int64_t stride_scales;
    int K;
    int64_t n_vec;
    u32x4* out_codes;
    float* out_scales;
    hipStream_t st;
    u32 seed;            // stochastic rounding only
};

template <int GROUP, int KT, bool FP, int BLOCK, int RU, bool SR = false>
int launch_reduce_kt(const ReduceArgs& a, size_t lds)
{
    return launch(grad_reduce_kernel<GROUP, KT, FP, BLOCK, RU, SR>, dim3(blocks_for(a.n_vec, BLOCK * RU)),
                  dim3(BLOCK), lds, a.st, a.in_codes, a.stride_codes, a.in_scales, a.stride_scales,
                  a.n_vec, a.out_codes, a.out_scales, a.seed);
}

template <int GROUP, bool FP, bool SR>
int launch_reduce_group(const ReduceArgs& a)
{
    const bool large = a.n_vec >= kReduceTwoVectorsFrom;
    // the stochastic variant has the compile-time shapes of K = 8 only, and runs the
    // run-time-K kernel for every other chunk count
    if constexpr (SR) {
        if (a.K == 8)
            return large ? launch_reduce_kt<GROUP, 8, FP, 256, 2, true>(a, kTwoPerCuLds)
                         : launch_reduce_kt<GROUP, 8, FP, 512, 1, true>(a, kTwoPerCuLds);
        return launch(grad_reduce_anyk_kernel<GROUP, FP, true>, dim3(blocks_for(a.n_vec, kAnyKBlock)),
                      dim3(kAnyKBlock), 0, a.st, a.in_codes, a.stride_codes, a.in_scales, a.stride_scales, a.K,
                      a.n_vec, a.out_codes, a.out_scales, a.seed);
    }
    switch (a.K) {
    case 1: return launch_reduce_kt<GROUP, 1, FP, 256, 2>(a, 0);
    case 2: return launch_reduce_kt<GROUP, 2, FP, 256, 2>(a, 0);
    case 8:
        return large ? launch_reduce_kt<GROUP, 8, FP, 256, 2>(a, kTwoPerCuLds)
                     : launch_reduce_kt<GROUP, 8, FP, 512, 1>(a, kTwoPerCuLds);
    case 3: if (!large) return launch_reduce_kt<GROUP, 3, FP, 512, 1>(a, 0); break;
    case 4: if (!large) return launch_reduce_kt<GROUP, 4, FP, 512, 1>(a, 0); break;
    case 5:
        return large ? launch_reduce_kt<GROUP, 5, FP, 256, 2>(a, kTwoPerCuLds)
                     : launch_reduce_kt<GROUP, 5, FP, 512, 1>(a, 0);
    case 6: if (large) return launch_reduce_kt<GROUP, 6, FP, 256, 2>(a, kTwoPerCuLds); break;
    case 7: if (large) return launch_reduce_kt<GROUP, 7, FP, 256, 2>(a, kTwoPerCuLds); break;
    case 12: if (large) return launch_reduce_kt<GROUP, 12, FP, 256, 2>(a, kTwoPerCuLds); break;
    case 16: if (large) return launch_reduce_kt<GROUP, 16, FP, 256, 2>(a, kTwoPerCuLds); break;
    default: break;
    }
    return launch(grad_reduce_anyk_kernel<GROUP, FP>, dim3(blocks_for(a.n_vec, kAnyKBlock)), dim3(kAnyKBlock),
                  0, a.st, a.in_codes, a.stride_codes, a.in_scales, a.stride_scales, a.K, a.n_vec,
                  a.out_codes, a.out_scales, 0u);
}

// Validation and launch shared by the int8 and E4M3 forms of the reduce.
template <bool FP, bool SR = false>
int launch_reduce(const void* in_codes, int64_t chunk_stride_codes, const float* in_scales,
                  int64_t chunk_stride_scales, int K, int64_t numel, int group, void* out_codes,
                  float* out_scales, void* stream, u32 seed = 0)
{
    if (!in_codes || !in_scales || !out_codes || !out_scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (K < 1 || K > 64) return AGOQ_ERR_K;
    if (chunk_stride_codes < numel || chunk_stride_scales < numel / group) return AGOQ_ERR_SHAPE;
    if (misaligned(in_codes) || misaligned(in_scales) || misaligned(out_codes) ||
        misaligned(out_scales) || (chunk_stride_codes & 15) != 0)
        return AGOQ_ERR_ALIGN;
    const ReduceArgs a{(const int8_t*)in_codes, chunk_stride_codes, in_scales, chunk_stride_scales, K,
                       numel / 16, (u32x4*)out_codes, out_scales, (hipStream_t)stream, seed};
    return group == 128 ? launch_reduce_group<128, FP, SR>(a) : launch_reduce_group<64, FP, SR>(a);
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
template <int GROUP, int UNROLL, bool FP = false, bool SR = false>
__global__ __launch_bounds__(kGqBlock) void grad_accumulate_f32_kernel(
    const u32* main_codes, const float* main_scales, const f32x4* __restrict__ g_new,
    int64_t n_groups, u32* out_codes, float* out_scales, u32 seed)
{
    constexpr int VPL = GROUP / 64;
    constexpr int VPG = GROUP / 4;
    constexpr int kBlock = kGqBlock;
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
                const int64_t vec = grp * VPG + p * 16 + lane16;      // = the block of its four elements
                u32 w = encode4_bytes<FP, SR>(acc[p][0], acc[p][1], acc[p][2], acc[p][3], inv, seed, vec);
                if (!keep) w = 0;   // dead group: no signed zeros; non-finite group: no codes
                st<true>(out_codes + vec, w);
            }
            if (lane16 == 0) st<true>(out_scales + grp, scale);
        }
    }
}

template <int GROUP, int UNROLL, bool FP = false, bool SR = false>
__global__ __launch_bounds__(kGbBlock) void grad_accumulate_bf16_kernel(
    const u32x2* main_codes, const float* main_scales, const u32x4* __restrict__ g_new,
    int64_t n_vec, u32x2* out_codes, float* out_scales, u32 seed)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = kGbBlock;
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
            u32 p0 = encode4_bytes<FP, SR>(acc[0], acc[1], acc[2], acc[3], inv, seed, 2 * vi);
            u32 p1 = encode4_bytes<FP, SR>(acc[4], acc[5], acc[6], acc[7], inv, seed, 2 * vi + 1);
            if (!keep) p0 = p1 = 0;   // dead group: no signed zeros; non-finite group: no codes
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
__global__ __launch_bounds__(kGdBlock) void grad_dequant_kernel(const u32* __restrict__ codes,
                                                                     const float* __restrict__ scales,
                                                                     int64_t n_vec,
                                                                     f32x4* __restrict__ out)
{
    constexpr int LANES = GROUP / 4;      // lanes per group
    constexpr int kBlock = kGdBlock;
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
        if (vi < n_vec) st<true>(out + vi, o);
        if (UNROLL > 1) __builtin_amdgcn_sched_barrier(0);
    }
}

// Validation and launch shared by the int8 and E4M3 forms of the gradient store.
template <bool FP, bool SR = false>
int launch_grad_quant(const float* grad, int64_t numel, int group, void* codes, float* scales, void* stream,
                      u32 seed = 0)
{
    if (!grad || !codes || !scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(grad) || misaligned(codes) || misaligned(scales)) return AGOQ_ERR_ALIGN;
    const int64_t n_groups = numel / group;
    const dim3 grid(blocks_for(n_groups * 16, kGqBlock * kGqUnroll)), block(kGqBlock);
    hipStream_t st = (hipStream_t)stream;
    if (group == 128)
        return launch(grad_quant_kernel<128, kGqUnroll, FP, SR>, grid, block, 0, st, (const f32x4*)grad, n_groups,
                      (u32*)codes, scales, seed);
    return launch(grad_quant_kernel<64, kGqUnroll, FP, SR>, grid, block, 0, st, (const f32x4*)grad, n_groups,
                  (u32*)codes, scales, seed);
}

// ... of the gradient dequantize.
template <bool FP>
int launch_grad_dequant(const void* codes, const float* scales, int64_t numel, int group, float* out,
                        void* stream)
{
    if (!codes || !scales || !out) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(codes) || misaligned(scales) || misaligned(out)) return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 4;
    const dim3 grid(blocks_for(n_vec, kGdBlock * kGdUnroll)), block(kGdBlock);
    hipStream_t st = (hipStream_t)stream;
    if (group == 128)
        return launch(grad_dequant_kernel<128, kGdUnroll, FP>, grid, block, 0, st, (const u32*)codes, scales,
                      n_vec, (f32x4*)out);
    return launch(grad_dequant_kernel<64, kGdUnroll, FP>, grid, block, 0, st, (const u32*)codes, scales, n_vec,
                  (f32x4*)out);
}

// ... of the local accumulation.
template <bool FP, bool SR = false>
int launch_accumulate(const void* main_codes, const float* main_scales, const void* g_new,
                      int g_new_is_bf16, int64_t numel, int group, void* out_codes,
                      float* out_scales, void* stream, u32 seed = 0)
{
    if (!main_codes || !main_scales || !g_new || !out_codes || !out_scales) return AGOQ_ERR_NULL;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(main_codes) || misaligned(main_scales) || misaligned(g_new) ||
        misaligned(out_codes) || misaligned(out_scales))
        return AGOQ_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (g_new_is_bf16) {
        const int64_t n_vec = numel / 8;
        const dim3 grid(blocks_for(n_vec, kGbBlock * kGbUnroll)), block(kGbBlock);
        if (group == 128)
            return launch(grad_accumulate_bf16_kernel<128, kGbUnroll, FP, SR>, grid, block, 0, st,
                          (const u32x2*)main_codes, main_scales, (const u32x4*)g_new, n_vec,
                          (u32x2*)out_codes, out_scales, seed);
        return launch(grad_accumulate_bf16_kernel<64, kGbUnroll, FP, SR>, grid, block, 0, st,
                      (const u32x2*)main_codes, main_scales, (const u32x4*)g_new, n_vec, (u32x2*)out_codes,
                      out_scales, seed);
    }
    const int64_t n_groups = numel / group;
    const dim3 grid(blocks_for(n_groups * 16, kGqBlock * kGqUnroll)), block(kGqBlock);
    if (group == 128)
        return launch(grad_accumulate_f32_kernel<128, kGqUnroll, FP, SR>, grid, block, kCapGa, st,
                      (const u32*)main_codes, main_scales, (const f32x4*)g_new, n_groups, (u32*)out_codes,
                      out_scales, seed);
    return launch(grad_accumulate_f32_kernel<64, kGqUnroll, FP, SR>, grid, block, kCapGa, st,
                  (const u32*)main_codes, main_scales, (const f32x4*)g_new, n_groups, (u32*)out_codes,
                  out_scales, seed);
}

}  // namespace

extern "C" {

int agoq_grad_quant(const float* grad, int64_t numel, int group, int8_t* codes, float* scales,
                    void* stream)
{
    return launch_grad_quant<false>(grad, numel, group, codes, scales, stream);
}

int agoq_grad_reduce_requant(const int8_t* in_codes, int64_t chunk_stride_codes,
                             const float* in_scales, int64_t chunk_stride_scales, int K,
                             int64_t numel, int group, int8_t* out_codes, float* out_scales,
                             void* stream)
{
    return launch_reduce<false>(in_codes, chunk_stride_codes, in_scales, chunk_stride_scales, K, numel,
                                group, out_codes, out_scales, stream);
}

int agoq_grad_accumulate(const int8_t* main_codes, const float* main_scales, const void* g_new,
                         int g_new_is_bf16, int64_t numel, int group, int8_t* out_codes,
                         float* out_scales, void* stream)
{
    return launch_accumulate<false>(main_codes, main_scales, g_new, g_new_is_bf16, numel, group,
                                    out_codes, out_scales, stream);
}

int agoq_grad_dequant(const int8_t* codes, const float* scales, int64_t numel, int group,
                      float* out, void* stream)
{
    return launch_grad_dequant<false>(codes, scales, numel, group, out, stream);
}

int agoq_grad_quant_sr(const float* grad, int64_t numel, int group, uint32_t seed, int8_t* codes,
                       float* scales, void* stream)
{
    return launch_grad_quant<false, true>(grad, numel, group, codes, scales, stream, seed);
}

int agoq_grad_reduce_requant_sr(const int8_t* in_codes, int64_t chunk_stride_codes, const float* in_scales,
                                int64_t chunk_stride_scales, int K, int64_t numel, int group,
                                uint32_t seed, int8_t* out_codes, float* out_scales, void* stream)
{
    return launch_reduce<false, true>(in_codes, chunk_stride_codes, in_scales, chunk_stride_scales, K, numel,
                                      group, out_codes, out_scales, stream, seed);
}

int agoq_grad_accumulate_sr(const int8_t* main_codes, const float* main_scales, const void* g_new,
                            int g_new_is_bf16, int64_t numel, int group, uint32_t seed,
                            int8_t* out_codes, float* out_scales, void* stream)
{
    return launch_accumulate<false, true>(main_codes, main_scales, g_new, g_new_is_bf16, numel, group,
                                          out_codes, out_scales, stream, seed);
}

int agoq_fp8_grad_quant(const float* grad, int64_t numel, int group, uint8_t* codes, float* scales,
                        void* stream)
{
    return launch_grad_quant<true>(grad, numel, group, codes, scales, stream);
}

int agoq_fp8_grad_reduce_requant(const uint8_t* in_codes, int64_t chunk_stride_codes,
                                 const float* in_scales, int64_t chunk_stride_scales, int K,
                                 int64_t numel, int group, uint8_t* out_codes, float* out_scales,
                                 void* stream)
{
    return launch_reduce<true>(in_codes, chunk_stride_codes, in_scales, chunk_stride_scales, K, numel,
                               group, out_codes, out_scales, stream);
}

int agoq_fp8_grad_accumulate(const uint8_t* main_codes, const float* main_scales, const void* g_new,
                             int g_new_is_bf16, int64_t numel, int group, uint8_t* out_codes,
                             float* out_scales, void* stream)
{
    return launch_accumulate<true>(main_codes, main_scales, g_new, g_new_is_bf16, numel, group,
                                   out_codes, out_scales, stream);
}

int agoq_fp8_grad_dequant(const uint8_t* codes, const float* scales, int64_t numel, int group,
                          float* out, void* stream)
{
    return launch_grad_dequant<true>(codes, scales, numel, group, out, stream);
}

}  // extern "C"
