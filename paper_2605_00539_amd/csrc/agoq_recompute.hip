// Kernels fused with the two layers whose INPUT is what gets stored (RMSNorm, SiLU &
// Multiply).  Backward side: dequantize and recompute the layer's forward from the
// dequantized value, which never goes to memory.  Forward side: compute the layer and store
// its quantized input in one pass over the input.
#include "agoq_device.hpp"

namespace {

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
// Forward side: compute the layer and store its quantized INPUT in one pass, so the
// input is read from memory once instead of once by the layer and once by the quantizer.
// ---------------------------------------------------------------------------

// RMSNorm forward + quantize(x): one workgroup per row (cols <= 2048 * VPT).
//   y = bf16(x * (1/r) * gamma), r = sqrt(mean(x^2) + eps);  codes, scales = quantize(x)
template <int BITS, int GROUP, int VPT>
__global__ __launch_bounds__(kNormBlock) void rmsnorm_fwd_quant_kernel(
    const u32x4* __restrict__ x, int64_t n_vec_total, int vecs_per_row,
    const f32x4* __restrict__ gamma, float eps, float inv_cols, u32x4* __restrict__ y,
    float* __restrict__ r_out, void* __restrict__ codes, float* __restrict__ scales)
{
    constexpr int LANES = GROUP / 8;
    __shared__ float wave_part[kNormBlock / 64];
    const int64_t row_vec0 = (int64_t)blockIdx.x * vecs_per_row;
    u32x4 v[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int c = threadIdx.x + u * kNormBlock;
        v[u] = u32x4{0, 0, 0, 0};
        if (c < vecs_per_row) v[u] = ld<true>(x + row_vec0 + c);
    }
    float f[VPT][8];
    float ss = 0.0f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int c = threadIdx.x + u * kNormBlock;
        const u32 m = group_max_bits<LANES>(unpack8_bf16(v[u], f[u]));
        quantize_store8<BITS, GROUP, false, true>(f[u], m, row_vec0 + c, n_vec_total,
                                                  c < vecs_per_row, codes, scales);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss = __fmaf_rn(f[u][j], f[u][j], ss);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float total = 0.0f;
#pragma unroll
    for (int w = 0; w < kNormBlock / 64; ++w) total += wave_part[w];
    const float r = __fsqrt_rn(__fmaf_rn(total, inv_cols, eps));
    const float rinv = __fdiv_rn(1.0f, r);
    if (threadIdx.x == 0 && r_out) r_out[blockIdx.x] = r;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int c = threadIdx.x + u * kNormBlock;
        if (c < vecs_per_row) {
            const f32x4 g0 = gamma[2 * c], g1 = gamma[2 * c + 1];
            float o[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[j] = __fmul_rn(__fmul_rn(f[u][j], rinv), g0[j]);
                o[4 + j] = __fmul_rn(__fmul_rn(f[u][4 + j], rinv), g1[j]);
            }
            st<true>(y + row_vec0 + c, u32x4{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]),
                                             pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])});
        }
    }
}

// SiLU & Multiply forward + quantize(gate), quantize(up), elementwise.
//   z = bf16(up * gate * sigmoid(gate))
template <int BITS_G, int BITS_U, int GROUP, int UNROLL>
__global__ __launch_bounds__(AGOQ_AQ_BLOCK) void silu_mul_fwd_quant_kernel(
    const u32x4* __restrict__ gate, const u32x4* __restrict__ up, int64_t n_vec,
    u32x4* __restrict__ z, void* __restrict__ gate_codes, float* __restrict__ gate_scales,
    void* __restrict__ up_codes, float* __restrict__ up_scales)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = AGOQ_AQ_BLOCK;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;
    u32x4 gv[UNROLL], uv[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        gv[u] = uv[u] = u32x4{0, 0, 0, 0};
        if (vi < n_vec) {
            gv[u] = ld<true>(gate + vi);
            uv[u] = ld<true>(up + vi);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t vi = base + (int64_t)u * kBlock;
        const bool valid = vi < n_vec;
        float g[8], w[8], o[8];
        const u32 mg = group_max_bits<LANES>(unpack8_bf16(gv[u], g));
        const u32 mu = group_max_bits<LANES>(unpack8_bf16(uv[u], w));
        quantize_store8<BITS_G, GROUP, false, true>(g, mg, vi, n_vec, valid, gate_codes, gate_scales);
        quantize_store8<BITS_U, GROUP, false, true>(w, mu, vi, n_vec, valid, up_codes, up_scales);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float e = __expf(-g[j]);                          // may be +inf: 1/(1+inf) = 0
            o[j] = __fmul_rn(__fmul_rn(w[j], g[j]), __builtin_amdgcn_rcpf(1.0f + e));
        }
        if (valid)
            st<true>(z + vi, u32x4{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]),
                                   pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])});
    }
}

}  // namespace

extern "C" {

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

int agoq_rmsnorm_fwd_quant(const void* x_bf16, int64_t rows, int64_t cols, const float* gamma,
                           float eps, int group, int bits, void* y_bf16, float* r_out, void* codes,
                           float* scales, void* stream)
{
    if (!x_bf16 || !gamma || !y_bf16 || !codes || !scales) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (group != 64 && group != 128) return AGOQ_ERR_GROUP;
    if (rows <= 0 || rows > 0x7FFFFFFF || cols <= 0 || cols % group != 0 ||
        cols > (int64_t)kNormBlock * 8 * 8)
        return AGOQ_ERR_SHAPE;
    if (misaligned(x_bf16) || misaligned(gamma) || misaligned(y_bf16) || misaligned(codes) ||
        misaligned(scales))
        return AGOQ_ERR_ALIGN;
    const int vecs_per_row = (int)(cols / 8);
    const int64_t n_vec_total = rows * vecs_per_row;
    const float inv_cols = 1.0f / (float)cols;
    int vpt = 1;
    while (kNormBlock * vpt < vecs_per_row) vpt *= 2;
    const dim3 grid((unsigned)rows), block(kNormBlock);
    hipStream_t st = (hipStream_t)stream;
    const u32x4* x = (const u32x4*)x_bf16;
    const f32x4* gm = (const f32x4*)gamma;
    u32x4* y = (u32x4*)y_bf16;
#define AGOQ_LAUNCH_NORM_FWD(B, G)                                                                \
    switch (vpt) {                                                                                \
    case 1: rmsnorm_fwd_quant_kernel<B, G, 1><<<grid, block, 0, st>>>(x, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out, codes, scales); break; \
    case 2: rmsnorm_fwd_quant_kernel<B, G, 2><<<grid, block, 0, st>>>(x, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out, codes, scales); break; \
    case 4: rmsnorm_fwd_quant_kernel<B, G, 4><<<grid, block, 0, st>>>(x, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out, codes, scales); break; \
    default: rmsnorm_fwd_quant_kernel<B, G, 8><<<grid, block, 0, st>>>(x, n_vec_total, vecs_per_row, gm, eps, inv_cols, y, r_out, codes, scales); break; \
    }
    if (group == 128) {
        switch (bits) {
        case 4: AGOQ_LAUNCH_NORM_FWD(4, 128) break;
        case 5: AGOQ_LAUNCH_NORM_FWD(5, 128) break;
        case 6: AGOQ_LAUNCH_NORM_FWD(6, 128) break;
        default: AGOQ_LAUNCH_NORM_FWD(8, 128) break;
        }
    } else {
        switch (bits) {
        case 4: AGOQ_LAUNCH_NORM_FWD(4, 64) break;
        case 5: AGOQ_LAUNCH_NORM_FWD(5, 64) break;
        case 6: AGOQ_LAUNCH_NORM_FWD(6, 64) break;
        default: AGOQ_LAUNCH_NORM_FWD(8, 64) break;
        }
    }
#undef AGOQ_LAUNCH_NORM_FWD
    return launch_status();
}

int agoq_silu_mul_fwd_quant(const void* gate_bf16, const void* up_bf16, int64_t numel, int group,
                            int gate_bits, int up_bits, void* z_bf16, void* gate_codes,
                            float* gate_scales, void* up_codes, float* up_scales, void* stream)
{
    if (!gate_bf16 || !up_bf16 || !z_bf16 || !gate_codes || !gate_scales || !up_codes || !up_scales)
        return AGOQ_ERR_NULL;
    if ((gate_bits != 4 && gate_bits != 5 && gate_bits != 6 && gate_bits != 8) ||
        (up_bits != 4 && up_bits != 5 && up_bits != 6 && up_bits != 8))
        return AGOQ_ERR_BITS;
    if (int rc = check_common(numel, group)) return rc;
    if (misaligned(gate_bf16) || misaligned(up_bf16) || misaligned(z_bf16) ||
        misaligned(gate_codes) || misaligned(gate_scales) || misaligned(up_codes) ||
        misaligned(up_scales))
        return AGOQ_ERR_ALIGN;
    const int64_t n_vec = numel / 8;
    constexpr int U = 2;
    const dim3 grid(blocks_for(n_vec, AGOQ_AQ_BLOCK * U)), block(AGOQ_AQ_BLOCK);
    hipStream_t st = (hipStream_t)stream;
    const u32x4* g = (const u32x4*)gate_bf16;
    const u32x4* up = (const u32x4*)up_bf16;
    u32x4* z = (u32x4*)z_bf16;
#define AGOQ_LAUNCH_SILU_FWD(BG, BU)                                                              \
    if (group == 128)                                                                             \
        silu_mul_fwd_quant_kernel<BG, BU, 128, U><<<grid, block, 0, st>>>(g, up, n_vec, z, gate_codes, gate_scales, up_codes, up_scales); \
    else                                                                                          \
        silu_mul_fwd_quant_kernel<BG, BU, 64, U><<<grid, block, 0, st>>>(g, up, n_vec, z, gate_codes, gate_scales, up_codes, up_scales);
#define AGOQ_SILU_FWD_UP(BG)                                                                      \
    switch (up_bits) {                                                                            \
    case 4: AGOQ_LAUNCH_SILU_FWD(BG, 4) break;                                                    \
    case 5: AGOQ_LAUNCH_SILU_FWD(BG, 5) break;                                                    \
    case 6: AGOQ_LAUNCH_SILU_FWD(BG, 6) break;                                                    \
    default: AGOQ_LAUNCH_SILU_FWD(BG, 8) break;                                                   \
    }
    switch (gate_bits) {
    case 4: AGOQ_SILU_FWD_UP(4) break;
    case 5: AGOQ_SILU_FWD_UP(5) break;
    case 6: AGOQ_SILU_FWD_UP(6) break;
    default: AGOQ_SILU_FWD_UP(8) break;
    }
#undef AGOQ_SILU_FWD_UP
#undef AGOQ_LAUNCH_SILU_FWD
    return launch_status();
}

}  // extern "C"
