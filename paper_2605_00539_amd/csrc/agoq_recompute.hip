// Kernels fused with the two layers whose INPUT is what gets stored (RMSNorm, SiLU &
// Multiply).  Backward side: dequantize and recompute the layer's forward from the
// dequantized value, which never goes to memory.  Forward side: compute the layer and store
// its quantized input in one pass over the input.
#include <type_traits>

#include "agoq_device.hpp"

namespace {

// RMSNorm recompute:  r = sqrt(mean(x'^2) + eps);  y = bf16(x' * (1/r) * gamma).
// A workgroup owns a set of rows (blockIdx.x, + gridDim.x, ...) and works through them one
// at a time; each lane owns the same VPT column vectors in every row, so its slice of
// gamma is loaded once and stays in registers.  While a row is being reduced and stored,
// the codes of the workgroup's next row are already in flight: a row's load -> reduce ->
// store chain would otherwise leave the memory pipes idle for most of a workgroup's life.
// The row waits in registers as the bf16 pairs it consists of.
constexpr int kNormMaxBlock = 1024;
constexpr int kNormPipeRows = 8;                 // rows per workgroup from which the steady loop pays
constexpr int64_t kNormMaxCols = 16384;          // widest row the row kernels take
// Most lanes a row kernel with VPT vectors per lane is ever launched with (the register
// budget per lane follows from it).
constexpr int norm_max_block(int vpt)
{
    return (int)(kNormMaxCols / 8 / vpt) < kNormMaxBlock ? (int)(kNormMaxCols / 8 / vpt) : kNormMaxBlock;
}
// Launch shape of the row kernels (measured on [8192,4096] and [8192,14336] tensors).
constexpr int kNormDepth = 2;       // rows of a workgroup in flight beyond the one being reduced
constexpr int kNormVpt = 4;         // column vectors per lane, 4-bit codes (doubled while a row needs > 1024 lanes)
constexpr int kNormVpt8 = 2;        // ... 8-bit codes, whose buffers are twice the size
constexpr int kNormFwdVpt = 2;      // ... the forward kernel
// 5- and 6-bit codes (three loads per vector): two per lane on rows of up to 1024 vectors, else four
constexpr int norm_vpt56(int vecs_per_row) { return vecs_per_row <= 1024 ? 2 : 4; }
constexpr int kNormResident = 1024; // lanes per compute unit the grid is sized for
// Rows of exactly 64 * VPT vectors for VPT = 8 or 10 (4096 and 5120 columns, the hidden sizes
// of the 8B and 32B models) take the wavefront-per-row kernels: measured 5-17 % faster on
// [8192,4096] and [4096,4096] tensors than two wavefronts per row with a barrier per row
// (4 wavefronts x 2 workgroups per compute unit; 2 x 4 and 8 x 1 are 2-8 % slower, more
// workgroups per unit slower still).
constexpr int kWaveRowVptA = 8, kWaveRowVptB = 10;
constexpr int kWaveRowWaves = 4;    // wavefronts (rows in progress) per workgroup
constexpr int kWaveRowPerCu = 2;    // workgroups per compute unit the grid is sized for
// With few rows per resident wavefront the kernels above win (half the work, or less, per
// wavefront on the one row it ever sees).  The recompute kernel changes over at one row per
// resident wavefront for 8-bit codes (whose other form puts four wavefronts on a row), two
// for 5 and 6 bits, four for 4 bits (measured on 4096- and 5120-wide rows, 1024 to 16384
// rows: 8-bit +2 to +14 % from 2048 rows on; 6-bit -6 % at 3072, +2 to +8 % from 4096;
// 4-bit -11 % at 3072, -5 % at 4096, +5 to +12 % at 8192); the forward kernel at half a row
// (+5 to +15 % from 1024 to 8192 rows, -15 % at 512).
constexpr int wave_row_min_rounds_recompute2(int bits) { return bits == 8 ? 2 : bits == 4 ? 8 : 4; }
constexpr int kWaveRowMinRoundsForward2 = 1;

// Sum of the per-wavefront partial sums of a workgroup, in wavefront order.
__device__ __forceinline__ float block_sum(float wave_total, float* wave_part)
{
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = wave_total;
    __syncthreads();
    float total = 0.0f;
    const int nw = blockDim.x >> 6;
    for (int w = 0; w < nw; ++w) total += wave_part[w];
    return total;
}

// y for the lane's 8 elements from x' (bf16 pairs), 1/r and gamma.
__device__ __forceinline__ u32x4 norm_out8(const u32 (&xp)[4], float rinv, const f32x4& g0,
                                           const f32x4& g1)
{
    float o[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float x0 = as_f32(xp[k] << 16), x1 = as_f32(xp[k] & 0xFFFF0000u);
        const f32x4& g = k < 2 ? g0 : g1;
        o[2 * k] = __fmul_rn(__fmul_rn(x0, rinv), g[(2 * k) & 3]);
        o[2 * k + 1] = __fmul_rn(__fmul_rn(x1, rinv), g[(2 * k + 1) & 3]);
    }
    return u32x4{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]),
                 pack_bf16x2(o[6], o[7])};
}

// Adds the squares of the lane's 8 elements (bf16 pairs) to ss, in element order.
__device__ __forceinline__ float sumsq8(const u32 (&xp)[4], float ss)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float x0 = as_f32(xp[k] << 16), x1 = as_f32(xp[k] & 0xFFFF0000u);
        ss = __fmaf_rn(x0, x0, ss);
        ss = __fmaf_rn(x1, x1, ss);
    }
    return ss;
}

// Addressing of the row kernels: a row's base pointers are uniform over the workgroup (scalar
// registers, scalar arithmetic) and a lane's byte offsets within a row never change, so the
// row loop spends one vector instruction per access on its address instead of the three or
// four that 64-bit index arithmetic per lane took (a seventh of the loop's instructions).
template <typename T>
__device__ __forceinline__ const T* at_bytes(const T* base, unsigned byte_offset)
{
    return (const T*)((const char*)base + byte_offset);
}
template <typename T>
__device__ __forceinline__ T* at_bytes(T* base, unsigned byte_offset)
{
    return (T*)((char*)base + byte_offset);
}

// The stored codes of vector v (index within the row) of a row whose nibble plane starts at
// row_lo and whose high-bit plane starts at row_hi.
template <int BITS>
__device__ __forceinline__ Codes8<BITS> load_row_codes8(const void* row_lo, const void* row_hi, unsigned v)
{
    Codes8<BITS> c;
    if constexpr (BITS == 8) {
        c.w = ld<true>(at_bytes((const uint64_t*)row_lo, v * 8u));
    } else {
        c.lo = ld<true>(at_bytes((const u32*)row_lo, v * 4u));
        if constexpr (BITS == 5) c.hi = ld<true>(at_bytes((const uint8_t*)row_hi, v));
        if constexpr (BITS == 6) c.hi = ld<true>(at_bytes((const uint16_t*)row_hi, v * 2u));
    }
    return c;
}

// PIPE: chosen by the host when every workgroup has many rows and the row has exactly
// VPT * blockDim.x vectors.  No lane is then ever past the end of a row, nothing in the row
// loop sits under a lane test, and the walk has a steady part (below).
template <int BITS, int GROUP, int VPT, bool FP = false, bool PIPE = false>
__global__ __launch_bounds__(norm_max_block(VPT)) void act_dequant_rmsnorm_kernel(
    const void* __restrict__ codes, const float* __restrict__ scales, int64_t n_vec_total,
    int64_t rows, int vecs_per_row, const f32x4* __restrict__ gamma, float eps, float inv_cols,
    u32x4* __restrict__ y, float* __restrict__ r_out)
{
    constexpr int LANES = GROUP / 8;
    __shared__ float wave_part[2][kNormMaxBlock / 64];
    f32x4 g0[VPT], g1[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int v = threadIdx.x + u * blockDim.x;
        g0[u] = g1[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (PIPE || v < vecs_per_row) {
            g0[u] = gamma[2 * v];
            g1[u] = gamma[2 * v + 1];
        }
    }
    // Row buffers in rotation: while one row is reduced and stored, the loads of the
    // workgroup's next kDepth rows are in flight.  The rotation is written out (no buffer is
    // ever copied into another: a copy would have to wait for the load that fills it).
    // Loads take no lane test (a lane past the end of the row re-reads the row's last vector
    // and uses scale 0, so it adds nothing to the row sum): a load under a branch would have
    // to be merged with the register's old value, which again waits for the data.
    constexpr int kDepth = kNormDepth;
    struct RowBuf {
        Codes8<BITS> c[VPT];
        float sc[VPT];
    };
    const int64_t step = gridDim.x;
    // the lane's vectors within a row (a lane past the end of the row: the row's last vector)
    unsigned vc[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int v = threadIdx.x + u * blockDim.x;
        vc[u] = (unsigned)(PIPE || v < vecs_per_row ? v : vecs_per_row - 1);
    }
    constexpr int kHighBytes = BITS == 6 ? 2 : 1;     // bytes per vector in the high-bit plane
    const uint8_t* const high = (const uint8_t*)codes + n_vec_total * 4;
    auto fetch = [&](RowBuf& b, int64_t row) {
        const int64_t first = row * vecs_per_row;                   // uniform over the workgroup
        const void* row_lo = (const uint8_t*)codes + first * (BITS == 8 ? 8 : 4);
        const void* row_hi = high + first * kHighBytes;
        const float* row_sc = scales + first / LANES;               // rows are whole groups
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            b.c[u] = load_row_codes8<BITS>(row_lo, row_hi, vc[u]);
            b.sc[u] = ld<false>(at_bytes(row_sc, vc[u] / LANES * 4u));
        }
    };
    // One row from its buffer to memory; `refill` (the same buffer, free once the row has
    // been decoded) then receives the row that is kDepth + 1 steps on.  SURE: the caller
    // knows that row to exist, and the refill is issued without a test.
    auto finish = [&](auto sure, const RowBuf& b, int64_t row, RowBuf& refill, int phase) {
        u32 xp[VPT][4];
        float ss = 0.0f;
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const bool valid = PIPE || (int)(threadIdx.x + u * blockDim.x) < vecs_per_row;
            dequant8_packed<BITS, FP>(b.c[u], valid ? b.sc[u] : 0.0f, xp[u]);
            ss = sumsq8(xp[u], ss);
        }
        const int64_t next = row + (kDepth + 1) * step;
        if (decltype(sure)::value || next < rows) fetch(refill, next);   // the same for every lane
        const float total = block_sum(wave_sum(ss), wave_part[phase]);
        const float r = __fsqrt_rn(__fmaf_rn(total, inv_cols, eps));
        const float rinv = __fdiv_rn(1.0f, r);
        if (threadIdx.x == 0) r_out[row] = r;
        u32x4* const y_row = y + row * vecs_per_row;                // uniform over the workgroup
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const int v = threadIdx.x + u * blockDim.x;
            if (PIPE || v < vecs_per_row)
                st<true>(at_bytes(y_row, vc[u] * 16u), norm_out8(xp[u], rinv, g0[u], g1[u]));
        }
    };
    constexpr std::true_type kSure{};
    constexpr std::false_type kTested{};
    // wave_part has two buffers used alternately: a wavefront is never more than one
    // barrier ahead of another, so a buffer is rewritten only after everyone has read it.
    //
    // PIPE: the walk has a steady part, in which every refill is known to lie inside the
    // tensor and no load of the loop sits under a branch, and a tail of at most
    // 2 * (kDepth + 1) - 1 rows with tested refills.  With a test around the loads the compiler
    // cannot count the loads issued since the one it waits for and waits for ALL outstanding
    // memory operations instead -- the younger rows' loads and the last row's stores included
    // -- once per rotation of the buffers.  Without PIPE (few rows per workgroup, where the
    // longer code costs more than the waits) the tail loop is the whole walk.
    int64_t row = blockIdx.x;                       // the grid never exceeds the row count
    int phase = 0;
    static_assert(kDepth == 2, "the walk below rotates three row buffers");
    RowBuf b0, b1, b2;
    if (PIPE && row + 5 * step < rows) {
        fetch(b0, row);
        fetch(b1, row + step);
        fetch(b2, row + 2 * step);
        do {
            finish(kSure, b0, row, b0, phase);
            finish(kSure, b1, row + step, b1, phase ^ 1);
            finish(kSure, b2, row + 2 * step, b2, phase);
            row += 3 * step;
            phase ^= 1;
        } while (row + 5 * step < rows);
    } else {
        fetch(b0, row);
        if (row + step < rows) fetch(b1, row + step);
        if (row + 2 * step < rows) fetch(b2, row + 2 * step);
    }
    while (true) {
        finish(kTested, b0, row, b0, phase);
        if ((row += step) >= rows) break;
        finish(kTested, b1, row, b1, phase ^ 1);
        if ((row += step) >= rows) break;
        finish(kTested, b2, row, b2, phase);
        if ((row += step) >= rows) break;
        finish(kTested, b0, row, b0, phase ^ 1);
        if ((row += step) >= rows) break;
        finish(kTested, b1, row, b1, phase);
        if ((row += step) >= rows) break;
        finish(kTested, b2, row, b2, phase ^ 1);
        if ((row += step) >= rows) break;
    }
}

// The same for rows of exactly 64 * VPT vectors, one wavefront per row: the row sum is a
// reduction within the wavefront, so the row loop has no barrier and the wavefronts of a
// workgroup drift apart freely (one's stores overlap another's loads).  A lane owns VPT
// vectors of every row; gamma would take 8 * VPT registers per lane and waits in LDS instead,
// staged once per workgroup.  Three rows per wavefront are in flight, as in the kernel above.
template <int BITS, int GROUP, int VPT, bool FP = false>
__global__ __launch_bounds__(kWaveRowWaves * 64) void act_dequant_rmsnorm_wave_kernel(
    const void* __restrict__ codes, const float* __restrict__ scales, int64_t n_vec_total, int64_t rows,
    const f32x4* __restrict__ gamma, float eps, float inv_cols, u32x4* __restrict__ y, float* __restrict__ r_out)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kWaveRowVecs = 64 * VPT;
    __shared__ f32x4 g_lo[kWaveRowVecs], g_hi[kWaveRowVecs];
    for (int v = threadIdx.x; v < kWaveRowVecs; v += kWaveRowWaves * 64) {
        g_lo[v] = gamma[2 * v];
        g_hi[v] = gamma[2 * v + 1];
    }
    __syncthreads();                                    // the only barrier: before any wavefront leaves
    const unsigned lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t step = (int64_t)gridDim.x * kWaveRowWaves;
    int64_t row = (int64_t)blockIdx.x * kWaveRowWaves + wave;     // uniform over the wavefront
    if (row >= rows) return;
    struct RowBuf {
        Codes8<BITS> c[VPT];
        float sc[VPT];
    };
    constexpr int kHighBytes = BITS == 6 ? 2 : 1;     // bytes per vector in the high-bit plane
    const uint8_t* const high = (const uint8_t*)codes + n_vec_total * 4;
    auto fetch = [&](RowBuf& b, int64_t r) {
        const int64_t first = r * kWaveRowVecs;
        const void* row_lo = (const uint8_t*)codes + first * (BITS == 8 ? 8 : 4);
        const void* row_hi = high + first * kHighBytes;
        const float* row_sc = scales + first / LANES;               // rows are whole groups
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const unsigned v = lane + 64u * u;
            b.c[u] = load_row_codes8<BITS>(row_lo, row_hi, v);
            b.sc[u] = ld<false>(at_bytes(row_sc, v / LANES * 4u));
        }
    };
    auto finish = [&](const RowBuf& b, int64_t r, RowBuf& refill) {
        u32 xp[VPT][4];
        float ss = 0.0f;
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            dequant8_packed<BITS, FP>(b.c[u], b.sc[u], xp[u]);
            ss = sumsq8(xp[u], ss);
        }
        const int64_t next = r + 3 * step;
        if (next < rows) fetch(refill, next);                      // the same for every lane
        // The row waits for its sum as the packed pairs: without this the compiler keeps the
        // unpacked floats of the first pass instead, 8 * VPT registers more, and the kernel no
        // longer fits two workgroups per compute unit.
#pragma unroll
        for (int u = 0; u < VPT; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) asm volatile("" : "+v"(xp[u][k]));
        const float total = wave_sum(ss);
        const float rr = __fsqrt_rn(__fmaf_rn(total, inv_cols, eps));
        const float rinv = __fdiv_rn(1.0f, rr);
        if (lane == 0) r_out[r] = rr;
        u32x4* const y_row = y + r * kWaveRowVecs;
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const unsigned v = lane + 64u * u;
            st<true>(at_bytes(y_row, v * 16u), norm_out8(xp[u], rinv, g_lo[v], g_hi[v]));
        }
    };
    RowBuf b0, b1, b2;
    fetch(b0, row);
    if (row + step < rows) fetch(b1, row + step);
    if (row + 2 * step < rows) fetch(b2, row + 2 * step);
    while (true) {
        finish(b0, row, b0);
        if ((row += step) >= rows) break;
        finish(b1, row, b1);
        if ((row += step) >= rows) break;
        finish(b2, row, b2);
        if ((row += step) >= rows) break;
    }
}

// SiLU & Multiply recompute: z = bf16(u' * g' * sigmoid(g')), elementwise over the two
// stored tensors (which may have different code widths).  The kernel is bound by vector
// instructions as much as by memory (two decodes, exp and rcp at a quarter of the rate), so a
// tile's base pointers are scalar, lane offsets are 32 bits wide, and only the one workgroup
// that straddles the end of the tensor clamps its loads (FULL = false).
template <int BITS_G, int BITS_U, int GROUP, int BLOCK, int UNROLL, bool FP, bool FULL>
__device__ __forceinline__ void dequant_silu_mul_tile(const void* __restrict__ gate_codes,
                                                      const float* __restrict__ gate_scales,
                                                      const void* __restrict__ up_codes,
                                                      const float* __restrict__ up_scales, int64_t n_vec,
                                                      u32x4* __restrict__ z)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kTile = BLOCK * UNROLL;
    const int64_t first = (int64_t)blockIdx.x * kTile;                  // uniform over the workgroup
    const unsigned left = FULL ? (unsigned)kTile : (unsigned)(n_vec - first);   // vectors from `first` on
    const uint8_t* const gate_bytes = (const uint8_t*)gate_codes;
    const uint8_t* const up_bytes = (const uint8_t*)up_codes;
    const void* g_lo = gate_bytes + first * (BITS_G == 8 ? 8 : 4);
    const void* g_hi = gate_bytes + n_vec * 4 + first * (BITS_G == 6 ? 2 : 1);
    const void* u_lo = up_bytes + first * (BITS_U == 8 ? 8 : 4);
    const void* u_hi = up_bytes + n_vec * 4 + first * (BITS_U == 6 ? 2 : 1);
    const float* g_sc = gate_scales + first / LANES;                    // a tile is whole groups
    const float* u_sc = up_scales + first / LANES;
    u32x4* const z_tile = z + first;
    // loads (unconditional: a lane past the end re-reads the last vector and stores nothing),
    // one point where all of them are waited for, then arithmetic and stores vector by vector
    Codes8<BITS_G> gc[UNROLL];
    Codes8<BITS_U> uc[UNROLL];
    float gs[UNROLL], us[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const unsigned lane = threadIdx.x + u * BLOCK;
        const unsigned vc = FULL || lane < left ? lane : left - 1;
        gc[u] = load_row_codes8<BITS_G>(g_lo, g_hi, vc);
        uc[u] = load_row_codes8<BITS_U>(u_lo, u_hi, vc);
        gs[u] = ld<false>(at_bytes(g_sc, vc / LANES * 4u));
        us[u] = ld<false>(at_bytes(u_sc, vc / LANES * 4u));
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        need_now(gc[u]);
        need_now(uc[u]);
        need_now(gs[u]);
        need_now(us[u]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const unsigned lane = threadIdx.x + u * BLOCK;
        float g[8], up[8], o[8];
        dequant8_bf16<BITS_G, FP>(gc[u], gs[u], g);
        dequant8_bf16<BITS_U, FP>(uc[u], us[u], up);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float e = __expf(-g[j]);                          // may be +inf: 1/(1+inf) = 0
            const float sig = __builtin_amdgcn_rcpf(1.0f + e);
            o[j] = __fmul_rn(__fmul_rn(up[j], g[j]), sig);
        }
        if (FULL || lane < left)
            st<true>(at_bytes(z_tile, lane * 16u),
                     u32x4{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]),
                           pack_bf16x2(o[6], o[7])});
    }
}

template <int BITS_G, int BITS_U, int GROUP, int BLOCK, int UNROLL, bool FP = false>
__global__ __launch_bounds__(BLOCK) void act_dequant_silu_mul_kernel(
    const void* __restrict__ gate_codes, const float* __restrict__ gate_scales,
    const void* __restrict__ up_codes, const float* __restrict__ up_scales, int64_t n_vec,
    u32x4* __restrict__ z)
{
    if (((int64_t)blockIdx.x + 1) * (BLOCK * UNROLL) <= n_vec)
        dequant_silu_mul_tile<BITS_G, BITS_U, GROUP, BLOCK, UNROLL, FP, true>(gate_codes, gate_scales, up_codes,
                                                                       up_scales, n_vec, z);
    else
        dequant_silu_mul_tile<BITS_G, BITS_U, GROUP, BLOCK, UNROLL, FP, false>(gate_codes, gate_scales, up_codes,
                                                                        up_scales, n_vec, z);
}

// ---------------------------------------------------------------------------
// Forward side: compute the layer and store its quantized INPUT in one pass, so the
// input is read from memory once instead of once by the layer and once by the quantizer.
// ---------------------------------------------------------------------------

// RMSNorm forward + quantize(x): one workgroup per row, shaped like the recompute kernel.
//   y = bf16(x * (1/r) * gamma), r = sqrt(mean(x^2) + eps);  codes, scales = quantize(x)
template <int BITS, int GROUP, int VPT, bool FP = false, bool PIPE = false>
__global__ __launch_bounds__(norm_max_block(VPT)) void rmsnorm_fwd_quant_kernel(
    const u32x4* __restrict__ x, int64_t n_vec_total, int64_t rows, int vecs_per_row,
    const f32x4* __restrict__ gamma, float eps, float inv_cols, u32x4* __restrict__ y,
    float* __restrict__ r_out, void* __restrict__ codes, float* __restrict__ scales)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kDepth = kNormDepth;
    __shared__ float wave_part[2][kNormMaxBlock / 64];
    f32x4 g0[VPT], g1[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int c = threadIdx.x + u * blockDim.x;
        g0[u] = g1[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (PIPE || c < vecs_per_row) {
            g0[u] = gamma[2 * c];
            g1[u] = gamma[2 * c + 1];
        }
    }
    // Row buffers in rotation, as in the recompute kernel: the row waits in registers as the
    // bf16 pairs it arrived in, and the next rows of the workgroup are already in flight.
    struct RowBuf {
        u32x4 v[VPT];
    };
    const int64_t step = gridDim.x;
    // the lane's vectors within a row (a lane past the end of the row: the row's last vector)
    unsigned vc[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int c = threadIdx.x + u * blockDim.x;
        vc[u] = (unsigned)(PIPE || c < vecs_per_row ? c : vecs_per_row - 1);
    }
    auto fetch = [&](RowBuf& b, int64_t row) {
        const u32x4* const x_row = x + row * vecs_per_row;          // uniform over the workgroup
#pragma unroll
        for (int u = 0; u < VPT; ++u) b.v[u] = ld<true>(at_bytes(x_row, vc[u] * 16u));
    };
    auto finish = [&](auto sure, const RowBuf& b, int64_t row, RowBuf& refill, int phase) {
        u32x4 v[VPT];
        float ss = 0.0f;
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const int c = threadIdx.x + u * blockDim.x;
            const bool valid = PIPE || c < vecs_per_row;
            v[u] = valid ? b.v[u] : u32x4{0, 0, 0, 0};
            float f[8];
            const u32 m = group_max_bits<LANES>(unpack8_bf16(v[u], f));
            quantize_store8<BITS, GROUP, FP, true>(f, m, row * vecs_per_row + c, n_vec_total,
                                                      valid, codes, scales);
#pragma unroll
            for (int j = 0; j < 8; ++j) ss = __fmaf_rn(f[j], f[j], ss);
        }
        const int64_t next = row + (kDepth + 1) * step;
        if (decltype(sure)::value || next < rows) fetch(refill, next);   // the same for every lane
        const float total = block_sum(wave_sum(ss), wave_part[phase]);
        const float r = __fsqrt_rn(__fmaf_rn(total, inv_cols, eps));
        const float rinv = __fdiv_rn(1.0f, r);
        if (threadIdx.x == 0 && r_out) r_out[row] = r;
        u32x4* const y_row = y + row * vecs_per_row;                // uniform over the workgroup
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const int c = threadIdx.x + u * blockDim.x;
            const u32 xp[4] = {v[u][0], v[u][1], v[u][2], v[u][3]};
            if (PIPE || c < vecs_per_row)
                st<true>(at_bytes(y_row, vc[u] * 16u), norm_out8(xp, rinv, g0[u], g1[u]));
        }
    };
    constexpr std::true_type kSure{};
    constexpr std::false_type kTested{};
    // steady part with untested refills, then the tail: see the recompute kernel
    int64_t row = blockIdx.x;                       // the grid never exceeds the row count
    int phase = 0;
    static_assert(kDepth == 2, "the walk below rotates three row buffers");
    RowBuf b0, b1, b2;
    if (PIPE && row + 5 * step < rows) {
        fetch(b0, row);
        fetch(b1, row + step);
        fetch(b2, row + 2 * step);
        do {
            finish(kSure, b0, row, b0, phase);
            finish(kSure, b1, row + step, b1, phase ^ 1);
            finish(kSure, b2, row + 2 * step, b2, phase);
            row += 3 * step;
            phase ^= 1;
        } while (row + 5 * step < rows);
    } else {
        fetch(b0, row);
        if (row + step < rows) fetch(b1, row + step);
        if (row + 2 * step < rows) fetch(b2, row + 2 * step);
    }
    while (true) {
        finish(kTested, b0, row, b0, phase);
        if ((row += step) >= rows) break;
        finish(kTested, b1, row, b1, phase ^ 1);
        if ((row += step) >= rows) break;
        finish(kTested, b2, row, b2, phase);
        if ((row += step) >= rows) break;
        finish(kTested, b0, row, b0, phase ^ 1);
        if ((row += step) >= rows) break;
        finish(kTested, b1, row, b1, phase);
        if ((row += step) >= rows) break;
        finish(kTested, b2, row, b2, phase ^ 1);
        if ((row += step) >= rows) break;
    }
}

// The same for rows of exactly 64 * VPT vectors, one wavefront per row (see the recompute
// kernel of that shape).
template <int BITS, int GROUP, int VPT, bool FP = false>
__global__ __launch_bounds__(kWaveRowWaves * 64) void rmsnorm_fwd_quant_wave_kernel(
    const u32x4* __restrict__ x, int64_t n_vec_total, int64_t rows, const f32x4* __restrict__ gamma, float eps,
    float inv_cols, u32x4* __restrict__ y, float* __restrict__ r_out, void* __restrict__ codes,
    float* __restrict__ scales)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kWaveRowVecs = 64 * VPT;
    __shared__ f32x4 g_lo[kWaveRowVecs], g_hi[kWaveRowVecs];
    for (int v = threadIdx.x; v < kWaveRowVecs; v += kWaveRowWaves * 64) {
        g_lo[v] = gamma[2 * v];
        g_hi[v] = gamma[2 * v + 1];
    }
    __syncthreads();                                    // the only barrier: before any wavefront leaves
    const unsigned lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t step = (int64_t)gridDim.x * kWaveRowWaves;
    int64_t row = (int64_t)blockIdx.x * kWaveRowWaves + wave;     // uniform over the wavefront
    if (row >= rows) return;
    struct RowBuf {
        u32x4 v[VPT];
    };
    auto fetch = [&](RowBuf& b, int64_t r) {
        const u32x4* const x_row = x + r * kWaveRowVecs;
#pragma unroll
        for (int u = 0; u < VPT; ++u) b.v[u] = ld<true>(at_bytes(x_row, (lane + 64u * u) * 16u));
    };
    auto finish = [&](const RowBuf& b, int64_t r, RowBuf& refill) {
        u32x4 v[VPT];
        float ss = 0.0f;
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            v[u] = b.v[u];
            float f[8];
            const u32 m = group_max_bits<LANES>(unpack8_bf16(v[u], f));
            quantize_store8<BITS, GROUP, FP, true>(f, m, r * kWaveRowVecs + lane + 64 * u, n_vec_total, true,
                                                      codes, scales);
#pragma unroll
            for (int j = 0; j < 8; ++j) ss = __fmaf_rn(f[j], f[j], ss);
        }
        const int64_t next = r + 3 * step;
        if (next < rows) fetch(refill, next);                      // the same for every lane
        const float total = wave_sum(ss);
        const float rr = __fsqrt_rn(__fmaf_rn(total, inv_cols, eps));
        const float rinv = __fdiv_rn(1.0f, rr);
        if (lane == 0 && r_out) r_out[r] = rr;
        u32x4* const y_row = y + r * kWaveRowVecs;
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const unsigned c = lane + 64u * u;
            const u32 xp[4] = {v[u][0], v[u][1], v[u][2], v[u][3]};
            st<true>(at_bytes(y_row, c * 16u), norm_out8(xp, rinv, g_lo[c], g_hi[c]));
        }
    };
    RowBuf b0, b1, b2;
    fetch(b0, row);
    if (row + step < rows) fetch(b1, row + step);
    if (row + 2 * step < rows) fetch(b2, row + 2 * step);
    while (true) {
        finish(b0, row, b0);
        if ((row += step) >= rows) break;
        finish(b1, row, b1);
        if ((row += step) >= rows) break;
        finish(b2, row, b2);
        if ((row += step) >= rows) break;
    }
}

// SiLU & Multiply forward + quantize(gate), quantize(up), elementwise.
//   z = bf16(up * gate * sigmoid(gate))
template <int BITS_G, int BITS_U, int GROUP, int UNROLL, bool FP = false>
__global__ __launch_bounds__(kAqBlock) void silu_mul_fwd_quant_kernel(
    const u32x4* __restrict__ gate, const u32x4* __restrict__ up, int64_t n_vec,
    u32x4* __restrict__ z, void* __restrict__ gate_codes, float* __restrict__ gate_scales,
    void* __restrict__ up_codes, float* __restrict__ up_scales)
{
    constexpr int LANES = GROUP / 8;
    constexpr int kBlock = kAqBlock;
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
        quantize_store8<BITS_G, GROUP, FP, true>(g, mg, vi, n_vec, valid, gate_codes, gate_scales);
        quantize_store8<BITS_U, GROUP, FP, true>(w, mu, vi, n_vec, valid, up_codes, up_scales);
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

// Launch shape of the row kernels: VPT vectors per lane and the number of lanes, a whole
// number of wavefronts.  VPT is the preferred count, or half of it when that leaves fewer
// lanes idle in the last wavefront (640 vectors: 4 per lane would idle a sixth of the
// lanes, 2 per lane none), doubled while a row would need more than 1024 lanes.
inline int norm_lanes(int vecs_per_row, int vpt) { return ((vecs_per_row + vpt - 1) / vpt + 63) / 64 * 64; }
inline void norm_launch_shape(int vecs_per_row, int preferred_vpt, int& vpt, int& threads)
{
    vpt = preferred_vpt;
    if (vpt >= 2 && norm_lanes(vecs_per_row, vpt / 2) * (vpt / 2) < norm_lanes(vecs_per_row, vpt) * vpt &&
        norm_lanes(vecs_per_row, vpt / 2) <= kNormMaxBlock)
        vpt /= 2;
    while ((vecs_per_row + vpt - 1) / vpt > kNormMaxBlock) vpt *= 2;
    threads = norm_lanes(vecs_per_row, vpt);
}

// Workgroups of a row kernel that walks its rows: as many as are resident at once when
// every compute unit holds kNormResident lanes -- one workgroup per unit for wide
// rows (workgroups of six wavefronts or more; measured +2-4 % on 14336-wide rows).
inline unsigned norm_grid(int64_t rows, int threads)
{
    const int per_cu = threads >= 384 ? 1 : kNormResident / threads;
    const int64_t resident = (int64_t)compute_units() * (per_cu > 0 ? per_cu : 1);
    return (unsigned)(rows < resident ? rows : resident);
}

// Workgroups of a wavefront-per-row kernel: kWaveRowPerCu per compute unit, or fewer when that
// already gives every row a wavefront.
inline unsigned wave_row_grid(int64_t rows)
{
    const int64_t resident = (int64_t)compute_units() * kWaveRowPerCu;
    const int64_t needed = (rows + kWaveRowWaves - 1) / kWaveRowWaves;
    return (unsigned)(needed < resident ? needed : resident);
}

// Whether a tensor of `rows` rows of vecs_per_row vectors goes to a wavefront-per-row kernel
// that changes over at min_rounds2 / 2 rows per resident wavefront.
inline bool wave_row_shape(int64_t rows, int vecs_per_row, int min_rounds2)
{
    const int64_t resident_waves = (int64_t)compute_units() * kWaveRowPerCu * kWaveRowWaves;
    return (vecs_per_row == 64 * kWaveRowVptA || vecs_per_row == 64 * kWaveRowVptB) &&
           2 * rows >= min_rounds2 * resident_waves;
}

// Calls f(std::integral_constant<int, VPT>) for the wavefront-per-row kernel of that row width.
template <typename F>
int dispatch_wave_row_vpt(int vecs_per_row, F&& f)
{
    return vecs_per_row == 64 * kWaveRowVptA ? f(std::integral_constant<int, kWaveRowVptA>{})
                                             : f(std::integral_constant<int, kWaveRowVptB>{});
}

// Calls f(std::integral_constant<int, VPT>) for vpt in {1, 2, 4}.
template <typename F>
int dispatch_vpt(int vpt, F&& f)
{
    switch (vpt) {
    case 1: return f(std::integral_constant<int, 1>{});
    case 2: return f(std::integral_constant<int, 2>{});
    default: return f(std::integral_constant<int, 4>{});
    }
}

int dequant_rmsnorm_impl(const void* codes, const float* scales, int64_t rows, int64_t cols, int group,
                         int bits, bool fp, const float* gamma, float eps, void* y_bf16, float* r_out,
                         void* stream)
{
    if (!codes || !scales || !gamma || !y_bf16 || !r_out) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (group != 64 && group != 128) return AGOQ_ERR_GROUP;
    if (rows <= 0 || rows > 0x7FFFFFFF || cols <= 0 || cols % group != 0 ||
        cols > kNormMaxCols)
        return AGOQ_ERR_SHAPE;
    if (misaligned(codes) || misaligned(scales) || misaligned(gamma) || misaligned(y_bf16))
        return AGOQ_ERR_ALIGN;
    const int vecs_per_row = (int)(cols / 8);
    const int64_t n_vec_total = rows * vecs_per_row;
    const float inv_cols = 1.0f / (float)cols;
    hipStream_t st = (hipStream_t)stream;
    const f32x4* gm = (const f32x4*)gamma;
    u32x4* y = (u32x4*)y_bf16;
    if (wave_row_shape(rows, vecs_per_row, wave_row_min_rounds_recompute2(bits))) {
        auto go = [&](auto kernel) {
            return launch(kernel, dim3(wave_row_grid(rows)), dim3(kWaveRowWaves * 64), 0, st, codes, scales,
                          n_vec_total, rows, gm, eps, inv_cols, y, r_out);
        };
        return dispatch_wave_row_vpt(vecs_per_row, [&](auto v) {
            constexpr int V = decltype(v)::value;
            if (fp)
                return group == 128 ? go(act_dequant_rmsnorm_wave_kernel<4, 128, V, true>)
                                    : go(act_dequant_rmsnorm_wave_kernel<4, 64, V, true>);
            return dispatch_bits_group(bits, group, [&](auto b, auto g) {
                return go(act_dequant_rmsnorm_wave_kernel<decltype(b)::value, decltype(g)::value, V>);
            });
        });
    }
    int vpt, threads;
    norm_launch_shape(vecs_per_row, bits == 8 ? kNormVpt8 : bits == 4 ? kNormVpt : norm_vpt56(vecs_per_row), vpt,
                      threads);
    const dim3 grid(norm_grid(rows, threads)), block(threads);
    const bool pipe = vecs_per_row == vpt * threads && rows >= (int64_t)grid.x * kNormPipeRows;
    auto go = [&](auto kernel) {
        return launch(kernel, grid, block, 0, st, codes, scales, n_vec_total, rows, vecs_per_row, gm, eps,
                      inv_cols, y, r_out);
    };
    return dispatch_vpt(vpt, [&](auto v) {
        constexpr int V = decltype(v)::value;
        if (fp) {
            if (group == 128)
                return pipe ? go(act_dequant_rmsnorm_kernel<4, 128, V, true, true>)
                            : go(act_dequant_rmsnorm_kernel<4, 128, V, true, false>);
            return pipe ? go(act_dequant_rmsnorm_kernel<4, 64, V, true, true>)
                        : go(act_dequant_rmsnorm_kernel<4, 64, V, true, false>);
        }
        return dispatch_bits_group(bits, group, [&](auto b, auto g) {
            constexpr int B = decltype(b)::value, G = decltype(g)::value;
            return pipe ? go(act_dequant_rmsnorm_kernel<B, G, V, false, true>)
                        : go(act_dequant_rmsnorm_kernel<B, G, V, false, false>);
        });
    });
}

int dequant_silu_mul_impl(const void* gate_codes, const float* gate_scales, int gate_bits,
                          const void* up_codes, const float* up_scales, int up_bits, bool fp,
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
    constexpr int U = kSiUnroll;
    hipStream_t st = (hipStream_t)stream;
    u32x4* z = (u32x4*)z_bf16;
    // workgroups of 128 lanes while a tensor's decode is several instructions per element
    // (measured +2-4 % at 4, 5 and 6 bits; -1 to -6 % for two 8-bit tensors, which keep 256)
    auto go = [&](auto kernel, int block) {
        return launch(kernel, dim3(blocks_for(n_vec, block * U)), dim3(block), 0, st, gate_codes, gate_scales,
                      up_codes, up_scales, n_vec, z);
    };
    if (fp)
        return group == 128 ? go(act_dequant_silu_mul_kernel<4, 4, 128, kSiBlockNarrow, U, true>, kSiBlockNarrow)
                            : go(act_dequant_silu_mul_kernel<4, 4, 64, kSiBlockNarrow, U, true>, kSiBlockNarrow);
    return dispatch_bits_group(gate_bits, group, [&](auto bg, auto g) {
        // the group is the same for both tensors: the inner dispatch only resolves the up width
        return dispatch_bits_group(up_bits, group, [&](auto bu, auto) {
            constexpr int BG = decltype(bg)::value, BU = decltype(bu)::value, G = decltype(g)::value;
            constexpr int B = (BG == 8 && BU == 8) ? kSiBlock : kSiBlockNarrow;
            return go(act_dequant_silu_mul_kernel<BG, BU, G, B, U>, B);
        });
    });
}

int rmsnorm_fwd_quant_impl(const void* x_bf16, int64_t rows, int64_t cols, const float* gamma, float eps,
                           int group, int bits, bool fp, void* y_bf16, float* r_out, void* codes,
                           float* scales, void* stream)
{
    if (!x_bf16 || !gamma || !y_bf16 || !codes || !scales) return AGOQ_ERR_NULL;
    if (bits != 4 && bits != 5 && bits != 6 && bits != 8) return AGOQ_ERR_BITS;
    if (group != 64 && group != 128) return AGOQ_ERR_GROUP;
    if (rows <= 0 || rows > 0x7FFFFFFF || cols <= 0 || cols % group != 0 ||
        cols > kNormMaxCols)
        return AGOQ_ERR_SHAPE;
    if (misaligned(x_bf16) || misaligned(gamma) || misaligned(y_bf16) || misaligned(codes) ||
        misaligned(scales))
        return AGOQ_ERR_ALIGN;
    const int vecs_per_row = (int)(cols / 8);
    const int64_t n_vec_total = rows * vecs_per_row;
    const float inv_cols = 1.0f / (float)cols;
    hipStream_t st = (hipStream_t)stream;
    const u32x4* x = (const u32x4*)x_bf16;
    const f32x4* gm = (const f32x4*)gamma;
    u32x4* y = (u32x4*)y_bf16;
    if (wave_row_shape(rows, vecs_per_row, kWaveRowMinRoundsForward2)) {
        auto go = [&](auto kernel) {
            return launch(kernel, dim3(wave_row_grid(rows)), dim3(kWaveRowWaves * 64), 0, st, x, n_vec_total, rows,
                          gm, eps, inv_cols, y, r_out, codes, scales);
        };
        return dispatch_wave_row_vpt(vecs_per_row, [&](auto v) {
            constexpr int V = decltype(v)::value;
            if (fp)
                return group == 128 ? go(rmsnorm_fwd_quant_wave_kernel<4, 128, V, true>)
                                    : go(rmsnorm_fwd_quant_wave_kernel<4, 64, V, true>);
            return dispatch_bits_group(bits, group, [&](auto b, auto g) {
                return go(rmsnorm_fwd_quant_wave_kernel<decltype(b)::value, decltype(g)::value, V>);
            });
        });
    }
    int vpt, threads;
    norm_launch_shape(vecs_per_row, kNormFwdVpt, vpt, threads);
    const dim3 grid(norm_grid(rows, threads)), block(threads);
    const bool pipe = vecs_per_row == vpt * threads && rows >= (int64_t)grid.x * kNormPipeRows;
    auto go = [&](auto kernel) {
        return launch(kernel, grid, block, 0, st, x, n_vec_total, rows, vecs_per_row, gm, eps, inv_cols, y,
                      r_out, codes, scales);
    };
    return dispatch_vpt(vpt, [&](auto v) {
        constexpr int V = decltype(v)::value;
        if (fp) {
            if (group == 128)
                return pipe ? go(rmsnorm_fwd_quant_kernel<4, 128, V, true, true>)
                            : go(rmsnorm_fwd_quant_kernel<4, 128, V, true, false>);
            return pipe ? go(rmsnorm_fwd_quant_kernel<4, 64, V, true, true>)
                        : go(rmsnorm_fwd_quant_kernel<4, 64, V, true, false>);
        }
        return dispatch_bits_group(bits, group, [&](auto b, auto g) {
            constexpr int B = decltype(b)::value, G = decltype(g)::value;
            return pipe ? go(rmsnorm_fwd_quant_kernel<B, G, V, false, true>)
                        : go(rmsnorm_fwd_quant_kernel<B, G, V, false, false>);
        });
    });
}

int silu_mul_fwd_quant_impl(const void* gate_bf16, const void* up_bf16, int64_t numel, int group,
                            int gate_bits, int up_bits, bool fp, void* z_bf16, void* gate_codes,
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
    const dim3 grid(blocks_for(n_vec, kAqBlock * U)), block(kAqBlock);
    hipStream_t st = (hipStream_t)stream;
    const u32x4* g = (const u32x4*)gate_bf16;
    const u32x4* up = (const u32x4*)up_bf16;
    u32x4* z = (u32x4*)z_bf16;
    auto go = [&](auto kernel) {
        return launch(kernel, grid, block, kCapSf, st, g, up, n_vec, z, gate_codes, gate_scales, up_codes,
                      up_scales);
    };
    if (fp)
        return group == 128 ? go(silu_mul_fwd_quant_kernel<4, 4, 128, U, true>)
                            : go(silu_mul_fwd_quant_kernel<4, 4, 64, U, true>);
    return dispatch_bits_group(gate_bits, group, [&](auto bg, auto gr) {
        return dispatch_bits_group(up_bits, group, [&](auto bu, auto) {
            return go(silu_mul_fwd_quant_kernel<decltype(bg)::value, decltype(bu)::value, decltype(gr)::value, U>);
        });
    });
}

}  // namespace

extern "C" {

int agoq_act_dequant_rmsnorm(const void* codes, const float* scales, int64_t rows, int64_t cols,
                             int group, int bits, const float* gamma, float eps, void* y_bf16,
                             float* r_out, void* stream)
{
    return dequant_rmsnorm_impl(codes, scales, rows, cols, group, bits, false, gamma, eps, y_bf16,
                                r_out, stream);
}

int agoq_act_dequant_silu_mul(const void* gate_codes, const float* gate_scales, int gate_bits,
                              const void* up_codes, const float* up_scales, int up_bits,
                              int64_t numel, int group, void* z_bf16, void* stream)
{
    return dequant_silu_mul_impl(gate_codes, gate_scales, gate_bits, up_codes, up_scales, up_bits,
                                 false, numel, group, z_bf16, stream);
}

int agoq_rmsnorm_fwd_quant(const void* x_bf16, int64_t rows, int64_t cols, const float* gamma,
                           float eps, int group, int bits, void* y_bf16, float* r_out, void* codes,
                           float* scales, void* stream)
{
    return rmsnorm_fwd_quant_impl(x_bf16, rows, cols, gamma, eps, group, bits, false, y_bf16, r_out,
                                  codes, scales, stream);
}

int agoq_silu_mul_fwd_quant(const void* gate_bf16, const void* up_bf16, int64_t numel, int group,
                            int gate_bits, int up_bits, void* z_bf16, void* gate_codes,
                            float* gate_scales, void* up_codes, float* up_scales, void* stream)
{
    return silu_mul_fwd_quant_impl(gate_bf16, up_bf16, numel, group, gate_bits, up_bits, false,
                                   z_bf16, gate_codes, gate_scales, up_codes, up_scales, stream);
}

int agoq_fp4_act_dequant_rmsnorm(const void* codes, const float* scales, int64_t rows, int64_t cols,
                                 int group, const float* gamma, float eps, void* y_bf16,
                                 float* r_out, void* stream)
{
    return dequant_rmsnorm_impl(codes, scales, rows, cols, group, 4, true, gamma, eps, y_bf16, r_out,
                                stream);
}

int agoq_fp4_act_dequant_silu_mul(const void* gate_codes, const float* gate_scales,
                                  const void* up_codes, const float* up_scales, int64_t numel,
                                  int group, void* z_bf16, void* stream)
{
    return dequant_silu_mul_impl(gate_codes, gate_scales, 4, up_codes, up_scales, 4, true, numel,
                                 group, z_bf16, stream);
}

int agoq_fp4_rmsnorm_fwd_quant(const void* x_bf16, int64_t rows, int64_t cols, const float* gamma,
                               float eps, int group, void* y_bf16, float* r_out, void* codes,
                               float* scales, void* stream)
{
    return rmsnorm_fwd_quant_impl(x_bf16, rows, cols, gamma, eps, group, 4, true, y_bf16, r_out,
                                  codes, scales, stream);
}

int agoq_fp4_silu_mul_fwd_quant(const void* gate_bf16, const void* up_bf16, int64_t numel, int group,
                                void* z_bf16, void* gate_codes, float* gate_scales, void* up_codes,
                                float* up_scales, void* stream)
{
    return silu_mul_fwd_quant_impl(gate_bf16, up_bf16, numel, group, 4, 4, true, z_bf16, gate_codes,
                                   gate_scales, up_codes, up_scales, stream);
}

}  // extern "C"
