// Host-only driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the CPU
// oracle (oracle/agoq_ref.c) and of the library's host helpers (csrc/agoq_host.cpp).
// Every buffer is a heap allocation of EXACTLY the size the call's contract states, so a
// read or write one byte past it aborts the run; group counts are ragged, strides exceed
// the extents, 5- and 6-bit planes and K = 64 are covered.  Test infrastructure; built and
// run by tests/test_sanitizers.py.  Touches no GPU.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "agoq.h"

extern "C" {
int agoq_ref_act_quant(const uint16_t*, int64_t, int, int, uint8_t*, float*);
int agoq_ref_act_dequant(const uint8_t*, const float*, int64_t, int, int, uint16_t*);
int agoq_ref_act_dequant_rmsnorm(const uint8_t*, const float*, int64_t, int64_t, int, int, const float*, float,
                                 uint16_t*, float*);
int agoq_ref_act_dequant_silu_mul(const uint8_t*, const float*, int, const uint8_t*, const float*, int, int64_t,
                                  int, uint16_t*);
int agoq_ref_rmsnorm_fwd(const uint16_t*, int64_t, int64_t, const float*, float, uint16_t*, float*);
int agoq_ref_silu_mul_fwd(const uint16_t*, const uint16_t*, int64_t, uint16_t*);
int agoq_ref_grad_quant(const float*, int64_t, int, int8_t*, float*);
int agoq_ref_grad_dequant(const int8_t*, const float*, int64_t, int, float*);
int agoq_ref_grad_reduce_requant(const int8_t*, int64_t, const float*, int64_t, int, int64_t, int, int8_t*, float*);
int agoq_ref_grad_reduce_f64(const int8_t*, int64_t, const float*, int64_t, int, int64_t, int, double*, double*);
int agoq_ref_grad_accumulate(const int8_t*, const float*, const void*, int, int64_t, int, int8_t*, float*);
int agoq_ref_fp4_act_quant(const uint16_t*, int64_t, int, uint8_t*, float*);
int agoq_ref_fp4_act_dequant(const uint8_t*, const float*, int64_t, int, uint16_t*);
int agoq_ref_fp8_grad_quant(const float*, int64_t, int, uint8_t*, float*);
int agoq_ref_fp8_grad_dequant(const uint8_t*, const float*, int64_t, int, float*);
int agoq_ref_fp8_grad_reduce_requant(const uint8_t*, int64_t, const float*, int64_t, int, int64_t, int, uint8_t*,
                                     float*);
int agoq_ref_fp8_grad_accumulate(const uint8_t*, const float*, const void*, int, int64_t, int, uint8_t*, float*);
int agoq_ref_dbca_bits(int, int, int*);
int agoq_ref_dbca_stored_microbatches(int, int);
float agoq_ref_bf16_to_f32(uint16_t);
uint16_t agoq_ref_f32_to_bf16(float);
void agoq_ref_set_threads(int);
}

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            printf("line %d: expectation failed: %s\n", __LINE__, #cond);   \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

static uint32_t state = 2463534242u;
static uint32_t rnd() { state ^= state << 13; state ^= state >> 17; state ^= state << 5; return state; }
static float bell() { return ((int)(rnd() % 2001) - 1000 + (int)(rnd() % 2001) - 1000) / 500.0f; }

// exact-size heap buffers (std::vector<T>::data() of a vector sized to the byte)
template <typename T> static std::vector<T> buf(int64_t n) { return std::vector<T>((size_t)n); }

static void activations()
{
    const int groups_list[] = {1, 3, 7, 13};
    for (int group : {64, 128})
        for (int bits : {4, 5, 6, 8})
            for (int groups : groups_list) {
                const int64_t n = (int64_t)group * groups;
                auto x = buf<uint16_t>(n);
                for (auto& v : x) v = agoq_ref_f32_to_bf16(bell() * ((rnd() & 31) == 0 ? 30.0f : 1.0f));
                if (groups > 1) memset(x.data() + group, 0, group * 2);      // a dead group
                auto codes = buf<uint8_t>(n * bits / 8);
                auto scales = buf<float>(groups);
                auto y = buf<uint16_t>(n);
                EXPECT(agoq_ref_act_quant(x.data(), n, group, bits, codes.data(), scales.data()) == 0);
                EXPECT(agoq_ref_act_dequant(codes.data(), scales.data(), n, group, bits, y.data()) == 0);
                for (int64_t i = 0; i < n; ++i) {
                    const float s = scales[i / group];
                    const double err = fabs((double)agoq_ref_bf16_to_f32(x[i]) - (double)agoq_ref_bf16_to_f32(y[i]));
                    EXPECT(err <= 0.5 * s * 1.001 + fabs(agoq_ref_bf16_to_f32(y[i])) / 256.0 + 1e-30);
                }
                if (bits == 4) {
                    EXPECT(agoq_ref_fp4_act_quant(x.data(), n, group, codes.data(), scales.data()) == 0);
                    EXPECT(agoq_ref_fp4_act_dequant(codes.data(), scales.data(), n, group, y.data()) == 0);
                }
            }
    // the fused layer functions: rows x cols with cols a ragged multiple of the group
    for (int group : {64, 128})
        for (int bits : {4, 5, 6, 8}) {
            const int64_t rows = 5, cols = (int64_t)group * 3, n = rows * cols;
            auto x = buf<uint16_t>(n), up = buf<uint16_t>(n), y = buf<uint16_t>(n), z = buf<uint16_t>(n);
            for (auto& v : x) v = agoq_ref_f32_to_bf16(bell());
            for (auto& v : up) v = agoq_ref_f32_to_bf16(bell());
            auto gamma = buf<float>(cols);
            for (auto& g : gamma) g = 1.0f + 0.1f * bell();
            auto r = buf<float>(rows);
            auto c0 = buf<uint8_t>(n * bits / 8), c1 = buf<uint8_t>(n * bits / 8);
            auto s0 = buf<float>(n / group), s1 = buf<float>(n / group);
            EXPECT(agoq_ref_rmsnorm_fwd(x.data(), rows, cols, gamma.data(), 1e-5f, y.data(), r.data()) == 0);
            EXPECT(agoq_ref_silu_mul_fwd(x.data(), up.data(), n, z.data()) == 0);
            EXPECT(agoq_ref_act_quant(x.data(), n, group, bits, c0.data(), s0.data()) == 0);
            EXPECT(agoq_ref_act_quant(up.data(), n, group, bits, c1.data(), s1.data()) == 0);
            EXPECT(agoq_ref_act_dequant_rmsnorm(c0.data(), s0.data(), rows, cols, group, bits, gamma.data(), 1e-5f,
                                                y.data(), r.data()) == 0);
            EXPECT(agoq_ref_act_dequant_silu_mul(c0.data(), s0.data(), bits, c1.data(), s1.data(), bits, n, group,
                                                 z.data()) == 0);
            for (int64_t i = 0; i < rows; ++i) EXPECT(r[i] > 0.0f);
        }
    // rejected arguments touch nothing
    uint8_t c = 0;
    float s = 0;
    uint16_t x = 0;
    EXPECT(agoq_ref_act_quant(&x, 100, 128, 4, &c, &s) != 0);
    EXPECT(agoq_ref_act_quant(&x, 128, 128, 7, &c, &s) != 0);
    EXPECT(agoq_ref_act_quant(&x, 128, 0, 4, &c, &s) != 0);
    EXPECT(agoq_ref_act_quant(&x, 8192, 8192, 4, &c, &s) != 0);
    EXPECT(agoq_ref_act_quant(nullptr, 128, 128, 4, &c, &s) != 0);
}

template <typename CODE, typename QUANT, typename DEQUANT, typename REDUCE, typename ACCUM>
static void gradients(QUANT quant, DEQUANT dequant, REDUCE reduce, ACCUM accum)
{
    for (int group : {64, 128})
        for (int groups : {1, 5, 11}) {
            const int64_t n = (int64_t)group * groups;
            auto g = buf<float>(n);
            for (auto& v : g) v = 1e-4f * bell() * ((rnd() & 127) == 0 ? 100.0f : 1.0f);
            auto codes = buf<CODE>(n);
            auto scales = buf<float>(groups);
            auto out = buf<float>(n);
            EXPECT(quant(g.data(), n, group, codes.data(), scales.data()) == 0);
            EXPECT(dequant(codes.data(), scales.data(), n, group, out.data()) == 0);
            // accumulation with an fp32 and with a bf16 addend, out of place and in place
            auto gb = buf<uint16_t>(n);
            for (int64_t i = 0; i < n; ++i) gb[i] = agoq_ref_f32_to_bf16(g[i]);
            auto oc = buf<CODE>(n);
            auto os = buf<float>(groups);
            EXPECT(accum(codes.data(), scales.data(), g.data(), 0, n, group, oc.data(), os.data()) == 0);
            EXPECT(accum(codes.data(), scales.data(), gb.data(), 1, n, group, oc.data(), os.data()) == 0);
            EXPECT(accum(codes.data(), scales.data(), g.data(), 0, n, group, codes.data(), scales.data()) == 0);
            for (int K : {1, 3, 16, 64}) {
                // chunk k starts k*stride into the receive buffer; the buffer ends with the last
                // chunk's last element: (K-1)*stride + extent
                const int64_t stride_c = n + 16 * 3, stride_s = groups + 5;
                auto ic = buf<CODE>((K - 1) * stride_c + n);
                auto is = buf<float>((K - 1) * stride_s + groups);
                for (auto& v : ic) v = (CODE)(rnd() & 0x77);          // finite in both code books
                for (auto& v : is) v = 1e-6f * (float)(1 + (rnd() & 1023));
                auto rc = buf<CODE>(n);
                auto rs = buf<float>(groups);
                EXPECT(reduce(ic.data(), stride_c, is.data(), stride_s, K, n, group, rc.data(), rs.data()) == 0);
                // strides equal to the extents: the tightest legal buffer
                auto tc = buf<CODE>((int64_t)K * n);
                auto ts = buf<float>((int64_t)K * groups);
                for (auto& v : tc) v = (CODE)(rnd() & 0x77);
                for (auto& v : ts) v = 1e-6f * (float)(1 + (rnd() & 1023));
                EXPECT(reduce(tc.data(), n, ts.data(), groups, K, n, group, rc.data(), rs.data()) == 0);
                EXPECT(reduce(tc.data(), n - 16, ts.data(), groups, K, n, group, rc.data(), rs.data()) != 0);
                EXPECT(reduce(tc.data(), n, ts.data(), groups, 65, n, group, rc.data(), rs.data()) != 0);
            }
        }
}

static void host_helpers()
{
    for (int bits = 0; bits <= 9; ++bits) {
        const int64_t b = agoq_codes_bytes(1024, bits);
        EXPECT((bits == 4 || bits == 5 || bits == 6 || bits == 8) ? b == 1024 * bits / 8 : b == -1);
    }
    EXPECT(agoq_codes_bytes(-1, 4) == -1);
    EXPECT(agoq_num_groups(1024, 128) == 8 && agoq_num_groups(1000, 128) == -1 && agoq_num_groups(0, 128) == -1);
    for (int n = 1; n <= 16; ++n)
        for (int stage = 0; stage <= n + 1; ++stage) {
            int b = -1, br = -1;
            const int rc = agoq_dbca_bits(n, stage, &b);
            const int rr = agoq_ref_dbca_bits(n, stage, &br);
            EXPECT((rc == 0) == (rr == 0));
            if (rc == 0) EXPECT(b == br && b >= 4 && b <= 8);
            EXPECT(agoq_dbca_stored_microbatches(n, stage) == agoq_ref_dbca_stored_microbatches(n, stage));
        }
    EXPECT(agoq_dbca_bits(4, 1, nullptr) == AGOQ_ERR_NULL);
    for (int target = 3; target <= 9; ++target) {
        int mix[AGOQ_LAYER_SLOTS], native[AGOQ_LAYER_SLOTS];
        const int rc = agoq_layer_bitmap(target, mix);
        EXPECT((rc == 0) == (target >= 4 && target <= 8));
        EXPECT((agoq_layer_bitmap_native(target, native) == 0) == (rc == 0));
        if (rc == 0) {
            EXPECT(agoq_layer_stored_bytes(4096, 4096, 14336, 128, mix, 1) > 0);
            EXPECT(agoq_layer_stored_bytes(4096, 4096, 14336, 128, native, 0) > 0);
        }
    }
    EXPECT(agoq_layer_bitmap(4, nullptr) == AGOQ_ERR_NULL);
    const int bad[AGOQ_LAYER_SLOTS] = {4, 4, 7, 4, 4};
    EXPECT(agoq_layer_stored_bytes(4096, 4096, 14336, 128, bad, 1) == -1);
    EXPECT(agoq_layer_stored_bytes(4096, 4100, 14336, 128, nullptr, 1) == -1);
    for (int status = -2; status <= 12; ++status) EXPECT(strlen(agoq_strerror(status)) > 0);
    EXPECT(agoq_version() > 0);
}

int main()
{
    for (int threads : {1, 4}) {
        agoq_ref_set_threads(threads);
        activations();
        gradients<int8_t>(agoq_ref_grad_quant, agoq_ref_grad_dequant, agoq_ref_grad_reduce_requant,
                          agoq_ref_grad_accumulate);
        gradients<uint8_t>(agoq_ref_fp8_grad_quant, agoq_ref_fp8_grad_dequant, agoq_ref_fp8_grad_reduce_requant,
                           agoq_ref_fp8_grad_accumulate);
    }
    // binary64 yardstick of the reduce
    {
        const int K = 5, group = 128;
        const int64_t n = 128 * 3;
        auto ic = buf<int8_t>((int64_t)K * n);
        auto is = buf<float>((int64_t)K * 3);
        for (auto& v : ic) v = (int8_t)(rnd() & 0xFF);
        for (auto& v : is) v = 1e-5f;
        auto sum = buf<double>(n), abs_sum = buf<double>(n);
        EXPECT(agoq_ref_grad_reduce_f64(ic.data(), n, is.data(), 3, K, n, group, sum.data(), abs_sum.data()) == 0);
    }
    host_helpers();
    printf("%s\n", failures ? "FAILED" : "sanitizer run clean");
    return failures ? 1 : 0;
}
