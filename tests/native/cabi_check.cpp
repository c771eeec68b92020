// A torch-free client of the C ABI: device memory from hipMalloc, inputs from a small
// linear congruential generator, results compared byte for byte with the CPU oracle
// (linked directly).  Exit status 0 = every comparison matched.
//
//   hipcc --offload-arch=gfx950 -O2 -I include tests/native/cabi_check.cpp \
//         -L paper_2605_00539_amd -lagoq -L oracle -lagoq_ref -o tests/native/cabi_check
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "agoq.h"

extern "C" {
int agoq_ref_act_quant(const uint16_t*, int64_t, int, int, uint8_t*, float*);
int agoq_ref_act_dequant(const uint8_t*, const float*, int64_t, int, int, uint16_t*);
int agoq_ref_grad_quant(const float*, int64_t, int, int8_t*, float*);
int agoq_ref_grad_reduce_requant(const int8_t*, int64_t, const float*, int64_t, int, int64_t, int,
                                 int8_t*, float*);
}

#define HIP_OK(x)                                                                       \
    do {                                                                                \
        hipError_t e_ = (x);                                                            \
        if (e_ != hipSuccess) {                                                         \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);       \
            return 2;                                                                   \
        }                                                                               \
    } while (0)

static uint32_t lcg_state = 12345u;
static uint32_t lcg() { return lcg_state = lcg_state * 1664525u + 1013904223u; }
// roughly bell-shaped value in (-6, 6): sum of twelve uniforms minus six
static float bell() {
    float s = 0.f;
    for (int i = 0; i < 12; ++i) s += (float)(lcg() >> 8) * (1.0f / 16777216.0f);
    return s - 6.0f;
}
static uint16_t to_bf16_trunc(float f) {   // inputs only: any bf16 pattern is a valid input
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

template <typename T>
static T* dev_copy(const std::vector<T>& h) {
    T* d = nullptr;
    if (hipMalloc(&d, h.size() * sizeof(T)) != hipSuccess) return nullptr;
    if (hipMemcpy(d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
    return d;
}

int main() {
    int failures = 0;
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    for (int group : {64, 128}) {
        for (int bits : {4, 5, 6, 8}) {
            const int64_t n = (int64_t)group * 4099;
            std::vector<uint16_t> x(n);
            for (auto& v : x) v = to_bf16_trunc(bell() * ((lcg() & 63) == 0 ? 30.f : 1.f));
            std::vector<uint8_t> codes_ref(n * bits / 8), codes(n * bits / 8);
            std::vector<float> scales_ref(n / group), scales(n / group);
            std::vector<uint16_t> y_ref(n), y(n);
            agoq_ref_act_quant(x.data(), n, group, bits, codes_ref.data(), scales_ref.data());
            agoq_ref_act_dequant(codes_ref.data(), scales_ref.data(), n, group, bits, y_ref.data());
            uint16_t* dx = dev_copy(x);
            uint8_t* dc = nullptr;
            float* ds = nullptr;
            uint16_t* dy = nullptr;
            HIP_OK(hipMalloc(&dc, codes.size()));
            HIP_OK(hipMalloc(&ds, scales.size() * 4));
            HIP_OK(hipMalloc(&dy, n * 2));
            if (!dx) return 2;
            int rc = agoq_act_quant(dx, n, group, bits, dc, ds, stream);
            if (rc == AGOQ_OK) rc = agoq_act_dequant(dc, ds, n, group, bits, dy, stream);
            if (rc != AGOQ_OK) { printf("status %d: %s\n", rc, agoq_strerror(rc)); return 2; }
            HIP_OK(hipStreamSynchronize(stream));
            HIP_OK(hipMemcpy(codes.data(), dc, codes.size(), hipMemcpyDeviceToHost));
            HIP_OK(hipMemcpy(scales.data(), ds, scales.size() * 4, hipMemcpyDeviceToHost));
            HIP_OK(hipMemcpy(y.data(), dy, n * 2, hipMemcpyDeviceToHost));
            const bool ok = codes == codes_ref && !memcmp(scales.data(), scales_ref.data(), scales.size() * 4) && y == y_ref;
            printf("act group %3d bits %d: %s\n", group, bits, ok ? "match" : "MISMATCH");
            failures += !ok;
            HIP_OK(hipFree(dx)); HIP_OK(hipFree(dc)); HIP_OK(hipFree(ds)); HIP_OK(hipFree(dy));
        }
        // gradient store and K-way reduce
        const int K = 5;
        const int64_t n = (int64_t)group * 2053, stride_c = n + 48, stride_s = n / group + 1;
        std::vector<float> g(n);
        for (auto& v : g) v = bell() * 1e-4f * ((lcg() & 1023) == 0 ? 100.f : 1.f);
        std::vector<int8_t> gc_ref(n), gc(n), in_codes(K * stride_c), rc_ref(n), rcodes(n);
        std::vector<float> gs_ref(n / group), gs(n / group), in_scales(K * stride_s), rs_ref(n / group), rs(n / group);
        agoq_ref_grad_quant(g.data(), n, group, gc_ref.data(), gs_ref.data());
        for (auto& v : in_codes) v = (int8_t)(lcg() >> 24);
        for (auto& v : in_scales) v = (float)(lcg() >> 8) * (1e-5f / 16777216.0f);
        agoq_ref_grad_reduce_requant(in_codes.data(), stride_c, in_scales.data(), stride_s, K, n, group,
                                     rc_ref.data(), rs_ref.data());
        float* dg = dev_copy(g);
        int8_t* dic = dev_copy(in_codes);
        float* dis = dev_copy(in_scales);
        int8_t *dgc = nullptr, *drc = nullptr;
        float *dgs = nullptr, *drs = nullptr;
        HIP_OK(hipMalloc(&dgc, n)); HIP_OK(hipMalloc(&drc, n));
        HIP_OK(hipMalloc(&dgs, (n / group) * 4)); HIP_OK(hipMalloc(&drs, (n / group) * 4));
        if (!dg || !dic || !dis) return 2;
        int rc = agoq_grad_quant(dg, n, group, dgc, dgs, stream);
        if (rc == AGOQ_OK) rc = agoq_grad_reduce_requant(dic, stride_c, dis, stride_s, K, n, group, drc, drs, stream);
        if (rc != AGOQ_OK) { printf("status %d: %s\n", rc, agoq_strerror(rc)); return 2; }
        HIP_OK(hipStreamSynchronize(stream));
        HIP_OK(hipMemcpy(gc.data(), dgc, n, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(gs.data(), dgs, (n / group) * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(rcodes.data(), drc, n, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(rs.data(), drs, (n / group) * 4, hipMemcpyDeviceToHost));
        const bool ok = gc == gc_ref && !memcmp(gs.data(), gs_ref.data(), gs.size() * 4) && rcodes == rc_ref &&
                        !memcmp(rs.data(), rs_ref.data(), rs.size() * 4);
        printf("grad group %3d store + %d-chunk reduce: %s\n", group, K, ok ? "match" : "MISMATCH");
        failures += !ok;
        HIP_OK(hipFree(dg)); HIP_OK(hipFree(dic)); HIP_OK(hipFree(dis)); HIP_OK(hipFree(dgc));
        HIP_OK(hipFree(drc)); HIP_OK(hipFree(dgs)); HIP_OK(hipFree(drs));
    }
    // one launch for a layer: three tensors of different sizes at three widths
    {
        const int group = 128;
        const int bits[3] = {8, 4, 6};
        const int64_t numel[3] = {(int64_t)group * 1031, (int64_t)group * 4099, (int64_t)group * 517};
        std::vector<uint16_t> x[3], y[3], y_ref[3];
        std::vector<uint8_t> c[3], c_ref[3];
        std::vector<float> sc[3], sc_ref[3];
        agoq_act_slot slots[3];
        for (int t = 0; t < 3; ++t) {
            const int64_t n = numel[t];
            x[t].resize(n); y[t].resize(n); y_ref[t].resize(n);
            c[t].resize(n * bits[t] / 8); c_ref[t].resize(n * bits[t] / 8);
            sc[t].resize(n / group); sc_ref[t].resize(n / group);
            for (auto& v : x[t]) v = to_bf16_trunc(bell() * ((lcg() & 63) == 0 ? 30.f : 1.f));
            agoq_ref_act_quant(x[t].data(), n, group, bits[t], c_ref[t].data(), sc_ref[t].data());
            agoq_ref_act_dequant(c_ref[t].data(), sc_ref[t].data(), n, group, bits[t], y_ref[t].data());
            uint8_t* dc = nullptr;
            float* ds = nullptr;
            HIP_OK(hipMalloc(&dc, c[t].size()));
            HIP_OK(hipMalloc(&ds, sc[t].size() * 4));
            slots[t].bf16 = dev_copy(x[t]);
            slots[t].codes = dc;
            slots[t].scales = ds;
            slots[t].numel = n;
            slots[t].bits = bits[t];
            if (!slots[t].bf16) return 2;
        }
        int rc = agoq_act_quant_layer(slots, 3, group, stream);
        if (rc != AGOQ_OK) { printf("status %d: %s\n", rc, agoq_strerror(rc)); return 2; }
        HIP_OK(hipStreamSynchronize(stream));
        for (int t = 0; t < 3; ++t)      // wipe the inputs: the dequantize must rewrite them
            HIP_OK(hipMemset(slots[t].bf16, 0xFF, numel[t] * 2));
        rc = agoq_act_dequant_layer(slots, 3, group, stream);
        if (rc != AGOQ_OK) { printf("status %d: %s\n", rc, agoq_strerror(rc)); return 2; }
        HIP_OK(hipStreamSynchronize(stream));
        bool ok = true;
        for (int t = 0; t < 3; ++t) {
            HIP_OK(hipMemcpy(c[t].data(), slots[t].codes, c[t].size(), hipMemcpyDeviceToHost));
            HIP_OK(hipMemcpy(sc[t].data(), slots[t].scales, sc[t].size() * 4, hipMemcpyDeviceToHost));
            HIP_OK(hipMemcpy(y[t].data(), slots[t].bf16, numel[t] * 2, hipMemcpyDeviceToHost));
            ok = ok && c[t] == c_ref[t] && !memcmp(sc[t].data(), sc_ref[t].data(), sc[t].size() * 4) &&
                 y[t] == y_ref[t];
            HIP_OK(hipFree(slots[t].bf16)); HIP_OK(hipFree(slots[t].codes)); HIP_OK(hipFree(slots[t].scales));
        }
        printf("layer launch, 3 tensors at 8/4/6 bits: %s\n", ok ? "match" : "MISMATCH");
        failures += !ok;
        if (agoq_act_quant_layer(slots, 0, group, stream) != AGOQ_ERR_COUNT) ++failures;
        if (agoq_act_quant_layer(slots, 9, group, stream) != AGOQ_ERR_COUNT) ++failures;
    }
    // error paths: nothing launched
    if (agoq_act_quant(nullptr, 128, 128, 4, nullptr, nullptr, nullptr) != AGOQ_ERR_NULL) ++failures;
    // An error that an earlier, unrelated HIP call of the caller left behind is neither reported
    // as a library call's status nor cleared by it.  (An invalid device ordinal is refused on
    // the host; nothing reaches the GPU.)
    {
        const int group = 128;
        const int64_t n = (int64_t)group * 64;
        std::vector<uint16_t> x(n);
        for (auto& v : x) v = to_bf16_trunc(bell());
        uint16_t* dx = dev_copy(x);
        uint8_t* dc = nullptr;
        float* ds = nullptr;
        HIP_OK(hipMalloc(&dc, n / 2));
        HIP_OK(hipMalloc(&ds, n / group * 4));
        const bool refused = hipSetDevice(12345) != hipSuccess;     // leaves the error behind
        const int rc = agoq_act_quant(dx, n, group, 4, dc, ds, stream);
        const bool still_there = hipPeekAtLastError() != hipSuccess;
        (void)hipGetLastError();                                     // the caller clears its own error
        HIP_OK(hipStreamSynchronize(stream));
        std::vector<uint8_t> c(n / 2), c_ref(n / 2);
        std::vector<float> sc(n / group), sc_ref(n / group);
        HIP_OK(hipMemcpy(c.data(), dc, c.size(), hipMemcpyDeviceToHost));
        agoq_ref_act_quant(x.data(), n, group, 4, c_ref.data(), sc_ref.data());
        // (whether the runtime itself keeps an error across later successful calls is its
        // business: reported, not required)
        const bool ok = refused && rc == AGOQ_OK && c == c_ref;
        printf("a caller's earlier HIP error is not this call's (%s afterwards): %s\n",
               still_there ? "still pending" : "gone", ok ? "match" : "MISMATCH");
        failures += !ok;
        HIP_OK(hipFree(dx)); HIP_OK(hipFree(dc)); HIP_OK(hipFree(ds));
    }
    HIP_OK(hipStreamDestroy(stream));
    printf("%s\n", failures ? "FAILED" : "all C-ABI checks passed");
    return failures ? 1 : 0;
}
