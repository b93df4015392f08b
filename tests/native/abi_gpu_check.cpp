// The C ABI of libtidal driven from a plain HIP host program: no Python, no framework, the system's HIP
// runtime.  Materialise three tensors (fp16, fp32, a ragged 1-D one), attach an adapter given by host
// pointers (pageable memory), swap to a second one, detach -- with ordered accumulation, so every state
// is compared bit for bit with the CPU oracle, which this test program links as its checker.
// Exit status 0 and the line "abi gpu check ok" on success.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "tidal.h"

extern "C" {
void orc_convert_to_bf16(const void* src, int dtype, int64_t n, uint16_t* dst);
void orc_lora_merge_bf16(uint16_t* W, int64_t out, int64_t in, const uint16_t* A, const uint16_t* B, int32_t r, float alpha,
                         int sign, int short_circuit);
void orc_lora_swap_bf16(uint16_t* W, int64_t out, int64_t in, const uint16_t* A_old, const uint16_t* B_old, int32_t r_old,
                        float alpha_old, const uint16_t* A_new, const uint16_t* B_new, int32_t r_new, float alpha_new);
}

#define CHECK_HIP(x)                                                                       \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            fprintf(stderr, "%s: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__);    \
            return 2;                                                                      \
        }                                                                                  \
    } while (0)
#define CHECK_TIDAL(x)                                                                     \
    do {                                                                                   \
        int rc_ = (x);                                                                     \
        if (rc_ != TIDAL_OK) {                                                             \
            fprintf(stderr, "%s = %d: %s (line %d)\n", #x, rc_, tidal_last_error(), __LINE__); \
            return 3;                                                                      \
        }                                                                                  \
    } while (0)

static uint32_t g_state = 12345u;
static float uniform(float scale) {                        // (-scale, scale), a plain LCG
    g_state = g_state * 1664525u + 1013904223u;
    return scale * ((float)(g_state >> 8) / 8388608.0f - 1.0f);
}

struct Adapter {
    int32_t r[2];
    float alpha[2];
    std::vector<float> A[2], B[2];                         // fp32 on the host, pageable
    std::vector<uint16_t> Ab[2], Bb[2];                    // what the device copy must hold: the oracle's conversion
};

int main() {
    int ndev = 0;
    CHECK_HIP(hipGetDeviceCount(&ndev));
    if (ndev < 1) { fprintf(stderr, "no GPU\n"); return 2; }
    CHECK_HIP(hipSetDevice(0));
    const tidal_slot_desc slots[3] = {{300, 520}, {64, 96}, {1, 7}};
    const int64_t elems[3] = {300 * 520, 64 * 96, 7};
    tidal_config cfg;
    CHECK_TIDAL(tidal_config_default(&cfg));
    cfg.chunk_bytes = 64 << 10;
    cfg.max_adapter_bytes = 1 << 20;
    cfg.flags = TIDAL_FLAG_ORDERED_ACCUM;
    const size_t need = tidal_template_required_bytes(slots, 3, &cfg);
    if (need == 0) { fprintf(stderr, "required_bytes: %s\n", tidal_last_error()); return 3; }
    void* arena = nullptr;
    CHECK_HIP(hipMalloc(&arena, need));
    CHECK_HIP(hipMemset(arena, 0x5A, need));
    tidal_template* t = nullptr;
    CHECK_TIDAL(tidal_template_create(slots, 3, arena, need, &cfg, &t));
    hipStream_t copy_s, comp_s;
    CHECK_HIP(hipStreamCreateWithFlags(&copy_s, hipStreamNonBlocking));
    CHECK_HIP(hipStreamCreateWithFlags(&comp_s, hipStreamNonBlocking));

    // sources: slot 0 fp16 (pinned), slot 1 fp32 (pinned), slot 2 fp32 (pageable: takes the gathered path)
    _Float16* s0 = nullptr;
    float* s1 = nullptr;
    CHECK_HIP(hipHostMalloc((void**)&s0, elems[0] * sizeof(_Float16), hipHostMallocDefault));
    CHECK_HIP(hipHostMalloc((void**)&s1, elems[1] * sizeof(float), hipHostMallocDefault));
    std::vector<float> s2(elems[2]);
    for (int64_t i = 0; i < elems[0]; ++i) s0[i] = (_Float16)uniform(0.05f);
    for (int64_t i = 0; i < elems[1]; ++i) s1[i] = uniform(0.05f);
    for (int64_t i = 0; i < elems[2]; ++i) s2[i] = uniform(0.05f);
    const tidal_src srcs[3] = {{0, TIDAL_F16, s0}, {1, TIDAL_F32, s1}, {2, TIDAL_F32, s2.data()}};
    CHECK_TIDAL(tidal_materialize(t, srcs, 3, copy_s, comp_s));
    CHECK_TIDAL(tidal_template_sync(t));

    std::vector<uint16_t> want[3], got[3];
    const int dt[3] = {TIDAL_F16, TIDAL_F32, TIDAL_F32};
    const void* sp[3] = {s0, s1, s2.data()};
    auto fetch = [&](int i) -> int {
        void* p = nullptr;
        size_t nb = 0;
        CHECK_TIDAL(tidal_template_slot_ptr(t, i, &p, &nb));
        if (nb != (size_t)elems[i] * 2) { fprintf(stderr, "slot %d: %zu bytes\n", i, nb); return 4; }
        got[i].resize(elems[i]);
        CHECK_HIP(hipMemcpy(got[i].data(), p, nb, hipMemcpyDeviceToHost));
        return 0;
    };
    auto same = [&](const char* what) -> int {
        for (int i = 0; i < 3; ++i) {
            int rc = fetch(i);
            if (rc) return rc;
            if (memcmp(got[i].data(), want[i].data(), (size_t)elems[i] * 2)) {
                int64_t bad = 0;
                for (int64_t e = 0; e < elems[i]; ++e) bad += got[i][e] != want[i][e];
                fprintf(stderr, "%s: slot %d differs from the oracle in %lld elements\n", what, i, (long long)bad);
                return 5;
            }
        }
        printf("%s: bit-exact\n", what);
        return 0;
    };
    for (int i = 0; i < 3; ++i) {
        want[i].resize(elems[i]);
        orc_convert_to_bf16(sp[i], dt[i], elems[i], want[i].data());
    }
    int rc = same("materialize");
    if (rc) return rc;

    // two adapters on slots 0 and 1, ranks that need padding
    Adapter ad[2];
    const int32_t ranks[2][2] = {{5, 16}, {24, 3}};
    for (int a = 0; a < 2; ++a)
        for (int k = 0; k < 2; ++k) {
            const int64_t out = slots[k].rows, in = slots[k].cols;
            const int32_t r = ranks[a][k];
            ad[a].r[k] = r;
            ad[a].alpha[k] = 2.0f * (float)r;
            ad[a].A[k].resize((size_t)r * in);
            ad[a].B[k].resize((size_t)out * r);
            for (float& v : ad[a].A[k]) v = uniform(0.05f);
            for (float& v : ad[a].B[k]) v = uniform(0.05f);
            ad[a].Ab[k].resize(ad[a].A[k].size());
            ad[a].Bb[k].resize(ad[a].B[k].size());
            orc_convert_to_bf16(ad[a].A[k].data(), TIDAL_F32, (int64_t)ad[a].A[k].size(), ad[a].Ab[k].data());
            orc_convert_to_bf16(ad[a].B[k].data(), TIDAL_F32, (int64_t)ad[a].B[k].size(), ad[a].Bb[k].data());
        }
    auto targets = [&](int a, tidal_lora_target* tg) {
        for (int k = 0; k < 2; ++k) tg[k] = tidal_lora_target{k, ad[a].r[k], ad[a].alpha[k], TIDAL_F32, ad[a].A[k].data(), ad[a].B[k].data()};
    };
    tidal_lora_target tg[2];
    targets(0, tg);
    CHECK_TIDAL(tidal_lora_attach(t, tg, 2, comp_s));
    CHECK_TIDAL(tidal_template_sync(t));
    for (int k = 0; k < 2; ++k)
        orc_lora_merge_bf16(want[k].data(), slots[k].rows, slots[k].cols, ad[0].Ab[k].data(), ad[0].Bb[k].data(), ad[0].r[k], ad[0].alpha[k], +1, 1);
    rc = same("attach");
    if (rc) return rc;

    targets(1, tg);
    CHECK_TIDAL(tidal_lora_swap(t, tg, 2, comp_s));
    CHECK_TIDAL(tidal_template_sync(t));
    for (int k = 0; k < 2; ++k)
        orc_lora_swap_bf16(want[k].data(), slots[k].rows, slots[k].cols, ad[0].Ab[k].data(), ad[0].Bb[k].data(), ad[0].r[k], ad[0].alpha[k],
                           ad[1].Ab[k].data(), ad[1].Bb[k].data(), ad[1].r[k], ad[1].alpha[k]);
    rc = same("swap");
    if (rc) return rc;

    CHECK_TIDAL(tidal_lora_detach(t, comp_s));
    CHECK_TIDAL(tidal_template_sync(t));
    for (int k = 0; k < 2; ++k)
        orc_lora_merge_bf16(want[k].data(), slots[k].rows, slots[k].cols, ad[1].Ab[k].data(), ad[1].Bb[k].data(), ad[1].r[k], ad[1].alpha[k], -1, 1);
    rc = same("detach");
    if (rc) return rc;

    // an error is a status and a message, nothing else: W untouched, no abort
    tg[0].slot = 17;
    if (tidal_lora_attach(t, tg, 2, comp_s) != TIDAL_E_INVAL || !strstr(tidal_last_error(), "slot")) {
        fprintf(stderr, "bad slot not rejected: %s\n", tidal_last_error());
        return 6;
    }
    if (tidal_lora_detach(t, comp_s) != TIDAL_E_STATE) { fprintf(stderr, "detach with nothing attached\n"); return 6; }
    rc = same("after rejected calls");
    if (rc) return rc;

    tidal_stats st;
    CHECK_TIDAL(tidal_get_stats(t, &st));
    if (st.h2d_bytes == 0 || st.lora_launches == 0) { fprintf(stderr, "stats empty\n"); return 7; }
    CHECK_TIDAL(tidal_template_destroy(t));
    CHECK_HIP(hipStreamDestroy(copy_s));
    CHECK_HIP(hipStreamDestroy(comp_s));
    CHECK_HIP(hipHostFree(s0));
    CHECK_HIP(hipHostFree(s1));
    CHECK_HIP(hipFree(arena));
    printf("abi gpu check ok\n");
    return 0;
}
