// Host-only paths of libtidal under AddressSanitizer and UndefinedBehaviorSanitizer: configuration,
// arena layout, the copy plan (seeded fuzz over tensor lists and chunk sizes), argument validation of
// every entry point, the LoRA launch plan over many shapes and rank pairs, the partial-residency
// arithmetic.  No GPU is needed: calls that would reach one must come back with an error code.
// Invariants are checked with plain ifs; any sanitizer report ends the process with a non-zero status.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "tidal.h"

static uint32_t g_seed = 2024;
static uint32_t rnd() { g_seed = g_seed * 1664525u + 1013904223u; return g_seed >> 8; }
#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "host driver: %s failed at line %d: %s\n", #c, __LINE__, tidal_last_error()); return 1; } } while (0)

static int fuzz_copy_plan() {
    for (int it = 0; it < 60; ++it) {
        const int n = 1 + rnd() % 40;
        std::vector<tidal_slot_desc> slots(n);
        for (auto& s : slots) {
            const int kind = rnd() % 4;
            s.rows = kind == 0 ? 1 : 1 + rnd() % (kind == 3 ? 300 : 40);
            s.cols = kind == 0 ? 1 + rnd() % 5000 : 1 + rnd() % (kind == 3 ? 3000 : 200);
            if (rnd() % 17 == 0) s.rows = 0;
        }
        tidal_config cfg;
        tidal_config_default(&cfg);
        cfg.chunk_bytes = (size_t)(16 + rnd() % 128) << 12;          // a multiple of 4 KiB, as the library rounds it
        cfg.coalesce_bytes = (size_t)(1 + rnd() % 64) << 10;
        cfg.max_adapter_bytes = 0;
        const size_t need = tidal_template_required_bytes(slots.data(), n, &cfg);
        REQUIRE(need > 0);
        tidal_template* t = nullptr;
        REQUIRE(tidal_template_create(slots.data(), n, (void*)(uintptr_t)0x700000000000ull, need, &cfg, &t) == TIDAL_OK);
        static char host[1];
        std::vector<tidal_src> srcs;
        for (int i = 0; i < n; ++i)
            if (rnd() % 5) srcs.push_back(tidal_src{i, (int32_t)(rnd() % 3), host});
        for (int pinned = 0; pinned < 2; ++pinned) {
            const int32_t cnt = tidal_materialize_plan(t, srcs.data(), (int32_t)srcs.size(), pinned, nullptr, 0);
            REQUIRE(cnt >= 0);
            std::vector<tidal_copy_piece> pieces((size_t)cnt + 1);
            REQUIRE(tidal_materialize_plan(t, srcs.data(), (int32_t)srcs.size(), pinned, pieces.data(), cnt) == cnt);
            // every source element is covered exactly once, in order, and no chunk overflows its buffer
            std::vector<int64_t> covered(n, 0);
            int32_t chunk = -1;
            int64_t fill = 0;
            for (int32_t k = 0; k < cnt; ++k) {
                const tidal_copy_piece& p = pieces[k];
                REQUIRE(p.slot >= 0 && p.slot < n && p.elems > 0);
                REQUIRE(p.elem_offset == covered[p.slot]);
                covered[p.slot] += p.elems;
                REQUIRE(p.chunk >= chunk);
                if (p.chunk != chunk) { chunk = p.chunk; fill = 0; }
                if (p.staging_offset >= 0) {
                    REQUIRE(p.staging_offset % 256 == 0 && p.staging_offset >= fill);
                    fill = p.staging_offset + p.src_bytes;
                    REQUIRE((size_t)fill <= cfg.chunk_bytes);
                }
            }
            for (const tidal_src& s : srcs) REQUIRE(covered[s.slot] == slots[s.slot].rows * slots[s.slot].cols);
        }
        // slots: aligned, in order, inside the arena
        size_t prev_end = 0;
        for (int i = 0; i < n; ++i) {
            void* p = nullptr;
            size_t bytes = 0;
            REQUIRE(tidal_template_slot_ptr(t, i, &p, &bytes) == TIDAL_OK);
            const size_t off = (size_t)((uintptr_t)p - 0x700000000000ull);
            REQUIRE(off % 256 == 0 && off >= prev_end && off + bytes <= need);
            prev_end = off + bytes;
        }
        int32_t ns = 0;
        size_t rb = 0;
        REQUIRE(tidal_template_resident_prefix(t, need / 3, &ns, &rb) == TIDAL_OK && ns >= 0 && ns <= n);
        REQUIRE(tidal_template_destroy(t) == TIDAL_OK);
    }
    return 0;
}

static int launch_plans() {
    tidal_slot_desc one = {64, 64};
    tidal_template* t = nullptr;
    REQUIRE(tidal_template_create(&one, 1, (void*)(uintptr_t)0x700000000000ull, (size_t)1 << 40, nullptr, &t) == TIDAL_OK);
    const int64_t dims[] = {1, 31, 32, 33, 255, 256, 257, 1000, 4096, 5120, 11008, 13824, 28672};
    const int ranks[] = {0, 1, 8, 16, 17, 32, 33, 64};
    const int counts[] = {1, 3, 33, 128, 129, 560};
    for (int64_t out : dims)
        for (int64_t in : dims)
            for (int r0 : ranks)
                for (int r1 : ranks)
                    for (int n : counts) {
                        if (r0 + r1 == 0) continue;
                        tidal_lora_launch info;
                        REQUIRE(tidal_lora_launch_info(t, out, in, n, r0, r1, 0, &info) == TIDAL_OK);
                        REQUIRE(info.launches >= 1 && (int64_t)info.launches * info.targets_per_launch >= n);
                        REQUIRE(info.targets_per_launch <= 128 && info.blocks_per_walk >= 1 && info.workgroups >= 1);
                        // the grid covers every 32-row block of every 256-column strip of every slot
                        const int64_t strips = (in + 255) / 256, rowblocks = (out + 31) / 32;
                        const bool lds = strncmp(info.kernel, "lora_mfma_lds", 13) == 0;
                        const int64_t per_wg = lds ? 4 * (int64_t)info.blocks_per_walk : (int64_t)info.blocks_per_walk;
                        const int64_t chunks = (rowblocks + per_wg - 1) / per_wg;
                        const int64_t wg = lds ? strips * chunks : (strips * chunks + 3) / 4;
                        REQUIRE(info.workgroups == wg * info.targets_per_launch);
                        if (r0 == 0) REQUIRE(tidal_lora_launch_info(t, out, in, n, 0, r1, 1, &info) == TIDAL_OK);
                    }
    tidal_lora_launch info;
    REQUIRE(tidal_lora_launch_info(t, 0, 5, 1, 0, 8, 0, &info) == TIDAL_E_INVAL);
    REQUIRE(tidal_lora_launch_info(t, 5, 5, 1, 65, 8, 0, &info) == TIDAL_E_INVAL);
    REQUIRE(tidal_lora_launch_info(t, 5, 5, 1, 8, 8, 1, &info) == TIDAL_E_INVAL);
    REQUIRE(tidal_template_destroy(t) == TIDAL_OK);
    return 0;
}

static int validation() {
    tidal_slot_desc slots[3] = {{8, 16}, {64, 64}, {0, 7}};
    tidal_config cfg;
    tidal_config_default(&cfg);
    cfg.max_adapter_bytes = 1 << 20;
    tidal_template* t = nullptr;
    REQUIRE(tidal_template_create(slots, 3, nullptr, 1 << 20, &cfg, &t) == TIDAL_E_INVAL);
    REQUIRE(tidal_template_create(slots, 3, (void*)(uintptr_t)0x700000000008ull, (size_t)1 << 40, &cfg, &t) == TIDAL_E_INVAL);
    REQUIRE(tidal_template_create(slots, 3, (void*)(uintptr_t)0x700000000000ull, 16, &cfg, &t) == TIDAL_E_NOMEM);
    REQUIRE(tidal_template_create(slots, 3, (void*)(uintptr_t)0x700000000000ull, (size_t)1 << 40, &cfg, &t) == TIDAL_OK);
    static float A[64 * 64], B[64 * 64];
    tidal_lora_target ok = {1, 4, 8.0f, TIDAL_F32, A, B};
    tidal_lora_target bad = ok;
    bad.slot = 7;
    REQUIRE(tidal_lora_attach(t, &bad, 1, nullptr) == TIDAL_E_INVAL);
    bad = ok; bad.r = 65;
    REQUIRE(tidal_lora_attach(t, &bad, 1, nullptr) == TIDAL_E_INVAL);
    bad = ok; bad.A = nullptr;
    REQUIRE(tidal_lora_attach(t, &bad, 1, nullptr) == TIDAL_E_INVAL);
    tidal_lora_target twice[2] = {ok, ok};
    REQUIRE(tidal_lora_attach(t, twice, 2, nullptr) == TIDAL_E_INVAL);
    REQUIRE(tidal_lora_attach(t, &ok, 1, nullptr) == TIDAL_E_STATE);          // slot never materialised
    REQUIRE(tidal_lora_swap(t, &ok, 1, nullptr) == TIDAL_E_STATE);
    REQUIRE(tidal_lora_detach(t, nullptr) == TIDAL_E_STATE);
    REQUIRE(tidal_adapter_required_bytes(t, &ok, 1) > 0);
    bad = ok; bad.r = 65;
    REQUIRE(tidal_adapter_required_bytes(t, &bad, 1) == 0);
    static char host[64 * 64 * 4];
    tidal_src src = {1, TIDAL_F32, host};
    tidal_src dup[2] = {src, src};
    REQUIRE(tidal_materialize(t, dup, 2, nullptr, nullptr) == TIDAL_E_INVAL);
    src.dtype = 9;
    REQUIRE(tidal_materialize(t, &src, 1, nullptr, nullptr) == TIDAL_E_INVAL);
    src.dtype = TIDAL_F32;
    REQUIRE(tidal_materialize(t, &src, 1, nullptr, nullptr) == TIDAL_E_HIP);   // valid, but there is no GPU here
    int32_t fslots[2] = {1, 0};
    REQUIRE(tidal_fork_required_bytes(t, fslots, 2) > 0);
    tidal_fork* f = nullptr;
    REQUIRE(tidal_fork_create(t, fslots, 2, (void*)(uintptr_t)0x710000000000ull, 1 << 20, &f) == TIDAL_OK);
    void* p = nullptr;
    REQUIRE(tidal_fork_slot_ptr(f, 1, &p, nullptr) == TIDAL_OK && tidal_fork_slot_ptr(f, 2, &p, nullptr) == TIDAL_E_INVAL);
    REQUIRE(tidal_fork_apply(f, nullptr, nullptr) == TIDAL_E_STATE);            // slots never materialised
    REQUIRE(tidal_fork_destroy(f) == TIDAL_OK);
    tidal_lora_segment seg = {0, 0, 4};
    REQUIRE(tidal_lora_apply(t, 1, nullptr, 0, &seg, 1, host, host, 4, host, 1 << 10, nullptr) == TIDAL_E_INVAL);   // adapter 0 of none
    REQUIRE(tidal_lora_apply_static(t, 1, nullptr, 0, &seg, 1, host, host, 1 << 20, nullptr) == TIDAL_E_INVAL);
    REQUIRE(tidal_template_slot_wait(t, 0, nullptr) == TIDAL_E_STATE);
    uint64_t sum = 0;
    REQUIRE(tidal_slot_checksum(t, 1, 1, nullptr, &sum) == TIDAL_E_STATE);
    REQUIRE(tidal_prefetch_bytes(1000, 1.0, 100.0) == 900 && tidal_prefetch_bytes(1000, 100.0, 100.0) == 0);
    tidal_stats st;
    REQUIRE(tidal_get_stats(t, &st) == TIDAL_OK && st.h2d_bytes == 0);
    REQUIRE(tidal_template_sync(t) == TIDAL_OK);
    REQUIRE(tidal_template_destroy(t) == TIDAL_OK);
    return 0;
}

// Groups of the adapter upload over stacks of mixed shapes, ranks and chunk sizes: every target in exactly one
// group, at most eight groups, and the planner's arithmetic under the sanitizers.
static int upload_plans() {
    static float fake[4];
    for (int round = 0; round < 60; ++round) {
        const int n = 2 + (int)(rnd() % 300);
        const int64_t dims[] = {1024, 4096, 5120, 8192, 13824, 28672};
        std::vector<tidal_slot_desc> slots((size_t)n);
        for (int i = 0; i < n; ++i) slots[(size_t)i] = {dims[rnd() % 6], dims[rnd() % 6]};
        tidal_config cfg;
        tidal_config_default(&cfg);
        cfg.chunk_bytes = (size_t)(1u << (24 + rnd() % 4));       // 16 to 128 MiB: the largest factor here is 7 MiB
        if (round % 7 == 3) cfg.flags |= TIDAL_FLAG_PIPELINED_UPLOAD;
        tidal_template* t = nullptr;
        REQUIRE(tidal_template_create(slots.data(), n, (void*)(uintptr_t)0x700000000000ull, (size_t)1 << 46, &cfg, &t) == TIDAL_OK);
        const int ranks[] = {0, 1, 8, 16, 32, 64};
        std::vector<tidal_lora_target> tg;
        for (int i = 0; i < n; ++i) {
            if (rnd() % 5 == 0) continue;                       // not every slot is a target
            const int r = ranks[rnd() % 6];
            tg.push_back(tidal_lora_target{i, r, r ? 2.0f * (float)r : 0.0f, (rnd() & 1) ? TIDAL_F16 : TIDAL_F32, r ? fake : nullptr, r ? fake : nullptr});
        }
        int32_t groups[16];
        const int32_t g = tidal_lora_upload_plan(t, tg.data(), (int32_t)tg.size(), round & 1, groups, 16);
        REQUIRE(g >= 1 && g <= 8);
        int64_t total = 0;
        for (int k = 0; k < g; ++k) { REQUIRE(groups[k] > 0 || tg.empty()); total += groups[k]; }
        REQUIRE(total == (int64_t)tg.size());
        REQUIRE(tidal_lora_upload_plan(t, tg.data(), (int32_t)tg.size(), 0, nullptr, 4) == TIDAL_E_INVAL);
        REQUIRE(tidal_template_destroy(t) == TIDAL_OK);
    }
    return 0;
}

int main() {
    if (fuzz_copy_plan()) return 1;
    if (launch_plans()) return 1;
    if (upload_plans()) return 1;
    if (validation()) return 1;
    puts("host sanitizer run ok");
    return 0;
}
