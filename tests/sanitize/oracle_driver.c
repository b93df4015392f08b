/* Runs every oracle routine on small inputs (ragged sizes, zero sizes, special values) in a
 * build with AddressSanitizer and UndefinedBehaviorSanitizer; any report ends the process with
 * a non-zero status.  Values are not checked here (the pins do that): this is about memory and
 * undefined behaviour. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint32_t orc_f16_bits_to_f32_bits(uint16_t h);
uint16_t orc_f32_bits_to_bf16_bits(uint32_t u);
void orc_convert_to_bf16(const void* src, int dtype, int64_t n, uint16_t* dst);
int64_t orc_layout(const int64_t* rows, const int64_t* cols, int32_t n, int64_t* off);
void orc_materialize_slot(uint8_t* arena, int64_t off, const void* src, int dtype, int64_t rows, int64_t cols);
void orc_lora_merge_bf16(uint16_t* W, int64_t out, int64_t in, const uint16_t* A, const uint16_t* B, int32_t r, float alpha, int sign, int sc);
void orc_lora_merge_f32(float* W, int64_t out, int64_t in, const uint16_t* A, const uint16_t* B, int32_t r, float alpha, int sign, int sc);
void orc_lora_swap_bf16(uint16_t* W, int64_t out, int64_t in, const uint16_t* A0, const uint16_t* B0, int32_t r0, float a0,
                        const uint16_t* A1, const uint16_t* B1, int32_t r1, float a1);
uint64_t orc_prefetch_bytes(uint64_t model, double ttft, double link);
int32_t orc_resident_prefix(const int64_t* rows, const int64_t* cols, int32_t n, uint64_t prefetch);
uint64_t orc_slot_checksum(const uint16_t* bits, int64_t n, int32_t passes);
void orc_materialize_merge_slot(const void* src, int dtype, int64_t out, int64_t in, const uint16_t* A, const uint16_t* B, int32_t r,
                                float alpha, uint16_t* slot);
void orc_lora_apply(const uint16_t* X, uint16_t* Y, int64_t in, int64_t out, const uint16_t* A, const uint16_t* B, int32_t r,
                    float alpha, int64_t t0, int64_t t1);

static uint32_t lcg(uint32_t* s) { *s = *s * 1664525u + 1013904223u; return *s; }

int main(void) {
    uint32_t seed = 12345;
    /* conversions: every exponent with a few mantissas, specials */
    for (uint32_t h = 0; h < 65536; h += 7) (void)orc_f16_bits_to_f32_bits((uint16_t)h);
    for (uint32_t i = 0; i < 100000; ++i) (void)orc_f32_bits_to_bf16_bits(lcg(&seed));
    const uint32_t special[] = {0u, 0x80000000u, 0x7F800000u, 0xFF800000u, 0x7FC00000u, 0x7F7FFFFFu, 0x00000001u, 0x807FFFFFu, 0x3F808000u};
    for (size_t i = 0; i < sizeof special / sizeof special[0]; ++i) (void)orc_f32_bits_to_bf16_bits(special[i]);
    for (int dtype = 0; dtype < 3; ++dtype) {
        for (int64_t n = 0; n < 70; n += 23) {
            const size_t isz = dtype == 0 ? 4 : 2;
            uint8_t* src = (uint8_t*)malloc(n * isz + 1);
            uint16_t* dst = (uint16_t*)malloc(n * 2 + 1);
            for (int64_t i = 0; i < (int64_t)(n * isz); ++i) src[i] = (uint8_t)lcg(&seed);
            orc_convert_to_bf16(src, dtype, n, dst);
            free(src);
            free(dst);
        }
    }
    /* layout + placement */
    const int64_t rows[] = {3, 1, 0, 17}, cols[] = {5, 129, 4, 33};
    int64_t off[5];
    const int64_t total = orc_layout(rows, cols, 4, off);
    if (total != off[4]) return 2;
    uint8_t* arena = (uint8_t*)calloc((size_t)total + 1, 1);
    for (int i = 0; i < 4; ++i) {
        const int64_t n = rows[i] * cols[i];
        float* src = (float*)malloc((size_t)n * 4 + 4);
        for (int64_t k = 0; k < n; ++k) src[k] = (float)(int32_t)lcg(&seed) * 1e-9f;
        orc_materialize_slot(arena, off[i], src, 0, rows[i], cols[i]);
        free(src);
    }
    (void)orc_resident_prefix(rows, cols, 4, 100);
    (void)orc_resident_prefix(rows, cols, 4, 1u << 30);
    (void)orc_prefetch_bytes(1000, 1.0, 10.0);
    (void)orc_prefetch_bytes(0, 0.0, 0.0);
    (void)orc_slot_checksum((const uint16_t*)(arena + off[3]), rows[3] * cols[3], 3);
    free(arena);
    /* merges: ragged shapes, ranks 0..64, both storage types, swap, fused materialise, apply */
    const int shapes[][3] = {{1, 1, 1}, {5, 7, 3}, {33, 65, 16}, {40, 24, 64}, {9, 130, 0}};
    for (size_t s = 0; s < sizeof shapes / sizeof shapes[0]; ++s) {
        const int out = shapes[s][0], in = shapes[s][1], r = shapes[s][2], r1 = (r * 2) % 65;
        uint16_t* W = (uint16_t*)malloc((size_t)out * in * 2);
        float* Wf = (float*)malloc((size_t)out * in * 4);
        uint16_t* A = (uint16_t*)malloc((size_t)(r + 1) * in * 2);
        uint16_t* B = (uint16_t*)malloc((size_t)out * (r + 1) * 2);
        uint16_t* A1 = (uint16_t*)malloc((size_t)(r1 + 1) * in * 2);
        uint16_t* B1 = (uint16_t*)malloc((size_t)out * (r1 + 1) * 2);
        for (int i = 0; i < out * in; ++i) { W[i] = (uint16_t)(0x3C00 + (lcg(&seed) & 0x1FF)); Wf[i] = 0.01f * (float)(i % 13); }
        for (int i = 0; i < (r + 1) * in; ++i) A[i] = (uint16_t)(0x3B00 + (lcg(&seed) & 0xFF));
        for (int i = 0; i < out * (r + 1); ++i) B[i] = (uint16_t)(0xBB00 + (lcg(&seed) & 0xFF));
        for (int i = 0; i < (r1 + 1) * in; ++i) A1[i] = (uint16_t)(0x3B00 + (lcg(&seed) & 0xFF));
        for (int i = 0; i < out * (r1 + 1); ++i) B1[i] = (uint16_t)(0x3B00 + (lcg(&seed) & 0xFF));
        orc_lora_merge_bf16(W, out, in, A, B, r, 2.0f * (float)r, +1, 1);
        orc_lora_merge_bf16(W, out, in, A, B, r, 2.0f * (float)r, -1, 0);
        orc_lora_merge_f32(Wf, out, in, A, B, r, 0.0f, +1, 0);
        orc_lora_merge_f32(Wf, out, in, A, B, r, 3.0f, +1, 1);
        orc_lora_swap_bf16(W, out, in, A, B, r, 1.0f, A1, B1, r1, 2.0f);
        uint16_t* slot = (uint16_t*)malloc((size_t)out * in * 2);
        orc_materialize_merge_slot(Wf, 0, out, in, A, B, r, 4.0f, slot);
        orc_materialize_merge_slot(W, 2, out, in, A, B, r, 4.0f, slot);
        free(slot);
        const int T = 6;
        uint16_t* X = (uint16_t*)malloc((size_t)T * in * 2);
        uint16_t* Y = (uint16_t*)malloc((size_t)T * out * 2);
        for (int i = 0; i < T * in; ++i) X[i] = (uint16_t)(0x3F00 + (lcg(&seed) & 0xFF));
        for (int i = 0; i < T * out; ++i) Y[i] = (uint16_t)(0xBF00 + (lcg(&seed) & 0xFF));
        orc_lora_apply(X, Y, in, out, A, B, r, 2.0f, 1, T);
        orc_lora_apply(X, Y, in, out, A, B, r, 2.0f, 3, 3);
        free(X); free(Y); free(W); free(Wf); free(A); free(B); free(A1); free(B1);
    }
    puts("oracle sanitizer run ok");
    return 0;
}
