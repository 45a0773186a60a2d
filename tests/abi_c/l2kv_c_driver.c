/*
 * The hot path driven from plain C: device memory from hipMalloc, the four calls
 * of the library (norms, selection, compaction, decode attention, the latter also
 * through the entry point that needs no workspace), results written to a file.
 * No Python, no tensor library: what a C caller of libl2kv.so does.
 *
 *   l2kv_c_driver <out.bin> <n_seq> <kv_heads> <group> <tokens> <keep_ratio>
 *
 * Inputs (bf16, head size 128) come from a counter-based integer mix of the
 * element index, so the test that checks the output file can rebuild the same
 * bits; the mix holds none of the method's arithmetic.
 * Output file: int64 header {n_heads, T, k, Hq, D}, then norms [n_heads][T] f32,
 * kept_idx [n_heads][k] i32, Kc, Vc [n_heads][k][D] bf16 bits, O [B][Hq][D] f32
 * from l2kv_decode_attn and the same from l2kv_decode_attn_static.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "l2kv.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_L2KV(x) do { l2kv_status s_ = (x); if (s_ != L2KV_OK) { \
    fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, l2kv_status_string(s_)); return 3; } } while (0)

/* value in [-1, 1) with 14 random bits, exact in fp32 */
static float unit_value(uint32_t i, uint32_t salt) {
    uint32_t x = i * 2654435761u + salt;
    x ^= x >> 15; x *= 0x2C1B3C6Du; x ^= x >> 12; x *= 0x297A2D39u; x ^= x >> 15;
    return (float)((x >> 9) & 0x3FFFu) * (1.0f / 8192.0f) - 1.0f;
}
static uint16_t bf16_bits(float f) {            /* truncation: the test rebuilds exactly this */
    uint32_t u; memcpy(&u, &f, 4); return (uint16_t)(u >> 16);
}

int main(int argc, char** argv) {
    if (argc != 7) { fprintf(stderr, "usage: %s out.bin n_seq kv_heads group tokens keep_ratio\n", argv[0]); return 1; }
    const char* path = argv[1];
    const int32_t B = atoi(argv[2]), Hkv = atoi(argv[3]), G = atoi(argv[4]), D = 128;
    const int64_t T = atol(argv[5]);
    const double r = atof(argv[6]);
    const int32_t Hq = Hkv * G;
    const int64_t n_heads = (int64_t)B * Hkv, k = l2kv_keep_count(T, r);
    if (k <= 0) { fprintf(stderr, "bad shape\n"); return 1; }
    const size_t n_kv = (size_t)n_heads * T * D, n_q = (size_t)B * Hq * D, n_c = (size_t)n_heads * k * D;

    uint16_t* hK = malloc(n_kv * 2); uint16_t* hV = malloc(n_kv * 2); uint16_t* hQ = malloc(n_q * 2);
    for (size_t i = 0; i < n_kv; ++i) {
        const uint32_t row = (uint32_t)(i / D);
        const float scale = 0.25f + (float)((row * 37u) % 64u) * (1.0f / 32.0f);   /* row norms differ */
        hK[i] = bf16_bits(unit_value((uint32_t)i, 0x11u) * scale);
        hV[i] = bf16_bits(unit_value((uint32_t)i, 0x22u));
    }
    for (size_t i = 0; i < n_q; ++i) hQ[i] = bf16_bits(unit_value((uint32_t)i, 0x33u) * 4.0f);

    void *dK, *dV, *dQ, *dKc, *dVc, *dSel, *dDec;
    float *dN, *dO, *dO2; int32_t* dIdx;
    const size_t sel_bytes = l2kv_select_workspace_bytes(n_heads, T);
    const size_t dec_bytes = l2kv_decode_workspace_bytes(B, Hq, k, D);
    CHECK_HIP(hipMalloc(&dK, n_kv * 2)); CHECK_HIP(hipMalloc(&dV, n_kv * 2)); CHECK_HIP(hipMalloc(&dQ, n_q * 2));
    CHECK_HIP(hipMalloc(&dKc, n_c * 2)); CHECK_HIP(hipMalloc(&dVc, n_c * 2));
    CHECK_HIP(hipMalloc((void**)&dN, (size_t)n_heads * T * 4)); CHECK_HIP(hipMalloc((void**)&dIdx, (size_t)n_heads * k * 4));
    CHECK_HIP(hipMalloc((void**)&dO, n_q * 4)); CHECK_HIP(hipMalloc((void**)&dO2, n_q * 4));
    CHECK_HIP(hipMalloc(&dSel, sel_bytes)); CHECK_HIP(hipMalloc(&dDec, dec_bytes));
    CHECK_HIP(hipMemcpy(dK, hK, n_kv * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dV, hV, n_kv * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dQ, hQ, n_q * 2, hipMemcpyHostToDevice));

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_L2KV(l2kv_decode_workspace_init(dDec, dec_bytes, stream));
    CHECK_L2KV(l2kv_norms(dK, L2KV_BF16, n_heads, T, D, T * D, dN, stream));
    CHECK_L2KV(l2kv_select(dN, n_heads, T, r, dIdx, NULL, dSel, sel_bytes, stream));
    CHECK_L2KV(l2kv_compact(dK, dV, L2KV_BF16, dIdx, n_heads, T, k, D, T * D, dKc, dVc, stream));
    CHECK_L2KV(l2kv_decode_attn(dQ, dKc, dVc, L2KV_BF16, B, Hq, Hkv, k, D, k * D, 0.0f, dO, dDec, dec_bytes, stream));
    CHECK_L2KV(l2kv_decode_attn_static(dQ, dKc, dVc, L2KV_BF16, B, Hq, Hkv, k, D, k * D, 0.0f, dO2, stream));
    CHECK_HIP(hipStreamSynchronize(stream));

    float* hN = malloc((size_t)n_heads * T * 4); int32_t* hIdx = malloc((size_t)n_heads * k * 4);
    uint16_t* hKc = malloc(n_c * 2); uint16_t* hVc = malloc(n_c * 2);
    float* hO = malloc(n_q * 4); float* hO2 = malloc(n_q * 4);
    CHECK_HIP(hipMemcpy(hN, dN, (size_t)n_heads * T * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hIdx, dIdx, (size_t)n_heads * k * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hKc, dKc, n_c * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hVc, dVc, n_c * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hO, dO, n_q * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hO2, dO2, n_q * 4, hipMemcpyDeviceToHost));

    FILE* f = fopen(path, "wb");
    if (!f) { perror(path); return 4; }
    const int64_t header[5] = {n_heads, T, k, Hq, D};
    fwrite(header, 8, 5, f);
    fwrite(hN, 4, (size_t)n_heads * T, f); fwrite(hIdx, 4, (size_t)n_heads * k, f);
    fwrite(hKc, 2, n_c, f); fwrite(hVc, 2, n_c, f); fwrite(hO, 4, n_q, f); fwrite(hO2, 4, n_q, f);
    fclose(f);
    printf("l2kv_c_driver: %lld heads x %lld tokens, kept %lld, library version %d\n",
           (long long)n_heads, (long long)T, (long long)k, (int)l2kv_version());
    return 0;
}
