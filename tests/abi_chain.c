/* The whole path through the C ABI from a plain C99 program: no Python, no PyTorch.  Device memory
 * comes from the HIP runtime's C API, every call runs on the default stream (stream = NULL).
 * Inputs come from a 32-bit linear congruential generator that the GPU test repeats in numpy, so
 * that the outputs this program writes can be checked against the CPU oracle.
 *
 *   abi_chain <output file>
 * writes, as raw little-endian arrays: encode output, frame vectors, scores, idx, n_sel, QA output.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "rekv.h"

enum { HQ = 4, HKV = 2, D = 64, NF = 5, FRAMES = 12, WINDOW_FRAMES = 3, NQ_TOKENS = 6, TOPK = 3 };

static uint32_t lcg_state = 12345u;
static float lcg_next(void) { /* uniform in [-0.5, 0.5), 24 bits */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)(lcg_state >> 8) * (1.0f / 16777216.0f) - 0.5f;
}
static float* host_array(size_t n, float scale) {
    float* p = (float*)malloc(n * sizeof(float));
    size_t i;
    if (!p) { fprintf(stderr, "out of host memory\n"); exit(2); }
    for (i = 0; i < n; ++i) p[i] = lcg_next() * scale;
    return p;
}
#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 3; } } while (0)
#define REKV_CALL(x) do { rekv_status s_ = (x); if (s_ != REKV_OK) { fprintf(stderr, "%s: status %d: %s\n", #x, (int)s_, rekv_last_error(ctx)); return 4; } } while (0)

static void* to_device(const void* src, size_t bytes) {
    void* d = NULL;
    if (hipMalloc(&d, bytes) != hipSuccess) return NULL;
    if (src && hipMemcpy(d, src, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return d;
}

int main(int argc, char** argv) {
    const size_t tokens = (size_t)FRAMES * NF;
    const size_t n_q = tokens * HQ * D, n_kv = tokens * HKV * D, d_prime = (size_t)HKV * D;
    const size_t n_qq = (size_t)NQ_TOKENS * HQ * D, n_qkv = (size_t)NQ_TOKENS * HKV * D;
    const size_t n_ret = (size_t)TOPK * NF * HKV * D;
    rekv_shape shape = {HQ, HKV, D, NF, REKV_F32, 0.0f};
    rekv_ctx* ctx = NULL;
    float *q, *k, *v, *qq, *qk, *qv;
    void *dq, *dk, *dv, *dqq, *dqk, *dqv, *d_out, *d_fk, *d_scores, *d_idx, *d_nsel, *d_gk, *d_gv, *d_qa;
    float *out, *fk, *scores, *qa;
    int32_t idx[TOPK], n_sel[1];
    FILE* f;
    if (argc != 2) { fprintf(stderr, "usage: %s <output file>\n", argv[0]); return 1; }

    /* the order of these draws is part of the test's contract */
    q = host_array(n_q, 2.0f); k = host_array(n_kv, 2.0f); v = host_array(n_kv, 2.0f);
    qq = host_array(n_qq, 2.0f); qk = host_array(n_qkv, 2.0f); qv = host_array(n_qkv, 2.0f);

    if (rekv_create(&shape, &ctx) != REKV_OK) { fprintf(stderr, "rekv_create: %s\n", rekv_last_error(NULL)); return 4; }
    dq = to_device(q, n_q * 4); dk = to_device(k, n_kv * 4); dv = to_device(v, n_kv * 4);
    dqq = to_device(qq, n_qq * 4); dqk = to_device(qk, n_qkv * 4); dqv = to_device(qv, n_qkv * 4);
    d_out = to_device(NULL, n_q * 4); d_fk = to_device(NULL, FRAMES * d_prime * 4);
    d_scores = to_device(NULL, FRAMES * 4); d_idx = to_device(NULL, TOPK * 4); d_nsel = to_device(NULL, 4);
    d_gk = to_device(NULL, n_ret * 4); d_gv = to_device(NULL, n_ret * 4); d_qa = to_device(NULL, n_qq * 4);
    if (!dq || !dk || !dv || !dqq || !dqk || !dqv || !d_out || !d_fk || !d_scores || !d_idx || !d_nsel || !d_gk || !d_gv || !d_qa) {
        fprintf(stderr, "device allocation or upload failed\n");
        return 3;
    }

    /* Eq. 1 for all chunks (one frame each), frame vectors, Eq. 2 + top-k, reload, Eq. 3 */
    REKV_CALL(rekv_encode_chunk(ctx, dq, dk, dv, 0, NF, FRAMES, WINDOW_FRAMES * NF, d_out, NULL));
    REKV_CALL(rekv_frame_keys(ctx, dk, FRAMES, (float*)d_fk, NULL));
    REKV_CALL(rekv_retrieve_topk(ctx, (const float*)d_fk, 0, FRAMES, dqq, 1, NQ_TOKENS, TOPK, (int32_t*)d_idx,
                                 (int32_t*)d_nsel, (float*)d_scores, NULL));
    REKV_CALL(rekv_gather_kv(ctx, dk, dv, 0, FRAMES, (const int32_t*)d_idx, 1, TOPK, d_gk, d_gv, NULL));
    REKV_CALL(rekv_qa_attention(ctx, dqq, d_gk, d_gv, TOPK * NF, (const int32_t*)d_nsel, dqk, dqv, 1, NQ_TOKENS, d_qa, NULL));
    /* an argument error is reported, not executed */
    if (rekv_frame_keys(ctx, NULL, FRAMES, (float*)d_fk, NULL) != REKV_ERR_INVALID_ARG) { fprintf(stderr, "null pointer accepted\n"); return 5; }
    HIP_OK(hipDeviceSynchronize());

    out = (float*)malloc(n_q * 4); fk = (float*)malloc(FRAMES * d_prime * 4); scores = (float*)malloc(FRAMES * 4);
    qa = (float*)malloc(n_qq * 4);
    if (!out || !fk || !scores || !qa) return 2;
    HIP_OK(hipMemcpy(out, d_out, n_q * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(fk, d_fk, FRAMES * d_prime * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(scores, d_scores, FRAMES * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(idx, d_idx, TOPK * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(n_sel, d_nsel, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(qa, d_qa, n_qq * 4, hipMemcpyDeviceToHost));
    rekv_destroy(ctx);

    f = fopen(argv[1], "wb");
    if (!f) { perror(argv[1]); return 6; }
    fwrite(out, 4, n_q, f); fwrite(fk, 4, FRAMES * d_prime, f); fwrite(scores, 4, FRAMES, f);
    fwrite(idx, 4, TOPK, f); fwrite(n_sel, 4, 1, f); fwrite(qa, 4, n_qq, f);
    if (fclose(f) != 0) return 6;
    printf("selected frames %d %d %d (n_sel %d)\n", (int)idx[0], (int)idx[1], (int)idx[2], (int)n_sel[0]);
    return 0;
}
