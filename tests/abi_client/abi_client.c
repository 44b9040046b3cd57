/*
 * A plain C99 caller of the C ABI declared in include/specsteer.h: no C++, no Python, no tensor
 * library -- device memory straight from the HIP runtime.  Test infrastructure: the GPU test
 * writes one block of inputs to a file, runs this program and compares what it wrote back with
 * the oracle.
 *
 * File format (little endian): int32 B, k_max, V, dtype, has_len; float lambda, beta, T; then
 * G, S_ctx, S_noctx ([B, k_max+1, V] of the dtype), draft [B, k_max] int32, draft_len [B] int32
 * (if has_len), uniforms [B, k_max+1] fp32.  Output: accepted_len [B] int32, next_token [B] int32,
 * next_token_logprob [B] fp32.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "specsteer.h"

#define CHECK_HIP(x)                                                                  \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                   \
            return 2;                                                                 \
        }                                                                             \
    } while (0)

static void *read_to_device(FILE *f, size_t bytes) {
    void *host = malloc(bytes ? bytes : 1), *dev = NULL;
    if (!host || fread(host, 1, bytes, f) != bytes) return NULL;
    if (hipMalloc(&dev, bytes ? bytes : 1) != hipSuccess) return NULL;
    if (hipMemcpy(dev, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    free(host);
    return dev;
}

int main(int argc, char **argv) {
    if (argc != 3) {
        fprintf(stderr, "usage: %s inputs.bin outputs.bin\n", argv[0]);
        return 1;
    }
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 1;
    int32_t hdr[5];
    float par[3];
    if (fread(hdr, sizeof(int32_t), 5, f) != 5 || fread(par, sizeof(float), 3, f) != 3) return 1;
    const int B = hdr[0], K = hdr[1], V = hdr[2];
    ss_params p;
    p.batch = B; p.k_max = K; p.vocab = V; p.dtype = hdr[3];
    p.stride_b = 0; p.stride_t = 0;
    p.lambda = par[0]; p.beta = par[1]; p.temperature = par[2];
    p.flags = 0;
    const size_t esz = hdr[3] == SS_BF16 ? 2 : 4;
    const size_t logits = (size_t)B * (K + 1) * V * esz;
    void *G = read_to_device(f, logits), *Sp = read_to_device(f, logits), *Sm = read_to_device(f, logits);
    int32_t *draft = (int32_t *)read_to_device(f, (size_t)B * K * 4);
    int32_t *len = hdr[4] ? (int32_t *)read_to_device(f, (size_t)B * 4) : NULL;
    float *u = (float *)read_to_device(f, (size_t)B * (K + 1) * 4);
    fclose(f);
    if (!G || !Sp || !Sm || !draft || (hdr[4] && !len) || !u) {
        fprintf(stderr, "could not stage the inputs\n");
        return 2;
    }

    const size_t ws_bytes = specsteer_workspace_bytes(&p);
    void *ws = NULL;
    int32_t *acc = NULL, *tok = NULL;
    float *lp = NULL;
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_HIP(hipMalloc((void **)&acc, (size_t)B * 4));
    CHECK_HIP(hipMalloc((void **)&tok, (size_t)B * 4));
    CHECK_HIP(hipMalloc((void **)&lp, (size_t)B * 4));

    /* an argument error must come back from the host with nothing enqueued */
    if (specsteer_verify_block(G, Sp, Sm, draft, len, u, &p, acc, tok, lp, NULL, NULL, ws, ws_bytes - 1, NULL) !=
        SS_ERR_WORKSPACE) {
        fprintf(stderr, "a short workspace was not refused\n");
        return 3;
    }
    const ss_status st = specsteer_verify_block(G, Sp, Sm, draft, len, u, &p, acc, tok, lp, NULL, NULL, ws, ws_bytes, NULL);
    if (st != SS_OK) {
        fprintf(stderr, "specsteer_verify_block: %s\n", specsteer_status_string(st));
        return 3;
    }
    CHECK_HIP(hipDeviceSynchronize());

    int32_t *h_acc = (int32_t *)malloc((size_t)B * 4), *h_tok = (int32_t *)malloc((size_t)B * 4);
    float *h_lp = (float *)malloc((size_t)B * 4);
    CHECK_HIP(hipMemcpy(h_acc, acc, (size_t)B * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(h_tok, tok, (size_t)B * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(h_lp, lp, (size_t)B * 4, hipMemcpyDeviceToHost));
    FILE *o = fopen(argv[2], "wb");
    if (!o) return 1;
    fwrite(h_acc, 4, (size_t)B, o);
    fwrite(h_tok, 4, (size_t)B, o);
    fwrite(h_lp, 4, (size_t)B, o);
    fclose(o);
    printf("specsteer %d: %d sequences verified from C\n", specsteer_version(), B);
    return 0;
}
