/* A plain C program that drives the library through include/pre3.h with nothing but the HIP
 * runtime for device memory: compile, bind, fill_mask, apply_mask, advance, advance_fill_mask,
 * apply_mask_argmax, jump_forward.  The inputs and the expected outputs (computed by the CPU
 * oracle) come from a fixture file written by tests/test_gpu_c_abi.py:
 *
 *   int32 header[8] = {n_grammar_bytes, n_vocab_bytes, n_tokens, eos_id, batch, cap, max_jump, 0}
 *   grammar text | vocab bytes | int64 offsets[n_tokens+1]
 *   int32 states[B] | data[B*cap] | len[B]                    (before the step)
 *   uint32 mask[B*W] | uint16 logits[B*V] | uint16 masked[B*V] | int32 argmax[B]
 *   int32 tokens[B] | err[B] | states1[B] | len1[B] | data1[B*cap] | uint32 mask1[B*W]
 *   uint8 jump_bytes[B*max_jump] | int32 jump_len[B] | int32 states2[B] | len2[B]
 *
 * Prints "C ABI OK" and returns 0 when everything matches bit for bit. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/pre3.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_PRE3(x) do { int r_ = (x); if (r_ != PRE3_OK) { fprintf(stderr, "%s: status %d: %s\n", #x, r_, pre3_last_error(h)); return 3; } } while (0)

static unsigned char *take(unsigned char **p, size_t n) { unsigned char *q = *p; *p += n; return q; }

static int same(const char *what, const void *got, const void *want, size_t n) {
    if (memcmp(got, want, n) == 0) return 1;
    fprintf(stderr, "MISMATCH in %s\n", what);
    return 0;
}

int main(int argc, char **argv) {
    if (argc < 2) { fprintf(stderr, "usage: check FIXTURE\n"); return 1; }
    FILE *f = fopen(argv[1], "rb");
    if (!f) { perror("fixture"); return 1; }
    fseek(f, 0, SEEK_END);
    long size = ftell(f);
    fseek(f, 0, SEEK_SET);
    unsigned char *buf = (unsigned char *)malloc((size_t)size), *p = buf;
    if (fread(buf, 1, (size_t)size, f) != (size_t)size) { fprintf(stderr, "short read\n"); return 1; }
    fclose(f);

    int32_t *hd = (int32_t *)take(&p, 8 * 4);
    const int n_gram = hd[0], n_vb = hd[1], V = hd[2], eos = hd[3], B = hd[4], cap = hd[5], max_jump = hd[6];
    const int W = (V + 31) / 32;
    char *grammar = (char *)malloc((size_t)n_gram + 1);
    memcpy(grammar, take(&p, (size_t)n_gram), (size_t)n_gram);
    grammar[n_gram] = 0;
    const uint8_t *vbytes = take(&p, (size_t)n_vb);
    int64_t *offsets = (int64_t *)malloc(sizeof(int64_t) * ((size_t)V + 1));
    memcpy(offsets, take(&p, 8 * ((size_t)V + 1)), 8 * ((size_t)V + 1));
    const size_t nB = (size_t)B * 4, nD = (size_t)B * cap * 4, nM = (size_t)B * W * 4, nL = (size_t)B * V * 2;
    const void *states0 = take(&p, nB), *data0 = take(&p, nD), *len0 = take(&p, nB);
    const void *mask0 = take(&p, nM), *logits = take(&p, nL), *masked = take(&p, nL), *argmax = take(&p, nB);
    const void *tokens = take(&p, nB), *err1 = take(&p, nB), *states1 = take(&p, nB), *len1 = take(&p, nB);
    const void *data1 = take(&p, nD), *mask1 = take(&p, nM);
    const void *jump_bytes = take(&p, (size_t)B * max_jump), *jump_len = take(&p, nB);
    const void *states2 = take(&p, nB), *len2 = take(&p, nB);
    const void *masked1 = take(&p, nL), *argmax1 = take(&p, nB);      /* the step's logits under the NEXT mask */
    if (p - buf != size) { fprintf(stderr, "fixture size mismatch\n"); return 1; }

    pre3_handle *h = NULL;
    pre3_vocab vocab = {vbytes, offsets, V, eos};
    pre3_options opt = {64, cap, 0, 0, 0};
    const char *texts[1] = {grammar};
    CHECK_PRE3(pre3_compile(texts, 1, &vocab, &opt, &h));

    int32_t *d_states, *d_data, *d_len, *d_err, *d_tokens, *d_arg, *d_jlen;
    uint32_t *d_mask;
    uint16_t *d_logits;
    uint8_t *d_jbytes;
    CHECK_HIP(hipMalloc((void **)&d_states, nB)); CHECK_HIP(hipMalloc((void **)&d_data, nD));
    CHECK_HIP(hipMalloc((void **)&d_len, nB)); CHECK_HIP(hipMalloc((void **)&d_err, nB));
    CHECK_HIP(hipMalloc((void **)&d_tokens, nB)); CHECK_HIP(hipMalloc((void **)&d_arg, nB));
    CHECK_HIP(hipMalloc((void **)&d_jlen, nB)); CHECK_HIP(hipMalloc((void **)&d_mask, nM));
    CHECK_HIP(hipMalloc((void **)&d_logits, nL)); CHECK_HIP(hipMalloc((void **)&d_jbytes, (size_t)B * max_jump + 1));
    CHECK_HIP(hipMemcpy(d_states, states0, nB, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_data, data0, nD, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_len, len0, nB, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_logits, logits, nL, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_tokens, tokens, nB, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(d_err, 0xFF, nB));

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    pre3_stacks stacks = {d_data, d_len, cap, B};
    CHECK_PRE3(pre3_bind_state(h, d_states, stacks, d_err));
    CHECK_PRE3(pre3_fill_mask(h, d_states, stacks, d_mask, stream));
    CHECK_PRE3(pre3_apply_mask_argmax(h, d_logits, V, d_mask, d_arg, stream));
    CHECK_PRE3(pre3_apply_mask(d_logits, d_mask, B, V, V, stream));
    CHECK_HIP(hipStreamSynchronize(stream));

    void *got = malloc(nL > nD ? nL : nD);
    int ok = 1;
    CHECK_HIP(hipMemcpy(got, d_mask, nM, hipMemcpyDeviceToHost)); ok &= same("mask", got, mask0, nM);
    CHECK_HIP(hipMemcpy(got, d_arg, nB, hipMemcpyDeviceToHost)); ok &= same("argmax", got, argmax, nB);
    CHECK_HIP(hipMemcpy(got, d_logits, nL, hipMemcpyDeviceToHost)); ok &= same("masked logits", got, masked, nL);

    CHECK_PRE3(pre3_advance_fill_mask(h, d_tokens, d_mask, 0, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(got, d_err, nB, hipMemcpyDeviceToHost)); ok &= same("err", got, err1, nB);
    CHECK_HIP(hipMemcpy(got, d_states, nB, hipMemcpyDeviceToHost)); ok &= same("states after advance", got, states1, nB);
    CHECK_HIP(hipMemcpy(got, d_len, nB, hipMemcpyDeviceToHost)); ok &= same("len after advance", got, len1, nB);
    CHECK_HIP(hipMemcpy(got, d_mask, nM, hipMemcpyDeviceToHost)); ok &= same("next mask", got, mask1, nM);
    CHECK_HIP(hipMemcpy(got, d_data, nD, hipMemcpyDeviceToHost));
    for (int b = 0; b < B && ok; b++)                        /* live entries only */
        ok &= same("stack after advance", (int32_t *)got + (size_t)b * cap, (const int32_t *)data1 + (size_t)b * cap,
                   4 * (size_t)((const int32_t *)len1)[b]);

    CHECK_PRE3(pre3_jump_forward(h, d_jbytes, d_jlen, max_jump, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(got, d_jlen, nB, hipMemcpyDeviceToHost)); ok &= same("jump lengths", got, jump_len, nB);
    CHECK_HIP(hipMemcpy(got, d_jbytes, (size_t)B * max_jump, hipMemcpyDeviceToHost));
    for (int b = 0; b < B && ok; b++)
        ok &= same("jump bytes", (uint8_t *)got + (size_t)b * max_jump, (const uint8_t *)jump_bytes + (size_t)b * max_jump,
                   (size_t)((const int32_t *)jump_len)[b]);
    CHECK_HIP(hipMemcpy(got, d_states, nB, hipMemcpyDeviceToHost)); ok &= same("states after jump", got, states2, nB);
    CHECK_HIP(hipMemcpy(got, d_len, nB, hipMemcpyDeviceToHost)); ok &= same("len after jump", got, len2, nB);

    /* the whole step as one call, from the first state again: advance, next mask, and that mask on the logits
     * (asked for as one kernel: 48 sequences are fewer than the library would choose it for), then the greedy form */
    for (int greedy = 0; greedy < 2; greedy++) {
        CHECK_HIP(hipMemcpy(d_states, states0, nB, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(d_data, data0, nD, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(d_len, len0, nB, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(d_logits, logits, nL, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemset(d_mask, 0x5A, nM));
        if (pre3_step_is_one_kernel(h, d_logits, V, PRE3_STEP_ONE_KERNEL) != 1) { fprintf(stderr, "one-kernel form refused\n"); ok = 0; }
        if (greedy)
            CHECK_PRE3(pre3_advance_fill_argmax(h, d_tokens, d_mask, d_logits, V, d_arg, PRE3_STEP_ONE_KERNEL, stream));
        else
            CHECK_PRE3(pre3_advance_fill_apply_mask(h, d_tokens, d_mask, d_logits, V, PRE3_STEP_ONE_KERNEL, stream));
        CHECK_HIP(hipStreamSynchronize(stream));
        CHECK_HIP(hipMemcpy(got, d_err, nB, hipMemcpyDeviceToHost)); ok &= same("err (one call)", got, err1, nB);
        CHECK_HIP(hipMemcpy(got, d_states, nB, hipMemcpyDeviceToHost)); ok &= same("states (one call)", got, states1, nB);
        CHECK_HIP(hipMemcpy(got, d_len, nB, hipMemcpyDeviceToHost)); ok &= same("len (one call)", got, len1, nB);
        CHECK_HIP(hipMemcpy(got, d_mask, nM, hipMemcpyDeviceToHost)); ok &= same("next mask (one call)", got, mask1, nM);
        CHECK_HIP(hipMemcpy(got, d_logits, nL, hipMemcpyDeviceToHost));
        ok &= same(greedy ? "logits left alone (greedy call)" : "masked logits (one call)", got, greedy ? logits : masked1, nL);
        if (greedy) { CHECK_HIP(hipMemcpy(got, d_arg, nB, hipMemcpyDeviceToHost)); ok &= same("argmax (one call)", got, argmax1, nB); }
    }

    /* the separate advance call on an empty batch and argument errors */
    pre3_stacks none = {NULL, NULL, cap, 0};
    ok &= pre3_fill_mask(h, NULL, none, NULL, stream) == PRE3_OK;
    ok &= pre3_advance(h, NULL, stream) == PRE3_E_BADARG;
    ok &= pre3_apply_mask(NULL, d_mask, B, V, V, stream) == PRE3_E_BADARG;

    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipStreamDestroy(stream));
    pre3_free(h);
    hipFree(d_states); hipFree(d_data); hipFree(d_len); hipFree(d_err); hipFree(d_tokens); hipFree(d_arg);
    hipFree(d_jlen); hipFree(d_mask); hipFree(d_logits); hipFree(d_jbytes);
    free(got); free(buf); free(grammar); free(offsets);
    if (!ok) return 4;
    printf("C ABI OK\n");
    return 0;
}
