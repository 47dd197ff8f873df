/* CPU-only driver of the oracle (oracle/pre3_oracle.c), built with AddressSanitizer and
 * UndefinedBehaviorSanitizer by tests/test_sanitizers.py.  Same inputs and the same output lines
 * as host_compile_check.cpp, computed by the oracle alone (LR(1) tables, the parse loop per
 * token), so the test can also compare the two programs line by line.
 * usage: oracle_check <dir>   (files as for host_compile_check) */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle oracle_t;
oracle_t *pre3o_build(const char *const *texts, int n, char *err, int errlen);
void pre3o_free(oracle_t *O);
int pre3o_n_states_total(const oracle_t *O);
void pre3o_mask_row(const oracle_t *O, const int32_t *stack, int len, int done, const uint8_t *bytes,
                    const int64_t *offsets, int n_tokens, int eos_id, uint32_t *out);
int pre3o_advance(const oracle_t *O, int32_t *stack, int32_t *len, int cap, const uint8_t *bytes, int n);

static char *slurp(const char *path, size_t *n) {
    FILE *f = fopen(path, "rb");
    if (!f) return NULL;
    fseek(f, 0, SEEK_END);
    long sz = ftell(f);
    fseek(f, 0, SEEK_SET);
    char *buf = (char *)malloc((size_t)sz + 1);
    if (fread(buf, 1, (size_t)sz, f) != (size_t)sz) { fclose(f); free(buf); return NULL; }
    buf[sz] = 0;
    fclose(f);
    if (n) *n = (size_t)sz;
    return buf;
}

static uint64_t fnv(const void *data, size_t bytes) {
    const unsigned char *p = (const unsigned char *)data;
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < bytes; ++i) h = (h ^ p[i]) * 1099511628211ull;
    return h;
}

int main(int argc, char **argv) {
    if (argc < 2) return 2;
    char path[4096];
    char *texts[64];
    int n_g = 0;
    for (; n_g < 64; ++n_g) {
        snprintf(path, sizeof path, "%s/grammar_%d.txt", argv[1], n_g);
        texts[n_g] = slurp(path, NULL);
        if (!texts[n_g]) break;
    }
    if (n_g == 0) return 2;
    char err[512];
    oracle_t *O = pre3o_build((const char *const *)texts, n_g, err, (int)sizeof err);
    if (!O) { printf("compile error\n"); for (int i = 0; i < n_g; ++i) free(texts[i]); return 0; }
    size_t vsz, ssz;
    snprintf(path, sizeof path, "%s/vocab.bin", argv[1]);
    char *vb = slurp(path, &vsz);
    snprintf(path, sizeof path, "%s/stacks.bin", argv[1]);
    char *sb = slurp(path, &ssz);
    if (!vb || !sb) return 2;
    int32_t n_tokens, eos;
    memcpy(&n_tokens, vb, 4);
    memcpy(&eos, vb + 4, 4);
    int64_t *offsets = (int64_t *)malloc(sizeof(int64_t) * ((size_t)n_tokens + 1));
    memcpy(offsets, vb + 8, sizeof(int64_t) * ((size_t)n_tokens + 1));
    const uint8_t *bytes = (const uint8_t *)vb + 8 + sizeof(int64_t) * ((size_t)n_tokens + 1);
    const int n_words = (n_tokens + 31) / 32;
    uint32_t *row = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n_words);
    printf("tables states %d\n", pre3o_n_states_total(O));
    const int32_t *p = (const int32_t *)sb;
    const int count = *p++;
    for (int k = 0; k < count; ++k) {
        const int len = *p++;
        const int cap = len + 4096;
        int32_t *st = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
        memcpy(st, p, sizeof(int32_t) * (size_t)len);
        p += len;
        const int token = *p++;
        pre3o_mask_row(O, st, len, 0, bytes, offsets, n_tokens, eos, row);
        int32_t nl = len;
        int rc = -1;
        if (token >= 0 && token < n_tokens && token != eos)
            rc = pre3o_advance(O, st, &nl, cap, bytes + offsets[token], (int)(offsets[token + 1] - offsets[token]));
        if (rc != 0) nl = len;
        printf("stack %d row %016llx advance %d %016llx\n", k, (unsigned long long)fnv(row, sizeof(uint32_t) * (size_t)n_words), rc,
               (unsigned long long)fnv(st, sizeof(int32_t) * (size_t)nl));
        free(st);
    }
    free(row); free(offsets); free(vb); free(sb);
    for (int i = 0; i < n_g; ++i) free(texts[i]);
    pre3o_free(O);
    return 0;
}
