/*
 * A plain C program against the C ABI: no Python, no PyTorch.  It allocates
 * with the HIP runtime, encodes on a stream it created, compares every parity
 * byte with the CPU oracle (linked in as test infrastructure), loses shards,
 * rebuilds them and compares again.  Built by paper_2605_00831_amd/build.py
 * (hipcc, host code only) and run by tests/test_gpu_c_abi.py.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/ghostserve_ec.h"

/* oracle entry points (oracle/gs_oracle.c) */
int gso_generator(int k, int m, uint8_t *P);
void gso_encode(int k, int m, const uint8_t *P, const uint8_t *const *data, uint8_t *const *parity, size_t S);

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_GS(x) do { int r_ = (x); if (r_ != GS_OK) { printf("gs error %d (%s) at line %d\n", r_, gs_strerror(r_), __LINE__); return 3; } } while (0)

static uint32_t rng_state = 0x67530005u;
static uint8_t next_byte(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return (uint8_t)(rng_state >> 11);
}

static int run(int k, int m, size_t S, const int *erased, int n_erased)
{
    enum { MAXN = 32 };
    uint8_t *host[MAXN] = {0}, *want[MAXN] = {0}, *back = NULL;
    void *dev[MAXN] = {0};
    uint8_t P[MAXN * MAXN];
    hipStream_t stream;
    gs_code *code = NULL;
    int rc = 0;

    CHECK_GS(gs_make_code(k, m, GS_CAUCHY, &code));
    CHECK_GS(gs_code_matrix(code, P));
    {
        uint8_t Po[MAXN * MAXN];
        if (gso_generator(k, m, Po) != 0 || memcmp(P, Po, (size_t)k * m) != 0) { printf("generator differs from the oracle\n"); return 4; }
    }
    CHECK_HIP(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));
    back = (uint8_t *)malloc(S + 64);
    for (int r = 0; r < k + m; r++) {
        host[r] = (uint8_t *)malloc(S ? S : 1);
        CHECK_HIP(hipMalloc(&dev[r], S + 64));
        CHECK_HIP(hipMemset(dev[r], 0xC7, S + 64));
        if (r < k) {
            for (size_t t = 0; t < S; t++) host[r][t] = next_byte();
            CHECK_HIP(hipMemcpy(dev[r], host[r], S, hipMemcpyHostToDevice));
        }
    }
    for (int i = 0; i < m; i++) want[i] = host[k + i];
    gso_encode(k, m, P, (const uint8_t *const *)host, want, S);

    CHECK_GS(gs_encode(code, (const void *const *)dev, dev + k, S, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    for (int i = 0; i < m && rc == 0; i++) {
        CHECK_HIP(hipMemcpy(back, dev[k + i], S + 64, hipMemcpyDeviceToHost));
        if (memcmp(back, want[i], S) != 0) { printf("parity %d differs from the oracle (k=%d m=%d S=%zu)\n", i, k, m, S); rc = 5; }
        for (size_t t = S; t < S + 64; t++) if (back[t] != 0xC7) { printf("parity %d written past the end\n", i); rc = 6; break; }
    }
    for (int x = 0; x < n_erased; x++) CHECK_HIP(hipMemset(dev[erased[x]], 0xA5, S));
    CHECK_GS(gs_reconstruct(code, dev, erased, n_erased, S, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    for (int x = 0; x < n_erased && rc == 0; x++) {
        CHECK_HIP(hipMemcpy(back, dev[erased[x]], S + 64, hipMemcpyDeviceToHost));
        if (memcmp(back, host[erased[x]], S) != 0) { printf("shard %d not rebuilt (k=%d m=%d S=%zu)\n", erased[x], k, m, S); rc = 7; }
        for (size_t t = S; t < S + 64; t++) if (back[t] != 0xC7) { printf("shard %d written past the end\n", erased[x]); rc = 8; break; }
    }
    /* error paths answer without touching anything */
    {
        int too_many[8] = {0, 1, 2, 3, 4, 5, 6, 7};
        if (gs_reconstruct(code, dev, too_many, m + 1, S, stream) != GS_ETOOMANY) { printf("missing GS_ETOOMANY\n"); rc = 9; }
    }
    for (int r = 0; r < k + m; r++) { free(host[r]); (void)hipFree(dev[r]); }
    free(back);
    (void)hipStreamDestroy(stream);
    gs_free_code(code);
    return rc;
}

int main(void)
{
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n < 1) { printf("no GPU\n"); return 1; }
    const int e42[] = {1, 3}, e83[] = {2, 5, 9}, e41[] = {4}, e202[] = {0, 21};
    int rc = run(4, 2, (2u << 20) + 5, e42, 2);
    if (!rc) rc = run(8, 3, 65536 + 5, e83, 3);
    if (!rc) rc = run(4, 1, 4097, e41, 1);
    if (!rc) rc = run(20, 2, 100000, e202, 2);
    if (!rc) printf("C ABI round trip OK\n");
    return rc;
}
