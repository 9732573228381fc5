/*
 * C-only parity check of the C-ABI: no Python, no torch.  Runs the library on
 * the GPU through <hip/hip_runtime_api.h> and compares with the CPU oracle
 * (linked as a second shared object), byte for byte.
 *
 *   abi_parity p block_bytes [algo]
 *
 * Prints one line and exits 0 on a match.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sparbit.h"

int oracle_allgather(int algo, int p, size_t B, const void *send, void *recv, int max_steps,
                     int32_t *step_info, int64_t *sent_per_rank, int32_t *trace, size_t trace_cap,
                     size_t *trace_len);
int oracle_naive_allgather(int p, size_t B, const void *send, void *recv);

#define CHECK_HIP(x)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__);      \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)

int main(int argc, char **argv)
{
    int p = argc > 1 ? atoi(argv[1]) : 6;
    size_t B = argc > 2 ? (size_t)atoll(argv[2]) : 1024;
    int algo = argc > 3 ? atoi(argv[3]) : SPARBIT_ALGO_SPARBIT;
    size_t ns = (size_t)p * B, nr = (size_t)p * p * B, i;
    uint8_t *send = malloc(ns), *want = malloc(nr), *got = malloc(nr);
    void *d_send = NULL, *d_recv = NULL;
    hipStream_t stream;
    uint64_t x = 0x9E3779B97F4A7C15ull, timeouts = 0;
    int rc;

    if (!send || !want || !got) return 2;
    for (i = 0; i < ns; i++) { /* any bytes will do: the path is value-oblivious */
        x ^= x << 13; x ^= x >> 7; x ^= x << 17;
        send[i] = (uint8_t)(x >> 24);
    }
    memset(want, 0xA5, nr);
    rc = algo == SPARBIT_ALGO_DIRECT ? oracle_naive_allgather(p, B, send, want)
                                     : oracle_allgather(algo, p, B, send, want, -1, NULL, NULL, NULL, 0, NULL);
    if (rc != 0) { fprintf(stderr, "oracle failed: %d\n", rc); return 2; }

    CHECK_HIP(hipMalloc(&d_send, ns));
    CHECK_HIP(hipMalloc(&d_recv, nr));
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_HIP(hipMemcpy(d_send, send, ns, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(d_recv, 0xA5, nr));
    CHECK_HIP(hipDeviceSynchronize());
    rc = sparbit_allgather_algo(d_send, d_recv, p, B, algo, stream);
    if (rc != SPARBIT_OK) { fprintf(stderr, "sparbit_allgather_algo: %s\n", sparbit_strerror(rc)); return 1; }
    CHECK_HIP(hipStreamSynchronize(stream));
    rc = sparbit_barrier_timeouts(stream, &timeouts);
    if (rc != SPARBIT_OK || timeouts) { fprintf(stderr, "bounded wait expired\n"); return 1; }
    CHECK_HIP(hipMemcpy(got, d_recv, nr, hipMemcpyDeviceToHost));
    rc = memcmp(got, want, nr) != 0;
    printf("abi_parity p=%d block_bytes=%zu algo=%d: %s\n", p, B, algo, rc ? "MISMATCH" : "match");
    sparbit_finalize();
    (void)hipFree(d_send);
    (void)hipFree(d_recv);
    (void)hipStreamDestroy(stream);
    free(send); free(want); free(got);
    return rc;
}
