/* A plain C program that drives the library through its C ABI with no Python
 * in between: 8 rank buffers in device memory, AllReduce (bf16 and f32) and
 * AllGather with the whole message on the device path and with 12 % of it on
 * the host-staged path, and the AllReduce that needs no communicator, every
 * result compared bit for bit with the CPU oracle.
 * Test infrastructure: built by tests/c_abi/build.py, run by the GPU tests.
 * Exit status 0 = every comparison passed. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "flexlink.h"

/* the CPU oracle (oracle/flex_oracle.c) */
void oracle_allreduce_f32(const void* const* bufs, int n, size_t count, void* out);
void oracle_allreduce_bf16(const void* const* bufs, int n, size_t count, void* out);
void oracle_allgather(const void* const* slices, int n, size_t slice_bytes, void* out);

#define N 8

#define HIP_OK(expr)                                                                  \
    do {                                                                              \
        hipError_t e_ = (expr);                                                       \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "%s failed: %s\n", #expr, hipGetErrorString(e_));         \
            return 2;                                                                 \
        }                                                                             \
    } while (0)

#define FLEX_OK_OR_FAIL(expr)                                                         \
    do {                                                                              \
        int s_ = (expr);                                                              \
        if (s_ != FLEX_OK) {                                                          \
            fprintf(stderr, "%s -> %s: %s\n", #expr, flex_status_string(s_), flex_last_error()); \
            return 3;                                                                 \
        }                                                                             \
    } while (0)

/* splitmix64: seeded, reproducible bit patterns */
static uint64_t next_u64(uint64_t* s) {
    uint64_t z = (*s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* finite bf16 / f32 patterns with exponents near 1.0, so that sums round */
static void fill_bf16(uint16_t* p, size_t n, uint64_t seed) {
    for (size_t i = 0; i < n; ++i) {
        uint64_t r = next_u64(&seed);
        p[i] = (uint16_t)(((r & 1) << 15) | ((0x7Cu + ((r >> 1) % 6)) << 7) | ((r >> 8) & 0x7F));
    }
}
static void fill_f32(uint32_t* p, size_t n, uint64_t seed) {
    for (size_t i = 0; i < n; ++i) {
        uint64_t r = next_u64(&seed);
        p[i] = (uint32_t)(((r & 1) << 31) | ((0x7Cu + ((r >> 1) % 6)) << 23) | ((r >> 8) & 0x7FFFFF));
    }
}

static int check(const char* what, const void* got, const void* want, size_t bytes) {
    if (memcmp(got, want, bytes) == 0) {
        printf("ok   %s\n", what);
        return 0;
    }
    printf("FAIL %s\n", what);
    return 1;
}

int main(void) {
    const size_t count = (1u << 20) + 2048 + 5; /* several tiles and a ragged tail */
    int failures = 0;
    int ndev = 0;
    HIP_OK(hipGetDeviceCount(&ndev));
    if (ndev < 1) {
        fprintf(stderr, "no HIP device\n");
        return 2;
    }
    HIP_OK(hipSetDevice(0));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    flex_config_t cfg;
    FLEX_OK_OR_FAIL(flex_config_default(&cfg));
    cfg.max_host_units = 10000;
    flex_comm_t* comm = NULL;
    FLEX_OK_OR_FAIL(flex_comm_create(&comm, N, 3, count * 4, &cfg));

    for (int dtype = FLEX_F32; dtype <= FLEX_BF16; ++dtype) {
        const size_t es = dtype == FLEX_F32 ? 4 : 2;
        void* host[N];
        void* dev[N];
        const void* dev_c[N];
        const void* host_c[N];
        for (int r = 0; r < N; ++r) {
            host[r] = malloc(count * es);
            if (!host[r]) return 2;
            if (dtype == FLEX_F32)
                fill_f32((uint32_t*)host[r], count, 1000 + (uint64_t)r);
            else
                fill_bf16((uint16_t*)host[r], count, 2000 + (uint64_t)r);
            HIP_OK(hipMalloc(&dev[r], count * es));
            HIP_OK(hipMemcpy(dev[r], host[r], count * es, hipMemcpyHostToDevice));
            dev_c[r] = dev[r];
            host_c[r] = host[r];
        }
        void* want_ar = malloc(count * es);
        void* want_ag = malloc(N * count * es);
        void* got = malloc(N * count * es);
        if (!want_ar || !want_ag || !got) return 2;
        if (dtype == FLEX_F32)
            oracle_allreduce_f32(host_c, N, count, want_ar);
        else
            oracle_allreduce_bf16(host_c, N, count, want_ar);
        oracle_allgather(host_c, N, count * es, want_ag);

        void* out_ar;
        void* out_ag;
        HIP_OK(hipMalloc(&out_ar, count * es));
        HIP_OK(hipMalloc(&out_ag, N * count * es));
        const uint32_t shares[2] = {0, 1200};
        for (int k = 0; k < 2; ++k) {
            char what[96];
            FLEX_OK_OR_FAIL(flex_set_split(comm, FLEX_ALLREDUCE, FLEX_SPLIT_STATIC, shares[k]));
            FLEX_OK_OR_FAIL(flex_set_split(comm, FLEX_ALLGATHER, FLEX_SPLIT_STATIC, shares[k]));
            HIP_OK(hipMemsetAsync(out_ar, 0, count * es, stream));
            HIP_OK(hipMemsetAsync(out_ag, 0, N * count * es, stream));
            FLEX_OK_OR_FAIL(flex_allreduce_local(comm, dev_c, out_ar, count, dtype, FLEX_SUM, stream));
            FLEX_OK_OR_FAIL(flex_allgather_local(comm, dev_c, out_ag, count, dtype, stream));
            HIP_OK(hipStreamSynchronize(stream));
            HIP_OK(hipMemcpy(got, out_ar, count * es, hipMemcpyDeviceToHost));
            snprintf(what, sizeof what, "allreduce %s host share %u/10000", dtype == FLEX_F32 ? "f32" : "bf16",
                     shares[k]);
            failures += check(what, got, want_ar, count * es);
            HIP_OK(hipMemcpy(got, out_ag, N * count * es, hipMemcpyDeviceToHost));
            snprintf(what, sizeof what, "allgather %s host share %u/10000", dtype == FLEX_F32 ? "f32" : "bf16",
                     shares[k]);
            failures += check(what, got, want_ag, N * count * es);
        }
        {
            /* the entry point that needs no communicator and allocates nothing */
            char what[96];
            HIP_OK(hipMemsetAsync(out_ar, 0, count * es, stream));
            FLEX_OK_OR_FAIL(flex_allreduce_staged_noalloc(dev_c, N, 3, out_ar, count, dtype, FLEX_SUM, 1200, stream));
            HIP_OK(hipStreamSynchronize(stream));
            HIP_OK(hipMemcpy(got, out_ar, count * es, hipMemcpyDeviceToHost));
            snprintf(what, sizeof what, "allreduce %s without a communicator, staged share 1200/10000",
                     dtype == FLEX_F32 ? "f32" : "bf16");
            failures += check(what, got, want_ar, count * es);
        }
        flex_stats_t st;
        FLEX_OK_OR_FAIL(flex_evaluator_drain(comm));
        FLEX_OK_OR_FAIL(flex_get_stats(comm, FLEX_ALLREDUCE, count, dtype, &st));
        if (st.split_calls < 1 || st.samples < 1) {
            printf("FAIL evaluator saw no split call\n");
            ++failures;
        }
        HIP_OK(hipFree(out_ar));
        HIP_OK(hipFree(out_ag));
        for (int r = 0; r < N; ++r) {
            HIP_OK(hipFree(dev[r]));
            free(host[r]);
        }
        free(want_ar);
        free(want_ag);
        free(got);
    }
    /* error behaviour: nothing is enqueued, a message is left for the caller */
    if (flex_allreduce_local(comm, NULL, NULL, 16, FLEX_BF16, FLEX_SUM, stream) != FLEX_ERR_INVALID_ARG ||
        strlen(flex_last_error()) == 0) {
        printf("FAIL null pointer array was not rejected\n");
        ++failures;
    }
    HIP_OK(hipStreamSynchronize(stream));
    FLEX_OK_OR_FAIL(flex_comm_destroy(comm));
    HIP_OK(hipStreamDestroy(stream));
    printf("%s\n", failures ? "C ABI check FAILED" : "C ABI check passed");
    return failures ? 1 : 0;
}
