/*
 * Seeded synthetic-tensor generator (host, plain C, pthreads).
 *
 * This file produces INPUT DATA only: random-init weight tensors.  It holds none
 * of the method's arithmetic and is the one piece of code that both the CPU
 * oracle's tests and the HIP library's tests/benchmarks may call.
 *
 * Element i of tensor `tid` under `seed` is a pure function of (seed, tid, i):
 *
 *   block   = Philox4x32-10( key = (seed, tid),
 *                            counter = (lo32(i/8), hi32(i/8), 0, 0) )
 *   h       = 16-bit half number (i % 8) of the 128-bit block
 *   value   = std * qtable[h] + mean
 *
 * where qtable[j] is the standard-normal quantile at (j + 0.5) / 65536, supplied
 * by the caller (the Python side computes it once).  The result is a 65536-level
 * discretisation of N(mean, std^2): far finer than bf16 can hold.  Because every
 * element depends only on its own index the generator is order- and
 * thread-count-independent.
 *
 * Philox4x32-10 is the counter-based generator of Salmon, Moraes, Dror and Shaw,
 * "Parallel random numbers: as easy as 1, 2, 3" (SC'11); the multipliers and Weyl
 * key increments below are the ones that paper publishes.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PHILOX_M0 0xD2511F53u
#define PHILOX_M1 0xCD9E8D57u
#define PHILOX_W0 0x9E3779B9u
#define PHILOX_W1 0xBB67AE85u

static inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                 uint32_t k0, uint32_t k1, uint32_t out[4]) {
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)PHILOX_M0 * c0;
        uint64_t p1 = (uint64_t)PHILOX_M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += PHILOX_W0; k1 += PHILOX_W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Exposed for the known-answer test of the generator itself. */
void synth_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1], out);
}

static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u; memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u); /* NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

typedef struct {
    void* dst; int dtype;            /* 0 = f32, 1 = bf16 */
    uint64_t begin, end;             /* element range [begin, end) */
    uint32_t seed, tid;
    const float* tab32;              /* per-call tables: value for each 16-bit draw */
    const uint16_t* tab16;
} job_t;

static void* worker(void* arg) {
    job_t* j = (job_t*)arg;
    uint64_t i = j->begin;
    while (i < j->end) {
        uint64_t blk = i >> 3;
        uint32_t r[4];
        philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u, j->seed, j->tid, r);
        uint16_t h[8];
        for (int q = 0; q < 4; ++q) { h[2 * q] = (uint16_t)(r[q] & 0xffffu); h[2 * q + 1] = (uint16_t)(r[q] >> 16); }
        uint64_t base = blk << 3;
        if (i == base && base + 8 <= j->end) {
            if (j->dtype == 0) { float* p = (float*)j->dst + base; for (int q = 0; q < 8; ++q) p[q] = j->tab32[h[q]]; }
            else { uint16_t* p = (uint16_t*)j->dst + base; for (int q = 0; q < 8; ++q) p[q] = j->tab16[h[q]]; }
            i = base + 8;
        } else {
            uint64_t stop = base + 8; if (stop > j->end) stop = j->end;
            for (; i < stop; ++i) {
                if (j->dtype == 0) ((float*)j->dst)[i] = j->tab32[h[i & 7u]];
                else               ((uint16_t*)j->dst)[i] = j->tab16[h[i & 7u]];
            }
        }
    }
    return NULL;
}

/* Fill dst[0..n) (f32 if dtype==0, bf16 bit patterns if dtype==1).  Returns 0, or
 * -1 on bad arguments.  n_threads <= 0 means 1. */
int synth_fill_normal(void* dst, uint64_t n, int dtype, uint32_t seed, uint32_t tid,
                      float mean, float std, const float* qtable, int n_threads) {
    if (!dst || !qtable || (dtype != 0 && dtype != 1)) return -1;
    if (n_threads <= 0) n_threads = 1;
    if (n_threads > 64) n_threads = 64;
    if (n < (1u << 16)) n_threads = 1;
    float* tab32 = (float*)malloc(65536 * sizeof(float));
    uint16_t* tab16 = (uint16_t*)malloc(65536 * sizeof(uint16_t));
    if (!tab32 || !tab16) { free(tab32); free(tab16); return -1; }
    for (int q = 0; q < 65536; ++q) { tab32[q] = std * qtable[q] + mean; tab16[q] = f32_to_bf16_rne(tab32[q]); }
    pthread_t th[64]; job_t jobs[64];
    uint64_t per = ((n / (uint64_t)n_threads) + 7u) & ~(uint64_t)7u;   /* whole blocks */
    if (per == 0) per = 8;
    int started = 0;
    for (int t = 0; t < n_threads; ++t) {
        uint64_t b = per * (uint64_t)t, e = (t == n_threads - 1) ? n : per * (uint64_t)(t + 1);
        if (b >= n) break;
        if (e > n) e = n;
        jobs[t] = (job_t){dst, dtype, b, e, seed, tid, tab32, tab16};
        if (n_threads == 1) { worker(&jobs[t]); break; }
        pthread_create(&th[t], NULL, worker, &jobs[t]);
        ++started;
    }
    for (int t = 0; t < started; ++t) pthread_join(th[t], NULL);
    free(tab32); free(tab16);
    return 0;
}

/* Fill dst[0..n) with the constant value (norm gains are initialised to 1). */
int synth_fill_const(void* dst, uint64_t n, int dtype, float value) {
    if (!dst || (dtype != 0 && dtype != 1)) return -1;
    if (dtype == 0) { float* p = (float*)dst; for (uint64_t i = 0; i < n; ++i) p[i] = value; }
    else { uint16_t b = f32_to_bf16_rne(value); uint16_t* p = (uint16_t*)dst;
           for (uint64_t i = 0; i < n; ++i) p[i] = b; }
    return 0;
}
