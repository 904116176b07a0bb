/*
 * All-core host baseline for the benchmark.  TEST AND MEASUREMENT INFRASTRUCTURE ONLY.
 *
 * This is NOT the oracle: the oracle (oracle/scan_oracle.c) is the sequential definition and stays untouched.  This file is
 * the textbook way to scan on a multi-core host, timed next to the GPU path so that the single-core oracle figure is
 * not the only host number: one thread per core; many rows -> rows are dealt to the threads; few rows -> every row is
 * cut into one chunk per thread, the chunks are summed, each thread adds up the sums of the chunks before its own and
 * scans its chunk again from that offset (the three steps of the paper's Section 2.2 with chunks as segments).
 * tests/test_host_threads.py checks it against the oracle; the product path never calls it.
 *
 * Arithmetic: integers in 64 bits, output the low 32; floats in fp64 over the exact input values, output rounded to
 * fp32.  The chunked order of the additions differs from the oracle's, by rounding in the 53rd bit only.
 */
#define _GNU_SOURCE
#include <pthread.h>
#include <sched.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { K_I32 = 0, K_F16 = 1, K_I8 = 2, K_F32 = 3, K_BF16 = 4 };

static double half_value(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 0) v = (double)m * 0x1p-24;                              /* subnormal: m * 2^-24 */
    else if (e == 31) v = m ? (0.0 / 0.0) : (1.0 / 0.0);
    else {
        uint64_t bits = ((uint64_t)(e - 15 + 1023) << 52) | ((uint64_t)m << 42);
        memcpy(&v, &bits, 8);
    }
    return sign ? -v : v;
}

static double float_at(const void *x, size_t i, int kind)
{
    if (kind == K_F32) return (double)((const float *)x)[i];
    if (kind == K_BF16) {
        uint32_t b = (uint32_t)((const uint16_t *)x)[i] << 16;
        float f;
        memcpy(&f, &b, 4);
        return (double)f;
    }
    return half_value(((const uint16_t *)x)[i]);
}

static int64_t int_at(const void *x, size_t i, int kind)
{
    return kind == K_I8 ? (int64_t)((const int8_t *)x)[i] : (int64_t)((const int32_t *)x)[i];
}

/* sum of x[lo, hi) */
static void range_sum(const void *x, int kind, size_t lo, size_t hi, int64_t *isum, double *fsum)
{
    if (kind == K_I32 || kind == K_I8) {
        int64_t a = 0;
        for (size_t i = lo; i < hi; ++i) a += int_at(x, i, kind);
        *isum = a;
    } else {
        double a = 0.0;
        for (size_t i = lo; i < hi; ++i) a += float_at(x, i, kind);
        *fsum = a;
    }
}

/* scan of x[lo, hi) into y, starting from the given sum of everything before lo */
static void range_scan(const void *x, int kind, void *y, size_t lo, size_t hi, int exclusive, int64_t ioff, double foff)
{
    if (kind == K_I32 || kind == K_I8) {
        int32_t *out = (int32_t *)y;
        int64_t a = ioff;
        for (size_t i = lo; i < hi; ++i) {
            const int64_t v = int_at(x, i, kind);
            if (exclusive) { out[i] = (int32_t)(uint32_t)(uint64_t)a; a += v; }
            else           { a += v; out[i] = (int32_t)(uint32_t)(uint64_t)a; }
        }
    } else {
        float *out = (float *)y;
        double a = foff;
        for (size_t i = lo; i < hi; ++i) {
            const double v = float_at(x, i, kind);
            if (exclusive) { out[i] = (float)a; a += v; }
            else           { a += v; out[i] = (float)a; }
        }
    }
}

typedef struct {
    const void *x;
    void *y;
    int kind, exclusive, threads, id;
    size_t rows, cols;
    int64_t *isums;          /* one per thread */
    double *fsums;
    pthread_barrier_t *bar;
} job_t;

static void *worker(void *arg)
{
    const job_t *j = (const job_t *)arg;
    const size_t T = (size_t)j->threads, id = (size_t)j->id;
    if (j->rows >= T) {                                  /* rows dealt to the threads, each scanned in one go */
        const size_t r0 = j->rows * id / T, r1 = j->rows * (id + 1) / T;
        for (size_t r = r0; r < r1; ++r) range_scan(j->x, j->kind, j->y, r * j->cols, (r + 1) * j->cols, j->exclusive, 0, 0.0);
        return NULL;
    }
    for (size_t r = 0; r < j->rows; ++r) {               /* every row: chunk sums, offsets, chunk scans */
        const size_t lo = r * j->cols + j->cols * id / T, hi = r * j->cols + j->cols * (id + 1) / T;
        range_sum(j->x, j->kind, lo, hi, &j->isums[id], &j->fsums[id]);
        pthread_barrier_wait(j->bar);
        int64_t ioff = 0;
        double foff = 0.0;
        for (size_t t = 0; t < id; ++t) { ioff += j->isums[t]; foff += j->fsums[t]; }
        range_scan(j->x, j->kind, j->y, lo, hi, j->exclusive, ioff, foff);
        pthread_barrier_wait(j->bar);                    /* the sums are overwritten by the next row */
    }
    return NULL;
}

/* Number of cores this process may run on. */
int host_threads_available(void)
{
    cpu_set_t set;
    if (sched_getaffinity(0, sizeof set, &set) != 0) return 1;
    const int n = CPU_COUNT(&set);
    return n > 0 ? n : 1;
}

/* y (int32 / fp32) <- scan of x (int32, int8 / f16, bf16, f32 bit patterns), rows x cols row-major, on `threads`
 * threads (<= 0: one per available core, at most 256).  Returns 0, or 1 for a bad argument, 2 if a thread or the
 * barrier could not be created. */
int host_threads_scan(const void *x, int kind, void *y, size_t rows, size_t cols, int exclusive, int threads)
{
    if (kind < 0 || kind > 4) return 1;
    if (rows == 0 || cols == 0) return 0;
    if (!x || !y) return 1;
    if (threads <= 0) threads = host_threads_available();
    if (threads > 256) threads = 256;
    int64_t isums[256];
    double fsums[256];
    memset(isums, 0, sizeof isums);
    memset(fsums, 0, sizeof fsums);
    pthread_barrier_t bar;
    if (pthread_barrier_init(&bar, NULL, (unsigned)threads) != 0) return 2;
    job_t jobs[256];
    pthread_t tid[256];
    int started = 0, rc = 0;
    for (int t = 0; t < threads; ++t) {
        jobs[t] = (job_t){x, y, kind, exclusive, threads, t, rows, cols, isums, fsums, &bar};
        if (pthread_create(&tid[t], NULL, worker, &jobs[t]) != 0) { rc = 2; break; }
        ++started;
    }
    if (rc != 0 && rows < (size_t)threads) {
        /* threads that started wait at a barrier sized for all of them: there is no clean way on; the caller's
         * process is a test or a benchmark, so give up loudly rather than deadlock */
        abort();
    }
    for (int t = 0; t < started; ++t) pthread_join(tid[t], NULL);
    pthread_barrier_destroy(&bar);
    return rc;
}
