/*
 * Host-cores baseline for the benchmark report.  TEST / BENCHMARK INFRASTRUCTURE ONLY, and NOT the oracle:
 * parity is always judged against the sequential loop of mmvseg_oracle.c, and this file is itself checked
 * against that loop (tests/test_host_threads.py).  It exists so that the benchmark can put "all cores of
 * the host" beside the GPU figure, next to the single-thread loop the paper uses as its CPU reference
 * (Sec. 5, experimental set-up).
 *
 * Segmented inclusive scan (Problem 2.1 of Sec. 2), int8 values -> int32 with wrap-around, one flag byte per
 * element, in the textbook three steps over T contiguous chunks:
 *   1. every thread scans its chunk as if the chunk started a segment, and notes the chunk's last value,
 *      whether the chunk holds a flag, and where its first flag is;
 *   2. one thread walks the T chunk summaries: the value that reaches chunk t from the left is the last
 *      value of chunk t-1, plus what reached chunk t-1 if that chunk held no flag;
 *   3. every thread adds what reached its chunk to the elements before the chunk's first flag.
 * Shares no code with the HIP library.
 */
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>

#define HOST_MAX_THREADS 256

typedef struct {
    const int8_t *x;
    const uint8_t *f;
    int32_t *z;
    uint64_t begin, end;      /* the chunk [begin, end) */
    uint64_t first_flag;      /* first i in the chunk with i == 0 or f[i] != 0; end if none */
    uint32_t last;            /* z[end-1] of the local scan */
    uint32_t carry;           /* what reaches the chunk from the left (step 2) */
} chunk_t;

static void *local_scan(void *arg)
{
    chunk_t *c = (chunk_t *)arg;
    const int8_t *x = c->x;
    const uint8_t *f = c->f;
    int32_t *z = c->z;
    const uint64_t end = c->end;
    uint64_t first = end;
    uint32_t acc = 0;
    for (uint64_t i = c->begin; i < end; ++i) {
        uint32_t xi = (uint32_t)(int32_t)x[i];
        if (i == 0 || f[i]) {
            if (first == end)
                first = i;
            acc = xi;
        } else {
            acc = acc + xi;
        }
        z[i] = (int32_t)acc;
    }
    c->first_flag = first;
    c->last = acc;
    return NULL;
}

static void *add_carry(void *arg)
{
    chunk_t *c = (chunk_t *)arg;
    int32_t *z = c->z;
    const uint64_t stop = c->first_flag;
    const uint32_t carry = c->carry;
    for (uint64_t i = c->begin; i < stop; ++i)
        z[i] = (int32_t)((uint32_t)z[i] + carry);
    return NULL;
}

/* Returns the number of threads used (chunks that hold at least one element), 0 for n == 0, -1 on a bad
 * argument or when a thread cannot be started. */
int host_threads_segscan_i8(const int8_t *x, const uint8_t *f, uint64_t n, int32_t *z, int threads)
{
    chunk_t ch[HOST_MAX_THREADS];
    pthread_t th[HOST_MAX_THREADS];
    if (threads < 1 || threads > HOST_MAX_THREADS || (n && (!x || !f || !z)))
        return -1;
    if (n == 0)
        return 0;
    if ((uint64_t)threads > n)
        threads = (int)n;
    for (int t = 0; t < threads; ++t) {
        ch[t].x = x; ch[t].f = f; ch[t].z = z;
        ch[t].begin = n / (uint64_t)threads * (uint64_t)t;
        ch[t].end = t == threads - 1 ? n : n / (uint64_t)threads * (uint64_t)(t + 1);
        ch[t].carry = 0;
    }
    for (int t = 0; t < threads; ++t)
        if (pthread_create(&th[t], NULL, local_scan, &ch[t]) != 0) {
            for (int u = 0; u < t; ++u) pthread_join(th[u], NULL);
            return -1;
        }
    for (int t = 0; t < threads; ++t)
        pthread_join(th[t], NULL);
    for (int t = 1; t < threads; ++t)
        ch[t].carry = ch[t - 1].last + (ch[t - 1].first_flag == ch[t - 1].end ? ch[t - 1].carry : 0u);
    for (int t = 1; t < threads; ++t)
        if (pthread_create(&th[t], NULL, add_carry, &ch[t]) != 0) {
            for (int u = 1; u < t; ++u) pthread_join(th[u], NULL);
            return -1;
        }
    for (int t = 1; t < threads; ++t)
        pthread_join(th[t], NULL);
    return threads;
}
