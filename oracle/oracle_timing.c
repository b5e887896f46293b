/*
 * oracle_timing.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Times the CPU oracle (lmc_oracle.c) as it stands, for the benchmark's "cpu_baseline"
 * figure: the store analogue (gather a chunk from the pages into a contiguous buffer,
 * then copy the buffer into the pool: paper section 5.1, one transfer per chunk) and the
 * retrieve analogue (copy the chunk out of the pool, scatter it into fresh pages).
 * Nothing of the oracle is changed or tuned: this file only calls orc_gather_chunk and
 * orc_scatter_chunk, with chunks dealt out to plain threads (chunk i goes to thread
 * i mod n_threads) and every buffer allocated before the clock starts.
 *
 * The geometry struct is declared here a second time, field for field as in
 * lmc_oracle.c, so that the oracle's source stays untouched.
 */
#define _POSIX_C_SOURCE 200809L
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

typedef struct {
    int32_t L, P, H, D, e, BS, NB, CT;
    int64_t plane_stride, block_stride, token_stride, head_stride;
} orc_geom_t;

int64_t orc_chunk_bytes(const orc_geom_t *g);
int orc_gather_chunk(const orc_geom_t *g, const uint8_t *const *layers, const int64_t *slot,
                     uint8_t *chunk);
int orc_scatter_chunk(const orc_geom_t *g, const uint8_t *chunk, const int64_t *slot,
                      uint8_t *const *layers);

typedef struct {
    const orc_geom_t *g;
    const uint8_t *const *src;   /* pages the chunks are stored from */
    uint8_t *const *dst;         /* pages the chunks are retrieved into */
    const int64_t *store_slots, *load_slots;   /* n_chunks * CT each */
    int64_t n_chunks;
    uint8_t *pool;               /* n_chunks * chunk_bytes */
    uint8_t *buffer;             /* this thread's contiguous chunk buffer */
    int tid, n_threads, retrieve;
    int status;
} job_t;

static void *run(void *arg)
{
    job_t *j = (job_t *)arg;
    const int64_t cb = orc_chunk_bytes(j->g);
    const int64_t CT = j->g->CT;
    for (int64_t i = j->tid; i < j->n_chunks; i += j->n_threads) {
        int rc;
        if (!j->retrieve) {
            rc = orc_gather_chunk(j->g, j->src, j->store_slots + i * CT, j->buffer);
            memcpy(j->pool + i * cb, j->buffer, (size_t)cb);
        } else {
            memcpy(j->buffer, j->pool + i * cb, (size_t)cb);
            rc = orc_scatter_chunk(j->g, j->buffer, j->load_slots + i * CT, j->dst);
        }
        if (rc != 0) j->status = rc;
    }
    return NULL;
}

static double now(void)
{
    struct timespec t;
    clock_gettime(CLOCK_MONOTONIC, &t);
    return (double)t.tv_sec + 1e-9 * (double)t.tv_nsec;
}

/* One pass of store (retrieve == 0) or retrieve over all chunks on n_threads threads.
 * pool: n_chunks * chunk_bytes; buffers: n_threads * chunk_bytes.  Returns the wall
 * time of the pass in seconds (threads started and joined inside), negative on error. */
double orc_time_pass(const orc_geom_t *g, const uint8_t *const *src, uint8_t *const *dst,
                     const int64_t *store_slots, const int64_t *load_slots, int64_t n_chunks,
                     uint8_t *pool, uint8_t *buffers, int n_threads, int retrieve)
{
    if (n_threads < 1 || n_threads > 1024) return -1.0;
    pthread_t *th = (pthread_t *)calloc((size_t)n_threads, sizeof *th);
    job_t *jobs = (job_t *)calloc((size_t)n_threads, sizeof *jobs);
    if (!th || !jobs) {
        free(th);
        free(jobs);
        return -1.0;
    }
    const int64_t cb = orc_chunk_bytes(g);
    for (int t = 0; t < n_threads; t++) {
        job_t j = {g, src, dst, store_slots, load_slots, n_chunks, pool, buffers + (int64_t)t * cb,
                   t, n_threads, retrieve, 0};
        jobs[t] = j;
    }
    int bad = 0, started = 0;
    const double t0 = now();
    for (int t = 0; t < n_threads; t++) {
        if (pthread_create(&th[t], NULL, run, &jobs[t]) != 0) {
            bad = 1;
            break;
        }
        started++;
    }
    for (int t = 0; t < started; t++) pthread_join(th[t], NULL);
    const double dt = now() - t0;
    for (int t = 0; t < started; t++) bad |= jobs[t].status != 0;
    free(th);
    free(jobs);
    return bad ? -1.0 : dt;
}
