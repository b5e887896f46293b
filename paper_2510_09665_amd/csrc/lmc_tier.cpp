// A lower tier under the CPU-memory pool, and the zero-copy rule of paper section 5.3
// ("Zero-Copy Operations"): a chunk that is written to several destinations at once is
// not duplicated; every destination holds one count on the shared bytes, reads them where
// they are, and gives its count back when its write completes.  Destinations here are
// directories (a local disk, a mounted remote store), one file per chunk.
// A policy layer on the library's own C ABI (lmc_chunk_acquire / lmc_chunk_release,
// lmc_put_host, lmc_find_slot): no HIP, no access to the context's insides.
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <cerrno>
#include <condition_variable>
#include <cstdio>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/lmc.h"

namespace {

struct Job {
    uint64_t id;
    const uint8_t *bytes;  // the chunk in the pinned pool, held by one count
    int32_t dir;
};

std::string file_name(const std::string &dir, uint64_t id, bool tmp) {
    char hex[40];
    std::snprintf(hex, sizeof hex, "/%016llx.kv%s", static_cast<unsigned long long>(id), tmp ? ".tmp" : "");
    return dir + hex;
}

// Whole buffer to a file under a temporary name, then the final name.  0 or errno.
int write_file(const std::string &dir, uint64_t id, const uint8_t *p, size_t n) {
    const std::string tmp = file_name(dir, id, true), fin = file_name(dir, id, false);
    const int fd = ::open(tmp.c_str(), O_WRONLY | O_CREAT | O_TRUNC | O_CLOEXEC, 0644);
    if (fd < 0) return errno;
    int err = 0;
    size_t done = 0;
    while (done < n) {
        const ssize_t w = ::write(fd, p + done, n - done);
        if (w < 0) {
            if (errno == EINTR) continue;
            err = errno;
            break;
        }
        done += size_t(w);
    }
    if (::close(fd) != 0 && err == 0) err = errno;
    if (err == 0 && ::rename(tmp.c_str(), fin.c_str()) != 0) err = errno;
    if (err != 0) (void)::unlink(tmp.c_str());
    return err;
}

}  // namespace

struct lmc_tier {
    lmc_ctx_t *ctx = nullptr;
    int64_t chunk_bytes = 0;
    std::vector<std::string> dirs;
    std::mutex mu;
    std::condition_variable work, idle;
    std::deque<Job> queue;
    int64_t unfinished = 0;  // queued or being written
    bool stop = false;
    int32_t first_errno = 0;  // of a failed file since the last wait
    int32_t last_errno = 0;   // what lmc_tier_errno reports
    uint64_t files_written = 0, bytes_written = 0, chunks_read = 0;
    std::vector<std::thread> workers;
    std::vector<uint8_t> bounce;  // read direction, under read_mu
    std::mutex read_mu;

    void run() {
        for (;;) {
            Job j;
            {
                std::unique_lock<std::mutex> lk(mu);
                work.wait(lk, [&] { return stop || !queue.empty(); });
                if (queue.empty()) return;  // stop, and nothing left to write
                j = queue.front();
                queue.pop_front();
            }
            const int err = write_file(dirs[size_t(j.dir)], j.id, j.bytes, size_t(chunk_bytes));
            // this destination is done with the bytes, whatever became of the file
            (void)lmc_chunk_release(ctx, j.id);
            std::lock_guard<std::mutex> lk(mu);
            if (err != 0) {
                if (first_errno == 0) first_errno = err;
            } else {
                files_written++;
                bytes_written += uint64_t(chunk_bytes);
            }
            if (--unfinished == 0) idle.notify_all();
        }
    }
};

extern "C" {

lmc_status_t lmc_tier_open(lmc_ctx_t *ctx, const char *const *dirs, int32_t n_dirs, int32_t n_threads,
                           lmc_tier_t **tier_out) {
    if (!ctx || !dirs || n_dirs < 1 || n_dirs > 16 || n_threads < 1 || n_threads > 64 || !tier_out)
        return LMC_ERR_INVAL;
    *tier_out = nullptr;
    for (int32_t d = 0; d < n_dirs; d++) {
        struct stat st;
        if (!dirs[d] || ::stat(dirs[d], &st) != 0 || !S_ISDIR(st.st_mode)) return LMC_ERR_INVAL;
    }
    lmc_tier *t = new (std::nothrow) lmc_tier();
    if (!t) return LMC_ERR_NOMEM;
    t->ctx = ctx;
    t->chunk_bytes = lmc_chunk_bytes(ctx);
    for (int32_t d = 0; d < n_dirs; d++) t->dirs.emplace_back(dirs[d]);
    for (int32_t i = 0; i < n_threads; i++) t->workers.emplace_back([t] { t->run(); });
    *tier_out = t;
    return LMC_OK;
}

lmc_status_t lmc_tier_close(lmc_tier_t *t) {
    if (!t) return LMC_ERR_INVAL;
    {
        std::lock_guard<std::mutex> lk(t->mu);
        t->stop = true;  // the workers drain the queue first
    }
    t->work.notify_all();
    for (std::thread &w : t->workers) w.join();
    delete t;
    return LMC_OK;
}

lmc_status_t lmc_tier_write(lmc_tier_t *t, const uint64_t *ids, int64_t n) {
    if (!t || n < 0 || (n > 0 && !ids)) return LMC_ERR_INVAL;
    const int32_t nd = int32_t(t->dirs.size());
    // one count per chunk and destination, taken before anything is queued
    std::vector<Job> jobs;
    jobs.reserve(size_t(n) * size_t(nd));
    lmc_status_t rc = LMC_OK;
    for (int64_t i = 0; i < n && rc == LMC_OK; i++)
        for (int32_t d = 0; d < nd && rc == LMC_OK; d++) {
            const void *p = nullptr;
            rc = lmc_chunk_acquire(t->ctx, ids[i], &p);
            if (rc == LMC_OK) jobs.push_back(Job{ids[i], static_cast<const uint8_t *>(p), d});
        }
    if (rc != LMC_OK) {
        for (const Job &j : jobs) (void)lmc_chunk_release(t->ctx, j.id);
        return rc;
    }
    {
        std::lock_guard<std::mutex> lk(t->mu);
        if (t->stop) {
            for (const Job &j : jobs) (void)lmc_chunk_release(t->ctx, j.id);
            return LMC_ERR_INVAL;
        }
        for (const Job &j : jobs) t->queue.push_back(j);
        t->unfinished += int64_t(jobs.size());
    }
    t->work.notify_all();
    return LMC_OK;
}

lmc_status_t lmc_tier_wait(lmc_tier_t *t) {
    if (!t) return LMC_ERR_INVAL;
    std::unique_lock<std::mutex> lk(t->mu);
    t->idle.wait(lk, [&] { return t->unfinished == 0; });
    if (t->first_errno != 0) {
        t->last_errno = t->first_errno;
        t->first_errno = 0;
        return LMC_ERR_IO;
    }
    return LMC_OK;
}

lmc_status_t lmc_tier_lookup(lmc_tier_t *t, int32_t dir, const uint64_t *ids, int64_t n, int64_t *n_hit_out) {
    if (!t || dir < 0 || dir >= int32_t(t->dirs.size()) || n < 0 || (n > 0 && !ids) || !n_hit_out)
        return LMC_ERR_INVAL;
    int64_t k = 0;
    while (k < n && ::access(file_name(t->dirs[size_t(dir)], ids[k], false).c_str(), R_OK) == 0) k++;
    *n_hit_out = k;
    return LMC_OK;
}

lmc_status_t lmc_tier_read(lmc_tier_t *t, int32_t dir, const uint64_t *ids, int64_t n) {
    if (!t || dir < 0 || dir >= int32_t(t->dirs.size()) || n < 0 || (n > 0 && !ids)) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> rl(t->read_mu);
    t->bounce.resize(size_t(t->chunk_bytes));
    for (int64_t i = 0; i < n; i++) {
        int64_t slot = -1;
        if (lmc_find_slot(t->ctx, ids[i], &slot) == LMC_OK) continue;  // already in the pool
        const int fd = ::open(file_name(t->dirs[size_t(dir)], ids[i], false).c_str(), O_RDONLY | O_CLOEXEC);
        if (fd < 0) {
            if (errno == ENOENT) return LMC_ERR_MISS;
            t->last_errno = errno;
            return LMC_ERR_IO;
        }
        size_t done = 0;
        int err = 0;
        while (done < t->bounce.size()) {
            const ssize_t r = ::read(fd, t->bounce.data() + done, t->bounce.size() - done);
            if (r < 0 && errno == EINTR) continue;
            if (r <= 0) {
                err = r < 0 ? errno : EIO;  // a short file is an error too
                break;
            }
            done += size_t(r);
        }
        (void)::close(fd);
        if (err != 0) {
            t->last_errno = err;
            return LMC_ERR_IO;
        }
        const lmc_status_t rc = lmc_put_host(t->ctx, &ids[i], 1, t->bounce.data());
        if (rc != LMC_OK) return rc;
        std::lock_guard<std::mutex> lk(t->mu);
        t->chunks_read++;
    }
    return LMC_OK;
}

int32_t lmc_tier_errno(const lmc_tier_t *t) { return t ? t->last_errno : 0; }

lmc_status_t lmc_tier_get_stats(lmc_tier_t *t, uint64_t *files_written, uint64_t *bytes_written,
                                uint64_t *chunks_read) {
    if (!t) return LMC_ERR_INVAL;
    std::lock_guard<std::mutex> lk(t->mu);
    if (files_written) *files_written = t->files_written;
    if (bytes_written) *bytes_written = t->bytes_written;
    if (chunks_read) *chunks_read = t->chunks_read;
    return LMC_OK;
}

}  // extern "C"
