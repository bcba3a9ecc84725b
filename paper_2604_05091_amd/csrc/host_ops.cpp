// Host-side arithmetic: Adam (Algorithm 1, "AdamUpdate" on the CPU; Section 3.1 optimizer
// update phase), bf16 conversion of the weights that StreamIn transfers, rotary tables.
#include "host_ops.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <atomic>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

namespace mt {

int host_threads() {
    static int n = [] {
        int v = 0;
        if (const char *e = getenv("MT_HOST_THREADS")) v = atoi(e);
        if (v <= 0) v = (int)std::thread::hardware_concurrency();
        if (v <= 0) v = 1;
        if (v > 128) v = 128;
        return v;
    }();
    return n;
}

namespace {

// Fork-join pool: host_threads() - 1 workers created on first use and kept for the life of the process (spawning
// 15 threads per call costs ~0.2 ms, a third of the Adam update of a 4 M-element tensor).  One job at a time;
// a caller that finds the pool busy (the optimizer thread and the weight-packing thread can overlap) falls back
// to threads of its own.  A job is a range cut into chunks that the threads take from a shared counter: inside a
// training step the cores are also running the launching thread, the copy workers and the driver's own threads,
// and with one fixed share per thread the whole job waited for whichever thread had lost its core.
struct ChunkedJob {
    const std::function<void(size_t, size_t)> *fn;
    size_t n, chunk;
    std::atomic<size_t> next{0};
    void drain() {
        for (;;) {
            const size_t b = next.fetch_add(1, std::memory_order_relaxed) * chunk;
            if (b >= n) return;
            (*fn)(b, b + chunk < n ? b + chunk : n);
        }
    }
};

class ForkJoinPool {
  public:
    ForkJoinPool() {
        const int n = host_threads() - 1;
        for (int i = 0; i < n; ++i) workers_.emplace_back([this] { work(); });
    }
    ~ForkJoinPool() {
        {
            std::lock_guard<std::mutex> lk(mu_);
            stop_ = true;
        }
        cv_work_.notify_all();
        for (auto &t : workers_) t.join();
    }
    bool try_run(ChunkedJob &job) {
        if (workers_.empty() || !job_mu_.try_lock()) return false;
        {
            std::lock_guard<std::mutex> lk(mu_);
            job_ = &job;
            pending_ = (int)workers_.size();
            ++gen_;
        }
        cv_work_.notify_all();
        job.drain();
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_done_.wait(lk, [this] { return pending_ == 0; });
        }
        job_mu_.unlock();
        return true;
    }

  private:
    void work() {
        uint64_t seen = 0;
        for (;;) {
            std::unique_lock<std::mutex> lk(mu_);
            cv_work_.wait(lk, [&] { return stop_ || gen_ != seen; });
            if (stop_) return;
            seen = gen_;
            ChunkedJob *job = job_;
            lk.unlock();
            job->drain();
            lk.lock();
            if (--pending_ == 0) cv_done_.notify_one();
        }
    }
    std::vector<std::thread> workers_;
    std::mutex mu_, job_mu_;
    std::condition_variable cv_work_, cv_done_;
    ChunkedJob *job_ = nullptr;
    uint64_t gen_ = 0;
    int pending_ = 0;
    bool stop_ = false;
};

}  // namespace

void parallel_for(size_t n, size_t min_chunk, const std::function<void(size_t, size_t)> &fn) {
    if (n == 0) return;
    size_t nt = (size_t)host_threads();
    if (min_chunk == 0) min_chunk = 1;
    const size_t max_by_size = (n + min_chunk - 1) / min_chunk;
    if (nt > max_by_size) nt = max_by_size;
    if (nt <= 1) {
        fn(0, n);
        return;
    }
    // about 16 chunks per thread, none below min_chunk; boundaries on multiples of 64 elements so vector loops
    // stay aligned
    size_t chunk = (n + nt * 16 - 1) / (nt * 16);
    if (chunk < min_chunk) chunk = min_chunk;
    chunk = (chunk + 63) & ~(size_t)63;
    ChunkedJob job;
    job.fn = &fn;
    job.n = n;
    job.chunk = chunk;
    static ForkJoinPool pool;
    if (pool.try_run(job)) return;
    std::vector<std::thread> th;
    th.reserve(nt);
    for (size_t t = 1; t < nt; ++t) th.emplace_back([&job] { job.drain(); });
    job.drain();
    for (auto &t : th) t.join();
}

namespace {

inline uint16_t bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__attribute__((target_clones("avx512f", "avx2", "default"))) void cvt_chunk(uint16_t *out, const float *in,
                                                                           size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = bf16_rne(in[i]);
}

__attribute__((target_clones("avx512f", "avx2", "default"))) void adam_chunk(float *p, const float *g, float *m,
                                                                            float *v, uint16_t *shadow, size_t n,
                                                                            float decay, float lr, float b1, float b2,
                                                                            float eps, float inv_c1, float inv_c2) {
    const float ob1 = 1.0f - b1, ob2 = 1.0f - b2;
    // Blocks of 2048 elements: the update loop and the bf16 conversion loop each vectorise fully on their own
    // (fused into one loop the mixed 32/16-bit stores halve the throughput); the block is still in L1 when
    // the conversion reads it back.
    constexpr size_t kBlock = 2048;
    for (size_t b0 = 0; b0 < n; b0 += kBlock) {
        const size_t b1e = b0 + kBlock < n ? b0 + kBlock : n;
        for (size_t i = b0; i < b1e; ++i) {
            const float gi = g[i];
            const float mi = b1 * m[i] + ob1 * gi;
            const float vi = b2 * v[i] + ob2 * gi * gi;
            const float pi = p[i] * decay - lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
            m[i] = mi;
            v[i] = vi;
            p[i] = pi;
        }
        if (shadow)
            for (size_t i = b0; i < b1e; ++i) shadow[i] = bf16_rne(p[i]);
    }
}

}  // namespace

void host_f32_to_bf16(uint16_t *out, const float *in, size_t n) {
    parallel_for(n, 1 << 16, [&](size_t b, size_t e) { cvt_chunk(out + b, in + b, e - b); });
}

void host_adam(float *p, const float *g, float *m, float *v, uint16_t *shadow, size_t n, float lr, float beta1,
               float beta2, float eps, float wd, int64_t step) {
    const double c1 = 1.0 - pow((double)beta1, (double)step), c2 = 1.0 - pow((double)beta2, (double)step);
    const float inv_c1 = (float)(1.0 / c1), inv_c2 = (float)(1.0 / c2);
    const float decay = (float)(1.0 - (double)lr * (double)wd);
    parallel_for(n, 1 << 16, [&](size_t b, size_t e) {
        adam_chunk(p + b, g + b, m + b, v + b, shadow ? shadow + b : nullptr, e - b, decay, lr, beta1, beta2, eps,
                   inv_c1, inv_c2);
    });
}

void host_zero(void *p, size_t bytes) {
    char *c = (char *)p;
    parallel_for(bytes, 1 << 22, [&](size_t b, size_t e) { memset(c + b, 0, e - b); });
}

void rope_table(float *cs, float *sn, int T, int hd, double base) {
    const int half = hd / 2;
    parallel_for((size_t)T, 256, [&](size_t b, size_t e) {
        for (size_t t = b; t < e; ++t)
            for (int j = 0; j < half; ++j) {
                const double ang = (double)t * pow(base, -2.0 * (double)j / (double)hd);
                cs[t * half + j] = (float)cos(ang);
                sn[t * half + j] = (float)sin(ang);
            }
    });
}

}  // namespace mt
