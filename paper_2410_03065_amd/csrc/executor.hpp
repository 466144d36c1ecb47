// Threaded executor of the two-ended race (App. A steps 3-6; Alg. 1): the caller's
// thread is the compute worker, a second thread is the load worker.  Both take their
// decisions from RaceCore under one mutex; a worker that decides to wait sleeps until
// the other side claims or completes something.
#pragma once
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "race_core.hpp"

namespace cake {

// What a worker does with a claimed chunk.  Both calls block until the chunk's KV is
// resident (stream drained) and return 0 or a negative cake_status.
struct Backend {
    virtual ~Backend() {}
    virtual int compute_chunk(int chunk, uint64_t* device_ns) = 0;
    virtual int load_chunk(int chunk) = 0;
    virtual void on_load_completed(int n_loaded_so_far) { (void)n_loaded_so_far; }
    // Progress of the load in flight: ns since it started and bytes the tier has delivered so far.
    virtual bool load_progress(uint64_t* elapsed_ns, uint64_t* bytes_done) { (void)elapsed_ns; (void)bytes_done; return false; }
};

inline uint64_t mono_ns() {
    return uint64_t(std::chrono::duration_cast<std::chrono::nanoseconds>(
                        std::chrono::steady_clock::now().time_since_epoch()).count());
}

// A thread that lives as long as its owner and runs the jobs handed to it one at a time, in the order
// they were handed over: the load worker of every race of a context runs here, and so do the loads
// queued by cake_load_chunk, so that no thread is created on the path whose latency is measured.
class WorkerThread {
public:
    WorkerThread() = default;
    WorkerThread(const WorkerThread&) = delete;
    WorkerThread& operator=(const WorkerThread&) = delete;
    ~WorkerThread() { stop(); }
    // on_start runs once on the new thread before the first job (e.g. binding the thread to a device)
    void start(std::function<void()> on_start) {
        if (th_.joinable()) return;
        th_ = std::thread([this, on_start] {
            if (on_start) on_start();
            std::unique_lock<std::mutex> lk(mu_);
            for (;;) {
                cv_.wait(lk, [&] { return quit_ || !jobs_.empty(); });
                if (jobs_.empty()) return;   // quit, and nothing left to run
                std::function<void()> j = std::move(jobs_.front());
                jobs_.pop_front();
                busy_ = true;
                lk.unlock();
                j();
                lk.lock();
                busy_ = false;
                cv_.notify_all();
            }
        });
    }
    bool running() const { return th_.joinable(); }
    // never blocks: the job runs after those handed over before it
    void submit(std::function<void()> job) {
        std::lock_guard<std::mutex> lk(mu_);
        jobs_.push_back(std::move(job));
        cv_.notify_all();
    }
    // until every job handed over so far has finished
    void wait() {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return !busy_ && jobs_.empty(); });
    }
    void stop() {
        if (!th_.joinable()) return;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return !busy_ && jobs_.empty(); });
            quit_ = true;
            cv_.notify_all();
        }
        th_.join();
    }

private:
    std::thread th_;
    std::mutex mu_;
    std::condition_variable cv_;
    std::deque<std::function<void()>> jobs_;
    bool busy_ = false, quit_ = false;
};

struct Executor {
    RaceCore core;
    std::mutex mu;
    std::condition_variable cv;
    uint64_t gen = 0;  // bumped on every claim / completion
    uint64_t t0 = 0;
    int first_error = CAKE_OK;
    int load_failed_chunk = -1;
    int n_loaded = 0;
    std::vector<cake_chunk_log> chunk_log;
    std::atomic<int32_t>* status = nullptr;  // per chunk cake_chunk_status, owned by the caller
    const int32_t* tok_begin = nullptr;      // per chunk
    const int32_t* tok_count = nullptr;

    uint64_t now() const { return mono_ns() - t0; }

    // call with the mutex held, before planning
    void refresh_load_progress(Backend& be) {
        uint64_t ns = 0, by = 0;
        if (core.w[W_LOAD].busy && be.load_progress(&ns, &by) && by > 0 && ns > 0) { core.load_prog_ns = ns; core.load_prog_bytes = by; }
        else { core.load_prog_ns = core.load_prog_bytes = 0; }
    }

    void worker(int who, Backend& be) {
        std::unique_lock<std::mutex> lk(mu);
        for (;;) {
            int c = -1;
            for (;;) {
                if (first_error != CAKE_OK || core.w[who].retired) return;
                // An empty range ends this worker only once the other side's chunk in flight
                // has landed: a failed load hands its chunk back to the range.
                if (core.range_empty() && !core.w[1 - who].busy) return;
                uint64_t seen = gen;
                refresh_load_progress(be);
                c = core.range_empty() ? -1 : core.decide(who, now());
                if (c >= 0) break;
                cv.wait(lk, [&] { return gen != seen || first_error != CAKE_OK; });
            }
            ++gen;
            cv.notify_all();
            uint64_t start = core.w[who].started;
            if (status) status[c].store(who == W_COMPUTE ? CAKE_CHUNK_COMPUTING : CAKE_CHUNK_LOADING);
            lk.unlock();
            uint64_t dev_ns = 0;
            int rc = (who == W_COMPUTE) ? be.compute_chunk(c, &dev_ns) : be.load_chunk(c);
            lk.lock();
            uint64_t end = now();
            bool failed = rc != CAKE_OK;
            core.complete(who, end, failed);
            if (failed) {
                if (status) status[c].store(CAKE_CHUNK_EMPTY);
                if (who == W_LOAD && !core.w[W_COMPUTE].retired) load_failed_chunk = c;
                else if (first_error == CAKE_OK) first_error = rc;
            } else {
                cake_chunk_log& cl = chunk_log[c];
                cl.source = who;
                cl.tok_begin = tok_begin[c];
                cl.tok_count = tok_count[c];
                cl.start_ns = start;
                cl.end_ns = end;
                cl.work = (who == W_COMPUTE) ? core.flops[c] : core.bytes[c];
                cl.device_ns = dev_ns;
                if (status) status[c].store(CAKE_CHUNK_RESIDENT);
                if (who == W_LOAD) {
                    ++n_loaded;
                    be.on_load_completed(n_loaded);
                }
            }
            ++gen;
            cv.notify_all();
            if (failed) return;
        }
    }

    // Runs the race to the end.  Returns the first hard error, or CAKE_OK.  The load worker runs on
    // `pool` if one is given and running, else on a thread of its own.
    int run(Backend& be, uint64_t* ttft_ns, WorkerThread* pool = nullptr) {
        chunk_log.assign(size_t(core.n), cake_chunk_log{CAKE_SRC_NONE, 0, 0, 0, 0, 0, 0});
        first_error = CAKE_OK;
        load_failed_chunk = -1;
        n_loaded = 0;
        gen = 0;
        t0 = mono_ns();
        std::thread loader;
        const bool have_loader = !core.w[W_LOAD].retired && core.n > 0;
        const bool pooled = have_loader && pool && pool->running();
        if (pooled) pool->submit([&] { worker(W_LOAD, be); });
        else if (have_loader) loader = std::thread([&] { worker(W_LOAD, be); });
        if (!core.w[W_COMPUTE].retired) worker(W_COMPUTE, be);
        if (pooled) pool->wait();
        else if (have_loader) loader.join();
        *ttft_ns = now();
        if (first_error != CAKE_OK) return first_error;
        std::lock_guard<std::mutex> g(mu);
        if (!core.range_empty()) return load_failed_chunk >= 0 ? CAKE_E_STORE_MISS : CAKE_E_STATE;
        return CAKE_OK;
    }
};

}  // namespace cake
