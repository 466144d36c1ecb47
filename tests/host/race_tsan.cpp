// Host-only stress of the threaded executor with a fake backend (sleeps instead of GPU work).
// Built with -fsanitize=thread by tests/test_host_api.py; checks: every chunk produced exactly once,
// computed chunks form a prefix and loaded chunks a suffix, a failing load is recomputed.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <thread>
#include <vector>

#include "../../paper_2410_03065_amd/csrc/executor.hpp"

using namespace cake;

struct FakeBackend : Backend {
    std::vector<std::atomic<int>> produced;
    std::vector<uint64_t> c_us, l_us;
    int fail_chunk;
    FakeBackend(int n, int fail) : produced(n), c_us(n), l_us(n), fail_chunk(fail) {
        for (int i = 0; i < n; ++i) { produced[i] = 0; c_us[i] = 40 + 10 * i; l_us[i] = 120; }
    }
    int compute_chunk(int i, uint64_t* dev) override {
        std::this_thread::sleep_for(std::chrono::microseconds(c_us[i]));
        produced[i]++;
        *dev = c_us[i] * 1000;
        return CAKE_OK;
    }
    int load_chunk(int i) override {
        std::this_thread::sleep_for(std::chrono::microseconds(l_us[i]));
        if (i == fail_chunk) return CAKE_E_STORE_MISS;
        produced[i]++;
        return CAKE_OK;
    }
};

static WorkerThread* g_pool = nullptr;   // the load worker runs here when set, else on a thread per race

static int run_case(int n, int mode, int forced, int fail) {
    std::vector<uint64_t> flops(n), bytes(n);
    std::vector<int32_t> tb(n), tc(n);
    for (int i = 0; i < n; ++i) { flops[i] = 1000 + 250 * i; bytes[i] = 1000; tb[i] = i * 64; tc[i] = 64; }
    std::vector<std::atomic<int32_t>> status(n);
    for (auto& s : status) s = 0;
    Executor ex;
    ex.core.est.prior_c_ns = 40000; ex.core.est.prior_c_flops = 1000;
    ex.core.est.prior_l_ns = 120000; ex.core.est.prior_l_bytes = 1000;
    ex.core.init(n, flops.data(), bytes.data(), mode, forced);
    std::vector<cake_decision_log> log(16 * n + 16);
    ex.core.log = log.data(); ex.core.log_cap = (int)log.size();
    ex.status = status.data(); ex.tok_begin = tb.data(); ex.tok_count = tc.data();
    FakeBackend be(n, fail);
    uint64_t ttft = 0;
    int rc = ex.run(be, &ttft, g_pool);
    if (mode == CAKE_LOAD_ONLY && fail >= 0) return rc == CAKE_E_STORE_MISS ? 0 : 1;
    if (rc != CAKE_OK) { std::printf("case n=%d mode=%d: rc %d\n", n, mode, rc); return 1; }
    bool seen_load = false;
    for (int i = 0; i < n; ++i) {
        if (be.produced[i] != 1) { std::printf("chunk %d produced %d times\n", i, be.produced[i].load()); return 1; }
        int src = ex.chunk_log[i].source;
        if (src == CAKE_SRC_LOAD) seen_load = true;
        else if (src != CAKE_SRC_COMPUTE || seen_load) { std::printf("chunk %d: source order broken\n", i); return 1; }
        if (status[i] != CAKE_CHUNK_RESIDENT) return 1;
    }
    if (fail >= 0 && ex.load_failed_chunk != fail) { std::printf("failure not reported\n"); return 1; }
    return 0;
}

int main() {
    int bad = 0;
    WorkerThread pool;
    std::atomic<int> started{0};
    pool.start([&] { started++; });
    for (int rep = 0; rep < 6; ++rep) {
        g_pool = (rep & 1) ? &pool : nullptr;
        for (int n : {1, 2, 7, 24}) {
            bad += run_case(n, CAKE_BIDIR, 0, -1);
            bad += run_case(n, CAKE_GREEDY, 0, -1);
            bad += run_case(n, CAKE_COMPUTE_ONLY, 0, -1);
            bad += run_case(n, CAKE_LOAD_ONLY, 0, -1);
            bad += run_case(n, CAKE_FORCED_SPLIT, n / 2, -1);
        }
        bad += run_case(24, CAKE_GREEDY, 0, 23);
        bad += run_case(24, CAKE_GREEDY, 0, 20);
        bad += run_case(8, CAKE_LOAD_ONLY, 0, 7);
    }
    g_pool = nullptr;
    pool.stop();
    pool.stop();                                  // a second stop is a no-op
    if (started != 1) { std::printf("start hook ran %d times\n", started.load()); ++bad; }
    std::printf(bad ? "FAILED %d\n" : "ok\n", bad);
    return bad ? 1 : 0;
}
