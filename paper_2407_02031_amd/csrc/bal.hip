// Bounded asynchronous LoRA loading, host side (Section 4.2, "Bounded asynchronous LoRA
// loading (BAL)").  When a request arrives its adapters start loading in the background, one
// loader thread per adapter (the paper loads several LoRAs in parallel), while the base model
// early-starts denoising unpatched.  At every step boundary the denoising loop asks this
// object what to do: as soon as all adapters are loaded it is told to patch (once); at step k,
// the bound, it is held until loading completes.  After the request the caller patches off.
// Pure host logic: the caller owns the copies to the device and the patch launches.
#include "common.hpp"

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

struct sd_bal {
    int n = 0;
    sd_bal_load_fn load = nullptr;
    void* user = nullptr;
    std::vector<std::thread> loaders;
    std::mutex mu;
    std::condition_variable cv;
    int done = 0;            // loaders that have returned
    int failed = 0;          // ... with a non-zero status
    bool started = false, patched = false;
    int patched_at_step = 0;
    double stall_s = 0.0, load_s = 0.0;
    std::chrono::steady_clock::time_point t_start;
};

using sd::set_error;

extern "C" sd_bal* sd_bal_create(int32_t n_adapters, sd_bal_load_fn load, void* user) {
    if (n_adapters < 0 || (n_adapters > 0 && !load)) {
        set_error("bal_create: n_adapters=%d load=%p", n_adapters, (void*)load);
        return nullptr;
    }
    sd_bal* b = new (std::nothrow) sd_bal;
    if (!b) return nullptr;
    b->n = n_adapters;
    b->load = load;
    b->user = user;
    return b;
}

extern "C" int sd_bal_start(sd_bal* b) {
    SD_REQUIRE(b, SD_EINVAL, "bal_start: null handle");
    SD_REQUIRE(!b->started, SD_EINVAL, "bal_start: already started");
    b->started = true;
    b->t_start = std::chrono::steady_clock::now();
    auto finished = [b](bool ok) {
        std::lock_guard<std::mutex> lk(b->mu);
        if (!ok) ++b->failed;
        if (++b->done == b->n)
            b->load_s = std::chrono::duration<double>(std::chrono::steady_clock::now() - b->t_start).count();
        b->cv.notify_all();
    };
    int not_started = 0;
    for (int i = 0; i < b->n; ++i) {
        // nothing may propagate out of an extern "C" function: an adapter whose thread cannot be
        // created counts as a failed, finished load, so the handle still reaches done == n
        try {
            b->loaders.emplace_back([b, i, finished] { finished(b->load(b->user, i) == 0); });
        } catch (...) {
            finished(false);
            ++not_started;
        }
    }
    SD_REQUIRE(not_started == 0, SD_ELOAD, "bal_start: %d of %d loader threads could not be created", not_started, b->n);
    return SD_OK;
}

extern "C" int sd_bal_loaded(sd_bal* b) {
    if (!b) return 0;
    std::lock_guard<std::mutex> lk(b->mu);
    return b->started && b->done == b->n ? 1 : 0;
}

extern "C" int sd_bal_before_step(sd_bal* b, int32_t step, int32_t k, double timeout_s, int32_t* patch_now) {
    SD_REQUIRE(b && patch_now, SD_EINVAL, "bal_before_step: null argument");
    SD_REQUIRE(b->started, SD_EINVAL, "bal_before_step: not started");
    SD_REQUIRE(step >= 1 && k >= 1, SD_EINVAL, "bal_before_step: step=%d k=%d (both count from 1)", step, k);
    *patch_now = 0;
    std::unique_lock<std::mutex> lk(b->mu);
    if (b->patched || b->n == 0) return SD_OK;
    if (b->done < b->n && step >= k) {   // the bound: hold the base model until the adapters are in
        const auto t0 = std::chrono::steady_clock::now();
        const bool ok = b->cv.wait_for(lk, std::chrono::duration<double>(timeout_s > 0 ? timeout_s : 0.0), [b] { return b->done == b->n; });
        b->stall_s += std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
        SD_REQUIRE(ok, SD_ETIMEOUT, "bal_before_step: adapters not loaded %.3f s after the bound (step %d, k %d)", timeout_s, step, k);
    }
    if (b->done == b->n) {
        SD_REQUIRE(b->failed == 0, SD_ELOAD, "bal_before_step: %d of %d adapter loads failed", b->failed, b->n);
        b->patched = true;
        b->patched_at_step = step;
        *patch_now = 1;
    }
    return SD_OK;
}

extern "C" int sd_bal_stats(sd_bal* b, int32_t* patched_at_step, double* stall_seconds, double* load_seconds) {
    SD_REQUIRE(b, SD_EINVAL, "bal_stats: null handle");
    std::lock_guard<std::mutex> lk(b->mu);
    if (patched_at_step) *patched_at_step = b->patched ? b->patched_at_step : 0;
    if (stall_seconds) *stall_seconds = b->stall_s;
    if (load_seconds) *load_seconds = b->done == b->n ? b->load_s : -1.0;
    return SD_OK;
}

extern "C" int sd_bal_finish(sd_bal* b, int32_t* unpatch_due) {
    SD_REQUIRE(b, SD_EINVAL, "bal_finish: null handle");
    for (auto& t : b->loaders)
        if (t.joinable()) t.join();
    b->loaders.clear();
    std::lock_guard<std::mutex> lk(b->mu);
    if (unpatch_due) *unpatch_due = b->patched ? 1 : 0;
    return SD_OK;
}

extern "C" void sd_bal_destroy(sd_bal* b) {
    if (!b) return;
    for (auto& t : b->loaders)
        if (t.joinable()) t.join();
    delete b;
}
