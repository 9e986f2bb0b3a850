// A whole tuning run on the GPU (Alg. 1): ask -> instantiate the generation concurrently on
// host threads -> time each child on the one GPU -> parity gate -> tell.
#include <atomic>
#include <chrono>
#include <cmath>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

#include "kernel.hpp"
#include "tuner.hpp"

using namespace opevo;

namespace {

struct Child {
    opevo_kernel *kernel = nullptr;
    int status = OPEVO_OK;
    double compile_ms = 0.0;
    std::string error;
    bool done = false;
};

double seconds_since(std::chrono::steady_clock::time_point t0)
{
    return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
}

// Kernels of the NEXT generation, built ahead of time while this generation is compiled and timed.
// Alg. 1 chooses the next children from the top-lambda of everything evaluated so far; late in a run
// most generations leave that set as it is, and then the next children follow from the tuner's state
// alone.  So the run asks a COPY of the tuner -- told this generation's children with fitness 0, i.e.
// "none of them makes the top-lambda" -- for its next children and builds those on spare compile
// workers.  When the real tuner later asks for a configuration that was built ahead, the kernel is
// taken from here; every other guess is thrown away.  The real tuner never sees any of this: the
// trajectory is the one Alg. 1 takes without it.
struct Ahead {
    std::mutex mu;
    std::condition_variable cv;
    int width = 0;
    std::vector<int32_t> cfgs;          // n * width
    std::vector<Child> kids;
    std::vector<char> taken;
    std::atomic<int> next{0};
    std::vector<std::thread> threads;

    int find(const int32_t *cfg) const
    {
        for (size_t i = 0; i < kids.size(); ++i)
            if (!taken[i] && std::memcmp(cfgs.data() + i * width, cfg, sizeof(int32_t) * width) == 0) return int(i);
        return -1;
    }
    bool all_built()
    {
        std::lock_guard<std::mutex> lock(mu);
        for (const Child &c : kids) if (!c.done) return false;
        return true;
    }
    // joins the builders and frees what nobody took
    void finish()
    {
        for (auto &t : threads) t.join();
        threads.clear();
        for (size_t i = 0; i < kids.size(); ++i)
            if (!taken[i] && kids[i].kernel) { opevo_kernel_destroy(kids[i].kernel); kids[i].kernel = nullptr; }
    }
};

}  // namespace

extern "C" int opevo_tune(const opevo_op *op, int variant, const opevo_tune_args *args,
                          int32_t *best_cfg_out, opevo_tune_result *result)
{
    if (!op || !args || !result) return fail(OPEVO_E_ARG, "tune: NULL argument");
    if (!args->a || !args->b || !args->c) return fail(OPEVO_E_ARG, "tune: device pointers a, b, c are required");
    if (args->trials < 1 || args->lambda < 1 || args->rho < 1 || args->samples < 1 || args->warmup < 0)
        return fail(OPEVO_E_ARG, "tune: trials, lambda, rho, samples must be >= 1");
    if (args->ref && args->n_ref_rows > 0) {
        if (!args->ref_row_index || args->ref_row_len < 1 || op->c_elems() % args->ref_row_len != 0)
            return fail(OPEVO_E_ARG, "tune: sampled reference needs row indices and a row length dividing the output");
    }
    std::memset(result, 0, sizeof *result);
    result->best_trial = -1;

    opevo_space *space = nullptr;
    if (int rc = opevo_op_space(op, variant, &space)) return rc;
    opevo_tuner *tuner = nullptr;
    if (int rc = opevo_tuner_create(space, args->lambda, args->rho, args->q, args->seed, &tuner)) {
        opevo_space_destroy(space);
        return rc;
    }
    if (args->mutation != 0) {
        if (int rc = opevo_tuner_set_mutation(tuner, args->mutation)) {
            opevo_tuner_destroy(tuner);
            opevo_space_destroy(space);
            return rc;
        }
    }
    const int w = space->width;
    const int gen_cap = std::max(args->lambda, args->rho);
    const int n_threads = std::max(1, args->compile_threads);
    hipStream_t stream = static_cast<hipStream_t>(args->stream);
    const auto t_start = std::chrono::steady_clock::now();
    std::vector<int32_t> cfgs(size_t(gen_cap) * w);
    std::vector<double> fit(gen_cap);
    int done = 0, rc_final = OPEVO_OK;
    double best = 0.0;
    std::shared_ptr<Ahead> ahead;                 // the guess for the generation that comes next
    std::vector<std::shared_ptr<Ahead>> stale;    // older guesses, joined and freed at the end
    // OPEVO_TUNE_TRACE=1 in the environment: one line on stderr per trial, before its kernel runs,
    // so that the log of a run that died names the configuration that was on the GPU
    const char *trace_env = std::getenv("OPEVO_TUNE_TRACE");
    const bool trace = trace_env && trace_env[0] && trace_env[0] != '0';

    while (done < args->trials) {
        const int n = tuner->ask(cfgs.data(), args->trials - done);
        if (n == 0) break;   // space exhausted

        // ---- instantiate the children concurrently (host threads), consume them in order
        std::vector<Child> kids(n);
        std::mutex mu;
        std::condition_variable cv;
        std::atomic<int> next(0);
        const auto t_compile = std::chrono::steady_clock::now();
        // children that were built ahead during the previous generation (possibly still being built)
        std::vector<int> from_ahead(n, -1);
        std::shared_ptr<Ahead> prev = ahead;
        if (prev)
            for (int i = 0; i < n; ++i) {
                const int j = prev->find(cfgs.data() + size_t(i) * w);
                if (j >= 0) { from_ahead[i] = j; prev->taken[j] = 1; }
            }
        // guess the next generation and start building it on the spare compile workers
        ahead.reset();
        if (args->speculate_threads > 0 && done + n < args->trials) {
            opevo_tuner guess(*tuner);
            std::vector<double> zeros(n, 0.0);
            guess.tell(cfgs.data(), zeros.data(), n);
            auto a = std::make_shared<Ahead>();
            a->width = w;
            a->cfgs.resize(size_t(gen_cap) * w);
            const int m = guess.ask(a->cfgs.data(), args->trials - done - n);
            if (m > 0) {
                a->kids.resize(m);
                a->taken.assign(m, 0);
                Ahead *ap = a.get();
                auto builder = [ap, op, variant, m, w]() {
                    for (;;) {
                        const int i = ap->next.fetch_add(1);
                        if (i >= m) return;
                        Child c;
                        c.status = build_kernel(*op, variant, ap->cfgs.data() + size_t(i) * w, &c.kernel, &c.compile_ms);
                        if (c.status != OPEVO_OK) c.error = last_error();
                        c.done = true;
                        {
                            std::lock_guard<std::mutex> lock(ap->mu);
                            ap->kids[i] = std::move(c);
                        }
                        ap->cv.notify_all();
                    }
                };
                for (int t = 0; t < std::min(args->speculate_threads, m); ++t) a->threads.emplace_back(builder);
                ahead = a;
            }
        }
        auto worker = [&]() {
            for (;;) {
                const int i = next.fetch_add(1);
                if (i >= n) return;
                if (from_ahead[i] >= 0) continue;       // comes from the previous generation's guess
                Child c;
                c.status = build_kernel(*op, variant, cfgs.data() + size_t(i) * w, &c.kernel, &c.compile_ms);
                if (c.status != OPEVO_OK) c.error = last_error();
                c.done = true;
                {
                    std::lock_guard<std::mutex> lock(mu);
                    kids[i] = std::move(c);
                }
                cv.notify_all();
            }
        };
        std::vector<std::thread> pool;
        for (int t = 0; t < std::min(n_threads, n); ++t) pool.emplace_back(worker);

        for (int i = 0; i < n; ++i) {
            if (from_ahead[i] >= 0) {
                std::unique_lock<std::mutex> lock(prev->mu);
                prev->cv.wait(lock, [&] { return prev->kids[from_ahead[i]].done; });
                kids[i] = std::move(prev->kids[from_ahead[i]]);
                prev->kids[from_ahead[i]].kernel = nullptr;
                result->n_built_ahead++;
            } else {
                std::unique_lock<std::mutex> lock(mu);
                cv.wait(lock, [&] { return kids[i].done; });
            }
            Child &c = kids[i];
            double tflops = 0.0, ms = 0.0;
            int status = c.status;
            // the build ran on a worker thread: its message becomes this thread's last error, so that the
            // caller of opevo_tune (and the trace) can read why the latest failed member failed
            if (status != OPEVO_OK && !c.error.empty()) set_error("%s", c.error.c_str());
            if (trace) {
                std::fprintf(stderr, "[opevo_tune] trial %d %s: built (status %d, %.0f ms)%s%s\n", done + i,
                             c.kernel ? c.kernel->name.c_str() : "-", status, c.compile_ms,
                             status == OPEVO_OK ? ", running" : ": ", status == OPEVO_OK ? "" : c.error.c_str());
                std::fflush(stderr);
            }
            if (status == OPEVO_OK && rc_final == OPEVO_OK) {
                const auto t_run = std::chrono::steady_clock::now();
                status = time_kernel(c.kernel, args->a, args->b, args->c, stream, args->warmup, args->warmup_ms,
                                     args->launches_per_sample, args->samples, args->trial_timeout_ms, &ms, nullptr);
                if (status == OPEVO_OK && args->ref) {
                    double mx = 0.0, fro = 0.0;
                    if (args->n_ref_rows > 0)
                        status = compare_f32(static_cast<const float *>(args->c), args->ref,
                                             int64_t(args->n_ref_rows) * args->ref_row_len, args->ref_row_index,
                                             args->ref_row_len, stream, &mx, &fro);
                    else
                        status = compare_f32(static_cast<const float *>(args->c), args->ref, op->c_elems(), nullptr, 1,
                                             stream, &mx, &fro);
                    if (status == OPEVO_OK && !(mx <= args->tol_max_scaled && fro <= args->tol_rel_fro)) {
                        status = OPEVO_E_PARITY;
                        set_error("parity: max scaled error %.3g, relative Frobenius error %.3g [%s]", mx, fro,
                                  c.kernel->defines.c_str());
                    }
                }
                result->run_s += seconds_since(t_run);
                if (status == OPEVO_OK && ms > 0.0) tflops = op->flops() / (ms * 1e-3) * 1e-12;
                if (status == OPEVO_E_HIP) {
                    // a failed launch is a property of the configuration; a dead device is not
                    (void)hipGetLastError();
                    if (hipStreamSynchronize(stream) != hipSuccess) rc_final = OPEVO_E_HIP;
                    else status = OPEVO_E_INVALID;
                }
            }
            if (trace || status == OPEVO_E_PARITY) {
                std::fprintf(stderr, "[opevo_tune] trial %d %s: status %d, %.3f ms, %.2f TFLOP/s%s%s\n", done + i,
                             c.kernel ? c.kernel->name.c_str() : "-", status, ms, tflops,
                             status == OPEVO_E_PARITY ? " PARITY FAILURE: " : "",
                             status == OPEVO_E_PARITY ? last_error() : "");
                std::fflush(stderr);
            }
            if (status == OPEVO_E_INVALID) result->n_invalid++;
            else if (status == OPEVO_E_HIPRTC) result->n_compile_fail++;
            else if (status == OPEVO_E_PARITY) result->n_parity_fail++;
            fit[i] = tflops;
            const int t = done + i;
            if (args->cfg_log) std::memcpy(args->cfg_log + size_t(t) * w, cfgs.data() + size_t(i) * w, sizeof(int32_t) * w);
            if (args->fitness_log) args->fitness_log[t] = tflops;
            if (args->status_log) args->status_log[t] = status;
            if (args->compile_ms_log) args->compile_ms_log[t] = c.compile_ms;
            if (args->run_ms_log) args->run_ms_log[t] = ms;
            if (args->wall_s_log) args->wall_s_log[t] = seconds_since(t_start);
            if (tflops > best) {
                best = tflops;
                result->best_trial = t;
                result->best_tflops = tflops;
                result->best_ms = ms;
                if (best_cfg_out) std::memcpy(best_cfg_out, cfgs.data() + size_t(i) * w, sizeof(int32_t) * w);
            }
            opevo_kernel_destroy(c.kernel);
            c.kernel = nullptr;
        }
        for (auto &th : pool) th.join();
        if (prev) stale.push_back(prev);    // its builders may still be busy with guesses nobody asked for
        for (size_t k = 0; k < stale.size();) {   // retire the guesses whose builders have finished
            if (stale[k]->all_built()) { stale[k]->finish(); stale.erase(stale.begin() + k); }
            else ++k;
        }
        result->compile_s += seconds_since(t_compile);
        if (rc_final != OPEVO_OK) break;
        tuner->tell(cfgs.data(), fit.data(), n);
        if (args->progress_every > 0 && (done + n) / args->progress_every != done / args->progress_every) {
            std::fprintf(stderr, "[opevo_tune] %d/%d trials, best %.2f TFLOP/s, %d invalid, %.1f s\n", done + n,
                         args->trials, best, result->n_invalid, seconds_since(t_start));
            std::fflush(stderr);
        }
        done += n;
    }
    if (ahead) stale.push_back(ahead);
    for (auto &a : stale) a->finish();
    // compile_s was measured around the whole generation; what is left after the GPU share
    result->compile_s = std::max(0.0, result->compile_s - result->run_s);
    result->n_trials = done;
    result->wall_s = seconds_since(t_start);
    opevo_tuner_destroy(tuner);
    opevo_space_destroy(space);
    if (rc_final != OPEVO_OK) return fail(rc_final, "tune: the device stopped responding after a failed launch");
    return OPEVO_OK;
}
