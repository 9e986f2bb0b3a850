// hipRTC compilation, in-process and on a pool of forked worker processes.
#include "pool.hpp"

#include <chrono>
#include <condition_variable>
#include <csignal>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <sstream>

#include <dirent.h>
#include <sys/types.h>
#include <sys/wait.h>
#include <unistd.h>

#include <hip/hiprtc.h>

#include "common.hpp"
#include "kernel.hpp"

namespace opevo {

CompileResult compile_source(const std::string &tmpl, const std::string &defines)
{
    CompileResult res;
    const auto t0 = std::chrono::steady_clock::now();
    const char *prologue = template_source("common");
    const char *body = template_source(tmpl.c_str());
    if (!prologue || !body) {
        res.status = OPEVO_E_ARG;
        res.log = "template " + tmpl + " is not built into the library";
        return res;
    }
    // The -D constants are written into the source as #define lines rather than passed as
    // options: hipRTC force-includes its runtime header first, and short macro names such as N
    // must not be visible while that header is parsed.
    std::string src;
    std::vector<std::string> opts;
    {
        std::istringstream is(defines);
        std::string t;
        while (is >> t) {
            const size_t eq = t.find('=');
            if (t.rfind("-D", 0) == 0 && eq != std::string::npos)
                src += "#define " + t.substr(2, eq - 2) + " " + t.substr(eq + 1) + "\n";
            else
                opts.push_back(t);
        }
    }
    src += std::string(prologue) + "\n" + body;
    hiprtcProgram prog;
    hiprtcResult r = hiprtcCreateProgram(&prog, src.c_str(), (tmpl + ".hip").c_str(), 0, nullptr, nullptr);
    if (r != HIPRTC_SUCCESS) {
        res.status = OPEVO_E_HIPRTC;
        res.log = std::string("hiprtcCreateProgram: ") + hiprtcGetErrorString(r);
        return res;
    }
    opts.insert(opts.end(), {"--offload-arch=gfx950", "-O3", "-std=c++17",
                             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"});
    std::vector<const char *> optv;
    for (const auto &o : opts) optv.push_back(o.c_str());
    r = hiprtcCompileProgram(prog, int(optv.size()), optv.data());
    if (r != HIPRTC_SUCCESS) {
        size_t n = 0;
        hiprtcGetProgramLogSize(prog, &n);
        std::string log(n, '\0');
        if (n) hiprtcGetProgramLog(prog, &log[0]);
        hiprtcDestroyProgram(&prog);
        if (log.size() > 1500) log.resize(1500);
        res.status = OPEVO_E_HIPRTC;
        res.log = std::string(hiprtcGetErrorString(r)) + "\n" + log;
        return res;
    }
    size_t code_size = 0;
    hiprtcGetCodeSize(prog, &code_size);
    res.code.resize(code_size);
    hiprtcGetCode(prog, res.code.data());
    hiprtcDestroyProgram(&prog);
    res.ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return res;
}

namespace {

struct Worker {
    pid_t pid = -1;
    int to = -1, from = -1;   // request pipe (write end), response pipe (read end)
    bool busy = false, dead = false;
};

std::mutex g_mu;
std::condition_variable g_cv;
std::vector<Worker> g_workers;

bool write_all(int fd, const void *buf, size_t n)
{
    const char *p = static_cast<const char *>(buf);
    while (n) {
        ssize_t w = ::write(fd, p, n);
        if (w < 0) { if (errno == EINTR) continue; return false; }
        p += w; n -= size_t(w);
    }
    return true;
}

bool read_all(int fd, void *buf, size_t n)
{
    char *p = static_cast<char *>(buf);
    while (n) {
        ssize_t r = ::read(fd, p, n);
        if (r < 0) { if (errno == EINTR) continue; return false; }
        if (r == 0) return false;
        p += r; n -= size_t(r);
    }
    return true;
}

bool write_str(int fd, const std::string &s)
{
    uint64_t n = s.size();
    return write_all(fd, &n, sizeof n) && (n == 0 || write_all(fd, s.data(), n));
}

bool read_str(int fd, std::string &s)
{
    uint64_t n = 0;
    if (!read_all(fd, &n, sizeof n) || n > (uint64_t(1) << 30)) return false;
    s.resize(n);
    return n == 0 || read_all(fd, &s[0], n);
}

[[noreturn]] void worker_main(int req, int resp)
{
    // drop every inherited descriptor (device files included) except the two pipe ends
    if (DIR *d = opendir("/proc/self/fd")) {
        std::vector<int> fds;
        while (dirent *e = readdir(d)) {
            int fd = atoi(e->d_name);
            if (e->d_name[0] >= '0' && e->d_name[0] <= '9' && fd > 2 && fd != req && fd != resp && fd != dirfd(d))
                fds.push_back(fd);
        }
        closedir(d);
        for (int fd : fds) ::close(fd);
    }
    signal(SIGPIPE, SIG_IGN);
    for (;;) {
        std::string tmpl, defines;
        if (!read_str(req, tmpl) || !read_str(req, defines)) break;
        CompileResult r = compile_source(tmpl, defines);
        int32_t status = r.status;
        std::string code(r.code.begin(), r.code.end());
        if (!write_all(resp, &status, sizeof status) || !write_all(resp, &r.ms, sizeof r.ms) ||
            !write_str(resp, code) || !write_str(resp, r.log))
            break;
    }
    _exit(0);   // no atexit handlers, no runtime teardown in the child
}

}  // namespace

int pool_size()
{
    std::lock_guard<std::mutex> lock(g_mu);
    int n = 0;
    for (const Worker &w : g_workers) n += !w.dead;
    return n;
}

int pool_start(int n)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int alive = 0;
    for (const Worker &w : g_workers) alive += !w.dead;
    if (alive > 0 || n <= 0) return alive;
    if (n > 64) n = 64;
    signal(SIGPIPE, SIG_IGN);
    for (int i = 0; i < n; ++i) {
        int req[2], resp[2];
        if (pipe(req) != 0) break;
        if (pipe(resp) != 0) { ::close(req[0]); ::close(req[1]); break; }
        pid_t pid = fork();
        if (pid < 0) { ::close(req[0]); ::close(req[1]); ::close(resp[0]); ::close(resp[1]); break; }
        if (pid == 0) {
            ::close(req[1]); ::close(resp[0]);
            worker_main(req[0], resp[1]);
        }
        ::close(req[0]); ::close(resp[1]);
        Worker w;
        w.pid = pid; w.to = req[1]; w.from = resp[0];
        g_workers.push_back(w);
    }
    return int(g_workers.size());
}

void pool_stop()
{
    std::vector<Worker> ws;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        ws.swap(g_workers);
    }
    for (Worker &w : ws) {
        if (w.to >= 0) ::close(w.to);       // the worker's read fails and it leaves its loop
        if (w.from >= 0) ::close(w.from);
        if (w.pid > 0) {
            int st = 0;
            waitpid(w.pid, &st, 0);
        }
    }
}

CompileResult pool_compile(const std::string &tmpl, const std::string &defines)
{
    int idx = -1;
    {
        std::unique_lock<std::mutex> lock(g_mu);
        for (;;) {
            bool any_alive = false;
            for (size_t i = 0; i < g_workers.size(); ++i) {
                if (g_workers[i].dead) continue;
                any_alive = true;
                if (!g_workers[i].busy) { idx = int(i); break; }
            }
            if (idx >= 0 || !any_alive) break;
            g_cv.wait(lock);
        }
        if (idx >= 0) g_workers[idx].busy = true;
    }
    if (idx < 0) return compile_source(tmpl, defines);

    int to, from;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        to = g_workers[idx].to; from = g_workers[idx].from;
    }
    CompileResult res;
    int32_t status = 0;
    std::string code;
    const bool ok = write_str(to, tmpl) && write_str(to, defines) && read_all(from, &status, sizeof status) &&
                    read_all(from, &res.ms, sizeof res.ms) && read_str(from, code) && read_str(from, res.log);
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (size_t(idx) < g_workers.size()) {
            g_workers[idx].busy = false;
            if (!ok) g_workers[idx].dead = true;
        }
    }
    g_cv.notify_all();
    if (!ok) return compile_source(tmpl, defines);   // worker died: compile here instead
    res.status = status;
    res.code.assign(code.begin(), code.end());
    return res;
}

}  // namespace opevo

extern "C" {

int opevo_compile_pool_start(int n_workers, int *n_running)
{
    const int n = opevo::pool_start(n_workers);
    if (n_running) *n_running = n;
    if (n_workers > 0 && n == 0) return opevo::fail(OPEVO_E_STATE, "compile_pool_start: could not fork a worker");
    return OPEVO_OK;
}

int opevo_compile_pool_stop(void)
{
    opevo::pool_stop();
    return OPEVO_OK;
}

}  // extern "C"
