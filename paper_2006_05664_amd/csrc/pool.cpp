// Pool of hipRTC worker processes: see pool.hpp.
#include "pool.hpp"

#include <cerrno>
#include <condition_variable>
#include <csignal>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <thread>

#include <dirent.h>
#include <dlfcn.h>
#include <fcntl.h>
#include <poll.h>
#include <sys/types.h>
#include <sys/wait.h>
#include <unistd.h>

#include "common.hpp"

namespace opevo {

namespace {

struct Worker {
    pid_t pid = -1;
    int to = -1, from = -1;   // request pipe (write end), response pipe (read end)
    bool busy = false, dead = false;
};

std::mutex g_mu;
std::condition_variable g_cv;
std::vector<Worker> g_workers;
int g_kind = -1;
double g_deadline_s = 0.0;        // > 0: a caller waits no longer than this for a compilation on a worker

// Has this process opened the GPU (KFD or a render node)?  Then it must not exec any more.
bool gpu_is_open()
{
    DIR *d = opendir("/proc/self/fd");
    if (!d) return true;   // cannot tell: be careful
    bool open = false;
    while (dirent *e = readdir(d)) {
        if (e->d_name[0] < '0' || e->d_name[0] > '9') continue;
        char link[64], target[256];
        snprintf(link, sizeof link, "/proc/self/fd/%s", e->d_name);
        ssize_t n = readlink(link, target, sizeof target - 1);
        if (n <= 0) continue;
        target[n] = '\0';
        if (strstr(target, "/dev/kfd") || strstr(target, "/dev/dri/")) { open = true; break; }
    }
    closedir(d);
    return open;
}

std::string worker_executable()
{
    Dl_info info;
    if (!dladdr(reinterpret_cast<const void *>(&pool_start), &info) || !info.dli_fname) return "";
    std::string path = info.dli_fname;
    const size_t slash = path.rfind('/');
    path = (slash == std::string::npos ? std::string(".") : path.substr(0, slash)) + "/opevo_rtc_worker";
    return access(path.c_str(), X_OK) == 0 ? path : "";
}

void close_other_fds(int keep_a, int keep_b)
{
    DIR *d = opendir("/proc/self/fd");
    if (!d) return;
    std::vector<int> fds;
    while (dirent *e = readdir(d)) {
        if (e->d_name[0] < '0' || e->d_name[0] > '9') continue;
        const int fd = atoi(e->d_name);
        if (fd > 2 && fd != keep_a && fd != keep_b && fd != dirfd(d)) fds.push_back(fd);
    }
    closedir(d);
    for (int fd : fds) ::close(fd);
}

}  // namespace

int pool_size()
{
    std::lock_guard<std::mutex> lock(g_mu);
    int n = 0;
    for (const Worker &w : g_workers) n += !w.dead;
    return n;
}

int pool_kind()
{
    std::lock_guard<std::mutex> lock(g_mu);
    return g_workers.empty() ? -1 : g_kind;
}

void pool_set_deadline(double seconds)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_deadline_s = seconds;
}

int pool_start(int n)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int alive = 0;
    for (const Worker &w : g_workers) alive += !w.dead;
    if (alive > 0 || n <= 0) return alive;
    if (n > 64) n = 64;
    signal(SIGPIPE, SIG_IGN);
    const std::string exe = gpu_is_open() ? std::string() : worker_executable();
    g_kind = exe.empty() ? 0 : 1;
    // Fork-only workers inherit the open device descriptors until their first action (closing them)
    // has run: keep their number below what a GPU machine allows to hold the device at one time.
    if (exe.empty() && n > 12) n = 12;
    for (int i = 0; i < n; ++i) {
        int req[2], resp[2];
        if (pipe(req) != 0) break;
        if (pipe(resp) != 0) { ::close(req[0]); ::close(req[1]); break; }
        const pid_t pid = fork();
        if (pid < 0) { ::close(req[0]); ::close(req[1]); ::close(resp[0]); ::close(resp[1]); break; }
        if (pid == 0) {
            ::close(req[1]); ::close(resp[0]);
            close_other_fds(req[0], resp[1]);
            if (!exe.empty()) {
                // the worker executable talks on descriptors 3 (requests) and 4 (responses)
                int a = dup(req[0]), b = dup(resp[1]);      // move out of the way of 3 and 4
                while (a <= 4) a = dup(a);
                while (b <= 4) b = dup(b);
                dup2(a, 3); dup2(b, 4);
                close_other_fds(3, 4);
                char *const argv[] = {const_cast<char *>(exe.c_str()), nullptr};
                execv(exe.c_str(), argv);
                _exit(127);
            }
            serve_compile_requests(req[0], resp[1]);
            _exit(0);   // no atexit handlers, no runtime teardown in the child
        }
        ::close(req[0]); ::close(resp[1]);
        Worker w;
        w.pid = pid; w.to = req[1]; w.from = resp[0];
        fcntl(w.to, F_SETFD, FD_CLOEXEC);
        fcntl(w.from, F_SETFD, FD_CLOEXEC);
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
    bool ok = write_str(to, tmpl) && write_str(to, defines);
    // A worker answers only when its compilation has ended.  With a deadline set, wait for the first byte of the
    // answer no longer than that.  hipRTC cannot be interrupted and no process is started once the GPU may be
    // open, so an overrunning compilation is left to finish: the caller is answered at once that the
    // configuration cannot be evaluated (Sec. 4.2: fitness 0), and a detached thread takes the late answer off
    // the pipe and hands the worker back to the pool.
    double deadline_s;
    pid_t pid;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        deadline_s = g_deadline_s;
        pid = g_workers[idx].pid;
    }
    if (ok && deadline_s > 0.0) {
        pollfd pfd = {from, POLLIN, 0};
        int rc;
        do rc = poll(&pfd, 1, int(deadline_s * 1e3)); while (rc < 0 && errno == EINTR);
        if (rc == 0) {
            std::thread([idx, from, pid]() {
                int32_t st = 0;
                double ms = 0.0;
                std::string code, log;
                const bool fine = read_all(from, &st, sizeof st) && read_all(from, &ms, sizeof ms) && read_str(from, code) && read_str(from, log);
                {
                    std::lock_guard<std::mutex> lock(g_mu);
                    if (size_t(idx) < g_workers.size() && g_workers[idx].pid == pid) {   // the pool may have been stopped meanwhile
                        g_workers[idx].busy = false;
                        if (!fine) g_workers[idx].dead = true;
                    }
                }
                g_cv.notify_all();
            }).detach();
            res.status = OPEVO_E_INVALID;
            res.log = "compilation exceeded the deadline of " + std::to_string(deadline_s) + " s";
            return res;
        }
    }
    ok = ok && read_all(from, &status, sizeof status) &&
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

int opevo_compile_pool_deadline(double seconds)
{
    if (!(seconds >= 0.0) || seconds > 1e6) return opevo::fail(OPEVO_E_ARG, "compile_pool_deadline: seconds must be in [0, 1e6]");
    opevo::pool_set_deadline(seconds);
    return OPEVO_OK;
}

int opevo_compile_pool_kind(int *kind)
{
    if (!kind) return opevo::fail(OPEVO_E_ARG, "compile_pool_kind: NULL argument");
    *kind = opevo::pool_kind();
    return OPEVO_OK;
}

}  // extern "C"
