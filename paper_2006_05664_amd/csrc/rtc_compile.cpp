// hipRTC compilation of a kernel template under one set of constants, and the request loop
// of a compile worker.  This file is built into libopevo.so and into the stand-alone worker
// executable (which links the ROCm installation's own hipRTC).
#include "pool.hpp"

#include <cerrno>
#include <chrono>
#include <csignal>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <sstream>
#include <vector>

#include <dirent.h>
#include <unistd.h>

#include <hip/hiprtc.h>

#include "opevo.h"

namespace opevo {

const char *template_source(const char *name);

namespace {
const char *const kFixedOptions[] = {"--offload-arch=gfx950", "-O3", "-std=c++17",
                                     "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                                     "-mllvm", "-pragma-unroll-threshold=400000"};
}

// The fixed options as one string: part of the key under which a code object is cached.
const char *compile_options_tag()
{
    static const std::string tag = [] {
        std::string t;
        for (const char *o : kFixedOptions) t += std::string(o) + " ";
        return t;
    }();
    return tag.c_str();
}

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
    // -pragma-unroll-threshold: the templates keep accumulators and fragments in register arrays and
    // mark every loop over them for full unrolling; the compiler's default size limit for such
    // loops makes it give up on the larger members, which then compile (slowly) into code objects
    // of megabytes that index those arrays through select chains.
    for (const char *o : kFixedOptions) opts.push_back(o);
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

void serve_compile_requests(int req, int resp)
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
}


}  // namespace opevo
