// Pool of hipRTC worker processes.
//
// hipRTC serialises compilations inside one process, so concurrent instantiation of a
// generation's children (the "8 CPU threads for compiling" of the paper's set-up, Sec. 6)
// needs separate processes.  A worker is the stand-alone executable opevo_rtc_worker next to
// the library (it links the ROCm installation's hipRTC), started with fork + exec while this
// process has not opened the GPU yet; once the GPU is open no exec is done any more and a
// worker is a plain fork of this process that only serves compile requests (it then uses the
// hipRTC this process is bound to).  Either kind closes every inherited descriptor except its
// two pipe ends and never touches the HIP runtime.
#pragma once

#include <string>
#include <vector>

namespace opevo {

struct CompileResult {
    int status = 0;              // OPEVO_OK or OPEVO_E_HIPRTC
    std::vector<char> code;
    std::string log;
    double ms = 0.0;
};

// The one place that calls hipRTC: used in-process and by the workers.
CompileResult compile_source(const std::string &tmpl, const std::string &defines);
// Request loop of a worker: (template name, constants) in, (status, ms, code object, log) out.
void serve_compile_requests(int req_fd, int resp_fd);
// Pipe helpers shared by both ends.
bool write_all(int fd, const void *buf, size_t n);
bool read_all(int fd, void *buf, size_t n);
bool write_str(int fd, const std::string &s);
bool read_str(int fd, std::string &s);

// Starts n workers (idempotent: a running pool is kept).  Returns the number running.
int pool_start(int n);
void pool_stop();
int pool_size();
// 1 if the workers are the stand-alone executable, 0 if forks of this process, -1 if no pool.
int pool_kind();
// seconds > 0: a caller waits no longer than this for a compilation on a worker; an overrunning one is answered
// OPEVO_E_INVALID while the worker finishes it in the background
void pool_set_deadline(double seconds);
// Compiles on a free worker (blocks until one is free); in-process if the pool is not running
// or the worker died.
CompileResult pool_compile(const std::string &tmpl, const std::string &defines);

}  // namespace opevo
