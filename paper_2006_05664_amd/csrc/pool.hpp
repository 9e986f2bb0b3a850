// Pool of hipRTC worker processes.
//
// hipRTC serialises compilations inside one process, so concurrent instantiation of a
// generation's children (the "8 CPU threads for compiling" of the paper's set-up, Sec. 6)
// needs separate processes.  Workers are forked from this process (no exec), close every
// inherited descriptor except their two pipe ends, never touch the HIP runtime, and serve
// compile requests (template name + -D options -> gfx950 code object) until their request
// pipe closes.
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

// Starts n workers (idempotent: a running pool is kept).  Returns the number running.
int pool_start(int n);
void pool_stop();
int pool_size();
// Compiles on a free worker (blocks until one is free); in-process if the pool is not running
// or the worker died.
CompileResult pool_compile(const std::string &tmpl, const std::string &defines);

}  // namespace opevo
