// Stand-alone hipRTC compile worker: serves requests on descriptor 3, answers on descriptor 4.
// Started by the library's compile pool; links the ROCm installation's hipRTC, never touches
// the GPU.
#include "pool.hpp"

int main()
{
    opevo::serve_compile_requests(3, 4);
    return 0;
}
