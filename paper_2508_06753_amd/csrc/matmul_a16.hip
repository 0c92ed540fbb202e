// w2a16 (placeholder until the bf16 MFMA kernels land): reports unsupported.
#include <hip/hip_runtime.h>

#include "w2_internal.h"

namespace w2 {

bool a16_smallm_supports(const A16Args& a) { return a.M >= 1 && a.M <= 16; }

int launch_a16_smallm(const A16Args&, hipStream_t)
{
    set_error("w2_matmul_a16: not implemented");
    return -2;
}

int launch_a16_tiled(const A16Args&, hipStream_t)
{
    set_error("w2_matmul_a16: not implemented");
    return -2;
}

}  // namespace w2
