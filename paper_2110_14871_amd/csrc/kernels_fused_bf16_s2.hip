// Instances of the fused GDWS kernel for bf16 storage, stride 2.
#include "fused_kernel.h"

namespace gdws {
namespace fusedk {

int launch_fused_bf16_s2(const FusedParams &p, int TW, bool big, int mb, bool nhwc, int npb, bool self, bool tap2,
                          dim3 grid, size_t lds_bytes, hipStream_t s)
{
    return launch_dispatch<GDWS_BF16, 2>(p, TW, big, mb, nhwc, npb, self, tap2, grid, lds_bytes, s);
}

}  // namespace fusedk
}  // namespace gdws
