// Instances of the fused GDWS kernel for f16 storage, stride 1.
#include "fused_kernel.h"

namespace gdws {
namespace fusedk {

int launch_fused_f16_s1(const FusedParams &p, int TW, bool big, int mb, bool nhwc, int npb, bool self, bool tap2,
                          dim3 grid, size_t lds_bytes, hipStream_t s)
{
    return launch_dispatch<GDWS_F16, 1>(p, TW, big, mb, nhwc, npb, self, tap2, grid, lds_bytes, s);
}

}  // namespace fusedk
}  // namespace gdws
