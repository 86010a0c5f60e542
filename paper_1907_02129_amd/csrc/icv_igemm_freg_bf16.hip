// Filter-in-registers kernel: the instantiations for ICV_BF16 tensors, plain output stage.
#include "icv_igemm_freg_kernel.h"

namespace icv {

int launch_freg_bf16(const Geometry& g, const FregArgs& a, int64_t grid, size_t lds, int T, int KS, hipStream_t s)
{
    return launch_freg_instances<ICV_BF16, false>(g, a, grid, lds, T, KS, s);
}

}  // namespace icv
