// Filter-in-registers kernel: the instantiations for ICV_F32 tensors, plain output stage.
#include "icv_igemm_freg_kernel.h"

namespace icv {

int launch_freg_f32(const Geometry& g, const FregArgs& a, int64_t grid, size_t lds, int T, int KS, hipStream_t s)
{
    return launch_freg_instances<ICV_F32, false>(g, a, grid, lds, T, KS, s);
}

}  // namespace icv
