// VALU tile kernels of the discount task: one translation unit per task so the
// tile shapes of the four tasks compile in parallel.
#include "mmlike_valu_impl.h"

namespace amulet {
template hipError_t launch_mmlike_valu_task<1>(int, const MmlikeArgs &, hipStream_t);
}
