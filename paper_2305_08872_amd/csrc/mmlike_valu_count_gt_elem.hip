// VALU tile kernels of the count_gt task, threshold operand form "elem": one translation
// unit per (task, form) so that the tile shapes compile in parallel.
#include "mmlike_valu_impl.h"

namespace amulet {
template hipError_t launch_mmlike_valu_task<3, 3>(int, const MmlikeArgs &, hipStream_t);
}
