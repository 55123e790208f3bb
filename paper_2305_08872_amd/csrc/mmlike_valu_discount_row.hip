// VALU tile kernels of the discount task, threshold operand form "row": one translation
// unit per (task, form) so that the tile shapes compile in parallel.
#include "mmlike_valu_impl.h"

namespace amulet {
template hipError_t launch_mmlike_valu_task<1, 1>(int, const MmlikeArgs &, hipStream_t);
}
