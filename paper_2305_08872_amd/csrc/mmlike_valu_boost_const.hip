// VALU tile kernels of the boost task, threshold operand form "const": one translation
// unit per (task, form) so that the tile shapes compile in parallel.
#include "mmlike_valu_impl.h"

namespace amulet {
template hipError_t launch_mmlike_valu_task<2, 2>(int, const MmlikeArgs &, hipStream_t);
}
