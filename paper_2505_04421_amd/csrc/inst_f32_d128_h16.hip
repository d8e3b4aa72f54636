// Explicit instantiation of the block kernels for one (element type, width, head width).
#include "block_kernel.h"
namespace longer {
LONGER_INSTANTIATE(float,128,16)
}
