// Explicit instantiation of the two-wave-per-tile kernels for one (width, head width), bf16.
#include "pair_kernel.h"
namespace longer {
LONGER_PAIR_INSTANTIATE(128,32)
}
