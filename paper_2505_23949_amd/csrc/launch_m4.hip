// Kernels for 4 x 4 blocks (see launch.hpp).
#include "launch_impl.hpp"

namespace tsenor_dev {
template bool launch_block_kernels<4>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
}
