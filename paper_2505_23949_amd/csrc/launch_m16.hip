// Kernels for 16 x 16 blocks (see launch.hpp).
#include "launch_impl.hpp"

namespace tsenor_dev {
template bool launch_block_kernels<16>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
}
