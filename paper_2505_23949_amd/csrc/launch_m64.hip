// Kernels for 64 x 64 blocks (see launch.hpp).
#include "launch_impl.hpp"

namespace tsenor_dev {
template bool launch_block_kernels<64>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
}
