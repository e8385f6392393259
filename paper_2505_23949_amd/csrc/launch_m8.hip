// Kernels for 8 x 8 blocks (see launch.hpp).
#include "launch_impl.hpp"

namespace tsenor_dev {
template bool launch_block_kernels<8>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
}
