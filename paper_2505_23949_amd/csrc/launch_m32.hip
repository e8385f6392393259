// Kernels for 32 x 32 blocks (see launch.hpp).
#include "launch_impl.hpp"

namespace tsenor_dev {
template bool launch_block_kernels<32>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
}
