// Instantiations of the forward kernel that run all three sweeps in one launch.
#include "fwd_kernel_impl.h"

namespace intattn {
namespace fwdk {
template int launch_shape<1, 2, 0>(const FwdParams &, int, int, hipStream_t);
template int launch_shape<2, 2, 0>(const FwdParams &, int, int, hipStream_t);
} // namespace fwdk
} // namespace intattn
