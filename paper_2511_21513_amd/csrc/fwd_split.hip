// Instantiations of the forward kernel that run sweeps A+B only, and sweep C only.
#include "fwd_kernel_impl.h"

namespace intattn {
namespace fwdk {
template int launch_shape<2, 2, 1>(const FwdParams &, int, int, hipStream_t);
template int launch_shape<1, 2, 2>(const FwdParams &, int, int, hipStream_t);
} // namespace fwdk
} // namespace intattn
