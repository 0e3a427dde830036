// Matrix-core (MFMA) attention kernel over the packed pool -- placeholder until the kernel lands.
#include "polykv_internal.hpp"

namespace polykv {

bool matrix_kernel_supports(int, int) { return false; }

hipError_t launch_attend_matrix(const polykv_pool*, const AttendPlan&, const void*, float*, float*, hipStream_t) {
    return hipErrorNotSupported;
}

}  // namespace polykv
