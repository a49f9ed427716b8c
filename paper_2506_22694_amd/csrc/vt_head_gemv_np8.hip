// Instantiations of the small-n draft-step kernel for NP = 8 padded hidden rows.
#include "vt_head_gemv_kernel.h"

namespace vt {

hipError_t launch_head_gemv_np8(bool bf16, int CS, const StepArgs &a, size_t lds, hipStream_t st) {
    if (bf16) {
        switch (CS) {
            case 1: return launch_gemv_inst<true, 8, 1>(a, lds, st);
            case 2: return launch_gemv_inst<true, 8, 2>(a, lds, st);
            case 3: return launch_gemv_inst<true, 8, 3>(a, lds, st);
            default: return hipErrorInvalidValue;
        }
    }
    switch (CS) {
        case 1: return launch_gemv_inst<false, 8, 1>(a, lds, st);
        case 2: return launch_gemv_inst<false, 8, 2>(a, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace vt
