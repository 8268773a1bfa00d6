// bf16 MFMA path (placeholder until the kernels land)
#include "mrt_internal.hpp"
namespace mrt {
hipError_t launch_bf16_stage_r(const KParams&, int, bool, bool, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bf16_stage_l(const KParams&, int, bool, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bf16_dense(const KParams&, int, hipStream_t) { return hipErrorNotSupported; }
}
