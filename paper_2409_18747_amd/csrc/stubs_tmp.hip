#include "launch.h"
namespace cottn {
hipError_t fwd_bidir_bf16(const CausalArgs&) { return hipErrorNotSupported; }
hipError_t bwd_bidir_bf16(const CausalArgs&) { return hipErrorNotSupported; }
hipError_t fwd_causal_f32(const CausalArgs&) { return hipErrorNotSupported; }
hipError_t bwd_causal_f32(const CausalArgs&) { return hipErrorNotSupported; }
hipError_t fwd_bidir_f32(const CausalArgs&) { return hipErrorNotSupported; }
hipError_t bwd_bidir_f32(const CausalArgs&) { return hipErrorNotSupported; }
}
