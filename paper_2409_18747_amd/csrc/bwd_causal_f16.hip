// The bwd causal kernels for IEEE half-precision elements: the same source as the bfloat16 build,
// compiled with the element type switched (see device_common.h).
#define COTTN_ELEM_F16
#include "bwd_causal_bf16.hip"
