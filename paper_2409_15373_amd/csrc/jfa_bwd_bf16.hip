#include "jfa_common.h"
namespace jfa {
hipError_t launch_bwd_bf16(const void *, const void *, const void *, const void *, const float *, const float *,
                           const int64_t *, int, int, int, Schedule, Schedule, void *, void *, void *, int,
                           hipStream_t) { return hipErrorNotSupported; }
}
