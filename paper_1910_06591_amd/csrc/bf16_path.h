// bf16 (matrix-core) path: state, support check and per-step kernel sequence.
#pragma once
#include <hip/hip_runtime.h>

#include <string>

#include "plan.h"

namespace seedinf {

struct Bf16State;

inline seed_status_t bf16_supported(const Plan&, std::string& err)
{
    err = "bf16 path not built yet";
    return SEED_ERR_UNSUPPORTED_ARCH;
}
inline seed_status_t bf16_create(const Plan&, const float*, const float*, Bf16State**, std::string& err)
{
    err = "bf16 path not built yet";
    return SEED_ERR_UNSUPPORTED_ARCH;
}
inline void bf16_destroy(Bf16State*) {}
inline seed_status_t bf16_step(Bf16State*, const Plan&, const float*, hipStream_t, int, const uint8_t*, const int32_t*,
                               const float*, const float*, const float*, float*, float*, float*, const float**, int*,
                               std::string& err)
{
    err = "bf16 path not built yet";
    return SEED_ERR_UNSUPPORTED_ARCH;
}
inline seed_status_t bf16_read_intermediate(Bf16State*, const Plan&, int, int, float*, hipStream_t, std::string& err)
{
    err = "bf16 path not built yet";
    return SEED_ERR_UNSUPPORTED_ARCH;
}

}  // namespace seedinf
