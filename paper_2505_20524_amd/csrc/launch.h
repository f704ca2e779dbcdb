// Host-side helpers shared by the entry points.
#pragma once
#include <hip/hip_runtime.h>
#include "../../include/fog.h"

// Maps the runtime's sticky launch error (if any) to a status code.
static inline fog_status fog_launch_status() { return hipGetLastError() == hipSuccess ? FOG_OK : FOG_ERR_HIP; }
