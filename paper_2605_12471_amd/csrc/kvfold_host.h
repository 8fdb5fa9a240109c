// Host-side helpers shared by the translation units that implement the C ABI.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/kvfold.h"

namespace kvfold {

// Records a HIP failure for kvfold_last_hip_error() of the calling thread, clears the runtime's sticky error and
// returns the status to hand back (KVFOLD_ERR_OOM for an allocation failure, KVFOLD_ERR_HIP otherwise).
int hip_fail(hipError_t e);

}  // namespace kvfold
