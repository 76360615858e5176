// Memory-system measurements of the current device (sam_membench.hip).
#pragma once
#include <stdint.h>

#include <string>

namespace sam {

// kind as SAM_MEMBENCH_* of the C ABI; returns SAM_OK or an error code with a
// message in err
int membench(int32_t kind, int64_t size, int64_t count, int32_t workgroups, double *result,
             std::string &err);

}  // namespace sam
