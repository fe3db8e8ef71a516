#include "variants.hpp"
#define G355_TU_LIST G355_VARIANTS_FP8_0
#define G355_TU_ES 1
#define G355_TU_NAME kLaunchFp8_0
#include "kernels.inc"
