#include "variants.hpp"
#define G355_TU_LIST G355_VARIANTS_FP8_1
#define G355_TU_ES 1
#define G355_TU_NAME kLaunchFp8_1
#include "kernels.inc"
