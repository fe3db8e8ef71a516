#include "variants.hpp"
#define G355_TU_LIST G355_VARIANTS_BF16_5
#define G355_TU_ES 2
#define G355_TU_NAME kLaunchBf16_5
#include "kernels.inc"
