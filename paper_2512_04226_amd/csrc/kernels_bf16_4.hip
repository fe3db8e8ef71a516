#include "variants.hpp"
#define G355_TU_LIST G355_VARIANTS_BF16_4
#define G355_TU_ES 2
#define G355_TU_NAME kLaunchBf16_4
#include "kernels.inc"
