// Kernels of one row variant (see variants.h).
#include "variants.h"
namespace ann {
ANN_DEFINE_ROW_VARIANT(kF16, kIP, 32, 6)
}
