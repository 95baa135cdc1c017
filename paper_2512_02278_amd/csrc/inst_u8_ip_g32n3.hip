// Kernels of one row variant (see variants.h).
#include "variants.h"
namespace ann {
ANN_DEFINE_ROW_VARIANT(kU8, kIP, 32, 3)
}
