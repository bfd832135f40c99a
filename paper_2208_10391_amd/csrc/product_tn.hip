// Product kernel instances: the buffer of A holds its transpose, B is stored as it is read.
#include "product_kernel.h"
#include "product_variant.h"

MOM_DEFINE_PRODUCT_VARIANT(tn, true, false)
