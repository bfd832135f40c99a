// Product kernel instances: A is stored as it is read, the buffer of B holds its transpose.
#include "product_kernel.h"
#include "product_variant.h"

MOM_DEFINE_PRODUCT_VARIANT(nt, false, true)
