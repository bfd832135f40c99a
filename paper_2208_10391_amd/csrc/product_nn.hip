// Product kernel instances: A and B both stored as the product reads them.
#include "product_kernel.h"
#include "product_variant.h"

MOM_DEFINE_PRODUCT_VARIANT(nn, false, false)
