// Product kernel instances: the buffers of A and of B both hold transposes.
#include "product_kernel.h"
#include "product_variant.h"

MOM_DEFINE_PRODUCT_VARIANT(tt, true, true)
