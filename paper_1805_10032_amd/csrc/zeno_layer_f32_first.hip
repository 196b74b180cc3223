// Streaming layer kernel, instantiations for fp32 operands without the second product.
#include "zeno_layer_impl.h"

ZENO_LAYER_INSTANCE(f32_first, false, false)
