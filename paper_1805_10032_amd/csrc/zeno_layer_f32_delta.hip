// Streaming layer kernel, instantiations for fp32 operands with the second product.
#include "zeno_layer_impl.h"

ZENO_LAYER_INSTANCE(f32_delta, false, true)
