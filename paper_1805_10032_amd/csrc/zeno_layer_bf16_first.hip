// Streaming layer kernel, instantiations for bf16 operands without the second product.
#include "zeno_layer_impl.h"

ZENO_LAYER_INSTANCE(bf16_first, true, false)
