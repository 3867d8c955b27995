// Kernel instantiations: f16 inputs, K = 128, L = 64.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 128, 64, f16_128_64)
