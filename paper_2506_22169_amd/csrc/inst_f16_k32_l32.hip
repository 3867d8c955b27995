// Kernel instantiations: f16 inputs, K = 32, L = 32.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 32, 32, f16_32_32)
