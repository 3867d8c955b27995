// Kernel instantiations: f16 inputs, K = 64, L = 64.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 64, 64, f16_64_64)
