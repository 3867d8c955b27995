// Kernel instantiations: f16 inputs, K = 256, L = 256.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 256, 256, f16_256_256)
