// Kernel instantiations: f16 inputs, K = 64, L = 256.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 64, 256, f16_64_256)
