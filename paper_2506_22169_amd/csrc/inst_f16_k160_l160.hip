// Kernel instantiations: f16 inputs, K = 160, L = 160 (rows padded to a pitch of 256 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 160, 160, f16_160_160)
