// Kernel instantiations: f16 inputs, K = 80, L = 80 (rows padded to a pitch of 128 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 80, 80, f16_80_80)
