// Kernel instantiations: f16 inputs, K = 96, L = 96 (rows padded to a pitch of 128 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 96, 96, f16_96_96)
