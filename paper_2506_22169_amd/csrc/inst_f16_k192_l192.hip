// Kernel instantiations: f16 inputs, K = 192, L = 192 (rows padded to a pitch of 256 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(_Float16, MCF_F16, 192, 192, f16_192_192)
