// Kernel instantiations: bf16 inputs, K = 80, L = 80 (rows padded to a pitch of 128 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 80, 80, bf16_80_80)
