// Kernel instantiations: bf16 inputs, K = 96, L = 96 (rows padded to a pitch of 128 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 96, 96, bf16_96_96)
