// Kernel instantiations: bf16 inputs, K = 160, L = 160 (rows padded to a pitch of 256 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 160, 160, bf16_160_160)
