// Kernel instantiations: bf16 inputs, K = 192, L = 192 (rows padded to a pitch of 256 in LDS).
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 192, 192, bf16_192_192)
