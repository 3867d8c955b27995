// Kernel instantiations: bf16 inputs, K = 32, L = 32.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 32, 32, bf16_32_32)
