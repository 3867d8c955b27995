// Kernel instantiations: bf16 inputs, K = 64, L = 64.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 64, 64, bf16_64_64)
