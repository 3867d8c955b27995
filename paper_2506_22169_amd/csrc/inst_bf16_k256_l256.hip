// Kernel instantiations: bf16 inputs, K = 256, L = 256.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 256, 256, bf16_256_256)
