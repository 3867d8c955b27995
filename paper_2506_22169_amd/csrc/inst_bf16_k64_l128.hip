// Kernel instantiations: bf16 inputs, K = 64, L = 128.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 64, 128, bf16_64_128)
