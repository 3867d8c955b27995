// Kernel instantiations: bf16 inputs, K = 128, L = 128.
#include "mcf_inst.h"

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 128, 128, bf16_128_128)
