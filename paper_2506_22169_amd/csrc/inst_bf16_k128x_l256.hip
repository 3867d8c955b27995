// Kernel instantiations with a k loop: bf16 inputs, K a multiple of T_K = 128, L = 256.
#include "mcf_inst.h"

MCF_DEFINE_KSPLIT_GROUP(__bf16, MCF_BF16, 128, 256, bf16_k128x_256)
