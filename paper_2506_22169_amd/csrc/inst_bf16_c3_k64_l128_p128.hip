// Kernel instantiations of the three-GEMM chain: bf16 inputs, K = 64, L = 128, P = 128.
#include "mcf_inst.h"

MCF_DEFINE_CHAIN3_GROUP(__bf16, MCF_BF16, 64, 128, 128, bf16_c3_64_128_128)
