// Kernel instantiations of the three-GEMM chain: bf16 inputs, K = 128, L = 64, P = 64.
#include "mcf_inst.h"

MCF_DEFINE_CHAIN3_GROUP(__bf16, MCF_BF16, 128, 64, 64, bf16_c3_128_64_64)
