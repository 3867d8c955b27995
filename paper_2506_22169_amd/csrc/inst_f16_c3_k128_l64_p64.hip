// Kernel instantiations of the three-GEMM chain: f16 inputs, K = 128, L = 64, P = 64.
#include "mcf_inst.h"

MCF_DEFINE_CHAIN3_GROUP(_Float16, MCF_F16, 128, 64, 64, f16_c3_128_64_64)
