// Kernel instantiations of the three-GEMM chain: f16 inputs, K = 64, L = 64, P = 128.
#include "mcf_inst.h"

MCF_DEFINE_CHAIN3_GROUP(_Float16, MCF_F16, 64, 64, 128, f16_c3_64_64_128)
