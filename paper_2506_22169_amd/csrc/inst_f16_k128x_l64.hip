// Kernel instantiations with a k loop: f16 inputs, K a multiple of T_K = 128, L = 64.
#include "mcf_inst.h"

MCF_DEFINE_KSPLIT_GROUP(_Float16, MCF_F16, 128, 64, f16_k128x_64)
