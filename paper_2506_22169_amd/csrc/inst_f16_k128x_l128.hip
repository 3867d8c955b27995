// Kernel instantiations with a k loop: f16 inputs, K a multiple of T_K = 128, L = 128.
#include "mcf_inst.h"

MCF_DEFINE_KSPLIT_GROUP(_Float16, MCF_F16, 128, 128, f16_k128x_128)
