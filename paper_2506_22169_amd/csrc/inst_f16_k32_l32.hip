// Kernel instantiations: f16 inputs, K = 32, L = 32.
#include "mcf_inst.h"

#define MCF_X(mb, rg, ns, nj)                                       \
    MCF_ROW(_Float16, MCF_F16, 32, 32, mb, rg, ns, nj, false, false) \
    MCF_ROW(_Float16, MCF_F16, 32, 32, mb, rg, ns, nj, false, true)  \
    MCF_ROW(_Float16, MCF_F16, 32, 32, mb, rg, ns, nj, true, false)  \
    MCF_ROW(_Float16, MCF_F16, 32, 32, mb, rg, ns, nj, true, true)
#define MCF_ROWS_f16_32_32 MCF_WAVE_SHAPES(MCF_X)

MCF_DEFINE_GROUP(_Float16, MCF_F16, 32, 32, f16_32_32)
