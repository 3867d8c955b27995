// Kernel instantiations: f16 inputs, K = 64, L = 64.
#include "mcf_inst.h"

#define MCF_X(mb, rg, ns, nj)                                       \
    MCF_ROW(_Float16, MCF_F16, 64, 64, mb, rg, ns, nj, false, false) \
    MCF_ROW(_Float16, MCF_F16, 64, 64, mb, rg, ns, nj, false, true)  \
    MCF_ROW(_Float16, MCF_F16, 64, 64, mb, rg, ns, nj, true, false)  \
    MCF_ROW(_Float16, MCF_F16, 64, 64, mb, rg, ns, nj, true, true)
#define MCF_ROWS_f16_64_64 MCF_WAVE_SHAPES(MCF_X)

MCF_DEFINE_GROUP(_Float16, MCF_F16, 64, 64, f16_64_64)
