// Kernel instantiations: f16 inputs, K = 128, L = 128.
#include "mcf_inst.h"

#define MCF_X(mb, rg, ns, nj)                                       \
    MCF_ROW(_Float16, MCF_F16, 128, 128, mb, rg, ns, nj, false, false) \
    MCF_ROW(_Float16, MCF_F16, 128, 128, mb, rg, ns, nj, false, true)  \
    MCF_ROW(_Float16, MCF_F16, 128, 128, mb, rg, ns, nj, true, false)  \
    MCF_ROW(_Float16, MCF_F16, 128, 128, mb, rg, ns, nj, true, true)
#define MCF_ROWS_f16_128_128 MCF_WAVE_SHAPES(MCF_X)

MCF_DEFINE_GROUP(_Float16, MCF_F16, 128, 128, f16_128_128)
