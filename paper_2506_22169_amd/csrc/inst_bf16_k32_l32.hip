// Kernel instantiations: bf16 inputs, K = 32, L = 32.
#include "mcf_inst.h"

#define MCF_X(mb, rg, ns, nj)                                       \
    MCF_ROW(__bf16, MCF_BF16, 32, 32, mb, rg, ns, nj, false, false) \
    MCF_ROW(__bf16, MCF_BF16, 32, 32, mb, rg, ns, nj, false, true)  \
    MCF_ROW(__bf16, MCF_BF16, 32, 32, mb, rg, ns, nj, true, false)  \
    MCF_ROW(__bf16, MCF_BF16, 32, 32, mb, rg, ns, nj, true, true)
#define MCF_ROWS_bf16_32_32 MCF_WAVE_SHAPES(MCF_X)

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 32, 32, bf16_32_32)
