// Kernel instantiations: bf16 inputs, K = 128, L = 128.
#include "mcf_inst.h"

#define MCF_X(mb, rg, ns, nj)                                       \
    MCF_ROW(__bf16, MCF_BF16, 128, 128, mb, rg, ns, nj, false, false) \
    MCF_ROW(__bf16, MCF_BF16, 128, 128, mb, rg, ns, nj, false, true)  \
    MCF_ROW(__bf16, MCF_BF16, 128, 128, mb, rg, ns, nj, true, false)  \
    MCF_ROW(__bf16, MCF_BF16, 128, 128, mb, rg, ns, nj, true, true)
#define MCF_ROWS_bf16_128_128 MCF_WAVE_SHAPES(MCF_X)

MCF_DEFINE_GROUP(__bf16, MCF_BF16, 128, 128, bf16_128_128)
