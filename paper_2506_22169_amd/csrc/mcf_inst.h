// Instantiation list: which (mb, rg, ns) wave arrangements are built for every (dtype, K, L).
#pragma once
#include "chain_kernel.hpp"

// X(mb, rg, ns): tm = 32*mb*rg rows per block, tn = 32*ns columns per n-iteration.
#define MCF_WAVE_SHAPES(X) \
    X(1, 4, 1)             \
    X(1, 2, 2)             \
    X(1, 1, 4)             \
    X(2, 4, 1)             \
    X(2, 2, 2)             \
    X(1, 2, 1)             \
    X(1, 1, 2)             \
    X(1, 4, 2)

#define MCF_ROW(T, DT, K, L, mb, rg, ns, sm, bkc) \
    {DT, K, L, mb, rg, ns, sm, bkc, &mcf::launch_chain<T, K, L, mb, rg, ns, sm, bkc>},

#define MCF_DEFINE_GROUP(T, DT, K, L, NAME)                                      \
    namespace mcf {                                                              \
    const Variant *variants_##NAME(int *count) {                                 \
        static const Variant table[] = {                                         \
            MCF_ROWS_##NAME                                                      \
        };                                                                       \
        *count = (int)(sizeof(table) / sizeof(table[0]));                        \
        return table;                                                            \
    }                                                                            \
    }
