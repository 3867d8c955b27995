// Instantiation list: which (mb, rg, ns) wave arrangements are built for every (dtype, K, L).
#pragma once
#include "chain_kernel.hpp"

// X(mb, rg, ns, nj): tm = 32*mb*rg rows per block, tn = 32*ns*nj columns per n-iteration.
#define MCF_WAVE_SHAPES(X) \
    X(1, 4, 1, 1)          \
    X(1, 2, 2, 1)          \
    X(1, 1, 4, 1)          \
    X(2, 4, 1, 1)          \
    X(2, 2, 2, 1)          \
    X(1, 4, 2, 1)          \
    X(1, 4, 1, 2)          \
    X(1, 2, 2, 2)          \
    X(1, 4, 2, 2)          \
    X(2, 4, 1, 2)          \
    X(2, 2, 2, 2)          \
    X(1, 4, 1, 4)          \
    X(2, 2, 4, 1)          \
    X(2, 1, 4, 1)          \
    X(4, 2, 4, 1)          \
    X(4, 1, 4, 1)          \
    X(4, 2, 2, 1)          \
    X(1, 8, 1, 1)          \
    X(1, 8, 1, 2)

#define MCF_ROW(T, DT, K, L, mb, rg, ns, nj, sm, bkc) \
    {DT, K, L, mb, rg, ns, nj, sm, bkc, mcf::launcher_or_null<T, K, L, mb, rg, ns, nj, sm, bkc>()},

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
