// Instantiation list: which (mb, rg, ns, nj) wave arrangements are built for every
// (dtype, K, L), each with and without softmax and for both layouts of B.
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
    X(1, 8, 1, 2)          \
    X(2, 4, 2, 1)          \
    X(2, 4, 2, 2)

namespace mcf {

// The variant table of one (dtype, K, L) group; arrangements that cannot exist for this
// (K, L) have a null launcher.
template <typename T, int DT, int K, int L>
const Variant *group_table(int *count) {
#define MCF_ROW(mb, rg, ns, nj, sm, bkc) {DT, K, L, mb, rg, ns, nj, sm, bkc, launcher_or_null<T, K, L, mb, rg, ns, nj, sm, bkc>()},
#define MCF_X(mb, rg, ns, nj)             \
    MCF_ROW(mb, rg, ns, nj, false, false) \
    MCF_ROW(mb, rg, ns, nj, false, true)  \
    MCF_ROW(mb, rg, ns, nj, true, false)  \
    MCF_ROW(mb, rg, ns, nj, true, true)
    static const Variant table[] = {MCF_WAVE_SHAPES(MCF_X)};
#undef MCF_X
#undef MCF_ROW
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

} // namespace mcf

// One per instantiation file: defines mcf::variants_<NAME>(int*).
#define MCF_DEFINE_GROUP(T, DT, K, L, NAME)                                                        \
    namespace mcf {                                                                                \
    const Variant *variants_##NAME(int *count) { return group_table<T, DT, K, L>(count); }         \
    }
