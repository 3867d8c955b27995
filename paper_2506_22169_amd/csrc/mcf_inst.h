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

// Arrangements built for the kernels with a k loop inside the block (T_K < K).
#define MCF_KSPLIT_SHAPES(X) \
    X(1, 4, 1, 1)            \
    X(1, 2, 2, 1)            \
    X(1, 1, 4, 1)            \
    X(1, 1, 2, 1)            \
    X(1, 1, 2, 2)            \
    X(1, 4, 2, 1)            \
    X(1, 2, 2, 2)            \
    X(1, 1, 4, 2)            \
    X(1, 2, 4, 1)            \
    X(1, 1, 8, 1)            \
    X(2, 2, 2, 1)            \
    X(2, 1, 4, 1)

// Arrangements built for the three-GEMM chain.
#define MCF_CHAIN3_SHAPES(X) \
    X(1, 4, 1, 1)            \
    X(1, 4, 1, 2)            \
    X(1, 8, 1, 1)            \
    X(1, 8, 1, 2)            \
    X(2, 4, 1, 1)            \
    X(2, 4, 1, 2)            \
    X(1, 1, 4, 1)            \
    X(1, 2, 2, 1)            \
    X(1, 2, 2, 2)            \
    X(1, 4, 2, 1)            \
    X(1, 4, 2, 2)            \
    X(2, 2, 2, 2)            \
    X(2, 2, 4, 1)            \
    X(2, 4, 2, 1)            \
    X(2, 4, 2, 2)

namespace mcf {

// The variant table of one (dtype, K, L) group; arrangements that cannot exist for this
// (K, L) have a null launcher.  KSPLIT: K is the chunk T_K of a k loop inside the block.
template <typename T, int DT, int K, int L, bool KSPLIT>
const Variant *group_table(int *count) {
#define MCF_ROW(mb, rg, ns, nj, sm, bkc) \
    {DT, K, L, mb, rg, ns, nj, sm, bkc, KSPLIT, 0, launcher_or_null<T, K, L, mb, rg, ns, nj, sm, bkc, KSPLIT>()},
#define MCF_X(mb, rg, ns, nj)             \
    MCF_ROW(mb, rg, ns, nj, false, false) \
    MCF_ROW(mb, rg, ns, nj, false, true)  \
    MCF_ROW(mb, rg, ns, nj, true, false)  \
    MCF_ROW(mb, rg, ns, nj, true, true)
    if constexpr (KSPLIT) {
        static const Variant table[] = {MCF_KSPLIT_SHAPES(MCF_X)};
        *count = (int)(sizeof(table) / sizeof(table[0]));
        return table;
    } else {
        static const Variant table[] = {MCF_WAVE_SHAPES(MCF_X)};
        *count = (int)(sizeof(table) / sizeof(table[0]));
        return table;
    }
#undef MCF_X
#undef MCF_ROW
}

// The variant table of one (dtype, K, L, P) group of the three-GEMM chain.
template <typename T, int DT, int K, int L, int P>
const Variant *group_table3(int *count) {
#define MCF_ROW(mb, rg, ns, nj, sm, bkc) \
    {DT, K, L, mb, rg, ns, nj, sm, bkc, 0, P, launcher_or_null<T, K, L, mb, rg, ns, nj, sm, bkc, false, P>()},
#define MCF_X(mb, rg, ns, nj)             \
    MCF_ROW(mb, rg, ns, nj, false, false) \
    MCF_ROW(mb, rg, ns, nj, false, true)  \
    MCF_ROW(mb, rg, ns, nj, true, false)  \
    MCF_ROW(mb, rg, ns, nj, true, true)
    static const Variant table[] = {MCF_CHAIN3_SHAPES(MCF_X)};
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
#undef MCF_X
#undef MCF_ROW
}

} // namespace mcf

// One per instantiation file: defines mcf::variants_<NAME>(int*).
#define MCF_DEFINE_GROUP(T, DT, K, L, NAME)                                                        \
    namespace mcf {                                                                                \
    const Variant *variants_##NAME(int *count) { return group_table<T, DT, K, L, false>(count); }  \
    }
#define MCF_DEFINE_CHAIN3_GROUP(T, DT, K, L, P, NAME)                                              \
    namespace mcf {                                                                                \
    const Variant *variants_##NAME(int *count) { return group_table3<T, DT, K, L, P>(count); }     \
    }
#define MCF_DEFINE_KSPLIT_GROUP(T, DT, TK, L, NAME)                                                \
    namespace mcf {                                                                                \
    const Variant *variants_##NAME(int *count) { return group_table<T, DT, TK, L, true>(count); }  \
    }
