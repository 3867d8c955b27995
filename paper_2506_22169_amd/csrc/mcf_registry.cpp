// Table of every built kernel variant, gathered from the instantiation files.
#include <vector>

#include "mcf_internal.h"

namespace mcf {

#define MCF_GROUPS(X) X(f16_32_32) X(f16_64_64) X(f16_128_128) X(bf16_32_32) X(bf16_64_64) X(bf16_128_128)
#define MCF_DECL(NAME) const Variant *variants_##NAME(int *count);
MCF_GROUPS(MCF_DECL)

static const std::vector<Variant> &all() {
    static const std::vector<Variant> table = [] {
        std::vector<Variant> t;
#define MCF_ADD(NAME)                                    \
    {                                                    \
        int n = 0;                                       \
        const Variant *v = variants_##NAME(&n);          \
        t.insert(t.end(), v, v + n);                     \
    }
        MCF_GROUPS(MCF_ADD)
        return t;
    }();
    return table;
}

const Variant *variants(int *count) {
    const auto &t = all();
    *count = (int)t.size();
    return t.data();
}

const Variant *find_variant(int dtype, int K, int L, int softmax, int b_kcontig, int mb, int rg, int ns) {
    for (const Variant &v : all())
        if (v.dtype == dtype && v.K == K && v.L == L && v.softmax == softmax && v.b_kcontig == b_kcontig &&
            v.mb == mb && v.rg == rg && v.ns == ns)
            return &v;
    return nullptr;
}

} // namespace mcf
