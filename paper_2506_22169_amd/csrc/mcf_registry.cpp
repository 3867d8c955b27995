// Table of every built kernel variant, gathered from the instantiation files.
#include <vector>

#include "mcf_internal.h"

namespace mcf {

#define MCF_GROUPS(X)                                                                                      \
    X(f16_32_32) X(f16_64_64) X(f16_128_128) X(f16_64_128) X(f16_128_64) X(f16_64_256) X(f16_256_256)         \
    X(bf16_32_32) X(bf16_64_64) X(bf16_128_128) X(bf16_64_128) X(bf16_128_64) X(bf16_64_256) X(bf16_256_256)
#define MCF_DECL(NAME) const Variant *variants_##NAME(int *count);
MCF_GROUPS(MCF_DECL)

// Registers / scratch of every kernel as the compiler built it (generated at build time).
struct Resources {
    int dtype, K, L, mb, rg, ns, nj, softmax, b_kcontig, vgprs, sgprs, scratch_bytes;
};
static const Resources kResources[] = {
#include "mcf_resources.inc"
};

static const std::vector<Variant> &all() {
    static const std::vector<Variant> table = [] {
        std::vector<Variant> t;
#define MCF_ADD(NAME)                                    \
    {                                                    \
        int n = 0;                                       \
        const Variant *v = variants_##NAME(&n);          \
        for (int i = 0; i < n; ++i)                      \
            if (v[i].launch) t.push_back(v[i]);          \
    }
        MCF_GROUPS(MCF_ADD)
        for (Variant &v : t) {
            v.vgprs = -1;
            v.scratch_bytes = 0;
            for (const Resources &r : kResources)
                if (r.dtype == v.dtype && r.K == v.K && r.L == v.L && r.mb == v.mb && r.rg == v.rg && r.ns == v.ns &&
                    r.nj == v.nj && r.softmax == v.softmax && r.b_kcontig == v.b_kcontig) {
                    v.vgprs = r.vgprs;
                    v.scratch_bytes = r.scratch_bytes;
                }
        }
        return t;
    }();
    return table;
}

const Variant *variants(int *count) {
    const auto &t = all();
    *count = (int)t.size();
    return t.data();
}

bool group_built(int dtype, int K, int L) {
    for (const Variant &v : all())
        if (v.dtype == dtype && v.K == K && v.L == L) return true;
    return false;
}

const Variant *find_variant(int dtype, int K, int L, int softmax, int b_kcontig, int mb, int rg, int ns, int nj) {
    for (const Variant &v : all())
        if (v.dtype == dtype && v.K == K && v.L == L && v.softmax == softmax && v.b_kcontig == b_kcontig &&
            v.mb == mb && v.rg == rg && v.ns == ns && v.nj == nj)
            return &v;
    return nullptr;
}

} // namespace mcf
