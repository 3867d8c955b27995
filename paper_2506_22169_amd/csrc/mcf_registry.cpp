// Table of every built kernel variant, gathered from the instantiation files.
#include <vector>

#include "mcf_internal.h"

namespace mcf {

#define MCF_GROUPS(X)                                                                                      \
    X(f16_32_32) X(f16_64_64) X(f16_128_128) X(f16_64_128) X(f16_128_64) X(f16_64_256) X(f16_256_256)         \
    X(bf16_32_32) X(bf16_64_64) X(bf16_128_128) X(bf16_64_128) X(bf16_128_64) X(bf16_64_256) X(bf16_256_256)      \
    X(f16_k128x_64) X(f16_k128x_128) X(f16_k128x_256) X(bf16_k128x_64) X(bf16_k128x_128) X(bf16_k128x_256)      \
    X(f16_80_80) X(bf16_80_80) X(f16_96_96) X(bf16_96_96) X(f16_160_160) X(bf16_160_160) X(f16_192_192) X(bf16_192_192)
#define MCF_GROUPS3(X)                                                                                     \
    X(f16_c3_64_64_64) X(f16_c3_128_128_128) X(bf16_c3_64_64_64) X(bf16_c3_128_128_128)                    \
    X(f16_c3_64_128_128) X(f16_c3_128_64_64) X(f16_c3_64_64_128) X(bf16_c3_64_128_128) X(bf16_c3_128_64_64) X(bf16_c3_64_64_128)
#define MCF_DECL(NAME) const Variant *variants_##NAME(int *count);
MCF_GROUPS(MCF_DECL)
MCF_GROUPS3(MCF_DECL)

// Registers / scratch of every kernel as the compiler built it (generated at build time).
struct Resources {
    int dtype, K, L, mb, rg, ns, nj, softmax, b_kcontig, ksplit, P, vgprs, sgprs, scratch_bytes, spills_in_loops;
};
static const Resources kResources[] = {
#include "mcf_resources.inc"
};

#define MCF_ADD(NAME)                                    \
    {                                                    \
        int n = 0;                                       \
        const Variant *v = variants_##NAME(&n);          \
        for (int i = 0; i < n; ++i)                      \
            if (v[i].launch) t.push_back(v[i]);          \
    }
static void attach_resources(std::vector<Variant> &t) {
    for (Variant &v : t) {
        v.vgprs = -1;
        v.scratch_bytes = 0;
        for (const Resources &r : kResources)
            if (r.dtype == v.dtype && r.K == v.K && r.L == v.L && r.mb == v.mb && r.rg == v.rg && r.ns == v.ns &&
                r.nj == v.nj && r.softmax == v.softmax && r.b_kcontig == v.b_kcontig && r.ksplit == v.ksplit && r.P == v.P) {
                v.vgprs = r.vgprs;
                // registers parked in scratch across the n loop (stored before it, fetched after it)
                // cost a block a handful of instructions and do not count; spill code inside a loop does
                v.scratch_bytes = r.spills_in_loops ? r.scratch_bytes : 0;
            }
    }
}

static const std::vector<Variant> &all() {
    static const std::vector<Variant> table = [] {
        std::vector<Variant> t;
        MCF_GROUPS(MCF_ADD)
        attach_resources(t);
        return t;
    }();
    return table;
}

static const std::vector<Variant> &all3() {
    static const std::vector<Variant> table = [] {
        std::vector<Variant> t;
        MCF_GROUPS3(MCF_ADD)
        attach_resources(t);
        return t;
    }();
    return table;
}

const Variant *variants3(int *count) {
    const auto &t = all3();
    *count = (int)t.size();
    return t.data();
}

const Variant *variants(int *count) {
    const auto &t = all();
    *count = (int)t.size();
    return t.data();
}

bool resolve_group(int dtype, int64_t K, int64_t L, int *tk, int *ksplit) {
    int best = 0;
    for (const Variant &v : all()) {
        if (v.dtype != dtype || v.L != L) continue;
        if (!v.ksplit && v.K == K) {
            *tk = v.K; *ksplit = 0;
            return true;
        }
        if (v.ksplit && K > v.K && K % v.K == 0 && v.K > best) best = v.K; // the largest chunk that divides K
    }
    if (!best) return false;
    *tk = best; *ksplit = 1;
    return true;
}

const Variant *find_variant(int dtype, int64_t K, int64_t L, int softmax, int b_kcontig, int mb, int rg, int ns, int nj) {
    int tk = 0, ksplit = 0;
    if (!resolve_group(dtype, K, L, &tk, &ksplit)) return nullptr;
    for (const Variant &v : all())
        if (v.dtype == dtype && v.K == tk && v.L == L && v.ksplit == ksplit && v.softmax == softmax &&
            v.b_kcontig == b_kcontig && v.mb == mb && v.rg == rg && v.ns == ns && v.nj == nj)
            return &v;
    return nullptr;
}

} // namespace mcf
