// Search-space generation and pruning (Sec. III-A to III-C), host only: the 4! deep and the 2
// flat tiling expressions of the two-GEMM chain as trees of loops, where each statement lands and
// how often it runs, what a block is left with once the spatial loops are bound to the block
// index (Rule 1), which of those keep a single partial C tile (Rule 2), how many tile-size
// choices survive the padding and on-chip-memory rules (Rules 3 and 4), and which points of the
// pruned space the built kernels are.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <set>
#include <string>
#include <tuple>
#include <vector>

#include "mcf_internal.h"

namespace mcf {
namespace {

constexpr const char kLoops[] = "mnkh"; // order of the extents arrays of this file's entry points
int loop_index(char c) {
    const char *p = strchr(kLoops, c);
    return (p && c) ? (int)(p - kLoops) : -1;
}

// A tiling expression as a tree: `xy` nests y in x, `(x,y)` runs x then y in one scope.
struct Tree {
    struct Node { char loop; int parent; };
    std::vector<Node> nodes;          // in order of appearance; node 0 is the outermost loop
    std::vector<std::vector<char>> chains; // every outermost-to-innermost chain, in order
    bool ok = false;
};

// nest := loop [ nest | '(' nest { ',' nest } ')' ]
bool parse_nest(const char *s, size_t &i, int parent, Tree &t) {
    if (loop_index(s[i]) < 0) return false;
    for (const Tree::Node &n : t.nodes)
        if (n.loop == s[i]) return false; // a loop appears once
    const int me = (int)t.nodes.size();
    t.nodes.push_back({s[i], parent});
    ++i;
    if (s[i] == '(') {
        ++i;
        for (;;) {
            if (!parse_nest(s, i, me, t)) return false;
            if (s[i] == ')') { ++i; return true; }
            if (s[i] != ',') return false;
            ++i;
        }
    }
    if (loop_index(s[i]) >= 0) return parse_nest(s, i, me, t);
    return true;
}

Tree parse(const char *expr) {
    Tree t;
    if (!expr) return t;
    size_t i = 0;
    if (!parse_nest(expr, i, -1, t) || expr[i] != '\0') return t;
    std::vector<bool> has_child(t.nodes.size(), false);
    for (const Tree::Node &n : t.nodes)
        if (n.parent >= 0) has_child[n.parent] = true;
    for (size_t leaf = 0; leaf < t.nodes.size(); ++leaf) {
        if (has_child[leaf]) continue;
        std::vector<char> chain;
        for (int at = (int)leaf; at >= 0; at = t.nodes[at].parent) chain.push_back(t.nodes[at].loop);
        std::reverse(chain.begin(), chain.end());
        t.chains.push_back(chain);
    }
    t.ok = true;
    return t;
}

bool holds(const std::vector<char> &chain, const char *loops) {
    for (const char *p = loops; *p; ++p)
        if (std::find(chain.begin(), chain.end(), *p) == chain.end()) return false;
    return true;
}

// Sec. III-B: a statement sits in the chain that holds every loop related to it, under the
// rightmost of them; loops of extent 1 are dead nodes and hold nothing; nothing leaves the loops
// bound to the block index.  Returns the product of the extents around it, -1 if no chain fits.
int64_t trips_of(const Tree &t, const char *related, const int64_t ext[4], bool keep_unit, const char *bound) {
    for (const std::vector<char> &chain : t.chains) {
        if (!holds(chain, related)) continue;
        std::vector<char> live;
        for (char l : chain)
            if (keep_unit || ext[loop_index(l)] != 1) live.push_back(l);
        int pos = -1;
        for (int i = 0; i < (int)live.size(); ++i)
            if (strchr(related, live[i]) || strchr(bound, live[i])) pos = i;
        int64_t n = 1;
        for (int i = 0; i <= pos; ++i) n *= ext[loop_index(live[i])];
        return n;
    }
    return -1;
}

struct Statement { const char *tensor_loops, *compute_loops; };
// C_C, C_E, L_A, L_B, L_D, S_E: the loops that index the tensor, the loops of the compute block it serves
constexpr Statement kStatements[6] = {{"mnk", "mnk"}, {"mnh", "mnh"}, {"mk", "mnk"}, {"kn", "mnk"}, {"nh", "mnh"}, {"mh", "mnh"}};

bool is_flat(const char *expr) { return strchr(expr, '(') != nullptr; }

// Rule 1: m and h, the spatial loops of the output, go to the block index.  In a flat expression
// h shares a scope with k (that is what makes it flat: C is computed once and used for every h),
// so there it stays inside the block.
std::string sub_expression(const char *expr) {
    std::string s;
    for (const char *p = expr; *p; ++p)
        if (*p != 'm' && (*p != 'h' || is_flat(expr))) s.push_back(*p);
    return s;
}

// Rule 2: k, the reduction loop of the intermediate tensor, must not enclose n, the spatial loop of
// C a block still runs: the block would hold one partial C tile per n.
bool violates_rule2(const std::string &sub) {
    const Tree t = parse(sub.c_str());
    for (const std::vector<char> &c : t.chains) {
        const auto k = std::find(c.begin(), c.end(), 'k'), n = std::find(c.begin(), c.end(), 'n');
        if (k != c.end() && n != c.end() && k < n) return true;
    }
    return false;
}

std::vector<std::string> all_expressions() {
    std::vector<std::string> out;
    std::string p = "hkmn"; // sorted: next_permutation walks all 24
    do out.push_back(p); while (std::next_permutation(p.begin(), p.end()));
    out.push_back("mn(k,h)");
    out.push_back("nm(k,h)");
    return out;
}

// Rule 3: a dimension that is a power of two takes no padding at all, any other less than 5 %.
bool padding_ok(int64_t dim, int64_t tile) {
    const int64_t padded = (dim + tile - 1) / tile * tile;
    if ((dim & (dim - 1)) == 0) return padded == dim;
    return (double)(padded - dim) / (double)dim < 0.05;
}

} // namespace
} // namespace mcf

using namespace mcf;

extern "C" int mcf_expression(int index, char *out, int cap) {
    static const std::vector<std::string> all = all_expressions();
    if (index < 0 || index >= (int)all.size() || !out || cap <= (int)all[index].size()) return MCF_EINVAL;
    snprintf(out, cap, "%s", all[index].c_str());
    return MCF_OK;
}

extern "C" int mcf_expression_trips(const char *expr, const int64_t extents[4], int flags, int64_t trips[6]) {
    const Tree t = parse(expr);
    if (!t.ok || t.nodes.size() != 4 || !extents || !trips) return MCF_EINVAL;
    for (int i = 0; i < 4; ++i)
        if (extents[i] < 1) return MCF_EINVAL;
    const bool hoist = !(flags & MCF_TRIPS_NO_HOIST), keep_unit = (flags & MCF_TRIPS_KEEP_UNIT_LOOPS) != 0;
    const char *bound = (flags & MCF_TRIPS_BIND_BLOCK) ? (is_flat(expr) ? "m" : "mh") : "";
    for (int s = 0; s < 6; ++s) {
        const char *related = (s < 2 || !hoist) ? kStatements[s].compute_loops : kStatements[s].tensor_loops;
        trips[s] = trips_of(t, related, extents, keep_unit, bound);
        if (trips[s] < 0) return MCF_EINVAL; // the expression splits the loops of a compute block over two scopes
    }
    return MCF_OK;
}

extern "C" int mcf_sub_expression(const char *expr, char *out, int cap, int *passes_rule2) {
    const Tree t = parse(expr);
    if (!t.ok || t.nodes.size() != 4 || !out) return MCF_EINVAL;
    const std::string s = sub_expression(expr);
    if (cap <= (int)s.size()) return MCF_EINVAL;
    snprintf(out, cap, "%s", s.c_str());
    if (passes_rule2) *passes_rule2 = violates_rule2(s) ? 0 : 1;
    return MCF_OK;
}

extern "C" int mcf_enumerate_space(const mcf_problem *p, int softmax, int64_t shm_max_bytes, mcf_space_report *out) {
    if (!p || !out || p->M < 1 || p->N < 1 || p->K < 1 || p->L < 1) return MCF_EINVAL;
    if (p->in_dtype != MCF_F16 && p->in_dtype != MCF_BF16) return MCF_EUNSUPPORTED;
    if (shm_max_bytes <= 0) shm_max_bytes = kLdsBytesPerBlock;
    memset(out, 0, sizeof(*out));
    // expressions, Rule 1, Rule 2
    for (const std::string &e : all_expressions()) {
        (is_flat(e.c_str()) ? out->n_flat : out->n_deep) += 1;
        const std::string sub = sub_expression(e.c_str());
        int at = 0;
        while (at < out->n_rule1 && sub != out->sub_expression[at]) ++at;
        if (at == out->n_rule1) {
            if (at == MCF_MAX_SUB_EXPRESSIONS) return MCF_EUNSUPPORTED;
            snprintf(out->sub_expression[at], sizeof(out->sub_expression[at]), "%s", sub.c_str());
            out->sub_kept[at] = violates_rule2(sub) ? 0 : 1;
            out->n_rule2 += out->sub_kept[at];
            ++out->n_rule1;
        }
        ++out->sub_members[at];
    }
    // tile sizes: multiples of 16 up to the dimension (Sec. III-A), Rule 3 per dimension
    const int64_t dims[4] = {p->M, p->N, p->K, p->L};
    std::vector<int64_t> ok[4];
    out->tile_choices = 1;
    for (int d = 0; d < 4; ++d) {
        const int64_t n = (dims[d] + 15) / 16;
        if (dims[d] > (1 << 24)) return MCF_EUNSUPPORTED; // (the survivors are walked one by one below)
        out->tile_choices *= n;
        for (int64_t i = 1; i <= n; ++i)
            if (padding_ok(dims[d], 16 * i)) ok[d].push_back(16 * i);
    }
    out->after_rule3 = (int64_t)ok[0].size() * (int64_t)ok[1].size() * (int64_t)ok[2].size() * (int64_t)ok[3].size();
    if (out->after_rule3 > (1ll << 26)) return MCF_EUNSUPPORTED;
    // the built kernels as points (T_M, T_N, T_K, T_L) of the space
    std::vector<mcf_tiles> cands(mcf_list_candidates(p, softmax, nullptr, 0));
    if (!cands.empty()) mcf_list_candidates(p, softmax, cands.data(), (int)cands.size());
    std::set<std::tuple<int64_t, int64_t, int64_t, int64_t>> built;
    for (const mcf_tiles &t : cands) built.insert(std::make_tuple((int64_t)t.tm, (int64_t)t.tn, (int64_t)t.tk, (int64_t)t.tl));
    // Rule 4: eq. (1) over the tiles of all five tensors, in bytes, against 1.2 x the on-chip memory
    const int64_t es = 2;
    for (int64_t tm : ok[0])
        for (int64_t tn : ok[1])
            for (int64_t tk : ok[2])
                for (int64_t th : ok[3]) {
                    const int64_t shm = es * (tm * tk + tk * tn + tm * tn + tn * th + tm * th);
                    if ((double)shm > 1.2 * (double)shm_max_bytes) continue;
                    ++out->after_rule4;
                    // nk with the h tiles as blocks of their own: a kernel with these four tile sizes;
                    // n(k,h) with the kernels' own h step of 32 columns: a kernel with T_L = L, which
                    // keeps the E tiles of every h in registers
                    if (built.count(std::make_tuple(tm, tn, tk, th))) ++out->built_deep;
                    if (th == 32 && built.count(std::make_tuple(tm, tn, tk, (int64_t)p->L))) ++out->built_flat;
                }
    out->candidates = (int64_t)(out->n_deep + out->n_flat) * out->tile_choices;
    out->candidates_pruned = (int64_t)out->n_rule2 * out->after_rule4;
    return MCF_OK;
}
