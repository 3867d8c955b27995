// C ABI entry points: argument validation, tile choice, variant dispatch, launch.
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "mcf_internal.h"

namespace mcf {

static thread_local char g_last_error[256] = "";
void set_last_error(const char *msg) { snprintf(g_last_error, sizeof(g_last_error), "%s", msg ? msg : ""); }

static bool all_zero(const int64_t s[3]) { return s[0] == 0 && s[1] == 0 && s[2] == 0; }

static void packed(int64_t out[3], int64_t rows, int64_t cols) {
    out[0] = rows * cols; out[1] = cols; out[2] = 1;
}

// An output [batch, rows, cols] (col stride 1): a batch must end before the next one starts.
static bool batches_disjoint(int64_t batch, int64_t rows, int64_t cols, const int64_t s[3]) {
    if (batch <= 1 || rows <= 0 || cols <= 0) return true;
    if (s[1] > (1ll << 40) || rows > (1ll << 31)) return false; // keeps the product below in range
    return s[0] >= (rows - 1) * s[1] + cols;
}

// Whether 1 + (batch-1) s0 + (rows-1) s1 + (cols-1) s2 stays below 2^60 elements.
static bool span_fits(int64_t batch, int64_t rows, int64_t cols, const int64_t s[3]) {
    const int64_t n[3] = {batch, rows, cols};
    __int128 total = 1;
    for (int d = 0; d < 3; ++d)
        if (n[d] > 1) total += (__int128)(n[d] - 1) * s[d];
    return total < ((__int128)1 << 60);
}

int decode_layout(const mcf_problem *p, Layout *o) {
    if (p->in_dtype != MCF_F16 && p->in_dtype != MCF_BF16) return MCF_EUNSUPPORTED;
    if (p->out_dtype != p->in_dtype && p->out_dtype != MCF_F32) return MCF_EUNSUPPORTED;
    {
        int tk = 0, ksplit = 0;
        if (p->K > 65536 || p->L > 4096 || !resolve_group(p->in_dtype, p->K, p->L, &tk, &ksplit)) return MCF_EUNSUPPORTED;
    }
    if (p->M >= (1ll << 31) - 512 || p->N >= (1ll << 31) - 512 || p->batch >= (1ll << 31)) return MCF_EUNSUPPORTED;
    const int64_t *in[4] = {p->a_stride, p->b_stride, p->d_stride, p->e_stride};
    int64_t *out[4] = {o->sa, o->sb, o->sd, o->se};
    const int64_t rows[4] = {p->M, p->K, p->N, p->M}, cols[4] = {p->K, p->N, p->L, p->L};
    for (int t = 0; t < 4; ++t) {
        if (all_zero(in[t])) packed(out[t], rows[t], cols[t]);
        else memcpy(out[t], in[t], 3 * sizeof(int64_t));
        for (int d = 0; d < 3; ++d)
            if (out[t][d] < 0) return MCF_EINVAL;
    }
    // contiguous index of each tensor
    if (o->sa[2] != 1 || o->sd[2] != 1 || o->se[2] != 1) return MCF_EUNSUPPORTED;
    // B: N contiguous (col stride 1) or K contiguous (row stride 1); N-contiguous wins a tie
    // unless only the K-contiguous kernels can take this N.
    if (o->sb[2] == 1 && !(o->sb[1] == 1 && p->N % 8 != 0)) o->b_kcontig = 0;
    else if (o->sb[1] == 1) o->b_kcontig = 1;
    else return MCF_EUNSUPPORTED;
    // rows must not overlap themselves
    if (p->M > 1 && o->sa[1] < p->K) return MCF_EINVAL;
    if (p->N > 1 && o->sd[1] < p->L) return MCF_EINVAL;
    if (p->M > 1 && o->se[1] < p->L) return MCF_EINVAL;
    if (o->b_kcontig ? (p->N > 1 && o->sb[2] < p->K) : (p->K > 1 && o->sb[1] < p->N)) return MCF_EINVAL;
    // Batches of the output must not overlap one another: blocks of different batches would
    // store to the same rows.  (The inputs are only read: a zero or overlapping batch stride
    // is a legal broadcast there.)
    if (!batches_disjoint(p->batch, p->M, p->L, o->se)) return MCF_EINVAL;
    // and every tensor's extent in elements must fit 64-bit arithmetic with room to spare
    for (int t = 0; t < 4; ++t)
        if (!span_fits(p->batch, rows[t], cols[t], out[t])) return MCF_EUNSUPPORTED;
    // 16-byte vector accesses: leading strides and batch strides in multiples of 8 elements
    const int64_t lead[4] = {o->sa[1], o->b_kcontig ? o->sb[2] : o->sb[1], o->sd[1], o->se[1]};
    const int64_t bstr[4] = {o->sa[0], o->sb[0], o->sd[0], o->se[0]};
    for (int t = 0; t < 4; ++t)
        if (lead[t] % 8 != 0 || bstr[t] % 8 != 0) return MCF_EALIGN;
    if (!o->b_kcontig && p->N % 8 != 0) return MCF_EUNSUPPORTED;
    // the kernels address a tile with 32-bit byte offsets from a 64-bit tile base
    for (int t = 0; t < 4; ++t)
        if (lead[t] >= (1ll << 21)) return MCF_EUNSUPPORTED;
    return MCF_OK;
}

// Elements spanned by a [batch, rows, cols] tensor with the given strides.
static int64_t span(int64_t batch, int64_t rows, int64_t cols, const int64_t s[3]) {
    if (batch == 0 || rows == 0 || cols == 0) return 0;
    return 1 + (batch - 1) * s[0] + (rows - 1) * s[1] + (cols - 1) * s[2];
}

// x: xe elements of xs bytes; y: ye elements of 2 bytes
static bool overlaps(const void *x, int64_t xe, int64_t xs, const void *y, int64_t ye) {
    const char *a = (const char *)x, *b = (const char *)y;
    return xe > 0 && ye > 0 && a < b + 2 * ye && b < a + xs * xe;
}

// Variant of the three-GEMM chain for (dtype, K, L, P) and an arrangement, or nullptr.
static const Variant *find_variant3(int dtype, int64_t K, int64_t L, int64_t P, int softmax, int b_kcontig, int mb, int rg,
                                    int ns, int nj) {
    int n = 0;
    const Variant *v = variants3(&n);
    for (int i = 0; i < n; ++i)
        if (v[i].dtype == dtype && v[i].K == K && v[i].L == L && v[i].P == P && v[i].softmax == softmax &&
            v[i].b_kcontig == b_kcontig && v[i].mb == mb && v[i].rg == rg && v[i].ns == ns && v[i].nj == nj)
            return &v[i];
    return nullptr;
}

// The arrangements built for the three-GEMM chain on (dtype, K, L, P, layout of B), each with
// the model terms of its two-GEMM part (the third GEMM adds the same work to all of them) and
// the LDS bytes of the three-GEMM kernel, in registry order.
int candidates3(const mcf_problem *p, int softmax, int b_kcontig, int64_t P, std::vector<mcf_tiles> *out) {
    int n = 0;
    const Variant *v = variants3(&n);
    out->clear();
    for (int i = 0; i < n; ++i) {
        if (v[i].dtype != p->in_dtype || v[i].K != p->K || v[i].L != p->L || v[i].P != P ||
            v[i].softmax != (softmax != 0) || v[i].b_kcontig != b_kcontig || v[i].scratch_bytes != 0)
            continue;
        mcf_tiles t;
        memset(&t, 0, sizeof(t));
        t.mb = v[i].mb; t.rg = v[i].rg; t.ns = v[i].ns; t.nj = v[i].nj;
        const int st = mcf_eval_tiles(p, softmax, &t);
        if (st != MCF_OK && st != MCF_EINVAL) continue;
        t.lds_bytes = lds_bytes_for(&v[i]); // with the F tile
        out->push_back(t);
    }
    return out->empty() ? MCF_EUNSUPPORTED : MCF_OK;
}

// Tile choice for the three-GEMM chain: the arrangement (among those built for it) whose
// two-GEMM part the model ranks best (ties broken as for the two-GEMM chain); the third GEMM
// adds the same work to each of them.
static int pick3(const mcf_problem *p, int softmax, int b_kcontig, int64_t P, mcf_tiles *out) {
    std::vector<mcf_tiles> c;
    const int st = candidates3(p, softmax, b_kcontig, P, &c);
    if (st != MCF_OK) return st;
    *out = c[0];
    for (const mcf_tiles &t : c)
        if (better(t, *out)) *out = t;
    return MCF_OK;
}

// P == 0: the two-GEMM chain into E[b, M, L].  P > 0: the three-GEMM chain; F[b, L, P] with
// strides fstr (all zero = packed), and E / e_stride describe the output [b, M, P].
static int run(const mcf_problem *p_in, int softmax, float scale, const void *A, const void *B, const void *D, void *E,
               const mcf_tiles *tiles, void *stream, int64_t P = 0, const int64_t *fstr = nullptr,
               const void *F = nullptr, bool causal = false, int64_t causal_off = 0) {
    set_last_error("");
    if (!p_in) return MCF_EINVAL;
    mcf_problem pc = *p_in;
    const mcf_problem *p = &pc;
    if (p->batch < 0 || p->M < 0 || p->K < 0 || p->N < 0 || p->L < 0 || P < 0) return MCF_EINVAL;
    const bool ch3 = P > 0;
    int64_t sg[3] = {0, 0, 0}, sf[3] = {0, 0, 0};
    if (ch3) {
        // A, B, D are laid out as in the two-GEMM chain; the output and F are checked here
        memcpy(sg, p->e_stride, sizeof(sg));
        memset(pc.e_stride, 0, sizeof(pc.e_stride));
        if (all_zero(sg)) packed(sg, p->M, P);
        if (fstr) memcpy(sf, fstr, sizeof(sf));
        if (all_zero(sf)) packed(sf, p->L, P);
        for (int d = 0; d < 3; ++d)
            if (sg[d] < 0 || sf[d] < 0) return MCF_EINVAL;
        if (sg[2] != 1 || sf[2] != 1) return MCF_EUNSUPPORTED;
        if ((p->M > 1 && sg[1] < P) || (p->L > 1 && sf[1] < P)) return MCF_EINVAL;
        if (sg[1] % 8 || sg[0] % 8 || sf[1] % 8 || sf[0] % 8) return MCF_EALIGN;
        if (sg[1] >= (1ll << 21) || sf[1] >= (1ll << 21)) return MCF_EUNSUPPORTED;
        if (!batches_disjoint(p->batch, p->M, P, sg)) return MCF_EINVAL;
        if (!span_fits(p->batch, p->M, P, sg) || !span_fits(p->batch, p->L, P, sf)) return MCF_EUNSUPPORTED;
    }
    Layout lay;
    int st = decode_layout(p, &lay);
    if (st != MCF_OK) return st;
    if (ch3) memcpy(lay.se, sg, sizeof(sg));
    if (softmax && !(scale == scale && fabsf(scale) <= 3.0e38f)) return MCF_EINVAL; // NaN / inf scale
    if (p->batch == 0 || p->M == 0 || p->L == 0) return MCF_OK;
    if (softmax && p->N == 0) return MCF_EINVAL;
    if (!A || !E || (p->N > 0 && (!B || !D)) || (ch3 && !F)) return MCF_EINVAL;

    const int64_t ea = span(p->batch, p->M, p->K, lay.sa), eb = span(p->batch, p->K, p->N, lay.sb);
    const int64_t ed = span(p->batch, p->N, p->L, lay.sd), ee = span(p->batch, p->M, ch3 ? P : p->L, lay.se);
    const int64_t ef = ch3 ? span(p->batch, p->L, P, sf) : 0;
    const int64_t es = p->out_dtype == MCF_F32 ? 4 : 2; // bytes per element of the output
    if (overlaps(E, ee, es, A, ea) || overlaps(E, ee, es, B, eb) || overlaps(E, ee, es, D, ed) || (ch3 && overlaps(E, ee, es, F, ef)))
        return MCF_EINVAL;
    const uintptr_t ptrs[5] = {(uintptr_t)A, (uintptr_t)B, (uintptr_t)D, (uintptr_t)E, (uintptr_t)F};
    for (int t = 0; t < 5; ++t)
        if (ptrs[t] % 16 != 0) return MCF_EALIGN;

    mcf_tiles chosen;
    if (tiles) {
        chosen = *tiles;
    } else {
        st = ch3 ? pick3(p, softmax, lay.b_kcontig, P, &chosen) : mcf_pick_tiles(p, softmax, &chosen);
        if (st != MCF_OK) return st;
    }
    const int64_t tl = ch3 ? p->L : (chosen.tl > 0 ? chosen.tl : p->L);
    if (p->L % tl != 0) return MCF_EINVAL;
    const int nj_ = chosen.nj > 0 ? chosen.nj : 1;
    const Variant *v = ch3 ? find_variant3(p->in_dtype, p->K, p->L, P, softmax, lay.b_kcontig, chosen.mb, chosen.rg, chosen.ns, nj_)
                           : find_variant(p->in_dtype, p->K, tl, softmax, lay.b_kcontig, chosen.mb, chosen.rg, chosen.ns, nj_);
    if (!v) {
        if (!ch3) return tiles ? MCF_EINVAL : MCF_EUNSUPPORTED;
        // no kernels for this (K, L, P) at all, or only this arrangement is missing?
        mcf_tiles any;
        return pick3(p, softmax, lay.b_kcontig, P, &any) == MCF_OK ? MCF_EINVAL : MCF_EUNSUPPORTED;
    }
    if (lds_bytes_for(v) > kLdsBytesPerBlock)
        return MCF_EINVAL; // more LDS than a compute unit has

    const int64_t tm = 32ll * v->mb * v->rg;
    const int64_t m_tiles = (p->M + tm - 1) / tm;
    const int64_t h_tiles = p->L / tl;
    if (p->batch * m_tiles * h_tiles >= (1ll << 31)) return MCF_EUNSUPPORTED;

    KParams k;
    memset(&k, 0, sizeof(k));
    k.A = A; k.B = B; k.D = D; k.E = E;
    k.sa_b = lay.sa[0]; k.sa_r = lay.sa[1];
    k.sb_b = lay.sb[0]; k.sb_r = lay.b_kcontig ? lay.sb[2] : lay.sb[1];
    k.sd_b = lay.sd[0]; k.sd_r = lay.sd[1];
    k.se_b = lay.se[0]; k.se_r = lay.se[1];
    k.M = (int32_t)p->M; k.N = (int32_t)p->N;
    k.m_tiles = (int32_t)m_tiles;
    k.h_tiles = (int32_t)h_tiles;
    k.n_blocks = (int32_t)(p->batch * m_tiles * h_tiles);
    division_magic((uint32_t)m_tiles, &k.m_magic, &k.m_shift);
    division_magic((uint32_t)h_tiles, &k.h_magic, &k.h_shift);
    k.c1 = 1.0f; k.a_mode = 0;
    k.k_chunks = (int32_t)(p->K / v->K);
    k.F = F; k.sf_b = sf[0]; k.sf_r = sf[1];
    if (p->out_dtype == MCF_F32) k.E = (void *)((uintptr_t)E | 1); // the kernels read bit 0 as "store fp32"
    if (softmax) {
        // row i sees the columns n <= i + causal_off, which the kernel forms in 32 bits; an offset
        // of N - 1 (or more) hides nothing and stands for "no mask", below -M nothing is seen either
        if (p->M + p->N >= (1ll << 31) - 1024) { set_last_error("softmax chain: M + N must stay below 2^31 - 1024"); return MCF_EUNSUPPORTED; }
        k.causal_off = (int32_t)(!causal || causal_off > p->N - 1 ? p->N - 1 : causal_off < -p->M - 1 ? -p->M - 1 : causal_off);
    }
    if (softmax) {
        // exp(scale*s - max) = exp2(|scale|*log2(e) * (s' - max')) with s' = +-s; a zero scale
        // makes every logit equal, which is what A := 0 gives.
        const float log2e = 1.4426950408889634f;
        if (scale == 0.0f) { k.a_mode = 2; k.c1 = log2e; }
        else { k.a_mode = scale < 0.0f ? 1 : 0; k.c1 = fabsf(scale) * log2e; }
    }
    int err = v->launch(k, stream);
    if (err != 0) {
        set_last_error(hipGetErrorString((hipError_t)err));
        return MCF_ELAUNCH;
    }
    return MCF_OK;
}

} // namespace mcf

extern "C" int mcf_gemm_chain(const mcf_problem *p, const void *A, const void *B, const void *D, void *E,
                              const mcf_tiles *tiles, void *stream) {
    return mcf::run(p, 0, 1.0f, A, B, D, E, tiles, stream);
}

extern "C" int mcf_softmax_gemm_chain(const mcf_problem *p, float scale, const void *A, const void *B, const void *D,
                                      void *E, const mcf_tiles *tiles, void *stream) {
    return mcf::run(p, 1, scale, A, B, D, E, tiles, stream);
}

extern "C" int mcf_causal_softmax_gemm_chain(const mcf_problem *p, float scale, int64_t causal_offset, const void *A,
                                             const void *B, const void *D, void *E, const mcf_tiles *tiles, void *stream) {
    return mcf::run(p, 1, scale, A, B, D, E, tiles, stream, 0, nullptr, nullptr, true, causal_offset);
}

extern "C" int mcf_gemm_chain3(const mcf_problem *p, int softmax, float scale, int64_t P, const int64_t *f_stride,
                               const void *A, const void *B, const void *D, const void *F, void *G,
                               const mcf_tiles *tiles, void *stream) {
    if (P <= 0) return P == 0 && p && p->batch >= 0 ? MCF_OK : MCF_EINVAL; // no output columns: nothing to do
    return mcf::run(p, softmax != 0, softmax ? scale : 1.0f, A, B, D, G, tiles, stream, P, f_stride, F);
}

extern "C" int mcf_pick_tiles3(const mcf_problem *p, int64_t P, int softmax, mcf_tiles *out) {
    mcf::Layout lay;
    if (!p || !out || P <= 0) return MCF_EINVAL;
    mcf_problem pc = *p;
    memset(pc.e_stride, 0, sizeof(pc.e_stride)); // describes G, which the tile choice does not depend on
    const int st = mcf::decode_layout(&pc, &lay);
    if (st != MCF_OK) return st;
    return mcf::pick3(&pc, softmax != 0, lay.b_kcontig, P, out);
}

namespace mcf {
// Problem of the two-GEMM part and layout of B for a three-GEMM problem (e_stride describes G).
int problem3(const mcf_problem *p, int64_t P, mcf_problem *pc, int *b_kcontig) {
    mcf::Layout lay;
    if (!p || P <= 0) return MCF_EINVAL;
    *pc = *p;
    memset(pc->e_stride, 0, sizeof(pc->e_stride));
    const int st = mcf::decode_layout(pc, &lay);
    if (st == MCF_OK) *b_kcontig = lay.b_kcontig;
    return st;
}
} // namespace mcf

extern "C" int mcf_list_candidates3(const mcf_problem *p, int64_t P, int softmax, mcf_tiles *out, int cap) {
    mcf_problem pc;
    int bk = 0;
    std::vector<mcf_tiles> c;
    if (mcf::problem3(p, P, &pc, &bk) != MCF_OK || mcf::candidates3(&pc, softmax != 0, bk, P, &c) != MCF_OK) return 0;
    for (int i = 0; i < (int)c.size() && out && i < cap; ++i) out[i] = c[i];
    return (int)c.size();
}

extern "C" int mcf_list_variants3(const mcf_problem *p, int64_t P, int softmax, int32_t *out, int cap) {
    mcf::Layout lay;
    if (!p) return 0;
    mcf_problem pc = *p;
    memset(pc.e_stride, 0, sizeof(pc.e_stride));
    if (mcf::decode_layout(&pc, &lay) != MCF_OK) return 0;
    int n = 0, total = 0;
    const mcf::Variant *v = mcf::variants3(&n);
    for (int i = 0; i < n; ++i) {
        if (v[i].dtype != p->in_dtype || v[i].K != p->K || v[i].L != p->L || v[i].P != P ||
            v[i].softmax != (softmax != 0) || v[i].b_kcontig != lay.b_kcontig)
            continue;
        if (out && total < cap) {
            out[4 * total] = v[i].mb; out[4 * total + 1] = v[i].rg; out[4 * total + 2] = v[i].ns; out[4 * total + 3] = v[i].nj;
        }
        ++total;
    }
    return total;
}

extern "C" const char *mcf_status_string(int s) {
    switch (s) {
    case MCF_OK: return "MCF_OK";
    case MCF_EINVAL: return "MCF_EINVAL: invalid argument";
    case MCF_EUNSUPPORTED: return "MCF_EUNSUPPORTED: no kernel variant covers this problem";
    case MCF_EALIGN: return "MCF_EALIGN: pointer or stride not 16-byte aligned";
    case MCF_ELAUNCH: return "MCF_ELAUNCH: HIP launch failed";
    default: return "unknown mcf status";
    }
}

extern "C" const char *mcf_last_error(void) { return mcf::g_last_error; }
