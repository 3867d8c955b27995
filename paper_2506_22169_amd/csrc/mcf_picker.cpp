// Tile picker: the analytical model of Sec. IV-A (eq. (2)-(5)) evaluated over the kernel
// variants built into the library, under Rule 3 (padding) and Rule 4 / eq. (1) (on-chip
// memory) of Sec. III-C.  Pure host arithmetic; needs no GPU.
//
// Per-block tiling expression: n( k(L_A, L_B, C_C), L_D, C_E ), S_E with T_K = K and T_L = L.
// k and h have extent 1, so (Sec. III-B) L_A is governed by m alone and S_E by m, h:
//     trips(L_A) = trips(S_E) = batch * m          m = ceil(M / T_M)
//     trips(L_B) = trips(L_D) = batch * m * n      n = ceil(N / T_N)
//     trips(C_C) = trips(C_E) = batch * m * n
// Differences from the printed model, each a reading made for this machine:
//   * eq. (3) charges every byte at one bandwidth W.  Here the first touch of each tensor (the
//     compulsory bytes) is charged at HBM bandwidth and the re-reads of B and D by the other
//     m-tiles of a batch at the L2 bandwidth, because on MI355X they are served by the XCD's
//     L2 / the memory-side cache, not by HBM.
//   * eq. (1) sums all five tiles against shared memory.  Here C and E (and A) live in
//     registers, so the sum is split: B and D tiles (two stages, padded rows) against the
//     160 KiB LDS, and A, C, E tiles against the share of the 512-entry VGPR file a lane gets.
//     The LDS figure is exact and the register figure is backed by the compiler's own
//     allocation (a variant that spills is never picked), so the 1.2x slack of Rule 4 is not
//     applied.  The LDS
//     holds a ring of 2..4 (B tile + D tile) stages, as deep as fits 80 KiB so that two
//     blocks share a compute unit.
//   * eq. (5) counts parallel work against parallel hardware, alpha = (N_block + N_SM) / N_block.
//     Here blocks run in rounds: a compute unit has four SIMDs, a block takes min(waves, 4) of
//     them (a block of 8 or 16 waves owns the unit like one of 4), a launch takes
//     ceil(units / (256 x 4)) rounds, and alpha is the capacity of those rounds over the units
//     that fill it -- the quantity the printed form bounds from above (ceil(x) <= x + 1).
//     Chosen by the regret of the closed-form pick against every candidate measured on 28
//     workloads: mean 1.016 (worst 1.12) against 1.061 (worst 1.58) for the printed form counted
//     in waves.
#include <math.h>
#include <string.h>

#include "mcf_geometry.h"
#include <vector>

#include "mcf_internal.h"

namespace mcf {

int stages_for(const Variant *v) {
    return ring_stages(v->K, v->L, v->mb, v->rg, v->ns, v->nj, v->softmax != 0, v->ksplit != 0,
                       v->P > 0 ? chain3_f_bytes(v->L, v->P) + 1024 : 0);
}
int lds_bytes_for(const Variant *v) {
    if (v->P > 0) return chain3_lds_bytes(v->K, v->L, v->P, v->mb, v->rg, v->ns, v->nj, stages_for(v));
    return total_lds_bytes(v->K, v->L, v->mb, v->rg, v->ns, v->nj, stages_for(v), v->ksplit != 0);
}

// Registers per lane (eq. (1) restricted to the register-resident tiles, in 32-bit registers):
// A tile (mb * K/16 operands of 4), E accumulators (mb * L/32 * 16), nj C accumulators and
// their 16-bit copies per mb (16 + 8; a pipelined softmax chain: two C tiles and the 16-bit
// copies, 16 + 16 + 8), the LDS operands in flight for one C tile (K/16 * 4 for
// B, L/32 * 8 for D), one load offset per wave-load of a stage, and a fixed allowance for
// addresses and softmax state.  It tracks the compiler's allocation to within about 25 %;
// the compiler's own numbers (scratch use) are the final arbiter, as PTX lowering is in
// Sec. VI-D1 of the paper.
// (With a k loop K is the chunk: the A operands of one chunk are what a lane holds, and there
// are two sets of load offsets, for the A + B chunk and for the D tile.)
int vgpr_estimate(int K, int L, int mb, int rg, int ns, int nj, int softmax, int ksplit) {
    const int slot = ksplit ? ksplit_slot_bytes(K, L, mb, rg, 32 * ns * nj) : stage_bytes(K, L, 32 * ns * nj);
    const int loads = (ksplit ? 2 : 1) * ((slot / 1024 + rg * ns - 1) / (rg * ns));
    const int hb = h_blocks(L);
    // a pipelined chain holds C of two consecutive n-tiles and the 16-bit P of one
    // (and fetches its LDS operands two MFMA steps ahead instead of a GEMM at a time)
    const bool piped = pipe_stages(K, L, mb, rg, ns, nj, softmax != 0, ksplit != 0) > 0;
    const int c_tiles = piped ? nj * mb * (16 + 16 + 8) : nj * mb * (16 + 8);
    const int operands = piped ? 16 : (K / 16) * 4 + hb * 8;
    return mb * (K / 16) * 4 + mb * hb * 16 + c_tiles + operands + loads + 24 + (softmax ? 16 : 0);
}

// Registers a lane may use: the 512-entry file of a SIMD is shared by the waves resident on
// it, and a block of w waves puts ceil(w/4) waves on each SIMD.
static int vgpr_cap(int waves) { return kVgprBudget / ((waves + 3) / 4); }

static bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }

// Rule 3: a power-of-two dimension takes no padding; otherwise the padding ratio stays < 0.05.
static bool padding_ok(int64_t dim, int64_t tile) {
    const int64_t padded = (dim + tile - 1) / tile * tile;
    if (is_pow2(dim)) return padded == dim;
    return (double)(padded - dim) < 0.05 * (double)dim;
}

static void eval_model(const mcf_problem *p, int softmax, const Variant *v, mcf_tiles *t) {
    const int mb = v->mb, rg = v->rg, ns = v->ns, nj = v->nj;
    memset(t, 0, sizeof(*t));
    t->mb = mb; t->rg = rg; t->ns = ns; t->nj = nj;
    t->tm = 32 * mb * rg; t->tn = 32 * ns * nj; t->tk = v->K; t->tl = v->L;
    t->waves = rg * ns;
    t->stages = stages_for(v);
    t->lds_bytes = lds_bytes_for(v);
    t->vgpr_est = vgpr_estimate(v->K, v->L, mb, rg, ns, nj, softmax, v->ksplit);
    t->vgpr_used = v->vgprs;
    t->scratch_bytes = v->scratch_bytes;
    const int64_t es = 2; // bytes per element, fp16 / bf16
    const int64_t m = (p->M + t->tm - 1) / t->tm, n = (p->N + t->tn - 1) / t->tn;
    // T_L < L: h is a second block dimension (deep expression m h n k): every h tile repeats
    // L_A, L_B and C_C of its (batch, m-tile)
    const int64_t h = p->L / t->tl;
    t->blocks = p->batch * m * h;
    // N_block of eq. (5) counted in SIMDs taken, against the machine's SIMDs (below)
    const int64_t units = t->blocks * (t->waves < kWaveUnitsPerBlock ? t->waves : kWaveUnitsPerBlock);
    t->compulsory_bytes = es * p->batch * (p->M * p->K + p->K * p->N + p->N * p->L + p->M * p->L);
    // with a live k loop (T_K < K) inside n, L_A is no longer hoisted out of n: trips m * n * k
    const int64_t k = (p->K + t->tk - 1) / t->tk;
    const int64_t la = (int64_t)t->tm * t->tk * es * p->batch * m * h * (k > 1 ? n * k : 1);
    const int64_t lb = (int64_t)t->tk * t->tn * es * p->batch * m * h * n * k;
    const int64_t ld = (int64_t)t->tn * t->tl * es * p->batch * m * h * n;
    const int64_t se = (int64_t)t->tm * t->tl * es * p->batch * m * h;
    t->model_bytes = la + lb + ld + se;
    t->flops = (2 * (int64_t)t->tm * t->tn * t->tk * k + 2 * (int64_t)t->tm * t->tn * t->tl) * p->batch * m * h * n;
    const int64_t reread = t->model_bytes > t->compulsory_bytes ? t->model_bytes - t->compulsory_bytes : 0;
    t->t_mem_s = (double)t->compulsory_bytes / kHbmBytesPerSec + (double)reread / kL2BytesPerSec;
    t->t_comp_s = (double)t->flops / kMfmaFlopsPerSec;
    const int64_t rounds = (units + kWaveUnits - 1) / kWaveUnits;
    t->alpha = units > 0 ? (double)(rounds * kWaveUnits) / (double)units : 1.0;
    t->t_est_s = (t->t_mem_s + t->t_comp_s) * t->alpha;
}

static bool feasible(const mcf_tiles &t) {
    return t.lds_bytes <= kLdsBytesPerBlock && t.vgpr_est <= vgpr_cap(t.waves) && t.scratch_bytes == 0;
}

// Strict ordering of candidates: smaller estimate first; among equal estimates (the model
// does not see how the waves of a block are arranged) more waves per block, then a block
// whose LDS leaves room for a second one on the compute unit, then fewer waves across n (less
// to combine), then more column slices per wave, then fewer rows per wave.
bool better(const mcf_tiles &a, const mcf_tiles &b) {
    if (a.t_est_s != b.t_est_s) return a.t_est_s < b.t_est_s;
    if (a.tl != b.tl) return a.tl > b.tl;
    if (a.waves != b.waves) return a.waves > b.waves;
    const bool a2 = 2 * a.lds_bytes <= kLdsBytesPerBlock, b2 = 2 * b.lds_bytes <= kLdsBytesPerBlock;
    if (a2 != b2) return a2;
    if (a.ns != b.ns) return a.ns < b.ns;
    if (a.nj != b.nj) return a.nj > b.nj;
    return a.mb < b.mb;
}

static int check_problem(const mcf_problem *p, Layout *lay) {
    if (!p) return MCF_EINVAL;
    if (p->batch < 0 || p->M < 0 || p->K < 0 || p->N < 0 || p->L < 0) return MCF_EINVAL;
    return decode_layout(p, lay);
}

} // namespace mcf

using namespace mcf;

extern "C" int mcf_list_variants(const mcf_problem *p, int softmax, int32_t *out, int cap) {
    Layout lay;
    if (check_problem(p, &lay) != MCF_OK) return 0;
    int n = 0, total = 0, tk = 0, ksplit = 0;
    if (!resolve_group(p->in_dtype, p->K, p->L, &tk, &ksplit)) return 0;
    const Variant *v = variants(&n);
    for (int i = 0; i < n; ++i) {
        if (v[i].dtype != p->in_dtype || v[i].K != tk || v[i].ksplit != ksplit || v[i].L != p->L ||
            v[i].softmax != (softmax != 0) || v[i].b_kcontig != lay.b_kcontig)
            continue;
        if (out && total < cap) {
            out[4 * total] = v[i].mb; out[4 * total + 1] = v[i].rg; out[4 * total + 2] = v[i].ns; out[4 * total + 3] = v[i].nj;
        }
        ++total;
    }
    return total;
}

extern "C" int mcf_eval_tiles(const mcf_problem *p, int softmax, mcf_tiles *t) {
    Layout lay;
    if (!t) return MCF_EINVAL;
    int st = check_problem(p, &lay);
    if (st != MCF_OK) return st;
    const int mb = t->mb, rg = t->rg, ns = t->ns, nj = t->nj > 0 ? t->nj : 1;
    const int64_t tl = t->tl > 0 ? t->tl : p->L;
    if (p->L % tl != 0) return MCF_EUNSUPPORTED;
    const Variant *v = find_variant(p->in_dtype, p->K, tl, softmax != 0, lay.b_kcontig, mb, rg, ns, nj);
    if (!v) return MCF_EUNSUPPORTED;
    eval_model(p, softmax != 0, v, t);
    return feasible(*t) ? MCF_OK : MCF_EINVAL;
}

// The candidates the picker and the search choose from: for T_L = L and then for every smaller
// T_L that divides L and has kernels, in registry order, the feasible variants that satisfy
// Rule 3; if Rule 3 leaves nothing (e.g. M smaller than every tile) it is dropped so that a
// feasible variant is always found when one covers the shape.
int mcf::feasible_candidates(const mcf_problem *p, int softmax, std::vector<mcf_tiles> *out) {
    Layout lay;
    int st = check_problem(p, &lay);
    if (st != MCF_OK) return st;
    int n = 0, tk = 0, ksplit = 0;
    if (!resolve_group(p->in_dtype, p->K, p->L, &tk, &ksplit)) return MCF_EUNSUPPORTED;
    const Variant *v = variants(&n);
    std::vector<int> tls; // T_L options, the full L first, then descending
    tls.push_back((int)p->L);
    for (int tl = (int)p->L / 2; tl >= 32; --tl) {
        int tk2 = 0, ks2 = 0;
        if (p->L % tl == 0 && resolve_group(p->in_dtype, p->K, tl, &tk2, &ks2)) tls.push_back(tl);
    }
    for (int pass = 0; pass < 2; ++pass) {
        out->clear();
        for (int tl : tls) {
            resolve_group(p->in_dtype, p->K, tl, &tk, &ksplit);
            for (int i = 0; i < n; ++i) {
                if (v[i].dtype != p->in_dtype || v[i].K != tk || v[i].ksplit != ksplit || v[i].L != tl ||
                    v[i].softmax != (softmax != 0) || v[i].b_kcontig != lay.b_kcontig)
                    continue;
                mcf_tiles t;
                eval_model(p, softmax != 0, &v[i], &t);
                if (!feasible(t)) continue;
                if (pass == 0 && p->M > 0 && p->N > 0 && !(padding_ok(p->M, t.tm) && padding_ok(p->N, t.tn))) continue;
                out->push_back(t);
            }
        }
        if (!out->empty()) return MCF_OK;
    }
    return MCF_EUNSUPPORTED;
}

extern "C" int mcf_list_candidates(const mcf_problem *p, int softmax, mcf_tiles *out, int cap) {
    std::vector<mcf_tiles> cands;
    if (feasible_candidates(p, softmax, &cands) != MCF_OK) return 0;
    for (int i = 0; i < (int)cands.size() && out && i < cap; ++i) out[i] = cands[i];
    return (int)cands.size();
}

extern "C" int mcf_pick_tiles(const mcf_problem *p, int softmax, mcf_tiles *out) {
    if (!out) return MCF_EINVAL;
    std::vector<mcf_tiles> cands;
    int st = feasible_candidates(p, softmax, &cands);
    if (st != MCF_OK) return st;
    const mcf_tiles *best = &cands[0];
    for (const mcf_tiles &t : cands)
        if (better(t, *best)) best = &t;
    *out = *best;
    return MCF_OK;
}
