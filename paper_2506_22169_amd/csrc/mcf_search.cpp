// Heuristic search over the built variants (Sec. IV-B, Alg. 1): model-ranked populations, the
// best-ranked few measured, convergence on the measured time, mutation of one loop's tile
// choice.  mcf_search_tiles takes the measurement as a callback; mcf_tune_tiles measures on
// the device with HIP events.
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "mcf_internal.h"

namespace mcf {
namespace {

// u_k = top 53 bits of SplitMix64(seed + k), k = 0, 1, ...
struct Uniforms {
    uint64_t seed, k = 0;
    explicit Uniforms(uint64_t s) : seed(s) {}
    double next() {
        uint64_t x = seed + k++ + 0x9E3779B97F4A7C15ull;
        x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
        x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
        x ^= x >> 31;
        return (double)(x >> 11) * (1.0 / 9007199254740992.0);
    }
    int below(int n) { return std::min((int)(next() * n), n - 1); }
};

// Candidates that differ from candidate i in the tile choice of one loop only
// (loop 0 = m: the pair mb, rg; loop 1 = n: the pair ns, nj; loop 2 = h: T_L).
constexpr int kLoops = 3;
std::vector<int> neighbours(const std::vector<mcf_tiles> &space, int i, int loop) {
    std::vector<int> out;
    const mcf_tiles &me = space[i];
    for (int j = 0; j < (int)space.size(); ++j) {
        const mcf_tiles &c = space[j];
        const bool same[kLoops] = {c.mb == me.mb && c.rg == me.rg, c.ns == me.ns && c.nj == me.nj, c.tl == me.tl};
        bool ok = j != i;
        for (int q = 0; q < kLoops; ++q) ok = ok && (q == loop ? !same[q] : same[q]);
        if (ok) out.push_back(j);
    }
    return out;
}

} // namespace
} // namespace mcf

namespace mcf {
namespace {

// State of one search: the candidate space with its model estimates, what has been measured so
// far, and the generation in hand.  A generation is a multiset of candidate indices.
class TileSearch {
  public:
    TileSearch(std::vector<mcf_tiles> space, int members, int shortlist, uint64_t seed, mcf_measure_fn fn, void *user,
               mcf_search_report *report)
        : space_(std::move(space)), members_(members), shortlist_(shortlist), rng_(seed), fn_(fn), user_(user),
          report_(report), time_(space_.size(), -1.0) {}

    // Generation 0: a random order of the whole space, cut to `members` or topped up with
    // independent draws (a space no larger than a generation is covered at once).
    void seed_generation() {
        const int C = (int)space_.size();
        std::vector<int> order(C);
        for (int i = 0; i < C; ++i) order[i] = i;
        gen_.resize(members_);
        for (int i = 0; i < members_; ++i) {
            if (i < C) {
                std::swap(order[i], order[i + rng_.below(C - i)]);
                gen_[i] = order[i];
            } else {
                gen_[i] = rng_.below(C);
            }
        }
    }

    // Orders the generation by the model (ties by index), times the first `shortlist` distinct
    // members that have no time yet, and returns the fastest of that shortlist; -1 if a
    // measurement failed.
    int evaluate(int generation) {
        std::sort(gen_.begin(), gen_.end(), [&](int a, int b) {
            return space_[a].t_est_s != space_[b].t_est_s ? space_[a].t_est_s < space_[b].t_est_s : a < b;
        });
        int front = -1, taken = 0;
        std::vector<char> seen(space_.size(), 0);
        for (int c : gen_) {
            if (seen[c]) continue;
            seen[c] = 1;
            if (time_[c] < 0.0) {
                const double t = fn_(&space_[c], user_);
                if (!(t >= 0.0) || !(t < INFINITY)) return -1;
                time_[c] = t;
                record(c, generation);
                if (overall_ < 0 || t < time_[overall_]) overall_ = c;
            }
            if (front < 0 || time_[c] < time_[front]) front = c;
            if (++taken == shortlist_) break;
        }
        return front;
    }

    // Next generation: each member descends from a member of this one, chosen with probability
    // proportional to 1 / estimate, with the tile choice of one loop replaced by that of a
    // random candidate that differs there only (none: the member is carried over).
    void breed() {
        std::vector<double> upto(gen_.size());
        double total = 0.0;
        for (size_t i = 0; i < gen_.size(); ++i) upto[i] = (total += 1.0 / space_[gen_[i]].t_est_s);
        std::vector<int> next(gen_.size());
        for (int &child : next) {
            const double mark = rng_.next() * total;
            const size_t at = std::upper_bound(upto.begin(), upto.end(), mark) - upto.begin();
            const int parent = gen_[std::min(at, gen_.size() - 1)];
            const int loop = rng_.below(kLoops);
            const double u = rng_.next();
            const std::vector<int> other = neighbours(space_, parent, loop);
            child = other.empty() ? parent : other[std::min((size_t)(u * other.size()), other.size() - 1)];
        }
        gen_.swap(next);
    }

    double time_of(int c) const { return time_[c]; }
    int fastest_measured() const { return overall_; }
    int measured() const { return n_measured_; }
    const mcf_tiles &tiles(int c) const { return space_[c]; }

  private:
    void record(int c, int generation) {
        if (report_ && n_measured_ < MCF_SEARCH_LOG_MAX) {
            mcf_search_entry &e = report_->log[n_measured_];
            const mcf_tiles &t = space_[c];
            e.mb = t.mb; e.rg = t.rg; e.ns = t.ns; e.nj = t.nj;
            e.generation = generation; e.tl = t.tl; e.t_est_s = t.t_est_s; e.t_meas_s = time_[c];
        }
        ++n_measured_;
    }

    std::vector<mcf_tiles> space_;
    int members_, shortlist_;
    Uniforms rng_;
    mcf_measure_fn fn_;
    void *user_;
    mcf_search_report *report_;
    std::vector<double> time_; // measured seconds per candidate, < 0: not measured
    std::vector<int> gen_;
    int overall_ = -1;         // fastest candidate measured so far, over all generations
    int n_measured_ = 0;
};

} // namespace
} // namespace mcf

using namespace mcf;

// Alg. 1 over a given space of candidates.
static int search_space(std::vector<mcf_tiles> space, const mcf_search_params *params, mcf_measure_fn measure, void *user,
                        mcf_tiles *best, mcf_search_report *report) {
    const int members = params && params->population > 0 ? params->population : 32;
    const int shortlist = params && params->top_n > 0 ? params->top_n : 8;
    const int max_gen = params && params->max_generations > 0 ? params->max_generations : 16;
    const double eps = params && params->epsilon > 0 ? params->epsilon : 0.02;
    if (report) {
        memset(report, 0, sizeof(*report));
        report->space = (int)space.size();
    }
    TileSearch search(std::move(space), members, shortlist, params ? params->seed : 0, measure, user, report);
    search.seed_generation();
    // The search stops when the fastest of a generation's shortlist is within eps (relative) of
    // the time the previous generations had settled on; what is returned is the fastest
    // candidate measured in any generation.
    double settled = 1e9;
    int generation = 0;
    bool converged = false;
    while (!converged && generation < max_gen) {
        const int front = search.evaluate(generation);
        if (front < 0) return MCF_ELAUNCH;
        ++generation;
        const double t = search.time_of(front);
        converged = fabs(t - settled) / settled < eps;
        if (converged || t < settled) settled = t;
        if (!converged && generation < max_gen) search.breed();
    }
    const int winner = search.fastest_measured();
    *best = search.tiles(winner);
    if (report) {
        report->generations = generation;
        report->measured = std::min(search.measured(), (int)MCF_SEARCH_LOG_MAX);
        report->converged = converged ? 1 : 0;
        report->best_t_s = search.time_of(winner);
    }
    return MCF_OK;
}

extern "C" int mcf_search_tiles(const mcf_problem *p, int softmax, const mcf_search_params *params,
                                mcf_measure_fn measure, void *user, mcf_tiles *best, mcf_search_report *report) {
    if (!measure || !best) return MCF_EINVAL;
    std::vector<mcf_tiles> space;
    const int st = feasible_candidates(p, softmax, &space);
    if (st != MCF_OK) return st;
    return search_space(std::move(space), params, measure, user, best, report);
}

extern "C" int mcf_search_tiles3(const mcf_problem *p, int64_t P, int softmax, const mcf_search_params *params,
                                 mcf_measure_fn measure, void *user, mcf_tiles *best, mcf_search_report *report) {
    if (!measure || !best) return MCF_EINVAL;
    mcf_problem pc;
    int bk = 0;
    std::vector<mcf_tiles> space;
    int st = problem3(p, P, &pc, &bk);
    if (st == MCF_OK) st = candidates3(&pc, softmax != 0, bk, P, &space);
    if (st != MCF_OK) return st;
    return search_space(std::move(space), params, measure, user, best, report);
}

namespace {

struct DeviceMeasure {
    const mcf_problem *p;
    int softmax;
    float scale;
    const void *A, *B, *D;
    void *E;
    int launches;
    hipStream_t stream;
    hipEvent_t e0, e1;
    int status; // first failure seen by the callback
    int64_t P;  // > 0: the three-GEMM chain, with F and its strides
    const int64_t *f_stride;
    const void *F;
};

double measure_on_device(const mcf_tiles *cand, void *user) {
    DeviceMeasure *m = (DeviceMeasure *)user;
    auto launch = [&]() {
        if (m->P > 0) return mcf_gemm_chain3(m->p, m->softmax, m->scale, m->P, m->f_stride, m->A, m->B, m->D, m->F, m->E, cand, m->stream);
        return m->softmax ? mcf_softmax_gemm_chain(m->p, m->scale, m->A, m->B, m->D, m->E, cand, m->stream)
                          : mcf_gemm_chain(m->p, m->A, m->B, m->D, m->E, cand, m->stream);
    };
    for (int i = 0; i < 3; ++i)
        if ((m->status = launch()) != MCF_OK) return -1.0;
    hipError_t err = hipEventRecord(m->e0, m->stream);
    for (int i = 0; i < m->launches && err == hipSuccess; ++i)
        if ((m->status = launch()) != MCF_OK) return -1.0;
    if (err == hipSuccess) err = hipEventRecord(m->e1, m->stream);
    if (err == hipSuccess) err = hipEventSynchronize(m->e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, m->e0, m->e1);
    if (err != hipSuccess) {
        set_last_error(hipGetErrorString(err));
        m->status = MCF_ELAUNCH;
        return -1.0;
    }
    return (double)ms * 1e-3 / m->launches;
}

} // namespace

// Alg. 1 measured on the device, for the two-GEMM chain (P == 0) or the three-GEMM chain.
static int tune(const mcf_problem *p, int softmax, float scale, int64_t P, const int64_t *f_stride, const void *A,
                const void *B, const void *D, const void *F, void *E, const mcf_search_params *params, int launches,
                void *stream, mcf_tiles *best, mcf_search_report *report) {
    if (!p || !best) return MCF_EINVAL;
    auto pick = [&](mcf_tiles *t) { return P > 0 ? mcf_pick_tiles3(p, P, softmax, t) : mcf_pick_tiles(p, softmax, t); };
    // an empty problem has nothing to measure: fall back on the model
    if (p->batch == 0 || p->M == 0 || p->L == 0 || p->N == 0) return pick(best);
    DeviceMeasure m{p, softmax != 0, scale, A, B, D, E, launches > 0 ? launches : 20, (hipStream_t)stream, nullptr, nullptr, MCF_OK,
                    P, f_stride, F};
    hipError_t err = hipEventCreate(&m.e0);
    if (err == hipSuccess) err = hipEventCreate(&m.e1);
    if (err != hipSuccess) {
        set_last_error(hipGetErrorString(err));
        if (m.e0) (void)hipEventDestroy(m.e0);
        return MCF_ELAUNCH;
    }
    // bring the clocks up before the first candidate is timed: a few hundred launches of the
    // model's choice (or 50 ms, whichever comes first)
    mcf_tiles warm;
    int st = pick(&warm);
    if (st == MCF_OK) {
        const double t1 = measure_on_device(&warm, &m);
        if (t1 > 0.0) {
            int rounds = (int)(0.05 / (t1 * m.launches));
            rounds = rounds < 1 ? 1 : rounds > 30 ? 30 : rounds;
            for (int r = 0; r < rounds && m.status == MCF_OK; ++r) (void)measure_on_device(&warm, &m);
        }
    }
    if (st == MCF_OK && m.status == MCF_OK)
        st = P > 0 ? mcf_search_tiles3(p, P, softmax, params, measure_on_device, &m, best, report)
                   : mcf_search_tiles(p, softmax, params, measure_on_device, &m, best, report);
    else if (st == MCF_OK) st = MCF_ELAUNCH;
    if (st == MCF_ELAUNCH && m.status != MCF_OK) st = m.status; // the chain call's own verdict (EINVAL, EALIGN, ...)
    (void)hipEventDestroy(m.e0);
    (void)hipEventDestroy(m.e1);
    return st;
}

extern "C" int mcf_tune_tiles(const mcf_problem *p, int softmax, float scale, const void *A, const void *B,
                              const void *D, void *E, const mcf_search_params *params, int launches, void *stream,
                              mcf_tiles *best, mcf_search_report *report) {
    return tune(p, softmax, scale, 0, nullptr, A, B, D, nullptr, E, params, launches, stream, best, report);
}

extern "C" int mcf_tune_tiles3(const mcf_problem *p, int softmax, float scale, int64_t P, const int64_t *f_stride,
                               const void *A, const void *B, const void *D, const void *F, void *G,
                               const mcf_search_params *params, int launches, void *stream, mcf_tiles *best,
                               mcf_search_report *report) {
    if (P <= 0) return MCF_EINVAL;
    return tune(p, softmax, scale, P, f_stride, A, B, D, F, G, params, launches, stream, best, report);
}
