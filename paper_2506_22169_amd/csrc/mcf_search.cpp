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

using namespace mcf;

extern "C" int mcf_search_tiles(const mcf_problem *p, int softmax, const mcf_search_params *params,
                                mcf_measure_fn measure, void *user, mcf_tiles *best, mcf_search_report *report) {
    if (!measure || !best) return MCF_EINVAL;
    std::vector<mcf_tiles> space;
    int st = feasible_candidates(p, softmax, &space);
    if (st != MCF_OK) return st;
    const int N = params && params->population > 0 ? params->population : 32;
    const int n = params && params->top_n > 0 ? params->top_n : 8;
    const int max_gen = params && params->max_generations > 0 ? params->max_generations : 16;
    const double eps = params && params->epsilon > 0 ? params->epsilon : 0.02;
    Uniforms rng(params ? params->seed : 0);
    const int C = (int)space.size();

    if (report) {
        memset(report, 0, sizeof(*report));
        report->space = C;
    }
    // first population: without repetition while unused candidates remain (a random permutation
    // of the space), topped up with random draws
    std::vector<int> population(N), perm(C);
    for (int i = 0; i < C; ++i) perm[i] = i;
    for (int i = 0; i < N; ++i) {
        if (i < C) {
            const int j = i + rng.below(C - i);
            std::swap(perm[i], perm[j]);
            population[i] = perm[i];
        } else {
            population[i] = rng.below(C);
        }
    }
    std::vector<double> measured(C, -1.0);
    double best_t = 1e9;
    int best_cand = -1, generation = 0, n_measured = 0;
    bool converged = false;
    for (;;) {
        // rank by the model; ties by candidate index
        std::sort(population.begin(), population.end(), [&](int a, int b) {
            return space[a].t_est_s != space[b].t_est_s ? space[a].t_est_s < space[b].t_est_s : a < b;
        });
        std::vector<int> topk;
        for (int c : population) {
            if (std::find(topk.begin(), topk.end(), c) == topk.end()) topk.push_back(c);
            if ((int)topk.size() == n) break;
        }
        for (int c : topk) {
            if (measured[c] >= 0.0) continue;
            const double t = measure(&space[c], user);
            if (!(t >= 0.0) || !(t < INFINITY)) return MCF_ELAUNCH;
            measured[c] = t;
            if (report && n_measured < MCF_SEARCH_LOG_MAX) {
                mcf_search_entry &e = report->log[n_measured];
                e.mb = space[c].mb; e.rg = space[c].rg; e.ns = space[c].ns; e.nj = space[c].nj;
                e.generation = generation; e.tl = space[c].tl; e.t_est_s = space[c].t_est_s; e.t_meas_s = t;
            }
            ++n_measured;
        }
        int top1 = topk[0];
        for (int c : topk)
            if (measured[c] < measured[top1]) top1 = c;
        const double top1_t = measured[top1];
        ++generation;
        if (fabs(top1_t - best_t) / best_t < eps) {
            best_cand = top1; best_t = top1_t; converged = true;
            break;
        }
        if (top1_t < best_t) { best_cand = top1; best_t = top1_t; }
        if (generation >= max_gen) break;
        // next population: parents with probability ~ 1 / estimate, one loop's choice replaced
        std::vector<double> cumulative(N);
        double total = 0.0;
        for (int i = 0; i < N; ++i) {
            total += 1.0 / space[population[i]].t_est_s;
            cumulative[i] = total;
        }
        std::vector<int> next(N);
        for (int i = 0; i < N; ++i) {
            const double target = rng.next() * total;
            int parent = population[N - 1];
            for (int q = 0; q < N; ++q)
                if (target < cumulative[q]) { parent = population[q]; break; }
            const int loop = rng.below(kLoops);
            const double u = rng.next();
            const std::vector<int> options = neighbours(space, parent, loop);
            next[i] = options.empty() ? parent : options[std::min((int)(u * options.size()), (int)options.size() - 1)];
        }
        population.swap(next);
    }
    *best = space[best_cand];
    if (report) {
        report->generations = generation;
        report->measured = std::min(n_measured, (int)MCF_SEARCH_LOG_MAX);
        report->converged = converged ? 1 : 0;
        report->best_t_s = best_t;
    }
    return MCF_OK;
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
};

double measure_on_device(const mcf_tiles *cand, void *user) {
    DeviceMeasure *m = (DeviceMeasure *)user;
    auto launch = [&]() {
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

extern "C" int mcf_tune_tiles(const mcf_problem *p, int softmax, float scale, const void *A, const void *B,
                              const void *D, void *E, const mcf_search_params *params, int launches, void *stream,
                              mcf_tiles *best, mcf_search_report *report) {
    if (!p || !best) return MCF_EINVAL;
    // an empty problem has nothing to measure: fall back on the model
    if (p->batch == 0 || p->M == 0 || p->L == 0 || p->N == 0) return mcf_pick_tiles(p, softmax, best);
    DeviceMeasure m{p, softmax != 0, scale, A, B, D, E, launches > 0 ? launches : 20, (hipStream_t)stream, nullptr, nullptr, MCF_OK};
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
    int st = mcf_pick_tiles(p, softmax, &warm);
    if (st == MCF_OK) {
        const double t1 = measure_on_device(&warm, &m);
        if (t1 > 0.0) {
            int rounds = (int)(0.05 / (t1 * m.launches));
            rounds = rounds < 1 ? 1 : rounds > 30 ? 30 : rounds;
            for (int r = 0; r < rounds && m.status == MCF_OK; ++r) (void)measure_on_device(&warm, &m);
        }
    }
    if (st == MCF_OK && m.status == MCF_OK) st = mcf_search_tiles(p, softmax, params, measure_on_device, &m, best, report);
    else if (st == MCF_OK) st = MCF_ELAUNCH;
    if (st == MCF_ELAUNCH && m.status != MCF_OK) st = m.status; // the chain call's own verdict (EINVAL, EALIGN, ...)
    (void)hipEventDestroy(m.e0);
    (void)hipEventDestroy(m.e1);
    return st;
}
