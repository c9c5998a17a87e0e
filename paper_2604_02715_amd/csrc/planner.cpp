// Budget-aware residency planner (paper Sec. 4.3, Alg. 2): host-side control logic, no HIP.
//
// State per rank: the class of every MoE layer (uncompressed-resident or pageable) and, for
// pageable layers, which of the 2 * L_r expert tensors are backed by pinned host memory
// instead of compressed GPU memory.  Because a layer gives up its tensors by descending
// expert index and restoration undoes steps strictly in reverse, the GPU-backed tensors of a
// type in a layer are always the experts [0, gpu_count): one counter per (layer, type) is the
// whole tensor-level state.
#include <cmath>
#include <cstring>
#include <limits>
#include <new>
#include <vector>

#include "fluxmoe_internal.h"

using fluxmoe::set_error;

struct fluxmoe_planner {
    uint32_t N = 0, Lr = 0, CI = 16;
    double theta = 0.9, AG = 0.25;
    std::vector<uint8_t> pageable;          // [N]
    std::vector<uint32_t> gpu_count[2];     // [type - 1][N]: experts [0, count) are GPU-backed
    std::vector<uint64_t> host_volume;      // [N], in down-projection tensors (fused counts 2)
    struct Step { int32_t type; uint32_t layer; uint32_t n; };   // type 0: layer became pageable
    std::vector<Step> steps;                // reclamation history
    std::vector<uint32_t> step_layers;      // layers of every tensor moved, in move order
    uint64_t iteration = 0;
    bool done = false;
};

namespace {

uint32_t step_size(const fluxmoe_planner* p, int type) {
    const double x = p->AG * double(p->Lr) * (type == 2 ? 1.0 : 0.5);
    return uint32_t(std::max(1.0, std::ceil(x - 1e-9)));
}

// The layer the next tensor of `type` leaves: smallest host volume, then the largest index.
int64_t next_layer(const fluxmoe_planner* p, int type) {
    int64_t best = -1;
    for (int64_t l = int64_t(p->N) - 1; l >= 0; --l) {
        if (!p->pageable[l] || p->gpu_count[type - 1][l] == 0) continue;
        if (best < 0 || p->host_volume[l] < p->host_volume[best]) best = l;
    }
    return best;
}

uint32_t do_reclaim(fluxmoe_planner* p, fluxmoe_planner_move* moves) {
    for (int64_t l = int64_t(p->N) - 1; l >= 0; --l)
        if (!p->pageable[l]) {                       // stage 1: one resident layer becomes pageable
            p->pageable[l] = 1;
            p->steps.push_back({0, uint32_t(l), 1});
            moves[0] = fluxmoe_planner_move{uint32_t(l), 0, 0, 1};
            return 1;
        }
    const int type = next_layer(p, 2) >= 0 ? 2 : 1;  // stage 2: down tensors first, then fused
    const uint32_t want = step_size(p, type);
    uint32_t n = 0;
    for (; n < want; ++n) {
        const int64_t l = next_layer(p, type);
        if (l < 0) break;
        const uint32_t e = --p->gpu_count[type - 1][l];
        p->host_volume[l] += type == 2 ? 1 : 2;
        p->step_layers.push_back(uint32_t(l));
        moves[n] = fluxmoe_planner_move{uint32_t(l), e, type, 1};
    }
    if (n) p->steps.push_back({type, 0, n});
    return n;
}

uint32_t do_restore(fluxmoe_planner* p, fluxmoe_planner_move* moves) {
    if (p->steps.empty()) return 0;
    const fluxmoe_planner::Step s = p->steps.back();
    p->steps.pop_back();
    if (s.type == 0) {
        p->pageable[s.layer] = 0;
        moves[0] = fluxmoe_planner_move{s.layer, 0, 0, 0};
        return 1;
    }
    for (uint32_t i = 0; i < s.n; ++i) {             // last tensor offloaded comes back first
        const uint32_t l = p->step_layers.back();
        p->step_layers.pop_back();
        const uint32_t e = p->gpu_count[s.type - 1][l]++;
        p->host_volume[l] -= s.type == 2 ? 1 : 2;
        moves[i] = fluxmoe_planner_move{l, e, s.type, 0};
    }
    return s.n;
}

int check(const fluxmoe_planner* p, const void* moves, size_t cap) {
    if (!p) return set_error(FLUXMOE_EINVAL, "planner is NULL");
    if (!moves || cap < fluxmoe_planner_max_moves(p))
        return set_error(FLUXMOE_ENOMEM, "moves holds %zu entries, a step can produce %u", cap,
                         fluxmoe_planner_max_moves(p));
    return FLUXMOE_OK;
}

}  // namespace

extern "C" {

int fluxmoe_balanced_split(double beta_gpu, double beta_cpu, uint32_t experts_per_rank, double* x_bw,
                           uint32_t* n_down, uint32_t* n_fused) {
    if (!(beta_gpu > 0) || !(beta_cpu >= 0) || !std::isfinite(beta_gpu) || !std::isfinite(beta_cpu))
        return set_error(FLUXMOE_EINVAL, "bandwidths must be finite, beta_gpu > 0, beta_cpu >= 0");
    if (experts_per_rank == 0) return set_error(FLUXMOE_EINVAL, "experts_per_rank must be positive");
    const double x = beta_cpu / (beta_gpu + beta_cpu);
    // a layer is 3 L_r down-projection volumes (a fused tensor is two of them)
    const uint64_t units = uint64_t(std::ceil(3.0 * experts_per_rank * x - 1e-12));
    const uint64_t down = std::min<uint64_t>(units, experts_per_rank);
    const uint64_t fused = std::min<uint64_t>(experts_per_rank, (units - down + 1) / 2);
    if (x_bw) *x_bw = x;
    if (n_down) *n_down = uint32_t(down);
    if (n_fused) *n_fused = uint32_t(fused);
    return FLUXMOE_OK;
}

int fluxmoe_planner_create(const fluxmoe_planner_desc* d, const uint8_t* uncompressed,
                           fluxmoe_planner** out) {
    if (!d || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if (d->n_layers == 0 || d->experts_per_rank == 0)
        return set_error(FLUXMOE_EINVAL, "n_layers and experts_per_rank must be positive");
    const double theta = d->theta == 0 ? 0.9 : d->theta, ag = d->adjustment_granularity == 0 ? 0.25 : d->adjustment_granularity;
    if (!(theta > 0 && theta <= 1)) return set_error(FLUXMOE_EINVAL, "theta must be in (0, 1]");
    if (!(ag > 0 && ag <= 1)) return set_error(FLUXMOE_EINVAL, "adjustment_granularity must be in (0, 1]");
    fluxmoe_planner* p = new (std::nothrow) fluxmoe_planner;
    if (!p) return set_error(FLUXMOE_ENOMEM, "out of host memory");
    p->N = d->n_layers;
    p->Lr = d->experts_per_rank;
    p->CI = d->control_interval ? d->control_interval : 16;
    p->theta = theta;
    p->AG = ag;
    p->pageable.assign(p->N, 1);
    if (uncompressed)
        for (uint32_t l = 0; l < p->N; ++l) p->pageable[l] = uncompressed[l] ? 0 : 1;
    p->gpu_count[0].assign(p->N, p->Lr);
    p->gpu_count[1].assign(p->N, p->Lr);
    p->host_volume.assign(p->N, 0);
    *out = p;
    return FLUXMOE_OK;
}

int fluxmoe_planner_destroy(fluxmoe_planner* p) {
    delete p;
    return FLUXMOE_OK;
}

uint32_t fluxmoe_planner_max_moves(const fluxmoe_planner* p) {
    return p ? std::max(step_size(p, 2), step_size(p, 1)) : 0;
}

int fluxmoe_planner_reclaim(fluxmoe_planner* p, fluxmoe_planner_move* moves, size_t cap, uint32_t* n_moves) {
    if (int rc = check(p, moves, cap)) return rc;
    const uint32_t n = do_reclaim(p, moves);
    if (n_moves) *n_moves = n;
    return FLUXMOE_OK;
}

int fluxmoe_planner_restore(fluxmoe_planner* p, fluxmoe_planner_move* moves, size_t cap, uint32_t* n_moves) {
    if (int rc = check(p, moves, cap)) return rc;
    const uint32_t n = do_restore(p, moves);
    if (n_moves) *n_moves = n;
    return FLUXMOE_OK;
}

int fluxmoe_planner_tick(fluxmoe_planner* p, uint64_t B_rem, uint64_t B_act, double tau_fwd,
                         const double* tau_load_layer, fluxmoe_planner_decision* out,
                         fluxmoe_planner_move* moves, size_t cap) {
    if (int rc = check(p, moves, cap)) return rc;
    if (!out) return set_error(FLUXMOE_EINVAL, "out is NULL");
    if (!(tau_fwd >= 0)) return set_error(FLUXMOE_EINVAL, "tau_fwd must be non-negative");
    double tau_load = 0;
    if (tau_load_layer)
        for (uint32_t l = 0; l < p->N; ++l) {
            if (!(tau_load_layer[l] >= 0)) return set_error(FLUXMOE_EINVAL, "tau_load_layer[%u] is negative or NaN", l);
            tau_load += tau_load_layer[l];
        }
    const double nan = std::numeric_limits<double>::quiet_NaN();
    *out = fluxmoe_planner_decision{FLUXMOE_PLAN_SKIP, 0, nan, nan, nan};
    if (p->done || B_rem == 0) {
        p->done = true;
        out->action = FLUXMOE_PLAN_DONE;
        return FLUXMOE_OK;
    }
    ++p->iteration;
    if (p->iteration % p->CI != 0 || B_act == 0) return FLUXMOE_OK;
    out->tau_eff = double(B_rem) / double(B_act) * tau_fwd;
    out->tau_load = tau_load;
    out->rho = tau_load == 0 ? std::numeric_limits<double>::infinity() : out->tau_eff / tau_load;
    out->action = FLUXMOE_PLAN_KEEP;
    if (out->rho > 1 && B_act < B_rem) {
        out->n_moves = do_reclaim(p, moves);
        if (out->n_moves) out->action = FLUXMOE_PLAN_RECLAIM;
    } else if (out->rho < p->theta) {
        out->n_moves = do_restore(p, moves);
        if (out->n_moves) out->action = FLUXMOE_PLAN_RESTORE;
    }
    return FLUXMOE_OK;
}

int fluxmoe_planner_state(const fluxmoe_planner* p, uint8_t* layer_pageable, uint8_t* on_host) {
    if (!p) return set_error(FLUXMOE_EINVAL, "planner is NULL");
    if (layer_pageable) std::memcpy(layer_pageable, p->pageable.data(), p->N);
    if (on_host)
        for (uint32_t l = 0; l < p->N; ++l)
            for (uint32_t e = 0; e < p->Lr; ++e)
                for (int t = 0; t < 2; ++t)
                    on_host[(uint64_t(l) * p->Lr + e) * 2 + t] = e >= p->gpu_count[t][l];
    return FLUXMOE_OK;
}

}  // extern "C"
