// Host helpers around the multi-rank part of the method (no GPU work):
//   symi_grad_source / symi_collect_grads   the Symi Optimizer's gradient collection plan
//                                           (paper App. A.4, Algorithm 2; Sec. 4.3)
//   symi_rank_group                         index of a pre-registered group of consecutive
//                                           ranks (Sec. 4.2)
//   symi_comm_cost                          the memory / data volume / communication time
//                                           model of Sec. 3.3 and App. A.1, A.5
// Slot q of a placement lives on rank q / s, s = S_tot / N slots per rank.
#include <math.h>

#include <vector>

#include "common.h"

namespace symi {

// ranks hosting class exp_id, ascending (same-class slots are contiguous, but no such
// assumption is made here)
static void hosts_of(const int32_t* placement, int S_tot, int s, int exp_id, std::vector<int>& out) {
  out.clear();
  for (int q = 0; q < S_tot; ++q) {
    if (placement[q] != exp_id) continue;
    const int r = q / s;
    if (out.empty() || out.back() != r) out.push_back(r);
  }
}

static int source_of(const std::vector<int>& hosts, int rank) {
  for (int h : hosts)
    if (h == rank) return rank;                     // the optimizer's own rank hosts the class
  return hosts[rank % (int)hosts.size()];           // otherwise round robin over the hosts
}

static int check_plan_args(const symi_cfg* cfg, const int32_t* placement, int rank, const char* who) {
  if (int rc = check_cfg(cfg, who)) return rc;
  SYMI_REQUIRE(placement, who, "NULL pointer");
  SYMI_REQUIRE(cfg->S_tot % cfg->N == 0, who, "S_tot must be a multiple of N (s slots per rank)");
  SYMI_REQUIRE(rank >= 0 && rank < cfg->N, who, "rank outside [0, N)");
  for (int q = 0; q < cfg->S_tot; ++q)
    SYMI_REQUIRE(placement[q] >= 0 && placement[q] < cfg->E, who, "placement entry outside [0, E)");
  return SYMI_OK;
}

}  // namespace symi

using namespace symi;

extern "C" int symi_grad_source(const symi_cfg* cfg, const int32_t* placement, int exp_id, int rank) {
  if (int rc = check_plan_args(cfg, placement, rank, "symi_grad_source")) return rc;
  SYMI_REQUIRE(exp_id >= 0 && exp_id < cfg->E, "symi_grad_source", "exp_id outside [0, E)");
  std::vector<int> hosts;
  hosts_of(placement, cfg->S_tot, cfg->S_tot / cfg->N, exp_id, hosts);
  SYMI_REQUIRE(!hosts.empty(), "symi_grad_source", "class has no slot in this placement");
  return source_of(hosts, rank);
}

extern "C" int symi_collect_grads(const symi_cfg* cfg, const int32_t* placement, int rank,
                                  int32_t* recv_src, int32_t* send_offsets, int32_t* send_dst,
                                  int send_capacity) {
  if (int rc = check_plan_args(cfg, placement, rank, "symi_collect_grads")) return rc;
  SYMI_REQUIRE(recv_src && send_offsets && (send_dst || send_capacity == 0), "symi_collect_grads",
               "NULL pointer");
  const int E = cfg->E, N = cfg->N, s = cfg->S_tot / N;
  std::vector<int> hosts;
  int n_send = 0;
  for (int e = 0; e < E; ++e) {
    hosts_of(placement, cfg->S_tot, s, e, hosts);
    SYMI_REQUIRE(!hosts.empty(), "symi_collect_grads", "a class has no slot in this placement");
    recv_src[e] = source_of(hosts, rank);           // recv tuple (source, this rank's partition)
    send_offsets[e] = n_send;
    bool local = false;
    for (int h : hosts) local = local || h == rank;
    if (!local) continue;
    for (int dst = 0; dst < N; ++dst) {
      if (source_of(hosts, dst) != rank) continue;
      SYMI_REQUIRE(n_send < send_capacity, "symi_collect_grads", "send_capacity too small");
      send_dst[n_send++] = dst;                     // send tuple (dst, partition dst)
    }
  }
  send_offsets[E] = n_send;
  return n_send;
}

extern "C" int symi_rank_group(int N, int first_rank, int last_rank) {
  if (N < 1 || first_rank < 0 || last_rank >= N || first_rank >= last_rank) {
    set_error("symi_rank_group: need 0 <= first_rank < last_rank < N");
    return SYMI_EINVAL;
  }
  // groups of >= 2 consecutive ranks, ordered by first rank, then by last rank:
  // first ranks 0 .. f-1 own (N-1) + (N-2) + ... + (N-f) groups
  const long long before = (long long)first_rank * (N - 1) - (long long)first_rank * (first_rank - 1) / 2;
  const long long g = before + (last_rank - first_rank - 1);
  if (g > 2147483647LL) {
    set_error("symi_rank_group: group index does not fit an int");
    return SYMI_EUNSUPPORTED;
  }
  return (int)g;
}

extern "C" int symi_comm_cost(const symi_cost_in* in, symi_cost_out* out) {
  if (!in || !out) {
    set_error("symi_comm_cost: NULL pointer");
    return SYMI_EINVAL;
  }
  const double E = in->E, N = in->N, s = in->s;
  if (!(in->E >= 1 && in->N >= 1 && in->s >= 1 && (long long)in->s * in->N >= in->E && in->G >= 0 &&
        in->W >= 0 && in->O >= 0 && in->bw_pci > 0 && in->bw_net > 0)) {
    set_error("symi_comm_cost: need E, N, s >= 1, s*N >= E, sizes >= 0, bandwidths > 0");
    return SYMI_EINVAL;
  }
  // (I) optimizer memory: E * (1/r) * r * O = E * (1/N) * N * O
  out->mem_static = E * in->O;
  out->mem_symi = E * in->O;
  // (II) data moved per iteration: sum_i r_i * (G/N) * N with sum_i r_i = s N
  out->data_grad_static = s * N * in->G;
  out->data_weight_static = s * N * in->W;
  out->data_grad_symi = s * N * in->G;
  out->data_weight_symi = s * N * in->W;
  // (III) time: every rank moves E/N of a tensor over the host link and the rest of its
  // slots' share over the network; bw_pci = +inf is the non-offloaded optimizer
  const double pci_g = in->bw_pci == INFINITY ? 0.0 : E / N * in->G / in->bw_pci;
  const double pci_w = in->bw_pci == INFINITY ? 0.0 : E / N * in->W / in->bw_pci;
  out->t_grad_static = pci_g + (s * N - E) / N * in->G / in->bw_net;
  out->t_weight_static = pci_w + (s * N - E) / N * in->W / in->bw_net;
  out->t_grad_symi = pci_g + (s * N - s) / N * in->G / in->bw_net;
  out->t_weight_symi = pci_w + (s * N - s) / N * in->W / in->bw_net;
  const double ratio = in->bw_pci == INFINITY ? 0.0 : in->bw_net / in->bw_pci;
  const double den = s * N - E * (1.0 - ratio);
  out->extra_fraction = den > 0 ? (E - s) / den : 0.0;
  return SYMI_OK;
}
