/* Scale-plan generation (section 5.1 of the paper, on generating the scale plan online from the network topology):
 * host-only code, no GPU call.  Given the nodes of a cluster, which of them hold the parameters
 * and which are spare, it picks targets and emits serial forwarding chains S -> T1 -> T2 -> ...
 * along which layers are pushed one by one, each node forwarding layer k while receiving k+1.
 *
 * Network model (section 5.1, the paragraph that models the network between GPUs): GPUs joined by a scale-up
 * fabric form one node and transfers inside it are free; every GPU of a node has a link of
 * `gpu_bw` bytes/s (each direction) to the leaf switch `leaf`; two nodes move data at the smaller
 * of their aggregated bandwidths n_gpus * gpu_bw (each GPU pair carries 1/n of the bytes: the
 * paper's parallel sharded transfer), divided by `oversub` >= 1 when they sit under different leaves.
 *
 * Greedy steps (the paper's listing is a figure; these follow its prose):
 *   1. drop sources whose outgoing direction already carries serving traffic (out_busy); if none
 *      is left keep them all and report `interferes`;
 *   2. choose `n_targets` spare nodes: leaves that have a usable source first, then larger
 *      aggregated bandwidth, then lower id;
 *   3. in a leaf with usable sources every such source roots a chain (strongest first) and the
 *      leaf's targets (strongest first) are dealt to these chains in turn; a target in a leaf
 *      without a usable source joins the root that reaches it fastest (ties: fewer nodes already
 *      in that chain, then lower root id);
 *   4. inside a chain targets are ordered by decreasing link speed from the root (ties: lower id).
 * The tail of each chain forwards to nobody and has the slowest link: the candidate for live
 * scaling (section 5.2, the paragraph on which instances are selected for it).
 *
 * Time model reported with the plan: store-and-forward per layer,
 *   ready(k, l) = max(ready(k-1, l), ready(k, l-1)) + layer_bytes / bw(hop k),
 * the root holding every layer at time 0; `ready_s` is ready(k, n_layers - 1). */
#ifndef BLITZ_PLAN_H
#define BLITZ_PLAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { BZ_PLAN_SOURCE = 0, BZ_PLAN_SPARE = 1, BZ_PLAN_OTHER = 2 };

typedef struct bz_plan_node {
    int32_t id;         /* caller's identifier, unique, >= 0 */
    int32_t n_gpus;     /* >= 1 */
    int32_t leaf;
    int32_t role;       /* BZ_PLAN_* */
    int32_t out_busy;   /* nonzero: outgoing direction carries serving traffic */
    int32_t reserved_;
    double  gpu_bw;     /* bytes/s per GPU and direction, > 0 */
} bz_plan_node;

typedef struct bz_plan_hop {
    int32_t chain;      /* 0-based, chains ordered by root id */
    int32_t from;       /* node id that sends */
    int32_t to;         /* node id that receives */
    int32_t is_tail;    /* 1 for the last hop of its chain */
    double  bw;         /* bytes/s of this hop under the model */
    double  ready_s;    /* when `to` holds all n_layers layers */
} bz_plan_hop;

/* Writes the plan's hops (host memory, caller-owned, `max_hops` entries; exactly n_targets are
 * produced), chain by chain in forwarding order.  n_chains / interferes may be NULL.
 * Returns 0, BZ_EINVAL (-1: null pointers, duplicate or negative ids, n_gpus < 1, gpu_bw <= 0,
 * unknown role, oversub < 1, n_layers < 1, layer_bytes <= 0, n_targets < 1) or BZ_ECAPACITY
 * (-7: no source, fewer spare nodes than n_targets, or max_hops < n_targets). */
int bz_plan_generate(const bz_plan_node* nodes, int n_nodes, int n_targets, double oversub, int n_layers,
                     double layer_bytes, bz_plan_hop* hops, int max_hops, int* n_hops, int* n_chains,
                     int* interferes);

#ifdef __cplusplus
}
#endif
#endif
