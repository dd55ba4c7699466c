/*
 * sn_runtime.h -- C ABI of the host-side memory scheduling of SuperNeurons (arXiv 1801.04380):
 * what decides, step by step, how many bytes are free for the convolution workspaces that
 * sn.h's CONV calls are handed (Sec. 3.5: "the memory left for convolution workspaces constantly
 * changes in every steps according to Liveness Analysis, UTP and Cost-Aware Recomputation").
 *
 * Everything here is host code working on sizes and step numbers: no device memory is touched,
 * nothing is launched.  Objects are created and destroyed by the caller through the calls below
 * and are not thread-safe.
 *
 *  - sn_pool_*   the heap memory pool of Sec. 3.2.1 ("Toward a High Performance Liveness
 *                Analysis"): one preallocated region cut into 1 KB blocks, a list of empty and a
 *                list of allocated nodes, first fit, deallocation by node id.  The pool hands out
 *                OFFSETS into the caller's region.
 *  - sn_net_*    a network as layers with predecessor lists; its execution order (Alg. 1); the
 *                memory used at every forward / backward step under the baseline allocation,
 *                Liveness Analysis (Sec. 3.2), Offloading / Prefetching with the CONV outputs as
 *                checkpoints (Sec. 3.3.1) and Recomputation (Sec. 3.4: speed-centric,
 *                memory-centric, cost-aware); the free bytes per step for a device capacity; and the
 *                CONV algorithms the planner of sn.h picks under those per-step budgets (Sec. 3.5).
 *
 * Step numbering follows Sec. 4.1: with N layers after the data layer, forward step s (1..N) runs
 * the s-th layer of the execution order and backward step N + k runs the (N + 1 - k)-th.
 *
 * The accounting (which tensors exist, which step needs which) is the one that reproduces the
 * figures the paper prints for AlexNet at batch 200 (Sec. 4.1: 36 tensors / 2189.437 MB, 1489.355 MB
 * at step 32 with 17 tensors, 9 tensors at step 39; Table 1: 993.018 / 886.23 / 886.23 MB and
 * 14 / 23 / 17 extra forward computations):
 *  - a layer's backward needs: CONV, FC its input; ACT, LRN, POOL input and output; BN its input;
 *    SOFTMAX its output; DROPOUT, JOIN nothing.  The data tensor is needed by forward steps only.
 *  - every layer's backward writes the gradient of each input into a tensor of its own, except
 *    ACT and LRN (the gradient of the input replaces the gradient of the output) and SOFTMAX (the
 *    gradient of its input replaces its own output); the data has no gradient.
 *  - an offloaded CONV output is on the GPU in the forward until its consumers have run, and in
 *    the backward during the steps from step s down to the backward of the nearest CONV layer at
 *    or before it, if one of those steps needs it (directly, or to start a recomputation from).
 *  - recomputation drops the outputs of ACT, LRN, POOL, BN and DROPOUT after their forward
 *    consumers have run.  A segment is a maximal connected set of such tensors.
 */
#ifndef SN_RUNTIME_H
#define SN_RUNTIME_H

#include "sn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- memory pool (Sec. 3.2.1) ---------------------------------------------------------------- */
#define SN_POOL_BLOCK 1024

typedef struct sn_pool sn_pool;

/* A pool over `bytes` bytes (rounded down to whole blocks).  NULL if out of host memory. */
sn_pool *sn_pool_create(size_t bytes);
void sn_pool_destroy(sn_pool *pool);
/* First empty node with enough blocks (lowest offset first).  *id (> 0) names the allocation,
 * *offset is its place in the region (a multiple of 1 KB); 0 bytes take one block.
 * SN_ERR_WORKSPACE_TOO_SMALL if no empty node is large enough (nothing changes then). */
sn_status sn_pool_alloc(sn_pool *pool, size_t bytes, uint64_t *id, size_t *offset);
/* Puts the node back among the empty ones; neighbouring empty nodes merge.  SN_ERR_BAD_ARG for
 * an id that is not allocated. */
sn_status sn_pool_free(sn_pool *pool, uint64_t id);
size_t sn_pool_used_bytes(const sn_pool *pool);      /* blocks in use now, in bytes */
size_t sn_pool_peak_bytes(const sn_pool *pool);      /* the most that was in use at once */
size_t sn_pool_high_water(const sn_pool *pool);      /* highest offset + size ever handed out */
size_t sn_pool_largest_free(const sn_pool *pool);    /* largest empty node: what a workspace can get */

/* ---- network, execution order, memory per step ------------------------------------------------ */
typedef enum {
    SN_L_DATA = 0, SN_L_CONV = 1, SN_L_ACT = 2, SN_L_LRN = 3, SN_L_POOL = 4, SN_L_BN = 5, SN_L_FC = 6,
    SN_L_DROPOUT = 7, SN_L_SOFTMAX = 8, SN_L_JOIN = 9, SN_L_KINDS = 10
} sn_layer_kind;

/* Which of the paper's techniques are on (each includes the ones before it). */
typedef enum { SN_MEM_BASELINE = 0, SN_MEM_LIVENESS = 1, SN_MEM_OFFLOAD = 2, SN_MEM_RECOMPUTE = 3 } sn_mem_level;
typedef enum { SN_RECOMP_SPEED = 0, SN_RECOMP_MEMORY = 1, SN_RECOMP_COST_AWARE = 2 } sn_recomp_strategy;

typedef struct sn_net sn_net;

sn_net *sn_net_create(void);
void sn_net_destroy(sn_net *net);
/* Adds a layer whose output tensor has out_bytes bytes and which reads the outputs of the layers
 * prev[0 .. nprev-1] (ids returned by earlier calls; a DATA layer has none).  Returns the new
 * layer's id (0, 1, 2, ...) or -1 on a bad argument. */
int sn_net_add_layer(sn_net *net, sn_layer_kind kind, size_t out_bytes, const int *prev, int nprev);
/* The CONV geometry of a CONV layer, for sn_net_plan_convs. */
sn_status sn_net_set_conv_shape(sn_net *net, int layer, const sn_conv_shape *shape);
int sn_net_layers(const sn_net *net);
/* Alg. 1: the execution order, data layers included; route[i] = layer id.  Returns the number of
 * layers in the order (those reachable from the data layers), or -1 if cap is too small. */
int sn_net_route(const sn_net *net, int *route, int cap);
/* Number of steps of one iteration, 2 N. */
int sn_net_steps(const sn_net *net);

typedef struct {
    size_t peak_bytes;       /* the most allocated at any moment of the iteration */
    int32_t peak_step;       /* the first step (1-based) where that happens */
    int32_t tensors;         /* tensors the baseline allocates (forward outputs + gradient tensors) */
    int32_t extra_forward;   /* layers computed again in the backward pass */
    size_t l_peak;           /* RECOMPUTE: peak of the memory-centric schedule, the bar of cost-aware */
} sn_mem_summary;

/* Memory per step.  bytes_per_step / live_per_step (either may be NULL) receive sn_net_steps
 * values: the most bytes, and the most tensors, allocated at any moment of each step.
 * `strategy` matters at SN_MEM_RECOMPUTE only. */
sn_status sn_net_memory_trace(const sn_net *net, sn_mem_level level, sn_recomp_strategy strategy,
                              size_t *bytes_per_step, int32_t *live_per_step, sn_mem_summary *summary);

/* Sec. 3.5: the bytes left for workspaces at each step on a device with capacity_bytes for
 * tensors: capacity - bytes in use, 0 where the step does not even fit. */
sn_status sn_net_step_budgets(const sn_net *net, sn_mem_level level, sn_recomp_strategy strategy,
                              size_t capacity_bytes, size_t *free_per_step);

typedef struct {
    int32_t layer;                       /* CONV layer id */
    int32_t fwd_step, bwd_step;          /* its forward and backward step */
    size_t fwd_budget, bwd_budget;       /* free bytes at those steps */
    int32_t algo_fwd, algo_bwd_data, algo_bwd_filter;   /* sn_conv_algo the planner picks */
    size_t ws_fwd, ws_bwd_data, ws_bwd_filter;          /* workspace each will use (<= budget) */
} sn_conv_step_plan;

/* For every CONV layer with a shape, in execution order: the budgets at its two steps and what
 * sn_conv_plan picks under them (forward at the forward step; backward-data and backward-filter
 * each under the backward step's budget -- they run one after the other and share it).  Returns
 * the number of plans written, or -1 if cap is too small or an argument is bad. */
int sn_net_plan_convs(const sn_net *net, sn_mem_level level, sn_recomp_strategy strategy,
                      size_t capacity_bytes, sn_conv_step_plan *plans, int cap);

#ifdef __cplusplus
}
#endif
#endif /* SN_RUNTIME_H */
