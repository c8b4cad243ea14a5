/*
 * symi.h - C ABI of the Symi MoE hot path for MI355X (gfx950).
 *
 * One GPU's share of one adaptive-replication MoE training iteration
 * (Symi, arXiv 2504.19925, Sec. 3.2, Fig. 5 steps 1-8):
 *
 *   forward    symi_route -> symi_dispatch (or symi_dispatch_capacity) -> symi_expert_fwd -> symi_combine
 *   backward   symi_combine_bwd -> symi_expert_bwd -> symi_dispatch_bwd -> symi_route_bwd
 *   optimizer  symi_place (next placement, Algorithm 1) -> symi_adam_to_replicas
 *   set-up     symi_create (one context per MoE layer and optimizer partition) ... symi_destroy
 *   optional   symi_router_fwd before symi_route, symi_router_bwd after symi_route_bwd;
 *              symi_expert_bwd_slots + symi_replica_allreduce instead of symi_expert_bwd;
 *              symi_expert_bwd_active + symi_adam_to_replicas_active instead of the plain
 *              pair when many classes get no tokens;
 *              host helpers for the multi-rank plan at the end of this file
 *
 * Conventions
 *   - Every function returns 0 (SYMI_OK) or a negative error code; symi_last_error()
 *     returns a description of the most recent failure on the calling thread.
 *   - Unless a parameter says "host", every pointer is a DEVICE pointer owned by the
 *     caller, valid until the work enqueued on `stream` has finished.  The device calls
 *     allocate nothing, create nothing and never synchronise with the host: everything the
 *     library owns (the validated configuration, a helper stream and three events for the
 *     backward where the shape calls for them) is made by symi_create and lives in the opaque
 *     symi_ctx until symi_destroy.  There is no process-wide state: calls on different
 *     contexts may run on different threads; calls on one context must not overlap.
 *     The device calls can be captured into a HIP graph (no memsets, no host synchronisation).
 *   - `ctx` is a HOST pointer from symi_create; every device call checks that the device it
 *     was created on is the current one (SYMI_EINVAL otherwise).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - `cfg` and `hp` are HOST pointers, read during the call only.
 *   - Activations and slot weights are fp32 or bf16 according to cfg->dtype; routing
 *     data, gradients of the weights and the Adam state are always fp32; all index
 *     arrays are int32.  Matrices are row-major, the last index contiguous.
 *   - Notation (paper Table 2): E expert classes, S_tot = s*N replica slots, N
 *     optimizer partitions, T tokens, k choices per token, A = T*k assignments,
 *     d model width, f FFN width, P_e = 3*d*f parameters per expert.
 *   - Shape limits checked by symi_validate: 1 <= k <= min(E, 16), E <= 1024,
 *     E <= S_tot <= 4096, P_e divisible by N, 0 <= shard < N; d, f and P_e/N
 *     multiples of 8.  Beyond the launch limits of the kernels (SYMI_EUNSUPPORTED):
 *     T*k/256 + S_tot + 256 <= 65535 m-tiles (fp32: 4*(T*k/256 + S_tot) <= 65535),
 *     T/128 <= 65535, 2*f*d <= 2^31 - 8192, d <= 2^22, f <= 2^21.
 */
#ifndef SYMI_H
#define SYMI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SYMI_OK = 0, SYMI_EINVAL = -1, SYMI_EUNSUPPORTED = -2, SYMI_EHIP = -3 };
enum { SYMI_F32 = 0, SYMI_BF16 = 1 };

typedef struct symi_cfg {
  int T;      /* tokens in this GPU's batch */
  int E;      /* expert classes */
  int k;      /* choices per token (top-k) */
  int d;      /* model width */
  int f;      /* FFN (hidden) width of one SwiGLU expert */
  int S_tot;  /* replica slots = slots per rank * ranks (eq. (2): sum_i r_i = sN) */
  int N;      /* optimizer partitions (ranks) */
  int shard;  /* which partition this GPU owns, 0 <= shard < N */
  int dtype;  /* SYMI_F32 or SYMI_BF16: activations and slot weights */
  int renorm; /* 1: the k gates of a token are renormalised to sum to 1 */
} symi_cfg;

typedef struct symi_adam {
  float lr, beta1, beta2, eps, weight_decay, grad_scale;
  int step; /* 1-based iteration count used for bias correction */
} symi_adam;

/* Host-only checks of a configuration (no GPU needed). */
int symi_validate(const symi_cfg* cfg);

/* The per-layer state of Fig. 5 that is not a tensor: an opaque, immutable context holding the
 * validated configuration of one MoE layer and optimizer partition (cfg->shard) together with
 * what the library needs to run it on the CURRENT device (queried once: compute units; created
 * once: the helper stream and events of the expert backward, only when the shape makes the two
 * gradient chains worth two streams).  Host function; the only one that creates anything.
 *   flags: 0 or an OR of
 *     SYMI_CTX_NO_OVERLAP  every kernel of symi_expert_bwd* stays on the caller's stream
 *                          (default: the weight-gradient chain runs on the helper stream,
 *                          forked from and joined back into `stream` with events, when the
 *                          products are only a few rounds of workgroups: for the caller
 *                          everything is still ordered on `stream`);
 *     SYMI_CTX_NO_SLICING  the two narrow products (Yp = H W2^T, dXp = dUV W1) never cut the
 *                          reduction of their last round's tiles into slices (default: they
 *                          do when that round would leave at least half the compute units
 *                          idle, and add the slices up in a fixed order: same bits on every
 *                          run, not the bits of the uncut reduction);
 *     SYMI_CTX_TIMING      measurement aid, see symi_timing_read.
 *   Neither of the first two changes what is computed beyond rounding order.
 * Errors: SYMI_EINVAL / SYMI_EUNSUPPORTED as symi_validate, SYMI_EHIP without a usable device.
 * symi_destroy(NULL) is a no-op; destroying a context does not wait for work in flight: the
 * caller synchronises first. */
typedef struct symi_ctx symi_ctx;
enum { SYMI_CTX_NO_OVERLAP = 1, SYMI_CTX_NO_SLICING = 2, SYMI_CTX_TIMING = 4 };
int symi_create(const symi_cfg* cfg, unsigned flags, symi_ctx** out);
int symi_destroy(symi_ctx* ctx);
/* Bytes of device workspace `ws` that symi_dispatch / symi_expert_fwd /
 * symi_expert_bwd / symi_router_bwd need for this configuration (0 if cfg is invalid).
 * The workspace is scratch: nothing in it has to survive from one call to the next, its
 * contents need no initialisation, and two calls that may run at the same time (on different
 * streams) must not share one. */
size_t symi_workspace_bytes(const symi_cfg* cfg);
const char* symi_last_error(void);

/* Sec. 2.1 (top-k gating) + Sec. 3.2 step 1 (per-class token count, the popularity
 * array kept by the Layer Metadata Store).
 *   logits [T,E] f32 in.  idx [T,k] i32 out: the k best classes of each token, best
 *   first, equal scores resolved towards the lower class index.  gate [T,k] f32 out:
 *   softmax over all E classes evaluated at idx, divided by their sum if cfg->renorm.
 *   hist [E] i32 out: number of (token, choice) pairs per class; sums to T*k.       */
int symi_route(const symi_ctx* ctx, const float* logits, int32_t* idx, float* gate,
               int32_t* hist, void* stream);

/* Backward of the gating of Sec. 2.1 (softmax over all classes, top-k, optional
 * renormalisation) as symi_route evaluates it: dlogits [T,E] f32 out from dgate [T,k] f32
 * (the router is learned, Sec. 2.1, so its logits need a gradient). */
int symi_route_bwd(const symi_ctx* ctx, const float* logits, const int32_t* idx,
                   const float* gate, const float* dgate, float* dlogits, void* stream);

/* Expert Placement Scheduler, Algorithm 1 (App. A.3; Sec. 3.4), in exact integer
 * arithmetic: replicas proportional to popularity, at least one per class, exactly
 * S_tot in total, same-class slots contiguous.  First extremum wins ties; an all-zero
 * popularity is read as uniform.
 *   popularity [E] i32 in (normally the previous iteration's hist).
 *   counts [E] i32 out (r_i), placement [S_tot] i32 out (slot -> class),
 *   first_slot [E+1] i32 out (prefix sums of counts).                               */
int symi_place(const symi_ctx* ctx, const int32_t* popularity, int32_t* counts,
               int32_t* placement, int32_t* first_slot, void* stream);
/* Same computation on HOST pointers (the paper runs the scheduler on every rank's CPU). */
int symi_place_host(const symi_cfg* cfg, const int32_t* popularity, int32_t* counts,
                    int32_t* placement, int32_t* first_slot);

/* Sec. 3.2 step 2: tokens go to their classes, and the rows of a class are spread over
 * that class's replicas under the CURRENT placement (counts, first_slot).
 *   Assignment a = t*k + j.  Rows are assignments in stable class order; replica i of
 *   class e owns c_e*i/r_e .. c_e*(i+1)/r_e (integer division) of the class's c_e rows.
 *   X [T,d] in; idx [T,k], hist [E] (this iteration's), counts [E], first_slot [E+1] in.
 *   row_of_assign [A], assign_of_row [A], slot_offsets [S_tot+1] i32 out;
 *   Xp [A,d] out: Xp[row] = X[assign_of_row[row] / k].                              */
int symi_dispatch(const symi_ctx* ctx, const void* X, const int32_t* idx, const int32_t* hist,
                  const int32_t* counts, const int32_t* first_slot, int32_t* row_of_assign,
                  int32_t* assign_of_row, int32_t* slot_offsets, void* Xp, void* ws,
                  void* stream);

/* symi_dispatch for callers that cannot allocate or bring a workspace along: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs
 * and results as symi_dispatch, bit for bit; the scratch (per-chunk class counts) lives in a
 * buffer of SYMI_DISPATCH_NOALLOC_SCRATCH_BYTES that is part of the library's code object (one
 * copy per GPU, held until the process ends; its address on the context's device is looked up
 * by symi_create).  The call allocates nothing and creates nothing.
 *   Limit: (ceil(T*k/1024) + 1) * E * 4 + 12 * E bytes (each term rounded up to 256) must fit
 *   the buffer, else SYMI_EUNSUPPORTED; a context created with SYMI_CTX_TIMING is refused
 *   (SYMI_EINVAL: such a context creates events per launch).
 *   All calls on one GPU share the one buffer, whatever their context or stream: calls that may
 *   overlap in time on a GPU race.  Nothing in it has to start at zero (every entry read was
 *   written earlier in the same call), so its contents after a call do not matter to the next. */
#define SYMI_DISPATCH_NOALLOC_SCRATCH_BYTES (4u << 20)
int symi_dispatch_noalloc(const symi_ctx* ctx, const void* X, const int32_t* idx, const int32_t* hist,
                          const int32_t* counts, const int32_t* first_slot, int32_t* row_of_assign,
                          int32_t* assign_of_row, int32_t* slot_offsets, void* Xp, void* stream);

/* Expert capacity under adaptive replication (Sec. 3.4):
 *   slot_capacity = capacity_factor * tokens_per_batch / (s*N),  capacity(e_i) = slot_capacity * r_i.
 * HOST function: returns slot_capacity for cfg (tokens_per_batch = T*k assignments), the
 * product evaluated in binary64 as capacity_factor * (T*k) / S_tot and rounded up to whole
 * rows (at least 1); a negative error code if cfg or capacity_factor (<= 0) is invalid.  */
int symi_slot_capacity(const symi_cfg* cfg, double capacity_factor);

/* symi_dispatch with that capacity rule: of the hist[e] assignments of class e, the first
 * slot_capacity * counts[e] in stable (assignment id) order are kept, the rest are dropped.
 *   row_of_assign [A] out: row of a kept assignment, -1 for a dropped one;
 *   assign_of_row [A] out: entries [0, A') valid, A' = number of kept assignments;
 *   slot_offsets [S_tot+1] out over the kept rows (no slot exceeds slot_capacity rows),
 *   slot_offsets[S_tot] = A': the token survival rate of the iteration (Sec. 5.2) is A'/A;
 *   Xp [A,d] out: rows [0, A') written.
 * symi_expert_fwd/bwd work on slot_offsets and so on the kept rows only; symi_combine,
 * symi_combine_bwd and symi_dispatch_bwd skip dropped assignments (they contribute
 * nothing to Y, dX, and get dgate = 0); gates are not renormalised after a drop.        */
int symi_dispatch_capacity(const symi_ctx* ctx, int slot_capacity, const void* X, const int32_t* idx,
                           const int32_t* hist, const int32_t* counts, const int32_t* first_slot,
                           int32_t* row_of_assign, int32_t* assign_of_row, int32_t* slot_offsets,
                           void* Xp, void* ws, void* stream);

/* Backward of Sec. 3.2 step 2 (the scatter of tokens to their replicas; the all-to-all of
 * Sec. 2.1 run in reverse): dX[t] = sum_j dXp[row_of_assign[t*k+j]] (j ascending, fp32 sum). */
int symi_dispatch_bwd(const symi_ctx* ctx, const void* dXp, const int32_t* row_of_assign,
                      void* dX, void* stream);

/* Expert SwiGLU FFN over replica slots (Sec. 2.1; the expert compute of Fig. 5).
 * For slot q with rows [slot_offsets[q], slot_offsets[q+1]):
 *   u = x Wg^T, v = x Wu^T, h = silu(u)*v, y = h Wd^T
 *   W1_slots [S_tot,2f,d]: rows 0..f-1 = Wg, rows f..2f-1 = Wu; W2_slots [S_tot,d,f] = Wd.
 *   UV [A,2f] (u | v), H [A,f] and Yp [A,d] out (UV and H are kept for the backward). */
int symi_expert_fwd(const symi_ctx* ctx, const void* Xp, const int32_t* slot_offsets,
                    const void* W1_slots, const void* W2_slots, void* UV, void* H, void* Yp,
                    void* ws, void* stream);

/* Backward of symi_expert_fwd.  dXp [A,d] out.  dW1_class [E,2f,d], dW2_class [E,d,f]
 * f32 out: the gradient of each class summed over ALL its rows, i.e. over all its
 * replica slots (the intra-rank part of the gradient all-reduce of Sec. 4.1); a class
 * without rows gets zeros.  first_slot [E+1] is the placement used by symi_dispatch. */
int symi_expert_bwd(const symi_ctx* ctx, const void* dYp, const void* Xp, const void* UV,
                    const void* H, const int32_t* slot_offsets, const int32_t* first_slot,
                    const void* W1_slots, const void* W2_slots, void* dXp, float* dW1_class,
                    float* dW2_class, void* ws, void* stream);

/* Sec. 2.1: the expert outputs return to their tokens (the gather all-to-all) and are mixed
 * with the gate weights: Y[t] = sum_j gate[t,j] * Yp[row_of_assign[t*k+j]], j ascending,
 * accumulated in fp32.  Y [T,d] out. */
int symi_combine(const symi_ctx* ctx, const void* Yp, const int32_t* row_of_assign,
                 const float* gate, void* Y, void* stream);

/* Backward of that gather and mix (Sec. 2.1; the all-to-all scatter of the backward pass):
 * dYp[row] = gate[t,j]*dY[t]; dgate[t,j] = <dY[t], Yp[row]>. */
int symi_combine_bwd(const symi_ctx* ctx, const void* dY, const void* Yp,
                     const int32_t* row_of_assign, const float* gate, void* dYp, float* dgate,
                     void* stream);

/* Sec. 3.2 steps 4-8 for optimizer partition cfg->shard (Symi Optimizer: static uniform
 * partition, Sec. 3.1/3.3; weight communication phase, Sec. 4.4).  The flat parameter
 * vector of a class is [W1 (2f*d) | W2 (d*f)]; partition n owns its range
 * [n*P_e/N, (n+1)*P_e/N).  On that range, for every class: Adam with bias correction
 * (eps outside the root, decoupled weight decay) on master_w, m, v [E, P_e/N] f32
 * (in/out) from grad_scale * dW_class; then the fresh weights, rounded to nearest-even
 * bf16 if cfg->dtype is bf16, are written into the same range of every slot
 * first_slot_next[e] .. first_slot_next[e+1]-1 of W1_slots / W2_slots: the placement of
 * the NEXT iteration.  Bytes written to slots are S_tot*P_e/N*sizeof(weight), whatever
 * the placement.  hp is a HOST pointer. */
int symi_adam_to_replicas(const symi_ctx* ctx, const symi_adam* hp, const float* dW1_class,
                          const float* dW2_class, float* master_w, float* m, float* v,
                          const int32_t* first_slot_next, void* W1_slots, void* W2_slots,
                          void* stream);

/* The gate network in front of symi_route (Sec. 2.1: a learned router scores every token
 * against every expert class), so that the layer is closed from X to dX:
 *   logits [T,E] f32 out = X Wr^T + b.   X [T,d], Wr [E,d] in the activation dtype (row e of
 *   Wr is class e's scoring vector), b [E] f32 or NULL.                                   */
int symi_router_fwd(const symi_ctx* ctx, const void* X, const void* Wr, const float* b,
                    float* logits, void* stream);

/* Backward of symi_router_fwd from dlogits [T,E] f32 (symi_route_bwd's output):
 *   dWr [E,d] f32 out = dlogits^T X;  db [E] f32 out = column sums of dlogits (NULL: skipped);
 *   dX [T,d] IN/OUT: dlogits Wr is ADDED to it (call after symi_dispatch_bwd).
 * Deterministic: the reduction over tokens is cut into fixed chunks summed in order.      */
int symi_router_bwd(const symi_ctx* ctx, const void* X, const void* Wr, const float* dlogits,
                    float* dWr, float* db, void* dX, void* ws, void* stream);

/* The same two calls for a batch that leaves many classes without tokens.  A rank of the
 * paper only ever forms gradients for the classes it hosts (Sec. 4.1; Algorithm 2 collects a
 * shard from a hosting rank), and a class no token chose contributes a zero gradient to the
 * optimizer step (Sec. 3.2 steps 4-6).  With one GPU standing in for all slots, writing
 * those zeros and reading them back is traffic the method does not have:
 *   symi_expert_bwd_active = symi_expert_bwd, except that dW1_class[e], dW2_class[e] of a class
 *     e without rows (slot_offsets[first_slot[e+1]] == slot_offsets[first_slot[e]]) are left
 *     UNTOUCHED (whatever the buffers held stays there);
 *   symi_adam_to_replicas_active = symi_adam_to_replicas, except that the gradient of such a
 *     class is taken as zero and its memory is not read.  slot_offsets [S_tot+1] and
 *     first_slot [E+1] are those of the iteration the gradients come from (device pointers).
 * Together they give bit for bit the master_w, m, v and slots of the plain pair.          */
int symi_expert_bwd_active(const symi_ctx* ctx, const void* dYp, const void* Xp, const void* UV,
                           const void* H, const int32_t* slot_offsets, const int32_t* first_slot,
                           const void* W1_slots, const void* W2_slots, void* dXp,
                           float* dW1_class, float* dW2_class, void* ws, void* stream);
int symi_adam_to_replicas_active(const symi_ctx* ctx, const symi_adam* hp, const float* dW1_class,
                                 const float* dW2_class, float* master_w, float* m, float* v,
                                 const int32_t* slot_offsets, const int32_t* first_slot,
                                 const int32_t* first_slot_next, void* W1_slots, void* W2_slots,
                                 void* stream);

/* The replica gradient path as the paper draws it (Sec. 4.1, Fig. 7), as an alternative to
 * symi_expert_bwd's fused per-class sum.  symi_expert_bwd_slots is symi_expert_bwd with one
 * weight gradient per replica SLOT, summed over that slot's own rows only:
 *   dW1_slot [S_tot,2f,d], dW2_slot [S_tot,d,f] f32 out (a slot without rows gets zeros).  */
int symi_expert_bwd_slots(const symi_ctx* ctx, const void* dYp, const void* Xp, const void* UV,
                          const void* H, const int32_t* slot_offsets, const int32_t* first_slot,
                          const void* W1_slots, const void* W2_slots, void* dXp, float* dW1_slot,
                          float* dW2_slot, void* ws, void* stream);

/* The intra-rank part of the inter+intra-rank all-reduce (Sec. 4.1 steps 1 and 3; step 2,
 * the exchange between ranks, has nothing to do on one GPU): for every class the first of
 * its slots is the representative, the class's other slots add their tensor to it in slot
 * order, the sum is multiplied by `scale` (the paper "normalizes" without stating the
 * divisor: pass 1 for the plain sum, 1/r or 1/N for an average) and copied to all of the
 * class's slots.  In place on dW1_slot [S_tot,2f,d], dW2_slot [S_tot,d,f] f32.          */
int symi_replica_allreduce(const symi_ctx* ctx, const int32_t* first_slot, float scale,
                           float* dW1_slot, float* dW2_slot, void* stream);

/* ---- host helpers for the multi-rank part of the method (no GPU work; all pointers HOST).
 * Slot q of a placement lives on rank q / s, s = S_tot / N (S_tot must divide by N). */

/* Gradient collection, Algorithm 2 (App. A.4; Sec. 4.3): the one rank that sends the
 * gradient shard of class exp_id to the optimizer partition on `rank`: `rank` itself if
 * it hosts the class, else host number (rank mod #hosts) of the ascending list of ranks
 * hosting it.  Returns the source rank (>= 0) or a negative error code.              */
int symi_grad_source(const symi_cfg* cfg, const int32_t* placement, int exp_id, int rank);

/* The communication tuples of `rank` for one iteration (Algorithm 2, collect_grads):
 *   recv_src [E] out: rank r receives the shard of class e for its partition from recv_src[e];
 *   send_offsets [E+1], send_dst [send_capacity] out: for a class e hosted on `rank`, the
 *   destinations send_dst[send_offsets[e] .. send_offsets[e+1]) whose partition this rank
 *   serves (ascending; empty for classes not hosted here).
 * Returns the number of send tuples, or a negative error code (SYMI_EINVAL also when
 * send_capacity is too small; N entries per hosted class always suffice).            */
int symi_collect_grads(const symi_cfg* cfg, const int32_t* placement, int rank, int32_t* recv_src,
                       int32_t* send_offsets, int32_t* send_dst, int send_capacity);

/* Communication group management (Sec. 4.2): index in [0, N(N-1)/2) of the pre-registered
 * group made of the consecutive ranks first_rank .. last_rank (first_rank < last_rank),
 * groups ordered by first rank, then by last rank.                                    */
int symi_rank_group(int N, int first_rank, int last_rank);

/* The cost model of Sec. 3.3 (App. A.1; App. A.5 with bw_pci = INFINITY).  Sizes in bytes
 * (or any one unit), bandwidths in that unit per second.                              */
typedef struct {
  int E, N, s;            /* expert classes, ranks, slots per rank                        */
  double G, W, O;         /* gradient, weight and optimizer-state size of ONE expert      */
  double bw_pci, bw_net;  /* host link and network bandwidth per rank                     */
} symi_cost_in;
typedef struct {
  double mem_static, mem_symi;                  /* (I)  optimizer memory, whole cluster   */
  double data_grad_static, data_weight_static;  /* (II) data moved per iteration          */
  double data_grad_symi, data_weight_symi;
  double t_grad_static, t_weight_static;        /* (III) time of the two phases per rank  */
  double t_grad_symi, t_weight_symi;
  double extra_fraction;                        /* (T_symi - T_static) / T_static, G = W  */
} symi_cost_out;
int symi_comm_cost(const symi_cost_in* in, symi_cost_out* out);

/* Measurement aid (not part of the method): every kernel launched through a context created
 * with SYMI_CTX_TIMING is bracketed by two HIP events recorded on the launch stream, so that a
 * benchmark can read per-kernel durations of its own timed region (such a context creates two
 * events per launch: a host-side allocation).  Kernel ids run from 0 to symi_kernel_count()-1
 * and have the names symi_kernel_name() returns.  symi_timing_read waits for the recorded
 * events of that kernel and returns the summed duration in milliseconds and the number of
 * launches since the last symi_timing_reset.  Host pointers. */
int symi_timing_reset(const symi_ctx* ctx);
int symi_timing_read(const symi_ctx* ctx, int kernel_id, double* total_ms, int* launches);
int symi_kernel_count(void);
const char* symi_kernel_name(int kernel_id);

#ifdef __cplusplus
}
#endif
#endif /* SYMI_H */
