/*
 * semmoe.h - C ABI of the semantic-parallel MoE layer hot path for AMD MI355X (gfx950).
 *
 * One MoE layer of Sem-MoE ("Semantic Parallelism", arxiv 2503.04398) on one GPU, with the
 * expert-parallel ranks simulated as D expert-placement groups:
 *
 *   route -> [coact_hist -> place : offline] -> reshuffle -> dispatch -> expert_ffn -> combine
 *
 * Conventions
 *   - Every function returns a status: SEMMOE_OK or a negative SEMMOE_E* code.  Arguments are
 *     validated before anything is launched, so argument errors need no GPU.
 *   - "dev" pointers are device memory, "host" pointers host memory.  The caller owns every
 *     buffer and the library allocates nothing.  Scratch comes from the caller's workspace `ws`
 *     of at least semmoe_workspace_bytes() bytes, 256-byte aligned; calls on one stream may
 *     share it.
 *   - No result depends on an earlier call.  What the library does keep between calls, all of it
 *     safe to use from several threads: per device, its compute-unit count and LDS limit (looked
 *     up once) and which kernels already had their LDS limit raised there; per thread, the last
 *     HIP error; per process, the tuning knobs of semmoe_set_tuning (tests and sweeps: a knob set
 *     by one thread changes the kernel choice of every thread); per device, the address of the
 *     fixed scratch array of semmoe_reshuffle_static.  The current device must be the device of
 *     `stream` and of the buffers.
 *   - Device calls enqueue on `stream` (a hipStream_t passed as void*; NULL = default stream)
 *     and return without synchronising.  Calls that share a workspace must not overlap.
 *   - Activations and weights ("act" type) are fp32 or bf16 as cfg->dtype says, row-major,
 *     rows 16-byte aligned (d % 8 == 0 and F % 8 == 0).  Index arrays are int32.
 *   - Notation: T tokens, d hidden width, E routed experts, k experts per token, F expert FFN
 *     width, D logical ranks, m = E/D experts per rank, P = T*k (token, expert) pairs;
 *     pair index p = i*k + j (token i, choice j).  "Physical" expert q = position of an expert
 *     after placement (rank-major: rank of q is q / m).
 */
#ifndef SEMMOE_H
#define SEMMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SEMMOE_OK 0
#define SEMMOE_EINVAL (-1)       /* null / negative / misaligned argument */
#define SEMMOE_ESHAPE (-2)       /* inconsistent shapes: E % D, k > E, cap*D < T, d % 8, groups ... */
#define SEMMOE_EWORKSPACE (-3)   /* workspace missing or too small */
#define SEMMOE_EHIP (-4)         /* a HIP call failed; see semmoe_last_hip_error() */
#define SEMMOE_EUNSUPPORTED (-5) /* dtype / score mode / size outside what the kernels cover */

#define SEMMOE_FP32 0
#define SEMMOE_BF16 1
#define SEMMOE_SOFTMAX 0
#define SEMMOE_SIGMOID 1

/* Limits of the kernels (validated): */
#define SEMMOE_MAX_E 512 /* experts */
#define SEMMOE_MAX_K 16  /* experts per token */
#define SEMMOE_MAX_D 64  /* logical ranks */

typedef struct semmoe_config {
  int32_t T, d, E, k, F, D;
  int32_t dtype;       /* SEMMOE_FP32 | SEMMOE_BF16 */
  int32_t score;       /* SEMMOE_SOFTMAX | SEMMOE_SIGMOID */
  int32_t renorm;      /* divide the k weights by their sum */
  int32_t n_group;     /* sigmoid mode: expert groups (1 = no group limit); E % n_group == 0 */
  int32_t topk_group;  /* sigmoid mode: groups kept */
  float routed_scale;  /* sigmoid mode: factor on the weights */
  int32_t cap;         /* reshuffle: tokens per rank at most; cap * D >= T */
  int32_t num_classes; /* rows of class_bias (0 when unused) */
} semmoe_config;

int32_t semmoe_version(void);
/* hipError_t of the last failed HIP call on this thread (0 if none). */
int32_t semmoe_last_hip_error(void);
/* Workspace size that covers every device call below for this config. */
int32_t semmoe_workspace_bytes(const semmoe_config* cfg, size_t* bytes_out /*host*/);

/*
 * Tuning knobs for tests and sweeps.  Process-wide state: a knob holds until it is set again and applies to every
 * call of every thread (each knob is one atomic integer; a call reads the knobs it needs once, when it picks its
 * kernels).  value < 0 restores the default, which the library picks per shape.  Results never depend on them beyond
 * fp32 summation order inside a GEMM tile.  semmoe_get_tuning reads a knob back (-1: default).
 *   SEMMOE_TUNE_GATEUP_TILE / SEMMOE_TUNE_DOWN_TILE: tile-shape id of the bf16 grouped GEMMs
 *     (0, 3, 4, 6: register-staged; 11, 12, 14, 15, 16: direct-to-LDS ring; 17, 18: skinny register-staged tiles;
 *     19, 25, 26, 27: skinny tiles with a direct-to-LDS ring for decode;
 *     28: 128 x 128 pieces throughout (the default when 256 x 256 tiles would fill less than half the compute units);
 *     20, 21, 22: four waves on a 256 x 256 tile with loads placed between the MFMAs; K must be a multiple of the
 *     K slice (32 for 20 and 21, 64 for 22) and hold at least a ring of slices (128); other K run as 16)
 *   SEMMOE_TUNE_BLOCKS_PER_CU: persistent workgroups per compute unit for those GEMMs
 *   SEMMOE_TUNE_HEAD_TAIL: with the 256 x 256 tile shapes (16, 20, 21, 22) a GEMM runs as two launches: the tiles that
 *     fill whole rounds of the persistent grid, then the rest as quarter tiles over the whole chip, when at most
 *     value/16 of a round is left over (default 8); 0 = always one launch
 *   SEMMOE_TUNE_TAIL_RING: how the rest is run.  Default: 128 x 128 pieces with the loads placed between the MFMAs, in
 *     the same launch as the big tiles (a workgroup takes pieces once its tiles are done; 128 x 64 pieces instead when
 *     so few tiles are left over that they fit the grid once; K a multiple of 64 with at least three slices, else
 *     the next).  2: the same without the smaller pieces.  1: 128 x 128 pieces as a second launch.  3 or 6: a second launch of
 *     128 x 64 pieces with the loads of a slice issued in a burst and an LDS ring of 3 (two workgroups per compute
 *     unit) or 6 (one)
 *   SEMMOE_TUNE_ROUTE_SPLIT: bf16 router with at most 512 tokens: parts the K dimension is split into over workgroups
 *     (partial sums added in order by a second kernel, then the selection kernel); 0 = always the fused kernel,
 *     default: as many parts as fill the chip, at most 16.  With more than 128 experts, where tiles of 256 tokens
 *     times up to 8 parts of K (at least 8 slices each) fill three quarters of the compute units, the logits come from
 *     the 256 x 256 tile of the grouped GEMM, followed by one kernel that adds the parts and selects; 100 + n forces
 *     that form with n parts at any token count (d must be n parts of whole 64-element slices, at least two each),
 *     0 switches it off too
 *   SEMMOE_TUNE_GRID_CAP: most workgroups a grouped GEMM launches (default: compute units x blocks per CU)
 *   SEMMOE_TUNE_INDEX_PATH: which implementation of the index kernels runs (default: single workgroup for
 *     T <= 2048; above, two launches per call in which every workgroup derives its prefixes from the table of
 *     per-workgroup counts, up to T = 131072; beyond, one kernel per phase); the single-workgroup kernels hold at
 *     most T = 32768; all give identical results
 */
#define SEMMOE_TUNE_GATEUP_TILE 0
#define SEMMOE_TUNE_DOWN_TILE 1
#define SEMMOE_TUNE_BLOCKS_PER_CU 2
#define SEMMOE_TUNE_INDEX_PATH 3 /* reshuffle / dispatch index: 1 = one kernel per phase, 2 = single workgroup, 3 = two launches */
#define SEMMOE_TUNE_HEAD_TAIL 5  /* 0: one launch per GEMM; default: big tiles for the full rounds + quarter tiles */
#define SEMMOE_TUNE_TAIL_RING 6  /* tail: default 128 x 128 pieces in the head's launch; 1: as a second launch; 3, 6: 128 x 64 pieces */
#define SEMMOE_TUNE_ROUTE_SPLIT 7 /* parts of K in the few-token router; 0 = fused kernel */
#define SEMMOE_TUNE_GRID_CAP 4   /* upper limit of the persistent GEMM grids (tests: many tiles per workgroup) */
int32_t semmoe_set_tuning(int32_t key, int32_t value);
int32_t semmoe_get_tuning(int32_t key, int32_t* value_out /*host*/);

/*
 * route - the gating function G(h) = top-k(softmax(W_g h + b_g)) of Sec. 3.2.
 *   logits[i,e] = sum_c X[i,c] W_r[e,c] + b_g[e] + class_bias[token_class[i], e]   (fp32 accumulate;
 *   token_class[i] < 0 adds nothing; the class term is the synthetic token->expert affinity).
 *   Selection and weights: see semmoe_route_from_logits.
 * dev in : X[T,d] act; W_r[E,d] act (one row per expert); b_g[E] f32 or NULL; token_class[T] i32
 *          and class_bias[num_classes,E] f32, both or neither; sel_bias[E] f32 or NULL.
 * dev out: logits_out[T,E] f32 or NULL (then the logits live in the workspace only);
 *          topk_ids[T,k] i32; topk_w[T,k] f32.
 */
int32_t semmoe_route(const semmoe_config* cfg, void* stream, const void* X, const void* W_r, const float* b_g,
                     const int32_t* token_class, const float* class_bias, const float* sel_bias,
                     float* logits_out, int32_t* topk_ids, float* topk_w, void* ws, size_t ws_bytes);

/*
 * route_from_logits - the selection half of the gating function (Sec. 3.2) on given fp32 logits.
 *   softmax: the k largest logits, descending, equal logits -> lower expert id; weight = softmax over
 *     all E at the chosen ids, divided by their sum if cfg->renorm.
 *   sigmoid: s = sigmoid(logit) evaluated as the fixed fp32 sequence  x=clamp(logit,-30,30);
 *     t=(-x)*log2e; n=rint(t); f=t-n; p=c6; p=p*f+c_i (i=5..0, product and sum rounded separately,
 *     c_i = ln2^i/i!); z=p*2^n; s=1/(1+z).  s' = s + sel_bias.  Experts form n_group contiguous groups;
 *     group score = sum of its two largest s'; the topk_group best groups are kept (equal -> lower
 *     group); the k largest s' among their experts are chosen (equal -> lower id); weight =
 *     s[id] (/ sum of the k if cfg->renorm) * routed_scale.
 * dev in : logits[T,E] f32 (finite); sel_bias[E] f32 or NULL.   dev out: topk_ids[T,k], topk_w[T,k].
 */
int32_t semmoe_route_from_logits(const semmoe_config* cfg, void* stream, const float* logits,
                                 const float* sel_bias, int32_t* topk_ids, float* topk_w);

/*
 * coact_hist - token->expert activation counts of Sec. 3.2 in key-free form, and the expert-expert
 * affinity that Alg. 1 consumes:  load[e] += #{(i,j): ids[i,j]=e};
 * coact[a,b] += #{i: a in ids[i] and b in ids[i]} for all ordered (a,b), a=b included.
 * ACCUMULATES: the caller zeroes load/coact before the first batch of a profile.
 * dev in : topk_ids[T_batch,k] (ids of one token distinct, in [0,E)).  dev in/out: load[E] u32, coact[E,E] u32.
 * cfg->T is ignored; T_batch >= 0 is the batch length.
 */
int32_t semmoe_coact_hist(const semmoe_config* cfg, void* stream, const int32_t* topk_ids, int32_t T_batch,
                          uint32_t* load, uint32_t* coact);

/*
 * place - Alg. 1 `expert_place` (App. B), request-affinity term dropped; HOST function, synchronous.
 *   Experts by load descending (equal -> lower id); expert e goes to the not-yet-full rank c maximising
 *   alpha*sum_{e' on c} coact[e,e'] - gamma*loads_cls[c] (equal -> smaller loads_cls, then smaller c);
 *   a rank is full at E/D experts.  Then at most ft_passes first-improvement sweeps over pairs e1<e2 on
 *   different ranks, swapping when alpha*(rise of the intra-rank co-activation mass) + gamma*(what the swap
 *   takes off the larger of the two ranks' loads) > 0 - both terms of the objective of Sec. 3.3 with the weights
 *   of the greedy pass; gamma = 0: the affinity gain alone; stops after a sweep with no swap.
 *   Physical order: rank-major, ascending original id inside a rank (the transparent gate-column shuffle
 *   of Sec. 3.3 "Model scheduling" is phys_of_expert).
 * host in : load[E] u64, coact[E*E] u64 (symmetric).  host out: expert_to_rank[E], phys_of_expert[E],
 *           expert_of_phys[E] i32.
 */
int32_t semmoe_place(const semmoe_config* cfg, const uint64_t* load, const uint64_t* coact, int64_t alpha,
                     int64_t gamma, int32_t ft_passes, int32_t* expert_to_rank, int32_t* phys_of_expert,
                     int32_t* expert_of_phys);

/*
 * coschedule - the model-data co-scheduling solver, Alg. 1 whole (App. B): the alternation of `expert_place` with its
 * request term and `req_sched`, for the co-clustering objective of Sec. 3.3.  HOST function, synchronous.
 * A unit is a request of the profiling set (or a token key standing for all its occurrences): unit_act[u,e] is its
 * activation mass on expert e (e.g. `semmoe_token_expert_hist` keyed by request number), unit_len[u] its tokens.
 *   expert_place(unit_rank): as `semmoe_place`, with score = alpha_e*EAfE[e,c] + beta_e*EAfR[e,c] - gamma_e*loads_cls[c],
 *     EAfR[e,c] = sum of unit_act[u,e] over the units scheduled to c; a fine-tuning swap is taken when
 *     alpha_e*(gain of intra-cluster co-activation mass) + beta_e*(gain of local activation mass) > 0.
 *   req_sched(placement): units longest first (equal -> lower index); unit u goes to the not-yet-full cluster c
 *     maximising alpha_r*RAfR[u,c] + beta_r*RAfE[u,c], RAfR = sum over units u' already on c of
 *     sum_e unit_act[u,e]*unit_act[u',e], RAfE = sum of unit_act[u,e] over c's experts (equal -> the cluster with fewer
 *     tokens so far, then smaller c); a cluster is full at ceil(U/D) units.
 *   Start: expert_place with no unit scheduled, then req_sched.  Then n_steps times expert_place, req_sched and
 *     score = w_load*(most tokens on a cluster) + w_comm*(activation mass whose expert is on another cluster than its
 *     unit); the pair of the lowest score is returned (equal -> the earlier step).
 * Exact integer arithmetic; total mass and total length must stay below 2^40 and every weight within +-2^20
 * (SEMMOE_EUNSUPPORTED otherwise).
 * host in : load[E], coact[E*E], unit_act[U*E], unit_len[U] u64; params.  host out: expert_to_rank[E],
 *           phys_of_expert[E], expert_of_phys[E], unit_rank[U] i32; step_score[n_steps] i64 and best_step (both may
 *           be NULL).
 */
typedef struct semmoe_cosched_params {
  int64_t alpha_e, beta_e, gamma_e; /* weights of expert_place */
  int64_t alpha_r, beta_r;          /* weights of req_sched */
  int64_t w_load, w_comm;           /* weights of the score, >= 0 */
  int32_t ft_passes;                /* fine-tuning sweeps per expert_place, >= 0 */
  int32_t n_steps;                  /* alternations, >= 1 */
} semmoe_cosched_params;

int32_t semmoe_coschedule(const semmoe_config* cfg, const uint64_t* load, const uint64_t* coact,
                          const uint64_t* unit_act, const uint64_t* unit_len, int32_t U,
                          const semmoe_cosched_params* params, int32_t* expert_to_rank, int32_t* phys_of_expert,
                          int32_t* expert_of_phys, int32_t* unit_rank, int64_t* step_score, int32_t* best_step);

/*
 * token_labels - the last lines of Alg. 1: per token key, the number of its occurrences in requests scheduled to each
 * cluster; label dev[v] = the cluster of the highest count (equal -> smallest), conf_q16[v] = floor(65536 * share of
 * that count), level[v] = share * k rounded half up (same forms as `semmoe_lookup_tables`, and usable in its place);
 * a key that never occurs gets dev = -1, conf_q16 = level = 0.  Keys outside [0,V) are skipped.  HOST function.
 * host in : req_offsets[n_req+1] (starts at 0, non-decreasing), token_key[req_offsets[n_req]], req_rank[n_req] in
 *           [0,D).  host out: dev[V], conf_q16[V], level[V] i32.
 */
int32_t semmoe_token_labels(const semmoe_config* cfg, const int32_t* req_offsets, int32_t n_req,
                            const int32_t* token_key, const int32_t* req_rank, int32_t V, int32_t* dev,
                            int32_t* conf_q16, int32_t* level);

/*
 * token_expert_hist - the token-to-expert activation table of Sec. 3.2, built while profiling:
 * table[v,e] += #{(i,j): token_key[i] = v and ids[i,j] = e}.  ACCUMULATES over batches: the caller zeroes the table
 * before the first one.  Pairs whose key lies outside [0,V) or whose expert lies outside [0,E) are skipped.
 * dev in : token_key[T_batch] i32, topk_ids[T_batch,k].  dev in/out: table[V,E] u32.  cfg->T is ignored.
 */
int32_t semmoe_token_expert_hist(const semmoe_config* cfg, void* stream, const int32_t* token_key,
                                 const int32_t* topk_ids, int32_t T_batch, int32_t V, uint32_t* table);

/*
 * lookup_tables - the token-to-device schedule table and its confidence (the tables T and T_p read by Alg. 2 and
 * Alg. 3) from the activation table and a placement; offline, on the host.  With the confidence of Sec. 3.2,
 * C_p[v,e] = table[v,e] / sum_e table[v,e], the probability that an activation of key v lands on rank r is
 * mass[v,r] / tot[v] with mass[v,r] = sum of table[v,e] over the experts of r.  In integers:
 *   dev[v] = argmax_r mass[v,r] (equal -> smallest r);  conf_q16[v] = floor(65536 * mass[v,dev[v]] / tot[v]);
 *   level[v] = floor((2 k mass[v,dev[v]] + tot[v]) / (2 tot[v])), the expected number of the token's k activations on
 *   that rank rounded half up: the keep priority, in [0,k].  A key with tot[v] = 0 gets dev = -1, conf_q16 = level = 0.
 * host in : table[V,E] u32, expert_to_rank[E] (each in [0,D), else SEMMOE_EINVAL).  host out: dev[V], conf_q16[V],
 *           level[V] i32.
 */
int32_t semmoe_lookup_tables(const semmoe_config* cfg, const uint32_t* table, const int32_t* expert_to_rank, int32_t V,
                             int32_t* dev, int32_t* conf_q16, int32_t* level);

/*
 * reshuffle - Alg. 3 `rebatch_tokens` (device ids, argsort, group_by_key, align, concat) with the
 * device id taken from the token's actual top-k:  g[i,r] = #{j: expert_to_rank[ids[i,j]] = r};
 * pref(i) = argmax_r g[i,r] (equal -> home(i) = i / ceil(T/D) if it is a maximiser, else the smallest);
 * conf(i) = g[i,pref(i)].  Keep: per rank the candidates ordered by (conf desc, i asc), the first cap stay.
 * Spill ("align"): the s-th spilled token (ascending i) takes the s-th free slot, ranks ascending.
 * shf = tokens stably sorted by token_rank (new position -> token); inv_shf[shf[q]] = q (`resume_tokens`).
 * dev in : topk_ids[T,k], expert_to_rank[E].  dev out: token_rank[T], shf[T], inv_shf[T], rank_count[D].
 */
int32_t semmoe_reshuffle(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                         const int32_t* expert_to_rank, int32_t* token_rank, int32_t* shf, int32_t* inv_shf,
                         int32_t* rank_count, void* ws, size_t ws_bytes);

/*
 * reshuffle_static - semmoe_reshuffle for callers that cannot allocate or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without `ws`, same kernels,
 * same results bit for bit; the scratch is a fixed array of SEMMOE_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (each GPU the library runs on holds its own copy until the process ends).  The call makes
 * no allocation of any kind.  The first call on a device looks the array's address up (the device of `stream` must
 * be the current device, as for every call here).
 * Limits: semmoe_workspace_bytes()'s reshuffle share must fit the array, which covers T = 131072 tokens at
 * D = 32, k = 8 and every workload of this library's benchmark; beyond, SEMMOE_EUNSUPPORTED is returned before
 * anything is launched.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race and give wrong results; calls in stream order on one stream are safe.  Nothing has to
 * be cleared between calls: no kernel reads scratch it has not written in the same call.
 */
#define SEMMOE_STATIC_SCRATCH_BYTES (4u << 20)
int32_t semmoe_reshuffle_static(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                const int32_t* expert_to_rank, int32_t* token_rank, int32_t* shf, int32_t* inv_shf,
                                int32_t* rank_count);

/*
 * reshuffle with gain-aware spill rounds - the capacity-bounded assignment pushed towards the objective of Sec. 3.3
 * (the most local pairs for a fixed placement), which the keep/spill of `semmoe_reshuffle` only approximates when
 * capacity binds.  Round 0 is the keep phase of `semmoe_reshuffle`.  In each further round every token still unplaced
 * proposes to its best rank among those with a free slot (equal gains -> home(i) if it is one of them, else the
 * smallest), and a rank accepts its proposers in the order (conf desc, i asc) up to its free slots.  After `rounds`
 * rounds (at most D are needed) the tokens left take the free slots in ascending rank order as in `semmoe_reshuffle`.
 * rounds = 1 gives exactly `semmoe_reshuffle`.  One launch per round plus one.  Same arguments and outputs as
 * `semmoe_reshuffle`; T <= 131072 (SEMMOE_EUNSUPPORTED above), rounds >= 1.
 */
int32_t semmoe_reshuffle_rounds(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                const int32_t* expert_to_rank, int32_t rounds, int32_t* token_rank, int32_t* shf,
                                int32_t* inv_shf, int32_t* rank_count, void* ws, size_t ws_bytes);

/*
 * reshuffle refined to the optimum - `semmoe_reshuffle_rounds`, then moves of already placed tokens until no
 * assignment under the capacity bound has more local pairs: the communication term of the Sec. 3.3 objective for a
 * fixed placement, with `align` of Alg. 3 as the bound.  An assignment is optimal exactly when its residual graph has
 * no closed walk of positive gain; the graph has the D ranks and a node Z for free room as nodes and
 *   a -> b (ranks)  w = max over the tokens i on a of g[i,b] - g[i,a];   a -> Z  w = 0 while a holds fewer than cap
 *   tokens;   Z -> b  w = 0.
 * One cycle: best_L[u][v] = the best walk of exactly L arcs; the smallest L in 2 .. D+1 with some best_L[u][u] > 0 (a
 * closed walk of least length visits no node twice), u0 = the smallest u with the largest best_L[u][u], walked back
 * through the smallest predecessor that attains the best at every step; m = the least, over the arcs that leave a
 * rank, of the number of tokens that attain the arc (free slots for an arc into Z); on every arc between ranks the m
 * tokens of smallest index that attain it move.  Stops when no such walk is left or after `max_cycles` cycles.
 * One workgroup holds all tokens in registers, so T <= 32768, D <= 16, k <= 15 (SEMMOE_EUNSUPPORTED beyond); five
 * launches on top of the starting assignment's.  rounds >= 1, max_cycles >= 0 (0: the starting assignment).
 * dev in / out as `semmoe_reshuffle` (the output arrays also serve as scratch while the call runs); dev out:
 * info[2] i32 = cycles applied, 1 if no walk of positive gain is left (the assignment is optimal) else 0.
 */
int32_t semmoe_reshuffle_refine(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                const int32_t* expert_to_rank, int32_t rounds, int32_t max_cycles, int32_t* token_rank,
                                int32_t* shf, int32_t* inv_shf, int32_t* rank_count, int32_t* info, void* ws,
                                size_t ws_bytes);

/*
 * reshuffle from the schedule table - Alg. 3 `rebatch_tokens` as it runs before the gate: the device id of a token is
 * looked up by its key, dev_ids = cond(T_p[B] > A_p[B], T[B], A[B]).  This form has no inter-layer table A: its
 * device is the token's home shard and its confidence A_p the constant thr_q16 (in 1/65536);
 * `semmoe_reshuffle_cond` is the form with both tables.  So
 *   pref(i) = dev[key_i], conf(i) = level[key_i]  if key_i in [0,V), dev[key_i] in [0,D) and conf_q16[key_i] > thr_q16,
 *   pref(i) = home(i),    conf(i) = 0             otherwise;
 * keep, spill and shuffle then exactly as in `semmoe_reshuffle`.  Two launches.
 * dev in : token_key[T], dev[V], conf_q16[V], level[V] i32.  dev out: token_rank[T], shf[T], inv_shf[T], rank_count[D].
 */
int32_t semmoe_reshuffle_lookup(const semmoe_config* cfg, void* stream, const int32_t* token_key, int32_t V,
                                const int32_t* dev, const int32_t* conf_q16, const int32_t* level, int32_t thr_q16,
                                int32_t* token_rank, int32_t* shf, int32_t* inv_shf, int32_t* rank_count, void* ws,
                                size_t ws_bytes);

/*
 * device_sequence - the row index of the inter-layer table of App. B ("modeling inter-layer activation conjugacy":
 * the rows are the sequences of devices selected at the previous l layers).  The device a token selects at a layer is
 * read as the rank holding most of its k experts (equal -> the smallest rank); seq_out[i] = seq_in[i] * D + device(i),
 * or just device(i) when seq_in is NULL, so chaining the call over l layers numbers the D^l rows with the oldest layer
 * most significant.  seq_in[i] < 0 (history unknown) gives -1.  The caller keeps D^l below 2^31.  Pairs whose expert or
 * rank is out of range are not counted.  The table itself is `semmoe_token_expert_hist` keyed by these numbers
 * (V = D^l) and A / A_p are its `semmoe_lookup_tables`.  One launch; cfg->T is ignored.
 * dev in : topk_ids[T_batch,k], expert_to_rank[E], seq_in[T_batch] or NULL.  dev out: seq_out[T_batch] (may alias
 *          seq_in).
 */
int32_t semmoe_device_sequence(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                               const int32_t* expert_to_rank, int32_t T_batch, const int32_t* seq_in, int32_t* seq_out);

/*
 * reshuffle with both schedule tables - Alg. 3 `rebatch_tokens` as printed: dev_ids = cond(T_p[B] > A_p[B], T[B], A[B]).
 * T / T_p / level are indexed by token_key (as in `semmoe_reshuffle_lookup`), A / A_p / level_a by seq_key (the
 * device sequence of `semmoe_device_sequence`).  An entry that does not exist - index outside its table, device outside
 * [0,D), negative confidence - counts as confidence -1: the other table wins, and with neither the token stays home.
 * Per token the entry of the strictly higher confidence is T's, otherwise A's; it is followed when its confidence
 * exceeds thr_q16 (-1: always): pref = its device, conf = its level; else pref = home, conf = 0.  Keep, spill and
 * shuffle then exactly as in `semmoe_reshuffle`.  Two launches.
 * dev in : token_key[T], dev[V], conf_q16[V], level[V], seq_key[T], dev_a[VA], conf_a_q16[VA], level_a[VA] i32.
 * dev out: token_rank[T], shf[T], inv_shf[T], rank_count[D].
 */
int32_t semmoe_reshuffle_cond(const semmoe_config* cfg, void* stream, const int32_t* token_key, int32_t V,
                              const int32_t* dev, const int32_t* conf_q16, const int32_t* level,
                              const int32_t* seq_key, int32_t VA, const int32_t* dev_a, const int32_t* conf_a_q16,
                              const int32_t* level_a, int32_t thr_q16, int32_t* token_rank, int32_t* shf,
                              int32_t* inv_shf, int32_t* rank_count, void* ws, size_t ws_bytes);

/*
 * request_schedule - online request scheduling of the Attention-DP scenario: Alg. 2 `get_dp_rank` and `schedule`,
 * with the request-to-cluster rule S_r = argmax_j sum_{i in r} R_ij of Sec. 3.3.  Request q owns the tokens
 * [req_offsets[q], req_offsets[q+1]); the schedule table holds one device per token key (`dev` of
 * `semmoe_lookup_tables`), so a request's score is a count: dev_score[r] = #{i in q: dev[token_key[i]] = r}; keys
 * outside [0,V) or with dev outside [0,D) count nowhere.  Requests are taken in order: a request goes to the unmasked
 * device of the highest score (equal -> the smallest id), that device is masked, and after D allocations the mask is
 * cleared, so D consecutive requests of a round reach D different ranks.  Every token inherits the rank of its request;
 * shf = tokens stably sorted by rank (no capacity bound: a rank holds whole requests), inv_shf[shf[p]] = p.
 * cfg->T = total tokens = req_offsets[n_req]; req_offsets[0] = 0, ascending (offsets are clamped into [0,T] when read;
 * the result is defined only for ascending ones).  0 <= n_req <= max(T,1); D <= 64 and T < 2^25, else
 * SEMMOE_EUNSUPPORTED.  Three launches.
 * dev in : req_offsets[n_req+1], token_key[T], dev[V] i32.
 * dev out: req_rank[n_req], token_rank[T], shf[T], inv_shf[T], rank_count[D].
 */
int32_t semmoe_request_schedule(const semmoe_config* cfg, void* stream, const int32_t* req_offsets, int32_t n_req,
                                const int32_t* token_key, int32_t V, const int32_t* dev, int32_t* req_rank,
                                int32_t* token_rank, int32_t* shf, int32_t* inv_shf, int32_t* rank_count, void* ws,
                                size_t ws_bytes);

/*
 * dispatch - the dispatch all2all of expert parallelism (Sec. 1) as a single-device permutation.
 *   Pairs are ordered by physical expert q = phys_of_expert[ids[i,j]], pairs of one expert by shuffled
 *   pair index p' = inv_shf[i]*k + j (arrival order of a rank-ordered all2all).  slot = that position.
 *   slot_of_pair[i*k+j] = slot; pair_of_slot[slot] = i*k+j; expert_offsets[q] = first slot of q
 *   ([E] = P); rank_offsets[r] = expert_offsets[r*m]; X_perm[slot,:] = X[i,:] (bit copy);
 *   send_matrix[s,r] = #{(i,j): token_rank[i]=s, rank of ids[i,j] = r};
 *   remote_pairs = sum_{s != r} send_matrix[s,r]  (alpha of the volume model alpha*k*B*S/G, Sec. 3.1, is
 *   remote_pairs / P).
 * dev in : X[T,d] act or NULL (then no rows are moved and X_perm may be NULL); topk_ids[T,k];
 *          token_rank[T]; shf[T] (a permutation; inv_shf is its inverse, not needed here);
 *          phys_of_expert[E].
 * dev out: X_perm[P,d] act; slot_of_pair[P]; pair_of_slot[P]; expert_offsets[E+1]; rank_offsets[D+1];
 *          send_matrix[D,D] u32; remote_pairs[1] u64.
 */
int32_t semmoe_dispatch(const semmoe_config* cfg, void* stream, const void* X, const int32_t* topk_ids,
                        const int32_t* token_rank, const int32_t* shf, const int32_t* phys_of_expert,
                        void* X_perm, int32_t* slot_of_pair, int32_t* pair_of_slot, int32_t* expert_offsets,
                        int32_t* rank_offsets, uint32_t* send_matrix, uint64_t* remote_pairs, void* ws,
                        size_t ws_bytes);

/*
 * dispatch_index / dispatch_rows - the two halves of semmoe_dispatch as separate calls (same passages:
 * Sec. 1 dispatch all2all, Sec. 3.1 volume model): the index half computes every output of semmoe_dispatch
 * except X_perm; the row half moves rows, X_perm[slot_of_pair[i*k+j],:] = X[i,:].  One index pass can serve
 * several row tensors, and the halves can be timed apart.  Arguments as in semmoe_dispatch.
 */
int32_t semmoe_dispatch_index(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                              const int32_t* token_rank, const int32_t* shf, const int32_t* phys_of_expert,
                              int32_t* slot_of_pair, int32_t* pair_of_slot, int32_t* expert_offsets,
                              int32_t* rank_offsets, uint32_t* send_matrix, uint64_t* remote_pairs, void* ws,
                              size_t ws_bytes);
int32_t semmoe_dispatch_rows(const semmoe_config* cfg, void* stream, const void* X, const int32_t* slot_of_pair,
                             void* X_perm);

/*
 * expert_ffn - the expert FFN (Sec. 2) in SwiGLU form, grouped over one rank's experts:
 *   for every physical expert q of `rank` (rank = -1: all), for slots s in [expert_offsets[q],
 *   expert_offsets[q+1]):  Y[s] = W_down[e] ( silu(W_gate[e] x_s) * (W_up[e] x_s) ),  e = expert_of_phys[q],
 *   W_gate[e] = W_gu[e, 0:F, :], W_up[e] = W_gu[e, F:2F, :].  fp32 accumulate; the hidden activation is
 *   rounded to the act type once.  Rows of other ranks in Y are not written.
 * dev in : X_perm[P,d] act; expert_offsets[E+1]; expert_of_phys[E]; W_gu[E,2F,d] act; W_down[E,d,F] act
 *          (both indexed by ORIGINAL expert id).   dev out: Y[P,d] act.
 */
int32_t semmoe_expert_ffn(const semmoe_config* cfg, void* stream, int32_t rank, const void* X_perm,
                          const int32_t* expert_offsets, const int32_t* expert_of_phys, const void* W_gu,
                          const void* W_down, void* Y, void* ws, size_t ws_bytes);

/*
 * shared_ffn - the same FFN with one set of weights applied to n_tokens rows (the always-active shared
 * expert of DeepSeek-style layers).  dev in: X[n_tokens,d]; W_gu_sh[2F,d]; W_down_sh[d,F].  dev out:
 * Y_shared[n_tokens,d].  n_tokens <= T*k.  ws: n_tokens*F activations + 512 bytes are enough.
 */
int32_t semmoe_shared_ffn(const semmoe_config* cfg, void* stream, const void* X, int32_t n_tokens,
                          const void* W_gu_sh, const void* W_down_sh, void* Y_shared, void* ws,
                          size_t ws_bytes);

/*
 * combine - the combine all2all (Sec. 1) plus `resume_tokens` (Alg. 3):
 *   Out[i] = sum_{j<k} topk_w[i,j] * Y[slot_of_pair[i*k+j]] (+ Y_shared[i]), accumulated in fp32 in
 *   ascending j, rounded once to the act type.
 * dev in : Y[P,d] act; slot_of_pair[P]; topk_w[T,k] f32; Y_shared[T,d] act or NULL.  dev out: Out[T,d] act.
 */
int32_t semmoe_combine(const semmoe_config* cfg, void* stream, const void* Y, const int32_t* slot_of_pair,
                       const float* topk_w, const void* Y_shared, void* Out);

/*
 * Probes of what the chip sustains, for reading roofline fractions against (not part of the layer; no passage of
 * the paper).  Each enqueues one kernel on `stream`; the caller times it.
 *   semmoe_probe_copy: dst[0..bytes) = src[0..bytes), device pointers, 16-byte aligned, bytes % 16 == 0; moves
 *     2*bytes through HBM.
 *   semmoe_probe_stream: the same walk over buf[0..bytes) (device, 16-byte aligned, bytes a multiple of 16384)
 *     reading only (write = 0; per-thread sums go to `sink`, device, 2048*256 words) or writing only (write != 0;
 *     buf is overwritten): the rates of an all-read and an all-write stream.
 *   semmoe_probe_mfma: 256 workgroups of 4 waves, each wave 16 independent 32x32x16 bf16 MFMAs per iteration on operand
 *     fragments read once from `operands` (device, 64 sets x 8 fragments x 64 lanes x 16 bytes = 512 KiB, any finite
 *     bf16 values: the data decide the power drawn and so the clock); `sink` (device, 256*256 floats) receives
 *     checksums; *flops_out (host, may be NULL) = flops of the launch.
 *   semmoe_probe_tile_loop: the steady-state K loop of the grouped GEMM's 256 x 256 tile and nothing else (no tile
 *     list, no epilogue, no ragged edge): 256 workgroups, each `n_slices` (>= 2) K slices of 64 through two LDS stages
 *     filled by direct global->LDS loads, on operand panels that neighbouring workgroups share, so the loads hit
 *     in L2.  `panels` (device, 16-byte aligned): n_panels (>= 96) panels of 256 rows of row_bytes bytes
 *     (row_bytes % 128 == 0) of finite bf16 values; the walk over K wraps around inside a row.  variant 0: the loop
 *     as the GEMM runs it, four waves of 128 x 128; 1: without the loads inside the loop; 2: without the fragment
 *     reads; 3: MFMAs and barriers only; 4 - 7: the same four with eight waves of 128 x 64 (two per SIMD).  The
 *     differences say what the loads and the LDS reads cost the MFMA stream: the ceiling of this tile design.
 *     `sink` (device, 256*512 floats) receives checksums; *flops_out (host, may be NULL) = flops of the launch.
 */
int32_t semmoe_probe_copy(void* stream, void* dst, const void* src, size_t bytes);
int32_t semmoe_probe_stream(void* stream, void* buf, size_t bytes, int32_t write, uint32_t* sink);
int32_t semmoe_probe_mfma(void* stream, const void* operands, int32_t iters, float* sink, double* flops_out);
int32_t semmoe_probe_tile_loop(void* stream, const void* panels, int32_t n_panels, int32_t row_bytes, int32_t variant,
                               int32_t n_slices, float* sink, double* flops_out);

#ifdef __cplusplus
}
#endif
#endif /* SEMMOE_H */
