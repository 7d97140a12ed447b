/*
 * hmy.h -- C ABI of the swap-aware training iteration for one MI355X (gfx950).
 *
 * The library runs ONE training iteration of a transformer stack whose model
 * state exceeds an imposed HBM budget, in the layer-pack-major order of the
 * Harmony paper (arxiv 2202.01306): weights, optimizer state, gradients and
 * checkpoints live in caller-owned pinned host memory; each layer pack is
 * swapped in once and run over all microbatches ("input-batch grouping",
 * Section 3, optimisation 1), backward packs run in reverse with recompute from
 * the stashed pack input (Section 4.3.1), the last pack runs forward+backward
 * per microbatch ("jit-compute") and every pack is updated right after its
 * backward ("jit-update", Section 3, optimisation 2).
 *
 * Conventions
 *   - every struct is plain data with fixed-width integers; no C++ types;
 *   - every function returns HMY_OK (0) or a negative hmy_error; nothing
 *     aborts or throws; hmy_last_error() gives a thread-local detail string;
 *   - "host" pointers are CPU addresses, "device" pointers are HBM addresses
 *     on the handle's GPU; "pinned" host memory was allocated page-locked
 *     (hmy_host_alloc or any hipHostMalloc-backed allocator);
 *   - a handle is used by one thread at a time;
 *   - layers: 0 = embedding, 1..n_blocks = transformer blocks,
 *     n_blocks+1 = final LayerNorm + LM head + loss; R = n_blocks + 2;
 *   - linear maps store W as [out, in] row-major, y = x W^T + bias;
 *   - GB means 1e9 bytes wherever a budget is quoted.
 */
#ifndef HMY_H
#define HMY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HMY_MAX_LAYERS 512
#define HMY_NAME_LEN 32

typedef enum hmy_error {
  HMY_OK = 0,
  HMY_E_INVALID = -1,          /* null pointer, bad shape, unsupported size          */
  HMY_E_BUDGET_TOO_SMALL = -2, /* no packing fits: even one layer per pack overflows */
  HMY_E_BAD_SCHEDULE = -3,     /* packs not contiguous / not covering / over budget  */
  HMY_E_HIP = -4,              /* a HIP runtime call failed (detail in last_error)   */
  HMY_E_NOT_BOUND = -5,        /* hmy_iteration before hmy_bind_state                */
  HMY_E_NO_DEVICE = -6         /* the call needs a GPU and none is usable            */
} hmy_error;

/* Tensor kinds of the paper's swap analysis (Figure "Tensors that need to be
 * swapped", appendix "Additional Swap Analysis") + the token ids/targets. */
typedef enum hmy_kind {
  HMY_KIND_W = 0,   /* weights in compute precision              */
  HMY_KIND_DW = 1,  /* weight gradients (exported once, fp32)    */
  HMY_KIND_K = 2,   /* optimizer state: (master,) m, v           */
  HMY_KIND_SX = 3,  /* stashed input of a backward pack          */
  HMY_KIND_XY = 4,  /* activations between packs (stay in HBM)   */
  HMY_KIND_DXDY = 5,/* their gradients (stay in HBM)             */
  HMY_KIND_IDS = 6, /* token ids and targets                     */
  HMY_NKINDS = 7
} hmy_kind;

#define HMY_PREC_FP32 0 /* fp32 weights, activations, math; K = (m, v)                  */
#define HMY_PREC_BF16 1 /* bf16 weights/activations, fp32 accumulate; K = (master, m, v) */

/* The model: what the paper's Decomposer would hand over as R sequential layers. */
typedef struct hmy_model_spec {
  int32_t n_blocks, d_model, n_heads, d_ffn, seq_len, vocab;
  int32_t causal;    /* 1 decoder (keys j<=i), 0 bidirectional encoder */
  int32_t precision; /* HMY_PREC_* */
  float ln_eps;
} hmy_model_spec;

/* Per-layer times measured on the device for one microbatch size (Section 4.2, Profiler:
 * "runs each layer individually and records ... compute time"), as hmy_measure_profile
 * returns them.  Times are nanoseconds for ONE microbatch of micro_batch sequences.  Every
 * time comes twice: with the device to itself, and (`_beside`) while host-link traffic runs
 * on other streams as it does beside the compute stream in an iteration (copies arriving
 * from pinned host memory; for the backward figures also a throttled kernel writing to it):
 * kernels run some 10-30 % slower then.  A `_beside` field of 0 means "as alone". */
typedef struct hmy_measured_profile {
  int32_t micro_batch;
  int32_t reserved_;
  uint64_t embed_fwd_ns, embed_bwd_ns;
  uint64_t block_fwd_ns;  /* forward of one block in a forward task (nothing kept)          */
  uint64_t block_bwd_ns;  /* one block in a backward task: forward keeping what backward
                             needs (the recompute), then backward                          */
  uint64_t head_ns;       /* final LayerNorm + vocabulary projection + loss, forward and
                             backward (the head only ever runs in the last pack)           */
  uint64_t embed_fwd_beside_ns, embed_bwd_beside_ns, block_fwd_beside_ns, block_bwd_beside_ns, head_beside_ns;
} hmy_measured_profile;

/* The machine model of Algorithm 1: memory capacity alpha, host-link bandwidth beta,
 * plus what the runtime estimate needs to turn the analytic profile into times, and
 * the ranges its configuration search may sweep.  A zero-filled struct but for
 * hbm_budget_bytes plans Algorithm 2 alone with three weight slots, prefetch distance 1
 * and the caller's microbatch size in both passes. */
typedef struct hmy_budget {
  uint64_t hbm_budget_bytes; /* everything the library keeps in HBM must fit                   */
  uint32_t host_link_MBps;   /* per direction, for the runtime estimate; 0 = 40000             */
  uint32_t compute_GFLOPs;   /* sustained model flops/s for layers without a measured time;
                                0 = 420000                                                     */
  uint32_t max_extra_packs;  /* 0: first feasible pack count (Algorithm 2 alone); n: also try the
                                next n feasible pack counts and keep the smallest estimated
                                iteration time (the search of Algorithm 1)                      */
  uint32_t update_site;      /* HMY_UPDATE_*: where the planned iteration will run its Weight Update
                                tasks; the estimate moves only the gradient over the link for
                                ON_HOST, and hmy_plan returns a schedule with this update site   */
  uint32_t min_weight_slots; /* hmy_plan tries every slot count in [min, max] (Section 4.4:       */
  uint32_t max_weight_slots; /* prefetch and double buffering); 0 = 3; range 2..HMY_MAX_WEIGHT_SLOTS */
  uint32_t max_fwd_micro_batch; /* U_FMAX and U_BMAX of Algorithm 1: hmy_plan sweeps the divisors  */
  uint32_t max_bwd_micro_batch; /* of the minibatch up to these; 0 = only the caller's micro_batch */
  uint32_t n_measured;       /* entries of `measured`                                          */
  const hmy_measured_profile *measured; /* host; a layer's time at a microbatch size comes from
                                the entry with that micro_batch if there is one, else from
                                flops / compute_GFLOPs; may be NULL                            */
} hmy_budget;

/* Order in which the tasks of one iteration run over the packs.
 * LAYER_PACK_MAJOR is the method (Section 3, "Key Optimizations": input-batch
 * grouping, jit-compute, jit-update): every pack is visited once per pass and run
 * over all microbatches.  MICROBATCH_MAJOR is the order the paper compares against
 * (Section 3, "Intuitive Example": per-GPU memory virtualisation): every microbatch
 * runs through all packs on its own, so weights cross the link once per pass AND
 * microbatch, and a pack's gradient sums go to the host array after each backward
 * task and come back before the next microbatch's (appendix "Additional Swap
 * Analysis"); the update of a pack follows its last microbatch's backward task.
 * Same packs, same arena, same kernels, same results up to summation order. */
#define HMY_ORDER_LAYER_PACK_MAJOR 0
#define HMY_ORDER_MICROBATCH_MAJOR 1

/* Where the Weight Update task of a pack runs (Section 4.4, first paragraph: the Runtime
 * can place that one task on the CPU instead of the GPU).  ON_DEVICE: optimizer state
 * comes in, the fused Adam kernel runs on the GPU, state, weights and gradient go out.
 * ON_HOST: only the pack's gradient goes out; a pool of CPU threads inside the library
 * applies the same Adam arithmetic to the caller's pinned arrays in place while the
 * GPU goes on with the next pack, so optimizer state and updated weights never cross
 * the link.  hmy_iteration returns once those threads are done too. */
#define HMY_UPDATE_ON_DEVICE 0
#define HMY_UPDATE_ON_HOST 1

/* What happens to a pack's fp32 gradient once its update has consumed it on the device
 * (Section 3, second optimisation: the update runs while W and dW are still resident, so
 * the method itself never moves dW).  EXPORTED: the update also writes it to
 * hmy_state.grads, for callers that want to look at gradients (4 bytes per parameter
 * more on the device->host link, counted under HMY_KIND_DW).  ON_DEVICE: it is dropped;
 * hmy_state.grads is not written by a layer-pack-major iteration and may be NULL there.
 * No effect with HMY_UPDATE_ON_HOST, where the exported gradient is the update's input,
 * and none on the gradient sums that HMY_ORDER_MICROBATCH_MAJOR parks in hmy_state.grads
 * between microbatches (only the final sums stay behind). */
#define HMY_GRADIENTS_EXPORTED 0
#define HMY_GRADIENTS_ON_DEVICE 1

/* Optimizer state kept on the device (Algorithm 3 lists, beside the CPU-GPU swap, a
 * channel that pins a tensor on the GPU).  SWAPPED: all of it lives in the caller's host
 * arrays and crosses the link in and out at every update.  RESIDENT_IN_SPARE_BUDGET: what
 * the HBM budget leaves unused after the arena (hmy_arena) holds optimizer state in whole
 * chunks of k_chunk_params parameters, starting with the chunk that is updated LAST in the
 * iteration (the first layers: their update has no compute left to hide behind) and going
 * backwards through the update order.  A resident chunk is read from the host arrays at
 * its first update after hmy_bind_state and from then on updated in place on the device:
 * its (master,) m and v cross the link neither way, only its weights and gradient go out.
 * The host arrays do not follow: hmy_sync_state writes the resident state back to them.
 * Only with HMY_UPDATE_ON_DEVICE; ignored with ON_HOST, where the state never moves. */
#define HMY_STATE_SWAPPED 0
#define HMY_STATE_RESIDENT_IN_SPARE_BUDGET 1

/* How device->host traffic leaves (Section 4.4: the swap-out stream).  KERNEL: through the
 * library's own throttled kernels that store to the pinned host arrays (the update kernel
 * writes its results there itself).  MEMCPY: hipMemcpyAsync on the swap-out stream, after an
 * update kernel that leaves its results in HBM.  Same bytes, same counters, same results. */
#define HMY_SWAP_OUT_KERNEL 0
#define HMY_SWAP_OUT_MEMCPY 1

#define HMY_MAX_WEIGHT_SLOTS 4

/* Configuration (Section 4.3.1: the 4-tuple U_F, P_F, U_B, P_B): forward and backward layer
 * packs as exclusive end indices over the R layers.  Backward packs cover 0..R; forward packs
 * cover exactly the layers before the last backward pack (the opening steps of Algorithm 2).
 * fwd_micro_batch, bwd_micro_batch: U_F and U_B in sequences; 0 = the caller's micro_batch.
 * Each must divide the minibatch (n_micro * micro_batch sequences): the forward tasks run it
 * as microbatches of U_F, the backward tasks (and the last pack, which runs forward and
 * backward together) as microbatches of U_B, gradients summed in ascending order of those.
 * HMY_ORDER_MICROBATCH_MAJOR needs U_F = U_B.
 * weight_slots (Section 4.4, double buffering): HBM slots that hold a pack's weights and,
 * in a backward task, its gradient; task v uses slot v mod weight_slots; 0 = 3.
 * prefetch_distance: the weights of task v + distance travel while task v computes;
 * 0 = 1; must be below weight_slots.  With distance + 1 slots the load of a task waits for
 * the write-back of the task that held its slot; one more slot lets it go ahead.
 * order: HMY_ORDER_*, update_site: HMY_UPDATE_*, gradients: HMY_GRADIENTS_*,
 * resident_state: HMY_STATE_*, swap_out: HMY_SWAP_OUT_*; hmy_plan returns LAYER_PACK_MAJOR,
 * EXPORTED, SWAPPED, KERNEL (all 0) and the update site of its budget argument; any value
 * other than those defined above is HMY_E_BAD_SCHEDULE. */
typedef struct hmy_schedule {
  int32_t n_fwd_packs, n_bwd_packs;
  int32_t fwd_pack_end[HMY_MAX_LAYERS];
  int32_t bwd_pack_end[HMY_MAX_LAYERS];
  int32_t order;
  int32_t update_site;
  int32_t gradients;
  int32_t resident_state;
  int32_t swap_out;
  int32_t weight_slots;
  int32_t prefetch_distance;
  int32_t fwd_micro_batch, bwd_micro_batch;
} hmy_schedule;

/* One minibatch as a list of n_micro microbatches of micro_batch sequences. */
typedef struct hmy_minibatch {
  int32_t n_micro, micro_batch;
  const int32_t *token_ids; /* host, pinned or pageable; [n_micro*micro_batch*seq_len] */
  const int32_t *targets;   /* host, same shape; -1 = position is not a target       */
} hmy_minibatch;

typedef struct hmy_adam {
  float lr, beta1, beta2, eps;
  int64_t step; /* 1-based */
} hmy_adam;

/* Caller-owned PINNED host arrays of n_params elements each, tensors in layout
 * order (hmy_layout), no padding.  weights: bf16 (HMY_PREC_BF16) or fp32.
 * master: fp32, only for HMY_PREC_BF16 (NULL otherwise: the fp32 weights are the
 * master).  adam_m, adam_v, grads: fp32.  After hmy_iteration they hold the
 * updated weights/state and this iteration's accumulated gradients (state that the
 * schedule keeps resident on the device: after hmy_sync_state).  Binding again makes
 * the engine read resident state afresh from the arrays.
 * With HMY_UPDATE_ON_HOST master, adam_m and adam_v may be ordinary (pageable) memory:
 * only the library's CPU threads touch them; weights and grads, which cross the
 * link, must be page-locked in every case. */
typedef struct hmy_host_state {
  void *weights;
  float *master;
  float *adam_m, *adam_v;
  float *grads;
  uint64_t n_params;
} hmy_host_state;

typedef struct hmy_stats {
  uint64_t h2d[HMY_NKINDS]; /* bytes enqueued host->device, per kind */
  uint64_t d2h[HMY_NKINDS]; /* bytes enqueued device->host, per kind */
  double loss;              /* sum over target positions / number of targets */
  double t_iter_s;          /* wall time of the iteration (host clock)      */
  /* the next four only at profiling level >= 1 (hmy_set_profiling), else 0: */
  double t_compute_s;       /* compute stream: first kernel to last (events) */
  double t_h2d_busy_s;      /* sum of H2D copy durations (events)           */
  double t_d2h_busy_s;      /* sum of D2H copy durations (events)           */
  double t_stall_s;         /* time the compute stream spent waiting on swaps */
  uint64_t n_targets;
  /* per GEMM kernel variant (index = 2*ta + tb): launches, algorithmic flops
   * (2*M*N*K each) and, only at profiling level 2, summed durations */
  uint64_t gemm_calls[4];
  double gemm_flops[4];
  double gemm_s[4];
  /* level 2: what two event records cost with nothing between them (smallest of a few
   * such pairs at the start of the iteration); already subtracted once per launch
   * from gemm_s, so that gemm_s is kernel time as a kernel trace reports it */
  double t_event_pair_s;
} hmy_stats;

typedef struct hmy_tensor_desc {
  char name[HMY_NAME_LEN]; /* "wte", "h3.wqkv", "lnf_g", ... */
  int32_t layer;
  int32_t rows, cols;      /* cols = 1 for vectors */
  uint64_t offset;         /* element offset inside every host array */
  uint64_t count;          /* rows*cols */
} hmy_tensor_desc;

/* Per-layer profile phi(type, U, layer) (Section 4.2) for one forward microbatch of U_F and
 * one backward microbatch of U_B sequences: times in nanoseconds (measured where the budget
 * brings a measurement for that microbatch size, else flops / compute rate, rounded up),
 * flop counts, and the byte footprints Algorithm 2 packs by. */
typedef struct hmy_layer_profile {
  int64_t ns_fwd;         /* the layer in a forward task                                   */
  int64_t ns_bwd;         /* the layer in a backward task: recompute + backward            */
  int64_t ns_fwd_beside;  /* the same two beside host-link traffic (= the figures above     */
  int64_t ns_bwd_beside;  /* unless the budget brings measurements of both)                */
  int64_t flops_fwd;      /* per forward microbatch; a backward task costs three times the
                             forward flops of its own microbatch size                      */
  uint64_t params;
  uint64_t mem_fwd;       /* weight_slots * weight bytes                                   */
  uint64_t mem_bwd;       /* weight_slots * (weight + fp32 gradient) bytes + activations   */
  uint64_t act_bwd;       /* activations one backward microbatch keeps                     */
} hmy_layer_profile;

typedef struct hmy_arena_plan {
  uint64_t total;         /* bytes of HBM the iteration needs (<= budget)          */
  uint64_t reserved;      /* everything that does not depend on the packs          */
  uint64_t slot_bytes;    /* one weight slot                                       */
  uint64_t act_bytes;     /* activation workspace of the largest backward pack     */
  uint64_t k_chunk_params;/* optimizer state streams through a ring of such chunks */
  int32_t weight_slots;   /* as resolved from the schedule                         */
  int32_t prefetch_distance;
  int32_t fwd_micro_batch, bwd_micro_batch;
} hmy_arena_plan;

/* One buffer of the HBM arena (hmy_arena_regions): byte range [offset, offset + bytes)
 * from the arena's base. */
typedef struct hmy_region {
  char name[HMY_NAME_LEN];
  uint64_t offset, bytes;
} hmy_region;

typedef struct hmy_handle hmy_handle;

/* ---- host-only calls (no GPU needed) ----------------------------------- */

const char *hmy_strerror(int err);
const char *hmy_last_error(void);

/* Number of layers R and of parameters; fails on shapes the kernels do not
 * support (d_model % n_heads, d_model % 8, d_ffn % 8, d_head not in {32,64,128}
 * ...). */
int hmy_model_size(const hmy_model_spec *spec, int32_t *n_layers, uint64_t *n_params);

/* Tensor table in storage order.  out may be NULL to query *n only; cap is the
 * capacity of out in entries. */
int hmy_layout(const hmy_model_spec *spec, hmy_tensor_desc *out, int32_t cap, int32_t *n);

/* Per-layer profile (out has R entries) and the pack-independent reserve, for the
 * microbatch sizes and slot count of *sched (NULL: the caller's micro_batch in both passes,
 * three slots; only those fields of it are read) and the rates / measurements of *budget
 * (NULL: the default rates). */
int hmy_profile(const hmy_model_spec *spec, const hmy_budget *budget, const hmy_schedule *sched,
                int32_t n_micro, int32_t micro_batch, hmy_layer_profile *out, uint64_t *reserved_bytes);

/* The configuration search of Algorithm 1 (Section 4.3.1) over what *budget lets it sweep:
 * backward microbatch size, weight slots, backward packs by balanced-time packing
 * (Algorithm 2) under the budget -- backward packs first, forward packs over the layers
 * before the last backward pack --, forward microbatch size; the configuration with the
 * smallest estimated iteration time (hmy_estimate) is returned. */
int hmy_plan(const hmy_model_spec *spec, const hmy_budget *budget, int32_t n_micro,
             int32_t micro_batch, hmy_schedule *out);

/* Runtime estimate (integer nanoseconds) of one iteration for a schedule: an
 * event-driven walk of the task list over the compute stream, the two directions of
 * the host link and, for HMY_UPDATE_ON_HOST, the CPU (Section 4.3.1, "Runtime
 * Estimator"), from the per-layer profile (hmy_profile) and the link rate of *budget.
 * A task's compute time lies between its layers' times alone and beside link traffic, in
 * proportion to the share of it for which the outgoing link has work queued at its start.
 * This is what hmy_plan minimises.  It models the layer-pack-major order with swapped
 * optimizer state only (sched->order and ->resident_state are not looked at). */
int hmy_estimate(const hmy_model_spec *spec, const hmy_schedule *sched, const hmy_budget *budget,
                 int32_t n_micro, int32_t micro_batch, uint64_t *iteration_ns);

/* Validate a schedule and size the HBM arena it needs. */
int hmy_arena(const hmy_model_spec *spec, const hmy_schedule *sched, int32_t n_micro,
              int32_t micro_batch, hmy_arena_plan *out);

/* Every buffer the engine addresses inside that arena, in address order: the
 * pack-independent buffers by name, "slot0".."slotN", and "acts".  out may be NULL to
 * query *n only; cap is the capacity of out in entries. */
int hmy_arena_regions(const hmy_model_spec *spec, const hmy_schedule *sched, int32_t n_micro,
                      int32_t micro_batch, hmy_region *out, int32_t cap, int32_t *n);

/* Walk the iteration's task list (in sched->order) exactly as hmy_iteration does,
 * touching no device: fills only the byte counters of *out. */
int hmy_count_swaps(const hmy_model_spec *spec, const hmy_schedule *sched, int32_t n_micro,
                    int32_t micro_batch, hmy_stats *out);

/* ---- device calls ------------------------------------------------------- */

/* Page-locked host memory for hmy_host_state (hipHostMalloc / hipHostFree). */
int hmy_host_alloc(uint64_t bytes, void **out);
int hmy_host_free(void *p);

/* Create the Runtime for one configuration (Section 4.4: "executes the task graph ...
 * with swap-in / compute / swap-out streams"; Section 4.3.2: one task per layer pack and
 * pass) on `hip_device`.  sched == NULL plans with hmy_plan; n_micro x micro_batch is the
 * minibatch as hmy_iteration will receive it.
 * arena: device pointer to at least hmy_arena().total bytes, 256-byte aligned,
 * owned by the caller for the handle's lifetime; NULL lets the library
 * allocate it.  Fails with HMY_E_BUDGET_TOO_SMALL if the arena exceeds the
 * budget. */
int hmy_create(const hmy_model_spec *spec, const hmy_budget *budget, int32_t n_micro,
               int32_t micro_batch, const hmy_schedule *sched, int32_t hip_device,
               void *arena, uint64_t arena_bytes, hmy_handle **out);
int hmy_get_schedule(const hmy_handle *h, hmy_schedule *out);
/* Hand over the model state that lives in host memory (Section 3: weights, gradients and
 * optimizer state stay in pinned CPU memory and are swapped per layer pack; Figure
 * "Tensors that need to be swapped").  The arrays stay the caller's; the library reads
 * and writes them during hmy_iteration only. */
int hmy_bind_state(hmy_handle *h, const hmy_host_state *state);

/* One iteration (Section 3, "Key Optimizations"; task order of Algorithm 3 at N = 1):
 * forward tasks over the forward packs, each over all microbatches (input-batch grouping);
 * the last pack forward + backward per microbatch (jit-compute); backward tasks in reverse
 * with recompute from the stashed pack input (Section 4.3.1), each followed by its Weight
 * Update (jit-update); swap-byte counters per tensor kind (appendix "Additional Swap
 * Analysis").  Produces the minibatch's gradients, Adam on every tensor, the loss and the
 * counters.  Returns with all streams idle. */
int hmy_iteration(hmy_handle *h, const hmy_minibatch *mb, const hmy_adam *adam, hmy_stats *out);

/* The Profiler of Section 4.2 for this library's kernels: runs the embedding, a pack of up
 * to three blocks and the head on `hip_device`, forward and backward as the tasks would run
 * them, for one microbatch of micro_batch sequences (pseudo-random inputs: the kernels'
 * time does not depend on the values, but all-zero operands draw less power and clock
 * higher), `reps` times each after a warm-up, once with the device to itself and once
 * beside host-link traffic on two more streams (see hmy_measured_profile), and reports
 * the average times, the blocks' divided by their number (several blocks, because one
 * block run over and over finds its weights and activations in the memory-side cache,
 * which the blocks of a pack in an iteration do not).  Allocates its own device memory (an
 * arena for those three packs, two 128 MiB staging buffers) and frees it; needs no host
 * state. */
int hmy_measure_profile(const hmy_model_spec *spec, int32_t micro_batch, int32_t hip_device,
                        int32_t reps, hmy_measured_profile *out);
/* Parameters whose optimizer state is resident on the device (0 unless the schedule says
 * HMY_STATE_RESIDENT_IN_SPARE_BUDGET and the budget leaves room for at least one chunk). */
int hmy_resident_params(const hmy_handle *h, uint64_t *n_params);
/* Write the resident optimizer state back to the bound host arrays (synchronous; not part
 * of any iteration's counters).  A no-op without resident state.  hmy_destroy does not
 * call it: the arrays may be gone by then. */
int hmy_sync_state(hmy_handle *h);
int hmy_destroy(hmy_handle *h);
/* What the next iterations time with HIP events, beyond the byte counters, the loss and
 * t_iter_s, which are always filled: level 0 (default) nothing -- timing events between
 * the copies and around the compute stream's waits cost a few percent of the iteration;
 * 1: every copy, every wait of the compute stream on a swap, and the compute span
 * (t_compute_s, t_h2d_busy_s, t_d2h_busy_s, t_stall_s); 2: also every GEMM launch
 * (gemm_s; two more event records per launch). */
int hmy_set_profiling(hmy_handle *h, int32_t level);
/* on != 0: a layer-pack-major iteration waits for the compute stream after every visit and
 * prints one line per visit to stderr.  For runs under a tool that serialises every kernel
 * dispatch (counter collection), where an iteration takes minutes: the lines show that it
 * advances.  Costs the overlap between visits; never use it for timing. */
int hmy_set_progress(hmy_handle *h, int32_t on);

/* 0 = reference kernels (plain tiled loops); 1 = MFMA kernels where they exist
 * (default: the GEMM that streams tiles HBM -> LDS with the load-to-LDS instruction
 * when the shape allows it, else the register-staged one).  2 and 3 are for tests only:
 * they force the register-staged MFMA GEMMs (the 128x128x64 one; the K-tile-32 one for
 * every shape) that the default path uses for ragged or misaligned operands, so that
 * those kernels can be checked on shapes where they would not be chosen.  Attention uses
 * its MFMA kernels for 1..3.  Process-wide. */
int hmy_set_kernel_path(int32_t use_mfma);

/* ---- single kernels (all pointers DEVICE, stream = hipStream_t or NULL) ---
 * prec selects the element type E of activations/weights (HMY_PREC_*).  These
 * are the per-layer operations of one microbatch, T = rows. */

/* The residual stream -- the activations x that run from block to block and, on the way
 * back, their gradients -- is fp32 in every precision: each block adds a small update to a
 * large running sum, and rounding that sum to bf16 after every addition piles the errors of
 * 2 * n_blocks roundings into every gradient.  So the x, res and dx arguments below are
 * float arrays whatever prec is; gamma, beta, y, dy and everything else a block computes
 * have the element type E(prec). */

/* x[T,d] (fp32) = wte[id] + wpe[t % s] */
int hmy_k_embed_fwd(int32_t prec, const int32_t *ids, const void *wte, const void *wpe, float *x,
                    int32_t T, int32_t d, int32_t s, int32_t vocab, void *stream);
/* dwte[id] += dx, dwpe[t % s] += dx  (dx fp32; fp32 accumulators) */
int hmy_k_embed_bwd(int32_t prec, const int32_t *ids, const float *dx, float *dwte, float *dwpe,
                    int32_t T, int32_t d, int32_t s, int32_t vocab, void *stream);
/* y (type E) = gamma * (x-mean)*rstd + beta; x fp32; mean,rstd [T] fp32 saved */
int hmy_k_layernorm_fwd(int32_t prec, const float *x, const void *gamma, const void *beta, void *y,
                        float *mean, float *rstd, int32_t T, int32_t d, float eps, void *stream);
/* dx (fp32) = (res ? res : 0) + LN'(dy); dgamma,dbeta += (fp32).  dy has type E; x, res and
 * dx are fp32; dx may alias res.  dx_e (may be NULL): a copy of dx rounded to type E, which is
 * what the GEMMs that consume this gradient read.
 * dres_sum (may be NULL; needs res): dres_sum[d] += column sums of res.  res is the gradient
 * arriving over the residual connection, which is also the gradient of the output of the linear
 * layer that closes the branch: its column sums are that layer's bias gradient, taken here
 * from the fp32 values while they pass through anyway.
 * workspace (device, may be NULL): with at least 256 * 2 * d floats (256 * 3 * d with
 * dres_sum) the per-workgroup partial sums go there and a second kernel adds them up;
 * without it they are added with atomics (same result up to summation order, slower). */
int hmy_k_layernorm_bwd(int32_t prec, const void *dy, const float *x, const float *mean,
                        const float *rstd, const void *gamma, const float *res, float *dx, void *dx_e,
                        float *dgamma, float *dbeta, float *dres_sum, int32_t T, int32_t d,
                        void *stream, float *workspace, uint64_t workspace_bytes);
/* hmy_k_layernorm_bwd for callers that cannot allocate device memory (code under HIP graph
 * capture, serving loops, harnesses that forbid hipMalloc): same arguments without the
 * workspace, same kernels, same results.  The per-workgroup partial sums go to an 8 MiB array
 * that the library's code object holds on every GPU it is loaded on (its address on the current
 * device is looked up at the first call there); the call allocates and frees nothing.
 * Limit: d <= 4096 (HMY_E_INVALID with a message beyond; the variant with a caller's workspace
 * has no such limit).  The current device must be the stream's.  All calls on one GPU share
 * the array: calls that may overlap there (different streams, different threads) race on it
 * and must be ordered by the caller; calls on one stream are ordered already.  Nothing in
 * the array has to be cleared between calls. */
int hmy_k_layernorm_bwd_static(int32_t prec, const void *dy, const float *x, const float *mean,
                               const float *rstd, const void *gamma, const float *res, float *dx,
                               void *dx_e, float *dgamma, float *dbeta, int32_t T, int32_t d,
                               void *stream);
/* g = gelu_tanh(u); du = dg * gelu'(u) (du may alias dg) */
int hmy_k_gelu_fwd(int32_t prec, const void *u, void *g, uint64_t n, void *stream);
int hmy_k_gelu_bwd(int32_t prec, const void *dg, const void *u, void *du, uint64_t n, void *stream);
/* the same on a [T,N] matrix, with db[N] += column sums of du as stored (the gradient of the
 * bias in front of the activation), so that du is not read again for them */
int hmy_k_gelu_bwd_colsum(int32_t prec, const void *dg, const void *u, void *du, float *db,
                          int32_t T, int32_t N, void *stream);
/* out[N] += column sums of a[T,N]  (fp32 accumulators; bias gradients) */
int hmy_k_colsum(int32_t prec, const void *a, float *out, int32_t T, int32_t N, void *stream);

/* C[M,N] = op(A) op(B) (+bias[N]) (+res[M,N]); optional second output
 * gelu_out = gelu(C).  A is [M,K] (ta=0) or stored [K,M] (ta=1); B is stored
 * [N,K] (tb=0: y = x W^T) or [K,N] (tb=1).  A, B, bias, res, gelu_out have
 * element type E(prec); C has type E, or fp32 if c_fp32.  accumulate: C += (only
 * with c_fp32).  res_fp32: res is an fp32 array (the residual stream; C is then fp32 too:
 * c_fp32 must be set).  Leading dimensions in elements.  gelu_out may be C itself: then C
 * ends up holding gelu of the (rounded) result and nothing else is stored -- what a
 * forward pass wants that keeps no pre-activation for a backward pass. */
typedef struct hmy_gemm_desc {
  int32_t prec, M, N, K;
  int32_t ta, tb, c_fp32, accumulate;
  const void *A; int64_t lda;
  const void *B; int64_t ldb;
  void *C; int64_t ldc;
  const void *bias;
  const void *res; int64_t ldr;
  void *gelu_out;
  int32_t res_fp32;
} hmy_gemm_desc;
int hmy_k_gemm(const hmy_gemm_desc *g, void *stream);

/* qkv[T,3d] (q|k|v thirds, head h = columns h*dh..) -> o[T,d], lse[b,H,s] fp32 */
int hmy_k_attn_fwd(int32_t prec, const void *qkv, void *o, float *lse, int32_t b, int32_t s,
                   int32_t H, int32_t dh, int32_t causal, void *stream);
/* dqkv[T,3d] from do[T,d]; delta[b,H,s] fp32 is scratch.  dbias (may be NULL): dbias[3d] +=
 * column sums of dqkv as stored, the gradient of the bias of the projection that produced qkv. */
int hmy_k_attn_bwd(int32_t prec, const void *qkv, const void *o, const void *d_o, const float *lse,
                   float *delta, void *dqkv, float *dbias, int32_t b, int32_t s, int32_t H,
                   int32_t dh, int32_t causal, void *stream);
/* rows with target>=0: loss_acc[0] += (lse - logit[target]) * inv_ntgt (fp64 atomics); dlogits = (softmax - onehot) * inv_ntgt; other rows: dlogits = 0.
 * logits fp32 [T,V] row stride ldl; dlogits type E, same stride. */
int hmy_k_xent(int32_t prec, const float *logits, const int32_t *targets, double *loss_acc,
               void *dlogits, int32_t T, int32_t V, int64_t ldl, float inv_ntgt, void *stream);
/* Adam with bias correction.  bf16: master/m/v fp32 updated, w_out = RNE bf16(master).
 * fp32: w (fp32, in w_out) is the master; master must be NULL. */
int hmy_k_adam(int32_t prec, const float *grad, float *master, float *m, float *v, void *w_out,
               uint64_t n, const hmy_adam *hp, void *stream);

/* ---- the host-side update on its own (all pointers HOST, no GPU needed) ----
 * What HMY_UPDATE_ON_HOST applies to each chunk of a pack (Section 4.4, update task on
 * the CPU): the arithmetic of hmy_k_adam, in place, over n elements, on `threads` CPU
 * threads (0 = as many as the engine would use).  Argument rules as for hmy_k_adam. */
int hmy_host_adam(int32_t prec, const float *grad, float *master, float *m, float *v, void *weights,
                  uint64_t n, const hmy_adam *hp, int32_t threads);

#ifdef __cplusplus
}
#endif
#endif /* HMY_H */
