// Internal declarations shared by the host logic and the kernel launchers.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "hmy.h"

namespace hmy {

// ---- errors ---------------------------------------------------------------
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// ---- model layout -----------------------------------------------------------
struct Tensor {
  std::string name;
  int layer;
  int rows, cols;
  uint64_t offset;  // element offset in every host array
  uint64_t count;
};

// indices of a block's tensors relative to the block's first tensor
enum BlockTensor { LN1_G, LN1_B, WQKV, BQKV, WO, BO, LN2_G, LN2_B, W1, B1, W2, B2, N_BLOCK_TENSORS };

struct Model {
  hmy_model_spec spec;
  int R;                            // layers
  std::vector<Tensor> tensors;      // storage order
  std::vector<int> first_tensor;    // per layer, index into tensors (size R+1)
  std::vector<uint64_t> layer_off;  // per layer, element offset (size R+1)
  uint64_t n_params;
  int elem_bytes() const { return spec.precision == HMY_PREC_BF16 ? 2 : 4; }
  int k_arrays() const { return spec.precision == HMY_PREC_BF16 ? 3 : 2; }  // K = (master,) m, v
  uint64_t params_in(int a, int e) const { return layer_off[e] - layer_off[a]; }
};

int build_model(const hmy_model_spec *spec, Model *out);

// ---- analytic profile and arena ---------------------------------------------
inline uint64_t a256(uint64_t x) { return (x + 255) & ~uint64_t(255); }

constexpr int kMaxSlots = HMY_MAX_WEIGHT_SLOTS;   // weight slots of a schedule: 2 .. kMaxSlots
constexpr int kDefaultSlots = 3;       // in use, being prefetched, being updated and written back
constexpr int kOutRing = 4;            // staging buffers for checkpoints going out
constexpr int kInRing = 4;             // pack-input buffers (checkpoints coming in, up to three microbatches ahead)
constexpr int kKRing = 3;              // optimizer-state ring slots
constexpr uint64_t kKChunkMax = 4ull << 20;  // parameters per optimizer chunk
constexpr int kLogitRows = 512;        // rows of the vocabulary projection per chunk
constexpr int kLnBlocks = 256;         // workgroups of a LayerNorm backward, each leaving one row of partial sums

struct BlockActs {  // byte offsets of one block's saved activations inside its region
  uint64_t x_in, a, qkv, o, x_mid, h, u, g, ln1_mean, ln1_rstd, ln2_mean, ln2_rstd, lse, size;
};
struct HeadActs {
  uint64_t x_in, z, mean, rstd, logits, dlogits, dz32, size;
  int chunk_rows;
  int64_t ldl;  // row stride of logits / dlogits in elements
};
BlockActs block_acts(const hmy_model_spec &s, int micro_batch);
HeadActs head_acts(const hmy_model_spec &s, int micro_batch);

struct Pack { int a, e; };
// One configuration: the 4-tuple of Section 4.3.1 plus how the runtime executes it.  uF / uB = 0 and
// slots / distance = 0 stand for "the caller's microbatch size" and the defaults until resolve() fills them in.
struct Packs {
  std::vector<Pack> fwd, bwd;
  int order = HMY_ORDER_LAYER_PACK_MAJOR;
  int update_site = HMY_UPDATE_ON_DEVICE;
  int gradients = HMY_GRADIENTS_EXPORTED;
  int resident_state = HMY_STATE_SWAPPED;
  int swap_out = HMY_SWAP_OUT_KERNEL;
  int slots = 0, distance = 0;
  int uF = 0, uB = 0;
};
// The minibatch of D sequences cut into MF forward microbatches of uF and MB backward microbatches of uB.
struct Split {
  int D, uF, uB;
  int MF() const { return D / uF; }
  int MB() const { return D / uB; }
};
// fills in the defaults of p (slots, distance, uF, uB) for a minibatch of n_micro x micro_batch and checks them
int resolve(Packs *p, int n_micro, int micro_batch, Split *out);

struct Reserved {  // pack-independent arena regions, byte offsets from the arena base
  uint64_t X;         // the minibatch's boundary activations (fp32), [D*s, d] contiguous
  uint64_t x_bytes_F, x_bytes_B;   // one forward / backward microbatch of it (unpadded)
  uint64_t ck_bytes_F, ck_bytes_B; // the same microbatch as a checkpoint: rounded to the element type
  uint64_t in_bytes, out_bytes;    // a256 of those: one buffer of the rings
  uint64_t inring;    // kInRing buffers of in_bytes
  uint64_t outring;   // kOutRing buffers of out_bytes
  uint64_t gbig;      // T_B*max(f,3d)*E : dg/du and dqkv
  uint64_t gsmall;    // T_B*d*E : dh, do, da, dz
  uint64_t dlow;      // T_B*d*E : the gradient of the residual stream rounded to the element type, for the GEMMs
  uint64_t delta;     // T_B*H*4
  uint64_t ids, targets;
  uint64_t misc;      // loss accumulators
  uint64_t kring;     // kKRing slots of k_arrays * karr_bytes
  uint64_t karr_bytes;
  uint64_t k_chunk_params;
  uint64_t size;
};
Reserved reserved_layout(const Model &m, const Split &sp);

// rates and measurements the profile turns flop counts into times with (defaults filled in)
struct Rates {
  uint64_t link_MBps = 40000, compute_GFLOPs = 420000;
  const hmy_measured_profile *measured = nullptr;
  uint32_t n_measured = 0;
};
Rates rates_of(const hmy_budget *b);
void layer_profile(const Model &m, const Rates &r, const Split &sp, int slots, std::vector<hmy_layer_profile> *out);

int schedule_to_packs(const Model &m, const hmy_schedule *s, Packs *out);
void packs_to_schedule(const Packs &p, hmy_schedule *out);

struct Arena {
  Reserved res;
  int slots;
  uint64_t slot_bytes;
  uint64_t slot_off[kMaxSlots];
  uint64_t act_off, act_bytes;
  uint64_t total;
};
// p must have been resolved
Arena arena_layout(const Model &m, const Packs &p, const Split &sp);
uint64_t pack_state_bwd(const Model &m, Pack p);   // a256(E*P) + a256(4*P)
uint64_t pack_state_fwd(const Model &m, Pack p);   // a256(E*P)
struct Region { std::string name; uint64_t offset, bytes; };
std::vector<Region> arena_regions(const Model &m, const Arena &a, const Split &sp);

int plan_packs(const Model &m, const hmy_budget &budget, int n_micro, int micro_batch, Packs *out);
uint64_t estimate_iteration_ns(const Model &m, const std::vector<hmy_layer_profile> &prof, const Packs &p,
                               const Split &sp, uint64_t link_MBps);

// ---- kernel launchers (all pointers device; stream is a hipStream_t) ---------
typedef void *stream_t;

// x, dx, res: the fp32 residual stream (whatever prec is); dx_e: optional copy of dx in the element type
int launch_embed_fwd(int prec, const int32_t *ids, const void *wte, const void *wpe, float *x,
                     int T, int d, int s, int vocab, stream_t st);
int launch_embed_bwd(int prec, const int32_t *ids, const float *dx, float *dwte, float *dwpe,
                     int T, int d, int s, int vocab, stream_t st);
int launch_layernorm_fwd(int prec, const float *x, const void *gamma, const void *beta, void *y,
                         float *mean, float *rstd, int T, int d, float eps, stream_t st);
int launch_layernorm_bwd(int prec, const void *dy, const float *x, const float *mean,
                         const float *rstd, const void *gamma, const float *res, float *dx, void *dx_e,
                         float *dgamma, float *dbeta, float *dres_sum, int T, int d, stream_t st,
                         float *workspace = nullptr, uint64_t workspace_bytes = 0);
int launch_layernorm_bwd_static(int prec, const void *dy, const float *x, const float *mean, const float *rstd,
                                const void *gamma, const float *res, float *dx, void *dx_e, float *dgamma, float *dbeta,
                                int T, int d, stream_t st);
int launch_convert_to_f32(int prec, const void *src, float *dst, uint64_t n, stream_t st);
int launch_gelu_fwd(int prec, const void *u, void *g, uint64_t n, stream_t st);
int launch_gelu_bwd(int prec, const void *dg, const void *u, void *du, uint64_t n, stream_t st);
int launch_gelu_bwd_colsum(int prec, const void *dg, const void *u, void *du, float *db, int T, int N, stream_t st);
int launch_colsum(int prec, const void *a, float *out, int T, int N, stream_t st);
int launch_gemm(const hmy_gemm_desc &g, stream_t st);

int launch_gemm_mfma32(const hmy_gemm_desc &g, stream_t st);
bool gemm_dma_eligible(const hmy_gemm_desc &g);
int launch_gemm_dma(const hmy_gemm_desc &g, stream_t st);
int launch_attn_fwd(int prec, const void *qkv, void *o, float *lse, int b, int s, int H, int dh,
                    int causal, stream_t st);
int launch_attn_bwd(int prec, const void *qkv, const void *o, const void *d_o, const float *lse,
                    float *delta, void *dqkv, float *dbias, int b, int s, int H, int dh, int causal,
                    stream_t st);
int launch_attn_fwd_mfma(const void *qkv, void *o, float *lse, int b, int s, int H, int dh, int causal, stream_t st);
int launch_attn_bwd_mfma(const void *qkv, const void *o, const void *d_o, const float *lse, float *delta, void *dqkv,
                         float *dbias, int b, int s, int H, int dh, int causal, stream_t st);
int launch_xent(int prec, const float *logits, const int32_t *targets, double *loss_acc,
                void *dlogits, int T, int V, int64_t ldl, float inv_ntgt, stream_t st);
int launch_adam(int prec, const float *grad, float *master, float *m, float *v, void *w_out,
                uint64_t n, const hmy_adam &hp, stream_t st);
int launch_adam_out(int prec, const float *grad, const float *in_master, const float *in_m, const float *in_v,
                    float *out_master, float *out_m, float *out_v, void *out_w, float *out_g, uint64_t n,
                    const hmy_adam &hp, bool alone, stream_t st);
int launch_fill_zero(void *p, uint64_t bytes, stream_t st);

// ---- Weight Update on the host CPU (host_update.cpp) ----
// One chunk of one pack: all pointers are host addresses of the same n elements.
struct HostAdamJob {
  void *ready;          // handed to the wait hook: the chunk's gradient has arrived in `grad` (NULL: it is there already)
  const float *grad;
  float *master;        // fp32 master (bf16 models) or NULL: then `weights` is the fp32 weight itself
  float *m, *v;
  void *weights;        // bf16 (with master) or fp32
  uint64_t n;
  float lr, b1, b2, eps, inv_bc1, inv_bc2;
};
HostAdamJob make_host_adam_job(void *ready, const float *grad, float *master, float *m, float *v, void *weights,
                               uint64_t n, const hmy_adam &hp);
int default_host_threads();   // min(16, hardware threads), or HMY_HOST_THREADS
// Jobs run in submission order on a dispatcher thread + worker pool; drain() returns once
// every submitted job has been applied (HMY_OK or the first error).
class HostUpdater {
 public:
  // hooks run on the dispatcher thread: thread_init(arg, NULL) once at its start,
  // wait_ready(arg, job.ready) before each job; both return HMY_OK or an error code
  typedef int (*Hook)(void *arg, void *ready);
  HostUpdater(int nthreads, Hook thread_init, Hook wait_ready, void *hook_arg);
  ~HostUpdater();
  HostUpdater(const HostUpdater &) = delete;
  HostUpdater &operator=(const HostUpdater &) = delete;
  void submit(const HostAdamJob &job);
  int drain();
  int threads() const;

 private:
  struct Impl;
  Impl *p;
};
// grid_cap bounds the workgroups: a copy to pinned host memory needs few of them to fill
// the link and must not crowd the compute units
int launch_copy(void *dst, const void *src, uint64_t bytes, stream_t st, int grid_cap = 2048);
int run_measure_profile(const Model &m, int micro_batch, int hip_device, int reps, hmy_measured_profile *out);
int launch_copy_out(void *dst_host, const void *src, uint64_t bytes, stream_t st);
int launch_convert_f32(int prec, const float *src, void *dst, uint64_t n, stream_t st);

extern int g_use_mfma;

}  // namespace hmy
