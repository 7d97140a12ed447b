// Swap engine + iteration executor: the layer-pack-major training iteration of
// the Harmony paper (Section 3; task order of Algorithm 3 at N = 1) on one GPU.
//
// Streams (the paper's Runtime uses compute / swap-in / swap-out streams plus
// events, Section 4.4; p2p streams have no role on one GPU):
//   s_comp  every layer kernel
//   s_in    token ids, weight packs (prefetched one visit ahead, in n_micro pieces
//           interleaved with the microbatch loop) and checkpoints coming back
//   s_kin   optimizer state coming in, chunk by chunk, up to the ring's depth ahead
//   s_out   everything going to the host: checkpoints, updated state, gradients; also the
//           fused Adam kernel, which writes its results to the host itself (s_upd is an
//           alias of s_out: the engine stays within the 4 hardware queues a process has)
// All ordering is by events; the host thread only enqueues and finally waits.
//
// A "visit" is one task of the ordered list: forward packs in order, then
// backward packs in reverse, each followed by its update (jit-update).  The
// first backward visit is the last pack, run forward+backward per microbatch
// (jit-compute).  Visit v uses weight slot v % S (S = the schedule's weight_slots); the
// weights of visit v + distance are prefetched while visit v computes.  The forward visits
// run the minibatch in microbatches of U_F sequences, the backward visits in microbatches
// of U_B (Section 4.3.1: the configuration's two microbatch sizes).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <thread>

#include "hmy_internal.h"

namespace hmy {
const char *last_error();
}
using namespace hmy;

struct Visit {
  bool bwd;
  bool last;    // the shared last pack (forward + backward, no recompute)
  Pack pack;
  int slot;
  uint64_t poff;     // element offset of the pack's first parameter
  uint64_t nparams;
  int index;         // position in hmy_handle::visits (copies of a visit keep it)
};

struct hmy_handle {
  Model model;
  Packs packs;
  Arena arena;
  Split sp{};
  int M = 0, b = 0;     // backward pass: microbatches and sequences in each (sp.MB(), sp.uB)
  int MF = 0, bF = 0;   // forward pass (sp.MF(), sp.uF)
  int device = -1;
  bool dry = false;
  char *base = nullptr;
  bool own_arena = false;
  hipStream_t s_comp = nullptr, s_in = nullptr, s_kin = nullptr, s_upd = nullptr, s_out = nullptr;
  hmy_host_state host{};
  bool bound = false;
  char *stash_host = nullptr;   // pinned: checkpoints [n_ckpt][rows of the minibatch][d]
  std::vector<int> ckpt_layers; // first layers of backward packs 1..n_B-2
  std::vector<Visit> visits;
  BlockActs bacts;     // one block's saved activations at the backward microbatch size
  BlockActs bacts_F;   // the forward pass's scratch block at its own microbatch size
  HeadActs hacts;

  // per-iteration bookkeeping
  std::vector<hipEvent_t> sync_events;
  size_t sync_used = 0;
  std::vector<hipEvent_t> time_events;
  size_t time_used = 0;
  struct Span { size_t a, b; int what;   int tag = 0;
};  // what: 0 h2d, 1 d2h, 2 stall, 3 compute
  std::vector<Span> spans;
  int tag = 0;   // what the spans recorded now belong to: 1000 * visit + microbatch (timeline dump)
  hmy_stats st{};
  int err = HMY_OK;
  bool timing = true;
  int profile_level = 0;      // 0 counters only, 1 copy / stall / compute spans, 2 also every GEMM launch
  bool progress = false;      // wait for the compute stream after every visit and say so on stderr
  bool profile_gemm = false;
  // true (HMY_SWAP_OUT_KERNEL): the Adam kernel writes its results directly into the pinned host arrays;
  // false (HMY_SWAP_OUT_MEMCPY): results go to the ring / slot and leave by hipMemcpyAsync on s_out
  bool fused_swap_out = true;
  HostUpdater *updater = nullptr;   // Weight Update on the CPU (packs.update_site == HMY_UPDATE_ON_HOST)
  // Optimizer state resident on the device (HMY_STATE_RESIDENT_IN_SPARE_BUDGET): whole update chunks, numbered
  // in update order over the backward visits; the last res_chunks of them live behind the arena
  std::vector<int> first_chunk;   // per visit: number of its first chunk (-1: forward visit)
  int total_chunks = 0;
  int res_chunks = 0;
  uint64_t res_off = 0;           // byte offset of the resident region from base
  std::vector<char> res_loaded;   // per resident chunk: read from the host arrays since the last bind
  uint64_t chunk_state_bytes() const { return uint64_t(model.k_arrays()) * arena.res.karr_bytes; }
};

#define HIPCHK(h, call)                                                                      \
  do {                                                                                       \
    if ((h)->err == HMY_OK) {                                                                \
      hipError_t e_ = (call);                                                                \
      if (e_ != hipSuccess)                                                                  \
        (h)->err = fail(HMY_E_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
    }                                                                                        \
  } while (0)

namespace {

// ---- events -----------------------------------------------------------------
hipEvent_t rec(hmy_handle *h, hipStream_t s) {
  if (h->dry || h->err) return nullptr;
  if (h->sync_used == h->sync_events.size()) {
    hipEvent_t e = nullptr;
    HIPCHK(h, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    if (h->err) return nullptr;
    h->sync_events.push_back(e);
  }
  hipEvent_t e = h->sync_events[h->sync_used++];
  HIPCHK(h, hipEventRecord(e, s));
  return e;
}
void wait(hmy_handle *h, hipStream_t s, hipEvent_t e) {
  if (h->dry || h->err || !e) return;
  HIPCHK(h, hipStreamWaitEvent(s, e, 0));
}
size_t trec(hmy_handle *h, hipStream_t s) {
  if (h->dry || h->err || !h->timing) return size_t(-1);
  if (h->time_used == h->time_events.size()) {
    hipEvent_t e = nullptr;
    HIPCHK(h, hipEventCreate(&e));
    if (h->err) return size_t(-1);
    h->time_events.push_back(e);
  }
  size_t i = h->time_used++;
  HIPCHK(h, hipEventRecord(h->time_events[i], s));
  return i;
}
void span(hmy_handle *h, size_t a, size_t b, int what) {
  if (a != size_t(-1) && b != size_t(-1)) h->spans.push_back({a, b, what, h->tag});
}
// what a pair of event records costs with nothing between them (span kind 20), so that the time of
// a kernel bracketed by such a pair can be told from the bracket's
void calibrate_event_pair(hmy_handle *h) {
  if (!h->profile_gemm) return;
  for (int i = 0; i < 8; ++i) {
    const size_t a = trec(h, h->s_comp);
    const size_t b = trec(h, h->s_comp);
    span(h, a, b, 20);
  }
}
// wait on a swap event from the compute stream, measuring the stall
void comp_wait(hmy_handle *h, hipEvent_t e) {
  if (h->dry || h->err || !e) return;
  size_t a = trec(h, h->s_comp);
  wait(h, h->s_comp, e);
  size_t b = trec(h, h->s_comp);
  span(h, a, b, 2);
}

// ---- copies (bytes are counted when enqueued) ---------------------------------
void h2d(hmy_handle *h, int kind, void *dst, const void *src, uint64_t bytes, hipStream_t s) {
  if (!bytes) return;
  h->st.h2d[kind] += bytes;
  if (h->dry || h->err) return;
  size_t a = trec(h, s);
  HIPCHK(h, hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, s));
  size_t b = trec(h, s);
  span(h, a, b, 0);
}
void d2h(hmy_handle *h, int kind, void *dst, const void *src, uint64_t bytes, hipStream_t s) {
  if (!bytes) return;
  h->st.d2h[kind] += bytes;
  if (h->dry || h->err) return;
  size_t a = trec(h, s);
  HIPCHK(h, hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, s));
  size_t b = trec(h, s);
  span(h, a, b, 1);
}

// device -> pinned host through a throttled copy kernel on stream s (the library's blit
// for hipMemcpyAsync floods the fabric with stores to the link and stalls the kernels
// running beside it)
void d2h_kernel(hmy_handle *h, int kind, void *dst, const void *src, uint64_t bytes, hipStream_t s) {
  if (!bytes) return;
  h->st.d2h[kind] += bytes;
  if (h->dry || h->err) return;
  size_t a = trec(h, s);
  int rc = launch_copy_out(dst, src, bytes, s);
  if (rc) h->err = rc;
  size_t b = trec(h, s);
  span(h, a, b, 1);
}

#define KCHK(h, call)                          \
  do {                                         \
    if (!(h)->dry && (h)->err == HMY_OK) {     \
      int rc_ = (call);                        \
      if (rc_ != HMY_OK) (h)->err = rc_;       \
    }                                          \
  } while (0)

// ---- addressing -----------------------------------------------------------------
struct PackPtrs {
  char *W;    // compute-precision weights of the pack
  float *dW;  // fp32 gradient accumulators (backward visits)
};
PackPtrs pack_ptrs(const hmy_handle *h, const Visit &v) {
  PackPtrs p;
  p.W = h->base + h->arena.slot_off[v.slot];
  p.dW = reinterpret_cast<float *>(p.W + a256(uint64_t(h->model.elem_bytes()) * v.nparams));
  return p;
}
const char *wptr(const hmy_handle *h, const Visit &v, const PackPtrs &p, int tensor) {
  return p.W + (h->model.tensors[tensor].offset - v.poff) * h->model.elem_bytes();
}
float *gptr(const hmy_handle *h, const Visit &v, const PackPtrs &p, int tensor) {
  return p.dW + (h->model.tensors[tensor].offset - v.poff);
}
// the boundary activations of the minibatch are one [rows, d] array: microbatch mb of either pass is a run of rows
float *Xbuf(const hmy_handle *h, int mb, bool fwd) {
  return (float *)(h->base + h->arena.res.X + uint64_t(mb) * (fwd ? h->arena.res.x_bytes_F : h->arena.res.x_bytes_B));
}
char *inring(const hmy_handle *h, int r) { return h->base + h->arena.res.inring + uint64_t(r) * h->arena.res.in_bytes; }
char *outring(const hmy_handle *h, int r) { return h->base + h->arena.res.outring + uint64_t(r) * h->arena.res.out_bytes; }
const int32_t *ids_dev(const hmy_handle *h, int mb, bool fwd) {
  return reinterpret_cast<const int32_t *>(h->base + h->arena.res.ids) +
         uint64_t(mb) * (fwd ? h->bF : h->b) * h->model.spec.seq_len;
}
const int32_t *tgt_dev(const hmy_handle *h, int mb) {
  return reinterpret_cast<const int32_t *>(h->base + h->arena.res.targets) + uint64_t(mb) * h->b * h->model.spec.seq_len;
}
// activation region of `layer` inside the workspace of the pack being run
char *act_region(const hmy_handle *h, const Pack &pk, int layer) {
  uint64_t off = 0;
  for (int l = pk.a; l < layer; ++l) {
    if (l == 0) continue;
    off += (l <= h->model.spec.n_blocks) ? h->bacts.size : h->hacts.size;
  }
  return h->base + h->arena.act_off + off;
}

hmy_gemm_desc gemm_desc(int prec, int M, int N, int K) {
  hmy_gemm_desc g;
  std::memset(&g, 0, sizeof(g));
  g.prec = prec;
  g.M = M;
  g.N = N;
  g.K = K;
  return g;
}
// every GEMM of the iteration goes through here: counts algorithmic flops per
// kernel variant and, when profiling, brackets the launch with timing events
void run_gemm(hmy_handle *h, const hmy_gemm_desc &g) {
  const int variant = 2 * g.ta + g.tb;
  h->st.gemm_calls[variant] += 1;
  h->st.gemm_flops[variant] += 2.0 * g.M * g.N * g.K;
  if (h->dry || h->err) return;
  const size_t a = h->profile_gemm ? trec(h, h->s_comp) : size_t(-1);
  KCHK(h, launch_gemm(g, h->s_comp));
  const size_t b = h->profile_gemm ? trec(h, h->s_comp) : size_t(-1);
  span(h, a, b, 10 + variant);
}
// C[M,N] = A[M,K] W[N,K]^T + bias (+ res).  With a residual, res and C are the fp32 residual stream.
void linear_fwd(hmy_handle *h, const void *A, const void *W, const void *bias, const float *res, void *C,
                void *gelu_out, int M, int N, int K) {
  hmy_gemm_desc g = gemm_desc(h->model.spec.precision, M, N, K);
  g.A = A; g.lda = K;
  g.B = W; g.ldb = K; g.tb = 0;
  g.C = C; g.ldc = N;
  g.bias = bias;
  g.res = res; g.ldr = N;
  if (res) g.res_fp32 = g.c_fp32 = 1;
  g.gelu_out = gelu_out;
  run_gemm(h, g);
}
// dX[M,K] = dY[M,N] W[N,K];  dW[N,K] += dY^T X;  db[N] += colsum(dY)
void linear_bwd(hmy_handle *h, const void *dY, const void *X, const void *W, void *dX, float *dW, float *db,
                int M, int N, int K) {
  const int prec = h->model.spec.precision;
  if (dX) {
    hmy_gemm_desc g = gemm_desc(prec, M, K, N);
    g.A = dY; g.lda = N;
    g.B = W; g.ldb = K; g.tb = 1;
    g.C = dX; g.ldc = K;
    run_gemm(h, g);
  }
  {
    hmy_gemm_desc g = gemm_desc(prec, N, K, M);
    g.A = dY; g.lda = N; g.ta = 1;
    g.B = X; g.ldb = K; g.tb = 1;
    g.C = dW; g.ldc = K; g.c_fp32 = 1; g.accumulate = 1;
    run_gemm(h, g);
  }
  if (db) KCHK(h, launch_colsum(prec, dY, db, M, N, h->s_comp));
}

struct BlockPtrs {
  float *x_in, *x_mid;   // the residual stream: fp32
  char *a, *qkv, *o, *hh, *u, *g;
  float *ln1_mean, *ln1_rstd, *ln2_mean, *ln2_rstd, *lse;
};
BlockPtrs block_ptrs(const BlockActs &b, char *region) {
  BlockPtrs p;
  p.x_in = (float *)(region + b.x_in); p.a = region + b.a; p.qkv = region + b.qkv; p.o = region + b.o;
  p.x_mid = (float *)(region + b.x_mid); p.hh = region + b.h; p.u = region + b.u; p.g = region + b.g;
  p.ln1_mean = (float *)(region + b.ln1_mean); p.ln1_rstd = (float *)(region + b.ln1_rstd);
  p.ln2_mean = (float *)(region + b.ln2_mean); p.ln2_rstd = (float *)(region + b.ln2_rstd);
  p.lse = (float *)(region + b.lse);
  return p;
}

// Forward of one block.  x_in -> x_mid -> y; in the forward pass all three are
// the resident boundary buffer (in place); in a backward visit they are distinct
// saved buffers and y == nullptr skips the second MLP GEMM (output not needed).
void block_forward(hmy_handle *h, const Visit &v, const PackPtrs &pp, int layer, const BlockPtrs &A,
                   const float *x_in, float *x_mid, float *y, bool keep_preactivation, int b) {
  const hmy_model_spec &s = h->model.spec;
  const int prec = s.precision, T = b * s.seq_len, d = s.d_model, f = s.d_ffn;
  const int t0 = h->model.first_tensor[layer];
  auto W = [&](int i) { return wptr(h, v, pp, t0 + i); };
  KCHK(h, launch_layernorm_fwd(prec, x_in, W(LN1_G), W(LN1_B), A.a, A.ln1_mean, A.ln1_rstd, T, d, s.ln_eps, h->s_comp));
  linear_fwd(h, A.a, W(WQKV), W(BQKV), nullptr, A.qkv, nullptr, T, 3 * d, d);
  KCHK(h, launch_attn_fwd(prec, A.qkv, A.o, A.lse, b, s.seq_len, s.n_heads, d / s.n_heads, s.causal, h->s_comp));
  linear_fwd(h, A.o, W(WO), W(BO), x_in, x_mid, nullptr, T, d, d);
  KCHK(h, launch_layernorm_fwd(prec, x_mid, W(LN2_G), W(LN2_B), A.hh, A.ln2_mean, A.ln2_rstd, T, d, s.ln_eps, h->s_comp));
  // the MLP's pre-activation u is only read by a backward pass: without one, only gelu(u) is stored
  linear_fwd(h, A.hh, W(W1), W(B1), nullptr, keep_preactivation ? A.u : A.g, A.g, T, f, d);
  if (y) linear_fwd(h, A.g, W(W2), W(B2), x_mid, y, nullptr, T, d, f);
}

// Backward of one block; D (fp32) holds dL/dy on entry and dL/dx_in on exit (in place), and the buffer
// `dlow` holds the same values rounded to the element type: that copy is what the GEMMs read.
void block_backward(hmy_handle *h, const Visit &v, const PackPtrs &pp, int layer, const BlockPtrs &A,
                    const float *x_in, float *D) {
  const hmy_model_spec &s = h->model.spec;
  const int prec = s.precision, T = h->b * s.seq_len, d = s.d_model, f = s.d_ffn;
  const int t0 = h->model.first_tensor[layer];
  auto W = [&](int i) { return wptr(h, v, pp, t0 + i); };
  auto G = [&](int i) { return gptr(h, v, pp, t0 + i); };
  char *gbig = h->base + h->arena.res.gbig;
  char *gsmall = h->base + h->arena.res.gsmall;
  char *dlow = h->base + h->arena.res.dlow;
  float *delta = (float *)(h->base + h->arena.res.delta);
  // The per-workgroup sums of the LayerNorm backward kernels go into the gradients with atomics, not through a
  // workspace and a second kernel: alone on the device the two take the same time (19.9 against 20.1 us), but inside
  // the iteration every small launch costs more than its work (the reduction kernel 11.5 us for 5 us of work).
  // The bias gradients (column sums of a linear layer's output gradient) are taken by the kernel that has that
  // gradient in its registers anyway: b2's and bo's by the LayerNorm backward that reads the gradient stream D as its
  // residual input (from the fp32 values), b1's by the GELU backward that produces du, bqkv's by the attention
  // backward kernels that produce dqkv.
  // y = x_mid + W2 gelu(W1 LN2(x_mid) + b1) + b2
  linear_bwd(h, dlow, A.g, W(W2), gbig, G(W2), nullptr, T, d, f);                // dg
  KCHK(h, launch_gelu_bwd_colsum(prec, gbig, A.u, gbig, G(B1), T, f, h->s_comp));   // du, db1
  linear_bwd(h, gbig, A.hh, W(W1), gsmall, G(W1), nullptr, T, f, d);             // dh
  KCHK(h, launch_layernorm_bwd(prec, gsmall, A.x_mid, A.ln2_mean, A.ln2_rstd, W(LN2_G), D, D, dlow, G(LN2_G), G(LN2_B),
                               G(B2), T, d, h->s_comp));                                               // D = dx_mid, db2
  // x_mid = x_in + Wo attn(Wqkv LN1(x_in) + bqkv) + bo
  linear_bwd(h, dlow, A.o, W(WO), gsmall, G(WO), nullptr, T, d, d);              // do
  KCHK(h, launch_attn_bwd(prec, A.qkv, A.o, gsmall, A.lse, delta, gbig, G(BQKV), h->b, s.seq_len, s.n_heads,
                          d / s.n_heads, s.causal, h->s_comp));                    // dqkv, dbqkv
  linear_bwd(h, gbig, A.a, W(WQKV), gsmall, G(WQKV), nullptr, T, 3 * d, d);      // da
  KCHK(h, launch_layernorm_bwd(prec, gsmall, x_in, A.ln1_mean, A.ln1_rstd, W(LN1_G), D, D, dlow, G(LN1_G), G(LN1_B),
                               G(BO), T, d, h->s_comp));                                               // D = dx_in, dbo
}

// Final norm, vocabulary projection, loss and their backward.  The fp32 logits exist one chunk of
// rows at a time; their gradient (element type) is kept for the whole microbatch, so that the two
// GEMMs consuming it run once with T rows.  Writes dL/dx into D.
void head_forward_backward(hmy_handle *h, const Visit &v, const PackPtrs &pp, int layer, char *region,
                           const float *x_in, int mb, float *D, float inv_ntgt) {
  const hmy_model_spec &s = h->model.spec;
  const int prec = s.precision, T = h->b * s.seq_len, d = s.d_model, V = s.vocab, E = h->model.elem_bytes();
  const HeadActs &ha = h->hacts;
  const int t0 = h->model.first_tensor[layer];
  const char *lnf_g = wptr(h, v, pp, t0 + 0), *lnf_b = wptr(h, v, pp, t0 + 1), *wh = wptr(h, v, pp, t0 + 2);
  float *g_lnf_g = gptr(h, v, pp, t0 + 0), *g_lnf_b = gptr(h, v, pp, t0 + 1), *g_wh = gptr(h, v, pp, t0 + 2);
  char *z = region + ha.z;
  float *mean = (float *)(region + ha.mean), *rstd = (float *)(region + ha.rstd);
  float *logits = (float *)(region + ha.logits);
  char *dlogits = region + ha.dlogits;
  char *dz = h->base + h->arena.res.gsmall;
  double *loss_acc = (double *)(h->base + h->arena.res.misc);
  KCHK(h, launch_layernorm_fwd(prec, x_in, lnf_g, lnf_b, z, mean, rstd, T, d, s.ln_eps, h->s_comp));
  for (int r0 = 0; r0 < T; r0 += ha.chunk_rows) {
    const int rows = std::min(ha.chunk_rows, T - r0);
    const char *zc = z + uint64_t(r0) * d * E;
    {  // logits = z Wh^T (fp32)
      hmy_gemm_desc g = gemm_desc(prec, rows, V, d);
      g.A = zc; g.lda = d;
      g.B = wh; g.ldb = d;
      g.C = logits; g.ldc = ha.ldl; g.c_fp32 = 1;
      run_gemm(h, g);
    }
    KCHK(h, launch_xent(prec, logits, tgt_dev(h, mb) + r0, loss_acc, dlogits + uint64_t(r0) * ha.ldl * E, rows, V, ha.ldl,
                        inv_ntgt, h->s_comp));
  }
  {  // dz = dlogits Wh: a vocabulary-long contraction (ragged, and split over workgroups when T is
     // small), so it is accumulated in fp32 and rounded afterwards
    float *dz32 = (float *)(region + ha.dz32);
    KCHK(h, launch_fill_zero(dz32, uint64_t(T) * d * 4, h->s_comp));
    hmy_gemm_desc g = gemm_desc(prec, T, d, V);
    g.A = dlogits; g.lda = ha.ldl;
    g.B = wh; g.ldb = d; g.tb = 1;
    g.C = dz32; g.ldc = d; g.c_fp32 = 1; g.accumulate = 1;
    run_gemm(h, g);
    KCHK(h, launch_convert_f32(prec, dz32, dz, uint64_t(T) * d, h->s_comp));
  }
  {  // dWh += dlogits^T z
    hmy_gemm_desc g = gemm_desc(prec, V, d, T);
    g.A = dlogits; g.lda = ha.ldl; g.ta = 1;
    g.B = z; g.ldb = d; g.tb = 1;
    g.C = g_wh; g.ldc = d; g.c_fp32 = 1; g.accumulate = 1;
    run_gemm(h, g);
  }
  KCHK(h, launch_layernorm_bwd(prec, dz, x_in, mean, rstd, lnf_g, nullptr, D, h->base + h->arena.res.dlow, g_lnf_g,
                               g_lnf_b, nullptr, T, d, h->s_comp));
}

struct PendingUpdate {
  const Visit *v = nullptr;
  hipEvent_t bwd_done = nullptr;
  int next = 0, n_chunks = 0;
};

struct IterState {
  PendingUpdate upd;
  bool compute_done = false;   // nothing is left to enqueue on the compute stream
  hipEvent_t slot_free[kMaxSlots] = {};
  hipEvent_t in_free[kInRing] = {};
  hipEvent_t in_ready[kInRing] = {};
  hipEvent_t out_free[kOutRing] = {};
  hipEvent_t k_free[kKRing] = {};
  hipEvent_t stash_all_out = nullptr;
  bool stash_waited = false;
  int out_count = 0;
  int k_count = 0;
  float inv_ntgt = 0.f;
};

int ckpt_index(const hmy_handle *h, int layer) {
  for (size_t i = 0; i < h->ckpt_layers.size(); ++i)
    if (h->ckpt_layers[i] == layer) return int(i);
  return -1;
}
// checkpoint ck of the whole minibatch is one [rows, d] array like X; either pass addresses its own microbatch in it
char *stash_slot(const hmy_handle *h, int ck, int mb, bool fwd) {
  const Reserved &r = h->arena.res;
  return h->stash_host + uint64_t(ck) * (uint64_t(h->M) * r.ck_bytes_B) + uint64_t(mb) * (fwd ? r.ck_bytes_F : r.ck_bytes_B);
}

void forward_visit_microbatch(hmy_handle *h, IterState &it, const Visit &v, int mb) {
  const hmy_model_spec &s = h->model.spec;
  const int T = h->bF * s.seq_len, d = s.d_model;
  const uint64_t xb = h->arena.res.ck_bytes_F;
  const PackPtrs pp = pack_ptrs(h, v);
  float *X = Xbuf(h, mb, true);
  const BlockPtrs scratch = block_ptrs(h->bacts_F, h->base + h->arena.act_off);
  for (int layer = v.pack.a; layer < v.pack.e; ++layer) {
    const int ck = ckpt_index(h, layer);
    if (ck >= 0) {  // this layer's input is a backward pack's checkpoint: send it to the host
      const int q = it.out_count++ % kOutRing;
      comp_wait(h, it.out_free[q]);
      // the checkpoint leaves rounded to the element type (one rounding per pack boundary)
      KCHK(h, launch_convert_f32(s.precision, X, outring(h, q), uint64_t(T) * d, h->s_comp));
      hipEvent_t e = rec(h, h->s_comp);
      wait(h, h->s_out, e);
      if (h->fused_swap_out) d2h_kernel(h, HMY_KIND_SX, stash_slot(h, ck, mb, true), outring(h, q), xb, h->s_out);
      else d2h(h, HMY_KIND_SX, stash_slot(h, ck, mb, true), outring(h, q), xb, h->s_out);
      it.out_free[q] = rec(h, h->s_out);
    }
    if (layer == 0) {
      const int t0 = h->model.first_tensor[0];
      KCHK(h, launch_embed_fwd(s.precision, ids_dev(h, mb, true), wptr(h, v, pp, t0), wptr(h, v, pp, t0 + 1), X, T, d,
                               s.seq_len, s.vocab, h->s_comp));
    } else {
      block_forward(h, v, pp, layer, scratch, X, X, X, false, h->bF);
    }
  }
}

// where the first layer of a backward visit's pack reads its input (fp32, inside the pack's workspace)
float *first_input(const hmy_handle *h, const Visit &v) {
  char *reg = act_region(h, v.pack, v.pack.a);
  return (float *)(v.pack.a <= h->model.spec.n_blocks ? reg + h->bacts.x_in : reg + h->hacts.x_in);
}

// enqueue whatever brings the input of backward visit v, microbatch mb: a checkpoint from the host into
// inring[mb % kInRing] (element type), or the still resident activations into the pack's workspace
void issue_pack_input(hmy_handle *h, IterState &it, const Visit &v, int mb) {
  const int r = mb % kInRing;
  const uint64_t xb = h->arena.res.ck_bytes_B;
  it.in_ready[r] = nullptr;
  if (v.pack.a == 0) return;  // starts at the embedding: restarts from the token ids
  if (v.last) {               // still resident from the forward pass: straight into the first layer's input buffer
    KCHK(h, launch_copy(first_input(h, v), Xbuf(h, mb, false), h->arena.res.x_bytes_B, h->s_comp));
    return;
  }
  const int ck = ckpt_index(h, v.pack.a);
  if (!it.stash_waited) {
    wait(h, h->s_in, it.stash_all_out);
    it.stash_waited = true;
  }
  wait(h, h->s_in, it.in_free[r]);
  h2d(h, HMY_KIND_SX, inring(h, r), stash_slot(h, ck, mb, false), xb, h->s_in);
  it.in_ready[r] = rec(h, h->s_in);
}

void backward_visit_microbatch(hmy_handle *h, IterState &it, const Visit &v, int mb) {
  const hmy_model_spec &s = h->model.spec;
  const int T = h->b * s.seq_len, d = s.d_model, L = s.n_blocks;
  const PackPtrs pp = pack_ptrs(h, v);
  const int r = mb % kInRing;
  float *D = Xbuf(h, mb, false);
  comp_wait(h, it.in_ready[r]);
  // where each layer of the pack reads its input
  auto input_of = [&](int layer) -> float * {
    char *reg = act_region(h, v.pack, layer);
    return (float *)(layer <= L ? reg + h->bacts.x_in : reg + h->hacts.x_in);
  };
  if (it.in_ready[r])   // a checkpoint has arrived in the ring: widen it into the first layer's input
    KCHK(h, launch_convert_to_f32(s.precision, inring(h, r), first_input(h, v), uint64_t(T) * d, h->s_comp));
  if (!v.last)          // the gradient handed down by the pack above, rounded for the GEMMs that read it
    KCHK(h, launch_convert_f32(s.precision, D, h->base + h->arena.res.dlow, uint64_t(T) * d, h->s_comp));
  // (re)compute the pack's forward, keeping what backward needs
  for (int layer = v.pack.a; layer < v.pack.e; ++layer) {
    const bool has_next = layer + 1 < v.pack.e;
    if (layer == 0) {
      if (!has_next) continue;  // embedding alone: its backward needs only ids and dY
      const int t0 = h->model.first_tensor[0];
      KCHK(h, launch_embed_fwd(s.precision, ids_dev(h, mb, false), wptr(h, v, pp, t0), wptr(h, v, pp, t0 + 1), input_of(1), T,
                               d, s.seq_len, s.vocab, h->s_comp));
    } else if (layer <= L) {
      const BlockPtrs A = block_ptrs(h->bacts, act_region(h, v.pack, layer));
      block_forward(h, v, pp, layer, A, input_of(layer), A.x_mid, has_next ? input_of(layer + 1) : nullptr, true, h->b);
    } else {
      head_forward_backward(h, v, pp, layer, act_region(h, v.pack, layer), input_of(layer), mb, D, it.inv_ntgt);
    }
  }
  // backward in reverse (the head's backward already ran, fused with its forward)
  for (int layer = std::min(v.pack.e - 1, L); layer >= v.pack.a; --layer) {
    if (layer == 0) {
      const int t0 = h->model.first_tensor[0];
      KCHK(h, launch_embed_bwd(s.precision, ids_dev(h, mb, false), D, gptr(h, v, pp, t0), gptr(h, v, pp, t0 + 1), T, d,
                               s.seq_len, s.vocab, h->s_comp));
    } else {
      const BlockPtrs A = block_ptrs(h->bacts, act_region(h, v.pack, layer));
      block_backward(h, v, pp, layer, A, input_of(layer), D);
    }
  }
  it.in_free[r] = rec(h, h->s_comp);
}

// jit-update of a visit's pack: optimizer state streams through the ring in chunks
// (in on s_upd, Adam on s_upd, results out by the same kernel or on s_out) while the
// next pack computes.  Chunks are enqueued a few at a time from the next visit's
// microbatch loop: a host->device copy that has to wait for its ring slot holds up every
// copy queued behind it on the copy engine, checkpoint reads of the running visit
// included, so no more of them are queued ahead than one microbatch's worth.
void update_chunk(hmy_handle *h, IterState &it, const hmy_adam &hp) {
  PendingUpdate &u = it.upd;
  const Visit &v = *u.v;
  const Reserved &R = h->arena.res;
  const int E = h->model.elem_bytes();
  const bool mixed = h->model.spec.precision == HMY_PREC_BF16;
  const PackPtrs pp = pack_ptrs(h, v);
  const uint64_t lo = uint64_t(u.next) * R.k_chunk_params;
  const uint64_t n = std::min<uint64_t>(R.k_chunk_params, v.nparams - lo);
  const uint64_t g0 = v.poff + lo;  // element offset in the host arrays
  // a chunk whose state lives on the device: updated in place there, nothing of it crosses the link
  const int rslot = h->first_chunk[v.index] + u.next - (h->total_chunks - h->res_chunks);
  const bool resident = rslot >= 0;
  const int r = resident ? 0 : it.k_count++ % kKRing;
  char *ring = resident ? h->base + h->res_off + uint64_t(rslot) * h->chunk_state_bytes()
                        : h->base + R.kring + uint64_t(r) * h->model.k_arrays() * R.karr_bytes;
  float *r_master = mixed ? (float *)ring : nullptr;
  float *r_m = (float *)(ring + (mixed ? 1 : 0) * R.karr_bytes);
  float *r_v = (float *)(ring + (mixed ? 2 : 1) * R.karr_bytes);
  if (resident) {
    if (!h->res_loaded[rslot]) {   // first update since the arrays were bound: read it as a swapped chunk would be
      if (mixed) h2d(h, HMY_KIND_K, r_master, h->dry ? nullptr : h->host.master + g0, n * 4, h->s_kin);
      h2d(h, HMY_KIND_K, r_m, h->dry ? nullptr : h->host.adam_m + g0, n * 4, h->s_kin);
      h2d(h, HMY_KIND_K, r_v, h->dry ? nullptr : h->host.adam_v + g0, n * 4, h->s_kin);
      wait(h, h->s_upd, rec(h, h->s_kin));
      if (!h->err) h->res_loaded[rslot] = 1;
    }
  } else {
    // on a stream of their own, so that chunk c+1 arrives while chunk c is updated
    wait(h, h->s_kin, it.k_free[r]);
    if (mixed) h2d(h, HMY_KIND_K, r_master, h->dry ? nullptr : h->host.master + g0, n * 4, h->s_kin);
    h2d(h, HMY_KIND_K, r_m, h->dry ? nullptr : h->host.adam_m + g0, n * 4, h->s_kin);
    h2d(h, HMY_KIND_K, r_v, h->dry ? nullptr : h->host.adam_v + g0, n * 4, h->s_kin);
    wait(h, h->s_upd, rec(h, h->s_kin));
  }
  if (u.next == 0) wait(h, h->s_upd, u.bwd_done);
  const bool export_g = h->packs.gradients == HMY_GRADIENTS_EXPORTED;
  if (h->fused_swap_out) {
    // the update kernel itself writes state, weights and (if exported) gradients to the host
    // arrays (device->host over the link at vector width); bytes are counted as for copies
    if (!resident) h->st.d2h[HMY_KIND_K] += uint64_t(h->model.k_arrays()) * n * 4;
    h->st.d2h[HMY_KIND_W] += n * E;
    if (export_g) h->st.d2h[HMY_KIND_DW] += n * 4;
    if (!h->dry && !h->err) {
      const size_t a = trec(h, h->s_upd);
      KCHK(h, launch_adam_out(h->model.spec.precision, pp.dW + lo, mixed ? r_master : (const float *)(pp.W + lo * E),
                              r_m, r_v, !mixed ? nullptr : resident ? r_master : h->host.master + g0,
                              resident ? r_m : h->host.adam_m + g0, resident ? r_v : h->host.adam_v + g0,
                              (char *)h->host.weights + g0 * E,
                              export_g ? h->host.grads + g0 : nullptr, n, hp, it.compute_done, h->s_upd));
      const size_t b2 = trec(h, h->s_upd);
      span(h, a, b2, 1);
    }
    if (!resident) it.k_free[r] = rec(h, h->s_upd);
  } else {
    KCHK(h, launch_adam(h->model.spec.precision, pp.dW + lo, r_master, r_m, r_v, pp.W + lo * E, n, hp, h->s_upd));
    hipEvent_t e = rec(h, h->s_upd);
    wait(h, h->s_out, e);
    if (!resident) {
      if (mixed) d2h(h, HMY_KIND_K, h->dry ? nullptr : h->host.master + g0, r_master, n * 4, h->s_out);
      d2h(h, HMY_KIND_K, h->dry ? nullptr : h->host.adam_m + g0, r_m, n * 4, h->s_out);
      d2h(h, HMY_KIND_K, h->dry ? nullptr : h->host.adam_v + g0, r_v, n * 4, h->s_out);
    }
    d2h(h, HMY_KIND_W, h->dry ? nullptr : (char *)h->host.weights + g0 * E, pp.W + lo * E, n * E, h->s_out);
    if (export_g) d2h(h, HMY_KIND_DW, h->dry ? nullptr : h->host.grads + g0, pp.dW + lo, n * 4, h->s_out);
    if (!resident) it.k_free[r] = rec(h, h->s_out);
  }
  if (++u.next == u.n_chunks) {   // the pack has left: its slot may be refilled
    it.slot_free[v.slot] = rec(h, h->fused_swap_out ? h->s_upd : h->s_out);
    u.v = nullptr;
  }
}
// enqueue chunks of the pending update until `upto` of them have been (all if negative)
void update_progress(hmy_handle *h, IterState &it, const hmy_adam &hp, int upto) {
  while (it.upd.v && (upto < 0 || it.upd.next < upto)) update_chunk(h, it, hp);
}
void update_begin(hmy_handle *h, IterState &it, const Visit &v, hipEvent_t bwd_done, const hmy_adam &hp) {
  update_progress(h, it, hp, -1);   // nothing of an older update may be left behind
  const uint64_t c = h->arena.res.k_chunk_params;
  it.upd.v = &v;
  it.upd.bwd_done = bwd_done;
  it.upd.next = 0;
  it.upd.n_chunks = int((v.nparams + c - 1) / c);
}

// Weight Update on the host: the pack's gradient leaves for the pinned gradient array chunk by
// chunk; each chunk's event is handed to the CPU threads, which apply Adam to the pinned state
// in place as soon as it has arrived.  Nothing else of the pack crosses the link.
void host_update_begin(hmy_handle *h, IterState &it, const Visit &v, hipEvent_t bwd_done, const hmy_adam &hp) {
  const uint64_t c = h->arena.res.k_chunk_params;
  const int E = h->model.elem_bytes();
  const bool mixed = h->model.spec.precision == HMY_PREC_BF16;
  const PackPtrs pp = pack_ptrs(h, v);
  wait(h, h->s_out, bwd_done);
  for (uint64_t lo = 0; lo < v.nparams; lo += c) {
    const uint64_t n = std::min<uint64_t>(c, v.nparams - lo), g0 = v.poff + lo;
    float *dst = h->dry ? nullptr : h->host.grads + g0;
    if (h->fused_swap_out) d2h_kernel(h, HMY_KIND_DW, dst, pp.dW + lo, n * 4, h->s_out);
    else d2h(h, HMY_KIND_DW, dst, pp.dW + lo, n * 4, h->s_out);
    hipEvent_t arrived = rec(h, h->s_out);
    if (h->dry || h->err) continue;
    h->updater->submit(make_host_adam_job(arrived, h->host.grads + g0, mixed ? h->host.master + g0 : nullptr,
                                          h->host.adam_m + g0, h->host.adam_v + g0, (char *)h->host.weights + g0 * E, n,
                                          hp));
  }
  it.slot_free[v.slot] = rec(h, h->s_out);
}
int updater_thread_init(void *arg, void *) {
  return hipSetDevice(static_cast<hmy_handle *>(arg)->device) == hipSuccess ? HMY_OK : HMY_E_HIP;
}
int updater_wait(void *, void *ready) {
  return hipEventSynchronize(static_cast<hipEvent_t>(ready)) == hipSuccess ? HMY_OK : HMY_E_HIP;
}
// the update that follows a pack's (last) backward task, wherever the schedule places it
void pack_update_begin(hmy_handle *h, IterState &it, const Visit &v, hipEvent_t bwd_done, const hmy_adam &hp) {
  if (h->packs.update_site == HMY_UPDATE_ON_HOST) host_update_begin(h, it, v, bwd_done, hp);
  else update_begin(h, it, v, bwd_done, hp);
}

void run_iteration(hmy_handle *h, const hmy_minibatch *mb, const hmy_adam &hp) {
  const hmy_model_spec &s = h->model.spec;
  const int M = h->M, E = h->model.elem_bytes();
  const uint64_t T = uint64_t(h->b) * s.seq_len;
  IterState it;
  std::memset(&h->st, 0, sizeof(h->st));
  h->sync_used = h->time_used = 0;
  h->spans.clear();

  if (!h->dry) {
    uint64_t nt = 0;
    for (uint64_t i = 0; i < uint64_t(M) * T; ++i) nt += mb->targets[i] >= 0;
    h->st.n_targets = nt;
    it.inv_ntgt = nt ? float(1.0 / double(nt)) : 0.f;
  }
  h2d(h, HMY_KIND_IDS, h->base + h->arena.res.ids, h->dry ? nullptr : mb->token_ids, uint64_t(M) * T * 4, h->s_in);
  h2d(h, HMY_KIND_IDS, h->base + h->arena.res.targets, h->dry ? nullptr : mb->targets, uint64_t(M) * T * 4, h->s_in);
  hipEvent_t ev_ids = rec(h, h->s_in);
  KCHK(h, launch_fill_zero(h->base + h->arena.res.misc, 4096, h->s_comp));
  const size_t t_first = trec(h, h->s_comp);
  calibrate_event_pair(h);

  // weight prefetch of a visit in `pieces` pieces.  Its slot was last used by the visit S places earlier: if that
  // one's update is still being handed out chunk by chunk, all of it has to be enqueued first, or the event
  // that says "the slot is free" does not exist yet.
  auto w_piece = [&](const Visit &v, int piece, int pieces) {
    const uint64_t total = uint64_t(E) * v.nparams;
    const uint64_t chunk = a256((total + pieces - 1) / pieces);
    const uint64_t lo = std::min(total, chunk * piece), hi = std::min(total, chunk * (piece + 1));
    if (piece == 0) {
      if (it.upd.v && it.upd.v->slot == v.slot) update_progress(h, it, hp, -1);
      wait(h, h->s_in, it.slot_free[v.slot]);
    }
    if (hi > lo) {
      char *dst = h->base + h->arena.slot_off[v.slot] + lo;
      const char *src = h->dry ? nullptr : (const char *)h->host.weights + v.poff * E + lo;
      h2d(h, HMY_KIND_W, dst, src, hi - lo, h->s_in);
    }
  };

  const int nv = int(h->visits.size()), dist = h->packs.distance;
  std::vector<hipEvent_t> ev_w(size_t(nv), nullptr);   // per visit: its weights have arrived
  for (int vi = 0; vi < std::min(dist, nv); ++vi) {
    w_piece(h->visits[vi], 0, 1);
    ev_w[vi] = rec(h, h->s_in);
  }
  for (int vi = 0; vi < nv; ++vi) {
    const Visit &v = h->visits[vi];
    const Visit *ahead = vi + dist < nv ? &h->visits[vi + dist] : nullptr;   // the visit whose weights travel now
    const bool final_visit = vi + 1 == nv;
    const int Mv = v.bwd ? M : h->MF;                                        // microbatches of this visit's pass
    // The slot those weights go to may still belong to the pack whose update is being handed out during this
    // visit (prefetch distance = slots - 1).  Then the load cannot start before that update has left anyway:
    // it is requested behind the update's last chunk, in the visit's last microbatch, instead of holding up the
    // link's queue (checkpoint reads of this visit included) from the visit's start.
    const bool defer = ahead && it.upd.v && it.upd.v->slot == ahead->slot;
    // With the update on the host the same slot is held by the gradient export of the visit before this one, which
    // is already on its way (it is enqueued in one go).  Requested now, the load would sit in the link's queue
    // until that export is over and hold up this visit's checkpoint reads behind it (measured on 32 blocks of
    // d = 4096 in two slots: the compute stream waited 45 ms per visit).  So the host thread itself waits for the
    // export, after it has enqueued all of this visit, and requests the load then: nothing queues behind a copy
    // that cannot start, and the GPU has this visit's work to go on with meanwhile.
    const bool after_export = ahead && !defer && h->packs.update_site == HMY_UPDATE_ON_HOST && vi >= 1 &&
                              h->visits[vi - 1].bwd && h->visits[vi - 1].slot == ahead->slot;
    comp_wait(h, ev_w[vi]);
    if (vi == 0) comp_wait(h, ev_ids);
    if (v.bwd) {
      if (!it.stash_all_out) it.stash_all_out = rec(h, h->s_out);  // every checkpoint has been queued out
      const PackPtrs pp = pack_ptrs(h, v);
      KCHK(h, launch_fill_zero(pp.dW, v.nparams * 4, h->s_comp));
    }
    for (int m = 0; m < Mv; ++m) {
      h->tag = 1000 * vi + m;
      if (v.bwd) {
        // checkpoints are requested kInRing - 1 microbatches ahead: the copy engine's queue
        // may hold optimizer chunks in front of them that wait for their ring slots
        const bool from_host = !v.last && v.pack.a != 0;
        if (m == 0)
          for (int q = 0; q < (from_host ? std::min(Mv, kInRing - 1) : 1); ++q) issue_pack_input(h, it, v, q);
        if (from_host && m + kInRing - 1 < Mv) issue_pack_input(h, it, v, m + kInRing - 1);
      }
      if (ahead && !defer && !after_export) w_piece(*ahead, m, Mv);
      // this microbatch's share of the previous visit's update
      // (not behind a final visit that is the embedding alone: it is over in a moment, and
      // what is left of the update then runs at the full link rate)
      const bool tiny_last = final_visit && v.pack.a == 0 && v.pack.e == 1;
      if (it.upd.v && !tiny_last) update_progress(h, it, hp, (it.upd.n_chunks * (m + 1) + Mv - 1) / Mv);
      if (ahead && defer && m == Mv - 1)
        for (int piece = 0; piece < Mv; ++piece) w_piece(*ahead, piece, Mv);
      if (v.bwd) {
        if (m > 0 && (v.last || v.pack.a == 0)) issue_pack_input(h, it, v, m);
        backward_visit_microbatch(h, it, v, m);
      } else {
        forward_visit_microbatch(h, it, v, m);
      }
    }
    if (ahead && !after_export) ev_w[vi + dist] = rec(h, h->s_in);
    if (!v.bwd) {
      it.slot_free[v.slot] = rec(h, h->s_comp);
    } else {
      if (final_visit) it.compute_done = true;   // nothing else will be enqueued on the compute stream
      pack_update_begin(h, it, v, rec(h, h->s_comp), hp);
    }
    if (after_export) {
      if (!h->dry && !h->err && it.slot_free[ahead->slot]) {
        // polled with short sleeps: a spinning wait would take a core from the threads that apply the update
        hipError_t q;
        while ((q = hipEventQuery(it.slot_free[ahead->slot])) == hipErrorNotReady)
          std::this_thread::sleep_for(std::chrono::microseconds(100));
        (void)hipGetLastError();   // "not ready" is no error, but the runtime may keep it as its last one
        HIPCHK(h, q);
      }
      w_piece(*ahead, 0, 1);
      ev_w[vi + dist] = rec(h, h->s_in);
    }
    if (h->progress && !h->dry && !h->err) {
      // for runs under a profiler that serialises every dispatch: a line per visit, once its kernels have run
      HIPCHK(h, hipStreamSynchronize(h->s_comp));
      std::fprintf(stderr, "hmy: visit %d of %d done (%s pack [%d, %d), %d microbatches)\n", vi + 1, nv,
                   v.bwd ? "backward" : "forward", v.pack.a, v.pack.e, Mv);
      std::fflush(stderr);
    }
  }
  it.compute_done = true;
  update_progress(h, it, hp, -1);   // the first pack's update has no visit to hide behind
  const size_t t_last = trec(h, h->s_comp);
  span(h, t_first, t_last, 3);
}

// The order the paper compares against (Section 3, "Intuitive Example"; appendix
// "Additional Swap Analysis" for the gradients): the same visits, but every microbatch
// walks through all of them before the next one starts.  Weights come in for every
// (visit, microbatch); a backward pack's gradient sums go home to the host gradient array
// after each of its tasks and come back before the next microbatch's; the update follows
// the last microbatch's task while the pack is still resident.  The next visit's weights are
// prefetched into another slot while the current one computes, as in the method's own order.
void run_iteration_microbatch_major(hmy_handle *h, const hmy_minibatch *mb, const hmy_adam &hp) {
  const hmy_model_spec &s = h->model.spec;
  const int M = h->M, E = h->model.elem_bytes();
  const uint64_t T = uint64_t(h->b) * s.seq_len;
  IterState it;
  std::memset(&h->st, 0, sizeof(h->st));
  h->sync_used = h->time_used = 0;
  h->spans.clear();

  if (!h->dry) {
    uint64_t nt = 0;
    for (uint64_t i = 0; i < uint64_t(M) * T; ++i) nt += mb->targets[i] >= 0;
    h->st.n_targets = nt;
    it.inv_ntgt = nt ? float(1.0 / double(nt)) : 0.f;
  }
  h2d(h, HMY_KIND_IDS, h->base + h->arena.res.ids, h->dry ? nullptr : mb->token_ids, uint64_t(M) * T * 4, h->s_in);
  h2d(h, HMY_KIND_IDS, h->base + h->arena.res.targets, h->dry ? nullptr : mb->targets, uint64_t(M) * T * 4, h->s_in);
  hipEvent_t ev_ids = rec(h, h->s_in);
  KCHK(h, launch_fill_zero(h->base + h->arena.res.misc, 4096, h->s_comp));
  const size_t t_first = trec(h, h->s_comp);
  calibrate_event_pair(h);

  // the visit sequence of the whole iteration; slots rotate over it
  const int nv = int(h->visits.size());
  std::vector<Visit> seq;
  seq.reserve(size_t(M) * nv);
  for (int m = 0; m < M; ++m)
    for (int vi = 0; vi < nv; ++vi) {
      Visit v = h->visits[vi];
      v.slot = int(seq.size() % size_t(h->packs.slots));
      seq.push_back(v);
    }
  std::vector<hipEvent_t> grads_home(nv, nullptr);   // per visit of a microbatch: its gradient sums have reached the host

  auto load_weights = [&](const Visit &v) {
    // the slot's last user may still have its update handed out chunk by chunk: all of it first (see run_iteration)
    if (it.upd.v && it.upd.v->slot == v.slot) update_progress(h, it, hp, -1);
    wait(h, h->s_in, it.slot_free[v.slot]);
    h2d(h, HMY_KIND_W, h->base + h->arena.slot_off[v.slot], h->dry ? nullptr : (const char *)h->host.weights + v.poff * E,
        uint64_t(E) * v.nparams, h->s_in);
    return rec(h, h->s_in);
  };
  // what earlier microbatches added to this pack's gradient; enqueued only after the task that
  // sent those sums out has been enqueued (two consecutive visits can be the same pack)
  auto load_gradient_sums = [&](const Visit &v, int vi) {
    wait(h, h->s_in, grads_home[vi]);
    h2d(h, HMY_KIND_DW, pack_ptrs(h, v).dW, h->dry ? nullptr : h->host.grads + v.poff, v.nparams * 4, h->s_in);
    return rec(h, h->s_in);
  };

  hipEvent_t ev_w = load_weights(seq[0]);
  const int total = M * nv;
  for (int g = 0; g < total; ++g) {
    const Visit &v = seq[g];
    const int m = g / nv, vi = g % nv;
    const Visit *next = g + 1 < total ? &seq[g + 1] : nullptr;
    const int next_m = (g + 1) / nv, next_vi = (g + 1) % nv;
    h->tag = 1000 * vi + m;
    comp_wait(h, ev_w);
    if (g == 0) comp_wait(h, ev_ids);
    if (v.bwd) {
      if (v.last) {   // first backward task of this microbatch: its checkpoints have all been queued out
        it.stash_all_out = rec(h, h->s_out);
        it.stash_waited = false;
      }
      if (m == 0) KCHK(h, launch_fill_zero(pack_ptrs(h, v).dW, v.nparams * 4, h->s_comp));
      issue_pack_input(h, it, v, m);
    }
    if (next) ev_w = load_weights(*next);
    update_progress(h, it, hp, -1);   // the update of the previous visit, if it had one
    if (v.bwd) backward_visit_microbatch(h, it, v, m);
    else forward_visit_microbatch(h, it, v, m);
    if (!v.bwd) {
      it.slot_free[v.slot] = rec(h, h->s_comp);
    } else if (m == M - 1) {
      if (!next) it.compute_done = true;
      pack_update_begin(h, it, v, rec(h, h->s_comp), hp);
    } else {
      wait(h, h->s_out, rec(h, h->s_comp));
      float *dst = h->dry ? nullptr : h->host.grads + v.poff;
      if (h->fused_swap_out) d2h_kernel(h, HMY_KIND_DW, dst, pack_ptrs(h, v).dW, v.nparams * 4, h->s_out);
      else d2h(h, HMY_KIND_DW, dst, pack_ptrs(h, v).dW, v.nparams * 4, h->s_out);
      grads_home[vi] = it.slot_free[v.slot] = rec(h, h->s_out);
    }
    if (next && next->bwd && next_m > 0) ev_w = load_gradient_sums(*next, next_vi);
  }
  it.compute_done = true;
  update_progress(h, it, hp, -1);
  const size_t t_last = trec(h, h->s_comp);
  span(h, t_first, t_last, 3);
}

void run_in_order(hmy_handle *h, const hmy_minibatch *mb, const hmy_adam &hp) {
  if (h->packs.order == HMY_ORDER_MICROBATCH_MAJOR) run_iteration_microbatch_major(h, mb, hp);
  else run_iteration(h, mb, hp);
}

}  // namespace

// ---- handle construction ---------------------------------------------------------
static int init_handle(hmy_handle *h, const hmy_model_spec *spec, const hmy_schedule *sched, const hmy_budget *budget,
                       int n_micro, int micro_batch) {
  int rc = build_model(spec, &h->model);
  if (rc) return rc;
  if (n_micro < 1 || micro_batch < 1) return fail(HMY_E_INVALID, "n_micro and micro_batch must be >= 1");
  if (sched) {
    rc = schedule_to_packs(h->model, sched, &h->packs);
  } else {
    if (!budget) return fail(HMY_E_INVALID, "neither schedule nor budget given");
    rc = plan_packs(h->model, *budget, n_micro, micro_batch, &h->packs);
  }
  if (rc) return rc;
  rc = resolve(&h->packs, n_micro, micro_batch, &h->sp);
  if (rc) return rc;
  h->M = h->sp.MB();
  h->b = h->sp.uB;
  h->MF = h->sp.MF();
  h->bF = h->sp.uF;
  h->fused_swap_out = h->packs.swap_out == HMY_SWAP_OUT_KERNEL;
  h->arena = arena_layout(h->model, h->packs, h->sp);
  // forward packs must fit a weight slot
  for (const Pack &q : h->packs.fwd)
    if (pack_state_fwd(h->model, q) > h->arena.slot_bytes) return fail(HMY_E_BAD_SCHEDULE, "forward pack over slot");
  if (budget && h->arena.total > budget->hbm_budget_bytes)
    return fail(sched ? HMY_E_BAD_SCHEDULE : HMY_E_BUDGET_TOO_SMALL, "schedule needs %llu B of HBM, budget is %llu B",
                (unsigned long long)h->arena.total, (unsigned long long)budget->hbm_budget_bytes);
  h->bacts = block_acts(h->model.spec, h->b);
  h->bacts_F = block_acts(h->model.spec, h->bF);
  h->hacts = head_acts(h->model.spec, h->b);
  h->ckpt_layers.clear();
  for (size_t k = 1; k + 1 < h->packs.bwd.size(); ++k) h->ckpt_layers.push_back(h->packs.bwd[k].a);
  h->visits.clear();
  auto mk = [&](bool bwd, bool last, Pack p) {
    Visit v;
    v.bwd = bwd;
    v.last = last;
    v.pack = p;
    v.slot = int(h->visits.size() % size_t(h->packs.slots));
    v.poff = h->model.layer_off[p.a];
    v.nparams = h->model.params_in(p.a, p.e);
    v.index = int(h->visits.size());
    h->visits.push_back(v);
  };
  for (const Pack &q : h->packs.fwd) mk(false, false, q);
  for (int k = int(h->packs.bwd.size()) - 1; k >= 0; --k) mk(true, k == int(h->packs.bwd.size()) - 1, h->packs.bwd[k]);
  h->first_chunk.assign(h->visits.size(), -1);
  h->total_chunks = 0;
  const uint64_t c = h->arena.res.k_chunk_params;
  for (size_t vi = 0; vi < h->visits.size(); ++vi) {
    if (!h->visits[vi].bwd) continue;
    h->first_chunk[vi] = h->total_chunks;
    h->total_chunks += int((h->visits[vi].nparams + c - 1) / c);
  }
  return HMY_OK;
}

namespace {
// calls f(resident slot, first element in the host arrays, elements) for every resident chunk
template <typename F> void for_each_resident_chunk(const hmy_handle *h, F f) {
  const uint64_t c = h->arena.res.k_chunk_params;
  const int first_resident = h->total_chunks - h->res_chunks;
  for (size_t vi = 0; vi < h->visits.size(); ++vi) {
    const Visit &v = h->visits[vi];
    if (!v.bwd) continue;
    const int nc = int((v.nparams + c - 1) / c);
    for (int k = 0; k < nc; ++k) {
      const int slot = h->first_chunk[vi] + k - first_resident;
      if (slot < 0) continue;
      const uint64_t lo = uint64_t(k) * c;
      f(slot, v.poff + lo, std::min<uint64_t>(c, v.nparams - lo));
    }
  }
}
}  // namespace

// ---- the Profiler (Section 4.2): each layer on its own, timed on the device -------------
namespace {
// small pseudo-random values (|x| < 0.05) in the element type: kernels whose operands are all zero
// draw less power and run at other clocks than in a real iteration
__global__ void k_fill_pattern(uint32_t *p, uint64_t n_words, int bf16) {
  const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n_words; i += stride) {
    uint32_t x = uint32_t(i) * 2654435761u;
    x ^= x >> 15;
    x *= 2246822519u;
    x ^= x >> 13;
    const float a = (float(x & 0xFFFF) * (1.0f / 65536.0f) - 0.5f) * 0.1f;
    const float b = (float(x >> 16) * (1.0f / 65536.0f) - 0.5f) * 0.1f;
    if (bf16) p[i] = (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xFFFF0000u);
    else p[i] = __float_as_uint(a);
  }
}
}  // namespace

int hmy::run_measure_profile(const Model &m, int micro_batch, int hip_device, int reps, hmy_measured_profile *out) {
  // a short copy of the model in three packs: embedding | up to three blocks | head.  The blocks are timed as one
  // pack and the time divided: run after one another they have weights, gradient sums and activations of their
  // own, as the blocks of a pack in an iteration have, where one block run over and over would find all of these
  // in the memory-side cache (measured on 48 blocks of d = 1600: backward visits 16 % slower in the iteration than
  // that way), and the recompute leaves out the last block's second MLP GEMM once per pack, not once per block
  const int nb = std::min(3, int(m.spec.n_blocks));
  hmy_model_spec s1 = m.spec;
  s1.n_blocks = nb;
  hmy_schedule sc;
  std::memset(&sc, 0, sizeof(sc));
  sc.n_fwd_packs = 2;
  sc.fwd_pack_end[0] = 1; sc.fwd_pack_end[1] = 1 + nb;
  sc.n_bwd_packs = 3;
  sc.bwd_pack_end[0] = 1; sc.bwd_pack_end[1] = 1 + nb; sc.bwd_pack_end[2] = 2 + nb;
  hmy_handle h;
  int rc = init_handle(&h, &s1, &sc, nullptr, 1, micro_batch);
  if (rc) return rc;
  h.ckpt_layers.clear();   // layers run on their own: nothing is stashed
  h.timing = false;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1 || hip_device < 0 || hip_device >= ndev)
    return fail(HMY_E_NO_DEVICE, "no usable HIP device %d (found %d)", hip_device, ndev);
  h.device = hip_device;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  // what runs beside the layers in an iteration: weights and optimizer state arriving (copy engine), results
  // leaving (the update kernel that writes to the host, launched as it is beside the compute stream: how much it
  // slows other kernels goes with the rate it reaches); one staging buffer on each side
  constexpr uint64_t kLoadBytes = 64ull << 20;
  char *load_host = nullptr, *load_dev = nullptr;
  HIPCHK(&h, hipSetDevice(hip_device));
  HIPCHK(&h, hipMalloc(reinterpret_cast<void **>(&h.base), h.arena.total));
  HIPCHK(&h, hipStreamCreateWithFlags(&h.s_comp, hipStreamNonBlocking));
  HIPCHK(&h, hipStreamCreateWithFlags(&h.s_in, hipStreamNonBlocking));
  HIPCHK(&h, hipStreamCreateWithFlags(&h.s_out, hipStreamNonBlocking));
  HIPCHK(&h, hipHostMalloc(reinterpret_cast<void **>(&load_host), 2 * kLoadBytes, hipHostMallocDefault));
  HIPCHK(&h, hipMalloc(reinterpret_cast<void **>(&load_dev), 2 * kLoadBytes));
  HIPCHK(&h, hipEventCreate(&e0));
  HIPCHK(&h, hipEventCreate(&e1));
  if (!h.err) {
    hipLaunchKernelGGL(k_fill_pattern, dim3(2048), dim3(256), 0, h.s_comp, reinterpret_cast<uint32_t *>(h.base),
                       h.arena.total / 4, h.model.spec.precision == HMY_PREC_BF16 ? 1 : 0);
    // token ids and targets must be valid indices: all zero
    KCHK(&h, launch_fill_zero(h.base + h.arena.res.ids, uint64_t(micro_batch) * s1.seq_len * 4, h.s_comp));
    KCHK(&h, launch_fill_zero(h.base + h.arena.res.targets, uint64_t(micro_batch) * s1.seq_len * 4, h.s_comp));
    KCHK(&h, launch_fill_zero(h.base + h.arena.res.misc, 4096, h.s_comp));
    KCHK(&h, launch_fill_zero(load_dev + kLoadBytes, kLoadBytes, h.s_comp));   // the update kernel's inputs: all zero
  }
  // as many parameters per update launch as both staging buffers hold: 16 bytes each in, at most 20 out
  const uint64_t upd_n = (kLoadBytes / 20) & ~uint64_t(255);
  const bool mixed = s1.precision == HMY_PREC_BF16;
  hmy_adam upd_hp;
  upd_hp.lr = 1e-4f; upd_hp.beta1 = 0.9f; upd_hp.beta2 = 0.999f; upd_hp.eps = 1e-8f; upd_hp.step = 1;
  auto update_out = [&]() {
    const float *in = reinterpret_cast<const float *>(load_dev + kLoadBytes);
    float *outp = reinterpret_cast<float *>(load_host + kLoadBytes);
    return launch_adam_out(s1.precision, in, in + upd_n, in + 2 * upd_n, in + 3 * upd_n, mixed ? outp : nullptr,
                           outp + upd_n, outp + 2 * upd_n, outp + 4 * upd_n, outp + 3 * upd_n, upd_n, upd_hp, false, h.s_out);
  };
  IterState it;
  it.inv_ntgt = 1.0f / float(uint64_t(micro_batch) * s1.seq_len);
  auto timed = [&](const Visit &v, uint64_t *beside_ns) -> uint64_t {
    auto once = [&]() {
      if (v.bwd) backward_visit_microbatch(&h, it, v, 0);
      else forward_visit_microbatch(&h, it, v, 0);
      h.sync_used = 0;   // the events a visit records for the swap engine are of no use here: recycle them
    };
    auto run = [&](int n) -> double {
      HIPCHK(&h, hipEventRecord(e0, h.s_comp));
      for (int r = 0; r < n; ++r) once();
      HIPCHK(&h, hipEventRecord(e1, h.s_comp));
      HIPCHK(&h, hipEventSynchronize(e1));
      float ms = 0.f;
      HIPCHK(&h, hipEventElapsedTime(&ms, e0, e1));
      return double(ms);
    };
    once();   // warm-up: code objects, caches, clocks
    const double alone_ms = run(reps) / reps;
    if (!h.err) {
      // enough traffic to last through the timed launches (about 40 GB/s each way beside kernels): incoming copies
      // for every visit, outgoing stores only for backward visits, whose updates are what writes to the host
      const int n_copies = int(std::min(400.0, 2.0 * reps * alone_ms * 1e-3 * 40e9 / double(kLoadBytes))) + 2;
      // (each of these queues holds at most a few hundred operations of 64 MiB)
      for (int c = 0; c < n_copies; ++c) {
        HIPCHK(&h, hipMemcpyAsync(load_dev, load_host, kLoadBytes, hipMemcpyHostToDevice, h.s_in));
        if (v.bwd) KCHK(&h, update_out());
      }
    }
    const double beside_ms = run(reps) / reps;
    hipStreamSynchronize(h.s_in);   // let what is left of the traffic drain before the next layer's turn
    hipStreamSynchronize(h.s_out);
    *beside_ns = uint64_t(std::max(alone_ms, beside_ms) * 1e6 + 0.5);
    return uint64_t(alone_ms * 1e6 + 0.5);
  };
  std::memset(out, 0, sizeof(*out));
  out->micro_batch = micro_batch;
  // visits: forward embedding, forward blocks, last pack (head, forward + backward), blocks (recompute + backward),
  // embedding alone (backward only: its recompute is not needed)
  out->embed_fwd_ns = timed(h.visits[0], &out->embed_fwd_beside_ns);
  out->block_fwd_ns = timed(h.visits[1], &out->block_fwd_beside_ns) / nb;
  out->block_fwd_beside_ns /= nb;
  out->head_ns = timed(h.visits[2], &out->head_beside_ns);
  out->block_bwd_ns = timed(h.visits[3], &out->block_bwd_beside_ns) / nb;
  out->block_bwd_beside_ns /= nb;
  out->embed_bwd_ns = timed(h.visits[4], &out->embed_bwd_beside_ns);
  if (h.s_comp) { hipStreamSynchronize(h.s_comp); hipStreamDestroy(h.s_comp); }
  if (h.s_in) { hipStreamSynchronize(h.s_in); hipStreamDestroy(h.s_in); }
  if (h.s_out) { hipStreamSynchronize(h.s_out); hipStreamDestroy(h.s_out); }
  if (load_host) hipHostFree(load_host);
  if (load_dev) hipFree(load_dev);
  if (e0) hipEventDestroy(e0);
  if (e1) hipEventDestroy(e1);
  for (hipEvent_t e : h.sync_events) hipEventDestroy(e);
  if (h.base) hipFree(h.base);
  return h.err;
}

extern "C" {

int hmy_count_swaps(const hmy_model_spec *spec, const hmy_schedule *sched, int32_t n_micro, int32_t micro_batch,
                    hmy_stats *out) {
  if (!spec || !sched || !out) return fail(HMY_E_INVALID, "null argument");
  hmy_handle h;
  h.dry = true;
  int rc = init_handle(&h, spec, sched, nullptr, n_micro, micro_batch);
  if (rc) return rc;
  hmy_adam hp{};
  run_in_order(&h, nullptr, hp);
  *out = h.st;
  return h.err;
}

int hmy_host_alloc(uint64_t bytes, void **out) {
  if (!out) return fail(HMY_E_INVALID, "null out");
  *out = nullptr;
  hipError_t e = hipHostMalloc(out, bytes ? bytes : 1, hipHostMallocDefault);
  if (e != hipSuccess) {
    // the runtime also remembers the failure as its "last error": taken out here, or the next launch check of a
    // caller who goes on (with less, or with ordinary memory) would report this allocation's failure as its own
    (void)hipGetLastError();
    return fail(HMY_E_HIP, "hipHostMalloc(%llu): %s", (unsigned long long)bytes, hipGetErrorString(e));
  }
  return HMY_OK;
}
int hmy_host_free(void *p) {
  if (!p) return HMY_OK;
  hipError_t e = hipHostFree(p);
  if (e != hipSuccess) return fail(HMY_E_HIP, "hipHostFree: %s", hipGetErrorString(e));
  return HMY_OK;
}

int hmy_create(const hmy_model_spec *spec, const hmy_budget *budget, int32_t n_micro, int32_t micro_batch,
               const hmy_schedule *sched, int32_t hip_device, void *arena, uint64_t arena_bytes, hmy_handle **out) {
  if (!spec || !budget || !out) return fail(HMY_E_INVALID, "null argument");
  *out = nullptr;
  hmy_handle *h = new hmy_handle();
  int rc = init_handle(h, spec, sched, budget, n_micro, micro_batch);
  if (rc) { delete h; return rc; }
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1 || hip_device < 0 || hip_device >= ndev) {
    delete h;
    return fail(HMY_E_NO_DEVICE, "no usable HIP device %d (found %d)", hip_device, ndev);
  }
  h->device = hip_device;
  HIPCHK(h, hipSetDevice(hip_device));
  // what the budget (and a caller's arena) leaves free behind the arena holds optimizer state
  if (h->packs.resident_state == HMY_STATE_RESIDENT_IN_SPARE_BUDGET && h->packs.update_site == HMY_UPDATE_ON_DEVICE) {
    uint64_t room = budget->hbm_budget_bytes > h->arena.total ? budget->hbm_budget_bytes - h->arena.total : 0;
    if (arena) room = std::min(room, arena_bytes > h->arena.total ? arena_bytes - h->arena.total : 0);
    h->res_chunks = int(std::min<uint64_t>(uint64_t(h->total_chunks), room / h->chunk_state_bytes()));
    h->res_off = h->arena.total;
    h->res_loaded.assign(size_t(h->res_chunks), 0);
  }
  if (arena) {
    if (arena_bytes < h->arena.total || (reinterpret_cast<uintptr_t>(arena) & 255)) {
      delete h;
      return fail(HMY_E_INVALID, "arena too small (%llu < %llu) or not 256-byte aligned", (unsigned long long)arena_bytes,
                  (unsigned long long)h->arena.total);
    }
    h->base = static_cast<char *>(arena);
  } else {
    HIPCHK(h, hipMalloc(reinterpret_cast<void **>(&h->base), h->arena.total + uint64_t(h->res_chunks) * h->chunk_state_bytes()));
    h->own_arena = true;
  }
  HIPCHK(h, hipStreamCreateWithFlags(&h->s_comp, hipStreamNonBlocking));
  HIPCHK(h, hipStreamCreateWithFlags(&h->s_in, hipStreamNonBlocking));
  HIPCHK(h, hipStreamCreateWithFlags(&h->s_kin, hipStreamNonBlocking));
  HIPCHK(h, hipStreamCreateWithFlags(&h->s_out, hipStreamNonBlocking));
  // Four streams, not five: a process has 4 hardware queues by default, a fifth stream shares one
  // with another stream, and every event wait queued on it then also holds up that stream's kernels
  // (measured: an engine whose update stream landed on the compute stream's queue ran 30 % slower).
  // The update kernels and the checkpoint writes barely overlap in time, so they share s_out.
  h->s_upd = h->s_out;
  if (h->packs.update_site == HMY_UPDATE_ON_HOST && !h->err) {
    h->updater = new HostUpdater(default_host_threads(), updater_thread_init, updater_wait, h);
  }
  const uint64_t stash_bytes = uint64_t(h->ckpt_layers.size()) * h->M * h->arena.res.x_bytes_B;
  if (stash_bytes) HIPCHK(h, hipHostMalloc(reinterpret_cast<void **>(&h->stash_host), stash_bytes, hipHostMallocDefault));
  if (h->err) {
    int e = h->err;
    hmy_destroy(h);
    return e;
  }
  *out = h;
  return HMY_OK;
}

int hmy_get_schedule(const hmy_handle *h, hmy_schedule *out) {
  if (!h || !out) return fail(HMY_E_INVALID, "null argument");
  packs_to_schedule(h->packs, out);
  return HMY_OK;
}

int hmy_bind_state(hmy_handle *h, const hmy_host_state *state) {
  if (!h || !state) return fail(HMY_E_INVALID, "null argument");
  const bool mixed = h->model.spec.precision == HMY_PREC_BF16;
  if (!state->weights || !state->adam_m || !state->adam_v)
    return fail(HMY_E_INVALID, "weights, adam_m and adam_v must be given");
  // the gradient array is written unless the update consumes the gradient on the device and drops it
  const bool grads_unused = h->packs.gradients == HMY_GRADIENTS_ON_DEVICE && h->packs.update_site == HMY_UPDATE_ON_DEVICE &&
                            h->packs.order == HMY_ORDER_LAYER_PACK_MAJOR;
  if (!state->grads && !grads_unused)
    return fail(HMY_E_INVALID, "grads must be given (only a layer-pack-major schedule with the update on the device "
                               "and HMY_GRADIENTS_ON_DEVICE leaves it unwritten)");
  if (mixed && !state->master) return fail(HMY_E_INVALID, "bf16 precision needs an fp32 master array");
  if (!mixed && state->master) return fail(HMY_E_INVALID, "fp32 precision: master must be NULL (weights are the master)");
  if (state->n_params != h->model.n_params)
    return fail(HMY_E_INVALID, "state has %llu parameters, model has %llu", (unsigned long long)state->n_params,
                (unsigned long long)h->model.n_params);
  h->host = *state;
  h->bound = true;
  std::fill(h->res_loaded.begin(), h->res_loaded.end(), 0);   // resident state is read afresh from these arrays
  return HMY_OK;
}

int hmy_resident_params(const hmy_handle *h, uint64_t *n_params) {
  if (!h || !n_params) return fail(HMY_E_INVALID, "null argument");
  uint64_t total = 0;
  for_each_resident_chunk(h, [&](int, uint64_t, uint64_t n) { total += n; });
  *n_params = total;
  return HMY_OK;
}

int hmy_sync_state(hmy_handle *h) {
  if (!h) return fail(HMY_E_INVALID, "null handle");
  if (!h->res_chunks) return HMY_OK;
  if (!h->bound) return fail(HMY_E_NOT_BOUND, "hmy_bind_state has not been called");
  h->err = HMY_OK;
  HIPCHK(h, hipSetDevice(h->device));
  HIPCHK(h, hipDeviceSynchronize());
  const bool mixed = h->model.spec.precision == HMY_PREC_BF16;
  const uint64_t arr = h->arena.res.karr_bytes;
  for_each_resident_chunk(h, [&](int slot, uint64_t g0, uint64_t n) {
    if (!h->res_loaded[slot]) return;   // never updated since the bind: the arrays are current
    const char *src = h->base + h->res_off + uint64_t(slot) * h->chunk_state_bytes();
    if (mixed) HIPCHK(h, hipMemcpy(h->host.master + g0, src, n * 4, hipMemcpyDeviceToHost));
    HIPCHK(h, hipMemcpy(h->host.adam_m + g0, src + (mixed ? 1 : 0) * arr, n * 4, hipMemcpyDeviceToHost));
    HIPCHK(h, hipMemcpy(h->host.adam_v + g0, src + (mixed ? 2 : 1) * arr, n * 4, hipMemcpyDeviceToHost));
  });
  return h->err;
}

int hmy_iteration(hmy_handle *h, const hmy_minibatch *mb, const hmy_adam *adam, hmy_stats *out) {
  if (!h || !mb || !adam) return fail(HMY_E_INVALID, "null argument");
  if (!h->bound) return fail(HMY_E_NOT_BOUND, "hmy_bind_state has not been called");
  if (int64_t(mb->n_micro) * mb->micro_batch != h->sp.D || mb->n_micro < 1)
    return fail(HMY_E_INVALID, "minibatch is %dx%d sequences, handle was created for %d", mb->n_micro, mb->micro_batch,
                h->sp.D);
  if (!mb->token_ids || !mb->targets) return fail(HMY_E_INVALID, "null token_ids/targets");
  if (adam->step < 1) return fail(HMY_E_INVALID, "adam step is 1-based");
  const hmy_model_spec &s = h->model.spec;
  const uint64_t n = uint64_t(h->M) * h->b * s.seq_len;
  for (uint64_t i = 0; i < n; ++i) {
    if (mb->token_ids[i] < 0 || mb->token_ids[i] >= s.vocab) return fail(HMY_E_INVALID, "token id out of range at %llu", (unsigned long long)i);
    if (mb->targets[i] < -1 || mb->targets[i] >= s.vocab) return fail(HMY_E_INVALID, "target out of range at %llu", (unsigned long long)i);
  }
  h->err = HMY_OK;
  HIPCHK(h, hipSetDevice(h->device));
  h->timing = out != nullptr && h->profile_level >= 1;
  auto t0 = std::chrono::steady_clock::now();
  run_in_order(h, mb, *adam);
  // always drain, even after an error, so no stream still touches caller memory
  hipStreamSynchronize(h->s_comp);
  hipStreamSynchronize(h->s_in);
  hipStreamSynchronize(h->s_kin);
  hipStreamSynchronize(h->s_upd);
  hipError_t e_last = hipStreamSynchronize(h->s_out);
  if (h->err == HMY_OK && e_last != hipSuccess) h->err = fail(HMY_E_HIP, "stream sync: %s", hipGetErrorString(e_last));
  if (h->updater) {   // the CPU threads may still be applying the last pack's update
    const int rc = h->updater->drain();
    if (h->err == HMY_OK && rc != HMY_OK) h->err = fail(rc, "the update on the host failed");
  }
  auto t1 = std::chrono::steady_clock::now();
  if (h->err) return h->err;
  double loss = 0.0;
  // on the compute stream, not the null stream: that one would claim a hardware queue of its own
  HIPCHK(h, hipMemcpyAsync(&loss, h->base + h->arena.res.misc, sizeof(double), hipMemcpyDeviceToHost, h->s_comp));
  HIPCHK(h, hipStreamSynchronize(h->s_comp));
  if (out) {
    h->st.loss = loss;
    h->st.t_iter_s = std::chrono::duration<double>(t1 - t0).count();
    double pair = -1.0;
    for (const auto &sp : h->spans) {
      float ms = 0.f;
      if (sp.what != 20 || hipEventElapsedTime(&ms, h->time_events[sp.a], h->time_events[sp.b]) != hipSuccess) continue;
      if (pair < 0 || ms * 1e-3 < pair) pair = ms * 1e-3;
    }
    h->st.t_event_pair_s = pair > 0 ? pair : 0.0;
    for (const auto &sp : h->spans) {
      float ms = 0.f;
      if (sp.what == 20 || hipEventElapsedTime(&ms, h->time_events[sp.a], h->time_events[sp.b]) != hipSuccess) continue;
      const double sec = ms * 1e-3;
      if (sp.what == 0) h->st.t_h2d_busy_s += sec;
      else if (sp.what == 1) h->st.t_d2h_busy_s += sec;
      else if (sp.what == 2) h->st.t_stall_s += sec;
      else if (sp.what == 3) h->st.t_compute_s += sec;
      else h->st.gemm_s[sp.what - 10] += std::max(0.0, sec - h->st.t_event_pair_s);
    }
    *out = h->st;
    if (const char *path = std::getenv("HMY_TIMELINE")) {
      // one line per timed span: what (0 h2d, 1 d2h/update kernel, 2 compute-stream wait, 3 compute span,
      // 10.. GEMM variants), tag (1000 * visit + microbatch at enqueue), start and end in ms
      // since the first span's start
      if (FILE *f = std::fopen(path, "w")) {
        for (const auto &sp : h->spans) {
          float a = 0.f, b = 0.f;
          if (hipEventElapsedTime(&a, h->time_events[h->spans[0].a], h->time_events[sp.a]) != hipSuccess) continue;
          if (hipEventElapsedTime(&b, h->time_events[h->spans[0].a], h->time_events[sp.b]) != hipSuccess) continue;
          std::fprintf(f, "%d %d %.3f %.3f\n", sp.what, sp.tag, a, b);
        }
        std::fclose(f);
      }
    }
  }
  return h->err;
}

int hmy_set_profiling(hmy_handle *h, int32_t level) {
  if (!h) return fail(HMY_E_INVALID, "null handle");
  if (level < 0 || level > 2) return fail(HMY_E_INVALID, "profiling level %d (0..2)", level);
  h->profile_level = level;
  h->profile_gemm = level >= 2;
  return HMY_OK;
}

int hmy_set_progress(hmy_handle *h, int32_t on) {
  if (!h) return fail(HMY_E_INVALID, "null handle");
  h->progress = on != 0;
  return HMY_OK;
}

int hmy_destroy(hmy_handle *h) {
  if (!h) return HMY_OK;
  delete h->updater;   // joins its threads
  h->updater = nullptr;
  if (!h->dry && h->device >= 0) {
    hipSetDevice(h->device);
    if (h->s_comp) { hipStreamSynchronize(h->s_comp); hipStreamDestroy(h->s_comp); }
    if (h->s_in) { hipStreamSynchronize(h->s_in); hipStreamDestroy(h->s_in); }
    if (h->s_kin) { hipStreamSynchronize(h->s_kin); hipStreamDestroy(h->s_kin); }
    if (h->s_upd && h->s_upd != h->s_out) { hipStreamSynchronize(h->s_upd); hipStreamDestroy(h->s_upd); }
    if (h->s_out) { hipStreamSynchronize(h->s_out); hipStreamDestroy(h->s_out); }
    for (hipEvent_t e : h->sync_events) hipEventDestroy(e);
    for (hipEvent_t e : h->time_events) hipEventDestroy(e);
    if (h->stash_host) hipHostFree(h->stash_host);
    if (h->own_arena && h->base) hipFree(h->base);
  }
  delete h;
  return HMY_OK;
}

}  // extern "C"
