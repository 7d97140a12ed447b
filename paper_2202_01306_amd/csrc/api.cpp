// C ABI: host-only entry points and the single-kernel entry points.  The engine's
// own entry points (create / bind / iteration / destroy / count_swaps) live next
// to the executor.
#include <cstring>

#include "hmy_internal.h"

namespace hmy {
const char *last_error();
}
using namespace hmy;

extern "C" {

const char *hmy_strerror(int err) {
  switch (err) {
    case HMY_OK: return "ok";
    case HMY_E_INVALID: return "invalid argument";
    case HMY_E_BUDGET_TOO_SMALL: return "HBM budget too small for any packing";
    case HMY_E_BAD_SCHEDULE: return "bad schedule";
    case HMY_E_HIP: return "HIP runtime error";
    case HMY_E_NOT_BOUND: return "host state not bound";
    case HMY_E_NO_DEVICE: return "no usable GPU";
    default: return "unknown error";
  }
}

const char *hmy_last_error(void) { return hmy::last_error(); }

int hmy_model_size(const hmy_model_spec *spec, int32_t *n_layers, uint64_t *n_params) {
  Model m;
  int rc = build_model(spec, &m);
  if (rc) return rc;
  if (n_layers) *n_layers = m.R;
  if (n_params) *n_params = m.n_params;
  return HMY_OK;
}

int hmy_layout(const hmy_model_spec *spec, hmy_tensor_desc *out, int32_t cap, int32_t *n) {
  if (!n) return fail(HMY_E_INVALID, "null n");
  Model m;
  int rc = build_model(spec, &m);
  if (rc) return rc;
  *n = int32_t(m.tensors.size());
  if (!out) return HMY_OK;
  if (cap < *n) return fail(HMY_E_INVALID, "layout: capacity %d < %d tensors", cap, *n);
  for (size_t i = 0; i < m.tensors.size(); ++i) {
    const Tensor &t = m.tensors[i];
    std::memset(&out[i], 0, sizeof(out[i]));
    std::strncpy(out[i].name, t.name.c_str(), HMY_NAME_LEN - 1);
    out[i].layer = t.layer;
    out[i].rows = t.rows;
    out[i].cols = t.cols;
    out[i].offset = t.offset;
    out[i].count = t.count;
  }
  return HMY_OK;
}

int hmy_profile(const hmy_model_spec *spec, const hmy_budget *budget, const hmy_schedule *sched, int32_t n_micro,
                int32_t micro_batch, hmy_layer_profile *out, uint64_t *reserved_bytes) {
  Model m;
  int rc = build_model(spec, &m);
  if (rc) return rc;
  Packs p;   // only the microbatch sizes and the slot count matter here
  if (sched) {
    if (sched->weight_slots < 0 || sched->fwd_micro_batch < 0 || sched->bwd_micro_batch < 0)
      return fail(HMY_E_BAD_SCHEDULE, "negative slot count or microbatch size");
    p.slots = sched->weight_slots;
    p.uF = sched->fwd_micro_batch;
    p.uB = sched->bwd_micro_batch;
  }
  Split sp;
  rc = resolve(&p, n_micro, micro_batch, &sp);
  if (rc) return rc;
  if (out) {
    std::vector<hmy_layer_profile> prof;
    layer_profile(m, rates_of(budget), sp, p.slots, &prof);
    for (int l = 0; l < m.R; ++l) out[l] = prof[l];
  }
  if (reserved_bytes) *reserved_bytes = reserved_layout(m, sp).size;
  return HMY_OK;
}

int hmy_plan(const hmy_model_spec *spec, const hmy_budget *budget, int32_t n_micro, int32_t micro_batch,
             hmy_schedule *out) {
  if (!budget || !out) return fail(HMY_E_INVALID, "null argument");
  Model m;
  int rc = build_model(spec, &m);
  if (rc) return rc;
  Packs p;
  rc = plan_packs(m, *budget, n_micro, micro_batch, &p);
  if (rc) return rc;
  packs_to_schedule(p, out);
  return HMY_OK;
}

int hmy_estimate(const hmy_model_spec *spec, const hmy_schedule *sched, const hmy_budget *budget, int32_t n_micro,
                 int32_t micro_batch, uint64_t *iteration_ns) {
  if (!budget || !iteration_ns) return fail(HMY_E_INVALID, "null argument");
  Model m;
  int rc = build_model(spec, &m);
  if (rc) return rc;
  Packs p;
  rc = schedule_to_packs(m, sched, &p);
  if (rc) return rc;
  Split sp;
  rc = resolve(&p, n_micro, micro_batch, &sp);
  if (rc) return rc;
  const Rates r = rates_of(budget);
  std::vector<hmy_layer_profile> prof;
  layer_profile(m, r, sp, p.slots, &prof);
  *iteration_ns = estimate_iteration_ns(m, prof, p, sp, r.link_MBps);
  return HMY_OK;
}

// schedule -> resolved packs, split and arena, with the checks every consumer of an arena wants
static int arena_of(const hmy_model_spec *spec, const hmy_schedule *sched, int n_micro, int micro_batch, Model *m,
                    Packs *p, Split *sp, Arena *a) {
  int rc = build_model(spec, m);
  if (rc) return rc;
  rc = schedule_to_packs(*m, sched, p);
  if (rc) return rc;
  rc = resolve(p, n_micro, micro_batch, sp);
  if (rc) return rc;
  *a = arena_layout(*m, *p, *sp);
  for (const Pack &q : p->fwd)
    if (pack_state_fwd(*m, q) > a->slot_bytes) return fail(HMY_E_BAD_SCHEDULE, "forward pack over slot");
  return HMY_OK;
}

int hmy_arena(const hmy_model_spec *spec, const hmy_schedule *sched, int32_t n_micro, int32_t micro_batch,
              hmy_arena_plan *out) {
  if (!out) return fail(HMY_E_INVALID, "null argument");
  Model m;
  Packs p;
  Split sp;
  Arena a;
  int rc = arena_of(spec, sched, n_micro, micro_batch, &m, &p, &sp, &a);
  if (rc) return rc;
  out->total = a.total;
  out->reserved = a.res.size;
  out->slot_bytes = a.slot_bytes;
  out->act_bytes = a.act_bytes;
  out->k_chunk_params = a.res.k_chunk_params;
  out->weight_slots = p.slots;
  out->prefetch_distance = p.distance;
  out->fwd_micro_batch = p.uF;
  out->bwd_micro_batch = p.uB;
  return HMY_OK;
}

int hmy_arena_regions(const hmy_model_spec *spec, const hmy_schedule *sched, int32_t n_micro, int32_t micro_batch,
                      hmy_region *out, int32_t cap, int32_t *n) {
  if (!n) return fail(HMY_E_INVALID, "null n");
  Model m;
  Packs p;
  Split sp;
  Arena a;
  int rc = arena_of(spec, sched, n_micro, micro_batch, &m, &p, &sp, &a);
  if (rc) return rc;
  const std::vector<Region> regs = arena_regions(m, a, sp);
  *n = int32_t(regs.size());
  if (!out) return HMY_OK;
  if (cap < *n) return fail(HMY_E_INVALID, "arena_regions: capacity %d < %d regions", cap, *n);
  for (size_t i = 0; i < regs.size(); ++i) {
    std::memset(&out[i], 0, sizeof(out[i]));
    std::strncpy(out[i].name, regs[i].name.c_str(), HMY_NAME_LEN - 1);
    out[i].offset = regs[i].offset;
    out[i].bytes = regs[i].bytes;
  }
  return HMY_OK;
}

int hmy_measure_profile(const hmy_model_spec *spec, int32_t micro_batch, int32_t hip_device, int32_t reps,
                        hmy_measured_profile *out) {
  if (!out) return fail(HMY_E_INVALID, "null argument");
  if (micro_batch < 1 || reps < 1 || reps > 1000) return fail(HMY_E_INVALID, "micro_batch >= 1, reps in 1..1000");
  Model m;
  int rc = build_model(spec, &m);
  if (rc) return rc;
  return run_measure_profile(m, micro_batch, hip_device, reps, out);
}

int hmy_set_kernel_path(int32_t use_mfma) {
  g_use_mfma = use_mfma < 0 ? 0 : (use_mfma > 3 ? 1 : use_mfma);
  return HMY_OK;
}

// ---- single kernels ----------------------------------------------------------------
#define NOTNULL(p) \
  if (!(p)) return fail(HMY_E_INVALID, "%s: null pointer %s", __func__, #p)

int hmy_k_embed_fwd(int32_t prec, const int32_t *ids, const void *wte, const void *wpe, float *x, int32_t T, int32_t d,
                    int32_t s, int32_t vocab, void *stream) {
  NOTNULL(ids); NOTNULL(wte); NOTNULL(wpe); NOTNULL(x);
  return launch_embed_fwd(prec, ids, wte, wpe, x, T, d, s, vocab, stream);
}
int hmy_k_embed_bwd(int32_t prec, const int32_t *ids, const float *dx, float *dwte, float *dwpe, int32_t T, int32_t d,
                    int32_t s, int32_t vocab, void *stream) {
  NOTNULL(ids); NOTNULL(dx); NOTNULL(dwte); NOTNULL(dwpe);
  return launch_embed_bwd(prec, ids, dx, dwte, dwpe, T, d, s, vocab, stream);
}
int hmy_k_layernorm_fwd(int32_t prec, const float *x, const void *gamma, const void *beta, void *y, float *mean,
                        float *rstd, int32_t T, int32_t d, float eps, void *stream) {
  NOTNULL(x); NOTNULL(gamma); NOTNULL(beta); NOTNULL(y); NOTNULL(mean); NOTNULL(rstd);
  return launch_layernorm_fwd(prec, x, gamma, beta, y, mean, rstd, T, d, eps, stream);
}
int hmy_k_layernorm_bwd(int32_t prec, const void *dy, const float *x, const float *mean, const float *rstd,
                        const void *gamma, const float *res, float *dx, void *dx_e, float *dgamma, float *dbeta,
                        float *dres_sum, int32_t T, int32_t d, void *stream, float *workspace, uint64_t workspace_bytes) {
  NOTNULL(dy); NOTNULL(x); NOTNULL(mean); NOTNULL(rstd); NOTNULL(gamma); NOTNULL(dx); NOTNULL(dgamma); NOTNULL(dbeta);
  return launch_layernorm_bwd(prec, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres_sum, T, d, stream,
                              workspace, workspace_bytes);
}
int hmy_k_layernorm_bwd_static(int32_t prec, const void *dy, const float *x, const float *mean, const float *rstd,
                               const void *gamma, const float *res, float *dx, void *dx_e, float *dgamma, float *dbeta,
                               int32_t T, int32_t d, void *stream) {
  NOTNULL(dy); NOTNULL(x); NOTNULL(mean); NOTNULL(rstd); NOTNULL(gamma); NOTNULL(dx); NOTNULL(dgamma); NOTNULL(dbeta);
  return launch_layernorm_bwd_static(prec, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, T, d, stream);
}
int hmy_k_gelu_fwd(int32_t prec, const void *u, void *g, uint64_t n, void *stream) {
  NOTNULL(u); NOTNULL(g);
  return launch_gelu_fwd(prec, u, g, n, stream);
}
int hmy_k_gelu_bwd(int32_t prec, const void *dg, const void *u, void *du, uint64_t n, void *stream) {
  NOTNULL(dg); NOTNULL(u); NOTNULL(du);
  return launch_gelu_bwd(prec, dg, u, du, n, stream);
}
int hmy_k_gelu_bwd_colsum(int32_t prec, const void *dg, const void *u, void *du, float *db, int32_t T, int32_t N,
                          void *stream) {
  NOTNULL(dg); NOTNULL(u); NOTNULL(du); NOTNULL(db);
  return launch_gelu_bwd_colsum(prec, dg, u, du, db, T, N, stream);
}
int hmy_k_colsum(int32_t prec, const void *a, float *out, int32_t T, int32_t N, void *stream) {
  NOTNULL(a); NOTNULL(out);
  return launch_colsum(prec, a, out, T, N, stream);
}
int hmy_k_gemm(const hmy_gemm_desc *g, void *stream) {
  NOTNULL(g);
  return launch_gemm(*g, stream);
}
int hmy_k_attn_fwd(int32_t prec, const void *qkv, void *o, float *lse, int32_t b, int32_t s, int32_t H, int32_t dh,
                   int32_t causal, void *stream) {
  NOTNULL(qkv); NOTNULL(o); NOTNULL(lse);
  return launch_attn_fwd(prec, qkv, o, lse, b, s, H, dh, causal, stream);
}
int hmy_k_attn_bwd(int32_t prec, const void *qkv, const void *o, const void *d_o, const float *lse, float *delta,
                   void *dqkv, float *dbias, int32_t b, int32_t s, int32_t H, int32_t dh, int32_t causal, void *stream) {
  NOTNULL(qkv); NOTNULL(o); NOTNULL(d_o); NOTNULL(lse); NOTNULL(delta); NOTNULL(dqkv);
  return launch_attn_bwd(prec, qkv, o, d_o, lse, delta, dqkv, dbias, b, s, H, dh, causal, stream);
}
int hmy_k_xent(int32_t prec, const float *logits, const int32_t *targets, double *loss_acc, void *dlogits, int32_t T,
               int32_t V, int64_t ldl, float inv_ntgt, void *stream) {
  NOTNULL(logits); NOTNULL(targets); NOTNULL(loss_acc); NOTNULL(dlogits);
  return launch_xent(prec, logits, targets, loss_acc, dlogits, T, V, ldl, inv_ntgt, stream);
}
int hmy_k_adam(int32_t prec, const float *grad, float *master, float *m, float *v, void *w_out, uint64_t n,
               const hmy_adam *hp, void *stream) {
  NOTNULL(grad); NOTNULL(m); NOTNULL(v); NOTNULL(w_out); NOTNULL(hp);
  return launch_adam(prec, grad, master, m, v, w_out, n, *hp, stream);
}

int hmy_host_adam(int32_t prec, const float *grad, float *master, float *m, float *v, void *weights, uint64_t n,
                  const hmy_adam *hp, int32_t threads) {
  if (!grad || !m || !v || !weights || !hp) return fail(HMY_E_INVALID, "null argument");
  if (prec != HMY_PREC_FP32 && prec != HMY_PREC_BF16) return fail(HMY_E_INVALID, "unknown precision %d", prec);
  if (prec == HMY_PREC_BF16 && !master) return fail(HMY_E_INVALID, "adam(bf16): master required");
  if (prec == HMY_PREC_FP32 && master) return fail(HMY_E_INVALID, "adam(fp32): master must be NULL");
  if (hp->step < 1) return fail(HMY_E_INVALID, "adam: step is 1-based");
  if (threads < 0 || threads > 256) return fail(HMY_E_INVALID, "threads out of range");
  if (!n) return HMY_OK;
  HostUpdater up(threads ? threads : default_host_threads(), nullptr, nullptr, nullptr);
  up.submit(make_host_adam_job(nullptr, grad, master, m, v, weights, n, *hp));
  return up.drain();
}

}  // extern "C"
