// Model layout: the R layers and their tensors in storage order, plus the
// thread-local error string of the C ABI.
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "hmy_internal.h"

namespace hmy {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

const char *last_error() { return g_err; }

int build_model(const hmy_model_spec *sp, Model *out) {
  if (!sp || !out) return fail(HMY_E_INVALID, "null spec");
  const hmy_model_spec &s = *sp;
  if (s.n_blocks < 1 || s.d_model < 1 || s.n_heads < 1 || s.d_ffn < 1 || s.seq_len < 1 || s.vocab < 2)
    return fail(HMY_E_INVALID, "non-positive model dimension");
  if (s.n_blocks + 2 > HMY_MAX_LAYERS)
    return fail(HMY_E_INVALID, "n_blocks+2 exceeds HMY_MAX_LAYERS=%d", HMY_MAX_LAYERS);
  if (s.d_model % s.n_heads) return fail(HMY_E_INVALID, "d_model %% n_heads != 0");
  const int dh = s.d_model / s.n_heads;
  if (dh != 32 && dh != 64 && dh != 128)
    return fail(HMY_E_INVALID, "head dimension %d not in {32,64,128}", dh);
  if (s.d_model % 8 || s.d_ffn % 8) return fail(HMY_E_INVALID, "d_model and d_ffn must be multiples of 8");
  if (s.precision != HMY_PREC_FP32 && s.precision != HMY_PREC_BF16)
    return fail(HMY_E_INVALID, "unknown precision %d", s.precision);
  if (s.causal != 0 && s.causal != 1) return fail(HMY_E_INVALID, "causal must be 0 or 1");
  if (!(s.ln_eps > 0.f)) return fail(HMY_E_INVALID, "ln_eps must be positive");

  Model m;
  m.spec = s;
  m.R = s.n_blocks + 2;
  uint64_t off = 0;
  auto add = [&](const std::string &name, int layer, int rows, int cols) {
    Tensor t{name, layer, rows, cols, off, uint64_t(rows) * uint64_t(cols)};
    off += t.count;
    m.tensors.push_back(t);
  };
  const int d = s.d_model, f = s.d_ffn;
  for (int l = 0; l < m.R; ++l) {
    m.first_tensor.push_back(int(m.tensors.size()));
    m.layer_off.push_back(off);
    if (l == 0) {
      add("wte", l, s.vocab, d);
      add("wpe", l, s.seq_len, d);
    } else if (l <= s.n_blocks) {
      const std::string p = "h" + std::to_string(l) + ".";
      add(p + "ln1_g", l, d, 1);
      add(p + "ln1_b", l, d, 1);
      add(p + "wqkv", l, 3 * d, d);
      add(p + "bqkv", l, 3 * d, 1);
      add(p + "wo", l, d, d);
      add(p + "bo", l, d, 1);
      add(p + "ln2_g", l, d, 1);
      add(p + "ln2_b", l, d, 1);
      add(p + "w1", l, f, d);
      add(p + "b1", l, f, 1);
      add(p + "w2", l, d, f);
      add(p + "b2", l, d, 1);
    } else {
      add("lnf_g", l, d, 1);
      add("lnf_b", l, d, 1);
      add("wh", l, s.vocab, d);
    }
  }
  m.first_tensor.push_back(int(m.tensors.size()));
  m.layer_off.push_back(off);
  m.n_params = off;
  *out = std::move(m);
  return HMY_OK;
}

}  // namespace hmy
