/*
 * CPU oracle for the Qwen3-style decoder forward pass (prefill + decode).
 *
 * TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may build, load or call this file.  It shares no code with
 * the GPU library and includes none of its headers; the weight-blob format and
 * the config fields are re-declared here.
 *
 * What it is: the plain definition of the computation, one token at a time, in
 * fp64 (weights are widened per element from the blob; every intermediate and
 * every accumulation is a double; sums run in index order).  OpenMP is used
 * only over independent output rows / heads, so results do not depend on the
 * thread count.  No blocking, fusion or reordering.
 *
 * Where it comes from: the paper evaluates the decode stage of Qwen3-0.6B
 * (F32/F16) and Qwen3-1.7B (F16) at batch 1, prompt first and then one token at
 * a time, reporting tokens/s (Section 4, experimental setup; Sections 4.1, 4.2),
 * and it attributes the cost to MatMul micro-kernels over packed weights under a
 * memory-bandwidth wall (Section 3.3.2; Sections 4.1, 4.2).  The paper prints no
 * equations for the model itself.  The forward pass below is therefore the
 * public Qwen3 decoder architecture with the hyper-parameters of the benchmark
 * configurations: RMSNorm (eps inside the square root, plain gain), bias-free
 * projections, per-head RMSNorm on q and k over head_dim with one gain vector
 * shared by all heads, rotary embedding after that norm with half-split pairing
 * (i, i + d/2) and frequency theta^(-2i/d), grouped-query attention with
 * contiguous groups (q head a reads kv head floor(a / G)), softmax scale
 * 1/sqrt(d), SwiGLU silu(gate) * up, residual adds, final RMSNorm, LM head
 * (the embedding matrix when tied) and greedy argmax with the lowest index
 * winning ties.  These conventions are pinned in the CPU tests by a black-box
 * comparison with an independent library model at a tiny shape, and the
 * individual functions by closed forms and brute force.
 *
 * Rounding points (flags, default none).  The 16-bit format of every rounding
 * point is bf16, or IEEE binary16 ("F16", the paper's own 16-bit precision,
 * Section 4, experimental setup) when ORC_ROUND_F16 is also set:
 *   ORC_ROUND_KV      k (after norm and RoPE) and v are rounded to 16 bits, round to
 *                     nearest even, before they enter the cache, and attention
 *                     uses the rounded values.  This mirrors a 16-bit KV cache.
 *   ORC_ROUND_GEMM_IN the input vector of each matmul (the two normed hidden
 *                     states, the attention output, the SwiGLU activation; the
 *                     LM-head input too when ORC_ROUND_HEAD_IN is also set) is
 *                     rounded to bf16 first.  This mirrors bf16 matrix-core
 *                     operands in prefill.
 *   ORC_ROUND_ATTN_QP the rotated query and the un-normalised softmax weights
 *                     exp(s - max) are rounded to bf16 before their products
 *                     (mirrors a matrix-core attention kernel); the softmax
 *                     denominator sums the rounded weights.
 *
 * Canonical blob (little endian, tensors contiguous, matrices row-major
 * [out, in] in the blob dtype, gains always fp32), in this order:
 *   embed [V,H]                              (if has_embed_and_head)
 *   per layer: g_in [H], Wq [Dq,H], Wk [Dkv,H], Wv [Dkv,H], g_q [d], g_k [d],
 *              Wo [H,Dq], g_post [H], Wgate [F,H], Wup [F,H], Wdown [H,F]
 *   g_final [H]                              (if has_embed_and_head)
 *   lm_head [V,H]                            (if has_embed_and_head and untied)
 */
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };
enum { ORC_ROUND_KV = 1, ORC_ROUND_GEMM_IN = 2, ORC_ROUND_ATTN_QP = 4, ORC_ROUND_HEAD_IN = 8,
       ORC_ROUND_F16 = 16 };

struct orc_config {
  uint32_t hidden, n_layers, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  uint32_t has_embed_and_head, tied_lm_head, blob_dtype;
  uint32_t max_batch, max_seq;
  double rms_eps, rope_theta;
};

}  // extern "C"

namespace {

/* A matrix or vector inside the borrowed blob. */
struct Tensor {
  const void *p = nullptr;
  int dtype = ORC_F32;
  double at(size_t i) const {
    if (dtype == ORC_F32) {
      float f;
      std::memcpy(&f, static_cast<const char *>(p) + 4 * i, 4);
      return (double)f;
    }
    uint16_t h;
    std::memcpy(&h, static_cast<const char *>(p) + 2 * i, 2);
    if (dtype == ORC_F16) {
      /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
      const int e = (h >> 10) & 31, f = h & 1023;
      double v;
      if (e == 0) v = std::ldexp((double)f, -24);
      else if (e == 31) v = f ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
      else v = std::ldexp((double)(1024 + f), e - 25);
      return (h & 0x8000) ? -v : v;
    }
    uint32_t b = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &b, 4);
    return (double)f;
  }
};

struct Layer {
  Tensor g_in, wq, wk, wv, g_q, g_k, wo, g_post, wgate, wup, wdown;
};

}  // namespace

struct orc_model {
  orc_config c;
  Tensor embed, g_final, lm_head;
  std::vector<Layer> layers;
  /* cache[layer][slot] holds max_seq rows of Dkv doubles for K and for V */
  std::vector<double> kcache, vcache;
  std::vector<uint32_t> len;
  size_t kv_index(uint32_t layer, uint32_t slot, uint32_t pos) const {
    return (((size_t)layer * c.max_batch + slot) * c.max_seq + pos) * ((size_t)c.n_kv_heads * c.head_dim);
  }
};

extern "C" {

/* ---- scalar helpers -------------------------------------------------- */

/* Nearest bf16 (8 significant bits, fp32 exponent range) of a double, ties to
 * even, returned as a double.  Rounds once, directly from fp64. */
double orc_bf16_round(double v) {
  if (v == 0.0 || !std::isfinite(v)) return v;
  int e;
  (void)std::frexp(std::fabs(v), &e); /* |v| = m * 2^e with m in [0.5, 1) */
  int q = e - 8;                      /* quantum 2^q keeps 8 significant bits */
  if (q < -133) q = -133;             /* bf16 subnormal spacing */
  double r = std::ldexp(std::nearbyint(std::ldexp(std::fabs(v), -q)), q);
  if (r >= std::ldexp(1.0, 128)) r = std::numeric_limits<double>::infinity();
  return v < 0 ? -r : r;
}

/* Same rounding from an fp32 value to the 16 stored bits. */
uint16_t orc_bf16_bits(float f) {
  if (std::isnan(f)) return 0x7fc0;
  const double r = orc_bf16_round((double)f);
  const float g = (float)r; /* exact: bf16 values are fp32 values */
  uint32_t b;
  std::memcpy(&b, &g, 4);
  return (uint16_t)(b >> 16);
}

/* Nearest IEEE binary16 value (11 significant bits, normal exponents -14..15,
 * subnormal spacing 2^-24, largest finite 65504) of a double, ties to even,
 * returned as a double.  Rounds once, directly from fp64. */
double orc_f16_round(double v) {
  if (v == 0.0 || !std::isfinite(v)) return v;
  int e;
  (void)std::frexp(std::fabs(v), &e);
  int q = e - 11;
  if (q < -24) q = -24;
  double r = std::ldexp(std::nearbyint(std::ldexp(std::fabs(v), -q)), q);
  if (r >= 65520.0) r = std::numeric_limits<double>::infinity(); /* 65520 = tie above 65504 -> even = inf */
  return v < 0 ? -r : r;
}

/* The 16 stored bits of the nearest binary16 of an fp32 value. */
uint16_t orc_f16_bits(float f) {
  if (std::isnan(f)) return 0x7e00;
  const double r = orc_f16_round((double)f);
  const uint16_t sgn = std::signbit(f) ? 0x8000 : 0;
  const double a = std::fabs(r);
  if (a == 0.0) return sgn;
  if (std::isinf(a)) return sgn | 0x7c00;
  int e;
  const double m = std::frexp(a, &e); /* a = m * 2^e, m in [0.5, 1) */
  if (e < -13) return sgn | (uint16_t)std::ldexp(a, 24); /* subnormal: multiples of 2^-24 */
  return sgn | (uint16_t)(((e + 14) << 10) | ((int)std::ldexp(m, 11) - 1024));
}

double orc_silu(double z) { return z / (1.0 + std::exp(-z)); }

/* ---- vector building blocks (each is used by the forward pass below) -- */

/* out_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i ; g may be NULL (gain 1). */
void orc_rmsnorm(const double *x, const double *g, uint32_t n, double eps, double *out) {
  double ss = 0.0;
  for (uint32_t j = 0; j < n; ++j) ss += x[j] * x[j];
  const double r = 1.0 / std::sqrt(ss / (double)n + eps);
  for (uint32_t i = 0; i < n; ++i) out[i] = x[i] * r * (g ? g[i] : 1.0);
}

/* Rotary embedding of one head vector u[d] at integer position pos:
 * pairs (i, i + d/2), angle pos * theta^(-2i/d). */
void orc_rope(const double *u, uint32_t d, uint32_t pos, double theta, double *out) {
  const uint32_t half = d / 2;
  for (uint32_t i = 0; i < half; ++i) {
    const double phi = (double)pos * std::pow(theta, -2.0 * (double)i / (double)d);
    const double c = std::cos(phi), s = std::sin(phi);
    const double a = u[i], b = u[i + half];
    out[i] = a * c - b * s;
    out[i + half] = b * c + a * s;
  }
}

/* w_j = exp(s_j - max s) / sum. */
void orc_softmax(const double *s, uint32_t n, double *w) {
  double m = s[0];
  for (uint32_t j = 1; j < n; ++j) m = s[j] > m ? s[j] : m;
  double z = 0.0;
  for (uint32_t j = 0; j < n; ++j) {
    w[j] = std::exp(s[j] - m);
    z += w[j];
  }
  for (uint32_t j = 0; j < n; ++j) w[j] /= z;
}

/* y = W x for a row-major [rows, cols] matrix stored as fp32 or bf16. */
void orc_matvec(const void *w, int dtype, uint32_t rows, uint32_t cols, const double *x, double *y) {
  Tensor t;
  t.p = w;
  t.dtype = dtype;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < (int64_t)rows; ++r) {
    double acc = 0.0;
    const size_t base = (size_t)r * cols;
    for (uint32_t k = 0; k < cols; ++k) acc += t.at(base + k) * x[k];
    y[r] = acc;
  }
}

/* One query against n cached rows: keys/values are [n, stride] with the head's
 * d elements starting at column 0 of the pointers given.
 * s_j = <q, K_j> / sqrt(d); o = sum_j softmax(s)_j V_j.
 * round_p: round exp(s_j - max) to 16 bits before use (see ORC_ROUND_ATTN_QP):
 * 0 = no, 1 = bf16, 2 = binary16. */
void orc_attend(const double *q, const double *keys, const double *vals, uint32_t n, uint32_t d,
                size_t stride, int round_p, double *out) {
  std::vector<double> s(n);
  const double scale = 1.0 / std::sqrt((double)d);
  for (uint32_t j = 0; j < n; ++j) {
    double acc = 0.0;
    for (uint32_t i = 0; i < d; ++i) acc += q[i] * keys[(size_t)j * stride + i];
    s[j] = acc * scale;
  }
  std::vector<double> w(n);
  double z = 1.0;
  if (!round_p) {
    orc_softmax(s.data(), n, w.data());
  } else {
    /* un-normalised weights rounded to 16 bits; the denominator sums what was used */
    double m = s[0];
    for (uint32_t j = 1; j < n; ++j) m = s[j] > m ? s[j] : m;
    z = 0.0;
    for (uint32_t j = 0; j < n; ++j) {
      const double ex = std::exp(s[j] - m);
      w[j] = round_p == 2 ? orc_f16_round(ex) : orc_bf16_round(ex);
      z += w[j];
    }
  }
  for (uint32_t i = 0; i < d; ++i) {
    double acc = 0.0;
    for (uint32_t j = 0; j < n; ++j) acc += w[j] * vals[(size_t)j * stride + i];
    out[i] = acc / z;
  }
}

/* Lowest index of the maximum; -1 if any entry is NaN. */
int32_t orc_argmax(const double *v, uint32_t n) {
  int32_t best = 0;
  for (uint32_t i = 0; i < n; ++i) {
    if (std::isnan(v[i])) return -1;
    if (v[i] > v[best]) best = (int32_t)i;
  }
  return best;
}

/* ---- model ------------------------------------------------------------ */

uint64_t orc_blob_bytes(const orc_config *c) {
  const uint64_t H = c->hidden, d = c->head_dim, Dq = (uint64_t)c->n_q_heads * d,
                 Dkv = (uint64_t)c->n_kv_heads * d, F = c->ffn, V = c->vocab;
  const uint64_t w = c->blob_dtype == ORC_F32 ? 4 : 2;
  uint64_t per_layer = w * (Dq * H + 2 * Dkv * H + H * Dq + 2 * F * H + H * F) + 4 * (2 * H + 2 * d);
  uint64_t total = per_layer * c->n_layers;
  if (c->has_embed_and_head) {
    total += w * V * H + 4 * H;
    if (!c->tied_lm_head) total += w * V * H;
  }
  return total;
}

orc_model *orc_create(const orc_config *c, const void *blob, uint64_t blob_bytes) {
  if (!c || !blob || blob_bytes != orc_blob_bytes(c)) return nullptr;
  if (c->n_kv_heads == 0 || c->n_q_heads % c->n_kv_heads || c->head_dim % 2) return nullptr;
  orc_model *m = new (std::nothrow) orc_model;
  if (!m) return nullptr;
  m->c = *c;
  const size_t H = c->hidden, d = c->head_dim, Dq = (size_t)c->n_q_heads * d,
               Dkv = (size_t)c->n_kv_heads * d, F = c->ffn, V = c->vocab;
  const size_t w = c->blob_dtype == ORC_F32 ? 4 : 2;
  const char *p = static_cast<const char *>(blob);
  auto mat = [&](size_t n) { Tensor t; t.p = p; t.dtype = (int)c->blob_dtype; p += w * n; return t; };
  auto gain = [&](size_t n) { Tensor t; t.p = p; t.dtype = ORC_F32; p += 4 * n; return t; };
  if (c->has_embed_and_head) m->embed = mat(V * H);
  m->layers.resize(c->n_layers);
  for (auto &L : m->layers) {
    L.g_in = gain(H);
    L.wq = mat(Dq * H);
    L.wk = mat(Dkv * H);
    L.wv = mat(Dkv * H);
    L.g_q = gain(d);
    L.g_k = gain(d);
    L.wo = mat(H * Dq);
    L.g_post = gain(H);
    L.wgate = mat(F * H);
    L.wup = mat(F * H);
    L.wdown = mat(H * F);
  }
  if (c->has_embed_and_head) {
    m->g_final = gain(H);
    m->lm_head = c->tied_lm_head ? m->embed : mat(V * H);
  }
  const size_t kv = (size_t)c->n_layers * c->max_batch * c->max_seq * Dkv;
  m->kcache.assign(kv, 0.0);
  m->vcache.assign(kv, 0.0);
  m->len.assign(c->max_batch, 0);
  return m;
}

void orc_destroy(orc_model *m) { delete m; }

void orc_kv_reset(orc_model *m, int32_t slot) {
  if (slot < 0) {
    for (auto &l : m->len) l = 0;
  } else if ((uint32_t)slot < m->c.max_batch) {
    m->len[slot] = 0;
  }
}

uint32_t orc_slot_len(const orc_model *m, uint32_t slot) { return m->len[slot]; }

/* Cached rows of one layer and slot: [max_seq, Dkv] doubles. which: 0 = K, 1 = V. */
const double *orc_kv_rows(const orc_model *m, uint32_t layer, uint32_t slot, int which) {
  return (which ? m->vcache.data() : m->kcache.data()) + m->kv_index(layer, slot, 0);
}

}  // extern "C"

namespace {

void gains(const Tensor &t, size_t n, std::vector<double> &g) {
  g.resize(n);
  for (size_t i = 0; i < n; ++i) g[i] = t.at(i);
}

void maybe_round(std::vector<double> &v, bool on, bool f16) {
  if (on)
    for (auto &e : v) e = f16 ? orc_f16_round(e) : orc_bf16_round(e);
}

/* One decoder layer for the token at position pos of `slot`; x is updated in place. */
void layer_forward(orc_model *m, uint32_t li, uint32_t slot, uint32_t pos, uint32_t flags,
                   std::vector<double> &x) {
  const orc_config &c = m->c;
  const Layer &L = m->layers[li];
  const uint32_t H = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads,
                 Dq = nq * d, Dkv = nkv * d, F = c.ffn, G = nq / nkv;
  const bool rin = flags & ORC_ROUND_GEMM_IN, rkv = flags & ORC_ROUND_KV, rqp = flags & ORC_ROUND_ATTN_QP,
             f16 = flags & ORC_ROUND_F16;
  std::vector<double> g, h(H), q(Dq), k(Dkv), v(Dkv), tmp(d), o(Dq), y(H);

  /* input norm, then q, k, v projections */
  gains(L.g_in, H, g);
  orc_rmsnorm(x.data(), g.data(), H, c.rms_eps, h.data());
  maybe_round(h, rin, f16);
  orc_matvec(L.wq.p, L.wq.dtype, Dq, H, h.data(), q.data());
  orc_matvec(L.wk.p, L.wk.dtype, Dkv, H, h.data(), k.data());
  orc_matvec(L.wv.p, L.wv.dtype, Dkv, H, h.data(), v.data());

  /* per-head norm on q and k (shared gain per layer), then rotary embedding */
  gains(L.g_q, d, g);
  for (uint32_t a = 0; a < nq; ++a) {
    orc_rmsnorm(&q[a * d], g.data(), d, c.rms_eps, tmp.data());
    orc_rope(tmp.data(), d, pos, c.rope_theta, &q[a * d]);
  }
  gains(L.g_k, d, g);
  for (uint32_t b = 0; b < nkv; ++b) {
    orc_rmsnorm(&k[b * d], g.data(), d, c.rms_eps, tmp.data());
    orc_rope(tmp.data(), d, pos, c.rope_theta, &k[b * d]);
  }
  maybe_round(k, rkv, f16);
  maybe_round(v, rkv, f16);
  maybe_round(q, rqp, f16);

  /* append to the cache at position pos */
  double *kc = m->kcache.data() + m->kv_index(li, slot, 0);
  double *vc = m->vcache.data() + m->kv_index(li, slot, 0);
  std::memcpy(kc + (size_t)pos * Dkv, k.data(), sizeof(double) * Dkv);
  std::memcpy(vc + (size_t)pos * Dkv, v.data(), sizeof(double) * Dkv);

  /* attention over positions 0..pos; q head a reads kv head a / G */
#pragma omp parallel for schedule(static)
  for (int64_t a = 0; a < (int64_t)nq; ++a) {
    const uint32_t b = (uint32_t)a / G;
    orc_attend(&q[a * d], kc + b * d, vc + b * d, pos + 1, d, Dkv, rqp ? (f16 ? 2 : 1) : 0, &o[a * d]);
  }

  /* output projection + residual */
  maybe_round(o, rin, f16);
  orc_matvec(L.wo.p, L.wo.dtype, H, Dq, o.data(), y.data());
  for (uint32_t i = 0; i < H; ++i) x[i] += y[i];

  /* post-attention norm, SwiGLU feed-forward, residual */
  gains(L.g_post, H, g);
  orc_rmsnorm(x.data(), g.data(), H, c.rms_eps, h.data());
  maybe_round(h, rin, f16);
  std::vector<double> gate(F), up(F), act(F);
  orc_matvec(L.wgate.p, L.wgate.dtype, F, H, h.data(), gate.data());
  orc_matvec(L.wup.p, L.wup.dtype, F, H, h.data(), up.data());
  for (uint32_t i = 0; i < F; ++i) act[i] = orc_silu(gate[i]) * up[i];
  maybe_round(act, rin, f16);
  orc_matvec(L.wdown.p, L.wdown.dtype, H, F, act.data(), y.data());
  for (uint32_t i = 0; i < H; ++i) x[i] += y[i];
}

int run_layers(orc_model *m, uint32_t slot, uint32_t flags, std::vector<double> &x) {
  const uint32_t pos = m->len[slot];
  if (pos >= m->c.max_seq) return 5;
  for (uint32_t li = 0; li < m->c.n_layers; ++li) layer_forward(m, li, slot, pos, flags, x);
  m->len[slot] = pos + 1;
  return 0;
}

}  // namespace

extern "C" {

/* One token through the whole model at the slot's next position.
 * logits_out (V doubles) and next_out may be NULL; with both NULL the final norm
 * and LM head are skipped (prefill positions before the last). Returns 0 on success. */
int orc_step_token(orc_model *m, uint32_t slot, int32_t token, uint32_t flags, double *logits_out,
                   int32_t *next_out) {
  const orc_config &c = m->c;
  if (!c.has_embed_and_head || slot >= c.max_batch || token < 0 || (uint32_t)token >= c.vocab) return 1;
  const uint32_t H = c.hidden, V = c.vocab;
  std::vector<double> x(H);
  for (uint32_t i = 0; i < H; ++i) x[i] = m->embed.at((size_t)token * H + i);
  if (int rc = run_layers(m, slot, flags, x)) return rc;
  if (!logits_out && !next_out) return 0;
  std::vector<double> g, xn(H), logits;
  gains(m->g_final, H, g);
  orc_rmsnorm(x.data(), g.data(), H, c.rms_eps, xn.data());
  maybe_round(xn, (flags & ORC_ROUND_GEMM_IN) && (flags & ORC_ROUND_HEAD_IN), flags & ORC_ROUND_F16);
  double *lp = logits_out;
  if (!lp) {
    logits.resize(V);
    lp = logits.data();
  }
  orc_matvec(m->lm_head.p, m->lm_head.dtype, V, H, xn.data(), lp);
  if (next_out) *next_out = orc_argmax(lp, V);
  return 0;
}

/* n tokens in order; logits (and argmax) of the last position only. */
int orc_prefill(orc_model *m, uint32_t slot, const int32_t *tokens, uint32_t n, uint32_t flags,
                double *logits_out, int32_t *next_out) {
  for (uint32_t t = 0; t < n; ++t) {
    const bool last = t + 1 == n;
    if (int rc = orc_step_token(m, slot, tokens[t], flags, last ? logits_out : nullptr,
                                last ? next_out : nullptr))
      return rc;
  }
  return 0;
}

/* Hidden-state in, hidden-state out (models without embedding and LM head). */
int orc_step_hidden(orc_model *m, uint32_t slot, const double *x_in, uint32_t flags, double *y_out) {
  if (slot >= m->c.max_batch) return 1;
  std::vector<double> x(x_in, x_in + m->c.hidden);
  if (int rc = run_layers(m, slot, flags, x)) return rc;
  std::memcpy(y_out, x.data(), sizeof(double) * m->c.hidden);
  return 0;
}

void orc_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int orc_get_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

}  // extern "C"
