// Host side of the C ABI declared in include/nnc.h: validation, one-time weight
// upload + repack, the fixed per-layer kernel sequence of one forward pass, graph
// capture of decode steps, per-kernel event timing.
//
// One "pass" pushes up to MAX_COLS activation columns through every layer.  A
// decode step is a pass whose columns are different KV slots; a prompt chunk is a
// pass whose columns are consecutive positions of one slot (the attention kernel
// takes each column's own position from device memory, so causal masking needs no
// special case).  The paper's run loop is the same: prompt first, then one token
// at a time, timed over the decoding stage (Section 4, experimental setup).
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <new>
#include <string>
#include <tuple>
#include <vector>

#include "../../include/nnc.h"
#include "nnc_internal.h"
#include "nnc_plan.h"

using namespace nnc;

namespace {

thread_local char g_err[512] = "";

nnc_status fail(nnc_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return st;
}

struct LayerW {
  float *g_in = nullptr, *g_q = nullptr, *g_k = nullptr, *g_post = nullptr;
  void *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wd = nullptr;
  // weight-only 8-bit models: per-row scales in packed row order (else NULL)
  float *sqkv = nullptr, *so = nullptr, *sgu = nullptr, *sd = nullptr;
  void *kc = nullptr, *vc = nullptr;
};

struct ProfRec {
  int fam;
  double bytes, flops;
  hipEvent_t e0, e1;
};

// One family per kernel; the skinny GEMM is split by the matrix it streams (same kernel, very
// different sizes), the reader adds what it wants.
enum Family { FAM_GEMM = 0, FAM_NORM, FAM_QKROPE, FAM_ATTN, FAM_COMBINE, FAM_EMBED, FAM_ARGMAX, FAM_MISC, FAM_PGEMM, FAM_PATTN,
              FAM_GEMM_O, FAM_GEMM_GU, FAM_GEMM_D, FAM_GEMM_HEAD, FAM_PGEMM_O, FAM_PGEMM_GU, FAM_PGEMM_D, FAM_COUNT };
const char* const kFamName[FAM_COUNT] = {"gemm_skinny.qkv", "rmsnorm_pack", "qknorm_rope_append", "attn_partial",
                                         "attn_combine", "embed", "argmax", "misc", "gemm_prefill.qkv", "attn_prefill",
                                         "gemm_skinny.o", "gemm_skinny.gate_up", "gemm_skinny.down", "gemm_skinny.lm_head",
                                         "gemm_prefill.o", "gemm_prefill.gate_up", "gemm_prefill.down"};

}  // namespace

struct nnc_model {
  nnc_config c{};
  bool f32 = false;
  int dt = 1;  // element type of weights and cache: 0 fp32, 1 bf16, 2 binary16 (nnc_dtype)
  int device = 0;
  hipStream_t stream = nullptr;
  nnc_device hooks{};
  bool use_hooks = false;
  std::vector<void*> allocs;

  void* embed = nullptr;
  void* lm_head = nullptr;
  float* g_final = nullptr;
  std::vector<LayerW> L;
  float2* rope = nullptr;

  ColState* st = nullptr;
  float* x = nullptr;        // [MAX_COLS][H] residual stream
  float* qkv = nullptr;      // [MAX_QKV_SLICES][MAX_COLS][Dq + 2 Dkv] (k-slice partial sums in fused decode passes)
  void* Xp = nullptr;        // packed operand, K = H
  void* Ap = nullptr;        // packed operand, K = max(Dq, F)
  float* rpart = nullptr;    // [MAX_KSPLIT][MAX_COLS][H] k-slice partials of the O / down projections
  float* partial = nullptr;  // attention partials
  void* qsplit = nullptr;    // [MAX_COLS][nq][3][128] bf16 pieces of the rotated queries (bf16 models)
  int max_chunks = 0;
  float* logits = nullptr;   // [32][V] when the caller passes no logits buffer
  float* am_val = nullptr;
  int32_t* am_idx = nullptr;
  int32_t* next = nullptr;   // [MAX_COLS]
  int32_t* token_log = nullptr;
  uint32_t token_log_steps = 0;

  std::vector<uint32_t> len;

  // prompt pass on large token blocks
  uint32_t pb_max = 0;         // tokens per block the buffers hold (multiple of 128), 0 if unavailable
  uint32_t opt_prefill_block = 0;  // tokens per block asked for (0: pb_max)
  float *pb_x = nullptr, *pb_qkv = nullptr;
  float* pb_part = nullptr;                 // k-slice partial sums of short blocks' O / down projections
  void *pb_fa = nullptr, *pb_fb = nullptr;  // fragment-order bf16 operands: K = H, K = max(Dq, F)
  void* pb_w = nullptr;  // byte-weight models: the matrix of the next prompt GEMM, widened to bf16 tiles
  int32_t* pb_tok = nullptr;
  void* pb_vt = nullptr;  // transposed V copy of the slot being prefilled
  uint32_t pb_vt_stride = 0;

  // resident decode kernel
  bool mk_ok = false;
  int n_cus = 256;
  int mk_nwg = 0, mk_ks_o = 1, mk_ks_d = 1;
  unsigned mk_tag = 1;  // next unused exchange tag
  void* mk_layers = nullptr;
  unsigned* mk_error = nullptr;
  unsigned* mk_error_host = nullptr;   // pinned copy of the flag, refreshed after every resident launch
  hipEvent_t mk_error_event = nullptr;  // recorded after that refresh
  bool mk_error_pending = false, mk_failed = false;
  unsigned mk_spin_limit = 0;
  void *mk_xq = nullptr, *mk_xatt = nullptr, *mk_xo = nullptr, *mk_xop = nullptr, *mk_xact = nullptr, *mk_xdp = nullptr,
       *mk_xamv = nullptr, *mk_xami = nullptr;
  unsigned long long* mk_trace = nullptr;
  int mk_trace_step = -1;

  bool opt_graph = true;
  int opt_decode_pieces = 0;  // 0: three pieces; 2 / 3: forced for batches of two or more
  int opt_prefill_exact = 0;  // 0: large blocks, pieces by length; 1: 21-token chunks, three pieces; 2: large blocks, two pieces
  bool opt_fuse_qk = true;    // decode passes: QK-norm / RoPE / append inside the attention kernel
  int opt_prefill_attn = -1;  // forced launch shape of the prompt attention, -1 = by size
  int opt_prefill_tile = -1;  // forced block tile of the large-block prompt GEMMs, -1 = by size
  int opt_prefill_kslices = 0;  // with a forced tile: forced k slices of the residual projections, 0 = by rule
  bool opt_persistent = true;
  bool opt_fuse_norm = false;  // decode passes: the norm after an O / down projection runs in that GEMM's tail (measured: no faster)
  uint32_t* tail_counters = nullptr;  // one per GEMM launch with a norm tail in a pass (2 per layer), zeroed per pass
  bool opt_planner = true;    // tile sizes from the analytic model (nnc_plan.h); false: the earlier hand rules
  std::map<std::tuple<int, int, int>, hipGraphExec_t> graphs;

  bool profiling = false;
  // Long prompts: the fp32-grade tail pass runs on a second stream, one layer behind the last
  // block (whose layers record layer_done after their cache append); created on first use.
  bool opt_tail_overlap = true;
  hipStream_t tail_stream = nullptr;
  std::vector<hipEvent_t> layer_done;   // one per layer, + [n_layers]: fork point, + [n_layers + 1]: join
  bool record_layers = false;           // prefill_block records layer_done[li]
  bool wait_layers = false;             // run_pass makes its stream wait for layer_done[li] before layer li
  std::vector<ProfRec> prof;

  uint32_t H() const { return c.hidden; }
  uint32_t Dq() const { return c.n_q_heads * c.head_dim; }
  uint32_t Dkv() const { return c.n_kv_heads * c.head_dim; }
  uint32_t F() const { return c.ffn; }
  uint32_t V() const { return c.vocab; }
  size_t esz() const { return f32 ? 4 : 2; }
  int ktile() const { return f32 ? 16 : 32; }
  bool w8 = false;  // the layers' matrices are signed bytes with per-row scales (blob_dtype NNC_W8)
  // bytes per weight and k per weight tile of the layers' matrices (embedding / LM head: esz, ktile)
  size_t wsz() const { return w8 ? 1 : esz(); }
  int wktile() const { return w8 ? 64 : ktile(); }
};

namespace {

constexpr uint32_t PREFILL_TAIL = 16;      // last tokens of a long prompt that run through the fp32-grade chunk path
constexpr uint32_t MAX_DECODE_BATCH = 21;  // 21 sequences x 3 pieces = 63 operand columns

nnc_status check_config(const nnc_config* c) {
  if (!c) return fail(NNC_E_ARG, "config is NULL");
  if (c->struct_bytes != sizeof(nnc_config))
    return fail(NNC_E_CONFIG, "struct_bytes %u != sizeof(nnc_config) %zu", c->struct_bytes, sizeof(nnc_config));
  if (!c->hidden || !c->n_q_heads || !c->n_kv_heads || !c->ffn || !c->max_batch || !c->max_seq)
    return fail(NNC_E_CONFIG, "zero dimension in config");
  if (c->head_dim != 128) return fail(NNC_E_CONFIG, "head_dim %u unsupported (kernels are written for 128)", c->head_dim);
  if (c->n_q_heads % c->n_kv_heads) return fail(NNC_E_CONFIG, "n_q_heads %% n_kv_heads != 0");
  if (c->hidden % 32 || c->ffn % 32) return fail(NNC_E_CONFIG, "hidden and ffn must be multiples of 32");
  if (c->has_embed_and_head && (c->vocab == 0 || c->vocab % 16))
    return fail(NNC_E_CONFIG, "vocab must be a positive multiple of 16");
  if (c->blob_dtype > NNC_W8 || c->compute_dtype > NNC_F16)
    return fail(NNC_E_CONFIG, "unknown dtype");
  if (c->blob_dtype == NNC_W8) {
    if (c->compute_dtype != NNC_BF16) return fail(NNC_E_CONFIG, "a weight-only 8-bit blob computes in bf16");
    if (c->hidden % 64 || c->ffn % 64) return fail(NNC_E_CONFIG, "8-bit weights need hidden and ffn to be multiples of 64");
  } else if (c->blob_dtype != NNC_F32 && c->blob_dtype != c->compute_dtype)
    return fail(NNC_E_CONFIG, "a 16-bit blob must be in the compute dtype (an fp32 blob is rounded once at create)");
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(NNC_E_CONFIG, "bad rms_eps / rope_theta");
  if (c->max_batch > 4096 || c->max_seq > (1u << 20)) return fail(NNC_E_CONFIG, "max_batch / max_seq too large");
  if (c->n_layers > 1024) return fail(NNC_E_CONFIG, "too many layers");
  return NNC_OK;
}

uint64_t blob_bytes_of(const nnc_config* c) {
  const uint64_t H = c->hidden, d = c->head_dim, Dq = (uint64_t)c->n_q_heads * d,
                 Dkv = (uint64_t)c->n_kv_heads * d, F = c->ffn, V = c->vocab;
  const uint64_t w = c->blob_dtype == NNC_F32 ? 4 : 2;
  uint64_t total = (uint64_t)c->n_layers * (w * (Dq * H + 2 * Dkv * H + H * Dq + 3 * F * H) + 4 * (2 * H + 2 * d));
  if (c->blob_dtype == NNC_W8)  // bytes + one fp32 scale per output row (embedding / LM head stay 16-bit)
    total = (uint64_t)c->n_layers * ((Dq * H + 2 * Dkv * H + H * Dq + 3 * F * H) + 4 * (Dq + 2 * Dkv + H + 2 * F + H) +
                                     4 * (2 * H + 2 * d));
  if (c->has_embed_and_head) {
    total += w * V * H + 4 * H;
    if (!c->tied_lm_head) total += w * V * H;
  }
  return total;
}

nnc_status dev_fail(hipError_t e, const char* what) {
  return fail(e == hipErrorOutOfMemory ? NNC_E_NOMEM : NNC_E_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(call)                                      \
  do {                                                     \
    hipError_t e_ = (call);                                \
    if (e_ != hipSuccess) return dev_fail(e_, #call);      \
  } while (0)

void* dev_alloc(nnc_model* m, size_t bytes) {
  void* p = nullptr;
  if (bytes == 0) bytes = 256;
  if (m->use_hooks) {
    p = m->hooks.alloc(bytes, m->hooks.ctx);
  } else if (hipMalloc(&p, bytes) != hipSuccess) {
    p = nullptr;
  }
  if (p) m->allocs.push_back(p);
  return p;
}

void release_all(nnc_model* m) {
  if (m->tail_stream) {
    (void)hipStreamSynchronize(m->tail_stream);
    (void)hipStreamDestroy(m->tail_stream);
    m->tail_stream = nullptr;
  }
  for (hipEvent_t e : m->layer_done) (void)hipEventDestroy(e);
  m->layer_done.clear();
  for (auto& kv : m->graphs) (void)hipGraphExecDestroy(kv.second);
  m->graphs.clear();
  for (auto& r : m->prof) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  m->prof.clear();
  for (void* p : m->allocs) {
    if (m->use_hooks)
      m->hooks.free(p, m->hooks.ctx);
    else
      (void)hipFree(p);
  }
  m->allocs.clear();
  if (m->mk_error_host) (void)hipHostFree(m->mk_error_host);
  if (m->mk_error_event) (void)hipEventDestroy(m->mk_error_event);
  m->mk_error_host = nullptr;
  m->mk_error_event = nullptr;
}

// ---- launch bookkeeping ------------------------------------------------------

struct Launch {
  nnc_model* m;
  int fam;
  double bytes, flops;
  Launch(nnc_model* m_, int fam_, double bytes_, double flops_) : m(m_), fam(fam_), bytes(bytes_), flops(flops_) {
    if (m->profiling) {
      ProfRec r{fam, bytes, flops, nullptr, nullptr};
      if (hipEventCreate(&r.e0) == hipSuccess && hipEventCreate(&r.e1) == hipSuccess) {
        (void)hipEventRecord(r.e0, m->stream);
        m->prof.push_back(r);
      }
    }
  }
  ~Launch() {
    if (m->profiling && !m->prof.empty()) (void)hipEventRecord(m->prof.back().e1, m->stream);
  }
};

#define RUN(fam, bytes, flops, call)                     \
  do {                                                   \
    hipError_t e_;                                       \
    {                                                    \
      Launch l_(m, fam, (double)(bytes), (double)(flops)); \
      e_ = (call);                                       \
    }                                                    \
    if (e_ != hipSuccess) return dev_fail(e_, #call);    \
  } while (0)

// k-slices for the narrow output projections: enough workgroups to cover the chip,
// but at least 8 k tiles (2 per wave) per workgroup.
// Prompt blocks may split the k range of their narrow (residual) projections over up to
// PB_SPLIT_MAX workgroups per output tile: any block when the tile model picks the launch, blocks of
// at most PB_SPLIT_TOKENS tokens on the 64-row tiles under the fixed rules.
constexpr int PB_SPLIT_MAX = 4;
constexpr uint32_t PB_SPLIT_TOKENS = 512;
constexpr int MAX_KSPLIT = 8;  // the norm kernel folds at most eight pending partials
int pick_kts(int n_tiles, int KT) {
  int ksplit = 512 / (n_tiles > 0 ? n_tiles : 1);
  if (ksplit < 1) ksplit = 1;
  if (ksplit > MAX_KSPLIT) ksplit = MAX_KSPLIT;
  int max_split = KT / 8;
  if (max_split < 1) max_split = 1;
  if (ksplit > max_split) ksplit = max_split;
  return (KT + ksplit - 1) / ksplit;
}

// Row tiles per workgroup and k slices of a weight-streaming GEMM from the analytic model
// (the hand rules: pick_kts above and the launcher's own row-tile rule, stay in `a` when the
// planner is switched off).
constexpr int MAX_QKV_SLICES = 4;  // k slices of the QKV projection that the fused attention kernel adds up
// wide: launches that may run alone on the chip (decode passes).  The chunk pass behind a long
// prompt runs beside the prompt's last block on a second stream; workgroups of 6 or 8 row tiles
// (240 registers per wave) do not fit next to that block's GEMM workgroups and cost the prompt 5 %.
int skinny_rt_choices(int dt, int epi, bool wide = true) {
  if (dt == (int)NNC_F32 || !wide) return epi == EPI_SWIGLU ? ((1 << 2) | (1 << 4)) : ((1 << 1) | (1 << 2) | (1 << 4));
  return epi == EPI_SWIGLU ? ((1 << 2) | (1 << 4) | (1 << 6) | (1 << 8)) : ((1 << 1) | (1 << 2) | (1 << 3) | (1 << 4) | (1 << 6));
}
void plan_skinny(const nnc_model* m, GemmArgs& a, int epi, int max_slices, bool wide) {
  if (!m->opt_planner) return;
  const Machine mc = machine_mi355x(m->n_cus);
  // byte weights: a weight tile meets two operand k tiles
  const bool w8 = a.wscale != nullptr;
  const SkinnyGemmPlan pl = plan_skinny_gemm(mc, a.n_tiles, a.KT, w8 ? 2 * a.ncols : a.ncols, a.nseq,
                                             skinny_rt_choices(m->dt, epi, wide), max_slices);
  if (pl.rt <= 0) return;
  a.rt = pl.rt;
  a.kts_per_split = pl.kts_per_split;
}

struct Pass {
  int ncols = 0;          // sequences (columns) in the pass
  int nsplit = 1;         // bf16 pieces per activation
  bool tokens = true;     // embed from ColState.tok; otherwise x already holds the input rows
  int head_col0 = 0;      // first column whose logits are wanted
  int head_ncols = 0;     // number of such columns (0: skip final norm + LM head)
  float* logits = nullptr;
  long logits_ld = 0;
  const uint32_t* step_ptr = nullptr;
  long step_stride = 0;
  int32_t* next = nullptr;  // arg-max output (device) or NULL
  int grid_chunks = 1;
  double kv_rows = 0;       // sum over columns of (position + 1): cached rows attention must read
  bool one_slot = false;    // the columns are consecutive positions of one slot (prompt chunk)
  bool decode = false;      // every column is a different slot: QK-norm, RoPE and the cache append may run inside the attention kernel
};

nnc_status run_pass(nnc_model* m, const Pass& p) {
  const nnc_config& c = m->c;
  hipStream_t s = m->stream;
  const int dt = m->dt;  // element type, passed to every launcher
  const int H = m->H(), Dq = m->Dq(), Dkv = m->Dkv(), F = m->F(), V = m->V();
  const int nq = c.n_q_heads, nkv = c.n_kv_heads;
  const int n = p.ncols, ns = p.nsplit, nc = n * ns;
  const double w = (double)m->wsz(), hw = (double)m->esz();  // bytes per weight: layers, embedding / LM head
  const int KTH = H / m->wktile(), KTQ = Dq / m->wktile(), KTF = F / m->wktile();
  const int Nqkv = Dq + 2 * Dkv;

  if (p.tokens) RUN(FAM_EMBED, n * H * hw, 0, launch_embed(s, dt, m->embed, H, m->st, n, m->x));

  const ColMap cm{m->st, 0, 0, 0};
  // k-slice partials of the previous projection still to be added to x
  int pending = 0;
  const long pstride = (long)n * H;
  // Decode passes run the norm that follows an O / down projection in that GEMM's tail
  // (NormTail): two kernels less per layer.  The head's norm stays a kernel when the head takes
  // a sub-range of the columns.
  const bool fuse_norm = p.decode && m->opt_fuse_norm && m->tail_counters && m->mk_error && H % 4 == 0 && H <= 8192;
  bool normed = false;  // Xp already holds the normed input of the next GEMM
  int tails = 0;
  auto norm_tail = [&](GemmArgs& a, const float* gain) {
    a.tail.counter = m->tail_counters + tails++;
    a.tail.x = m->x; a.tail.ldx = H; a.tail.gain = gain; a.tail.H = H; a.tail.eps = c.rms_eps;
    a.tail.Xp = m->Xp; a.tail.NC = nc; a.tail.nsplit = ns;
    a.tail.spin_limit = m->mk_spin_limit ? m->mk_spin_limit : (1u << 20);
    a.tail.error = m->mk_error;
  };
  if (fuse_norm) HIP_TRY(launch_zero_words(s, m->tail_counters, 2 * (int)c.n_layers));
  for (uint32_t li = 0; li < c.n_layers; ++li) {
    const LayerW& L = m->L[li];
    if (m->wait_layers) HIP_TRY(hipStreamWaitEvent(s, m->layer_done[li], 0));
    if (!normed)
      RUN(FAM_NORM, n * H * 8.0, 0,
          launch_rmsnorm_pack(s, dt, m->x, H, m->rpart, pending, pstride, L.g_in, H, c.rms_eps, n, m->Xp, nc, ns));
    normed = false;
    const bool fuse = p.decode && m->opt_fuse_qk && attn_partial_can_fuse(dt, nq, nkv);
    int qkv_slices = 1;
    {
      GemmArgs a{};
      a.Wp = L.wqkv; a.wscale = L.sqkv; a.n_tiles = Nqkv / 16; a.KT = KTH; a.kts_per_split = KTH;
      a.Xp = m->Xp; a.NC = nc; a.ncols = nc; a.nsplit = ns; a.nseq = n;
      a.out = m->qkv; a.ldo = Nqkv; a.split_stride = (long)n * Nqkv;
      // the fused attention kernel adds k-slice partial sums itself; every other consumer wants full sums
      plan_skinny(m, a, EPI_STORE, fuse ? MAX_QKV_SLICES : 1, p.decode);
      qkv_slices = (KTH + a.kts_per_split - 1) / a.kts_per_split;
      RUN(FAM_GEMM, (double)Nqkv * H * w, 2.0 * Nqkv * H * n, launch_gemm(s, dt, EPI_STORE, a));
    }
    const AttnFuseArgs fz{L.g_q, L.g_k, c.rms_eps, m->rope, qkv_slices, (long)n * Nqkv};
    if (!fuse)
      RUN(FAM_QKROPE, n * Nqkv * 4.0, 0,
          launch_qknorm_rope_append(s, dt, m->qkv, nq, nkv, L.g_q, L.g_k, c.rms_eps, m->rope, cm, n,
                                    L.kc, L.vc, c.max_batch, c.max_seq, m->qsplit, nullptr, 0));
    RUN(FAM_ATTN, p.kv_rows * 2.0 * Dkv * hw, p.kv_rows * 4.0 * Dq,
        launch_attn_partial(s, dt, m->qkv, m->qsplit, nq, nkv, L.kc, L.vc, c.max_batch, c.max_seq, cm, n,
                            p.grid_chunks, m->partial, m->max_chunks, fuse ? &fz : nullptr, p.one_slot));
    RUN(FAM_COMBINE, 0, 0,
        launch_attn_combine(s, dt, m->partial, m->max_chunks, nq, cm, n, m->Ap, nc, ns));
    {
      GemmArgs a{};
      a.Wp = L.wo; a.wscale = L.so; a.n_tiles = H / 16; a.KT = KTQ; a.kts_per_split = pick_kts(a.n_tiles, KTQ);
      a.Xp = m->Ap; a.NC = nc; a.ncols = nc; a.nsplit = ns; a.nseq = n;
      a.out = m->rpart; a.ldo = H; a.split_stride = pstride;
      plan_skinny(m, a, EPI_STORE, MAX_KSPLIT, p.decode);
      pending = (KTQ + a.kts_per_split - 1) / a.kts_per_split;
      if (fuse_norm) norm_tail(a, L.g_post);
      RUN(FAM_GEMM_O, (double)H * Dq * w, 2.0 * H * Dq * n, launch_gemm(s, dt, EPI_STORE, a));
    }
    if (!fuse_norm)
      RUN(FAM_NORM, n * H * 8.0, 0,
          launch_rmsnorm_pack(s, dt, m->x, H, m->rpart, pending, pstride, L.g_post, H, c.rms_eps, n, m->Xp, nc, ns));
    {
      GemmArgs a{};
      a.Wp = L.wgu; a.wscale = L.sgu; a.n_tiles = 2 * F / 16; a.KT = KTH; a.kts_per_split = KTH;
      a.Xp = m->Xp; a.NC = nc; a.ncols = nc; a.nsplit = ns; a.nseq = n;
      a.packed_out = m->Ap; a.NC_out = nc; a.nsplit_out = ns;
      plan_skinny(m, a, EPI_SWIGLU, 1, p.decode);
      RUN(FAM_GEMM_GU, 2.0 * F * H * w, 4.0 * F * H * n, launch_gemm(s, dt, EPI_SWIGLU, a));
    }
    {
      GemmArgs a{};
      a.Wp = L.wd; a.wscale = L.sd; a.n_tiles = H / 16; a.KT = KTF; a.kts_per_split = pick_kts(a.n_tiles, KTF);
      a.Xp = m->Ap; a.NC = nc; a.ncols = nc; a.nsplit = ns; a.nseq = n;
      a.out = m->rpart; a.ldo = H; a.split_stride = pstride;
      plan_skinny(m, a, EPI_STORE, MAX_KSPLIT, p.decode);
      pending = (KTF + a.kts_per_split - 1) / a.kts_per_split;
      // the norm this output feeds: the next layer's input norm, or the final norm when the head
      // wants every column
      const bool last = li + 1 == c.n_layers;
      const bool head_all = c.has_embed_and_head && p.head_ncols == n && p.head_col0 == 0;
      if (fuse_norm && (!last || head_all)) {
        norm_tail(a, last ? m->g_final : m->L[li + 1].g_in);
        normed = true;
      }
      RUN(FAM_GEMM_D, (double)H * F * w, 2.0 * H * F * n, launch_gemm(s, dt, EPI_STORE, a));
      if (normed) pending = 0;
    }
  }

  if (c.has_embed_and_head && p.head_ncols > 0) {
    const int hn = p.head_ncols, hc = hn * ns;
    if (!normed)
      RUN(FAM_NORM, hn * H * 8.0, 0,
          launch_rmsnorm_pack(s, dt, m->x + (size_t)p.head_col0 * H, H, m->rpart + (size_t)p.head_col0 * H, pending,
                              pstride, m->g_final, H, c.rms_eps, hn, m->Xp, hc, ns));
    GemmArgs a{};
    const int KTV = H / m->ktile();  // the LM head is in the model's 16-bit format also when the layers are bytes
    a.Wp = m->lm_head; a.n_tiles = V / 16; a.KT = KTV; a.kts_per_split = KTV;
    a.Xp = m->Xp; a.NC = hc; a.ncols = hc; a.nsplit = ns; a.nseq = hn;
    a.out = p.logits; a.ldo = p.logits_ld; a.step_ptr = p.step_ptr; a.step_stride = p.step_stride;
    plan_skinny(m, a, EPI_STORE, 1, p.decode);
    RUN(FAM_GEMM_HEAD, (double)V * H * hw, 2.0 * V * H * hn, launch_gemm(s, dt, EPI_STORE, a));
    if (p.next)
      RUN(FAM_ARGMAX, hn * V * 4.0, 0,
          launch_argmax(s, p.logits, p.logits_ld, V, hn, p.step_ptr, p.step_stride, m->am_val, m->am_idx,
                        p.next));
  } else if (!c.has_embed_and_head && pending > 0) {
    // hidden-state models return x itself: add the last projection's partials now
    RUN(FAM_MISC, 0, 0, launch_fold_residual(s, m->x, m->rpart, pending, pstride, (size_t)n * H));
  }
  return NNC_OK;
}

// 16-bit pieces per activation in decode.  Three carry an fp32 value to within 2^-25 relative, so
// a batch of B sequences computes what B batch-1 steps compute; two carry it to 2^-17 (still 64
// times finer than a binary16 activation, the paper's own 16-bit precision: Section 4, setup) and
// are taken where they save a whole 16-column operand block of every decode GEMM (6-8 sequences:
// one block instead of two; 11-16: two instead of three; 17-21: three instead of four).
int decode_nsplit(const nnc_model* m, uint32_t batch) {
  if (m->f32) return 1;
  if (m->opt_decode_pieces && batch >= 2) return m->opt_decode_pieces;
  return (2 * batch + 15) / 16 < (3 * batch + 15) / 16 ? 2 : 3;
}

// Chunk count of an attention launch, rounded up to a multiple of 8 (the captured decode graphs
// are keyed by it: a new one every 512 positions, and at most 7 idle workgroups per sequence
// and kv head instead of up to half of them).
int chunks_grid(uint32_t max_pos) {
  const int need = (int)(max_pos / ATT_CHUNK) + 1;
  return (need + 7) / 8 * 8;
}

nnc_status check_slots(const nnc_model* m, const uint32_t* slots, uint32_t batch, uint32_t n_steps) {
  if (!m) return fail(NNC_E_ARG, "model is NULL");
  if (!slots) return fail(NNC_E_ARG, "slots is NULL");
  if (batch == 0 || batch > m->c.max_batch || batch > MAX_DECODE_BATCH)
    return fail(NNC_E_ARG, "batch %u out of range (max_batch %u, limit %u)", batch, m->c.max_batch, MAX_DECODE_BATCH);
  for (uint32_t i = 0; i < batch; ++i) {
    if (slots[i] >= m->c.max_batch) return fail(NNC_E_ARG, "slot %u out of range", slots[i]);
    for (uint32_t j = 0; j < i; ++j)
      if (slots[j] == slots[i]) return fail(NNC_E_ARG, "slot %u appears twice", slots[i]);
    if ((uint64_t)m->len[slots[i]] + n_steps > m->c.max_seq)
      return fail(NNC_E_KV_FULL, "slot %u: length %u + %u exceeds max_seq %u", slots[i], m->len[slots[i]], n_steps,
                  m->c.max_seq);
  }
  return NNC_OK;
}

nnc_status set_decode_state(nnc_model* m, const uint32_t* slots, const int32_t* tokens, uint32_t batch,
                            uint32_t* max_pos_out, double* kv_rows_out) {
  uint32_t pos[MAX_COLS];
  uint32_t mx = 0;
  double rows = 0;
  for (uint32_t i = 0; i < batch; ++i) {
    pos[i] = m->len[slots[i]];
    mx = pos[i] > mx ? pos[i] : mx;
    rows += pos[i] + 1.0;
  }
  *max_pos_out = mx;
  *kv_rows_out = rows;
  HIP_TRY(launch_set_state(m->stream, m->st, (int)batch, tokens, slots, pos, 0));
  return NNC_OK;
}

// One greedy decode step (pass + token feedback) as a graph, captured on first use
// per (batch, pieces, attention grid).
nnc_status greedy_step(nnc_model* m, uint32_t batch, int nsplit, int grid_chunks, bool allow_graph,
                       double kv_rows) {
  Pass p;
  p.decode = true;
  p.kv_rows = kv_rows;
  p.ncols = (int)batch;
  p.nsplit = nsplit;
  p.head_ncols = (int)batch;
  p.logits = m->logits;
  p.logits_ld = m->V();
  p.next = m->next;
  p.grid_chunks = grid_chunks;
  const bool graph = allow_graph && m->opt_graph && !m->profiling && m->stream != nullptr;
  if (!graph) {
    if (nnc_status st = run_pass(m, p)) return st;
    HIP_TRY(launch_finish_step(m->stream, m->st, (int)batch, m->next, m->token_log));
    return NNC_OK;
  }
  const auto key = std::make_tuple((int)batch, nsplit, grid_chunks);
  auto it = m->graphs.find(key);
  if (it == m->graphs.end()) {
    hipGraph_t g = nullptr;
    HIP_TRY(hipStreamBeginCapture(m->stream, hipStreamCaptureModeThreadLocal));
    nnc_status st = run_pass(m, p);
    hipError_t e1 = st == NNC_OK ? launch_finish_step(m->stream, m->st, (int)batch, m->next, m->token_log)
                                 : hipSuccess;
    hipError_t e2 = hipStreamEndCapture(m->stream, &g);
    if (st != NNC_OK) {
      if (g) (void)hipGraphDestroy(g);
      return st;
    }
    if (e1 != hipSuccess) return dev_fail(e1, "capture finish_step");
    if (e2 != hipSuccess) return dev_fail(e2, "hipStreamEndCapture");
    hipGraphExec_t ge = nullptr;
    hipError_t e3 = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
    (void)hipGraphDestroy(g);
    if (e3 != hipSuccess) return dev_fail(e3, "hipGraphInstantiate");
    it = m->graphs.emplace(key, ge).first;
  }
  HIP_TRY(hipGraphLaunch(it->second, m->stream));
  return NNC_OK;
}

bool use_persistent(const nnc_model* m, uint32_t batch) {
  return m->mk_ok && m->opt_persistent && !m->profiling && batch == 1;
}

// n_steps greedy decode steps of one sequence in one resident kernel, starting from
// `token` at the slot's current length.  Tokens land in token_log [n_steps].
// The give-up flag of the kernels that wait for other workgroups (the resident decode kernel, the
// norm tails of decode GEMMs) travels to pinned host memory behind the launches; the next call on
// this model that finds the copy complete looks at it (resident_failed).
nnc_status fetch_wait_flag(nnc_model* m) {
  if (!m->mk_error) return NNC_OK;
  HIP_TRY(hipMemcpyAsync(m->mk_error_host, m->mk_error, sizeof(unsigned), hipMemcpyDeviceToHost, m->stream));
  HIP_TRY(hipEventRecord(m->mk_error_event, m->stream));
  m->mk_error_pending = true;
  return NNC_OK;
}

nnc_status persistent_steps(nnc_model* m, uint32_t slot, int32_t token, uint32_t n_steps, float* logits_out) {
  const nnc_config& c = m->c;
  MkPlan p{};
  p.nwg = m->mk_nwg;
  p.n_layers = (int)c.n_layers; p.H = (int)m->H(); p.nq = (int)c.n_q_heads; p.nkv = (int)c.n_kv_heads;
  p.F = (int)m->F(); p.V = (int)m->V();
  p.eps = c.rms_eps; p.max_seq = c.max_seq; p.max_chunks = m->max_chunks;
  p.tok0 = token; p.pos0 = m->len[slot]; p.slot = slot;
  p.n_steps = (int)n_steps;
  p.tag_base = m->mk_tag;
  p.ks_o = m->mk_ks_o; p.ks_d = m->mk_ks_d;
  p.f16 = m->dt == NNC_F16;
  {
    // gate/up pairs and attention units start at workgroup 0 (attention workgroups then have
    // nothing to prefetch before they wait for q); output-projection units end at the last
    // workgroup; down-projection units start after the attention workgroups
    const int o_units = (int)(m->H() / 16) * p.ks_o;
    const int att_units = (int)c.n_kv_heads * ((int)(m->len[slot] + n_steps - 1) / ATT_CHUNK + 1);
    auto wrap = [&](int v) { return ((v % p.nwg) + p.nwg) % p.nwg; };
    p.off_att = 0;
    p.off_o = wrap(p.nwg - o_units);
    p.off_d = wrap(att_units);
  }
  const uint64_t tags = (uint64_t)n_steps * mk_tags_per_step((int)c.n_layers);
  if ((uint64_t)m->mk_tag + tags >= 0xffffffffull)
    return fail(NNC_E_STATE, "exchange tags exhausted (after ~2^32 / %u decode steps); recreate the model",
                mk_tags_per_step((int)c.n_layers));
  MkBuffers b{};
  b.layers = m->mk_layers; b.embed = m->embed; b.lm_head = m->lm_head; b.g_final = m->g_final; b.rope = m->rope;
  b.error = m->mk_error;
  b.xq = m->mk_xq; b.xatt = m->mk_xatt; b.xo = m->mk_xo; b.xop = m->mk_xop; b.xact = m->mk_xact; b.xdp = m->mk_xdp;
  b.xamv = m->mk_xamv; b.xami = m->mk_xami;
  b.logits = logits_out; b.token_log = m->token_log;
  b.trace = m->mk_trace_step >= 0 ? m->mk_trace : nullptr;
  b.trace_step = m->mk_trace_step;
  b.trace_points = mk_trace_points((int)c.n_layers);
  p.spin_max = m->mk_spin_limit;
  HIP_TRY(launch_decode_resident(m->stream, p, b));
  m->mk_tag += (unsigned)tags;
  // the kernel's give-up flag travels to pinned host memory behind the launch; the next call
  // on this model that finds the copy complete looks at it (resident_failed)
  return fetch_wait_flag(m);
}

// True once a resident launch has given up on a wait (a lost exchange word): every workgroup
// of that launch exited early and its outputs are invalid.  The condition is sticky.
bool resident_failed(nnc_model* m, bool wait) {
  if (m->mk_error_pending) {
    hipError_t e = wait ? hipEventSynchronize(m->mk_error_event) : hipEventQuery(m->mk_error_event);
    if (e == hipSuccess) {
      m->mk_error_pending = false;
      if (*m->mk_error_host) m->mk_failed = true;
    }
  }
  return m->mk_failed;
}

}  // namespace

// =============================================================================
// public ABI
// =============================================================================
extern "C" {

const char* nnc_last_error(void) { return g_err; }

uint64_t nnc_blob_bytes(const nnc_config* cfg) {
  if (check_config(cfg) != NNC_OK) return 0;
  return blob_bytes_of(cfg);
}

nnc_status nnc_model_create(const nnc_config* cfg, const void* blob, size_t blob_bytes, const nnc_device* dev,
                            nnc_model** out) {
  if (!out) return fail(NNC_E_ARG, "out is NULL");
  if (nnc_status st = check_config(cfg)) return st;
  if (!blob) return fail(NNC_E_ARG, "blob is NULL");
  if ((uint64_t)blob_bytes != blob_bytes_of(cfg))
    return fail(NNC_E_BLOB, "blob has %zu bytes, config needs %llu", blob_bytes,
                (unsigned long long)blob_bytes_of(cfg));

  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) return fail(NNC_E_DEVICE, "no HIP device");
  int device = 0;
  HIP_TRY(hipGetDevice(&device));
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, device));
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(NNC_E_DEVICE, "device is %s; this library is built for gfx950 only", prop.gcnArchName);

  nnc_model* m = new (std::nothrow) nnc_model;
  if (!m) return fail(NNC_E_NOMEM, "host allocation failed");
  m->c = *cfg;
  m->f32 = cfg->compute_dtype == NNC_F32;
  m->dt = (int)cfg->compute_dtype;
  m->w8 = cfg->blob_dtype == NNC_W8;
  m->device = device;
  m->n_cus = prop.multiProcessorCount;
  if (dev) {
    m->stream = static_cast<hipStream_t>(dev->stream);
    if (dev->alloc && dev->free) {
      m->hooks = *dev;
      m->use_hooks = true;
    }
  }
  m->opt_prefill_exact = 0;
  const nnc_config& c = m->c;
  const size_t H = m->H(), Dq = m->Dq(), Dkv = m->Dkv(), F = m->F(), V = m->V(), d = c.head_dim;
  const size_t w = m->esz(), bw = c.blob_dtype == NNC_F32 ? 4 : 2, lw = m->wsz();
  const bool src_f32 = c.blob_dtype == NNC_F32;
  hipStream_t s = m->stream;

  nnc_status st = NNC_OK;
  auto bail = [&](nnc_status code) {
    (void)hipStreamSynchronize(s);
    release_all(m);
    delete m;
    return code;
  };
#define ALLOC(ptr, type, bytes)                                                              \
  do {                                                                                       \
    (ptr) = static_cast<type>(dev_alloc(m, (bytes)));                                        \
    if (!(ptr)) return bail(fail(NNC_E_NOMEM, "device allocation of %zu bytes failed", (size_t)(bytes))); \
  } while (0)
#define TRY_OR_BAIL(call)                                  \
  do {                                                     \
    hipError_t e_ = (call);                                \
    if (e_ != hipSuccess) return bail(dev_fail(e_, #call)); \
  } while (0)

  // staging buffer for one canonical matrix at a time
  size_t stage_elems = std::max(std::max(Dq * H, 2 * 0 + F * H), c.has_embed_and_head ? V * H : 0);
  void* stage = nullptr;
  ALLOC(stage, void*, stage_elems * bw);

  const char* bp = static_cast<const char*>(blob);
  auto upload_gain = [&](float*& dst, size_t n) -> hipError_t {
    dst = static_cast<float*>(dev_alloc(m, n * 4));
    if (!dst) return hipErrorOutOfMemory;
    hipError_t e = hipMemcpyAsync(dst, bp, n * 4, hipMemcpyHostToDevice, s);
    bp += n * 4;
    return e;
  };
  auto upload_matrix = [&](void* dst, size_t rows, size_t K, int tile_stride, int tile_offset) -> hipError_t {
    hipError_t e = hipMemcpyAsync(stage, bp, rows * K * bw, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    bp += rows * K * bw;
    return launch_repack(s, src_f32, m->dt, stage, dst, (int)rows, (int)K, tile_stride, tile_offset);
  };

  // A matrix of a layer.  Byte-weight blobs: rows x K signed bytes, then rows fp32 scales, which go
  // into `scales` (host, packed row order: tile nt of the sub-matrix becomes tile
  // nt * tile_stride + tile_offset) and are uploaded once per fused matrix.
  std::vector<float> scales;
  auto upload_layer_matrix = [&](void* dst, size_t rows, size_t K, int tile_stride, int tile_offset) -> hipError_t {
    if (!m->w8) return upload_matrix(dst, rows, K, tile_stride, tile_offset);
    hipError_t e = hipMemcpyAsync(stage, bp, rows * K, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    bp += rows * K;
    for (size_t nt = 0; nt < rows / 16; ++nt) {
      const size_t dt_ = (nt * tile_stride + tile_offset) * 16;
      if (scales.size() < dt_ + 16) scales.resize(dt_ + 16, 0.f);
      memcpy(&scales[dt_], bp + nt * 64, 64);
    }
    bp += rows * 4;
    return launch_repack_w8(s, stage, dst, (int)rows, (int)K, tile_stride, tile_offset);
  };
  auto upload_scales = [&](float*& dst) -> hipError_t {
    if (!m->w8) return hipSuccess;
    dst = static_cast<float*>(dev_alloc(m, scales.size() * 4));
    if (!dst) return hipErrorOutOfMemory;
    // synchronous: `scales` is reused for the next matrix
    hipError_t e = hipMemcpyAsync(dst, scales.data(), scales.size() * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    scales.clear();
    return e;
  };

  if (c.has_embed_and_head) {
    ALLOC(m->embed, void*, V * H * w);
    TRY_OR_BAIL(upload_matrix(m->embed, V, H, 1, 0));
  }
  m->L.resize(c.n_layers);
  for (auto& L : m->L) {
    TRY_OR_BAIL(upload_gain(L.g_in, H));
    ALLOC(L.wqkv, void*, (Dq + 2 * Dkv) * H * lw);
    TRY_OR_BAIL(upload_layer_matrix(L.wqkv, Dq, H, 1, 0));
    TRY_OR_BAIL(upload_layer_matrix(L.wqkv, Dkv, H, 1, (int)(Dq / 16)));
    TRY_OR_BAIL(upload_layer_matrix(L.wqkv, Dkv, H, 1, (int)((Dq + Dkv) / 16)));
    TRY_OR_BAIL(upload_scales(L.sqkv));
    TRY_OR_BAIL(upload_gain(L.g_q, d));
    TRY_OR_BAIL(upload_gain(L.g_k, d));
    ALLOC(L.wo, void*, H * Dq * lw);
    TRY_OR_BAIL(upload_layer_matrix(L.wo, H, Dq, 1, 0));
    TRY_OR_BAIL(upload_scales(L.so));
    TRY_OR_BAIL(upload_gain(L.g_post, H));
    ALLOC(L.wgu, void*, 2 * F * H * lw);
    TRY_OR_BAIL(upload_layer_matrix(L.wgu, F, H, 2, 0));
    TRY_OR_BAIL(upload_layer_matrix(L.wgu, F, H, 2, 1));
    TRY_OR_BAIL(upload_scales(L.sgu));
    ALLOC(L.wd, void*, H * F * lw);
    TRY_OR_BAIL(upload_layer_matrix(L.wd, H, F, 1, 0));
    TRY_OR_BAIL(upload_scales(L.sd));
    const size_t kv_bytes = (size_t)c.max_batch * c.n_kv_heads * c.max_seq * d * w;
    ALLOC(L.kc, void*, kv_bytes);
    ALLOC(L.vc, void*, kv_bytes);
    // The attention kernels load rows past the last cached position of a chunk (clamped to a valid
    // row) and give them weight zero; a slot's first rows are read that way before they are
    // written, so they must hold finite values from the start.
    TRY_OR_BAIL(hipMemsetAsync(L.kc, 0, kv_bytes, s));
    TRY_OR_BAIL(hipMemsetAsync(L.vc, 0, kv_bytes, s));
  }
  if (c.has_embed_and_head) {
    TRY_OR_BAIL(upload_gain(m->g_final, H));
    if (c.tied_lm_head) {
      m->lm_head = m->embed;
    } else {
      ALLOC(m->lm_head, void*, V * H * w);
      TRY_OR_BAIL(upload_matrix(m->lm_head, V, H, 1, 0));
    }
  }

  // rotary table: cos/sin of pos * theta^(-2i/d), evaluated in fp64, stored as fp32
  {
    const size_t n = (size_t)c.max_seq * 64;
    std::vector<float2> tab(n);
    for (uint32_t p = 0; p < c.max_seq; ++p)
      for (int i = 0; i < 64; ++i) {
        const double phi = (double)p * std::pow((double)c.rope_theta, -2.0 * i / 128.0);
        tab[(size_t)p * 64 + i] = make_float2((float)std::cos(phi), (float)std::sin(phi));
      }
    ALLOC(m->rope, float2*, n * sizeof(float2));
    TRY_OR_BAIL(hipMemcpyAsync(m->rope, tab.data(), n * sizeof(float2), hipMemcpyHostToDevice, s));
    TRY_OR_BAIL(hipStreamSynchronize(s));  // tab goes out of scope
  }

  m->max_chunks = chunks_grid(c.max_seq - 1);
  ALLOC(m->st, ColState*, sizeof(ColState));
  ALLOC(m->x, float*, (size_t)MAX_COLS * H * 4);
  ALLOC(m->qkv, float*, (size_t)MAX_QKV_SLICES * MAX_COLS * (Dq + 2 * Dkv) * 4);
  ALLOC(m->Xp, void*, (size_t)MAX_COLS * H * w);
  ALLOC(m->Ap, void*, (size_t)MAX_COLS * std::max(Dq, F) * w);
  ALLOC(m->rpart, float*, (size_t)MAX_KSPLIT * MAX_COLS * H * 4);
  ALLOC(m->partial, float*, (size_t)MAX_COLS * c.n_q_heads * m->max_chunks * 132 * 4);
  if (!m->f32) ALLOC(m->qsplit, void*, (size_t)MAX_COLS * c.n_q_heads * 3 * 128 * 2);
  ALLOC(m->next, int32_t*, MAX_COLS * 4);
  m->token_log_steps = c.max_seq;
  ALLOC(m->token_log, int32_t*, (size_t)m->token_log_steps * MAX_DECODE_BATCH * 4);
  if (c.has_embed_and_head) {
    ALLOC(m->logits, float*, (size_t)MAX_DECODE_BATCH * V * 4);
    ALLOC(m->am_val, float*, MAX_COLS * 64 * 4);
    ALLOC(m->am_idx, int32_t*, MAX_COLS * 64 * 4);
  }
  // prompt pass on large token blocks (16-bit token models; byte-weight models widen the matrix
  // of each GEMM into a scratch buffer first)
  if (!m->f32 && c.has_embed_and_head) {
    uint32_t pb = (c.max_seq + 127) / 128 * 128;
    if (pb > 4096) pb = 4096;
    m->pb_max = pb;
    ALLOC(m->pb_x, float*, (size_t)pb * H * 4);
    ALLOC(m->pb_qkv, float*, (size_t)pb * (Dq + 2 * Dkv) * 4);
    // up to two bf16 pieces per activation
    const size_t frag_rows = 2 * (size_t)pb;
    ALLOC(m->pb_fa, void*, frag_rows * H * 2);
    ALLOC(m->pb_fb, void*, frag_rows * std::max(Dq, F) * 2);
    ALLOC(m->pb_tok, int32_t*, (size_t)pb * 4);
    if (m->w8) ALLOC(m->pb_w, void*, std::max(std::max(Dq + 2 * Dkv, 2 * F) * H, H * std::max(Dq, F)) * 2);
    // k-slice partials of the narrow projections (up to PB_SPLIT_MAX - 1 buffers of a whole block)
    ALLOC(m->pb_part, float*, (size_t)(PB_SPLIT_MAX - 1) * pb * H * 4);
    // transposed V copy of one slot: [kv head][128][positions, padded to a multiple of 32];
    // zero-filled once so that positions never written read as finite values
    m->pb_vt_stride = (c.max_seq + 31) / 32 * 32;
    ALLOC(m->pb_vt, void*, (size_t)c.n_kv_heads * 128 * m->pb_vt_stride * 2);
    TRY_OR_BAIL(hipMemsetAsync(m->pb_vt, 0, (size_t)c.n_kv_heads * 128 * m->pb_vt_stride * 2, s));
  }

  // give-up flag of the kernels whose workgroups wait for each other, and the arrival counters of
  // the norm tails (two GEMM launches per layer)
  {
    void* err = dev_alloc(m, 256);
    if (!err) TRY_OR_BAIL(hipErrorOutOfMemory);
    TRY_OR_BAIL(hipMemsetAsync(err, 0, 256, s));
    m->mk_error = static_cast<unsigned*>(err);
    TRY_OR_BAIL(hipHostMalloc(reinterpret_cast<void**>(&m->mk_error_host), sizeof(unsigned), hipHostMallocDefault));
    *m->mk_error_host = 0;
    TRY_OR_BAIL(hipEventCreateWithFlags(&m->mk_error_event, hipEventDisableTiming));
    void* cnt = dev_alloc(m, (2 * (size_t)c.n_layers + 2) * 4);
    if (!cnt) TRY_OR_BAIL(hipErrorOutOfMemory);
    TRY_OR_BAIL(hipMemsetAsync(cnt, 0, (2 * (size_t)c.n_layers + 2) * 4, s));
    m->tail_counters = static_cast<uint32_t*>(cnt);
  }

  // resident decode kernel: per-layer pointer table, exchange buffers (16-bit weights only)
  if (!m->f32 && !m->w8 && c.has_embed_and_head && c.n_layers > 0 && H <= 4096 && (c.n_q_heads / c.n_kv_heads) % 2 == 0 &&
      c.n_q_heads / c.n_kv_heads <= 16) {
    const int qkv_tiles = (int)((Dq + 2 * Dkv) / 16);
    m->mk_nwg = prop.multiProcessorCount < qkv_tiles ? prop.multiProcessorCount : qkv_tiles;
    // k slices of the narrow projections (units = 16-row tiles x slices, dealt round-robin to the
    // workgroups): at most 4 (a consumer adds at most four partial vectors), at least 32 k tiles
    // per slice and a multiple of 4 (the four waves share a slice evenly); among those the count
    // that leaves the busiest workgroup the fewest bytes, ties going to 2, 3, 4, 1 in that order
    // (measured: fewer partials to add beat more parallelism, one slice per tile is slowest).
    auto pick_ks = [&](size_t K) {
      const int KT = (int)(K / 32), tiles = (int)(H / 16), nwg = m->mk_nwg;
      int best = 1;
      double best_m = 1e30;
      for (int ks : {2, 3, 4, 1}) {
        if (ks > 1 && (ks > KT / 32 || KT % (4 * ks))) continue;
        const double mload = (double)((tiles * ks + nwg - 1) / nwg) / ks;
        if (mload < best_m * 0.999) best_m = mload, best = ks;
      }
      return best;
    };
    m->mk_ks_o = pick_ks(Dq);
    m->mk_ks_d = pick_ks(F);
    MkPlan plan{};
    plan.H = (int)H; plan.nq = (int)c.n_q_heads; plan.nkv = (int)c.n_kv_heads; plan.F = (int)F;
    plan.ks_o = m->mk_ks_o; plan.ks_d = m->mk_ks_d;
    plan.f16 = m->dt == NNC_F16;
    // The grid's workgroups wait for each other, so all of them must be resident at once: ask
    // the runtime how many fit (registers, LDS).  If the grid does not fit, batch-1 decode
    // falls back to the per-stage kernels; it is not an error.
    if (m->mk_ks_o <= 4 && m->mk_ks_d <= 4 && mk_opnd_bytes(plan) <= 96 * 1024 &&
        mk_max_resident_workgroups(plan, m->n_cus) >= m->mk_nwg) {
      const size_t lb = mk_layer_bytes();
      std::vector<char> table(lb * c.n_layers);
      for (uint32_t i = 0; i < c.n_layers; ++i) {
        const LayerW& L = m->L[i];
        mk_fill_layer(table.data() + lb * i, L.wqkv, L.wo, L.wgu, L.wd, L.g_in, L.g_q, L.g_k, L.g_post, L.kc, L.vc);
      }
      ALLOC(m->mk_layers, void*, table.size());
      TRY_OR_BAIL(hipMemcpyAsync(m->mk_layers, table.data(), table.size(), hipMemcpyHostToDevice, s));
      auto zeroed = [&](void*& ptr, size_t bytes) -> hipError_t {
        ptr = dev_alloc(m, bytes);
        if (!ptr) return hipErrorOutOfMemory;
        return hipMemsetAsync(ptr, 0, bytes, s);
      };
      TRY_OR_BAIL(zeroed(m->mk_xq, (Dq + 2 * Dkv) * 8));
      TRY_OR_BAIL(zeroed(m->mk_xatt, (size_t)c.n_q_heads * m->max_chunks * 132 * 8));
      TRY_OR_BAIL(zeroed(m->mk_xo, Dq * 8));
      TRY_OR_BAIL(zeroed(m->mk_xop, 4 * H * 8));
      TRY_OR_BAIL(zeroed(m->mk_xact, F * 8));
      TRY_OR_BAIL(zeroed(m->mk_xdp, 4 * H * 8));
      TRY_OR_BAIL(zeroed(m->mk_xamv, (size_t)m->mk_nwg * 8));
      TRY_OR_BAIL(zeroed(m->mk_xami, (size_t)m->mk_nwg * 8));
      void* tr = nullptr;
      TRY_OR_BAIL(zeroed(tr, (size_t)m->mk_nwg * mk_trace_points((int)c.n_layers) * 8));
      m->mk_trace = static_cast<unsigned long long*>(tr);
      TRY_OR_BAIL(hipStreamSynchronize(s));  // table goes out of scope
      m->mk_ok = true;
    }
  }
  m->len.assign(c.max_batch, 0);
  TRY_OR_BAIL(hipStreamSynchronize(s));
  (void)st;
#undef ALLOC
#undef TRY_OR_BAIL
  *out = m;
  return NNC_OK;
}

void nnc_model_destroy(nnc_model* m) {
  if (!m) return;
  (void)hipStreamSynchronize(m->stream);
  release_all(m);
  delete m;
}

nnc_status nnc_kv_reset(nnc_model* m, int32_t slot) {
  if (!m) return fail(NNC_E_ARG, "model is NULL");
  if (slot < -1 || (slot >= 0 && (uint32_t)slot >= m->c.max_batch)) return fail(NNC_E_ARG, "slot %d out of range", slot);
  if (slot < 0)
    for (auto& l : m->len) l = 0;
  else
    m->len[slot] = 0;
  return NNC_OK;
}

nnc_status nnc_synchronize(nnc_model* m) {
  if (!m) return fail(NNC_E_ARG, "model is NULL");
  HIP_TRY(hipStreamSynchronize(m->stream));
  if (resident_failed(m, true))
    return fail(NNC_E_DEVICE, "a resident decode launch gave up waiting for an exchange word; its outputs are invalid, recreate the model");
  return NNC_OK;
}

nnc_status nnc_slot_len(const nnc_model* m, uint32_t slot, uint32_t* len_out) {
  if (!m || !len_out) return fail(NNC_E_ARG, "NULL argument");
  if (slot >= m->c.max_batch) return fail(NNC_E_ARG, "slot %u out of range", slot);
  *len_out = m->len[slot];
  return NNC_OK;
}

nnc_status nnc_set_option(nnc_model* m, nnc_option opt, int32_t value) {
  if (!m) return fail(NNC_E_ARG, "model is NULL");
  switch (opt) {
    case NNC_OPT_GRAPH: m->opt_graph = value != 0; return NNC_OK;
    case NNC_OPT_PREFILL_EXACT:
      if (value < 0 || value > 2) return fail(NNC_E_ARG, "prefill precision mode must be 0, 1 or 2");
      m->opt_prefill_exact = value;
      return NNC_OK;
    case NNC_OPT_PERSISTENT: m->opt_persistent = value != 0; return NNC_OK;
    case NNC_OPT_PREFILL_TILE:
      if (value < -1 || value > 6) return fail(NNC_E_ARG, "prefill tile must be -1 (automatic) or 0 .. 6");
      m->opt_prefill_tile = value;
      return NNC_OK;
    case NNC_OPT_PREFILL_KSLICES:
      if (value < 0 || value > PB_SPLIT_MAX) return fail(NNC_E_ARG, "prefill k slices must be 0 (by rule) or 1 .. %d", PB_SPLIT_MAX);
      m->opt_prefill_kslices = value;
      return NNC_OK;
    case NNC_OPT_TAIL_OVERLAP: m->opt_tail_overlap = value != 0; return NNC_OK;
    case NNC_OPT_PLANNER:
      m->opt_planner = value != 0;
      // captured decode graphs contain the launches of one or the other choice
      for (auto& kv : m->graphs) (void)hipGraphExecDestroy(kv.second);
      m->graphs.clear();
      return NNC_OK;
    case NNC_OPT_PREFILL_BLOCK:
      if (value != 0 && (value < 128 || value % 128)) return fail(NNC_E_ARG, "prefill block must be 0 (largest) or a multiple of 128");
      m->opt_prefill_block = (uint32_t)value;
      return NNC_OK;
    case NNC_OPT_PREFILL_ATTN:
      if (value < -1 || value > 3) return fail(NNC_E_ARG, "prefill attention shape must be -1 (automatic) or 0 .. 3");
      m->opt_prefill_attn = value;
      return NNC_OK;
    case NNC_OPT_FUSE_QK:
      m->opt_fuse_qk = value != 0;
      // captured decode graphs contain one or the other set of kernels
      for (auto& kv : m->graphs) (void)hipGraphExecDestroy(kv.second);
      m->graphs.clear();
      return NNC_OK;
    case NNC_OPT_FUSE_NORM:
      m->opt_fuse_norm = value != 0;
      for (auto& kv : m->graphs) (void)hipGraphExecDestroy(kv.second);
      m->graphs.clear();
      return NNC_OK;
    case NNC_OPT_DECODE_PIECES:
      if (value != 0 && value != 2 && value != 3) return fail(NNC_E_ARG, "decode pieces must be 0 (default), 2 or 3");
      m->opt_decode_pieces = value;
      return NNC_OK;
    case NNC_OPT_SPIN_LIMIT:
      if (value < 0) return fail(NNC_E_ARG, "spin limit must be >= 0");
      m->mk_spin_limit = (unsigned)value;
      return NNC_OK;
    case NNC_OPT_STAGE_TRACE:
      if (!m->mk_ok) return fail(NNC_E_STATE, "the resident decode kernel is not available for this model");
      m->mk_trace_step = value - 1;
      return NNC_OK;
  }
  return fail(NNC_E_ARG, "unknown option %d", (int)opt);
}

// Prompt pass over one block of up to pb_max tokens of one slot with the LDS-staged
// matrix-core GEMMs.  Activations entering a GEMM are rounded to bf16 once.
static nnc_status prefill_block(nnc_model* m, uint32_t slot, const int32_t* tokens, uint32_t n, uint32_t pos0,
                                bool want_head, float* logits_out, int32_t* next_dev) {
  const nnc_config& c = m->c;
  hipStream_t s = m->stream;
  const int H = m->H(), Dq = m->Dq(), Dkv = m->Dkv(), F = m->F(), V = m->V();
  const int nq = c.n_q_heads, nkv = c.n_kv_heads, Nqkv = Dq + 2 * Dkv;
  const bool f16 = m->dt == NNC_F16;
  const int tt = (int)((n + 15) / 16);  // token tiles; rows up to 16 * tt exist in every buffer
  // Short prompts are bound by streaming the weights, not by the matrix cores: carry the
  // activations as two bf16 pieces (fp32-grade) and use small row tiles for more workgroups.
  // Long prompts are matrix-core bound: one bf16 per activation, 256-row tiles.
  const int pieces = (n <= 512 || m->opt_prefill_exact == 2) ? 2 : 1;
  const int ct = tt * pieces;  // operand column tiles
  // Block tile per GEMM.  Two workgroups fit on a CU and a launch runs in rounds of 2 x CUs of
  // them: of 256 / 192 / 128 x 128 take the shape whose last round is fullest (larger tiles do
  // a little more per byte of LDS traffic, hence the weights); 64 x 128, or 64 x 64 when even
  // those are fewer than the CUs, for launches that cannot give every CU a larger tile.
  const Machine mc = machine_mi355x(m->n_cus);
  auto tile_shape = [&](int n_tiles) {
    if (m->opt_prefill_tile >= 0) return m->opt_prefill_tile;
    const long cols = (ct + 7) / 8, slots = 2L * m->n_cus;
    const int nts[3] = {16, 12, 8}, codes[3] = {1, 4, 2};
    const double weight[3] = {1.0, 0.97, 0.93};
    int best = -1;
    double best_eff = 0.0;
    for (int i = 0; i < 3; ++i) {
      const long wgs = (long)((n_tiles + nts[i] - 1) / nts[i]) * cols;
      if (wgs < (long)m->n_cus) continue;
      const double eff = weight[i] * (double)wgs / (double)((wgs + slots - 1) / slots * slots);
      if (eff > best_eff) best_eff = eff, best = codes[i];
    }
    if (best >= 0) return best;
    if ((long)((n_tiles + 3) / 4) * cols >= (long)m->n_cus) return 0;
    return 3;
  };
  // k slices of a residual projection under the fixed rules (planner off, or a forced tile without
  // a forced slice count): only with the 64-row tiles, when the launch would leave most CUs without
  // a workgroup, and with at least 8 k steps per slice
  const long part_stride = (long)m->pb_max * H;
  auto resid_split = [&](PrefillGemmArgs& a, int shape) {
    if ((shape != 0 && shape != 3) || n > PB_SPLIT_TOKENS) return 0;
    const long wgs = (long)((a.n_tiles + 3) / 4) * ((ct + (shape == 3 ? 3 : 7)) / (shape == 3 ? 4 : 8));
    int ks = (int)std::min<long>(PB_SPLIT_MAX, m->n_cus / (wgs > 0 ? wgs : 1));
    ks = std::min(ks, a.KT / 8);
    if (ks < 2) return 0;
    a.kts_per_split = (a.KT + ks - 1) / ks;
    a.part = m->pb_part;
    a.part_stride = part_stride;
    return (a.KT + a.kts_per_split - 1) / a.kts_per_split - 1;  // partial buffers to fold later
  };
  // Block tile and k slices of one prompt GEMM: from the analytic model, unless a tile is
  // forced or the planner is switched off (then the two rules above).  Returns the tile; sets
  // the k split in `a` and the number of partial buffers the next norm kernel has to fold.
  auto plan_gemm = [&](PrefillGemmArgs& a, int epi, int* pend) {
    if (pend) *pend = 0;
    if (!m->opt_planner || m->opt_prefill_tile >= 0) {
      const int shape = tile_shape(a.n_tiles);
      if (m->opt_prefill_kslices > 0 && m->opt_prefill_tile >= 0) {
        // forced slice count of the residual projections (every tile's kernel takes one)
        const int ks = std::min(m->opt_prefill_kslices, a.KT);
        if (epi == EPI_RESID && ks > 1) {
          a.kts_per_split = (a.KT + ks - 1) / ks;
          a.part = m->pb_part;
          a.part_stride = part_stride;
          if (pend) *pend = (a.KT + a.kts_per_split - 1) / a.kts_per_split - 1;
        }
        return shape;
      }
      if (pend) *pend = resid_split(a, shape);
      return shape;
    }
    const int max_ks = epi == EPI_RESID ? PB_SPLIT_MAX : 1;
    const PrefillGemmPlan pl = plan_prefill_gemm(mc, a.n_tiles, a.KT, ct, (int)n, pieces, epi, max_ks);
    if (pl.k_slices > 1) {
      a.kts_per_split = pl.kts_per_split;
      a.part = m->pb_part;
      a.part_stride = part_stride;
      if (pend) *pend = pl.k_slices - 1;
    }
    return pl.tile;
  };
  int pending = 0;  // partial buffers of the previous projection still to be added to pb_x
  const double w = 2.0, T = n;
  // byte-weight models: the GEMM's matrix is widened to bf16 tiles in a scratch buffer (exact), and
  // the GEMM's epilogue applies the row scales
  auto weights_of = [&](PrefillGemmArgs& a, const void* Wp, const float* scale, int rows, int K) -> nnc_status {
    a.Wp = Wp;
    if (m->w8) {
      RUN(FAM_MISC, (double)rows * K * 3.0, 0, launch_widen_w8(s, Wp, m->pb_w, rows / 16, K / 64));
      a.Wp = m->pb_w;
      a.wscale = scale;
    }
    return NNC_OK;
  };
  HIP_TRY(hipMemcpyAsync(m->pb_tok, tokens, (size_t)n * 4, hipMemcpyHostToDevice, s));
  RUN(FAM_EMBED, T * H * w, 0, launch_embed_rows(s, f16, m->embed, H, m->pb_tok, (int)n, m->pb_x));
  for (uint32_t li = 0; li < c.n_layers; ++li) {
    const LayerW& L = m->L[li];
    RUN(FAM_NORM, T * H * 6.0, 0, launch_rmsnorm_frag(s, f16, m->pb_x, m->pb_part, pending, part_stride, L.g_in, H, c.rms_eps, (int)n, tt, pieces, m->pb_fa));
    {
      PrefillGemmArgs a{};
      if (nnc_status st_ = weights_of(a, L.wqkv, L.sqkv, Nqkv, H)) return st_;
      a.n_tiles = Nqkv / 16; a.KT = H / 32; a.Xf = m->pb_fa; a.t_tiles = ct;
      a.out = m->pb_qkv; a.ldo = Nqkv;
      RUN(FAM_PGEMM, (double)Nqkv * H * w, 2.0 * Nqkv * H * T, launch_gemm_prefill(s, f16, EPI_STORE, a, pieces, plan_gemm(a, EPI_STORE, nullptr)));
    }
    {
      const ColMap cm{nullptr, slot, pos0, 0};
      RUN(FAM_QKROPE, T * Nqkv * 4.0, 0,
          launch_qknorm_rope_append(s, m->dt, m->pb_qkv, nq, nkv, L.g_q, L.g_k, c.rms_eps, m->rope, cm, (int)n, L.kc,
                                    L.vc, c.max_batch, c.max_seq, nullptr, m->pb_vt, m->pb_vt_stride));
      if (m->record_layers) HIP_TRY(hipEventRecord(m->layer_done[li], s));
    }
    {
      // causal attention of the block on the matrix cores, over a transposed copy of the
      // slot's V rows (positions of earlier blocks included)
      double rows = 0;
      for (uint32_t i = 0; i < n; ++i) rows += pos0 + i + 1.0;
      // the block's own V rows were written transposed by the append kernel; rows of earlier
      // blocks come from the cache
      if (pos0 > 0)
        RUN(FAM_MISC, pos0 * Dkv * 2.0 * w, 0,
            launch_v_transpose(s, L.vc, slot, nkv, c.max_seq, pos0, m->pb_vt, m->pb_vt_stride));
      RUN(FAM_PATTN, (pos0 + T) * 2.0 * Dkv * w + T * Dq * 6.0, rows * 4.0 * Dq,
          launch_attn_prefill(s, f16, m->pb_qkv, nq, nkv, L.kc, m->pb_vt, m->pb_vt_stride, slot, c.max_seq, pos0, (int)n,
                              pieces, m->pb_fb, m->n_cus, m->opt_prefill_attn));
    }
    {
      PrefillGemmArgs a{};
      if (nnc_status st_ = weights_of(a, L.wo, L.so, H, Dq)) return st_;
      a.n_tiles = H / 16; a.KT = Dq / 32; a.Xf = m->pb_fb; a.t_tiles = ct;
      a.out = m->pb_x; a.ldo = H;
      const int shape = plan_gemm(a, EPI_RESID, &pending);
      RUN(FAM_PGEMM_O, (double)H * Dq * w, 2.0 * H * Dq * T, launch_gemm_prefill(s, f16, EPI_RESID, a, pieces, shape));
    }
    RUN(FAM_NORM, T * H * 6.0, 0, launch_rmsnorm_frag(s, f16, m->pb_x, m->pb_part, pending, part_stride, L.g_post, H, c.rms_eps, (int)n, tt, pieces, m->pb_fa));
    {
      PrefillGemmArgs a{};
      if (nnc_status st_ = weights_of(a, L.wgu, L.sgu, 2 * F, H)) return st_;
      a.n_tiles = 2 * F / 16; a.KT = H / 32; a.Xf = m->pb_fa; a.t_tiles = ct;
      a.packed_out = m->pb_fb;
      RUN(FAM_PGEMM_GU, 2.0 * F * H * w, 4.0 * F * H * T, launch_gemm_prefill(s, f16, EPI_SWIGLU, a, pieces, plan_gemm(a, EPI_SWIGLU, nullptr)));
    }
    {
      PrefillGemmArgs a{};
      if (nnc_status st_ = weights_of(a, L.wd, L.sd, H, F)) return st_;
      a.n_tiles = H / 16; a.KT = F / 32; a.Xf = m->pb_fb; a.t_tiles = ct;
      a.out = m->pb_x; a.ldo = H;
      const int shape = plan_gemm(a, EPI_RESID, &pending);
      RUN(FAM_PGEMM_D, (double)H * F * w, 2.0 * H * F * T, launch_gemm_prefill(s, f16, EPI_RESID, a, pieces, shape));
    }
  }
  if (want_head) {
    // logits of the block's last token: fp32-grade (three-piece) GEMV over the LM head
    RUN(FAM_NORM, H * 8.0, 0,
        launch_rmsnorm_pack(s, m->dt, m->pb_x + (size_t)(n - 1) * H, H, m->pb_part + (size_t)(n - 1) * H, pending,
                            part_stride, m->g_final, H, c.rms_eps, 1, m->Xp, 3, 3));
    GemmArgs a{};
    a.Wp = m->lm_head; a.n_tiles = V / 16; a.KT = H / 32; a.kts_per_split = H / 32;
    a.Xp = m->Xp; a.NC = 3; a.ncols = 3; a.nsplit = 3; a.nseq = 1;
    a.out = logits_out ? logits_out : m->logits; a.ldo = V;
    RUN(FAM_GEMM_HEAD, (double)V * H * w, 2.0 * V * H, launch_gemm(s, m->dt, EPI_STORE, a));
    if (next_dev)
      RUN(FAM_ARGMAX, V * 4.0, 0, launch_argmax(s, a.out, V, V, 1, nullptr, 0, m->am_val, m->am_idx, next_dev));
  }
  return NNC_OK;
}

// Second stream and per-layer events for the tail of a long prompt; false if they cannot be had
// (the tail then follows the last block on the model's stream).
static bool ensure_tail_stream(nnc_model* m) {
  if (m->tail_stream) return true;
  hipStream_t st = nullptr;
  if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) return false;
  std::vector<hipEvent_t> ev(m->c.n_layers + 2, nullptr);
  for (auto& e : ev)
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
      for (hipEvent_t d : ev)
        if (d) (void)hipEventDestroy(d);
      (void)hipStreamDestroy(st);
      return false;
    }
  m->tail_stream = st;
  m->layer_done = ev;
  return true;
}

// While alive, the model's passes are enqueued on the tail stream and wait, layer by layer, for
// the last block's cache appends.
struct TailStreamScope {
  nnc_model* m;
  hipStream_t main;
  bool on;
  TailStreamScope(nnc_model* m_, bool on_) : m(m_), main(m_->stream), on(on_) {
    if (on) {
      m->stream = m->tail_stream;
      m->wait_layers = true;
    }
  }
  ~TailStreamScope() {
    if (on) {
      m->stream = main;
      m->wait_layers = false;
    }
  }
};

static nnc_status prefill_common(nnc_model* m, uint32_t slot, const int32_t* tokens, const float* x, uint32_t n,
                                 float* logits_out, int32_t* next_out, float* y) {
  if (slot >= m->c.max_batch) return fail(NNC_E_ARG, "slot %u out of range", slot);
  if (n == 0) return fail(NNC_E_ARG, "n is 0");
  if ((uint64_t)m->len[slot] + n > m->c.max_seq)
    return fail(NNC_E_KV_FULL, "slot %u: length %u + %u exceeds max_seq %u", slot, m->len[slot], n, m->c.max_seq);
  if (tokens)
    for (uint32_t i = 0; i < n; ++i)
      if (tokens[i] < 0 || (uint32_t)tokens[i] >= m->c.vocab) return fail(NNC_E_ARG, "token %d out of range", tokens[i]);
  uint32_t done = 0;  // tokens already processed by the large-block path
  bool overlap = false;
  if (tokens && m->pb_max && m->opt_prefill_exact != 1) {
    const uint32_t len0 = m->len[slot];
    // Blocks of up to pb_max tokens (NNC_OPT_PREFILL_BLOCK may ask for less).  A block of more than 512 tokens rounds its matrix-core
    // inputs to bf16 once; that noise must not reach the logits directly, so the last
    // PREFILL_TAIL tokens of a longer prompt (the last of which yields the logits) go through
    // the fp32-grade chunk path below instead: one more pass over the weights, about the cost
    // of one decode step.
    uint32_t head = n;
    if (m->opt_prefill_exact == 0 && n > 512) head = n - PREFILL_TAIL;
    // The tail pass streams every weight once more at a few percent of the matrix cores' rate,
    // the last block is bound by the matrix cores: the two run side by side, the tail's layer l
    // starting when the block's layer l has appended its K / V rows.
    overlap = head < n && m->opt_tail_overlap && !m->profiling && ensure_tail_stream(m);
    for (uint32_t t0 = 0; t0 < head;) {
      const uint32_t blk = m->opt_prefill_block ? std::min(m->opt_prefill_block, m->pb_max) : m->pb_max;
      const uint32_t nb = std::min(blk, head - t0);
      const bool last = t0 + nb == n;
      const bool fork = overlap && t0 + nb == head;
      if (fork) {
        HIP_TRY(hipEventRecord(m->layer_done[m->c.n_layers], m->stream));  // everything enqueued so far
        m->record_layers = true;
      }
      const nnc_status st = prefill_block(m, slot, tokens + t0, nb, len0 + t0, last && (logits_out || next_out),
                                          logits_out, next_out ? m->next : nullptr);
      m->record_layers = false;
      if (st) return st;
      t0 += nb;
    }
    if (head == n) {
      if (next_out) HIP_TRY(hipMemcpyAsync(next_out, m->next, 4, hipMemcpyDeviceToDevice, m->stream));
      m->len[slot] = len0 + n;
      return NNC_OK;
    }
    done = head;
  }
  const int nsplit = m->f32 ? 1 : 3;
  const uint32_t chunk = MAX_COLS / nsplit;
  const size_t H = m->H();
  const uint32_t len0 = m->len[slot];
  hipStream_t main_stream = m->stream;
  if (overlap) HIP_TRY(hipStreamWaitEvent(m->tail_stream, m->layer_done[m->c.n_layers], 0));
  {
  TailStreamScope scope(m, overlap);
  for (uint32_t t0 = done; t0 < n; t0 += chunk) {
    const uint32_t nc = std::min(chunk, n - t0);
    uint32_t slots[MAX_COLS], pos[MAX_COLS];
    for (uint32_t i = 0; i < nc; ++i) {
      slots[i] = slot;
      pos[i] = len0 + t0 + i;
    }
    HIP_TRY(launch_set_state(m->stream, m->st, (int)nc, tokens ? tokens + t0 : nullptr, slots, pos, 0));
    Pass p;
    p.ncols = (int)nc;
    p.nsplit = nsplit;
    p.tokens = tokens != nullptr;
    p.grid_chunks = chunks_grid(pos[nc - 1]);
    p.one_slot = true;
    for (uint32_t i = 0; i < nc; ++i) p.kv_rows += pos[i] + 1.0;
    const bool last = t0 + nc == n;
    if (!tokens)
      HIP_TRY(launch_copy_rows(m->stream, x + (size_t)t0 * H, m->x, (size_t)nc * H));
    if (last && tokens && (logits_out || next_out)) {
      p.head_col0 = (int)nc - 1;
      p.head_ncols = 1;
      p.logits = logits_out ? logits_out : m->logits;
      p.logits_ld = m->V();
      p.next = next_out ? m->next : nullptr;
    }
    if (nnc_status st = run_pass(m, p)) return st;
    if (!tokens) HIP_TRY(launch_copy_rows(m->stream, m->x, y + (size_t)t0 * H, (size_t)nc * H));
    if (last && next_out && tokens)
      HIP_TRY(hipMemcpyAsync(next_out, m->next, 4, hipMemcpyDeviceToDevice, m->stream));
  }
  }
  if (overlap) {  // the model's stream continues after the tail
    HIP_TRY(hipEventRecord(m->layer_done[m->c.n_layers + 1], m->tail_stream));
    HIP_TRY(hipStreamWaitEvent(main_stream, m->layer_done[m->c.n_layers + 1], 0));
  }
  m->len[slot] = len0 + n;
  return NNC_OK;
}

nnc_status nnc_prefill(nnc_model* m, uint32_t slot, const int32_t* tokens, uint32_t n, float* logits_out,
                       int32_t* next_out) {
  if (!m || !tokens) return fail(NNC_E_ARG, "NULL argument");
  if (!m->c.has_embed_and_head) return fail(NNC_E_STATE, "model has no embedding; use nnc_prefill_hidden");
  if (resident_failed(m, false))
    return fail(NNC_E_DEVICE, "an earlier decode launch gave up waiting for its other workgroups; recreate the model");
  return prefill_common(m, slot, tokens, nullptr, n, logits_out, next_out, nullptr);
}

nnc_status nnc_prefill_hidden(nnc_model* m, uint32_t slot, const float* x, uint32_t n, float* y) {
  if (!m || !x || !y) return fail(NNC_E_ARG, "NULL argument");
  if (m->c.has_embed_and_head) return fail(NNC_E_STATE, "model takes tokens; use nnc_prefill");
  return prefill_common(m, slot, nullptr, x, n, nullptr, nullptr, y);
}

nnc_status nnc_decode_step(nnc_model* m, const uint32_t* slots, const int32_t* tokens, uint32_t batch,
                           float* logits_out, int32_t* next_out) {
  if (!m || !tokens) return fail(NNC_E_ARG, "NULL argument");
  if (!m->c.has_embed_and_head) return fail(NNC_E_STATE, "model has no embedding; use nnc_decode_step_hidden");
  if (resident_failed(m, false))
    return fail(NNC_E_DEVICE, "an earlier decode launch gave up waiting for its other workgroups; recreate the model");
  if (nnc_status st = check_slots(m, slots, batch, 1)) return st;
  for (uint32_t i = 0; i < batch; ++i)
    if (tokens[i] < 0 || (uint32_t)tokens[i] >= m->c.vocab) return fail(NNC_E_ARG, "token %d out of range", tokens[i]);
  uint32_t max_pos = 0;
  double kv_rows = 0;
  if (nnc_status st = set_decode_state(m, slots, tokens, batch, &max_pos, &kv_rows)) return st;
  const int nsplit = decode_nsplit(m, batch);
  if (use_persistent(m, batch)) {
    if (nnc_status st = persistent_steps(m, slots[0], tokens[0], 1, logits_out)) return st;
    if (next_out) HIP_TRY(hipMemcpyAsync(next_out, m->token_log, batch * 4, hipMemcpyDeviceToDevice, m->stream));
    for (uint32_t i = 0; i < batch; ++i) m->len[slots[i]] += 1;
    return NNC_OK;
  }
  if (logits_out) {
    Pass p;
    p.decode = true;
    p.ncols = (int)batch;
    p.nsplit = nsplit;
    p.head_ncols = (int)batch;
    p.logits = logits_out;
    p.logits_ld = m->V();
    p.next = next_out ? m->next : nullptr;
    p.grid_chunks = chunks_grid(max_pos);
    p.kv_rows = kv_rows;
    if (nnc_status st = run_pass(m, p)) return st;
  } else {
    if (nnc_status st = greedy_step(m, batch, nsplit, chunks_grid(max_pos), true, kv_rows)) return st;
  }
  if (next_out) HIP_TRY(hipMemcpyAsync(next_out, m->next, batch * 4, hipMemcpyDeviceToDevice, m->stream));
  for (uint32_t i = 0; i < batch; ++i) m->len[slots[i]] += 1;
  return fetch_wait_flag(m);
}

// ---- decode step for callers that cannot allocate -------------------------------
// The workspace of the pass (column state, residual stream, projection outputs, packed operands,
// k-slice partials, attention partials, logits, arg-max partials) lives in one file-scope
// device array instead of buffers obtained at create.  Host code never uses the array's name
// as an address: the per-device address comes from hipGetSymbolAddress, once per device.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)NNC_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {};  // this device's copy of `scratch`, by device ordinal

// Workspace pointers of the model while a pass runs out of the static array; restored on exit.
struct WorkspaceSwap {
  nnc_model* m;
  ColState* st; float *x, *qkv, *rpart, *partial, *logits, *am_val; void *Xp, *Ap, *qsplit;
  int32_t *am_idx, *next; int max_chunks;
  explicit WorkspaceSwap(nnc_model* m_)
      : m(m_), st(m_->st), x(m_->x), qkv(m_->qkv), rpart(m_->rpart), partial(m_->partial), logits(m_->logits),
        am_val(m_->am_val), Xp(m_->Xp), Ap(m_->Ap), qsplit(m_->qsplit), am_idx(m_->am_idx), next(m_->next),
        max_chunks(m_->max_chunks) {}
  ~WorkspaceSwap() {
    m->st = st; m->x = x; m->qkv = qkv; m->rpart = rpart; m->partial = partial; m->logits = logits;
    m->am_val = am_val; m->Xp = Xp; m->Ap = Ap; m->qsplit = qsplit; m->am_idx = am_idx; m->next = next;
    m->max_chunks = max_chunks;
  }
};
}  // namespace

nnc_status nnc_decode_step_static(nnc_model* m, const uint32_t* slots, const int32_t* tokens, uint32_t batch,
                                  float* logits_out, int32_t* next_out) {
  if (!m || !tokens) return fail(NNC_E_ARG, "NULL argument");
  if (!m->c.has_embed_and_head) return fail(NNC_E_STATE, "model has no embedding");
  if (m->profiling) return fail(NNC_E_STATE, "per-kernel profiling creates events; not available here");
  if (resident_failed(m, false))
    return fail(NNC_E_DEVICE, "an earlier decode launch gave up waiting for its other workgroups; recreate the model");
  if (batch > NNC_STATIC_MAX_BATCH)
    return fail(NNC_E_ARG, "batch %u exceeds the static workspace limit of %d sequences", batch, NNC_STATIC_MAX_BATCH);
  if (nnc_status st = check_slots(m, slots, batch, 1)) return st;
  for (uint32_t i = 0; i < batch; ++i)
    if (tokens[i] < 0 || (uint32_t)tokens[i] >= m->c.vocab) return fail(NNC_E_ARG, "token %d out of range", tokens[i]);
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != m->device) return fail(NNC_E_STATE, "the model lives on device %d, the current device is %d", m->device, dev);
  if (dev < 0 || dev >= MAX_DEVICES) return fail(NNC_E_DEVICE, "device ordinal %d not supported", dev);

  // carve the workspace; sizes follow this call's batch and longest context, not max_seq
  uint32_t max_pos = 0;
  for (uint32_t i = 0; i < batch; ++i) max_pos = std::max(max_pos, m->len[slots[i]]);
  const int nsplit = decode_nsplit(m, batch), grid_chunks = chunks_grid(max_pos);
  const size_t H = m->H(), Dq = m->Dq(), Dkv = m->Dkv(), F = m->F(), V = m->V(), w = m->esz(), B = batch;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + 255) / 256 * 256;
    return at;
  };
  const size_t o_st = take(sizeof(ColState)), o_x = take(B * H * 4), o_qkv = take((size_t)MAX_QKV_SLICES * B * (Dq + 2 * Dkv) * 4),
               o_Xp = take(B * nsplit * H * w), o_Ap = take(B * nsplit * std::max(Dq, F) * w),
               o_rpart = take((size_t)MAX_KSPLIT * B * H * 4),
               o_partial = take(B * m->c.n_q_heads * (size_t)grid_chunks * 132 * 4),
               o_qsplit = take(B * m->c.n_q_heads * 3 * 128 * 2), o_next = take(B * 4), o_amv = take(B * 64 * 4),
               o_ami = take(B * 64 * 4), o_logits = logits_out ? 0 : take(B * V * 4);
  if (off > STATIC_SCRATCH_BYTES)
    return fail(NNC_E_ARG, "this step needs %zu bytes of workspace (batch %u, context %u); the static workspace holds %zu",
                off, batch, max_pos + 1, STATIC_SCRATCH_BYTES);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(NNC_E_DEVICE, "hipGetSymbolAddress returned NULL");
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  unsigned char* base = g_scratch_ptr[dev];

  WorkspaceSwap keep(m);
  m->st = reinterpret_cast<ColState*>(base + o_st);
  m->x = reinterpret_cast<float*>(base + o_x);
  m->qkv = reinterpret_cast<float*>(base + o_qkv);
  m->Xp = base + o_Xp;
  m->Ap = base + o_Ap;
  m->rpart = reinterpret_cast<float*>(base + o_rpart);
  m->partial = reinterpret_cast<float*>(base + o_partial);
  m->max_chunks = grid_chunks;  // row stride of the partial records
  m->qsplit = base + o_qsplit;
  m->next = reinterpret_cast<int32_t*>(base + o_next);
  m->am_val = reinterpret_cast<float*>(base + o_amv);
  m->am_idx = reinterpret_cast<int32_t*>(base + o_ami);

  double kv_rows = 0;
  if (nnc_status st = set_decode_state(m, slots, tokens, batch, &max_pos, &kv_rows)) return st;
  Pass p;
  p.decode = true;
  p.ncols = (int)batch;
  p.nsplit = nsplit;
  p.head_ncols = (int)batch;
  p.logits = logits_out ? logits_out : reinterpret_cast<float*>(base + o_logits);
  p.logits_ld = (long)V;
  p.next = next_out ? m->next : nullptr;
  p.grid_chunks = grid_chunks;
  p.kv_rows = kv_rows;
  if (nnc_status st = run_pass(m, p)) return st;
  if (next_out) HIP_TRY(hipMemcpyAsync(next_out, m->next, batch * 4, hipMemcpyDeviceToDevice, m->stream));
  for (uint32_t i = 0; i < batch; ++i) m->len[slots[i]] += 1;
  return fetch_wait_flag(m);
}

nnc_status nnc_decode_greedy(nnc_model* m, const uint32_t* slots, const int32_t* first_tokens, uint32_t batch,
                             uint32_t n_steps, int32_t* tokens_out, float* logits_out) {
  if (!m || !first_tokens || !tokens_out) return fail(NNC_E_ARG, "NULL argument");
  if (!m->c.has_embed_and_head) return fail(NNC_E_STATE, "model has no embedding");
  if (resident_failed(m, false))
    return fail(NNC_E_DEVICE, "an earlier decode launch gave up waiting for its other workgroups; recreate the model");
  if (n_steps == 0) return fail(NNC_E_ARG, "n_steps is 0");
  if (n_steps > m->token_log_steps) return fail(NNC_E_ARG, "n_steps %u exceeds %u", n_steps, m->token_log_steps);
  if (nnc_status st = check_slots(m, slots, batch, n_steps)) return st;
  for (uint32_t i = 0; i < batch; ++i)
    if (first_tokens[i] < 0 || (uint32_t)first_tokens[i] >= m->c.vocab)
      return fail(NNC_E_ARG, "token %d out of range", first_tokens[i]);
  uint32_t max_pos = 0;
  double kv_rows = 0;
  if (nnc_status st = set_decode_state(m, slots, first_tokens, batch, &max_pos, &kv_rows)) return st;
  const int nsplit = decode_nsplit(m, batch);
  if (use_persistent(m, batch)) {
    if (nnc_status st = persistent_steps(m, slots[0], first_tokens[0], n_steps, logits_out)) return st;
    HIP_TRY(hipMemcpyAsync(tokens_out, m->token_log, (size_t)n_steps * batch * 4, hipMemcpyDeviceToDevice, m->stream));
    for (uint32_t i = 0; i < batch; ++i) m->len[slots[i]] += n_steps;
    return NNC_OK;
  }
  for (uint32_t step = 0; step < n_steps; ++step) {
    const int gc = chunks_grid(max_pos + step);
    if (logits_out) {
      Pass p;
      p.decode = true;
      p.ncols = (int)batch;
      p.nsplit = nsplit;
      p.head_ncols = (int)batch;
      p.logits = logits_out + (size_t)step * batch * m->V();
      p.logits_ld = m->V();
      p.next = m->next;
      p.grid_chunks = gc;
      p.kv_rows = kv_rows + (double)step * batch;
      if (nnc_status st = run_pass(m, p)) return st;
      HIP_TRY(launch_finish_step(m->stream, m->st, (int)batch, m->next, m->token_log));
    } else {
      if (nnc_status st = greedy_step(m, batch, nsplit, gc, true, kv_rows + (double)step * batch)) return st;
    }
  }
  HIP_TRY(hipMemcpyAsync(tokens_out, m->token_log, (size_t)n_steps * batch * 4, hipMemcpyDeviceToDevice, m->stream));
  for (uint32_t i = 0; i < batch; ++i) m->len[slots[i]] += n_steps;
  return fetch_wait_flag(m);
}

nnc_status nnc_decode_step_hidden(nnc_model* m, const uint32_t* slots, const float* x, uint32_t batch, float* y) {
  if (!m || !x || !y) return fail(NNC_E_ARG, "NULL argument");
  if (m->c.has_embed_and_head) return fail(NNC_E_STATE, "model takes tokens; use nnc_decode_step");
  if (nnc_status st = check_slots(m, slots, batch, 1)) return st;
  uint32_t max_pos = 0;
  double kv_rows = 0;
  if (nnc_status st = set_decode_state(m, slots, nullptr, batch, &max_pos, &kv_rows)) return st;
  HIP_TRY(launch_copy_rows(m->stream, x, m->x, (size_t)batch * m->H()));
  Pass p;
  p.decode = true;
  p.kv_rows = kv_rows;
  p.ncols = (int)batch;
  p.nsplit = decode_nsplit(m, batch);
  p.tokens = false;
  p.grid_chunks = chunks_grid(max_pos);
  if (nnc_status st = run_pass(m, p)) return st;
  HIP_TRY(launch_copy_rows(m->stream, m->x, y, (size_t)batch * m->H()));
  for (uint32_t i = 0; i < batch; ++i) m->len[slots[i]] += 1;
  return fetch_wait_flag(m);
}

nnc_status nnc_kv_read(nnc_model* m, uint32_t layer, uint32_t slot, uint32_t which, uint32_t pos0, uint32_t n,
                       float* out) {
  if (!m || !out) return fail(NNC_E_ARG, "NULL argument");
  if (layer >= m->c.n_layers || slot >= m->c.max_batch || which > 1 || n == 0 ||
      (uint64_t)pos0 + n > m->len[slot])
    return fail(NNC_E_ARG, "kv_read range out of bounds");
  const size_t slot_elems = (size_t)m->c.n_kv_heads * m->c.max_seq * 128;
  const char* base = static_cast<const char*>(which ? m->L[layer].vc : m->L[layer].kc) + slot * slot_elems * m->esz();
  HIP_TRY(launch_kv_read(m->stream, m->dt, base, m->c.max_seq, (int)m->c.n_kv_heads, pos0, n, out));
  return NNC_OK;
}

nnc_status nnc_stage_trace(nnc_model* m, uint64_t* out, uint32_t cap, uint32_t* workgroups, uint32_t* points) {
  if (!m || !out || !workgroups || !points) return fail(NNC_E_ARG, "NULL argument");
  if (!m->mk_ok || m->mk_trace_step < 0) return fail(NNC_E_STATE, "stage tracing is off");
  const uint32_t np = (uint32_t)mk_trace_points((int)m->c.n_layers);
  if ((uint64_t)cap < (uint64_t)m->mk_nwg * np) return fail(NNC_E_ARG, "trace buffer too small");
  HIP_TRY(hipStreamSynchronize(m->stream));
  HIP_TRY(hipMemcpy(out, m->mk_trace, (size_t)m->mk_nwg * np * 8, hipMemcpyDeviceToHost));
  *workgroups = (uint32_t)m->mk_nwg;
  *points = np;
  return NNC_OK;
}

nnc_status nnc_plan_prefill_gemm_query(uint32_t rows, uint32_t k, uint32_t n_tokens, uint32_t pieces, uint32_t epilogue,
                                       uint32_t max_k_slices, uint32_t n_cus, nnc_gemm_plan* out) {
  if (!out) return fail(NNC_E_ARG, "out is NULL");
  if (!rows || rows % 16 || !k || k % 32 || !n_tokens || pieces < 1 || pieces > 2 || epilogue > 2 || !max_k_slices)
    return fail(NNC_E_ARG, "bad GEMM shape for the planner");
  const Machine mc = machine_mi355x((int)n_cus);
  const int ct = (int)((n_tokens + 15) / 16 * pieces);
  const PrefillGemmPlan p = plan_prefill_gemm(mc, (int)(rows / 16), (int)(k / 32), ct, (int)n_tokens, (int)pieces,
                                              (int)epilogue, (int)max_k_slices);
  nnc_gemm_plan o{};
  o.tile_rows = (uint32_t)p.nt * 16; o.tile_cols = (uint32_t)p.tt * 16; o.tile_code = p.tile;
  o.k_slices = (uint32_t)p.k_slices; o.workgroups = (uint32_t)p.workgroups;
  o.t_comp_us = p.t_comp_us; o.t_mem_us = p.t_mem_us; o.t_us = p.t_us;
  o.candidates = (uint32_t)p.candidates; o.rejected_by_capacity = (uint32_t)p.rejected_by_capacity;
  *out = o;
  return NNC_OK;
}

nnc_status nnc_plan_skinny_gemm_query(uint32_t rows, uint32_t k, uint32_t n_seq, uint32_t pieces, uint32_t epilogue,
                                      uint32_t max_k_slices, uint32_t n_cus, nnc_gemm_plan* out) {
  if (!out) return fail(NNC_E_ARG, "out is NULL");
  if (!rows || rows % 16 || !k || k % 32 || !n_seq || pieces < 1 || pieces > 3 || n_seq * pieces > (uint32_t)MAX_COLS ||
      epilogue > 2 || epilogue == 1 || !max_k_slices)
    return fail(NNC_E_ARG, "bad GEMM shape for the planner");
  const Machine mc = machine_mi355x((int)n_cus);
  const SkinnyGemmPlan p = plan_skinny_gemm(mc, (int)(rows / 16), (int)(k / 32), (int)(n_seq * pieces), (int)n_seq,
                                            skinny_rt_choices((int)NNC_BF16, (int)epilogue),
                                            (int)std::min<uint32_t>(max_k_slices, MAX_KSPLIT));
  nnc_gemm_plan o{};
  o.tile_rows = (uint32_t)p.rt * 16; o.tile_cols = n_seq * pieces; o.tile_code = p.rt;
  o.k_slices = (uint32_t)p.k_slices; o.workgroups = (uint32_t)p.workgroups;
  o.t_comp_us = p.t_operand_us; o.t_mem_us = p.t_mem_us; o.t_us = p.t_us;
  *out = o;
  return NNC_OK;
}

nnc_status nnc_profile_begin(nnc_model* m) {
  if (!m) return fail(NNC_E_ARG, "model is NULL");
  HIP_TRY(hipStreamSynchronize(m->stream));
  for (auto& r : m->prof) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  m->prof.clear();
  m->profiling = true;
  return NNC_OK;
}

nnc_status nnc_profile_end(nnc_model* m, nnc_kernel_stat* out, uint32_t cap, uint32_t* n_out) {
  if (!m || !n_out) return fail(NNC_E_ARG, "NULL argument");
  m->profiling = false;
  HIP_TRY(hipStreamSynchronize(m->stream));
  nnc_kernel_stat acc[FAM_COUNT];
  memset(acc, 0, sizeof acc);
  for (int f = 0; f < FAM_COUNT; ++f) snprintf(acc[f].name, sizeof acc[f].name, "%s", kFamName[f]);
  for (auto& r : m->prof) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
      acc[r.fam].launches += 1;
      acc[r.fam].total_ms += ms;
      acc[r.fam].bytes += r.bytes;
      acc[r.fam].flops += r.flops;
    }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  m->prof.clear();
  uint32_t k = 0;
  for (int f = 0; f < FAM_COUNT && k < cap; ++f)
    if (acc[f].launches && out) out[k++] = acc[f];
  *n_out = k;
  return NNC_OK;
}

}  // extern "C"
