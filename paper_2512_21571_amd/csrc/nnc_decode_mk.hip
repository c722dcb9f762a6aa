// Resident whole-step decode kernel for batch 1 (bf16 models).
//
// Batch-1 decode of a 0.6B-shaped model moves ~1.2 GB per token: 150 us at HBM
// speed, spread over ~140 dependent matmul / attention stages of about 1 us each.
// Run as separate kernels, every stage pays a launch-drain-launch bubble of several
// microseconds, and that is where the time goes.  The paper observes the same on
// CPUs: fork-join barriers of a threading runtime limit scaling, and a static
// partition with cheap, deterministic communication wins (Section 4.2,
// architectural discussion).  Here one resident grid (at most one workgroup per
// compute unit) runs all the decode steps of a call:
//
//   * every stage is statically partitioned over the workgroups;
//   * there are no grid barriers.  Whatever one workgroup produces for others is
//     written as 64-bit words (fp32 value, 32-bit tag) with relaxed agent-scope
//     atomic stores, which go to the memory side past the per-XCD L2s; the tag
//     names the (step, layer, stage) that produced it.  A consumer simply loads
//     the words it needs (relaxed agent-scope atomic loads) and repeats until
//     every tag is the one it expects.  Synchronisation and data transfer are
//     one and the same memory round trip (~1.7 us for an all-to-all of a hidden
//     vector among 256 workgroups, measured), and no cache write-back or
//     invalidate is ever issued (those cost ~10 us each on this part);
//   * the weights of a workgroup's next stage are loaded into registers while the
//     current stage finishes and the exchange is in flight;
//   * the residual stream never goes through memory: every workgroup keeps its own
//     copy in registers and adds the exchanged projection outputs to it.
//
// Why a producer may overwrite an exchange buffer without asking: each buffer is
// rewritten one layer later at the same stage, and before that can happen its
// readers have produced something the writer (transitively) waited for.  This
// needs every workgroup to own at least one QKV tile per layer, so the grid is
// min(compute units, QKV tiles).
//
// Weights, gains, the rotary table and cached K/V rows older than the current
// step are immutable during a launch and use ordinary loads.
#include <cstring>

#include "nnc_half.h"
#include "nnc_internal.h"
#include "nnc_lanes.h"

namespace nnc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Weights are read once per step: a streaming (non-temporal) load keeps them from displacing
// the operands and exchange words that every workgroup re-reads from L2.
__device__ __forceinline__ uint4 ldw(const uint4* p) {
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return uint4{t.x, t.y, t.z, t.w};
}
typedef unsigned long long u64;

namespace {

// One wave per SIMD: each wave may then use the whole 512-entry register file, which holds the
// prefetched weights of the next stage (64 KiB per workgroup) without any spilling.
constexpr int MK_THREADS = 256;
constexpr int MK_WAVES = MK_THREADS / 64;
constexpr unsigned MK_SPIN_MAX = 1u << 20;
constexpr int MK_PF = 8;      // prefetched 16-byte weight loads per lane and 16-row tile (32 KiB per workgroup)
constexpr int MK_MAX_KS = 4;  // k slices of a narrow projection
constexpr int MK_DIRECT_MERGE_MAX = 4;  // attention chunks up to which every output-projection unit merges by itself

// ---- memory-side accesses ----------------------------------------------------
__device__ __forceinline__ unsigned ld_u32(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_u32(unsigned* p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 ld_t(const u64* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_t(u64* p, float v, unsigned tag) {
  __hip_atomic_store(p, (u64)__float_as_uint(v) | ((u64)tag << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float t_val(u64 w) { return __uint_as_float((unsigned)w); }
__device__ __forceinline__ bool t_ok(u64 w, unsigned tag) { return (unsigned)(w >> 32) == tag; }

// Returns v, but the compiler must assume it changed.  Used on lane / thread indices at the
// top of each stage helper so that the dozens of per-load address offsets are recomputed
// where they are used instead of being hoisted out of the layer loop, where they would
// occupy (and spill) registers that the in-flight weight prefetch needs.
__device__ __forceinline__ int opaque(int v) {
  asm volatile("" : "+v"(v));
  return v;
}

// Workgroup barrier that orders LDS traffic only: outstanding global loads (the
// weight prefetch) stay in flight across it.
__device__ __forceinline__ void wg_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

}  // namespace

struct MkLayer {
  const uint4 *wqkv, *wo, *wgu, *wd;
  const float *g_in, *g_q, *g_k, *g_post;
  uint16_t *kc, *vc;
};

struct MkArgs {
  const MkLayer* layers;
  int n_layers, H, nq, nkv, F, V;
  float eps;
  const uint4* embed;
  const uint4* lm_head;
  const float* g_final;
  const float2* rope;
  uint32_t max_seq;
  unsigned* error;
  unsigned spin_max;    // polls of one wait before the launch gives up
  int tok0;             // first token
  uint32_t pos0, slot;  // position of the first step, KV slot
  int n_steps;
  unsigned tag_base;
  int ks_o, ks_d;  // k slices of the output / down projections
  // Unit u of a stage runs on workgroup (u + offset) % workgroups.  The offsets keep the
  // few-unit stages (attention, output projection, down projection) on different
  // workgroups, so that a workgroup's weight prefetch for its next role is issued early.
  int off_att, off_o, off_d;
  // exchange buffers of (value, tag) words
  u64* xq;    // [Dq + 2 Dkv] raw q | k | v
  u64* xatt;  // [nq][max_chunks][132] attention partials: 128 sums, max, sum
  int max_chunks;
  u64* xo;    // [Dq] merged attention output (used when the context spans many chunks)
  u64* xop;   // [ks_o][H]
  u64* xact;  // [F]
  u64* xdp;   // [ks_d][H]
  u64* xamv;  // [workgroups] best logit
  u64* xami;  // [workgroups] its index
  float* logits;       // [n_steps][V] or NULL
  int32_t* token_log;  // [n_steps]
  unsigned long long* trace;  // [workgroups][trace_points] wall-clock stamps of one step, or NULL
  int trace_step, trace_points;
};

namespace {

constexpr int MK_VS = 66;  // row stride of the staged V chunk in 32-bit words (128 bf16 + pad: conflict-free gathers)

struct Smem {
  union {
    float red[MK_WAVES][2][256];          // GEMM: per-wave accumulator tiles
    uint32_t Vs[ATT_CHUNK][MK_VS];        // attention: the chunk's V rows, two bf16 per word
    float mrg[MK_WAVES][128];             // merge stage: per-wave weighted sums of one head
  };
  float wsum[MK_WAVES];
  float sc[16][ATT_CHUNK];                                          // scores per head
  __attribute__((aligned(16))) uint16_t qp[3][16][128];            // rotated queries, three bf16 pieces
  __attribute__((aligned(16))) uint16_t pw[3][16][ATT_CHUNK];      // softmax weights, three bf16 pieces
  __attribute__((aligned(16))) uint16_t knew[128], vnew[128];      // this step's K and V rows (bf16 bits)
  float att_m[16], att_l[16];
  __attribute__((aligned(16))) float outv[16][128];                // value sums of the chunk per head, for publication
  float bestv[MK_WAVES];
  int besti[MK_WAVES];
  int tok;
  int abort;
};

// Called by a thread whose wait ran out (or that saw another workgroup give up).
__device__ __forceinline__ void give_up(const MkArgs& a, Smem& sm) {
  st_u32(a.error, 1u);
  sm.abort = 1;
}
__device__ __forceinline__ bool spin_over(const MkArgs& a, unsigned& spins) {
  ++spins;
  return spins > a.spin_max || ((spins & 255u) == 0 && ld_u32(a.error) != 0);
}

// bf16 pieces of the pair (v.x, v.y) = activations k, k+1 (k even, relative to the
// operand's first k) into the packed LDS operand: 4 columns of 16 bytes per 8 k
// (three pieces and one unused column).
template <class HF>
__device__ __forceinline__ void put_pair(uint4* opnd, int k, float2 v) {
  float rx = v.x, ry = v.y;
  uint32_t* base = reinterpret_cast<uint32_t*>(opnd + (size_t)(k >> 3) * 4) + ((k & 7) >> 1);
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const uint32_t bx = HF::bits(rx), by = HF::bits(ry);
    base[s * 4] = bx | (by << 16);
    rx -= HF::widen(bx);
    ry -= HF::widen(by);
  }
}

// Prefetched weights of one GEMM unit: MK_PF loads per lane for each of its RT tiles.
template <int RT>
struct Pf {
  uint4 v[MK_PF * RT];
};

// Issue the first MK_PF * RT weight loads of a GEMM unit (same order gemm_unit consumes them).
template <int RT>
__device__ __forceinline__ void pf_issue(Pf<RT>& pf, const uint4* __restrict__ W, size_t tile0, int KT, int kt_begin,
                                         int kt_end) {
  const int tid = opaque(threadIdx.x);
  const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int j = 0; j < MK_PF * RT; ++j) {
    const int kt = kt_begin + wave + MK_WAVES * (j / RT);
    const int rt = j % RT;
    pf.v[j] = kt < kt_end ? ldw(&W[((tile0 + rt) * KT + kt) * 64 + lane]) : uint4{0, 0, 0, 0};
  }
}

// One GEMM unit: RT adjacent 16-row tiles x k tiles [kt_begin, kt_end), the
// waves taking k tiles round-robin; the operand in LDS starts at k tile opnd_kt0.
// Every wave leaves its partial tile in red[wave][rt]; the caller synchronises.
template <int RT, bool USE_PF, class HF>
__device__ __forceinline__ void gemm_unit(Smem& sm, const uint4* __restrict__ W, size_t tile0, int KT, int kt_begin,
                                          int kt_end, const Pf<RT>& pf, const uint4* opnd, int opnd_kt0) {
  const int tid = opaque(threadIdx.x);
  const int wave = tid >> 6, lane = tid & 63;
  const int c16 = lane & 15, g = lane >> 4;
  const bool colok = c16 < 3;
  f32x4 acc[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
  constexpr int U = MK_PF;  // k tiles per group
  auto consume = [&](int kt0, const uint4 (&av)[U][RT]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kt = kt0 + MK_WAVES * u;
      uint4 bv = uint4{0, 0, 0, 0};
      if (kt < kt_end && colok) bv = opnd[((size_t)(kt - opnd_kt0) * 4 + g) * 4 + c16];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        acc[rt] = HF::mfma(__builtin_bit_cast(u32x4, av[u][rt]), __builtin_bit_cast(u32x4, bv), acc[rt]);
    }
  };
  int kt0 = kt_begin + wave;
  if constexpr (USE_PF) {
    uint4 av[U][RT];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) av[u][rt] = pf.v[u * RT + rt];
    consume(kt0, av);
    kt0 += MK_WAVES * U;
  }
  for (; kt0 < kt_end; kt0 += MK_WAVES * U) {
    uint4 av[U][RT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kt = kt0 + MK_WAVES * u;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        av[u][rt] = kt < kt_end ? ldw(&W[((tile0 + rt) * KT + kt) * 64 + lane]) : uint4{0, 0, 0, 0};
    }
    consume(kt0, av);
  }
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm.red[wave][rt][i * 64 + lane] = acc[rt][i];
}

// Sum of the waves' partial tiles and of the three bf16 pieces for output row
// `row` of tile rt; call after wg_sync().  Accumulator element i of lane l is output
// row (l / 16) * 4 + i, operand column l % 16.
__device__ __forceinline__ float tile_total(const Smem& sm, int rt, int row) {
  float v = 0.f;
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const int idx = (row & 3) * 64 + (row >> 2) * 16 + s;
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < MK_WAVES; ++w) t += sm.red[w][rt][idx];
    v += t;
  }
  return v;
}

// x[j] += sum over `ks` slices of the exchanged vector `buf` ([ks][H] tagged words), for
// the pairs k = 2 * (tid + MK_THREADS * j) this thread owns.  Loads are repeated until
// every word carries `tag`.
template <int NP>
__device__ __forceinline__ void add_exchanged(const MkArgs& a, Smem& sm, float2 (&x)[NP], int H, const u64* buf, int ks,
                                              unsigned tag) {
  constexpr int JB = NP < 4 ? NP : 4;  // pairs per thread whose words are in flight together
  const int tid = opaque(threadIdx.x);
#pragma unroll
  for (int j0 = 0; j0 < NP; j0 += JB) {
    unsigned spins = 0;
    for (;;) {
      u64 w[JB][MK_MAX_KS][2];
#pragma unroll
      for (int j = 0; j < JB; ++j) {
        const int k = 2 * (tid + MK_THREADS * (j0 + j));
        if (k < H) {
#pragma unroll
          for (int p = 0; p < MK_MAX_KS; ++p)
            if (p < ks) {
              w[j][p][0] = ld_t(buf + (size_t)p * H + k);
              w[j][p][1] = ld_t(buf + (size_t)p * H + k + 1);
            }
        }
      }
      bool ok = true;
#pragma unroll
      for (int j = 0; j < JB; ++j) {
        const int k = 2 * ((int)threadIdx.x + MK_THREADS * (j0 + j));
        if (k < H) {
#pragma unroll
          for (int p = 0; p < MK_MAX_KS; ++p)
            if (p < ks) ok = ok && t_ok(w[j][p][0], tag) && t_ok(w[j][p][1], tag);
        }
      }
      if (ok) {
#pragma unroll
        for (int j = 0; j < JB; ++j) {
          const int k = 2 * ((int)threadIdx.x + MK_THREADS * (j0 + j));
          if (k < H) {
            float2 add = make_float2(t_val(w[j][0][0]), t_val(w[j][0][1]));
#pragma unroll
            for (int p = 1; p < MK_MAX_KS; ++p)
              if (p < ks) {
                add.x += t_val(w[j][p][0]);
                add.y += t_val(w[j][p][1]);
              }
            x[j0 + j].x += add.x;
            x[j0 + j].y += add.y;
          }
        }
        break;
      }
      if (spin_over(a, spins)) {
        give_up(a, sm);
        return;
      }
    }
  }
}

// Row r of the packed embedding matrix, pairs owned by this thread.
template <int NP, class HF>
__device__ __forceinline__ void gather_embed(float2 (&x)[NP], int H, const uint4* embed, int r) {
  const int KTH = H / 32;
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int k = 2 * ((int)threadIdx.x + MK_THREADS * j);
    x[j] = make_float2(0.f, 0.f);
    if (k < H) {
      const size_t e = (((size_t)(r >> 4) * KTH + (k >> 5)) * 64 + (r & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
      const uint32_t two = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint16_t*>(embed) + e);
      x[j] = make_float2(HF::lo(two), HF::hi(two));
    }
  }
}

// RMSNorm in two halves, so that neither waits for the other: the operand packed here is
// x * gain (not yet divided by the root mean square); each wave leaves its sum of squares in
// sm.wsum, and the GEMM epilogues multiply their outputs by rms_scale(), which is exact
// because the matmul is linear.  Caller synchronises before the GEMM as it must anyway.
// Gains of the pairs this thread owns.  Loaded before the wait for the exchanged vector, so
// that their latency (an L2 hit, ~0.7 us) overlaps with it instead of following it.
template <int NP>
__device__ __forceinline__ void load_gain(float2 (&gg)[NP], int H, const float* gain) {
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int k = 2 * ((int)threadIdx.x + MK_THREADS * j);
    gg[j] = k < H ? *reinterpret_cast<const float2*>(gain + k) : make_float2(0.f, 0.f);
  }
}

// 1 / sqrt(mean(x^2) + eps) from the per-wave sums of squares (after a workgroup barrier).
__device__ __forceinline__ float rms_from_sums(const Smem& sm, int H, float eps) {
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < MK_WAVES; ++w) t += sm.wsum[w];
  return 1.0f / sqrtf(t / (float)H + eps);
}

// A format with a narrow exponent range (binary16) cannot split an un-normalised row of small
// magnitude into pieces without losing bits, so there the row is normalised first (one more
// workgroup barrier) and the epilogues multiply by one.
template <int NP, class HF>
__device__ __forceinline__ void norm_pack(Smem& sm, uint4* opnd, int H, float eps, const float2 (&x)[NP],
                                          const float2 (&gg)[NP]) {
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < NP; ++j) ss += x[j].x * x[j].x + x[j].y * x[j].y;  // unowned pairs are zero
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) sm.wsum[threadIdx.x >> 6] = ss;
  float r = 1.0f;
  if constexpr (HF::kNarrowRange) {
    wg_sync();
    r = rms_from_sums(sm, H, eps);
  }
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int k = 2 * ((int)threadIdx.x + MK_THREADS * j);
    if (k < H) put_pair<HF>(opnd, k, make_float2(x[j].x * gg[j].x * r, x[j].y * gg[j].y * r));
  }
}

// What the GEMM epilogues after norm_pack multiply their outputs by (after the workgroup barrier).
template <class HF>
__device__ __forceinline__ float rms_scale(const Smem& sm, int H, float eps) {
  if constexpr (HF::kNarrowRange) return 1.0f;
  else return rms_from_sums(sm, H, eps);
}

}  // namespace

// GH = query heads sharing one kv head that a workgroup handles together (divides nq/nkv).
// NP = (k, k+1) pairs of a hidden-state row per thread: hidden <= 2 * MK_THREADS * NP.
template <int GH, int NP, class HF>
__global__ __launch_bounds__(MK_THREADS, 1) void k_decode_resident(MkArgs a) {
  extern __shared__ uint4 opnd[];  // packed activation operand of the current GEMM stage
  __shared__ Smem sm;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nwg = gridDim.x, wg = blockIdx.x;
  const int H = a.H, F = a.F, V = a.V, nq = a.nq, nkv = a.nkv;
  const int Dq = nq * 128, Dkv = nkv * 128, Nqkv = Dq + 2 * Dkv;
  const int KTH = H / 32, KTQ = Dq / 32, KTF = F / 32;
  const int G = nq / nkv;

  if (ld_u32(a.error)) return;
  if (tid == 0) sm.abort = 0;
  wg_sync();

  // static partition of every stage
  const int qkv_tiles = Nqkv / 16, o_tiles = H / 16, gu_pairs = F / 16, v_tiles = V / 16;
  const int kts_o = (KTQ + a.ks_o - 1) / a.ks_o, kts_d = (KTF + a.ks_d - 1) / a.ks_d;
  const int o_units = o_tiles * a.ks_o, d_units = o_tiles * a.ks_d;
  const unsigned tags_per_step = 5u * (unsigned)a.n_layers + 1u;

  // optional stage trace: thread 0 stamps the 100 MHz wall clock at stage boundaries
  int tp = 0;
  auto stamp = [&](int step) {
    if (a.trace && tid == 0 && step == a.trace_step && tp < a.trace_points)
      a.trace[(size_t)wg * a.trace_points + tp++] = wall_clock64();
  };

  // this workgroup's first unit in the stages that are placed with an offset
  const int wg_att = (wg + nwg - a.off_att) % nwg, wg_o = (wg + nwg - a.off_o) % nwg,
            wg_d = (wg + nwg - a.off_d) % nwg;

  // Prefetched weights of this workgroup's first unit in each GEMM stage, one register set
  // per stage.  Issuing a set costs the wave ~0.3 us of address traffic, and loads return in
  // order, so a wait issued after a prefetch cannot complete before the prefetch has landed
  // (~2 us).  Both are free just before a wait that is long anyway, and that is where the
  // three prefetch points sit; none follows a wait directly.
  Pf<1> pf1, pf3, pf5;
  Pf<2> pf4;
  if (wg < qkv_tiles) pf_issue<1>(pf1, a.layers[0].wqkv, (size_t)wg, KTH, 0, KTH);

  float2 x[NP];  // this workgroup's copy of the residual stream (pairs owned by the thread)
  int tok = a.tok0;

  for (int step = 0; step < a.n_steps; ++step) {
    const uint32_t pos = a.pos0 + step;
    const unsigned t_step = a.tag_base + (unsigned)step * tags_per_step;
    for (int li = 0; li < a.n_layers; ++li) {
      const MkLayer L = a.layers[li];
      const unsigned t_q = t_step + 5u * li, t_att = t_q + 1, t_op = t_q + 2, t_act = t_q + 3, t_dp = t_q + 4;
      stamp(step);  // 0: layer start

      // ============ stage 1: residual update + input norm + QKV projection ============
      float2 gg[NP];
      load_gain<NP>(gg, H, L.g_in);
      if (li == 0)
        gather_embed<NP, HF>(x, H, a.embed, tok);
      else
        add_exchanged<NP>(a, sm, x, H, a.xdp, a.ks_d, t_dp - 5u);
      norm_pack<NP, HF>(sm, opnd, H, a.eps, x, gg);
      wg_sync();
      if (sm.abort) return;
      stamp(step);  // 1: operand ready
      for (int t = wg; t < qkv_tiles; t += nwg) {
        if (t == wg)
          gemm_unit<1, true, HF>(sm, L.wqkv, (size_t)t, KTH, 0, KTH, pf1, opnd, 0);
        else
          gemm_unit<1, false, HF>(sm, L.wqkv, (size_t)t, KTH, 0, KTH, pf1, opnd, 0);
        wg_sync();
        if (tid < 16) st_t(a.xq + t * 16 + tid, tile_total(sm, 0, tid) * rms_scale<HF>(sm, H, a.eps), t_q);
        wg_sync();
      }
      // prefetch point A (a long wait follows: attention has to run first): output projection
      if (wg_o < o_units) {
        const int to = wg_o / a.ks_o, so = wg_o % a.ks_o;
        pf_issue<1>(pf3, L.wo, (size_t)to, KTQ, so * kts_o, min(KTQ, (so + 1) * kts_o));
      }
      stamp(step);  // 2: q | k | v published

      // ============ stage 2: QK-norm + RoPE + KV append + attention partials ============
      // A unit = (kv head, chunk of 64 positions) for all G query heads of the kv head, both
      // products on the matrix cores with the heads as operand columns:
      //   S^T = K Q^T   A = this wave's 16 cached K rows straight from the cache, B = the queries
      //                 (three bf16 pieces from LDS: fp32-grade);
      //   O^T = V^T P^T A = one head dimension x 8 positions gathered from the V rows staged in
      //                 LDS, B = the softmax weights (three pieces, split once per head).
      // The step's own K / V row is not in the cache when the loads are issued: the lane /
      // LDS row that stands for position `pos` takes it from the role waves instead.
      const int nch = (int)(pos / ATT_CHUNK) + 1;  // chunks that hold positions 0 .. pos
      for (int u = wg_att; u < nkv * nch; u += nwg) {
        const int chunk = u % nch, kvh = u / nch;
        const uint32_t j0 = (uint32_t)chunk * ATT_CHUNK;
        const bool owns_new = pos - j0 < ATT_CHUNK;
        const size_t cbase = ((size_t)a.slot * nkv + kvh) * a.max_seq * 128;
        const int c16 = lane & 15, g = lane >> 4;
        const int head0 = kvh * G;
        // cached rows of the chunk, loaded up front (rows from `pos` on re-read an older row:
        // valid memory; replaced, zeroed or masked below)
        const uint32_t jlast = pos > 0 ? pos - 1 : 0;
        uint2 vreg[4][2];
        u32x4 kf[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const uint32_t j = min(j0 + (uint32_t)((tid >> 4) + 16 * it), jlast);
          const uint4 v = *reinterpret_cast<const uint4*>(L.vc + cbase + (size_t)j * 128 + (tid & 15) * 8);
          vreg[it][0] = make_uint2(v.x, v.y);
          vreg[it][1] = make_uint2(v.z, v.w);
        }
        const uint32_t jk = j0 + (uint32_t)(wave * 16 + c16);  // this lane's A-operand row
        {
          const uint32_t jc = min(jk, jlast);
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            kf[ks] = *reinterpret_cast<const u32x4*>(L.kc + cbase + (size_t)jc * 128 + ks * 32 + g * 8);
        }
        wg_sync();  // LDS of the previous unit / stage is free
        // roles 0..G-1: q heads; role G: the step's k row; role G+1: its v row
        for (int role = wave; role < G + 2; role += MK_WAVES) {
          if (role >= G && !owns_new) continue;
          const u64* src = role < G ? a.xq + (size_t)(head0 + role) * 128
                                    : a.xq + Dq + (size_t)(role == G ? 0 : Dkv) + (size_t)kvh * 128;
          // rotary factors and norm gains first: their loads overlap with the wait for q
          const float* gsrc = role < G ? L.g_q : L.g_k;
          const float g0 = gsrc[lane], g1 = gsrc[lane + 64];
          const float2 cs = a.rope[(size_t)pos * 64 + lane];
          u64 w0, w1;
          unsigned spins = 0;
          for (;;) {
            w0 = ld_t(src + lane);
            w1 = ld_t(src + lane + 64);
            if (t_ok(w0, t_q) && t_ok(w1, t_q)) break;
            if (spin_over(a, spins)) {
              give_up(a, sm);
              break;
            }
          }
          float x0 = t_val(w0), x1 = t_val(w1);
          if (role <= G) {
            const float ss = wave_sum(x0 * x0 + x1 * x1);
            const float r = 1.0f / sqrtf(ss * (1.0f / 128.0f) + a.eps);
            x0 = x0 * r * g0;
            x1 = x1 * r * g1;
            const float r0 = x0 * cs.x - x1 * cs.y, r1 = x1 * cs.x + x0 * cs.y;
            x0 = r0;
            x1 = r1;
          }
          if (role < G) {
#pragma unroll
            for (int pc = 0; pc < 3; ++pc) {
              const uint32_t b0 = HF::bits(x0), b1 = HF::bits(x1);
              sm.qp[pc][role][lane] = (uint16_t)b0;
              sm.qp[pc][role][lane + 64] = (uint16_t)b1;
              x0 -= HF::widen(b0);
              x1 -= HF::widen(b1);
            }
          } else {
            const uint32_t b0 = HF::bits(x0), b1 = HF::bits(x1);
            uint16_t* dst = (role == G ? L.kc : L.vc) + cbase + (size_t)pos * 128;
            // memory-side 32-bit stores (two bf16 each): other workgroups read this row next step
            const uint32_t n0 = __shfl_down(b0, 1, 64), n1 = __shfl_down(b1, 1, 64);
            if ((lane & 1) == 0) {
              st_u32(reinterpret_cast<unsigned*>(dst + lane), b0 | (n0 << 16));
              st_u32(reinterpret_cast<unsigned*>(dst + lane + 64), b1 | (n1 << 16));
            }
            uint16_t* keep = role == G ? sm.knew : sm.vnew;
            keep[lane] = (uint16_t)b0;
            keep[lane + 64] = (uint16_t)b1;
          }
        }
        wg_sync();
        if (sm.abort) return;
        // scores: one 16 x 16 tile per wave (rows = positions, columns = heads)
        if (jk == pos) {
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) kf[ks] = *reinterpret_cast<const u32x4*>(&sm.knew[ks * 32 + g * 8]);
        }
        f32x4 sv = f32x4{0.f, 0.f, 0.f, 0.f};
        {
          const int hq = min(c16, G - 1);
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int pc = 0; pc < 3; ++pc) {
              const u32x4 t = *reinterpret_cast<const u32x4*>(&sm.qp[pc][hq][ks * 32 + g * 8]);
              const u32x4 qf = c16 < G ? t : u32x4{0u, 0u, 0u, 0u};
              sv = HF::mfma(kf[ks], qf, sv);
            }
        }
        // lane (c16 = head, g): positions wave * 16 + g * 4 + i of the chunk
        if (c16 < G) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int jl = wave * 16 + g * 4 + i;
            sm.sc[c16][jl] = j0 + (uint32_t)jl <= pos ? sv[i] * 0.08838834764831845f : -INFINITY;
          }
        }
        // V rows into LDS; the step's own row from the role wave
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int row = (tid >> 4) + 16 * it;
          uint2* d = reinterpret_cast<uint2*>(&sm.Vs[row][(tid & 15) * 4]);
          if (j0 + (uint32_t)row == pos) {
            const uint2* nv = reinterpret_cast<const uint2*>(&sm.vnew[(tid & 15) * 8]);
            d[0] = nv[0];
            d[1] = nv[1];
          } else if (j0 + (uint32_t)row > pos) {
            d[0] = d[1] = make_uint2(0u, 0u);  // masked rows: weight 0 times a finite value
          } else {
            d[0] = vreg[it][0];
            d[1] = vreg[it][1];
          }
        }
        wg_sync();
        // chunk max, weights exp(s - max) split into pieces, chunk sum: one wave per head
        for (int h = wave; h < G; h += MK_WAVES) {
          const float x = sm.sc[h][lane];
          const float m = wave_max(x);
          const float w = expf(x - m);  // exp(-inf) = 0 for masked positions; position j0 is always valid
          float r = w;
#pragma unroll
          for (int pc = 0; pc < 3; ++pc) {
            const uint32_t b = HF::bits(r);
            sm.pw[pc][h][lane] = (uint16_t)b;
            r -= HF::widen(b);
          }
          const float l = wave_sum(w);
          if (lane == 0) {
            sm.att_m[h] = m;
            sm.att_l[h] = l;
          }
        }
        wg_sync();
        // weighted value sums: this wave's two 16-dim tiles, two halves of 32 positions
        f32x4 acc2[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          u32x4 pf[3];
#pragma unroll
          for (int pc = 0; pc < 3; ++pc) {
            const u32x4 t = *reinterpret_cast<const u32x4*>(&sm.pw[pc][min(c16, G - 1)][half * 32 + g * 8]);
            pf[pc] = c16 < G ? t : u32x4{0u, 0u, 0u, 0u};
          }
#pragma unroll
          for (int dtl = 0; dtl < 2; ++dtl) {
            const int dim = (wave * 2 + dtl) * 16 + c16;  // A-operand row c16 = this head dimension
            uint32_t b[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const uint32_t two = sm.Vs[half * 32 + g * 8 + e][dim >> 1];
              b[e] = (dim & 1) ? (two >> 16) : (two & 0xffffu);
            }
            const u32x4 vf = u32x4{b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16)};
#pragma unroll
            for (int pc = 0; pc < 3; ++pc)
              acc2[dtl] = HF::mfma(vf, pf[pc], acc2[dtl]);
          }
        }
        // acc2[dtl] element i of lane (c16 = head, g): dimension (wave * 2 + dtl) * 16 + g * 4 + i.
        // Through LDS, so that every thread publishes one word (the consumers are waiting).
        if (c16 < G) {
#pragma unroll
          for (int dtl = 0; dtl < 2; ++dtl)
            *reinterpret_cast<float4*>(&sm.outv[c16][(wave * 2 + dtl) * 16 + g * 4]) =
                make_float4(acc2[dtl][0], acc2[dtl][1], acc2[dtl][2], acc2[dtl][3]);
        }
        wg_sync();
        // The unit that appended this step's K / V row publishes nothing before those stores are
        // complete: every wave waits for its own outstanding memory operations (only the role
        // waves have any: the two row stores, issued microseconds ago), so a reader that has seen
        // all words of this unit's records -- every wave writes some of them -- and everything
        // that transitively waits for them is ordered after the row.  Other workgroups read the
        // row with ordinary loads from the next step on.
        if (owns_new) __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0), the other counters left alone
        for (int o = tid; o < G * 128; o += MK_THREADS) {
          const int h = o >> 7, i = o & 127;
          u64* rec = a.xatt + ((size_t)(head0 + h) * a.max_chunks + chunk) * 132;
          st_t(rec + i, sm.outv[h][i], t_att);
          if (i == 0) {
            st_t(rec + 128, sm.att_m[h], t_att);
            st_t(rec + 129, sm.att_l[h], t_att);
          }
        }
      }
      stamp(step);  // 3: attention partials published

      // prefetch point B (the waits of stages 3 and 4 follow, both long): gate/up and down
      if (wg < gu_pairs) pf_issue<2>(pf4, L.wgu, (size_t)wg * 2, KTH, 0, KTH);
      if (wg_d < d_units) {
        const int td = wg_d / a.ks_d, sd = wg_d % a.ks_d;
        pf_issue<1>(pf5, L.wd, (size_t)td, KTF, sd * kts_d, min(KTF, (sd + 1) * kts_d));
      }
      // ============ stage 3: merge attention chunks + output projection ============
      // Few chunks: every output-projection unit merges the chunk records of its k range itself
      // (no extra exchange).  Many chunks: that repeated merge would dominate, so one workgroup
      // per query head merges its records once and publishes the head's output, at the cost of
      // one more exchange.
      const bool merged = nch > MK_DIRECT_MERGE_MAX;
      if (merged) {
        for (int h = nwg - 1 - wg_att; h < nq; h += nwg) {
          wg_sync();
          // wave w takes chunks w, w + 4, ...; lane l the sums of dimensions l and l + 64
          const u64* rec0 = a.xatt + (size_t)h * a.max_chunks * 132;
          float M = -INFINITY, n0 = 0.f, n1 = 0.f, den = 0.f;
          for (int c0 = wave; c0 < nch; c0 += 4 * MK_WAVES) {
            u64 wm[4], wl[4], wa[4], wb[4];
            unsigned spins = 0;
            for (;;) {
              bool ok = true;
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const u64* rec = rec0 + (size_t)min(c0 + MK_WAVES * q, nch - 1) * 132;
                wm[q] = ld_t(rec + 128);
                wl[q] = ld_t(rec + 129);
                wa[q] = ld_t(rec + lane);
                wb[q] = ld_t(rec + lane + 64);
              }
#pragma unroll
              for (int q = 0; q < 4; ++q)
                ok = ok && t_ok(wm[q], t_att) && t_ok(wl[q], t_att) && t_ok(wa[q], t_att) && t_ok(wb[q], t_att);
              if (ok) break;
              if (spin_over(a, spins)) {
                give_up(a, sm);
                break;
              }
            }
            float Mn = M;
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (c0 + MK_WAVES * q < nch) Mn = fmaxf(Mn, t_val(wm[q]));
            const float sc = expf(M - Mn);  // 0 on the first group (M = -inf)
            n0 *= sc;
            n1 *= sc;
            den *= sc;
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (c0 + MK_WAVES * q < nch) {
                const float f = expf(t_val(wm[q]) - Mn);
                n0 += f * t_val(wa[q]);
                n1 += f * t_val(wb[q]);
                den += f * t_val(wl[q]);
              }
            M = Mn;
          }
          sm.mrg[wave][lane] = n0;
          sm.mrg[wave][lane + 64] = n1;
          if (lane == 0) {
            sm.att_m[wave] = M;
            sm.att_l[wave] = den;
          }
          wg_sync();
          if (sm.abort) return;
          if (tid < 128) {
            float Mt = sm.att_m[0];
#pragma unroll
            for (int w = 1; w < MK_WAVES; ++w) Mt = fmaxf(Mt, sm.att_m[w]);
            float num = 0.f, dn = 0.f;
#pragma unroll
            for (int w = 0; w < MK_WAVES; ++w) {
              const float f = expf(sm.att_m[w] - Mt);  // waves without a chunk: exp(-inf) = 0
              num += f * sm.mrg[w][tid];
              dn += f * sm.att_l[w];
            }
            st_t(a.xo + (size_t)h * 128 + tid, num / dn, t_att);
          }
        }
      }
      // The operand of a unit is its k slice of the attention output; a workgroup's units
      // usually share the slice (workgroups % slices == 0), which is then loaded once.
      int s_loaded = -1;
      for (int u = wg_o; u < o_units; u += nwg) {
        const int t = u / a.ks_o, s = u % a.ks_o;
        const int kt0 = s * kts_o, kt1 = min(KTQ, (s + 1) * kts_o);
        wg_sync();
        if (s == s_loaded) {
          // operand already in LDS
        } else if (merged) {
          // four (k, k+1) pairs of the merged output per thread at a time, loaded together
          for (int kb = kt0 * 32 + 2 * tid; kb < kt1 * 32; kb += 8 * MK_THREADS) {
            unsigned spins = 0;
            for (;;) {
              u64 w[4][2];
              bool ok = true;
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const int k = kb + 2 * MK_THREADS * j;
                if (k < kt1 * 32) {
                  w[j][0] = ld_t(a.xo + k);
                  w[j][1] = ld_t(a.xo + k + 1);
                }
              }
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const int k = kb + 2 * MK_THREADS * j;
                if (k < kt1 * 32) ok = ok && t_ok(w[j][0], t_att) && t_ok(w[j][1], t_att);
              }
              if (ok) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                  const int k = kb + 2 * MK_THREADS * j;
                  if (k < kt1 * 32) put_pair<HF>(opnd, k - kt0 * 32, make_float2(t_val(w[j][0]), t_val(w[j][1])));
                }
                break;
              }
              if (spin_over(a, spins)) {
                give_up(a, sm);
                break;
              }
            }
          }
        } else {
          // two (k, k+1) pairs per thread at a time, four chunk records each, all in flight together
          for (int kb = kt0 * 32 + 2 * tid; kb < kt1 * 32; kb += 4 * MK_THREADS) {
            float M[2], n0[2], n1[2], den[2];
  #pragma unroll
            for (int r = 0; r < 2; ++r) {
              M[r] = -INFINITY;
              n0[r] = n1[r] = den[r] = 0.f;
            }
            for (int c0 = 0; c0 < nch; c0 += 4) {
              u64 wm[2][4], wl[2][4], wa[2][4], wb[2][4];
              unsigned spins = 0;
              for (;;) {
                bool ok = true;
  #pragma unroll
                for (int r = 0; r < 2; ++r) {
                  const int k = kb + 2 * MK_THREADS * r;
                  if (k < kt1 * 32) {
                    const u64* rec0 = a.xatt + (size_t)(k >> 7) * a.max_chunks * 132;
  #pragma unroll
                    for (int q = 0; q < 4; ++q) {
                      const u64* rec = rec0 + (size_t)min(c0 + q, nch - 1) * 132;
                      wm[r][q] = ld_t(rec + 128);
                      wl[r][q] = ld_t(rec + 129);
                      wa[r][q] = ld_t(rec + (k & 127));
                      wb[r][q] = ld_t(rec + (k & 127) + 1);
                    }
                  }
                }
  #pragma unroll
                for (int r = 0; r < 2; ++r)
                  if (kb + 2 * MK_THREADS * r < kt1 * 32) {
  #pragma unroll
                    for (int q = 0; q < 4; ++q)
                      ok = ok && t_ok(wm[r][q], t_att) && t_ok(wl[r][q], t_att) && t_ok(wa[r][q], t_att) &&
                           t_ok(wb[r][q], t_att);
                  }
                if (ok) break;
                if (spin_over(a, spins)) {
                  give_up(a, sm);
                  break;
                }
              }
              // online merge of the chunk records
  #pragma unroll
              for (int r = 0; r < 2; ++r)
                if (kb + 2 * MK_THREADS * r < kt1 * 32) {
                  float Mn = M[r];
  #pragma unroll
                  for (int q = 0; q < 4; ++q)
                    if (c0 + q < nch) Mn = fmaxf(Mn, t_val(wm[r][q]));
                  const float sc = expf(M[r] - Mn);  // 0 on the first group (M = -inf)
                  n0[r] *= sc;
                  n1[r] *= sc;
                  den[r] *= sc;
  #pragma unroll
                  for (int q = 0; q < 4; ++q)
                    if (c0 + q < nch) {
                      const float f = expf(t_val(wm[r][q]) - Mn);
                      n0[r] += f * t_val(wa[r][q]);
                      n1[r] += f * t_val(wb[r][q]);
                      den[r] += f * t_val(wl[r][q]);
                    }
                  M[r] = Mn;
                }
            }
  #pragma unroll
            for (int r = 0; r < 2; ++r) {
              const int k = kb + 2 * MK_THREADS * r;
              if (k < kt1 * 32) put_pair<HF>(opnd, k - kt0 * 32, make_float2(n0[r] / den[r], n1[r] / den[r]));
            }
          }
        }
        s_loaded = s;
        wg_sync();
        if (sm.abort) return;
        if (u == wg_o)
          gemm_unit<1, true, HF>(sm, L.wo, (size_t)t, KTQ, kt0, kt1, pf3, opnd, kt0);
        else
          gemm_unit<1, false, HF>(sm, L.wo, (size_t)t, KTQ, kt0, kt1, pf3, opnd, kt0);
        wg_sync();
        if (tid < 16) st_t(a.xop + (size_t)s * H + t * 16 + tid, tile_total(sm, 0, tid), t_op);
      }
      stamp(step);  // 4: attention block output published

      // ============ stage 4: residual update + post-attention norm + gate/up + SwiGLU ============
      load_gain<NP>(gg, H, L.g_post);
      add_exchanged<NP>(a, sm, x, H, a.xop, a.ks_o, t_op);
      norm_pack<NP, HF>(sm, opnd, H, a.eps, x, gg);
      wg_sync();
      if (sm.abort) return;
      stamp(step);  // 5: operand ready
      for (int pr = wg; pr < gu_pairs; pr += nwg) {
        if (pr == wg)
          gemm_unit<2, true, HF>(sm, L.wgu, (size_t)pr * 2, KTH, 0, KTH, pf4, opnd, 0);
        else
          gemm_unit<2, false, HF>(sm, L.wgu, (size_t)pr * 2, KTH, 0, KTH, pf4, opnd, 0);
        wg_sync();
        if (tid < 16) {
          const float r = rms_scale<HF>(sm, H, a.eps);
          const float gate = tile_total(sm, 0, tid) * r, up = tile_total(sm, 1, tid) * r;
          st_t(a.xact + pr * 16 + tid, gate / (1.0f + expf(-gate)) * up, t_act);
        }
        wg_sync();
      }
      stamp(step);  // 6: activations published

      // prefetch point C (the activation exchange follows): QKV of the next layer / next step
      if (wg < qkv_tiles && (li + 1 < a.n_layers || step + 1 < a.n_steps))
        pf_issue<1>(pf1, a.layers[li + 1 < a.n_layers ? li + 1 : 0].wqkv, (size_t)wg, KTH, 0, KTH);
      // ============ stage 5: down projection (k slices) ============
      s_loaded = -1;
      for (int u = wg_d; u < d_units; u += nwg) {
        const int t = u / a.ks_d, s = u % a.ks_d;
        const int kt0 = s * kts_d, kt1 = min(KTF, (s + 1) * kts_d);
        wg_sync();
        // four (k, k+1) pairs per thread at a time, loaded together
        for (int kb = kt0 * 32 + 2 * tid; s != s_loaded && kb < kt1 * 32; kb += 8 * MK_THREADS) {
          unsigned spins = 0;
          for (;;) {
            u64 w[4][2];
            bool ok = true;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int k = kb + 2 * MK_THREADS * j;
              if (k < kt1 * 32) {
                w[j][0] = ld_t(a.xact + k);
                w[j][1] = ld_t(a.xact + k + 1);
              }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int k = kb + 2 * MK_THREADS * j;
              if (k < kt1 * 32) ok = ok && t_ok(w[j][0], t_act) && t_ok(w[j][1], t_act);
            }
            if (ok) {
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const int k = kb + 2 * MK_THREADS * j;
                if (k < kt1 * 32) put_pair<HF>(opnd, k - kt0 * 32, make_float2(t_val(w[j][0]), t_val(w[j][1])));
              }
              break;
            }
            if (spin_over(a, spins)) {
              give_up(a, sm);
              break;
            }
          }
        }
        s_loaded = s;
        wg_sync();
        if (sm.abort) return;
        if (u == wg_d)
          gemm_unit<1, true, HF>(sm, L.wd, (size_t)t, KTF, kt0, kt1, pf5, opnd, kt0);
        else
          gemm_unit<1, false, HF>(sm, L.wd, (size_t)t, KTF, kt0, kt1, pf5, opnd, kt0);
        wg_sync();
        if (tid < 16) st_t(a.xdp + (size_t)s * H + t * 16 + tid, tile_total(sm, 0, tid), t_dp);
      }
      stamp(step);  // 7: MLP output published
    }

    // ============ final norm + LM head + arg-max ============
    const unsigned t_am = t_step + tags_per_step - 1u;
    {
      float2 gg[NP];
      load_gain<NP>(gg, H, a.g_final);
      add_exchanged<NP>(a, sm, x, H, a.xdp, a.ks_d, t_am - 1u);
      norm_pack<NP, HF>(sm, opnd, H, a.eps, x, gg);
    }
    wg_sync();
    if (sm.abort) return;
    stamp(step);  // LM head operand ready
    {
      // every wave walks whole 16-row tiles of the vocabulary on its own (no k split,
      // no workgroup synchronisation): tile = global wave index, stride = all waves
      const int c16 = lane & 15, g = lane >> 4;
      const bool colok = c16 < 3;
      float best = -INFINITY;
      int besti = 0x7fffffff;
      const float rms = rms_scale<HF>(sm, H, a.eps);
      float* lg = a.logits ? a.logits + (size_t)step * V : nullptr;
      for (int t = wg * MK_WAVES + wave; t < v_tiles; t += nwg * MK_WAVES) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        const uint4* Wt = a.lm_head + (size_t)t * KTH * 64 + lane;
        for (int kt0 = 0; kt0 < KTH; kt0 += 16) {
          uint4 av[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) av[u] = kt0 + u < KTH ? Wt[(size_t)(kt0 + u) * 64] : uint4{0, 0, 0, 0};
#pragma unroll
          for (int u = 0; u < 16; ++u) {
            uint4 bv = uint4{0, 0, 0, 0};
            if (kt0 + u < KTH && colok) bv = opnd[((size_t)(kt0 + u) * 4 + g) * 4 + c16];
            acc = HF::mfma(__builtin_bit_cast(u32x4, av[u]), __builtin_bit_cast(u32x4, bv), acc);
          }
        }
        // add the three pieces: columns 0, 1, 2 sit in adjacent lanes
        f32x4 s;
#pragma unroll
        for (int i = 0; i < 4; ++i) s[i] = (acc[i] + __shfl_down(acc[i], 1, 64) + __shfl_down(acc[i], 2, 64)) * rms;
        if (c16 == 0) {
          const int row0 = t * 16 + g * 4;
          if (lg) *reinterpret_cast<float4*>(lg + row0) = make_float4(s[0], s[1], s[2], s[3]);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (s[i] > best) {  // rows increase, strict > keeps the lowest index
              best = s[i];
              besti = row0 + i;
            }
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(besti, o, 64);
        if (ov > best || (ov == best && oi < besti)) {
          best = ov;
          besti = oi;
        }
      }
      if (lane == 0) {
        sm.bestv[wave] = best;
        sm.besti[wave] = besti;
      }
      wg_sync();
      if (tid == 0) {
        float v = sm.bestv[0];
        int i = sm.besti[0];
        for (int w = 1; w < MK_WAVES; ++w)
          if (sm.bestv[w] > v || (sm.bestv[w] == v && sm.besti[w] < i)) {
            v = sm.bestv[w];
            i = sm.besti[w];
          }
        st_t(a.xamv + wg, v, t_am);
        st_t(a.xami + wg, __int_as_float(i), t_am);
      }
    }
    stamp(step);  // winners published

    // every workgroup reduces the per-workgroup winners itself: the next token needs no
    // further exchange
    if (wave == 0) {
      float v = -INFINITY;
      int i = 0x7fffffff;
      for (int w0 = lane; w0 < nwg; w0 += 256) {
        u64 wv[4], wi[4];
        unsigned spins = 0;
        for (;;) {
          bool ok = true;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int w = min(w0 + 64 * q, nwg - 1);
            wv[q] = ld_t(a.xamv + w);
            wi[q] = ld_t(a.xami + w);
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) ok = ok && t_ok(wv[q], t_am) && t_ok(wi[q], t_am);
          if (ok) break;
          if (spin_over(a, spins)) {
            give_up(a, sm);
            break;
          }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float ov = t_val(wv[q]);
          const int oi = __float_as_int(t_val(wi[q]));
          if (w0 + 64 * q < nwg && (ov > v || (ov == v && oi < i))) {
            v = ov;
            i = oi;
          }
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, 64);
        const int oi = __shfl_xor(i, o, 64);
        if (ov > v || (ov == v && oi < i)) {
          v = ov;
          i = oi;
        }
      }
      if (lane == 0) {
        const int t = i == 0x7fffffff ? 0 : i;
        sm.tok = t;
        if (wg == 0) a.token_log[step] = t;
      }
    }
    wg_sync();
    if (sm.abort) return;
    tok = sm.tok;
    stamp(step);  // token known
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
size_t mk_layer_bytes() { return sizeof(MkLayer); }

void mk_fill_layer(void* dst, const void* wqkv, const void* wo, const void* wgu, const void* wd, const float* g_in,
                   const float* g_q, const float* g_k, const float* g_post, void* kc, void* vc) {
  MkLayer l;
  l.wqkv = static_cast<const uint4*>(wqkv);
  l.wo = static_cast<const uint4*>(wo);
  l.wgu = static_cast<const uint4*>(wgu);
  l.wd = static_cast<const uint4*>(wd);
  l.g_in = g_in;
  l.g_q = g_q;
  l.g_k = g_k;
  l.g_post = g_post;
  l.kc = static_cast<uint16_t*>(kc);
  l.vc = static_cast<uint16_t*>(vc);
  memcpy(dst, &l, sizeof l);
}

// Operand bytes in LDS: the widest k range any stage holds at once (4 columns of 16 bytes per 8 k).
size_t mk_opnd_bytes(const MkPlan& p) {
  const int kts_o = (p.nq * 128 / 32 + p.ks_o - 1) / p.ks_o, kts_d = (p.F / 32 + p.ks_d - 1) / p.ks_d;
  int kt = p.H / 32;
  if (kts_o > kt) kt = kts_o;
  if (kts_d > kt) kt = kts_d;
  return (size_t)kt * 4 * 4 * 16;
}

// Workgroups of the resident kernel (for this plan's template instance and LDS size) that the
// device can hold at once, 0 on error: the grid must fit, since its workgroups wait for each other.
int mk_max_resident_workgroups(const MkPlan& p, int n_cus) {
  const int G = p.nkv > 0 ? p.nq / p.nkv : 0;
  const size_t dyn = mk_opnd_bytes(p);
  int per_cu = 0;
  hipError_t e = hipErrorInvalidValue;
#define MK_OCC(GH, NP)                                                                                        \
  do {                                                                                                        \
    if (p.f16) {                                                                                              \
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_resident<GH, NP, Fp16>),                \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);                          \
      if (e == hipSuccess)                                                                                    \
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_decode_resident<GH, NP, Fp16>, MK_THREADS, dyn); \
    } else {                                                                                                  \
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_resident<GH, NP, Bf16>),                \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);                          \
      if (e == hipSuccess)                                                                                    \
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_decode_resident<GH, NP, Bf16>, MK_THREADS, dyn); \
    }                                                                                                         \
  } while (0)
#define MK_OCC_NP(GH)                    \
  do {                                   \
    if (p.H <= 1024) MK_OCC(GH, 2);      \
    else if (p.H <= 2048) MK_OCC(GH, 4); \
    else MK_OCC(GH, 8);                  \
  } while (0)
  if (G % 4 == 0) MK_OCC_NP(4);
  else MK_OCC_NP(2);
#undef MK_OCC_NP
#undef MK_OCC
  if (e != hipSuccess || per_cu < 1) return 0;
  return per_cu * n_cus;
}

hipError_t launch_decode_resident(hipStream_t s, const MkPlan& p, const MkBuffers& bf) {
  const int G = p.nq / p.nkv;
  if (p.H > 4096 || p.ks_o > MK_MAX_KS || p.ks_d > MK_MAX_KS || p.ks_o < 1 || p.ks_d < 1 || (G % 2) != 0 || G > 16 ||
      p.nwg < 1 || p.nwg > (p.nq + 2 * p.nkv) * 8)
    return hipErrorInvalidValue;
  MkArgs a{};
  a.layers = static_cast<const MkLayer*>(bf.layers);
  a.n_layers = p.n_layers; a.H = p.H; a.nq = p.nq; a.nkv = p.nkv; a.F = p.F; a.V = p.V;
  a.eps = p.eps;
  a.embed = static_cast<const uint4*>(bf.embed);
  a.lm_head = static_cast<const uint4*>(bf.lm_head);
  a.g_final = bf.g_final;
  a.rope = bf.rope;
  a.max_seq = p.max_seq;
  a.error = bf.error;
  a.spin_max = p.spin_max ? p.spin_max : MK_SPIN_MAX;
  a.tok0 = p.tok0; a.pos0 = p.pos0; a.slot = p.slot;
  a.n_steps = p.n_steps;
  a.tag_base = p.tag_base;
  a.ks_o = p.ks_o; a.ks_d = p.ks_d;
  a.off_att = p.off_att % p.nwg; a.off_o = p.off_o % p.nwg; a.off_d = p.off_d % p.nwg;
  a.xq = static_cast<u64*>(bf.xq); a.xatt = static_cast<u64*>(bf.xatt); a.max_chunks = p.max_chunks;
  a.xo = static_cast<u64*>(bf.xo);
  a.xop = static_cast<u64*>(bf.xop); a.xact = static_cast<u64*>(bf.xact); a.xdp = static_cast<u64*>(bf.xdp);
  a.xamv = static_cast<u64*>(bf.xamv); a.xami = static_cast<u64*>(bf.xami);
  a.logits = bf.logits; a.token_log = bf.token_log;
  a.trace = bf.trace; a.trace_step = bf.trace_step; a.trace_points = bf.trace_points;
  const size_t dyn = mk_opnd_bytes(p);
  hipError_t e;
#define MK_LAUNCH(GH, NP)                                                                                     \
  do {                                                                                                        \
    if (p.f16) {                                                                                              \
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_resident<GH, NP, Fp16>),                \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);                          \
      if (e != hipSuccess) return e;                                                                          \
      k_decode_resident<GH, NP, Fp16><<<p.nwg, MK_THREADS, dyn, s>>>(a);                                      \
    } else {                                                                                                  \
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_resident<GH, NP, Bf16>),                \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);                          \
      if (e != hipSuccess) return e;                                                                          \
      k_decode_resident<GH, NP, Bf16><<<p.nwg, MK_THREADS, dyn, s>>>(a);                                      \
    }                                                                                                         \
  } while (0)
#define MK_LAUNCH_NP(GH)                    \
  do {                                      \
    if (p.H <= 1024) MK_LAUNCH(GH, 2);      \
    else if (p.H <= 2048) MK_LAUNCH(GH, 4); \
    else MK_LAUNCH(GH, 8);                  \
  } while (0)
  if (G % 4 == 0) MK_LAUNCH_NP(4);
  else MK_LAUNCH_NP(2);
#undef MK_LAUNCH_NP
#undef MK_LAUNCH
  return hipGetLastError();
}

}  // namespace nnc
