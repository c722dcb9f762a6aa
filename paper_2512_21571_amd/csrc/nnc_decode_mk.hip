// Persistent whole-step decode kernel for small batches (bf16 models).
//
// Batch-1 decode of a 0.6B-shaped model moves ~1.2 GB per token: 150 us at HBM
// speed, spread over ~140 dependent matmul / attention stages of about 1 us each.
// Run as separate kernels, every stage costs a launch-drain-launch bubble of
// several microseconds, which is where the time goes; the paper observes the same
// thing on CPUs, where fork-join barriers of a threading runtime limit scaling and
// a static partition with cheap synchronisation wins (Section 5.2, architectural
// discussion).  Here one resident grid (one workgroup per compute unit) runs whole
// decode steps: every stage is statically partitioned over the workgroups, the
// stages are separated by a grid-wide barrier built from per-workgroup flags, and
// the weights of the next stage are already in flight (prefetched into registers)
// while a stage finishes and the barrier is crossed.
//
// Coherence protocol (8 XCDs, one L2 each, no cross-L2 coherence for ordinary
// accesses): everything one workgroup writes for another to read is written and
// read with relaxed agent-scope atomic accesses, which go to the memory side.  A
// barrier is: wait for this wave's stores to be acknowledged, workgroup barrier,
// publish flag = epoch, poll everyone's flag.  No cache write-back / invalidate
// is needed and none is issued (they cost ~10 us per barrier on this part).
// Weights, gains, the rotary table and cached K/V rows older than the current
// step are immutable during a launch and use ordinary loads.
#include <cstring>

#include "nnc_internal.h"

namespace nnc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int MK_THREADS = 512;
constexpr int MK_WAVES = MK_THREADS / 64;
constexpr unsigned MK_SPIN_MAX = 1u << 21;
constexpr int MK_PF = 8;  // 16-byte weight loads per lane kept in flight across a barrier

// ---- memory-side accesses ----------------------------------------------------
__device__ __forceinline__ unsigned ld_u32(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_u32(unsigned* p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_f(const float* p) {
  return __uint_as_float(ld_u32(reinterpret_cast<const unsigned*>(p)));
}
__device__ __forceinline__ void st_f(float* p, float v) {
  st_u32(reinterpret_cast<unsigned*>(p), __float_as_uint(v));
}
__device__ __forceinline__ float2 ld_f2(const float* p) {
  const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
}
__device__ __forceinline__ void st_f2(float* p, float2 v) {
  const unsigned long long u = (unsigned long long)__float_as_uint(v.x) |
                               ((unsigned long long)__float_as_uint(v.y) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), u, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
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
  unsigned* flags;  // one per workgroup, 128 bytes apart
  unsigned* error;
  const ColState* st;
  int nseq, n_steps;
  int ks_o, ks_d;  // k slices of the output / down projections
  float* X0;       // residual stream, two buffers [nseq][H]
  float* X1;
  float* qkv;      // [nseq][Dq + 2 Dkv] raw projections
  float* att;      // attention partials [nseq][nq][max_chunks][132]
  int max_chunks;
  float* opart;    // [ks_o][nseq][H]
  float* act;      // [nseq][F]
  float* dpart;    // [ks_d][nseq][H]
  float* am_val;   // [workgroups][nseq]
  int32_t* am_idx;
  float* logits;   // [n_steps][nseq][V] or NULL
  int32_t* token_log;  // [n_steps][nseq]
  unsigned long long* trace;  // [workgroups][trace_points] wall-clock stamps of one step, or NULL
  int trace_step, trace_points;
};

namespace {

struct Smem {
  float red[MK_WAVES][2][256];  // per-wave accumulator tiles
  float wsum[MK_WAVES];
  float sc[4][ATT_CHUNK];
  float qs[4][128];
  float knew[128], vnew[128];
  float att_m[4], att_l[4];
  float ared[MK_WAVES][4][128];
  float bestv[MK_WAVES][8];
  int besti[MK_WAVES][8];
  int tok[8];
};

// Grid-wide barrier.  Returns false (for the whole workgroup) if it timed out or
// another workgroup reported an error; the caller then leaves the kernel.
__device__ __forceinline__ bool grid_barrier(const MkArgs& a, unsigned& epoch) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // this wave's stores are acknowledged
  __syncthreads();
  ++epoch;
  const unsigned nwg = gridDim.x;
  if (threadIdx.x == 0) st_u32(a.flags + blockIdx.x * 32, epoch);
  bool ok = true;
  for (unsigned w = threadIdx.x; w < nwg; w += MK_THREADS) {
    unsigned spins = 0;
    while ((int)(ld_u32(a.flags + w * 32) - epoch) < 0) {
      if (++spins > MK_SPIN_MAX || ((spins & 1023u) == 0 && ld_u32(a.error))) {
        st_u32(a.error, 1u);
        ok = false;
        break;
      }
    }
  }
  return __syncthreads_and(ok);
}

__device__ __forceinline__ float block_sum(float v, Smem& sm) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.wsum[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < MK_WAVES; ++w) t += sm.wsum[w];
  return t;
}

// Write the bf16 pieces of the pair (v.x, v.y) = activations k, k+1 (k even) of
// sequence `seq` into the packed LDS operand (k is relative to the operand's start).
__device__ __forceinline__ void put_pair(uint4* opnd, int NC, int seq, int k, float2 v) {
  float rx = v.x, ry = v.y;
  uint32_t* base = reinterpret_cast<uint32_t*>(opnd + (size_t)(k >> 3) * NC + seq * 3) + ((k & 7) >> 1);
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const uint32_t bx = bf16_bits(rx), by = bf16_bits(ry);
    base[s * 4] = bx | (by << 16);
    rx -= bf16_to_f32(bx);
    ry -= bf16_to_f32(by);
  }
}

struct Pf {
  uint4 v[MK_PF];
};

constexpr int MK_MAX_KS = 4;  // k slices of a narrow projection (partial vectors a consumer adds)

// Pairs (k, k+1) owned by a thread: k = 2 * (tid + MK_THREADS * j), j < NP (H <= 1024 NP).
// xv[j] = [X] + sum of `ksd` slices of d + sum of `kso` slices of o, every load issued
// before the first use so that the memory-side round trips overlap.
template <int NP>
__device__ __forceinline__ void gather_resid(float2 (&xv)[NP], int H, const float* X, const float* d, int ksd,
                                             const float* o, int kso, long pstride) {
  float2 tx[NP], td[NP][MK_MAX_KS], to[NP][MK_MAX_KS];
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int k = 2 * ((int)threadIdx.x + MK_THREADS * j);
    if (k < H) {
      if (X) tx[j] = ld_f2(X + k);
#pragma unroll
      for (int p = 0; p < MK_MAX_KS; ++p)
        if (p < ksd) td[j][p] = ld_f2(d + (size_t)p * pstride + k);
#pragma unroll
      for (int p = 0; p < MK_MAX_KS; ++p)
        if (p < kso) to[j][p] = ld_f2(o + (size_t)p * pstride + k);
    }
  }
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int k = 2 * ((int)threadIdx.x + MK_THREADS * j);
    if (k < H) {
      float2 v = X ? tx[j] : xv[j];
      if (ksd > 0) {
        float2 add = td[j][0];
#pragma unroll
        for (int p = 1; p < MK_MAX_KS; ++p)
          if (p < ksd) {
            add.x += td[j][p].x;
            add.y += td[j][p].y;
          }
        v.x += add.x;
        v.y += add.y;
      }
      if (kso > 0) {
        float2 add = to[j][0];
#pragma unroll
        for (int p = 1; p < MK_MAX_KS; ++p)
          if (p < kso) {
            add.x += to[j][p].x;
            add.y += to[j][p].y;
          }
        v.x += add.x;
        v.y += add.y;
      }
      xv[j] = v;
    }
  }
}

// Row `r` of the packed embedding, pairs owned by this thread.
template <int NP>
__device__ __forceinline__ void gather_embed(float2 (&xv)[NP], int H, const uint4* embed, int r) {
  const int KTH = H / 32;
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int k = 2 * ((int)threadIdx.x + MK_THREADS * j);
    xv[j] = make_float2(0.f, 0.f);
    if (k < H) {
      const size_t e = (((size_t)(r >> 4) * KTH + (k >> 5)) * 64 + (r & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
      const uint32_t two = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint16_t*>(embed) + e);
      xv[j] = make_float2(bf16_to_f32(two & 0xffffu), bf16_to_f32(two >> 16));
    }
  }
}

// RMSNorm of the gathered row and packing as the GEMM operand of sequence b.
template <int NP>
__device__ __forceinline__ void norm_pack(Smem& sm, uint4* opnd, int NC, int b, int H, float eps,
                                          const float2 (&xv)[NP], const float* gain) {
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < NP; ++j) ss += xv[j].x * xv[j].x + xv[j].y * xv[j].y;  // unowned pairs are zero
  ss = block_sum(ss, sm);
  const float r = 1.0f / sqrtf(ss / (float)H + eps);
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int k = 2 * ((int)threadIdx.x + MK_THREADS * j);
    if (k < H) {
      const float2 gg = *reinterpret_cast<const float2*>(gain + k);
      put_pair(opnd, NC, b, k, make_float2(xv[j].x * r * gg.x, xv[j].y * r * gg.y));
    }
  }
}

// Issue the first MK_PF weight loads of a GEMM unit (same order gemm_unit consumes them).
template <int RT>
__device__ __forceinline__ void pf_issue(Pf& pf, const uint4* __restrict__ W, size_t tile0, int KT, int kt_begin,
                                         int kt_end) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int j = 0; j < MK_PF; ++j) {
    const int kt = kt_begin + wave + MK_WAVES * (j / RT);
    const int rt = j % RT;
    pf.v[j] = kt < kt_end ? W[((tile0 + rt) * KT + kt) * 64 + lane] : uint4{0, 0, 0, 0};
  }
}

// One GEMM unit: RT adjacent 16-row tiles x k tiles [kt_begin, kt_end), the eight
// waves taking k tiles round-robin.  The operand in LDS starts at k tile `opnd_kt0`.
// Result: red[wave][rt][256] holds every wave's partial tile; caller synchronises.
template <int RT, bool USE_PF>
__device__ __forceinline__ void gemm_unit(Smem& sm, const uint4* __restrict__ W, size_t tile0, int KT, int kt_begin,
                                          int kt_end, const Pf& pf, const uint4* opnd, int opnd_kt0, int NC,
                                          int ncols) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c16 = lane & 15, g = lane >> 4;
  const bool colok = c16 < ncols;
  f32x4 acc[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
  constexpr int U = MK_PF / RT;  // k tiles per group
  auto consume = [&](int kt0, const uint4 (&av)[U][RT]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kt = kt0 + MK_WAVES * u;
      uint4 bv = uint4{0, 0, 0, 0};
      if (kt < kt_end && colok) bv = opnd[((size_t)(kt - opnd_kt0) * 4 + g) * NC + c16];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[u][rt]),
                                                          __builtin_bit_cast(bf16x8, bv), acc[rt], 0, 0, 0);
    }
  };
  int kt0 = kt_begin + wave;
  if constexpr (USE_PF) {
    // the first group was loaded before the preceding barrier
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
        av[u][rt] = kt < kt_end ? W[((tile0 + rt) * KT + kt) * 64 + lane] : uint4{0, 0, 0, 0};
    }
    consume(kt0, av);
  }
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm.red[wave][rt][i * 64 + lane] = acc[rt][i];
}

// Sum of the eight waves' partial tiles and of the three bf16 pieces for output
// (rt, row, seq); call after __syncthreads().
__device__ __forceinline__ float tile_total(const Smem& sm, int rt, int row, int seq) {
  float v = 0.f;
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const int col = seq * 3 + s;
    const int idx = (row & 3) * 64 + (row >> 2) * 16 + col;
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < MK_WAVES; ++w) t += sm.red[w][rt][idx];
    v += t;
  }
  return v;
}

}  // namespace

// GH = query heads sharing one kv head that a workgroup handles together (nq/nkv).
// NP = (k, k+1) pairs of a hidden-state row per thread: hidden <= 1024 * NP.
template <int GH, int NP>
__global__ __launch_bounds__(MK_THREADS, 1) void k_decode_persistent(MkArgs a) {
  extern __shared__ uint4 opnd[];  // packed activation operand of the current GEMM stage
  __shared__ Smem sm;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nwg = gridDim.x, wg = blockIdx.x;
  const int H = a.H, F = a.F, V = a.V, nq = a.nq, nkv = a.nkv, nseq = a.nseq;
  const int Dq = nq * 128, Dkv = nkv * 128, Nqkv = Dq + 2 * Dkv;
  const int KTH = H / 32, KTQ = Dq / 32, KTF = F / 32;
  const int NC = nseq == 1 ? 4 : 16, ncols = nseq * 3;
  const int G = nq / nkv;

  if (ld_u32(a.error)) return;
  unsigned epoch = ld_u32(a.flags + wg * 32);  // all flags are equal between launches

  // static partition of every stage
  const int qkv_tiles = Nqkv / 16, o_tiles = H / 16, gu_pairs = F / 16, v_tiles = V / 16;
  const int kts_o = (KTQ + a.ks_o - 1) / a.ks_o, kts_d = (KTF + a.ks_d - 1) / a.ks_d;
  const int o_units = o_tiles * a.ks_o, d_units = o_tiles * a.ks_d;
  const long pstride = (long)nseq * H;

  // optional stage trace: thread 0 stamps the 100 MHz wall clock at every stage boundary
  int tp = 0;
  auto stamp = [&](int step) {
    if (a.trace && tid == 0 && step == a.trace_step && tp < a.trace_points)
      a.trace[(size_t)wg * a.trace_points + tp++] = wall_clock64();
  };

  // Cached K and V rows of one attention unit (64 positions of one kv head): two rows of
  // each per lane, loaded as soon as the unit is known; only the step's own new row,
  // which does not exist yet, is excluded (it comes from LDS later).
  const int att_units = nseq * nkv * a.max_chunks;
  auto kv_issue = [&](const MkLayer& L, int u, int step, uint4 (&kreg)[2], uint4 (&vreg)[2]) {
    const int chunk = u % a.max_chunks;
    const int kvh = (u / a.max_chunks) % nkv;
    const int b = u / (a.max_chunks * nkv);
    const uint32_t pos = a.st->pos[b] + step, slot = a.st->slot[b];
    const size_t cbase = ((size_t)slot * nkv + kvh) * a.max_seq * 128;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const uint32_t j = (uint32_t)chunk * ATT_CHUNK + it * 32 + wave * 4 + (lane >> 4);
      kreg[it] = vreg[it] = uint4{0, 0, 0, 0};
      if (j < pos) {
        kreg[it] = *reinterpret_cast<const uint4*>(L.kc + cbase + (size_t)j * 128 + (lane & 15) * 8);
        vreg[it] = *reinterpret_cast<const uint4*>(L.vc + cbase + (size_t)j * 128 + (lane & 15) * 8);
      }
    }
  };
  uint4 kpf[2], vpf[2];

  Pf pf;
  // prefetch for the very first stage (layer 0 QKV)
  if (wg < qkv_tiles) pf_issue<1>(pf, a.layers[0].wqkv, (size_t)wg, KTH, 0, KTH);

  for (int step = 0; step < a.n_steps; ++step) {
    float* Xa = a.X0;
    float* Xb = a.X1;
    for (int li = 0; li < a.n_layers; ++li) {
      const MkLayer L = a.layers[li];
      stamp(step);

      // ================= stage 1: input norm + QKV projection =================
      // x = (layer 0 ? embedding row : Xa + down-projection slices of the previous layer)
      for (int b = 0; b < nseq; ++b) {
        float2 xv[NP];
        if (li == 0) {
          gather_embed(xv, H, a.embed, step == 0 ? a.st->tok[b] : sm.tok[b]);
        } else {
#pragma unroll
          for (int j = 0; j < NP; ++j) xv[j] = make_float2(0.f, 0.f);
          gather_resid(xv, H, Xa + (size_t)b * H, a.dpart + (size_t)b * H, a.ks_d, nullptr, 0, pstride);
        }
        norm_pack(sm, opnd, NC, b, H, a.eps, xv, L.g_in);
      }
      stamp(step);
      __syncthreads();
      for (int t = wg; t < qkv_tiles; t += nwg) {
        if (t == wg)
          gemm_unit<1, true>(sm, L.wqkv, (size_t)t, KTH, 0, KTH, pf, opnd, 0, NC, ncols);
        else
          gemm_unit<1, false>(sm, L.wqkv, (size_t)t, KTH, 0, KTH, pf, opnd, 0, NC, ncols);
        __syncthreads();
        if (tid < 16 * nseq) {
          const int seq = tid >> 4, row = tid & 15;
          st_f(a.qkv + (size_t)seq * Nqkv + t * 16 + row, tile_total(sm, 0, row, seq));
        }
        __syncthreads();
      }
      // next GEMM stage with weights: output projection (stage 3)
      if (wg < o_units) {
        const int t = wg / a.ks_o, s = wg % a.ks_o;
        pf_issue<1>(pf, L.wo, (size_t)t, KTQ, s * kts_o, min(KTQ, (s + 1) * kts_o));
      }
      if (wg < att_units) kv_issue(L, wg, step, kpf, vpf);
      stamp(step);
      if (!grid_barrier(a, epoch)) return;
      stamp(step);

      // ================= stage 2: QK-norm + RoPE + KV append + attention partials ==========
      {
        const int units = att_units;
        for (int u = wg; u < units; u += nwg) {
          const int chunk = u % a.max_chunks;
          const int kvh = (u / a.max_chunks) % nkv;
          const int b = u / (a.max_chunks * nkv);
          const uint32_t pos = a.st->pos[b] + step, slot = a.st->slot[b];
          const uint32_t j0 = (uint32_t)chunk * ATT_CHUNK;
          if (j0 > pos) continue;  // uniform per workgroup
          uint4 kreg[2], vreg[2];
          if (u == wg) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
              kreg[it] = kpf[it];
              vreg[it] = vpf[it];
            }
          } else {
            kv_issue(L, u, step, kreg, vreg);
          }
          const bool owns_new = pos - j0 < ATT_CHUNK;
          const size_t cbase = ((size_t)slot * nkv + kvh) * a.max_seq * 128;
          const float* qrow = a.qkv + (size_t)b * Nqkv;
          for (int hg = 0; hg < G; hg += GH) {
            const int head0 = kvh * G + hg;
            __syncthreads();
            // waves 0..GH-1: q heads; wave GH: new k row; wave GH+1: new v row
            if (wave < GH + 2 && (wave < GH || (owns_new && hg == 0))) {
              const float* src = wave < GH ? qrow + (size_t)(head0 + wave) * 128
                                           : qrow + Dq + (size_t)(wave == GH ? 0 : Dkv) + (size_t)kvh * 128;
              float x0 = ld_f(src + lane), x1 = ld_f(src + lane + 64);
              if (wave <= GH) {
                const float ss = wave_sum(x0 * x0 + x1 * x1);
                const float r = 1.0f / sqrtf(ss * (1.0f / 128.0f) + a.eps);
                const float* gg = wave < GH ? L.g_q : L.g_k;
                x0 = x0 * r * gg[lane];
                x1 = x1 * r * gg[lane + 64];
                const float2 cs = a.rope[(size_t)pos * 64 + lane];
                const float r0 = x0 * cs.x - x1 * cs.y, r1 = x1 * cs.x + x0 * cs.y;
                x0 = r0;
                x1 = r1;
              }
              if (wave < GH) {
                sm.qs[wave][lane] = x0;
                sm.qs[wave][lane + 64] = x1;
              } else {
                const uint32_t b0 = bf16_bits(x0), b1 = bf16_bits(x1);
                uint16_t* dst = (wave == GH ? L.kc : L.vc) + cbase + (size_t)pos * 128;
                // 16-bit stores cannot be atomic accesses; pair lanes into 32-bit memory-side stores
                const uint32_t n0 = __shfl_down(b0, 1, 64), n1 = __shfl_down(b1, 1, 64);
                if ((lane & 1) == 0) {
                  st_u32(reinterpret_cast<unsigned*>(dst + lane), b0 | (n0 << 16));
                  st_u32(reinterpret_cast<unsigned*>(dst + lane + 64), b1 | (n1 << 16));
                }
                float* keep = wave == GH ? sm.knew : sm.vnew;
                keep[lane] = bf16_to_f32(b0);
                keep[lane + 64] = bf16_to_f32(b1);
              }
            }
            __syncthreads();
            const int c16 = lane & 15, jj = lane >> 4;
            float q[GH][8];
#pragma unroll
            for (int h = 0; h < GH; ++h)
#pragma unroll
              for (int e = 0; e < 8; ++e) q[h][e] = sm.qs[h][c16 * 8 + e];
            // scores
#pragma unroll
            for (int it = 0; it < ATT_CHUNK / 32; ++it) {
              const int jl = it * 32 + wave * 4 + jj;
              const uint32_t j = j0 + jl;
              float kv[8];
#pragma unroll
              for (int e = 0; e < 8; ++e) kv[e] = 0.f;
              if (j < pos) {
                const uint4 x = kreg[it];
                kv[0] = __uint_as_float(x.x << 16); kv[1] = __uint_as_float(x.x & 0xffff0000u);
                kv[2] = __uint_as_float(x.y << 16); kv[3] = __uint_as_float(x.y & 0xffff0000u);
                kv[4] = __uint_as_float(x.z << 16); kv[5] = __uint_as_float(x.z & 0xffff0000u);
                kv[6] = __uint_as_float(x.w << 16); kv[7] = __uint_as_float(x.w & 0xffff0000u);
              } else if (j == pos) {
#pragma unroll
                for (int e = 0; e < 8; ++e) kv[e] = sm.knew[c16 * 8 + e];
              }
#pragma unroll
              for (int h = 0; h < GH; ++h) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d += q[h][e] * kv[e];
                d += __shfl_xor(d, 1, 64);
                d += __shfl_xor(d, 2, 64);
                d += __shfl_xor(d, 4, 64);
                d += __shfl_xor(d, 8, 64);
                if (c16 == 0) sm.sc[h][jl] = j <= pos ? d * 0.08838834764831845f : -INFINITY;
              }
            }
            __syncthreads();
            if (wave < GH) {
              const float s = sm.sc[wave][lane];
              const float m = wave_max(s);
              const float w = expf(s - m);
              sm.sc[wave][lane] = w;
              const float l = wave_sum(w);
              if (lane == 0) {
                sm.att_m[wave] = m;
                sm.att_l[wave] = l;
              }
            }
            __syncthreads();
            float acc[GH][8];
#pragma unroll
            for (int h = 0; h < GH; ++h)
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
#pragma unroll
            for (int it = 0; it < ATT_CHUNK / 32; ++it) {
              const int jl = it * 32 + wave * 4 + jj;
              const uint32_t j = j0 + jl;
              if (j <= pos) {
                float vv[8];
                if (j < pos) {
                  const uint4 x = vreg[it];
                  vv[0] = __uint_as_float(x.x << 16); vv[1] = __uint_as_float(x.x & 0xffff0000u);
                  vv[2] = __uint_as_float(x.y << 16); vv[3] = __uint_as_float(x.y & 0xffff0000u);
                  vv[4] = __uint_as_float(x.z << 16); vv[5] = __uint_as_float(x.z & 0xffff0000u);
                  vv[6] = __uint_as_float(x.w << 16); vv[7] = __uint_as_float(x.w & 0xffff0000u);
                } else {
#pragma unroll
                  for (int e = 0; e < 8; ++e) vv[e] = sm.vnew[c16 * 8 + e];
                }
#pragma unroll
                for (int h = 0; h < GH; ++h) {
                  const float w = sm.sc[h][jl];
#pragma unroll
                  for (int e = 0; e < 8; ++e) acc[h][e] += w * vv[e];
                }
              }
            }
#pragma unroll
            for (int h = 0; h < GH; ++h)
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                float v = acc[h][e];
                v += __shfl_xor(v, 16, 64);
                v += __shfl_xor(v, 32, 64);
                if (jj == 0) sm.ared[wave][h][c16 * 8 + e] = v;
              }
            __syncthreads();
            for (int o = tid; o < GH * 128; o += MK_THREADS) {
              const int h = o >> 7, i = o & 127;
              float v = 0.f;
#pragma unroll
              for (int w = 0; w < MK_WAVES; ++w) v += sm.ared[w][h][i];
              float* rec = a.att + (((size_t)b * nq + head0 + h) * a.max_chunks + chunk) * 132;
              st_f(rec + i, v);
              if (i == 0) {
                st_f(rec + 128, sm.att_m[h]);
                st_f(rec + 129, sm.att_l[h]);
              }
            }
          }
        }
      }
      stamp(step);
      if (!grid_barrier(a, epoch)) return;
      stamp(step);

      // ================= stage 3: merge attention chunks + output projection =================
      for (int u = wg; u < o_units; u += nwg) {
        const int t = u / a.ks_o, s = u % a.ks_o;
        const int kt0 = s * kts_o, kt1 = min(KTQ, (s + 1) * kts_o);
        __syncthreads();
        for (int b = 0; b < nseq; ++b) {
          const int nch = (int)((a.st->pos[b] + step) / ATT_CHUNK) + 1;
          for (int k = kt0 * 32 + 2 * tid; k < kt1 * 32; k += 2 * MK_THREADS) {
            const int head = k >> 7, i = k & 127;
            const float* rec0 = a.att + ((size_t)b * nq + head) * a.max_chunks * 132;
            // online merge, four chunks' records in flight at a time
            float M = -INFINITY, n0 = 0.f, n1 = 0.f, den = 0.f;
            for (int c0 = 0; c0 < nch; c0 += 4) {
              float mm[4], ll[4];
              float2 oo[4];
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const float* rec = rec0 + (size_t)min(c0 + q, nch - 1) * 132;
                mm[q] = ld_f(rec + 128);
                ll[q] = ld_f(rec + 129);
                oo[q] = ld_f2(rec + i);
              }
              float Mn = M;
#pragma unroll
              for (int q = 0; q < 4; ++q)
                if (c0 + q < nch) Mn = fmaxf(Mn, mm[q]);
              const float sc = expf(M - Mn);  // 0 on the first group (M = -inf)
              n0 *= sc;
              n1 *= sc;
              den *= sc;
#pragma unroll
              for (int q = 0; q < 4; ++q)
                if (c0 + q < nch) {
                  const float f = expf(mm[q] - Mn);
                  n0 += f * oo[q].x;
                  n1 += f * oo[q].y;
                  den += f * ll[q];
                }
              M = Mn;
            }
            put_pair(opnd, NC, b, k - kt0 * 32, make_float2(n0 / den, n1 / den));
          }
        }
        __syncthreads();
        if (u == wg)
          gemm_unit<1, true>(sm, L.wo, (size_t)t, KTQ, kt0, kt1, pf, opnd, kt0, NC, ncols);
        else
          gemm_unit<1, false>(sm, L.wo, (size_t)t, KTQ, kt0, kt1, pf, opnd, kt0, NC, ncols);
        __syncthreads();
        if (tid < 16 * nseq) {
          const int seq = tid >> 4, row = tid & 15;
          st_f(a.opart + (size_t)s * pstride + (size_t)seq * H + t * 16 + row, tile_total(sm, 0, row, seq));
        }
      }
      // next: gate/up (stage 4)
      if (wg < gu_pairs) pf_issue<2>(pf, L.wgu, (size_t)wg * 2, KTH, 0, KTH);
      stamp(step);
      if (!grid_barrier(a, epoch)) return;
      stamp(step);

      // ================= stage 4: residual + post-attention norm + gate/up + SwiGLU ==========
      for (int b = 0; b < nseq; ++b) {
        float2 xv[NP];
        if (li == 0) {
          gather_embed(xv, H, a.embed, step == 0 ? a.st->tok[b] : sm.tok[b]);
          gather_resid(xv, H, nullptr, nullptr, 0, a.opart + (size_t)b * H, a.ks_o, pstride);
        } else {
#pragma unroll
          for (int j = 0; j < NP; ++j) xv[j] = make_float2(0.f, 0.f);
          gather_resid(xv, H, Xa + (size_t)b * H, a.dpart + (size_t)b * H, a.ks_d, a.opart + (size_t)b * H, a.ks_o,
                       pstride);
        }
        if (wg == 0) {
#pragma unroll
          for (int j = 0; j < NP; ++j) {
            const int k = 2 * (tid + MK_THREADS * j);
            if (k < H) st_f2(Xb + (size_t)b * H + k, xv[j]);
          }
        }
        norm_pack(sm, opnd, NC, b, H, a.eps, xv, L.g_post);
      }
      __syncthreads();
      stamp(step);
      for (int pr = wg; pr < gu_pairs; pr += nwg) {
        if (pr == wg)
          gemm_unit<2, true>(sm, L.wgu, (size_t)pr * 2, KTH, 0, KTH, pf, opnd, 0, NC, ncols);
        else
          gemm_unit<2, false>(sm, L.wgu, (size_t)pr * 2, KTH, 0, KTH, pf, opnd, 0, NC, ncols);
        __syncthreads();
        if (tid < 16 * nseq) {
          const int seq = tid >> 4, row = tid & 15;
          const float gate = tile_total(sm, 0, row, seq), up = tile_total(sm, 1, row, seq);
          st_f(a.act + (size_t)seq * F + pr * 16 + row, gate / (1.0f + expf(-gate)) * up);
        }
        __syncthreads();
      }
      // next: down projection (stage 5)
      if (wg < d_units) {
        const int t = wg / a.ks_d, s = wg % a.ks_d;
        pf_issue<1>(pf, L.wd, (size_t)t, KTF, s * kts_d, min(KTF, (s + 1) * kts_d));
      }
      stamp(step);
      if (!grid_barrier(a, epoch)) return;
      stamp(step);

      // ================= stage 5: down projection (k slices) =================
      for (int u = wg; u < d_units; u += nwg) {
        const int t = u / a.ks_d, s = u % a.ks_d;
        const int kt0 = s * kts_d, kt1 = min(KTF, (s + 1) * kts_d);
        __syncthreads();
        for (int b = 0; b < nseq; ++b) {
          float2 av[4];  // a slice is at most 4096 wide: four pairs per thread, loaded together
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int k = kt0 * 32 + 2 * (tid + MK_THREADS * j);
            if (k < kt1 * 32) av[j] = ld_f2(a.act + (size_t)b * F + k);
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int k = kt0 * 32 + 2 * (tid + MK_THREADS * j);
            if (k < kt1 * 32) put_pair(opnd, NC, b, k - kt0 * 32, av[j]);
          }
        }
        __syncthreads();
        if (u == wg)
          gemm_unit<1, true>(sm, L.wd, (size_t)t, KTF, kt0, kt1, pf, opnd, kt0, NC, ncols);
        else
          gemm_unit<1, false>(sm, L.wd, (size_t)t, KTF, kt0, kt1, pf, opnd, kt0, NC, ncols);
        __syncthreads();
        if (tid < 16 * nseq) {
          const int seq = tid >> 4, row = tid & 15;
          st_f(a.dpart + (size_t)s * pstride + (size_t)seq * H + t * 16 + row, tile_total(sm, 0, row, seq));
        }
      }
      // next: QKV of the next layer (the LM head streams on its own)
      if (li + 1 < a.n_layers && wg < qkv_tiles) pf_issue<1>(pf, a.layers[li + 1].wqkv, (size_t)wg, KTH, 0, KTH);
      stamp(step);
      if (!grid_barrier(a, epoch)) return;

      // the residual stream written in stage 4 becomes the input of the next layer
      float* tmp = Xa;
      Xa = Xb;
      Xb = tmp;
    }

    stamp(step);
    // ================= final norm + LM head + arg-max =================
    for (int b = 0; b < nseq; ++b) {
      float2 xv[NP];
#pragma unroll
      for (int j = 0; j < NP; ++j) xv[j] = make_float2(0.f, 0.f);
      gather_resid(xv, H, Xa + (size_t)b * H, a.dpart + (size_t)b * H, a.ks_d, nullptr, 0, pstride);
      norm_pack(sm, opnd, NC, b, H, a.eps, xv, a.g_final);
    }
    __syncthreads();
    {
      // every wave walks whole 16-row tiles of the vocabulary on its own (no k split,
      // no workgroup synchronisation): tile = global wave index, stride = all waves
      const int c16 = lane & 15, g = lane >> 4;
      const bool colok = c16 < ncols;
      float best[5];
      int besti[5];
#pragma unroll
      for (int b = 0; b < 5; ++b) {
        best[b] = -INFINITY;
        besti[b] = 0x7fffffff;
      }
      float* lg = a.logits ? a.logits + (size_t)step * nseq * V : nullptr;
      for (int t = wg * MK_WAVES + wave; t < v_tiles; t += nwg * MK_WAVES) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        const uint4* Wt = a.lm_head + (size_t)t * KTH * 64 + lane;
        for (int kt0 = 0; kt0 < KTH; kt0 += 8) {
          uint4 av[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) av[u] = kt0 + u < KTH ? Wt[(size_t)(kt0 + u) * 64] : uint4{0, 0, 0, 0};
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            uint4 bv = uint4{0, 0, 0, 0};
            if (kt0 + u < KTH && colok) bv = opnd[((size_t)(kt0 + u) * 4 + g) * NC + c16];
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[u]),
                                                          __builtin_bit_cast(bf16x8, bv), acc, 0, 0, 0);
          }
        }
        // add the three pieces: columns 3b, 3b+1, 3b+2 sit in adjacent lanes
        f32x4 s;
#pragma unroll
        for (int i = 0; i < 4; ++i) s[i] = acc[i] + __shfl_down(acc[i], 1, 64) + __shfl_down(acc[i], 2, 64);
        const int seq = c16 / 3;
        if (c16 % 3 == 0 && seq < nseq) {
          const int row0 = t * 16 + g * 4;
          if (lg) *reinterpret_cast<float4*>(lg + (size_t)seq * V + row0) = make_float4(s[0], s[1], s[2], s[3]);
#pragma unroll
          for (int b = 0; b < 5; ++b)
            if (b == seq) {
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (s[i] > best[b]) {  // rows increase, strict > keeps the lowest index
                  best[b] = s[i];
                  besti[b] = row0 + i;
                }
            }
        }
      }
      // lanes that own sequence b: c16 == 3b, four of them (g = 0..3) per wave
#pragma unroll
      for (int b = 0; b < 5; ++b) {
        float v = best[b];
        int i = besti[b];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
          const float ov = __shfl_xor(v, o, 64);
          const int oi = __shfl_xor(i, o, 64);
          if (ov > v || (ov == v && oi < i)) {
            v = ov;
            i = oi;
          }
        }
        if (lane == 0 && b < nseq) {
          sm.bestv[wave][b] = v;
          sm.besti[wave][b] = i;
        }
      }
      __syncthreads();
      if (tid < nseq) {
        float v = sm.bestv[0][tid];
        int i = sm.besti[0][tid];
        for (int w = 1; w < MK_WAVES; ++w) {
          const float ov = sm.bestv[w][tid];
          const int oi = sm.besti[w][tid];
          if (ov > v || (ov == v && oi < i)) {
            v = ov;
            i = oi;
          }
        }
        st_f(a.am_val + (size_t)wg * nseq + tid, v);
        st_u32(reinterpret_cast<unsigned*>(a.am_idx) + (size_t)wg * nseq + tid, (unsigned)i);
      }
    }
    if (step + 1 < a.n_steps && wg < qkv_tiles) pf_issue<1>(pf, a.layers[0].wqkv, (size_t)wg, KTH, 0, KTH);
    stamp(step);
    if (!grid_barrier(a, epoch)) return;
    stamp(step);

    // every workgroup reduces the per-workgroup winners itself: the next token needs no
    // further exchange
    if (wave < nseq) {
      float v = -INFINITY;
      int i = 0x7fffffff;
      for (int w0 = lane; w0 < nwg; w0 += 256) {
        float ov[4];
        int oi[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int w = min(w0 + 64 * q, nwg - 1);
          ov[q] = ld_f(a.am_val + (size_t)w * nseq + wave);
          oi[q] = (int)ld_u32(reinterpret_cast<const unsigned*>(a.am_idx) + (size_t)w * nseq + wave);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (w0 + 64 * q < nwg && (ov[q] > v || (ov[q] == v && oi[q] < i))) {
            v = ov[q];
            i = oi[q];
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
        sm.tok[wave] = t;
        if (wg == 0) a.token_log[(size_t)step * nseq + wave] = t;
      }
    }
    __syncthreads();
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

// Operand bytes in LDS: the widest k range any stage holds at once.
size_t mk_opnd_bytes(const MkPlan& p) {
  const int NC = p.nseq == 1 ? 4 : 16;
  const int kts_o = (p.nq * 128 / 32 + p.ks_o - 1) / p.ks_o, kts_d = (p.F / 32 + p.ks_d - 1) / p.ks_d;
  int kt = p.H / 32;
  if (kts_o > kt) kt = kts_o;
  if (kts_d > kt) kt = kts_d;
  return (size_t)kt * 4 * NC * 16;
}

hipError_t launch_decode_persistent(hipStream_t s, const MkPlan& p, const MkBuffers& bf) {
  MkArgs a{};
  a.layers = static_cast<const MkLayer*>(bf.layers);
  a.n_layers = p.n_layers; a.H = p.H; a.nq = p.nq; a.nkv = p.nkv; a.F = p.F; a.V = p.V;
  a.eps = p.eps;
  a.embed = static_cast<const uint4*>(bf.embed);
  a.lm_head = static_cast<const uint4*>(bf.lm_head);
  a.g_final = bf.g_final;
  a.rope = bf.rope;
  a.max_seq = p.max_seq;
  a.flags = bf.flags; a.error = bf.error;
  a.st = bf.st;
  a.nseq = p.nseq; a.n_steps = p.n_steps;
  a.ks_o = p.ks_o; a.ks_d = p.ks_d;
  a.X0 = bf.X0; a.X1 = bf.X1; a.qkv = bf.qkv; a.att = bf.att; a.max_chunks = p.max_chunks;
  a.opart = bf.opart; a.act = bf.act; a.dpart = bf.dpart; a.am_val = bf.am_val; a.am_idx = bf.am_idx;
  a.logits = bf.logits; a.token_log = bf.token_log;
  a.trace = bf.trace; a.trace_step = bf.trace_step; a.trace_points = bf.trace_points;
  const size_t dyn = mk_opnd_bytes(p);
  const int G = p.nq / p.nkv;
  hipError_t e;
#define MK_LAUNCH(GH, NP)                                                                                        \
  do {                                                                                                           \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_persistent<GH, NP>),                         \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);                               \
    if (e != hipSuccess) return e;                                                                               \
    k_decode_persistent<GH, NP><<<p.nwg, MK_THREADS, dyn, s>>>(a);                                               \
  } while (0)
#define MK_LAUNCH_NP(GH)              \
  do {                                \
    if (p.H <= 1024) MK_LAUNCH(GH, 1); \
    else if (p.H <= 2048) MK_LAUNCH(GH, 2); \
    else MK_LAUNCH(GH, 4);            \
  } while (0)
  if (p.H > 4096 || p.ks_o > MK_MAX_KS || p.ks_d > MK_MAX_KS) return hipErrorInvalidValue;
  if (G % 4 == 0) MK_LAUNCH_NP(4);
  else if (G % 2 == 0) MK_LAUNCH_NP(2);
  else MK_LAUNCH_NP(1);
#undef MK_LAUNCH_NP
#undef MK_LAUNCH
  return hipGetLastError();
}

}  // namespace nnc
