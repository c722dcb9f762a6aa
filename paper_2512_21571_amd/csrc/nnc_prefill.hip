// Prompt-pass kernels for large token blocks (bf16 models): an LDS-staged matrix-core GEMM
// over the packed weights, and the row-wise passes that produce its operands.
//
// This is the compute-bound side of the path: with T tokens every weight byte is used T
// times, so the matmuls run at matrix-core speed, not HBM speed.  As in the paper's packed
// "pass-through" chain (Section 3.1.2, Eq. (1)) activations stay in the blocked layout of
// the tensor unit between operators: norms, the SwiGLU epilogue and the attention merge
// write bf16 values directly in the fragment order the next GEMM loads, and nothing is
// unpacked in between.  Activations entering a GEMM are rounded to bf16 once (round to
// nearest even): that is the precision contract of this path.
#include "nnc_half.h"
#include "nnc_internal.h"
#include "nnc_lanes.h"

#include <type_traits>
#include <utility>

namespace nnc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

// Workgroup barrier that orders LDS traffic only: the global loads of the register ring stay
// in flight across it (a plain __syncthreads() would wait for all of them at every k step).
__device__ __forceinline__ void lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a
// compile-time constant in the body, so register arrays indexed by it stay in registers.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Block tile: NT row tiles (16 rows each) x TT column tiles (16 operand columns each), k step
// 32.  4 waves in a 2 x 2 arrangement, each NT/2 x TT/2 accumulator tiles.
//   NT = 16, TT = 8  (256 x 128, 128 x 64 per wave): the matrix-core-bound shape; per k step a
//                    wave reads 12 fragments from LDS for 32 matrix-core instructions.
//   NT = 12, TT = 8  (192 x 128) and NT = 8, TT = 8 (128 x 128): launches whose 256 x 128
//                    workgroups would fill the last round of two per CU badly.
//   NT = 4,  TT = 8  (64 x 128): short prompts, where the launch would otherwise leave most of
//                    the chip idle.
//   NT = 4,  TT = 4  (64 x 64): the same, for launches that even so have fewer workgroups than CUs.
// PIECES = 1: one bf16 per activation, a column tile is 16 tokens.  PIECES = 2: every
// activation is carried as two bf16 pieces (value, remainder) in adjacent column tiles, whose
// products the epilogue adds: fp32-grade activations at twice the matrix-core work, which is
// free while the GEMM is bound by streaming the weights (short prompts).

}  // namespace

// Epilogue of the prompt GEMMs for one token tile: v[i] = the accumulators (pieces already added)
// of the wave's row tiles nt_first + i for column tile `ct` (token tile ct / PIECES).
// accumulator element e of lane l: row (l / 16) * 4 + e of the row tile, operand column l % 16.
template <int EPI, int WI, int PIECES, class HF>
__device__ __forceinline__ void pg_epilogue_col_impl(const PrefillGemmArgs& a, const f32x4 (&v)[WI], int nt_first, int ct,
                                                     int lane, int kslice) {
  // Every product and sum below is rounded on its own: the block tiles promise the same bits, and
  // left free the compiler contracts e.g. the last product inside expf with the "1 +" that follows
  // in one tile's instantiation and not in another's.
#pragma clang fp contract(off)
  const int c16 = lane & 15, g = lane >> 4;
  const int tt = ct / PIECES;        // token tile
  const size_t t = (size_t)tt * 16 + c16;
  if constexpr (EPI == EPI_SWIGLU) {
    // row tiles come as (gate, up) pairs; feature tile = row tile / 2
    const int FKT = a.n_tiles / 4;  // k tiles of the next GEMM: features / 32
#pragma unroll
    for (int i = 0; i < WI; i += 2) {
      const int nt = nt_first + i;
      if (nt >= a.n_tiles) continue;
      const int f0 = (nt >> 1) * 16 + g * 4;
      uint32_t h[PIECES][4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float gate = v[i][e], up = v[i + 1][e];
        float act = gate / (1.0f + expf(-gate)) * up;
#pragma unroll
        for (int pc = 0; pc < PIECES; ++pc) {
          h[pc][e] = HF::bits(act);
          act -= HF::widen(h[pc][e]);
        }
      }
      // features f0 .. f0+3 of token t: 8 bytes inside one 16-byte fragment element
#pragma unroll
      for (int pc = 0; pc < PIECES; ++pc) {
        const size_t el =
            (((size_t)(tt * PIECES + pc) * FKT + (f0 >> 5)) * 64 + c16 + 16 * ((f0 & 31) >> 3)) * 8 + (f0 & 7);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.packed_out) + el) =
            make_uint2(h[pc][0] | (h[pc][1] << 16), h[pc][2] | (h[pc][3] << 16));
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < WI; ++i) {
      const int nt = nt_first + i;
      if (nt >= a.n_tiles) continue;
      // k slice 0 owns the output; slice s > 0 stores its partial sums in buffer s - 1, which
      // the next norm kernel adds in a fixed order
      float* base = kslice == 0 ? a.out : a.part + (size_t)(kslice - 1) * a.part_stride;
      float4* dst = reinterpret_cast<float4*>(base + t * a.ldo + (size_t)nt * 16 + g * 4);
      float4 o = make_float4(v[i][0], v[i][1], v[i][2], v[i][3]);
      if constexpr (EPI == EPI_RESID) {
        if (kslice == 0) {
          const float4 p = *dst;
          o = make_float4(p.x + o.x, p.y + o.y, p.z + o.z, p.w + o.w);
        }
      }
      *dst = o;
    }
  }
}

template <int EPI, int WI, int PIECES, class HF>
__device__ __forceinline__ void pg_epilogue_col(const PrefillGemmArgs& a, const f32x4 (&v)[WI], int nt_first, int ct,
                                                int lane, int kslice) {
  if (a.wscale) {
    // byte weights: the sums are over the bytes; the row's scale makes them the products.  The
    // product is rounded on its own: left free, the compiler fuses it with the residual add in
    // one instantiation and not in another, and the block tiles stop giving the same bits.
#pragma clang fp contract(off)
    const int g = lane >> 4;
    f32x4 sv[WI];
#pragma unroll
    for (int i = 0; i < WI; ++i) {
      const int nt = min(nt_first + i, a.n_tiles - 1);
      const float4 sc = *reinterpret_cast<const float4*>(a.wscale + (size_t)nt * 16 + g * 4);
      sv[i] = f32x4{v[i][0] * sc.x, v[i][1] * sc.y, v[i][2] * sc.z, v[i][3] * sc.w};
    }
    pg_epilogue_col_impl<EPI, WI, PIECES, HF>(a, sv, nt_first, ct, lane, kslice);
  } else {
    pg_epilogue_col_impl<EPI, WI, PIECES, HF>(a, v, nt_first, ct, lane, kslice);
  }
}

// Epilogue of the prompt GEMMs: the accumulators of wave (wn, wt) of the block at (nt0, tt0).
// With two pieces, column tiles 2q and 2q+1 are the two pieces of token tile q and their
// accumulators are added.
template <int EPI, int NT, int TT, int PIECES, class HF>
__device__ __forceinline__ void pg_epilogue(const PrefillGemmArgs& a, f32x4 (&acc)[NT / 2][TT / 2], int nt0, int tt0,
                                            int wn, int wt, int lane, int kslice = 0) {
  constexpr int WI = NT / 2, WJ = TT / 2;
#pragma unroll
  for (int j = 0; j < WJ; j += PIECES) {
    const int ct = tt0 + wt * WJ + j;  // column tile
    if (ct >= a.t_tiles) continue;
    f32x4 v[WI];
#pragma unroll
    for (int i = 0; i < WI; ++i) {
      v[i] = acc[i][j];
      if constexpr (PIECES == 2) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[i][e] += acc[i][j + 1][e];
      }
    }
    pg_epilogue_col<EPI, WI, PIECES, HF>(a, v, nt0 + wn * WI, ct, lane, kslice);
  }
}

// Both operands are already stored in fragment order in memory (1 KiB per 16 x 32 tile, one
// 16-byte element per lane), so staging is a straight copy: global -> registers -> LDS, and
// every LDS access is a conflict-free 16-byte access at lane * 16.  Double-buffered in LDS,
// fed from a register ring eight k steps deep; one workgroup barrier per k step.  This is the
// kernel of the small block tiles (64 rows: short prompts, bound by streaming the weights, where
// the deep ring matters); the large tiles use k_gemm_prefill_dl below.
template <int EPI, int NT, int TT, int PIECES, class HF>
__global__ __launch_bounds__(256, 2) void k_gemm_prefill(PrefillGemmArgs a) {
  constexpr int WI = NT / 2;   // row tiles per wave
  constexpr int AL = NT / 4;   // 16-byte A loads per thread and k step
  constexpr int WJ = TT / 2;   // column tiles per wave
  constexpr int BL = TT / 4;   // 16-byte B loads per thread and k step
  __shared__ u32x4 As[2][NT][64];
  __shared__ u32x4 Bs[2][TT][64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wn = wave >> 1, wt = wave & 1;
  // blockIdx.z = k slice (narrow launches of short prompts split k for more workgroups)
  const int kts = a.kts_per_split > 0 ? a.kts_per_split : a.KT;
  const int kt_first = blockIdx.z * kts;
  const int KT = min(a.KT, kt_first + kts) - kt_first;  // k steps of this slice
  const int nt0 = blockIdx.x * NT, tt0 = blockIdx.y * TT;
  const u32x4* __restrict__ W = static_cast<const u32x4*>(a.Wp) + (size_t)kt_first * 64;
  const u32x4* __restrict__ X = static_cast<const u32x4*>(a.Xf) + (size_t)kt_first * 64;

  f32x4 acc[WI][WJ];
#pragma unroll
  for (int i = 0; i < WI; ++i)
#pragma unroll
    for (int j = 0; j < WJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Register ring of D k steps: the loads of step kt + D are issued when step kt starts, so D
  // steps of matrix-core work cover the memory latency even with one workgroup per CU.
  constexpr int D = 8;  // even
  u32x4 ra[D][AL], rb[D][BL];  // native vectors: arrays of the HIP uint4 struct end up in scratch memory
  // Load addresses = wave-uniform base of the k step (scalar registers) + a per-thread 32-bit
  // byte offset fixed for the whole kernel (tile indices clamped to the last valid one: rows /
  // columns past the edge compute garbage that is never stored).  The steady-state loop thus
  // has no vector address arithmetic and no data-dependent branch, and the compiler waits per
  // ring stage.
  uint32_t voa[AL], vob[BL];
#pragma unroll
  for (int j = 0; j < AL; ++j) {
    const int idx = tid + 256 * j, tile = min(nt0 + (idx >> 6), a.n_tiles - 1);
    voa[j] = ((uint32_t)tile * (uint32_t)a.KT * 64u + (uint32_t)(idx & 63)) * 16u;
  }
#pragma unroll
  for (int j = 0; j < BL; ++j) {
    const int idx = tid + 256 * j, tile = min(tt0 + (idx >> 6), a.t_tiles - 1);
    vob[j] = ((uint32_t)tile * (uint32_t)a.KT * 64u + (uint32_t)(idx & 63)) * 16u;
  }
  auto gload = [&](auto stc, int kt) __attribute__((always_inline)) {
    constexpr int st = decltype(stc)::value;
    const char* wb = reinterpret_cast<const char*>(W) + (size_t)kt * 1024;
    const char* xb = reinterpret_cast<const char*>(X) + (size_t)kt * 1024;
#pragma unroll
    for (int j = 0; j < AL; ++j) ra[st][j] = *reinterpret_cast<const u32x4*>(wb + voa[j]);
#pragma unroll
    for (int j = 0; j < BL; ++j) rb[st][j] = *reinterpret_cast<const u32x4*>(xb + vob[j]);
  };
  auto sstore = [&](auto stc, auto bufc) __attribute__((always_inline)) {
    constexpr int st = decltype(stc)::value, buf = decltype(bufc)::value;
#pragma unroll
    for (int j = 0; j < AL; ++j) {
      const int idx = tid + 256 * j;
      As[buf][idx >> 6][idx & 63] = ra[st][j];
    }
#pragma unroll
    for (int j = 0; j < BL; ++j) {
      const int idx = tid + 256 * j;
      Bs[buf][idx >> 6][idx & 63] = rb[st][j];
    }
  };
  // One k step: ring stage d holds step kt (already copied to LDS buffer d & 1; D is even).
  // LOAD: the step D ahead exists and is fetched into the stage that this step frees.
  auto step = [&](int kt, auto dc, auto loadc) __attribute__((always_inline)) {
    constexpr int d = decltype(dc)::value;
    if constexpr (decltype(loadc)::value) gload(dc, kt + D);
    u32x4 af[WI], bf[WJ];
#pragma unroll
    for (int i = 0; i < WI; ++i) af[i] = As[d & 1][wn * WI + i][lane];
#pragma unroll
    for (int j = 0; j < WJ; ++j) bf[j] = Bs[d & 1][wt * WJ + j][lane];
#pragma unroll
    for (int i = 0; i < WI; ++i)
#pragma unroll
      for (int j = 0; j < WJ; ++j)
        acc[i][j] = HF::mfma(af[i], bf[j], acc[i][j]);
    // step kt + 1 into the other buffer (past the end: a stale copy nobody reads)
    sstore(std::integral_constant<int, (d + 1) % D>{}, std::integral_constant<int, (d + 1) & 1>{});
    lds_sync();
  };

  // prologue: the first min(D, KT) steps into the ring, step 0 into LDS
  static_for<D>([&](auto dc) __attribute__((always_inline)) {
    if (decltype(dc)::value < KT) gload(dc, decltype(dc)::value);
  });
  sstore(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
  lds_sync();
  int kt0 = 0;
  // steady state: whole rounds of D steps whose look-ahead loads all exist
  for (; kt0 + 2 * D <= KT; kt0 += D)
    static_for<D>([&](auto dc) __attribute__((always_inline)) {
      step(kt0 + decltype(dc)::value, dc, std::true_type{});
    });
  // the last steps (fewer than 2 D), without look-ahead loads past the end
  for (; kt0 < KT; kt0 += D)
    static_for<D>([&](auto dc) __attribute__((always_inline)) {
      const int kt = kt0 + decltype(dc)::value;
      if (kt < KT) {
        if (kt + D < KT) gload(dc, kt + D);
        step(kt, dc, std::false_type{});
      }
    });

  pg_epilogue<EPI, NT, TT, PIECES, HF>(a, acc, nt0, tt0, wn, wt, lane, (int)blockIdx.z);
}

// The same GEMM with the operands copied global -> LDS directly (16 bytes per lane, a wave's 64
// lanes land on 1 KiB contiguous: exactly one fragment), without passing through registers.
// Three LDS stages and two register sets of fragments: when step kt starts, the copies of step
// kt + 3 are issued into the stage whose fragments step kt already holds in registers, and the
// fragments of step kt + 1 are read while the matrix cores work on step kt; one barrier per k
// step.
template <int EPI, int NT, int TT, int PIECES, class HF>
__global__ __launch_bounds__(256, 2) void k_gemm_prefill_dl(PrefillGemmArgs a) {
  constexpr int WI = NT / 2, AL = NT / 4, WJ = TT / 2, BL = TT / 4;
  constexpr int ST = 3;
  __shared__ u32x4 As[ST][NT][64];
  __shared__ u32x4 Bs[ST][TT][64];
  // (the wave index as a scalar: the LDS addresses of the copies below are then scalar arithmetic
  // instead of a vector op + lane read in front of every copy)
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int wn = wave >> 1, wt = wave & 1;
  // blockIdx.z = k slice (residual projections whose tiles alone would leave CUs idle)
  const int kts = a.kts_per_split > 0 ? a.kts_per_split : a.KT;
  const int kt_first = blockIdx.z * kts;
  const int KT = min(a.KT, kt_first + kts) - kt_first;  // k steps of this slice
  const int nt0 = blockIdx.x * NT, tt0 = blockIdx.y * TT;
  const char* __restrict__ W = static_cast<const char*>(a.Wp) + (size_t)kt_first * 1024;
  const char* __restrict__ X = static_cast<const char*>(a.Xf) + (size_t)kt_first * 1024;

  f32x4 acc[WI][WJ];
#pragma unroll
  for (int i = 0; i < WI; ++i)
#pragma unroll
    for (int j = 0; j < WJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // wave w copies fragments w, w + 4, ...; per-thread byte offsets are fixed for the kernel
  // (tile indices clamped to the last valid one: rows / columns past the edge compute garbage
  // that is never stored)
  uint32_t voa[AL], vob[BL];
#pragma unroll
  for (int j = 0; j < AL; ++j) voa[j] = ((uint32_t)min(nt0 + wave + 4 * j, a.n_tiles - 1) * (uint32_t)a.KT * 64u + lane) * 16u;
#pragma unroll
  for (int j = 0; j < BL; ++j) vob[j] = ((uint32_t)min(tt0 + wave + 4 * j, a.t_tiles - 1) * (uint32_t)a.KT * 64u + lane) * 16u;
  // The copy instruction is written as inline assembly: the compiler, when it sees one, makes
  // every later LDS read wait for all of them (it cannot tell which stage a read touches), which
  // would undo the look-ahead.  Hidden from it, the waits are the explicit ones below.
  // m0 = LDS byte address of the fragment (wave-uniform); lane l's 16 bytes land at m0 + 16 l.
  typedef __attribute__((address_space(3))) void* lptr;
  auto copy1 = [&](const char* base, uint32_t voff, uint32_t lds_addr) __attribute__((always_inline)) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(base)
                 : "memory", "m0");
  };
  auto issue = [&](int kt, int st) __attribute__((always_inline)) {
    const size_t ko = (size_t)kt * 1024;
#pragma unroll
    for (int j = 0; j < AL; ++j) copy1(W + ko, voa[j], (uint32_t)(size_t)(lptr)&As[st][wave + 4 * j][0]);
#pragma unroll
    for (int j = 0; j < BL; ++j) copy1(X + ko, vob[j], (uint32_t)(size_t)(lptr)&Bs[st][wave + 4 * j][0]);
  };
  // s_waitcnt vmcnt(n) with the other counters left alone
  constexpr int L = AL + BL;  // copy instructions per wave and k step
  auto wait_vm = [](auto nc) __attribute__((always_inline)) {
    constexpr int n = decltype(nc)::value;
    __builtin_amdgcn_s_waitcnt((n & 0xf) | (7 << 4) | (15 << 8) | ((n >> 4) << 14));
  };
  // Fragments live in two register sets: while the matrix cores work on step kt (set kt & 1),
  // the fragments of step kt + 1 are read from LDS into the other set.
  u32x4 af[2][WI], bf[2][WJ];
  auto read_frags = [&](auto setc, int st) __attribute__((always_inline)) {
    constexpr int P = decltype(setc)::value;
#pragma unroll
    for (int i = 0; i < WI; ++i) af[P][i] = As[st][wn * WI + i][lane];
#pragma unroll
    for (int j = 0; j < WJ; ++j) bf[P][j] = Bs[st][wt * WJ + j][lane];
  };
  constexpr std::integral_constant<int, 0> c0{};
  constexpr std::integral_constant<int, 1> c1{};
  constexpr std::integral_constant<int, L> cL{};
  constexpr std::integral_constant<int, 2 * L> c2L{};
  // Step kt: stage kt % 3 is already in registers and free again, stage (kt + 1) % 3 must have
  // landed (its copies were issued two steps ago), stage (kt + 2) % 3 is in flight.
  auto step = [&](auto setc, int kt, int st) __attribute__((always_inline)) {
    constexpr int P = decltype(setc)::value;
    if (kt + 2 < KT) wait_vm(cL);  // all but the newest issue
    else wait_vm(c0);
    lds_sync();
    if (kt + 3 < KT) issue(kt + 3, st);
    if (kt + 1 < KT) read_frags(std::integral_constant<int, 1 - P>{}, st == 2 ? 0 : st + 1);
#pragma unroll
    for (int i = 0; i < WI; ++i)
#pragma unroll
      for (int j = 0; j < WJ; ++j)
        acc[i][j] = HF::mfma(af[P][i], bf[P][j], acc[i][j]);
  };
  issue(0, 0);
  if (KT > 1) issue(1, 1);
  if (KT > 2) issue(2, 2);
  if (KT > 2) wait_vm(c2L);
  else if (KT > 1) wait_vm(cL);
  else wait_vm(c0);
  lds_sync();
  read_frags(c0, 0);
  int st = 0;
  for (int kt = 0; kt < KT; kt += 2) {
    step(c0, kt, st);
    st = st == 2 ? 0 : st + 1;
    if (kt + 1 < KT) {
      step(c1, kt + 1, st);
      st = st == 2 ? 0 : st + 1;
    }
  }
  pg_epilogue<EPI, NT, TT, PIECES, HF>(a, acc, nt0, tt0, wn, wt, lane, (int)blockIdx.z);
}

// 256 x 256 block tile, one workgroup per CU, 128 x 128 per wave: per k step a wave reads 16
// fragments from LDS for 64 matrix-core instructions (0.25 KiB per instruction against 0.375 for
// the 128 x 64 wave tile above), which is what the large-tile kernel above is bound by.  The
// 64 accumulator tiles fill the wave's 256 accumulation registers; the compiler, asked to keep
// them there, shuffles them through the ordinary registers every k step, so the kernel names
// them itself: tile (i, j) lives in a[(8 i + j) * 4 .. + 3] and the matrix-core instructions,
// the zeroing and the read-out are inline assembly with those names.  Being opaque to the
// compiler they get no automatic wait states: the ones the hardware needs between a write of an
// accumulation register and a product that reads it, and between the last product and the first
// read of its result, are put in by hand (s_nop).  The copies and fragment reads of the next
// steps are placed one at a time behind single products (one wave per SIMD: nothing else hides
// their issue slots); compiler barriers keep that order.
template <class HF, int N>
__device__ __forceinline__ void big_mfma(u32x4 a, u32x4 b) {
  if constexpr (HF::kDtype == DT_F16)
    asm volatile("v_mfma_f32_16x16x32_f16 a[%2:%3], %0, %1, a[%2:%3]" : : "v"(a), "v"(b), "n"(N), "n"(N + 3));
  else
    asm volatile("v_mfma_f32_16x16x32_bf16 a[%2:%3], %0, %1, a[%2:%3]" : : "v"(a), "v"(b), "n"(N), "n"(N + 3));
}
template <int N>
__device__ __forceinline__ f32x4 big_acc_read() {
  f32x4 v;
  asm volatile("v_accvgpr_read_b32 %0, a[%4]\n\tv_accvgpr_read_b32 %1, a[%5]\n\t"
               "v_accvgpr_read_b32 %2, a[%6]\n\tv_accvgpr_read_b32 %3, a[%7]"
               : "=v"(v[0]), "=v"(v[1]), "=v"(v[2]), "=v"(v[3])
               : "n"(N), "n"(N + 1), "n"(N + 2), "n"(N + 3));
  return v;
}
template <int N>
__device__ __forceinline__ void big_acc_zero() {
  asm volatile("v_accvgpr_write_b32 a[%0], 0\n\tv_accvgpr_write_b32 a[%1], 0\n\t"
               "v_accvgpr_write_b32 a[%2], 0\n\tv_accvgpr_write_b32 a[%3], 0"
               :
               : "n"(N), "n"(N + 1), "n"(N + 2), "n"(N + 3));
}

template <int EPI, int PIECES, class HF, int NT>
__global__ __launch_bounds__(256, 1) void k_gemm_prefill_big(PrefillGemmArgs a) {
  // NT = 16: 256 x 256; NT = 12: 192 x 256 (96 x 128 per wave), for launches whose 256-row blocks
  // would leave the last round of one workgroup per CU half empty
  constexpr int TT = 16, WI = NT / 2, WJ = 8, AL = NT / 4, BL = 4;
  // Three LDS stages (a fourth changed nothing: the copies are not bound by latency).
  constexpr int ST = 3;
  __shared__ u32x4 As[ST][NT][64];
  __shared__ u32x4 Bs[ST][TT][64];
  // (the wave index as a scalar: the LDS addresses of the copies below are then scalar arithmetic
  // instead of a vector op + lane read in front of every copy)
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int wn = wave >> 1, wt = wave & 1;
  // blockIdx.z = k slice (residual projections whose tiles alone would leave CUs idle)
  const int kts = a.kts_per_split > 0 ? a.kts_per_split : a.KT;
  const int kt_first = blockIdx.z * kts;
  const int KT = min(a.KT, kt_first + kts) - kt_first;  // k steps of this slice
  // Block order.  The workgroups resident together (one per CU, 256 at a time in launch order)
  // should share operands: panels of 16 row blocks x all column blocks, and inside a panel groups of
  // 16 x 16 blocks.  The hardware deals consecutive workgroups to the 8 XCDs in turn, so within a
  // group XCD x takes a patch of 4 row blocks x 8 column blocks: its L2 then serves 12 operand
  // streams to its 32 workgroups instead of 18.
  int bx, by;
  {
    const int gx = gridDim.x, gy = gridDim.y;
    const int w = blockIdx.x + gx * blockIdx.y;
    const int p = w / (16 * gy), within = w - p * 16 * gy;
    const int rows = min(16, gx - p * 16);
    if (rows == 16 && gy % 16 == 0) {
      const int grp = within / 256, wi = within - grp * 256;
      const int xcd = wi & 7, l = wi >> 3;
      bx = p * 16 + (xcd >> 1) * 4 + (l & 3);
      by = grp * 16 + (xcd & 1) * 8 + (l >> 2);
    } else {
      bx = p * 16 + within % rows;
      by = within / rows;
    }
  }
  const int nt0 = bx * NT, tt0 = by * TT;
  const char* __restrict__ W = static_cast<const char*>(a.Wp) + (size_t)kt_first * 1024;
  const char* __restrict__ X = static_cast<const char*>(a.Xf) + (size_t)kt_first * 1024;

  // every accumulation register is this kernel's: naming the first and the last as clobbered makes
  // the compiler allocate all 256 to the wave.  It has no reason to touch them itself (the kernel
  // needs about 150 ordinary registers), and the library is built with the compiler's
  // "spill ordinary registers into accumulation registers" option off, so it never does.
  asm volatile("" ::: "a0", "a255");
  static_for<WI * WJ>([&](auto n) __attribute__((always_inline)) { big_acc_zero<decltype(n)::value * 4>(); });

  uint32_t voa[AL], vob[BL];
#pragma unroll
  for (int j = 0; j < AL; ++j) voa[j] = ((uint32_t)min(nt0 + wave + 4 * j, a.n_tiles - 1) * (uint32_t)a.KT * 64u + lane) * 16u;
#pragma unroll
  for (int j = 0; j < BL; ++j) vob[j] = ((uint32_t)min(tt0 + wave + 4 * j, a.t_tiles - 1) * (uint32_t)a.KT * 64u + lane) * 16u;
  typedef __attribute__((address_space(3))) void* lptr;
  auto copy1 = [&](const char* base, uint32_t voff, uint32_t lds_addr) __attribute__((always_inline)) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(base)
                 : "memory", "m0");
  };
  // copy number c (0 .. 7) of k step kt into stage st: four weight fragments, four operand fragments
  auto issue1 = [&](auto cc, int kt, int st) __attribute__((always_inline)) {
    constexpr int c = decltype(cc)::value;
    const size_t ko = (size_t)kt * 1024;
    if constexpr (c < AL) copy1(W + ko, voa[c], (uint32_t)(size_t)(lptr)&As[st][wave + 4 * c][0]);
    else copy1(X + ko, vob[c - AL], (uint32_t)(size_t)(lptr)&Bs[st][wave + 4 * (c - AL)][0]);
  };
  auto issue = [&](int kt, int st) __attribute__((always_inline)) {
    static_for<AL + BL>([&](auto cc) __attribute__((always_inline)) { issue1(cc, kt, st); });
  };
  constexpr int L = AL + BL;
  auto wait_vm = [](auto nc) __attribute__((always_inline)) {
    constexpr int n = decltype(nc)::value;
    __builtin_amdgcn_s_waitcnt((n & 0xf) | (7 << 4) | (15 << 8) | ((n >> 4) << 14));
  };
  // wait until at most r whole steps of copies (r <= ST - 2) are still in flight
  auto wait_steps = [&](int r) __attribute__((always_inline)) {
    if (r >= 2 && ST >= 4) wait_vm(std::integral_constant<int, 2 * L>{});
    else if (r >= 1) wait_vm(std::integral_constant<int, L>{});
    else wait_vm(std::integral_constant<int, 0>{});
  };
  u32x4 af[2][WI], bf[2][WJ];
  constexpr std::integral_constant<int, 0> c0{};
  constexpr std::integral_constant<int, 1> c1{};
  // Step kt (fragments in register set P): stage kt % ST is in registers and free, stage
  // (kt + 1) % ST must have landed, the stages after it are in flight.  Group g = copy g of step
  // kt + ST (MORE), fragments of step kt + 1 into the other set (NEXT), interleaved with the 64 products.
  auto step = [&](auto setc, auto morec, auto nextc, int kt, int st) __attribute__((always_inline)) {
    constexpr int P = decltype(setc)::value;
    constexpr bool MORE = decltype(morec)::value, NEXT = decltype(nextc)::value;
    if constexpr (MORE) wait_vm(std::integral_constant<int, (ST - 2) * L>{});
    else wait_steps(min(KT - kt - 2, ST - 2));
    lds_sync();
    const int nx = st == ST - 1 ? 0 : st + 1;
    // One wave per SIMD: the wave's issue pointer is never more than one product ahead of the
    // matrix core, so everything else has to fit into the 16 cycles a product runs, one
    // instruction (or one copy: scalar add, m0, copy) at a time.  Fragment reads of step kt + 1
    // behind the even products of the first half (none is outstanding at the barrier that ends the
    // step), the copies of step kt + ST behind every fourth product of the second half.
    static_for<WI * WJ>([&](auto mc) __attribute__((always_inline)) {
      constexpr int m = decltype(mc)::value, g = m / WJ, j = m % WJ;
      big_mfma<HF, m * 4>(af[P][g], bf[P][j]);
      if constexpr (NEXT && m % 2 == 0 && m < 2 * (WI + WJ)) {
        constexpr int q = m / 2;
        if constexpr (q < WI) af[1 - P][q] = As[nx][wn * WI + q][lane];
        else bf[1 - P][q - WI] = Bs[nx][wt * WJ + q - WI][lane];
      }
      constexpr int M0 = WI * WJ / 2 + 1, SP = (WI * WJ - M0) / L;  // first copy slot, spacing
      if constexpr (MORE && m >= M0 && (m - M0) % SP == 0 && (m - M0) / SP < L)
        issue1(std::integral_constant<int, (m - M0) / SP>{}, kt + ST, st);
      asm volatile("" ::: "memory");
    });
  };
#pragma unroll
  for (int q = 0; q < ST; ++q)
    if (q < KT) issue(q, q);
  wait_steps(min(KT, ST) - 1);
  lds_sync();
#pragma unroll
  for (int i = 0; i < WI; ++i) af[0][i] = As[0][wn * WI + i][lane];
#pragma unroll
  for (int j = 0; j < WJ; ++j) bf[0][j] = Bs[0][wt * WJ + j][lane];
  asm volatile("s_nop 7" ::: "memory");  // zeroed accumulation registers -> first products
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  int st = 0, kt = 0;
  auto next_stage = [&]() __attribute__((always_inline)) { st = st == ST - 1 ? 0 : st + 1; };
  // steady state: pairs of steps that both copy ST steps ahead
  for (; kt + 1 + ST < KT; kt += 2) {
    step(c0, yes, yes, kt, st);
    next_stage();
    step(c1, yes, yes, kt + 1, st);
    next_stage();
  }
  // the last steps: kt is even here
  for (; kt < KT; kt += 2) {
    if (kt + ST < KT) step(c0, yes, yes, kt, st);
    else if (kt + 1 < KT) step(c0, no, yes, kt, st);
    else step(c0, no, no, kt, st);
    next_stage();
    if (kt + 1 < KT) {
      if (kt + 1 + ST < KT) step(c1, yes, yes, kt + 1, st);
      else if (kt + 2 < KT) step(c1, no, yes, kt + 1, st);
      else step(c1, no, no, kt + 1, st);
      next_stage();
    }
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // last products -> read-out
  static_for<WJ / PIECES>([&](auto qc) __attribute__((always_inline)) {
    constexpr int j = decltype(qc)::value * PIECES;
    const int ct = tt0 + wt * WJ + j;
    f32x4 v[WI];
    static_for<WI>([&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      v[i] = big_acc_read<(i * WJ + j) * 4>();
      if constexpr (PIECES == 2) {
        const f32x4 w = big_acc_read<(i * WJ + j + 1) * 4>();
#pragma unroll
        for (int e = 0; e < 4; ++e) v[i][e] += w[e];
      }
    });
    if (ct < a.t_tiles) pg_epilogue_col<EPI, WI, PIECES, HF>(a, v, nt0 + wn * WI, ct, lane, (int)blockIdx.z);
  });
}

__global__ __launch_bounds__(256) void k_widen_w8(const uint4* __restrict__ src, u32x4* __restrict__ dst, int KT8,
                                                  size_t total) {
  const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= total) return;
  const int lane = (int)(v & 63);
  const size_t t = v >> 6;  // byte tile: nt * KT8 + kt8
  const size_t nt = t / KT8, kt8 = t - nt * KT8;
  const uint4 b = src[v];
  u32x4* o = dst + ((nt * KT8 + kt8) * 2) * 64 + lane;
  o[0] = Bf16W8::widen8(b.x, b.y);
  o[64] = Bf16W8::widen8(b.z, b.w);
}

hipError_t launch_widen_w8(hipStream_t s, const void* src, void* dst, int n_tiles, int KT8) {
  if (n_tiles <= 0 || KT8 <= 0) return hipErrorInvalidValue;
  const size_t total = (size_t)n_tiles * KT8 * 64;
  k_widen_w8<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(static_cast<const uint4*>(src), static_cast<u32x4*>(dst),
                                                             KT8, total);
  return hipGetLastError();
}

// a.t_tiles counts operand column tiles (token tiles x pieces).  shape: 0 = 64 x 128 block
// tiles, 1 = 256 x 128, 2 = 128 x 128, 3 = 64 x 64, 4 = 192 x 128, 5 = 256 x 256 (one workgroup
// per CU, 128 x 128 per wave: 16 fragments from LDS per 64 matrix-core instructions), 6 = 192 x 256
// (the same kernel with 96 x 128 per wave).
hipError_t launch_gemm_prefill(hipStream_t s, bool f16, int epi, const PrefillGemmArgs& a, int pieces, int shape) {
  if (a.n_tiles <= 0 || a.t_tiles <= 0 || a.KT <= 0 || (pieces != 1 && pieces != 2) || a.t_tiles % pieces ||
      shape < 0 || shape > 6)
    return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU && a.n_tiles % 4) return hipErrorInvalidValue;
  const int NT = (shape == 1 || shape == 5) ? 16 : (shape == 4 || shape == 6) ? 12 : shape == 2 ? 8 : 4,
            TT = shape == 3 ? 4 : shape >= 5 ? 16 : 8;
  int ksplit = 1;
  if (a.kts_per_split > 0) {  // only the residual epilogue, and a place for the partials
    if (epi != EPI_RESID || !a.part) return hipErrorInvalidValue;
    ksplit = (a.KT + a.kts_per_split - 1) / a.kts_per_split;
  }
  dim3 grid((a.n_tiles + NT - 1) / NT, (a.t_tiles + TT - 1) / TT, ksplit);
#define PG_LAUNCH_H(E, P, HF)                                                          \
  do {                                                                                 \
    if (shape == 0) k_gemm_prefill<E, 4, 8, P, HF><<<grid, 256, 0, s>>>(a);            \
    else if (shape == 1) k_gemm_prefill_dl<E, 16, 8, P, HF><<<grid, 256, 0, s>>>(a);   \
    else if (shape == 2) k_gemm_prefill_dl<E, 8, 8, P, HF><<<grid, 256, 0, s>>>(a);    \
    else if (shape == 4) k_gemm_prefill_dl<E, 12, 8, P, HF><<<grid, 256, 0, s>>>(a);   \
    else if (shape == 5) k_gemm_prefill_big<E, P, HF, 16><<<grid, 256, 0, s>>>(a);     \
    else if (shape == 6) k_gemm_prefill_big<E, P, HF, 12><<<grid, 256, 0, s>>>(a);     \
    else k_gemm_prefill<E, 4, 4, P, HF><<<grid, 256, 0, s>>>(a);                       \
  } while (0)
#define PG_LAUNCH_P(E, P)              \
  do {                                 \
    if (f16) PG_LAUNCH_H(E, P, Fp16);  \
    else PG_LAUNCH_H(E, P, Bf16);      \
  } while (0)
#define PG_LAUNCH(E)                    \
  do {                                  \
    if (pieces == 2) PG_LAUNCH_P(E, 2); \
    else PG_LAUNCH_P(E, 1);             \
  } while (0)
  switch (epi) {
    case EPI_STORE: PG_LAUNCH(EPI_STORE); break;
    case EPI_RESID: PG_LAUNCH(EPI_RESID); break;
    case EPI_SWIGLU: PG_LAUNCH(EPI_SWIGLU); break;
    default: return hipErrorInvalidValue;
  }
#undef PG_LAUNCH
#undef PG_LAUNCH_P
#undef PG_LAUNCH_H
  return hipGetLastError();
}

// One workgroup per token row: h = x / sqrt(mean(x^2) + eps) * g as `pieces` bf16 values
// (value, remainder), written in fragment order: token tile q occupies column tiles
// q * pieces + piece.  Rows beyond n_rows are zero-filled so that padded tiles are defined.
// The pending k-slice partials of the previous projection are added to x first (fixed order,
// written back: x is the residual stream).
template <class HF>
__global__ __launch_bounds__(256) void k_rmsnorm_frag(float* __restrict__ x, const float* __restrict__ part,
                                                      int nparts, long part_stride,
                                                      const float* __restrict__ gain, int H, float eps, int n_rows,
                                                      int pieces, void* __restrict__ Xf) {
  __shared__ float sm[4];
  const int t = blockIdx.x, KT = H / 32;
  uint4* out = static_cast<uint4*>(Xf) + ((size_t)(t >> 4) * pieces * KT) * 64 + (t & 15);
  const size_t piece_stride = (size_t)KT * 64;
  if (t >= n_rows) {
    for (int kg = threadIdx.x; kg < H / 8; kg += 256)
      for (int pc = 0; pc < pieces; ++pc)
        out[pc * piece_stride + (size_t)(kg >> 2) * 64 + 16 * (kg & 3)] = uint4{0, 0, 0, 0};
    return;
  }
  float* xr = x + (size_t)t * H;
  if (nparts > 0) {
    const float* pr = part + (size_t)t * H;
    for (int i = threadIdx.x * 4; i < H; i += 1024) {
      float4 add = *reinterpret_cast<const float4*>(pr + i);
      for (int p = 1; p < nparts; ++p) {
        const float4 q = *reinterpret_cast<const float4*>(pr + (size_t)p * part_stride + i);
        add = make_float4(add.x + q.x, add.y + q.y, add.z + q.z, add.w + q.w);
      }
      const float4 v = *reinterpret_cast<const float4*>(xr + i);
      *reinterpret_cast<float4*>(xr + i) = make_float4(v.x + add.x, v.y + add.y, v.z + add.z, v.w + add.w);
    }
    __syncthreads();  // the folded row is read back below by other threads of the workgroup
  }
  // the row stays in registers between the sum of squares and the conversion: groups of 8
  // consecutive elements (one 16-byte fragment element each), up to four per thread
  constexpr int MAXG = 4;
  float v[MAXG][8];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < MAXG; ++j) {
    const int kg = threadIdx.x + 256 * j;
    if (kg < H / 8) {
      const float4 a0 = *reinterpret_cast<const float4*>(xr + kg * 8), a1 = *reinterpret_cast<const float4*>(xr + kg * 8 + 4);
      v[j][0] = a0.x; v[j][1] = a0.y; v[j][2] = a0.z; v[j][3] = a0.w;
      v[j][4] = a1.x; v[j][5] = a1.y; v[j][6] = a1.z; v[j][7] = a1.w;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += v[j][e] * v[j][e];
    }
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float r = 1.0f / sqrtf(((sm[0] + sm[1]) + (sm[2] + sm[3])) / (float)H + eps);
#pragma unroll
  for (int j = 0; j < MAXG; ++j) {
    const int kg = threadIdx.x + 256 * j;
    if (kg < H / 8) {
      const float4 g0 = *reinterpret_cast<const float4*>(gain + kg * 8), g1 = *reinterpret_cast<const float4*>(gain + kg * 8 + 4);
      const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      float y[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] = v[j][e] * r * gg[e];
      for (int pc = 0; pc < pieces; ++pc) {
        uint32_t h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          h[e] = HF::pack2(y[2 * e], y[2 * e + 1]);
          y[2 * e] -= HF::lo(h[e]);
          y[2 * e + 1] -= HF::hi(h[e]);
        }
        out[pc * piece_stride + (size_t)(kg >> 2) * 64 + 16 * (kg & 3)] = uint4{h[0], h[1], h[2], h[3]};
      }
    }
  }
}

hipError_t launch_rmsnorm_frag(hipStream_t s, bool f16, float* x, const float* part, int nparts, long part_stride,
                               const float* gain, int H, float eps, int n_rows, int token_tiles, int pieces,
                               void* Xf) {
  if (H % 32 || H > 8192 || nparts < 0 || (nparts > 0 && !part) || n_rows <= 0) return hipErrorInvalidValue;
  if (f16)
    k_rmsnorm_frag<Fp16><<<token_tiles * 16, 256, 0, s>>>(x, part, nparts, part_stride, gain, H, eps, n_rows, pieces, Xf);
  else
    k_rmsnorm_frag<Bf16><<<token_tiles * 16, 256, 0, s>>>(x, part, nparts, part_stride, gain, H, eps, n_rows, pieces, Xf);
  return hipGetLastError();
}

// x[t][k] = E[tokens[t]][k] from the packed 16-bit embedding matrix.
template <class HF>
__global__ __launch_bounds__(256) void k_embed_rows(const void* __restrict__ Ep, int H,
                                                    const int32_t* __restrict__ tokens, float* __restrict__ x) {
  const int t = blockIdx.x, r = tokens[t], KT = H / 32;
  const uint4* row = static_cast<const uint4*>(Ep) + ((size_t)(r >> 4) * KT) * 64 + (r & 15);
  for (int kg = threadIdx.x; kg < H / 8; kg += 256) {
    const uint4 v = row[(size_t)(kg >> 2) * 64 + 16 * (kg & 3)];
    float* dst = x + (size_t)t * H + kg * 8;
    *reinterpret_cast<float4*>(dst) = make_float4(HF::lo(v.x), HF::hi(v.x), HF::lo(v.y), HF::hi(v.y));
    *reinterpret_cast<float4*>(dst + 4) = make_float4(HF::lo(v.z), HF::hi(v.z), HF::lo(v.w), HF::hi(v.w));
  }
}

hipError_t launch_embed_rows(hipStream_t s, bool f16, const void* Ep, int H, const int32_t* tokens_dev, int n, float* x) {
  if (f16) k_embed_rows<Fp16><<<n, 256, 0, s>>>(Ep, H, tokens_dev, x);
  else k_embed_rows<Bf16><<<n, 256, 0, s>>>(Ep, H, tokens_dev, x);
  return hipGetLastError();
}


// ---------------------------------------------------------------------------
// causal prompt attention on the matrix cores
// ---------------------------------------------------------------------------
// Transposed copy of one slot's cached V rows, positions [0, n_pos): Vt[kv head][d][position]
// (row stride S, a multiple of 32).  The attention kernel below wants, for a fixed head
// dimension, eight consecutive positions in one 16-byte load.
__global__ __launch_bounds__(256) void k_v_transpose(const uint16_t* __restrict__ vc, uint32_t slot, int nkv,
                                                     uint32_t max_seq, uint32_t n_pos, uint16_t* __restrict__ vt,
                                                     uint32_t S) {
  __shared__ uint16_t tile[64][130];  // 64 positions x 128 dims, rows padded to 65 words
  const int kvh = blockIdx.y, tid = threadIdx.x;
  const uint32_t p0 = blockIdx.x * 64;
  const uint16_t* src = vc + (((size_t)slot * nkv + kvh) * max_seq) * 128;
  for (int q = tid; q < 64 * 16; q += 256) {
    const uint32_t pr = q >> 4, dc = q & 15, pos = min(p0 + pr, n_pos - 1);
    const uint4 v = *reinterpret_cast<const uint4*>(src + (size_t)pos * 128 + dc * 8);
    uint32_t* t = reinterpret_cast<uint32_t*>(&tile[pr][dc * 8]);
    t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
  }
  __syncthreads();
  for (int q = tid; q < 128 * 8; q += 256) {
    const int d = q >> 3, seg = q & 7;  // 8 positions p0 + seg * 8 .. + 7 of dimension d
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = tile[seg * 8 + 2 * e][d] | ((uint32_t)tile[seg * 8 + 2 * e + 1][d] << 16);
    if (p0 + seg * 8 < S)
      *reinterpret_cast<uint4*>(vt + ((size_t)kvh * 128 + d) * S + p0 + seg * 8) = uint4{w[0], w[1], w[2], w[3]};
  }
}

hipError_t launch_v_transpose(hipStream_t s, const void* vc, uint32_t slot, int nkv, uint32_t max_seq, uint32_t n_pos,
                              void* vt, uint32_t S) {
  if (n_pos == 0 || S % 32 || n_pos > S) return hipErrorInvalidValue;
  dim3 grid((n_pos + 63) / 64, nkv);
  k_v_transpose<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(vc), slot, nkv, max_seq, n_pos,
                                     static_cast<uint16_t*>(vt), S);
  return hipGetLastError();
}

// Scores and weighted sums of 16 prompt tokens x GH query heads (sharing one kv head) per wave,
// four waves (64 consecutive tokens) per workgroup, flash style: positions are walked in chunks
// of 32 with a running maximum and sum per row.
// Both products run transposed, so that no operand needs a shuffle between them:
//   S^T = K Q^T   A = 16 cached K rows (their 128 dims in four k steps), B = the wave's 16
//                 query rows; D holds, per lane, one query token (column) and 4 + 4 positions
//                 of the two 16-row tiles.  The K rows of the two tiles are picked so that
//                 these are 8 consecutive positions g*8 .. g*8+7.
//   O^T = V^T P^T A = 16 head dims x 32 positions from the transposed V copy (16 bytes per
//                 lane), B = the lane's own 8 weights: exactly the B-operand layout (column =
//                 query token, 8 consecutive k).
// The 16 fragments of a chunk (8 K, 8 V^T, 1 KiB each) are the same for all four waves: the
// workgroup copies them once, global -> registers -> LDS, one chunk ahead of the products
// (double-buffered, one barrier per chunk), and each wave reads them from LDS for its GH heads.
// A wave keeps only its queries and accumulators in registers, so two workgroups fit on a CU
// and one wave's softmax arithmetic overlaps another's matrix-core work.
// Masked positions get weight exp(-inf) = 0; their K / V^T values are finite (the copy and the
// cache rows read are initialised memory), so 0 x value = 0.
// PIECES = 2: queries and weights enter the matrix cores as two bf16 pieces (16 significant
// bits); PIECES = 1: one bf16 each.  The row sum adds the weights as they are multiplied.
template <int GH, int PIECES, class HF>
__global__ __launch_bounds__(256, 2) void k_attn_prefill(const float* __restrict__ qkv, int nq, int nkv,
                                                         const uint16_t* __restrict__ kc,
                                                         const uint16_t* __restrict__ vt, uint32_t S, uint32_t slot,
                                                         uint32_t max_seq, uint32_t pos0, int n, int paired,
                                                         void* __restrict__ Of) {
  __shared__ u32x4 Fs[2][16][64];  // fragments 0-3: K tile a, 4-7: K tile b (k steps), 8-15: V^T (dim tiles)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c16 = lane & 15, g = lane >> 4;
  const int G = nq / nkv;
  const int kvh = blockIdx.y / (G / GH), head0 = kvh * G + (blockIdx.y % (G / GH)) * GH;
  // Rows near the end of the prompt see many more positions than rows near its start.  Unpaired:
  // one 64-token block per workgroup, the longest dispatched first.  Paired (launches whose
  // workgroups are all resident at once, so dispatch order cannot balance them): every workgroup
  // does block NB-1-i and then block i, the same number of chunks for all of them.
  const int NB = (n + 63) / 64;
  for (int pass = 0; pass < (paired ? 2 : 1); ++pass) {
  const int tq4 = pass == 0 ? NB - 1 - (int)blockIdx.x : (int)blockIdx.x;
  if (pass == 1 && tq4 >= NB - 1 - (int)blockIdx.x) break;  // the middle block of an odd count is done
  const int tq = tq4 * 4 + wave;
  const bool active = tq * 16 < n;  // a wave past the prompt only helps with the copies
  const int ld = (nq + 2 * nkv) * 128;
  const int t = min(tq * 16 + c16, n - 1);  // rows past the prompt repeat the last token (never stored)
  const uint32_t p = pos0 + (uint32_t)t;    // position of this lane's query token

  // query fragments: lane (column c16 = token, g) holds dims ks*32 + g*8 .. +7 of its token
  u32x4 qf[GH][4][PIECES];
#pragma unroll
  for (int h = 0; h < GH; ++h)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const float* src = qkv + (size_t)t * ld + (size_t)(head0 + h) * 128 + ks * 32 + g * 8;
      const float4 x0 = *reinterpret_cast<const float4*>(src), x1 = *reinterpret_cast<const float4*>(src + 4);
      float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
      for (int pc = 0; pc < PIECES; ++pc) {
        uint32_t b[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          b[e] = HF::pack2(v[2 * e], v[2 * e + 1]);
          v[2 * e] -= HF::lo(b[e]);
          v[2 * e + 1] -= HF::hi(b[e]);
        }
        qf[h][ks][pc] = u32x4{b[0], b[1], b[2], b[3]};
      }
    }

  f32x4 acc[GH][8], lacc[GH];  // lacc: the row sums, every element of a lane the sum of its token
  float mrun[GH];
#pragma unroll
  for (int h = 0; h < GH; ++h) {
    mrun[h] = -INFINITY;
    lacc[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[h][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const uint16_t* kbase = kc + (((size_t)slot * nkv + kvh) * max_seq) * 128;
  const uint16_t* vbase = vt + (size_t)kvh * 128 * S;
  const uint32_t p_first = pos0 + (uint32_t)tq * 16;                  // positions up to here are visible to every row
  const uint32_t p_last = pos0 + (uint32_t)min(tq * 16 + 15, n - 1);  // last position any row of the wave's tile sees
  const uint32_t p_last_wg = pos0 + (uint32_t)min(tq4 * 64 + 63, n - 1);

  // copy of a chunk: thread tid moves element (tid & 63) of fragments (tid >> 6) + 4 j, i.e.
  // fragments wave (K tile a, k step = wave), wave + 4 (K tile b), wave + 8 and wave + 12
  // (V^T dim tiles).  Addresses = a base that is uniform over the workgroup + a byte offset per
  // thread that is fixed for the whole kernel.
  const int r4 = (c16 >> 2) * 8 + (c16 & 3);  // K row of tile a for A-operand row c16; tile b: + 4
  const uint32_t ok = (uint32_t)(r4 * 128 + wave * 32 + g * 8) * 2u;
  const uint32_t ov0 = ((uint32_t)(wave * 16 + c16) * S + (uint32_t)g * 8u) * 2u, ov1 = ov0 + 64u * S * 2u;
  u32x4 stage[4];
  auto gload = [&](uint32_t kv0) __attribute__((always_inline)) {  // kv0 < S, a multiple of 32
    const char* kb = reinterpret_cast<const char*>(kbase) + (size_t)kv0 * 256;
    const char* vb = reinterpret_cast<const char*>(vbase) + (size_t)kv0 * 2;
    if (kv0 + 32 <= max_seq) {
      stage[0] = *reinterpret_cast<const u32x4*>(kb + ok);
      stage[1] = *reinterpret_cast<const u32x4*>(kb + ok + 4 * 256);
    } else {  // the cache ends inside the chunk: repeat its last row (those positions are masked)
      const uint32_t ra = min(kv0 + r4, max_seq - 1), rb = min(kv0 + r4 + 4, max_seq - 1);
      stage[0] = *reinterpret_cast<const u32x4*>(kbase + (size_t)ra * 128 + wave * 32 + g * 8);
      stage[1] = *reinterpret_cast<const u32x4*>(kbase + (size_t)rb * 128 + wave * 32 + g * 8);
    }
    stage[2] = *reinterpret_cast<const u32x4*>(vb + ov0);
    stage[3] = *reinterpret_cast<const u32x4*>(vb + ov1);
  };
  auto sstore = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) Fs[buf][wave + 4 * j][lane] = stage[j];
  };

  // maxima without the NaN-quieting copies that fmaxf brings (no operand here is a NaN)
  auto max3 = [](float x, float y, float z) __attribute__((always_inline)) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(y), "v"(z));
    return r;
  };
  auto max2 = [](float x, float y) __attribute__((always_inline)) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
  };
  const u32x4 ones = u32x4{HF::kOnes2, HF::kOnes2, HF::kOnes2, HF::kOnes2};  // 1.0 x 8

  auto do_chunk = [&](int buf, uint32_t kv0) __attribute__((always_inline)) {
    u32x4 pf[GH][PIECES];
    // all 16 fragments are requested up front: the V^T reads complete under the first product
    // and the softmax arithmetic (two heads with two pieces each have no registers left for
    // that: they read each V^T fragment where it is used)
    constexpr bool kVfUpFront = !(GH == 2 && PIECES == 2);
    u32x4 vf[8];
    {
      u32x4 ka[4], kb[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        ka[ks] = Fs[buf][ks][lane];
        kb[ks] = Fs[buf][4 + ks][lane];
      }
      if constexpr (kVfUpFront) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) vf[dt] = Fs[buf][8 + dt][lane];
      }
#pragma unroll
      for (int h = 0; h < GH; ++h) {
        f32x4 sa = f32x4{0.f, 0.f, 0.f, 0.f}, sb = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
          for (int pc = 0; pc < PIECES; ++pc) {
            sa = HF::mfma(ka[ks], qf[h][ks][pc], sa);
            sb = HF::mfma(kb[ks], qf[h][ks][pc], sb);
          }
        // element i of sa: position kv0 + g*8 + i; of sb: kv0 + g*8 + 4 + i; column = this lane's token
        float sc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) sc[i] = i < 4 ? sa[i] : sb[i - 4];
        if (kv0 + 31 > p_first) {  // the chunk reaches past the tile's first token: mask per lane
#pragma unroll
          for (int i = 0; i < 8; ++i) sc[i] = kv0 + g * 8 + i <= p ? sc[i] : -INFINITY;
        }
        // scores in units of log 2: exp(s / sqrt(128)) = exp2(s * log2(e) / sqrt(128))
        constexpr float kScale = 0.12751743082459868f;
        const float mx = max2(max3(sc[0], sc[1], sc[2]), max3(sc[3], sc[4], max3(sc[5], sc[6], sc[7]))) * kScale;
        // The running maximum is the same in the four lanes of a token.  It only has to bound the
        // scores: while no lane exceeds it, nothing is exchanged or rescaled.
        if (__any(mx > mrun[h])) {
          const float mn = max2(mrun[h], col4_max(mx));  // finite from the first chunk on: position 0 is visible to every token
          const float alpha = __builtin_amdgcn_exp2f(mrun[h] - mn);
          mrun[h] = mn;
#pragma unroll
          for (int e = 0; e < 4; ++e) lacc[h][e] *= alpha;
#pragma unroll
          for (int dt = 0; dt < 8; ++dt)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[h][dt][e] *= alpha;
        }
        const float mn = mrun[h];
        uint32_t pw[PIECES][4];  // weights as packed bf16 pairs: the B operand of the second product
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
          float w0 = __builtin_amdgcn_exp2f(fmaf(sc[i], kScale, -mn));
          float w1 = __builtin_amdgcn_exp2f(fmaf(sc[i + 1], kScale, -mn));
#pragma unroll
          for (int pc = 0; pc < PIECES; ++pc) {
            pw[pc][i / 2] = HF::pack2(w0, w1);
            if (pc + 1 < PIECES) {
              w0 -= HF::lo(pw[pc][i / 2]);
              w1 -= HF::hi(pw[pc][i / 2]);
            }
          }
        }
#pragma unroll
        for (int pc = 0; pc < PIECES; ++pc) {
          pf[h][pc] = u32x4{pw[pc][0], pw[pc][1], pw[pc][2], pw[pc][3]};
          // row sums of the weights as multiplied (all pieces): a product with a tile of ones
          lacc[h] = HF::mfma(ones, pf[h][pc], lacc[h]);
        }
      }
    }
    // every V^T fragment feeds all GH heads
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      if constexpr (!kVfUpFront) vf[dt] = Fs[buf][8 + dt][lane];
#pragma unroll
      for (int h = 0; h < GH; ++h)
#pragma unroll
        for (int pc = 0; pc < PIECES; ++pc)
          acc[h][dt] = HF::mfma(vf[dt], pf[h][pc], acc[h][dt]);
    }
  };

  gload(0);
  sstore(0);
  lds_sync();
  int buf = 0;
  for (uint32_t kv0 = 0; kv0 <= p_last_wg; kv0 += 32, buf ^= 1) {
    const bool more = kv0 + 32 <= p_last_wg;  // uniform over the workgroup
    if (more) gload(kv0 + 32);
    if (active && kv0 <= p_last) do_chunk(buf, kv0);
    if (more) sstore(buf ^ 1);
    lds_sync();
  }
  if (!active) continue;

  // acc[h][dt] element e: head dim dt*16 + g*4 + e of this lane's token.  Output goes straight
  // into the fragment order the output projection reads: operand index k = head * 128 + dim.
  const int KTQ = nq * 4;
#pragma unroll
  for (int h = 0; h < GH; ++h) {
    const float inv = 1.0f / lacc[h][0];
    if (tq * 16 + c16 < n) {
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const int k0 = (head0 + h) * 128 + dt * 16 + g * 4;
        float v[4] = {acc[h][dt][0] * inv, acc[h][dt][1] * inv, acc[h][dt][2] * inv, acc[h][dt][3] * inv};
#pragma unroll
        for (int pc = 0; pc < PIECES; ++pc) {
          const uint32_t b0 = HF::pack2(v[0], v[1]), b1 = HF::pack2(v[2], v[3]);
          v[0] -= HF::lo(b0);
          v[1] -= HF::hi(b0);
          v[2] -= HF::lo(b1);
          v[3] -= HF::hi(b1);
          const size_t el = (((size_t)(tq * PIECES + pc) * KTQ + (k0 >> 5)) * 64 + c16 + 16 * ((k0 & 31) >> 3)) * 8 + (k0 & 7);
          *reinterpret_cast<uint2*>(static_cast<uint16_t*>(Of) + el) = make_uint2(b0, b1);
        }
      }
    }
  }
  }  // pass
}

// qkv: [tokens][(nq + 2 nkv) * 128] fp32 with the query heads already normed and rotated.
// kc: the layer's K cache; vt: transposed V copy of the slot (row stride S) covering positions
// 0 .. pos0 + n - 1.  Of: fragment-order bf16 output ([token tile x pieces][nq*4][64][8]).
hipError_t launch_attn_prefill(hipStream_t s, bool f16, const float* qkv, int nq, int nkv, const void* kc, const void* vt,
                               uint32_t S, uint32_t slot, uint32_t max_seq, uint32_t pos0, int n, int pieces, void* Of,
                               int n_cus, int shape) {
  const int G = nq / nkv;
  if (n <= 0 || G < 1 || nq % nkv || (pieces != 1 && pieces != 2) || S % 32 || pos0 + (uint32_t)n > S)
    return hipErrorInvalidValue;
  // Two heads per wave halve the LDS reads per product; one head per wave doubles the
  // workgroups.  Pairing needs two workgroups per CU after halving their number.
  const int NB = (n + 63) / 64, slots = 2 * n_cus;
  int GH = 1, paired = 0;
  if (G % 2 == 0 && (NB + 1) / 2 * nkv * (G / 2) >= slots) GH = 2, paired = 1;
  else if ((NB + 1) / 2 * nkv * G >= slots) paired = 1;
  else if (G % 2 == 0 && NB * nkv * (G / 2) >= slots) GH = 2;
  if (shape >= 0) {  // forced: bit 0 = paired, bit 1 = two heads per wave (where the group size allows)
    if (shape > 3) return hipErrorInvalidValue;
    paired = shape & 1;
    GH = (shape & 2) && G % 2 == 0 ? 2 : 1;
  }
  dim3 grid(paired ? (NB + 1) / 2 : NB, nkv * (G / GH));
  const uint16_t* k = static_cast<const uint16_t*>(kc);
  const uint16_t* v = static_cast<const uint16_t*>(vt);
#define AP_LAUNCH_H(GHV, HF)                                                                                        \
  do {                                                                                                              \
    if (pieces == 2) k_attn_prefill<GHV, 2, HF><<<grid, 256, 0, s>>>(qkv, nq, nkv, k, v, S, slot, max_seq, pos0, n, paired, Of); \
    else k_attn_prefill<GHV, 1, HF><<<grid, 256, 0, s>>>(qkv, nq, nkv, k, v, S, slot, max_seq, pos0, n, paired, Of);           \
  } while (0)
#define AP_LAUNCH(GHV)                \
  do {                                \
    if (f16) AP_LAUNCH_H(GHV, Fp16);  \
    else AP_LAUNCH_H(GHV, Bf16);      \
  } while (0)
  if (GH == 2) AP_LAUNCH(2);
  else AP_LAUNCH(1);
#undef AP_LAUNCH
#undef AP_LAUNCH_H
  return hipGetLastError();
}

}  // namespace nnc
