// gfx950 (CDNA4) kernels of the Qwen3-style decoder forward pass.
//
// The matmuls follow the paper's packed-layout idea (Section 3.1.2, Auto
// Vectorize: keep operands in the hardware-intrinsic blocked layout end to end;
// Section 3.3.2: MatMul micro-kernels over packed operands): weights are stored
// once in matrix-core fragment order and every lane streams them with 16-byte
// loads.  Everything else (norms, RoPE, SwiGLU, attention) is the public Qwen3
// decoder arithmetic in fp32.
#include "nnc_half.h"
#include "nnc_internal.h"
#include "nnc_lanes.h"

namespace nnc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------

// Launch one instance of a kernel template for the model's element type: inside the statement
// F32 is a constant expression and HF names the 16-bit format (unused by fp32 instances).
#define NNC_FOR_HALF(dt, ...)   \
  do {                          \
    if ((dt) == DT_F16) {       \
      using HF = Fp16;          \
      __VA_ARGS__;              \
    } else {                    \
      using HF = Bf16;          \
      __VA_ARGS__;              \
    }                           \
  } while (0)
#define NNC_FOR_DTYPE(dt, ...)              \
  do {                                      \
    if ((dt) == DT_F32) {                   \
      constexpr bool F32 = true;            \
      using HF = Bf16;                      \
      __VA_ARGS__;                          \
    } else if ((dt) == DT_BF16) {           \
      constexpr bool F32 = false;           \
      using HF = Bf16;                      \
      __VA_ARGS__;                          \
    } else {                                \
      constexpr bool F32 = false;           \
      using HF = Fp16;                      \
      __VA_ARGS__;                          \
    }                                       \
  } while (0)

__device__ __forceinline__ float block_sum_256(float v, float* sm) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  return (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

// ---------------------------------------------------------------------------
// weight repack: canonical row-major [rows, K] -> matrix-core tile order
// ---------------------------------------------------------------------------
// One thread per (tile row-block nt, k tile kt, lane).  The destination tile index is
// nt * tile_stride + tile_offset, which expresses both "append below" (stride 1,
// offset = first tile of the sub-matrix in a fused matrix) and "interleave with a
// sibling matrix in 16-row tiles" (stride 2, offset 0 or 1).
template <bool SRC_F32, bool DST_F32, class HF>
__global__ __launch_bounds__(256) void k_repack(const void* __restrict__ src, void* __restrict__ dst,
                                                int rows, int K, int tile_stride, int tile_offset) {
  constexpr int VEC = DST_F32 ? 4 : 8;
  constexpr int KTILE = VEC * 4;
  const int KT = K / KTILE;
  const size_t total = (size_t)(rows / 16) * KT * 64;
  const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= total) return;
  const int lane = (int)(v & 63);
  const size_t t = v >> 6;
  const int kt = (int)(t % KT);
  const int nt = (int)(t / KT);
  const size_t r = (size_t)nt * 16 + (lane & 15);
  const size_t k0 = (size_t)kt * KTILE + (lane >> 4) * VEC;
  const size_t dvec = ((size_t)(nt * tile_stride + tile_offset) * KT + kt) * 64 + lane;
  if constexpr (DST_F32) {
    static_assert(SRC_F32 || !DST_F32, "16-bit blobs are never widened");
    const float4 x = *reinterpret_cast<const float4*>(static_cast<const float*>(src) + r * K + k0);
    reinterpret_cast<float4*>(dst)[dvec] = x;
  } else if constexpr (SRC_F32) {
    const float* p = static_cast<const float*>(src) + r * K + k0;
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    uint4 o;
    o.x = HF::bits(a.x) | (HF::bits(a.y) << 16);
    o.y = HF::bits(a.z) | (HF::bits(a.w) << 16);
    o.z = HF::bits(b.x) | (HF::bits(b.y) << 16);
    o.w = HF::bits(b.z) | (HF::bits(b.w) << 16);
    reinterpret_cast<uint4*>(dst)[dvec] = o;
  } else {
    reinterpret_cast<uint4*>(dst)[dvec] =
        *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(src) + r * K + k0);
  }
}

// src_f32: the blob holds fp32; dst_dt: the model's element type (a 16-bit blob is already in it).
hipError_t launch_repack(hipStream_t s, bool src_f32, int dst_dt, const void* src, void* dst,
                         int rows, int K, int tile_stride, int tile_offset) {
  const int ktile = dst_dt == DT_F32 ? 16 : 32;
  const size_t total = (size_t)(rows / 16) * (K / ktile) * 64;
  const unsigned grid = (unsigned)((total + 255) / 256);
  if (dst_dt == DT_F32)
    k_repack<true, true, Bf16><<<grid, 256, 0, s>>>(src, dst, rows, K, tile_stride, tile_offset);
  else if (src_f32 && dst_dt == DT_BF16)
    k_repack<true, false, Bf16><<<grid, 256, 0, s>>>(src, dst, rows, K, tile_stride, tile_offset);
  else if (src_f32)
    k_repack<true, false, Fp16><<<grid, 256, 0, s>>>(src, dst, rows, K, tile_stride, tile_offset);
  else
    k_repack<false, false, Bf16><<<grid, 256, 0, s>>>(src, dst, rows, K, tile_stride, tile_offset);
  return hipGetLastError();
}

// Weight-only 8-bit matrices: a tile is 16 rows x 64 k; lane (row c16, group g) holds the 8 bytes
// k = 64 kt + 8 g .. + 7 and then the 8 bytes k = 64 kt + 32 + 8 g .. + 7, i.e. its share of the
// two 32-wide matrix-core k tiles the byte tile covers.
__global__ __launch_bounds__(256) void k_repack_w8(const int8_t* __restrict__ src, uint4* __restrict__ dst, int rows,
                                                   int K, int tile_stride, int tile_offset) {
  const int KT = K / 64;
  const size_t total = (size_t)(rows / 16) * KT * 64;
  const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= total) return;
  const int lane = (int)(v & 63);
  const size_t t = v >> 6;
  const int kt = (int)(t % KT);
  const int nt = (int)(t / KT);
  const int8_t* p = src + ((size_t)nt * 16 + (lane & 15)) * K + (size_t)kt * 64 + (lane >> 4) * 8;
  const uint2 a = *reinterpret_cast<const uint2*>(p), b = *reinterpret_cast<const uint2*>(p + 32);
  dst[((size_t)(nt * tile_stride + tile_offset) * KT + kt) * 64 + lane] = make_uint4(a.x, a.y, b.x, b.y);
}

hipError_t launch_repack_w8(hipStream_t s, const void* src, void* dst, int rows, int K, int tile_stride,
                            int tile_offset) {
  if (rows % 16 || K % 64) return hipErrorInvalidValue;
  const size_t total = (size_t)(rows / 16) * (K / 64) * 64;
  k_repack_w8<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(static_cast<const int8_t*>(src), static_cast<uint4*>(dst),
                                                              rows, K, tile_stride, tile_offset);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// column state
// ---------------------------------------------------------------------------
struct StateInit {
  int32_t tok[MAX_COLS];
  uint32_t slot[MAX_COLS];
  uint32_t pos[MAX_COLS];
};

__global__ void k_set_state(ColState* st, StateInit init, int ncols, uint32_t step) {
  const int i = threadIdx.x;
  if (i < ncols) {
    st->tok[i] = init.tok[i];
    st->slot[i] = init.slot[i];
    st->pos[i] = init.pos[i];
  }
  if (i == 0) st->step = step;
}

hipError_t launch_set_state(hipStream_t s, ColState* st, int ncols, const int32_t* tok,
                            const uint32_t* slot, const uint32_t* pos, uint32_t step) {
  StateInit init;
  for (int i = 0; i < MAX_COLS; ++i) {
    init.tok[i] = (i < ncols && tok) ? tok[i] : 0;
    init.slot[i] = i < ncols ? slot[i] : 0;
    init.pos[i] = i < ncols ? pos[i] : 0;
  }
  k_set_state<<<1, MAX_COLS, 0, s>>>(st, init, ncols, step);
  return hipGetLastError();
}

// After a greedy step: feed the chosen token back, advance positions, log the token.
__global__ void k_finish_step(ColState* st, int ncols, const int32_t* next, int32_t* token_log) {
  const int i = threadIdx.x;
  const uint32_t step = st->step;
  __syncthreads();
  if (i < ncols) {
    const int32_t t = next[i];
    st->tok[i] = t;
    st->pos[i] += 1;
    token_log[(size_t)step * ncols + i] = t;
  }
  if (i == 0) st->step = step + 1;
}

hipError_t launch_finish_step(hipStream_t s, ColState* st, int ncols, const int32_t* next,
                              int32_t* token_log) {
  k_finish_step<<<1, MAX_COLS, 0, s>>>(st, ncols, next, token_log);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// embedding gather from the packed matrix: x[col][k] = E[tok[col]][k]
// ---------------------------------------------------------------------------
template <bool F32, class HF>
__global__ __launch_bounds__(256) void k_embed(const void* __restrict__ Ep, int H,
                                               const ColState* __restrict__ st, float* __restrict__ x) {
  constexpr int VEC = F32 ? 4 : 8;
  constexpr int KTILE = VEC * 4;
  const int col = blockIdx.x;
  const int r = st->tok[col];
  const int KT = H / KTILE;
  const size_t nt = (size_t)(r >> 4);
  for (int k = threadIdx.x; k < H; k += 256) {
    const int kt = k / KTILE, kk = k % KTILE;
    const int lane = (r & 15) + 16 * (kk / VEC);
    const size_t e = ((nt * KT + kt) * 64 + lane) * VEC + (kk % VEC);
    float v;
    if constexpr (F32)
      v = static_cast<const float*>(Ep)[e];
    else
      v = HF::widen(static_cast<const uint16_t*>(Ep)[e]);
    x[(size_t)col * H + k] = v;
  }
}

hipError_t launch_embed(hipStream_t s, int dt, const void* Ep, int H, const ColState* st,
                        int ncols, float* x) {
  NNC_FOR_DTYPE(dt, k_embed<F32, HF><<<ncols, 256, 0, s>>>(Ep, H, st, x));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// RMSNorm of one column, written as a packed (split) GEMM operand
//   h_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i
// ---------------------------------------------------------------------------
template <bool F32, class HF>
__device__ __forceinline__ void store_packed(void* Xp, int NC, int nsplit, int seq, int k, float v) {
  if constexpr (F32) {
    static_cast<float*>(Xp)[((size_t)(k >> 2) * NC + seq) * 4 + (k & 3)] = v;
  } else {
    uint32_t piece[3];
    split_pieces<HF>(v, nsplit, piece);
    uint16_t* p = static_cast<uint16_t*>(Xp) + ((size_t)(k >> 3) * NC + seq * nsplit) * 8 + (k & 7);
#pragma unroll
    for (int s = 0; s < 3; ++s)
      if (s < nsplit) p[s * 8] = (uint16_t)piece[s];
  }
}

// The three places of the row norm where a compiler may or may not contract a multiply and an
// add, written out, so that the norm kernel and the norm in a GEMM's tail round alike.
__device__ __forceinline__ float sumsq4(float ss, float4 v) {
  ss = __builtin_fmaf(v.x, v.x, ss);
  ss = __builtin_fmaf(v.y, v.y, ss);
  ss = __builtin_fmaf(v.z, v.z, ss);
  return __builtin_fmaf(v.w, v.w, ss);
}
// (#pragma clang fp contract(off): the products and sums of the function carry no permission to
// be fused, here or after inlining; the compiler's own choice depends on the surrounding code.)
__device__ __forceinline__ float rms_rinv(float ss, int H, float eps) {
#pragma clang fp contract(off)
  return 1.0f / sqrtf(ss / (float)H + eps);
}
__device__ __forceinline__ float norm_elem(float v, float r, float g) {
#pragma clang fp contract(off)
  const float vr = v * r;
  return vr * g;
}

// norm_elem of four consecutive elements i .. i+3 of a row -> the packed operand layout
template <bool F32, class HF>
__device__ __forceinline__ void store_normed4(void* Xp, int NC, int nsplit, int seq, int i, float4 v, float r, float4 g) {
  const float h[4] = {norm_elem(v.x, r, g.x), norm_elem(v.y, r, g.y), norm_elem(v.z, r, g.z), norm_elem(v.w, r, g.w)};
  if constexpr (F32) {
    *reinterpret_cast<float4*>(static_cast<float*>(Xp) + ((size_t)(i >> 2) * NC + seq) * 4) =
        make_float4(h[0], h[1], h[2], h[3]);
  } else {
    // elements i .. i+3 of one 8-element group: 8 bytes per piece
    uint32_t pc[4][3];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_pieces<HF>(h[e], nsplit, pc[e]);
    uint16_t* dst = static_cast<uint16_t*>(Xp) + ((size_t)(i >> 3) * NC + seq * nsplit) * 8 + (i & 7);
#pragma unroll
    for (int sp = 0; sp < 3; ++sp)
      if (sp < nsplit)
        *reinterpret_cast<uint2*>(dst + sp * 8) = make_uint2(pc[0][sp] | (pc[1][sp] << 16), pc[2][sp] | (pc[3][sp] << 16));
  }
}

// Before the norm, the pending output of the previous projection is added to the
// residual stream: x += part[0] + part[1] + ... (k slices of that GEMM, fixed order),
// and the updated x is written back.  part_seq0 is the column of `part` that
// corresponds to blockIdx.x == 0 (the LM head norms a sub-range of the columns).
// NV = float4 groups per thread: the whole row (H <= 1024 * NV) lives in registers, every load
// (row, pending partials, gains) is issued before the first use, and the row is neither
// re-read nor re-written more than once.
template <bool F32, int NV, class HF>
__global__ __launch_bounds__(256) void k_rmsnorm_pack(float* __restrict__ x, long ldx,
                                                      const float* __restrict__ part, int nparts,
                                                      long part_stride, const float* __restrict__ gain,
                                                      int H, float eps, void* __restrict__ Xp, int NC,
                                                      int nsplit) {
  __shared__ float sm[4];
  const int seq = blockIdx.x;
  float* xr = x + (size_t)seq * ldx;
  constexpr int MAXP = 8;  // most k slices a projection is split into
  float4 v[NV], g[NV], pp[NV][MAXP];
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int i = (threadIdx.x + 256 * q) * 4;
    v[q] = g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < H) {
      v[q] = *reinterpret_cast<const float4*>(xr + i);
      g[q] = *reinterpret_cast<const float4*>(gain + i);
#pragma unroll
      for (int p = 0; p < MAXP; ++p)
        if (p < nparts) pp[q][p] = *reinterpret_cast<const float4*>(part + (size_t)p * part_stride + (size_t)seq * H + i);
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int i = (threadIdx.x + 256 * q) * 4;
    if (i < H && nparts > 0) {
      float4 add = pp[q][0];  // slices are added in a fixed order
#pragma unroll
      for (int p = 1; p < MAXP; ++p)
        if (p < nparts) add = make_float4(add.x + pp[q][p].x, add.y + pp[q][p].y, add.z + pp[q][p].z, add.w + pp[q][p].w);
      v[q] = make_float4(v[q].x + add.x, v[q].y + add.y, v[q].z + add.z, v[q].w + add.w);
      *reinterpret_cast<float4*>(xr + i) = v[q];
    }
    ss = sumsq4(ss, v[q]);
  }
  ss = block_sum_256(ss, sm);
  const float r = rms_rinv(ss, H, eps);
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int i = (threadIdx.x + 256 * q) * 4;
    if (i >= H) continue;
    store_normed4<F32, HF>(Xp, NC, nsplit, seq, i, v[q], r, g[q]);
  }
}

hipError_t launch_rmsnorm_pack(hipStream_t s, int dt, float* x, long ldx, const float* part, int nparts,
                               long part_stride, const float* gain, int H, float eps, int ncols, void* Xp,
                               int NC, int nsplit) {
  if (H % 4 || H > 8192 || nparts > 8 || nparts < 0 || ldx % 4) return hipErrorInvalidValue;
#define RN_LAUNCH(NV) \
  NNC_FOR_DTYPE(dt, k_rmsnorm_pack<F32, NV, HF><<<ncols, 256, 0, s>>>(x, ldx, part, nparts, part_stride, gain, H, eps, Xp, NC, nsplit))
  if (H <= 1024) RN_LAUNCH(1);
  else if (H <= 2048) RN_LAUNCH(2);
  else if (H <= 4096) RN_LAUNCH(4);
  else RN_LAUNCH(8);
#undef RN_LAUNCH
  return hipGetLastError();
}

__global__ void k_zero_words(uint32_t* p, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0u;
}
hipError_t launch_zero_words(hipStream_t s, uint32_t* p, int n) {
  if (n <= 0) return hipSuccess;
  k_zero_words<<<1, 256, 0, s>>>(p, n);
  return hipGetLastError();
}

// x += part[0] + part[1] + ... for n contiguous floats (all columns), fixed order.
__global__ __launch_bounds__(256) void k_fold_residual(float* __restrict__ x, const float* __restrict__ part,
                                                       int nparts, long part_stride, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    float add = part[i];
    for (int p = 1; p < nparts; ++p) add += part[(size_t)p * part_stride + i];
    x[i] += add;
  }
}

hipError_t launch_fold_residual(hipStream_t s, float* x, const float* part, int nparts, long part_stride,
                                size_t n) {
  const unsigned grid = (unsigned)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  k_fold_residual<<<grid ? grid : 1, 256, 0, s>>>(x, part, nparts, part_stride, n);
  return hipGetLastError();
}

// A float written by another workgroup of the running launch with a write-through store: read
// past this CU's L1 and this XCD's L2, which may hold the line from before that store.
__device__ __forceinline__ float load_coherent(const float* p) {
  return __uint_as_float(__hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void store_through(float* p, float v) {
  __hip_atomic_store(reinterpret_cast<uint32_t*>(p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Tail of a GEMM launch whose output feeds an RMSNorm (NormTail).  Called by every thread of
// every workgroup after its last partial-tile store.  sm: 8 words of LDS nobody else uses now.
template <bool F32, class HF>
__device__ __forceinline__ void gemm_norm_tail(const NormTail& t, const float* part, long part_stride, int nparts,
                                               int nseq, float* sm) {
  // this thread's stores have reached memory; after the barrier, the whole workgroup's have
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
  __syncthreads();
  const unsigned total = gridDim.x * gridDim.y;
  const unsigned takers = total < (unsigned)nseq ? total : (unsigned)nseq;  // the last `takers` workgroups run the norm
  int* si = reinterpret_cast<int*>(sm);
  if (threadIdx.x == 0) {
    const unsigned done_before = __hip_atomic_fetch_add(t.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int role = -1;
    if (done_before + takers >= total) {
      role = (int)(done_before - (total - takers));
      // at most takers - 1 workgroups are still running: the others among the takers
      unsigned polls = 0;
      while (__hip_atomic_load(t.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < total) {
        if (++polls > t.spin_limit) {
          __hip_atomic_store(t.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          role = -1;
          break;
        }
        __builtin_amdgcn_s_sleep(4);
      }
    }
    si[4] = role;
  }
  __syncthreads();
  const int role = si[4];
  if (role < 0) return;
  const int H = t.H;
  for (int seq = role; seq < nseq; seq += (int)takers) {
    float* xr = t.x + (size_t)seq * t.ldx;
    float4 v[8], g[8];
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i = (threadIdx.x + 256 * q) * 4;
      v[q] = g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < H) {
        v[q] = *reinterpret_cast<const float4*>(xr + i);
        g[q] = *reinterpret_cast<const float4*>(t.gain + i);
        const float* pp = part + (size_t)seq * H + i;
        float4 add = make_float4(load_coherent(pp), load_coherent(pp + 1), load_coherent(pp + 2), load_coherent(pp + 3));
        for (int p = 1; p < nparts; ++p) {  // slices are added in a fixed order
          const float* q4 = pp + (size_t)p * part_stride;
          add = make_float4(add.x + load_coherent(q4), add.y + load_coherent(q4 + 1), add.z + load_coherent(q4 + 2),
                            add.w + load_coherent(q4 + 3));
        }
        v[q] = make_float4(v[q].x + add.x, v[q].y + add.y, v[q].z + add.z, v[q].w + add.w);
        *reinterpret_cast<float4*>(xr + i) = v[q];
      }
      ss = sumsq4(ss, v[q]);
    }
    ss = block_sum_256(ss, sm);
    const float r = rms_rinv(ss, H, t.eps);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i = (threadIdx.x + 256 * q) * 4;
      if (i < H) store_normed4<F32, HF>(t.Xp, t.NC, t.nsplit, seq, i, v[q], r, g[q]);
    }
    __syncthreads();  // sm is reused by the next sequence's block sum
  }
}

// ---------------------------------------------------------------------------
// skinny GEMM on the matrix cores (decode GEMV, batched decode, prompt chunks)
// ---------------------------------------------------------------------------
// Workgroup = 4 waves.  blockIdx.x picks RT adjacent 16-row tiles, blockIdx.y a
// slice of the k tiles; the four waves take k tiles of the slice round-robin, so
// the workgroup walks memory contiguously.  Per k tile a wave loads RT x 1 KiB of
// weights (one 16-byte load per lane per tile) and NCB operand fragments, and
// issues RT x NCB matrix-core instructions (x4 k-steps for fp32).  Partial
// accumulators of the four waves meet in LDS; the epilogue adds the bf16 pieces
// of each activation column and stores / accumulates / applies SwiGLU.
template <bool F32, int NCB, int RT, int EPI, int U, class HF>
__global__ __launch_bounds__(256) void k_gemm_skinny(GemmArgs a) {
  constexpr bool W8 = !F32 && HF::kW8;  // byte weights: two operand k tiles per weight tile
  constexpr int XT = W8 ? 2 : 1;
  constexpr int RC = RT % 2 == 0 ? 2 : 1;  // row tiles per round of the cross-wave reduction
  __shared__ float red[4][RC][NCB][256];
  // the wave index as a scalar: every k-tile address below is then a scalar base plus a
  // per-lane offset that does not change in the loop
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int c16 = lane & 15, g = lane >> 4;
  const int KT = a.KT;
  const int kt_begin = blockIdx.y * a.kts_per_split;
  const int kt_end = min(KT, kt_begin + a.kts_per_split);
  const uint4* __restrict__ W = static_cast<const uint4*>(a.Wp);
  const uint4* __restrict__ X = static_cast<const uint4*>(a.Xp);
  const size_t tile0 = (size_t)blockIdx.x * RT;

  f32x4 acc[RT][NCB];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[rt][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Two register sets of U k tiles each: the loads of the next group are in flight while the
  // matrix cores work on the current one.  The pipelined loop runs over this wave's full groups
  // of U k tiles; its loads are unconditional (a group index past the end is clamped to the
  // wave's last k tile: a repeated read that is never multiplied), so the loop has no
  // data-dependent branch and no select on loaded data, and the compiler waits for exactly the
  // set it needs.  The k tiles left over (fewer than U) follow one at a time.  Native vector
  // types: arrays of the HIP uint4 struct carried across a loop end up in scratch memory.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4* __restrict__ Wv = reinterpret_cast<const u32x4*>(W);
  const u32x4* __restrict__ Xv = reinterpret_cast<const u32x4*>(X);
  // Loads go through buffer descriptors: a scalar descriptor, a per-lane byte offset that never
  // changes (lane * 16 for the weights, the lane's operand fragment within a k tile for the
  // operand) and a scalar offset per k tile.  No vector register is written to form an address
  // inside the loop.  (With 64-bit vector addresses the compiler recycled registers of earlier
  // load results for them and waited for every outstanding load before it issued the next set.)
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<u32x4*>(Wv + tile0 * KT * 64), 0, RT * KT * 1024, 0x00020000);
  const __amdgpu_buffer_rsrc_t xres =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4*>(Xv), 0, KT * XT * 64 * a.NC, 0x00020000);
  const uint32_t wvoff = (uint32_t)lane * 16u;
  uint32_t xvoff[NCB];  // operand fragment of this lane within a k tile's 4 x NC groups of 16 bytes
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) xvoff[cb] = (uint32_t)(g * a.NC + min(cb * 16 + c16, a.NC - 1)) * 16u;
  // this wave's k tiles: first, first + 4, ... (n_mine of them)
  const int first = kt_begin + wave;
  const int n_mine = first < kt_end ? (kt_end - first + 3) >> 2 : 0;
  const int last_kt = first + 4 * (n_mine - 1);
  u32x4 avA[U][RT], bvA[U][XT * NCB], avB[U][RT], bvB[U][XT * NCB];
  auto load_tile = [&](int kt, u32x4(&av)[RT], u32x4(&bv)[XT * NCB]) __attribute__((always_inline)) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)  // aux 2: non-temporal, each weight byte is used once per pass
      av[rt] = __builtin_amdgcn_raw_buffer_load_b128(wres, wvoff, (rt * KT + kt) * 1024, 2);
#pragma unroll
    for (int x = 0; x < XT; ++x)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
        bv[x * NCB + cb] = __builtin_amdgcn_raw_buffer_load_b128(xres, xvoff[cb], (kt * XT + x) * 64 * a.NC, 0);
  };
  auto load_group = [&](int t0, u32x4(&av)[U][RT], u32x4(&bv)[U][XT * NCB]) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < U; ++u) load_tile(min(first + 4 * (t0 + u), last_kt), av[u], bv[u]);
  };
  auto mma_tile = [&](const u32x4(&av)[RT], const u32x4(&bv)[XT * NCB]) __attribute__((always_inline)) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      if constexpr (W8) {
        const u32x4 a0 = HF::widen8(av[rt][0], av[rt][1]), a1 = HF::widen8(av[rt][2], av[rt][3]);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
          acc[rt][cb] = HF::mfma(a0, bv[cb], acc[rt][cb]);
          acc[rt][cb] = HF::mfma(a1, bv[NCB + cb], acc[rt][cb]);
        }
        continue;
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        if constexpr (F32) {
          const float4 af = __builtin_bit_cast(float4, av[rt]);
          const float4 bf = __builtin_bit_cast(float4, bv[cb]);
          acc[rt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, bf.x, acc[rt][cb], 0, 0, 0);
          acc[rt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, bf.y, acc[rt][cb], 0, 0, 0);
          acc[rt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, bf.z, acc[rt][cb], 0, 0, 0);
          acc[rt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, bf.w, acc[rt][cb], 0, 0, 0);
        } else {
          acc[rt][cb] = HF::mfma(av[rt], bv[cb], acc[rt][cb]);
        }
      }
    }
  };
  auto mma_group = [&](const u32x4(&av)[U][RT], const u32x4(&bv)[U][XT * NCB]) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < U; ++u) mma_tile(av[u], bv[u]);
  };
  const int n_groups = n_mine / U;
  if (n_groups > 0) {
    load_group(0, avA, bvA);
    // The scheduling barriers keep the order written here: the next set's loads are issued before
    // the matrix-core work on the current set starts.  Without them the scheduler sinks each set's
    // loads below the preceding products (shorter live ranges), so that nothing is in flight
    // while a set is consumed and every pass of the loop pays one full memory latency.
    for (int gi = 0;;) {
      load_group((gi + 1) * U, avB, bvB);
      __builtin_amdgcn_sched_barrier(0);
      mma_group(avA, bvA);
      __builtin_amdgcn_sched_barrier(0);
      if (++gi >= n_groups) break;
      load_group((gi + 1) * U, avA, bvA);
      __builtin_amdgcn_sched_barrier(0);
      mma_group(avB, bvB);
      __builtin_amdgcn_sched_barrier(0);
      if (++gi >= n_groups) break;
    }
  }
  for (int t = n_groups * U; t < n_mine; ++t) {
    load_tile(first + 4 * t, avA[0], bvA[0]);
    mma_tile(avA[0], bvA[0]);
  }

  // accumulator element i of a lane is output row (lane/16)*4 + i, operand column lane%16.
  // The four waves' partial tiles meet in LDS, RC row tiles at a time (one SwiGLU pair), so the
  // buffer does not grow with RT.
  const int nsplit = a.nsplit, nseq = a.nseq;
  float* out = a.out;
  if constexpr (EPI != EPI_SWIGLU)
    if (a.step_ptr) out += (size_t)(*a.step_ptr) * a.step_stride;
#pragma unroll
  for (int ch = 0; ch < RT / RC; ++ch) {
    if (ch) __syncthreads();
#pragma unroll
    for (int r = 0; r < RC; ++r)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[wave][r][cb][i * 64 + lane] = acc[ch * RC + r][cb][i];
    __syncthreads();
    auto total = [&](int r, int row, int seq) {
      float v = 0.f;
      for (int s = 0; s < nsplit; ++s) {
        const int col = seq * nsplit + s;
        const int idx = (row & 3) * 64 + (row >> 2) * 16 + (col & 15);
        const int cb = col >> 4;
        v += (red[0][r][cb][idx] + red[1][r][cb][idx]) + (red[2][r][cb][idx] + red[3][r][cb][idx]);
      }
      return v;
    };
    if constexpr (EPI == EPI_SWIGLU) {
      static_assert(EPI != EPI_SWIGLU || RT % 2 == 0, "SwiGLU needs (gate, up) tile pairs");
      for (int o = tid; o < 16 * nseq; o += 256) {
        const int seq = o >> 4, row = o & 15;
        float gate = total(0, row, seq);
        float up = total(1, row, seq);
        if constexpr (W8) {
          const float* sc = a.wscale + ((size_t)blockIdx.x * RT + ch * 2) * 16 + row;
          gate *= sc[0];
          up *= sc[16];
        }
        const float act = gate / (1.0f + expf(-gate)) * up;
        const int f = (blockIdx.x * (RT / 2) + ch) * 16 + row;
        store_packed<F32, HF>(a.packed_out, a.NC_out, a.nsplit_out, seq, f, act);
      }
    } else {
      for (int o = tid; o < RC * 16 * nseq; o += 256) {
        const int r = o / (16 * nseq);
        const int rem = o - r * 16 * nseq;
        const int seq = rem >> 4, row = rem & 15;
        // each k slice stores its own partial sums: slice s goes to out + s * split_stride
        float* dst = out + (size_t)blockIdx.y * a.split_stride + (size_t)seq * a.ldo + (tile0 + ch * RC + r) * 16 + row;
        float y = total(r, row, seq);
        if constexpr (W8) y *= a.wscale[(tile0 + ch * RC + r) * 16 + row];
        if (a.tail.counter) store_through(dst, y);
        else *dst = y;
      }
    }
  }
  if constexpr (EPI == EPI_STORE) {
    if (a.tail.counter) {
      __syncthreads();  // every wave is done with the reduction buffer
      gemm_norm_tail<F32, HF>(a.tail, out, a.split_stride, (int)gridDim.y, nseq, &red[0][0][0][0]);
    }
  }
}

template <bool F32, int NCB, int RT, int EPI, class HF>
static hipError_t gemm_dispatch(hipStream_t s, const GemmArgs& a) {
  const int ksplit = (a.KT + a.kts_per_split - 1) / a.kts_per_split;
  dim3 grid(a.n_tiles / RT, ksplit);
  constexpr int U = (RT * NCB <= 2) ? 4 : 2;
  k_gemm_skinny<F32, NCB, RT, EPI, U, HF><<<grid, 256, 0, s>>>(a);
  return hipGetLastError();
}

template <bool F32, int EPI, int RT, class HF>
static hipError_t gemm_dispatch_ncb(hipStream_t s, const GemmArgs& a) {
  const int ncb = (a.ncols + 15) / 16;
  switch (ncb) {
    case 1: return gemm_dispatch<F32, 1, RT, EPI, HF>(s, a);
    case 2: return gemm_dispatch<F32, 2, RT, EPI, HF>(s, a);
    case 3: return gemm_dispatch<F32, 3, RT, EPI, HF>(s, a);
    case 4: return gemm_dispatch<F32, 4, RT, EPI, HF>(s, a);
    default: return hipErrorInvalidValue;
  }
}

// RT (16-row tiles per workgroup) is 2 for SwiGLU and for matrices with many rows,
// 1 for the narrow output projections, where more workgroups matter more.  Those
// also split k across workgroups; each slice stores its own partial result and the
// consumer (k_rmsnorm_pack / k_fold_residual) adds the slices in a fixed order, so
// results do not depend on scheduling.  With more than 16 operand columns (batched decode)
// every workgroup re-reads the whole operand from L2, all of them the same lines at about the
// same time; twice the row tiles per workgroup halve that traffic, and a launch takes them
// unless that leaves the last round of workgroups over the CUs clearly emptier (8B gate|up:
// 768 workgroups of two tile pairs fill three rounds, 384 of four only 1.5; 1.7B QKV: 256
// workgroups of one tile rather than 128 of two; the LM head has thousands either way).
static int cu_count() {
  static const int n = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
      v = 256;
    return v;
  }();
  return n;
}

template <bool F32, int EPI, int RT, class HF>
static hipError_t gemm_dispatch_rt(hipStream_t s, const GemmArgs& a) {
  const int ncb = (a.ncols + 15) / 16;
  if (ncb >= 2 && ncb <= 3 && a.n_tiles % (2 * RT) == 0) {
    const int ks = (a.KT + a.kts_per_split - 1) / a.kts_per_split, cus = cu_count();
    auto fullness = [&](int wgs) { return (double)wgs / ((double)((wgs + cus - 1) / cus) * cus); };
    if (fullness(a.n_tiles / (2 * RT) * ks) >= fullness(a.n_tiles / RT * ks) - 0.05)
      return gemm_dispatch_ncb<F32, EPI, 2 * RT, HF>(s, a);
  }
  return gemm_dispatch_ncb<F32, EPI, RT, HF>(s, a);
}

hipError_t launch_gemm(hipStream_t s, int dt, int epi, const GemmArgs& a) {
  if (a.ncols <= 0 || a.ncols > MAX_COLS || a.ncols > a.NC || a.nseq * a.nsplit != a.ncols ||
      a.kts_per_split <= 0 || a.n_tiles <= 0)
    return hipErrorInvalidValue;
  const bool wide = a.n_tiles >= 1024 && (a.n_tiles % 2 == 0);
  if (epi != EPI_STORE && epi != EPI_SWIGLU) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU && (a.n_tiles % 2 || a.kts_per_split < a.KT)) return hipErrorInvalidValue;
  if (a.tail.counter && (epi != EPI_STORE || a.step_ptr || a.ldo != a.tail.H || a.tail.H != a.n_tiles * 16 ||
                         a.tail.H % 4 || a.tail.H > 8192 || !a.tail.error || (a.KT + a.kts_per_split - 1) / a.kts_per_split > 8))
    return hipErrorInvalidValue;
  if (a.wscale) {  // byte weights, bf16 activations
    if (dt != DT_BF16 || a.tail.counter) return hipErrorInvalidValue;
    const int rt = a.rt > 0 ? a.rt : (epi == EPI_SWIGLU || wide ? 2 : 1);
    if (a.n_tiles % rt) return hipErrorInvalidValue;
    if (epi == EPI_SWIGLU) {
      if (rt == 2) return gemm_dispatch_ncb<false, EPI_SWIGLU, 2, Bf16W8>(s, a);
      if (rt == 4) return gemm_dispatch_ncb<false, EPI_SWIGLU, 4, Bf16W8>(s, a);
      if (rt == 6) return gemm_dispatch_ncb<false, EPI_SWIGLU, 6, Bf16W8>(s, a);
      if (rt == 8) return gemm_dispatch_ncb<false, EPI_SWIGLU, 8, Bf16W8>(s, a);
      return hipErrorInvalidValue;
    }
    if (rt == 1) return gemm_dispatch_ncb<false, EPI_STORE, 1, Bf16W8>(s, a);
    if (rt == 2) return gemm_dispatch_ncb<false, EPI_STORE, 2, Bf16W8>(s, a);
    if (rt == 3) return gemm_dispatch_ncb<false, EPI_STORE, 3, Bf16W8>(s, a);
    if (rt == 4) return gemm_dispatch_ncb<false, EPI_STORE, 4, Bf16W8>(s, a);
    if (rt == 6) return gemm_dispatch_ncb<false, EPI_STORE, 6, Bf16W8>(s, a);
    return hipErrorInvalidValue;
  }
  if (a.rt > 0) {  // row tiles per workgroup chosen by the caller (the analytic planner)
    if (a.n_tiles % a.rt || (epi == EPI_SWIGLU && a.rt % 2)) return hipErrorInvalidValue;
    if (epi == EPI_SWIGLU) {
      if (a.rt == 2) NNC_FOR_DTYPE(dt, return gemm_dispatch_ncb<F32, EPI_SWIGLU, 2, HF>(s, a));
      if (a.rt == 4) NNC_FOR_DTYPE(dt, return gemm_dispatch_ncb<F32, EPI_SWIGLU, 4, HF>(s, a));
      if (dt == DT_F32) return hipErrorInvalidValue;
      if (a.rt == 6) NNC_FOR_HALF(dt, return gemm_dispatch_ncb<false, EPI_SWIGLU, 6, HF>(s, a));
      if (a.rt == 8) NNC_FOR_HALF(dt, return gemm_dispatch_ncb<false, EPI_SWIGLU, 8, HF>(s, a));
      return hipErrorInvalidValue;
    }
    if (a.rt == 1) NNC_FOR_DTYPE(dt, return gemm_dispatch_ncb<F32, EPI_STORE, 1, HF>(s, a));
    if (a.rt == 2) NNC_FOR_DTYPE(dt, return gemm_dispatch_ncb<F32, EPI_STORE, 2, HF>(s, a));
    if (a.rt == 4) NNC_FOR_DTYPE(dt, return gemm_dispatch_ncb<F32, EPI_STORE, 4, HF>(s, a));
    if (dt == DT_F32) return hipErrorInvalidValue;
    if (a.rt == 3) NNC_FOR_HALF(dt, return gemm_dispatch_ncb<false, EPI_STORE, 3, HF>(s, a));
    if (a.rt == 6) NNC_FOR_HALF(dt, return gemm_dispatch_ncb<false, EPI_STORE, 6, HF>(s, a));
    return hipErrorInvalidValue;
  }
  if (epi == EPI_SWIGLU) NNC_FOR_DTYPE(dt, return gemm_dispatch_rt<F32, EPI_SWIGLU, 2, HF>(s, a));
  if (wide) NNC_FOR_DTYPE(dt, return gemm_dispatch_rt<F32, EPI_STORE, 2, HF>(s, a));
  NNC_FOR_DTYPE(dt, return gemm_dispatch_rt<F32, EPI_STORE, 1, HF>(s, a));
}

// Which sequence position a column of a pass stands for: decode passes look it up in the
// device-resident column state; prompt blocks are `ncols` consecutive positions of one slot.
__device__ __forceinline__ uint32_t col_pos(const ColMap& cm, int col) { return cm.st ? cm.st->pos[col] : cm.pos0 + col; }
__device__ __forceinline__ uint32_t col_slot(const ColMap& cm, int col) { return cm.st ? cm.st->slot[col] : cm.slot; }

// QK-norm and rotary embedding of one head held as (a, b) = elements (lane, lane + 64) of a wave:
// the one definition both the separate kernel and the fused attention kernel use.  Every
// multiply-add is written out (fused by builtin, or left unfused under contract(off)), so the two
// kernels round alike whatever the compiler would contract on its own.
__device__ __forceinline__ void qk_norm_rope(float& a, float& b, float eps, float ga, float gb, float2 cs) {
#pragma clang fp contract(off)
  const float bb = b * b;
  const float ss = wave_sum(__builtin_fmaf(a, a, bb));
  const float r = 1.0f / sqrtf(__builtin_fmaf(ss, 1.0f / 128.0f, eps));
  const float ar = a * r, br = b * r;
  a = ar * ga;
  b = br * gb;
  const float bsn = b * cs.y, asn = a * cs.y;
  const float ra = __builtin_fmaf(a, cs.x, -bsn);
  const float rb = __builtin_fmaf(b, cs.x, asn);
  a = ra;
  b = rb;
}

// ---------------------------------------------------------------------------
// per-head QK RMSNorm + rotary embedding + KV append (head_dim 128)
// ---------------------------------------------------------------------------
// One wave per (column, head).  Lane i holds elements i and i+64 of the head,
// which is exactly one rotary pair (half-split pairing).  q heads are normed,
// rotated and written back in place (fp32); k heads are normed, rotated and
// stored in the cache; v heads are stored as they are.
// Cache layout: [slot][kv head][position][128], one such array per layer.
template <bool F32, class HF>
__global__ __launch_bounds__(64) void k_qknorm_rope_append(
    float* __restrict__ qkv, int nq, int nkv, const float* __restrict__ gq, const float* __restrict__ gk,
    float eps, const float2* __restrict__ rope, ColMap cm, void* __restrict__ kc,
    void* __restrict__ vc, uint32_t max_seq, uint16_t* __restrict__ qsplit, uint16_t* __restrict__ vt,
    uint32_t vt_stride) {
  const int col = blockIdx.y, hh = blockIdx.x, lane = threadIdx.x;
  const int ld = (nq + 2 * nkv) * 128;
  float* p = qkv + (size_t)(cm.row0 + col) * ld + (size_t)hh * 128;
  const uint32_t pos = col_pos(cm, col), slot = col_slot(cm, col);
  float a = p[lane], b = p[lane + 64];
  const bool is_v = hh >= nq + nkv;
  if (!is_v) {
    const float* gg = hh < nq ? gq : gk;
    qk_norm_rope(a, b, eps, gg[lane], gg[lane + 64], rope[(size_t)pos * 64 + lane]);
  }
  if (hh < nq) {
    p[lane] = a;
    p[lane + 64] = b;
    if (qsplit) {
      // the query also as three bf16 pieces [column][head][piece][128]: the matrix-core
      // attention kernel loads them as operand fragments without converting anything
      uint32_t pa[3], pb[3];
      split_pieces<HF>(a, 3, pa);
      split_pieces<HF>(b, 3, pb);
      uint16_t* q = qsplit + ((size_t)col * nq + hh) * 3 * 128;
#pragma unroll
      for (int pc = 0; pc < 3; ++pc) {
        q[pc * 128 + lane] = (uint16_t)pa[pc];
        q[pc * 128 + lane + 64] = (uint16_t)pb[pc];
      }
    }
    return;
  }
  const int kvh = is_v ? hh - nq - nkv : hh - nq;
  const size_t row = (((size_t)slot * nkv + kvh) * max_seq + pos) * 128;
  void* dst = is_v ? vc : kc;
  if constexpr (F32) {
    static_cast<float*>(dst)[row + lane] = a;
    static_cast<float*>(dst)[row + lane + 64] = b;
  } else {
    static_cast<uint16_t*>(dst)[row + lane] = (uint16_t)HF::bits(a);
    static_cast<uint16_t*>(dst)[row + lane + 64] = (uint16_t)HF::bits(b);
    if (is_v && vt) {
      // prompt blocks: also the transposed copy [kv head][dim][position] that the
      // matrix-core prompt attention reads
      vt[((size_t)kvh * 128 + lane) * vt_stride + pos] = (uint16_t)HF::bits(a);
      vt[((size_t)kvh * 128 + lane + 64) * vt_stride + pos] = (uint16_t)HF::bits(b);
    }
  }
}

hipError_t launch_qknorm_rope_append(hipStream_t s, int dt, float* qkv, int nq, int nkv,
                                     const float* gq, const float* gk, float eps,
                                     const float2* rope, const ColMap& cm, int ncols, void* kc,
                                     void* vc, uint32_t max_batch, uint32_t max_seq, void* qsplit, void* vt,
                                     uint32_t vt_stride) {
  (void)max_batch;
  dim3 grid(nq + 2 * nkv, ncols);
  uint16_t* qs = static_cast<uint16_t*>(qsplit);
  if (dt == DT_F32) {
    qs = nullptr;
    vt = nullptr;
    vt_stride = 0;
  }
  NNC_FOR_DTYPE(dt, k_qknorm_rope_append<F32, HF><<<grid, 64, 0, s>>>(qkv, nq, nkv, gq, gk, eps, rope, cm, kc, vc, max_seq,
                                                                       qs, static_cast<uint16_t*>(vt), vt_stride));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// split-KV attention for one new token per column (decode, and prompt chunks
// whose columns are consecutive positions of one slot)
// ---------------------------------------------------------------------------
// grid (chunk, kv head x head groups, column); 4 waves.  A workgroup covers
// ATT_CHUNK cached positions of one kv head for GH query heads that share it, so
// each cached byte is read once per group.  Scores go through LDS; the chunk's
// own max / sum / weighted value sum (un-normalised) are written as a partial
// that k_attn_combine merges with the other chunks (online-softmax rescaling).
// 16 lanes cover one cached row (8 elements each), a wave covers 4 rows per step.
template <bool F32, class HF>
__device__ __forceinline__ void load_row8(const void* base, size_t elem, float* v) {
  if constexpr (F32) {
    const float4 x = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
    const float4 y = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem + 4);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
  } else {
    const uint4 x = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem);
    v[0] = HF::lo(x.x); v[1] = HF::hi(x.x);
    v[2] = HF::lo(x.y); v[3] = HF::hi(x.y);
    v[4] = HF::lo(x.z); v[5] = HF::hi(x.z);
    v[6] = HF::lo(x.w); v[7] = HF::hi(x.w);
  }
}

// The same 8-element slice as raw register data (no conversion yet), so that all loads of a
// chunk can be in flight before the first one is used.
template <bool F32>
struct Row8Raw {
  float4 a, b;  // fp32: 8 floats; 16-bit formats: `a` reinterpreted as 8 stored values
};
template <bool F32>
__device__ __forceinline__ Row8Raw<F32> load_row8_raw(const void* base, size_t elem) {
  Row8Raw<F32> r;
  if constexpr (F32) {
    r.a = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
    r.b = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem + 4);
  } else {
    r.a = *reinterpret_cast<const float4*>(static_cast<const uint16_t*>(base) + elem);
    r.b = r.a;
  }
  return r;
}
template <bool F32, class HF>
__device__ __forceinline__ void widen_row8(const Row8Raw<F32>& r, float* v) {
  if constexpr (F32) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w;
    v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
  } else {
    const uint32_t x = __float_as_uint(r.a.x), y = __float_as_uint(r.a.y), z = __float_as_uint(r.a.z),
                   w = __float_as_uint(r.a.w);
    v[0] = HF::lo(x); v[1] = HF::hi(x);
    v[2] = HF::lo(y); v[3] = HF::hi(y);
    v[4] = HF::lo(z); v[5] = HF::hi(z);
    v[6] = HF::lo(w); v[7] = HF::hi(w);
  }
}

template <bool F32, int GH, class HF>
__global__ __launch_bounds__(256) void k_attn_partial(
    const float* __restrict__ qkv, int nq, int nkv, const void* __restrict__ kc,
    const void* __restrict__ vc, uint32_t max_seq, ColMap cm,
    float* __restrict__ partial, int max_chunks) {
  __shared__ float sc[GH][ATT_CHUNK];      // scores, then softmax weights
  __shared__ float red[4][4][GH][128];     // value sums per wave and per row group of 16 lanes
  __shared__ float sm_m[GH], sm_l[GH];
  const int chunk = blockIdx.x, col = blockIdx.z;
  const int G = nq / nkv;
  const int groups = G / GH;
  const int kvh = blockIdx.y / groups, hg = blockIdx.y % groups;
  const int head0 = kvh * G + hg * GH;
  const uint32_t pos = col_pos(cm, col), slot = col_slot(cm, col);
  const uint32_t j0 = (uint32_t)chunk * ATT_CHUNK;
  if (j0 > pos) return;  // chunk lies entirely in the future (uniform for the workgroup)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c16 = lane & 15, jj = lane >> 4;
  const int ld = (nq + 2 * nkv) * 128;
  const size_t base = ((size_t)slot * nkv + kvh) * max_seq * 128;

  // this lane's 8-element slice of each query head
  float q[GH][8];
#pragma unroll
  for (int h = 0; h < GH; ++h) {
    const float* qp = qkv + (size_t)(cm.row0 + col) * ld + (size_t)(head0 + h) * 128 + c16 * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) q[h][e] = qp[e];
  }
  const float scale = 0.08838834764831845f;  // 1 / sqrt(128)

  // all K and V rows of the chunk that this lane group touches, loaded up front (rows past
  // `pos` re-read row `pos`: valid memory, masked below)
  Row8Raw<F32> kraw[ATT_CHUNK / 16], vraw[ATT_CHUNK / 16];
#pragma unroll
  for (int it = 0; it < ATT_CHUNK / 16; ++it) {
    const uint32_t j = min(j0 + (uint32_t)(it * 16 + wave * 4 + jj), pos);
    kraw[it] = load_row8_raw<F32>(kc, base + (size_t)j * 128 + c16 * 8);
    vraw[it] = load_row8_raw<F32>(vc, base + (size_t)j * 128 + c16 * 8);
  }

  // scores s[h][j] = <q_h, K_j> / sqrt(d); positions beyond `pos` get -inf
#pragma unroll
  for (int it = 0; it < ATT_CHUNK / 16; ++it) {
    const int jl = it * 16 + wave * 4 + jj;
    const uint32_t j = j0 + jl;
    const bool valid = j <= pos;
    float kv[8];
    widen_row8<F32, HF>(kraw[it], kv);
#pragma unroll
    for (int h = 0; h < GH; ++h) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d += q[h][e] * kv[e];
      d = row16_sum(d);
      if (c16 == 0) sc[h][jl] = valid ? d * scale : -INFINITY;
    }
  }
  __syncthreads();

  // chunk max, weights exp(s - max), chunk sum: one wave per head
  for (int h = wave; h < GH; h += 4) {
    const float s = sc[h][lane];  // ATT_CHUNK == 64 == wave size
    const float m = wave_max(s);
    const float w = expf(s - m);  // exp(-inf) = 0 for masked positions; position j0 is always valid
    sc[h][lane] = w;
    const float l = wave_sum(w);
    if (lane == 0) {
      sm_m[h] = m;
      sm_l[h] = l;
    }
  }
  __syncthreads();

  // weighted value sum
  float acc[GH][8];
#pragma unroll
  for (int h = 0; h < GH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
#pragma unroll
  for (int it = 0; it < ATT_CHUNK / 16; ++it) {
    const int jl = it * 16 + wave * 4 + jj;
    float vv[8];
    widen_row8<F32, HF>(vraw[it], vv);  // masked positions have weight 0 and hold row `pos` (finite)
#pragma unroll
    for (int h = 0; h < GH; ++h) {
      const float w = sc[h][jl];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] += w * vv[e];
    }
  }
#pragma unroll
  for (int h = 0; h < GH; ++h) {
    float4* dst = reinterpret_cast<float4*>(&red[wave][jj][h][c16 * 8]);
    dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
    dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
  }
  __syncthreads();
  // partial record per (column, head, chunk): 128 value sums, then max, then sum
  for (int o = tid; o < GH * 128; o += 256) {
    const int h = o >> 7, i = o & 127;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) v += (red[w][0][h][i] + red[w][1][h][i]) + (red[w][2][h][i] + red[w][3][h][i]);
    float* rec = partial + (((size_t)col * nq + head0 + h) * max_chunks + chunk) * 132;
    rec[i] = v;
    if (i == 0) {
      rec[128] = sm_m[h];
      rec[129] = sm_l[h];
    }
  }
}

// The same partial on the matrix cores (bf16 cache): one workgroup per (chunk, kv head,
// column) handles ALL query heads of the kv head as the 16 operand columns (G <= 16).
//   S^T = K Q^T : A = the wave's 16 cached K rows straight from the cache, B = the query heads
//                 (three bf16 pieces each: fp32-grade), one 16 x 16 tile of scores per wave.
//   softmax     : scores meet in LDS, one wave per head (64 positions = 64 lanes).
//   O^T = V^T P^T : the chunk's V rows are staged in LDS as they are; a lane gathers its
//                 A fragment (one head dimension, 8 positions) with eight 32-bit LDS reads
//                 (row stride 66 words: conflict-free), B = the weights in three pieces.
// Replaces 8 multiply-adds per cached element and head on the vector ALU, which bounded the
// vector version at about half of the HBM rate.
// FUSED (decode passes: every column is a different slot, G <= 8): the workgroup also does what
// k_qknorm_rope_append does for its column and kv head -- QK-norm and RoPE of the G query heads
// from the raw projection output (every chunk's workgroup repeats that: 128 values per head),
// and, in the workgroup whose chunk holds the new position, of the new K row, which it appends
// to the cache together with the V row and patches into its own operands (the row is not in the
// cache when the loads are issued).  One kernel less per layer.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
struct AttnFuse {
  const float* qkv;   // [slices][columns][(nq + 2 nkv) * 128] raw q | k | v, as k-slice partial sums
  const float* gq;    // QK-norm gains
  const float* gk;
  float eps;
  const float2* rope;
  int slices;         // partial sums to add, in slice order (>= 1)
  long slice_stride;  // floats between them
};
template <bool FUSED, class HF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(FUSED ? 6 : 5, FUSED ? 6 : 5))) void k_attn_partial_mc(const uint16_t* __restrict__ qsplit, AttnFuse fz, int nq,
                                                         int nkv, uint16_t* __restrict__ kc,
                                                         uint16_t* __restrict__ vc, uint32_t max_seq, ColMap cm,
                                                         float* __restrict__ partial, int max_chunks) {
  constexpr int VS = 66;  // row stride of the staged V chunk in 32-bit words (128 bf16 + pad)
  __shared__ uint32_t Vs[ATT_CHUNK][VS];
  constexpr int HMAX = FUSED ? 8 : 16;  // query heads per kv head the variant serves
  // scores per head; one word of padding per row: the four lanes that write one position of four
  // heads then hit four banks instead of one
  __shared__ float sc[HMAX][ATT_CHUNK + 1];
  // softmax weights as three bf16 pieces; before the scores exist the same bytes hold the query
  // pieces of the fused variant ([3][8][128]), which every wave has in registers by then
  // (fused: 8 heads at a row stride of 96 elements = 48 words, so that the 16-byte reads of four
  // heads' rows fall on disjoint banks; the query pieces that share the bytes are [3][8][128] with
  // the 16-byte chunks of a row rotated by the head, for the same reason)
  constexpr int PWS = FUSED ? 96 : ATT_CHUNK;
  __shared__ __attribute__((aligned(16))) uint16_t pwbuf[3 * 16 * ATT_CHUNK];  // = 3 * 8 * 128
  static_assert(3 * HMAX * PWS <= 3 * 16 * ATT_CHUNK, "the weights fit the shared bytes");
  uint16_t(*pw)[HMAX][PWS] = reinterpret_cast<uint16_t(*)[HMAX][PWS]>(&pwbuf[0]);
  __shared__ __attribute__((aligned(16))) uint16_t knew[128], vnew[128];
  __shared__ float sm_m[16], sm_l[16];
  const int kvh = blockIdx.y, col = blockIdx.z;
  const int G = nq / nkv, head0 = kvh * G;
  const uint32_t pos = col_pos(cm, col), slot = col_slot(cm, col);
  const int chunk = blockIdx.x;
  const uint32_t j0 = (uint32_t)chunk * ATT_CHUNK;
  if (j0 > pos) return;  // chunk lies entirely in the future (uniform for the workgroup)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c16 = lane & 15, g = lane >> 4;
  const size_t base = ((size_t)slot * nkv + kvh) * max_seq * 128;

  // rows past the last cached one re-read it: valid memory, finite values, masked / weight 0
  // below (fused: row `pos` is not cached yet; it is patched in from the role waves)
  const uint32_t jlast = FUSED ? (pos > 0 ? pos - 1 : 0) : pos;
  const bool owns_new = pos - j0 < (uint32_t)ATT_CHUNK;
  uint2 vreg[4][2];
  u32x4_t kf[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t j = min(j0 + (uint32_t)((tid >> 4) + 16 * i), jlast);
    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(vc + base + (size_t)j * 128 + (tid & 15) * 8);
    vreg[i][0] = make_uint2(v.x, v.y);
    vreg[i][1] = make_uint2(v.z, v.w);
  }
  {
    // K fragments: A-operand row c16 = position j0 + wave * 16 + c16, 8 dims per lane and k step
    const uint32_t jk = min(j0 + (uint32_t)(wave * 16 + c16), jlast);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      kf[ks] = *reinterpret_cast<const u32x4_t*>(kc + base + (size_t)jk * 128 + ks * 32 + g * 8);
  }
  uint16_t(*qp)[8][128] = reinterpret_cast<uint16_t(*)[8][128]>(&pwbuf[0]);
  // element e of head row r sits in 16-byte chunk (e / 8) ^ (4 * (r & 3)) of the row
  auto qsw = [](int r, int e) __attribute__((always_inline)) { return (((e >> 3) ^ ((r & 3) << 2)) << 3) | (e & 7); };
  if constexpr (FUSED) {
    // roles 0 .. G-1: query heads; G: the new K row; G + 1: the new V row (same arithmetic, in
    // the same order, as k_qknorm_rope_append)
    const int ld = (nq + 2 * nkv) * 128;
    const float* row = fz.qkv + (size_t)col * ld;
    for (int role = wave; role < G + 2; role += 4) {
      if (role >= G && !owns_new) continue;
      const float* p = role < G ? row + (size_t)(head0 + role) * 128
                                : row + (size_t)(nq + (role == G ? 0 : nkv) + kvh) * 128;
      float a = p[lane], b = p[lane + 64];
      for (int sl = 1; sl < fz.slices; ++sl) {
        a += p[(size_t)sl * fz.slice_stride + lane];
        b += p[(size_t)sl * fz.slice_stride + lane + 64];
      }
      if (role <= G) {
        const float* gg = role < G ? fz.gq : fz.gk;
        qk_norm_rope(a, b, fz.eps, gg[lane], gg[lane + 64], fz.rope[(size_t)pos * 64 + lane]);
      }
      if (role < G) {
        uint32_t pa[3], pb[3];
        split_pieces<HF>(a, 3, pa);
        split_pieces<HF>(b, 3, pb);
#pragma unroll
        for (int pc = 0; pc < 3; ++pc) {
          qp[pc][role][qsw(role, lane)] = (uint16_t)pa[pc];
          qp[pc][role][qsw(role, lane + 64)] = (uint16_t)pb[pc];
        }
      } else {
        const uint16_t ha = (uint16_t)HF::bits(a), hb = (uint16_t)HF::bits(b);
        uint16_t* dst = (role == G ? kc : vc) + base + (size_t)pos * 128;
        dst[lane] = ha;
        dst[lane + 64] = hb;
        uint16_t* keep = role == G ? knew : vnew;
        keep[lane] = ha;
        keep[lane + 64] = hb;
      }
    }
    __syncthreads();
    if (j0 + (uint32_t)(wave * 16 + c16) == pos) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) kf[ks] = *reinterpret_cast<const u32x4_t*>(&knew[ks * 32 + g * 8]);
    }
  }

  // query fragments: operand column c16 = head head0 + c16, three pieces as written by
  // k_qknorm_rope_append
  u32x4_t qf[4][3];
  {
    const uint16_t* qg = qsplit + ((size_t)col * nq + head0 + min(c16, G - 1)) * 3 * 128 + g * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int pc = 0; pc < 3; ++pc) {
        const u32x4_t t = FUSED ? *reinterpret_cast<const u32x4_t*>(&qp[pc][min(c16, G - 1)][qsw(min(c16, G - 1), ks * 32 + g * 8)])
                                : *reinterpret_cast<const u32x4_t*>(qg + pc * 128 + ks * 32);
        qf[ks][pc] = t;  // columns beyond G repeat head G - 1: their results are never stored
      }
  }

  {
    f32x4 sv = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int pc = 0; pc < 3; ++pc)
        sv = HF::mfma(kf[ks], qf[ks][pc], sv);
    // lane (c16 = head, g): positions wave * 16 + g * 4 + i of the chunk
    if (c16 < G) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int jl = wave * 16 + g * 4 + i;
        sc[c16][jl] = j0 + (uint32_t)jl <= pos ? sv[i] * 0.08838834764831845f : -INFINITY;
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint2* d = reinterpret_cast<uint2*>(&Vs[(tid >> 4) + 16 * i][(tid & 15) * 4]);
      if (FUSED && j0 + (uint32_t)((tid >> 4) + 16 * i) == pos) {
        const uint2* nv = reinterpret_cast<const uint2*>(&vnew[(tid & 15) * 8]);
        d[0] = nv[0];
        d[1] = nv[1];
      } else {
        d[0] = vreg[i][0];
        d[1] = vreg[i][1];
      }
    }
    __syncthreads();  // (fused: every wave holds its query fragments in registers; the LDS behind them becomes pw)

    // chunk max, weights exp(s - max), chunk sum: one wave per head
    for (int h = wave; h < G; h += 4) {
      const float x = sc[h][lane];
      const float m = wave_max(x);
      const float w = expf(x - m);  // exp(-inf) = 0 for masked positions; position j0 is always valid
      // the weights go to LDS already split into bf16 pieces (once, not once per consuming wave)
      float r = w;
#pragma unroll
      for (int pc = 0; pc < 3; ++pc) {
        const uint32_t b = HF::bits(r);
        pw[pc][h][lane] = (uint16_t)b;
        r -= HF::widen(b);
      }
      const float l = wave_sum(w);
      if (lane == 0) {
        sm_m[h] = m;
        sm_l[h] = l;
      }
    }
    __syncthreads();

    // weighted value sums: this wave's two 16-dim tiles, two halves of 32 positions
    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // B operand: lane (c16 = head, g) holds the weights of positions half * 32 + g * 8 .. + 7
      u32x4_t pf[3];
#pragma unroll
      for (int pc = 0; pc < 3; ++pc) {
        const u32x4_t t = *reinterpret_cast<const u32x4_t*>(&pw[pc][min(c16, G - 1)][half * 32 + g * 8]);
        pf[pc] = t;
      }
#pragma unroll
      for (int dtl = 0; dtl < 2; ++dtl) {
        const int dim = (wave * 2 + dtl) * 16 + c16;  // A-operand row c16 = this head dimension
        // the lane's dimension is the low or the high half of a staged word: one byte permute
        // takes that half of two positions' words at once
        const uint32_t sel = (dim & 1) ? 0x07060302u : 0x05040100u;
        uint32_t two[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) two[e] = Vs[half * 32 + g * 8 + e][dim >> 1];
        const u32x4_t vf = u32x4_t{__builtin_amdgcn_perm(two[1], two[0], sel), __builtin_amdgcn_perm(two[3], two[2], sel),
                                   __builtin_amdgcn_perm(two[5], two[4], sel), __builtin_amdgcn_perm(two[7], two[6], sel)};
#pragma unroll
        for (int pc = 0; pc < 3; ++pc)
          acc[dtl] = HF::mfma(vf, pf[pc], acc[dtl]);
      }
    }
    // acc[dtl] element i of lane (c16 = head, g): dimension (wave * 2 + dtl) * 16 + g * 4 + i
    if (c16 < G) {
      float* rec = partial + (((size_t)col * nq + head0 + c16) * max_chunks + chunk) * 132;
#pragma unroll
      for (int dtl = 0; dtl < 2; ++dtl)
        *reinterpret_cast<float4*>(rec + (wave * 2 + dtl) * 16 + g * 4) =
            make_float4(acc[dtl][0], acc[dtl][1], acc[dtl][2], acc[dtl][3]);
    }
    if (tid < G) {
      float* rec = partial + (((size_t)col * nq + head0 + tid) * max_chunks + chunk) * 132;
      rec[128] = sm_m[tid];
      rec[129] = sm_l[tid];
    }
  }
}

// Prompt chunks (the columns are consecutive positions of one slot): the same arithmetic per
// (column, head) as k_attn_partial_mc, but one workgroup serves every column from one read of its
// cache chunk -- the (column, head) pairs are the operand columns, sixteen at a time.
template <class HF>
__global__ __launch_bounds__(256) void k_attn_partial_shared(const uint16_t* __restrict__ qsplit, int nq, int nkv,
                                                             const uint16_t* __restrict__ kc,
                                                             const uint16_t* __restrict__ vc, uint32_t max_seq,
                                                             ColMap cm, int ncols, float* __restrict__ partial,
                                                             int max_chunks) {
  constexpr int VS = 66;
  __shared__ uint32_t Vs[ATT_CHUNK][VS];
  __shared__ float sc[16][ATT_CHUNK];
  __shared__ __attribute__((aligned(16))) uint16_t pw[3][16][ATT_CHUNK];
  __shared__ float sm_m[16], sm_l[16];
  const int kvh = blockIdx.y, chunk = blockIdx.x;
  const int G = nq / nkv, head0 = kvh * G;
  const uint32_t pos0 = col_pos(cm, 0), slot = col_slot(cm, 0);  // column c stands for position pos0 + c
  const uint32_t pos_last = pos0 + (uint32_t)ncols - 1;  // every column's row is in the cache already
  const uint32_t j0 = (uint32_t)chunk * ATT_CHUNK;
  if (j0 > pos_last) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c16 = lane & 15, g = lane >> 4;
  const size_t base = ((size_t)slot * nkv + kvh) * max_seq * 128;
  // rows past the last cached one re-read it: valid memory, finite values, masked below
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t j = min(j0 + (uint32_t)((tid >> 4) + 16 * i), pos_last);
    const uint4 v = *reinterpret_cast<const uint4*>(vc + base + (size_t)j * 128 + (tid & 15) * 8);
    uint2* d = reinterpret_cast<uint2*>(&Vs[(tid >> 4) + 16 * i][(tid & 15) * 4]);
    d[0] = make_uint2(v.x, v.y);
    d[1] = make_uint2(v.z, v.w);
  }
  u32x4_t kf[4];
  {
    const uint32_t jk = min(j0 + (uint32_t)(wave * 16 + c16), pos_last);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      kf[ks] = *reinterpret_cast<const u32x4_t*>(kc + base + (size_t)jk * 128 + ks * 32 + g * 8);
  }
  const int nops = ncols * G;  // operand columns: (column, head of this kv head)
  for (int op0 = 0; op0 < nops; op0 += 16) {
    const int op = op0 + c16;
    const bool valid = op < nops;
    const int col = valid ? op / G : ncols - 1, hd = valid ? op - col * G : 0;
    const uint32_t pos = pos0 + (uint32_t)col;
    u32x4_t qf[4][3];
    {
      const uint16_t* qg = qsplit + ((size_t)col * nq + head0 + hd) * 3 * 128 + g * 8;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int pc = 0; pc < 3; ++pc) {
          const u32x4_t t = *reinterpret_cast<const u32x4_t*>(qg + pc * 128 + ks * 32);
          qf[ks][pc] = valid ? t : u32x4_t{0u, 0u, 0u, 0u};
        }
    }
    f32x4 sv = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int pc = 0; pc < 3; ++pc)
        sv = HF::mfma(kf[ks], qf[ks][pc], sv);
    // lane (c16 = operand column, g): positions wave * 16 + g * 4 + i of the chunk
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int jl = wave * 16 + g * 4 + i;
      sc[c16][jl] = valid && j0 + (uint32_t)jl <= pos ? sv[i] * 0.08838834764831845f : -INFINITY;
    }
    __syncthreads();  // scores (and, the first time round, the staged V rows) are in LDS

    // chunk max, weights exp(s - max), chunk sum: one wave per operand column; a column whose
    // position lies before this chunk has no valid score (weights 0, nothing stored)
    for (int r = wave; r < 16; r += 4) {
      const float x = sc[r][lane];
      const float m = wave_max(x);
      const float w = m == -INFINITY ? 0.f : expf(x - m);
      float rr = w;
#pragma unroll
      for (int pc = 0; pc < 3; ++pc) {
        const uint32_t b = HF::bits(rr);
        pw[pc][r][lane] = (uint16_t)b;
        rr -= HF::widen(b);
      }
      const float l = wave_sum(w);
      if (lane == 0) {
        sm_m[r] = m;
        sm_l[r] = l;
      }
    }
    __syncthreads();

    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      u32x4_t pf[3];
#pragma unroll
      for (int pc = 0; pc < 3; ++pc) pf[pc] = *reinterpret_cast<const u32x4_t*>(&pw[pc][c16][half * 32 + g * 8]);
#pragma unroll
      for (int dtl = 0; dtl < 2; ++dtl) {
        const int dim = (wave * 2 + dtl) * 16 + c16;
        // the lane's dimension is the low or the high half of a staged word: one byte permute
        // takes that half of two positions' words at once
        const uint32_t sel = (dim & 1) ? 0x07060302u : 0x05040100u;
        uint32_t two[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) two[e] = Vs[half * 32 + g * 8 + e][dim >> 1];
        const u32x4_t vf = u32x4_t{__builtin_amdgcn_perm(two[1], two[0], sel), __builtin_amdgcn_perm(two[3], two[2], sel),
                                   __builtin_amdgcn_perm(two[5], two[4], sel), __builtin_amdgcn_perm(two[7], two[6], sel)};
#pragma unroll
        for (int pc = 0; pc < 3; ++pc)
          acc[dtl] = HF::mfma(vf, pf[pc], acc[dtl]);
      }
    }
    if (valid && j0 <= pos) {
      float* rec = partial + (((size_t)col * nq + head0 + hd) * max_chunks + chunk) * 132;
#pragma unroll
      for (int dtl = 0; dtl < 2; ++dtl)
        *reinterpret_cast<float4*>(rec + (wave * 2 + dtl) * 16 + g * 4) =
            make_float4(acc[dtl][0], acc[dtl][1], acc[dtl][2], acc[dtl][3]);
    }
    if (tid < 16 && op0 + tid < nops) {
      const int c2 = (op0 + tid) / G, h2 = (op0 + tid) - c2 * G;
      if (j0 <= pos0 + (uint32_t)c2) {
        float* rec = partial + (((size_t)c2 * nq + head0 + h2) * max_chunks + chunk) * 132;
        rec[128] = sm_m[tid];
        rec[129] = sm_l[tid];
      }
    }
    __syncthreads();  // scores, weights and row statistics have been read
  }
}

bool attn_partial_can_fuse(int dt, int nq, int nkv) { return dt != DT_F32 && nq / nkv <= 8; }

// fuse != NULL: raw projection output, gains and rotary table for the fused variant (the caller
// then does not launch k_qknorm_rope_append; columns must be different slots).
hipError_t launch_attn_partial(hipStream_t s, int dt, const float* qkv, const void* qsplit, int nq, int nkv,
                               void* kc, void* vc, uint32_t max_batch, uint32_t max_seq,
                               const ColMap& cm, int ncols, int grid_chunks, float* partial,
                               int max_chunks, const AttnFuseArgs* fuse, bool one_slot) {
  (void)max_batch;
  const int G = nq / nkv;
  const bool f32 = dt == DT_F32, f16 = dt == DT_F16;
  if (fuse) {
    if (!attn_partial_can_fuse(dt, nq, nkv) || cm.row0 != 0 || !cm.st) return hipErrorInvalidValue;
    dim3 grid(grid_chunks, nkv, ncols);
    const AttnFuse fz{qkv, fuse->gq, fuse->gk, fuse->eps, fuse->rope, fuse->qkv_slices > 1 ? fuse->qkv_slices : 1,
                      fuse->qkv_slice_stride};
    if (f16)
      k_attn_partial_mc<true, Fp16><<<grid, 256, 0, s>>>(nullptr, fz, nq, nkv, static_cast<uint16_t*>(kc),
                                                         static_cast<uint16_t*>(vc), max_seq, cm, partial, max_chunks);
    else
      k_attn_partial_mc<true, Bf16><<<grid, 256, 0, s>>>(nullptr, fz, nq, nkv, static_cast<uint16_t*>(kc),
                                                         static_cast<uint16_t*>(vc), max_seq, cm, partial, max_chunks);
    return hipGetLastError();
  }
  if (!f32 && G <= 16 && qsplit && cm.row0 == 0 && one_slot && ncols > 1) {
    // prompt chunk: consecutive positions of one slot share each read of the cache
    dim3 grid(grid_chunks, nkv);
    if (f16)
      k_attn_partial_shared<Fp16><<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(qsplit), nq, nkv,
                                                       static_cast<const uint16_t*>(kc), static_cast<const uint16_t*>(vc),
                                                       max_seq, cm, ncols, partial, max_chunks);
    else
      k_attn_partial_shared<Bf16><<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(qsplit), nq, nkv,
                                                       static_cast<const uint16_t*>(kc), static_cast<const uint16_t*>(vc),
                                                       max_seq, cm, ncols, partial, max_chunks);
    return hipGetLastError();
  }
  if (!f32 && G <= 16 && qsplit && cm.row0 == 0) {
    dim3 grid(grid_chunks, nkv, ncols);
    if (f16)
      k_attn_partial_mc<false, Fp16><<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(qsplit), AttnFuse{}, nq, nkv,
                                                          static_cast<uint16_t*>(kc), static_cast<uint16_t*>(vc), max_seq,
                                                          cm, partial, max_chunks);
    else
      k_attn_partial_mc<false, Bf16><<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(qsplit), AttnFuse{}, nq, nkv,
                                                          static_cast<uint16_t*>(kc), static_cast<uint16_t*>(vc), max_seq,
                                                          cm, partial, max_chunks);
    return hipGetLastError();
  }
  const int GH = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  dim3 grid(grid_chunks, nkv * (G / GH), ncols);
#define NNC_ATT(H) \
  NNC_FOR_DTYPE(dt, k_attn_partial<F32, H, HF><<<grid, 256, 0, s>>>(qkv, nq, nkv, kc, vc, max_seq, cm, partial, max_chunks))
  if (GH == 4) NNC_ATT(4); else if (GH == 2) NNC_ATT(2); else NNC_ATT(1);
#undef NNC_ATT
  return hipGetLastError();
}

// Merge the chunk partials of one (column, head) and write the attention output
// as the packed operand of the output projection (k index = head * 128 + i).
//   M = max_c m_c;  o = sum_c e^{m_c - M} O_c / sum_c e^{m_c - M} l_c
// Output: split-bf16 (or fp32) columns of the skinny GEMM operand.
template <bool F32, class HF>
__global__ __launch_bounds__(512) void k_attn_combine(const float* __restrict__ partial, int max_chunks,
                                                      int nq, ColMap cm, void* __restrict__ Op, int NC,
                                                      int nsplit) {
  // four groups of 128 threads (one per head dimension) take the chunks round-robin and merge
  // them online; the four running (max, sum, weighted sum) triples meet in LDS
  __shared__ float sM[4], sden[4], snum[4][128];
  const int head = blockIdx.x, col = blockIdx.y, i = threadIdx.x & 127, q = threadIdx.x >> 7;
  const int nchunks = (int)(col_pos(cm, col) / ATT_CHUNK) + 1;
  const float* rec0 = partial + ((size_t)col * nq + head) * max_chunks * 132;
  float M = -INFINITY, num = 0.f, den = 0.f;
#pragma unroll 4
  for (int c = q; c < nchunks; c += 4) {
    const float* rec = rec0 + (size_t)c * 132;
    const float m = rec[128], l = rec[129], a = rec[i];
    const float Mn = fmaxf(M, m);
    const float sc = expf(M - Mn), f = expf(m - Mn);  // sc = 0 on the first chunk (M = -inf)
    num = num * sc + f * a;
    den = den * sc + f * l;
    M = Mn;
  }
  snum[q][i] = num;
  if (i == 0) {
    sM[q] = M;
    sden[q] = den;
  }
  __syncthreads();
  if (q != 0) return;
  const float Mt = fmaxf(fmaxf(sM[0], sM[1]), fmaxf(sM[2], sM[3]));
  float n = 0.f, d = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float f = expf(sM[w] - Mt);  // groups without a chunk: exp(-inf) = 0
    n += f * snum[w][i];
    d += f * sden[w];
  }
  store_packed<F32, HF>(Op, NC, nsplit, col, head * 128 + i, n / d);
}

hipError_t launch_attn_combine(hipStream_t s, int dt, const float* partial, int max_chunks, int nq,
                               const ColMap& cm, int ncols, void* Op, int NC, int nsplit) {
  dim3 grid(nq, ncols);
  NNC_FOR_DTYPE(dt, k_attn_combine<F32, HF><<<grid, 512, 0, s>>>(partial, max_chunks, nq, cm, Op, NC, nsplit));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// greedy arg-max over the vocabulary (lowest index wins ties)
// ---------------------------------------------------------------------------
constexpr int ARGMAX_BLOCKS = 64;

__device__ __forceinline__ void argmax_merge(float& v, int32_t& i, float ov, int32_t oi) {
  if (ov > v || (ov == v && oi < i)) {
    v = ov;
    i = oi;
  }
}

__global__ __launch_bounds__(256) void k_argmax_part(const float* __restrict__ logits, long ld, int V,
                                                     const uint32_t* step_ptr, long step_stride,
                                                     float* __restrict__ pv, int32_t* __restrict__ pi) {
  __shared__ float sv[4];
  __shared__ int32_t si[4];
  const int col = blockIdx.y;
  const float* row = logits + (size_t)col * ld;
  if (step_ptr) row += (size_t)(*step_ptr) * step_stride;
  float best = -INFINITY;
  int32_t bi = 0x7fffffff;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < V; i += ARGMAX_BLOCKS * 256) {
    const float v = row[i];
    if (v > best) {  // indices increase within a thread, so strict > keeps the lowest
      best = v;
      bi = i;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int32_t oi = __shfl_xor(bi, o, 64);
    argmax_merge(best, bi, ov, oi);
  }
  if ((threadIdx.x & 63) == 0) {
    sv[threadIdx.x >> 6] = best;
    si[threadIdx.x >> 6] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) argmax_merge(best, bi, sv[w], si[w]);
    pv[col * ARGMAX_BLOCKS + blockIdx.x] = best;
    pi[col * ARGMAX_BLOCKS + blockIdx.x] = bi;
  }
}

__global__ __launch_bounds__(64) void k_argmax_final(const float* __restrict__ pv,
                                                     const int32_t* __restrict__ pi,
                                                     int32_t* __restrict__ next) {
  const int col = blockIdx.x;
  float best = pv[col * ARGMAX_BLOCKS + threadIdx.x];
  int32_t bi = pi[col * ARGMAX_BLOCKS + threadIdx.x];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int32_t oi = __shfl_xor(bi, o, 64);
    argmax_merge(best, bi, ov, oi);
  }
  if (threadIdx.x == 0) next[col] = bi == 0x7fffffff ? 0 : bi;
}

hipError_t launch_argmax(hipStream_t s, const float* logits, long ld, int V, int ncols,
                         const uint32_t* step_ptr, long step_stride, float* scratch_val,
                         int32_t* scratch_idx, int32_t* next) {
  static_assert(ARGMAX_BLOCKS == 64, "final pass assumes one wave of partials");
  k_argmax_part<<<dim3(ARGMAX_BLOCKS, ncols), 256, 0, s>>>(logits, ld, V, step_ptr, step_stride,
                                                           scratch_val, scratch_idx);
  k_argmax_final<<<ncols, 64, 0, s>>>(scratch_val, scratch_idx, next);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// inspection / plumbing
// ---------------------------------------------------------------------------
// cache [kv head][position][128] of one slot and layer -> out [n][nkv*128] fp32
template <bool F32, class HF>
__global__ __launch_bounds__(128) void k_kv_read(const void* __restrict__ cache, uint32_t max_seq, int nkv,
                                                 uint32_t pos0, float* __restrict__ out) {
  const int kvh = blockIdx.x, t = blockIdx.y, i = threadIdx.x;
  const size_t e = ((size_t)kvh * max_seq + pos0 + t) * 128 + i;
  float v;
  if constexpr (F32)
    v = static_cast<const float*>(cache)[e];
  else
    v = HF::widen(static_cast<const uint16_t*>(cache)[e]);
  out[((size_t)t * nkv + kvh) * 128 + i] = v;
}

hipError_t launch_kv_read(hipStream_t s, int dt, const void* cache, uint32_t max_seq, int nkv,
                          uint32_t pos0, uint32_t n, float* out) {
  dim3 grid(nkv, n);
  NNC_FOR_DTYPE(dt, k_kv_read<F32, HF><<<grid, 128, 0, s>>>(cache, max_seq, nkv, pos0, out));
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_copy(const float* __restrict__ src, float* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy_rows(hipStream_t s, const float* src, float* dst, size_t n) {
  const unsigned grid = (unsigned)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  k_copy<<<grid ? grid : 1, 256, 0, s>>>(src, dst, n);
  return hipGetLastError();
}

}  // namespace nnc
