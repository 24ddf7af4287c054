// gfx950 (MI355X) kernels of the DISCO speculative-decoding hot path.
//
// Data layout shared by the kernels
//   * packed weights: 1 KiB tiles of 16 rows x 32 columns in the operand order of
//     v_mfma_f32_16x16x32_bf16 (lane l holds row l % 16, columns 8 * (l / 16) .. + 7), tiles of one
//     16-row group contiguous along K.  A wavefront fetches a tile with one 128-bit load per lane,
//     1 KiB contiguous, and streams a row group as one contiguous slab.
//   * activation panels ("xpack"): the token side of the same instruction.  Activations stay fp32
//     between kernels in value: each is split into bf16 hi = rne(x) and lo = rne(x - hi), so the
//     bf16 matrix unit reproduces fp32-grade products.  For M <= 8 tokens one panel holds hi in
//     columns 0..7 and lo in columns 8..15 (one MFMA per weight tile); for M <= 16 two panels
//     (hi, lo).  Panel element (column n, k) lives at ((kt * 64) + (k % 32 / 8) * 16 + n) * 8 + k % 8,
//     kt = k / 32, panels K * 16 elements apart.
//   * paged KV: [layer][physical page][K | V][kv head] blocks of page_tokens x d_head bf16; a K block
//     is [token][d_head], a V block is transposed, [d_head][token] (see the attention kernel).
#include "disco_internal.h"

#include <mutex>

namespace disco {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define NEG_BIG (-1.0e30f)

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_to_f32(bf16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even (the hardware conversion of gfx950)
  return __builtin_bit_cast(bf16_t, (__bf16)f);
}

__device__ __forceinline__ bool gated(const uint32_t* gate) {
  return gate != nullptr && __builtin_nontemporal_load(gate) != 0u;
}
// The halt flag's value, requested but not waited for: kernels of the draft loop issue their first
// operand loads behind it and test it just before they would wait for those, so that the flag's round
// trip does not stand in front of every launch of the step (a halted step's launches still end there).
__device__ __forceinline__ uint32_t gate_request(const uint32_t* gate) {
  return gate != nullptr ? __builtin_nontemporal_load(gate) : 0u;
}

// Stores and loads of data that another workgroup of the SAME launch reads or has written (COH): agent-scope
// relaxed atomics, which on gfx950 are write-through stores and L2-bypassing loads, coherent across the
// eight XCDs' separate L2s.  Without COH they are plain accesses (the consumer is a later launch).
template <bool COH> __device__ __forceinline__ void st_f4(float* p, float a, float b, float c, float d) {
  if (COH) {
    const unsigned long long v0 = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
    const unsigned long long v1 = (unsigned long long)__float_as_uint(c) | ((unsigned long long)__float_as_uint(d) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), v0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p) + 1, v1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
  }
}
template <bool COH> __device__ __forceinline__ float4 ld_f4(const float* p) {
  if (COH) {
    const unsigned long long v0 = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long v1 = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float4(__uint_as_float((uint32_t)v0), __uint_as_float((uint32_t)(v0 >> 32)), __uint_as_float((uint32_t)v1), __uint_as_float((uint32_t)(v1 >> 32)));
  }
  return *reinterpret_cast<const float4*>(p);
}
template <bool COH> __device__ __forceinline__ float ld_f1(const float* p) {
  if (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return *p;
}
template <bool COH> __device__ __forceinline__ void st_f1(float* p, float v) {
  if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}
template <bool COH> __device__ __forceinline__ void st_u2(bf16_t* p, uint2 v) {
  if (COH) __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), (unsigned long long)v.x | ((unsigned long long)v.y << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *reinterpret_cast<uint2*>(p) = v;
}
template <bool COH> __device__ __forceinline__ void st_h1(bf16_t* p, bf16_t v) {
  if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}

// Store 4 consecutive-k activations of token m into the packed panels as bf16 hi/lo.
template <bool COH = false>
__device__ __forceinline__ void xpack_store4(bf16_t* X, int KT, int M, int m, int k, const float* v) {
  const int kt = k >> 5, grp = (k & 31) >> 3, e = k & 7;
  uint32_t hi[2], lo[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    bf16_t h0 = f32_to_bf16(v[2 * i]), h1 = f32_to_bf16(v[2 * i + 1]);
    bf16_t l0 = f32_to_bf16(v[2 * i] - bf16_to_f32(h0)), l1 = f32_to_bf16(v[2 * i + 1] - bf16_to_f32(h1));
    hi[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    lo[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);
  }
  const size_t base = ((size_t)kt * 64 + grp * 16) * 8 + e;
  size_t off_hi, off_lo;
  if (M <= 8) { off_hi = base + (size_t)m * 8; off_lo = base + (size_t)(m + 8) * 8; }
  else { off_hi = base + (size_t)m * 8; off_lo = (size_t)KT * 512 + base + (size_t)m * 8; }
  st_u2<COH>(X + off_hi, make_uint2(hi[0], hi[1]));
  st_u2<COH>(X + off_lo, make_uint2(lo[0], lo[1]));
}

// Wavefront reductions on the DPP cross-lane network (no LDS traffic): xor-1, xor-2 inside quads,
// half-row mirror, row mirror, then row broadcasts 15 and 31; lane 63 ends up with the result, which
// is broadcast through a scalar register.  The combination order is fixed, so sums are reproducible.
#define DPP_QUAD_XOR1 0xB1
#define DPP_QUAD_XOR2 0x4E
#define DPP_ROW_HALF_MIRROR 0x141
#define DPP_ROW_MIRROR 0x140
#define DPP_ROW_BCAST15 0x142
#define DPP_ROW_BCAST31 0x143

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float old, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xF, false);
}

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<DPP_QUAD_XOR1, 0xF>(0.f, v);
  v += dpp_f<DPP_QUAD_XOR2, 0xF>(0.f, v);
  v += dpp_f<DPP_ROW_HALF_MIRROR, 0xF>(0.f, v);
  v += dpp_f<DPP_ROW_MIRROR, 0xF>(0.f, v);
  v += dpp_f<DPP_ROW_BCAST15, 0xA>(0.f, v);
  v += dpp_f<DPP_ROW_BCAST31, 0xC>(0.f, v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<DPP_QUAD_XOR1, 0xF>(v, v));
  v = fmaxf(v, dpp_f<DPP_QUAD_XOR2, 0xF>(v, v));
  v = fmaxf(v, dpp_f<DPP_ROW_HALF_MIRROR, 0xF>(v, v));
  v = fmaxf(v, dpp_f<DPP_ROW_MIRROR, 0xF>(v, v));
  v = fmaxf(v, dpp_f<DPP_ROW_BCAST15, 0xA>(v, v));
  v = fmaxf(v, dpp_f<DPP_ROW_BCAST31, 0xC>(v, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Hand-off between workgroups of one launch (split reductions).  Data written by one workgroup and
// read by another inside the same kernel moves with agent-scope relaxed atomic stores / loads: on
// gfx950 these are write-through / L2-bypassing accesses (sc1), coherent across the eight XCDs'
// separate L2s without the L2-wide write-back and invalidate that an agent-scope fence costs.  The
// writers drain their stores (s_waitcnt 0) before the workgroup barrier that precedes the ticket.
__device__ __forceinline__ void st_agent2(float* p, float a, float b) {
  const unsigned long long v = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_agent2(const float* p) {
  const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32)));
}
// Ticket of a split reduction: true in every thread of the workgroup that arrives last.
// Ordering: the hand-off data moves with write-through stores and L2-bypassing loads (above), so no cache
// maintenance is needed, and an agent-scope release / acquire on the ticket would add exactly that (an
// L2-wide write-back and invalidate, measured at 8 - 13 us per use on MI355X).  What IS needed is that the
// stores have completed before the ticket is taken (the explicit wait) and that the compiler keeps the
// hand-off accesses on their side of the ticket: the two signal fences are compiler-only barriers.
__device__ __forceinline__ bool last_arrival(int* counter, int n, int* s_flag) {
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_waitcnt(0);                 // this wavefront's hand-off stores have completed
  __syncthreads();
  if (threadIdx.x == 0) {
    const int t = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_flag = (t == n - 1) ? 1 : 0;
    if (t == n - 1) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
  }
  __syncthreads();
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  return *s_flag != 0;
}

// Across the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48), every lane gets the result.
__device__ __forceinline__ float row4_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16));
  return fmaxf(v, __shfl_xor(v, 32));
}
__device__ __forceinline__ float row4_sum(float v) {
  v += __shfl_xor(v, 16);
  return v + __shfl_xor(v, 32);
}

// Block-wide sum in a fixed order (deterministic); every thread gets the result.
template <int NT>
__device__ __forceinline__ float block_sum(float v, float* smem /* NT/64 + 1 floats */) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) t += smem[i];
  return t;
}

// (value, index) arg-max: larger value wins, lower index on equal values.
struct VI { float v; int i; };
__device__ __forceinline__ VI vi_best(VI a, VI b) {
  return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ VI vi_step(VI x) {
  VI y; y.v = dpp_f<CTRL, ROW_MASK>(x.v, x.v); y.i = dpp_i<CTRL, ROW_MASK>(x.i, x.i);
  return vi_best(x, y);
}
__device__ __forceinline__ VI wave_argmax(VI x) {
  x = vi_step<DPP_QUAD_XOR1, 0xF>(x);
  x = vi_step<DPP_QUAD_XOR2, 0xF>(x);
  x = vi_step<DPP_ROW_HALF_MIRROR, 0xF>(x);
  x = vi_step<DPP_ROW_MIRROR, 0xF>(x);
  x = vi_step<DPP_ROW_BCAST15, 0xA>(x);
  x = vi_step<DPP_ROW_BCAST31, 0xC>(x);
  VI r;
  r.v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x.v), 63));
  r.i = __builtin_amdgcn_readlane(x.i, 63);
  return r;
}
template <int NT>
__device__ __forceinline__ VI block_argmax(VI x, float* sv, int* si) {
  x = wave_argmax(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = x.v; si[threadIdx.x >> 6] = x.i; }
  __syncthreads();
  VI r; r.v = sv[0]; r.i = si[0];
#pragma unroll
  for (int i = 1; i < NT / 64; ++i) { VI y; y.v = sv[i]; y.i = si[i]; r = vi_best(r, y); }
  return r;
}

// ---------------------------------------------------------------------------------------------
// weight packing (one-time layout transform)
// ---------------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_pack(const bf16_t* __restrict__ src, int64_t n, int64_t k,
                                             bf16_t* __restrict__ dst, int64_t tile_mul, int64_t tile_add) {
  // one thread per 8-element group of the destination
  const int64_t KT = k >> 5;
  const int64_t total = n * k / 8;
  for (int64_t gidx = (int64_t)blockIdx.x * 256 + threadIdx.x; gidx < total; gidx += (int64_t)gridDim.x * 256) {
    const int64_t lane = gidx & 63, tile = gidx >> 6;
    const int64_t rt = tile / KT, kt = tile % KT;
    const int64_t row = rt * 16 + (lane & 15), col = kt * 32 + (lane >> 4) * 8;
    const uint4 v = *reinterpret_cast<const uint4*>(src + row * k + col);
    const int64_t drt = rt * tile_mul + tile_add;
    *reinterpret_cast<uint4*>(dst + ((drt * KT + kt) * 64 + lane) * 8) = v;
  }
}

hipError_t launch_pack(const bf16_t* src, int64_t n, int64_t k, bf16_t* dst, int64_t tile_mul,
                       int64_t tile_add, hipStream_t s) {
  const int64_t total = n * k / 8;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_pack, dim3((unsigned)blocks), dim3(256), 0, s, src, n, k, dst, tile_mul, tile_add);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// skinny GEMM: weights streamed once from HBM, M <= 16 tokens on the matrix unit's column side
// ---------------------------------------------------------------------------------------------
//
// A work unit is (row group b of RT 16-row tiles, k-tile range [kt_begin, kt_end)).  The NW wavefronts
// of the workgroup interleave over the k-tiles of the range, each keeping U k-tiles of loads in
// flight, and reduce through LDS in a fixed order.  When a row group's K range is covered by n_seg > 1
// units (of different workgroups), each stores its partial 16 x 16 tiles to a plane and takes a
// ticket; the last one to arrive adds the planes in range order and runs the epilogue: no float
// atomics, no waiting, bitwise reproducible results.
//
// k_gemm launches a grid of (row groups, K ranges): every workgroup owns one unit.

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
  union { u32x4 u; bf16x8 b; } c; c.u = v; return c.b;
}

// QKV epilogue of one lane: output features n0 .. n0+3 (lo4) and their rotary partners n0 + d_head/2 ..
// (hi4) of token row m at position pos: rotation, then the query row or the paged K / V entry.
template <bool COH = false>
__device__ __forceinline__ void qkv_store(const GemmArgs& a, float* q, const int n0, const int m, const int pos,
                                          float (&lo4)[4], float (&hi4)[4]) {
  const int dsh = a.dh == 128 ? 7 : 6;            // d_head is 64 or 128
  const int head = n0 >> dsh, c = n0 & (a.dh - 1), half = a.dh >> 1;
  const bool is_v = head >= a.nq + a.nkv;
  if (a.rope_tab != nullptr && !is_v) {
    // (cos, sin) of pos * base^(-2 (c + v) / d_head), tabulated per cached position
    const float4* tab = reinterpret_cast<const float4*>(a.rope_tab + ((size_t)pos * half + c) * 2);
    const float4 t0 = tab[0], t1 = tab[1];
    const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float x0 = lo4[v], x1 = hi4[v];
      lo4[v] = x0 * cs[v] - x1 * sn[v];
      hi4[v] = x1 * cs[v] + x0 * sn[v];
    }
  }
  if (head < a.nq) {
    float* qp = q + (size_t)m * a.ldq + head * a.dh + c;
    st_f4<COH>(qp, lo4[0], lo4[1], lo4[2], lo4[3]);
    st_f4<COH>(qp + half, hi4[0], hi4[1], hi4[2], hi4[3]);
  } else {
    const int sel = is_v ? 1 : 0;
    const int kvh = head - a.nq - sel * a.nkv;
    const int pt = a.page_tokens;
    const bool pow2 = (pt & (pt - 1)) == 0;
    const int lp = pow2 ? pos >> __builtin_ctz(pt) : pos / pt, off = pos - lp * pt;
    const int pp = a.page_table ? a.page_table[lp] : lp;
    bf16_t* blk = a.kv_layer + (((size_t)pp * 2 + sel) * a.nkv + kvh) * a.page_tokens * a.dh;
    if (!is_v) {                 // K: [token][d_head]
      bf16_t* dst = blk + (size_t)off * a.dh + c;
      uint2 u0, u1;
      u0.x = (uint32_t)f32_to_bf16(lo4[0]) | ((uint32_t)f32_to_bf16(lo4[1]) << 16);
      u0.y = (uint32_t)f32_to_bf16(lo4[2]) | ((uint32_t)f32_to_bf16(lo4[3]) << 16);
      u1.x = (uint32_t)f32_to_bf16(hi4[0]) | ((uint32_t)f32_to_bf16(hi4[1]) << 16);
      u1.y = (uint32_t)f32_to_bf16(hi4[2]) | ((uint32_t)f32_to_bf16(hi4[3]) << 16);
      st_u2<COH>(dst, u0);
      st_u2<COH>(dst + half, u1);
    } else {                     // V: transposed, [d_head][token]
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        st_h1<COH>(blk + (size_t)(c + v) * a.page_tokens + off, f32_to_bf16(lo4[v]));
        st_h1<COH>(blk + (size_t)(c + half + v) * a.page_tokens + off, f32_to_bf16(hi4[v]));
      }
    }
  }
}

template <int EPI> struct EpiTraits { static constexpr bool pair = (EPI == EPI_QKV || EPI == EPI_SWIGLU); };

// Register buffers (k-tiles in flight per wavefront) by row tiles per unit and activation panels: as many as the
// register file of a workgroup of eight wavefronts holds next to the accumulators; with two panels two buffers
// measured best at every tile count (a same-box sweep over 2 / 3 / 4 at the 13B shapes).
constexpr int gemm_buffers(int rt, int panels) { return panels >= 2 ? 2 : (rt >= 8 ? 3 : 4); }

// LDS of one GEMM work unit.
template <int RT, int NW, bool LN = false>
struct GemmSmem {
  f32x4 red[NW][RT][64];
  float red_ssq[NW][64];
  float red_sum[LN ? NW : 1][64];                 // per-tile sums of a deferred LayerNorm
  int s_last;
};

// Row tiles of work unit b: RT consecutive tiles, or RT / 2 pairs (tile, tile + grp) for the two-tile epilogues.
template <int RT, int EPI>
__device__ __forceinline__ void gemm_unit_tiles(const GemmArgs& a, const int b, int (&rt)[RT]) {
  constexpr bool PAIR = EpiTraits<EPI>::pair;
  constexpr int UNITS = PAIR ? RT / 2 : RT;
  if (PAIR) {
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      const int bp = b * UNITS + u, gs = __builtin_ctz(a.grp);   // the pairing distance is a power of two
      rt[2 * u] = ((bp >> gs) << (gs + 1)) + (bp & (a.grp - 1));
      rt[(2 * u + 1) % RT] = rt[2 * u] + a.grp;
    }
  } else {
#pragma unroll
    for (int r = 0; r < RT; ++r) rt[r] = b * RT + r;
  }
}

// COH: the unit's inputs were written, and its outputs are read, by other workgroups of the same launch
// (persistent kernel): hand-off accesses instead of plain ones; the activation panels are still plain loads
// (the persistent kernel gives every phase panels at addresses that nobody has read before in the launch).
// `hook` runs once, right after the unit's first weight tiles (two steps per wavefront) have been requested and
// before anything that depends on the unit's inputs is touched: a persistent kernel waits there for the grid
// barrier that ends the phase before, so the weight stream is in flight while that phase drains.
struct NoHook { __device__ __forceinline__ void operator()() const {} };

// LN: the input's norm is a LayerNorm (deferred like the RMSNorm: the panels hold g * h, the producer left per-tile
// sums and sums of squares, and the epilogue applies rstd * (y - mean * wg) + wb).
template <int P, int RT, int EPI, int NW, int U, bool COH = false, typename Hook = NoHook, bool LN = false>
__device__ __forceinline__ void gemm_unit(const GemmArgs& a, const int b, const int kt_begin, const int kt_end,
                                          const int seg, const int n_seg, GemmSmem<RT, NW, LN>& sm, const Hook hook = Hook()) {
  constexpr bool PAIR = EpiTraits<EPI>::pair;
  constexpr int UNITS = PAIR ? RT / 2 : RT;       // output units handled by one wavefront each
  static_assert(!PAIR || RT % 2 == 0, "pair epilogues need an even tile count");
  static_assert(UNITS <= NW, "one epilogue wavefront per unit");
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const uint32_t halted = gate_request(a.gate);
  uint32_t aborted = 0u;                          // requested here, used by the last store
  if (EPI == EPI_STORE) aborted = a.abort_word != nullptr ? __builtin_nontemporal_load(a.abort_word) : 0u;
  int rt[RT];
  gemm_unit_tiles<RT, EPI>(a, b, rt);

  // one accumulator per row tile: with two panels (hi, lo) both products are added into it
  f32x4 acc[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int KT = a.KT;
  const u32x4* Wp[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) Wp[r] = reinterpret_cast<const u32x4*>(a.W) + (size_t)rt[r] * KT * 64 + lane;
  const u32x4* Xp = reinterpret_cast<const u32x4*>(a.X) + lane;

  // U register buffers, one k-tile each: wavefront w takes k-tiles kt_begin + w, + NW, ...; the loads of the next
  // U - 1 steps are in flight while the matrix unit works on a step (U * RT KiB of weights per wavefront: the
  // stream is bound by the bytes in flight, see the launch shapes below).
  auto load_w = [&](u32x4 (&A)[RT], const int k) {
#pragma unroll
    for (int r = 0; r < RT; ++r) A[r] = __builtin_nontemporal_load(Wp[r] + (size_t)k * 64);
  };
  auto load_x = [&](u32x4 (&B)[P], const int k) {
#pragma unroll
    for (int p = 0; p < P; ++p) B[p] = Xp[((size_t)p * KT + k) * 64];
  };
  u32x4 A[U][RT], B[U][P];
  const int kt0 = kt_begin + w;
  // the weights of the first U steps depend on nothing: they go out first
#pragma unroll
  for (int i = 0; i < U; ++i)
    if (kt0 + i * NW < kt_end) load_w(A[i], kt0 + i * NW);
  asm volatile("" ::: "memory");
  hook();

  // deferred RMSNorm: the panels hold g * h (not normalised).  The producer left one sum of squares
  // per token and 16-column tile; every lane fetches a few of them now (lane = token lane % 16,
  // slots (lane / 16) * NW + w + 4 NW k), the loads complete behind the weight stream, and the
  // epilogue adds them up in a fixed order to get 1 / rms.
  constexpr bool NORMED = (EPI != EPI_PARTIAL);
  constexpr int MAXS = NORMED ? 128 / NW : 1;
  static_assert(!LN || NORMED, "only epilogues that read a normalised input defer a LayerNorm");
  float sv[MAXS], su[LN ? MAXS : 1];
  if (NORMED) {
#pragma unroll
    for (int k = 0; k < MAXS; ++k) sv[k] = 0.f;
    if (LN) {
#pragma unroll
      for (int k = 0; k < MAXS; ++k) su[k] = 0.f;
    }
    // rounds of 4 NW slots; the rounds past n_ssq are skipped by a uniform branch (a 768-wide model
    // needs 2 of the 16 rounds: per-lane tests of all 16 cost more than the loads)
    const int rounds = a.ssq != nullptr ? (a.n_ssq + 4 * NW - 1) / (4 * NW) : 0;
#pragma unroll
    for (int k = 0; k < MAXS; ++k) {
      if (k < rounds) {
        const int idx = (lane >> 4) * NW + w + 4 * NW * k;
        sv[k] = idx < a.n_ssq ? a.ssq[idx * 16 + (lane & 15)] : 0.f;   // [slot][token]; plain loads: see k_forward
        if (LN) su[k] = idx < a.n_ssq ? a.sum[idx * 16 + (lane & 15)] : 0.f;
      }
    }
    asm volatile("" ::: "memory");     // keep these loads ahead of the rest of the stream
  }
#pragma unroll
  for (int i = 0; i < U; ++i)
    if (kt0 + i * NW < kt_end) load_x(B[i], kt0 + i * NW);
  if (halted != 0u) return;                       // uniform over the launch; nothing has been written yet
  for (int kt = kt0; kt < kt_end; kt += U * NW) {
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int k = kt + i * NW;
      if (k < kt_end) {
#pragma unroll
        for (int p = 0; p < P; ++p)                // panel outside: RT independent instructions between two on one accumulator
#pragma unroll
          for (int r = 0; r < RT; ++r)
            acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(A[i][r]), as_bf16x8(B[i][p]), acc[r], 0, 0, 0);
        const int kn = k + U * NW;                 // the buffer's next k-tile
        if (kn < kt_end) { load_w(A[i], kn); load_x(B[i], kn); }
      }
    }
  }

  // hi + lo: same panel, columns n and n + 8 (P == 1), or two panels (P == 2)
  __syncthreads();                                // a previous unit of this workgroup has left the buffers
#pragma unroll
  for (int r = 0; r < RT; ++r) {
    f32x4 y = acc[r];
    if (P == 1) {
#pragma unroll
      for (int v = 0; v < 4; ++v) y[v] = acc[r][v] + __shfl_xor(acc[r][v], 8);
    }
    sm.red[w][r][lane] = y;
  }
  if (NORMED) {
    float part = 0.f;
#pragma unroll
    for (int k = 0; k < MAXS; ++k) {
      asm volatile("" : "+v"(sv[k]));  // first use of the early loads is here, after the stream
      part += sv[k];
    }
    sm.red_ssq[w][lane] = part;
    if (LN) {
      float ps = 0.f;
#pragma unroll
      for (int k = 0; k < MAXS; ++k) {
        asm volatile("" : "+v"(su[k]));
        ps += su[k];
      }
      sm.red_sum[w][lane] = ps;
    }
  }
  __syncthreads();
  constexpr int TPU = PAIR ? 2 : 1;               // tiles per unit
  const bool ep = w < UNITS;                      // this wavefront finishes one output unit
  const int m = lane & 15, g = lane >> 4;         // token column, 4-row group of the 16x16 result
  f32x4 y[TPU];
  int urt[TPU];
#pragma unroll
  for (int i = 0; i < TPU; ++i) {
    const int r = (ep ? w : 0) * TPU + i;
    // (runtime index into rt[] would spill it: select with a compile-time loop)
    urt[i] = 0;
#pragma unroll
    for (int rr = 0; rr < RT; ++rr) if (rr == r) urt[i] = rt[rr];
    y[i] = sm.red[0][r][lane];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) y[i] += sm.red[ww][r][lane];   // fixed order: deterministic
  }

  // operands of the residual update that do not depend on other workgroups are fetched before the ticket
  float4 h = make_float4(0.f, 0.f, 0.f, 0.f), gn = h;
  float* hp = nullptr;
  if (EPI == EPI_PARTIAL) {
    const int col = urt[0] * 16 + 4 * g;
    hp = a.h + (size_t)m * a.ld_out + col;
    if (ep && m < a.M) {
      h = ld_f4<COH>(hp);
      if (a.Xout != nullptr) gn = *reinterpret_cast<const float4*>(a.gain + col);
    }
  }

  if (n_seg > 1) {
    // this unit covers part of K: store the partial tiles, take a ticket; the last unit of the row
    // group to arrive adds all partial tiles in range order (so the sum does not depend on arrival
    // order) and finishes the row group.  Nobody waits for anybody.
    float* plane = a.planes + ((size_t)b * GEMM_MAX_SPLIT * RT) * 256 + (size_t)lane * 4;
    if (ep) {
#pragma unroll
      for (int i = 0; i < TPU; ++i) {
        float* dst = plane + ((size_t)seg * RT + (w * TPU + i)) * 256;
        st_agent2(dst, y[i][0], y[i][1]);
        st_agent2(dst + 2, y[i][2], y[i][3]);
      }
    }
    if (!last_arrival(a.counters + b, n_seg, &sm.s_last)) return;
    if (ep) {
#pragma unroll
      for (int i = 0; i < TPU; ++i) {
        float2 pa[GEMM_MAX_SPLIT], pb[GEMM_MAX_SPLIT];
#pragma unroll
        for (int sp = 0; sp < GEMM_MAX_SPLIT; ++sp)
          if (sp < n_seg) {
            const float* src = plane + ((size_t)sp * RT + (w * TPU + i)) * 256;
            pa[sp] = ld_agent2(src); pb[sp] = ld_agent2(src + 2);
          }
        y[i] = f32x4{pa[0].x, pa[0].y, pb[0].x, pb[0].y};
#pragma unroll
        for (int sp = 1; sp < GEMM_MAX_SPLIT; ++sp)
          if (sp < n_seg) { y[i][0] += pa[sp].x; y[i][1] += pa[sp].y; y[i][2] += pb[sp].x; y[i][3] += pb[sp].y; }
      }
    }
  }
  if (NORMED && a.ssq != nullptr) {
    float ss = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww)
#pragma unroll
      for (int gg = 0; gg < 4; ++gg) ss += sm.red_ssq[ww][gg * 16 + m];
    if (LN) {
      float sx = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) sx += sm.red_sum[ww][gg * 16 + m];
      const float mean = sx / (float)a.d_in;
      const float var = fmaxf(ss / (float)a.d_in - mean * mean, 0.f);
      const float rstd = 1.0f / sqrtf(var + a.eps);
#pragma unroll
      for (int i = 0; i < TPU; ++i) {
        const int row = urt[i] * 16 + 4 * g;
        const float4 cg = *reinterpret_cast<const float4*>(a.wg + row), cb = *reinterpret_cast<const float4*>(a.wb + row);
        y[i][0] = rstd * (y[i][0] - mean * cg.x) + cb.x; y[i][1] = rstd * (y[i][1] - mean * cg.y) + cb.y;
        y[i][2] = rstd * (y[i][2] - mean * cg.z) + cb.z; y[i][3] = rstd * (y[i][3] - mean * cg.w) + cb.w;
      }
    } else {
      const float rstd = 1.0f / sqrtf(ss / (float)a.d_in + a.eps);
#pragma unroll
      for (int i = 0; i < TPU; ++i) y[i] *= rstd;
    }
  }

  if (EPI == EPI_PARTIAL) {
    // residual-stream update h += X.W^T
    if (!ep || m >= a.M) return;
    const int col = urt[0] * 16 + 4 * g;
    h.x += y[0][0]; h.y += y[0][1]; h.z += y[0][2]; h.w += y[0][3];
    st_f4<COH>(hp, h.x, h.y, h.z, h.w);
    if (a.Xout != nullptr) {
      // feed the next RMSNorm'ed GEMM: panels of gain * h and this tile's sum of squares
      const float o[4] = {h.x * gn.x, h.y * gn.y, h.z * gn.z, h.w * gn.w};
      xpack_store4<COH>(a.Xout, a.KT_out, a.M, m, col, o);
      const float sq = row4_sum((h.x * h.x + h.y * h.y) + (h.z * h.z + h.w * h.w));
      if (g == 0) st_f1<COH>(a.ssq_out + urt[0] * 16 + m, sq);              // [slot][token]
      if (a.sum_out != nullptr) {
        const float sx = row4_sum((h.x + h.y) + (h.z + h.w));
        if (g == 0) st_f1<COH>(a.sum_out + urt[0] * 16 + m, sx);
      }
    }
    return;
  }
  if (!ep || m >= a.M) return;
  if (EPI == EPI_STORE) {
    if (a.only_row >= 0 && m != a.only_row) return;
    const size_t row_off = a.only_row >= 0 ? 0 : (size_t)m * a.ld_out;
    if (aborted != 0u) y[0] = f32x4{NAN, NAN, NAN, NAN};   // the forward's data is unusable: say so in its result
    st_f4<COH>(a.out + row_off + urt[0] * 16 + 4 * g, y[0][0], y[0][1], y[0][2], y[0][3]);
  } else if (EPI == EPI_QKV) {
    // two tiles: features c .. c+3 and their rotary partners c + dh/2 .. of one head
    float lo4[4], hi4[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) { lo4[v] = y[0][v]; hi4[v] = y[TPU - 1][v]; }
    qkv_store<COH>(a, a.q, urt[0] * 16 + 4 * g, m, a.pos0 + m, lo4, hi4);
  } else if (EPI == EPI_SWIGLU) {
    // tile 0 = gate rows, tile 1 = the matching up rows
    const int f = (urt[0] >> 1) * 16 + 4 * g;
    float act[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float gt = y[0][v];
      act[v] = gt / (1.0f + expf(-gt)) * y[TPU - 1][v];
    }
    xpack_store4<COH>(a.Xout, a.KT_out, a.M, m, f, act);
  } else if (EPI == EPI_GELU) {
    float act[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) act[v] = 0.5f * y[0][v] * (1.0f + erff(y[0][v] * 0.70710678118654752f));
    xpack_store4<COH>(a.Xout, a.KT_out, a.M, m, urt[0] * 16 + 4 * g, act);
  }
}

template <int P, int RT, int EPI, int NW, int U, bool LN = false>
__global__ __launch_bounds__(NW * 64) void k_gemm(GemmArgs a) {
  __shared__ GemmSmem<RT, NW, LN> sm;
  const int split = blockIdx.y;
  const int kt_begin = (int)((int64_t)a.KT * split / a.n_split), kt_end = (int)((int64_t)a.KT * (split + 1) / a.n_split);
  gemm_unit<P, RT, EPI, NW, U, false, NoHook, LN>(a, blockIdx.x, kt_begin, kt_end, split, a.n_split, sm);
}

template <int P, int RT, int EPI, int NW, int U>
static hipError_t launch_gemm_cfg(const GemmArgs& a, hipStream_t s) {
  constexpr int rows = RT * 16;
  if (a.n_rows % rows) return hipErrorInvalidValue;
  if constexpr (EPI == EPI_QKV || EPI == EPI_GELU || EPI == EPI_STORE) {
    if (a.sum != nullptr) {                       // deferred LayerNorm
      hipLaunchKernelGGL((k_gemm<P, RT, EPI, NW, U, true>), dim3(a.n_rows / rows, a.n_split), dim3(NW * 64), 0, s, a);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((k_gemm<P, RT, EPI, NW, U>), dim3(a.n_rows / rows, a.n_split), dim3(NW * 64), 0, s, a);
  return hipGetLastError();
}

// Launch shapes, from sweeps on MI355X at the 13B-class and 68M-class sizes.  Eight wavefronts per
// workgroup and one k-tile per wavefront and step (two register buffers) were best everywhere.  The
// activation panels are re-read from L2 by every workgroup, so wide outputs take 64 or 128 rows per
// workgroup; narrow outputs (d_model rows) take 64 rows and split K so that about 480 workgroups are
// in flight, small matrices take 16-row workgroups.
// Share of the chip's 256 compute units that stay busy when `wgs` equal workgroups are spread over them.
static double cu_fill(long wgs) { return wgs <= 0 ? 0.0 : (double)wgs / (256.0 * (double)((wgs + 255) / 256)); }

int gemm_split_for(int n_rows, int KT, int M) {
  (void)M;
  int s;
  if (n_rows % 64 == 0 && n_rows >= 2048) {
    // about 480 workgroups for a short K, about 240 for a long one (fewer, longer streams), but never a count that
    // leaves a large part of the chip idle in the last round (288 workgroups keep 56 % of the units busy, 480 keep 94 %)
    // and not more than two rounds (96 row groups: 480 workgroups measured 1 - 1.5 % better than 768)
    const int groups = n_rows / 64, target = KT > 256 ? 240 : 480;
    double best = -1.0;
    s = 1;
    for (int c = 1; c <= GEMM_MAX_SPLIT && c <= KT / 16; ++c) {
      const long wgs = (long)groups * c;
      if (c > 1 && wgs > 512) break;
      const double dist = (double)(wgs > target ? wgs - target : target - wgs) / target;
      const double score = cu_fill(wgs) - 0.05 * dist;
      if (score > best + 1e-9) { best = score; s = c; }
    }
  } else {
    s = KT / 24;
  }
  return s < 1 ? 1 : (s > GEMM_MAX_SPLIT ? GEMM_MAX_SPLIT : s);
}

template <int P, int EPI>
static hipError_t launch_gemm_p(const GemmArgs& a, hipStream_t s) {
  constexpr bool PAIR = EpiTraits<EPI>::pair;
  const int n = a.n_rows;
  if constexpr (EPI == EPI_PARTIAL) {
    if (n % 64 == 0 && n >= 2048) return launch_gemm_cfg<P, 4, EPI, 8, gemm_buffers(4, P)>(a, s);
    if (n % 32 == 0 && (int64_t)(n / 32) * a.n_split >= 200) return launch_gemm_cfg<P, 2, EPI, 8, gemm_buffers(2, P)>(a, s);
    return launch_gemm_cfg<P, 1, EPI, 8, gemm_buffers(1, P)>(a, s);
  } else {
    if (EPI != EPI_QKV && a.KT >= 64 && n % 128 == 0 && n / 128 >= 200) return launch_gemm_cfg<P, 8, EPI, 8, gemm_buffers(8, P)>(a, s);
    // 96-row workgroups where they fill the compute units clearly better than 64 rows (24576 rows: 256 workgroups against 384)
    if (EPI != EPI_QKV && a.KT >= 64 && n % 96 == 0 && n / 96 >= 200 && cu_fill(n / 96) > cu_fill(n / 64) + 0.1)
      return launch_gemm_cfg<P, 6, EPI, 8, gemm_buffers(6, P)>(a, s);
    if (n % 64 == 0 && n / 64 >= 200) {
      // a short K (a wavefront sees at most four k-tiles: the 68M-class LM head) is served best by two buffers
      if constexpr (EPI == EPI_STORE) { if (a.KT <= 32) return launch_gemm_cfg<P, 4, EPI, 8, 2>(a, s); }
      return launch_gemm_cfg<P, 4, EPI, 8, gemm_buffers(4, P)>(a, s);
    }
    if constexpr (PAIR) {
      return launch_gemm_cfg<P, 2, EPI, 8, gemm_buffers(2, P)>(a, s);
    } else {
      if (n % 32 == 0 && n / 32 >= 200) return launch_gemm_cfg<P, 2, EPI, 8, gemm_buffers(2, P)>(a, s);
      return launch_gemm_cfg<P, 1, EPI, 8, gemm_buffers(1, P)>(a, s);
    }
  }
}

hipError_t launch_gemm(const GemmArgs& a0, int epi, hipStream_t s) {
  if (a0.M < 1 || a0.M > 16 || a0.KT < 1 || (a0.n_rows & 15)) return hipErrorInvalidValue;
  GemmArgs a = a0;
  if (a.n_split < 1) a.n_split = 1;
  if (epi != EPI_PARTIAL && a.n_split != 1) return hipErrorInvalidValue;
  if (epi == EPI_PARTIAL && (a.h == nullptr || a.n_split > GEMM_MAX_SPLIT || (a.n_split > 1 && (a.counters == nullptr || a.planes == nullptr)))) return hipErrorInvalidValue;
  if (a.ssq != nullptr && (a.n_ssq < 1 || a.n_ssq > 512)) return hipErrorInvalidValue;
  if (a.n_split > a.KT) return hipErrorInvalidValue;
  if (epi != EPI_QKV) a.grp = 1;
  if ((epi == EPI_QKV || epi == EPI_SWIGLU) && (a.n_rows % 32)) return hipErrorInvalidValue;
  if (epi == EPI_QKV && (a.grp < 1 || (a.grp & (a.grp - 1)) != 0 || (a.dh != 64 && a.dh != 128))) return hipErrorInvalidValue;
  const bool p1 = a.M <= 8;
  switch (epi) {
    case EPI_PARTIAL: return p1 ? launch_gemm_p<1, EPI_PARTIAL>(a, s) : launch_gemm_p<2, EPI_PARTIAL>(a, s);
    case EPI_STORE: return p1 ? launch_gemm_p<1, EPI_STORE>(a, s) : launch_gemm_p<2, EPI_STORE>(a, s);
    case EPI_GELU: return p1 ? launch_gemm_p<1, EPI_GELU>(a, s) : launch_gemm_p<2, EPI_GELU>(a, s);
    case EPI_QKV: return p1 ? launch_gemm_p<1, EPI_QKV>(a, s) : launch_gemm_p<2, EPI_QKV>(a, s);
    case EPI_SWIGLU: return p1 ? launch_gemm_p<1, EPI_SWIGLU>(a, s) : launch_gemm_p<2, EPI_SWIGLU>(a, s);
    default: return hipErrorInvalidValue;
  }
}

// ---------------------------------------------------------------------------------------------
// (embedding +) LayerNorm / RMSNorm -> packed activation panels
// ---------------------------------------------------------------------------------------------

// One workgroup per token row.  The row lives in registers: embedding gather (written to the
// residual stream) or the residual stream itself, then the statistics, then the normalised row as
// packed bf16 hi/lo panels -- or, for a deferred RMSNorm, gain * h panels plus the sum of squares.
// tok_override >= 0 replaces the token id read from a.tokens (embedding mode).  COH: the row is handed to other
// workgroups of the same launch.
template <int NT, bool COH = false>
__device__ __forceinline__ void norm_row(const NormArgs& a, const int row, const int tok_override, float* red /* NT / 64 + 1 */,
                                         const uint32_t halted) {
  constexpr int VPT = 2;                       // float4 per thread: d <= NT * 8
  // row = token slot; slots beyond 16 belong to further groups of 16 (prompt pass), whose panels and
  // sums of squares follow those of group 0
  const int m = row & 15, grp = row >> 4, t = threadIdx.x, d = a.d;
  float* h = a.h + (size_t)row * d;
  bf16_t* Xout = a.Xout + (size_t)grp * d * 32;
  float4 v[VPT];
  const bf16_t* e = nullptr; const bf16_t* pe = nullptr;
  if (a.tokens || tok_override >= 0) {
    int tok = tok_override >= 0 ? tok_override : ((a.n_tok == 0 || row < a.n_tok) ? a.tokens[row] : 0);   // padding slots: token 0
    tok = tok < 0 ? 0 : (tok >= a.vocab ? a.vocab - 1 : tok);
    int pos = a.pos0 + row;
    if (pos >= a.max_pos) pos = a.max_pos - 1;
    e = a.tok_emb + (size_t)tok * a.tok_stride;
    pe = a.pos_emb ? a.pos_emb + (size_t)pos * d : nullptr;
  }
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int k = (i * NT + t) * 4;
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k < d) {
      if (e) {
        const uint2 u = *reinterpret_cast<const uint2*>(e + k);
        v[i] = make_float4(bf16_to_f32(u.x & 0xFFFF), bf16_to_f32(u.x >> 16), bf16_to_f32(u.y & 0xFFFF), bf16_to_f32(u.y >> 16));
        if (pe) {
          const uint2 p = *reinterpret_cast<const uint2*>(pe + k);
          v[i].x += bf16_to_f32(p.x & 0xFFFF); v[i].y += bf16_to_f32(p.x >> 16);
          v[i].z += bf16_to_f32(p.y & 0xFFFF); v[i].w += bf16_to_f32(p.y >> 16);
        }
      } else {
        v[i] = ld_f4<COH>(h + k);
      }
    }
  }
  if (halted != 0u) return;                       // uniform over the launch; nothing has been written yet
  if (e) {
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int k = (i * NT + t) * 4;
      if (k < d) st_f4<COH>(h + k, v[i].x, v[i].y, v[i].z, v[i].w);
    }
  }
  if (a.ssq_out != nullptr) {
    // deferred RMSNorm: panels of gain * h, and the row's sum of squares in slot 0 of its ssq row
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) ss += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
    ss = block_sum<NT>(ss, red);
    float* sq = a.ssq_out + (size_t)grp * a.n_ssq_out * 16;
    for (int i = t; i < a.n_ssq_out; i += NT) st_f1<COH>(sq + i * 16 + m, (i == 0) ? ss : 0.f);   // [slot][token]
    if (a.sum_out != nullptr) {                   // the consumer's norm is a LayerNorm: the row's sum as well
      float sx = 0.f;
#pragma unroll
      for (int i = 0; i < VPT; ++i) sx += (v[i].x + v[i].y) + (v[i].z + v[i].w);   // zero beyond d
      sx = block_sum<NT>(sx, red);
      float* su = a.sum_out + (size_t)grp * a.n_ssq_out * 16;
      for (int i = t; i < a.n_ssq_out; i += NT) st_f1<COH>(su + i * 16 + m, (i == 0) ? sx : 0.f);
    }
    const int KT = d >> 5;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int k = (i * NT + t) * 4;
      if (k < d) {
        const float4 g = *reinterpret_cast<const float4*>(a.g + k);
        const float o[4] = {v[i].x * g.x, v[i].y * g.y, v[i].z * g.z, v[i].w * g.w};
        xpack_store4<COH>(Xout, KT, a.M, m, k, o);
      }
    }
    return;
  }
  float mean = 0.f;
  if (a.layernorm) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);   // zero beyond d
    mean = block_sum<NT>(s, red) / (float)d;
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    if ((i * NT + t) * 4 < d) {
      const float x0 = v[i].x - mean, x1 = v[i].y - mean, x2 = v[i].z - mean, x3 = v[i].w - mean;
      ss += (x0 * x0 + x1 * x1) + (x2 * x2 + x3 * x3);
    }
  }
  const float var = block_sum<NT>(ss, red) / (float)d;
  const float rstd = 1.0f / sqrtf(var + a.eps);
  const int KT = d >> 5;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int k = (i * NT + t) * 4;
    if (k < d) {
      const float4 g = *reinterpret_cast<const float4*>(a.g + k);
      float o[4] = {(v[i].x - mean) * rstd * g.x, (v[i].y - mean) * rstd * g.y, (v[i].z - mean) * rstd * g.z, (v[i].w - mean) * rstd * g.w};
      if (a.b) {
        const float4 bb = *reinterpret_cast<const float4*>(a.b + k);
        o[0] += bb.x; o[1] += bb.y; o[2] += bb.z; o[3] += bb.w;
      }
      xpack_store4<COH>(Xout, KT, a.M, m, k, o);
    }
  }
}

template <int NT>
__global__ __launch_bounds__(NT) void k_norm(NormArgs a) {
  __shared__ float red[NT / 64 + 1];
  norm_row<NT>(a, blockIdx.x, -1, red, gate_request(a.gate));
}

// One-token activation panel of an fp32 vector (the operand of the GEMVs that give the correction vectors of a
// deferred LayerNorm, W . g and W . b).
__global__ __launch_bounds__(256) void k_vec_panel(const float* __restrict__ v, int d, bf16_t* __restrict__ Xout) {
  const int k = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (k >= d) return;
  float o[4] = {0.f, 0.f, 0.f, 0.f};
  if (v != nullptr) { const float4 x = *reinterpret_cast<const float4*>(v + k); o[0] = x.x; o[1] = x.y; o[2] = x.z; o[3] = x.w; }
  xpack_store4(Xout, d >> 5, 1, 0, k, o);
}

hipError_t launch_vec_panel(const float* v, int d, bf16_t* Xout, hipStream_t s) {
  if (d < 32 || (d & 31) || Xout == nullptr) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_vec_panel, dim3((d / 4 + 255) / 256), dim3(256), 0, s, v, d, Xout);
  return hipGetLastError();
}

hipError_t launch_norm(const NormArgs& a, hipStream_t s) {
  if (a.M < 1 || a.M > 16 || (a.d & 31) || a.d > 8192) return hipErrorInvalidValue;
  // prompt pass: n_groups groups of 16 slots each (then M == 16: two-panel layout)
  if (a.n_groups < 0 || (a.n_groups > 0 && a.M != 16)) return hipErrorInvalidValue;
  const unsigned rows = a.n_groups > 0 ? 16u * (unsigned)a.n_groups : (unsigned)a.M;
  if (a.d <= 2048) hipLaunchKernelGGL(k_norm<256>, dim3(rows), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(k_norm<1024>, dim3(rows), dim3(1024), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// paged attention: M <= 16 queries of one head against cached positions, causal inside the block
// ---------------------------------------------------------------------------------------------

// Workgroup = (query head, range of split_len cached positions), 8 wavefronts; a wavefront takes 32
// positions per step straight from the paged cache into matrix-unit operands:
//   S^T[key][query]  = K[16 keys x d_head] . Q^T      (16x16x32 bf16; K rows are 128-bit loads;
//                                                     q is fp32 split into bf16 hi + lo)
//   O^T[chan][query] = V^T[16 chan x 16 keys] . P^T   (16x16x16 bf16; the S accumulator layout is
//                                                     exactly this instruction's P operand layout,
//                                                     so probabilities never leave registers)
// which is why V is cached transposed ([d_head][token] inside a page).  Soft-max statistics run
// per query across the four 16-lane rows; P is fed as bf16 hi + lo.  The wavefronts merge
// their (max, sum, O) through LDS and write one partial record per (head, range, query).

typedef __attribute__((ext_vector_type(4))) short s16x4;

// One wavefront's share of the attention of one head: 32 cached positions per step.
// QCOH: the queries were written by other workgroups of this launch (hand-off loads); VCOH: so were entries of
// the transposed V blocks, in 128-byte lines that an earlier step of the same launch may have read (a draft loop
// inside one launch), so V tiles are fetched with L2-bypassing loads.
// LO: q and P enter the matrix unit as bf16 hi + lo (fp32 grade); without it as bf16 only (the prompt pass with bf16
// activations: half the matrix instructions).
template <int DH, bool QCOH = false, bool VCOH = false, bool LO = true>
struct AttnWave {
  static constexpr int KS = DH / 32, CT = DH / 16;
  // raw operands of one step: K rows of two 16-position tiles, V^T tiles of the same positions
  struct Raw { u32x4 k[2][KS]; uint2 v[2][CT]; };
  const AttnArgs& a;
  const float* qb;
  int j, g, kvh, total, s1, pt, pshift, qpos;
  size_t kv_head_elems, page_elems;
  bf16x8 qh[KS], ql[KS];
  f32x4 O[CT];
  float m_run, l_run;

  // pos0_ / q_: first position and query rows of this object's token group when they are not the launch's (prompt pass:
  // one workgroup serves two groups of 16 tokens); s1_ < 0: the range ends with the group's own tokens
  __device__ __forceinline__ AttnWave(const AttnArgs& a_, int head, int s1_, int pos0_ = -1, const float* q_ = nullptr) : a(a_) {
    const int lane = threadIdx.x & 63;
    j = lane & 15; g = lane >> 4;
    kvh = head / (a.nq / a.nkv);
    const int pos0 = pos0_ < 0 ? a.pos0 : pos0_;
    qb = q_ != nullptr ? q_ : a.q;
    total = pos0 + a.M; s1 = s1_ < 0 ? total : s1_; pt = a.page_tokens;
    pshift = (pt & (pt - 1)) == 0 ? __builtin_ctz(pt) : -1;     // power-of-two pages: shifts instead of divisions
    qpos = pos0 + j;                                              // last position query j may see
    kv_head_elems = (size_t)pt * DH;                              // one head's K (or V) block in a page
    page_elems = 2 * (size_t)a.nkv * kv_head_elems;
#pragma unroll
    for (int c = 0; c < CT; ++c) O[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    m_run = NEG_BIG; l_run = 0.f;
  }

  // every load of a step is issued at once; none depends on the queries
  __device__ __forceinline__ void issue(Raw& r, const int base) const {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int kb = base + 16 * t;
      if (kb < s1) {
        const int p = min(kb + j, total - 1), lp = pshift >= 0 ? p >> pshift : p / pt, off = p - lp * pt;
        const int pp = a.page_table ? a.page_table[lp] : lp;
        const bf16_t* kp = a.kv_layer + (size_t)pp * page_elems + (size_t)kvh * kv_head_elems + (size_t)off * DH + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) r.k[t][ks] = *reinterpret_cast<const u32x4*>(kp + ks * 32);
      }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int kb = base + 16 * t;
      if (kb < s1) {
        // V^T operand: channel row = lane % 16 of each 16-channel tile, 4 consecutive positions
        const int p0 = kb + 4 * g;
        const int pc = min(p0, (total - 1) & ~3), lp = pshift >= 0 ? pc >> pshift : pc / pt, off = pc - lp * pt;
        const int pp = a.page_table ? a.page_table[lp] : lp;
        const bf16_t* vp = a.kv_layer + (size_t)pp * page_elems + (size_t)(a.nkv + kvh) * kv_head_elems + (size_t)j * pt + off;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
          if (VCOH) {
            const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(vp + (size_t)c * 16 * pt), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r.v[t][c] = make_uint2((uint32_t)u, (uint32_t)(u >> 32));
          } else {
            r.v[t][c] = *reinterpret_cast<const uint2*>(vp + (size_t)c * 16 * pt);
          }
        }
      }
    }
  }

  // query operand: column j holds query min(j, M-1) (surplus columns are never stored)
  __device__ __forceinline__ void load_q(int head) {
    const float* qp = qb + (size_t)min(j, a.M - 1) * a.ldq + head * DH + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const float4 x0 = ld_f4<QCOH>(qp + ks * 32), x1 = ld_f4<QCOH>(qp + ks * 32 + 4);
      const float xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
      union { bf16_t u[8]; bf16x8 v; } h, l;
#pragma unroll
      for (int i = 0; i < 8; ++i) { h.u[i] = f32_to_bf16(xv[i]); l.u[i] = LO ? f32_to_bf16(xv[i] - bf16_to_f32(h.u[i])) : (bf16_t)0; }
      qh[ks] = h.v; ql[ks] = l.v;
    }
  }

  // scores, running soft-max and P.V of one step
  __device__ __forceinline__ void step(const Raw& r, const int base) {
    f32x4 S[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int kb = base + 16 * t;
      S[t] = f32x4{NEG_BIG, NEG_BIG, NEG_BIG, NEG_BIG};
      if (kb < s1) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 kk = as_bf16x8(r.k[t][ks]);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, qh[ks], acc, 0, 0, 0);
          if (LO) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, ql[ks], acc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int pos = kb + 4 * g + v;
          if (pos < s1 && pos <= qpos) S[t][v] = acc[v] * a.scale;
        }
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(S[0][0], S[0][1]), fmaxf(S[0][2], S[0][3])), fmaxf(fmaxf(S[1][0], S[1][1]), fmaxf(S[1][2], S[1][3])));
    mx = row4_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __expf(m_run - m_new);
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float e = (S[t][v] > 0.5f * NEG_BIG) ? __expf(S[t][v] - m_new) : 0.f;   // hardware exp2: a few ulp, far inside the bf16 split of P
        S[t][v] = e;
        sum += e;
      }
    sum = row4_sum(sum);
    l_run = l_run * alpha + sum;
    m_run = m_new;
#pragma unroll
    for (int c = 0; c < CT; ++c) O[c] *= alpha;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int kb = base + 16 * t;
      if (kb < s1) {
        union { bf16_t u[4]; s16x4 v; } ph, pl;
#pragma unroll
        for (int v = 0; v < 4; ++v) { ph.u[v] = f32_to_bf16(S[t][v]); pl.u[v] = LO ? f32_to_bf16(S[t][v] - bf16_to_f32(ph.u[v])) : (bf16_t)0; }
        // positions at or beyond `total` hold stale bytes: zero them (0 * NaN would poison the sum)
        const int p0 = kb + 4 * g;
        uint2 keep;
        keep.x = (p0 < total ? 0x0000FFFFu : 0u) | (p0 + 1 < total ? 0xFFFF0000u : 0u);
        keep.y = (p0 + 2 < total ? 0x0000FFFFu : 0u) | (p0 + 3 < total ? 0xFFFF0000u : 0u);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
          uint2 raw = r.v[t][c];
          raw.x &= keep.x; raw.y &= keep.y;
          union { uint2 u; s16x4 v; } vv; vv.u = raw;
          O[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vv.v, ph.v, O[c], 0, 0, 0);
          if (LO) O[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vv.v, pl.v, O[c], 0, 0, 0);
        }
      }
    }
  }
};

// LDS of one attention work unit of NWV wavefronts.
template <int DH, int NWV>
struct AttnSmem {
  f32x4 o_s[NWV][DH / 16][64];
  float m_s[NWV][16], l_s[NWV][16];
  int s_last;
};

// Work unit (query head, range `split` of split_len cached positions) run by NWV wavefronts; the last range of
// a head to finish merges all of the head's records and writes the O-projection panels.
// `hook` runs once before anything that other workgroups of the launch may still be writing is touched (the queries,
// cache entries at or beyond `safe_end`): a wavefront whose first 32 positions lie below safe_end requests them
// before the hook, so those loads are in flight while the hook waits.  The workgroup that merges the head also
// zeroes `reset_word` (the counter the hook waited on), if given.
template <int DH, int NWV, bool COH = false, bool VCOH = false, bool QCOH = false, typename Hook = NoHook>
__device__ __forceinline__ void attn_range(const AttnArgs& a, const int head, const int split, AttnSmem<DH, NWV>& sm,
                                           const uint32_t halted, const Hook hook = Hook(), const int safe_end = 0x7fffff00,
                                           int* reset_word = nullptr) {
  constexpr int CT = DH / 16, WKEYS = 32;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int total = a.pos0 + a.M;
  const int s0 = split * a.split_len, s1 = min(s0 + a.split_len, total);
  AttnWave<DH, QCOH, VCOH> aw(a, head, s1);      // (a persistent kernel gives the queries a fresh address per layer)
  typename AttnWave<DH, QCOH, VCOH>::Raw r0, r1;
  // the first step's cache loads go out ahead of the q loads; later steps' loads are in flight during
  // the arithmetic of the step before
  constexpr int STEP = NWV * WKEYS;
  int base = s0 + w * WKEYS;
  const bool early = base + WKEYS <= safe_end;
  if (base < s1 && early) aw.issue(r0, base);
  hook();
  if (base < s1 && !early) aw.issue(r0, base);
  aw.load_q(head);
  if (halted != 0u) return;                       // uniform over the launch; nothing has been written yet
  while (base < s1) {
    if (base + STEP < s1) aw.issue(r1, base + STEP);
    aw.step(r0, base);
    base += STEP;
    if (base >= s1) break;
    if (base + STEP < s1) aw.issue(r0, base + STEP);
    aw.step(r1, base);
    base += STEP;
  }

  // merge the wavefronts (fixed order), then one record per query: o[DH], max, sum
  __syncthreads();                                // a previous unit of this workgroup has left the buffers
#pragma unroll
  for (int c = 0; c < CT; ++c) sm.o_s[w][c][lane] = aw.O[c];
  if (g == 0) { sm.m_s[w][j] = aw.m_run; sm.l_s[w][j] = aw.l_run; }
  __syncthreads();
  float mm = sm.m_s[0][j];
#pragma unroll
  for (int ww = 1; ww < NWV; ++ww) mm = fmaxf(mm, sm.m_s[ww][j]);
  float f[NWV], ll = 0.f;
#pragma unroll
  for (int ww = 0; ww < NWV; ++ww) { f[ww] = expf(sm.m_s[ww][j] - mm); ll += sm.l_s[ww][j] * f[ww]; }
  if (j < a.M) {
    float* rec = a.part + (((size_t)head * a.n_splits + split) * 16 + j) * (DH + 2);
    // channel tiles are dealt to the wavefronts: tiles w, w + NWV, ..
#pragma unroll
    for (int ci = 0; ci < (CT + NWV - 1) / NWV; ++ci) {
      const int c = w + ci * NWV;
      if (c < CT) {
        f32x4 o = sm.o_s[0][c][lane] * f[0];
#pragma unroll
        for (int ww = 1; ww < NWV; ++ww) o += sm.o_s[ww][c][lane] * f[ww];
        st_agent2(rec + c * 16 + 4 * g, o[0], o[1]);
        st_agent2(rec + c * 16 + 4 * g + 2, o[2], o[3]);
      }
    }
    if (w == 0 && g == 0) st_agent2(rec + DH, mm, ll);
  }
  // the last range of this head to finish merges all ranges (in range order) into the panels that
  // feed the O-projection
  if (!last_arrival(a.counters + head, a.n_splits, &sm.s_last)) return;
  if (reset_word != nullptr && threadIdx.x == 0) __hip_atomic_store(reset_word, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  // 8 channels per thread: DH / 8 threads per query, so that all 16 queries of a block are merged in one
  // pass (a second pass would put a second round trip to the records behind the first)
  constexpr int TPQ = DH / 8;
  const int tq = threadIdx.x % TPQ;
  for (int qm = threadIdx.x / TPQ; qm < a.M; qm += NWV * 64 / TPQ) {
    const float* rbase = a.part + (((size_t)head * a.n_splits) * 16 + qm) * (DH + 2);
    const size_t stride = (size_t)16 * (DH + 2);
    // running (max, sum, o) over the ranges in range order; eight ranges' records are fetched at a
    // time so that their round trips overlap
    float mx = NEG_BIG, L = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int sp0 = 0; sp0 < a.n_splits; sp0 += 8) {
      float2 ml[8], v[8][4];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (sp0 + i < a.n_splits) {
          const float* rc = rbase + (size_t)(sp0 + i) * stride;
          ml[i] = ld_agent2(rc + DH);
#pragma unroll
          for (int c = 0; c < 4; ++c) v[i][c] = ld_agent2(rc + 8 * tq + 2 * c);
        }
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (sp0 + i < a.n_splits) {
          const float m_new = fmaxf(mx, ml[i].x);
          const float f_old = expf(mx - m_new), f_new = expf(ml[i].x - m_new);
          L = L * f_old + ml[i].y * f_new;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            o[2 * c] = o[2 * c] * f_old + v[i][c].x * f_new;
            o[2 * c + 1] = o[2 * c + 1] * f_old + v[i][c].y * f_new;
          }
          mx = m_new;
        }
    }
    const float inv = 1.0f / L;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] *= inv;
    xpack_store4<COH>(a.Xout, (a.nq * DH) >> 5, a.M, qm, head * DH + 8 * tq, o);
    xpack_store4<COH>(a.Xout, (a.nq * DH) >> 5, a.M, qm, head * DH + 8 * tq + 4, o + 4);
  }
}

template <int DH>
__global__ __launch_bounds__(512) void k_attn_partial(AttnArgs a) {
  __shared__ AttnSmem<DH, 8> sm;                  // eight wavefronts: a range of 256 positions is one step each (measured
  attn_range<DH, 8>(a, blockIdx.x, blockIdx.y, sm, gate_request(a.gate));   // 1.3 % of a 13B verification block against four)
}

// Short contexts: one workgroup of eight wavefronts takes a whole head (256 positions per step, the
// loads of step i + 1 in flight during the arithmetic of step i), merges its wavefronts through LDS
// and writes the O-projection panels itself: no partial records, no hand-off between workgroups.
template <int DH>
__device__ __forceinline__ void attn_whole_head(const AttnArgs& a, const int head, const uint32_t halted = 0u) {
  constexpr int CT = DH / 16, NWV = 8, WKEYS = 32, STEP = NWV * WKEYS;
  __shared__ f32x4 o_s[NWV][CT][64];
  __shared__ float m_s[NWV][16], l_s[NWV][16];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int total = a.pos0 + a.M;
  AttnWave<DH> aw(a, head, total);
  typename AttnWave<DH>::Raw r0, r1;
  int base = w * WKEYS;
  if (base < total) aw.issue(r0, base);
  aw.load_q(head);
  if (halted != 0u) return;                       // uniform over the launch; nothing has been written yet
  while (base < total) {
    if (base + STEP < total) aw.issue(r1, base + STEP);
    aw.step(r0, base);
    base += STEP;
    if (base >= total) break;
    if (base + STEP < total) aw.issue(r0, base + STEP);
    aw.step(r1, base);
    base += STEP;
  }
#pragma unroll
  for (int c = 0; c < CT; ++c) o_s[w][c][lane] = aw.O[c];
  if (g == 0) { m_s[w][j] = aw.m_run; l_s[w][j] = aw.l_run; }
  __syncthreads();
  if (w >= CT || j >= a.M) return;                               // wavefront w finishes channel tile w
  float mm = m_s[0][j];
#pragma unroll
  for (int ww = 1; ww < NWV; ++ww) mm = fmaxf(mm, m_s[ww][j]);
  float ll = 0.f;
  f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ww = 0; ww < NWV; ++ww) {                             // fixed order: deterministic
    const float f = expf(m_s[ww][j] - mm);
    ll += l_s[ww][j] * f;
    o += o_s[ww][w][lane] * f;
  }
  const float inv = 1.0f / ll;
  const float out4[4] = {o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
  xpack_store4(a.Xout, (a.nq * DH) >> 5, a.M, j, head * DH + w * 16 + 4 * g, out4);
}

template <int DH>
__global__ __launch_bounds__(512) void k_attn_head(AttnArgs a) {
  attn_whole_head<DH>(a, blockIdx.x, gate_request(a.gate));
}

// Prompt pass: workgroup = (query head, two consecutive groups of 16 prompt tokens).  Group r sits at positions
// pos0 + 16 r .. and sees everything up to its own tokens.  The eight wavefronts share the cached positions (32 per
// wavefront and step); every K and V tile a wavefront fetches serves the queries of both groups (half the cache reads
// and half the workgroups of one group per workgroup: the kernel waits on those reads), each group with its own
// running soft-max.  The groups are merged across the wavefronts one after the other through one LDS buffer.  The
// longest ranges are scheduled first.
constexpr int ATTN_MG = 2;
template <int DH, bool LO>
__global__ __launch_bounds__(512) void k_attn_groups(AttnArgs a, int n_groups, size_t x_stride) {
  constexpr int CT = DH / 16, NWV = 8, WKEYS = 32, STEP = NWV * WKEYS, NG = ATTN_MG;
  __shared__ f32x4 o_s[NWV][CT][64];
  __shared__ float m_s[NWV][16], l_s[NWV][16];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int head = blockIdx.x;
  const int nb = (n_groups + NG - 1) / NG;
  const int r0g = (nb - 1 - (int)blockIdx.y) * NG;                // first group of this workgroup
  const int ng = min(NG, n_groups - r0g);
  auto grp = [&](int i) { return r0g + min(i, ng - 1); };          // a surplus slot repeats the last group and stores nothing
  auto wave_of = [&](int i) { return AttnWave<DH, false, false, LO>(a, head, -1, a.pos0 + 16 * grp(i), a.q + (size_t)grp(i) * 16 * a.ldq); };
  AttnWave<DH, false, false, LO> aw[NG] = {wave_of(0), wave_of(1)};
  static_assert(NG == 2, "the initialiser above lists two groups");
  const int total = aw[NG - 1].total;                              // the longest range: its object issues the loads
  // one set of raw operands per wavefront (two would not fit beside the state of two groups); the other wavefront of
  // the SIMD covers the wait (re-issuing the K loads between the two halves of a step measured slower)
  typename AttnWave<DH, false, false, LO>::Raw ra;
  int base = w * WKEYS;
  if (base < total) aw[NG - 1].issue(ra, base);
#pragma unroll
  for (int i = 0; i < NG; ++i) aw[i].load_q(head);
  while (base < total) {
#pragma unroll
    for (int i = 0; i < NG; ++i)
      if (base < aw[i].total) aw[i].step(ra, base);
    base += STEP;
    if (base < total) aw[NG - 1].issue(ra, base);
  }
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    if (i > 0) __syncthreads();                                    // the merge of the group before has read the buffer
#pragma unroll
    for (int c = 0; c < CT; ++c) o_s[w][c][lane] = aw[i].O[c];
    if (g == 0) { m_s[w][j] = aw[i].m_run; l_s[w][j] = aw[i].l_run; }
    __syncthreads();
    if (i < ng && w < CT) {                                        // wavefront w finishes channel tile w
      float mm = m_s[0][j];
#pragma unroll
      for (int ww = 1; ww < NWV; ++ww) mm = fmaxf(mm, m_s[ww][j]);
      float ll = 0.f;
      f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ww = 0; ww < NWV; ++ww) {                           // fixed order: deterministic
        const float f = expf(m_s[ww][j] - mm);
        ll += l_s[ww][j] * f;
        o += o_s[ww][w][lane] * f;
      }
      const float inv = 1.0f / ll;
      const float out4[4] = {o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
      xpack_store4(a.Xout + (size_t)(r0g + i) * x_stride, (a.nq * DH) >> 5, a.M, j, head * DH + w * 16 + 4 * g, out4);
    }
  }
}

constexpr int ATTN_HEAD_MAX_CTX = 256;    // positions up to which the whole-head kernel is used (one step per wavefront);
                                          // beyond it the arithmetic of a head is worth spreading over several compute units

// Positions per attention workgroup: short ranges give many workgroups but one hand-off record per
// range and query; measured best on MI355X at the 13B-class shape: 128 up to ~768 positions, then
// about total / 4 .. total / 8.
int attn_split_len(int total) {
  if (total <= 768) return ATTN_SPLIT_LEN;
  if (total <= 1536) return 2 * ATTN_SPLIT_LEN;
  if (total <= 3072) return 4 * ATTN_SPLIT_LEN;
  return 8 * ATTN_SPLIT_LEN;
}

hipError_t launch_attn(const AttnArgs& a, hipStream_t s) {
  if (a.M < 1 || a.M > 16 || a.n_splits < 1 || a.counters == nullptr) return hipErrorInvalidValue;
  if (a.pos0 + a.M <= ATTN_HEAD_MAX_CTX) {
    if (a.dh == 128) hipLaunchKernelGGL(k_attn_head<128>, dim3(a.nq), dim3(512), 0, s, a);
    else if (a.dh == 64) hipLaunchKernelGGL(k_attn_head<64>, dim3(a.nq), dim3(512), 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  const dim3 g1(a.nq, a.n_splits);
  if (a.dh == 128) hipLaunchKernelGGL(k_attn_partial<128>, g1, dim3(512), 0, s, a);
  else if (a.dh == 64) hipLaunchKernelGGL(k_attn_partial<64>, g1, dim3(512), 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_attn_groups(const AttnArgs& a, int n_groups, size_t x_stride, bool bf16_operands, hipStream_t s) {
  if (a.M != 16 || n_groups < 1 || n_groups > 65535) return hipErrorInvalidValue;
  const dim3 g1(a.nq, (n_groups + ATTN_MG - 1) / ATTN_MG);
  if (a.dh == 128) {
    if (bf16_operands) hipLaunchKernelGGL((k_attn_groups<128, false>), g1, dim3(512), 0, s, a, n_groups, x_stride);
    else hipLaunchKernelGGL((k_attn_groups<128, true>), g1, dim3(512), 0, s, a, n_groups, x_stride);
  } else if (a.dh == 64) {
    if (bf16_operands) hipLaunchKernelGGL((k_attn_groups<64, false>), g1, dim3(512), 0, s, a, n_groups, x_stride);
    else hipLaunchKernelGGL((k_attn_groups<64, true>), g1, dim3(512), 0, s, a, n_groups, x_stride);
  } else return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Eq. 2 in one launch: soft-max top-10, entropy, arg-max -> classifier -> halt decision
// ---------------------------------------------------------------------------------------------

struct ClfOut {  // mirrors disco_clf_out
  int32_t token; float feats[12]; float score; uint32_t halt; uint32_t executed;
};

constexpr int FEAT_NT = 1024;

// One workgroup, the whole logit vector in registers (V4 float4 per thread, one round of 128-bit
// loads).  Arg-max, soft-max sums and entropy are DPP wave reductions merged across the 16
// wavefronts in a fixed order.  Top-10: every wavefront finds the ten largest of the values its
// lanes hold by ten cross-lane arg-max rounds, and one wavefront picks the ten largest of those 160.
constexpr int CM_NT = 512;     // threads per slice inside the persistent draft loop (its workgroups have 512 threads): 2048 logits
constexpr int CM_MULTI_NT = 256;   // threads per slice of the many-workgroup launch: 1024 logits (32 workgroups at vocab 32000, 64
                                   // records at most: measured 2 us per draft step better than slices of 2048)
constexpr int CM_REC = 16;     // floats per record

// Order-preserving map float -> uint32 (larger float <=> larger key; -inf maps above key 0, which marks
// a dropped slot) and back.
__device__ __forceinline__ uint32_t f32_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_f32(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}
// Wavefront maximum of unsigned keys: the cross-lane moves fold into the max instructions (one DPP
// instruction per step; 0 is the identity, so lanes a step does not reach keep their value).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_max_u32(uint32_t v) {
  const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
  return v > o ? v : o;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = dpp_max_u32<DPP_QUAD_XOR1, 0xF>(v);
  v = dpp_max_u32<DPP_QUAD_XOR2, 0xF>(v);
  v = dpp_max_u32<DPP_ROW_HALF_MIRROR, 0xF>(v);
  v = dpp_max_u32<DPP_ROW_MIRROR, 0xF>(v);
  v = dpp_max_u32<DPP_ROW_BCAST15, 0xA>(v);
  v = dpp_max_u32<DPP_ROW_BCAST31, 0xC>(v);
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// The ten largest of the N values per lane held by one wavefront, descending, written by lane 0 to
// out10: ten rounds of a cross-lane maximum over order-preserving integer keys; the first lane that
// holds the maximum drops one instance of it (branch-free).  No LDS traffic and no workgroup barrier
// inside; c is consumed.
template <int N>
__device__ __forceinline__ void wave_top10(float (&c)[N], float* out10) {
  const int lane = threadIdx.x & 63;
  uint32_t k[N];
#pragma unroll
  for (int e = 0; e < N; ++e) k[e] = f32_key(c[e]);
#pragma unroll 1
  for (int rnd = 0; rnd < 10; ++rnd) {
    uint32_t cur = k[0];
#pragma unroll
    for (int e = 1; e < N; ++e) cur = cur > k[e] ? cur : k[e];
    const uint32_t w = wave_max_u32(cur);
    if (lane == 0) out10[rnd] = key_f32(w);
    const unsigned long long owners = __ballot(cur == w);
    bool drop = owners != 0ull && lane == __builtin_ctzll(owners);
#pragma unroll
    for (int e = 0; e < N; ++e) {
      const bool hit = drop && k[e] == w;
      k[e] = hit ? 0u : k[e];
      drop = drop && !hit;
    }
  }
}

// Ten largest of a workgroup's values: every wavefront's ten, then one thread per candidate ranks it:
// a candidate's rank is the number of candidates that beat it (larger, or equal with a lower slot), a
// permutation of 0 .. n-1, and ranks below ten are the answer in order.  No dependent cross-lane chain.
template <int NT, int N>
__device__ __forceinline__ void block_top10(float (&c)[N], float (*wtop)[10], float* top_s) {
  const int wv = threadIdx.x >> 6;
  wave_top10<N>(c, wtop[wv]);
  __syncthreads();
  constexpr int NC = (NT / 64) * 10;
  if ((int)threadIdx.x < NC) {
    const int me = threadIdx.x;
    const float* cand = &wtop[0][0];
    const float mine = cand[me];
    float o[NC];
#pragma unroll
    for (int j = 0; j < NC; ++j) o[j] = cand[j];          // all reads in flight at once (broadcasts)
    int rank = 0;
#pragma unroll
    for (int j = 0; j < NC; ++j) rank += (o[j] > mine || (o[j] == mine && j < me)) ? 1 : 0;
    if (rank < 10) top_s[rank] = mine;
  }
  __syncthreads();
}

template <int V4>
__global__ __launch_bounds__(FEAT_NT) void k_classify(ClassifyArgs a) {
  ClfOut* out = reinterpret_cast<ClfOut*>(a.out);
  if (a.gate != nullptr && *a.gate != 0u) {
    if (threadIdx.x == 0) out->executed = 0u;
    return;
  }
  __shared__ float sv[FEAT_NT / 64 + 1];
  __shared__ int si[FEAT_NT / 64 + 1];
  __shared__ float wtop[FEAT_NT / 64][10];
  __shared__ float top_s[10];
  __shared__ float feat_s[12];
  const int t = threadIdx.x, V = a.vocab, lane = t & 63, wv = t >> 6;
  const float* x = a.logits;

  float4 r[V4];
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int idx = (i * FEAT_NT + t) * 4;
    if (idx + 3 < V) {
      r[i] = *reinterpret_cast<const float4*>(x + idx);
    } else {
      r[i].x = idx < V ? x[idx] : -INFINITY;
      r[i].y = idx + 1 < V ? x[idx + 1] : -INFINITY;
      r[i].z = idx + 2 < V ? x[idx + 2] : -INFINITY;
      r[i].w = -INFINITY;
    }
  }

  // maximum and arg-max (lowest index on ties); `mine` is this thread's own maximum
  VI mine; mine.v = -INFINITY; mine.i = 0x7fffffff;
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int idx = (i * FEAT_NT + t) * 4;
    VI y;
    y.v = r[i].x; y.i = idx; mine = vi_best(mine, y);
    y.v = r[i].y; y.i = idx + 1; mine = vi_best(mine, y);
    y.v = r[i].z; y.i = idx + 2; mine = vi_best(mine, y);
    y.v = r[i].w; y.i = idx + 3; mine = vi_best(mine, y);
  }
  VI best = block_argmax<FEAT_NT>(mine, sv, si);
  int force = -1;
  if (a.force_token) { force = *a.force_token; if (force >= V) force = -1; }
  if (force >= 0) {
    const float forced_val = best.v + 4.0f;
    best.v = forced_val; best.i = force;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int idx = (i * FEAT_NT + t) * 4;
      if (force == idx) r[i].x = forced_val;
      if (force == idx + 1) r[i].y = forced_val;
      if (force == idx + 2) r[i].z = forced_val;
      if (force == idx + 3) r[i].w = forced_val;
    }
    if ((force >> 2) % FEAT_NT == t) { mine.v = forced_val; mine.i = force; a.logits[force] = forced_val; }
  }
  const float mx = best.v;

  // S = sum e^(x - max), T = sum e^(x - max) (x - max)
  float S = 0.f, T = 0.f;
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const float d0 = r[i].x - mx, d1 = r[i].y - mx, d2 = r[i].z - mx, d3 = r[i].w - mx;
    const float e0 = expf(d0), e1 = expf(d1), e2 = expf(d2), e3 = expf(d3);
    S += (e0 + e1) + (e2 + e3);
    // e^(-inf) * (-inf) would be NaN: padded slots contribute nothing
    T += (e0 > 0.f ? e0 * d0 : 0.f) + (e1 > 0.f ? e1 * d1 : 0.f) + (e2 > 0.f ? e2 * d2 : 0.f) + (e3 > 0.f ? e3 * d3 : 0.f);
  }
  S = block_sum<FEAT_NT>(S, sv);
  T = block_sum<FEAT_NT>(T, sv);

  // ten largest logits: every wavefront's ten by cross-lane maximum rounds over the values its lanes
  // hold (the first lane that holds the maximum drops one instance; the row is not needed afterwards),
  // then wavefront 0 picks from the 160 candidates
  {
#pragma unroll 1
    for (int rnd = 0; rnd < 10; ++rnd) {
      float cur = -INFINITY;
#pragma unroll
      for (int i = 0; i < V4; ++i) cur = fmaxf(cur, fmaxf(fmaxf(r[i].x, r[i].y), fmaxf(r[i].z, r[i].w)));
      const float wn = wave_max(cur);
      if (lane == 0) wtop[wv][rnd] = wn;
      const unsigned long long owners = __ballot(cur == wn);
      if (owners != 0ull && lane == __builtin_ctzll(owners)) {
        bool done = false;
#pragma unroll
        for (int i = 0; i < V4; ++i) {
          if (!done && r[i].x == wn) { r[i].x = -INFINITY; done = true; }
          if (!done && r[i].y == wn) { r[i].y = -INFINITY; done = true; }
          if (!done && r[i].z == wn) { r[i].z = -INFINITY; done = true; }
          if (!done && r[i].w == wn) { r[i].w = -INFINITY; done = true; }
        }
      }
    }
    __syncthreads();
    if (wv == 0) {
      float c3[3];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const int ci = lane + 64 * k;
        c3[k] = ci < (FEAT_NT / 64) * 10 ? wtop[ci / 10][ci % 10] : -INFINITY;
      }
      wave_top10<3>(c3, top_s);
    }
  }
  __syncthreads();
  if (t < 10) feat_s[t] = (top_s[t] == -INFINITY) ? 0.f : expf(top_s[t] - mx) / S;
  if (t == 10) feat_s[10] = logf(S) - T / S;
  if (t == 11) feat_s[11] = a.pos_feature;
  __syncthreads();

  // classifier: hidden unit per thread
  float contrib = 0.f;
  if (a.clf_params && t < a.hidden) {
    const float* W1 = a.clf_params + t * 12;
    float acc = a.clf_params[a.hidden * 12 + t];
#pragma unroll
    for (int i = 0; i < 12; ++i) acc += W1[i] * feat_s[i];
    contrib = fmaxf(acc, 0.f) * a.clf_params[a.hidden * 13 + t];
  }
  const float z = block_sum<FEAT_NT>(contrib, sv);
  if (t == 0) {
    float score = __builtin_nanf("");
    uint32_t halt = a.force_halt ? 1u : 0u;
    if (a.clf_params) {
      score = 1.0f / (1.0f + expf(-(z + a.clf_params[a.hidden * 14])));
      if (score < a.tau) halt = 1u;
    }
    // reference lookahead: a token that differs from the known continuation ends the block and is
    // not part of it (bit 1 of halt)
    bool mismatch = false;
    if (a.ref_token) { const int ref = *a.ref_token; mismatch = ref >= 0 && best.i != ref; }
    if (mismatch) halt = 3u;
    // perplexity rule (App. F's rule-based baseline): the block's draft tokens so far have perplexity
    // exp(-(1/j) sum ln p_i), p_i the draft's probability of its own token (the largest one); above the
    // threshold this token is the block's last.  The running sum sits in the word after sl_count.
    if (a.ppl_threshold > 0.f && a.sl_count) {
      float* nll = reinterpret_cast<float*>(a.sl_count + 1);
      const float sum = *nll - logf(feat_s[0]);
      *nll = sum;
      score = expf(sum / (float)(*a.sl_count + 1));
      if (score > a.ppl_threshold) halt |= 1u;
    }
    out->token = best.i;
#pragma unroll
    for (int i = 0; i < 12; ++i) out->feats[i] = feat_s[i];
    out->score = score; out->halt = halt; out->executed = 1u;
    if (!mismatch) {
      if (a.token_next) *a.token_next = best.i;
      if (a.block_slot) *a.block_slot = best.i;
      if (a.sl_count) *a.sl_count += 1;
    }
    if (a.gate && halt) *a.gate = 1u;
  }
}

// Classifier coefficients of one thread (hidden unit threadIdx.x), fetched early by the caller.
struct ClfCoef { float w1[12]; float b1, w2, b2; };

// Last stage of the feature / classifier computation, run by ONE workgroup of NT threads over nb
// records {max, arg-max, S, T relative to the record's max, its ten largest values} (16 floats each,
// written with agent-scope stores by the workgroups that reduced the logits): merged statistics in
// record order, the ten largest of the nb * 10 candidates (CPT per thread), the forced logit in closed
// form, features, classifier, halt decision and the loop's bookkeeping words.
template <int NT, int CPT>
__device__ __forceinline__ int classify_merge_finish(const ClassifyArgs& a, const float* recs, const int nb, const int force,
                                                      const float xf, const ClfCoef& k, float* sv, int* si, float (*wtop)[10],
                                                      float* top_s, float* feat_s) {
  ClfOut* out = reinterpret_cast<ClfOut*>(a.out);
  const int t = threadIdx.x;
  VI bm; bm.v = -INFINITY; bm.i = 0x7fffffff;
  float Sb = 0.f, Tb = 0.f, mb = 0.f;
  if (t < nb) {
    const float2 p0 = ld_agent2(recs + (size_t)t * CM_REC), p1 = ld_agent2(recs + (size_t)t * CM_REC + 2);
    bm.v = p0.x; bm.i = __float_as_int(p0.y); mb = p0.x; Sb = p1.x; Tb = p1.y;
  }
  VI gbest = block_argmax<NT>(bm, sv, si);
  float Sg = 0.f, Tg = 0.f;
  if (t < nb) {
    const float d = mb - gbest.v, f = expf(d);
    Sg = Sb * f; Tg = f > 0.f ? f * (Tb + d * Sb) : 0.f;
  }
  Sg = block_sum<NT>(Sg, sv);
  Tg = block_sum<NT>(Tg, sv);
  // ten largest of the nb * 10 candidates (up to 3 per thread)
  float cc[CPT];
#pragma unroll
  for (int q = 0; q < CPT; ++q) {
    const int ci = t + q * NT;                               // candidate ci = record ci / 10, slot ci % 10
    cc[q] = -INFINITY;
    if (ci < nb * 10) {
      const int rb = ci / 10, sl = ci % 10;
      const float2 p = ld_agent2(recs + (size_t)rb * CM_REC + 4 + (sl & ~1));
      cc[q] = (sl & 1) ? p.y : p.x;
    }
  }
  block_top10<NT, CPT>(cc, wtop, top_s);
  float mx = gbest.v;
  if (force >= 0) {
    // raise logit[force] from x_f to M + 4: shift every term to the new maximum, take the old
    // contribution of x_f out and put the new one (e^0 = 1, with (x - max) = 0) in
    const float mnew = gbest.v + 4.0f;
    const float sh = expf(-4.0f), ef = expf(xf - mnew);
    Tg = sh * (Tg - 4.0f * Sg) - (ef > 0.f ? ef * (xf - mnew) : 0.f);
    Sg = sh * Sg - ef + 1.0f;
    if (t == 0) {
      // new top ten: M + 4 first, then the old ones without one instance of x_f (or without the last)
      float old[10];
      for (int i = 0; i < 10; ++i) old[i] = top_s[i];
      int drop = 9;
      for (int i = 9; i >= 0; --i) if (old[i] == xf) drop = i;
      top_s[0] = mnew;
      for (int i = 0, o = 1; i < 10 && o < 10; ++i) if (i != drop) top_s[o++] = old[i];
      st_f1<true>(a.logits + force, mnew);
    }
    mx = mnew; gbest.v = mnew; gbest.i = force;
    __syncthreads();
  }
  if (t < 10) feat_s[t] = (top_s[t] == -INFINITY) ? 0.f : expf(top_s[t] - mx) / Sg;
  if (t == 10) feat_s[10] = logf(Sg) - Tg / Sg;
  if (t == 11) feat_s[11] = a.pos_feature;
  __syncthreads();
  float contrib = 0.f;
  if (a.clf_params && t < a.hidden) {
    float acc = k.b1;
#pragma unroll
    for (int i = 0; i < 12; ++i) acc += k.w1[i] * feat_s[i];
    contrib = fmaxf(acc, 0.f) * k.w2;
  }
  const float z = block_sum<NT>(contrib, sv);
  if (t == 0) {
    float score = __builtin_nanf("");
    uint32_t halt = a.force_halt ? 1u : 0u;
    if (a.clf_params) {
      score = 1.0f / (1.0f + expf(-(z + k.b2)));
      if (score < a.tau) halt = 1u;
    }
    // reference lookahead: a token that differs from the known continuation ends the block and is
    // not part of it (bit 1 of halt)
    bool mismatch = false;
    if (a.ref_token) { const int ref = *a.ref_token; mismatch = ref >= 0 && gbest.i != ref; }
    if (mismatch) halt = 3u;
    // perplexity rule (App. F's rule-based baseline): the block's draft tokens so far have perplexity
    // exp(-(1/j) sum ln p_i), p_i the draft's probability of its own token (the largest one); above the
    // threshold this token is the block's last.  The running sum sits in the word after sl_count.
    // (the loop's words may have been written by another workgroup of the same launch: hand-off accesses)
    const int sl_before = a.sl_count ? __hip_atomic_load(a.sl_count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
    if (a.ppl_threshold > 0.f && a.sl_count) {
      float* nll = reinterpret_cast<float*>(a.sl_count + 1);
      const float sum = ld_f1<true>(nll) - logf(feat_s[0]);
      st_f1<true>(nll, sum);
      score = expf(sum / (float)(sl_before + 1));
      if (score > a.ppl_threshold) halt |= 1u;
    }
    out->token = gbest.i;
#pragma unroll
    for (int i = 0; i < 12; ++i) out->feats[i] = feat_s[i];
    out->score = score; out->halt = halt; out->executed = 1u;
    if (!mismatch) {
      if (a.token_next) *a.token_next = gbest.i;
      if (a.block_slot) *a.block_slot = gbest.i;
      if (a.sl_count) __hip_atomic_store(a.sl_count, sl_before + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (a.gate && halt) __hip_atomic_store(a.gate, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return gbest.i;
}

// The same computation spread over ceil(V / (4 NT)) workgroups (used when the caller gives scratch
// memory).  Each workgroup reduces its slice of the logits (4 per thread) to a record {max, arg-max, S, T relative to its own
// max, its ten largest values}; the last workgroup to finish (ticket, no waiting) merges the
// records in index order: S = sum S_b e^(m_b - M), T = sum e^(m_b - M) (T_b + (m_b - M) S_b), the ten
// largest of the records' candidates (ten per record), then features, classifier and halt decision.  Forcing a token
// to max + 4 is applied to the merged sums in closed form.
// b = index of this workgroup's slice of NT * 4 logits, nb = number of slices.  Returns the arg-max token in
// every thread of the workgroup that finished the computation (the last to arrive), -1 in all others.
// COH: the logits were written by other workgroups of the same launch.
template <int NT, bool COH = false>
__device__ __forceinline__ int classify_unit(const ClassifyArgs& a, const int b, const int nb, const uint32_t halted) {
  ClfOut* out = reinterpret_cast<ClfOut*>(a.out);
  __shared__ float sv[NT / 64 + 1];
  __shared__ int si[NT / 64 + 1];
  __shared__ float top_s[10];
  __shared__ float wtop[NT / 64][10];
  __shared__ float feat_s[12];
  __shared__ int s_last;
  const int t = threadIdx.x, V = a.vocab;
  const float* x = a.logits;
  float* rec = a.scratch + 64 + (size_t)b * CM_REC;          // scratch[0] is the ticket counter
  const int idx = (b * NT + t) * 4;
  float r4[4];
  if (idx + 3 < V) {
    const float4 v = ld_f4<COH>(x + idx);
    r4[0] = v.x; r4[1] = v.y; r4[2] = v.z; r4[3] = v.w;
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) r4[e] = idx + e < V ? ld_f1<COH>(x + idx + e) : -INFINITY;
  }
  // operands of the final stage that depend on no reduction are fetched now, so that the merging
  // workgroup does not pay their round trips one after another at the end
  int force = -1;
  float xf = 0.f;
  if (a.force_token) { force = *a.force_token; if (force >= V) force = -1; }
  if (force >= 0) xf = ld_f1<COH>(x + force);
  float w1[12], cb1 = 0.f, cw2 = 0.f, cb2 = 0.f;
#pragma unroll
  for (int i = 0; i < 12; ++i) w1[i] = 0.f;
  if (a.clf_params) {
    cb2 = a.clf_params[a.hidden * 14];
    if (t < a.hidden) {
#pragma unroll
      for (int i = 0; i < 12; ++i) w1[i] = a.clf_params[t * 12 + i];
      cb1 = a.clf_params[a.hidden * 12 + t];
      cw2 = a.clf_params[a.hidden * 13 + t];
    }
  }
  if (halted != 0u) {                             // uniform over the launch; the loads above are dropped
    if (threadIdx.x == 0 && b == 0) out->executed = 0u;
    return -1;
  }
  VI mine; mine.v = -INFINITY; mine.i = 0x7fffffff;
#pragma unroll
  for (int e = 0; e < 4; ++e) { VI y; y.v = r4[e]; y.i = idx + e; mine = vi_best(mine, y); }
  const VI best = block_argmax<NT>(mine, sv, si);
  float S = 0.f, T = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float d = r4[e] - best.v, ex = expf(d);
    S += ex; T += ex > 0.f ? ex * d : 0.f;
  }
  S = block_sum<NT>(S, sv);
  T = block_sum<NT>(T, sv);
  // this workgroup's ten largest values
  {
    float c4[4] = {r4[0], r4[1], r4[2], r4[3]};
    block_top10<NT, 4>(c4, wtop, top_s);
  }
  if (t == 0) { st_agent2(rec, best.v, __int_as_float(best.i)); st_agent2(rec + 2, S, T); }
  if (t >= 2 && t < 7) st_agent2(rec + 2 * t, top_s[2 * t - 4], top_s[2 * t - 3]);
  if (!last_arrival(reinterpret_cast<int*>(a.scratch), nb, &s_last)) return -1;

  ClfCoef k;
#pragma unroll
  for (int i = 0; i < 12; ++i) k.w1[i] = w1[i];
  k.b1 = cb1; k.w2 = cw2; k.b2 = cb2;
  // at most 64 slices (65536 logits at NT = 256): 640 candidates
  constexpr int CPT = (640 * 256 / NT + NT - 1) / NT;
  return classify_merge_finish<NT, CPT>(a, a.scratch + 64, nb, force, xf, k, sv, si, wtop, top_s, feat_s);
}

__global__ __launch_bounds__(CM_MULTI_NT) void k_classify_multi(ClassifyArgs a) {
  classify_unit<CM_MULTI_NT>(a, blockIdx.x, gridDim.x, gate_request(const_cast<const uint32_t*>(a.gate)));
}

hipError_t launch_classify(const ClassifyArgs& a, hipStream_t s) {
  if (a.vocab < 1 || a.vocab > 65536) return hipErrorInvalidValue;
  if (a.scratch != nullptr && a.vocab >= 4096) {
    hipLaunchKernelGGL(k_classify_multi, dim3((a.vocab + 4 * CM_MULTI_NT - 1) / (4 * CM_MULTI_NT)), dim3(CM_MULTI_NT), 0, s, a);
    return hipGetLastError();
  }
  if (a.vocab <= 8192) hipLaunchKernelGGL(k_classify<2>, dim3(1), dim3(FEAT_NT), 0, s, a);
  else if (a.vocab <= 32768) hipLaunchKernelGGL(k_classify<8>, dim3(1), dim3(FEAT_NT), 0, s, a);
  else hipLaunchKernelGGL(k_classify<16>, dim3(1), dim3(FEAT_NT), 0, s, a);
  return hipGetLastError();
}

// Scratch of the allocation-free form of the classify call (callers that cannot allocate): one copy of
// this array per GPU, held from module load until the process ends.  In host code the name is only a
// handle for hipGetSymbolAddress; kernels and clears get the device address looked up below.
static __device__ __align__(256) unsigned char scratch[CLASSIFY_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static float* g_scratch_ptr[MAX_DEVICES];        // device address of `scratch` on each GPU, once looked up

// Device address of the current GPU's copy of `scratch` (looked up once per device, with that device current).
hipError_t classify_static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// per-row arg-max of the verification logits; acceptance; KV fill; draft-loop bookkeeping
// ---------------------------------------------------------------------------------------------

// abort_word (may be null): set by a persistent forward whose grid barrier gave up; the rows then get -1.
__global__ __launch_bounds__(1024) void k_argmax_rows(const float* __restrict__ logits, int vocab, int32_t* __restrict__ out,
                                                      const unsigned* abort_word) {
  __shared__ float sv[17];
  __shared__ int si[17];
  const float* x = logits + (size_t)blockIdx.x * vocab;
  VI mine; mine.v = -INFINITY; mine.i = 0x7fffffff;
  if ((vocab & 3) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0) {
    // eight 128-bit loads per thread in flight at once (a row of 32768 logits in one round), then the comparisons
    const float4* x4 = reinterpret_cast<const float4*>(x);
    const int n4 = vocab >> 2;
    for (int base = 0; base < n4; base += 8 * 1024) {
      float4 v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int i = base + k * 1024 + threadIdx.x;
        v[k] = i < n4 ? x4[i] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int i = 4 * (base + k * 1024 + threadIdx.x);
        const float e[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) { VI y; y.v = e[c]; y.i = i + c; if (i + c < vocab) mine = vi_best(mine, y); }
      }
    }
  } else {
    for (int i = threadIdx.x; i < vocab; i += 1024) { VI y; y.v = x[i]; y.i = i; mine = vi_best(mine, y); }
  }
  const VI b = block_argmax<1024>(mine, sv, si);
  if (threadIdx.x == 0) out[blockIdx.x] = (abort_word != nullptr && *abort_word != 0u) ? -1 : b.i;
}

hipError_t launch_argmax_rows(const float* logits, int M, int vocab, int32_t* out, const unsigned* abort_word, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax_rows, dim3(M), dim3(1024), 0, s, logits, vocab, out, abort_word);
  return hipGetLastError();
}

struct AcceptOut { int32_t n; int32_t n_emit; int32_t emit[16]; };

__global__ void k_accept(const int32_t* block, const int32_t* argmax, int n_block, const int32_t* dev_n_block,
                         AcceptOut* out, AcceptOut* host_out) {
  if (threadIdx.x != 0) return;
  int nb = n_block;
  if (dev_n_block) { const int v = *dev_n_block; nb = v < 1 ? 1 : (v > n_block ? n_block : v); }
  int n = 0;
  while (n < nb - 1 && block[n + 1] == argmax[n]) ++n;
  AcceptOut r;
  r.n = n; r.n_emit = n + 1;
  for (int i = 0; i < 16; ++i) r.emit[i] = (i < n) ? block[i + 1] : (i == n ? argmax[n] : -1);
  *out = r;
  if (host_out) { *host_out = r; __threadfence_system(); }
}

hipError_t launch_accept(const int32_t* block, const int32_t* argmax, int n_block, const int32_t* dev_n_block,
                         void* dev_out, void* host_out, hipStream_t s) {
  hipLaunchKernelGGL(k_accept, dim3(1), dim3(64), 0, s, block, argmax, n_block, dev_n_block,
                     reinterpret_cast<AcceptOut*>(dev_out), reinterpret_cast<AcceptOut*>(host_out));
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_kv_fill(const bf16_t* __restrict__ src, bf16_t* __restrict__ pages,
                                                 const int32_t* __restrict__ page_table, int n_layers, int n_pages,
                                                 int pt, int nkv, int dh, int ctx) {
  // src [layer][sel][pos][kvh][dh]; one thread per 8 elements
  const int64_t vec_per_row = dh / 8;
  const int64_t total = (int64_t)n_layers * 2 * ctx * nkv * vec_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int64_t r = i;
    const int cv = (int)(r % vec_per_row); r /= vec_per_row;
    const int kvh = (int)(r % nkv); r /= nkv;
    const int pos = (int)(r % ctx); r /= ctx;
    const int sel = (int)(r % 2); r /= 2;
    const int layer = (int)r;
    const int lp = pos / pt, off = pos % pt;
    const int pp = page_table ? page_table[lp] : lp;
    const size_t blk = ((((size_t)layer * n_pages + pp) * 2 + sel) * nkv + kvh) * pt * dh;
    const uint4 val = *reinterpret_cast<const uint4*>(src + i * 8);
    if (sel == 0) {                                   // K: [token][d_head]
      *reinterpret_cast<uint4*>(pages + blk + (size_t)off * dh + cv * 8) = val;
    } else {                                          // V: transposed, [d_head][token]
      const uint32_t wv[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
      for (int e = 0; e < 8; ++e)
        pages[blk + (size_t)(cv * 8 + e) * pt + off] = (bf16_t)(wv[e >> 1] >> ((e & 1) * 16));
    }
  }
}

hipError_t launch_kv_fill(const bf16_t* src, bf16_t* pages, const int32_t* page_table, int n_layers, int n_pages,
                          int page_tokens, int nkv, int dh, int ctx, hipStream_t s) {
  const int64_t total = (int64_t)n_layers * 2 * ctx * nkv * (dh / 8);
  int64_t blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_kv_fill, dim3((unsigned)blocks), dim3(256), 0, s, src, pages, page_table, n_layers, n_pages,
                     page_tokens, nkv, dh, ctx);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// sampling at temperature > 0: draws by inverse CDF in vocabulary order, speculative acceptance
// ---------------------------------------------------------------------------------------------
//
// One workgroup of 1024 threads per row; the row lives in registers (V4 float4 per thread, element
// (i * 1024 + t) * 4 + e in slot i of thread t, one round of coalesced 128-bit loads).  Cumulative
// sums follow the vocabulary order: segment i (4096 elements) before segment i + 1, inside a segment
// thread by thread.  Every wavefront scans its 64 per-thread sums of every segment across lanes, the
// (segment, wavefront) totals go through LDS once, and every thread then knows the cumulative sum at
// the start of each of its float4 groups.  The group that holds u * total is walked by its owner.
// All sums are fp32.

constexpr int SMP_NT = 1024;
constexpr int SMP_NW = SMP_NT / 64;

template <int V4>
struct SmpRow { float4 w[V4]; };     // weights (or raw logits) of one row, register resident

template <int V4>
__device__ __forceinline__ void smp_load(SmpRow<V4>& r, const float* x, int V, float pad) {
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int idx = (i * SMP_NT + threadIdx.x) * 4;
    r.w[i] = (idx < V) ? *reinterpret_cast<const float4*>(x + idx) : make_float4(pad, pad, pad, pad);   // V % 4 == 0
  }
}

template <int V4>
__device__ __forceinline__ float smp_block_max(const SmpRow<V4>& r, float* smem) {
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < V4; ++i) mx = fmaxf(mx, fmaxf(fmaxf(r.w[i].x, r.w[i].y), fmaxf(r.w[i].z, r.w[i].w)));
  mx = wave_max(mx);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = mx;
  __syncthreads();
  float t = smem[0];
#pragma unroll
  for (int i = 1; i < SMP_NW; ++i) t = fmaxf(t, smem[i]);
  __syncthreads();
  return t;
}

// Cumulative sum (vocabulary order) of the weights before each of this thread's float4 groups, and
// the row total.  seg_tot: LDS [V4][SMP_NW].
template <int V4>
__device__ __forceinline__ float smp_prefix(const SmpRow<V4>& r, float (&excl)[V4], float* seg_tot) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  float own[V4];
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    own[i] = (r.w[i].x + r.w[i].y) + (r.w[i].z + r.w[i].w);
    float inc = own[i];
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const float o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    excl[i] = inc - own[i];                                   // inside the wavefront so far
    if (lane == 63) seg_tot[i * SMP_NW + wv] = inc;
  }
  __syncthreads();
  float run = 0.f;
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    float before = 0.f, seg = 0.f;
#pragma unroll
    for (int ww = 0; ww < SMP_NW; ++ww) { const float v = seg_tot[i * SMP_NW + ww]; if (ww < wv) before += v; seg += v; }
    excl[i] += run + before;
    run += seg;
  }
  __syncthreads();
  return run;
}

// Inverse CDF at u * total: the smallest index whose cumulative sum exceeds the target (the last
// index with a positive weight if rounding leaves the target at the very end).
template <int V4>
__device__ __forceinline__ int smp_draw(const SmpRow<V4>& r, float u, float* seg_tot, int* ismem) {
  float excl[V4];
  const float total = smp_prefix<V4>(r, excl, seg_tot);
  const float target = u * total;
  int key = -1;                                               // last group (in order) that starts at or before the target
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const float own = (r.w[i].x + r.w[i].y) + (r.w[i].z + r.w[i].w);
    if (own > 0.f && excl[i] <= target) key = i * SMP_NT + threadIdx.x;
  }
  int best = key;
  best = max(best, __shfl_xor(best, 1)); best = max(best, __shfl_xor(best, 2)); best = max(best, __shfl_xor(best, 4));
  best = max(best, __shfl_xor(best, 8)); best = max(best, __shfl_xor(best, 16)); best = max(best, __shfl_xor(best, 32));
  if ((threadIdx.x & 63) == 0) ismem[threadIdx.x >> 6] = best;
  __syncthreads();
  int win = -1;
#pragma unroll
  for (int i = 0; i < SMP_NW; ++i) win = max(win, ismem[i]);
  __syncthreads();
  if (win >= 0 && key == win) {
    float4 g = r.w[0]; float c = excl[0];
#pragma unroll
    for (int i = 1; i < V4; ++i) if (i == win / SMP_NT) { g = r.w[i]; c = excl[i]; }
    const float w4[4] = {g.x, g.y, g.z, g.w};
    int pick = -1, last_pos = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (w4[e] > 0.f) last_pos = e;
      c += w4[e];
      if (pick < 0 && c > target) pick = e;
    }
    ismem[0] = win * 4 + (pick >= 0 ? pick : last_pos);
  }
  __syncthreads();
  const int res = win >= 0 ? ismem[0] : 0;
  __syncthreads();
  return res;
}

// r := e^((x - max) / T) elementwise (padding becomes 0); returns max, *sum gets the row sum.
template <int V4>
__device__ __forceinline__ float smp_exp(SmpRow<V4>& r, float inv_t, float* smem, float* seg_tot, float* sum) {
  const float m = smp_block_max<V4>(r, smem);
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    r.w[i].x = expf((r.w[i].x - m) * inv_t); r.w[i].y = expf((r.w[i].y - m) * inv_t);
    r.w[i].z = expf((r.w[i].z - m) * inv_t); r.w[i].w = expf((r.w[i].w - m) * inv_t);
  }
  float excl[V4];
  *sum = smp_prefix<V4>(r, excl, seg_tot);
  return m;
}

// Draw one token per row from softmax(logits / T); optionally store the probability row.
template <int V4>
__global__ __launch_bounds__(SMP_NT) void k_sample_rows(SampleArgs a) {
  if (gated(a.gate)) return;
  __shared__ float smem[SMP_NW];
  __shared__ float seg_tot[V4 * SMP_NW];
  __shared__ int ismem[SMP_NW];
  const int row = blockIdx.x, V = a.vocab;
  SmpRow<V4> r;
  smp_load<V4>(r, a.logits + (size_t)row * a.ld, V, -INFINITY);
  float S;
  smp_exp<V4>(r, a.inv_t, smem, seg_tot, &S);
  const int tok = smp_draw<V4>(r, a.u[row], seg_tot, ismem);
  if (a.probs) {
    float* p = a.probs + (size_t)row * V;
    const float inv_s = 1.0f / S;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int idx = (i * SMP_NT + threadIdx.x) * 4;
      if (idx < V) *reinterpret_cast<float4*>(p + idx) = make_float4(r.w[i].x * inv_s, r.w[i].y * inv_s, r.w[i].z * inv_s, r.w[i].w * inv_s);
    }
  }
  if (threadIdx.x == 0) {
    a.tokens[row] = tok;
    if (row == 0 && a.token_next) *a.token_next = tok;
    if (row == 0 && a.block_slot) *a.block_slot = tok;
  }
}

hipError_t launch_sample_rows(const SampleArgs& a, int n_rows, hipStream_t s) {
  if (n_rows < 1 || a.vocab < 4 || (a.vocab & 3) || a.vocab > 65536 || (a.ld & 3)) return hipErrorInvalidValue;
  if (a.vocab <= 8192) hipLaunchKernelGGL(k_sample_rows<2>, dim3(n_rows), dim3(SMP_NT), 0, s, a);
  else if (a.vocab <= 32768) hipLaunchKernelGGL(k_sample_rows<8>, dim3(n_rows), dim3(SMP_NT), 0, s, a);
  else hipLaunchKernelGGL(k_sample_rows<16>, dim3(n_rows), dim3(SMP_NT), 0, s, a);
  return hipGetLastError();
}

// Speculative sampling over one block: keep d_j while u_j q_j(d_j) < p_{j-1}(d_j); the last token is
// drawn from norm(max(0, p_n - q_n)) at the first rejection, from p_SL when everything is kept.
template <int V4>
__global__ __launch_bounds__(SMP_NT) void k_accept_sample(AcceptSampleArgs a) {
  __shared__ float smem[SMP_NW];
  __shared__ float seg_tot[V4 * SMP_NW];
  __shared__ int ismem[SMP_NW];
  __shared__ float p_tok;
  const int V = a.vocab;
  int nb = a.n_block;
  if (a.dev_n_block) { const int v = *a.dev_n_block; nb = v < 1 ? 1 : (v > a.n_block ? a.n_block : v); }
  const int sl = nb - 1;
  int n = 0;
  bool rejected = false;
  SmpRow<V4> r;
  float S = 1.f;
  for (;;) {
    // target distribution after block[0..n]
    smp_load<V4>(r, a.target_logits + (size_t)n * V, V, -INFINITY);
    smp_exp<V4>(r, a.inv_t, smem, seg_tot, &S);
    if (n == sl) break;
    int tok = a.block[n + 1];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    // the thread that holds the draft token publishes its target probability
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int idx = (i * SMP_NT + threadIdx.x) * 4;
      if (tok >= idx && tok < idx + 4) {
        const float w4[4] = {r.w[i].x, r.w[i].y, r.w[i].z, r.w[i].w};
        p_tok = w4[tok - idx] * (1.0f / S);
      }
    }
    __syncthreads();
    const float p = p_tok;
    const float q = a.draft_probs[(size_t)n * V + tok];
    __syncthreads();
    if (a.u_accept[n] * q < p) ++n; else { rejected = true; break; }
  }
  if (rejected) {
    // residual max(0, p - q) of row n
    const float inv_s = 1.0f / S;
    const float* q = a.draft_probs + (size_t)n * V;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int idx = (i * SMP_NT + threadIdx.x) * 4;
      float4 qq = make_float4(0.f, 0.f, 0.f, 0.f);
      if (idx < V) qq = *reinterpret_cast<const float4*>(q + idx);
      r.w[i].x = fmaxf(0.f, r.w[i].x * inv_s - qq.x); r.w[i].y = fmaxf(0.f, r.w[i].y * inv_s - qq.y);
      r.w[i].z = fmaxf(0.f, r.w[i].z * inv_s - qq.z); r.w[i].w = fmaxf(0.f, r.w[i].w * inv_s - qq.w);
    }
  }
  const int last = smp_draw<V4>(r, a.u_resample[n], seg_tot, ismem);
  if (threadIdx.x == 0) {
    AcceptOut o;
    o.n = n; o.n_emit = n + 1;
    for (int i = 0; i < 16; ++i) o.emit[i] = (i < n) ? a.block[i + 1] : (i == n ? last : -1);
    *reinterpret_cast<AcceptOut*>(a.out) = o;
    if (a.host_out) { *reinterpret_cast<AcceptOut*>(a.host_out) = o; __threadfence_system(); }
  }
}

hipError_t launch_accept_sample(const AcceptSampleArgs& a, hipStream_t s) {
  if (a.n_block < 1 || a.n_block > 16 || a.vocab < 4 || (a.vocab & 3) || a.vocab > 65536) return hipErrorInvalidValue;
  if (a.vocab <= 8192) hipLaunchKernelGGL(k_accept_sample<2>, dim3(1), dim3(SMP_NT), 0, s, a);
  else if (a.vocab <= 32768) hipLaunchKernelGGL(k_accept_sample<8>, dim3(1), dim3(SMP_NT), 0, s, a);
  else hipLaunchKernelGGL(k_accept_sample<16>, dim3(1), dim3(SMP_NT), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// classifier training and evaluation (the step after the loop: features and labels in, parameters out)
// ---------------------------------------------------------------------------------------------
//
// One workgroup; thread h owns hidden unit h (its row of W1, b1[h], w2[h]) and its gradients, so the
// only cross-thread quantity is the pre-sigmoid output z of a sample (a workgroup sum per sample).
// The standardised training set sits in LDS for the whole run.  Full-batch gradient descent on the
// mean binary cross-entropy; all arithmetic fp32 except the feature statistics (double).

constexpr int TRAIN_MAX_N = 2560;               // samples that fit in LDS (12 floats each)

__global__ __launch_bounds__(256) void k_clf_train(TrainArgs a) {
  __shared__ float fs[TRAIN_MAX_N * 12];
  __shared__ float mu_s[12], isd_s[12];
  __shared__ float zpart[4];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6, nw = blockDim.x >> 6;
  const int N = a.n, H = a.hidden;
  if (t < 12) {
    double sum = 0.0;
    for (int n = 0; n < N; ++n) sum += (double)a.feats[(size_t)n * 12 + t];
    const double mu = sum / N;
    double var = 0.0;
    for (int n = 0; n < N; ++n) { const double d = (double)a.feats[(size_t)n * 12 + t] - mu; var += d * d; }
    double sd = sqrt(var / N);
    if (sd < 1e-6) sd = 1e-6;
    mu_s[t] = (float)mu; isd_s[t] = (float)(1.0 / sd);
  }
  __syncthreads();
  for (int i = t; i < N * 12; i += blockDim.x) fs[i] = (a.feats[i] - mu_s[i % 12]) * isd_s[i % 12];
  const bool live = t < H;
  float w1[12], b1 = 0.f, w2 = 0.f, b2 = a.params[H * 14];
#pragma unroll
  for (int i = 0; i < 12; ++i) w1[i] = live ? a.params[t * 12 + i] : 0.f;
  if (live) { b1 = a.params[H * 12 + t]; w2 = a.params[H * 13 + t]; }
  __syncthreads();
  const float inv_n = 1.0f / (float)N;
  for (int ep = 0; ep < a.epochs; ++ep) {
    float gw1[12], gb1 = 0.f, gw2 = 0.f, gb2 = 0.f, loss = 0.f;
#pragma unroll
    for (int i = 0; i < 12; ++i) gw1[i] = 0.f;
    for (int n = 0; n < N; ++n) {
      const float* f = fs + n * 12;
      float pre = b1;
#pragma unroll
      for (int i = 0; i < 12; ++i) pre += w1[i] * f[i];
      const float act = live ? fmaxf(pre, 0.f) : 0.f;
      float z = wave_sum(w2 * act);
      if (nw > 1) {
        if (lane == 0) zpart[wv] = z;
        __syncthreads();
        z = zpart[0];
        for (int ww = 1; ww < nw; ++ww) z += zpart[ww];
        __syncthreads();
      }
      z += b2;
      const float y = (float)a.labels[n];
      loss += fmaxf(z, 0.f) - z * y + log1pf(expf(-fabsf(z)));
      const float dz = (1.0f / (1.0f + expf(-z)) - y) * inv_n;
      gw2 += dz * act;
      gb2 += dz;
      const float da = pre > 0.f ? dz * w2 : 0.f;
      gb1 += da;
#pragma unroll
      for (int i = 0; i < 12; ++i) gw1[i] += da * f[i];
    }
    if (t == 0 && a.loss) a.loss[ep] = loss * inv_n;
#pragma unroll
    for (int i = 0; i < 12; ++i) w1[i] -= a.lr * gw1[i];
    b1 -= a.lr * gb1; w2 -= a.lr * gw2; b2 -= a.lr * gb2;
  }
  // fold the standardisation into W1 and b1: the classifier consumes raw features
  if (live) {
    float shift = 0.f;
#pragma unroll
    for (int i = 0; i < 12; ++i) {
      const float wf = w1[i] * isd_s[i];
      a.params[t * 12 + i] = wf;
      shift += wf * mu_s[i];
    }
    a.params[H * 12 + t] = b1 - shift;
    a.params[H * 13 + t] = w2;
  }
  if (t == 0) a.params[H * 14] = b2;
}

hipError_t launch_clf_train(const TrainArgs& a, hipStream_t s) {
  if (a.n < 1 || a.n > TRAIN_MAX_N || a.hidden < 1 || a.hidden > 256 || a.epochs < 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_clf_train, dim3(1), dim3(((a.hidden + 63) / 64) * 64), 0, s, a);
  return hipGetLastError();
}

// Scores of given feature vectors and the confusion counts of "accepted iff C >= tau" against the
// labels: counts[0..3] = true positives, false positives, false negatives, true negatives.
__global__ __launch_bounds__(256) void k_clf_eval(EvalArgs a) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= a.n) return;
  const int H = a.hidden;
  float f[12];
#pragma unroll
  for (int i = 0; i < 12; ++i) f[i] = a.feats[(size_t)n * 12 + i];
  float z = 0.f;
  for (int h = 0; h < H; ++h) {                    // fixed order
    float pre = a.params[H * 12 + h];
#pragma unroll
    for (int i = 0; i < 12; ++i) pre += a.params[h * 12 + i] * f[i];
    z += fmaxf(pre, 0.f) * a.params[H * 13 + h];
  }
  const float c = 1.0f / (1.0f + expf(-(z + a.params[H * 14])));
  if (a.scores) a.scores[n] = c;
  if (a.counts && a.labels) {
    const int pred = c >= a.tau ? 1 : 0, y = a.labels[n] != 0 ? 1 : 0;
    atomicAdd(a.counts + (pred ? (y ? 0 : 1) : (y ? 2 : 3)), 1);
  }
}

hipError_t launch_clf_eval(const EvalArgs& a, hipStream_t s) {
  if (a.n < 1 || a.hidden < 1 || a.hidden > 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_clf_eval, dim3((a.n + 255) / 256), dim3(256), 0, s, a);
  return hipGetLastError();
}

// Training examples of the labelling run (App. D.1): from the classify record of every position, the twelve
// features, the draft's token and the label "the draft's token equals the target's token there".
__global__ __launch_bounds__(256) void k_clf_examples(const ClfOut* __restrict__ rec, int n, const int32_t* __restrict__ ref_tokens,
                                                      float* __restrict__ feats, int32_t* __restrict__ labels, int32_t* __restrict__ tokens) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const ClfOut r = rec[i];
#pragma unroll
  for (int k = 0; k < 12; ++k) feats[(size_t)i * 12 + k] = r.feats[k];
  labels[i] = (r.token == ref_tokens[i]) ? 1 : 0;
  if (tokens != nullptr) tokens[i] = r.token;
}

hipError_t launch_clf_examples(const void* rec, int n, const int32_t* ref_tokens, float* feats, int32_t* labels, int32_t* tokens,
                               hipStream_t s) {
  hipLaunchKernelGGL(k_clf_examples, dim3((n + 255) / 256), dim3(256), 0, s, reinterpret_cast<const ClfOut*>(rec), n, ref_tokens,
                     feats, labels, tokens);
  return hipGetLastError();
}

struct LoopOut { int32_t sl; int32_t block[16]; int32_t halted; };   // mirrors disco_loop_out

__global__ void k_loop_init(uint32_t* gate, int32_t* sl_count, const int32_t* tokens_in, int n_in, LoopOut* out) {
  if (threadIdx.x != 0) return;
  *gate = 0u; sl_count[0] = 0; sl_count[1] = 0;     // second word: the perplexity rule's running sum (0.0f)
  out->sl = 0; out->halted = 0;
  out->block[0] = tokens_in[n_in - 1];
  for (int i = 1; i < 16; ++i) out->block[i] = 0;
}

__global__ void k_loop_finish(const int32_t* sl_count, const uint32_t* gate, LoopOut* out, LoopOut* host_out, const unsigned* abort_word) {
  if (threadIdx.x != 0) return;
  out->sl = (abort_word != nullptr && *abort_word != 0u) ? -1 : *sl_count;
  out->halted = (int32_t)*gate;
  if (host_out) { *host_out = *out; __threadfence_system(); }
}

__global__ __launch_bounds__(256) void k_zero(int* p, int n) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) p[i] = 0;
}

// Rotary table: (cos, sin) of pos * base^(-2 i / d_head) for every cached position and channel pair
// i; the angle is formed in double precision, the table holds floats.
__global__ __launch_bounds__(256) void k_rope_fill(float* tab, int n_pos, int dh, float base) {
  const int half = dh >> 1;
  const int64_t total = (int64_t)n_pos * half;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int pos = (int)(idx / half), i = (int)(idx % half);
    const double inv_freq = exp2(-(2.0 * (double)i / (double)dh) * log2((double)base));
    double sn, cs;
    sincos((double)pos * inv_freq, &sn, &cs);
    tab[idx * 2] = (float)cs;
    tab[idx * 2 + 1] = (float)sn;
  }
}

hipError_t launch_rope_fill(float* tab, int n_pos, int dh, float base, hipStream_t s) {
  const int64_t total = (int64_t)n_pos * (dh / 2);
  int64_t blocks = (total + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_rope_fill, dim3((unsigned)blocks), dim3(256), 0, s, tab, n_pos, dh, base);
  return hipGetLastError();
}

hipError_t launch_zero(int* p, int n, hipStream_t s) {
  hipLaunchKernelGGL(k_zero, dim3(n > 4096 ? 16 : 1), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

hipError_t launch_loop_init(uint32_t* gate, int32_t* sl_count, const int32_t* tokens_in, int n_in, void* dev_loop_out,
                            hipStream_t s) {
  hipLaunchKernelGGL(k_loop_init, dim3(1), dim3(64), 0, s, gate, sl_count, tokens_in, n_in,
                     reinterpret_cast<LoopOut*>(dev_loop_out));
  return hipGetLastError();
}

// Host values into device slots: the pending tokens of an iteration (n <= 2) and, for an iteration that
// drafts nothing, the one-token block.
__global__ void k_put_tokens(int32_t* tokens, int t0, int t1, int n, LoopOut* out, LoopOut* host_out) {
  if (threadIdx.x != 0) return;
  if (tokens) { tokens[0] = t0; if (n > 1) tokens[1] = t1; }
  if (out) {
    out->sl = 0; out->halted = 1; out->block[0] = n > 1 ? t1 : t0;
    for (int i = 1; i < 16; ++i) out->block[i] = 0;
    if (host_out) *host_out = *out;
  }
}

hipError_t launch_put_tokens(int32_t* tokens, int t0, int t1, int n, void* dev_loop_out, void* host_loop_out, hipStream_t s) {
  hipLaunchKernelGGL(k_put_tokens, dim3(1), dim3(64), 0, s, tokens, t0, t1, n, reinterpret_cast<LoopOut*>(dev_loop_out),
                     reinterpret_cast<LoopOut*>(host_loop_out));
  return hipGetLastError();
}

hipError_t launch_loop_finish(const int32_t* sl_count, const uint32_t* gate, void* dev_loop_out, void* host_loop_out,
                              const unsigned* abort_word, hipStream_t s) {
  hipLaunchKernelGGL(k_loop_finish, dim3(1), dim3(64), 0, s, sl_count, gate, reinterpret_cast<LoopOut*>(dev_loop_out),
                     reinterpret_cast<LoopOut*>(host_loop_out), abort_word);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// dense prompt pass: the GEMMs of a forward over many groups of 16 tokens at once
// ---------------------------------------------------------------------------------------------
//
// The prompt is processed before the first iteration (Sec. 2: the target model is given a prompt).
// With hundreds of tokens per pass the GEMMs are bound by the matrix unit, not by the weight stream,
// so the tiling differs from the skinny kernel: a wavefront owns RT weight row tiles x 4 token groups
// (16 x 16 accumulators each), walks the whole K range itself (no K split, no cross-wavefront
// reduction), and every weight tile it fetches feeds 8 matrix instructions (hi and lo panel of 4
// groups).  The four wavefronts of a workgroup take neighbouring row tiles and the SAME token groups.
// Workgroup ids are dealt round-robin to the 8 XCDs; every row block belongs to one XCD, whose
// workgroups walk tiles of several row blocks x several token blocks (see the kernel), so that its L2
// serves each weight and activation slab to all workgroups of the tile.  Operand layouts, precision (bf16 hi + lo activations, fp32
// accumulation) and epilogue arithmetic are those of the skinny kernel.

// Epilogues of the dense kernels for one wavefront: RT row tiles x CG token groups of accumulators.
template <int EPI, int RT, int CG>
__device__ __forceinline__ void dense_epilogue(const DenseArgs& d, const int cb, const int (&rt)[RT], f32x4 (&acc)[RT][CG]) {
  constexpr bool PAIR = EpiTraits<EPI>::pair;
  constexpr int UNITS = PAIR ? RT / 2 : RT, TPU = PAIR ? 2 : 1;
  constexpr bool NORMED = (EPI != EPI_PARTIAL);
  const GemmArgs& a = d.g;
  const int lane = threadIdx.x & 63;
  const int m = lane & 15, g = lane >> 4;         // token column, 4-row group of the 16 x 16 result
#pragma unroll
  for (int c = 0; c < CG; ++c) {
    const int ci = cb * CG + c;
    if (ci < d.n_groups) {
    float rstd = 1.f;
    if (NORMED && d.rstd != nullptr) rstd = d.rstd[ci * 16 + m];
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      f32x4 y0 = acc[u * TPU][c] * rstd, y1 = acc[u * TPU + TPU - 1][c] * rstd;
      const int t0 = rt[u * TPU];
      if (EPI == EPI_PARTIAL) {
        // residual-stream update h += X.W^T, panels of gain * h and this tile's sums of squares for the next GEMM
        const int col = t0 * 16 + 4 * g;
        float4* hp = reinterpret_cast<float4*>(a.h + (size_t)ci * d.hs + (size_t)m * a.ld_out + col);
        float4 h = *hp;
        h.x += y0[0]; h.y += y0[1]; h.z += y0[2]; h.w += y0[3];
        *hp = h;
        if (a.Xout != nullptr) {                  // deferred RMSNorm of the next GEMM (LayerNorm models: a norm launch instead)
          const float4 gn = *reinterpret_cast<const float4*>(a.gain + col);
          const float o[4] = {h.x * gn.x, h.y * gn.y, h.z * gn.z, h.w * gn.w};
          xpack_store4(a.Xout + (size_t)ci * d.xouts, a.KT_out, 16, m, col, o);
          const float sq = row4_sum((h.x * h.x + h.y * h.y) + (h.z * h.z + h.w * h.w));
          if (g == 0) a.ssq_out[(size_t)ci * d.ssq_outs + t0 * 16 + m] = sq;    // [slot][token]
        }
      } else if (EPI == EPI_GELU) {
        float act[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) act[v] = 0.5f * y0[v] * (1.0f + erff(y0[v] * 0.70710678118654752f));
        xpack_store4(a.Xout + (size_t)ci * d.xouts, a.KT_out, 16, m, t0 * 16 + 4 * g, act);
      } else if (EPI == EPI_QKV) {
        float lo4[4] = {y0[0], y0[1], y0[2], y0[3]}, hi4[4] = {y1[0], y1[1], y1[2], y1[3]};
        qkv_store(a, a.q + (size_t)ci * d.qs, t0 * 16 + 4 * g, m, a.pos0 + 16 * ci + m, lo4, hi4);
      } else if (EPI == EPI_SWIGLU) {
        const int f = (t0 >> 1) * 16 + 4 * g;
        float act[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) act[v] = y0[v] / (1.0f + expf(-y0[v])) * y1[v];
        xpack_store4(a.Xout + (size_t)ci * d.xouts, a.KT_out, 16, m, f, act);
      }
    }
    }
  }
}

// The activation tiles are shared through LDS: wavefront w fetches the hi and lo tile
// of token group w only (a quarter of the workgroup's activation tiles), a two-stage LDS ring hands
// them to the other three, and the registers freed that way hold NB k-tiles of loads in flight.  One
// workgroup barrier per k-tile; every wavefront runs the same trip count (idle ones compute on clamped
// rows and store nothing).
// HI: bf16 activations.  Only the hi panels are read, and the LDS slots and matrix instructions that the lo
// panels took serve four more token groups instead: a workgroup then covers 8 token groups, the work per weight
// tile is unchanged and the weights are fetched half as often.
template <int EPI, int NB, int RT, bool HI>
__global__ __launch_bounds__(256) void k_gemm_dense(DenseArgs d) {
  constexpr int CG = HI ? 8 : 4, NWV = 4, NS = NB + 1;
  constexpr bool PAIR = EpiTraits<EPI>::pair;
  constexpr int UNITS = PAIR ? RT / 2 : RT;
  __shared__ u32x4 bs[HI ? 3 : 2][8][64];
  const GemmArgs& a = d.g;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n_tiles = a.n_rows >> 4;
  const int ncb = (d.n_groups + CG - 1) / CG;
  const int nrb = (n_tiles + RT * NWV - 1) / (RT * NWV);
  // Workgroup ids go round-robin to the 8 XCDs.  Within an XCD consecutive ids walk a tile of tile_r row
  // blocks x tile_t token blocks (about as many workgroups as the XCD runs at once), so that what its L2
  // must fetch for the workgroups in flight is tile_r weight slabs + tile_t activation slabs.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per_tile = d.tile_r * d.tile_t, n_tg = (ncb + d.tile_t - 1) / d.tile_t;
  const int tile = slot / per_tile, in_tile = slot % per_tile;
  const int rbl = (tile / n_tg) * d.tile_r + in_tile / d.tile_t;          // row block index within the XCD
  const int rb = rbl * 8 + xcd, cb = (tile % n_tg) * d.tile_t + in_tile % d.tile_t;
  if (rb >= nrb || cb >= ncb) return;             // whole workgroup
  const bool live = (rb * NWV + w) * RT < n_tiles;
  const int b = live ? rb * NWV + w : n_tiles / RT - 1;
  int rt[RT];
  if (PAIR) {
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      const int bp = b * UNITS + u, gs = __builtin_ctz(a.grp);   // the pairing distance is a power of two
      rt[2 * u] = ((bp >> gs) << (gs + 1)) + (bp & (a.grp - 1));
      rt[2 * u + 1] = rt[2 * u] + a.grp;
    }
  } else {
#pragma unroll
    for (int r = 0; r < RT; ++r) rt[r] = b * RT + r;
  }
  const int KT = a.KT;
  const u32x4* Wp[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) Wp[r] = reinterpret_cast<const u32x4*>(a.W) + (size_t)rt[r] * KT * 64 + lane;
  // the two activation tiles this wavefront hands to the workgroup per k-tile: hi and lo panel of token group w, or
  // (HI) the hi panels of token groups 2w and 2w + 1
  const u32x4* Xw = reinterpret_cast<const u32x4*>(a.X + (size_t)min(cb * CG + (HI ? 2 * w : w), d.n_groups - 1) * d.xs) + lane;
  const u32x4* Xw1 = HI ? reinterpret_cast<const u32x4*>(a.X + (size_t)min(cb * CG + 2 * w + 1, d.n_groups - 1) * d.xs) + lane
                        : Xw + (size_t)a.KT * 64;
  f32x4 acc[RT][CG];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int c = 0; c < CG; ++c) acc[r][c] = f32x4{0.f, 0.f, 0.f, 0.f};

  u32x4 A[NS][RT], Bw[NS][2];
  auto gload = [&](u32x4 (&Ad)[RT], u32x4 (&Bd)[2], const int kt) {
    const size_t t = (size_t)(kt < KT ? kt : KT - 1) * 64;
    if (HI) { Bd[0] = Xw[t]; Bd[1] = Xw1[t]; }    // first: the pipelined form needs them one k-tile earlier than the weights
#pragma unroll
    for (int r = 0; r < RT; ++r) Ad[r] = Wp[r][t];
    if (!HI) { Bd[0] = Xw[t]; Bd[1] = Xw1[t]; }
  };
#pragma unroll
  for (int i = 0; i < NB; ++i) gload(A[i], Bw[i], i);
  if constexpr (HI) {
    // Three LDS stages, fragments read one k-tile ahead (with half the matrix work per k-tile the LDS round trip at the
    // head of an iteration shows; with hi + lo panels it hides behind twice the matrix instructions, and this form,
    // which asks for the activation tiles a k-tile earlier, measured slower there).  Iteration kt: request k-tile
    // kt + NB from memory, read the fragments of k-tile kt + 1 from stage (kt + 1) % 3 (written an iteration ago,
    // barrier passed) while the matrix instructions of k-tile kt run on the fragments read an iteration ago, put this
    // wavefront's share of k-tile kt + 2 into stage (kt + 2) % 3 (its last readers passed two barriers ago), barrier.
    static_assert(!HI || NB >= 3, "the activation tiles of k-tile kt + 2 go to LDS in iteration kt: they must have been requested before it");
    bs[0][2 * w][lane] = Bw[0][0]; bs[0][2 * w + 1][lane] = Bw[0][1];
    bs[1][2 * w][lane] = Bw[1][0]; bs[1][2 * w + 1][lane] = Bw[1][1];
    __syncthreads();
    u32x4 Bf[8], Bn[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) Bf[t] = bs[0][t][lane];
    int st1 = 1, st2 = 2;                         // (kt + 1) % 3, (kt + 2) % 3
    for (int kt0 = 0; kt0 < KT; kt0 += NS) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int kt = kt0 + i;
        if (kt < KT) {                            // uniform over the workgroup
          gload(A[(i + NB) % NS], Bw[(i + NB) % NS], kt + NB);
#pragma unroll
          for (int t = 0; t < 8; ++t) Bn[t] = bs[st1][t][lane];
          bs[st2][2 * w][lane] = Bw[(i + 2) % NS][0];
          bs[st2][2 * w + 1][lane] = Bw[(i + 2) % NS][1];
#pragma unroll
          for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int c = 0; c < 8; ++c)
              acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(A[i][r]), as_bf16x8(Bf[c]), acc[r][c], 0, 0, 0);
#pragma unroll
          for (int t = 0; t < 8; ++t) Bf[t] = Bn[t];
          st1 = st2; st2 = st2 == 2 ? 0 : st2 + 1;
          __syncthreads();
        }
      }
    }
  } else {
    static_assert(NB >= 2, "the slot refilled in an iteration must not be the one it hands to LDS");
    bs[0][2 * w][lane] = Bw[0][0]; bs[0][2 * w + 1][lane] = Bw[0][1];
    __syncthreads();
    // Iteration kt: request k-tile kt + NB from memory, read the fragments of k-tile kt from LDS stage
    // kt % 2, put this wavefront's share of k-tile kt + 1 into the other stage (its readers passed the
    // barrier of the iteration before), run the matrix instructions of k-tile kt, barrier.
    for (int kt0 = 0; kt0 < KT; kt0 += NS) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int kt = kt0 + i;
        if (kt < KT) {                            // uniform over the workgroup
          gload(A[(i + NB) % NS], Bw[(i + NB) % NS], kt + NB);
          u32x4 Bf[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) Bf[t] = bs[kt & 1][t][lane];
          bs[(kt + 1) & 1][2 * w][lane] = Bw[(i + 1) % NS][0];
          bs[(kt + 1) & 1][2 * w + 1][lane] = Bw[(i + 1) % NS][1];
          // hi panels of all accumulators, then lo panels: no instruction reads the result of the one before it
#pragma unroll
          for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
              for (int c = 0; c < CG; ++c)
                acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(A[i][r]), as_bf16x8(Bf[2 * c + p]), acc[r][c], 0, 0, 0);
          __syncthreads();
        }
      }
    }
  }
  if (live) dense_epilogue<EPI, RT, CG>(d, cb, rt, acc);
}

template <int EPI, int NB, int RT, bool HI>
static hipError_t launch_gemm_dense_rt(const DenseArgs& d, hipStream_t s) {
  constexpr int CG = HI ? 8 : 4;
  const int n_tiles = d.g.n_rows / 16, ncb = (d.n_groups + CG - 1) / CG;
  const int nrb = (n_tiles + 4 * RT - 1) / (4 * RT);
  DenseArgs a = d;
  // about 64 workgroups run on an XCD at once: 8 x 8 for long prompts, 16 x 4 measured better at 8 token blocks
  a.tile_t = ncb >= 16 ? 8 : (ncb < 4 ? ncb : 4);
  const int nrbl = (nrb + 7) / 8;                 // row blocks per XCD
  a.tile_r = 64 / a.tile_t < nrbl ? 64 / a.tile_t : nrbl;
  const long long blocks = 8LL * ((nrbl + a.tile_r - 1) / a.tile_r) * ((ncb + a.tile_t - 1) / a.tile_t) * a.tile_r * a.tile_t;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((k_gemm_dense<EPI, NB, RT, HI>), dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

// Row tiles per wavefront (a workgroup covers 4 x RT tiles x CG token groups).  Larger tiles fetch every operand less
// often, but the grid should fill the 256 compute units in its last round too: 5120 rows x 2048 tokens are 320
// workgroups at RT = 4 (the last 64 run alone) and exactly 256 at RT = 5.  A tile count is taken only if it fills the
// chip clearly better than the next larger one.  Two-tile epilogues need an even count; 128-row tiles need the bf16-activation
// form (their accumulators fill the accumulation registers).
template <int EPI, bool HI>
static hipError_t launch_gemm_dense_e(const DenseArgs& d, hipStream_t s) {
  constexpr bool PAIR = EpiTraits<EPI>::pair;
  constexpr int CG = HI ? 8 : 4;
  constexpr int NB = HI ? 4 : 5;                  // k-tiles of loads in flight per wavefront (measured best of 3..5 with two panels)
  const int n_tiles = d.g.n_rows / 16, ncb = (d.n_groups + CG - 1) / CG;
  auto wgs_of = [&](int rt) { return (long)((n_tiles + 4 * rt - 1) / (4 * rt)) * ncb; };
  // 64-row wavefront tiles unless they would leave compute units without a workgroup; 128-row tiles for the wide
  // projections with bf16 activations
  int best = wgs_of(4) >= 256 ? 4 : 2;
  if (HI && (n_tiles % 8) == 0 && wgs_of(8) >= 256) best = 8;
  if (wgs_of(best) <= 2 * 256 && cu_fill(wgs_of(best)) < 0.9) {        // at most two rounds: the idle share of the last one counts
    const int cand[] = {6, 5, 4, 3, 2};            // largest first
    for (int rt : cand) {
      if ((PAIR && (rt & 1)) || n_tiles % rt) continue;
      if (wgs_of(rt) >= 256 && cu_fill(wgs_of(rt)) >= 0.95) { best = rt; break; }
    }
  }
  switch (best) {
    case 8: if constexpr (HI) return launch_gemm_dense_rt<EPI, 3, 8, true>(d, s); else break;
    case 6: return launch_gemm_dense_rt<EPI, HI ? 4 : 3, 6, HI>(d, s);   // fewer tiles in flight: 6 x NB weight tiles must fit the registers
    case 5: if constexpr (!PAIR) return launch_gemm_dense_rt<EPI, 4, 5, HI>(d, s); else break;
    case 4: return launch_gemm_dense_rt<EPI, NB, 4, HI>(d, s);
    case 3: if constexpr (!PAIR) return launch_gemm_dense_rt<EPI, NB, 3, HI>(d, s); else break;
    default: break;
  }
  return launch_gemm_dense_rt<EPI, NB, 2, HI>(d, s);
}

template <int EPI>
static hipError_t launch_gemm_dense_h(const DenseArgs& d, hipStream_t s) {
  return d.hi_only ? launch_gemm_dense_e<EPI, true>(d, s) : launch_gemm_dense_e<EPI, false>(d, s);
}

hipError_t launch_gemm_dense(const DenseArgs& d, int epi, hipStream_t s) {
  const GemmArgs& a = d.g;
  if (a.M != 16 || d.n_groups < 1 || a.KT < 1 || a.n_rows < 64 || (a.n_rows % 64) != 0) return hipErrorInvalidValue;
  if ((epi == EPI_QKV || epi == EPI_SWIGLU) && (a.grp < 1 || (a.grp & (a.grp - 1)) != 0 || (a.n_rows / 32) % a.grp != 0)) return hipErrorInvalidValue;
  if (epi == EPI_QKV && a.dh != 64 && a.dh != 128) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_QKV: return launch_gemm_dense_h<EPI_QKV>(d, s);
    case EPI_SWIGLU: return launch_gemm_dense_h<EPI_SWIGLU>(d, s);
    case EPI_PARTIAL: return launch_gemm_dense_h<EPI_PARTIAL>(d, s);
    case EPI_GELU: return launch_gemm_dense_h<EPI_GELU>(d, s);
    default: return hipErrorInvalidValue;
  }
}

// 1 / rms of every row of the prompt pass from its per-tile sums of squares, added in slot order.
__global__ __launch_bounds__(256) void k_rstd_groups(const float* __restrict__ ssq, int n_ssq, int d, float eps,
                                                     float* __restrict__ rstd) {
  __shared__ float part[16][16];
  const int r = blockIdx.x, m = threadIdx.x & 15, p = threadIdx.x >> 4;
  const float* sq = ssq + (size_t)r * n_ssq * 16;
  float s = 0.f;
  for (int i = p; i < n_ssq; i += 16) s += sq[i * 16 + m];
  part[p][m] = s;
  __syncthreads();
  if (p == 0) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) tot += part[i][m];
    rstd[r * 16 + m] = 1.0f / sqrtf(tot / (float)d + eps);
  }
}

hipError_t launch_rstd_groups(const float* ssq, int n_ssq, int d, float eps, float* rstd, int n_groups, hipStream_t s) {
  if (n_groups < 1 || n_ssq < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_rstd_groups, dim3(n_groups), dim3(256), 0, s, ssq, n_ssq, d, eps, rstd);
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------
// QKV projection and attention of one layer in ONE launch (models whose heads all have their own K / V)
// ---------------------------------------------------------------------------------------------
//
// The attention of head h needs only the 3 d_head rows of the QKV projection that belong to h, so the dependency
// between the two phases is per head, not grid-wide.  The launch has the QKV projection's workgroups, dealt so that
// the G = 3 d_head / (16 RT) workgroups holding the q, K and V rows of one head are neighbours.  Each finishes its
// rows (rotary, query rows, cache entries: write-through stores), adds 1 to the head's counter, and then acts as
// range `j` of the head's attention: it waits until the counter shows G (bounded: after `limit` polls it sets the
// abort word and goes on with unusable data; the LM head then stores NaN logits and the arg-max and loop-finish
// kernels turn a set abort word into -1 outputs), with its first cache loads already in flight where they cannot touch a 128-byte line that the
// head's other workgroups are still writing.  The head's ranges are merged by the last one to finish, as in the
// stand-alone attention kernel; that workgroup also zeroes the head's counter for the next launch.  Nobody waits
// before it has signalled, so the launch completes whenever all its workgroups are resident at once; the launcher
// checks that they fit.  The counters are 256 bytes apart.
constexpr int QA_READY_SLOT = QKV_ATTN_READY_SLOT;   // ints between two heads' counters

struct HeadWaitHook {
  int* ready; int n; unsigned* abort_word; int limit;   // limit: polls (each a memory round trip, about 1 us) before giving up
  __device__ __forceinline__ void operator()() const {
    if (threadIdx.x == 0) {
      int spins = 0;
      if (limit < 0) __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      while (limit >= 0 && __hip_atomic_load(ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < n) {
        if (++spins > limit) {
          __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
};

template <int P, int RT, int U, int DH>
__global__ __launch_bounds__(512) void k_qkv_attn(GemmArgs g, AttnArgs a, int* ready, unsigned* abort_word, int safe_end, int limit) {
  constexpr int UH = DH / (16 * RT), G = 3 * UH;   // workgroups per q / K / V part of a head, per head
  static_assert(UH >= 1 && UH * 16 * RT == DH, "a head part is a whole number of workgroups");
  union Smem { GemmSmem<RT, 8> gemm; AttnSmem<DH, 8> attn; };
  __shared__ Smem sm;
  const int head = blockIdx.x / G, j = blockIdx.x % G;
  const int part = j / UH, sub = j % UH;
  const int hu = part == 0 ? head : (part == 1 ? g.nq + head : g.nq + g.nkv + head);
  const uint32_t halted = gate_request(g.gate);
  gemm_unit<P, RT, EPI_QKV, 8, U, true>(g, hu * UH + sub, 0, g.KT, 0, 1, sm.gemm);
  if (halted != 0u) return;                       // uniform over the launch; nothing has been written
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_waitcnt(0);                  // this wavefront's write-through stores have completed
  __syncthreads();                                // ... and those of the whole workgroup
  int* rdy = ready + head * QA_READY_SLOT;
  if (threadIdx.x == 0) __hip_atomic_fetch_add(rdy, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (j >= a.n_splits) return;
  attn_range<DH, 8, false, false, true, HeadWaitHook>(a, head, j, sm.attn, 0u, HeadWaitHook{rdy, G, abort_word, limit}, safe_end, rdy);
}

// Workgroups of `kernel` (512 threads, static LDS only) that the device holds at once.
static long resident_capacity(const void* kernel) {
  int per_cu = 0, dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 512, 0) != hipSuccess || per_cu < 1) return 0;
  return (long)per_cu * prop.multiProcessorCount;
}

template <int P, int RT, int DH>
static hipError_t launch_qkv_attn_cfg(const GemmArgs& g, const AttnArgs& a, int* ready, unsigned* abort_word, int safe_end, int limit,
                                      bool* launched, hipStream_t s) {
  constexpr int U = gemm_buffers(RT, P);
  static const long capacity = resident_capacity(reinterpret_cast<const void*>(k_qkv_attn<P, RT, U, DH>));
  const int wgs = g.n_rows / (16 * RT);
  if (wgs > capacity) return hipSuccess;          // not all resident at once: the caller launches the two kernels
  hipLaunchKernelGGL((k_qkv_attn<P, RT, U, DH>), dim3(wgs), dim3(512), 0, s, g, a, ready, abort_word, safe_end, limit);
  *launched = true;
  return hipGetLastError();
}

// Sets *launched and enqueues the fused launch when the shape allows it; otherwise leaves *launched false and does
// nothing (the caller then launches the QKV projection and the attention separately).  a.split_len / a.n_splits are
// chosen here.
hipError_t launch_qkv_attn(const GemmArgs& g0, const AttnArgs& a0, int* ready, unsigned* abort_word, int limit, bool* launched, hipStream_t s) {
  *launched = false;
  if (ready == nullptr || abort_word == nullptr) return hipSuccess;
  if (g0.sum != nullptr || g0.nq != g0.nkv || (g0.dh != 64 && g0.dh != 128)) return hipSuccess;
  if (g0.M < 1 || g0.M > 16 || g0.KT < 1 || g0.n_rows != 3 * g0.nq * g0.dh || g0.grp != g0.dh / 32) return hipSuccess;
  if (g0.ssq != nullptr && (g0.n_ssq < 1 || g0.n_ssq > 512)) return hipErrorInvalidValue;
  if (a0.M != g0.M || a0.nq != g0.nq || a0.nkv != g0.nkv || a0.dh != g0.dh || a0.pos0 != g0.pos0 || a0.counters == nullptr) return hipErrorInvalidValue;
  GemmArgs g = g0;
  g.n_split = 1;
  AttnArgs a = a0;
  const int n = g.n_rows, total = a.pos0 + a.M, pt = a.page_tokens;
  const int rt = (n % 64 == 0 && n / 64 >= 200) ? 4 : 2;                 // the row tiles of the stand-alone QKV launch
  const int G = 3 * g.dh / (16 * rt);
  int len = ((total + G - 1) / G + 31) / 32 * 32;
  if (len < ATTN_SPLIT_LEN) len = ATTN_SPLIT_LEN;                        // (the records are sized for ranges of at least this)
  a.split_len = len; a.n_splits = (total + len - 1) / len;
  // positions below safe_end share no 128-byte line with the block's own positions: K rows are 128 bytes or more per
  // position; a V^T row holds the positions of one page, 64 to a line
  const int safe_end = (pt % 64 == 0) ? (a.pos0 & ~63) : (a.pos0 / pt) * pt;
  const bool p1 = g.M <= 8;
  if (g.dh == 128) {
    if (rt == 4) return p1 ? launch_qkv_attn_cfg<1, 4, 128>(g, a, ready, abort_word, safe_end, limit, launched, s) : launch_qkv_attn_cfg<2, 4, 128>(g, a, ready, abort_word, safe_end, limit, launched, s);
    return p1 ? launch_qkv_attn_cfg<1, 2, 128>(g, a, ready, abort_word, safe_end, limit, launched, s) : launch_qkv_attn_cfg<2, 2, 128>(g, a, ready, abort_word, safe_end, limit, launched, s);
  }
  if (rt == 4) return p1 ? launch_qkv_attn_cfg<1, 4, 64>(g, a, ready, abort_word, safe_end, limit, launched, s) : launch_qkv_attn_cfg<2, 4, 64>(g, a, ready, abort_word, safe_end, limit, launched, s);
  return p1 ? launch_qkv_attn_cfg<1, 2, 64>(g, a, ready, abort_word, safe_end, limit, launched, s) : launch_qkv_attn_cfg<2, 2, 64>(g, a, ready, abort_word, safe_end, limit, launched, s);
}


// ---------------------------------------------------------------------------------------------
// one launch per forward or per draft loop: persistent workgroups, phases separated by a grid barrier
// ---------------------------------------------------------------------------------------------
//
// A forward of the RMSNorm / rotary / SwiGLU family is a chain of phases (per layer: QKV projection, attention,
// O-projection, gate/up, down; then the LM head), each of which needs everything the phase before it wrote.
// Launched one kernel per phase, every boundary costs a ramp (first weight bytes arrive 2 - 3 us after the
// launch) on top of the phase's own tail.  Here one cooperative launch of one workgroup per compute unit runs
// all phases; a workgroup's share of a phase is fixed by its index, so at the end of a phase it knows which
// weight tiles it will need first in the next one and requests them BEFORE it waits at the grid barrier: the
// weight stream of phase i + 1 is in flight while phase i drains and the barrier's round trips pass.
//
// Coherence inside the launch: the eight XCDs have separate L2s, and an L2-wide write-back / invalidate at
// every barrier costs more than the barrier (measured: 8 - 13 us).  Instead (a) every store that another
// workgroup will read is a write-through store and small hand-off data is read with L2-bypassing loads
// (COH accesses above); (b) what MANY workgroups of a phase read (the activation panels with their sums of
// squares, the queries) is given a fresh address per phase ("versions"), so no L2 can hold an older copy
// and plain loads are safe and hit in the reader's own L2 after the first touch: L2-bypassing loads of the
// same few lines from every workgroup queue up on a few memory channels.
//
// Grid barrier, two levels: workgroup i adds 1 to the counter of its group i % 16; the workgroup that completes
// a group adds 1 to the top counter; the one that completes the top counter writes the barrier's number into
// the 16 release words, and every workgroup polls only the release word of its own group (16 pollers per
// word: with every workgroup polling every counter, the polls of 256 workgroups queue up on a few memory
// channels and the workgroups leave the barrier microseconds apart).  All words are 256 bytes apart.  The
// host zeroes them before the launch.  Every wait is bounded: after BAR_SPIN_LIMIT polls the workgroup
// sets the abort word, every later barrier falls through at once, and the launch drains with unusable
// results (the arg-max and loop-finish kernels turn a set abort word into -1 outputs).

constexpr int BAR_GROUPS = 16;
constexpr int BAR_SLOT = 64;                 // ints between two words (256 bytes)
constexpr int BAR_TOP = BAR_GROUPS;          // word index (in slots) of the top counter
constexpr int BAR_RELEASE = BAR_GROUPS + 1;  // first release word
constexpr int BAR_ABORT = 2 * BAR_GROUPS + 1;
constexpr int BAR_SPIN_LIMIT = 1 << 20;      // polls (each a memory round trip, about 1 us) before giving up

// n = number of this barrier (1, 2, ..), per_group = workgroups per group
__device__ __forceinline__ void bar_arrive(unsigned* bar, const unsigned n, const unsigned per_group) {
  __builtin_amdgcn_s_waitcnt(0);             // this wavefront's hand-off stores have completed
  __builtin_amdgcn_s_barrier();              // ... and those of the whole workgroup
  if (threadIdx.x == 0) {
    const unsigned old = __hip_atomic_fetch_add(bar + (blockIdx.x % BAR_GROUPS) * BAR_SLOT, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == n * per_group) {
      const unsigned old_top = __hip_atomic_fetch_add(bar + BAR_TOP * BAR_SLOT, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old_top + 1 == n * BAR_GROUPS) {
#pragma unroll
        for (int g = 0; g < BAR_GROUPS; ++g)
          __hip_atomic_store(bar + (BAR_RELEASE + g) * BAR_SLOT, n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  asm volatile("" ::: "memory");
}

__device__ __forceinline__ void bar_wait(unsigned* bar, const unsigned n) {
  if (threadIdx.x == 0) {
    unsigned* rel = bar + (BAR_RELEASE + blockIdx.x % BAR_GROUPS) * BAR_SLOT;
    unsigned* abort_word = bar + BAR_ABORT * BAR_SLOT;
    int spins = 0;
    while ((int)(__hip_atomic_load(rel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - n) < 0) {
      ++spins;
      if ((spins & 255) == 0 && __hip_atomic_load(abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
      if (spins > BAR_SPIN_LIMIT) {
        __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
  }
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Row tiles per work unit of the four GEMM kinds, by model class (chosen so that a phase has about one unit
// per compute unit): wide models and narrow ones.
struct FwdBig { static constexpr int QKV = 4, PART = 4, UP = 8, LM = 8; };
struct FwdSmall { static constexpr int QKV = 2, PART = 1, UP = 2, LM = 8; };

// LDS of the persistent kernel: one arena, every phase lays its own structure over it (the phases are
// separate functions, so that each gets its own register allocation).
constexpr int FWD_SMEM_BYTES = 68 * 1024;
__shared__ __align__(16) unsigned char g_fwd_smem[FWD_SMEM_BYTES];
template <typename T> __device__ __forceinline__ T& fwd_smem() {
  static_assert(sizeof(T) <= FWD_SMEM_BYTES, "phase structure larger than the arena");
  return *reinterpret_cast<T*>(g_fwd_smem);
}

// The launch's arguments stay in the kernel-argument segment; the phase functions read them through this
// pointer (scalar loads).
typedef const FwdArgs __attribute__((address_space(4)))* FwdArgsPtr;

// What a phase function needs beyond the launch's arguments.
struct FwdCtx { FwdArgsPtr f; int step, l, M, pos0; unsigned bar_n; };   // bar_n: number of the barrier that ends the phase before (0: none)

struct FwdWaitHook {
  unsigned* bar; unsigned n;
  __device__ __forceinline__ void operator()() const { if (n != 0u) bar_wait(bar, n); }
};

__device__ __forceinline__ GemmArgs fwd_base_args(FwdArgsPtr f, const int M) {
  GemmArgs g{};
  g.M = M; g.n_split = 1; g.grp = 1; g.planes = f->planes; g.counters = f->gemm_counters; g.only_row = -1;
  return g;
}
// the sums of squares of a panel version follow its two panels
__device__ __forceinline__ float* fwd_ssq_of(FwdArgsPtr f, const bf16_t* xn_version) {
  return reinterpret_cast<float*>(const_cast<bf16_t*>(xn_version) + (size_t)32 * f->d);
}
__device__ __forceinline__ void fwd_normed_input(FwdArgsPtr f, GemmArgs& g, const bf16_t* x) {
  g.X = x; g.KT = f->d >> 5; g.ssq = fwd_ssq_of(f, x); g.n_ssq = f->d >> 4; g.d_in = f->d; g.eps = f->eps;
}
__device__ __forceinline__ void fwd_residual(FwdArgsPtr f, GemmArgs& g, const bf16_t* w, const bf16_t* x, const int k, const int split,
                                             const float* next_gain, bf16_t* xout) {
  g.W = w; g.X = x; g.KT = k >> 5; g.n_rows = f->d; g.h = f->h; g.ld_out = f->d; g.n_split = split;
  g.Xout = xout; g.KT_out = f->d >> 5; g.gain = next_gain; g.ssq_out = fwd_ssq_of(f, xout); g.n_ssq_out = f->d >> 4;
}
// panel versions of a step: xn has 2 L + 1 per step, xattn and xact L each
__device__ __forceinline__ bf16_t* fwd_xn(FwdArgsPtr f, const int step, const int v) {
  return f->xn + ((size_t)step * (2 * f->n_layers + 1) + v) * f->xn_stride;
}
__device__ __forceinline__ float* fwd_q(FwdArgsPtr f, const int step, const int l) {
  return f->q + ((size_t)step * f->n_layers + l) * 16 * f->d_q;
}
__device__ __forceinline__ bf16_t* fwd_xattn(FwdArgsPtr f, const int step, const int l) {
  return f->xattn + ((size_t)step * f->n_layers + l) * f->xattn_stride;
}
__device__ __forceinline__ bf16_t* fwd_xact(FwdArgsPtr f, const int step, const int l) {
  return f->xact + ((size_t)step * f->n_layers + l) * f->xact_stride;
}

// One GEMM phase: unit u = (row group u % groups, K range u / groups); workgroup i takes units i, i + G, ...
// Its first unit waits for the phase before (after requesting its first weight tiles); a workgroup without a
// unit just waits.  Ends with the arrival at the phase's own barrier.
template <int P, int RT, int EPI>
__device__ __forceinline__ void fwd_gemm_phase(const FwdCtx& c, const GemmArgs& ga, const int groups) {
  GemmSmem<RT, 8>& sm = fwd_smem<GemmSmem<RT, 8>>();
  const FwdWaitHook hook{c.f->bar, c.bar_n};
  const int n_units = groups * ga.n_split;
  int u = blockIdx.x;
  if (u >= n_units) {
    hook();
  } else {
    bool first = true;
    for (; u < n_units; u += gridDim.x) {
      const int b = u % groups, seg = u / groups;
      const int kt_begin = (int)((int64_t)ga.KT * seg / ga.n_split), kt_end = (int)((int64_t)ga.KT * (seg + 1) / ga.n_split);
      // (inside one launch the buffers filled before the barrier are the only prefetch across it: deeper buffers than the
      //  per-phase launches take with two panels)
      constexpr int U = RT >= 8 ? (P >= 2 ? 2 : 3) : 4;
      if (first) gemm_unit<P, RT, EPI, 8, U, true, FwdWaitHook>(ga, b, kt_begin, kt_end, seg, ga.n_split, sm, hook);
      else gemm_unit<P, RT, EPI, 8, U, true, FwdWaitHook>(ga, b, kt_begin, kt_end, seg, ga.n_split, sm, FwdWaitHook{nullptr, 0u});
      first = false;
    }
  }
  bar_arrive(c.f->bar, c.bar_n + 1, gridDim.x / BAR_GROUPS);
}

#define FWD_PHASE_FN __forceinline__

template <int P, typename C>
__device__ FWD_PHASE_FN void fwd_qkv(const FwdCtx c) {
  FwdArgsPtr f = c.f;
  GemmArgs g = fwd_base_args(f, c.M);
  g.W = f->layers[c.l].wqkv; fwd_normed_input(f, g, fwd_xn(f, c.step, 2 * c.l)); g.n_rows = f->d_qkv;
  g.grp = f->dh >> 5; g.q = fwd_q(f, c.step, c.l); g.ldq = f->d_q; g.nq = f->nq; g.nkv = f->nkv; g.dh = f->dh; g.pos0 = c.pos0;
  g.rope_tab = f->rope; g.kv_layer = f->kv_pages + (size_t)c.l * f->kv_layer_stride; g.page_table = f->page_table;
  g.page_tokens = f->page_tokens;
  fwd_gemm_phase<P, C::QKV, EPI_QKV>(c, g, f->d_qkv / (16 * C::QKV));
}

template <bool LOOP>
__device__ FWD_PHASE_FN void fwd_attn(const FwdCtx c) {
  FwdArgsPtr f = c.f;
  AttnArgs at{};
  at.q = fwd_q(f, c.step, c.l); at.ldq = f->d_q; at.kv_layer = f->kv_pages + (size_t)c.l * f->kv_layer_stride; at.page_table = f->page_table;
  at.page_tokens = f->page_tokens; at.nq = f->nq; at.nkv = f->nkv; at.dh = f->dh; at.M = c.M; at.pos0 = c.pos0;
  at.scale = f->attn_scale; at.part = f->part; at.split_len = f->attn_split_len;
  at.n_splits = (c.pos0 + c.M + f->attn_split_len - 1) / f->attn_split_len;
  at.Xout = fwd_xattn(f, c.step, c.l); at.counters = f->attn_counters;
  FwdWaitHook{f->bar, c.bar_n}();
  const int n_units = f->nq * at.n_splits;
  for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
    const int head = u % f->nq, split = u / f->nq;
    if (f->dh == 128) attn_range<128, 8, true, LOOP>(at, head, split, fwd_smem<AttnSmem<128, 8>>(), 0u);
    else attn_range<64, 8, true, LOOP>(at, head, split, fwd_smem<AttnSmem<64, 8>>(), 0u);
  }
  bar_arrive(f->bar, c.bar_n + 1, gridDim.x / BAR_GROUPS);
}

template <int P, typename C>
__device__ FWD_PHASE_FN void fwd_o(const FwdCtx c) {
  FwdArgsPtr f = c.f;
  GemmArgs g = fwd_base_args(f, c.M);
  fwd_residual(f, g, f->layers[c.l].wo, fwd_xattn(f, c.step, c.l), f->d_q, f->split_o, f->layers[c.l].norm2_g,
               fwd_xn(f, c.step, 2 * c.l + 1));
  fwd_gemm_phase<P, C::PART, EPI_PARTIAL>(c, g, f->d / (16 * C::PART));
}

template <int P, typename C>
__device__ FWD_PHASE_FN void fwd_up(const FwdCtx c) {
  FwdArgsPtr f = c.f;
  GemmArgs g = fwd_base_args(f, c.M);
  g.W = f->layers[c.l].w_in; fwd_normed_input(f, g, fwd_xn(f, c.step, 2 * c.l + 1)); g.n_rows = 2 * f->d_ff;
  g.Xout = fwd_xact(f, c.step, c.l); g.KT_out = f->d_ff >> 5;
  fwd_gemm_phase<P, C::UP, EPI_SWIGLU>(c, g, 2 * f->d_ff / (16 * C::UP));
}

template <int P, typename C>
__device__ FWD_PHASE_FN void fwd_down(const FwdCtx c) {
  FwdArgsPtr f = c.f;
  GemmArgs g = fwd_base_args(f, c.M);
  const bool last = (c.l + 1 == f->n_layers);
  fwd_residual(f, g, f->layers[c.l].w_out, fwd_xact(f, c.step, c.l), f->d_ff, f->split_dn,
               last ? f->normf_g : f->layers[last ? c.l : c.l + 1].norm1_g, fwd_xn(f, c.step, 2 * c.l + 2));
  fwd_gemm_phase<P, C::PART, EPI_PARTIAL>(c, g, f->d / (16 * C::PART));
}

template <int P, typename C>
__device__ FWD_PHASE_FN void fwd_lm(const FwdCtx c) {
  FwdArgsPtr f = c.f;
  GemmArgs g = fwd_base_args(f, c.M);
  g.W = f->wlm; fwd_normed_input(f, g, fwd_xn(f, c.step, 2 * f->n_layers)); g.n_rows = f->vocab;
  g.out = f->logits; g.ld_out = f->vocab; g.only_row = f->only_last ? c.M - 1 : -1;
  fwd_gemm_phase<P, C::LM, EPI_STORE>(c, g, f->vocab / (16 * C::LM));
}

// Draft loop: Eq. 2 features and classifier on the step's logits; the workgroup that finishes them embeds the
// next step's token (row 0 of the residual stream, the first panel version of that step, the sums of squares).
__device__ FWD_PHASE_FN void fwd_classify(const FwdCtx c) {
  FwdArgsPtr f = c.f;
  FwdWaitHook{f->bar, c.bar_n}();
  ClassifyArgs ca{};
  ca.logits = f->clf.logits; ca.vocab = f->clf.vocab; ca.clf_params = f->clf.clf_params; ca.hidden = f->clf.hidden;
  ca.tau = f->clf.tau; ca.token_next = f->clf.token_next; ca.gate = f->clf.gate; ca.sl_count = f->clf.sl_count;
  ca.ppl_threshold = f->clf.ppl_threshold; ca.scratch = f->clf.scratch;
  ca.pos_feature = f->clf.pos_feature + (float)c.step;
  ca.force_halt = (c.step + 1 == f->n_steps && !f->open_end) ? 1 : 0;
  ca.out = reinterpret_cast<ClfOut*>(f->clf.out) + c.step;
  ca.block_slot = f->clf.block_slot + c.step;
  ca.force_token = f->clf.force_token ? f->clf.force_token + c.step : nullptr;
  ca.ref_token = f->clf.ref_token ? f->clf.ref_token + c.step : nullptr;
  const int nb = (f->vocab + 4 * CM_NT - 1) / (4 * CM_NT);
  if ((int)blockIdx.x < nb) {
    const int tok = classify_unit<CM_NT, true>(ca, blockIdx.x, nb, 0u);
    if (tok >= 0 && c.step + 1 < f->n_steps) {
      NormArgs na{};
      na.h = f->h; na.d = f->d; na.M = 1; na.layernorm = 0; na.eps = f->eps; na.g = f->layers[0].norm1_g;
      na.Xout = fwd_xn(f, c.step + 1, 0);
      na.ssq_out = fwd_ssq_of(f, na.Xout); na.n_ssq_out = f->d >> 4; na.tok_emb = f->tok_emb; na.tok_stride = f->tok_stride;
      na.vocab = f->vocab; na.max_pos = 1 << 30;
      __syncthreads();
      norm_row<CM_NT, true>(na, 0, tok, reinterpret_cast<float*>(g_fwd_smem), 0u);
    }
  }
  bar_arrive(f->bar, c.bar_n + 1, gridDim.x / BAR_GROUPS);
}

template <int P, typename C, bool LOOP>
__global__ __launch_bounds__(512) void k_forward(FwdArgs f_by_value) {
  (void)f_by_value;                           // read through the kernel-argument segment (first argument, offset 0)
  FwdArgsPtr f = (FwdArgsPtr)__builtin_amdgcn_kernarg_segment_ptr();
  unsigned epoch = 0;                         // barriers this workgroup has arrived at
  const int n_steps = LOOP ? f->n_steps : 1, n_layers = f->n_layers;
  for (int step = 0; step < n_steps; ++step) {
    FwdCtx c;
    c.f = f; c.step = step;
    c.M = (LOOP && step > 0) ? 1 : f->M;
    c.pos0 = (LOOP && step > 0) ? f->pos0 + f->M + (step - 1) : f->pos0;
    for (int l = 0; l < n_layers; ++l) {
      c.l = l;
      c.bar_n = epoch++; fwd_qkv<P, C>(c);
      c.bar_n = epoch++; fwd_attn<LOOP>(c);
      c.bar_n = epoch++; fwd_o<P, C>(c);
      c.bar_n = epoch++; fwd_up<P, C>(c);
      c.bar_n = epoch++; fwd_down<P, C>(c);
    }
    c.l = 0;
    c.bar_n = epoch++; fwd_lm<P, C>(c);
    if (!LOOP) break;
    c.bar_n = epoch++; fwd_classify(c);
    // every workgroup learns the verdict of the step (the wait also orders the next step behind the embedding)
    bar_wait(f->bar, epoch);
    if (__hip_atomic_load(f->clf.gate, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
  }
}

// Workgroups of the persistent launch: one per compute unit, a multiple of the barrier's counter count; 0 if
// the device cannot hold them all at once (then there is no persistent launch).
template <typename K>
static int forward_grid_for(K kernel) {
  int dev = 0, cus = 0, per_cu = 0, coop = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 512, 0) != hipSuccess || per_cu < 1) return 0;
  return cus / BAR_GROUPS * BAR_GROUPS;
}

template <int P, typename C, bool LOOP>
static hipError_t launch_forward_cfg(const FwdArgs& f0, hipStream_t s) {
  static int grid = -1;                        // per process: the library serves the devices of one kind
  if (grid < 0) grid = forward_grid_for(k_forward<P, C, LOOP>);
  if (grid < BAR_GROUPS) return hipErrorCooperativeLaunchTooLarge;
  FwdArgs f = f0;
  // K ranges of the two residual-update GEMMs: about one work unit per workgroup, at least one k-tile per wavefront
  auto split_for = [&](int k) {
    const int groups = f.d / (16 * C::PART), kt = k >> 5;
    int sp = grid / groups;
    if (sp > kt / 8) sp = kt / 8;
    return sp < 1 ? 1 : (sp > GEMM_MAX_SPLIT ? GEMM_MAX_SPLIT : sp);
  };
  f.split_o = split_for(f.d_q);
  f.split_dn = split_for(f.d_ff);
  // attention ranges: about one (head, range) unit per workgroup, never shorter than the records were sized for
  const int total = f.pos0 + f.M + (LOOP ? f.n_steps - 1 : 0);
  const int target = grid / f.nq < 1 ? 1 : grid / f.nq;
  int len = ((total + target - 1) / target + 31) / 32 * 32;
  f.attn_split_len = len < ATTN_SPLIT_LEN ? ATTN_SPLIT_LEN : len;
  void* params[] = {&f};
  return hipLaunchCooperativeKernel(reinterpret_cast<void*>(k_forward<P, C, LOOP>), dim3(grid), dim3(512), params, 0, s);
}

bool forward_shape_ok(int d, int d_q, int d_qkv, int d_ff, int dh, int vocab, bool big) {
  const int rq = big ? FwdBig::QKV : FwdSmall::QKV, rp = big ? FwdBig::PART : FwdSmall::PART, ru = big ? FwdBig::UP : FwdSmall::UP;
  if (d % (16 * rp) || d_qkv % (16 * rq) || (2 * d_ff) % (16 * ru) || vocab % 128) return false;
  if (d % 32 || d_q % 32 || d_ff % 32) return false;
  if (dh != 64 && dh != 128) return false;
  return true;
}

hipError_t launch_forward(const FwdArgs& f, bool big, bool loop, hipStream_t s) {
  if (f.M < 1 || f.M > 16 || !forward_shape_ok(f.d, f.d_q, f.d_qkv, f.d_ff, f.dh, f.vocab, big)) return hipErrorInvalidValue;
  if (f.layers == nullptr || f.bar == nullptr) return hipErrorInvalidValue;
  if (loop) {
    if (f.M > 8 || f.n_steps < 1 || f.d > 4096 || f.clf.scratch == nullptr || f.clf.gate == nullptr) return hipErrorInvalidValue;
    return big ? launch_forward_cfg<1, FwdBig, true>(f, s) : launch_forward_cfg<1, FwdSmall, true>(f, s);
  }
  if (f.M <= 8) return big ? launch_forward_cfg<1, FwdBig, false>(f, s) : launch_forward_cfg<1, FwdSmall, false>(f, s);
  return big ? launch_forward_cfg<2, FwdBig, false>(f, s) : launch_forward_cfg<2, FwdSmall, false>(f, s);
}

}  // namespace disco
