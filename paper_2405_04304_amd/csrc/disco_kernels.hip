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
//   * paged KV: [layer][physical page][K | V][kv head][token in page][d_head] bf16.
#include "disco_internal.h"

namespace disco {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define NEG_BIG (-1.0e30f)

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_to_f32(bf16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even; inputs finite
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ bool gated(const uint32_t* gate) {
  return gate != nullptr && __builtin_nontemporal_load(gate) != 0u;
}

// Store 4 consecutive-k activations of token m into the packed panels as bf16 hi/lo.
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
  *reinterpret_cast<uint2*>(X + off_hi) = make_uint2(hi[0], hi[1]);
  *reinterpret_cast<uint2*>(X + off_lo) = make_uint2(lo[0], lo[1]);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
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
__device__ __forceinline__ VI wave_argmax(VI x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    VI y; y.v = __shfl_xor(x.v, o); y.i = __shfl_xor(x.i, o);
    x = vi_best(x, y);
  }
  return x;
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

constexpr int GEMM_NW = 8;  // wavefronts per workgroup; they split K and reduce through LDS
constexpr int GEMM_U = 4;   // k-tiles in flight per wavefront

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
  union { u32x4 u; bf16x8 b; } c; c.u = v; return c.b;
}

template <int P, int RT, int EPI>
__global__ __launch_bounds__(GEMM_NW * 64) void k_gemm(GemmArgs a) {
  if (gated(a.gate)) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int b = blockIdx.x;
  int rt[RT];
  if (RT == 1) { rt[0] = b; }
  else { rt[0] = (b / a.grp) * (2 * a.grp) + (b % a.grp); rt[RT - 1] = rt[0] + a.grp; }

  f32x4 acc[RT][P];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int p = 0; p < P; ++p) acc[r][p] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int KT = a.KT;
  const u32x4* Wp[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) Wp[r] = reinterpret_cast<const u32x4*>(a.W) + (size_t)rt[r] * KT * 64 + lane;
  const u32x4* Xp = reinterpret_cast<const u32x4*>(a.X) + lane;

  int kt = w;
  for (; kt + (GEMM_U - 1) * GEMM_NW < KT; kt += GEMM_U * GEMM_NW) {
    u32x4 A[GEMM_U][RT], B[GEMM_U][P];
#pragma unroll
    for (int u = 0; u < GEMM_U; ++u) {
      const size_t t = (size_t)(kt + u * GEMM_NW) * 64;
#pragma unroll
      for (int r = 0; r < RT; ++r) A[u][r] = __builtin_nontemporal_load(Wp[r] + t);
#pragma unroll
      for (int p = 0; p < P; ++p) B[u][p] = Xp[(size_t)p * KT * 64 + t];
    }
#pragma unroll
    for (int u = 0; u < GEMM_U; ++u)
#pragma unroll
      for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int p = 0; p < P; ++p)
          acc[r][p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(A[u][r]), as_bf16x8(B[u][p]),
                                                              acc[r][p], 0, 0, 0);
  }
  for (; kt < KT; kt += GEMM_NW) {
    const size_t t = (size_t)kt * 64;
    u32x4 A[RT], B[P];
#pragma unroll
    for (int r = 0; r < RT; ++r) A[r] = __builtin_nontemporal_load(Wp[r] + t);
#pragma unroll
    for (int p = 0; p < P; ++p) B[p] = Xp[(size_t)p * KT * 64 + t];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
      for (int p = 0; p < P; ++p)
        acc[r][p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(A[r]), as_bf16x8(B[p]), acc[r][p], 0, 0, 0);
  }

  // hi + lo: same panel, columns n and n + 8 (P == 1), or two panels (P == 2)
  __shared__ f32x4 red[GEMM_NW][RT][64];
#pragma unroll
  for (int r = 0; r < RT; ++r) {
    f32x4 y;
    if (P == 1) {
#pragma unroll
      for (int v = 0; v < 4; ++v) y[v] = acc[r][0][v] + __shfl_xor(acc[r][0][v], 8);
    } else {
      y = acc[r][0] + acc[r][P - 1];
    }
    red[w][r][lane] = y;
  }
  __syncthreads();
  if (w != 0) return;
  f32x4 y[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) {
    y[r] = red[0][r][lane];
#pragma unroll
    for (int ww = 1; ww < GEMM_NW; ++ww) y[r] += red[ww][r][lane];   // fixed order: deterministic
  }
  const int m = lane & 15, g = lane >> 4;   // token column, 4-row group of the 16x16 result
  if (m >= a.M) return;

  if (EPI == EPI_RESID) {
#pragma unroll
    for (int r = 0; r < RT; ++r) {
      float4* p = reinterpret_cast<float4*>(a.out + (size_t)m * a.ld_out + rt[r] * 16 + 4 * g);
      float4 h = *p;
      h.x += y[r][0]; h.y += y[r][1]; h.z += y[r][2]; h.w += y[r][3];
      *p = h;
    }
  } else if (EPI == EPI_STORE) {
    if (a.only_row >= 0 && m != a.only_row) return;
    const size_t row_off = a.only_row >= 0 ? 0 : (size_t)m * a.ld_out;
#pragma unroll
    for (int r = 0; r < RT; ++r)
      *reinterpret_cast<float4*>(a.out + row_off + rt[r] * 16 + 4 * g) = make_float4(y[r][0], y[r][1], y[r][2], y[r][3]);
  } else if (EPI == EPI_QKV) {
    // two tiles: features c .. c+3 and their rotary partners c + dh/2 .. of one head
    const int n0 = rt[0] * 16 + 4 * g;
    const int head = n0 / a.dh, c = n0 % a.dh, half = a.dh >> 1;
    float lo4[4], hi4[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) { lo4[v] = y[0][v]; hi4[v] = y[RT - 1][v]; }
    const int pos = a.pos0 + m;
    const bool is_v = head >= a.nq + a.nkv;
    if (a.rope && !is_v) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const double inv_freq = exp2(-(2.0 * (double)(c + v) / (double)a.dh) * log2((double)a.rope_base));
        double sn, cs;
        sincos((double)pos * inv_freq, &sn, &cs);
        const float x0 = lo4[v], x1 = hi4[v];
        lo4[v] = x0 * (float)cs - x1 * (float)sn;
        hi4[v] = x1 * (float)cs + x0 * (float)sn;
      }
    }
    if (head < a.nq) {
      float* qp = a.q + (size_t)m * a.ldq + head * a.dh + c;
      *reinterpret_cast<float4*>(qp) = make_float4(lo4[0], lo4[1], lo4[2], lo4[3]);
      *reinterpret_cast<float4*>(qp + half) = make_float4(hi4[0], hi4[1], hi4[2], hi4[3]);
    } else {
      const int sel = is_v ? 1 : 0;
      const int kvh = head - a.nq - sel * a.nkv;
      const int lp = pos / a.page_tokens, off = pos % a.page_tokens;
      const int pp = a.page_table ? a.page_table[lp] : lp;
      bf16_t* dst = a.kv_layer + ((((size_t)pp * 2 + sel) * a.nkv + kvh) * a.page_tokens + off) * a.dh + c;
      uint2 u0, u1;
      u0.x = (uint32_t)f32_to_bf16(lo4[0]) | ((uint32_t)f32_to_bf16(lo4[1]) << 16);
      u0.y = (uint32_t)f32_to_bf16(lo4[2]) | ((uint32_t)f32_to_bf16(lo4[3]) << 16);
      u1.x = (uint32_t)f32_to_bf16(hi4[0]) | ((uint32_t)f32_to_bf16(hi4[1]) << 16);
      u1.y = (uint32_t)f32_to_bf16(hi4[2]) | ((uint32_t)f32_to_bf16(hi4[3]) << 16);
      *reinterpret_cast<uint2*>(dst) = u0;
      *reinterpret_cast<uint2*>(dst + half) = u1;
    }
  } else if (EPI == EPI_SWIGLU) {
    // tile 0 = gate rows, tile 1 = the matching up rows
    const int f = (rt[0] >> 1) * 16 + 4 * g;
    float act[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float gt = y[0][v];
      act[v] = gt / (1.0f + expf(-gt)) * y[RT - 1][v];
    }
    xpack_store4(a.Xout, a.KT_out, a.M, m, f, act);
  } else if (EPI == EPI_GELU) {
#pragma unroll
    for (int r = 0; r < RT; ++r) {
      float act[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) act[v] = 0.5f * y[r][v] * (1.0f + erff(y[r][v] * 0.70710678118654752f));
      xpack_store4(a.Xout, a.KT_out, a.M, m, rt[r] * 16 + 4 * g, act);
    }
  }
}

template <int P, int RT>
static hipError_t launch_gemm_epi(const GemmArgs& a, int epi, int grid, hipStream_t s) {
  const dim3 g(grid), b(GEMM_NW * 64);
  switch (epi) {
    case EPI_RESID: hipLaunchKernelGGL((k_gemm<P, RT, EPI_RESID>), g, b, 0, s, a); break;
    case EPI_STORE: hipLaunchKernelGGL((k_gemm<P, RT, EPI_STORE>), g, b, 0, s, a); break;
    case EPI_GELU: hipLaunchKernelGGL((k_gemm<P, RT, EPI_GELU>), g, b, 0, s, a); break;
    case EPI_QKV:
      if (RT == 2) hipLaunchKernelGGL((k_gemm<P, 2, EPI_QKV>), g, b, 0, s, a); else return hipErrorInvalidValue;
      break;
    case EPI_SWIGLU:
      if (RT == 2) hipLaunchKernelGGL((k_gemm<P, 2, EPI_SWIGLU>), g, b, 0, s, a); else return hipErrorInvalidValue;
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, int epi, hipStream_t s) {
  if (a.M < 1 || a.M > 16 || a.KT < 1 || (a.n_rows & 15)) return hipErrorInvalidValue;
  const bool pair = (epi == EPI_QKV || epi == EPI_SWIGLU);
  // two row tiles per workgroup halve the activation re-reads; keep >= ~2 workgroups per CU
  const bool two = pair || ((a.n_rows % 32 == 0) && (a.n_rows / 32 >= 480));
  if (pair && (a.n_rows % 32)) return hipErrorInvalidValue;
  GemmArgs b = a;
  if (!pair) b.grp = 1;
  const int grid = two ? a.n_rows / 32 : a.n_rows / 16;
  if (a.M <= 8) return two ? launch_gemm_epi<1, 2>(b, epi, grid, s) : launch_gemm_epi<1, 1>(b, epi, grid, s);
  return two ? launch_gemm_epi<2, 2>(b, epi, grid, s) : launch_gemm_epi<2, 1>(b, epi, grid, s);
}

// ---------------------------------------------------------------------------------------------
// (embedding +) LayerNorm / RMSNorm -> packed activation panels
// ---------------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_norm(NormArgs a) {
  if (gated(a.gate)) return;
  __shared__ float red[8];
  const int m = blockIdx.x, t = threadIdx.x, d = a.d;
  float* h = a.h + (size_t)m * d;
  if (a.tokens) {
    int tok = a.tokens[m];
    tok = tok < 0 ? 0 : (tok >= a.vocab ? a.vocab - 1 : tok);
    int pos = a.pos0 + m;
    if (pos >= a.max_pos) pos = a.max_pos - 1;
    const bf16_t* e = a.tok_emb + (size_t)tok * a.tok_stride;
    const bf16_t* pe = a.pos_emb ? a.pos_emb + (size_t)pos * d : nullptr;
    for (int k = t * 4; k < d; k += 1024) {
      const uint2 u = *reinterpret_cast<const uint2*>(e + k);
      float4 v = make_float4(bf16_to_f32(u.x & 0xFFFF), bf16_to_f32(u.x >> 16), bf16_to_f32(u.y & 0xFFFF), bf16_to_f32(u.y >> 16));
      if (pe) {
        const uint2 p = *reinterpret_cast<const uint2*>(pe + k);
        v.x += bf16_to_f32(p.x & 0xFFFF); v.y += bf16_to_f32(p.x >> 16);
        v.z += bf16_to_f32(p.y & 0xFFFF); v.w += bf16_to_f32(p.y >> 16);
      }
      *reinterpret_cast<float4*>(h + k) = v;   // each thread re-reads only what it wrote
    }
  }
  float mean = 0.f;
  if (a.layernorm) {
    float s = 0.f;
    for (int k = t * 4; k < d; k += 1024) { const float4 v = *reinterpret_cast<const float4*>(h + k); s += (v.x + v.y) + (v.z + v.w); }
    mean = block_sum<256>(s, red) / (float)d;
  }
  float ss = 0.f;
  for (int k = t * 4; k < d; k += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(h + k);
    const float x0 = v.x - mean, x1 = v.y - mean, x2 = v.z - mean, x3 = v.w - mean;
    ss += (x0 * x0 + x1 * x1) + (x2 * x2 + x3 * x3);
  }
  const float var = block_sum<256>(ss, red) / (float)d;
  const float rstd = 1.0f / sqrtf(var + a.eps);
  const int KT = d >> 5;
  for (int k = t * 4; k < d; k += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(h + k);
    const float4 g = *reinterpret_cast<const float4*>(a.g + k);
    float o[4] = {(v.x - mean) * rstd * g.x, (v.y - mean) * rstd * g.y, (v.z - mean) * rstd * g.z, (v.w - mean) * rstd * g.w};
    if (a.b) {
      const float4 bb = *reinterpret_cast<const float4*>(a.b + k);
      o[0] += bb.x; o[1] += bb.y; o[2] += bb.z; o[3] += bb.w;
    }
    xpack_store4(a.Xout, KT, a.M, m, k, o);
  }
}

hipError_t launch_norm(const NormArgs& a, hipStream_t s) {
  if (a.M < 1 || a.M > 16 || (a.d & 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_norm, dim3(a.M), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// paged attention: M <= 16 queries of one head against cached positions, causal inside the block
// ---------------------------------------------------------------------------------------------

constexpr int ATTN_CH = 64;  // positions staged in LDS per step

template <int DH>
__global__ __launch_bounds__(256) void k_attn_partial(AttnArgs a) {
  if (gated(a.gate)) return;
  constexpr int LDK = DH + 8;                 // padded row (elements) against LDS bank conflicts
  constexpr int G = 256 / DH;                 // query groups in the P.V phase
  constexpr int MAXQ = (16 + G - 1) / G;
  __shared__ float q_s[16][DH];
  __shared__ __attribute__((aligned(16))) bf16_t k_s[ATTN_CH][LDK];
  __shared__ __attribute__((aligned(16))) bf16_t v_s[ATTN_CH][LDK];
  __shared__ float p_s[16][ATTN_CH];
  __shared__ float m_s[16], l_s[16], al_s[16];

  const int head = blockIdx.x, split = blockIdx.y, t = threadIdx.x;
  const int kvh = head / (a.nq / a.nkv);
  const int total = a.pos0 + a.M;
  const int s0 = split * a.split_len;
  const int s1 = min(s0 + a.split_len, total);

  for (int i = t; i < a.M * DH; i += 256) q_s[i / DH][i % DH] = a.q[(size_t)(i / DH) * a.ldq + head * DH + (i % DH)];
  if (t < 16) { m_s[t] = NEG_BIG; l_s[t] = 0.f; al_s[t] = 1.f; }
  float o[MAXQ];
#pragma unroll
  for (int i = 0; i < MAXQ; ++i) o[i] = 0.f;
  __syncthreads();

  for (int t0 = s0; t0 < s1; t0 += ATTN_CH) {
    const int n_tok = min(ATTN_CH, s1 - t0);
    // stage K and V rows of this chunk
    constexpr int VPR = DH / 8;               // 16-byte vectors per row
    for (int rr = t / VPR; rr < n_tok; rr += 256 / VPR) {
      const int pos = t0 + rr, lp = pos / a.page_tokens, off = pos % a.page_tokens;
      const int pp = a.page_table ? a.page_table[lp] : lp;
      const bf16_t* kp = a.kv_layer + ((((size_t)pp * 2 + 0) * a.nkv + kvh) * a.page_tokens + off) * DH + (t % VPR) * 8;
      const bf16_t* vp = kp + (size_t)a.nkv * a.page_tokens * DH;
      *reinterpret_cast<uint4*>(&k_s[rr][(t % VPR) * 8]) = *reinterpret_cast<const uint4*>(kp);
      *reinterpret_cast<uint4*>(&v_s[rr][(t % VPR) * 8]) = *reinterpret_cast<const uint4*>(vp);
    }
    __syncthreads();
    // scores: thread = (position j, query group)
    {
      const int j = t & 63;
      for (int m = t >> 6; m < a.M; m += 4) {
        float sc = NEG_BIG;
        if (j < n_tok && t0 + j <= a.pos0 + m) {
          float acc = 0.f;
#pragma unroll
          for (int c = 0; c < DH; c += 8) {
            const uint4 kk = *reinterpret_cast<const uint4*>(&k_s[j][c]);
            const float* qq = &q_s[m][c];
            acc += qq[0] * bf16_to_f32(kk.x & 0xFFFF) + qq[1] * bf16_to_f32(kk.x >> 16)
                 + qq[2] * bf16_to_f32(kk.y & 0xFFFF) + qq[3] * bf16_to_f32(kk.y >> 16)
                 + qq[4] * bf16_to_f32(kk.z & 0xFFFF) + qq[5] * bf16_to_f32(kk.z >> 16)
                 + qq[6] * bf16_to_f32(kk.w & 0xFFFF) + qq[7] * bf16_to_f32(kk.w >> 16);
          }
          sc = acc * a.scale;
        }
        p_s[m][j] = sc;
      }
    }
    __syncthreads();
    // running soft-max per query: wavefront w owns queries w, w + 4, ..
    {
      const int lane = t & 63;
      for (int m = t >> 6; m < a.M; m += 4) {
        const float sc = p_s[m][lane];
        const float m_old = m_s[m];
        const float m_new = fmaxf(m_old, wave_max(sc));
        const float e = (sc > 0.5f * NEG_BIG) ? expf(sc - m_new) : 0.f;
        const float sum = wave_sum(e);
        const float alpha = expf(m_old - m_new);
        p_s[m][lane] = e;
        if (lane == 0) { m_s[m] = m_new; l_s[m] = l_s[m] * alpha + sum; al_s[m] = alpha; }
      }
    }
    __syncthreads();
    // o = o * alpha + P . V : thread = (channel c, query group)
    {
      const int c = t % DH, mg = t / DH;
#pragma unroll
      for (int i = 0; i < MAXQ; ++i) {
        const int m = mg + i * G;
        if (m < a.M) {
          float acc = o[i] * al_s[m];
          for (int j = 0; j < n_tok; ++j) acc += p_s[m][j] * bf16_to_f32(v_s[j][c]);
          o[i] = acc;
        }
      }
    }
    __syncthreads();
  }
  // partial record per (head, split, query): o[DH], running max, running sum
  {
    const int c = t % DH, mg = t / DH;
#pragma unroll
    for (int i = 0; i < MAXQ; ++i) {
      const int m = mg + i * G;
      if (m < a.M) {
        float* rec = a.part + (((size_t)head * a.n_splits + split) * 16 + m) * (DH + 2);
        rec[c] = o[i];
        if (c == 0) { rec[DH] = m_s[m]; rec[DH + 1] = l_s[m]; }
      }
    }
  }
}

template <int DH>
__global__ __launch_bounds__(DH / 4) void k_attn_merge(AttnArgs a) {
  if (gated(a.gate)) return;
  const int head = blockIdx.x, m = blockIdx.y, t = threadIdx.x;
  const float* base = a.part + (((size_t)head * a.n_splits) * 16 + m) * (DH + 2);
  const size_t stride = (size_t)16 * (DH + 2);
  float mx = NEG_BIG;
  for (int s = 0; s < a.n_splits; ++s) mx = fmaxf(mx, base[s * stride + DH]);
  float L = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < a.n_splits; ++s) {
    const float* rec = base + s * stride;
    const float wgt = expf(rec[DH] - mx);
    L += rec[DH + 1] * wgt;
    const float4 v = *reinterpret_cast<const float4*>(rec + 4 * t);
    o[0] += v.x * wgt; o[1] += v.y * wgt; o[2] += v.z * wgt; o[3] += v.w * wgt;
  }
  const float inv = 1.0f / L;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] *= inv;
  xpack_store4(a.Xout, (a.nq * DH) >> 5, a.M, m, head * DH + 4 * t, o);
}

hipError_t launch_attn(const AttnArgs& a, hipStream_t s) {
  if (a.M < 1 || a.M > 16 || a.n_splits < 1) return hipErrorInvalidValue;
  const dim3 g1(a.nq, a.n_splits), g2(a.nq, a.M);
  if (a.dh == 128) {
    hipLaunchKernelGGL(k_attn_partial<128>, g1, dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_attn_merge<128>, g2, dim3(32), 0, s, a);
  } else if (a.dh == 64) {
    hipLaunchKernelGGL(k_attn_partial<64>, g1, dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_attn_merge<64>, g2, dim3(16), 0, s, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Eq. 2 in one launch: soft-max top-10, entropy, arg-max -> classifier -> halt decision
// ---------------------------------------------------------------------------------------------

struct ClfOut {  // mirrors disco_clf_out
  int32_t token; float feats[12]; float score; uint32_t halt; uint32_t executed;
};

constexpr int FEAT_NT = 1024;
constexpr int FEAT_CAND = 1024;

__global__ __launch_bounds__(FEAT_NT) void k_classify(ClassifyArgs a) {
  ClfOut* out = reinterpret_cast<ClfOut*>(a.out);
  if (a.gate != nullptr && *a.gate != 0u) {
    if (threadIdx.x == 0) out->executed = 0u;
    return;
  }
  __shared__ float sv[FEAT_NT / 64 + 1];
  __shared__ int si[FEAT_NT / 64 + 1];
  __shared__ float cand[FEAT_CAND];
  __shared__ int n_cand;
  __shared__ float top_s[10];
  __shared__ float feat_s[12];
  const int t = threadIdx.x, V = a.vocab;
  const float* x = a.logits;

  // pass 1: maximum and arg-max (lowest index on ties); also each thread's own maximum
  VI mine; mine.v = -INFINITY; mine.i = 0x7fffffff;
  for (int i = t; i < V; i += FEAT_NT) { VI y; y.v = x[i]; y.i = i; mine = vi_best(mine, y); }
  VI best = block_argmax<FEAT_NT>(mine, sv, si);
  int force = -1;
  if (a.force_token) { force = *a.force_token; if (force >= V) force = -1; }
  float forced_val = 0.f;
  if (force >= 0) {
    forced_val = best.v + 4.0f;
    best.v = forced_val; best.i = force;
    if (t == (force % FEAT_NT)) { mine.v = forced_val; mine.i = force; }
  }
  const float mx = best.v;

  // pass 2: S = sum e^(x - max), T = sum e^(x - max) (x - max)
  float S = 0.f, T = 0.f;
  for (int i = t; i < V; i += FEAT_NT) {
    const float d = ((i == force) ? forced_val : x[i]) - mx;
    const float e = expf(d);
    S += e; T += e * d;
  }
  S = block_sum<FEAT_NT>(S, sv);
  T = block_sum<FEAT_NT>(T, sv);

  // top-10 values.  The 10th largest of the per-thread maxima bounds the 10th largest element from
  // below, so only elements >= that bound can be in the top 10.
  if (t == 0) n_cand = 0;
  float bound = 0.f;
  {
    VI cur = mine; cur.i = t;
    for (int r = 0; r < 10; ++r) {
      const VI b = block_argmax<FEAT_NT>(cur, sv, si);
      bound = b.v;
      if (b.i == t) cur.v = -INFINITY;
    }
  }
  __syncthreads();
  for (int i = t; i < V; i += FEAT_NT) {
    const float v = (i == force) ? forced_val : x[i];
    if (v >= bound) {
      const int slot = atomicAdd(&n_cand, 1);
      if (slot < FEAT_CAND) cand[slot] = v;
    }
  }
  __syncthreads();
  const int nc = n_cand;
  if (nc <= FEAT_CAND) {
    VI cur; cur.v = (t < nc) ? cand[t] : -INFINITY; cur.i = t;
    for (int r = 0; r < 10; ++r) {
      const VI b = block_argmax<FEAT_NT>(cur, sv, si);
      if (t == 0) top_s[r] = b.v;
      if (b.i == t) cur.v = -INFINITY;
    }
  } else {
    // more candidates than the list holds (massive ties): ten full selection rounds, each taking
    // the largest element that comes after the previous pick in (value desc, index asc) order
    VI prev; prev.v = INFINITY; prev.i = -1;
    for (int r = 0; r < 10; ++r) {
      VI c; c.v = -INFINITY; c.i = 0x7fffffff;
      for (int i = t; i < V; i += FEAT_NT) {
        const float v = (i == force) ? forced_val : x[i];
        const bool after = (v < prev.v) || (v == prev.v && i > prev.i);
        if (after) { VI y; y.v = v; y.i = i; c = vi_best(c, y); }
      }
      prev = block_argmax<FEAT_NT>(c, sv, si);
      if (t == 0) top_s[r] = prev.v;
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
    out->token = best.i;
#pragma unroll
    for (int i = 0; i < 12; ++i) out->feats[i] = feat_s[i];
    out->score = score; out->halt = halt; out->executed = 1u;
    if (force >= 0) a.logits[force] = forced_val;
    if (a.token_next) *a.token_next = best.i;
    if (a.block_slot) *a.block_slot = best.i;
    if (a.sl_count) *a.sl_count += 1;
    if (a.gate && halt) *a.gate = 1u;
  }
}

hipError_t launch_classify(const ClassifyArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_classify, dim3(1), dim3(FEAT_NT), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// per-row arg-max of the verification logits; acceptance; KV fill; draft-loop bookkeeping
// ---------------------------------------------------------------------------------------------

__global__ __launch_bounds__(1024) void k_argmax_rows(const float* __restrict__ logits, int vocab, int32_t* __restrict__ out) {
  __shared__ float sv[17];
  __shared__ int si[17];
  const float* x = logits + (size_t)blockIdx.x * vocab;
  VI mine; mine.v = -INFINITY; mine.i = 0x7fffffff;
  for (int i = threadIdx.x; i < vocab; i += 1024) { VI y; y.v = x[i]; y.i = i; mine = vi_best(mine, y); }
  const VI b = block_argmax<1024>(mine, sv, si);
  if (threadIdx.x == 0) out[blockIdx.x] = b.i;
}

hipError_t launch_argmax_rows(const float* logits, int M, int vocab, int32_t* out, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax_rows, dim3(M), dim3(1024), 0, s, logits, vocab, out);
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
    const size_t dst = (((((size_t)layer * n_pages + pp) * 2 + sel) * nkv + kvh) * pt + off) * dh + cv * 8;
    *reinterpret_cast<uint4*>(pages + dst) = *reinterpret_cast<const uint4*>(src + i * 8);
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

struct LoopOut { int32_t sl; int32_t block[16]; };

__global__ void k_loop_init(uint32_t* gate, int32_t* sl_count, const int32_t* tokens_in, int n_in, LoopOut* out) {
  if (threadIdx.x != 0) return;
  *gate = 0u; *sl_count = 0;
  out->sl = 0;
  out->block[0] = tokens_in[n_in - 1];
  for (int i = 1; i < 16; ++i) out->block[i] = 0;
}

__global__ void k_loop_finish(const int32_t* sl_count, LoopOut* out, LoopOut* host_out) {
  if (threadIdx.x != 0) return;
  out->sl = *sl_count;
  if (host_out) { *host_out = *out; __threadfence_system(); }
}

hipError_t launch_loop_init(uint32_t* gate, int32_t* sl_count, const int32_t* tokens_in, int n_in, void* dev_loop_out,
                            hipStream_t s) {
  hipLaunchKernelGGL(k_loop_init, dim3(1), dim3(64), 0, s, gate, sl_count, tokens_in, n_in,
                     reinterpret_cast<LoopOut*>(dev_loop_out));
  return hipGetLastError();
}

hipError_t launch_loop_finish(const int32_t* sl_count, void* dev_loop_out, void* host_loop_out, hipStream_t s) {
  hipLaunchKernelGGL(k_loop_finish, dim3(1), dim3(64), 0, s, sl_count, reinterpret_cast<LoopOut*>(dev_loop_out),
                     reinterpret_cast<LoopOut*>(host_loop_out));
  return hipGetLastError();
}

}  // namespace disco
