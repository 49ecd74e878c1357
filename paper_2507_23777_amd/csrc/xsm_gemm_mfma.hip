// Weight-streaming GEMM for the small-M regime on bf16 MFMA (gfx950):
//   Y[m][n] = sum_k A[m][k] * W[n][k],  M = sequences x block rows (a few to ~100).
//
// The weight matrix sits on the MFMA's 16-row "A" side (v_mfma_f32_16x16x32_bf16:
// D[n][m] += W[n][k] A[m][k]), the activation rows on the 16-column side, so no lane
// streams padding from HBM.  Weights are re-laid at load time into fragment order: tile
// (nt, kt) = 16 rows x 32 k is 1 KB, lane l holds row l%16, k (l/16)*8..+8, so one wavefront
// load instruction is one contiguous kilobyte.  One workgroup owns one 16-row tile; its four
// wavefronts split the contraction index and are summed through LDS in a fixed order.  The
// first weight fragments are requested before the activation prologue runs, because they
// do not depend on it.
//
// Prologues: RMSNorm of fp32 rows (optionally gathered by a row index), fp32 rows.
// Epilogues: store, residual add, erf-GELU, rotary + q / cache write (fused QKV),
// decoding-head activation r = g + SiLU(y + b).
//
// Five kernels share the fragment layout and the epilogues; launch_fgemm picks by row count
// and prologue (first match):
//   k_gemm_blk  M > 256, input as bf16 hi/lo operand planes (written by the norm pass in front
//               of it, or by the producing kernel): 128 x 128 (or 64 x 128) register blocks,
//               activations through double-buffered LDS; residual-add projections with the
//               contraction cut into slices whose sum the next norm pass takes in
//   k_gemm_wt   17 <= M <= 256, normalised input, at least 64 column tiles (QKV, FFN-up,
//               unembedding): one 16-row weight tile per workgroup over the whole contraction,
//               operand fragments straight from the norm pass's planes
//   k_gemm_ws   17 <= M <= 256, everything else (the residual-add projections): 64 weight rows
//               x 256 of the contraction index per workgroup, all held in registers from one
//               request; partial products merged by the last workgroup to finish, or left to
//               the next norm pass (fixed order either way)
//   k_gemm_big  M > 32 where none of the above applies (fp32 input, contraction that cannot
//               be cut): row-blocked, weights re-read from the XCD's L2 per row block
//   k_fgemm     M <= 16 on the per-stage path, and the fallback for any shape: one tile per
//               workgroup, whole contraction length, norm fused, up to 64 rows per pass
#include "xsm_device.h"
#include "xsm_internal.h"

namespace xsm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kBigMinM = 32;        // rows above which the row-blocked kernel is used

// ---------------------------------------------------------------------------
// canonical [N][K] -> fragment-ordered tiles.  rope_hd > 0: the first two thirds of the
// rows are q and k of a fused QKV matrix; inside each head the rows of a tile are arranged
// as 8 low dims + their 8 rotary partners (dim + hd/2) so that a tile holds whole pairs.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int qkv_src_row(int nt, int r, int d, int hd) {
  const int tiles_per_sec = d / 16, tiles_per_head = hd / 16;
  const int sec = nt / tiles_per_sec, ts = nt % tiles_per_sec;
  const int h = ts / tiles_per_head, tt = ts % tiles_per_head;
  int dim;
  if (sec < 2) dim = r < 8 ? tt * 8 + r : hd / 2 + tt * 8 + (r - 8);
  else dim = tt * 16 + r;
  return sec * d + h * hd + dim;
}

__global__ void k_tile_weights(const uint16_t* __restrict__ W, uint4* __restrict__ out, int N, int K,
                               int rope_d, int rope_hd) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;       // one 16-byte fragment piece
  const int KT = K / 32;
  if (idx >= (long)(N / 16) * KT * 64) return;
  const int lane = (int)(idx & 63);
  const int kt = (int)((idx >> 6) % KT), nt = (int)((idx >> 6) / KT);
  const int r = lane & 15, g = lane >> 4;
  const int row = rope_hd > 0 ? qkv_src_row(nt, r, rope_d, rope_hd) : nt * 16 + r;
  out[idx] = *reinterpret_cast<const uint4*>(W + (size_t)row * K + kt * 32 + g * 8);
}
void launch_tile_weights(const void* W, void* out, int N, int K, int rope_d, int rope_hd,
                         hipStream_t s) {
  TraceScope trace_("tile_weights", s);
  const long n = (long)(N / 16) * (K / 32) * 64;
  hipLaunchKernelGGL(k_tile_weights, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                     (const uint16_t*)W, (uint4*)out, N, K, rope_d, rope_hd);
}

__global__ void k_copy_u16(const uint16_t* src, uint16_t* dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
void launch_copy_u16(const void* src, void* dst, int n, hipStream_t s) {
  hipLaunchKernelGGL(k_copy_u16, dim3((n + 255) / 256), dim3(256), 0, s, (const uint16_t*)src,
                     (uint16_t*)dst, n);
}

// ---------------------------------------------------------------------------
// the GEMM
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_erf_f(float x) {
  return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f));
}
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) { return f2bf_pair(a, b); }
// An fp32 activation enters the bf16 MFMA as two operands, hi = bf16(x) and lo = bf16(x - hi),
// multiplied against the same weight fragment: the activation keeps ~16 mantissa bits, so what
// is left of the bf16 format in a projection is the weights' own rounding (which the model
// definition shares).  At these M the second MFMA is free.
// shared epilogue of the fused QKV projection for one element: rotary pair (v, partner), then
// q to the fp32 query buffer, k / v to the bf16 cache
__device__ __forceinline__ void qkv_store(const FastGemm& g, int nt, int nrow, int m, float v, float partner) {
  const int b = m / g.R, j = m % g.R;
  const int len = g.eff_len[b];
  if (len < 0) return;
  const int d = g.H * g.hd, tps = d / 16, tph = g.hd / 16, half = g.hd / 2;
  const int sec = nt / tps, ts = nt % tps, h = ts / tph, tt = ts % tph;
  const int pos = len + j;
  int dim;
  float o = v;
  if (sec < 2) {
    const int pi = tt * 8 + (nrow & 7);
    const float2 cs = g.rope[(size_t)pos * half + pi];
    if (nrow < 8) { dim = pi; o = v * cs.x - partner * cs.y; }
    else { dim = half + pi; o = partner * cs.y + v * cs.x; }
  } else {
    dim = tt * 16 + nrow;
  }
  const size_t head = (size_t)g.slot[b] * g.H + h;
  if (sec == 0) g.Y[(size_t)m * g.ldy + h * g.hd + dim] = o;
  else if (sec == 1) g.Kc[(head * g.cap + pos) * g.hd + dim] = f2bf(o);
  else if (g.v_transposed) g.Vc[(head * g.hd + dim) * g.cap + pos] = f2bf(o);
  else g.Vc[(head * g.cap + pos) * g.hd + dim] = f2bf(o);
}

template <int PRO, int EPI, int MT>
__global__ __launch_bounds__(256) void k_fgemm(const FastGemm g) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int KC = g.KC, stride = KC + 8;                 // LDS row stride in bf16 elements
  const size_t plane = (size_t)16 * MT * stride;        // hi plane, then lo plane
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);
  float* red = reinterpret_cast<float*>(smem + 2 * plane * 2);
  float* srms = red + 4 * MT * 256;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nt = blockIdx.x, KT = g.K / 32;
  const uint4* wbase = g.Wt + (size_t)nt * KT * 64 + lane;

  for (int m0 = 0; m0 < g.M; m0 += 16 * MT) {
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int kc0 = 0; kc0 < g.K; kc0 += KC) {
      const int kc = min(KC, g.K - kc0), ktc = kc / 32;
      const int per = (ktc + 3) >> 2;
      const int kt_lo = kc0 / 32 + wave * per;
      const int kt_hi = min(kc0 / 32 + ktc, kt_lo + per);
      uint4 wa[8], wb[8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (kt_lo + i < kt_hi) wa[i] = wbase[(size_t)(kt_lo + i) * 64];

      __syncthreads();                                   // earlier readers of As / srms are done
      if (PRO == PRO_NORM && kc0 == 0) {                 // row scales over the full contraction length
        for (int r = wave; r < 16 * MT; r += 4) {
          const int m = m0 + r;
          float ss = 0.f;
          if (m < g.M) {
            const float* x = g.X + (size_t)(g.row_index ? g.row_index[m] : m) * g.ldx;
            for (int c = lane * 4; c < g.K; c += 256) {
              const float4 v = *reinterpret_cast<const float4*>(x + c);
              ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            }
          }
          ss = wave_sum(ss);
          if (lane == 0) srms[r] = 1.0f / sqrtf(ss / (float)g.K + g.eps);
        }
        __syncthreads();
      }
      // stage the activation chunk as bf16 hi / lo planes
      for (int r = wave; r < 16 * MT; r += 4) {
        const int m = m0 + r;
        uint16_t* dst = As + (size_t)r * stride;
        if (m >= g.M) {
          for (int c = lane * 4; c < kc; c += 256) {
            *reinterpret_cast<uint2*>(dst + c) = uint2{0, 0};
            *reinterpret_cast<uint2*>(dst + plane + c) = uint2{0, 0};
          }
        } else {
          const float* x = g.X + (size_t)(g.row_index ? g.row_index[m] : m) * g.ldx + kc0;
          const float sc = PRO == PRO_NORM ? srms[r] : 1.0f;
          for (int c = lane * 4; c < kc; c += 256) {
            float4 v = *reinterpret_cast<const float4*>(x + c);
            if (PRO == PRO_NORM) {
              const uint2 gg = *reinterpret_cast<const uint2*>(g.gain + kc0 + c);
              v.x *= sc * __uint_as_float(gg.x << 16); v.y *= sc * __uint_as_float(gg.x & 0xFFFF0000u);
              v.z *= sc * __uint_as_float(gg.y << 16); v.w *= sc * __uint_as_float(gg.y & 0xFFFF0000u);
            }
            uint2 hi, lo;
            split4(v, hi, lo);
            *reinterpret_cast<uint2*>(dst + c) = hi;
            *reinterpret_cast<uint2*>(dst + plane + c) = lo;
          }
        }
      }
      __syncthreads();

      const uint16_t* arow = As + (size_t)(lane & 15) * stride + (lane >> 4) * 8;
      auto mac = [&](const uint4& wfrag, int kt) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, wfrag);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const uint16_t* bp = arow + (size_t)mt * 16 * stride + (kt * 32 - kc0);
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              a, __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp)), acc[mt], 0, 0, 0);
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              a, __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp + plane)), acc[mt], 0, 0, 0);
        }
      };
      for (int kt = kt_lo; kt < kt_hi; kt += 16) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (kt + 8 + i < kt_hi) wb[i] = wbase[(size_t)(kt + 8 + i) * 64];
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (kt + i < kt_hi) mac(wa[i], kt + i);
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (kt + 16 + i < kt_hi) wa[i] = wbase[(size_t)(kt + 16 + i) * 64];
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (kt + 8 + i < kt_hi) mac(wb[i], kt + 8 + i);
      }
    }

    // sum the four wavefronts' partial tiles in a fixed order
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      *reinterpret_cast<f32x4*>(red + ((size_t)(wave * MT + mt) * 64 + lane) * 4) = acc[mt];
    __syncthreads();
    const int li = lane, ii = wave;                       // this thread finishes D[nrow][mcol]
    const int nrow = (li >> 4) * 4 + ii, mcol = li & 15;
    const int n = nt * 16 + nrow;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) v += red[((size_t)(w * MT + mt) * 64 + li) * 4 + ii];
      const int m = m0 + mt * 16 + mcol;
      if (EPI == FEPI_QKV) {
        const float partner = lane_xor<32>(v);    // row nrow +- 8 of the same tile
        if (m < g.M) qkv_store(g, nt, nrow, m, v, partner);
      } else if (m < g.M) {
        if (EPI == FEPI_STORE) g.Y[(size_t)m * g.ldy + n] = v;
        else if (EPI == FEPI_ADD) g.Y[(size_t)m * g.ldy + n] += v;
        else if (EPI == FEPI_GELU) g.Y[(size_t)m * g.ldy + n] = gelu_erf_f(v);
        else if (EPI == FEPI_HEAD) {
          // n = k*d + c: head k, column c; r = g + SiLU(y + b_k[c]) with g the normalised row
          const int c = n % g.K;
          const float pre = v + bf2f(g.bias[n]);
          const float x = g.X[(size_t)(g.row_index ? g.row_index[m] : m) * g.ldx + c];
          const float gn = x * bf2f(g.gain[c]) * srms[mt * 16 + mcol];
          g.Y[(size_t)m * g.ldy + n] = gn + pre / (1.0f + __expf(-pre));
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Larger M (tens to a thousand rows): two 16-row weight tiles x 64 or 128 activation rows per
// workgroup, activations staged through LDS (hi / lo planes) in 128-wide slices of the
// contraction index and shared by the four wavefronts, weight fragments streamed from global
// memory (HBM once, then the XCD's L2: all row blocks of one weight tile pair are placed on the
// same XCD).  RMSNorm is done once per row by k_norm_rows instead of once per workgroup.
// ---------------------------------------------------------------------------
// normalised row piece (4 consecutive columns from c, c % 4 == 0) -> fp32 row of out, or (split) the planes
__device__ __forceinline__ void norm_out(float* out, bool split, int M, int m, int K, int c, float4 v) {
  if (!split) {
    *reinterpret_cast<float4*>(out + (size_t)m * K + c) = v;
  } else {
    plane_store4(out, M, K, m, c, v);
  }
}

__global__ __launch_bounds__(256) void k_norm_rows(const float* X, int ldx, const int32_t* row_index,
                                                   const uint16_t* gain, float eps, float* out, int K, int split) {
  __shared__ float red[8];
  const int m = blockIdx.x;
  const float* x = X + (size_t)(row_index ? row_index[m] : m) * ldx;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < K; c += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(x + c);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)K + eps);
  for (int c = threadIdx.x * 4; c < K; c += 1024) {
    float4 v = *reinterpret_cast<const float4*>(x + c);
    const uint2 gg = *reinterpret_cast<const uint2*>(gain + c);
    v.x *= inv * __uint_as_float(gg.x << 16); v.y *= inv * __uint_as_float(gg.x & 0xFFFF0000u);
    v.z *= inv * __uint_as_float(gg.y << 16); v.w *= inv * __uint_as_float(gg.y & 0xFFFF0000u);
    norm_out(out, split != 0, gridDim.x, m, K, c, v);
  }
}

constexpr int kBigKC = 128;

// MTW: 16-row activation tiles per wavefront; a workgroup covers BM = 32*MTW rows
// (two wavefronts per weight tile, each taking half of the rows) and two weight tiles.
template <int EPI, int MTW>
__global__ __launch_bounds__(256) void k_gemm_big(const FastGemm g) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int ST = kBigKC + 8, BM = 32 * MTW;
  constexpr int NPF = BM * (kBigKC / 4) / 256;          // float4 pieces of one slice per thread
  constexpr int PLANE = BM * ST;
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int KT = g.K / 32;
  const int MB = (g.M + BM - 1) / BM;
  // workgroup ids go round-robin over the 8 XCDs: keep the row blocks of one weight tile pair together
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int nb = xcd + 8 * (q / MB), mb = q % MB;
  const int nt = nb * 2 + (wave >> 1);                  // this wavefront's 16-row weight tile
  const int mh = wave & 1;                              // its half of the rows
  const int m0 = mb * BM;
  const uint4* wbase = g.Wt + (size_t)nt * KT * 64 + lane;
  f32x4 acc[MTW];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // software pipeline: the next slice's weight fragments and activation pieces are in
  // registers while the current slice is multiplied out of LDS
  uint4 wa[4];
  float4 ap[NPF];
  auto fetch = [&](int kc0) {
    const int kc = min(kBigKC, g.K - kc0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i * 32 < kc) wa[i] = wbase[(size_t)(kc0 / 32 + i) * 64];
#pragma unroll
    for (int p = 0; p < NPF; ++p) {
      const int idx = tid + 256 * p, row = idx / (kBigKC / 4), c4 = idx % (kBigKC / 4);
      ap[p] = float4{0.f, 0.f, 0.f, 0.f};
      if (m0 + row < g.M && c4 * 4 < kc)
        ap[p] = *reinterpret_cast<const float4*>(g.X + (size_t)(m0 + row) * g.ldx + kc0 + c4 * 4);
    }
  };
  fetch(0);
  for (int kc0 = 0; kc0 < g.K; kc0 += kBigKC) {
    const int kc = min(kBigKC, g.K - kc0);
    __syncthreads();                                     // previous slice fully consumed
#pragma unroll
    for (int p = 0; p < NPF; ++p) {
      const int idx = tid + 256 * p, row = idx / (kBigKC / 4), c4 = idx % (kBigKC / 4);
      uint2 hi, lo;
      split4(ap[p], hi, lo);
      *reinterpret_cast<uint2*>(As + (size_t)row * ST + c4 * 4) = hi;
      *reinterpret_cast<uint2*>(As + PLANE + (size_t)row * ST + c4 * 4) = lo;
    }
    uint4 wc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) wc[i] = wa[i];
    __syncthreads();
    if (kc0 + kBigKC < g.K) fetch(kc0 + kBigKC);
    const uint16_t* arow = As + (size_t)(mh * 16 * MTW + (lane & 15)) * ST + (lane >> 4) * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i * 32 < kc) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, wc[i]);
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
          const uint16_t* bp = arow + (size_t)mt * 16 * ST + i * 32;
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              a, __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp)), acc[mt], 0, 0, 0);
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              a, __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp + PLANE)), acc[mt], 0, 0, 0);
        }
      }
  }

  // lane holds D[n0 + i][m], i = 0..3, n0 = nt*16 + (lane>>4)*4, for each of its row tiles
  const int n0 = nt * 16 + (lane >> 4) * 4;
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt) {
    const int m = m0 + (mh * MTW + mt) * 16 + (lane & 15);
    if (EPI == FEPI_QKV) {
      float pr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) pr[i] = lane_xor<32>(acc[mt][i]);
      if (m < g.M) {
#pragma unroll
        for (int i = 0; i < 4; ++i) qkv_store(g, nt, (lane >> 4) * 4 + i, m, acc[mt][i], pr[i]);
      }
    } else if (m < g.M) {
      const f32x4 v = acc[mt];
      f32x4* y = reinterpret_cast<f32x4*>(g.Y + (size_t)m * g.ldy + n0);
      if (EPI == FEPI_STORE) {
        *y = v;
      } else if (EPI == FEPI_ADD) {
        *y = *y + v;
      } else if (EPI == FEPI_GELU) {
        *y = f32x4{gelu_erf_f(v[0]), gelu_erf_f(v[1]), gelu_erf_f(v[2]), gelu_erf_f(v[3])};
      } else if (EPI == FEPI_HEAD) {
        f32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = n0 + i, c = n % g.K;
          const float pre = v[i] + bf2f(g.bias[n]);
          o[i] = g.X[(size_t)m * g.ldx + c] + pre / (1.0f + __expf(-pre));   // X: normalised rows here
        }
        *y = o;
      }
    }
  }
}

template <int EPI, int MTW>
static void big_launch_t(const FastGemm& g, hipStream_t s) {
  constexpr int BM = 32 * MTW;
  const int MB = (g.M + BM - 1) / BM;
  const size_t lds = (size_t)2 * BM * (kBigKC + 8) * 2;
  auto kfn = k_gemm_big<EPI, MTW>;
  allow_dynamic_lds((const void*)kfn, lds);
  hipLaunchKernelGGL(kfn, dim3((g.N / 32) * MB), dim3(256), lds, s, g);
}
template <int EPI>
static void big_launch(const FastGemm& g, hipStream_t s) {
  // row block: 64 rows when that covers M or is needed to fill the chip, else 128
  const long tiles128 = (long)(g.N / 32) * ((g.M + 127) / 128);
  if (g.M <= 64) big_launch_t<EPI, 2>(g, s);
  else if (g.M > 128 && tiles128 < 512) big_launch_t<EPI, 2>(g, s);
  else big_launch_t<EPI, 4>(g, s);
}

static bool big_gemm(int pro, int epi, FastGemm g, hipStream_t s) {
  if (g.M <= kBigMinM || g.N % 256 != 0 || !g.nscratch) return false;
  if (pro == PRO_NORM) {
    hipLaunchKernelGGL(k_norm_rows, dim3(g.M), dim3(256), 0, s, g.X, g.ldx, g.row_index, g.gain, g.eps,
                       g.nscratch, g.K, 0);
    g.X = g.nscratch; g.ldx = g.K; g.row_index = nullptr;
  }
  switch (epi) {
    case FEPI_STORE: big_launch<FEPI_STORE>(g, s); break;
    case FEPI_ADD: big_launch<FEPI_ADD>(g, s); break;
    case FEPI_GELU: big_launch<FEPI_GELU>(g, s); break;
    case FEPI_QKV: big_launch<FEPI_QKV>(g, s); break;
    case FEPI_HEAD: big_launch<FEPI_HEAD>(g, s); break;
    default: return false;
  }
  return true;
}

// ---------------------------------------------------------------------------
// Mid-size M (17..256 rows).  A weight matrix of a few MB is smaller than what the memory
// system holds in flight, so the only way to stream it at speed is to have it requested all at
// once: every workgroup takes 64 weight rows x 256 of the contraction index (32 KB, eight
// fragments per lane and tile) in one go, the activation slice [M][256] is staged through LDS
// (hi / lo planes) and shared by the four wavefronts (2 weight tiles x 4 row tiles each), and
// the K/256 partial products of an output block are summed in slice order by whichever
// workgroup finishes last, which also applies the epilogue.
// ---------------------------------------------------------------------------
constexpr int kWsKS = 256, kWsBM = 128, kWsST = kWsKS + 8, kWsPlane = kWsBM * kWsST;
constexpr int kWsMaxM = 256;

__device__ __forceinline__ void ws_st2(uint64_t* p, float a, float b) {
  __hip_atomic_store(p, (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}

// Partial products live as contiguous blocks [column group][slice][row][64] so that both sides
// address them as (uniform base) + (one per-thread offset): with dozens of loads in flight the
// address registers, not the data, would otherwise run the register file over.
//
// RED = false (residual-add projections only): the kernel stops after writing its partial
// block; the RMSNorm pass that always follows such a projection adds the slices to the residual
// rows while it reads them anyway (k_norm_rows with a pending sum).

// fused-QKV epilogue for the column pair (n, n + 1) of row m; everything that depends on n only
// is precomputed in QkvCols
struct QkvCols { int sec, h, dim0, pi0; bool low; };
__device__ __forceinline__ QkvCols qkv_cols(const FastGemm& g, int n) {
  const int d = g.H * g.hd, nt = n >> 4, nrow = n & 15;
  const int tps = d / 16, tph = g.hd / 16;
  QkvCols c;
  c.sec = nt / tps;
  const int ts = nt % tps, tt = ts % tph;
  c.h = ts / tph;
  c.low = nrow < 8;
  c.pi0 = tt * 8 + (nrow & 7);
  c.dim0 = c.sec < 2 ? (c.low ? c.pi0 : g.hd / 2 + c.pi0) : tt * 16 + nrow;
  return c;
}
__device__ __forceinline__ void qkv_pair_store(const FastGemm& g, const QkvCols& c, int m, float2 v, float2 partner) {
  const int b = m / g.R, j = m - b * g.R;
  const int len = g.eff_len[b];
  if (len < 0) return;
  const int pos = len + j;
  float2 o = v;
  if (c.sec < 2) {
    const float4 cs = *reinterpret_cast<const float4*>(&g.rope[(size_t)pos * (g.hd / 2) + c.pi0]);   // (cos, sin) x 2
    if (c.low) { o.x = v.x * cs.x - partner.x * cs.y; o.y = v.y * cs.z - partner.y * cs.w; }
    else { o.x = partner.x * cs.y + v.x * cs.x; o.y = partner.y * cs.w + v.y * cs.z; }
  }
  const size_t head = (size_t)g.slot[b] * g.H + c.h;
  if (c.sec == 0) {
    *reinterpret_cast<float2*>(g.Y + (size_t)m * g.ldy + c.h * g.hd + c.dim0) = o;
  } else if (c.sec == 1) {
    *reinterpret_cast<uint32_t*>(g.Kc + (head * g.cap + pos) * g.hd + c.dim0) = pack_bf16(o.x, o.y);
  } else if (g.v_transposed) {
    g.Vc[(head * g.hd + c.dim0) * g.cap + pos] = f2bf(o.x);
    g.Vc[(head * g.hd + c.dim0 + 1) * g.cap + pos] = f2bf(o.y);
  } else {
    *reinterpret_cast<uint32_t*>(g.Vc + (head * g.cap + pos) * g.hd + c.dim0) = pack_bf16(o.x, o.y);
  }
}

template <int EPI, bool RED>
__global__ __launch_bounds__(256) void k_gemm_ws(const FastGemm g) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int sm_last;
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, gq = lane >> 4;
  const int KT = g.K / 32, KSPL = g.K / kWsKS, NG = g.N / 64, total = NG * KSPL;
  // workgroup ids go round-robin over the 8 XCDs; make the workgroups of one slice of the
  // contraction index neighbours on one XCD, whose L2 then holds that activation slice once
  int id = blockIdx.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int ks = id / NG, ng = id % NG;
  const int wn = wave & 1, wm = wave >> 1;            // weight tiles 2wn, 2wn+1; row tiles 4wm..4wm+3
  const int MB = (g.M + kWsBM - 1) / kWsBM;

  // activation pieces (row, 4 columns) p = tid + 256 j, row = tid/64 + 4j: a whole row block
  // (up to 32 pieces per thread) is requested at once, the next block while this one is multiplied
  const unsigned st_off = (unsigned)(tid >> 6) * (unsigned)g.ldx * 4u + (unsigned)(tid & 63) * 16u;
  float4 v[32];
  auto request = [&](int mb) {
    const int m0 = mb * kWsBM, rows = min(kWsBM, g.M - m0);
    const char* xb = reinterpret_cast<const char*>(g.X + (size_t)m0 * g.ldx + ks * kWsKS);
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      v[j] = float4{0.f, 0.f, 0.f, 0.f};
      if (4 * j + (tid >> 6) < rows) v[j] = *reinterpret_cast<const float4*>(xb + (size_t)j * 16 * g.ldx + st_off);
    }
  };
  request(0);
  uint4 wf[2][8];                                      // the workgroup's weights: one request, kept
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint4* wb = g.Wt + ((size_t)(ng * 4 + wn * 2 + t) * KT + ks * (kWsKS / 32)) * 64 + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i) wf[t][i] = wb[(size_t)i * 64];
  }

  const size_t blk = (size_t)g.M * 64;                 // floats of one (column group, slice) block
  float* const part_ng = g.ws_part + (size_t)ng * KSPL * blk;
  for (int mb = 0; mb < MB; ++mb) {
    const int m0 = mb * kWsBM, rows = min(kWsBM, g.M - m0), rows16 = (rows + 15) & ~15;
    __syncthreads();                                   // LDS and sm_last of the previous block are free
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const int row = 4 * j + (tid >> 6);
      if (row < rows16) {
        uint2 hi, lo;
        split4(v[j], hi, lo);
        uint16_t* dst = As + (size_t)row * kWsST + (tid & 63) * 4;
        *reinterpret_cast<uint2*>(dst) = hi;
        *reinterpret_cast<uint2*>(dst + kWsPlane) = lo;
      }
    }
    __syncthreads();
    if (mb + 1 < MB) request(mb + 1);

    f32x4 acc[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[t][q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int mt = wm * 4 + q;
      if (mt * 16 < rows16) {
        const uint16_t* bp = As + (size_t)(mt * 16 + r) * kWsST + gq * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp + i * 32));
          const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp + kWsPlane + i * 32));
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, wf[t][i]);
            acc[t][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc[t][q], 0, 0, 0);
            acc[t][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc[t][q], 0, 0, 0);
          }
        }
      }
    }
    // partial products of this slice: lane holds D[n0 + e][m], e = 0..3
    {
      char* pb = reinterpret_cast<char*>(part_ng + (size_t)ks * blk + (size_t)m0 * 64);
      const unsigned po = ((unsigned)(wm * 64 + r) * 64u + (unsigned)(wn * 32 + gq * 4)) * 4u;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (m0 + (wm * 4 + q) * 16 + r < g.M) {
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            char* dst = pb + (size_t)(q * 16 * 64 + t * 16) * 4 + po;
            if (RED) {
              ws_st2(reinterpret_cast<uint64_t*>(dst), acc[t][q][0], acc[t][q][1]);
              ws_st2(reinterpret_cast<uint64_t*>(dst) + 1, acc[t][q][2], acc[t][q][3]);
            } else {
              *reinterpret_cast<f32x4*>(dst) = acc[t][q];
            }
          }
        }
      }
    }
    if (!RED) continue;
    __builtin_amdgcn_s_waitcnt(0);                     // this workgroup's partial is in memory
    __syncthreads();
    if (tid == 0) {
      uint32_t* tk = g.ws_tickets + ng * MB + mb;
      const uint32_t old = __hip_atomic_fetch_add(tk, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sm_last = old == (uint32_t)(KSPL - 1);
      if (sm_last) __hip_atomic_store(tk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!sm_last) continue;
    // last to arrive: sum the slices in order, finish the block [rows][64 columns]; a thread
    // takes column pairs, sixteen at a time with four slices each in flight
    const int npairs = rows * 32;
    const int n = ng * 64 + (tid & 31) * 2;            // this thread's column pair, the same in every round
    QkvCols qc{};
    if (EPI == FEPI_QKV) qc = qkv_cols(g, n);
    for (int i0 = 0; i0 < npairs; i0 += 256 * 16) {
      float2 sum[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) sum[u] = float2{0.f, 0.f};
      for (int k0 = 0; k0 < KSPL; k0 += 4) {
        uint64_t t[16][4];
        const char* sb = reinterpret_cast<const char*>(part_ng + (size_t)k0 * blk + (size_t)m0 * 64) + (size_t)i0 * 8;
#pragma unroll
        for (int u = 0; u < 16; ++u)
          if (i0 + 256 * u + tid < npairs) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (k0 + j < KSPL)
                t[u][j] = __hip_atomic_load(reinterpret_cast<const uint64_t*>(sb + (size_t)j * blk * 4 + (size_t)u * 2048 + (unsigned)tid * 8u),
                                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
#pragma unroll
        for (int u = 0; u < 16; ++u)
          if (i0 + 256 * u + tid < npairs) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (k0 + j < KSPL) {
                sum[u].x += __uint_as_float((uint32_t)t[u][j]);
                sum[u].y += __uint_as_float((uint32_t)(t[u][j] >> 32));
              }
          }
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int idx = i0 + 256 * u + tid;
        if (idx < npairs) {
          const int m = m0 + (idx >> 5);
          if (EPI == FEPI_QKV) {
            // rows n +- 8 of the same 16-row tile sit four column pairs away
            const float2 partner = float2{__shfl_xor(sum[u].x, 4, WAVE), __shfl_xor(sum[u].y, 4, WAVE)};
            qkv_pair_store(g, qc, m, sum[u], partner);
          } else {
            float2* y = reinterpret_cast<float2*>(g.Y + (size_t)m * g.ldy + n);
            if (EPI == FEPI_STORE) {
              *y = sum[u];
            } else if (EPI == FEPI_ADD) {
              const float2 o = *y;
              *y = float2{o.x + sum[u].x, o.y + sum[u].y};
            } else if (EPI == FEPI_GELU) {
              *y = float2{gelu_erf_f(sum[u].x), gelu_erf_f(sum[u].y)};
            } else if (EPI == FEPI_HEAD) {
              const int c = n % g.K;                     // X: normalised rows here
              const float p0 = sum[u].x + bf2f(g.bias[n]), p1 = sum[u].y + bf2f(g.bias[n + 1]);
              const float2 gn = *reinterpret_cast<const float2*>(g.X + (size_t)m * g.ldx + c);
              *y = float2{gn.x + p0 / (1.0f + __expf(-p0)), gn.y + p1 / (1.0f + __expf(-p1))};
            }
          }
        }
      }
    }
  }
}

// One workgroup per row: adds the pending partial products of a residual-add projection to the
// row (slices in order), writes it back, and (out != nullptr) writes its RMSNorm to out.
__global__ __launch_bounds__(256) void k_norm_rows_pending(float* X, int ldx, const float* part, int kspl, int Mtot,
                                                           const uint16_t* gain, float eps, float* out, int K,
                                                           int split) {
  __shared__ float red[8];
  const int m = blockIdx.x;
  float* x = X + (size_t)m * ldx;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < K; c += 1024) {
    float4 a = *reinterpret_cast<const float4*>(x + c);
    const float* pp = part + ((size_t)(c >> 6) * kspl * Mtot + m) * 64 + (c & 63);
    for (int k0 = 0; k0 < kspl; k0 += 8) {
      float4 t[8];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (k0 + j < kspl) t[j] = *reinterpret_cast<const float4*>(pp + (size_t)(k0 + j) * Mtot * 64);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (k0 + j < kspl) { a.x += t[j].x; a.y += t[j].y; a.z += t[j].z; a.w += t[j].w; }
    }
    *reinterpret_cast<float4*>(x + c) = a;
    ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
  }
  if (!out) return;
  ss = block_sum(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)K + eps);
  for (int c = threadIdx.x * 4; c < K; c += 1024) {
    float4 a = *reinterpret_cast<const float4*>(x + c);       // this thread's own stores
    const uint2 gg = *reinterpret_cast<const uint2*>(gain + c);
    a.x *= inv * __uint_as_float(gg.x << 16); a.y *= inv * __uint_as_float(gg.x & 0xFFFF0000u);
    a.z *= inv * __uint_as_float(gg.y << 16); a.w *= inv * __uint_as_float(gg.y & 0xFFFF0000u);
    norm_out(out, split != 0, gridDim.x, m, K, c, a);
  }
}

void launch_norm_rows(const float* X, int ldx, const int32_t* row_index, const uint16_t* gain, float eps, float* out,
                      int M, int K, hipStream_t s) {
  TraceScope trace_("norm_rows", s);
  hipLaunchKernelGGL(k_norm_rows, dim3(M), dim3(256), 0, s, X, ldx, row_index, gain, eps, out, K, 0);
}

void flush_pending_add(PendingAdd* p, hipStream_t s) {
  if (!p || !p->active) return;
  hipLaunchKernelGGL(k_norm_rows_pending, dim3(p->M), dim3(256), 0, s, p->Y, p->ldy, p->part, p->kspl, p->M, nullptr,
                     0.f, nullptr, p->N, 0);
  p->active = false;
}

bool ws_gemm_shape_ok(int M, int N, int K) {
  return M > 16 && M <= kWsMaxM && K % kWsKS == 0 && K >= 2 * kWsKS && N % 64 == 0;
}
size_t ws_gemm_part_floats(int M, int N, int K) {
  return (size_t)(K / kWsKS) * (size_t)(M < kWsMaxM ? M : kWsMaxM) * N;
}

template <int EPI, bool RED>
static void ws_launch(const FastGemm& g, hipStream_t s) {
  const size_t lds = (size_t)2 * kWsPlane * 2;
  auto kfn = k_gemm_ws<EPI, RED>;
  allow_dynamic_lds((const void*)kfn, lds);
  hipLaunchKernelGGL(kfn, dim3((g.N / 64) * (g.K / kWsKS)), dim3(256), lds, s, g);
}

static bool ws_gemm_usable(const FastGemm& g) {
  return ws_gemm_shape_ok(g.M, g.N, g.K) && g.ws_part && g.ws_tickets && g.nscratch &&
         (size_t)(g.N / 64) * ((g.M + kWsBM - 1) / kWsBM) <= kWsTickets;
}

// the same epilogue for four consecutive tile rows of one activation row (vector stores)
struct QkvRow { int m, pos; size_t head0; bool ok; };
__device__ __forceinline__ QkvRow qkv_row(const FastGemm& g, int m) {
  QkvRow q{m, 0, 0, false};
  if (m < g.M) {
    const int b = m / g.R, j = m - b * g.R;
    const int len = g.eff_len[b];
    if (len >= 0) { q.pos = len + j; q.head0 = (size_t)g.slot[b] * g.H; q.ok = true; }
  }
  return q;
}
// four consecutive tile rows (n..n+3, n a multiple of 4) of row q.m: v and the values 8 tile rows away
__device__ __forceinline__ void qkv_quad_store(const FastGemm& g, const QkvCols& c, const QkvRow& q, f32x4 v, f32x4 partner) {
  if (!q.ok) return;
  f32x4 o = v;
  if (c.sec < 2) {
    const float4* rp = reinterpret_cast<const float4*>(&g.rope[(size_t)q.pos * (g.hd / 2) + c.pi0]);
    const float4 cs0 = rp[0], cs1 = rp[1];             // (cos, sin) of pi0, pi0+1 | pi0+2, pi0+3
    const float co[4] = {cs0.x, cs0.z, cs1.x, cs1.z}, si[4] = {cs0.y, cs0.w, cs1.y, cs1.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = c.low ? v[e] * co[e] - partner[e] * si[e] : partner[e] * si[e] + v[e] * co[e];
  }
  const size_t head = q.head0 + c.h;
  if (c.sec == 0) {
    *reinterpret_cast<f32x4*>(g.Y + (size_t)q.m * g.ldy + c.h * g.hd + c.dim0) = o;
  } else if (c.sec == 1) {
    *reinterpret_cast<uint2*>(g.Kc + (head * g.cap + q.pos) * g.hd + c.dim0) = uint2{pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
  } else if (g.v_transposed) {
#pragma unroll
    for (int e = 0; e < 4; ++e) g.Vc[(head * g.hd + c.dim0 + e) * g.cap + q.pos] = f2bf(o[e]);
  } else {
    *reinterpret_cast<uint2*>(g.Vc + (head * g.cap + q.pos) * g.hd + c.dim0) = uint2{pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
  }
}

// ---------------------------------------------------------------------------
// Same M range, projections whose input is a normalised row block and that have at least 64
// column tiles (QKV, FFN up, unembedding, stacked heads): no split of the contraction index
// across workgroups and no LDS staging.  The norm pass writes the rows as bf16 hi / lo planes;
// one workgroup owns one 16-row weight tile over the whole contraction length (its four
// wavefronts take a quarter each, fragments in registers from one request) and reads the
// MFMA "B" fragments straight from the planes, one contiguous KB per request, 64 rows (four row
// tiles) per pass with the fragments of four k-tiles in flight: the contraction loop is a chain of L2
// round trips, and four tiles x four k-tiles beat eight tiles x two.  The four partial tiles are
// summed through LDS in a fixed order.
// ---------------------------------------------------------------------------
constexpr int kWtMaxKW = 16;                           // k-tiles per wavefront: K <= 2048

// 16-byte load that does not allocate in the compute unit's vector cache (policy bit sc1):
// activation blocks are read once per workgroup out of L2, and going through the vector cache
// more than halves the rate a compute unit sustains on such a stream.  Reads past the end of the
// buffer return zero.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t stream_rsrc(const void* base, size_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 stream_ld16(__amdgpu_buffer_rsrc_t rs, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, 16);
  return uint4{v.x, v.y, v.z, v.w};
}

// k_gemm_wt: finish the 4 columns lg*4.. of weight tile nt for row m (every lane of the wavefront
// calls it: the rotary partner, tile rows +- 8 = fragment lane ^ 32, is held by the thread PX further)
template <int EPI, int PX>
__device__ __forceinline__ void wt_finish(const FastGemm& g, const uint16_t* Bh, size_t lo_off, int nt, int m, int lg, f32x4 v) {
  const int n0 = nt * 16 + lg * 4;
  if (EPI == FEPI_QKV) {
    f32x4 pr;
#pragma unroll
    for (int e = 0; e < 4; ++e) pr[e] = lane_xor<PX>(v[e]);
    qkv_quad_store(g, qkv_cols(g, n0), qkv_row(g, m), v, pr);
  } else if (m < g.M) {
    f32x4* y = reinterpret_cast<f32x4*>(g.Y + (size_t)m * g.ldy + n0);
    if (EPI == FEPI_STORE) {
      *y = v;
    } else if (EPI == FEPI_ADD) {
      *y = *y + v;
    } else if (EPI == FEPI_GELU) {
      *y = f32x4{gelu_erf_f(v[0]), gelu_erf_f(v[1]), gelu_erf_f(v[2]), gelu_erf_f(v[3])};
    } else if (EPI == FEPI_HEAD) {
      f32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int n = n0 + e, c = n % g.K;
        const float pre = v[e] + bf2f(g.bias[n]);
        const size_t pi = plane_index(g.K, m, c);
        const float gn = bf2f(Bh[pi]) + bf2f(Bh[lo_off + pi]);
        o[e] = gn + pre / (1.0f + __expf(-pre));
      }
      *y = o;
    }
  }
}

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_wt(const FastGemm g) {
  __shared__ __align__(16) float red[4][4][64][4];      // [wavefront][row tile][lane][4]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nt = blockIdx.x, KT = g.K / 32, KW = KT / 4;
  const uint16_t* Bh = reinterpret_cast<const uint16_t*>(g.X);          // bf16 hi plane, then lo plane
  const size_t lo_off = plane_elems(g.M, g.K);
  const __amdgpu_buffer_rsrc_t brs = stream_rsrc(Bh, lo_off * 4);

  uint4 wf[kWtMaxKW];
  {
    const uint4* wb = g.Wt + ((size_t)nt * KT + wave * KW) * 64 + lane;
#pragma unroll
    for (int i = 0; i < kWtMaxKW; ++i)
      if (i < KW) wf[i] = wb[(size_t)i * 64];
  }
  for (int m0 = 0; m0 < g.M; m0 += 64) {
    const int ntile = (min(64, g.M - m0) + 15) >> 4;
    const unsigned bp = (unsigned)((((m0 >> 4) * KT + wave * KW) * 64 + lane) * 16);
    f32x4 acc[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint4 b0[4][2], b1[4][2], b2[4][2], b3[4][2];
    auto fetch = [&](uint4 (&b)[4][2], int i) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        if (mt < ntile) {
          const unsigned o = bp + (unsigned)(mt * KT + i) * 1024u;
          b[mt][0] = stream_ld16(brs, o);
          b[mt][1] = stream_ld16(brs, o + (unsigned)lo_off * 2u);
        }
    };
    auto mac = [&](const uint4 (&b)[4][2], const uint4& w) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, w);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        if (mt < ntile) {
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b[mt][1]), acc[mt], 0, 0, 0);
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b[mt][0]), acc[mt], 0, 0, 0);
        }
    };
    fetch(b0, 0);
    if (1 < KW) fetch(b1, 1);
    if (2 < KW) fetch(b2, 2);
#pragma unroll
    for (int i = 0; i < kWtMaxKW; i += 4) {
      if (i < KW) {
        if (i + 3 < KW) fetch(b3, i + 3);
        mac(b0, wf[i]);
        if (i + 1 < KW) {
          if (i + 4 < KW) fetch(b0, i + 4);
          mac(b1, wf[i + 1]);
        }
        if (i + 2 < KW) {
          if (i + 5 < KW) fetch(b1, i + 5);
          mac(b2, wf[i + 2]);
        }
        if (i + 3 < KW) {
          if (i + 6 < KW) fetch(b2, i + 6);
          mac(b3, wf[i + 3]);
        }
      }
    }
    __syncthreads();                                   // red is free (previous pass finished)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
      if (mt < ntile) *reinterpret_cast<f32x4*>(&red[wave][mt][lane][0]) = acc[mt];
    __syncthreads();
    // thread: row tile tid / 64, lane tid % 64 of it
    const int mt = tid >> 6;
    if (mt < ntile) {
      const int ll = tid & 63, lr = ll & 15, lg = ll >> 4;
      f32x4 v = *reinterpret_cast<const f32x4*>(&red[0][mt][ll][0]);
      v += *reinterpret_cast<const f32x4*>(&red[1][mt][ll][0]);
      f32x4 v2 = *reinterpret_cast<const f32x4*>(&red[2][mt][ll][0]);
      v2 += *reinterpret_cast<const f32x4*>(&red[3][mt][ll][0]);
      v += v2;
      wt_finish<EPI, 32>(g, Bh, lo_off, nt, m0 + mt * 16 + lr, lg, v);
    }
  }
}

static bool wt_gemm_usable(int pro, const FastGemm& g) {
  return pro == PRO_NORM && g.M > 16 && g.M <= kWsMaxM && g.N % 16 == 0 && g.N / 16 >= 64 && g.K % 128 == 0 &&
         g.K / 128 <= kWtMaxKW && g.nscratch;
}

template <int EPI>
static void wt_launch(const FastGemm& g, hipStream_t s) {
  hipLaunchKernelGGL(k_gemm_wt<EPI>, dim3(g.N / 16), dim3(256), 0, s, g);
}

// the RMSNorm pass in front of a projection; takes in a pending residual sum when there is one
static void norm_pass(FastGemm& g, int split, hipStream_t s) {
  PendingAdd* pend = g.pend;
  if (pend && pend->active && pend->Y == g.X && pend->M == g.M && pend->N == g.K && !g.row_index) {
    hipLaunchKernelGGL(k_norm_rows_pending, dim3(g.M), dim3(256), 0, s, pend->Y, pend->ldy, pend->part, pend->kspl,
                       pend->M, g.gain, g.eps, g.nscratch, g.K, split);
    pend->active = false;
  } else {
    flush_pending_add(pend, s);
    hipLaunchKernelGGL(k_norm_rows, dim3(g.M), dim3(256), 0, s, g.X, g.ldx, g.row_index, g.gain, g.eps,
                       g.nscratch, g.K, split);
  }
  g.X = g.nscratch; g.ldx = g.K; g.row_index = nullptr;
}

static void wt_gemm(int epi, FastGemm g, hipStream_t s) {
  norm_pass(g, 1, s);
  switch (epi) {
    case FEPI_STORE: wt_launch<FEPI_STORE>(g, s); break;
    case FEPI_GELU: wt_launch<FEPI_GELU>(g, s); break;
    case FEPI_QKV: wt_launch<FEPI_QKV>(g, s); break;
    case FEPI_HEAD: wt_launch<FEPI_HEAD>(g, s); break;
    default: break;
  }
}

// ---------------------------------------------------------------------------
// Large M (more than 256 rows): register-blocked.  A workgroup computes 32 WN weight rows x
// 32 WM activation rows, its four wavefronts 2 x 2 with WN x WM MFMA tiles each (16 accumulator
// tiles at 4 x 4), so every operand fragment feeds four MFMA pairs and LDS reads do not bound the
// kernel.  Weight fragments go from global memory / L2 straight to registers (they are stored in
// fragment order), one stage of 64 k ahead; the normalised rows are staged through double-buffered
// LDS as bf16 hi / lo planes (copied from the norm pass's fragment-ordered planes, one contiguous
// KB per wavefront request), one barrier per stage.  No split of the contraction index; row
// blocks of one weight block run next to each other on one XCD.
// ---------------------------------------------------------------------------
constexpr int kBlkKC = 64, kBlkST = kBlkKC + 8;        // contraction slice per stage, LDS row stride (bf16)
constexpr int kBlkKT = kBlkKC / 32;

// SINGLE: the input is exact in bf16 (one plane, one MFMA per fragment pair)
template <int EPI, int WN, int WM, bool SINGLE>
__global__ __launch_bounds__(256) void k_gemm_blk(const FastGemm g) {
  constexpr int BN = 32 * WN, BM = 32 * WM;
  constexpr int PLANE = BM * kBlkST, BUF = (SINGLE ? 1 : 2) * PLANE;   // hi plane, lo plane; two buffers
  constexpr int NPC = BM * (kBlkKC / 8) / 256;          // 16-byte pieces per thread, plane and stage
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, gq = lane >> 4;
  // FEPI_ADD with g.ksplit > 1: a workgroup contracts one slice of K and stores its partial tile
  const int KS = EPI == FEPI_ADD && g.ksplit > 1 ? g.ksplit : 1;
  const int KT = g.K / 32, NS = g.K / kBlkKC / KS, MBk = (g.M + BM - 1) / BM, total = (g.N / BN) * KS * MBk;
  int id = blockIdx.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  // (consecutive blocks, i.e. one XCD, stay inside one slice: they share its activation columns)
  const int wb = id / MBk, mb = id % MBk, nb = wb % (g.N / BN), ks = wb / (g.N / BN), st0 = ks * NS;
  const int wn = wave & 1, wm = wave >> 1;
  const int nt0 = nb * (BN / 16) + wn * WN, m0 = mb * BM, m_base = m0 + wm * WM * 16;
  const uint4* wbase = g.Wt + (size_t)nt0 * KT * 64 + lane;
  const uint16_t* Bh = reinterpret_cast<const uint16_t*>(g.X);          // bf16 hi plane, then lo plane
  const size_t lo_off = plane_elems(g.M, g.K);

  f32x4 acc[WN][WM];
#pragma unroll
  for (int t = 0; t < WN; ++t)
#pragma unroll
    for (int q = 0; q < WM; ++q) acc[t][q] = f32x4{0.f, 0.f, 0.f, 0.f};

  // staging piece p of a stage: row tile p / 128, k-tile (p / 64) % 2, lane p % 64 of that fragment
  // (one wavefront request = one contiguous KB of a plane); it lands at row, column of the LDS tile
  uint4 wreg[WN][kBlkKT];
  uint4 breg[2 * NPC];
  auto request = [&](int st) {
#pragma unroll
    for (int t = 0; t < WN; ++t)
#pragma unroll
      for (int i = 0; i < kBlkKT; ++i) wreg[t][i] = wbase[((size_t)t * KT + (st0 + st) * kBlkKT + i) * 64];
#pragma unroll
    for (int j = 0; j < NPC; ++j) {
      const int p = tid + 256 * j, mtl = p >> 7, ktl = (p >> 6) & 1;
      breg[2 * j] = uint4{0, 0, 0, 0}; breg[2 * j + 1] = uint4{0, 0, 0, 0};
      if (m0 + mtl * 16 < g.M) {
        const uint16_t* src = Bh + ((size_t)(((m0 >> 4) + mtl) * KT + (st0 + st) * kBlkKT + ktl) * 64 + (p & 63)) * 8;
        breg[2 * j] = *reinterpret_cast<const uint4*>(src);
        if (!SINGLE) breg[2 * j + 1] = *reinterpret_cast<const uint4*>(src + lo_off);
      }
    }
  };
  auto deposit = [&](int buf) {
    uint16_t* dst = As + buf * BUF;
#pragma unroll
    for (int j = 0; j < NPC; ++j) {
      const int p = tid + 256 * j, ln = p & 63;
      const int row = (p >> 7) * 16 + (ln & 15), c8 = ((p >> 6) & 1) * 4 + (ln >> 4);
      *reinterpret_cast<uint4*>(dst + row * kBlkST + c8 * 8) = breg[2 * j];
      if (!SINGLE) *reinterpret_cast<uint4*>(dst + PLANE + row * kBlkST + c8 * 8) = breg[2 * j + 1];
    }
  };
  request(0);
  deposit(0);
  uint4 wcur[WN][kBlkKT];
#pragma unroll
  for (int t = 0; t < WN; ++t)
#pragma unroll
    for (int i = 0; i < kBlkKT; ++i) wcur[t][i] = wreg[t][i];
  __syncthreads();
  for (int st = 0; st < NS; ++st) {
    if (st + 1 < NS) request(st + 1);
    const uint16_t* bp = As + (st & 1) * BUF + (size_t)(wm * WM * 16 + r) * kBlkST + gq * 8;
#pragma unroll
    for (int i = 0; i < kBlkKT; ++i)
#pragma unroll
      for (int q = 0; q < WM; ++q) {
        const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp + q * 16 * kBlkST + i * 32));
        // the two products into one accumulator are kept WN MFMAs apart (a dependent MFMA issued
        // back to back waits out the first one's latency)
        if (!SINGLE) {
          const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bp + PLANE + q * 16 * kBlkST + i * 32));
#pragma unroll
          for (int t = 0; t < WN; ++t)
            acc[t][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wcur[t][i]), bl, acc[t][q], 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < WN; ++t)
          acc[t][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wcur[t][i]), bh, acc[t][q], 0, 0, 0);
      }
    if (st + 1 < NS) {
      deposit((st + 1) & 1);                           // that buffer was last read one stage ago
#pragma unroll
      for (int t = 0; t < WN; ++t)
#pragma unroll
        for (int i = 0; i < kBlkKT; ++i) wcur[t][i] = wreg[t][i];
    }
    __syncthreads();
  }

  // lane holds D[n0 + e][m], e = 0..3, n0 = (nt0 + t)*16 + gq*4, m = m_base + q*16 + r
  if (EPI == FEPI_QKV) {
    QkvRow rows[WM];
#pragma unroll
    for (int q = 0; q < WM; ++q) rows[q] = qkv_row(g, m_base + q * 16 + r);
#pragma unroll
    for (int t = 0; t < WN; ++t) {
      const QkvCols c = qkv_cols(g, (nt0 + t) * 16 + gq * 4);
#pragma unroll
      for (int q = 0; q < WM; ++q) {
        f32x4 pr;
#pragma unroll
        for (int e = 0; e < 4; ++e) pr[e] = lane_xor<32>(acc[t][q][e]);   // tile row +- 8
        qkv_quad_store(g, c, rows[q], acc[t][q], pr);
      }
    }
    return;
  }
#pragma unroll
  for (int q = 0; q < WM; ++q) {
    const int m = m_base + q * 16 + r;
    if (m >= g.M) continue;
#pragma unroll
    for (int t = 0; t < WN; ++t) {
      const int n0 = (nt0 + t) * 16 + gq * 4;
      const f32x4 v = acc[t][q];
      f32x4* y = reinterpret_cast<f32x4*>(g.Y + (size_t)m * g.ldy + n0);
      if (EPI == FEPI_STORE) {
        *y = v;
      } else if (EPI == FEPI_ADD) {
        // slices: partial tile [n / 64][slice][m][64], summed onto the rows in slice order by the
        // RMSNorm pass that follows
        if (KS > 1) *reinterpret_cast<f32x4*>(g.ws_part + (((size_t)(n0 >> 6) * KS + ks) * g.M + m) * 64 + (n0 & 63)) = v;
        else *y = *y + v;
      } else if (EPI == FEPI_GELU) {
        const float4 u = float4{gelu_erf_f(v[0]), gelu_erf_f(v[1]), gelu_erf_f(v[2]), gelu_erf_f(v[3])};
        if (g.y_planes) plane_store4(g.Y, g.M, g.N, m, n0, u);      // operand planes of the next projection
        else *y = f32x4{u.x, u.y, u.z, u.w};
      } else if (EPI == FEPI_HEAD) {
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int n = n0 + e, c = n % g.K;
          const float pre = v[e] + bf2f(g.bias[n]);
          const size_t pi = plane_index(g.K, m, c);
          const float gn = bf2f(Bh[pi]) + bf2f(Bh[lo_off + pi]);
          o[e] = gn + pre / (1.0f + __expf(-pre));
        }
        *y = o;
      }
    }
  }
}

bool fgemm_planes_ok(int M, int N, int K) {
  return M > kWsMaxM && N % 64 == 0 && K % kBlkKC == 0 && plane_elems(M, K) * 4 < (1ull << 31);
}
static bool blk_gemm_usable(int pro, const FastGemm& g) {
  if (g.x_single && pro != PRO_PLANES) return false;
  if (pro == PRO_PLANES) return fgemm_planes_ok(g.M, g.N, g.K);
  return pro == PRO_NORM && g.nscratch && fgemm_planes_ok(g.M, g.N, g.K);
}

// A residual-add projection from operand planes has few output blocks (N = model width): its
// contraction is cut into 2, 4 or 8 slices of at least 512 until 128 x 128 blocks fill the chip.
int blk_add_split(int M, int N, int K) {
  if (!fgemm_planes_ok(M, N, K) || N % 128 != 0) return 1;
  const long blocks128 = (long)(N / 128) * ((M + 127) / 128);
  int ks = 1;
  while (blocks128 * ks < 200 && ks < 8 && K % (ks * 2 * kBlkKC) == 0 && K / (ks * 2) >= 512) ks *= 2;
  return ks;
}
size_t blk_add_part_floats(int Mmax, int N, int K) {
  size_t need = 0;
  for (int M = kWsMaxM + 1; M <= Mmax; ++M) {
    const int ks = blk_add_split(M, N, K);
    if (ks > 1 && (size_t)ks * M * N > need) need = (size_t)ks * M * N;
  }
  return need;
}

template <int EPI, int WN, int WM, bool SINGLE = false>
static void blk_launch_t(const FastGemm& g, hipStream_t s) {
  constexpr int BN = 32 * WN, BM = 32 * WM;
  const size_t lds = (size_t)2 * (SINGLE ? 1 : 2) * BM * kBlkST * 2;
  auto kfn = k_gemm_blk<EPI, WN, WM, SINGLE>;
  allow_dynamic_lds((const void*)kfn, lds);
  const int KS = EPI == FEPI_ADD && g.ksplit > 1 ? g.ksplit : 1;
  hipLaunchKernelGGL(kfn, dim3((g.N / BN) * KS * ((g.M + BM - 1) / BM)), dim3(256), lds, s, g);
}
template <int EPI>
static void blk_launch(const FastGemm& g, hipStream_t s) {
  // 128 x 128 blocks when they fill the chip, else 64 weight rows x 128 activation rows
  const long blocks128 = (long)(g.N / 128) * ((g.M + 127) / 128) * (EPI == FEPI_ADD && g.ksplit > 1 ? g.ksplit : 1);
  const bool big = g.N % 128 == 0 && blocks128 >= 200;
  if (EPI == FEPI_STORE && g.x_single) {
    if (big) blk_launch_t<FEPI_STORE, 4, 4, true>(g, s);
    else blk_launch_t<FEPI_STORE, 2, 4, true>(g, s);
  } else if (big) {
    blk_launch_t<EPI, 4, 4>(g, s);
  } else {
    blk_launch_t<EPI, 2, 4>(g, s);
  }
}

static void blk_gemm(int pro, int epi, FastGemm g, hipStream_t s) {
  if (pro == PRO_NORM) norm_pass(g, 1, s);
  else flush_pending_add(g.pend, s);                   // (input planes come from the producing kernel)
  switch (epi) {
    case FEPI_STORE: blk_launch<FEPI_STORE>(g, s); break;
    case FEPI_GELU: blk_launch<FEPI_GELU>(g, s); break;
    case FEPI_QKV: blk_launch<FEPI_QKV>(g, s); break;
    case FEPI_HEAD: blk_launch<FEPI_HEAD>(g, s); break;
    case FEPI_ADD:
      g.ksplit = pro == PRO_PLANES && g.pend && g.ws_part ? blk_add_split(g.M, g.N, g.K) : 1;
      blk_launch<FEPI_ADD>(g, s);
      if (g.ksplit > 1) *g.pend = PendingAdd{true, g.ws_part, g.ksplit, g.M, g.N, g.Y, g.ldy};
      break;
    default: break;
  }
}

static void ws_gemm(int pro, int epi, FastGemm g, hipStream_t s) {
  PendingAdd* pend = g.pend;
  if (pro == PRO_NORM) norm_pass(g, 0, s);
  else flush_pending_add(pend, s);
  switch (epi) {
    case FEPI_STORE: ws_launch<FEPI_STORE, true>(g, s); break;
    case FEPI_ADD:
      if (pend) {                                      // leave the sum to the RMSNorm pass that follows
        ws_launch<FEPI_ADD, false>(g, s);
        *pend = PendingAdd{true, g.ws_part, g.K / kWsKS, g.M, g.N, g.Y, g.ldy};
      } else {
        ws_launch<FEPI_ADD, true>(g, s);
      }
      break;
    case FEPI_GELU: ws_launch<FEPI_GELU, true>(g, s); break;
    case FEPI_QKV: ws_launch<FEPI_QKV, true>(g, s); break;
    case FEPI_HEAD: ws_launch<FEPI_HEAD, true>(g, s); break;
    default: break;
  }
}

static size_t fgemm_lds(int MT, int KC) {
  return (size_t)2 * 16 * MT * (KC + 8) * 2 + (size_t)4 * MT * 256 * 4 + (size_t)16 * MT * 4;
}

bool fgemm_supported(int N, int K) { return N % 16 == 0 && K % 32 == 0; }

template <int PRO, int EPI>
static void fgemm_launch(FastGemm g, hipStream_t s) {
  const int MT = g.M <= 16 ? 1 : g.M <= 32 ? 2 : 4;
  // largest chunk of the contraction index (multiple of 128) whose staging fits 160 KB of LDS
  const size_t budget = 160 * 1024;
  int KC = g.K;
  while (fgemm_lds(MT, KC) > budget) KC = ((KC / 2) + 127) / 128 * 128;
  g.KC = KC;
  const size_t lds = fgemm_lds(MT, KC);
  const dim3 grid(g.N / 16), blk(256);
#define XSM_FG(MTV)                                                                             \
  {                                                                                             \
    auto kfn = k_fgemm<PRO, EPI, MTV>;                                                          \
    allow_dynamic_lds((const void*)kfn, lds > 64 * 1024 ? budget : lds);                         \
    hipLaunchKernelGGL(kfn, grid, blk, lds, s, g);                                              \
  }
  if (MT == 1) XSM_FG(1) else if (MT == 2) XSM_FG(2) else XSM_FG(4)
#undef XSM_FG
}

bool launch_fgemm(int pro, int epi, const FastGemm& g, hipStream_t s) {
  if (g.M <= 0) return true;
  // operand planes in (PRO_PLANES) or out (y_planes) exist only on the row-blocked kernel
  if ((pro == PRO_PLANES || g.y_planes) && !blk_gemm_usable(pro, g)) return false;
  // (the residual-add projections read fp32 rows and have few column blocks: k_gemm_big is faster there)
  if (blk_gemm_usable(pro, g)) {
    TraceScope trace_("gemm_blk", s);
    blk_gemm(pro, epi, g, s);
    return true;
  }
  if (wt_gemm_usable(pro, g) && epi != FEPI_ADD) {
    TraceScope trace_("gemm_wt", s);
    wt_gemm(epi, g, s);
    return true;
  }
  if (ws_gemm_usable(g)) {
    TraceScope trace_("gemm_ws", s);
    ws_gemm(pro, epi, g, s);
    return true;
  }
  flush_pending_add(g.pend, s);                        // the other kernels read finished rows
  if (g.M > kBigMinM) {
    TraceScope trace_("gemm_big", s);
    if (big_gemm(pro, epi, g, s)) return true;
  }
  TraceScope trace_("fgemm", s);
  if (pro == PRO_NORM && epi == FEPI_QKV) fgemm_launch<PRO_NORM, FEPI_QKV>(g, s);
  else if (pro == PRO_NORM && epi == FEPI_STORE) fgemm_launch<PRO_NORM, FEPI_STORE>(g, s);
  else if (pro == PRO_NORM && epi == FEPI_GELU) fgemm_launch<PRO_NORM, FEPI_GELU>(g, s);
  else if (pro == PRO_NORM && epi == FEPI_HEAD) fgemm_launch<PRO_NORM, FEPI_HEAD>(g, s);
  else if (pro == PRO_F32 && epi == FEPI_ADD) fgemm_launch<PRO_F32, FEPI_ADD>(g, s);
  else if (pro == PRO_F32 && epi == FEPI_STORE) fgemm_launch<PRO_F32, FEPI_STORE>(g, s);
  else return false;
  return true;
}

}  // namespace xsm
