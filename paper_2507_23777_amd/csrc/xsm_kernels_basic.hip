// General-shape kernels of the decoder forward: embedding gather, RMSNorm,
// row-streaming GEMM on vector ALUs, rotary embedding + cache write, attention
// with per-thread online softmax.  They accept any shape the configuration
// allows and both storage types; the fp32 model runs entirely on them.
#include "xsm_device.h"
#include "xsm_internal.h"

namespace xsm {

// ---------------------------------------------------------------------------
// rotary table: tab[pos][i] = (cos, sin)(pos * theta^(-2i/hd)), evaluated in fp64
// ---------------------------------------------------------------------------
__global__ void k_rope_table(float2* tab, int max_ctx, int half, int hd, double theta) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)max_ctx * half) return;
  const int pos = (int)(idx / half), i = (int)(idx % half);
  const double freq = pow(theta, -2.0 * (double)i / (double)hd);
  const double ang = (double)pos * freq;
  tab[idx] = make_float2((float)cos(ang), (float)sin(ang));
}
void launch_rope_table(float2* tab, int max_ctx, int head_dim, float theta, hipStream_t s) {
  TraceScope trace_("rope_table", s);
  const long n = (long)max_ctx * (head_dim / 2);
  hipLaunchKernelGGL(k_rope_table, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, tab, max_ctx,
                     head_dim / 2, head_dim, (double)theta);
}

// ---------------------------------------------------------------------------
// per-step input validation
// ---------------------------------------------------------------------------
__global__ void k_prepare(const int32_t* kv_len, const int32_t* slot, const int32_t* block,
                          int n_seq, int R, int vocab, int max_batch, int max_ctx, int bound,
                          int32_t* eff_len, int32_t* slot_out, uint32_t* wflags) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= n_seq) return;
  uint32_t f = 0;
  const int n = kv_len[b], sl = slot[b];
  if (n < 0 || n + R > max_ctx || n > bound) f |= XSM_FLAG_BAD_LEN;
  if (sl < 0 || sl >= max_batch) f |= XSM_FLAG_BAD_SLOT;
  for (int j = 0; j < R; ++j) {
    const int t = block[b * R + j];
    if (t < 0 || t >= vocab) f |= XSM_FLAG_BAD_TOKEN;
  }
  eff_len[b] = f ? -1 : n;
  slot_out[b] = (f & XSM_FLAG_BAD_SLOT) ? 0 : sl;
  wflags[b] = f;
}
void launch_prepare(const int32_t* kv_len, const int32_t* slot, const int32_t* block, int n_seq,
                    int R, int vocab, int max_batch, int max_ctx, int kv_len_bound,
                    int32_t* eff_len, int32_t* slot_out, uint32_t* wflags, hipStream_t s) {
  TraceScope trace_("prepare", s);
  hipLaunchKernelGGL(k_prepare, dim3((n_seq + 63) / 64), dim3(64), 0, s, kv_len, slot, block, n_seq,
                     R, vocab, max_batch, max_ctx, kv_len_bound, eff_len, slot_out, wflags);
}

__global__ void k_fill_i32(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
void launch_fill_i32(int32_t* p, int n, int32_t v, hipStream_t s) {
  TraceScope trace_("fill_i32", s);
  hipLaunchKernelGGL(k_fill_i32, dim3((n + 255) / 256), dim3(256), 0, s, p, n, v);
}

__global__ void k_copy_f32(const float* src, float* dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
void launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s) {
  TraceScope trace_("copy_f32", s);
  if (n == 0) return;
  hipLaunchKernelGGL(k_copy_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, dst, n);
}

// ---------------------------------------------------------------------------
// layer-0 hidden states
// ---------------------------------------------------------------------------
template <typename T>
__global__ void k_embed(const T* E, const int32_t* block, const int32_t* eff_len, float* X, int R,
                        int d) {
  const int m = blockIdx.x, b = m / R;
  const bool live = eff_len[b] >= 0;
  const T* row = E + (size_t)(live ? block[m] : 0) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) X[(size_t)m * d + i] = live ? ldf(row + i) : 0.f;
}
void launch_embed(int dtype, const void* E, const int32_t* block, const int32_t* eff_len, float* X,
                  int n_seq, int R, int d, hipStream_t s) {
  TraceScope trace_("embed", s);
  if (dtype == XSM_BF16)
    hipLaunchKernelGGL(k_embed<bf16_t>, dim3(n_seq * R), dim3(256), 0, s, (const bf16_t*)E, block,
                       eff_len, X, R, d);
  else
    hipLaunchKernelGGL(k_embed<float>, dim3(n_seq * R), dim3(256), 0, s, (const float*)E, block,
                       eff_len, X, R, d);
}

template <typename T>
__global__ void k_load_rows(const T* emb, float* X, int C, int row0, int rows_per_seq, int d) {
  const int m = blockIdx.x, b = m / C, j = m % C;
  const T* row = emb + ((size_t)b * rows_per_seq + row0 + j) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) X[(size_t)m * d + i] = ldf(row + i);
}
void launch_load_rows(int dtype, const void* emb, float* X, int n_seq, int C, int row0,
                      int rows_per_seq, int d, hipStream_t s) {
  TraceScope trace_("load_rows", s);
  if (dtype == XSM_BF16)
    hipLaunchKernelGGL(k_load_rows<bf16_t>, dim3(n_seq * C), dim3(256), 0, s, (const bf16_t*)emb, X,
                       C, row0, rows_per_seq, d);
  else
    hipLaunchKernelGGL(k_load_rows<float>, dim3(n_seq * C), dim3(256), 0, s, (const float*)emb, X,
                       C, row0, rows_per_seq, d);
}

// bf16 input rows as one MFMA operand plane in fragment order (the values are bf16 already, so
// there is no low part): thread = 8 consecutive columns of one row, 16 bytes in and out
__global__ void k_load_rows_plane(const uint16_t* emb, uint16_t* plane, int M, int C, int row0, int rows_per_seq, int d) {
  const int idx = blockIdx.x * 256 + threadIdx.x, per_row = d / 8;
  if (idx >= M * per_row) return;
  const int m = idx / per_row, k = (idx % per_row) * 8, b = m / C, j = m % C;
  const uint4 v = *reinterpret_cast<const uint4*>(emb + ((size_t)b * rows_per_seq + row0 + j) * d + k);
  *reinterpret_cast<uint4*>(plane + plane_index(d, m, k)) = v;
}
void launch_load_rows_plane(const void* emb, void* plane, int n_seq, int C, int row0, int rows_per_seq, int d,
                            hipStream_t s) {
  TraceScope trace_("load_rows", s);
  const int M = n_seq * C, n = M * (d / 8);
  hipLaunchKernelGGL(k_load_rows_plane, dim3((n + 255) / 256), dim3(256), 0, s, (const uint16_t*)emb, (uint16_t*)plane,
                     M, C, row0, rows_per_seq, d);
}

// ---------------------------------------------------------------------------
// RMSNorm: Y = X * g / sqrt(mean(X^2) + eps), one workgroup per row
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const float* X, const T* g, float* Y, int d,
                                                 float eps) {
  __shared__ float red[8];
  const float* x = X + (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) ss += x[i] * x[i];
  ss = block_sum(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) Y[(size_t)blockIdx.x * d + i] = x[i] * ldf(g + i) * inv;
}
void launch_rmsnorm(int dtype, const float* X, const void* gain, float* Y, int M, int d, float eps,
                    hipStream_t s) {
  TraceScope trace_("rmsnorm", s);
  if (dtype == XSM_BF16)
    hipLaunchKernelGGL(k_rmsnorm<bf16_t>, dim3(M), dim3(256), 0, s, X, (const bf16_t*)gain, Y, d, eps);
  else
    hipLaunchKernelGGL(k_rmsnorm<float>, dim3(M), dim3(256), 0, s, X, (const float*)gain, Y, d, eps);
}

// ---------------------------------------------------------------------------
// Row-streaming GEMM: Y[m][n] (op)= sum_k A[m][k] W[n][k].  One wavefront per
// weight row n and 8 activation rows; lanes stride the contraction index with
// 16-byte loads, fixed butterfly reduction.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_rows(const float* __restrict__ A, int lda,
                                                   const T* __restrict__ W, float* Y, int ldy, int M,
                                                   int N, int K) {
  constexpr int VEC = VecOf<T>::n;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + wave;
  const int m0 = blockIdx.y * 8;
  if (n >= N) return;
  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;
  const T* wrow = W + (size_t)n * K;
  for (int k = lane * VEC; k < K; k += 64 * VEC) {
    float wv[VEC];
    ldvec(wrow + k, wv);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int m = m0 + r;
      if (m < M) {
        const float* a = A + (size_t)m * lda + k;
#pragma unroll
        for (int v = 0; v < VEC; v += 4) {
          const float4 av = *reinterpret_cast<const float4*>(a + v);
          acc[r] = fmaf(av.x, wv[v], acc[r]);
          acc[r] = fmaf(av.y, wv[v + 1], acc[r]);
          acc[r] = fmaf(av.z, wv[v + 2], acc[r]);
          acc[r] = fmaf(av.w, wv[v + 3], acc[r]);
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = wave_sum(acc[r]);
  if (lane < 8) {
    const int m = m0 + lane;
    float v = acc[0];
#pragma unroll
    for (int r = 1; r < 8; ++r) v = (lane == r) ? acc[r] : v;
    if (m < M) {
      float* y = Y + (size_t)m * ldy + n;
      if (EPI == EPI_ADD) *y += v;
      else if (EPI == EPI_GELU) *y = gelu_erf(v);
      else *y = v;
    }
  }
}
template <typename T>
static void gemm_dispatch(int epi, const float* A, int lda, const T* W, float* Y, int ldy, int M,
                          int N, int K, hipStream_t s) {
  const dim3 grid((N + 3) / 4, (M + 7) / 8), blk(256);
  if (epi == EPI_ADD)
    hipLaunchKernelGGL((k_gemm_rows<T, EPI_ADD>), grid, blk, 0, s, A, lda, W, Y, ldy, M, N, K);
  else if (epi == EPI_GELU)
    hipLaunchKernelGGL((k_gemm_rows<T, EPI_GELU>), grid, blk, 0, s, A, lda, W, Y, ldy, M, N, K);
  else
    hipLaunchKernelGGL((k_gemm_rows<T, EPI_STORE>), grid, blk, 0, s, A, lda, W, Y, ldy, M, N, K);
}
void launch_gemm(int dtype, int epi, const float* A, int lda, const void* W, float* Y, int ldy,
                 int M, int N, int K, hipStream_t s) {
  TraceScope trace_("gemm", s);
  if (M <= 0) return;
  if (dtype == XSM_BF16) gemm_dispatch<bf16_t>(epi, A, lda, (const bf16_t*)W, Y, ldy, M, N, K, s);
  else gemm_dispatch<float>(epi, A, lda, (const float*)W, Y, ldy, M, N, K, s);
}

// ---------------------------------------------------------------------------
// rotary embedding of q,k and cache write.  One thread per (row, head, pair).
// ---------------------------------------------------------------------------
template <typename T>
__global__ void k_rope_kv(const float* QKV, const float2* rope, const int32_t* eff_len,
                          const int32_t* slot, float* Qr, T* Kc, T* Vc, int n_rows, int R, int H,
                          int hd, int max_ctx) {
  const int half = hd / 2, d = H * hd;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)n_rows * H * half) return;
  const int i = (int)(idx % half), h = (int)((idx / half) % H), m = (int)(idx / ((long)half * H));
  const int b = m / R, j = m % R;
  const int n = eff_len[b];
  if (n < 0) return;
  const int pos = n + j;
  const float2 cs = rope[(size_t)pos * half + i];
  const float* row = QKV + (size_t)m * 3 * d;
  const int c = h * hd + i;
  const float qa = row[c], qb = row[c + half];
  const float ka = row[d + c], kb = row[d + c + half];
  Qr[(size_t)m * d + c] = qa * cs.x - qb * cs.y;
  Qr[(size_t)m * d + c + half] = qa * cs.y + qb * cs.x;
  const size_t base = (((size_t)slot[b] * H + h) * max_ctx + pos) * hd;
  stf(Kc + base + i, ka * cs.x - kb * cs.y);
  stf(Kc + base + i + half, ka * cs.y + kb * cs.x);
  stf(Vc + base + i, row[2 * d + c]);
  stf(Vc + base + i + half, row[2 * d + c + half]);
}
void launch_rope_kv(int dtype, const float* QKV, const float2* rope, const int32_t* eff_len,
                    const int32_t* slot, float* Qr, void* Kc, void* Vc, int n_seq, int R, int H,
                    int hd, int max_ctx, hipStream_t s) {
  TraceScope trace_("rope_kv", s);
  const long n = (long)n_seq * R * H * (hd / 2);
  const dim3 grid((unsigned)((n + 255) / 256)), blk(256);
  if (dtype == XSM_BF16)
    hipLaunchKernelGGL(k_rope_kv<bf16_t>, grid, blk, 0, s, QKV, rope, eff_len, slot, Qr, (bf16_t*)Kc,
                       (bf16_t*)Vc, n_seq * R, R, H, hd, max_ctx);
  else
    hipLaunchKernelGGL(k_rope_kv<float>, grid, blk, 0, s, QKV, rope, eff_len, slot, Qr, (float*)Kc,
                       (float*)Vc, n_seq * R, R, H, hd, max_ctx);
}

template <typename T>
__global__ void k_store_cond(const float* KV, const int32_t* slot, T* Kc, T* Vc, int n_rows, int C,
                             int row0, int H, int hd, int cap, int v_transposed) {
  const int d = H * hd;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)n_rows * d) return;
  const int c = (int)(idx % d), m = (int)(idx / d);
  const int b = m / C, j = m % C, h = c / hd, i = c % hd;
  const size_t head = (size_t)slot[b] * H + h;
  stf(Kc + (head * cap + row0 + j) * hd + i, KV[(size_t)m * 2 * d + c]);
  const size_t vi = v_transposed ? (head * hd + i) * cap + row0 + j : (head * cap + row0 + j) * hd + i;
  stf(Vc + vi, KV[(size_t)m * 2 * d + d + c]);
}
void launch_store_cond(int dtype, const float* KV, const int32_t* slot, void* Kc, void* Vc,
                       int n_seq, int C, int row0, int H, int hd, int cap, int v_transposed,
                       hipStream_t s) {
  TraceScope trace_("store_cond", s);
  const long n = (long)n_seq * C * H * hd;
  const dim3 grid((unsigned)((n + 255) / 256)), blk(256);
  if (dtype == XSM_BF16)
    hipLaunchKernelGGL(k_store_cond<bf16_t>, grid, blk, 0, s, KV, slot, (bf16_t*)Kc, (bf16_t*)Vc,
                       n_seq * C, C, row0, H, hd, cap, v_transposed);
  else
    hipLaunchKernelGGL(k_store_cond<float>, grid, blk, 0, s, KV, slot, (float*)Kc, (float*)Vc,
                       n_seq * C, C, row0, H, hd, cap, v_transposed);
}

// ---------------------------------------------------------------------------
// Attention, one workgroup per (row, head): every thread keeps an online-softmax
// state (max, sum, weighted values) over keys tid, tid+256, ...; states are
// merged by a fixed butterfly inside each wavefront and then across the four
// wavefronts through LDS.
// ---------------------------------------------------------------------------
template <int HD>
__device__ __forceinline__ void merge_state(float& m, float& l, float (&acc)[HD], float m2, float l2,
                                            const float (&acc2)[HD]) {
  const float mn = fmaxf(m, m2);
  const float f1 = (m == -INFINITY) ? 0.f : expf(m - mn);
  const float f2 = (m2 == -INFINITY) ? 0.f : expf(m2 - mn);
  l = l * f1 + l2 * f2;
#pragma unroll
  for (int i = 0; i < HD; ++i) acc[i] = acc[i] * f1 + acc2[i] * f2;
  m = mn;
}

template <typename T, int HD>
__global__ __launch_bounds__(256) void k_attn_rows(const float* Q, const T* Kc, const T* Vc,
                                                   const int32_t* eff_len, const int32_t* slot,
                                                   float* O, int R, int H, int cap,
                                                   int fixed_limit) {
  constexpr int VEC = VecOf<T>::n;
  __shared__ float sm[4][HD + 2];
  const int m = blockIdx.x, h = blockIdx.y, b = m / R, j = m % R;
  const int d = H * HD;
  const int n = eff_len[b];
  float* out = O + (size_t)m * d + h * HD;
  if (n < 0) {
    for (int i = threadIdx.x; i < HD; i += 256) out[i] = 0.f;
    return;
  }
  const int limit = fixed_limit > 0 ? fixed_limit : n + j + 1;
  const size_t base = ((size_t)slot[b] * H + h) * (size_t)cap * HD;
  const T* kb = Kc + base;
  const T* vb = Vc + base;
  const float scale = rsqrtf((float)HD);
  float q[HD], acc[HD];
#pragma unroll
  for (int i = 0; i < HD; ++i) {
    q[i] = Q[(size_t)m * d + h * HD + i] * scale;
    acc[i] = 0.f;
  }
  float mx = -INFINITY, l = 0.f;
  for (int t = threadIdx.x; t < limit; t += 256) {
    const T* kr = kb + (size_t)t * HD;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < HD; i += VEC) {
      float kv[VEC];
      ldvec(kr + i, kv);
#pragma unroll
      for (int v = 0; v < VEC; ++v) s = fmaf(q[i + v], kv[v], s);
    }
    if (s > mx) {
      const float f = (mx == -INFINITY) ? 0.f : expf(mx - s);
      l *= f;
#pragma unroll
      for (int i = 0; i < HD; ++i) acc[i] *= f;
      mx = s;
    }
    const float p = expf(s - mx);
    l += p;
    const T* vr = vb + (size_t)t * HD;
#pragma unroll
    for (int i = 0; i < HD; i += VEC) {
      float vv[VEC];
      ldvec(vr + i, vv);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[i + v] = fmaf(p, vv[v], acc[i + v]);
    }
  }
  // butterfly merge inside the wavefront
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(mx, o, WAVE), l2 = __shfl_xor(l, o, WAVE);
    float a2[HD];
#pragma unroll
    for (int i = 0; i < HD; ++i) a2[i] = __shfl_xor(acc[i], o, WAVE);
    merge_state<HD>(mx, l, acc, m2, l2, a2);
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) {
    sm[wave][HD] = mx;
    sm[wave][HD + 1] = l;
#pragma unroll
    for (int i = 0; i < HD; ++i) sm[wave][i] = acc[i];
  }
  __syncthreads();
  if (threadIdx.x < HD) {
    const int i = threadIdx.x;
    float mg = sm[0][HD];
    for (int w = 1; w < 4; ++w) mg = fmaxf(mg, sm[w][HD]);
    float num = 0.f, den = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float mw = sm[w][HD];
      const float f = (mw == -INFINITY) ? 0.f : expf(mw - mg);
      num += sm[w][i] * f;
      den += sm[w][HD + 1] * f;
    }
    out[i] = num / den;
  }
}
template <typename T>
static void attn_dispatch(const float* Q, const T* Kc, const T* Vc, const int32_t* eff_len,
                          const int32_t* slot, float* O, int n_seq, int R, int H, int hd, int cap,
                          int fixed_limit, hipStream_t s) {
  const dim3 grid(n_seq * R, H), blk(256);
#define XSM_ATTN_CASE(HDV)                                                                       \
  case HDV:                                                                                      \
    hipLaunchKernelGGL((k_attn_rows<T, HDV>), grid, blk, 0, s, Q, Kc, Vc, eff_len, slot, O, R, H, \
                       cap, fixed_limit);                                                        \
    break;
  switch (hd) {
    XSM_ATTN_CASE(16)
    XSM_ATTN_CASE(32)
    XSM_ATTN_CASE(64)
    XSM_ATTN_CASE(128)
  }
#undef XSM_ATTN_CASE
}
void launch_attention(int dtype, const float* Q, const void* Kc, const void* Vc,
                      const int32_t* eff_len, const int32_t* slot, float* O, int n_seq, int R,
                      int H, int hd, int cap, int fixed_limit, hipStream_t s) {
  TraceScope trace_("attention", s);
  if (dtype == XSM_BF16)
    attn_dispatch<bf16_t>(Q, (const bf16_t*)Kc, (const bf16_t*)Vc, eff_len, slot, O, n_seq, R, H, hd,
                          cap, fixed_limit, s);
  else
    attn_dispatch<float>(Q, (const float*)Kc, (const float*)Vc, eff_len, slot, O, n_seq, R, H, hd,
                         cap, fixed_limit, s);
}

// ---------------------------------------------------------------------------
// cache <-> float staging [H][n_pos][hd] (debug import / export), any cache layout
// ---------------------------------------------------------------------------
template <typename T>
__global__ void k_kv_convert(T* base, float* staging, int H, int pos0, int n_pos, int hd,
                             size_t stride_h, size_t stride_p, size_t stride_i, int to_cache) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)H * n_pos * hd) return;
  const int i = (int)(idx % hd), p = (int)((idx / hd) % n_pos), h = (int)(idx / ((long)hd * n_pos));
  T* c = base + h * stride_h + (size_t)(pos0 + p) * stride_p + i * stride_i;
  if (to_cache) stf(c, staging[idx]);
  else staging[idx] = ldf(c);
}
void launch_kv_convert(int dtype, void* slot_base, float* staging, int H, int pos0, int n_pos,
                       int hd, size_t stride_h, size_t stride_p, size_t stride_i, int to_cache,
                       hipStream_t s) {
  TraceScope trace_("kv_convert", s);
  const long n = (long)H * n_pos * hd;
  const dim3 grid((unsigned)((n + 255) / 256)), blk(256);
  if (dtype == XSM_BF16)
    hipLaunchKernelGGL(k_kv_convert<bf16_t>, grid, blk, 0, s, (bf16_t*)slot_base, staging, H, pos0,
                       n_pos, hd, stride_h, stride_p, stride_i, to_cache);
  else
    hipLaunchKernelGGL(k_kv_convert<float>, grid, blk, 0, s, (float*)slot_base, staging, H, pos0,
                       n_pos, hd, stride_h, stride_p, stride_i, to_cache);
}

__global__ void k_fill_u64(uint64_t* p, size_t n, uint64_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
void launch_fill_u64(uint64_t* p, size_t n, uint64_t v, hipStream_t s) {
  hipLaunchKernelGGL(k_fill_u64, dim3(2048), dim3(256), 0, s, p, n, v);
}

__global__ void k_gather_head_dbg(const float* head_all, const int32_t* acc, float* out, int R, int K,
                                  int V) {
  const int b = blockIdx.y, k = blockIdx.z;
  const int a = acc[b] < 0 ? 0 : acc[b];
  const float* src = head_all + ((size_t)(b * R + a) * K + k) * V;
  float* dst = out + ((size_t)b * K + k) * V;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < V; i += gridDim.x * blockDim.x) dst[i] = src[i];
}
void launch_gather_head_dbg(const float* head_all, const int32_t* acc, float* out, int n_seq, int R,
                            int K, int V, hipStream_t s) {
  hipLaunchKernelGGL(k_gather_head_dbg, dim3(4, n_seq, K), dim3(256), 0, s, head_all, acc, out, R, K, V);
}

__global__ void k_head_rows(const int32_t* acc, int32_t* row_index, int n_seq, int R) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < n_seq) row_index[b] = b * R + (acc[b] < 0 ? 0 : acc[b]);
}
void launch_head_rows(const int32_t* acc, int32_t* row_index, int n_seq, int R, hipStream_t s) {
  TraceScope trace_("head_rows", s);
  hipLaunchKernelGGL(k_head_rows, dim3((n_seq + 63) / 64), dim3(64), 0, s, acc, row_index, n_seq, R);
}

// Cross-attention heads: residual rows Rk[b][k][:] = G[b][:] and the (sequence, head) -> cache
// "slot" / skip-flag arrays of the one attention call over all heads.
__global__ void k_head_ca_prep(const float* G, float* Rk, const int32_t* eff, const int32_t* slot,
                               int32_t* eff2, int32_t* slot2, int n_seq, int K, int d, int max_batch) {
  const int bk = blockIdx.x, b = bk / K, k = bk % K;
  if (threadIdx.x == 0) { eff2[bk] = eff[b] < 0 ? -1 : 0; slot2[bk] = k * max_batch + slot[b]; }
  for (int c = threadIdx.x; c < d; c += blockDim.x) Rk[(size_t)bk * d + c] = G[(size_t)b * d + c];
}
void launch_head_ca_prep(const float* G, float* Rk, const int32_t* eff, const int32_t* slot, int32_t* eff2,
                         int32_t* slot2, int n_seq, int K, int d, int max_batch, hipStream_t s) {
  TraceScope trace_("head_ca_prep", s);
  hipLaunchKernelGGL(k_head_ca_prep, dim3(n_seq * K), dim3(256), 0, s, G, Rk, eff, slot, eff2, slot2, n_seq, K, d,
                     max_batch);
}

}  // namespace xsm
