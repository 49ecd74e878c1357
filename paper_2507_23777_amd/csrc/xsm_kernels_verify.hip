// Verification, resampling and emission (Sec. 4.2; Alg. 1 inner while loop,
// resample line and "s <- s*"): accept scan over the draft block, token draw from
// the backbone row at the first rejected position, gather of that row's hidden
// state for the decoding heads, draws from the head distributions, and the
// length-only cache rollback.  One 256-thread workgroup per sequence; all
// reductions run in a fixed order so results do not depend on timing.
#include "xsm_device.h"
#include "xsm_internal.h"
#include "xsm_verify_device.h"

namespace xsm {

// accept scan + backbone draw + hidden-state gather
__global__ __launch_bounds__(256) void k_verify(const float* Z0, const float* Hf,
                                                const int32_t* block, const int32_t* eff_len,
                                                const int32_t* slot, xsm_verify_params vp,
                                                int32_t* acc, int32_t* y0, uint32_t* wflags,
                                                float* G, int R, int V, int d) {
  __shared__ RowScratch sm;
  const int b = blockIdx.x;
  const int n = eff_len[b];
  if (n < 0) {
    if (threadIdx.x == 0) { acc[b] = -1; y0[b] = 0; }
    if (G) for (int i = threadIdx.x; i < d; i += 256) G[(size_t)b * d + i] = 0.f;
    return;
  }
  uint32_t flag = 0;
  int a = 0;
  for (int j = 1; j < R; ++j) {
    const float* z = Z0 + (size_t)(b * R + j - 1) * V;
    const int x = block[b * R + j];
    bool near;
    const bool ok = row_accepts(z, V, x, vp, sm, &near);
    if (near) flag |= XSM_FLAG_NEAR_TIE;
    if (!ok) break;
    ++a;
  }
  const int tok = row_sample(Z0 + (size_t)(b * R + a) * V, V, vp, (uint32_t)(n + a + 1), 0u,
                             (uint32_t)slot[b], sm, &flag);
  if (threadIdx.x == 0) { acc[b] = a; y0[b] = tok; wflags[b] |= flag; }
  if (G) {
    const float* h = Hf + (size_t)(b * R + a) * d;
    for (int i = threadIdx.x; i < d; i += 256) G[(size_t)b * d + i] = h[i];
  }
}
void launch_verify(const float* Z0, const float* Hf, const int32_t* block, const int32_t* eff_len,
                   const int32_t* slot, const xsm_verify_params& vp, int32_t* acc, int32_t* y0,
                   uint32_t* wflags, float* G, int n_seq, int R, int V, int d, hipStream_t s) {
  TraceScope trace_("verify", s);
  hipLaunchKernelGGL(k_verify, dim3(n_seq), dim3(256), 0, s, Z0, Hf, block, eff_len, slot, vp, acc,
                     y0, wflags, G, R, V, d);
}

// r_k = g + SiLU(W_k g + b_k): Hh holds W_k g for all heads, [n_seq][K][d]
struct BiasPtrs { const void* p[16]; };
template <typename T>
__global__ void k_head_act(const float* G, const float* Hh, BiasPtrs bias, float* Rk, int K, int d,
                           long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int i = (int)(idx % d), k = (int)((idx / d) % K), b = (int)(idx / ((long)d * K));
  const float pre = Hh[idx] + ldf((const T*)bias.p[k] + i);
  Rk[idx] = G[(size_t)b * d + i] + pre / (1.0f + expf(-pre));
}
void launch_head_act(int dtype, const float* G, const float* Hh, const void* const* bias_ptrs,
                     float* Rk, int n_seq, int K, int d, hipStream_t s) {
  TraceScope trace_("head_act", s);
  BiasPtrs bp;
  for (int k = 0; k < 16; ++k) bp.p[k] = k < K ? bias_ptrs[k] : nullptr;
  const long total = (long)n_seq * K * d;
  const dim3 grid((unsigned)((total + 255) / 256)), blk(256);
  if (dtype == XSM_BF16)
    hipLaunchKernelGGL(k_head_act<bf16_t>, grid, blk, 0, s, G, Hh, bp, Rk, K, d, total);
  else
    hipLaunchKernelGGL(k_head_act<float>, grid, blk, 0, s, G, Hh, bp, Rk, K, d, total);
}

// independent draws from the K head rows, one workgroup per (head, sequence): cand[b][k], and
// near-tie flags OR-ed into dflags[b]
__global__ __launch_bounds__(256) void k_draw_heads(const float* Zh, xsm_verify_params vp, const int32_t* eff_len,
                                                    const int32_t* slot, const int32_t* acc, int32_t* cand,
                                                    uint32_t* dflags, int K, int V) {
  __shared__ RowScratch sm;
  const int k = blockIdx.x + 1, b = blockIdx.y;
  const int n = eff_len[b];
  if (n < 0) return;
  uint32_t flag = 0;
  const int t = row_sample(Zh + (size_t)(b * K + k - 1) * V, V, vp, (uint32_t)(n + acc[b] + 1 + k), (uint32_t)k,
                           (uint32_t)slot[b], sm, &flag);
  if (threadIdx.x == 0) {
    cand[b * 16 + k] = t;
    if (flag) atomicOr(&dflags[b], flag);
  }
}

// probability-tree draw if asked for, then emit: accepted tokens, count, next block, new length
__global__ __launch_bounds__(256) void k_emit(const float* Zh, xsm_verify_params vp, const int32_t* drawn,
                                              const int32_t* eff_len, const int32_t* slot,
                                              const int32_t* acc, const int32_t* y0,
                                              const uint32_t* wflags, int32_t* block,
                                              int32_t* kv_len, int32_t* out_tokens,
                                              int32_t* n_accepted, uint32_t* flags, int R, int K,
                                              int V) {
  __shared__ RowScratch sm;
  __shared__ int old_block[16];
  __shared__ int cand[16];
  const int b = blockIdx.x;
  const int n = eff_len[b];
  if (n < 0) {
    if (threadIdx.x == 0) { n_accepted[b] = 0; flags[b] = wflags[b]; }
    return;
  }
  const int a = acc[b];
  if (threadIdx.x < R) old_block[threadIdx.x] = block[b * R + threadIdx.x];
  uint32_t flag = 0;
  if (vp.sample == 2 && K > 0) {
    const float u = philox_uniform(vp.seed, (uint32_t)(n + a + 1), 254u, (uint32_t)slot[b]);
    if (pts_draw(Zh + (size_t)b * K * V, K, V, vp.top_ks, 1.0f / vp.temperature, vp.pts_prune, u, sm, cand))
      flag = XSM_FLAG_NEAR_TIE;
  } else if (threadIdx.x >= 1 && threadIdx.x <= K) {
    cand[threadIdx.x] = drawn[b * 16 + threadIdx.x];          // k_draw_heads ran before this kernel
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int j = 0; j < a; ++j) out_tokens[b * R + j] = old_block[j + 1];
    out_tokens[b * R + a] = y0[b];
    for (int j = a + 1; j < R; ++j) out_tokens[b * R + j] = -1;
    block[b * R] = y0[b];
    for (int k = 1; k <= K; ++k) block[b * R + k] = cand[k];
    n_accepted[b] = a + 1;
    kv_len[b] = n + a + 1;
    flags[b] = wflags[b] | flag;
  }
}
void launch_emit(const float* Zh, const xsm_verify_params& vp, const int32_t* eff_len,
                 const int32_t* slot, const int32_t* acc, const int32_t* y0,
                 uint32_t* wflags, int32_t* drawn, int32_t* block, int32_t* kv_len, int32_t* out_tokens,
                 int32_t* n_accepted, uint32_t* flags, int n_seq, int R, int K, int V,
                 hipStream_t s) {
  TraceScope trace_("emit", s);
  if (K > 0 && vp.sample != 2)
    hipLaunchKernelGGL(k_draw_heads, dim3(K, n_seq), dim3(256), 0, s, Zh, vp, eff_len, slot, acc, drawn, wflags, K, V);
  hipLaunchKernelGGL(k_emit, dim3(n_seq), dim3(256), 0, s, Zh, vp, drawn, eff_len, slot, acc, y0, wflags,
                     block, kv_len, out_tokens, n_accepted, flags, R, K, V);
}

}  // namespace xsm
