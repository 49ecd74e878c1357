// Device-side verification and sampling primitives over rows of logits (Sec. 4.2; Sec. 5.4
// "Verification criterion"; appendix "Sampling strategies"): argmax with its margin, rank of a
// candidate, softmax probability of a candidate, categorical draw by inverse CDF, top-K_s
// probability-tree draw.  Written for one 256-thread workgroup per logits row; all reductions
// run in a fixed order.  Shared by the verify / emit kernels of the per-stage path and by the
// single-launch step's last stage.
#pragma once
#include "xsm_device.h"
#include "../../include/xsm.h"

namespace xsm {

constexpr float kTieMargin = 1e-2f;      // logit gap of an argmax or rank decision
constexpr float kCdfMargin = 2e-5f;      // distance of a draw's uniform from a CDF edge, relative to the total weight
constexpr float kCutMargin = 1e-4f;      // relative distance of a tree path's weight from the cut-off

struct RowScratch {
  float redf[8];
  int redi[8];
  float part[256];
  float bestv[4], secv[4];
  int besti[4];
};

// argmax with lowest index among equal maxima; *margin = top1 - top2
__device__ inline int row_argmax(const float* z, int V, RowScratch& sm, float* margin) {
  float bv = -INFINITY, sv = -INFINITY;
  int bi = 0x7FFFFFFF;
  auto feed = [&](float x, int v) {
    if (x > bv || (x == bv && v < bi)) { sv = bv; bv = x; bi = v; }
    else sv = fmaxf(sv, x);
  };
  if ((V & 3) == 0) {                 // 16-byte loads, several in flight per thread
    const float4* z4 = reinterpret_cast<const float4*>(z);
    const int n4 = V >> 2;
    for (int q0 = threadIdx.x; q0 < n4; q0 += 1024) {
      float4 x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        x[u] = q0 + u * 256 < n4 ? z4[q0 + u * 256] : float4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int v = (q0 + u * 256) * 4;
        if (q0 + u * 256 < n4) { feed(x[u].x, v); feed(x[u].y, v + 1); feed(x[u].z, v + 2); feed(x[u].w, v + 3); }
      }
    }
  } else {
    for (int v = threadIdx.x; v < V; v += 256) feed(z[v], v);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float bv2 = __shfl_xor(bv, o, WAVE), sv2 = __shfl_xor(sv, o, WAVE);
    const int bi2 = __shfl_xor(bi, o, WAVE);
    const bool take = (bv2 > bv) || (bv2 == bv && bi2 < bi);
    sv = fmaxf(fmaxf(sv, sv2), fminf(bv, bv2));
    if (take) { bv = bv2; bi = bi2; }
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) {
    sm.bestv[threadIdx.x >> 6] = bv; sm.secv[threadIdx.x >> 6] = sv; sm.besti[threadIdx.x >> 6] = bi;
  }
  __syncthreads();
  bv = sm.bestv[0]; sv = sm.secv[0]; bi = sm.besti[0];
  for (int w = 1; w < 4; ++w) {
    const float bv2 = sm.bestv[w], sv2 = sm.secv[w];
    const int bi2 = sm.besti[w];
    const bool take = (bv2 > bv) || (bv2 == bv && bi2 < bi);
    sv = fmaxf(fmaxf(sv, sv2), fminf(bv, bv2));
    if (take) { bv = bv2; bi = bi2; }
  }
  *margin = bv - sv;
  return bi;
}

// number of tokens ranked ahead of x (larger logit, or equal logit and lower index);
// *gap = distance of z[x] to the nearest other logit on either side of the K_a boundary
__device__ inline int row_rank(const float* z, int V, int x, RowScratch& sm) {
  const float zx = z[x];
  int c = 0;
  if ((V & 3) == 0) {
    const float4* z4 = reinterpret_cast<const float4*>(z);
    const int n4 = V >> 2;
#pragma unroll 4
    for (int q = threadIdx.x; q < n4; q += 256) {
      const float4 y = z4[q];
      const int v = q * 4;
      c += (y.x > zx || (y.x == zx && v < x)) + (y.y > zx || (y.y == zx && v + 1 < x)) +
           (y.z > zx || (y.z == zx && v + 2 < x)) + (y.w > zx || (y.w == zx && v + 3 < x));
    }
  } else {
    for (int v = threadIdx.x; v < V; v += 256) {
      const float y = z[v];
      c += (y > zx || (y == zx && v < x)) ? 1 : 0;
    }
  }
  return block_sum_i(c, sm.redi);
}

// near-tie test for the rank criterion: is some other logit within the margin of z[x]
// while x sits at rank ka-1 or ka (a small change could flip the decision)
__device__ inline bool rank_near_boundary(const float* z, int V, int x, int rank, int ka, RowScratch& sm) {
  const float zx = z[x];
  int above = 0, below = 0;                      // neighbours within the margin
#pragma unroll 4
  for (int v = threadIdx.x; v < V; v += 256) {
    const float dlt = z[v] - zx;
    if (v != x && dlt >= 0.f && dlt <= kTieMargin) ++above;
    if (v != x && dlt < 0.f && -dlt <= kTieMargin) ++below;
  }
  above = block_sum_i(above, sm.redi);
  below = block_sum_i(below, sm.redi);
  // accepted (rank < ka) could become rejected if enough close-below tokens overtake it,
  // rejected could become accepted if enough close-above tokens drop behind it
  if (rank < ka) return rank + below >= ka;
  return rank - above < ka;
}

// softmax(z/T)[x]
__device__ inline float row_prob(const float* z, int V, int x, float invT, RowScratch& sm) {
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < V; v += 256) mx = fmaxf(mx, z[v]);
  mx = block_max(mx, sm.redf);
  float s = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) s += expf((z[v] - mx) * invT);
  s = block_sum(s, sm.redf);
  return expf((z[x] - mx) * invT) / s;
}

// categorical draw by inverse CDF over ascending token index; *near_edge: the uniform lies within
// kCdfMargin (relative to the total weight) of a CDF edge
__device__ inline int row_categorical(const float* z, int V, float invT, float u, RowScratch& sm, bool* near_edge) {
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < V; v += 256) mx = fmaxf(mx, z[v]);
  mx = block_max(mx, sm.redf);
  const int chunk = (V + 255) / 256;
  const int v0 = threadIdx.x * chunk, v1 = min(V, v0 + chunk);
  float loc = 0.f;
  for (int v = v0; v < v1; ++v) loc += expf((z[v] - mx) * invT);
  __syncthreads();
  sm.part[threadIdx.x] = loc;
  __syncthreads();
  if (threadIdx.x == 0) {                       // exclusive scan, fixed order
    float run = 0.f;
    for (int t = 0; t < 256; ++t) { const float p = sm.part[t]; sm.part[t] = run; run += p; }
    sm.redf[4] = run;
  }
  __syncthreads();
  const float target = u * sm.redf[4], band = kCdfMargin * sm.redf[4];
  float run = sm.part[threadIdx.x];
  int hit = 0x7FFFFFFF, lastpos = -1, close = fabsf(run - target) <= band ? 1 : 0;
  for (int v = v0; v < v1; ++v) {
    const float w = expf((z[v] - mx) * invT);
    run += w;
    if (w > 0.f) lastpos = v;
    if (hit == 0x7FFFFFFF && run > target) hit = v;
    close |= fabsf(run - target) <= band ? 1 : 0;
  }
  *near_edge = block_max_i(close, sm.redi) != 0;
  hit = block_min_i(hit, sm.redi);
  if (hit != 0x7FFFFFFF) return hit;
  return block_max_i(lastpos, sm.redi);
}

// ---- the same decisions for rows of 1024 C4 logits (C4 = 1, 2, 4, 8) with the row held in
// registers: thread t owns the 4 C4 consecutive tokens from t * 4 C4 on, memory is read once, the
// running sum over threads is a wavefront scan plus the wavefronts' totals in order, and the three
// reductions of a draw share one exchange.  exp(y) is the hardware's 2^(y log2 e) (1 ulp). ----
constexpr float kLog2e = 1.44269504088896340736f;

template <int C4>
__device__ __forceinline__ void row_to_regs(const float* z, float (&x)[4 * C4]) {
  const float4* p = reinterpret_cast<const float4*>(z) + (size_t)threadIdx.x * C4;
#pragma unroll
  for (int i = 0; i < C4; ++i) {
    const float4 v = p[i];
    x[4 * i] = v.x; x[4 * i + 1] = v.y; x[4 * i + 2] = v.z; x[4 * i + 3] = v.w;
  }
}

template <int C4>
__device__ inline int row_categorical_regs(const float* z, float invT, float u, RowScratch& sm, bool* near_edge) {
  constexpr int C = 4 * C4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, v0 = threadIdx.x * C;
  float x[C];
  row_to_regs<C4>(z, x);
  float mx = x[0];
#pragma unroll
  for (int i = 1; i < C; ++i) mx = fmaxf(mx, x[i]);
  mx = block_max(mx, sm.redf);
  const float c = invT * kLog2e;
  float loc = 0.f;
#pragma unroll
  for (int i = 0; i < C; ++i) { x[i] = __builtin_amdgcn_exp2f((x[i] - mx) * c); loc += x[i]; }   // x: now the weights
  float incl = loc;                                   // inclusive sum over the lanes, lane order
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float t = __shfl_up(incl, o, WAVE);
    if (lane >= o) incl += t;
  }
  float run = __shfl_up(incl, 1, WAVE);
  if (lane == 0) run = 0.f;
  __syncthreads();
  if (lane == 63) sm.redf[4 + wave] = incl;
  __syncthreads();
  float off = 0.f, total = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (q == wave) off = total;
    total += sm.redf[4 + q];
  }
  run += off;
  const float target = u * total, band = kCdfMargin * total;
  int hit = 0x7FFFFFFF, lastpos = -1, close = fabsf(run - target) <= band ? 1 : 0;
#pragma unroll
  for (int i = 0; i < C; ++i) {
    run += x[i];
    if (x[i] > 0.f) lastpos = v0 + i;
    if (hit == 0x7FFFFFFF && run > target) hit = v0 + i;
    close |= fabsf(run - target) <= band ? 1 : 0;
  }
  hit = wave_min_i(hit); lastpos = wave_max_i(lastpos); close = wave_max_i(close);
  __syncthreads();
  if (lane == 0) { sm.redi[wave] = hit; sm.redi[4 + wave] = lastpos; sm.besti[wave] = close; }
  __syncthreads();
  hit = min(min(sm.redi[0], sm.redi[1]), min(sm.redi[2], sm.redi[3]));
  lastpos = max(max(sm.redi[4], sm.redi[5]), max(sm.redi[6], sm.redi[7]));
  *near_edge = (sm.besti[0] | sm.besti[1] | sm.besti[2] | sm.besti[3]) != 0;
  return hit != 0x7FFFFFFF ? hit : lastpos;            // rounding left nothing above the target: the last token with weight
}

template <int C4>
__device__ inline float row_prob_regs(const float* z, int xtok, float invT, RowScratch& sm) {
  constexpr int C = 4 * C4;
  float x[C];
  row_to_regs<C4>(z, x);
  const float zx = z[xtok];
  float mx = x[0];
#pragma unroll
  for (int i = 1; i < C; ++i) mx = fmaxf(mx, x[i]);
  mx = block_max(mx, sm.redf);
  const float c = invT * kLog2e;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < C; ++i) s += __builtin_amdgcn_exp2f((x[i] - mx) * c);
  s = block_sum(s, sm.redf);
  return __builtin_amdgcn_exp2f((zx - mx) * c) / s;
}

// rank of candidate xtok and whether a logit change within the margin could move it across ka
template <int C4>
__device__ inline int row_rank_regs(const float* z, int xtok, int ka, RowScratch& sm, bool* near_boundary) {
  constexpr int C = 4 * C4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, v0 = threadIdx.x * C;
  float x[C];
  row_to_regs<C4>(z, x);
  const float zx = z[xtok];
  int cnt = 0, above = 0, below = 0;
#pragma unroll
  for (int i = 0; i < C; ++i) {
    const int v = v0 + i;
    const float dlt = x[i] - zx;
    cnt += (dlt > 0.f || (dlt == 0.f && v < xtok)) ? 1 : 0;
    if (v != xtok && dlt >= 0.f && dlt <= kTieMargin) ++above;
    if (v != xtok && dlt < 0.f && -dlt <= kTieMargin) ++below;
  }
  cnt = wave_sum_i(cnt); above = wave_sum_i(above); below = wave_sum_i(below);
  __syncthreads();
  if (lane == 0) { sm.redi[wave] = cnt; sm.redi[4 + wave] = above; sm.besti[wave] = below; }
  __syncthreads();
  cnt = sm.redi[0] + sm.redi[1] + sm.redi[2] + sm.redi[3];
  above = sm.redi[4] + sm.redi[5] + sm.redi[6] + sm.redi[7];
  below = sm.besti[0] + sm.besti[1] + sm.besti[2] + sm.besti[3];
  *near_boundary = cnt < ka ? cnt + below >= ka : cnt - above < ka;
  return cnt;
}

// dispatch on the row length: the register versions for V = 1024, 2048, 4096, 8192
__device__ inline int row_draw(const float* z, int V, float invT, float u, RowScratch& sm, bool* near_edge) {
  switch (V) {
    case 1024: return row_categorical_regs<1>(z, invT, u, sm, near_edge);
    case 2048: return row_categorical_regs<2>(z, invT, u, sm, near_edge);
    case 4096: return row_categorical_regs<4>(z, invT, u, sm, near_edge);
    case 8192: return row_categorical_regs<8>(z, invT, u, sm, near_edge);
    default: return row_categorical(z, V, invT, u, sm, near_edge);
  }
}

// One accept decision (Sec. 5.4 "Verification criterion"): is candidate xtok accepted against the
// logits row z under the criterion of vp, and is the decision a near-tie
__device__ inline bool row_accepts(const float* z, int V, int xtok, const xsm_verify_params& vp, RowScratch& sm, bool* near) {
  if (vp.mode == XSM_VERIFY_THRESHOLD) {
    const float invT = 1.0f / vp.temperature;
    float p;
    switch (V) {
      case 1024: p = row_prob_regs<1>(z, xtok, invT, sm); break;
      case 2048: p = row_prob_regs<2>(z, xtok, invT, sm); break;
      case 4096: p = row_prob_regs<4>(z, xtok, invT, sm); break;
      case 8192: p = row_prob_regs<8>(z, xtok, invT, sm); break;
      default: p = row_prob(z, V, xtok, invT, sm);
    }
    // p crosses delta when the candidate's logit moves by about T |ln(p / delta)|
    *near = p > 0.f && vp.delta > 0.f && vp.temperature * fabsf(logf(p) - logf(vp.delta)) <= kTieMargin;
    return p > vp.delta;
  }
  const int ka = vp.mode == XSM_VERIFY_GREEDY ? 1 : vp.top_ka;
  int rank;
  switch (V) {
    case 1024: rank = row_rank_regs<1>(z, xtok, ka, sm, near); break;
    case 2048: rank = row_rank_regs<2>(z, xtok, ka, sm, near); break;
    case 4096: rank = row_rank_regs<4>(z, xtok, ka, sm, near); break;
    case 8192: rank = row_rank_regs<8>(z, xtok, ka, sm, near); break;
    default:
      rank = row_rank(z, V, xtok, sm);
      *near = rank_near_boundary(z, V, xtok, rank, ka, sm);
  }
  return rank < ka;
}

__device__ inline int row_sample(const float* z, int V, const xsm_verify_params& vp, uint32_t pos,
                          uint32_t head, uint32_t seq, RowScratch& sm, uint32_t* flag) {
  if (vp.sample == 0) {
    float margin;
    const int t = row_argmax(z, V, sm, &margin);
    if (margin <= kTieMargin) *flag |= XSM_FLAG_NEAR_TIE;
    return t;
  }
  const float u = philox_uniform(vp.seed, pos, head, seq);
  bool near_edge;
  const int t = row_draw(z, V, 1.0f / vp.temperature, u, sm, &near_edge);
  if (near_edge) *flag |= XSM_FLAG_NEAR_TIE;
  return t;
}

// Top-K_s probability-tree sampling of the K head tokens (appendix "Sampling strategies"): level d
// holds the ks most probable tokens of softmax(z_d / T) with their probabilities as edge weights;
// a complete path survives if its weight (a product of numbers <= 1, so the smallest of its
// prefixes' weights) is at least `prune`; one survivor is drawn in proportion to its weight by
// inverse CDF in depth-first (= lexicographic) order.  Two steps, so that the levels can be built
// side by side: row_topk_probs makes one level, pts_pick draws the path.
struct TreeLevels {
  int idx[16][4];
  float p[16][4];
};

// One level: the ks (<= 4) largest logits of the row, lower index among equals, with their
// softmax(z / T) probabilities -> idx[0..ks), p[0..ks) (workgroup-shared memory; idx = 0x7FFFFFFF,
// p = 0 where the row has fewer than ks tokens).  Ends with a barrier.
__device__ inline void row_topk_probs(const float* z, int V, int ks, float invT, RowScratch& sm, int* idx, float* p) {
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < V; v += 256) mx = fmaxf(mx, z[v]);
  mx = block_max(mx, sm.redf);
  float sum = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) sum += expf((z[v] - mx) * invT);
  sum = block_sum(sum, sm.redf);
  for (int j = 0; j < ks; ++j) {                 // j-th largest logit, lower index among equals
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int v = threadIdx.x; v < V; v += 256) {
      bool taken = false;
      for (int q = 0; q < j; ++q) taken |= idx[q] == v;
      const float x = z[v];
      if (!taken && (x > bv || (x == bv && v < bi))) { bv = x; bi = v; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float bv2 = __shfl_xor(bv, o, WAVE);
      const int bi2 = __shfl_xor(bi, o, WAVE);
      if (bv2 > bv || (bv2 == bv && bi2 < bi)) { bv = bv2; bi = bi2; }
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sm.bestv[threadIdx.x >> 6] = bv; sm.besti[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = 1; w < 4; ++w)
        if (sm.bestv[w] > bv || (sm.bestv[w] == bv && sm.besti[w] < bi)) { bv = sm.bestv[w]; bi = sm.besti[w]; }
      idx[j] = bi;
      p[j] = bi == 0x7FFFFFFF ? 0.f : expf((bv - mx) * invT) / sum;     // V < ks: no such token
    }
    __syncthreads();
  }
}

// One level from registers, for rows of 1024 C4 logits: one memory pass; every round of the
// selection is a local scan of the thread's own tokens plus one workgroup argmax.
template <int C4>
__device__ inline void row_topk_probs_regs(const float* z, int ks, float invT, RowScratch& sm, int* idx, float* p) {
  constexpr int C = 4 * C4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, v0 = threadIdx.x * C;
  float x[C];
  row_to_regs<C4>(z, x);
  float mx = x[0];
#pragma unroll
  for (int i = 1; i < C; ++i) mx = fmaxf(mx, x[i]);
  mx = block_max(mx, sm.redf);
  const float c = invT * kLog2e;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < C; ++i) sum += __builtin_amdgcn_exp2f((x[i] - mx) * c);
  sum = block_sum(sum, sm.redf);
  for (int j = 0; j < ks; ++j) {                 // j-th largest logit, lower index among equals
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
#pragma unroll
    for (int i = 0; i < C; ++i)
      if (x[i] > bv) { bv = x[i]; bi = v0 + i; }      // (ascending index: the first of equals stays)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float bv2 = __shfl_xor(bv, o, WAVE);
      const int bi2 = __shfl_xor(bi, o, WAVE);
      if (bv2 > bv || (bv2 == bv && bi2 < bi)) { bv = bv2; bi = bi2; }
    }
    __syncthreads();
    if (lane == 0) { sm.bestv[wave] = bv; sm.besti[wave] = bi; }
    __syncthreads();
    bv = sm.bestv[0]; bi = sm.besti[0];
    for (int w = 1; w < 4; ++w)
      if (sm.bestv[w] > bv || (sm.bestv[w] == bv && sm.besti[w] < bi)) { bv = sm.bestv[w]; bi = sm.besti[w]; }
    if (threadIdx.x == 0) {
      idx[j] = bi;
      p[j] = bi == 0x7FFFFFFF ? 0.f : __builtin_amdgcn_exp2f((bv - mx) * c) / sum;
    }
    // the winner leaves the contest (its owner marks it taken)
#pragma unroll
    for (int i = 0; i < C; ++i)
      if (v0 + i == bi) x[i] = -INFINITY;
  }
  __syncthreads();
}

__device__ inline void row_level(const float* z, int V, int ks, float invT, RowScratch& sm, int* idx, float* p) {
  switch (V) {
    case 1024: row_topk_probs_regs<1>(z, ks, invT, sm, idx, p); break;
    case 2048: row_topk_probs_regs<2>(z, ks, invT, sm, idx, p); break;
    case 4096: row_topk_probs_regs<4>(z, ks, invT, sm, idx, p); break;
    case 8192: row_topk_probs_regs<8>(z, ks, invT, sm, idx, p); break;
    default: row_topk_probs(z, V, ks, invT, sm, idx, p);
  }
}

// The draw over the tree that levels lv[0..K) span, with the uniform u: cand[1..K] receives the
// tokens.  Returns true (to every thread) when the draw is a near-tie: the uniform within
// kCdfMargin of a path boundary, or a path's weight within kCutMargin (relative) of the cut-off.
__device__ inline bool pts_pick(const TreeLevels& lv, int K, int ks, float prune, float u, RowScratch& sm, int* cand) {
  const int (*top_i)[4] = lv.idx;
  const float (*top_p)[4] = lv.p;
  // leaves in lexicographic order, a contiguous run per thread; running sums in double, thread
  // partials combined in thread order
  __shared__ double pt_part[256];
  __shared__ double pt_total;
  __shared__ int pt_last;
  int n_paths = 1;
  for (int k = 0; k < K; ++k) n_paths *= ks;
  auto weight = [&](int leaf) {                    // digits of `leaf` base ks, first head most significant
    double w = 1.0;
    int rem = leaf, div = n_paths;
    for (int k = 0; k < K; ++k) { div /= ks; w *= (double)top_p[k][rem / div]; rem %= div; }
    return (w >= (double)prune && w > 0.0) ? w : 0.0;   // cut paths carry no weight
  };
  auto raw_weight = [&](int leaf) {
    double w = 1.0;
    int rem = leaf, div = n_paths;
    for (int k = 0; k < K; ++k) { div /= ks; w *= (double)top_p[k][rem / div]; rem %= div; }
    return w;
  };
  const int chunk = (n_paths + 255) / 256;
  const int l0 = min(n_paths, (int)threadIdx.x * chunk), l1 = min(n_paths, l0 + chunk);
  double loc = 0.0;
  int lastpos = -1, close = 0;
  for (int leaf = l0; leaf < l1; ++leaf) {
    const double w = weight(leaf);
    loc += w;
    if (w > 0.0) lastpos = leaf;
    if (fabs(raw_weight(leaf) - (double)prune) <= (double)kCutMargin * (double)prune) close = 1;
  }
  pt_part[threadIdx.x] = loc;
  lastpos = block_max_i(lastpos, sm.redi);
  __syncthreads();
  if (threadIdx.x == 0) {
    double run = 0.0;
    for (int t = 0; t < 256; ++t) { const double p = pt_part[t]; pt_part[t] = run; run += p; }
    pt_total = run;
    pt_last = lastpos;
  }
  __syncthreads();
  int hit = 0x7FFFFFFF;
  if (pt_last >= 0) {
    const double target = (double)u * pt_total, band = (double)kCdfMargin * pt_total;
    double run = pt_part[threadIdx.x];
    if (fabs(run - target) <= band) close = 1;
    for (int leaf = l0; leaf < l1; ++leaf) {
      const double w = weight(leaf);
      run += w;
      if (fabs(run - target) <= band) close = 1;
      if (hit == 0x7FFFFFFF && w > 0.0 && run > target) hit = leaf;
    }
  }
  close = block_max_i(close, sm.redi);
  hit = block_min_i(hit, sm.redi);
  if (threadIdx.x == 0) {
    // no survivor: the most probable token of every head; rounding left nothing above the target: the last survivor
    const int pick = pt_last < 0 ? 0 : (hit == 0x7FFFFFFF ? pt_last : hit);
    int rem = pick, div = n_paths;
    for (int k = 0; k < K; ++k) { div /= ks; cand[k + 1] = top_i[k][rem / div]; rem %= div; }
  }
  __syncthreads();
  return close != 0;
}

// both steps in one workgroup: Zh = the K head rows, consecutive
__device__ inline bool pts_draw(const float* Zh, int K, int V, int ks, float invT, float prune, float u,
                         RowScratch& sm, int* cand) {
  __shared__ TreeLevels lv;
  for (int k = 0; k < K; ++k) row_level(Zh + (size_t)k * V, V, ks, invT, sm, lv.idx[k], lv.p[k]);
  return pts_pick(lv, K, ks, prune, u, sm, cand);
}

}  // namespace xsm
