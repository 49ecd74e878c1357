// One speculative (or plain) decoding step as ONE persistent kernel, for the
// latency regime: at most 16 block rows in total (batch x (K+1) <= 16), bf16,
// d_model 1024-class models with head_dim 64, greedy verification.
//
// At batch 1 a step streams every weight once (hundreds of MB) through ~150 dependent
// stages of a few MB each, so what bounds it is not bandwidth inside a stage but the
// latency of handing a few KB of activations from one stage's producers to the next
// stage's consumers.  Kernel boundaries cost several microseconds each; here all 256
// workgroups (one per compute unit) stay resident for the whole step and exchange
// activations through memory with a flag in every 8-byte word:
//     word = { 32-bit payload (one fp32 or two bf16), 32-bit tag }, tag = step epoch.
// A producer writes words with device-coherent stores; a consumer loads the words it
// needs with device-coherent loads and retries until every tag equals the current
// epoch, so arrival of the data IS the synchronisation (no barrier, no second round
// trip).  Each (layer, stage) owns its own buffer, so there is no reuse hazard inside a
// step; the epoch makes last step's contents invalid.  Every wait is bounded: a
// workgroup that does not see its inputs within the spin budget raises the error word
// and leaves, and so does every workgroup waiting on it.
//
// Weights never depend on activations, so each workgroup requests the fragments of the
// tile it will need one layer ahead and holds them in registers; HBM stays busy while
// the dependency chain is waiting.  Stages per layer (Sec. 4.1 block = self-attention +
// feed-forward; Alg. 1 "forward with causal mask"):
//   QKV   192 tiles  RMSNorm + projection + rotary, new k/v also written to the cache
//   ATT   B*H*S units  MFMA attention over a slice of the cached keys (+ the new block)
//   COMB  merge of the S slices (skipped when S == 1)
//   OPROJ 64 tiles   output projection + residual
//   UP    256 tiles  RMSNorm + W1 + erf-GELU
//   DOWN  64 tiles   W2 + residual
// then the decoding heads on every block row (Alg. 1 runs each head on h_{s:s+D}), the
// shared unembedding over backbone and head rows with a per-tile top-2 reduction, and one
// workgroup per sequence that does the accept scan, picks the tokens at the first rejected
// position and rolls the cache length back (Alg. 1 inner loop, resample line, s <- s*).
#include "xsm_device.h"
#include "xsm_internal.h"

namespace xsm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kSpinBudget = 150000;         // polls before a wait gives up (a fraction of a second)
constexpr float kTieMarginS = 1e-2f;

__device__ __forceinline__ uint64_t ll_ld(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_st(uint64_t* p, uint32_t payload, uint32_t tag) {
  __hip_atomic_store(p, ((uint64_t)tag << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t pk2(float a, float b) {
  return (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16);
}

// Wait for NG groups of GW consecutive tagged words (groups gstride words apart); all loads
// of a round are issued before any is checked.  Payloads go to out.  On timeout, or when an
// earlier wait of this lane already failed, ok is false and out is zero.
template <int NG, int GW>
__device__ __forceinline__ void ll_wait_groups(const uint64_t* p, size_t gstride, uint32_t tag,
                                               uint32_t (&out)[NG * GW], bool& ok) {
  if (ok) {
    for (int spin = 0; spin < kSpinBudget; ++spin) {
      uint64_t w[NG * GW];
#pragma unroll
      for (int gi = 0; gi < NG; ++gi)
#pragma unroll
        for (int e = 0; e < GW; ++e) w[gi * GW + e] = ll_ld(p + gi * gstride + e);
      bool good = true;
#pragma unroll
      for (int i = 0; i < NG * GW; ++i) good &= (uint32_t)(w[i] >> 32) == tag;
      if (good) {
#pragma unroll
        for (int i = 0; i < NG * GW; ++i) out[i] = (uint32_t)w[i];
        return;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    ok = false;
  }
#pragma unroll
  for (int i = 0; i < NG * GW; ++i) out[i] = 0u;
}
template <int N>
__device__ __forceinline__ void ll_wait(const uint64_t* p, uint32_t tag, uint32_t (&out)[N], bool& ok) {
  ll_wait_groups<1, N>(p, 0, tag, out, ok);
}

template <int N>
__device__ __forceinline__ void load_frags(uint4 (&w)[N], const uint4* Wt, int nt, int KT, int kt0,
                                           int lane) {
  const uint4* p = Wt + ((size_t)nt * KT + kt0) * 64 + lane;
#pragma unroll
  for (int i = 0; i < N; ++i) w[i] = p[(size_t)i * 64];
}

struct Shared {
  float red[4][64][4];          // cross-wavefront tile reduction
  float rowsum[4][16];          // RMSNorm partial sums
  float att_ml[4][2][16];
  float att_o[4][4][64][4];
  int len[16], slot[16];
  uint32_t flag[16];
  uint32_t tag;
  int fail;
  float st_max[80], st_sec[80];  // FINAL: per-row reductions
  int st_idx[80];
};

}  // namespace

// Sum the four wavefronts' partial 16x16 tiles; thread (wave i, lane) gets element
// D[nrow = (lane>>4)*4 + i][m = lane & 15].
__device__ __forceinline__ float tile_reduce(Shared& sm, f32x4 acc, int wave, int lane) {
  __syncthreads();
  *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
  __syncthreads();
  return (sm.red[0][lane][wave] + sm.red[1][lane][wave]) + (sm.red[2][lane][wave] + sm.red[3][lane][wave]);
}

// B-operand fragments (activation rows) of one wavefront's NKT k-tiles from fp32 tagged
// words: lane (m = lane&15, g = lane>>4) takes columns (kt0 + i)*32 + g*8 .. +8 of row m.
// vals keeps the fp32 values (for the RMSNorm), ss their sum of squares.
template <int NKT>
__device__ __forceinline__ void poll_rows_f32(const uint64_t* buf, int ld, int m, bool live, int kt0,
                                              int g, uint32_t tag, float (&vals)[NKT][8], float& ss,
                                              bool& ok) {
  ss = 0.f;
  uint32_t pw[NKT * 8];
  if (live) {
    ll_wait_groups<NKT, 8>(buf + (size_t)m * ld + kt0 * 32 + g * 8, 32, tag, pw, ok);
  } else {
#pragma unroll
    for (int i = 0; i < NKT * 8; ++i) pw[i] = 0u;
  }
#pragma unroll
  for (int i = 0; i < NKT; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      vals[i][e] = __uint_as_float(pw[i * 8 + e]);
      ss += vals[i][e] * vals[i][e];
    }
}

template <int D, int F>
__global__ __launch_bounds__(256) void k_step_small(const SmallArgs a) {
  constexpr int H = D / 64;
  constexpr int KTD = D / 32, KTF = F / 32;          // k-tiles of the two contraction lengths
  constexpr int KD = KTD / 4, KF = KTF / 4;          // per wavefront
  constexpr int NQ = 3 * D / 16, NO = D / 16, NU = F / 16;
  constexpr int O_BASE = NQ, DN_BASE = 128;
  static_assert(NQ + NO <= 256 && DN_BASE + NO <= 256 && NU <= 256, "tile roles must fit 256 workgroups");
  __shared__ Shared sm;

  const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int R = a.R, K = R - 1, M = a.n_seq * R, S = a.S, V = a.V;

  // ---- set-up: epoch and per-sequence validation (every workgroup, redundantly) ----
  if (tid == 0) {
    sm.tag = __hip_atomic_load(a.ctrl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm.fail = (int)__hip_atomic_load(a.ctrl + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (tid < 16) {
    int len = -1, sl = 0;
    uint32_t f = 0;
    if (tid < a.n_seq) {
      const int n = a.kv_len[tid];
      sl = a.slot[tid];
      if (n < 0 || n + R > a.max_ctx || n > a.bound) f |= XSM_FLAG_BAD_LEN;
      if (sl < 0 || sl >= a.max_batch) { f |= XSM_FLAG_BAD_SLOT; sl = 0; }
      for (int j = 0; j < R; ++j) {
        const int t = a.block[tid * R + j];
        if (t < 0 || t >= V) f |= XSM_FLAG_BAD_TOKEN;
      }
      len = f ? -1 : n;
    }
    sm.len[tid] = len; sm.slot[tid] = sl; sm.flag[tid] = f;
  }
  __syncthreads();
  if (sm.fail != 0) return;                 // an earlier step timed out: stay down until reset
  const uint32_t tag = sm.tag;
  // this lane's activation row (MFMA column) m = r
  const int mb = r / R, mj = r % R;
  const bool row_in = r < M;
  const int len_m = row_in ? sm.len[mb] : -1;
  const bool live = row_in && len_m >= 0;              // rows of skipped sequences carry zeros
  // the output element this thread finishes after tile_reduce: (nrow, m = r)
  const int nrow = g * 4 + wave;

  const size_t LS = a.ll_layer_stride;                 // words per layer
  uint64_t* const llb = a.ll;
  const size_t OFF_X = 0, OFF_Q = 16 * D, OFF_KN = 2 * 16 * D, OFF_VN = 3 * 16 * D, OFF_O = 4 * 16 * D,
               OFF_XM = 5 * 16 * D, OFF_U = 6 * 16 * D, OFF_P = 6 * 16 * D + 16 * (F / 2);

  const bool has_q = w < NQ, has_o = w >= O_BASE && w < O_BASE + NO, has_u = w < NU,
             has_d = w >= DN_BASE && w < DN_BASE + NO;
  uint4 wq[KD], wo[KD], wu[KD], wd[KF];
  if (has_q) load_frags<KD>(wq, a.layers[0].Wqkv, w, KTD, wave * KD, lane);
  if (has_o) load_frags<KD>(wo, a.layers[0].Wo, w - O_BASE, KTD, wave * KD, lane);
  if (has_u) load_frags<KD>(wu, a.layers[0].W1, w, KTD, wave * KD, lane);
  if (has_d) load_frags<KF>(wd, a.layers[0].W2, w - DN_BASE, KTF, wave * KF, lane);

  // ---- EMBED: layer-0 residual rows as tagged words ----
  for (int idx = w * 256 + tid; idx < M * D; idx += 256 * 256) {
    const int m = idx / D, c = idx % D, b = m / R;
    const float x = sm.len[b] >= 0 ? bf2f(a.E[(size_t)a.block[m] * D + c]) : 0.f;
    ll_st(llb + OFF_X + (size_t)m * D + c, __float_as_uint(x), tag);
  }

  bool ok = true;
  for (int l = 0; l < a.L; ++l) {
    uint64_t* const lb = llb + (size_t)l * LS;
    const LayerTab lt = a.layers[l];

    // ================= QKV =================
    if (has_q) {
      float xv[KD][8];
      float ss;
      poll_rows_f32<KD>(lb + OFF_X, D, r, live, wave * KD, g, tag, xv, ss, ok);
      ss += __shfl_xor(ss, 16, WAVE);
      ss += __shfl_xor(ss, 32, WAVE);
      if (g == 0) sm.rowsum[wave][r] = ss;
      __syncthreads();
      const float inv = 1.0f / sqrtf(((sm.rowsum[0][r] + sm.rowsum[1][r]) + (sm.rowsum[2][r] + sm.rowsum[3][r])) / (float)D + a.eps);
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < KD; ++i) {
        const uint4 gg = *reinterpret_cast<const uint4*>(lt.g1 + (wave * KD + i) * 32 + g * 8);
        const uint32_t gw[4] = {gg.x, gg.y, gg.z, gg.w};
        uint32_t bw[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          bw[e] = pk2(xv[i][2 * e] * inv * __uint_as_float(gw[e] << 16),
                      xv[i][2 * e + 1] * inv * __uint_as_float(gw[e] & 0xFFFF0000u));
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wq[i]),
                                                      __builtin_bit_cast(bf16x8, uint4{bw[0], bw[1], bw[2], bw[3]}), acc, 0, 0, 0);
      }
      if (l + 1 < a.L) load_frags<KD>(wq, a.layers[l + 1].Wqkv, w, KTD, wave * KD, lane);
      const float v = tile_reduce(sm, acc, wave, lane);
      const float partner = __shfl_xor(v, 32, WAVE);
      if (live) {
        const int pos = len_m + mj;
        const int sec = w / (D / 16), ts = w % (D / 16), h = ts >> 2, tt = ts & 3;
        float o = v;
        int dim;
        if (sec < 2) {
          const int pi = tt * 8 + (nrow & 7);
          const float2 cs = a.rope[(size_t)pos * 32 + pi];
          if (nrow < 8) { dim = pi; o = v * cs.x - partner * cs.y; }
          else { dim = 32 + pi; o = partner * cs.y + v * cs.x; }
        } else {
          dim = tt * 16 + nrow;
        }
        const size_t col = (size_t)r * D + h * 64 + dim;
        const size_t head = (size_t)sm.slot[mb] * H + h;
        if (sec == 0) {
          ll_st(lb + OFF_Q + col, __float_as_uint(o), tag);
        } else if (sec == 1) {
          ll_st(lb + OFF_KN + col, __float_as_uint(o), tag);
          lt.Kc[(head * a.cap + pos) * 64 + dim] = f2bf(o);
        } else {
          ll_st(lb + OFF_VN + col, __float_as_uint(o), tag);
          lt.Vt[(head * 64 + dim) * a.cap + pos] = f2bf(o);
        }
      }
    }

    // ================= ATT =================
    const int n_units = a.n_seq * H * S;
    if (w < n_units) {
      const int b = w / (H * S), h = (w / S) % H, s = w % S;
      const int n = sm.len[b];
      const int nn = n < 0 ? 0 : n;                       // skipped sequence: no cached keys read
      const int NC = (nn + 63) >> 6, CPS = (NC + S - 1) / S;
      const int c_lo = s * CPS, c_hi = min(NC, c_lo + CPS);
      const size_t head = (size_t)sm.slot[b] * H + h;
      const uint16_t* kb = lt.Kc + head * (size_t)a.cap * 64;
      const uint16_t* vb = lt.Vt + head * 64 * (size_t)a.cap;
      // queries of this sequence: MFMA column r is query j = r (r < R)
      uint4 qf[2] = {uint4{0, 0, 0, 0}, uint4{0, 0, 0, 0}};
      const bool qlive = r < R && n >= 0;
      if (qlive) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          uint32_t pw[8];
          ll_wait<8>(lb + OFF_Q + (size_t)(b * R + r) * D + h * 64 + hf * 32 + g * 8, tag, pw, ok);
          qf[hf] = uint4{pk2(__uint_as_float(pw[0]), __uint_as_float(pw[1])), pk2(__uint_as_float(pw[2]), __uint_as_float(pw[3])),
                         pk2(__uint_as_float(pw[4]), __uint_as_float(pw[5])), pk2(__uint_as_float(pw[6]), __uint_as_float(pw[7]))};
        }
      }
      const bf16x8 q0 = __builtin_bit_cast(bf16x8, qf[0]), q1 = __builtin_bit_cast(bf16x8, qf[1]);
      float m_run = -INFINITY, l_run = 0.f;
      f32x4 o[4];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

      // cached keys 0..n-1: every live query sees all of them
      for (int c = c_lo + wave; c < c_hi; c += 4) {
        const int key0 = c << 6;
        uint4 kf[4][2], vf[4][2];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint16_t* kr = kb + (size_t)(key0 + (r >> 2) * 16 + t * 4 + (r & 3)) * 64 + g * 8;
          kf[t][0] = *reinterpret_cast<const uint4*>(kr);
          kf[t][1] = *reinterpret_cast<const uint4*>(kr + 32);
        }
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const uint16_t* vr = vb + (size_t)(dt * 16 + r) * a.cap + key0 + g * 16;
          vf[dt][0] = *reinterpret_cast<const uint4*>(vr);
          vf[dt][1] = *reinterpret_cast<const uint4*>(vr + 8);
        }
        f32x4 sc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[t][0]), q0, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
          sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[t][1]), q1, sc[t], 0, 0, 0);
        }
        const int kbase = key0 + g * 16;
        const bool edge = key0 + 64 > nn || !qlive;
        const int lim = qlive ? nn : 0;
        float cmax = -INFINITY;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float v = sc[t][i] * a.scale_log2;
            if (edge && kbase + t * 4 + i >= lim) v = -INFINITY;
            sc[t][i] = v;
            cmax = fmaxf(cmax, v);
          }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16, WAVE));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32, WAVE));
        const float m_new = fmaxf(m_run, cmax);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_use);
        float psum = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p = exp2f(sc[t][i] - m_use);
            sc[t][i] = p;
            psum += p;
          }
        psum += __shfl_xor(psum, 16, WAVE);
        psum += __shfl_xor(psum, 32, WAVE);
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
        if (key0 + 64 > nn) {                            // positions >= n are not cached history
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
              uint32_t* wv = reinterpret_cast<uint32_t*>(&vf[dt][jj]);
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (kbase + jj * 8 + e >= nn) wv[e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
            }
        }
        uint4 pf[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          pf[jj] = uint4{pk2(sc[2 * jj][0], sc[2 * jj][1]), pk2(sc[2 * jj][2], sc[2 * jj][3]),
                         pk2(sc[2 * jj + 1][0], sc[2 * jj + 1][1]), pk2(sc[2 * jj + 1][2], sc[2 * jj + 1][3])};
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int jj = 0; jj < 2; ++jj)
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[dt][jj]),
                                                            __builtin_bit_cast(bf16x8, pf[jj]), o[dt], 0, 0, 0);
      }

      // the R new keys of this step (positions n..n+R-1): one 16-key tile, taken by wavefront 3
      // of slice 0, straight from the tagged k/v words; query j sees new key i iff i <= j
      if (s == 0 && wave == 3 && n >= 0) {
        // A operand of S^T: lane (key r, g) holds k_new[r][hf*32 + g*8 .. +8]
        uint4 kn[2] = {uint4{0, 0, 0, 0}, uint4{0, 0, 0, 0}};
        if (r < R) {
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            uint32_t pw[8];
            ll_wait<8>(lb + OFF_KN + (size_t)(b * R + r) * D + h * 64 + hf * 32 + g * 8, tag, pw, ok);
            kn[hf] = uint4{pk2(__uint_as_float(pw[0]), __uint_as_float(pw[1])), pk2(__uint_as_float(pw[2]), __uint_as_float(pw[3])),
                           pk2(__uint_as_float(pw[4]), __uint_as_float(pw[5])), pk2(__uint_as_float(pw[6]), __uint_as_float(pw[7]))};
          }
        }
        f32x4 sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kn[0]), q0, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kn[1]), q1, sc, 0, 0, 0);
        // lane (query r, g) holds new keys g*4 + i
        float cmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int key = g * 4 + i;
          float v = sc[i] * a.scale_log2;
          if (!(qlive && key <= r && key < R)) v = -INFINITY;
          sc[i] = v;
          cmax = fmaxf(cmax, v);
        }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16, WAVE));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32, WAVE));
        const float m_new = fmaxf(m_run, cmax);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_use);
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float p = exp2f(sc[i] - m_use);
          sc[i] = p;
          psum += p;
        }
        psum += __shfl_xor(psum, 16, WAVE);
        psum += __shfl_xor(psum, 32, WAVE);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        // contraction index of the second product: k = g*8 + e  <->  new key g*4 + e (e < 4)
        const uint4 pfrag = uint4{pk2(sc[0], sc[1]), pk2(sc[2], sc[3]), 0u, 0u};
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          // A operand: lane (dim dt*16 + r, g) holds v_new[key g*4 + e][dim], e < 4
          float vv[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int key = g * 4 + e;
            if (key < R) {
              uint32_t pw[1];
              ll_wait<1>(lb + OFF_VN + (size_t)(b * R + key) * D + h * 64 + dt * 16 + r, tag, pw, ok);
              vv[e] = __uint_as_float(pw[0]);
            }
          }
          const uint4 vfrag = uint4{pk2(vv[0], vv[1]), pk2(vv[2], vv[3]), 0u, 0u};
          o[dt] = o[dt] * alpha;
          o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vfrag),
                                                          __builtin_bit_cast(bf16x8, pfrag), o[dt], 0, 0, 0);
        }
      }

      // merge the four wavefronts; wavefront i finishes dim tile i
      __syncthreads();
      if (g == 0) { sm.att_ml[wave][0][r] = m_run; sm.att_ml[wave][1][r] = l_run; }
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) *reinterpret_cast<f32x4*>(&sm.att_o[wave][dt][lane][0]) = o[dt];
      __syncthreads();
      float Mx = -INFINITY;
#pragma unroll
      for (int q = 0; q < 4; ++q) Mx = fmaxf(Mx, sm.att_ml[q][0][r]);
      float Lx = 0.f;
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float mw = sm.att_ml[q][0][r];
        const float f = mw == -INFINITY ? 0.f : exp2f(mw - Mx);
        Lx += sm.att_ml[q][1][r] * f;
        acc += *reinterpret_cast<const f32x4*>(&sm.att_o[q][wave][lane][0]) * f;
      }
      if (S == 1) {
        if (r < R) {
          const float inv = n >= 0 ? 1.0f / Lx : 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            ll_st(lb + OFF_O + (size_t)(b * R + r) * D + h * 64 + wave * 16 + g * 4 + i,
                  __float_as_uint(n >= 0 ? acc[i] * inv : 0.f), tag);
        }
      } else {
        uint64_t* part = lb + OFF_P + (size_t)w * 1056;
        if (wave == 0 && g == 0) {
          ll_st(part + r, __float_as_uint(Mx), tag);
          ll_st(part + 16 + r, __float_as_uint(Lx), tag);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
          ll_st(part + 32 + (size_t)(wave * 16 + g * 4 + i) * 16 + r, __float_as_uint(acc[i]), tag);
      }
    }

    // ================= COMB =================
    if (S > 1 && w < n_units) {
      const int b = w / (H * S), h = (w / S) % H, s = w % S;
      const int dps = 64 / S;                               // dims finished by this unit
      for (int qd = tid >> 4; qd < dps; qd += 16) {
        if (r >= R) break;
        const int dim = s * dps + qd;
        const uint64_t* p0 = lb + OFF_P + (size_t)(w - s) * 1056;
        float Mg = -INFINITY, mk[16];
        for (int k = 0; k < S; ++k) {
          uint32_t pw[1];
          ll_wait<1>(p0 + (size_t)k * 1056 + r, tag, pw, ok);
          mk[k] = __uint_as_float(pw[0]);
          Mg = fmaxf(Mg, mk[k]);
        }
        float Lg = 0.f, og = 0.f;
        for (int k = 0; k < S; ++k) {
          uint32_t pl[1], po[1];
          ll_wait<1>(p0 + (size_t)k * 1056 + 16 + r, tag, pl, ok);
          ll_wait<1>(p0 + (size_t)k * 1056 + 32 + (size_t)dim * 16 + r, tag, po, ok);
          const float f = mk[k] == -INFINITY ? 0.f : exp2f(mk[k] - Mg);
          Lg += __uint_as_float(pl[0]) * f;
          og += __uint_as_float(po[0]) * f;
        }
        const float outv = sm.len[b] >= 0 ? og / Lg : 0.f;
        ll_st(lb + OFF_O + (size_t)(b * R + r) * D + h * 64 + dim, __float_as_uint(outv), tag);
      }
    }

    // ================= OPROJ =================
    if (has_o) {
      const int nt = w - O_BASE;
      float xv[KD][8];
      float ss;
      poll_rows_f32<KD>(lb + OFF_O, D, r, row_in, wave * KD, g, tag, xv, ss, ok);
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < KD; ++i) {
        const uint4 bfrag = uint4{pk2(xv[i][0], xv[i][1]), pk2(xv[i][2], xv[i][3]), pk2(xv[i][4], xv[i][5]), pk2(xv[i][6], xv[i][7])};
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wo[i]),
                                                      __builtin_bit_cast(bf16x8, bfrag), acc, 0, 0, 0);
      }
      if (l + 1 < a.L) load_frags<KD>(wo, a.layers[l + 1].Wo, nt, KTD, wave * KD, lane);
      const float v = tile_reduce(sm, acc, wave, lane);
      if (row_in) {
        uint32_t px[1];
        ll_wait<1>(lb + OFF_X + (size_t)r * D + nt * 16 + nrow, tag, px, ok);
        ll_st(lb + OFF_XM + (size_t)r * D + nt * 16 + nrow, __float_as_uint(__uint_as_float(px[0]) + v), tag);
      }
    }

    // ================= UP =================
    if (has_u) {
      float xv[KD][8];
      float ss;
      poll_rows_f32<KD>(lb + OFF_XM, D, r, row_in, wave * KD, g, tag, xv, ss, ok);
      ss += __shfl_xor(ss, 16, WAVE);
      ss += __shfl_xor(ss, 32, WAVE);
      __syncthreads();
      if (g == 0) sm.rowsum[wave][r] = ss;
      __syncthreads();
      const float inv = 1.0f / sqrtf(((sm.rowsum[0][r] + sm.rowsum[1][r]) + (sm.rowsum[2][r] + sm.rowsum[3][r])) / (float)D + a.eps);
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < KD; ++i) {
        const uint4 gg = *reinterpret_cast<const uint4*>(lt.g2 + (wave * KD + i) * 32 + g * 8);
        const uint32_t gw[4] = {gg.x, gg.y, gg.z, gg.w};
        uint32_t bw[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          bw[e] = pk2(xv[i][2 * e] * inv * __uint_as_float(gw[e] << 16),
                      xv[i][2 * e + 1] * inv * __uint_as_float(gw[e] & 0xFFFF0000u));
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wu[i]),
                                                      __builtin_bit_cast(bf16x8, uint4{bw[0], bw[1], bw[2], bw[3]}), acc, 0, 0, 0);
      }
      if (l + 1 < a.L) load_frags<KD>(wu, a.layers[l + 1].W1, w, KTD, wave * KD, lane);
      __syncthreads();
      *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
      __syncthreads();
      // threads 0..127: row m = tid&15, output pair (2p, 2p+1), p = tid>>4
      if (tid < 128 && r < M) {
        const int p = tid >> 4;
        float v2[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int nr = 2 * p + q, ln = (nr >> 2) * 16 + r, ii = nr & 3;
          const float v = (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
          v2[q] = 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
        }
        ll_st(lb + OFF_U + (size_t)r * (F / 2) + w * 8 + p, pk2(v2[0], v2[1]), tag);
      }
    }

    // ================= DOWN =================
    if (has_d) {
      const int nt = w - DN_BASE;
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i0 = 0; i0 < KF; i0 += 8) {
        uint32_t pw[32];
        if (row_in) {
          ll_wait_groups<8, 4>(lb + OFF_U + (size_t)r * (F / 2) + (wave * KF + i0) * 16 + g * 4, 16, tag, pw, ok);
        } else {
#pragma unroll
          for (int i = 0; i < 32; ++i) pw[i] = 0u;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              __builtin_bit_cast(bf16x8, wd[i0 + i]),
              __builtin_bit_cast(bf16x8, uint4{pw[4 * i], pw[4 * i + 1], pw[4 * i + 2], pw[4 * i + 3]}), acc, 0, 0, 0);
      }
      if (l + 1 < a.L) load_frags<KF>(wd, a.layers[l + 1].W2, nt, KTF, wave * KF, lane);
      const float v = tile_reduce(sm, acc, wave, lane);
      if (row_in) {
        uint32_t px[1];
        ll_wait<1>(lb + OFF_XM + (size_t)r * D + nt * 16 + nrow, tag, px, ok);
        ll_st(lb + LS + OFF_X + (size_t)r * D + nt * 16 + nrow, __float_as_uint(__uint_as_float(px[0]) + v), tag);
      }
    }

    // a workgroup that timed out anywhere leaves (its consumers will time out in turn)
    if (__syncthreads_or(!ok)) {
      if (tid == 0) __hip_atomic_store(a.ctrl + 1, 1u + (uint32_t)l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
  }

  // =========================== tail ===========================
  uint64_t* const tb = llb + (size_t)a.L * LS;             // XB[L] lives at the start of this block
  const size_t OFF_RB = 16 * D;                            // head outputs: [16*K rows][D/2] bf16x2 words
  const size_t OFF_ST = OFF_RB + (size_t)16 * 15 * (D / 2); // per (tile, row) top-2 statistics: 4 words
  const int NTV = V / 16;                                  // vocabulary tiles
  const int rows_all = M + M * K;                          // backbone rows, then head rows (m, k)

  // final-normed hidden state of every row, as this lane's B fragments (all workgroups need it)
  uint4 hfrag[KD];
  float hval[KD][8];
  {
    float ss;
    poll_rows_f32<KD>(tb + OFF_X, D, r, row_in, wave * KD, g, tag, hval, ss, ok);
    ss += __shfl_xor(ss, 16, WAVE);
    ss += __shfl_xor(ss, 32, WAVE);
    __syncthreads();
    if (g == 0) sm.rowsum[wave][r] = ss;
    __syncthreads();
    const float inv = 1.0f / sqrtf(((sm.rowsum[0][r] + sm.rowsum[1][r]) + (sm.rowsum[2][r] + sm.rowsum[3][r])) / (float)D + a.eps);
#pragma unroll
    for (int i = 0; i < KD; ++i) {
      const uint4 gg = *reinterpret_cast<const uint4*>(a.gf + (wave * KD + i) * 32 + g * 8);
      const uint32_t gw[4] = {gg.x, gg.y, gg.z, gg.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        hval[i][2 * e] *= inv * __uint_as_float(gw[e] << 16);
        hval[i][2 * e + 1] *= inv * __uint_as_float(gw[e] & 0xFFFF0000u);
      }
      hfrag[i] = uint4{pk2(hval[i][0], hval[i][1]), pk2(hval[i][2], hval[i][3]), pk2(hval[i][4], hval[i][5]), pk2(hval[i][6], hval[i][7])};
    }
  }

  // ---- HEADS on every row: r_k = g + SiLU(W_k g + b_k)  (Eq. 4, MLP variant) ----
  for (int t = w; t < K * (D / 16); t += 256) {
    uint4 wh[KD];
    load_frags<KD>(wh, a.Wh, t, KTD, wave * KD, lane);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < KD; ++i)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wh[i]), __builtin_bit_cast(bf16x8, hfrag[i]), acc, 0, 0, 0);
    __syncthreads();
    *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
    // the normalised hidden values of the 16 output columns of this tile, for the residual
    const int kh = t / (D / 16), c0 = (t % (D / 16)) * 16;   // head index, first column
    __syncthreads();
    if (tid < 128 && r < M) {
      const int p = tid >> 4;
      float v2[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int nr = 2 * p + q, ln = (nr >> 2) * 16 + r, ii = nr & 3;
        const float y = (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
        const float pre = y + bf2f(a.hb[(size_t)kh * D + c0 + nr]);
        // g[c] recomputed from the tagged residual words (fp32), same arithmetic as above
        uint32_t px[1];
        ll_wait<1>(tb + OFF_X + (size_t)r * D + c0 + nr, tag, px, ok);
        const float tot = (sm.rowsum[0][r] + sm.rowsum[1][r]) + (sm.rowsum[2][r] + sm.rowsum[3][r]);
        const float gn = __uint_as_float(px[0]) * (1.0f / sqrtf(tot / (float)D + a.eps)) * bf2f(a.gf[c0 + nr]);
        v2[q] = gn + pre / (1.0f + __expf(-pre));
      }
      ll_st(tb + OFF_RB + ((size_t)r * K + kh) * (D / 2) + (c0 >> 1) + p, pk2(v2[0], v2[1]), tag);
    }
  }

  // ---- UNEMBED over backbone rows and head rows, per-tile top-2 per row ----
  for (int t = w; t < NTV; t += 256) {
    uint4 wv[KD];
    load_frags<KD>(wv, a.WU, t, KTD, wave * KD, lane);
    for (int mt = 0; mt * 16 < rows_all; ++mt) {
      // rows of this m-tile: global row q = mt*16 + r; q < M: backbone row q; else head row q - M
      const int qrow = mt * 16 + r;
      uint4 bfr[KD];
      if (qrow < M) {                       // backbone rows lead tile 0: fragments are at hand
#pragma unroll
        for (int i = 0; i < KD; ++i) bfr[i] = hfrag[i];
      } else {
        uint32_t pw[KD * 4];
        if (qrow < rows_all) {
          ll_wait_groups<KD, 4>(tb + OFF_RB + (size_t)(qrow - M) * (D / 2) + wave * KD * 16 + g * 4, 16, tag, pw, ok);
        } else {
#pragma unroll
          for (int i = 0; i < KD * 4; ++i) pw[i] = 0u;
        }
#pragma unroll
        for (int i = 0; i < KD; ++i) bfr[i] = uint4{pw[4 * i], pw[4 * i + 1], pw[4 * i + 2], pw[4 * i + 3]};
      }
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < KD; ++i)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[i]), __builtin_bit_cast(bf16x8, bfr[i]), acc, 0, 0, 0);
      __syncthreads();
      *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
      __syncthreads();
      // threads 0..15: row qrow = mt*16 + tid; scan the tile's 16 vocabulary entries in order
      if (tid < 16 && mt * 16 + tid < rows_all) {
        const int q = mt * 16 + tid;
        float bv = -INFINITY, sv = -INFINITY;
        int bi = 0;
        float* dbg = nullptr;
        if (q < M) { if (a.logits_dbg) dbg = a.logits_dbg + (size_t)q * V; }
        else if (a.head_logits_dbg) {
          // head rows are ordered (m, k); the debug array wants the heads of the accepted row only,
          // which is not known yet: the full [M][K][V] block is written to the workspace copy
          dbg = a.head_all_dbg + (size_t)(q - M) * V;
        }
#pragma unroll
        for (int nr = 0; nr < 16; ++nr) {
          const int ln = (nr >> 2) * 16 + tid, ii = nr & 3;
          const float z = (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
          if (dbg) dbg[t * 16 + nr] = z;
          if (z > bv) { sv = bv; bv = z; bi = t * 16 + nr; }
          else sv = fmaxf(sv, z);
        }
        uint64_t* st = tb + OFF_ST + ((size_t)t * 80 + q) * 4;
        ll_st(st, __float_as_uint(bv), tag);
        ll_st(st + 1, (uint32_t)bi, tag);
        ll_st(st + 2, __float_as_uint(sv), tag);
      }
    }
  }

  // ---- FINAL: workgroup b finishes sequence b ----
  if (w < a.n_seq) {
    const int b = w;
    const int n = sm.len[b];
    // global top-2 of rows: backbone rows b*R + j (j < R) and head rows ((b*R + j)*K + k)
    const int nrows_b = R + R * K;
    for (int q = wave; q < nrows_b; q += 4) {
      const int grow = q < R ? b * R + q : M + (b * R + (q - R) / K) * K + (q - R) % K;
      float bv = -INFINITY, sv = -INFINITY;
      int bi = 0x7FFFFFFF;
      for (int t = lane; t < NTV; t += 64) {
        uint32_t pw[3];
        ll_wait<3>(tb + OFF_ST + ((size_t)t * 80 + grow) * 4, tag, pw, ok);
        const float tv = __uint_as_float(pw[0]), ts = __uint_as_float(pw[2]);
        const int ti = (int)pw[1];
        if (tv > bv || (tv == bv && ti < bi)) { sv = fmaxf(bv, fmaxf(sv, ts)); bv = tv; bi = ti; }
        else sv = fmaxf(sv, fmaxf(tv, ts));
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float bv2 = __shfl_xor(bv, o, WAVE), sv2 = __shfl_xor(sv, o, WAVE);
        const int bi2 = __shfl_xor(bi, o, WAVE);
        const bool take = (bv2 > bv) || (bv2 == bv && bi2 < bi);
        sv = fmaxf(fmaxf(sv, sv2), fminf(bv, bv2));
        if (take) { bv = bv2; bi = bi2; }
      }
      if (lane == 0) { sm.st_max[q] = bv; sm.st_sec[q] = sv; sm.st_idx[q] = bi; }
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t fl = sm.flag[b];
      if (n < 0) {
        a.n_accepted[b] = 0;
        a.flags[b] = fl;
      } else {
        int acc_n = 0;
        for (int j = 1; j <= K; ++j) {                    // accept while the candidate is the argmax
          const bool hit = a.block[b * R + j] == sm.st_idx[j - 1];
          if (sm.st_max[j - 1] - sm.st_sec[j - 1] <= kTieMarginS) fl |= XSM_FLAG_NEAR_TIE;
          if (!hit) break;
          ++acc_n;
        }
        if (sm.st_max[acc_n] - sm.st_sec[acc_n] <= kTieMarginS) fl |= XSM_FLAG_NEAR_TIE;
        int oldb[16];
        for (int j = 0; j < R; ++j) oldb[j] = a.block[b * R + j];
        const int y0 = sm.st_idx[acc_n];
        for (int j = 0; j < acc_n; ++j) a.out_tokens[b * R + j] = oldb[j + 1];
        a.out_tokens[b * R + acc_n] = y0;
        for (int j = acc_n + 1; j < R; ++j) a.out_tokens[b * R + j] = -1;
        a.block[b * R] = y0;
        for (int k = 0; k < K; ++k) {
          const int q = R + acc_n * K + k;
          a.block[b * R + 1 + k] = sm.st_idx[q];
          if (sm.st_max[q] - sm.st_sec[q] <= kTieMarginS) fl |= XSM_FLAG_NEAR_TIE;
        }
        a.n_accepted[b] = acc_n + 1;
        a.kv_len[b] = n + acc_n + 1;
        a.flags[b] = fl;
        if (a.acc_out) a.acc_out[b] = acc_n;
      }
    }
  }
  if (__syncthreads_or(!ok)) {
    if (tid == 0) __hip_atomic_store(a.ctrl + 1, 1000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }
  // workgroup 0 closes the step: its FINAL needed every workgroup's statistics, so every
  // workgroup has long since read the epoch
  if (w == 0 && tid == 0)
    __hip_atomic_store(a.ctrl, tag + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

size_t small_ll_words(int n_layers, int D, int F, int K) {
  const size_t layer = (size_t)6 * 16 * D + (size_t)16 * (F / 2) + (size_t)256 * 1056;
  const size_t tail = (size_t)16 * D + (size_t)16 * 15 * (D / 2) + (size_t)4096 * 80 * 4;
  (void)K;
  return layer * n_layers + (tail > layer ? tail : layer);
}
size_t small_ll_layer_stride(int D, int F) {
  return (size_t)6 * 16 * D + (size_t)16 * (F / 2) + (size_t)256 * 1056;
}

bool small_supported(int D, int F) { return D == 1024 && F == 4096; }

void launch_step_small(const SmallArgs& a, int D, int F, hipStream_t s) {
  TraceScope trace_("step_small", s);
  if (D == 1024 && F == 4096)
    hipLaunchKernelGGL((k_step_small<1024, 4096>), dim3(256), dim3(256), 0, s, a);
}

}  // namespace xsm
