// One speculative (or plain) decoding step as ONE persistent kernel, for the
// latency regime: at most 16 block rows in total (batch x (K+1) <= 16), bf16,
// d_model 1024 / FFN 4096 / head_dim 64 models, greedy verification.
//
// At batch 1 a step streams every weight once (hundreds of MB) through ~150 dependent
// stages of a few MB each, so what bounds it is not bandwidth inside a stage but the
// latency of handing a few KB of activations from one stage's producers to the next
// stage's consumers.  Kernel boundaries cost several microseconds each; here all 256
// workgroups (one per compute unit) stay resident for the whole step and exchange
// activations through memory with a flag in every 8-byte word:
//     word = { 32-bit payload (one fp32 value), 32-bit tag }, tag = step epoch.
// A producer writes words with device-coherent stores; a consumer loads the words it
// needs with device-coherent loads and retries until every tag equals the current
// epoch, so arrival of the data IS the synchronisation (no barrier, no second round
// trip).  Each (layer, stage) owns its own buffer, so there is no reuse hazard inside a
// step; the epoch makes last step's contents invalid.  Every wait is bounded: a
// workgroup that does not see its inputs within the spin budget raises the error word
// and leaves, and so does every workgroup waiting on it.
//
// Coherent loads bypass the caches, so they are issued fully coalesced (a wavefront reads
// 1 KB of consecutive words) and the activation block is re-laid through LDS into MFMA
// operand order; a lane-scattered read of the same words costs an order of magnitude more.
//
// Activations travel as fp32 and enter the bf16 MFMAs as two operands, hi = bf16(x) and
// lo = bf16(x - hi), against the same weight fragment, so the result carries the weights'
// bf16 rounding (part of the model) but not a second one from the activations.
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
//   DOWN  64 tiles x 4 slices of the FFN width: W2 partial products on all 256 workgroups;
//         the workgroup of the last slice (which also made the tile's OPROJ output) adds the
//         other three and the residual
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
// 16 bytes per lane from global memory straight into LDS: lane l's piece lands at lds + 16 l
__device__ __forceinline__ void lds_direct16(const void* gptr, void* lds) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds, 16, 0, 0);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// raw buffer descriptor word 3 (32-bit data format, no swizzle) and the cache-policy bits of a
// load that is coherent across the device (sc1)
constexpr int kRawBufferFlags = 0x00020000, kCoherentLoad = 16;

constexpr int kQS = 72;                     // LDS row stride (bf16) of the attention q / new-k / new-v tiles

__device__ __forceinline__ uint64_t ll_ld(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_st(uint64_t* p, uint32_t payload, uint32_t tag) {
  __hip_atomic_store(p, ((uint64_t)tag << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t pk2(float a, float b) { return f2bf_pair(a, b); }
__device__ __forceinline__ float lo_bf(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Wait for the tagged words at p + off[i] (entries with off[i] < 0 are skipped); payloads to
// out.  Meant for small blocks: the words are simply re-read together until every tag
// matches, one round trip from arrival to use.  On timeout, or when an earlier wait of this
// lane already failed, ok is false and out is zero.
template <int N>
__device__ __forceinline__ void ll_wait_list(const uint64_t* p, const int (&off)[N], uint32_t tag,
                                             uint32_t (&out)[N], bool& ok) {
  bool any = false;
#pragma unroll
  for (int i = 0; i < N; ++i) any |= off[i] >= 0;
  if (ok && any) {
    for (int spin = 0; spin < kSpinBudget; ++spin) {
      uint64_t w[N];
#pragma unroll
      for (int i = 0; i < N; ++i)
        if (off[i] >= 0) w[i] = ll_ld(p + off[i]);
      bool good = true;
#pragma unroll
      for (int i = 0; i < N; ++i)
        if (off[i] >= 0) good &= (uint32_t)(w[i] >> 32) == tag;
      if (good) {
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = off[i] >= 0 ? (uint32_t)w[i] : 0u;
        return;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    ok = false;
  }
#pragma unroll
  for (int i = 0; i < N; ++i) out[i] = 0u;
}
__device__ __forceinline__ uint32_t ll_wait1(const uint64_t* p, uint32_t tag, bool& ok) {
  const int off[1] = {0};
  uint32_t out[1];
  ll_wait_list<1>(p, off, tag, out, ok);
  return out[0];
}

// The same for pairs of adjacent words (even word offsets off[i], < 0: skipped) of a block of
// nbytes bytes at p: each pair is one 16-byte device-coherent load, payloads to out[2i], out[2i+1].
template <int N>
__device__ __forceinline__ void ll_wait_pairs(const uint64_t* p, int nbytes, const int (&off)[N], uint32_t tag,
                                              uint32_t (&out)[2 * N], bool& ok) {
  bool any = false;
#pragma unroll
  for (int i = 0; i < N; ++i) any |= off[i] >= 0;
  if (ok && any) {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint64_t*>(p), 0, nbytes, kRawBufferFlags);
    for (int spin = 0; spin < kSpinBudget; ++spin) {
      u32x4 q[N];
#pragma unroll
      for (int i = 0; i < N; ++i)
        if (off[i] >= 0) q[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off[i] * 8, 0, kCoherentLoad);
      bool good = true;
#pragma unroll
      for (int i = 0; i < N; ++i)
        if (off[i] >= 0) good &= q[i].y == tag && q[i].w == tag;
      if (good) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
          out[2 * i] = off[i] >= 0 ? q[i].x : 0u;
          out[2 * i + 1] = off[i] >= 0 ? q[i].z : 0u;
        }
        return;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    ok = false;
  }
#pragma unroll
  for (int i = 0; i < 2 * N; ++i) out[i] = 0u;
}

// Every poll of a word that another XCD is about to write costs fabric traffic that slows the
// writes everybody is waiting for, so a workgroup polls with one lane: it watches one word of the
// block until it carries the tag while the rest sit at the barrier; the block is read afterwards
// (and re-read in the rare case that other producers' words lag).  Must be reached by every
// thread of the workgroup.
__device__ __forceinline__ void watch_then_sync(const uint64_t* word, uint32_t tag, bool active, int tid) {
  if (tid == 0 && active) {
    int spin = 0;
    while ((uint32_t)(ll_ld(word) >> 32) != tag && ++spin < kSpinBudget) __builtin_amdgcn_s_sleep(1);
  }
  __syncthreads();
}

// Cooperative, coalesced wait for rows [m0, m0 + ROWS) (clipped to nrows), W words of each, of a
// block of tagged words with row stride RS: thread t takes the word pairs 2(t + 256 j), +1, j < W/512, of
// every row, so a wavefront instruction covers 1 KB of consecutive words.
template <int W, int RS, int ROWS>
__device__ __forceinline__ void coop_wait(const uint64_t* buf, int m0, int nrows, int tid, uint32_t tag,
                                          uint32_t (&pay)[ROWS * (W / 512) * 2], bool& ok, uint64_t* stamp = nullptr) {
  constexpr int PP = W / 512, N = ROWS * PP * 2;
  const int rows = min(ROWS, nrows - m0);
  const uint64_t* base = buf + (size_t)m0 * RS + 2 * tid;
  // (later rounds of a block come from the same producers as its first rows: no watch, its poll
  // would be one more round trip in front of the read)
  if (m0 == 0) watch_then_sync(base + (size_t)(rows > 0 ? rows - 1 : 0) * RS + (PP - 1) * 512 + 1, tag, ok && rows > 0, tid);
  if (stamp && tid == 0) stamp[0] = wall_clock64();
  if (ok && rows > 0) {
    // a thread's two adjacent words travel as one 16-byte device-coherent load (each word is
    // validated by its own tag, so the pair needs no atomicity of its own)
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint64_t*>(buf + (size_t)m0 * RS), 0, rows * RS * 8, kRawBufferFlags);
    int spin = 0;
    for (; spin < kSpinBudget; ++spin) {
      u32x4 q[N / 2];                                     // {payload, tag, payload, tag}
#pragma unroll
      for (int m = 0; m < ROWS; ++m)
#pragma unroll
        for (int j = 0; j < PP; ++j)
          if (m < rows)
            q[m * PP + j] = __builtin_amdgcn_raw_buffer_load_b128(rs, ((m * RS + j * 512 + 2 * tid) * 8), 0, kCoherentLoad);
      bool good = true;
#pragma unroll
      for (int m = 0; m < ROWS; ++m)
#pragma unroll
        for (int j = 0; j < PP; ++j)
          if (m < rows) good &= q[m * PP + j].y == tag && q[m * PP + j].w == tag;
      if (good) {
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
          pay[2 * i] = (i / PP) < rows ? q[i].x : 0u;
          pay[2 * i + 1] = (i / PP) < rows ? q[i].z : 0u;
        }
        if (stamp && tid == 0) stamp[1] = wall_clock64();
        return;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    ok = false;
  }
#pragma unroll
  for (int i = 0; i < N; ++i) pay[i] = 0u;
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
  float st_max[kSmallMaxRows], st_sec[kSmallMaxRows];  // FINAL: per-row reductions
  int st_idx[kSmallMaxRows];
  LayerTab tab[48];
};

// Sum the four wavefronts' partial 16x16 tiles; thread t gets element D[column t % 16][row t / 16],
// so that the 16 words of one row's tile leave in one 128-byte store.
__device__ __forceinline__ float tile_reduce(Shared& sm, f32x4 acc, int wave, int lane, int tid) {
  __syncthreads();
  *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
  __syncthreads();
  const int oc = tid & 15, om = tid >> 4;
  const int ln = (oc >> 2) * 16 + om, ii = oc & 3;        // MFMA lane and slot that hold D[oc][om]
  return (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
}

// bf16 pair of (a, b) and of what that rounding dropped
__device__ __forceinline__ void split2(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  hi = pk2(x0, x1);
  lo = pk2(x0 - lo_bf(hi), x1 - hi_bf(hi));
}

// Stage nrows rows, D columns each, of an fp32-payload block with row stride RS words into LDS
// rows dst_row.. as two bf16 planes of row stride D + 8: hi at As, lo at As + 16 * (D + 8).
// NORM 1: RMSNorm over the D columns with the gain pairs gpair[j] (columns 2(tid + 256 j), +1).
// NORM 2: only the gains are applied and the rows' sums of squares are left in sm.rowsum[.][row];
// the caller multiplies its products by row_scale(row) - the rows reach LDS without waiting for
// the sums to be exchanged.
template <int D, int RS, int NORM>
__device__ __forceinline__ void stage_rows_f32(Shared& sm, uint16_t* As, int dst_row, const uint64_t* buf,
                                               int nrows, const uint32_t (&gpair)[D / 512], float eps, int tid,
                                               uint32_t tag, bool& ok, uint64_t* stamp = nullptr) {
  constexpr int PP = D / 512, ST = D + 8, LO = 16 * ST;
  constexpr int RB = PP >= 4 ? 4 : 8;                    // rows per round: at most 32 words in flight per thread
  const int wave = tid >> 6, lane = tid & 63;
  for (int m0 = 0; m0 < nrows; m0 += RB) {
    uint32_t pay[RB * PP * 2];
    coop_wait<D, RS, RB>(buf, m0, nrows, tid, tag, pay, ok, stamp);
    if (NORM) {
      if (NORM == 1 && m0 > 0) __syncthreads();          // this call's earlier readers of rowsum are done
      // eight row sums per wavefront in ten lane exchanges instead of forty-eight: each exchange
      // step halves the rows a lane carries (lane bits 5, 4, 3 pick the row), then three steps
      // finish the one row left.  Cross-lane moves cost LDS-like latency at one wavefront per SIMD.
      static_assert(RB == 8, "row-sum exchange is written for eight rows");
      float ss[8];
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        ss[m] = 0.f;
#pragma unroll
        for (int j = 0; j < PP * 2; ++j) {
          const float x = __uint_as_float(pay[m * PP * 2 + j]);
          ss[m] += x * x;
        }
      }
      const bool b5 = lane & 32, b4 = lane & 16, b3 = lane & 8;
      float s4[4], s2[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) s4[i] = (b5 ? ss[4 + i] : ss[i]) + lane_xor<32>(b5 ? ss[i] : ss[4 + i]);
#pragma unroll
      for (int i = 0; i < 2; ++i) s2[i] = (b4 ? s4[2 + i] : s4[i]) + lane_xor<16>(b4 ? s4[i] : s4[2 + i]);
      float s1 = (b3 ? s2[1] : s2[0]) + lane_xor<8>(b3 ? s2[0] : s2[1]);
      s1 += lane_xor<4>(s1);
      s1 += lane_xor<2>(s1);
      s1 += lane_xor<1>(s1);
      if ((lane & 7) == 0) sm.rowsum[wave][(NORM == 2 ? m0 : 0) + (b5 ? 4 : 0) + (b4 ? 2 : 0) + (b3 ? 1 : 0)] = s1;
      if (NORM == 1) __syncthreads();
    }
    // every thread forms the scales itself, all rows at once (hardware reciprocal square root, 1 ulp)
    float scl[RB];
#pragma unroll
    for (int m = 0; m < RB; ++m)
      scl[m] = NORM == 1 ? __builtin_amdgcn_rsqf(((sm.rowsum[0][m] + sm.rowsum[1][m]) + (sm.rowsum[2][m] + sm.rowsum[3][m])) * (1.0f / (float)D) + eps)
                    : 1.0f;
#pragma unroll
    for (int m = 0; m < RB; ++m) {
      if (m0 + m < nrows) {
        const float sc = scl[m];
#pragma unroll
        for (int j = 0; j < PP; ++j) {
          float x0 = __uint_as_float(pay[(m * PP + j) * 2]), x1 = __uint_as_float(pay[(m * PP + j) * 2 + 1]);
          if (NORM == 1) { x0 *= sc * lo_bf(gpair[j]); x1 *= sc * hi_bf(gpair[j]); }
          if (NORM == 2) { x0 *= lo_bf(gpair[j]); x1 *= hi_bf(gpair[j]); }
          uint32_t hi, lo;
          split2(x0, x1, hi, lo);
          uint16_t* dst = As + (size_t)(dst_row + m0 + m) * ST + 2 * (tid + 256 * j);
          *reinterpret_cast<uint32_t*>(dst) = hi;
          *reinterpret_cast<uint32_t*>(dst + LO) = lo;
        }
      }
    }
  }
  __syncthreads();
}

// 1 / rms of a row staged with NORM 2 (hardware reciprocal square root, 1 ulp)
template <int D>
__device__ __forceinline__ float row_scale(const Shared& sm, int row, float eps) {
  return __builtin_amdgcn_rsqf(((sm.rowsum[0][row] + sm.rowsum[1][row]) + (sm.rowsum[2][row] + sm.rowsum[3][row])) * (1.0f / (float)D) + eps);
}

// acc = sum_i Wfrag[i] . (hi + lo) over k-tiles kt0 .. kt0 + N - 1 of activation row `row` of an
// LDS tile staged by stage_rows_f32 (row stride ST, lo plane 16 rows further).  All operand
// fragments are requested from LDS before the first product (the scheduler otherwise sinks every
// read next to its use, and each product then waits out a full LDS round trip), and the hi and lo
// products run as two independent accumulation chains.
template <int N>
__device__ __forceinline__ f32x4 mac_tiles(const uint4 (&wf)[N], const uint16_t* As, int ST, int row, int kt0, int g) {
  const uint16_t* p = As + (size_t)row * ST + kt0 * 32 + g * 8;
  uint4 bh[N], bl[N];
#pragma unroll
  for (int i = 0; i < N; ++i) {
    bh[i] = *reinterpret_cast<const uint4*>(p + i * 32);
    bl[i] = *reinterpret_cast<const uint4*>(p + i * 32 + 16 * ST);
  }
  __builtin_amdgcn_sched_barrier(0);
  f32x4 a0 = f32x4{0.f, 0.f, 0.f, 0.f}, a1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const bf16x8 wa = __builtin_bit_cast(bf16x8, wf[i]);
    a0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, bl[i]), a0, 0, 0, 0);
    a1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, bh[i]), a1, 0, 0, 0);
  }
  return a0 + a1;
}

}  // namespace

template <int D, int F>
__global__ __launch_bounds__(256) void k_step_small(const SmallArgs a) {
  constexpr int H = D / 64;
  constexpr int KTD = D / 32, KTF = F / 32;          // k-tiles of the two contraction lengths
  constexpr int KD = KTD / 4;                        // per wavefront
  constexpr int NQ = 3 * D / 16, NO = D / 16, NU = F / 16;
  constexpr int O_BASE = NQ;
  constexpr int FS = F / 4;                          // DOWN: slice of the FFN width per workgroup
  constexpr int KFS = FS / 32 / 4;                   // its k-tiles per wavefront
  constexpr int STD = D + 8, STS = FS + 8;           // LDS row strides (bf16 elements)
  static_assert(NQ + NO <= 256 && NU <= 256 && NO * 4 == 256, "tile roles must fit 256 workgroups");
  static_assert(FS % 512 == 0 && FS <= D, "DOWN slice is staged like a model-width row block");
  static_assert(D % 512 == 0 && F % 1024 == 0, "cooperative staging needs whole pair rounds");
  __shared__ Shared sm;
  extern __shared__ __align__(16) unsigned char dyn[];
  uint16_t* const As = reinterpret_cast<uint16_t*>(dyn);     // activation tile(s), several layouts

  const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int R = a.R, K = R - 1, M = a.n_seq * R, V = a.V;

  // ---- set-up: epoch, layer table, per-sequence validation (every workgroup, redundantly) ----
  if (tid == 0) {
    sm.tag = __hip_atomic_load(a.ctrl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm.fail = (int)__hip_atomic_load(a.ctrl + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  for (int i = tid; i < a.L * (int)(sizeof(LayerTab) / 8); i += 256)
    reinterpret_cast<uint64_t*>(sm.tab)[i] = reinterpret_cast<const uint64_t*>(a.layers)[i];
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
  // A bounded wait gave up, in this step or an earlier one: sequence b produced nothing.  The
  // caller sees it in the step's own outputs (n_accepted 0, the timeout flag), and the verify /
  // emit kernels that follow a deferred step skip the sequence.
  auto report_timeout = [&](int b) {
    const uint32_t f = sm.flag[b] | XSM_FLAG_DEVICE_TIMEOUT;
    a.n_accepted[b] = 0;
    a.flags[b] = f;
    if (a.eff_out) { a.eff_out[b] = -1; a.wflags_out[b] = f; }
  };
  if (sm.fail != 0) {                       // an earlier step timed out: stay down until reset
    if (w < a.n_seq && tid == 0) report_timeout(w);
    return;
  }
  const uint32_t tag = sm.tag;
  // Key slices per (sequence, head), from the longest live cache (every workgroup reads the same
  // lengths, so all agree).  The cached keys and values come from HBM at full memory latency and a
  // workgroup has at most 128 KB of them in flight, so the attention stage is as fast as the
  // number of workgroups sharing a key range: measured at contexts 100..4353, 8 slices win from
  // three 64-key chunks on (even with most slices empty and the merge stage added), 16 from about
  // twenty chunks on.
  int S = a.S;
  if (a.s_auto) {
    int longest = 0;
    for (int b = 0; b < a.n_seq; ++b) longest = max(longest, sm.len[b]);
    const int chunks = (longest + 63) >> 6;
    const int want = chunks <= 2 ? 1 : chunks <= 20 ? 8 : 16;
    while (S > want) S >>= 1;
  }
  // this lane's activation row (MFMA column) m = r
  // the output element this thread finishes after tile_reduce: tile column nrow of row om
  const int om = tid >> 4, nrow = tid & 15;
  const int mb = om / R, mj = om % R;
  const bool row_in = om < M;
  const int len_m = row_in ? sm.len[mb] : -1;
  const bool live = row_in && len_m >= 0;              // rows of skipped sequences carry zeros

  const size_t LS = a.ll_layer_stride;                 // words per layer
  uint64_t* const llb = a.ll;
  const size_t OFF_X = 0, OFF_Q = 16 * D, OFF_KN = 2 * 16 * D, OFF_VN = 3 * 16 * D, OFF_O = 4 * 16 * D,
               OFF_XM = 5 * 16 * D, OFF_U = 6 * 16 * D, OFF_PD = OFF_U + 16 * F, OFF_P = OFF_PD + 3 * 16 * D;

  const bool has_q = w < NQ, has_o = w >= O_BASE && w < O_BASE + NO, has_u = w < NU;
  const int d_nt = w % NO, d_ks = w / NO;              // DOWN: output tile and slice of the FFN width
  // Weight fragments live in registers and are requested ahead of use.  A wavefront's loads
  // return in order, so a bulk request delays whatever wait is issued right behind it; each
  // request is therefore placed where its workgroup is about to sit out a stage:
  //   workgroups with a QKV tile: this layer's UP and DOWN tiles and next layer's QKV tile after
  //     COMB - they have no OPROJ tile;
  //   the OPROJ workgroups: next layer's OPROJ, UP and DOWN tiles after DOWN - they sit out QKV
  //     and attention.
  uint4 wq[KD], wu[KD], wd[KFS];           // wq doubles as the OPROJ tile (disjoint workgroups)
  auto load_down = [&](const uint4* W2) { load_frags<KFS>(wd, W2, d_nt, KTF, d_ks * (FS / 32) + wave * KFS, lane); };
  if (has_q) load_frags<KD>(wq, sm.tab[0].Wqkv, w, KTD, wave * KD, lane);
  if (has_o) {
    load_frags<KD>(wq, sm.tab[0].Wo, w - O_BASE, KTD, wave * KD, lane);
    load_frags<KD>(wu, sm.tab[0].W1, w, KTD, wave * KD, lane);
    load_down(sm.tab[0].W2);
  }
  float xm = 0.f;                          // OPROJ workgroups: their element of the mid-layer residual

  // ---- EMBED: layer-0 residual rows as tagged words ----
  for (int idx = w * 256 + tid; idx < M * D; idx += 256 * 256) {
    const int m = idx / D, c = idx % D, b = m / R;
    const float x = sm.len[b] >= 0 ? bf2f(a.E[(size_t)a.block[m] * D + c]) : 0.f;
    ll_st(llb + OFF_X + (size_t)m * D + c, __float_as_uint(x), tag);
  }

  // optional timeline: thread 0 of every workgroup stamps the 100 MHz clock at stage boundaries
  uint64_t* const tl = a.tlog ? a.tlog + (size_t)w * (a.L * 16 + 8) : nullptr;
#define XSM_STAMP(idx) do { if (tl && tid == 0) tl[idx] = wall_clock64(); } while (0)
  bool ok = true;
  for (int l = 0; l < a.L; ++l) {
    uint64_t* const lb = llb + (size_t)l * LS;
    const LayerTab& lt = sm.tab[l];
    XSM_STAMP(l * 16 + 0);

    // ================= QKV =================
    if (has_q) {
      uint32_t gp[D / 512];                            // gain pairs and rotary entry: requested before waiting
#pragma unroll
      for (int j = 0; j < D / 512; ++j) gp[j] = *reinterpret_cast<const uint32_t*>(lt.g1 + 2 * (tid + 256 * j));
      const int q_sec = w / (D / 16), q_ts = w % (D / 16), q_h = q_ts >> 2, q_tt = q_ts & 3;
      float2 cs = float2{1.f, 0.f};
      if (live && q_sec < 2) cs = a.rope[(size_t)(len_m + mj) * 32 + q_tt * 8 + (nrow & 7)];
      stage_rows_f32<D, D, 2>(sm, As, 0, lb + OFF_X, M, gp, a.eps, tid, tag, ok);
      XSM_STAMP(l * 16 + 8);
      const f32x4 acc = mac_tiles<KD>(wq, As, STD, r, wave * KD, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid) * row_scale<D>(sm, om, a.eps);
      const float partner = lane_xor<8>(v);        // tile column nrow +- 8
      if (live) {
        const int pos = len_m + mj;
        float o = v;
        int dim;
        if (q_sec < 2) {
          const int pi = q_tt * 8 + (nrow & 7);
          if (nrow < 8) { dim = pi; o = v * cs.x - partner * cs.y; }
          else { dim = 32 + pi; o = partner * cs.y + v * cs.x; }
        } else {
          dim = q_tt * 16 + nrow;
        }
        const size_t col = (size_t)om * D + q_h * 64 + dim;
        const size_t head = (size_t)sm.slot[mb] * H + q_h;
        if (q_sec == 0) {
          ll_st(lb + OFF_Q + col, __float_as_uint(o), tag);
        } else if (q_sec == 1) {
          ll_st(lb + OFF_KN + col, __float_as_uint(o), tag);
          lt.Kc[(head * a.cap + pos) * 64 + dim] = f2bf(o);
        } else {
          ll_st(lb + OFF_VN + col, __float_as_uint(o), tag);
          lt.Vt[(head * 64 + dim) * a.cap + pos] = f2bf(o);
        }
      }
    }
    XSM_STAMP(l * 16 + 1);

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
      // this step's q, k, v rows of (sequence b, head h): [R][64] each, staged as bf16 tiles
      uint16_t* const qs = As;                            // q: hi plane, lo plane 16 rows further
      uint16_t* const kns = As + 32 * kQS;                // new k / v: as the cache will hold them
      uint16_t* const vns = As + 48 * kQS;
      // the first chunk of cached keys/values does not depend on this step: request it before waiting.
      // While a wavefront works on one chunk, the next one is on its way from HBM straight into LDS
      // (LDS-direct loads: no registers - a second register set for it spills - and lane l's 16
      // bytes of a request land at base + 16 l, i.e. already in fragment order), 16 KB per wavefront
      unsigned char* const ring = dyn + 16384 + wave * 16384;
      uint4 kf[4][2], vf[4][2];
      auto load_k = [&](int c) {
        const int key0 = c << 6;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint16_t* kr = kb + (size_t)(key0 + (r >> 2) * 16 + t * 4 + (r & 3)) * 64 + g * 8;
          kf[t][0] = *reinterpret_cast<const uint4*>(kr);
          kf[t][1] = *reinterpret_cast<const uint4*>(kr + 32);
        }
      };
      auto load_v = [&](int c) {
        const int key0 = c << 6;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const uint16_t* vr = vb + (size_t)(dt * 16 + r) * a.cap + key0 + g * 16;
          vf[dt][0] = *reinterpret_cast<const uint4*>(vr);
          vf[dt][1] = *reinterpret_cast<const uint4*>(vr + 8);
        }
      };
      auto request_next = [&](int c) {
        const int key0 = c << 6;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint16_t* kr = kb + (size_t)(key0 + (r >> 2) * 16 + t * 4 + (r & 3)) * 64 + g * 8;
          lds_direct16(kr, ring + (t * 2) * 1024);
          lds_direct16(kr + 32, ring + (t * 2 + 1) * 1024);
        }
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const uint16_t* vr = vb + (size_t)(dt * 16 + r) * a.cap + key0 + g * 16;
          lds_direct16(vr, ring + 8192 + (dt * 2) * 1024);
          lds_direct16(vr + 8, ring + 8192 + (dt * 2 + 1) * 1024);
        }
      };
      auto take_next = [&]() {                              // (waits for the requests above)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            kf[t][j] = *reinterpret_cast<const uint4*>(ring + (t * 2 + j) * 1024 + lane * 16);
            vf[t][j] = *reinterpret_cast<const uint4*>(ring + 8192 + (t * 2 + j) * 1024 + lane * 16);
          }
      };
      if (c_lo + wave < c_hi) { load_k(c_lo + wave); load_v(c_lo + wave); }
      if (c_lo + wave + 4 < c_hi) request_next(c_lo + wave + 4);   // the wavefront's second chunk too
      watch_then_sync(lb + OFF_VN + (size_t)(b * R + R - 1) * D + h * 64 + 63, tag, ok && n >= 0, tid);
      if (n >= 0) {
        const int j0 = tid >> 5, c = 2 * (tid & 31);      // rows j0, j0+8; columns c, c+1 as one word pair
        int off[6];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int j = j0 + 8 * q;
          const int base = (b * R + j) * D + h * 64 + c;
          off[3 * q] = j < R ? (int)OFF_Q + base : -1;
          off[3 * q + 1] = j < R ? (int)OFF_KN + base : -1;
          off[3 * q + 2] = j < R ? (int)OFF_VN + base : -1;
        }
        uint32_t pw[12];
        ll_wait_pairs<6>(lb, (int)OFF_U * 8, off, tag, pw, ok);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int j = j0 + 8 * q;
          if (j < R) {
            uint32_t qh, ql;
            split2(__uint_as_float(pw[6 * q]), __uint_as_float(pw[6 * q + 1]), qh, ql);
            *reinterpret_cast<uint32_t*>(qs + j * kQS + c) = qh;
            *reinterpret_cast<uint32_t*>(qs + (16 + j) * kQS + c) = ql;
            *reinterpret_cast<uint32_t*>(kns + j * kQS + c) = pk2(__uint_as_float(pw[6 * q + 2]), __uint_as_float(pw[6 * q + 3]));
            *reinterpret_cast<uint32_t*>(vns + j * kQS + c) = pk2(__uint_as_float(pw[6 * q + 4]), __uint_as_float(pw[6 * q + 5]));
          }
        }
      }
      __syncthreads();
      XSM_STAMP(l * 16 + 9);
      const bool qlive = r < R && n >= 0;                 // MFMA column r is query j = r
      bf16x8 qh[2], ql[2];                                // dims g*8.. and 32 + g*8.., hi and lo parts
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        qh[hf] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qs + r * kQS + hf * 32 + g * 8));
        ql[hf] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qs + (16 + r) * kQS + hf * 32 + g * 8));
      }
      float m_run = -INFINITY, l_run = 0.f;
      f32x4 o[4];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

      // cached keys 0..n-1: every live query sees all of them
      for (int c = c_lo + wave; c < c_hi; c += 4) {
        const int key0 = c << 6;
        const bool more = c + 4 < c_hi;
        if (more && c != c_lo + wave) request_next(c + 4);
        f32x4 sc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            const bf16x8 kk = __builtin_bit_cast(bf16x8, kf[t][hf]);
            sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, ql[hf], sc[t], 0, 0, 0);
            sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, qh[hf], sc[t], 0, 0, 0);
          }
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
        cmax = fmaxf(cmax, lane_xor<16>(cmax));
        cmax = fmaxf(cmax, lane_xor<32>(cmax));
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
        psum += lane_xor<16>(psum);
        psum += lane_xor<32>(psum);
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
        uint4 ph[2], pl[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          split2(sc[2 * jj][0], sc[2 * jj][1], ph[jj].x, pl[jj].x);
          split2(sc[2 * jj][2], sc[2 * jj][3], ph[jj].y, pl[jj].y);
          split2(sc[2 * jj + 1][0], sc[2 * jj + 1][1], ph[jj].z, pl[jj].z);
          split2(sc[2 * jj + 1][2], sc[2 * jj + 1][3], ph[jj].w, pl[jj].w);
        }
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const bf16x8 vv = __builtin_bit_cast(bf16x8, vf[dt][jj]);
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv, __builtin_bit_cast(bf16x8, pl[jj]), o[dt], 0, 0, 0);
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv, __builtin_bit_cast(bf16x8, ph[jj]), o[dt], 0, 0, 0);
          }
        if (more) take_next();
      }

      // the R new keys of this step (positions n..n+R-1): one 16-key tile, taken by wavefront 3
      // of slice 0; query j sees new key i iff i <= j
      if (s == 0 && wave == 3 && n >= 0) {
        // A operand of S^T: lane (key r, g) holds k_new[r][hf*32 + g*8 .. +8]
        const bf16x8 k0 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(kns + r * kQS + g * 8));
        const bf16x8 k1 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(kns + r * kQS + 32 + g * 8));
        f32x4 sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, ql[0], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, ql[1], sc, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qh[0], sc, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qh[1], sc, 0, 0, 0);
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
        cmax = fmaxf(cmax, lane_xor<16>(cmax));
        cmax = fmaxf(cmax, lane_xor<32>(cmax));
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
        psum += lane_xor<16>(psum);
        psum += lane_xor<32>(psum);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        // contraction index of the second product: k = g*8 + e  <->  new key g*4 + e (e < 4)
        uint4 pfh = uint4{0u, 0u, 0u, 0u}, pfl = uint4{0u, 0u, 0u, 0u};
        split2(sc[0], sc[1], pfh.x, pfl.x);
        split2(sc[2], sc[3], pfh.y, pfl.y);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          // A operand: lane (dim dt*16 + r, g) holds v_new[key g*4 + e][dim], e < 4
          uint32_t vw[2] = {0u, 0u};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int key = g * 4 + e;
            const uint32_t x = key < R ? (uint32_t)vns[key * kQS + dt * 16 + r] : 0u;
            vw[e >> 1] |= x << ((e & 1) * 16);
          }
          const uint4 vfrag = uint4{vw[0], vw[1], 0u, 0u};
          o[dt] = o[dt] * alpha;
          o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vfrag),
                                                          __builtin_bit_cast(bf16x8, pfl), o[dt], 0, 0, 0);
          o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vfrag),
                                                          __builtin_bit_cast(bf16x8, pfh), o[dt], 0, 0, 0);
        }
      }

      XSM_STAMP(l * 16 + 10);
      // merge the four wavefronts; wavefront i finishes dim tile i
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
    XSM_STAMP(l * 16 + 2);

    // ================= COMB =================
    if (S > 1 && w < n_units) {
      const int b = w / (H * S), h = (w / S) % H, s = w % S;
      const int dps = 64 / S;                               // dims finished by this unit
      const int P = 32 + dps * 16;                          // words needed from each slice: m, l, O^T rows
      const uint64_t* p0 = lb + OFF_P + (size_t)(w - s) * 1056;
      float* const cb = reinterpret_cast<float*>(As);       // [S][P]
      watch_then_sync(p0 + (size_t)(S - 1) * 1056 + 32 + (s * dps + dps - 1) * 16, tag, ok, tid);
      {
        // word pairs 2 tid + 512 q of the S x P words (P is even: a pair stays inside one slice)
        int off[3];
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          const int i = 2 * tid + 512 * q;
          const int k = i / P, j = i % P;
          off[q] = i < S * P ? k * 1056 + (j < 32 ? j : 32 + s * dps * 16 + (j - 32)) : -1;
        }
        uint32_t pw[6];
        ll_wait_pairs<3>(p0, S * 1056 * 8, off, tag, pw, ok);
#pragma unroll
        for (int q = 0; q < 3; ++q)
          if (off[q] >= 0) {
            cb[2 * tid + 512 * q] = __uint_as_float(pw[2 * q]);
            cb[2 * tid + 512 * q + 1] = __uint_as_float(pw[2 * q + 1]);
          }
      }
      __syncthreads();
      for (int qd = tid >> 4; qd < dps; qd += 16) {
        const int rq = tid & 15;
        if (rq < R) {
          float Mg = -INFINITY;
          for (int k = 0; k < S; ++k) Mg = fmaxf(Mg, cb[k * P + rq]);
          float Lg = 0.f, og = 0.f;
          for (int k = 0; k < S; ++k) {
            const float mk = cb[k * P + rq];
            const float f = mk == -INFINITY ? 0.f : exp2f(mk - Mg);
            Lg += cb[k * P + 16 + rq] * f;
            og += cb[k * P + 32 + qd * 16 + rq] * f;
          }
          const float outv = sm.len[b] >= 0 ? og / Lg : 0.f;
          ll_st(lb + OFF_O + (size_t)(b * R + rq) * D + h * 64 + s * dps + qd, __float_as_uint(outv), tag);
        }
      }
    }
    XSM_STAMP(l * 16 + 3);
    if (has_q) {
      load_frags<KD>(wu, lt.W1, w, KTD, wave * KD, lane);
      load_down(lt.W2);
      if (l + 1 < a.L) load_frags<KD>(wq, sm.tab[l + 1].Wqkv, w, KTD, wave * KD, lane);
    }

    // ================= OPROJ =================
    if (has_o) {
      const int nt = w - O_BASE;
      // residual entering the layer: published a stage ago
      const uint32_t px = row_in ? ll_wait1(lb + OFF_X + (size_t)om * D + nt * 16 + nrow, tag, ok) : 0u;
      const uint32_t nogain[D / 512] = {};
      __syncthreads();
      stage_rows_f32<D, D, 0>(sm, As, 0, lb + OFF_O, M, nogain, a.eps, tid, tag, ok);
      XSM_STAMP(l * 16 + 14);
      const f32x4 acc = mac_tiles<KD>(wq, As, STD, r, wave * KD, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid);
      xm = __uint_as_float(px) + v;
      if (row_in) ll_st(lb + OFF_XM + (size_t)om * D + nt * 16 + nrow, __float_as_uint(xm), tag);
    }
    XSM_STAMP(l * 16 + 4);

    // ================= UP =================
    if (has_u) {
      uint32_t gp[D / 512];
#pragma unroll
      for (int j = 0; j < D / 512; ++j) gp[j] = *reinterpret_cast<const uint32_t*>(lt.g2 + 2 * (tid + 256 * j));
      __syncthreads();
      stage_rows_f32<D, D, 2>(sm, As, 0, lb + OFF_XM, M, gp, a.eps, tid, tag, ok, tl ? tl + l * 16 + 13 : nullptr);
      XSM_STAMP(l * 16 + 7);
      const f32x4 acc = mac_tiles<KD>(wu, As, STD, r, wave * KD, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid) * row_scale<D>(sm, om, a.eps);
      if (row_in)
        ll_st(lb + OFF_U + (size_t)om * F + w * 16 + nrow,
              __float_as_uint(0.5f * v * (1.0f + erff(v * 0.70710678118654752f))), tag);
    }
    XSM_STAMP(l * 16 + 5);

    // ================= DOWN =================
    {
      const uint32_t nogain[FS / 512] = {};
      __syncthreads();
      stage_rows_f32<FS, F, 0>(sm, As, 0, lb + OFF_U + d_ks * FS, M, nogain, a.eps, tid, tag, ok);
      XSM_STAMP(l * 16 + 12);
      const f32x4 acc = mac_tiles<KFS>(wd, As, STS, r, wave * KFS, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid);
      const size_t col = (size_t)om * D + d_nt * 16 + nrow;
      if (d_ks < 3) {
        if (row_in) ll_st(lb + OFF_PD + (size_t)d_ks * 16 * D + col, __float_as_uint(v), tag);
      } else {
        // last slice: the other three partial products, then the residual this workgroup made in OPROJ
        const int off[3] = {row_in ? (int)col : -1, row_in ? (int)(16 * D + col) : -1, row_in ? (int)(32 * D + col) : -1};
        uint32_t pw[3];
        watch_then_sync(lb + OFF_PD + (size_t)32 * D + d_nt * 16, tag, ok, tid);
        ll_wait_list<3>(lb + OFF_PD, off, tag, pw, ok);
        const float x = xm + ((__uint_as_float(pw[0]) + __uint_as_float(pw[1])) + (__uint_as_float(pw[2]) + v));
        if (row_in) ll_st(lb + LS + OFF_X + col, __float_as_uint(x), tag);
      }
    }
    XSM_STAMP(l * 16 + 6);
    if (has_o && l + 1 < a.L) {
      load_frags<KD>(wq, sm.tab[l + 1].Wo, w - O_BASE, KTD, wave * KD, lane);
      load_frags<KD>(wu, sm.tab[l + 1].W1, w, KTD, wave * KD, lane);
      load_down(sm.tab[l + 1].W2);
    }
    // a workgroup that timed out anywhere leaves (its consumers will time out in turn)
    if (__syncthreads_or(!ok)) {
      if (tid == 0) {
        __hip_atomic_store(a.ctrl + 1, 1u + (uint32_t)l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (w < a.n_seq) report_timeout(w);
      }
      return;
    }
  }

  // =========================== tail ===========================
  uint64_t* const tb = llb + (size_t)a.L * LS;             // XB[L] lives at the start of this block
  const size_t OFF_RB = 16 * D;                            // head outputs: [16*K rows][D] fp32 words
  const size_t OFF_ST = OFF_RB + (size_t)16 * 15 * D;      // per (tile, row) top-2 statistics: 4 words
  const int NTV = V / 16;                                  // vocabulary tiles
  const int rows_all = M + M * K;                          // backbone rows, then head rows (m, k)
  uint16_t* const T0 = As;                                 // rows 0..15 of the unembedding input (hi, lo planes)
  uint16_t* const T1 = As + 32 * STD;                      // later row tiles, one at a time

  // first tiles of the head and unembedding matrices: requested before the last residual arrives
  uint4 wh[KD], wv[KD];
  if (w < K * (D / 16)) load_frags<KD>(wh, a.Wh, w, KTD, wave * KD, lane);
  if (w < NTV) load_frags<KD>(wv, a.WU, w, KTD, wave * KD, lane);

  XSM_STAMP(a.L * 16 + 0);
  {
    uint32_t gp[D / 512];
#pragma unroll
    for (int j = 0; j < D / 512; ++j) gp[j] = *reinterpret_cast<const uint32_t*>(a.gf + 2 * (tid + 256 * j));
    __syncthreads();
    stage_rows_f32<D, D, 1>(sm, T0, 0, tb + OFF_X, M, gp, a.eps, tid, tag, ok);
  }
  XSM_STAMP(a.L * 16 + 1);

  // ---- HEADS on every row: r_k = g + SiLU(W_k g + b_k)  (Eq. 4, MLP variant) ----
  for (int t = w; t < K * (D / 16); t += 256) {
    if (t != w) load_frags<KD>(wh, a.Wh, t, KTD, wave * KD, lane);
    const f32x4 acc = mac_tiles<KD>(wh, T0, STD, r, wave * KD, g);
    const float y = tile_reduce(sm, acc, wave, lane, tid);
    const int kh = t / (D / 16), c = (t % (D / 16)) * 16 + nrow;   // head index, column
    if (row_in) {
      const float pre = y + bf2f(a.hb[(size_t)kh * D + c]);
      const float gn = bf2f(T0[(size_t)om * STD + c]) + bf2f(T0[(size_t)(16 + om) * STD + c]);
      ll_st(tb + OFF_RB + ((size_t)om * K + kh) * D + c, __float_as_uint(gn + pre / (1.0f + __expf(-pre))), tag);
    }
  }
  XSM_STAMP(a.L * 16 + 2);

  // ---- UNEMBED over backbone rows and head rows, per-tile top-2 per row ----
  // row q < M: backbone row q (already in T0); row q >= M: head row q - M = m*K + k
  const int n_mt = (rows_all + 15) / 16;
  for (int mt = 0; mt < n_mt; ++mt) {
    uint16_t* const T = mt == 0 ? T0 : T1;
    const int q_lo = mt == 0 ? M : mt * 16, q_hi = min(rows_all, mt * 16 + 16);
    if (w < NTV) {                                     // only workgroups with a vocabulary tile need the rows
      __syncthreads();
      if (q_hi > q_lo) {
        const uint32_t nogain[D / 512] = {};
        stage_rows_f32<D, D, 0>(sm, T, q_lo - mt * 16, tb + OFF_RB + (size_t)(q_lo - M) * D, q_hi - q_lo, nogain,
                                    a.eps, tid, tag, ok);
      }
    }
    for (int t = w; t < NTV; t += 256) {
      if (t != w) load_frags<KD>(wv, a.WU, t, KTD, wave * KD, lane);
      const f32x4 acc = mac_tiles<KD>(wv, T, STD, r, wave * KD, g);
      __syncthreads();
      *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
      __syncthreads();
      // threads 0..15: row q = mt*16 + tid; scan the tile's 16 vocabulary entries in order
      if (tid < 16 && mt * 16 + tid < rows_all) {
        const int q = mt * 16 + tid;
        float bv = -INFINITY, sv = -INFINITY;
        int bi = 0;
        float* dbg = nullptr;
        if (q < M) { if (a.logits_dbg) dbg = a.logits_dbg + (size_t)q * V; }
        else if (a.head_logits_dbg) dbg = a.head_all_dbg + (size_t)(q - M) * V;
#pragma unroll
        for (int nr = 0; nr < 16; ++nr) {
          const int ln = (nr >> 2) * 16 + tid, ii = nr & 3;
          const float z = (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
          if (dbg) dbg[t * 16 + nr] = z;
          if (z > bv) { sv = bv; bv = z; bi = t * 16 + nr; }
          else sv = fmaxf(sv, z);
        }
        uint64_t* st = tb + OFF_ST + ((size_t)t * kSmallMaxRows + q) * 4;
        ll_st(st, __float_as_uint(bv), tag);
        ll_st(st + 1, (uint32_t)bi, tag);
        ll_st(st + 2, __float_as_uint(sv), tag);
      }
    }
    // a workgroup with several vocabulary tiles starts the next row tile from its first again
    if (NTV > 256 && w < NTV && mt + 1 < n_mt) load_frags<KD>(wv, a.WU, w, KTD, wave * KD, lane);
  }
  XSM_STAMP(a.L * 16 + 3);

  // ---- FINAL: workgroup b finishes sequence b (greedy verification with argmax draws; the other
  // criteria and sampling rules read the full logits rows in kernels of their own) ----
  if (w < a.n_seq && !a.defer_verify) {
    const int b = w;
    const int n = sm.len[b];
    // global top-2 of a logits row from the per-tile statistics (one wavefront per row, four tiles
    // per lane and request, all twelve words of a request in flight together) -> slot q of sm.st_*
    auto row_top2 = [&](int q, int grow) {
      float bv = -INFINITY, sv = -INFINITY;
      int bi = 0x7FFFFFFF;
      for (int t0 = 0; t0 < NTV; t0 += 256) {
        int off[12];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int t = t0 + lane + 64 * i;
#pragma unroll
          for (int j = 0; j < 3; ++j) off[3 * i + j] = t < NTV ? (t * kSmallMaxRows + grow) * 4 + j : -1;
        }
        uint32_t pw[12];
        ll_wait_list<12>(tb + OFF_ST, off, tag, pw, ok);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (off[3 * i] < 0) continue;
          const float tv = __uint_as_float(pw[3 * i]), ts = __uint_as_float(pw[3 * i + 2]);
          const int ti = (int)pw[3 * i + 1];
          if (tv > bv || (tv == bv && ti < bi)) { sv = fmaxf(bv, fmaxf(sv, ts)); bv = tv; bi = ti; }
          else sv = fmaxf(sv, fmaxf(tv, ts));
        }
      }
#define XSM_FOLD(O)                                                          \
      {                                                                        \
        const float bv2 = lane_xor<O>(bv), sv2 = lane_xor<O>(sv);              \
        const int bi2 = lane_xor<O>(bi);                                       \
        const bool take = (bv2 > bv) || (bv2 == bv && bi2 < bi);               \
        sv = fmaxf(fmaxf(sv, sv2), fminf(bv, bv2));                            \
        if (take) { bv = bv2; bi = bi2; }                                      \
      }
      XSM_FOLD(32) XSM_FOLD(16) XSM_FOLD(8) XSM_FOLD(4) XSM_FOLD(2) XSM_FOLD(1)
#undef XSM_FOLD
      if (lane == 0) { sm.st_max[q] = bv; sm.st_sec[q] = sv; sm.st_idx[q] = bi; }
    };
    // the R backbone rows first; they fix the accepted length, and only the K head rows of that
    // position are needed after it (slots R .. R + K - 1)
    for (int q = wave; q < R; q += 4) row_top2(q, b * R + q);
    __syncthreads();
    int acc_all = 0;                                      // (every thread: same values, same result)
    if (n >= 0)
      for (int j = 1; j <= K; ++j) {
        if (a.block[b * R + j] != sm.st_idx[j - 1]) break;
        ++acc_all;
      }
    for (int k = wave; k < K; k += 4) row_top2(R + k, M + (b * R + acc_all) * K + k);
    const bool late = __syncthreads_or(!ok);              // some statistics never arrived: nothing to emit
    if (tid == 0) {
      uint32_t fl = sm.flag[b];
      if (late) {
        report_timeout(b);
      } else if (n < 0) {
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
          const int q = R + k;
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
  XSM_STAMP(a.L * 16 + 4);
  if (__syncthreads_or(!ok)) {
    if (tid == 0) {
      __hip_atomic_store(a.ctrl + 1, 1000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (w < a.n_seq) report_timeout(w);
    }
    return;
  }
  // workgroup 0 closes the step: its FINAL needed every workgroup's statistics, so every
  // workgroup has long since read the epoch
  if (w == 0 && tid == 0)
    __hip_atomic_store(a.ctrl, tag + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#undef XSM_STAMP
}

size_t small_ll_words(int n_layers, int D, int F, int K) {
  const size_t layer = small_ll_layer_stride(D, F);
  const size_t tail = (size_t)16 * D + (size_t)16 * 15 * D + (size_t)4096 * kSmallMaxRows * 4;
  (void)K;
  return layer * n_layers + (tail > layer ? tail : layer);
}
size_t small_ll_layer_stride(int D, int F) {
  return (size_t)6 * 16 * D + (size_t)16 * F + (size_t)3 * 16 * D + (size_t)256 * 1056;
}

bool small_supported(int D, int F) { return D == 1024 && F == 4096; }

void launch_step_small(const SmallArgs& a, int D, int F, hipStream_t s) {
  TraceScope trace_("step_small", s);
  if (D == 1024 && F == 4096) {
    auto kfn = k_step_small<1024, 4096>;
    // activation tiles as bf16 hi + lo planes: two 16-row model-width tiles in the tail
    const size_t lds = (size_t)4 * 16 * (1024 + 8) * 2;
    allow_dynamic_lds((const void*)kfn, lds);
    hipLaunchKernelGGL(kfn, dim3(256), dim3(256), lds, s, a);
  }
}

}  // namespace xsm
