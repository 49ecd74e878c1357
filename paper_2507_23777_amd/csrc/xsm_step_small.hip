// One speculative (or plain) decoding step as ONE persistent kernel, for the
// latency regime: at most 16 block rows in total (batch x (K+1) <= 16), bf16,
// d_model 1024 / FFN 4096 / head_dim 64 models, every acceptance criterion and sampling rule.
//
// At batch 1 a step streams every weight once (hundreds of MB) through ~120 dependent
// stages of a few MB each, so what bounds it is not bandwidth inside a stage but the
// latency of handing a few KB of activations from one stage's producers to the next
// stage's consumers.  Kernel boundaries cost several microseconds each; here all 256
// workgroups (one per compute unit) stay resident for the whole step and exchange
// activations through memory with a flag in every 4-byte word:
//     word = { 24-bit payload: an fp32 value rounded to 16 significant bits, 8-bit tag },
//     tag  = 1 + (step epoch - 1) mod 255.
// A producer writes words with device-coherent stores; a consumer loads the words it
// needs with device-coherent loads and retries until every tag equals the current
// one, so arrival of the data IS the synchronisation (no barrier, no second round
// trip).  Each (layer, stage) owns its own buffer, so there is no reuse hazard inside a
// step.  A word written 255 steps ago would carry the current tag again: in every step
// whose tag is 1 the workgroups first clear the whole exchange region and meet at a
// barrier of their own (one word per workgroup carrying the full epoch).  Every wait is
// bounded: a workgroup that does not see its inputs within the spin budget raises the
// error word and leaves, and so does every workgroup waiting on it.
//
// 16 significant bits are what the consumer can use: an activation enters the bf16 MFMAs as
// two operands, hi = bf16(x) and lo = bf16(x - hi), against the same weight fragment, so the
// result carries the weights' bf16 rounding (part of the model) but none of the activations'
// beyond the 2^-17 of the exchange word.  Values that must arrive exactly are made exact
// before they are sent: new keys / values are rounded to bf16 by their producer (what the
// cache holds), attention's running maxima are rounded up to integers.
//
// Coherent loads bypass the caches, so they are issued fully coalesced (a wavefront reads
// 1 KB of consecutive words, a thread 16 bytes = four words of one row) and the activation
// block is re-laid through LDS into MFMA operand order.  What such a read costs is one
// round trip of about a microsecond almost regardless of its size (up to ~100 KB per
// workgroup when all loads are in flight together), so a consumer may as well read
// several partial blocks and add them itself; two dependent hand-offs per layer are
// saved that way:
//   - the FFN-down products of the four slices of the FFN width are not summed by anybody:
//     the next layer's QKV stage (and its O-projection, for the residual) reads the four
//     partial blocks; the last slice's workgroup has added the mid-layer residual to its own;
//   - with up to 4 key slices per (sequence, head) attention's partial outputs are merged by
//     the O-projection workgroups while they stage them; only longer contexts (8 or 16
//     slices) keep a merge stage of their own.
//
// Weights never depend on activations, so each workgroup requests the fragments of the
// tile it will need one layer ahead and holds them in registers; HBM stays busy while
// the dependency chain is waiting.  Stages per layer (Sec. 4.1 block = self-attention +
// feed-forward; Alg. 1 "forward with causal mask"):
//   QKV   192 tiles  residual = sum of 4 partial blocks, RMSNorm + projection + rotary,
//                    new k/v also written to the cache
//   ATT   B*H*S units  MFMA attention over a slice of the cached keys (+ the new block)
//   COMB  merge of the S slices (S = 8 or 16 only)
//   OPROJ 64 tiles   merge of up to 4 slices, output projection + residual
//   UP    256 tiles  RMSNorm + W1 + erf-GELU
//   DOWN  64 tiles x 4 slices of the FFN width: W2 partial products on all 256 workgroups
// then the decoding heads on every block row (Alg. 1 runs each head on h_{s:s+D}), the
// shared unembedding over backbone and head rows with a per-tile top-2 reduction, and one
// workgroup per sequence that does the accept scan, picks the tokens at the first rejected
// position and rolls the cache length back (Alg. 1 inner loop, resample line, s <- s*).
// Greedy verification with argmax draws needs nothing but the per-tile statistics; the other
// criteria and sampling rules (Sec. 5.4 "Verification criterion"; appendix "Sampling strategies")
// read whole logits rows: each accept check, and each draw for every accepted length the scan
// could end at, runs as a task on a workgroup of its own and posts its result as a tagged word.
#include <type_traits>
#include "xsm_device.h"
#include "xsm_internal.h"
#include "xsm_verify_device.h"

namespace xsm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kSpinBudget = 150000;         // polls before a wait gives up (a fraction of a second)
constexpr float kTieMarginS = 1e-2f;
constexpr float kEmptySliceMax = -30000.f;  // running maximum published by a key slice that saw no key
// 16 bytes per lane from global memory straight into LDS: lane l's piece lands at lds + 16 l
__device__ __forceinline__ void lds_direct16(const void* gptr, void* lds) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds, 16, 0, 0);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Pointers that went through LDS (the layer table) have lost their address space, and a load
// through one is a FLAT load: the compiler cannot count those against younger loads and waits for
// every outstanding access instead.  Weights and cache are global memory: say so.
typedef const __attribute__((address_space(1))) u32x4* gptr16;
__device__ __forceinline__ gptr16 as_global(const void* p) { return (gptr16)(p); }
__device__ __forceinline__ uint4 ldg16(gptr16 p, int piece) { return __builtin_bit_cast(uint4, p[piece]); }
// raw buffer descriptor word 3 (32-bit data format, no swizzle) and the cache-policy bits of an
// access that is coherent across the device (sc1)
constexpr int kRawBufferFlags = 0x00020000, kCoherent = 16;

// 2^x on the hardware's exponential instruction alone (1 ulp; results below the normal range come
// out as zero, which is what a softmax weight that small is worth).  The library routine wraps the
// same instruction in a range fix-up of five more, and at one wavefront per SIMD an instruction
// costs about eight cycles: attention takes seventeen exponentials per 64-key chunk and lane.
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int kQS = 72;                     // LDS row stride (bf16) of the attention q / new-k / new-v tiles

// ---- 8-byte tagged words {32-bit payload, full epoch}: the tail's per-tile logits statistics ----
__device__ __forceinline__ uint64_t ll_ld(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_st(uint64_t* p, uint32_t payload, uint32_t tag) {
  __hip_atomic_store(p, ((uint64_t)tag << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
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

// ---- 4-byte tagged words {24-bit payload, 8-bit tag}: everything else ----
// fp32 -> 16 significant bits (round to nearest even on bit 8) with the tag in the low byte
__device__ __forceinline__ uint32_t enc24(float x, uint32_t t8) {
  uint32_t u = __float_as_uint(x);
  u += 0x7Fu + ((u >> 8) & 1u);
  return (u & 0xFFFFFF00u) | t8;
}
__device__ __forceinline__ float dec24(uint32_t w) { return __uint_as_float(w & 0xFFFFFF00u); }
__device__ __forceinline__ f32x4 dec24(u32x4 q) { return f32x4{dec24(q.x), dec24(q.y), dec24(q.z), dec24(q.w)}; }
// all-zero low byte iff all four tags match
__device__ __forceinline__ uint32_t tagdiff(u32x4 q, uint32_t t8) { return (q.x ^ t8) | (q.y ^ t8) | (q.z ^ t8) | (q.w ^ t8); }
__device__ __forceinline__ void st32(uint32_t* p, float x, uint32_t t8) {
  __hip_atomic_store(p, enc24(x, t8), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// four consecutive words (16-byte aligned, `word` counted from the start of the buffer rs describes)
// as one device-coherent store; every word carries its own tag.  The descriptor must be the same
// in all lanes (it lives in scalar registers); the offset is the lane's own.
__device__ __forceinline__ void st32x4(__amdgpu_buffer_rsrc_t rs, int word, f32x4 v, uint32_t t8) {
  __builtin_amdgcn_raw_buffer_store_b128(u32x4{enc24(v[0], t8), enc24(v[1], t8), enc24(v[2], t8), enc24(v[3], t8)}, rs,
                                         word * 4, 0, kCoherent);
}
__device__ __forceinline__ uint32_t ld32(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// the same small-block wait for 4-byte words; payloads decoded to floats
template <int N>
__device__ __forceinline__ void wait_words(const uint32_t* p, const int (&off)[N], uint32_t t8, float (&out)[N], bool& ok) {
  bool any = false;
#pragma unroll
  for (int i = 0; i < N; ++i) any |= off[i] >= 0;
  if (ok && any) {
    for (int spin = 0; spin < kSpinBudget; ++spin) {
      uint32_t w[N];
#pragma unroll
      for (int i = 0; i < N; ++i)
        if (off[i] >= 0) w[i] = ld32(p + off[i]);
      uint32_t bad = 0;
#pragma unroll
      for (int i = 0; i < N; ++i)
        if (off[i] >= 0) bad |= w[i] ^ t8;
      if ((bad & 0xFFu) == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = off[i] >= 0 ? dec24(w[i]) : 0.f;
        return;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    ok = false;
  }
#pragma unroll
  for (int i = 0; i < N; ++i) out[i] = 0.f;
}

// Every poll of a word that another XCD is about to write costs fabric traffic that slows the
// writes everybody is waiting for, so a workgroup polls with one lane: it watches one word of the
// block until it carries the tag while the rest sit at the barrier; the block is read afterwards
// (and re-read in the rare case that other producers' words lag).  Must be reached by every
// thread of the workgroup.  (Measured: several polls in flight, or a different watch word per
// workgroup, both cost more than they gain.)
__device__ __forceinline__ void watch_then_sync(const uint32_t* word, uint32_t t8, bool active, int tid) {
  if (tid == 0 && active) {
    int spin = 0;
    while ((ld32(word) & 0xFFu) != t8 && ++spin < kSpinBudget) __builtin_amdgcn_s_sleep(1);
  }
  __syncthreads();
}

// The same for a consumer whose wavefronts each depend on a few producers of their own: lane i
// polls the word at base + off (off < 0: none) and the wavefront goes on, without a barrier, once
// every polled word carries the tag.  A stage with few consumer workgroups can afford the polls,
// and a block read that finds a producer's words missing costs it a whole second round trip.
__device__ __forceinline__ void wave_watch(const uint32_t* base, int off, uint32_t t8, bool& ok) {
  bool pending = off >= 0 && ok;
  for (int spin = 0; __builtin_amdgcn_ballot_w64(pending) != 0; ++spin) {
    if (spin >= kSpinBudget) { ok = false; break; }
    if (pending) pending = (ld32(base + off) & 0xFFu) != t8;
    __builtin_amdgcn_s_sleep(1);
  }
}

// Cooperative, coalesced wait for rows [m0, m0 + RB) (clipped to nrows) of NB blocks of tagged
// words (1024 words per row, row stride RS, block stride BS; buf = block 0, row 0): thread t
// takes words 4t .. 4t+3 of every row, so a wavefront instruction covers 1 KB of consecutive
// words; v[m] = the blocks' values added in the fixed order ((b0 + b1) + (b2 + b3)), zero for
// m >= RB.  All loads of a round are in flight together (NB x RB x 4 registers): a round costs one
// round trip whatever NB is.
// rows a reader's result array holds: 8, or 12 for the single-block rounds of up to 12 rows
constexpr int rows_held(int RB) { return RB <= 8 ? 8 : 12; }
struct NoHook { __device__ __forceinline__ void operator()() const {} };
// a hook that requests nothing: picks the reader below (one wide read, then single rows) where
// that is wanted without anything to place behind the read
struct NothingBehind { __device__ __forceinline__ void operator()() const {} };

// One row (this thread's four words of each of NB blocks) that the wide read found incomplete:
// re-read until every tag matches.  The slow path of read_rows; one row at a time keeps it small.
template <int NB>
__device__ __forceinline__ f32x4 retry_row(__amdgpu_buffer_rsrc_t rs, int word0, int BS, uint32_t t8, bool& ok) {
  if (ok) {
    for (int spin = 0; spin < kSpinBudget; ++spin) {
      __builtin_amdgcn_s_sleep(4);
      u32x4 q[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b) q[b] = __builtin_amdgcn_raw_buffer_load_b128(rs, (b * BS + word0) * 4, 0, kCoherent);
      uint32_t bad = 0;
#pragma unroll
      for (int b = 0; b < NB; ++b) bad |= tagdiff(q[b], t8);
      if ((bad & 0xFFu) == 0) {
        if constexpr (NB == 4) return (dec24(q[0]) + dec24(q[1])) + (dec24(q[2]) + dec24(q[3]));
        else return dec24(q[0]);
      }
    }
    ok = false;
  }
  return f32x4{0.f, 0.f, 0.f, 0.f};
}

// Cooperative, coalesced wait for rows [m0, m0 + RB) (clipped to nrows) of NB blocks of tagged
// words (1024 words per row, row stride RS, block stride BS; buf = block 0, row 0): thread t
// takes words 4t .. 4t+3 of every row, so a wavefront instruction covers 1 KB of consecutive
// words; v[m] = the blocks' values added in the fixed order ((b0 + b1) + (b2 + b3)), zero for
// m >= RB.  All loads of a round are in flight together (NB x RB x 4 registers): a round costs one
// round trip whatever NB is; a row that turns out incomplete (rare after the watch) is re-read on
// its own.  after_issue runs once, between the issue of the loads and the wait for them:
// requests placed there (weights, cached keys) travel behind the block instead of in front of
// the next stage's poll - a wavefront's loads return in order.
template <int NB, int RB, class Hook>
__device__ __forceinline__ void read_rows(const uint32_t* buf, int BS, int RS, int m0, int nrows, int tid, uint32_t t8,
                                          bool watch, f32x4 (&v)[rows_held(RB)], bool& ok, uint64_t* stamp, Hook&& after_issue) {
  static_assert((NB == 1 || NB == 4) && RB <= 8, "one block, or four partial blocks; at most 8 rows a round");
  const int rows = min(RB, nrows - m0);
  // (later rounds of a block come from the same producers as its first rows: no watch, its poll
  // would be one more round trip in front of the read)
  if (watch)
    watch_then_sync(buf + (size_t)(NB - 1) * BS + (size_t)(m0 + (rows > 0 ? rows - 1 : 0)) * RS + 513, t8, ok && rows > 0, tid);
  if (stamp && tid == 0) stamp[0] = wall_clock64();
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(buf + (size_t)m0 * RS), 0, ((NB - 1) * BS + (rows > 0 ? rows : 0) * RS) * 4, kRawBufferFlags);
  u32x4 q[NB][RB];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int m = 0; m < RB; ++m)
      if (m < rows) q[b][m] = __builtin_amdgcn_raw_buffer_load_b128(rs, (b * BS + m * RS + 4 * tid) * 4, 0, kCoherent);
  // (the hook's requests stay between the block's loads and their first use: without the fences
  // the compiler sinks them to where their data is used, stages later)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  after_issue();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int m = RB; m < 8; ++m) v[m] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int m = 0; m < RB; ++m) {
    if (m < rows) {
      uint32_t bad = 0;
#pragma unroll
      for (int b = 0; b < NB; ++b) bad |= tagdiff(q[b][m], t8);
      if ((bad & 0xFFu) == 0 && ok) {
        if constexpr (NB == 4) v[m] = (dec24(q[0][m]) + dec24(q[1][m])) + (dec24(q[2][m]) + dec24(q[3][m]));
        else v[m] = dec24(q[0][m]);
      } else {
        v[m] = retry_row<NB>(rs, m * RS + 4 * tid, BS, t8, ok);
      }
    } else {
      v[m] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  if (stamp && tid == 0) stamp[1] = wall_clock64();
}

// The reader without a hook: everything is re-read until every tag matches (when the watched word is
// in but another producer's words are not yet, one more round trip brings all of them).
template <int NB, int RB>
__device__ __forceinline__ void read_rows_plain(const uint32_t* buf, int BS, int RS, int m0, int nrows, int tid, uint32_t t8,
                                                bool watch, f32x4 (&v)[rows_held(RB)], bool& ok, uint64_t* stamp) {
  static_assert(RB <= 12 && (NB == 1 || RB <= 8), "up to 12 rows of one block a round, up to 8 of four");
  const int rows = min(RB, nrows - m0);
  if (watch)
    watch_then_sync(buf + (size_t)(NB - 1) * BS + (size_t)(m0 + (rows > 0 ? rows - 1 : 0)) * RS + 513, t8, ok && rows > 0, tid);
  if (stamp && tid == 0) stamp[0] = wall_clock64();
  if (ok && rows > 0) {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t*>(buf + (size_t)m0 * RS), 0, ((NB - 1) * BS + rows * RS) * 4, kRawBufferFlags);
    for (int spin = 0; spin < kSpinBudget; ++spin) {
      u32x4 q[NB][RB];
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int m = 0; m < RB; ++m)
          if (m < rows) q[b][m] = __builtin_amdgcn_raw_buffer_load_b128(rs, (b * BS + m * RS + 4 * tid) * 4, 0, kCoherent);
      uint32_t bad = 0;
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int m = 0; m < RB; ++m)
          if (m < rows) bad |= tagdiff(q[b][m], t8);
      if ((bad & 0xFFu) == 0) {
#pragma unroll
        for (int m = RB; m < rows_held(RB); ++m) v[m] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int m = 0; m < RB; ++m) {
          if (m < rows) {
            if constexpr (NB == 4) v[m] = (dec24(q[0][m]) + dec24(q[1][m])) + (dec24(q[2][m]) + dec24(q[3][m]));
            else v[m] = dec24(q[0][m]);
          } else {
            v[m] = f32x4{0.f, 0.f, 0.f, 0.f};
          }
        }
        if (stamp && tid == 0) stamp[1] = wall_clock64();
        return;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    ok = false;
  }
#pragma unroll
  for (int m = 0; m < rows_held(RB); ++m) v[m] = f32x4{0.f, 0.f, 0.f, 0.f};
}

template <int N>
__device__ __forceinline__ void load_frags(uint4 (&w)[N], const uint4* Wt, int nt, int KT, int kt0,
                                           int lane) {
  const gptr16 p = as_global(Wt + ((size_t)nt * KT + kt0) * 64 + lane);
#pragma unroll
  for (int i = 0; i < N; ++i) w[i] = ldg16(p, i * 64);
}

// all ones or zero, hidden from the optimiser.  Requests placed between a block read's loads and
// their first use must be unconditional: behind a branch the compiler cannot count what is in
// flight on which path and waits for everything; and arithmetic on a visible condition it turns
// back into a branch.
__device__ __forceinline__ int opaque_mask(bool use) {
  int m = use ? -1 : 0;
  asm volatile("" : "+v"(m));
  return m;
}

struct Shared {
  float red[4][64][4];          // cross-wavefront tile reduction
  float rowsum[4][16];          // RMSNorm partial sums
  float att_ml[4][2][16];
  float att_o[4][4][64][4];     // attention: the wavefronts' partial outputs; O-projection: the slices' (m, l)
  int len[16], slot[16];
  int blk[16];                  // the step's input block rows (tokens), read once at set-up
  uint32_t flag[16];
  uint32_t tag;
  int fail;
  float st_max[kSmallMaxRows], st_sec[kSmallMaxRows];  // FINAL: per-row reductions
  int st_idx[kSmallMaxRows];
  LayerTab tab[48];
};

// Sum the four wavefronts' partial 16x16 tiles; thread t gets element D[column t % 16][row t / 16],
// so that the 16 words of one row's tile leave in one 64-byte store.
__device__ __forceinline__ float tile_reduce(Shared& sm, f32x4 acc, int wave, int lane, int tid) {
  __syncthreads();
  *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
  __syncthreads();
  const int oc = tid & 15, om = tid >> 4;
  const int ln = (oc >> 2) * 16 + om, ii = oc & 3;        // MFMA lane and slot that hold D[oc][om]
  return (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
}

// four floats -> LDS rows of the hi and lo planes (row stride ST bf16, lo plane 16 rows further)
__device__ __forceinline__ void put4(uint16_t* As, int ST, int row, int col, f32x4 x) {
  uint2 hi, lo;
  split4(float4{x[0], x[1], x[2], x[3]}, hi, lo);
  uint16_t* dst = As + (size_t)row * ST + col;
  *reinterpret_cast<uint2*>(dst) = hi;
  *reinterpret_cast<uint2*>(dst + 16 * ST) = lo;
}

constexpr int kST = 1024 + 8;               // LDS row stride (bf16) of a staged 1024-column tile

// Stage nrows rows, 1024 columns each, of NB tagged-word blocks (added up, see read_rows) into LDS
// rows dst_row.. as two bf16 planes of row stride kST: hi at As, lo at As + 16 * kST.
// NORM 1: RMSNorm over the columns with the gains g4 (this thread's columns 4 tid .. 4 tid + 3).
// NORM 2: only the gains are applied and the rows' sums of squares are left in sm.rowsum[.][row];
// the caller multiplies its products by row_scale(row) - the rows reach LDS without waiting for
// the sums to be exchanged.
template <int NB, int NORM, int RB, class Hook = NoHook>
__device__ __forceinline__ void stage_rows(Shared& sm, uint16_t* As, int dst_row, const uint32_t* buf, int BS, int RS,
                                           int nrows, f32x4 g4, float eps, int tid, uint32_t t8, bool& ok,
                                           uint64_t* stamp = nullptr, Hook&& after_issue = NoHook{}, bool watch0 = true) {
  const int wave = tid >> 6, lane = tid & 63;
  for (int m0 = 0; m0 < nrows; m0 += RB) {
    static_assert(NORM == 0 || RB <= 8, "the row sums are exchanged eight rows at a time");
    f32x4 v[rows_held(RB)];
    if constexpr (std::is_same<typename std::decay<Hook>::type, NoHook>::value) {
      read_rows_plain<NB, RB>(buf, BS, RS, m0, nrows, tid, t8, m0 == 0 && watch0, v, ok, stamp);
    } else {
      if (m0 == 0) read_rows<NB, RB>(buf, BS, RS, m0, nrows, tid, t8, watch0, v, ok, stamp, after_issue);
      else read_rows_plain<NB, RB>(buf, BS, RS, m0, nrows, tid, t8, false, v, ok, stamp);
    }
    if (NORM) {
      if (NORM == 1 && m0 > 0) __syncthreads();          // this call's earlier readers of rowsum are done
      // eight row sums per wavefront in ten lane exchanges instead of forty-eight: each exchange
      // step halves the rows a lane carries (lane bits 5, 4, 3 pick the row), then three steps
      // finish the one row left.  Cross-lane moves cost LDS-like latency at one wavefront per SIMD.
      float ss[8];
#pragma unroll
      for (int m = 0; m < 8; ++m) ss[m] = (v[m][0] * v[m][0] + v[m][1] * v[m][1]) + (v[m][2] * v[m][2] + v[m][3] * v[m][3]);
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
      const int ri = (b5 ? 4 : 0) + (b4 ? 2 : 0) + (b3 ? 1 : 0);     // the row whose sum this lane ended up with
      if ((lane & 7) == 0 && ri < RB) sm.rowsum[wave][(NORM == 2 ? m0 : 0) + ri] = s1;
      if (NORM == 1) __syncthreads();
    }
#pragma unroll
    for (int m = 0; m < RB; ++m) {
      if (m0 + m < nrows) {
        f32x4 x = v[m];
        if (NORM == 1) {      // (hardware reciprocal square root, 1 ulp)
          const float sc = __builtin_amdgcn_rsqf(((sm.rowsum[0][m] + sm.rowsum[1][m]) + (sm.rowsum[2][m] + sm.rowsum[3][m])) * (1.0f / 1024.0f) + eps);
          x = x * sc * g4;
        }
        if (NORM == 2) x = x * g4;
        put4(As, kST, dst_row + m0 + m, 4 * tid, x);
      }
    }
  }
  __syncthreads();
}

// 1 / rms of a row staged with NORM 2 (hardware reciprocal square root, 1 ulp)
__device__ __forceinline__ float row_scale(const Shared& sm, int row, float eps) {
  return __builtin_amdgcn_rsqf(((sm.rowsum[0][row] + sm.rowsum[1][row]) + (sm.rowsum[2][row] + sm.rowsum[3][row])) * (1.0f / 1024.0f) + eps);
}

// bf16 gains of this thread's four columns
__device__ __forceinline__ f32x4 gains4(const uint16_t* g, int tid) {
  const uint2 w = *reinterpret_cast<const uint2*>(g + 4 * tid);
  return f32x4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xFFFF0000u), __uint_as_float(w.y << 16),
               __uint_as_float(w.y & 0xFFFF0000u)};
}

// acc = sum_i Wfrag[i] . (hi + lo) over k-tiles kt0 .. kt0 + N - 1 of activation row `row` of an
// LDS tile staged by stage_rows (row stride ST, lo plane 16 rows further).  All operand
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

// bf16 pair of (a, b) and of what that rounding dropped
__device__ __forceinline__ uint32_t pk2(float a, float b) { return f2bf_pair(a, b); }
__device__ __forceinline__ float lo_bf(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ void split2(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  hi = pk2(x0, x1);
  lo = pk2(x0 - lo_bf(hi), x1 - hi_bf(hi));
}

// Attention's output rows as the O-projection's operand: the partial rows of the S_eff key slices
// (blocks of 16 x 1024 words at word off_op + slice * blk of the layer buffer rs describes) are
// merged while they are staged into LDS, O = sum_s f_s O_s / sum_s f_s l_s with f_s = 2^(m_s - max m).
// The slices' (maximum, sum) pairs of all rows and heads are [16 rows][H][4 slices][2] words at
// off_ml.  RB rows a round, all loads of a round in flight together; S_eff = 1, 2 or 4.
template <int H, int RB, int S_eff>
__device__ __forceinline__ void stage_attn_out(Shared& sm, uint16_t* As, __amdgpu_buffer_rsrc_t rs, const uint32_t* lb, int watch_off,
                                               int off_op, int blk, int off_ml, int M, int tid, uint32_t t8, bool& ok) {
  float* const mls = &sm.att_o[0][0][0][0];
  const int wave = tid >> 6, lane = tid & 63;
  // wavefront w stages the columns of heads 4 w .. 4 w + 3 and waits for those heads' producers
  wave_watch(lb, watch_off, t8, ok);
  for (int m0 = 0; m0 < M; m0 += RB) {
    const int rows = min(RB, M - m0);
    u32x4 q[4][RB], mlq[2];
    // (maximum, sum) pieces of the wavefront's own heads: lane = (row % 8, head, slice pair), rows
    // 0..7 and 8..15; piece (row, head, pair) holds slices 2 pair and 2 pair + 1
    bool need_ml[2];
    int mlp[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = (lane >> 3) + 8 * j;
      mlp[j] = (row * H + 4 * wave + ((lane >> 1) & 3)) * 2 + (lane & 1);
      need_ml[j] = m0 == 0 && row < M && (lane & 1) * 2 < S_eff;
    }
    bool got = false;
    if (ok) {
      for (int spin = 0; spin < kSpinBudget; ++spin) {
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
          for (int m = 0; m < RB; ++m)
            if (sl < S_eff && m < rows)
              q[sl][m] = __builtin_amdgcn_raw_buffer_load_b128(rs, (off_op + sl * blk + (m0 + m) * 1024 + 4 * tid) * 4, 0, kCoherent);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          if (need_ml[j]) mlq[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, (off_ml + 4 * mlp[j]) * 4, 0, kCoherent);
        uint32_t bad = 0;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
          for (int m = 0; m < RB; ++m)
            if (sl < S_eff && m < rows) bad |= tagdiff(q[sl][m], t8);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          if (need_ml[j]) {
            bad |= (mlq[j].x ^ t8) | (mlq[j].y ^ t8);
            if ((lane & 1) * 2 + 1 < S_eff) bad |= (mlq[j].z ^ t8) | (mlq[j].w ^ t8);
          }
        if ((bad & 0xFFu) == 0) { got = true; break; }
        __builtin_amdgcn_s_sleep(4);
      }
      if (!got) ok = false;
    }
    if (m0 == 0) {
      // The merge weights w_s = f_s / sum_s f_s l_s are made once per (row, head), by the lanes
      // that hold its (maximum, sum) pairs (the slice pairs of one (row, head) sit in neighbouring
      // lanes), and go to the columns' threads through LDS: [row][head][4 slices]
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const f32x4 v = dec24(mlq[j]);
        const bool va = need_ml[j] && got, vb = va && (lane & 1) * 2 + 1 < S_eff;
        const float ma = va ? v[0] : -INFINITY, mb = vb ? v[2] : -INFINITY;
        float Mg = fmaxf(ma, mb);
        Mg = fmaxf(Mg, lane_xor<1>(Mg));
        const float fa = va ? exp2_hw(ma - Mg) : 0.f, fb = vb ? exp2_hw(mb - Mg) : 0.f;
        float Lg = (va ? v[1] * fa : 0.f) + (vb ? v[3] * fb : 0.f);
        Lg += lane_xor<1>(Lg);
        const float inv = Lg > 0.f ? 1.0f / Lg : 0.f;
        if ((lane >> 3) + 8 * j < M) *reinterpret_cast<float2*>(mls + 2 * mlp[j]) = float2{fa * inv, fb * inv};
      }
      __syncthreads();
    }
    const int hd = tid >> 4;                              // head of this thread's four columns
#pragma unroll
    for (int m = 0; m < RB; ++m) {
      if (m < rows) {
        f32x4 x = f32x4{0.f, 0.f, 0.f, 0.f};
        if (got) {
          const f32x4 wgt = *reinterpret_cast<const f32x4*>(mls + ((m0 + m) * H + hd) * 4);
#pragma unroll
          for (int sl = 0; sl < 4; ++sl)
            if (sl < S_eff) x += dec24(q[sl][m]) * wgt[sl];
        }
        put4(As, kST, m0 + m, 4 * tid, x);
      }
    }
  }
  __syncthreads();
}

}  // namespace

// RC, BC, VC: rows per sequence, sequences and vocabulary as compile-time constants (0: read from the
// arguments).  TL: with the stage clock (the stamps cost 1 % of a step, so the instantiations that
// production steps run are built without them)
template <int D, int F, int RC, int BC, int VC = 0, bool TL = false>
__global__ __launch_bounds__(256) void k_step_small(const SmallArgs a) {
  const int n_seq = BC ? BC : a.n_seq;
  constexpr int H = D / 64;
  constexpr int KTD = D / 32, KTF = F / 32;          // k-tiles of the two contraction lengths
  constexpr int KD = KTD / 4;                        // per wavefront
  constexpr int NQ = 3 * D / 16, NO = D / 16, NU = F / 16;
  constexpr int O_BASE = NQ;
  constexpr int FS = F / 4;                          // DOWN: slice of the FFN width per workgroup
  constexpr int KFS = FS / 32 / 4;                   // its k-tiles per wavefront
  constexpr int STD = kST;
  static_assert(NQ + NO <= 256 && NU <= 256 && NO * 4 == 256, "tile roles must fit 256 workgroups");
  static_assert(D == 1024 && FS == 1024, "a thread stages four words of a 1024-word row");
  __shared__ Shared sm;
  extern __shared__ __align__(16) unsigned char dyn[];
  uint16_t* const As = reinterpret_cast<uint16_t*>(dyn);     // activation tile(s), several layouts

  const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int R = RC ? RC : a.R, K = R - 1, M = n_seq * R, V = VC ? VC : a.V;

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
    if (tid < n_seq) {
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
    sm.blk[tid] = tid < M ? a.block[tid] : 0;
  }
  __syncthreads();
  // A bounded wait gave up, in this step or an earlier one: sequence b produced nothing.  The
  // caller sees it in the step's own outputs (n_accepted 0, the timeout flag).
  auto report_timeout = [&](int b) {
    a.n_accepted[b] = 0;
    a.flags[b] = sm.flag[b] | XSM_FLAG_DEVICE_TIMEOUT;
  };
  if (sm.fail != 0) {                       // an earlier step timed out: stay down until reset
    if (w < n_seq && tid == 0) report_timeout(w);
    return;
  }
  const uint32_t tag = sm.tag;                          // full epoch: 8-byte words, barrier words
  const uint32_t t8 = 1u + (tag - 1u) % 255u;           // tag of the 4-byte words
  bool ok = true;

  // ---- once per 255 steps: clear the exchange region (words of 255 steps ago would pass for
  // this step's), then a barrier of all workgroups before anybody writes ----
  if (t8 == 1u) {
    const size_t n16 = a.ll_words / 4;
    // (device-coherent stores: a plain store could sit in this XCD's L2 and be written back over
    // newer words later; the region is smaller than 2 GB, the launcher checks)
    const __amdgpu_buffer_rsrc_t zr = __builtin_amdgcn_make_buffer_rsrc(a.ll, 0, (int)(n16 * 16), kRawBufferFlags);
    for (size_t i = (size_t)w * 256 + tid; i < n16; i += 65536)
      __builtin_amdgcn_raw_buffer_store_b128(u32x4{0u, 0u, 0u, 0u}, zr, (int)(i * 16), 0, kCoherent);
    __threadfence();                                    // this thread's clears have landed
    __syncthreads();
    uint32_t* const arrive = a.ctrl + 64;               // [256]: epoch of the last clear each workgroup finished
    if (tid == 0) __hip_atomic_store(arrive + w, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int spin = 0;
    while (ld32(arrive + tid) != tag && ++spin < kSpinBudget) __builtin_amdgcn_s_sleep(8);
    if (spin >= kSpinBudget) ok = false;
    if (__syncthreads_or(!ok)) {
      if (tid == 0) {
        __hip_atomic_store(a.ctrl + 1, 2000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (w < n_seq) report_timeout(w);
      }
      return;
    }
  }

  // Key slices per (sequence, head), from the longest live cache (every workgroup reads the same
  // lengths, so all agree).  The cached keys and values come from HBM at full memory latency and a
  // workgroup has at most 128 KB of them in flight, so the attention stage is as fast as the
  // number of workgroups sharing a key range.  Up to 4 slices are merged by the O-projection's
  // workgroups as they read them; 8 and 16 slices need a merge stage of their own, which pays
  // from about two thousand keys on.
  int S = a.S;
  if (a.s_auto) {
    int longest = 0;
    for (int b = 0; b < n_seq; ++b) longest = max(longest, sm.len[b]);
    const int chunks = (longest + 63) >> 6;
    const int want = chunks <= 2 ? 1 : chunks <= 6 ? 2 : chunks <= 28 ? 4 : 16;
    while (S > want) S >>= 1;
  }
  const int S_eff = S <= 4 ? S : 1;                    // slices the O-projection merges itself
  // Rows a read round of four partial blocks takes: all of them when there are at most 5 (20
  // loads in flight per thread), else 4 (16 loads) - what the register file holds next to the
  // weight tiles.  The 9 rows of K = 8 at batch 1 go in two rounds of 5 instead of three of 4, but
  // only where the row count is a compile-time constant: in the instantiation that reads it from
  // the arguments the flag has to stay `M <= 5`, from which the compiler knows that a 5-row round
  // is the only one and drops the round loops (folding 9 and 10 rows into it there gained 4 % at
  // K = 8 and cost 4 % at K = 4).
  const bool few = M <= 5 || (RC != 0 && BC != 0 && (M == 9 || M == 10));
  // this lane's activation row (MFMA column) m = r
  // the output element this thread finishes after tile_reduce: tile column nrow of row om
  const int om = tid >> 4, nrow = tid & 15;
  const int mb = om / R, mj = om % R;
  const bool row_in = om < M;
  const int len_m = row_in ? sm.len[mb] : -1;
  const bool live = row_in && len_m >= 0;              // rows of skipped sequences carry zeros

  const size_t LS = a.ll_layer_stride;                 // words per layer
  uint32_t* const llb = a.ll;
  constexpr int BLK = 16 * D;                          // one [16 rows][D] block
  constexpr int OFF_XP = 0,                            // [4][16][D]  the layer's input residual as four partial blocks
                OFF_Q = 4 * BLK, OFF_KN = 5 * BLK, OFF_VN = 6 * BLK,
                OFF_OP = 7 * BLK,                      // [4][16][D]  attention outputs of up to 4 key slices (unnormalised)
                OFF_ML = 11 * BLK,                     // [16 rows][H][4 slices][2]  their (maximum, sum)
                OFF_XM = OFF_ML + 16 * H * 8, OFF_U = OFF_XM + BLK,
                OFF_P = OFF_U + 16 * F;                // [256 units][1056]  partials of the merge stage (8 / 16 slices)

  const bool has_q = w < NQ, has_o = w >= O_BASE && w < O_BASE + NO, has_u = w < NU;
  const int d_nt = w % NO, d_ks = w / NO;              // DOWN: output tile and slice of the FFN width
  // Weight fragments live in registers and are requested ahead of use.  A wavefront's loads
  // return in order, so a request delays whatever wait is issued right behind it: a poll that
  // follows a request to HBM comes back a memory latency later.  Requests are therefore placed
  // where their workgroup is about to sit out a stage, or right behind a block read's loads (they
  // then travel behind data that is waited for anyway):
  //   workgroups with a QKV tile: this layer's UP and DOWN tiles and next layer's QKV tile after
  //     attention (the O-projection runs elsewhere meanwhile); the attention unit's first chunk of
  //     cached keys / values behind the QKV stage's block read, two hand-offs before it is used
  //     (measured: 8 % of a step; the next QKV tile behind the UP stage's block read instead: a loss);
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

  // ---- EMBED: layer-0 residual rows as tagged words (partial block 3; the others are zero) ----
  for (int idx = w * 256 + tid; idx < M * D; idx += 256 * 256) {
    const int m = idx / D, c = idx % D, b = m / R;
    const float x = sm.len[b] >= 0 ? bf2f(a.E[(size_t)sm.blk[m] * D + c]) : 0.f;
#pragma unroll
    for (int p = 0; p < 4; ++p) st32(llb + OFF_XP + p * BLK + (size_t)m * D + c, p == 3 ? x : 0.f, t8);
  }

  // optional timeline: thread 0 of every workgroup stamps the 100 MHz clock at stage boundaries
  uint64_t* const tl = TL && a.tlog ? a.tlog + (size_t)w * (a.L * 16 + 8) : nullptr;
#define XSM_STAMP(idx) do { if (TL && tl && tid == 0) tl[idx] = wall_clock64(); } while (0)
  for (int l = 0; l < a.L; ++l) {
    uint32_t* const lb = llb + (size_t)l * LS;
    const LayerTab& lt = sm.tab[l];
    const __amdgpu_buffer_rsrc_t lrs = __builtin_amdgcn_make_buffer_rsrc(lb, 0, (int)(LS * 4), kRawBufferFlags);
    XSM_STAMP(l * 16 + 0);

    // the attention unit of this workgroup: slice s of the keys of (sequence b, head h)
    const int n_units = n_seq * H * S;
    const bool att = w < n_units;
    const int b = att ? w / (H * S) : 0, h = (w / S) % H, s = w % S;
    const int n = att ? sm.len[b] : -1;
    const int nn = n < 0 ? 0 : n;                         // skipped sequence: no cached keys read
    const int NC = (nn + 63) >> 6, CPS = (NC + S - 1) / S;
    const int c_lo = s * CPS, c_hi = att ? min(NC, c_lo + CPS) : 0;
    const size_t uhead = (size_t)sm.slot[b] * H + h;
    const uint16_t* const kb = lt.Kc + uhead * (size_t)a.cap * 64;
    const uint16_t* const vb = lt.Vt + uhead * 64 * (size_t)a.cap;
    // A wavefront holds one 64-key chunk of cached keys / values in registers.  The first one does
    // not depend on this step; it is requested behind the QKV stage's block read, two hand-offs
    // before attention needs it.
    uint4 kf[4][2], vf[4][2];
    // the wavefront's first chunk, without a branch (see opaque_mask): a wavefront that has none
    // re-reads one piece of the head's first key
    auto first_chunk = [&]() {
      const bool use = c_lo + wave < c_hi;
      const int m = opaque_mask(use);
      const int key0 = (c_lo + wave) << 6;
      const gptr16 kq = as_global(kb), vq = as_global(vb);             // 16-byte pieces
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int piece = ((key0 + (r >> 2) * 16 + t * 4 + (r & 3)) * 8 + g) & m;    // 8 pieces per key row
        kf[t][0] = ldg16(kq, piece);
        kf[t][1] = ldg16(kq, piece + (4 & m));
      }
      const int capp = a.cap >> 3;                                      // pieces per value row
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const int piece = ((dt * 16 + r) * capp + (key0 >> 3) + g * 2) & m;
        vf[dt][0] = ldg16(vq, piece);
        vf[dt][1] = ldg16(vq, piece + (1 & m));
      }
    };

    // OPROJ workgroups: their element of the residual entering the layer (four partial words),
    // read while the others run QKV and attention
    float px = 0.f;
    auto read_px = [&]() {
      const int col = om * D + (w - O_BASE) * 16 + nrow;
      const int off[4] = {row_in ? OFF_XP + col : -1, row_in ? OFF_XP + BLK + col : -1, row_in ? OFF_XP + 2 * BLK + col : -1,
                          row_in ? OFF_XP + 3 * BLK + col : -1};
      float pv[4];
      wait_words<4>(lb, off, t8, pv, ok);
      px = (pv[0] + pv[1]) + (pv[2] + pv[3]);
    };
    if (has_o) read_px();

    // ================= QKV =================
    if (has_q) {
      const f32x4 g4 = gains4(lt.g1, tid);             // gains and rotary entry: requested before waiting
      const int q_sec = w / (D / 16), q_ts = w % (D / 16), q_h = q_ts >> 2, q_tt = q_ts & 3;
      float2 cs = float2{1.f, 0.f};
      if (live && q_sec < 2) cs = a.rope[(size_t)(len_m + mj) * 32 + q_tt * 8 + (nrow & 7)];
      // From the second layer on a QKV workgroup comes here straight from its own FFN-down tile, when
      // the other tiles are landing too: it reads the four partial blocks at once instead of watching
      // a word first (the read takes longer than the stragglers do, and a row that did come too
      // early is re-read on its own) - one poll round trip less per layer.  The barriers of
      // FFN-down's tile sum already separate its LDS reads from the rows staged here.
      const bool watch0 = l == 0;
      if (few) stage_rows<4, 2, 5>(sm, As, 0, lb + OFF_XP, BLK, D, M, g4, a.eps, tid, t8, ok, nullptr, first_chunk, watch0);
      else stage_rows<4, 2, 4>(sm, As, 0, lb + OFF_XP, BLK, D, M, g4, a.eps, tid, t8, ok, nullptr, first_chunk, watch0);
      XSM_STAMP(l * 16 + 8);
      const f32x4 acc = mac_tiles<KD>(wq, As, STD, r, wave * KD, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid) * row_scale(sm, om, a.eps);
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
          st32(lb + OFF_Q + col, o, t8);
        } else {
          // new keys / values travel as the bf16 values the cache holds (exact in an exchange word)
          const uint16_t ob = f2bf(o);
          if (q_sec == 1) {
            st32(lb + OFF_KN + col, bf2f(ob), t8);
            lt.Kc[(head * a.cap + pos) * 64 + dim] = ob;
          } else {
            st32(lb + OFF_VN + col, bf2f(ob), t8);
            lt.Vt[(head * 64 + dim) * a.cap + pos] = ob;
          }
        }
      }
    }
    else first_chunk();                                   // (an attention unit without a QKV tile)
    XSM_STAMP(l * 16 + 1);

    // ================= ATT =================
    if (att) {
      // this step's q, k, v rows of (sequence b, head h): [R][64] each, staged as bf16 tiles
      uint16_t* const qs = As;                            // q: hi plane, lo plane 16 rows further
      uint16_t* const kns = As + 32 * kQS;                // new k / v: as the cache will hold them
      uint16_t* const vns = As + 48 * kQS;
      // While a wavefront works on one chunk, the next one is on its way from HBM straight into LDS
      // (LDS-direct loads: no registers - a second register set for it spills - and lane l's 16
      // bytes of a request land at base + 16 l, i.e. already in fragment order), 16 KB per wavefront
      unsigned char* const ring = dyn + 16384 + wave * 16384;
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
      if (c_lo + wave + 4 < c_hi) request_next(c_lo + wave + 4);   // the wavefront's second chunk
      watch_then_sync(lb + OFF_VN + (size_t)(b * R + R - 1) * D + h * 64 + 63, t8, ok && n >= 0, tid);
      if (n >= 0) {
        // thread (row j, four columns c4..) of the 16 x 64 q / new-k / new-v blocks of this head
        const int j = tid >> 4, c4 = 4 * (tid & 15);
        if (j < R && ok) {
          const int base = ((b * R + j) * D + h * 64 + c4) * 4;
          bool got = false;
          for (int spin = 0; spin < kSpinBudget; ++spin) {
            const u32x4 wq4 = __builtin_amdgcn_raw_buffer_load_b128(lrs, OFF_Q * 4 + base, 0, kCoherent);
            const u32x4 wk4 = __builtin_amdgcn_raw_buffer_load_b128(lrs, OFF_KN * 4 + base, 0, kCoherent);
            const u32x4 wv4 = __builtin_amdgcn_raw_buffer_load_b128(lrs, OFF_VN * 4 + base, 0, kCoherent);
            if (((tagdiff(wq4, t8) | tagdiff(wk4, t8) | tagdiff(wv4, t8)) & 0xFFu) == 0) {
              const f32x4 q4 = dec24(wq4), k4 = dec24(wk4), v4 = dec24(wv4);
              uint2 hi, lo;
              split4(float4{q4[0], q4[1], q4[2], q4[3]}, hi, lo);
              *reinterpret_cast<uint2*>(qs + j * kQS + c4) = hi;
              *reinterpret_cast<uint2*>(qs + (16 + j) * kQS + c4) = lo;
              *reinterpret_cast<uint2*>(kns + j * kQS + c4) = uint2{pk2(k4[0], k4[1]), pk2(k4[2], k4[3])};
              *reinterpret_cast<uint2*>(vns + j * kQS + c4) = uint2{pk2(v4[0], v4[1]), pk2(v4[2], v4[3])};
              got = true;
              break;
            }
            __builtin_amdgcn_s_sleep(4);
          }
          if (!got) ok = false;
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
        const float alpha = exp2_hw(m_run - m_use);
        float psum = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p = exp2_hw(sc[t][i] - m_use);
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
        const float alpha = exp2_hw(m_run - m_use);
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float p = exp2_hw(sc[i] - m_use);
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
        const float f = mw == -INFINITY ? 0.f : exp2_hw(mw - Mx);
        Lx += sm.att_ml[q][1][r] * f;
        acc += *reinterpret_cast<const f32x4*>(&sm.att_o[q][wave][lane][0]) * f;
      }
      // What leaves the unit is relative to a maximum that an exchange word holds exactly: the
      // next integer above it (a slice without keys says so with a very low maximum and sum 0;
      // rows of a skipped sequence are zeros with sum 1).
      const bool none = Mx == -INFINITY;
      const float Mref = n < 0 ? 0.f : none ? kEmptySliceMax : ceilf(Mx);
      const float resc = none ? 0.f : exp2_hw(Mx - Mref);
      const float Lout = n < 0 ? 1.f : Lx * resc;
      acc = n < 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : acc * resc;
      if (S <= 4) {
        if (r < R) {
          st32x4(lrs, OFF_OP + s * BLK + (b * R + r) * D + h * 64 + wave * 16 + g * 4, acc, t8);
          if (wave == 0 && g == 0) {
            uint32_t* ml = lb + OFF_ML + (size_t)(((b * R + r) * H + h) * 4 + s) * 2;
            st32(ml, Mref, t8);
            st32(ml + 1, Lout, t8);
          }
        }
      } else {
        uint32_t* part = lb + OFF_P + (size_t)w * 1056;
        if (wave == 0 && g == 0) {
          st32(part + r, Mref, t8);
          st32(part + 16 + r, Lout, t8);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) st32(part + 32 + (size_t)(wave * 16 + g * 4 + i) * 16 + r, acc[i], t8);
      }
    }
    XSM_STAMP(l * 16 + 2);

    // ================= COMB (8 or 16 key slices) =================
    if (S > 4 && att) {
      const int dps = 64 / S;                               // dims finished by this unit
      const int P = 32 + dps * 16;                          // words needed from each slice: m, l, O^T rows
      const uint32_t* p0 = lb + OFF_P + (size_t)(w - s) * 1056;
      float* const cb = reinterpret_cast<float*>(As);       // [S][P]
      watch_then_sync(p0 + (size_t)(S - 1) * 1056 + 32 + (s * dps + dps - 1) * 16, t8, ok, tid);
      if (ok) {
        // 16-byte pieces tid + 256 q of the S x P words (P is a multiple of 4: a piece stays inside
        // one slice and on one side of its (m, l) words)
        const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p0), 0, S * 1056 * 4, kRawBufferFlags);
        int off[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int i = 4 * (tid + 256 * q);
          const int k = i / P, j = i % P;
          off[q] = i < S * P ? k * 1056 + (j < 32 ? j : 32 + s * dps * 16 + (j - 32)) : -1;
        }
        bool got = false;
        for (int spin = 0; spin < kSpinBudget; ++spin) {
          u32x4 pq[2];
          uint32_t bad = 0;
#pragma unroll
          for (int q = 0; q < 2; ++q)
            if (off[q] >= 0) pq[q] = __builtin_amdgcn_raw_buffer_load_b128(prs, off[q] * 4, 0, kCoherent);
#pragma unroll
          for (int q = 0; q < 2; ++q)
            if (off[q] >= 0) bad |= tagdiff(pq[q], t8);
          if ((bad & 0xFFu) == 0) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
              if (off[q] >= 0) *reinterpret_cast<f32x4*>(cb + 4 * (tid + 256 * q)) = dec24(pq[q]);
            got = true;
            break;
          }
          __builtin_amdgcn_s_sleep(4);
        }
        if (!got) ok = false;
      }
      __syncthreads();
      for (int qd = tid >> 4; qd < dps; qd += 16) {
        const int rq = tid & 15;
        if (rq < R) {
          float Mg = -INFINITY;
          for (int k = 0; k < S; ++k) Mg = fmaxf(Mg, cb[k * P + rq]);
          float Lg = 0.f, og = 0.f;
          for (int k = 0; k < S; ++k) {
            const float f = exp2_hw(cb[k * P + rq] - Mg);
            Lg += cb[k * P + 16 + rq] * f;
            og += cb[k * P + 32 + qd * 16 + rq] * f;
          }
          const float outv = (sm.len[b] >= 0 && Lg > 0.f) ? og / Lg : 0.f;
          st32(lb + OFF_OP + (size_t)(b * R + rq) * D + h * 64 + s * dps + qd, outv, t8);
        }
      }
      // the merged rows stand in partial block 0 with maximum 0 and sum 1
      if (s == 0 && tid < R) {
        uint32_t* ml = lb + OFF_ML + (size_t)(((b * R + tid) * H + h) * 4) * 2;
        st32(ml, 0.f, t8);
        st32(ml + 1, 1.f, t8);
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
      __syncthreads();
      // lane (head of the wavefront's four, producer j): the word that producer's last wavefront
      // stores last.  Up to 4 slices: unit (sequence, slice) of the head, its partial row R - 1,
      // dim 63; merged slices: unit (sequence, slice) finished dims s dps .. of block 0
      int watch_off = -1;
      {
        const int hh = 4 * wave + (lane & 3), j = lane >> 2, P = S > 4 ? S : S_eff;
        if (j < n_seq * P) {
          const int row = (j / P) * R + R - 1, sl = j % P;
          watch_off = S > 4 ? OFF_OP + row * D + hh * 64 + sl * (64 / S) + 64 / S - 1
                            : OFF_OP + sl * BLK + row * D + hh * 64 + 63;
        }
      }
      // (the number of partial blocks as a template argument: loads, tag checks and the merge of the
      // slices that are not there drop out of the code instead of being predicated)
#define XSM_ATTN_OUT(RB_, SE_) stage_attn_out<H, RB_, SE_>(sm, As, lrs, lb, watch_off, OFF_OP, BLK, OFF_ML, M, tid, t8, ok)
      if (few) {
        if (S_eff == 1) XSM_ATTN_OUT(5, 1); else if (S_eff == 2) XSM_ATTN_OUT(5, 2); else XSM_ATTN_OUT(5, 4);
      } else {
        if (S_eff == 1) XSM_ATTN_OUT(4, 1); else if (S_eff == 2) XSM_ATTN_OUT(4, 2); else XSM_ATTN_OUT(4, 4);
      }
#undef XSM_ATTN_OUT
      XSM_STAMP(l * 16 + 14);
      const f32x4 acc = mac_tiles<KD>(wq, As, STD, r, wave * KD, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid);
      xm = px + v;
      if (row_in) st32(lb + OFF_XM + (size_t)om * D + nt * 16 + nrow, xm, t8);
    }
    XSM_STAMP(l * 16 + 4);

    // ================= UP =================
    if (has_u) {
      const f32x4 g4 = gains4(lt.g2, tid);
      __syncthreads();
      // (rows a round as a template argument: with 5 rows, a round sized for 8 spends a third of
      // its staging arithmetic on rows that do not exist)
      if (few) stage_rows<1, 2, 5>(sm, As, 0, lb + OFF_XM, 0, D, M, g4, a.eps, tid, t8, ok, tl ? tl + l * 16 + 13 : nullptr);
      else stage_rows<1, 2, 8>(sm, As, 0, lb + OFF_XM, 0, D, M, g4, a.eps, tid, t8, ok, tl ? tl + l * 16 + 13 : nullptr);
      XSM_STAMP(l * 16 + 7);
      const f32x4 acc = mac_tiles<KD>(wu, As, STD, r, wave * KD, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid) * row_scale(sm, om, a.eps);
      if (row_in) st32(lb + OFF_U + (size_t)om * F + w * 16 + nrow, 0.5f * v * (1.0f + erff(v * 0.70710678118654752f)), t8);
    }
    XSM_STAMP(l * 16 + 5);

    // ================= DOWN =================
    {
      __syncthreads();
      if (few) stage_rows<1, 0, 5>(sm, As, 0, lb + OFF_U + d_ks * FS, 0, F, M, f32x4{1.f, 1.f, 1.f, 1.f}, a.eps, tid, t8, ok);
      else stage_rows<1, 0, 8>(sm, As, 0, lb + OFF_U + d_ks * FS, 0, F, M, f32x4{1.f, 1.f, 1.f, 1.f}, a.eps, tid, t8, ok);
      XSM_STAMP(l * 16 + 12);
      const f32x4 acc = mac_tiles<KFS>(wd, As, STD, r, wave * KFS, g);
      const float v = tile_reduce(sm, acc, wave, lane, tid);
      // partial block d_ks of the next layer's input; the last slice's workgroup made this tile's
      // mid-layer residual in OPROJ and adds it to its own partial
      if (row_in) st32(lb + LS + OFF_XP + (size_t)d_ks * BLK + (size_t)om * D + d_nt * 16 + nrow, d_ks == 3 ? xm + v : v, t8);
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
        if (w < n_seq) report_timeout(w);
      }
      return;
    }
  }

  // =========================== tail ===========================
  uint32_t* const tb = llb + (size_t)a.L * LS;             // the last layer's output partials live at the start of this block
  constexpr int OFF_RB = 4 * BLK;                          // head outputs: [16*K rows][D] words
  constexpr int OFF_ST = OFF_RB + 16 * 15 * D;             // per (row, tile) top-2 statistics: 4 8-byte words, a row's tiles side by side
  constexpr int kStatTiles = 4096;                         // tiles per row the region is laid out for
  uint64_t* const stb = reinterpret_cast<uint64_t*>(tb + OFF_ST);
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
    const f32x4 g4 = gains4(a.gf, tid);
    __syncthreads();
    // (read without a watch poll, like the QKV stage's input: every workgroup comes here from its
    // own tile of the last FFN-down)
    if (few) stage_rows<4, 1, 5>(sm, T0, 0, tb + OFF_XP, BLK, D, M, g4, a.eps, tid, t8, ok, nullptr, NothingBehind{}, false);
    else stage_rows<4, 1, 4>(sm, T0, 0, tb + OFF_XP, BLK, D, M, g4, a.eps, tid, t8, ok, nullptr, NothingBehind{}, false);
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
      st32(tb + OFF_RB + ((size_t)om * K + kh) * D + c, gn + pre / (1.0f + __expf(-pre)), t8);
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
      if (q_hi > q_lo)
        stage_rows<1, 0, 12>(sm, T, q_lo - mt * 16, tb + OFF_RB + (size_t)(q_lo - M) * D, 0, D, q_hi - q_lo,
                         f32x4{1.f, 1.f, 1.f, 1.f}, a.eps, tid, t8, ok);
    }
    for (int t = w; t < NTV; t += 256) {
      if (t != w) load_frags<KD>(wv, a.WU, t, KTD, wave * KD, lane);
      const f32x4 acc = mac_tiles<KD>(wv, T, STD, r, wave * KD, g);
      __syncthreads();
      *reinterpret_cast<f32x4*>(&sm.red[wave][lane][0]) = acc;
      __syncthreads();
      // The logits themselves, where somebody reads them (every criterion but greedy-with-argmax, and
      // the debug copies): thread (row tid / 16, column tid % 16) stores its entry with a
      // device-coherent store and waits for it, so that after the barrier the whole tile has
      // arrived; the statistics words stored after it double as the completion flag of this
      // tile's piece of each row
      if (a.logits_dbg) {
        const int q = mt * 16 + (tid >> 4), nr = tid & 15;
        float* dbg = nullptr;
        if (q < M) dbg = a.logits_dbg + (size_t)q * V;
        else if (q < rows_all && a.head_logits_dbg) dbg = a.head_all_dbg + (size_t)(q - M) * V;
        if (dbg) {
          const int ln = (nr >> 2) * 16 + (tid >> 4), ii = nr & 3;
          const float z = (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
          __hip_atomic_store(dbg + t * 16 + nr, z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
      }
      // threads 0..15: row q = mt*16 + tid; scan the tile's 16 vocabulary entries in order
      if (tid < 16 && mt * 16 + tid < rows_all) {
        const int q = mt * 16 + tid;
        float bv = -INFINITY, sv = -INFINITY;
        int bi = 0;
#pragma unroll
        for (int nr = 0; nr < 16; ++nr) {
          const int ln = (nr >> 2) * 16 + tid, ii = nr & 3;
          const float z = (sm.red[0][ln][ii] + sm.red[1][ln][ii]) + (sm.red[2][ln][ii] + sm.red[3][ln][ii]);
          if (z > bv) { sv = bv; bv = z; bi = t * 16 + nr; }
          else sv = fmaxf(sv, z);
        }
        uint64_t* st = stb + ((size_t)q * kStatTiles + t) * 4;
        ll_st(st, __float_as_uint(bv), tag);
        ll_st(st + 1, (uint32_t)bi, tag);
        ll_st(st + 2, __float_as_uint(sv), tag);
      }
    }
    // a workgroup with several vocabulary tiles starts the next row tile from its first again
    if (NTV > 256 && w < NTV && mt + 1 < n_mt) load_frags<KD>(wv, a.WU, w, KTD, wave * KD, lane);
  }
  XSM_STAMP(a.L * 16 + 3);

  // ---- FINAL: workgroup b finishes sequence b.  Greedy verification with argmax draws works from
  // the per-tile statistics alone.  The other criteria and sampling rules need whole logits rows
  // (Sec. 5.4 "Verification criterion"; appendix "Sampling strategies"): every accept check, and
  // every draw for every possible accepted length, is a task of its own on its own workgroup, all
  // of them side by side; a task posts its result as a tagged word and workgroup b picks the
  // ones its accepted length selects ----
  uint64_t* const res = stb + 3;                           // result word i: the spare fourth word of statistics group i
  const int slots_seq = K + R * R;                         // per sequence: K checks, then (accepted length, draw)
  uint64_t* const top2_res = res + (size_t)3072 * 4;       // greedy: three words per logits row, behind the tree levels
  // Global top-2 of nr logits rows (row i = grow_of(i)) from their per-tile statistics -> slots
  // slot0 + i of sm.st_*.  All rows at once: thread t takes tiles t, t + 256, ... of every row
  // (two 16-byte loads per row and tile, up to eight rows' loads in flight together), the lanes
  // of a wavefront are folded, and thread i combines the four wavefronts' results of row i in
  // wavefront order.  Called by the whole workgroup.
  __shared__ float t2v[4][16], t2s[4][16];
  __shared__ int t2i[4][16];
  const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(stb, 0, kSmallMaxRows * kStatTiles * 32, kRawBufferFlags);
  auto top2_rows = [&](int nr, auto&& grow_of, int slot0) {
    for (int i0 = 0; i0 < nr; i0 += 8) {
      float bv[8], sv[8];
      int bi[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { bv[i] = -INFINITY; sv[i] = -INFINITY; bi[i] = 0x7FFFFFFF; }
      for (int t = tid; t < NTV; t += 256) {
        u32x4 qa[8], qb[8];
        bool got = false;
        for (int spin = 0; ok && spin < kSpinBudget; ++spin) {
          uint32_t bad = 0;
#pragma unroll
          for (int i = 0; i < 8; ++i)
            if (i0 + i < nr) {
              const int off = (grow_of(i0 + i) * kStatTiles + t) * 32;
              qa[i] = __builtin_amdgcn_raw_buffer_load_b128(srs, off, 0, kCoherent);
              qb[i] = __builtin_amdgcn_raw_buffer_load_b128(srs, off + 16, 0, kCoherent);
            }
#pragma unroll
          for (int i = 0; i < 8; ++i)
            if (i0 + i < nr) bad |= (qa[i].y ^ tag) | (qa[i].w ^ tag) | (qb[i].y ^ tag);
          if (bad == 0) { got = true; break; }
          __builtin_amdgcn_s_sleep(4);
        }
        if (!got) { ok = false; break; }
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (i0 + i < nr) {
            const float tv = __uint_as_float(qa[i].x), ts = __uint_as_float(qb[i].x);
            const int ti = (int)qa[i].z;
            if (tv > bv[i] || (tv == bv[i] && ti < bi[i])) { sv[i] = fmaxf(bv[i], fmaxf(sv[i], ts)); bv[i] = tv; bi[i] = ti; }
            else sv[i] = fmaxf(sv[i], fmaxf(tv, ts));
          }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (i0 + i >= nr) break;                            // (uniform)
#define XSM_FOLD(O)                                                                \
        {                                                                        \
          const float bv2 = lane_xor<O>(bv[i]), sv2 = lane_xor<O>(sv[i]);        \
          const int bi2 = lane_xor<O>(bi[i]);                                    \
          const bool take = (bv2 > bv[i]) || (bv2 == bv[i] && bi2 < bi[i]);      \
          sv[i] = fmaxf(fmaxf(sv[i], sv2), fminf(bv[i], bv2));                   \
          if (take) { bv[i] = bv2; bi[i] = bi2; }                                \
        }
        XSM_FOLD(32) XSM_FOLD(16) XSM_FOLD(8) XSM_FOLD(4) XSM_FOLD(2) XSM_FOLD(1)
#undef XSM_FOLD
        if (lane == 0) { t2v[wave][i] = bv[i]; t2s[wave][i] = sv[i]; t2i[wave][i] = bi[i]; }
      }
      __syncthreads();
      if (tid < 8 && i0 + tid < nr) {
        float cv = t2v[0][tid], cs = t2s[0][tid];
        int ci = t2i[0][tid];
        for (int q = 1; q < 4; ++q) {
          const float v2 = t2v[q][tid], s2 = t2s[q][tid];
          const int i2 = t2i[q][tid];
          const bool take = (v2 > cv) || (v2 == cv && i2 < ci);
          cs = fmaxf(fmaxf(cs, s2), fminf(cv, v2));
          if (take) { cv = v2; ci = i2; }
        }
        sm.st_max[slot0 + i0 + tid] = cv; sm.st_sec[slot0 + i0 + tid] = cs; sm.st_idx[slot0 + i0 + tid] = ci;
      }
      __syncthreads();
    }
  };
  if (a.full_verify) {
    const xsm_verify_params& vp = a.vp;
    const float invT = 1.0f / vp.temperature;
    RowScratch& rs = *reinterpret_cast<RowScratch*>(&sm.att_o[0][0][0][0]);
    __shared__ int tree_tok[17];
    __shared__ TreeLevels lv;
    // Tasks per sequence: K accept checks, then per accepted length the draws.  Categorical: the
    // backbone's token and each head's.  Tree: the backbone's token, each head's level of the
    // tree, and (in a second group behind all of these, which it waits for) the joint draw of the
    // heads.  Argmax draws come from the statistics and need no task.
    const int ks = vp.top_ks;
    const int per_m = vp.sample == 0 ? 0 : R;
    const int per_seq = K + R * per_m;
    const int n_first = n_seq * per_seq;
    const int n_tasks = n_first + (vp.sample == 2 && K > 0 ? n_seq * R : 0);
    uint64_t* const lev = res + (size_t)512 * 4;          // tree levels: 8 words per head row, behind the result words
    // true (in every thread) once logits rows [g0, g0 + nr) are complete: their statistics words
    // of all tiles carry the tag, and each was stored after its tile's piece of the row had arrived
    auto rows_complete = [&](int g0, int nr) {
      bool live = !__syncthreads_or(!ok);
      for (int spin = 0; live; ++spin) {
        bool good = true;
        for (int i = tid; i < nr * NTV; i += 256)
          good &= (uint32_t)(ll_ld(stb + ((size_t)(g0 + i / NTV) * kStatTiles + i % NTV) * 4) >> 32) == tag;
        if (__syncthreads_and(good)) break;
        if (spin >= kSpinBudget) { ok = false; live = false; }
        __builtin_amdgcn_s_sleep(4);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      return live;
    };
    // (tasks go to the workgroups from the far end: the low ones finish sequences)
    for (int task = 255 - w; task < n_tasks; task += 256) {
      if (task >= n_first) {                               // joint draw of the heads for accepted length m
        const int b = (task - n_first) / R, m = (task - n_first) % R;
        const int n = sm.len[b];
        if (n < 0) continue;
        if (tid < K * ks * 2) {
          const int k = tid / (2 * ks), j = tid % (2 * ks);
          const int off[1] = {(((b * R + m) * K + k) * 8 + j) * 4};
          uint32_t pw[1];
          ll_wait_list<1>(lev, off, tag, pw, ok);
          if (j < ks) lv.idx[k][j] = (int)pw[0];
          else lv.p[k][j - ks] = __uint_as_float(pw[0]);
        }
        if (__syncthreads_or(!ok)) break;
        const bool nb = pts_pick(lv, K, ks, vp.pts_prune, philox_uniform(vp.seed, (uint32_t)(n + m + 1), 254u, (uint32_t)sm.slot[b]),
                                 rs, tree_tok);
        if (tid < K)
          ll_st(res + (size_t)(b * slots_seq + K + m * R + tid + 1) * 4, (uint32_t)tree_tok[tid + 1] | (nb ? 0x80000000u : 0u), tag);
        __syncthreads();
        continue;
      }
      const int b = task / per_seq, i = task % per_seq;
      const int n = sm.len[b];
      if (n < 0) continue;
      uint64_t* const out = res + (size_t)b * slots_seq * 4;
      if (i < K) {                                         // accept check of candidate j = i + 1 against row j - 1
        const int grow = b * R + i;
        if (!rows_complete(grow, 1)) break;
        const float* z = a.logits_dbg + (size_t)grow * V;
        const int x = sm.blk[b * R + i + 1];
        bool nb;
        const bool good = row_accepts(z, V, x, vp, rs, &nb);
        if (tid == 0) ll_st(out + (size_t)i * 4, (good ? 1u : 0u) | (nb ? 2u : 0u), tag);
      } else {
        const int m = (i - K) / per_m, d = (i - K) % per_m;  // accepted length; 0 = the backbone's draw
        const uint32_t pos0 = (uint32_t)(n + m + 1), sq = (uint32_t)sm.slot[b];
        uint64_t* const om_ = out + (size_t)(K + m * R) * 4;
        if (d == 0 || vp.sample == 1) {
          const int grow = d == 0 ? b * R + m : M + (b * R + m) * K + d - 1;
          if (!rows_complete(grow, 1)) break;
          const float* z = d == 0 ? a.logits_dbg + (size_t)grow * V : a.head_all_dbg + (size_t)(grow - M) * V;
          bool nb;
          const int t = row_draw(z, V, invT, philox_uniform(vp.seed, pos0 + (uint32_t)d, (uint32_t)d, sq), rs, &nb);
          if (tid == 0) ll_st(om_ + (size_t)d * 4, (uint32_t)t | (nb ? 0x80000000u : 0u), tag);
        } else {                                           // level d - 1 of the tree: head d's ks most probable tokens
          const int grow = M + (b * R + m) * K + d - 1;
          if (!rows_complete(grow, 1)) break;
          row_level(a.head_all_dbg + (size_t)(grow - M) * V, V, ks, invT, rs, lv.idx[0], lv.p[0]);
          uint64_t* const lo = lev + (size_t)(grow - M) * 8 * 4;
          if (tid < ks) {
            ll_st(lo + (size_t)tid * 4, (uint32_t)lv.idx[0][tid], tag);
            ll_st(lo + (size_t)(ks + tid) * 4, __float_as_uint(lv.p[0][tid]), tag);
          }
        }
      }
      __syncthreads();
    }
  } else {
    // greedy with argmax draws: one task per logits row folds the row's per-tile statistics and
    // posts (maximum, its token, runner-up); all rows side by side instead of three rounds of
    // rows in the finishing workgroup
    for (int task = 255 - w; task < rows_all; task += 256) {
      top2_rows(1, [&](int) { return task; }, 0);
      if (tid < 3 && ok) {
        const uint32_t pay = tid == 0 ? __float_as_uint(sm.st_max[0]) : tid == 1 ? (uint32_t)sm.st_idx[0] : __float_as_uint(sm.st_sec[0]);
        ll_st(top2_res + (size_t)(task * 3 + tid) * 4, pay, tag);
      }
      __syncthreads();
    }
  }
  if (w < n_seq) {
    const int b = w;
    const int n = sm.len[b];
    if (a.full_verify) {
      __shared__ int cand[17];                            // [0] the backbone's token, [k] head k's
      __shared__ uint32_t chk_s[16], near_s[17];
      const xsm_verify_params& vp = a.vp;
      const int base = b * slots_seq * 4;
      uint32_t fl = sm.flag[b];
      int acc_n = 0;
      bool late = false;
      if (n >= 0) {
        if (tid < K) {
          const int off[1] = {base + tid * 4};
          uint32_t pw[1];
          ll_wait_list<1>(res, off, tag, pw, ok);
          chk_s[tid + 1] = pw[0];
        }
        late = __syncthreads_or(!ok);
        if (!late)
          for (int j = 1; j <= K; ++j) {                    // accept until the first candidate that fails
            if (chk_s[j] & 2u) fl |= XSM_FLAG_NEAR_TIE;
            if (!(chk_s[j] & 1u)) break;
            ++acc_n;
          }
        // draw d of the accepted length: 0 = the backbone's token from row acc_n, k = head k's
        if (vp.sample == 0) {
          top2_rows(K + 1, [&](int d) { return d == 0 ? b * R + acc_n : M + (b * R + acc_n) * K + d - 1; }, 0);
          if (tid <= K) { cand[tid] = sm.st_idx[tid]; near_s[tid] = sm.st_max[tid] - sm.st_sec[tid] <= kTieMargin ? 1u : 0u; }
        } else if (tid <= K) {
          const int off[1] = {base + (K + acc_n * R + tid) * 4};
          uint32_t pw[1];
          ll_wait_list<1>(res, off, tag, pw, ok);
          cand[tid] = (int)(pw[0] & 0x7FFFFFFFu);
          near_s[tid] = pw[0] >> 31;
        }
        late = __syncthreads_or(!ok) || late;
      }
      if (tid == 0) {
        if (late) {
          report_timeout(b);
        } else if (n < 0) {
          a.n_accepted[b] = 0;
          a.flags[b] = fl;
        } else {
          for (int d = 0; d <= K; ++d)
            if (near_s[d]) fl |= XSM_FLAG_NEAR_TIE;
          int oldb[16];
          for (int j = 0; j < R; ++j) oldb[j] = sm.blk[b * R + j];
          const int y0 = cand[0];
          for (int j = 0; j < acc_n; ++j) a.out_tokens[b * R + j] = oldb[j + 1];
          a.out_tokens[b * R + acc_n] = y0;
          for (int j = acc_n + 1; j < R; ++j) a.out_tokens[b * R + j] = -1;
          a.block[b * R] = y0;
          for (int k = 1; k <= K; ++k) a.block[b * R + k] = cand[k];
          a.n_accepted[b] = acc_n + 1;
          a.kv_len[b] = n + acc_n + 1;
          a.flags[b] = fl;
          if (a.acc_out) a.acc_out[b] = acc_n;
        }
      }
    } else {
    // the folded rows of this sequence: slots 0 .. R - 1 the backbone rows, slot R + j K + k head
    // k's row at accepted length j
    for (int i = tid; i < (R + R * K) * 3; i += 256) {
      const int q = i / 3, grow = q < R ? b * R + q : M + b * R * K + (q - R);
      const int off[1] = {(grow * 3 + i % 3) * 4};
      uint32_t pw[1];
      ll_wait_list<1>(top2_res, off, tag, pw, ok);
      if (i % 3 == 0) sm.st_max[q] = __uint_as_float(pw[0]);
      else if (i % 3 == 1) sm.st_idx[q] = (int)pw[0];
      else sm.st_sec[q] = __uint_as_float(pw[0]);
    }
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
          const bool hit = sm.blk[b * R + j] == sm.st_idx[j - 1];
          if (sm.st_max[j - 1] - sm.st_sec[j - 1] <= kTieMarginS) fl |= XSM_FLAG_NEAR_TIE;
          if (!hit) break;
          ++acc_n;
        }
        if (sm.st_max[acc_n] - sm.st_sec[acc_n] <= kTieMarginS) fl |= XSM_FLAG_NEAR_TIE;
        int oldb[16];
        for (int j = 0; j < R; ++j) oldb[j] = sm.blk[b * R + j];
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
  }
  XSM_STAMP(a.L * 16 + 4);
  if (__syncthreads_or(!ok)) {
    if (tid == 0) {
      __hip_atomic_store(a.ctrl + 1, 1000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (w < n_seq) report_timeout(w);
    }
    return;
  }
  // workgroup 0 closes the step: its FINAL needed every workgroup's statistics, so every
  // workgroup has long since read the epoch
  if (w == 0 && tid == 0)
    __hip_atomic_store(a.ctrl, tag + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#undef XSM_STAMP
}

// 4-byte words of one layer's exchange buffers, and of the whole region (layers + tail)
size_t small_ll_layer_stride(int D, int F) {
  return (size_t)12 * 16 * D + (size_t)16 * (D / 64) * 8 + (size_t)16 * F + (size_t)256 * 1056;
}
size_t small_ll_words(int n_layers, int D, int F, int K) {
  const size_t layer = small_ll_layer_stride(D, F);
  const size_t tail = (size_t)4 * 16 * D + (size_t)16 * 15 * D + (size_t)4096 * kSmallMaxRows * 4 * 2;
  (void)K;
  return layer * n_layers + (tail > layer ? tail : layer);
}

bool small_supported(int D, int F) { return D == 1024 && F == 4096; }

template <int RC, int BC, int VC = 0, bool TL = false>
static void launch_small_t(const SmallArgs& a, size_t lds, hipStream_t s) {
  auto kfn = k_step_small<1024, 4096, RC, BC, VC, TL>;
  allow_dynamic_lds((const void*)kfn, lds);
  hipLaunchKernelGGL(kfn, dim3(256), dim3(256), lds, s, a);
}

void launch_step_small(const SmallArgs& a, int D, int F, hipStream_t s) {
  TraceScope trace_("step_small", s);
  if (D == 1024 && F == 4096 && a.ll_words * 4 < ((size_t)1 << 31)) {
    // activation tiles as bf16 hi + lo planes: two 16-row model-width tiles in the tail
    const size_t lds = (size_t)4 * 16 * (1024 + 8) * 2;
    // One sequence with K = 0, 2, 4 or 8 heads, two or three with K = 4, plain steps of eight: the rows per sequence and the batch are compile-time
    // constants of the instantiation (row loops and their predicates fold away: 8 % of a K = 4
    // step), for K = 4 with the latency model's vocabulary also that (1.3 %); everything else takes
    // the instantiation that reads them from the arguments.
    if (a.tlog) {                                          // the stage clock was asked for
      if (a.n_seq == 1 && a.R == 5 && a.V == 4096) launch_small_t<5, 1, 4096, true>(a, lds, s);
      else launch_small_t<0, 0, 0, true>(a, lds, s);
    } else if (a.n_seq == 1 && a.R == 5 && a.V == 4096) launch_small_t<5, 1, 4096>(a, lds, s);
    else if (a.n_seq == 1 && a.R == 5) launch_small_t<5, 1>(a, lds, s);
    else if (a.n_seq == 2 && a.R == 5) launch_small_t<5, 2>(a, lds, s);
    else if (a.n_seq == 3 && a.R == 5) launch_small_t<5, 3>(a, lds, s);
    else if (a.n_seq == 1 && a.R == 1) launch_small_t<1, 1>(a, lds, s);
    else if (a.n_seq == 8 && a.R == 1) launch_small_t<1, 8>(a, lds, s);
    else if (a.n_seq == 1 && a.R == 3) launch_small_t<3, 1>(a, lds, s);
    else if (a.n_seq == 1 && a.R == 9) launch_small_t<9, 1>(a, lds, s);
    else launch_small_t<0, 0>(a, lds, s);
  }
}

}  // namespace xsm
