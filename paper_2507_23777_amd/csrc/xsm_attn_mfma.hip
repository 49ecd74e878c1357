// Block-causal KV-cache attention for R query rows per sequence on bf16 MFMA (gfx950),
// head_dim 64.  Query row j of sequence b sits at position n_b + j and sees cache positions
// 0..n_b + j (Sec. 4.2: causal mask inside the draft block x_{s:s+D}).  k_fattn: a workgroup takes
// one tile of 16 query rows (a speculative step has one tile); k_pattn, further down, serves the
// prefill passes with many tiles per sequence.
//
// HBM-bound: every cached key and value is read once per step, so the layout is chosen for
// the loads.  Keys are [position][64] (128 B rows); values are stored transposed,
// [64][capacity], so that both MFMA "A" operands are read with 16-byte lane loads:
//   S^T[key][query] = K[key][:] . Q[query][:]      A = 16 keys x 32 dims of K
//   O^T[dim][query] = V^T[dim][key] . P^T[key][query]   A = 16 dims x 32 keys of V^T
// A wavefront takes 64 keys at a time.  The 16-key score tiles are formed from keys
// {g*16 + t*4 + i}, so that the probabilities a lane holds after the first product are
// exactly the 16 consecutive keys it must supply as the "B" operand of the second one, and no
// cross-lane movement is needed.  The fp32 queries and probabilities enter the MFMAs as bf16
// hi + lo operand pairs, so the only bf16 rounding left in attention is the cache's own.
// Online softmax in fp32 (base 2); the key range of one
// (sequence, head) is split over S workgroups whose partial (max, sum, O) are merged in
// fixed order by the last one to finish.
#include "xsm_device.h"
#include "xsm_internal.h"

namespace xsm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPartFloats = (2 + 64) * 16;     // per split: m[16], l[16], O^T[64][16]

__device__ __forceinline__ void st_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_coherent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t pack2(float a, float b) { return f2bf_pair(a, b); }

// (a, b) -> packed bf16 pair of the rounded values and of what the rounding dropped
__device__ __forceinline__ void split2(float a, float b, uint32_t& hi, uint32_t& lo) {
  hi = pack2(a, b);
  lo = pack2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}

// four consecutive dims (col % 4 == 0) of output row `row`: fp32, or operand planes for the projection that follows
__device__ __forceinline__ void store_out4(const FastAttn& a, int row, int col, float4 v) {
  if (a.o_planes) plane_store4(a.O, a.o_rows, a.ldo, row, col, v);
  else *reinterpret_cast<float4*>(a.O + (size_t)row * a.ldo + col) = v;
}

// fp32 query row (64 dims at q, or nullptr for an MFMA column with no query) -> the lane's operand
// halves (dims g*8.. and 32 + g*8..), each as bf16 hi and lo parts
__device__ __forceinline__ void load_queries(const FastAttn& a, bf16x8 (&qh)[2], bf16x8 (&ql)[2], const float* q, int g) {
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    float qv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (q) {
      const float4 x0 = *reinterpret_cast<const float4*>(q + half * 32 + g * 8);
      const float4 x1 = *reinterpret_cast<const float4*>(q + half * 32 + g * 8 + 4);
      qv[0] = x0.x; qv[1] = x0.y; qv[2] = x0.z; qv[3] = x0.w;
      qv[4] = x1.x; qv[5] = x1.y; qv[6] = x1.z; qv[7] = x1.w;
    }
    uint32_t hw[4], lw[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split2(qv[2 * e], qv[2 * e + 1], hw[e], lw[e]);
    qh[half] = __builtin_bit_cast(bf16x8, uint4{hw[0], hw[1], hw[2], hw[3]});
    ql[half] = __builtin_bit_cast(bf16x8, uint4{lw[0], lw[1], lw[2], lw[3]});
  }
}

// One 64-key chunk (keys key0..key0+63, fragments kf / vf as the cache loads deliver them) for the
// wavefront's 16 queries: scores, online softmax (base 2), second product.  Query r sees keys
// below lim; below first_masked every live query sees the key; keys at or past Ltot may hold
// garbage (their values are zeroed so that 0 x garbage cannot become NaN).
__device__ __forceinline__ void attn_chunk(const uint4 (&kf)[4][2], uint4 (&vf)[4][2], const bf16x8 (&qh)[2],
                                           const bf16x8 (&ql)[2], int key0, int g, bool qlive, int lim,
                                           int first_masked, int Ltot, float scale_log2, float& m_run,
                                           float& l_run, f32x4 (&o)[4]) {
  f32x4 sc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const bf16x8 kk = __builtin_bit_cast(bf16x8, kf[t][half]);
      sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, ql[half], sc[t], 0, 0, 0);
      sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, qh[half], sc[t], 0, 0, 0);
    }
  }
  // this lane's 16 scores belong to keys key0 + g*16 + t*4 + i
  const int kbase = key0 + g * 16;
  const bool edge = key0 + 64 > first_masked || !qlive;
  float cmax = -INFINITY;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v = sc[t][i] * scale_log2;
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
  if (key0 + 64 > Ltot) {                         // slots past the live range hold garbage
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        uint32_t* w = reinterpret_cast<uint32_t*>(&vf[dt][jj]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (kbase + jj * 8 + e >= Ltot) w[e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
        }
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
}

__global__ __launch_bounds__(256) void k_fattn(const FastAttn a) {
  __shared__ float sm_ml[4][2][16];
  __shared__ __align__(16) float sm_o[4][4][64][4];
  __shared__ int sm_last;
  const int S = a.S, QT = (a.R + 15) >> 4;
  const int s = blockIdx.x % S, qt = blockIdx.x / S, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int R = min(16, a.R - qt * 16);            // query rows of this tile
  const int row0 = b * a.R + qt * 16;              // its first row in Q / O
  const int nseq = a.eff_len[b];
  if (nseq < 0) {                                  // skipped sequence: defined (zero) output
    if (s == 0)
      for (int i = tid; i < R * 16; i += 256)
        store_out4(a, row0 + i / 16, h * 64 + (i & 15) * 4, float4{0.f, 0.f, 0.f, 0.f});
    return;
  }
  const int n = nseq + qt * 16;                    // keys every query of this tile sees
  const int Ltot = a.fixed_limit > 0 ? a.fixed_limit : n + R;
  const int NC = (Ltot + 63) >> 6, CPS = (NC + S - 1) / S;
  const int c_lo = s * CPS, c_hi = min(NC, c_lo + CPS);
  const size_t head = (size_t)a.slot[b] * a.H + h;
  const uint16_t* kb = a.Kc + head * (size_t)a.cap * 64;
  const uint16_t* vb = a.Vt + head * 64 * (size_t)a.cap;
  // keys visible to this lane's query: positions < lim
  const int lim = r < R ? (a.fixed_limit > 0 ? Ltot : n + r + 1) : 0;
  const int first_masked = a.fixed_limit > 0 ? Ltot : n + 1;     // below this every live query sees the key

  bf16x8 qh[2], ql[2];
  load_queries(a, qh, ql, r < R ? a.Q + (size_t)(row0 + r) * a.ldq + h * 64 : nullptr, g);

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

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
    attn_chunk(kf, vf, qh, ql, key0, g, r < R, lim, first_masked, Ltot, a.scale_log2, m_run, l_run, o);
  }

  // merge the four wavefronts (fixed order); wavefront w finishes dim tile w
  if (g == 0) { sm_ml[wave][0][r] = m_run; sm_ml[wave][1][r] = l_run; }
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) *reinterpret_cast<f32x4*>(&sm_o[wave][dt][lane][0]) = o[dt];
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; ++w) M = fmaxf(M, sm_ml[w][0][r]);
  float L = 0.f;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float mw = sm_ml[w][0][r];
    const float f = mw == -INFINITY ? 0.f : exp2f(mw - M);
    L += sm_ml[w][1][r] * f;
    acc += *reinterpret_cast<const f32x4*>(&sm_o[w][wave][lane][0]) * f;
  }
  const int dt = wave;                                // dims dt*16 + g*4 + i, query r
  if (S == 1) {
    if (r < R) {
      const float inv = 1.0f / L;
      store_out4(a, row0 + r, h * 64 + dt * 16 + g * 4, float4{acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv});
    }
    return;
  }
  // split keys: publish this workgroup's partial, the last one to arrive merges all S
  const size_t unit = (size_t)(b * a.H + h) * QT + qt;          // (sequence, head, query tile)
  float* part = a.part + (unit * S + s) * kPartFloats;
  if (wave == 0 && g == 0) { st_coherent(part + r, M); st_coherent(part + 16 + r, L); }
#pragma unroll
  for (int i = 0; i < 4; ++i) st_coherent(part + 32 + (dt * 16 + g * 4 + i) * 16 + r, acc[i]);
  __builtin_amdgcn_s_waitcnt(0);                      // partial is complete in memory
  __syncthreads();
  if (tid == 0) {
    uint32_t* tk = a.tickets + unit;
    const uint32_t old = __hip_atomic_fetch_add(tk, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm_last = old == (uint32_t)(S - 1);
    if (sm_last) __hip_atomic_store(tk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!sm_last) return;
  const float* p0 = a.part + unit * S * kPartFloats;
  float Mg = -INFINITY;
  for (int k = 0; k < S; ++k) Mg = fmaxf(Mg, ld_coherent(p0 + (size_t)k * kPartFloats + r));
  float Lg = 0.f;
  f32x4 og = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < S; ++k) {
    const float* pk = p0 + (size_t)k * kPartFloats;
    const float mk = ld_coherent(pk + r);
    const float f = mk == -INFINITY ? 0.f : exp2f(mk - Mg);
    Lg += ld_coherent(pk + 16 + r) * f;
#pragma unroll
    for (int i = 0; i < 4; ++i) og[i] += ld_coherent(pk + 32 + (dt * 16 + g * 4 + i) * 16 + r) * f;
  }
  if (r < R) {
    const float inv = 1.0f / Lg;
    store_out4(a, row0 + r, h * 64 + dt * 16 + g * 4, float4{og[0] * inv, og[1] * inv, og[2] * inv, og[3] * inv});
  }
}

// ---------------------------------------------------------------------------
// Prefill passes (more than 16 query rows per sequence): a workgroup takes 64 query rows of one
// (sequence, head), one 16-row tile per wavefront, and all four wavefronts walk the keys together,
// so a chunk of keys and values is fetched once per 64 rows instead of once per 16.  The chunk
// goes from L2 / HBM straight into LDS (LDS-direct loads; lane l's 16 bytes of a request land at
// base + 16 l, so the LDS image is already in fragment order and is read back conflict-free), double
// buffered, one barrier per chunk; each wavefront stops computing at its own causal limit.  No key
// split: a pass of C rows has C/128 x H workgroups per sequence, each taking an early and a late block.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void lds_direct16(const void* gptr, void* lds) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds, 16, 0, 0);
}

__global__ __launch_bounds__(256) void k_pattn(const FastAttn a) {
  __shared__ __align__(16) unsigned char kv[2][16384];    // per buffer: 8 key fragments, 8 value fragments (1 KB each)
  const int h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int nseq = a.eff_len[b];
  const bool fixed = a.fixed_limit > 0;
  const size_t head = (size_t)a.slot[b] * a.H + h;
  const uint16_t* kb = a.Kc + head * (size_t)a.cap * 64;
  const uint16_t* vb = a.Vt + head * 64 * (size_t)a.cap;
  // wavefront w requests key tile w and value tile w of a chunk (the same addresses k_fattn loads)
  auto request = [&](int c) {
    const int key0 = c << 6;
    unsigned char* dst = kv[c & 1];
    const uint16_t* kr = kb + (size_t)(key0 + (r >> 2) * 16 + wave * 4 + (r & 3)) * 64 + g * 8;
    lds_direct16(kr, dst + (wave * 2) * 1024);
    lds_direct16(kr + 32, dst + (wave * 2 + 1) * 1024);
    const uint16_t* vr = vb + (size_t)(wave * 16 + r) * a.cap + key0 + g * 16;
    lds_direct16(vr, dst + 8192 + (wave * 2) * 1024);
    lds_direct16(vr + 8, dst + 8192 + (wave * 2 + 1) * 1024);
  };
  // a workgroup takes 64-row block x and then block NQ - 1 - x: under the causal mask the later a
  // block, the more keys it walks, and the two together walk the same number for every workgroup
  const int NQ = (a.R + 63) >> 6;
  for (int pass = 0; pass < 2; ++pass) {
    const int qb = pass == 0 ? (int)blockIdx.x : NQ - 1 - (int)blockIdx.x;
    if (pass == 1 && qb == (int)blockIdx.x) break;
    const int rows_end = min(a.R, (qb + 1) * 64);          // rows of the sequence up to the end of this block
    if (nseq < 0) {                                        // skipped sequence: defined (zero) output
      for (int i = tid; i < (rows_end - qb * 64) * 16; i += 256)
        store_out4(a, b * a.R + qb * 64 + i / 16, h * 64 + (i & 15) * 4, float4{0.f, 0.f, 0.f, 0.f});
      continue;
    }
    const int qt = qb * 4 + wave;                          // this wavefront's query tile
    const int R = max(0, min(16, a.R - qt * 16));          // its rows (0: none, it only helps fetching)
    const int row0 = b * a.R + qt * 16;
    const int n = nseq + qt * 16;                          // keys every query of the tile sees
    const int Ltot = fixed ? a.fixed_limit : n + R;
    const int lim = r < R ? (fixed ? Ltot : n + r + 1) : 0;
    const int first_masked = fixed ? Ltot : n + 1;
    const int NC = ((fixed ? a.fixed_limit : nseq + rows_end) + 63) >> 6;   // chunks the block walks
    const int NCw = R > 0 ? (Ltot + 63) >> 6 : 0;                           // chunks this wavefront uses

    bf16x8 qh[2], ql[2];
    load_queries(a, qh, ql, r < R ? a.Q + (size_t)(row0 + r) * a.ldq + h * 64 : nullptr, g);
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    request(0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int c = 0; c < NC; ++c) {
      uint4 kf[4][2], vf[4][2];
      if (c < NCw) {
        const unsigned char* src = kv[c & 1] + lane * 16;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            kf[t][j] = *reinterpret_cast<const uint4*>(src + (t * 2 + j) * 1024);
            vf[t][j] = *reinterpret_cast<const uint4*>(src + 8192 + (t * 2 + j) * 1024);
          }
      }
      // the other buffer was last read one iteration ago, before the barrier every wavefront passed
      if (c + 1 < NC) request(c + 1);
      if (c < NCw) attn_chunk(kf, vf, qh, ql, c << 6, g, r < R, lim, first_masked, Ltot, a.scale_log2, m_run, l_run, o);
      __builtin_amdgcn_s_waitcnt(0);                 // this wavefront's part of the next chunk has landed
      __syncthreads();                               // ... and everybody's; everybody has read this one
    }
    if (r < R) {
      const float inv = 1.0f / l_run;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
        store_out4(a, row0 + r, h * 64 + dt * 16 + g * 4,
                   float4{o[dt][0] * inv, o[dt][1] * inv, o[dt][2] * inv, o[dt][3] * inv});
    }
  }
}

void launch_fattn(const FastAttn& a, int n_seq, hipStream_t s) {
  TraceScope trace_("fattn", s);
  if (a.R > 16) {                                    // prefill pass
    hipLaunchKernelGGL(k_pattn, dim3(((a.R + 63) / 64 + 1) / 2, a.H, n_seq), dim3(256), 0, s, a);
    return;
  }
  hipLaunchKernelGGL(k_fattn, dim3(a.S * ((a.R + 15) / 16), a.H, n_seq), dim3(256), 0, s, a);
}

size_t fattn_part_bytes(size_t entries) { return entries * kPartFloats * sizeof(float); }

}  // namespace xsm
