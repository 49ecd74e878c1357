// C ABI of libxsm: context, buffer layout, weight upload, prefill, speculative
// and plain decoding steps.  All device work is enqueued on the caller's
// stream; nothing here allocates device memory.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "xsm_internal.h"

using namespace xsm;

namespace {

thread_local std::string g_create_err;

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

int fail(xsm_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_err = msg;
  return code;
}

#define XSM_HIP(call)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (call);                                                             \
    if (e_ != hipSuccess)                                                               \
      return fail(ctx, XSM_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));    \
  } while (0)

void build_weight_offsets(xsm_ctx* c) {
  const xsm_config& g = c->cfg;
  const size_t d = g.d_model, F = g.d_ffn, V = g.vocab;
  WeightOff& o = c->woff;
  size_t p = 0;
  auto take = [&](size_t n) { size_t r = p; p += n; return r; };
  o.E = take(V * d);
  o.layer.resize(g.n_layers);
  for (int l = 0; l < g.n_layers; ++l) {
    LayerOff& L = o.layer[l];
    L.g1 = take(d); L.Wqkv = take(3 * d * d); L.Wo = take(d * d);
    if (g.n_cond > 0) { L.gc = take(d); L.Wcq = take(d * d); L.Wckv = take(2 * d * d); L.Wco = take(d * d); }
    else { L.gc = L.Wcq = L.Wckv = L.Wco = 0; }
    L.g2 = take(d); L.W1 = take(F * d); L.W2 = take(d * F);
  }
  o.gf = take(d); o.WU = take(V * d);
  o.hW.resize(g.n_draft); o.hb.resize(g.n_draft);
  o.hq.resize(g.n_draft); o.hkv.resize(g.n_draft); o.ho.resize(g.n_draft); o.hU.resize(g.n_draft);
  for (int k = 0; k < g.n_draft; ++k) {
    if (g.head_kind == XSM_HEAD_CA) { o.hq[k] = take(d * d); o.hkv[k] = take(2 * d * d); o.ho[k] = take(d * d); o.hU[k] = take(V * d); }
    else { o.hW[k] = take(d * d); o.hb[k] = take(d); }
  }
  o.total = p;
}

// Layout of a workspace.  step_only: sized for decoding steps alone (max_batch x 16 rows, no
// prefill passes, no exchange buffers of the single-launch step) - the layout of the static
// scratch array.
void build_work_offsets(const xsm_ctx* c, bool step_only, WorkOff& w, size_t& rows_max, size_t& part_entries,
                        size_t& n_tickets) {
  const xsm_config& g = c->cfg;
  const size_t d = g.d_model, F = g.d_ffn, V = g.vocab, K = g.n_draft;
  size_t Mmax = (size_t)g.max_batch * kMaxRows;           // rows of one backbone pass
  if (c->fast && !step_only && Mmax < (size_t)kFastPassRows) Mmax = kFastPassRows;   // prefill chunks of few sequences
  rows_max = Mmax;
  const size_t Mb = (size_t)g.max_batch * (K + 1);        // rows of one step
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t r = p; p = align_up(p + bytes); return r; };
  w.X = take(Mmax * d * 4); w.QKV = take(Mmax * 3 * d * 4);
  w.Xn = take(((Mmax + 15) & ~(size_t)15) * d * 4);       // (as bf16 hi / lo planes it covers whole 16-row tiles)
  const size_t Mpad = (Mmax + 15) & ~(size_t)15;          // (AO and U may hold operand planes: whole 16-row tiles)
  w.Qr = take(Mmax * d * 4); w.AO = take(Mpad * d * 4); w.U = take(Mpad * F * 4);
  w.Z0 = take(Mb * V * 4);
  w.G = take((size_t)g.max_batch * d * 4);
  w.Hh = take((size_t)g.max_batch * (K ? K : 1) * d * 4);
  w.Rk = take((size_t)g.max_batch * (K ? K : 1) * d * 4);
  w.Zh = take((size_t)g.max_batch * (K ? K : 1) * V * 4);
  w.eff_len = take(g.max_batch * 4); w.slot = take(g.max_batch * 4); w.acc = take(g.max_batch * 4);
  w.y0 = take(g.max_batch * 4); w.wflags = take(g.max_batch * 4);
  w.toks = take((size_t)g.max_batch * kMaxRows * 4);
  w.rowidx = take(g.max_batch * 4);
  w.eff2 = take((size_t)g.max_batch * (K ? K : 1) * 4); w.slot2 = take((size_t)g.max_batch * (K ? K : 1) * 4);
  // (sequence, head) pairs of one attention call: the backbone's, or all cross-attention decoding heads at once
  size_t attn_pairs = (size_t)g.max_batch * g.n_heads * (g.head_kind == XSM_HEAD_CA && K ? K : 1);
  if (attn_pairs < Mmax / 16 * g.n_heads) attn_pairs = Mmax / 16 * g.n_heads;   // (sequence, head, query tile) units
  part_entries = attn_pairs < 1024 ? 1024 : attn_pairs;
  n_tickets = attn_pairs;
  w.part = take(fattn_part_bytes(part_entries));
  w.tickets = take(attn_pairs * 4);
  w.gpart = w.gtickets = 0;
  if (c->fast) {
    // partial products of the split-contraction GEMM, for the largest projection it may run
    const int shapes[6][2] = {{(int)(3 * d), (int)d}, {(int)d, (int)d}, {(int)F, (int)d}, {(int)d, (int)F},
                              {(int)V, (int)d}, {(int)((K ? K : 1) * d), (int)d}};
    size_t fl = 0;
    for (auto& sh : shapes) {
      const size_t need = ws_gemm_part_floats((int)(Mmax > Mb ? Mmax : Mb), sh[0], sh[1]);
      if (need > fl) fl = need;
    }
    // the residual-add projections in slices on the row-blocked kernel (a few hundred rows)
    const size_t need_dn = blk_add_part_floats((int)Mmax, (int)d, (int)F), need_o = blk_add_part_floats((int)Mmax, (int)d, (int)d);
    if (need_dn > fl) fl = need_dn;
    if (need_o > fl) fl = need_o;
    w.gpart = take(fl * 4);
    w.gtickets = take(kWsTickets * 4);
  }
  w.ll = w.ctrl = w.head_all = w.tlog = 0;
  if (c->small_ok && !step_only) {
    w.ll = take(small_ll_words(g.n_layers, g.d_model, g.d_ffn, g.n_draft) * 4);
    w.ctrl = take(kSmallCtrlBytes);
    w.head_all = take((size_t)kSmallMaxRows * V * 4);
    w.tlog = take((size_t)256 * (g.n_layers * 16 + 8) * 8);
  }
  w.total = p;
}

// ---- the scratch of the step entry point that allocates nothing ------------------------------
// One array per GPU, held from the time the library is loaded until the process ends; every
// xsm_spec_step_static call on that GPU works in it, whatever its context.  In host code the
// array's name is only a handle: its device address is looked up once per device (xsm_bind, with
// that device current) and kernels, fills and copies are given the looked-up pointer.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on first use, then kept)
int static_scratch_lookup(xsm_ctx* ctx, int* dev_out, char** ptr_out) {
  int dev = 0;
  XSM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(ctx, XSM_EINVAL, "device index beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    XSM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(ctx, XSM_EHIP, "hipGetSymbolAddress returned a null address for the static scratch");
    g_scratch_ptr[dev] = (char*)p;
  }
  *dev_out = dev;
  *ptr_out = g_scratch_ptr[dev];
  return XSM_OK;
}

// Fragment-ordered copies of the bf16 matrices, placed after the rotary table.
size_t build_tiled_offsets(xsm_ctx* c, size_t start) {
  const xsm_config& g = c->cfg;
  const size_t d = g.d_model, F = g.d_ffn, V = g.vocab, K = g.n_draft;
  size_t p = start;
  auto take = [&](size_t elems) { size_t r = p; p = align_up(p + elems * 2); return r; };
  TiledOff& t = c->toff;
  t.layer.resize(g.n_layers);
  for (int l = 0; l < g.n_layers; ++l) {
    TiledLayer& L = t.layer[l];
    L.Wqkv = take(3 * d * d); L.Wo = take(d * d);
    if (g.n_cond > 0) { L.Wcq = take(d * d); L.Wckv = take(2 * d * d); L.Wco = take(d * d); } else { L.Wcq = L.Wckv = L.Wco = 0; }
    L.W1 = take(F * d); L.W2 = take(d * F);
  }
  t.WU = take(V * d);
  t.Wh = take((K ? K : 1) * d * d);
  t.hb = take((K ? K : 1) * d);
  t.Who.assign(K, 0); t.WhU.assign(K, 0); t.Whkv.assign(K, 0);
  if (g.head_kind == XSM_HEAD_CA)
    for (size_t k = 0; k < K; ++k) { t.Who[k] = take(d * d); t.WhU[k] = take(V * d); t.Whkv[k] = take(2 * d * d); }
  return p;
}

struct LayerPtrs {
  const char *g1, *Wqkv, *Wo, *gc, *Wcq, *Wckv, *Wco, *g2, *W1, *W2;
};
LayerPtrs layer_ptrs(const xsm_ctx* c, int l) {
  const LayerOff& L = c->woff.layer[l];
  const char* b = c->d_w;
  const size_t e = c->esz;
  return {b + L.g1 * e, b + L.Wqkv * e, b + L.Wo * e, b + L.gc * e, b + L.Wcq * e, b + L.Wckv * e,
          b + L.Wco * e, b + L.g2 * e, b + L.W1 * e, b + L.W2 * e};
}

// cache addressing: self cache [L][2][max_batch][H][max_ctx][hd], then cross cache
// [L][2][max_batch][H][n_cond][hd]
char* self_cache(const xsm_ctx* c, int layer, int which) {
  const xsm_config& g = c->cfg;
  const size_t per = (size_t)g.max_batch * g.n_heads * c->cap_self * g.head_dim;
  return c->d_kv + ((size_t)layer * 2 + which) * per * c->esz;
}
char* cross_cache(const xsm_ctx* c, int layer, int which) {
  const xsm_config& g = c->cfg;
  const size_t per = (size_t)g.max_batch * g.n_heads * c->cap_cross * g.head_dim;
  return c->d_kv + (c->kv_self_elems + ((size_t)layer * 2 + which) * per) * c->esz;
}
// condition cache of the cross-attention decoding heads: [2][K][max_batch][H][n_cond][hd], so that
// (head k, slot s) is "slot" k*max_batch + s of one attention call over all heads
char* head_cache(const xsm_ctx* c, int k, int which) {
  const xsm_config& g = c->cfg;
  const size_t per = (size_t)g.max_batch * g.n_heads * c->cap_cross * g.head_dim;
  return c->d_kv + (c->kv_self_elems + c->kv_cross_elems + ((size_t)which * g.n_draft + k) * per) * c->esz;
}

// Key-range slices per (sequence, head, query tile).  A workgroup streams chunks/S 64-key chunks
// plus a fixed start-up and merge cost (about 8 chunks' worth), and the BH*S workgroups run in
// ceil(BH*S / 256) rounds over the compute units: take the S that minimises rounds x per-workgroup
// time (whole rounds matter: 384 workgroups on 256 compute units take as long as 512), at least
// 4 chunks per workgroup, bounded by the partial slots in the workspace.
int attn_splits(const xsm_ctx* c, int n_units, int len_bound) {
  const int BH = n_units * c->cfg.n_heads;           // n_units: sequences x query tiles
  const int chunks = (len_bound + 63) / 64;
  if (c->force_splits > 0) {
    int S = c->force_splits;
    if (S > chunks / 4) S = chunks / 4;
    if ((size_t)S * BH > c->part_entries) S = (int)(c->part_entries / BH);
    return S < 1 ? 1 : S;
  }
  int best = 1;
  double best_cost = 0;
  for (int S = 1; S <= 16; ++S) {
    if (S > 1 && (S > chunks / 4 || (size_t)S * BH > c->part_entries)) break;
    const double cost = (double)((BH * S + 255) / 256) * ((double)chunks / S + 8.0);
    if (S == 1 || cost < best_cost * 0.999) { best = S; best_cost = cost; }
  }
  return best;
}

// A projection on the MFMA path; a (prologue, epilogue) pair no kernel takes is remembered and
// reported by the entry point (nothing is enqueued for it, so its output would be stale).
void fgemm(xsm_ctx* c, int pro, int epi, const FastGemm& g, hipStream_t s) {
  if (!launch_fgemm(pro, epi, g, s)) c->gemm_unmatched = true;
}
int unmatched_gemm(xsm_ctx* c) {
  if (!c->gemm_unmatched) return XSM_OK;
  c->gemm_unmatched = false;
  return fail(c, XSM_EINVAL, "internal: a projection found no kernel for its prologue / epilogue at this shape");
}

// MFMA path: all decoder blocks over M = n_seq*R rows held in ws.X (fp32 residual stream).
void forward_blocks_fast(xsm_ctx* c, int n_seq, int R, int len_bound, hipStream_t s) {
  const xsm_config& g = c->cfg;
  const int d = g.d_model, F = g.d_ffn, H = g.n_heads, hd = g.head_dim;
  const int M = n_seq * R;
  char* ws = c->d_ws;
  float* X = (float*)(ws + c->ws.X);
  float* Xn = (float*)(ws + c->ws.Xn);            // normalised rows for the GEMMs that do not fuse the norm
  float* gpart = (float*)(ws + c->ws.gpart);
  uint32_t* gtick = (uint32_t*)(ws + c->ws.gtickets);
  PendingAdd* const PEND = &c->pend;
  float* Qr = (float*)(ws + c->ws.Qr);
  float* AO = (float*)(ws + c->ws.AO);
  float* U = (float*)(ws + c->ws.U);
  const int32_t* eff = (const int32_t*)(ws + c->ws.eff_len);
  const int32_t* slot = (const int32_t*)(ws + c->ws.slot);
  const float2* rope = (const float2*)(c->d_w + c->rope_off);
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)hd);
  // The row-blocked kernel reads its input as bf16 hi/lo operand planes.  When the residual-add
  // projections (d output columns) have enough 64 x 128 blocks to fill the chip, attention and the
  // FFN-up epilogue write such planes directly and those projections run on it too (no fp32 round
  // trip, no conversion in the GEMM): 8 % on a 2048-row prefill pass; with fewer blocks (1152 rows
  // at d = 1024: 144) the kernel with smaller blocks that converts fp32 rows on the way in is faster.
  const bool planes = fgemm_planes_ok(M, d, d) && fgemm_planes_ok(M, d, F) && fgemm_planes_ok(M, F, d) &&
                      (d / 64) * ((M + 127) / 128) >= 256;
  // With fewer rows they still run there when their contraction can be cut into slices that give
  // the chip enough blocks (the sum is left to the next RMSNorm pass): FFN-down into up to 8
  // slices (75 -> 37 us at 1152 rows), the O-projections into 2 (22 -> 19 us).
  const bool o_planes = planes || blk_add_split(M, d, d) > 1;
  const bool dn_planes = planes || (fgemm_planes_ok(M, F, d) && blk_add_split(M, d, F) > 1);
  for (int l = 0; l < g.n_layers; ++l) {
    const LayerPtrs P = layer_ptrs(c, l);
    const TiledLayer& T = c->toff.layer[l];
    FastGemm q{};
    q.Wt = (const uint4*)(c->d_w + T.Wqkv); q.N = 3 * d; q.K = d; q.M = M;
    q.X = X; q.ldx = d; q.gain = (const uint16_t*)P.g1; q.eps = g.rms_eps;
    q.Y = Qr; q.ldy = d; q.nscratch = Xn; q.ws_part = gpart; q.ws_tickets = gtick; q.pend = PEND;
    q.rope = rope; q.eff_len = eff; q.slot = slot; q.R = R; q.H = H; q.hd = hd; q.cap = c->cap_self;
    q.v_transposed = 1; q.Kc = (uint16_t*)self_cache(c, l, 0); q.Vc = (uint16_t*)self_cache(c, l, 1);
    fgemm(c, PRO_NORM, FEPI_QKV, q, s);

    FastAttn a{};
    a.Q = Qr; a.ldq = d; a.Kc = (const uint16_t*)self_cache(c, l, 0); a.Vt = (const uint16_t*)self_cache(c, l, 1);
    a.eff_len = eff; a.slot = slot; a.O = AO; a.ldo = d;
    a.part = (float*)(ws + c->ws.part); a.tickets = (uint32_t*)(ws + c->ws.tickets);
    a.R = R; a.H = H; a.cap = c->cap_self; a.S = attn_splits(c, n_seq * ((R + 15) / 16), len_bound + R); a.fixed_limit = 0;
    a.scale_log2 = scale_log2; a.o_planes = o_planes ? 1 : 0; a.o_rows = M;
    launch_fattn(a, n_seq, s);

    FastGemm o{};
    o.Wt = (const uint4*)(c->d_w + T.Wo); o.N = d; o.K = d; o.M = M;
    o.X = AO; o.ldx = d; o.Y = X; o.ldy = d; o.nscratch = Xn; o.ws_part = gpart; o.ws_tickets = gtick; o.pend = PEND;
    fgemm(c, o_planes ? PRO_PLANES : PRO_F32, FEPI_ADD, o, s);

    if (g.n_cond > 0) {
      FastGemm cq{};
      cq.Wt = (const uint4*)(c->d_w + T.Wcq); cq.N = d; cq.K = d; cq.M = M;
      cq.X = X; cq.ldx = d; cq.gain = (const uint16_t*)P.gc; cq.eps = g.rms_eps;
      cq.Y = Qr; cq.ldy = d; cq.nscratch = Xn; cq.ws_part = gpart; cq.ws_tickets = gtick; cq.pend = PEND;
      fgemm(c, PRO_NORM, FEPI_STORE, cq, s);
      FastAttn ca = a;
      ca.Kc = (const uint16_t*)cross_cache(c, l, 0); ca.Vt = (const uint16_t*)cross_cache(c, l, 1);
      ca.cap = c->cap_cross; ca.fixed_limit = g.n_cond; ca.S = attn_splits(c, n_seq * ((R + 15) / 16), g.n_cond);
      launch_fattn(ca, n_seq, s);
      FastGemm co = o;
      co.Wt = (const uint4*)(c->d_w + T.Wco);
      fgemm(c, o_planes ? PRO_PLANES : PRO_F32, FEPI_ADD, co, s);
    }

    FastGemm u{};
    u.Wt = (const uint4*)(c->d_w + T.W1); u.N = F; u.K = d; u.M = M;
    u.X = X; u.ldx = d; u.gain = (const uint16_t*)P.g2; u.eps = g.rms_eps;
    u.Y = U; u.ldy = F; u.nscratch = Xn; u.ws_part = gpart; u.ws_tickets = gtick; u.pend = PEND;
    u.y_planes = dn_planes ? 1 : 0;
    fgemm(c, PRO_NORM, FEPI_GELU, u, s);

    FastGemm dn{};
    dn.Wt = (const uint4*)(c->d_w + T.W2); dn.N = d; dn.K = F; dn.M = M;
    dn.X = U; dn.ldx = F; dn.Y = X; dn.ldy = d; dn.nscratch = Xn; dn.ws_part = gpart; dn.ws_tickets = gtick; dn.pend = PEND;
    fgemm(c, dn_planes ? PRO_PLANES : PRO_F32, FEPI_ADD, dn, s);
  }
  flush_pending_add(PEND, s);                     // the residual rows are read by the caller next
}

// All decoder blocks over M = n_seq*R rows held in ws.X; row m = b*R + j sits at position
// eff_len[b] + j.  Leaves the final residual stream in ws.X.
void forward_blocks(xsm_ctx* c, int n_seq, int R, int len_bound, hipStream_t s) {
  if (c->fast) { forward_blocks_fast(c, n_seq, R, len_bound, s); return; }
  const xsm_config& g = c->cfg;
  const int d = g.d_model, F = g.d_ffn, H = g.n_heads, hd = g.head_dim, dt = g.dtype;
  const int M = n_seq * R;
  char* ws = c->d_ws;
  float* X = (float*)(ws + c->ws.X);
  float* Xn = (float*)(ws + c->ws.Xn);
  float* QKV = (float*)(ws + c->ws.QKV);
  float* Qr = (float*)(ws + c->ws.Qr);
  float* AO = (float*)(ws + c->ws.AO);
  float* U = (float*)(ws + c->ws.U);
  const int32_t* eff = (const int32_t*)(ws + c->ws.eff_len);
  const int32_t* slot = (const int32_t*)(ws + c->ws.slot);
  const float2* rope = (const float2*)(c->d_w + c->rope_off);
  for (int l = 0; l < g.n_layers; ++l) {
    const LayerPtrs P = layer_ptrs(c, l);
    launch_rmsnorm(dt, X, P.g1, Xn, M, d, g.rms_eps, s);
    launch_gemm(dt, EPI_STORE, Xn, d, P.Wqkv, QKV, 3 * d, M, 3 * d, d, s);
    launch_rope_kv(dt, QKV, rope, eff, slot, Qr, self_cache(c, l, 0), self_cache(c, l, 1), n_seq, R,
                   H, hd, c->cap_self, s);
    launch_attention(dt, Qr, self_cache(c, l, 0), self_cache(c, l, 1), eff, slot, AO, n_seq, R, H,
                     hd, c->cap_self, 0, s);
    launch_gemm(dt, EPI_ADD, AO, d, P.Wo, X, d, M, d, d, s);
    if (g.n_cond > 0) {
      launch_rmsnorm(dt, X, P.gc, Xn, M, d, g.rms_eps, s);
      launch_gemm(dt, EPI_STORE, Xn, d, P.Wcq, Qr, d, M, d, d, s);
      launch_attention(dt, Qr, cross_cache(c, l, 0), cross_cache(c, l, 1), eff, slot, AO, n_seq, R,
                       H, hd, c->cap_cross, g.n_cond, s);
      launch_gemm(dt, EPI_ADD, AO, d, P.Wco, X, d, M, d, d, s);
    }
    launch_rmsnorm(dt, X, P.g2, Xn, M, d, g.rms_eps, s);
    launch_gemm(dt, EPI_GELU, Xn, d, P.W1, U, F, M, F, d, s);
    launch_gemm(dt, EPI_ADD, U, F, P.W2, X, d, M, d, F, s);
  }
}

int check_ready(xsm_ctx* ctx) {
  if (!ctx) return XSM_EINVAL;
  if (!ctx->d_w || !ctx->d_kv || !ctx->d_ws) return fail(ctx, XSM_ESTATE, "buffers not bound");
  if (!ctx->loaded) return fail(ctx, XSM_ESTATE, "weights not loaded");
  return XSM_OK;
}

int step_common(xsm_ctx* ctx, const xsm_batch* bt, const xsm_verify_params* vp, xsm_stream stream,
                int R) {
  int rc = check_ready(ctx);
  if (rc) return rc;
  if (!bt || !vp) return fail(ctx, XSM_EINVAL, "null batch or verify params");
  const xsm_config& g = ctx->cfg;
  if (bt->n_seq < 1) return fail(ctx, XSM_EINVAL, "n_seq < 1");
  if (bt->n_seq > g.max_batch) return fail(ctx, XSM_ECAPACITY, "n_seq > max_batch");
  if (!bt->slot || !bt->kv_len || !bt->block || !bt->out_tokens || !bt->n_accepted || !bt->flags)
    return fail(ctx, XSM_EINVAL, "null batch array");
  if (bt->kv_len_bound < 0) return fail(ctx, XSM_EINVAL, "kv_len_bound < 0");
  if ((long)bt->kv_len_bound + R > g.max_ctx)
    return fail(ctx, XSM_ECAPACITY, "kv_len_bound + rows per step exceeds max_ctx");
  if (vp->mode < 0 || vp->mode > 2) return fail(ctx, XSM_EINVAL, "bad verify mode");
  if (vp->mode == XSM_VERIFY_TOPK && vp->top_ka < 1) return fail(ctx, XSM_EINVAL, "top_ka < 1");
  if ((vp->sample == 1 || vp->mode == XSM_VERIFY_THRESHOLD) && !(vp->temperature > 0.f))
    return fail(ctx, XSM_EINVAL, "temperature must be > 0");
  if (vp->sample < 0 || vp->sample > 2) return fail(ctx, XSM_EINVAL, "bad sample rule");
  if (vp->sample == 2) {
    if (!(vp->temperature > 0.f)) return fail(ctx, XSM_EINVAL, "temperature must be > 0");
    if (vp->top_ks < 1 || vp->top_ks > 4) return fail(ctx, XSM_EINVAL, "top_ks must be in [1, 4]");
    long paths = 1;
    for (int k = 0; k < R - 1; ++k) paths *= vp->top_ks;
    if (paths > 4096) return fail(ctx, XSM_EINVAL, "probability tree too large (top_ks^K > 4096)");
    if (!(vp->pts_prune >= 0.f)) return fail(ctx, XSM_EINVAL, "pts_prune must be >= 0");
  }

  hipStream_t s = (hipStream_t)stream;
  const int n_seq = bt->n_seq, K = R - 1, d = g.d_model, V = g.vocab, dt = g.dtype;
  const int M = n_seq * R;
  char* ws = ctx->d_ws;
  float* X = (float*)(ws + ctx->ws.X);
  float* Xn = (float*)(ws + ctx->ws.Xn);
  float* Z0 = (float*)(ws + ctx->ws.Z0);
  float* gpart = (float*)(ws + ctx->ws.gpart);
  uint32_t* gtick = (uint32_t*)(ws + ctx->ws.gtickets);
  PendingAdd* const PEND = &ctx->pend;
  float* G = (float*)(ws + ctx->ws.G);
  float* Hh = (float*)(ws + ctx->ws.Hh);
  float* Rk = (float*)(ws + ctx->ws.Rk);
  float* Zh = (float*)(ws + ctx->ws.Zh);
  int32_t* eff = (int32_t*)(ws + ctx->ws.eff_len);
  int32_t* slot = (int32_t*)(ws + ctx->ws.slot);
  int32_t* acc = (int32_t*)(ws + ctx->ws.acc);
  int32_t* y0 = (int32_t*)(ws + ctx->ws.y0);
  uint32_t* wfl = (uint32_t*)(ws + ctx->ws.wflags);
  const char* wb = ctx->d_w;
  const size_t e = ctx->esz;

  if (ctx->small_ok && ctx->small_dev && ctx->use_small && !ctx->small_failed && M <= 16 && M + M * K <= kSmallMaxRows && n_seq * g.n_heads <= 256) {
    // the whole step as one persistent kernel.  Greedy verification with argmax draws works from
    // per-tile top-2 statistics; the other criteria and sampling rules make the kernel write the
    // logits rows (into the workspace) and its last stage read them back
    const bool full = !(vp->mode == XSM_VERIFY_GREEDY && vp->sample == 0);
    SmallArgs a{};
    a.full_verify = full ? 1 : 0;
    a.vp = *vp;
    a.layers = (const LayerTab*)(wb + ctx->layer_tab_off); a.L = g.n_layers;
    a.E = (const uint16_t*)(wb + ctx->woff.E * e); a.gf = (const uint16_t*)(wb + ctx->woff.gf * e);
    a.hb = (const uint16_t*)(wb + ctx->toff.hb);
    a.WU = (const uint4*)(wb + ctx->toff.WU); a.Wh = (const uint4*)(wb + ctx->toff.Wh);
    a.rope = (const float2*)(wb + ctx->rope_off);
    a.ll = (uint32_t*)(ws + ctx->ws.ll); a.ll_layer_stride = small_ll_layer_stride(d, g.d_ffn);
    a.ll_words = small_ll_words(g.n_layers, d, g.d_ffn, K);
    a.ctrl = (uint32_t*)(ws + ctx->ws.ctrl);
    a.slot = bt->slot; a.kv_len = bt->kv_len; a.block = bt->block; a.out_tokens = bt->out_tokens;
    a.n_accepted = bt->n_accepted; a.flags = bt->flags;
    a.logits_dbg = full ? Z0 : bt->logits_dbg;
    a.head_logits_dbg = full ? Zh : bt->head_logits_dbg;       // non-null: keep the head logits of every row
    a.head_all_dbg = (float*)(ws + ctx->ws.head_all); a.acc_out = acc;
    a.tlog = ctx->timeline ? (uint64_t*)(ws + ctx->ws.tlog) : nullptr;
    a.n_seq = n_seq; a.R = R; a.V = V; a.max_batch = g.max_batch; a.max_ctx = g.max_ctx;
    a.bound = bt->kv_len_bound; a.cap = ctx->cap_self;
    a.eps = g.rms_eps; a.scale_log2 = 1.4426950408889634f / sqrtf((float)g.head_dim);
    // upper limit of the key slices per (sequence, head): S * n_seq * H <= 256 workgroups; the kernel
    // picks the count from the cache lengths it reads (a forced count is taken as it is)
    int S = 1;
    const int want = ctx->force_splits > 0 ? ctx->force_splits : 16;
    while (S * 2 <= want && S < 16 && 2 * S * n_seq * g.n_heads <= 256) S *= 2;
    a.s_auto = ctx->force_splits > 0 ? 0 : 1;
    a.S = S;
    launch_step_small(a, d, g.d_ffn, s);
    if (full && bt->logits_dbg) launch_copy_f32(Z0, bt->logits_dbg, (size_t)M * V, s);
    if (bt->head_logits_dbg && K > 0) launch_gather_head_dbg(a.head_all_dbg, acc, bt->head_logits_dbg, n_seq, R, K, V, s);
    hipError_t e3 = hipGetLastError();
    if (e3 != hipSuccess) return fail(ctx, XSM_EHIP, std::string("launch: ") + hipGetErrorString(e3));
    return XSM_OK;
  }
  launch_prepare(bt->kv_len, bt->slot, bt->block, n_seq, R, V, g.max_batch, g.max_ctx,
                 bt->kv_len_bound, eff, slot, wfl, s);
  launch_embed(dt, wb + ctx->woff.E * e, bt->block, eff, X, n_seq, R, d, s);
  forward_blocks(ctx, n_seq, R, bt->kv_len_bound, s);
  if (ctx->fast) {
    // Eq. 3 logits straight from the residual stream: final RMSNorm is the GEMM prologue
    FastGemm z{};
    z.Wt = (const uint4*)(wb + ctx->toff.WU); z.N = V; z.K = d; z.M = M;
    z.X = X; z.ldx = d; z.gain = (const uint16_t*)(wb + ctx->woff.gf * e); z.eps = g.rms_eps;
    z.Y = Z0; z.ldy = V; z.nscratch = Xn; z.ws_part = gpart; z.ws_tickets = gtick; z.pend = PEND;
    fgemm(ctx, PRO_NORM, FEPI_STORE, z, s);
    if (bt->logits_dbg) launch_copy_f32(Z0, bt->logits_dbg, (size_t)M * V, s);
    launch_verify(Z0, nullptr, bt->block, eff, slot, *vp, acc, y0, wfl, nullptr, n_seq, R, V, d, s);
    if (K > 0 && g.head_kind == XSM_HEAD_CA) {
      // Eq. 4 with cross-attention heads, all heads of all sequences at once: q = Wq_k g (one
      // stacked GEMM), one attention call over the heads' cached condition keys/values with
      // (sequence, head) as the batch index, then per head the output projection onto the
      // residual g and the head's own unembedding.
      int32_t* rowidx = (int32_t*)(ws + ctx->ws.rowidx);
      int32_t* eff2 = (int32_t*)(ws + ctx->ws.eff2);
      int32_t* slot2 = (int32_t*)(ws + ctx->ws.slot2);
      float* Qh = Hh;                                        // [n_seq][K][d]
      float* Oh = (float*)(ws + ctx->ws.Qr);                 // [n_seq][K][d]
      launch_head_rows(acc, rowidx, n_seq, R, s);
      launch_norm_rows(X, d, rowidx, z.gain, g.rms_eps, G, n_seq, d, s);
      launch_head_ca_prep(G, Rk, eff, slot, eff2, slot2, n_seq, K, d, g.max_batch, s);
      FastGemm hq{};
      hq.Wt = (const uint4*)(wb + ctx->toff.Wh); hq.N = K * d; hq.K = d; hq.M = n_seq;
      hq.X = G; hq.ldx = d; hq.Y = Qh; hq.ldy = K * d;
      hq.nscratch = Xn; hq.ws_part = gpart; hq.ws_tickets = gtick; hq.pend = PEND;
      fgemm(ctx, PRO_F32, FEPI_STORE, hq, s);
      FastAttn ha{};
      ha.Q = Qh; ha.ldq = d; ha.Kc = (const uint16_t*)head_cache(ctx, 0, 0); ha.Vt = (const uint16_t*)head_cache(ctx, 0, 1);
      ha.eff_len = eff2; ha.slot = slot2; ha.O = Oh; ha.ldo = d;
      ha.part = (float*)(ws + ctx->ws.part); ha.tickets = (uint32_t*)(ws + ctx->ws.tickets);
      ha.R = 1; ha.H = g.n_heads; ha.cap = ctx->cap_cross; ha.S = attn_splits(ctx, n_seq * K, g.n_cond);
      ha.fixed_limit = g.n_cond; ha.scale_log2 = 1.4426950408889634f / sqrtf((float)g.head_dim);
      launch_fattn(ha, n_seq * K, s);
      for (int k = 0; k < K; ++k) {
        FastGemm ho{};
        ho.Wt = (const uint4*)(wb + ctx->toff.Who[k]); ho.N = d; ho.K = d; ho.M = n_seq;
        ho.X = Oh + (size_t)k * d; ho.ldx = K * d; ho.Y = Rk + (size_t)k * d; ho.ldy = K * d;
        ho.nscratch = Xn; ho.ws_part = gpart; ho.ws_tickets = gtick; ho.pend = nullptr;
        fgemm(ctx, PRO_F32, FEPI_ADD, ho, s);
        FastGemm zu{};
        zu.Wt = (const uint4*)(wb + ctx->toff.WhU[k]); zu.N = V; zu.K = d; zu.M = n_seq;
        zu.X = Rk + (size_t)k * d; zu.ldx = K * d; zu.Y = Zh + (size_t)k * V; zu.ldy = K * V;
        zu.nscratch = Xn; zu.ws_part = gpart; zu.ws_tickets = gtick; zu.pend = PEND;
        fgemm(ctx, PRO_F32, FEPI_STORE, zu, s);
      }
      if (bt->head_logits_dbg) launch_copy_f32(Zh, bt->head_logits_dbg, (size_t)n_seq * K * V, s);
    } else if (K > 0) {
      int32_t* rowidx = (int32_t*)(ws + ctx->ws.rowidx);
      launch_head_rows(acc, rowidx, n_seq, R, s);
      FastGemm hg{};                               // all K heads at once: [K*d][d] stacked
      hg.Wt = (const uint4*)(wb + ctx->toff.Wh); hg.N = K * d; hg.K = d; hg.M = n_seq;
      hg.X = X; hg.ldx = d; hg.gain = z.gain; hg.eps = g.rms_eps; hg.row_index = rowidx;
      hg.Y = Rk; hg.ldy = K * d; hg.bias = (const uint16_t*)(wb + ctx->toff.hb);
      hg.nscratch = Xn; hg.ws_part = gpart; hg.ws_tickets = gtick; hg.pend = PEND;
      fgemm(ctx, PRO_NORM, FEPI_HEAD, hg, s);
      FastGemm zh{};
      zh.Wt = z.Wt; zh.N = V; zh.K = d; zh.M = n_seq * K;
      zh.X = Rk; zh.ldx = d; zh.Y = Zh; zh.ldy = V; zh.nscratch = Xn; zh.ws_part = gpart; zh.ws_tickets = gtick; zh.pend = PEND;
      fgemm(ctx, PRO_F32, FEPI_STORE, zh, s);
      if (bt->head_logits_dbg) launch_copy_f32(Zh, bt->head_logits_dbg, (size_t)n_seq * K * V, s);
    }
  } else {
    launch_rmsnorm(dt, X, wb + ctx->woff.gf * e, Xn, M, d, g.rms_eps, s);            // Hf
    launch_gemm(dt, EPI_STORE, Xn, d, wb + ctx->woff.WU * e, Z0, V, M, V, d, s);      // Eq. 3 logits
    if (bt->logits_dbg) launch_copy_f32(Z0, bt->logits_dbg, (size_t)M * V, s);
    launch_verify(Z0, Xn, bt->block, eff, slot, *vp, acc, y0, wfl, K > 0 ? G : nullptr, n_seq, R, V,
                  d, s);
    if (K > 0 && g.head_kind == XSM_HEAD_CA) {
      int32_t* eff2 = (int32_t*)(ws + ctx->ws.eff2);
      int32_t* slot2 = (int32_t*)(ws + ctx->ws.slot2);
      float* Qh = Hh;
      float* Oh = (float*)(ws + ctx->ws.Qr);
      launch_head_ca_prep(G, Rk, eff, slot, eff2, slot2, n_seq, K, d, g.max_batch, s);
      for (int k = 0; k < K; ++k)
        launch_gemm(dt, EPI_STORE, G, d, wb + ctx->woff.hq[k] * e, Qh + (size_t)k * d, K * d, n_seq, d, d, s);
      launch_attention(dt, Qh, head_cache(ctx, 0, 0), head_cache(ctx, 0, 1), eff2, slot2, Oh, n_seq * K, 1,
                       g.n_heads, g.head_dim, ctx->cap_cross, g.n_cond, s);
      for (int k = 0; k < K; ++k) {
        launch_gemm(dt, EPI_ADD, Oh + (size_t)k * d, K * d, wb + ctx->woff.ho[k] * e, Rk + (size_t)k * d, K * d,
                    n_seq, d, d, s);
        launch_gemm(dt, EPI_STORE, Rk + (size_t)k * d, K * d, wb + ctx->woff.hU[k] * e, Zh + (size_t)k * V, K * V,
                    n_seq, V, d, s);
      }
      if (bt->head_logits_dbg) launch_copy_f32(Zh, bt->head_logits_dbg, (size_t)n_seq * K * V, s);
    } else if (K > 0) {
      const void* bias[16];
      for (int k = 0; k < K; ++k) {
        launch_gemm(dt, EPI_STORE, G, d, wb + ctx->woff.hW[k] * e, Hh + (size_t)k * d, K * d, n_seq, d,
                    d, s);
        bias[k] = wb + ctx->woff.hb[k] * e;
      }
      launch_head_act(dt, G, Hh, bias, Rk, n_seq, K, d, s);
      launch_gemm(dt, EPI_STORE, Rk, d, wb + ctx->woff.WU * e, Zh, V, n_seq * K, V, d, s);
      if (bt->head_logits_dbg) launch_copy_f32(Zh, bt->head_logits_dbg, (size_t)n_seq * K * V, s);
    }
  }
  launch_emit(Zh, *vp, eff, slot, acc, y0, wfl, (int32_t*)(ws + ctx->ws.toks), bt->block, bt->kv_len, bt->out_tokens,
              bt->n_accepted, bt->flags, n_seq, R, K, V, s);
  hipError_t e2 = hipGetLastError();
  if (e2 != hipSuccess) return fail(ctx, XSM_EHIP, std::string("launch: ") + hipGetErrorString(e2));
  return unmatched_gemm(ctx);
}

}  // namespace

extern "C" {

int xsm_create(const xsm_config* cfg, xsm_ctx** out) {
  if (!cfg || !out) return fail(nullptr, XSM_EINVAL, "null argument");
  const xsm_config& g = *cfg;
  auto bad = [&](const char* m) { return fail(nullptr, XSM_EINVAL, m); };
  if (g.n_layers < 1 || g.d_model < 8 || g.n_heads < 1 || g.d_ffn < 8 || g.vocab < 2)
    return bad("model dimensions out of range");
  if (g.n_heads * g.head_dim != g.d_model) return bad("n_heads * head_dim != d_model");
  if (g.head_dim != 16 && g.head_dim != 32 && g.head_dim != 64 && g.head_dim != 128)
    return bad("head_dim must be 16, 32, 64 or 128");
  if (g.d_model % 8 || g.d_ffn % 8) return bad("d_model and d_ffn must be multiples of 8");
  if (g.n_draft < 0 || g.n_draft + 1 > kMaxRows) return bad("n_draft must be in [0, 15]");
  if (g.max_batch < 1 || g.max_ctx < kMaxRows) return bad("max_batch < 1 or max_ctx < 16");
  if (g.n_cond < 0) return bad("n_cond < 0");
  if (g.head_kind != XSM_HEAD_MLP && g.head_kind != XSM_HEAD_CA) return bad("head_kind must be XSM_HEAD_MLP or XSM_HEAD_CA");
  if (g.head_kind == XSM_HEAD_CA && g.n_cond < 1) return bad("cross-attention heads need condition tokens (n_cond > 0)");
  if (g.dtype != XSM_F32 && g.dtype != XSM_BF16) return bad("dtype must be XSM_F32 or XSM_BF16");
  if (!(g.rope_theta > 1.f) || !(g.rms_eps > 0.f)) return bad("rope_theta must be > 1, rms_eps > 0");
  xsm_ctx* c = new (std::nothrow) xsm_ctx();
  if (!c) return bad("out of host memory");
  c->cfg = g;
  c->esz = g.dtype == XSM_BF16 ? 2 : 4;
  c->fast = g.dtype == XSM_BF16 && g.head_dim == 64 && g.d_model % 32 == 0 && g.d_ffn % 32 == 0 &&
            g.vocab % 16 == 0;
  c->small_ok = c->fast && g.n_cond == 0 && small_supported(g.d_model, g.d_ffn) && g.vocab <= 65536 &&
                g.n_layers <= 48;
  build_weight_offsets(c);
  {
    size_t n_tickets = 0;
    build_work_offsets(c, false, c->ws, c->rows_max, c->part_entries, n_tickets);
    build_work_offsets(c, true, c->ws_static, c->rows_max_static, c->part_entries_static, c->n_tickets_static);
  }
  // cache capacities in positions: whole 64-key chunks.  Each (slot, head) owns one contiguous
  // stretch of a cache plane and the attention kernel streams hundreds of those stretches side by
  // side; measured on gfx950, stretches whose length lies within 8 KB of a multiple of 1 MiB
  // (127, 129 or 257 chunks at head width 64) cost 11 % of a whole step against any length that
  // is 24 KB or more away, so the capacity grows by a few chunks until it is.
  auto spread_chunks = [&](int n) {
    int ch = (n + 63) / 64;
    const long chunk_bytes = 64L * g.head_dim * (long)c->esz, mib = 1L << 20, clear = 24L << 10;
    for (;; ++ch) {
      const long r = (ch * chunk_bytes) & (mib - 1);
      if (ch * chunk_bytes < mib - clear || (r >= clear && mib - r >= clear)) break;
    }
    return ch * 64;
  };
  c->cap_self = spread_chunks(g.max_ctx);
  c->cap_cross = g.n_cond > 0 ? spread_chunks(g.n_cond) : 0;
  c->w_canon_bytes = align_up(c->woff.total * c->esz);
  c->rope_off = c->w_canon_bytes;
  c->weights_bytes = c->rope_off + align_up((size_t)g.max_ctx * (g.head_dim / 2) * sizeof(float2));
  if (c->fast) c->weights_bytes = build_tiled_offsets(c, c->weights_bytes);
  if (c->small_ok) {
    c->layer_tab_off = c->weights_bytes;
    c->weights_bytes += align_up(sizeof(LayerTab) * g.n_layers);
  }
  c->kv_self_elems = (size_t)g.n_layers * 2 * g.max_batch * g.n_heads * c->cap_self * g.head_dim;
  c->kv_cross_elems = (size_t)g.n_layers * 2 * g.max_batch * g.n_heads * c->cap_cross * g.head_dim;
  const size_t hcross = g.head_kind == XSM_HEAD_CA
                            ? (size_t)g.n_draft * 2 * g.max_batch * g.n_heads * c->cap_cross * g.head_dim : 0;
  c->kv_bytes = align_up((c->kv_self_elems + c->kv_cross_elems + hcross) * c->esz);
  *out = c;
  return XSM_OK;
}

void xsm_destroy(xsm_ctx* ctx) { delete ctx; }

const char* xsm_last_error(const xsm_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

size_t xsm_weights_bytes(const xsm_ctx* ctx) { return ctx ? ctx->weights_bytes : 0; }
size_t xsm_kv_bytes(const xsm_ctx* ctx) { return ctx ? ctx->kv_bytes : 0; }
size_t xsm_workspace_bytes(const xsm_ctx* ctx) { return ctx ? ctx->ws.total : 0; }
size_t xsm_canonical_weight_elems(const xsm_ctx* ctx) { return ctx ? ctx->woff.total : 0; }

int xsm_bind(xsm_ctx* ctx, void* d_weights, void* d_kv, void* d_workspace) {
  if (!ctx) return XSM_EINVAL;
  if (!d_weights || !d_kv || !d_workspace) return fail(ctx, XSM_EINVAL, "null buffer");
  if (((uintptr_t)d_weights | (uintptr_t)d_kv | (uintptr_t)d_workspace) & 255)
    return fail(ctx, XSM_EINVAL, "buffers must be 256-byte aligned");
  ctx->d_w = (char*)d_weights; ctx->d_kv = (char*)d_kv; ctx->d_ws = (char*)d_workspace;
  ctx->loaded = false;
  {
    const int rc = static_scratch_lookup(ctx, &ctx->dev, &ctx->d_static);
    if (rc) return rc;
  }
  // The single-launch step hands data between its 256 workgroups, one per compute unit (each
  // takes most of a unit's LDS), so all of them must be resident together: a device, or a
  // partition of one, with fewer units takes the per-stage path.
  ctx->small_dev = false;
  if (ctx->small_ok) {
    int dev = 0, units = 0;
    XSM_HIP(hipGetDevice(&dev));
    XSM_HIP(hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, dev));
    ctx->small_dev = units >= 256;
  }
  return XSM_OK;
}

int xsm_load_weights(xsm_ctx* ctx, const void* h_canonical, size_t n_elems, xsm_stream stream) {
  if (!ctx) return XSM_EINVAL;
  if (!ctx->d_w) return fail(ctx, XSM_ESTATE, "buffers not bound");
  if (!h_canonical) return fail(ctx, XSM_EINVAL, "null weights");
  if (n_elems != ctx->woff.total) return fail(ctx, XSM_EINVAL, "weight element count does not match the configuration");
  hipStream_t s = (hipStream_t)stream;
  XSM_HIP(hipMemcpyAsync(ctx->d_w, h_canonical, n_elems * ctx->esz, hipMemcpyHostToDevice, s));
  launch_rope_table((float2*)(ctx->d_w + ctx->rope_off), ctx->cfg.max_ctx, ctx->cfg.head_dim,
                    ctx->cfg.rope_theta, s);
  if (ctx->fast) {             // fragment-ordered copies for the MFMA kernels
    const xsm_config& g = ctx->cfg;
    const int d = g.d_model, F = g.d_ffn, V = g.vocab;
    char* wb = ctx->d_w;
    for (int l = 0; l < g.n_layers; ++l) {
      const LayerPtrs P = layer_ptrs(ctx, l);
      const TiledLayer& T = ctx->toff.layer[l];
      launch_tile_weights(P.Wqkv, wb + T.Wqkv, 3 * d, d, d, g.head_dim, s);
      launch_tile_weights(P.Wo, wb + T.Wo, d, d, 0, 0, s);
      if (g.n_cond > 0) {
        launch_tile_weights(P.Wcq, wb + T.Wcq, d, d, 0, 0, s);
        launch_tile_weights(P.Wckv, wb + T.Wckv, 2 * d, d, 0, 0, s);
        launch_tile_weights(P.Wco, wb + T.Wco, d, d, 0, 0, s);
      }
      launch_tile_weights(P.W1, wb + T.W1, F, d, 0, 0, s);
      launch_tile_weights(P.W2, wb + T.W2, d, F, 0, 0, s);
    }
    launch_tile_weights(wb + ctx->woff.WU * 2, wb + ctx->toff.WU, V, d, 0, 0, s);
    for (int k = 0; k < g.n_draft; ++k) {
      if (g.head_kind == XSM_HEAD_CA) {
        launch_tile_weights(wb + ctx->woff.hq[k] * 2, wb + ctx->toff.Wh + (size_t)k * d * d * 2, d, d, 0, 0, s);
        launch_tile_weights(wb + ctx->woff.ho[k] * 2, wb + ctx->toff.Who[k], d, d, 0, 0, s);
        launch_tile_weights(wb + ctx->woff.hU[k] * 2, wb + ctx->toff.WhU[k], V, d, 0, 0, s);
        launch_tile_weights(wb + ctx->woff.hkv[k] * 2, wb + ctx->toff.Whkv[k], 2 * d, d, 0, 0, s);
      } else {
        launch_tile_weights(wb + ctx->woff.hW[k] * 2, wb + ctx->toff.Wh + (size_t)k * d * d * 2, d, d, 0, 0, s);
        launch_copy_u16(wb + ctx->woff.hb[k] * 2, wb + ctx->toff.hb + (size_t)k * d * 2, d, s);
      }
    }
    {
      size_t attn_pairs = (size_t)g.max_batch * g.n_heads * (g.head_kind == XSM_HEAD_CA && g.n_draft ? g.n_draft : 1);
      if (attn_pairs < ctx->rows_max / 16 * g.n_heads) attn_pairs = ctx->rows_max / 16 * g.n_heads;
      launch_fill_i32((int32_t*)(ctx->d_ws + ctx->ws.tickets), (int)attn_pairs, 0, s);
    }
    launch_fill_i32((int32_t*)(ctx->d_ws + ctx->ws.gtickets), (int)kWsTickets, 0, s);
    if (ctx->small_ok) {
      ctx->layer_tab.resize(g.n_layers);
      for (int l = 0; l < g.n_layers; ++l) {
        const LayerPtrs P = layer_ptrs(ctx, l);
        const TiledLayer& T = ctx->toff.layer[l];
        ctx->layer_tab[l] = LayerTab{(const uint4*)(wb + T.Wqkv), (const uint4*)(wb + T.Wo),
                                     (const uint4*)(wb + T.W1), (const uint4*)(wb + T.W2),
                                     (const uint16_t*)P.g1, (const uint16_t*)P.g2,
                                     (uint16_t*)self_cache(ctx, l, 0), (uint16_t*)self_cache(ctx, l, 1)};
      }
      XSM_HIP(hipMemcpyAsync(wb + ctx->layer_tab_off, ctx->layer_tab.data(),
                             sizeof(LayerTab) * g.n_layers, hipMemcpyHostToDevice, s));
      // exchange words start with tag 0; the step epoch starts at 1, error word and barrier words clear
      launch_fill_u64((uint64_t*)(ctx->d_ws + ctx->ws.ll),
                      small_ll_words(g.n_layers, g.d_model, g.d_ffn, g.n_draft) / 2, 0ull, s);
      launch_fill_u64((uint64_t*)(ctx->d_ws + ctx->ws.ctrl), kSmallCtrlBytes / 8, 0ull, s);
      launch_fill_u64((uint64_t*)(ctx->d_ws + ctx->ws.ctrl), 1, 1ull, s);
    }
  }
  XSM_HIP(hipGetLastError());
  ctx->loaded = true;
  ctx->small_failed = false;
  return XSM_OK;
}

int xsm_prefill(xsm_ctx* ctx, int32_t n_seq, const int32_t* h_slot, const void* d_prefix_emb,
                int32_t P, const void* d_cond, xsm_stream stream) {
  int rc = check_ready(ctx);
  if (rc) return rc;
  const xsm_config& g = ctx->cfg;
  if (n_seq < 1 || !h_slot) return fail(ctx, XSM_EINVAL, "n_seq < 1 or null slots");
  if (n_seq > g.max_batch) return fail(ctx, XSM_ECAPACITY, "n_seq > max_batch");
  if (P < 0 || (P > 0 && !d_prefix_emb)) return fail(ctx, XSM_EINVAL, "bad prefix");
  if (P > g.max_ctx) return fail(ctx, XSM_ECAPACITY, "prefix longer than max_ctx");
  if (g.n_cond > 0 && !d_cond) return fail(ctx, XSM_EINVAL, "condition tokens required");
  for (int i = 0; i < n_seq; ++i) {
    if (h_slot[i] < 0 || h_slot[i] >= g.max_batch) return fail(ctx, XSM_EINVAL, "slot out of range");
    for (int j = 0; j < i; ++j)
      if (h_slot[j] == h_slot[i]) return fail(ctx, XSM_EINVAL, "duplicate slot");
  }
  hipStream_t s = (hipStream_t)stream;
  char* ws = ctx->d_ws;
  const int d = g.d_model, dt = g.dtype;
  float* X = (float*)(ws + ctx->ws.X);
  float* QKV = (float*)(ws + ctx->ws.QKV);
  int32_t* eff = (int32_t*)(ws + ctx->ws.eff_len);
  int32_t* slot = (int32_t*)(ws + ctx->ws.slot);
  XSM_HIP(hipMemcpyAsync(slot, h_slot, (size_t)n_seq * 4, hipMemcpyHostToDevice, s));
  // rows per sequence per pass: 16 on the general kernels; on the MFMA path as many as the
  // workspace holds (whole query tiles), so that a pass streams the weights for up to 8192 rows
  int chunk = kPrefillChunk;
  if (ctx->fast) {
    size_t pass_rows = ctx->rows_max;
    if (ctx->prefill_rows > 0 && (size_t)ctx->prefill_rows < pass_rows) pass_rows = ctx->prefill_rows;
    chunk = (int)(pass_rows / n_seq) / 16 * 16;
    if (chunk > kFastPassRows) chunk = kFastPassRows;
    if (chunk < 16) chunk = 16;
  }
  if (g.n_cond > 0) {      // per-layer cross-attention keys/values of the condition tokens
    float* Xn = (float*)(ws + ctx->ws.Xn);
    float* gpart = (float*)(ws + ctx->ws.gpart);
    uint32_t* gtick = (uint32_t*)(ws + ctx->ws.gtickets);
    bool cond_plane = false;
    auto project = [&](const void* Wcanon, size_t Wtiled, int M, char* kc, char* vc, int C, int r0) {
      if (ctx->fast) {
        FastGemm p{};
        p.Wt = (const uint4*)(ctx->d_w + Wtiled); p.N = 2 * d; p.K = d; p.M = M;
        p.X = X; p.ldx = d; p.Y = QKV; p.ldy = 2 * d;
        p.nscratch = Xn; p.ws_part = gpart; p.ws_tickets = gtick; p.pend = &ctx->pend;
        p.x_single = cond_plane ? 1 : 0;             // (X then holds the condition rows as one bf16 operand plane)
        fgemm(ctx, cond_plane ? PRO_PLANES : PRO_F32, FEPI_STORE, p, s);
      } else {
        launch_gemm(dt, EPI_STORE, X, d, Wcanon, QKV, 2 * d, M, 2 * d, d, s);
      }
      launch_store_cond(dt, QKV, slot, kc, vc, n_seq, C, r0, g.n_heads, g.head_dim, ctx->cap_cross,
                        ctx->fast ? 1 : 0, s);
    };
    for (int r0 = 0; r0 < g.n_cond; r0 += chunk) {
      const int C = g.n_cond - r0 < chunk ? g.n_cond - r0 : chunk;
      // the condition tokens are bf16: in a pass large enough for the row-blocked kernel they go in
      // as they are (one operand plane, no low part, half the products of an fp32 activation)
      cond_plane = ctx->fast && fgemm_planes_ok(n_seq * C, 2 * d, d);
      if (cond_plane) launch_load_rows_plane(d_cond, X, n_seq, C, r0, g.n_cond, d, s);
      else launch_load_rows(dt, d_cond, X, n_seq, C, r0, g.n_cond, d, s);
      for (int l = 0; l < g.n_layers; ++l) {
        const LayerPtrs L = layer_ptrs(ctx, l);
        project(L.Wckv, ctx->fast ? ctx->toff.layer[l].Wckv : 0, n_seq * C, cross_cache(ctx, l, 0), cross_cache(ctx, l, 1), C, r0);
      }
      if (g.head_kind == XSM_HEAD_CA)          // the decoding heads' own keys/values of the condition
        for (int k = 0; k < g.n_draft; ++k)
          project(ctx->d_w + ctx->woff.hkv[k] * ctx->esz, ctx->fast ? ctx->toff.Whkv[k] : 0, n_seq * C,
                  head_cache(ctx, k, 0), head_cache(ctx, k, 1), C, r0);
    }
  }
  for (int r0 = 0; r0 < P; r0 += chunk) {
    const int C = P - r0 < chunk ? P - r0 : chunk;
    launch_fill_i32(eff, n_seq, r0, s);
    launch_load_rows(dt, d_prefix_emb, X, n_seq, C, r0, P, d, s);
    forward_blocks(ctx, n_seq, C, r0, s);
  }
  XSM_HIP(hipGetLastError());
  return unmatched_gemm(ctx);
}

int xsm_spec_step(xsm_ctx* ctx, const xsm_batch* batch, const xsm_verify_params* vp,
                  xsm_stream stream) {
  if (!ctx) return XSM_EINVAL;
  if (ctx->cfg.n_draft < 1) return fail(ctx, XSM_EINVAL, "speculative step needs n_draft >= 1");
  return step_common(ctx, batch, vp, stream, ctx->cfg.n_draft + 1);
}

int xsm_plain_step(xsm_ctx* ctx, const xsm_batch* batch, const xsm_verify_params* vp,
                   xsm_stream stream) {
  if (!ctx) return XSM_EINVAL;
  return step_common(ctx, batch, vp, stream, 1);
}

int xsm_spec_step_static(xsm_ctx* ctx, const xsm_batch* batch, const xsm_verify_params* vp,
                         xsm_stream stream) {
  if (!ctx) return XSM_EINVAL;
  if (ctx->cfg.n_draft < 1) return fail(ctx, XSM_EINVAL, "speculative step needs n_draft >= 1");
  int rc = check_ready(ctx);
  if (rc) return rc;
  if (ctx->ws_static.total > kStaticScratchBytes)
    return fail(ctx, XSM_ECAPACITY, "this configuration's steps need " + std::to_string(ctx->ws_static.total) +
                                        " bytes of scratch, the static array holds " +
                                        std::to_string(kStaticScratchBytes) + ": use xsm_spec_step with a bound workspace");
  int dev = -1;
  XSM_HIP(hipGetDevice(&dev));
  if (dev != ctx->dev || !ctx->d_static)
    return fail(ctx, XSM_ESTATE, "the current device is not the one the buffers were bound on");
  // The step's kernels find their activations, partial products and arrival counters through
  // the context's workspace pointer and layout: for this call those name the static array.
  struct Swap {
    xsm_ctx* c; char* d_ws; WorkOff ws; size_t part_entries, rows_max; bool use_small;
    explicit Swap(xsm_ctx* x) : c(x), d_ws(x->d_ws), ws(x->ws), part_entries(x->part_entries),
                                rows_max(x->rows_max), use_small(x->use_small) {
      c->d_ws = c->d_static; c->ws = c->ws_static; c->part_entries = c->part_entries_static;
      c->rows_max = c->rows_max_static;
      c->use_small = false;          // (the single-launch step's exchange buffers are not part of this layout)
    }
    ~Swap() { c->d_ws = d_ws; c->ws = ws; c->part_entries = part_entries; c->rows_max = rows_max; c->use_small = use_small; }
  } swap(ctx);
  // The array keeps what the last call on this GPU left (of any context, any layout): the
  // arrival counters must start at zero.  Fill kernels, not memset nodes, so that a caller may
  // capture the call in a graph.
  hipStream_t s = (hipStream_t)stream;
  launch_fill_i32((int32_t*)(ctx->d_ws + ctx->ws.tickets), (int)ctx->n_tickets_static, 0, s);
  if (ctx->fast) launch_fill_i32((int32_t*)(ctx->d_ws + ctx->ws.gtickets), (int)kWsTickets, 0, s);
  return step_common(ctx, batch, vp, stream, ctx->cfg.n_draft + 1);
}

int xsm_set_option(xsm_ctx* ctx, int32_t option, int32_t value) {
  if (!ctx) return XSM_EINVAL;
  if (option == XSM_OPT_SINGLE_LAUNCH) { ctx->use_small = value != 0; return XSM_OK; }
  if (option == XSM_OPT_TIMELINE) { ctx->timeline = value != 0; return XSM_OK; }
  if (option == XSM_OPT_ATTN_SPLITS) { ctx->force_splits = value > 0 ? value : 0; return XSM_OK; }
  if (option == XSM_OPT_PREFILL_ROWS) { ctx->prefill_rows = value > 0 ? value : 0; return XSM_OK; }
  return fail(ctx, XSM_EINVAL, "unknown option");
}

int xsm_debug_timeline(xsm_ctx* ctx, uint64_t* h_out, size_t n_words) {
  if (!ctx || !h_out) return XSM_EINVAL;
  if (!ctx->small_ok || !ctx->d_ws) return fail(ctx, XSM_ESTATE, "no single-launch step for this model");
  const size_t have = (size_t)256 * (ctx->cfg.n_layers * 16 + 8);
  if (n_words < have) return fail(ctx, XSM_EINVAL, "timeline buffer too small");
  XSM_HIP(hipDeviceSynchronize());
  XSM_HIP(hipMemcpy(h_out, ctx->d_ws + ctx->ws.tlog, have * 8, hipMemcpyDeviceToHost));
  return XSM_OK;
}

int xsm_check_device(xsm_ctx* ctx) {
  if (!ctx) return XSM_EINVAL;
  XSM_HIP(hipDeviceSynchronize());
  if (!ctx->small_ok || !ctx->d_ws || !ctx->loaded) return XSM_OK;
  uint32_t c[2] = {0, 0};
  XSM_HIP(hipMemcpy(c, ctx->d_ws + ctx->ws.ctrl, 8, hipMemcpyDeviceToHost));
  if (c[1] != 0) {
    // reported once: the error word is cleared and this context's later steps take the per-stage
    // kernels (the exchange buffers may hold half a step; loading weights again resets them)
    const uint32_t zero = 0;
    XSM_HIP(hipMemcpy(ctx->d_ws + ctx->ws.ctrl + 4, &zero, 4, hipMemcpyHostToDevice));
    ctx->small_failed = true;
    return fail(ctx, XSM_EDEVICE, "single-launch step: a wait for stage inputs timed out (stage code " +
                                      std::to_string(c[1]) + "); the sequences of that step carry n_accepted = 0 and "
                                      "XSM_FLAG_DEVICE_TIMEOUT, later steps run on the per-stage kernels");
  }
  return XSM_OK;
}

int xsm_debug_inject_device_error(xsm_ctx* ctx, uint32_t code) {
  if (!ctx) return XSM_EINVAL;
  if (!ctx->small_ok || !ctx->d_ws || !ctx->loaded) return fail(ctx, XSM_ESTATE, "no single-launch step for this model");
  XSM_HIP(hipDeviceSynchronize());
  XSM_HIP(hipMemcpy(ctx->d_ws + ctx->ws.ctrl + 4, &code, 4, hipMemcpyHostToDevice));
  return XSM_OK;
}

static int kv_debug(xsm_ctx* ctx, int32_t layer, int32_t which, int32_t slot, int32_t pos0,
                    int32_t n_pos, float* h_buf, bool to_cache) {
  if (!ctx) return XSM_EINVAL;
  if (!ctx->d_kv || !ctx->d_ws) return fail(ctx, XSM_ESTATE, "buffers not bound");
  const xsm_config& g = ctx->cfg;
  const bool cross = which >= 2;
  const int cap = cross ? g.n_cond : g.max_ctx;
  if (layer < 0 || layer >= g.n_layers || which < 0 || which > 3 || slot < 0 || slot >= g.max_batch ||
      pos0 < 0 || n_pos < 1 || pos0 + n_pos > cap || !h_buf)
    return fail(ctx, XSM_EINVAL, "bad cache range");
  char* base = cross ? cross_cache(ctx, layer, which - 2) : self_cache(ctx, layer, which);
  const int capp = cross ? ctx->cap_cross : ctx->cap_self;       // padded capacity
  char* rows = base + (size_t)slot * g.n_heads * capp * g.head_dim * ctx->esz;
  const bool tr = ctx->fast && (which & 1);                       // values are cached transposed
  const size_t st_h = (size_t)capp * g.head_dim;
  const size_t st_p = tr ? 1 : (size_t)g.head_dim, st_i = tr ? (size_t)capp : 1;
  // staged through the activation region of the workspace in pieces that fit
  const size_t stage_elems = (size_t)g.max_batch * kMaxRows * g.d_model * 2;   // X + Xn regions
  float* stage = (float*)(ctx->d_ws + ctx->ws.X);
  const int per = (int)(stage_elems / ((size_t)g.n_heads * g.head_dim));
  XSM_HIP(hipDeviceSynchronize());
  for (int p = 0; p < n_pos; p += per) {
    const int np = n_pos - p < per ? n_pos - p : per;
    const size_t n = (size_t)g.n_heads * np * g.head_dim;
    std::vector<float> tmp(n);
    if (to_cache) {
      for (int h = 0; h < g.n_heads; ++h)
        memcpy(&tmp[(size_t)h * np * g.head_dim], h_buf + ((size_t)h * n_pos + p) * g.head_dim,
               (size_t)np * g.head_dim * 4);
      XSM_HIP(hipMemcpy(stage, tmp.data(), n * 4, hipMemcpyHostToDevice));
      launch_kv_convert(g.dtype, rows, stage, g.n_heads, pos0 + p, np, g.head_dim, st_h, st_p, st_i, 1, 0);
      XSM_HIP(hipDeviceSynchronize());
    } else {
      XSM_HIP(hipDeviceSynchronize());
      launch_kv_convert(g.dtype, rows, stage, g.n_heads, pos0 + p, np, g.head_dim, st_h, st_p, st_i, 0, 0);
      XSM_HIP(hipMemcpy(tmp.data(), stage, n * 4, hipMemcpyDeviceToHost));
      for (int h = 0; h < g.n_heads; ++h)
        memcpy(h_buf + ((size_t)h * n_pos + p) * g.head_dim, &tmp[(size_t)h * np * g.head_dim],
               (size_t)np * g.head_dim * 4);
    }
  }
  return XSM_OK;
}

int xsm_debug_kv_clone(xsm_ctx* ctx, int32_t src_slot, int32_t dst_slot) {
  if (!ctx) return XSM_EINVAL;
  if (!ctx->d_kv) return fail(ctx, XSM_ESTATE, "buffers not bound");
  const xsm_config& g = ctx->cfg;
  if (src_slot < 0 || dst_slot < 0 || src_slot >= g.max_batch || dst_slot >= g.max_batch)
    return fail(ctx, XSM_EINVAL, "slot out of range");
  XSM_HIP(hipDeviceSynchronize());
  if (src_slot == dst_slot) return XSM_OK;
  for (int l = 0; l < g.n_layers; ++l)
    for (int which = 0; which < 2; ++which) {
      const size_t per = (size_t)g.n_heads * ctx->cap_self * g.head_dim * ctx->esz;
      char* base = self_cache(ctx, l, which);
      XSM_HIP(hipMemcpy(base + dst_slot * per, base + src_slot * per, per, hipMemcpyDeviceToDevice));
      if (g.n_cond > 0) {
        const size_t perc = (size_t)g.n_heads * ctx->cap_cross * g.head_dim * ctx->esz;
        char* cb = cross_cache(ctx, l, which);
        XSM_HIP(hipMemcpy(cb + dst_slot * perc, cb + src_slot * perc, perc, hipMemcpyDeviceToDevice));
      }
    }
  if (g.head_kind == XSM_HEAD_CA)
    for (int k = 0; k < g.n_draft; ++k)
      for (int which = 0; which < 2; ++which) {
        const size_t perc = (size_t)g.n_heads * ctx->cap_cross * g.head_dim * ctx->esz;
        char* hb = head_cache(ctx, k, which);
        XSM_HIP(hipMemcpy(hb + dst_slot * perc, hb + src_slot * perc, perc, hipMemcpyDeviceToDevice));
      }
  XSM_HIP(hipDeviceSynchronize());
  return XSM_OK;
}

int xsm_debug_kv_export(xsm_ctx* ctx, int32_t layer, int32_t which, int32_t slot, int32_t pos0,
                        int32_t n_pos, float* h_out) {
  return kv_debug(ctx, layer, which, slot, pos0, n_pos, h_out, false);
}
int xsm_debug_kv_import(xsm_ctx* ctx, int32_t layer, int32_t which, int32_t slot, int32_t pos0,
                        int32_t n_pos, const float* h_in) {
  return kv_debug(ctx, layer, which, slot, pos0, n_pos, const_cast<float*>(h_in), true);
}

}  // extern "C"
