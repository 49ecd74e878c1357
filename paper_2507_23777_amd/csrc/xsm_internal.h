// Host-side internals of libxsm: context, buffer layouts, kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "../../include/xsm.h"

namespace xsm {

constexpr int kPrefillChunk = 16;   // prefix rows per sequence per backbone pass (general kernels)
constexpr int kFastPassRows = 8192; // rows of one backbone pass the MFMA path's workspace always holds (prefill chunks)
constexpr int kMaxRows = 16;        // rows per sequence per pass (K+1 <= 16)

// Element offsets of the canonical weight tensors (same order as the weight file).
struct LayerOff {
  size_t g1, Wqkv, Wo, gc, Wcq, Wckv, Wco, g2, W1, W2;
};
struct WeightOff {
  size_t E, gf, WU, total;
  std::vector<LayerOff> layer;
  std::vector<size_t> hW, hb;                 // MLP heads
  std::vector<size_t> hq, hkv, ho, hU;        // cross-attention heads
};

// Byte offsets inside the caller's workspace buffer.
struct WorkOff {
  size_t X, Xn, QKV, Qr, AO, U, Z0, G, Hh, Rk, Zh;
  size_t eff_len, slot, acc, y0, wflags, toks, rowidx, eff2, slot2;   // int32 arrays
  size_t part, tickets, gpart, gtickets;                                  // split-key attention partials
  size_t ll, ctrl, head_all, tlog;                       // single-launch step: exchange buffers
  size_t total;
};

// Byte offsets of the fragment-ordered (tiled) bf16 matrices inside the weights buffer.
struct TiledLayer { size_t Wqkv, Wo, Wcq, Wckv, Wco, W1, W2; };
struct TiledOff {
  std::vector<TiledLayer> layer;
  size_t WU, Wh, hb;       // unembedding, stacked head matrices [K*d][d] (MLP: W_k, CA: Wq_k), stacked head biases [K][d]
  std::vector<size_t> Who, WhU, Whkv;   // cross-attention heads: output projections, unembeddings, key/value projections
  bool wu_ok;              // vocabulary is a multiple of 16
};

// Per-layer pointers of the single-launch step (uploaded to the device at load time).
// Output of a residual-add projection that is still in split-contraction partial blocks
// [N/64][kspl][M][64]; the next RMSNorm pass over Y (or flush_pending_add) adds it in.
struct PendingAdd {
  bool active = false;
  const float* part = nullptr;
  int kspl = 0, M = 0, N = 0;
  float* Y = nullptr;
  int ldy = 0;
};
void flush_pending_add(PendingAdd* p, hipStream_t s);

struct LayerTab {
  const uint4 *Wqkv, *Wo, *W1, *W2;     // fragment-ordered weights
  const uint16_t *g1, *g2;              // RMSNorm gains (bf16)
  uint16_t *Kc, *Vt;                    // this layer's key cache and transposed value cache
};

}  // namespace xsm

struct xsm_ctx {
  xsm_config cfg;
  xsm::WeightOff woff;
  xsm::WorkOff ws;
  size_t esz;              // bytes per storage element
  size_t w_canon_bytes;    // canonical weights
  size_t rope_off;         // byte offset of the rotary table in the weights buffer
  size_t weights_bytes, kv_bytes;
  size_t kv_self_elems;    // elements of the self-attention cache (cross cache follows)
  size_t kv_cross_elems;   // elements of the layers' cross cache (the heads' condition cache follows)
  bool fast = false;       // bf16 MFMA path (head_dim 64, values cached transposed)
  bool small_ok = false;   // single-launch step available for this model shape
  bool use_small = true;   // xsm_set_option(XSM_OPT_SINGLE_LAUNCH)
  bool small_dev = false;  // the bound device can hold the single launch's 256 workgroups at once
  bool small_failed = false;   // xsm_check_device found a timed-out wait: per-stage kernels until weights are loaded again
  bool gemm_unmatched = false; // a projection found no kernel for its (prologue, epilogue) pair: the step reports it
  bool timeline = false;   // xsm_set_option(XSM_OPT_TIMELINE)
  int force_splits = 0;    // xsm_set_option(XSM_OPT_ATTN_SPLITS): key-range slices per (sequence, head), 0 = automatic
  int prefill_rows = 0;              // XSM_OPT_PREFILL_ROWS: rows per prefill pass, 0 = what the workspace holds
  size_t layer_tab_off = 0;              // byte offset of the LayerTab array in the weights buffer
  std::vector<xsm::LayerTab> layer_tab;  // host copy (source of the upload)
  xsm::TiledOff toff;
  int cap_self = 0, cap_cross = 0;   // cache capacities in positions, padded to 64
  xsm::PendingAdd pend;              // see PendingAdd
  size_t part_entries = 0;           // (sequence, head, query tile, split) partial slots in the workspace
  size_t rows_max = 0;               // rows of one backbone pass the workspace holds
  // layout of the static scratch array (decoding steps only) for xsm_spec_step_static
  xsm::WorkOff ws_static;
  size_t part_entries_static = 0, rows_max_static = 0, n_tickets_static = 0;
  int dev = -1;                      // device the buffers were bound on
  char* d_static = nullptr;          // that device's address of the static scratch array
  char* d_w = nullptr;
  char* d_kv = nullptr;
  char* d_ws = nullptr;
  bool loaded = false;
  std::string err;
};

namespace xsm {

// Optional per-kernel timing with HIP events on the launch stream (off by default; used by
// the benchmark to attribute step time to kernels).  A scope brackets one launch.
// A kernel's dynamic-LDS limit above 64 KB is a property of (kernel, device): raised once for
// each pair, and again if a later launch of the kernel needs more.
inline void allow_dynamic_lds(const void* kfn, size_t bytes) {
  if (bytes <= 64 * 1024) return;
  static std::mutex mu;
  static std::map<std::pair<const void*, int>, size_t> granted;
  int dev = 0;
  (void)hipGetDevice(&dev);
  std::lock_guard<std::mutex> lock(mu);
  size_t& have = granted[{kfn, dev}];
  if (bytes > have) {
    (void)hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    have = bytes;
  }
}

struct TraceScope {
  TraceScope(const char* name, hipStream_t s);
  ~TraceScope();
  hipStream_t s_;
  int idx_;
};

// ---- launchers (xsm_kernels_basic.hip) -------------------------------------
// dtype: XSM_F32 or XSM_BF16 selects the storage type of weights / cache / embeddings.
void launch_rope_table(float2* tab, int max_ctx, int head_dim, float theta, hipStream_t s);

// Validate one step's inputs: eff_len[b] = kv_len[b] or -1 (sequence skipped), slot copy,
// flag bits.
void launch_prepare(const int32_t* kv_len, const int32_t* slot, const int32_t* block, int n_seq,
                    int R, int vocab, int max_batch, int max_ctx, int kv_len_bound,
                    int32_t* eff_len, int32_t* slot_out, uint32_t* wflags, hipStream_t s);
void launch_fill_i32(int32_t* p, int n, int32_t v, hipStream_t s);

void launch_embed(int dtype, const void* E, const int32_t* block, const int32_t* eff_len, float* X,
                  int n_seq, int R, int d, hipStream_t s);
// X[b*C + j] = emb[b][row0 + j] for j < C
// bf16 rows -> one fragment-ordered operand plane [n_seq*C][d] (d % 32 == 0)
void launch_load_rows_plane(const void* emb, void* plane, int n_seq, int C, int row0, int rows_per_seq, int d,
                            hipStream_t s);
void launch_load_rows(int dtype, const void* emb, float* X, int n_seq, int C, int row0,
                      int rows_per_seq, int d, hipStream_t s);
void launch_rmsnorm(int dtype, const float* X, const void* gain, float* Y, int M, int d, float eps,
                    hipStream_t s);
enum { EPI_STORE = 0, EPI_ADD = 1, EPI_GELU = 2 };
// Y[m][n] (op)= sum_k A[m][k] * W[n][k]
void launch_gemm(int dtype, int epi, const float* A, int lda, const void* W, float* Y, int ldy,
                 int M, int N, int K, hipStream_t s);
// rotate q,k of QKV[M][3d], write q to Qr[M][d], k/v into the cache at eff_len[b] + j
void launch_rope_kv(int dtype, const float* QKV, const float2* rope, const int32_t* eff_len,
                    const int32_t* slot, float* Qr, void* Kc, void* Vc, int n_seq, int R, int H,
                    int hd, int max_ctx, hipStream_t s);
// cond K/V rows of one chunk into the cross cache: KV[M][2d] -> caches at rows row0..row0+C-1
void launch_store_cond(int dtype, const float* KV, const int32_t* slot, void* Kc, void* Vc,
                       int n_seq, int C, int row0, int H, int hd, int cap, int v_transposed,
                       hipStream_t s);
// attention of row m = b*R + j over cache positions < (fixed_limit > 0 ? fixed_limit
// : eff_len[b] + j + 1)
void launch_attention(int dtype, const float* Q, const void* Kc, const void* Vc,
                      const int32_t* eff_len, const int32_t* slot, float* O, int n_seq, int R,
                      int H, int hd, int cap, int fixed_limit, hipStream_t s);

// ---- MFMA path (xsm_gemm_mfma.hip, xsm_attn_mfma.hip) ----------------------------
enum { PRO_NORM = 0, PRO_F32 = 1, PRO_PLANES = 2 };   // PRO_PLANES: X holds fragment-ordered bf16 hi/lo planes (M > 256 only)
enum { FEPI_STORE = 0, FEPI_ADD = 1, FEPI_GELU = 2, FEPI_QKV = 3, FEPI_HEAD = 4 };
struct FastGemm {
  const uint4* Wt;             // fragment-ordered weights [N/16][K/32][64 lanes][8]
  int N, K, M, KC;
  const float* X; int ldx;     // fp32 input rows (PRO_PLANES: the planes, ldx unused)
  int x_single;                // PRO_PLANES: the input is exact in bf16, only the hi plane exists (FEPI_STORE only)
  const uint16_t* gain;        // bf16 RMSNorm gain [K] (PRO_NORM)
  float eps;
  const int32_t* row_index;    // optional gather: input row of output row m
  float* Y; int ldy;           // fp32 output (for FEPI_QKV: the rotated queries [M][d])
  int y_planes;                // FEPI_GELU in the row-blocked kernel: write Y as operand planes [M][N] instead
  const uint16_t* bias;        // FEPI_HEAD: stacked biases [N]
  float* nscratch;             // [M][K] fp32: normalised rows for the kernels that do not fuse the norm
  int ksplit;                  // row-blocked kernel, FEPI_ADD: slices of the contraction index (set by the launcher)
  float* ws_part; uint32_t* ws_tickets;   // split-contraction partial products and arrival counters
  PendingAdd* pend;            // host-side: where a residual-add projection may leave its sum pending
  // FEPI_QKV
  const float2* rope; const int32_t* eff_len; const int32_t* slot;
  int R, H, hd, cap, v_transposed;
  uint16_t* Kc; uint16_t* Vc;
};
bool fgemm_supported(int N, int K);
// true when a projection of these sizes can take its input as operand planes (PRO_PLANES)
bool fgemm_planes_ok(int M, int N, int K);
// slices of the contraction index the row-blocked kernel takes for a residual-add projection
// from operand planes (1 = whole contraction per workgroup), and the partial-product floats
// such projections need for up to Mmax rows
int blk_add_split(int M, int N, int K);
size_t blk_add_part_floats(int Mmax, int N, int K);
constexpr size_t kWsTickets = 4096;      // arrival counters of the split-contraction GEMM
bool ws_gemm_shape_ok(int M, int N, int K);
size_t ws_gemm_part_floats(int M, int N, int K);
// false: no kernel takes this (prologue, epilogue) pair at this shape; nothing was enqueued
bool launch_fgemm(int pro, int epi, const FastGemm& g, hipStream_t s);
void launch_tile_weights(const void* W, void* out, int N, int K, int rope_d, int rope_hd, hipStream_t s);
void launch_copy_u16(const void* src, void* dst, int n, hipStream_t s);

struct FastAttn {
  const float* Q; int ldq;            // fp32 rotated queries [M][d]
  const uint16_t* Kc;                 // layer's keys [slot][H][cap][64]
  const uint16_t* Vt;                 // layer's values, transposed [slot][H][64][cap]
  const int32_t* eff_len; const int32_t* slot;
  float* O; int ldo;                  // fp32 output [M][d]
  int o_planes, o_rows;               // o_planes: write O as operand planes [o_rows][ldo] instead (o_rows = M)
  float* part; uint32_t* tickets;     // split-key partials and arrival counters
  int R, H, cap, S, fixed_limit;
  float scale_log2;                   // log2(e) / sqrt(head_dim)
};
void launch_fattn(const FastAttn& a, int n_seq, hipStream_t s);
size_t fattn_part_bytes(size_t entries);
// row_index[b] = b*R + acc[b] (the hidden state the decoding heads read)
void launch_head_rows(const int32_t* acc, int32_t* row_index, int n_seq, int R, hipStream_t s);
void launch_head_ca_prep(const float* G, float* Rk, const int32_t* eff, const int32_t* slot, int32_t* eff2,
                         int32_t* slot2, int n_seq, int K, int d, int max_batch, hipStream_t s);
// out[m][:] = RMSNorm(X[row_index ? row_index[m] : m][:]) * gain (fp32 in and out, bf16 gain)
void launch_norm_rows(const float* X, int ldx, const int32_t* row_index, const uint16_t* gain, float eps, float* out,
                      int M, int K, hipStream_t s);

// ---- single-launch step for <= 16 block rows (xsm_step_small.hip) -------------------
struct SmallArgs {
  const LayerTab* layers; int L;
  const uint16_t* E; const uint16_t* gf; const uint16_t* hb;
  const uint4* WU; const uint4* Wh;
  const float2* rope;
  uint32_t* ll; size_t ll_layer_stride;  // tagged-word exchange buffers (4-byte words), words per layer
  size_t ll_words;                       // words of the whole exchange region
  uint32_t* ctrl;                        // [0] step epoch, [1] error word, [64..319] the workgroups' barrier words
  const int32_t* slot; int32_t* kv_len; int32_t* block; int32_t* out_tokens; int32_t* n_accepted;
  uint32_t* flags;
  float* logits_dbg; float* head_logits_dbg; float* head_all_dbg; int32_t* acc_out;
  uint64_t* tlog;                        // optional stage timeline [256][L*16 + 8] clock stamps
  int n_seq, R, S, V, max_batch, max_ctx, bound, cap;   // S: key slices per (sequence, head), or their upper limit
  int s_auto;                            // 1: the kernel picks the slice count <= S from the cache lengths it reads
  int full_verify;                       // 0: greedy verification with argmax draws from the per-tile top-2 statistics;
                                         // 1: the last stage reads the full logits rows (logits_dbg / head_all_dbg must
                                         // be set) and applies the criterion and sampling rule of vp
  xsm_verify_params vp;
  float eps, scale_log2;
};
constexpr int kSmallMaxRows = 144;     // backbone rows + head rows (M + M K) of one single-launch step
bool small_supported(int D, int F);
size_t small_ll_words(int n_layers, int D, int F, int K);     // 4-byte words
size_t small_ll_layer_stride(int D, int F);
constexpr size_t kSmallCtrlBytes = 2048;
void launch_step_small(const SmallArgs& a, int D, int F, hipStream_t s);
void launch_fill_u64(uint64_t* p, size_t n, uint64_t v, hipStream_t s);
// head_logits_dbg[b][k][:] = head_all[(b*R + acc[b])*K + k][:]
void launch_gather_head_dbg(const float* head_all, const int32_t* acc, float* out, int n_seq, int R,
                            int K, int V, hipStream_t s);

// ---- launchers (xsm_kernels_verify.hip) --------------------------------------
void launch_verify(const float* Z0, const float* Hf, const int32_t* block, const int32_t* eff_len,
                   const int32_t* slot, const xsm_verify_params& vp, int32_t* acc, int32_t* y0,
                   uint32_t* wflags, float* G, int n_seq, int R, int V, int d, hipStream_t s);
void launch_head_act(int dtype, const float* G, const float* Hh, const void* const* bias_ptrs,
                     float* Rk, int n_seq, int K, int d, hipStream_t s);
void launch_emit(const float* Zh, const xsm_verify_params& vp, const int32_t* eff_len,
                 const int32_t* slot, const int32_t* acc, const int32_t* y0,
                 uint32_t* wflags, int32_t* drawn /*[n_seq][16] scratch*/, int32_t* block, int32_t* kv_len,
                 int32_t* out_tokens, int32_t* n_accepted, uint32_t* flags, int n_seq, int R, int K, int V,
                 hipStream_t s);
void launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s);
// cache <-> float staging [H][n_pos][hd]; element (h, p, i) of the slot lives at
// base[h*stride_h + p*stride_p + i*stride_i]
void launch_kv_convert(int dtype, void* slot_base, float* staging, int H, int pos0, int n_pos,
                       int hd, size_t stride_h, size_t stride_p, size_t stride_i, int to_cache,
                       hipStream_t s);

}  // namespace xsm
