// Internal declarations shared by the HIP sources of libd2o (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "d2o.h"

namespace d2o {

constexpr int kPartRecDoubles = 32;  // doubles of a part record of the split closing kernels
constexpr int kMaxQuerySlices = 16;  // block append: workgroups that share the queries of a (head, chunk)
constexpr int kMinAutoSplitRows = 6144, kMaxAutoSplitRows = 16384;  // bounds of the automatic split_rows (below the lower one the two extra launches cost more than a single closing workgroup)
constexpr int kChunk = 256;        // cache slots handled by one workgroup in the decode kernels
constexpr int kColBN = 256;        // keys per workgroup, column-sum pass (bf16)

// A strided [b][head][token][d] (or [layer][b][head][d]) tensor, strides in elements.
struct View {
  void* ptr;
  int64_t sb, sh, sn;
};

inline View to_view(const d2o_view& v) { return View{v.ptr, v.stride_b, v.stride_h, v.stride_n}; }

// Per-(layer, sequence, KV head) cache geometry, mirrored on the device as int32[4].
struct LayerMeta {
  int32_t base;        // first slot of this layer's region inside a (sequence, KV head) cache
  int32_t budget;      // S_l
  int32_t recent;      // M
  int32_t chunk_base;  // first chunk index of this layer in the decode partial buffers
};

enum LayerPhase { kEmpty = 0, kAttended = 1, kReady = 2 };

struct LayerState {
  int phase = kEmpty;
  int32_t n = 0;          // prompt length seen by the prefill calls
  int32_t next_pos = 0;   // position of the next generated token
  std::vector<LayerMeta> meta;  // [B][Hkv]
};

}  // namespace d2o

struct d2o_timed_launch {
  int id;
  hipEvent_t start, stop;
};

struct d2o_ctx {
  d2o_config cfg;
  std::string err;
  int timing = 0;                    // 0 off; n: time every launch, decode kernels every n-th
  int64_t launch_no[D2O_K_COUNT] = {};
  std::vector<d2o_timed_launch> timed;
  std::vector<d2o::LayerState> layers;
  std::vector<int64_t> used_slots;   // [B][Hkv]
  std::vector<int64_t> used_chunks;  // [B][Hkv]
  int32_t last_compress_layer = -1;
  int32_t last_append_layer = -1;
  int32_t grow = 1;                  // rows a layer's cache region holds beyond its budget: max(1, max_append)
  int32_t esize = 2;                 // bytes per element of Q/K/V (and of the cache, unless it is fp8)
  int32_t csize = 2;                 // bytes per element of a cache row: esize, or 1 for an fp8 cache
  int32_t npad = 0;                  // max_prompt_len rounded up to 128
  int64_t nchunk_cap = 0;            // chunk slots per (sequence, KV head) in decode partials

  // ---- persistent workspace (device) ----
  float* score_pre = nullptr;    // [L][B][Hkv][npad]   cumulative prompt scores per key
  double* head_var = nullptr;    // [L][B][Hq]          per-query-head variance of column sums
  double* layer_F = nullptr;     // [L][B]              density statistic
  void* cacheK = nullptr;        // [B][Hkv][slots][d]
  void* cacheV = nullptr;        // [B][Hkv][slots][d]
  int8_t* cKe = nullptr;         // [B][Hkv][slots] fp8 cache: the power of two of every K row
  int8_t* cVe = nullptr;         // [B][Hkv][slots] the same for V
  int32_t* meta_stage = nullptr; // [L][B][Hkv][4] fp8 cache: `meta` with base 0, the geometry of the bf16 staging rows
  double* cscore = nullptr;      // [B][Hkv][slots]
  int32_t* cpos = nullptr;       // [B][Hkv][slots]
  int32_t* ccount = nullptr;     // [L][B][Hkv]
  int32_t* ctotal = nullptr;     // [L][B][Hkv] entries of the running decode step (count + 1), fixed for the whole step
  double* ctau = nullptr;        // [L][B][Hkv]
  int32_t* meta = nullptr;       // [L][B][Hkv][4]
  int32_t* ev_evicted = nullptr; // [L][B][Hkv]
  int32_t* ev_target = nullptr;  // [L][B][Hkv]
  double* ev_ustar = nullptr;    // [L][B][Hkv]
  int32_t* ccand = nullptr;      // [L][B][Hkv][decode_candidates()] eviction candidates (slots, -1 none)
  uint32_t* cticket = nullptr;   // [L][B][Hkv] chunk counter of the running decode step (0 between steps)
  uint32_t* cmiss = nullptr;     // [L][B][Hkv] evictions of a token outside the predicted candidates, since the last reset

  // ---- scratch workspace (device) ----
  // prefill attention
  float* lse = nullptr;          // [B][Hq][npad]   row log-sum-exp (natural log, scaled logits)
  void* vt = nullptr;            // [B][Hkv][npad/64][d][64] transposed values, tile by tile, as scaled fp16 (bf16 path)
  uint32_t* vmax_bits = nullptr; // [B][Hkv] bit pattern of max |v|
  float* vt_unscale = nullptr;   // [B][Hkv] power of two that undoes the fp16 scaling
  double* varpart = nullptr;     // [B][Hq][npad/128][2] partial sums of s and s^2
  // token-level prefill stages, all [B][Hkv][npad] unless noted
  int32_t* sel_ret = nullptr;    // retained positions, ascending
  int32_t* sel_evi = nullptr;    // evicted positions, ascending
  int32_t* sel_cnt = nullptr;    // [B][Hkv][2]  n_ret, n_evi
  float* invnorm = nullptr;      // 1/|k_j| of every prompt key (fp32, filter only)
  int32_t* m_cand = nullptr;     // filter's best retained rank per evicted row; bit 31 = ambiguous
  float* m_thr = nullptr;        // filter's acceptance threshold of a flagged row
  int32_t* amb_list = nullptr;   // flagged evicted ranks, ascending
  int32_t* amb_cnt = nullptr;    // [B][Hkv]
  int32_t* m_ncand = nullptr;    // candidates collected for a flagged row
  int32_t* m_clist = nullptr;    // [..][npad][8] their retained ranks
  double* m_ustar = nullptr;     // exact best similarity per evicted row
  int32_t* m_tgt = nullptr;      // exact match (retained rank)
  uint8_t* m_pass = nullptr;     // threshold test
  int32_t* g_cnt = nullptr;      // [..][npad+1] sources per retained slot
  int32_t* g_off = nullptr;      // [..][npad+1] exclusive prefix of g_cnt
  int32_t* g_cur = nullptr;      // [..][npad+1] fill cursors
  int32_t* g_src = nullptr;      // evicted ranks grouped by target (unordered inside a group)
  // fp8 cache: the bf16 rows of the layer being compressed (the prompt-phase kernels work on
  // them; encode_layer then writes the cache) and of a head being imported or exported
  void* st_K = nullptr;          // [B][Hkv][npad][d]
  void* st_V = nullptr;          // [B][Hkv][npad][d]
  // multi-token append: the cache in ascending token position (block-level Eq. 7-12 run on it)
  void* app_K = nullptr;         // [B][Hkv][npad][d]
  void* app_V = nullptr;         // [B][Hkv][npad][d]
  double* app_score = nullptr;   // [B][Hkv][npad] cumulative scores, fp64
  int32_t* app_pos = nullptr;    // [B][Hkv][npad] token positions, ascending
  int32_t* app_rank = nullptr;   // [B][Hkv][npad] rank of every cache slot's position
  int32_t* app_n = nullptr;      // [B][Hkv] entries
  // block attention of d2o_append_chunk (contexts with max_append > 1)
  int32_t ap_maxq = 0, ap_nch = 0;  // queries per head (max_append * G, rounded up to 16) and chunks per head the arrays hold
  double* ap_q = nullptr;        // [B][Hkv][ap_maxq][d] the block's queries as fp64
  double* ap_stat = nullptr;     // [ap_nch][B][Hkv][ap_maxq][2] per chunk: softmax maximum and exp-sum of every query
  double* ap_norm = nullptr;     // [B][Hkv][ap_maxq][2] maximum and normaliser of every query
  float* ap_out = nullptr;       // [ap_nch][B][Hkv][ap_maxq][d] partial outputs per chunk
  double* ap_spart = nullptr;    // [kMaxQuerySlices][B][Hkv][ap_nch * 256] per row: sum of the slice's probabilities
  // decode
  double* d_logit = nullptr;     // [nchunk][B][Hkv][G][256] exp(logit - sub-chunk max), chunk-major
  double* d_rec = nullptr;       // [nchunk][B][Hkv][4][32] per 64 slots: softmax maxima and sums, candidates' best cosine and slot
  double* d_part = nullptr;      // [nchunk][B][Hkv][kPartRecDoubles] records of the split closing kernels (one per part, at its first chunk)
  float* d_pacc = nullptr;       // [nchunk][B][Hkv][4][G][d] partial outputs
  double* d_vecs = nullptr;      // [L][B][Hkv][G + candidates][d] queries and candidate keys, fp64
  double* d_cnorm = nullptr;     // [L][B][Hkv][candidates] norms of the candidate keys
};

namespace d2o {

int fail(d2o_ctx* ctx, int code, const std::string& msg);

#define D2O_HIP_CHECK(ctx, expr)                                                        \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess)                                                               \
      return d2o::fail(ctx, D2O_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

// Brackets the launches made during its lifetime with two events when timing is enabled.
struct KernelTimer {
  d2o_ctx* c;
  hipStream_t s;
  bool on;
  d2o_timed_launch t;
  KernelTimer(d2o_ctx* ctx, int id, hipStream_t stream) : c(ctx), s(stream), on(ctx->timing > 0) {
    if (on && (id == D2O_K_DECODE_ATTEND || id == D2O_K_DECODE_PREPARE)) on = ctx->launch_no[id]++ % ctx->timing == ctx->timing - 1;
    if (!on) return;
    t.id = id;
    if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(t.start, s);
  }
  ~KernelTimer() {
    if (!on) return;
    (void)hipEventRecord(t.stop, s);
    c->timed.push_back(t);
  }
};

// ---- kernel launchers (one per stage), defined in the .hip files ----
hipError_t launch_prefill_f32(d2o_ctx* c, int layer, View Q, View K, View V, View O, int n,
                              hipStream_t s);
hipError_t launch_prefill_bf16(d2o_ctx* c, int layer, View Q, View K, View V, View O, int n,
                               hipStream_t s);
hipError_t launch_density(d2o_ctx* c, int layer, int n, hipStream_t s);
// append = true: the stages run on the position-ordered copy of the cache (app_*): fp64 scores,
// per-head entry counts, positions through app_pos, EMA form of the threshold
hipError_t launch_select(d2o_ctx* c, int layer, int n, hipStream_t s, bool append = false);
hipError_t launch_gather(d2o_ctx* c, int layer, View K, View V, int n, hipStream_t s, bool append = false);
hipError_t launch_match(d2o_ctx* c, int layer, View K, int n, hipStream_t s);
hipError_t launch_threshold_group(d2o_ctx* c, int layer, int n, hipStream_t s, bool append = false);
hipError_t launch_cache_sort(d2o_ctx* c, int layer, hipStream_t s);  // cache -> app_* in ascending position
// A block of m tokens: rows appended, attention and Eq. 6 for every token of the block, nothing evicted.
hipError_t launch_block_attend(d2o_ctx* c, int layer, View q, View k, View v, View out, int m, int first_pos,
                               hipStream_t s);
hipError_t launch_merge(d2o_ctx* c, int layer, View K, View V, int n, hipStream_t s);
// Where the prompt-phase kernels (compaction, matching, merge) keep a layer's cache rows: in the
// cache itself, or - fp8 cache - in bf16 staging rows [B][Hkv][npad][d] that encode_layer turns
// into cache rows once the layer's merges are done.
inline void* prompt_rows_K(const d2o_ctx* c) { return c->cfg.cache_fp8 ? c->st_K : c->cacheK; }
inline void* prompt_rows_V(const d2o_ctx* c) { return c->cfg.cache_fp8 ? c->st_V : c->cacheV; }
inline int64_t prompt_rows_stride(const d2o_ctx* c) { return c->cfg.cache_fp8 ? c->npad : c->cfg.slots_per_seq; }
inline const int32_t* prompt_rows_meta(const d2o_ctx* c, int layer) {
  return (c->cfg.cache_fp8 ? c->meta_stage : c->meta) + size_t(layer) * c->cfg.batch * c->cfg.n_kv_heads * 4;
}
// fp8 cache: staging rows of a layer -> cache rows (all heads), and one head's rows either way
hipError_t launch_encode_layer(d2o_ctx* c, int layer, hipStream_t s);
hipError_t launch_encode_head(d2o_ctx* c, int layer, int b, int hk, int count, hipStream_t s);  // staging -> cache
hipError_t launch_decode_head(d2o_ctx* c, int layer, int b, int hk, int count, hipStream_t s);  // cache -> staging
// static_scratch: nullptr = the context's scratch workspace; otherwise the device address of the
// library's static scratch array, which then holds the step's partial results and operands
hipError_t launch_decode(d2o_ctx* c, int layer0, int nl, View q, View k, View v, View out,
                         int new_pos, hipStream_t s, unsigned char* static_scratch = nullptr);
hipError_t static_scratch_address(unsigned char** out);  // per device; first call per device looks it up
size_t decode_static_scratch_need(const d2o_ctx* c);     // bytes of it a decode step of this context uses
size_t decode_static_scratch_capacity();
int decode_candidates();  // eviction candidates tracked per (layer, sequence, KV head)
hipError_t launch_init_candidates(d2o_ctx* c, int layer, int new_pos, hipStream_t s);
hipError_t launch_write_meta(d2o_ctx* c, int layer, hipStream_t s);  // the layer's host meta -> device, by a kernel

}  // namespace d2o
