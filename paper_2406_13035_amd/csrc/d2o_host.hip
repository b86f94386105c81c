// Host side of libd2o: context, workspace layout, argument checks, stage sequencing and the
// host-only budget allocation.  All device arithmetic lives in the kernel files.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <numeric>

#include "d2o_internal.h"

namespace d2o {

int fail(d2o_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg;
  return code;
}

namespace {

// Walks the workspace layout; with base == nullptr it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  template <typename T>
  void take(T*& field, size_t count) {
    off = (off + 255) & ~size_t(255);
    field = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
  }
  void take_raw(void*& field, size_t bytes) {
    off = (off + 255) & ~size_t(255);
    field = base ? static_cast<void*>(base + off) : nullptr;
    off += bytes;
  }
};

int check_config(const d2o_config* c) {
  if (!c) return D2O_ERR_INVALID_ARG;
  if (c->batch < 1 || c->n_layers < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return D2O_ERR_INVALID_ARG;
  if (c->n_q_heads % c->n_kv_heads) return D2O_ERR_INVALID_ARG;
  if (c->max_prompt_len < 1 || c->slots_per_seq < 2 || c->n_sink < 0) return D2O_ERR_INVALID_ARG;
  if (!(c->beta >= 0.0 && c->beta < 1.0)) return D2O_ERR_INVALID_ARG;
  if (c->dtype == D2O_BF16) {
    if (c->head_dim != 128) return D2O_ERR_UNSUPPORTED;
  } else if (c->dtype == D2O_F32) {
    if (c->head_dim != 64 && c->head_dim != 128) return D2O_ERR_UNSUPPORTED;
  } else {
    return D2O_ERR_UNSUPPORTED;
  }
  const int G = c->n_q_heads / c->n_kv_heads;  // the decode kernels are built for these group sizes
  if ((G != 1 && G != 2 && G != 4 && G != 8) || c->n_q_heads > 256) return D2O_ERR_UNSUPPORTED;
  if (c->out_f32 != 0 && c->out_f32 != 1) return D2O_ERR_INVALID_ARG;
  if (c->merge_average != 0 && c->merge_average != 1) return D2O_ERR_INVALID_ARG;
  if (c->max_append < 0 || c->max_append >= c->max_prompt_len) return D2O_ERR_INVALID_ARG;
  if (c->split_rows != 0 && c->split_rows < 256) return D2O_ERR_INVALID_ARG;
  if (c->cache_fp8 != 0 && c->cache_fp8 != 1) return D2O_ERR_INVALID_ARG;
  if (c->cache_fp8 && c->dtype != D2O_BF16) return D2O_ERR_UNSUPPORTED;
  return D2O_OK;
}

void layout(d2o_ctx* x, char* persistent, char* scratch, size_t* pbytes, size_t* sbytes) {
  const d2o_config& c = x->cfg;
  const size_t B = c.batch, L = c.n_layers, Hq = c.n_q_heads, Hkv = c.n_kv_heads, d = c.head_dim;
  const size_t slots = c.slots_per_seq, es = x->esize, np = x->npad, G = Hq / Hkv;
  const size_t nch = x->nchunk_cap;
  Carver p{persistent};
  p.take(x->score_pre, L * B * Hkv * np);
  p.take(x->head_var, L * B * Hq);
  p.take(x->layer_F, L * B);
  const size_t f8 = c.cache_fp8 ? 1 : 0;
  p.take_raw(x->cacheK, B * Hkv * slots * d * x->csize);
  p.take_raw(x->cacheV, B * Hkv * slots * d * x->csize);
  p.take(x->cKe, f8 * B * Hkv * slots);
  p.take(x->cVe, f8 * B * Hkv * slots);
  p.take(x->meta_stage, f8 * L * B * Hkv * 4);
  p.take(x->cscore, B * Hkv * slots);
  p.take(x->cpos, B * Hkv * slots);
  p.take(x->ccount, L * B * Hkv);
  p.take(x->ctotal, L * B * Hkv);
  p.take(x->ctau, L * B * Hkv);
  p.take(x->meta, L * B * Hkv * 4);
  p.take(x->ev_evicted, L * B * Hkv);
  p.take(x->ev_target, L * B * Hkv);
  p.take(x->ev_ustar, L * B * Hkv);
  const size_t nc = decode_candidates();
  p.take(x->ccand, L * B * Hkv * nc);
  p.take(x->cticket, L * B * Hkv);
  p.take(x->cmiss, L * B * Hkv);
  *pbytes = (p.off + 255) & ~size_t(255);

  Carver s{scratch};
  s.take(x->lse, B * Hq * np);
  s.take_raw(x->vt, c.dtype == D2O_BF16 ? B * Hkv * d * np * es : 0);
  s.take(x->vmax_bits, B * Hkv);
  s.take(x->vt_unscale, B * Hkv);
  s.take(x->varpart, B * Hq * (np / 128) * 2);
  const size_t bh = B * Hkv;
  s.take(x->sel_ret, bh * np);
  s.take(x->sel_evi, bh * np);
  s.take(x->sel_cnt, bh * 2);
  s.take(x->invnorm, bh * np);
  s.take(x->m_cand, bh * np);
  s.take(x->m_thr, bh * np);
  s.take(x->amb_list, bh * np);
  s.take(x->amb_cnt, bh);
  s.take(x->m_ncand, bh * np);
  s.take(x->m_clist, bh * np * 8);
  s.take(x->m_ustar, bh * np);
  s.take(x->m_tgt, bh * np);
  s.take(x->m_pass, bh * np);
  s.take(x->g_cnt, bh * (np + 1));
  s.take(x->g_off, bh * (np + 1));
  s.take(x->g_cur, bh * (np + 1));
  s.take(x->g_src, bh * np);
  const size_t ap = c.max_append > 1 ? 1 : 0;  // the position-ordered copy exists only when blocks can be appended
  s.take_raw(x->st_K, f8 * bh * np * d * es);
  s.take_raw(x->st_V, f8 * bh * np * d * es);
  s.take_raw(x->app_K, ap * bh * np * d * es);
  s.take_raw(x->app_V, ap * bh * np * d * es);
  s.take(x->app_score, ap * bh * np);
  s.take(x->app_pos, ap * bh * np);
  s.take(x->app_rank, ap * bh * np);
  s.take(x->app_n, ap * bh);
  x->ap_maxq = ap ? int((size_t(c.max_append) * G + 15) / 16 * 16) : 0;
  x->ap_nch = ap ? int(std::min<int64_t>(np, c.slots_per_seq) / kChunk + 2) : 0;
  s.take(x->ap_q, ap * bh * x->ap_maxq * d);
  s.take(x->ap_stat, ap * x->ap_nch * bh * x->ap_maxq * 2);
  s.take(x->ap_norm, ap * bh * x->ap_maxq * 2);
  s.take(x->ap_out, ap * x->ap_nch * bh * x->ap_maxq * d);
  s.take(x->ap_spart, ap * kMaxQuerySlices * bh * x->ap_nch * kChunk);
  s.take(x->d_logit, nch * B * Hq * kChunk);
  const size_t nsub = nch * 4;  // partial results are kept per 64 slots, a quarter of a chunk
  s.take(x->d_rec, bh * nsub * 32);
  s.take(x->d_pacc, bh * nsub * G * d);
  s.take(x->d_part, bh * nch * kPartRecDoubles + L * bh * 16);  // part records, then 16 doubles per head
  s.take(x->d_vecs, L * bh * (G + nc) * d);
  s.take(x->d_cnorm, L * bh * nc);

  *sbytes = (s.off + 255) & ~size_t(255);
}

void init_sizes(d2o_ctx* x) {
  x->esize = x->cfg.dtype == D2O_BF16 ? 2 : 4;
  x->csize = x->cfg.cache_fp8 ? 1 : x->esize;
  x->npad = (x->cfg.max_prompt_len + 127) / 128 * 128;
  x->grow = std::max(1, x->cfg.max_append);
  x->nchunk_cap = x->cfg.slots_per_seq / kChunk + x->cfg.n_layers + 1;
}

bool view_ok(const d2o_ctx* x, const d2o_view& v, int esize = 0) {
  const int64_t al = 16 / (esize ? esize : x->esize);  // 16-byte vector loads
  if (!v.ptr || (reinterpret_cast<uintptr_t>(v.ptr) & 15)) return false;
  return v.stride_b % al == 0 && v.stride_h % al == 0 && v.stride_n % al == 0 && v.stride_n >= 0;
}

// budget, recent: [B][Hkv] when per_head, else [B] (every KV head of a sequence alike)
int reserve_layer(d2o_ctx* x, int32_t layer, int32_t n, const int32_t* budget_in, const int32_t* recent_in,
                  bool per_head = false) {
  const d2o_config& c = x->cfg;
  LayerState& st = x->layers[layer];
  const int nbh = c.batch * c.n_kv_heads;
  std::vector<LayerMeta> meta(nbh);
  std::vector<int32_t> budget(nbh), recent(nbh);
  for (int i = 0; i < nbh; ++i) {
    budget[i] = budget_in[per_head ? i : i / c.n_kv_heads];
    recent[i] = recent_in[per_head ? i : i / c.n_kv_heads];
  }
  for (int b = 0; b < nbh; ++b) {
    if (budget[b] < 1 || recent[b] < 0 || budget[b] < c.n_sink + recent[b])
      return fail(x, D2O_ERR_INVALID_ARG, "budget must be >= 1 and >= n_sink + recent");
    if (n < c.n_sink) return fail(x, D2O_ERR_INVALID_ARG, "prompt shorter than the sink tokens");
    const int64_t need = int64_t(budget[b]) + x->grow;
    if (c.max_append > 1 && int64_t(budget[b]) + c.max_append > x->npad)
      return fail(x, D2O_ERR_CAPACITY, "budget + max_append exceeds max_prompt_len (rounded up to 128)");
    if (c.cache_fp8 && int64_t(budget[b]) + 1 > x->npad)
      return fail(x, D2O_ERR_CAPACITY, "fp8 cache: budget + 1 exceeds max_prompt_len (rounded up to 128), the rows the staging area holds");
    if (x->used_slots[b] + need > c.slots_per_seq)
      return fail(x, D2O_ERR_CAPACITY, "slots_per_seq too small for the layer budgets");
    meta[b].base = int32_t(x->used_slots[b]);
    meta[b].budget = budget[b];
    meta[b].recent = recent[b];
    meta[b].chunk_base = int32_t(x->used_chunks[b]);
  }
  for (int b = 0; b < nbh; ++b) {
    x->used_slots[b] += int64_t(budget[b]) + x->grow;
    x->used_chunks[b] += (int64_t(budget[b]) + x->grow + kChunk - 1) / kChunk;
  }
  st.meta = meta;
  st.n = n;
  st.next_pos = n;
  return D2O_OK;
}

// Fill of 32-bit words by a kernel: the state reset below may be part of a caller's captured
// graph, where memset nodes are not reliable.
__global__ void fill_words(uint32_t* p, uint32_t v, size_t n) {
  for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += size_t(gridDim.x) * blockDim.x) p[i] = v;
}
hipError_t fill32(void* p, uint32_t v, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  const unsigned blocks = unsigned(std::min<size_t>((n + 255) / 256, 1024));
  fill_words<<<blocks, 256, 0, s>>>(static_cast<uint32_t*>(p), v, n);
  return hipGetLastError();
}

// The per-sequence geometry of one layer travels to the device as kernel arguments (up to
// kMetaPerLaunch sequences per launch): no host buffer has to outlive the call, so the caller's
// stream is neither synchronised nor fed from pageable memory.
constexpr int kMetaPerLaunch = 16;
struct MetaPack {
  int32_t v[kMetaPerLaunch * 4];
};
__global__ void write_meta_kernel(int32_t* dst, MetaPack m, int n_words) {
  const int i = threadIdx.x;
  if (i < n_words) dst[i] = m.v[i];
}

}  // namespace

hipError_t launch_write_meta(d2o_ctx* x, int layer, hipStream_t s) {
  const LayerState& st = x->layers[layer];
  const int B = x->cfg.batch * x->cfg.n_kv_heads;  // one entry per (sequence, KV head)
  for (int b0 = 0; b0 < B; b0 += kMetaPerLaunch) {
    const int nb = std::min(kMetaPerLaunch, B - b0);
    MetaPack m;
    for (int i = 0; i < nb; ++i) {
      const LayerMeta& t = st.meta[b0 + i];
      m.v[4 * i + 0] = t.base;
      m.v[4 * i + 1] = t.budget;
      m.v[4 * i + 2] = t.recent;
      m.v[4 * i + 3] = t.chunk_base;
    }
    write_meta_kernel<<<1, kMetaPerLaunch * 4, 0, s>>>(x->meta + (size_t(layer) * B + b0) * 4, m, nb * 4);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (x->cfg.cache_fp8) {  // the staging rows of a head start at row 0
      for (int i = 0; i < nb; ++i) m.v[4 * i + 0] = 0;
      write_meta_kernel<<<1, kMetaPerLaunch * 4, 0, s>>>(x->meta_stage + (size_t(layer) * B + b0) * 4, m, nb * 4);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

}  // namespace d2o

using namespace d2o;

extern "C" {

int d2o_workspace_bytes(const d2o_config* cfg, size_t* persistent, size_t* scratch) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!persistent || !scratch) return D2O_ERR_INVALID_ARG;
  d2o_ctx tmp;
  tmp.cfg = *cfg;
  init_sizes(&tmp);
  layout(&tmp, nullptr, nullptr, persistent, scratch);
  return D2O_OK;
}

int d2o_create(const d2o_config* cfg, void* persistent_dev, size_t persistent_bytes,
               void* scratch_dev, size_t scratch_bytes, void* stream, d2o_ctx** out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!persistent_dev || !scratch_dev || !out) return D2O_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(persistent_dev) | reinterpret_cast<uintptr_t>(scratch_dev)) & 255)
    return D2O_ERR_INVALID_ARG;
  d2o_ctx* x = new d2o_ctx;
  x->cfg = *cfg;
  init_sizes(x);
  size_t pb = 0, sb = 0;
  layout(x, static_cast<char*>(persistent_dev), static_cast<char*>(scratch_dev), &pb, &sb);
  if (pb > persistent_bytes || sb > scratch_bytes) {
    delete x;
    return D2O_ERR_CAPACITY;
  }
  x->layers.assign(cfg->n_layers, LayerState{});
  x->used_slots.assign(size_t(cfg->batch) * cfg->n_kv_heads, 0);
  x->used_chunks.assign(size_t(cfg->batch) * cfg->n_kv_heads, 0);
  rc = d2o_reset(x, stream);
  if (rc) {
    delete x;
    return rc;
  }
  // set-up time is when this device's address of the static scratch array is looked up
  // (d2o_decode_step_static then finds it cached and makes no runtime query of its own)
  unsigned char* stat = nullptr;
  if (static_scratch_address(&stat) != hipSuccess) {
    delete x;
    return D2O_ERR_HIP;
  }
  *out = x;
  return D2O_OK;
}

void d2o_destroy(d2o_ctx* ctx) {
  if (!ctx) return;
  for (auto& t : ctx->timed) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  delete ctx;
}

const char* d2o_last_error(const d2o_ctx* ctx) { return ctx ? ctx->err.c_str() : ""; }

int d2o_reset(d2o_ctx* x, void* stream) {
  if (!x) return D2O_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const d2o_config& c = x->cfg;
  const size_t lbh = size_t(c.n_layers) * c.batch * c.n_kv_heads;
  // Only the small per-head state needs defined contents; 0xFF bytes read as NaN / -1.
  D2O_HIP_CHECK(x, fill32(x->layer_F, 0xFFFFFFFFu, sizeof(double) * c.n_layers * c.batch, s));
  D2O_HIP_CHECK(x, fill32(x->head_var, 0xFFFFFFFFu, sizeof(double) * c.n_layers * c.batch * c.n_q_heads, s));
  D2O_HIP_CHECK(x, fill32(x->ccount, 0u, sizeof(int32_t) * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->ctotal, 0u, sizeof(int32_t) * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->ctau, 0xFFFFFFFFu, sizeof(double) * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->meta, 0u, sizeof(int32_t) * 4 * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->ev_evicted, 0xFFFFFFFFu, sizeof(int32_t) * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->ev_target, 0xFFFFFFFFu, sizeof(int32_t) * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->ev_ustar, 0xFFFFFFFFu, sizeof(double) * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->ccand, 0xFFFFFFFFu, sizeof(int32_t) * lbh * decode_candidates(), s));
  D2O_HIP_CHECK(x, fill32(x->cticket, 0u, sizeof(uint32_t) * lbh, s));
  D2O_HIP_CHECK(x, fill32(x->cmiss, 0u, sizeof(uint32_t) * lbh, s));
  for (auto& l : x->layers) l = LayerState{};
  std::fill(x->used_slots.begin(), x->used_slots.end(), 0);
  std::fill(x->used_chunks.begin(), x->used_chunks.end(), 0);
  x->last_compress_layer = -1;
  x->last_append_layer = -1;
  return D2O_OK;
}

int d2o_prefill_attend(d2o_ctx* x, int32_t layer, d2o_view Q, d2o_view K, d2o_view V, int32_t n,
                       d2o_view O, void* stream) {
  if (!x) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(x, D2O_ERR_INVALID_ARG, "layer out of range");
  if (n < 1 || n > c.max_prompt_len) return fail(x, D2O_ERR_INVALID_ARG, "n out of range");
  if (!view_ok(x, Q) || !view_ok(x, K) || !view_ok(x, V) || (O.ptr && !view_ok(x, O, x->cfg.out_f32 ? 4 : 0)))
    return fail(x, D2O_ERR_INVALID_ARG, "null, misaligned or badly strided tensor view");
  if (Q.stride_n < c.head_dim || K.stride_n < c.head_dim || V.stride_n < c.head_dim ||
      (O.ptr && O.stride_n < c.head_dim))
    return fail(x, D2O_ERR_INVALID_ARG, "token stride smaller than head_dim");
  LayerState& st = x->layers[layer];
  if (st.phase == kReady) return fail(x, D2O_ERR_STATE, "layer already compressed");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = c.dtype == D2O_BF16
                     ? launch_prefill_bf16(x, layer, to_view(Q), to_view(K), to_view(V), to_view(O), n, s)
                     : launch_prefill_f32(x, layer, to_view(Q), to_view(K), to_view(V), to_view(O), n, s);
  if (e != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("prefill attention: ") + hipGetErrorString(e));
  e = launch_density(x, layer, n, s);
  if (e != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("density: ") + hipGetErrorString(e));
  st.phase = kAttended;
  st.n = n;
  return D2O_OK;
}

int d2o_get_density(d2o_ctx* x, double* F_layers, double* F_heads, void* stream) {
  if (!x || !F_layers) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::vector<double> lf(size_t(c.n_layers) * c.batch), hv(size_t(c.n_layers) * c.batch * c.n_q_heads);
  D2O_HIP_CHECK(x, hipMemcpyAsync(lf.data(), x->layer_F, lf.size() * sizeof(double), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(hv.data(), x->head_var, hv.size() * sizeof(double), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  for (int b = 0; b < c.batch; ++b)
    for (int l = 0; l < c.n_layers; ++l) {
      F_layers[size_t(b) * c.n_layers + l] = lf[size_t(l) * c.batch + b];
      if (F_heads)
        for (int h = 0; h < c.n_q_heads; ++h)
          F_heads[(size_t(b) * c.n_layers + l) * c.n_q_heads + h] = hv[(size_t(l) * c.batch + b) * c.n_q_heads + h];
    }
  return D2O_OK;
}

// Sec. 4.1 Eq. 5 with the clipping and integer rules stated in d2o.h.
int d2o_allocate_budgets(const double* F, int32_t L, int32_t seq_len, int64_t total, int32_t min_budget,
                         int32_t* S_out) {
  return d2o_allocate_budgets_policy(D2O_ALLOC_SOFTMAX, F, L, seq_len, total, min_budget, S_out);
}

int d2o_allocate_budgets_policy(int32_t policy, const double* F, int32_t L, int32_t seq_len, int64_t total,
                                int32_t min_budget, int32_t* S_out) {
  if (!F || !S_out || L < 1 || seq_len < 1 || min_budget < 0) return D2O_ERR_INVALID_ARG;
  if (policy < D2O_ALLOC_SOFTMAX || policy > D2O_ALLOC_UNIFORM) return D2O_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l)
    if (!std::isfinite(F[l]) || (policy == D2O_ALLOC_RECIPROCAL && !(F[l] > 0.0))) return D2O_ERR_INVALID_ARG;
  if (policy == D2O_ALLOC_EXP_DECAY) {  // the layer's own ratio, no sum constraint
    if (min_budget > seq_len) return D2O_ERR_INVALID_ARG;
    for (int l = 0; l < L; ++l) {
      const double v = std::floor(std::exp(-F[l]) * double(seq_len));
      S_out[l] = v < double(min_budget) ? min_budget : v > double(seq_len) ? seq_len : int32_t(v);
    }
    return D2O_OK;
  }
  if (total < int64_t(L) * min_budget || total > int64_t(L) * seq_len) return D2O_ERR_INVALID_ARG;
  std::vector<char> pinned(L, 0);
  std::vector<double> share(L, 0.0), w(L, 0.0);
  int64_t remaining = total;
  const double hi = double(seq_len), lo = double(min_budget);
  for (;;) {
    double fmin = std::numeric_limits<double>::infinity();
    int nfree = 0;
    for (int l = 0; l < L; ++l)
      if (!pinned[l]) {
        fmin = std::min(fmin, F[l]);
        ++nfree;
      }
    if (!nfree) break;
    double wsum = 0.0;
    for (int l = 0; l < L; ++l)
      if (!pinned[l]) {
        w[l] = policy == D2O_ALLOC_SOFTMAX ? std::exp(-(F[l] - fmin)) : policy == D2O_ALLOC_RECIPROCAL ? 1.0 / F[l] : 1.0;
        wsum += w[l];
      }
    double excess = 0.0, deficit = 0.0;
    int nover = 0, nunder = 0;
    for (int l = 0; l < L; ++l)
      if (!pinned[l]) {
        share[l] = double(remaining) * (w[l] / wsum);
        if (share[l] > hi) {
          excess += share[l] - hi;
          ++nover;
        }
      }
    for (int l = 0; l < L; ++l)
      if (!pinned[l] && share[l] < lo) {
        deficit += lo - share[l];
        ++nunder;
      }
    if (!nover && !nunder) break;
    if (nover && excess >= deficit) {
      for (int l = 0; l < L; ++l)
        if (!pinned[l] && share[l] > hi) {
          pinned[l] = 1;
          S_out[l] = seq_len;
          remaining -= seq_len;
        }
    } else {
      for (int l = 0; l < L; ++l)
        if (!pinned[l] && share[l] < lo) {
          pinned[l] = 1;
          S_out[l] = min_budget;
          remaining -= min_budget;
        }
    }
  }
  std::vector<int> free_layers;
  int64_t given = 0;
  for (int l = 0; l < L; ++l)
    if (!pinned[l]) {
      S_out[l] = int32_t(std::floor(share[l]));
      given += S_out[l];
      free_layers.push_back(l);
    }
  int64_t left = remaining - given;
  std::stable_sort(free_layers.begin(), free_layers.end(), [&](int a, int b) {
    return (share[a] - std::floor(share[a])) > (share[b] - std::floor(share[b]));
  });
  for (size_t t = 0; left > 0 && !free_layers.empty(); ++t) {
    int l = free_layers[t % free_layers.size()];
    if (S_out[l] < seq_len) {
      ++S_out[l];
      --left;
    }
  }
  return D2O_OK;
}

int d2o_scores_import(d2o_ctx* x, int32_t layer, const float* scores, int32_t n, void* stream) {
  if (!x || !scores) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers || n < 1 || n > c.max_prompt_len)
    return fail(x, D2O_ERR_INVALID_ARG, "layer or n out of range");
  LayerState& st = x->layers[layer];
  if (st.phase == kReady) return fail(x, D2O_ERR_STATE, "layer already compressed");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t bh = size_t(c.batch) * c.n_kv_heads;
  float* dst = x->score_pre + size_t(layer) * bh * x->npad;
  D2O_HIP_CHECK(x, hipMemcpy2DAsync(dst, sizeof(float) * x->npad, scores, sizeof(float) * n,
                                    sizeof(float) * n, bh, hipMemcpyHostToDevice, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  st.phase = kAttended;
  st.n = n;
  return D2O_OK;
}

int d2o_scores_export(d2o_ctx* x, int32_t layer, float* scores, int32_t n, void* stream) {
  if (!x || !scores) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers || n < 1 || n > c.max_prompt_len)
    return fail(x, D2O_ERR_INVALID_ARG, "layer or n out of range");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t bh = size_t(c.batch) * c.n_kv_heads;
  const float* src = x->score_pre + size_t(layer) * bh * x->npad;
  D2O_HIP_CHECK(x, hipMemcpy2DAsync(scores, sizeof(float) * n, src, sizeof(float) * x->npad,
                                    sizeof(float) * n, bh, hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  return D2O_OK;
}

int d2o_layer_reserve(d2o_ctx* x, int32_t layer, int32_t n, const int32_t* budget, const int32_t* recent) {
  if (!x || !budget || !recent) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers || n < 1) return fail(x, D2O_ERR_INVALID_ARG, "layer or n out of range");
  LayerState& st = x->layers[layer];
  if (st.phase == kReady) return fail(x, D2O_ERR_STATE, "layer already reserved");
  int rc = reserve_layer(x, layer, n, budget, recent);
  if (rc) return rc;
  // no stream argument: the metadata goes out on the default stream and the call waits for it
  hipError_t e = launch_write_meta(x, layer, nullptr);
  if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  if (e != hipSuccess) return fail(x, D2O_ERR_HIP, hipGetErrorString(e));
  st.phase = kReady;
  return D2O_OK;
}

static int compress_layer_impl(d2o_ctx* x, int32_t layer, d2o_view K, d2o_view V, int32_t n,
                               const int32_t* budget, const int32_t* recent, bool per_head, void* stream) {
  if (!x || !budget || !recent) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(x, D2O_ERR_INVALID_ARG, "layer out of range");
  LayerState& st = x->layers[layer];
  if (st.phase == kEmpty) return fail(x, D2O_ERR_STATE, "layer has no scores: call d2o_prefill_attend first");
  if (st.phase == kReady) return fail(x, D2O_ERR_STATE, "layer already compressed");
  if (n != st.n) return fail(x, D2O_ERR_INVALID_ARG, "n differs from the attention call");
  if (!view_ok(x, K) || !view_ok(x, V) || K.stride_n < c.head_dim || V.stride_n < c.head_dim)
    return fail(x, D2O_ERR_INVALID_ARG, "null, misaligned or badly strided tensor view");
  int rc = reserve_layer(x, layer, n, budget, recent, per_head);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if ((e = launch_write_meta(x, layer, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("meta: ") + hipGetErrorString(e));
  if ((e = launch_select(x, layer, n, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("select: ") + hipGetErrorString(e));
  if ((e = launch_gather(x, layer, to_view(K), to_view(V), n, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("gather: ") + hipGetErrorString(e));
  if ((e = launch_match(x, layer, to_view(K), n, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("match: ") + hipGetErrorString(e));
  if ((e = launch_threshold_group(x, layer, n, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("threshold: ") + hipGetErrorString(e));
  if ((e = launch_merge(x, layer, to_view(K), to_view(V), n, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("merge: ") + hipGetErrorString(e));
  if (c.cache_fp8 && (e = launch_encode_layer(x, layer, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("encode: ") + hipGetErrorString(e));
  if ((e = launch_init_candidates(x, layer, st.next_pos, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("candidates: ") + hipGetErrorString(e));
  // (a failed launch leaves the layer's slots reserved but the layer not ready: d2o_reset recovers)
  st.phase = kReady;
  x->last_compress_layer = layer;
  return D2O_OK;
}

int d2o_compress_layer(d2o_ctx* x, int32_t layer, d2o_view K, d2o_view V, int32_t n, const int32_t* budget,
                       const int32_t* recent, void* stream) {
  return compress_layer_impl(x, layer, K, V, n, budget, recent, false, stream);
}

int d2o_compress_layer_heads(d2o_ctx* x, int32_t layer, d2o_view K, d2o_view V, int32_t n, const int32_t* budget,
                             const int32_t* recent, void* stream) {
  return compress_layer_impl(x, layer, K, V, n, budget, recent, true, stream);
}

// App. A.8: Eq. 5 over all (layer, KV head) pairs; a KV head's statistic is the mean of the
// variances of the query heads it serves.
int d2o_allocate_budgets_heads(const double* F_heads, int32_t L, int32_t Hq, int32_t Hkv, int32_t seq_len,
                               int64_t total, int32_t min_budget, int32_t* S_out) {
  if (!F_heads || !S_out || L < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv) return D2O_ERR_INVALID_ARG;
  const int G = Hq / Hkv;
  std::vector<double> F(size_t(L) * Hkv);
  for (int l = 0; l < L; ++l)
    for (int h = 0; h < Hkv; ++h) {
      double sum = 0.0;
      for (int g = 0; g < G; ++g) sum += F_heads[size_t(l) * Hq + h * G + g];  // ascending head order
      F[size_t(l) * Hkv + h] = sum / double(G);
    }
  return d2o_allocate_budgets_policy(D2O_ALLOC_SOFTMAX, F.data(), L * Hkv, seq_len, total, min_budget, S_out);
}

int d2o_prefill_compress(d2o_ctx* x, int32_t layer, d2o_view Q, d2o_view K, d2o_view V, int32_t n,
                         d2o_view O, const int32_t* budget, const int32_t* recent, void* stream) {
  int rc = d2o_prefill_attend(x, layer, Q, K, V, n, O, stream);
  if (rc) return rc;
  return d2o_compress_layer(x, layer, K, V, n, budget, recent, stream);
}

static int decode_step_impl(d2o_ctx* x, int32_t layer, int32_t nl, d2o_view q, d2o_view k_new, d2o_view v_new,
                            d2o_view out, void* stream, bool use_static) {
  if (!x) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || nl < 1 || layer + nl > c.n_layers) return fail(x, D2O_ERR_INVALID_ARG, "layer range");
  if (!view_ok(x, q) || !view_ok(x, k_new) || !view_ok(x, v_new) || !view_ok(x, out, c.out_f32 ? 4 : 0))
    return fail(x, D2O_ERR_INVALID_ARG, "null, misaligned or badly strided tensor view");
  const int32_t new_pos = x->layers[layer].next_pos;
  for (int l = layer; l < layer + nl; ++l) {
    if (x->layers[l].phase != kReady) return fail(x, D2O_ERR_STATE, "layer not compressed");
    if (x->layers[l].next_pos != new_pos)
      return fail(x, D2O_ERR_STATE, "layers of one call must be at the same token position");
  }
  unsigned char* stat = nullptr;
  if (use_static) {
    const size_t need = decode_static_scratch_need(x), cap = decode_static_scratch_capacity();
    if (need > cap)
      return fail(x, D2O_ERR_CAPACITY, "a decode step of this context needs " + std::to_string(need) +
                                           " bytes of scratch, the static array holds " + std::to_string(cap));
    const hipError_t e = static_scratch_address(&stat);
    if (e != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("static scratch: ") + hipGetErrorString(e));
  }
  const int timing = x->timing;
  if (use_static) x->timing = 0;  // timing events are runtime objects: none are created on this path
  hipError_t e = launch_decode(x, layer, nl, to_view(q), to_view(k_new), to_view(v_new), to_view(out),
                               new_pos, static_cast<hipStream_t>(stream), stat);
  x->timing = timing;
  if (e != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("decode: ") + hipGetErrorString(e));
  for (int l = layer; l < layer + nl; ++l) ++x->layers[l].next_pos;
  return D2O_OK;
}

int d2o_decode_step(d2o_ctx* x, int32_t layer, int32_t nl, d2o_view q, d2o_view k_new, d2o_view v_new,
                    d2o_view out, void* stream) {
  return decode_step_impl(x, layer, nl, q, k_new, v_new, out, stream, false);
}

int d2o_decode_step_static(d2o_ctx* x, int32_t layer, int32_t nl, d2o_view q, d2o_view k_new, d2o_view v_new,
                           d2o_view out, void* stream) {
  return decode_step_impl(x, layer, nl, q, k_new, v_new, out, stream, true);
}

int d2o_append_chunk(d2o_ctx* x, int32_t layer, d2o_view Q, d2o_view K, d2o_view V, int32_t m, d2o_view O,
                     void* stream) {
  if (!x) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(x, D2O_ERR_INVALID_ARG, "layer out of range");
  if (c.max_append < 2) return fail(x, D2O_ERR_STATE, "the context was created without room for blocks (max_append < 2)");
  if (m < 1 || m > c.max_append) return fail(x, D2O_ERR_INVALID_ARG, "block size must be in [1, max_append]");
  if (!view_ok(x, Q) || !view_ok(x, K) || !view_ok(x, V) || !view_ok(x, O, c.out_f32 ? 4 : 0))
    return fail(x, D2O_ERR_INVALID_ARG, "null, misaligned or badly strided tensor view");
  if (Q.stride_n < c.head_dim || K.stride_n < c.head_dim || V.stride_n < c.head_dim || O.stride_n < c.head_dim)
    return fail(x, D2O_ERR_INVALID_ARG, "token stride smaller than head_dim");
  LayerState& st = x->layers[layer];
  if (st.phase != kReady) return fail(x, D2O_ERR_STATE, "layer not compressed");
  hipStream_t s = static_cast<hipStream_t>(stream);
  // ---- the block's rows appended, every token's attention over the cache and the block's earlier
  //      tokens, Eq. 6 for every token; no eviction inside the block
  {
    const hipError_t e = launch_block_attend(x, layer, to_view(Q), to_view(K), to_view(V), to_view(O), m, st.next_pos, s);
    if (e != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, attention: ") + hipGetErrorString(e));
  }
  st.next_pos += m;
  // ---- Eq. 7-12 once on every cache, in ascending token position
  int max_budget = 0;
  for (const auto& mt : st.meta) max_budget = std::max(max_budget, mt.budget);
  const int n_eff = max_budget + m;  // upper bound of the entries of any head
  const View aK{x->app_K, int64_t(c.n_kv_heads) * x->npad * c.head_dim, int64_t(x->npad) * c.head_dim, c.head_dim};
  const View aV{x->app_V, aK.sb, aK.sh, aK.sn};
  hipError_t e;
  if ((e = launch_cache_sort(x, layer, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, ordering: ") + hipGetErrorString(e));
  if ((e = launch_select(x, layer, n_eff, s, true)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, select: ") + hipGetErrorString(e));
  if ((e = launch_gather(x, layer, aK, aV, n_eff, s, true)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, gather: ") + hipGetErrorString(e));
  if ((e = launch_match(x, layer, aK, n_eff, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, match: ") + hipGetErrorString(e));
  if ((e = launch_threshold_group(x, layer, n_eff, s, true)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, threshold: ") + hipGetErrorString(e));
  if ((e = launch_merge(x, layer, aK, aV, n_eff, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, merge: ") + hipGetErrorString(e));
  if (c.cache_fp8 && (e = launch_encode_layer(x, layer, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, encode: ") + hipGetErrorString(e));
  if ((e = launch_init_candidates(x, layer, st.next_pos, s)) != hipSuccess) return fail(x, D2O_ERR_HIP, std::string("append, candidates: ") + hipGetErrorString(e));
  x->last_append_layer = layer;
  x->last_compress_layer = -1;  // the prompt-phase events shared the scratch lists and are gone
  return D2O_OK;
}

static int head_args_ok(d2o_ctx* x, int32_t layer, int32_t b, int32_t h) {
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers || b < 0 || b >= c.batch || h < 0 || h >= c.n_kv_heads)
    return fail(x, D2O_ERR_INVALID_ARG, "layer, sequence or head out of range");
  return D2O_OK;
}

int d2o_cache_export(d2o_ctx* x, int32_t layer, int32_t b, int32_t h, void* K, void* V, double* score,
                     int32_t* pos, int32_t* count, double* tau, void* stream) {
  if (!x) return D2O_ERR_INVALID_ARG;
  int rc = head_args_ok(x, layer, b, h);
  if (rc) return rc;
  const d2o_config& c = x->cfg;
  LayerState& st = x->layers[layer];
  if (st.phase != kReady) return fail(x, D2O_ERR_STATE, "layer not compressed");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t lbh = (size_t(layer) * c.batch + b) * c.n_kv_heads + h;
  int32_t cnt = 0;
  double t = 0;
  D2O_HIP_CHECK(x, hipMemcpyAsync(&cnt, x->ccount + lbh, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(&t, x->ctau + lbh, sizeof(double), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  if (count) *count = cnt;
  if (tau) *tau = t;
  if (cnt <= 0) return D2O_OK;
  const size_t slot0 = (size_t(b) * c.n_kv_heads + h) * c.slots_per_seq + st.meta[size_t(b) * c.n_kv_heads + h].base;
  const size_t row = size_t(c.head_dim) * x->esize;
  std::vector<char> k(cnt * row), v(cnt * row);
  std::vector<double> sc(cnt);
  std::vector<int32_t> ps(cnt);
  if (c.cache_fp8) {  // decoded into the head's bf16 staging rows first (the decoded values are exact in bf16)
    const size_t stage0 = (size_t(b) * c.n_kv_heads + h) * x->npad;
    D2O_HIP_CHECK(x, launch_decode_head(x, layer, b, h, cnt, s));
    D2O_HIP_CHECK(x, hipMemcpyAsync(k.data(), static_cast<char*>(x->st_K) + stage0 * row, cnt * row, hipMemcpyDeviceToHost, s));
    D2O_HIP_CHECK(x, hipMemcpyAsync(v.data(), static_cast<char*>(x->st_V) + stage0 * row, cnt * row, hipMemcpyDeviceToHost, s));
  } else {
    D2O_HIP_CHECK(x, hipMemcpyAsync(k.data(), static_cast<char*>(x->cacheK) + slot0 * row, cnt * row, hipMemcpyDeviceToHost, s));
    D2O_HIP_CHECK(x, hipMemcpyAsync(v.data(), static_cast<char*>(x->cacheV) + slot0 * row, cnt * row, hipMemcpyDeviceToHost, s));
  }
  D2O_HIP_CHECK(x, hipMemcpyAsync(sc.data(), x->cscore + slot0, cnt * sizeof(double), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(ps.data(), x->cpos + slot0, cnt * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  std::vector<int32_t> order(cnt);
  std::iota(order.begin(), order.end(), 0);
  std::sort(order.begin(), order.end(), [&](int a, int bb) { return ps[a] < ps[bb]; });
  for (int i = 0; i < cnt; ++i) {
    const int src = order[i];
    if (K) std::memcpy(static_cast<char*>(K) + i * row, k.data() + src * row, row);
    if (V) std::memcpy(static_cast<char*>(V) + i * row, v.data() + src * row, row);
    if (score) score[i] = sc[src];
    if (pos) pos[i] = ps[src];
  }
  return D2O_OK;
}

int d2o_cache_import(d2o_ctx* x, int32_t layer, int32_t b, int32_t h, const void* K, const void* V,
                     const double* score, const int32_t* pos, int32_t count, double tau, int32_t next_pos,
                     void* stream) {
  if (!x || !K || !V || !score || !pos) return D2O_ERR_INVALID_ARG;
  int rc = head_args_ok(x, layer, b, h);
  if (rc) return rc;
  const d2o_config& c = x->cfg;
  LayerState& st = x->layers[layer];
  if (st.phase != kReady) return fail(x, D2O_ERR_STATE, "layer not reserved");
  if (count < 0 || count > st.meta[size_t(b) * c.n_kv_heads + h].budget) return fail(x, D2O_ERR_INVALID_ARG, "count exceeds the budget");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t lbh = (size_t(layer) * c.batch + b) * c.n_kv_heads + h;
  const size_t slot0 = (size_t(b) * c.n_kv_heads + h) * c.slots_per_seq + st.meta[size_t(b) * c.n_kv_heads + h].base;
  const size_t row = size_t(c.head_dim) * x->esize;
  if (c.cache_fp8) {  // the bf16 rows go to the head's staging rows and are encoded from there
    const size_t stage0 = (size_t(b) * c.n_kv_heads + h) * x->npad;
    D2O_HIP_CHECK(x, hipMemcpyAsync(static_cast<char*>(x->st_K) + stage0 * row, K, count * row, hipMemcpyHostToDevice, s));
    D2O_HIP_CHECK(x, hipMemcpyAsync(static_cast<char*>(x->st_V) + stage0 * row, V, count * row, hipMemcpyHostToDevice, s));
    D2O_HIP_CHECK(x, launch_encode_head(x, layer, b, h, count, s));
  } else {
    D2O_HIP_CHECK(x, hipMemcpyAsync(static_cast<char*>(x->cacheK) + slot0 * row, K, count * row, hipMemcpyHostToDevice, s));
    D2O_HIP_CHECK(x, hipMemcpyAsync(static_cast<char*>(x->cacheV) + slot0 * row, V, count * row, hipMemcpyHostToDevice, s));
  }
  D2O_HIP_CHECK(x, hipMemcpyAsync(x->cscore + slot0, score, count * sizeof(double), hipMemcpyHostToDevice, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(x->cpos + slot0, pos, count * sizeof(int32_t), hipMemcpyHostToDevice, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(x->ccount + lbh, &count, sizeof(int32_t), hipMemcpyHostToDevice, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(x->ctau + lbh, &tau, sizeof(double), hipMemcpyHostToDevice, s));
  // the imported rows have no known eviction candidates yet
  D2O_HIP_CHECK(x, fill32(x->ccand + lbh * decode_candidates(), 0xFFFFFFFFu, sizeof(int32_t) * decode_candidates(), s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  st.next_pos = next_pos;
  return D2O_OK;
}

int d2o_last_events(d2o_ctx* x, int32_t layer, int32_t* evicted_pos, int32_t* target_pos, double* u_star,
                    void* stream) {
  if (!x) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(x, D2O_ERR_INVALID_ARG, "layer out of range");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t bh = size_t(c.batch) * c.n_kv_heads, off = size_t(layer) * bh;
  if (evicted_pos) D2O_HIP_CHECK(x, hipMemcpyAsync(evicted_pos, x->ev_evicted + off, bh * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (target_pos) D2O_HIP_CHECK(x, hipMemcpyAsync(target_pos, x->ev_target + off, bh * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (u_star) D2O_HIP_CHECK(x, hipMemcpyAsync(u_star, x->ev_ustar + off, bh * sizeof(double), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  return D2O_OK;
}

int d2o_prefill_events(d2o_ctx* x, int32_t layer, int32_t b, int32_t h, int32_t* retained_pos, int32_t* n_ret,
                       int32_t* evicted_pos, int32_t* n_evi, int32_t* target_pos, double* u_star,
                       uint8_t* passed, void* stream) {
  if (!x) return D2O_ERR_INVALID_ARG;
  int rc = head_args_ok(x, layer, b, h);
  if (rc) return rc;
  if (layer != x->last_compress_layer)
    return fail(x, D2O_ERR_STATE, "prefill events are kept for the most recently compressed layer only");
  const d2o_config& c = x->cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t bh = size_t(b) * c.n_kv_heads + h;
  int32_t cnt[2] = {0, 0};
  D2O_HIP_CHECK(x, hipMemcpyAsync(cnt, x->sel_cnt + bh * 2, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  if (n_ret) *n_ret = cnt[0];
  if (n_evi) *n_evi = cnt[1];
  const size_t o = bh * x->npad;
  std::vector<int32_t> ret(cnt[0]), tgt(cnt[1]);
  D2O_HIP_CHECK(x, hipMemcpyAsync(ret.data(), x->sel_ret + o, cnt[0] * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (evicted_pos && cnt[1]) D2O_HIP_CHECK(x, hipMemcpyAsync(evicted_pos, x->sel_evi + o, cnt[1] * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (cnt[1]) D2O_HIP_CHECK(x, hipMemcpyAsync(tgt.data(), x->m_tgt + o, cnt[1] * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (u_star && cnt[1]) D2O_HIP_CHECK(x, hipMemcpyAsync(u_star, x->m_ustar + o, cnt[1] * sizeof(double), hipMemcpyDeviceToHost, s));
  if (passed && cnt[1]) D2O_HIP_CHECK(x, hipMemcpyAsync(passed, x->m_pass + o, cnt[1], hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  if (retained_pos) std::memcpy(retained_pos, ret.data(), cnt[0] * sizeof(int32_t));
  if (target_pos)
    for (int i = 0; i < cnt[1]; ++i) target_pos[i] = ret[tgt[i]];
  return D2O_OK;
}

int d2o_append_events(d2o_ctx* x, int32_t layer, int32_t b, int32_t h, int32_t* evicted_pos, int32_t* n_evi,
                      int32_t* target_pos, double* u_star, uint8_t* passed, void* stream) {
  if (!x) return D2O_ERR_INVALID_ARG;
  int rc = head_args_ok(x, layer, b, h);
  if (rc) return rc;
  if (layer != x->last_append_layer)
    return fail(x, D2O_ERR_STATE, "block events are kept for the layer of the most recent d2o_append_chunk only");
  const d2o_config& c = x->cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t bh = size_t(b) * c.n_kv_heads + h, o = bh * x->npad;
  int32_t cnt[2] = {0, 0}, n = 0;
  D2O_HIP_CHECK(x, hipMemcpyAsync(cnt, x->sel_cnt + bh * 2, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(&n, x->app_n + bh, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  if (n_evi) *n_evi = cnt[1];
  if (cnt[1] == 0) return D2O_OK;
  std::vector<int32_t> ret(cnt[0]), evi(cnt[1]), tgt(cnt[1]), pos(n);
  D2O_HIP_CHECK(x, hipMemcpyAsync(ret.data(), x->sel_ret + o, cnt[0] * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(evi.data(), x->sel_evi + o, cnt[1] * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(tgt.data(), x->m_tgt + o, cnt[1] * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipMemcpyAsync(pos.data(), x->app_pos + o, n * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (u_star) D2O_HIP_CHECK(x, hipMemcpyAsync(u_star, x->m_ustar + o, cnt[1] * sizeof(double), hipMemcpyDeviceToHost, s));
  if (passed) D2O_HIP_CHECK(x, hipMemcpyAsync(passed, x->m_pass + o, cnt[1], hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  for (int i = 0; i < cnt[1]; ++i) {  // ranks in the position-ordered copy -> token positions
    if (evicted_pos) evicted_pos[i] = pos[evi[i]];
    if (target_pos) target_pos[i] = pos[ret[tgt[i]]];
  }
  return D2O_OK;
}

int d2o_candidate_misses(d2o_ctx* x, int64_t* misses, void* stream) {
  if (!x || !misses) return D2O_ERR_INVALID_ARG;
  const d2o_config& c = x->cfg;
  const size_t n = size_t(c.n_layers) * c.batch * c.n_kv_heads;
  std::vector<uint32_t> h(n);
  hipStream_t s = static_cast<hipStream_t>(stream);
  D2O_HIP_CHECK(x, hipMemcpyAsync(h.data(), x->cmiss, n * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  D2O_HIP_CHECK(x, hipStreamSynchronize(s));
  int64_t t = 0;
  for (uint32_t v : h) t += v;
  *misses = t;
  return D2O_OK;
}

int d2o_timing_enable(d2o_ctx* x, int32_t on) {
  if (!x) return D2O_ERR_INVALID_ARG;
  if (on < 0) return D2O_ERR_INVALID_ARG;
  x->timing = on;
  for (auto& v : x->launch_no) v = 0;
  return D2O_OK;
}

int d2o_timing_read(d2o_ctx* x, int32_t kernel_id, double* total_ms, int64_t* launches, void* stream) {
  if (!x || !total_ms || !launches || kernel_id < 0 || kernel_id >= D2O_K_COUNT) return D2O_ERR_INVALID_ARG;
  D2O_HIP_CHECK(x, hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  double ms = 0.0;
  int64_t cnt = 0;
  std::vector<d2o_timed_launch> keep;
  for (auto& t : x->timed) {
    if (t.id != kernel_id) {
      keep.push_back(t);
      continue;
    }
    float f = 0.f;
    D2O_HIP_CHECK(x, hipEventSynchronize(t.stop));
    D2O_HIP_CHECK(x, hipEventElapsedTime(&f, t.start, t.stop));
    ms += f;
    ++cnt;
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  x->timed.swap(keep);
  *total_ms = ms;
  *launches = cnt;
  return D2O_OK;
}

}  // extern "C"
