// One generation step over the compressed cache (Sec. 3 Eq. 2-3; Sec. 4.2 Eq. 6-12), for a
// range of layers in one set of launches.  The step is bound by HBM traffic (every K and V row
// of every layer is read once), so all decision-bearing arithmetic - logits, softmax
// normaliser, score accumulation, eviction arg-min, cosine arg-max, EMA threshold and the
// merge - is done in fp64 with the operation order of the defining formulas; only the
// attention output (P V) accumulates in fp32.
//
// Kernels, per (layer, sequence, KV head):
//   decode_append  writes the new token's k, v into the free slot (score 0, its position).
//   decode_attend  split over chunks of 256 slots: fp64 logits of the G query heads (kept in
//                  scratch), chunk-local softmax statistics and partial P V.
//   decode_update  combines the chunks into the output rows, forms the exact normaliser, adds
//                  the softmax rows to the scores (Eq. 6, generation case) and picks the token
//                  to evict (Eq. 7-8: lowest score outside sinks and the recent window; equal
//                  scores evict the later position).
//   decode_cosine  split over chunks: cosine of the evicted key against every survivor (Eq. 9).
//   decode_finish  arg-max (ties: earlier position), EMA threshold (Eq. 10), merge or discard
//                  (Eq. 11-12 with one source), and moves the last slot into the freed one.
// Slots are physically unordered; a token's identity is its position.
#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace {

struct DecodeArgs {
  int32_t* ccount;
  double* ctau;
  const int32_t* meta;
  void* cK;
  void* cV;
  double* cscore;
  int32_t* cpos;
  double* logit;
  double* pm;
  float* pl;
  float* pacc;
  int32_t* eslot;
  double* cu;
  int32_t* cslot;
  int32_t* ev_evicted;
  int32_t* ev_target;
  double* ev_ustar;
  int64_t slots;
  int64_t nchunk_cap;
  int layer0, B, Hkv, G, new_pos, n_sink, out_f32;
  double beta, tau_force;
};

template <typename T>
__device__ __forceinline__ void load_chunk(const T* p, double* out);
template <>
__device__ __forceinline__ void load_chunk<uint16_t>(const uint16_t* p, double* out) {  // 8 elements
  const u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = double(__uint_as_float(v[i] << 16));
    out[2 * i + 1] = double(__uint_as_float(v[i] & 0xFFFF0000u));
  }
}
template <>
__device__ __forceinline__ void load_chunk<float>(const float* p, double* out) {  // 4 elements
  const float4 a = *reinterpret_cast<const float4*>(p);
  out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
}
template <typename T>
__device__ __forceinline__ void load_chunk_f32(const T* p, float* out);
template <>
__device__ __forceinline__ void load_chunk_f32<uint16_t>(const uint16_t* p, float* out) {
  const u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(v[i] << 16);
    out[2 * i + 1] = __uint_as_float(v[i] & 0xFFFF0000u);
  }
}
template <>
__device__ __forceinline__ void load_chunk_f32<float>(const float* p, float* out) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
}

template <typename T, int D>
__global__ __launch_bounds__(128) void decode_append(DecodeArgs a, const T* __restrict__ kn, View kv,
                                                     const T* __restrict__ vn, View vv) {
  const int li = blockIdx.y, l = a.layer0 + li, b = blockIdx.x / a.Hkv, hk = blockIdx.x % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int count = a.ccount[lbh];
  const int64_t slot = (int64_t(b) * a.Hkv + hk) * a.slots + a.meta[(l * a.B + b) * 4 + 0] + count;
  const int c = threadIdx.x;
  if (c < D) {
    static_cast<T*>(a.cK)[slot * D + c] = kn[li * kv.sn + b * kv.sb + hk * kv.sh + c];
    static_cast<T*>(a.cV)[slot * D + c] = vn[li * vv.sn + b * vv.sb + hk * vv.sh + c];
  }
  if (c == 0) {
    a.cscore[slot] = 0.0;
    a.cpos[slot] = a.new_pos;
  }
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_attend(DecodeArgs a, const T* __restrict__ q, View qv) {
  constexpr int kVec = 16 / sizeof(T);       // elements per 16-byte load
  constexpr int TPR = D / kVec;              // threads per row
  constexpr int RPP = 256 / TPR;             // rows per pass
  __shared__ double qs[G][D];
  __shared__ double slog[G][kChunk];
  __shared__ float ps[G][kChunk];
  __shared__ float red[RPP][D];
  __shared__ double redd[4];
  const int li = blockIdx.z, l = a.layer0 + li, b = blockIdx.y / a.Hkv, hk = blockIdx.y % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int total = a.ccount[lbh] + 1;       // the new token has been appended
  const int chunk = blockIdx.x;
  if (chunk * kChunk >= total) return;
  const int tid = threadIdx.x;
  const int32_t* mt = a.meta + (l * a.B + b) * 4;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt[0];
  const T* Kc = static_cast<const T*>(a.cK) + slot0 * D;
  const T* Vc = static_cast<const T*>(a.cV) + slot0 * D;
  const int rows = min(kChunk, total - chunk * kChunk);
  for (int i = tid; i < G * D; i += 256) {
    const int g = i / D, c = i % D;
    qs[g][c] = Elem<T>::to_f64(q[li * qv.sn + b * qv.sb + (hk * G + g) * qv.sh + c]);
  }
  __syncthreads();
  const int tr = tid / TPR, tc = (tid % TPR) * kVec;
  const double root_d = sqrt(double(D));
  // ---- logits, fp64
  for (int r0 = 0; r0 < rows; r0 += RPP) {
    const int r = r0 + tr;
    double dot[G];
#pragma unroll
    for (int g = 0; g < G; ++g) dot[g] = 0.0;
    if (r < rows) {
      double x[kVec];
      load_chunk<T>(Kc + int64_t(chunk * kChunk + r) * D + tc, x);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < kVec; ++e) dot[g] += x[e] * qs[g][tc + e];
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int o = TPR / 2; o > 0; o >>= 1) dot[g] += __shfl_xor(dot[g], o, 64);
      if (r < rows && (tid % TPR) == 0) {
        const double s = dot[g] / root_d;
        slog[g][r] = s;
        a.logit[(int64_t(b) * a.Hkv * G + hk * G + g) * a.slots + mt[0] + chunk * kChunk + r] = s;
      }
    }
  }
  __syncthreads();
  // ---- chunk-local softmax statistics
  const int64_t pidx = (bh * a.nchunk_cap + mt[3] + chunk) * G;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    double mx = tid < rows ? slog[g][tid] : -INFINITY;
    mx = wave_max(mx);
    __syncthreads();
    if ((tid & 63) == 0) redd[tid >> 6] = mx;
    __syncthreads();
    mx = fmax(fmax(redd[0], redd[1]), fmax(redd[2], redd[3]));
    const float p = tid < rows ? expf(float(slog[g][tid] - mx)) : 0.f;
    ps[g][tid] = p;
    float sm = wave_sum(p);
    __syncthreads();
    if ((tid & 63) == 0) redd[tid >> 6] = double(sm);
    __syncthreads();
    if (tid == 0) {
      a.pm[pidx + g] = mx;
      a.pl[pidx + g] = float(redd[0]) + float(redd[1]) + float(redd[2]) + float(redd[3]);
    }
  }
  __syncthreads();
  // ---- partial P V, fp32
  float acc[G][kVec];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < kVec; ++e) acc[g][e] = 0.f;
  for (int r0 = 0; r0 < rows; r0 += RPP) {
    const int r = r0 + tr;
    if (r < rows) {
      float x[kVec];
      load_chunk_f32<T>(Vc + int64_t(chunk * kChunk + r) * D + tc, x);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = ps[g][r];
#pragma unroll
        for (int e = 0; e < kVec; ++e) acc[g][e] = fmaf(p, x[e], acc[g][e]);
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kVec; ++e) red[tr][tc + e] = acc[g][e];
    __syncthreads();
    if (tid < D) {
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < RPP; ++i) t += red[i][tid];
      a.pacc[(pidx + g) * D + tid] = t;
    }
  }
}

template <typename T, typename OT, int D, int G>
__global__ __launch_bounds__(256) void decode_update(DecodeArgs a, OT* __restrict__ out, View ov) {
  __shared__ double red[4];
  __shared__ double Msh[G], Lsh[G];
  __shared__ double bscore[4];
  __shared__ int bpos[4], bslot[4];
  const int li = blockIdx.y, l = a.layer0 + li, b = blockIdx.x / a.Hkv, hk = blockIdx.x % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int total = a.ccount[lbh] + 1;
  const int nchunk = (total + kChunk - 1) / kChunk;
  const int tid = threadIdx.x;
  const int32_t* mt = a.meta + (l * a.B + b) * 4;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt[0];
  const int64_t pbase = (bh * a.nchunk_cap + mt[3]) * G;
  for (int g = 0; g < G; ++g) {
    double mx = -INFINITY;
    for (int c = tid; c < nchunk; c += 256) mx = fmax(mx, a.pm[pbase + int64_t(c) * G + g]);
    mx = wave_max(mx);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
    if (tid == 0) Msh[g] = mx;
    // output row of query head g: chunks combined in ascending order
    if (tid < D) {
      float num = 0.f, den = 0.f;
      for (int c = 0; c < nchunk; ++c) {
        const int64_t pi = pbase + int64_t(c) * G + g;
        const float f = expf(float(a.pm[pi] - mx));
        den = fmaf(a.pl[pi], f, den);
        num = fmaf(a.pacc[pi * D + tid], f, num);
      }
      out[li * ov.sn + b * ov.sb + (hk * G + g) * ov.sh + tid] = Elem<OT>::from_f32(num / den);
    }
    // exact normaliser: sum_j exp(s_j - max), fp64; the exponentials replace the logits
    double* lg = a.logit + (int64_t(b) * a.Hkv * G + hk * G + g) * a.slots + mt[0];
    double part = 0.0;
    for (int j = tid; j < total; j += 256) {
      const double e = exp(lg[j] - mx);
      lg[j] = e;
      part += e;
    }
    const double L = block_sum(part, red);
    if (tid == 0) Lsh[g] = L;
  }
  __syncthreads();
  // scores (Eq. 6) and the eviction candidate (Eq. 7-8 on count+1 entries)
  const bool evict = total > mt[1];
  const int recent = mt[2];
  double best = INFINITY;
  int bp = -1, bs = -1;
  for (int j = tid; j < total; j += 256) {
    double sc = a.cscore[slot0 + j];
    for (int g = 0; g < G; ++g) {
      const double* lg = a.logit + (int64_t(b) * a.Hkv * G + hk * G + g) * a.slots + mt[0];
      sc += lg[j] / Lsh[g];
    }
    a.cscore[slot0 + j] = sc;
    const int p = a.cpos[slot0 + j];
    const bool cand = p >= a.n_sink && p <= a.new_pos - recent;
    if (cand && (sc < best || (sc == best && p > bp))) {
      best = sc;
      bp = p;
      bs = j;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double ob = __shfl_xor(best, o, 64);
    const int op = __shfl_xor(bp, o, 64), os = __shfl_xor(bs, o, 64);
    if (os >= 0 && (bs < 0 || ob < best || (ob == best && op > bp))) {
      best = ob;
      bp = op;
      bs = os;
    }
  }
  if ((tid & 63) == 0) {
    bscore[tid >> 6] = best;
    bpos[tid >> 6] = bp;
    bslot[tid >> 6] = bs;
  }
  __syncthreads();
  if (tid == 0) {
    for (int i = 1; i < 4; ++i)
      if (bslot[i] >= 0 && (bs < 0 || bscore[i] < best || (bscore[i] == best && bpos[i] > bp))) {
        best = bscore[i];
        bp = bpos[i];
        bs = bslot[i];
      }
    if (evict) {
      a.eslot[lbh] = bs;  // a candidate always exists: total > budget >= T + M
    } else {
      a.eslot[lbh] = -1;
      a.ccount[lbh] = total;
      a.ev_evicted[lbh] = -1;
      a.ev_target[lbh] = -1;
      a.ev_ustar[lbh] = __longlong_as_double(0x7FF8000000000000ll);
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_cosine(DecodeArgs a) {
  constexpr int kVec = 16 / sizeof(T);
  constexpr int TPR = D / kVec;
  constexpr int RPP = 256 / TPR;
  __shared__ double ke[D];
  __shared__ double red[4];
  __shared__ double bu[4];
  __shared__ int bpos[4], bslot[4];
  const int li = blockIdx.z, l = a.layer0 + li, b = blockIdx.y / a.Hkv, hk = blockIdx.y % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int es = a.eslot[lbh];
  if (es < 0) return;
  const int total = a.ccount[lbh] + 1;
  const int chunk = blockIdx.x;
  if (chunk * kChunk >= total) return;
  const int tid = threadIdx.x;
  const int32_t* mt = a.meta + (l * a.B + b) * 4;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt[0];
  const T* Kc = static_cast<const T*>(a.cK) + slot0 * D;
  double part = 0.0;
  if (tid < D) {
    const double x = Elem<T>::to_f64(Kc[int64_t(es) * D + tid]);
    ke[tid] = x;
    part = x * x;
  }
  const double sne = sqrt(block_sum(part, red));
  const int rows = min(kChunk, total - chunk * kChunk);
  const int tr = tid / TPR, tc = (tid % TPR) * kVec;
  double best = -2.0;
  int bp = 0x7FFFFFFF, bs = -1;
  for (int r0 = 0; r0 < rows; r0 += RPP) {
    const int r = r0 + tr, j = chunk * kChunk + r;
    double dot = 0.0, nr = 0.0;
    if (r < rows) {
      double x[kVec];
      load_chunk<T>(Kc + int64_t(j) * D + tc, x);
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        dot += x[e] * ke[tc + e];
        nr += x[e] * x[e];
      }
    }
#pragma unroll
    for (int o = TPR / 2; o > 0; o >>= 1) {
      dot += __shfl_xor(dot, o, 64);
      nr += __shfl_xor(nr, o, 64);
    }
    if (r < rows && j != es && (tid % TPR) == 0) {
      const double den = sne * sqrt(nr);
      const double u = den > 0.0 ? dot / den : 0.0;
      const int p = a.cpos[slot0 + j];
      if (u > best || (u == best && p < bp)) {
        best = u;
        bp = p;
        bs = j;
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double ob = __shfl_xor(best, o, 64);
    const int op = __shfl_xor(bp, o, 64), os = __shfl_xor(bs, o, 64);
    if (os >= 0 && (bs < 0 || ob > best || (ob == best && op < bp))) {
      best = ob;
      bp = op;
      bs = os;
    }
  }
  if ((tid & 63) == 0) {
    bu[tid >> 6] = best;
    bpos[tid >> 6] = bp;
    bslot[tid >> 6] = bs;
  }
  __syncthreads();
  if (tid == 0) {
    for (int i = 1; i < 4; ++i)
      if (bslot[i] >= 0 && (bs < 0 || bu[i] > best || (bu[i] == best && bpos[i] < bp))) {
        best = bu[i];
        bp = bpos[i];
        bs = bslot[i];
      }
    const int64_t ci = bh * a.nchunk_cap + mt[3] + chunk;
    a.cu[ci] = best;
    a.cslot[ci] = bs;  // -1 when the chunk holds only the evicted slot
  }
}

template <typename T, int D>
__global__ __launch_bounds__(128) void decode_finish(DecodeArgs a) {
  __shared__ int sh_t, sh_merge;
  __shared__ double sh_u;
  const int li = blockIdx.y, l = a.layer0 + li, b = blockIdx.x / a.Hkv, hk = blockIdx.x % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int es = a.eslot[lbh];
  if (es < 0) return;
  const int total = a.ccount[lbh] + 1, last = total - 1;
  const int nchunk = (total + kChunk - 1) / kChunk;
  const int tid = threadIdx.x;
  const int32_t* mt = a.meta + (l * a.B + b) * 4;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt[0];
  T* Kc = static_cast<T*>(a.cK) + slot0 * D;
  T* Vc = static_cast<T*>(a.cV) + slot0 * D;
  if (tid == 0) {
    double best = -2.0;
    int bp = 0x7FFFFFFF, bs = -1;
    for (int c = 0; c < nchunk; ++c) {
      const int64_t ci = bh * a.nchunk_cap + mt[3] + c;
      const int s = a.cslot[ci];
      if (s < 0) continue;
      const double u = a.cu[ci];
      const int p = a.cpos[slot0 + s];
      if (bs < 0 || u > best || (u == best && p < bp)) {
        best = u;
        bp = p;
        bs = s;
      }
    }
    bool do_merge;
    if (isnan(a.tau_force)) {
      const double told = a.ctau[lbh];
      const double tnew = isnan(told) ? best
                                      : __dadd_rn(__dmul_rn(a.beta, best), __dmul_rn(1.0 - a.beta, told));
      a.ctau[lbh] = tnew;
      do_merge = best >= tnew;
    } else {
      do_merge = best >= a.tau_force;
    }
    sh_t = bs;
    sh_u = best;
    sh_merge = do_merge ? 1 : 0;
    a.ev_evicted[lbh] = a.cpos[slot0 + es];
    a.ev_target[lbh] = do_merge ? bp : -1;
    a.ev_ustar[lbh] = best;
  }
  __syncthreads();
  if (tid == 0) a.ccount[lbh] = last;  // after every thread has read the old count
  const int ts = sh_t;
  if (sh_merge && tid < D) {
    const double e1 = 2.718281828459045;
    const double w = exp(sh_u);
    const double z = __dadd_rn(e1, w);
    const double kk = __dadd_rn(__dmul_rn(e1, Elem<T>::to_f64(Kc[int64_t(ts) * D + tid])),
                                __dmul_rn(w, Elem<T>::to_f64(Kc[int64_t(es) * D + tid])));
    const double vv = __dadd_rn(__dmul_rn(e1, Elem<T>::to_f64(Vc[int64_t(ts) * D + tid])),
                                __dmul_rn(w, Elem<T>::to_f64(Vc[int64_t(es) * D + tid])));
    Kc[int64_t(ts) * D + tid] = Elem<T>::from_f64(kk / z);
    Vc[int64_t(ts) * D + tid] = Elem<T>::from_f64(vv / z);
  }
  __syncthreads();
  if (es != last) {  // the last slot fills the hole
    if (tid < D) {
      Kc[int64_t(es) * D + tid] = Kc[int64_t(last) * D + tid];
      Vc[int64_t(es) * D + tid] = Vc[int64_t(last) * D + tid];
    }
    if (tid == 0) {
      a.cscore[slot0 + es] = a.cscore[slot0 + last];
      a.cpos[slot0 + es] = a.cpos[slot0 + last];
    }
  }
}

template <typename T, int D, int G>
hipError_t run_decode(d2o_ctx* c, const DecodeArgs& a, int nl, int maxchunks, View q, View k, View v, View out, hipStream_t s) {
  const int bh = a.B * a.Hkv;
  decode_append<T, D><<<dim3(bh, nl), 128, 0, s>>>(a, (const T*)k.ptr, k, (const T*)v.ptr, v);
  {
    KernelTimer kt(c, D2O_K_DECODE_ATTEND, s);
    decode_attend<T, D, G><<<dim3(maxchunks, bh, nl), 256, 0, s>>>(a, (const T*)q.ptr, q);
  }
  {
  KernelTimer kt(c, D2O_K_DECODE_UPDATE, s);
  if (a.out_f32)
    decode_update<T, float, D, G><<<dim3(bh, nl), 256, 0, s>>>(a, (float*)out.ptr, out);
  else
    decode_update<T, T, D, G><<<dim3(bh, nl), 256, 0, s>>>(a, (T*)out.ptr, out);
  }
  {
    KernelTimer kt(c, D2O_K_DECODE_COSINE, s);
    decode_cosine<T, D><<<dim3(maxchunks, bh, nl), 256, 0, s>>>(a);
  }
  KernelTimer kt(c, D2O_K_DECODE_FINISH, s);
  decode_finish<T, D><<<dim3(bh, nl), 128, 0, s>>>(a);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t run_decode_g(d2o_ctx* c, const DecodeArgs& a, int nl, int mc, View q, View k, View v, View out, hipStream_t s) {
  switch (a.G) {
    case 1: return run_decode<T, D, 1>(c, a, nl, mc, q, k, v, out, s);
    case 2: return run_decode<T, D, 2>(c, a, nl, mc, q, k, v, out, s);
    case 4: return run_decode<T, D, 4>(c, a, nl, mc, q, k, v, out, s);
    case 8: return run_decode<T, D, 8>(c, a, nl, mc, q, k, v, out, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_decode(d2o_ctx* c, int layer0, int nl, View q, View k, View v, View out, int new_pos,
                         hipStream_t s) {
  const d2o_config& cf = c->cfg;
  DecodeArgs a;
  a.ccount = c->ccount;
  a.ctau = c->ctau;
  a.meta = c->meta;
  a.cK = c->cacheK;
  a.cV = c->cacheV;
  a.cscore = c->cscore;
  a.cpos = c->cpos;
  a.logit = c->d_logit;
  a.pm = c->d_pm;
  a.pl = c->d_pl;
  a.pacc = c->d_pacc;
  a.eslot = c->d_eslot;
  a.cu = c->d_cu;
  a.cslot = c->d_cslot;
  a.ev_evicted = c->ev_evicted;
  a.ev_target = c->ev_target;
  a.ev_ustar = c->ev_ustar;
  a.slots = cf.slots_per_seq;
  a.nchunk_cap = c->nchunk_cap;
  a.layer0 = layer0;
  a.B = cf.batch;
  a.Hkv = cf.n_kv_heads;
  a.G = cf.n_q_heads / cf.n_kv_heads;
  a.new_pos = new_pos;
  a.n_sink = cf.n_sink;
  a.out_f32 = cf.out_f32;
  a.beta = cf.beta;
  a.tau_force = cf.tau_force;
  int maxchunks = 1;
  for (int l = layer0; l < layer0 + nl; ++l)
    for (const auto& mt : c->layers[l].meta) maxchunks = std::max(maxchunks, (mt.budget + 1 + kChunk - 1) / kChunk);
  if (cf.dtype == D2O_BF16) return run_decode_g<uint16_t, 128>(c, a, nl, maxchunks, q, k, v, out, s);
  if (cf.head_dim == 64) return run_decode_g<float, 64>(c, a, nl, maxchunks, q, k, v, out, s);
  return run_decode_g<float, 128>(c, a, nl, maxchunks, q, k, v, out, s);
}

}  // namespace d2o
