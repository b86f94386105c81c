// Building blocks of the decode-step kernels in csrc/decode.hip: kernel arguments, element
// conversions, the orders in which matches and evictions are decided, and the step's closing
// arithmetic (Eq. 9-12 with one source).  Header-only; not part of the C ABI.
#pragma once

#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace dec {

// Eviction candidates whose similarities ride along with the attention pass.  One: the token
// with the lowest score after a step is, with very few exceptions, the one evicted at the next
// (scores only grow, and the lowest tokens are the ones that receive next to no attention); on
// the benchmark workloads no eviction of 5 x 10^5 to 2 x 10^6 head-steps took another token.
// Every further candidate costs the K pass another fp64 dot product per cache row (with three,
// configuration 4 ran 6 % and an fp8 cache 11 % slower); a miss costs one head a second pass
// over its keys.
constexpr int kCand = 1;
constexpr int kMaxLayersPerCall = 64;
// Doubles per sub-chunk record: the G softmax maxima, the G exp-sums, then per candidate its
// best cosine and that key's slot; rounded up to a multiple of eight (64 bytes).
__host__ __device__ constexpr int rec_doubles(int G) { return (2 * G + 2 * kCand + 7) / 8 * 8; }
constexpr int kPiece = 64;              // bytes of a cache row staged per LDS round
constexpr int kPitch = kPiece + 16;     // LDS pitch of a staged row piece (20 words: the lanes' reads spread over all banks)
constexpr int kStageBytes = 4 * 64 * kPitch;
constexpr int kSub = 64;                // rows one wavefront handles at a time (lane = row)
constexpr int kGroup = 1;               // chunks of 256 slots per workgroup

struct DecodeArgs {
  int32_t* ccount;
  int32_t* ctotal;    // [L][B][Hkv] entries of this step (count + 1): written by decode_prepare, never by decode_attend
  double* ctau;
  const int32_t* meta;
  void* cK;
  void* cV;
  int8_t* cKe;        // fp8 cache only: the power of two of every K row, [B][Hkv][slots]
  int8_t* cVe;        // the same for V
  double* cscore;
  int32_t* cpos;
  int32_t* cand;      // [L][B][Hkv][kCand] candidate slots for this step, -1 = none
  uint32_t* ticket;   // [L][B][Hkv] finished chunks of the running step
  uint32_t* cmiss;    // [L][B][Hkv] evictions whose token was not among the predicted candidates (since the last reset)
  double* elog;       // [chunk][B][Hkv][G][256] exp(logit - sub-chunk max)
  double* rec;        // [chunk][B][Hkv][4][rec_doubles(G)] per sub-chunk record: [0..G) softmax maxima of the
                      // query heads, [G..2G) exp-sums relative to them, [2G..2G+kCand) the candidates' best
                      // cosine, [2G+kCand..2G+2kCand) its slot (-1 none); written with one store
  float* pacc;        // [chunk][B][Hkv][G][d] partial outputs, relative to the chunk's softmax maximum
  double* vecs;       // [L][B][Hkv][G + kCand][d] queries and candidate keys as fp64
  double* cnorm;      // [L][B][Hkv][kCand] |k| of the candidates
  int32_t* ev_evicted;
  int32_t* ev_target;
  double* ev_ustar;
  int64_t slots;
  int layer0, nl, B, Hkv, G, new_pos, n_sink, out_f32, merge_average;
  int big_rows;       // heads with more entries are closed by the split kernels, not by their last workgroup
  int part_chunks;    // chunks per workgroup of decode_close_part
  double* part;       // [chunk][B][Hkv][kPartRecDoubles] part records (at a part's first chunk)
  double* hnorm;      // [L][B][Hkv][16] of a head closed in parts: [0..G) softmax maxima, [G..2G) exact normalisers
  double beta, tau_force;
  int32_t lay_off[kMaxLayersPerCall + 1];  // first flat chunk-group index of each entry of lay_id
  int32_t lay_id[kMaxLayersPerCall];       // layers of the call (relative), most chunks first
};

template <typename T>
__device__ __forceinline__ void cvt16(const u32x4& v, double* out);  // 16 bytes -> 8 or 4 doubles
template <>
__device__ __forceinline__ void cvt16<uint16_t>(const u32x4& v, double* out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = double(__uint_as_float(v[i] << 16));
    out[2 * i + 1] = double(__uint_as_float(v[i] & 0xFFFF0000u));
  }
}
template <>
__device__ __forceinline__ void cvt16<float>(const u32x4& v, double* out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = double(__uint_as_float(v[i]));
}
template <>
__device__ __forceinline__ void cvt16<uint8_t>(const u32x4& v, double* out) {  // sixteen fp8 codes, without the row's power of two
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[4 * i] = double(__builtin_amdgcn_cvt_f32_fp8(int(v[i]), 0));
    out[4 * i + 1] = double(__builtin_amdgcn_cvt_f32_fp8(int(v[i]), 1));
    out[4 * i + 2] = double(__builtin_amdgcn_cvt_f32_fp8(int(v[i]), 2));
    out[4 * i + 3] = double(__builtin_amdgcn_cvt_f32_fp8(int(v[i]), 3));
  }
}
template <typename T>
__device__ __forceinline__ void cvt16f(const u32x4& v, float* out);
template <>
__device__ __forceinline__ void cvt16f<uint16_t>(const u32x4& v, float* out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(v[i] << 16);
    out[2 * i + 1] = __uint_as_float(v[i] & 0xFFFF0000u);
  }
}
template <>
__device__ __forceinline__ void cvt16f<float>(const u32x4& v, float* out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = __uint_as_float(v[i]);
}
template <>
__device__ __forceinline__ void cvt16f<uint8_t>(const u32x4& v, float* out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[4 * i] = __builtin_amdgcn_cvt_f32_fp8(int(v[i]), 0);
    out[4 * i + 1] = __builtin_amdgcn_cvt_f32_fp8(int(v[i]), 1);
    out[4 * i + 2] = __builtin_amdgcn_cvt_f32_fp8(int(v[i]), 2);
    out[4 * i + 3] = __builtin_amdgcn_cvt_f32_fp8(int(v[i]), 3);
  }
}

// N consecutive elements (4, 8 or 16 bytes) held as raw bits, and their conversion to doubles.
template <int BYTES> struct RawBits;
template <> struct RawBits<16> { typedef u32x4 type; };
template <> struct RawBits<8> { typedef u32x2 type; };
template <> struct RawBits<4> { typedef uint32_t type; };
template <> struct RawBits<2> { typedef uint16_t type; };
__device__ __forceinline__ uint32_t raw_word(const uint16_t& r, int) { return r; }
__device__ __forceinline__ uint32_t raw_word(const u32x4& r, int i) { return r[i]; }
__device__ __forceinline__ uint32_t raw_word(const u32x2& r, int i) { return r[i]; }
__device__ __forceinline__ uint32_t raw_word(const uint32_t& r, int) { return r; }
template <typename T, int N, typename R>
__device__ __forceinline__ void raw_to_f64(const R& r, double* out) {
  if constexpr (sizeof(T) == 1) {  // two or four fp8 codes in one word, without the row's power of two
    static_assert(N == 2 || N == 4, "fp8 codes come two or four at a time");
    const int wd = int(raw_word(r, 0));
    out[0] = double(__builtin_amdgcn_cvt_f32_fp8(wd, 0));
    out[1] = double(__builtin_amdgcn_cvt_f32_fp8(wd, 1));
    if constexpr (N == 4) {
      out[2] = double(__builtin_amdgcn_cvt_f32_fp8(wd, 2));
      out[3] = double(__builtin_amdgcn_cvt_f32_fp8(wd, 3));
    }
  } else if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
      out[2 * i] = double(__uint_as_float(raw_word(r, i) << 16));
      out[2 * i + 1] = double(__uint_as_float(raw_word(r, i) & 0xFFFF0000u));
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) out[i] = double(__uint_as_float(raw_word(r, i)));
  }
}

// The partial results of a step are laid out chunk-major: [layer's chunk offset + chunk]
// [sequence][KV head]...  Workgroups are dispatched head-fastest, so the results that are written
// at about the same time are neighbours in memory (per-head contiguous arrays scatter them; a
// streaming probe with this kernel's store pattern lost 6.2 -> 5.0 TB/s of read rate to the
// scattered form and 6.2 -> 5.3 to this one).
__device__ __forceinline__ int64_t sub_index(const DecodeArgs& a, int64_t bh, int chunk0, int c) {  // sub-chunk c of the head
  return ((int64_t(chunk0) + (c >> 2)) * (a.B * a.Hkv) + bh) * 4 + (c & 3);
}
__device__ __forceinline__ int64_t chunk_index(const DecodeArgs& a, int64_t bh, int chunk0, int chunk) {  // chunk of the head
  return (int64_t(chunk0) + chunk) * (a.B * a.Hkv) + bh;
}
__device__ __forceinline__ int64_t elog_index(const DecodeArgs& a, int64_t bh, int chunk0, int G, int g, int j) {  // slot j
  return (((int64_t(chunk0) + (j >> 8)) * (a.B * a.Hkv) + bh) * G + g) * kChunk + (j & (kChunk - 1));
}

// Pins the point where a scalar-loaded value must have arrived; nothing is scheduled across it.
__device__ __forceinline__ void arrived(double v) {
  asm volatile("" ::"s"(v));
  __builtin_amdgcn_sched_barrier(0);
}

// Data that one workgroup of decode_attend hands to another (the head's last workgroup) goes
// through agent-scope stores and loads: they write through / read around the per-XCD L2, so
// the hand-over needs no L2 write-back (a release fence at agent scope writes the whole L2
// back, once per workgroup, which costs more than the attention pass itself).
template <typename U>
__device__ __forceinline__ void st_agent(U* p, U v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename U>
__device__ __forceinline__ U ld_agent(const U* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float4 ld_agent4(const float* p) {  // 16 bytes as two 8-byte loads
  const uint64_t lo = ld_agent(reinterpret_cast<const uint64_t*>(p));
  const uint64_t hi = ld_agent(reinterpret_cast<const uint64_t*>(p) + 1);
  return make_float4(__uint_as_float(uint32_t(lo)), __uint_as_float(uint32_t(lo >> 32)),
                     __uint_as_float(uint32_t(hi)), __uint_as_float(uint32_t(hi >> 32)));
}

// Which entry of the call's layer list a flat chunk index belongs to (block-uniform).  The
// list is sorted by size, so the workgroups dispatched last belong to the smallest caches.
// Unused entries of lay_off hold INT_MAX, so the search is a fixed chain of scalar compares on
// kernel arguments: no memory round trip precedes the loads that depend on the layer.
__device__ __forceinline__ int find_entry(const DecodeArgs& a, int x) {
  int entry = 0;
#pragma unroll
  for (int i = 1; i < kMaxLayersPerCall; ++i) entry += x >= a.lay_off[i] ? 1 : 0;
  return entry;
}

// (u larger, then position smaller) wins; slot < 0 means "no entry".
struct Best {
  double u;
  int pos, slot;
};
__device__ __forceinline__ bool better_match(double u, int p, int s, const Best& b) {
  return s >= 0 && (b.slot < 0 || u > b.u || (u == b.u && p < b.pos));
}
// Wavefront arg-max of that order for one entry per lane whose positions are all different and
// whose u is never below -1 (a cosine): largest u, then smallest position, then that lane's slot.
__device__ __forceinline__ Best fast_wave_best_match(double u, int pos, int slot) {
  const bool live = slot >= 0;
  const double umax = fast_wave_max(live ? u : -INFINITY);
  const bool top = live && u == umax;
  const int pmin = fast_wave_min(top ? pos : 0x7FFFFFFF);
  const unsigned long long who = __ballot(top && pos == pmin);
  if (who == 0ull) return Best{0.0, 0, -1};
  const int src = __ffsll((long long)who) - 1;
  return Best{umax, pmin, __builtin_amdgcn_readlane(slot, src)};
}
// (score smaller, then position larger) wins: the order in which tokens are evicted.
__device__ __forceinline__ bool evicts_before(double s, int p, int sl, const Best& b) {
  return sl >= 0 && (b.slot < 0 || s < b.u || (s == b.u && p > b.pos));
}
// Wavefront-wide first of that order, for one entry per lane whose positions are all different.
__device__ __forceinline__ Best fast_wave_first_evicted(const Best& b) {
  const bool live = b.slot >= 0;
  const double smin = -fast_wave_max(live ? -b.u : -INFINITY);
  const bool top = live && b.u == smin;
  const int pmax = -fast_wave_min(top ? -b.pos : 0x7FFFFFFF);
  const unsigned long long who = __ballot(top && b.pos == pmax);
  if (who == 0ull) return Best{0.0, 0, -1};
  const int src = __ffsll((long long)who) - 1;
  return Best{smin, pmax, __builtin_amdgcn_readlane(b.slot, src)};
}
// Eq. 9 arg-max result -> Eq. 10 threshold, Eq. 11-12 merge with one source, slot bookkeeping.
// Called by every thread of a workgroup (at least D threads) with block-uniform arguments.
// told: the head's threshold before the step; (kl, vl): this thread's element of the last slot's
// row as it was before the step; (sl, pl): that slot's updated score and its position.
template <typename T, int D>
__device__ __forceinline__ void finish_head(const DecodeArgs& a, int64_t lbh, int64_t slot0, int es, int total,
                                            double best, int bp, int bs, double told, T kl, T vl, double sl,
                                            int pl, double* red) {
  T* Kc = static_cast<T*>(a.cK) + slot0 * D;
  T* Vc = static_cast<T*>(a.cV) + slot0 * D;
  const int tid = threadIdx.x, last = total - 1;
  bool do_merge;
  if (isnan(a.tau_force)) {
    const double tnew = isnan(told) ? best : __dadd_rn(__dmul_rn(a.beta, best), __dmul_rn(1.0 - a.beta, told));
    do_merge = best >= tnew;
    if (tid == 0) a.ctau[lbh] = tnew;
  } else {
    do_merge = best >= a.tau_force;
  }
  if (tid == 0) {
    a.ev_evicted[lbh] = es == last ? pl : a.cpos[slot0 + es];
    a.ev_target[lbh] = do_merge ? bp : -1;
    a.ev_ustar[lbh] = best;
    a.ccount[lbh] = last;
  }
  // exp(1), the retained token's self-similarity weight; average merging weighs both rows 1
  const double e1 = a.merge_average ? 1.0 : 2.718281828459045;
  const double w = a.merge_average ? 1.0 : exp(best);
  const double z = __dadd_rn(e1, w);
  if constexpr (sizeof(T) == 1) {
    // fp8 cache: rows are codes times the row's power of two.  The merged row is rounded to the
    // cache's logical type (bf16) and encoded again with a power of two of its own, which takes
    // its largest magnitude: a reduction over the workgroup (`red`: one double per wavefront).
    int8_t* Ke = a.cKe + slot0;
    int8_t* Ve = a.cVe + slot0;
    int ekl = Ke[last], evl = Ve[last];  // the last row's powers of two travel with its codes
    if (do_merge) {
      double km = 0.0, vm = 0.0;
      if (tid < D) {
        const double ke = Elem<T>::to_f64(es == last ? kl : Kc[int64_t(es) * D + tid]) * pow2_f64(Ke[es]);
        const double ve = Elem<T>::to_f64(es == last ? vl : Vc[int64_t(es) * D + tid]) * pow2_f64(Ve[es]);
        const double kt = Elem<T>::to_f64(bs == last ? kl : Kc[int64_t(bs) * D + tid]) * pow2_f64(Ke[bs]);
        const double vt = Elem<T>::to_f64(bs == last ? vl : Vc[int64_t(bs) * D + tid]) * pow2_f64(Ve[bs]);
        const double kk = __dadd_rn(__dmul_rn(e1, kt), __dmul_rn(w, ke));
        const double vv = __dadd_rn(__dmul_rn(e1, vt), __dmul_rn(w, ve));
        km = Elem<uint16_t>::to_f64(Elem<uint16_t>::from_f64(kk / z));
        vm = Elem<uint16_t>::to_f64(Elem<uint16_t>::from_f64(vv / z));
      }
      const double ak = wave_max(fabs(km)), av = wave_max(fabs(vm));
      __syncthreads();
      if ((tid & 63) == 0) {
        red[tid >> 6] = ak;
        red[4 + (tid >> 6)] = av;
      }
      __syncthreads();
      const int ek = fp8_row_exponent(fmax(fmax(red[0], red[1]), fmax(red[2], red[3])));
      const int ev = fp8_row_exponent(fmax(fmax(red[4], red[5]), fmax(red[6], red[7])));
      const T kc = fp8_encode(ldexp(km, -ek)), vc = fp8_encode(ldexp(vm, -ev));
      if (bs == last) {  // the merged row is the one that moves into the hole
        kl = kc;
        vl = vc;
        ekl = ek;
        evl = ev;
      } else {
        if (tid < D) {
          Kc[int64_t(bs) * D + tid] = kc;
          Vc[int64_t(bs) * D + tid] = vc;
        }
        if (tid == 0) {
          Ke[bs] = int8_t(ek);
          Ve[bs] = int8_t(ev);
        }
      }
    }
    if (es != last) {  // the last slot fills the hole
      if (tid < D) {
        Kc[int64_t(es) * D + tid] = kl;
        Vc[int64_t(es) * D + tid] = vl;
      }
      if (tid == 0) {
        Ke[es] = int8_t(ekl);
        Ve[es] = int8_t(evl);
      }
    }
  } else {
    if (tid < D) {
      if (do_merge) {
        const T ke = es == last ? kl : Kc[int64_t(es) * D + tid], ve = es == last ? vl : Vc[int64_t(es) * D + tid];
        const T kt = bs == last ? kl : Kc[int64_t(bs) * D + tid], vt = bs == last ? vl : Vc[int64_t(bs) * D + tid];
        const double kk = __dadd_rn(__dmul_rn(e1, Elem<T>::to_f64(kt)), __dmul_rn(w, Elem<T>::to_f64(ke)));
        const double vv = __dadd_rn(__dmul_rn(e1, Elem<T>::to_f64(vt)), __dmul_rn(w, Elem<T>::to_f64(ve)));
        const T km = Elem<T>::from_f64(kk / z), vm = Elem<T>::from_f64(vv / z);
        if (bs == last) {  // the merged row is the one that moves into the hole
          kl = km;
          vl = vm;
        } else {
          Kc[int64_t(bs) * D + tid] = km;
          Vc[int64_t(bs) * D + tid] = vm;
        }
      }
      if (es != last) {  // the last slot fills the hole
        Kc[int64_t(es) * D + tid] = kl;
        Vc[int64_t(es) * D + tid] = vl;
      }
    }
  }
  if (es != last && tid == 0) {
    a.cscore[slot0 + es] = sl;
    a.cpos[slot0 + es] = pl;
  }
}

// Cosine of the evicted key against every other row of the head (Eq. 9) by the whole workgroup;
// returns the arg-max per wavefront-reduced lane (the caller reduces over the wavefronts).
// ke: D doubles of shared memory, red: one double per wavefront.  NT = threads of the workgroup.
template <typename T, int D, int NT = 256>
__device__ __forceinline__ Best scan_matches(const DecodeArgs& a, int64_t slot0, int es, int total, double* ke,
                                             double* red) {
  constexpr int kVec = 16 / sizeof(T);
  constexpr int TPR = D / kVec;
  constexpr int RPP = NT / TPR;
  const int tid = threadIdx.x;
  const T* Kc = static_cast<const T*>(a.cK) + slot0 * D;
  double part = 0.0;
  __syncthreads();
  if (tid < D) {
    double x = Elem<T>::to_f64(Kc[int64_t(es) * D + tid]);
    if constexpr (sizeof(T) == 1) x *= pow2_f64(a.cKe[slot0 + es]);
    ke[tid] = x;
    part = x * x;
  }
  const double sne = sqrt(block_sum(part, red));
  const int tr = tid / TPR, tc = (tid % TPR) * kVec;
  Best m{0.0, 0, -1};
  for (int r0 = 0; r0 < total; r0 += RPP) {
    const int j = r0 + tr;
    double dot = 0.0, nr = 0.0;
    if (j < total) {
      double x[kVec];
      cvt16<T>(*reinterpret_cast<const u32x4*>(Kc + int64_t(j) * D + tc), x);
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        dot = fma(x[e], ke[tc + e], dot);
        nr = fma(x[e], x[e], nr);
      }
    }
#pragma unroll
    for (int o = TPR / 2; o > 0; o >>= 1) {
      dot += __shfl_xor(dot, o, 64);
      nr += __shfl_xor(nr, o, 64);
    }
    if constexpr (sizeof(T) == 1) {  // the row's power of two: exact on sums that are exact
      const double sc = pow2_f64(a.cKe[slot0 + min(j, total - 1)]);
      dot *= sc;
      nr *= sc * sc;
    }
    if (j < total && j != es && (tid % TPR) == 0) {
      const double den = sne * sqrt(nr);
      const double u = den > 0.0 ? dot / den : 0.0;
      const int p = a.cpos[slot0 + j];
      if (better_match(u, p, j, m)) m = Best{u, p, j};
    }
  }
  return m;
}


// The end of a head's closing work, by a workgroup of 256 threads.  On entry every thread holds
// its own first-evicted entry `ev` and its sorted list `low` of the next step's lowest evictable
// entries (a thread's entries belong to slots no other thread holds); LDS holds, per wavefront
// and candidate, the best match found (`wcm_u`, `wcm_ps` = (position, slot)), the last slot's
// updated score and position (sred[4], ired[8]) and its row as it was before the step
// (`park_kv`: K at [0, D), V at [256, 256 + D)).  The function reduces them over the workgroup,
// writes the next step's candidates, resets the head's ticket, finds the merge target (from the
// candidates' results, else by a pass over the head's keys) and finishes the step.
template <typename T, int D>
__device__ __forceinline__ void close_head(const DecodeArgs& a, int64_t lbh, int64_t slot0, int total, bool evict,
                                           Best ev, Best (&low)[kCand + 1], const int (&cl)[kCand], double told,
                                           double* sred, int* ired, double* dred, const double* wcm_u,
                                           const int2* wcm_ps, const T* park_kv) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int last = total - 1;
  // evicted token: block-wide
  ev = fast_wave_first_evicted(ev);
  lds_barrier();
  if (lane == 0) {
    sred[w] = ev.u;
    ired[w] = ev.pos;
    ired[4 + w] = ev.slot;
  }
  lds_barrier();
  const double s_last = sred[4];
  const int p_last = ired[8];
  ev = Best{sred[0], ired[0], ired[4]};
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (evicts_before(sred[i], ired[i], ired[4 + i], ev)) ev = Best{sred[i], ired[i], ired[4 + i]};
  const int es = evict ? ev.slot : -1;  // a candidate always exists: total > budget >= T + M
  // the kCand + 1 lowest of the next step's evictable tokens: repeated block-wide extraction
  int nxt[kCand + 1];
#pragma unroll
  for (int r = 0; r <= kCand; ++r) {
    Best h = fast_wave_first_evicted(low[0]);
    lds_barrier();
    if (lane == 0) {
      sred[w] = h.u;
      ired[w] = h.pos;
      ired[4 + w] = h.slot;
    }
    lds_barrier();
    h = Best{sred[0], ired[0], ired[4]};
#pragma unroll
    for (int i = 1; i < 4; ++i)
      if (evicts_before(sred[i], ired[i], ired[4 + i], h)) h = Best{sred[i], ired[i], ired[4 + i]};
    nxt[r] = h.slot;
    if (h.slot >= 0 && low[0].slot == h.slot) {  // the owner pops its head
#pragma unroll
      for (int i = 0; i < kCand; ++i) low[i] = low[i + 1];
      low[kCand].slot = -1;
    }
  }
  int ci = -1;
#pragma unroll
  for (int i = kCand - 1; i >= 0; --i)
    if (es >= 0 && cl[i] == es) ci = i;
  if (tid == 0) {  // the next step's candidates (every thread holds this step's list in registers)
    int k = 0;
    for (int r = 0; r <= kCand && k < kCand; ++r) {
      int s = nxt[r];
      if (s < 0 || s == es) continue;
      if (es >= 0 && s == last) s = es;  // the last slot is about to move into the freed one
      a.cand[lbh * kCand + k++] = s;
    }
    for (; k < kCand; ++k) a.cand[lbh * kCand + k] = -1;
    st_agent(&a.ticket[lbh], 0u);
  }
  if (!evict) {
    if (tid == 0) {
      a.ccount[lbh] = total;
      a.ev_evicted[lbh] = -1;
      a.ev_target[lbh] = -1;
      a.ev_ustar[lbh] = __longlong_as_double(0x7FF8000000000000ll);
    }
    return;
  }
  Best m{0.0, 0, -1};
  if (ci < 0) {
    // Not foreseen (the first step after a cache import, or a candidate overtaken by a token
    // outside the list): a second pass over the head's keys.
    if (tid == 0) a.cmiss[lbh] += 1u;
    m = scan_matches<T, D>(a, slot0, es, total, dred, sred);
  } else {
    if (tid < 4) {  // the four wavefronts' results (written before the barriers of the score pass)
      const int2 q = wcm_ps[tid * kCand + ci];
      m = Best{wcm_u[tid * kCand + ci], q.x, q.y};
    }
  }
  m = fast_wave_best_match(m.u, m.pos, m.slot);
  lds_barrier();
  if (lane == 0) {
    sred[w] = m.u;
    ired[w] = m.pos;
    ired[4 + w] = m.slot;
  }
  lds_barrier();
  m = Best{sred[0], ired[0], ired[4]};
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (better_match(sred[i], ired[i], ired[4 + i], m)) m = Best{sred[i], ired[i], ired[4 + i]};
  T kl = T(), vl = T();
  if (tid < D) {
    kl = park_kv[tid];
    vl = park_kv[256 + tid];
  }
  finish_head<T, D>(a, lbh, slot0, es, total, m.u, m.pos, m.slot, told, kl, vl, s_last, p_last, sred);
}

// The two launches that close the heads with more than a.big_rows entries (decode_split.hip).
// `max_chunks[i]`: the chunks the largest head of the call's layer i can occupy in this step.
hipError_t launch_decode_split(d2o_ctx* c, const DecodeArgs& attend, const int* max_chunks, int nl, View out,
                               hipStream_t s);

}  // namespace dec

}  // namespace d2o
