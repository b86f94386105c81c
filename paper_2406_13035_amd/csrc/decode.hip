// One generation step over the compressed cache (Sec. 3 Eq. 2-3; Sec. 4.2 Eq. 6-12), for a
// range of layers in one set of launches.  The step is bound by HBM traffic, so the design
// reads every K and V row of every layer exactly once per step:
//
//   decode_prepare  per (layer, sequence, KV head): writes the new token's k, v into the free
//                   slot (score 0, its position) and lays out, in fp64, the vectors the
//                   attention pass multiplies every cache key with: the G queries and the keys
//                   of kCand eviction candidates chosen at the end of the previous step.
//   decode_attend   one workgroup per chunk of 256 slots, each of its four wavefronts working
//                   alone on 64 of them.  K pass: the keys go through LDS so that one lane owns
//                   one cache row; the lane forms, in fp64, the G logits, the dot products with
//                   the candidate keys and the row's squared norm (the vectors come in through
//                   scalar loads, so there is no cross-lane reduction).  Then the softmax
//                   statistics of the 64 rows, the candidates' best cosine among them (Eq. 9),
//                   and the partial P V in fp32.
//                   The last workgroup of a head to finish (a ticket counter, no waiting)
//                   closes the head: output rows, exact fp64 normaliser, score update (Eq. 6,
//                   generation case), the token to evict (Eq. 7-8: lowest score outside sinks
//                   and the recent window; equal scores evict the later position) and the
//                   candidates of the next step (the lowest scores that remain).  When the
//                   evicted token is one of this step's candidates, which is the normal case,
//                   its similarities are already there; otherwise (the first step after a cache
//                   import, or a candidate overtaken by a token outside the list) the same
//                   workgroup makes a second pass over the head's keys.  Then: arg-max (ties:
//                   earlier position), EMA threshold (Eq. 10, update first, then test), merge
//                   or discard (Eq. 11-12 with one source), and the last slot moves into the
//                   freed one.
//
// All decision-bearing arithmetic - logits, softmax normaliser, score accumulation, eviction
// arg-min, cosine arg-max, EMA threshold, merge - is fp64 in the operation order of the
// defining formulas; only the attention output (P V) accumulates in fp32.
// Slots are physically unordered; a token's identity is its position.
#include <algorithm>
#include <type_traits>

#include "decode_common.h"

namespace d2o {

// Scratch memory of d2o_decode_step_static: the partial results and operand vectors of one
// generation step, for callers that cannot hand over (or allocate) a scratch workspace.  One
// copy per GPU, held from the moment the library's code is loaded on it until the process ends.
// In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device, and is what kernels and launchers are given.
constexpr size_t kStaticScratchBytes = size_t(64) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
unsigned char* g_static_scratch[kMaxDevices] = {};  // device address of `scratch` per device (0: not looked up yet)

}  // namespace

// Device address of the static scratch array on the current device (looked up on the first
// call per device; allocates nothing: the array is part of the loaded code object).
hipError_t static_scratch_address(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  unsigned char* p = __atomic_load_n(&g_static_scratch[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!sym) return hipErrorInvalidSymbol;
    p = static_cast<unsigned char*>(sym);
    __atomic_store_n(&g_static_scratch[dev], p, __ATOMIC_RELEASE);  // every thread would store the same address
  }
  *out = p;
  return hipSuccess;
}

namespace {

using namespace dec;

// T: the cache's element type (uint8_t: fp8 codes), IT: the type of q, k_new, v_new.
template <typename T, typename IT, int D, int G>
__global__ __launch_bounds__(128) void decode_prepare(DecodeArgs a, const IT* __restrict__ q, View qv,
                                                      const IT* __restrict__ kn, View kv, const IT* __restrict__ vn,
                                                      View vv) {
  __shared__ double red[2 * kCand > 4 ? 2 * kCand : 4];
  const int li = blockIdx.y, l = a.layer0 + li, b = blockIdx.x / a.Hkv, hk = blockIdx.x % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int count = a.ccount[lbh];
  const int64_t slot0 = (int64_t(b) * a.Hkv + hk) * a.slots + a.meta[lbh * 4 + 0];
  const int c = threadIdx.x;
  T* Kc = static_cast<T*>(a.cK) + slot0 * D;
  T* Vc = static_cast<T*>(a.cV) + slot0 * D;
  if constexpr (sizeof(T) == 1) {
    // fp8 cache: the new row is encoded as it enters the cache (its largest magnitude decides
    // the row's power of two: a reduction over the two wavefronts)
    static_assert(D == 128, "one element per thread");
    const double kx = Elem<IT>::to_f64(kn[li * kv.sn + b * kv.sb + hk * kv.sh + c]);
    const double vx = Elem<IT>::to_f64(vn[li * vv.sn + b * vv.sb + hk * vv.sh + c]);
    const double ak = wave_max(fabs(kx)), av = wave_max(fabs(vx));
    if ((c & 63) == 0) {
      red[c >> 6] = ak;
      red[2 + (c >> 6)] = av;
    }
    __syncthreads();
    const int ek = fp8_row_exponent(fmax(red[0], red[1])), ev = fp8_row_exponent(fmax(red[2], red[3]));
    Kc[int64_t(count) * D + c] = fp8_encode(ldexp(kx, -ek));
    Vc[int64_t(count) * D + c] = fp8_encode(ldexp(vx, -ev));
    if (c == 0) {
      a.cKe[slot0 + count] = int8_t(ek);
      a.cVe[slot0 + count] = int8_t(ev);
    }
    __syncthreads();  // `red` is used again below
  } else {
    if (c < D) {
      Kc[int64_t(count) * D + c] = kn[li * kv.sn + b * kv.sb + hk * kv.sh + c];
      Vc[int64_t(count) * D + c] = vn[li * vv.sn + b * vv.sb + hk * vv.sh + c];
    }
  }
  if (c == 0) {
    a.cscore[slot0 + count] = 0.0;
    a.cpos[slot0 + count] = a.new_pos;
    // The step's entry count gets a word of its own: the head's closing workgroup overwrites
    // ccount while other workgroups of the same launch may not have started yet, and those
    // must still see the count the step began with.
    a.ctotal[lbh] = count + 1;
  }
  double* vec = a.vecs + lbh * (G + kCand) * D;
#pragma unroll
  for (int g = 0; g < G; ++g)
    if (c < D) vec[g * D + c] = Elem<IT>::to_f64(q[li * qv.sn + b * qv.sb + (hk * G + g) * qv.sh + c]);
  // the candidates' keys: all slot numbers first, then all rows, then one exchange for the
  // norms (one memory round trip each instead of one per candidate)
  int cs[kCand];
#pragma unroll
  for (int i = 0; i < kCand; ++i) cs[i] = a.cand[lbh * kCand + i];  // older slots: never the one just written
  double x[kCand], part[kCand];
#pragma unroll
  for (int i = 0; i < kCand; ++i) {
    x[i] = (cs[i] >= 0 && c < D) ? Elem<T>::to_f64(Kc[int64_t(cs[i]) * D + c]) : 0.0;
    if constexpr (sizeof(T) == 1) x[i] *= pow2_f64(a.cKe[slot0 + max(cs[i], 0)]);
  }
#pragma unroll
  for (int i = 0; i < kCand; ++i) {
    if (c < D) vec[(G + i) * D + c] = x[i];
    part[i] = wave_sum(x[i] * x[i]);
  }
  if ((c & 63) == 0) {
#pragma unroll
    for (int i = 0; i < kCand; ++i) red[(c >> 6) * kCand + i] = part[i];
  }
  __syncthreads();
  if (c < kCand) a.cnorm[lbh * kCand + c] = sqrt(red[c] + red[kCand + c]);  // wavefront 0's sum first
}

// Softmax maximum and exact normaliser sum_j exp(s_j - max) of each query head of one head, from
// its sub-chunk records (fixed summation tree), by one workgroup of 256 threads of the launch
// that wrote the records; result: hn[g] = maximum, hn[G + g] = normaliser.
template <int G>
__device__ __forceinline__ void head_normaliser(const DecodeArgs& a, int64_t bh, int ch0, int nsub, double* hn,
                                                double* dred, double* sred) {
  constexpr int kRec = rec_doubles(G);
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  double Mg[G], part[G];
#pragma unroll
  for (int g = 0; g < G; ++g) Mg[g] = -INFINITY;
  for (int c = tid; c < nsub; c += 256) {
    const int64_t x = sub_index(a, bh, ch0, c) * kRec;
#pragma unroll
    for (int g = 0; g < G; ++g) Mg[g] = fmax(Mg[g], ld_agent(&a.rec[x + g]));
  }
#pragma unroll
  for (int g = 0; g < G; ++g) Mg[g] = wave_max(Mg[g]);
  __syncthreads();
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) dred[w * G + g] = Mg[g];
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < G; ++g) {
    Mg[g] = fmax(fmax(dred[g], dred[G + g]), fmax(dred[2 * G + g], dred[3 * G + g]));
    part[g] = 0.0;
  }
  for (int c = tid; c < nsub; c += 256) {
    const int64_t x = sub_index(a, bh, ch0, c) * kRec;
#pragma unroll
    for (int g = 0; g < G; ++g) part[g] += ld_agent(&a.rec[x + G + g]) * exp(ld_agent(&a.rec[x + g]) - Mg[g]);
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const double lg = block_sum(part[g], sred);
    if (tid == 0) {
      hn[g] = Mg[g];
      hn[G + g] = lg;
    }
  }
}

// Closing work of a head, by one workgroup of 256 threads: combine the sub-chunks, update the
// scores, choose the evicted token and the next candidates, find the merge target and finish the
// step.  Every load whose address does not depend on a result of this function is issued before
// the first of the workgroup-wide reductions, so the function costs a few memory round trips.
template <typename T, typename OT, int D, int G>
__device__ __forceinline__ void head_tail(const DecodeArgs& a, OT* __restrict__ out, const View& ov, int li, int b,
                                          int hk, int64_t lbh, int total, int nsub, double* sred, int* ired,
                                          float* fred, double* dred, unsigned char* park) {
  constexpr int kRec = rec_doubles(G);
  constexpr int U = G >= 8 ? 1 : G >= 4 ? 3 : G >= 2 ? 4 : 6;  // slots per thread and batch of the score pass
  constexpr int C4 = D / 4;                           // threads across an output row (four columns each)
  constexpr int RG = 256 / C4;                        // groups of threads that share the sub-chunks
  constexpr int PB = 4;                               // partial rows in flight per thread
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int last = total - 1;
  const int32_t* mt = a.meta + lbh * 4;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt[0];
  const int ch0 = mt[3];  // the layer's first chunk in the partial-result arrays
  const T* Kc = static_cast<const T*>(a.cK) + slot0 * D;
  const T* Vc = static_cast<const T*>(a.cV) + slot0 * D;
  // ---- loads that depend on nothing: the threshold, this step's candidates, the last slot's row
  const double told = a.ctau[lbh];
  int cl[kCand];
#pragma unroll
  for (int i = 0; i < kCand; ++i) cl[i] = a.cand[lbh * kCand + i];
  // Results that are needed only at the end wait in LDS, not in registers: per wavefront and
  // candidate the best match found so far (`wcm`), and the last slot's row (two elements per thread).
  double* wcm_u = sred + 8 + 8;                            // [4][kCand], behind sred and ired
  int2* wcm_ps = reinterpret_cast<int2*>(wcm_u + 4 * kCand);  // [4][kCand] (position, slot)
  T* park_kv = reinterpret_cast<T*>(wcm_ps + 4 * kCand);
  if (tid < D) {
    park_kv[tid] = Kc[int64_t(last) * D + tid];
    park_kv[256 + tid] = Vc[int64_t(last) * D + tid];
  }
  // ---- head maximum and exact normaliser sum_j exp(s_j - max) of each query head (fixed tree),
  //      all query heads in one sweep over the sub-chunk records.  exp(m_sub - max) of every
  //      sub-chunk and query head is kept in LDS (`em`, behind the parked values) for the output
  //      and score passes; for a head with more sub-chunks than fit, the factors overwrite the
  //      maxima in the records and the score pass brings them into LDS segment by segment.
  constexpr int kEmCap = (kStageBytes - 8192) / int(sizeof(double));
  double* em = reinterpret_cast<double*>(park);  // [nsub][G]
  const bool em_lds = nsub * G <= kEmCap;
  double Mg[G], Lg[G];
  // The record of sub-chunk `tid` (the only one of this thread unless the head has more than 256
  // sub-chunks) is read once, whole, and kept: the sweeps below then cost one memory round trip
  // instead of three.
  double own_m[G], own_l[G], own_u[kCand];
  int own_s[kCand];
  {
#pragma unroll
    for (int g = 0; g < G; ++g) Mg[g] = -INFINITY;
    for (int c = tid; c < nsub; c += 256) {
      const int64_t x = sub_index(a, bh, ch0, c) * kRec;
      if (c == tid) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          own_m[g] = ld_agent(&a.rec[x + g]);
          own_l[g] = ld_agent(&a.rec[x + G + g]);
        }
#pragma unroll
        for (int i = 0; i < kCand; ++i) {
          own_u[i] = ld_agent(&a.rec[x + 2 * G + i]);
          own_s[i] = int(ld_agent(&a.rec[x + 2 * G + kCand + i]));
        }
#pragma unroll
        for (int g = 0; g < G; ++g) Mg[g] = fmax(Mg[g], own_m[g]);
      } else {
#pragma unroll
        for (int g = 0; g < G; ++g) Mg[g] = fmax(Mg[g], ld_agent(&a.rec[x + g]));
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) Mg[g] = wave_max(Mg[g]);
    __syncthreads();
    if (lane == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) dred[w * G + g] = Mg[g];
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < G; ++g) Mg[g] = fmax(fmax(dred[g], dred[G + g]), fmax(dred[2 * G + g], dred[3 * G + g]));
    double part[G];
#pragma unroll
    for (int g = 0; g < G; ++g) part[g] = 0.0;
    for (int c = tid; c < nsub; c += 256) {
      const int64_t x = sub_index(a, bh, ch0, c) * kRec;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const double t = exp((c == tid ? own_m[g] : ld_agent(&a.rec[x + g])) - Mg[g]);
        part[g] += (c == tid ? own_l[g] : ld_agent(&a.rec[x + G + g])) * t;
        if (em_lds)
          em[c * G + g] = t;
        else
          st_agent(&a.rec[x + g], t);  // the factor replaces the maximum (nobody needs it again)
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) Lg[g] = block_sum(part[g], sred);
    __syncthreads();  // `em` is complete (in memory: the stores have been acknowledged)
    // the table holds the factors already divided by the normaliser: a probability is then
    // one product, exp(s_j - m_sub) * em
    if (em_lds) {
      for (int c = tid; c < nsub; c += 256) {
#pragma unroll
        for (int g = 0; g < G; ++g) em[c * G + g] /= Lg[g];
      }
      lds_barrier();
    }
  }
  // ---- Eq. 9 arg-max over the sub-chunks' results, for every candidate of this step (which of
  //      them is evicted is not known yet; ties: earlier position)
  Best cm[kCand];
#pragma unroll
  for (int i = 0; i < kCand; ++i) cm[i] = Best{0.0, 0, -1};
  for (int c = tid; c < nsub; c += 256) {
    const int64_t x = sub_index(a, bh, ch0, c) * kRec;
#pragma unroll
    for (int i = 0; i < kCand; ++i) {
      const int s = c == tid ? own_s[i] : int(ld_agent(&a.rec[x + 2 * G + kCand + i]));
      if (s >= 0) {
        const double u = c == tid ? own_u[i] : ld_agent(&a.rec[x + 2 * G + i]);
        const int p = a.cpos[slot0 + s];
        if (better_match(u, p, s, cm[i])) cm[i] = Best{u, p, s};
      }
    }
  }
#pragma unroll
  for (int i = 0; i < kCand; ++i) {  // (a thread's entries come from different sub-chunks: all positions differ)
    const Best r = fast_wave_best_match(cm[i].u, cm[i].pos, cm[i].slot);
    if (lane == 0) {
      wcm_u[w * kCand + i] = r.u;
      wcm_ps[w * kCand + i] = make_int2(r.pos, r.slot);
    }
  }
  // ---- score pass, set-up
  const bool evict = total > mt[1];
  const int recent = mt[2];
  Best ev{0.0, 0, -1};
  Best low[kCand + 1];
#pragma unroll
  for (int i = 0; i <= kCand; ++i) low[i] = Best{0.0, 0, -1};
  double sc[U], e[U][G];
  int ps[U];
  int seg0 = 0, jend = total;  // the segment of sub-chunks whose factors `em` holds, and its last slot + 1
  auto load_batch = [&](int j0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = min(j0 + u * 256, jend - 1);
      sc[u] = a.cscore[slot0 + j];
      ps[u] = a.cpos[slot0 + j];
#pragma unroll
      for (int g = 0; g < G; ++g) e[u][g] = ld_agent(&a.elog[elog_index(a, bh, ch0, G, g, j)]);
    }
  };
  // Eq. 6 for the batch's slots, the token to evict (Eq. 7-8 on count+1 entries) and the lowest
  // scores among the tokens evictable at the next step
  auto apply_batch = [&](int j0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = j0 + u * 256;
      if (j < jend) {
        double s2 = sc[u];
#pragma unroll
        for (int g = 0; g < G; ++g) s2 = fma(e[u][g], em[(j / kSub - seg0) * G + g], s2);
        a.cscore[slot0 + j] = s2;
        const int p = ps[u];
        if (j == last) {  // kept for the move into the freed slot
          sred[4] = s2;
          ired[8] = p;
        }
        if (p >= a.n_sink && p <= a.new_pos - recent && evicts_before(s2, p, j, ev)) ev = Best{s2, p, j};
        if (p >= a.n_sink && p <= a.new_pos + 1 - recent && evicts_before(s2, p, j, low[kCand])) {
          low[kCand] = Best{s2, p, j};
#pragma unroll
          for (int i = kCand; i > 0; --i)
            if (evicts_before(low[i].u, low[i].pos, low[i].slot, low[i - 1])) {
              const Best t = low[i - 1];
              low[i - 1] = low[i];
              low[i] = t;
            }
        }
      }
      __builtin_amdgcn_sched_barrier(0);  // one slot after the other: interleaving them costs registers
    }
  };
  // ---- output rows: thread (rg, c4) adds the chunks rg, rg + RG, ... of four columns, PB
  //      loads in flight; the groups' sums are added in ascending order
  const int c4 = tid % C4, rg = tid / C4;
  const int nchunk = (nsub + 3) / 4;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float num[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = rg; c0 < nchunk; c0 += PB * RG) {
      float4 v[PB];
      double fc[PB];
#pragma unroll
      for (int u = 0; u < PB; ++u) {
        const int cc = min(c0 + u * RG, nchunk - 1);
        v[u] = ld_agent4(a.pacc + (chunk_index(a, bh, ch0, cc) * G + g) * D + c4 * 4);
        fc[u] = 0.0;  // exp(chunk maximum - max): the largest of its sub-chunks' factors
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (cc * 4 + i < nsub)
            fc[u] = fmax(fc[u], em_lds ? em[(cc * 4 + i) * G + g]
                                       : ld_agent(&a.rec[sub_index(a, bh, ch0, cc * 4 + i) * kRec + g]) / Lg[g]);
      }
#pragma unroll
      for (int u = 0; u < PB; ++u) {
        const float f = c0 + u * RG < nchunk ? float(fc[u]) : 0.f;
        num[0] = fmaf(v[u].x, f, num[0]);
        num[1] = fmaf(v[u].y, f, num[1]);
        num[2] = fmaf(v[u].z, f, num[2]);
        num[3] = fmaf(v[u].w, f, num[3]);
      }
    }
    lds_barrier();
#pragma unroll
    for (int e = 0; e < 4; ++e) fred[e * 256 + tid] = num[e];
    lds_barrier();
    if (tid < D) {  // column tid: element tid % 4 of the threads (rg, tid / 4)
      const float* fr = fred + (tid % 4) * 256 + tid / 4;
      float t = fr[0];
#pragma unroll
      for (int i = 1; i < RG; ++i) t += fr[i * C4];
      out[li * ov.sn + b * ov.sb + (hk * G + g) * ov.sh + tid] = Elem<OT>::from_f32(t);
    }
    __builtin_amdgcn_sched_barrier(0);  // one query head after the other (registers)
  }
  // ---- score pass: batches of U slots per thread, their loads in flight together
  constexpr int kSegSubs = kEmCap / G;  // sub-chunks whose factors fit `em`
#pragma unroll 1
  for (seg0 = 0; seg0 < nsub; seg0 += kSegSubs) {
    const int nseg = min(kSegSubs, nsub - seg0);
    jend = min(total, (seg0 + nseg) * kSub);
    if (!em_lds) {  // a head of several segments: (re)fill the table for this one
      lds_barrier();
#pragma unroll 1
      for (int i = tid; i < nseg * G; i += 256) {
        double lg = Lg[0];
#pragma unroll
        for (int g = 1; g < G; ++g) lg = (i % G == g) ? Lg[g] : lg;
        em[i] = ld_agent(&a.rec[sub_index(a, bh, ch0, seg0 + i / G) * kRec + i % G]) / lg;
      }
      lds_barrier();
    }
#pragma unroll 1
    for (int j0 = seg0 * kSub + tid; j0 < jend; j0 += U * 256) {
      load_batch(j0);
      apply_batch(j0);
    }
  }
  close_head<T, D>(a, lbh, slot0, total, evict, ev, low, cl, told, sred, ired, dred, wcm_u, wcm_ps, park_kv);
}

template <typename T, typename OT, int D, int G>
__global__ __launch_bounds__(256) void decode_attend(DecodeArgs a, OT* __restrict__ out, View ov) {
  constexpr int VB = sizeof(T) == 1 ? 8 : 16;   // V pass: bytes per lane and load (fp8: 8, which keeps the
                                                // partial sums at eight per lane and query head)
  constexpr int kVec = VB / sizeof(T);          // elements per load
  typedef typename RawBits<VB>::type VRaw;
  constexpr int RB = D * sizeof(T);             // bytes of a cache row
  constexpr int NP = RB / kPiece;               // row pieces staged through LDS
  constexpr int EP = kPiece / sizeof(T);        // elements of a piece
  constexpr int TPR = RB / VB;                  // V pass: lanes per row
  constexpr int RPI = 64 / TPR;                 // V pass: rows per load instruction
  constexpr int NVL = kSub / RPI;               // V pass: loads per lane
  constexpr int NV = G + kCand;
  constexpr int kRec = rec_doubles(G);
  constexpr int ES = NV <= 4 ? 4 : 2;           // elements per K-pass step (scalar register budget)
  constexpr int NST = EP / ES;                  // steps per piece (even)
  typedef typename RawBits<ES * sizeof(T)>::type Raw;
  __shared__ __attribute__((aligned(16))) unsigned char stage[kStageBytes];
  __shared__ float ps[4][G][kSub];
  __shared__ double wmax[4][G];  // per wavefront: softmax maximum of its sub-chunk (-inf: no rows)
  __shared__ int sh_last;

  // Grid: x = head (fastest), y = flat chunk group over the layers.  Workgroups go round-robin to
  // the XCDs in index order, so with a head count that is a multiple of the XCD count every chunk
  // of a head, and the workgroup that closes it, run on one XCD.
  const int entry = find_entry(a, blockIdx.y), grp = blockIdx.y - a.lay_off[entry];
  const int li = a.lay_id[entry];
  const int l = a.layer0 + li, b = blockIdx.x / a.Hkv, hk = blockIdx.x % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  // Everything the workgroup needs to know about its head comes through the scalar cache in one
  // round trip (the loads are independent of each other): the fill level, the layer's slot and
  // sub-chunk offsets, the candidates.  The kernel that wrote them has completed.
  typedef const int32_t __attribute__((address_space(4))) * ciptr;
  typedef const double __attribute__((address_space(4))) * cptr;
  const ciptr mt = (ciptr)a.meta + lbh * 4;
  const int total = ((ciptr)a.ctotal)[lbh];  // the new token has been appended; constant during this launch
  const int mt0 = mt[0], mt3 = mt[3];
  int cs[kCand];
  double cn[kCand];
#pragma unroll
  for (int c = 0; c < kCand; ++c) {
    cs[c] = ((ciptr)a.cand)[lbh * kCand + c];
    cn[c] = ((cptr)a.cnorm)[lbh * kCand + c];
  }
  asm volatile("" ::"s"(total), "s"(mt0), "s"(mt3));  // all of them are on their way before the first wait
  if (grp * kGroup * kChunk >= total) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt0;
  const unsigned char* Kh = static_cast<const unsigned char*>(a.cK) + slot0 * RB;
  const unsigned char* Vh = static_cast<const unsigned char*>(a.cV) + slot0 * RB;
  // A workgroup owns kGroup consecutive chunks of 256 slots; each wavefront works alone on 64
  // rows ("sub-chunk") of each of them, in a software pipeline: while it computes on one
  // sub-chunk, the V rows of that sub-chunk and the K rows of its next one are in flight.
  // There is no workgroup barrier until the ticket.
  cptr S = (cptr)(a.vecs + lbh * NV * D);
  unsigned char* mine = stage + w * 64 * kPitch;
  int ln = lane;  // the lane number as the loop body sees it
  const double root_d = sqrt(double(D));
  // K loads of a sub-chunk.  The K pass takes a row's bytes in pieces of 64 (one LDS staging round
  // each); the loads fetch two pieces at a time as whole 128-byte lines: 8 lanes per row, 8 rows
  // per load, 8 loads.  They are non-temporal like the V loads below: every K and V byte is
  // needed once per step, and a stream that does not settle in the caches leaves them to the
  // step's small read-write arrays (measured on a streaming probe with this access pattern:
  // 6.25 -> 6.7 TB/s; in 64-byte half lines the hint costs bandwidth instead, the second half
  // of a line then comes from memory again).  The next pair is requested as soon as this one
  // sits in LDS.
  static_assert(NP % 2 == 0, "pieces are loaded in pairs");
  u32x4 kreg[8];
  auto load_pair = [&](int sub, int rows, int p0) {
    const unsigned char* Kc = Kh + int64_t(sub) * kSub * RB;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = min(i * 8 + (ln >> 3), rows - 1);  // rows past the end repeat the last one
      kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Kc + int64_t(r) * RB + p0 * kPiece + (ln & 7) * 16));
    }
  };
  const int sub0 = grp * kGroup * (kChunk / kSub) + w;
#pragma unroll
  for (int it = 0; it < kGroup; ++it) {
    const int sub = sub0 + it * (kChunk / kSub);
    const int rows = min(kSub, total - sub * kSub);  // <= 0: nothing (more) for this wavefront
    if (rows <= 0) {  // nothing (more) for this wavefront: it only takes part in the combination
      if (ln < G) wmax[w][ln] = -INFINITY;
      break;
    }
    // With more than one pass, address arithmetic hoisted out of the loop would cost more
    // registers than the occupancy allows; an opaque lane number keeps it inside.
    if (kGroup > 1) asm volatile("" : "+v"(ln));
    const int tr = ln / TPR, tc = ln % TPR;
    load_pair(sub, rows, 0);
    const unsigned char* Vc = Vh + int64_t(sub) * kSub * RB;
    // ---- K pass: lane = row.  The queries and candidate keys arrive through scalar loads.
    double acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) acc[v] = 0.0;
    double nr = 0.0;
    Raw rawA, rawB;
    double sA[NV][ES], sB[NV][ES];
    auto fetch = [&](int e0, int st, Raw& raw, double (&sv)[NV][ES]) {  // e0: first element of the piece
      raw = *reinterpret_cast<const Raw*>(mine + ln * kPitch + st * ES * int(sizeof(T)));
#pragma unroll
      for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int e = 0; e < ES; ++e) sv[v][e] = S[v * D + e0 + st * ES + e];
    };
    auto step = [&](const Raw& raw, const double (&sv)[NV][ES]) {
      double x[ES];
      raw_to_f64<T, ES>(raw, x);
#pragma unroll
      for (int e = 0; e < ES; ++e) nr = fma(x[e], x[e], nr);
#pragma unroll
      for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int e = 0; e < ES; ++e) acc[v] = fma(x[e], sv[v][e], acc[v]);
    };
    // V rows travel in quarters of the sub-chunk through two register sets: two quarters are on
    // their way while the lanes finish the K pass, the others follow as the sets are consumed
    // (a whole sub-chunk in registers would cost the kernel a quarter of its occupancy).
    constexpr int VQ = NVL / 4;
    VRaw vbuf[2][VQ];
    auto load_vq = [&](int q, int set) {
#pragma unroll
      for (int i = 0; i < VQ; ++i) {
        const int r = min((q * VQ + i) * RPI + tr, rows - 1);  // repeated rows meet a zero probability
        vbuf[set][i] = __builtin_nontemporal_load(reinterpret_cast<const VRaw*>(Vc + int64_t(r) * RB + tc * VB));
      }
    };
    // this lane's score-side loads ride along
    const bool valid = ln < rows;
    const int j = sub * kSub + ln;
    const int pos = valid ? a.cpos[slot0 + j] : 0;
    // fp8 cache: the powers of two of this lane's K and V row
    int rek = 0, rev = 0;
    if constexpr (sizeof(T) == 1) {
      rek = valid ? a.cKe[slot0 + j] : 0;
      rev = valid ? a.cVe[slot0 + j] : 0;
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      // The staging area is private to the wavefront and LDS serves a wavefront's requests in
      // order, so the piece hand-over needs compiler ordering only.
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (((ln >> 2) & 1) == (p & 1)) {  // the lanes that hold this piece's half of the lines
#pragma unroll
        for (int i = 0; i < 8; ++i)
          *reinterpret_cast<u32x4*>(mine + (i * 8 + (ln >> 3)) * kPitch + (ln & 3) * 16) = kreg[i];
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if ((p & 1) && p + 1 < NP) load_pair(sub, rows, p + 1);
      if (p == NP - 1) {  // the first half of this sub-chunk's V rows
        load_vq(0, 0);
        load_vq(1, 1);
      }
      // ES elements per step.  The row's bits and the scalar operands of a step are fetched one
      // step ahead (two register sets), so their latency hides behind the previous step's FMAs.
      const int e0 = p * EP;
      fetch(e0, 0, rawA, sA);
#pragma unroll 1
      for (int st = 0; st < NST; st += 2) {
        // the wait for a set comes before the other set's fetches are issued (scalar loads
        // return out of order, so a wait after them would cover them too)
        arrived(sA[0][0]);
        fetch(e0, st + 1, rawB, sB);
        __builtin_amdgcn_sched_barrier(0);  // the fetches go out before the FMAs, not among them
        step(rawA, sA);
        arrived(sB[0][0]);
        fetch(e0, min(st + 2, NST - 1), rawA, sA);
        __builtin_amdgcn_sched_barrier(0);
        step(rawB, sB);
      }
    }
    if constexpr (sizeof(T) == 1) {
      // the K pass worked on the codes: the row's power of two scales its dot products and its
      // squared norm (exactly: the sums are exact, see the precision notes of the file header)
      const double sk = pow2_f64(rek);
#pragma unroll
      for (int v = 0; v < NV; ++v) acc[v] *= sk;
      nr *= sk * sk;
    }
    // ---- softmax statistics of the sub-chunk; the lane owns cache row sub*kSub + lane
    const int64_t pidx = sub_index(a, bh, mt3, sub) * G;
    double recv = 0.0;  // this lane's element of the sub-chunk record
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const double sg = acc[g] / root_d;
      const double mx = fast_wave_max(valid ? sg : -INFINITY);
      const double e = valid ? exp(sg - mx) : 0.0;
      // (fp8 cache: the V pass works on the codes, so the row's power of two rides on its probability)
      ps[w][g][ln] = sizeof(T) == 1 ? float(e) * pow2_f32(rev) : float(e);
      if (valid) st_agent(&a.elog[elog_index(a, bh, mt3, G, g, j)], e);
      const double sm = fast_wave_sum(e);
      if (ln == g) {
        recv = mx;
        wmax[w][g] = mx;
      }
      if (ln == G + g) recv = sm;
    }
    // candidates: cosine of this row against each candidate key (Eq. 9), sub-chunk arg-max
    const double nrow = sqrt(nr);
#pragma unroll
    for (int c = 0; c < kCand; ++c) {
      const double den = cn[c] * nrow;
      const double u = den > 0.0 ? acc[G + c] / den : 0.0;
      const Best m = fast_wave_best_match(u, pos, (valid && cs[c] >= 0 && j != cs[c]) ? j : -1);
      if (ln == 2 * G + c) recv = m.u;
      if (ln == 2 * G + kCand + c) recv = double(m.slot);
    }
    if (ln < kRec) st_agent(&a.rec[(pidx / G) * kRec + ln], recv);  // the record in one store
    // ---- partial P V, fp32: TPR lanes per row, RPI rows per load, then a sum over the row groups
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    float pv[G][kVec];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < kVec; ++e) pv[g][e] = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int i = 0; i < VQ; ++i) {
        const int r = (q * VQ + i) * RPI + tr;
        float x[kVec];
        if constexpr (sizeof(T) == 1) {  // eight codes in two words (the byte selector is an immediate)
          static_assert(sizeof(T) != 1 || kVec == 8, "two words of codes");
#pragma unroll
          for (int wd = 0; wd < 2; ++wd) {
            const int bits = int(raw_word(vbuf[q & 1][i], wd));
            x[4 * wd] = __builtin_amdgcn_cvt_f32_fp8(bits, 0);
            x[4 * wd + 1] = __builtin_amdgcn_cvt_f32_fp8(bits, 1);
            x[4 * wd + 2] = __builtin_amdgcn_cvt_f32_fp8(bits, 2);
            x[4 * wd + 3] = __builtin_amdgcn_cvt_f32_fp8(bits, 3);
          }
        } else {
          cvt16f<T>(vbuf[q & 1][i], x);
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float p = ps[w][g][r];  // 0 for rows beyond the end
#pragma unroll
          for (int e = 0; e < kVec; ++e) pv[g][e] = fmaf(p, x[e], pv[g][e]);
        }
      }
      if (q + 2 < 4) load_vq(q + 2, q & 1);
    }
    // sum over the row groups; the wavefront's partial rows (one per query head) go to its
    // staging area, which is free again, for the combination over the workgroup
    float* xch = reinterpret_cast<float*>(mine);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        float t = pv[g][e];
#pragma unroll
        for (int o = TPR; o < 64; o <<= 1) t += __shfl_xor(t, o, 64);
        pv[g][e] = t;
      }
      if (tr == 0) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) xch[g * D + tc * kVec + e] = pv[g][e];
      }
    }
  }
  // ---- one partial output row per chunk and query head: the four wavefronts' rows, each
  //      rescaled from its sub-chunk's maximum to the chunk's (fp32, like the rows themselves).
  //      A quarter of the partial-output bytes of a row per sub-chunk: on this chip a written
  //      byte costs the stream of K and V rows several read bytes.
  static_assert(kGroup == 1, "one chunk per workgroup");
  lds_barrier();
  for (int g = w; g < G; g += 4) {
    double mc = wmax[0][g];
#pragma unroll
    for (int i = 1; i < 4; ++i) mc = fmax(mc, wmax[i][g]);
    if (lane * 2 < D) {
      float o0 = 0.f, o1 = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const double mw = wmax[i][g];
        if (mw != -INFINITY) {
          const float f = expf(float(mw - mc));
          const float* xr = reinterpret_cast<const float*>(stage + i * 64 * kPitch) + g * D + lane * 2;
          o0 = fmaf(f, xr[0], o0);
          o1 = fmaf(f, xr[1], o1);
        }
      }
      const uint64_t two = uint64_t(__float_as_uint(o0)) | (uint64_t(__float_as_uint(o1)) << 32);
      st_agent(reinterpret_cast<uint64_t*>(a.pacc + (chunk_index(a, bh, mt3, grp) * G + g) * D + lane * 2), two);
    }
  }
  // ---- ticket: the last workgroup of the head to arrive closes the head.  Every store above
  //      that it will read is a write-through store; they have completed once the memory
  //      counters are zero, before the barrier that precedes the ticket.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (tid == 0) {
    const int ngroup = (total + kGroup * kChunk - 1) / (kGroup * kChunk);
    sh_last = (__hip_atomic_fetch_add(&a.ticket[lbh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
               unsigned(ngroup - 1)) ? 1 : 0;
  }
  __syncthreads();
  if (!sh_last) return;
  // Consumer side of the hand-over.  The other workgroups' results (rec, elog, pacc) are read
  // below through ld_agent only, which goes around this XCD's L2 whatever the compiler does
  // with plain loads; this fence keeps the compiler from moving any load of the closing code
  // above the ticket.  Plain loads in the closing code are limited to data that no other
  // workgroup of this launch writes: cscore, cpos, cK, cV, ctau, cand, meta of this head.
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  // the staging area is free: it holds the closing code's exchange buffers
  float* fred = reinterpret_cast<float*>(stage);
  double* dred = reinterpret_cast<double*>(stage + 4 * 256 * sizeof(float));
  double* sred = dred + D;
  int* ired = reinterpret_cast<int*>(sred + 8);
  if (total > a.big_rows) {
    // A very large head: two more launches close it (decode_close_part / _final).  All its
    // sub-chunk records are there now, so this workgroup leaves them the head's softmax
    // maxima and exact normalisers (the sweep and summation tree of the single-workgroup form),
    // while other heads' chunks still stream.
    head_normaliser<G>(a, int64_t(b) * a.Hkv + hk, mt3, (total + kSub - 1) / kSub, a.hnorm + lbh * 16, dred, sred);
    return;
  }
  head_tail<T, OT, D, G>(a, out, ov, li, b, hk, lbh, total, (total + kSub - 1) / kSub, sred, ired, fred, dred,
                         stage + 8192);
}

// The type of q, k_new, v_new and (unless fp32 is asked for) of the outputs: the cache's own
// type, or bf16 when the cache holds fp8 codes.
template <typename T>
struct TensorType {
  typedef typename std::conditional<sizeof(T) == 1, uint16_t, T>::type type;
};

template <typename T, int D>
hipError_t run_prepare_g(d2o_ctx* c, const DecodeArgs& a, int nl, View q, View k, View v, hipStream_t s) {
  typedef typename TensorType<T>::type IT;
  const int bh = a.B * a.Hkv;
  KernelTimer kt(c, D2O_K_DECODE_PREPARE, s);
  const dim3 grid(bh, nl);
  switch (a.G) {
    case 1: decode_prepare<T, IT, D, 1><<<grid, 128, 0, s>>>(a, (const IT*)q.ptr, q, (const IT*)k.ptr, k, (const IT*)v.ptr, v); break;
    case 2: decode_prepare<T, IT, D, 2><<<grid, 128, 0, s>>>(a, (const IT*)q.ptr, q, (const IT*)k.ptr, k, (const IT*)v.ptr, v); break;
    case 4: decode_prepare<T, IT, D, 4><<<grid, 128, 0, s>>>(a, (const IT*)q.ptr, q, (const IT*)k.ptr, k, (const IT*)v.ptr, v); break;
    case 8: decode_prepare<T, IT, D, 8><<<grid, 128, 0, s>>>(a, (const IT*)q.ptr, q, (const IT*)k.ptr, k, (const IT*)v.ptr, v); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename T, typename OT, int D, int G>
hipError_t run_attend(d2o_ctx* c, const DecodeArgs& a, int flat_chunks, View out, hipStream_t s) {
  KernelTimer kt(c, D2O_K_DECODE_ATTEND, s);
  decode_attend<T, OT, D, G><<<dim3(a.B * a.Hkv, flat_chunks), 256, 0, s>>>(a, (OT*)out.ptr, out);
  return hipGetLastError();
}

template <typename T, int D, int G>
hipError_t run_decode(d2o_ctx* c, const DecodeArgs& a, int fc, View out, hipStream_t s) {
  if (a.out_f32) return run_attend<T, float, D, G>(c, a, fc, out, s);
  return run_attend<T, typename TensorType<T>::type, D, G>(c, a, fc, out, s);
}

template <typename T, int D>
hipError_t run_decode_g(d2o_ctx* c, const DecodeArgs& a, int fc, View out, hipStream_t s) {
  switch (a.G) {
    case 1: return run_decode<T, D, 1>(c, a, fc, out, s);
    case 2: return run_decode<T, D, 2>(c, a, fc, out, s);
    case 4: return run_decode<T, D, 4>(c, a, fc, out, s);
    case 8: return run_decode<T, D, 8>(c, a, fc, out, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

int decode_candidates() { return kCand; }


// The eviction candidates of the first generation step of one layer, chosen after prompt
// compression: the kCand lowest scores among the cached tokens that are evictable when token
// `new_pos` arrives (Eq. 7-8 on count + 1 entries: neither sink nor inside the recent window).
// A prediction like the one every step makes for the next: a miss costs that step's closing
// workgroup a second pass over the keys and nothing else.
__global__ __launch_bounds__(256) void init_candidates(const int32_t* __restrict__ ccount,
                                                       const int32_t* __restrict__ meta,  // the layer's [B][Hkv][4]
                                                       const double* __restrict__ cscore,
                                                       const int32_t* __restrict__ cpos, int32_t* __restrict__ cand,
                                                       int layer, int B, int Hkv, int64_t slots, int new_pos,
                                                       int n_sink) {
  __shared__ double sred[4];
  __shared__ int ired[8];
  const int hk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t lbh = (int64_t(layer) * B + b) * Hkv + hk;
  const int total = ccount[lbh], recent = meta[(b * Hkv + hk) * 4 + 2];
  const int64_t slot0 = (int64_t(b) * Hkv + hk) * slots + meta[(b * Hkv + hk) * 4 + 0];
  Best low[kCand + 1];
#pragma unroll
  for (int i = 0; i <= kCand; ++i) low[i] = Best{0.0, 0, -1};
  for (int j = tid; j < total; j += 256) {
    const double sc = cscore[slot0 + j];
    const int p = cpos[slot0 + j];
    if (p >= n_sink && p <= new_pos - recent && evicts_before(sc, p, j, low[kCand - 1])) {
      low[kCand - 1] = Best{sc, p, j};
#pragma unroll
      for (int i = kCand - 1; i > 0; --i)
        if (evicts_before(low[i].u, low[i].pos, low[i].slot, low[i - 1])) {
          const Best t = low[i - 1];
          low[i - 1] = low[i];
          low[i] = t;
        }
    }
  }
#pragma unroll
  for (int r = 0; r < kCand; ++r) {  // repeated block-wide extraction of the first in eviction order
    Best h = fast_wave_first_evicted(low[0]);
    __syncthreads();
    if (lane == 0) {
      sred[w] = h.u;
      ired[w] = h.pos;
      ired[4 + w] = h.slot;
    }
    __syncthreads();
    h = Best{sred[0], ired[0], ired[4]};
#pragma unroll
    for (int i = 1; i < 4; ++i)
      if (evicts_before(sred[i], ired[i], ired[4 + i], h)) h = Best{sred[i], ired[i], ired[4 + i]};
    if (tid == 0) cand[lbh * kCand + r] = h.slot;
    if (h.slot >= 0 && low[0].slot == h.slot) {  // the owner pops its head
#pragma unroll
      for (int i = 0; i < kCand; ++i) low[i] = low[i + 1];
    }
  }
}

hipError_t launch_init_candidates(d2o_ctx* c, int layer, int new_pos, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  init_candidates<<<dim3(cf.n_kv_heads, cf.batch), 256, 0, s>>>(c->ccount, c->meta + size_t(layer) * cf.batch * cf.n_kv_heads * 4,
                                                                c->cscore, c->cpos, c->ccand, layer, cf.batch,
                                                                cf.n_kv_heads, cf.slots_per_seq, new_pos, cf.n_sink);
  return hipGetLastError();
}

// Sizes (in bytes, each rounded up to 256) of the six scratch arrays of a decode step, in the
// order elog, rec, pacc, vecs, cnorm, part.
static void decode_scratch_sizes(const d2o_ctx* c, size_t (&sz)[6]) {
  const d2o_config& cf = c->cfg;
  const size_t B = cf.batch, L = cf.n_layers, Hq = cf.n_q_heads, Hkv = cf.n_kv_heads, d = cf.head_dim;
  const size_t G = Hq / Hkv, bh = B * Hkv, nch = c->nchunk_cap, nsub = nch * 4;
  sz[0] = nch * B * Hq * kChunk * sizeof(double);
  sz[1] = bh * nsub * rec_doubles(int(G)) * sizeof(double);  // one record per 64 slots
  sz[2] = bh * nch * G * d * sizeof(float);                  // one partial output row per chunk and query head
  sz[3] = L * bh * (G + kCand) * d * sizeof(double);
  sz[4] = L * bh * kCand * sizeof(double);
  sz[5] = (bh * nch * kPartRecDoubles + L * bh * 16) * sizeof(double);  // part records, then 16 doubles per head
  for (size_t& x : sz) x = (x + 255) & ~size_t(255);
}

size_t decode_static_scratch_need(const d2o_ctx* c) {
  size_t sz[6];
  decode_scratch_sizes(c, sz);
  return sz[0] + sz[1] + sz[2] + sz[3] + sz[4] + sz[5];
}
size_t decode_static_scratch_capacity() { return kStaticScratchBytes; }

hipError_t launch_decode(d2o_ctx* c, int layer0, int nl_all, View q, View k, View v, View out, int new_pos,
                         hipStream_t s, unsigned char* static_scratch) {
  const d2o_config& cf = c->cfg;
  DecodeArgs a;
  a.ccount = c->ccount;
  a.ctotal = c->ctotal;
  a.ctau = c->ctau;
  a.meta = c->meta;
  a.cK = c->cacheK;
  a.cV = c->cacheV;
  a.cKe = c->cKe;
  a.cVe = c->cVe;
  a.cscore = c->cscore;
  a.cpos = c->cpos;
  a.cand = c->ccand;
  a.ticket = c->cticket;
  a.cmiss = c->cmiss;
  a.elog = c->d_logit;
  a.rec = c->d_rec;
  a.pacc = c->d_pacc;
  a.vecs = c->d_vecs;
  a.cnorm = c->d_cnorm;
  a.part = c->d_part;
  if (static_scratch) {  // the same six arrays, carved from the library's static device array
    size_t sz[6];
    decode_scratch_sizes(c, sz);
    unsigned char* p = static_scratch;
    a.elog = reinterpret_cast<double*>(p);
    a.rec = reinterpret_cast<double*>(p += sz[0]);
    a.pacc = reinterpret_cast<float*>(p += sz[1]);
    a.vecs = reinterpret_cast<double*>(p += sz[2]);
    a.cnorm = reinterpret_cast<double*>(p += sz[3]);
    a.part = reinterpret_cast<double*>(p += sz[4]);
  }
  a.ev_evicted = c->ev_evicted;
  a.ev_target = c->ev_target;
  a.ev_ustar = c->ev_ustar;
  a.slots = cf.slots_per_seq;
  a.B = cf.batch;
  a.Hkv = cf.n_kv_heads;
  a.G = cf.n_q_heads / cf.n_kv_heads;
  a.new_pos = new_pos;
  a.n_sink = cf.n_sink;
  a.out_f32 = cf.out_f32;
  a.merge_average = cf.merge_average;
  a.part_chunks = cf.split_rows > 0 ? std::min(8, std::max(1, cf.split_rows / (4 * kChunk))) : 8;
  a.beta = cf.beta;
  a.tau_force = cf.tau_force;
  // the per-layer tensors of one call are [layer][...]: groups of at most kMaxLayersPerCall
  for (int g0 = 0; g0 < nl_all; g0 += kMaxLayersPerCall) {
    const int nl = std::min(kMaxLayersPerCall, nl_all - g0);
    a.layer0 = layer0 + g0;
    a.nl = nl;
    int mc[kMaxLayersPerCall], chunk_id[kMaxLayersPerCall];
    const int nc = nl;
    int64_t rows = 0;  // cache rows this launch streams
    for (int i = 0; i < nl; ++i) {
      chunk_id[i] = i;
      mc[i] = 1;
      for (const auto& mt : c->layers[a.layer0 + i].meta) {
        mc[i] = std::max(mc[i], (mt.budget + 1 + kGroup * kChunk - 1) / (kGroup * kChunk));
        rows += mt.budget + 1;
      }
    }
    // Which heads are too large for one closing workgroup.  A head's last workgroup closes it
    // while the other heads' chunks still stream, which costs nothing as long as the head is a
    // small part of the launch; a head that holds more than about half a percent of the
    // launch's rows (a few giant layers after Eq. 5, or a launch of one layer) would leave the
    // chip waiting for its closing workgroup, and is finished by the split kernels instead.
    a.hnorm = a.part + size_t(cf.batch) * cf.n_kv_heads * c->nchunk_cap * kPartRecDoubles;
    a.big_rows = cf.split_rows > 0 ? cf.split_rows
                                   : int(std::min<int64_t>(kMaxAutoSplitRows, std::max<int64_t>(kMinAutoSplitRows, rows / 200)));
    auto shift = [&](View x, int elem_bytes) {  // first layer of this group
      x.ptr = static_cast<char*>(x.ptr) + size_t(g0) * x.sn * elem_bytes;
      return x;
    };
    const int es = c->esize, os = cf.out_f32 ? 4 : c->esize;
    const View qg = shift(q, es), kg = shift(k, es), vg = shift(v, es), og = shift(out, os);
    hipError_t e;
    // ---- append + operand set-up for every layer of the group
    if (cf.cache_fp8)
      e = run_prepare_g<uint8_t, 128>(c, a, nl, qg, kg, vg, s);
    else if (cf.dtype == D2O_BF16)
      e = run_prepare_g<uint16_t, 128>(c, a, nl, qg, kg, vg, s);
    else if (cf.head_dim == 64)
      e = run_prepare_g<float, 64>(c, a, nl, qg, kg, vg, s);
    else
      e = run_prepare_g<float, 128>(c, a, nl, qg, kg, vg, s);
    if (e != hipSuccess) return e;
    // ---- attention over the caches, one workgroup per 256 slots; the layers with most chunks first
    {
      std::stable_sort(chunk_id, chunk_id + nc, [&](int x, int y) { return mc[x] > mc[y]; });
      int flat = 0;
      for (int i = 0; i < nc; ++i) {
        a.lay_id[i] = chunk_id[i];
        a.lay_off[i] = flat;
        flat += mc[chunk_id[i]];
      }
      for (int i = nc; i <= kMaxLayersPerCall; ++i) a.lay_off[i] = i == nc ? flat : 0x7FFFFFFF;
      if (cf.cache_fp8)
        e = run_decode_g<uint8_t, 128>(c, a, flat, og, s);
      else if (cf.dtype == D2O_BF16)
        e = run_decode_g<uint16_t, 128>(c, a, flat, og, s);
      else if (cf.head_dim == 64)
        e = run_decode_g<float, 64>(c, a, flat, og, s);
      else
        e = run_decode_g<float, 128>(c, a, flat, og, s);
      if (e != hipSuccess) return e;
      // ---- heads too large for one closing workgroup (their entry count can reach budget + rows
      //      appended since): the same grid finishes them in parts
      bool big = false;
      for (int i = 0; i < nl; ++i) big = big || int64_t(mc[i]) * kChunk > a.big_rows;
      if (big) {
        e = launch_decode_split(c, a, mc, nl, og, s);
        if (e != hipSuccess) return e;
      }
    }
  }
  return hipSuccess;
}

}  // namespace d2o
