// Closing work of very large heads in a generation step (Sec. 4.2 Eq. 6-12), split over many
// workgroups.  decode_attend leaves the closing work of a head - exact normaliser, output rows,
// score update, eviction arg-min, next candidates, merge - to the head's last workgroup.  That
// is the right shape for the usual cache of a few thousand entries, but a layer that the
// allocation (Eq. 5) hands most of a long prompt's budget leaves one workgroup walking tens of
// thousands of slots while the rest of the chip is idle.  For a head with more than
// `big_rows` entries decode_attend therefore stops after its partial results, and two more
// launches finish the head:
//
//   decode_close_part   one workgroup per `part_chunks` chunks of the head.  The head's softmax
//                       maxima and exact normalisers are there already (the head's last
//                       attention workgroup computed them from the sub-chunk records while
//                       other heads still streamed); for its own chunks the part does the partial
//                       output rows, the score update (Eq. 6), its first-evicted entry (Eq. 7-8),
//                       its kCand + 1 lowest entries for the next step and the candidates' best
//                       matches (Eq. 9).  Results: one record of kPartRec doubles per part, and
//                       the part's output row in place of its first chunk's partial row.
//   decode_close_final  one workgroup per head: adds the parts' output rows in ascending
//                       order, reduces the parts' records, and ends the step exactly as the
//                       single-workgroup form does (close_head).
//
// Both kernels run after decode_attend has completed, so they read its results with ordinary
// loads.  Scores, decisions and events are those of the single-workgroup form (the same fp64
// operations per slot; the normaliser's fixed summation tree is the same); the output rows
// differ from it only in the order of the fp32 additions over chunks.
#include <algorithm>
#include <type_traits>

#include "decode_common.h"

namespace d2o {
namespace {

using namespace dec;

constexpr int kMaxPartChunks = 8;

// Record of one part (doubles; integers are stored as doubles, exactly):
//   [0..3)   first-evicted entry (score, position, slot; slot -1: none)
//   [3..15)  the kCand + 1 lowest entries evictable at the next step, in eviction order (room for four)
//   [15..24) best match of each candidate (cosine, position, slot)
//   [24..26) the head's last slot: updated score, position (written by the part that owns it)
constexpr int kPartRec = kPartRecDoubles;
static_assert(kPartRec >= 26 && 3 + 3 * (kCand + 1) <= 15 && 15 + 3 * kCand <= 24, "record too small");

__device__ __forceinline__ void put(double* r, const Best& b) {
  r[0] = b.u;
  r[1] = double(b.pos);
  r[2] = double(b.slot);
}
__device__ __forceinline__ Best get(const double* r) { return Best{r[0], int(r[1]), int(r[2])}; }

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_close_part(DecodeArgs a) {
  constexpr int kRec = rec_doubles(G);
  constexpr int U = G >= 8 ? 2 : 4;  // slots per thread and batch of the score pass
  constexpr int C4 = D / 4;          // threads across an output row (four columns each)
  constexpr int RG = 256 / C4;       // groups of threads that share the part's chunks
  static_assert(kGroup == 1, "a flat index is one chunk");
  __shared__ double em[kMaxPartChunks * 4 * G];  // exp(m_sub - max) / normaliser of the part's sub-chunks
  __shared__ float fred[4 * 256];
  __shared__ double sred[8];
  __shared__ int ired[8];
  // grid: x = head, y = flat part index over the layers that can hold large heads (lay_off counts parts here)
  const int entry = find_entry(a, blockIdx.y), grp = (blockIdx.y - a.lay_off[entry]) * a.part_chunks;
  const int li = a.lay_id[entry];
  const int l = a.layer0 + li, b = blockIdx.x / a.Hkv, hk = blockIdx.x % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int total = a.ctotal[lbh];
  if (total <= a.big_rows || grp * kChunk >= total) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int32_t* mt = a.meta + lbh * 4;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt[0];
  const int ch0 = mt[3], last = total - 1;
  const int nsub = (total + kSub - 1) / kSub, nchunk = (total + kChunk - 1) / kChunk;
  const int c_lo = grp, c_hi = min(grp + a.part_chunks, nchunk);  // the part's chunks
  const int s_lo = c_lo * 4, s_hi = min(c_hi * 4, nsub);          // its sub-chunks
  const int j_lo = c_lo * kChunk, j_hi = min(c_hi * kChunk, total);  // its slots
  double* prec = a.part + chunk_index(a, bh, ch0, c_lo) * kPartRec;
  // ---- head maximum and exact normaliser of each query head, left by the head's last attention
  //      workgroup; exp(m_sub - max) / normaliser of the part's sub-chunks goes to LDS
  double Mg[G], Lg[G];
  {
    const double* hn = a.hnorm + lbh * 16;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      Mg[g] = hn[g];
      Lg[g] = hn[G + g];
    }
    for (int i = tid; i < (s_hi - s_lo) * G; i += 256) {
      const int c = s_lo + i / G, g = i % G;
      double mg = Mg[0], lg = Lg[0];
#pragma unroll
      for (int k = 1; k < G; ++k) {
        mg = g == k ? Mg[k] : mg;
        lg = g == k ? Lg[k] : lg;
      }
      em[i] = exp(a.rec[sub_index(a, bh, ch0, c) * kRec + g] - mg) / lg;
    }
    __syncthreads();
  }
  // ---- Eq. 9: best match of every candidate among the part's sub-chunks (ties: earlier position)
  {
    Best cm[kCand];
#pragma unroll
    for (int i = 0; i < kCand; ++i) cm[i] = Best{0.0, 0, -1};
    for (int c = s_lo + tid; c < s_hi; c += 256) {
      const int64_t x = sub_index(a, bh, ch0, c) * kRec;
#pragma unroll
      for (int i = 0; i < kCand; ++i) {
        const int s = int(a.rec[x + 2 * G + kCand + i]);
        if (s >= 0) {
          const double u = a.rec[x + 2 * G + i];
          const int p = a.cpos[slot0 + s];
          if (better_match(u, p, s, cm[i])) cm[i] = Best{u, p, s};
        }
      }
    }
    // at most 64 sub-chunks: they all sit in wavefront 0
    static_assert(kMaxPartChunks * 4 <= 64, "one wavefront holds a part's sub-chunks");
    if (w == 0) {
#pragma unroll
      for (int i = 0; i < kCand; ++i) {
        const Best r = fast_wave_best_match(cm[i].u, cm[i].pos, cm[i].slot);
        if (lane == 0) put(prec + 15 + 3 * i, r);
      }
    }
  }
  // ---- output rows of the part: thread (rg, c4) adds the chunks c_lo + rg, + RG, ... of four
  //      columns; the groups' sums are added in ascending order.  The row replaces the partial
  //      row of the part's first chunk (every read of it precedes the barrier before the write).
  {
    const int c4 = tid % C4, rg = tid / C4;
#pragma unroll 1
    for (int g = 0; g < G; ++g) {
      float num[4] = {0.f, 0.f, 0.f, 0.f};
      for (int cc = c_lo + rg; cc < c_hi; cc += RG) {
        const float4 v = *reinterpret_cast<const float4*>(a.pacc + (chunk_index(a, bh, ch0, cc) * G + g) * D + c4 * 4);
        double fc = 0.0;  // exp(chunk maximum - max): the largest of its sub-chunks' factors
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (cc * 4 + i < s_hi) fc = fmax(fc, em[(cc * 4 + i - s_lo) * G + g]);
        const float f = float(fc);
        num[0] = fmaf(v.x, f, num[0]);
        num[1] = fmaf(v.y, f, num[1]);
        num[2] = fmaf(v.z, f, num[2]);
        num[3] = fmaf(v.w, f, num[3]);
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 4; ++e) fred[e * 256 + tid] = num[e];
      __syncthreads();
      if (tid < D) {  // column tid: element tid % 4 of the threads (rg, tid / 4)
        const float* fr = fred + (tid % 4) * 256 + tid / 4;
        float t = fr[0];
#pragma unroll
        for (int i = 1; i < RG; ++i) t += fr[i * C4];
        a.pacc[(chunk_index(a, bh, ch0, c_lo) * G + g) * D + tid] = t;
      }
    }
  }
  // ---- score pass over the part's slots (Eq. 6), its first-evicted entry (Eq. 7-8 on count + 1
  //      entries) and the lowest scores among the tokens evictable at the next step
  const int recent = mt[2];
  Best ev{0.0, 0, -1};
  Best low[kCand + 1];
#pragma unroll
  for (int i = 0; i <= kCand; ++i) low[i] = Best{0.0, 0, -1};
#pragma unroll 1
  for (int j0 = j_lo + tid; j0 < j_hi; j0 += U * 256) {
    double sc[U], e[U][G];
    int ps[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = min(j0 + u * 256, j_hi - 1);
      sc[u] = a.cscore[slot0 + j];
      ps[u] = a.cpos[slot0 + j];
#pragma unroll
      for (int g = 0; g < G; ++g) e[u][g] = a.elog[elog_index(a, bh, ch0, G, g, j)];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = j0 + u * 256;
      if (j < j_hi) {
        double s2 = sc[u];
#pragma unroll
        for (int g = 0; g < G; ++g) s2 = fma(e[u][g], em[(j / kSub - s_lo) * G + g], s2);
        a.cscore[slot0 + j] = s2;
        const int p = ps[u];
        if (j == last) {  // kept for the move into the freed slot
          prec[24] = s2;
          prec[25] = double(p);
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
    }
  }
  // block-wide: the first evicted, then the kCand + 1 lowest by repeated extraction
#pragma unroll
  for (int r = -1; r <= kCand; ++r) {
    Best h = fast_wave_first_evicted(r < 0 ? ev : low[0]);
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
    if (tid == 0) put(prec + (r < 0 ? 0 : 3 + 3 * r), h);
    if (r >= 0 && h.slot >= 0 && low[0].slot == h.slot) {  // the owner pops its head
#pragma unroll
      for (int i = 0; i < kCand; ++i) low[i] = low[i + 1];
      low[kCand].slot = -1;
    }
  }
}

template <typename T, typename OT, int D, int G>
__global__ __launch_bounds__(256) void decode_close_final(DecodeArgs a, OT* __restrict__ out, View ov) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[8192];
  __shared__ float fred[4 * 256];
  const int li = blockIdx.y, l = a.layer0 + li, b = blockIdx.x / a.Hkv, hk = blockIdx.x % a.Hkv;
  const int64_t lbh = (int64_t(l) * a.B + b) * a.Hkv + hk;
  const int total = a.ctotal[lbh];
  if (total <= a.big_rows) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int32_t* mt = a.meta + lbh * 4;
  const int64_t bh = int64_t(b) * a.Hkv + hk;
  const int64_t slot0 = bh * a.slots + mt[0];
  const int ch0 = mt[3], last = total - 1;
  const int nchunk = (total + kChunk - 1) / kChunk, nparts = (nchunk + a.part_chunks - 1) / a.part_chunks;
  const T* Kc = static_cast<const T*>(a.cK) + slot0 * D;
  const T* Vc = static_cast<const T*>(a.cV) + slot0 * D;
  // LDS: the exchange buffers of close_head
  double* dred = reinterpret_cast<double*>(smem);  // [D] (a pass over the keys, if one is needed)
  double* sred = dred + D;
  int* ired = reinterpret_cast<int*>(sred + 8);
  double* wcm_u = sred + 8 + 8;
  int2* wcm_ps = reinterpret_cast<int2*>(wcm_u + 4 * kCand);
  T* park_kv = reinterpret_cast<T*>(wcm_ps + 4 * kCand);
  static_assert((D + 16 + 4 * kCand * 2) * 8 + 512 * sizeof(T) <= 8192, "exchange buffers");
  const double told = a.ctau[lbh];
  int cl[kCand];
#pragma unroll
  for (int i = 0; i < kCand; ++i) cl[i] = a.cand[lbh * kCand + i];
  if (tid < D) {
    park_kv[tid] = Kc[int64_t(last) * D + tid];
    park_kv[256 + tid] = Vc[int64_t(last) * D + tid];
  }
  auto record = [&](int p) { return a.part + chunk_index(a, bh, ch0, p * a.part_chunks) * kPartRec; };
  // ---- the parts' records: thread t takes the parts t, t + 256, ...
  Best ev{0.0, 0, -1};
  Best low[kCand + 1], cm[kCand];
#pragma unroll
  for (int i = 0; i <= kCand; ++i) low[i] = Best{0.0, 0, -1};
#pragma unroll
  for (int i = 0; i < kCand; ++i) cm[i] = Best{0.0, 0, -1};
  for (int p = tid; p < nparts; p += 256) {
    const double* r = record(p);
    const Best e = get(r);
    if (evicts_before(e.u, e.pos, e.slot, ev)) ev = e;
#pragma unroll
    for (int k = 0; k <= kCand; ++k) {
      const Best x = get(r + 3 + 3 * k);
      if (evicts_before(x.u, x.pos, x.slot, low[kCand])) {
        low[kCand] = x;
#pragma unroll
        for (int i = kCand; i > 0; --i)
          if (evicts_before(low[i].u, low[i].pos, low[i].slot, low[i - 1])) {
            const Best t = low[i - 1];
            low[i - 1] = low[i];
            low[i] = t;
          }
      }
    }
#pragma unroll
    for (int i = 0; i < kCand; ++i) {
      const Best x = get(r + 15 + 3 * i);
      if (better_match(x.u, x.pos, x.slot, cm[i])) cm[i] = x;
    }
  }
#pragma unroll
  for (int i = 0; i < kCand; ++i) {
    const Best r = fast_wave_best_match(cm[i].u, cm[i].pos, cm[i].slot);
    if (lane == 0) {
      wcm_u[w * kCand + i] = r.u;
      wcm_ps[w * kCand + i] = make_int2(r.pos, r.slot);
    }
  }
  if (tid == 0) {
    const double* r = record(nparts - 1);
    sred[4] = r[24];
    ired[8] = int(r[25]);
  }
  // ---- output rows: thread (rg, c4) adds the parts rg, rg + RG, ... of four columns, PB loads in
  //      flight; the groups' sums are added in ascending order
  {
    constexpr int C4 = D / 4, RG = 256 / C4, PB = 4;
    const int c4 = tid % C4, rg = tid / C4;
#pragma unroll 1
    for (int g = 0; g < G; ++g) {
      float num[4] = {0.f, 0.f, 0.f, 0.f};
      for (int p0 = rg; p0 < nparts; p0 += PB * RG) {
        float4 v[PB];
#pragma unroll
        for (int u = 0; u < PB; ++u) {
          const int p = min(p0 + u * RG, nparts - 1);
          v[u] = *reinterpret_cast<const float4*>(a.pacc + (chunk_index(a, bh, ch0, p * a.part_chunks) * G + g) * D + c4 * 4);
        }
#pragma unroll
        for (int u = 0; u < PB; ++u)
          if (p0 + u * RG < nparts) {
            num[0] += v[u].x;
            num[1] += v[u].y;
            num[2] += v[u].z;
            num[3] += v[u].w;
          }
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 4; ++e) fred[e * 256 + tid] = num[e];
      __syncthreads();
      if (tid < D) {  // column tid: element tid % 4 of the threads (rg, tid / 4)
        const float* fr = fred + (tid % 4) * 256 + tid / 4;
        float t = fr[0];
#pragma unroll
        for (int i = 1; i < RG; ++i) t += fr[i * C4];
        out[li * ov.sn + b * ov.sb + (hk * G + g) * ov.sh + tid] = Elem<OT>::from_f32(t);
      }
    }
  }
  const bool evict = total > mt[1];
  close_head<T, D>(a, lbh, slot0, total, evict, ev, low, cl, told, sred, ired, dred, wcm_u, wcm_ps, park_kv);
}

template <typename T, typename OT, int D, int G>
hipError_t run_split(d2o_ctx* c, const DecodeArgs& a, int flat_parts, int nl, View out, hipStream_t s) {
  KernelTimer kt(c, D2O_K_DECODE_CLOSE, s);
  decode_close_part<T, D, G><<<dim3(a.B * a.Hkv, flat_parts), 256, 0, s>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  decode_close_final<T, OT, D, G><<<dim3(a.B * a.Hkv, nl), 256, 0, s>>>(a, (OT*)out.ptr, out);
  return hipGetLastError();
}

template <typename T, int D, int G>
hipError_t run_split_o(d2o_ctx* c, const DecodeArgs& a, int fc, int nl, View out, hipStream_t s) {
  if (a.out_f32) return run_split<T, float, D, G>(c, a, fc, nl, out, s);
  return run_split<T, typename std::conditional<sizeof(T) == 1, uint16_t, T>::type, D, G>(c, a, fc, nl, out, s);
}

template <typename T, int D>
hipError_t run_split_g(d2o_ctx* c, const DecodeArgs& a, int fc, int nl, View out, hipStream_t s) {
  switch (a.G) {
    case 1: return run_split_o<T, D, 1>(c, a, fc, nl, out, s);
    case 2: return run_split_o<T, D, 2>(c, a, fc, nl, out, s);
    case 4: return run_split_o<T, D, 4>(c, a, fc, nl, out, s);
    case 8: return run_split_o<T, D, 8>(c, a, fc, nl, out, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

namespace dec {

hipError_t launch_decode_split(d2o_ctx* c, const DecodeArgs& attend, const int* max_chunks, int nl, View out,
                               hipStream_t s) {
  if (attend.part_chunks < 1 || attend.part_chunks > kMaxPartChunks) return hipErrorInvalidValue;
  // the part kernel's layer list: only the layers whose caches can exceed big_rows, counted in parts
  DecodeArgs a = attend;
  int n = 0, flat = 0;
  for (int i = 0; i < nl; ++i) {
    if (int64_t(max_chunks[i]) * kChunk <= a.big_rows) continue;
    a.lay_id[n] = i;
    a.lay_off[n++] = flat;
    flat += (max_chunks[i] + a.part_chunks - 1) / a.part_chunks;
  }
  if (n == 0) return hipSuccess;
  for (int i = n; i <= kMaxLayersPerCall; ++i) a.lay_off[i] = i == n ? flat : 0x7FFFFFFF;
  if (c->cfg.cache_fp8) return run_split_g<uint8_t, 128>(c, a, flat, nl, out, s);
  if (c->cfg.dtype == D2O_BF16) return run_split_g<uint16_t, 128>(c, a, flat, nl, out, s);
  if (c->cfg.head_dim == 64) return run_split_g<float, 64>(c, a, flat, nl, out, s);
  return run_split_g<float, 128>(c, a, flat, nl, out, s);
}

}  // namespace dec
}  // namespace d2o
