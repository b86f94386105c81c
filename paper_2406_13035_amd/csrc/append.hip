// Multi-token append (a block of m new tokens on one layer's compressed caches).  Two stages:
// the block's attention (block_* kernels, further down: rows appended, every token's softmax row
// added to the scores, nothing evicted), then Eq. 7-12 once on every cache.  The second stage is
// the prompt-phase kernels of tokens.hip, which work on rows in ascending token position; a
// cache's slots are physically unordered, so this file lays every cache of the layer out in
// position order first:
//
//   rank_by_position   per (sequence, KV head): rank of every slot's position among the head's
//                      positions (positions are distinct), the ordered positions and fp64 scores,
//                      and the number of entries;
//   permute_rows       K and V rows of every slot to their rank in the ordered copy.
#include <type_traits>

#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace {

constexpr int kRankTile = 4096;  // positions held in LDS at a time

__global__ __launch_bounds__(256) void rank_by_position(const int32_t* __restrict__ ccount,   // the layer's [B][Hkv]
                                                        const int32_t* __restrict__ meta,     // the layer's [B][Hkv][4]
                                                        const double* __restrict__ cscore,
                                                        const int32_t* __restrict__ cpos, int32_t* __restrict__ rank,
                                                        int32_t* __restrict__ opos, double* __restrict__ oscore,
                                                        int32_t* __restrict__ on, int npad, int64_t slots) {
  __shared__ __attribute__((aligned(16))) int32_t tile[kRankTile];
  const int hk = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x, tid = threadIdx.x;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int n = ccount[bh];
  const int64_t slot0 = bh * slots + meta[bh * 4 + 0];
  if (tid == 0 && blockIdx.z == 0) on[bh] = n;
  // A workgroup owns 1024 slots at a time (a thread four of them; the workgroups of a head stride
  // over its slots); all positions of the head pass through LDS tile by tile, and each owned
  // slot counts the smaller ones (all threads read the same LDS words, eight at a time).
  for (int j0 = blockIdx.z * 1024; j0 < n; j0 += gridDim.z * 1024) {
    int mine[4], cnt[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 256 + tid;
      mine[u] = j < n ? cpos[slot0 + j] : 0x7FFFFFFF;
      cnt[u] = 0;
    }
    for (int t0 = 0; t0 < n; t0 += kRankTile) {
      __syncthreads();
      for (int i = tid; i < kRankTile; i += 256) tile[i] = t0 + i < n ? cpos[slot0 + t0 + i] : 0x7FFFFFFF;
      __syncthreads();
      const int lim = min(kRankTile, (n - t0 + 7) & ~7);  // the padding compares as "not smaller"
      for (int i = 0; i < lim; i += 8) {
        const int4 pa = *reinterpret_cast<const int4*>(&tile[i]), pb = *reinterpret_cast<const int4*>(&tile[i + 4]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
          cnt[u] += (pa.x < mine[u]) + (pa.y < mine[u]) + (pa.z < mine[u]) + (pa.w < mine[u]) + (pb.x < mine[u]) +
                    (pb.y < mine[u]) + (pb.z < mine[u]) + (pb.w < mine[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 256 + tid;
      if (j < n) {
        rank[bh * npad + j] = cnt[u];
        opos[bh * npad + cnt[u]] = mine[u];
        oscore[bh * npad + cnt[u]] = cscore[slot0 + j];
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void permute_rows(const int32_t* __restrict__ on, const int32_t* __restrict__ meta,
                                                    const int32_t* __restrict__ rank, const T* __restrict__ cK,
                                                    const T* __restrict__ cV, T* __restrict__ oK, T* __restrict__ oV,
                                                    int npad, int d, int64_t slots) {
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int64_t bh = int64_t(b) * Hkv + hk;
  constexpr int kVec = 16 / sizeof(T);
  const int tpr = d / kVec, rows_per_blk = 256 / tpr;
  const int j = blockIdx.x * rows_per_blk + threadIdx.x / tpr;
  if (j >= on[bh]) return;
  const int c = (threadIdx.x % tpr) * kVec;
  const int64_t src = (bh * slots + meta[bh * 4 + 0] + j) * d + c;
  const int64_t dst = (bh * npad + rank[bh * npad + j]) * d + c;
  *reinterpret_cast<u32x4*>(oK + dst) = *reinterpret_cast<const u32x4*>(cK + src);
  *reinterpret_cast<u32x4*>(oV + dst) = *reinterpret_cast<const u32x4*>(cV + src);
}


// ---------------------------------------------------------------------------------------------
// Attention of a block of m new tokens over the cache (Sec. 3 Eq. 2-3, Eq. 6 for every token of
// the block, nothing evicted): the block's rows are appended first; query i*G + g (token i, query
// head g of the group) then attends to the cache's N - m old entries and to the block's tokens
// 0..i.  Logits, softmax and score accumulation in fp64 as in the generation step; P V in fp32.
//
//   block_begin   per head: appends the block's K, V rows (score 0, positions first_pos + i),
//                 lays the queries out as fp64 vectors, sets the entry count to N.
//   block_stats   per (head, 256 rows): a lane owns a cache row and multiplies it with eight
//                 queries at a time, which reach the FMAs as scalar operands; per query the
//                 maximum and exp-sum over the chunk's visible rows.
//   block_norm    per head and query: maximum and exact normaliser over the chunks.
//   block_apply   per (head, 256 rows): logits again, p = exp(s - max) / normaliser; per row the
//                 sum of the p of every query that sees it, in the order (token, query head) of
//                 the defining formula; partial P V per chunk (the probabilities travel from
//                 the row's lane to all lanes through scalar registers, a lane owns D / 64
//                 output columns).
//   block_scores  per row: score += the sums (Eq. 6).
//   block_finish  per head and query: the chunks' partial output rows added in ascending order.
// block_stats and block_apply cut a head's queries into up to kMaxQuerySlices slices that run as
// workgroups of their own (a block on a cache of a few thousand rows is too little work per head
// to fill the chip otherwise); a row's score then grows by the slices' sums in slice order.
constexpr int kQG = 8;             // queries per pass over a row

template <typename T, typename IT, int D>
__global__ __launch_bounds__(256) void block_begin(const int32_t* __restrict__ ccount, int32_t* __restrict__ ctotal,
                                                   const int32_t* __restrict__ meta, T* __restrict__ cK,
                                                   T* __restrict__ cV, double* __restrict__ cscore,
                                                   int32_t* __restrict__ cpos, const IT* __restrict__ q, View qv,
                                                   const IT* __restrict__ kn, View kv, const IT* __restrict__ vn, View vv,
                                                   double* __restrict__ aq, int m, int G, int maxq, int first_pos,
                                                   int64_t slots) {
  const int hk = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x;
  const int tid = blockIdx.z * 256 + threadIdx.x, nt = gridDim.z * 256;  // the head's work is strided over its workgroups
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int count = ccount[bh];  // the entry count moves to N in block_norm, when no workgroup of this launch reads it any more
  const int64_t slot0 = bh * slots + meta[bh * 4 + 0];
  if constexpr (sizeof(T) == sizeof(IT)) {  // (an fp8 cache gets its rows from block_rows_fp8)
    for (int x = tid; x < m * D; x += nt) {
      const int i = x / D, c = x % D;
      cK[(slot0 + count + i) * D + c] = kn[b * kv.sb + hk * kv.sh + int64_t(i) * kv.sn + c];
      cV[(slot0 + count + i) * D + c] = vn[b * vv.sb + hk * vv.sh + int64_t(i) * vv.sn + c];
    }
  }
  for (int i = tid; i < m; i += nt) {
    cscore[slot0 + count + i] = 0.0;
    cpos[slot0 + count + i] = first_pos + i;
  }
  const int nq = m * G, nq_pad = (nq + kQG - 1) / kQG * kQG;  // the queries of a last, partial group are zero
  for (int x = tid; x < nq_pad * D; x += nt) {
    const int qi = x / D, c = x % D;
    double v = 0.0;
    if (qi < nq) v = Elem<IT>::to_f64(q[b * qv.sb + (hk * G + qi % G) * qv.sh + int64_t(qi / G) * qv.sn + c]);
    aq[(bh * maxq + qi) * D + c] = v;
  }
  if (tid == 0) ctotal[bh] = count + m;
}

// Pins the point where a scalar-loaded value must have arrived; nothing is scheduled across it.
__device__ __forceinline__ void scalar_arrived(double v) {
  asm volatile("" ::"s"(v));
  __builtin_amdgcn_sched_barrier(0);
}

template <typename T, int D>
struct BlockRows {
  static constexpr int RB = D * sizeof(T);   // bytes of a cache row
  static constexpr int kPitch = RB + 16;     // LDS pitch of a staged row
  static constexpr int kWaveBytes = 64 * kPitch;
  // The wavefront's 64 rows [r0, r0 + 64) of `src` (rows past `last` repeat it) into its staging
  // area, coalesced; afterwards every lane reads its own row from there.
  static __device__ __forceinline__ void stage(const T* src, int64_t slot0, int r0, int last, unsigned char* mine,
                                               int lane) {
#pragma unroll
    for (int i = 0; i < RB / 16; ++i) {
      const int ch = i * 64 + lane, row = ch / (RB / 16), col = ch % (RB / 16);
      *reinterpret_cast<u32x4*>(mine + row * kPitch + col * 16) =
          *reinterpret_cast<const u32x4*>(src + (slot0 + min(r0 + row, last)) * D + col * (16 / sizeof(T)));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
};

// Logits of the lane's row (staged in LDS at `myrow`) against the kQG queries from q0 on (fp64,
// exact for bf16 inputs).  Two elements per step: the row's bits come from LDS, the queries'
// elements through scalar loads, both fetched one step ahead (two register sets; the wait for a
// set is pinned before the other set's loads are issued, because scalar loads return out of
// order).
template <typename T, int D>
__device__ __forceinline__ void block_logits(const unsigned char* myrow, const double* aq_head, int q0, double* s,
                                             double row_scale) {
  typedef const double __attribute__((address_space(4))) * cptr;
  constexpr int ES = 2, NST = D / ES;
  typedef typename std::conditional<sizeof(T) == 1, uint16_t,
                                    typename std::conditional<sizeof(T) == 2, uint32_t, u32x2>::type>::type Raw;
  const cptr Qv = (cptr)(aq_head + int64_t(q0) * D);
#pragma unroll
  for (int u = 0; u < kQG; ++u) s[u] = 0.0;
  Raw rawA, rawB;
  double sA[kQG][ES], sB[kQG][ES];
  auto fetch = [&](int st, Raw& raw, double (&sv)[kQG][ES]) {
    raw = *reinterpret_cast<const Raw*>(myrow + st * ES * int(sizeof(T)));
#pragma unroll
    for (int u = 0; u < kQG; ++u)
#pragma unroll
      for (int e = 0; e < ES; ++e) sv[u][e] = Qv[u * D + st * ES + e];
  };
  auto step = [&](const Raw& raw, const double (&sv)[kQG][ES]) {
    double k[ES];
    if constexpr (sizeof(T) == 1) {  // fp8 codes, without the row's power of two (the caller applies it)
      k[0] = double(__builtin_amdgcn_cvt_f32_fp8(int(raw), 0));
      k[1] = double(__builtin_amdgcn_cvt_f32_fp8(int(raw), 1));
    } else if constexpr (sizeof(T) == 2) {
      k[0] = double(__uint_as_float(raw << 16));
      k[1] = double(__uint_as_float(raw & 0xFFFF0000u));
    } else {
      k[0] = double(__uint_as_float(raw[0]));
      k[1] = double(__uint_as_float(raw[1]));
    }
#pragma unroll
    for (int e = 0; e < ES; ++e)
#pragma unroll
      for (int u = 0; u < kQG; ++u) s[u] = fma(k[e], sv[u][e], s[u]);
  };
  fetch(0, rawA, sA);
#pragma unroll 1
  for (int st = 0; st < NST; st += 2) {
    scalar_arrived(sA[0][0]);
    fetch(st + 1, rawB, sB);
    __builtin_amdgcn_sched_barrier(0);  // the fetches go out before the FMAs, not among them
    step(rawA, sA);
    scalar_arrived(sB[0][0]);
    fetch(min(st + 2, NST - 1), rawA, sA);
    __builtin_amdgcn_sched_barrier(0);
    step(rawB, sB);
  }
  const double root_d = sqrt(double(D));
#pragma unroll
  for (int u = 0; u < kQG; ++u) s[u] = (sizeof(T) == 1 ? s[u] * row_scale : s[u]) / root_d;  // exact scaling of exact sums
}

template <typename T, int D>
__global__ __launch_bounds__(256) void block_stats(const int32_t* __restrict__ ctotal, const int32_t* __restrict__ meta,
                                                   const T* __restrict__ cK, const int8_t* __restrict__ cKe,
                                                   const double* __restrict__ aq, double* __restrict__ stat, int m, int G,
                                                   int maxq, int64_t slots) {
  typedef BlockRows<T, D> BR;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [4][64 rows] staged keys
  __shared__ double wm[4][kQG], wl[4][kQG];
  const int bhN = gridDim.x, bh = blockIdx.x, chunk = blockIdx.y;
  const int N = ctotal[bh];
  if (chunk * kChunk >= N) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t slot0 = int64_t(bh) * slots + meta[bh * 4 + 0];
  const int j = chunk * kChunk + tid, nc = N - m;
  const bool valid = j < N;
  unsigned char* mine = smem + w * BR::kWaveBytes;
  BR::stage(cK, slot0, chunk * kChunk + w * 64, N - 1, mine, lane);
  const unsigned char* myrow = mine + lane * BR::kPitch;
  double ksc = 1.0;
  if constexpr (sizeof(T) == 1) ksc = pow2_f64(cKe[slot0 + min(j, N - 1)]);
  const int nq = m * G, ngrp = (nq + kQG - 1) / kQG, gper = (ngrp + gridDim.z - 1) / gridDim.z;
  const int q_lo = blockIdx.z * gper * kQG, q_hi = min(nq, q_lo + gper * kQG);  // this workgroup's slice of the queries
  for (int q0 = q_lo; q0 < q_hi; q0 += kQG) {
    double s[kQG];
    block_logits<T, D>(myrow, aq + int64_t(bh) * maxq * D, q0, s, ksc);
#pragma unroll
    for (int u = 0; u < kQG; ++u) {
      const bool vis = valid && j <= nc + (q0 + u) / G;
      const double mw = wave_max(vis ? s[u] : -INFINITY);
      const double lw = wave_sum(vis ? exp(s[u] - mw) : 0.0);
      if (lane == 0) {
        wm[w][u] = mw;
        wl[w][u] = lw;
      }
    }
    __syncthreads();
    if (tid < kQG && q0 + tid < nq) {
      double M = fmax(fmax(wm[0][tid], wm[1][tid]), fmax(wm[2][tid], wm[3][tid]));
      double L = 0.0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (wm[i][tid] != -INFINITY) L += wl[i][tid] * exp(wm[i][tid] - M);
      double* st = stat + ((int64_t(chunk) * bhN + bh) * maxq + q0 + tid) * 2;
      st[0] = M;
      st[1] = L;
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void block_norm(const int32_t* __restrict__ ctotal, int32_t* __restrict__ ccount,
                                                  const double* __restrict__ stat, double* __restrict__ norm, int m, int G,
                                                  int maxq) {
  const int bhN = gridDim.x, bh = blockIdx.x;
  const int N = ctotal[bh], nch = (N + kChunk - 1) / kChunk, nq = m * G;
  if (threadIdx.x == 0) ccount[bh] = N;
  for (int q = threadIdx.x; q < nq; q += 256) {
    double M = -INFINITY;
    for (int c = 0; c < nch; ++c) M = fmax(M, stat[((int64_t(c) * bhN + bh) * maxq + q) * 2]);
    double L = 0.0;
    for (int c = 0; c < nch; ++c) {
      const double* st = stat + ((int64_t(c) * bhN + bh) * maxq + q) * 2;
      if (st[0] != -INFINITY) L += st[1] * exp(st[0] - M);
    }
    norm[(int64_t(bh) * maxq + q) * 2] = M;
    norm[(int64_t(bh) * maxq + q) * 2 + 1] = L;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void block_apply(const int32_t* __restrict__ ctotal, const int32_t* __restrict__ meta,
                                                   const T* __restrict__ cK, const T* __restrict__ cV,
                                                   const int8_t* __restrict__ cKe, const int8_t* __restrict__ cVe,
                                                   double* __restrict__ spart, const double* __restrict__ aq,
                                                   const double* __restrict__ norm, float* __restrict__ pout, int m,
                                                   int G, int maxq, int64_t slots, int rows_cap) {
  typedef BlockRows<T, D> BR;
  constexpr int CPL = D / 64;  // output columns per lane
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [4][64 rows] staged keys
  __shared__ float xch[4][kQG][D];
  const int bhN = gridDim.x, bh = blockIdx.x, chunk = blockIdx.y;
  const int N = ctotal[bh];
  if (chunk * kChunk >= N) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t slot0 = int64_t(bh) * slots + meta[bh * 4 + 0];
  const int r0 = chunk * kChunk + w * 64;  // the wavefront's first row
  const int j = r0 + lane, nc = N - m;
  const bool valid = j < N;
  unsigned char* mine = smem + w * BR::kWaveBytes;
  BR::stage(cK, slot0, r0, N - 1, mine, lane);
  const unsigned char* myrow = mine + lane * BR::kPitch;
  // the wavefront's 64 value rows, this lane's CPL columns of each, as raw words (fp8: two codes
  // in half a word; the row's power of two rides on the row's probability)
  constexpr int VW = sizeof(T) == 1 ? 1 : CPL * sizeof(T) / 4;
  uint32_t vraw[64][VW];
#pragma unroll
  for (int r = 0; r < 64; ++r) {
    if constexpr (sizeof(T) == 1) {
      static_assert(sizeof(T) != 1 || CPL == 2, "two codes per lane");
      vraw[r][0] = reinterpret_cast<const uint16_t*>(cV + (slot0 + min(r0 + r, N - 1)) * D)[lane];
    } else {
      const uint32_t* vr = reinterpret_cast<const uint32_t*>(cV + (slot0 + min(r0 + r, N - 1)) * D + lane * CPL);
#pragma unroll
      for (int c = 0; c < VW; ++c) vraw[r][c] = vr[c];
    }
  }
  double ksc = 1.0;
  float vsc = 1.f;
  if constexpr (sizeof(T) == 1) {
    ksc = pow2_f64(cKe[slot0 + min(j, N - 1)]);
    vsc = pow2_f32(cVe[slot0 + min(j, N - 1)]);
  }
  double sc = 0.0;
  const int nq = m * G, ngrp = (nq + kQG - 1) / kQG, gper = (ngrp + gridDim.z - 1) / gridDim.z;
  const int q_lo = blockIdx.z * gper * kQG, q_hi = min(nq, q_lo + gper * kQG);  // this workgroup's slice of the queries
  typedef const double __attribute__((address_space(4))) * cptr;
  for (int q0 = q_lo; q0 < q_hi; q0 += kQG) {
    double s[kQG];
    block_logits<T, D>(myrow, aq + int64_t(bh) * maxq * D, q0, s, ksc);
    const cptr nm = (cptr)(norm + (int64_t(bh) * maxq + q0) * 2);
    float p32[kQG];
#pragma unroll
    for (int u = 0; u < kQG; ++u) {
      const bool vis = valid && q0 + u < nq && j <= nc + (q0 + u) / G;
      const double p = vis ? exp(s[u] - nm[2 * u]) / nm[2 * u + 1] : 0.0;
      sc += p;  // Eq. 6: the slice's probabilities, in (token, query head) order
      p32[u] = sizeof(T) == 1 ? float(p) * vsc : float(p);
    }
    float acc[kQG][CPL];
#pragma unroll
    for (int u = 0; u < kQG; ++u)
#pragma unroll
      for (int c = 0; c < CPL; ++c) acc[u][c] = 0.f;
#pragma unroll
    for (int r = 0; r < 64; ++r) {
#pragma unroll
      for (int u = 0; u < kQG; ++u) {
        const float pr = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(p32[u]), r));
        if constexpr (sizeof(T) == 1) {
          acc[u][0] = fmaf(pr, __builtin_amdgcn_cvt_f32_fp8(int(vraw[r][0]), 0), acc[u][0]);
          acc[u][1] = fmaf(pr, __builtin_amdgcn_cvt_f32_fp8(int(vraw[r][0]), 1), acc[u][1]);
        } else if constexpr (sizeof(T) == 2) {
          static_assert(sizeof(T) != 2 || CPL == 2, "two bf16 columns per lane");
          acc[u][0] = fmaf(pr, __uint_as_float(vraw[r][0] << 16), acc[u][0]);
          acc[u][1] = fmaf(pr, __uint_as_float(vraw[r][0] & 0xFFFF0000u), acc[u][1]);
        } else {
#pragma unroll
          for (int c = 0; c < CPL; ++c) acc[u][c] = fmaf(pr, __uint_as_float(vraw[r][c]), acc[u][c]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kQG; ++u)
#pragma unroll
      for (int c = 0; c < CPL; ++c) xch[w][u][lane * CPL + c] = acc[u][c];
    __syncthreads();
    for (int x = tid; x < kQG * D; x += 256) {
      const int u = x / D, c = x % D;
      if (q0 + u < nq)
        pout[((int64_t(chunk) * bhN + bh) * maxq + q0 + u) * D + c] = (xch[0][u][c] + xch[1][u][c]) + (xch[2][u][c] + xch[3][u][c]);
    }
    __syncthreads();
  }
  if (valid) spart[(int64_t(blockIdx.z) * bhN + bh) * rows_cap + j] = sc;
}

// Eq. 6 for the block: a row's score grows by the slices' sums, added in slice order (slices hold
// ascending ranges of (token, query head)).
__global__ __launch_bounds__(256) void block_scores(const int32_t* __restrict__ ctotal, const int32_t* __restrict__ meta,
                                                    double* __restrict__ cscore, const double* __restrict__ spart,
                                                    int nslice, int64_t slots, int rows_cap) {
  const int bhN = gridDim.x, bh = blockIdx.x, j = blockIdx.y * 256 + threadIdx.x;
  if (j >= ctotal[bh]) return;
  const int64_t slot0 = int64_t(bh) * slots + meta[bh * 4 + 0];
  double sc = cscore[slot0 + j];
  for (int z = 0; z < nslice; ++z) sc += spart[(int64_t(z) * bhN + bh) * rows_cap + j];
  cscore[slot0 + j] = sc;
}

template <typename OT, int D>
__global__ __launch_bounds__(D) void block_finish(const int32_t* __restrict__ ctotal, const float* __restrict__ pout,
                                                  OT* __restrict__ out, View ov, int G, int maxq, int Hkv) {
  const int bhN = gridDim.x, bh = blockIdx.x, q = blockIdx.y, c = threadIdx.x;
  const int N = ctotal[bh], nch = (N + kChunk - 1) / kChunk;
  float t = 0.f;
  for (int ch = 0; ch < nch; ++ch) t += pout[((int64_t(ch) * bhN + bh) * maxq + q) * D + c];
  const int b = bh / Hkv, hk = bh % Hkv;
  out[b * ov.sb + (hk * G + q % G) * ov.sh + int64_t(q / G) * ov.sn + c] = Elem<OT>::from_f32(t);
}

// fp8 cache: the same permutation, decoding every row into the bf16 copy on the way (a code times
// a power of two has four significant bits: exact in bf16).  One wavefront per row, D = 128.
__global__ __launch_bounds__(256) void permute_decode_rows(const int32_t* __restrict__ on, const int32_t* __restrict__ meta,
                                                           const int32_t* __restrict__ rank, const uint8_t* __restrict__ cK,
                                                           const uint8_t* __restrict__ cV, const int8_t* __restrict__ cKe,
                                                           const int8_t* __restrict__ cVe, uint16_t* __restrict__ oK,
                                                           uint16_t* __restrict__ oV, int npad, int64_t slots) {
  constexpr int D = 128;
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y, lane = threadIdx.x & 63;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= on[bh]) return;
  const int64_t src = bh * slots + meta[bh * 4 + 0] + j;
  const int64_t dst = (bh * npad + rank[bh * npad + j]) * D;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const uint16_t codes = reinterpret_cast<const uint16_t*>((which ? cV : cK) + src * D)[lane];
    const float sc = pow2_f32((which ? cVe : cKe)[src]);
    const float v0 = Elem<uint8_t>::to_f32(uint8_t(codes & 0xFF)) * sc, v1 = Elem<uint8_t>::to_f32(uint8_t(codes >> 8)) * sc;
    reinterpret_cast<uint32_t*>((which ? oV : oK) + dst)[lane] = (__float_as_uint(v0) >> 16) | (__float_as_uint(v1) & 0xFFFF0000u);
  }
}

// fp8 cache: the block's K and V rows encoded into the cache (one wavefront per new row).
__global__ __launch_bounds__(256) void block_rows_fp8(const int32_t* __restrict__ ccount, const int32_t* __restrict__ meta,
                                                      uint8_t* __restrict__ cK, uint8_t* __restrict__ cV,
                                                      int8_t* __restrict__ cKe, int8_t* __restrict__ cVe,
                                                      const uint16_t* __restrict__ kn, View kv,
                                                      const uint16_t* __restrict__ vn, View vv, int m, int64_t slots) {
  constexpr int D = 128;
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y, lane = threadIdx.x & 63;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= m) return;
  const int64_t dst = bh * slots + meta[bh * 4 + 0] + ccount[bh] + i;  // (the entry count moves later, in block_norm)
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const uint16_t* src = which ? vn + b * vv.sb + hk * vv.sh + int64_t(i) * vv.sn : kn + b * kv.sb + hk * kv.sh + int64_t(i) * kv.sn;
    const uint32_t two = reinterpret_cast<const uint32_t*>(src)[lane];
    const double x0 = double(__uint_as_float(two << 16)), x1 = double(__uint_as_float(two & 0xFFFF0000u));
    const int e = fp8_row_exponent(wave_max(fmax(fabs(x0), fabs(x1))));
    reinterpret_cast<uint16_t*>((which ? cV : cK) + dst * D)[lane] =
        uint16_t(fp8_encode(ldexp(x0, -e))) | uint16_t(uint16_t(fp8_encode(ldexp(x1, -e))) << 8);
    if (lane == 0) (which ? cVe : cKe)[dst] = int8_t(e);
  }
}

template <typename T, int D>
hipError_t run_block_attend(d2o_ctx* c, int layer, View q, View k, View v, View out, int m, int first_pos, hipStream_t s) {
  typedef typename std::conditional<sizeof(T) == 1, uint16_t, T>::type IT;  // the tensors' type (an fp8 cache takes bf16 tensors)
  const d2o_config& cf = c->cfg;
  const int G = cf.n_q_heads / cf.n_kv_heads, bh = cf.batch * cf.n_kv_heads, maxq = c->ap_maxq;
  const size_t lo = size_t(layer) * bh;
  int32_t* ccount = c->ccount + lo;
  int32_t* ctotal = c->ctotal + lo;
  const int32_t* meta = c->meta + lo * 4;
  int max_rows = 0;
  for (const auto& mt : c->layers[layer].meta) max_rows = std::max(max_rows, mt.budget + m);
  const int nch = (max_rows + kChunk - 1) / kChunk;
  if (nch > c->ap_nch || m * G > maxq) return hipErrorInvalidValue;
  // few heads and chunks give few workgroups: the queries of a head are cut into slices that run
  // as workgroups of their own, enough of them to fill the chip a few times over
  const int ngrp = (m * G + kQG - 1) / kQG;
  const int nslice = std::max(1, std::min({kMaxQuerySlices, ngrp, 4096 / std::max(1, bh * nch)}));
  block_begin<T, IT, D><<<dim3(cf.n_kv_heads, cf.batch, 8), 256, 0, s>>>(ccount, ctotal, meta, (T*)c->cacheK, (T*)c->cacheV, c->cscore,
                                                                         c->cpos, (const IT*)q.ptr, q, (const IT*)k.ptr, k,
                                                                         (const IT*)v.ptr, v, c->ap_q, m, G, maxq, first_pos,
                                                                         cf.slots_per_seq);
  if constexpr (sizeof(T) == 1)
    block_rows_fp8<<<dim3((m + 3) / 4, cf.n_kv_heads, cf.batch), 256, 0, s>>>(ccount, meta, (uint8_t*)c->cacheK, (uint8_t*)c->cacheV,
                                                                               c->cKe, c->cVe, (const uint16_t*)k.ptr, k,
                                                                               (const uint16_t*)v.ptr, v, m, cf.slots_per_seq);
  constexpr int kRowsLds = 4 * BlockRows<T, D>::kWaveBytes;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(block_stats<T, D>), hipFuncAttributeMaxDynamicSharedMemorySize, kRowsLds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(block_apply<T, D>), hipFuncAttributeMaxDynamicSharedMemorySize, kRowsLds);
  if (e != hipSuccess) return e;
  block_stats<T, D><<<dim3(bh, nch, nslice), 256, kRowsLds, s>>>(ctotal, meta, (const T*)c->cacheK, c->cKe, c->ap_q, c->ap_stat, m, G,
                                                              maxq, cf.slots_per_seq);
  block_norm<<<dim3(bh), 256, 0, s>>>(ctotal, ccount, c->ap_stat, c->ap_norm, m, G, maxq);
  const int rows_cap = c->ap_nch * kChunk;
  block_apply<T, D><<<dim3(bh, nch, nslice), 256, kRowsLds, s>>>(ctotal, meta, (const T*)c->cacheK, (const T*)c->cacheV, c->cKe, c->cVe,
                                                              c->ap_spart, c->ap_q, c->ap_norm, c->ap_out, m, G, maxq,
                                                              cf.slots_per_seq, rows_cap);
  block_scores<<<dim3(bh, nch), 256, 0, s>>>(ctotal, meta, c->cscore, c->ap_spart, nslice, cf.slots_per_seq, rows_cap);
  if (cf.out_f32)
    block_finish<float, D><<<dim3(bh, m * G), D, 0, s>>>(ctotal, c->ap_out, (float*)out.ptr, out, G, maxq, cf.n_kv_heads);
  else
    block_finish<IT, D><<<dim3(bh, m * G), D, 0, s>>>(ctotal, c->ap_out, (IT*)out.ptr, out, G, maxq, cf.n_kv_heads);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_cache_sort(d2o_ctx* c, int layer, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int32_t* meta = c->meta + size_t(layer) * cf.batch * cf.n_kv_heads * 4;
  const int32_t* ccount = c->ccount + size_t(layer) * cf.batch * cf.n_kv_heads;
  int max_rows = 0;
  for (const auto& mt : c->layers[layer].meta) max_rows = std::max(max_rows, mt.budget + c->grow);
  rank_by_position<<<dim3(cf.n_kv_heads, cf.batch, (max_rows + 1023) / 1024), 256, 0, s>>>(ccount, meta, c->cscore, c->cpos, c->app_rank,
                                                                  c->app_pos, c->app_score, c->app_n, c->npad,
                                                                  cf.slots_per_seq);
  if (cf.cache_fp8) {
    permute_decode_rows<<<dim3((max_rows + 3) / 4, cf.n_kv_heads, cf.batch), 256, 0, s>>>(
        c->app_n, meta, c->app_rank, (const uint8_t*)c->cacheK, (const uint8_t*)c->cacheV, c->cKe, c->cVe,
        (uint16_t*)c->app_K, (uint16_t*)c->app_V, c->npad, cf.slots_per_seq);
  } else if (cf.dtype == D2O_BF16) {
    const int rows = 256 / (cf.head_dim / 8);
    permute_rows<uint16_t><<<dim3((max_rows + rows - 1) / rows, cf.n_kv_heads, cf.batch), 256, 0, s>>>(
        c->app_n, meta, c->app_rank, (const uint16_t*)c->cacheK, (const uint16_t*)c->cacheV, (uint16_t*)c->app_K,
        (uint16_t*)c->app_V, c->npad, cf.head_dim, cf.slots_per_seq);
  } else {
    const int rows = 256 / (cf.head_dim / 4);
    permute_rows<float><<<dim3((max_rows + rows - 1) / rows, cf.n_kv_heads, cf.batch), 256, 0, s>>>(
        c->app_n, meta, c->app_rank, (const float*)c->cacheK, (const float*)c->cacheV, (float*)c->app_K,
        (float*)c->app_V, c->npad, cf.head_dim, cf.slots_per_seq);
  }
  return hipGetLastError();
}

hipError_t launch_block_attend(d2o_ctx* c, int layer, View q, View k, View v, View out, int m, int first_pos,
                               hipStream_t s) {
  const d2o_config& cf = c->cfg;
  if (cf.cache_fp8) return run_block_attend<uint8_t, 128>(c, layer, q, k, v, out, m, first_pos, s);
  if (cf.dtype == D2O_BF16) return run_block_attend<uint16_t, 128>(c, layer, q, k, v, out, m, first_pos, s);
  if (cf.head_dim == 64) return run_block_attend<float, 64>(c, layer, q, k, v, out, m, first_pos, s);
  return run_block_attend<float, 128>(c, layer, q, k, v, out, m, first_pos, s);
}

}  // namespace d2o
