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

template <int U>  // slots per thread: 4 amortises the LDS reads on large caches, 1 gives small ones more workgroups
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
  // A workgroup owns 256 U slots at a time (a thread U of them; the workgroups of a head stride
  // over its slots); all positions of the head pass through LDS tile by tile, and each owned
  // slot counts the smaller ones (all threads read the same LDS words, eight at a time).
  for (int j0 = blockIdx.z * 256 * U; j0 < n; j0 += gridDim.z * 256 * U) {
    int mine[U], cnt[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = j0 + u * 256 + tid;
      mine[u] = j < n ? cpos[slot0 + j] : 0x7FFFFFFF;
      cnt[u] = 0;
    }
    for (int t0 = 0; t0 < n; t0 += kRankTile) {
      __syncthreads();
      const int lim = min(kRankTile, (n - t0 + 7) & ~7);  // the padding compares as "not smaller"
      for (int i = tid; i < lim; i += 256) tile[i] = t0 + i < n ? cpos[slot0 + t0 + i] : 0x7FFFFFFF;
      __syncthreads();
      for (int i = 0; i < lim; i += 8) {
        const int4 pa = *reinterpret_cast<const int4*>(&tile[i]), pb = *reinterpret_cast<const int4*>(&tile[i + 4]);
#pragma unroll
        for (int u = 0; u < U; ++u)
          cnt[u] += (pa.x < mine[u]) + (pa.y < mine[u]) + (pa.z < mine[u]) + (pa.w < mine[u]) + (pb.x < mine[u]) +
                    (pb.y < mine[u]) + (pb.z < mine[u]) + (pb.w < mine[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
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
// Both products are dense contractions (rows x queries x d, queries x d x rows) and run on the
// matrix cores: the fp64 16x16x4 instruction for the logits (its sums of products of bf16 or
// fp8 values are exact, so they do not depend on the order of the contraction), the fp32
// 16x16x4 instruction for P V.
//
//   block_begin   per head: appends the block's K, V rows (score 0, positions first_pos + i),
//                 lays the queries out as fp64 vectors, sets the entry count to N.
//   block_stats   per (head, 256 rows, slice of the queries): the rows are staged in LDS once; a
//                 wavefront takes tiles of 16 queries and forms their logits against the 256
//                 rows, 64 rows at a time; per query the maximum and exp-sum over the chunk's
//                 visible rows.
//   block_norm    per head and query: maximum and exact normaliser over the chunks.
//   block_apply   the same tiling: logits again, p = exp(s - max) / normaliser; per row the sum
//                 of the p of every query that sees it; the wavefront's 16 x d partial output
//                 tile over the 256 rows, accumulated by the fp32 matrix instruction whose A
//                 operand is the probability tile as the logits' instruction left it.
//   block_scores  per row: score += the sums (Eq. 6).
//   block_finish  per head and query: the chunks' partial output rows added in ascending order.
// A head's queries are cut into up to kMaxQuerySlices slices that run as workgroups of their own
// (a block on a cache of a few thousand rows is too little work per head to fill the chip
// otherwise); a row's score then grows by the slices' sums in slice order.
//
// Register layouts of the two instructions (lane l, c = l % 16, kq = l / 16):
//   operands   A[i = c][k = kq], B[k = kq][j = c]
//   fp64 result register r: D[i = 4 r + kq][j = c]
//   fp32 result register r: D[i = 4 kq + r][j = c]
// so with rows as i and queries as j, lane l holds the logits of query c against the rows
// 16 t + 4 r + kq of a 64-row group (t = 0..3), and for fixed (t, r) these values, taken as the A
// operand of the fp32 instruction (i = query c, k = kq), meet the four consecutive rows
// 16 t + 4 r + kq of V as B.
constexpr int kQT = 16;  // queries per tile

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
  const int nq = m * G, nq_pad = (nq + kQT - 1) / kQT * kQT;  // the queries of a last, partial tile are zero
  for (int x = tid; x < nq_pad * D; x += nt) {
    const int qi = x / D, c = x % D;
    double v = 0.0;
    if (qi < nq) v = Elem<IT>::to_f64(q[b * qv.sb + (hk * G + qi % G) * qv.sh + int64_t(qi / G) * qv.sn + c]);
    aq[(bh * maxq + qi) * D + c] = v;
  }
  if (tid == 0) ctotal[bh] = count + m;
}

template <typename T, int D>
struct BlockRows {
  static constexpr int RB = D * sizeof(T);   // bytes of a cache row
  static constexpr int kPitch = RB + 16;     // LDS pitch of a staged row (conflict-free for the operand reads below)
  static constexpr int kWaveBytes = 64 * kPitch;
  static constexpr int kRowsBytes = 4 * kWaveBytes;                 // the chunk's 256 rows
  static constexpr int kScaleBytes = sizeof(T) == 1 ? 256 * 12 : 0;  // fp8: the rows' powers of two (K as fp64, V as fp32)
  static constexpr int KS = D / 4;           // contraction steps of the logits
  static constexpr int CT = D / 16;          // output column tiles of P V (lane c holds columns CT c .. CT c + CT - 1)
  // The chunk's rows [r0, r0 + 256) of `src` (rows past `last` repeat it) into LDS, each
  // wavefront 64 of them, coalesced; fp8: the rows' powers of two behind them.
  static __device__ __forceinline__ void stage(const T* src, const int8_t* ke, const int8_t* ve, int64_t slot0, int r0,
                                               int last, unsigned char* smem, int tid) {
    const int lane = tid & 63, w = tid >> 6;
    unsigned char* mine = smem + w * kWaveBytes;
#pragma unroll
    for (int i = 0; i < RB / 16; ++i) {
      const int ch = i * 64 + lane, row = ch / (RB / 16), col = ch % (RB / 16);
      *reinterpret_cast<u32x4*>(mine + row * kPitch + col * 16) =
          *reinterpret_cast<const u32x4*>(src + (slot0 + min(r0 + w * 64 + row, last)) * D + col * (16 / sizeof(T)));
    }
    if constexpr (sizeof(T) == 1) {
      reinterpret_cast<double*>(smem + kRowsBytes)[tid] = pow2_f64(ke[slot0 + min(r0 + tid, last)]);
      reinterpret_cast<float*>(smem + kRowsBytes + 256 * 8)[tid] = pow2_f32(ve[slot0 + min(r0 + tid, last)]);
    }
    __syncthreads();
  }
  // element k of staged row `row` (0..255) as fp64 (fp8: the code, without the row's power of two)
  static __device__ __forceinline__ double elem(const unsigned char* smem, int row, int k) {
    const unsigned char* p = smem + row * kPitch + k * int(sizeof(T));
    if constexpr (sizeof(T) == 1) return double(__builtin_amdgcn_cvt_f32_fp8(int(*p), 0));
    else if constexpr (sizeof(T) == 2) return double(__uint_as_float(uint32_t(*reinterpret_cast<const uint16_t*>(p)) << 16));
    else return double(*reinterpret_cast<const float*>(p));
  }
  // The query tile's B operands: bq[s] = element 4 s + kq of query q0 + c.
  static __device__ __forceinline__ void load_queries(const double* aq_head, int q0, int lane, double (&bq)[KS]) {
    const double* qp = aq_head + int64_t(q0 + (lane & 15)) * D + (lane >> 4);
#pragma unroll
    for (int s = 0; s < KS; ++s) bq[s] = qp[4 * s];
  }
  // Logits of the tile's 16 queries against the rows [64 g, 64 g + 64) of the chunk:
  // S[t][r] = (row 64 g + 16 t + 4 r + kq) . (query c) / sqrt(d) (fp8: times the row's power of two, exactly).
  static __device__ __forceinline__ void logits(const unsigned char* smem, int g, int lane, const double (&bq)[KS],
                                                f64x4 (&S)[4]) {
    const int c = lane & 15, kq = lane >> 4;
#pragma unroll
    for (int t = 0; t < 4; ++t) S[t] = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int t = 0; t < 4; ++t)
        S[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(elem(smem, g * 64 + t * 16 + c, 4 * s + kq), bq[s], S[t], 0, 0, 0);
    // (times the rounded reciprocal of sqrt(d), exact for d = 64: a block's logits are compared
    // within the float tolerance, and a division per element would cost a tenth of the pass)
    const double inv_root_d = 1.0 / sqrt(double(D));
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        double v = S[t][r];
        if constexpr (sizeof(T) == 1) v *= reinterpret_cast<const double*>(smem + kRowsBytes)[g * 64 + t * 16 + 4 * r + kq];
        S[t][r] = v * inv_root_d;
      }
  }
};

// sum / maximum over the four lanes that hold the same query column (kq = 0..3)
__device__ __forceinline__ double kq_max(double v) {
  v = fmax(v, __shfl_xor(v, 16, 64));
  return fmax(v, __shfl_xor(v, 32, 64));
}
__device__ __forceinline__ double kq_sum(double v) {
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void block_stats(const int32_t* __restrict__ ctotal, const int32_t* __restrict__ meta,
                                                   const T* __restrict__ cK, const int8_t* __restrict__ cKe,
                                                   const double* __restrict__ aq, double* __restrict__ stat, int m, int G,
                                                   int maxq, int64_t slots, int tiles_per_slice) {
  typedef BlockRows<T, D> BR;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int bhN = gridDim.x, bh = blockIdx.x, chunk = blockIdx.y;
  const int N = ctotal[bh];
  if (chunk * kChunk >= N) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, c = lane & 15, kq = lane >> 4;
  const int64_t slot0 = int64_t(bh) * slots + meta[bh * 4 + 0];
  const int nc = N - m, nq = m * G, ntile = (nq + kQT - 1) / kQT;
  BR::stage(cK, cKe, cKe, slot0, chunk * kChunk, N - 1, smem, tid);
  const int ngroup = min(4, (N - chunk * kChunk + 63) / 64);  // 64-row groups of the chunk that hold rows
  const int t_hi = min(ntile, (blockIdx.z + 1) * tiles_per_slice);
  for (int qt = blockIdx.z * tiles_per_slice + w; qt < t_hi; qt += 4) {  // this wavefront's query tiles
    const int q0 = qt * kQT, query = q0 + c;
    double bq[BR::KS];
    BR::load_queries(aq + int64_t(bh) * maxq * D, q0, lane, bq);
    const int seen = nc + query / G;  // the last row this query attends to
    double M = -INFINITY, L = 0.0;
#pragma unroll 1
    for (int g = 0; g < ngroup; ++g) {
      f64x4 S[4];
      BR::logits(smem, g, lane, bq, S);
      const int j0 = chunk * kChunk + g * 64 + kq;
      double mg = -INFINITY;
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int j = j0 + t * 16 + 4 * r;
          if (j < N && j <= seen) mg = fmax(mg, S[t][r]);
        }
      mg = kq_max(mg);
      if (mg == -INFINITY) continue;  // (the same for the four lanes of a query)
      double lg = 0.0;
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int j = j0 + t * 16 + 4 * r;
          if (j < N && j <= seen) lg += exp(S[t][r] - mg);
        }
      lg = kq_sum(lg);
      const double Mn = fmax(M, mg);
      L = (M == -INFINITY ? 0.0 : L * exp(M - Mn)) + lg * exp(mg - Mn);
      M = Mn;
    }
    if (kq == 0 && query < nq) {
      double* st = stat + ((int64_t(chunk) * bhN + bh) * maxq + query) * 2;
      st[0] = M;
      st[1] = L;
    }
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
                                                   int G, int maxq, int64_t slots, int rows_cap, int tiles_per_slice) {
  typedef BlockRows<T, D> BR;
  constexpr int CT = BR::CT;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // behind the rows (and the fp8 scales): per wavefront and row, the sum of its queries' probabilities
  double* rs = reinterpret_cast<double*>(smem + BR::kRowsBytes + BR::kScaleBytes);
  const int bhN = gridDim.x, bh = blockIdx.x, chunk = blockIdx.y;
  const int N = ctotal[bh];
  if (chunk * kChunk >= N) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, c = lane & 15, kq = lane >> 4;
  const int64_t slot0 = int64_t(bh) * slots + meta[bh * 4 + 0];
  const int nc = N - m, nq = m * G, ntile = (nq + kQT - 1) / kQT;
#pragma unroll
  for (int i = 0; i < 4; ++i) rs[i * 256 + tid] = 0.0;
  BR::stage(cK, cKe, cVe, slot0, chunk * kChunk, N - 1, smem, tid);
  const int ngroup = min(4, (N - chunk * kChunk + 63) / 64);
  const int t_hi = min(ntile, (blockIdx.z + 1) * tiles_per_slice);
  for (int qt = blockIdx.z * tiles_per_slice + w; qt < t_hi; qt += 4) {
    const int q0 = qt * kQT, query = q0 + c;
    double bq[BR::KS];
    BR::load_queries(aq + int64_t(bh) * maxq * D, q0, lane, bq);
    const int seen = query < nq ? nc + query / G : -1;  // a padding query sees nothing
    const double M = norm[(int64_t(bh) * maxq + query) * 2], Linv = 1.0 / norm[(int64_t(bh) * maxq + query) * 2 + 1];
    f32x4 O[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) O[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int g = 0; g < ngroup; ++g) {
      f64x4 S[4];
      BR::logits(smem, g, lane, bq, S);
      const int j0 = chunk * kChunk + g * 64 + kq;
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = g * 64 + t * 16 + 4 * r + kq, j = j0 + t * 16 + 4 * r;
          // (the division by the normaliser is a multiplication by its reciprocal here: the
          // probabilities are compared within the float tolerance, never bit for bit)
          const double p = (j < N && j <= seen) ? exp(S[t][r] - M) * Linv : 0.0;
          // Eq. 6: the row's sum over the tile's queries, then over the wavefront's tiles
          double ps = p;
          ps += __shfl_xor(ps, 1, 64);
          ps += __shfl_xor(ps, 2, 64);
          ps += __shfl_xor(ps, 4, 64);
          ps += __shfl_xor(ps, 8, 64);
          if (c == 0) rs[w * 256 + row] += ps;
          // P V: this (t, r) is one contraction step over the rows 16 t + 4 r + kq
          float pa = float(p);
          if constexpr (sizeof(T) == 1) pa *= reinterpret_cast<const float*>(smem + BR::kRowsBytes + 256 * 8)[row];
          const T* vrow = cV + (slot0 + min(j, N - 1)) * D + c * CT;
          float vb[CT];
          if constexpr (sizeof(T) == 1) {
            static_assert(sizeof(T) != 1 || CT == 8, "eight codes per lane");
            const u32x2 raw = *reinterpret_cast<const u32x2*>(vrow);
#pragma unroll
            for (int wd = 0; wd < 2; ++wd) {
              vb[4 * wd] = __builtin_amdgcn_cvt_f32_fp8(int(raw[wd]), 0);
              vb[4 * wd + 1] = __builtin_amdgcn_cvt_f32_fp8(int(raw[wd]), 1);
              vb[4 * wd + 2] = __builtin_amdgcn_cvt_f32_fp8(int(raw[wd]), 2);
              vb[4 * wd + 3] = __builtin_amdgcn_cvt_f32_fp8(int(raw[wd]), 3);
            }
          } else if constexpr (sizeof(T) == 2) {
            static_assert(sizeof(T) != 2 || CT == 8, "eight bf16 columns per lane");
            const u32x4 raw = *reinterpret_cast<const u32x4*>(vrow);
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
              vb[2 * wd] = __uint_as_float(raw[wd] << 16);
              vb[2 * wd + 1] = __uint_as_float(raw[wd] & 0xFFFF0000u);
            }
          } else {
#pragma unroll
            for (int x = 0; x < CT; x += 4) {
              const u32x4 raw = *reinterpret_cast<const u32x4*>(vrow + x);
#pragma unroll
              for (int e = 0; e < 4; ++e) vb[x + e] = __uint_as_float(raw[e]);
            }
          }
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) O[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(pa, vb[ct], O[ct], 0, 0, 0);
        }
    }
    // O[ct][r]: query q0 + 4 kq + r, column CT c + ct
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int qo = q0 + 4 * kq + r;
      if (qo < nq) {
        float* dst = pout + ((int64_t(chunk) * bhN + bh) * maxq + qo) * D + c * CT;
#pragma unroll
        for (int x = 0; x < CT; x += 4) *reinterpret_cast<f32x4*>(dst + x) = f32x4{O[x][r], O[x + 1][r], O[x + 2][r], O[x + 3][r]};
      }
    }
  }
  __syncthreads();
  const int j = chunk * kChunk + tid;
  if (j < N) spart[(int64_t(blockIdx.z) * bhN + bh) * rows_cap + j] = (rs[tid] + rs[256 + tid]) + (rs[512 + tid] + rs[768 + tid]);
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
  // few heads and chunks give few workgroups: the query tiles of a head are cut into slices that
  // run as workgroups of their own (whole rounds of the four wavefronts), enough of them to fill
  // the chip a few times over
  const int ntile = (m * G + kQT - 1) / kQT;
  const int want = std::max(1, std::min(kMaxQuerySlices, 2048 / std::max(1, bh * nch)));
  const int tiles_per_slice = 4 * ((ntile + 4 * want - 1) / (4 * want));
  const int nslice = (ntile + tiles_per_slice - 1) / tiles_per_slice;
  block_begin<T, IT, D><<<dim3(cf.n_kv_heads, cf.batch, 8), 256, 0, s>>>(ccount, ctotal, meta, (T*)c->cacheK, (T*)c->cacheV, c->cscore,
                                                                         c->cpos, (const IT*)q.ptr, q, (const IT*)k.ptr, k,
                                                                         (const IT*)v.ptr, v, c->ap_q, m, G, maxq, first_pos,
                                                                         cf.slots_per_seq);
  if constexpr (sizeof(T) == 1)
    block_rows_fp8<<<dim3((m + 3) / 4, cf.n_kv_heads, cf.batch), 256, 0, s>>>(ccount, meta, (uint8_t*)c->cacheK, (uint8_t*)c->cacheV,
                                                                               c->cKe, c->cVe, (const uint16_t*)k.ptr, k,
                                                                               (const uint16_t*)v.ptr, v, m, cf.slots_per_seq);
  typedef BlockRows<T, D> BR;
  constexpr int kStatsLds = BR::kRowsBytes + BR::kScaleBytes, kApplyLds = kStatsLds + 4 * 256 * int(sizeof(double));
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(block_stats<T, D>), hipFuncAttributeMaxDynamicSharedMemorySize, kStatsLds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(block_apply<T, D>), hipFuncAttributeMaxDynamicSharedMemorySize, kApplyLds);
  if (e != hipSuccess) return e;
  block_stats<T, D><<<dim3(bh, nch, nslice), 256, kStatsLds, s>>>(ctotal, meta, (const T*)c->cacheK, c->cKe, c->ap_q, c->ap_stat, m, G,
                                                               maxq, cf.slots_per_seq, tiles_per_slice);
  block_norm<<<dim3(bh), 256, 0, s>>>(ctotal, ccount, c->ap_stat, c->ap_norm, m, G, maxq);
  const int rows_cap = c->ap_nch * kChunk;
  block_apply<T, D><<<dim3(bh, nch, nslice), 256, kApplyLds, s>>>(ctotal, meta, (const T*)c->cacheK, (const T*)c->cacheV, c->cKe, c->cVe,
                                                               c->ap_spart, c->ap_q, c->ap_norm, c->ap_out, m, G, maxq,
                                                               cf.slots_per_seq, rows_cap, tiles_per_slice);
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
  if (max_rows <= 8192)
    rank_by_position<1><<<dim3(cf.n_kv_heads, cf.batch, (max_rows + 255) / 256), 256, 0, s>>>(
        ccount, meta, c->cscore, c->cpos, c->app_rank, c->app_pos, c->app_score, c->app_n, c->npad, cf.slots_per_seq);
  else
    rank_by_position<4><<<dim3(cf.n_kv_heads, cf.batch, (max_rows + 1023) / 1024), 256, 0, s>>>(
        ccount, meta, c->cscore, c->cpos, c->app_rank, c->app_pos, c->app_score, c->app_n, c->npad, cf.slots_per_seq);
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
