// Token-level operation after prompt encoding (Sec. 4.2): selection (Eq. 7-8), compaction into
// the cache, nearest-neighbour matching (Eq. 9), the initial threshold (Eq. 10, t = 0) and the
// similarity-weighted merge (Eq. 11-12).
//
// Every decision (top-N membership, arg-max of the cosine, threshold test) is taken on exact
// integer keys or in fp64 with the operation order of the defining formulas, so that index
// outputs do not depend on reduction shapes; the bf16 matrix-core product in match_filter_bf16
// only pre-selects candidates and flags rows whose two best candidates are too close for fp32.
#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace {

// ------------------------------------------------------------------------------------------
// Selection.  One workgroup per (sequence, KV head).  Radix-select of the N_hh-th largest
// score among positions [T, n-M) on order-preserving 32-bit keys, then an ordered compaction
// that keeps, among keys equal to the threshold, the lowest positions first.

__device__ __forceinline__ uint32_t order_key(float x) {
  if (x == 0.f) x = 0.f;  // -0 and +0 compare equal
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ uint64_t order_key(double x) {
  if (x == 0.0) x = 0.0;
  const uint64_t b = uint64_t(__double_as_longlong(x));
  return (b & 0x8000000000000000ull) ? ~b : (b | 0x8000000000000000ull);
}

// Exclusive prefix sums of two 0/1 flags over the block, in thread order.  Returns the
// exclusive counts and adds the block totals to *tot_a / *tot_b (read by all threads).
__device__ __forceinline__ void block_scan2(bool fa, bool fb, int& ex_a, int& ex_b, int& tot_a, int& tot_b,
                                            int* wa, int* wb) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const unsigned long long ma = __ballot(fa), mb = __ballot(fb);
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  const int pa = __popcll(ma & below), pb = __popcll(mb & below);
  __syncthreads();
  if (lane == 0) {
    wa[w] = __popcll(ma);
    wb[w] = __popcll(mb);
  }
  __syncthreads();
  int oa = 0, ob = 0, ta = 0, tb = 0;
  for (int i = 0; i < nw; ++i) {
    if (i < w) {
      oa += wa[i];
      ob += wb[i];
    }
    ta += wa[i];
    tb += wb[i];
  }
  ex_a = oa + pa;
  ex_b = ob + pb;
  tot_a = ta;
  tot_b = tb;
}

// Exclusive prefix sums of one integer per thread over the block, in thread order, and the
// block total (read by all threads).
__device__ __forceinline__ void block_scan_int(int v, int& ex, int& tot, int* wa) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) wa[w] = inc;
  __syncthreads();
  int off = 0, total = 0;
  for (int i = 0; i < nw; ++i) {
    if (i < w) off += wa[i];
    total += wa[i];
  }
  ex = off + inc - v;
  tot = total;
}

// S: score type (fp32 column sums after prompt encoding; fp64 cumulative scores of a cache that a
// block of tokens was appended to).  nvec, when given, holds the number of entries per head.
template <typename S>
__global__ __launch_bounds__(1024) void select_kernel(const S* __restrict__ score, const int32_t* __restrict__ meta,
                                                      int32_t* __restrict__ ret, int32_t* __restrict__ evi,
                                                      int32_t* __restrict__ cnt, int n_all, const int32_t* __restrict__ nvec,
                                                      int npad, int n_sink) {
  typedef decltype(order_key(S())) Key;
  constexpr int kTopShift = int(sizeof(Key)) * 8 - 8;
  __shared__ int hist[256];
  __shared__ int wa[16];
  __shared__ Key sh_prefix;
  __shared__ int sh_need;
  const int hk = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int n = nvec ? nvec[bh] : n_all;
  const S* sc = score + bh * npad;
  int32_t* r = ret + bh * npad;
  int32_t* e = evi + bh * npad;
  const int budget = meta[bh * 4 + 1], recent = meta[bh * 4 + 2];
  const int tid = threadIdx.x;
  if (budget >= n) {
    for (int j = tid; j < n; j += blockDim.x) r[j] = j;
    if (tid == 0) {
      cnt[bh * 2] = n;
      cnt[bh * 2 + 1] = 0;
    }
    return;
  }
  const int lo = n_sink, hi = n - recent;   // middle range [lo, hi)
  const int nhh = budget - n_sink - recent;  // heavy hitters to keep, 0 <= nhh < hi - lo
  // ---- radix select: find the key value of the nhh-th largest and how many equal keys to take
  Key prefix = 0, mask = 0;
  int need = nhh;
  if (nhh > 0) {
    for (int shift = kTopShift; shift >= 0; shift -= 8) {
      for (int i = tid; i < 256; i += blockDim.x) hist[i] = 0;
      __syncthreads();
      for (int j = lo + tid; j < hi; j += blockDim.x) {
        const Key k = order_key(sc[j]);
        if ((k & mask) == prefix) atomicAdd(&hist[int(k >> shift) & 255], 1);
      }
      __syncthreads();
      if (tid < 64) {
        // the highest bin at which the count of keys in this and all higher bins reaches `need`
        // (it exists: the candidates number at least `need`): lane i holds the bins 255 - 4 i
        // down to 252 - 4 i, and a scan over the lanes counts the keys above them
        const int b0 = 255 - 4 * tid;
        const int h0 = hist[b0], h1 = hist[b0 - 1], h2 = hist[b0 - 2], h3 = hist[b0 - 3];
        const int tot = h0 + h1 + h2 + h3;
        int inc = tot;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int v = __shfl_up(inc, o, 64);
          if (tid >= o) inc += v;
        }
        const int above = inc - tot;
        if (above < need && need <= inc) {
          int rem = need - above, bin = b0;
          if (h0 < rem) {
            rem -= h0;
            bin = b0 - 1;
            if (h1 < rem) {
              rem -= h1;
              bin = b0 - 2;
              if (h2 < rem) {
                rem -= h2;
                bin = b0 - 3;
              }
            }
          }
          sh_prefix = prefix | (Key(bin) << shift);
          sh_need = rem;
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      need = sh_need;
      mask |= Key(0xFF) << shift;
      __syncthreads();
    }
  }
  // prefix = threshold key; `need` of the keys equal to it are kept, lowest positions first.
  // Ordered compaction, four consecutive positions per thread and round: two block-wide scans
  // (ties, then kept entries) per 4096 positions.
  constexpr int PT = 4;
  int base_keep = 0, base_eq = 0;
  for (int j0 = 0; j0 < n; j0 += PT * blockDim.x) {
    const int jt = j0 + PT * tid;
    bool keep[PT], eq[PT];
    int neq = 0;
#pragma unroll
    for (int u = 0; u < PT; ++u) {
      const int j = jt + u;
      keep[u] = false;
      eq[u] = false;
      if (j < n) {
        if (j < lo || j >= hi) {
          keep[u] = true;
        } else if (nhh > 0) {
          const Key k = order_key(sc[j]);
          keep[u] = k > prefix;
          eq[u] = k == prefix;
        }
      }
      neq += eq[u] ? 1 : 0;
    }
    int ex_eq, tot_eq;
    block_scan_int(neq, ex_eq, tot_eq, wa);
    int nkeep = 0, seen_eq = base_eq + ex_eq;
#pragma unroll
    for (int u = 0; u < PT; ++u) {
      if (eq[u]) {
        if (seen_eq < need) keep[u] = true;
        ++seen_eq;
      }
      nkeep += keep[u] ? 1 : 0;
    }
    int ex_keep, tot_keep;
    block_scan_int(nkeep, ex_keep, tot_keep, wa);
    int kept = base_keep + ex_keep;  // kept entries before position jt + u
#pragma unroll
    for (int u = 0; u < PT; ++u) {
      const int j = jt + u;
      if (j < n) {
        if (keep[u])
          r[kept] = j;
        else
          e[j - kept] = j;
      }
      kept += keep[u] ? 1 : 0;
    }
    base_keep += tot_keep;
    base_eq += tot_eq;
  }
  if (tid == 0) {
    cnt[bh * 2] = base_keep;
    cnt[bh * 2 + 1] = n - base_keep;
  }
}

// ------------------------------------------------------------------------------------------
// Compaction: retained rows of K, V into the layer's cache region; scores widen to fp64.
// APPEND: the source is the position-ordered copy of a cache: fp64 scores (sc64) and token
// positions (apos) indexed like its rows.
template <typename T, bool APPEND>
__global__ __launch_bounds__(256) void gather_kernel(const T* __restrict__ K, View kv, const T* __restrict__ V, View vv,
                                                     const float* __restrict__ score, const double* __restrict__ sc64,
                                                     const int32_t* __restrict__ apos, const int32_t* __restrict__ ret,
                                                     const int32_t* __restrict__ cnt, const int32_t* __restrict__ meta,
                                                     T* __restrict__ cK, T* __restrict__ cV, double* __restrict__ cscore,
                                                     int32_t* __restrict__ cpos, int32_t* __restrict__ ccount,
                                                     int npad, int d, int64_t slots, const int32_t* __restrict__ row_meta,
                                                     int64_t row_slots) {
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int nret = cnt[bh * 2];
  constexpr int kVec = 16 / sizeof(T);
  const int tpr = d / kVec;                 // threads per row
  const int rows_per_blk = 256 / tpr;
  const int slot = blockIdx.x * rows_per_blk + threadIdx.x / tpr;
  if (blockIdx.x == 0 && threadIdx.x == 0) ccount[bh] = nret;
  if (slot >= nret) return;
  const int c = (threadIdx.x % tpr) * kVec;
  const int pos = ret[bh * npad + slot];
  const int64_t dst = (bh * slots + meta[bh * 4 + 0] + slot);
  // (the rows may live elsewhere than scores and positions: the bf16 staging rows of an fp8 cache)
  const int64_t dst_row = (bh * row_slots + row_meta[bh * 4 + 0] + slot);
  *reinterpret_cast<u32x4*>(cK + dst_row * d + c) =
      *reinterpret_cast<const u32x4*>(K + b * kv.sb + hk * kv.sh + int64_t(pos) * kv.sn + c);
  *reinterpret_cast<u32x4*>(cV + dst_row * d + c) =
      *reinterpret_cast<const u32x4*>(V + b * vv.sb + hk * vv.sh + int64_t(pos) * vv.sn + c);
  if (c == 0) {
    cscore[dst] = APPEND ? sc64[bh * npad + pos] : double(score[bh * npad + pos]);
    cpos[dst] = APPEND ? apos[bh * npad + pos] : pos;
  }
}

// ------------------------------------------------------------------------------------------
// Matching.

// 1/|k_j| in fp32 for every prompt key (used by the bf16 candidate filter only).
__global__ __launch_bounds__(256) void invnorm_bf16(const uint16_t* __restrict__ K, View kv, float* __restrict__ invn,
                                                    int n, int npad) {
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int row = blockIdx.x * 16 + threadIdx.x / 16, c = (threadIdx.x % 16) * 8;
  float s = 0.f;
  if (row < n) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(K + b * kv.sb + hk * kv.sh + int64_t(row) * kv.sn + c);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xFFFF0000u);
      s = fmaf(lo, lo, s);
      s = fmaf(hi, hi, s);
    }
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (row < n && (threadIdx.x % 16) == 0)
    invn[(int64_t(b) * Hkv + hk) * npad + row] = s > 0.f ? 1.0f / sqrtf(s) : 0.f;
}

// Candidate filter on the matrix cores.  A workgroup owns 128 evicted rows (4 wavefronts x 32,
// the stationary B operand) and streams the retained keys, read contiguously from the cache
// region they were compacted into, in double-buffered tiles of 64 through LDS (the A operand),
// so each lane owns one evicted row and sees 16 retained keys per MFMA tile.
//   COLLECT = false: per row, track the best and second-best fp32 cosine and the best's
//     retained rank.  A row whose two best values differ by less than kAmbiguous is flagged and
//     its acceptance threshold (best - kAmbiguous, in the un-normalised domain) is stored.
//   COLLECT = true: second sweep over the flagged rows only (compacted list): every retained
//     key whose fp32 cosine reaches the row's threshold is appended to the row's candidate
//     list (up to kMaxCand; more than that falls back to the exhaustive search).  The sweep
//     repeats the first one's arithmetic exactly, so the best value is found again.  Few rows are
//     flagged (a workgroup or two per head), so the retained keys are split over `ksplit`
//     workgroups per row block: the lists are appended with atomics and read order-free.
// kAmbiguous bounds twice the error of one filtered cosine: at most one rounding per accumulated
// product (128 * 2^-24 of |k_i||k_j|) plus the two fp32 inverse norms, 1.6e-5 in total, plus the
// four mantissa bits that carry the register number (2 * 16 * 2^-24 = 1.9e-6).
constexpr float kAmbiguous = 2.4e-5f;
constexpr int kMaxCand = 8;
constexpr int kLdM = 128 + 8;

template <bool COLLECT>
__global__ __launch_bounds__(256) void match_filter_bf16(const uint16_t* __restrict__ K, View kv,
                                                         const uint16_t* __restrict__ cK,
                                                         const int32_t* __restrict__ meta, int64_t slots,
                                                         const float* __restrict__ invn,
                                                         const int32_t* __restrict__ ret,
                                                         const int32_t* __restrict__ evi,
                                                         const int32_t* __restrict__ cnt, int32_t* __restrict__ cand,
                                                         float* __restrict__ thr, const int32_t* __restrict__ amb_list,
                                                         const int32_t* __restrict__ amb_cnt,
                                                         int32_t* __restrict__ ncand, int32_t* __restrict__ clist,
                                                         int npad, int ksplit) {
  constexpr int kTile = 64;     // retained keys per LDS tile
  constexpr int NCH = kTile * 16 / 256;  // 16-byte chunks of a tile per thread
  __shared__ __attribute__((aligned(16))) uint16_t Rs[2][kTile * kLdM];
  __shared__ __attribute__((aligned(16))) float rin[2][kTile];    // 1/|k| of the staged retained keys
  __shared__ __attribute__((aligned(16))) float rbias[2][kTile];  // 0, or -3e38 for padding rows (finite: the low
                                                                  // mantissa bits of a value get overwritten below)
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int nret = cnt[bh * 2], nevi = cnt[bh * 2 + 1];
  const int nrows = COLLECT ? amb_cnt[bh] : nevi;
  const int e0 = (int(blockIdx.x) / ksplit) * 128, part = int(blockIdx.x) % ksplit;
  if (e0 >= nrows) return;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, h = lane >> 5;
  const uint16_t* kb = K + b * kv.sb + hk * kv.sh;
  // the retained keys, in retained order, already sit contiguously in the layer's cache
  // region (compaction runs first; merging, which changes them, runs after the matching)
  const uint16_t* rk = cK + (bh * slots + meta[bh * 4 + 0]) * 128;
  const int32_t* rl = ret + bh * npad;
  const int32_t* el = evi + bh * npad;
  const float* inl = invn + bh * npad;
  const int row = e0 + w * 32 + m;
  const bool live = row < nrows;
  const int erank = COLLECT ? amb_list[bh * npad + min(row, nrows - 1)] : min(row, nrows - 1);
  const int epos = el[erank];
  bf16x8 be[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
    be[ks] = *reinterpret_cast<const bf16x8*>(kb + int64_t(epos) * kv.sn + ks * 16 + h * 8);
  float m1 = -INFINITY, m2 = -INFINITY;
  int isub = 0;  // first retained rank of the sub-tile the running best came from
  const float mythr = COLLECT ? thr[bh * npad + erank] : 0.f;
  // Tiles travel global -> registers -> LDS: the next tile is requested when work on a tile
  // starts and written to the other LDS buffer when it ends.
  u32x4 rg[NCH];
  float rv = 0.f;
  const int ntile = (nret + kTile - 1) / kTile;
  const int tper = (ntile + ksplit - 1) / ksplit;
  const int tbeg = part * tper, tend = min(ntile, tbeg + tper);  // this workgroup's tiles
  if (tbeg >= tend) return;
  auto issue = [&](int t) {
    const int r0 = t * kTile;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + 256 * i, rrow = c >> 4, col = (c & 15) * 8;
      rg[i] = *reinterpret_cast<const u32x4*>(rk + int64_t(min(r0 + rrow, nret - 1)) * 128 + col);
    }
    if (tid < kTile) rv = (r0 + tid < nret) ? inl[rl[r0 + tid]] : -1.f;  // -1 marks a padding row
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + 256 * i, rrow = c >> 4, col = (c & 15) * 8;
      *reinterpret_cast<u32x4*>(&Rs[buf][rrow * kLdM + col]) = rg[i];
    }
    if (tid < kTile) {
      rin[buf][tid] = rv < 0.f ? 0.f : rv;
      rbias[buf][tid] = rv < 0.f ? -3.0e38f : 0.f;
    }
  };
  auto one_tile = [&](int t) {
    const int buf = t & 1, r0 = t * kTile;
    if (t + 1 < tend) issue(t + 1);
    const int nsub = min(kTile / 32, (nret - r0 + 31) / 32);
    const bool padded = r0 + kTile > nret;  // only the last tile can hold rows past the end
    auto mma = [&](int st) -> f32x16 {
      bf16x8 a[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        a[ks] = *reinterpret_cast<const bf16x8*>(&Rs[buf][(st * 32 + m) * kLdM + ks * 16 + h * 8]);
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      f32x16 s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], be[0], zero, 0, 0, 0);
#pragma unroll
      for (int ks = 1; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], be[ks], s, 0, 0, 0);
      return s;
    };
    auto post = [&](const f32x16& s, int st) {
      // register r: retained row st*32 + (r/4)*8 + 4h + r%4 of this tile, evicted row = lane's;
      // the four rows of a register group are neighbours, so their 1/|k| come in one LDS read
      float tv[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int rb = st * 32 + g4 * 8 + h * 4;
        const f32x4 ri = *reinterpret_cast<const f32x4*>(&rin[buf][rb]);
#pragma unroll
        for (int i = 0; i < 4; ++i) tv[g4 * 4 + i] = s[g4 * 4 + i] * ri[i];
        if (padded) {  // block-uniform
          const f32x4 bi = *reinterpret_cast<const f32x4*>(&rbias[buf][rb]);
#pragma unroll
          for (int i = 0; i < 4; ++i) tv[g4 * 4 + i] += bi[i];
        }
      }
      if (COLLECT) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rr = st * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
          if (live && tv[r] >= mythr) {
            const int k = atomicAdd(&ncand[bh * npad + erank], 1);
            if (k < kMaxCand) clist[(bh * npad + erank) * kMaxCand + k] = r0 + rr;
          }
        }
      } else {
        // Running best and second best of the lane's row, two operations per value: the low four
        // mantissa bits of a value are replaced by its register number (a change of at most 16
        // units in the last place, which kAmbiguous covers), so that the maximum carries the
        // position inside the sub-tile with it; which sub-tile it came from is noted once per
        // sub-tile.  Values that are equal up to those bits end up flagged as ambiguous and are
        // decided by the exact refinement.
        const float before = m1;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float key = __uint_as_float((__float_as_uint(tv[r]) & ~15u) | uint32_t(r));
          m2 = __builtin_amdgcn_fmed3f(m1, m2, key);
          // (the maximum as the instruction itself: fmaxf would first re-canonicalise a value
          // that was put together from bits)
          asm("v_max_f32 %0, %1, %2" : "=v"(m1) : "v"(m1), "v"(key));
        }
        isub = (m1 != before) ? (r0 + st * 32) : isub;
      }
    };
    // (two sub-tiles as two independent accumulation chains need 160 registers and cost a
    // wavefront per SIMD: slower)
    for (int st = 0; st < nsub; ++st) post(mma(st), st);
    if (t + 1 < tend) stage(buf ^ 1);
    __syncthreads();
  };
  issue(tbeg);
  stage(tbeg & 1);
  __syncthreads();
#pragma unroll 1
  for (int t = tbeg; t < tend; ++t) one_tile(t);
  if (COLLECT) return;
  // the best's retained rank: its sub-tile, and the register number carried in its low bits
  const int rbest = int(__float_as_uint(m1) & 15u);
  const int i1 = isub + (rbest >> 2) * 8 + h * 4 + (rbest & 3);
  // combine the two lane halves that share an evicted row
  const float om1 = __shfl_xor(m1, 32, 64), om2 = __shfl_xor(m2, 32, 64);
  const int oi1 = __shfl_xor(i1, 32, 64);
  const float best = fmaxf(m1, om1);
  const float second = fmaxf(fminf(m1, om1), fmaxf(m2, om2));
  const int bi = (om1 > m1) ? oi1 : i1;
  if (h == 0 && live) {
    const float ie = inl[epos];
    const float margin = ie > 0.f ? kAmbiguous / ie : INFINITY;  // threshold in the un-normalised domain
    const bool amb = !(best - second >= margin);                // also true for NaN / equal / zero norm
    cand[bh * npad + erank] = bi | (amb ? int(0x80000000u) : 0);
    thr[bh * npad + erank] = best - margin;
  }
}

// Ordered list of the flagged rows of one (sequence, KV head), and cleared candidate counters.
__global__ __launch_bounds__(1024) void amb_compact_kernel(const int32_t* __restrict__ cand, const int32_t* __restrict__ cnt,
                                                           int32_t* __restrict__ amb_list, int32_t* __restrict__ amb_cnt,
                                                           int32_t* __restrict__ ncand, int npad) {
  __shared__ int wa[16], wb[16];
  const int hk = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int nevi = cnt[bh * 2 + 1];
  int base = 0;
  for (int i0 = 0; i0 < nevi; i0 += blockDim.x) {
    const int i = i0 + threadIdx.x;
    const bool amb = i < nevi && cand[bh * npad + i] < 0;
    if (i < nevi) ncand[bh * npad + i] = 0;
    int ex, exd, tot, totd;
    block_scan2(amb, false, ex, exd, tot, totd, wa, wb);
    if (amb) amb_list[bh * npad + base + ex] = i;
    base += tot;
  }
  if (threadIdx.x == 0) amb_cnt[bh] = base;
}

// Exact similarity in fp64, operation order of Eq. 9 as written: dot / (|k_i| * |k_j|), 0 when
// a norm is 0.  A group of 16 lanes (one 16-byte slice of the key each) serves one evicted row:
// unambiguous rows evaluate their single candidate, ambiguous rows their short candidate list;
// rows without a usable list (and every row when no filter ran) are then searched exhaustively,
// one at a time, with the wavefront's lanes striding over the retained keys, first maximum in
// ascending retained order.  Products of bf16 values are exact in fp64 and their sums stay
// exact at these magnitudes, so the result does not depend on the summation tree.
template <typename T>
__device__ __forceinline__ void load8(const T* p, double* out);
template <>
__device__ __forceinline__ void load8<uint16_t>(const uint16_t* p, double* out) {
  const u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = double(__uint_as_float(v[i] << 16));
    out[2 * i + 1] = double(__uint_as_float(v[i] & 0xFFFF0000u));
  }
}
template <>
__device__ __forceinline__ void load8<float>(const float* p, double* out) {  // 16 bytes: 4 elements
  const float4 a = reinterpret_cast<const float4*>(p)[0];
  out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
}

// Lanes of one row group (TPR lanes: 16, or 32 for 512-byte rows) add their partial sums.
template <int TPR>
__device__ __forceinline__ double group_sum(double v) {
  v = row16_sum(v);
  if constexpr (TPR == 32) v += __shfl_xor(v, 16, 64);
  return v;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void match_refine(const T* __restrict__ K, View kv, const int32_t* __restrict__ ret,
                                                    const int32_t* __restrict__ evi, const int32_t* __restrict__ cnt,
                                                    const int32_t* __restrict__ cand, const int32_t* __restrict__ ncand,
                                                    const int32_t* __restrict__ clist, double* __restrict__ ustar,
                                                    int32_t* __restrict__ tgt, int npad, int use_filter) {
  constexpr int kVec = 16 / sizeof(T);  // elements per 16-byte load
  constexpr int TPR = D / kVec;         // lanes that share one evicted row
  constexpr int RW = 64 / TPR;          // evicted rows per wavefront
  __shared__ double ke[4][D];
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int nret = cnt[bh * 2], nevi = cnt[bh * 2 + 1];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, grp = lane / TPR, tc = lane % TPR;
  if (int(blockIdx.x) * 4 * RW >= nevi) return;  // block-uniform
  const int erank_raw = (blockIdx.x * 4 + w) * RW + grp;
  const bool valid = erank_raw < nevi;
  const int erank = valid ? erank_raw : nevi - 1;
  const T* kb = K + b * kv.sb + hk * kv.sh;
  const int32_t* rl = ret + bh * npad;
  const int epos = evi[bh * npad + erank];
  // this lane's slice of the evicted key
  double x[kVec];
  load8<T>(kb + int64_t(epos) * kv.sn + tc * kVec, x);
  double ne = 0.0;
#pragma unroll
  for (int e = 0; e < kVec; ++e) ne = fma(x[e], x[e], ne);
  const double sne = sqrt(group_sum<TPR>(ne));
  // candidates: one (unambiguous), a short list (ambiguous), or every retained key (ncd < 0)
  int ncd = -1, single = -1;
  const int32_t* cl = clist + (bh * npad + erank) * kMaxCand;
  if (use_filter) {
    const int cnd = cand[bh * npad + erank];
    if (cnd >= 0) {
      single = cnd;
      ncd = 1;
    } else {
      ncd = ncand[bh * npad + erank];
      if (ncd > kMaxCand || ncd == 0) ncd = -1;  // overflow (or zero-norm row): exhaustive search
    }
  }
  double best = -2.0;
  int bj = 0x7FFFFFFF;
  // ---- listed candidates: the row group evaluates them one after the other
  int nloop = max(ncd, 0);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) nloop = max(nloop, __shfl_xor(nloop, o, 64));
  for (int q = 0; q < nloop; ++q) {
    const bool on = q < ncd;
    const int j = on ? (single >= 0 ? single : cl[q]) : 0;
    double y[kVec];
    load8<T>(kb + int64_t(rl[j]) * kv.sn + tc * kVec, y);
    double dot = 0.0, nr = 0.0;
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
      dot = fma(x[e], y[e], dot);
      nr = fma(y[e], y[e], nr);
    }
    dot = group_sum<TPR>(dot);
    nr = group_sum<TPR>(nr);
    const double den = sne * sqrt(nr);
    const double u = den > 0.0 ? dot / den : 0.0;
    if (on && (u > best || (u == best && j < bj))) {
      best = u;
      bj = j;
    }
  }
  // ---- exhaustive search, one row at a time, the wavefront's lanes striding over the retained keys
  unsigned long long todo = __ballot(valid && ncd < 0 && tc == 0);
  while (todo) {
    const int src = __ffsll((long long)todo) - 1;  // first lane of the row group to serve
    todo &= todo - 1;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane / TPR == src / TPR) {
#pragma unroll
      for (int e = 0; e < kVec; ++e) ke[w][tc * kVec + e] = x[e];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const double sne_r = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(sne), src),
                                          __builtin_amdgcn_readlane(__double2loint(sne), src));
    double fb = -2.0;
    int fj = 0x7FFFFFFF;
    for (int j = lane; j < nret; j += 64) {
      const T* rr = kb + int64_t(rl[j]) * kv.sn;
      double dot = 0.0, nr = 0.0;
      for (int c = 0; c < D; c += kVec) {
        double y[kVec];
        load8<T>(rr + c, y);
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
          dot = fma(ke[w][c + i], y[i], dot);
          nr = fma(y[i], y[i], nr);
        }
      }
      const double den = sne_r * sqrt(nr);
      const double u = den > 0.0 ? dot / den : 0.0;
      if (u > fb) {  // j ascends within a lane: strict > keeps the first maximum
        fb = u;
        fj = j;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const double ob = __shfl_xor(fb, o, 64);
      const int oj = __shfl_xor(fj, o, 64);
      if (ob > fb || (ob == fb && oj < fj)) {
        fb = ob;
        fj = oj;
      }
    }
    if (lane == src) {
      best = fb;
      bj = fj;
    }
  }
  if (tc == 0 && valid) {
    ustar[bh * npad + erank] = best;
    tgt[bh * npad + erank] = bj;
  }
}

// ------------------------------------------------------------------------------------------
// Threshold (Eq. 10, t = 0) and grouping of the passing tokens by target.  One workgroup per
// (sequence, KV head).  Group members are stored unordered; merge_kernel visits them in
// ascending evicted order.
__global__ __launch_bounds__(1024) void threshold_group_kernel(const double* __restrict__ ustar,
                                                               const int32_t* __restrict__ tgt,
                                                               const int32_t* __restrict__ cnt, uint8_t* __restrict__ pass,
                                                               int32_t* __restrict__ gcnt, int32_t* __restrict__ goff,
                                                               int32_t* __restrict__ gcur, int32_t* __restrict__ gsrc,
                                                               double* __restrict__ tau_out, int npad, double tau_force,
                                                               int ema, double beta) {
  __shared__ double red[16];
  __shared__ int wa[16], wb[16];
  const int hk = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int nret = cnt[bh * 2], nevi = cnt[bh * 2 + 1];
  const int tid = threadIdx.x;
  const double* us = ustar + bh * npad;
  const int32_t* tg = tgt + bh * npad;
  uint8_t* ps = pass + bh * npad;
  int32_t* gc = gcnt + bh * (npad + 1);
  int32_t* go = goff + bh * (npad + 1);
  int32_t* gu = gcur + bh * (npad + 1);
  int32_t* gs = gsrc + bh * npad;
  if (nevi == 0) {
    // no sources anywhere: merge_kernel reads the offsets of every slot, so they must say so
    for (int j = tid; j <= nret; j += blockDim.x) {
      gc[j] = 0;
      go[j] = 0;
    }
    return;  // tau keeps its value (unset, NaN, after prompt encoding)
  }
  double part = 0.0;
  for (int i = tid; i < nevi; i += blockDim.x) part += us[i];
  double tau = block_sum(part, red) / double(nevi);
  if (ema) {  // a step that evicts several tokens at once: Eq. 10 on their mean best similarity
    const double prev = tau_out[bh];
    if (!isnan(prev)) tau = __dadd_rn(__dmul_rn(beta, tau), __dmul_rn(1.0 - beta, prev));
    __syncthreads();  // every thread has read the previous value
  }
  if (tid == 0 && !(ema && !isnan(tau_force))) tau_out[bh] = tau;  // (a forced threshold leaves the EMA state alone)
  const double thr = isnan(tau_force) ? tau : tau_force;
  for (int j = tid; j <= nret; j += blockDim.x) {
    gc[j] = 0;
    gu[j] = 0;
  }
  __syncthreads();
  for (int i = tid; i < nevi; i += blockDim.x) {
    const bool ok = us[i] >= thr;
    ps[i] = ok ? 1 : 0;
    if (ok) atomicAdd(&gc[tg[i]], 1);
  }
  __syncthreads();
  // exclusive prefix of gc over [0, nret]
  int base = 0;
  for (int j0 = 0; j0 <= nret; j0 += blockDim.x) {
    const int j = j0 + tid;
    const int v = (j < nret) ? gc[j] : 0;
    // inclusive scan within the wavefront
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o, 64);
      if ((tid & 63) >= o) inc += t;
    }
    __syncthreads();
    if ((tid & 63) == 63) wa[tid >> 6] = inc;
    __syncthreads();
    int woff = 0, tot = 0;
    for (int i = 0; i < int(blockDim.x >> 6); ++i) {
      if (i < (tid >> 6)) woff += wa[i];
      tot += wa[i];
    }
    if (j <= nret) go[j] = base + woff + inc - v;
    base += tot;
  }
  __syncthreads();
  for (int i = tid; i < nevi; i += blockDim.x) {
    if (ps[i]) {
      const int t = tg[i];
      const int k = atomicAdd(&gu[t], 1);
      gs[go[t] + k] = i;
    }
  }
  (void)wb;
}

// PER consecutive elements of a row as one load / one store.
template <typename T, int PER>
__device__ __forceinline__ void load_elems(const T* p, double* out) {
  static_assert(PER * sizeof(T) == 4 || PER * sizeof(T) == 8, "one 4- or 8-byte access");
  T tmp[PER];
  if constexpr (PER * sizeof(T) == 4)
    *reinterpret_cast<uint32_t*>(tmp) = *reinterpret_cast<const uint32_t*>(p);
  else
    *reinterpret_cast<uint64_t*>(tmp) = *reinterpret_cast<const uint64_t*>(p);
#pragma unroll
  for (int i = 0; i < PER; ++i) out[i] = Elem<T>::to_f64(tmp[i]);
}
template <typename T, int PER>
__device__ __forceinline__ void store_elems(T* p, const double* v, double z) {
  T tmp[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) tmp[i] = Elem<T>::from_f64(v[i] / z);
  if constexpr (PER * sizeof(T) == 4)
    *reinterpret_cast<uint32_t*>(p) = *reinterpret_cast<const uint32_t*>(tmp);
  else
    *reinterpret_cast<uint64_t*>(p) = *reinterpret_cast<const uint64_t*>(tmp);
}

// Merge (Eq. 11-12).  One wavefront per retained slot that has sources; lane i owns elements
// PER*i .. PER*i + PER - 1 of the row.  fp64, operation order of the definition: acc = e * k_c;
// for each source in ascending evicted order: w = exp(u), Z += w, acc += w * k_e; result
// acc / Z rounded once to the cache dtype.  Products and sums are kept unfused so the sequence
// is the one written in the formula.
// The source list of a slot is unordered, and its length varies widely (the keys nearest to a
// cluster centre collect hundreds of sources; a small budget lengthens every list).
//   up to 64 sources      one source per lane: the lanes rank their sources (count the smaller
//                         ones), fetch weight and position in parallel;
//   up to kMergeCap       the same ranking through LDS, weight and position stored at the rank;
//   beyond                the next source is extracted by a scan per step.
// The rows are then read kMergeBatch sources at a time in rank order.
constexpr int kMergeCap = 512;
constexpr int kMergeBatch = 8;
template <typename T, int D, bool AVERAGE>
__global__ __launch_bounds__(256) void merge_kernel(const T* __restrict__ K, View kv, const T* __restrict__ V, View vv,
                                                    const int32_t* __restrict__ evi, const int32_t* __restrict__ cnt,
                                                    const double* __restrict__ ustar, const int32_t* __restrict__ goff,
                                                    const int32_t* __restrict__ gsrc, const int32_t* __restrict__ meta,
                                                    T* __restrict__ cK, T* __restrict__ cV, int npad, int64_t slots) {
  __shared__ int s_src[4][kMergeCap];
  __shared__ int s_pos[4][kMergeCap];
  __shared__ double s_w[4][kMergeCap];
  const int hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int slot = blockIdx.x * 4 + w;  // < npad: both offsets below are inside the array
  const int nret = cnt[bh * 2];
  const int32_t* go = goff + bh * (npad + 1);  // exclusive prefix of the list sizes over [0, nret]
  const int off0 = go[slot], off1 = go[slot + 1];
  if (slot >= nret) return;
  const int ns = off1 - off0;
  if (ns == 0) return;
  const int32_t* src = gsrc + bh * npad + off0;
  const int32_t* el = evi + bh * npad;
  const double* us = ustar + bh * npad;
  const T* kb = K + b * kv.sb + hk * kv.sh;
  const T* vb = V + b * vv.sb + hk * vv.sh;
  constexpr int PER = D / 64;
  const int64_t dst = (bh * slots + meta[bh * 4 + 0] + slot) * D + lane * PER;
  // exp(1), the retained token's self-similarity weight; average merging weighs every member 1
  const double e1 = AVERAGE ? 1.0 : 2.718281828459045;
  auto weight = [&](double u) __attribute__((always_inline)) { return AVERAGE ? 1.0 : exp(u); };
  double ak[PER], av[PER];
  load_elems<T, PER>(cK + dst, ak);
  load_elems<T, PER>(cV + dst, av);
#pragma unroll
  for (int p = 0; p < PER; ++p) {
    ak[p] = __dmul_rn(e1, ak[p]);
    av[p] = __dmul_rn(e1, av[p]);
  }
  double z = e1;
  auto add_source = [&](double wgt, const double* xk, const double* xv) {
    z = __dadd_rn(z, wgt);
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      ak[p] = __dadd_rn(ak[p], __dmul_rn(wgt, xk[p]));
      av[p] = __dadd_rn(av[p], __dmul_rn(wgt, xv[p]));
    }
  };
  // rows of kMergeBatch sources in flight; weight and position of source s come from `at`
  auto stream = [&](auto at) {
    for (int s0 = 0; s0 < ns; s0 += kMergeBatch) {
      double wq[kMergeBatch], xk[kMergeBatch][PER], xv[kMergeBatch][PER];
#pragma unroll
      for (int u = 0; u < kMergeBatch; ++u) {
        int pos;
        at(min(s0 + u, ns - 1), wq[u], pos);
        load_elems<T, PER>(kb + int64_t(pos) * kv.sn + lane * PER, xk[u]);
        load_elems<T, PER>(vb + int64_t(pos) * vv.sn + lane * PER, xv[u]);
      }
#pragma unroll
      for (int u = 0; u < kMergeBatch; ++u)
        if (s0 + u < ns) add_source(wq[u], xk[u], xv[u]);
    }
  };
  if (ns <= 64) {
    const bool have = lane < ns;
    const int mine = have ? src[lane] : 0x7FFFFFFF;
    const double wmine = have ? weight(us[mine]) : 0.0;
    const int pmine = have ? el[mine] : 0;
    int rank = 0;  // sources are distinct: the ranks are a permutation of 0 .. ns-1
    for (int i = 0; i < ns; ++i) rank += __builtin_amdgcn_readlane(mine, i) < mine ? 1 : 0;
    stream([&](int s, double& wgt, int& pos) {
      const int owner = __ffsll((long long)__ballot(have && rank == s)) - 1;
      wgt = lane_f64(wmine, owner);
      pos = __builtin_amdgcn_readlane(pmine, owner);
    });
  } else if (ns <= kMergeCap) {
    for (int t = lane; t < ns; t += 64) s_src[w][t] = src[t];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int t = lane; t < ns; t += 64) {
      const int mine = s_src[w][t];
      const double wm = weight(us[mine]);
      const int pm = el[mine];
      int rank = 0;
      for (int i = 0; i < ns; ++i) rank += s_src[w][i] < mine ? 1 : 0;
      s_w[w][rank] = wm;
      s_pos[w][rank] = pm;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    stream([&](int s, double& wgt, int& pos) {
      wgt = s_w[w][s];
      pos = s_pos[w][s];
    });
  } else {
    int prev = -1;
    for (int s = 0; s < ns; ++s) {
      int cur = 0x7FFFFFFF;
      for (int t = lane; t < ns; t += 64) {
        const int r = src[t];
        if (r > prev && r < cur) cur = r;
      }
      cur = wave_min(cur);
      const double wgt = weight(us[cur]);
      const int64_t pos = el[cur];
      double xk[PER], xv[PER];
      load_elems<T, PER>(kb + pos * kv.sn + lane * PER, xk);
      load_elems<T, PER>(vb + pos * vv.sn + lane * PER, xv);
      add_source(wgt, xk, xv);
      prev = cur;
    }
  }
  store_elems<T, PER>(cK + dst, ak, z);
  store_elems<T, PER>(cV + dst, av, z);
}

}  // namespace

// ---------------------------------------------------------------------------------------------

hipError_t launch_select(d2o_ctx* c, int layer, int n, hipStream_t s, bool append) {
  const d2o_config& cf = c->cfg;
  const float* score = c->score_pre + size_t(layer) * cf.batch * cf.n_kv_heads * c->npad;
  const int32_t* meta = c->meta + size_t(layer) * cf.batch * cf.n_kv_heads * 4;
  KernelTimer kt(c, D2O_K_SELECT, s);
  if (append)
    select_kernel<double><<<dim3(cf.n_kv_heads, cf.batch), 1024, 0, s>>>(c->app_score, meta, c->sel_ret, c->sel_evi,
                                                                         c->sel_cnt, n, c->app_n, c->npad, cf.n_sink);
  else
    select_kernel<float><<<dim3(cf.n_kv_heads, cf.batch), 1024, 0, s>>>(score, meta, c->sel_ret, c->sel_evi, c->sel_cnt,
                                                                        n, nullptr, c->npad, cf.n_sink);
  return hipGetLastError();
}

template <typename T>
static void run_gather(d2o_ctx* c, int layer, View K, View V, int max_budget, bool append, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const float* score = c->score_pre + size_t(layer) * cf.batch * cf.n_kv_heads * c->npad;
  const int32_t* meta = c->meta + size_t(layer) * cf.batch * cf.n_kv_heads * 4;
  int32_t* ccount = c->ccount + size_t(layer) * cf.batch * cf.n_kv_heads;
  const int rows = 256 / (cf.head_dim * int(sizeof(T)) / 16);
  const dim3 grid((max_budget + rows - 1) / rows, cf.n_kv_heads, cf.batch);
  if (append)
    gather_kernel<T, true><<<grid, 256, 0, s>>>((const T*)K.ptr, K, (const T*)V.ptr, V, score, c->app_score, c->app_pos,
                                                c->sel_ret, c->sel_cnt, meta, (T*)prompt_rows_K(c), (T*)prompt_rows_V(c), c->cscore,
                                                c->cpos, ccount, c->npad, cf.head_dim, cf.slots_per_seq,
                                                prompt_rows_meta(c, layer), prompt_rows_stride(c));
  else
    gather_kernel<T, false><<<grid, 256, 0, s>>>((const T*)K.ptr, K, (const T*)V.ptr, V, score, nullptr, nullptr,
                                                 c->sel_ret, c->sel_cnt, meta, (T*)prompt_rows_K(c), (T*)prompt_rows_V(c), c->cscore,
                                                 c->cpos, ccount, c->npad, cf.head_dim, cf.slots_per_seq,
                                                 prompt_rows_meta(c, layer), prompt_rows_stride(c));
}

hipError_t launch_gather(d2o_ctx* c, int layer, View K, View V, int n, hipStream_t s, bool append) {
  const d2o_config& cf = c->cfg;
  int max_budget = 0;
  for (const auto& mt : c->layers[layer].meta) max_budget = std::max(max_budget, std::min(mt.budget, n));
  if (cf.dtype == D2O_BF16)
    run_gather<uint16_t>(c, layer, K, V, max_budget, append, s);
  else
    run_gather<float>(c, layer, K, V, max_budget, append, s);
  return hipGetLastError();
}

static int max_evicted(const d2o_ctx* c, int layer, int n) {
  int m = 0;
  for (const auto& mt : c->layers[layer].meta) m = std::max(m, n - std::min(mt.budget, n));
  return m;
}

hipError_t launch_match(d2o_ctx* c, int layer, View K, int n, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int me = max_evicted(c, layer, n);
  if (me == 0) return hipSuccess;
  const int refine_rows = 4 * 64 / ((cf.head_dim * c->esize) / 16);  // evicted rows per workgroup of match_refine
  const dim3 gr((me + refine_rows - 1) / refine_rows, cf.n_kv_heads, cf.batch);
  if (cf.dtype == D2O_BF16) {
    const dim3 gf((me + 127) / 128, cf.n_kv_heads, cf.batch);
    invnorm_bf16<<<dim3((n + 15) / 16, cf.n_kv_heads, cf.batch), 256, 0, s>>>((const uint16_t*)K.ptr, K, c->invnorm, n,
                                                                             c->npad);
    {
      KernelTimer kt(c, D2O_K_MATCH_FILTER, s);
      match_filter_bf16<false><<<gf, 256, 0, s>>>((const uint16_t*)K.ptr, K, (const uint16_t*)prompt_rows_K(c),
                                                  prompt_rows_meta(c, layer), prompt_rows_stride(c),
                                                  c->invnorm, c->sel_ret, c->sel_evi,
                                                  c->sel_cnt, c->m_cand, c->m_thr, c->amb_list, c->amb_cnt,
                                                  c->m_ncand, c->m_clist, c->npad, 1);
      amb_compact_kernel<<<dim3(cf.n_kv_heads, cf.batch), 1024, 0, s>>>(c->m_cand, c->sel_cnt, c->amb_list,
                                                                        c->amb_cnt, c->m_ncand, c->npad);
      constexpr int kSplit = 8;
      match_filter_bf16<true><<<dim3(gf.x * kSplit, gf.y, gf.z), 256, 0, s>>>((const uint16_t*)K.ptr, K, (const uint16_t*)prompt_rows_K(c),
                                                 prompt_rows_meta(c, layer), prompt_rows_stride(c),
                                                 c->invnorm, c->sel_ret, c->sel_evi,
                                                 c->sel_cnt, c->m_cand, c->m_thr, c->amb_list, c->amb_cnt,
                                                 c->m_ncand, c->m_clist, c->npad, kSplit);
    }
    KernelTimer kt(c, D2O_K_MATCH_REFINE, s);
    match_refine<uint16_t, 128><<<gr, 256, 0, s>>>((const uint16_t*)K.ptr, K, c->sel_ret, c->sel_evi, c->sel_cnt,
                                                   c->m_cand, c->m_ncand, c->m_clist, c->m_ustar, c->m_tgt, c->npad, 1);
  } else if (cf.head_dim == 64) {
    KernelTimer kt(c, D2O_K_MATCH_REFINE, s);
    match_refine<float, 64><<<gr, 256, 0, s>>>((const float*)K.ptr, K, c->sel_ret, c->sel_evi, c->sel_cnt, c->m_cand,
                                               c->m_ncand, c->m_clist, c->m_ustar, c->m_tgt, c->npad, 0);
  } else {
    KernelTimer kt(c, D2O_K_MATCH_REFINE, s);
    match_refine<float, 128><<<gr, 256, 0, s>>>((const float*)K.ptr, K, c->sel_ret, c->sel_evi, c->sel_cnt, c->m_cand,
                                                c->m_ncand, c->m_clist, c->m_ustar, c->m_tgt, c->npad, 0);
  }
  return hipGetLastError();
}

hipError_t launch_threshold_group(d2o_ctx* c, int layer, int n, hipStream_t s, bool append) {
  const d2o_config& cf = c->cfg;
  double* tau = c->ctau + size_t(layer) * cf.batch * cf.n_kv_heads;
  threshold_group_kernel<<<dim3(cf.n_kv_heads, cf.batch), 1024, 0, s>>>(c->m_ustar, c->m_tgt, c->sel_cnt, c->m_pass,
                                                                        c->g_cnt, c->g_off, c->g_cur, c->g_src, tau,
                                                                        c->npad, cf.tau_force, append ? 1 : 0, cf.beta);
  return hipGetLastError();
}

template <typename T, int D>
static void run_merge(d2o_ctx* c, const int32_t* meta, View K, View V, int max_budget, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const dim3 grid((max_budget + 3) / 4, cf.n_kv_heads, cf.batch);
  if (cf.merge_average)
    merge_kernel<T, D, true><<<grid, 256, 0, s>>>((const T*)K.ptr, K, (const T*)V.ptr, V, c->sel_evi, c->sel_cnt,
                                                  c->m_ustar, c->g_off, c->g_src, meta, (T*)prompt_rows_K(c), (T*)prompt_rows_V(c),
                                                  c->npad, prompt_rows_stride(c));
  else
    merge_kernel<T, D, false><<<grid, 256, 0, s>>>((const T*)K.ptr, K, (const T*)V.ptr, V, c->sel_evi, c->sel_cnt,
                                                   c->m_ustar, c->g_off, c->g_src, meta, (T*)prompt_rows_K(c), (T*)prompt_rows_V(c),
                                                   c->npad, prompt_rows_stride(c));
}

hipError_t launch_merge(d2o_ctx* c, int layer, View K, View V, int n, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  if (max_evicted(c, layer, n) == 0) return hipSuccess;
  int max_budget = 0;
  for (const auto& mt : c->layers[layer].meta) max_budget = std::max(max_budget, std::min(mt.budget, n));
  const int32_t* meta = prompt_rows_meta(c, layer);  // the merge kernel touches rows only
  KernelTimer kt(c, D2O_K_MERGE, s);
  if (cf.dtype == D2O_BF16)
    run_merge<uint16_t, 128>(c, meta, K, V, max_budget, s);
  else if (cf.head_dim == 64)
    run_merge<float, 64>(c, meta, K, V, max_budget, s);
  else
    run_merge<float, 128>(c, meta, K, V, max_budget, s);
  return hipGetLastError();
}

}  // namespace d2o
