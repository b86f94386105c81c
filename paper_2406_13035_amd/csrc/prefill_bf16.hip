// Prompt-phase attention for bf16 tensors on the CDNA4 matrix cores (head_dim 128).
//
// Pass 1, attn_fwd_bf16 (Sec. 4.1 Eq. 4; Sec. 3 Eq. 3): row-stationary flash attention.  A
//   workgroup owns 256 query rows (8 wavefronts x 32), streams 64-key tiles of K and of the
//   pre-transposed V through LDS and keeps S^T = K Q^T in the MFMA accumulator layout, where
//   one lane owns one query column: row maxima and sums are then in-register reductions.
//   Emits O and the row log-sum-exp (base 2, of the scaled logits).
//   The P V product runs in fp16, not bf16: probabilities rounded to bf16 (8 significant bits)
//   alone cost up to 2^-8 relative on O, fp16 (11 bits) keeps it below 2^-11.  V is converted
//   once, in the transposing pre-pass, with a per-head power-of-two scale that maps max|v| to
//   2^13 (exact for bf16 inputs inside fp16's exponent range), and P carries a factor 2^12 so
//   that small probabilities stay in fp16's normal range; both factors cancel in O.
// Pass 2, colsum_bf16 (column sums of the attention matrix, Sec. 4.1; Eq. 6 prompt case):
//   key-stationary.  A workgroup owns 256 keys, streams query tiles, recomputes S^T with the
//   keys as the stationary MFMA operand, and accumulates P = exp2(S - lse) per key in
//   registers; the column sums come out without atomics, the G query heads of a KV group are
//   added in ascending order, and per-query-head partial sums of the column sums and their
//   squares feed the variance of Eq. 4.
// The column sums need every row's final normaliser, so they cannot come out of the single
// online-softmax pass; the second QK^T product is implementation overhead.
//
// v_mfma_f32_32x32x16_bf16 operand layout (lane l, m = l % 32, h = l / 32):
//   A[m][8h .. 8h+7], B[8h .. 8h+7][m], D[(r/4)*8 + 4h + r%4][m] for r = 0..15.
#include "d2o_internal.h"
#include <algorithm>
#include <type_traits>

#include "device_utils.h"

namespace d2o {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kD = 128;
constexpr int kLdK = kD + 8;   // LDS row pitch (elements) of [token][d] tiles
constexpr int kLdV = 64 + 8;   // LDS row pitch of the [d][key] tile
constexpr float kPShift = 12.f;  // probabilities are formed as 2^12 * p before the fp16 rounding
constexpr float kLazy = 3.f;     // log2 of the growth the exponent reference tolerates before it moves

__global__ void zero_u32(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// max |v| per (sequence, KV head), as the bit pattern of the non-negative float.
__global__ __launch_bounds__(256) void vabsmax_kernel(const uint16_t* __restrict__ V, View vv, uint32_t* __restrict__ vmax,
                                                      int n) {
  __shared__ uint32_t red[4];
  const int h = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const uint16_t* src = V + b * vv.sb + h * vv.sh;
  uint32_t m = 0;
  for (int c = blockIdx.x * 256 + threadIdx.x; c < n * 16; c += gridDim.x * 256) {
    const int row = c >> 4, col = (c & 15) * 8;
    const u32x4 v = *reinterpret_cast<const u32x4*>(src + int64_t(row) * vv.sn + col);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      m = max(m, (v[i] << 16) & 0x7FFFFFFFu);
      m = max(m, v[i] & 0x7FFF0000u);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, o, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) atomicMax(&vmax[b * Hkv + h], max(max(red[0], red[1]), max(red[2], red[3])));
}

// Power-of-two factor that maps max|v| into [2^13, 2^14) (1 when the head is all zero).
__device__ __forceinline__ float v_scale_from_max(uint32_t maxbits) {
  const int e = int((maxbits >> 23) & 0xFF);  // biased exponent of max |v|
  if (e == 0 || e == 255) return 1.0f;
  const int k = min(max(e - 127 - 13, -100), 100);
  return __uint_as_float(uint32_t(127 - k) << 23);  // 2^-k
}

// V [b][h][n][d] (bf16) -> VT [b][h][npad/64][d][64] (fp16, scaled), zero for keys >= n: the
// transposed values of every 64-key tile are contiguous (a [d][npad] layout would put a tile's
// rows a power-of-two stride apart, all on one memory channel).
__global__ __launch_bounds__(256) void transpose_v(const uint16_t* __restrict__ V, View vv, uint16_t* __restrict__ VT,
                                                   const uint32_t* __restrict__ vmax, float* __restrict__ unscale,
                                                   int n, int npad) {
  __shared__ uint16_t t[64][kD + 2];
  const int k0 = blockIdx.x * 64, h = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const float mul = v_scale_from_max(vmax[b * Hkv + h]);
  if (blockIdx.x == 0 && threadIdx.x == 0) unscale[b * Hkv + h] = 1.0f / mul;
  const uint16_t* src = V + b * vv.sb + h * vv.sh;
  for (int c = threadIdx.x; c < 64 * 16; c += 256) {
    const int row = c >> 4, col = (c & 15) * 8;
    u32x4 v = {0, 0, 0, 0};
    if (k0 + row < n) v = *reinterpret_cast<const u32x4*>(src + int64_t(k0 + row) * vv.sn + col);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const _Float16 lo = (_Float16)(__uint_as_float(v[i] << 16) * mul);
      const _Float16 hi = (_Float16)(__uint_as_float(v[i] & 0xFFFF0000u) * mul);
      t[row][col + 2 * i] = __builtin_bit_cast(uint16_t, lo);
      t[row][col + 2 * i + 1] = __builtin_bit_cast(uint16_t, hi);
    }
  }
  __syncthreads();
  uint16_t* dst = VT + (int64_t(b) * Hkv + h) * kD * npad;
  for (int c = threadIdx.x; c < kD * 8; c += 256) {
    const int dd = c >> 3, kc = (c & 7) * 8;
    uint16_t o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = t[kc + i][dd];
    u32x4 v;
    v[0] = o[0] | (uint32_t(o[1]) << 16); v[1] = o[2] | (uint32_t(o[3]) << 16);
    v[2] = o[4] | (uint32_t(o[5]) << 16); v[3] = o[6] | (uint32_t(o[7]) << 16);
    *reinterpret_cast<u32x4*>(dst + (int64_t(blockIdx.x) * kD + dd) * 64 + kc) = v;
  }
}

// MFMA row m -> key offset inside a 32-key sub-tile, chosen so that accumulator registers
// 8*kb .. 8*kb+7 of lane-half h hold the 8 consecutive keys 16*kb + 8*h .. +7: exactly the
// B-operand slice the P V product needs, with no cross-lane movement.
__device__ __forceinline__ int perm_key(int m) { return (m & ~0xC) | ((m & 4) << 1) | ((m & 8) >> 1); }

// Workgroups are handed to the chip's eight XCDs (each with its own L2) round-robin in launch
// order.  With the head as the slow grid index a head's workgroups land on all eight, and every
// L2 fetches every head's K / V tiles from memory.  This remaps (block, head) so that all
// workgroups of a head run on one XCD, heads that share a KV head on the same one, and an XCD
// works through its heads one after the other: the workgroups of a head, which walk the same
// tiles at about the same time, then share them in one L2.  hz = head + heads * sequence.
__device__ __forceinline__ void xcd_remap(int nx, int nhz, int& bx, int& hz) {
  constexpr int kXcd = 8;
  if (nhz % kXcd) return;  // identity when the heads do not divide over the XCDs
  const int lin = bx + nx * hz, xcd = lin % kXcd, s = lin / kXcd;
  hz = xcd * (nhz / kXcd) + s / nx;
  bx = s % nx;
}

constexpr int kKsElems = 64 * kLdK;   // one K tile in LDS
constexpr int kVsElems = kD * kLdV;   // one V^T tile in LDS
constexpr int kAttnSmemBytes = 2 * (kKsElems + kVsElems) * 2;
constexpr int kAttnRW = 1;                     // 32-row blocks per wavefront
constexpr int kAttnNW = 8;                     // wavefronts per workgroup
constexpr int kAttnBM = 32 * kAttnRW * kAttnNW;

// NW wavefronts per workgroup, each owning RW 32-row MFMA column blocks (blocks of one
// wavefront share every K / V^T operand read from LDS).  Built as 8 x 1: 256 query rows per
// workgroup, two wavefronts per SIMD, which measured faster than 4 x 2.  K and V^T tiles of 64
// keys are double-buffered in LDS.  A tile costs a wavefront about as many vector-ALU cycles
// (32 exponentials per lane at a quarter of the ALU rate) as matrix-core cycles (32 MFMAs), so
// the two wavefronts of a SIMD alternate between the two units (see the schedule below).
template <int RW, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_bf16(const uint16_t* __restrict__ Q, View qv,
                                                     const uint16_t* __restrict__ K, View kv,
                                                     const uint16_t* __restrict__ VT, const float* __restrict__ unscale,
                                                     void* __restrict__ O, View ov, float* __restrict__ lse2, int n,
                                                     int npad, int G, int out_f32, int nblk) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* Ks = smem;                 // [2][kKsElems]
  uint16_t* Vs = smem + 2 * kKsElems;  // [2][kVsElems]
  const int Hq = gridDim.y, Hkv = Hq / G;
  int bx = blockIdx.x, hz = blockIdx.y + Hq * blockIdx.z;
  xcd_remap(gridDim.x, Hq * gridDim.z, bx, hz);
  const int hq = hz % Hq, b = hz / Hq, hk = hq / G;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, h = lane >> 5;
  constexpr int kWR = 32 * RW;   // rows per wavefront
  constexpr int NT = 64 * NW;    // threads
  constexpr int NCH = 1024 / NT;  // 16-byte chunks of each tile per thread
  constexpr int BM = NW * kWR;   // query rows per workgroup
  const float scale2 = kLog2e / sqrtf(float(kD));
  // The work of a row block grows with its position (causal).  A workgroup takes row block
  // nblk - 1 - x (the longer one first) and then row block x: every workgroup has the same
  // amount of work and the launch fills the chip in whole rounds (with one row block per
  // workgroup the longest ones ran on a nearly empty chip at the end: 80 % packing).
  for (int pass = 0; pass < 2; ++pass) {
  const int blk = pass == 0 ? nblk - 1 - bx : bx;
  if (pass == 1 && blk >= nblk - 1 - bx) break;
  const int rb = blk * BM;
  const int wr0 = rb + w * kWR;  // first row of this wavefront

  bf16x8 bq[RW][8];
#pragma unroll
  for (int j = 0; j < RW; ++j) {
    const uint16_t* qp = Q + b * qv.sb + hq * qv.sh + int64_t(min(wr0 + j * 32 + m, n - 1)) * qv.sn;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) bq[j][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16 + h * 8);
  }
  const uint16_t* kbase = K + b * kv.sb + hk * kv.sh;
  const uint16_t* vtbase = VT + (int64_t(b) * Hkv + hk) * kD * npad;

  f32x16 o[RW][4];
#pragma unroll
  for (int j = 0; j < RW; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[j][i][r] = 0.f;
  float mrun[RW], lsum[RW];
#pragma unroll
  for (int j = 0; j < RW; ++j) {
    mrun[j] = -INFINITY;
    lsum[j] = 0.f;
  }

  const int last_key = min(rb + BM - 1, n - 1);
  const int ntile = last_key / 64 + 1;

  // staging: each thread moves NCH 16-byte chunks of K and NCH of V^T per tile
  u32x4 kr[NCH], vr[NCH];
  auto issue_k = [&](int t) {
    const int k0 = t * 64;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + NT * i;
      const int row = c >> 4, col = (c & 15) * 8;
      kr[i] = *reinterpret_cast<const u32x4*>(kbase + int64_t(min(k0 + row, n - 1)) * kv.sn + col);
    }
  };
  auto issue_v = [&](int t) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + NT * i;
      const int dd = c >> 3, kc = (c & 7) * 8;
      vr[i] = *reinterpret_cast<const u32x4*>(vtbase + (int64_t(t) * kD + dd) * 64 + kc);
    }
  };
  auto stage_k = [&](int t) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + NT * i;
      const int row = c >> 4, col = (c & 15) * 8;
      // key r of a 32-key sub-tile is stored at LDS row perm_key(r) (an involution), so that
      // MFMA row m, which must see key perm_key(m), reads LDS row m: consecutive rows, no
      // bank conflicts
      const int lrow = (row & 32) | perm_key(row & 31);
      *reinterpret_cast<u32x4*>(&Ks[(t & 1) * kKsElems + lrow * kLdK + col]) = kr[i];
    }
  };
  auto stage_v = [&](int t) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + NT * i;
      const int dd = c >> 3, kc = (c & 7) * 8;
      *reinterpret_cast<u32x4*>(&Vs[(t & 1) * kVsElems + dd * kLdV + kc]) = vr[i];
    }
  };
  // ---- the three stages of a tile, for this wavefront's rows
  f32x16 s[RW][2];
  f16x8 pb[RW][2][2];
  auto active = [&](int t) { return t * 64 <= wr0 + kWR - 1; };  // else the tile is above the diagonal
  auto qk = [&](int t) {  // S^T = K Q^T of tile t (K from its LDS buffer)
    const uint16_t* ksb = Ks + (t & 1) * kKsElems;
#pragma unroll
    for (int j = 0; j < RW; ++j)
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[j][st][r] = 0.f;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&ksb[(st * 32 + m) * kLdK + ks * 16 + h * 8]);
#pragma unroll
        for (int j = 0; j < RW; ++j)
          s[j][st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[j][ks], s[j][st], 0, 0, 0);
      }
  };
  auto softmax = [&](int t) {  // s -> probabilities pb (fp16, scaled), running maximum and sum, rescale of o
    const int k0 = t * 64;
    // register r of sub-tile st holds key k0 + 32*st + 16*(r/8) + 8*h + r%8
    const bool diag = k0 + 63 > wr0;
#pragma unroll
    for (int j = 0; j < RW; ++j) {
      const int q_row = wr0 + j * 32 + m;
      if (diag) {
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + st * 32 + (r >> 3) * 16 + h * 8 + (r & 7);
            if (key > q_row) s[j][st][r] = -INFINITY;
          }
      }
      float mx = s[j][0][0];
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[j][st][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // Exponent reference with 2^12 headroom.  It follows the row maximum lazily: it moves only
      // when the maximum has outgrown it by more than 2^kLazy, so the probabilities stay below
      // 2^(12 + kLazy), inside fp16, and the rescale of the accumulators becomes rare.
      const float mcand = fmaf(mx, scale2, -kPShift);
      const bool grew = mcand > mrun[j] + kLazy;
      const float mnew = grew ? mcand : mrun[j];
      const float alpha = __builtin_amdgcn_exp2f(mrun[j] - mnew);
      mrun[j] = mnew;
      float psum = 0.f;
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[j][st][r], scale2, -mnew));
          psum += p;
          pb[j][st][r >> 3][r & 7] = (_Float16)p;
        }
      lsum[j] = fmaf(lsum[j], alpha, psum);
      if (__any(grew)) {  // wavefront-uniform: skip the rescale when no row's maximum moved
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[j][i][r] *= alpha;
      }
    }
  };
  // o += V^T P^T of tile t, then (WITH_QK) S^T = K Q^T of tile t + 1: 16 + 16 MFMAs whose LDS
  // operands are fetched two batches of four ahead, so that the matrix core never waits for an
  // LDS round trip (the compiler, left alone, keeps only two reads in flight).
  auto mma_operand = [&](int t, int idx) -> u32x4 {
    if (idx < 16) {  // P V: idx = (st, kb, dc)
      const int st = idx >> 3, kb = (idx >> 2) & 1, dc = idx & 3;
      return *reinterpret_cast<const u32x4*>(&Vs[(t & 1) * kVsElems + (dc * 32 + m) * kLdV + st * 32 + kb * 16 + h * 8]);
    }
    const int st = (idx - 16) & 1, ks = (idx - 16) >> 1;  // Q K^T of the next tile, the two sub-tiles alternating
    return *reinterpret_cast<const u32x4*>(&Ks[((t + 1) & 1) * kKsElems + (st * 32 + m) * kLdK + ks * 16 + h * 8]);
  };
  auto mma_issue = [&](int idx, const u32x4& a) {
    if (idx < 16) {
      const int st = idx >> 3, kb = (idx >> 2) & 1, dc = idx & 3;
#pragma unroll
      for (int j = 0; j < RW; ++j)
        o[j][dc] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), pb[j][st][kb], o[j][dc], 0, 0, 0);
    } else {
      const int st = (idx - 16) & 1, ks = (idx - 16) >> 1;
#pragma unroll
      for (int j = 0; j < RW; ++j) {
        if (ks == 0) {
          const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          s[j][st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), bq[j][ks], zero, 0, 0, 0);
        } else {
          s[j][st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), bq[j][ks], s[j][st], 0, 0, 0);
        }
      }
    }
  };
  auto mma_phase = [&](int t, auto with_qk) {
    constexpr int NB = decltype(with_qk)::value ? 8 : 4;  // batches of four MFMAs
    u32x4 A[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) A[0][i] = mma_operand(t, i);
#pragma unroll
    for (int i = 0; i < 4; ++i) A[1][i] = mma_operand(t, 4 + i);
#pragma unroll
    for (int bt = 0; bt < NB; ++bt) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) mma_issue(4 * bt + i, A[bt & 1][i]);
      __builtin_amdgcn_sched_barrier(0);
      if (bt + 2 < NB) {
#pragma unroll
        for (int i = 0; i < 4; ++i) A[bt & 1][i] = mma_operand(t, 4 * (bt + 2) + i);
      }
    }
  };
  auto pv_qk = [&](int t, bool with_qk) {
    if (with_qk)
      mma_phase(t, std::true_type{});
    else
      mma_phase(t, std::false_type{});
  };

  // ---- ping-pong schedule.  The two wavefronts that share a SIMD (w and w + NW/2) run half a
  // tile apart: while one forms its probabilities on the vector ALU, the other runs its two
  // matrix products (P V of the tile, then Q K^T of the next) on the matrix core, and they swap
  // in the middle of the iteration.  K is staged two tiles ahead, V^T one tile ahead.
  const bool late = w >= NW / 2;
  // Pin the arrival of the Q operands here: otherwise the wait for them is placed inside the
  // loop, behind the tile loads issued there, and stalls the matrix products on those.
#pragma unroll
  for (int j = 0; j < RW; ++j)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(bq[j][ks]));
  issue_k(0);
  issue_v(0);
  stage_k(0);
  stage_v(0);
  if (ntile > 1) {
    issue_k(1);
    stage_k(1);
  }
  __syncthreads();
  if (active(0)) {
    qk(0);
    if (!late) softmax(0);
  }
  __syncthreads();
  for (int t = 0; t < ntile; ++t) {
    const bool more = t + 1 < ntile, more2 = t + 2 < ntile;
    if (more2) issue_k(t + 2);
    if (more) issue_v(t + 1);
    if (active(t)) {
      if (late) {
        softmax(t);
      } else {
        pv_qk(t, more && active(t + 1));
      }
    }
    // no barrier between the two halves of an iteration: tiles are staged into buffers that
    // nobody reads during this iteration, and the half-tile offset between the two wavefronts
    // of a SIMD is re-established by the barrier at the end of every iteration
    if (late) {
      if (active(t)) pv_qk(t, more && active(t + 1));
    } else if (more && active(t + 1)) {
      softmax(t + 1);
    }
    // V(t-1) and K(t) were last read before this iteration: their buffers take V(t+1), K(t+2)
    if (more) stage_v(t + 1);
    if (more2) stage_k(t + 2);
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < RW; ++j) {
    const int q_row = wr0 + j * 32 + m;
    const float ltot = lsum[j] + __shfl_xor(lsum[j], 32, 64);
    if (q_row < n) {
      if (h == 0) lse2[(int64_t(b) * Hq + hq) * npad + q_row] = mrun[j] + log2f(ltot);
      if (O) {
        const float inv = unscale[b * Hkv + hk] / ltot;
        const int64_t ooff = b * ov.sb + hq * ov.sh + int64_t(q_row) * ov.sn;
#pragma unroll
        for (int dc = 0; dc < 4; ++dc)
#pragma unroll
          for (int rg = 0; rg < 4; ++rg) {
            // registers 4*rg .. 4*rg+3 hold d = 32*dc + 8*rg + 4*h + 0..3
            const int dd = dc * 32 + rg * 8 + h * 4;
            if (out_f32) {
              f32x4 v;
#pragma unroll
              for (int i = 0; i < 4; ++i) v[i] = o[j][dc][4 * rg + i] * inv;
              *reinterpret_cast<f32x4*>(static_cast<float*>(O) + ooff + dd) = v;
            } else {
              u32x2 v;
              v[0] = Elem<uint16_t>::from_f32(o[j][dc][4 * rg + 0] * inv) |
                     (uint32_t(Elem<uint16_t>::from_f32(o[j][dc][4 * rg + 1] * inv)) << 16);
              v[1] = Elem<uint16_t>::from_f32(o[j][dc][4 * rg + 2] * inv) |
                     (uint32_t(Elem<uint16_t>::from_f32(o[j][dc][4 * rg + 3] * inv)) << 16);
              *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(O) + ooff + dd) = v;
            }
          }
      }
    }
  }
  }
}

// 256 keys per workgroup (8 wavefronts x 32 keys, the stationary A operand).  Query tiles of
// 64 rows are double-buffered in LDS and visited from the END of the prompt downwards: every
// workgroup of a head then reads the same query tiles at about the same time (all start at
// the last tile), so the tiles are served from L2 instead of HBM.
constexpr int kColNW = 8;
__global__ __launch_bounds__(64 * kColNW) __attribute__((amdgpu_waves_per_eu(4, 4))) void colsum_bf16(const uint16_t* __restrict__ Q, View qv,
                                                           const uint16_t* __restrict__ K, View kv,
                                                           const float* __restrict__ lse2, float* __restrict__ score,
                                                           double* __restrict__ varpart, int n, int npad, int G,
                                                           int Hq, int nblk) {
  __shared__ __attribute__((aligned(16))) uint16_t Qs[2][64 * kLdK];
  __shared__ float ls[2][64];
  __shared__ float cs[kColBN];
  __shared__ double red[kColNW];
  constexpr int NT = 64 * kColNW;
  constexpr int NCH = 1024 / NT;
  const int Hkv = gridDim.y;
  int bx = blockIdx.x, hz = blockIdx.y + Hkv * blockIdx.z;
  xcd_remap(gridDim.x, Hkv * gridDim.z, bx, hz);
  const int hk = hz % Hkv, b = hz / Hkv;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, h = lane >> 5;
  const float scale2 = kLog2e / sqrtf(float(kD));
  // The work of a key block grows with the number of queries behind it (causal), from one
  // query tile for the last block to all of them for the first.  A workgroup takes block x and
  // then block nblk - 1 - x: every workgroup then has the same amount of work and the launch
  // fills the chip in whole rounds (with one block per workgroup the CUs held 1.3 of 2 possible
  // workgroups on average, and the longest workgroup alone was a fifth of the kernel time).
  for (int pass = 0; pass < 2; ++pass) {
  const int tile = pass == 0 ? bx : nblk - 1 - bx;
  if (pass == 1 && tile <= bx) break;
  const int kb0 = tile * kColBN, kw0 = kb0 + w * 32;  // first key of the workgroup / wavefront

  const uint16_t* kp = K + b * kv.sb + hk * kv.sh + int64_t(min(kw0 + m, n - 1)) * kv.sn;
  bf16x8 ak[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) ak[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 16 + h * 8);

  const int nqt = (n - kb0 + 63) / 64;  // query tiles [kb0 + 64 j, kb0 + 64 j + 64), visited j descending
  float total = 0.f;                    // thread t < 256 owns key kb0 + t
  for (int g = 0; g < G; ++g) {
    const int hq = hk * G + g;
    const uint16_t* qb = Q + b * qv.sb + hq * qv.sh;
    const float* lrow = lse2 + (int64_t(b) * Hq + hq) * npad;
    float acc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    u32x4 qr[NCH];
    float lr = 0.f;
    auto issue = [&](int j) {
      const int q0 = kb0 + 64 * j;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = tid + NT * i, row = c >> 4, col = (c & 15) * 8;
        qr[i] = *reinterpret_cast<const u32x4*>(qb + int64_t(min(q0 + row, n - 1)) * qv.sn + col);
      }
      if (tid < 64) lr = (q0 + tid < n) ? lrow[q0 + tid] : INFINITY;  // +inf => p = 0
    };
    auto stage = [&](int buf) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = tid + NT * i, row = c >> 4, col = (c & 15) * 8;
        *reinterpret_cast<u32x4*>(&Qs[buf][row * kLdK + col]) = qr[i];
      }
      if (tid < 64) ls[buf][tid] = lr;
    };
    __syncthreads();  // previous head's readers are done with both buffers
    issue(nqt - 1);
    stage(0);
    __syncthreads();
    for (int it = 0; it < nqt; ++it) {
      const int j = nqt - 1 - it, buf = it & 1, q0 = kb0 + 64 * j;
      if (j > 0) issue(j - 1);
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        const int qbase = q0 + qt * 32;
        if (qbase + 31 < kw0) continue;  // every query precedes every key of this wavefront
        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 bqv = *reinterpret_cast<const bf16x8*>(&Qs[buf][(qt * 32 + m) * kLdK + ks * 16 + h * 8]);
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak[ks], bqv, sacc, 0, 0, 0);
        }
        // register r: key kw0 + (r/4)*8 + 4h + r%4, query qbase + m
        const float lq = ls[buf][qt * 32 + m];
        const int query = qbase + m;
        if (qbase < kw0 + 31) {  // diagonal tile: mask query < key
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kw0 + (r >> 2) * 8 + h * 4 + (r & 3);
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[r], scale2, -lq));
            acc[r] += (query >= key) ? p : 0.f;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[r] += __builtin_amdgcn_exp2f(fmaf(sacc[r], scale2, -lq));
        }
      }
      if (j > 0) stage(buf ^ 1);
      __syncthreads();
    }
    // add the 32 query columns held by the lanes of each half
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = acc[r];
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      acc[r] = v;
    }
    if (m == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) cs[w * 32 + (r >> 2) * 8 + h * 4 + (r & 3)] = acc[r];
    }
    __syncthreads();
    double c1 = 0.0, c2 = 0.0;
    if (tid < kColBN && kb0 + tid < n) {
      const float c = cs[tid];
      total += c;
      c1 = double(c);
      c2 = double(c) * double(c);
    }
    // partial sums per 128-key block (the unit the density reduction adds up)
    const bool lo = tid < 128;
    const double s1a = block_sum(lo ? c1 : 0.0, red), s2a = block_sum(lo ? c2 : 0.0, red);
    const double s1b = block_sum(lo ? 0.0 : c1, red), s2b = block_sum(lo ? 0.0 : c2, red);
    if (tid == 0) {
      double* vp = varpart + ((int64_t(b) * Hq + hq) * (npad / 128) + tile * 2) * 2;
      vp[0] = s1a;
      vp[1] = s2a;
      if (kb0 + 128 < npad) {
        vp[2] = s1b;
        vp[3] = s2b;
      }
    }
  }
  if (tid < kColBN && kb0 + tid < n) score[(int64_t(b) * Hkv + hk) * npad + kb0 + tid] = total;
  }
}

}  // namespace

hipError_t launch_prefill_bf16(d2o_ctx* c, int layer, View Q, View K, View V, View O, int n, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int G = cf.n_q_heads / cf.n_kv_heads;
  float* score = c->score_pre + size_t(layer) * cf.batch * cf.n_kv_heads * c->npad;
  const int nblk = (n + kAttnBM - 1) / kAttnBM;
  const int nblk_col = (n + kColBN - 1) / kColBN;
  {  // the attribute is per device; setting it is a cheap host-side call, so it is not cached
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fwd_bf16<kAttnRW, kAttnNW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kAttnSmemBytes);
    if (e != hipSuccess) return e;
  }
  const int nbh = cf.batch * cf.n_kv_heads;
  zero_u32<<<(nbh + 255) / 256, 256, 0, s>>>(c->vmax_bits, nbh);
  vabsmax_kernel<<<dim3(std::min(64, (n * 16 + 255) / 256), cf.n_kv_heads, cf.batch), 256, 0, s>>>(
      (const uint16_t*)V.ptr, V, c->vmax_bits, n);
  transpose_v<<<dim3(c->npad / 64, cf.n_kv_heads, cf.batch), 256, 0, s>>>((const uint16_t*)V.ptr, V, (uint16_t*)c->vt,
                                                                         c->vmax_bits, c->vt_unscale, n, c->npad);
  {
  KernelTimer kt(c, D2O_K_ATTN_FWD, s);
  attn_fwd_bf16<kAttnRW, kAttnNW><<<dim3((nblk + 1) / 2, cf.n_q_heads, cf.batch), 64 * kAttnNW, kAttnSmemBytes, s>>>(
      (const uint16_t*)Q.ptr, Q, (const uint16_t*)K.ptr, K, (const uint16_t*)c->vt, c->vt_unscale, O.ptr, O, c->lse, n,
      c->npad, G, cf.out_f32, nblk);
  }
  KernelTimer kt(c, D2O_K_COLSUM, s);
  colsum_bf16<<<dim3((nblk_col + 1) / 2, cf.n_kv_heads, cf.batch), 64 * kColNW, 0, s>>>(
      (const uint16_t*)Q.ptr, Q, (const uint16_t*)K.ptr, K, c->lse, score, c->varpart, n, c->npad, G, cf.n_q_heads,
      nblk_col);
  return hipGetLastError();
}

}  // namespace d2o
