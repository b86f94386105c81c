// Upstream step of the hot path (Sec. 3 Eq. 1): Q = X W_Q, K = X W_K, V = X W_V for one layer as
// ONE matrix product on the CDNA4 matrix cores, with the rotary position embedding of queries
// and keys applied to the fp32 accumulators before they are stored, and the three results
// written directly in the [sequence][head][token][d] layout that the prompt attention reads.
//
// bf16 operands, fp32 accumulation, head_dim 128.  X [B * n][hidden] and the stacked weights
// W [(Hq + 2 Hkv) * 128][hidden] are both contiguous along `hidden`, which is the layout both
// operands of v_mfma_f32_32x32x16_bf16 want (lane l: row l % 32, eight consecutive k from
// 8 * (l / 32)).
//
// A workgroup (8 wavefronts) computes 256 tokens x 256 features = two heads; a wavefront owns 64
// tokens x one head's 128 features (2 x 4 accumulator blocks: six LDS operand reads feed eight
// matrix instructions).  The feature pair (c, c + 64) that the rotary embedding mixes lives in the same
// lane and register of accumulator blocks j and j + 2, so the rotation needs no exchange.  The
// rotated tile goes through LDS once so that every lane stores 16 contiguous bytes of a token's
// head vector.
#include <algorithm>

#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace {

constexpr int kBM = 256, kBN = 128, kBK = 32;  // kBN: one head; a workgroup's tile holds kHeadsPerWg of them
constexpr int kHeadsPerWg = 2, kThreads = 512;
constexpr int kLd = kBK;                     // LDS pitch (elements) of the operand tiles: 64 bytes = four 16-byte chunks,
                                             // chunk k of row r stored at position k ^ ((r >> 2) & 3): the 16 lanes of a
                                             // 128-bit access phase then cover all 64 banks once, for the staging stores
                                             // (four consecutive rows x four chunks) and for the operand reads (sixteen
                                             // consecutive rows, one chunk)
constexpr int kLdC = kBN + 8;                // LDS pitch of the result tile
constexpr int kOperandElems = 2 * (kBM + kHeadsPerWg * kBN) * kLd;  // two stages
constexpr int kResultElems = kBM / 2 * kLdC;          // the result tile passes through LDS in two halves
constexpr int kSmemElems = kOperandElems > kResultElems ? kOperandElems : kResultElems;

struct QkvArgs {
  const uint16_t* X;
  const uint16_t* W;
  View q, k, v;        // [b][head][token][d]
  int M, n, hidden, Hq, Hkv, pos0;
  double log2_base;
};

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void qkv_rope_bf16(QkvArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t smem[kSmemElems];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, h = lane >> 5;
  // Workgroups go to the eight XCDs round-robin in launch order.  Each XCD takes one eighth of
  // the heads (its slice of W stays close to it) and walks the token tiles with its heads as
  // the fast index, so the workgroups that run together share a few token tiles and that slice.
  int ftile = blockIdx.x;  // feature tile = a pair of heads out of [Q heads | K heads | V heads]
  int rt = blockIdx.y;     // token tile
  if (gridDim.x % 8 == 0) {
    const int lin = blockIdx.x + gridDim.x * blockIdx.y, xcd = lin & 7, s_ = lin >> 3, fpx = gridDim.x / 8;
    ftile = xcd * fpx + s_ % fpx;
    rt = s_ / fpx;
  }
  const int nheads = a.Hq + 2 * a.Hkv;
  const int wm = w & 3, wn = w >> 2;      // the wavefront's 64 tokens, and which head of the pair
  const int ft = ftile * kHeadsPerWg + wn;  // this wavefront's head (an odd head count leaves the last tile's second half idle)
  const bool live = ft < nheads;
  const int row0 = rt * kBM;  // first token (flattened over sequences) of the tile
  const uint16_t* Xb = a.X;
  const uint16_t* Wb = a.W + int64_t(ftile) * kHeadsPerWg * kBN * a.hidden;
  const int wrows = min(kHeadsPerWg * kBN, (nheads - ftile * kHeadsPerWg) * kBN);  // weight rows this tile has
  constexpr int kStageElems = (kBM + kHeadsPerWg * kBN) * kLd;
  auto As = [&](int st) { return smem + st * kStageElems; };
  auto Bs = [&](int st) { return smem + st * kStageElems + kBM * kLd; };

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // staging: a tile row holds 64 bytes = four 16-byte chunks; 1024 chunks of X and 512 of W.
  // Two register sets: the loads of k-tile t + 2 are issued while tile t is multiplied, and a
  // tile moves from its registers to LDS one iteration after that, so a load has two
  // iterations (and the other resident workgroup's) to arrive; one iteration is shorter than
  // an L2 round trip under load.
  auto swz = [](int row, int col) { return col ^ (((row >> 2) & 3) << 3); };  // col: element offset of a 16-byte chunk
  constexpr int NA = kBM * 4 / kThreads, NB = kHeadsPerWg * kBN * 4 / kThreads;  // 16-byte chunks per thread
  struct Regs {
    u32x4 a[NA], b[NB];
  } R0, R1;
  auto issue = [&](int kt, Regs& R) {
    const int k0 = kt * kBK;
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const int c = tid + kThreads * i, row = c >> 2, col = (c & 3) * 8;
      R.a[i] = *reinterpret_cast<const u32x4*>(Xb + int64_t(min(row0 + row, a.M - 1)) * a.hidden + k0 + col);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int c = tid + kThreads * i, row = c >> 2, col = (c & 3) * 8;
      R.b[i] = *reinterpret_cast<const u32x4*>(Wb + int64_t(min(row, wrows - 1)) * a.hidden + k0 + col);
    }
  };
  auto stage = [&](int st, const Regs& R) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const int c = tid + kThreads * i, row = c >> 2, col = (c & 3) * 8;
      *reinterpret_cast<u32x4*>(As(st) + row * kLd + swz(row, col)) = R.a[i];
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int c = tid + kThreads * i, row = c >> 2, col = (c & 3) * 8;
      *reinterpret_cast<u32x4*>(Bs(st) + row * kLd + swz(row, col)) = R.b[i];
    }
  };
  // all operand reads of a stage first, then its sixteen matrix instructions back to back
  auto multiply = [&](int st) {
    bf16x8 av[kBK / 16][2], bv[kBK / 16][4];
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
        av[ks][i] = *reinterpret_cast<const bf16x8*>(As(st) + (wm * 64 + i * 32 + m) * kLd + swz(m, ks * 16 + h * 8));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        bv[ks][j] = *reinterpret_cast<const bf16x8*>(Bs(st) + (wn * kBN + j * 32 + m) * kLd + swz(m, ks * 16 + h * 8));
    }
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ks][i], bv[ks][j], acc[i][j], 0, 0, 0);
  };
  const int nk = a.hidden / kBK;
  issue(0, R0);
  if (nk > 1) issue(1, R1);
  stage(0, R0);
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    // LDS stage 0 holds tile kt, R1 tile kt + 1
    if (kt + 2 < nk) issue(kt + 2, R0);
    multiply(0);
    if (kt + 1 < nk) stage(1, R1);
    __syncthreads();
    if (kt + 1 >= nk) break;
    // LDS stage 1 holds tile kt + 1, R0 tile kt + 2
    if (kt + 3 < nk) issue(kt + 3, R1);
    multiply(1);
    if (kt + 2 < nk) stage(0, R0);
    __syncthreads();
  }
  // ---- rotary embedding on queries and keys.  Accumulator layout: acc[i][j][r] is token
  //      wm*64 + i*32 + (r/4)*8 + 4h + r%4 of the tile, feature j*32 + m of the wavefront's head.  Features c < 64 pair with
  //      c + 64: blocks (0, 2) and (1, 3) of the same lane and register.
  const bool rotate = live && ft < a.Hq + a.Hkv;
  if (rotate) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int c = j * 32 + m;
      // turns (angle / 2 pi) per position step of this feature pair
      const double turns_per_pos = exp2(-(2.0 * double(c) / double(kBN)) * a.log2_base) * 0.15915494309189535;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int t = row0 + wm * 64 + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
          const int pos = a.pos0 + (t % a.n);
          // the angle in fp64, reduced to a fraction of a turn before the fp32 sine and cosine
          // (positions reach 10^5: an fp32 product would be off by a hundredth of a radian); the
          // hardware sine and cosine take their argument in turns
          const double turns = double(pos) * turns_per_pos;
          const float frac = float(turns - rint(turns));
          const float sn = __builtin_amdgcn_sinf(frac), cs = __builtin_amdgcn_cosf(frac);
          const float x0 = acc[i][j][r], x1 = acc[i][j + 2][r];
          acc[i][j][r] = x0 * cs - x1 * sn;
          acc[i][j + 2][r] = x1 * cs + x0 * sn;
        }
    }
  }
  // ---- through LDS (the operand tiles are no longer needed; the loop's last barrier has passed),
  //      one head and 128 tokens at a time: [token][feature] in bf16, then 16 contiguous bytes per lane
  uint16_t* Cs = smem;
#pragma unroll 1
  for (int pass = 0; pass < 2 * kHeadsPerWg; ++pass) {
    const int half = pass & 1, hsel = pass >> 1;
    if (wn == hsel && (wm >> 1) == half) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int row = (wm & 1) * 64 + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
            Cs[row * kLdC + j * 32 + m] = Elem<uint16_t>::from_f32(acc[i][j][r]);
          }
    }
    __syncthreads();
    // which tensor and head this pass writes
    const int fh = ftile * kHeadsPerWg + hsel;
    if (fh < nheads) {
      View dst = a.q;
      int head = fh;
      if (fh >= a.Hq + a.Hkv) {
        dst = a.v;
        head = fh - a.Hq - a.Hkv;
      } else if (fh >= a.Hq) {
        dst = a.k;
        head = fh - a.Hq;
      }
      uint16_t* out = static_cast<uint16_t*>(dst.ptr);
#pragma unroll
      for (int i = 0; i < kBM / 2 * kBN / 8 / kThreads; ++i) {
        const int c = tid + kThreads * i, row = c >> 4, col = (c & 15) * 8;
        const int t = row0 + half * (kBM / 2) + row;
        if (t < a.M) {
          const int b = t / a.n, tok = t % a.n;
          *reinterpret_cast<u32x4*>(out + b * dst.sb + head * dst.sh + int64_t(tok) * dst.sn + col) =
              *reinterpret_cast<const u32x4*>(Cs + row * kLdC + col);
        }
      }
    }
    __syncthreads();
  }
}

}  // namespace
}  // namespace d2o

using namespace d2o;

extern "C" int d2o_qkv_project(int32_t batch, int32_t n, int32_t hidden, int32_t n_q_heads, int32_t n_kv_heads,
                               int32_t head_dim, int32_t dtype, const void* X, const void* W, d2o_view Q,
                               d2o_view K, d2o_view V, int32_t pos0, double rope_base, void* stream) {
  if (batch < 1 || n < 1 || hidden < 1 || n_q_heads < 1 || n_kv_heads < 1 || !X || !W || pos0 < 0 ||
      !(rope_base > 1.0))
    return D2O_ERR_INVALID_ARG;
  if (dtype != D2O_BF16 || head_dim != kBN) return D2O_ERR_UNSUPPORTED;
  if (hidden % kBK) return D2O_ERR_UNSUPPORTED;
  if (int64_t(batch) * n > 0x7FFFFFFF) return D2O_ERR_INVALID_ARG;
  for (const d2o_view* v : {&Q, &K, &V}) {
    if (!v->ptr || (reinterpret_cast<uintptr_t>(v->ptr) & 15) || v->stride_b % 8 || v->stride_h % 8 ||
        v->stride_n % 8 || v->stride_n < head_dim)
      return D2O_ERR_INVALID_ARG;
  }
  if ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(W)) & 15) return D2O_ERR_INVALID_ARG;
  QkvArgs a;
  a.X = static_cast<const uint16_t*>(X);
  a.W = static_cast<const uint16_t*>(W);
  a.q = to_view(Q);
  a.k = to_view(K);
  a.v = to_view(V);
  a.M = batch * n;
  a.n = n;
  a.hidden = hidden;
  a.Hq = n_q_heads;
  a.Hkv = n_kv_heads;
  a.pos0 = pos0;
  a.log2_base = std::log2(rope_base);
  const dim3 grid((n_q_heads + 2 * n_kv_heads + kHeadsPerWg - 1) / kHeadsPerWg, (a.M + kBM - 1) / kBM);
  qkv_rope_bf16<<<grid, kThreads, 0, static_cast<hipStream_t>(stream)>>>(a);
  return hipGetLastError() == hipSuccess ? D2O_OK : D2O_ERR_HIP;
}
