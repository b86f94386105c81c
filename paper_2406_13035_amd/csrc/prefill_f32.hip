// Prompt-phase attention for fp32 tensors (the small configuration) and the density
// reduction shared by both dtypes.  fp32 inputs are never down-converted: products and sums
// are plain fp32 FMAs on the vector ALU, one wavefront per query row (pass 1) and per key
// (pass 2).  The bf16 path in prefill_bf16.hip uses the matrix cores instead.
//
// Pass 1 (Sec. 4.1 Eq. 4, Sec. 3 Eq. 3): O = softmax(Q K^T / sqrt(d)) V, causal, and the row
//   log-sum-exp.  Pass 2 (column sums of the attention matrix, Sec. 4.1; Eq. 6 prompt case):
//   score[j] = sum_g sum_{i >= j} exp(s_ij - lse_i), plus per-query-head partial sums of the
//   column sums and their squares for the variance of Eq. 4.
#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace {

constexpr float kLog2e = 1.4426950408889634f;

// One wavefront per query row; lanes stride over the keys j <= i with private online-softmax
// state that is combined across the wavefront at the end.
template <int D>
__global__ __launch_bounds__(256) void attn_rows_f32(const float* __restrict__ Q, View qv, const float* __restrict__ K,
                                                     View kv, const float* __restrict__ V, View vv, float* __restrict__ O,
                                                     View ov, float* __restrict__ lse2, int n, int npad, int G) {
  __shared__ float qs[4][D];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + w, hq = blockIdx.y, b = blockIdx.z, hk = hq / G;
  const bool live = i < n;
  const int ii = live ? i : n - 1;
  const float* qrow = Q + b * qv.sb + hq * qv.sh + int64_t(ii) * qv.sn;
  for (int c = lane; c < D; c += 64) qs[w][c] = qrow[c];
  __syncthreads();
  const float scale2 = kLog2e / sqrtf(float(D));
  const float* kb = K + b * kv.sb + hk * kv.sh;
  const float* vb = V + b * vv.sb + hk * vv.sh;
  float m = -INFINITY, l = 0.f;
  float acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.f;
  for (int j = lane; j <= ii; j += 64) {
    const float4* kr = reinterpret_cast<const float4*>(kb + int64_t(j) * kv.sn);
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < D / 4; ++c) {
      const float4 k4 = kr[c];
      s = fmaf(qs[w][4 * c + 0], k4.x, s);
      s = fmaf(qs[w][4 * c + 1], k4.y, s);
      s = fmaf(qs[w][4 * c + 2], k4.z, s);
      s = fmaf(qs[w][4 * c + 3], k4.w, s);
    }
    s *= scale2;
    const float mn = fmaxf(m, s);
    const float a = exp2f(m - mn), p = exp2f(s - mn);
    l = l * a + p;
    const float4* vr = reinterpret_cast<const float4*>(vb + int64_t(j) * vv.sn);
#pragma unroll
    for (int c = 0; c < D / 4; ++c) {
      const float4 v4 = vr[c];
      acc[4 * c + 0] = fmaf(acc[4 * c + 0], a, p * v4.x);
      acc[4 * c + 1] = fmaf(acc[4 * c + 1], a, p * v4.y);
      acc[4 * c + 2] = fmaf(acc[4 * c + 2], a, p * v4.z);
      acc[4 * c + 3] = fmaf(acc[4 * c + 3], a, p * v4.w);
    }
    m = mn;
  }
  const float M = wave_max(m);
  const float f = (m == -INFINITY) ? 0.f : exp2f(m - M);
  const float lt = wave_sum(l * f);
  float* orow = O ? O + b * ov.sb + hq * ov.sh + int64_t(ii) * ov.sn : nullptr;
#pragma unroll
  for (int c = 0; c < D; ++c) {
    const float t = wave_sum(acc[c] * f);
    if (live && orow && lane == (c & 63)) orow[c] = t / lt;
  }
  if (live && lane == 0) lse2[(int64_t(b) * gridDim.y + hq) * npad + i] = M + log2f(lt);
}

// One workgroup per 128 keys of a KV head, one wavefront per key in turn; lanes stride over
// the query rows i >= j.  Adds the G query heads of the group in ascending order.
template <int D>
__global__ __launch_bounds__(256) void colsum_f32(const float* __restrict__ Q, View qv, const float* __restrict__ K,
                                                  View kv, const float* __restrict__ lse2, float* __restrict__ score,
                                                  double* __restrict__ varpart, int n, int npad, int G, int Hq) {
  __shared__ float ks[4][D];
  __shared__ float cs[128];
  __shared__ double red[4];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int tile = blockIdx.x, hk = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const float scale2 = kLog2e / sqrtf(float(D));
  const float* kb = K + b * kv.sb + hk * kv.sh;
  float total = 0.f;  // thread t < 128 owns key tile*128 + t
  for (int g = 0; g < G; ++g) {
    const int hq = hk * G + g;
    const float* qb = Q + b * qv.sb + hq * qv.sh;
    const float* lrow = lse2 + (int64_t(b) * Hq + hq) * npad;
    for (int t = 0; t < 32; ++t) {
      const int jl = w * 32 + t, j = tile * 128 + jl;
      __syncthreads();
      if (j < n)
        for (int c = lane; c < D; c += 64) ks[w][c] = kb[int64_t(j) * kv.sn + c];
      __syncthreads();
      float sum = 0.f;
      if (j < n) {
        for (int i = j + lane; i < n; i += 64) {
          const float4* qr = reinterpret_cast<const float4*>(qb + int64_t(i) * qv.sn);
          float s = 0.f;
#pragma unroll
          for (int c = 0; c < D / 4; ++c) {
            const float4 q4 = qr[c];
            s = fmaf(q4.x, ks[w][4 * c + 0], s);
            s = fmaf(q4.y, ks[w][4 * c + 1], s);
            s = fmaf(q4.z, ks[w][4 * c + 2], s);
            s = fmaf(q4.w, ks[w][4 * c + 3], s);
          }
          sum += exp2f(s * scale2 - lrow[i]);
        }
      }
      sum = wave_sum(sum);
      if (lane == 0) cs[jl] = sum;
    }
    __syncthreads();
    double s1 = 0.0, s2 = 0.0;
    if (threadIdx.x < 128 && tile * 128 + int(threadIdx.x) < n) {
      const float c = cs[threadIdx.x];
      total += c;
      s1 = double(c);
      s2 = double(c) * double(c);
    }
    s1 = block_sum(s1, red);
    s2 = block_sum(s2, red);
    if (threadIdx.x == 0) {
      double* vp = varpart + ((int64_t(b) * Hq + hq) * (npad / 128) + tile) * 2;
      vp[0] = s1;
      vp[1] = s2;
    }
  }
  if (threadIdx.x < 128 && tile * 128 + int(threadIdx.x) < n)
    score[(int64_t(b) * Hkv + hk) * npad + tile * 128 + threadIdx.x] = total;
}

// Per sequence: variance of every query head's column sums (population, Eq. 4) from the
// per-tile partial sums, added in ascending tile order, and their mean over heads.
__global__ void density_kernel(const double* __restrict__ varpart, double* __restrict__ head_var,
                               double* __restrict__ layer_F, int n, int npad, int Hq) {
  __shared__ double hv[256];
  const int b = blockIdx.x;
  const int ntile = (n + 127) / 128;
  for (int hq = threadIdx.x; hq < Hq; hq += blockDim.x) {
    const double* vp = varpart + (int64_t(b) * Hq + hq) * (npad / 128) * 2;
    double s1 = 0.0, s2 = 0.0;
    for (int t = 0; t < ntile; ++t) {
      s1 += vp[2 * t];
      s2 += vp[2 * t + 1];
    }
    const double mu = s1 / double(n);
    const double var = s2 / double(n) - mu * mu;
    head_var[int64_t(b) * Hq + hq] = var;
    hv[hq] = var;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int hq = 0; hq < Hq; ++hq) t += hv[hq];
    layer_F[b] = t / double(Hq);
  }
}

}  // namespace

hipError_t launch_prefill_f32(d2o_ctx* c, int layer, View Q, View K, View V, View O, int n, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int G = cf.n_q_heads / cf.n_kv_heads;
  float* score = c->score_pre + size_t(layer) * cf.batch * cf.n_kv_heads * c->npad;
  dim3 g1((n + 3) / 4, cf.n_q_heads, cf.batch), g2((n + 127) / 128, cf.n_kv_heads, cf.batch);
  if (cf.head_dim == 64) {
    { KernelTimer kt(c, D2O_K_ATTN_FWD, s);
    attn_rows_f32<64><<<g1, 256, 0, s>>>((const float*)Q.ptr, Q, (const float*)K.ptr, K, (const float*)V.ptr, V,
                                         (float*)O.ptr, O, c->lse, n, c->npad, G); }
    KernelTimer kt(c, D2O_K_COLSUM, s);
    colsum_f32<64><<<g2, 256, 0, s>>>((const float*)Q.ptr, Q, (const float*)K.ptr, K, c->lse, score, c->varpart, n,
                                      c->npad, G, cf.n_q_heads);
  } else {
    { KernelTimer kt(c, D2O_K_ATTN_FWD, s);
    attn_rows_f32<128><<<g1, 256, 0, s>>>((const float*)Q.ptr, Q, (const float*)K.ptr, K, (const float*)V.ptr, V,
                                          (float*)O.ptr, O, c->lse, n, c->npad, G); }
    KernelTimer kt(c, D2O_K_COLSUM, s);
    colsum_f32<128><<<g2, 256, 0, s>>>((const float*)Q.ptr, Q, (const float*)K.ptr, K, c->lse, score, c->varpart, n,
                                       c->npad, G, cf.n_q_heads);
  }
  return hipGetLastError();
}

hipError_t launch_density(d2o_ctx* c, int layer, int n, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  density_kernel<<<cf.batch, 256, 0, s>>>(c->varpart, c->head_var + size_t(layer) * cf.batch * cf.n_q_heads,
                                          c->layer_F + size_t(layer) * cf.batch, n, c->npad, cf.n_q_heads);
  return hipGetLastError();
}

}  // namespace d2o
