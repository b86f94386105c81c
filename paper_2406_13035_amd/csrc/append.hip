// Multi-token append, ordering stage.  After the tokens of a block have been appended and have
// added their softmax rows to the scores (the decode kernels, one token after the other, nothing
// evicted), Eq. 7-12 are applied once to every cache.  Those stages are the prompt-phase kernels
// of tokens.hip, which work on rows in ascending token position; a cache's slots are physically
// unordered, so this file lays every cache of the layer out in position order first:
//
//   rank_by_position   per (sequence, KV head): rank of every slot's position among the head's
//                      positions (positions are distinct), the ordered positions and fp64 scores,
//                      and the number of entries;
//   permute_rows       K and V rows of every slot to their rank in the ordered copy.
#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace {

constexpr int kRankTile = 4096;  // positions held in LDS at a time

__global__ __launch_bounds__(1024) void rank_by_position(const int32_t* __restrict__ ccount,   // the layer's [B][Hkv]
                                                         const int32_t* __restrict__ meta,     // the layer's [B][Hkv][4]
                                                         const double* __restrict__ cscore,
                                                         const int32_t* __restrict__ cpos, int32_t* __restrict__ rank,
                                                         int32_t* __restrict__ opos, double* __restrict__ oscore,
                                                         int32_t* __restrict__ on, int npad, int64_t slots) {
  __shared__ int32_t tile[kRankTile];
  const int hk = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x, tid = threadIdx.x;
  const int64_t bh = int64_t(b) * Hkv + hk;
  const int n = ccount[bh];
  const int64_t slot0 = bh * slots + meta[bh * 4 + 0];
  if (tid == 0) on[bh] = n;
  // every thread owns the slots tid, tid + 1024, ...; the positions pass through LDS tile by tile
  // and each owned slot counts the smaller ones (all threads read the same LDS word at a time)
  for (int j0 = 0; j0 < n; j0 += 4 * 1024) {
    int mine[4], cnt[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 1024 + tid;
      mine[u] = j < n ? cpos[slot0 + j] : 0x7FFFFFFF;
      cnt[u] = 0;
    }
    for (int t0 = 0; t0 < n; t0 += kRankTile) {
      __syncthreads();
      for (int i = tid; i < kRankTile; i += 1024) tile[i] = t0 + i < n ? cpos[slot0 + t0 + i] : 0x7FFFFFFF;
      __syncthreads();
      const int lim = min(kRankTile, n - t0);
      for (int i = 0; i < lim; ++i) {
        const int p = tile[i];
#pragma unroll
        for (int u = 0; u < 4; ++u) cnt[u] += p < mine[u] ? 1 : 0;
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 1024 + tid;
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

}  // namespace

hipError_t launch_cache_sort(d2o_ctx* c, int layer, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int32_t* meta = c->meta + size_t(layer) * cf.batch * cf.n_kv_heads * 4;
  const int32_t* ccount = c->ccount + size_t(layer) * cf.batch * cf.n_kv_heads;
  int max_rows = 0;
  for (const auto& mt : c->layers[layer].meta) max_rows = std::max(max_rows, mt.budget + c->grow);
  rank_by_position<<<dim3(cf.n_kv_heads, cf.batch), 1024, 0, s>>>(ccount, meta, c->cscore, c->cpos, c->app_rank,
                                                                  c->app_pos, c->app_score, c->app_n, c->npad,
                                                                  cf.slots_per_seq);
  if (cf.dtype == D2O_BF16) {
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

}  // namespace d2o
