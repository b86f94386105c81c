// fp8 cache encoding (d2o_config::cache_fp8): a cache row is d codes of the 8-bit float format
// E4M3 and one power of two, value = code * 2^e with e the smallest exponent that brings the
// row's largest magnitude to 448 or below, codes rounded to nearest even.  The paper names the
// combination with KV-cache quantisation as future work and fixes no format; this is the
// reading the oracle states.
//
// The prompt-phase kernels (compaction, matching, merge) work on bf16 staging rows
// [B][Hkv][npad][d]; encode_rows turns a layer's finished rows into cache rows.  The same
// kernel, on one head, serves d2o_cache_import; decode_rows is its inverse for
// d2o_cache_export.  (The generation step encodes and decodes rows inside its own kernels.)
#include "d2o_internal.h"
#include "device_utils.h"

namespace d2o {
namespace {

// One wavefront per row, two elements per lane (head_dim 128, bf16 staging rows).
__global__ __launch_bounds__(256) void encode_rows(const int32_t* __restrict__ ccount, const int32_t* __restrict__ meta,
                                                   const uint16_t* __restrict__ sK, const uint16_t* __restrict__ sV,
                                                   uint8_t* __restrict__ cK, uint8_t* __restrict__ cV,
                                                   int8_t* __restrict__ cKe, int8_t* __restrict__ cVe, int npad,
                                                   int64_t slots, int head0, int count_arg) {
  constexpr int D = 128;
  const int bh = head0 + blockIdx.y, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int count = count_arg >= 0 ? count_arg : ccount[bh];
  if (row >= count) return;
  const int64_t dst = int64_t(bh) * slots + meta[bh * 4 + 0] + row;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const uint16_t* src = (which ? sV : sK) + (int64_t(bh) * npad + row) * D;
    const uint32_t two = reinterpret_cast<const uint32_t*>(src)[lane];
    const double x0 = double(__uint_as_float(two << 16)), x1 = double(__uint_as_float(two & 0xFFFF0000u));
    const int e = fp8_row_exponent(wave_max(fmax(fabs(x0), fabs(x1))));
    const uint16_t codes = uint16_t(fp8_encode(ldexp(x0, -e))) | uint16_t(uint16_t(fp8_encode(ldexp(x1, -e))) << 8);
    reinterpret_cast<uint16_t*>((which ? cV : cK) + dst * D)[lane] = codes;
    if (lane == 0) (which ? cVe : cKe)[dst] = int8_t(e);
  }
}

__global__ __launch_bounds__(256) void decode_rows(const int32_t* __restrict__ meta, const uint8_t* __restrict__ cK,
                                                   const uint8_t* __restrict__ cV, const int8_t* __restrict__ cKe,
                                                   const int8_t* __restrict__ cVe, uint16_t* __restrict__ sK,
                                                   uint16_t* __restrict__ sV, int npad, int64_t slots, int bh, int count) {
  constexpr int D = 128;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= count) return;
  const int64_t src = int64_t(bh) * slots + meta[bh * 4 + 0] + row;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const uint16_t codes = reinterpret_cast<const uint16_t*>((which ? cV : cK) + src * D)[lane];
    const float sc = pow2_f32((which ? cVe : cKe)[src]);
    // a code times a power of two has four significant bits: exact in bf16
    const float v0 = Elem<uint8_t>::to_f32(uint8_t(codes & 0xFF)) * sc, v1 = Elem<uint8_t>::to_f32(uint8_t(codes >> 8)) * sc;
    reinterpret_cast<uint32_t*>((which ? sV : sK) + (int64_t(bh) * npad + row) * D)[lane] =
        (__float_as_uint(v0) >> 16) | (__float_as_uint(v1) & 0xFFFF0000u);
  }
}

}  // namespace

hipError_t launch_encode_layer(d2o_ctx* c, int layer, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int bh = cf.batch * cf.n_kv_heads;
  int max_rows = 1;
  for (const auto& mt : c->layers[layer].meta) max_rows = std::max(max_rows, mt.budget);
  encode_rows<<<dim3((max_rows + 3) / 4, bh), 256, 0, s>>>(
      c->ccount + size_t(layer) * bh, c->meta + size_t(layer) * bh * 4, (const uint16_t*)c->st_K, (const uint16_t*)c->st_V,
      (uint8_t*)c->cacheK, (uint8_t*)c->cacheV, c->cKe, c->cVe, c->npad, cf.slots_per_seq, 0, -1);
  return hipGetLastError();
}

hipError_t launch_encode_head(d2o_ctx* c, int layer, int b, int hk, int count, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int bh = cf.batch * cf.n_kv_heads;
  if (count < 1) return hipSuccess;
  encode_rows<<<dim3((count + 3) / 4, 1), 256, 0, s>>>(
      c->ccount + size_t(layer) * bh, c->meta + size_t(layer) * bh * 4, (const uint16_t*)c->st_K, (const uint16_t*)c->st_V,
      (uint8_t*)c->cacheK, (uint8_t*)c->cacheV, c->cKe, c->cVe, c->npad, cf.slots_per_seq, b * cf.n_kv_heads + hk, count);
  return hipGetLastError();
}

hipError_t launch_decode_head(d2o_ctx* c, int layer, int b, int hk, int count, hipStream_t s) {
  const d2o_config& cf = c->cfg;
  const int bh = cf.batch * cf.n_kv_heads;
  if (count < 1) return hipSuccess;
  decode_rows<<<dim3((count + 3) / 4), 256, 0, s>>>(c->meta + size_t(layer) * bh * 4, (const uint8_t*)c->cacheK,
                                                    (const uint8_t*)c->cacheV, c->cKe, c->cVe, (uint16_t*)c->st_K,
                                                    (uint16_t*)c->st_V, c->npad, cf.slots_per_seq,
                                                    b * cf.n_kv_heads + hk, count);
  return hipGetLastError();
}

}  // namespace d2o
