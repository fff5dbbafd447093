// Images of the selected K / V pages for the bf16 MFMA forward kernel (paper Sec. 4.2:
// every query tile of a chunk attends the same page list -- or, with one list per query
// page, lists drawn from one union -- so the pages are gathered through the page table and
// re-laid out once per call instead of once per query tile).  An image is one half page
// (64 tokens x 128 dims, 16 KiB) in exactly the byte order of the LDS tile that the kernel
// reads, so that its staging is a plain copy:
//   K, natural:    token r, granule c (dims 8c .. 8c+7) at (r * 16 + (c ^ (r & 15))) * 16
//   V, transposed: row = dim d, granule o = 2u + hh holds tokens 16u + 4hh + {0..3, 8..11};
//                  at (d * 8 + (o ^ ((d >> 1) & 7))) * 16
// Layout of the image buffer: [K | V][KV head][half tile 0 .. 2 * max_len - 1], where half
// tile ht is keys 64 (ht % 2) .. + 63 of list entry ht / 2.
#include "mfma_common.h"
#include "launch.h"

namespace oomb {

constexpr int KV_IMG = 16384;

size_t kv_image_bytes(const Params& p, int32_t max_len) {
  return 2 * (size_t)p.Hkv * (size_t)(2 * max_len) * KV_IMG;
}

__global__ __launch_bounds__(256) void kv_layout_kernel(Params p, int32_t max_len, unsigned char* __restrict__ img) {
  __shared__ __align__(16) unsigned char tile[64 * 272];  // 64 tokens x 128 bf16, rows padded by 16 bytes
  const int ht = blockIdx.x, g = blockIdx.y, is_v = blockIdx.z, tid = threadIdx.x;
  const int32_t j = ht >> 1;
  if (j >= owned_len(p, g)) return;
  const int64_t l = owned_at(p, g, j);
  const bf16_t* src = (is_v ? (const bf16_t*)p.v_pool : (const bf16_t*)p.k_pool) +
                      (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride +
                      (int64_t)(ht & 1) * 64 * p.pool_tok_stride;
  unsigned char* out = img + (((size_t)is_v * p.Hkv + g) * (size_t)(2 * max_len) + ht) * KV_IMG;
  if (!is_v) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int gi = tid + 256 * x, r = gi >> 4, cg = gi & 15;
      const uint4 v = *reinterpret_cast<const uint4*>(src + (int64_t)r * p.pool_tok_stride + 8 * cg);
      *reinterpret_cast<uint4*>(out + (r * 16 + (cg ^ (r & 15))) * 16) = v;
    }
    return;
  }
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int gi = tid + 256 * x, r = gi >> 4, cg = gi & 15;
    *reinterpret_cast<uint4*>(tile + r * 272 + cg * 16) =
        *reinterpret_cast<const uint4*>(src + (int64_t)r * p.pool_tok_stride + 8 * cg);
  }
  __syncthreads();
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int gi = tid + 256 * x, d = gi >> 3, o = gi & 7, u = o >> 1, h2 = o & 1;
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const int r0 = 16 * u + 4 * h2 + ((2 * e2) & 3) + 8 * ((2 * e2) >> 2);
      const uint32_t lo = *reinterpret_cast<const unsigned short*>(tile + r0 * 272 + d * 2);
      const uint32_t hi = *reinterpret_cast<const unsigned short*>(tile + (r0 + 1) * 272 + d * 2);
      w[e2] = lo | (hi << 16);
    }
    *reinterpret_cast<uint4*>(out + (d * 8 + (o ^ ((d >> 1) & 7))) * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

hipError_t launch_kv_layout(const Params& p, int32_t max_len, void* img, hipStream_t st) {
  ProfScope prof_("kv_layout", st);
  kv_layout_kernel<<<dim3((unsigned)(2 * max_len), (unsigned)p.Hkv, 2), dim3(256), 0, st>>>(p, max_len, (unsigned char*)img);
  return hipGetLastError();
}

}  // namespace oomb
