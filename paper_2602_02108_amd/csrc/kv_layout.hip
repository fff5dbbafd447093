// Images of the selected K / V pages for the bf16 MFMA attention kernels (paper
// Sec. 4.2: every query tile of a chunk attends the same page list -- or, with one list
// per query page, lists drawn from one union -- so the pages are gathered through the
// page table and re-laid out once per call instead of once per query tile).  An image is one half page (64 tokens x 128 dims, 16 KiB) in exactly
// the byte order of the LDS tile that the kernels read, so that their staging is a
// plain copy:
//   natural:    token r, granule c (dims 8c .. 8c+7) at (r * 16 + (c ^ (r & 15))) * 16
//   transposed: row = dim d, granule o = 2u + hh holds tokens 16u + 4hh + {0..3, 8..11};
//               at (d * 8 + (o ^ ((d >> 1) & 7))) * 16
// Layout of the image buffer: [kind][KV head][half tile 0 .. 2 * max_len - 1], where
// half tile ht is keys 64 (ht % 2) .. + 63 of list entry ht / 2 and the kinds are the
// set bits of `kinds` in the order K natural, V natural, K transposed, V transposed.
#include "mfma_common.h"
#include "launch.h"

namespace oomb {

constexpr int KV_IMG = 16384;
enum { IMG_K_NAT = 1, IMG_V_NAT = 2, IMG_K_TR = 4, IMG_V_TR = 8 };

static inline int img_kind_count(int kinds) { return __builtin_popcount(kinds); }
// index of kind bit `bit` among the set bits of `kinds`
__host__ __device__ static inline int img_kind_index(int kinds, int bit) { return __builtin_popcount(kinds & (bit - 1)); }

size_t kv_image_bytes(const Params& p, int32_t max_len, int kinds) {
  return (size_t)img_kind_count(kinds) * (size_t)p.Hkv * (size_t)(2 * max_len) * KV_IMG;
}

// offset of the images of one kind and KV head
__host__ __device__ static inline size_t kv_image_base(int32_t Hkv, int32_t max_len, int kinds, int bit, int g) {
  return ((size_t)img_kind_index(kinds, bit) * Hkv + g) * (size_t)(2 * max_len) * KV_IMG;
}

__global__ __launch_bounds__(256) void kv_layout_kernel(Params p, int32_t max_len, int kinds,
                                                        unsigned char* __restrict__ img) {
  __shared__ __align__(16) unsigned char tile[64 * 272];  // 64 tokens x 128 bf16, rows padded by 16 bytes
  const int ht = blockIdx.x, g = blockIdx.y, is_v = blockIdx.z, tid = threadIdx.x;
  const int nat_bit = is_v ? IMG_V_NAT : IMG_K_NAT, tr_bit = is_v ? IMG_V_TR : IMG_K_TR;
  if (!(kinds & (nat_bit | tr_bit))) return;
  const int32_t j = ht >> 1;
  if (j >= owned_len(p, g)) return;
  const int64_t l = owned_at(p, g, j);
  const bf16_t* src = (is_v ? (const bf16_t*)p.v_pool : (const bf16_t*)p.k_pool) +
                      (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride +
                      (int64_t)(ht & 1) * 64 * p.pool_tok_stride;
  unsigned char* out_nat = img + kv_image_base(p.Hkv, max_len, kinds, nat_bit, g) + (size_t)ht * KV_IMG;
  unsigned char* out_tr = img + kv_image_base(p.Hkv, max_len, kinds, tr_bit, g) + (size_t)ht * KV_IMG;
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int gi = tid + 256 * x, r = gi >> 4, cg = gi & 15;
    const uint4 v = *reinterpret_cast<const uint4*>(src + (int64_t)r * p.pool_tok_stride + 8 * cg);
    *reinterpret_cast<uint4*>(tile + r * 272 + cg * 16) = v;
    if (kinds & nat_bit) *reinterpret_cast<uint4*>(out_nat + (r * 16 + (cg ^ (r & 15))) * 16) = v;
  }
  if (!(kinds & tr_bit)) return;
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
    *reinterpret_cast<uint4*>(out_tr + (d * 8 + (o ^ ((d >> 1) & 7))) * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

hipError_t launch_kv_layout(const Params& p, int32_t max_len, int kinds, void* img, hipStream_t st) {
  ProfScope prof_("kv_layout", st);
  kv_layout_kernel<<<dim3((unsigned)(2 * max_len), (unsigned)p.Hkv, 2), dim3(256), 0, st>>>(p, max_len, kinds,
                                                                                             (unsigned char*)img);
  return hipGetLastError();
}

}  // namespace oomb
