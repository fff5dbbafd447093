// Offloaded KV cache (paper Sec. 4.3): the K / V pools and their gradient pools live in
// pinned host memory; the pages a chunk attends are fetched into small device staging
// pools, the attention kernels run on those, and the gradients of the fetched pages are
// added back to the host pools.
//
// The copies are kernels that read (write) the pinned host memory directly over the
// host link with 16-byte accesses, tile by tile ((page, KV head) = P rows): the
// page list never leaves the device, so no host round trip sits between the selection
// and the transfer, and a fetch on its own stream overlaps whatever computes meanwhile.
// They run on a FEW workgroups that walk the tiles: host accesses take microseconds, and
// a grid that covers the chip fills the memory pipeline of every compute unit with them,
// which stalls a concurrently running kernel almost completely (measured: with 128 or more
// workgroups nothing overlaps); 12 workgroups of 256 threads already saturate the link (about
// 50 GB/s each way) and disturb only the compute units they sit on.
//   offload_plan       which KV heads hold each page (bit mask over the lists: one list per
//                      KV head, or one per KV head and query page) and the staging slot of
//                      every held page (ascending logical page order), one workgroup.  The
//                      slot table is the page table of the staging pools; it never points
//                      past their capacity (a page that does not fit gets slot 0 and the
//                      count of held pages tells the caller)
//   offload_fetch      stage[slot][g] = host[page_table[l]][g]  (K and V) for the held
//                      (page, head) tiles, optionally zeroing the gradient staging tiles
//   offload_writeback  host[page_table[l]][g] += stage[slot][g]  (dK and dV)
#include <cstdlib>

#include "common.h"
#include "launch.h"

namespace oomb {

constexpr int PLAN_THREADS = 1024;

// lists: p.sel [Hkv][lists_per_head][p.sel_stride], p.sel_count [Hkv][lists_per_head]
__global__ __launch_bounds__(PLAN_THREADS) void offload_plan_kernel(Params p, int32_t lists_per_head, int32_t stage_cap,
                                                                    int32_t* __restrict__ stage_table,
                                                                    int32_t* __restrict__ slot_pages,
                                                                    uint32_t* __restrict__ head_mask,
                                                                    int32_t* __restrict__ n_slots) {
  __shared__ int32_t wave_tot[PLAN_THREADS / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t n = (int32_t)p.n;
  for (int32_t l = tid; l < n; l += PLAN_THREADS) head_mask[l] = 0u;
  __syncthreads();
  const int32_t per_head = lists_per_head * p.sel_stride;
  for (int g = 0; g < p.Hkv; ++g)
    for (int32_t e = tid; e < per_head; e += PLAN_THREADS) {
      const int32_t q = e / p.sel_stride, j = e - q * p.sel_stride;
      if (j >= p.sel_count[g * lists_per_head + q]) continue;
      const int32_t l = p.sel[(int64_t)g * per_head + e];
      if (l >= 0 && l < n) atomicOr(&head_mask[l], 1u << g);  // (a bit set: independent of the order)
    }
  __syncthreads();
  // exclusive scan of "held" over the logical pages: every thread takes a run of consecutive pages
  const int32_t per = (n + PLAN_THREADS - 1) / PLAN_THREADS;
  const int32_t l0 = tid * per < n ? tid * per : n, l1 = l0 + per < n ? l0 + per : n;
  int32_t mine = 0;
  for (int32_t l = l0; l < l1; ++l) mine += head_mask[l] != 0u;
  int32_t inc = mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int32_t t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int32_t before = 0, total = 0;
  for (int w = 0; w < PLAN_THREADS / 64; ++w) {
    const int32_t t = wave_tot[w];
    if (w < wave) before += t;
    total += t;
  }
  int32_t at = before + inc - mine;
  for (int32_t l = l0; l < l1; ++l) {
    if (head_mask[l]) {
      stage_table[l] = at < stage_cap ? at : 0;
      if (at < stage_cap) slot_pages[at] = l;
      ++at;
    } else {
      stage_table[l] = -1;
    }
  }
  if (tid == 0) {
    n_slots[0] = total < stage_cap ? total : stage_cap;  // slots in use
    n_slots[1] = total;                                   // pages held: more than stage_cap = overflow
  }
}

// Tile (slot s, KV head g): P rows of D elements.  The workgroups walk the tiles with stride gridDim.x.
// MODE 0: fetch K and V (and zero the gradient staging tiles if given); MODE 1: add dK / dV back.
template <int MODE, typename TG>
__global__ __launch_bounds__(256) void offload_tile_kernel(Params p, const int32_t* __restrict__ slot_pages,
                                                           const uint32_t* __restrict__ head_mask,
                                                           const int32_t* __restrict__ n_slots, int32_t stage_cap,
                                                           unsigned char* __restrict__ a_host, unsigned char* __restrict__ b_host,
                                                           unsigned char* __restrict__ a_stage, unsigned char* __restrict__ b_stage,
                                                           unsigned char* __restrict__ ga_stage, unsigned char* __restrict__ gb_stage,
                                                           int es, int gs) {
  const int32_t slots = n_slots[0] < stage_cap ? n_slots[0] : stage_cap;
  for (int32_t tile = blockIdx.x; tile < slots * p.Hkv; tile += gridDim.x) {
    const int32_t slot = tile / p.Hkv;
    const int g = tile - slot * p.Hkv;
    const int32_t l = slot_pages[slot];
    if (l < 0 || l >= p.n || !((head_mask[l] >> g) & 1u)) continue;
    const int64_t h_off = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    const int64_t s_off = (int64_t)slot * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    if (MODE == 0) {
      const int gran = p.D * es / 16;  // 16-byte granules per token row
      for (int x = threadIdx.x; x < p.P * gran; x += 256) {
        const int t = x / gran, c = x - t * gran;
        const int64_t ho = (h_off + (int64_t)t * p.pool_tok_stride) * es + 16 * c;
        const int64_t so = (s_off + (int64_t)t * p.pool_tok_stride) * es + 16 * c;
        *reinterpret_cast<uint4*>(a_stage + so) = *reinterpret_cast<const uint4*>(a_host + ho);
        *reinterpret_cast<uint4*>(b_stage + so) = *reinterpret_cast<const uint4*>(b_host + ho);
      }
      if (ga_stage) {
        const int ggran = p.D * gs / 16;
        for (int x = threadIdx.x; x < p.P * ggran; x += 256) {
          const int t = x / ggran, c = x - t * ggran;
          const int64_t so = (s_off + (int64_t)t * p.pool_tok_stride) * gs + 16 * c;
          *reinterpret_cast<uint4*>(ga_stage + so) = make_uint4(0, 0, 0, 0);
          *reinterpret_cast<uint4*>(gb_stage + so) = make_uint4(0, 0, 0, 0);
        }
      }
    } else {
      constexpr int EPG = 16 / (int)sizeof(TG);  // elements per granule
      const int ggran = p.D / EPG;
      for (int x = threadIdx.x; x < p.P * ggran; x += 256) {
        const int t = x / ggran, c = x - t * ggran;
        const int64_t ho = h_off + (int64_t)t * p.pool_tok_stride + EPG * c;
        const int64_t so = s_off + (int64_t)t * p.pool_tok_stride + EPG * c;
#pragma unroll
        for (int which = 0; which < 2; ++which) {
          TG* hp = (TG*)(which ? b_host : a_host) + ho;
          const TG* sp = (const TG*)(which ? b_stage : a_stage) + so;
          uint4 hv = *reinterpret_cast<const uint4*>(hp);
          const uint4 sv = *reinterpret_cast<const uint4*>(sp);
          TG* he = reinterpret_cast<TG*>(&hv);
          const TG* se = reinterpret_cast<const TG*>(&sv);
#pragma unroll
          for (int e = 0; e < EPG; ++e) {
            float sum = Elem<TG>::load(he + e) + Elem<TG>::load(se + e);
            Elem<TG>::store(he + e, sum);
          }
          *reinterpret_cast<uint4*>(hp) = hv;
        }
      }
    }
  }
}

// A pointer the device can dereference: device memory, or host memory that the runtime has
// pinned and mapped.  Returns nullptr for anything else (so that nothing is launched on it).
void* device_view(const void* ptr) {
  if (!ptr) return nullptr;
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, ptr) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  if (attr.type != hipMemoryTypeHost && attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) return nullptr;
  return attr.devicePointer;
}

// workgroups of a transfer kernel (OOMB_OFFLOAD_WGS overrides the default, for experiments)
static unsigned transfer_wgs(int64_t tiles) {
  static int v = 0;
  if (!v) {
    const char* e = std::getenv("OOMB_OFFLOAD_WGS");
    v = e ? std::atoi(e) : 12;
    if (v < 1) v = 12;
  }
  return (unsigned)(tiles < v ? (tiles > 0 ? tiles : 1) : v);
}

hipError_t launch_offload_plan(const Params& p, int32_t lists_per_head, int32_t stage_cap, int32_t* stage_table,
                               int32_t* slot_pages, uint32_t* head_mask, int32_t* n_slots, hipStream_t st) {
  ProfScope prof_("offload_plan", st);
  offload_plan_kernel<<<dim3(1), dim3(PLAN_THREADS), 0, st>>>(p, lists_per_head, stage_cap, stage_table, slot_pages, head_mask,
                                                              n_slots);
  return hipGetLastError();
}

hipError_t launch_offload_fetch(const Params& p, bool is_bf16, const int32_t* slot_pages, const uint32_t* head_mask,
                                const int32_t* n_slots, int32_t stage_cap, void* host_k, void* host_v, void* stage_k,
                                void* stage_v, void* stage_dk, void* stage_dv, hipStream_t st) {
  ProfScope prof_("offload_fetch", st);
  offload_tile_kernel<0, float><<<dim3(transfer_wgs((int64_t)stage_cap * p.Hkv)), dim3(256), 0, st>>>(
      p, slot_pages, head_mask, n_slots, stage_cap, (unsigned char*)host_k, (unsigned char*)host_v, (unsigned char*)stage_k,
      (unsigned char*)stage_v, (unsigned char*)stage_dk, (unsigned char*)stage_dv, is_bf16 ? 2 : 4, p.grad_is_bf16 ? 2 : 4);
  return hipGetLastError();
}

hipError_t launch_offload_writeback(const Params& p, const int32_t* slot_pages, const uint32_t* head_mask,
                                    const int32_t* n_slots, int32_t stage_cap, void* stage_dk, void* stage_dv, void* host_dk,
                                    void* host_dv, hipStream_t st) {
  ProfScope prof_("offload_writeback", st);
  dim3 grid(transfer_wgs((int64_t)stage_cap * p.Hkv));
  if (p.grad_is_bf16)
    offload_tile_kernel<1, bf16_t><<<grid, dim3(256), 0, st>>>(p, slot_pages, head_mask, n_slots, stage_cap,
                                                               (unsigned char*)host_dk, (unsigned char*)host_dv,
                                                               (unsigned char*)stage_dk, (unsigned char*)stage_dv, nullptr, nullptr, 2, 2);
  else
    offload_tile_kernel<1, float><<<grid, dim3(256), 0, st>>>(p, slot_pages, head_mask, n_slots, stage_cap,
                                                              (unsigned char*)host_dk, (unsigned char*)host_dv,
                                                              (unsigned char*)stage_dk, (unsigned char*)stage_dv, nullptr, nullptr, 4, 4);
  return hipGetLastError();
}

}  // namespace oomb
