// One page list per (KV head, query page) (paper Sec. 4.2: the votes of a query page's
// tokens pick that page's own top-K key pages).  The attention kernels need three
// things that the lists do not give directly, all derived here on the device, once per
// call, without atomics on anything that reaches a result:
//   * the union of a KV head's lists (ascending): the pages whose K/V images the forward
//     lays out, and the pages that one dK/dV workgroup each owns;
//   * for every list entry its position in that union (where the forward finds its image);
//   * for every union page the query pages whose list holds it (inverse lists, CSR,
//     ascending), cut into dK/dV work units of at most QP_SLICE query pages; a page cut
//     into several units gets partial-sum slots, added to the pool in a fixed order.  The
//     unit table is ordered by the first query page of the units (in windows of QP_SLICE),
//     so that workgroups running at the same time walk rows of neighbouring query pages.
// One workgroup per KV head; its phases are separated by workgroup barriers.
#include "common.h"
#include "launch.h"

namespace oomb {

constexpr int QP_THREADS = 1024;
#ifndef OOMB_QP_SLICE
#define OOMB_QP_SLICE 8
#endif
constexpr int QP_SLICE = OOMB_QP_SLICE;  // query pages per dK/dV work unit (at most 64: they are held in one register)

struct QpLayout {
  int32_t un_cap, max_units, max_pslots, max_multi;
  size_t off_cnt, off_fill, off_slot, off_un, off_uncnt, off_invoff, off_invqp, off_units, off_ucnt, off_pbase, off_ns;
  size_t off_multi, off_mcnt;
  size_t bytes;
};

static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

QpLayout qp_layout(const Params& p, int32_t stride) {
  QpLayout L{};
  const int64_t entries = (int64_t)p.m * stride;
  L.un_cap = (int32_t)(entries < p.n ? entries : p.n);
  L.max_units = (int32_t)(L.un_cap + entries / QP_SLICE + 1);
  // a page held by c > QP_SLICE lists is cut into ceil(c / QP_SLICE) < 2 c / QP_SLICE units
  L.max_pslots = (int32_t)(2 * entries / QP_SLICE + 1);
  L.max_multi = (int32_t)(entries / (QP_SLICE + 1) + 1);  // such a page is held by more than QP_SLICE lists
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o += up256(bytes); return at; };
  L.off_cnt = take((size_t)p.Hkv * p.n * 4);
  L.off_fill = take((size_t)p.Hkv * L.un_cap * 4);
  L.off_slot = take((size_t)p.Hkv * entries * 4);
  L.off_un = take((size_t)p.Hkv * L.un_cap * 4);
  L.off_uncnt = take((size_t)p.Hkv * 4);
  L.off_invoff = take((size_t)p.Hkv * (L.un_cap + 1) * 4);
  L.off_invqp = take((size_t)p.Hkv * entries * 4);
  L.off_units = take((size_t)p.Hkv * L.max_units * 16);
  L.off_ucnt = take((size_t)p.Hkv * 4);
  L.off_pbase = take((size_t)p.Hkv * L.un_cap * 4);
  L.off_ns = take((size_t)p.Hkv * L.un_cap * 4);
  L.off_multi = take((size_t)p.Hkv * L.max_multi * 4);
  L.off_mcnt = take((size_t)p.Hkv * 4);
  L.bytes = o;
  return L;
}

size_t qp_maps_bytes(const Params& p, int32_t stride) { return qp_layout(p, stride).bytes; }
int32_t qp_union_cap(const Params& p, int32_t stride) { return qp_layout(p, stride).un_cap; }
int32_t qp_max_units(const Params& p, int32_t stride) { return qp_layout(p, stride).max_units; }
int32_t qp_max_pslots(const Params& p, int32_t stride) { return qp_layout(p, stride).max_pslots; }
int32_t qp_max_multi(const Params& p, int32_t stride) { return qp_layout(p, stride).max_multi; }

// exclusive prefix of v over the workgroup's threads (thread order) and the total; two barriers
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t* wave_tot, int32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int32_t t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int32_t before = 0, all = 0;
  for (int w = 0; w < QP_THREADS / 64; ++w) {
    const int32_t t = wave_tot[w];
    if (w < wave) before += t;
    all += t;
  }
  total = all;
  __syncthreads();
  return before + inc - v;
}

__global__ __launch_bounds__(QP_THREADS) void qp_prepare_kernel(Params p, int32_t* __restrict__ cnt_all,
                                                                int32_t* __restrict__ fill_all, int32_t* __restrict__ slot_all,
                                                                int32_t* __restrict__ un_all, int32_t* __restrict__ uncnt,
                                                                int32_t* __restrict__ invoff_all, int32_t* __restrict__ invqp_all,
                                                                int4* __restrict__ units_all, int32_t* __restrict__ ucnt,
                                                                int32_t* __restrict__ pbase_all, int32_t* __restrict__ ns_all,
                                                                int32_t* __restrict__ multi_all, int32_t* __restrict__ mcnt,
                                                                int32_t max_pslots) {
  __shared__ int32_t wave_tot[QP_THREADS / 64];
  const int g = blockIdx.x, tid = threadIdx.x;
  const int32_t n = (int32_t)p.n, m = p.m, stride = p.sel_stride;
  const int32_t entries = m * stride;
  int32_t* cnt = cnt_all + (int64_t)g * n;
  int32_t* fill = fill_all + (int64_t)g * p.un_stride;
  int32_t* slot = slot_all + (int64_t)g * entries;
  int32_t* un = un_all + (int64_t)g * p.un_stride;
  int32_t* invoff = invoff_all + (int64_t)g * (p.un_stride + 1);
  int32_t* invqp = invqp_all + (int64_t)g * entries;
  int4* units = units_all + (int64_t)g * p.max_units;
  int32_t* pbase = pbase_all + (int64_t)g * p.un_stride;
  int32_t* ns_out = ns_all + (int64_t)g * p.un_stride;
  int32_t* multi = multi_all + (int64_t)g * p.max_multi;
  const int32_t* sel = p.sel + (int64_t)g * entries;
  const int32_t* sel_count = p.sel_count + (int64_t)g * m;

  // 1. how many lists hold each logical page
  for (int32_t l = tid; l < n; l += QP_THREADS) cnt[l] = 0;
  for (int32_t u = tid; u < p.un_stride; u += QP_THREADS) fill[u] = 0;
  __syncthreads();
  for (int32_t e = tid; e < entries; e += QP_THREADS) {
    const int32_t tau = e / stride, j = e - tau * stride;
    if (j < sel_count[tau]) {
      const int32_t l = sel[e];
      if (l >= 0 && l < n) atomicAdd(&cnt[l], 1);  // integer counts: the result does not depend on the order
    }
  }
  __syncthreads();

  // 2. union list and CSR offsets: every thread takes a run of consecutive logical pages
  const int32_t per = (n + QP_THREADS - 1) / QP_THREADS;
  const int32_t l0 = tid * per < n ? tid * per : n, l1 = l0 + per < n ? l0 + per : n;
  int32_t my_used = 0, my_ent = 0;
  for (int32_t l = l0; l < l1; ++l) {
    const int32_t c = cnt[l];
    my_used += c > 0;
    my_ent += c;
  }
  int32_t n_un, n_ent;
  int32_t u_at = block_exclusive_scan(my_used, wave_tot, n_un);
  int32_t e_at = block_exclusive_scan(my_ent, wave_tot, n_ent);
  for (int32_t l = l0; l < l1; ++l) {
    const int32_t c = cnt[l];
    if (c > 0) {
      un[u_at] = l;
      invoff[u_at] = e_at;
      cnt[l] = u_at;  // from here on: position of the page in the union
      ++u_at;
      e_at += c;
    }
  }
  if (tid == 0) {
    invoff[n_un] = n_ent;
    uncnt[g] = n_un;
  }
  __syncthreads();

  // 3. position of every list entry in the union; inverse lists filled query page by query page, so
  //    that they come out ascending (the entries of one list are distinct pages: no two threads of a
  //    round touch the same counter)
  for (int32_t tau = 0; tau < m; ++tau) {
    const int32_t len = sel_count[tau];
    for (int32_t j = tid; j < stride; j += QP_THREADS) {
      int32_t s = 0;  // (entries that are not page ids are ignored; their position is never used for a result)
      const int32_t l = j < len ? sel[tau * stride + j] : -1;
      if (l >= 0 && l < n) {
        s = cnt[l];
        const int32_t k = fill[s];
        fill[s] = k + 1;
        invqp[invoff[s] + k] = tau;
      }
      slot[tau * stride + j] = s;
    }
    __syncthreads();
  }

  // 4. dK/dV work units: union entry u with c query pages -> ceil(c / QP_SLICE) units
  const int32_t per_u = (n_un + QP_THREADS - 1) / QP_THREADS;
  const int32_t u0 = tid * per_u < n_un ? tid * per_u : n_un, u1 = u0 + per_u < n_un ? u0 + per_u : n_un;
  int32_t my_units = 0, my_slots = 0, my_multi = 0;
  for (int32_t u = u0; u < u1; ++u) {
    const int32_t ns = (invoff[u + 1] - invoff[u] + QP_SLICE - 1) / QP_SLICE;
    my_units += ns;
    my_slots += ns > 1 ? ns : 0;
    my_multi += ns > 1;
  }
  int32_t n_units_all, n_slots, n_multi;
  (void)block_exclusive_scan(my_units, wave_tot, n_units_all);
  int32_t s_at = block_exclusive_scan(my_slots, wave_tot, n_slots);
  int32_t m_at = block_exclusive_scan(my_multi, wave_tot, n_multi);
  for (int32_t u = u0; u < u1; ++u) {
    const int32_t c = invoff[u + 1] - invoff[u];
    const int32_t ns = (c + QP_SLICE - 1) / QP_SLICE;
    pbase[u] = ns > 1 ? g * max_pslots + s_at : -1;
    ns_out[u] = ns;
    if (ns > 1) {
      s_at += ns;
      multi[m_at++] = u;
    }
  }
  // the unit table, ordered by the window (QP_SLICE consecutive query pages) that holds a unit's first
  // query page, then by page: workgroups that run at the same time start on rows of the same few query
  // pages.  One scan per window.
  int32_t n_units = 0;
  const int32_t windows = (m + QP_SLICE - 1) / QP_SLICE;
  for (int32_t win = 0; win < windows; ++win) {
    int32_t mine = 0;
    for (int32_t u = u0; u < u1; ++u) {
      const int32_t c = invoff[u + 1] - invoff[u];
      for (int32_t q0 = 0; q0 < c; q0 += QP_SLICE) mine += invqp[invoff[u] + q0] / QP_SLICE == win;
    }
    int32_t total;
    int32_t k_at = n_units + block_exclusive_scan(mine, wave_tot, total);
    for (int32_t u = u0; u < u1; ++u) {
      const int32_t c = invoff[u + 1] - invoff[u];
      for (int32_t q0 = 0, sl = 0; q0 < c; q0 += QP_SLICE, ++sl) {
        if (invqp[invoff[u] + q0] / QP_SLICE != win) continue;
        const int32_t qc = c - q0 < QP_SLICE ? c - q0 : QP_SLICE;
        units[k_at++] = make_int4(u, q0, qc, pbase[u] >= 0 ? pbase[u] + sl : -1);
      }
    }
    n_units += total;
  }
  if (tid == 0) {
    ucnt[g] = n_units;
    mcnt[g] = n_multi;
  }
}

// Points the maps of `p` into the workspace block `ws` (qp_maps_bytes long) and enqueues the kernel
// that fills them.  p.sel / p.sel_count / p.sel_stride must be set.
hipError_t launch_qp_prepare(Params& p, void* ws, hipStream_t st) {
  const QpLayout L = qp_layout(p, p.sel_stride);
  unsigned char* b = (unsigned char*)ws;
  p.qp = 1;
  p.un_stride = L.un_cap;
  p.max_units = L.max_units;
  p.qp_slot = (const int32_t*)(b + L.off_slot);
  p.un_list = (const int32_t*)(b + L.off_un);
  p.un_count = (const int32_t*)(b + L.off_uncnt);
  p.inv_off = (const int32_t*)(b + L.off_invoff);
  p.inv_qp = (const int32_t*)(b + L.off_invqp);
  p.units = (const int4*)(b + L.off_units);
  p.unit_count = (const int32_t*)(b + L.off_ucnt);
  p.un_pbase = (const int32_t*)(b + L.off_pbase);
  p.un_ns = (const int32_t*)(b + L.off_ns);
  p.multi_list = (const int32_t*)(b + L.off_multi);
  p.multi_count = (const int32_t*)(b + L.off_mcnt);
  p.max_multi = L.max_multi;
  ProfScope prof_("qp_prepare", st);
  qp_prepare_kernel<<<dim3((unsigned)p.Hkv), dim3(QP_THREADS), 0, st>>>(
      p, (int32_t*)(b + L.off_cnt), (int32_t*)(b + L.off_fill), (int32_t*)(b + L.off_slot), (int32_t*)(b + L.off_un),
      (int32_t*)(b + L.off_uncnt), (int32_t*)(b + L.off_invoff), (int32_t*)(b + L.off_invqp), (int4*)(b + L.off_units),
      (int32_t*)(b + L.off_ucnt), (int32_t*)(b + L.off_pbase), (int32_t*)(b + L.off_ns), (int32_t*)(b + L.off_multi),
      (int32_t*)(b + L.off_mcnt), L.max_pslots);
  return hipGetLastError();
}

}  // namespace oomb
