// Constrained-decoding mask (Section 4.5, last sentence of the error analysis: mask out the
// registers that are occupied while the allocation is generated): for the occurrence a
// decoder has reached, the bases that keep consistency, realizability and safety
// (Section 3.4) intact against the occurrences already emitted.  One workgroup per query;
// P(i) is rebuilt from the analysis' event stream the way the verifier's pair search does.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

#include "vl_dev.h"

using namespace vl;

namespace {

struct DevQuery {
  const DevMir *mir;
  const DevLive *live;
  const uint16_t *cand;
  uint32_t occ, pad;
};

__global__ __launch_bounds__(256) void k_free_bases(const DevQuery *__restrict__ queries, uint32_t *__restrict__ masks) {
  const DevQuery &Q = queries[blockIdx.x];
  const DevMir VL_GLOBAL &m = *as_global(Q.mir);
  const DevLive VL_GLOBAL &L = *as_global(Q.live);
  const uint16_t *row = Q.cand;
  uint32_t *out = masks + (size_t)blockIdx.x * 16;
  extern __shared__ uint32_t in_p[];   // [W] members of P(i)
  __shared__ uint32_t blocked[17];     // registers that are taken or reserved (word 16: always zero)
  const uint32_t q = Q.occ, v = m.occ_vreg[q], i = m.occ_instr[q];
  const uint32_t attr = m.vattr[v], cls = attr_class(attr), width = attr_width(attr), align = attr_align(attr);
  const uint32_t F = m.class_size[cls];
  const uint32_t first_v = L.first[v];
  for (uint32_t x = threadIdx.x; x < m.W; x += blockDim.x) in_p[x] = 0;
  if (threadIdx.x < 17) blocked[threadIdx.x] = (threadIdx.x < 16 && m.has_reserved) ? m.reserved[cls][threadIdx.x] : 0u;
  __syncthreads();
  if (first_v >= q) {   // the first mention of v: everything in P(i) that already has a register is in the way
    flip_members_of_p(m, L, i, in_p, threadIdx.x, blockDim.x);
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < m.V; b += blockDim.x) {   // one vreg per lane
      if (!((in_p[b >> 5] >> (b & 31)) & 1u)) continue;
      const uint32_t ab = m.vattr[b], fb = L.first[b];
      if (b == v || attr_class(ab) != cls || fb >= q) continue;
      const uint32_t pb = row[fb], wb = attr_width(ab);
      for (uint32_t r = pb; r < pb + wb && r < 512u; ++r) atomicOr(&blocked[r >> 5], 1u << (r & 31));
    }
    __syncthreads();
  }
  const uint32_t forced = first_v < q ? (uint32_t)row[first_v] : kNone;   // a later mention: only its own register
  const uint32_t wm = width == 32 ? 0xFFFFFFFFu : ((1u << width) - 1u);
  for (uint32_t p = threadIdx.x; p < 512u; p += blockDim.x) {
    const uint64_t window = ((uint64_t)blocked[p >> 5] | ((uint64_t)blocked[(p >> 5) + 1] << 32)) >> (p & 31);
    bool ok = p % align == 0 && p + width <= F && ((uint32_t)window & wm) == 0;
    if (forced != kNone && p != forced) ok = false;
    const uint64_t ballot = __ballot(ok);
    // a wavefront covers 64 consecutive bases: two words of the mask
    if ((threadIdx.x & 63u) == 0) { out[p >> 5] = (uint32_t)ballot; out[(p >> 5) + 1] = (uint32_t)(ballot >> 32); }
  }
}

// the query table on the device, one per device; reused from call to call
struct Table {
  std::mutex mu;
  DevQuery *dev = nullptr;
  DevQuery *host = nullptr;   // pinned
  uint32_t cap = 0;
  hipEvent_t consumed = nullptr;   // recorded after the kernel that reads the table
};
Table g_table[16];

}  // namespace

extern "C" int32_t vl_free_bases_multi(const vl_mask_query *queries, uint32_t n, uint32_t *masks, vl_stream stream_) {
  if (!queries || !masks) return VL_E_NULL;
  if (n == 0) return VL_E_SHAPE;
  uint32_t max_w = 1;
  for (uint32_t j = 0; j < n; ++j) {
    const vl_mask_query &u = queries[j];
    if (!u.mir || !u.live || !u.cand) return VL_E_NULL;
    if (u.mir->magic != kMirMagic || u.live->magic != kLiveMagic || u.live->mir != u.mir || u.reserved0 != 0 || u.mir->lowered) return VL_E_ARG;
    if (u.occ >= u.mir->h.O) return VL_E_SHAPE;
    max_w = std::max(max_w, u.mir->h.W);
  }
  hipStream_t stream = (hipStream_t)stream_;
  int device = 0;
  VL_HIP(hipGetDevice(&device));
  if (device < 0 || device >= 16) return VL_E_ARG;
  Table &t = g_table[device];
  std::lock_guard<std::mutex> lock(t.mu);
  // the previous call's kernel must have read the table before it is overwritten
  if (t.consumed) VL_HIP(hipEventSynchronize(t.consumed));
  if (t.cap < n) {
    if (t.dev) (void)hipFree(t.dev);
    if (t.host) (void)hipHostFree(t.host);
    t.dev = nullptr; t.host = nullptr; t.cap = 0;
    const uint32_t cap = std::max(1024u, n);
    VL_HIP(hipMalloc((void **)&t.dev, (size_t)cap * sizeof(DevQuery)));
    VL_HIP(hipHostMalloc((void **)&t.host, (size_t)cap * sizeof(DevQuery), hipHostMallocDefault));
    if (!t.consumed) VL_HIP(hipEventCreateWithFlags(&t.consumed, hipEventDisableTiming));
    t.cap = cap;
  }
  for (uint32_t j = 0; j < n; ++j) {
    DevQuery &d = t.host[j];
    d.mir = queries[j].mir->dev; d.live = queries[j].live->dev; d.cand = queries[j].cand; d.occ = queries[j].occ; d.pad = 0;
  }
  VL_HIP(hipMemcpyAsync(t.dev, t.host, (size_t)n * sizeof(DevQuery), hipMemcpyHostToDevice, stream));
  k_free_bases<<<n, 128, (size_t)max_w * 4, stream>>>(t.dev, masks);
  VL_HIP(hipGetLastError());
  VL_HIP(hipEventRecord(t.consumed, stream));
  return VL_OK;
}
