// Liveness analysis on the GPU, batched over kernels (one grid slice per kernel).
//
// Pipeline (every step is a kernel below; the host only sizes buffers):
//   1. group operand occurrences by vreg, ascending (count / scan / place / sort)
//   2. per-block use and def bitsets from the first mention of each vreg in a block
//   3. backward dataflow to the least fixed point, one bitset word per lane
//   4. per occurrence: liveness after its instruction, kill flag, and its role in
//      the verifier's event stream
//   5. count, scan and write the event stream, the live intervals and the
//      per-tile live-in lists; optionally the dense per-point bitsets
// The paper defers this to "following the control and data dependency"
// (Section 4.6); the dataflow equations are the textbook ones its Safety
// condition (Section 3.4) needs to know which lifetimes overlap.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "vl_dev.h"

using namespace vl;

#define MIRS const DevMir *const *__restrict__ mirs, DevLive *__restrict__ lives

namespace {

template <class P> __device__ inline bool bit_get(P row, uint32_t v) { return (row[v >> 5] >> (v & 31)) & 1u; }

// first index in [lo,hi) with a[idx] >= key
template <class P> __device__ inline uint32_t lower_bound(P a, uint32_t lo, uint32_t hi, uint32_t key) {
  while (lo < hi) {
    uint32_t mid = (lo + hi) >> 1;
    if (a[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// ---- 1. occurrences grouped by vreg -------------------------------------------------
constexpr uint32_t kSlice = 8192;   // occurrences per workgroup in the counting kernels

// Occurrences per vreg.  A few vregs (base addresses, accumulators) are mentioned
// thousands of times, so each workgroup first counts its slice in an LDS histogram and
// then adds the non-zero bins to the global counters once.
template <bool kLds>
__global__ __launch_bounds__(1024) void k_count(MIRS) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  extern __shared__ uint32_t sm[];
  const uint32_t o0 = blockIdx.x * kSlice;
  if (o0 >= m.O) return;
  const uint32_t o1 = min(m.O, o0 + kSlice);
  if (!kLds) {
    for (uint32_t o = o0 + threadIdx.x; o < o1; o += 1024) atomicAdd(&L.vcnt[m.occ_vreg[o]], 1u);
    return;
  }
  for (uint32_t v = threadIdx.x; v < m.V; v += 1024) sm[v] = 0;
  __syncthreads();
  for (uint32_t o = o0 + threadIdx.x; o < o1; o += 1024) atomicAdd(&sm[m.occ_vreg[o]], 1u);
  __syncthreads();
  for (uint32_t v = threadIdx.x; v < m.V; v += 1024)
    if (sm[v]) atomicAdd(&L.vcnt[v], sm[v]);
}

constexpr uint32_t kShortList = 16;   // longer occurrence lists go to the bitmap sort

enum { kScanVreg = 0, kScanItems = 1, kScanSeg = 2, kScanSeed = 3 };   // kScanSeg: per-entry run counts

// In-place exclusive scan of p[0..n), total to p[n]; one 1024-thread block per kernel.
// (The array is chosen at compile time: a run-time switch over the four arrays was
// seen to pick the wrong pointer in its default branch.)
template <int kWhich>
__device__ inline void f_scan(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L) {
  uint32_t VL_GLOBAL *p = kWhich == kScanVreg ? L.vcnt : kWhich == kScanItems ? L.item_off : kWhich == kScanSeg ? L.ent_seg : L.seed_off;
  const uint32_t n = kWhich == kScanVreg ? m.V : kWhich == kScanItems ? m.N + m.B : kWhich == kScanSeg ? m.O : L.T;
  // Each of the 16 wavefronts owns a contiguous sixteenth of the array and walks it 256
  // elements at a time (four consecutive elements per lane, one 16-byte access): first to
  // total its part, then, once the parts' totals are prefixed, to write the exclusive sums.
  __shared__ uint32_t part[16];
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t per = ((n + 15u) / 16u + 255u) & ~255u;
  const uint32_t lo = min(n, wave * per), hi = min(n, lo + per);
  auto load4 = [&](uint32_t i) {
    u32x4 x = 0;
    if (i + 4 <= hi) x = *reinterpret_cast<const u32x4 VL_GLOBAL *>(p + i);
    else {
      if (i < hi) x.x = p[i];
      if (i + 1 < hi) x.y = p[i + 1];
      if (i + 2 < hi) x.z = p[i + 2];
    }
    return x;
  };
  uint32_t sum = 0;
  for (uint32_t i = lo + lane * 4; i < hi; i += 4 * 256) {   // four reads in flight
    u32x4 x[4];
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) x[u] = load4(i + u * 256);   // zeros beyond hi
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) sum += x[u].x + x[u].y + x[u].z + x[u].w;
  }
  for (int d = 32; d >= 1; d >>= 1) sum += (uint32_t)__shfl_xor((int)sum, d, 64);
  if (lane == 0) part[wave] = sum;
  __syncthreads();
  uint32_t base = 0, total = 0;
  for (uint32_t k = 0; k < 16; ++k) {
    if (k < wave) base += part[k];
    total += part[k];
  }
  for (uint32_t i00 = lo; i00 < hi; i00 += 4 * 256) {
    u32x4 ahead[4];   // the array is rewritten in place: the reads of four rounds go before their writes
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) ahead[u] = load4(i00 + u * 256 + lane * 4);
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) {
      const uint32_t i0 = i00 + u * 256;
      if (i0 >= hi) break;
      const uint32_t i = i0 + lane * 4;
      const u32x4 x = ahead[u];
      const uint32_t s4 = x.x + x.y + x.z + x.w;
      uint32_t incl = s4;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = (uint32_t)__shfl_up((int)incl, d, 64);
        if ((int)lane >= d) incl += y;
      }
      const uint32_t e0 = base + incl - s4;
      const u32x4 out = {e0, e0 + x.x, e0 + x.x + x.y, e0 + x.x + x.y + x.z};
      if (kWhich == kScanVreg) {   // the counts are list lengths: queue the lists the bitmap sort will take
        if (x.x > kShortList) L.long_queue[atomicAdd(&L.counters[kCtrLong], 1u)] = i;
        if (x.y > kShortList) L.long_queue[atomicAdd(&L.counters[kCtrLong], 1u)] = i + 1;
        if (x.z > kShortList) L.long_queue[atomicAdd(&L.counters[kCtrLong], 1u)] = i + 2;
        if (x.w > kShortList) L.long_queue[atomicAdd(&L.counters[kCtrLong], 1u)] = i + 3;
      }
      if (i + 4 <= hi) *reinterpret_cast<u32x4 VL_GLOBAL *>(p + i) = out;
      else {
        if (i < hi) p[i] = out.x;
        if (i + 1 < hi) p[i + 1] = out.y;
        if (i + 2 < hi) p[i + 2] = out.z;
      }
      base += (uint32_t)__shfl((int)incl, 63, 64);
    }
  }
  if (threadIdx.x == 0) p[n] = total;
}

template <int kWhich>
__global__ __launch_bounds__(1024) void k_scan(MIRS) {
  f_scan<kWhich>(*as_global(mirs[blockIdx.x]), *as_global_rw(&lives[blockIdx.x]));
}

// Places each occurrence into its vreg's range (order inside a range is fixed later).
// Same privatisation: the slice reserves a sub-range per vreg with one global atomic,
// then ranks its own occurrences in LDS.
template <bool kLds>
__global__ __launch_bounds__(1024) void k_place(MIRS) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  extern __shared__ uint32_t sm[];
  const uint32_t o0 = blockIdx.x * kSlice;
  if (o0 >= m.O) return;
  const uint32_t o1 = min(m.O, o0 + kSlice);
  if (!kLds) {
    for (uint32_t o = o0 + threadIdx.x; o < o1; o += 1024) {
      const uint32_t v = m.occ_vreg[o];
      L.vocc_tmp[L.vcnt[v] + atomicAdd(&L.vcur[v], 1u)] = o;
    }
    return;
  }
  // one word per vreg: first the slice's count, then the next free position of the
  // sub-range reserved for the slice
  uint32_t *cnt = sm;
  for (uint32_t v = threadIdx.x; v < m.V; v += 1024) cnt[v] = 0;
  __syncthreads();
  for (uint32_t o = o0 + threadIdx.x; o < o1; o += 1024) atomicAdd(&cnt[m.occ_vreg[o]], 1u);
  __syncthreads();
  for (uint32_t v = threadIdx.x; v < m.V; v += 1024) {
    const uint32_t c = cnt[v];
    if (c) cnt[v] = L.vcnt[v] + atomicAdd(&L.vcur[v], c);
  }
  __syncthreads();
  for (uint32_t o = o0 + threadIdx.x; o < o1; o += 1024) L.vocc_tmp[atomicAdd(&cnt[m.occ_vreg[o]], 1u)] = o;
}

// Lists of up to kShortList occurrences are rank-sorted by one lane (the longer ones were
// queued by the scan of the list lengths).
__device__ inline void f_sort_short(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx) {
  const uint32_t v = bx * 256 + tx;
  if (v >= m.V) return;
  const uint32_t lo = L.vcnt[v], len = L.vcnt[v + 1] - lo;
  if (len == 0) { L.first[v] = kNone; return; }
  if (len > kShortList) return;
  // (the vreg of each sorted entry is recorded too, for the kernels that walk the entries)
  auto put = [&](uint32_t at, uint32_t x) {
    L.vocc[at] = x;
    L.ent_v[at] = v;
    if (at == lo) L.first[v] = x;
  };
  if (len <= 8) {
    // the common case: all loads issued at once, ranks computed in registers (absent
    // elements are larger than any occurrence index)
    uint32_t a[8];
#pragma unroll
    for (uint32_t k = 0; k < 8; ++k) a[k] = k < len ? L.vocc_tmp[lo + k] : kNone;
#pragma unroll
    for (uint32_t j = 0; j < 8; ++j) {
      uint32_t r = 0;
#pragma unroll
      for (uint32_t k = 0; k < 8; ++k) r += a[k] < a[j];
      if (j < len) put(lo + r, a[j]);
    }
    return;
  }
  // up to kShortList: the same with twice the registers (a lane or two of most wavefronts)
  static_assert(kShortList <= 16, "the register sort holds 16 occurrences");
  uint32_t a[16];
#pragma unroll
  for (uint32_t k = 0; k < 16; ++k) a[k] = k < len ? L.vocc_tmp[lo + k] : kNone;
#pragma unroll
  for (uint32_t j = 0; j < 16; ++j) {
    uint32_t r = 0;
#pragma unroll
    for (uint32_t k = 0; k < 16; ++k) r += a[k] < a[j];
    if (j < len) put(lo + r, a[j]);
  }
}

constexpr uint32_t kBitmapWords = 2048;              // 8 KB of LDS
constexpr uint32_t kBitmapSpan = kBitmapWords * 32;  // occurrences per window
constexpr uint32_t kLongBlocks = 64;                 // workgroups per kernel that take long lists

// Long lists: occurrence indices are distinct, so marking them in a bitmap and reading
// the bitmap back in order sorts them, one window of kBitmapSpan occurrences at a time.
__device__ inline void f_sort_long(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tid) {
  __shared__ uint32_t bm[kBitmapWords];
  __shared__ uint32_t wave_total[4];
  const uint32_t n_long = L.counters[kCtrLong];
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  for (uint32_t q = bx; q < n_long; q += kLongBlocks) {
    const uint32_t v = L.long_queue[q];
    const uint32_t lo = L.vcnt[v], len = L.vcnt[v + 1] - lo;
    uint32_t written = 0;
    for (uint32_t wb = 0; wb < m.O; wb += kBitmapSpan) {
      const uint32_t span = min(kBitmapSpan, m.O - wb), nw = (span + 31u) / 32u;
      for (uint32_t w = tid; w < nw; w += 256) bm[w] = 0;
      __syncthreads();
      for (uint32_t j = tid; j < len; j += 256) {
        uint32_t x = L.vocc_tmp[lo + j] - wb;
        if (x < span) atomicOr(&bm[x >> 5], 1u << (x & 31));
      }
      __syncthreads();
      const uint32_t chunk = (nw + 255u) / 256u;
      const uint32_t w0 = min(nw, tid * chunk), w1 = min(nw, w0 + chunk);
      uint32_t cnt = 0;
      for (uint32_t w = w0; w < w1; ++w) cnt += __popc(bm[w]);
      // exclusive prefix of cnt over the 256 threads: within the wavefront by shuffles,
      // across the four wavefronts through LDS
      uint32_t incl = cnt;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = (uint32_t)__shfl_up((int)incl, d, 64);
        if ((int)lane >= d) incl += y;
      }
      if (lane == 63) wave_total[wave] = incl;
      __syncthreads();
      uint32_t before = 0, total = 0;
      for (uint32_t k = 0; k < 4; ++k) {
        if (k < wave) before += wave_total[k];
        total += wave_total[k];
      }
      uint32_t pos = lo + written + before + incl - cnt;
      for (uint32_t w = w0; w < w1; ++w) {
        uint32_t bits = bm[w];
        while (bits) {
          uint32_t b = __ffs(bits) - 1;
          bits &= bits - 1;
          uint32_t x = wb + w * 32 + b;
          if (pos == lo) L.first[v] = x;
          L.ent_v[pos] = v;
          L.vocc[pos++] = x;
        }
      }
      written += total;
      __syncthreads();
    }
  }
}

// both sorts in one launch: the first kLongBlocks workgroups of each kernel take the long lists
__global__ __launch_bounds__(256) void k_sort(MIRS) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  if (blockIdx.x < kLongBlocks) f_sort_long(m, L, blockIdx.x, threadIdx.x);
  else f_sort_short(m, L, blockIdx.x - kLongBlocks, threadIdx.x);
}

// ---- 2. block summaries ---------------------------------------------------------------
// def[b]: vregs written in b.  use[b]: vregs whose first mention in b reads them
// (an instruction reads before it writes).
// Each workgroup takes a slice of the sorted entries, whose vregs span a narrow range of
// bitset words.  The bits are collected in an LDS table [block][word of the range] and each
// non-zero word goes to memory once; when the table would not fit, runs of equal
// (block, word) are combined by shuffles and every run issues its own atomics.
constexpr uint32_t kSumSlice = 1024, kSumThreads = 256;   // measured: 4096 / 1024 took 58 us, this 45 us, smaller no less
constexpr uint32_t kSumWords = kSumSlice / 32 + 1;   // most words a slice can touch

__global__ __launch_bounds__(kSumThreads) void k_summary(MIRS, const uint32_t lds_words) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  extern __shared__ uint32_t sm[];
  const uint32_t s0 = blockIdx.x * kSumSlice;
  if (s0 >= m.O) return;
  const uint32_t s1 = min(m.O, s0 + kSumSlice);
  const int lane = threadIdx.x & 63;
  // (vregs that are never mentioned take no entries but widen the range: a slice whose
  // table would not fit in the LDS given takes the other path)
  const uint32_t w_lo = L.ent_v[s0] >> 5, nw = (L.ent_v[s1 - 1] >> 5) - w_lo + 1;
  const bool lds = (size_t)2 * m.B * nw <= lds_words;
  if (lds) {
    for (uint32_t x = threadIdx.x; x < 2 * m.B * nw; x += kSumThreads) sm[x] = 0;
    __syncthreads();
  }
  uint32_t *def_l = sm, *use_l = sm + m.B * nw;
  // the lane's entries of the slice, each a chain of three dependent reads (occurrence, its
  // record, its block): the chains run side by side
  constexpr uint32_t kPer = kSumSlice / kSumThreads;
  uint64_t recs[kPer];
  uint32_t blks[kPer];
  {
    uint32_t occ[kPer];
#pragma unroll
    for (uint32_t u = 0; u < kPer; ++u) {
      const uint32_t e = s0 + u * kSumThreads + threadIdx.x;
      occ[u] = e < s1 ? L.vocc[e] : kNone;
    }
#pragma unroll
    for (uint32_t u = 0; u < kPer; ++u) recs[u] = occ[u] != kNone ? m.occ_rec[occ[u]] : 0ull;
#pragma unroll
    for (uint32_t u = 0; u < kPer; ++u) blks[u] = occ[u] != kNone ? m.instr_blk[(uint32_t)(recs[u] >> 34)] : kNone;
  }
  // the three entries below the wavefront's first one, held by lanes 0..2 (lane l: the entry
  // l + 1 below), for the lanes whose earlier neighbours are not in this wavefront
  uint64_t below_rec[kPer];
  uint32_t below_blk[kPer];
  {
    uint32_t occ[kPer];
#pragma unroll
    for (uint32_t u = 0; u < kPer; ++u) {
      const uint32_t wave_first = s0 + u * kSumThreads + (threadIdx.x & ~63u);
      occ[u] = (lane < 3 && wave_first < s1 && wave_first >= (uint32_t)lane + 1u) ? L.vocc[wave_first - 1u - lane] : kNone;
    }
#pragma unroll
    for (uint32_t u = 0; u < kPer; ++u) below_rec[u] = occ[u] != kNone ? m.occ_rec[occ[u]] : ~0ull;   // none: another vreg
#pragma unroll
    for (uint32_t u = 0; u < kPer; ++u) below_blk[u] = occ[u] != kNone ? m.instr_blk[(uint32_t)(below_rec[u] >> 34)] : kNone;
  }
#pragma unroll
  for (uint32_t u = 0; u < kPer; ++u) {
    const uint32_t e0 = s0 + u * kSumThreads;
    if (e0 >= s1) break;
    const uint32_t e = e0 + threadIdx.x;
    uint32_t b = kNone, w = 0, dbits = 0, ubits = 0, v = kNone, i = kNone, fl = 0;
    if (e < s1) {
      // also records instruction and flags of each sorted entry for the kernels that follow
      const uint64_t rec = recs[u];
      v = (uint32_t)rec;
      const uint32_t ifl = (uint32_t)(rec >> 32);
      L.ent_instr[e] = ifl;
      i = ifl >> 2;
      fl = ifl & 3u;
      b = blks[u];
      w = v >> 5;
      if (fl & VL_OCC_DEF) dbits = 1u << (v & 31);
    }
    // Is this mention group the first of its vreg in the block?  The nearest earlier entry
    // with another instruction decides; it usually sits an entry or two below.
    bool decided = !(fl & VL_OCC_USE), first_in_block = false;
    const uint32_t bv = (uint32_t)below_rec[u], bi = (uint32_t)(below_rec[u] >> 34), bb = below_blk[u];
    for (int d = 1; d <= 3; ++d) {
      uint32_t pv = __shfl_up(v, d, 64), pi = __shfl_up(i, d, 64), pb = __shfl_up(b, d, 64);
      const int src = (d - 1 - lane) & 63;   // for the lanes below d: the lane that holds their entry d below
      const uint32_t hv = __shfl(bv, src, 64), hi = __shfl(bi, src, 64), hb = __shfl(bb, src, 64);
      if (lane < d) { pv = hv; pi = hi; pb = hb; }
      if (!decided) {
        if (pv != v) { first_in_block = true; decided = true; }
        else if (pi != i) { first_in_block = pb != b; decided = true; }
      }
    }
    if (!decided) {   // four or more mentions in one instruction: look the start of the group up
      const uint32_t lo = L.vcnt[v];
      uint32_t gs = e;
      while (gs > lo && (uint32_t)(m.occ_rec[L.vocc[gs - 1]] >> 34) == i) --gs;
      first_in_block = gs == lo || m.instr_blk[(uint32_t)(m.occ_rec[L.vocc[gs - 1]] >> 34)] != b;
    }
    if ((fl & VL_OCC_USE) && first_in_block) ubits = 1u << (v & 31);
    if (lds) {
      if (dbits) atomicOr(&def_l[b * nw + (w - w_lo)], dbits);
      if (ubits) atomicOr(&use_l[b * nw + (w - w_lo)], ubits);
      continue;
    }
    // entries are sorted by vreg, then instruction: neighbours in a wavefront mostly hit
    // the same word of the same block.  OR them together along runs of equal (block, word)
    // and let the last lane of each run issue the atomics.
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t pb = __shfl_up(b, d, 64), pw = __shfl_up(w, d, 64);
      const uint32_t pd = __shfl_up(dbits, d, 64), pu = __shfl_up(ubits, d, 64);
      // a run of equal keys is contiguous, so equality with the lane d below means the
      // whole span in between belongs to the run
      if (lane >= d && pb == b && pw == w) { dbits |= pd; ubits |= pu; }
    }
    const uint32_t nb = __shfl_down(b, 1, 64), nxw = __shfl_down(w, 1, 64);
    const bool last = lane == 63 || nb != b || nxw != w;
    if (b != kNone && last) {
      if (dbits) atomicOr(&L.def[(size_t)b * m.W + w], dbits);
      if (ubits) atomicOr(&L.use[(size_t)b * m.W + w], ubits);
    }
  }
  if (!lds) return;
  __syncthreads();
  // the first and the last word of the range may be shared with the neighbouring slices
  for (uint32_t x = threadIdx.x; x < m.B * nw; x += kSumThreads) {
    const uint32_t blk = x / nw, w = w_lo + x % nw;
    if (def_l[x]) atomicOr(&L.def[(size_t)blk * m.W + w], def_l[x]);
    if (use_l[x]) atomicOr(&L.use[(size_t)blk * m.W + w], use_l[x]);
  }
}

// ---- 3. fixed point -------------------------------------------------------------------
// out[b] = OR of in[s] over successors; in[b] = use[b] | (out[b] & ~def[b]).  Bit columns
// do not interact, so each lane iterates its own word to its own fixed point; blocks are
// swept in reverse linear order.  LDS holds in/use/def of the wave's 64 words when the
// block count allows, otherwise the sweep runs on global memory.
template <bool kLds>
__global__ __launch_bounds__(64) void k_fixpoint(MIRS) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  extern __shared__ uint32_t sm[];
  const uint32_t lane = threadIdx.x, w = blockIdx.x * 64 + lane;
  if (blockIdx.x * 64 >= m.W) return;
  const bool act = w < m.W;
  const uint32_t B = m.B, W = m.W;
  // in_l has one row more than there are blocks: row B stays empty and stands for "no successor"
  uint32_t *in_l = sm, *use_l = sm + (size_t)(B + 1) * 64, *def_l = use_l + (size_t)B * 64;
  // the successor lists are walked once per block and sweep: they sit in LDS too, and the
  // first two successors of each block (absent ones: row B) in arrays of their own
  uint32_t *succ_off_l = def_l + (size_t)B * 64, *succ_l = succ_off_l + B + 1;
  uint32_t *s0_l = succ_l + m.E, *s1_l = s0_l + B;
  if (kLds) {
    for (uint32_t x = lane; x <= B; x += 64) succ_off_l[x] = m.succ_off[x];
    for (uint32_t x = lane; x < m.E; x += 64) succ_l[x] = m.succ[x];
    for (uint32_t x = lane; x < B; x += 64) {
      const uint32_t e0 = m.succ_off[x], e1 = m.succ_off[x + 1];
      s0_l[x] = e0 < e1 ? m.succ[e0] : B;
      s1_l[x] = e0 + 1 < e1 ? m.succ[e0 + 1] : B;
    }
    in_l[B * 64 + lane] = 0;
    for (uint32_t b0 = 0; b0 < B; b0 += 8) {   // the rows of eight blocks in flight
      uint32_t uu[8], dd[8];
#pragma unroll
      for (uint32_t t = 0; t < 8; ++t) {
        const bool in = act && b0 + t < B;
        uu[t] = in ? L.use[(size_t)(b0 + t) * W + w] : 0;
        dd[t] = in ? L.def[(size_t)(b0 + t) * W + w] : 0;
      }
#pragma unroll
      for (uint32_t t = 0; t < 8; ++t)
        if (b0 + t < B) {
          in_l[(b0 + t) * 64 + lane] = 0;
          use_l[(b0 + t) * 64 + lane] = uu[t];
          def_l[(b0 + t) * 64 + lane] = dd[t];
        }
    }
  }
  uint32_t sweeps = 0;
  bool changed = true;
  while (kLds && __any(changed)) {   // monotone on a finite lattice: terminates
    // A block's step is: read the rows of its successors, combine, write its own row.  What
    // does not depend on the row just written (the successors' indices, use, def and the old
    // row of the next block) is fetched one block ahead.
    changed = false;
    ++sweeps;
    uint32_t s0 = s0_l[B - 1], s1 = s1_l[B - 1], u = use_l[(B - 1) * 64 + lane], d = def_l[(B - 1) * 64 + lane];
    uint32_t n_succ = succ_off_l[B] - succ_off_l[B - 1];
    for (uint32_t b = B; b-- > 0;) {
      uint32_t out = in_l[s0 * 64 + lane] | in_l[s1 * 64 + lane];
      const uint32_t old = in_l[b * 64 + lane];
      if (n_succ > 2)
        for (uint32_t e = succ_off_l[b] + 2; e < succ_off_l[b + 1]; ++e) out |= in_l[succ_l[e] * 64 + lane];
      const uint32_t nin = u | (out & ~d);
      if (b > 0) {
        s0 = s0_l[b - 1]; s1 = s1_l[b - 1];
        u = use_l[(b - 1) * 64 + lane]; d = def_l[(b - 1) * 64 + lane];
        n_succ = succ_off_l[b] - succ_off_l[b - 1];
      }
      if (nin != old) {
        changed = true;
        in_l[b * 64 + lane] = nin;
      }
    }
  }
  while (!kLds && __any(changed)) {
    changed = false;
    ++sweeps;
    for (uint32_t b = B; b-- > 0;) {
      uint32_t out = 0;
      const uint32_t e0 = kLds ? succ_off_l[b] : m.succ_off[b], e1 = kLds ? succ_off_l[b + 1] : m.succ_off[b + 1];
      for (uint32_t e = e0; e < e1; ++e) {
        uint32_t s = kLds ? succ_l[e] : m.succ[e];
        out |= kLds ? in_l[s * 64 + lane] : (act ? L.live_in[(size_t)s * W + w] : 0);
      }
      uint32_t u = kLds ? use_l[b * 64 + lane] : (act ? L.use[(size_t)b * W + w] : 0);
      uint32_t d = kLds ? def_l[b * 64 + lane] : (act ? L.def[(size_t)b * W + w] : 0);
      uint32_t nin = u | (out & ~d);
      uint32_t old = kLds ? in_l[b * 64 + lane] : (act ? L.live_in[(size_t)b * W + w] : 0);
      if (nin != old) {
        changed = true;
        if (kLds) in_l[b * 64 + lane] = nin; else if (act) L.live_in[(size_t)b * W + w] = nin;
      }
    }
  }
  // write-out: in (when it lived in LDS) and out
  if (kLds) {
#pragma unroll 4
    for (uint32_t b = 0; b < B; ++b) {
      uint32_t out = in_l[s0_l[b] * 64 + lane] | in_l[s1_l[b] * 64 + lane];
      if (succ_off_l[b + 1] - succ_off_l[b] > 2)
        for (uint32_t e = succ_off_l[b] + 2; e < succ_off_l[b + 1]; ++e) out |= in_l[succ_l[e] * 64 + lane];
      if (act) {
        L.live_out[(size_t)b * W + w] = out;
        L.live_in[(size_t)b * W + w] = in_l[b * 64 + lane];
      }
    }
  }
  for (uint32_t b = 0; !kLds && b < B; ++b) {
    uint32_t out = 0;
    const uint32_t e0 = kLds ? succ_off_l[b] : m.succ_off[b], e1 = kLds ? succ_off_l[b + 1] : m.succ_off[b + 1];
    for (uint32_t e = e0; e < e1; ++e) {
      uint32_t s = kLds ? succ_l[e] : m.succ[e];
      out |= kLds ? in_l[s * 64 + lane] : (act ? L.live_in[(size_t)s * W + w] : 0);
    }
    if (act) {
      L.live_out[(size_t)b * W + w] = out;
      if (kLds) L.live_in[(size_t)b * W + w] = in_l[b * 64 + lane];
    }
  }
  // last block each vreg is live into (0 when there is none after the entry): lets the interval
  // kernels stop looking at later blocks.  Blocks in descending order; a lane owns its 32 vregs.
  uint32_t seen = 0;
  for (uint32_t b = B; b-- > 1;) {
    const uint32_t in_b = kLds ? in_l[b * 64 + lane] : (act ? L.live_in[(size_t)b * W + w] : 0);
    uint32_t fresh = in_b & ~seen;
    seen |= in_b;
    while (act && fresh) {
      const uint32_t v = w * 32 + __ffs(fresh) - 1;
      fresh &= fresh - 1;
      if (v < m.V) L.last_live[v] = b;
    }
  }
  uint32_t in0 = kLds ? in_l[lane] : (act ? L.live_in[w] : 0);
  if (act && in0) L.counters[kCtrNotStrict] = 1;
  if (lane == 0) atomicMax(&L.counters[kCtrSweeps], sweeps);
}

// one-byte summary of where membership in P(.) changes inside a mention group's stretch
constexpr uint8_t kStartI = 1, kStartI1 = 2, kEndI = 4, kEndI1 = 8, kEndN = 16, kAgain = 32, kOpenBefore = 64;

// ---- 4. per-occurrence liveness, kill flags and event roles ---------------------------
// For the mentions of v at instruction i (its "group"): v is live after i iff the next
// mention of v in the same block reads it, or, with no later mention in the block, v is
// in the block's live-out.  P(i) contains v iff it is live after i or written at i.
constexpr uint32_t kEvtThreads = 256, kEvtHalo = 16, kEvtWindow = kEvtThreads + 2 * kEvtHalo;

// (One-dimensional grid: block_map names the kernel and the stretch of 256 entries of every
// workgroup, so that no workgroup is launched for stretches a smaller kernel does not have.)
__global__ __launch_bounds__(kEvtThreads) void k_events(MIRS, const uint2 *__restrict__ block_map) {
  const uint2 where = block_map[blockIdx.x];
  const DevMir VL_GLOBAL &m = *as_global(mirs[where.x]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[where.x]);
  // The neighbours of an entry in the sorted order (its own mention group, the groups before
  // and after it) are looked at many times: the workgroup's stretch of entries plus a halo
  // on both sides is staged in LDS once, and only what lies beyond the halo is read from
  // memory.
  __shared__ uint32_t s_ifl[kEvtWindow], s_occ[kEvtWindow], s_v[kEvtWindow];
  const uint32_t base = where.y * kEvtThreads;
  if (base >= m.O) return;
  const uint32_t win_lo = base - kEvtHalo;   // may wrap below zero: window indices are taken modulo 2^32
  for (uint32_t r = threadIdx.x; r < kEvtWindow; r += kEvtThreads) {
    const uint32_t x = win_lo + r;
    const bool in = x < m.O;   // false for the wrapped indices too
    s_ifl[r] = in ? L.ent_instr[x] : 0u;
    s_occ[r] = in ? L.vocc[x] : 0u;
    s_v[r] = in ? L.ent_v[x] : kNone;
  }
  __syncthreads();
  const uint32_t e = base + threadIdx.x;
  if (e >= m.O) return;
  auto ent = [&](uint32_t x) { const uint32_t r = x - win_lo; return r < kEvtWindow ? s_ifl[r] : L.ent_instr[x]; };
  auto occ_at = [&](uint32_t x) { const uint32_t r = x - win_lo; return r < kEvtWindow ? s_occ[r] : L.vocc[x]; };
  const uint32_t o = s_occ[threadIdx.x + kEvtHalo], v = s_v[threadIdx.x + kEvtHalo];
  const uint32_t ifl = s_ifl[threadIdx.x + kEvtHalo], i = ifl >> 2;
  // What is read from memory depends on (v, i) first and on the blocks found second: the reads
  // of each level are issued together, with indices clamped where the value may not be needed,
  // so that a lane waits for memory twice instead of once per branch taken.
  const uint32_t lo = L.vcnt[v], hi = L.vcnt[v + 1];
  const uint32_t b = m.instr_blk[i], blk_before = m.instr_blk[i > 0 ? i - 1 : 0];
  const bool keeps = m.instr_keep[i] != 0, kept_before = m.instr_keep[i > 0 ? i - 1 : 0] != 0;
  const uint32_t attr = m.vattr[v], last_live_v = L.last_live[v];
  uint32_t gs = e, ge = e + 1;
  while (gs > lo && (ent(gs - 1) >> 2) == i) --gs;
  while (ge < hi && (ent(ge) >> 2) == i) ++ge;
  bool has_use = false, has_def = false;
  uint32_t first_use = kNone, first_def = kNone;
  for (uint32_t x = gs; x < ge; ++x) {
    const uint32_t f = x == e ? ifl : ent(x);
    if (f & VL_OCC_USE) { has_use = true; if (first_use == kNone) first_use = x; }
    if (f & VL_OCC_DEF) { has_def = true; if (first_def == kNone) first_def = x; }
  }
  const uint32_t nxt = ge < hi ? ent(ge) : 0u;
  // second level
  const uint32_t vw = v >> 5, vbit = 1u << (v & 31);
  const uint32_t blk_next = m.instr_blk[nxt >> 2];
  const bool out_b = (L.live_out[(size_t)b * m.W + vw] & vbit) != 0;
  const bool out_below = (L.live_out[(size_t)(b > 0 ? b - 1 : 0) * m.W + vw] & vbit) != 0;
  const bool out_before = (L.live_out[(size_t)blk_before * m.W + vw] & vbit) != 0;
  const uint32_t start_b = m.blk_start[b], start_b1 = m.blk_start[b + 1], start_b2 = m.blk_start[min(b + 2, m.B)];
  const bool in_after = (L.live_in[(size_t)min(b + 1, m.B - 1) * m.W + vw] & vbit) != 0;   // live into the block after b
  const uint32_t F = m.class_size[attr_class(attr)];
  bool la;
  if (ge < hi && blk_next == b) {
    la = (nxt & VL_OCC_USE) != 0;
    for (uint32_t x = ge + 1; x < hi && (ent(x) >> 2) == (nxt >> 2); ++x) la |= (ent(x) & VL_OCC_USE) != 0;
  } else {
    la = out_b;
  }
  const uint32_t fl = ifl & 3u;
  const bool kill = (fl & VL_OCC_USE) && !has_def && !la;
  uint8_t role = 0;
  // an instruction with an early-clobber definition keeps what it reads occupied until it has
  // written: the operand that dies here is released after the definitions have been tested
  if (!has_def && !la && e == first_use) role |= keeps ? kRolePostKill : kRolePreKill;
  if (has_def && e == first_def) {
    if (!has_use) role |= kRoleTestSet;
    if (!la) role |= kRolePostKill;
  }
  if (e == lo) role |= kRoleFirst;
  L.occ_role[o] = role | (kill ? kRoleKill : 0);
  const uint32_t prev = e > lo ? occ_at(e - 1) : kNone;
  if (prev != kNone && o - prev >= 0xFFFFu) L.prev_occ[o] = prev;
  // the occurrence's check record (its events are counted per instruction by a later pass over the roles)
  {
    // when an occurrence is checked the ring ends with that occurrence's chunk
    const uint32_t next = e + 1 < hi ? occ_at(e + 1) : o;
    const bool keep = o + kWalkReach < (next / kWalkChunk + 1u) * kWalkChunk && next - o <= kKeepMaxGap;
    const uint32_t delta = prev == kNone ? 0u : min(o - prev, 0xFFFFu);
    const bool near = prev != kNone && delta != 0xFFFFu && prev + kWalkReach >= (o / kWalkChunk + 1u) * kWalkChunk;
    const uint32_t width = attr_width(attr), align = attr_align(attr);
    const bool is_first = (role & kRoleFirst) != 0;
    const bool generic = is_first && ((align & (align - 1u)) != 0 || m.has_reserved || width > F);
    const bool simple = is_first && !generic;
    u32x4 r;
    r.x = (is_first ? kPlanFirst : kPlanChk) | (keep ? kPlanKeep : 0u) | (near ? kChkNear : 0u) | (generic ? kChkGeneric : 0u) |
          ((o % kWalkRing) << 8) | (((near ? prev : o) % kWalkRing) << 20);
    r.y = delta | (attr << 16);
    r.z = simple ? (align - 1u) * 0x10001u : 0u;
    r.w = simple ? min(F - width, 0xFFFFu) * 0x10001u : 0xFFFFFFFFu;
    L.chk[o] = r;
  }
  L.ent_info[e] = (uint8_t)((la ? kEntLiveAfter : 0) | (has_use ? kEntHasUse : 0) | (has_def ? kEntHasDef : 0) |
                            (e == gs ? kEntGroupStart : 0) | (keeps && has_use ? kEntKept : 0));

  // ---- live intervals, counting pass (the filling pass and the reasoning are at f_seg) ----
  // The first entry of each mention group owns the stretch from i up to the next mention of v
  // and counts the run starts in it; what the neighbouring groups contribute is worked out
  // from their flags here, since their own threads may not have run yet.
  if (e != gs) { L.ent_seg[e] = 0; L.ent_sf[e] = 0; return; }
  bool cur;   // was v occupied just before this stretch?
  if (i == 0) cur = false;
  else if (gs > lo && (ent(gs - 1) >> 2) == i - 1) {
    bool prev_def = false, prev_use = false;
    for (uint32_t x = gs; x-- > lo && (ent(x) >> 2) == i - 1;) {
      prev_def |= (ent(x) & VL_OCC_DEF) != 0;
      prev_use |= (ent(x) & VL_OCC_USE) != 0;
    }
    // live after i - 1: this group is the next mention; in another block the block's live-out decides
    const bool prev_la = blk_before == b ? has_use : out_before;
    cur = prev_def || prev_la || (prev_use && kept_before);
  } else if (i > start_b) cur = has_use;
  else cur = out_below;
  uint8_t sf = cur ? kOpenBefore : 0;
  uint32_t n_start = 0;
  auto span = [&](uint32_t s, uint32_t t, bool member) {
    if (t <= s) return;
    if (member && !cur) {
      ++n_start;
      sf |= s == i ? kStartI : s == i + 1 ? kStartI1 : kAgain;
    }
    if (!member && cur) sf |= s == i ? kEndI : s == i + 1 ? kEndI1 : kAgain;
    cur = member;
  };
  span(i, i + 1, has_def || la || (keeps && has_use));
  const uint32_t i2 = ge < hi ? nxt >> 2 : m.N;
  const uint32_t b2 = ge < hi ? blk_next : m.B;
  const uint32_t start_next = m.blk_start[b2];   // third level; only needed when the next mention is in another block
  if (b2 == b) {
    span(i + 1, i2, la);
  } else {
    span(i + 1, start_b1, la);
    // blocks in between: v is live into none of them after its last live block.  The block
    // right after b (nearly always the only one) was read with the second level.
    const uint32_t xe = min(b2, max(b + 1, last_live_v + 1));
    if (b + 1 < xe) span(start_b1, start_b2, in_after);
    for (uint32_t x = b + 2; x < xe; ++x)
      span(m.blk_start[x], m.blk_start[x + 1], bit_get(L.live_in + (size_t)x * m.W, v));
    if (xe < b2) {
      if (xe == b + 1) span(start_b1, start_b2, false);
      else span(m.blk_start[xe], m.blk_start[xe + 1], false);
    }
    if (ge < hi) {
      bool next_use = false;
      for (uint32_t x = ge; x < hi && (ent(x) >> 2) == i2; ++x) next_use |= (ent(x) & VL_OCC_USE) != 0;
      span(start_next, i2, next_use);
    }
  }
  if (ge >= hi && cur) sf |= kEndN;
  if (n_start > 1) sf |= kAgain;   // two starts in one stretch cannot be told apart by the summary
  L.ent_seg[e] = n_start;
  L.ent_sf[e] = sf;
}

// ---- 5a. event stream -----------------------------------------------------------------
__device__ inline uint32_t item_of_instr(const DevMir VL_GLOBAL &m, uint32_t i) { return i + m.instr_blk[i] + 1; }

__device__ inline uint32_t wave_incl_scan(uint32_t x) {
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t y = __shfl_up(x, d, 64);
    if ((int)(threadIdx.x & 63) >= d) x += y;
  }
  return x;
}

// nearest occurrence of v before instruction `at`, else the first at or after it
__device__ inline uint32_t source_occurrence(const DevLive VL_GLOBAL &L, uint32_t v, uint32_t at) {
  const uint32_t lo = L.vcnt[v], hi = L.vcnt[v + 1];
  uint32_t x = lower_bound(L.ent_instr, lo, hi, at << 2);   // entries hold instruction << 2 | flags
  return x > lo ? L.vocc[x - 1] : (x < hi ? L.vocc[x] : 0u);
}

// The record of one occupancy event (layout in vl_dev.h).  `near`: the occurrence is
// certainly inside the verifier's ring when the event is replayed.
__device__ inline u32x4 event_record(uint32_t o, uint32_t v, uint32_t attr, bool tested, bool near) {
  const uint32_t width = attr_width(attr);
  const bool slow = !near || attr_straddle(attr) || width == 32;
  u32x4 r;
  r.x = (o % kWalkRing) | (v << 8);
  r.y = width == 32 ? 0xFFFFFFFFu : ((1u << width) - 1u);
  r.z = attr_word(attr) * 256u;
  r.w = o | (slow ? kEvtSlow : 0u) | (tested ? kEvtTested : 0u);
  return r;
}
__device__ inline u32x4 event_record(const DevMir VL_GLOBAL &m, uint32_t o, uint32_t v, bool tested, bool near) {
  return event_record(o, v, m.vattr[v], tested, near);
}

// Between two blocks adjacent in the linear order the occupied set changes from the
// earlier block's live-out to the later block's live-in: one wave per boundary lists the
// values that leave (release) and those that enter (occupy without test).
template <bool kFill>
__device__ inline void f_boundary(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                  const uint32_t bdim) {
  const uint32_t b = bx, lane = tx;
  if (b >= m.B) return;
  const uint32_t item = m.blk_start[b] + b;
  if (b == 0) {
    if (!kFill && lane == 0) L.item_off[item] = 0;
    return;
  }
  const uint32_t W = m.W, at = m.blk_start[b];
  const uint32_t VL_GLOBAL *out_prev = L.live_out + (size_t)(b - 1) * W;
  const uint32_t VL_GLOBAL *in_cur = L.live_in + (size_t)b * W;
  uint32_t base = kFill ? L.item_off[item] : 0, total = 0;
  // Filling: a lane first lists the vregs of its word in LDS; then the wavefront completes
  // one record per lane, so that the look-ups of the source occurrences run side by side.
  constexpr uint32_t kList = 512;
  __shared__ uint32_t s_list[kFill ? 4 * kList : 1];
  uint32_t *list = s_list + (kFill ? (threadIdx.x >> 6) * kList : 0);
  auto record = [&](uint32_t v) {
    const uint32_t src = source_occurrence(L, v, at);
    // replayed with the block's first instruction, when the readable window ends at
    // most 127 occurrences after that instruction's first operand
    const bool near = src < m.occ_off[at] && src + (kWalkReach - 2 * kWalkChunk + 1) >= m.occ_off[at];
    return event_record(m, src, v, false, near);
  };
  if (!kFill) {   // counting needs no positions: both directions at once, one reduction at the end
    uint32_t mine = 0;
    for (uint32_t w = lane; w < W; w += 64) mine += __popc(out_prev[w] ^ in_cur[w]);
    for (int d = 32; d >= 1; d >>= 1) mine += (uint32_t)__shfl_xor((int)mine, d, 64);
    if (lane == 0) L.item_off[item] = mine;
    return;
  }
  for (int pass = 0; pass < 2; ++pass) {  // 0: leaving, 1: entering
    for (uint32_t w0 = 0; w0 < W; w0 += 64) {
      const uint32_t w = w0 + lane;
      uint32_t bits = 0;
      if (w < W) bits = pass == 0 ? (out_prev[w] & ~in_cur[w]) : (in_cur[w] & ~out_prev[w]);
      const uint32_t c = __popc(bits), incl = wave_incl_scan(c);
      const uint32_t n_here = __shfl(incl, 63, 64);
      if (kFill && n_here) {
        uint32_t pos = incl - c;
        const bool listed = n_here <= kList;   // the same in every lane
        while (bits) {
          const uint32_t v = w * 32 + __ffs(bits) - 1;
          bits &= bits - 1;
          if (listed) list[pos++] = v;
          else L.plan[base + total + pos++] = record(v);
        }
        if (listed) {
          __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
          __builtin_amdgcn_wave_barrier();
          for (uint32_t x = lane; x < n_here; x += 64) L.plan[base + total + x] = record(list[x]);
          __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
          __builtin_amdgcn_wave_barrier();
        }
      }
      total += n_here;
    }
  }
  if (!kFill && lane == 0) L.item_off[item] = total;
}

// Occupancy events of each instruction, in the order they take effect: releases of
// operands that die here, then test-and-occupy of the values written, then releases of
// values that are dead once the instruction has executed.
__device__ inline void f_plan_fill(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                   const uint32_t bdim) {
  uint32_t i = bx * bdim + tx;
  if (i >= m.N) return;
  const uint32_t base = L.item_off[item_of_instr(m, i)];
  const uint32_t o0 = m.occ_off[i], o1 = m.occ_off[i + 1];
  uint32_t n_pre = 0, n_set = 0;
  if (o1 - o0 <= 4) {
    // the common case: roles and vregs of all operands are read together, then their
    // attributes, so that the lane waits once per level instead of once per operand
    const uint32_t n = o1 - o0;
    uint32_t role[4], vv[4], aa[4];
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) {
      role[u] = u < n ? (uint32_t)L.occ_role[o0 + u] : 0u;
      vv[u] = u < n ? m.occ_vreg[o0 + u] : 0u;
    }
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) aa[u] = m.vattr[vv[u]];
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) {
      if (u < n) L.occ_kill[o0 + u] = (role[u] & kRoleKill) ? 1 : 0;
      n_pre += (role[u] & kRolePreKill) ? 1u : 0u;
      n_set += (role[u] & kRoleTestSet) ? 1u : 0u;
    }
    uint32_t at_pre = base, at_set = base + n_pre, at_post = base + n_pre + n_set;
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) {
      if (!(role[u] & (kRolePreKill | kRoleTestSet | kRolePostKill))) continue;
      const u32x4 r = event_record(o0 + u, vv[u], aa[u], false, true);
      if (role[u] & kRolePreKill) L.plan[at_pre++] = r;
      if (role[u] & kRoleTestSet) { u32x4 q = r; q.w |= kEvtTested; L.plan[at_set++] = q; }
      if (role[u] & kRolePostKill) { u32x4 q = r; q.w |= kEvtPost; L.plan[at_post++] = q; }
    }
    return;
  }
  for (uint32_t o = o0; o < o1; ++o) {
    const uint32_t role = L.occ_role[o];
    L.occ_kill[o] = (role & kRoleKill) ? 1 : 0;   // kill flags, in occurrence order
    n_pre += (role & kRolePreKill) ? 1u : 0u;
    n_set += (role & kRoleTestSet) ? 1u : 0u;
  }
  uint32_t at_pre = base, at_set = base + n_pre, at_post = base + n_pre + n_set;
  for (uint32_t o = o0; o < o1; ++o) {
    const uint32_t role = L.occ_role[o];
    if (!(role & (kRolePreKill | kRoleTestSet | kRolePostKill))) continue;
    // an instruction's own operands are always inside the ring when its events are replayed
    const u32x4 r = event_record(m, o, m.occ_vreg[o], false, true);
    if (role & kRolePreKill) L.plan[at_pre++] = r;
    if (role & kRoleTestSet) { u32x4 q = r; q.w |= kEvtTested; L.plan[at_set++] = q; }
    if (role & kRolePostKill) { u32x4 q = r; q.w |= kEvtPost; L.plan[at_post++] = q; }
  }
}

// number of events of each instruction: the roles of its operands (the counterpart of the
// filling pass above)
__device__ inline void f_item_count(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                    const uint32_t bdim) {
  const uint32_t i = bx * bdim + tx;
  if (i >= m.N) return;
  uint32_t n_evt = 0;
  for (uint32_t o = m.occ_off[i]; o < m.occ_off[i + 1]; ++o)
    n_evt += __popc(L.occ_role[o] & (kRolePreKill | kRoleTestSet | kRolePostKill));
  L.item_off[item_of_instr(m, i)] = n_evt;
}

// evt_cut[c] = index of the first event of the first item whose operands end in chunk c or
// later (an item's events may be replayed once occurrences [0, 64 (c + 1)) are staged).
__device__ inline void f_evt_cut(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                 const uint32_t bdim) {
  const uint32_t c = bx * bdim + tx;
  const uint32_t n_chunk = (m.O + 63) / 64;
  if (c > n_chunk) return;
  // first instruction i with occ_off[i + 1] > 64 c: the one that occurrence 64 c belongs to
  const uint32_t lo = 64 * c < m.O ? m.occ_instr[64 * c] : m.N;
  uint32_t cut;
  if (lo >= m.N || c == n_chunk) cut = L.item_off[m.N + m.B];
  else {
    const uint32_t b = m.instr_blk[lo];
    cut = L.item_off[m.blk_start[b] == lo ? lo + b : lo + b + 1];   // boundary events go with their block's first instruction
  }
  L.evt_cut[c] = cut;
}

// ---- 5b. live intervals ---------------------------------------------------------------
// Membership of v in P(.) changes only at instructions that mention v and at block
// boundaries.  The lane of each mention group (all mentions of v at one instruction) owns
// the stretch from its instruction up to the next mention of v (the last group: up to the
// end of the program) and finds the run starts and ends inside it; what holds just before
// the stretch is known locally.  Groups are sorted by (vreg, instruction), so a prefix sum
// of the start counts numbers the runs in CSR order; the j-th end belongs to the j-th start.
__device__ inline void f_seg_fill(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                  const uint32_t bdim) {
  const uint32_t e = bx * bdim + tx;
  if (e >= m.O) return;
  // The counting pass (in the per-occurrence kernel) left a one-byte summary per entry.
  // Nearly every stretch changes membership only at its own instruction i, at i + 1 or at
  // the end of the program, and then the summary says everything needed here; the other
  // stretches (those with changes at block boundaries) are worked out again.
  const uint8_t sf = L.ent_sf[e];
  if (!(sf & (kStartI | kStartI1 | kEndI | kEndI1 | kEndN | kAgain))) return;
  const uint32_t i = L.ent_instr[e] >> 2;
  // runs that started before this stretch and ended before it: the end index lags the
  // start index by one exactly while a run is open
  size_t n_start = L.ent_seg[e];
  size_t n_end = n_start - ((sf & kOpenBefore) ? 1u : 0u);
  if (!(sf & kAgain)) {
    if (sf & kStartI) L.seg[2 * n_start] = i;
    if (sf & kStartI1) L.seg[2 * n_start] = i + 1;
    if (sf & kEndI) L.seg[2 * n_end++ + 1] = i;
    if (sf & kEndI1) L.seg[2 * n_end++ + 1] = i + 1;
    if (sf & kEndN) L.seg[2 * n_end + 1] = m.N;
    return;
  }
  const uint8_t info = L.ent_info[e];
  const uint32_t v = L.ent_v[e];
  const uint32_t hi = L.vcnt[v + 1], b = m.instr_blk[i];
  bool cur = (sf & kOpenBefore) != 0;
  auto span = [&](uint32_t s, uint32_t t, bool member) {
    if (t <= s) return;
    if (member && !cur) L.seg[2 * n_start++] = s;
    if (!member && cur) L.seg[2 * n_end++ + 1] = s;
    cur = member;
  };
  uint32_t ge = e + 1;
  while (ge < hi && (L.ent_instr[ge] >> 2) == i) ++ge;
  const bool la = (info & kEntLiveAfter) != 0;
  span(i, i + 1, (info & (kEntHasDef | kEntKept)) || la);
  const uint32_t i2 = ge < hi ? L.ent_instr[ge] >> 2 : m.N;
  const uint32_t b2 = ge < hi ? m.instr_blk[i2] : m.B;
  if (b2 == b) {
    span(i + 1, i2, la);
  } else {
    span(i + 1, m.blk_start[b + 1], la);
    const uint32_t xe = min(b2, max(b + 1, L.last_live[v] + 1));
    for (uint32_t x = b + 1; x < xe; ++x)
      span(m.blk_start[x], m.blk_start[x + 1], bit_get(L.live_in + (size_t)x * m.W, v));
    if (xe < b2) span(m.blk_start[xe], m.blk_start[xe + 1], false);
    if (ge < hi) span(m.blk_start[b2], i2, (L.ent_info[ge] & kEntHasUse) != 0);
  }
  if (ge >= hi && cur) L.seg[2 * n_end + 1] = m.N;
}

// seg_off per vreg from the per-entry prefix sums
__device__ inline void f_seg_off(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                 const uint32_t bdim) {
  const uint32_t v = bx * bdim + tx;
  if (v > m.V) return;
  L.seg_off[v] = L.ent_seg[v < m.V ? L.vcnt[v] : m.O];
}

// hull of each vreg from its (ascending) runs: [first start, last end), or [0,0) without runs
__device__ inline void f_hull(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                              const uint32_t bdim) {
  const uint32_t v = bx * bdim + tx;
  if (v >= m.V) return;
  const uint32_t s0 = L.seg_off[v], s1 = L.seg_off[v + 1];
  L.hull[2 * v] = s1 > s0 ? L.seg[2 * (size_t)s0] : 0u;
  L.hull[2 * v + 1] = s1 > s0 ? L.seg[2 * (size_t)s1 - 1] : 0u;
}

// ---- 5c. tile live-ins ------------------------------------------------------------------
// Tile t starts at instruction t * tile_len; its seed is the set live before that
// instruction.  Replaying every occupancy event of the program from the start (nothing is
// live into the entry) gives exactly that set, and every event flips one bit, so the seed
// of tile t is the exclusive-or of all flips of the tiles before it.
// k_tile_delta: one workgroup per tile XORs the tile's flips into an LDS row: the events
// of its instructions (an occurrence with an odd number of roles flips its vreg) and of
// the block boundaries right after its instructions (live-out of the earlier block XOR
// live-in of the later one).
__device__ inline void f_tile_delta(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                    const uint32_t bdim) {
  extern __shared__ uint32_t row[];
  const uint32_t t = bx;
  if (t >= L.T) return;
  const uint32_t W = m.W, i0 = t * L.tile_len, i1 = min(m.N, i0 + L.tile_len);
  for (uint32_t w = tx; w < W; w += 256) row[w] = 0;
  __syncthreads();
  const uint32_t o_end = m.occ_off[i1];
  for (uint32_t o = m.occ_off[i0] + tx; o < o_end; o += 4 * 256) {   // four reads of each kind in flight
    uint32_t role[4], vv[4];
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) {
      const uint32_t x = o + u * 256;
      role[u] = x < o_end ? (uint32_t)L.occ_role[x] : 0u;
      vv[u] = x < o_end ? m.occ_vreg[x] : 0u;
    }
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u)
      if (__popc(role[u] & (kRolePreKill | kRoleTestSet | kRolePostKill)) & 1) atomicXor(&row[vv[u] >> 5], 1u << (vv[u] & 31));
  }
  // boundaries b whose last earlier instruction (blk_start[b] - 1) lies in this tile
  const uint32_t b_lo = m.instr_blk[i0] + 1, b_hi = m.instr_blk[i1 - 1] + 1;   // blocks starting in (i0, i1]
  for (uint32_t b = b_lo; b <= b_hi && b < m.B; ++b) {
    if (m.blk_start[b] - 1 < i0 || m.blk_start[b] - 1 >= i1) continue;
    for (uint32_t w = tx; w < W; w += 256)
      atomicXor(&row[w], L.live_out[(size_t)(b - 1) * W + w] ^ L.live_in[(size_t)b * W + w]);
  }
  __syncthreads();
  for (uint32_t w = tx; w < W; w += 256) L.tile_live[(size_t)t * W + w] = row[w];
}

// exclusive prefix-XOR over the tiles, one bitset word per lane
__device__ inline void f_tile_prefix(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                     const uint32_t bdim) {
  const uint32_t w = bx * bdim + tx;
  if (w >= m.W) return;
  uint32_t acc = 0;
  for (uint32_t t0 = 0; t0 < L.T; t0 += 8) {   // eight tiles' words in flight
    uint32_t d[8];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) d[u] = t0 + u < L.T ? L.tile_live[(size_t)(t0 + u) * m.W + w] : 0u;
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) {
      if (t0 + u < L.T) L.tile_live[(size_t)(t0 + u) * m.W + w] = acc;
      acc ^= d[u];
    }
  }
}

// One wavefront per tile lists the members of its seed row as occupy-without-test entries
// whose register is taken from the nearest earlier occurrence of the vreg.
template <bool kFill>
__device__ inline void f_seed(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                              const uint32_t bdim) {
  const uint32_t t = bx, lane = tx;
  if (t >= L.T) return;
  const uint32_t W = m.W;
  uint32_t total = 0;
  const uint32_t base = kFill ? L.seed_off[t] : 0;
  if (!kFill) {   // counting needs no positions: one reduction at the end
    uint32_t mine = 0;
    if (t > 0)
      for (uint32_t w = lane; w < W; w += 64) mine += __popc(L.tile_live[(size_t)t * W + w]);
    for (int d = 32; d >= 1; d >>= 1) mine += (uint32_t)__shfl_xor((int)mine, d, 64);
    if (lane == 0) L.seed_off[t] = mine;
    return;
  }
  for (uint32_t w0 = 0; w0 < W; w0 += 64) {
    const uint32_t w = w0 + lane;
    uint32_t bits = (w < W && t > 0) ? L.tile_live[(size_t)t * W + w] : 0u;
    const uint32_t c = __popc(bits), incl = wave_incl_scan(c);
    if (kFill) {
      uint32_t pos = base + total + incl - c;
      while (bits) {
        const uint32_t v = w * 32 + __ffs(bits) - 1;
        bits &= bits - 1;
        u32x4 r = {v, t, 0u, 0u};   // completed by k_seed_src
        L.seeds[pos++] = r;
      }
    }
    total += __shfl(incl, 63, 64);
  }
  if (!kFill && lane == 0) L.seed_off[t] = total;
}

// completes each seed entry: the register comes from the nearest earlier occurrence
__device__ inline void f_seed_src(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                  const uint32_t bdim) {
  const uint32_t k = bx * bdim + tx;
  if (k >= L.n_seed) return;
  const u32x4 raw = L.seeds[k];
  const uint32_t v = raw.x, t = raw.y;
  // the register is always gathered from memory: the ring offset stays unused
  const uint32_t at = t * L.tile_len, lo = L.vcnt[v], hi = L.vcnt[v + 1];
  const uint32_t x = lower_bound(L.ent_instr, lo, hi, at << 2);   // first mention at or after the tile's start
  u32x4 r = event_record(m, x > lo ? L.vocc[x - 1] : (x < hi ? L.vocc[x] : 0u), v, false, true);
  r.x &= ~0xFFu;   // only the vreg: the register is always gathered from memory
  // the verifier keeps the gathered registers at hand for the link of that first mention
  if (x > lo && x < hi && (L.ent_instr[x] >> 2) < min(m.N, at + L.tile_len)) r.w |= kSeedLinked;
  L.seeds[k] = r;
}

// Clears `vecs` 16-byte vectors.  A kernel rather than a memset so that a caller may record
// the steady-state analysis into a stream capture (the arenas are 256-byte aligned and every
// region's length is a multiple of 256 bytes).
__global__ void k_zero(u32x4 VL_GLOBAL *p, size_t vecs) {
  const u32x4 z = {0, 0, 0, 0};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < vecs; i += (size_t)gridDim.x * blockDim.x) p[i] = z;
}

static inline void zero_async(void *p, size_t bytes, hipStream_t stream) {
  if (!bytes) return;
  const size_t vecs = bytes / 16;
  const uint32_t blocks = (uint32_t)std::min<size_t>(8192, (vecs + 255) / 256);
  k_zero<<<blocks, 256, 0, stream>>>((u32x4 VL_GLOBAL *)p, vecs);
}

__global__ void k_collect(MIRS, uint32_t n) {
  uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n) return;
  const DevMir VL_GLOBAL &m = *as_global(mirs[k]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[k]);
  L.counters[kCtrPlanLen] = L.item_off[m.N + m.B];
  L.counters[kCtrSeg] = L.ent_seg[m.O];
  L.counters[kCtrSeed] = L.seed_off[L.T];
}

__device__ inline void f_tile_range(const DevMir VL_GLOBAL &m, DevLive VL_GLOBAL &L, const uint32_t bx, const uint32_t tx,
                                    const uint32_t bdim) {
  uint32_t t = bx * bdim + tx;
  if (t >= L.T) return;
  const uint32_t i0 = t * L.tile_len, i1 = min(m.N, i0 + L.tile_len);
  L.tile_range[2 * t] = L.item_off[item_of_instr(m, i0)];
  uint32_t end;
  if (i1 == m.N) end = L.item_off[m.N + m.B];
  else {
    const uint32_t b = m.instr_blk[i1];
    // a tile ending at a block boundary leaves the boundary entries out: the next tile
    // starts from that block's live-in
    end = m.blk_start[b] == i1 ? L.item_off[i1 + b] : L.item_off[i1 + b + 1];
  }
  L.tile_range[2 * t + 1] = end;
}

// ---- stages ---------------------------------------------------------------------------
// After the per-occurrence pass three chains are independent: the event stream (boundary
// counts, scan, chunk cuts, fill), the intervals (count, scan, offsets, fill) and the tile
// live-ins (flips, prefix, count, scan, fill, sources).  Each stage below runs one step of
// every chain in one launch, the block index selecting the part, so that the short serial
// steps of one chain (scans, prefixes) overlap the bandwidth-heavy steps of another.  A
// part made of one wavefront per item gets four items per 256-thread block.
struct StageGrid { uint32_t a, b, c; };   // blocks of the three parts, in launch order
// The grids are sized for the largest kernel of the batch, so most blocks belong to smaller
// kernels and exit at once.  A block of the part that counts each instruction's events (light
// work) takes this many stretches of 256 instructions, which keeps their number down; the
// heavier parts are faster with one stretch per block.
constexpr uint32_t kStageReps = 4;

__global__ __launch_bounds__(256) void k_stage_count(MIRS, StageGrid g) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  const uint32_t bx = blockIdx.x, tx = threadIdx.x;
  if (bx < g.a) f_tile_delta(m, L, bx, tx, 256);
  else if (bx < g.a + g.b) f_boundary<false>(m, L, (bx - g.a) * 4 + (tx >> 6), tx & 63u, 64);
  else
    for (uint32_t r = 0; r < kStageReps; ++r) f_item_count(m, L, (bx - g.a - g.b) * kStageReps + r, tx, 256);
}

__global__ __launch_bounds__(1024) void k_stage_scan(MIRS, StageGrid g) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  const uint32_t bx = blockIdx.x;
  if (bx == 0) f_scan<kScanSeg>(m, L);
  else if (bx == 1) f_scan<kScanItems>(m, L);
  else f_tile_prefix(m, L, bx - 2, threadIdx.x, 1024);
}

__global__ __launch_bounds__(256) void k_stage_offsets(MIRS, StageGrid g) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  const uint32_t bx = blockIdx.x, tx = threadIdx.x;
  if (bx < g.a) f_seed<false>(m, L, bx * 4 + (tx >> 6), tx & 63u, 64);
  else if (bx < g.a + g.b) f_evt_cut(m, L, bx - g.a, tx, 256);
  else f_seg_off(m, L, bx - g.a - g.b, tx, 256);
}

// One-dimensional grid.  Part a: per_a workgroups for every kernel; parts b and c: one
// workgroup per stretch of 256 instructions / entries that exists, named by the block maps.
__global__ __launch_bounds__(256) void k_stage_fill(MIRS, StageGrid g, uint32_t per_a, const uint2 *__restrict__ map_instr,
                                                    const uint2 *__restrict__ map_occ) {
  const uint32_t bx = blockIdx.x, tx = threadIdx.x;
  uint2 where;
  if (bx < g.a) where = make_uint2(bx / per_a, bx % per_a);
  else if (bx < g.a + g.b) where = map_instr[bx - g.a];
  else where = map_occ[bx - g.a - g.b];
  const DevMir VL_GLOBAL &m = *as_global(mirs[where.x]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[where.x]);
  if (bx < g.a) f_seed<true>(m, L, where.y * 4 + (tx >> 6), tx & 63u, 64);
  else if (bx < g.a + g.b) f_plan_fill(m, L, where.y, tx, 256);
  else f_seg_fill(m, L, where.y, tx, 256);
}

__global__ __launch_bounds__(256) void k_stage_finish(MIRS, StageGrid g) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  const uint32_t bx = blockIdx.x, tx = threadIdx.x;
  if (bx < g.a) f_boundary<true>(m, L, bx * 4 + (tx >> 6), tx & 63u, 64);
  else if (bx < g.a + g.b) f_tile_range(m, L, bx - g.a, tx, 256);
  else if (bx < g.a + g.b + g.c) f_seed_src(m, L, bx - g.a - g.b, tx, 256);
  else f_hull(m, L, bx - g.a - g.b - g.c, tx, 256);
}

// ---- 5d. dense per-point bitsets (optional) ---------------------------------------------
// Every occupy / release event flips one bit of the occupied set.  First each event is
// XOR-ed into the row of the instruction at which it takes effect, then each tile
// prefix-XORs its rows downwards from the tile's live-in row.
__global__ void k_dense_delta(MIRS) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.y]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.y]);
  uint32_t q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= m.N + m.B) return;
  // item q is either the boundary of block b (q == blk_start[b] + b) or an instruction of
  // block b: b is the last block whose boundary item is at or before q
  uint32_t b = 0, hi = m.B;
  while (hi - b > 1) {
    uint32_t mid = (b + hi) >> 1;
    if (m.blk_start[mid] + mid <= q) b = mid; else hi = mid;
  }
  const uint32_t row = (q == m.blk_start[b] + b) ? m.blk_start[b] : q - b - 1;
  // a tile that starts exactly at this block start takes its row from the seed instead
  if (q == m.blk_start[b] + b && row % L.tile_len == 0) return;
  for (uint32_t e = L.item_off[q]; e < L.item_off[q + 1]; ++e) {
    const uint32_t v = L.plan[e].x >> 8;
    atomicXor(&L.live_after[(size_t)row * m.W + (v >> 5)], 1u << (v & 31));
  }
}

__global__ __launch_bounds__(64) void k_dense_scan(MIRS) {
  const DevMir VL_GLOBAL &m = *as_global(mirs[blockIdx.z]);
  DevLive VL_GLOBAL &L = *as_global_rw(&lives[blockIdx.z]);
  const uint32_t t = blockIdx.y, w = blockIdx.x * 64 + threadIdx.x;
  if (t >= L.T || w >= m.W) return;
  const uint32_t i0 = t * L.tile_len, i1 = min(m.N, i0 + L.tile_len);
  uint32_t cur = t ? L.tile_live[(size_t)t * m.W + w] : 0u;
  for (uint32_t i = i0; i < i1; ++i) {
    cur ^= L.live_after[(size_t)i * m.W + w];
    L.live_after[(size_t)i * m.W + w] = cur;
  }
}

struct Bump {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t at = off;
    off += (bytes + 255) & ~(size_t)255;
    return at;
  }
};

}  // namespace

// A batch owns the device storage of n analyses made by one call.
struct vl_batch {
  uint32_t n = 0, refs = 0;
  int device = 0;
  void *arena1 = nullptr, *arena2 = nullptr;
  size_t cap1 = 0, cap2 = 0;
  const DevMir **dev_mirs = nullptr;  // device array [n]
  DevLive *dev_lives = nullptr;       // device array [n]
  uint32_t *host_counters = nullptr;  // pinned [n][kCounters]
  const DevMir **stage_mirs = nullptr;  // pinned [n]
  DevLive *stage_a = nullptr, *stage_b = nullptr;  // pinned [n] each: first and second upload
  std::vector<vl_live *> lives;
  // result sizes of the last successful call (the analysis of the same kernels with the same
  // options is deterministic, so a recycling call need not read them back)
  bool sized = false, sized_dense = false;
  uint32_t sized_tile_len = 0;
  std::vector<uint32_t> sizes;   // [n][3]: events, interval segments, tile live-ins
  std::vector<char> uploaded;    // the DevLive table as it stands on the device after the last successful call
  uint2 *stage_map = nullptr;    // pinned: the block maps (kernel, stretch of 256) of the per-instruction and per-entry launches
  size_t map_cap = 0;
};

static void batch_free(vl_batch *b) {
  if (b->arena1) (void)hipFree(b->arena1);
  if (b->arena2) (void)hipFree(b->arena2);
  if (b->host_counters) (void)hipHostFree(b->host_counters);
  if (b->stage_mirs) (void)hipHostFree(b->stage_mirs);
  if (b->stage_a) (void)hipHostFree(b->stage_a);
  if (b->stage_b) (void)hipHostFree(b->stage_b);
  if (b->stage_map) (void)hipHostFree(b->stage_map);
  delete b;
}

extern "C" void vl_live_destroy(vl_live *l) {
  if (!l || l->magic != kLiveMagic) return;
  l->magic = 0;
  vl_batch *b = l->batch;
  delete l;
  if (--b->refs == 0) batch_free(b);
}

static inline dim3 grid1(uint32_t items, uint32_t threads, uint32_t n) {
  return dim3(std::max(1u, (items + threads - 1) / threads), n, 1);
}

extern "C" int32_t vl_liveness_multi(const vl_mir *const *mirs, uint32_t n, uint32_t flags, uint32_t tile_len,
                                     vl_stream stream_, vl_live **live) {
  if (!mirs || !live) return VL_E_NULL;
  if (n == 0 || n > 65535) return VL_E_SHAPE;
  if (flags & ~VL_DENSE_POINTS) return VL_E_RANGE;
  for (uint32_t k = 0; k < n; ++k)
    if (!mirs[k] || mirs[k]->magic != kMirMagic) return VL_E_NULL;
  hipStream_t stream = (hipStream_t)stream_;
  if (tile_len == 0) {
    // Default: 512 instructions per tile when that gives the verifier a thousand tiles or more
    // over the batch; a small batch gets shorter tiles (down to 128), so that its candidate
    // walk has workgroups for more of the device (one kernel of 8,000 instructions with 1,000
    // candidates: 0.043 ms with tiles of 128 against 0.091 ms with tiles of 512).
    uint64_t total = 0;
    for (uint32_t k = 0; k < n; ++k) total += mirs[k]->h.N;
    tile_len = kDefaultTile;
    while (tile_len > 128 && total / tile_len < 1024) tile_len /= 2;
  }
  const bool dense = (flags & VL_DENSE_POINTS) != 0;

  // recycle or create the batch
  vl_batch *batch = nullptr;
  bool fresh = false;
  if (live[0]) {
    for (uint32_t k = 0; k < n; ++k) {
      if (!live[k] || live[k]->magic != kLiveMagic || live[k]->index != k) return VL_E_ARG;
      if (live[k]->batch != live[0]->batch || live[k]->mir != mirs[k]) return VL_E_ARG;
    }
    batch = live[0]->batch;
    if (batch->n != n) return VL_E_ARG;
  } else {
    for (uint32_t k = 0; k < n; ++k)
      if (live[k]) return VL_E_ARG;
    batch = new (std::nothrow) vl_batch;
    if (!batch) return VL_E_SHAPE;
    batch->n = n;
    fresh = true;
    hipError_t e = hipGetDevice(&batch->device);
    if (e == hipSuccess) e = hipHostMalloc((void **)&batch->host_counters, (size_t)n * kCounters * 4, hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void **)&batch->stage_mirs, (size_t)n * sizeof(DevMir *), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void **)&batch->stage_a, (size_t)n * sizeof(DevLive), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void **)&batch->stage_b, (size_t)n * sizeof(DevLive), hipHostMallocDefault);
    if (e != hipSuccess) { batch_free(batch); return hip_fail(e); }
  }
  auto fail = [&](int32_t rc) {
    if (fresh) batch_free(batch);
    return rc;
  };

  // ---- arena 1 layout: [zeroed zone | counters | rest | device tables] ----
  std::vector<DevLive> h(n);
  struct Off1 { size_t last_live, vcnt, vcur, use, def, in, seed_off, seed_cur, out, tmp, vocc, ent_instr, ent_v, ent_info, first, prev,
                role, kill, item, seg_off, hull, queue, bitmap, ent_seg, ent_sf, chk, evt_cut, tile_live; };
  std::vector<Off1> off(n);
  Bump bump;
  uint32_t maxO = 1, maxV = 1, maxN = 1, maxB = 1, maxW = 1, maxT = 1, maxE = 0;
  for (uint32_t k = 0; k < n; ++k) {
    const DevMir &m = mirs[k]->h;
    const uint32_t T = (m.N + tile_len - 1) / tile_len;
    memset(&h[k], 0, sizeof(DevLive));
    h[k].T = T; h[k].tile_len = tile_len; h[k].dense = dense;
    const size_t bw = (size_t)m.B * std::max(1u, m.W) * 4;
    off[k].vcnt = bump.take((size_t)(m.V + 1) * 4);
    off[k].vcur = bump.take((size_t)(m.V + 1) * 4);
    off[k].last_live = bump.take((size_t)(m.V + 1) * 4);
    off[k].use = bump.take(bw); off[k].def = bump.take(bw); off[k].in = bump.take(bw);
    off[k].seed_off = bump.take((size_t)(T + 1) * 4); off[k].seed_cur = bump.take((size_t)(T + 1) * 4);
    off[k].item = bump.take((size_t)(m.N + m.B + 1) * 4);   // event counts are accumulated with atomics
    maxO = std::max(maxO, m.O); maxV = std::max(maxV, m.V); maxN = std::max(maxN, m.N);
    maxB = std::max(maxB, m.B); maxW = std::max(maxW, m.W); maxT = std::max(maxT, T); maxE = std::max(maxE, m.E);
  }
  const size_t o_counters = bump.take((size_t)n * kCounters * 4);
  const size_t zero_bytes = bump.off;
  for (uint32_t k = 0; k < n; ++k) {
    const DevMir &m = mirs[k]->h;
    const size_t O1 = std::max(1u, m.O), bw = (size_t)m.B * std::max(1u, m.W) * 4;
    off[k].out = bump.take(bw);
    off[k].tmp = bump.take(O1 * 4); off[k].vocc = bump.take(O1 * 4); off[k].ent_instr = bump.take(O1 * 4);
    off[k].ent_v = bump.take(O1 * 4);
    off[k].ent_info = bump.take(O1); off[k].first = bump.take((size_t)(m.V + 1) * 4); off[k].prev = bump.take(O1 * 4);
    off[k].role = bump.take(O1); off[k].kill = bump.take(O1);
    off[k].seg_off = bump.take((size_t)(m.V + 1) * 4); off[k].hull = bump.take((size_t)(m.V + 1) * 8);
    off[k].queue = bump.take((size_t)(m.V + 1) * 4);
    off[k].ent_seg = bump.take((O1 + 1) * 4);
    off[k].ent_sf = bump.take(O1);
    off[k].chk = bump.take(O1 * sizeof(u32x4));
    off[k].tile_live = bump.take((size_t)h[k].T * std::max(1u, m.W) * 4);
    off[k].evt_cut = bump.take(((size_t)(m.O + 63) / 64 + 2) * 4);
    off[k].bitmap = 0;
  }
  const size_t o_mirs = bump.take((size_t)n * sizeof(DevMir *));
  const size_t o_lives = bump.take((size_t)n * sizeof(DevLive));
  // block maps: one entry per stretch of 256 instructions, then one per stretch of 256 entries
  size_t blocks_instr = 0, blocks_occ = 0;
  for (uint32_t k = 0; k < n; ++k) {
    blocks_instr += (mirs[k]->h.N + 255u) / 256u;
    blocks_occ += (mirs[k]->h.O + 255u) / 256u;
  }
  if (blocks_instr + blocks_occ > 0x7FFFFFFFull) return fail(VL_E_RANGE);
  const size_t o_map = bump.take((blocks_instr + blocks_occ + 1) * sizeof(uint2));
  if (bump.off > batch->cap1) {
    if (batch->arena1) { VL_HIP(hipStreamSynchronize(stream)); (void)hipFree(batch->arena1); batch->arena1 = nullptr; batch->cap1 = 0; }
    hipError_t e = hipMalloc(&batch->arena1, bump.off);
    if (e != hipSuccess) return fail(hip_fail(e));
    batch->cap1 = bump.off;
  }
  char *a1 = (char *)batch->arena1;
  const DevMir **mir_ptrs = batch->stage_mirs;
  for (uint32_t k = 0; k < n; ++k) {
    DevLive &L = h[k];
    L.vcnt = (uint32_t VL_GLOBAL *)(a1 + off[k].vcnt); L.vcur = (uint32_t VL_GLOBAL *)(a1 + off[k].vcur);
    L.last_live = (uint32_t VL_GLOBAL *)(a1 + off[k].last_live);
    L.use = (uint32_t VL_GLOBAL *)(a1 + off[k].use); L.def = (uint32_t VL_GLOBAL *)(a1 + off[k].def);
    L.live_in = (uint32_t VL_GLOBAL *)(a1 + off[k].in); L.live_out = (uint32_t VL_GLOBAL *)(a1 + off[k].out);
    L.seed_off = (uint32_t VL_GLOBAL *)(a1 + off[k].seed_off); L.seed_cur = (uint32_t VL_GLOBAL *)(a1 + off[k].seed_cur);
    L.vocc_tmp = (uint32_t VL_GLOBAL *)(a1 + off[k].tmp); L.ent_v = (uint32_t VL_GLOBAL *)(a1 + off[k].ent_v); L.vocc = (uint32_t VL_GLOBAL *)(a1 + off[k].vocc);
    L.ent_instr = (uint32_t VL_GLOBAL *)(a1 + off[k].ent_instr); L.ent_info = (uint8_t VL_GLOBAL *)(a1 + off[k].ent_info);
    L.first = (uint32_t VL_GLOBAL *)(a1 + off[k].first); L.prev_occ = (uint32_t VL_GLOBAL *)(a1 + off[k].prev);
    L.occ_role = (uint8_t VL_GLOBAL *)(a1 + off[k].role); L.occ_kill = (uint8_t VL_GLOBAL *)(a1 + off[k].kill);
    L.item_off = (uint32_t VL_GLOBAL *)(a1 + off[k].item); L.seg_off = (uint32_t VL_GLOBAL *)(a1 + off[k].seg_off);
    L.hull = (uint32_t VL_GLOBAL *)(a1 + off[k].hull); L.long_queue = (uint32_t VL_GLOBAL *)(a1 + off[k].queue);
    L.ent_seg = (uint32_t VL_GLOBAL *)(a1 + off[k].ent_seg);
    L.ent_sf = (uint8_t VL_GLOBAL *)(a1 + off[k].ent_sf);
    L.chk = (u32x4 VL_GLOBAL *)(a1 + off[k].chk); L.tile_live = (uint32_t VL_GLOBAL *)(a1 + off[k].tile_live); L.evt_cut = (uint32_t VL_GLOBAL *)(a1 + off[k].evt_cut);
    L.bitmap = (uint32_t VL_GLOBAL *)nullptr;
    L.counters = (uint32_t VL_GLOBAL *)(a1 + o_counters) + (size_t)k * kCounters;
    mir_ptrs[k] = mirs[k]->dev;
  }
  batch->dev_mirs = (const DevMir **)(a1 + o_mirs);
  batch->dev_lives = (DevLive *)(a1 + o_lives);
  // Recycled handles of a call with the same options: the result sizes and the absence of
  // contract violations are known from it (the analysis of the same kernels is
  // deterministic), so nothing is read back and the host does not wait.  (The pinned staging
  // buffers are then rewritten with the bytes they already hold.)  Putting the three chains
  // that are independent after the per-occurrence pass on streams of their own shortened the
  // analysis by a sixth but cost more than that in host-side event calls; it is one stream.
  const bool known = !fresh && batch->sized && batch->sized_tile_len == tile_len && batch->sized_dense == dense;
  if (!known) batch->sized = false;

  // ---- arena 2, sized from the counts ----
  struct Off2 { size_t plan, seeds, seg, range, dense; };
  std::vector<Off2> off2(n);
  size_t zero2_lo = 0, zero2_hi = 0;
  uint32_t max_seed = 0;
  auto layout2 = [&]() -> int32_t {
    Bump b2;
    if (dense) {
      zero2_lo = b2.off;
      for (uint32_t k = 0; k < n; ++k) {
        const DevMir &m = mirs[k]->h;
        off2[k].dense = b2.take((size_t)m.N * std::max(1u, m.W) * 4);
      }
      zero2_hi = b2.off;
    }
    for (uint32_t k = 0; k < n; ++k) {
      h[k].plan_len = batch->sizes[3 * k]; h[k].n_seg = batch->sizes[3 * k + 1]; h[k].n_seed = batch->sizes[3 * k + 2];
      max_seed = std::max(max_seed, h[k].n_seed);
      off2[k].plan = b2.take(((size_t)h[k].plan_len + 8) * sizeof(u32x4));
      off2[k].seeds = b2.take((size_t)std::max(1u, h[k].n_seed) * sizeof(u32x4));
      off2[k].seg = b2.take((size_t)std::max(1u, h[k].n_seg) * 8);
      off2[k].range = b2.take((size_t)h[k].T * 8);
    }
    if (b2.off > batch->cap2) {
      if (batch->arena2) { (void)hipFree(batch->arena2); batch->arena2 = nullptr; batch->cap2 = 0; }
      hipError_t ae = hipMalloc(&batch->arena2, b2.off);
      if (ae != hipSuccess) return hip_fail(ae);
      batch->cap2 = b2.off;
    }
    char *a2 = (char *)batch->arena2;
    for (uint32_t k = 0; k < n; ++k) {
      DevLive &L = h[k];
      L.plan = (u32x4 VL_GLOBAL *)(a2 + off2[k].plan); L.seeds = (u32x4 VL_GLOBAL *)(a2 + off2[k].seeds);
      L.seg = (uint32_t VL_GLOBAL *)(a2 + off2[k].seg); L.tile_range = (uint32_t VL_GLOBAL *)(a2 + off2[k].range);
      L.live_after = dense ? (uint32_t VL_GLOBAL *)(a2 + off2[k].dense) : (uint32_t VL_GLOBAL *)nullptr;
    }
    return VL_OK;
  };
  if (known) {
    const int32_t rc2 = layout2();
    if (rc2 != VL_OK) return fail(rc2);
  }

  // pinned staging: stage_a / stage_mirs are read by the copies below; when the sizes are not
  // known yet the host waits further down and stage_b carries the second upload after that
  zero_async(a1, zero_bytes, stream);
  hipError_t e = hipSuccess;
  // with known sizes the tables on the device are usually the ones this call would upload
  const bool tables_current = known && batch->uploaded.size() == (size_t)n * sizeof(DevLive) &&
                              memcmp(batch->uploaded.data(), h.data(), batch->uploaded.size()) == 0;
  if (!tables_current) {
    batch->uploaded.clear();
    memcpy(batch->stage_a, h.data(), (size_t)n * sizeof(DevLive));
    if (e == hipSuccess) e = hipMemcpyAsync(a1 + o_mirs, mir_ptrs, (size_t)n * sizeof(DevMir *), hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(a1 + o_lives, batch->stage_a, (size_t)n * sizeof(DevLive), hipMemcpyHostToDevice, stream);
    if (e == hipSuccess && batch->map_cap < blocks_instr + blocks_occ + 1) {
      // (an earlier copy out of the old buffer is complete: growing means other kernels, and
      // then the sizes were not known and that call waited for the stream)
      if (batch->stage_map) (void)hipHostFree(batch->stage_map);
      batch->stage_map = nullptr; batch->map_cap = 0;
      e = hipHostMalloc((void **)&batch->stage_map, (blocks_instr + blocks_occ + 1) * sizeof(uint2), hipHostMallocDefault);
      if (e == hipSuccess) batch->map_cap = blocks_instr + blocks_occ + 1;
    }
    if (e == hipSuccess) {
      uint2 *at = batch->stage_map;
      for (uint32_t k = 0; k < n; ++k)
        for (uint32_t x = 0; x < (mirs[k]->h.N + 255u) / 256u; ++x) *at++ = make_uint2(k, x);
      for (uint32_t k = 0; k < n; ++k)
        for (uint32_t x = 0; x < (mirs[k]->h.O + 255u) / 256u; ++x) *at++ = make_uint2(k, x);
      e = hipMemcpyAsync(a1 + o_map, batch->stage_map, (blocks_instr + blocks_occ) * sizeof(uint2), hipMemcpyHostToDevice, stream);
    }
  }
  if (e != hipSuccess) return fail(hip_fail(e));
  const uint2 *map_instr = (const uint2 *)(a1 + o_map), *map_occ = map_instr + blocks_instr;

  const DevMir *const *dm = batch->dev_mirs;
  DevLive *dl = batch->dev_lives;
  const uint32_t TB = 256;
  // LDS histograms over the vregs when they fit (4 bytes per vreg to count, 8 to place)
  static const bool lds_ok = [] {
    hipError_t a = hipFuncSetAttribute((const void *)k_count<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    hipError_t b = hipFuncSetAttribute((const void *)k_place<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    return a == hipSuccess && b == hipSuccess;
  }();
  const bool hist_lds = lds_ok && (size_t)maxV * 4 <= 128 * 1024;
  const dim3 slices((maxO + kSlice - 1) / kSlice, n);
  if (hist_lds) k_count<true><<<slices, 1024, (size_t)maxV * 4, stream>>>(dm, dl);
  else k_count<false><<<slices, 1024, 0, stream>>>(dm, dl);
  k_scan<kScanVreg><<<n, 1024, 0, stream>>>(dm, dl);
  if (hist_lds) k_place<true><<<slices, 1024, (size_t)maxV * 4, stream>>>(dm, dl);
  else k_place<false><<<slices, 1024, 0, stream>>>(dm, dl);
  k_sort<<<dim3(kLongBlocks + (maxV + 255) / 256, n), 256, 0, stream>>>(dm, dl);
  {
    const size_t lds = std::min<size_t>((size_t)maxB * std::min(maxW, kSumWords) * 8, 48 * 1024);
    k_summary<<<grid1(maxO, kSumSlice, n), kSumThreads, lds, stream>>>(dm, dl, (uint32_t)(lds / 4));
  }
  {
    const size_t lds = ((size_t)maxB * 3 + 1) * 64 * 4 + ((size_t)maxB * 3 + 1 + maxE) * 4;
    if (lds <= 64 * 1024) k_fixpoint<true><<<grid1(maxW, 64, n), 64, lds, stream>>>(dm, dl);
    else k_fixpoint<false><<<grid1(maxW, 64, n), 64, 0, stream>>>(dm, dl);
  }
  static_assert(kEvtThreads == 256, "the block map counts stretches of 256 entries");
  if (blocks_occ) k_events<<<(uint32_t)blocks_occ, kEvtThreads, 0, stream>>>(dm, dl, map_occ);
  auto blocks = [](uint32_t items, uint32_t per) { return std::max(1u, (items + per - 1) / per); };
  const StageGrid g_count = {maxT, blocks(maxB, 4), blocks(maxN, TB * kStageReps)};
  const StageGrid g_scan = {1, 1, blocks(maxW, 1024)};
  const StageGrid g_off = {blocks(maxT, 4), blocks(maxO / 64 + 2, TB), blocks(maxV + 1, TB)};
  k_stage_count<<<dim3(g_count.a + g_count.b + g_count.c, n), 256, (size_t)maxW * 4, stream>>>(dm, dl, g_count);
  k_stage_scan<<<dim3(g_scan.a + g_scan.b + g_scan.c, n), 1024, 0, stream>>>(dm, dl, g_scan);
  k_stage_offsets<<<dim3(g_off.a + g_off.b + g_off.c, n), 256, 0, stream>>>(dm, dl, g_off);
  k_scan<kScanSeed><<<n, 1024, 0, stream>>>(dm, dl);
  e = hipGetLastError();
  if (e != hipSuccess) return fail(hip_fail(e));
  if (!known) {
    k_collect<<<(n + 63) / 64, 64, 0, stream>>>(dm, dl, n);
    e = hipMemcpyAsync(batch->host_counters, a1 + o_counters, (size_t)n * kCounters * 4, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(hip_fail(e));
    for (uint32_t k = 0; k < n; ++k)
      if (batch->host_counters[(size_t)k * kCounters + kCtrNotStrict]) return fail(VL_E_NOT_STRICT);
    batch->sizes.resize((size_t)n * 3);
    for (uint32_t k = 0; k < n; ++k) {
      const uint32_t *c = batch->host_counters + (size_t)k * kCounters;
      batch->sizes[3 * k] = c[kCtrPlanLen]; batch->sizes[3 * k + 1] = c[kCtrSeg]; batch->sizes[3 * k + 2] = c[kCtrSeed];
    }
    const int32_t rc2 = layout2();
    if (rc2 != VL_OK) return fail(rc2);
    memcpy(batch->stage_b, h.data(), (size_t)n * sizeof(DevLive));
    e = hipMemcpyAsync(a1 + o_lives, batch->stage_b, (size_t)n * sizeof(DevLive), hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return fail(hip_fail(e));
  }
  if (dense) {
    zero_async((char *)batch->arena2 + zero2_lo, zero2_hi - zero2_lo, stream);
  }
  const uint32_t per_a = blocks(maxT, 4);
  const StageGrid g_fill = {per_a * n, (uint32_t)blocks_instr, (uint32_t)blocks_occ};
  const StageGrid g_fin = {blocks(maxB, 4), blocks(maxT, TB), blocks(max_seed, TB)};
  k_stage_fill<<<g_fill.a + g_fill.b + g_fill.c, 256, 0, stream>>>(dm, dl, g_fill, per_a, map_instr, map_occ);
  k_stage_finish<<<dim3(g_fin.a + g_fin.b + g_fin.c + blocks(maxV, TB), n), 256, 0, stream>>>(dm, dl, g_fin);
  if (dense) {
    k_dense_delta<<<grid1(maxN + maxB, TB, n), TB, 0, stream>>>(dm, dl);
    k_dense_scan<<<dim3((maxW + 63) / 64, maxT, n), 64, 0, stream>>>(dm, dl);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return fail(hip_fail(e));

  // ---- handles ----
  if (fresh) {
    batch->lives.resize(n);
    for (uint32_t k = 0; k < n; ++k) {
      vl_live *l = new (std::nothrow) vl_live;
      if (!l) {
        for (uint32_t j = 0; j < k; ++j) delete batch->lives[j];
        batch_free(batch);
        return VL_E_SHAPE;
      }
      l->batch = batch; l->index = k; l->mir = mirs[k]; l->magic = kLiveMagic;
      batch->lives[k] = l;
    }
    batch->refs = n;
  }
  for (uint32_t k = 0; k < n; ++k) {
    vl_live *l = batch->lives[k];
    l->h = h[k];
    l->dev = batch->dev_lives + k;
    live[k] = l;
  }
  batch->uploaded.assign((const char *)h.data(), (const char *)h.data() + (size_t)n * sizeof(DevLive));
  batch->sized = true;
  batch->sized_tile_len = tile_len;
  batch->sized_dense = dense;
  return VL_OK;
}

extern "C" int32_t vl_liveness(const vl_mir *mir, uint32_t flags, vl_stream stream, vl_live **live) {
  if (!live) return VL_E_NULL;
  return vl_liveness_multi(&mir, 1, flags, 0, stream, live);
}

extern "C" int32_t vl_live_get(const vl_live *l, vl_live_view *v) {
  if (!l || !v) return VL_E_NULL;
  if (l->magic != kLiveMagic) return VL_E_ARG;
  const DevMir &m = l->mir->h;
  v->n_instr = m.N; v->n_vreg = m.V; v->n_block = m.B; v->n_occ = m.O; v->words = m.W;
  v->n_seg = l->h.n_seg; v->n_tile = l->h.T; v->tile_len = l->h.tile_len;
  v->plan_len = l->h.plan_len + m.O;   // occupancy events + one check per occurrence
  v->sweeps = l->batch->host_counters[(size_t)l->index * kCounters + kCtrSweeps];
  v->live_in = (const uint32_t *)l->h.live_in; v->live_out = (const uint32_t *)l->h.live_out;
  v->live_after = (const uint32_t *)l->h.live_after; v->occ_kill = (const uint8_t *)l->h.occ_kill;
  v->seg_off = (const uint32_t *)l->h.seg_off; v->seg = (const uint32_t *)l->h.seg; v->hull = (const uint32_t *)l->h.hull;
  return VL_OK;
}
