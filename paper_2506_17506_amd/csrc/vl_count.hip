// All violations of each candidate instead of the first (Section 4.5 sorts the model's
// failures into dataflow and hardware-constraint violations; Section 6 proposes the
// verifier as feedback or reward).  With T(v) = the register of v's first occurrence:
//   n_cons  occurrences whose register differs from T(their vreg)
//   n_real  mentioned vregs whose T(v) breaks a hardware rule, real_bits the rules broken
//   n_safe  pairs of one class that are in some P(i) together and whose tuples overlap
// The pairs (the interference relation) depend on the program only: they are enumerated
// once per program from the live intervals and kept with the program handle.  Per call the
// registers T are gathered into a table [vreg][candidate], so that a wavefront that walks
// the pairs with one candidate per lane reads one line per endpoint.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <utility>
#include <vector>

#include "vl_dev.h"

using namespace vl;

namespace {

// ---- interference pairs ------------------------------------------------------------------
// do the interval lists [a0, a1) and [b0, b1) of `seg` (ascending runs [start, end)) share a point?
__device__ inline bool lists_meet(const uint32_t VL_GLOBAL *seg, uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1) {
  uint32_t x = a0, y = b0;
  while (x < a1 && y < b1) {
    const uint32_t xs = seg[2 * (size_t)x], xe = seg[2 * (size_t)x + 1], ys = seg[2 * (size_t)y], ye = seg[2 * (size_t)y + 1];
    if (max(xs, ys) < min(xe, ye)) return true;
    if (xe <= ye) ++x; else ++y;
  }
  return false;
}

// One wavefront per vreg a, its lanes striding over b > a; blockIdx.y = program.  kFill = false:
// cnt[a] = number of partners; kFill = true: the pairs are written from off[a] on, in ascending b,
// each vreg with its width in the upper byte (vreg numbers stay below 2^24: VL_MAX_VREG).
// Vregs are taken 64 at a time, and a group whose hulls taken together ([earliest start, latest
// end), from k_hull_groups) miss a's hull is passed over: vregs are mostly numbered in the
// order they are first written, so most groups lie entirely before or after a.
struct PairJob {
  const DevMir *mir;
  const DevLive *live;
  uint32_t *cnt;         // [V]
  const uint64_t *off;   // [V]
  uint32_t *pairs;       // [n_pairs rounded up to 32][2]: vreg | width << 24
  uint2 *groups;         // [(V + 63) / 64] (earliest start, latest end) of the group's non-empty hulls
};

// one wavefront per group of 64 vregs
__global__ __launch_bounds__(256) void k_hull_groups(const PairJob *__restrict__ jobs) {
  const PairJob &J = jobs[blockIdx.y];
  const DevMir VL_GLOBAL &m = *as_global(J.mir);
  const DevLive VL_GLOBAL &L = *as_global(J.live);
  const uint32_t lane = threadIdx.x & 63u, g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if ((size_t)g * 64 >= m.V) return;
  const uint32_t v = g * 64 + lane;
  uint32_t lo = 0xFFFFFFFFu, hi = 0;
  if (v < m.V && L.hull[2 * (size_t)v + 1] != 0) { lo = L.hull[2 * (size_t)v]; hi = L.hull[2 * (size_t)v + 1]; }   // (0, 0): never in any P(i)
  for (int d = 32; d >= 1; d >>= 1) {
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, d, 64));
  }
  if (lane == 0) J.groups[g] = make_uint2(lo, hi);
}

// off[a] = number of pairs of the vregs below a, totals[program] = all of them: one workgroup
// per program, a contiguous run of vregs per thread
__global__ __launch_bounds__(1024) void k_pair_offsets(const PairJob *__restrict__ jobs, uint64_t *__restrict__ totals) {
  const PairJob &J = jobs[blockIdx.x];
  const uint32_t V = as_global(J.mir)->V;
  uint64_t *off = const_cast<uint64_t *>(J.off);   // written here, read by the filling launch
  __shared__ uint64_t part[16];
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t per = (V + 1023u) / 1024u, lo = min(V, threadIdx.x * per), hi = min(V, lo + per);
  uint64_t mine = 0;
  for (uint32_t a = lo; a < hi; ++a) mine += J.cnt[a];
  uint64_t incl = mine;
  for (int d = 1; d < 64; d <<= 1) {
    const uint64_t y = __shfl_up(incl, d, 64);
    if ((int)lane >= d) incl += y;
  }
  if (lane == 63) part[wave] = incl;
  __syncthreads();
  uint64_t run = incl - mine, total = 0;
  for (uint32_t k = 0; k < 16; ++k) {
    if (k < wave) run += part[k];
    total += part[k];
  }
  for (uint32_t a = lo; a < hi; ++a) { off[a] = run; run += J.cnt[a]; }
  if (threadIdx.x == 0) totals[blockIdx.x] = total;
}

template <bool kFill>
__global__ __launch_bounds__(256) void k_pairs(const PairJob *__restrict__ jobs) {
  const PairJob &J = jobs[blockIdx.y];
  const DevMir VL_GLOBAL &m = *as_global(J.mir);
  const DevLive VL_GLOBAL &L = *as_global(J.live);
  const uint32_t lane = threadIdx.x & 63u, a = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (a >= m.V) return;   // whole wavefronts leave; nothing below synchronises the workgroup
  const uint32_t h0 = L.hull[2 * (size_t)a], h1 = L.hull[2 * (size_t)a + 1];
  const uint32_t s0 = L.seg_off[a], s1 = L.seg_off[a + 1], cls = attr_class(m.vattr[a]), width_a = attr_width(m.vattr[a]);
  uint64_t at = kFill ? J.off[a] : 0;
  uint32_t n = 0;
  const uint32_t n_groups = (m.V + 63u) / 64u;
  for (uint32_t g0 = a / 64; g0 < n_groups; g0 += 64) {   // 64 groups at a time, one per lane
    uint2 span = make_uint2(0xFFFFFFFFu, 0u);
    if (g0 + lane < n_groups) span = J.groups[g0 + lane];
    uint64_t todo = __ballot(span.x < h1 && h0 < span.y);
    while (todo) {
      const uint32_t b = (g0 + (uint32_t)__builtin_ctzll(todo)) * 64 + lane;
      todo &= todo - 1;
      bool hit = false;
      const uint32_t attr_b = b > a && b < m.V ? m.vattr[b] : 0u;
      if (b > a && b < m.V && attr_class(attr_b) == cls && L.hull[2 * (size_t)b] < h1 && h0 < L.hull[2 * (size_t)b + 1])
        hit = lists_meet(L.seg, s0, s1, L.seg_off[b], L.seg_off[b + 1]);
      const uint64_t hits = __ballot(hit);
      if (kFill) {
        if (hit) {
          const uint64_t pos = at + __popcll(hits & ((1ull << lane) - 1ull));
          J.pairs[2 * pos] = a | (width_a << 24);
          J.pairs[2 * pos + 1] = b | (attr_width(attr_b) << 24);
        }
        at += __popcll(hits);
      } else {
        n += __popcll(hits);
      }
    }
  }
  if (!kFill && lane == 0) J.cnt[a] = n;
  // the list ends with pairs of the last vreg with itself, widths 0 (they overlap nothing and
  // keep a ascending), up to the next multiple of 32 pairs, so that it can be read in pieces
  // without a tail
  if (kFill && a == m.V - 1 && (at & 31u) && lane < 32u - (uint32_t)(at & 31u)) {
    J.pairs[2 * (at + lane)] = a;
    J.pairs[2 * (at + lane) + 1] = a;
  }
}

// ---- per call ----------------------------------------------------------------------------
struct DevCountJob {
  const DevMir *mir;
  const DevLive *live;
  const uint16_t *cand;
  vl_counts *out;
  uint16_t *table;         // [V][k_pad] registers of the first occurrences
  const uint32_t *pairs;   // [n_pairs rounded up to 32][2]: vreg | width << 24, the padding of width 0
  uint64_t ld, n_pairs;
  uint32_t K, k_pad, V, pad1;
};

__global__ void k_cnt_clear(const DevCountJob *__restrict__ jobs) {
  const DevCountJob &J = jobs[blockIdx.y];
  const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k < J.K) J.out[k] = vl_counts{0, 0, 0, 0, 0, {0, 0, 0}};
}

// table[v][k] = cand[k][first[v]] through a 64 x 64 tile in LDS: reads run along a candidate
// row (first occurrences mostly ascend with the vreg), writes along the candidates.  The
// thread that writes a candidate's entries also tests them against the hardware rules
// (realizability: the vregs that are mentioned, each once).
__global__ __launch_bounds__(256) void k_cnt_table(const DevCountJob *__restrict__ jobs, uint32_t tiles_k) {
  const DevCountJob &J = jobs[blockIdx.y];
  const DevMir VL_GLOBAL &m = *as_global(J.mir);
  const DevLive VL_GLOBAL &L = *as_global(J.live);
  const uint32_t v0 = (blockIdx.x / tiles_k) * 64, k0 = (blockIdx.x % tiles_k) * 64;
  if (v0 >= m.V || k0 >= J.k_pad) return;
  __shared__ uint16_t tile[64][66];
  __shared__ uint32_t attrs[64];   // kNone: never mentioned, or past the last vreg
  const uint32_t tx = threadIdx.x & 63u, ty = threadIdx.x >> 6;
  const uint32_t v = v0 + tx;
  const uint32_t fo = v < m.V ? L.first[v] : kNone;
  if (ty == 0) attrs[tx] = fo != kNone ? m.vattr[v] : kNone;
  for (uint32_t kk = ty; kk < 64; kk += 4) {
    const uint32_t k = k0 + kk;
    tile[kk][tx] = (k < J.K && fo != kNone) ? J.cand[(uint64_t)k * J.ld + fo] : (uint16_t)0;
  }
  __syncthreads();
  uint32_t n = 0, bits = 0;
  for (uint32_t vv = ty; vv < 64; vv += 4) {
    if (v0 + vv >= m.V || k0 + tx >= J.k_pad) continue;
    const uint32_t p = tile[tx][vv];
    J.table[(size_t)(v0 + vv) * J.k_pad + k0 + tx] = (uint16_t)p;
    if (attrs[vv] == kNone) continue;
    const uint32_t bad = bad_bits(m, attrs[vv], p);
    n += bad != 0;
    bits |= bad;
  }
  if (k0 + tx < J.K && n) {
    atomicAdd(&J.out[k0 + tx].n_real, n);
    atomicOr(&J.out[k0 + tx].real_bits, bits);
  }
}

// consistency: a workgroup takes 64 candidates (blockIdx.y) and 1024 occurrences.  64
// occurrences of the 64 rows at a time go through LDS, read along the rows; then a lane is a
// candidate and compares, occurrence by occurrence, its register with its entry in the
// table row of the occurrence's vreg (one coalesced read for the 64 candidates).
__global__ __launch_bounds__(256) void k_cnt_cons(const DevCountJob *__restrict__ jobs) {
  const DevCountJob &J = jobs[blockIdx.z];
  const DevMir VL_GLOBAL &m = *as_global(J.mir);
  const uint32_t k0 = blockIdx.y * 64, o0 = blockIdx.x * 1024;
  if (k0 >= J.K || o0 >= m.O) return;
  __shared__ uint16_t tile[64][66];
  const uint32_t lane = threadIdx.x & 63u, first = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) * 16u;
  const uint32_t o_end = min(m.O, o0 + 1024u);
  uint32_t n = 0;
  for (uint32_t oc = o0; oc < o_end; oc += 64) {
    const bool in = oc + lane < o_end;
    // this wavefront's 16 rows, all loads in flight together
    uint16_t mine[16];
#pragma unroll
    for (uint32_t u = 0; u < 16; ++u) {
      const uint32_t k = k0 + first + u;
      mine[u] = (in && k < J.K) ? J.cand[(uint64_t)k * J.ld + oc + lane] : (uint16_t)0;
    }
    const uint32_t my_v = in ? m.occ_vreg[oc + lane] : 0u;
#pragma unroll
    for (uint32_t u = 0; u < 16; ++u) tile[first + u][lane] = mine[u];
    __syncthreads();
    const uint32_t cnt = min(64u, o_end - oc);
    // this wavefront's quarter of the 64 occurrences; rows past the last candidate hold zeros
    // in the tile and in the table
    uint32_t q[16];
#pragma unroll
    for (uint32_t u = 0; u < 16; ++u)
      q[u] = J.table[(size_t)__builtin_amdgcn_readlane(my_v, first + u) * J.k_pad + k0 + lane];
#pragma unroll
    for (uint32_t u = 0; u < 16; ++u) n += (first + u < cnt && tile[lane][first + u] != q[u]) ? 1u : 0u;
    __syncthreads();
  }
  if (k0 + lane < J.K && n) atomicAdd(&J.out[k0 + lane].n_cons, n);
}

// safety: the wavefronts of a program take its pairs in stretches of 256 and walk each once
// for every group of 128 candidates: a lane holds two neighbouring candidates, whose registers
// are one 32-bit word of a table row.  Both are tested at once with saturating 16-bit
// arithmetic, exact for any 16-bit register number: with u = max(pa - pb, 0) and
// v = max(pb - pa, 0), the tuples overlap iff u < width(b) and v < width(a).  What bounds the
// kernel is the number of instructions a pair takes, of any kind: seven vector ones for the
// test; the pairs (with the widths in their upper bytes) arrive through scalar loads, sixteen
// pairs at a time and the next sixteen fetched ahead, and a table row is addressed by a scalar
// offset plus the lane's own.  The pairs are stored in ascending (a, b), so the sixteen mostly
// share a, whose row is then read once.
// A program has at most 1024 workgroups, whose wavefronts take its stretches in turn.  (Running
// all workgroups of a program on one of the eight dies, so that its table stays in one L2, cut
// the memory traffic by ten and made the kernel slower: the dies were then unevenly loaded.)
constexpr uint32_t kPairsPerWave = 256, kPairsPerGroup = 4 * kPairsPerWave, kSafeGroupsPerProgram = 1024;
constexpr uint32_t kPairsAtOnce = 16;   // the pair list of a program is padded with empty pairs to a multiple of this
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
#define VL_CONSTANT __attribute__((address_space(4)))
__device__ inline u16x2 both(uint32_t x) { return __builtin_bit_cast(u16x2, x); }
template <bool kBig>
__global__ __launch_bounds__(256) void k_cnt_safe(const DevCountJob *__restrict__ jobs) {
  const DevCountJob &J = jobs[blockIdx.y];
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t n_waves = gridDim.x * 4u;
  const uint32_t wave = blockIdx.x * 4u + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if ((uint64_t)wave * kPairsPerWave >= J.n_pairs) return;
  const uint32_t words = J.k_pad / 2;   // 32-bit words per table row (k_pad is a multiple of 64)
  const uint32_t row_bytes = words * 4u;
  // 1 in both halves, in a form the compiler cannot see through: a minimum with a known 1 is
  // turned into two compares and a merge instead of one packed instruction
  u16x2 one;
  asm volatile("v_mov_b32 %0, 0x10001" : "=v"(one));
  for (uint32_t w0 = 0; w0 < words; w0 += 64) {
    // lanes past the row repeat its last word; not counted
    const uint32_t lane_off = min(w0 + lane, words - 1) * 4u;
    // A row is fetched with a buffer read: descriptor and row offset in scalar registers, the
    // lane brings its offset inside the row.  The scalar offset has 32 bits; for a table of
    // 4 GB or more (kBig) every row gets a descriptor of its own instead.
    const __amdgpu_buffer_rsrc_t whole = __builtin_amdgcn_make_buffer_rsrc((void *)J.table, 0, kBig ? 0 : (int)(J.V * row_bytes), 0x00020000);
    auto row = [&](uint32_t packed) __attribute__((always_inline)) {   // this lane's word of the row of vreg (packed & 0xFFFFFF)
      const uint32_t v = packed & 0xFFFFFFu;
      if (kBig) {
        const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((char *)J.table + (uint64_t)v * row_bytes, 0, (int)row_bytes, 0x00020000);
        return both(__builtin_amdgcn_raw_buffer_load_b32(r, lane_off, 0, 0));
      }
      return both(__builtin_amdgcn_raw_buffer_load_b32(whole, lane_off, v * row_bytes, 0));
    };
    auto width2 = [&](uint32_t packed) __attribute__((always_inline)) {
      const uint16_t width = (uint16_t)(packed >> 24);
      return u16x2{width, width};
    };
    uint32_t n_lo = 0, n_hi = 0;
    for (uint64_t e0 = (uint64_t)wave * kPairsPerWave; e0 < J.n_pairs; e0 += (uint64_t)n_waves * kPairsPerWave) {
      const uint64_t e1 = min(J.n_pairs, e0 + kPairsPerWave);
      // eight pairs per 64-byte piece; e0 is a multiple of 256
      const u32x16 VL_CONSTANT *pieces = (const u32x16 VL_CONSTANT *)(uintptr_t)(J.pairs + 2 * e0);
      u16x2 n = {0, 0};   // at most 256 per half
      auto count = [&](u16x2 ra, u16x2 rb, u16x2 sa, u16x2 sb) __attribute__((always_inline)) {
        const u16x2 u = __builtin_elementwise_sub_sat(ra, rb), v = __builtin_elementwise_sub_sat(rb, ra);
        const u16x2 room = __builtin_elementwise_min(__builtin_elementwise_sub_sat(sb, u), __builtin_elementwise_sub_sat(sa, v));
        n += __builtin_elementwise_min(room, one);
      };
      const uint32_t n_groups = (uint32_t)((e1 - e0 + kPairsAtOnce - 1) / kPairsAtOnce);
      auto group = [&](const u32x16 lo, const u32x16 hi) __attribute__((always_inline)) {
        u16x2 rb[kPairsAtOnce];
        if ((lo[0] & 0xFFFFFFu) == (hi[14] & 0xFFFFFFu)) {
          // the usual case: one row for a
          const u16x2 ra = row(lo[0]), sa = width2(lo[0]);
#pragma unroll
          for (uint32_t t = 0; t < 8; ++t) { rb[t] = row(lo[2 * t + 1]); rb[8 + t] = row(hi[2 * t + 1]); }
          __builtin_amdgcn_s_waitcnt(0x0F70);   // all rows at once (vmcnt 0) rather than one wait per pair
#pragma unroll
          for (uint32_t t = 0; t < 8; ++t) count(ra, rb[t], sa, width2(lo[2 * t + 1]));
#pragma unroll
          for (uint32_t t = 0; t < 8; ++t) count(ra, rb[8 + t], sa, width2(hi[2 * t + 1]));
        } else {
          u16x2 ra[kPairsAtOnce];
#pragma unroll
          for (uint32_t t = 0; t < 8; ++t) {
            ra[t] = row(lo[2 * t]); rb[t] = row(lo[2 * t + 1]);
            ra[8 + t] = row(hi[2 * t]); rb[8 + t] = row(hi[2 * t + 1]);
          }
          __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
          for (uint32_t t = 0; t < 8; ++t) count(ra[t], rb[t], width2(lo[2 * t]), width2(lo[2 * t + 1]));
#pragma unroll
          for (uint32_t t = 0; t < 8; ++t) count(ra[8 + t], rb[8 + t], width2(hi[2 * t]), width2(hi[2 * t + 1]));
        }
      };
      // two groups per turn, each one's pairs fetched while the other is counted
      u32x16 a_lo = pieces[0], a_hi = pieces[1];
      for (uint32_t g = 0; g < n_groups; g += 2) {
        u32x16 b_lo = a_lo, b_hi = a_hi;
        if (g + 1 < n_groups) { b_lo = pieces[2 * g + 2]; b_hi = pieces[2 * g + 3]; }
        group(a_lo, a_hi);
        if (g + 1 < n_groups) {
          if (g + 2 < n_groups) { a_lo = pieces[2 * g + 4]; a_hi = pieces[2 * g + 5]; }
          group(b_lo, b_hi);
        }
      }
      n_lo += n.x;
      n_hi += n.y;
    }
    const uint32_t k = 2 * (w0 + lane);
    if (w0 + lane < words) {
      if (k < J.K && n_lo) atomicAdd(&J.out[k].n_safe, n_lo);
      if (k + 1 < J.K && n_hi) atomicAdd(&J.out[k + 1].n_safe, n_hi);
    }
  }
}

__global__ void k_cnt_kinds(const DevCountJob *__restrict__ jobs) {
  const DevCountJob &J = jobs[blockIdx.y];
  const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= J.K) return;
  vl_counts &c = J.out[k];
  c.kinds = (c.n_cons ? 1u : 0u) | (c.n_real ? 2u : 0u) | (c.n_safe ? 4u : 0u);
}

// per-device workspace: the job table (device + pinned copy) and the register tables
struct Work {
  std::mutex mu;
  DevCountJob *dev = nullptr, *host = nullptr;
  uint32_t cap = 0;
  void *tables = nullptr;
  size_t tables_cap = 0;
  hipEvent_t consumed = nullptr;   // recorded after the last kernel of a call
};
Work g_work[16];

// Enumerates the interference pairs of the programs that do not have them yet, from the
// intervals of their analyses (which must be complete or enqueued on `stream`): one counting
// launch over all of them, the offsets summed per program on the device, one filling launch.  Synchronises
// the stream twice.
int32_t build_pairs(const std::vector<std::pair<vl_mir *, const vl_live *>> &todo, hipStream_t stream) {
  const size_t n = todo.size();
  size_t total_v = 0;
  uint32_t max_v = 0;
  std::vector<size_t> base(n);
  for (size_t j = 0; j < n; ++j) {
    base[j] = total_v;
    total_v += todo[j].first->h.V;
    max_v = std::max(max_v, todo[j].first->h.V);
  }
  if (total_v == 0) {
    for (auto &t : todo) { t.first->edges = nullptr; t.first->n_edges = 0; t.first->edges_built = true; }
    return VL_OK;
  }
  // device scratch: counts, offsets, the job table; host: the same, pageable (copies wait for the stream)
  uint32_t *cnt = nullptr;
  uint64_t *off = nullptr;
  uint2 *groups = nullptr;
  uint64_t *totals_dev = nullptr;
  PairJob *jobs_dev = nullptr;
  void *all_pairs = nullptr;   // one allocation for the pairs of every program of this call, handed to them on success
  auto cleanup = [&]() { (void)hipFree(cnt); (void)hipFree(off); (void)hipFree(groups); (void)hipFree(totals_dev); (void)hipFree(jobs_dev); };
  auto fail = [&](hipError_t err) {
    cleanup();
    (void)hipFree(all_pairs);
    return hip_fail(err);
  };
  // (a kernel's groups start at base / 64 + its index: at most one entry per kernel is left unused)
  hipError_t e = hipMalloc((void **)&cnt, total_v * 4);
  if (e == hipSuccess) e = hipMalloc((void **)&off, total_v * 8);
  if (e == hipSuccess) e = hipMalloc((void **)&groups, (total_v / 64 + n + 1) * sizeof(uint2));
  if (e == hipSuccess) e = hipMalloc((void **)&totals_dev, n * 8);
  if (e == hipSuccess) e = hipMalloc((void **)&jobs_dev, n * sizeof(PairJob));
  if (e != hipSuccess) return fail(e);
  std::vector<PairJob> jobs(n);
  for (size_t j = 0; j < n; ++j)
    jobs[j] = PairJob{todo[j].first->dev, todo[j].second->dev, cnt + base[j], off + base[j], nullptr, groups + base[j] / 64 + j};
  e = hipMemcpyAsync(jobs_dev, jobs.data(), n * sizeof(PairJob), hipMemcpyHostToDevice, stream);
  if (e != hipSuccess) return fail(e);
  const dim3 grid((max_v + 3) / 4, (uint32_t)n);
  k_hull_groups<<<dim3(((max_v + 63) / 64 + 3) / 4, (uint32_t)n), 256, 0, stream>>>(jobs_dev);
  k_pairs<false><<<grid, 256, 0, stream>>>(jobs_dev);
  k_pair_offsets<<<(uint32_t)n, 1024, 0, stream>>>(jobs_dev, totals_dev);
  std::vector<uint64_t> totals(n), first_pair(n);
  e = hipMemcpyAsync(totals.data(), totals_dev, n * 8, hipMemcpyDeviceToHost, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e != hipSuccess) return fail(e);
  uint64_t all = 0;
  for (size_t j = 0; j < n; ++j) {
    first_pair[j] = all;
    all += (totals[j] + 31) & ~(uint64_t)31;   // every program's pairs start on a 256-byte boundary
  }
  if (all) {
    e = hipMalloc(&all_pairs, (size_t)all * 8);
    if (e != hipSuccess) return fail(e);
  }
  for (size_t j = 0; j < n; ++j) jobs[j].pairs = totals[j] ? (uint32_t *)all_pairs + 2 * first_pair[j] : nullptr;
  e = hipMemcpyAsync(jobs_dev, jobs.data(), n * sizeof(PairJob), hipMemcpyHostToDevice, stream);
  if (e == hipSuccess) {
    k_pairs<true><<<grid, 256, 0, stream>>>(jobs_dev);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipStreamSynchronize(stream);   // the host vectors and the scratch go away below
  if (e != hipSuccess) return fail(e);
  cleanup();
  EdgeBlock *block = nullptr;
  if (all_pairs) {
    uint32_t holders = 0;
    for (size_t j = 0; j < n; ++j) holders += totals[j] != 0;
    block = new (std::nothrow) EdgeBlock{all_pairs, {holders}};
    if (!block) { (void)hipFree(all_pairs); return VL_E_SHAPE; }
  }
  for (size_t j = 0; j < n; ++j) {
    todo[j].first->edges = jobs[j].pairs;
    todo[j].first->n_edges = totals[j];
    todo[j].first->edge_block = totals[j] ? block : nullptr;
    todo[j].first->edges_built = true;
  }
  return VL_OK;
}

}  // namespace

extern "C" int32_t vl_count_violations_multi(const vl_count_job *jobs, uint32_t n_jobs, vl_stream stream_) {
  if (!jobs) return VL_E_NULL;
  if (n_jobs == 0 || n_jobs > 65535) return VL_E_SHAPE;
  for (uint32_t j = 0; j < n_jobs; ++j) {
    const vl_count_job &u = jobs[j];
    if (!u.mir || !u.live || !u.cand || !u.out) return VL_E_NULL;
    if (u.mir->magic != kMirMagic || u.live->magic != kLiveMagic || u.live->mir != u.mir || u.mir->lowered) return VL_E_ARG;
    if (u.K == 0 || u.K > 65535 || u.ld < u.mir->h.O) return VL_E_SHAPE;
  }
  hipStream_t stream = (hipStream_t)stream_;
  int device = 0;
  VL_HIP(hipGetDevice(&device));
  if (device < 0 || device >= 16) return VL_E_ARG;
  Work &w = g_work[device];
  std::lock_guard<std::mutex> lock(w.mu);
  // the pairs of programs seen for the first time (the handle is the cache: not const here)
  {
    std::vector<std::pair<vl_mir *, const vl_live *>> todo;
    for (uint32_t j = 0; j < n_jobs; ++j) {
      vl_mir *mir = const_cast<vl_mir *>(jobs[j].mir);
      if (!mir->edges_built) todo.emplace_back(mir, jobs[j].live);
    }
    // the same program may appear in several jobs
    std::sort(todo.begin(), todo.end(), [](const auto &x, const auto &y) { return x.first < y.first; });
    todo.erase(std::unique(todo.begin(), todo.end(), [](const auto &x, const auto &y) { return x.first == y.first; }), todo.end());
    if (!todo.empty()) {
      const int32_t rc = build_pairs(todo, stream);
      if (rc != VL_OK) return rc;
    }
  }
  // the previous call's kernels must be done with the job table and the register tables
  if (w.consumed) VL_HIP(hipEventSynchronize(w.consumed));
  if (w.cap < n_jobs) {
    if (w.dev) (void)hipFree(w.dev);
    if (w.host) (void)hipHostFree(w.host);
    w.dev = nullptr; w.host = nullptr; w.cap = 0;
    const uint32_t cap = std::max(256u, n_jobs);
    VL_HIP(hipMalloc((void **)&w.dev, (size_t)cap * sizeof(DevCountJob)));
    VL_HIP(hipHostMalloc((void **)&w.host, (size_t)cap * sizeof(DevCountJob), hipHostMallocDefault));
    w.cap = cap;
  }
  if (!w.consumed) VL_HIP(hipEventCreateWithFlags(&w.consumed, hipEventDisableTiming));
  size_t bytes = 0;
  std::vector<size_t> at(n_jobs);
  uint32_t maxK = 0, maxV = 1, maxO = 1, max_kpad = 64;
  uint64_t max_pairs = 0;
  bool big_table = false;   // some table has 4 GB or more
  for (uint32_t j = 0; j < n_jobs; ++j) {
    const uint32_t k_pad = (jobs[j].K + 63u) & ~63u;
    at[j] = bytes;
    bytes += (((size_t)jobs[j].mir->h.V * k_pad * 2) + 255) & ~(size_t)255;
    maxK = std::max(maxK, jobs[j].K); maxV = std::max(maxV, jobs[j].mir->h.V); maxO = std::max(maxO, jobs[j].mir->h.O);
    max_kpad = std::max(max_kpad, k_pad);
    max_pairs = std::max(max_pairs, jobs[j].mir->n_edges);
    big_table |= (uint64_t)jobs[j].mir->h.V * k_pad * 2 >= (1ull << 32);
  }
  if (bytes > w.tables_cap) {
    if (w.tables) (void)hipFree(w.tables);
    w.tables = nullptr; w.tables_cap = 0;
    VL_HIP(hipMalloc(&w.tables, bytes));
    w.tables_cap = bytes;
  }
  for (uint32_t j = 0; j < n_jobs; ++j) {
    DevCountJob &d = w.host[j];
    memset(&d, 0, sizeof(d));
    d.mir = jobs[j].mir->dev; d.live = jobs[j].live->dev; d.cand = jobs[j].cand; d.out = jobs[j].out;
    d.table = (uint16_t *)((char *)w.tables + at[j]);
    d.pairs = (const uint32_t *)jobs[j].mir->edges; d.n_pairs = jobs[j].mir->n_edges;
    d.ld = jobs[j].ld; d.K = jobs[j].K; d.k_pad = (jobs[j].K + 63u) & ~63u; d.V = jobs[j].mir->h.V;
  }
  VL_HIP(hipMemcpyAsync(w.dev, w.host, (size_t)n_jobs * sizeof(DevCountJob), hipMemcpyHostToDevice, stream));
  const uint32_t tiles_k = max_kpad / 64, tiles_v = (maxV + 63) / 64;
  const uint32_t stretches = (uint32_t)std::min<uint64_t>(1u << 20, std::max<uint64_t>(1, (max_pairs + kPairsPerGroup - 1) / kPairsPerGroup));
  k_cnt_clear<<<dim3((maxK + 255) / 256, n_jobs), 256, 0, stream>>>(w.dev);
  k_cnt_table<<<dim3(tiles_v * tiles_k, n_jobs), 256, 0, stream>>>(w.dev, tiles_k);
  k_cnt_cons<<<dim3((maxO + 1023) / 1024, tiles_k, n_jobs), 256, 0, stream>>>(w.dev);
  {
    const dim3 grid(std::min(stretches, kSafeGroupsPerProgram), n_jobs);
    if (big_table) k_cnt_safe<true><<<grid, 256, 0, stream>>>(w.dev);
    else k_cnt_safe<false><<<grid, 256, 0, stream>>>(w.dev);
  }
  k_cnt_kinds<<<dim3((maxK + 255) / 256, n_jobs), 256, 0, stream>>>(w.dev);
  VL_HIP(hipGetLastError());
  VL_HIP(hipEventRecord(w.consumed, stream));
  return VL_OK;
}
