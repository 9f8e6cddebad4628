// Internal device-side layouts shared by the liveness and verification kernels.
#ifndef VL_DEV_H
#define VL_DEV_H
#include <hip/hip_runtime.h>

#include <atomic>
#include <stdint.h>

#include "../../include/vl.h"

// Device arrays reached through the structures below are declared as pointers into global
// memory, so that the compiler emits global / scalar loads for them rather than flat ones.
#define VL_GLOBAL __attribute__((address_space(1)))

namespace vl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kMaxClass = 8;
constexpr uint32_t kMaxOperands = 64;      // per instruction
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint32_t kDefaultTile = 512;     // instructions per verification tile

// Kernel (program) on the device.  All pointers are device memory.
struct DevMir {
  uint32_t N, V, B, O, C, E, W;
  uint32_t occ_words;              // occupancy words per candidate: every class may address 16 words from its
                                   // first one (classes are laid out smallest first, so this is rarely more
                                   // than the words the files need)
  const uint32_t VL_GLOBAL *blk_start;       // [B+1]
  const uint32_t VL_GLOBAL *succ_off;        // CSR successors
  const uint32_t VL_GLOBAL *succ;
  const uint32_t VL_GLOBAL *occ_off;         // [N+1]
  const uint32_t VL_GLOBAL *occ_vreg;        // [O]
  const uint32_t VL_GLOBAL *occ_instr;       // [O] instruction of each occurrence
  const uint32_t VL_GLOBAL *instr_blk;       // [N] block of each instruction
  const uint32_t VL_GLOBAL *vattr;           // [V] packed attributes, see attr_* below
  const uint8_t VL_GLOBAL *occ_flags;        // [O]
  const uint64_t VL_GLOBAL *occ_rec;         // [O] vreg | (instruction << 2 | DEF/USE flags) << 32: one read instead of three
  const uint8_t VL_GLOBAL *instr_keep;       // [N] 1 iff the instruction has an early-clobber definition: what it reads
                                             // stays occupied through it
  // a program made by vl_mir_create_lanes (every lane of a partly accessed vreg a value of its own): for
  // each of its occurrences the caller's occurrence, for each of its values the caller's vreg; else null
  const uint32_t VL_GLOBAL *occ_src;         // [O]
  const uint32_t VL_GLOBAL *val_vreg;        // [V]
  uint32_t has_reserved;
  uint16_t class_size[kMaxClass];
  uint16_t class_word[kMaxClass];  // first occupancy word of the class
  uint32_t reserved[kMaxClass][16];
};

// Packed vreg attributes: class | (width-1) << 3 | (align-1) << 8 | straddle << 13.
// straddle = a correctly aligned tuple may cross a 32-register word.
__host__ __device__ inline uint32_t attr_pack(uint32_t cls, uint32_t width, uint32_t align) {
  bool word_safe = (32u % align == 0u) && width <= align;
  return cls | ((width - 1u) << 3) | ((align - 1u) << 8) | ((word_safe ? 0u : 1u) << 13);
}
__host__ __device__ inline uint32_t attr_class(uint32_t a) { return a & 7u; }
__host__ __device__ inline uint32_t attr_width(uint32_t a) { return ((a >> 3) & 31u) + 1u; }
__host__ __device__ inline uint32_t attr_align(uint32_t a) { return ((a >> 8) & 31u) + 1u; }
__host__ __device__ inline uint32_t attr_straddle(uint32_t a) { return (a >> 13) & 1u; }
// bits 16 and up of a program's vattr[]: the first occupancy-mask word of the vreg's class
__host__ __device__ inline uint32_t attr_word(uint32_t a) { return a >> 16; }
__host__ __device__ inline uint64_t entry_pack(uint32_t x, uint32_t y) { return (uint64_t)x | ((uint64_t)y << 32); }

// The verifier reads
// "chk": one 16-byte record per occurrence, in occurrence order, everything a consistency /
//   realizability check needs that does not depend on the candidate:
//   x: flags (kPlanChk or kPlanFirst, kPlanKeep, kChkNear, kChkGeneric)
//      | ring slot of the occurrence << 8 | ring slot of the previous occurrence of the
//      same vreg << 20 (slot = index % kWalkRing; the verifier scales it by its row pitch)
//   y: distance to that previous occurrence (16 bits, saturated) | packed attributes << 16
//   z: alignment - 1 in both halves (two candidates per 32-bit operation); 0 when nothing is to be tested
//   w: the largest base that fits, in both halves; all ones when there is no limit
// "seeds": per tile, the values live into it, as event records (below) whose x holds only the vreg:
//   w names an occurrence of the vreg, from which the candidate's register is taken
// "plan": the occupancy events in the order they take effect, as 16-byte records (below).
// For each instruction: releases of operands that die there, then test-and-occupy of the
// values it writes, then releases of values dead once it has executed; the events of a
// block boundary (values that stop / start being live between two blocks adjacent in the
// linear order) precede those of the later block's first instruction.
constexpr uint32_t kPlanChk = 1u;    // compare with the previous occurrence of the vreg
constexpr uint32_t kPlanFirst = 2u;  // first occurrence of the vreg: realizability check
constexpr uint32_t kChkNear = 4u;    // the previous occurrence is still in the ring when this one is checked
                                     // (unless the tile starts in between)
constexpr uint32_t kChkGeneric = 8u; // realizability needs the general test: alignment not a power of two,
                                     // reserved registers, or a tuple wider than its file
constexpr uint32_t kPlanKeep = 64u;  // (chk) the next occurrence of the vreg is likely beyond the verifier's
                                     // LDS window: worth keeping this one's registers at hand

// Geometry of the verifier's LDS window, which the analysis needs for kPlanKeep: occurrences
// are staged kWalkChunk at a time into a ring of kWalkRing.
constexpr uint32_t kWalkChunk = 64, kWalkRing = 192;
// While a chunk is processed the next one is being written over the oldest of the three,
// so what may be read is the chunk itself and the one before it.
constexpr uint32_t kWalkReach = 2 * kWalkChunk;
constexpr uint32_t kKeepMaxGap = 4096;   // longer gaps are not worth a slot

// An occupancy event in the form the verifier's occupancy wavefront consumes it, four
// scalar registers that need no further decoding:
//   x  ring slot (index % kWalkRing) of the occurrence that carries the register | vreg << 8
//   y  the tuple's mask at bit 0 (width ones)
//   z  byte offset of the first mask word of the vreg's class (class_word * 256)
//   w  that occurrence (24 bits) | kEvtPost | kEvtSlow | kEvtTested
// The mask word of register p is word (p >> 5) & 15 of the class: every class can address
// 16 words, so no clamp is needed (see DevMir::occ_words).
constexpr uint32_t kEvtPost = 1u << 29;    // release of a value that is dead once its instruction has executed
                                           // (the value still belongs to P of that instruction)
constexpr uint32_t kEvtSlow = 1u << 30;    // not for the fast path: the tuple may cross a mask word, is 32 wide,
                                           // or its register has to come from outside the ring
constexpr uint32_t kEvtTested = 1u << 31;  // occupy with test (a definition); otherwise a plain flip
constexpr uint32_t kSeedLinked = 1u << 28; // (tile live-in lists only) the vreg's next mention after the source occurrence lies
                                           // inside the tile: that mention's consistency link reaches back across the tile's start

// Per-occurrence roles computed by the event kernel.
constexpr uint8_t kRolePreKill = 1, kRoleTestSet = 2, kRolePostKill = 4, kRoleFirst = 8;
constexpr uint8_t kRoleKill = 16;   // the occurrence's kill flag, copied to occ_kill in occurrence order later
// Per sorted-entry info bits.
constexpr uint8_t kEntLiveAfter = 1, kEntHasUse = 2, kEntHasDef = 4, kEntGroupStart = 8,
                  kEntKept = 16;   // read by an instruction with an early-clobber definition: in P(i) whatever follows

// Liveness analysis of one kernel on the device.
struct DevLive {
  // --- sized from the program alone ---
  uint32_t VL_GLOBAL *vcnt;       // [V+1] occurrences per vreg -> exclusive offsets (vocc_off)
  uint32_t VL_GLOBAL *vcur;       // [V] placement cursors
  uint32_t VL_GLOBAL *last_live;  // [V] last block the vreg is live into (0: none after the entry)
  uint32_t VL_GLOBAL *vocc_tmp;   // [O] occurrences grouped by vreg, unordered
  uint32_t VL_GLOBAL *vocc;       // [O] occurrences grouped by vreg, ascending
  uint32_t VL_GLOBAL *ent_instr;  // [O] instruction << 2 | occurrence flags of each sorted entry (ascending per vreg)
  uint32_t VL_GLOBAL *ent_v;      // [O] vreg of each sorted entry
  uint8_t VL_GLOBAL *ent_info;    // [O] kEnt* bits of each sorted entry
  uint32_t VL_GLOBAL *first;      // [V] first occurrence or kNone
  uint32_t VL_GLOBAL *prev_occ;   // [O] previous occurrence of the same vreg, written only where the 16-bit
                                  //     distance of the check record is saturated
  uint8_t VL_GLOBAL *occ_role;    // [O] kRole* bits, kRoleKill
  uint8_t VL_GLOBAL *occ_kill;    // [O]
  uint32_t VL_GLOBAL *use;        // [B][W] block bitsets
  uint32_t VL_GLOBAL *def;
  uint32_t VL_GLOBAL *live_in;
  uint32_t VL_GLOBAL *live_out;
  uint32_t VL_GLOBAL *item_off;   // [N+B+1] plan offset of each item (boundary b at blk_start[b]+b,
                        //          instruction i of block b at i+b+1)
  uint32_t VL_GLOBAL *seg_off;    // [V+1]
  u32x4 VL_GLOBAL *chk;           // [O] check records
  uint32_t VL_GLOBAL *evt_cut;    // [ceil(O/64)+1] first event replayable once chunk c is staged
  uint32_t VL_GLOBAL *ent_seg;    // [O+1] runs starting in each mention group's stretch -> prefix sums
  uint8_t VL_GLOBAL *ent_sf;      // [O] where membership changes in the stretch, for the interval filling pass
  uint32_t VL_GLOBAL *hull;       // [V][2]
  uint32_t VL_GLOBAL *seed_off;   // [T+1]
  uint32_t VL_GLOBAL *seed_cur;   // [T]
  uint32_t VL_GLOBAL *long_queue; // [V] vregs whose occurrence list needs the bitmap sort
  uint32_t VL_GLOBAL *bitmap;     // [ceil(O/32)] scratch for the bitmap sort, one list at a time per block
  uint32_t VL_GLOBAL *counters;   // [kCounters]
  // --- sized after the counting pass ---
  u32x4 VL_GLOBAL *plan;          // [plan_len + 8] occupancy events (the last 8 are padding, never applied)
  u32x4 VL_GLOBAL *seeds;         // [n_seed] event records
  uint32_t VL_GLOBAL *seg;        // [n_seg][2]
  uint32_t VL_GLOBAL *tile_range; // [T][2] plan range of each tile
  uint32_t VL_GLOBAL *tile_live;  // [T][W] live-before row of each tile start (dense mode)
  uint32_t VL_GLOBAL *live_after; // [N][W] (dense mode)
  uint32_t T, tile_len, plan_len, n_seg, n_seed, dense;
};

template <class T> __host__ __device__ inline const T VL_GLOBAL *as_global(const T *p) {
  return (const T VL_GLOBAL *)p;
}
template <class T> __host__ __device__ inline T VL_GLOBAL *as_global_rw(T *p) {
  return (T VL_GLOBAL *)p;
}

// atomics on global-memory pointers (the HIP header ones take generic pointers)
#define VL_ATOMIC(name, builtin)                                                        \
  __device__ inline uint32_t name(uint32_t VL_GLOBAL *p, uint32_t v) {                  \
    return builtin(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);                   \
  }
VL_ATOMIC(atomicAdd, __hip_atomic_fetch_add)
VL_ATOMIC(atomicOr, __hip_atomic_fetch_or)
VL_ATOMIC(atomicXor, __hip_atomic_fetch_xor)
VL_ATOMIC(atomicMin, __hip_atomic_fetch_min)
VL_ATOMIC(atomicMax, __hip_atomic_fetch_max)
#undef VL_ATOMIC

enum { kCtrLong = 0, kCtrNotStrict = 1, kCtrSweeps = 2, kCtrPlanLen = 3, kCtrSeg = 4, kCtrSeed = 5,
       kCounters = 8 };

}  // namespace vl

// host-side handles
namespace vl {
// Which hardware rules a base register breaks for a vreg with these attributes (VL_BAD_*).
__device__ inline uint32_t bad_bits(const DevMir VL_GLOBAL &m, uint32_t attr, uint32_t p) {
  const uint32_t cls = attr_class(attr), width = attr_width(attr), align = attr_align(attr);
  uint32_t bad = 0;
  if (p + width > m.class_size[cls]) bad |= VL_BAD_BOUNDS;
  if (p % align != 0) bad |= VL_BAD_ALIGN;
  if (m.has_reserved)
    for (uint32_t r = p; r < p + width; ++r)
      if (r < 512 && ((m.reserved[cls][r >> 5] >> (r & 31)) & 1u)) bad |= VL_BAD_RESERVED;
  return bad;
}

// P(i) = live_after(i) + defs(i) as a vreg bitset: the live-in list of i's tile, then every
// event up to those of i, flips one bit each (in any order); the releases of values dead once
// i has executed are left out, since such values still belong to P(i).  in_p: [W] words in
// LDS, cleared by the caller (with a barrier in between); the caller also adds the barrier
// after this call.
__device__ inline void flip_members_of_p(const DevMir VL_GLOBAL &m, const DevLive VL_GLOBAL &L, const uint32_t i, uint32_t *in_p,
                                         const uint32_t tid, const uint32_t n_threads) {
  const uint32_t tile = i / L.tile_len;
  auto flip_vreg = [&](uint32_t v) {   // records carry their vreg in x (above the ring slot)
    __hip_atomic_fetch_xor(&in_p[v >> 5], 1u << (v & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  };
  if (tile > 0)
    for (uint32_t s = L.seed_off[tile] + tid; s < L.seed_off[tile + 1]; s += n_threads) flip_vreg(L.seeds[s].x >> 8);
  const uint32_t item = i + m.instr_blk[i] + 1;   // boundary items come before their block's instructions
  const uint32_t e_own = L.item_off[item], e_end = L.item_off[item + 1];
  for (uint32_t e = L.tile_range[2 * tile] + tid; e < e_end; e += n_threads) {
    const u32x4 r = L.plan[e];
    if (e >= e_own && (r.w & kEvtPost)) continue;
    flip_vreg(r.x >> 8);
  }
}
}  // namespace vl

namespace vl {
// One device allocation that holds the interference pairs of several programs; freed with the
// last of them.
struct EdgeBlock {
  void *mem;
  std::atomic<uint32_t> refs;
};
}  // namespace vl

struct vl_mir {
  vl::DevMir h;        // host mirror (device pointers inside)
  vl::DevMir *dev;     // device copy
  void *arena;         // single allocation holding every array
  int device;
  uint64_t magic;
  // interference pairs (a < b, one class, some point in common), built on first use by the
  // all-violations mode and kept for the life of the handle: they depend on the program only
  void *edges = nullptr;       // device: n_edges pairs of uint32, inside edge_block
  uint64_t n_edges = 0;
  bool edges_built = false;
  vl::EdgeBlock *edge_block = nullptr;   // the allocation the pairs sit in, shared with the other programs of that call
  // vl_mir_create_lanes: the caller's sizes and the device maps between the two numberings
  bool lowered = false;
  uint32_t src_occ = 0, src_vreg = 0;
  const uint32_t *occ_src = nullptr;    // [O] device
  const uint8_t *occ_add = nullptr;     // [O] device: the lane, i.e. what is added to the caller's register
  const uint32_t *val_vreg = nullptr;   // [V] device
  const uint8_t *val_lane = nullptr;    // [V] device: lane, or 0xFF for a whole vreg
};

struct vl_batch;
struct vl_live {
  vl_batch *batch;
  uint32_t index;
  const vl_mir *mir;
  vl::DevLive h;       // host mirror
  vl::DevLive *dev;    // element of the batch's device array
  uint64_t magic;
};

namespace vl {
constexpr uint64_t kMirMagic = 0x564c4d4952ull, kLiveMagic = 0x564c4c495645ull;
int32_t hip_fail(hipError_t e);
#define VL_HIP(call)                                   \
  do {                                                 \
    hipError_t e_ = (call);                            \
    if (e_ != hipSuccess) return vl::hip_fail(e_);     \
  } while (0)
}  // namespace vl

#endif
