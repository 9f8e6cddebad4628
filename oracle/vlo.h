/*
 * vlo -- plain CPU oracle for register-allocation verification.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, obviously-correct reference
 * that the GPU library is compared against.  Nothing in the product path may
 * include, link or call it; it shares no code, header or table with the HIP
 * sources.
 *
 * What it decides is the paper's notion of a correct allocation
 * (Introduction, item (1)/(2); Section 2 "Register Allocation"; Section 3.4
 * "Verifier-guided Inference": Consistency, Safety, Realizability):
 *   (1) every occurrence of a virtual register carries the same physical
 *       register,
 *   (2) virtual registers whose lifetimes overlap occupy disjoint physical
 *       registers,
 *   (3) the assignment is realizable on the hardware: a value of width w
 *       sits in w consecutive 32-bit registers inside its register file,
 *       suitably aligned, avoiding reserved registers.
 * The paper decides these with an SMT solver and remarks (Section 4.6) that
 * the common case only needs the control and data dependencies; lifetimes
 * here come from the textbook backward may-liveness over the CFG.
 *
 * Parity status: every function below is pinned by tests that do not use the
 * function itself (path enumeration on tiny CFGs with one and with several
 * bitset words per row, a literal per-point all-pairs checker, a register-marking
 * check in Python at thousands of instructions, hand-worked examples,
 * allocator/mutation invariants).
 * Agreement with the paper's own Z3 verdicts is UNPINNED: the SMT encoding is
 * not published and no solver or dataset is available.
 *
 * Conventions.  Instructions 0..N-1 in one linear order; block b is the
 * contiguous range [blk_start[b], blk_start[b+1]); occurrences (operand
 * slots) are numbered in instruction order, then operand order.  A bitset
 * row has W = ceil(V/32) words; vreg v is bit (v & 31) of word (v >> 5).
 */
#ifndef VLO_H
#define VLO_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VLO_OCC_DEF 1u
#define VLO_OCC_USE 2u
/* Early-clobber: a DEF with this bit is written before the instruction has read its
 * operands, so it may not share a register with any of them.  Reading taken: the
 * values an instruction with such a definition reads stay occupied through it, i.e.
 * they belong to P(i) even when they die there (the bit acts on the whole instruction). */
#define VLO_OCC_EARLY 4u

typedef struct {
  uint32_t n_instr, n_vreg, n_block, n_occ, n_class, n_edge;
  const uint32_t *blk_start;     /* [n_block+1] */
  const uint32_t *succ_off;      /* [n_block+1] CSR into succ */
  const uint32_t *succ;          /* [n_edge] successor block ids */
  const uint32_t *instr_occ_off; /* [n_instr+1] CSR into occurrences */
  const uint32_t *occ_vreg;      /* [n_occ] */
  const uint8_t *occ_flags;      /* [n_occ] VLO_OCC_DEF | VLO_OCC_USE */
  const uint8_t *vreg_class;     /* [n_vreg] */
  const uint8_t *vreg_width;     /* [n_vreg] in 32-bit registers */
  const uint8_t *vreg_align;     /* [n_vreg] required divisor of the base */
  const uint16_t *class_size;    /* [n_class] registers in the file */
  const uint32_t *class_reserved;/* [n_class][16] 512-bit masks or NULL */
} vlo_mir;

typedef struct { uint32_t status, where, a, b; } vlo_result;
enum { VLO_OK = 0, VLO_CONSISTENCY = 1, VLO_REALIZABILITY = 2, VLO_SAFETY = 3 };
enum { VLO_BAD_BOUNDS = 1, VLO_BAD_ALIGN = 2, VLO_BAD_RESERVED = 4 };

typedef struct { uint32_t a, b, first; } vlo_edge; /* a < b, first common point */

/* Block-level liveness: least fixed point of
 *   out[b] = union of in[s] over successors s,  in[b] = use[b] | (out[b] \ def[b]).
 * live_in / live_out: [n_block][n_vreg] membership bytes (0/1), caller-owned.
 * Returns the number of sweeps over the blocks that were needed. */
int vlo_block_liveness(const vlo_mir *m, uint8_t *live_in, uint8_t *live_out);

/* Per-point liveness: live_after[i] for every instruction, by the backward
 * walk inside each block from live_out.  Bit-packed rows [n_instr][W]. */
void vlo_points(const vlo_mir *m, const uint8_t *live_out, uint32_t *live_after);

/* Occupancy rows P(i) = live_after[i] | defs(i), [n_instr][W]. */
void vlo_occupancy(const vlo_mir *m, const uint32_t *live_after, uint32_t *P);

/* Kill flag of each occurrence: 1 iff it is a USE of v at i and v is not in
 * P(i); 0 otherwise (in particular for pure DEF occurrences). [n_occ] */
void vlo_kill_flags(const vlo_mir *m, const uint32_t *live_after, uint8_t *occ_kill);

/* Live intervals: for each vreg the maximal runs of {i : v in P(i)} in linear
 * order as half-open [start,end).  seg_off[V+1]; seg holds up to cap pairs.
 * hull[v] = [min start, max end) or [0,0) if v is never occupied.
 * Returns the total number of segments; seg and hull are only written when
 * cap is large enough (call with seg = NULL, cap = 0 to size). */
uint64_t vlo_segments(const vlo_mir *m, const uint32_t *P, uint32_t *seg_off,
                      uint32_t *seg, uint64_t cap, uint32_t *hull);

/* Interference relation by the pairwise O(V^2) test: for all a < b of the
 * same class whose interval lists share a point, the smallest such point.
 * Returns the number of edges (call with cap = 0 to size). */
uint64_t vlo_interference(const vlo_mir *m, const uint32_t *seg_off,
                          const uint32_t *seg, vlo_edge *edges, uint64_t cap,
                          int n_threads);

/* first[v] = smallest occurrence index of v, or UINT32_MAX. [n_vreg] */
void vlo_first_occurrence(const vlo_mir *m, uint32_t *first);

/* Verify K candidates (row k at cand + k*ld, one uint16 per occurrence)
 * against the interference relation.  out[K]. */
void vlo_verify(const vlo_mir *m, const vlo_edge *edges, uint64_t n_edges,
                const uint16_t *cand, uint32_t K, uint64_t ld, vlo_result *out,
                int n_threads);

/* The definition written out with no interference relation: at every point,
 * every pair of P(i).  One candidate. */
void vlo_verify_points(const vlo_mir *m, const uint32_t *P, const uint16_t *cand,
                       vlo_result *out);

/* Input contract used by the tile-parallel GPU walk: 0 if live_in[entry] is
 * empty and every non-entry block has a predecessor earlier in linear order;
 * 1 if the entry has live-ins; 2 if some block lacks an earlier predecessor. */
int vlo_contract(const vlo_mir *m, const uint8_t *live_in);

/* The regeneration loop of Section 3.4 tries samples one after the other until
 * the verifier accepts one or the attempts are exhausted; Section 4.2 reports
 * the number of attempts (average, maximum) and whether any of K samples
 * passes (Pass@K).  Over the verdicts of one kernel's K samples, in sampling
 * order: first_ok = index of the first accepted sample, K if none;
 * passed = 1 iff some sample is accepted; hist[s] = samples with status s. */
typedef struct { uint32_t first_ok, passed, hist[4]; } vlo_summary;
void vlo_summarize(const vlo_result *res, uint32_t K, vlo_summary *out);

/* Over n kernels: n_passed kernels with an accepted sample; tries of a kernel =
 * first_ok + 1 if it passed, else all its K samples; max_tries and sum_tries
 * over the kernels; hist summed. */
typedef struct { uint32_t n_passed, max_tries; uint64_t sum_tries; uint64_t hist[4]; } vlo_loop_stats;
void vlo_loop(const vlo_summary *s, const uint32_t *K, uint32_t n, vlo_loop_stats *out);

/* All violations of a candidate instead of the first (Section 4.5 sorts the failures of
 * the model into dataflow and hardware-constraint violations; Section 6 proposes the
 * verifier as feedback or reward during training).  With T(v) = the register of v's first
 * occurrence:
 *   n_cons    occurrences whose register differs from T(their vreg)   (Consistency)
 *   n_real    mentioned vregs for which T(v) breaks a hardware rule; real_bits = the
 *             rules broken, OR-ed (VLO_BAD_*)                          (Realizability)
 *   n_safe    pairs a < b of one class that are in P(i) together for some i and whose
 *             tuples at T(a), T(b) overlap (the edges of vlo_interference)  (Safety)
 *   kinds     bit 0: n_cons > 0, bit 1: n_real > 0, bit 2: n_safe > 0
 * The status of vlo_verify is the lowest bit set in kinds (0 if none). */
typedef struct { uint32_t kinds, n_cons, n_real, n_safe, real_bits, pad[3]; } vlo_counts;
void vlo_count_violations(const vlo_mir *m, const vlo_edge *edges, uint64_t n_edges,
                          const uint16_t *cand, uint32_t K, uint64_t ld, vlo_counts *out,
                          int n_threads);

/* Register-bank conflicts, a quality measure beside validity (Section 2: registers are
 * organised in banks, four on NVIDIA GPUs; reading several values from one bank stalls
 * the pipeline one cycle per extra value, and the compiler picks R4, R6, R9 for an FFMA
 * because they lie in different banks).  Register r is in bank r mod n_banks.  For each
 * instruction the 32-bit registers it reads are those of its distinct USE vregs (a tuple of
 * width w at base p reads p .. p + w - 1; the base is the one of the vreg's first USE
 * operand of that instruction); the banks deliver in parallel, so the instruction stalls
 * max over banks of (registers read from that bank) - 1 cycles, 0 if it reads nothing.
 * out[k] = the sum over all instructions for candidate k. */
void vlo_bank_conflicts(const vlo_mir *m, const uint16_t *cand, uint32_t K, uint64_t ld,
                        uint32_t n_banks, uint32_t *out);

/* Constrained decoding (Section 4.5, last sentence of the error analysis: mask
 * out the registers that are occupied while the allocation is generated).  A
 * decoder emits the candidate one occurrence after the other; when it reaches
 * occurrence q, of vreg v at instruction i, the occurrences before q are
 * fixed.  out[16] receives the 512-bit set of bases p that keep the three
 * conditions of Section 3.4 intact against what is fixed:
 *   Realizability  p is a multiple of v's alignment, p + width fits the file
 *                  of v's class, no register of the tuple is reserved;
 *   Consistency    if v has an earlier occurrence, only that occurrence's
 *                  register remains (and nothing else is asked of it: what v
 *                  may share was settled when v got its register);
 *   Safety         otherwise (q is v's first occurrence) the tuple is disjoint
 *                  from the tuple of every other vreg b of the class that is
 *                  in P(i) and already has a register (its first occurrence
 *                  lies before q), b's register being the one of its first
 *                  occurrence.  A value that dies at i is not in P(i): its
 *                  register may be given to a value written at i.
 * P: the occupancy rows of vlo_occupancy.  Registers from 512 on are never
 * offered. */
void vlo_free_bases(const vlo_mir *m, const uint32_t *P, const uint16_t *cand, uint32_t q, uint32_t out[16]);

/* ---- liveness of parts of a tuple (sub-register liveness) -------------------------------
 * Section 2: a wide value lives in consecutive 32-bit registers; the paper treats a vreg as
 * one unit.  Reading taken for instructions that read or write only part of a tuple: lane j
 * (0 <= j < width) of vreg v is the 32-bit register at base + j, and every occurrence carries
 * a mask of the lanes it accesses (occ_lanes[o], bit j = lane j; NULL, or a mask of 0, means
 * all lanes).  A DEF writes the lanes of its mask and leaves the others as they were; a USE
 * reads the lanes of its mask.  Everything is then the textbook analysis per (vreg, lane):
 *   lane liveness     backward may-analysis with use / def sets of (vreg, lane) pairs
 *   P(i)              the lanes live after i or written at i (or read at i, when the
 *                     instruction has an early-clobber definition)
 *   Safety            at every i the registers base(v) + j of the lanes in P(i) are claimed by
 *                     at most one vreg per class; the first violation is the smallest
 *                     (i, a, b), a < b two vregs of one class that claim the same register at i
 *   Consistency, Realizability   per vreg and whole tuple, as without lanes (the hardware
 *                     rules speak of the tuple, whatever part of it is in use)
 * Lane (v, j) has the index lane_base[v] + j, lane_base = exclusive prefix sums of the widths;
 * Lt = lane_base[V] lanes in all.  With all masks full the lanes of a vreg behave alike and
 * everything reduces to the functions above (which is one of the pins). */
void vlo_lane_base(const vlo_mir *m, uint32_t *lane_base /* [V+1] */);
/* live_in / live_out: [n_block][Lt] bytes.  Returns the number of sweeps. */
int vlo_block_liveness_lanes(const vlo_mir *m, const uint32_t *occ_lanes, uint8_t *live_in, uint8_t *live_out);
/* live_after, P: [n_instr][Lt] bytes */
void vlo_points_lanes(const vlo_mir *m, const uint32_t *occ_lanes, const uint8_t *live_out, uint8_t *live_after);
void vlo_occupancy_lanes(const vlo_mir *m, const uint32_t *occ_lanes, const uint8_t *live_after, uint8_t *P);
/* occ_kill[o]: the lanes that the USE occurrence o reads for the last time: read at i,
 * neither live after i nor written at i. */
void vlo_kill_lanes(const vlo_mir *m, const uint32_t *occ_lanes, const uint8_t *live_after, uint32_t *occ_kill);
/* maximal runs of {i : lane in P(i)} per lane, as vlo_segments per vreg */
uint64_t vlo_segments_lanes(const vlo_mir *m, const uint8_t *P, uint32_t *seg_off /* [Lt+1] */, uint32_t *seg,
                            uint64_t cap, uint32_t *hull /* [Lt][2] */);
/* one candidate against P (bytes [n_instr][Lt]) */
void vlo_verify_lanes(const vlo_mir *m, const uint8_t *P, const uint16_t *cand, vlo_result *out);

#ifdef __cplusplus
}
#endif
#endif
