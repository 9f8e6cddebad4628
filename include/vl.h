/*
 * vl -- GPU (gfx950) verifier core for sampled register allocations.
 *
 * Decides, for many candidate virtual-to-physical register assignments of one
 * machine-IR kernel at once, the conditions under which the paper calls an
 * allocation correct (Section 1, items (1) and (2); Section 2 "Register
 * Allocation"; Section 3.4 Consistency / Safety / Realizability), using the
 * polynomial check along control and data dependencies that Section 4.6
 * points to instead of an SMT solver.  Two stages:
 *
 *   vl_liveness       backward dataflow liveness over the CFG as bitset
 *                     union / and-not per basic block, iterated to the least
 *                     fixed point; per-point live sets, kill flags, live
 *                     intervals; and the event stream the verifier replays.
 *   vl_verify_batch   replays that stream for K candidates, 64 candidates per
 *                     wavefront, and reports each candidate's status and its
 *                     first violation.
 *
 * All entry points are plain C.  Pointers marked [host] are read during the
 * call only; pointers marked [device] must be device memory valid on the
 * current HIP device and are never owned or freed by the library.  Handles
 * are created and destroyed by the library.  Every function returns VL_OK (0)
 * or a negative error code and never aborts; a candidate that breaks a
 * condition is not an error but a status in the output.
 *
 * Program model.  Instructions 0..N-1 in one linear order; block b is the
 * contiguous range [blk_start[b], blk_start[b+1]), block 0 is the entry;
 * operand occurrences are numbered in instruction order, then operand order.
 * An instruction reads its USE operands before it writes its DEF operands
 * (a DEF may reuse the register of an operand that dies at that instruction),
 * unless a DEF is flagged VL_OCC_EARLY.
 * Bitset rows have W = ceil(n_vreg/32) words; vreg v is bit (v & 31) of word
 * (v >> 5).
 */
#ifndef VL_H
#define VL_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  VL_OK = 0,
  VL_E_NULL = -1,       /* a required pointer is NULL */
  VL_E_SHAPE = -2,      /* inconsistent sizes: offsets not monotone, K == 0, ld < n_occ, ... */
  VL_E_RANGE = -3,      /* vreg id >= n_vreg, class >= n_class, file > 512, width 0 or > 32,
                           align 0 or > 32, more than 8 classes, more than 64 operands in one
                           instruction, unknown occurrence flag bits, successor >= n_block,
                           2^24 or more occurrences, 2^28 or more instructions, more than
                           VL_MAX_VREG vregs */
  VL_E_LAYOUT = -4,     /* blocks do not tile 0..N-1, a block is empty, or a non-entry block has
                           no predecessor placed before it in the linear order */
  VL_E_NOT_STRICT = -5, /* some value is live into the entry block */
  VL_E_HIP = -6,        /* a HIP runtime call failed; see vl_last_hip_error */
  VL_E_ARG = -7,        /* handle does not belong to this call (wrong program, stale, ...) */
  VL_E_LIMIT = -8       /* vl_verify_batch_static: more than VL_STATIC_MAX_K candidates */
};

/* Most vregs a program may have: a bitset row over them (15,360 words, 60 KB) must fit the
 * 64 KB of LDS a workgroup gets without further arrangement, beside a few KB of other use. */
#define VL_MAX_VREG 491520u

#define VL_OCC_DEF 1u
#define VL_OCC_USE 2u
/* Early-clobber, on a DEF only: the value is written before the instruction has read its
 * operands, so it cannot share a register with any of them.  The values an instruction
 * with such a definition reads stay occupied through it: they belong to P(i) even when
 * they die there (the bit acts on the whole instruction). */
#define VL_OCC_EARLY 4u

/* vl_liveness flags */
#define VL_DENSE_POINTS 1u /* also materialise live_after[N][W] */

/* Description of one kernel; every pointer is [host]. */
typedef struct {
  uint32_t n_instr, n_vreg, n_block, n_occ, n_class, n_edge;
  const uint32_t *blk_start;      /* [n_block+1], blk_start[0] = 0, last = n_instr */
  const uint32_t *succ_off;       /* [n_block+1] CSR offsets into succ */
  const uint32_t *succ;           /* [n_edge] successor block ids */
  const uint32_t *instr_occ_off;  /* [n_instr+1] CSR offsets into occurrences */
  const uint32_t *occ_vreg;       /* [n_occ] */
  const uint8_t *occ_flags;       /* [n_occ] VL_OCC_DEF | VL_OCC_USE, VL_OCC_EARLY on a DEF */
  const uint8_t *vreg_class;      /* [n_vreg] */
  const uint8_t *vreg_width;      /* [n_vreg] width in 32-bit registers, 1..32 */
  const uint8_t *vreg_align;      /* [n_vreg] base must be a multiple of this, 1..32 */
  const uint16_t *class_size;     /* [n_class] registers in the file, <= 512 */
  const uint32_t *class_reserved; /* [n_class][16] 512-bit masks of unusable registers, or NULL */
} vl_mir_desc;

typedef struct vl_mir vl_mir;   /* a kernel resident on the device */
typedef struct vl_live vl_live; /* its liveness analysis, resident on the device */
typedef void *vl_stream;        /* a hipStream_t (NULL = the default stream) */

/* Validates the description (Section 2: programs in MIR, virtual registers,
 * register classes and tuples) and copies it to the current device.
 * Synchronous.  *out is written only on success. */
int32_t vl_mir_create(const vl_mir_desc *desc, vl_mir **out);
void vl_mir_destroy(vl_mir *mir);

/* Liveness of parts of a tuple.  The paper treats a vreg as one unit; Section 2 places a wide
 * value in consecutive 32-bit registers.  Reading taken for instructions that read or write
 * only part of a tuple: lane j (0 <= j < width) of a vreg is the register at base + j, and
 * occ_lanes [host] [n_occ] names the lanes each occurrence accesses (bit j = lane j; 0, or a
 * NULL array, = all of them; a bit at or above the width is VL_E_RANGE).  A DEF writes its
 * lanes and leaves the others as they were, a USE reads its lanes; liveness, P(i) and the
 * live intervals are the analysis per (vreg, lane), Safety is tested on the registers of the
 * lanes in P(i), Consistency and Realizability stay per vreg and whole tuple.
 *
 * The handle holds a rewritten program: every vreg that is accessed in part somewhere is
 * followed by one value per lane (one register wide, no alignment), vregs never accessed in
 * part stay as they are; values are numbered vreg by vreg, a vreg before its lanes.  An
 * occurrence of a split vreg becomes a mention of the whole vreg (it neither reads nor
 * writes) followed by one occurrence per lane accessed (at most 64 occurrences per
 * instruction afterwards, VL_E_RANGE otherwise).  vl_liveness and vl_live_get describe that
 * program (vl_mir_lanes_get gives the maps back to the caller's numbering); vl_verify_batch /
 * vl_verify_multi take candidate rows in its numbering, which vl_lanes_expand makes from the
 * caller's rows, and report results in the caller's numbering: occurrences and vregs of the
 * description given here, SAFETY with the smallest pair of the caller's vregs.
 * vl_count_violations_multi, vl_free_bases_multi and vl_bank_conflicts do not take such a
 * handle (VL_E_ARG). */
int32_t vl_mir_create_lanes(const vl_mir_desc *desc, const uint32_t *occ_lanes, vl_mir **out);
typedef struct {
  uint32_t n_occ, n_vreg;          /* of the caller's description */
  uint32_t n_occ_low, n_vreg_low;  /* of the rewritten program */
  const uint32_t *occ_src;         /* [device] [n_occ_low] the caller's occurrence */
  const uint8_t *occ_add;          /* [device] [n_occ_low] the lane: added to the caller's register */
  const uint32_t *val_vreg;        /* [device] [n_vreg_low] the caller's vreg */
  const uint8_t *val_lane;         /* [device] [n_vreg_low] the lane, 0xFF for a whole vreg */
} vl_lanes_view;
int32_t vl_mir_lanes_get(const vl_mir *mir, vl_lanes_view *out);
/* cand_low[k][o'] = cand[k][occ_src[o']] + occ_add[o'] for K rows (16-bit arithmetic);
 * cand [device] K rows of pitch ld >= n_occ, cand_low [device] K rows of pitch
 * ld_low >= n_occ_low, caller-owned.  Asynchronous on `stream`.  Errors: VL_E_NULL, VL_E_ARG
 * (not such a handle), VL_E_SHAPE (K == 0 or above 65535, a pitch too small). */
int32_t vl_lanes_expand(const vl_mir *mir, const uint16_t *cand, uint32_t K, uint64_t ld, uint16_t *cand_low,
                        uint64_t ld_low, vl_stream stream);

/* Liveness analysis of n kernels in one batch of launches (Section 3.2: the
 * control flow and data dependency of the input; Section 3.4 Safety: which
 * lifetimes overlap).  Enqueues on `stream`, synchronises it once to read the
 * result sizes and error flags back, then enqueues the remaining work; the
 * results are complete once the stream has been synchronised again.
 *
 * live[0..n): on entry either all NULL, or the n handles a previous call with
 * these same kernels returned, whose device storage is then reused (no
 * allocation when it is large enough).  When that call also had the same flags
 * and tile_len, the result sizes are known from it: nothing is read back and
 * the call does not synchronise at all.  From the second such call on it
 * enqueues kernels only (no copy, no memset): that call, vl_verify_multi and
 * vl_summarize_multi with an unchanged job table may then be recorded in a
 * stream capture and replayed.  On success live[i] describes mirs[i].
 * On error no handle is created; recycled handles stay allocated but their
 * contents are undefined until the next successful call.
 * tile_len: instructions per verification tile, 0 = library default (512, less for batches of
 * fewer than half a million instructions in total, down to 128).
 * Errors: VL_E_NOT_STRICT / VL_E_LAYOUT refer to the first offending kernel. */
int32_t vl_liveness_multi(const vl_mir *const *mirs, uint32_t n, uint32_t flags, uint32_t tile_len,
                          vl_stream stream, vl_live **live);
/* The same for one kernel. */
int32_t vl_liveness(const vl_mir *mir, uint32_t flags, vl_stream stream, vl_live **live);
void vl_live_destroy(vl_live *live);

/* Device views of one analysis; every pointer is [device], owned by the
 * handle, valid until it is destroyed or recycled. */
typedef struct {
  uint32_t n_instr, n_vreg, n_block, n_occ, words; /* words = W */
  uint32_t n_seg;                 /* total number of live-interval segments */
  uint32_t n_tile, tile_len;      /* verification tiles */
  uint32_t plan_len;              /* entries of the verifier's event stream */
  uint32_t sweeps;                /* fixed-point sweeps of the slowest word column */
  const uint32_t *live_in;        /* [n_block][W] */
  const uint32_t *live_out;       /* [n_block][W] */
  const uint32_t *live_after;     /* [n_instr][W], NULL unless VL_DENSE_POINTS */
  const uint8_t *occ_kill;        /* [n_occ] 1 iff a USE of v at i, v neither live after i nor written at i */
  const uint32_t *seg_off;        /* [n_vreg+1] CSR offsets into seg */
  const uint32_t *seg;            /* [n_seg][2] maximal runs of {i : v in P(i)} as [start,end) */
  const uint32_t *hull;           /* [n_vreg][2] [min start, max end) or [0,0) */
} vl_live_view;
int32_t vl_live_get(const vl_live *live, vl_live_view *out);

/* Result per candidate.
 * status 0 OK            where = a = b = 0
 *        1 CONSISTENCY   where = smallest occurrence o whose register differs from that of the
 *                        first occurrence of its vreg; a = vreg; b = that first occurrence
 *        2 REALIZABILITY where = first occurrence of the offending vreg with the smallest first
 *                        occurrence; a = vreg; b = VL_BAD_* bits
 *        3 SAFETY        where = smallest instruction i at which two vregs of one class, both in
 *                        P(i) = live_after(i) + defs(i), have overlapping register ranges;
 *                        (a, b), a < b, the lexicographically smallest such pair at i
 * Consistency outranks realizability outranks safety. */
typedef struct { uint32_t status, where, a, b; } vl_result;
enum { VL_STATUS_OK = 0, VL_STATUS_CONSISTENCY = 1, VL_STATUS_REALIZABILITY = 2, VL_STATUS_SAFETY = 3 };
enum { VL_BAD_BOUNDS = 1, VL_BAD_ALIGN = 2, VL_BAD_RESERVED = 4 };

/* Checks K candidates of one kernel (Section 3.4; Section 3.4's regeneration
 * loop supplies the K samples).  cand [device]: K rows of uint16, row k at
 * cand + k*ld, one physical base register per operand occurrence; ld >= n_occ.
 * Rows are read fastest when cand is 16-byte aligned and ld is a multiple of 8; when ld is
 * also at least n_occ rounded up to a multiple of 64, rows are fetched in whole 128-byte
 * lines up to that bound, so all K x ld elements must then belong to the buffer (what the
 * padding holds is ignored).
 * out [device]: K results.  Asynchronous on `stream`. */
int32_t vl_verify_batch(const vl_mir *mir, const vl_live *live, const uint16_t *cand, uint32_t K,
                        uint64_t ld, vl_result *out, vl_stream stream);

/* vl_verify_batch for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid it.  Same arguments, same results.
 * Its job table and the list of candidates whose clashing pair is still to be found live in
 * a fixed device array inside the library (8 bytes per candidate, VL_STATIC_MAX_K of them:
 * 512 KB per GPU the library runs on, held until the process ends); the call allocates and
 * frees nothing, on the host or the device, and copies nothing from host memory: it only
 * enqueues kernels on `stream`.  Every call on a GPU uses that GPU's one array: calls that
 * overlap on one GPU (different streams, or threads) race; calls on one stream are ordered.
 * Errors: as vl_verify_batch, and VL_E_LIMIT for K above VL_STATIC_MAX_K (nothing is
 * launched then). */
#define VL_STATIC_MAX_K 65536u
int32_t vl_verify_batch_static(const vl_mir *mir, const vl_live *live, const uint16_t *cand, uint32_t K,
                               uint64_t ld, vl_result *out, vl_stream stream);

/* Many kernels in one launch: the K samples that Section 3.4's regeneration loop draws for
 * every kernel of a suite (Section 4.2 evaluates Pass@100), checked as vl_verify_batch checks
 * one kernel's.  jobs is [host] and is copied before the call returns;
 * cand/out inside are [device].  Asynchronous on `stream`; calls on different streams may
 * overlap on the device.  Device memory owned by the library: per device and calling
 * stream (up to four streams at a time; a fifth takes over the least recently used slot
 * after waiting for the device) a copy of the job table and a list of the candidates whose
 * clashing pair has to be found.  Both grow on demand, which waits for the stream and
 * allocates; a call whose jobs are no more, and whose candidates in total are no more, than
 * in an earlier call on that stream allocates nothing, and when its job table is unchanged
 * it only enqueues kernels.  Errors: VL_E_NULL (a pointer missing), VL_E_ARG (a handle that
 * is not a live handle of its program, or more than 16 devices), VL_E_SHAPE (n_jobs = 0 or
 * above 65,535, K = 0, ld below n_occ), VL_E_HIP. */
typedef struct {
  const vl_mir *mir;
  const vl_live *live;
  const uint16_t *cand;
  uint32_t K;
  uint64_t ld;
  vl_result *out;
} vl_job;
int32_t vl_verify_multi(const vl_job *jobs, uint32_t n_jobs, vl_stream stream);

/* The same (Section 3.4, the samples of the regeneration loop) for candidates stored
 * occurrence-major, which is how a batched decoder leaves them (one step emits one occurrence of all K samples): jobs[j].cand is [n_occ][ld] with
 * cand[o * ld + k] the register of occurrence o in candidate k, ld >= K.  Requires cand on a
 * 16-byte boundary and ld a multiple of 8 (VL_E_SHAPE otherwise); the up to 7 elements of
 * padding after the K-th candidate of each occurrence are read and ignored.  Results as for
 * vl_verify_multi. */
int32_t vl_verify_multi_occ_major(const vl_job *jobs, uint32_t n_jobs, vl_stream stream);

/* Regeneration-loop reductions (Section 3.4, last paragraph: samples are tried until the
 * verifier accepts one or the attempts are exhausted; Section 4.2: Pass@K, average and
 * maximum number of attempts).  Reads the results a preceding vl_verify_multi /
 * vl_verify_batch on the same stream wrote into jobs[j].out, in sampling order k = 0..K-1.
 * summaries [device]: n_jobs records, first_ok = index of the first accepted candidate
 * (K if none), passed = 1 iff one is accepted, hist[s] = candidates with status s.
 * stats [device], may be NULL: one record over all jobs; a job's attempts are
 * first_ok + 1 if it passed, else all its K candidates.  Asynchronous on `stream`. */
typedef struct { uint32_t first_ok, passed, hist[4]; } vl_summary;
typedef struct { uint32_t n_passed, max_tries; uint64_t sum_tries; uint64_t hist[4]; } vl_loop_stats;
int32_t vl_summarize_multi(const vl_job *jobs, uint32_t n_jobs, vl_summary *summaries, vl_loop_stats *stats,
                           vl_stream stream);

/* All violations of each candidate instead of the first (Section 4.5 sorts the model's
 * failures into dataflow and hardware-constraint violations; Section 6 proposes the verifier
 * as feedback or reward during training).  With T(v) = the register of v's first occurrence:
 *   n_cons    occurrences whose register differs from T(their vreg)       (Consistency)
 *   n_real    mentioned vregs for which T(v) breaks a hardware rule;
 *             real_bits = the rules broken, OR-ed (VL_BAD_*)              (Realizability)
 *   n_safe    pairs a < b of one class that are in P(i) together for some i and whose
 *             tuples at T(a), T(b) overlap                                (Safety)
 *   kinds     bit 0: n_cons > 0, bit 1: n_real > 0, bit 2: n_safe > 0
 * The status vl_verify_batch reports is the lowest bit set in kinds (0 if none).
 * jobs is [host]; cand and out inside are [device]; out receives K records.  The first call
 * that sees a program enumerates its interfering pairs from `live` (whose analysis must be
 * complete or enqueued on `stream`), synchronising the stream, and keeps them with the
 * vl_mir handle; later calls are asynchronous on `stream` but wait on the host until the
 * previous call's kernels have finished with the library's workspace.
 * Errors: VL_E_NULL, VL_E_ARG (handles of different programs), VL_E_SHAPE (n_jobs == 0 or
 * above 65535, K == 0 or above 65535, ld < n_occ); nothing is launched on error. */
typedef struct { uint32_t kinds, n_cons, n_real, n_safe, real_bits, reserved[3]; } vl_counts;
typedef struct {
  const vl_mir *mir;
  const vl_live *live;
  const uint16_t *cand;
  uint32_t K;
  uint64_t ld;
  vl_counts *out;
} vl_count_job;
int32_t vl_count_violations_multi(const vl_count_job *jobs, uint32_t n_jobs, vl_stream stream);

/* Register-bank conflicts, a quality measure beside validity (Section 2: registers are
 * organised in banks, four on NVIDIA GPUs; reading several values from one bank stalls the
 * pipeline one cycle per extra value, which is why the FFMA of the overview figure reads R4,
 * R6 and R9).  Register r is in bank r mod n_banks.  An instruction reads the registers of its
 * distinct USE vregs (a tuple of width w at base p reads p .. p + w - 1, the base taken from
 * the vreg's first USE operand of that instruction); the banks deliver in parallel, so it
 * stalls max over banks of (registers read from that bank) - 1 cycles, 0 if it reads nothing.
 * out [device]: K sums over all instructions, one per candidate row of cand [device].  Needs
 * no analysis.  Asynchronous on `stream`.
 * Errors: VL_E_NULL, VL_E_ARG, VL_E_SHAPE (K == 0 or above 65535, ld < n_occ), VL_E_RANGE
 * (n_banks == 0 or above 64). */
int32_t vl_bank_conflicts(const vl_mir *mir, const uint16_t *cand, uint32_t K, uint64_t ld, uint32_t n_banks,
                          uint32_t *out, vl_stream stream);

/* Constrained decoding (Section 4.5, last sentence of the error analysis: mask out the
 * registers that are occupied while the allocation is generated).  A decoder emits a
 * candidate one occurrence after the other; query j asks which bases it may give occurrence
 * `occ` (of vreg v, at instruction i) of the row `cand`, whose occurrences before `occ` are
 * fixed and the only ones read.  masks [device]: 16 words per query, bit p set iff
 *   p is a multiple of v's alignment, p + width fits the file of v's class and no register
 *   of the tuple is reserved (Section 3.4 Realizability), and
 *   when v has an earlier occurrence: p is that occurrence's register (Consistency), else:
 *   the tuple is disjoint from that of every other vreg of the class that is in P(i) and
 *   whose first occurrence lies before `occ`, taken at its first occurrence's register
 *   (Safety; a value that dies at i is not in P(i)).
 * queries is [host]; cand and masks are [device].  Asynchronous on `stream`; the call waits
 * on the host for the previous call's queries to have been consumed.
 * Errors: VL_E_NULL, VL_E_ARG (handles of different programs), VL_E_SHAPE (n == 0, occ past
 * the program's occurrences); nothing is launched on error. */
typedef struct {
  const vl_mir *mir;
  const vl_live *live;
  const uint16_t *cand;
  uint32_t occ;
  uint32_t reserved0; /* must be 0 */
} vl_mask_query;
int32_t vl_free_bases_multi(const vl_mask_query *queries, uint32_t n, uint32_t *masks, vl_stream stream);

const char *vl_strerror(int32_t code);
/* hipError_t of the last failed runtime call on this thread (0 if none). */
int32_t vl_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif
