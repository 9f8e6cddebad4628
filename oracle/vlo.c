/*
 * vlo -- plain CPU oracle (see vlo.h).  TEST INFRASTRUCTURE ONLY.
 *
 * Every function is the definition written out with nested loops over byte
 * or bit membership arrays; nothing is blocked, fused or reordered.  Threads
 * (OpenMP) only split independent outer iterations: candidates, or the first
 * vreg of a pair.
 */
#include "vlo.h"
#include <stdlib.h>
#include <string.h>

static inline int bit_get(const uint32_t *row, uint32_t v) {
  return (row[v >> 5] >> (v & 31)) & 1u;
}
static inline void bit_set(uint32_t *row, uint32_t v) { row[v >> 5] |= 1u << (v & 31); }
static inline void bit_clr(uint32_t *row, uint32_t v) { row[v >> 5] &= ~(1u << (v & 31)); }

static uint32_t words_per_row(const vlo_mir *m) { return (m->n_vreg + 31u) / 32u; }

/* ---- block-level liveness (Section 3.2: control flow and data dependency of
 * the input; Section 3.4 Safety: "overlapping life cycles") ---------------- */
int vlo_block_liveness(const vlo_mir *m, uint8_t *live_in, uint8_t *live_out) {
  const uint32_t V = m->n_vreg, B = m->n_block;
  uint8_t *use = (uint8_t *)calloc((size_t)B * V + 1, 1);
  uint8_t *def = (uint8_t *)calloc((size_t)B * V + 1, 1);
  /* use[b]: read in b before any write in b; an instruction reads its USE
   * operands before it writes its DEF operands. */
  for (uint32_t b = 0; b < B; ++b) {
    uint8_t *u = use + (size_t)b * V, *d = def + (size_t)b * V;
    for (uint32_t i = m->blk_start[b]; i < m->blk_start[b + 1]; ++i) {
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if ((m->occ_flags[o] & VLO_OCC_USE) && !d[m->occ_vreg[o]]) u[m->occ_vreg[o]] = 1;
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_DEF) d[m->occ_vreg[o]] = 1;
    }
  }
  memset(live_in, 0, (size_t)B * V);
  memset(live_out, 0, (size_t)B * V);
  int sweeps = 0, changed = 1;
  while (changed) {
    changed = 0;
    ++sweeps;
    for (uint32_t b = 0; b < B; ++b) {
      uint8_t *in = live_in + (size_t)b * V, *out = live_out + (size_t)b * V;
      for (uint32_t e = m->succ_off[b]; e < m->succ_off[b + 1]; ++e) {
        const uint8_t *sin = live_in + (size_t)m->succ[e] * V;
        for (uint32_t v = 0; v < V; ++v)
          if (sin[v] && !out[v]) { out[v] = 1; changed = 1; }
      }
      for (uint32_t v = 0; v < V; ++v) {
        uint8_t nv = (uint8_t)(use[(size_t)b * V + v] | (out[v] & !def[(size_t)b * V + v]));
        if (nv && !in[v]) { in[v] = 1; changed = 1; }
      }
    }
  }
  free(use);
  free(def);
  return sweeps;
}

/* ---- per-point liveness ------------------------------------------------- */
void vlo_points(const vlo_mir *m, const uint8_t *live_out, uint32_t *live_after) {
  const uint32_t V = m->n_vreg, W = words_per_row(m);
  uint32_t *cur = (uint32_t *)calloc(W + 1, 4);
  for (uint32_t b = 0; b < m->n_block; ++b) {
    memset(cur, 0, (size_t)W * 4);
    for (uint32_t v = 0; v < V; ++v)
      if (live_out[(size_t)b * V + v]) bit_set(cur, v);
    for (uint32_t i = m->blk_start[b + 1]; i-- > m->blk_start[b];) {
      memcpy(live_after + (size_t)i * W, cur, (size_t)W * 4);
      /* live_before[i] = uses(i) | (live_after[i] \ defs(i)) */
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_DEF) bit_clr(cur, m->occ_vreg[o]);
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_USE) bit_set(cur, m->occ_vreg[o]);
    }
  }
  free(cur);
}

void vlo_occupancy(const vlo_mir *m, const uint32_t *live_after, uint32_t *P) {
  const uint32_t W = words_per_row(m);
  memcpy(P, live_after, (size_t)m->n_instr * W * 4);
  for (uint32_t i = 0; i < m->n_instr; ++i) {
    int early = 0;
    for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o) {
      if (m->occ_flags[o] & VLO_OCC_DEF) bit_set(P + (size_t)i * W, m->occ_vreg[o]);
      if (m->occ_flags[o] & VLO_OCC_EARLY) early = 1;
    }
    /* an early-clobber definition: what the instruction reads is still occupied */
    if (early)
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_USE) bit_set(P + (size_t)i * W, m->occ_vreg[o]);
  }
}

/* a USE of v at i is the last one iff v is neither live after i nor written at i */
void vlo_kill_flags(const vlo_mir *m, const uint32_t *live_after, uint8_t *occ_kill) {
  const uint32_t W = words_per_row(m);
  for (uint32_t i = 0; i < m->n_instr; ++i)
    for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o) {
      int written = 0;
      for (uint32_t x = m->instr_occ_off[i]; x < m->instr_occ_off[i + 1]; ++x)
        if ((m->occ_flags[x] & VLO_OCC_DEF) && m->occ_vreg[x] == m->occ_vreg[o]) written = 1;
      occ_kill[o] = (uint8_t)((m->occ_flags[o] & VLO_OCC_USE) && !written &&
                              !bit_get(live_after + (size_t)i * W, m->occ_vreg[o]));
    }
}

/* ---- live intervals ----------------------------------------------------- */
uint64_t vlo_segments(const vlo_mir *m, const uint32_t *P, uint32_t *seg_off,
                      uint32_t *seg, uint64_t cap, uint32_t *hull) {
  /* A run of v starts at i when v is in P(i) but not in P(i-1) and ends at the
   * first later i where v has left.  Rows are visited in order (two passes:
   * count the runs per vreg, then write them), which only changes the order
   * in which the same membership tests are made. */
  const uint32_t W = words_per_row(m), N = m->n_instr, V = m->n_vreg;
  uint32_t *cnt = (uint32_t *)calloc((size_t)V + 1, 4);
  for (uint32_t i = 0; i < N; ++i)
    for (uint32_t v = 0; v < V; ++v)
      if (bit_get(P + (size_t)i * W, v) && !(i && bit_get(P + (size_t)(i - 1) * W, v))) ++cnt[v];
  uint64_t n = 0;
  for (uint32_t v = 0; v < V; ++v) { seg_off[v] = (uint32_t)n; n += cnt[v]; cnt[v] = 0; }
  seg_off[V] = (uint32_t)n;
  for (uint32_t v = 0; v < V; ++v) { hull[2 * v] = 0; hull[2 * v + 1] = 0; }
  if (n <= cap && seg) {
    for (uint32_t i = 0; i <= N; ++i)
      for (uint32_t v = 0; v < V; ++v) {
        int in_now = i < N && bit_get(P + (size_t)i * W, v);
        int in_was = i && bit_get(P + (size_t)(i - 1) * W, v);
        if (in_now && !in_was) {
          seg[2 * ((size_t)seg_off[v] + cnt[v])] = i;
          if (cnt[v] == 0) hull[2 * v] = i;
        } else if (!in_now && in_was) {
          seg[2 * ((size_t)seg_off[v] + cnt[v]) + 1] = i;
          hull[2 * v + 1] = i;
          ++cnt[v];
        }
      }
  }
  free(cnt);
  return n;
}

/* ---- interference: pairwise O(V^2) -------------------------------------- */
/* smallest point contained in a segment of a and in a segment of b, or -1 */
static int64_t first_common_point(const uint32_t *seg, uint32_t a0, uint32_t a1,
                                  uint32_t b0, uint32_t b1) {
  uint32_t x = a0, y = b0;
  while (x < a1 && y < b1) {
    uint32_t lo = seg[2 * x] > seg[2 * y] ? seg[2 * x] : seg[2 * y];
    uint32_t hi = seg[2 * x + 1] < seg[2 * y + 1] ? seg[2 * x + 1] : seg[2 * y + 1];
    if (lo < hi) return lo;
    if (seg[2 * x + 1] <= seg[2 * y + 1]) ++x; else ++y;
  }
  return -1;
}

uint64_t vlo_interference(const vlo_mir *m, const uint32_t *seg_off,
                          const uint32_t *seg, vlo_edge *edges, uint64_t cap,
                          int n_threads) {
  const uint32_t V = m->n_vreg;
  /* per-a counts first, so that the edge list comes out in (a,b) order
   * whatever the thread schedule */
  uint64_t *cnt = (uint64_t *)calloc((size_t)V + 1, sizeof(uint64_t));
  if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 16) num_threads(n_threads)
  for (uint32_t a = 0; a < V; ++a) {
    uint64_t c = 0;
    for (uint32_t b = a + 1; b < V; ++b) {
      if (m->vreg_class[a] != m->vreg_class[b]) continue;
      if (first_common_point(seg, seg_off[a], seg_off[a + 1], seg_off[b], seg_off[b + 1]) >= 0) ++c;
    }
    cnt[a] = c;
  }
  uint64_t total = 0;
  for (uint32_t a = 0; a < V; ++a) { uint64_t c = cnt[a]; cnt[a] = total; total += c; }
  if (total <= cap && edges) {
#pragma omp parallel for schedule(dynamic, 16) num_threads(n_threads)
    for (uint32_t a = 0; a < V; ++a) {
      uint64_t w = cnt[a];
      for (uint32_t b = a + 1; b < V; ++b) {
        if (m->vreg_class[a] != m->vreg_class[b]) continue;
        int64_t p = first_common_point(seg, seg_off[a], seg_off[a + 1], seg_off[b], seg_off[b + 1]);
        if (p >= 0) { edges[w].a = a; edges[w].b = b; edges[w].first = (uint32_t)p; ++w; }
      }
    }
  }
  free(cnt);
  return total;
}

/* ---- verification ------------------------------------------------------- */
void vlo_first_occurrence(const vlo_mir *m, uint32_t *first) {
  for (uint32_t v = 0; v < m->n_vreg; ++v) first[v] = UINT32_MAX;
  for (uint32_t o = m->n_occ; o-- > 0;) first[m->occ_vreg[o]] = o;
}

/* Section 3.4 Realizability; Section 2 (a wide value takes consecutive 32-bit
 * registers); Section 3.1 (number of available registers, reserved registers). */
static uint32_t realizability_bits(const vlo_mir *m, uint32_t v, uint32_t preg) {
  const uint32_t c = m->vreg_class[v], w = m->vreg_width[v], al = m->vreg_align[v];
  uint32_t bad = 0;
  if (preg + w > m->class_size[c]) bad |= VLO_BAD_BOUNDS;
  if (preg % al != 0) bad |= VLO_BAD_ALIGN;
  if (m->class_reserved)
    for (uint32_t r = preg; r < preg + w; ++r)
      if (r < 512 && ((m->class_reserved[c * 16 + (r >> 5)] >> (r & 31)) & 1u)) bad |= VLO_BAD_RESERVED;
  return bad;
}

/* consistency, then realizability; returns 1 if a result was written */
static int check_table(const vlo_mir *m, const uint32_t *first, const uint16_t *c, vlo_result *r) {
  /* Consistency: the same virtual register always maps to the same physical one */
  for (uint32_t o = 0; o < m->n_occ; ++o) {
    uint32_t v = m->occ_vreg[o];
    if (c[o] != c[first[v]]) {
      r->status = VLO_CONSISTENCY; r->where = o; r->a = v; r->b = first[v];
      return 1;
    }
  }
  uint32_t best = UINT32_MAX, bv = 0, bbits = 0;
  for (uint32_t v = 0; v < m->n_vreg; ++v) {
    if (first[v] == UINT32_MAX) continue;
    uint32_t bits = realizability_bits(m, v, c[first[v]]);
    if (bits && first[v] < best) { best = first[v]; bv = v; bbits = bits; }
  }
  if (best != UINT32_MAX) {
    r->status = VLO_REALIZABILITY; r->where = best; r->a = bv; r->b = bbits;
    return 1;
  }
  return 0;
}

static int ranges_meet(const vlo_mir *m, const uint32_t *first, const uint16_t *c,
                       uint32_t a, uint32_t b) {
  uint32_t pa = c[first[a]], pb = c[first[b]];
  return pa < pb + m->vreg_width[b] && pb < pa + m->vreg_width[a];
}

void vlo_verify(const vlo_mir *m, const vlo_edge *edges, uint64_t n_edges,
                const uint16_t *cand, uint32_t K, uint64_t ld, vlo_result *out,
                int n_threads) {
  uint32_t *first = (uint32_t *)malloc(((size_t)m->n_vreg + 1) * 4);
  vlo_first_occurrence(m, first);
  if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
  for (uint32_t k = 0; k < K; ++k) {
    const uint16_t *c = cand + (size_t)k * ld;
    vlo_result r = {VLO_OK, 0, 0, 0};
    if (!check_table(m, first, c, &r)) {
      /* Safety: overlapping lifetimes need disjoint registers; report the
       * lexicographically smallest (point, a, b) */
      int found = 0;
      for (uint64_t e = 0; e < n_edges; ++e) {
        const vlo_edge *g = &edges[e];
        if (!ranges_meet(m, first, c, g->a, g->b)) continue;
        if (!found || g->first < r.where || (g->first == r.where && (g->a < r.a || (g->a == r.a && g->b < r.b)))) {
          r.status = VLO_SAFETY; r.where = g->first; r.a = g->a; r.b = g->b;
          found = 1;
        }
      }
    }
    out[k] = r;
  }
  free(first);
}

void vlo_verify_points(const vlo_mir *m, const uint32_t *P, const uint16_t *c, vlo_result *out) {
  const uint32_t W = words_per_row(m), V = m->n_vreg;
  uint32_t *first = (uint32_t *)malloc(((size_t)V + 1) * 4);
  vlo_first_occurrence(m, first);
  vlo_result r = {VLO_OK, 0, 0, 0};
  if (!check_table(m, first, c, &r)) {
    for (uint32_t i = 0; i < m->n_instr && r.status == VLO_OK; ++i) {
      const uint32_t *row = P + (size_t)i * W;
      for (uint32_t a = 0; a < V && r.status == VLO_OK; ++a) {
        if (!bit_get(row, a)) continue;
        for (uint32_t b = a + 1; b < V; ++b) {
          if (!bit_get(row, b) || m->vreg_class[a] != m->vreg_class[b]) continue;
          if (ranges_meet(m, first, c, a, b)) {
            r.status = VLO_SAFETY; r.where = i; r.a = a; r.b = b;
            break;
          }
        }
      }
    }
  }
  *out = r;
  free(first);
}

int vlo_contract(const vlo_mir *m, const uint8_t *live_in) {
  for (uint32_t v = 0; v < m->n_vreg; ++v)
    if (live_in[v]) return 1;
  uint8_t *has = (uint8_t *)calloc((size_t)m->n_block + 1, 1);
  for (uint32_t b = 0; b < m->n_block; ++b)
    for (uint32_t e = m->succ_off[b]; e < m->succ_off[b + 1]; ++e)
      if (b < m->succ[e]) has[m->succ[e]] = 1;
  int bad = 0;
  for (uint32_t b = 1; b < m->n_block; ++b)
    if (!has[b]) bad = 2;
  free(has);
  return bad;
}

/* ---- regeneration-loop reductions (Section 3.4 last paragraph, Section 4.2 metrics) ---- */
void vlo_summarize(const vlo_result *res, uint32_t K, vlo_summary *out) {
  out->first_ok = K;
  out->passed = 0;
  for (int s = 0; s < 4; ++s) out->hist[s] = 0;
  for (uint32_t k = 0; k < K; ++k) {
    out->hist[res[k].status] += 1;
    if (res[k].status == VLO_OK && !out->passed) {
      out->first_ok = k;
      out->passed = 1;
    }
  }
}

void vlo_loop(const vlo_summary *s, const uint32_t *K, uint32_t n, vlo_loop_stats *out) {
  out->n_passed = 0;
  out->max_tries = 0;
  out->sum_tries = 0;
  for (int t = 0; t < 4; ++t) out->hist[t] = 0;
  for (uint32_t j = 0; j < n; ++j) {
    uint32_t tries = s[j].passed ? s[j].first_ok + 1 : K[j];
    out->n_passed += s[j].passed;
    if (tries > out->max_tries) out->max_tries = tries;
    out->sum_tries += tries;
    for (int t = 0; t < 4; ++t) out->hist[t] += s[j].hist[t];
  }
}

/* ---- constrained decoding (Section 4.5, error analysis: masking occupied registers) ---- */
void vlo_free_bases(const vlo_mir *m, const uint32_t *P, const uint16_t *cand, uint32_t q, uint32_t out[16]) {
  const uint32_t W = words_per_row(m), V = m->n_vreg;
  uint32_t *first = (uint32_t *)malloc(((size_t)V + 1) * 4);
  vlo_first_occurrence(m, first);
  const uint32_t v = m->occ_vreg[q];
  uint32_t i = 0;
  while (m->instr_occ_off[i + 1] <= q) ++i; /* the instruction of occurrence q */
  const uint32_t cls = m->vreg_class[v], w = m->vreg_width[v], al = m->vreg_align[v], F = m->class_size[cls];
  uint8_t blocked[512];
  memset(blocked, 0, sizeof blocked);
  if (m->class_reserved)
    for (uint32_t r = 0; r < 512; ++r)
      if ((m->class_reserved[cls * 16 + (r >> 5)] >> (r & 31)) & 1u) blocked[r] = 1;
  const uint32_t *row = P + (size_t)i * W;
  for (uint32_t b = 0; b < V; ++b) {
    if (first[v] < q) break; /* a later mention of v: consistency alone decides */
    if (b == v || !bit_get(row, b) || m->vreg_class[b] != cls || first[b] >= q) continue;
    const uint32_t pb = cand[first[b]];
    for (uint32_t r = pb; r < pb + m->vreg_width[b]; ++r)
      if (r < 512) blocked[r] = 1;
  }
  for (int t = 0; t < 16; ++t) out[t] = 0;
  for (uint32_t p = 0; p < 512; ++p) {
    int ok = p % al == 0 && p + w <= F;
    for (uint32_t r = p; ok && r < p + w; ++r)
      if (r >= 512 || blocked[r]) ok = 0;
    if (first[v] < q && p != cand[first[v]]) ok = 0;
    if (ok) out[p >> 5] |= 1u << (p & 31);
  }
  free(first);
}

/* ---- all violations (Section 4.5 error taxonomy; Section 6 verifier as reward) ---------- */
void vlo_count_violations(const vlo_mir *m, const vlo_edge *edges, uint64_t n_edges,
                          const uint16_t *cand, uint32_t K, uint64_t ld, vlo_counts *out,
                          int n_threads) {
  uint32_t *first = (uint32_t *)malloc(((size_t)m->n_vreg + 1) * 4);
  vlo_first_occurrence(m, first);
  if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
  for (uint32_t k = 0; k < K; ++k) {
    const uint16_t *c = cand + (size_t)k * ld;
    vlo_counts r;
    memset(&r, 0, sizeof r);
    for (uint32_t o = 0; o < m->n_occ; ++o)
      if (c[o] != c[first[m->occ_vreg[o]]]) r.n_cons += 1;
    for (uint32_t v = 0; v < m->n_vreg; ++v) {
      if (first[v] == UINT32_MAX) continue;
      uint32_t bits = realizability_bits(m, v, c[first[v]]);
      if (bits) { r.n_real += 1; r.real_bits |= bits; }
    }
    for (uint64_t e = 0; e < n_edges; ++e)
      if (ranges_meet(m, first, c, edges[e].a, edges[e].b)) r.n_safe += 1;
    r.kinds = (r.n_cons ? 1u : 0u) | (r.n_real ? 2u : 0u) | (r.n_safe ? 4u : 0u);
    out[k] = r;
  }
  free(first);
}

/* ---- register-bank conflicts (Section 2: banks, the FFMA example) ----------------------- */
void vlo_bank_conflicts(const vlo_mir *m, const uint16_t *cand, uint32_t K, uint64_t ld,
                        uint32_t n_banks, uint32_t *out) {
  uint32_t *per_bank = (uint32_t *)malloc((size_t)n_banks * 4);
  for (uint32_t k = 0; k < K; ++k) {
    const uint16_t *c = cand + (size_t)k * ld;
    uint32_t total = 0;
    for (uint32_t i = 0; i < m->n_instr; ++i) {
      for (uint32_t b = 0; b < n_banks; ++b) per_bank[b] = 0;
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o) {
        if (!(m->occ_flags[o] & VLO_OCC_USE)) continue;
        const uint32_t v = m->occ_vreg[o];
        int seen = 0; /* an earlier USE operand of this instruction with the same vreg */
        for (uint32_t x = m->instr_occ_off[i]; x < o; ++x)
          if ((m->occ_flags[x] & VLO_OCC_USE) && m->occ_vreg[x] == v) seen = 1;
        if (seen) continue;
        for (uint32_t j = 0; j < m->vreg_width[v]; ++j) per_bank[((uint32_t)c[o] + j) % n_banks] += 1;
      }
      uint32_t worst = 0;
      for (uint32_t b = 0; b < n_banks; ++b)
        if (per_bank[b] > worst) worst = per_bank[b];
      if (worst > 1) total += worst - 1;
    }
    out[k] = total;
  }
  free(per_bank);
}

/* ---- liveness of parts of a tuple (see vlo.h) -------------------------------------------- */
void vlo_lane_base(const vlo_mir *m, uint32_t *lane_base) {
  uint32_t n = 0;
  for (uint32_t v = 0; v < m->n_vreg; ++v) { lane_base[v] = n; n += m->vreg_width[v]; }
  lane_base[m->n_vreg] = n;
}

/* does occurrence o access lane j of its vreg? */
static int touches(const vlo_mir *m, const uint32_t *occ_lanes, uint32_t o, uint32_t j) {
  if (!occ_lanes || occ_lanes[o] == 0) return 1;
  (void)m;
  return (occ_lanes[o] >> j) & 1u;
}

int vlo_block_liveness_lanes(const vlo_mir *m, const uint32_t *occ_lanes, uint8_t *live_in, uint8_t *live_out) {
  const uint32_t B = m->n_block;
  uint32_t *base = (uint32_t *)malloc(((size_t)m->n_vreg + 1) * 4);
  vlo_lane_base(m, base);
  const uint32_t Lt = base[m->n_vreg];
  uint8_t *use = (uint8_t *)calloc((size_t)B * Lt + 1, 1);
  uint8_t *def = (uint8_t *)calloc((size_t)B * Lt + 1, 1);
  for (uint32_t b = 0; b < B; ++b) {
    uint8_t *u = use + (size_t)b * Lt, *d = def + (size_t)b * Lt;
    for (uint32_t i = m->blk_start[b]; i < m->blk_start[b + 1]; ++i) {
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_USE)
          for (uint32_t j = 0; j < m->vreg_width[m->occ_vreg[o]]; ++j)
            if (touches(m, occ_lanes, o, j) && !d[base[m->occ_vreg[o]] + j]) u[base[m->occ_vreg[o]] + j] = 1;
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_DEF)
          for (uint32_t j = 0; j < m->vreg_width[m->occ_vreg[o]]; ++j)
            if (touches(m, occ_lanes, o, j)) d[base[m->occ_vreg[o]] + j] = 1;
    }
  }
  memset(live_in, 0, (size_t)B * Lt);
  memset(live_out, 0, (size_t)B * Lt);
  int sweeps = 0, changed = 1;
  while (changed) {
    changed = 0;
    ++sweeps;
    for (uint32_t b = 0; b < B; ++b) {
      uint8_t *in = live_in + (size_t)b * Lt, *out = live_out + (size_t)b * Lt;
      for (uint32_t e = m->succ_off[b]; e < m->succ_off[b + 1]; ++e) {
        const uint8_t *sin = live_in + (size_t)m->succ[e] * Lt;
        for (uint32_t x = 0; x < Lt; ++x)
          if (sin[x] && !out[x]) { out[x] = 1; changed = 1; }
      }
      for (uint32_t x = 0; x < Lt; ++x) {
        uint8_t nv = (uint8_t)(use[(size_t)b * Lt + x] | (out[x] & !def[(size_t)b * Lt + x]));
        if (nv && !in[x]) { in[x] = 1; changed = 1; }
      }
    }
  }
  free(use);
  free(def);
  free(base);
  return sweeps;
}

void vlo_points_lanes(const vlo_mir *m, const uint32_t *occ_lanes, const uint8_t *live_out, uint8_t *live_after) {
  uint32_t *base = (uint32_t *)malloc(((size_t)m->n_vreg + 1) * 4);
  vlo_lane_base(m, base);
  const uint32_t Lt = base[m->n_vreg];
  uint8_t *cur = (uint8_t *)calloc((size_t)Lt + 1, 1);
  for (uint32_t b = 0; b < m->n_block; ++b) {
    memcpy(cur, live_out + (size_t)b * Lt, Lt);
    for (uint32_t i = m->blk_start[b + 1]; i-- > m->blk_start[b];) {
      memcpy(live_after + (size_t)i * Lt, cur, Lt);
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_DEF)
          for (uint32_t j = 0; j < m->vreg_width[m->occ_vreg[o]]; ++j)
            if (touches(m, occ_lanes, o, j)) cur[base[m->occ_vreg[o]] + j] = 0;
      for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
        if (m->occ_flags[o] & VLO_OCC_USE)
          for (uint32_t j = 0; j < m->vreg_width[m->occ_vreg[o]]; ++j)
            if (touches(m, occ_lanes, o, j)) cur[base[m->occ_vreg[o]] + j] = 1;
    }
  }
  free(cur);
  free(base);
}

void vlo_occupancy_lanes(const vlo_mir *m, const uint32_t *occ_lanes, const uint8_t *live_after, uint8_t *P) {
  uint32_t *base = (uint32_t *)malloc(((size_t)m->n_vreg + 1) * 4);
  vlo_lane_base(m, base);
  const uint32_t Lt = base[m->n_vreg];
  memcpy(P, live_after, (size_t)m->n_instr * Lt);
  for (uint32_t i = 0; i < m->n_instr; ++i) {
    int early = 0;
    for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
      if (m->occ_flags[o] & VLO_OCC_EARLY) early = 1;
    for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o)
      if ((m->occ_flags[o] & VLO_OCC_DEF) || (early && (m->occ_flags[o] & VLO_OCC_USE)))
        for (uint32_t j = 0; j < m->vreg_width[m->occ_vreg[o]]; ++j)
          if (touches(m, occ_lanes, o, j)) P[(size_t)i * Lt + base[m->occ_vreg[o]] + j] = 1;
  }
  free(base);
}

void vlo_kill_lanes(const vlo_mir *m, const uint32_t *occ_lanes, const uint8_t *live_after, uint32_t *occ_kill) {
  uint32_t *base = (uint32_t *)malloc(((size_t)m->n_vreg + 1) * 4);
  vlo_lane_base(m, base);
  const uint32_t Lt = base[m->n_vreg];
  for (uint32_t i = 0; i < m->n_instr; ++i)
    for (uint32_t o = m->instr_occ_off[i]; o < m->instr_occ_off[i + 1]; ++o) {
      const uint32_t v = m->occ_vreg[o];
      uint32_t killed = 0;
      for (uint32_t j = 0; j < m->vreg_width[v]; ++j) {
        if (!(m->occ_flags[o] & VLO_OCC_USE) || !touches(m, occ_lanes, o, j)) continue;
        int written = 0;
        for (uint32_t x = m->instr_occ_off[i]; x < m->instr_occ_off[i + 1]; ++x)
          if ((m->occ_flags[x] & VLO_OCC_DEF) && m->occ_vreg[x] == v && touches(m, occ_lanes, x, j)) written = 1;
        if (!written && !live_after[(size_t)i * Lt + base[v] + j]) killed |= 1u << j;
      }
      occ_kill[o] = killed;
    }
  free(base);
}

uint64_t vlo_segments_lanes(const vlo_mir *m, const uint8_t *P, uint32_t *seg_off, uint32_t *seg, uint64_t cap,
                            uint32_t *hull) {
  uint32_t *base = (uint32_t *)malloc(((size_t)m->n_vreg + 1) * 4);
  vlo_lane_base(m, base);
  const uint32_t Lt = base[m->n_vreg], N = m->n_instr;
  free(base);
  uint64_t n = 0;
  /* lane by lane, the maximal runs of membership in order */
  for (uint32_t x = 0; x < Lt; ++x) {
    seg_off[x] = (uint32_t)n;
    hull[2 * x] = hull[2 * x + 1] = 0;
    int first = 1;
    for (uint32_t i = 0; i < N; ++i) {
      if (!P[(size_t)i * Lt + x] || (i && P[(size_t)(i - 1) * Lt + x])) continue;
      uint32_t e = i;
      while (e < N && P[(size_t)e * Lt + x]) ++e;
      if (seg && n < cap) { seg[2 * n] = i; seg[2 * n + 1] = e; }
      if (first) { hull[2 * x] = i; first = 0; }
      hull[2 * x + 1] = e;
      ++n;
    }
  }
  seg_off[Lt] = (uint32_t)n;
  return n;
}

void vlo_verify_lanes(const vlo_mir *m, const uint8_t *P, const uint16_t *c, vlo_result *out) {
  const uint32_t V = m->n_vreg;
  uint32_t *first = (uint32_t *)malloc(((size_t)V + 1) * 4);
  uint32_t *base = (uint32_t *)malloc(((size_t)V + 1) * 4);
  vlo_first_occurrence(m, first);
  vlo_lane_base(m, base);
  const uint32_t Lt = base[V];
  vlo_result r = {VLO_OK, 0, 0, 0};
  if (!check_table(m, first, c, &r)) {
    /* Safety on the lanes in use: who claims each register of each file at i */
    uint32_t *owner = (uint32_t *)malloc((size_t)m->n_class * 512 * 4);
    for (uint32_t i = 0; i < m->n_instr && r.status == VLO_OK; ++i) {
      for (uint32_t x = 0; x < m->n_class * 512; ++x) owner[x] = UINT32_MAX;
      uint32_t ba = UINT32_MAX, bb = UINT32_MAX;
      for (uint32_t v = 0; v < V; ++v)          /* ascending: the first claimant of a register is its smallest vreg */
        for (uint32_t j = 0; j < m->vreg_width[v]; ++j) {
          if (!P[(size_t)i * Lt + base[v] + j]) continue;
          const uint32_t reg = (uint32_t)c[first[v]] + j;   /* in bounds: realizability holds */
          uint32_t *w = &owner[m->vreg_class[v] * 512 + reg];
          if (*w == UINT32_MAX) *w = v;
          else if (*w != v && (*w < ba || (*w == ba && v < bb))) { ba = *w; bb = v; }
        }
      if (ba != UINT32_MAX) { r.status = VLO_SAFETY; r.where = i; r.a = ba; r.b = bb; }
    }
    free(owner);
  }
  *out = r;
  free(first);
  free(base);
}
