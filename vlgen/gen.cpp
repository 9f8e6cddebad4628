// Seeded synthetic inputs: machine-IR kernels shaped like GEMM and attention
// kernels, allocations for them, and deliberately damaged allocations.
//
// INPUT GENERATION ONLY.  Nothing here analyses a program or checks an
// allocation: the builder records, for each virtual register it creates, a
// conservative range of instructions it may occupy (known from how the
// generator placed its definitions and uses, and from which loops it made the
// value cross) and hands those ranges to a first-fit allocator.  Whether the
// resulting rows are really valid is for the oracle and the GPU library to say.
//
// The paper's datasets (Section 4.1, Appendix A) are not available; these
// kernels take their structure from its description: GEMM with tiles, unrolled
// bodies and software pipelines, accumulators held in a unified
// VGPR/AccVGPR file (Section 4.7); attention with projection / score / weighted
// sum phases and many more basic blocks (Section 4.1, Appendix A).
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

struct Rng {  // SplitMix64
  uint64_t s;
  explicit Rng(uint64_t seed) : s(seed) {}
  uint64_t next() {
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  uint32_t below(uint32_t n) { return n ? (uint32_t)(next() % n) : 0; }
  bool chance(uint32_t num, uint32_t den) { return below(den) < num; }
  uint32_t geometric(uint32_t mean) {  // on {1,2,..}, success probability 1/mean
    uint32_t g = 1;
    while (below(mean) != 0 && g < 100000) ++g;
    return g;
  }
};

constexpr uint8_t DEF = 1, USE = 2;
constexpr uint32_t NONE = 0xFFFFFFFFu;

struct Loop { uint32_t lo, hi; };

struct Kernel {
  std::vector<uint32_t> blk_start{0};
  std::vector<std::vector<uint32_t>> succ;
  std::vector<uint32_t> occ_off{0};
  std::vector<uint32_t> occ_vreg;
  std::vector<uint8_t> occ_flags;
  std::vector<uint8_t> vclass, vwidth, valign;
  std::vector<uint16_t> class_size;
  // what the generator knows by construction
  std::vector<uint32_t> lo, hi;        // conservative occupancy range [lo,hi)
  std::vector<uint32_t> sure_lo, sure_hi;  // range where occupancy is certain (may be empty)
  std::vector<uint32_t> n_def, def_blk, n_occ_of;
  std::vector<uint8_t> local;          // all occurrences in one block, definition first
  std::vector<Loop> loops;
  bool closed = false;

  uint32_t n_instr() const { return (uint32_t)occ_off.size() - 1; }
  uint32_t n_vreg() const { return (uint32_t)vclass.size(); }
  uint32_t cur_block() const { return (uint32_t)blk_start.size() - 1; }

  uint32_t vreg(uint32_t cls, uint32_t width) {
    vclass.push_back((uint8_t)cls); vwidth.push_back((uint8_t)width); valign.push_back((uint8_t)width);
    lo.push_back(NONE); hi.push_back(0); sure_lo.push_back(0); sure_hi.push_back(0);
    n_def.push_back(0); def_blk.push_back(NONE); n_occ_of.push_back(0); local.push_back(1);
    return n_vreg() - 1;
  }
  void touch(uint32_t v, uint32_t i, bool is_def) {
    lo[v] = std::min(lo[v], i);
    hi[v] = std::max(hi[v], is_def ? i + 1 : i);
    uint32_t b = cur_block();
    if (is_def) {
      if (n_occ_of[v] != 0) local[v] = 0;  // defined after another occurrence
      ++n_def[v];
      def_blk[v] = b;
    } else if (def_blk[v] != b) {
      local[v] = 0;
    }
    ++n_occ_of[v];
  }
  uint32_t emit(const std::vector<uint32_t>& defs, const std::vector<uint32_t>& uses) {
    uint32_t i = n_instr();
    for (uint32_t d : defs) { occ_vreg.push_back(d); occ_flags.push_back(DEF); }
    for (uint32_t u : uses) { occ_vreg.push_back(u); occ_flags.push_back(USE); }
    // uses are read before defs are written: record them in that order
    for (uint32_t u : uses) touch(u, i, false);
    for (uint32_t d : defs) touch(d, i, true);
    occ_off.push_back((uint32_t)occ_vreg.size());
    return i;
  }
  void end_block(std::vector<uint32_t> successors) {
    blk_start.push_back(n_instr());
    succ.push_back(std::move(successors));
  }
  void add_loop(uint32_t first_instr, uint32_t end_instr) { loops.push_back({first_instr, end_instr}); }

  // After the last block: widen ranges over the loops a value crosses and
  // derive the certain ranges of block-local single-definition values.
  void close() {
    const uint32_t V = n_vreg(), O = (uint32_t)occ_vreg.size();
    std::vector<uint32_t> occ_instr(O);
    for (uint32_t i = 0; i < n_instr(); ++i)
      for (uint32_t o = occ_off[i]; o < occ_off[i + 1]; ++o) occ_instr[o] = i;
    // per vreg occurrence lists
    std::vector<uint32_t> off(V + 1, 0), lst(O);
    for (uint32_t o = 0; o < O; ++o) ++off[occ_vreg[o] + 1];
    for (uint32_t v = 0; v < V; ++v) off[v + 1] += off[v];
    { std::vector<uint32_t> cur(off.begin(), off.end() - 1);
      for (uint32_t o = 0; o < O; ++o) lst[cur[occ_vreg[o]]++] = o; }
    // innermost loops were added first or last in no fixed order: iterate to a
    // fixed point so that nested extensions propagate outwards
    bool again = true;
    while (again) {
      again = false;
      for (const Loop& L : loops) {
        for (uint32_t v = 0; v < V; ++v) {
          if (lo[v] == NONE) continue;
          bool inside = false, before = lo[v] < L.lo, first_is_use = false;
          for (uint32_t e = off[v]; e < off[v + 1]; ++e) {
            uint32_t i = occ_instr[lst[e]];
            if (i >= L.lo && i < L.hi) {
              if (!inside) {
                inside = true;
                // a use anywhere in the first mentioning instruction counts
                for (uint32_t f = e; f < off[v + 1] && occ_instr[lst[f]] == i; ++f)
                  if (occ_flags[lst[f]] & USE) first_is_use = true;
              }
            }
          }
          // also values whose range already straddles the loop entry
          bool straddles = lo[v] < L.lo && hi[v] > L.lo;
          if ((inside && (before || first_is_use)) || straddles) {
            uint32_t nlo = std::min(lo[v], L.lo), nhi = std::max(hi[v], L.hi);
            if (inside && first_is_use && !before) nlo = std::min(nlo, L.lo);
            if (nlo != lo[v] || nhi != hi[v]) { lo[v] = nlo; hi[v] = nhi; again = true; }
          }
        }
      }
    }
    for (uint32_t v = 0; v < V; ++v) {
      if (lo[v] == NONE) { lo[v] = hi[v] = 0; continue; }
      if (local[v] && n_def[v] == 1 && sure_hi[v] == 0) {
        // defined once, then only read further down the same block: occupied
        // from the definition up to (not including) the last read
        uint32_t d = occ_instr[lst[off[v]]];
        uint32_t last = occ_instr[lst[off[v + 1] - 1]];
        sure_lo[v] = d;
        sure_hi[v] = std::max(last, d + 1);
      }
    }
    closed = true;
  }
};

// ---------------------------------------------------------------------------
// kernel shapes
// ---------------------------------------------------------------------------

uint32_t pick_width(Rng& r, const uint32_t* w, const uint32_t* pct, int n) {
  uint32_t x = r.below(100), acc = 0;
  for (int i = 0; i < n; ++i) { acc += pct[i]; if (x < acc) return w[i]; }
  return w[n - 1];
}

// config 1: one block, instruction i defines v_i and reads two earlier values
Kernel* make_straight(uint64_t seed, uint32_t N) {
  Rng r(seed);
  Kernel* k = new Kernel;
  k->class_size = {256};
  for (uint32_t i = 0; i < N; ++i) {
    uint32_t v = k->vreg(0, 1);
    std::vector<uint32_t> uses;
    if (i > 0)
      for (int j = 0; j < 2; ++j) uses.push_back(i - std::min(i, r.geometric(10)));
    k->emit({v}, uses);
  }
  k->end_block({});
  k->close();
  return k;
}

// Emits straight-line filler into the current block.
struct Filler {
  Kernel* k; Rng* r;
  const uint32_t* widths; const uint32_t* pct; int nw;
  uint32_t sgpr_pct;           // share of new values in the scalar class
  std::vector<uint32_t> recent;   // defined in this block, in order
  std::vector<uint32_t> globals;  // readable anywhere in this block
  int64_t* defs_left; int64_t* slots_left;

  void begin() { recent.clear(); }
  uint32_t operand() {
    uint32_t g = r->geometric(10);
    if (g <= recent.size()) return recent[recent.size() - g];
    if (!globals.empty()) return globals[r->below((uint32_t)globals.size())];
    if (!recent.empty()) return recent[r->below((uint32_t)recent.size())];
    return NONE;
  }
  // one generic instruction; defines a new value when the budget says so
  void one() {
    bool def = *defs_left > 0 && (int64_t)r->below((uint32_t)std::max<int64_t>(*slots_left, 1)) < *defs_left;
    std::vector<uint32_t> uses;
    for (int j = 0; j < 2; ++j) { uint32_t u = operand(); if (u != NONE) uses.push_back(u); }
    std::vector<uint32_t> defs;
    // a second definition when the budget has fallen behind the slots left
    int n_def = def ? ((*defs_left - 1 > *slots_left - 1) ? 2 : 1) : 0;
    for (int d = 0; d < n_def; ++d) {
      uint32_t cls = r->below(100) < sgpr_pct ? 1 : 0;
      uint32_t w = pick_width(*r, widths, pct, nw);
      if (cls == 1 && w > 4) w = 4;
      defs.push_back(k->vreg(cls, w));
      --*defs_left;
    }
    k->emit(defs, uses);
    for (uint32_t d : defs) recent.push_back(d);
    --*slots_left;
  }
  void run(uint32_t n) { for (uint32_t i = 0; i < n; ++i) one(); }
};

// config 2: prologue / loop body with a back edge / epilogue
Kernel* make_loop3(uint64_t seed, uint32_t n_pro, uint32_t n_body, uint32_t n_epi, uint32_t V, uint32_t n_cross) {
  Rng r(seed);
  Kernel* k = new Kernel;
  k->class_size = {256, 102};
  static const uint32_t W[] = {1, 2, 4}, P[] = {70, 20, 10};
  int64_t defs_left = V, slots_left = (int64_t)n_pro + n_body + n_epi;
  Filler f{k, &r, W, P, 3, 20, {}, {}, &defs_left, &slots_left};
  // values that cross the back edge: half are set once in the prologue and read
  // in the body; half are set in the prologue, read early in the body and set
  // again late in the body for the next trip
  std::vector<uint32_t> cross;
  for (uint32_t c = 0; c < n_cross; ++c) {
    uint32_t cls = r.below(100) < 20 ? 1 : 0;
    cross.push_back(k->vreg(cls, pick_width(r, W, P, 3)));
  }
  defs_left -= n_cross;
  f.begin();
  for (uint32_t i = 0; i < n_pro; ++i) {
    uint32_t slot = n_pro - n_cross;
    if (i >= slot) {  // last n_cross prologue instructions define the crossing values
      k->emit({cross[i - slot]}, {});
      --slots_left;
    } else f.one();
  }
  k->end_block({1});
  uint32_t body_lo = k->n_instr();
  f.begin();
  uint32_t early = n_body / 8, late = n_body - n_body / 8;
  for (uint32_t i = 0; i < n_body; ++i) {
    if (i < early && i < n_cross) {           // read every crossing value early
      k->emit({}, {cross[i]}); --slots_left;
    } else if (i >= late && (i - late) < n_cross / 2) {  // set half of them again late
      uint32_t u = f.operand();
      std::vector<uint32_t> uses; if (u != NONE) uses.push_back(u);
      k->emit({cross[i - late]}, uses); --slots_left;
    } else f.one();
  }
  k->end_block({1, 2});
  k->add_loop(body_lo, k->n_instr());
  f.begin();
  f.run(n_epi);
  k->end_block({});
  // exact V: any budget left over becomes values defined in... (none: slots >= defs)
  k->close();
  return k;
}

struct Shape {
  Kernel* k; Rng r;
  int64_t defs_left, slots_left;
  explicit Shape(uint64_t seed) : k(new Kernel), r(seed), defs_left(0), slots_left(0) {}
};

// GEMM-shaped: prologue, then phases of { accumulator init, outer-loop head,
// inner-loop body, outer-loop tail, epilogue }, then a final block.
Kernel* make_gemm(uint64_t seed, uint32_t N, uint32_t V) {
  Shape s(seed);
  Kernel* k = s.k; Rng& r = s.r;
  k->class_size = {512, 102};
  static const uint32_t W[] = {1, 2, 4}, P[] = {60, 25, 15};
  const uint32_t n_phase = 4, n_acc = 16;
  // structural values are set aside first; the rest of V is spread over fillers
  s.defs_left = (int64_t)V - (6 + n_phase * (n_acc + 2)); s.slots_left = (int64_t)N - 1;
  Filler f{k, &r, W, P, 3, 15, {}, {}, &s.defs_left, &s.slots_left};
  auto fixed = [&](const std::vector<uint32_t>& d, const std::vector<uint32_t>& u) {
    k->emit(d, u); --s.slots_left;
  };
  auto newv = [&](uint32_t cls, uint32_t w) { return k->vreg(cls, w); };          // structural
  auto newb = [&](uint32_t cls, uint32_t w) { --s.defs_left; return k->vreg(cls, w); };  // from the budget
  // budget of instructions per block
  uint32_t n_pro = std::max<uint32_t>(N / 40, 12), n_fin = std::max<uint32_t>(N / 40, 8);
  uint32_t per_phase = (N - n_pro - n_fin) / n_phase;
  uint32_t n_init = n_acc + 2, n_oh = std::max<uint32_t>(per_phase / 20, 6);
  uint32_t n_ot = std::max<uint32_t>(per_phase / 40, 4), n_ep = std::max<uint32_t>(per_phase / 7, n_acc + 4);
  // prologue: scalar base addresses (pairs) that live to the end
  std::vector<uint32_t> addr;
  f.begin();
  for (int a = 0; a < 6; ++a) { uint32_t v = newv(1, 2); fixed({v}, {}); addr.push_back(v); }
  f.globals = addr;
  f.run(n_pro - 6);
  k->end_block({1});
  for (uint32_t p = 0; p < n_phase; ++p) {
    uint32_t base_blk = 1 + 5 * p;
    uint32_t n_ib = per_phase - n_init - n_oh - n_ot - n_ep;
    if (p == n_phase - 1) {  // absorb rounding in the last inner body
      uint32_t used = k->n_instr() + n_init + n_oh + n_ot + n_ep + n_fin;
      n_ib = N - used;
    }
    // accumulator init (outside both loops)
    std::vector<uint32_t> acc;
    f.begin();
    for (uint32_t a = 0; a < n_acc; ++a) { uint32_t v = newv(0, 16); fixed({v}, {}); acc.push_back(v); }
    uint32_t oc = newv(1, 1); fixed({oc}, {addr[0]});
    f.run(n_init - n_acc - 1);
    k->end_block({base_blk + 1});
    // outer head
    uint32_t outer_lo = k->n_instr();
    f.begin();
    uint32_t ic = newv(1, 1); fixed({ic}, {oc});
    f.run(n_oh - 1);
    k->end_block({base_blk + 2});
    // inner body: loads, MFMA-style accumulate, temporaries
    uint32_t inner_lo = k->n_instr();
    f.begin();
    std::vector<uint32_t> loads;
    uint32_t j = 0, next_acc = 0;
    while (j + 1 < n_ib) {
      uint32_t what = r.below(100);
      if (what < 30 && s.defs_left > 0) {          // wide load through a base address
        uint32_t v = newb(0, 4);
        fixed({v}, {addr[r.below((uint32_t)addr.size())]});
        loads.push_back(v);
      } else if (what < 55 && loads.size() >= 2) {  // acc += a * b
        uint32_t a = loads[loads.size() - std::min<uint32_t>((uint32_t)loads.size(), r.geometric(6))];
        uint32_t b = loads[loads.size() - std::min<uint32_t>((uint32_t)loads.size(), r.geometric(6))];
        uint32_t c = acc[next_acc++ % n_acc];
        fixed({c}, {c, a, b});
      } else f.one();
      ++j;
    }
    fixed({ic}, {ic});  // inner trip counter update + branch
    k->end_block({base_blk + 2, base_blk + 3});
    k->add_loop(inner_lo, k->n_instr());
    // outer tail
    f.begin();
    f.run(n_ot - 1);
    fixed({oc}, {oc});
    k->end_block({base_blk + 1, base_blk + 4});
    k->add_loop(outer_lo, k->n_instr());
    // epilogue: read every accumulator once (convert + store)
    f.begin();
    for (uint32_t a = 0; a < n_acc; ++a) {
      if (s.defs_left > 0) { uint32_t t = newb(0, 4); fixed({t}, {acc[a]}); f.recent.push_back(t); }
      else fixed({}, {acc[a], addr[1]});
    }
    f.run(n_ep - n_acc);
    k->end_block({base_blk + 5});
  }
  f.begin();
  uint32_t left = N - k->n_instr();
  for (uint32_t i = 0; i + 1 < left; ++i) f.one();
  {  // last instruction reads the base addresses so that they live to the end
    k->emit({}, addr); --s.slots_left;
  }
  k->end_block({});
  k->close();
  return k;
}

// Attention-shaped: outer key/value loop holding an inner score loop, a
// softmax section with four if/else diamonds, and an inner weighted-sum loop.
Kernel* make_mha(uint64_t seed, uint32_t N, uint32_t V) {
  Shape s(seed);
  Kernel* k = s.k; Rng& r = s.r;
  k->class_size = {512, 102};
  static const uint32_t W[] = {1, 2, 4, 8, 16}, P[] = {55, 22, 15, 6, 2};
  const uint32_t n_out = 8, n_sc = 4, n_q = 4, n_stat = 8;
  s.defs_left = (int64_t)V - (8 + n_q + n_stat + n_out + 1 + n_sc + 1 + n_sc + 1 + 8);
  s.slots_left = (int64_t)N - 1;
  Filler f{k, &r, W, P, 5, 12, {}, {}, &s.defs_left, &s.slots_left};
  auto fixed = [&](const std::vector<uint32_t>& d, const std::vector<uint32_t>& u) {
    k->emit(d, u); --s.slots_left;
  };
  auto newv = [&](uint32_t cls, uint32_t w) { return k->vreg(cls, w); };          // structural
  auto newb = [&](uint32_t cls, uint32_t w) { --s.defs_left; return k->vreg(cls, w); };  // from the budget
  uint32_t n_pro = std::max<uint32_t>(N / 25, 40), n_epi = std::max<uint32_t>(N / 20, 40);
  uint32_t loop_n = N - n_pro - n_epi;
  uint32_t n_oh = std::max<uint32_t>(loop_n / 12, 12), n_ot = std::max<uint32_t>(loop_n / 40, 6);
  uint32_t n_sm = std::max<uint32_t>(loop_n / 4, 60);   // softmax section incl. diamonds
  uint32_t n_ib1 = (loop_n - n_oh - n_ot - n_sm) / 2;
  uint32_t n_ib2 = loop_n - n_oh - n_ot - n_sm - n_ib1;
  // block ids: 0 prologue, 1 outer head, 2 score loop, 3 softmax head,
  // 4+3d / 5+3d / 6+3d then/else/join of diamond d (d = 0..3), 16 weighted-sum
  // loop, 17 outer tail, 18 epilogue
  // prologue: addresses, query fragments, running statistics, output accumulators
  std::vector<uint32_t> addr, q, stat, out;
  f.begin();
  for (int a = 0; a < 8; ++a) { uint32_t v = newv(1, 2); fixed({v}, {}); addr.push_back(v); }
  for (uint32_t a = 0; a < n_q; ++a) { uint32_t v = newv(0, 8); fixed({v}, {addr[0]}); q.push_back(v); }
  for (uint32_t a = 0; a < n_stat; ++a) { uint32_t v = newv(0, 1); fixed({v}, {}); stat.push_back(v); }
  for (uint32_t a = 0; a < n_out; ++a) { uint32_t v = newv(0, 16); fixed({v}, {}); out.push_back(v); }
  uint32_t oc = newv(1, 1); fixed({oc}, {addr[1]});
  f.globals = addr;
  f.run(n_pro - (8 + n_q + n_stat + n_out + 1));
  k->end_block({1});
  // outer head: score accumulators zeroed, key loads
  uint32_t outer_lo = k->n_instr();
  f.begin();
  std::vector<uint32_t> sc;
  for (uint32_t a = 0; a < n_sc; ++a) { uint32_t v = newv(0, 16); fixed({v}, {}); sc.push_back(v); }
  uint32_t ic = newv(1, 1); fixed({ic}, {oc});
  f.run(n_oh - n_sc - 1);
  k->end_block({2});
  // score loop
  uint32_t lo1 = k->n_instr();
  f.begin();
  { std::vector<uint32_t> loads; uint32_t nxt = 0;
    for (uint32_t j = 0; j + 1 < n_ib1; ++j) {
      uint32_t what = r.below(100);
      if (what < 28 && s.defs_left > 0) { uint32_t v = newb(0, 4); fixed({v}, {addr[2 + r.below(2)]}); loads.push_back(v); }
      else if (what < 50 && !loads.empty()) {
        uint32_t a = loads[loads.size() - std::min<uint32_t>((uint32_t)loads.size(), r.geometric(5))];
        uint32_t c = sc[nxt++ % n_sc];
        fixed({c}, {c, a, q[r.below(n_q)]});
      } else f.one();
    }
    fixed({ic}, {ic});
  }
  k->end_block({2, 3});
  k->add_loop(lo1, k->n_instr());
  // softmax head: reads the scores into row maxima
  uint32_t n_dia = 4, per_d = n_sm / (n_dia + 1);
  uint32_t n_head = n_sm - per_d * n_dia;
  f.begin();
  std::vector<uint32_t> rowmax;
  for (uint32_t a = 0; a < n_sc; ++a) { uint32_t v = newv(0, 1); fixed({v}, {sc[a]}); rowmax.push_back(v); f.recent.push_back(v); }
  uint32_t cond = newv(1, 1);
  f.run(n_head - n_sc - 1);
  fixed({cond}, {rowmax[0], stat[0]});
  k->end_block({4, 5});
  for (uint32_t d = 0; d < n_dia; ++d) {
    uint32_t bt = 4 + 3 * d, be = bt + 1, bj = bt + 2;
    uint32_t n_then = per_d / 3, n_else = per_d / 4, n_join = per_d - n_then - n_else;
    uint32_t z = newv(0, r.chance(1, 2) ? 1 : 2);   // set on both sides, read at the join
    // then: rescale (read-modify-write of a statistic and, for d == 2, the outputs)
    f.begin();
    fixed({stat[d]}, {stat[d], rowmax[d % n_sc]});
    uint32_t used = 1;
    if (d == 2) for (uint32_t a = 0; a < n_out && used + 1 < n_then; ++a) { fixed({out[a]}, {out[a], stat[d]}); ++used; }
    if (used + 1 < n_then) f.run(n_then - used - 1);
    { uint32_t u = f.operand(); std::vector<uint32_t> us{stat[d]}; if (u != NONE) us.push_back(u); fixed({z}, us); }
    k->end_block({bj});
    // else
    f.begin();
    if (n_else > 1) f.run(n_else - 1);
    fixed({z}, {rowmax[(d + 1) % n_sc]});
    k->end_block({bj});
    // join
    f.begin();
    fixed({stat[4 + d]}, {stat[4 + d], z});
    uint32_t nxt_cond = newv(1, 1);
    if (n_join > 2) f.run(n_join - 2);
    fixed({nxt_cond}, {stat[(d + 1) % n_stat], cond});
    cond = nxt_cond;
    if (d + 1 < n_dia) k->end_block({bj + 1, bj + 2}); else k->end_block({16});
  }
  // weighted-sum loop: out += p * v
  uint32_t lo2 = k->n_instr();
  f.begin();
  uint32_t ic2 = ic;
  { std::vector<uint32_t> loads; uint32_t nxt = 0;
    for (uint32_t j = 0; j + 1 < n_ib2; ++j) {
      uint32_t what = r.below(100);
      if (what < 28 && s.defs_left > 0) { uint32_t v = newb(0, 4); fixed({v}, {addr[4 + r.below(2)]}); loads.push_back(v); }
      else if (what < 50 && !loads.empty()) {
        uint32_t a = loads[loads.size() - std::min<uint32_t>((uint32_t)loads.size(), r.geometric(5))];
        uint32_t c = out[nxt++ % n_out];
        fixed({c}, {c, a, sc[r.below(n_sc)]});
      } else f.one();
    }
    fixed({ic2}, {ic2, cond});
  }
  k->end_block({16, 17});
  k->add_loop(lo2, k->n_instr());
  // outer tail
  f.begin();
  f.run(n_ot - 1);
  fixed({oc}, {oc});
  k->end_block({1, 18});
  k->add_loop(outer_lo, k->n_instr());
  // epilogue: normalise and store the outputs
  f.begin();
  for (uint32_t a = 0; a < n_out; ++a) fixed({out[a]}, {out[a], stat[a % n_stat]});
  for (uint32_t a = 0; a < n_out; ++a) fixed({}, {out[a], addr[6]});
  uint32_t left = N - k->n_instr();
  for (uint32_t i = 0; i + 1 < left; ++i) f.one();
  { std::vector<uint32_t> us = addr; for (uint32_t a = 0; a < n_stat; ++a) us.push_back(stat[a]);
    for (uint32_t a = 0; a < n_q; ++a) us.push_back(q[a]);
    k->emit({}, us); --s.slots_left; }
  k->end_block({});
  k->close();
  return k;
}

// ---------------------------------------------------------------------------
// allocation (first fit over the recorded ranges) and damage
// ---------------------------------------------------------------------------

struct Mut { uint32_t kind, vreg, other, expect; };

bool first_fit(const Kernel& k, Rng& r, bool randomized, std::vector<uint16_t>& table) {
  const uint32_t V = k.n_vreg();
  std::vector<uint32_t> order;
  for (uint32_t v = 0; v < V; ++v) if (k.hi[v] > k.lo[v]) order.push_back(v);
  std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return k.lo[a] < k.lo[b]; });
  const uint32_t C = (uint32_t)k.class_size.size();
  std::vector<std::vector<uint8_t>> busy(C);
  std::vector<uint32_t> start(C, 0);
  for (uint32_t c = 0; c < C; ++c) {
    busy[c].assign(k.class_size[c], 0);
    if (randomized) start[c] = r.below(k.class_size[c]);
  }
  uint32_t skip_pct = randomized ? r.below(12) : 0;
  // active values ordered by range end
  std::vector<std::pair<uint32_t, uint32_t>> active;  // min-heap on (end, vreg)
  auto cmp = [](const std::pair<uint32_t, uint32_t>& a, const std::pair<uint32_t, uint32_t>& b) { return a > b; };
  table.assign(V, 0);
  for (uint32_t v : order) {
    while (!active.empty() && active.front().first <= k.lo[v]) {
      uint32_t u = active.front().second;
      std::pop_heap(active.begin(), active.end(), cmp); active.pop_back();
      for (uint32_t x = 0; x < k.vwidth[u]; ++x) busy[k.vclass[u]][table[u] + x] = 0;
    }
    const uint32_t c = k.vclass[v], w = k.vwidth[v], a = k.valign[v], F = k.class_size[c];
    const uint32_t n_slot = (F >= w) ? (F - w) / a + 1 : 0;
    if (!n_slot) return false;
    uint32_t s0 = (start[c] / a) % n_slot;
    bool placed = false;
    bool may_skip = skip_pct && w <= 2;
    for (int pass = 0; pass < 2 && !placed; ++pass) {
      for (uint32_t t = 0; t < n_slot; ++t) {
        uint32_t base = ((s0 + t) % n_slot) * a;
        bool free_ = true;
        for (uint32_t x = 0; x < w; ++x) if (busy[c][base + x]) { free_ = false; break; }
        if (!free_) continue;
        if (pass == 0 && may_skip && r.below(100) < skip_pct) continue;
        table[v] = (uint16_t)base;
        placed = true;
        break;
      }
    }
    if (!placed) return false;
    for (uint32_t x = 0; x < w; ++x) busy[c][table[v] + x] = 1;
    active.emplace_back(k.hi[v], v);
    std::push_heap(active.begin(), active.end(), cmp);
  }
  return true;
}

void fill_row(const Kernel& k, const std::vector<uint16_t>& table, uint16_t* row) {
  const size_t O = k.occ_vreg.size();
  for (size_t o = 0; o < O; ++o) row[o] = table[k.occ_vreg[o]];
}

struct Damage {
  const Kernel& k; Rng& r;
  std::vector<std::vector<uint32_t>> occs;  // per vreg
  std::vector<uint32_t> used, multi, aligned, sure;  // candidate victims
  explicit Damage(const Kernel& kk, Rng& rr) : k(kk), r(rr), occs(kk.n_vreg()) {
    for (uint32_t o = 0; o < k.occ_vreg.size(); ++o) occs[k.occ_vreg[o]].push_back(o);
    for (uint32_t v = 0; v < k.n_vreg(); ++v) {
      if (occs[v].empty()) continue;
      used.push_back(v);
      if (occs[v].size() >= 2) multi.push_back(v);
      if (k.valign[v] > 1) aligned.push_back(v);
      if (k.sure_hi[v] > k.sure_lo[v]) sure.push_back(v);
    }
  }
  void set_all(uint16_t* row, uint32_t v, uint16_t p) { for (uint32_t o : occs[v]) row[o] = p; }
  // M1: one occurrence differs from the others
  bool m1(uint16_t* row, Mut& m) {
    if (multi.empty()) return false;
    uint32_t v = multi[r.below((uint32_t)multi.size())];
    uint32_t o = occs[v][r.below((uint32_t)occs[v].size())];
    uint32_t F = k.class_size[k.vclass[v]];
    uint16_t nv = (uint16_t)((row[o] + 1 + r.below(F - 1)) % F);
    row[o] = nv;
    m = {1, v, o, 1};
    return true;
  }
  // M2: base + 1 for an aligned value
  bool m2(uint16_t* row, Mut& m) {
    if (aligned.empty()) return false;
    uint32_t v = aligned[r.below((uint32_t)aligned.size())];
    set_all(row, v, (uint16_t)(row[occs[v][0]] + 1));
    m = {2, v, 0, 2};
    return true;
  }
  // M3: the last register of the tuple falls just outside the file
  bool m3(uint16_t* row, Mut& m) {
    if (used.empty()) return false;
    uint32_t v = used[r.below((uint32_t)used.size())];
    uint32_t F = k.class_size[k.vclass[v]];
    set_all(row, v, (uint16_t)(F - k.vwidth[v] + 1));
    m = {3, v, 0, 2};
    return true;
  }
  // M4: move v onto a register of some u that certainly coexists with it
  bool m4(uint16_t* row, Mut& m) {
    if (sure.size() < 2) return false;
    for (int attempt = 0; attempt < 64; ++attempt) {
      uint32_t v = sure[r.below((uint32_t)sure.size())];
      uint32_t at = k.sure_lo[v];
      // look for a partner among a random window of the candidates
      for (int t = 0; t < 64; ++t) {
        uint32_t u = sure[r.below((uint32_t)sure.size())];
        if (u == v || k.vclass[u] != k.vclass[v]) continue;
        if (!(k.sure_lo[u] <= at && at < k.sure_hi[u])) continue;
        uint32_t pu = row[occs[u][0]], w = k.vwidth[v], a = k.valign[v];
        uint32_t F = k.class_size[k.vclass[v]];
        uint32_t base = (pu / a) * a;
        if (base + w <= pu) continue;              // does not reach u (cannot happen when a == w)
        if (base + w > F) continue;
        if (base == row[occs[v][0]]) continue;
        set_all(row, v, (uint16_t)base);
        m = {4, v, u, 3};
        return true;
      }
    }
    return false;
  }
  // M5: a random aligned in-bounds base; may or may not stay valid
  bool m5(uint16_t* row, Mut& m) {
    if (used.empty()) return false;
    uint32_t v = used[r.below((uint32_t)used.size())];
    uint32_t F = k.class_size[k.vclass[v]], w = k.vwidth[v], a = k.valign[v];
    uint32_t n_slot = (F - w) / a + 1;
    // stay near the registers the row already uses, so that a fair share of
    // these reassignments land on an occupied register
    uint32_t top = 0;
    for (size_t o = 0; o < k.occ_vreg.size(); ++o) if (k.vclass[k.occ_vreg[o]] == k.vclass[v]) top = std::max<uint32_t>(top, row[o]);
    n_slot = std::min(n_slot, top / a + 2);
    if (n_slot < 2) return false;
    uint32_t cur = row[occs[v][0]], base;
    do base = r.below(n_slot) * a; while (base == cur);
    set_all(row, v, (uint16_t)base);
    m = {5, v, 0, 255};
    return true;
  }
};

}  // namespace

extern "C" {

struct vlgen_mut { uint32_t kind, vreg, other, expect; };

// kind: 1 straight line, 2 three-block loop, 3 GEMM-shaped, 4 attention-shaped
void* vlgen_make(int kind, uint64_t seed, uint32_t n_instr, uint32_t n_vreg) {
  switch (kind) {
    case 1: return make_straight(seed, n_instr);
    case 2: {
      uint32_t pro = n_instr * 3 / 20, epi = pro, body = n_instr - pro - epi;
      return make_loop3(seed, pro, body, epi, n_vreg, n_vreg / 20);
    }
    case 3: return make_gemm(seed, n_instr, n_vreg);
    case 4: return make_mha(seed, n_instr, n_vreg);
  }
  return nullptr;
}
void vlgen_free(void* h) { delete (Kernel*)h; }
void vlgen_sizes(void* h, uint32_t* out) {
  Kernel* k = (Kernel*)h;
  uint32_t ne = 0; for (auto& s : k->succ) ne += (uint32_t)s.size();
  out[0] = k->n_instr(); out[1] = k->n_vreg(); out[2] = (uint32_t)k->succ.size();
  out[3] = (uint32_t)k->occ_vreg.size(); out[4] = (uint32_t)k->class_size.size(); out[5] = ne;
}
void vlgen_copy(void* h, uint32_t* blk_start, uint32_t* succ_off, uint32_t* succ, uint32_t* occ_off,
                uint32_t* occ_vreg, uint8_t* occ_flags, uint8_t* vclass, uint8_t* vwidth, uint8_t* valign,
                uint16_t* class_size, uint32_t* range, uint32_t* sure) {
  Kernel* k = (Kernel*)h;
  std::copy(k->blk_start.begin(), k->blk_start.end(), blk_start);
  uint32_t e = 0;
  for (size_t b = 0; b < k->succ.size(); ++b) { succ_off[b] = e; for (uint32_t s : k->succ[b]) succ[e++] = s; }
  succ_off[k->succ.size()] = e;
  std::copy(k->occ_off.begin(), k->occ_off.end(), occ_off);
  std::copy(k->occ_vreg.begin(), k->occ_vreg.end(), occ_vreg);
  std::copy(k->occ_flags.begin(), k->occ_flags.end(), occ_flags);
  std::copy(k->vclass.begin(), k->vclass.end(), vclass);
  std::copy(k->vwidth.begin(), k->vwidth.end(), vwidth);
  std::copy(k->valign.begin(), k->valign.end(), valign);
  std::copy(k->class_size.begin(), k->class_size.end(), class_size);
  for (uint32_t v = 0; v < k->n_vreg(); ++v) {
    range[2 * v] = k->lo[v]; range[2 * v + 1] = k->hi[v];
    sure[2 * v] = k->sure_lo[v]; sure[2 * v + 1] = k->sure_hi[v];
  }
}

// Fills K rows.  mode 0: all rows from the plain first fit, no damage.
// mode 1: plain first fit; of n_mut damaged rows half get M5, half M1.
// mode 2: randomized first fit; damaged rows get one of M1..M4 in the paper's
//         error proportions (Section 4.5: most failures overwrite live values,
//         about a quarter break hardware rules, a few are malformed).
// mode 3: randomized first fit; damaged rows get 1..3 M4 conflicts.
// Returns 0, or -1 if no allocation was found (caller takes another seed).
int vlgen_candidates(void* h, uint64_t seed, uint32_t K, uint32_t n_mut, int mode, uint16_t* rows,
                     uint64_t ld, vlgen_mut* log) {
  Kernel* k = (Kernel*)h;
  Rng r(seed);
  std::vector<uint16_t> table;
  std::vector<uint8_t> damaged(K, 0);
  {  // choose which rows are damaged
    std::vector<uint32_t> idx(K);
    for (uint32_t i = 0; i < K; ++i) idx[i] = i;
    for (uint32_t i = 0; i < n_mut && i < K; ++i) {
      uint32_t j = i + r.below(K - i);
      std::swap(idx[i], idx[j]);
      damaged[idx[i]] = 1;
    }
  }
  Damage dmg(*k, r);
  uint32_t n_done = 0;
  for (uint32_t row = 0; row < K; ++row) {
    Rng rr(r.next());
    bool ok = false;
    if (mode <= 1) ok = first_fit(*k, rr, false, table);
    else {
      for (int t = 0; t < 8 && !ok; ++t) ok = first_fit(*k, rr, true, table);
      if (!ok) ok = first_fit(*k, rr, false, table);
    }
    if (!ok) return -1;
    uint16_t* out = rows + (size_t)row * ld;
    fill_row(*k, table, out);
    Mut m{0, 0, 0, 0};
    if (damaged[row]) {
      bool did = false;
      if (mode == 1) {
        did = (n_done % 2 == 0) ? dmg.m5(out, m) : dmg.m1(out, m);
      } else if (mode == 2) {
        uint32_t x = r.below(100);
        if (x < 70) did = dmg.m4(out, m);
        else if (x < 83) did = dmg.m2(out, m);
        else if (x < 95) did = dmg.m3(out, m);
        else did = dmg.m1(out, m);
        if (!did) did = dmg.m3(out, m);
      } else if (mode == 3) {
        uint32_t n = 1 + r.below(3);
        for (uint32_t t = 0; t < n; ++t) { Mut mm; if (dmg.m4(out, mm)) { if (!did) m = mm; did = true; } }
        if (!did) did = dmg.m3(out, m);
      }
      ++n_done;
      if (!did) m = {0, 0, 0, 0};
    }
    if (log) { log[row].kind = m.kind; log[row].vreg = m.vreg; log[row].other = m.other; log[row].expect = m.expect; }
  }
  return 0;
}

}  // extern "C"
