// Program handles: validation of a kernel description and its copy to the device.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "vl_dev.h"

namespace vl {
static thread_local int32_t g_last_hip = 0;
int32_t hip_fail(hipError_t e) {
  g_last_hip = (int32_t)e;
  (void)hipGetLastError();
  return VL_E_HIP;
}
}  // namespace vl

extern "C" int32_t vl_last_hip_error(void) { return vl::g_last_hip; }

extern "C" const char *vl_strerror(int32_t code) {
  switch (code) {
    case VL_OK: return "ok";
    case VL_E_NULL: return "a required pointer is NULL";
    case VL_E_SHAPE: return "inconsistent sizes or offsets";
    case VL_E_RANGE: return "a value is outside its allowed range";
    case VL_E_LAYOUT: return "blocks are not contiguous, a block is empty, or a block has no earlier predecessor";
    case VL_E_NOT_STRICT: return "a value is live into the entry block";
    case VL_E_HIP: return "a HIP runtime call failed";
    case VL_E_ARG: return "handle does not belong to this call";
    case VL_E_LIMIT: return "more candidates than the entry point that allocates nothing has room for (VL_STATIC_MAX_K)";
  }
  return "unknown error code";
}

// mentions: occurrences that neither read nor write are allowed (programs made by vl_mir_create_lanes)
static int32_t validate(const vl_mir_desc *d, bool mentions) {
  if (!d->blk_start || !d->succ_off || !d->instr_occ_off || !d->class_size) return VL_E_NULL;
  if (d->n_edge && !d->succ) return VL_E_NULL;
  if (d->n_occ && (!d->occ_vreg || !d->occ_flags)) return VL_E_NULL;
  if (d->n_vreg && (!d->vreg_class || !d->vreg_width || !d->vreg_align)) return VL_E_NULL;
  if (d->n_instr == 0 || d->n_block == 0 || d->n_class == 0) return VL_E_SHAPE;
  if (d->n_class > vl::kMaxClass) return VL_E_RANGE;
  if (d->n_occ >= (1u << 24) || d->n_instr >= (1u << 28) || d->n_vreg > VL_MAX_VREG) return VL_E_RANGE;
  for (uint32_t c = 0; c < d->n_class; ++c)
    if (d->class_size[c] == 0 || d->class_size[c] > 512) return VL_E_RANGE;
  if (d->blk_start[0] != 0 || d->blk_start[d->n_block] != d->n_instr) return VL_E_LAYOUT;
  for (uint32_t b = 0; b < d->n_block; ++b)
    if (d->blk_start[b + 1] <= d->blk_start[b]) return VL_E_LAYOUT;
  if (d->succ_off[0] != 0 || d->succ_off[d->n_block] != d->n_edge) return VL_E_SHAPE;
  for (uint32_t b = 0; b < d->n_block; ++b)
    if (d->succ_off[b + 1] < d->succ_off[b]) return VL_E_SHAPE;
  for (uint32_t e = 0; e < d->n_edge; ++e)
    if (d->succ[e] >= d->n_block) return VL_E_RANGE;
  if (d->instr_occ_off[0] != 0 || d->instr_occ_off[d->n_instr] != d->n_occ) return VL_E_SHAPE;
  for (uint32_t i = 0; i < d->n_instr; ++i) {
    if (d->instr_occ_off[i + 1] < d->instr_occ_off[i]) return VL_E_SHAPE;
    if (d->instr_occ_off[i + 1] - d->instr_occ_off[i] > vl::kMaxOperands) return VL_E_RANGE;
  }
  for (uint32_t o = 0; o < d->n_occ; ++o) {
    if (d->occ_vreg[o] >= d->n_vreg) return VL_E_RANGE;
    const uint8_t f = d->occ_flags[o];
    if (((f & (VL_OCC_DEF | VL_OCC_USE)) == 0 && !mentions) || (f & ~(VL_OCC_DEF | VL_OCC_USE | VL_OCC_EARLY))) return VL_E_RANGE;
    if ((f & VL_OCC_EARLY) && !(f & VL_OCC_DEF)) return VL_E_RANGE;
  }
  for (uint32_t v = 0; v < d->n_vreg; ++v) {
    if (d->vreg_class[v] >= d->n_class) return VL_E_RANGE;
    if (d->vreg_width[v] == 0 || d->vreg_width[v] > 32) return VL_E_RANGE;
    if (d->vreg_align[v] == 0 || d->vreg_align[v] > 32) return VL_E_RANGE;
  }
  // every non-entry block needs a predecessor placed before it
  std::vector<uint8_t> has(d->n_block, 0);
  for (uint32_t b = 0; b < d->n_block; ++b)
    for (uint32_t e = d->succ_off[b]; e < d->succ_off[b + 1]; ++e)
      if (b < d->succ[e]) has[d->succ[e]] = 1;
  for (uint32_t b = 1; b < d->n_block; ++b)
    if (!has[b]) return VL_E_LAYOUT;
  return VL_OK;
}

namespace {
struct Bump {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t at = off;
    off += (bytes + 255) & ~(size_t)255;
    return at;
  }
};
}  // namespace

namespace {
// the maps of a program made by vl_mir_create_lanes (host arrays), or null
struct LaneMaps {
  const uint32_t *occ_src;
  const uint8_t *occ_add;
  const uint32_t *val_vreg;
  const uint8_t *val_lane;
  uint32_t src_occ, src_vreg;
};

int32_t create_impl(const vl_mir_desc *d, const LaneMaps *maps, vl_mir **out) {
  if (!d || !out) return VL_E_NULL;
  int32_t rc = validate(d, maps != nullptr);
  if (rc != VL_OK) return rc;
  const uint32_t N = d->n_instr, V = d->n_vreg, B = d->n_block, O = d->n_occ, E = d->n_edge;
  // derived index arrays (plain expansions of the CSR offsets) and packed attributes
  std::vector<uint32_t> occ_instr(O ? O : 1), instr_blk(N), vattr(V ? V : 1);
  for (uint32_t i = 0; i < N; ++i)
    for (uint32_t o = d->instr_occ_off[i]; o < d->instr_occ_off[i + 1]; ++o) occ_instr[o] = i;
  for (uint32_t b = 0; b < B; ++b)
    for (uint32_t i = d->blk_start[b]; i < d->blk_start[b + 1]; ++i) instr_blk[i] = b;
  std::vector<uint64_t> occ_rec(O ? O : 1);
  for (uint32_t o = 0; o < O; ++o)
    occ_rec[o] = (uint64_t)d->occ_vreg[o] | ((uint64_t)((occ_instr[o] << 2) | (d->occ_flags[o] & 3u)) << 32);
  std::vector<uint8_t> instr_keep(N, 0);
  for (uint32_t o = 0; o < O; ++o)
    if (d->occ_flags[o] & VL_OCC_EARLY) instr_keep[occ_instr[o]] = 1;

  // the device header's class tables come first: the packed attributes carry the class's mask word
  vl::DevMir hh;
  memset(&hh, 0, sizeof(hh));
  // mask words: classes smallest first, so that the 16 words every class may address from
  // its first one mostly fall on words of later classes
  std::vector<uint32_t> order(d->n_class);
  for (uint32_t c = 0; c < d->n_class; ++c) order[c] = c;
  std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return d->class_size[a] < d->class_size[b]; });
  uint32_t words = 0, reach = 0;
  for (uint32_t c : order) {
    hh.class_word[c] = (uint16_t)words;
    reach = std::max(reach, words + 16u);
    words += (d->class_size[c] + 31u) / 32u;
  }
  hh.occ_words = reach;
  for (uint32_t c = 0; c < d->n_class; ++c) {
    hh.class_size[c] = d->class_size[c];
    if (d->class_reserved)
      for (int w = 0; w < 16; ++w) {
        hh.reserved[c][w] = d->class_reserved[c * 16 + w];
        if (hh.reserved[c][w]) hh.has_reserved = 1;
      }
  }
  for (uint32_t v = 0; v < V; ++v)
    vattr[v] = vl::attr_pack(d->vreg_class[v], d->vreg_width[v], d->vreg_align[v]) | ((uint32_t)hh.class_word[d->vreg_class[v]] << 16);

  Bump bump;
  size_t o_blk = bump.take((B + 1) * 4), o_soff = bump.take((B + 1) * 4), o_succ = bump.take((size_t)(E ? E : 1) * 4);
  size_t o_ooff = bump.take((size_t)(N + 1) * 4), o_ov = bump.take((size_t)(O ? O : 1) * 4);
  size_t o_oi = bump.take((size_t)(O ? O : 1) * 4), o_ib = bump.take((size_t)N * 4);
  size_t o_va = bump.take((size_t)(V ? V : 1) * 4), o_of = bump.take((size_t)(O ? O : 1));
  size_t o_rec = bump.take((size_t)(O ? O : 1) * 8);
  size_t o_keep = bump.take((size_t)N);
  size_t o_src = 0, o_add = 0, o_vv = 0, o_vl = 0;
  if (maps) {
    o_src = bump.take((size_t)(O ? O : 1) * 4); o_add = bump.take((size_t)(O ? O : 1));
    o_vv = bump.take((size_t)(V ? V : 1) * 4); o_vl = bump.take((size_t)(V ? V : 1));
  }
  size_t o_dev = bump.take(sizeof(vl::DevMir));

  vl_mir *m = new (std::nothrow) vl_mir;
  if (!m) return VL_E_SHAPE;
  m->h = hh;
  m->arena = nullptr;
  m->magic = vl::kMirMagic;
  hipError_t e = hipGetDevice(&m->device);
  if (e == hipSuccess) e = hipMalloc(&m->arena, bump.off);
  if (e != hipSuccess) { delete m; return vl::hip_fail(e); }
  char *base = (char *)m->arena;
  // the arena is put together on the host and sent in one copy
  std::vector<char> image(bump.off, 0);
  auto up = [&](size_t off, const void *src, size_t bytes) {
    if (bytes) memcpy(image.data() + off, src, bytes);
  };
  up(o_blk, d->blk_start, (B + 1) * 4);
  up(o_soff, d->succ_off, (B + 1) * 4);
  up(o_succ, d->succ, (size_t)E * 4);
  up(o_ooff, d->instr_occ_off, (size_t)(N + 1) * 4);
  up(o_ov, d->occ_vreg, (size_t)O * 4);
  up(o_oi, occ_instr.data(), (size_t)O * 4);
  up(o_ib, instr_blk.data(), (size_t)N * 4);
  up(o_va, vattr.data(), (size_t)V * 4);
  up(o_of, d->occ_flags, (size_t)O);
  up(o_rec, occ_rec.data(), (size_t)O * 8);
  up(o_keep, instr_keep.data(), (size_t)N);
  if (maps) {
    up(o_src, maps->occ_src, (size_t)O * 4); up(o_add, maps->occ_add, (size_t)O);
    up(o_vv, maps->val_vreg, (size_t)V * 4); up(o_vl, maps->val_lane, (size_t)V);
  }

  vl::DevMir &h = m->h;
  h.N = N; h.V = V; h.B = B; h.O = O; h.C = d->n_class; h.E = E; h.W = (V + 31) / 32;
  h.blk_start = (const uint32_t VL_GLOBAL *)(base + o_blk);
  h.succ_off = (const uint32_t VL_GLOBAL *)(base + o_soff);
  h.succ = (const uint32_t VL_GLOBAL *)(base + o_succ);
  h.occ_off = (const uint32_t VL_GLOBAL *)(base + o_ooff);
  h.occ_vreg = (const uint32_t VL_GLOBAL *)(base + o_ov);
  h.occ_instr = (const uint32_t VL_GLOBAL *)(base + o_oi);
  h.instr_blk = (const uint32_t VL_GLOBAL *)(base + o_ib);
  h.vattr = (const uint32_t VL_GLOBAL *)(base + o_va);
  h.occ_flags = (const uint8_t VL_GLOBAL *)(base + o_of);
  h.occ_rec = (const uint64_t VL_GLOBAL *)(base + o_rec);
  h.instr_keep = (const uint8_t VL_GLOBAL *)(base + o_keep);
  if (maps) {
    h.occ_src = (const uint32_t VL_GLOBAL *)(base + o_src);
    h.val_vreg = (const uint32_t VL_GLOBAL *)(base + o_vv);
    m->lowered = true;
    m->src_occ = maps->src_occ; m->src_vreg = maps->src_vreg;
    m->occ_src = (const uint32_t *)(base + o_src); m->occ_add = (const uint8_t *)(base + o_add);
    m->val_vreg = (const uint32_t *)(base + o_vv); m->val_lane = (const uint8_t *)(base + o_vl);
  }
  m->dev = (vl::DevMir *)(base + o_dev);
  up(o_dev, &h, sizeof(h));
  e = hipMemcpy(base, image.data(), bump.off, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(m->arena);
    delete m;
    return vl::hip_fail(e);
  }
  *out = m;
  return VL_OK;
}
}  // namespace

extern "C" int32_t vl_mir_create(const vl_mir_desc *d, vl_mir **out) { return create_impl(d, nullptr, out); }

// Lane masks: the program is rewritten on the host so that every lane of a vreg that is
// accessed in part somewhere is a value of its own (one register wide), and everything
// else in the library runs on the rewritten program as it stands.  An occurrence of such a
// vreg becomes a mention of the whole vreg, which neither reads nor writes but carries the
// register (consistency and realizability stay per vreg and whole tuple), followed by one
// occurrence per lane it accesses, whose register is the vreg's plus the lane.  Values are
// numbered vreg by vreg, the whole vreg before its lanes.
extern "C" int32_t vl_mir_create_lanes(const vl_mir_desc *d, const uint32_t *occ_lanes, vl_mir **out) {
  if (!d || !out) return VL_E_NULL;
  int32_t rc = validate(d, false);
  if (rc != VL_OK) return rc;
  const uint32_t N = d->n_instr, V = d->n_vreg, O = d->n_occ;
  std::vector<uint8_t> split(V ? V : 1, 0);
  for (uint32_t o = 0; o < O && occ_lanes; ++o) {
    const uint32_t v = d->occ_vreg[o], w = d->vreg_width[v];
    const uint32_t full = w == 32 ? 0xFFFFFFFFu : ((1u << w) - 1u);
    if (occ_lanes[o] & ~full) return VL_E_RANGE;   // a lane the vreg does not have
    if (occ_lanes[o] != 0 && occ_lanes[o] != full) split[v] = 1;
  }
  std::vector<uint32_t> id(V + 1), val_vreg;
  std::vector<uint8_t> val_lane, vclass, vwidth, valign;
  for (uint32_t v = 0; v < V; ++v) {
    id[v] = (uint32_t)val_vreg.size();
    val_vreg.push_back(v); val_lane.push_back(0xFF);
    vclass.push_back(d->vreg_class[v]); vwidth.push_back(d->vreg_width[v]); valign.push_back(d->vreg_align[v]);
    if (split[v])
      for (uint32_t j = 0; j < d->vreg_width[v]; ++j) {
        val_vreg.push_back(v); val_lane.push_back((uint8_t)j);
        vclass.push_back(d->vreg_class[v]); vwidth.push_back(1); valign.push_back(1);
      }
  }
  std::vector<uint32_t> off(N + 1, 0), occ_v, occ_src;
  std::vector<uint8_t> occ_f, occ_add;
  for (uint32_t i = 0; i < N; ++i) {
    for (uint32_t o = d->instr_occ_off[i]; o < d->instr_occ_off[i + 1]; ++o) {
      const uint32_t v = d->occ_vreg[o], w = d->vreg_width[v];
      if (!split[v]) {
        occ_v.push_back(id[v]); occ_f.push_back(d->occ_flags[o]); occ_src.push_back(o); occ_add.push_back(0);
        continue;
      }
      occ_v.push_back(id[v]); occ_f.push_back(0); occ_src.push_back(o); occ_add.push_back(0);
      const uint32_t lanes = (occ_lanes && occ_lanes[o]) ? occ_lanes[o] : (w == 32 ? 0xFFFFFFFFu : ((1u << w) - 1u));
      for (uint32_t j = 0; j < w; ++j)
        if ((lanes >> j) & 1u) {
          occ_v.push_back(id[v] + 1 + j); occ_f.push_back(d->occ_flags[o]); occ_src.push_back(o); occ_add.push_back((uint8_t)j);
        }
    }
    off[i + 1] = (uint32_t)occ_v.size();
    if (off[i + 1] - off[i] > vl::kMaxOperands) return VL_E_RANGE;   // too many operands once the lanes are spelt out
  }
  if (val_vreg.size() > VL_MAX_VREG || occ_v.size() >= (1u << 24)) return VL_E_RANGE;
  vl_mir_desc low = *d;
  low.n_vreg = (uint32_t)val_vreg.size();
  low.n_occ = (uint32_t)occ_v.size();
  low.instr_occ_off = off.data();
  low.occ_vreg = occ_v.data(); low.occ_flags = occ_f.data();
  low.vreg_class = vclass.data(); low.vreg_width = vwidth.data(); low.vreg_align = valign.data();
  const LaneMaps maps = {occ_src.data(), occ_add.data(), val_vreg.data(), val_lane.data(), O, V};
  return create_impl(&low, &maps, out);
}

extern "C" int32_t vl_mir_lanes_get(const vl_mir *m, vl_lanes_view *v) {
  if (!m || !v) return VL_E_NULL;
  if (m->magic != vl::kMirMagic || !m->lowered) return VL_E_ARG;
  v->n_occ = m->src_occ; v->n_vreg = m->src_vreg; v->n_occ_low = m->h.O; v->n_vreg_low = m->h.V;
  v->occ_src = m->occ_src; v->occ_add = m->occ_add; v->val_vreg = m->val_vreg; v->val_lane = m->val_lane;
  return VL_OK;
}

namespace {
__global__ __launch_bounds__(256) void k_lanes_expand(const uint16_t *__restrict__ cand, uint64_t ld, uint16_t *__restrict__ low,
                                                      uint64_t ld_low, const uint32_t *__restrict__ occ_src,
                                                      const uint8_t *__restrict__ occ_add, uint32_t n_low) {
  const uint32_t o = blockIdx.x * blockDim.x + threadIdx.x, k = blockIdx.y;
  if (o < n_low) low[(uint64_t)k * ld_low + o] = (uint16_t)(cand[(uint64_t)k * ld + occ_src[o]] + occ_add[o]);
}
}  // namespace

extern "C" int32_t vl_lanes_expand(const vl_mir *m, const uint16_t *cand, uint32_t K, uint64_t ld, uint16_t *cand_low,
                                   uint64_t ld_low, vl_stream stream) {
  if (!m || !cand || !cand_low) return VL_E_NULL;
  if (m->magic != vl::kMirMagic || !m->lowered) return VL_E_ARG;
  if (K == 0 || K > 65535 || ld < m->src_occ || ld_low < m->h.O) return VL_E_SHAPE;
  if (m->h.O == 0) return VL_OK;
  k_lanes_expand<<<dim3((m->h.O + 255) / 256, K), 256, 0, (hipStream_t)stream>>>(cand, ld, cand_low, ld_low, m->occ_src, m->occ_add,
                                                                                   m->h.O);
  VL_HIP(hipGetLastError());
  return VL_OK;
}

extern "C" void vl_mir_destroy(vl_mir *m) {
  if (!m || m->magic != vl::kMirMagic) return;
  m->magic = 0;
  if (m->arena) (void)hipFree(m->arena);
  if (m->edge_block && m->edge_block->refs.fetch_sub(1) == 1) {
    (void)hipFree(m->edge_block->mem);
    delete m->edge_block;
  }
  delete m;
}
