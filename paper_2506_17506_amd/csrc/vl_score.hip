// Register-bank conflicts of candidates, a quality measure beside validity (Section 2:
// registers are organised in banks, four on NVIDIA GPUs; reading several values from one
// bank stalls the pipeline a cycle per extra value).  A workgroup takes 256 instructions and
// a slab of candidates.  What does not depend on the candidate is found once: for every
// operand of these instructions, the width of its vreg if the operand is the first USE of
// that vreg in its instruction, else 0 (a byte per operand in LDS).  Then one lane per
// instruction loops over the slab: the lanes of a wavefront, being neighbouring instructions,
// read neighbouring entries of a candidate row.  For every bank the registers read from it
// are counted in closed form from base and width; the worst bank gives the stall.
#include "vl_dev.h"

using namespace vl;

namespace {

// how many of the registers p .. p + w - 1 lie in bank b of n
__device__ inline uint32_t in_bank(uint32_t p, uint32_t w, uint32_t b, uint32_t n) {
  const uint32_t first = (b + n - p % n) % n;   // offset of the first register of the tuple in bank b
  return first < w ? (w - 1u - first) / n + 1u : 0u;
}

constexpr uint32_t kScoreInstr = 256;   // instructions per workgroup
constexpr uint32_t kScoreCands = 8;     // candidates per workgroup

__global__ __launch_bounds__(256) void k_bank_score(const DevMir *mir, const uint16_t *__restrict__ cand, uint32_t K, uint64_t ld,
                                                    uint32_t n_banks, uint32_t *__restrict__ out) {
  const DevMir VL_GLOBAL &m = *as_global(mir);
  const uint32_t i_lo = blockIdx.x * kScoreInstr;
  if (i_lo >= m.N) return;
  __shared__ uint32_t sums[kScoreCands];
  __shared__ uint8_t read_width[kScoreInstr * kMaxOperands];
  const uint32_t i_hi = min(m.N, i_lo + kScoreInstr), o_lo = m.occ_off[i_lo], o_hi = m.occ_off[i_hi];
  const uint32_t k0 = blockIdx.y * kScoreCands, kn = min(kScoreCands, K - k0);
  if (threadIdx.x < kScoreCands) sums[threadIdx.x] = 0;
  for (uint32_t o = o_lo + threadIdx.x; o < o_hi; o += blockDim.x) {
    uint32_t w = 0;
    if (m.occ_flags[o] & VL_OCC_USE) {
      const uint32_t v = m.occ_vreg[o];
      bool seen = false;   // an earlier USE operand of the instruction with the same vreg
      for (uint32_t x = m.occ_off[m.occ_instr[o]]; x < o; ++x) seen |= (m.occ_flags[x] & VL_OCC_USE) && m.occ_vreg[x] == v;
      if (!seen) w = attr_width(m.vattr[v]);
    }
    read_width[o - o_lo] = (uint8_t)w;
  }
  __syncthreads();
  const uint32_t i = i_lo + threadIdx.x;
  const uint32_t o0 = i < i_hi ? m.occ_off[i] : 0u, o1 = i < i_hi ? m.occ_off[i + 1] : 0u;
  for (uint32_t c = 0; c < kn; ++c) {
    const uint16_t VL_GLOBAL *row = as_global(cand) + (uint64_t)(k0 + c) * ld;
    uint32_t worst = 0;
    if (n_banks == 4) {
      // the counts of the four banks are four 16-bit fields of one word: a tuple of width w
      // at base p adds w / 4 to every bank and one more to the w % 4 banks from p % 4 on (a
      // rotation of the field pattern); at most 64 x 9 per bank
      uint64_t counts = 0;
      for (uint32_t o = o0; o < o1; ++o) {
        const uint32_t w = read_width[o - o_lo];
        if (!w) continue;
        const uint32_t p = row[o], rest = w & 3u, sh = (p & 3u) * 16u;
        const uint64_t ones = rest == 0 ? 0ull : rest == 1 ? 0x1ull : rest == 2 ? 0x10001ull : 0x100010001ull;
        counts += (uint64_t)(w >> 2) * 0x0001000100010001ull + ((ones << sh) | (sh ? ones >> (64u - sh) : 0ull));
      }
      const uint32_t lo = (uint32_t)counts, hi = (uint32_t)(counts >> 32);
      worst = max(max(lo & 0xFFFFu, lo >> 16), max(hi & 0xFFFFu, hi >> 16));
    } else {
      for (uint32_t b = 0; b < n_banks; ++b) {
        uint32_t n = 0;
        for (uint32_t o = o0; o < o1; ++o) {
          const uint32_t w = read_width[o - o_lo];
          if (w) n += in_bank(row[o], w, b, n_banks);
        }
        worst = max(worst, n);
      }
    }
    uint32_t stall = worst > 1 ? worst - 1 : 0;
    for (int d = 32; d >= 1; d >>= 1) stall += (uint32_t)__shfl_xor((int)stall, d, 64);
    if ((threadIdx.x & 63u) == 0 && stall) atomicAdd(&sums[c], stall);
  }
  __syncthreads();
  if (threadIdx.x < kn && sums[threadIdx.x]) atomicAdd(&out[k0 + threadIdx.x], sums[threadIdx.x]);
}

__global__ void k_score_clear(uint32_t *out, uint32_t K) {
  const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k < K) out[k] = 0;
}

}  // namespace

extern "C" int32_t vl_bank_conflicts(const vl_mir *mir, const uint16_t *cand, uint32_t K, uint64_t ld, uint32_t n_banks,
                                     uint32_t *out, vl_stream stream_) {
  if (!mir || !cand || !out) return VL_E_NULL;
  if (mir->magic != kMirMagic || mir->lowered) return VL_E_ARG;
  if (K == 0 || K > 65535 || ld < mir->h.O) return VL_E_SHAPE;
  if (n_banks == 0 || n_banks > 64) return VL_E_RANGE;
  hipStream_t stream = (hipStream_t)stream_;
  k_score_clear<<<(K + 255) / 256, 256, 0, stream>>>(out, K);
  k_bank_score<<<dim3((mir->h.N + kScoreInstr - 1) / kScoreInstr, (K + kScoreCands - 1) / kScoreCands), 256, 0, stream>>>(mir->dev, cand, K, ld, n_banks, out);
  VL_HIP(hipGetLastError());
  return VL_OK;
}
