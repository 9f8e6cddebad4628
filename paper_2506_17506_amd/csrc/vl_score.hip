// Register-bank conflicts of candidates, a quality measure beside validity (Section 2:
// registers are organised in banks, four on NVIDIA GPUs; reading several values from one
// bank stalls the pipeline a cycle per extra value).  One lane per (candidate, instruction):
// for every bank the registers the instruction's distinct USE vregs read from it are counted
// in closed form from base and width, the worst bank gives the stall.
#include "vl_dev.h"

using namespace vl;

namespace {

// how many of the registers p .. p + w - 1 lie in bank b of n
__device__ inline uint32_t in_bank(uint32_t p, uint32_t w, uint32_t b, uint32_t n) {
  const uint32_t first = (b + n - p % n) % n;   // offset of the first register of the tuple in bank b
  return first < w ? (w - 1u - first) / n + 1u : 0u;
}

constexpr uint32_t kScoreInstr = 256;   // instructions per workgroup

__global__ __launch_bounds__(256) void k_bank_score(const DevMir *mir, const uint16_t *__restrict__ cand, uint32_t K, uint64_t ld,
                                                    uint32_t n_banks, uint32_t *__restrict__ out) {
  const DevMir VL_GLOBAL &m = *as_global(mir);
  const uint32_t k = blockIdx.y, i = blockIdx.x * kScoreInstr + threadIdx.x;
  if (blockIdx.x * kScoreInstr >= m.N) return;
  const uint16_t *row = cand + (uint64_t)k * ld;
  uint32_t stall = 0;
  if (i < m.N) {
    const uint32_t o0 = m.occ_off[i], o1 = m.occ_off[i + 1];
    uint32_t worst = 0;
    for (uint32_t b = 0; b < n_banks; ++b) {
      uint32_t n = 0;
      for (uint32_t o = o0; o < o1; ++o) {
        if (!(m.occ_flags[o] & VL_OCC_USE)) continue;
        const uint32_t v = m.occ_vreg[o];
        bool seen = false;   // an earlier USE operand with the same vreg
        for (uint32_t x = o0; x < o; ++x) seen |= (m.occ_flags[x] & VL_OCC_USE) && m.occ_vreg[x] == v;
        if (!seen) n += in_bank(row[o], attr_width(m.vattr[v]), b, n_banks);
      }
      worst = max(worst, n);
    }
    stall = worst > 1 ? worst - 1 : 0;
  }
  for (int d = 32; d >= 1; d >>= 1) stall += (uint32_t)__shfl_xor((int)stall, d, 64);
  if ((threadIdx.x & 63u) == 0 && stall) atomicAdd(&out[k], stall);
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
  k_bank_score<<<dim3((mir->h.N + kScoreInstr - 1) / kScoreInstr, K), 256, 0, stream>>>(mir->dev, cand, K, ld, n_banks, out);
  VL_HIP(hipGetLastError());
  return VL_OK;
}
