// Philox4x32-10 for device code (Salmon et al., SC'11): counter c[4], key k[2], ten
// rounds, key bumped by the Weyl constants before every round but the first.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace lgp {

// 64-bit draw for (key, vertex, hop, slot): counter = (vertex, 0, hop, slot); the draw
// is output word 0 (low half) | output word 1 (high half).  Vertex ids are < 2^31, so
// the counter's second word is always zero.
__device__ __forceinline__ uint64_t philox_draw64(uint32_t k0, uint32_t k1, uint32_t vertex, uint32_t hop,
                                                  uint32_t slot) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = vertex, c1 = 0u, c2 = hop, c3 = slot;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += W0; k1 += W1;
  }
  return uint64_t(c0) | (uint64_t(c1) << 32);
}

}  // namespace lgp
