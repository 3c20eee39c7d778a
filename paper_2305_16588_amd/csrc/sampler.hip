// Neighbour sampler (Sec. 2.2 step 2; Sec. 5 "neighbor sampler") for gfx950.
//
// A group of P = next_pow2(fanout) lanes owns one frontier vertex; lane i is sample
// slot i.  One load of the HBM row table gives the row's offset and degree and says
// whether its column ids sit in the HBM topology cache or in the CPU-resident CSR (read
// in place over PCIe), so an uncached vertex costs one PCIe round trip, not two.  All slots draw their
// Philox number at once; Floyd's sequential "already taken?" test becomes fanout-1
// group broadcasts.  The kernel is bound by dependent loads and by the bitmap atomics, not by
// issue slots, so the grid is capped at four workgroups per CU (see launch_one).
#include "common.hpp"
#include "philox_dev.hpp"

namespace lgp {
namespace {

template <typename IdxT, int P>
__global__ __launch_bounds__(256) void sample_hop_kernel(
    const uint64_t* __restrict__ row_tab, const IdxT* __restrict__ h_indptr, const int32_t* __restrict__ h_indices,
    const int32_t* __restrict__ t_indices, int64_t num_vertices,
    const int32_t* __restrict__ frontier, int32_t* __restrict__ n_frontier, int64_t cap, int32_t f, int32_t hop,
    uint32_t k0, uint32_t k1, int32_t* __restrict__ nbr, int32_t* __restrict__ cnt, uint32_t* __restrict__ mark_bits,
    uint32_t* __restrict__ self_bits, uint32_t* __restrict__ topo_hot, uint32_t* __restrict__ d_err, int shift) {
  constexpr int G = 256 / P;                      // vertices per workgroup pass
  // self_bits != nullptr: this is the first hop; the frontier is the caller's seed list of `cap`
  // ids, whose size is published here and whose members are marked in the gather set.
  if (self_bits && blockIdx.x == 0 && threadIdx.x == 0) *n_frontier = int32_t(cap);
  int64_t n = self_bits ? cap : int64_t(*n_frontier);
  if (n > cap) n = cap;                           // never trust a count beyond the buffer
  const int i = threadIdx.x % P;                  // sample slot
  const int gidx = threadIdx.x / P;
  // Three loads depend on one another (frontier id -> row-table entry -> column id); many waves in
  // flight hide them.  (Loading the id two passes ahead and the row-table entry one pass ahead was
  // measured too: the same time to within 1 % on every workload, so the loop stays plain.)
  const int64_t stride = int64_t(gridDim.x) * G;
  const uint64_t nv = uint64_t(num_vertices);
  for (int64_t g = int64_t(blockIdx.x) * G + gidx; g - gidx < n; g += stride) {
    const int32_t v = g < n ? frontier[g] : 0;
    const uint64_t e = (g < n && uint32_t(v) < nv) ? row_tab[v] : 0;
    const bool active = g < n;
    bool bad = active && uint32_t(v) >= nv;
    int64_t s = 0, d64 = 0;
    const int32_t* colbase = h_indices;
    if (active && !bad) {
      const uint32_t d24 = uint32_t(e) & kRowDegOverflow;
      if (d24 != kRowDegOverflow) {
        s = int64_t((e >> kRowStartShift) & kRowStartMask);
        d64 = d24;
        if (e & kRowCachedBit) colbase = t_indices;
      } else {                                     // degree does not fit the entry: CPU-resident CSR
        s = int64_t(h_indptr[v]);
        d64 = int64_t(h_indptr[int64_t(v) + 1]) - s;
      }
      if (d64 < 0 || d64 > 0x7fffffff) { bad = true; d64 = 0; }
    }
    if (bad) {
      if (i == 0) atomicOr(d_err, ERR_BAD_ID);
      d64 = 0;
    }
    const int32_t d = int32_t(d64);
    const bool big = active && d > f;
    int32_t p = i;                                 // position inside the row
    if (__any(big)) {
      int32_t t = -1, j = 0;
      if (big && i < f) {
        j = d - f + i;
        t = int32_t(__umul64hi(philox_draw64(k0, k1, uint32_t(v), uint32_t(hop), uint32_t(i)), uint64_t(j) + 1));
      }
      int32_t pc = t;
      bool moved = false;
      for (int k = 0; k + 1 < f; ++k) {            // slot k is final once slots < k are
        const int32_t pk = __shfl(pc, k, P);
        if (big && i > k && !moved && t == pk) { pc = j; moved = true; }
      }
      if (big) p = pc;
    }
    if (active && i < f) {
      const bool valid = big || i < d;
      int32_t u = -1;
      if (valid) {
        u = colbase[s + p];
        if (uint32_t(u) >= uint64_t(num_vertices)) {
          atomicOr(d_err, ERR_BAD_ID);
          u = -1;
        } else {
          const uint64_t b = uint64_t(uint32_t(u)) << shift;
          atomicOr(&mark_bits[b >> 5], 1u << (uint32_t(b) & 31u));
        }
      }
      if (nbr) nbr[g * f + i] = u;
    }
    if (active && i == 0) {
      if (self_bits && !bad) {
        const uint64_t b = uint64_t(uint32_t(v)) << shift;
        atomicOr(&self_bits[b >> 5], 1u << (uint32_t(b) & 31u));
      }
      const int32_t c = d < f ? d : f;
      if (cnt) cnt[g] = c;
      if (topo_hot && c > 0) atomicAdd(&topo_hot[v], uint32_t(c));
    }
  }
}

__global__ void accumulate_sizes_kernel(const int32_t* __restrict__ n, int32_t count,
                                        unsigned long long* __restrict__ acc) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    unsigned long long sum = 0;
    for (int32_t h = 0; h < count; ++h) sum += (unsigned long long)(n[h]);
    acc[0] += sum;                                // one writer, stream-ordered
  }
}

template <typename IdxT, int P>
void launch_one(const DeviceInfo& di, const TopoView& tv, const int32_t* frontier, int32_t* n_frontier,
                int64_t cap, int32_t f, int32_t hop, uint64_t seed, int32_t* nbr, int32_t* cnt, uint32_t* mark_bits,
                uint32_t* self_bits, uint32_t* topo_hot, uint32_t* d_err, hipStream_t s) {
  constexpr int G = 256 / P;
  int64_t blocks = (cap + G - 1) / G;
  // 4 workgroups x 4 waves = 16 waves per CU.  The kernel is bound by memory-side atomics and
  // dependent loads, not by issue slots: 16 waves per CU are as fast as 32 when it runs alone
  // (0.133 -> 0.128 ms per batch at 2.4 M vertices, 0.1025 -> 0.100 ms at 111 M) and disturb a
  // PCIe-bound gather running beside it less (pipelined step 2.50 -> 2.43 ms).
  const int64_t full = int64_t(di.num_cus) * 4;
  if (blocks > full) blocks = full;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL((sample_hop_kernel<IdxT, P>), dim3(unsigned(blocks)), dim3(256), 0, s,
                     tv.row_tab, static_cast<const IdxT*>(tv.h_indptr), tv.h_indices, tv.t_indices,
                     tv.num_vertices, frontier, n_frontier, cap, f, hop, uint32_t(seed), uint32_t(seed >> 32), nbr,
                     cnt, mark_bits, self_bits, topo_hot, d_err, di.spread_shift);
}

template <typename IdxT>
void dispatch_p(int P, const DeviceInfo& di, const TopoView& tv, const int32_t* frontier, int32_t* n_frontier,
                int64_t cap, int32_t f, int32_t hop, uint64_t seed, int32_t* nbr, int32_t* cnt, uint32_t* mark_bits,
                uint32_t* self_bits, uint32_t* topo_hot, uint32_t* d_err, hipStream_t s) {
#define LGP_CASE(PP)                                                                                            \
  case PP:                                                                                                      \
    launch_one<IdxT, PP>(di, tv, frontier, n_frontier, cap, f, hop, seed, nbr, cnt, mark_bits, self_bits, topo_hot, \
                         d_err, s);                                                                              \
    break;
  switch (P) {
    LGP_CASE(1) LGP_CASE(2) LGP_CASE(4) LGP_CASE(8) LGP_CASE(16) LGP_CASE(32) LGP_CASE(64)
  }
#undef LGP_CASE
}

}  // namespace

void launch_sample_hop(const DeviceInfo& di, const TopoView& tv, const int32_t* frontier, int32_t* n_frontier,
                       int64_t cap, int32_t fanout, int32_t hop, uint64_t rng_seed, int32_t* nbr, int32_t* cnt,
                       uint32_t* mark_bits, uint32_t* self_bits, uint32_t* topo_hot, uint32_t* d_err, hipStream_t s) {
  int P = 1;
  while (P < fanout) P <<= 1;
  if (tv.indptr_bytes == 8)
    dispatch_p<int64_t>(P, di, tv, frontier, n_frontier, cap, fanout, hop, rng_seed, nbr, cnt, mark_bits, self_bits,
                        topo_hot, d_err, s);
  else
    dispatch_p<int32_t>(P, di, tv, frontier, n_frontier, cap, fanout, hop, rng_seed, nbr, cnt, mark_bits, self_bits,
                        topo_hot, d_err, s);
}

void launch_accumulate_sizes(const int32_t* n, int32_t count, unsigned long long* acc, hipStream_t s) {
  hipLaunchKernelGGL(accumulate_sizes_kernel, dim3(1), dim3(64), 0, s, n, count, acc);
}

}  // namespace lgp
