// Cache candidate selection and fill-up (Sec. 4.2.2 steps S2-S3).  With one GPU per
// clique Algorithm 1 reduces to ranking the vertices by descending hotness; the size
// rules are Eq. 3 (topology) and Eq. 6 (features), evaluated with an inclusive scan
// along the ranking and a binary search for the budget, as in Sec. 4.3.3.  This is
// one-off set-up work: the sort and the scan are rocPRIM device primitives, the rest
// are small kernels.
#include "common.hpp"

#include <cstring>

#include <rocprim/rocprim.hpp>

#include "philox_dev.hpp"

namespace lgp {
namespace {

struct TopoCost {
  const int32_t* deg;
  const int32_t* order;
  __host__ __device__ uint64_t operator()(int64_t r) const { return uint64_t(deg[order[r]]) * 4u + 8u; }
};

struct HotAlong {
  const uint32_t* hot;
  const int32_t* order;
  __host__ __device__ uint64_t operator()(int64_t r) const { return uint64_t(hot[order[r]]); }
};

struct U128 {
  uint64_t hi, lo;
};
__device__ __forceinline__ U128 mul64(uint64_t a, uint64_t b) { return U128{__umul64hi(a, b), a * b}; }
__device__ __forceinline__ U128 add128(U128 a, U128 b) {
  const uint64_t lo = a.lo + b.lo;
  return U128{a.hi + b.hi + (lo < a.lo ? 1u : 0u), lo};
}
__device__ __forceinline__ bool less128(U128 a, U128 b) { return a.hi < b.hi || (a.hi == b.hi && a.lo < b.lo); }

// Cost model of Sec. 4.3.2 for every candidate alpha at once (Sec. 4.3.3): thread i owns plan i.
__global__ __launch_bounds__(1024) void alpha_search_kernel(
    const uint64_t* __restrict__ cost_scan, const uint64_t* __restrict__ hot_t_scan,
    const uint64_t* __restrict__ hot_f_scan, int64_t num_vertices, uint64_t row_bytes,
    const uint64_t* __restrict__ m_topo, uint64_t total_budget, uint64_t n_tsum, uint64_t per_row, int32_t n_alpha,
    lgp_plan_point* __restrict__ points, int32_t* __restrict__ best) {
  __shared__ uint64_t key_hi[1024], key_lo[1024];
  const int i = threadIdx.x;
  const uint64_t all_t = hot_t_scan[num_vertices - 1], all_f = hot_f_scan[num_vertices - 1];
  if (i < n_alpha) {
    const uint64_t mt = m_topo[i], mf = total_budget - mt;
    int64_t lo = 0, hi = num_vertices;           // Eq. 3: rows of Q_T whose running cost stays within m_T
    while (lo < hi) {
      const int64_t mid = lo + (hi - lo) / 2;
      if (cost_scan[mid] <= mt) lo = mid + 1;
      else hi = mid;
    }
    const int64_t n_t = lo;
    uint64_t rows_f = mf / row_bytes;             // Eq. 6
    const int64_t n_f = rows_f < uint64_t(num_vertices) ? int64_t(rows_f) : num_vertices;
    const uint64_t unc_t = all_t - (n_t ? hot_t_scan[n_t - 1] : 0);   // Eq. 4 numerator, complemented
    const uint64_t unc_f = all_f - (n_f ? hot_f_scan[n_f - 1] : 0);   // Eq. 7
    points[i].m_topo = mt;
    points[i].m_feat = mf;
    points[i].n_topo = n_t;
    points[i].n_feat = n_f;
    points[i].uncached_topo_hot = unc_t;
    points[i].uncached_feat_hot = unc_f;
    // N_total * all_t = n_tsum * unc_t + (per_row * unc_f) * all_t      (Eq. 2, 5, 8)
    U128 key = mul64(per_row * unc_f, all_t ? all_t : 1);
    if (all_t) key = add128(key, mul64(n_tsum, unc_t));
    key_hi[i] = key.hi;
    key_lo[i] = key.lo;
  }
  __syncthreads();
  if (i == 0) {
    int b = 0;
    for (int k = 1; k < n_alpha; ++k)
      if (less128(U128{key_hi[k], key_lo[k]}, U128{key_hi[b], key_lo[b]})) b = k;
    *best = b;
  }
}

__global__ void shuffle_keys_kernel(uint64_t* __restrict__ keys, int64_t n, uint32_t k0, uint32_t k1, uint32_t epoch) {
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += int64_t(gridDim.x) * blockDim.x)
    keys[i] = philox_draw64(k0, k1, uint32_t(i), epoch, 0u);
}

// Algorithm 1 step 1 + the arg-max of step 3: one thread per vertex walks its column.
__global__ void colsum_argmax_kernel(const uint32_t* __restrict__ hot, int32_t k_g, int64_t num_vertices,
                                     uint64_t* __restrict__ acc, int32_t* __restrict__ owner) {
  for (int64_t v = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; v < num_vertices;
       v += int64_t(gridDim.x) * blockDim.x) {
    uint64_t sum = 0;
    uint32_t best = 0;
    int32_t arg = 0;
    for (int32_t g = 0; g < k_g; ++g) {
      const uint32_t h = hot[int64_t(g) * num_vertices + v];
      sum += h;
      if (h > best) { best = h; arg = g; }
    }
    acc[v] = sum;
    owner[v] = arg;
  }
}

// key[r] = owner of the r-th ranked vertex; also counts queue lengths (LDS histogram per workgroup).
__global__ __launch_bounds__(256) void owner_along_kernel(const int32_t* __restrict__ owner,
                                                          const int32_t* __restrict__ order, int64_t num_vertices,
                                                          uint32_t* __restrict__ key,
                                                          unsigned long long* __restrict__ counts, int32_t k_g) {
  __shared__ unsigned int hist[64];
  if (threadIdx.x < 64) hist[threadIdx.x] = 0;
  __syncthreads();
  for (int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; r < num_vertices;
       r += int64_t(gridDim.x) * blockDim.x) {
    const int32_t g = owner[order[r]];
    key[r] = uint32_t(g);
    atomicAdd(&hist[g], 1u);
  }
  __syncthreads();
  if (int(threadIdx.x) < k_g && hist[threadIdx.x]) atomicAdd(&counts[threadIdx.x], (unsigned long long)hist[threadIdx.x]);
}

template <typename IdxT>
__global__ void degrees_kernel(const IdxT* __restrict__ indptr, int64_t num_vertices, int32_t* __restrict__ deg) {
  for (int64_t v = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; v < num_vertices;
       v += int64_t(gridDim.x) * blockDim.x)
    deg[v] = int32_t(indptr[v + 1] - indptr[v]);
}

__global__ void prefix_within_budget_kernel(const uint64_t* __restrict__ scan, int64_t n, uint64_t budget,
                                            uint64_t* __restrict__ result) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  int64_t lo = 0, hi = n;                       // first index with scan[idx] > budget
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo) / 2;
    if (scan[mid] <= budget) lo = mid + 1;
    else hi = mid;
  }
  result[0] = uint64_t(lo);
  result[1] = lo > 0 ? scan[lo - 1] : 0;
}

__global__ void topo_offsets_kernel(const uint64_t* __restrict__ cost_scan, int64_t n_topo,
                                    int64_t* __restrict__ t_indptr) {
  for (int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; r <= n_topo;
       r += int64_t(gridDim.x) * blockDim.x)
    t_indptr[r] = r == 0 ? 0 : int64_t((cost_scan[r - 1] - 8u * uint64_t(r)) / 4u);   // undo Eq. 3's +8 per row
}

// 16 lanes per cached row: rows average a few dozen ids, hubs just take more passes.
template <typename IdxT>
__global__ __launch_bounds__(256) void fill_topo_kernel(const IdxT* __restrict__ h_indptr,
                                                        const int32_t* __restrict__ h_indices,
                                                        const int32_t* __restrict__ order, int64_t n_topo,
                                                        const int64_t* __restrict__ t_indptr,
                                                        int32_t* __restrict__ t_indices) {
  const int sub = threadIdx.x & 15;
  for (int64_t r = (int64_t(blockIdx.x) * 256 + threadIdx.x) >> 4; r < n_topo; r += (int64_t(gridDim.x) * 256) >> 4) {
    const int32_t v = order[r];
    const int64_t s = int64_t(h_indptr[v]);
    const int64_t d = int64_t(h_indptr[int64_t(v) + 1]) - s;
    const int64_t dst = t_indptr[r];
    for (int64_t k = sub; k < d; k += 16) t_indices[dst + k] = __builtin_nontemporal_load(h_indices + s + k);
  }
}

template <typename IdxT>
__global__ void init_row_table_kernel(const IdxT* __restrict__ indptr, int64_t num_vertices,
                                      uint64_t* __restrict__ row_tab) {
  for (int64_t v = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; v < num_vertices;
       v += int64_t(gridDim.x) * blockDim.x) {
    const uint64_t s = uint64_t(indptr[v]);
    const uint64_t d = uint64_t(indptr[v + 1]) - s;
    const uint64_t d24 = d < kRowDegOverflow ? d : kRowDegOverflow;
    row_tab[v] = ((s & kRowStartMask) << kRowStartShift) | d24;
  }
}

__global__ void set_cached_rows_kernel(const int32_t* __restrict__ order, int64_t n_topo,
                                       const int64_t* __restrict__ t_indptr, uint64_t* __restrict__ row_tab) {
  for (int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; r < n_topo; r += int64_t(gridDim.x) * blockDim.x) {
    const uint64_t s = uint64_t(t_indptr[r]);
    const uint64_t d = uint64_t(t_indptr[r + 1]) - s;
    if (d < kRowDegOverflow) row_tab[order[r]] = kRowCachedBit | ((s & kRowStartMask) << kRowStartShift) | d;
  }
}

__global__ void fill_i32_kernel(int32_t* __restrict__ p, int64_t n, int32_t value) {
  for (int64_t k = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; k < n; k += int64_t(gridDim.x) * blockDim.x)
    p[k] = value;
}

__global__ void iota_i32_kernel(int32_t* __restrict__ p, int64_t n) {
  for (int64_t k = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; k < n; k += int64_t(gridDim.x) * blockDim.x)
    p[k] = int32_t(k);
}

__global__ void scatter_rank_kernel(const int32_t* __restrict__ order, int64_t n, int32_t* __restrict__ remap) {
  for (int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; r < n; r += int64_t(gridDim.x) * blockDim.x)
    remap[order[r]] = int32_t(r);
}

inline unsigned grid_for(const DeviceInfo& di, int64_t n, int per_block = 256) {
  int64_t blocks = (n + per_block - 1) / per_block;
  const int64_t full = int64_t(di.num_cus) * 8;
  if (blocks > full) blocks = full;
  if (blocks < 1) blocks = 1;
  return unsigned(blocks);
}

}  // namespace

hipError_t rank_by_hotness(const uint32_t* hot, int64_t num_vertices, int32_t* order, hipStream_t s) {
  uint32_t* keys_out = nullptr;
  void* temp = nullptr;
  size_t temp_bytes = 0;
  hipError_t e = hipMalloc(&keys_out, sizeof(uint32_t) * size_t(num_vertices));
  if (e != hipSuccess) return e;
  rocprim::counting_iterator<int32_t> ids(0);
  // Stable descending radix sort: equal hotness keeps ascending id order.
  e = rocprim::radix_sort_pairs_desc(nullptr, temp_bytes, hot, keys_out, ids, order, size_t(num_vertices), 0, 32, s);
  if (e == hipSuccess) e = hipMalloc(&temp, temp_bytes ? temp_bytes : 16);
  if (e == hipSuccess)
    e = rocprim::radix_sort_pairs_desc(temp, temp_bytes, hot, keys_out, ids, order, size_t(num_vertices), 0, 32, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (temp) (void)hipFree(temp);
  (void)hipFree(keys_out);
  return e;
}

void launch_degrees(const DeviceInfo& di, const void* h_indptr, int32_t indptr_bytes, int64_t num_vertices,
                    int32_t* deg, hipStream_t s) {
  if (indptr_bytes == 8)
    hipLaunchKernelGGL(degrees_kernel<int64_t>, dim3(grid_for(di, num_vertices)), dim3(256), 0, s,
                       static_cast<const int64_t*>(h_indptr), num_vertices, deg);
  else
    hipLaunchKernelGGL(degrees_kernel<int32_t>, dim3(grid_for(di, num_vertices)), dim3(256), 0, s,
                       static_cast<const int32_t*>(h_indptr), num_vertices, deg);
}

hipError_t scan_topo_cost(const int32_t* deg, const int32_t* order, int64_t num_vertices, uint64_t* cost_scan,
                          hipStream_t s) {
  auto in = rocprim::make_transform_iterator(rocprim::counting_iterator<int64_t>(0), TopoCost{deg, order});
  void* temp = nullptr;
  size_t temp_bytes = 0;
  hipError_t e = rocprim::inclusive_scan(nullptr, temp_bytes, in, cost_scan, size_t(num_vertices),
                                         rocprim::plus<uint64_t>(), s);
  if (e == hipSuccess) e = hipMalloc(&temp, temp_bytes ? temp_bytes : 16);
  if (e == hipSuccess)
    e = rocprim::inclusive_scan(temp, temp_bytes, in, cost_scan, size_t(num_vertices), rocprim::plus<uint64_t>(), s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (temp) (void)hipFree(temp);
  return e;
}

hipError_t scan_hotness(const uint32_t* hot, const int32_t* order, int64_t num_vertices, uint64_t* hot_scan,
                        hipStream_t s) {
  auto in = rocprim::make_transform_iterator(rocprim::counting_iterator<int64_t>(0), HotAlong{hot, order});
  void* temp = nullptr;
  size_t temp_bytes = 0;
  hipError_t e = rocprim::inclusive_scan(nullptr, temp_bytes, in, hot_scan, size_t(num_vertices),
                                         rocprim::plus<uint64_t>(), s);
  if (e == hipSuccess) e = hipMalloc(&temp, temp_bytes ? temp_bytes : 16);
  if (e == hipSuccess)
    e = rocprim::inclusive_scan(temp, temp_bytes, in, hot_scan, size_t(num_vertices), rocprim::plus<uint64_t>(), s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (temp) (void)hipFree(temp);
  return e;
}

void launch_alpha_search(const uint64_t* cost_scan, const uint64_t* hot_t_scan, const uint64_t* hot_f_scan,
                         int64_t num_vertices, uint64_t row_bytes, const uint64_t* m_topo, uint64_t total_budget,
                         uint64_t n_tsum, uint64_t per_row, int32_t n_alpha, lgp_plan_point* points, int32_t* best,
                         hipStream_t s) {
  hipLaunchKernelGGL(alpha_search_kernel, dim3(1), dim3(1024), 0, s, cost_scan, hot_t_scan, hot_f_scan, num_vertices,
                     row_bytes, m_topo, total_budget, n_tsum, per_row, n_alpha, points, best);
}

hipError_t shuffle_by_key(const DeviceInfo& di, const int32_t* in, int32_t* out, int64_t n, uint64_t seed,
                          uint32_t epoch, hipStream_t s) {
  uint64_t *keys = nullptr, *keys_out = nullptr;
  void* temp = nullptr;
  size_t temp_bytes = 0;
  hipError_t e = hipMalloc(&keys, sizeof(uint64_t) * size_t(n));
  if (e == hipSuccess) e = hipMalloc(&keys_out, sizeof(uint64_t) * size_t(n));
  if (e == hipSuccess) {
    hipLaunchKernelGGL(shuffle_keys_kernel, dim3(grid_for(di, n)), dim3(256), 0, s, keys, n, uint32_t(seed),
                       uint32_t(seed >> 32), epoch);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = rocprim::radix_sort_pairs(nullptr, temp_bytes, keys, keys_out, in, out, size_t(n), 0, 64, s);
  if (e == hipSuccess) e = hipMalloc(&temp, temp_bytes + 16);
  if (e == hipSuccess) e = rocprim::radix_sort_pairs(temp, temp_bytes, keys, keys_out, in, out, size_t(n), 0, 64, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  for (void* p : {static_cast<void*>(keys), static_cast<void*>(keys_out), temp})
    if (p) (void)hipFree(p);
  return e;
}

hipError_t cslp_rank(const DeviceInfo& di, int32_t k_g, int64_t num_vertices, const uint32_t* hot, uint64_t* acc,
                     int32_t* order, int32_t* owner, int32_t* queues, unsigned long long* counts, hipStream_t s) {
  const size_t V = size_t(num_vertices);
  uint64_t* keys_out = nullptr;
  uint32_t *okey = nullptr, *okey_out = nullptr;
  void* temp = nullptr;
  size_t t1 = 0, t2 = 0;
  int bits = 1;
  while ((1 << bits) < k_g) ++bits;
  hipError_t e = hipMalloc(&keys_out, sizeof(uint64_t) * V);
  if (e == hipSuccess) e = hipMalloc(&okey, sizeof(uint32_t) * V);
  if (e == hipSuccess) e = hipMalloc(&okey_out, sizeof(uint32_t) * V);
  if (e == hipSuccess) e = hipMemsetAsync(counts, 0, sizeof(unsigned long long) * size_t(k_g), s);
  rocprim::counting_iterator<int32_t> ids(0);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(colsum_argmax_kernel, dim3(grid_for(di, num_vertices)), dim3(256), 0, s, hot, k_g,
                       num_vertices, acc, owner);
    e = hipGetLastError();
  }
  // step 2: stable descending sort of the 64-bit sums -> equal sums keep ascending id order
  if (e == hipSuccess) e = rocprim::radix_sort_pairs_desc(nullptr, t1, acc, keys_out, ids, order, V, 0, 64, s);
  // step 3: stable ascending sort by owner over the ranked list -> the per-GPU queues, end to end
  if (e == hipSuccess) e = rocprim::radix_sort_pairs(nullptr, t2, okey, okey_out, order, queues, V, 0, bits, s);
  if (e == hipSuccess) e = hipMalloc(&temp, (t1 > t2 ? t1 : t2) + 16);
  if (e == hipSuccess) e = rocprim::radix_sort_pairs_desc(temp, t1, acc, keys_out, ids, order, V, 0, 64, s);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(owner_along_kernel, dim3(grid_for(di, num_vertices)), dim3(256), 0, s, owner, order,
                       num_vertices, okey, counts, k_g);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = rocprim::radix_sort_pairs(temp, t2, okey, okey_out, order, queues, V, 0, bits, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  for (void* p : {static_cast<void*>(keys_out), static_cast<void*>(okey), static_cast<void*>(okey_out), temp})
    if (p) (void)hipFree(p);
  return e;
}

void launch_prefix_within_budget(const uint64_t* scan, int64_t n, uint64_t budget, uint64_t* result, hipStream_t s) {
  hipLaunchKernelGGL(prefix_within_budget_kernel, dim3(1), dim3(64), 0, s, scan, n, budget, result);
}

void launch_topo_offsets(const DeviceInfo& di, const uint64_t* cost_scan, int64_t n_topo, int64_t* t_indptr,
                         hipStream_t s) {
  hipLaunchKernelGGL(topo_offsets_kernel, dim3(grid_for(di, n_topo + 1)), dim3(256), 0, s, cost_scan, n_topo,
                     t_indptr);
}

void launch_fill_topo(const DeviceInfo& di, const void* h_indptr, int32_t indptr_bytes, const int32_t* h_indices,
                      const int32_t* order, int64_t n_topo, const int64_t* t_indptr, int32_t* t_indices,
                      hipStream_t s) {
  if (n_topo <= 0) return;
  const unsigned grid = grid_for(di, n_topo, 16);
  if (indptr_bytes == 8)
    hipLaunchKernelGGL(fill_topo_kernel<int64_t>, dim3(grid), dim3(256), 0, s, static_cast<const int64_t*>(h_indptr),
                       h_indices, order, n_topo, t_indptr, t_indices);
  else
    hipLaunchKernelGGL(fill_topo_kernel<int32_t>, dim3(grid), dim3(256), 0, s, static_cast<const int32_t*>(h_indptr),
                       h_indices, order, n_topo, t_indptr, t_indices);
}

void launch_fill_i32(const DeviceInfo& di, int32_t* p, int64_t n, int32_t value, hipStream_t s) {
  hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(di, n)), dim3(256), 0, s, p, n, value);
}

void launch_init_row_table(const DeviceInfo& di, const void* h_indptr, int32_t indptr_bytes, int64_t num_vertices,
                           uint64_t* row_tab, hipStream_t s) {
  if (indptr_bytes == 8)
    hipLaunchKernelGGL(init_row_table_kernel<int64_t>, dim3(grid_for(di, num_vertices)), dim3(256), 0, s,
                       static_cast<const int64_t*>(h_indptr), num_vertices, row_tab);
  else
    hipLaunchKernelGGL(init_row_table_kernel<int32_t>, dim3(grid_for(di, num_vertices)), dim3(256), 0, s,
                       static_cast<const int32_t*>(h_indptr), num_vertices, row_tab);
}

void launch_set_cached_rows(const DeviceInfo& di, const int32_t* order, int64_t n_topo, const int64_t* t_indptr,
                            uint64_t* row_tab, hipStream_t s) {
  if (n_topo <= 0) return;
  hipLaunchKernelGGL(set_cached_rows_kernel, dim3(grid_for(di, n_topo)), dim3(256), 0, s, order, n_topo, t_indptr,
                     row_tab);
}

void launch_iota_i32(const DeviceInfo& di, int32_t* p, int64_t n, hipStream_t s) {
  hipLaunchKernelGGL(iota_i32_kernel, dim3(grid_for(di, n)), dim3(256), 0, s, p, n);
}

void launch_scatter_rank(const DeviceInfo& di, const int32_t* order, int64_t n, int32_t* remap, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(scatter_rank_kernel, dim3(grid_for(di, n)), dim3(256), 0, s, order, n, remap);
}

}  // namespace lgp
