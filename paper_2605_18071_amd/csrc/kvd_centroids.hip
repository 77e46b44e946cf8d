// The hierarchical index (System Overview: the page means form higher-level centroids for
// similarity grouping; Pipeline Optimization: the number of centroids is a tunable of the index).
//
// Build (set-up helper, not on the decode path): Lloyd's k-means over the page summaries of every
// unit, in fp64 so that its decisions can be checked against a plain CPU implementation: initial
// centroids = the pages at evenly spaced positions, nearest centroid by squared Euclidean distance
// (ties to the lower centroid), new centroid = mean of the cluster's summaries summed in ascending
// page order (an empty cluster keeps its centroid), a fixed number of rounds; the stored centroid
// is rounded once to the KV dtype and each cluster's pages are listed in ascending order.
//
// Decode: the scoring kernel runs over the centroids instead of the page summaries (half the
// bytes when there are half as many centroids as pages); cluster_select_kernel then takes whole
// clusters in (score descending, cluster ascending) order until the page budget is used up, the
// first cluster that does not fit giving its lowest pages; sink / recent pages are in first and
// are not counted as members of their clusters.
#include "kvd_cluster_body.h"
#include "kvd_device.h"
#include "kvd_internal.h"

namespace kvd {

// ---------------------------------------------------------------------------------------------
// build
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ double widen_kv(uint16_t raw) {
  return (double)(BF16 ? as_f32((u32)raw << 16) : (float)__builtin_bit_cast(_Float16, raw));
}

// cent64 [U][Nc][D] <- summaries of the pages floor((c + 1/2) * n_valid / Nc)
template <bool BF16>
__global__ __launch_bounds__(kHeadDim) void kmeans_init_kernel(const uint16_t* __restrict__ summ, double* __restrict__ cent64,
                                                              const int32_t* __restrict__ seq_len, int NP, int Nc, int P,
                                                              int Hkv) {
  const int c = blockIdx.x, u = blockIdx.y, d = threadIdx.x;
  int n_valid = (seq_len[u / Hkv] + P - 1) / P;
  n_valid = n_valid < NP ? n_valid : NP;
  const int page = (int)(((double)c + 0.5) * (double)n_valid / (double)Nc);
  cent64[((size_t)u * Nc + c) * kHeadDim + d] = widen_kv<BF16>(summ[((size_t)u * NP + page) * kHeadDim + d]);
}

constexpr int kAssignThreads = 256;
constexpr int kAssignPoints = 16;     // points per block

// Block (x, u): points 16x .. 16x+15 of unit u against all centroids.  The points sit in LDS as
// fp64; thread t takes centroids t, t + 256, ... and keeps, for each of the 16 points, the best
// (distance, centroid) it has seen; the threads' bests are then reduced per point.
template <bool BF16>
__global__ __launch_bounds__(kAssignThreads) void kmeans_assign_kernel(const uint16_t* __restrict__ summ,
                                                                      const double* __restrict__ cent64,
                                                                      int32_t* __restrict__ assign,   // [U][NP]
                                                                      const int32_t* __restrict__ seq_len, int NP, int Nc,
                                                                      int P, int Hkv) {
  __shared__ double pts[kAssignPoints][kHeadDim];
  __shared__ double best_d[kAssignPoints][kAssignThreads / kWave];
  __shared__ int best_c[kAssignPoints][kAssignThreads / kWave];
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  int n_valid = (seq_len[u / Hkv] + P - 1) / P;
  n_valid = n_valid < NP ? n_valid : NP;
  const int p0 = blockIdx.x * kAssignPoints;
  if (p0 >= n_valid) return;
  for (int i = tid; i < kAssignPoints * kHeadDim; i += kAssignThreads) {
    const int pi = i / kHeadDim, d = i % kHeadDim;
    const int page = (p0 + pi) < n_valid ? (p0 + pi) : (n_valid - 1);
    pts[pi][d] = widen_kv<BF16>(summ[((size_t)u * NP + page) * kHeadDim + d]);
  }
  __syncthreads();
  double bd[kAssignPoints];
  int bc[kAssignPoints];
#pragma unroll
  for (int i = 0; i < kAssignPoints; ++i) { bd[i] = INFINITY; bc[i] = 0x7fffffff; }
  for (int c = tid; c < Nc; c += kAssignThreads) {
    const double* crow = cent64 + ((size_t)u * Nc + c) * kHeadDim;
    double acc[kAssignPoints];
#pragma unroll
    for (int i = 0; i < kAssignPoints; ++i) acc[i] = 0.0;
    for (int d = 0; d < kHeadDim; d += 2) {
      const double2 cv = *reinterpret_cast<const double2*>(crow + d);
#pragma unroll
      for (int i = 0; i < kAssignPoints; ++i) {
        const double e0 = pts[i][d] - cv.x, e1 = pts[i][d + 1] - cv.y;
        acc[i] = fma(e0, e0, acc[i]);
        acc[i] = fma(e1, e1, acc[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < kAssignPoints; ++i)
      if (acc[i] < bd[i]) { bd[i] = acc[i]; bc[i] = c; }       // centroids come in ascending order per thread
  }
  // smallest (distance, centroid) per point over the block
#pragma unroll
  for (int i = 0; i < kAssignPoints; ++i) {
    double d = bd[i];
    int c = bc[i];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      const double od = __shfl_xor(d, m, kWave);
      const int oc = __shfl_xor(c, m, kWave);
      if (od < d || (od == d && oc < c)) { d = od; c = oc; }
    }
    if (lane == 0) { best_d[i][w] = d; best_c[i][w] = c; }
  }
  __syncthreads();
  if (tid < kAssignPoints && p0 + tid < n_valid) {
    double d = best_d[tid][0];
    int c = best_c[tid][0];
    for (int j = 1; j < kAssignThreads / kWave; ++j) {
      const double od = best_d[tid][j];
      const int oc = best_c[tid][j];
      if (od < d || (od == d && oc < c)) { d = od; c = oc; }
    }
    assign[(size_t)u * NP + p0 + tid] = c;
  }
}

constexpr int kCsrThreads = 1024;

// One block per unit: cluster_start [Nc+1] and cluster_pages [NP] (pages of every cluster in
// ascending order) from assign.
__global__ __launch_bounds__(kCsrThreads) void kmeans_csr_kernel(const int32_t* __restrict__ assign,
                                                                int32_t* __restrict__ cluster_start,   // [U][Nc+1]
                                                                int32_t* __restrict__ cluster_pages,   // [U][NP]
                                                                int32_t* __restrict__ cursor,          // [U][Nc] scratch
                                                                const int32_t* __restrict__ seq_len, int NP, int Nc,
                                                                int P, int Hkv) {
  __shared__ int scan_smem[kCsrThreads / kWave + 1];
  __shared__ int carry;
  const int u = blockIdx.x, tid = threadIdx.x;
  int n_valid = (seq_len[u / Hkv] + P - 1) / P;
  n_valid = n_valid < NP ? n_valid : NP;
  const int32_t* as = assign + (size_t)u * NP;
  int32_t* start = cluster_start + (size_t)u * (Nc + 1);
  int32_t* pages = cluster_pages + (size_t)u * NP;
  int32_t* cur = cursor + (size_t)u * Nc;
  for (int c = tid; c < Nc; c += kCsrThreads) cur[c] = 0;
  for (int p = n_valid + tid; p < NP; p += kCsrThreads) pages[p] = -1;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int p = tid; p < n_valid; p += kCsrThreads) atomicAdd(&cur[as[p]], 1);
  __syncthreads();
  // exclusive scan of the counts, 1024 clusters at a time
  for (int c0 = 0; c0 < Nc; c0 += kCsrThreads) {
    const int c = c0 + tid;
    const int cnt = c < Nc ? cur[c] : 0;
    int total;
    const int ex = block_exclusive_scan<kCsrThreads>(cnt, scan_smem, total);
    const int base = carry;
    if (c < Nc) start[c] = base + ex;
    __syncthreads();
    if (tid == 0) carry = base + total;
    __syncthreads();
  }
  if (tid == 0) start[Nc] = carry;
  for (int c = tid; c < Nc; c += kCsrThreads) cur[c] = 0;
  __syncthreads();
  for (int p = tid; p < n_valid; p += kCsrThreads) {
    const int c = as[p];
    pages[start[c] + atomicAdd(&cur[c], 1)] = p;
  }
  __syncthreads();
  // every cluster's list in ascending page order (lists are short: insertion sort by one thread)
  for (int c = tid; c < Nc; c += kCsrThreads) {
    const int b = start[c], e = start[c + 1];
    for (int i = b + 1; i < e; ++i) {
      const int v = pages[i];
      int j = i - 1;
      while (j >= b && pages[j] > v) { pages[j + 1] = pages[j]; --j; }
      pages[j + 1] = v;
    }
  }
}

// Block (c, u), thread d: new centroid = mean of the members' summaries in ascending page order.
template <bool BF16>
__global__ __launch_bounds__(kHeadDim) void kmeans_update_kernel(const uint16_t* __restrict__ summ, double* __restrict__ cent64,
                                                                const int32_t* __restrict__ cluster_start,
                                                                const int32_t* __restrict__ cluster_pages, int NP, int Nc) {
  const int c = blockIdx.x, u = blockIdx.y, d = threadIdx.x;
  const int b = cluster_start[(size_t)u * (Nc + 1) + c], e = cluster_start[(size_t)u * (Nc + 1) + c + 1];
  if (e == b) return;                                       // an empty cluster keeps its centroid
  const int32_t* pages = cluster_pages + (size_t)u * NP;
  double acc = 0.0;
  for (int i = b; i < e; ++i) acc += widen_kv<BF16>(summ[((size_t)u * NP + pages[i]) * kHeadDim + d]);
  cent64[((size_t)u * Nc + c) * kHeadDim + d] = acc / (double)(e - b);
}

template <bool BF16>
__global__ __launch_bounds__(kHeadDim) void kmeans_store_kernel(const double* __restrict__ cent64, uint16_t* __restrict__ centroids,
                                                               int Nc) {
  const size_t i = ((size_t)blockIdx.y * Nc + blockIdx.x) * kHeadDim + threadIdx.x;
  centroids[i] = f64_to_kv<BF16>(cent64[i]);
}

// ---------------------------------------------------------------------------------------------
// decode: clusters -> pages (see kvd_cluster_body.h)
// ---------------------------------------------------------------------------------------------
constexpr int kClusterThreads = 1024;

// One block per unit.
__global__ __launch_bounds__(kClusterThreads) void cluster_select_kernel(const float* __restrict__ scores,
                                                                        const int32_t* __restrict__ cluster_start,
                                                                        const int32_t* __restrict__ cluster_pages,
                                                                        int32_t* __restrict__ sel_pages,
                                                                        const int32_t* __restrict__ seq_len, int NP, int Nc,
                                                                        int P, int k, int sink, int recent, int Hkv, int u0) {
  extern __shared__ __align__(16) unsigned char cs_raw[];
  ClusterSelectSmem<kClusterThreads>& sm = *reinterpret_cast<ClusterSelectSmem<kClusterThreads>*>(cs_raw);
  cluster_select_body<kClusterThreads, false>(scores, cluster_start, cluster_pages, sel_pages, seq_len, NP, Nc, P, k, sink,
                                              recent, Hkv, blockIdx.x + u0, sm);
}

// page_cluster [NP] of unit blockIdx.x from its cluster lists: -1, then the cluster of every listed page.
__global__ __launch_bounds__(kCsrThreads) void cluster_inverse_kernel(const int32_t* __restrict__ cluster_start,
                                                                     const int32_t* __restrict__ cluster_pages,
                                                                     int32_t* __restrict__ page_cluster, int NP, int Nc) {
  const int u = blockIdx.x, tid = threadIdx.x;
  const int32_t* start = cluster_start + (size_t)u * (Nc + 1);
  const int32_t* pages = cluster_pages + (size_t)u * NP;
  int32_t* pc = page_cluster + (size_t)u * NP;
  for (int p = tid; p < NP; p += kCsrThreads) pc[p] = -1;
  __syncthreads();
  for (int c = tid; c < Nc; c += kCsrThreads) {
    int b = start[c], e = start[c + 1];
    b = b < 0 ? 0 : b;
    e = e > NP ? NP : e;
    for (int i = b; i < e; ++i) {
      const int p = pages[i];
      if (p >= 0 && p < NP) pc[p] = c;
    }
  }
}

}  // namespace kvd

bool kvd_centroid_mode(const kvd_ctx* c) { return c->Nc > 0; }

hipError_t kvd_prepare_cluster_select(void) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kvd::cluster_select_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(kvd::ClusterSelectSmem<kvd::kClusterThreads>));
}

hipError_t kvd_launch_cluster_select(kvd_ctx* c, int layer, const float* scores, int32_t* sel_pages, int u0, int u1,
                                     hipStream_t s) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  const size_t lu = (size_t)layer * c->U;
  hipLaunchKernelGGL(cluster_select_kernel, dim3(u1 - u0), dim3(kClusterThreads), sizeof(ClusterSelectSmem<kClusterThreads>), s, scores,
                     c->cluster_start + lu * (c->Nc + 1), c->cluster_pages + lu * c->NP, sel_pages, c->d_seq_len, c->NP, c->Nc,
                     c->P, c->k, c->cfg.sink_pages, c->cfg.recent_pages, c->Hkv, u0);
  return hipGetLastError();
}

hipError_t kvd_launch_cluster_inverse(kvd_ctx* c, int layer, hipStream_t s) {
  using namespace kvd;
  const size_t lu = (size_t)layer * c->U;
  hipLaunchKernelGGL(cluster_inverse_kernel, dim3(c->U), dim3(kCsrThreads), 0, s, c->cluster_start + lu * (c->Nc + 1),
                     c->cluster_pages + lu * c->NP, c->d_page_cluster + lu * c->NP, c->NP, c->Nc);
  return hipGetLastError();
}

// k-means over the layer's page summaries; assign_trace (device, [iterations][U][NP], or null)
// receives the assignment of every round.  Synchronous; uses temporary device memory.
hipError_t kvd_run_build_centroids(kvd_ctx* c, int layer, int iterations, int32_t* assign_trace, hipStream_t s) {
  using namespace kvd;
  const size_t lu = (size_t)layer * c->U;
  const uint16_t* summ = reinterpret_cast<const uint16_t*>(c->summaries) + lu * c->NP * kHeadDim;
  uint16_t* cent = reinterpret_cast<uint16_t*>(c->centroids) + lu * c->Nc * kHeadDim;
  int32_t* cstart = c->cluster_start + lu * (c->Nc + 1);
  int32_t* cpages = c->cluster_pages + lu * c->NP;
  double* cent64 = nullptr;
  int32_t* assign = nullptr;
  int32_t* cursor = nullptr;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&cent64), (size_t)c->U * c->Nc * kHeadDim * sizeof(double));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&assign), (size_t)c->U * c->NP * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&cursor), (size_t)c->U * c->Nc * sizeof(int32_t));
  if (e == hipSuccess) {
    const dim3 per_centroid(c->Nc, c->U), per_points((c->NP + kAssignPoints - 1) / kAssignPoints, c->U);
#define KVD_DT(KERNEL, ...)                                                    \
  do {                                                                         \
    if (c->bf16) hipLaunchKernelGGL((KERNEL<true>), __VA_ARGS__);              \
    else hipLaunchKernelGGL((KERNEL<false>), __VA_ARGS__);                     \
  } while (0)
    KVD_DT(kmeans_init_kernel, per_centroid, dim3(kHeadDim), 0, s, summ, cent64, c->d_seq_len, c->NP, c->Nc, c->P, c->Hkv);
    for (int it = 0; it < iterations && e == hipSuccess; ++it) {
      KVD_DT(kmeans_assign_kernel, per_points, dim3(kAssignThreads), 0, s, summ, cent64, assign, c->d_seq_len, c->NP, c->Nc,
             c->P, c->Hkv);
      if (assign_trace != nullptr)
        e = hipMemcpyAsync(assign_trace + (size_t)it * c->U * c->NP, assign, (size_t)c->U * c->NP * sizeof(int32_t),
                           hipMemcpyDeviceToDevice, s);
      hipLaunchKernelGGL(kmeans_csr_kernel, dim3(c->U), dim3(kCsrThreads), 0, s, assign, cstart, cpages, cursor, c->d_seq_len,
                         c->NP, c->Nc, c->P, c->Hkv);
      KVD_DT(kmeans_update_kernel, per_centroid, dim3(kHeadDim), 0, s, summ, cent64, cstart, cpages, c->NP, c->Nc);
    }
    KVD_DT(kmeans_store_kernel, per_centroid, dim3(kHeadDim), 0, s, cent64, cent, c->Nc);
#undef KVD_DT
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = kvd_launch_cluster_inverse(c, layer, s);   // the page -> cluster table of the new lists
    const hipError_t e2 = hipStreamSynchronize(s);
    if (e == hipSuccess) e = e2;
  }
  if (cent64) (void)hipFree(cent64);
  if (assign) (void)hipFree(assign);
  if (cursor) (void)hipFree(cursor);
  return e;
}
