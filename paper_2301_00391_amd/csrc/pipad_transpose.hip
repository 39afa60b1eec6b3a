// pipad_frame_transpose: the frame of the transposed parts with the forward normalisation.
// A translation unit of its own, so that the library sort it uses is only loaded when it is called.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "pipad_internal.h"

namespace pipad {
namespace {

// Last row i in [lo, hi] with rowptr[i] <= e, given rowptr[lo] <= e < rowptr[hi + 1].
__device__ inline int32_t row_of_entry(const int32_t *rp, int32_t lo, int32_t hi, int32_t e) {
  while (lo < hi) {
    const int32_t mid = lo + ((hi - lo + 1) >> 1);
    if (rp[mid] <= e) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// row[e] = row that holds entry e: one thread per entry, bisection over the row pointers.
__global__ __launch_bounds__(kBlock) void k_entry_rows(const int32_t *rowptr, int32_t n, int32_t nnz,
                                                        int32_t *row) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= nnz) return;
  row[e] = row_of_entry(rowptr, 0, n - 1, (int32_t)e);
}

// Row pointers of a CSR whose entries' row ids are given in ascending order:
// rowptr[i] = number of ids below i, for i in [0, n].
__global__ __launch_bounds__(kBlock) void k_rowptr_of_sorted(const uint32_t *ids, int32_t nnz,
                                                              int32_t n, int32_t *rowptr) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i > n) return;
  int32_t lo = 0, hi = nnz;
  while (lo < hi) {
    const int32_t mid = lo + ((hi - lo) >> 1);
    if (ids[mid] < (uint32_t)i) lo = mid + 1; else hi = mid;
  }
  rowptr[i] = lo;
}

// w[e] = dinv_t[col[e]] for one part and one snapshot.
__global__ __launch_bounds__(kBlock) void k_entry_scales(const int32_t *col, int32_t nnz,
                                                          const float *dinv_t, float *w) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e < nnz) w[e] = dinv_t[col[e]];
}

__global__ void k_class_totals(int32_t n, int32_t k, const uint32_t *hubidx, const uint32_t *segoff,
                               const uint32_t *shortidx, const uint32_t *split_total,
                               uint32_t *out) {
  const int q = threadIdx.x;
  if (q == 0) {
    out[0] = hubidx[n];
    out[1] = segoff[n];
    out[2] = shortidx[n];
  }
  if (q <= k) out[3 + q] = split_total[q];
}

}  // namespace

// The frame of the transposed patterns with the SAME D^-1/2: aggregating with it multiplies by
// the transposed normalised adjacency.  Every part is transposed on its own (the transpose of an
// intersection is the intersection of the transposes): entries are tagged with their row, sorted
// by column with a stable radix sort (a library primitive, rocPRIM) - rows arrive in ascending
// order, so they leave in ascending order within every column - and the new row pointers are read
// off the sorted columns.
int transpose_frame(const pipad_frame *f, pipad_alloc_fn alloc, void *alloc_ctx, hipStream_t st,
                    pipad_frame **out) {
  const int32_t n = f->n, k = f->k;
  pipad_frame *g = new (std::nothrow) pipad_frame;
  if (!g) return PIPAD_ERR_ALLOC;
  g->n = n;
  g->k = k;
  g->device = f->device;
  g->own_memory = alloc == nullptr;
  g->alloc = alloc;
  g->alloc_ctx = alloc_ctx;
  g->opt = f->opt;  // the transposed frame keeps the options of the frame it comes from
  g->short_max = f->short_max;
  g->mid_max = f->mid_max;
  g->hub_threshold = f->hub_threshold;
  g->hub_segment = f->hub_segment;
  g->sub_log2 = f->sub_log2;
  g->nclass = f->nclass;
  g->nnz_c = f->nnz_c;
  for (int t = 0; t < k; ++t) g->nnz_d[t] = f->nnz_d[t];
  Allocator A{alloc, alloc_ctx, g};
  void *temp = nullptr;
  auto fail = [&](int code) {
    if (temp && !alloc) (void)hipFree(temp);
    release(g);
    return code;
  };
  auto hipcheck = [&](hipError_t e, const char *what) { return e == hipSuccess ? 0 : hip_fail(e, what); };
#define PIPAD_TRY_T(call)                                 \
  do {                                                    \
    int rc__ = hipcheck((call), #call);                   \
    if (rc__ != 0) return fail(rc__);                     \
  } while (0)

  Arena keep;
  keep.want(&g->rowptr_c, (size_t)n + 1);
  for (int t = 0; t < k; ++t) keep.want(&g->rowptr_d[t], (size_t)n + 1);
  keep.want(&g->dinv, (size_t)k * n);
  keep.want(&g->dinv_nk, (size_t)k * n);
  keep.want(&g->col_c, (size_t)g->nnz_c);
  for (int t = 0; t < k; ++t) {
    keep.want(&g->col_d[t], (size_t)g->nnz_d[t]);
    keep.want(&g->wc[t], (size_t)g->nnz_c);
    keep.want(&g->wd[t], (size_t)g->nnz_d[t]);
  }
  {
    void *base = A.get(keep.total);
    if (!base) return fail(PIPAD_ERR_ALLOC);
    keep.assign(base);
  }
  if (n == 0) {
    *out = g;
    return PIPAD_OK;
  }

  int32_t max_nnz = g->nnz_c;
  for (int t = 0; t < k; ++t) max_nnz = std::max(max_nnz, g->nnz_d[t]);
  int bits = 1;
  while (((int64_t)1 << bits) < n) ++bits;
  size_t sort_bytes = 0;
  if (max_nnz > 0)
    PIPAD_TRY_T(rocprim::radix_sort_pairs(nullptr, sort_bytes, (const uint32_t *)nullptr,
                                          (uint32_t *)nullptr, (const int32_t *)nullptr,
                                          (int32_t *)nullptr, (size_t)max_nnz, 0, bits, st));
  const uint32_t scan_len = (uint32_t)n + 1;
  Arena tmp;
  int32_t *rows = nullptr;
  uint32_t *sorted = nullptr, *bsum = nullptr, *shortidx = nullptr, *hubidx = nullptr,
           *segoff = nullptr, *totals = nullptr, *split_total = nullptr;
  char *sort_tmp = nullptr;
  tmp.want(&rows, (size_t)max_nnz);
  tmp.want(&sorted, (size_t)max_nnz);
  tmp.want(&sort_tmp, sort_bytes);
  tmp.want(&bsum, 3 * scan_block_words(scan_len) + 1);
  tmp.want(&shortidx, (size_t)scan_len);
  tmp.want(&hubidx, (size_t)scan_len);
  tmp.want(&segoff, (size_t)scan_len);
  tmp.want(&totals, (size_t)PIPAD_MAX_K + 8);
  tmp.want(&split_total, (size_t)PIPAD_MAX_K + 1);
  if (alloc) {
    temp = alloc(tmp.total, alloc_ctx);
    g->temp_ptr = temp;
    g->temp_bytes = temp ? tmp.total : 0;
  } else if (hipMalloc(&temp, tmp.total) != hipSuccess) {
    (void)hipGetLastError();
    temp = nullptr;
  }
  if (!temp) return fail(PIPAD_ERR_ALLOC);
  tmp.assign(temp);

  PIPAD_TRY_T(hipMemcpyAsync(g->dinv, f->dinv, sizeof(float) * (size_t)k * n,
                             hipMemcpyDeviceToDevice, st));
  PIPAD_TRY_T(hipMemcpyAsync(g->dinv_nk, f->dinv_nk, sizeof(float) * (size_t)k * n,
                             hipMemcpyDeviceToDevice, st));
  for (int part = 0; part <= k; ++part) {
    const int32_t nnz = part == 0 ? f->nnz_c : f->nnz_d[part - 1];
    const int32_t *rp = part == 0 ? f->rowptr_c : f->rowptr_d[part - 1];
    const int32_t *col = part == 0 ? f->col_c : f->col_d[part - 1];
    int32_t *rp_out = part == 0 ? g->rowptr_c : g->rowptr_d[part - 1];
    int32_t *col_out = part == 0 ? g->col_c : g->col_d[part - 1];
    if (nnz > 0) {
      hipLaunchKernelGGL(k_entry_rows, grid1(nnz, kBlock), dim3(kBlock), 0, st, rp, n, nnz, rows);
      PIPAD_TRY_T(hipGetLastError());
      size_t bytes = sort_bytes;
      PIPAD_TRY_T(rocprim::radix_sort_pairs(sort_tmp, bytes, reinterpret_cast<const uint32_t *>(col),
                                            sorted, rows, col_out, (size_t)nnz, 0, bits, st));
    }
    hipLaunchKernelGGL(k_rowptr_of_sorted, grid1((int64_t)n + 1, kBlock), dim3(kBlock), 0, st, sorted,
                       nnz, n, rp_out);
    for (int t = 0; t < k && nnz > 0; ++t) {
      if (part != 0 && t != part - 1) continue;  // an exclusive part carries its own snapshot's scales
      float *w = part == 0 ? g->wc[t] : g->wd[t];
      hipLaunchKernelGGL(k_entry_scales, grid1(nnz, kBlock), dim3(kBlock), 0, st, col_out, nnz,
                         g->dinv + (size_t)t * n, w);
    }
    PIPAD_TRY_T(hipGetLastError());
  }

  {
    const int rc = launch_classify(g, shortidx, hubidx, segoff, split_total, st);
    if (rc != 0) return fail(rc);
  }
  {
    uint32_t *three[3] = {shortidx, hubidx, segoff};
    const int rc = scan_exclusive(three, 3, scan_len, bsum, st);
    if (rc != 0) return fail(rc);
  }
  uint32_t host_totals[PIPAD_MAX_K + 8] = {};
  hipLaunchKernelGGL(k_class_totals, dim3(1), dim3(kWave), 0, st, n, k, hubidx, segoff, shortidx,
                     split_total, totals);
  PIPAD_TRY_T(hipGetLastError());
  PIPAD_TRY_T(hipMemcpyAsync(host_totals, totals, sizeof(uint32_t) * (size_t)(k + 4),
                             hipMemcpyDeviceToHost, st));
  PIPAD_TRY_T(hipStreamSynchronize(st));
  {
    const int rc = set_list_sizes(g, host_totals[0], host_totals[1], host_totals[2], host_totals + 3);
    if (rc != 0) return fail(rc);
  }

  Arena lists;
  uint32_t *ulen = nullptr, *ubsum = nullptr;
  want_lists(lists, g, &ulen, &ubsum);
  {
    void *base = A.get(lists.total);
    if (!base) return fail(PIPAD_ERR_ALLOC);
    lists.assign(base);
  }
  launch_row_lists(n, shortidx, hubidx, segoff, g, st);
  PIPAD_TRY_T(hipGetLastError());
  {
    const int rc = build_split_arrays(g, ulen, ubsum, st);
    if (rc != 0) return fail(rc);
  }
  if (!alloc) {
    PIPAD_TRY_T(hipStreamSynchronize(st));  // the temporaries are freed next
    (void)hipFree(temp);
  }
#undef PIPAD_TRY_T
  *out = g;
  return PIPAD_OK;
}

}  // namespace pipad
