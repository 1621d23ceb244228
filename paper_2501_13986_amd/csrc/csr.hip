// Integer graph preparation on the device: COO -> CSR by receiver plus the transpose
// permutation (paper Sec. 3.5: the fused kernels need row-sorted edges, and the backward pass
// a permutation that transposes the adjacency), and two small helpers of the conv path.
// Statically compiled (nothing here depends on the irreps).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <mutex>

#include <rocprim/rocprim.hpp>

#include "csr.hpp"

namespace cgtp {
namespace {

constexpr int kBlock = 256;

template <class K>
__global__ void k_make_keys(const int64_t* __restrict__ recv, const int64_t* __restrict__ send, int64_t E, int64_t V,
                            K* __restrict__ keys, int64_t* __restrict__ idx, int* __restrict__ bad) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  int64_t r = recv[e], s = send[e];
  if (r < 0 || r >= V || s < 0 || s >= V) {
    *bad = 1;  // plain store of the same value from any thread
    r = 0;
    s = 0;
  }
  keys[e] = (K)((uint64_t)r * (uint64_t)V + (uint64_t)s);
  idx[e] = e;
}

// first position whose key is >= target, for targets j*stride, j = 0..V
template <class K>
__global__ void k_lower_bounds(const K* __restrict__ keys, int64_t E, int64_t V, uint64_t stride,
                               int64_t* __restrict__ ptr) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j > V) return;
  uint64_t target = (uint64_t)j * stride;
  int64_t lo = 0, hi = E;
  while (lo < hi) {
    int64_t mid = (lo + hi) >> 1;
    if ((uint64_t)keys[mid] < target) lo = mid + 1; else hi = mid;
  }
  ptr[j] = lo;
}

template <class K>
__global__ void k_col_from_perm(const int64_t* __restrict__ send, const int64_t* __restrict__ perm, int64_t E,
                                int64_t* __restrict__ col, K* __restrict__ colkey, int64_t* __restrict__ pos) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  int64_t c = send[perm[e]];
  col[e] = c;
  colkey[e] = (K)c;
  pos[e] = e;
}

// receiver (CSR row) of the edge at every position of the transposed order
__global__ void k_recv_of_tperm(const int64_t* __restrict__ row_ptr, const int64_t* __restrict__ t_perm, int64_t V,
                                int64_t E, int64_t* __restrict__ t_recv) {
  int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= E) return;
  int64_t e = t_perm[q];
  int64_t lo = 0, hi = V;  // row_ptr[lo] <= e < row_ptr[hi]
  while (hi - lo > 1) {
    int64_t mid = (lo + hi) >> 1;
    if (row_ptr[mid] <= e) lo = mid; else hi = mid;
  }
  t_recv[q] = lo;
}

__global__ void k_fill_zero(uint32_t* __restrict__ p, int64_t n_words) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n_words; i += step) p[i] = 0u;
}

template <typename T>
__global__ void k_add_inplace(T* __restrict__ a, const T* __restrict__ b, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) a[i] += b[i];
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

// Scratch for the entry point that allocates nothing (conv_forward_static): device memory that exists from the
// moment the library's code is loaded on a GPU until the process ends.  Every GPU holds its own copy at its own
// address; in host code the name below is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// keeps the array in the code object although no statically compiled kernel of the library reads it: the
// kernels that use it are compiled at run time and get its address as an argument
__attribute__((used)) __attribute__((used)) __global__ void k_touch_static_scratch(int v) {
  if (v == 0x7fffffff) scratch[0] = 0;
}

}  // namespace

hipError_t static_scratch(void** ptr, size_t* bytes) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* per_device[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!per_device[dev]) {   // first call on this device, which is the current one
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

hipError_t launch_recv_of_tperm(const int64_t* row_ptr, const int64_t* t_perm, int64_t V, int64_t E, int64_t* t_recv,
                                hipStream_t st) {
  if (E == 0) return hipSuccess;
  hipLaunchKernelGGL(k_recv_of_tperm, dim3(blocks_for(E)), dim3(kBlock), 0, st, row_ptr, t_perm, V, E, t_recv);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  int64_t words = (int64_t)(bytes / 4);
  unsigned nb = (unsigned)std::min<int64_t>((words + kBlock - 1) / kBlock, 65536);
  hipLaunchKernelGGL(k_fill_zero, dim3(nb), dim3(kBlock), 0, st, (uint32_t*)p, words);
  return hipGetLastError();
}

hipError_t launch_add_inplace(void* a, const void* b, int64_t n, bool f64, hipStream_t st) {
  if (n == 0) return hipSuccess;
  unsigned nb = (unsigned)std::min<int64_t>((n + kBlock - 1) / kBlock, 65536);
  if (f64) hipLaunchKernelGGL(k_add_inplace<double>, dim3(nb), dim3(kBlock), 0, st, (double*)a, (const double*)b, n);
  else hipLaunchKernelGGL(k_add_inplace<float>, dim3(nb), dim3(kBlock), 0, st, (float*)a, (const float*)b, n);
  return hipGetLastError();
}

#define CSR_TRY(expr)                \
  do {                               \
    hipError_t e_ = (expr);          \
    if (e_ != hipSuccess) return e_; \
  } while (0)

namespace {

// only the bits a key can have take part in the sorts: recv * V + send < V * V, sender < V
unsigned bits_for(uint64_t max_value) {
  unsigned b = 1;
  while (b < 64 && (max_value >> b) != 0) ++b;
  return b;
}

struct CsrLayout {
  size_t arr = 0, tmp = 0, total = 0;   // one E-sized array (rounded), sort scratch, everything
};

// keys are 32 bits wide whenever recv * V + send fits (V <= 65 536): half the key traffic of every sort pass
bool narrow_keys(int64_t V) { return (uint64_t)V * (uint64_t)V <= ((uint64_t)1 << 32); }

template <class K>
hipError_t sort_scratch_bytes(int64_t E, unsigned bits_rs, unsigned bits_s, size_t& bytes) {
  K *keys_in = nullptr, *keys_out = nullptr;
  int64_t *vals_in = nullptr, *vals_out = nullptr;
  size_t tmp1 = 0, tmp2 = 0;
  CSR_TRY(rocprim::radix_sort_pairs(nullptr, tmp1, keys_in, keys_out, vals_in, vals_out, (size_t)E, 0, bits_rs, (hipStream_t)0));
  CSR_TRY(rocprim::radix_sort_pairs(nullptr, tmp2, keys_in, keys_out, vals_in, vals_out, (size_t)E, 0, bits_s, (hipStream_t)0));
  bytes = std::max(tmp1, tmp2);
  return hipSuccess;
}

hipError_t csr_layout(int64_t E, int64_t V, CsrLayout& L) {
  const unsigned bits_rs = bits_for((uint64_t)V * (uint64_t)V - 1), bits_s = bits_for((uint64_t)(V > 1 ? V - 1 : 1));
  size_t tmp = 0;
  if (narrow_keys(V)) CSR_TRY(sort_scratch_bytes<uint32_t>(E, bits_rs, bits_s, tmp));
  else CSR_TRY(sort_scratch_bytes<uint64_t>(E, bits_rs, bits_s, tmp));
  L.arr = ((size_t)E * 8 + 255) / 256 * 256;
  L.tmp = (tmp + 255) / 256 * 256;
  L.total = 3 * L.arr + 256 + L.tmp;
  return hipSuccess;
}

// the sorts and searches of csr_from_coo_async for one key width
template <class K>
hipError_t csr_build(const int64_t* recv, const int64_t* send, int64_t E, int64_t V, int64_t* row_ptr, int64_t* col, int64_t* perm,
                     int64_t* t_row_ptr, int64_t* t_perm, char* block, const CsrLayout& L, int* bad, hipStream_t st) {
  const bool transpose = t_row_ptr != nullptr;
  const unsigned bits_rs = bits_for((uint64_t)V * (uint64_t)V - 1), bits_s = bits_for((uint64_t)(V > 1 ? V - 1 : 1));
  K* keys_in = (K*)block;   // keys in / out, values in, range-check flag, sort scratch
  K* keys_out = (K*)(block + L.arr);
  int64_t* vals_in = (int64_t*)(block + 2 * L.arr);
  void* tmp = block + 3 * L.arr + 256;
  size_t tmp_bytes = L.tmp;
  hipLaunchKernelGGL(k_make_keys<K>, dim3(blocks_for(E)), dim3(kBlock), 0, st, recv, send, E, V, keys_in, vals_in, bad);
  CSR_TRY(hipGetLastError());
  // stable LSD radix sort: equal (receiver, sender) keep their original order
  CSR_TRY(rocprim::radix_sort_pairs(tmp, tmp_bytes, keys_in, keys_out, vals_in, perm, (size_t)E, 0, bits_rs, st));
  hipLaunchKernelGGL(k_lower_bounds<K>, dim3(blocks_for(V + 1)), dim3(kBlock), 0, st, (const K*)keys_out, E, V, (uint64_t)V, row_ptr);
  CSR_TRY(hipGetLastError());
  // col, and the keys of the transpose: CSR positions stably sorted by sender
  hipLaunchKernelGGL(k_col_from_perm<K>, dim3(blocks_for(E)), dim3(kBlock), 0, st, send, (const int64_t*)perm, E, col, keys_in, vals_in);
  CSR_TRY(hipGetLastError());
  if (transpose) {
    tmp_bytes = L.tmp;
    CSR_TRY(rocprim::radix_sort_pairs(tmp, tmp_bytes, keys_in, keys_out, vals_in, t_perm, (size_t)E, 0, bits_s, st));
    hipLaunchKernelGGL(k_lower_bounds<K>, dim3(blocks_for(V + 1)), dim3(kBlock), 0, st, (const K*)keys_out, E, V, (uint64_t)1, t_row_ptr);
    CSR_TRY(hipGetLastError());
  }
  return hipSuccess;
}

}  // namespace

hipError_t csr_workspace_bytes(int64_t E, int64_t V, size_t* bytes) {
  *bytes = 256;
  if (E <= 0) return hipSuccess;
  CsrLayout L;
  CSR_TRY(csr_layout(E, V, L));
  *bytes = L.total;
  return hipSuccess;
}

// Enqueues everything on `st` and returns: no allocation, no synchronisation.  *bad_flag (device, may be null)
// receives 1 if an index lies outside [0, V), else 0.  t_row_ptr == t_perm == nullptr skips the transpose.
hipError_t csr_from_coo_async(const int64_t* recv, const int64_t* send, int64_t E, int64_t V, int64_t* row_ptr, int64_t* col,
                              int64_t* perm, int64_t* t_row_ptr, int64_t* t_perm, void* workspace, size_t workspace_bytes,
                              int* bad_flag, hipStream_t st) {
  const bool transpose = t_row_ptr != nullptr;
  if (E == 0) {
    CSR_TRY(launch_fill_zero(row_ptr, (size_t)(V + 1) * 8, st));
    if (transpose) CSR_TRY(launch_fill_zero(t_row_ptr, (size_t)(V + 1) * 8, st));
    if (bad_flag) CSR_TRY(launch_fill_zero(bad_flag, 4, st));
    return hipSuccess;
  }
  CsrLayout L;
  CSR_TRY(csr_layout(E, V, L));
  if (!workspace || workspace_bytes < L.total) return hipErrorInvalidValue;
  char* block = (char*)workspace;
  int* bad = bad_flag ? bad_flag : (int*)(block + 3 * L.arr);
  CSR_TRY(launch_fill_zero(bad, 4, st));
  if (narrow_keys(V)) return csr_build<uint32_t>(recv, send, E, V, row_ptr, col, perm, t_row_ptr, t_perm, block, L, bad, st);
  return csr_build<uint64_t>(recv, send, E, V, row_ptr, col, perm, t_row_ptr, t_perm, block, L, bad, st);
}

}  // namespace cgtp
