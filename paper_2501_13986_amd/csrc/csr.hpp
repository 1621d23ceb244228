// Host entry points of the statically compiled integer kernels (csr.hip).
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

namespace cgtp {

// COO -> CSR by (receiver, sender, original index) and the transpose permutation.  Device pointers.  Everything is
// enqueued on `st`; nothing is allocated and nothing synchronises.  `workspace` needs csr_workspace_bytes(E, V) bytes.
// *bad_flag (device int, may be null) is set to 1 if any index lies outside [0, V), else to 0.  With
// t_row_ptr == t_perm == nullptr the transpose is skipped.  hipErrorInvalidValue if the workspace is too small.
hipError_t csr_workspace_bytes(int64_t E, int64_t V, size_t* bytes);
hipError_t csr_from_coo_async(const int64_t* recv, const int64_t* send, int64_t E, int64_t V, int64_t* row_ptr, int64_t* col,
                              int64_t* perm, int64_t* t_row_ptr, int64_t* t_perm, void* workspace, size_t workspace_bytes,
                              int* bad_flag, hipStream_t st);

// The library's static device scratch array on the current device (address looked up once per device) and its size.
hipError_t static_scratch(void** ptr, size_t* bytes);

// t_recv[q] = CSR row (receiver) of edge t_perm[q]
hipError_t launch_recv_of_tperm(const int64_t* row_ptr, const int64_t* t_perm, int64_t V, int64_t E, int64_t* t_recv,
                                hipStream_t st);

// zero `bytes` bytes (multiple of 4) with a fill kernel (safe inside graph capture)
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
// a[i] += b[i], i < n (fp32 or fp64)
hipError_t launch_add_inplace(void* a, const void* b, int64_t n, bool f64, hipStream_t st);

}  // namespace cgtp
