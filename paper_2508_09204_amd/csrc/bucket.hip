// Dispatch counts (the n_i of MoQE Eq. 2), their exclusive prefix sum, and the STABLE
// permutation that makes each expert's samples contiguous.  One work-group.
#include "bucket_device.h"

namespace moqe {

__global__ __launch_bounds__(256) void k_bucket(const int32_t* __restrict__ expert_idx, int S, int K,
                                                 int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                 int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
  bucket_body(expert_idx, S, K, counts, offsets, perm, inv_perm);
}

int32_t launch_bucket(const int32_t* idx, int S, int K, int32_t* counts, int32_t* offsets,
                      int32_t* perm, int32_t* inv_perm, hipStream_t st) {
  ProfileScope ps(MOQE_PK_BUCKET, st);
  hipLaunchKernelGGL(k_bucket, dim3(1), dim3(256), 0, st, idx, S, K, counts, offsets, perm, inv_perm);
  return check_launch("bucket");
}

}  // namespace moqe
