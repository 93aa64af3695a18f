// Internal launch interface between the C ABI (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>

#include "chunkflow.h"

namespace cf {

// Backward scratch inside the caller's workspace:
//   delta     [Hq][T] fp32 = rowsum(dO * O)
//   worklist  bf16 MFMA path only: the dK/dV kernel's work items, written by a small kernel of the same call
//             (layout in attn_mfma_bwd.hip); worklist_items = capacity of its item array
struct BwdWorkspace {
    float *delta;
    int *worklist;
    int64_t worklist_items;
};
// Upper bound on the dK/dV work items of a launch (one item = a key tile and a set of query heads of one group).
int64_t dkv_worklist_capacity(const cf_attn_fwd_params &p);

// One-shot event pair recorded around the main kernel of the next launch on this thread (see
// cf_profile_next_call); both NULL when unset.
struct ProfileHook {
    hipEvent_t start = nullptr, stop = nullptr;
};
ProfileHook take_profile_hook();

// Plain scalar kernels: any supported head_dim, fp32 or bf16 storage, fp32 arithmetic.
hipError_t launch_simple_fwd(const cf_attn_fwd_params &p, hipStream_t s);
hipError_t launch_simple_bwd(const cf_attn_bwd_params &p, const BwdWorkspace &ws, hipStream_t s);

// delta[h][t] = sum_d dO[t][h][d] * O[t][h][d].
hipError_t launch_delta(const cf_attn_bwd_params &p, const BwdWorkspace &ws, hipStream_t s);

// bf16 MFMA kernels, head_dim 128.
hipError_t launch_mfma_fwd(const cf_attn_fwd_params &p, hipStream_t s);
// Forward of 1..CF_FWD_BATCH_MAX chunks as one launch, workgroups dealt in the order of `chunks`.
constexpr int CF_FWD_BATCH_MAX = 16;
hipError_t launch_mfma_fwd_batch(const cf_attn_fwd_params *const *chunks, int n, hipStream_t s);
hipError_t launch_mfma_bwd(const cf_attn_bwd_params &p, const BwdWorkspace &ws, hipStream_t s);
// Backward of 1..CF_BWD_BATCH_MAX chunks: one dQ launch (workgroups dealt in the order dq_order, indices into
// chunks), then the dK/dV kernels in the order of `chunks`.
constexpr int CF_BWD_BATCH_MAX = 8;
hipError_t launch_mfma_bwd_batch(const cf_attn_bwd_params *const *chunks, const BwdWorkspace *ws, const int *dq_order,
                                 int n, hipStream_t s);

}  // namespace cf
