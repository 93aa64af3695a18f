#include "kernels.h"
namespace cf {
hipError_t launch_mfma_bwd(const cf_attn_bwd_params &p, const BwdWorkspace &ws, hipStream_t s) { return launch_simple_bwd(p, ws, s); }
}
