#include "kernels.h"
namespace cf {
hipError_t launch_mfma_fwd(const cf_attn_fwd_params &p, hipStream_t s) { return launch_simple_fwd(p, s); }
}
