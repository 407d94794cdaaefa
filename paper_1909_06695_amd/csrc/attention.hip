// Dispatch between the MFMA attention kernels and the general per-row kernels.
#include "common.h"

namespace ouro {

hipError_t launch_attn_fwd_plain(hipStream_t s, int dtype, const AttnDesc& a);
hipError_t launch_attn_bwd_plain(hipStream_t s, int dtype, const AttnDesc& a);
bool attn_mfma_ok(int dtype, const AttnDesc& a);
hipError_t launch_attn_fwd_mfma(hipStream_t s, const AttnDesc& a);
hipError_t launch_attn_bwd_mfma(hipStream_t s, const AttnDesc& a);
bool attn_xl_ok(int dtype, const AttnDesc& a);
hipError_t launch_attn_fwd_xl(hipStream_t s, const AttnDesc& a);
hipError_t launch_attn_bwd_xl(hipStream_t s, const AttnDesc& a);

hipError_t launch_attn_fwd(hipStream_t s, int dtype, const AttnDesc& a, int force_generic) {
  if (!force_generic && attn_mfma_ok(dtype, a)) return launch_attn_fwd_mfma(s, a);
  if (!force_generic && attn_xl_ok(dtype, a)) return launch_attn_fwd_xl(s, a);
  return launch_attn_fwd_plain(s, dtype, a);
}
hipError_t launch_attn_bwd(hipStream_t s, int dtype, const AttnDesc& a, int force_generic) {
  if (!force_generic && attn_mfma_ok(dtype, a)) return launch_attn_bwd_mfma(s, a);
  if (!force_generic && attn_xl_ok(dtype, a) && a.du && a.dvb && a.dr) return launch_attn_bwd_xl(s, a);
  return launch_attn_bwd_plain(s, dtype, a);
}

}  // namespace ouro
