// SDDMM launch entry points: light rows and hub chunks.
#include "launch.h"

namespace autosage {

hipError_t sddmm_rows_f32(const SddmmArgs&, const Resolved&, hipStream_t);
hipError_t sddmm_rows_bf16(const SddmmArgs&, const Resolved&, hipStream_t);
hipError_t sddmm_rows_f16(const SddmmArgs&, const Resolved&, hipStream_t);
hipError_t sddmm_hub_f32(const SddmmArgs&, const Resolved&, const HubMeta&, hipStream_t);
hipError_t sddmm_hub_bf16(const SddmmArgs&, const Resolved&, const HubMeta&, hipStream_t);
hipError_t sddmm_hub_f16(const SddmmArgs&, const Resolved&, const HubMeta&, hipStream_t);

hipError_t launch_sddmm_rows(const SddmmArgs& a, const Resolved& r, hipStream_t stream)
{
    if (a.dt == DT_BF16) return sddmm_rows_bf16(a, r, stream);
    if (a.dt == DT_F16) return sddmm_rows_f16(a, r, stream);
    return sddmm_rows_f32(a, r, stream);
}

hipError_t launch_sddmm_hub(const SddmmArgs& a, const Resolved& r, const HubMeta& meta, hipStream_t stream)
{
    if (meta.cap_hub == 0 || meta.cap_chunks == 0) return hipSuccess;
    if (a.dt == DT_BF16) return sddmm_hub_bf16(a, r, meta, stream);
    if (a.dt == DT_F16) return sddmm_hub_f16(a, r, meta, stream);
    return sddmm_hub_f32(a, r, meta, stream);
}

}  // namespace autosage
