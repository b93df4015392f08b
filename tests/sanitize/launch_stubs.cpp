// Stand-ins for the kernel launchers of libtidal in the host-only sanitizer build: the driver never
// reaches a launch (there is no GPU in that run), so each one only reports that.
#include "tidal_internal.h"

namespace tidal {
hipError_t launch_convert(const ConvertBatch&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_slot_checksum(const void*, int64_t, int, void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_rmw_probe(void*, int64_t, int64_t, int64_t, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_pack(const PackBatch&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_copy_from_host(const CopyBatch&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_lora_mfma(const LoraGroup&, const LoraLaunchPlan&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_lora_mfma_lds(const LoraGroup&, const LoraLaunchPlan&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_lora_ordered(const LoraGroup&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_convert_merge(const FusedPiece&, bool, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_apply_shrink(const ApplyLongBatch&, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_apply_expand(const ApplyLongBatch&, int, int, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_apply_fused(const ApplyLongBatch&, int, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_apply_ordered(const ApplyLongBatch&, int, bool, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_apply_shrink_short(const ApplyShortBatch&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_apply_expand_short(const ApplyShortBatch&, int, hipStream_t) { return hipErrorNotSupported; }
}  // namespace tidal
