// BLAST fused kernels (placeholder until implemented).
#include "blr_common.h"
namespace blr {
bool blast_fused_supported(int64_t, int, int, int) { return false; }
hipError_t launch_blast_stage12(const void*, const void*, const void*, void*, int64_t, int, int, int, hipStream_t) { return hipErrorNotSupported; }
bool blast_full_fusion_supported(int64_t, int, int, int, int) { return false; }
hipError_t launch_blast_full(const void*, const void*, const void*, const void*, void*, int64_t, int, int, int, int, hipStream_t) { return hipErrorNotSupported; }
}
