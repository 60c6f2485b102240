// Fused sweep, MFMA paths (placeholder until the matrix-core kernels land).
#include "bsse_internal.h"

namespace bsse {

bool mfma_supported(int, int, int, int) { return false; }
long long mfma_num_blocks(const GameView &, PathKind, long long) { return 0; }
hipError_t launch_sweep_mfma(const GameView &, PathKind, const SweepArgs &, bool, hipStream_t)
{
    return hipErrorNotSupported;
}
void mfma_pack(int, int, int, int, const float *, const float *, void **Bpack, size_t *Bbytes,
               void **ATpack, size_t *ATbytes, int *, int *)
{
    *Bpack = nullptr; *ATpack = nullptr; *Bbytes = 0; *ATbytes = 0;
}

}  // namespace bsse
