// placeholder until the MFMA kernels land
#include "common.h"
namespace dlcx {
int launch_project_p_mfma(int, int64_t, int64_t, int, int, const PtrPack<const float *> &,
                          const float *, const PtrPack<float *> &, void *, hipStream_t) { return DLCX_EUNSUPPORTED; }
int launch_project_q_mfma(int, int64_t, int64_t, int, int, const PtrPack<const float *> &,
                          const float *, const PtrPack<float *> &, void *, hipStream_t) { return DLCX_EUNSUPPORTED; }
int launch_reconstruct_mfma(int, int64_t, int64_t, int, const float *, const float *, float *, int,
                            const PtrPack<float *> &, hipStream_t) { return DLCX_EUNSUPPORTED; }
size_t mfma_project_workspace_bytes(int, int64_t, int64_t, int, int) { return 0; }
}
