// Matrix-core kernels of the bf16 mode.
#include "mfma.hpp"

namespace sdlm {

bool mfma_supported(const sdlm_model_cfg *) { return false; }
size_t mfma_pad_n(size_t N) { return (N + 31) / 32 * 32; }
size_t mfma_packed_elems(bool packed, size_t N, size_t K) { return (packed ? mfma_pad_n(N) : N) * K; }
size_t mfma_attn_scratch_bytes(const sdlm_model_cfg *, const sdlm_run_cfg *, int) { return 256; }
void launch_pack_mfma(hipStream_t, void *, const void *, int, int, int, int, int) {}
void launch_gemm_mfma(hipStream_t, int, const GemmArgs &) {}
void launch_attn_mfma(hipStream_t, const void *, void *, const void *, const KvGeom &, const RowMeta &, const SeqState &, int, int, int, void *) {}
void launch_lmhead_mfma(hipStream_t, const void *, const void *, int, int, int, float, int, float *, void *, int32_t *, float *) {}

}  // namespace sdlm
