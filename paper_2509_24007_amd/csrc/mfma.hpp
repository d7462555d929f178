// Matrix-core (MFMA) kernels of the bf16 mode: declarations.
#pragma once
#include "internal.hpp"

namespace sdlm {

// True when the bf16 matrix-core path serves this model (bf16, head_dim 128, sizes multiples of the tile steps).
bool mfma_supported(const sdlm_model_cfg *m);
// Rows of a packed weight matrix are padded to a multiple of the 32-row tile.
size_t mfma_pad_n(size_t N);
// Elements a packed [N, K] matrix occupies (N * K when `packed` is false).
size_t mfma_packed_elems(bool packed, size_t N, size_t K);
// Bytes of scratch the split-KV attention needs for its per-chunk partial results.
size_t mfma_attn_scratch_bytes(const sdlm_model_cfg *m, const sdlm_run_cfg *r, int max_rows);
// Bytes of scratch for the LM head's per-vocabulary-block partials.
size_t mfma_lm_scratch_bytes(int V, int max_rows);
// Smallest KV chunk (in 16-key tiles) the attention launch over `groups` row groups may use with this much scratch.
int mfma_attn_chunk_floor(const sdlm_model_cfg *m, int max_seq_len, int groups, size_t scratch_bytes);
// Rows of one sequence that form one attention work item (rows x query heads per kv head <= 64).
int mfma_group_rows(const sdlm_model_cfg *m);

// Repack rows of a row-major [N, K] bf16 matrix into tile order at row offset dst_row0 of a packed matrix with
// dst_rows rows.  interleave: 0 plain; 1 / 2: the matrix is the gate / up half of the fused gate-up matrix,
// whose 32-row tiles alternate gate, up.
void launch_pack_mfma(hipStream_t s, void *dst, const void *src, int N, int K, int dst_row0, int dst_rows, int interleave);
// The launch shape launch_gemm_mfma would take (host logic only): row-tile height in 32-row units, 32-column bands per
// wavefront, number of k splits, wavefronts per workgroup (a workgroup's tile is 32 MT rows x 32 NT wavefronts columns).
void mfma_gemm_plan(int epi, int rows, int min_rows, int N, int K, size_t slab_room_floats, int *MT, int *NT, int *splits, int *wavefronts);
// Returns the number of split-k slabs written to `slabs` (1: the result is complete in a.Yf / a.Yt).  For
// EPI_STORE_F32 the consumer always adds the slabs; for EPI_RESID the slabs are added to a.Yf here unless
// defer_reduce, in which case the next RMSNorm adds them (slab stride = a.max_rows * a.N floats).
int launch_gemm_mfma(hipStream_t s, int epi, const GemmArgs &a, float *slabs, size_t slab_room_floats, bool defer_reduce);
// part 0: the attention kernel; part 1: the merge of the split-KV partials (a no-op when the launch has a single
// chunk).  Returns whether the launch shape needs the merge.  two_staging: row groups of this pass may read a second
// staging tile (a verification pass whose rows do not fit one tile).
bool launch_attn_mfma(hipStream_t s, const sdlm_model_cfg *m, int max_seq_len, const void *q, void *out, const void *pool_layer,
                      const KvGeom &kg, const RowMeta &rm, const SeqState &st, int D, int max_groups, void *scratch, size_t scratch_bytes,
                      int part, bool two_staging);
// Steps of at most 32 rows: QKV projection, rotation and K/V placement in one launch (same results as the projection
// followed by the RoPE + K/V placement kernel, up to the order in which the k partial sums are added).
bool qkv_rope_skinny_applies(const sdlm_model_cfg *m, int max_rows);
void launch_qkv_rope_skinny(hipStream_t s, const sdlm_model_cfg *m, const void *X, const void *w_packed, const void *bias, const int32_t *p_rows,
                            int max_rows, void *q_out, void *pool_layer, const KvGeom &kg, const RowMeta &rm, const SeqState &st, const float2 *rope);
void launch_lmhead_mfma(hipStream_t s, const void *xhat, const void *w_packed, const int32_t *p_rows, int max_rows, int min_rows, int V, int h,
                        float scale, int conf_fn, float *logits_out, void *scratch, int32_t *ids, float *conf);

}  // namespace sdlm
