// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "sdlm.h"

namespace sdlm {

constexpr int PAGE = 16;        // tokens per K/V tile (page)
constexpr int GROUP_ROWS = 16;  // most rows of one sequence handled together by one attention work item
constexpr int MAX_D = 16;

typedef uint16_t bf16_t;        // bf16 bit pattern

__host__ __device__ inline float bf16_to_f(bf16_t v)
{
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)v << 16;
    return c.f;
}
__host__ __device__ inline bf16_t f_to_bf16(float f)   // round to nearest even
{
    union { uint32_t u; float f; } c;
    c.f = f;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((c.u >> 16) | 0x40);   // NaN stays NaN
    c.u += 0x7fffu + ((c.u >> 16) & 1u);
    return (bf16_t)(c.u >> 16);
}

// two floats -> packed bf16 pair with the hardware conversion (round to nearest even)
typedef __attribute__((ext_vector_type(2))) float sdlm_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 sdlm_bf16x2;
__device__ inline uint32_t pack_bf16(float lo, float hi)
{
    sdlm_f32x2 v = {lo, hi};
    sdlm_bf16x2 b = __builtin_convertvector(v, sdlm_bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

template <typename T> __device__ inline float to_f(T v);
template <> __device__ inline float to_f<float>(float v) { return v; }
template <> __device__ inline float to_f<bf16_t>(bf16_t v) { return bf16_to_f(v); }
template <typename T> __device__ inline T from_f(float v);
template <> __device__ inline float from_f<float>(float v) { return v; }
template <> __device__ inline bf16_t from_f<bf16_t>(float v) { return f_to_bf16(v); }

// ---- K/V tile layout -------------------------------------------------------------------------------------
// The cache is a pool of tiles.  One tile holds 16 consecutive positions of one (layer, kv head): first a K
// block then a V block of 16*d elements each.  Inside the blocks the elements are ordered the way the
// matrix-core attention kernel consumes them, so that a wavefront's operand load is one contiguous run:
//   K block: [d/8][16 slots][8]        element (slot, i) at (i/8)*128 + slot*8 + i%8
//   V block: [d/16][4][16][4 slots]    element (slot, i) at ((i/16)*4 + slot/4)*64 + (i%16)*4 + slot%4
// Pool order: [layer][tile][kv head][K block | V block].  Tiles n_pages .. n_pages+max_batch-1 of every layer
// are the per-sequence staging tiles that hold the D block rows' K/V during a step; the staging tiles of a
// verification pass follow them.
__host__ __device__ inline int k_off(int slot, int i) { return (i >> 3) * (PAGE * 8) + slot * 8 + (i & 7); }
__host__ __device__ inline int v_off(int slot, int i) { return (((i >> 4) << 2) + (slot >> 2)) * 64 + ((i & 15) << 2) + (slot & 3); }

// Tiles per KV chunk for an attention launch whose (row group, kv head) items cover `item_pages` 16-key tiles in all:
// large enough that the launch has about 2.25 work items per compute unit (measured by whole-step time on the 7B and 32B
// shapes, batch 64 and 32: all work items resident at once, two to three per unit, is the fastest split; finer chunks
// add partial results to merge, coarser ones leave the units unevenly loaded),
// a multiple of 8, and never below `floor_pages` (the host's bound: partial-result scratch, 64 chunks per item).
__host__ __device__ inline int attn_chunk_pages(long item_pages, int floor_pages)
{
    long cp = (item_pages + 575) / 576;
    cp = (cp + 7) / 8 * 8;
    return cp > floor_pages ? (int)cp : floor_pages;
}

__host__ __device__ inline int attn_group_hint(int max_lim, int rows, int chunk_pages)
{
    int pages = (max_lim + PAGE - 1) / PAGE, chunks = (pages + chunk_pages - 1) / chunk_pages;
    return (chunks < 1 ? 1 : chunks > 255 ? 255 : chunks) | rows << 8;
}

// Packed description of the rows of one forward pass (device arrays).
struct RowMeta {
    int32_t *tok, *pos, *seq, *kind, *lim;  // [max_rows]; kind: -1 = K/V go to the cache slot of pos, else the slot in the
                                            // row's staging tile; lim: visible cache keys [0, lim)
    int32_t *stg, *smask;                   // [max_rows]; staging tile of the row (-1: none): its K/V go to slot `kind` of it; bits 0..15
                                            // of smask: the slots of that tile the row sees; bits 16..31: the slots it sees of stg2
    int32_t *stg2;                          // [max_rows]; a second staging tile the row reads (-1: none): the shared causal rows of a
                                            // verification pass
    int32_t *grp_row0, *grp_n, *grp_seq;    // [max_groups]: runs of <= GROUP_ROWS rows of one sequence that share their staging tiles
    int32_t *grp_stg, *grp_stg2;            // [max_groups]: those tiles (-1: none)
    int32_t *grp_hint;                      // [max_groups]: KV chunks of the group's attention work (bits 0..7) and its rows (bits 8..15); lets
                                            // the merge kernel request exactly the partial results that exist before it has looked the group up
    int32_t *blk_row;                       // [max_batch*D]: packed row index of the rows that go through the LM head
    int32_t *counts;                        // [4]: rows R, groups, LM-head rows, tiles per KV chunk of the attention launch
};

// Per-sequence state (device arrays).
struct SeqState {
    int32_t *n, *c, *last_tok;      // [B]
    int32_t *pend_tok;              // [B][D]: tokens at positions c..n-1
    int32_t *page_table;            // [B][pages_per_seq]
    int32_t *pages_backed;          // [B]
    int32_t *alloc;                 // [0] next free page, [1] error bits (1: pool exhausted, 2: count clamped, 4: bad override id)
    int32_t *last_ids, *last_count; // [B][D], [B]: the last step's result
};

struct KvGeom {
    int32_t n_kv_heads, head_dim, pages_per_seq, staging_base;  // staging tile of sequence b = staging_base + b; D tiles per
                                                                 // sequence for a verification pass follow at staging_base + B + b D
    size_t layer_stride;                                         // elements per layer of the pool
    __host__ __device__ size_t tile(int page, int kvh) const { return ((size_t)page * n_kv_heads + kvh) * (size_t)(2 * PAGE * head_dim); }
};

// ---- kernel launchers (generic kernels: any supported shape, fp32 or bf16 storage, fp32 arithmetic) ----------
enum GemmEpi { EPI_STORE_F32 = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct GemmArgs {
    const void *X;      // [R, K] elem
    const void *W;      // [N, K] elem
    const void *W2;     // second matrix for EPI_SWIGLU (up projection)
    const void *bias;   // [N] elem or null
    float *Yf;          // fp32 destination (STORE_F32 / RESID / LOGITS)
    void *Yt;           // elem destination (SWIGLU)
    const int32_t *pR;  // device row count
    int max_rows, N, K;
    float scale;
    int min_rows;       // host-known lower bound of the device row count (0: unknown); only steers the launch shape
};

void launch_assemble_decode(hipStream_t s, const SeqState &st, const RowMeta &rm, int B, int D, int mask_id, int group_rows,
                            int staging_base, int causal, int n_kv_heads, int chunk_floor);
// Rows one sequence contributes to a verification pass, (D-2) causal rows + (D-1) D block rows, and whether they share
// one staging tile (they fit its 16 slots: D <= 4) or take one tile per input plus one for the causal rows.
int verify_rows_per_seq(int D, bool *shared_tile);
// Row groups of those rows for groups of at most `gr` rows (one tile: consecutive runs; else the causal rows and every
// input's block are grouped on their own).
__host__ __device__ inline int verify_groups_per_seq(int D, int gr)
{
    if (D < 2) return 0;
    const int rows = (D - 2) + (D - 1) * D;
    if (rows <= PAGE) return (rows + gr - 1) / gr;
    return (D - 2 + gr - 1) / gr + (D - 1) * ((D + gr - 1) / gr);
}
void launch_assemble_verify(hipStream_t s, const SeqState &st, const RowMeta &rm, int B, int D, int mask_id, int group_rows,
                            int staging_base, int causal, int n_kv_heads, int chunk_floor);
void launch_verify_accept(hipStream_t s, const SeqState &st, const int32_t *ids_rows, int B, int D, int rule,
                          int32_t *ids_out, int32_t *count_out);
void launch_embed(hipStream_t s, int dtype, float *x, const void *E, const RowMeta &rm, int max_rows, int h, int V);
void launch_rmsnorm(hipStream_t s, int dtype, void *out, float *x, const void *g, int h, float eps, const int32_t *row_index,
                    const int32_t *p_count, int max_rows, int min_rows, const float *slabs, int n_slabs, size_t slab_stride);   // min_rows: rows that certainly exist
void launch_gemm_generic(hipStream_t s, int dtype, int epi, const GemmArgs &a);
void launch_rope_scatter(hipStream_t s, int dtype, const float *qkv, int n_slabs, size_t slab_stride, void *q_out, void *pool_layer,
                         const KvGeom &kg, const RowMeta &rm, const SeqState &st, const float2 *rope, int n_q_heads, int max_rows, int min_rows);
void launch_attn_generic(hipStream_t s, int dtype, const void *q, void *out, const void *pool_layer, const KvGeom &kg,
                         const RowMeta &rm, const SeqState &st, int n_q_heads, int max_rows);
void launch_lm_reduce(hipStream_t s, const float *logits, int V, int32_t *ids, float *conf, int conf_fn,
                      const int32_t *p_rows, int max_rows);
void launch_accept(hipStream_t s, const SeqState &st, const int32_t *ids_rows, const float *conf_rows, int B, int D,
                   float tau, int rule, int32_t *ids_out, int32_t *count_out, float *conf_out);
void launch_commit(hipStream_t s, const SeqState &st, int B, int D, const int32_t *ids_ovr, const int32_t *cnt_ovr,
                   int paged, int n_pages, int pages_per_seq, int V);
void launch_read_kv(hipStream_t s, int dtype, const void *pool_layer, const KvGeom &kg, const SeqState &st, int seq,
                    int kvh, int pos0, int count, float *k_out, float *v_out);

}  // namespace sdlm
