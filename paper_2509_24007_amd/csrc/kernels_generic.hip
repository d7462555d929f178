// Shape-generic kernels of the block-decode step: row assembly, embedding gather, RMSNorm, a tiled FMA GEMM with
// fused epilogues, RoPE + K/V placement, block-masked attention, the vocabulary reduction, prefix acceptance
// and commit.  Storage is fp32 or bf16; all arithmetic is fp32.  They serve the fp32 debug mode and every small
// integer/elementwise step of the bf16 mode; the bf16 mode's contractions run on the matrix-core kernels.
#include "internal.hpp"

namespace sdlm {

// ------------------------------------------------------------------------------------------------ row assembly
// Rows of a decode step, per sequence: the pending tokens (positions c..n-1, causal), then the block
// [x_last, [m] x (D-1)] at positions n-1 .. n+D-2 (block definition, Sec. 3.2).  A block row may see the cache
// below position s = n-1 only; the causal copy of x_last at s is for later steps.
__global__ void assemble_decode_k(SeqState st, RowMeta rm, int B, int D, int mask_id, int gr, int stg0, int causal, int Hkv, int cp_floor)
{
    __shared__ int row0[1025], grp0[1025], cp_s;
    if (threadIdx.x == 0) {
        int r = 0, g = 0;
        long tiles = 0;   // 16-key tiles the attention's work items stream, per kv head
        for (int b = 0; b < B; ++b) {
            row0[b] = r; grp0[b] = g;
            int rows = st.n[b] - st.c[b] + D, ng = (rows + gr - 1) / gr;
            r += rows;
            g += ng;
            tiles += (long)ng * ((st.n[b] + PAGE - 1) / PAGE);
        }
        row0[B] = r; grp0[B] = g;
        cp_s = attn_chunk_pages(tiles * Hkv, cp_floor);
        rm.counts[0] = r; rm.counts[1] = g; rm.counts[2] = B * D; rm.counts[3] = cp_s;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        int n = st.n[b], c = st.c[b], p = n - c, r = row0[b];
        for (int i = 0; i < p; ++i, ++r) {
            rm.tok[r] = st.pend_tok[b * D + i];
            rm.pos[r] = c + i; rm.seq[r] = b; rm.kind[r] = -1; rm.lim[r] = c + i + 1;
            rm.stg[r] = -1; rm.smask[r] = 0; rm.stg2[r] = -1;
        }
        for (int j = 0; j < D; ++j, ++r) {
            rm.tok[r] = j == 0 ? st.last_tok[b] : mask_id;
            rm.pos[r] = n - 1 + j; rm.seq[r] = b; rm.kind[r] = j; rm.lim[r] = n - 1;
            rm.stg[r] = stg0 + b; rm.smask[r] = (1 << (causal ? j + 1 : D)) - 1;   // block keys: all D, or (causal variant) up to the row itself
            rm.stg2[r] = -1;
            rm.blk_row[b * D + j] = r;
        }
        int rows = p + D, g = grp0[b];
        for (int o = 0; o < rows; o += gr, ++g) {
            const int gn = min(gr, rows - o);
            rm.grp_row0[g] = row0[b] + o;
            rm.grp_n[g] = gn;
            rm.grp_seq[g] = b;
            rm.grp_stg[g] = stg0 + b;
            rm.grp_stg2[g] = -1;
            // largest visible-key limit of the group's rows: pending row i has c + i + 1, block rows n - 1
            const int last = o + gn - 1, lim_max = o < p ? c + min(last, p - 1) + 1 : n - 1;
            rm.grp_hint[g] = attn_group_hint(lim_max, gn, cp_s);
        }
    }
}

void launch_assemble_decode(hipStream_t s, const SeqState &st, const RowMeta &rm, int B, int D, int mask_id, int group_rows, int staging_base,
                            int causal, int n_kv_heads, int chunk_floor)
{
    hipLaunchKernelGGL(assemble_decode_k, dim3(1), dim3(256), 0, s, st, rm, B, D, mask_id, group_rows, staging_base, causal, n_kv_heads, chunk_floor);
}

// Rows of the verification pass of a self-speculative step (Sec. 3.4, "Self-Speculative Decoding").  With yhat^1..yhat^D
// the tokens of the step just computed and n the number of known tokens, verification input j (j = 2..D; input 1 is
// the step itself) is the sequence extended by yhat^1..yhat^{j-1}:
//   j-2 causal rows   yhat^1..yhat^{j-2} at positions n..n+j-3
//   D block rows      [yhat^{j-1}, [m] x (D-1)] at positions n+j-2 ..
// All of them see the cache keys [0, n) (written by the step: every known token including x_last has its causal K/V
// there) and keep their own K/V in staging tiles; nothing is written to the cache.  The causal row of yhat^i is the
// same in every input that has it (same token, same position, same visible keys), so it is computed once per sequence:
// a sequence contributes its D-2 causal rows, then the D block rows of each input, (D-2) + (D-1) D rows in all.  Only the
// first block row of each input goes through the LM head: its arg-max is ytilde^j.
//   shared != 0 (all those rows fit the 16 slots of one tile, D <= 4): one tile per sequence; the causal rows sit in slots
//     0 .. D-3, input j's block in slots D-2 + (j-2) D ..., and its rows see the causal slots 0 .. j-3 and their own block.
//     The rows of a sequence then form row groups regardless of the input they belong to.
//   shared == 0: the causal rows live in a tile of their own (the sequence's last staging tile), every input's block in the
//     input's tile; a block row reads two staging tiles, its input's (slots 0 .. D-1) and the causal one (slots 0 .. j-3,
//     upper half of its slot mask).  Row groups do not straddle inputs, so a group reads at most these two tiles.
__global__ void assemble_verify_k(SeqState st, RowMeta rm, int B, int D, int mask_id, int gr, int stg0, int causal, int shared, int Hkv, int cp_floor)
{
    __shared__ int row0[1025], grp0[1025], cp_s;
    const int rows_seq = (D - 2) + (D - 1) * D;
    const int groups_seq = verify_groups_per_seq(D, gr);
    if (threadIdx.x == 0) {
        long tiles = 0;
        for (int b = 0; b < B; ++b) {
            row0[b] = b * rows_seq; grp0[b] = b * groups_seq;
            tiles += (long)groups_seq * ((st.n[b] + PAGE - 1) / PAGE);
        }
        rm.counts[0] = B * rows_seq; rm.counts[1] = B * groups_seq; rm.counts[2] = B * (D - 1);
        cp_s = attn_chunk_pages(tiles * Hkv, cp_floor);
        rm.counts[3] = cp_s;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const int n = st.n[b];
        const int32_t *yhat = st.last_ids + b * D;
        int r = row0[b], g = grp0[b];
        if (shared) {
            const int tile = stg0 + B + b * D;
            for (int i = 0; i < D - 2; ++i, ++r) {
                rm.tok[r] = yhat[i]; rm.pos[r] = n + i; rm.seq[r] = b; rm.kind[r] = i; rm.lim[r] = n;
                rm.stg[r] = tile; rm.smask[r] = (1 << (i + 1)) - 1; rm.stg2[r] = -1;
            }
            for (int j = 2; j <= D; ++j) {
                const int base = (D - 2) + (j - 2) * D, common = (1 << (j - 2)) - 1;
                for (int t = 0; t < D; ++t, ++r) {
                    rm.tok[r] = t == 0 ? yhat[j - 2] : mask_id; rm.pos[r] = n + j - 2 + t; rm.seq[r] = b; rm.kind[r] = base + t;
                    rm.lim[r] = n; rm.stg[r] = tile; rm.smask[r] = common | (((1 << (causal ? t + 1 : D)) - 1) << base); rm.stg2[r] = -1;
                    if (t == 0) rm.blk_row[b * (D - 1) + (j - 2)] = r;
                }
            }
            for (int o = 0; o < rows_seq; o += gr, ++g) {
                rm.grp_row0[g] = row0[b] + o;
                rm.grp_n[g] = min(gr, rows_seq - o);
                rm.grp_seq[g] = b;
                rm.grp_stg[g] = tile; rm.grp_stg2[g] = -1;
                rm.grp_hint[g] = attn_group_hint(n, min(gr, rows_seq - o), cp_s);
            }
            continue;
        }
        // tiles of sequence b: stg0 + B + b D + (j - 2) for input j, and stg0 + B + b D + (D - 1) for the causal rows
        const int ctile = stg0 + B + b * D + (D - 1);
        for (int i = 0; i < D - 2; ++i, ++r) {
            rm.tok[r] = yhat[i]; rm.pos[r] = n + i; rm.seq[r] = b; rm.kind[r] = i; rm.lim[r] = n;
            rm.stg[r] = ctile; rm.smask[r] = (1 << (i + 1)) - 1; rm.stg2[r] = -1;
        }
        for (int o = 0; o < D - 2; o += gr, ++g) {
            rm.grp_row0[g] = row0[b] + o;
            rm.grp_n[g] = min(gr, D - 2 - o);
            rm.grp_seq[g] = b;
            rm.grp_stg[g] = ctile; rm.grp_stg2[g] = -1;
            rm.grp_hint[g] = attn_group_hint(n, min(gr, D - 2 - o), cp_s);
        }
        for (int j = 2; j <= D; ++j) {
            const int tile = stg0 + B + b * D + (j - 2), first = r;
            const int common = (1 << (j - 2)) - 1;   // causal slots 0 .. j-3 of the causal tile
            for (int t = 0; t < D; ++t, ++r) {
                rm.tok[r] = t == 0 ? yhat[j - 2] : mask_id; rm.pos[r] = n + j - 2 + t; rm.seq[r] = b; rm.kind[r] = t;
                rm.lim[r] = n; rm.stg[r] = tile; rm.stg2[r] = common ? ctile : -1;
                rm.smask[r] = (int32_t)((uint32_t)((1 << (causal ? t + 1 : D)) - 1) | ((uint32_t)common << 16));
                if (t == 0) rm.blk_row[b * (D - 1) + (j - 2)] = r;
            }
            for (int o = 0; o < D; o += gr, ++g) {
                rm.grp_row0[g] = first + o;
                rm.grp_n[g] = min(gr, D - o);
                rm.grp_seq[g] = b;
                rm.grp_stg[g] = tile; rm.grp_stg2[g] = common ? ctile : -1;
                rm.grp_hint[g] = attn_group_hint(n, min(gr, D - o), cp_s);
            }
        }
    }
}

int verify_rows_per_seq(int D, bool *shared_tile)
{
    if (D < 2) { if (shared_tile) *shared_tile = true; return 0; }
    if (shared_tile) *shared_tile = (D - 2) + (D - 1) * D <= PAGE;   // every row of a sequence fits one staging tile
    return (D - 2) + (D - 1) * D;
}

void launch_assemble_verify(hipStream_t s, const SeqState &st, const RowMeta &rm, int B, int D, int mask_id, int group_rows,
                            int staging_base, int causal, int n_kv_heads, int chunk_floor)
{
    bool shared;
    verify_rows_per_seq(D, &shared);
    hipLaunchKernelGGL(assemble_verify_k, dim3(1), dim3(256), 0, s, st, rm, B, D, mask_id, group_rows, staging_base, causal, shared ? 1 : 0, n_kv_heads,
                       chunk_floor);
}

// gamma_verify (Eq. 10) from the step's tokens yhat and the verification predictions (ids_rows: ytilde^2..ytilde^D per
// sequence; ytilde^1 = yhat^1 because input 1 is the step itself).  rule 0: longest prefix on which all positions
// agree; rule 1: the largest agreeing index, as the equation is printed.  The result replaces the step's own count,
// so that a commit without overrides publishes the verified tokens.
__global__ void verify_accept_k(SeqState st, const int32_t *ids_rows, int B, int D, int rule, int32_t *ids_out, int32_t *count_out)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t *yhat = st.last_ids + b * D;
    int best = 1;
    bool run = true;
    for (int j = 1; j <= D; ++j) {
        int yt = j == 1 ? yhat[0] : ids_rows[b * (D - 1) + (j - 2)];
        if (ids_out) ids_out[b * D + j - 1] = yt;
        bool eq = yt == yhat[j - 1];
        run = run && eq;
        if (rule == 1 ? eq : run) best = j;
    }
    st.last_count[b] = best;
    if (count_out) count_out[b] = best;
}

void launch_verify_accept(hipStream_t s, const SeqState &st, const int32_t *ids_rows, int B, int D, int rule,
                          int32_t *ids_out, int32_t *count_out)
{
    hipLaunchKernelGGL(verify_accept_k, dim3((B + 63) / 64), dim3(64), 0, s, st, ids_rows, B, D, rule, ids_out, count_out);
}

// ------------------------------------------------------------------------------------------------ embedding
template <typename T>
__global__ void embed_k(float *x, const T *E, const int32_t *tok, const int32_t *pR, int h, int V)
{
    int r = blockIdx.x;
    if (r >= *pR) return;
    const T *e = E + (size_t)min(max(tok[r], 0), V - 1) * h;
    for (int k = threadIdx.x; k < h; k += blockDim.x) x[(size_t)r * h + k] = to_f<T>(e[k]);
}

void launch_embed(hipStream_t s, int dtype, float *x, const void *E, const RowMeta &rm, int max_rows, int h, int V)
{
    if (dtype == 0) hipLaunchKernelGGL(embed_k<float>, dim3(max_rows), dim3(256), 0, s, x, (const float *)E, rm.tok, rm.counts, h, V);
    else hipLaunchKernelGGL(embed_k<bf16_t>, dim3(max_rows), dim3(256), 0, s, x, (const bf16_t *)E, rm.tok, rm.counts, h, V);
}

// ------------------------------------------------------------------------------------------------ RMSNorm
__device__ inline float block_sum(float v, float *red)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += red[i];
    return t;
}

// out[j,:] = x[row,:] * g / sqrt(mean(x[row,:]^2) + eps), row = row_index ? row_index[j] : j.  When the projection
// that produced the residual update was split along k, its partial sums (n_slabs slabs of [rows, h]) are first added
// to x[row,:] in slab order and written back, so the residual stream is complete after this kernel.
// A row lives in registers between the two passes (NV float4 per thread, h <= 1024 NV).
template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_k(T *out, float *x, const T *g, int h, float eps, const int32_t *row_index,
                                                 const int32_t *p_count, int sure, const float *slabs, int n_slabs, size_t slab_stride)
{
    __shared__ float red[4];
    const int j = blockIdx.x;
    if (j >= sure && j >= *p_count) return;   // the first `sure` rows exist for certain: no wait for the device count
    const int row = row_index ? row_index[j] : j;
    float *xr = x + (size_t)row * h;
    float4 v[NV], gv[NV];   // the gains are requested together with the row, not after the reduction
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = (i * 256 + threadIdx.x) * 4;
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        gv[i] = v[i];
        if (k < h) {
            v[i] = *(const float4 *)(xr + k);
            if constexpr (sizeof(T) == 2) {
                const uint2 u = *(const uint2 *)(g + k);
                gv[i] = make_float4(bf16_to_f((bf16_t)(u.x & 0xffff)), bf16_to_f((bf16_t)(u.x >> 16)),
                                    bf16_to_f((bf16_t)(u.y & 0xffff)), bf16_to_f((bf16_t)(u.y >> 16)));
            } else {
                gv[i] = *(const float4 *)(g + k);
            }
        }
    }
    // The slabs are added in slab order, but requested SU at a time (as many as the registers of the row width allow): one
    // memory round trip per SU slabs instead of one per slab.  A slab index past the end is clamped for the load (a valid address, a cache hit) and its add skipped.
    constexpr int SU = NV <= 2 ? 8 : (NV <= 4 ? 4 : (NV == 8 ? 2 : 1));
    for (int s0 = 0; s0 < n_slabs; s0 += SU) {
        float4 p[SU][NV];
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int sl = min(s0 + u, n_slabs - 1);
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int k = (i * 256 + threadIdx.x) * 4;
                p[u][i] = k < h ? *(const float4 *)(slabs + sl * slab_stride + (size_t)row * h + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            if (s0 + u < n_slabs) {
#pragma unroll
                for (int i = 0; i < NV; ++i) { v[i].x += p[u][i].x; v[i].y += p[u][i].y; v[i].z += p[u][i].z; v[i].w += p[u][i].w; }
            }
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = (i * 256 + threadIdx.x) * 4;
        if (k < h && n_slabs > 0) *(float4 *)(xr + k) = v[i];
        ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    }
    ss = block_sum(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)h + eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = (i * 256 + threadIdx.x) * 4;
        if (k >= h) continue;
        const float o0 = v[i].x * inv * gv[i].x, o1 = v[i].y * inv * gv[i].y;
        const float o2 = v[i].z * inv * gv[i].z, o3 = v[i].w * inv * gv[i].w;
        T *dst = out + (size_t)j * h + k;
        if constexpr (sizeof(T) == 2) {
            *(uint2 *)dst = make_uint2((uint32_t)f_to_bf16(o0) | ((uint32_t)f_to_bf16(o1) << 16),
                                       (uint32_t)f_to_bf16(o2) | ((uint32_t)f_to_bf16(o3) << 16));
        } else {
            *(float4 *)dst = make_float4(o0, o1, o2, o3);
        }
    }
}

template <typename T>
static void rmsnorm_t(hipStream_t s, void *out, float *x, const void *g, int h, float eps, const int32_t *row_index,
                      const int32_t *p_count, int max_rows, int min_rows, const float *slabs, int n_slabs, size_t slab_stride)
{
#define SDLM_RMS(NV) hipLaunchKernelGGL((rmsnorm_k<T, NV>), dim3(max_rows), dim3(256), 0, s, (T *)out, x, (const T *)g, h, eps, row_index, p_count, min_rows, slabs, n_slabs, slab_stride)
    if (h <= 2048) SDLM_RMS(2); else if (h <= 4096) SDLM_RMS(4); else if (h <= 8192) SDLM_RMS(8); else SDLM_RMS(16);
#undef SDLM_RMS
}

void launch_rmsnorm(hipStream_t s, int dtype, void *out, float *x, const void *g, int h, float eps, const int32_t *row_index,
                    const int32_t *p_count, int max_rows, int min_rows, const float *slabs, int n_slabs, size_t slab_stride)
{
    if (dtype == 0) rmsnorm_t<float>(s, out, x, g, h, eps, row_index, p_count, max_rows, min_rows, slabs, n_slabs, slab_stride);
    else rmsnorm_t<bf16_t>(s, out, x, g, h, eps, row_index, p_count, max_rows, min_rows, slabs, n_slabs, slab_stride);
}

// ------------------------------------------------------------------------------------------------ GEMM (FMA)
// Y[r, n] = sum_k X[r, k] * W[n, k]; 64x64 tile, 16-deep slices through LDS, 4x4 outputs per thread.
__device__ inline float silu_f(float v) { return v / (1.0f + __expf(-v)); }

template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_k(GemmArgs a)
{
    const int R = min(*a.pR, a.max_rows);
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    if (m0 >= R) return;
    constexpr bool DUAL = EPI == EPI_SWIGLU;
    __shared__ float Xs[16][65], Ws[16][65], Us[DUAL ? 16 : 1][65];
    const T *X = (const T *)a.X, *W = (const T *)a.W, *W2 = (const T *)a.W2;
    const int t = threadIdx.x, tx = t & 15, ty = t >> 4, K = a.K, N = a.N;
    float acc[4][4] = {}, acc2[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int e = t; e < 1024; e += 256) {
            int row = e >> 4, kk = e & 15;
            bool kin = k0 + kk < K;
            Xs[kk][row] = (kin && m0 + row < R) ? to_f<T>(X[(size_t)(m0 + row) * K + k0 + kk]) : 0.f;
            bool nin = kin && n0 + row < N;
            Ws[kk][row] = nin ? to_f<T>(W[(size_t)(n0 + row) * K + k0 + kk]) : 0.f;
            if (DUAL) Us[kk][row] = nin ? to_f<T>(W2[(size_t)(n0 + row) * K + k0 + kk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float xv[4], wv[4], uv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { xv[i] = Xs[kk][ty * 4 + i]; wv[i] = Ws[kk][tx * 4 + i]; uv[i] = DUAL ? Us[kk][tx * 4 + i] : 0.f; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] += xv[i] * wv[j];
                    if (DUAL) acc2[i][j] += xv[i] * uv[j];
                }
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        int r = m0 + ty * 4 + i;
        if (r >= R) continue;
        for (int j = 0; j < 4; ++j) {
            int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            size_t o = (size_t)r * N + n;
            if (EPI == EPI_STORE_F32) a.Yf[o] = acc[i][j] + (a.bias ? to_f<T>(((const T *)a.bias)[n]) : 0.f);
            else if (EPI == EPI_RESID) a.Yf[o] += acc[i][j];
            else if (EPI == EPI_SWIGLU) ((T *)a.Yt)[o] = from_f<T>(silu_f(acc[i][j]) * acc2[i][j]);
            else a.Yf[o] = acc[i][j] * a.scale;
        }
    }
}

template <typename T>
static void gemm_generic_t(hipStream_t s, int epi, const GemmArgs &a)
{
    dim3 grid((a.N + 63) / 64, (a.max_rows + 63) / 64), block(256);
    switch (epi) {
    case EPI_STORE_F32: hipLaunchKernelGGL((gemm_generic_k<T, EPI_STORE_F32>), grid, block, 0, s, a); break;
    case EPI_RESID: hipLaunchKernelGGL((gemm_generic_k<T, EPI_RESID>), grid, block, 0, s, a); break;
    case EPI_SWIGLU: hipLaunchKernelGGL((gemm_generic_k<T, EPI_SWIGLU>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((gemm_generic_k<T, EPI_LOGITS>), grid, block, 0, s, a); break;
    }
}

void launch_gemm_generic(hipStream_t s, int dtype, int epi, const GemmArgs &a)
{
    if (dtype == 0) gemm_generic_t<float>(s, epi, a);
    else gemm_generic_t<bf16_t>(s, epi, a);
}

// ------------------------------------------------------------------------------------------------ RoPE + K/V placement
// qkv: raw projections [R, (Hq + 2 Hkv) d] fp32, given as n_slabs partial sums that are added in order.  Queries and keys are rotated at the row's position (rotate-half
// pairing i <-> i + d/2).  A pending row's K/V go to the cache slot of its position: they are final.  A block
// row's K/V (and, in a verification pass, every row's) go to slot `kind` of the row's staging tile: they are never cached.
// grid (rows, ceil((Hq + 2 Hkv) / 4)): one wavefront per (row, head), lane i < d/2 owns the pair (i, i + d/2).
template <typename T>
__global__ __launch_bounds__(256) void rope_scatter_k(const float *qkv, int n_slabs, size_t slab_stride, T *q_out, T *pool, KvGeom kg,
                                                      RowMeta rm, SeqState st, const float2 *rope, int Hq, int sure)
{
    const int r = blockIdx.x;
    const int d = kg.head_dim, half = d >> 1, Hk = kg.n_kv_heads, nq = Hq * d, nk = Hk * d;
    const int head = blockIdx.y * 4 + (threadIdx.x >> 6), i = threadIdx.x & 63;   // heads: Hq of q, then Hkv of k, then Hkv of v
    if (head >= Hq + 2 * Hk || i >= half || (r >= sure && r >= rm.counts[0])) return;   // certain rows: no wait for the count
    const float *src = qkv + (size_t)r * (nq + 2 * nk) + head * d + i;
    const int pos = rm.pos[r], kind = rm.kind[r], b = rm.seq[r], stg = rm.stg[r];   // requested together with the projections
    float x0 = src[0], x1 = src[half];
    for (int s0 = 1; s0 < n_slabs; s0 += 4) {   // four slabs per memory round trip, added in slab order
        float p0[4], p1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t o = (size_t)min(s0 + u, n_slabs - 1) * slab_stride;
            p0[u] = src[o];
            p1[u] = src[o + half];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (s0 + u < n_slabs) { x0 += p0[u]; x1 += p1[u]; }
    }
    if (head < Hq) {
        const float2 t = rope[(size_t)pos * half + i];
        T *q = q_out + (size_t)r * nq + head * d + i;
        q[0] = from_f<T>(x0 * t.x - x1 * t.y);
        q[half] = from_f<T>(x1 * t.x + x0 * t.y);
        return;
    }
    int page, slot;
    if (kind < 0) { page = st.page_table[(size_t)b * kg.pages_per_seq + pos / PAGE]; slot = pos % PAGE; }
    else { page = stg; slot = kind; }
    if (page < 0) return;   // unbacked position: only reachable after a reported pool exhaustion
    const bool is_k = head < Hq + Hk;
    const int hk = is_k ? head - Hq : head - Hq - Hk;
    T *tile = pool + kg.tile(page, hk);
    if (is_k) {
        const float2 t = rope[(size_t)pos * half + i];
        tile[k_off(slot, i)] = from_f<T>(x0 * t.x - x1 * t.y);
        tile[k_off(slot, i + half)] = from_f<T>(x1 * t.x + x0 * t.y);
    } else {
        T *Vb = tile + PAGE * d;
        Vb[v_off(slot, i)] = from_f<T>(x0);
        Vb[v_off(slot, i + half)] = from_f<T>(x1);
    }
}

void launch_rope_scatter(hipStream_t s, int dtype, const float *qkv, int n_slabs, size_t slab_stride, void *q_out, void *pool_layer,
                         const KvGeom &kg, const RowMeta &rm, const SeqState &st, const float2 *rope, int n_q_heads, int max_rows, int min_rows)
{
    dim3 grid(max_rows, (n_q_heads + 2 * kg.n_kv_heads + 3) / 4);
    if (dtype == 0) hipLaunchKernelGGL(rope_scatter_k<float>, grid, dim3(256), 0, s, qkv, n_slabs, slab_stride, (float *)q_out, (float *)pool_layer, kg, rm, st, rope, n_q_heads, min_rows);
    else hipLaunchKernelGGL(rope_scatter_k<bf16_t>, grid, dim3(256), 0, s, qkv, n_slabs, slab_stride, (bf16_t *)q_out, (bf16_t *)pool_layer, kg, rm, st, rope, n_q_heads, min_rows);
}

// ------------------------------------------------------------------------------------------------ attention
// One wavefront per (row, query head).  Keys: the cache positions [0, lim) of the row's sequence and the slots of
// the row's staging tiles named by its slot masks; for a block row these are the D keys of its block (mask equation, Sec. 3.3:
// causal below the block start, full mutual attention inside the block).  Each lane walks a strided subset of the keys with a running
// (max, sum, output); the 64 partial results are merged at the end.
template <typename T, int HD>
__global__ __launch_bounds__(64) void attn_generic_k(const T *q, T *out, const T *pool, KvGeom kg, RowMeta rm, SeqState st,
                                                     int Hq)
{
    const int r = blockIdx.y;
    if (r >= rm.counts[0]) return;
    const int hq = blockIdx.x, G = Hq / kg.n_kv_heads, hk = hq / G, lane = threadIdx.x;
    const int b = rm.seq[r], lim = rm.lim[r], stg = rm.stg[r], stg2 = rm.stg2[r];
    const uint32_t sm_all = (uint32_t)rm.smask[r];
    const uint32_t smask = stg >= 0 ? sm_all & 0xffffu : 0u, smask2 = stg2 >= 0 ? sm_all >> 16 : 0u;
    // key index lim + i stands for slot i of the second staging tile (i < 16), lim + 16 + i for slot i of the row's own tile
    const int total = lim + (smask ? 16 + 32 - __clz(smask) : (smask2 ? 32 - __clz(smask2) : 0));
    __shared__ float qs[HD];
    __shared__ float part[64][HD + 1];
    const float scale = 1.0f / sqrtf((float)HD);
    for (int i = lane; i < HD; i += 64) qs[i] = to_f<T>(q[((size_t)r * Hq + hq) * HD + i]);
    __syncthreads();
    float m = -INFINITY, l = 0.f, o[HD];
#pragma unroll
    for (int i = 0; i < HD; ++i) o[i] = 0.f;
    for (int j = lane; j < total; j += 64) {
        int page, slot;
        if (j < lim) { page = st.page_table[(size_t)b * kg.pages_per_seq + j / PAGE]; slot = j % PAGE; }
        else if (j < lim + 16) { page = stg2; slot = j - lim; if (!((smask2 >> slot) & 1u)) continue; }
        else { page = stg; slot = j - lim - 16; if (!((smask >> slot) & 1u)) continue; }
        const T *Kb = pool + kg.tile(page, hk), *Vb = Kb + PAGE * HD;
        float sdot = 0.f;
#pragma unroll
        for (int i = 0; i < HD; ++i) sdot += qs[i] * to_f<T>(Kb[k_off(slot, i)]);
        sdot *= scale;
        float mn = fmaxf(m, sdot), corr = __expf(m - mn), p = __expf(sdot - mn);
        l = l * corr + p;
#pragma unroll
        for (int i = 0; i < HD; ++i) o[i] = o[i] * corr + p * to_f<T>(Vb[v_off(slot, i)]);
        m = mn;
    }
    float M = m;
    for (int s = 32; s > 0; s >>= 1) M = fmaxf(M, __shfl_xor(M, s));
    float f = (m == -INFINITY) ? 0.f : __expf(m - M);
    float L = l * f;
    for (int s = 32; s > 0; s >>= 1) L += __shfl_xor(L, s);
#pragma unroll
    for (int i = 0; i < HD; ++i) part[lane][i] = o[i] * f;
    __syncthreads();
    for (int i = lane; i < HD; i += 64) {
        float acc = 0.f;
        for (int w = 0; w < 64; ++w) acc += part[w][i];
        out[((size_t)r * Hq + hq) * HD + i] = from_f<T>(acc / L);
    }
}

template <typename T>
static void attn_generic_t(hipStream_t s, const void *q, void *out, const void *pool_layer, const KvGeom &kg,
                           const RowMeta &rm, const SeqState &st, int Hq, int max_rows)
{
    dim3 grid(Hq, max_rows), block(64);
    switch (kg.head_dim) {
    case 32: hipLaunchKernelGGL((attn_generic_k<T, 32>), grid, block, 0, s, (const T *)q, (T *)out, (const T *)pool_layer, kg, rm, st, Hq); break;
    case 64: hipLaunchKernelGGL((attn_generic_k<T, 64>), grid, block, 0, s, (const T *)q, (T *)out, (const T *)pool_layer, kg, rm, st, Hq); break;
    case 96: hipLaunchKernelGGL((attn_generic_k<T, 96>), grid, block, 0, s, (const T *)q, (T *)out, (const T *)pool_layer, kg, rm, st, Hq); break;
    default: hipLaunchKernelGGL((attn_generic_k<T, 128>), grid, block, 0, s, (const T *)q, (T *)out, (const T *)pool_layer, kg, rm, st, Hq); break;
    }
}

void launch_attn_generic(hipStream_t s, int dtype, const void *q, void *out, const void *pool_layer, const KvGeom &kg,
                         const RowMeta &rm, const SeqState &st, int n_q_heads, int max_rows)
{
    if (dtype == 0) attn_generic_t<float>(s, q, out, pool_layer, kg, rm, st, n_q_heads, max_rows);
    else attn_generic_t<bf16_t>(s, q, out, pool_layer, kg, rm, st, n_q_heads, max_rows);
}

// ------------------------------------------------------------------------------------------------ vocabulary reduction
// Per block row: arg-max (lowest index on ties), and the confidence of Sec. 3.4: (1) softmax probability of the
// arg-max token = 1 / sum exp(z - max); (2) 1 - H / log|V| with H = log S - (sum e^{z-m} (z-m)) / S.
__global__ __launch_bounds__(256) void lm_reduce_k(const float *logits, int V, int32_t *ids, float *conf, int conf_fn,
                                                   const int32_t *p_rows)
{
    int row = blockIdx.x;
    if (row >= *p_rows) return;
    const float *z = logits + (size_t)row * V;
    __shared__ float sm[4];
    __shared__ int si[4];
    __shared__ float red[4];
    float m = -INFINITY;
    int arg = 0;   // stays a valid id even if every logit is NaN
    for (int v = threadIdx.x; v < V; v += 256) {
        float t = z[v];
        if (t > m) { m = t; arg = v; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        float om = __shfl_xor(m, o);
        int oa = __shfl_xor(arg, o);
        if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
    }
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = m; si[threadIdx.x >> 6] = arg; }
    __syncthreads();
    m = sm[0]; arg = si[0];
    for (int w = 1; w < 4; ++w)
        if (sm[w] > m || (sm[w] == m && si[w] < arg)) { m = sm[w]; arg = si[w]; }
    float S = 0.f, E = 0.f;
    for (int v = threadIdx.x; v < V; v += 256) {
        float dlt = z[v] - m, e = __expf(dlt);
        S += e;
        E += e * dlt;
    }
    S = block_sum(S, red);
    E = block_sum(E, red);
    if (threadIdx.x == 0) {
        ids[row] = arg;
        conf[row] = conf_fn == 0 ? 1.0f / S : 1.0f - (logf(S) - E / S) / logf((float)V);
    }
}

void launch_lm_reduce(hipStream_t s, const float *logits, int V, int32_t *ids, float *conf, int conf_fn,
                      const int32_t *p_rows, int max_rows)
{
    hipLaunchKernelGGL(lm_reduce_k, dim3(max_rows), dim3(256), 0, s, logits, V, ids, conf, conf_fn, p_rows);
}

// ------------------------------------------------------------------------------------------------ acceptance
// gamma_tau (Sec. 3.4): the largest j in 1..D whose cumulative product of confidences is >= tau, at least 1.
// The product is a float product taken left to right.  rule 1: leading positions whose own confidence is >= tau.
__global__ void accept_k(SeqState st, const int32_t *ids_rows, const float *conf_rows, int B, int D, float tau, int rule,
                         int32_t *ids_out, int32_t *count_out, float *conf_out)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int best = 1;
    if (rule == 0) {
        float prod = 1.0f;
        for (int j = 1; j <= D; ++j) {
            prod = prod * conf_rows[b * D + j - 1];
            if (prod >= tau && j > best) best = j;
        }
    } else {
        int j = 0;
        while (j < D && conf_rows[b * D + j] >= tau) ++j;
        if (j > best) best = j;
    }
    st.last_count[b] = best;
    count_out[b] = best;
    for (int j = 0; j < D; ++j) {
        int id = ids_rows[b * D + j];
        st.last_ids[b * D + j] = id;
        ids_out[b * D + j] = id;
        if (conf_out) conf_out[b * D + j] = conf_rows[b * D + j];
    }
}

void launch_accept(hipStream_t s, const SeqState &st, const int32_t *ids_rows, const float *conf_rows, int B, int D,
                   float tau, int rule, int32_t *ids_out, int32_t *count_out, float *conf_out)
{
    hipLaunchKernelGGL(accept_k, dim3((B + 63) / 64), dim3(64), 0, s, st, ids_rows, conf_rows, B, D, tau, rule, ids_out, count_out, conf_out);
}

// ------------------------------------------------------------------------------------------------ commit
// c <- n (the pending K/V, already in place, become cache); the accepted tokens become the pending tokens;
// n <- n + count; the page table grows so that every position < n is backed.
__global__ void commit_k(SeqState st, int B, int D, const int32_t *ids_ovr, const int32_t *cnt_ovr, int paged, int n_pages,
                         int pages_per_seq, int V)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t *ids = ids_ovr ? ids_ovr + b * D : st.last_ids + b * D;
    int cnt = cnt_ovr ? cnt_ovr[b] : st.last_count[b];
    if (cnt < 1 || cnt > D) { atomicOr(&st.alloc[1], 2); cnt = cnt < 1 ? 1 : D; }
    int n = st.n[b], n_new = n + cnt;
    int need = (n_new + PAGE - 1) / PAGE - st.pages_backed[b];
    if (need > 0) {
        if (!paged || st.pages_backed[b] + need > pages_per_seq) { atomicOr(&st.alloc[1], 1); return; }
        int first = atomicAdd(&st.alloc[0], need);
        if (first + need > n_pages) { atomicOr(&st.alloc[1], 1); return; }
        for (int i = 0; i < need; ++i) st.page_table[(size_t)b * pages_per_seq + st.pages_backed[b] + i] = first + i;
        st.pages_backed[b] += need;
    }
    for (int i = 0; i < cnt; ++i) {
        int id = ids[i];
        if (id < 0 || id >= V) { atomicOr(&st.alloc[1], 4); id = 0; }   // an override token outside the vocabulary
        st.pend_tok[b * D + i] = id;
    }
    st.last_tok[b] = st.pend_tok[b * D + cnt - 1];
    st.c[b] = n;
    st.n[b] = n_new;
}

void launch_commit(hipStream_t s, const SeqState &st, int B, int D, const int32_t *ids_ovr, const int32_t *cnt_ovr,
                   int paged, int n_pages, int pages_per_seq, int V)
{
    hipLaunchKernelGGL(commit_k, dim3((B + 63) / 64), dim3(64), 0, s, st, B, D, ids_ovr, cnt_ovr, paged, n_pages, pages_per_seq, V);
}

// ------------------------------------------------------------------------------------------------ debug read-back
template <typename T>
__global__ void read_kv_k(const T *pool, KvGeom kg, SeqState st, int seq, int kvh, int pos0, int count, float *k_out, float *v_out)
{
    int d = kg.head_dim;
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < count * d; e += gridDim.x * blockDim.x) {
        int pos = pos0 + e / d, i = e % d;
        int page, slot;
        if (pos0 < 0) { page = kg.staging_base + seq; slot = e / d; }   // the block rows' staging tile
        else { page = st.page_table[(size_t)seq * kg.pages_per_seq + pos / PAGE]; slot = pos % PAGE; }
        const T *Kb = pool + kg.tile(page, kvh), *Vb = Kb + PAGE * d;
        k_out[e] = to_f<T>(Kb[k_off(slot, i)]);
        v_out[e] = to_f<T>(Vb[v_off(slot, i)]);
    }
}

void launch_read_kv(hipStream_t s, int dtype, const void *pool_layer, const KvGeom &kg, const SeqState &st, int seq,
                    int kvh, int pos0, int count, float *k_out, float *v_out)
{
    int blocks = (count * kg.head_dim + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    if (dtype == 0) hipLaunchKernelGGL(read_kv_k<float>, dim3(blocks), dim3(256), 0, s, (const float *)pool_layer, kg, st, seq, kvh, pos0, count, k_out, v_out);
    else hipLaunchKernelGGL(read_kv_k<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)pool_layer, kg, st, seq, kvh, pos0, count, k_out, v_out);
}

}  // namespace sdlm
