// Block-masked decode attention on the matrix cores (bf16 cache, head_dim 128, GQA).
//
// Work item = (row group, kv head, KV chunk).  A row group is a run of rows of one sequence (its pending causal
// rows and its D block rows) small enough that rows x (query heads per kv head) <= 64 query vectors; all of them
// consume each K/V tile once, so the cache is streamed from HBM once per (sequence, kv head, layer).
//   scores   S^T[key, query] = K Q^T     v_mfma_f32_16x16x32_bf16, A = one 16-key K tile, B = 16 queries
//   output   O^T[d, query]  += V^T P^T   same instruction, A = V^T of two tiles (32 keys), B = P^T
// The cache tiles are stored in exactly the operand order of these instructions (see internal.hpp), so a
// workgroup copies a tile pair (32 keys, 16 KB) global -> LDS as one contiguous run and every wavefront reads its
// operands from LDS with conflict-free 16-byte / 8-byte reads.  Each of the four wavefronts owns 16 of the (at
// most 64) query vectors, so its state is small (32 accumulator registers) and four workgroups fit on a CU.
// The mask of the method lives in registers: every row sees cache keys [0, lim) and the slots of the group's
// staging tiles that its slot masks name (its own tile, and for a verification block the tile of the shared causal rows).  A pending row at position p has lim = p + 1 and no staging slots; a block row has lim = s
// and the D keys of its own block in the staging tile.
// Chunks of one (group, head) are merged by a second small kernel when there is more than one.
#include "mfma.hpp"

namespace sdlm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int NQ = 4;     // 16-query tiles per work item
constexpr int QMAX = NQ * 16;
constexpr int HD = 128;
constexpr float RESCALE_GAP = 8.0f;   // log2 units

struct AttnArgs {
    const bf16_t *q;
    bf16_t *out;
    const bf16_t *pool;
    KvGeom kg;
    RowMeta rm;
    SeqState st;
    int Hq, G, D, chunk_pages, max_chunks;
    float *part_o;      // [item][QMAX][HD]
    float2 *part_ml;    // [item][QMAX]
    float c;            // log2(e) / sqrt(d)
};

union Op8 { bf16x8 v; uint4 u; uint2 h[2]; uint32_t w[4]; };

// TWO_STG: row groups may read a second staging tile (verification passes of block sizes above 4); decode steps and
// prefill passes use the variant without it, which keeps the kernel at four workgroups per compute unit without spills.
template <bool TWO_STG>
__global__ __launch_bounds__(256, 4) void attn_mfma_k(AttnArgs a)
{
    const int g = blockIdx.x, hk = blockIdx.y, chunk = blockIdx.z;
    // The start of a work item is a chain of dependent lookups (group count -> group -> row limits -> page table ->
    // K/V).  The group's entries are in bounds for every group of the grid, and the page-table entries of the first
    // two tile pairs depend on the sequence and the chunk alone, so each is requested one step early: three memory
    // round trips before the first K/V request instead of five.
    const int n_groups = a.rm.counts[1];
    const int cp = max(a.rm.counts[3], a.chunk_pages);   // tiles per KV chunk: chosen on the device from the actual lengths, never below the host's floor
    const int row0 = a.rm.grp_row0[g], nrows = a.rm.grp_n[g], b = a.rm.grp_seq[g];
    if (g >= n_groups) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const int G = a.G, QR = nrows * G;
    const int32_t *ptab = a.st.page_table + (size_t)b * a.kg.pages_per_seq;
    int pg_first[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) pg_first[u] = ptab[min(chunk * cp + u, a.kg.pages_per_seq - 1)];

    int lim_l = lane < nrows ? a.rm.lim[row0 + lane] : 0;
    int blk_l = lane < nrows ? a.rm.smask[row0 + lane] : 0;   // OR over the group's rows: which staging tiles are seen at all
    int min_l = lane < nrows ? lim_l : 0x7fffffff;
    for (int o = 32; o > 0; o >>= 1) {
        lim_l = max(lim_l, __shfl_xor(lim_l, o));
        blk_l |= __shfl_xor(blk_l, o);
        min_l = min(min_l, __shfl_xor(min_l, o));
    }
    const int max_lim = lim_l, min_lim = min_l, any_blk = blk_l;
    const int n_pages = (max_lim + PAGE - 1) / PAGE;
    const int n_chunks = max(1, (n_pages + cp - 1) / cp);
    if (chunk >= n_chunks) return;
    const int c0 = chunk * cp, c1 = min(n_pages, c0 + cp);
    const int n_cache = c1 - c0;
    // Staging tiles follow the cache tiles of chunk 0: first the group's second tile (if a row sees it: upper half of
    // the slot masks), then its own tile (lower half).
    const bool has1 = (any_blk & 0xffff) != 0, has2 = TWO_STG && ((uint32_t)any_blk >> 16) != 0;
    const int nv = n_cache + (chunk == 0 ? (int)has1 + (int)has2 : 0);   // virtual tiles of this chunk; the last ones may be staging
    const int n_pairs = (nv + 1) / 2;

    // This wavefront's 16 queries: B operands, lane (n = lane%16, group lg) holds q[32 kk + 8 lg .. +8] of query 16 wave + n
    const int qi = wave * 16 + ln;
    const bool qvalid = qi < QR;
    const bool wave_active = wave * 16 < QR;
    const int rl = qvalid ? qi / G : 0, hg = qvalid ? qi % G : 0, qrow = row0 + rl;
    const int lim_q = qvalid ? a.rm.lim[qrow] : 0;
    // staging slots this query sees, re-packed by virtual tile: low half for tile n_cache, high half for tile n_cache + 1
    const uint32_t smask_raw = qvalid ? (uint32_t)a.rm.smask[qrow] : 0u;
    const uint32_t smask_q = has2 ? (smask_raw >> 16) | (smask_raw << 16) : smask_raw & 0xffffu;   // !TWO_STG: the tile's own mask
    Op8 qop[4];
    {
        const bf16_t *qp = a.q + ((size_t)qrow * a.Hq + hk * G + hg) * HD + lg * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            qop[kk].u = make_uint4(0, 0, 0, 0);
            if (qvalid) qop[kk].u = *(const uint4 *)(qp + kk * 32);
        }
    }
    f32x4 O[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    // K/V of one tile pair (32 keys, 16 KB) is fetched by the whole workgroup, 64 bytes per thread, and shared
    // through LDS in the cache's own operand order; two LDS buffers, the next two pairs ride in registers meanwhile.
    __shared__ __attribute__((aligned(16))) bf16_t kv[2][2][2 * PAGE * HD];   // [buffer][tile A/B][K block | V block]
    const size_t tile_elems = 2 * PAGE * HD;
    const int stg_last = max(a.rm.grp_stg[g], 0), stg_first = (TWO_STG && has2) ? max(a.rm.grp_stg2[g], 0) : stg_last;
    auto stg_of = [&](int u) { return (TWO_STG && u == n_cache) ? stg_first : stg_last; };   // staging tile behind virtual tile u >= n_cache
    u32x4 rA[4], rB[4];   // two tile pairs in flight: the next one and the one after it
    auto fetch_pages = [&](int pgA, int pgB, u32x4 (&r)[4]) {
        const bf16_t *tA = a.pool + ((size_t)pgA * a.kg.n_kv_heads + hk) * tile_elems;
        const bf16_t *tB = a.pool + ((size_t)pgB * a.kg.n_kv_heads + hk) * tile_elems;
        r[0] = *(const u32x4 *)(tA + tid * 8);
        r[1] = *(const u32x4 *)(tA + (256 + tid) * 8);
        r[2] = *(const u32x4 *)(tB + tid * 8);
        r[3] = *(const u32x4 *)(tB + (256 + tid) * 8);
    };
    auto fetch = [&](int pp, u32x4 (&r)[4]) {
        const int uA = 2 * pp, uB = 2 * pp + 1;
        const int pgA = uA >= n_cache ? stg_of(uA) : ptab[c0 + uA];
        const int pgB = uB >= nv ? pgA : (uB >= n_cache ? stg_of(uB) : ptab[c0 + uB]);
        fetch_pages(pgA, pgB, r);
    };
    auto fetch_first = [&](int pA, int pB, int uA, u32x4 (&r)[4]) {   // pairs 0 and 1: page ids requested at the top
        const int uB = uA + 1;
        const int pgA = uA >= n_cache ? stg_of(uA) : pA;
        const int pgB = uB >= nv ? pgA : (uB >= n_cache ? stg_of(uB) : pB);
        fetch_pages(pgA, pgB, r);
    };
    auto stash = [&](int buf, const u32x4 (&r)[4]) {
        *(u32x4 *)(&kv[buf][0][0] + tid * 8) = r[0];
        *(u32x4 *)(&kv[buf][0][0] + (256 + tid) * 8) = r[1];
        *(u32x4 *)(&kv[buf][1][0] + tid * 8) = r[2];
        *(u32x4 *)(&kv[buf][1][0] + (256 + tid) * 8) = r[3];
    };
    auto compute = [&](int pp, int buf) {
        if (wave_active) {
            const int uA = 2 * pp, uB = 2 * pp + 1;
            const bool hasB = uB < nv;
            const bool stgA = uA >= n_cache, stgB = hasB && uB >= n_cache;
            const bf16_t *KA = &kv[buf][0][0], *KB = &kv[buf][1][0];
            // scores: lane (query n, group lg) gets keys 4 lg .. 4 lg + 3 of each tile
            f32x4 sA = {0.f, 0.f, 0.f, 0.f}, sB = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                Op8 ka, kb;
                ka.u = *(const uint4 *)(KA + (kk * 64 + lane) * 8);
                kb.u = *(const uint4 *)(KB + (kk * 64 + lane) * 8);
                sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka.v, qop[kk].v, sA, 0, 0, 0);
                sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb.v, qop[kk].v, sB, 0, 0, 0);
            }
            const bool fullA = !stgA && (c0 + uA + 1) * PAGE <= min_lim;
            const bool fullB = hasB && !stgB && (c0 + uB + 1) * PAGE <= min_lim;
            if (!(fullA && fullB)) {
                const int keyA = (c0 + uA) * PAGE + lg * 4, keyB = (c0 + uB) * PAGE + lg * 4;
                // slot masks of the staging tile behind A / B
                const uint32_t mA = TWO_STG ? (smask_q >> (uA == n_cache ? 0 : 16)) & 0xffffu : smask_q;
                const uint32_t mB = TWO_STG ? (smask_q >> (uB == n_cache ? 0 : 16)) & 0xffffu : smask_q;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    bool visA = stgA ? ((mA >> (lg * 4 + v)) & 1u) != 0 : (keyA + v < lim_q);
                    bool visB = hasB && (stgB ? ((mB >> (lg * 4 + v)) & 1u) != 0 : (keyB + v < lim_q));
                    sA[v] = visA ? sA[v] : -INFINITY;
                    sB[v] = visB ? sB[v] : -INFINITY;
                }
            }
            // raw scores; the softmax scale is folded into the exponent: p = 2^(c s - c m)
            float mx = fmaxf(fmaxf(fmaxf(sA[0], sA[1]), fmaxf(sA[2], sA[3])), fmaxf(fmaxf(sB[0], sB[1]), fmaxf(sB[2], sB[3])));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // The reference maximum only moves when it is exceeded by more than RESCALE_GAP / c (p stays below
            // 2^RESCALE_GAP, harmless in fp32 sums and bf16 products); the accumulators are rescaled only then.
            if (__any((mx - m_run) * a.c > RESCALE_GAP || (m_run == -INFINITY && mx > -INFINITY))) {
                const float m_new = fmaxf(m_run, mx);
                const float corr = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((m_run - m_new) * a.c);
                l_run *= corr;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) O[dt] *= corr;
                m_run = m_new;
            }
            const float mc = m_run == -INFINITY ? 0.f : m_run * a.c;
            float p[8];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                p[v] = __builtin_amdgcn_exp2f(fmaf(sA[v], a.c, -mc));
                p[4 + v] = __builtin_amdgcn_exp2f(fmaf(sB[v], a.c, -mc));
            }
            l_run += (p[0] + p[1]) + (p[2] + p[3]) + (p[4] + p[5]) + (p[6] + p[7]);
            Op8 pop;
            pop.w[0] = pack_bf16(p[0], p[1]); pop.w[1] = pack_bf16(p[2], p[3]);
            pop.w[2] = pack_bf16(p[4], p[5]); pop.w[3] = pack_bf16(p[6], p[7]);
            const bf16_t *VA = KA + PAGE * HD, *VB = KB + PAGE * HD;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                Op8 vo;
                vo.h[0] = *(const uint2 *)(VA + (dt * 64 + lane) * 4);
                vo.h[1] = *(const uint2 *)(VB + (dt * 64 + lane) * 4);
                O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vo.v, pop.v, O[dt], 0, 0, 0);
            }
        }
    };
    fetch_first(pg_first[0], pg_first[1], 0, rB);   // both requests are out before the first is waited for
    if (n_pairs > 1) fetch_first(pg_first[2], pg_first[3], 2, rA);
    stash(0, rB);
    __syncthreads();
    // iteration pp: regs hold pair pp+1, pair pp+2 is requested, pair pp is consumed from LDS
    for (int pp = 0; pp < n_pairs; pp += 2) {
        if (pp + 2 < n_pairs) fetch(pp + 2, rB);
        compute(pp, 0);
        if (pp + 1 < n_pairs) stash(1, rA);
        __syncthreads();
        if (pp + 1 >= n_pairs) break;
        if (pp + 3 < n_pairs) fetch(pp + 3, rA);
        compute(pp + 1, 1);
        if (pp + 2 < n_pairs) stash(0, rB);
        __syncthreads();
    }
    if (!qvalid) return;
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    const bool single = n_chunks == 1;
    const size_t item = ((size_t)g * a.kg.n_kv_heads + hk) * a.max_chunks + chunk;
    const float inv = single ? 1.0f / l_run : 1.0f;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        f32x4 o = O[dt] * inv;
        const int d4 = dt * 16 + lg * 4;
        if (single) {
            bf16_t *op = a.out + ((size_t)qrow * a.Hq + hk * G + hg) * HD + d4;
            *(uint2 *)op = make_uint2(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]));
        } else {
            *(f32x4 *)(a.part_o + (item * QMAX + qi) * HD + d4) = o;
        }
    }
    if (!single && lg == 0) a.part_ml[item * QMAX + qi] = make_float2(m_run, l_run);
}

// Merge the chunks of one (group, kv head): out = sum_c 2^{c(m_c - M)} o_c / sum_c 2^{c(m_c - M)} l_c.  A separate
// launch rather than "the last workgroup merges": the chunks run on different XCDs, whose L2s only agree at
// kernel boundaries, and a device-scope fence in every workgroup costs more than this launch.
// grid (group, kv head, 16-query tile); the tile's scale factors are computed once and shared through LDS.
// The kernel is a chain of dependent memory round trips and little else, so the partial results are requested
// before the group is looked up: the row assembly leaves, per group, how many chunks and rows it has (grp_hint), and
// exactly those partial results and running maxima are requested one round trip in.  The hint only steers these early
// requests: the chunk count that decides the result is derived from the rows' limits as in the attention kernel, and
// what a hint misses is fetched afterwards.
__global__ __launch_bounds__(256) void attn_combine_k(AttnArgs a)
{
    constexpr int CU = 4, V4 = HD / 4, EPT = 16 * V4 / 256;   // chunks requested together; float4 per query; elements per thread
    const int g = blockIdx.x, hk = blockIdx.y, nq = blockIdx.z, tid = threadIdx.x, lane = tid & 63;
    const size_t item0 = ((size_t)g * a.kg.n_kv_heads + hk) * a.max_chunks;
    const int hint = a.rm.grp_hint[g];   // in bounds for every group of the grid
    const int n_groups = a.rm.counts[1];
    const int cp = max(a.rm.counts[3], a.chunk_pages);
    const int row0 = a.rm.grp_row0[g], nrows = a.rm.grp_n[g];
    const int hc = min(hint & 0xff, a.max_chunks), hq = ((hint >> 8) & 0xff) * a.G;   // chunks and queries to expect
    const int mq = tid & 15, mc = tid >> 4;
    float2 ml0 = make_float2(0.f, 0.f);
    f32x4 po[EPT][CU];
    const bool ml_early = hc > 1 && mc < hc;
    if (ml_early) ml0 = a.part_ml[(item0 + mc) * QMAX + nq * 16 + mq];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int e = tid + j * 256, qi = nq * 16 + e / V4, d4 = (e % V4) * 4;
#pragma unroll
        for (int u = 0; u < CU; ++u) {
            po[j][u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (hc > 1 && u < hc && qi < hq) po[j][u] = *(const f32x4 *)(a.part_o + ((item0 + u) * QMAX + qi) * HD + d4);
        }
    }
    if (g >= n_groups) return;
    const int QR = nrows * a.G;
    if (nq * 16 >= QR) return;
    int lim = lane < nrows ? a.rm.lim[row0 + lane] : 0;   // a group has at most QMAX rows: every wavefront finds the maximum itself
    for (int o = 32; o > 0; o >>= 1) lim = max(lim, __shfl_xor(lim, o));
    const int n_pages = (lim + PAGE - 1) / PAGE;
    const int n_chunks = max(1, (n_pages + cp - 1) / cp);
    if (n_chunks == 1) return;   // the attention kernel wrote the final result itself
    __shared__ float sf[16][65], sl[16][65];   // [query][chunk]: running maximum, then 2^{c(m_c - M)} / L; row sum
    for (int c = mc; c < n_chunks; c += 16) {
        const float2 ml = (c < 16 && ml_early) ? ml0 : a.part_ml[(item0 + c) * QMAX + nq * 16 + mq];
        sf[mq][c] = ml.x;
        sl[mq][c] = ml.y;
    }
    __syncthreads();
    if (tid < 16 && nq * 16 + tid < QR) {
        float M = -INFINITY;
        for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, sf[tid][c]);
        float L = 0.f;
        for (int c = 0; c < n_chunks; ++c) {
            const float m = sf[tid][c];
            const float f = m == -INFINITY ? 0.f : exp2f((m - M) * a.c);
            sf[tid][c] = f;
            L += sl[tid][c] * f;
        }
        const float inv = 1.0f / L;
        for (int c = 0; c < n_chunks; ++c) sf[tid][c] *= inv;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int e = tid + j * 256, ql = e / V4, d4 = (e % V4) * 4, qi = nq * 16 + ql;
        if (qi >= QR) continue;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
        for (int c0 = 0; c0 < n_chunks; c0 += CU) {
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                const bool have = c0 == 0 && hc > 1 && u < hc && qi < hq;   // requested at the top
                if (!have && c0 + u < n_chunks) po[j][u] = *(const f32x4 *)(a.part_o + ((item0 + c0 + u) * QMAX + qi) * HD + d4);
            }
#pragma unroll
            for (int u = 0; u < CU; ++u)
                if (c0 + u < n_chunks) o += po[j][u] * sf[ql][c0 + u];
        }
        const int rl = qi / a.G, hg = qi % a.G;
        bf16_t *op = a.out + ((size_t)(row0 + rl) * a.Hq + hk * a.G + hg) * HD + d4;
        *(uint2 *)op = make_uint2(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]));
    }
}

int mfma_group_rows(const sdlm_model_cfg *m)
{
    int G = m->n_q_heads / m->n_kv_heads;
    int gr = QMAX / G;
    return gr > GROUP_ROWS ? GROUP_ROWS : (gr < 1 ? 1 : gr);
}

// chunk size (in 16-key tiles) and chunk count for a launch over `groups` row groups
static void chunking(const sdlm_model_cfg *m, int max_seq_len, int groups, int *chunk_pages, int *max_chunks)
{
    int pages = (max_seq_len + PAGE - 1) / PAGE;
    long items = (long)groups * m->n_kv_heads;
    int cp = 64;                                     // 1024 keys
    while (cp > 8 && items * ((pages + cp - 1) / cp) < 512) cp >>= 1;
    while ((pages + cp - 1) / cp > 64) cp <<= 1;     // the merge kernel keeps at most 64 scale factors per query
    *chunk_pages = cp;
    *max_chunks = (pages + cp - 1) / cp;
}

// The smallest chunk size a launch over `groups` row groups may use (the device may pick a larger one from the actual
// lengths, see attn_chunk_pages): the policy above, made coarser until the partial results fit the scratch area.
static void chunk_floor(const sdlm_model_cfg *m, int max_seq_len, int groups, size_t scratch_bytes, int *chunk_pages, int *max_chunks)
{
    chunking(m, max_seq_len, groups, chunk_pages, max_chunks);
    const int pages = (max_seq_len + PAGE - 1) / PAGE;
    size_t items = (size_t)groups * m->n_kv_heads * *max_chunks;
    while (*max_chunks > 1 && items * ((size_t)QMAX * HD * 4 + QMAX * 8) > scratch_bytes) {
        *chunk_pages *= 2;
        *max_chunks = (pages + *chunk_pages - 1) / *chunk_pages;
        items = (size_t)groups * m->n_kv_heads * *max_chunks;
    }
}

int mfma_attn_chunk_floor(const sdlm_model_cfg *m, int max_seq_len, int groups, size_t scratch_bytes)
{
    int cp, mc;
    chunk_floor(m, max_seq_len, groups, scratch_bytes, &cp, &mc);
    return cp;
}

size_t mfma_attn_scratch_bytes(const sdlm_model_cfg *m, const sdlm_run_cfg *r, int max_rows)
{
    if (!mfma_supported(m)) return 256;
    int gr = mfma_group_rows(m);
    // decode: every sequence has at most ceil(2D / gr) groups; prefill: at most max_rows groups of >= 1 row, but
    // then each group is short: bound both by the launch that needs the most (groups x chunks)
    size_t worst = 0;
    // ... and the verification pass
    int cand[3] = {r->max_batch * ((2 * r->block_D + gr - 1) / gr), max_rows / gr + r->max_batch,
                   r->max_batch * verify_groups_per_seq(r->block_D, gr)};
    for (int i = 0; i < 3; ++i) {
        if (cand[i] < 1) continue;
        int cp, mc;
        chunking(m, r->max_seq_len, cand[i], &cp, &mc);
        size_t items = (size_t)cand[i] * m->n_kv_heads * mc;
        worst = items > worst ? items : worst;
    }
    return worst * ((size_t)QMAX * HD * 4 + QMAX * 8) + 256;
}

bool launch_attn_mfma(hipStream_t s, const sdlm_model_cfg *m, int max_seq_len, const void *q, void *out, const void *pool_layer,
                      const KvGeom &kg, const RowMeta &rm, const SeqState &st, int D, int max_groups, void *scratch, size_t scratch_bytes,
                      int part, bool two_staging)
{
    AttnArgs a;
    a.q = (const bf16_t *)q; a.out = (bf16_t *)out; a.pool = (const bf16_t *)pool_layer;
    a.kg = kg; a.rm = rm; a.st = st; a.Hq = m->n_q_heads; a.G = m->n_q_heads / m->n_kv_heads; a.D = D;
    chunk_floor(m, max_seq_len, max_groups, scratch_bytes, &a.chunk_pages, &a.max_chunks);
    const size_t items = (size_t)max_groups * kg.n_kv_heads * a.max_chunks;
    a.part_o = (float *)scratch;
    a.part_ml = (float2 *)((char *)scratch + items * QMAX * HD * 4);
    a.c = 1.4426950408889634f / sqrtf((float)HD);
    if (part == 0) {
        if (two_staging) hipLaunchKernelGGL(attn_mfma_k<true>, dim3(max_groups, kg.n_kv_heads, a.max_chunks), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(attn_mfma_k<false>, dim3(max_groups, kg.n_kv_heads, a.max_chunks), dim3(256), 0, s, a);
    }
    else if (a.max_chunks > 1) hipLaunchKernelGGL(attn_combine_k, dim3(max_groups, kg.n_kv_heads, NQ), dim3(256), 0, s, a);
    return a.max_chunks > 1;
}

}  // namespace sdlm
