// Matrix-core (MFMA) GEMMs of the bf16 mode: the QKV / O / gate-up / down projections and the LM head with its
// fused vocabulary reduction.  These are the path's only true dense contractions.
//
// Y[r, n] = sum_k X[r, k] W[n, k], R activation rows (8 .. 2048) against N weight rows: every weight byte is
// needed exactly once per step, so the kernels are organised around streaming W from HBM.
//   * W is repacked once (sdlm_init_weights) into the operand order of v_mfma_f32_32x32x16_bf16: tile (n/32,
//     k/16) is 64 lanes x 8 bf16 = 1 KB contiguous and the tiles of one 32-row band follow each other along k,
//     so a wavefront's operand stream is a plain contiguous run, loaded global -> registers with 16-byte loads
//     and never staged in LDS (no other wavefront of the workgroup needs the same weights).
//   * The weight tile is the A operand (M = 32 output features), the activation rows are the B operand
//     (N = 32 rows).  A workgroup is 4 wavefronts; each owns NT bands of output features and all of them
//     share the MT*32 activation rows of the workgroup, which are staged in LDS (64-deep k slices, double
//     buffered, rows padded to 144 bytes so that the 16-byte operand reads do not collide on banks).
//   * Skinny problems (few rows, few output features) are split along k; the partial sums go to a scratch
//     slab per split and are added in a fixed order by the consumer, so results do not depend on timing.
//   * Workgroup ids are remapped so that the row blocks of one weight band run on the same XCD and share its L2,
//     and so that the row blocks which may be empty come last in the grid (see the kernel).
#include "mfma.hpp"

namespace sdlm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int XS_STRIDE = 72;   // bf16 elements per LDS row of the activation slice (64 + 8 padding)

bool mfma_supported(const sdlm_model_cfg *m)
{
    return m->dtype == 1 && m->head_dim == 128 && m->hidden % 64 == 0 && m->ffn % 64 == 0 &&
           (m->n_q_heads * m->head_dim) % 64 == 0 && m->n_q_heads / m->n_kv_heads <= 64;
}
size_t mfma_pad_n(size_t N) { return (N + 31) / 32 * 32; }
size_t mfma_packed_elems(bool packed, size_t N, size_t K) { return (packed ? mfma_pad_n(N) : N) * K; }

// ------------------------------------------------------------------------------------------------ weight packing
// dst tile order: [n/32][k/16][lane][8] with lane = (n % 32) + 32 * ((k % 16) / 8).
__global__ void pack_mfma_k(bf16_t *dst, const bf16_t *src, int N, int K, int dst_row0, int interleave)
{
    const int KS = K / 16;
    size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 8-element group
    size_t total = (size_t)((N + 31) / 32) * KS * 64;
    if (g >= total) return;
    int lane = (int)(g & 63);
    size_t t = g >> 6;
    int ks = (int)(t % KS), nt = (int)(t / KS);
    int n = nt * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) v = *(const uint4 *)(src + (size_t)n * K + k);
    int dtile = interleave == 0 ? dst_row0 / 32 + nt : 2 * nt + (interleave - 1);
    *(uint4 *)(dst + (((size_t)dtile * KS + ks) * 64 + lane) * 8) = v;
}

void launch_pack_mfma(hipStream_t s, void *dst, const void *src, int N, int K, int dst_row0, int, int interleave)
{
    size_t total = (size_t)((N + 31) / 32) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_mfma_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (bf16_t *)dst, (const bf16_t *)src, N, K, dst_row0, interleave);
}

// ------------------------------------------------------------------------------------------------ GEMM
struct MfmaArgs {
    const bf16_t *X, *Wp, *bias;
    float *Yf;          // STORE_F32 / RESID destination, or split-k slabs
    bf16_t *Yt;         // SWIGLU destination
    float *logits;      // LM head: optional [rows, N] logits
    float4 *lm_part;    // LM head: [n_blocks][max_rows] partial (max, sum, entropy sum, argmax bits)
    const int32_t *pR;
    int max_rows, N, K, n_tiles, n_blocks, m_blocks, splits, stages_per_split, n_out;   // n_out: row length of the destination
    int m_sure;         // row blocks below this index certainly hold rows; they come first in the grid
    int rows_sure;      // rows below this index certainly exist (host-known lower bound of the device row count)
    size_t slab;        // elements between split-k slabs
    float scale;
};

enum { EPI_LMHEAD = 4 };

__device__ inline float silu_f(float v) { return v / (1.0f + __expf(-v)); }

// The largest tile keeps two register sets of weights instead of three so that accumulators + operands fit in 256
// registers: two workgroups then share a compute unit and one's barrier and load waits are covered by the other.
template <int MT, int NT> constexpr int w_sets() { return (MT >= 4) ? 2 : 3; }

// WV wavefronts per workgroup: 4, or 8 (a 128-row x 512-column tile whose activation slice is staged once for eight
// wavefronts instead of once for four: fewer bytes through the compute unit's load path per MFMA).
template <int MT, int NT, int EPI, int WV = 4>
__global__ __launch_bounds__(WV * 64, (WV == 8 ? 1 : (MT == 4 ? 2 : 1))) void gemm_mfma_k(MfmaArgs a)
{
    static_assert(WV == 4 || (WV == 8 && MT % 2 == 0), "eight wavefronts stage two 32-row sub-tiles per load round");
    __shared__ __attribute__((aligned(16))) bf16_t Xs[2][MT * 32][XS_STRIDE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps the weight stream's base in SGPRs
    // workgroup id -> tile.  The grid has two parts: the row blocks that certainly hold rows (mblk < m_sure), then the
    // others, which usually exit at once; mixing them would leave the compute units that draw an empty block idle.
    // Within a part, ids that land on one XCD (id % 8) get consecutive tiles, the row blocks of one weight band first.
    const int n_first = a.n_blocks * a.splits * a.m_sure, first8 = (n_first + 7) & ~7;
    int mblk, rest;
    if ((int)blockIdx.x < first8) {
        const int per = first8 >> 3, t = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
        if (t >= n_first) return;
        mblk = t % a.m_sure; rest = t / a.m_sure;
    } else {
        const int bid = blockIdx.x - first8, m_rest = a.m_blocks - a.m_sure;
        const int per = (gridDim.x - first8) >> 3, t = (bid & 7) * per + (bid >> 3);
        if (t >= a.n_blocks * a.splits * m_rest) return;
        mblk = a.m_sure + t % m_rest; rest = t / m_rest;
    }
    const int split = rest % a.splits, nblk = rest / a.splits;
    const int m0 = mblk * MT * 32;
    // A row block that lies entirely below the host-known row bound does not wait for the device-side row count: its
    // first operand requests go out at once (the count is one more memory round trip at the head of the kernel).
    const int R = m0 + MT * 32 <= a.rows_sure ? a.rows_sure : min(*a.pR, a.max_rows);
    if (m0 >= R) return;
    const int KS = a.K >> 4, S = a.K >> 6;
    const int s_begin = split * a.stages_per_split, s_end = min(S, s_begin + a.stages_per_split);
    if (s_begin >= s_end) return;

    // Addresses are (wave-uniform base) + (32-bit per-lane offset): the loads then take their base from SGPRs and
    // no address register is ever the destination of a load still in flight.
    const bf16_t *wp[NT];
    int ntile[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        ntile[nt] = (nblk * WV + wave) * NT + nt;
        int tl = min(ntile[nt], a.n_tiles - 1);
        wp[nt] = a.Wp + ((size_t)tl * KS) * 512;
    }
    const uint32_t wlane = lane * 8;
    // activation slice: MT*32 rows x 64 k = MT*256 16-byte chunks, XC per thread (a round of loads covers XR rows)
    constexpr int XR = WV * 8, XC = MT * 32 / XR;
    const int xrow = tid >> 3, xchunk = tid & 7;
    uint32_t xoff[XC];
#pragma unroll
    for (int i = 0; i < XC; ++i) xoff[i] = (uint32_t)min(m0 + i * XR + xrow, R - 1) * (uint32_t)a.K + xchunk * 8;

    f32x16 acc[NT][MT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nt][mt][v] = 0.f;

    // Software pipeline.  Small tiles (MT < 4): three rotating weight register sets, the weights of slice s+2 and the
    // activations of slice s+1 are requested at the top of slice s (the loop is unrolled by three so that the sets keep
    // static names).  128-row tiles: two weight sets and one activation operand set, so that accumulators + operands
    // fit in 256 registers and two workgroups share a compute unit; the loads of slice s+1 are spread over slice s.
    // In both, the activations go registers -> LDS at the bottom of the slice, and activation loads are issued before
    // weight loads: the counter that orders returns is in program order, so waiting for the (L2-hot) activations
    // leaves the (HBM) weight loads in flight.
    bf16x8 w0[NT][4], w1[NT][4], w2[w_sets<MT, NT>() == 3 ? NT : 1][4];
    u32x4 xr[XC];
    const int s_last = s_end - 1;
#define SDLM_LOAD_W(dst, stage)                                                                                   \
    {                                                                                                             \
        const size_t so_ = (size_t)min((stage), s_last) * 4 * 512;                                                \
        /* in the order the next slice's k-steps consume them */                                                  \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                         \
            _Pragma("unroll") for (int nt = 0; nt < NT; ++nt) dst[nt][ks] = *(const bf16x8 *)(wp[nt] + so_ + ks * 512 + wlane); \
    }
#define SDLM_LOAD_X(stage)                                                                                        \
    {                                                                                                             \
        const size_t xo_ = (size_t)min((stage), s_last) * 64;                                                     \
        _Pragma("unroll") for (int i = 0; i < XCA_; ++i) xr[i] = *(const u32x4 *)(a.X + xo_ + xoff[i]);          \
    }
    constexpr int WSETS = w_sets<MT, NT>();
    const int brow = lane & 31, bk = (lane >> 5) * 8;
/* ---- three weight sets (small tiles): one k-step = request the LDS operands of the next k-step, run this k-step's
   MFMAs, and pin that order; the slice's global loads are issued at its top */
#define SDLM_KSTEP(WC, ks, has_next)                                                                              \
    {                                                                                                             \
        if (has_next) {                                                                                           \
            _Pragma("unroll") for (int mt = 0; mt < MTA_; ++mt)                                                  \
                bn_[mt] = *(const bf16x8 *)&Xs[buf][mt * 32 + brow][((ks) + 1) * 16 + bk];                        \
        }                                                                                                         \
        _Pragma("unroll") for (int mt = 0; mt < MTA_; ++mt)                                                      \
            _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                                    \
                acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WC[nt][ks], bc_[mt], acc[nt][mt], 0, 0, 0); \
        __builtin_amdgcn_sched_group_barrier(0x100, (has_next) ? MTA_ : 0, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, MTA_ * NT, 0);                                                \
        _Pragma("unroll") for (int mt = 0; mt < MTA_; ++mt) bc_[mt] = bn_[mt];                                   \
    }
#define SDLM_STAGE3(WC, WN, stage)                                                                                \
    {                                                                                                             \
        SDLM_LOAD_X((stage) + 1);                                                                                 \
        SDLM_LOAD_W(WN, (stage) + 2);                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        bf16x8 bc_[MT], bn_[MT];                                                                                  \
        _Pragma("unroll") for (int mt = 0; mt < MTA_; ++mt) bc_[mt] = *(const bf16x8 *)&Xs[buf][mt * 32 + brow][bk]; \
        __builtin_amdgcn_sched_group_barrier(0x100, MTA_, 0);                                                     \
        SDLM_KSTEP(WC, 0, 1) SDLM_KSTEP(WC, 1, 1) SDLM_KSTEP(WC, 2, 1) SDLM_KSTEP(WC, 3, 0)                       \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        _Pragma("unroll") for (int i = 0; i < XCA_; ++i) *(u32x4 *)&Xs[buf ^ 1][i * XR + xrow][xchunk * 8] = xr[i]; \
        buf ^= 1;                                                                                                 \
        __syncthreads();                                                                                          \
    }
/* ---- two weight sets (128-row tiles): a single activation operand set bq_; each fragment is re-read in place
   right after the MFMAs that used it (slot = the MFMAs of one 32-row sub-tile at one k-step).  The slice is pipelined
   across its own boundary so that the MFMA stream never waits for LDS:
     k-steps 0, 1   MFMAs; the weight loads of the next slice dealt out over the slots (the load unit never holds the
                    wavefront up)
     publish        the activations of the next slice (requested a whole slice ago) go registers -> the other LDS buffer
     k-step 2       MFMAs; the activation loads of the slice after next, one per slot
     barrier        the other buffer is complete; nobody reads this slice's buffer after k-step 2 (the fragments of
                    k-step 3 are already in registers)
     k-step 3       MFMAs; each fragment register is refilled with the next slice's first fragment from the other buffer
   The next slice therefore starts with its operands in registers, and the LDS writes complete under k-step 2. */
#define SDLM_SLOT(WC, ks, mt, SRC, koff, vm)                                                                      \
    if constexpr ((mt) < MTA_) {                                                                                  \
        _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                                        \
            acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WC[nt][ks], bq_[mt], acc[nt][mt], 0, 0, 0);     \
        bq_[mt] = *(const bf16x8 *)&Xs[SRC][(mt) * 32 + brow][(koff) + bk];                                       \
        __builtin_amdgcn_sched_group_barrier(0x020, (vm), 0);                                                     \
        __builtin_amdgcn_sched_group_barrier(0x008, NT, 0);                                                       \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                        \
    }
/* weight loads of slot i of the 2 MTA_ slots of k-steps 0 and 1: 4 NT loads spread evenly */
#define SDLM_WVM(i) (((i) + 1) * 4 * NT / (2 * MTA_) - (i) * 4 * NT / (2 * MTA_))
#define SDLM_KSTEP2(WC, ks, SRC, koff, VM)                                                                        \
    SDLM_SLOT(WC, ks, 0, SRC, koff, VM(0)) SDLM_SLOT(WC, ks, 1, SRC, koff, VM(1)) SDLM_SLOT(WC, ks, 2, SRC, koff, VM(2)) \
    SDLM_SLOT(WC, ks, 3, SRC, koff, VM(3)) SDLM_SLOT(WC, ks, 4, SRC, koff, VM(4)) SDLM_SLOT(WC, ks, 5, SRC, koff, VM(5))
#define SDLM_VM_W0(mt) SDLM_WVM(mt)
#define SDLM_VM_W1(mt) SDLM_WVM(MTA_ + (mt))
#define SDLM_VM_ONE(mt) ((mt) < XCA_ ? 1 : 0)
#define SDLM_VM_NONE(mt) 0
#define SDLM_STAGE2(WC, WN, stage)                                                                                \
    {                                                                                                             \
        SDLM_LOAD_W(WN, (stage) + 1);                                                                             \
        SDLM_KSTEP2(WC, 0, buf, 16, SDLM_VM_W0) SDLM_KSTEP2(WC, 1, buf, 32, SDLM_VM_W1)                           \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        _Pragma("unroll") for (int i = 0; i < XCA_; ++i) *(u32x4 *)&Xs[buf ^ 1][i * XR + xrow][xchunk * 8] = xr[i]; \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        SDLM_LOAD_X((stage) + 2);                                                                                 \
        SDLM_KSTEP2(WC, 2, buf, 48, SDLM_VM_ONE)                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        __syncthreads();                                                                                          \
        SDLM_KSTEP2(WC, 3, buf ^ 1, 0, SDLM_VM_NONE)                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        buf ^= 1;                                                                                                 \
    }
/* The whole k loop for a row block of which only the first MTA_VALUE 32-row sub-tiles hold rows (the last block of
   a launch is usually ragged): the empty sub-tiles' loads, LDS traffic and MFMAs are not issued at all.  Full
   triples (pairs) of slices run without any branch inside the loop (a conditional stage would make the compiler
   drain all outstanding loads at the loop head); the remaining slices are peeled. */
#define SDLM_MAIN(MTA_VALUE)                                                                                      \
    {                                                                                                             \
        constexpr int MTA_ = MTA_VALUE, XCA_ = (MTA_VALUE * 32 + XR - 1) / XR;   /* live sub-tiles; load rounds that cover them */ \
        int buf = 0;                                                                                              \
        SDLM_LOAD_X(s_begin);                                                                                     \
        SDLM_LOAD_W(w0, s_begin);                                                                                 \
        if (WSETS == 3) SDLM_LOAD_W(w1, s_begin + 1);                                                             \
        _Pragma("unroll") for (int i = 0; i < XCA_; ++i) *(u32x4 *)&Xs[0][i * XR + xrow][xchunk * 8] = xr[i];    \
        __syncthreads();                                                                                          \
        bf16x8 bq_[MT];                                                                                           \
        if constexpr (WSETS == 2) {   /* the pipelined slice expects its first fragments and the next activations */ \
            SDLM_LOAD_X(s_begin + 1);                                                                             \
            _Pragma("unroll") for (int mt = 0; mt < MTA_; ++mt) bq_[mt] = *(const bf16x8 *)&Xs[0][mt * 32 + brow][bk]; \
        }                                                                                                         \
        int s = s_begin;                                                                                          \
        if constexpr (WSETS == 3) {                                                                               \
            for (; s + 3 <= s_end; s += 3) {                                                                      \
                SDLM_STAGE3(w0, w2, s)                                                                            \
                SDLM_STAGE3(w1, w0, s + 1)                                                                        \
                SDLM_STAGE3(w2, w1, s + 2)                                                                        \
            }                                                                                                     \
            if (s < s_end) {                                                                                      \
                SDLM_STAGE3(w0, w2, s)                                                                            \
                if (s + 1 < s_end) SDLM_STAGE3(w1, w0, s + 1)                                                     \
            }                                                                                                     \
        } else {                                                                                                  \
            for (; s + 2 <= s_end; s += 2) {                                                                      \
                SDLM_STAGE2(w0, w1, s)                                                                            \
                SDLM_STAGE2(w1, w0, s + 1)                                                                        \
            }                                                                                                     \
            if (s < s_end) SDLM_STAGE2(w0, w1, s)                                                                 \
        }                                                                                                         \
    }
    const int mt_act = min(MT, (R - m0 + 31) >> 5);   // >= 1: m0 < R
    if constexpr (MT == 6) {
        if (mt_act == 6) SDLM_MAIN(6) else if (mt_act == 5) SDLM_MAIN(5) else if (mt_act == 4) SDLM_MAIN(4) else if (mt_act == 3) SDLM_MAIN(3)
        else if (mt_act == 2) SDLM_MAIN(2) else SDLM_MAIN(1)
    } else if constexpr (MT == 4) {
        if (mt_act == 4) SDLM_MAIN(4) else if (mt_act == 3) SDLM_MAIN(3) else if (mt_act == 2) SDLM_MAIN(2) else SDLM_MAIN(1)
    } else if constexpr (MT == 2) {
        if (mt_act == 2) SDLM_MAIN(2) else SDLM_MAIN(1)
    } else {
        SDLM_MAIN(1)
    }
#undef SDLM_MAIN
#undef SDLM_STAGE3
#undef SDLM_STAGE2
#undef SDLM_KSTEP
#undef SDLM_KSTEP2
#undef SDLM_SLOT
#undef SDLM_WVM
#undef SDLM_VM_W0
#undef SDLM_VM_W1
#undef SDLM_VM_ONE
#undef SDLM_VM_NONE
#undef SDLM_LOAD_W
#undef SDLM_LOAD_X

    // accumulator element v of lane l: output feature 8*(v/4) + 4*(l/32) + v%4 of the tile, activation row l%32
    const int fbase = (lane >> 5) * 4;
    if (EPI == EPI_STORE_F32 || EPI == EPI_RESID) {
        float *dst = a.Yf + (a.splits > 1 ? (size_t)split * a.slab : 0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (ntile[nt] >= a.n_tiles) continue;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                int r = m0 + mt * 32 + brow;
                if (r >= R) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int n = ntile[nt] * 32 + q * 8 + fbase;
                    if (n >= a.N) continue;
                    float4 v = make_float4(acc[nt][mt][q * 4], acc[nt][mt][q * 4 + 1], acc[nt][mt][q * 4 + 2], acc[nt][mt][q * 4 + 3]);
                    float4 *p = (float4 *)(dst + (size_t)r * a.n_out + n);
                    if (EPI == EPI_STORE_F32) {
                        if (a.bias && split == 0) {
                            v.x += bf16_to_f(a.bias[n]); v.y += bf16_to_f(a.bias[n + 1]);
                            v.z += bf16_to_f(a.bias[n + 2]); v.w += bf16_to_f(a.bias[n + 3]);
                        }
                        *p = v;
                    } else if (a.splits > 1) {
                        *p = v;
                    } else {
                        float4 o = *p;
                        o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
                        *p = o;
                    }
                }
            }
        }
    } else if (EPI == EPI_SWIGLU) {
        // the fused matrix alternates 32-row tiles of gate and up: tiles (2j, 2j+1) belong to features 32j..32j+31
        static_assert(EPI != EPI_SWIGLU || NT == 2, "gate and up tiles must sit in one wavefront");
        const int j = ntile[0] >> 1;
        if (ntile[0] + 1 < a.n_tiles + 1 && ntile[0] < a.n_tiles) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                int r = m0 + mt * 32 + brow;
                if (r >= R) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int n = j * 32 + q * 8 + fbase;
                    if (n >= a.N) continue;
                    float o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = silu_f(acc[0][mt][q * 4 + e]) * acc[NT - 1][mt][q * 4 + e];
                    *(uint2 *)(a.Yt + (size_t)r * a.n_out + n) = make_uint2(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]));
                }
            }
        }
    } else {
        // LM head: logits of this workgroup's 128*NT vocabulary entries -> per-row (max, argmax, sum exp, entropy sum)
        __shared__ float sm_m[WV][MT * 32];
        __shared__ int sm_a[WV][MT * 32];
        __shared__ float sm_s[WV][MT * 32], sm_e[WV][MT * 32];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int r = m0 + mt * 32 + brow;
            float m = -INFINITY;
            int arg = 0;   // stays a valid id even if every logit is NaN
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int n = ntile[nt] * 32 + (v >> 2) * 8 + fbase + (v & 3);
                    float z = acc[nt][mt][v] * a.scale;
                    acc[nt][mt][v] = z;
                    if (n < a.N) {
                        if (a.logits && r < R) a.logits[(size_t)r * a.N + n] = z;
                        if (z > m || (z == m && n < arg)) { m = z; arg = n; }
                    }
                }
            float om = __shfl_xor(m, 32);
            int oa = __shfl_xor(arg, 32);
            if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
            if (lane < 32) { sm_m[wave][mt * 32 + lane] = m; sm_a[wave][mt * 32 + lane] = arg; }
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float m = sm_m[0][mt * 32 + brow];
#pragma unroll
            for (int w = 1; w < WV; ++w) m = fmaxf(m, sm_m[w][mt * 32 + brow]);
            float S = 0.f, E = 0.f;
            if (m > -INFINITY) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int n = ntile[nt] * 32 + (v >> 2) * 8 + fbase + (v & 3);
                        if (n < a.N) {
                            float dlt = acc[nt][mt][v] - m, e = __expf(dlt);
                            S += e;
                            E += e * dlt;
                        }
                    }
            }
            S += __shfl_xor(S, 32);
            E += __shfl_xor(E, 32);
            if (lane < 32) { sm_s[wave][mt * 32 + lane] = S; sm_e[wave][mt * 32 + lane] = E; }
        }
        __syncthreads();
        for (int i = tid; i < MT * 32; i += WV * 64) {
            int r = m0 + i;
            if (r >= R) continue;
            float m = sm_m[0][i];
            int arg = sm_a[0][i];
            float S = sm_s[0][i], E = sm_e[0][i];
            for (int w = 1; w < WV; ++w) {
                if (sm_m[w][i] > m || (sm_m[w][i] == m && sm_a[w][i] < arg)) { m = sm_m[w][i]; arg = sm_a[w][i]; }
                S += sm_s[w][i];
                E += sm_e[w][i];
            }
            a.lm_part[(size_t)nblk * a.max_rows + r] = make_float4(m, S, E, __int_as_float(arg));
        }
    }
}

// x[r, :] += sum over split slabs (fixed order)
__global__ __launch_bounds__(256) void reduce_slabs_k(float *x, const float *part, int splits, size_t slab, int n, const int32_t *pR, int max_rows)
{
    int r = blockIdx.x;
    if (r >= min(*pR, max_rows)) return;
    for (int c = threadIdx.x * 4; c < n; c += 1024) {
        float4 o = *(float4 *)(x + (size_t)r * n + c);
        for (int s = 0; s < splits; ++s) {
            float4 v = *(const float4 *)(part + s * slab + (size_t)r * n + c);
            o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
        }
        *(float4 *)(x + (size_t)r * n + c) = o;
    }
}

// Combine the LM head's per-block partials of one row: overall arg-max (lowest index on ties), and with
// M = max_i m_i:  S = sum_i S_i e^{m_i - M},  E = sum_i e^{m_i - M} (E_i + S_i (m_i - M)).
__global__ __launch_bounds__(256) void lm_combine_k(const float4 *part, int n_blocks, int max_rows, const int32_t *p_rows, int V, int conf_fn,
                                                    int32_t *ids, float *conf)
{
    int r = blockIdx.x;
    if (r >= min(*p_rows, max_rows)) return;
    __shared__ float sm[4];
    __shared__ int sa[4];
    __shared__ float red[4];
    float m = -INFINITY;
    int arg = 0;
    for (int i = threadIdx.x; i < n_blocks; i += 256) {
        float4 p = part[(size_t)i * max_rows + r];
        int a = __float_as_int(p.w);
        if (p.x > m || (p.x == m && a < arg)) { m = p.x; arg = a; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        float om = __shfl_xor(m, o);
        int oa = __shfl_xor(arg, o);
        if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
    }
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = m; sa[threadIdx.x >> 6] = arg; }
    __syncthreads();
    m = sm[0]; arg = sa[0];
    for (int w = 1; w < 4; ++w)
        if (sm[w] > m || (sm[w] == m && sa[w] < arg)) { m = sm[w]; arg = sa[w]; }
    float S = 0.f, E = 0.f;
    for (int i = threadIdx.x; i < n_blocks; i += 256) {
        float4 p = part[(size_t)i * max_rows + r];
        float dm = p.x - m, f = __expf(dm);
        S += p.y * f;
        E += f * (p.z + p.y * dm);
    }
    for (int o = 32; o > 0; o >>= 1) { S += __shfl_xor(S, o); E += __shfl_xor(E, o); }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = S; red[threadIdx.x >> 6] = E; }
    __syncthreads();
    if (threadIdx.x == 0) {
        S = sm[0] + sm[1] + sm[2] + sm[3];
        E = red[0] + red[1] + red[2] + red[3];
        ids[r] = arg;
        conf[r] = conf_fn == 0 ? 1.0f / S : 1.0f - (logf(S) - E / S) / logf((float)V);
    }
}

// ------------------------------------------------------------------------------------------------ gate/up for <= 32 rows
// The step of a single sequence has at most 2D <= 32 rows, and the gate/up projection cannot be split along k between
// workgroups (SiLU(gate) * up needs complete sums): the tiled kernel above would run it as N/128 workgroups, far too
// few to keep the weight stream busy.  Here a workgroup owns one 32-feature block (its gate tile and its up tile),
// its four wavefronts each take a quarter of k, and the quarters are added in wavefront order through LDS.  Both
// operands come straight from global memory in the MFMA operand order: the weights as a contiguous run, the rows
// (at most 32 x K, shared by every workgroup, so served by L2) 16 bytes per lane and k step; rows beyond the live
// ones repeat the last row and their results are dropped.  Loads are issued eight k steps at a time into two register
// sets: sixteen k steps (48 KB per wavefront) are in flight before the first MFMA.
constexpr int SK_U = 8, SK_W = 4;   // k steps per register set; wavefronts (measured: eight wavefronts are slower)

__global__ __launch_bounds__(SK_W * 64) void swiglu_skinny_k(MfmaArgs a)
{
    __shared__ float part[SK_W][2][16][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = blockIdx.x;   // features 32j .. 32j+31: tiles 2j (gate) and 2j+1 (up) of the fused matrix
    const int KS = a.K >> 4, per = (KS + SK_W - 1) / SK_W;
    const int k_begin = wave * per, k_end = min(KS, k_begin + per);
    const bf16_t *wg = a.Wp + ((size_t)(2 * j) * KS) * 512 + lane * 8, *wu = wg + (size_t)KS * 512;
    bf16x8 g0[SK_U], u0[SK_U], x0[SK_U], g1[SK_U], u1[SK_U], x1[SK_U];
#define SDLM_SK_LOAD_W(G, U, kb) \
    _Pragma("unroll") for (int u = 0; u < SK_U; ++u) { \
        const size_t o = (size_t)min((kb) + u, KS - 1) * 512; \
        G[u] = *(const bf16x8 *)(wg + o); U[u] = *(const bf16x8 *)(wu + o); }
#define SDLM_SK_LOAD_X(X, kb) \
    _Pragma("unroll") for (int u = 0; u < SK_U; ++u) X[u] = *(const bf16x8 *)(xp + min((kb) + u, KS - 1) * 16);
#define SDLM_SK_MMA(G, U, X, kb) \
    _Pragma("unroll") for (int u = 0; u < SK_U; ++u) if ((kb) + u < k_end) { \
        ag = __builtin_amdgcn_mfma_f32_32x32x16_bf16(G[u], X[u], ag, 0, 0, 0); \
        au = __builtin_amdgcn_mfma_f32_32x32x16_bf16(U[u], X[u], au, 0, 0, 0); }
    SDLM_SK_LOAD_W(g0, u0, k_begin)   // the weights do not wait for the row count
    if (k_begin + SK_U < k_end) { SDLM_SK_LOAD_W(g1, u1, k_begin + SK_U) }
    const int R = min(*a.pR, a.max_rows);
    if (R <= 0) return;
    const bf16_t *xp = a.X + (size_t)min(lane & 31, R - 1) * a.K + (lane >> 5) * 8;
    SDLM_SK_LOAD_X(x0, k_begin)
    if (k_begin + SK_U < k_end) { SDLM_SK_LOAD_X(x1, k_begin + SK_U) }
    f32x16 ag, au;
#pragma unroll
    for (int v = 0; v < 16; ++v) { ag[v] = 0.f; au[v] = 0.f; }
    for (int k0 = k_begin; k0 < k_end; k0 += 2 * SK_U) {
        SDLM_SK_MMA(g0, u0, x0, k0)
        if (k0 + 2 * SK_U < k_end) { SDLM_SK_LOAD_W(g0, u0, k0 + 2 * SK_U) SDLM_SK_LOAD_X(x0, k0 + 2 * SK_U) }
        SDLM_SK_MMA(g1, u1, x1, k0 + SK_U)
        if (k0 + 3 * SK_U < k_end) { SDLM_SK_LOAD_W(g1, u1, k0 + 3 * SK_U) SDLM_SK_LOAD_X(x1, k0 + 3 * SK_U) }
    }
#undef SDLM_SK_LOAD_W
#undef SDLM_SK_LOAD_X
#undef SDLM_SK_MMA
#pragma unroll
    for (int v = 0; v < 16; ++v) { part[wave][0][v][lane] = ag[v]; part[wave][1][v][lane] = au[v]; }
    __syncthreads();
    // accumulator element v of lane l: feature 8*(v/4) + 4*(l/32) + v%4 of the block, activation row l%32;
    // wavefront w finishes the elements EL*w .. EL*w + EL-1 of every lane: EL consecutive features of one row
    constexpr int EL = 16 / SK_W;
    static_assert(EL == 2 || EL == 4, "an output store is one or two bf16 pairs");
    const int row = lane & 31, v0 = wave * EL, n = j * 32 + (v0 >> 2) * 8 + (lane >> 5) * 4 + (v0 & 3);
    if (row >= R || n >= a.N) return;
    float o[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) {
        float gs = part[0][0][v0 + e][lane], us = part[0][1][v0 + e][lane];
#pragma unroll
        for (int w = 1; w < SK_W; ++w) { gs += part[w][0][v0 + e][lane]; us += part[w][1][v0 + e][lane]; }
        o[e] = silu_f(gs) * us;
    }
    bf16_t *dst = a.Yt + (size_t)row * a.n_out + n;
    if constexpr (EL == 4) *(uint2 *)dst = make_uint2(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]));
    else *(uint32_t *)dst = pack_bf16(o[0], o[EL - 1]);
}

// ------------------------------------------------------------------------------------------------ QKV + RoPE + K/V placement for <= 32 rows
// For steps of at most 32 rows (a single sequence, or a few with small blocks) the QKV projection, the rotation and the
// K/V placement are one kernel: such steps are bound by their kernel boundaries, and here the projection needs no split
// along k between workgroups, so its epilogue sees complete sums.  Same scheme as the gate/up kernel above: a workgroup
// owns two 32-feature tiles, here features [32 t, 32 t + 32) and the same range 64 further on of one head, i.e. both
// members of every rotate-half pair (i, i + d/2); its four wavefronts each take a quarter of k and the quarters are added
// in wavefront order through LDS.  The epilogue is the RoPE + K/V placement kernel's: queries and keys rotated at the
// row's position, a pending row's K/V to the cache slot of its position, any other row's to slot `kind` of its staging tile.
struct QkvSkinnyArgs {
    const bf16_t *X, *Wp, *bias;
    const int32_t *pR;
    int max_rows, K, Hq;
    bf16_t *q_out, *pool;
    KvGeom kg;
    RowMeta rm;
    SeqState st;
    const float2 *rope;
};

constexpr int QK_U = 12;   // k steps per register set: two sets cover a quarter of k = 1536 at once (one memory round trip)

__global__ __launch_bounds__(SK_W * 64) void qkv_rope_skinny_k(QkvSkinnyArgs a)
{
    __shared__ float part[SK_W][2][16][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int head = blockIdx.x >> 1, hh = blockIdx.x & 1;   // heads: Hq of q, then Hkv of k, then Hkv of v; hh: which 32 of the first 64 features
    const int KS = a.K >> 4, per = (KS + SK_W - 1) / SK_W;
    const int k_begin = wave * per, k_end = min(KS, k_begin + per);
    const bf16_t *wa = a.Wp + ((size_t)(head * 4 + hh) * KS) * 512 + lane * 8, *wb = wa + (size_t)2 * KS * 512;
    bf16x8 g0[QK_U], u0[QK_U], x0[QK_U], g1[QK_U], u1[QK_U], x1[QK_U];
#define SDLM_SK_LOAD_W(G, U, kb) \
    _Pragma("unroll") for (int u = 0; u < QK_U; ++u) { \
        const size_t o = (size_t)min((kb) + u, KS - 1) * 512; \
        G[u] = *(const bf16x8 *)(wa + o); U[u] = *(const bf16x8 *)(wb + o); }
#define SDLM_SK_LOAD_X(X, kb) \
    _Pragma("unroll") for (int u = 0; u < QK_U; ++u) X[u] = *(const bf16x8 *)(xp + min((kb) + u, KS - 1) * 16);
#define SDLM_SK_MMA(G, U, X, kb) \
    _Pragma("unroll") for (int u = 0; u < QK_U; ++u) if ((kb) + u < k_end) { \
        aa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(G[u], X[u], aa, 0, 0, 0); \
        ab = __builtin_amdgcn_mfma_f32_32x32x16_bf16(U[u], X[u], ab, 0, 0, 0); }
    SDLM_SK_LOAD_W(g0, u0, k_begin)   // the weights do not wait for the row count
    if (k_begin + QK_U < k_end) { SDLM_SK_LOAD_W(g1, u1, k_begin + QK_U) }
    const int R = min(*a.pR, a.max_rows);
    if (R <= 0) return;
    const int row = lane & 31, rr = min(row, R - 1);
    const int pos = a.rm.pos[rr], kind = a.rm.kind[rr], b = a.rm.seq[rr], stg = a.rm.stg[rr];   // requested with the operands
    const bf16_t *xp = a.X + (size_t)rr * a.K + (lane >> 5) * 8;
    SDLM_SK_LOAD_X(x0, k_begin)
    if (k_begin + QK_U < k_end) { SDLM_SK_LOAD_X(x1, k_begin + QK_U) }
    // what the epilogue needs beside the sums is requested now as well: rotation factors, bias, the page of a cached position
    const int d = a.kg.head_dim, half = d >> 1, Hk = a.kg.n_kv_heads;
    const int i0 = hh * 32 + wave * 8 + (lane >> 5) * 4;   // this lane's four features: index within the first half of the head
    const bool is_q = head < a.Hq, is_v = head >= a.Hq + Hk;
    float2 t[4];
    float blo[4] = {0.f, 0.f, 0.f, 0.f}, bhi[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        t[e] = is_v ? make_float2(1.f, 0.f) : a.rope[(size_t)pos * half + i0 + e];
        if (a.bias) { blo[e] = bf16_to_f(a.bias[head * d + i0 + e]); bhi[e] = bf16_to_f(a.bias[head * d + half + i0 + e]); }
    }
    int page = stg, slot = kind;
    if (!is_q && kind < 0) { page = a.st.page_table[(size_t)b * a.kg.pages_per_seq + pos / PAGE]; slot = pos % PAGE; }
    f32x16 aa, ab;
#pragma unroll
    for (int v = 0; v < 16; ++v) { aa[v] = 0.f; ab[v] = 0.f; }
    for (int k0 = k_begin; k0 < k_end; k0 += 2 * QK_U) {
        SDLM_SK_MMA(g0, u0, x0, k0)
        if (k0 + 2 * QK_U < k_end) { SDLM_SK_LOAD_W(g0, u0, k0 + 2 * QK_U) SDLM_SK_LOAD_X(x0, k0 + 2 * QK_U) }
        SDLM_SK_MMA(g1, u1, x1, k0 + QK_U)
        if (k0 + 3 * QK_U < k_end) { SDLM_SK_LOAD_W(g1, u1, k0 + 3 * QK_U) SDLM_SK_LOAD_X(x1, k0 + 3 * QK_U) }
    }
#undef SDLM_SK_LOAD_W
#undef SDLM_SK_LOAD_X
#undef SDLM_SK_MMA
#pragma unroll
    for (int v = 0; v < 16; ++v) { part[wave][0][v][lane] = aa[v]; part[wave][1][v][lane] = ab[v]; }
    __syncthreads();
    // accumulator element v of lane l: feature 8*(v/4) + 4*(l/32) + v%4 of the tile, activation row l%32; wavefront w
    // finishes elements 4w .. 4w+3 of every lane: four consecutive features of one row, and their partners 64 further on
    static_assert(SK_W == 4, "one wavefront finishes four consecutive features");
    if (row >= R) return;
    float lo[4], hi[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float sa = part[0][0][wave * 4 + e][lane], sb = part[0][1][wave * 4 + e][lane];
#pragma unroll
        for (int w = 1; w < SK_W; ++w) { sa += part[w][0][wave * 4 + e][lane]; sb += part[w][1][wave * 4 + e][lane]; }
        sa += blo[e]; sb += bhi[e];
        lo[e] = is_v ? sa : sa * t[e].x - sb * t[e].y;
        hi[e] = is_v ? sb : sb * t[e].x + sa * t[e].y;
    }
    if (is_q) {
        bf16_t *q = a.q_out + ((size_t)row * a.Hq + head) * d + i0;
        *(uint2 *)q = make_uint2(pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]));
        *(uint2 *)(q + half) = make_uint2(pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3]));
        return;
    }
    if (page < 0) return;   // unbacked position: only reachable after a reported pool exhaustion
    const int hk = is_v ? head - a.Hq - Hk : head - a.Hq;
    bf16_t *tile = a.pool + a.kg.tile(page, hk);
    if (!is_v) {
        // k_off(slot, i) keeps eight consecutive features of a slot together: i0 is a multiple of four
        *(uint2 *)(tile + k_off(slot, i0)) = make_uint2(pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]));
        *(uint2 *)(tile + k_off(slot, i0 + half)) = make_uint2(pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3]));
    } else {
        bf16_t *Vb = tile + PAGE * d;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            Vb[v_off(slot, i0 + e)] = f_to_bf16(lo[e]);
            Vb[v_off(slot, i0 + half + e)] = f_to_bf16(hi[e]);
        }
    }
}

bool qkv_rope_skinny_applies(const sdlm_model_cfg *m, int max_rows)
{
    return mfma_supported(m) && max_rows <= 32 && m->head_dim == 128;
}

void launch_qkv_rope_skinny(hipStream_t s, const sdlm_model_cfg *m, const void *X, const void *w_packed, const void *bias, const int32_t *p_rows,
                            int max_rows, void *q_out, void *pool_layer, const KvGeom &kg, const RowMeta &rm, const SeqState &st, const float2 *rope)
{
    QkvSkinnyArgs a;
    a.X = (const bf16_t *)X; a.Wp = (const bf16_t *)w_packed; a.bias = (const bf16_t *)bias; a.pR = p_rows;
    a.max_rows = max_rows; a.K = m->hidden; a.Hq = m->n_q_heads;
    a.q_out = (bf16_t *)q_out; a.pool = (bf16_t *)pool_layer; a.kg = kg; a.rm = rm; a.st = st; a.rope = rope;
    hipLaunchKernelGGL(qkv_rope_skinny_k, dim3(2 * (m->n_q_heads + 2 * m->n_kv_heads)), dim3(SK_W * 64), 0, s, a);
}

// ------------------------------------------------------------------------------------------------ launch policy
struct TileChoice { int MT, NT, splits, WV; };

static int sure_blocks(int rows, int min_rows, int MT)
{
    const int mb = (rows + MT * 32 - 1) / (MT * 32);
    if (min_rows <= 0) return mb;
    const int ms = (min_rows + MT * 32 - 1) / (MT * 32);
    return ms < 1 ? 1 : (ms > mb ? mb : ms);
}

// rows: bound of the launch (grid); min_rows: rows that are certainly there.
static TileChoice choose(int epi, int rows, int min_rows, int N, int K, size_t slab_room_floats)
{
    TileChoice c;
    c.MT = rows <= 32 ? 1 : rows <= 64 ? 2 : 4;
    c.NT = 2;
    c.WV = 4;
    // Gate/up with 129..192 certain rows and enough column blocks for one workgroup on (nearly) every compute unit: one
    // 192-row block per column block, so that no weight band is streamed by two workgroups.  (For the split-k
    // projections the same tile was measured: it wants more splits, and the slab traffic costs more than it saves.)
    if (epi == EPI_SWIGLU && min_rows > 128 && min_rows <= 192 && rows <= 384 && (N + 127) / 128 >= 192) c.MT = 6;
    if (epi != EPI_SWIGLU && epi != EPI_LMHEAD && c.MT < 4) {
        int mb = (rows + c.MT * 32 - 1) / (c.MT * 32);
        if ((long)((N + 255) / 256) * mb < 256) c.NT = 1;
    }
    c.splits = 1;
    if (epi == EPI_STORE_F32 || epi == EPI_RESID) {
        const int S = K / 64;
        const int cap_k = S / 4 > 0 ? S / 4 : 1;                             // at least 4 stages (256 deep) per split
        const long cap_m = (long)(slab_room_floats / ((size_t)rows * N));    // slabs must fit the scratch area
        auto clamp = [&](long sp) { sp = sp > cap_k ? cap_k : sp; sp = sp > cap_m ? cap_m : sp; sp = sp > 16 ? 16 : sp; return (int)(sp < 1 ? 1 : sp); };
        if (c.MT == 4) {
            // Workgroups are dealt out to the compute units round robin and two heavy ones on one unit take twice as
            // long as one: the fastest shape is one workgroup on as many units as possible, i.e. the largest split
            // count that keeps (column blocks x occupied row blocks x splits) within the 256 units.  The 256-wide
            // tile is the more efficient one; the 128-wide tile takes over when the wide one would leave more
            // than a quarter of the units without work.
            const long ms = sure_blocks(rows, min_rows, c.MT), nb2 = (N + 255) / 256, nb1 = (N + 127) / 128;
            int sp2 = clamp(256 / (nb2 * ms));
            if (K <= 4096 && sp2 > 3) sp2 = 3;   // short k loops: beyond three splits the slabs' write + read-back costs more than the idle units
            if (nb2 * ms * sp2 >= 192) { c.NT = 2; c.splits = sp2; }
            else { c.NT = 1; c.splits = clamp(256 / (nb1 * ms)); }
        } else {
            const long wgs = (long)((N + 128 * c.NT - 1) / (128 * c.NT)) * ((rows + c.MT * 32 - 1) / (c.MT * 32));
            c.splits = clamp((512 + wgs - 1) / wgs);
        }
    }
    // every split must own at least one 64-deep slice: with ceil(S / splits) slices per split the last splits of an
    // uneven division would be empty and their slabs never written
    if (c.splits > 1) {
        const int S = K / 64, per = (S + c.splits - 1) / c.splits;
        c.splits = (S + per - 1) / per;
    }
    // A launch that would put two 128 x 256 workgroups on every compute unit runs as 128 x 512 workgroups of eight wavefronts
    // (measured on the 7B gate/up shape: 2.5 % faster; with fewer workgroups than units the wider tile only idles units)
    if ((epi == EPI_SWIGLU || epi == EPI_RESID) && c.MT == 4 && c.NT == 2 && c.splits == 1) {   // (measured and not faster: the LM head, the prefill QKV projection)
        const long blocks4 = epi == EPI_SWIGLU ? (N + 127) / 128 : (N + 255) / 256;
        if (blocks4 * sure_blocks(rows, min_rows, c.MT) > 256) c.WV = 8;
    }
    return c;
}

template <int EPI>
static void launch_cfg(hipStream_t s, const TileChoice &c, MfmaArgs &a, int min_rows)
{
    a.n_blocks = (a.n_tiles + c.WV * c.NT - 1) / (c.WV * c.NT);
    a.m_blocks = (a.max_rows + c.MT * 32 - 1) / (c.MT * 32);
    a.splits = c.splits;
    int S = a.K / 64;
    a.stages_per_split = (S + c.splits - 1) / c.splits;
    a.m_sure = sure_blocks(a.max_rows, min_rows, c.MT);
    a.rows_sure = min_rows < 0 ? 0 : (min_rows > a.max_rows ? a.max_rows : min_rows);
    const int first = a.n_blocks * a.splits * a.m_sure, rest = a.n_blocks * a.splits * (a.m_blocks - a.m_sure);
    dim3 grid((first + 7) / 8 * 8 + (rest + 7) / 8 * 8), block(c.WV * 64);
#define SDLM_GO(MT_, NT_) hipLaunchKernelGGL((gemm_mfma_k<MT_, NT_, EPI>), grid, block, 0, s, a)
    if (EPI == EPI_SWIGLU || EPI == EPI_LMHEAD || c.NT == 2) {
        if (c.MT == 1) SDLM_GO(1, 2); else if (c.MT == 2) SDLM_GO(2, 2); else if (c.MT == 6 && EPI == EPI_SWIGLU) hipLaunchKernelGGL((gemm_mfma_k<(EPI == EPI_SWIGLU ? 6 : 4), 2, EPI>), grid, block, 0, s, a);
        else if (c.WV == 8) hipLaunchKernelGGL((gemm_mfma_k<4, 2, EPI, 8>), grid, block, 0, s, a);
        else SDLM_GO(4, 2);
    } else {
        if (EPI == EPI_STORE_F32 || EPI == EPI_RESID) {
            if (c.MT == 1) hipLaunchKernelGGL((gemm_mfma_k<1, 1, (EPI == EPI_STORE_F32 || EPI == EPI_RESID) ? EPI : EPI_RESID>), grid, block, 0, s, a);
            else if (c.MT == 2) hipLaunchKernelGGL((gemm_mfma_k<2, 1, (EPI == EPI_STORE_F32 || EPI == EPI_RESID) ? EPI : EPI_RESID>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((gemm_mfma_k<4, 1, (EPI == EPI_STORE_F32 || EPI == EPI_RESID) ? EPI : EPI_RESID>), grid, block, 0, s, a);
        }
    }
#undef SDLM_GO
}

void mfma_gemm_plan(int epi, int rows, int min_rows, int N, int K, size_t slab_room_floats, int *MT, int *NT, int *splits, int *wavefronts)
{
    TileChoice c = choose(epi, rows, min_rows, N, K, slab_room_floats);
    *MT = c.MT; *NT = c.NT; *splits = c.splits; *wavefronts = c.WV;
}

int launch_gemm_mfma(hipStream_t s, int epi, const GemmArgs &g, float *slabs, size_t slab_room_floats, bool defer_reduce)
{
    MfmaArgs a{};
    a.X = (const bf16_t *)g.X; a.Wp = (const bf16_t *)g.W; a.bias = (const bf16_t *)g.bias;
    a.Yf = g.Yf; a.Yt = (bf16_t *)g.Yt; a.pR = g.pR; a.max_rows = g.max_rows; a.N = g.N; a.K = g.K; a.scale = g.scale;
    a.n_out = g.N;
    a.n_tiles = epi == EPI_SWIGLU ? 2 * (int)(mfma_pad_n(g.N) / 32) : (int)(mfma_pad_n(g.N) / 32);
    if (epi == EPI_SWIGLU && g.max_rows <= 32) {
        hipLaunchKernelGGL(swiglu_skinny_k, dim3(a.n_tiles / 2), dim3(SK_W * 64), 0, s, a);
        return 1;
    }
    TileChoice c = choose(epi, g.max_rows, g.min_rows, g.N, g.K, slab_room_floats);
    a.slab = (size_t)g.max_rows * g.N;
    if (c.splits > 1) a.Yf = slabs;
    switch (epi) {
    case EPI_STORE_F32: launch_cfg<EPI_STORE_F32>(s, c, a, g.min_rows); break;
    case EPI_RESID: launch_cfg<EPI_RESID>(s, c, a, g.min_rows); break;
    default: launch_cfg<EPI_SWIGLU>(s, c, a, g.min_rows); break;
    }
    if (c.splits > 1 && epi == EPI_RESID && !defer_reduce)
        hipLaunchKernelGGL(reduce_slabs_k, dim3(g.max_rows), dim3(256), 0, s, g.Yf, slabs, c.splits, a.slab, g.N, g.pR, g.max_rows);
    return c.splits;   // slabs left for the consumer: always for STORE_F32, for RESID when defer_reduce
}

void launch_lmhead_mfma(hipStream_t s, const void *xhat, const void *w_packed, const int32_t *p_rows, int max_rows, int min_rows, int V, int h, float scale,
                        int conf_fn, float *logits_out, void *scratch, int32_t *ids, float *conf)
{
    MfmaArgs a{};
    a.X = (const bf16_t *)xhat; a.Wp = (const bf16_t *)w_packed; a.pR = p_rows; a.max_rows = max_rows; a.N = V; a.K = h; a.scale = scale;
    a.n_out = V; a.logits = logits_out; a.lm_part = (float4 *)scratch;
    a.n_tiles = (int)(mfma_pad_n(V) / 32);
    TileChoice c = choose(EPI_LMHEAD, max_rows, min_rows, V, h, 0);
    launch_cfg<EPI_LMHEAD>(s, c, a, min_rows);
    hipLaunchKernelGGL(lm_combine_k, dim3(max_rows), dim3(256), 0, s, (const float4 *)scratch, a.n_blocks, max_rows, p_rows, V, conf_fn, ids, conf);
}

size_t mfma_lm_scratch_bytes(int V, int max_rows) { return (size_t)((mfma_pad_n(V) / 32 + 7) / 8) * max_rows * sizeof(float4); }

}  // namespace sdlm
