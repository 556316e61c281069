// gfx950 kernels: partial attention computation (paper Alg. 2) over the scheduled
// task lists, and partial output reduction (Alg. 3) per query (Alg. 4).
//
// Partial attention.  One persistent 256-thread workgroup per (slot, KV head)
// walks the slot's task list.  A task is a KV slice of a node together with the
// query rows of the requests below the node: rows = requests x heads of the GQA
// group, gathered straight from the query tensor into MFMA operand registers
// (the on-chip query assembly of Sec. 4.1).  The four waves take interleaved
// 32-token blocks of the slice, so every K and V byte is fetched from HBM once
// per task and serves all rows.
//
// Per block a wave computes S^T = K Q^T (tokens x rows) with
// v_mfma_f32_16x16x32: K rows are the A operand, loaded as 16-byte pieces
// straight from the paged pool in operand layout; Q is the B operand.  The
// accumulator layout (lane = row, 4 tokens per lane and tile) is already the B
// operand layout of the second product O^T = V^T P^T once the eight tokens a
// lane holds are taken as its k-slice, so P never moves between lanes.  V is
// loaded with the matching token-to-lane map (lane group G takes tokens
// 4G..4G+3 of both 16-token tiles, 16 bytes = 8 channels each) and turned into
// the A operand by an 8x8 16-bit transpose inside each lane (v_perm_b32): no LDS
// traffic in the main loop.  A lane ends up owning 32 consecutive channels of
// one row.  Softmax statistics stay in fp32, in log2 units.
//
// At the end of a task the four waves' states are merged through LDS and wave 0
// writes the unnormalised partial output with (max, sum) per row.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace codec {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kHeadDim = 128;

template <int DT>
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c)
{
    if constexpr (DT == CODEC_DTYPE_FP16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                       __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                        __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Two fp32 values -> one dword of two 16-bit values (round to nearest even), lo in bits 0..15.
template <int DT>
__device__ __forceinline__ unsigned int pack2(float lo, float hi)
{
    if constexpr (DT == CODEC_DTYPE_FP16) {
        typedef __attribute__((ext_vector_type(2))) _Float16 h2;
        h2 v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(unsigned int, v);
    } else {
        typedef __attribute__((ext_vector_type(2))) __bf16 b2;
        b2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(unsigned int, v);
    }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ u32x4 ld16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }

// K and V registers of one 32-token block.
struct BlockRegs {
    u32x4 k[2][4];      // [16-token tile][32-channel k-step]: token = tile*16 + lane%16, channels 32*ks + 8*(lane/16)..+7
    u32x4 v[8];         // [e]: token = (e/4)*16 + 4*(lane/16) + e%4, channels 8*(lane%16)..+7
};

struct WaveCtx {
    const char *k_base;     // pool base + KV-head offset, bytes
    const char *v_base;
    int64_t page_bytes, token_bytes;
    const int32_t *pages;   // the slice's first page id
    int32_t kv_len;
    int32_t page_size;
    int l16, grp;
};

// Issue the loads of block `tb` (32 tokens).  Tiles that start beyond the slice are redirected to
// tile 0 so that no address leaves the slice's pages; their scores are masked later.
__device__ __forceinline__ void load_block(const WaveCtx &c, int tb, BlockRegs &r)
{
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        int tok0 = tb * 32 + j * 16;
        if (tok0 >= c.kv_len) tok0 = 0;
        const int pg = c.pages[tok0 / c.page_size];
        const int slot0 = tok0 % c.page_size;
        const int64_t tile_off = int64_t(pg) * c.page_bytes + int64_t(slot0) * c.token_bytes;
        const char *kp = c.k_base + tile_off + int64_t(c.l16) * c.token_bytes + c.grp * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) r.k[j][ks] = ld16(kp + ks * 64);
        const char *vp = c.v_base + tile_off + int64_t(c.grp * 4) * c.token_bytes + c.l16 * 16;
#pragma unroll
        for (int e = 0; e < 4; ++e) r.v[j * 4 + e] = ld16(vp + int64_t(e) * c.token_bytes);
    }
}

template <int DT, int NT>
struct RowState {
    f32x4 o[NT][8];     // [row tile][channel tile dt]: row = 16*nt + lane%16, channel = 32*(lane/16) + 8*e + dt
    float m[NT];        // running maximum, log2 units (same in the 4 lanes that share a row)
    float l[NT];        // this lane's share of the running sum of exponentials
};

template <int DT, int NT>
__device__ __forceinline__ void compute_block(const WaveCtx &c, int tb, BlockRegs &r,
                                              const u32x4 (&qb)[NT][4], RowState<DT, NT> &st,
                                              float scale_log2e)
{
    f32x4 s[2][NT];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) acc = mfma16<DT>(r.k[j][ks], qb[nt][ks], acc);
            s[j][nt] = acc;
        }

    const int valid = c.kv_len - tb * 32;           // >= 1
    if (valid < 32) {
        // ragged tail: tokens past the slice score -inf and their V rows count as zero
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool dead = j * 16 + c.grp * 4 + e >= valid;
                if (dead) {
                    r.v[j * 4 + e] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) s[j][nt][e] = -INFINITY;
                }
            }
    }

    u32x4 pb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float mx = fmaxf(fmaxf(fmaxf(s[0][nt][0], s[0][nt][1]), fmaxf(s[0][nt][2], s[0][nt][3])),
                         fmaxf(fmaxf(s[1][nt][0], s[1][nt][1]), fmaxf(s[1][nt][2], s[1][nt][3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(st.m[nt], mx * scale_log2e);
        const float alpha = fast_exp2(st.m[nt] - m_new);
        float p[2][4];
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                p[j][e] = fast_exp2(__builtin_fmaf(s[j][nt][e], scale_log2e, -m_new));
                sum += p[j][e];
            }
        st.l[nt] = st.l[nt] * alpha + sum;
        st.m[nt] = m_new;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) st.o[nt][dt] *= alpha;
        pb[nt] = u32x4{pack2<DT>(p[0][0], p[0][1]), pack2<DT>(p[0][2], p[0][3]),
                       pack2<DT>(p[1][0], p[1][1]), pack2<DT>(p[1][2], p[1][3])};
    }

    // 8x8 transpose inside the lane: v[e] holds 8 channels of token e, va[dt] holds 8 tokens of channel dt
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        const unsigned int sel = (dt & 1) ? 0x07060302u : 0x05040100u;
        u32x4 va;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            va[k] = __builtin_amdgcn_perm(r.v[2 * k + 1][dt >> 1], r.v[2 * k][dt >> 1], sel);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) st.o[nt][dt] = mfma16<DT>(va, pb[nt], st.o[nt][dt]);
    }
}

// exp2(a - m) with the convention that the side holding the maximum weighs exactly 1
// (keeps "-inf minus -inf" of a wave that saw no token out of the arithmetic).
__device__ __forceinline__ float weight(float a, float m) { return a == m ? 1.f : fast_exp2(a - m); }

template <int DT, int NT>
__device__ void run_task(const PacParams &P, const DevTask &t, int head, float *lds)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, grp = lane >> 4;
    const int rows = t.n_req * P.group;

    // query rows -> B operand registers
    u32x4 qb[NT][4];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = nt * 16 + l16;
        const bool live = row < rows;
        const int qi = live ? row / P.group : 0;
        const int hj = live ? row - qi * P.group : 0;
        const int req = P.node_q[t.q_off + qi];
        const char *qp = static_cast<const char *>(P.q)
                         + (int64_t(req) * P.h_q + int64_t(head) * P.group + hj) * (kHeadDim * 2) + grp * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qb[nt][ks] = live ? ld16(qp + ks * 64) : u32x4{0u, 0u, 0u, 0u};
    }

    WaveCtx c;
    c.k_base = static_cast<const char *>(P.k_pages) + int64_t(head) * P.head_stride * 2;
    c.v_base = static_cast<const char *>(P.v_pages) + int64_t(head) * P.head_stride * 2;
    c.page_bytes = P.page_stride * 2;
    c.token_bytes = P.token_stride * 2;
    c.pages = P.page_ids + t.page_off;
    c.kv_len = t.kv_len;
    c.page_size = P.page_size;
    c.l16 = l16;
    c.grp = grp;

    RowState<DT, NT> st;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        st.m[nt] = -INFINITY;
        st.l[nt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) st.o[nt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // software pipeline: the loads of the wave's next block are in flight while it computes this one
    const int nblk = (t.kv_len + 31) >> 5;
    BlockRegs ra, rb;
    int tb = wave;
    if (tb < nblk) load_block(c, tb, ra);
    while (tb < nblk) {
        int nb = tb + kWaves;
        if (nb < nblk) load_block(c, nb, rb);
        compute_block<DT, NT>(c, tb, ra, qb, st, P.scale_log2e);
        tb = nb;
        if (tb >= nblk) break;
        nb = tb + kWaves;
        if (nb < nblk) load_block(c, nb, ra);
        compute_block<DT, NT>(c, tb, rb, qb, st, P.scale_log2e);
        tb = nb;
    }

#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        st.l[nt] += __shfl_xor(st.l[nt], 16);
        st.l[nt] += __shfl_xor(st.l[nt], 32);
    }

    // merge the four waves: wave w hands its state to wave w-1 through LDS, 3 -> 2 -> 1 -> 0
    f32x4 *lds_o = reinterpret_cast<f32x4 *>(lds);                     // [NT][8][64]
    float *lds_m = lds + NT * 8 * 64 * 4;                               // [NT][64]
    float *lds_l = lds_m + NT * 64;
#pragma unroll 1
    for (int src = kWaves - 1; src >= 1; --src) {
        if (wave == src) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) lds_o[(nt * 8 + dt) * 64 + lane] = st.o[nt][dt];
                lds_m[nt * 64 + lane] = st.m[nt];
                lds_l[nt * 64 + lane] = st.l[nt];
            }
        }
        __syncthreads();
        if (wave == src - 1) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float m2 = lds_m[nt * 64 + lane], l2 = lds_l[nt * 64 + lane];
                const float mm = fmaxf(st.m[nt], m2);
                const float a = weight(st.m[nt], mm), b = weight(m2, mm);
                st.l[nt] = st.l[nt] * a + l2 * b;
                st.m[nt] = mm;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
                    st.o[nt][dt] = st.o[nt][dt] * a + lds_o[(nt * 8 + dt) * 64 + lane] * b;
            }
        }
        __syncthreads();
    }

    if (wave == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int row = nt * 16 + l16;
            if (row < rows) {
                const int64_t prow = int64_t(head) * P.part_rows + t.part_row_base + row;
                float *po = P.part_o + prow * kHeadDim + grp * 32;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    f32x4 lo = {st.o[nt][0][e], st.o[nt][1][e], st.o[nt][2][e], st.o[nt][3][e]};
                    f32x4 hi = {st.o[nt][4][e], st.o[nt][5][e], st.o[nt][6][e], st.o[nt][7][e]};
                    *reinterpret_cast<f32x4 *>(po + e * 8) = lo;
                    *reinterpret_cast<f32x4 *>(po + e * 8 + 4) = hi;
                }
                if (grp == 0) {
                    float2 ml = {st.m[nt], st.l[nt]};
                    *reinterpret_cast<float2 *>(P.part_ml + prow * 2) = ml;
                }
            }
        }
    }
}

template <int DT, int MAXNT>
__global__ void __launch_bounds__(kThreads, MAXNT >= 4 ? 1 : 2) pac_kernel(const PacParams P)
{
    __shared__ __attribute__((aligned(16))) float lds[MAXNT * 8 * 64 * 4 + MAXNT * 64 * 2];
    const int head = blockIdx.x % P.h_kv;
    const int slot = blockIdx.x / P.h_kv;
    const int t0 = P.slot_off[slot], t1 = P.slot_off[slot + 1];
#pragma unroll 1
    for (int i = t0; i < t1; ++i) {
        const DevTask t = P.tasks[P.slot_tasks[i]];
        const int rows = t.n_req * P.group;
        if (rows <= 16)
            run_task<DT, 1>(P, t, head, lds);
        else if (MAXNT >= 2 && rows <= 32)
            run_task<DT, (MAXNT >= 2 ? 2 : 1)>(P, t, head, lds);
        else if (MAXNT >= 4)
            run_task<DT, (MAXNT >= 4 ? 4 : 1)>(P, t, head, lds);
    }
}

// Partial output reduction (Alg. 3), n-ary: one wave per (request, query head) folds the request's
// partials in list order; each lane owns two channels.
template <int DT>
__global__ void __launch_bounds__(kThreads) merge_kernel(const MergeParams P)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (row >= P.num_requests * P.h_q) return;
    const int r = row / P.h_q, hq = row - r * P.h_q;
    const int head = hq / P.group, hj = hq - head * P.group;
    const int e0 = P.req_part_off[r], e1 = P.req_part_off[r + 1];
    float M = -INFINITY, L = 0.f, a0 = 0.f, a1 = 0.f;
    for (int e = e0; e < e1; ++e) {
        const int64_t prow = int64_t(head) * P.part_rows + P.req_part[e] + hj;
        const float2 ml = *reinterpret_cast<const float2 *>(P.part_ml + prow * 2);
        const float2 o = *reinterpret_cast<const float2 *>(P.part_o + prow * kHeadDim + lane * 2);
        const float mm = fmaxf(M, ml.x);
        const float wa = weight(M, mm), wb = weight(ml.x, mm);
        L = L * wa + ml.y * wb;
        a0 = a0 * wa + o.x * wb;
        a1 = a1 * wa + o.y * wb;
        M = mm;
    }
    const float inv = 1.f / L;
    unsigned int *out = static_cast<unsigned int *>(P.out) + int64_t(row) * (kHeadDim / 2) + lane;
    *out = pack2<DT>(a0 * inv, a1 * inv);
}

}  // namespace

int launch_pac(const PacParams &p, int dtype, int num_slots, int max_rows_in_plan, void *stream)
{
    const dim3 grid(unsigned(num_slots) * unsigned(p.h_kv)), block(kThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool wide = max_rows_in_plan > 32;
    if (dtype == CODEC_DTYPE_FP16) {
        if (wide) hipLaunchKernelGGL((pac_kernel<CODEC_DTYPE_FP16, 4>), grid, block, 0, s, p);
        else      hipLaunchKernelGGL((pac_kernel<CODEC_DTYPE_FP16, 2>), grid, block, 0, s, p);
    } else {
        if (wide) hipLaunchKernelGGL((pac_kernel<CODEC_DTYPE_BF16, 4>), grid, block, 0, s, p);
        else      hipLaunchKernelGGL((pac_kernel<CODEC_DTYPE_BF16, 2>), grid, block, 0, s, p);
    }
    return int(hipGetLastError());
}

int launch_merge(const MergeParams &p, int dtype, void *stream)
{
    const int rows = p.num_requests * p.h_q;
    const dim3 grid(unsigned((rows + kWaves - 1) / kWaves)), block(kThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == CODEC_DTYPE_FP16) hipLaunchKernelGGL((merge_kernel<CODEC_DTYPE_FP16>), grid, block, 0, s, p);
    else                           hipLaunchKernelGGL((merge_kernel<CODEC_DTYPE_BF16>), grid, block, 0, s, p);
    return int(hipGetLastError());
}

}  // namespace codec
