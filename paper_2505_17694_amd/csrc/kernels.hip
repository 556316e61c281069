// gfx950 kernels: partial attention computation (paper Alg. 2) over the scheduled
// task lists, and partial output reduction (Alg. 3) per query (Alg. 4).
//
// Partial attention.  One persistent workgroup per (slot, KV head) walks the
// slot's task list (256 threads in the narrow launch variant, 512 in the wide one).
// A task is a KV slice of a node together with the query rows of the requests
// below the node: rows = requests x heads of the GQA group, gathered straight from
// the query tensor into MFMA operand registers (the on-chip query assembly of
// Sec. 4.1).  Every K and V byte of the slice is fetched from HBM once per task and
// serves all rows.
//
// Arithmetic of one 32-token block, per wave: S^T = K Q^T (tokens x rows) on the
// matrix unit, K rows as the A operand, Q as the B operand.  The accumulator
// layout (a query row per lane column, several tokens per lane) is already the
// B-operand layout of the second product O^T = V^T P^T once the tokens a lane
// holds are taken as its k-slice, so P never moves between lanes; V is brought in
// with the matching token-to-lane map.  Softmax statistics stay in fp32, in log2
// units.
//
// Two task shapes share that arithmetic:
//  * "stream" (tasks of at most 16 rows, in both launch variants): 16 x 16 x 32
//    tiles; the waves of the workgroup take interleaved 32-token blocks of the
//    slice as one team, each with all rows; K and V go from HBM straight to
//    registers (no LDS in the loop; V becomes an A operand by an 8x8 16-bit
//    transpose inside each lane, v_perm_b32); the waves' states are merged through
//    LDS at the end.  Runs of short tasks are handed out one wave each instead.
//  * "dense" (tasks of 17..256 rows, wide variant): 32 x 32 x 16 tiles; eight waves
//    split the rows (32 each) and walk the slice together; blocks are copied HBM ->
//    LDS asynchronously into a ring of 16 KB slots (six or eight blocks in flight)
//    and read by all waves, V through transposing LDS reads (ds_read_b64_tr_b16).
//    Long slices under at most 128 rows put two waves on each row group, on
//    alternate blocks.
//
// K and V slices that a single task reads, in plans that read little twice, are
// loaded with the streaming (nontemporal) hint; the plan marks those tasks.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

#include "kernels.hpp"

namespace codec {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kHeadDim = 128;       // the dense path; the stream path and the reduction take the head
                                    // dimension D (64, 128 or 256) as a template parameter
constexpr int kNarrowWaves = 4;     // stream-only kernel variant: 4 waves, two workgroups per CU
constexpr int kWideWaves = 8;       // all task shapes: 8 waves (two per SIMD), one workgroup per CU
// Row tiles of the stream path in the narrow variant: one tile of 16 rows, or two (32 rows) with 64
// channels, where the accumulators of a second tile still fit the registers.
constexpr int stream_tiles(int d) { return d == 64 ? 2 : 1; }
constexpr int kMergeWaves = 2;      // reduction kernel (workgroups of two waves: measured against one and four, the
                                    // launch that follows a reduction starts up to 3 us sooner)
// Channel tiles of 16 that a stream task accumulates: 8 per 128 channels (with 64 channels half of each
// tile's rows are idle, see BlockRegs).
constexpr int channel_tiles(int d) { return d <= 128 ? 8 : d / 16; }
// LDS for merging the waves' states at the end of a stream task: W/2 states of NT row tiles
constexpr int merge_bytes(int waves, int nt, int d) { return (waves / 2) * (nt * channel_tiles(d) * 64 * 4 + nt * 64 * 2) * 4; }
// LDS of a wave that runs a task on its own: its 16 partial rows, fp32, 16 bytes between rows (the 16
// lanes of a row group then cover all banks).  256 channels: none (the rows go out as the lanes hold them).
constexpr int solo_stage_pitch(int d) { return d * 4 + 16; }
constexpr int solo_stage_bytes(int d) { return d <= 128 ? 16 * solo_stage_pitch(d) : 0; }

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

// acc + lo + hi of a dword of two 16-bit values (a two-element dot product with ones, exact products,
// fp32 sum).  Row sums are taken over the probabilities as rounded for the second product: the
// normaliser then matches the numerator, and a pair costs one instruction.
template <int DT>
__device__ __forceinline__ float add_pair(unsigned int packed, float acc)
{
    if constexpr (DT == CODEC_DTYPE_FP16) {
        typedef __attribute__((ext_vector_type(2))) _Float16 h2;
        const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, packed), ones, acc, false);
    } else {
        typedef __attribute__((ext_vector_type(2))) __bf16 b2;
        const b2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2, packed), ones, acc, false);
    }
}

__device__ __forceinline__ u32x4 ld16(const char *p) { return *reinterpret_cast<const u32x4 *>(p); }
// The same load with the streaming hint (the `nt` bit).  K and V slices that one task alone reads are
// fetched this way: bytes on their way through then do not displace each other, nor the slices that
// several tasks read, in the caches.  Slices with several readers keep plain loads: their re-reads live
// on cache hits.
__device__ __forceinline__ u32x4 ld16_once(const char *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// Accesses that are coherent across the whole device without cache maintenance: relaxed atomic
// accesses at device scope go past the caches that are not coherent at that scope (the `sc1` forms of
// the load and store instructions).  The single-launch mode moves partial results between workgroups
// of one launch through them; everywhere else partial results cross a kernel boundary and use plain
// accesses.
__device__ __forceinline__ void st8_device(float *p, float a, float b)
{
    const float2 v = {a, b};
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld8_device(const float *p)
{
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(float2, v);
}
// 16 bytes of a partial row: plain (the row is read by a later launch) or device-coherent
__device__ __forceinline__ void st16_partial(float *p, f32x4 v, bool coherent)
{
    if (coherent) {
        st8_device(p, v[0], v[1]);
        st8_device(p + 2, v[2], v[3]);
    } else {
        *reinterpret_cast<f32x4 *>(p) = v;
    }
}
__device__ __forceinline__ void st8_partial(float *p, float a, float b, bool coherent)
{
    if (coherent) st8_device(p, a, b);
    else          *reinterpret_cast<float2 *>(p) = float2{a, b};
}

// The lane index as a value the optimiser cannot trace back to the thread id.  Each task path derives
// its lane constants (operand addresses, row and channel positions) from it, which keeps them inside
// the path: hoisted out of the task loop they would stay live across all paths and cost the dense
// path, which needs nearly every register, a dozen spills.
__device__ __forceinline__ int opaque_lane()
{
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));
    return lane;
}

// Slice being processed: wave-uniform values only, so that addresses are SGPR base + 32-bit lane offset.
struct SliceCtx {
    const char *k_head;         // K pool + KV-head offset
    const char *v_head;
    const int32_t *pages;       // page ids of the slice, first page first
    uint32_t page_bytes;
    uint32_t token_bytes;
    int32_t kv_len;
    int32_t page_shift;         // log2(page_size)
    int32_t page_mask;
    int32_t read_once;          // no other task reads this slice
};

// Page ids are read through the scalar data path (s_load_dword, a read-only access): a vector load
// would sit in the same in-order return queue as the K/V traffic, and waiting for it would drain every
// prefetched block.  The page table does not change while a launch runs, so the load goes through a
// pointer to the constant address space; with a wave-uniform index the compiler then picks the scalar
// path and places the wait at the first use, which lets callers load an id a whole step ahead.
__device__ __forceinline__ int uniform_load(const int32_t *p, int index)
{
    typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
    return ((const_i32_ptr)(uintptr_t)p)[uint32_t(__builtin_amdgcn_readfirstlane(index))];
}

// Byte offset of a page slot: page id `pg`, token slot `slot` inside the page (wave-uniform).
__device__ __forceinline__ int64_t page_offset(const SliceCtx &c, int pg, int slot)
{
    return int64_t(uint64_t(uint32_t(pg)) * c.page_bytes + uint64_t(uint32_t(slot) * c.token_bytes));
}

// K and V registers of one 32-token block (stream path), head dimension D.
template <int D>
struct BlockRegs {
    static constexpr int KS = D / 32;                   // k-steps of the scores
    static constexpr int VU = D <= 128 ? 1 : D / 128;   // 16-byte V pieces per token and lane
    u32x4 k[2][KS];     // [tile][k-step]: token = tile*16 + lane%16, channels 32*ks + 8*(lane/16)..+7
    u32x4 v[8][VU];     // [e][u]: token = (e/4)*16 + 4*(lane/16) + e%4, channels 128*u + 8*(lane%16)..+7;
                        // D = 64: lanes 8..15 repeat the pieces of lanes 0..7 (their rows of the
                        // accumulated tiles stand for channels that do not exist and are never stored)
    uint32_t visible;   // masked tasks: bit t = the lane's row sees token t of the block
};

// Issue the loads of block `tb`.  A tile that starts beyond the slice is not loaded (its registers are
// cleared; its scores are masked later): no address leaves the slice's pages, and the sixteen load
// instructions of a block, each of which holds a place in the CU's queue of memory instructions in
// flight whatever it fetches, become eight for the last tile of a ragged slice and for one-token
// nodes.  ONCE: with the streaming hint.
template <bool ONCE, int D>
__device__ __forceinline__ void load_block(const SliceCtx &c, int tb, uint32_t koff, uint32_t voff, BlockRegs<D> &r,
                                           bool masked, const uint32_t *mask_row)
{
    // the word of the row's visibility mask for this block (a slice with masks starts at token 0 of its
    // node; a row without a mask sees everything)
    if (masked) r.visible = mask_row ? mask_row[tb] : 0xFFFFFFFFu;
    int tok[2], pg[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        tok[j] = tb * 32 + j * 16;
        pg[j] = tok[j] < c.kv_len ? uniform_load(c.pages, tok[j] >> c.page_shift) : 0;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (j == 1 && tok[j] >= c.kv_len) {     // wave-uniform: the slice ends inside the first tile
#pragma unroll
            for (int ks = 0; ks < BlockRegs<D>::KS; ++ks) r.k[j][ks] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int u = 0; u < BlockRegs<D>::VU; ++u) r.v[j * 4 + e][u] = u32x4{0u, 0u, 0u, 0u};
            continue;
        }
        const int64_t off = page_offset(c, pg[j], tok[j] & c.page_mask);
        const char *kt = c.k_head + off;
        const char *vt = c.v_head + off;
#pragma unroll
        for (int ks = 0; ks < BlockRegs<D>::KS; ++ks)
            r.k[j][ks] = ONCE ? ld16_once(kt + koff + ks * 64) : ld16(kt + koff + ks * 64);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int u = 0; u < BlockRegs<D>::VU; ++u) {
                const char *p = vt + size_t(e) * c.token_bytes + voff + u * 256;
                r.v[j * 4 + e][u] = ONCE ? ld16_once(p) : ld16(p);
            }
    }
}

// Initial reference of a row.  Finite, so that a block in which a row sees no token at all (every score
// -inf under its visibility mask) yields exp2(-inf - m) = 0 and not exp2(-inf + inf); so low that the
// first finite score raises the reference and wipes (multiplies by exp2 of -1e30) whatever it scaled.
constexpr float kNoReference = -1e30f;

template <int NT, int D>
struct RowState {
    static constexpr int CT = channel_tiles(D);
    f32x4 o[NT][CT];    // [row tile][dt]: row = 16*nt + lane%16; channel of component e is
                        // 128*(dt/8) + 32*(lane/16) + 8*e + dt%8
    float m[NT];        // reference subtracted before exponentiation, log2 units (same in the 4 lanes
                        // that share a row); kNoReference until the row has seen a score above -inf
    float l[NT];        // the lane's share of the row sum; the row sum after finish()

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            m[nt] = kNoReference;
            l[nt] = 0.f;
#pragma unroll
            for (int dt = 0; dt < CT; ++dt) o[nt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // each lane summed its own 8 tokens per block: the four lanes of a row are added up
    __device__ __forceinline__ void finish()
    {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            l[nt] += __shfl_xor(l[nt], 16);
            l[nt] += __shfl_xor(l[nt], 32);
        }
    }
};

// ---- one 32-token block of online softmax, in pieces so that callers can interleave them ---------
//
// The reference m of a row is allowed to lag behind the row's true running maximum by up to kLag
// (log2 units): softmax is invariant to the reference, and with the lag bounded every exponential
// stays <= 2^kLag, well inside fp16/bf16 and fp32 range.  A block therefore only needs each lane's own
// maximum over its 8 scores and one wave-wide vote; the cross-lane maximum and the rescaling of the
// accumulators run only when some row's scores outgrow the lag (always on a wave's first block,
// rarely afterwards).
constexpr float kLag = 8.f;

// Scores of tokens past `valid` become -inf (ragged last block of a slice).
template <int NT>
__device__ __forceinline__ void mask_scores(f32x4 (&s)[2][NT], int valid, int grp)
{
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool dead = j * 16 + grp * 4 + e >= valid;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) s[j][nt][e] = dead ? -INFINITY : s[j][nt][e];
        }
}

// Scores of tokens the row does not see become -inf (visibility mask, Sec. 4.1): bit t of `visible` is
// token t of the block.
template <int NT>
__device__ __forceinline__ void mask_invisible(f32x4 (&s)[2][NT], uint32_t visible, int grp)
{
    static_assert(NT == 1, "one mask word per lane: one row per lane");
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool seen = (visible >> (j * 16 + grp * 4 + e)) & 1u;
            s[j][0][e] = seen ? s[j][0][e] : -INFINITY;
        }
}

// V rows of tokens past `valid` count as zero (their memory may hold anything).
template <int VU>
__device__ __forceinline__ void mask_values(u32x4 (&v)[8][VU], int valid, int grp)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bool dead = (e >> 2) * 16 + grp * 4 + (e & 3) >= valid;
#pragma unroll
        for (int u = 0; u < VU; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) v[e][u][c] = dead ? 0u : v[e][u][c];
    }
}

// Each lane's maximum over its 8 scores per row tile, in log2 units.
template <int NT>
__device__ __forceinline__ void lane_maxima(const f32x4 (&s)[2][NT], float scale_log2e, float (&lm)[NT])
{
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float a = fmaxf(fmaxf(s[0][nt][0], s[0][nt][1]), s[0][nt][2]);
        a = fmaxf(fmaxf(a, s[0][nt][3]), s[1][nt][0]);
        a = fmaxf(fmaxf(a, s[1][nt][1]), s[1][nt][2]);
        lm[nt] = fmaxf(a, s[1][nt][3]) * scale_log2e;
    }
}

template <int NT, int D>
__device__ __forceinline__ bool outgrown(const float (&lm)[NT], const RowState<NT, D> &st)
{
    bool any = false;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) any |= lm[nt] > st.m[nt] + kLag;
    return any;
}

// Move every row's reference up to its true running maximum and rescale its accumulators.
template <int NT, int D>
__device__ __forceinline__ void raise_reference(const float (&lm)[NT], RowState<NT, D> &st)
{
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float mx = lm[nt];
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(st.m[nt], mx);
        const float alpha = fast_exp2(st.m[nt] - m_new);       // 0 on the first block (m = -inf)
        st.l[nt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < RowState<NT, D>::CT; ++dt) st.o[nt][dt] *= alpha;
        st.m[nt] = m_new;
    }
}

// P = exp2(scale * S - m), rounded to 16 bits in B-operand layout; the lane adds its 8 exponentials to
// its share of the row sum.
template <int DT, int NT, int D>
__device__ __forceinline__ void probabilities(const f32x4 (&s)[2][NT], RowState<NT, D> &st,
                                              float scale_log2e, u32x4 (&pb)[NT])
{
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float p[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                p[j][e] = fast_exp2(__builtin_fmaf(s[j][nt][e], scale_log2e, -st.m[nt]));
        pb[nt] = u32x4{pack2<DT>(p[0][0], p[0][1]), pack2<DT>(p[0][2], p[0][3]),
                       pack2<DT>(p[1][0], p[1][1]), pack2<DT>(p[1][2], p[1][3])};
#pragma unroll
        for (int d = 0; d < 4; ++d) st.l[nt] = add_pair<DT>(pb[nt][d], st.l[nt]);
    }
}

// O^T += V^T P^T for the channel tiles dt = 8*U + 4*HALF .. +3.  `vh[e]` holds dwords 2*HALF and
// 2*HALF+1 (channels 4*HALF .. 4*HALF+3 of the lane's 8) of token e's V row piece U; the 16-bit
// transpose inside each lane turns them into A operands.
template <int DT, int NT, int D, int U, int HALF>
__device__ __forceinline__ void accumulate_half(const unsigned int (&vh)[8][2], const u32x4 (&pb)[NT],
                                                RowState<NT, D> &st)
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const int dt = 8 * U + 4 * HALF + d;
        const unsigned int sel = (d & 1) ? 0x07060302u : 0x05040100u;
        u32x4 va;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            va[k] = __builtin_amdgcn_perm(vh[2 * k + 1][d >> 1], vh[2 * k][d >> 1], sel);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) st.o[nt][dt] = mfma16<DT>(va, pb[nt], st.o[nt][dt]);
    }
}

// Same for V row piece U of every token (16 bytes each) held in registers.
template <int DT, int NT, int D, int U>
__device__ __forceinline__ void accumulate_piece(const u32x4 (&v)[8][BlockRegs<D>::VU], const u32x4 (&pb)[NT],
                                                 RowState<NT, D> &st)
{
    unsigned int lo[8][2], hi[8][2];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        lo[e][0] = v[e][U][0]; lo[e][1] = v[e][U][1];
        hi[e][0] = v[e][U][2]; hi[e][1] = v[e][U][3];
    }
    accumulate_half<DT, NT, D, U, 0>(lo, pb, st);
    accumulate_half<DT, NT, D, U, 1>(hi, pb, st);
}
template <int DT, int NT, int D>
__device__ __forceinline__ void accumulate(const u32x4 (&v)[8][BlockRegs<D>::VU], const u32x4 (&pb)[NT],
                                           RowState<NT, D> &st)
{
    accumulate_piece<DT, NT, D, 0>(v, pb, st);
    if constexpr (BlockRegs<D>::VU > 1) accumulate_piece<DT, NT, D, 1>(v, pb, st);
    static_assert(BlockRegs<D>::VU <= 2, "head dimensions up to 256");
}

// Gather the wave's query rows (task rows row0 .. row0 + 16*NT) into B-operand registers.
template <int NT, int D>
__device__ __forceinline__ void gather_q(const PacParams &P, const DevTask &t, int head, int row0, int rows,
                                         int l16, int grp, u32x4 (&qb)[NT][D / 32])
{
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = row0 + nt * 16 + l16;
        const bool live = row < rows;
        const int qi = live ? row / P.group : 0;
        const int hj = live ? row - qi * P.group : 0;
        const int req = t.single_req >= 0 ? t.single_req : P.node_q[t.q_off + qi];
        const char *qp = static_cast<const char *>(P.q)
                         + (int64_t(req) * P.h_q + int64_t(head) * P.group + hj) * (D * 2) + grp * 16;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) qb[nt][ks] = live ? ld16(qp + ks * 64) : u32x4{0u, 0u, 0u, 0u};
    }
}

// The same for a wave that ran the task on its own, through its staging area in LDS.  In registers a
// lane holds 16-byte pieces of one row, so a store instruction of the wave would carry 16 bytes for each
// of 16 lines, and a task of `group` rows would take eight of them however few its rows; every
// vector-memory instruction takes a place in the CU's queue of instructions in flight, and a short task
// has few to spare.  Staged, the task's rows (they are neighbours in the partial array) go out 1 KB of
// consecutive memory per instruction: two instructions for four rows of 128 channels.
template <int D>
__device__ __forceinline__ void store_partial_staged(const PacParams &P, const DevTask &t, int head, int rows,
                                                     int lane, const RowState<1, D> &st, char *stage)
{
    static_assert(D <= 128, "staging area is sized for up to 128 channels");
    constexpr int PITCH = solo_stage_pitch(D), ROW = D * 4;
    const int l16 = lane & 15, grp = lane >> 4;
    const bool coherent = P.arrive != nullptr;
    char *put = stage + l16 * PITCH + grp * 128;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (grp * 32 + e * 8 >= D) continue;            // channels the head does not have
        const f32x4 lo = {st.o[0][0][e], st.o[0][1][e], st.o[0][2][e], st.o[0][3][e]};
        const f32x4 hi = {st.o[0][4][e], st.o[0][5][e], st.o[0][6][e], st.o[0][7][e]};
        *reinterpret_cast<f32x4 *>(put + e * 32) = lo;
        *reinterpret_cast<f32x4 *>(put + e * 32 + 16) = hi;
    }
    const int64_t prow = int64_t(head) * P.part_rows + t.part_row_base;
    if (grp == 0 && l16 < rows) st8_partial(P.part_ml + (prow + l16) * 2, st.m[0], st.l[0], coherent);
    __builtin_amdgcn_wave_barrier();                    // LDS serves a wave's accesses in order: no wait needed
    float *po = P.part_o + prow * D;
    const int bytes = rows * ROW;
#pragma unroll
    for (int i = 0; i < 16 * ROW / 1024; ++i) {
        if (i * 1024 >= bytes) break;                   // wave-uniform
        const int off = i * 1024 + lane * 16;
        if (off < bytes) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(stage + (off / ROW) * PITCH + off % ROW);
            st16_partial(po + off / 4, x, coherent);
        }
    }
    __builtin_amdgcn_wave_barrier();                    // the area is read before the wave's next task writes it
}

// Write one wave's rows of the partial result: unnormalised output, (reference, sum) per row.
template <int NT, int D>
__device__ __forceinline__ void store_partial(const PacParams &P, const DevTask &t, int head, int row0, int rows,
                                              int l16, int grp, const RowState<NT, D> &st)
{
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = row0 + nt * 16 + l16;
        if (row < rows) {
            const int64_t prow = int64_t(head) * P.part_rows + t.part_row_base + row;
            float *po = P.part_o + prow * D + grp * 32;
#pragma unroll
            for (int u = 0; u < BlockRegs<D>::VU; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (D < 128 && grp * 32 + e * 8 >= D) continue;     // channels the head does not have
                    const f32x4 lo = {st.o[nt][8 * u + 0][e], st.o[nt][8 * u + 1][e], st.o[nt][8 * u + 2][e], st.o[nt][8 * u + 3][e]};
                    const f32x4 hi = {st.o[nt][8 * u + 4][e], st.o[nt][8 * u + 5][e], st.o[nt][8 * u + 6][e], st.o[nt][8 * u + 7][e]};
                    st16_partial(po + u * 128 + e * 8, lo, P.arrive != nullptr);
                    st16_partial(po + u * 128 + e * 8 + 4, hi, P.arrive != nullptr);
                }
            if (grp == 0) st8_partial(P.part_ml + prow * 2, st.m[nt], st.l[nt], P.arrive != nullptr);
        }
    }
}

__device__ __forceinline__ SliceCtx make_ctx(const PacParams &P, const DevTask &t, int head)
{
    SliceCtx c;
    c.k_head = static_cast<const char *>(P.k_pages) + int64_t(head) * P.head_stride * 2;
    c.v_head = static_cast<const char *>(P.v_pages) + int64_t(head) * P.head_stride * 2;
    c.pages = P.page_ids + t.page_off;
    c.page_bytes = uint32_t(P.page_stride * 2);
    c.token_bytes = uint32_t(P.token_stride * 2);
    c.kv_len = t.kv_len;
    c.page_shift = P.page_shift;
    c.page_mask = (1 << P.page_shift) - 1;
    c.read_once = t.flags & kTaskReadOnce;
    return c;
}

// exp2(a - m) with the convention that the side holding the maximum weighs exactly 1
// (keeps "-inf minus -inf" of a wave that saw no token out of the arithmetic).
__device__ __forceinline__ float weight(float a, float m) { return a == m ? 1.f : fast_exp2(a - m); }

// ---- stream path: rows <= 16*NT (NT = 2 for 17 .. 32 rows of 64 channels, else 1), a team of W waves splits the tokens
// `wave` is the wave's index in its team.  A team of one wave (W = 1) uses no LDS and no barrier, so
// several such waves may work on different tasks at the same time.
template <int DT, bool ONCE, int NT, int W, int D>
__device__ void run_stream(const PacParams &P, const DevTask &t, int head, char *lds_raw, int wave,
                           char *stage = nullptr)      // W = 1, up to 128 channels: the wave's staging area
{
    constexpr int KS = D / 32, CT = channel_tiles(D);
    const int lane = opaque_lane();
    const int l16 = lane & 15, grp = lane >> 4;
    const int rows = t.n_req * P.group;

    u32x4 qb[NT][KS];
    gather_q<NT, D>(P, t, head, 0, rows, l16, grp, qb);
    const SliceCtx c = make_ctx(P, t, head);
    const uint32_t koff = uint32_t(l16) * c.token_bytes + grp * 16;
    const uint32_t voff = uint32_t(grp * 4) * c.token_bytes + (D < 128 ? (l16 & (D / 8 - 1)) : l16) * 16;

    // visibility mask of the lane's row, if the task has any (masked tasks hold at most 16 rows and are
    // never slices of a node: block tb of the task is word tb of the mask)
    const bool masked = (t.flags & kTaskMasked) != 0;
    const uint32_t *mask_row = nullptr;
    if (masked && l16 < rows) {
        const int off = P.nodeq_mask[t.q_off + l16 / P.group];
        if (off >= 0) mask_row = P.mask_words + off;
    }

    RowState<NT, D> st;
    st.clear();

    auto compute = [&](int tb, BlockRegs<D> &r) {
        f32x4 s[2][NT];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16<DT>(r.k[j][ks], qb[nt][ks], acc);
                s[j][nt] = acc;
            }
        const int valid = c.kv_len - tb * 32;
        if (valid < 32) {
            mask_scores<NT>(s, valid, grp);
            mask_values<BlockRegs<D>::VU>(r.v, valid, grp);
        }
        if constexpr (NT == 1) {            // tasks with masks are planned as tiles of at most 16 rows
            if (masked) mask_invisible<NT>(s, r.visible, grp);
        }
        float lm[NT];
        lane_maxima<NT>(s, P.scale_log2e, lm);
        if (__any(outgrown<NT, D>(lm, st))) raise_reference<NT, D>(lm, st);
        u32x4 pb[NT];
        probabilities<DT, NT, D>(s, st, P.scale_log2e, pb);
        accumulate<DT, NT, D>(r.v, pb, st);
    };

    // software pipeline: the loads of the wave's next block are in flight while it computes this one
    const int nblk = (t.kv_len + 31) >> 5;
    BlockRegs<D> ra, rb;
    int tb = wave;
    if (tb < nblk) load_block<ONCE, D>(c, tb, koff, voff, ra, masked, mask_row);
    while (tb < nblk) {
        int nb = tb + W;
        if (nb < nblk) load_block<ONCE, D>(c, nb, koff, voff, rb, masked, mask_row);
        compute(tb, ra);
        tb = nb;
        if (tb >= nblk) break;
        nb = tb + W;
        if (nb < nblk) load_block<ONCE, D>(c, nb, koff, voff, ra, masked, mask_row);
        compute(tb, rb);
        tb = nb;
    }

    st.finish();

    // merge the waves' states pairwise through LDS: waves [h, 2h) hand theirs to waves [0, h), h = W/2 .. 1
    constexpr int kState = NT * CT * 64 * 4 + NT * 64 * 2;             // floats per handed-over state
    float *lds = reinterpret_cast<float *>(lds_raw);
#pragma unroll 1
    for (int h = W / 2; h >= 1; h >>= 1) {
        if (wave >= h && wave < 2 * h) {
            float *base = lds + (wave - h) * kState;
            f32x4 *lo = reinterpret_cast<f32x4 *>(base);                // [NT][CT][64]
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int dt = 0; dt < CT; ++dt) lo[(nt * CT + dt) * 64 + lane] = st.o[nt][dt];
                base[NT * CT * 64 * 4 + nt * 64 + lane] = st.m[nt];
                base[NT * CT * 64 * 4 + NT * 64 + nt * 64 + lane] = st.l[nt];
            }
        }
        __syncthreads();
        if (wave < h) {
            const float *base = lds + wave * kState;
            const f32x4 *lo = reinterpret_cast<const f32x4 *>(base);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float m2 = base[NT * CT * 64 * 4 + nt * 64 + lane];
                const float l2 = base[NT * CT * 64 * 4 + NT * 64 + nt * 64 + lane];
                const float mm = fmaxf(st.m[nt], m2);
                const float a = weight(st.m[nt], mm), b = weight(m2, mm);
                st.l[nt] = st.l[nt] * a + l2 * b;
                st.m[nt] = mm;
#pragma unroll
                for (int dt = 0; dt < CT; ++dt)
                    st.o[nt][dt] = st.o[nt][dt] * a + lo[(nt * CT + dt) * 64 + lane] * b;
            }
        }
        __syncthreads();
    }
    if constexpr (W == 1 && NT == 1 && D <= 128) {
        store_partial_staged<D>(P, t, head, rows, lane, st, stage);
    } else {
        if (wave == 0) store_partial<NT, D>(P, t, head, 0, rows, l16, grp, st);
    }
}

// ---- dense path: 1..256 rows, the 8 waves split the rows (32 each) and share each block ------------
//
// Blocks travel HBM -> LDS without passing through registers (global_load_lds_dwordx4: every lane
// moves 16 bytes, a wave fills 1 KB of consecutive LDS).  A ring of kRing block slots (16 KB each:
// 32 K rows then 32 V rows of 256 B) keeps six (eight with two-block intervals) blocks in flight per
// workgroup.  Rows are stored unpadded; the 16-byte column index is XORed with a function of the row so
// that the operand reads spread over all banks.  The swizzle is applied on the global side: the lane that fills LDS
// column c of a row fetches column c ^ f(row).
//
// The compiler does not see these loads (inline asm), so the waits are explicit: loads complete in
// issue order, block b is in LDS once at most 2 * (blocks issued after b) of the wave's loads are
// outstanding, and the barrier that follows publishes all eight waves' parts.
constexpr int kRing = 10;                    // slots allocated; a path may cycle through fewer
constexpr int kBlockBytes = 16384;
constexpr int kRingBytes = kRing * kBlockBytes;
constexpr int kSplitBlocksMaxRows = 128;     // dense tasks up to this many rows, and at least
constexpr int kSplitBlocksMinLen = 1024;     // this many tokens: two waves per row group
// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding: bits 3:0 and 15:14)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

// One block's K piece and V piece for this wave: each lane fetches 16 bytes at gk + voff_k (gv + voff_v)
// and the wave's 64 pieces land in 1 KB of consecutive LDS at lds_addr (the V piece 8 KB behind).  M0
// holds the LDS address for the instruction and is put back afterwards.
__device__ __forceinline__ void dma16_pair(uint32_t lds_addr, uint32_t voff_k, uint32_t voff_v, const char *gk,
                                           const char *gv, int read_once)
{
    uint32_t m0_saved;
    if (read_once) {
        asm volatile("s_mov_b32 %0, m0\n\t"
                     "s_mov_b32 m0, %1\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %2, %4 nt\n\t"
                     "s_add_u32 m0, m0, 0x2000\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %3, %5 nt\n\t"
                     "s_mov_b32 m0, %0\n"
                     : "=&s"(m0_saved)
                     : "s"(lds_addr), "v"(voff_k), "v"(voff_v), "s"(gk), "s"(gv)
                     : "memory", "scc");
    } else {
        asm volatile("s_mov_b32 %0, m0\n\t"
                     "s_mov_b32 m0, %1\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %2, %4\n\t"
                     "s_add_u32 m0, m0, 0x2000\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %3, %5\n\t"
                     "s_mov_b32 m0, %0\n"
                     : "=&s"(m0_saved)
                     : "s"(lds_addr), "v"(voff_k), "v"(voff_v), "s"(gk), "s"(gv)
                     : "memory", "scc");
    }
}

// One 16-byte piece per lane from a per-lane address: lane i's piece lands at lds_addr + 16 * i.  Used for
// the query rows of a dense task, which are queued between the copies of K/V blocks: a load into
// registers there would have to be waited for by the compiler, which counts the copies as its own loads
// and would wait for all of them; through LDS the rows take the same asynchronous path as the blocks,
// no register is written behind the compiler's back, and the rows are read from LDS by ordinary loads
// once the hand-placed wait has passed.
__device__ __forceinline__ void dma16_rows(uint32_t lds_addr, const char *gp)
{
    uint32_t m0_saved;
    asm volatile("s_mov_b32 %0, m0\n\t"
                 "s_mov_b32 m0, %1\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, off\n\t"
                 "s_mov_b32 m0, %0\n"
                 : "=&s"(m0_saved)
                 : "s"(lds_addr), "v"(gp)
                 : "memory", "scc");
}

// ---- dense path with 32 query rows per wave ---------------------------------------------------------
//
// v_mfma_f32_32x32x16: A operand lane = (row lane%32, k-group lane/32), 8 k-values per lane; B operand
// lane = (column lane%32, k-group lane/32); result register r of lane (column lane%32, group lane/32)
// is row 8*(r/4) + 4*(lane/32) + r%4.  As in the 16-row tiles, S^T = K Q^T comes out with a query row
// per lane column, which is the layout the B operand of O^T += V^T P^T wants: register 8t + i of the
// scores becomes k-value i of k-step t, and the A operand (V^T) is read with the same token order.
// Compared with 16 x 16 x 32 tiles a block costs half as many matrix instructions for the same
// arithmetic; the path is bound by the instructions a wave can issue, not by the matrix unit.
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int DT>
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c)
{
    if constexpr (DT == CODEC_DTYPE_FP16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                       __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                        __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Keeps the computation of `x` where it is written (the compiler otherwise sinks work whose result
// is only used after the next barrier below that barrier).
__device__ __forceinline__ void pin(u32x4 &x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(float &x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(int &x) { asm volatile("" : "+v"(x)); }

// Roles of a wave in a dense task.  A wave with rows owns 32 of them; in the two live roles the halves
// of a step come in opposite orders, for the two waves of a SIMD.  Waves without rows only help moving
// blocks.  All eight waves run the same barriers.
//
// STRIDE = 1: a live wave takes every block (tasks of more than 128 rows, up to eight row groups; and
// short slices of any task, see run_dense32).
// STRIDE = 2: tasks of at most 128 rows have at most four row groups; waves w and w+4 (one SIMD) share
// group w, the first takes the even blocks, the second the odd ones, and their two states are merged
// through LDS when the slice is done.  An interval then covers two blocks.  Without the split a SIMD
// would hold a single computing wave and the other one would idle.
enum { kHelper = 0, kMatrixFirst = 1, kVectorFirst = 2 };

// One wave's share of a dense task: task rows row0 .. row0+31 (none for a helper).
template <int DT, int ROLE, int STRIDE>
__device__ __forceinline__ void dense32_wave(const PacParams &P, const DevTask &t, int head, char *lds,
                                             int wave, int row0, int rows)
{
    constexpr bool LIVE = ROLE != kHelper;
    static_assert(STRIDE == 1 || STRIDE == 2, "a row group is shared by one or two waves");
    // slots in use: an interval of two blocks wants a deeper ring to keep as many bytes in flight
    constexpr int RING = STRIDE == 2 ? kRing : 8;
    // the wave's blocks are first, first + STRIDE, ...
    const int first = (STRIDE == 2 && ROLE == kVectorFirst) ? 1 : 0;
    auto blk = [&](int k) { return first + k * STRIDE; };
    const int lane = opaque_lane();
    const int l32 = lane & 31, kg = lane >> 5;
    const int l16 = lane & 15, grp = lane >> 4;

    u32x4 qb[8];            // B operand of the scores: row l32, channels 16*ks + 8*kg .. +7
    f32x16 o[4];            // O^T: row l32, channel 32*ct + 8*(r/4) + 4*kg + r%4
    float m = -INFINITY;    // reference, log2 units, integer-valued (same in the two lanes of a row)
    float l4[4] = {0.f, 0.f, 0.f, 0.f};     // this lane's share of the row sum, in four partial sums
    if constexpr (LIVE) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[ct][r] = 0.f;
    }
    const SliceCtx c = make_ctx(P, t, head);

    // Asynchronous copies.  Wave w moves tokens 4w .. 4w+3 of every block, 1 KB of K and 1 KB of V;
    // lane (grp, l16) writes the 16-byte slot l16 of LDS row 4w + grp.  A K row keeps its 16-byte
    // column g in slot g ^ (token & 15), a V row in slot g ^ 4*(token & 3): the swizzles that make
    // the operand reads below free of bank conflicts (a transposing V read takes, per 32 lanes, 4 rows
    // x 64 bytes: the four rows must land in four different quarters of the 256 bytes of banks).
    const uint32_t lds_base = uint32_t(uintptr_t(lds));
    const int tok_w = wave * 4 + grp;
    const uint32_t voff_k = uint32_t(grp) * c.token_bytes + uint32_t((l16 ^ (tok_w & 15)) << 4);
    const uint32_t voff_v = uint32_t(grp) * c.token_bytes + uint32_t((l16 ^ ((tok_w & 3) << 2)) << 4);
    // a group of four tokens past the end of the slice is redirected to token 0 (its rows are masked
    // later) so that no address leaves the slice's pages
    auto first_token = [&](int bb) {
        const int tok0 = bb * 32 + wave * 4;
        return tok0 >= c.kv_len ? 0 : tok0;
    };
    auto page_issue = [&](int bb) { return uniform_load(c.pages, first_token(bb) >> c.page_shift); };
    auto dma_block = [&](int bb, int pg) {                              // pg: page id from page_issue(bb)
        const int64_t off = page_offset(c, pg, first_token(bb) & c.page_mask);
        const uint32_t slot = lds_base + uint32_t(bb % RING) * kBlockBytes + uint32_t(wave) * 1024;
        dma16_pair(slot, voff_k, voff_v, c.k_head + off, c.v_head + off, c.read_once);
    };

    // Operand reads.
    // K (A operand of the scores): lane (l32, kg) reads column 2*ks + kg of token row l32; with the
    // swizzle its address is the ks = 0 address with (ks << 5) XORed in.
    // V (A operand of the accumulation, channel tile ct, k-step t): ds_read_b64_tr_b16 hands lane i of a
    // 16-lane group column i of the 4 x 16 tile whose row k the group's lanes 4k .. 4k+3 address 8 bytes
    // apiece.  Lane group (kg, ch) = (lane/32, lane/16 % 2), lane (k, q) in it, addresses token
    // 16*t + 8*h + 4*kg + k, channels 32*ct + 16*ch + 4*q .. +3: two reads (h = 0, 1) give the lane its
    // channel 32*ct + lane%32 for the 8 tokens of its k-group.  ct is XORed into the address like ks.
    const uint32_t ka_lane = uint32_t(l32 * 256 + ((kg ^ (l32 & 15)) << 4));
    const int vk = l16 >> 2, vq = l16 & 3, vch = grp & 1;
    const int vrow = 4 * kg + vk;
    const uint32_t va_lane =
        uint32_t(8192 + vrow * 256 + ((((2 * vch + (vq >> 1)) ^ ((vrow & 3) << 2)) & 15) << 4) + 8 * (vq & 1));
    u32x4 kr[8];            // K operands of one block, by k-step
    u32x4 vr[4][2];         // V operands of one block, by channel tile and k-step
    auto key_base = [&](int bb) { return lds_base + uint32_t(bb % RING) * kBlockBytes + ka_lane; };
    auto value_base = [&](int bb) { return lds_base + uint32_t(bb % RING) * kBlockBytes + va_lane; };
    auto load_key = [&](uint32_t base, int ks) {                        // K operand of k-step ks
        kr[ks] = *reinterpret_cast<const u32x4 __attribute__((address_space(3))) *>(uintptr_t(base ^ uint32_t(ks << 5)));
    };
    typedef __attribute__((ext_vector_type(4))) short s16x4;
    typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;
    auto load_value = [&](uint32_t base, int ct, int tt) {              // V operand of channel tile ct, k-step tt
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t addr = (base ^ uint32_t(ct << 6)) + tt * 4096 + h * 2048;
            const s16x4 x = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_s16x4_ptr>(uintptr_t(addr)));
            const uint2 w = __builtin_bit_cast(uint2, x);
            vr[ct][tt][2 * h] = w.x;
            vr[ct][tt][2 * h + 1] = w.y;
        }
    };
    auto load_keys = [&](int bb) {
        const uint32_t base = key_base(bb);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) load_key(base, ks);
    };
    auto load_values = [&](int bb) {
        const uint32_t base = value_base(bb);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) load_value(base, ct, tt);
    };
    // tokens past `valid` count as zero in V (the slot may hold anything there, NaN patterns included)
    // and as -inf in the scores
    auto mask_values = [&](int valid) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int tok = 16 * tt + 8 * (d >> 1) + 4 * kg + 2 * (d & 1);  // low half; high half tok+1
                const unsigned int keep = (tok < valid ? 0x0000FFFFu : 0u) | (tok + 1 < valid ? 0xFFFF0000u : 0u);
#pragma unroll
                for (int ct = 0; ct < 4; ++ct) vr[ct][tt][d] &= keep;
            }
    };
    auto mask_scores32 = [&](f32x16 &s, int valid) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool dead = 8 * (r >> 2) + 4 * kg + (r & 3) >= valid;
            s[r] = dead ? -INFINITY : s[r];
        }
    };

    f32x16 s;               // scores: row l32, token 8*(r/4) + 4*kg + r%4
    u32x4 p[2];             // probabilities, B operand: k-step t holds registers 8t .. 8t+7 of the scores
    auto scores32 = [&]() {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = mfma32<DT>(kr[i], qb[i], acc);
        s = acc;
    };
    auto accumulate32 = [&]() {
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i & 3] = mfma32<DT>(vr[i & 3][i >> 2], p[i >> 2], o[i & 3]);
    };
    // The matrix half of a FULL step: O^T += V^T P^T of the block in vr and the scores of the block in
    // kr; the two alternate so that no instruction waits for the one before it.  With one wave per row
    // group (compute-bound tasks) each pair is followed by the LDS reads that refill the operand
    // registers it has just consumed (K of block kb, V of block vb): the reads are issued while the
    // matrix unit works on the pair.
    auto matrix_half = [&](int kb, int vb, auto after_first_pair) {
        const uint32_t kbase = key_base(kb), vbase = value_base(vb);
        // the wave in its matrix half goes first when both waves of the SIMD have an instruction ready:
        // measured, the other order starves the matrix instructions (1150 against 1010 clk per half)
        __builtin_amdgcn_s_setprio(3);
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            o[i & 3] = mfma32<DT>(vr[i & 3][i >> 2], p[i >> 2], o[i & 3]);
            acc = mfma32<DT>(kr[i], qb[i], acc);
            if constexpr (STRIDE == 1) {
                load_value(vbase, i & 3, i >> 2);
                load_key(kbase, i);
            }
            if (i == 0) after_first_pair();
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
        if constexpr (STRIDE == 2) {        // memory-bound tasks: measured faster with the reads in one go
            load_keys(kb);
            load_values(vb);
            __builtin_amdgcn_sched_barrier(0);
        }
        s = acc;
    };
    // The vector work of a block, in three pieces.  reference(): the lane's maximum over its 16 scores;
    // when a row has outgrown its reference by more than the lag, the reference moves up to the
    // (rounded-up) row maximum and everything accumulated against the old one is rescaled.
    // probabilities(t): P = exp2(scale * S - m) for k-step t in B-operand layout, and the lane's share
    // of the row sum.
    auto reference = [&]() {
        float a = __builtin_fmaxf(__builtin_fmaxf(s[0], s[1]), s[2]);
#pragma unroll
        for (int r = 3; r + 1 < 16; r += 2) a = __builtin_fmaxf(__builtin_fmaxf(a, s[r]), s[r + 1]);
        const float lm = __builtin_fmaxf(a, s[15]) * P.scale_log2e;
        if (__any(lm > m + kLag)) {
            const float mx = fmaxf(lm, __shfl_xor(lm, 32));
            const float m_new = __builtin_ceilf(fmaxf(m, mx));
            const float alpha = fast_exp2(m - m_new);                   // 0 on the first block (m = -inf)
#pragma unroll
            for (int d = 0; d < 4; ++d) l4[d] *= alpha;
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[ct][r] *= alpha;
            m = m_new;
        }
    };
    auto probabilities32 = [&](int tt) {
        float e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) e[i] = fast_exp2(__builtin_fmaf(s[8 * tt + i], P.scale_log2e, -m));
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            p[tt][d] = pack2<DT>(e[2 * d], e[2 * d + 1]);
            l4[d] = add_pair<DT>(p[tt][d], l4[d]);
        }
        pin(p[tt]);
    };

    // Common to all roles.  Blocks 0 .. 7 are requested up front; interval j (j = 0 .. nint-1) starts
    // with a barrier behind which blocks S*j+8 .. S*j+8+S-1 (S = STRIDE) are requested into the slots
    // that blocks S*j .. S*j+S-1 have left, so those are read from LDS before that barrier.  The LDS
    // reads of interval j reach up to block S*j + 3*S - 1, which must have landed at its barrier: each
    // wave issues 2 loads per block and loads complete in order, so a block has landed once at most
    // 2 * (blocks issued after it) loads are outstanding; near the end of the slice, where fewer blocks
    // follow, the wait is for everything.
    const int nblk = (t.kv_len + 31) >> 5;
    const int nint = (nblk + STRIDE - 1) / STRIDE - 1;                  // the same for every wave
    // Start of the task.  What the first matrix instruction waits for is a chain of dependent reads:
    // page ids and the rows' requests, then the first blocks and the query rows.  The two reads of a
    // stage are issued together; the query rows (32 rows of 32 bytes per instruction, the slowest
    // requests to issue) are queued behind the copies of the first 2S blocks only.  They travel through
    // LDS like the blocks (dma16_rows): each wave parks its 8 KB in the last four slots of the ring,
    // whose blocks are requested once every wave has taken its rows into registers, behind the barrier
    // that ends this start-up; the other blocks of the ring are requested right behind the rows.
    constexpr int EARLY = RING - 4;                                     // blocks requested ahead of that barrier
    static_assert(EARLY >= 2 * STRIDE && 8 * 8192 == 4 * kBlockBytes, "the rows' parking space is the last four slots");
    int pg_late[4];
    {
        int pg[RING];
#pragma unroll
        for (int d = 0; d < RING; ++d) pg[d] = page_issue(d < nblk ? d : 0);
        const char *qp = nullptr;
        bool live = false;
        if constexpr (LIVE) {
            const int row = row0 + l32;
            live = row < rows;
            const int qi = live ? row / P.group : row0 / P.group;       // a dead row reads row0's
            const int hj = live ? row - qi * P.group : row0 - qi * P.group;
            int req = t.single_req >= 0 ? t.single_req : P.node_q[t.q_off + qi];
            pin(req);                           // the wait for it stands here, ahead of the copies
            qp = static_cast<const char *>(P.q)
                 + (int64_t(req) * P.h_q + int64_t(head) * P.group + hj) * (kHeadDim * 2) + kg * 16;
        }
#pragma unroll
        for (int d = 0; d < 4; ++d) pg_late[d] = pg[EARLY + d];
#pragma unroll
        for (int d = 0; d < 2 * STRIDE; ++d)
            if (d < nblk) dma_block(d, pg[d]);
        const uint32_t park = lds_base + uint32_t(EARLY) * kBlockBytes + uint32_t(wave) * 8192;   // wave-uniform
        const uint32_t parked = park + uint32_t(lane) * 16;
        if constexpr (LIVE) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) dma16_rows(park + ks * 1024, qp + ks * 32);
        }
#pragma unroll
        for (int d = 2 * STRIDE; d < EARLY; ++d)
            if (d < nblk) dma_block(d, pg[d]);
        // loads complete in order: with at most the copies of blocks 2S .. EARLY-1 outstanding, blocks
        // 0 .. 2S-1 and the query rows have landed
        if (nblk >= EARLY) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * (EARLY - 2 * STRIDE)));
        else                __builtin_amdgcn_s_waitcnt(0x0F70);
        if constexpr (LIVE) {
            typedef const u32x4 __attribute__((address_space(3))) *lds_u32x4_ptr;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const u32x4 x = *reinterpret_cast<lds_u32x4_ptr>(uintptr_t(parked + ks * 1024));   // the piece this lane sent
                qb[ks] = live ? x : u32x4{0u, 0u, 0u, 0u};
            }
            // the rows are in registers before this wave passes the barrier below, behind which the
            // parking space is overwritten
            __builtin_amdgcn_s_waitcnt(0xC07F);
        }
    }
    int pg_next[STRIDE];                                                // pages of the blocks interval 0 requests
#pragma unroll
    for (int u = 0; u < STRIDE; ++u) pg_next[u] = page_issue(RING + u);
    __syncthreads();
#pragma unroll
    for (int d = 0; d < 4; ++d)
        if (EARLY + d < nblk) dma_block(EARLY + d, pg_late[d]);

    // more: blocks S*j+8 .. S*j+8+S-1 all exist
    auto wait_and_sync = [&](auto more) {
        if constexpr (decltype(more)::value) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * (RING - 3 * STRIDE)));
        else                                 __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();                    // blocks up to S*j+3S-1 are complete; everyone is done with block(s) S*j ..
    };
    auto request_blocks = [&](int j, auto more) {                       // any time inside interval j
        if constexpr (decltype(more)::value) {
#pragma unroll
            for (int u = 0; u < STRIDE; ++u) dma_block(STRIDE * j + RING + u, pg_next[u]);
#pragma unroll
            for (int u = 0; u < STRIDE; ++u) pg_next[u] = page_issue(STRIDE * (j + 1) + RING + u);
        } else if constexpr (STRIDE == 2) {
            if (2 * j + RING < nblk) dma_block(2 * j + RING, pg_next[0]);         // an odd block left over
        }
    };
    auto enter_interval = [&](int j, auto more) {                       // j < nint
        wait_and_sync(more);
        request_blocks(j, more);
    };
    using yes = std::true_type;
    using no = std::false_type;
    auto short_block = [&](int b) { return c.kv_len - b * 32; };        // valid tokens if below 32
    auto more_follow = [&](int j) { return STRIDE * j + RING + STRIDE - 1 < nblk; };

    if constexpr (LIVE) {
        // The wave's k-th block is b_k = blk(k), nmine of them.  Per block a vector half V(b_k) (scores
        // of the block -> probabilities) and a matrix half M(b_k) (accumulation of b_k, alternating with
        // the scores of b_k+1), in the order V(b_0) M(b_0) V(b_1) M(b_1) ...; right after M(b_k) has read
        // its operands the operands of M(b_k+1) (K of block b_k+2, V of block b_k+1) are requested from
        // LDS, to arrive during V(b_k+1).  A vector-first wave places the barrier of interval k before
        // V(b_k), a matrix-first wave before M(b_k): the two waves of a SIMD run in opposite phases,
        // one's matrix work beside the other's vector work.
        constexpr bool VFIRST = ROLE == kVectorFirst;
        const int nmine = nblk > first ? (nblk - first + STRIDE - 1) / STRIDE : 0;
        auto vector_half_of = [&](int b) {
            if (short_block(b) < 32) mask_scores32(s, short_block(b));
            reference();
            probabilities32(0);
            probabilities32(1);
        };
        // With one wave per row group the copies of the interval are requested from inside the matrix
        // half: their address arithmetic issues while the matrix unit works, instead of ahead of it.
        constexpr bool REQUEST_INSIDE = STRIDE == 1;
        auto matrix_half_and_loads = [&](int k, auto more) {            // M(b_k), k + 1 < nmine
            matrix_half(blk(k + 2), blk(k + 1), [&]() {
                if constexpr (REQUEST_INSIDE) request_blocks(k, more);
            });
            __builtin_amdgcn_sched_barrier(0);
        };
        auto interval = [&](int k, auto more) {
            wait_and_sync(more);
            if constexpr (!REQUEST_INSIDE) request_blocks(k, more);
            if (STRIDE == 1 || k + 1 < nmine) {                         // else: the other wave's last block only
                if constexpr (VFIRST) {
                    vector_half_of(blk(k));
                    __builtin_amdgcn_sched_barrier(0);
                    matrix_half_and_loads(k, more);
                } else {
                    matrix_half_and_loads(k, more);
                    vector_half_of(blk(k + 1));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        if (STRIDE == 1 || nmine > 0) {
            load_keys(blk(0));
            scores32();
            __builtin_amdgcn_sched_barrier(0);
            load_keys(blk(1));
            load_values(blk(0));
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!VFIRST) {
                vector_half_of(blk(0));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        int k = 0;
#pragma unroll 1
        for (; k < nint && more_follow(k); ++k) interval(k, yes{});
#pragma unroll 1
        for (; k < nint; ++k) interval(k, no{});
        if (STRIDE == 1 || nmine > 0) {
            const int last = blk(nmine - 1);
            if constexpr (VFIRST) vector_half_of(last);
            if (short_block(last) < 32) mask_values(short_block(last));
            accumulate32();
        }
    } else {
        int k = 0;
#pragma unroll 1
        for (; k < nint && more_follow(k); ++k) enter_interval(k, yes{});
#pragma unroll 1
        for (; k < nint; ++k) enter_interval(k, no{});
    }

    __syncthreads();                        // every block has been read: the ring is free
    float l = (l4[0] + l4[1]) + (l4[2] + l4[3]);
    if constexpr (STRIDE == 2) {
        // The odd-block wave hands its state to the even-block wave of its row group: 64 accumulator
        // registers, reference and sum share per lane, register-major so that a wave's store or load
        // covers consecutive words.
        float *x = reinterpret_cast<float *>(lds) + (wave & 3) * (66 * 64) + lane;
        if constexpr (ROLE == kVectorFirst) {
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) x[(ct * 16 + r) * 64] = o[ct][r];
            x[64 * 64] = m;
            x[65 * 64] = l;
        }
        __syncthreads();
        if constexpr (ROLE == kMatrixFirst) {
            const float m2 = x[64 * 64], l2 = x[65 * 64];
            const float m_new = fmaxf(m, m2);
            const float a1 = weight(m, m_new), a2 = weight(m2, m_new);
            l = l * a1 + l2 * a2;
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[ct][r] = o[ct][r] * a1 + x[(ct * 16 + r) * 64] * a2;
            m = m_new;
        }
    }

    // The partial rows go out through LDS: in registers a lane holds 16-byte pieces of one row, and a
    // store instruction of the wave would touch 32 rows with 32 bytes each (measured: 3.1 us to issue
    // the 128 KB of a 256-row task, the address unit taking one such piece about every two cycles).
    // Each wave writes its 32 x 128 floats into an area of its own (rows 528 bytes apart: 16 lanes
    // then cover all banks) and reads them back row by row: a store instruction covers two whole rows,
    // 1 KB of consecutive memory.  With two waves per row group the area is the one the hand-over
    // above has just used, and only its own wave touches it from here on.
    constexpr int kStageRow = 528, kStageWave = 66 * 64 * 4;
    static_assert(32 * kStageRow <= kStageWave && 8 * kStageWave <= kRingBytes, "staging areas fit the ring");
    if constexpr (ROLE == kMatrixFirst || (STRIDE == 1 && LIVE)) {
        l += __shfl_xor(l, 32);
        typedef f32x4 __attribute__((address_space(3))) *lds_f32x4_ptr;
        const uint32_t area = lds_base + uint32_t(STRIDE == 2 ? (wave & 3) : wave) * kStageWave;
        const uint32_t put = area + uint32_t(l32) * kStageRow + uint32_t(kg) * 16;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 x4 = {o[ct][4 * q], o[ct][4 * q + 1], o[ct][4 * q + 2], o[ct][4 * q + 3]};
                *reinterpret_cast<lds_f32x4_ptr>(uintptr_t(put + ct * 128 + q * 32)) = x4;
            }
        const int row = row0 + l32;
        if (row < rows && kg == 0) {
            const int64_t prow = int64_t(head) * P.part_rows + t.part_row_base + row;
            st8_partial(P.part_ml + prow * 2, m, l, P.arrive != nullptr);
        }
        const uint32_t get = area + uint32_t(kg) * kStageRow + uint32_t(l32) * 16;
        float *po = P.part_o + (int64_t(head) * P.part_rows + t.part_row_base + row0 + kg) * kHeadDim + l32 * 4;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const f32x4 x4 = *reinterpret_cast<lds_f32x4_ptr>(uintptr_t(get + j * 2 * kStageRow));
            if (row0 + 2 * j + kg < rows) st16_partial(po + j * 2 * kHeadDim, x4, P.arrive != nullptr);
        }
    }
    __syncthreads();                        // the staging areas (and the hand-over area) are free for the next task
}

// Dense task.  More than 128 rows: wave w owns rows 32w .. 32w+31; waves 4 .. 7 share their SIMDs with
// waves 0 .. 3 and run in the opposite phase.  Up to 128 rows: waves w and w+4 share rows 32w .. 32w+31
// and take alternate blocks, again in opposite phases; short slices, for which the hand-over at the end
// costs more than the overlap gains (about 1 us per task), keep one wave per row group.
template <int DT>
__device__ void run_dense32(const PacParams &P, const DevTask &t, int head, char *lds)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rows = t.n_req * P.group;
    if (rows > kSplitBlocksMaxRows || t.kv_len < kSplitBlocksMinLen) {
        const int row0 = wave * 32;
        if (row0 >= rows)  dense32_wave<DT, kHelper, 1>(P, t, head, lds, wave, 0, 0);
        else if (wave & 4) dense32_wave<DT, kVectorFirst, 1>(P, t, head, lds, wave, row0, rows);
        else               dense32_wave<DT, kMatrixFirst, 1>(P, t, head, lds, wave, row0, rows);
    } else {
        const int row0 = (wave & 3) * 32;
        if (row0 >= rows)  dense32_wave<DT, kHelper, 2>(P, t, head, lds, wave, 0, 0);
        else if (wave & 4) dense32_wave<DT, kVectorFirst, 2>(P, t, head, lds, wave, row0, rows);
        else               dense32_wave<DT, kMatrixFirst, 2>(P, t, head, lds, wave, row0, rows);
    }
}

// Partial output reduction (Alg. 3), n-ary: one wave folds the partials of RPW consecutive query heads
// of one request (hq .. hq + RPW - 1, all of one KV head) in list order.  Partials are taken eight or
// fifteen at a time: their loads are issued together, then they are folded against their common maximum
// (by associativity of the reduction this equals any binary bracketing).
//
// RPW = 1: each lane owns D / 64 channels of the one row.  RPW = 256 / D (the reduction kernel, when
// the group size allows it): each lane owns four channels of one of the rows; the rows of consecutive
// heads are neighbours in the partial arrays and in the output, so every load of partial rows is one
// full 1 KB instruction and a reduction costs half (a quarter for 64 channels) the memory instructions
// per row.  The kernel is bound by those: each takes a place in the CU's queue of memory instructions
// in flight whatever it moves.  For the same reason it loads only the partials that exist (inside the
// attention kernel, single-launch mode, every slot of a round is loaded: rows behind the end of a list
// read as row 0, which is valid memory, and the straight-line code keeps that kernel as it is).
template <int DT, bool COHERENT, int D, int RPW = 1>
__device__ __forceinline__ void merge_one(const MergeParams &P, int r, int hq, int wave_lane)
{
    constexpr int kChunk = 8;
    constexpr int LPR = 64 / RPW;       // lanes per row
    constexpr int CPL = D / LPR;        // channels per lane: 1, 2 or 4
    static_assert(CPL == 1 || CPL == 2 || CPL == 4, "channels per lane");
    const int lane = wave_lane % LPR;   // the lane's place in its row
    hq += wave_lane / LPR;              // the lane's row
    const int head = hq / P.group, hj = hq - head * P.group;
    // The request's line: its number of partial rows and the first kInlineParts of them, read together
    // (no address waits for another read).  Lists of up to eight rows, and of up to kInlineParts, are
    // folded in one round of loads; what lies beyond comes from the CSR arrays, eight rows a round.
    const int32_t *line = P.req_inline + int64_t(r) * (kInlineParts + 1);
    const int total = line[0];
    int first[kInlineParts];
#pragma unroll
    for (int j = 0; j < kInlineParts; ++j) first[j] = line[1 + j];  // zero behind the end: a valid row
    const int64_t head_base = int64_t(head) * P.part_rows + hj;
    float M = -INFINITY, L = 0.f, acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
    auto fold = [&](const int *rows, int cnt, auto width) {
        constexpr int N = decltype(width)::value;
        float2 ml[N];
        float o[N][CPL];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            if constexpr (!COHERENT)        // the reduction kernel: no load for a partial that does not exist
                if (j >= cnt) {             // (wave-uniform)
                    ml[j] = float2{0.f, 0.f};
#pragma unroll
                    for (int c = 0; c < CPL; ++c) o[j][c] = 0.f;
                    continue;
                }
            const int64_t prow = head_base + rows[j];
            const float *src = P.part_o + prow * D + lane * CPL;
            if constexpr (COHERENT) {       // rows written by other workgroups of this launch
                ml[j] = ld8_device(P.part_ml + prow * 2);
                if constexpr (CPL == 1) {
                    o[j][0] = __builtin_bit_cast(float, __hip_atomic_load(reinterpret_cast<const unsigned int *>(src),
                                                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                } else {
#pragma unroll
                    for (int c = 0; c < CPL; c += 2) {
                        const float2 x = ld8_device(src + c);
                        o[j][c] = x.x;
                        o[j][c + 1] = x.y;
                    }
                }
            } else {
                ml[j] = *reinterpret_cast<const float2 *>(P.part_ml + prow * 2);
                if constexpr (CPL == 1) {
                    o[j][0] = *src;
                } else if constexpr (CPL == 2) {
                    const float2 x = *reinterpret_cast<const float2 *>(src);
                    o[j][0] = x.x;
                    o[j][1] = x.y;
                } else {
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(src);
#pragma unroll
                    for (int c = 0; c < 4; ++c) o[j][c] = x[c];
                }
            }
        }
        float mm = M;
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j < cnt) mm = fmaxf(mm, ml[j].x);
        const float wa = weight(M, mm);
        L *= wa;
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] *= wa;
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j < cnt) {
                const float wb = weight(ml[j].x, mm);
                L += ml[j].y * wb;
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c] += o[j][c] * wb;
            }
        M = mm;
    };
    if (total <= kChunk) {
        fold(first, total, std::integral_constant<int, kChunk>{});
    } else {
        fold(first, total < kInlineParts ? total : kInlineParts, std::integral_constant<int, kInlineParts>{});
        if (total > kInlineParts) {
            const int32_t *list = P.req_part + P.req_part_off[r];
#pragma unroll 1
            for (int base = kInlineParts; base < total; base += kChunk) {
                const int cnt = total - base < kChunk ? total - base : kChunk;
                int rows[kChunk];
#pragma unroll
                for (int j = 0; j < kChunk; ++j) rows[j] = list[base + (j < cnt ? j : 0)];
                fold(rows, cnt, std::integral_constant<int, kChunk>{});
            }
        }
    }
    const float inv = 1.f / L;
    char *out = static_cast<char *>(P.out) + ((int64_t(r) * P.h_q + hq) * D + lane * CPL) * 2;
    if constexpr (CPL == 1) {
        *reinterpret_cast<unsigned short *>(out) = static_cast<unsigned short>(pack2<DT>(acc[0] * inv, 0.f) & 0xFFFFu);
    } else {
#pragma unroll
        for (int c = 0; c < CPL; c += 2)
            *reinterpret_cast<unsigned int *>(out + c * 2) = pack2<DT>(acc[c] * inv, acc[c + 1] * inv);
    }
}

template <int DT, int D, int RPW>
__global__ void __launch_bounds__(kMergeWaves * 64) merge_kernel(const MergeParams P)
{
    const int per_req = P.h_q / RPW;            // the launch has checked that RPW divides the group size
    const int unit = blockIdx.x * kMergeWaves + (threadIdx.x >> 6);
    if (unit >= P.num_requests * per_req) return;
    const int r = unit / per_req;
    merge_one<DT, false, D, RPW>(P, r, (unit - r * per_req) * RPW, threadIdx.x & 63);
}

// ---- single-launch mode: the reduction inside the attention launch (Sec. 4.3, parallel reduction) ----
//
// Every task delivers one partial result to each of its requests.  arrive[head][request] counts them
// (device-scope atomics); the delivery that completes a request's reduction list (its length is the
// first word of the request's line) makes the delivering workgroup reduce that request's rows of this
// KV head right away, and put the counter back to zero for the next launch.  In this mode partial rows
// are written and read with device-coherent accesses (st8_device / ld8_device), so no cache has to be
// written back or invalidated: a delivering wave waits until its stores have been acknowledged (they are
// then visible device-wide), and only then counts; the workgroup that sees the last count reads the rows
// after that.  (Fences at device scope instead, with plain accesses, cost a write-back and an
// invalidation of the whole L2 per task: measured, several times the launch they were to save.)
__device__ __forceinline__ bool deliver(const PacParams &P, const DevTask &t, int head, int i, int &req)
{
    req = t.single_req >= 0 ? t.single_req : P.node_q[t.q_off + i];
    const int want = P.merge.req_inline[int64_t(req) * (kInlineParts + 1)];
    int32_t *c = P.arrive + int64_t(head) * P.merge.num_requests + req;
    const int old = __hip_atomic_fetch_add(c, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 != want) return false;
    __hip_atomic_store(c, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // nobody else counts on it in this launch
    return true;
}

// A task that the whole workgroup ran (every thread calls this after the task).
template <int DT, int D>
__device__ void task_delivered_by_workgroup(const PacParams &P, const DevTask &t, int head, char *lds_raw, int waves)
{
    int *count = reinterpret_cast<int *>(lds_raw), *ready = count + 1;
    __syncthreads();                    // every wave has waited for its stores of partial rows; LDS is free
    if (threadIdx.x == 0) *count = 0;
    __syncthreads();
    if (int(threadIdx.x) < t.n_req) {
        int req;
        if (deliver(P, t, head, threadIdx.x, req)) ready[atomicAdd(count, 1)] = req;
    }
    __syncthreads();
    const int n = *count * P.group;
    if (n > 0) {
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");     // no load of a partial row moves above the count
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll 1
        for (int i = wave; i < n; i += waves) {
            const int k = i / P.group;
            merge_one<DT, true, D>(P.merge, ready[k], head * P.group + (i - k * P.group), threadIdx.x & 63);
        }
    }
    __syncthreads();                    // the list is done with before LDS is used again
}

// A task that one wave ran on its own (no barrier: the other waves are inside other tasks).
template <int DT, int D>
__device__ void task_delivered_by_wave(const PacParams &P, const DevTask &t, int head)
{
    const int lane = threadIdx.x & 63;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // waits for the wave's stores of partial rows
    int req = 0;
    const bool last = lane < t.n_req && deliver(P, t, head, lane, req);
    unsigned long long ready = __ballot(last);
    if (ready == 0) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll 1
    while (ready) {
        const int src = __builtin_ctzll(ready);
        ready &= ready - 1;
        const int r = __shfl(req, src);
#pragma unroll 1
        for (int hj = 0; hj < P.group; ++hj) merge_one<DT, true, D>(P.merge, r, head * P.group + hj, lane);
    }
}

// WIDE: kRingBytes of dynamic LDS.  The dense path XORs the channel tile into operand addresses, so
// the ring must start on a 256-byte boundary (no static LDS in that variant).
extern __shared__ __attribute__((aligned(1024))) char dyn_lds[];

template <int DT, int WIDE, int D>
__global__ void __launch_bounds__(WIDE ? kWideWaves * 64 : kNarrowWaves * 64, D > 128 ? 1 : 2)
pac_kernel(const PacParams P)     // 256 channels: two blocks of K and V in registers need a wave per SIMD
{
    static_assert(WIDE == 0 || D == kHeadDim, "the dense path exists for 128 channels only");
    constexpr int W = WIDE ? kWideWaves : kNarrowWaves;
    char *lds;
    if constexpr (WIDE != 0) {
        lds = dyn_lds;
    } else {
        __shared__ __attribute__((aligned(16))) char static_lds[merge_bytes(kNarrowWaves, stream_tiles(D), D) + kNarrowWaves * solo_stage_bytes(D)];
        lds = static_lds;
    }
    const int head = blockIdx.x % P.h_kv;
    const int slot = blockIdx.x / P.h_kv;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // staging area of this wave for tasks it runs on its own: behind the area in which a team merges its
    // states (in the wide variant both lie in the ring, which only dense tasks fill)
    static_assert(merge_bytes(kWideWaves, 1, kHeadDim) + kWideWaves * solo_stage_bytes(kHeadDim) <= kRingBytes, "staging areas fit the ring");
    char *stage = lds + merge_bytes(W, WIDE ? 1 : stream_tiles(D), D) + wave * solo_stage_bytes(D);
    // Runs the task records recs[t0 .. t1).  Tasks of more than 16 rows take the dense path (wide variant
    // only).  Tasks of at most 16 rows take the stream path, as a rule with all waves of the workgroup
    // as one team.  Runs of two or more short ones are handed out one wave each through a counter in
    // LDS: the latencies of a short task (descriptor, query rows, page ids, first blocks, merge of a
    // team) then overlap with the other tasks' instead of adding up.  In a slot's list the plan marks
    // such runs (they are neighbours there, the list being sorted by cost); an entry of the run-time
    // queue with several tasks is one such run.
    auto run_tasks = [&](const DevTask *recs, int t0, int t1, bool marked) __attribute__((always_inline)) {
        int i = t0;
#pragma unroll 1
        while (i < t1) {
            const DevTask t = recs[i];
            const int n = marked ? t.solo_run : t1 - i;
            if (n >= 2) {
                // Wave w starts with task w of the run, every further task is the next one nobody has
                // taken.  The run is in order of decreasing cost and the first waves are the older ones
                // of the pairs that share a SIMD, which the hardware serves first (measured: in a run
                // they move two to three times the tokens of their partners), so the longest tasks start
                // on the fastest waves.
                int *next = reinterpret_cast<int *>(lds);
                if (threadIdx.x == 0) *next = W;
                __syncthreads();
                int k = wave;
#pragma unroll 1
                while (k < n) {
                    const DevTask mine = recs[i + k];
                    if (mine.flags & kTaskReadOnce) run_stream<DT, true, 1, 1, D>(P, mine, head, lds, 0, stage);
                    else                run_stream<DT, false, 1, 1, D>(P, mine, head, lds, 0, stage);
                    if (P.arrive) task_delivered_by_wave<DT, D>(P, mine, head);
                    k = 0;
                    if ((threadIdx.x & 63) == 0) k = atomicAdd(next, 1);
                    k = __builtin_amdgcn_readfirstlane(k);
                }
                __syncthreads();                // the counter is done with before LDS is used again
                i += n;
            } else {
                if (t.n_req * P.group <= 16) {
                    if (t.flags & kTaskReadOnce) run_stream<DT, true, 1, W, D>(P, t, head, lds, wave);
                    else             run_stream<DT, false, 1, W, D>(P, t, head, lds, wave);
                }
                else if constexpr (WIDE != 0) run_dense32<DT>(P, t, head, lds);
                else if constexpr (stream_tiles(D) == 2) {      // 17 .. 32 rows of 64 channels: two row tiles
                    if (t.flags & kTaskReadOnce) run_stream<DT, true, 2, W, D>(P, t, head, lds, wave);
                    else             run_stream<DT, false, 2, W, D>(P, t, head, lds, wave);
                }
                if (P.arrive) task_delivered_by_workgroup<DT, D>(P, t, head, lds, W);
                ++i;
            }
        }
    };

    // Static schedule: the slot's own list, once.  Run-time queue: entry `slot` is this workgroup's
    // first; every further one is the next entry nobody has taken, fetched by one thread (one atomic)
    // and spread to the waves through LDS.  Every path through run_tasks ends with a barrier behind
    // its last LDS access, so the word can be written right away; the second barrier keeps the next
    // task's block copies from overwriting it before everyone has read it.
    const bool queued = P.queue_off != nullptr;
    const bool fetching = queued && P.num_entries > P.num_slots;        // else: an entry per workgroup at most
    const DevTask *recs = queued ? P.queue_recs : P.slot_recs;
    const int32_t *off = queued ? P.queue_off : P.slot_off;
    const int limit = queued ? P.num_entries : slot + 1;
    int32_t *taken = P.counters + 2 * head, *finished = taken + 1;
    int *word = reinterpret_cast<int *>(lds);
    int e = slot;
#pragma unroll 1
    while (e < limit) {
        run_tasks(recs, off[e], off[e + 1], !queued);
        if (!fetching) break;
        // taken when the workgroup is free, not ahead of time: an entry reserved early would wait for
        // the end of a long task while other workgroups idle
        if (threadIdx.x == 0) *word = P.num_slots + atomicAdd(taken, 1);
        __syncthreads();
        e = __builtin_amdgcn_readfirstlane(*word);
        __syncthreads();
    }
    // the last workgroup of this KV head to get here leaves the counters at zero for the next launch
    if (fetching && threadIdx.x == 0 && atomicAdd(finished, 1) == P.num_slots - 1) {
        atomicExch(taken, 0);
        atomicExch(finished, 0);
    }
}

// Read-only streaming kernel (measurement support): every thread sums 16-byte loads; a workgroup takes
// whole 4 KB chunks, chunk c of the walk being chunk perm(c) of the buffer, so that the order can be
// that of a paged pool.  One value per workgroup is written so that the loads cannot be dropped.
template <bool ONCE>
__global__ void __launch_bounds__(256) stream_read_kernel(const char *buf, uint64_t chunks, uint64_t mult,
                                                          uint32_t *sink)
{
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (uint64_t c = blockIdx.x; c < chunks; c += gridDim.x) {
        const uint64_t at = (c * mult) & (chunks - 1);          // chunks is a power of two, mult odd: a permutation
        const char *p = buf + at * 4096 + threadIdx.x * 16;
        const u32x4 x = ONCE ? ld16_once(p) : ld16(p);
        acc ^= x;
    }
    const uint32_t v = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (v == 0x9E3779B9u && threadIdx.x == 0) sink[blockIdx.x] = v;       // practically never: keeps the loads alive
}

}  // namespace

// Scratch for callers that cannot provide a workspace (codec_decode_attention_static): partial outputs
// and their softmax statistics of one decode call.  Every GPU the library is loaded on holds one copy
// of this array at an address of its own until the process ends.  In host code the name below is only a
// handle for hipGetSymbolAddress; kernels get the address that call returns, as an ordinary argument.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch_address(void **ptr)
{
    // one lookup per device, with that device current; the table is filled under a lock and read-only after
    constexpr int kMaxDevices = 64;
    static void *address[kMaxDevices] = {};
    static std::mutex lock;
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev)) return int(e);
    if (dev < 0 || dev >= kMaxDevices) return int(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> guard(lock);
    if (!address[dev]) {
        void *p = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return int(e);
        address[dev] = p;
    }
    *ptr = address[dev];
    return 0;
}

// The wide variant needs more dynamic LDS than the 64 KB a kernel gets by default.  Set once per
// process and device, outside any stream capture (codec_plan_upload calls this).
int prepare_kernels()
{
    constexpr int kMaxDevices = 64;
    static bool done[kMaxDevices] = {};
    static std::mutex lock;
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev)) return int(e);
    if (dev < 0 || dev >= kMaxDevices) return int(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> guard(lock);
    if (done[dev]) return 0;
    if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pac_kernel<CODEC_DTYPE_FP16, 1, 128>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kRingBytes))
        return int(e);
    if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pac_kernel<CODEC_DTYPE_BF16, 1, 128>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kRingBytes))
        return int(e);
    done[dev] = true;
    return 0;
}

template <int DT, int D>
void launch_narrow(const PacParams &p, dim3 grid, hipStream_t s)
{
    hipLaunchKernelGGL((pac_kernel<DT, 0, D>), grid, dim3(kNarrowWaves * 64), 0, s, p);
}

int launch_pac(const PacParams &p, int dtype, int head_dim, int num_slots, int max_rows_in_plan, void *stream)
{
    if (head_dim != 64 && head_dim != 128 && head_dim != 256) return int(hipErrorInvalidValue);
    const bool wide = head_dim == kHeadDim && max_rows_in_plan > 16;
    // the planner never builds a plan with more rows per task than the variant runs
    if (!wide && max_rows_in_plan > 16 * stream_tiles(head_dim)) return int(hipErrorInvalidValue);
    const dim3 grid(unsigned(num_slots) * unsigned(p.h_kv)), block((wide ? kWideWaves : kNarrowWaves) * 64);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f16 = dtype == CODEC_DTYPE_FP16;
    if (wide) {
        if (f16) hipLaunchKernelGGL((pac_kernel<CODEC_DTYPE_FP16, 1, 128>), grid, block, kRingBytes, s, p);
        else     hipLaunchKernelGGL((pac_kernel<CODEC_DTYPE_BF16, 1, 128>), grid, block, kRingBytes, s, p);
    } else if (head_dim == 64) {
        if (f16) launch_narrow<CODEC_DTYPE_FP16, 64>(p, grid, s); else launch_narrow<CODEC_DTYPE_BF16, 64>(p, grid, s);
    } else if (head_dim == 128) {
        if (f16) launch_narrow<CODEC_DTYPE_FP16, 128>(p, grid, s); else launch_narrow<CODEC_DTYPE_BF16, 128>(p, grid, s);
    } else if (head_dim == 256) {
        if (f16) launch_narrow<CODEC_DTYPE_FP16, 256>(p, grid, s); else launch_narrow<CODEC_DTYPE_BF16, 256>(p, grid, s);
    } else {
        return int(hipErrorInvalidValue);
    }
    return int(hipGetLastError());
}

int launch_stream_read(const void *buf, uint64_t chunks, uint64_t mult, int once, int blocks, void *sink, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const char *b = static_cast<const char *>(buf);
    uint32_t *k = static_cast<uint32_t *>(sink);
    if (once) hipLaunchKernelGGL(stream_read_kernel<true>, dim3(unsigned(blocks)), dim3(256), 0, s, b, chunks, mult, k);
    else      hipLaunchKernelGGL(stream_read_kernel<false>, dim3(unsigned(blocks)), dim3(256), 0, s, b, chunks, mult, k);
    return int(hipGetLastError());
}

template <int DT, int D>
void launch_merge_of(const MergeParams &p, hipStream_t s)
{
    // a wave reduces 256 / D rows at a time where the rows of a KV head's group divide that evenly
    constexpr int kWide = 256 / D;
    const bool wide = kWide > 1 && p.group % kWide == 0;
    const int units = p.num_requests * (p.h_q / (wide ? kWide : 1));
    const dim3 grid(unsigned((units + kMergeWaves - 1) / kMergeWaves)), block(kMergeWaves * 64);
    if (wide) hipLaunchKernelGGL((merge_kernel<DT, D, kWide>), grid, block, 0, s, p);
    else      hipLaunchKernelGGL((merge_kernel<DT, D, 1>), grid, block, 0, s, p);
}

int launch_merge(const MergeParams &p, int dtype, int head_dim, void *stream)
{
    if (head_dim != 64 && head_dim != 128 && head_dim != 256) return int(hipErrorInvalidValue);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool half = dtype == CODEC_DTYPE_FP16;
    if (head_dim == 64)       half ? launch_merge_of<CODEC_DTYPE_FP16, 64>(p, s) : launch_merge_of<CODEC_DTYPE_BF16, 64>(p, s);
    else if (head_dim == 128) half ? launch_merge_of<CODEC_DTYPE_FP16, 128>(p, s) : launch_merge_of<CODEC_DTYPE_BF16, 128>(p, s);
    else                      half ? launch_merge_of<CODEC_DTYPE_FP16, 256>(p, s) : launch_merge_of<CODEC_DTYPE_BF16, 256>(p, s);
    return int(hipGetLastError());
}

}  // namespace codec
