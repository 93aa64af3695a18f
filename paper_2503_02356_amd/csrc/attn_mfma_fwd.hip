// bf16 MFMA forward kernel for one chunk, head_dim 128 (paper sections 2.1, 2.2, 4.2: causal mask per
// packed sequence; a dependent chunk's queries also read the retained key/value prefix).
//
// One workgroup = 4 wavefronts; each wavefront owns a unit = 32 consecutive query rows of one query head.  A tile
// of 128 rows and the G query heads of a key/value head make 4 G units, dealt four at a time (block-major) to G
// workgroups: the units of a workgroup share the key/value head and (almost) the key range.  Key/value tiles
// of 64 rows are copied straight from global memory into LDS (buffer loads with an LDS destination, double
// buffered, XOR-swizzled rows) and shared by the four wavefronts.
// Everything is computed TRANSPOSED so that a lane owns one query:
//     S^T = K Q^T   (A = K tile rows from LDS, B = Q^T kept in registers for the whole kernel)
//     O^T += V^T P^T (A = V^T through transposing LDS reads, B = P^T straight from the S^T registers)
// With the query on the lane axis the row maximum and row sum are in-lane reductions plus one exchange
// between lane l and lane l^32, the running rescale is one scalar per lane, and P never leaves registers.
// Only tiles that intersect the causal diagonal apply a mask; tiles above it are never visited.
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "mfma_common.h"

namespace cf {
namespace {

constexpr int BM = 128;        // query rows per workgroup
constexpr int BN = 64;         // key rows per tile
constexpr int D = 128;
constexpr int TILE_BYTES = BN * 256;          // one swizzled K or V tile (see mfma_common.h)
constexpr int STAGE_BYTES = 2 * TILE_BYTES;   // K then V
constexpr float kLazy = 8.f;                  // log2 units a row maximum may exceed the running reference before O is rescaled

// id: index of the workgroup among those of this chunk
__device__ __forceinline__ void fwd_body(const cf_attn_fwd_params &p, int id, char *stage_a, char *stage_b)
{
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int half = lane >> 5, col = lane & 31;

    // Block id -> (tile rank, head).  The key/value head varies fastest so that the workgroups an XCD
    // receives (ids are dealt round-robin over the 8 XCDs) keep re-reading the same K/V head in its L2.
    const int G = p.n_q_heads / p.n_kv_heads;
    const int kh = id % p.n_kv_heads;
    id /= p.n_kv_heads;
    const int j = id % G;                            // which of the G workgroups of this (tile, key/value head)
    const int rank = id / G;
    // The tile's 4 G units (32-row block, query head of the group) are dealt out four at a time, block-major:
    // the wavefronts of a workgroup then share at most two neighbouring blocks, so that they need (almost) the
    // same key tiles and a ragged last tile costs workgroups in proportion to its rows.
    const int unit = 4 * j + wave;
    const int blk = unit / G;
    const int h = kh * G + (unit - blk * G);

    int tile_in_seg, q_seg0, lq, k_seg0, lk;
    if (p.q_tiles != nullptr) {
        if (rank >= p.n_q_tiles) return;
        const QTile t = read_q_tile(p.q_tiles, rank);
        tile_in_seg = t.tile_in_seg, q_seg0 = t.q_begin, lq = t.q_len, k_seg0 = t.k_begin, lk = t.k_len;
    } else {
        TileLocation loc;
        if (!locate_tile(p.cu_seqlens_q, p.cu_seqlens_k, p.n_segments, BM, rank, loc)) return;
        // (the same in every lane, but values that leave the search loop do not look that way to the compiler)
        tile_in_seg = uniform(loc.tile_in_seg);
        q_seg0 = uniform(loc.begin), lq = uniform(loc.len), k_seg0 = uniform(loc.other_begin), lk = uniform(loc.other_len);
    }
    const int off = lk - lq;                         // prefix keys every row of the segment sees
    const int q_tile0 = tile_in_seg * BM;
    const int rows_valid = min(BM, lq - q_tile0);
    if (q_tile0 + (4 * j) / G * 32 >= lq) return;    // all four units lie beyond the last row
    const int kmax = q_tile0 + min(rows_valid, ((4 * j + 3) / G + 1) * 32) + off;   // keys [0, kmax) are visible to some row of the workgroup
    const int n_tiles = (kmax + BN - 1) / BN;

    const int wq0 = q_tile0 + blk * 32;              // first row of this wavefront (segment-local)
    const int wave_kmax = min(kmax, wq0 + 32 + off); // keys this wavefront needs (<= 0 rows valid: nothing)
    const bool wave_active = wq0 < lq;
    const int iq = wq0 + col;                        // this lane's query row
    const int amax = iq + off;                       // last visible key of this lane's row

    const int64_t kv_row_bytes = p.kv_stride_tok * 2;
    const char *kbase = uniform((const char *)p.k + ((int64_t)k_seg0 * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2);
    const char *vbase = uniform((const char *)p.v + ((int64_t)k_seg0 * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2);
    TileDma<BN> dma;
    dma.init(kv_row_bytes);

    // Q^T fragments: lane (col, half) holds row iq, d = 16*ks + 8*half + 0..7.
    bf16x8 qf[8];
    {
        const int row = q_seg0 + min(iq, lq - 1);
        const char *qrow = (const char *)p.q + ((int64_t)row * p.q_stride_tok + (int64_t)h * p.q_stride_head) * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8 *)(qrow + ks * 32 + half * 16);
    }
    const LaneOffsets lo = lane_offsets();

    f32x16 o_acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) o_acc[i][j] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;            // running max (log2 units) and this lane's partial row sum
    const float c2 = p.softmax_scale * 1.44269504088896340736f;

    auto issue_tile = [&](int tile_start, char *stage) {
        dma.issue(kbase + (int64_t)tile_start * kv_row_bytes, lk - 1 - tile_start, stage);
        dma.issue(vbase + (int64_t)tile_start * kv_row_bytes, lk - 1 - tile_start, stage + TILE_BYTES);
    };
    issue_tile(0, stage_a);
    wait_lds_dma();
    __syncthreads();

    auto do_tile = [&](int t, const char *stage, char *next_stage) {
        const int tile_start = t * BN;
        if (t + 1 < n_tiles) issue_tile(tile_start + BN, next_stage);

        if (wave_active && tile_start < wave_kmax) {
            // ---- S^T = K Q^T : two 32-key blocks
            // All 16 K fragments are requested before the first MFMA: the LDS latency is paid once per tile,
            // not once per MFMA (the matrix unit then consumes them in arrival order).
            f32x16 s[2];
            bf16x8 ka[2][8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) ka[mb][ks] = lds_read_b128(stage + mb * 8192 + lo.row_unit[ks]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) s[mb][j] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) s[mb] = mfma32(ka[mb][ks], qf[ks], s[mb]);
            // ---- causal mask, only on tiles that cross this wavefront's diagonal
            if (tile_start + BN - 1 > wq0 + off) {
                // register i of block mb is key tile_start + 32*mb + (i/4)*8 + 4*half + i%4: masked iff the
                // compile-time part of that exceeds lim (one compare with a constant + one select per element)
                const int lim = amax - tile_start - half * 4;
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (mb * 32 + (i >> 2) * 8 + (i & 3) > lim) s[mb][i] = -INFINITY;
            }
            // ---- online softmax (log2 domain)
            float mx = s[0][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[0][i]);
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[1][i]);
            mx = max_with_other_half(mx);
            // Lazy rescale: the running reference m_run only moves when a row's new maximum exceeds it by more than
            // 2^kLazy; until then P = exp2(s - m_run) <= 2^kLazy, exact enough in the fp32 sums and in bf16 alike,
            // and O needs no rescale.  The final division by l_tot and the LSE absorb whatever reference was used.
            const float mx2 = mx * c2;
            const bool grow = mx2 > m_run + kLazy;        // first tile: m_run = -inf
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float m_new = grow ? mx2 : m_run;
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // first tile: exp2(-inf) = 0
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int j = 0; j < 16; ++j) o_acc[db][j] *= alpha;
            }
            float rs = 0.f;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    s[mb][i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][i], c2, -m_run));
                    rs += s[mb][i];
                }
            l_run += rs;
            // ---- O^T += V^T P^T : contraction over the 64 keys in 4 groups of 16
            const char *vst = stage + TILE_BYTES;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int tq = 0; tq < 2; ++tq) {
                    // register 8*tq + j of block mb is key mb*32 + 16*tq + (j/4)*8 + 4*half + j%4
                    const bf16x8 pb = pack8(s[mb][8 * tq + 0], s[mb][8 * tq + 1], s[mb][8 * tq + 2], s[mb][8 * tq + 3],
                                            s[mb][8 * tq + 4], s[mb][8 * tq + 5], s[mb][8 * tq + 6], s[mb][8 * tq + 7]);
                    const char *va = vst + mb * 8192 + tq * 4096;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        o_acc[j] = mfma32(lds_read_tr_pair(va + lo.tr_lo[j], va + lo.tr_hi[j]), pb, o_acc[j]);
                }
        }
        wait_lds_dma();
        __syncthreads();
    };
    for (int t = 0; t < n_tiles; t += 2) {
        do_tile(t, stage_a, stage_b);
        if (t + 1 < n_tiles) do_tile(t + 1, stage_b, stage_a);
    }

    if (!wave_active) return;
    const float l_tot = sum_with_other_half(l_run);
    // O rows leave through this wavefront's part of the (now idle) stage buffers, whole rows per store instruction.
    // The scale of a padding row (l_tot = 0 cannot happen: every real row sees its own key) is never stored.
    char *scratch = (wave < 2 ? stage_a : stage_b) + (wave & 1) * kRowScratchBytes;
    store_rows_bf16(o_acc, 1.f / l_tot, scratch, lq - wq0, [&](int r) {
        return (char *)p.o + ((int64_t)(q_seg0 + wq0 + r) * p.o_stride_tok + (int64_t)h * p.o_stride_head) * 2;
    });
    if (iq < lq && half == 0)
        p.lse[(int64_t)h * p.n_tokens + q_seg0 + iq] = m_run * 0.69314718055994530942f + __logf(l_tot);
}

__global__ __launch_bounds__(256, 2) void mfma_fwd_kernel(cf_attn_fwd_params p)
{
    // Two separate arrays (not one array with two halves): the compiler must see that the direct-to-LDS
    // loads of the next tile cannot alias the reads of the current one, or it waits for them too early.
    __shared__ __attribute__((aligned(16))) char stage_a[STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char stage_b[STAGE_BYTES];
    fwd_body(p, blockIdx.x, stage_a, stage_b);
}

// Several chunks in one launch: workgroups [first_block[c], first_block[c+1]) belong to chunk c.  The host
// puts the heaviest chunk first, so the last, partly filled wave of workgroups of a big chunk is filled by
// the next chunk's workgroups instead of leaving compute units idle.
struct FwdBatch {
    int n;
    int first_block[CF_FWD_BATCH_MAX + 1];
    cf_attn_fwd_params p[CF_FWD_BATCH_MAX];
};
__global__ __launch_bounds__(256, 2) void mfma_fwd_batch_kernel(FwdBatch b)
{
    __shared__ __attribute__((aligned(16))) char stage_a[STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char stage_b[STAGE_BYTES];
    const int id = blockIdx.x;
    int c = 0;
    while (c + 1 < b.n && id >= b.first_block[c + 1]) ++c;
    fwd_body(b.p[c], id - b.first_block[c], stage_a, stage_b);
}

// Upper bound on the number of 128-row tiles: sum_g ceil(Lq_g / BM) <= T / BM + n_segments.
int64_t fwd_blocks(const cf_attn_fwd_params &p)
{
    return (p.q_tiles ? (int64_t)p.n_q_tiles : (int64_t)p.n_tokens / BM + p.n_segments) * p.n_q_heads;
}

}  // namespace

hipError_t launch_mfma_fwd_batch(const cf_attn_fwd_params *const *chunks, int n, hipStream_t s)
{
    if (n < 1 || n > CF_FWD_BATCH_MAX) return hipErrorInvalidValue;
    FwdBatch b;
    b.n = n;
    int64_t total = 0;
    for (int c = 0; c < n; ++c) {
        b.first_block[c] = (int)total;
        b.p[c] = *chunks[c];
        total += fwd_blocks(*chunks[c]);
        if (total > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    }
    b.first_block[n] = (int)total;
    mfma_fwd_batch_kernel<<<dim3((unsigned)total), 256, 0, s>>>(b);
    return hipGetLastError();
}

hipError_t launch_mfma_fwd(const cf_attn_fwd_params &p, hipStream_t s)
{
    const int64_t blocks = fwd_blocks(p);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const ProfileHook hook = take_profile_hook();
    if (hook.start) (void)hipEventRecord(hook.start, s);
    mfma_fwd_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(p);
    const hipError_t e = hipGetLastError();
    if (hook.stop) (void)hipEventRecord(hook.stop, s);
    return e;
}

}  // namespace cf
