// bf16 MFMA backward kernels for one chunk, head_dim 128 (paper section 4.2: key/value gradients of the
// retained prefix rows are accumulated by the later chunks' backward passes; section 2.2: per-sequence
// causal mask inside a packed chunk).
//
// Two kernels, no dQ atomics:
//
//  dkv kernel  A workgroup (8 wavefronts) owns 128 consecutive key rows of one segment.  Wavefronts w and w + 4
//              own the same 32 of them: one keeps their dV^T, the other their dK^T (fp32, 64 registers each)
//              for the whole kernel.  The workgroup loops over the 64-row query tiles that can see its keys, for
//              one or several query heads of its key/value head; Q and dO tiles go straight from global memory
//              into a ring of three XOR-swizzled LDS stages (row reads and transposing reads are both free of
//              bank conflicts).  Per 32-row block of queries:
//                  role 0:  S = Q K_w^T          P = exp2(S c - LSE)  -> LDS       dV_w^T += dO^T P
//                  role 1:  dP = dO V_w^T        dS = P (dP - delta)               dK_w^T += Q^T dS
//              (A operands from LDS rows resp. transposing LDS reads, B operands K_w / V_w / P / dS in registers).
//              FUSED_HEADS = true : one workgroup per key tile and key/value head loops over ALL query heads
//                  of the group and is the only writer of its dK/dV rows (plain read-modify-write, bitwise
//                  reproducible).  Used when the launch has enough key tiles to fill the GPU.
//              FUSED_HEADS = false: a work list built on the device cuts the (key tile, query heads) work into
//                  items of similar length, longest first; the items of one key/value head meet in dK/dV
//                  through fp32 atomic adds (once per workgroup, at the end).
//
//  dq kernel   Same shape as the forward kernel: a workgroup owns 128 query rows of one head, key/value
//              tiles of 64 rows go through LDS, everything transposed so that a lane owns one query:
//                  S^T = K Q^T   dP^T = V dO^T   dS^T = P^T (dP^T - delta)   dQ^T += K^T dS^T
//              LSE and delta are one scalar per lane; dS^T feeds the last product straight from registers.
//              It also computes delta = <dO, O> (which the dK/dV kernel, launched after it, reads).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kernels.h"
#include "mfma_common.h"

namespace cf {
namespace {

constexpr int D = 128;
constexpr float kLog2e = 1.44269504088896340736f;

// =====================================================================================================
// dK / dV
// =====================================================================================================
constexpr int BQ = 64;                                // query rows per tile (two 32-row blocks)
constexpr int BKV = 128;                              // key rows per workgroup
constexpr int DKV_WAVES = 8;                          // 4 pairs: (S, P, dV) wavefront + (dP, dS, dK) wavefront
constexpr int QTILE_BYTES = BQ * 256;                 // one swizzled Q or dO tile
constexpr int TROW = 132;                             // floats per row of the end-of-kernel transpose scratch (128 + 4)
// One stage: Q tile, dO tile, LSE[64], delta[64]; rounded up so that a stage also holds the end-of-kernel
// transpose scratch of two wavefronts (2 x 32 rows x TROW floats).  The P exchange area has the same size:
// 4 pairs x 2 slots x 4 KB, and the scratch of the last two wavefronts.
constexpr int DKV_STAGE_BYTES = 2 * 32 * TROW * 4;
constexpr int EXCH_SLOT_BYTES = 32 * 32 * 4;          // one 32 x 32 fp32 block of P
static_assert(DKV_STAGE_BYTES >= 2 * QTILE_BYTES + 512, "stage too small");
static_assert(DKV_STAGE_BYTES >= 4 * 2 * EXCH_SLOT_BYTES, "exchange area too small");

// ---- work list of the dK/dV kernel (not used in the fused mode) -------------------------------------------
// One item = (segment, key tile, first head of the group's share, number of heads): the workgroups of one
// key/value head.  A key tile seen by few query tiles keeps all G heads of the group in ONE item (one
// prologue, one epilogue, one set of atomic updates instead of G); a tile seen by many query tiles is split
// over up to G items so that no workgroup runs much longer than kSplitTarget tile iterations.
// The list is ordered by DESCENDING duration (heads x query tiles; a counting sort): workgroups start in list
// order, and starting the longest first is what keeps the last compute units from running one long item alone
// (a packed 8K chunk has ~500 items of 7 to 130 iterations for 256 compute units).
// Workspace layout (ints): [0] = number of items, [1] = 0 (a second list, unused), [64 ...] = the items; an item
// is int4 {segment, kt0, g0, n_heads}.
constexpr int kSplitTarget = 48;
constexpr int kDurationBuckets = 256;

// Runs in ONE workgroup of any size: as a kernel of its own (whole-plan launches) or as the first workgroup of the dQ
// launch, which the dK/dV kernel follows anyway (no launch of its own on the per-chunk path).
__device__ __forceinline__ void build_dkv_worklist(const cf_attn_fwd_params &p, int *wl, int capacity)
{
    __shared__ int bucket[kDurationBuckets];        // items per duration, then the next free slot of each duration
    __shared__ int n_items;
    for (int i = threadIdx.x; i < kDurationBuckets; i += (int)blockDim.x) bucket[i] = 0;
    __syncthreads();
    const int G = p.n_q_heads / p.n_kv_heads;
    i32x4 *items = (i32x4 *)(wl + 64);
    // Segments one after the other (their bounds are uniform loads), the key tiles of a segment in parallel.
    auto for_each_item = [&](auto &&visit) {
        for (int seg = 0; seg < p.n_segments; ++seg) {
            const int lq = p.cu_seqlens_q[seg + 1] - p.cu_seqlens_q[seg];
            const int lk = p.cu_seqlens_k[seg + 1] - p.cu_seqlens_k[seg];
            const int off = lk - lq;
            const int n_head_qt = off < 128 ? min((lq + 63) / 64, (128 - off + 63) / 64) : 0;
            for (int kt0 = threadIdx.x * 128; kt0 < lk; kt0 += (int)blockDim.x * 128) {
                const int qt_first = kt0 == 0 ? n_head_qt : max(0, kt0 - off) / 64;
                const int n_qt = (lq + 63) / 64 - qt_first;
                if (n_qt <= 0) continue;
                const int sp = min(G, (G * n_qt + kSplitTarget - 1) / kSplitTarget);
                for (int s = 0; s < sp; ++s) {
                    const int g0 = s * G / sp, g1 = (s + 1) * G / sp;
                    visit(i32x4{seg, kt0, g0, g1 - g0}, min((g1 - g0) * n_qt, kDurationBuckets - 1));
                }
            }
        }
    };
    for_each_item([&](i32x4, int duration) { atomicAdd(&bucket[duration], 1); });
    __syncthreads();
    if (threadIdx.x == 0) {                          // longest first: slots are handed out from the top bucket down
        int next = 0;
        for (int d = kDurationBuckets - 1; d >= 0; --d) {
            const int n = bucket[d];
            bucket[d] = next;
            next += n;
        }
        n_items = next;
    }
    __syncthreads();
    for_each_item([&](i32x4 item, int duration) {
        const int slot = atomicAdd(&bucket[duration], 1);
        if (slot < capacity) items[slot] = item;     // (capacity is an upper bound on the item count; see dkv_worklist_capacity)
    });
    __syncthreads();
    if (threadIdx.x == 0) {
        wl[0] = min(n_items, capacity);
        wl[1] = 0;
    }
}
__global__ __launch_bounds__(1024) void dkv_worklist_kernel(cf_attn_fwd_params p, int *wl, int capacity)
{
    build_dkv_worklist(p, wl, capacity);
}

// HEAD_TILES = false: a main block.  It leaves out the tile pairs made of a sequence's first 128
//     positions (query rows at positions < 128 x key tile 0): those rows see few keys, their P and dS are
//     large, and the bf16 rounding of P and dS would be the largest error in dK/dV.
// HEAD_TILES = true : a head block, one per (segment, key/value head), that does exactly those tile pairs and
//     feeds the MFMAs the bf16 values AND their bf16 rounding residuals.  (A run-time flag, uniform over the
//     workgroup: one code path keeps one register allocation.)
//
// Eight wavefronts, two per SIMD.  Wavefronts w and w + 4 own the same 32 keys and split the work per 32-row
// block of queries so that each keeps only ONE accumulator (64 registers) and one operand fragment:
//     role 0 (w < 4)  : S = Q K_w^T,  P = exp2(S c - LSE)  -> fp32 P into an LDS slot,   dV_w^T += dO^T P
//     role 1 (w >= 4) : dP = dO V_w^T,  dS = P (dP - delta) with P read from the slot,    dK_w^T += Q^T dS
// Role 1 runs one block behind role 0 (a workgroup barrier per block), so on every SIMD one wavefront is
// multiplying while the other does the exp / dS arithmetic.  Q/dO tiles rotate through three LDS stages: the
// copy of tile t + 2 starts when role 1 has left tile t - 1 and has two block steps to land.
template <bool FUSED_HEADS>
__device__ __forceinline__ void dkv_body(const cf_attn_bwd_params &b, const float *__restrict__ delta, int id,
                                         const bool HEAD_TILES, const int *__restrict__ wl, int capacity, char *st0,
                                         char *st1, char *st2, char *exch_all)
{
    const cf_attn_fwd_params &p = b.f;
    const int tid = threadIdx.x, lane = tid & 63, wave = wave_id();
    const int half = lane >> 5, col = lane & 31;
    const int role = wave >> 2, pw = wave & 3;       // role (uniform per wavefront), index of the 32-key slice

    // Block id -> (item, key/value head); the key/value head varies fastest (XCD L2 locality, see forward).
    //   fused mode : item = key tile rank, all G heads of the group
    //   otherwise  : head blocks: item = segment, all G heads; main blocks: item = entry of the work list
    const int G = p.n_q_heads / p.n_kv_heads;
    const int kh = id % p.n_kv_heads;
    id /= p.n_kv_heads;
    int seg, kt0 = 0, g0 = 0, n_heads = G;
    if (HEAD_TILES) {
        seg = id;                                    // one head block per (segment, key/value head)
        if (seg >= p.n_segments) return;
    } else if (FUSED_HEADS) {
        TileLocation loc;
        if (!locate_tile(p.cu_seqlens_k, p.cu_seqlens_q, p.n_segments, BKV, id, loc)) return;
        seg = loc.seg;
        // locate_tile numbers tiles from the end; the FIRST key tiles of a segment are seen by the most rows, so
        // flip the order inside the segment to start the heaviest tiles first.
        kt0 = ((loc.len + BKV - 1) / BKV - 1 - loc.tile_in_seg) * BKV;
    } else {
        if (id >= wl[0]) return;
        const i32x4 *items = (const i32x4 *)(wl + 64);
        const i32x4 item = items[id];
        seg = uniform(item[0]);
        kt0 = uniform(item[1]);
        g0 = uniform(item[2]);
        n_heads = uniform(item[3]);
    }
    // (seg, kt0 are the same in every lane, but values that leave locate_tile's search loop do not look that way to
    // the compiler: say so, or everything derived from them lives in vector registers.)
    seg = uniform(seg);
    kt0 = uniform(kt0);
    const int h_first = kh * G + g0;
    const int q_seg0 = p.cu_seqlens_q[seg], lq = p.cu_seqlens_q[seg + 1] - q_seg0;
    const int k_seg0 = p.cu_seqlens_k[seg], lk = p.cu_seqlens_k[seg + 1] - k_seg0;
    const int off = lk - lq;
    const int i_min = max(0, kt0 - off);             // first query row that sees any key of this tile
    // query tiles whose rows sit at positions < 128 of the sequence (only key tile 0 can see them)
    const int n_head_qt = off < 128 ? min((lq + BQ - 1) / BQ, (128 - off + BQ - 1) / BQ) : 0;
    const int qt_first = HEAD_TILES ? 0 : (kt0 == 0 ? n_head_qt : i_min / BQ);
    const int n_qt = HEAD_TILES ? n_head_qt : (lq + BQ - 1) / BQ - qt_first;
    if (n_qt <= 0) return;                           // whole workgroup leaves before any barrier
    const int n_tiles = n_heads * n_qt;              // (head, query tile) pairs, head by head
    const int n_blk = 2 * n_tiles;                   // 32-row blocks; step k: role 0 does block k, role 1 block k - 1
    const int qt_end = qt_first + n_qt;

    const int kv_idx = kt0 + 32 * pw + col;          // this lane's key (segment-local)
    const float c2 = p.softmax_scale * kLog2e;

    // Operand fragment kept for the whole kernel (B operand of S resp. dP): K_w for role 0, V_w for role 1;
    // lane = key row, 8 consecutive d per step.
    bf16x8 wf[8];
    {
        const int64_t row = k_seg0 + min(kv_idx, lk - 1);
        const char *src = (const char *)(role ? p.v : p.k) + (row * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) wf[ks] = *(const bf16x8 *)(src + ks * 32 + half * 16);
    }
    f32x16 acc[4];                                   // role 0: dV_w^T, role 1: dK_w^T
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    const LaneOffsets lo = lane_offsets();
    char *exch = exch_all + pw * 2 * EXCH_SLOT_BYTES + lane * 16;   // this lane's 16 bytes of row group 0, slot 0

    // Tile staging: Q and dO rows go straight from global memory into the swizzled LDS tiles (the first two tiles by the
    // role-1 wavefronts, later ones shared: role 0 copies the Q tile, role 1 the dO tile, four copy instructions per
    // wavefront and tile); LSE and delta go through one register of 64 + 64 threads, loaded when the copy starts and turned
    // into their LDS form (LSE as log2, +inf for rows past the segment so that P = 0; delta 0
    // there) one step later, so that nothing waits for memory right after the copies start.
    const int stid = tid - 256;                      // threads 256..319 / 320..383 (role 1) carry LSE / delta
    const float *stat_src = stid < 64 ? p.lse : delta;
    TileDma<BQ, 4> dma_q, dma_do;                    // a tile is copied by the four wavefronts of one role
    dma_q.init(p.q_stride_tok * 2, pw);
    dma_do.init(b.do_stride_tok * 2, pw);
    int nx_h = h_first, nx_qt = qt_first;            // the tile the next copy fetches (advances by additions only)
    int stat_q0 = 0;                                 // first row of the tile the pending stat register belongs to
    float stat = 0.f;
    auto issue_tile = [&](char *stage, bool with_q, bool with_do) {
        const int h = nx_h, q0 = nx_qt * BQ;
        const int64_t row0 = q_seg0 + q0;
        if (with_q)
            dma_q.issue(uniform((const char *)p.q + (row0 * p.q_stride_tok + (int64_t)h * p.q_stride_head) * 2), lq - 1 - q0, stage);
        if (with_do)
            dma_do.issue(uniform((const char *)b.d_o + (row0 * b.do_stride_tok + (int64_t)h * b.do_stride_head) * 2), lq - 1 - q0,
                         stage + QTILE_BYTES);
        if (stid >= 0 && stid < 128) stat = stat_src[(int64_t)h * p.n_tokens + q_seg0 + min(q0 + (tid & 63), lq - 1)];
        stat_q0 = q0;
        if (++nx_qt == qt_end) {
            nx_qt = qt_first;
            ++nx_h;
        }
    };
    auto publish_stats = [&](char *stage) {
        if (stid < 128) {
            const bool live = stat_q0 + (tid & 63) < lq;
            const float v = stid < 64 ? (live ? stat * kLog2e : INFINITY) : (live ? stat : 0.f);
            ((float *)(stage + 2 * QTILE_BYTES))[stid] = v;
        }
    };

    if (role == 1) {
        issue_tile(st0, true, true);
        publish_stats(st0);
        if (n_tiles > 1) {
            issue_tile(st1, true, true);
            publish_stats(st1);
        }
        wait_lds_dma();
    } else {                                         // role 0 shares the later copies: its tile counter moves along
        issue_tile(st0, false, false);
        if (n_tiles > 1) issue_tile(st1, false, false);
    }
    __syncthreads();

    int cur_qt = qt_first;                           // query tile of the block this wavefront works on

    // role 0, block kb of the tile in `stage`: S, P (to the exchange slot), dV
    // Operands that a wavefront requests at the END of a step for its next block, so that the LDS latency passes
    // while it waits at the barrier: role 0 the Q rows of block k + 1, role 1 the transposed Q operands of block k.
    bf16x8 aq[8], t_q[2][4];
    auto fetch_q_rows = [&](int kb, const char *stage) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) aq[ks] = lds_read_b128(stage + (kb & 1) * 8192 + lo.row_unit[ks]);
    };
    // next_stage: stage of block kb + 1 (its tile is resident one step ahead), or nullptr after the last block
    auto block_p_dv = [&](int kb, const char *stage, char *slot, const char *next_stage) {
        const int mb = kb & 1, q0 = cur_qt * BQ;
        const char *dos = stage + QTILE_BYTES;
        const float *lse_s = (const float *)(stage + 2 * QTILE_BYTES);
        f32x16 s;
#pragma unroll
        for (int j = 0; j < 16; ++j) s[j] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) s = mfma32(aq[ks], wf[ks], s);
        // transposed operands of the second product, requested now so that they arrive during the arithmetic:
        // k-slot 8*half + e of group tq is query row 32*mb + 16*tq + (e/4)*8 + 4*half + e%4
        bf16x8 t_do[2][4];
#pragma unroll
        for (int tq = 0; tq < 2; ++tq)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ta = mb * 8192 + tq * 4096;
                t_do[tq][j] = lds_read_tr_pair(dos + ta + lo.tr_lo[j], dos + ta + lo.tr_hi[j]);
            }
        // P: register i is query row q0 + 32*mb + (i/4)*8 + 4*half + i%4, column = this lane's key.  The causal
        // mask is a select on every block (no branch around arithmetic that feeds the MFMAs).
        const int lim = kv_idx - off - q0 - mb * 32 - half * 4;   // masked iff lim > 8*g4 + j
        // only a block that crosses the diagonal (its last key lies after its first query) needs the selects
        const bool crosses = kt0 + 32 * pw + 31 - off - q0 - mb * 32 > 0;     // wave-uniform
        if (!crosses) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 l4 = *(const f32x4 *)(lse_s + mb * 32 + g4 * 8 + half * 4);
                f32x4 pw4;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[g4 * 4 + j], c2, -l4[j]));
                    s[g4 * 4 + j] = pv;
                    pw4[j] = pv;
                }
                *(f32x4 *)(slot + g4 * 1024) = pw4;
            }
        } else
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const f32x4 l4 = *(const f32x4 *)(lse_s + mb * 32 + g4 * 8 + half * 4);
            f32x4 pw4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[g4 * 4 + j], c2, -l4[j]));
                if (lim > g4 * 8 + j) pv = 0.f;
                s[g4 * 4 + j] = pv;
                pw4[j] = pv;
            }
            *(f32x4 *)(slot + g4 * 1024) = pw4;      // lane-private position: role 1 reads it back at the same place
        }
        // dV_w^T += dO^T P : contraction over these 32 query rows in 2 groups of 16
#pragma unroll
        for (int tq = 0; tq < 2; ++tq) {
            const bf16x8 pb = pack8(s[8 * tq + 0], s[8 * tq + 1], s[8 * tq + 2], s[8 * tq + 3], s[8 * tq + 4],
                                    s[8 * tq + 5], s[8 * tq + 6], s[8 * tq + 7]);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = mfma32(t_do[tq][j], pb, acc[j]);
            if (HEAD_TILES) {   // add the bf16 rounding residual of P
                bf16x8 pl;
#pragma unroll
                for (int e = 0; e < 8; ++e) pl[e] = (__bf16)(s[8 * tq + e] - (float)pb[e]);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = mfma32(t_do[tq][j], pl, acc[j]);
            }
        }
        if (mb && ++cur_qt == qt_end) cur_qt = qt_first;
        __builtin_amdgcn_sched_barrier(0);
        if (kb + 1 < n_blk) fetch_q_rows(kb + 1, next_stage);
    };
    // role 1 works on two blocks per step, ordered so that its phases fall into the gaps of role 0's (which runs
    // S-MFMAs, P arithmetic, dV-MFMAs in that order): first the dS arithmetic of block k - 1 (while role 0 multiplies),
    // then the dK MFMAs of block k - 1 and the dP MFMAs of block k (while role 0 does its arithmetic).  dP of block k
    // stays in registers until the next step.
    f32x16 dp;
#pragma unroll
    for (int j = 0; j < 16; ++j) dp[j] = 0.f;
    // transposed Q operands of block kb: k-slot 8*half + e of group tq is query row 32*mb + 16*tq + (e/4)*8 + 4*half + e%4
    auto fetch_q_transposed = [&](int kb, const char *stage) {
#pragma unroll
        for (int tq = 0; tq < 2; ++tq)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ta = (kb & 1) * 8192 + tq * 4096;
                t_q[tq][j] = lds_read_tr_pair(stage + ta + lo.tr_lo[j], stage + ta + lo.tr_hi[j]);
            }
    };
    // dO rows of block kb (A operand of dP), requested before the dK MFMAs of the previous block are issued
    bf16x8 ado[8];
    auto fetch_do_rows = [&](int kb, const char *stage) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) ado[ks] = lds_read_b128(stage + QTILE_BYTES + (kb & 1) * 8192 + lo.row_unit[ks]);
    };
    // next_stage: stage of block kb + 1 (for its dO rows), or nullptr
    auto finish_ds_dk = [&](int kb, const char *stage, const char *slot, const char *next_stage) {
        const int mb = kb & 1;
        const float *del_s = (const float *)(stage + 2 * QTILE_BYTES) + 64;
        // P and delta; the transposed operands of dK were requested at the end of the previous step.
        f32x4 d4[4], p4[4];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            d4[g4] = *(const f32x4 *)(del_s + mb * 32 + g4 * 8 + half * 4);
            p4[g4] = *(const f32x4 *)(slot + g4 * 1024);
        }
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
            for (int j = 0; j < 4; ++j) dp[g4 * 4 + j] = p4[g4][j] * (dp[g4 * 4 + j] - d4[g4][j]);
        __builtin_amdgcn_sched_barrier(0);
        if (kb + 1 < n_blk) fetch_do_rows(kb + 1, next_stage);
        // dK_w^T += Q^T dS : contraction over these 32 query rows in 2 groups of 16
#pragma unroll
        for (int tq = 0; tq < 2; ++tq) {
            const bf16x8 dsb = pack8(dp[8 * tq + 0], dp[8 * tq + 1], dp[8 * tq + 2], dp[8 * tq + 3], dp[8 * tq + 4],
                                     dp[8 * tq + 5], dp[8 * tq + 6], dp[8 * tq + 7]);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = mfma32(t_q[tq][j], dsb, acc[j]);
            if (HEAD_TILES) {   // add the bf16 rounding residual of dS
                bf16x8 dl;
#pragma unroll
                for (int e = 0; e < 8; ++e) dl[e] = (__bf16)(dp[8 * tq + e] - (float)dsb[e]);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = mfma32(t_q[tq][j], dl, acc[j]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // dP of block kb from the dO rows already requested; then request the transposed Q operands of the same block
    auto start_dp = [&](int kb, const char *stage) {
#pragma unroll
        for (int j = 0; j < 16; ++j) dp[j] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) dp = mfma32(ado[ks], wf[ks], dp);
        __builtin_amdgcn_sched_barrier(0);
        fetch_q_transposed(kb, stage);
    };

    // Step k of n_blk + 1.  s_cur: stage of tile k/2 (role 0's block), s_prev: stage of tile (k-1)/2 (role 1's older
    // block), s_next: stage the copy started in this step (odd k: tile (k+3)/2) lands in.  The two roles run two
    // separate copies of the loop (same number of barriers): a value that only one role keeps across steps must not
    // occupy registers in the other.
    auto run = [&](auto role_tag) {
        constexpr int ROLE = decltype(role_tag)::value;
        // s_cur1: stage of block k + 1
        auto step = [&](int k, const char *s_cur, const char *s_prev, char *s_next, const char *s_cur1) {
            const bool odd = k & 1;
            if (odd && (k + 3) / 2 < n_tiles) issue_tile(s_next, ROLE == 0, ROLE == 1);
            if (ROLE == 0) {
                if (k < n_blk) block_p_dv(k, s_cur, exch + (k & 1) * EXCH_SLOT_BYTES, s_cur1);
            } else {
                if (k >= 1) finish_ds_dk(k - 1, s_prev, exch + ((k - 1) & 1) * EXCH_SLOT_BYTES, s_cur);
                if (k < n_blk) start_dp(k, s_cur);
            }
            if (!odd) {                              // the copy started one step ago has had a full step to land
                if (ROLE == 1 && k >= 2 && (k + 2) / 2 < n_tiles) publish_stats(const_cast<char *>(s_cur == st0 ? st1 : s_cur == st1 ? st2 : st0));
                wait_lds_dma();
            }
            // The plain barrier instruction, not __syncthreads(): that one also orders memory, for which the compiler
            // waits until a copy started in this very step has landed; the copies are waited for explicitly above, a
            // step later.  lgkmcnt(0): this wavefront's own LDS writes (P, LSE, delta) are done.
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
        };
        // Six steps = three tiles per trip, so that every stage is a compile-time array in every position.
        for (int k = 0; k <= n_blk; k += 6) {
            step(k, st0, st2, nullptr, st0);
            if (k + 1 <= n_blk) step(k + 1, st0, st0, st2, st1);
            if (k + 2 <= n_blk) step(k + 2, st1, st0, nullptr, st1);
            if (k + 3 <= n_blk) step(k + 3, st1, st1, st0, st2);
            if (k + 4 <= n_blk) step(k + 4, st2, st1, nullptr, st2);
            if (k + 5 <= n_blk) step(k + 5, st2, st2, st1, st0);
        }
    };
    if (role == 0) {
        fetch_q_rows(0, st0);
        run(std::integral_constant<int, 0>());
    } else {
        fetch_do_rows(0, st0);
        run(std::integral_constant<int, 1>());
    }

    // dK, dV: lane = key row; register group g4 of accumulator j = 4 consecutive d starting at 32*j + 8*g4 + 4*half.
    // Each wavefront turns its 32 x 128 block around in LDS (its own 16.5 KB half of a stage / of the exchange area,
    // all free after the loop's last barrier) and then updates whole rows, 64 lanes = 64 consecutive floats: a
    // lane-per-row update would touch 64 cache lines per instruction.
    //   FUSED_HEADS : this workgroup is the only writer of these rows in this launch: plain load, add, store.
    //   otherwise   : the query heads of a group add into the same rows: fp32 atomic adds.
    char *area = wave < 2 ? st0 : wave < 4 ? st1 : wave < 6 ? st2 : exch_all;
    float *tr = (float *)area + (wave & 1) * 32 * TROW;
    const int rows_valid = min(32, lk - (kt0 + 32 * pw));        // <= 0: this wavefront has no real keys
    const float out_scale = role ? p.softmax_scale : 1.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            f32x4 a;
#pragma unroll
            for (int e = 0; e < 4; ++e) a[e] = acc[j][g4 * 4 + e] * out_scale;
            *(f32x4 *)(tr + col * TROW + j * 32 + g4 * 8 + half * 4) = a;
        }
    __builtin_amdgcn_wave_barrier();
    float *gbase = (role ? b.d_k : b.d_v) + (int64_t)(k_seg0 + kt0 + 32 * pw) * b.dkv_stride_tok + (int64_t)kh * b.dkv_stride_head;
    // 8 rows per step: all 16 LDS reads first, then the 16 global updates (one LDS latency per step)
    for (int r0 = 0; r0 < rows_valid; r0 += 8) {
        float v[16];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[2 * e] = tr[(r0 + e) * TROW + lane];
            v[2 * e + 1] = tr[(r0 + e) * TROW + 64 + lane];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (r0 + e < rows_valid) {
                float *g = gbase + (int64_t)(r0 + e) * b.dkv_stride_tok;
                if (FUSED_HEADS) {
                    g[lane] += v[2 * e];
                    g[64 + lane] += v[2 * e + 1];
                } else {
                    unsafeAtomicAdd(g + lane, v[2 * e]);
                    unsafeAtomicAdd(g + 64 + lane, v[2 * e + 1]);
                }
            }
        }
    }
}

// Blocks [0, head_blocks) do the head tiles (one per (segment, key/value head)), the others the main work.
template <bool FUSED_HEADS>
__global__ __launch_bounds__(64 * DKV_WAVES) void mfma_dkv_kernel(cf_attn_bwd_params b, const float *__restrict__ delta,
                                                                 int head_blocks, const int *__restrict__ wl, int capacity)
{
    // Separate arrays (not one array with parts): the compiler must see that the direct-to-LDS copy of a coming
    // tile cannot alias the reads of the tiles in use, or it waits for the copy too early.
    __shared__ __attribute__((aligned(16))) char st0[DKV_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char st1[DKV_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char st2[DKV_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char exch[DKV_STAGE_BYTES];
    const int id = blockIdx.x;
    const bool head = id < head_blocks;
    dkv_body<FUSED_HEADS>(b, delta, head ? id : id - head_blocks, head, wl, capacity, st0, st1, st2, exch);
}

// =====================================================================================================
// dQ
// =====================================================================================================
constexpr int BM = 128;                      // query rows per workgroup
constexpr int BN = 64;                       // key rows per tile
constexpr int KVTILE_BYTES = BN * 256;       // one swizzled K or V tile
constexpr int DQ_STAGE_BYTES = 2 * KVTILE_BYTES;

// HEAD_TILES as in the dK/dV kernel: the main blocks skip the 128-row tile that starts a sequence (rows at
// positions < 128); the head blocks (one per (segment, head)) do it with dS residuals.  They also replace
// delta of their rows: delta = <dO, O> is computed from the ROUNDED O, and for rows that see few keys
// (large P, large |O|) that rounding would be the largest error of the whole backward pass (it lands in dK
// of the first keys of each sequence).  The head blocks first run over their (at most 4) key tiles once to
// form delta = sum_j P_j dP_j, which needs no O, store it for the dK/dV head blocks, then run again for dQ.
__device__ __forceinline__ void dq_body(const cf_attn_bwd_params &b, float *__restrict__ delta, int id,
                                        const bool HEAD_TILES, char *stage_a, char *stage_b)
{
    const cf_attn_fwd_params &p = b.f;
    const int tid = threadIdx.x, lane = tid & 63, wave = wave_id();
    const int half = lane >> 5, col = lane & 31;

    const int G = p.n_q_heads / p.n_kv_heads;
    const int kh = id % p.n_kv_heads;
    id /= p.n_kv_heads;
    const int j = id % G;                            // which of the G workgroups of this (tile, key/value head)
    const int rank = id / G;
    // Main blocks: the tile's 4 G units (32-row block, query head of the group) are dealt out four at a time,
    // block-major (as in the forward kernel).  Head blocks: one query head, wavefront w takes block w.
    const int unit = 4 * j + wave;
    const int blk = HEAD_TILES ? wave : unit / G;
    const int h = kh * G + (HEAD_TILES ? j : unit - blk * G);
    const int blk_first = HEAD_TILES ? 0 : (4 * j) / G, blk_last = HEAD_TILES ? 3 : (4 * j + 3) / G;

    int tile_in_seg = 0, q_seg0, lq, k_seg0, lk;
    if (HEAD_TILES) {
        const int seg = rank;                        // one block per (segment, head)
        if (seg >= p.n_segments) return;
        q_seg0 = p.cu_seqlens_q[seg], lq = p.cu_seqlens_q[seg + 1] - q_seg0;
        k_seg0 = p.cu_seqlens_k[seg], lk = p.cu_seqlens_k[seg + 1] - k_seg0;
    } else if (p.q_tiles != nullptr) {
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
    const int off = lk - lq;
    const int q_tile0 = tile_in_seg * BM;
    // the tile whose rows sit among the first 128 positions of a sequence belongs to the head blocks
    if ((q_tile0 + off < 128) != HEAD_TILES) return;
    const int rows_valid = min(BM, lq - q_tile0);
    if (q_tile0 + blk_first * 32 >= lq) return;      // all four units lie beyond the last row
    const int kmax = q_tile0 + min(rows_valid, (blk_last + 1) * 32) + off;   // keys [0, kmax) are visible to some row of the workgroup
    const int n_tiles = (kmax + BN - 1) / BN;
    const int wq0 = q_tile0 + blk * 32;
    const int wave_kmax = min(kmax, wq0 + 32 + off);
    const bool wave_active = wq0 < lq;
    const int iq = wq0 + col;                        // this lane's query row
    const int amax = iq + off;                       // last visible key of this lane's row

    const int64_t kv_row_bytes = p.kv_stride_tok * 2;
    const char *kbase = uniform((const char *)p.k + ((int64_t)k_seg0 * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2);
    const char *vbase = uniform((const char *)p.v + ((int64_t)k_seg0 * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2);
    TileDma<BN> dma;
    dma.init(kv_row_bytes);

    // Q^T and dO^T fragments (B operands): lane holds row iq, d = 16*ks + 8*half + 0..7
    bf16x8 qf[8], dof[8];
    float lse2, dlt;
    const int64_t stat_at = (int64_t)h * p.n_tokens + q_seg0 + min(iq, lq - 1);
    {
        const int row = q_seg0 + min(iq, lq - 1);
        const char *qrow = (const char *)p.q + ((int64_t)row * p.q_stride_tok + (int64_t)h * p.q_stride_head) * 2;
        const char *dorow = (const char *)b.d_o + ((int64_t)row * b.do_stride_tok + (int64_t)h * b.do_stride_head) * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            qf[ks] = *(const bf16x8 *)(qrow + ks * 32 + half * 16);
            dof[ks] = *(const bf16x8 *)(dorow + ks * 32 + half * 16);
        }
        lse2 = iq < lq ? p.lse[stat_at] * kLog2e : INFINITY;   // padding rows: P = 0
        // delta = <dO, O> of this lane's row (section 4.2's backward needs it for dS): each lane half sums its 64 d.
        // The main blocks publish it for the dK/dV kernel; the head blocks replace it below.
        dlt = 0.f;
        if (!HEAD_TILES) {
            const char *orow = (const char *)p.o + ((int64_t)row * p.o_stride_tok + (int64_t)h * p.o_stride_head) * 2;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 of = *(const bf16x8 *)(orow + ks * 32 + half * 16);
#pragma unroll
                for (int e = 0; e < 8; ++e) dlt = __builtin_fmaf((float)of[e], (float)dof[ks][e], dlt);
            }
            dlt = sum_with_other_half(dlt);
            if (iq < lq && half == 0) delta[stat_at] = dlt;
        }
    }
    const float c2 = p.softmax_scale * kLog2e;
    const LaneOffsets lo = lane_offsets();

    f32x16 dq[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) dq[i][j] = 0.f;

    auto issue_tile = [&](int tile_start, char *stage) {
        dma.issue(kbase + (int64_t)tile_start * kv_row_bytes, lk - 1 - tile_start, stage);
        dma.issue(vbase + (int64_t)tile_start * kv_row_bytes, lk - 1 - tile_start, stage + KVTILE_BYTES);
    };

    // One sweep over the key tiles.  DELTA_PASS: only accumulate sum_j P_j dP_j (this lane's keys) in dsum.
    float dsum = 0.f;
    auto sweep = [&](auto delta_pass_tag) {
        constexpr bool DELTA_PASS = decltype(delta_pass_tag)::value;
        issue_tile(0, stage_a);
        wait_lds_dma();
        __syncthreads();
        auto do_tile = [&](int t, const char *stage, char *next_stage) {
            const int tile_start = t * BN;
            const char *ks_ = stage;
            const char *vs_ = stage + KVTILE_BYTES;
            if (t + 1 < n_tiles) issue_tile(tile_start + BN, next_stage);

            if (wave_active && tile_start < wave_kmax) {
                const bool need_mask = tile_start + BN - 1 > wq0 + off;
                // register i of block mb is key tile_start + 32*mb + (i/4)*8 + 4*half + i%4: masked iff the
                // compile-time part of that exceeds lim
                const int lim = amax - tile_start - half * 4;
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    // S^T and dP^T for 32 keys: register i is key tile_start + 32*mb + (i/4)*8 + 4*half + i%4
                    // All 16 fragments are requested before the first MFMA: the LDS latency is paid once per
                    // block, not once per MFMA.
                    f32x16 s, dp;
                    bf16x8 ka[8], va[8];
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        ka[ks] = lds_read_b128(ks_ + mb * 8192 + lo.row_unit[ks]);
                        va[ks] = lds_read_b128(vs_ + mb * 8192 + lo.row_unit[ks]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < 16; ++j) s[j] = dp[j] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        s = mfma32(ka[ks], qf[ks], s);
                        dp = mfma32(va[ks], dof[ks], dp);
                    }
                    // K^T fragments of the dQ contraction: requested now, so that they arrive during the arithmetic
                    bf16x8 kt[2][4];
                    if (!DELTA_PASS) {
#pragma unroll
                        for (int tq = 0; tq < 2; ++tq)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const char *ka_ = ks_ + mb * 8192 + tq * 4096;
                                kt[tq][j] = lds_read_tr_pair(ka_ + lo.tr_lo[j], ka_ + lo.tr_hi[j]);
                            }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (!need_mask) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], c2, -lse2));
                            if (DELTA_PASS) dsum += pv * dp[i];
                            else dp[i] = pv * (dp[i] - dlt);
                        }
                    } else
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], c2, -lse2));
                        if (need_mask && mb * 32 + (i >> 2) * 8 + (i & 3) > lim) pv = 0.f;
                        if (DELTA_PASS) dsum += pv * dp[i];
                        else dp[i] = pv * (dp[i] - dlt);
                    }
                    if (DELTA_PASS) continue;
                    // dQ^T += K^T dS^T : contraction over these 32 keys in 2 groups of 16
#pragma unroll
                    for (int tq = 0; tq < 2; ++tq) {
                        const bf16x8 dsb = pack8(dp[8 * tq + 0], dp[8 * tq + 1], dp[8 * tq + 2], dp[8 * tq + 3],
                                                 dp[8 * tq + 4], dp[8 * tq + 5], dp[8 * tq + 6], dp[8 * tq + 7]);
#pragma unroll
                        for (int j = 0; j < 4; ++j) dq[j] = mfma32(kt[tq][j], dsb, dq[j]);
                        if (HEAD_TILES) {   // add the bf16 rounding residual of dS
                            bf16x8 dl;
#pragma unroll
                            for (int e = 0; e < 8; ++e) dl[e] = (__bf16)(dp[8 * tq + e] - (float)dsb[e]);
#pragma unroll
                            for (int j = 0; j < 4; ++j) dq[j] = mfma32(kt[tq][j], dl, dq[j]);
                        }
                    }
                }
            }
            wait_lds_dma();
            __syncthreads();
        };
        for (int t = 0; t < n_tiles; t += 2) {
            do_tile(t, stage_a, stage_b);
            if (t + 1 < n_tiles) do_tile(t + 1, stage_b, stage_a);
        }
    };
    if (HEAD_TILES) {
        sweep(std::true_type());
        dlt = sum_with_other_half(dsum);             // the two lane halves hold different keys of the same row
        if (wave_active && iq < lq && half == 0) delta[stat_at] = dlt;
    }
    sweep(std::false_type());

    if (wave_active) {
        // dQ rows leave through this wavefront's part of the (now idle) stage buffers, whole rows per store instruction
        char *scratch = (wave < 2 ? stage_a : stage_b) + (wave & 1) * kRowScratchBytes;
        store_rows_bf16(dq, p.softmax_scale, scratch, lq - wq0, [&](int r) {
            return (char *)b.d_q + ((int64_t)(q_seg0 + wq0 + r) * b.dq_stride_tok + (int64_t)h * b.dq_stride_head) * 2;
        });
    }
}

// Blocks [0, head_blocks) do the head tiles (one per (segment, head)), the others the main work.
// wl != nullptr: the launch has one extra workgroup (the first) that builds the dK/dV work list.
__global__ __launch_bounds__(256, 2) void mfma_dq_kernel(cf_attn_bwd_params b, float *__restrict__ delta, int head_blocks,
                                                         int *wl, int capacity)
{
    // The list builder is workgroup 0: it starts with the first wave of workgroups and is long done when the
    // launch ends (as the last workgroup it would start last and could be what the launch ends with).
    if (wl != nullptr && blockIdx.x == 0) {
        build_dkv_worklist(b.f, wl, capacity);
        return;
    }
    // Two separate arrays (not one array with two halves): the compiler must see that the direct-to-LDS
    // loads of the next tile cannot alias the reads of the current one, or it waits for them too early.
    __shared__ __attribute__((aligned(16))) char stage_a[DQ_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char stage_b[DQ_STAGE_BYTES];
    const int id = (int)blockIdx.x - (wl != nullptr ? 1 : 0);
    const bool head = id < head_blocks;   // a run-time flag, uniform over the workgroup: one code path, one register allocation
    dq_body(b, delta, head ? id : id - head_blocks, head, stage_a, stage_b);
}

// Several chunks in one launch (workgroups [first_block[c], first_block[c+1]) belong to chunk c, heaviest chunk
// first): dQ and delta of a chunk depend on nothing another chunk's backward writes, so the last, partly filled
// wave of workgroups of a big chunk can be filled by the next chunk's.
struct DqBatch {
    int n;
    int first_block[CF_BWD_BATCH_MAX + 1];
    int head_blocks[CF_BWD_BATCH_MAX];
    float *delta[CF_BWD_BATCH_MAX];
    cf_attn_bwd_params b[CF_BWD_BATCH_MAX];
};
__global__ __launch_bounds__(256, 2) void mfma_dq_batch_kernel(DqBatch q)
{
    __shared__ __attribute__((aligned(16))) char stage_a[DQ_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char stage_b[DQ_STAGE_BYTES];
    int c = 0;
    while (c + 1 < q.n && (int)blockIdx.x >= q.first_block[c + 1]) ++c;
    const int id = blockIdx.x - q.first_block[c];
    const bool head = id < q.head_blocks[c];
    dq_body(q.b[c], q.delta[c], head ? id : id - q.head_blocks[c], head, stage_a, stage_b);
}

// Launch geometry of one chunk's backward.
struct BwdShape {
    bool fused;              // dK/dV: one workgroup per key tile and kv head loops over the query heads (plain RMW)
    int64_t dq_blocks, dkv_blocks;
    int head_dq, head_dkv;
    bool ok;
};
BwdShape bwd_shape(const cf_attn_fwd_params &p, const BwdWorkspace &ws)
{
    BwdShape g;
    // Upper bounds on tile counts: sum_g ceil(L_g / tile) <= total / tile + n_segments.
    const int64_t kv_tiles = (int64_t)p.n_kv_tokens / BKV + p.n_segments;
    const int64_t q_tiles = p.q_tiles ? (int64_t)p.n_q_tiles : (int64_t)p.n_tokens / BM + p.n_segments;
    // Fusing the heads of a group into one workgroup needs enough key tiles to fill 256 CUs several times.
    g.fused = kv_tiles * p.n_kv_heads >= 4096 || (p.flags & CF_FLAG_DKV_SINGLE_WRITER);
    g.dq_blocks = q_tiles * p.n_q_heads;
    g.head_dq = p.n_segments * p.n_q_heads;
    g.head_dkv = p.n_segments * p.n_kv_heads;
    g.dkv_blocks = (g.fused ? kv_tiles : ws.worklist_items) * p.n_kv_heads;
    g.ok = g.dkv_blocks + g.head_dkv <= 0x7fffffffLL && g.dq_blocks + g.head_dq <= 0x7fffffffLL && ws.worklist_items <= 0x7fffffffLL;
    return g;
}

hipError_t launch_worklist(const cf_attn_fwd_params &p, const BwdWorkspace &ws, const BwdShape &g, hipStream_t s)
{
    if (g.fused) return hipSuccess;
    dkv_worklist_kernel<<<1, 1024, 0, s>>>(p, ws.worklist, (int)ws.worklist_items);
    return hipGetLastError();
}

hipError_t launch_dkv(const cf_attn_bwd_params &b, const BwdWorkspace &ws, const BwdShape &g, const ProfileHook &hook, hipStream_t s)
{
    if (hook.start) (void)hipEventRecord(hook.start, s);
    if (g.fused) {
        // Fused mode updates dK/dV with plain read-modify-write: head blocks and main blocks of key tile 0 must
        // not run concurrently, so they get launches of their own (stream order).
        mfma_dkv_kernel<true><<<dim3((unsigned)g.dkv_blocks), 64 * DKV_WAVES, 0, s>>>(b, ws.delta, 0, nullptr, 0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        mfma_dkv_kernel<true><<<dim3((unsigned)g.head_dkv), 64 * DKV_WAVES, 0, s>>>(b, ws.delta, g.head_dkv, nullptr, 0);
        if (hook.stop) (void)hipEventRecord(hook.stop, s);      // after BOTH launches: together they are the dK/dV pass
    } else {
        mfma_dkv_kernel<false><<<dim3((unsigned)(g.dkv_blocks + g.head_dkv)), 64 * DKV_WAVES, 0, s>>>(b, ws.delta, g.head_dkv, ws.worklist,
                                                                                         (int)ws.worklist_items);
        if (hook.stop) (void)hipEventRecord(hook.stop, s);
    }
    return hipGetLastError();
}

}  // namespace

int64_t dkv_worklist_capacity(const cf_attn_fwd_params &p)
{
    // sum over segments of ceil(Lk / 128) <= n_kv_tokens / 128 + n_segments key tiles, each split in at most G items
    return ((int64_t)p.n_kv_tokens / BKV + p.n_segments) * (p.n_q_heads / p.n_kv_heads);
}

hipError_t launch_mfma_bwd(const cf_attn_bwd_params &b, const BwdWorkspace &ws, hipStream_t s)
{
    const cf_attn_fwd_params &p = b.f;
    const BwdShape g = bwd_shape(p, ws);
    if (!g.ok) return hipErrorInvalidConfiguration;
    hipError_t e;
    // dQ first: it also produces delta (main blocks: <dO, O>; head blocks: the exact sum for the head rows), which
    // the dK/dV kernel reads; its first workgroup builds the dK/dV work list where one is needed.
    int *wl = g.fused ? nullptr : ws.worklist;
    mfma_dq_kernel<<<dim3((unsigned)(g.dq_blocks + g.head_dq + (wl ? 1 : 0))), 256, 0, s>>>(b, ws.delta, g.head_dq, wl,
                                                                                             (int)ws.worklist_items);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    return launch_dkv(b, ws, g, take_profile_hook(), s);
}

// Backward of 1..CF_BWD_BATCH_MAX chunks: work lists, ONE dQ launch over all chunks (dealt in the order of `dq_order`,
// indices into chunks), then the dK/dV kernels chunk by chunk in the order of `chunks`, which is therefore the order
// in which a shared dK/dV state accumulates.
hipError_t launch_mfma_bwd_batch(const cf_attn_bwd_params *const *chunks, const BwdWorkspace *ws, const int *dq_order, int n,
                                 hipStream_t s)
{
    if (n < 1 || n > CF_BWD_BATCH_MAX) return hipErrorInvalidValue;
    BwdShape g[CF_BWD_BATCH_MAX];
    hipError_t e;
    for (int c = 0; c < n; ++c) {
        g[c] = bwd_shape(chunks[c]->f, ws[c]);
        if (!g[c].ok) return hipErrorInvalidConfiguration;
        if ((e = launch_worklist(chunks[c]->f, ws[c], g[c], s)) != hipSuccess) return e;
    }
    DqBatch q;
    q.n = n;
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        const int c = dq_order[i];
        q.first_block[i] = (int)total;
        q.head_blocks[i] = g[c].head_dq;
        q.delta[i] = ws[c].delta;
        q.b[i] = *chunks[c];
        total += g[c].dq_blocks + g[c].head_dq;
        if (total > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    }
    q.first_block[n] = (int)total;
    mfma_dq_batch_kernel<<<dim3((unsigned)total), 256, 0, s>>>(q);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    for (int c = 0; c < n; ++c)
        if ((e = launch_dkv(*chunks[c], ws[c], g[c], ProfileHook(), s)) != hipSuccess) return e;
    return hipSuccess;
}

}  // namespace cf
