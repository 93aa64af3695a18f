// bf16 MFMA backward kernels for one chunk, head_dim 128 (paper section 4.2: key/value gradients of the
// retained prefix rows are accumulated by the later chunks' backward passes; section 2.2: per-sequence
// causal mask inside a packed chunk).
//
// Two kernels, no dQ atomics:
//
//  dkv kernel  A workgroup (4 wavefronts) owns 128 consecutive key rows of one segment; each wavefront owns
//              32 of them and keeps their dK^T and dV^T (fp32, 128 registers) for the whole kernel.  It
//              loops over the 64-row query tiles that can see its keys; Q and dO tiles are staged through
//              LDS (double buffered, XOR-swizzled so that row reads and transposing reads are both free
//              of bank conflicts).  Per tile and wavefront:
//                  S = Q K_w^T          dP = dO V_w^T           (A from LDS rows, B = K_w / V_w registers)
//                  P = exp2(S c - LSE)  dS = P (dP - delta)
//                  dV_w^T += dO^T P     dK_w^T += Q^T dS        (A by transposing LDS reads, B registers)
//              FUSED_HEADS = true : the workgroup also loops over the query heads of its key/value head
//                  and is the only writer of its dK/dV rows (plain read-modify-write, bitwise
//                  reproducible).  Used when the launch has enough key tiles to fill the GPU.
//              FUSED_HEADS = false: one workgroup per (key tile, query head), 7x..8x more workgroups for
//                  short chunks; the heads of a group meet in dK/dV through fp32 atomic adds (once per
//                  workgroup, at the end).
//
//  dq kernel   Same shape as the forward kernel: a workgroup owns 128 query rows of one head, key/value
//              tiles of 64 rows go through LDS, everything transposed so that a lane owns one query:
//                  S^T = K Q^T   dP^T = V dO^T   dS^T = P^T (dP^T - delta)   dQ^T += K^T dS^T
//              LSE and delta are one scalar per lane; dS^T feeds the last product straight from registers.
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "mfma_common.h"

namespace cf {
namespace {

constexpr int D = 128;
constexpr float kLog2e = 1.44269504088896340736f;

// =====================================================================================================
// dK / dV
// =====================================================================================================
constexpr int BQ = 64;                                // query rows per tile
constexpr int BKV = 128;                              // key rows per workgroup
constexpr int QTILE_BYTES = BQ * 256;                 // one swizzled Q or dO tile
constexpr int DKV_STAGE_BYTES = 2 * QTILE_BYTES + 512;  // Q, dO, LSE[64], delta[64]

constexpr int TROW = 132;   // floats per row of the end-of-kernel transpose scratch (128 + 4)
constexpr int DKV_SMEM_BYTES = 2 * DKV_STAGE_BYTES > 4 * 32 * TROW * 4 ? 2 * DKV_STAGE_BYTES : 4 * 32 * TROW * 4;

struct QTileRegs {
    i32x4 q[4], d_o[4];
    float stat;
};

template <bool FUSED_HEADS>
__global__ __launch_bounds__(256) void mfma_dkv_kernel(cf_attn_bwd_params b, const float *__restrict__ delta)
{
    const cf_attn_fwd_params &p = b.f;
    __shared__ __attribute__((aligned(16))) char smem[DKV_SMEM_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31, r16 = lane & 15, blk = (lane >> 4) & 1;

    // Block id -> (key tile rank, head); the key/value head varies fastest (XCD L2 locality, see forward).
    const int G = p.n_q_heads / p.n_kv_heads;
    int id = blockIdx.x;
    const int kh = id % p.n_kv_heads;
    id /= p.n_kv_heads;
    const int h_first = FUSED_HEADS ? kh * G : kh * G + id % G;
    const int n_heads = FUSED_HEADS ? G : 1;
    const int rank = FUSED_HEADS ? id : id / G;

    int seg, t_rev;
    if (!locate_tile(p.cu_seqlens_k, p.n_segments, BKV, rank, seg, t_rev)) return;
    const int q_seg0 = p.cu_seqlens_q[seg], lq = p.cu_seqlens_q[seg + 1] - q_seg0;
    const int k_seg0 = p.cu_seqlens_k[seg], lk = p.cu_seqlens_k[seg + 1] - k_seg0;
    const int off = lk - lq;
    // locate_tile numbers tiles from the end; the FIRST key tiles of a segment are seen by the most rows,
    // so flip the order inside the segment to start the heaviest tiles first.
    const int kt0 = ((lk + BKV - 1) / BKV - 1 - t_rev) * BKV;
    const int i_min = max(0, kt0 - off);             // first query row that sees any key of this tile
    const int qt_first = i_min / BQ;
    const int n_qt = (lq + BQ - 1) / BQ - qt_first;  // >= 1 because kt0 < lk = lq + off
    const int n_iter = n_heads * n_qt;

    const int kv_idx = kt0 + 32 * wave + col;        // this lane's key (segment-local)
    const float c2 = p.softmax_scale * kLog2e;

    // K_w and V_w operand fragments (B operands of S and dP): lane = key row, 8 consecutive d per step
    bf16x8 kf[8], vf[8];
    {
        const int64_t row = k_seg0 + min(kv_idx, lk - 1);
        const char *kr = (const char *)p.k + (row * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2;
        const char *vr = (const char *)p.v + (row * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            kf[ks] = *(const bf16x8 *)(kr + ks * 32 + half * 16);
            vf[ks] = *(const bf16x8 *)(vr + ks * 32 + half * 16);
        }
    }

    f32x16 dk[4], dv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) dk[i][j] = dv[i][j] = 0.f;

    // tile staging: 256 threads x 4 x 16 bytes for Q and for dO; threads 0..63 LSE, 64..127 delta
    auto load_tile = [&](QTileRegs &r, int it) {
        const int h = h_first + it / n_qt;
        const int q0 = (qt_first + it % n_qt) * BQ;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int idx = tid + 256 * c;
            const int64_t row = q_seg0 + min(q0 + (idx >> 4), lq - 1);
            r.q[c] = *(const i32x4 *)((const char *)p.q + (row * p.q_stride_tok + (int64_t)h * p.q_stride_head) * 2 +
                                      (idx & 15) * 16);
            r.d_o[c] = *(const i32x4 *)((const char *)b.d_o +
                                        (row * b.do_stride_tok + (int64_t)h * b.do_stride_head) * 2 + (idx & 15) * 16);
        }
        if (tid < 128) {
            const int i = q0 + (tid & 63);
            const int64_t at = (int64_t)h * p.n_tokens + q_seg0 + min(i, lq - 1);
            // rows past the segment get LSE = +inf (P = 0) and delta = 0
            if (tid < 64) r.stat = i < lq ? p.lse[at] * kLog2e : INFINITY;
            else r.stat = i < lq ? delta[at] : 0.f;
        }
    };
    auto store_tile = [&](const QTileRegs &r, int buf) {
        char *st = smem + buf * DKV_STAGE_BYTES;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int idx = tid + 256 * c;
            const int o = tile_off(idx >> 4, idx & 15);
            *(i32x4 *)(st + o) = r.q[c];
            *(i32x4 *)(st + QTILE_BYTES + o) = r.d_o[c];
        }
        if (tid < 128) ((float *)(st + 2 * QTILE_BYTES))[tid] = r.stat;
    };

    QTileRegs regs;
    load_tile(regs, 0);
    store_tile(regs, 0);
    __syncthreads();

    for (int it = 0; it < n_iter; ++it) {
        const int q0 = (qt_first + it % n_qt) * BQ;
        const char *qs = smem + (it & 1) * DKV_STAGE_BYTES;
        const char *dos = qs + QTILE_BYTES;
        const float *lse_s = (const float *)(qs + 2 * QTILE_BYTES);
        const float *del_s = lse_s + 64;
        const bool more = it + 1 < n_iter;
        if (more) load_tile(regs, it + 1);

        // S = Q K_w^T and dP = dO V_w^T for the tile's two 32-row blocks
        f32x16 s[2], dp[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
            for (int j = 0; j < 16; ++j) s[mb][j] = dp[mb][j] = 0.f;
            const int row = mb * 32 + col;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                s[mb] = mfma32(lds_read_b128(qs + tile_off(row, 2 * ks + half)), kf[ks], s[mb]);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                dp[mb] = mfma32(lds_read_b128(dos + tile_off(row, 2 * ks + half)), vf[ks], dp[mb]);
        }
        // P and dS (register i of block mb is query row q0 + 32*mb + (i/4)*8 + 4*half + i%4, column = this lane's key)
        const bool need_mask = kt0 + BKV - 1 > q0 + off;
        // Rows among the first 128 positions of a sequence see few keys, so their P and dS are large and
        // their bf16 rounding would be the largest error in dK/dV; those tiles add the rounding residuals.
#ifdef EXP_NO_PRECISE
        const bool precise = false;
#else
        const bool precise = kt0 == 0 && q0 + off < 128;
#endif
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int rbase = mb * 32 + g4 * 8 + half * 4;
                const f32x4 l4 = *(const f32x4 *)(lse_s + rbase);
                const f32x4 d4 = *(const f32x4 *)(del_s + rbase);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = g4 * 4 + j;
                    float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][i], c2, -l4[j]));
                    if (need_mask && kv_idx > q0 + rbase + j + off) pv = 0.f;
                    s[mb][i] = pv;
                    dp[mb][i] = pv * (dp[mb][i] - d4[j]);
                }
            }
        // dV_w^T += dO^T P and dK_w^T += Q^T dS : contraction over the 64 query rows in 4 groups of 16
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int tq = 0; tq < 2; ++tq) {
                const bf16x8 pb = pack8(s[mb][8 * tq + 0], s[mb][8 * tq + 1], s[mb][8 * tq + 2], s[mb][8 * tq + 3],
                                        s[mb][8 * tq + 4], s[mb][8 * tq + 5], s[mb][8 * tq + 6], s[mb][8 * tq + 7]);
                const bf16x8 dsb = pack8(dp[mb][8 * tq + 0], dp[mb][8 * tq + 1], dp[mb][8 * tq + 2], dp[mb][8 * tq + 3],
                                         dp[mb][8 * tq + 4], dp[mb][8 * tq + 5], dp[mb][8 * tq + 6], dp[mb][8 * tq + 7]);
                // k-slot 8*half + j is query row 32*mb + 16*tq + (j/4)*8 + 4*half + j%4:
                // first transposing read rows r_lo .. r_lo+3 (by lane group), second 8 rows further
                const int r_lo = mb * 32 + 16 * tq + 4 * half + (r16 >> 2), r_hi = r_lo + 8;
                const int sub = 8 * (r16 & 1), u0 = 2 * blk + ((r16 >> 1) & 1);
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const int o_lo = tile_off(r_lo, 4 * db + u0) + sub, o_hi = tile_off(r_hi, 4 * db + u0) + sub;
                    dv[db] = mfma32(lds_read_tr_pair(dos + o_lo, dos + o_hi), pb, dv[db]);
                    dk[db] = mfma32(lds_read_tr_pair(qs + o_lo, qs + o_hi), dsb, dk[db]);
                }
                if (precise) {
                    bf16x8 pl, dl;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        pl[j] = (__bf16)(s[mb][8 * tq + j] - (float)pb[j]);
                        dl[j] = (__bf16)(dp[mb][8 * tq + j] - (float)dsb[j]);
                    }
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const int o_lo = tile_off(r_lo, 4 * db + u0) + sub, o_hi = tile_off(r_hi, 4 * db + u0) + sub;
                        dv[db] = mfma32(lds_read_tr_pair(dos + o_lo, dos + o_hi), pl, dv[db]);
                        dk[db] = mfma32(lds_read_tr_pair(qs + o_lo, qs + o_hi), dl, dk[db]);
                    }
                }
            }
        if (more) store_tile(regs, (it + 1) & 1);
        __syncthreads();
    }

    // dK, dV: lane = key row, register group g4 of block db = 4 consecutive d starting at 32*db + 8*g4 + 4*half
    if (FUSED_HEADS) {   // only writer of these rows in this launch: plain read-modify-write
        if (kv_idx < lk) {
            const int64_t row = k_seg0 + kv_idx;
            float *gk = b.d_k + row * b.dkv_stride_tok + (int64_t)kh * b.dkv_stride_head;
            float *gv = b.d_v + row * b.dkv_stride_tok + (int64_t)kh * b.dkv_stride_head;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int d0 = db * 32 + g4 * 8 + half * 4;
                    f32x4 a = *(f32x4 *)(gk + d0), c = *(f32x4 *)(gv + d0);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        a[j] += dk[db][g4 * 4 + j] * p.softmax_scale;
                        c[j] += dv[db][g4 * 4 + j];
                    }
                    *(f32x4 *)(gk + d0) = a;
                    *(f32x4 *)(gv + d0) = c;
                }
        }
    } else {
        // The query heads of a group add into the same rows: fp32 atomics.  A lane-per-row atomic touches
        // 64 cache lines per instruction, so each wavefront first turns its 32 x 128 block around in LDS
        // (its own 16.5 KB slice of the workgroup's LDS, free after the loop's last barrier) and then adds
        // whole rows: 64 lanes = 64 consecutive floats.
        float *tr = (float *)smem + wave * 32 * TROW;
        const int rows_valid = min(32, lk - (kt0 + 32 * wave));      // <= 0: this wavefront has no real keys
#pragma unroll
        for (int which = 0; which < 2; ++which) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    f32x4 a;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        a[j] = which == 0 ? dk[db][g4 * 4 + j] * p.softmax_scale : dv[db][g4 * 4 + j];
                    *(f32x4 *)(tr + col * TROW + db * 32 + g4 * 8 + half * 4) = a;
                }
            __builtin_amdgcn_wave_barrier();
            float *gbase = (which == 0 ? b.d_k : b.d_v) + (int64_t)(k_seg0 + kt0 + 32 * wave) * b.dkv_stride_tok +
                           (int64_t)kh * b.dkv_stride_head;
            for (int r = 0; r < rows_valid; ++r) {
                unsafeAtomicAdd(gbase + (int64_t)r * b.dkv_stride_tok + lane, tr[r * TROW + lane]);
                unsafeAtomicAdd(gbase + (int64_t)r * b.dkv_stride_tok + 64 + lane, tr[r * TROW + 64 + lane]);
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// =====================================================================================================
// dQ
// =====================================================================================================
constexpr int BM = 128;                      // query rows per workgroup
constexpr int BN = 64;                       // key rows per tile
constexpr int KVTILE_BYTES = BN * 256;       // one swizzled K or V tile
constexpr int DQ_STAGE_BYTES = 2 * KVTILE_BYTES;

struct KVTileRegs {
    i32x4 k[4], v[4];
};

__global__ __launch_bounds__(256, 2) void mfma_dq_kernel(cf_attn_bwd_params b, const float *__restrict__ delta)
{
    const cf_attn_fwd_params &p = b.f;
    __shared__ __attribute__((aligned(16))) char smem[2 * DQ_STAGE_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31, r16 = lane & 15, blk = (lane >> 4) & 1;

    const int G = p.n_q_heads / p.n_kv_heads;
    int id = blockIdx.x;
    const int kh = id % p.n_kv_heads;
    id /= p.n_kv_heads;
    const int h = kh * G + id % G;
    const int rank = id / G;

    int seg, tile_in_seg;
    if (!locate_tile(p.cu_seqlens_q, p.n_segments, BM, rank, seg, tile_in_seg)) return;
    const int q_seg0 = p.cu_seqlens_q[seg], lq = p.cu_seqlens_q[seg + 1] - q_seg0;
    const int k_seg0 = p.cu_seqlens_k[seg], lk = p.cu_seqlens_k[seg + 1] - k_seg0;
    const int off = lk - lq;
    const int q_tile0 = tile_in_seg * BM;
    const int rows_valid = min(BM, lq - q_tile0);
    const int kmax = q_tile0 + rows_valid + off;     // keys [0, kmax) are visible to some row of the tile
    const int n_tiles = (kmax + BN - 1) / BN;
    const int wq0 = q_tile0 + wave * 32;
    const int wave_kmax = min(kmax, wq0 + 32 + off);
    const bool wave_active = wq0 < lq;
    const int iq = wq0 + col;                        // this lane's query row
    const int amax = iq + off;                       // last visible key of this lane's row
    // rows among the first 128 positions of a sequence: carry dS as bf16 value + bf16 residual
    const bool precise = q_tile0 + off < 128;

    const int64_t kv_row_bytes = p.kv_stride_tok * 2;
    const char *kbase = (const char *)p.k + ((int64_t)k_seg0 * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2;
    const char *vbase = (const char *)p.v + ((int64_t)k_seg0 * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2;

    // Q^T and dO^T fragments (B operands): lane holds row iq, d = 16*ks + 8*half + 0..7
    bf16x8 qf[8], dof[8];
    float lse2, dlt;
    {
        const int row = q_seg0 + min(iq, lq - 1);
        const char *qrow = (const char *)p.q + ((int64_t)row * p.q_stride_tok + (int64_t)h * p.q_stride_head) * 2;
        const char *dorow = (const char *)b.d_o + ((int64_t)row * b.do_stride_tok + (int64_t)h * b.do_stride_head) * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            qf[ks] = *(const bf16x8 *)(qrow + ks * 32 + half * 16);
            dof[ks] = *(const bf16x8 *)(dorow + ks * 32 + half * 16);
        }
        lse2 = iq < lq ? p.lse[(int64_t)h * p.n_tokens + row] * kLog2e : INFINITY;   // padding rows: P = 0
        dlt = delta[(int64_t)h * p.n_tokens + row];
    }
    const float c2 = p.softmax_scale * kLog2e;

    f32x16 dq[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) dq[i][j] = 0.f;

    auto load_tile = [&](KVTileRegs &r, int tile_start) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int idx = tid + 256 * c;
            const int row = min(tile_start + (idx >> 4), lk - 1);
            const int64_t o = (int64_t)row * kv_row_bytes + (idx & 15) * 16;
            r.k[c] = *(const i32x4 *)(kbase + o);
            r.v[c] = *(const i32x4 *)(vbase + o);
        }
    };
    auto store_tile = [&](const KVTileRegs &r, char *stage) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int idx = tid + 256 * c;
            const int o = tile_off(idx >> 4, idx & 15);
            *(i32x4 *)(stage + o) = r.k[c];
            *(i32x4 *)(stage + KVTILE_BYTES + o) = r.v[c];
        }
    };

    KVTileRegs regs;
    load_tile(regs, 0);
    store_tile(regs, smem);
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
        const int tile_start = t * BN;
        char *stage = smem + (t & 1) * DQ_STAGE_BYTES;
        const char *ks_ = stage;
        const char *vs_ = stage + KVTILE_BYTES;
        const bool more = t + 1 < n_tiles;
        if (more) load_tile(regs, tile_start + BN);

        if (wave_active && tile_start < wave_kmax) {
            const bool need_mask = tile_start + BN - 1 > wq0 + off;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                // S^T and dP^T for 32 keys: register i is key tile_start + 32*mb + (i/4)*8 + 4*half + i%4
                f32x16 s, dp;
#pragma unroll
                for (int j = 0; j < 16; ++j) s[j] = dp[j] = 0.f;
                const int row = mb * 32 + col;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    s = mfma32(lds_read_b128(ks_ + tile_off(row, 2 * ks + half)), qf[ks], s);
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    dp = mfma32(lds_read_b128(vs_ + tile_off(row, 2 * ks + half)), dof[ks], dp);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], c2, -lse2));
                    if (need_mask && tile_start + mb * 32 + (i >> 2) * 8 + half * 4 + (i & 3) > amax) pv = 0.f;
                    dp[i] = pv * (dp[i] - dlt);
                }
                // dQ^T += K^T dS^T : contraction over these 32 keys in 2 groups of 16
#pragma unroll
                for (int tq = 0; tq < 2; ++tq) {
                    const bf16x8 dsb = pack8(dp[8 * tq + 0], dp[8 * tq + 1], dp[8 * tq + 2], dp[8 * tq + 3],
                                             dp[8 * tq + 4], dp[8 * tq + 5], dp[8 * tq + 6], dp[8 * tq + 7]);
                    const int r_lo = mb * 32 + 16 * tq + 4 * half + (r16 >> 2), r_hi = r_lo + 8;
                    const int sub = 8 * (r16 & 1), u0 = 2 * blk + ((r16 >> 1) & 1);
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const int o_lo = tile_off(r_lo, 4 * db + u0) + sub, o_hi = tile_off(r_hi, 4 * db + u0) + sub;
                        dq[db] = mfma32(lds_read_tr_pair(ks_ + o_lo, ks_ + o_hi), dsb, dq[db]);
                    }
                    if (precise) {
                        bf16x8 dl;
#pragma unroll
                        for (int j = 0; j < 8; ++j) dl[j] = (__bf16)(dp[8 * tq + j] - (float)dsb[j]);
#pragma unroll
                        for (int db = 0; db < 4; ++db) {
                            const int o_lo = tile_off(r_lo, 4 * db + u0) + sub, o_hi = tile_off(r_hi, 4 * db + u0) + sub;
                            dq[db] = mfma32(lds_read_tr_pair(ks_ + o_lo, ks_ + o_hi), dl, dq[db]);
                        }
                    }
                }
            }
        }
        if (more) store_tile(regs, smem + ((t + 1) & 1) * DQ_STAGE_BYTES);
        __syncthreads();
    }

    if (wave_active && iq < lq) {
        const int row = q_seg0 + iq;
        char *out = (char *)b.d_q + ((int64_t)row * b.dq_stride_tok + (int64_t)h * b.dq_stride_head) * 2;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                bf16x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = (__bf16)(dq[db][g4 * 4 + j] * p.softmax_scale);
                *(bf16x4 *)(out + (db * 32 + g4 * 8 + half * 4) * 2) = w;
            }
    }
}

}  // namespace

hipError_t launch_mfma_bwd(const cf_attn_bwd_params &b, const BwdWorkspace &ws, hipStream_t s)
{
    const cf_attn_fwd_params &p = b.f;
    // Upper bounds on tile counts: sum_g ceil(L_g / tile) <= total / tile + n_segments.
    const int64_t kv_tiles = (int64_t)p.n_kv_tokens / BKV + p.n_segments;
    const int64_t q_tiles = (int64_t)p.n_tokens / BM + p.n_segments;
    // Fusing the heads of a group into one workgroup needs enough key tiles to fill 256 CUs several times.
#ifdef EXP_FORCE_FUSED
    const bool fused = true;
#else
    const bool fused = kv_tiles * p.n_kv_heads >= 4096;
#endif
    const int64_t dkv_blocks = kv_tiles * (fused ? p.n_kv_heads : p.n_q_heads);
    const int64_t dq_blocks = q_tiles * p.n_q_heads;
    if (dkv_blocks > 0x7fffffffLL || dq_blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const ProfileHook hook = take_profile_hook();
    if (hook.start) (void)hipEventRecord(hook.start, s);
    if (fused) mfma_dkv_kernel<true><<<dim3((unsigned)dkv_blocks), 256, 0, s>>>(b, ws.delta);
    else mfma_dkv_kernel<false><<<dim3((unsigned)dkv_blocks), 256, 0, s>>>(b, ws.delta);
    hipError_t e = hipGetLastError();
    if (hook.stop) (void)hipEventRecord(hook.stop, s);
    if (e != hipSuccess) return e;
    mfma_dq_kernel<<<dim3((unsigned)dq_blocks), 256, 0, s>>>(b, ws.delta);
    return hipGetLastError();
}

}  // namespace cf
