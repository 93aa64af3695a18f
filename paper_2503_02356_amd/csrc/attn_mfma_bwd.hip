// bf16 MFMA backward kernel for one chunk, head_dim 128 (paper section 4.2: key/value gradients of the
// retained prefix rows are accumulated by the later chunks' backward passes; section 2.2: per-sequence
// causal mask inside a packed chunk).
//
// One workgroup = 4 wavefronts owns 128 consecutive key rows of one segment and one key/value head; each
// wavefront owns 32 of them and keeps their dK^T and dV^T (fp32, 128 registers) for the whole kernel.
// The workgroup loops over the query heads of the group and over the 64-row query tiles that can see
// its keys; Q and dO tiles are staged through LDS (double buffered).  Per tile and wavefront:
//     S  = Q K_w^T            dP = dO V_w^T              (A from LDS rows, B = K_w / V_w in registers)
//     P  = exp2(S c - LSE)    dS = P (dP - delta)
//     dV_w^T += dO^T P        dK_w^T += Q^T dS           (A through transposing LDS reads, B from registers)
//     dQ[:, 32w..32w+32) += dS_all K[:, 32w..32w+32)     (dS of all four wavefronts exchanged through LDS)
// The workgroup is the only writer of its dK/dV rows (plain read-modify-write at the end, so results are
// bitwise reproducible); dQ partial sums from different key tiles meet in an fp32 accumulator through
// atomic adds and are scaled and converted by a second small kernel.
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "mfma_common.h"

namespace cf {
namespace {

constexpr int BQ = 64;          // query rows per tile
constexpr int BKV = 128;        // key rows per workgroup
constexpr int D = 128;
constexpr int ROW = 272;        // LDS bytes per Q / dO / K row (256 + 16)
constexpr int DST_ROW = 192;    // LDS bytes per dS^T row (64 queries * 2 + 64)
constexpr int TILE_BYTES = BQ * ROW;                 // one Q or dO tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES + 512;    // Q, dO, LSE[64], delta[64]
constexpr int DST_BYTES = BKV * DST_ROW;
constexpr int SMEM_BYTES = 2 * STAGE_BYTES + 2 * DST_BYTES;   // dS^T twice: bf16 value and its rounding residual
static_assert(BKV * ROW <= 2 * STAGE_BYTES, "the K tile is staged over the Q/dO buffers before the main loop");

struct TileRegs {
    i32x4 q[4], d_o[4];
    float stat;
};

__global__ __launch_bounds__(256) void mfma_bwd_kernel(cf_attn_bwd_params b, const float *__restrict__ delta,
                                                      float *__restrict__ dq_acc)
{
    const cf_attn_fwd_params &p = b.f;
    __shared__ __attribute__((aligned(16))) char smem[SMEM_BYTES];
    char *dst = smem + 2 * STAGE_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31, r16 = lane & 15, blk = (lane >> 4) & 1;

    const int G = p.n_q_heads / p.n_kv_heads;
    const int kh = blockIdx.x % p.n_kv_heads;
    const int rank = blockIdx.x / p.n_kv_heads;
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
    const int n_iter = G * n_qt;

    const int kv_local = 32 * wave + col;            // this lane's key row inside the tile
    const int kv_idx = kt0 + kv_local;               // segment-local key index
    const float c2 = p.softmax_scale * 1.44269504088896340736f;

    // ---- K_w and V_w operand fragments (B operands of S and dP): lane = key row, 8 consecutive d per step
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
    // ---- K[:, 32w..32w+32) as B operand of dQ = dS K (contraction over the 128 keys): staged through LDS
    //      once and read transposed; k-slot 8*half + j of step ks is key 16*ks + 8*half + j.
    bf16x8 kt[8];
    {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int idx = tid + 256 * c, row = idx >> 4;
            const int64_t grow = k_seg0 + min(kt0 + row, lk - 1);
            const char *src = (const char *)p.k + (grow * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head) * 2;
            *(i32x4 *)(smem + row * ROW + (idx & 15) * 16) = *(const i32x4 *)(src + (idx & 15) * 16);
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const char *a = smem + (16 * ks + 8 * half + (r16 >> 2)) * ROW + (32 * wave + 16 * blk + 4 * (r16 & 3)) * 2;
            kt[ks] = lds_read_tr_pair(a, a + 4 * ROW);
        }
        __syncthreads();
    }

    f32x16 dk[4], dv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) dk[i][j] = dv[i][j] = 0.f;

    // ---- tile staging: 256 threads x 4 x 16 bytes for Q and for dO; threads 0..63 LSE, 64..127 delta
    auto load_tile = [&](TileRegs &r, int it) {
        const int h = kh * G + it / n_qt;
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
            if (tid < 64) r.stat = i < lq ? p.lse[at] * 1.44269504088896340736f : INFINITY;
            else r.stat = i < lq ? delta[at] : 0.f;
        }
    };
    auto store_tile = [&](const TileRegs &r, int buf) {
        char *st = smem + buf * STAGE_BYTES;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int idx = tid + 256 * c;
            *(i32x4 *)(st + (idx >> 4) * ROW + (idx & 15) * 16) = r.q[c];
            *(i32x4 *)(st + TILE_BYTES + (idx >> 4) * ROW + (idx & 15) * 16) = r.d_o[c];
        }
        if (tid < 128) ((float *)(st + 2 * TILE_BYTES))[tid] = r.stat;
    };

    TileRegs regs;
    load_tile(regs, 0);
    store_tile(regs, 0);
    __syncthreads();

    for (int it = 0; it < n_iter; ++it) {
        const int h = kh * G + it / n_qt;
        const int q0 = (qt_first + it % n_qt) * BQ;
        const char *qs = smem + (it & 1) * STAGE_BYTES;
        const char *dos = qs + TILE_BYTES;
        const float *lse_s = (const float *)(qs + 2 * TILE_BYTES);
        const float *del_s = lse_s + 64;
        const bool more = it + 1 < n_iter;
        if (more) load_tile(regs, it + 1);

        // ---- S = Q K_w^T and dP = dO V_w^T for the tile's two 32-row blocks
        f32x16 s[2], dp[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
            for (int j = 0; j < 16; ++j) s[mb][j] = dp[mb][j] = 0.f;
            const int arow = (mb * 32 + col) * ROW + half * 16;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) s[mb] = mfma32(lds_read_b128(qs + arow + ks * 32), kf[ks], s[mb]);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) dp[mb] = mfma32(lds_read_b128(dos + arow + ks * 32), vf[ks], dp[mb]);
        }
        // ---- P and dS (register i of block mb is query row q0 + 32*mb + (i/4)*8 + 4*half + i%4, column = this lane's key)
        const bool need_mask = kt0 + BKV - 1 > q0 + off;
        // Rows among the first 128 positions of a sequence see few keys, so their P and dS are large and the
        // bf16 rounding of dS would show in dQ (whose own bf16 rounding already uses most of the error
        // budget for |dQ| >= 4).  For those tiles dS is carried as bf16 value + bf16 residual into dQ.
        const bool precise = kt0 == 0 && q0 + off < 128;
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
                // dS^T[key][query] for the dQ contraction: 4 consecutive query rows = 8 bytes
                bf16x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = (__bf16)dp[mb][g4 * 4 + j];
                *(bf16x4 *)(dst + kv_local * DST_ROW + rbase * 2) = w;
                if (precise) {
                    bf16x4 lo;
#pragma unroll
                    for (int j = 0; j < 4; ++j) lo[j] = (__bf16)(dp[mb][g4 * 4 + j] - (float)w[j]);
                    *(bf16x4 *)(dst + DST_BYTES + kv_local * DST_ROW + rbase * 2) = lo;
                }
            }
        // ---- dV_w^T += dO^T P and dK_w^T += Q^T dS : contraction over the 64 query rows in 4 groups of 16
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int tq = 0; tq < 2; ++tq) {
                const bf16x8 pb = pack8(s[mb][8 * tq + 0], s[mb][8 * tq + 1], s[mb][8 * tq + 2], s[mb][8 * tq + 3],
                                        s[mb][8 * tq + 4], s[mb][8 * tq + 5], s[mb][8 * tq + 6], s[mb][8 * tq + 7]);
                const bf16x8 dsb = pack8(dp[mb][8 * tq + 0], dp[mb][8 * tq + 1], dp[mb][8 * tq + 2], dp[mb][8 * tq + 3],
                                         dp[mb][8 * tq + 4], dp[mb][8 * tq + 5], dp[mb][8 * tq + 6], dp[mb][8 * tq + 7]);
                // k-slot 8*half + j is query row 32*mb + 16*tq + (j/4)*8 + 4*half + j%4
                const int a_off = (mb * 32 + 16 * tq + 4 * half + (r16 >> 2)) * ROW + (16 * blk + 4 * (r16 & 3)) * 2;
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const bf16x8 a_do = lds_read_tr_pair(dos + a_off + db * 64, dos + a_off + db * 64 + 8 * ROW);
                    dv[db] = mfma32(a_do, pb, dv[db]);
                    const bf16x8 a_q = lds_read_tr_pair(qs + a_off + db * 64, qs + a_off + db * 64 + 8 * ROW);
                    dk[db] = mfma32(a_q, dsb, dk[db]);
                }
                if (precise) {   // add the bf16 rounding residuals of P and dS
                    bf16x8 pl, dl;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        pl[j] = (__bf16)(s[mb][8 * tq + j] - (float)pb[j]);
                        dl[j] = (__bf16)(dp[mb][8 * tq + j] - (float)dsb[j]);
                    }
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const bf16x8 a_do = lds_read_tr_pair(dos + a_off + db * 64, dos + a_off + db * 64 + 8 * ROW);
                        dv[db] = mfma32(a_do, pl, dv[db]);
                        const bf16x8 a_q = lds_read_tr_pair(qs + a_off + db * 64, qs + a_off + db * 64 + 8 * ROW);
                        dk[db] = mfma32(a_q, dl, dk[db]);
                    }
                }
            }
        __syncthreads();   // dS^T of all four wavefronts is in LDS
        // ---- dQ[64 x 32 columns of this wavefront] = dS[64 x 128 keys] K[128 keys x 32]
        f32x16 dq[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
            for (int j = 0; j < 16; ++j) dq[mb][j] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const char *a = dst + (16 * ks + 8 * half + (r16 >> 2)) * DST_ROW + (mb * 32 + 16 * blk + 4 * (r16 & 3)) * 2;
                dq[mb] = mfma32(lds_read_tr_pair(a, a + 4 * DST_ROW), kt[ks], dq[mb]);
            }
            if (precise) {
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const char *a = dst + DST_BYTES + (16 * ks + 8 * half + (r16 >> 2)) * DST_ROW +
                                    (mb * 32 + 16 * blk + 4 * (r16 & 3)) * 2;
                    dq[mb] = mfma32(lds_read_tr_pair(a, a + 4 * DST_ROW), kt[ks], dq[mb]);
                }
            }
        }
        {
            float *acc = dq_acc + ((int64_t)q_seg0 * p.n_q_heads + h) * D + 32 * wave + col;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int qrow = q0 + mb * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
                    if (qrow < lq) unsafeAtomicAdd(acc + (int64_t)qrow * p.n_q_heads * D, dq[mb][i]);
                }
        }
        if (more) store_tile(regs, (it + 1) & 1);
        __syncthreads();   // next tile staged; dS^T buffer free again
    }

    // ---- dK, dV: this workgroup is the only writer of these rows in this launch
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
}

// dQ = bf16(scale * dq_acc); 8 elements per thread.
__global__ __launch_bounds__(256) void dq_convert_kernel(cf_attn_bwd_params b, const float *__restrict__ dq_acc)
{
    const cf_attn_fwd_params &p = b.f;
    const int64_t n8 = (int64_t)p.n_tokens * p.n_q_heads * (D / 8);
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const int64_t th = i / (D / 8);
    const int d0 = (int)(i % (D / 8)) * 8;
    const int64_t tok = th / p.n_q_heads, h = th % p.n_q_heads;
    const f32x4 a = *(const f32x4 *)(dq_acc + th * D + d0), c = *(const f32x4 *)(dq_acc + th * D + d0 + 4);
    const float s = p.softmax_scale;
    const bf16x8 w = pack8(a[0] * s, a[1] * s, a[2] * s, a[3] * s, c[0] * s, c[1] * s, c[2] * s, c[3] * s);
    *(bf16x8 *)((char *)b.d_q + (tok * b.dq_stride_tok + h * b.dq_stride_head + d0) * 2) = w;
}

}  // namespace

hipError_t launch_mfma_bwd(const cf_attn_bwd_params &b, const BwdWorkspace &ws, hipStream_t s)
{
    const cf_attn_fwd_params &p = b.f;
    const int64_t tiles_max = (int64_t)p.n_kv_tokens / BKV + p.n_segments;
    const int64_t blocks = tiles_max * p.n_kv_heads;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const ProfileHook hook = take_profile_hook();
    if (hook.start) (void)hipEventRecord(hook.start, s);
    mfma_bwd_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(b, ws.delta, ws.dq_acc);
    hipError_t e = hipGetLastError();
    if (hook.stop) (void)hipEventRecord(hook.stop, s);
    if (e != hipSuccess) return e;
    const int64_t n8 = (int64_t)p.n_tokens * p.n_q_heads * (D / 8);
    dq_convert_kernel<<<dim3((unsigned)((n8 + 255) / 256)), 256, 0, s>>>(b, ws.dq_acc);
    return hipGetLastError();
}

}  // namespace cf
