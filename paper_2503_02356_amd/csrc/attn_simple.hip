// Plain scalar attention kernels for one chunk: fp32 arithmetic, fp32 or bf16 storage.
// One wavefront per query row (forward, dQ) or per key row (dK/dV).  They serve the fp32
// configuration and every shape the MFMA kernels do not cover.
//
// Math (paper sections 2.1, 2.2, 4.2 give the masking and the state dependency; the formulas are
// the standard softmax-attention gradient):
//   query i of a segment sees keys j <= i + (Lk - Lq);  S = scale * q.k;  P = exp(S - LSE);
//   O = sum_j P v_j;  dV_j += sum_i P dO_i;  dS = P (dO_i.v_j - delta_i);
//   dQ_i = scale sum_j dS k_j;  dK_j += scale sum_i dS q_i.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace cf {
namespace {

constexpr int kWaves = 4;  // wavefronts per workgroup

__device__ inline float ld(const float *p) { return *p; }
__device__ inline float ld(const unsigned short *p) { return __uint_as_float(((unsigned)*p) << 16); }
__device__ inline void st(float *p, float x) { *p = x; }
__device__ inline void st(unsigned short *p, float x)
{  // round to nearest even bf16
    unsigned u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    *p = (unsigned short)(u >> 16);
}

__device__ inline float wave_max(float x)
{
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ inline float wave_sum(float x)
{
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// Largest g in [0, n) with cu[g] <= row  (cu non-decreasing, cu[0] = 0, zero-length segments skipped).
__device__ inline int find_segment(const int32_t *cu, int n, int row)
{
    int lo = 0, hi = n;  // invariant: cu[lo] <= row < cu[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= row) lo = mid; else hi = mid;
    }
    return lo;
}

template <typename T, int D>
__global__ __launch_bounds__(kWaves * 64) void simple_fwd_kernel(cf_attn_fwd_params p)
{
    __shared__ float sq[kWaves][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * kWaves + wave;
    if (row >= p.n_tokens) return;  // whole wavefront leaves together; no barrier below
    const int h = blockIdx.y, kh = h / (p.n_q_heads / p.n_kv_heads);
    const int g = find_segment(p.cu_seqlens_q, p.n_segments, row);
    const int q0 = p.cu_seqlens_q[g], lq = p.cu_seqlens_q[g + 1] - q0;
    const int k0 = p.cu_seqlens_k[g], lk = p.cu_seqlens_k[g + 1] - k0;
    const int n_vis = lk - lq + (row - q0) + 1;
    const T *q = (const T *)p.q + (int64_t)row * p.q_stride_tok + (int64_t)h * p.q_stride_head;
    const T *kb = (const T *)p.k + (int64_t)kh * p.kv_stride_head;
    const T *vb = (const T *)p.v + (int64_t)kh * p.kv_stride_head;
    constexpr int DPL = D / 64;
    for (int t = 0; t < DPL; ++t) sq[wave][lane + 64 * t] = ld(q + lane + 64 * t);
    __builtin_amdgcn_wave_barrier();
    float m = -INFINITY, z = 0.f, acc[DPL];
    for (int t = 0; t < DPL; ++t) acc[t] = 0.f;
    for (int j0 = 0; j0 < n_vis; j0 += 64) {
        const int j = j0 + lane;
        float s = -INFINITY;
        if (j < n_vis) {
            const T *kj = kb + (int64_t)(k0 + j) * p.kv_stride_tok;
            float d = 0.f;
            for (int x = 0; x < D; ++x) d += sq[wave][x] * ld(kj + x);
            s = d * p.softmax_scale;
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float pr = (j < n_vis) ? expf(s - m_new) : 0.f;
        const float corr = expf(m - m_new);  // m = -inf on the first block gives 0
        z = z * corr + wave_sum(pr);
        for (int t = 0; t < DPL; ++t) acc[t] *= corr;
        const int cnt = min(64, n_vis - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(pr, jj);
            const T *vj = vb + (int64_t)(k0 + j0 + jj) * p.kv_stride_tok;
            for (int t = 0; t < DPL; ++t) acc[t] += pj * ld(vj + lane + 64 * t);
        }
        m = m_new;
    }
    T *o = (T *)p.o + (int64_t)row * p.o_stride_tok + (int64_t)h * p.o_stride_head;
    const float inv = 1.f / z;
    for (int t = 0; t < DPL; ++t) st(o + lane + 64 * t, acc[t] * inv);
    if (lane == 0) p.lse[(int64_t)h * p.n_tokens + row] = m + logf(z);
}

template <typename T, int D>
__global__ __launch_bounds__(kWaves * 64) void simple_dq_kernel(cf_attn_bwd_params b, const float *delta)
{
    const cf_attn_fwd_params &p = b.f;
    __shared__ float sq[kWaves][D], sdo[kWaves][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * kWaves + wave;
    if (row >= p.n_tokens) return;
    const int h = blockIdx.y, kh = h / (p.n_q_heads / p.n_kv_heads);
    const int g = find_segment(p.cu_seqlens_q, p.n_segments, row);
    const int q0 = p.cu_seqlens_q[g], lq = p.cu_seqlens_q[g + 1] - q0;
    const int k0 = p.cu_seqlens_k[g], lk = p.cu_seqlens_k[g + 1] - k0;
    const int n_vis = lk - lq + (row - q0) + 1;
    const T *q = (const T *)p.q + (int64_t)row * p.q_stride_tok + (int64_t)h * p.q_stride_head;
    const T *d_o = (const T *)b.d_o + (int64_t)row * b.do_stride_tok + (int64_t)h * b.do_stride_head;
    const T *kb = (const T *)p.k + (int64_t)kh * p.kv_stride_head;
    const T *vb = (const T *)p.v + (int64_t)kh * p.kv_stride_head;
    constexpr int DPL = D / 64;
    for (int t = 0; t < DPL; ++t) {
        sq[wave][lane + 64 * t] = ld(q + lane + 64 * t);
        sdo[wave][lane + 64 * t] = ld(d_o + lane + 64 * t);
    }
    __builtin_amdgcn_wave_barrier();
    const float lse = p.lse[(int64_t)h * p.n_tokens + row];
    const float dl = delta[(int64_t)h * p.n_tokens + row];
    float acc[DPL];
    for (int t = 0; t < DPL; ++t) acc[t] = 0.f;
    for (int j0 = 0; j0 < n_vis; j0 += 64) {
        const int j = j0 + lane;
        float ds = 0.f;
        if (j < n_vis) {
            const T *kj = kb + (int64_t)(k0 + j) * p.kv_stride_tok;
            const T *vj = vb + (int64_t)(k0 + j) * p.kv_stride_tok;
            float s = 0.f, dp = 0.f;
            for (int x = 0; x < D; ++x) {
                s += sq[wave][x] * ld(kj + x);
                dp += sdo[wave][x] * ld(vj + x);
            }
            ds = expf(s * p.softmax_scale - lse) * (dp - dl);
        }
        const int cnt = min(64, n_vis - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float dj = __shfl(ds, jj);
            const T *kj = kb + (int64_t)(k0 + j0 + jj) * p.kv_stride_tok;
            for (int t = 0; t < DPL; ++t) acc[t] += dj * ld(kj + lane + 64 * t);
        }
    }
    T *dq = (T *)b.d_q + (int64_t)row * b.dq_stride_tok + (int64_t)h * b.dq_stride_head;
    for (int t = 0; t < DPL; ++t) st(dq + lane + 64 * t, acc[t] * p.softmax_scale);
}

// One wavefront per (key row, key/value head): the only writer of that row of dK and dV.
template <typename T, int D>
__global__ __launch_bounds__(kWaves * 64) void simple_dkv_kernel(cf_attn_bwd_params b, const float *delta)
{
    const cf_attn_fwd_params &p = b.f;
    __shared__ float sk[kWaves][D], sv[kWaves][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int krow = blockIdx.x * kWaves + wave;
    if (krow >= p.n_kv_tokens) return;
    const int kh = blockIdx.y, G = p.n_q_heads / p.n_kv_heads;
    const int g = find_segment(p.cu_seqlens_k, p.n_segments, krow);
    const int q0 = p.cu_seqlens_q[g], lq = p.cu_seqlens_q[g + 1] - q0;
    const int k0 = p.cu_seqlens_k[g], lk = p.cu_seqlens_k[g + 1] - k0;
    const int j = krow - k0, prefix = lk - lq;
    const int i_first = j > prefix ? j - prefix : 0;  // first query row that sees this key
    const T *kj = (const T *)p.k + (int64_t)krow * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head;
    const T *vj = (const T *)p.v + (int64_t)krow * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head;
    constexpr int DPL = D / 64;
    for (int t = 0; t < DPL; ++t) {
        sk[wave][lane + 64 * t] = ld(kj + lane + 64 * t);
        sv[wave][lane + 64 * t] = ld(vj + lane + 64 * t);
    }
    __builtin_amdgcn_wave_barrier();
    float dk[DPL], dv[DPL];
    for (int t = 0; t < DPL; ++t) dk[t] = dv[t] = 0.f;
    for (int h = kh * G; h < (kh + 1) * G; ++h) {
        const T *qb = (const T *)p.q + (int64_t)h * p.q_stride_head;
        const T *dob = (const T *)b.d_o + (int64_t)h * b.do_stride_head;
        for (int i0 = i_first; i0 < lq; i0 += 64) {
            const int i = i0 + lane;
            float pr = 0.f, ds = 0.f;
            if (i < lq) {
                const T *qi = qb + (int64_t)(q0 + i) * p.q_stride_tok;
                const T *doi = dob + (int64_t)(q0 + i) * b.do_stride_tok;
                float s = 0.f, dp = 0.f;
                for (int x = 0; x < D; ++x) {
                    s += ld(qi + x) * sk[wave][x];
                    dp += ld(doi + x) * sv[wave][x];
                }
                pr = expf(s * p.softmax_scale - p.lse[(int64_t)h * p.n_tokens + q0 + i]);
                ds = pr * (dp - delta[(int64_t)h * p.n_tokens + q0 + i]);
            }
            const int cnt = min(64, lq - i0);
            for (int ii = 0; ii < cnt; ++ii) {
                const float pi = __shfl(pr, ii), di = __shfl(ds, ii);
                const T *qi = qb + (int64_t)(q0 + i0 + ii) * p.q_stride_tok;
                const T *doi = dob + (int64_t)(q0 + i0 + ii) * b.do_stride_tok;
                for (int t = 0; t < DPL; ++t) {
                    dv[t] += pi * ld(doi + lane + 64 * t);
                    dk[t] += di * ld(qi + lane + 64 * t);
                }
            }
        }
    }
    float *gk = b.d_k + (int64_t)krow * b.dkv_stride_tok + (int64_t)kh * b.dkv_stride_head;
    float *gv = b.d_v + (int64_t)krow * b.dkv_stride_tok + (int64_t)kh * b.dkv_stride_head;
    for (int t = 0; t < DPL; ++t) {
        gk[lane + 64 * t] += dk[t] * p.softmax_scale;
        gv[lane + 64 * t] += dv[t];
    }
}

// delta[h][t] = <dO_t, O_t>: 16 lanes per (token, head), 8 (or 4) consecutive d per lane and step.
template <typename T, int D>
__global__ __launch_bounds__(256) void delta_kernel(cf_attn_bwd_params b, float *delta)
{
    const cf_attn_fwd_params &p = b.f;
    const int64_t pair = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);   // (token, head) pair
    const int sub = threadIdx.x & 15;
    float s = 0.f;
    int64_t row = 0, h = 0;
    const bool live = pair < (int64_t)p.n_tokens * p.n_q_heads;
    if (live) {
        row = pair / p.n_q_heads;
        h = pair % p.n_q_heads;
        const T *o = (const T *)p.o + row * p.o_stride_tok + h * p.o_stride_head;
        const T *d_o = (const T *)b.d_o + row * b.do_stride_tok + h * b.do_stride_head;
        constexpr int V = 16 / sizeof(T);   // elements per 16-byte load
        for (int d0 = sub * V; d0 < D; d0 += 16 * V) {
            const uint4 a = *(const uint4 *)(o + d0), c = *(const uint4 *)(d_o + d0);
            const T *pa = (const T *)&a, *pc = (const T *)&c;
#pragma unroll
            for (int j = 0; j < V; ++j) s += ld(pa + j) * ld(pc + j);
        }
    }
    for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (live && sub == 0) delta[h * p.n_tokens + row] = s;
}

// O arrives rounded to the storage type, and for a row that sees only a few keys (large P, large |O|)
// that rounding would be the largest error of the whole backward pass (it lands in dK of the first keys of
// each sequence).  Rows that see at most 64 keys therefore get delta = sum_j P_tj <dO_t, v_j> instead,
// one key per lane, which needs no O at all.  One wavefront per (segment, one of its first 64 rows, head);
// runs after delta_kernel and overwrites its value for those rows (scalar backward path; the MFMA path
// does the same inside its dQ head blocks).
template <typename T, int D>
__global__ __launch_bounds__(kWaves * 64) void delta_head_rows_kernel(cf_attn_bwd_params b, float *delta)
{
    const cf_attn_fwd_params &p = b.f;
    __shared__ float sq[kWaves][D], sdo[kWaves][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = blockIdx.x / (64 / kWaves);
    const int i = (blockIdx.x % (64 / kWaves)) * kWaves + wave;        // row inside the segment, 0..63
    const int h = blockIdx.y;
    const int q0 = p.cu_seqlens_q[g], lq = p.cu_seqlens_q[g + 1] - q0;
    const int k0 = p.cu_seqlens_k[g], lk = p.cu_seqlens_k[g + 1] - k0;
    const int n_vis = lk - lq + i + 1;
    if (i >= lq || n_vis > 64) return;   // whole wavefront leaves together; only wave-level barriers below
    const int row = q0 + i;
    const int kh = h / (p.n_q_heads / p.n_kv_heads);
    const T *q = (const T *)p.q + (int64_t)row * p.q_stride_tok + (int64_t)h * p.q_stride_head;
    const T *d_o = (const T *)b.d_o + (int64_t)row * b.do_stride_tok + (int64_t)h * b.do_stride_head;
    for (int t = 0; t < D / 64; ++t) {
        sq[wave][lane + 64 * t] = ld(q + lane + 64 * t);
        sdo[wave][lane + 64 * t] = ld(d_o + lane + 64 * t);
    }
    __builtin_amdgcn_wave_barrier();
    float s = 0.f;
    if (lane < n_vis) {
        const T *kj = (const T *)p.k + (int64_t)(k0 + lane) * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head;
        const T *vj = (const T *)p.v + (int64_t)(k0 + lane) * p.kv_stride_tok + (int64_t)kh * p.kv_stride_head;
        float sc = 0.f, dp = 0.f;
        for (int x = 0; x < D; ++x) {
            sc += sq[wave][x] * ld(kj + x);
            dp += sdo[wave][x] * ld(vj + x);
        }
        s = expf(sc * p.softmax_scale - p.lse[(int64_t)h * p.n_tokens + row]) * dp;
    }
    s = wave_sum(s);
    if (lane == 0) delta[(int64_t)h * p.n_tokens + row] = s;
}

template <typename T, int D>
hipError_t run_fwd(const cf_attn_fwd_params &p, hipStream_t s)
{
    dim3 grid((p.n_tokens + kWaves - 1) / kWaves, p.n_q_heads);
    const ProfileHook hook = take_profile_hook();
    if (hook.start) (void)hipEventRecord(hook.start, s);
    simple_fwd_kernel<T, D><<<grid, kWaves * 64, 0, s>>>(p);
    const hipError_t e = hipGetLastError();
    if (hook.stop) (void)hipEventRecord(hook.stop, s);
    return e;
}

template <typename T, int D>
hipError_t run_bwd(const cf_attn_bwd_params &b, const BwdWorkspace &ws, hipStream_t s)
{
    const cf_attn_fwd_params &p = b.f;
    // exact delta for rows that see at most 64 keys (overwrites delta_kernel's value for them)
    dim3 gh(p.n_segments * (64 / kWaves), p.n_q_heads);
    delta_head_rows_kernel<T, D><<<gh, kWaves * 64, 0, s>>>(b, ws.delta);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    dim3 gq((p.n_tokens + kWaves - 1) / kWaves, p.n_q_heads);
    const ProfileHook hook = take_profile_hook();
    if (hook.start) (void)hipEventRecord(hook.start, s);
    simple_dq_kernel<T, D><<<gq, kWaves * 64, 0, s>>>(b, ws.delta);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) {
        dim3 gk((p.n_kv_tokens + kWaves - 1) / kWaves, p.n_kv_heads);
        simple_dkv_kernel<T, D><<<gk, kWaves * 64, 0, s>>>(b, ws.delta);
        e = hipGetLastError();
    }
    if (hook.stop) (void)hipEventRecord(hook.stop, s);
    return e;
}

template <typename T, int D>
hipError_t run_delta(const cf_attn_bwd_params &b, const BwdWorkspace &ws, hipStream_t s)
{
    const int64_t pairs = (int64_t)b.f.n_tokens * b.f.n_q_heads;
    delta_kernel<T, D><<<dim3((unsigned)((pairs + 15) / 16)), 256, 0, s>>>(b, ws.delta);
    return hipGetLastError();
}

}  // namespace

#define CF_DISPATCH(fn, dtype, D, ...)                                              \
    do {                                                                            \
        if ((dtype) == CF_FP32 && (D) == 64) return fn<float, 64>(__VA_ARGS__);     \
        if ((dtype) == CF_FP32 && (D) == 128) return fn<float, 128>(__VA_ARGS__);   \
        if ((dtype) == CF_BF16 && (D) == 64) return fn<unsigned short, 64>(__VA_ARGS__);   \
        if ((dtype) == CF_BF16 && (D) == 128) return fn<unsigned short, 128>(__VA_ARGS__); \
        return hipErrorInvalidValue;                                                \
    } while (0)

hipError_t launch_simple_fwd(const cf_attn_fwd_params &p, hipStream_t s)
{
    CF_DISPATCH(run_fwd, p.dtype, p.head_dim, p, s);
}
hipError_t launch_simple_bwd(const cf_attn_bwd_params &b, const BwdWorkspace &ws, hipStream_t s)
{
    CF_DISPATCH(run_bwd, b.f.dtype, b.f.head_dim, b, ws, s);
}
hipError_t launch_delta(const cf_attn_bwd_params &b, const BwdWorkspace &ws, hipStream_t s)
{
    CF_DISPATCH(run_delta, b.f.dtype, b.f.head_dim, b, ws, s);
}

}  // namespace cf
