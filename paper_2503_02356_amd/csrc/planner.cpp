// Host planner: chunk construction (paper Algorithm 1, section 4.1) and state-aware chunk
// scheduling (Algorithm 2, section 4.2).  Integer-only, no HIP.
#include <algorithm>
#include <climits>
#include <cstring>
#include <new>
#include <numeric>
#include <queue>
#include <utility>
#include <vector>

#include "common.h"

namespace cf {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace cf

struct cf_plan {
    int64_t chunk_size = 0, total_tokens = 0;
    std::vector<int64_t> chunk_seg_ptr{0};
    std::vector<int32_t> chunk_tokens;
    std::vector<int64_t> chunk_prefix_len;
    std::vector<int32_t> chunk_group, chunk_idx_in_group;
    std::vector<int64_t> seg_seq_id, seg_seq_start;
    std::vector<int32_t> seg_len;
    std::vector<int32_t> cu_seqlens;
    std::vector<int64_t> group_chunk_ptr{0}, group_chunks, group_seq_id;
    std::vector<cf_sched_op> sched;

    // Appends one chunk made of the given (sequence, start, length) segments to group `group`.
    void add_chunk(int32_t group, int32_t idx_in_group, int64_t prefix,
                   const std::vector<int64_t> &ids, const std::vector<int64_t> &starts,
                   const std::vector<int32_t> &lens)
    {
        int32_t tokens = 0;
        cu_seqlens.push_back(0);
        for (size_t s = 0; s < ids.size(); ++s) {
            seg_seq_id.push_back(ids[s]);
            seg_seq_start.push_back(starts[s]);
            seg_len.push_back(lens[s]);
            tokens += lens[s];
            cu_seqlens.push_back(tokens);
        }
        chunk_seg_ptr.push_back((int64_t)seg_len.size());
        chunk_tokens.push_back(tokens);
        chunk_prefix_len.push_back(prefix);
        chunk_group.push_back(group);
        chunk_idx_in_group.push_back(idx_in_group);
        group_chunks.push_back((int64_t)chunk_tokens.size() - 1);
    }
};

// One packing attempt: sequences in `order` (longest first) each go to the least-loaded bin, ties
// to the lowest bin index.  Fails as soon as a bin would exceed `cap`.
static bool try_pack(const std::vector<int64_t> &order, const int64_t *lens, int64_t n_bins,
                     int64_t cap, std::vector<std::vector<int64_t>> &bins)
{
    using Item = std::pair<int64_t, int64_t>;  // (load, bin): the smallest pair is the target bin
    std::priority_queue<Item, std::vector<Item>, std::greater<Item>> heap;
    for (int64_t b = 0; b < n_bins; ++b) heap.push({0, b});
    bins.assign((size_t)n_bins, {});
    for (int64_t i : order) {
        Item top = heap.top();
        heap.pop();
        if (top.first + lens[i] > cap) return false;
        top.first += lens[i];
        bins[(size_t)top.second].push_back(i);
        heap.push(top);
    }
    return true;
}

extern "C" int cf_build_chunks(const int64_t *seq_lens, int64_t n_seqs, int64_t chunk_size,
                               cf_plan **out)
{
    if (!out) return cf::fail(CF_EINVAL, "cf_build_chunks: out is NULL");
    if (n_seqs < 0) return cf::fail(CF_EINVAL, "cf_build_chunks: n_seqs = %lld < 0", (long long)n_seqs);
    if (n_seqs > 0 && !seq_lens) return cf::fail(CF_EINVAL, "cf_build_chunks: seq_lens is NULL");
    if (chunk_size < 1 || chunk_size > INT32_MAX)
        return cf::fail(CF_EINVAL, "cf_build_chunks: chunk_size %lld outside [1, 2^31)", (long long)chunk_size);
    for (int64_t i = 0; i < n_seqs; ++i)
        if (seq_lens[i] < 1)
            return cf::fail(CF_EINVAL, "cf_build_chunks: seq_lens[%lld] = %lld < 1", (long long)i,
                            (long long)seq_lens[i]);
    cf_plan *p = nullptr;
    try {
        p = new cf_plan();
        p->chunk_size = chunk_size;
        const int64_t C = chunk_size;
        std::vector<int64_t> shorts;
        int64_t short_tokens = 0;
        for (int64_t i = 0; i < n_seqs; ++i) {
            p->total_tokens += seq_lens[i];
            if (seq_lens[i] <= C) {  // exactly chunk_size tokens: one full standalone chunk
                shorts.push_back(i);
                short_tokens += seq_lens[i];
                continue;
            }
            const int32_t group = (int32_t)p->group_seq_id.size();
            int32_t m = 0;
            for (int64_t start = 0; start < seq_lens[i]; start += C, ++m)
                p->add_chunk(group, m, start, {i}, {start}, {(int32_t)std::min(C, seq_lens[i] - start)});
            p->group_seq_id.push_back(i);
            p->group_chunk_ptr.push_back((int64_t)p->group_chunks.size());
        }
        if (!shorts.empty()) {
            std::vector<int64_t> order = shorts;
            std::stable_sort(order.begin(), order.end(),
                             [&](int64_t a, int64_t b) { return seq_lens[a] > seq_lens[b]; });
            // Bin counts below ceil(tokens / C) cannot hold the tokens, so every attempt there fails:
            // starting at that count gives the same answer as starting at 1.
            std::vector<std::vector<int64_t>> bins;
            int64_t n_bins = std::max<int64_t>(1, (short_tokens + C - 1) / C);
            while (!try_pack(order, seq_lens, n_bins, C, bins)) ++n_bins;
            for (auto &members : bins) {
                if (members.empty()) continue;
                std::sort(members.begin(), members.end());
                std::vector<int64_t> starts(members.size(), 0);
                std::vector<int32_t> lens;
                for (int64_t i : members) lens.push_back((int32_t)seq_lens[i]);
                p->add_chunk((int32_t)p->group_seq_id.size(), 0, 0, members, starts, lens);
                p->group_seq_id.push_back(-1);
                p->group_chunk_ptr.push_back((int64_t)p->group_chunks.size());
            }
        }
    } catch (const std::bad_alloc &) {
        delete p;
        return cf::fail(CF_ENOMEM, "cf_build_chunks: out of host memory");
    }
    *out = p;
    return CF_OK;
}

extern "C" void cf_plan_free(cf_plan *plan) { delete plan; }

extern "C" int cf_plan_get(const cf_plan *p, cf_plan_view *v)
{
    if (!p || !v) return cf::fail(CF_EINVAL, "cf_plan_get: NULL argument");
    v->n_chunks = (int64_t)p->chunk_tokens.size();
    v->n_segments = (int64_t)p->seg_len.size();
    v->n_groups = (int64_t)p->group_seq_id.size();
    v->total_tokens = p->total_tokens;
    v->chunk_size = p->chunk_size;
    v->chunk_seg_ptr = p->chunk_seg_ptr.data();
    v->chunk_tokens = p->chunk_tokens.data();
    v->chunk_prefix_len = p->chunk_prefix_len.data();
    v->chunk_group = p->chunk_group.data();
    v->chunk_idx_in_group = p->chunk_idx_in_group.data();
    v->seg_seq_id = p->seg_seq_id.data();
    v->seg_seq_start = p->seg_seq_start.data();
    v->seg_len = p->seg_len.data();
    v->cu_seqlens = p->cu_seqlens.data();
    v->group_chunk_ptr = p->group_chunk_ptr.data();
    v->group_chunks = p->group_chunks.data();
    v->group_seq_id = p->group_seq_id.data();
    return CF_OK;
}

extern "C" int cf_build_schedule(cf_plan *p, int32_t K, const cf_sched_op **ops, int64_t *n_ops)
{
    if (!p || !ops || !n_ops) return cf::fail(CF_EINVAL, "cf_build_schedule: NULL argument");
    if (K < 1) return cf::fail(CF_EINVAL, "cf_build_schedule: K = %d < 1", K);
    try {
        p->sched.clear();
        const int64_t n_groups = (int64_t)p->group_seq_id.size();
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t *c = p->group_chunks.data() + p->group_chunk_ptr[g];
            const int64_t N = p->group_chunk_ptr[g + 1] - p->group_chunk_ptr[g];
            const int64_t kept_from = N > K ? N - K : 0;  // the LAST K chunks keep activations
            for (int64_t m = 0; m < N; ++m)
                p->sched.push_back({m >= kept_from ? CF_OP_FWD_KEEP : CF_OP_FWD_DISCARD, 0, c[m]});
            for (int64_t m = N - 1; m >= kept_from; --m) p->sched.push_back({CF_OP_BWD, 0, c[m]});
            for (int64_t m = kept_from - 1; m >= 0; --m) {  // descending: later gradients first
                p->sched.push_back({CF_OP_FWD_KEEP, 0, c[m]});
                p->sched.push_back({CF_OP_BWD, 0, c[m]});
            }
        }
    } catch (const std::bad_alloc &) {
        return cf::fail(CF_ENOMEM, "cf_build_schedule: out of host memory");
    }
    *ops = p->sched.data();
    *n_ops = (int64_t)p->sched.size();
    return CF_OK;
}

extern "C" int cf_schedule_stats(cf_plan *p, int32_t K, cf_sched_stats *out)
{
    if (!out) return cf::fail(CF_EINVAL, "cf_schedule_stats: NULL out");
    const cf_sched_op *ops = nullptr;
    int64_t n_ops = 0;
    if (int rc = cf_build_schedule(p, K, &ops, &n_ops)) return rc;
    cf_sched_stats st = {};
    int64_t kept_chunks = 0, kept_tokens = 0;
    for (int64_t i = 0; i < n_ops; ++i) {
        const int64_t tokens = p->chunk_tokens[ops[i].chunk];
        if (ops[i].op == CF_OP_BWD) {
            ++st.n_backward;
            --kept_chunks;
            kept_tokens -= tokens;
        } else {
            ++st.n_forward;
            if (ops[i].op == CF_OP_FWD_KEEP) {
                ++kept_chunks;
                kept_tokens += tokens;
                if (kept_chunks > st.peak_kept_chunks) st.peak_kept_chunks = kept_chunks;
                if (kept_tokens > st.peak_kept_tokens) st.peak_kept_tokens = kept_tokens;
            }
        }
    }
    st.n_reforward = st.n_forward - (int64_t)p->chunk_tokens.size();
    const int64_t n_groups = (int64_t)p->group_seq_id.size();
    for (int64_t g = 0; g < n_groups; ++g) {
        if (p->group_seq_id[g] < 0) continue;          // packed chunk: no state
        int64_t len = 0;
        for (int64_t j = p->group_chunk_ptr[g]; j < p->group_chunk_ptr[g + 1]; ++j) len += p->chunk_tokens[p->group_chunks[j]];
        if (len > st.state_tokens) st.state_tokens = len;
    }
    *out = st;
    return CF_OK;
}

extern "C" int64_t cf_count_pairs(const int32_t *cu_q, const int32_t *cu_k, int32_t n_segments)
{
    if (!cu_q || !cu_k || n_segments < 0) return cf::fail(CF_EINVAL, "cf_count_pairs: bad argument");
    int64_t pairs = 0;
    for (int32_t g = 0; g < n_segments; ++g) {
        const int64_t lq = cu_q[g + 1] - cu_q[g], lk = cu_k[g + 1] - cu_k[g];
        if (lq < 0 || lk < lq) return cf::fail(CF_EINVAL, "cf_count_pairs: segment %d has Lq=%lld Lk=%lld", g,
                                               (long long)lq, (long long)lk);
        pairs += lq * (lk - lq) + lq * (lq + 1) / 2;
    }
    return pairs;
}

extern "C" const char *cf_last_error(void) { return cf::g_err; }
extern "C" int cf_version(void) { return 100; }
