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

// One item of the packing: the whole short sequence `seq`, or (is_tail) the last, partial slice of a split one.
struct PackItem {
    int64_t seq, start;
    int32_t len;
    bool is_tail;
};

// One packing attempt: items in `order` (longest first) each go to the least-loaded bin, ties to the lowest bin
// index; a tail only goes to a bin that holds no tail yet (a chunk then depends on at most one split sequence).
// Fails as soon as an item does not fit its bin, or a tail finds no tail-free bin.
static bool try_pack(const std::vector<PackItem> &order, int64_t n_bins, int64_t cap,
                     std::vector<std::vector<int64_t>> &bins)
{
    using Entry = std::pair<int64_t, int64_t>;  // (load, bin): the smallest pair is the target bin
    std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
    std::vector<int64_t> load((size_t)n_bins, 0);
    std::vector<char> has_tail((size_t)n_bins, 0);
    for (int64_t b = 0; b < n_bins; ++b) heap.push({0, b});
    bins.assign((size_t)n_bins, {});
    for (size_t n = 0; n < order.size(); ++n) {
        const PackItem &it = order[n];
        int64_t b = -1;
        if (!it.is_tail) {
            while (heap.top().first != load[(size_t)heap.top().second]) heap.pop();   // entries a tail made stale
            b = heap.top().second;
            heap.pop();
        } else {
            for (int64_t x = 0; x < n_bins; ++x)
                if (!has_tail[(size_t)x] && (b < 0 || load[(size_t)x] < load[(size_t)b])) b = x;
            if (b < 0) return false;
            has_tail[(size_t)b] = 1;
        }
        if (load[(size_t)b] + it.len > cap) return false;
        load[(size_t)b] += it.len;
        bins[(size_t)b].push_back((int64_t)n);
        heap.push({load[(size_t)b], b});
    }
    return true;
}

extern "C" int cf_build_chunks_ex(const int64_t *seq_lens, int64_t n_seqs, int64_t chunk_size, uint32_t flags,
                                  cf_plan **out)
{
    if (!out) return cf::fail(CF_EINVAL, "cf_build_chunks: out is NULL");
    if (n_seqs < 0) return cf::fail(CF_EINVAL, "cf_build_chunks: n_seqs = %lld < 0", (long long)n_seqs);
    if (n_seqs > 0 && !seq_lens) return cf::fail(CF_EINVAL, "cf_build_chunks: seq_lens is NULL");
    if (chunk_size < 1 || chunk_size > INT32_MAX)
        return cf::fail(CF_EINVAL, "cf_build_chunks: chunk_size %lld outside [1, 2^31)", (long long)chunk_size);
    if (flags & ~(uint32_t)CF_PLAN_MERGE_TAILS)
        return cf::fail(CF_EINVAL, "cf_build_chunks_ex: unknown flags 0x%x", flags);
    for (int64_t i = 0; i < n_seqs; ++i)
        if (seq_lens[i] < 1)
            return cf::fail(CF_EINVAL, "cf_build_chunks: seq_lens[%lld] = %lld < 1", (long long)i,
                            (long long)seq_lens[i]);
    const bool merge_tails = flags & CF_PLAN_MERGE_TAILS;
    cf_plan *p = nullptr;
    try {
        p = new cf_plan();
        p->chunk_size = chunk_size;
        const int64_t C = chunk_size;
        std::vector<PackItem> items;     // what the packing places: short sequences and, if asked, tails
        std::vector<int32_t> tail_group((size_t)n_seqs, -1), tail_idx((size_t)n_seqs, 0);
        int64_t item_tokens = 0;
        for (int64_t i = 0; i < n_seqs; ++i) {
            p->total_tokens += seq_lens[i];
            if (seq_lens[i] <= C) {  // exactly chunk_size tokens: one full standalone chunk
                items.push_back({i, 0, (int32_t)seq_lens[i], false});
                item_tokens += seq_lens[i];
                continue;
            }
            const int32_t group = (int32_t)p->group_seq_id.size();
            int32_t m = 0;
            for (int64_t start = 0; start < seq_lens[i]; start += C, ++m) {
                const int32_t n = (int32_t)std::min(C, seq_lens[i] - start);
                if (merge_tails && n < C) {          // the partial last slice joins the packing instead
                    items.push_back({i, start, n, true});
                    item_tokens += n;
                    tail_group[(size_t)i] = group;
                    tail_idx[(size_t)i] = m;
                    break;
                }
                p->add_chunk(group, m, start, {i}, {start}, {n});
            }
            p->group_seq_id.push_back(i);
            p->group_chunk_ptr.push_back((int64_t)p->group_chunks.size());
        }
        if (!items.empty()) {
            std::vector<PackItem> order = items;     // items are in sequence order: a stable sort keeps it among equals
            std::stable_sort(order.begin(), order.end(),
                             [](const PackItem &a, const PackItem &b) { return a.len > b.len; });
            // Bin counts below ceil(tokens / C) cannot hold the tokens, so every attempt there fails:
            // starting at that count gives the same answer as starting at 1.
            std::vector<std::vector<int64_t>> bins;
            int64_t n_bins = std::max<int64_t>(1, (item_tokens + C - 1) / C);
            while (!try_pack(order, n_bins, C, bins)) ++n_bins;
            // A chunk that holds a tail is the last chunk of that sequence's group; it is inserted into the
            // group lists afterwards (group_chunks is laid out group by group).
            std::vector<std::vector<int64_t>> extra(p->group_seq_id.size());
            std::vector<int64_t> packed_chunks;
            for (auto &members : bins) {
                if (members.empty()) continue;
                std::sort(members.begin(), members.end(),
                          [&](int64_t a, int64_t b) { return order[(size_t)a].seq < order[(size_t)b].seq; });
                std::vector<int64_t> ids, starts;
                std::vector<int32_t> lens;
                int64_t prefix = 0;
                int32_t group = -1, idx = 0;
                for (int64_t n : members) {
                    const PackItem &it = order[(size_t)n];
                    ids.push_back(it.seq);
                    starts.push_back(it.start);
                    lens.push_back(it.len);
                    if (it.is_tail) {
                        prefix = it.start;
                        group = tail_group[(size_t)it.seq];
                        idx = tail_idx[(size_t)it.seq];
                    }
                }
                const int64_t chunk_id = (int64_t)p->chunk_tokens.size();
                p->add_chunk(group, idx, prefix, ids, starts, lens);
                p->group_chunks.pop_back();          // placed below, where its group's list is
                if (group >= 0) extra[(size_t)group].push_back(chunk_id);
                else packed_chunks.push_back(chunk_id);
            }
            // rebuild the group lists: split sequences (slices, then the chunk with their tail), then one group per
            // remaining packed chunk
            std::vector<int64_t> chunks_of, ptr{0};
            const size_t n_long = p->group_seq_id.size();
            for (size_t g = 0; g < n_long; ++g) {
                for (int64_t j = p->group_chunk_ptr[g]; j < p->group_chunk_ptr[g + 1]; ++j) chunks_of.push_back(p->group_chunks[(size_t)j]);
                for (int64_t c : extra[g]) chunks_of.push_back(c);
                ptr.push_back((int64_t)chunks_of.size());
            }
            for (int64_t c : packed_chunks) {
                p->chunk_group[(size_t)c] = (int32_t)p->group_seq_id.size();
                p->group_seq_id.push_back(-1);
                chunks_of.push_back(c);
                ptr.push_back((int64_t)chunks_of.size());
            }
            p->group_chunks = chunks_of;
            p->group_chunk_ptr = ptr;
        }
    } catch (const std::bad_alloc &) {
        delete p;
        return cf::fail(CF_ENOMEM, "cf_build_chunks: out of host memory");
    }
    *out = p;
    return CF_OK;
}

extern "C" int cf_build_chunks(const int64_t *seq_lens, int64_t n_seqs, int64_t chunk_size, cf_plan **out)
{
    return cf_build_chunks_ex(seq_lens, n_seqs, chunk_size, 0, out);
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
        int64_t len = 0;   // the split sequence's own tokens (a chunk with a merged tail also holds others)
        for (int64_t j = p->group_chunk_ptr[g]; j < p->group_chunk_ptr[g + 1]; ++j) {
            const int64_t c = p->group_chunks[j];
            for (int64_t s = p->chunk_seg_ptr[c]; s < p->chunk_seg_ptr[c + 1]; ++s)
                if (p->seg_seq_id[s] == p->group_seq_id[g]) len += p->seg_len[s];
        }
        if (len > st.state_tokens) st.state_tokens = len;
    }
    *out = st;
    return CF_OK;
}

// ---- pipeline bubble simulator (sections 3.3, 4.3, 5) ---------------------------------------------------------
namespace {

struct SimOp {
    bool backward;
    int64_t ticks;
    int32_t group;      // dependency group of the op's chunk (plain 1F1B: one group per micro-batch)
    bool keeps;         // a forward whose activations stay until the chunk's backward
};

// Order in which one stage runs the ops: forward-type ops in list order, backward ops in list order, a forward
// that keeps activations while fewer than `limit` chunks are held or while the next backward may not run yet,
// otherwise the next backward.  An op may run once the previous op of its group (prev[i], or -1) has run here.
bool stage_order(const std::vector<SimOp> &ops, const std::vector<int64_t> &prev, int64_t limit, std::vector<int64_t> &order)
{
    const int64_t n = (int64_t)ops.size();
    std::vector<char> ran((size_t)n, 0);
    order.clear();
    int64_t f = 0, b = 0, held = 0;
    auto next_of = [&](int64_t from, bool backward) {
        while (from < n && ops[(size_t)from].backward != backward) ++from;
        return from;
    };
    f = next_of(0, false);
    b = next_of(0, true);
    auto allowed = [&](int64_t i) { return i < n && (prev[(size_t)i] < 0 || ran[(size_t)prev[(size_t)i]]); };
    while (f < n || b < n) {
        const bool f_ok = allowed(f), b_ok = allowed(b);
        int64_t take;
        if (f_ok && (!ops[(size_t)f].keeps || held < limit || !b_ok)) {
            take = f;
            held += ops[(size_t)f].keeps;
            f = next_of(f + 1, false);
        } else if (b_ok) {
            take = b;
            --held;
            b = next_of(b + 1, true);
        } else {
            return false;
        }
        ran[(size_t)take] = 1;
        order.push_back(take);
    }
    return true;
}

// Earliest-start timeline of the per-stage orders: a forward-type op waits for the same op one stage up the
// pipeline, a backward op for the same op one stage down.  A stage is re-examined when a neighbour finishes an
// op (a queue of stages to look at; no repeated sweeps).
int simulate_pipeline(const std::vector<SimOp> &ops, int32_t n_stages, const char *who, cf_pipeline_stats *out)
{
    const int64_t n = (int64_t)ops.size();
    const int32_t p = n_stages;
    std::vector<int64_t> prev((size_t)n, -1);
    {
        std::vector<int64_t> last;
        for (int64_t i = 0; i < n; ++i) {
            const size_t g = (size_t)ops[(size_t)i].group;
            if (last.size() <= g) last.resize(g + 1, -1);
            prev[(size_t)i] = last[g];
            last[g] = i;
        }
    }
    std::vector<std::vector<int64_t>> order((size_t)p);
    for (int32_t s = 0; s < p; ++s)
        if (!stage_order(ops, prev, p - s, order[(size_t)s]))
            return cf::fail(CF_EINVAL, "%s: the schedule cannot be followed on stage %d", who, s);
    std::vector<std::vector<int64_t>> end((size_t)p, std::vector<int64_t>((size_t)n, -1));
    std::vector<int64_t> cursor((size_t)p, 0), free_at((size_t)p, 0);
    std::vector<int32_t> todo;
    std::vector<char> queued((size_t)p, 1);
    for (int32_t s = p - 1; s >= 0; --s) todo.push_back(s);     // popped from the back: stage 0 first
    int64_t done = 0, busy = 0;
    while (!todo.empty()) {
        const int32_t s = todo.back();
        todo.pop_back();
        queued[(size_t)s] = 0;
        bool progressed = false;
        while (cursor[(size_t)s] < n) {
            const int64_t i = order[(size_t)s][(size_t)cursor[(size_t)s]];
            const SimOp &op = ops[(size_t)i];
            const int32_t from = op.backward ? s + 1 : s - 1;
            int64_t ready = 0;
            if (from >= 0 && from < p) {
                ready = end[(size_t)from][(size_t)i];
                if (ready < 0) break;
            }
            const int64_t start = ready > free_at[(size_t)s] ? ready : free_at[(size_t)s];
            free_at[(size_t)s] = end[(size_t)s][(size_t)i] = start + op.ticks;
            if (s == 0) busy += op.ticks;
            ++cursor[(size_t)s];
            ++done;
            progressed = true;
        }
        if (progressed)
            for (int32_t nb : {s - 1, s + 1})
                if (nb >= 0 && nb < p && !queued[(size_t)nb] && cursor[(size_t)nb] < n) {
                    queued[(size_t)nb] = 1;
                    todo.push_back(nb);
                }
    }
    if (done != n * p) return cf::fail(CF_EINVAL, "%s: the stage orders deadlock", who);
    cf_pipeline_stats st = {};
    st.n_stages = p;
    st.n_ops = n;
    st.busy_per_stage = busy;
    for (int32_t s = 0; s < p; ++s)
        if (free_at[(size_t)s] > st.makespan) st.makespan = free_at[(size_t)s];
    st.total_ticks = (int64_t)p * st.makespan;
    st.bubble_ticks = st.total_ticks - (int64_t)p * busy;
    *out = st;
    return CF_OK;
}

}  // namespace

extern "C" int cf_sim_1f1b_sequences(const int64_t *seq_lens, int64_t n_seqs, int32_t n_stages, cf_pipeline_stats *out)
{
    const char *who = "cf_sim_1f1b_sequences";
    if (!out || n_seqs < 0 || (n_seqs > 0 && !seq_lens)) return cf::fail(CF_EINVAL, "%s: bad argument", who);
    if (n_stages < 1) return cf::fail(CF_EINVAL, "%s: n_stages = %d < 1", who, n_stages);
    try {
        // every micro-batch is a group of its own: forward (kept), then backward -- Algorithm 2 with N = 1
        std::vector<SimOp> ops;
        for (int64_t i = 0; i < n_seqs; ++i) {
            if (seq_lens[i] < 1 || seq_lens[i] > (INT64_MAX >> 24)) return cf::fail(CF_EINVAL, "%s: seq_lens[%lld] out of range", who, (long long)i);
            ops.push_back({false, seq_lens[i], (int32_t)i, true});
            ops.push_back({true, 2 * seq_lens[i], (int32_t)i, false});
        }
        return simulate_pipeline(ops, n_stages, who, out);
    } catch (const std::bad_alloc &) {
        return cf::fail(CF_ENOMEM, "%s: out of host memory", who);
    }
}

extern "C" int cf_sim_1f1b(cf_plan *p, int32_t K, int32_t n_stages, uint32_t flags, cf_pipeline_stats *out)
{
    const char *who = "cf_sim_1f1b";
    if (!p || !out) return cf::fail(CF_EINVAL, "%s: NULL argument", who);
    if (K < 1 || n_stages < 1) return cf::fail(CF_EINVAL, "%s: K = %d, n_stages = %d must be >= 1", who, K, n_stages);
    if (flags & ~(uint32_t)CF_SIM_PLAN_ORDER) return cf::fail(CF_EINVAL, "%s: unknown flags 0x%x", who, flags);
    try {
        const int64_t n_groups = (int64_t)p->group_seq_id.size();
        std::vector<int64_t> group_order;
        if (flags & CF_SIM_PLAN_ORDER) {
            for (int64_t g = 0; g < n_groups; ++g) group_order.push_back(g);
        } else {                                   // standalone chunks first, then the dependent groups
            for (int pass = 0; pass < 2; ++pass)
                for (int64_t g = 0; g < n_groups; ++g)
                    if ((p->group_seq_id[g] >= 0) == (pass == 1)) group_order.push_back(g);
        }
        std::vector<SimOp> ops;
        for (size_t n = 0; n < group_order.size(); ++n) {
            const int64_t g = group_order[n];
            const int64_t *c = p->group_chunks.data() + p->group_chunk_ptr[g];
            const int64_t N = p->group_chunk_ptr[g + 1] - p->group_chunk_ptr[g];
            const int64_t kept_from = N > K ? N - K : 0;
            auto fwd = [&](int64_t m, bool keep) { ops.push_back({false, (int64_t)p->chunk_tokens[c[m]], (int32_t)n, keep}); };
            auto bwd = [&](int64_t m) { ops.push_back({true, 2 * (int64_t)p->chunk_tokens[c[m]], (int32_t)n, false}); };
            for (int64_t m = 0; m < N; ++m) fwd(m, m >= kept_from);
            for (int64_t m = N - 1; m >= kept_from; --m) bwd(m);
            for (int64_t m = kept_from - 1; m >= 0; --m) {
                fwd(m, true);
                bwd(m);
            }
        }
        return simulate_pipeline(ops, n_stages, who, out);
    } catch (const std::bad_alloc &) {
        return cf::fail(CF_ENOMEM, "%s: out of host memory", who);
    }
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

extern "C" int64_t cf_attn_q_tiles(const int32_t *cu_q, const int32_t *cu_k, int32_t n_segments, cf_q_tile *out,
                                   int64_t capacity)
{
    if (!cu_q || !cu_k || n_segments < 1) return cf::fail(CF_EINVAL, "cf_attn_q_tiles: bad argument");
    constexpr int64_t kRows = 128, kKeysPerStep = 64;
    int64_t n_tiles = 0;
    for (int32_t g = 0; g < n_segments; ++g) {
        const int64_t lq = cu_q[g + 1] - cu_q[g], lk = cu_k[g + 1] - cu_k[g];
        if (lq < 1 || lk < lq) return cf::fail(CF_EINVAL, "cf_attn_q_tiles: segment %d has Lq=%lld Lk=%lld", g,
                                               (long long)lq, (long long)lk);
        n_tiles += (lq + kRows - 1) / kRows;
    }
    if (!out) return n_tiles;
    if (capacity < n_tiles) return cf::fail(CF_EINVAL, "cf_attn_q_tiles: capacity %lld < %lld tiles", (long long)capacity,
                                            (long long)n_tiles);
    try {
        std::vector<std::pair<int64_t, int64_t>> order;   // (-steps, index): ascending pairs = longest first, then list order
        order.reserve((size_t)n_tiles);
        int64_t n = 0;
        for (int32_t g = 0; g < n_segments; ++g) {
            const int64_t lq = cu_q[g + 1] - cu_q[g], lk = cu_k[g + 1] - cu_k[g];
            for (int64_t t = 0; t * kRows < lq; ++t, ++n) {
                const int64_t keys = std::min((t + 1) * kRows, lq) + (lk - lq);   // keys the tile's last row sees
                order.push_back({-((keys + kKeysPerStep - 1) / kKeysPerStep), n});
                out[n] = cf_q_tile{cu_q[g], (int32_t)lq, cu_k[g], (int32_t)lk, (int32_t)t, g, {0, 0}};
            }
        }
        std::sort(order.begin(), order.end());
        std::vector<cf_q_tile> sorted((size_t)n_tiles);
        for (int64_t i = 0; i < n_tiles; ++i) sorted[(size_t)i] = out[order[(size_t)i].second];
        std::copy(sorted.begin(), sorted.end(), out);
    } catch (const std::bad_alloc &) {
        return cf::fail(CF_ENOMEM, "cf_attn_q_tiles: out of host memory");
    }
    return n_tiles;
}

extern "C" const char *cf_last_error(void) { return cf::g_err; }
extern "C" int cf_version(void) { return 100; }
