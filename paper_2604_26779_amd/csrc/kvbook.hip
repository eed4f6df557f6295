// Device-side KV bookkeeping: page reservation before the forward pass and the commit after
// sampling.  Both run as one workgroup so that the order in which pages leave and re-enter the
// free stack is a pure function of the batch order (a block-wide exclusive scan gives every
// batch entry its place on the stack).
#include "common.h"

namespace specv {

constexpr int KVB_THREADS = 256;

__device__ inline int block_exclusive_scan(int v, int* lds, int* total)
{
    int t = threadIdx.x;
    lds[t] = v;
    __syncthreads();
    for (int off = 1; off < KVB_THREADS; off <<= 1) {
        int add = (t >= off) ? lds[t - off] : 0;
        __syncthreads();
        lds[t] += add;
        __syncthreads();
    }
    int incl = lds[t];
    *total = lds[KVB_THREADS - 1];
    __syncthreads();
    return incl - v;
}

// error bits
constexpr int KV_ERR_NOMEM = 1, KV_ERR_SEQ = 2, KV_ERR_LEN = 4;

// Batch entries as the kernels may use them: clean[b] = seq_ids[b] if that id is inside [0, max_seqs) and no earlier
// batch entry names it, else -1 (flagged with KV_ERR_SEQ): an entry that would index the bookkeeping out of bounds,
// or write the same cache slots as another, is dropped from the step instead.  owner[max_seqs] is scratch that holds
// INT_MAX between calls.  One workgroup; ends with a barrier.
__device__ inline void sanitise_ids(int B, const int32_t* __restrict__ seq_ids, int max_seqs, int32_t* __restrict__ owner,
                                    int32_t* __restrict__ clean, int32_t* __restrict__ error)
{
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const int seq = seq_ids[b];
        if (seq >= 0 && seq < max_seqs) atomicMin(&owner[seq], b);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const int seq = seq_ids[b];
        const bool ok = seq >= 0 && seq < max_seqs && __hip_atomic_load(&owner[seq], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == b;
        clean[b] = ok ? seq : -1;
        if (!ok) atomicOr(error, KV_ERR_SEQ);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const int seq = seq_ids[b];
        if (seq >= 0 && seq < max_seqs) __hip_atomic_store(&owner[seq], 0x7fffffff, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
}

__global__ __launch_bounds__(KVB_THREADS) void kv_reserve_kernel(
    int B, int k, const int32_t* __restrict__ seq_ids, int max_seqs, int max_pages,
    const int32_t* __restrict__ ctx_len, int32_t* __restrict__ n_held, int32_t* __restrict__ page_table,
    const int32_t* __restrict__ free_stack, int32_t* __restrict__ free_count, int32_t* __restrict__ error,
    int32_t* __restrict__ owner, int32_t* __restrict__ entry_seq, int32_t* __restrict__ starved)
{
    __shared__ int lds[KVB_THREADS];
    __shared__ int s_free;
    if (threadIdx.x == 0) s_free = *free_count;
    sanitise_ids(B, seq_ids, max_seqs, owner, entry_seq, error);     // entry_seq: what the forward pass's kernels index by
    for (int base = 0; base < B; base += KVB_THREADS) {
        int b = base + threadIdx.x;
        int seq = -1, held = 0, want = 0;
        if (b < B) seq = entry_seq[b];
        if (seq >= 0) {
            held = n_held[seq];
            int need = (ctx_len[seq] + k + 1 + SPEC_PAGE_SIZE - 1) / SPEC_PAGE_SIZE;
            if (need > max_pages) { atomicOr(error, KV_ERR_LEN); need = held; }
            want = need > held ? need - held : 0;
        }
        int total;
        int off = block_exclusive_scan(want, lds, &total);
        int avail = s_free;
        __syncthreads();
        if (total > avail) {
            // not enough pages for this group of entries: nobody grows, the step is flagged.  An entry that needed a page is
            // left out of the step like one with a bad id - its rows are not computed, nothing of it is written to the cache
            // - and its sequence is marked, so that the commit leaves it as it is and reports -1 for it.
            if (threadIdx.x == 0) atomicOr(error, KV_ERR_NOMEM);
            if (seq >= 0) {
                starved[seq] = want > 0 ? 1 : 0;
                if (want > 0) entry_seq[b] = -1;
            }
        } else {
            for (int j = 0; j < want; ++j)
                page_table[(int64_t)seq * max_pages + held + j] = free_stack[avail - 1 - off - j];
            if (want > 0) n_held[seq] = held + want;
            if (seq >= 0) starved[seq] = 0;
            if (threadIdx.x == 0) s_free = avail - total;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) *free_count = s_free;
}

__global__ __launch_bounds__(KVB_THREADS) void kv_commit_kernel(
    int B, int k, const int32_t* __restrict__ seq_ids, const int32_t* __restrict__ accept_len, int max_seqs,
    int max_pages, int32_t* __restrict__ ctx_len, int32_t* __restrict__ n_held,
    int32_t* __restrict__ page_table, int32_t* __restrict__ free_stack, int32_t* __restrict__ free_count,
    int32_t* __restrict__ error, int32_t* __restrict__ new_ctx_len, int32_t* __restrict__ commit_slots,
    int32_t* __restrict__ owner, int32_t* __restrict__ clean, int32_t* __restrict__ starved)
{
    __shared__ int lds[KVB_THREADS];
    __shared__ int s_free;
    if (threadIdx.x == 0) s_free = *free_count;
    sanitise_ids(B, seq_ids, max_seqs, owner, clean, error);
    for (int base = 0; base < B; base += KVB_THREADS) {
        int b = base + threadIdx.x;
        int seq = -1, held = 0, keep = 0, release = 0;
        if (b < B) seq = clean[b];
        if (seq >= 0 && starved[seq]) {                  // its step found no page: nothing was computed for it, nothing is kept
            starved[seq] = 0;
            seq = -1;
        }
        if (seq >= 0) {
            held = n_held[seq];
            int ctx = ctx_len[seq];
            int n = accept_len[b];
            n = n < 0 ? 0 : (n > k ? k : n);
            int fresh = ctx + n + 1;
            int cap = held * SPEC_PAGE_SIZE;           // a step that could not reserve keeps what fits
            if (fresh > cap) fresh = cap > ctx ? cap : ctx;
            for (int i = 0; i <= k; ++i) {
                int pos = ctx + i;
                int slot = -1;
                if (pos < fresh)
                    slot = page_table[(int64_t)seq * max_pages + pos / SPEC_PAGE_SIZE] * SPEC_PAGE_SIZE +
                           pos % SPEC_PAGE_SIZE;
                if (commit_slots) commit_slots[(int64_t)b * (k + 1) + i] = slot;
            }
            keep = (fresh + SPEC_PAGE_SIZE - 1) / SPEC_PAGE_SIZE;
            release = held > keep ? held - keep : 0;
            ctx_len[seq] = fresh;
            if (new_ctx_len) new_ctx_len[b] = fresh;
        } else if (b < B) {
            if (new_ctx_len) new_ctx_len[b] = -1;
            if (commit_slots)
                for (int i = 0; i <= k; ++i) commit_slots[(int64_t)b * (k + 1) + i] = -1;
        }
        int total;
        int off = block_exclusive_scan(release, lds, &total);
        int top = s_free;
        __syncthreads();
        for (int j = 0; j < release; ++j) {             // last logical page first
            int64_t at = (int64_t)seq * max_pages + held - 1 - j;
            free_stack[top + off + j] = page_table[at];
            page_table[at] = -1;
        }
        if (release > 0) n_held[seq] = keep;
        if (threadIdx.x == 0) s_free = top + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) *free_count = s_free;
}

// Roll sequences back to min(current, len[b] + delta) cached positions; pages wholly beyond return to
// the free stack in the same order the commit uses (batch order, a sequence's last page first).
__global__ __launch_bounds__(KVB_THREADS) void kv_truncate_kernel(
    int B, const int32_t* __restrict__ seq_ids, const int32_t* __restrict__ len, int delta, int max_seqs, int max_pages,
    int32_t* __restrict__ ctx_len, int32_t* __restrict__ n_held, int32_t* __restrict__ page_table,
    int32_t* __restrict__ free_stack, int32_t* __restrict__ free_count, int32_t* __restrict__ error,
    int32_t* __restrict__ new_len, int32_t* __restrict__ owner, int32_t* __restrict__ clean)
{
    __shared__ int lds[KVB_THREADS];
    __shared__ int s_free;
    if (threadIdx.x == 0) s_free = *free_count;
    sanitise_ids(B, seq_ids, max_seqs, owner, clean, error);
    for (int base = 0; base < B; base += KVB_THREADS) {
        int b = base + threadIdx.x;
        int seq = -1, held = 0, keep = 0, release = 0;
        if (b < B) seq = clean[b];
        if (seq >= 0) {
            held = n_held[seq];
            int ctx = ctx_len[seq];
            int want = len[b] + delta;
            if (want < 0) { atomicOr(error, KV_ERR_LEN); want = 0; }
            int fresh = want < ctx ? want : ctx;
            keep = (fresh + SPEC_PAGE_SIZE - 1) / SPEC_PAGE_SIZE;
            release = held > keep ? held - keep : 0;
            ctx_len[seq] = fresh;
            if (new_len) new_len[b] = fresh;
        } else if (b < B) {
            if (new_len) new_len[b] = -1;
        }
        int total;
        int off = block_exclusive_scan(release, lds, &total);
        int top = s_free;
        __syncthreads();
        for (int j = 0; j < release; ++j) {
            int64_t at = (int64_t)seq * max_pages + held - 1 - j;
            free_stack[top + off + j] = page_table[at];
            page_table[at] = -1;
        }
        if (release > 0) n_held[seq] = keep;
        if (threadIdx.x == 0) s_free = top + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) *free_count = s_free;
}

// Slot bookkeeping of a continuous rollout: finished sequences leave their slot, waiting ones take it over in
// batch order (a block scan over "this slot needs a successor" hands out the queue entries), the rest idle.
__global__ __launch_bounds__(KVB_THREADS) void rollout_retire_kernel(
    int B, int k, int n_seqs, int32_t* __restrict__ slot_seq, int32_t* __restrict__ active,
    const int32_t* __restrict__ accept_len, int32_t* __restrict__ gen_len, const int32_t* __restrict__ target_len,
    const int32_t* __restrict__ queue, int queue_len, int32_t* __restrict__ queue_head,
    const int32_t* __restrict__ first_token, int32_t* __restrict__ tokens, int32_t* __restrict__ release_seq,
    int32_t* __restrict__ keep_len, long long* __restrict__ produced)
{
    __shared__ int lds[KVB_THREADS];
    __shared__ int s_head;
    if (threadIdx.x == 0) s_head = *queue_head;
    __syncthreads();
    long long made_sum = 0;
    for (int base = 0; base < B; base += KVB_THREADS) {
        const int b = base + threadIdx.x;
        int wants = 0, made = 0;
        if (b < B) {
            const int s = slot_seq[b];
            release_seq[b] = s;
            const bool live = active[b] != 0 && s >= 0 && s < n_seqs;
            if (!live) {
                keep_len[b] = 0;
            } else {
                int n = accept_len[b];
                n = n < 0 ? 0 : (n > k ? k : n);
                const int left = target_len[s] - gen_len[s];
                made = n + 1 < left ? n + 1 : left;
                if (made < 0) made = 0;
                gen_len[s] += made;
                if (made >= left) { wants = 1; keep_len[b] = 0; }
                else keep_len[b] = 1 << 30;
            }
        }
        int total;
        const int rank = block_exclusive_scan(wants, lds, &total);
        const int head = s_head;
        __syncthreads();
        if (wants) {
            if (head + rank < queue_len) {
                const int nxt = queue[head + rank];
                slot_seq[b] = nxt;
                tokens[(int64_t)b * (k + 1)] = nxt >= 0 && nxt < n_seqs ? first_token[nxt] : 0;
            } else {
                active[b] = 0;
            }
        }
        if (threadIdx.x == 0) s_head = head + total < queue_len ? head + total : queue_len;
        made_sum += made;
        __syncthreads();
    }
    // tokens counted this step, summed over the block
    int total;
    block_exclusive_scan((int)made_sum, lds, &total);
    if (threadIdx.x == 0) { *queue_head = s_head; *produced += total; }
}

spec_status launch_rollout_retire(int B, int k, int n_seqs, int32_t* slot_seq, int32_t* active, const int32_t* accept_len,
                                  int32_t* gen_len, const int32_t* target_len, const int32_t* queue, int queue_len,
                                  int32_t* queue_head, const int32_t* first_token, int32_t* tokens, int32_t* release_seq,
                                  int32_t* keep_len, int64_t* produced, hipStream_t s)
{
    rollout_retire_kernel<<<1, KVB_THREADS, 0, s>>>(B, k, n_seqs, slot_seq, active, accept_len, gen_len, target_len, queue,
                                                    queue_len, queue_head, first_token, tokens, release_seq, keep_len,
                                                    (long long*)produced);
    SPEC_LAUNCH_CHECK("rollout_retire_kernel");
    return SPEC_OK;
}

// Stable partition of the slots by liveness.  One workgroup; pass 1 copies everything to scratch and scans the
// flags, pass 2 writes the rows back at their new places.
__global__ __launch_bounds__(KVB_THREADS) void rollout_compact_kernel(int B, int k, int32_t* __restrict__ slot_seq,
                                                                      int32_t* __restrict__ active, int32_t* __restrict__ tokens,
                                                                      int32_t* __restrict__ n_live, int32_t* __restrict__ scratch)
{
    __shared__ int lds[KVB_THREADS];
    __shared__ int s_live_total;
    const int T = k + 1;
    int32_t* sc_seq = scratch;                 // [B]
    int32_t* sc_dst = scratch + B;             // [B] new index of old slot b
    int32_t* sc_tok = scratch + 2 * B;         // [B, T]
    // number of live slots first (the idle ones start behind them)
    int count = 0;
    for (int b = threadIdx.x; b < B; b += KVB_THREADS) count += active[b] != 0;
    int total;
    block_exclusive_scan(count, lds, &total);
    if (threadIdx.x == 0) s_live_total = total;
    __syncthreads();
    const int live_total = s_live_total;
    int live_before = 0;                       // live slots in the groups already handled
    for (int base = 0; base < B; base += KVB_THREADS) {
        const int b = base + threadIdx.x;
        const int is_live = b < B && active[b] != 0;
        int group_live;
        const int rank = block_exclusive_scan(is_live, lds, &group_live);
        if (b < B) {
            // live slot: its rank among the live ones; idle slot: behind all live ones, in order
            const int dst = is_live ? live_before + rank : live_total + (b - (live_before + rank));
            sc_dst[b] = dst;
            sc_seq[b] = slot_seq[b];
            for (int i = 0; i < T; ++i) sc_tok[(int64_t)b * T + i] = tokens[(int64_t)b * T + i];
        }
        live_before += group_live;
        __syncthreads();
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += KVB_THREADS) {
        const int dst = sc_dst[b];
        slot_seq[dst] = sc_seq[b];
        active[dst] = dst < live_total ? 1 : 0;
        for (int i = 0; i < T; ++i) tokens[(int64_t)dst * T + i] = sc_tok[(int64_t)b * T + i];
    }
    if (threadIdx.x == 0) *n_live = live_total;
}

spec_status launch_rollout_compact(int B, int k, int32_t* slot_seq, int32_t* active, int32_t* tokens, int32_t* n_live,
                                   int32_t* scratch, hipStream_t s)
{
    rollout_compact_kernel<<<1, KVB_THREADS, 0, s>>>(B, k, slot_seq, active, tokens, n_live, scratch);
    SPEC_LAUNCH_CHECK("rollout_compact_kernel");
    return SPEC_OK;
}

// pending[b] = (prev_token[s], first_token[s]) for the live slots whose sequence s changed in the retire step
__global__ void rollout_pending_kernel(int B, int n_seqs, const int32_t* __restrict__ slot_seq_before, const int32_t* __restrict__ slot_seq,
                                       const int32_t* __restrict__ active, const int32_t* __restrict__ prev_token,
                                       const int32_t* __restrict__ first_token, int32_t* __restrict__ pending)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int s = slot_seq[b];
    if (!active[b] || s == slot_seq_before[b] || s < 0 || s >= n_seqs) return;
    pending[2 * b] = prev_token[s];
    pending[2 * b + 1] = first_token[s];
}

// pending_hidden[b] = seq_hidden[s] (two rows of d floats) for the live slots whose sequence s changed in the retire step
__global__ void rollout_pending_hidden_kernel(int B, int n_seqs, int d, const int32_t* __restrict__ slot_seq_before,
                                              const int32_t* __restrict__ slot_seq, const int32_t* __restrict__ active,
                                              const float* __restrict__ seq_hidden, float* __restrict__ pending_hidden)
{
    const int b = blockIdx.x;
    const int s = slot_seq[b];
    if (!active[b] || s == slot_seq_before[b] || s < 0 || s >= n_seqs) return;
    const float* src = seq_hidden + (int64_t)s * 2 * d;
    float* dst = pending_hidden + (int64_t)b * 2 * d;
    for (int i = threadIdx.x; i < 2 * d; i += blockDim.x) dst[i] = src[i];
}

spec_status launch_rollout_pending_hidden(int B, int n_seqs, int d, const int32_t* slot_seq_before, const int32_t* slot_seq,
                                          const int32_t* active, const float* seq_hidden, float* pending_hidden, hipStream_t s)
{
    rollout_pending_hidden_kernel<<<(unsigned)B, 256, 0, s>>>(B, n_seqs, d, slot_seq_before, slot_seq, active, seq_hidden, pending_hidden);
    SPEC_LAUNCH_CHECK("rollout_pending_hidden_kernel");
    return SPEC_OK;
}

spec_status launch_rollout_pending(int B, int n_seqs, const int32_t* slot_seq_before, const int32_t* slot_seq, const int32_t* active,
                                   const int32_t* prev_token, const int32_t* first_token, int32_t* pending, hipStream_t s)
{
    rollout_pending_kernel<<<(unsigned)cdiv(B, 256), 256, 0, s>>>(B, n_seqs, slot_seq_before, slot_seq, active, prev_token, first_token, pending);
    SPEC_LAUNCH_CHECK("rollout_pending_kernel");
    return SPEC_OK;
}

spec_status launch_kv_truncate(spec_kv* kv, int B, const int32_t* dev_seq_ids, const int32_t* dev_len, int delta,
                               int32_t* dev_new_len, hipStream_t s)
{
    kv_truncate_kernel<<<1, KVB_THREADS, 0, s>>>(B, dev_seq_ids, dev_len, delta, kv->max_seqs, kv->max_pages, kv->d_ctx_len,
                                                 kv->d_n_held, kv->d_page_table, kv->d_free_stack, kv->d_free_count,
                                                 kv->d_error, dev_new_len, kv->d_owner, kv->d_entry_tmp);
    SPEC_LAUNCH_CHECK("kv_truncate_kernel");
    return SPEC_OK;
}

spec_status launch_kv_reserve(spec_kv* kv, int B, int k, const int32_t* dev_seq_ids, hipStream_t s)
{
    kv_reserve_kernel<<<1, KVB_THREADS, 0, s>>>(B, k, dev_seq_ids, kv->max_seqs, kv->max_pages, kv->d_ctx_len,
                                                kv->d_n_held, kv->d_page_table, kv->d_free_stack,
                                                kv->d_free_count, kv->d_error, kv->d_owner, kv->d_entry_seq, kv->d_starved);
    SPEC_LAUNCH_CHECK("kv_reserve_kernel");
    return SPEC_OK;
}

spec_status launch_kv_commit(spec_kv* kv, int B, int k, const int32_t* dev_seq_ids, const int32_t* dev_accept_len,
                             int32_t* dev_new_ctx_len, int32_t* dev_commit_slots, hipStream_t s)
{
    kv_commit_kernel<<<1, KVB_THREADS, 0, s>>>(B, k, dev_seq_ids, dev_accept_len, kv->max_seqs, kv->max_pages,
                                               kv->d_ctx_len, kv->d_n_held, kv->d_page_table, kv->d_free_stack,
                                               kv->d_free_count, kv->d_error, dev_new_ctx_len, dev_commit_slots, kv->d_owner,
                                               kv->d_entry_tmp, kv->d_starved);
    SPEC_LAUNCH_CHECK("kv_commit_kernel");
    return SPEC_OK;
}

}  // namespace specv
