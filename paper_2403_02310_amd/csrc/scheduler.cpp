// Stall-free batching, one iteration (paper Algorithm 3, section 4.2).  Host only.
//
// The batch is filled in three passes under a token budget: all running decodes, then the
// next chunk of each request whose prefill is under way, then waiting requests in arrival
// order while memory lasts.  Because the decodes are placed first and prefills only get the
// leftover budget, a co-running prefill can never push a decode out of an iteration.
//
// Readings of the listing: the admission loop appends the new request to the batch and moves
// on to the next waiting request after each admission (as Algorithm 2 does); chunk_size is a
// cap next to the token budget; a request may be admitted only if the pages of its whole
// prompt are free, and reserves them at once.
#include <algorithm>

#include "internal.h"

namespace {

// Largest chunk the leftover budget admits (section 4.2, the chunk-size computation of Algorithm 3).
inline int32_t next_chunk_size(const sarathi_request &r, int32_t chunk_size, int32_t token_budget, int64_t n_t) {
    if (n_t >= token_budget) return 0;
    int64_t left = (int64_t)r.prompt_len - r.num_prefilled;
    int64_t c = std::min<int64_t>({left, (int64_t)chunk_size, (int64_t)token_budget - n_t});
    return (int32_t)std::max<int64_t>(c, 0);
}

inline void push(sarathi_batch *b, int64_t id, int32_t q_len, int32_t ctx_len) {
    const int32_t i = b->num_seqs;
    b->seq_id[i] = id;
    b->q_start[i] = b->num_tokens;
    b->q_len[i] = q_len;
    b->ctx_len[i] = ctx_len;
    b->num_seqs = i + 1;
    b->num_tokens += q_len;
}

}  // namespace

extern "C" sarathi_status sarathi_build_stall_free_batch(
    int32_t token_budget, int32_t chunk_size,
    const sarathi_request *running_decodes, int32_t n_running_decodes,
    const sarathi_request *running_prefills, int32_t n_running_prefills,
    const sarathi_request *waiting_prefills, int32_t n_waiting,
    int64_t free_pages, int32_t page_size, int32_t max_batch_size, sarathi_batch *out) {
    if (!out || !out->seq_id || !out->q_start || !out->q_len || !out->ctx_len) return SARATHI_EINVAL;
    if (token_budget < 1 || chunk_size < 1 || page_size < 1 || max_batch_size < 1 || free_pages < 0) return SARATHI_EINVAL;
    if (n_running_decodes < 0 || n_running_prefills < 0 || n_waiting < 0) return SARATHI_EINVAL;
    if ((n_running_decodes && !running_decodes) || (n_running_prefills && !running_prefills) ||
        (n_waiting && !waiting_prefills))
        return SARATHI_EINVAL;
    out->num_seqs = out->num_tokens = out->num_decodes = out->num_prefill_chunks = out->num_admitted = 0;
    out->reserved = 0;
    out->free_pages_left = free_pages;
    if (n_running_decodes > max_batch_size) return SARATHI_ECAPACITY;

    // Pass 1: every running decode, one token each; the budget never drops one.
    for (int32_t i = 0; i < n_running_decodes; ++i) {
        const sarathi_request &r = running_decodes[i];
        if (r.prompt_len < 1 || r.num_prefilled != r.prompt_len || r.num_decoded < 0) return SARATHI_EINVAL;
        push(out, r.id, 1, r.prompt_len + r.num_decoded + 1);
    }
    out->num_decodes = out->num_seqs;
    int64_t n_t = out->num_tokens;

    // Pass 2: next chunk of each partially prefilled request.
    for (int32_t i = 0; i < n_running_prefills; ++i) {
        const sarathi_request &r = running_prefills[i];
        if (r.prompt_len < 1 || r.num_prefilled < 0 || r.num_prefilled >= r.prompt_len) return SARATHI_EINVAL;
        if (out->num_seqs >= max_batch_size) break;
        const int32_t c = next_chunk_size(r, chunk_size, token_budget, n_t);
        if (c > 0) {
            push(out, r.id, c, r.num_prefilled + c);
            n_t += c;
            out->num_prefill_chunks++;
        }
    }

    // Pass 3: admit waiting requests first come first served while pages and budget last.
    for (int32_t i = 0; i < n_waiting; ++i) {
        const sarathi_request &r = waiting_prefills[i];
        if (r.prompt_len < 1 || r.num_prefilled < 0 || r.num_prefilled >= r.prompt_len) return SARATHI_EINVAL;
        const int64_t pages = ((int64_t)r.prompt_len + page_size - 1) / page_size;
        const bool can_allocate = pages <= out->free_pages_left;
        if (!(can_allocate && n_t < token_budget && out->num_seqs < max_batch_size)) break;
        const int32_t c = next_chunk_size(r, chunk_size, token_budget, n_t);
        if (c <= 0) break;
        push(out, r.id, c, r.num_prefilled + c);
        n_t += c;
        out->free_pages_left -= pages;
        out->num_prefill_chunks++;
        out->num_admitted++;
    }
    return SARATHI_OK;
}
