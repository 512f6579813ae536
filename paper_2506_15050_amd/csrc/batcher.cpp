// tppo_batcher_*: slot bookkeeping of successive batching (Sec. 3.2, Alg. 1
// line 2).  Host code only, integers only: a constant number of slots; a
// sequence that has ended (end-of-sequence token, or response at the maximum
// length) is replaced by a new prompt before the next step, the others stay and
// their previous window becomes context.  The layout it exports is the input of
// tppo_select, once for the policy tokens (context = everything before the
// current window) and once for the value tokens (context = the prompt only,
// tail_drop = INT32_MAX: exactly the whole responses of finished sequences).
#include <stdint.h>

#include <new>
#include <vector>

#include "tppo.h"

struct tppo_batcher {
    struct Slot {
        int64_t id;
        int32_t prompt, ctx, win;
        bool used, done;
    };
    std::vector<Slot> slots;
    int32_t window, max_response;
    int64_t next_id;
};

extern "C" tppo_batcher* tppo_batcher_create(int64_t slots, int32_t window, int32_t max_response) {
    if (slots <= 0 || slots > (1 << 24) || window <= 0 || max_response < window) return nullptr;
    tppo_batcher* b = new (std::nothrow) tppo_batcher;
    if (!b) return nullptr;
    b->slots.assign((size_t)slots, tppo_batcher::Slot{0, 0, 0, 0, false, false});
    b->window = window;
    b->max_response = max_response;
    b->next_id = 0;
    return b;
}

extern "C" void tppo_batcher_destroy(tppo_batcher* b) { delete b; }

extern "C" int tppo_batcher_refill(tppo_batcher* b, const int32_t* prompt_len, int64_t n_available, int64_t* n_taken) {
    if (!b || (n_available > 0 && !prompt_len)) return TPPO_ERR_NULL;
    if (n_available < 0) return TPPO_ERR_SIZE;
    int64_t free_slots = 0;
    for (const auto& s : b->slots) free_slots += (!s.used || s.done) ? 1 : 0;
    const int64_t to_take = free_slots < n_available ? free_slots : n_available;
    for (int64_t i = 0; i < to_take; ++i)
        if (prompt_len[i] < 1) return TPPO_ERR_PARAM;                // a state needs at least one token; nothing changed
    int64_t taken = 0;
    for (auto& s : b->slots) {
        if ((!s.used || s.done) && taken < to_take) {
            const int32_t p = prompt_len[taken];
            s = tppo_batcher::Slot{b->next_id++, p, p, 0, true, false};
            ++taken;
        }
    }
    if (n_taken) *n_taken = taken;
    return TPPO_OK;
}

extern "C" int tppo_batcher_advance(tppo_batcher* b, const int32_t* gen_len, const int32_t* eos) {
    if (!b || !gen_len || !eos) return TPPO_ERR_NULL;
    // validate everything first: a rejected call changes nothing
    for (size_t k = 0; k < b->slots.size(); ++k) {
        const auto& s = b->slots[k];
        if (!s.used || s.done) return TPPO_ERR_PARAM;                // refill first
        const int64_t so_far = (int64_t)s.ctx + s.win - s.prompt, g = gen_len[k];
        if (g < 0 || g > b->window || so_far + g > b->max_response) return TPPO_ERR_SIZE;
        if (!eos[k] && g < b->window && so_far + g < b->max_response) return TPPO_ERR_PARAM;
        if ((int64_t)s.ctx + s.win + g > INT32_MAX) return TPPO_ERR_SIZE;
    }
    for (size_t k = 0; k < b->slots.size(); ++k) {
        auto& s = b->slots[k];
        const int32_t so_far = s.ctx + s.win - s.prompt;
        s.ctx += s.win;
        s.win = gen_len[k];
        s.done = eos[k] != 0 || so_far + gen_len[k] == b->max_response;
    }
    return TPPO_OK;
}

extern "C" int tppo_batcher_layout(const tppo_batcher* b, int32_t* cu_seqlens, int32_t* ctx_len, int32_t* prompt_len,
                                   int32_t* done, int64_t* seq_id) {
    if (!b || !cu_seqlens || !ctx_len || !prompt_len || !done) return TPPO_ERR_NULL;
    int64_t total = 0;
    cu_seqlens[0] = 0;
    for (size_t k = 0; k < b->slots.size(); ++k) {
        const auto& s = b->slots[k];
        if (!s.used) return TPPO_ERR_PARAM;
        total += (int64_t)s.ctx + s.win;
        if (total > INT32_MAX) return TPPO_ERR_SIZE;
        cu_seqlens[k + 1] = (int32_t)total;
        ctx_len[k] = s.ctx;
        prompt_len[k] = s.prompt;
        done[k] = s.done ? 1 : 0;
        if (seq_id) seq_id[k] = s.id;
    }
    return TPPO_OK;
}
