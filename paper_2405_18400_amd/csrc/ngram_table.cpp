// Host-side construction of the device n-gram store: one exact-key open-addressing table
// holding every n-gram's count (the frequency tables of Section 4: one entry per distinct n-gram)
// plus, per distinct context, the sum of the counts of its continuations -- the denominator of
// p_{n-gram}(x | context) = count(context, x) / sum_x' count(context, x').
#include "spd_internal.h"

#include <cstring>

uint64_t ngram_capacity_for(const spd_ngram_host_tables *t) {
    uint64_t n = 0;
    for (int o = 0; o < SPD_N_ORDERS; ++o) n += (uint64_t)(t->n_entries[o] > 0 ? t->n_entries[o] : 0);
    // every entry may add one context-total entry; keep the load factor <= 0.7
    uint64_t cap = (uint64_t)((double)(2 * n) / 0.7) + 64;
    return cap;
}

namespace {
struct Builder {
    NgramHostTable &tab;
    uint64_t cap;
    // Finds the slot of `key`, or the empty slot where it belongs.
    NgramSlot *locate(const int32_t *key, bool &found) {
        uint64_t at = ngram_home(ngram_hash(key), cap);
        for (int32_t p = 0;; ++p, at = (at + 1 == cap) ? 0 : at + 1) {
            NgramSlot &s = tab.slots[at];
            if (s.tok[0] == NG_EMPTY) {
                found = false;
                if (p > tab.max_probe) tab.max_probe = p;
                return &s;
            }
            if (std::memcmp(s.tok, key, sizeof(s.tok)) == 0) {
                found = true;
                return &s;
            }
        }
    }
};
}  // namespace

int ngram_build(const spd_ngram_host_tables *t, int32_t vocab, uint64_t capacity, NgramHostTable &out,
                std::string &err) {
    NgramSlot empty;
    for (int q = 0; q < 6; ++q) empty.tok[q] = NG_PAD;
    empty.tok[0] = NG_EMPTY;
    empty.cnt_lo = empty.cnt_hi = 0;
    out.slots.assign(capacity, empty);
    out.max_probe = 0;
    Builder b{out, capacity};
    for (int o = 0; o < SPD_N_ORDERS; ++o) {
        const int n = o + SPD_MIN_ORDER;
        const int64_t N = t->n_entries[o];
        out.present[o] = N > 0;
        if (N < 0) { err = "negative entry count"; return SPD_EINVAL; }
        if (N > 0 && (!t->keys[o] || !t->counts[o])) { err = "null keys/counts for a non-empty order"; return SPD_EINVAL; }
        for (int64_t e = 0; e < N; ++e) {
            const int32_t *src = t->keys[o] + e * n;
            int32_t key[6];
            for (int q = 0; q < 6; ++q) key[q] = NG_PAD;
            for (int q = 0; q < n; ++q) {
                if (src[q] < 0 || src[q] >= vocab) {
                    err = "order " + std::to_string(n) + " entry " + std::to_string(e) + ": token id outside [0, vocab)";
                    return SPD_ETABLE;
                }
                key[q] = src[q];
            }
            const uint32_t c = t->counts[o][e];
            if (c == 0) {
                err = "order " + std::to_string(n) + " entry " + std::to_string(e) + ": zero count";
                return SPD_ETABLE;
            }
            bool found;
            NgramSlot *s = b.locate(key, found);
            if (found) {
                err = "order " + std::to_string(n) + " entry " + std::to_string(e) + ": duplicate key";
                return SPD_ETABLE;
            }
            std::memcpy(s->tok, key, sizeof(key));
            s->cnt_lo = c;
            s->cnt_hi = 0;
            key[n - 1] = NG_TOTAL;   // the context's running total
            s = b.locate(key, found);
            uint64_t tot = found ? (((uint64_t)s->cnt_hi << 32) | s->cnt_lo) : 0;
            tot += c;
            std::memcpy(s->tok, key, sizeof(key));
            s->cnt_lo = (uint32_t)tot;
            s->cnt_hi = (uint32_t)(tot >> 32);
        }
    }
    return SPD_OK;
}
