// Expert Buffering, cache management (paper Sec. 6, "Cache Management"): which expert's parameters
// occupy which device slot, what is copied in for a batch and what is thrown out.  Host logic only --
// no HIP call in this file -- so it can be exercised without a GPU.
//
// The experts with a positive token count are the batch's active experts; they are visited in
// increasing id order (the order in which the paper's systems execute the experts of a device).
// A resident expert is a hit.  A miss takes a free slot, else the slot of a victim: first the
// residents that are not active in this batch, then the active ones, and inside each class the one
// that entered the cache last (Last In, First Out) -- with a cache of 2 and experts (1, 2, 3)
// needed, 3 replaces 2 and 1 stays, the paper's example.
//
// Execution stages: a victim that already ran in this batch must finish computing before its slot
// is overwritten, so its replacement runs one stage later; otherwise stages are as early as
// possible and never decrease along the id order.  Inside a stage every expert has its own slot.
#include <new>
#include <vector>

#include "moe_internal.h"

struct moe_cache_policy {
    int E = 0, slots = 0;
    std::vector<int> slot_expert;        // [slots] expert held, -1 free
    std::vector<int> where;              // [E] slot of a resident expert, -1 otherwise
    std::vector<long long> inserted;     // [E] when it entered the cache
    long long clock = 0, hits = 0, misses = 0;
};

namespace moe355 {

int cache_policy_step(moe_cache_policy *p, const int32_t *counts, int32_t *slot_of, int32_t *stage_of,
                      int32_t *loads, int32_t max_loads, int32_t *n_loads, int32_t *n_stages)
{
    int stage = 0, nl = 0;
    bool any = false;
    for (int e = 0; e < p->E; ++e) {
        slot_of[e] = -1;
        stage_of[e] = -1;
    }
    for (int e = 0; e < p->E; ++e) {
        if (counts[e] <= 0) continue;
        any = true;
        ++p->clock;
        if (p->where[e] >= 0) {
            ++p->hits;
        } else {
            ++p->misses;
            int slot = -1, victim = -1;
            for (int s = 0; s < p->slots && slot < 0; ++s)
                if (p->slot_expert[s] < 0) slot = s;
            if (slot < 0) {
                // idle residents first, then active ones; last in first out inside the class
                long long best = -1;
                bool best_idle = false;
                for (int s = 0; s < p->slots; ++s) {
                    const int r = p->slot_expert[s];
                    const bool idle = counts[r] <= 0;
                    if (victim < 0 || (idle && !best_idle) || (idle == best_idle && p->inserted[r] > best)) {
                        victim = r;
                        best = p->inserted[r];
                        best_idle = idle;
                    }
                }
                slot = p->where[victim];
                p->where[victim] = -1;
                if (stage_of[victim] >= 0 && stage_of[victim] + 1 > stage) stage = stage_of[victim] + 1;
            }
            p->slot_expert[slot] = e;
            p->where[e] = slot;
            p->inserted[e] = p->clock;
            if (nl < max_loads) {
                loads[4 * nl + 0] = e;
                loads[4 * nl + 1] = slot;
                loads[4 * nl + 2] = victim;
                loads[4 * nl + 3] = stage;
            }
            ++nl;
        }
        slot_of[e] = p->where[e];
        stage_of[e] = stage;
    }
    *n_loads = nl;
    *n_stages = any ? stage + 1 : 0;
    if (nl > max_loads) {
        set_error("load list holds %d entries, %d are needed", max_loads, nl);
        return MOE_ERR_INVALID_ARG;
    }
    return MOE_OK;
}

}  // namespace moe355

extern "C" {

int moe_cache_policy_create(int32_t E, int32_t slots, moe_cache_policy_t **out)
{
    if (!out || E < 1 || E > MOE_MAX_E || slots < 1) {
        moe355::set_error("cache policy: E = %d or slots = %d out of range, or out is NULL", E, slots);
        return MOE_ERR_INVALID_ARG;
    }
    moe_cache_policy *p = new (std::nothrow) moe_cache_policy;
    if (!p) {
        moe355::set_error("out of host memory");
        return MOE_ERR_INVALID_ARG;
    }
    p->E = E;
    p->slots = slots;
    p->slot_expert.assign(slots, -1);
    p->where.assign(E, -1);
    p->inserted.assign(E, 0);
    *out = p;
    return MOE_OK;
}

int moe_cache_policy_destroy(moe_cache_policy_t *p)
{
    delete p;
    return MOE_OK;
}

int moe_cache_policy_reset(moe_cache_policy_t *p)
{
    if (!p) {
        moe355::set_error("cache policy is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    p->slot_expert.assign(p->slots, -1);
    p->where.assign(p->E, -1);
    p->clock = p->hits = p->misses = 0;
    return MOE_OK;
}

int moe_cache_policy_step(moe_cache_policy_t *p, const int32_t *counts, int32_t *slot_of, int32_t *stage_of,
                          int32_t *loads, int32_t max_loads, int32_t *n_loads, int32_t *n_stages)
{
    if (!p || !counts || !slot_of || !stage_of || !n_loads || !n_stages || (max_loads > 0 && !loads) || max_loads < 0) {
        moe355::set_error("cache policy step: NULL argument");
        return MOE_ERR_INVALID_ARG;
    }
    return moe355::cache_policy_step(p, counts, slot_of, stage_of, loads, max_loads, n_loads, n_stages);
}

int moe_cache_policy_stats(const moe_cache_policy_t *p, int64_t *hits, int64_t *misses, int32_t *slot_expert)
{
    if (!p) {
        moe355::set_error("cache policy is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (hits) *hits = p->hits;
    if (misses) *misses = p->misses;
    if (slot_expert)
        for (int s = 0; s < p->slots; ++s) slot_expert[s] = p->slot_expert[s];
    return MOE_OK;
}

}  // extern "C"
