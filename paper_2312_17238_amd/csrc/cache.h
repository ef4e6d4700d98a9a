// Host-side bookkeeping of the expert cache and the staging buffers: pure C++, no HIP.
//
// Sec. 3.1: every layer keeps the k most recently used experts on the device and evicts the least
// recently used one.  Sec. 3.3: speculatively loaded experts go to b extra buffers shared by all
// layers, replace nothing when they arrive, and on use replace the next layer's least recently used
// entry; the total number of equal-size buffers is fixed.  Buffers are identified by an index into
// the context's pool, so "replace" is an exchange of indices, never a device copy.
//
// Sec. 3.3 also describes hosts that cannot hold every expert: experts are then split between host and
// device buffers, and loading one writes the evicted one back ("swap").  The decisions are the same; what
// changes is which buffer a miss is loaded into (a free staging buffer when there is one, so that the load
// does not wait for the evicted expert to drain out of the slot's old buffer) and the record of the buffer
// the victim has to be read from.
#pragma once
#include <algorithm>
#include <cstdint>
#include <vector>

namespace moe {

struct StagedGuess { int32_t expert; int32_t buf; };

struct CopyOp { int32_t expert; int32_t buf; uint64_t offset = 0, bytes = 0; int32_t host_buf = -1; };   // bytes [offset, offset+bytes) of the host blob of `expert` (in host buffer host_buf) -> pool buffer `buf`

struct AccessRec { int32_t expert, status, slot, victim, buf; int32_t victim_buf = -1; };   // victim_buf: pool buffer the victim occupied

struct LayerCache {
    int32_t k = 0, n_experts = 0;
    std::vector<int32_t> slot_expert;   // -1 = empty
    std::vector<uint64_t> slot_stamp;
    std::vector<int32_t> slot_buf;      // pool buffer behind each slot
    std::vector<StagedGuess> staged;    // guesses loaded for this layer, not yet used

    int find(int32_t e) const
    {
        for (int s = 0; s < k; ++s)
            if (slot_expert[s] == e) return s;
        return -1;
    }
    int find_staged(int32_t e) const
    {
        for (size_t i = 0; i < staged.size(); ++i)
            if (staged[i].expert == e) return (int)i;
        return -1;
    }
};

struct Counters {
    uint64_t steps = 0, needed = 0, hits = 0, prefetch_hits = 0, misses = 0, evictions = 0, spec_issued = 0,
             spec_wasted = 0, bytes_demand = 0, bytes_spec = 0, bytes_writeback = 0;
};

struct BufferPool {
    std::vector<int32_t> free_staging;  // indices of staging buffers holding nothing that is still wanted
    uint64_t clock = 0;                 // one recency clock for all layers
};

// Resolve the accesses of one step: `needed` ascending and distinct.  Resident experts are touched
// first, then absent ones, each in ascending id.  Appends demand copies to `copies`.
// redirect: a miss that evicts takes a free staging buffer for the slot, when there is one, and frees the victim's
// (swap mode: the victim is still draining out of its buffer; a step that needs more experts than the layer has
// slots: the victim's buffer is still being read by this step's earlier kernels).
inline void resolve_accesses(LayerCache &c, BufferPool &pool, Counters &st, const std::vector<int32_t> &needed,
                             bool forget_first, std::vector<AccessRec> &out, std::vector<CopyOp> &copies,
                             bool redirect = false)
{
    if (forget_first)
        for (int s = 0; s < c.k; ++s) c.slot_expert[s] = -1;
    st.steps++;
    st.needed += needed.size();
    for (int32_t e : needed) {
        int s = c.find(e);
        if (s < 0) continue;
        c.slot_stamp[s] = ++pool.clock;
        st.hits++;
        out.push_back({e, 0 /*HIT*/, s, -1, c.slot_buf[s], -1});
    }
    const size_t n_res = out.size();
    for (int32_t e : needed) {
        bool was_resident = false;
        for (size_t i = 0; i < n_res; ++i)
            if (out[i].expert == e) was_resident = true;
        if (was_resident) continue;
        int s = c.find(-1);
        int32_t victim = -1;
        if (s < 0) {
            s = 0;
            for (int i = 1; i < c.k; ++i)
                if (c.slot_stamp[i] < c.slot_stamp[s]) s = i;
            victim = c.slot_expert[s];
            st.evictions++;
        }
        int g = c.find_staged(e);
        int32_t status;
        const int32_t old_buf = c.slot_buf[s];
        if (g >= 0) {                       // used guess: its buffer becomes the slot, the slot's old buffer is freed
            status = 1;                     // PREFETCH_HIT
            std::swap(c.slot_buf[s], c.staged[g].buf);
            pool.free_staging.push_back(c.staged[g].buf);
            c.staged.erase(c.staged.begin() + g);
            st.prefetch_hits++;
        } else {
            status = 2;                     // MISS
            if (redirect && victim >= 0 && !pool.free_staging.empty()) {
                auto it = std::min_element(pool.free_staging.begin(), pool.free_staging.end());
                c.slot_buf[s] = *it;        // one buffer taken, one given back: the number of free buffers,
                *it = old_buf;              // the only thing decisions depend on, does not change
            }
            copies.push_back({e, c.slot_buf[s]});
            st.misses++;
        }
        c.slot_expert[s] = e;
        c.slot_stamp[s] = ++pool.clock;
        out.push_back({e, status, s, victim, c.slot_buf[s], victim >= 0 ? old_buf : -1});
    }
    // guesses this step did not use are dropped; their buffers are free again
    st.spec_wasted += c.staged.size();
    for (const StagedGuess &g : c.staged) pool.free_staging.push_back(g.buf);
    c.staged.clear();
}

// Order experts by (score descending, id ascending) and keep the first m.
inline std::vector<int32_t> top_m(const double *score, int32_t n, int32_t m)
{
    std::vector<int32_t> ord(n);
    for (int i = 0; i < n; ++i) ord[i] = i;
    std::stable_sort(ord.begin(), ord.end(), [&](int a, int b) { return score[a] > score[b]; });
    ord.resize(std::min(n, m));
    return ord;
}

// Stage guesses for layer `c` (the next layer): skip those resident or already staged; stop issuing
// when no staging buffer is free.  Touches no recency stamp and evicts nothing.
inline void stage_guesses(LayerCache &c, BufferPool &pool, Counters &st, const std::vector<int32_t> &guess,
                          std::vector<int32_t> &issued, std::vector<CopyOp> &copies)
{
    for (int32_t e : guess) {
        bool go = c.find(e) < 0 && c.find_staged(e) < 0 && !pool.free_staging.empty();
        if (go) {
            // take the lowest-numbered free buffer: keeps the choice independent of release order details
            auto it = std::min_element(pool.free_staging.begin(), pool.free_staging.end());
            int32_t buf = *it;
            pool.free_staging.erase(it);
            c.staged.push_back({e, buf});
            copies.push_back({e, buf});
            st.spec_issued++;
        }
        issued.push_back(go ? 1 : 0);
    }
}

}  // namespace moe
