// Host-side bookkeeping of the carry chain's status-word tags.  Plain C++ (no HIP): a CPU test compiles this file
// on its own, with TCUSCAN_TAG_MOD shrunk so that the tags wrap after a handful of calls.
//
// A status word carries a 30-bit tag.  Tag 0 is what a zero-filled word reads as; tags 1 .. kTagMod go round with
// the process-wide call counter, so within one round ("generation") every call's tag is unique and a word left by
// an earlier call never reads as published.  After kTagMod calls the tags repeat: a word last written exactly one
// generation earlier would then pass for a word of the current call.  The library therefore remembers, per
// workspace, the generation in which its status words were last known to be free of older generations' tags, and
// has them cleared (by the caller of needs_clear(), with a fill kernel on the call's stream) the first time a
// workspace is used in a new generation.  The last value of the tag field, kClearFirstTag, is never drawn from the
// counter: it belongs to calls that clear their status words themselves before every run (calls recorded by stream
// capture, which are replayed with the tag they were recorded with, and calls on workspace regions whose former
// contents the library cannot vouch for).
#ifndef TCUSCAN_CHAIN_TAGS_H
#define TCUSCAN_CHAIN_TAGS_H

#include <stddef.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#ifndef TCUSCAN_TAG_MOD
#define TCUSCAN_TAG_MOD ((1u << 30) - 2u)
#endif

namespace chain_tags {

constexpr uint32_t kTagMod = TCUSCAN_TAG_MOD;            // tags drawn from the call counter: 1 .. kTagMod
constexpr uint32_t kClearFirstTag = (1u << 30) - 1u;     // reserved: the call clears its own status words first
static_assert(kTagMod >= 1u && kTagMod < kClearFirstTag, "counter tags must leave 0 and the reserved tag free");

struct CallId {
    uint32_t tag;            // 1 .. kTagMod
    uint64_t generation;     // 1, 2, ...: how many times the tags have gone round, plus one
};

// The `index`-th call of the process (0-based, from a 64-bit counter that cannot wrap in practice).
inline CallId call_id(uint64_t index)
{
    CallId id;
    id.tag = (uint32_t)(index % kTagMod) + 1u;
    id.generation = index / kTagMod + 1u;
    return id;
}

// Which workspaces are known to hold nothing that could pass for a status word of the current call, and how many
// bytes of each.
class CleanTable {
public:
    static constexpr int kSlots = 64;

    // Must the status words in the first `bytes` bytes of the workspace at `ws` be cleared before a call of
    // `generation` uses them?  Answers yes once per workspace, generation and growth in size (and after every
    // mark_dirty), and records the workspace as clean on the assumption that the caller then does clear them (in
    // stream order, before the call).
    //
    // In generation 1 a workspace the table does not know needs no clear: no older generation exists, and a
    // workspace is zero-filled by its owner before its first use.  From generation 2 on an unknown workspace (first
    // use in this generation, or its entry was displaced by 64 more recently used ones) is cleared: clearing too
    // often costs a fill kernel, never a result.
    bool needs_clear(uintptr_t ws, size_t bytes, uint64_t generation)
    {
        if (generation <= 1u && !tracking_.load(std::memory_order_acquire)) return false;    // nothing recorded yet
        std::lock_guard<std::mutex> lock(mu_);
        Entry *e = find(ws);
        if (e) {
            const bool clean = e->generation == generation && bytes <= e->bytes;
            if (e->generation != generation) e->bytes = 0;
            e->generation = generation;
            if (bytes > e->bytes) e->bytes = bytes;
            e->used = ++clock_;
            return !clean;
        }
        if (generation <= 1u && !strict_) return false;
        insert(Entry{ws, bytes, generation, ++clock_});
        return true;
    }

    // The workspace at `ws` has been given contents other than status words (the row maps of a segmented scan)
    // where a later call of another shape may expect status words: whatever the table knew about it is void.
    void mark_dirty(uintptr_t ws, uint64_t generation)
    {
        std::lock_guard<std::mutex> lock(mu_);
        tracking_.store(true, std::memory_order_release);
        Entry *e = find(ws);
        if (e) { e->bytes = 0; e->generation = generation; e->used = ++clock_; }
        else insert(Entry{ws, 0, generation, ++clock_});
    }

private:
    struct Entry {
        uintptr_t ws;
        size_t bytes;            // 0: dirty
        uint64_t generation;     // 0: empty slot
        uint64_t used;
    };
    Entry *find(uintptr_t ws)
    {
        for (int i = 0; i < kSlots; ++i)
            if (slot_[i].generation != 0u && slot_[i].ws == ws) return &slot_[i];
        return nullptr;
    }
    void insert(const Entry &n)
    {
        int victim = 0;
        for (int i = 1; i < kSlots; ++i)
            if (slot_[i].used < slot_[victim].used) victim = i;      // least recently used (empty slots: used == 0)
        // a displaced "dirty" mark is knowledge lost: from now on unknown workspaces are cleared in generation 1 too
        if (slot_[victim].generation != 0u && slot_[victim].bytes == 0) strict_ = true;
        slot_[victim] = n;
    }
    std::mutex mu_;
    std::atomic<bool> tracking_{false};
    bool strict_ = false;
    uint64_t clock_ = 0;
    Entry slot_[kSlots] = {};
};

}  // namespace chain_tags

#endif
