// C entry points around paper_2411_17887_amd/csrc/chain_tags.h for tests/test_chain_tags_cpu.py, which compiles this
// file with g++ and a small -DTCUSCAN_TAG_MOD so that the tags wrap after a handful of calls.
#include "../paper_2411_17887_amd/csrc/chain_tags.h"

extern "C" {

unsigned shim_tag_mod(void) { return chain_tags::kTagMod; }
unsigned shim_clear_first_tag(void) { return chain_tags::kClearFirstTag; }
int shim_slots(void) { return chain_tags::CleanTable::kSlots; }

void shim_call_id(unsigned long long index, unsigned *tag, unsigned long long *generation)
{
    const chain_tags::CallId id = chain_tags::call_id(index);
    *tag = id.tag;
    *generation = id.generation;
}

void *shim_table_new(void) { return new chain_tags::CleanTable(); }
void shim_table_free(void *t) { delete (chain_tags::CleanTable *)t; }
int shim_needs_clear(void *t, unsigned long long ws, unsigned long long bytes, unsigned long long generation)
{
    return ((chain_tags::CleanTable *)t)->needs_clear((uintptr_t)ws, (size_t)bytes, generation) ? 1 : 0;
}
void shim_mark_dirty(void *t, unsigned long long ws, unsigned long long generation)
{
    ((chain_tags::CleanTable *)t)->mark_dirty((uintptr_t)ws, generation);
}

}
