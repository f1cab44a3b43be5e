// The hash table of the de-duplication: open addressing over 64-bit words {id : 32 | position : 32},
// all ones = empty.  A slot is claimed with one compare-and-swap; later positions of the same ID fold in
// with a 64-bit atomic minimum (the ID is in the high half, so the minimum orders by position), which
// leaves in every slot the first position that holds its ID however the threads were scheduled.
#pragma once
#include "common.hpp"

namespace helios {

constexpr unsigned long long kEmptySlot = ~0ull;

__device__ __forceinline__ uint32_t hash_id(uint32_t id, uint32_t mask) {
    uint32_t h = id * 0x9E3779B1u;
    h ^= h >> 15;
    h *= 0x85EBCA77u;
    h ^= h >> 13;
    return h & mask;
}

// Inserts (id, pos) and returns the slot of the ID.  The table has at least twice as many slots as
// insertions, so an empty slot is always reached.
__device__ __forceinline__ uint32_t table_insert(unsigned long long* table, uint32_t mask, uint32_t id, uint32_t pos) {
    const unsigned long long mine = (static_cast<unsigned long long>(id) << 32) | pos;
    uint32_t slot = hash_id(id, mask);
    while (true) {
        // try to claim straight away: one round trip when the slot is free (the common case)
        const unsigned long long cur = atomicCAS(table + slot, kEmptySlot, mine);
        if (cur == kEmptySlot) break;                               // claimed
        if (static_cast<uint32_t>(cur >> 32) == id) {
            if (mine < cur) atomicMin(table + slot, mine);
            break;
        }
        slot = (slot + 1) & mask;
    }
    return slot;
}

// A table that a producing kernel inserts its outputs into as it writes them, so that the
// de-duplication of those outputs needs no insert pass of its own.
struct InsertInto {
    unsigned long long* table;   // nullable: nothing is inserted
    uint32_t n_slots;            // power of two
    int32_t* slot_of;            // [position] slot of every inserted element, -1 for a value that is no node ID
};

// A table to be set to all ones on the way by a kernel that runs before the table's first insert.
struct ClearJob {
    unsigned long long* table;   // nullable
    uint32_t n_slots;
};

__device__ __forceinline__ void clear_slots(const ClearJob& c) {
    if (!c.table) return;
    for (uint32_t w = blockIdx.x * blockDim.x + threadIdx.x; w < c.n_slots; w += gridDim.x * blockDim.x) c.table[w] = kEmptySlot;
}

}  // namespace helios
