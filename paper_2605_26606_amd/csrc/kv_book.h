// Host-side bookkeeping of the paged KV cache: slots (one per live prompt or sequence), their block lists,
// reference counts of the shared prefix blocks, the free lists and the host mirrors of the device block table.
// Plain C++, no HIP calls, no device code: the context (api.hip) owns one of these, and the same code runs on
// the CPU under the address / undefined-behaviour sanitizers (tests/host/host_checks.hip).
#pragma once

#include <stdint.h>

#include <vector>

namespace pc {

struct Slot {
    bool used = false;
    bool is_prompt = false;
    int len = 0;          // tokens whose K/V are in the cache
    int capacity = 0;     // tokens the slot's blocks can hold
    int limit = 0;        // tokens the slot may hold: prompt length + reserved new tokens, at most max_ctx
    int prompt = -1;      // sequences: the prompt slot they were forked from
    std::vector<int32_t> blocks;
};

struct KvBook {
    int block_size = 0, max_slots = 0, max_blocks_per_slot = 0;
    int64_t n_blocks = 0;
    std::vector<Slot> slots;
    std::vector<int32_t> refcnt, free_blocks, free_slots;
    std::vector<int32_t> h_table, h_len;   // mirrors of the device block table [slot][max_blocks_per_slot] / lengths

    void init(int block_size_, int max_slots_, int max_ctx, int64_t n_blocks_) {
        block_size = block_size_;
        max_slots = max_slots_;
        n_blocks = n_blocks_;
        max_blocks_per_slot = (max_ctx + block_size - 1) / block_size;
        h_table.assign((size_t)max_slots * max_blocks_per_slot, 0);
        h_len.assign(max_slots, 0);
        refcnt.assign((size_t)n_blocks, 0);
        free_blocks.clear();
        free_blocks.reserve((size_t)n_blocks);
        for (int64_t b = n_blocks - 1; b >= 0; --b) free_blocks.push_back((int32_t)b);
        slots.assign(max_slots, Slot());
        free_slots.clear();
        free_slots.reserve(max_slots);
        for (int s = max_slots - 1; s >= 0; --s) free_slots.push_back(s);
    }
    bool live_prompt(int h) const { return h >= 0 && h < max_slots && slots[h].used && slots[h].is_prompt; }
    bool live_sequence(int s) const { return s >= 0 && s < max_slots && slots[s].used && !slots[s].is_prompt; }
    int64_t prompt_blocks(int len) const { return (len + block_size - 1) / block_size; }
    // blocks a fork of this prompt takes from the pool: everything behind the prompt's full blocks
    int64_t fork_blocks(int prompt, int max_new_tokens) const {
        const int len = slots[prompt].len;
        return (len + max_new_tokens + block_size - 1) / block_size - len / block_size;
    }
    void write_table_row(int slot) {
        const Slot &s = slots[slot];
        int32_t *row = h_table.data() + (size_t)slot * max_blocks_per_slot;
        for (size_t i = 0; i < s.blocks.size(); ++i) row[i] = s.blocks[i];
        h_len[slot] = s.len;
    }
    int32_t take_block() {
        const int32_t b = free_blocks.back();
        free_blocks.pop_back();
        refcnt[b] = 1;
        return b;
    }
    // The caller has checked that a slot and prompt_blocks(len) blocks are free.
    int take_prompt(int len) {
        const int slot = free_slots.back();
        free_slots.pop_back();
        Slot &s = slots[slot];
        s.used = true;
        s.is_prompt = true;
        s.len = len;
        const int nb = (int)prompt_blocks(len);
        s.capacity = nb * block_size;
        s.limit = len;
        for (int i = 0; i < nb; ++i) s.blocks.push_back(take_block());
        write_table_row(slot);
        return slot;
    }
    // The caller has checked that a slot and fork_blocks(...) blocks are free.  A partially filled last prompt
    // block gets a private copy: (source, destination) is appended to copy_pairs.
    int take_fork(int prompt, int max_new_tokens, std::vector<int32_t> &copy_pairs) {
        const int slot = free_slots.back();
        free_slots.pop_back();
        const Slot &ps = slots[prompt];
        Slot &s = slots[slot];
        s.used = true;
        s.is_prompt = false;
        s.prompt = prompt;
        s.len = ps.len;
        const int n_full = ps.len / block_size, total = (ps.len + max_new_tokens + block_size - 1) / block_size;
        for (int b = 0; b < n_full; ++b) {
            s.blocks.push_back(ps.blocks[b]);
            refcnt[ps.blocks[b]]++;
        }
        for (int b = n_full; b < total; ++b) {
            const int32_t nb = take_block();
            s.blocks.push_back(nb);
            if (b == n_full && ps.len % block_size) {
                copy_pairs.push_back(ps.blocks[b]);
                copy_pairs.push_back(nb);
            }
        }
        s.capacity = total * block_size;
        s.limit = ps.len + max_new_tokens;
        write_table_row(slot);
        return slot;
    }
    void release(int slot) {
        Slot &s = slots[slot];
        for (int32_t b : s.blocks)
            if (--refcnt[b] == 0) free_blocks.push_back(b);
        s = Slot();
        free_slots.push_back(slot);
    }
    void advance(int slot) {
        slots[slot].len++;
        h_len[slot]++;
    }
};

}  // namespace pc
