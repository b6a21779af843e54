// Block manager: many weight stacks, one universal stack of residual blocks, one byte budget
// (Section 2.2: blocks are loaded or offloaded as the available memory changes; Section 2.3: the
// universal stack orders all blocks, level by level; the appendix on minimal transmission units:
// a block is the unit that moves, and Eq. 9 is its size).  Host logic only: it drives the stacks
// through bitstack_push_block / bitstack_pop_block of the public interface.
#include <cstddef>
#include <cstdint>
#include <new>
#include <vector>

#include "../../include/bitstack.h"

struct bitstack_manager {
    std::vector<bitstack_weight_t*> stacks;
    std::vector<size_t> block_bytes;            // Eq. 9 per stack
    std::vector<int> slots;                     // blocks a stack can hold
    std::vector<std::vector<const void*>> staged;   // [stack][block]: host staging buffers (caller-owned)
    std::vector<int> order;                     // universal stack: entry e loads the next block of stack order[e]
    int position = 0;                           // entries of the universal stack that are loaded
    size_t resident_bytes = 0;
};

extern "C" {

int bitstack_order_check(int n_stacks, const int* slots, const int* order, int count) {
    if (!slots || (!order && count > 0)) return BITSTACK_E_NULL;
    if (n_stacks < 1 || count < 0) return BITSTACK_E_RANGE;
    std::vector<int> h;
    try {
        h.assign(n_stacks, 0);
    } catch (const std::bad_alloc&) {
        return BITSTACK_E_BUFSIZE;
    }
    for (int e = 0; e < count; ++e) {
        const int s = order[e];
        if (s < 0 || s >= n_stacks) return BITSTACK_E_RANGE;
        if (h[s] >= slots[s]) return BITSTACK_E_RANGE;   // more blocks than the stack has
        // no stack takes block i + 1 before every stack that has a block i has taken it
        for (int t = 0; t < n_stacks; ++t)
            if (h[t] < h[s] && h[t] < slots[t]) return BITSTACK_E_ARG;
        ++h[s];
    }
    return BITSTACK_OK;
}

int bitstack_budget_position(int n_stacks, const size_t* block_bytes, const int* order, int count, size_t budget,
                             int* position, size_t* bytes) {
    if (!block_bytes || (!order && count > 0) || !position) return BITSTACK_E_NULL;
    if (n_stacks < 1 || count < 0) return BITSTACK_E_RANGE;
    size_t total = 0;
    int e = 0;
    for (; e < count; ++e) {
        const int s = order[e];
        if (s < 0 || s >= n_stacks) return BITSTACK_E_RANGE;
        if (block_bytes[s] > budget - total) break;   // total <= budget always holds here
        total += block_bytes[s];
    }
    *position = e;
    if (bytes) *bytes = total;
    return BITSTACK_OK;
}

int bitstack_manager_create(int n_stacks, bitstack_weight_t* const* stacks, bitstack_manager_t** handle) {
    if (!handle) return BITSTACK_E_NULL;
    *handle = nullptr;
    if (!stacks) return BITSTACK_E_NULL;
    if (n_stacks < 1) return BITSTACK_E_RANGE;
    bitstack_manager* m = new (std::nothrow) bitstack_manager;
    if (!m) return BITSTACK_E_BUFSIZE;
    try {
        for (int s = 0; s < n_stacks; ++s) {
            if (!stacks[s]) {
                delete m;
                return BITSTACK_E_NULL;
            }
            int out = 0, in = 0, k = 0, n = 0, mb = 0;
            int rc = bitstack_weight_shape(stacks[s], &out, &in, &k, &n, &mb);
            if (rc == BITSTACK_OK && bitstack_resident_blocks(stacks[s]) != 0) rc = BITSTACK_E_ARG;   // starts empty
            if (rc != BITSTACK_OK) {
                delete m;
                return rc;
            }
            m->stacks.push_back(stacks[s]);
            m->block_bytes.push_back(bitstack_block_bytes(out, in, k));
            m->slots.push_back(n);
            m->staged.emplace_back(size_t(n), nullptr);
        }
    } catch (const std::bad_alloc&) {
        delete m;
        return BITSTACK_E_BUFSIZE;
    }
    *handle = m;
    return BITSTACK_OK;
}

void bitstack_manager_release(bitstack_manager_t* m) { delete m; }

int bitstack_manager_set_block(bitstack_manager_t* m, int stack, int block, const void* staging) {
    if (!m || !staging) return BITSTACK_E_NULL;
    if (stack < 0 || stack >= int(m->stacks.size())) return BITSTACK_E_RANGE;
    if (block < 0 || block >= m->slots[stack]) return BITSTACK_E_RANGE;
    m->staged[stack][block] = staging;
    return BITSTACK_OK;
}

int bitstack_manager_set_order(bitstack_manager_t* m, const int* order, int count) {
    if (!m) return BITSTACK_E_NULL;
    if (m->position != 0) return BITSTACK_E_ARG;   // only while nothing is loaded
    const int rc = bitstack_order_check(int(m->stacks.size()), m->slots.data(), order, count);
    if (rc != BITSTACK_OK) return rc;
    try {
        m->order.assign(order, order + count);
    } catch (const std::bad_alloc&) {
        return BITSTACK_E_BUFSIZE;
    }
    return BITSTACK_OK;
}

int bitstack_manager_set_budget(bitstack_manager_t* m, size_t budget_bytes, bitstack_stream_t stream, int* loaded,
                                int* offloaded) {
    if (!m) return BITSTACK_E_NULL;
    if (loaded) *loaded = 0;
    if (offloaded) *offloaded = 0;
    int target = 0;
    int rc = bitstack_budget_position(int(m->stacks.size()), m->block_bytes.data(), m->order.data(),
                                      int(m->order.size()), budget_bytes, &target, nullptr);
    if (rc != BITSTACK_OK) return rc;
    // every block on the way up must have been staged: checked before anything moves
    {
        std::vector<int> h;
        try {
            h.resize(m->stacks.size());
        } catch (const std::bad_alloc&) {
            return BITSTACK_E_BUFSIZE;
        }
        for (size_t s = 0; s < m->stacks.size(); ++s) h[s] = bitstack_resident_blocks(m->stacks[s]);
        for (int e = m->position; e < target; ++e) {
            const int s = m->order[e];
            if (!m->staged[s][h[s]]) return BITSTACK_E_NULL;
            ++h[s];
        }
    }
    while (m->position > target) {   // offload from the top of the universal stack
        const int s = m->order[m->position - 1];
        rc = bitstack_pop_block(m->stacks[s]);
        if (rc != BITSTACK_OK) return rc;
        --m->position;
        m->resident_bytes -= m->block_bytes[s];
        if (offloaded) ++*offloaded;
    }
    while (m->position < target) {   // load in the order of the universal stack
        const int s = m->order[m->position];
        const int b = bitstack_resident_blocks(m->stacks[s]);
        rc = bitstack_push_block(m->stacks[s], m->staged[s][b], stream);
        if (rc != BITSTACK_OK) return rc;
        ++m->position;
        m->resident_bytes += m->block_bytes[s];
        if (loaded) ++*loaded;
    }
    return BITSTACK_OK;
}

int bitstack_manager_position(const bitstack_manager_t* m) { return m ? m->position : BITSTACK_E_NULL; }

size_t bitstack_manager_resident_bytes(const bitstack_manager_t* m) { return m ? m->resident_bytes : 0; }

int bitstack_manager_n_loaded(const bitstack_manager_t* m, int stack) {
    if (!m) return BITSTACK_E_NULL;
    if (stack < 0 || stack >= int(m->stacks.size())) return BITSTACK_E_RANGE;
    return bitstack_resident_blocks(m->stacks[stack]);
}

}  // extern "C"
