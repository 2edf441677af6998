// Host-side free list of physical KV blocks: which block a request gets when its cache crosses a
// block boundary (Section 4: sub-blocks are the unit in which the growing KV cache is managed).
#include <algorithm>
#include <new>
#include <vector>

#include "../../include/distattn.h"

struct da_block_pool {
    int32_t num_blocks;
    std::vector<int32_t> free_ids;  // stack: back() is handed out next
    std::vector<uint8_t> in_use;
};

extern "C" {

da_status da_block_pool_create(int32_t num_phys_blocks, da_block_pool **pool)
{
    if (!pool) return DA_ERR_INVALID_ARG;
    *pool = nullptr;
    if (num_phys_blocks < 1) return DA_ERR_INVALID_ARG;
    da_block_pool *p = new (std::nothrow) da_block_pool();
    if (!p) return DA_ERR_HIP;
    p->num_blocks = num_phys_blocks;
    p->free_ids.resize(num_phys_blocks);
    for (int32_t i = 0; i < num_phys_blocks; ++i) p->free_ids[i] = num_phys_blocks - 1 - i;  // block 0 goes first
    p->in_use.assign(num_phys_blocks, 0);
    *pool = p;
    return DA_OK;
}

da_status da_block_pool_destroy(da_block_pool *pool)
{
    delete pool;
    return DA_OK;
}

da_status da_block_pool_free_count(const da_block_pool *pool, int32_t *count)
{
    if (!pool || !count) return DA_ERR_INVALID_ARG;
    *count = (int32_t)pool->free_ids.size();
    return DA_OK;
}

da_status da_block_pool_grow(da_block_pool *pool, int32_t block_tokens, int32_t max_blocks_per_seq,
                             int32_t *block_table_row_host, int32_t cur_len, int32_t new_len)
{
    if (!pool || !block_table_row_host || block_tokens < 1 || max_blocks_per_seq < 1 || cur_len < 0 || new_len < cur_len)
        return DA_ERR_INVALID_ARG;
    const int64_t have = ((int64_t)cur_len + block_tokens - 1) / block_tokens;
    const int64_t need = ((int64_t)new_len + block_tokens - 1) / block_tokens;
    if (need > max_blocks_per_seq) return DA_ERR_INVALID_ARG;
    if (need - have > (int64_t)pool->free_ids.size()) return DA_ERR_NO_SPACE;  // nothing is taken
    for (int64_t b = have; b < need; ++b) {
        const int32_t id = pool->free_ids.back();
        pool->free_ids.pop_back();
        pool->in_use[id] = 1;
        block_table_row_host[b] = id;
    }
    return DA_OK;
}

da_status da_block_pool_release(da_block_pool *pool, int32_t block_tokens, int32_t *block_table_row_host, int32_t len)
{
    if (!pool || !block_table_row_host || block_tokens < 1 || len < 0) return DA_ERR_INVALID_ARG;
    const int64_t have = ((int64_t)len + block_tokens - 1) / block_tokens;
    for (int64_t b = 0; b < have; ++b) {  // validate first: nothing is returned on error
        const int32_t id = block_table_row_host[b];
        if (id < 0 || id >= pool->num_blocks || !pool->in_use[id]) return DA_ERR_INVALID_ARG;
        for (int64_t c = 0; c < b; ++c)
            if (block_table_row_host[c] == id) return DA_ERR_INVALID_ARG;
    }
    for (int64_t b = have - 1; b >= 0; --b) {
        const int32_t id = block_table_row_host[b];
        pool->in_use[id] = 0;
        pool->free_ids.push_back(id);
        block_table_row_host[b] = -1;
    }
    return DA_OK;
}

}  // extern "C"
