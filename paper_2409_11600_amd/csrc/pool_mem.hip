// Size-keyed device memory pool and name-keyed cache (section "Caching and Pooling" of the paper).
//
// Pool: a dictionary from the byte size of a tensor to a list of free device pointers of exactly that size.  A request
// pops a pointer from its size's list, or allocates one when the list is empty (the first iteration); a release
// appends the pointer to its size's list instead of freeing it.  A training step that asks for the same sizes in
// every iteration therefore allocates nothing from the second iteration on.
// Cache: a dictionary from a name to a device pointer that lives until the pool is destroyed (the paper keeps the
// gradient buffers of parameters this way: looked up by parameter name, accumulated into, zeroed by the optimizer).
//
// Host code only.  The backing allocator is hipMalloc/hipFree, or plain aligned host memory for a pool created with
// NSK_POOL_HOST (pinned staging is not needed on this path; the host mode exists so that the bookkeeping can be used
// and tested on a machine without a GPU).  A pool is not thread-safe: one pool per thread, as one per stream.
#include <stdlib.h>

#include <map>
#include <string>
#include <unordered_map>
#include <vector>

#include "nsk_internal.h"

struct nsk_pool {
    int kind;
    std::map<size_t, std::vector<void *>> free_lists;      // size -> free pointers of that size
    std::unordered_map<void *, size_t> size_of;            // every pointer this pool ever allocated -> its size
    std::unordered_map<void *, bool> live;                 // pointer -> handed out and not yet returned
    std::unordered_map<std::string, std::pair<void *, size_t>> cache;
    size_t bytes_allocated = 0, allocations = 0, hits = 0, requests = 0;
};

namespace {

size_t round_up(size_t bytes) { return (bytes + 255) / 256 * 256; }

int backend_alloc(nsk_pool *p, size_t bytes, void **out)
{
    if (p->kind == NSK_POOL_HOST) {
        *out = aligned_alloc(256, bytes);
        return *out ? NSK_OK : NSK_ERR_HIP;
    }
    const hipError_t e = hipMalloc(out, bytes);
    if (e != hipSuccess) {
        nsk::set_last_hip_error(e);
        *out = nullptr;
        return NSK_ERR_HIP;
    }
    return NSK_OK;
}

void backend_free(nsk_pool *p, void *ptr)
{
    if (p->kind == NSK_POOL_HOST)
        free(ptr);
    else
        (void)hipFree(ptr);
}

}  // namespace

extern "C" {

int nsk_pool_create(int kind, nsk_pool_t **pool)
{
    if (!pool) return NSK_ERR_NULL;
    if (kind != NSK_POOL_DEVICE && kind != NSK_POOL_HOST) return NSK_ERR_BAD_DESC;
    nsk_pool *p = new (std::nothrow) nsk_pool();
    if (!p) return NSK_ERR_HIP;
    p->kind = kind;
    *pool = p;
    return NSK_OK;
}

int nsk_pool_get(nsk_pool_t *pool, size_t bytes, void **ptr)
{
    if (!pool || !ptr) return NSK_ERR_NULL;
    if (bytes == 0) return NSK_ERR_BAD_DESC;
    const size_t size = round_up(bytes);
    pool->requests++;
    std::vector<void *> &list = pool->free_lists[size];
    if (!list.empty()) {
        *ptr = list.back();
        list.pop_back();
        pool->hits++;
    } else {
        void *fresh = nullptr;
        const int st = backend_alloc(pool, size, &fresh);
        if (st != NSK_OK) return st;
        pool->size_of[fresh] = size;
        pool->bytes_allocated += size;
        pool->allocations++;
        *ptr = fresh;
    }
    pool->live[*ptr] = true;
    return NSK_OK;
}

int nsk_pool_put(nsk_pool_t *pool, void *ptr)
{
    if (!pool || !ptr) return NSK_ERR_NULL;
    auto it = pool->live.find(ptr);
    if (it == pool->live.end() || !it->second) return NSK_ERR_BAD_DESC;   // not from this pool, or returned twice
    it->second = false;
    pool->free_lists[pool->size_of[ptr]].push_back(ptr);
    return NSK_OK;
}

int nsk_pool_cached(nsk_pool_t *pool, const char *name, size_t bytes, void **ptr, int *created)
{
    if (!pool || !name || !ptr) return NSK_ERR_NULL;
    if (bytes == 0) return NSK_ERR_BAD_DESC;
    auto it = pool->cache.find(name);
    if (it != pool->cache.end()) {
        if (it->second.second != round_up(bytes)) return NSK_ERR_BAD_DESC;   // the same name with another size
        *ptr = it->second.first;
        if (created) *created = 0;
        return NSK_OK;
    }
    void *fresh = nullptr;
    const size_t size = round_up(bytes);
    const int st = backend_alloc(pool, size, &fresh);
    if (st != NSK_OK) return st;
    pool->cache[name] = std::make_pair(fresh, size);
    pool->bytes_allocated += size;
    pool->allocations++;
    *ptr = fresh;
    if (created) *created = 1;
    return NSK_OK;
}

int nsk_pool_stats(const nsk_pool_t *pool, size_t *bytes_allocated, size_t *allocations, size_t *requests, size_t *hits)
{
    if (!pool) return NSK_ERR_NULL;
    if (bytes_allocated) *bytes_allocated = pool->bytes_allocated;
    if (allocations) *allocations = pool->allocations;
    if (requests) *requests = pool->requests;
    if (hits) *hits = pool->hits;
    return NSK_OK;
}

int nsk_pool_destroy(nsk_pool_t *pool)
{
    if (!pool) return NSK_ERR_NULL;
    for (auto &kv : pool->size_of) backend_free(pool, kv.first);
    for (auto &kv : pool->cache) backend_free(pool, kv.second.first);
    delete pool;
    return NSK_OK;
}

}  // extern "C"
