// A small caching allocator for device memory.  hipMalloc / hipFree of the 100 MB-class buffers of
// a graph translation cost more than the translation's kernels, so blocks that are given back are
// kept (per device) and handed out again to later requests of a similar size.
//
// Safety rule (kept by every caller in this library): a block is only returned once no kernel that
// uses it can still be running -- after a stream synchronisation inside tcg_sgt_build, or in
// tcg_sgt_free, whose caller guarantees it.
#include "common.h"

#include <mutex>
#include <vector>

namespace tcg {

namespace {

struct Block {
    void *ptr;
    size_t size;
    int device;
    bool in_use;
};

std::mutex g_mu;
std::vector<Block> g_blocks;
constexpr size_t kGranule = 2u << 20;             // sizes are rounded up to 2 MiB
constexpr size_t kMaxCachedBytes = 8ull << 30;    // free blocks kept per process

size_t cached_bytes_locked()
{
    size_t t = 0;
    for (const Block &b : g_blocks)
        if (!b.in_use) t += b.size;
    return t;
}

}  // namespace

int pool_alloc(void **p, size_t bytes)
{
    *p = nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        set_hip_error(hipGetLastError(), "hipGetDevice");
        return TCG_EHIP;
    }
    const size_t want = (std::max<size_t>(bytes, 1) + kGranule - 1) / kGranule * kGranule;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        Block *best = nullptr;
        for (Block &b : g_blocks)
            if (!b.in_use && b.device == dev && b.size >= want && b.size <= want + want / 4 + 4 * kGranule &&
                (!best || b.size < best->size))
                best = &b;
        if (best) {
            best->in_use = true;
            *p = best->ptr;
            return TCG_OK;
        }
    }
    void *q = nullptr;
    hipError_t e = hipMalloc(&q, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        pool_release_all();               // give cached blocks back to the driver and retry once
        e = hipMalloc(&q, want);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        set_hip_error(e, "hipMalloc");
        return TCG_ENOMEM;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    g_blocks.push_back(Block{q, want, dev, true});
    *p = q;
    return TCG_OK;
}

void pool_free(void *p)
{
    if (!p) return;
    std::lock_guard<std::mutex> lk(g_mu);
    for (size_t i = 0; i < g_blocks.size(); ++i) {
        if (g_blocks[i].ptr != p) continue;
        g_blocks[i].in_use = false;
        // Over the cap: hand the largest free blocks back to the driver.
        while (cached_bytes_locked() > kMaxCachedBytes) {
            size_t big = g_blocks.size();
            for (size_t k = 0; k < g_blocks.size(); ++k)
                if (!g_blocks[k].in_use && (big == g_blocks.size() || g_blocks[k].size > g_blocks[big].size)) big = k;
            if (big == g_blocks.size()) break;
            (void)hipFree(g_blocks[big].ptr);
            g_blocks.erase(g_blocks.begin() + big);
        }
        return;
    }
    (void)hipFree(p);   // not one of ours
}

void pool_release_all()
{
    std::lock_guard<std::mutex> lk(g_mu);
    for (size_t i = 0; i < g_blocks.size();) {
        if (!g_blocks[i].in_use) {
            (void)hipFree(g_blocks[i].ptr);
            g_blocks.erase(g_blocks.begin() + i);
        } else {
            ++i;
        }
    }
}

}  // namespace tcg
