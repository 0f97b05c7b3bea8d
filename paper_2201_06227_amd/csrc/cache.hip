// Activation cache (Section 4.3 of the paper, Figure 6): a table in GPU memory
// keyed by sample id whose value is the sample's activation at the last frozen
// layer; the recent `window` mini-batches are kept (five in the paper).
//
// Layout of the caller-owned cache memory:
//   header   256 B   word 0 magic, word 2 the number of puts so far
//   ids      int64 [window * batch]   sample id of every row slot, -1 = empty;
//                                     mini-batch number t owns slots (t % window) * batch ...
//   keys     int64 [cap]              open-addressing table (linear probing), -1 = empty,
//   vals     uint64 [cap]             cap = power of two >= 2 * window * batch;
//                                     value = (rank of the slot's mini-batch << 32) | slot
//   rows     [window * batch][row stride]   row stride = row bytes rounded up to 16
//
// A put is two launches: the rows go to the slots of the mini-batch that the
// put counter names (any number of workgroups, pure copy), then one workgroup
// records the ids, rebuilds the table from the ids of all slots and advances
// the counter.  Rebuilding instead of deleting keeps the table free of
// tombstones however long training runs, and it is small: the table never
// holds more than window * batch keys.  Where an id sits in several slots the
// table keeps the largest value, i.e. the newest mini-batch and, within one
// mini-batch, the last occurrence (a 64-bit atomic maximum, so the outcome does
// not depend on the order in which threads arrive).  A get probes the table
// once per row and copies the row; rows of ids that are not found are not
// touched.  Both copies are bound by HBM: 2 * row bytes moved per row.
#include "common.hpp"

namespace egeria {

namespace {

constexpr uint32_t kCacheMagic = 0xE6E7CAC4u;
constexpr int64_t kEmptyKey = -1;
constexpr int kCopyThreads = 256;
constexpr int64_t kChunkBytes = 32768;        // bytes of a row one workgroup copies

struct CacheLayout {
    bool ok = false;
    int64_t slots = 0;          // window * batch
    uint32_t cap = 0;           // table entries, power of two
    size_t row_bytes = 0, row_stride = 0;
    size_t off_ids = 0, off_keys = 0, off_vals = 0, off_rows = 0, total = 0;
};

CacheLayout cache_layout(const egeria_cache_desc *d)
{
    CacheLayout L;
    if (!d || d->window < 1 || d->batch < 1 || d->row_elems < 1) return L;
    if (d->dtype != EGERIA_F32 && d->dtype != EGERIA_BF16) return L;
    L.slots = (int64_t)d->window * d->batch;
    if (L.slots > (1 << 20) || d->batch > 65535) return L;
    if (d->row_elems > ((int64_t)1 << 40)) return L;
    uint32_t cap = 64;
    while ((int64_t)cap < 2 * L.slots) cap <<= 1;
    L.cap = cap;
    L.row_bytes = (size_t)d->row_elems * (d->dtype == EGERIA_F32 ? 4 : 2);
    L.row_stride = align_up(L.row_bytes, 16);
    size_t off = 256;
    L.off_ids = off;  off += align_up((size_t)L.slots * 8, 256);
    L.off_keys = off; off += align_up((size_t)cap * 8, 256);
    L.off_vals = off; off += align_up((size_t)cap * 8, 256);
    L.off_rows = off; off += (size_t)L.slots * L.row_stride;
    L.total = off;
    L.ok = true;
    return L;
}

__device__ __forceinline__ uint32_t hash_id(int64_t id, uint32_t mask)
{
    // the 64-bit finaliser of SplitMix64 (Steele, Lea, Flood 2014)
    uint64_t x = (uint64_t)id;
    x ^= x >> 30; x *= 0xbf58476d1ce4e5b9ull;
    x ^= x >> 27; x *= 0x94d049bb133111ebull;
    x ^= x >> 31;
    return (uint32_t)x & mask;
}

struct CachePtrs {
    uint32_t *header;
    int64_t *ids;
    long long *keys;
    unsigned long long *vals;
    uint8_t *rows;
    int32_t window, batch;
    int64_t slots;
    uint32_t cap;
    size_t row_bytes, row_stride;
};

__global__ __launch_bounds__(256) void cache_init_kernel(CachePtrs c)
{
    const int64_t i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, step = (int64_t)gridDim.x * blockDim.x;
    if (i0 == 0) {
        c.header[0] = kCacheMagic;
        c.header[2] = 0u;
    }
    for (int64_t i = i0; i < c.slots; i += step) c.ids[i] = kEmptyKey;
    for (int64_t i = i0; i < c.cap; i += step) {
        c.keys[i] = kEmptyKey;
        c.vals[i] = 0ull;
    }
}

// One row, or one 32 KiB chunk of it, per workgroup: blockIdx.y = row, blockIdx.x = chunk.
template <int VEC>
__device__ __forceinline__ void copy_chunk(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst, size_t row_bytes)
{
    const size_t b0 = (size_t)blockIdx.x * kChunkBytes;
    const size_t b1 = b0 + kChunkBytes < row_bytes ? b0 + kChunkBytes : row_bytes;
    if (VEC == 16) {
        // four 16-byte loads in flight per thread
        size_t o = b0 + (size_t)threadIdx.x * 16;
        for (; o + 3 * kCopyThreads * 16 < b1; o += 4 * kCopyThreads * 16) {
            const uint4 v0 = *(const uint4 *)(src + o), v1 = *(const uint4 *)(src + o + kCopyThreads * 16);
            const uint4 v2 = *(const uint4 *)(src + o + 2 * kCopyThreads * 16);
            const uint4 v3 = *(const uint4 *)(src + o + 3 * kCopyThreads * 16);
            *(uint4 *)(dst + o) = v0;
            *(uint4 *)(dst + o + kCopyThreads * 16) = v1;
            *(uint4 *)(dst + o + 2 * kCopyThreads * 16) = v2;
            *(uint4 *)(dst + o + 3 * kCopyThreads * 16) = v3;
        }
        for (; o < b1; o += kCopyThreads * 16) *(uint4 *)(dst + o) = *(const uint4 *)(src + o);
    } else if (VEC == 4) {
        for (size_t o = b0 + (size_t)threadIdx.x * 4; o < b1; o += kCopyThreads * 4)
            *(uint32_t *)(dst + o) = *(const uint32_t *)(src + o);
    } else {
        for (size_t o = b0 + (size_t)threadIdx.x * 2; o < b1; o += kCopyThreads * 2)
            *(uint16_t *)(dst + o) = *(const uint16_t *)(src + o);
    }
}

template <int VEC>
__global__ __launch_bounds__(kCopyThreads) void cache_scatter_kernel(CachePtrs c, const uint8_t *__restrict__ rows)
{
    const uint32_t t = c.header[2];                               // number of this put
    const int64_t slot = (int64_t)(t % (uint32_t)c.window) * c.batch + blockIdx.y;
    copy_chunk<VEC>(rows + (size_t)blockIdx.y * c.row_bytes, c.rows + (size_t)slot * c.row_stride, c.row_bytes);
}

// One workgroup: record the put's ids, rebuild the table, advance the counter.
__global__ __launch_bounds__(1024) void cache_index_kernel(CachePtrs c, const int64_t *__restrict__ ids, int n)
{
    const uint32_t t = c.header[2];
    const int g_now = (int)(t % (uint32_t)c.window);
    for (int i = threadIdx.x; i < c.batch; i += blockDim.x)
        c.ids[(int64_t)g_now * c.batch + i] = i < n ? ids[i] : kEmptyKey;
    for (uint32_t i = threadIdx.x; i < c.cap; i += blockDim.x) {
        c.keys[i] = kEmptyKey;
        c.vals[i] = 0ull;
    }
    __syncthreads();
    const uint32_t mask = c.cap - 1;
    for (int64_t s = threadIdx.x; s < c.slots; s += blockDim.x) {
        const int64_t id = c.ids[s];
        if (id < 0) continue;
        const int g = (int)(s / c.batch);
        const int age = (g_now - g + c.window) % c.window;        // 0 = the mini-batch being put in
        const unsigned long long val = ((unsigned long long)(c.window - age) << 32) | (unsigned long long)s;
        uint32_t h = hash_id(id, mask);
        for (uint32_t probe = 0; probe < c.cap; ++probe) {         // load factor <= 1/2: a free entry always exists
            const long long k = atomicCAS((unsigned long long *)&c.keys[h], (unsigned long long)kEmptyKey,
                                          (unsigned long long)id);
            if (k == kEmptyKey || k == id) {
                atomicMax(&c.vals[h], val);
                break;
            }
            h = (h + 1) & mask;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) c.header[2] = t + 1u;
}

template <int VEC>
__global__ __launch_bounds__(kCopyThreads) void cache_gather_kernel(CachePtrs c, const int64_t *__restrict__ ids,
                                                                    uint8_t *__restrict__ out,
                                                                    uint8_t *__restrict__ hit)
{
    const int64_t row = blockIdx.y;
    const int64_t id = ids[row];
    // every thread probes (the same entries: broadcast loads), so the result is uniform without a barrier
    int64_t slot = -1;
    if (id >= 0) {
        const uint32_t mask = c.cap - 1;
        uint32_t h = hash_id(id, mask);
        for (uint32_t probe = 0; probe < c.cap; ++probe) {
            const long long k = c.keys[h];
            if (k == kEmptyKey) break;
            if (k == id) {
                slot = (int64_t)(c.vals[h] & 0xffffffffull);
                break;
            }
            h = (h + 1) & mask;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) hit[row] = slot >= 0 ? 1 : 0;
    if (slot < 0) return;
    copy_chunk<VEC>(c.rows + (size_t)slot * c.row_stride, out + (size_t)row * c.row_bytes, c.row_bytes);
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

CachePtrs make_ptrs(const egeria_cache_desc *d, const CacheLayout &L, void *cache)
{
    char *b = (char *)cache;
    CachePtrs c;
    c.header = (uint32_t *)b;
    c.ids = (int64_t *)(b + L.off_ids);
    c.keys = (long long *)(b + L.off_keys);
    c.vals = (unsigned long long *)(b + L.off_vals);
    c.rows = (uint8_t *)(b + L.off_rows);
    c.window = d->window;
    c.batch = d->batch;
    c.slots = L.slots;
    c.cap = L.cap;
    c.row_bytes = L.row_bytes;
    c.row_stride = L.row_stride;
    return c;
}

int copy_width(const CacheLayout &L, const void *user_rows)
{
    if (L.row_bytes % 16 == 0 && aligned16(user_rows)) return 16;
    return L.row_bytes % 4 == 0 && ((uintptr_t)user_rows & 3u) == 0 ? 4 : 2;
}

}  // namespace

}  // namespace egeria

using namespace egeria;

extern "C" {

size_t egeria_cache_bytes(const egeria_cache_desc *desc)
{
    const CacheLayout L = cache_layout(desc);
    return L.ok ? L.total : 0;
}

egeria_status egeria_cache_init(const egeria_cache_desc *desc, void *cache, size_t cache_bytes, void *stream)
{
    const CacheLayout L = cache_layout(desc);
    if (!L.ok || !cache || !aligned16(cache)) return EGERIA_ERR_INVALID_ARG;
    if (cache_bytes < L.total) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    const CachePtrs c = make_ptrs(desc, L, cache);
    int64_t blocks = ((int64_t)L.cap + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipError_t e = launch_k(EGERIA_KERNEL_NONE, cache_init_kernel, dim3((unsigned)blocks), dim3(256), 0,
                            (hipStream_t)stream, c);
    return e == hipSuccess ? EGERIA_OK : EGERIA_ERR_HIP;
}

egeria_status egeria_cache_put(const egeria_cache_desc *desc, void *cache, size_t cache_bytes, const int64_t *ids,
                               int32_t n, const void *rows, void *stream)
{
    const CacheLayout L = cache_layout(desc);
    if (!L.ok || !cache || !aligned16(cache) || n < 0 || n > desc->batch) return EGERIA_ERR_INVALID_ARG;
    if (n > 0 && (!ids || !rows || ((uintptr_t)ids & 7u) || ((uintptr_t)rows & 1u))) return EGERIA_ERR_INVALID_ARG;
    if (cache_bytes < L.total) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    const CachePtrs c = make_ptrs(desc, L, cache);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (n > 0) {
        const int64_t chunks = ((int64_t)L.row_bytes + kChunkBytes - 1) / kChunkBytes;
        if (chunks > 0x7fffffffLL) return EGERIA_ERR_UNSUPPORTED;
        const dim3 grid((unsigned)chunks, (unsigned)n), block(kCopyThreads);
        const int w = copy_width(L, rows);
        if (w == 16) e = launch_k(EGERIA_KERNEL_CACHE_COPY, cache_scatter_kernel<16>, grid, block, 0, st, c, (const uint8_t *)rows);
        else if (w == 4) e = launch_k(EGERIA_KERNEL_CACHE_COPY, cache_scatter_kernel<4>, grid, block, 0, st, c, (const uint8_t *)rows);
        else e = launch_k(EGERIA_KERNEL_CACHE_COPY, cache_scatter_kernel<2>, grid, block, 0, st, c, (const uint8_t *)rows);
        if (e != hipSuccess) return EGERIA_ERR_HIP;
    }
    e = launch_k(EGERIA_KERNEL_NONE, cache_index_kernel, dim3(1), dim3(1024), 0, st, c, ids, (int)n);
    return e == hipSuccess ? EGERIA_OK : EGERIA_ERR_HIP;
}

egeria_status egeria_cache_get(const egeria_cache_desc *desc, const void *cache, size_t cache_bytes,
                               const int64_t *ids, int64_t n, void *out, uint8_t *hit, void *stream)
{
    const CacheLayout L = cache_layout(desc);
    if (!L.ok || !cache || !aligned16(cache) || n < 0 || n > 65535) return EGERIA_ERR_INVALID_ARG;
    if (n == 0) return EGERIA_OK;
    if (!ids || !out || !hit || ((uintptr_t)ids & 7u) || ((uintptr_t)out & 1u)) return EGERIA_ERR_INVALID_ARG;
    if (cache_bytes < L.total) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    const CachePtrs c = make_ptrs(desc, L, const_cast<void *>(cache));
    const int64_t chunks = ((int64_t)L.row_bytes + kChunkBytes - 1) / kChunkBytes;
    if (chunks > 0x7fffffffLL) return EGERIA_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)chunks, (unsigned)n), block(kCopyThreads);
    hipStream_t st = (hipStream_t)stream;
    const int w = copy_width(L, out);
    hipError_t e;
    if (w == 16) e = launch_k(EGERIA_KERNEL_CACHE_COPY, cache_gather_kernel<16>, grid, block, 0, st, c, ids, (uint8_t *)out, hit);
    else if (w == 4) e = launch_k(EGERIA_KERNEL_CACHE_COPY, cache_gather_kernel<4>, grid, block, 0, st, c, ids, (uint8_t *)out, hit);
    else e = launch_k(EGERIA_KERNEL_CACHE_COPY, cache_gather_kernel<2>, grid, block, 0, st, c, ids, (uint8_t *)out, hit);
    return e == hipSuccess ? EGERIA_OK : EGERIA_ERR_HIP;
}

}  // extern "C"
