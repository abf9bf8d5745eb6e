// Batched launches: B buckets that need not be contiguous in memory, processed by ONE kernel launch
// (Section 3.1 "Bucketing": a training run hands over its buckets one by one, each too small to fill the chip).
//
// A batched entry point writes a table into the caller's workspace and launches the ordinary chunk kernel over the
// concatenation of all buckets' chunks; a workgroup finds its bucket by a binary search over the buckets' first
// unit indices (B + 1 uniform 8-byte loads at most log2(B) deep, served by the scalar cache).  The table travels to
// the device as kernel arguments of small upload launches: no host-to-device copy, no synchronisation, and the host
// arrays may be reused as soon as the call returns.
//
// Table layout (8-byte words):  first_unit[0..B]  (first_unit[B] = units in the launch), padded to 16 bytes, then B
// entries of `entry_words` words each (layout per entry point, see the kernels).
#pragma once
#include <vector>

#include "common.hpp"

namespace bagua {

struct BatchView {
    const uint64_t* first_unit;  // [B + 1]
    const uint64_t* entries;     // [B][entry_words]
    uint32_t B;
    uint32_t entry_words;
};

inline size_t batch_first_words(size_t B) { return (B + 1 + 1) & ~static_cast<size_t>(1); }  // 16-byte multiple
inline size_t batch_table_words(size_t B, size_t entry_words) { return batch_first_words(B) + B * entry_words; }
// Words per entry that bagua_batch_workspace_bytes(B, k) provides for.
inline size_t batch_entry_words_for(int k) { return 6 + 2 * static_cast<size_t>(k > 0 ? k : 0); }

inline BatchView batch_view(const void* workspace, size_t B, size_t entry_words)
{
    const uint64_t* w = static_cast<const uint64_t*>(workspace);
    return BatchView{w, w + batch_first_words(B), static_cast<uint32_t>(B), static_cast<uint32_t>(entry_words)};
}

// A device pointer read from the table.  The table holds integers; the cast goes through the global address space so
// that accesses through the result compile to global memory instructions.  Without it the compiler has to assume a
// generic ("flat") pointer: flat loads and stores count against both wait counters, cannot be kept in flight past LDS
// or scalar-memory waits, and made the batched server steps run at 0.46 of peak where the same data through
// kernel-argument pointers ran at 0.74.
template <typename T>
__device__ __forceinline__ T* table_ptr(uint64_t v)
{
    typedef __attribute__((address_space(1))) T* global_ptr;
    return (T*)reinterpret_cast<global_ptr>(v);
}

// Bucket that owns unit g: the largest b with first_unit[b] <= g.  Wave-uniform.
__device__ __forceinline__ uint32_t batch_find(const BatchView& bv, uint64_t g)
{
    uint32_t lo = 0, hi = bv.B;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (bv.first_unit[mid] <= g) lo = mid;
        else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------- table upload through kernel arguments
constexpr int kUploadWords = 448;  // 3584 bytes of payload per upload launch (kernel arguments are limited to 4 KiB)
struct UploadBlob {
    uint64_t w[kUploadWords];
};
__global__ void k_upload_words(UploadBlob blob, uint32_t words, uint64_t* __restrict__ dst);

// Enqueues the launches that write `words` 8-byte words from host memory to device memory at dst.
int batch_upload(const uint64_t* host, size_t words, uint64_t* dst, hipStream_t stream);

// Aliasing rule of a batched call: as RangeCheck, for any number of ranges.
struct RangeList {
    struct Item {
        uintptr_t lo, hi;
        bool written;
    };
    std::vector<Item> item;
    void add(const void* p, size_t bytes, bool written)
    {
        if (!p || bytes == 0) return;
        const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
        item.push_back(Item{lo, lo + bytes, written});
    }
    void writes(const void* p, size_t bytes) { add(p, bytes, true); }
    void reads(const void* p, size_t bytes) { add(p, bytes, false); }
    bool disjoint()
    {
        std::sort(item.begin(), item.end(), [](const Item& a, const Item& b) { return a.lo < b.lo; });
        uintptr_t end_any = 0, end_written = 0;
        for (const Item& r : item) {
            if (r.lo < (r.written ? end_any : end_written)) return false;
            if (r.hi > end_any) end_any = r.hi;
            if (r.written && r.hi > end_written) end_written = r.hi;
        }
        return true;
    }
};

}  // namespace bagua
