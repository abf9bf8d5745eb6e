// Batched launches: B buckets that need not be contiguous in memory, processed by ONE kernel launch
// (Section 3.1 "Bucketing": a training run hands over its buckets one by one, each too small to fill the chip).
//
// A batched entry point writes a table into the caller's workspace and launches the ordinary chunk kernel over the
// concatenation of all buckets' chunks; a workgroup finds its bucket from the buckets' first unit indices through a
// small lookup table (two or three dependent uniform loads, served by the scalar cache).  The table travels to
// the device as kernel arguments of small upload launches: no host-to-device copy, no synchronisation, and the host
// arrays may be reused as soon as the call returns.
//
// Table layout (8-byte words):  first_unit[0..B]  (first_unit[B] = units in the launch), padded to 16 bytes, then B
// entries of `entry_words` words each (layout per entry point, see the kernels), then a unit -> bucket lookup table of
// 16..1024 32-bit entries (see batch_find).
#pragma once
#include <vector>

#include "common.hpp"

namespace bagua {

struct BatchView {
    const uint64_t* first_unit;  // [B + 1]
    const uint64_t* entries;     // [B][entry_words]
    const uint32_t* lut;         // [lut entries]: lut[i] = bucket that owns unit i << shift
    uint32_t B;
    uint32_t entry_words;
    uint32_t shift;
};

inline size_t batch_first_words(size_t B) { return (B + 1 + 1) & ~static_cast<size_t>(1); }  // 16-byte multiple
// Entries of the unit -> bucket lookup table: a power of two, about four per bucket, 16..1024.
inline size_t batch_lut_entries(size_t B)
{
    size_t L = 16;
    while (L < 4 * B && L < 1024) L *= 2;
    return L;
}
inline size_t batch_lut_words(size_t B) { return batch_lut_entries(B) / 2; }   // 32-bit entries in 64-bit words
inline size_t batch_table_words(size_t B, size_t entry_words)
{
    return batch_first_words(B) + B * entry_words + batch_lut_words(B);
}
// Words per entry that bagua_batch_workspace_bytes(B, k) provides for.
inline size_t batch_entry_words_for(int k) { return 6 + 2 * static_cast<size_t>(k > 0 ? k : 0); }
// Smallest shift with (total_units - 1) >> shift < lut entries.
inline uint32_t batch_lut_shift(size_t B, size_t total_units)
{
    const size_t L = batch_lut_entries(B);
    uint32_t s = 0;
    while (total_units > 0 && ((total_units - 1) >> s) >= L) ++s;
    return s;
}

inline BatchView batch_view(const void* workspace, size_t B, size_t entry_words, size_t total_units)
{
    const uint64_t* w = static_cast<const uint64_t*>(workspace);
    const uint64_t* entries = w + batch_first_words(B);
    return BatchView{w, entries, reinterpret_cast<const uint32_t*>(entries + B * entry_words), static_cast<uint32_t>(B),
                     static_cast<uint32_t>(entry_words), batch_lut_shift(B, total_units)};
}

// Host side: fills the lookup table at the end of `table` (whose first_unit[0..B] are already set).
inline void batch_fill_lut(uint64_t* table, size_t B, size_t entry_words)
{
    const size_t total = table[B];
    const uint32_t shift = batch_lut_shift(B, total);
    uint32_t* lut = reinterpret_cast<uint32_t*>(table + batch_first_words(B) + B * entry_words);
    size_t b = 0;
    for (size_t i = 0; i < batch_lut_entries(B); ++i) {
        const uint64_t u = static_cast<uint64_t>(i) << shift;
        while (b + 1 < B && table[b + 1] <= u) ++b;       // the largest b with first_unit[b] <= u (buckets are non-empty)
        lut[i] = static_cast<uint32_t>(b);
    }
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

// Bucket that owns unit g: the largest b with first_unit[b] <= g.  Wave-uniform.  The lookup table gives the bucket of
// the unit at the start of g's stride; a few steps forward (none when buckets are longer than the stride) reach g's
// own: two or three dependent scalar loads instead of log2(B) + 1, which matters for the kernels whose workgroups are
// small (a 2048-element chunk of the sign codec).
__host__ __device__ __forceinline__ uint32_t batch_find(const BatchView& bv, uint64_t g)
{
    uint32_t b = bv.lut[g >> bv.shift];
    while (bv.first_unit[b + 1] <= g) ++b;     // first_unit[B] = all units > g: stops at b <= B - 1
    return b;
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
