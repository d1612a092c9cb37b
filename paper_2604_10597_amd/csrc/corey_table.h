// Bit-pattern table of a 16-bit tensor: how often each of the 65536 storage bit patterns occurs.
//
// The fixed-bin histogram of Eq. 1 needs the tensor's range before a value can be binned, which is why the paper's
// estimator makes two passes (a min/max pass, then a bin-count pass).  For 16-bit storage there is a range-free
// intermediate: count the bit patterns in ONE pass, then take range and bin counts from the table (the bin of a value
// depends on the value and the range only, so binning 65536 patterns with their multiplicities gives exactly the counts
// of binning every element).  Whoever produces or reads the tensor anyway can fill the table on the way.
//
// A workgroup of kLanes lanes keeps the whole table in LDS: 32768 words, each holding two 16-bit counters (the pattern
// of magnitude m with sign 0 in the low half, with sign 1 in the high half).  A counter uses 15 bits; bit 15 is a
// guard.  An element adds 1 to its half with a returning LDS atomic; the lane that sees its counter go from 0x7fff to
// 0x8000 takes 0x8000 off again and records the pattern in the workgroup's overflow list (one entry = 32768
// occurrences).  The workgroup meets at a barrier at least every kRoundAdds = 32768 elements: a counter starts a round
// below 0x8000 and gains at most 32768, so its half never carries into its neighbour's, sees at most one guard crossing
// per round, and is below 0x8000 again at the barrier whatever the interleaving of the lanes.  All arithmetic is integer
// and every element is counted exactly once: the table is exact and independent of scheduling.
// The pattern 0x0000 (+0.0: most of a sparse activation tensor) is counted in a word of the lane's own instead (32 bits,
// no guard needed), which keeps a wave full of zeros from queueing on one LDS address.  A lane issues the adds of a whole
// 16-byte word (8 elements) before it looks at what they returned, and it looks first at the OR of the returned words:
// a guard crossing needs bit 14 of a counter set beforehand, so when neither half of any returned word has it (the usual
// case: a workgroup sees a few dozen occurrences of a pattern) no element needs the exact test.
// At the end the workgroup writes its table as it is (128 KiB, two bytes per pattern) plus a small tail (zeros, overflow
// list) to its own slab of the caller's workspace: no global atomics, nothing to clear beforehand.
#ifndef COREY_TABLE_H
#define COREY_TABLE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "corey_range.h"

namespace corey_table {

constexpr int kLanes = 1024;            // lanes per workgroup of a kernel that fills a table (16 waves: one workgroup per compute unit)
constexpr int kWords = 32768;           // LDS words of the table
constexpr int kRoundAdds = 32768;       // most elements a workgroup may add between two barriers
constexpr int kMaxSlabs = 256;          // most workgroups that fill tables in one launch (one per compute unit)
constexpr int kMaxOver = 1024;          // overflow entries a workgroup can record: 32768 elements each, 2^25 elements per workgroup
constexpr int kParts = corey_range::kParts;

struct Head {                           // per workgroup: what its slab does not hold
    uint32_t n_over;                    // entries of the workgroup's overflow list in use
    uint32_t zeros;                     // occurrences of pattern 0x0000
};
struct Tail {                           // per workgroup: the overflow list
    uint16_t over[kMaxOver];            // patterns that crossed the guard bit (each entry stands for 32768 occurrences)
};

struct Shared {                         // LDS bookkeeping beside the table
    uint32_t n_over;
    uint16_t over[kMaxOver];
    uint32_t zeros[kLanes];             // per lane: occurrences of pattern 0x0000
};

// Layout of the caller's workspace (corey_pattern_table_workspace() bytes, 256-byte aligned).
struct Workspace {
    corey_range::RangeSlot* slots;      // [1]   range of the histogram, for the reduction kernel
    uint32_t* parts;                    // [kParts][COREY_MAX_BINS] partial histograms the binning kernel adds into
    corey_range::RangePart* rparts;     // [kMaxSlabs] partial ranges of the kernel that filled the tables
    uint32_t* nslabs;                   // [1]   slabs that kernel wrote
    Head* heads;                        // [kMaxSlabs]
    Tail* tails;                        // [kMaxSlabs]
    uint32_t* slabs;                    // [kMaxSlabs][kWords]
};

constexpr size_t kSlotsBytes = 256;
constexpr size_t kPartsBytes = (size_t)kParts * COREY_MAX_BINS * sizeof(uint32_t);
constexpr size_t kRpartsBytes = (size_t)kMaxSlabs * sizeof(corey_range::RangePart);
constexpr size_t kCountBytes = 256;
constexpr size_t kHeadsBytes = (size_t)kMaxSlabs * sizeof(Head);
constexpr size_t kTailsBytes = ((size_t)kMaxSlabs * sizeof(Tail) + 255) / 256 * 256;
constexpr size_t kSlabsBytes = (size_t)kMaxSlabs * kWords * sizeof(uint32_t);
constexpr size_t kWorkspaceBytes = kSlotsBytes + kPartsBytes + kRpartsBytes + kCountBytes + kHeadsBytes + kTailsBytes + kSlabsBytes;

inline __host__ __device__ Workspace carve(void* base)
{
    char* p = static_cast<char*>(base);
    Workspace w;
    w.slots = reinterpret_cast<corey_range::RangeSlot*>(p);
    p += kSlotsBytes;
    w.parts = reinterpret_cast<uint32_t*>(p);
    p += kPartsBytes;
    w.rparts = reinterpret_cast<corey_range::RangePart*>(p);
    p += kRpartsBytes;
    w.nslabs = reinterpret_cast<uint32_t*>(p);
    p += kCountBytes;
    w.heads = reinterpret_cast<Head*>(p);
    p += kHeadsBytes;
    w.tails = reinterpret_cast<Tail*>(p);
    p += kTailsBytes;
    w.slabs = reinterpret_cast<uint32_t*>(p);
    return w;
}

// Clear the workgroup's table and bookkeeping; also this workgroup's share of the partial histograms (the binning kernel,
// which runs after every table is written, adds into them).  Ends with a barrier.
__device__ __forceinline__ void begin(uint32_t* s_tab, Shared& sh, const Workspace& ws)
{
    typedef uint32_t word4 __attribute__((ext_vector_type(4)));
    const word4 zero = {0u, 0u, 0u, 0u};
    for (int i = threadIdx.x; i < kWords / 4; i += kLanes) reinterpret_cast<word4*>(s_tab)[i] = zero;
    if (threadIdx.x == 0) sh.n_over = 0u;
    sh.zeros[threadIdx.x] = 0u;
    for (int i = blockIdx.x * kLanes + threadIdx.x; i < kParts * COREY_MAX_BINS; i += gridDim.x * kLanes) ws.parts[i] = 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) *ws.nslabs = gridDim.x;
    __syncthreads();
}

// The exact test after an add returned `old`: did this add take the element's counter from 0x7fff to 0x8000?  Then take
// 32768 off again and record them.
__device__ __forceinline__ void settle(uint32_t* s_tab, Shared& sh, uint32_t p, uint32_t old)
{
    if (p == 0u) return;                                      // the lane's own 32-bit zero counter has no guard
    const uint32_t hi = p >> 15;
    const uint32_t cnt = (hi ? old >> 16 : old) & 0xffffu;
    if (cnt == 0x7fffu) {
        atomicAdd(&s_tab[p & 0x7fffu], 0u - ((hi ? 0x10000u : 1u) << 15));
        const uint32_t slot = atomicAdd(&sh.n_over, 1u);
        if (slot < (uint32_t)kMaxOver) sh.over[slot] = (uint16_t)p;
    }
}

// Issue the add for one element with storage bits p (0 ... 65535); returns what the counter's word held before.
__device__ __forceinline__ uint32_t add_issue(uint32_t* s_tab, Shared& sh, uint32_t p)
{
    const uint32_t inc = (p >> 15) ? 0x10000u : 1u;           // the sign bit picks the half
    uint32_t* word = (p == 0u) ? &sh.zeros[threadIdx.x] : &s_tab[p & 0x7fffu];
    return atomicAdd(word, inc);                              // returning LDS atomic
}

// Count one element.
__device__ __forceinline__ void add(uint32_t* s_tab, Shared& sh, uint32_t p)
{
    settle(s_tab, sh, p, add_issue(s_tab, sh, p));
}

// The eight elements of one 16-byte word: all adds first, then one look at the OR of what they returned.
__device__ __forceinline__ void add_word4(uint32_t* s_tab, Shared& sh, const uint32_t (&w)[4])
{
    uint32_t old[8], any = 0u;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        old[2 * k] = add_issue(s_tab, sh, w[k] & 0xffffu);
        old[2 * k + 1] = add_issue(s_tab, sh, w[k] >> 16);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) any |= old[e];
    if (any & 0x40004000u) {                                  // some counter (or a zero counter) was at 16384 or more
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            settle(s_tab, sh, w[k] & 0xffffu, old[2 * k]);
            settle(s_tab, sh, w[k] >> 16, old[2 * k + 1]);
        }
    }
}

// Write the workgroup's table, tail and partial range to its slab.  The range keys are reduced over the workgroup on the
// way (valid in thread 0 afterwards); the barriers of that reduction also see every add land before the table is read.
__device__ __forceinline__ void end(uint32_t* s_tab, Shared& sh, const Workspace& ws, uint32_t& klo, uint32_t& khi, uint32_t& knan)
{
    typedef uint32_t word4 __attribute__((ext_vector_type(4)));
    corey_range::reduce_range_keys<kLanes>(klo, khi, knan);   // holds a barrier: every add has landed
    uint32_t zeros = sh.zeros[threadIdx.x];
    for (int off = 32; off > 0; off >>= 1) zeros += (uint32_t)__shfl_xor((int)zeros, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.zeros[threadIdx.x >> 6] = zeros;      // the waves' totals (all lanes have read their own)
    __syncthreads();
    word4* slab = reinterpret_cast<word4*>(ws.slabs + (size_t)blockIdx.x * kWords);
    for (int i = threadIdx.x; i < kWords / 4; i += kLanes) slab[i] = reinterpret_cast<const word4*>(s_tab)[i];
    Tail* tail = ws.tails + blockIdx.x;
    const uint32_t n_over = sh.n_over < (uint32_t)kMaxOver ? sh.n_over : (uint32_t)kMaxOver;
    for (uint32_t i = threadIdx.x; i < n_over; i += kLanes) tail->over[i] = sh.over[i];
    if (threadIdx.x == 0) {
        uint32_t z = 0u;
        for (int w = 0; w < kLanes / 64; ++w) z += sh.zeros[w];
        Head h;
        h.n_over = n_over;
        h.zeros = z;
        ws.heads[blockIdx.x] = h;
        corey_range::RangePart rp;
        rp.lo_key = klo; rp.hi_key = khi; rp.saw_nan = knan; rp.pad = 0u;
        ws.rparts[blockIdx.x] = rp;
    }
}

}  // namespace corey_table
#endif
