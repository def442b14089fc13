// Geometry of the work (wave tiles, supertiles, scan chunks, radix digits) and the descriptor
// tables the host uploads.  Part of scalecom.hip's single translation unit.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "scalecom.h"

namespace {

constexpr int kLanes = 64;                       // wavefront width on CDNA
constexpr int kVec = 4;                          // elements per lane per access (16 B of fp32)
constexpr int kWaveTile = kLanes * kVec;         // 256 consecutive positions handled by one wave
constexpr int kTilesPerSuper = 32;               // wave tiles per supertile
constexpr int kSuper = kWaveTile * kTilesPerSuper;   // 8192 positions
constexpr int kBlock = 256;                      // threads per block in the streaming kernels
constexpr int kWaves = kBlock / kLanes;          // 4
constexpr int kUpdateBlocksPerSuper = kTilesPerSuper / kWaves;   // update: one wave tile per wave
constexpr int kUpdateLearnersPerLaunch = 8;      // update: learners streamed side by side (one per XCD)
constexpr int kChunk = 1024;                     // supertiles per chunk of the prefix scan
constexpr int kOwnScanMaxSt = 10240;             // up to this many supertiles k_slots scans the supertile totals itself
constexpr int kManySupertiles = 32768;           // beyond: one wave per supertile means several rounds of waves on the chip
constexpr int kSlotsBatch = 4;                   // supertiles per wave of the slot kernel then
constexpr int kSlotsOwnScanBlock = 1024;         // threads of its blocks then (16 waves = 16 supertiles)

constexpr int kBits0 = 12, kBits1 = 12, kBits2 = 7;          // 31-bit key = 12 + 12 + 7
constexpr int kBins0 = 1 << kBits0, kBins1 = 1 << kBits1, kBins2 = 1 << kBits2;
constexpr int kHistGridMax = 2048;              // blocks of the search levels' kernels, plus at most one per tensor
constexpr int kCandSlice = 512;                  // candidate slots per supertile (1/16 of its positions)
constexpr uint32_t kModeFull = 0, kModeCand = 1;

struct SegDesc {          // one per tensor (segment of the flat vector)
    int32_t begin, end;   // positions [begin, end)
    int32_t k;            // size of this segment's index set
    int32_t out_base;     // first output slot of this segment
    int32_t st_first;     // first supertile
    int32_t st_count;     // number of supertiles
    int32_t chunk_first;  // first scan chunk
    int32_t chunk_count;
    int32_t sel_chunk;    // chunk-wise selector: elements per chunk of this segment (0 in exact mode)
    int32_t pad;
};

struct StDesc {           // one per supertile; carries what the streaming kernels need of its segment
    int32_t seg;
    int32_t a0;           // first position, a multiple of 4 (may lie up to 3 before begin)
    int32_t begin, end;   // the segment's positions [begin, end)
    int32_t slot_end;     // one past the segment's last output slot
    int32_t pad[3];
};

struct HistBlock {        // one block of the kernels of the search levels: consecutive supertiles of ONE segment
    int32_t seg;
    int32_t st_lo, st_hi; // supertiles [st_lo, st_hi)
    int32_t owner;        // 1: holds the segment's first supertile; that block passes the segment's state on
    int32_t a0;           // first position of supertile st_lo
    int32_t begin, end;   // the segment's positions [begin, end)
    int32_t pad;
};

struct ChunkDesc {        // one per scan chunk: up to kChunk consecutive supertiles of one segment
    int32_t seg;
    int32_t st_begin;
    int32_t st_count;
    int32_t pad;
};

struct SegState {         // selection state of one segment after a level; every field is rewritten by k_level0 each step
    uint32_t prefix;      // key bits fixed so far (level 0: 12 bits, level 1: 24 bits)
    uint32_t k_rem;       // members still to be found inside the current bucket
    uint32_t T;           // threshold key (after level 2)
    uint32_t q;           // number of keys == T that are members (the lowest positions)
    uint32_t done;        // 1: empty index set, nothing to refine
    uint32_t mode;        // kModeCand: levels 1, 2 and the tile counts work on the candidate list
    uint32_t collected;   // 1: the candidate list was filled by the predicted single pass
    uint32_t l1_done;     // 1: levels 0 and 1 are known from the counts of the predicted pass
    uint32_t pending;     // 1: the last histogram was counted but not searched yet (the next kernel's blocks do that)
    uint32_t l2_done;     // 1: T and q are final already, and the tile counts and masks are written (a segment of
                          //    one supertile is searched and counted by one block)
    uint32_t w_next;      // width of the next step's range, for the kernel that ends a search without prediction
    uint32_t l1_bits;     // key bits that level 1 resolves: 12, or the 1..5 bits that a wide range's counts left open
};
static_assert(sizeof(SegState) == 48, "twelve words, no padding to carry along in copies");
// One state per 128-byte line: blocks that work on different segments run on different XCDs, and
// four states in one line made the per-segment searches three times slower with 200 segments.
// (The stride is kept out of the struct so that copies of a state stay in registers.)
constexpr size_t kStateStride = 128;
__host__ __device__ inline SegState& state_at(SegState* base, size_t seg)
{
    return *reinterpret_cast<SegState*>(reinterpret_cast<char*>(base) + seg * kStateStride);
}
__host__ __device__ inline const SegState& state_at(const SegState* base, size_t seg)
{
    return *reinterpret_cast<const SegState*>(reinterpret_cast<const char*>(base) + seg * kStateStride);
}

// The predicted pass works on a RANGE of keys around the threshold it expects: 2^w keys, counted in
// bins.  Up to w = 19 a bin is 128 keys (at most 4096 bins; a hit then fixes the key's top 24 bits)
// and every listed key costs one atomic in memory.  Those are carried out at the memory side, one
// by one: half a million of them double the time of the pass.  So a wider range has 64 bins only,
// counted in LDS first (64 atomics in memory per block at most); a hit then leaves w - 13 more bits
// to level 1, which counts them on the listed keys of that one bin.  The range starts at a multiple
// of the bin width, and the counts exist in as many slotted copies as fit into 4096 words.
// w follows the density of keys around the threshold and how far the threshold moves from step to
// step: with error feedback the magnitudes pile up just below it (after some hundred steps a
// twelve-bit bucket around the threshold holds 7 % of all elements), so a fixed range would come to
// hold far more keys than the index set has members; while the memories are still small the
// threshold follows every batch's gradient norm, and a range of +-3 % would miss it every other step.
constexpr int kSpecBitsMax = kBits1 + kBits2;    // 19: the widest range with bins of 128 keys (+-3 % of the threshold)
constexpr int kSpecBitsWide = kSpecBitsMax + 5;  // 24: the widest range, 2^24 keys (two binades)
constexpr int kSpecBitsMin = kBits2 + 3;         // 10: 2^10 keys, 8 counts
constexpr int kSpecWideBinsLog = 6;              // a range wider than 2^19 keys has 64 bins
// log2 of the keys per bin of a range of 2^w keys
__host__ __device__ constexpr uint32_t spec_bin_shift(uint32_t w)
{
    return w > static_cast<uint32_t>(kSpecBitsMax) ? w - kSpecWideBinsLog : static_cast<uint32_t>(kBits2);
}
static_assert(kSpecBitsWide - kSpecWideBinsLog - kBits2 <= kBits1, "level 1 resolves at most twelve bits");
// A width as read from memory, forced into the range the kernels' index arithmetic is made for.
__host__ __device__ constexpr uint32_t clamp_width(uint32_t w)
{
    return w < static_cast<uint32_t>(kSpecBitsMin) ? static_cast<uint32_t>(kSpecBitsMin)
                                                  : (w > static_cast<uint32_t>(kSpecBitsWide) ? static_cast<uint32_t>(kSpecBitsWide) : w);
}
// The prediction kept per segment between steps, and the one a step works with.
constexpr int kPredWords = 8;                    // [0] 1 if there is one, [1] top 24 bits of the last threshold, [2] w,
                                                 // [3] steps in a row in which the threshold fell into the range's middle half,
                                                 // [4] (float) by how much the last leader's threshold grew since its previous turn
constexpr uint32_t kCalmSteps = 8;               // so many of those before the range is made narrower
// Counts of the predicted pass, per segment: [0] keys above the range, [1] keys inside it.
// Blocks add into one of kPartSlots copies (same-address atomics from thousands of blocks would
// serialise); readers sum the copies.
constexpr int kPartSlots = 64;
constexpr int kPartWords = 8;

// What the selections of a context ran into, counted on the device (64-bit words), per (step, tensor)
// pair with a non-empty index set and more than one supertile.  Only events are counted.
constexpr int kStatWords = 8;
enum : int {
    kStatMissed = 0,        // had a prediction and its range did not hold the threshold: two more leader passes
    kStatNoPrediction = 1,  // had no prediction (first step with a layout, or the step after a miss)
    kStatFullMode = 2,      // the threshold bucket did not fit the candidate list: refinement by full leader passes
    kStatWideRange = 3,     // hit with a range wider than 2^19 keys: one more pass over the listed keys
    kStatSteps = 4          // selections enqueued (one per step, whatever the number of tensors)
};

struct LearnerPtrs {
    float* mem[SCALECOM_MAX_LEARNERS];
    const void* grad[SCALECOM_MAX_LEARNERS];
};

}  // namespace
