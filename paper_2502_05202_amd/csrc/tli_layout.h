// tli_layout.h -- Sizes and table formats that the host-side map builder and the kernels must agree on: how a logit row is cut into
// chunks, and how the residual scan's tables (staging table, pair lists) are laid out.  Plain C++ (no HIP), so
// that the builder also compiles on its own for a sanitizer build on the CPU.
#pragma once

#include <cstdint>

#include "tli.h"

namespace tli_layout {

constexpr int kWave = 64;   // lanes of a wavefront
constexpr int kLoads = 4;   // 16-byte loads a lane makes per chunk: a chunk is kWave * kLoads vectors
constexpr int kMaxVocab = 1 << 30;  // vocabulary sizes the chunk arithmetic (int32 ids, counts rounded up to whole chunks) is written for
inline bool vocab_ok(int V) { return V >= 1 && V <= kMaxVocab; }

template <int DT> struct Traits;
template <> struct Traits<TLI_F32> {
    static constexpr int EPV = 4;  // elements per 16-byte vector
    static constexpr int ESZ = 4;
};
template <> struct Traits<TLI_BF16> {
    static constexpr int EPV = 8;
    static constexpr int ESZ = 2;
};
template <int DT> constexpr int chunk_elems() { return kWave * kLoads * Traits<DT>::EPV; }

// ---- the residual scan's workgroup: LDS plan and list formats
constexpr int kScanWG = 1024;
constexpr int kScanWaves = kScanWG / kWave;
constexpr int kSlotBytes = kWave * kLoads * 16;  // one chunk
constexpr int kTrashBytes = kWave * 4;           // LDS [0, 256): a word per lane for the elements a lane does not keep
constexpr int kPartBytes = 92 * 1024;            // then the staged drafter logits of a part, the last 16 bytes of the
                                                 // area hold the -inf logit that padding entries point at
constexpr int kScanLds = kPartBytes + kScanWaves * kSlotBytes;  // then one chunk slot per wave
constexpr int kPairG = 2 * kWave;      // entries in a group of a chunk's pair list: two per lane
constexpr int kPairU = 6;              // groups fetched with a chunk (more: late loop)
constexpr int kPairShift = 16;         // entry = byte offset in chunk (< 4096) | index of the staged logit << 16
constexpr int kMaxPartChunks = kWave * kScanWaves;  // a wave keeps a lane per chunk it handles
static_assert(kScanLds <= 160 * 1024, "LDS of one CU");
// pairs a part may hold, and the index of the -inf logit
template <int DT> constexpr int part_cap() { return (kPartBytes - kTrashBytes - 16) / Traits<DT>::ESZ; }
template <int DT> constexpr int dummy_index() { return part_cap<DT>(); }
static_assert(dummy_index<TLI_BF16>() < (1 << 16) && dummy_index<TLI_F32>() < (1 << 16), "16-bit staged index");

// two 32-bit words, laid out as the device's int2 / uint2
struct Int2 { int32_t x, y; };
struct UInt2 { uint32_t x, y; };

}  // namespace tli_layout
