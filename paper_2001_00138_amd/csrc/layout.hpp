// Host-side description of an encoded layer: the paper's FKW arrays (section 5.3)
// plus the per-filter-group, channel-major layouts that the tiled kernels read.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/patdnn.h"

namespace patdnn {

// ---------------------------------------------------------------------------
// The 56 four-entry patterns that keep the centre (section 4.1), numbered by the
// lexicographic order of their three non-centre positions.  Tiled kernels carry one
// straight-line body per entry of this table, so a layer may use any subset of it.
// ---------------------------------------------------------------------------
constexpr int kUniverse = 56;

constexpr uint16_t universe_mask(int idx)
{
    const int others[8] = {0, 1, 2, 3, 5, 6, 7, 8};
    int k = 0;
    for (int a = 0; a < 8; ++a)
        for (int b = a + 1; b < 8; ++b)
            for (int c = b + 1; c < 8; ++c) {
                if (k == idx)
                    return (uint16_t)((1u << 4) | (1u << others[a]) | (1u << others[b]) |
                                      (1u << others[c]));
                ++k;
            }
    return 0;
}

int universe_index(uint16_t mask);   // -1 if the mask is not one of the 56

// ---------------------------------------------------------------------------
// FKW (section 5.3): filter-major, kernels of a filter ordered by pattern.
// ---------------------------------------------------------------------------
struct Fkw {
    int32_t taps = 4;                 // weights per stored kernel (9 for a dense layer)
    int32_t num_patterns = 0;         // P (1 for a dense layer)
    std::vector<int32_t> offset;      // [c_out+1]
    std::vector<int32_t> reorder;     // [c_out]   stored filter -> original output channel
    std::vector<int32_t> index;       // [kept]    input channel
    std::vector<int32_t> stride;      // [c_out][P+1]
    std::vector<float> weight;        // [kept][taps]
    std::vector<uint16_t> masks;      // [P] pattern masks (0x1FF for dense)
};

// ---------------------------------------------------------------------------
// Tiled layout for one kernel variant.  G filters share a filter group (one wavefront);
// which ones is chosen so that the groups have equal work in every chunk of input
// channels (encoder.cpp).  Sparse layers: per filter group and per chunk of `ck` input
// channels, a sequence of fixed-size steps (kStepDwords = 24 dwords) that the kernel's
// interpreter executes in order.  All kernels of a step read ONE input channel.
// Kernels are listed channel-major so that one window load serves every kernel of the
// group on that channel (filter-level load-redundancy elimination, section 5.4), and
// by pattern inside a channel (kernel reorder, section 5.2).  A kernel's code block
// sits at table_off + ((window set*G + slot)*56 + universe index) * block_bytes from
// the code base; control block k at k * ctrl_bytes.
//
// Call dispatch, one step:
//   dwords  0..15  the four weights of up to 4 kernels
//   dwords 16..19  per kernel, the offset of its code block; the first unused entry
//                  holds the "step done" control block (kCtrlDoneA / B for an even / odd
//                  step of the chunk)
//   dword  20      control block run when the step starts: load a window into register
//                  set A or B, nothing, or the end of the chunk's stream
//   dword  21      LDS byte offset, inside the staged chunk, of the channel that block loads
//   dwords 22..23  zero
// Threaded dispatch, one step:
//   dwords 6i..6i+5 (i = 0..2)  record i: four weights, offset of its code block, zero
//   The record after the last kernel holds only an offset: the control block that enters
//   the NEXT step (3*set + action: set = 0 / 1 for an even / odd step of the chunk,
//   action 0 nothing, 1 / 2 load a window into register set 0 / 1), or kThreadedEnd.
//   After three kernels that offset is dword 22.
//   dword  23      LDS byte offset of the channel whose window the step's OWN entry block loads
//   The control block that enters the first step of a chunk is stored beside the chunk's
//   first-step index (bits 28..31 of chunk_ptr).
// With two sets of window registers the window loaded when a step starts is the one the
// NEXT channel's kernels use; the stream then opens with a step that only loads the first.
// ---------------------------------------------------------------------------
constexpr int kStepDwords = 24;
// control blocks of call dispatch, in code order
enum { kCtrlLoadA = 0, kCtrlLoadB = 1, kCtrlNone = 2, kCtrlDoneA = 3, kCtrlDoneB = 4, kCtrlEnd = 5 };
// threaded dispatch
constexpr int kThreadedEnd = 6, kThreadedRecDwords = 6, kThreadedTermFull = 22, kThreadedWoff = 23;
// chunk_ptr packing
constexpr uint32_t kChunkStepMask = 0x0FFFFFFFu;
constexpr int kChunkEntryShift = 28;

struct TiledParams {
    int32_t G = 0;
    int32_t ck = 0;                      // channels per chunk (sparse only)
    uint32_t block_bytes = 0, table_off = 0, ctrl_bytes = 0, records = 0;
    bool double_window = false, threaded = false;
    uint32_t channel_bytes = 0;          // LDS bytes of one staged channel
};

struct Tiled {
    int32_t G = 0;
    int32_t num_groups = 0;
    int32_t ck = 0, num_chunks = 0;
    bool dense = false;
    bool overflow = false;               // more steps than chunk_ptr can address
    std::vector<int32_t> slot_channel;   // [num_groups*G] original output channel, -1 = empty slot
    std::vector<int64_t> group_kernels;  // [num_groups] kept kernels per group
    // sparse layers
    std::vector<uint32_t> chunk_ptr;     // [num_groups][num_chunks] first step of the chunk | entry block << 28
    std::vector<uint32_t> steps;         // [steps + 1][kStepDwords] (weights as bit patterns)
    // dense layers
    std::vector<float> w9;               // [num_groups][c_in][G][9]
    size_t bytes() const
    {
        return 4 * (slot_channel.size() + chunk_ptr.size() + steps.size() + w9.size());
    }
};

struct LayerHost {
    patdnn_layer_desc_t desc{};          // pattern_masks pointer is not kept; see fkw.masks
    bool depthwise = false;
    bool dense = false;
    bool all_in_universe = true;         // every used mask is one of the 56
    int64_t kept = 0;
    Fkw fkw;
    std::vector<uint8_t> universe_of_pattern;  // [P] universe index per pattern id (255 = none)
};

// Validation + FKR + FKW.  Returns PATDNN_OK or an error with `err` filled.
patdnn_status_t build_fkw(const patdnn_layer_desc_t& d, const float* w, const uint8_t* ids,
                          const uint8_t* mask, LayerHost& out, std::string& err);

// Filter-group layout of one variant, derived from the FKW arrays.
void build_tiled(const LayerHost& L, const TiledParams& p, Tiled& out);

// Inverse of build_fkw from the five arrays (any output may be null).
void decode_fkw(const LayerHost& L, const Fkw& f, float* w, uint8_t* ids, uint8_t* mask);

}  // namespace patdnn
