// Launch plan of the fused dilated-attention kernels: host-side construction.
//
// Query rows of one head are grouped by the set of (branch, segment) pairs that keep them
// (section 3.1, Eq. 1: a row is kept by branch (w, r) iff n mod r equals the head's start
// offset, and its keys are the kept rows of segment floor(n / w)).  Rows of one group share
// one key list per member branch, so a tile of such rows runs a single online softmax over
// the concatenated key lists - which is exactly the log-sum-exp merge of the branches.
#pragma once
#include <cstdint>
#include <vector>
#include "../../include/dfa.h"

namespace dfa {

constexpr int kTileRows = 256;   // query rows per workgroup (4 waves x 64 rows)
constexpr int kTileBlocks = 8;   // a wave's 64 rows are two blocks of 32, each with its own softmax state
constexpr int kBlockRows = 32;
constexpr int kPackWindow = 32;  // row groups (in signature order) after a group that are tried as its tile mates
constexpr int kFwdWorkgroupsPerCu = 2;   // workgroups of the bf16 forward kernel that fit one compute unit
constexpr int kTailItemsPerDie = 96;     // launch order: items at the end of a die's list that go heaviest first
constexpr int kMaxTileSegs = 32; // key progressions per tile (the kernels hold a tile's list in LDS)
constexpr int kMaxCoalesceLcm = 64;   // largest common period of a tile's dilation rates that is coalesced

// One arithmetic progression of a tile's key list: keys key0 + stride * j, j < count.  Either the
// kept keys of one segment of one branch (multiplicity 1), or, where the member branches of a
// tile keep some keys more than once, a piece of their multiset union in which every key has the
// same multiplicity m: the key is then visited once and its softmax weight multiplied by m, which
// is what visiting it m times adds up to.  log2_mult = log2(m) is added to the scaled score.
struct KeySeg {
    int32_t key0, stride, count;
    float log2_mult;
};
struct Tile {
    int32_t h;          // head
    int32_t row_begin;  // first entry in the row list
    int32_t nrows;      // 1 .. kTileRows: slots of the tile (a packed tile's list has entries < 0, see HostPlan::rows)
    int32_t seg_begin;  // first entry in the key-segment list
    int32_t nseg;       // 0 = rows kept by no branch (output 0, lse -inf)
    int32_t n_steps;    // 64-key steps of the whole list: sum of ceil(count / 64)
};
struct Item {        // one workgroup of the launch
    int32_t tile;    // -1 = padding, nothing to do
    int32_t b;       // batch index
    Tile t;          // copy of tiles[tile]: a workgroup reads what it needs to start in one load
};

// What the planner needs to know of the chip: workgroup i of a launch runs on die i mod dies (each
// die has its own L2).  The library reads both numbers from the device; the default is the MI355X.
struct ChipShape {
    int32_t dies = 8;
    int32_t cus = 256;
    int32_t fwd_slots() const { return cus * kFwdWorkgroupsPerCu; }          // forward workgroups resident at once
    int32_t fwd_slots_per_die() const { return fwd_slots() / (dies > 0 ? dies : 1); }
};

// Split launches (few workgroups, see split_plan): workgroup g of the launch walks share `part` of `nparts` of the
// 64-key steps of launch item `item` and leaves its partial result in block g of the workspace
// (kSplitBlockBytes: out [256 rows][64] in fp16, each row divided by its largest magnitude, then lse [256] and
// those row scales [256] in fp32; rows in tile order).
struct SplitWg {
    int32_t item;
    int32_t part_nparts;    // part | nparts << 16
};
struct ItemParts {          // per launch item: its workgroups are first_wg .. first_wg + nparts - 1 (nparts = 0: padding)
    int32_t first_wg;
    int32_t nparts;
};
constexpr int kSplitBlockBytes = kTileRows * (DFA_HEAD_DIM * 2 + 8);
constexpr int kMaxSplit = 4;             // most shares a tile is cut into
constexpr int kMinShareSteps = 8;        // a share of fewer 64-key steps is not worth a partial result and its merge

struct HostPlan {
    std::vector<Tile> tiles;
    // token positions, tile after tile.  A tile that packs several row groups starts each group on a 32-row block of
    // its own; the slots in between hold ~n of a row n of the group (valid to load, never stored).
    std::vector<int32_t> rows;
    std::vector<KeySeg> segs;
    std::vector<int32_t> seg_mult;   // multiplicity of each entry of segs (packed tiles: the largest of its blocks)
    std::vector<int32_t> block_mult; // [segs][kTileBlocks]: multiplicity for the rows of each 32-row block, 0 = they skip the keys
    bool packed_tiles = false;       // some tile packs several row groups (block_mult differs between blocks, filler slots)
    std::vector<Item> items;
    std::vector<SplitWg> split_wgs;      // empty: the launch is not split
    std::vector<ItemParts> item_parts;
};

// Validates the branch list (DFA_OK or a negative status).  offsets: [nb][H] or nullptr.
int check_branches(int32_t H, int32_t N, const dfa_branch_t* br, int32_t nb, const int32_t* offsets);

// Start offset of head h in branch x.
inline int32_t head_offset(const int32_t* offsets, int32_t H, int32_t x, int32_t h, int32_t r) {
    return offsets ? offsets[(int64_t)x * H + h] : h % r;
}

// Builds tiles, row lists, key segments and the launch order for B images.
// order_mode: 3 = default (see dfa_plan.cpp), 0 to 2 are alternatives kept for measurement.
// pack: row groups of fewer than eight 32-row blocks may share a tile (only the bf16 forward kernel reads such
// tiles: it takes its multiplicities per block from block_mult).
void build_plan(int32_t B, int32_t H, int32_t N, const dfa_branch_t* br, int32_t nb,
                const int32_t* offsets, int order_mode, const ChipShape& chip, bool pack, HostPlan* plan);

// Launches of the bf16 forward kernel with fewer workgroups than half the chip's slots are as long as their longest
// tile's walk.  There the walks are cut: every tile gets one workgroup, then the workgroup slots left over go one by
// one to the tile whose shares are longest (up to kMaxSplit shares, none shorter than kMinShareSteps), and a second,
// small launch merges the partial results of the tiles that were cut by their log-sum-exp weights (a tile left whole
// is written out by its one workgroup).  Launches that fill more than half the slots are left alone: cutting their
// longest walks fills every CU with two workgroups, which slows every step by more than the shorter walks save
// (two 1024^2 images: 54.7 us against 46.1 us).  Fills plan->split_wgs / item_parts, or
// leaves them empty when the launch is not to be split.
void split_plan(HostPlan* plan, const ChipShape& chip);

}  // namespace dfa
