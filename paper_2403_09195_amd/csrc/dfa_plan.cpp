#include "dfa_plan.h"

#include <algorithm>
#include <array>
#include <cmath>
#include <map>
#include <numeric>

namespace dfa {

namespace {

int64_t steps_of(const std::vector<KeySeg>& segs) {
    int64_t n = 0;
    for (const KeySeg& s : segs) n += (s.count + 63) / 64;
    return n;
}

// Multiplicities of one progression's keys for the (up to kTileBlocks) row groups of a tile; 0 = the group's rows
// do not attend to these keys.
using MultVec = std::array<int32_t, kTileBlocks>;

// The multiset union of the progressions in `plain` rewritten as progressions in which every key has one
// multiplicity.  A tile of one row group has one plain progression per member branch; a tile that packs several
// row groups has the distinct progressions of all of them, and member[g] says which ones group g's rows attend
// to (bit x = plain[x]): a key's multiplicity is then a number per group.  With L the least common multiple of
// the strides, a residue class mod L is either inside or outside each progression's own class, so along one
// class the multiplicities only change where a progression starts or ends.  Classes covered by the same
// progressions are joined into coarser strides where they line up.
// Returns false (outputs untouched) when L is too large, the list would not fit a tile, or no 64-key step
// would be saved against walking the plain progressions one after the other.
bool coalesce(const std::vector<KeySeg>& plain, const std::vector<uint32_t>& member, std::vector<KeySeg>* out,
              std::vector<MultVec>* out_mult) {
    const int ns = (int)plain.size(), ng = (int)member.size();
    if (ns < 2 || ns > 32) return false;
    int64_t L = 1;
    for (const KeySeg& s : plain) {
        L = std::lcm<int64_t>(L, s.stride);
        if (L > kMaxCoalesceLcm) return false;
    }
    std::vector<int64_t> last(ns);
    for (int x = 0; x < ns; ++x) last[x] = plain[x].key0 + (int64_t)(plain[x].count - 1) * plain[x].stride;

    std::vector<uint32_t> mask_of(L, 0);
    for (int64_t rho = 0; rho < L; ++rho)
        for (int x = 0; x < ns; ++x)
            if ((rho - plain[x].key0) % plain[x].stride == 0) mask_of[rho] |= 1u << x;

    std::vector<KeySeg> segs;
    std::vector<MultVec> mult;
    std::vector<char> used(L, 0);
    for (int64_t rho0 = 0; rho0 < L; ++rho0) {
        const uint32_t mask = mask_of[rho0];
        if (used[rho0] || mask == 0) continue;
        // where the multiplicity can change along these classes
        std::vector<int64_t> cuts;
        for (int x = 0; x < ns; ++x)
            if (mask >> x & 1) {
                cuts.push_back(plain[x].key0);
                cuts.push_back(last[x] + 1);
            }
        std::sort(cuts.begin(), cuts.end());
        cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
        // the classes with this mask, as progressions (a mod g), smallest stride first
        for (int64_t g = 1; g <= L; ++g) {
            if (L % g) continue;
            for (int64_t a = 0; a < g; ++a) {
                bool all = true;
                for (int64_t rho = a; rho < L && all; rho += g) all = !used[rho] && mask_of[rho] == mask;
                if (!all) continue;
                for (int64_t rho = a; rho < L; rho += g) used[rho] = 1;
                size_t open = segs.size();                      // pieces of this (a mod g) start here
                for (size_t c = 0; c + 1 < cuts.size(); ++c) {
                    const int64_t lo = cuts[c], hi = cuts[c + 1];
                    uint32_t cover = 0;                             // progressions that hold the keys of [lo, hi) in these classes
                    for (int x = 0; x < ns; ++x)
                        if ((mask >> x & 1) && plain[x].key0 <= lo && hi - 1 <= last[x]) cover |= 1u << x;
                    if (cover == 0) continue;
                    MultVec m{};
                    for (int gi = 0; gi < ng; ++gi) m[gi] = __builtin_popcount(cover & member[gi]);
                    const int64_t key0 = lo + (((a - lo) % g) + g) % g;
                    if (key0 >= hi) continue;
                    const int32_t count = (int32_t)((hi - 1 - key0) / g + 1);
                    if (segs.size() > open && mult.back() == m &&
                        segs.back().key0 + (int64_t)segs.back().count * g == key0) {
                        segs.back().count += count;             // the progression runs on with the same multiplicity
                    } else {
                        segs.push_back(KeySeg{(int32_t)key0, (int32_t)g, count, std::log2((float)std::max(m[0], 1))});
                        mult.push_back(m);
                    }
                }
            }
        }
    }
    if ((int)segs.size() > kMaxTileSegs || steps_of(segs) >= steps_of(plain)) return false;
    // ascending first keys: consecutive steps then read neighbouring rows
    std::vector<size_t> order(segs.size());
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](size_t i, size_t j) { return segs[i].key0 < segs[j].key0; });
    out->clear();
    out_mult->clear();
    for (size_t i : order) {
        out->push_back(segs[i]);
        out_mult->push_back(mult[i]);
    }
    return true;
}

// Rows of one head that share their key lists: the same parts of the same branches keep them.
struct RowGroup {
    std::vector<int32_t> rows;
    std::vector<KeySeg> plain;        // one progression per member branch
    std::vector<int64_t> plain_id;    // which (branch, part) each one is
    std::vector<KeySeg> list;         // what a tile of these rows alone walks
    std::vector<MultVec> list_mult;   // entry 0: the multiplicity of the progression's keys
    int64_t key_lo = 0, key_hi = -1;  // first and last key of its progressions
};

int blocks_of(const RowGroup& g) { return ((int)g.rows.size() + kBlockRows - 1) / kBlockRows; }

// Key list of a tile whose rows come from the groups in `pack` (group i of the pack = entry i of the
// multiplicities): the coalesced union of their progressions where that saves steps, else the distinct
// progressions one after the other.  False when the list would not fit a tile.
bool tile_list(const std::vector<const RowGroup*>& pack, std::vector<KeySeg>* list, std::vector<MultVec>* mult) {
    std::vector<KeySeg> plain;
    std::vector<int64_t> ids;
    std::vector<uint32_t> member(pack.size(), 0);
    for (size_t gi = 0; gi < pack.size(); ++gi)
        for (size_t x = 0; x < pack[gi]->plain.size(); ++x) {
            size_t at = std::find(ids.begin(), ids.end(), pack[gi]->plain_id[x]) - ids.begin();
            if (at == ids.size()) {
                if (ids.size() == 32) return false;
                ids.push_back(pack[gi]->plain_id[x]);
                plain.push_back(pack[gi]->plain[x]);
            }
            member[gi] |= 1u << at;
        }
    if (coalesce(plain, member, list, mult)) return true;
    if ((int)plain.size() > kMaxTileSegs) return false;
    list->assign(plain.begin(), plain.end());
    mult->assign(plain.size(), MultVec{});
    for (size_t x = 0; x < plain.size(); ++x)
        for (size_t gi = 0; gi < pack.size(); ++gi) (*mult)[x][gi] = member[gi] >> x & 1;
    return true;
}

}  // namespace

int check_branches(int32_t H, int32_t N, const dfa_branch_t* br, int32_t nb, const int32_t* offsets) {
    if (nb < 1 || nb > DFA_MAX_BRANCHES) return DFA_ERR_BRANCHES;
    if (!br) return DFA_ERR_NULL;
    if (H <= 0 || N <= 0) return DFA_ERR_SHAPE;
    for (int x = 0; x < nb; ++x) {
        const int32_t w = br[x].w, r = br[x].r;
        if (r < 1 || w < 1) return DFA_ERR_SHAPE;
        if (offsets)
            for (int h = 0; h < H; ++h) {
                const int32_t o = offsets[(int64_t)x * H + h];
                if (o < 0 || o >= r) return DFA_ERR_SHAPE;
            }
    }
    return DFA_OK;
}

void build_plan(int32_t B, int32_t H, int32_t N, const dfa_branch_t* br, int32_t nb,
                const int32_t* offsets, int order_mode, const ChipShape& chip, bool pack, HostPlan* plan) {
    const int kNumXcd = std::max(chip.dies, 1);
    const int kSlotsPerDie = std::max(chip.fwd_slots_per_die(), 1);
    plan->tiles.clear();
    plan->rows.clear();
    plan->segs.clear();
    plan->seg_mult.clear();
    plan->block_mult.clear();
    plan->items.clear();
    plan->packed_tiles = false;

    std::vector<int64_t> tile_cost;   // (query, key) pairs of each tile
    // appends a key list; block_group[w] = which entry of a progression's multiplicities the rows of block w take (-1: none)
    auto add_list = [&](const std::vector<KeySeg>& list, const std::vector<MultVec>& mult, const int (&block_group)[kTileBlocks]) {
        const int32_t seg_begin = (int32_t)plan->segs.size();
        plan->segs.insert(plan->segs.end(), list.begin(), list.end());
        for (const MultVec& m : mult) {
            int32_t most = 0;
            for (int w = 0; w < kTileBlocks; ++w) {
                const int32_t mw = block_group[w] < 0 ? 0 : m[block_group[w]];
                plan->block_mult.push_back(mw);
                most = std::max(most, mw);
            }
            plan->seg_mult.push_back(most);
        }
        return seg_begin;
    };
    // heads with the same start offsets in every branch have the same rows, lists and tiles: the later one's tiles
    // are copies of the earlier one's (pointing at the same rows and progressions) under its own head number
    std::map<std::vector<int32_t>, std::pair<size_t, size_t>> tiles_of_offsets;
    for (int32_t h = 0; h < H; ++h) {
        std::vector<int32_t> head_key(nb);
        for (int x = 0; x < nb; ++x) head_key[x] = head_offset(offsets, H, x, h, br[x].r);
        const auto twin = tiles_of_offsets.find(head_key);
        if (twin != tiles_of_offsets.end()) {
            for (size_t t = twin->second.first; t < twin->second.second; ++t) {
                Tile copy = plan->tiles[t];
                copy.h = h;
                plan->tiles.push_back(copy);
                tile_cost.push_back(tile_cost[t]);
            }
            continue;
        }
        const size_t first_tile = plan->tiles.size();
        // signature of a row: for each branch the part that keeps it, or -1
        std::map<std::vector<int32_t>, RowGroup> by_sig;
        std::vector<int32_t> sig(nb);
        for (int32_t n = 0; n < N; ++n) {
            for (int x = 0; x < nb; ++x) {
                const int32_t o = head_offset(offsets, H, x, h, br[x].r);
                const int32_t part = n / br[x].w, pos = n - part * br[x].w - o;   // position inside the part
                sig[x] = (pos >= 0 && pos % br[x].r == 0) ? part : -1;
            }
            by_sig[sig].rows.push_back(n);
        }
        std::vector<RowGroup*> groups;
        for (auto& kv : by_sig) {
            const std::vector<int32_t>& s = kv.first;
            RowGroup& g = kv.second;
            for (int x = 0; x < nb; ++x) {
                if (s[x] < 0) continue;
                const int32_t o = head_offset(offsets, H, x, h, br[x].r);
                // kept keys of the part: first, first + r, ... below the end of the part (the last part
                // is shorter when w does not divide N)
                const int64_t first = (int64_t)s[x] * br[x].w + o;
                const int64_t end = std::min<int64_t>((int64_t)(s[x] + 1) * br[x].w, N);
                const int32_t count = (int32_t)((end - 1 - first) / br[x].r + 1);   // >= 1: a row of the part is kept
                g.plain.push_back(KeySeg{(int32_t)first, br[x].r, count, 0.f});
                g.plain_id.push_back((int64_t)x * ((int64_t)N + 1) + s[x]);
                const int64_t last_key = first + (int64_t)(count - 1) * br[x].r;
                if (g.key_hi < g.key_lo) {
                    g.key_lo = first;
                    g.key_hi = last_key;
                } else {
                    g.key_lo = std::min(g.key_lo, first);
                    g.key_hi = std::max(g.key_hi, last_key);
                }
            }
            // keys that several member branches keep are visited once, weighted by how many keep them
            if (!g.plain.empty()) tile_list({&g}, &g.list, &g.list_mult);
            groups.push_back(&g);
        }

        // Row groups that fill only part of a tile.  Where such groups attend to many of the same keys (rows of one
        // window of a narrow branch that differ in which wider, dilated branches also keep them), a tile takes
        // several of them, each in 32-row blocks of its own (half a wave: the unit that has its own softmax state in the
        // kernel): the tile walks the union of their lists once, and a block whose
        // rows do not attend to a progression masks its scores (multiplicity 0).  A group joins a tile when at least
        // half the steps of the shorter of the two lists are saved.
        const size_t G = groups.size();
        std::vector<char> done(G, 0);
        for (size_t i = 0; i < G; ++i) {
            if (done[i]) continue;
            done[i] = 1;
            const RowGroup& g = *groups[i];
            const bool small = pack && !g.plain.empty() && blocks_of(g) < kTileBlocks;
            std::vector<const RowGroup*> members = {&g};
            std::vector<KeySeg> list = g.list;
            std::vector<MultVec> list_mult = g.list_mult;
            int blocks = blocks_of(g);
            int64_t key_lo = g.key_lo, key_hi = g.key_hi;
            while (small && blocks < kTileBlocks) {
                int64_t best = -1, best_saved = 0;
                std::vector<KeySeg> best_list;
                std::vector<MultVec> best_mult;
                const int64_t have = steps_of(list);
                for (size_t j = i + 1; j < std::min(G, i + 1 + kPackWindow); ++j) {
                    const RowGroup& c = *groups[j];
                    if (done[j] || c.plain.empty() || blocks + blocks_of(c) > kTileBlocks) continue;
                    if (c.key_hi < key_lo || key_hi < c.key_lo) continue;      // no key in common: nothing to save
                    std::vector<const RowGroup*> trial = members;
                    trial.push_back(&c);
                    std::vector<KeySeg> tl;
                    std::vector<MultVec> tm;
                    if (!tile_list(trial, &tl, &tm)) continue;
                    const int64_t own = steps_of(c.list), saved = have + own - steps_of(tl);
                    if (saved * 2 < std::min(have, own) || saved <= best_saved) continue;
                    best = (int64_t)j;
                    best_saved = saved;
                    best_list.swap(tl);
                    best_mult.swap(tm);
                }
                if (best < 0) break;
                done[best] = 1;
                members.push_back(groups[best]);
                blocks += blocks_of(*groups[best]);
                key_lo = std::min(key_lo, groups[best]->key_lo);
                key_hi = std::max(key_hi, groups[best]->key_hi);
                list.swap(best_list);
                list_mult.swap(best_mult);
            }
            const int32_t nseg = (int32_t)list.size();
            if (members.size() == 1) {
                // tiles of one group: cut its rows into tiles that share the list; every block takes entry 0
                const int block_group[kTileBlocks] = {0, 0, 0, 0, 0, 0, 0, 0};
                const int32_t seg_begin = add_list(list, list_mult, block_group);
                int64_t keys = 0;
                for (const KeySeg& sg : list) keys += sg.count;
                for (size_t lo = 0; lo < g.rows.size(); lo += kTileRows) {
                    const int32_t cnt = (int32_t)std::min<size_t>(kTileRows, g.rows.size() - lo);
                    Tile t{h, (int32_t)plan->rows.size(), cnt, seg_begin, nseg, (int32_t)steps_of(list)};
                    plan->rows.insert(plan->rows.end(), g.rows.begin() + lo, g.rows.begin() + lo + cnt);
                    plan->tiles.push_back(t);
                    tile_cost.push_back(keys * cnt);
                }
                continue;
            }
            // one tile of several groups: each starts on a block of its own; the slots between the end of a group and
            // the next block hold ~row of the group's last row (a valid row to load, never stored)
            plan->packed_tiles = true;
            int block_group[kTileBlocks] = {-1, -1, -1, -1, -1, -1, -1, -1};
            const int32_t row_begin = (int32_t)plan->rows.size();
            int w0 = 0;
            int64_t pairs = 0;
            for (size_t gi = 0; gi < members.size(); ++gi) {
                const RowGroup& m = *members[gi];
                if (gi > 0) {
                    const int32_t filler = ~members[gi - 1]->rows.back();
                    while ((int32_t)plan->rows.size() - row_begin < w0 * kBlockRows) plan->rows.push_back(filler);
                }
                plan->rows.insert(plan->rows.end(), m.rows.begin(), m.rows.end());
                for (int w = 0; w < blocks_of(m); ++w) block_group[w0 + w] = (int)gi;
                w0 += blocks_of(m);
                for (size_t x = 0; x < list.size(); ++x)
                    pairs += (int64_t)list[x].count * (list_mult[x][gi] ? 1 : 0) * (int64_t)m.rows.size();
            }
            const int32_t seg_begin = add_list(list, list_mult, block_group);
            plan->tiles.push_back(Tile{h, row_begin, (int32_t)plan->rows.size() - row_begin, seg_begin, nseg, (int32_t)steps_of(list)});
            tile_cost.push_back(pairs);
        }
        tiles_of_offsets[head_key] = {first_tile, plan->tiles.size()};
    }

    // Launch order.  Workgroup i runs on die i mod 8, each die has its own L2, and the tiles
    // of one (b, h) read the same K/V rows: keep a (b, h) unit on one die when there are
    // enough units to balance the dies, otherwise spread single tiles.  Within a die the
    // heaviest tiles go first so the tail of the launch is made of short ones.
    const int32_t T = (int32_t)plan->tiles.size();
    std::vector<std::vector<int32_t>> tiles_of_head(H);
    std::vector<int64_t> head_cost(H, 0);
    for (int32_t t = 0; t < T; ++t) {
        tiles_of_head[plan->tiles[t].h].push_back(t);
        head_cost[plan->tiles[t].h] += tile_cost[t];
    }
    std::vector<std::vector<Item>> per_die(kNumXcd);
    std::vector<int64_t> die_cost(kNumXcd, 0);
    auto lightest = [&]() {
        return (int)(std::min_element(die_cost.begin(), die_cost.end()) - die_cost.begin());
    };
    // whole units per die when that balances the dies to within an eighth (always with 4 units per die or more);
    // every die then reads only its own units' K/V rows from memory
    const int64_t units = (int64_t)B * H;
    const bool by_unit = units >= 4 * kNumXcd ||
                         (units >= kNumXcd && ((units + kNumXcd - 1) / kNumXcd) * kNumXcd * 8 <= units * 9);
    if (by_unit) {
        for (int32_t b = 0; b < B; ++b)
            for (int32_t h = 0; h < H; ++h) {
                const int d = lightest();
                for (int32_t t : tiles_of_head[h]) per_die[d].push_back(Item{t, b, plan->tiles[t]});
                die_cost[d] += head_cost[h];
            }
    } else {
        std::vector<int32_t> order(T);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(),
                         [&](int32_t a, int32_t c) { return tile_cost[a] > tile_cost[c]; });
        for (int32_t t : order)
            for (int32_t b = 0; b < B; ++b) {
                const int d = lightest();
                per_die[d].push_back(Item{t, b, plan->tiles[t]});
                die_cost[d] += std::max<int64_t>(tile_cost[t], 1);
            }
    }
    // Order inside a die.  Mode 3 (default): unit after unit, each unit's tiles heaviest first, so
    // that the workgroups running at the same time read the same K/V rows from the die's L2 and
    // every row comes from HBM about once; only the last kTailItemsPerDie items of the die are
    // ordered heaviest first as one group, so that the launch ends on short tiles (long lists only).  Mode 2: the
    // multi-progression tiles of one unit together, the single-progression tiles of all units
    // last as filler.  Mode 1: strictly unit after unit.  Mode 0: heaviest first overall.
    size_t longest = 0;
    for (auto& v : per_die) {
        // a die with fewer than four items per workgroup slot is too short a list for mode 3's
        // unit-after-unit body to balance: it gets mode 2
        if (order_mode == 3 && v.size() < 4 * (size_t)kSlotsPerDie) order_mode = 2;
        if (order_mode == 0 || !by_unit) {
            std::stable_sort(v.begin(), v.end(), [&](const Item& a, const Item& c) {
                return tile_cost[a.tile] > tile_cost[c.tile];
            });
        } else {
            // v is unit-major already; sort each unit's run by cost, then (mode 2) move the
            // single-segment tiles behind everything else, keeping their order
            size_t lo = 0;
            while (lo < v.size()) {
                size_t hi = lo;
                while (hi < v.size() && v[hi].b == v[lo].b &&
                       plan->tiles[v[hi].tile].h == plan->tiles[v[lo].tile].h) ++hi;
                std::stable_sort(v.begin() + lo, v.begin() + hi, [&](const Item& a, const Item& c) {
                    return tile_cost[a.tile] > tile_cost[c.tile];
                });
                lo = hi;
            }
            if (order_mode == 2)
                std::stable_partition(v.begin(), v.end(),
                                      [&](const Item& a) { return plan->tiles[a.tile].nseg > 1; });
            if (order_mode == 3) {
                const size_t tail = std::min<size_t>(v.size(), kTailItemsPerDie);
                std::stable_sort(v.end() - tail, v.end(), [&](const Item& a, const Item& c) {
                    return tile_cost[a.tile] > tile_cost[c.tile];
                });
            }
        }
        longest = std::max(longest, v.size());
    }
    plan->items.reserve(longest * kNumXcd);
    for (size_t p = 0; p < longest; ++p)
        for (int d = 0; d < kNumXcd; ++d)
            plan->items.push_back(p < per_die[d].size() ? per_die[d][p] : Item{-1, 0, Tile{0, 0, 0, 0, 0, 0}});
}

void split_plan(HostPlan* plan, const ChipShape& chip) {
    plan->split_wgs.clear();
    plan->item_parts.clear();
    const int64_t slots = chip.fwd_slots(), n_items = (int64_t)plan->items.size();
    if (n_items == 0 || n_items * 2 > slots) return;
    std::vector<int32_t> parts(n_items, 0);
    int64_t total = 0;
    for (int64_t i = 0; i < n_items; ++i)
        if (plan->items[i].tile >= 0) {
            parts[i] = 1;
            ++total;
        }
    // one more share for the tile with the longest shares, as long as slots are left and the shares stay long enough
    bool any = false;
    while (total < slots) {
        int64_t best = -1;
        int32_t best_share = 0;
        for (int64_t i = 0; i < n_items; ++i) {
            if (parts[i] == 0 || parts[i] >= kMaxSplit) continue;
            const int32_t steps = plan->items[i].t.n_steps;
            if (steps / (parts[i] + 1) < kMinShareSteps) continue;
            const int32_t share = (steps + parts[i] - 1) / parts[i];
            if (share > best_share) {
                best_share = share;
                best = i;
            }
        }
        if (best < 0) break;
        ++parts[best];
        ++total;
        any = true;
    }
    if (!any) return;
    plan->item_parts.resize(n_items);
    for (int64_t i = 0; i < n_items; ++i) {
        plan->item_parts[i] = ItemParts{(int32_t)plan->split_wgs.size(), parts[i]};
        for (int32_t x = 0; x < parts[i]; ++x) plan->split_wgs.push_back(SplitWg{(int32_t)i, x | (parts[i] << 16)});
    }
}

}  // namespace dfa
