// C ABI of the dilated flash attention library: argument checks, launch-plan cache, launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <list>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/dfa.h"
#include "../../include/dfa_bench.h"
#include "dfa_device.h"
#include "dfa_plan.h"

// Scratch memory of dfa_forward_static, the entry point for callers that cannot allocate: the launch plan
// of the shape last used on this device, followed by the partial results of a split launch.  One copy
// per GPU, held until the process ends.  Host code never uses this name as an address: the device address
// of each GPU's copy comes from hipGetSymbolAddress, taken in dfa_forward_static with that GPU current.
constexpr size_t kStaticScratchBytes = (size_t)40 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using namespace dfa;

// A launch plan in device memory.  Immutable once built, shared by every call with its shape (also from
// several threads and streams); freed when the cache has dropped it and the last call using it has returned.
struct DevicePlan {
    void* base = nullptr;
    const int32_t* rows = nullptr;
    const KeySeg* segs = nullptr;
    const Item* items = nullptr;
    const float* block_mult = nullptr;   // plans of the bf16 forward only
    bool packed_tiles = false;          // some tile packs several row groups: the kernel variant that reads block_mult
    int32_t n_items = 0;
    int device = 0;
    size_t bytes = 0;
    // launches with few workgroups walk their tiles with n_split_wgs workgroups in all (see split_plan and
    // launch_fwd_bf16_split) when the caller brings a workspace for their partial results; 0: never split
    const SplitWg* split_wgs = nullptr;
    const ItemParts* item_parts = nullptr;
    int32_t n_split_wgs = 0;
    bool owned = true;          // base came from hipMalloc and is freed with the plan

    DevicePlan() = default;
    DevicePlan(const DevicePlan&) = delete;
    DevicePlan& operator=(const DevicePlan&) = delete;
    ~DevicePlan() {
        if (!base || !owned) return;
        int cur = 0;
        const bool have_cur = hipGetDevice(&cur) == hipSuccess;
        // kernels still reading the plan finish first
        if (hipSetDevice(device) == hipSuccess) {
            (void)hipDeviceSynchronize();
            (void)hipFree(base);
        }
        if (have_cur) (void)hipSetDevice(cur);
    }
};
using PlanRef = std::shared_ptr<const DevicePlan>;

// The host plan laid out as the kernels read it: rows, then key progressions (plus one spare entry: a tile
// without progressions still reads inside the array), then launch items, then the workgroups and the per-item
// shares of a split launch, each part 256-byte aligned.
struct PackedPlan {
    std::vector<char> bytes;
    size_t off_segs = 0, off_items = 0, off_split_wgs = 0, off_item_parts = 0, off_block_mult = 0;
    int32_t n_items = 0;
    int32_t n_split_wgs = 0;
    bool packed_tiles = false;
};

constexpr int kPlanOrder = 3;              // launch order of build_plan (see dfa_plan.cpp)
constexpr size_t kMaxCachedPlans = 64;     // least recently used plans beyond these bounds are dropped
constexpr size_t kMaxCachedBytes = (size_t)256 << 20;

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// partial results of a split launch: one block (a tile's rows of out in fp16, then their lse and scales in fp32) per workgroup
size_t split_bytes(int32_t n_split_wgs) {
    return n_split_wgs > 0 ? align256((size_t)n_split_wgs * kSplitBlockBytes) : 0;
}

// packed: the plan of the bf16 forward kernel (row groups may share a tile, multiplicities per wave); the fp32 and
// backward kernels read the plain one.
int pack_plan(int32_t B, int32_t H, int32_t N, const dfa_branch_t* br, int32_t nb, const int32_t* offsets,
              const ChipShape& chip, bool packed, PackedPlan* out) {
    HostPlan hp;
    build_plan(B, H, N, br, nb, offsets, kPlanOrder, chip, packed, &hp);
    if (hp.items.size() > (size_t)0x7fffffff) return DFA_ERR_TOO_LARGE;
    const size_t b_rows = align256(hp.rows.size() * sizeof(int32_t));
    const size_t b_segs = align256(hp.segs.size() * sizeof(KeySeg) + sizeof(KeySeg));
    const size_t b_items = align256(hp.items.size() * sizeof(Item));
    if (packed) split_plan(&hp, chip);
    const size_t b_wgs = align256(hp.split_wgs.size() * sizeof(SplitWg));
    const size_t b_parts = align256(hp.item_parts.size() * sizeof(ItemParts));
    const size_t b_wmult = packed ? align256((hp.segs.size() + 1) * kTileBlocks * sizeof(float)) : 0;
    out->bytes.assign(b_rows + b_segs + b_items + b_wgs + b_parts + b_wmult, 0);
    out->off_segs = b_rows;
    out->off_items = b_rows + b_segs;
    out->off_split_wgs = out->off_items + b_items;
    out->off_item_parts = out->off_split_wgs + b_wgs;
    out->off_block_mult = out->off_item_parts + b_parts;
    if (packed) {
        // log2 of the multiplicities, -inf where a block's rows skip the progression
        float* wm = reinterpret_cast<float*>(out->bytes.data() + out->off_block_mult);
        for (size_t x = 0; x < hp.block_mult.size(); ++x) wm[x] = hp.block_mult[x] > 0 ? std::log2((float)hp.block_mult[x]) : -INFINITY;
    }
    if (!hp.rows.empty()) std::memcpy(out->bytes.data(), hp.rows.data(), hp.rows.size() * sizeof(int32_t));
    if (!hp.segs.empty()) std::memcpy(out->bytes.data() + b_rows, hp.segs.data(), hp.segs.size() * sizeof(KeySeg));
    if (!hp.items.empty()) std::memcpy(out->bytes.data() + b_rows + b_segs, hp.items.data(), hp.items.size() * sizeof(Item));
    if (!hp.split_wgs.empty()) {
        std::memcpy(out->bytes.data() + out->off_split_wgs, hp.split_wgs.data(), hp.split_wgs.size() * sizeof(SplitWg));
        std::memcpy(out->bytes.data() + out->off_item_parts, hp.item_parts.data(), hp.item_parts.size() * sizeof(ItemParts));
    }
    out->n_items = (int32_t)hp.items.size();
    out->n_split_wgs = (int32_t)hp.split_wgs.size();
    out->packed_tiles = hp.packed_tiles;
    return DFA_OK;
}

void point_plan(DevicePlan* dp, void* base, const PackedPlan& pp, int device) {
    char* b = static_cast<char*>(base);
    dp->base = base;
    dp->rows = reinterpret_cast<const int32_t*>(b);
    dp->segs = reinterpret_cast<const KeySeg*>(b + pp.off_segs);
    dp->items = reinterpret_cast<const Item*>(b + pp.off_items);
    dp->n_items = pp.n_items;
    dp->device = device;
    dp->bytes = pp.bytes.size();
    dp->split_wgs = reinterpret_cast<const SplitWg*>(b + pp.off_split_wgs);
    dp->item_parts = reinterpret_cast<const ItemParts*>(b + pp.off_item_parts);
    dp->n_split_wgs = pp.n_split_wgs;
    dp->block_mult = reinterpret_cast<const float*>(b + pp.off_block_mult);
    dp->packed_tiles = pp.packed_tiles;
}

std::vector<int32_t> plan_key(int device, bool packed, int32_t B, int32_t H, int32_t N, const dfa_branch_t* br,
                              int32_t nb, const int32_t* offsets) {
    std::vector<int32_t> key = {device, packed ? 1 : 0, B, H, N, nb, offsets ? 1 : 0};
    for (int x = 0; x < nb; ++x) {
        key.push_back(br[x].w);
        key.push_back(br[x].r);
    }
    if (offsets) key.insert(key.end(), offsets, offsets + (size_t)nb * H);
    return key;
}

std::mutex g_mu;
// plan cache, most recently used first
using PlanKey = std::vector<int32_t>;
std::list<std::pair<PlanKey, PlanRef>> g_lru;
std::map<PlanKey, std::list<std::pair<PlanKey, PlanRef>>::iterator> g_plans;
size_t g_cached_bytes = 0;
std::map<int, ChipShape> g_chips;

// Number of compute units and of accelerator dies of a device, read once per device.  Holds g_mu.
int chip_of(int device, ChipShape* out) {
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_chips.find(device);
    if (it == g_chips.end()) {
        ChipShape c;
        int cus = 0, dies = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
            return DFA_ERR_LAUNCH;
        if (hipDeviceGetAttribute(&dies, hipDeviceAttributeNumberOfXccs, device) != hipSuccess || dies <= 0) {
            (void)hipGetLastError();
            dies = 1;
        }
        c.cus = cus;
        c.dies = dies;
        it = g_chips.emplace(device, c).first;
    }
    *out = it->second;
    return DFA_OK;
}

int current_chip(int* device, ChipShape* chip) {
    if (hipGetDevice(device) != hipSuccess) return DFA_ERR_LAUNCH;
    return chip_of(*device, chip);
}

// Looks the plan of the current device up, building and uploading it on first use (the only device
// allocation the library makes).  Plans pushed out of the cache are freed once no call holds them.
int get_plan(bool packed, int32_t B, int32_t H, int32_t N, const dfa_branch_t* br, int32_t nb,
             const int32_t* offsets, PlanRef* out) {
    int device = 0;
    ChipShape chip;
    int rc = current_chip(&device, &chip);
    if (rc != DFA_OK) return rc;
    PlanKey key = plan_key(device, packed, B, H, N, br, nb, offsets);
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_plans.find(key);
        if (it != g_plans.end()) {
            g_lru.splice(g_lru.begin(), g_lru, it->second);
            *out = it->second->second;
            return DFA_OK;
        }
    }
    // built outside the lock: two threads may both build a new shape, the second result replaces the first
    PackedPlan pp;
    rc = pack_plan(B, H, N, br, nb, offsets, chip, packed, &pp);
    if (rc != DFA_OK) return rc;
    auto dp = std::make_shared<DevicePlan>();
    void* base = nullptr;
    if (hipMalloc(&base, pp.bytes.size()) != hipSuccess) {
        (void)hipGetLastError();   // reported here; a later launch's check must not see it again
        return DFA_ERR_LAUNCH;
    }
    point_plan(dp.get(), base, pp, device);
    if (hipMemcpy(base, pp.bytes.data(), pp.bytes.size(), hipMemcpyHostToDevice) != hipSuccess) return DFA_ERR_LAUNCH;

    std::vector<PlanRef> dropped;      // released after the lock: freeing synchronises the device
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_plans.find(key);
        if (it != g_plans.end()) {
            g_cached_bytes -= it->second->second->bytes;
            dropped.push_back(it->second->second);
            g_lru.erase(it->second);
            g_plans.erase(it);
        }
        g_lru.emplace_front(key, dp);
        g_plans[key] = g_lru.begin();
        g_cached_bytes += dp->bytes;
        while (g_lru.size() > 1 && (g_lru.size() > kMaxCachedPlans || g_cached_bytes > kMaxCachedBytes)) {
            g_cached_bytes -= g_lru.back().second->bytes;
            dropped.push_back(g_lru.back().second);
            g_plans.erase(g_lru.back().first);
            g_lru.pop_back();
        }
    }
    *out = dp;
    return DFA_OK;
}

int elem_size(dfa_dtype_t dt) { return dt == DFA_BF16 ? 2 : 4; }

bool aligned_rows(const void* p, dfa_strides_t s, int esize) {
    if (reinterpret_cast<uintptr_t>(p) % 16) return false;
    return (s.b * esize) % 16 == 0 && (s.n * esize) % 16 == 0 && (s.h * esize) % 16 == 0;
}

int check_common(int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt) {
    if (B <= 0 || H <= 0 || N <= 0 || D != DFA_HEAD_DIM) return DFA_ERR_SHAPE;
    if (dt != DFA_BF16 && dt != DFA_F32) return DFA_ERR_DTYPE;
    if ((int64_t)B * H * N > ((int64_t)1 << 40)) return DFA_ERR_TOO_LARGE;
    return DFA_OK;
}

// The stand-alone stage kernels carry b (and h) in grid.y / grid.z and index one image with
// 32-bit counters.
int check_stage_grid(int32_t B, int32_t H, int32_t N) {
    if (B > 65535 || H > 65535 || (int64_t)N * H * 16 >= ((int64_t)1 << 31)) return DFA_ERR_TOO_LARGE;
    return DFA_OK;
}

// Largest stride a key progression of the plan can have: a branch's dilation rate, or, for keys that
// several branches share, a divisor of the rates' common period (at most kMaxCoalesceLcm).
int64_t max_key_stride(const dfa_branch_t* br, int32_t nb) {
    int64_t s = nb > 1 ? kMaxCoalesceLcm : 1;
    for (int x = 0; x < nb; ++x) s = std::max<int64_t>(s, br[x].r);
    return s;
}

int make_offsets(const int32_t* head_offsets, int32_t H, int32_t r, HeadOffsets* o) {
    std::memset(o, 0, sizeof(*o));
    if (!head_offsets) return DFA_OK;
    if (H > kMaxExplicitHeads) return DFA_ERR_TOO_LARGE;
    o->explicit_table = 1;
    for (int h = 0; h < H; ++h) {
        if (head_offsets[h] < 0 || head_offsets[h] >= r) return DFA_ERR_SHAPE;
        o->o[h] = head_offsets[h];
    }
    return DFA_OK;
}

// Per-device state of dfa_forward_static: where this GPU's copy of `scratch` lives and which plan it holds.
struct StaticScratch {
    unsigned char* ptr = nullptr;      // from hipGetSymbolAddress with this device current
    bool holds_plan = false;
    PlanKey key;
    DevicePlan plan;                   // points into ptr, not owned
    size_t plan_bytes = 0;             // 256-byte aligned; the split partial results follow
};
std::mutex g_static_mu;
std::map<int, StaticScratch> g_static;

// Argument checks of the attention entry points (everything that can be found without the GPU).
int check_forward_args(const void* q, const void* k, const void* v, dfa_strides_t sq, dfa_strides_t sk,
                       dfa_strides_t sv, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                       float scale, const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets,
                       const void* out, const float* lse) {
    if (!q || !k || !v || !out) return DFA_ERR_NULL;
    int rc = check_common(B, H, N, D, dt);
    if (rc != DFA_OK) return rc;
    rc = check_branches(H, N, branches, nb, head_offsets);
    if (rc != DFA_OK) return rc;
    if (!std::isfinite(scale) || scale <= 0.f) return DFA_ERR_SHAPE;
    const int es = elem_size(dt);
    if (!aligned_rows(q, sq, es) || !aligned_rows(k, sk, es) || !aligned_rows(v, sv, es)) return DFA_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(out) % 16 || (lse && reinterpret_cast<uintptr_t>(lse) % 4)) return DFA_ERR_ALIGN;
    // the copy lanes address a 64-key step with 32-bit byte offsets from its first row
    if (sk.n <= 0 || sv.n <= 0 || sq.n <= 0) return DFA_ERR_TOO_LARGE;
    if (64 * max_key_stride(branches, nb) * std::max(sk.n, sv.n) * es + 128 >= ((int64_t)1 << 31)) return DFA_ERR_TOO_LARGE;
    return DFA_OK;
}

// Enqueues the launches of one forward call on a plan.  split_ws: room for the plan's split partial
// results (split_bytes) or nullptr, in which case a launch with few workgroups runs unsplit.
int launch_forward(const DevicePlan& dp, const void* q, const void* k, const void* v, dfa_strides_t sq,
                   dfa_strides_t sk, dfa_strides_t sv, int32_t B, int32_t H, int32_t N, dfa_dtype_t dt,
                   float scale, void* out, bool out_f32, float* lse, float* split_ws, void* stream) {
    FwdParams p;
    p.q = q; p.k = k; p.v = v;
    p.sqb = sq.b; p.sqn = sq.n; p.sqh = sq.h;
    p.skb = sk.b; p.skn = sk.n; p.skh = sk.h;
    p.svb = sv.b; p.svn = sv.n; p.svh = sv.h;
    p.out = out; p.lse = lse;
    p.rows = dp.rows; p.segs = dp.segs; p.items = dp.items; p.block_mult = dp.block_mult;
    p.H = H; p.N = N; p.scale = scale;
    p.split_wgs = dp.split_wgs; p.item_parts = dp.item_parts; p.split_ws = split_ws;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (dt == DFA_BF16 && !out_f32 && dp.n_split_wgs > 0 && split_ws) {
        // few workgroups: partial results per share of the key walk, then their log-sum-exp merge
        e = launch_fwd_bf16_split(p, dp.n_split_wgs, dp.packed_tiles, st);
        if (e == hipSuccess) e = launch_merge_split(p, dp.n_items, st);
    } else if (dt == DFA_BF16) {
        e = launch_fwd_bf16(p, dp.n_items, out_f32, dp.packed_tiles, st);
    } else {
        e = launch_fwd_f32(p, dp.n_items, st);         // fp32 inputs always give fp32 output
    }
    return e == hipSuccess ? DFA_OK : DFA_ERR_LAUNCH;
}

int forward_impl(const void* q, const void* k, const void* v, dfa_strides_t sq, dfa_strides_t sk,
                 dfa_strides_t sv, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                 float scale, const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets,
                 void* out, bool out_f32, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_forward_args(q, k, v, sq, sk, sv, B, H, N, D, dt, scale, branches, nb, head_offsets, out, lse);
    if (rc != DFA_OK) return rc;
    if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return DFA_ERR_ALIGN;
    PlanRef dp;
    // fp32 output from bf16 inputs is the unmerged single branch of dfa_forward_branch: the plain plan
    rc = get_plan(dt == DFA_BF16 && !out_f32, B, H, N, branches, nb, head_offsets, &dp);
    if (rc != DFA_OK) return rc;
    float* split_ws = nullptr;
    if (workspace && dt == DFA_BF16 && !out_f32 && dp->n_split_wgs > 0) {
        if (workspace_bytes < split_bytes(dp->n_split_wgs)) return DFA_ERR_WORKSPACE;
        split_ws = static_cast<float*>(workspace);
    }
    return launch_forward(*dp, q, k, v, sq, sk, sv, B, H, N, dt, scale, out, out_f32, lse, split_ws, stream);
}

}  // namespace

extern "C" {

int dfa_version(void) { return 200; }

const char* dfa_error_string(int code) {
    switch (code) {
        case DFA_OK: return "ok";
        case DFA_ERR_NULL: return "a required pointer is NULL";
        case DFA_ERR_SHAPE: return "bad shape, branch (w, r), head offset or scale";
        case DFA_ERR_BRANCHES: return "number of branches outside 1..DFA_MAX_BRANCHES";
        case DFA_ERR_DTYPE: return "unknown dtype";
        case DFA_ERR_ALIGN: return "pointer or stride breaks 16-byte row alignment";
        case DFA_ERR_LAUNCH: return "HIP runtime error (allocation, copy or launch)";
        case DFA_ERR_TOO_LARGE: return "problem too large for the kernel's index arithmetic";
        case DFA_ERR_WORKSPACE: return "workspace smaller than dfa_workspace_bytes() asks for";
        default: return "unknown error code";
    }
}

int dfa_index_map(int32_t N, int32_t H, dfa_branch_t br, const int32_t* head_offsets, int32_t* out_idx) {
    if (!out_idx) return DFA_ERR_NULL;
    if (H <= 0 || N <= 0 || br.r < 1 || br.w < br.r || br.w > N || N % br.w || br.w % br.r) return DFA_ERR_SHAPE;
    const int32_t per_seg = br.w / br.r, per_head = N / br.r;
    for (int32_t h = 0; h < H; ++h) {
        const int32_t o = head_offsets ? head_offsets[h] : h % br.r;
        if (o < 0 || o >= br.r) return DFA_ERR_SHAPE;
        int32_t* dst = out_idx + (int64_t)h * per_head;
        for (int32_t slot = 0; slot < per_head; ++slot)
            dst[slot] = (slot / per_seg) * br.w + o + (slot % per_seg) * br.r;
    }
    return DFA_OK;
}

int dfa_index_map_device(int32_t N, int32_t H, dfa_branch_t br, const int32_t* head_offsets,
                         int32_t* d_out_idx, void* stream) {
    if (!d_out_idx) return DFA_ERR_NULL;
    if (H <= 0 || N <= 0 || br.r < 1 || br.w < br.r || br.w > N || N % br.w || br.w % br.r) return DFA_ERR_SHAPE;
    HeadOffsets offs;
    const int rc = make_offsets(head_offsets, H, br.r, &offs);
    if (rc != DFA_OK) return rc;
    return launch_index_map(N, H, br.w, br.r, offs, d_out_idx, static_cast<hipStream_t>(stream)) == hipSuccess
               ? DFA_OK : DFA_ERR_LAUNCH;
}

int dfa_forward(const void* q, const void* k, const void* v, dfa_strides_t sq, dfa_strides_t sk,
                dfa_strides_t sv, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets,
                void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    try {
        return forward_impl(q, k, v, sq, sk, sv, B, H, N, D, dt, scale, branches, nb, head_offsets,
                            out, dt == DFA_F32, lse, workspace, workspace_bytes, stream);
    } catch (const std::bad_alloc&) {
        return DFA_ERR_LAUNCH;
    }
}

int dfa_forward_static(const void* q, const void* k, const void* v, dfa_strides_t sq, dfa_strides_t sk,
                       dfa_strides_t sv, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                       const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets,
                       void* out, float* lse, void* stream) {
    int rc = check_forward_args(q, k, v, sq, sk, sv, B, H, N, D, dt, scale, branches, nb, head_offsets, out, lse);
    if (rc != DFA_OK) return rc;
    try {
        int device = 0;
        ChipShape chip;
        rc = current_chip(&device, &chip);
        if (rc != DFA_OK) return rc;
        // held until the launches are enqueued: two host threads must not repoint the scratch under each other
        std::lock_guard<std::mutex> lock(g_static_mu);
        StaticScratch& ss = g_static[device];
        if (!ss.ptr) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                return DFA_ERR_LAUNCH;
            }
            ss.ptr = static_cast<unsigned char*>(p);
            ss.plan.owned = false;
        }
        PlanKey key = plan_key(device, dt == DFA_BF16, B, H, N, branches, nb, head_offsets);
        if (!ss.holds_plan || ss.key != key) {
            PackedPlan pp;
            rc = pack_plan(B, H, N, branches, nb, head_offsets, chip, dt == DFA_BF16, &pp);
            if (rc != DFA_OK) return rc;
            const size_t plan_bytes = align256(pp.bytes.size());
            const size_t part_bytes = dt == DFA_BF16 ? split_bytes(pp.n_split_wgs) : 0;
            if (plan_bytes + part_bytes > kStaticScratchBytes) return DFA_ERR_WORKSPACE;
            // launches of earlier calls may still be reading the plan that is about to be overwritten
            ss.holds_plan = false;
            if (hipDeviceSynchronize() != hipSuccess ||
                hipMemcpy(ss.ptr, pp.bytes.data(), pp.bytes.size(), hipMemcpyHostToDevice) != hipSuccess) {
                (void)hipGetLastError();
                return DFA_ERR_LAUNCH;
            }
            point_plan(&ss.plan, ss.ptr, pp, device);
            ss.plan_bytes = plan_bytes;
            ss.key = std::move(key);
            ss.holds_plan = true;
        } else if (dt == DFA_BF16 && ss.plan_bytes + split_bytes(ss.plan.n_split_wgs) > kStaticScratchBytes) {
            return DFA_ERR_WORKSPACE;      // the plan was left by a call in the other precision, which needs no partial results
        }
        // the partial results of a split launch are written in full by that launch before its merge reads them:
        // nothing in the scratch has to start at zero
        float* split_ws = ss.plan.n_split_wgs > 0 ? reinterpret_cast<float*>(ss.ptr + ss.plan_bytes) : nullptr;
        return launch_forward(ss.plan, q, k, v, sq, sk, sv, B, H, N, dt, scale, out, dt == DFA_F32, lse, split_ws, stream);
    } catch (const std::bad_alloc&) {
        return DFA_ERR_LAUNCH;
    }
}

int dfa_forward_branch(const void* q, const void* k, const void* v, dfa_strides_t sq, dfa_strides_t sk,
                       dfa_strides_t sv, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                       float scale, dfa_branch_t br, const int32_t* head_offsets,
                       float* out_b, float* lse_b, void* stream) {
    if (!lse_b) return DFA_ERR_NULL;
    try {
        return forward_impl(q, k, v, sq, sk, sv, B, H, N, D, dt, scale, &br, 1, head_offsets,
                            out_b, true, lse_b, nullptr, 0, stream);
    } catch (const std::bad_alloc&) {
        return DFA_ERR_LAUNCH;
    }
}

int dfa_merge(const float* out_b, const float* lse_b, int32_t nb, int32_t B, int32_t H, int32_t N,
              int32_t D, dfa_dtype_t dt, void* out, float* lse, void* stream) {
    if (!out_b || !lse_b || !out) return DFA_ERR_NULL;
    if (nb < 1 || nb > DFA_MAX_BRANCHES) return DFA_ERR_BRANCHES;
    int rc = check_common(B, H, N, D, dt);
    if (rc != DFA_OK) return rc;
    rc = check_stage_grid(B, H, N);
    if (rc != DFA_OK) return rc;
    if (reinterpret_cast<uintptr_t>(out_b) % 16 || reinterpret_cast<uintptr_t>(out) % 16) return DFA_ERR_ALIGN;
    return launch_merge(out_b, lse_b, nb, B, H, N, dt == DFA_BF16, out, lse,
                        static_cast<hipStream_t>(stream)) == hipSuccess ? DFA_OK : DFA_ERR_LAUNCH;
}

int dfa_gather(const void* x, dfa_strides_t sx, int32_t B, int32_t H, int32_t N, int32_t D,
               dfa_dtype_t dt, dfa_branch_t br, const int32_t* head_offsets, void* xg, void* stream) {
    if (!x || !xg) return DFA_ERR_NULL;
    int rc = check_common(B, H, N, D, dt);
    if (rc != DFA_OK) return rc;
    if (br.r < 1 || br.w < br.r || br.w > N || N % br.w || br.w % br.r) return DFA_ERR_SHAPE;
    rc = check_stage_grid(B, H, N);
    if (rc != DFA_OK) return rc;
    HeadOffsets offs;
    rc = make_offsets(head_offsets, H, br.r, &offs);
    if (rc != DFA_OK) return rc;
    if (!aligned_rows(x, sx, elem_size(dt)) || reinterpret_cast<uintptr_t>(xg) % 16) return DFA_ERR_ALIGN;
    return launch_gather(x, sx.b, sx.n, sx.h, B, H, N, elem_size(dt), br.w, br.r, offs, xg,
                         static_cast<hipStream_t>(stream)) == hipSuccess ? DFA_OK : DFA_ERR_LAUNCH;
}

int dfa_scatter(const void* og, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                dfa_branch_t br, const int32_t* head_offsets, void* out, void* stream) {
    if (!og || !out) return DFA_ERR_NULL;
    int rc = check_common(B, H, N, D, dt);
    if (rc != DFA_OK) return rc;
    if (br.r < 1 || br.w < br.r || br.w > N || N % br.w || br.w % br.r) return DFA_ERR_SHAPE;
    rc = check_stage_grid(B, H, N);
    if (rc != DFA_OK) return rc;
    HeadOffsets offs;
    rc = make_offsets(head_offsets, H, br.r, &offs);
    if (rc != DFA_OK) return rc;
    if (reinterpret_cast<uintptr_t>(og) % 16 || reinterpret_cast<uintptr_t>(out) % 16) return DFA_ERR_ALIGN;
    return launch_scatter(og, B, H, N, elem_size(dt), br.w, br.r, offs, out,
                          static_cast<hipStream_t>(stream)) == hipSuccess ? DFA_OK : DFA_ERR_LAUNCH;
}

int dfa_backward(const void* q, const void* k, const void* v, const void* out, const float* lse,
                 const void* dout, dfa_strides_t sq, dfa_strides_t sk, dfa_strides_t sv,
                 int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                 const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets,
                 float* delta_ws, void* dq, void* dk, void* dv, void* stream) {
    if (!q || !k || !v || !out || !lse || !dout || !delta_ws || !dq || !dk || !dv) return DFA_ERR_NULL;
    int rc = check_common(B, H, N, D, dt);
    if (rc != DFA_OK) return rc;
    rc = check_branches(H, N, branches, nb, head_offsets);
    if (rc != DFA_OK) return rc;
    if (!std::isfinite(scale) || scale <= 0.f) return DFA_ERR_SHAPE;
    const int es = elem_size(dt);
    if (!aligned_rows(q, sq, es) || !aligned_rows(k, sk, es) || !aligned_rows(v, sv, es)) return DFA_ERR_ALIGN;
    for (const void* ptr : {out, dout, (const void*)dq, (const void*)dk, (const void*)dv})
        if (reinterpret_cast<uintptr_t>(ptr) % 16) return DFA_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(lse) % 4 || reinterpret_cast<uintptr_t>(delta_ws) % 4) return DFA_ERR_ALIGN;
    rc = check_stage_grid(B, H, N);          // the per-row preparation carries b on the grid
    if (rc != DFA_OK) return rc;
    // the copy lanes address a 64-row step with 32-bit byte offsets from its first row
    {
        const int64_t widest = std::max(std::max(sq.n, sk.n), std::max(sv.n, (int64_t)H * D));
        if (sq.n <= 0 || sk.n <= 0 || sv.n <= 0 || 64 * max_key_stride(branches, nb) * widest * es + 128 >= ((int64_t)1 << 31))
            return DFA_ERR_TOO_LARGE;
    }
    try {
        PlanRef plan;
        rc = get_plan(false, B, H, N, branches, nb, head_offsets, &plan);
        if (rc != DFA_OK) return rc;
        const DevicePlan& dp = *plan;
        BwdParams p;
        p.q = q; p.k = k; p.v = v; p.out = out; p.dout = dout;
        p.sqb = sq.b; p.sqn = sq.n; p.sqh = sq.h;
        p.skb = sk.b; p.skn = sk.n; p.skh = sk.h;
        p.svb = sv.b; p.svn = sv.n; p.svh = sv.h;
        p.lse = lse; p.ndelta = delta_ws; p.lse2 = delta_ws + (int64_t)B * H * N; p.dq = dq; p.dk = dk; p.dv = dv;
        p.rows = dp.rows; p.segs = dp.segs; p.items = dp.items;
        p.H = H; p.N = N; p.scale = scale;
        return launch_bwd(p, dp.n_items, B, dt == DFA_BF16, static_cast<hipStream_t>(stream)) == hipSuccess
                   ? DFA_OK : DFA_ERR_LAUNCH;
    } catch (const std::bad_alloc&) {
        return DFA_ERR_LAUNCH;
    }
}

int dfa_linear(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
               int64_t ldx, int64_t ldw, int64_t ldy, void* stream) {
    if (!x || !w || !y) return DFA_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || M % 256 || N % 128 || K % 64) return DFA_ERR_SHAPE;
    if (ldx < K || ldw < K || ldy < N) return DFA_ERR_SHAPE;
    if (ldx % 8 || ldw % 8 || ldy % 8 || reinterpret_cast<uintptr_t>(x) % 16 ||
        reinterpret_cast<uintptr_t>(w) % 16 || reinterpret_cast<uintptr_t>(y) % 16) return DFA_ERR_ALIGN;
    // lane offsets inside an 8-row group are 32-bit; tiles are counted in 32 bits
    if (ldx >= ((int64_t)1 << 26) || ldw >= ((int64_t)1 << 26) || (M / 256) * (int64_t)(N / 128) >= ((int64_t)1 << 30))
        return DFA_ERR_TOO_LARGE;
    int device = 0;
    ChipShape chip;
    const int rc = current_chip(&device, &chip);
    if (rc != DFA_OK) return rc;
    return launch_linear_bf16(x, w, y, M, N, K, ldx, ldw, ldy, chip, static_cast<hipStream_t>(stream)) == hipSuccess
               ? DFA_OK : DFA_ERR_LAUNCH;
}

int dfa_encoder_stack(const void* x, const void* w_qkv, const void* w_o, int32_t layers,
                      int32_t B, int32_t H, int32_t N, int32_t D, float scale,
                      const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets,
                      void* qkv_ws, void* attn_ws, void* y, void* workspace, size_t workspace_bytes, void* stream) {
    if (!x || !w_qkv || !w_o || !qkv_ws || !attn_ws || !y) return DFA_ERR_NULL;
    if (layers < 1) return DFA_ERR_SHAPE;
    int rc = check_common(B, H, N, D, DFA_BF16);
    if (rc != DFA_OK) return rc;
    const int64_t E = (int64_t)H * D, M = (int64_t)B * N;
    if (M % 256 || E % 128) return DFA_ERR_SHAPE;
    const uint16_t* wq = static_cast<const uint16_t*>(w_qkv);
    const uint16_t* wo = static_cast<const uint16_t*>(w_o);
    const uint16_t* qkv = static_cast<const uint16_t*>(qkv_ws);
    // q, k, v of token (b, n), head h live at qkv[((b*N + n)*3 + t)*E + h*D ..]
    const dfa_strides_t sq = {(int64_t)N * 3 * E, 3 * E, D};
    // every argument error is found here, before the first launch overwrites a workspace
    rc = check_forward_args(qkv, qkv + E, qkv + 2 * E, sq, sq, sq, B, H, N, D, DFA_BF16, scale, branches, nb,
                            head_offsets, attn_ws, nullptr);
    if (rc != DFA_OK) return rc;
    for (const void* ptr : {x, w_qkv, w_o, (const void*)y})
        if (reinterpret_cast<uintptr_t>(ptr) % 16) return DFA_ERR_ALIGN;
    if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return DFA_ERR_ALIGN;
    try {
        PlanRef dp;
        rc = get_plan(true, B, H, N, branches, nb, head_offsets, &dp);
        if (rc != DFA_OK) return rc;
        if (workspace && dp->n_split_wgs > 0 && workspace_bytes < split_bytes(dp->n_split_wgs))
            return DFA_ERR_WORKSPACE;
        for (int l = 0; l < layers; ++l) {
            rc = dfa_linear(l == 0 ? x : y, wq + (int64_t)l * 3 * E * E, qkv_ws, M, (int32_t)(3 * E), (int32_t)E,
                            E, E, 3 * E, stream);
            if (rc != DFA_OK) return rc;
            rc = launch_forward(*dp, qkv, qkv + E, qkv + 2 * E, sq, sq, sq, B, H, N, DFA_BF16, scale, attn_ws, false,
                                nullptr, dp->n_split_wgs > 0 ? static_cast<float*>(workspace) : nullptr, stream);
            if (rc != DFA_OK) return rc;
            rc = dfa_linear(attn_ws, wo + (int64_t)l * E * E, y, M, (int32_t)E, (int32_t)E, E, E, E, stream);
            if (rc != DFA_OK) return rc;
        }
    } catch (const std::bad_alloc&) {
        return DFA_ERR_LAUNCH;
    }
    return DFA_OK;
}

size_t dfa_workspace_bytes(int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                           const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets) {
    if (check_common(B, H, N, D, dt) != DFA_OK || check_branches(H, N, branches, nb, head_offsets) != DFA_OK) return 0;
    if (dt != DFA_BF16) return 0;
    try {
        int device = 0;
        ChipShape chip;                    // the MI355X when no device can be asked
        if (current_chip(&device, &chip) != DFA_OK) (void)hipGetLastError();
        HostPlan hp;
        build_plan(B, H, N, branches, nb, head_offsets, kPlanOrder, chip, true, &hp);
        split_plan(&hp, chip);
        return split_bytes((int32_t)hp.split_wgs.size());
    } catch (const std::bad_alloc&) {
        return 0;
    }
}

namespace {

int describe_plan(bool packed, int32_t B, int32_t H, int32_t N, const dfa_branch_t* branches, int32_t nb,
                  const int32_t* head_offsets, int32_t* n_tiles, int32_t* n_rows, int32_t* n_segs,
                  int32_t* n_items, int32_t* tiles, int32_t* rows, int32_t* segs, int32_t* block_mult, int32_t* items) {
    if (!n_tiles || !n_rows || !n_segs || !n_items) return DFA_ERR_NULL;
    if (B <= 0) return DFA_ERR_SHAPE;
    const int rc = check_branches(H, N, branches, nb, head_offsets);
    if (rc != DFA_OK) return rc;
    try {
        HostPlan hp;
        build_plan(B, H, N, branches, nb, head_offsets, kPlanOrder, ChipShape(), packed, &hp);
        *n_tiles = (int32_t)hp.tiles.size();
        *n_rows = (int32_t)hp.rows.size();
        *n_segs = (int32_t)hp.segs.size();
        *n_items = (int32_t)hp.items.size();
        if (tiles)
            for (size_t t = 0; t < hp.tiles.size(); ++t) {
                const Tile& x = hp.tiles[t];
                const int32_t rec[6] = {x.h, x.row_begin, x.nrows, x.seg_begin, x.nseg, x.n_steps};
                std::memcpy(tiles + 6 * t, rec, sizeof(rec));
            }
        if (rows) std::memcpy(rows, hp.rows.data(), hp.rows.size() * sizeof(int32_t));
        if (segs)
            for (size_t s = 0; s < hp.segs.size(); ++s) {
                segs[4 * s] = hp.segs[s].key0;
                segs[4 * s + 1] = hp.segs[s].stride;
                segs[4 * s + 2] = hp.segs[s].count;
                segs[4 * s + 3] = hp.seg_mult[s];
            }
        if (block_mult) std::memcpy(block_mult, hp.block_mult.data(), hp.block_mult.size() * sizeof(int32_t));
        if (items)
            for (size_t i = 0; i < hp.items.size(); ++i) {
                items[2 * i] = hp.items[i].tile;
                items[2 * i + 1] = hp.items[i].b;
            }
    } catch (const std::bad_alloc&) {
        return DFA_ERR_LAUNCH;
    }
    return DFA_OK;
}

}  // namespace

int dfa_plan_describe(int32_t B, int32_t H, int32_t N, const dfa_branch_t* branches, int32_t nb,
                      const int32_t* head_offsets, int32_t* n_tiles, int32_t* n_rows, int32_t* n_segs,
                      int32_t* n_items, int32_t* tiles, int32_t* rows, int32_t* segs, int32_t* items) {
    return describe_plan(false, B, H, N, branches, nb, head_offsets, n_tiles, n_rows, n_segs, n_items, tiles, rows, segs,
                         nullptr, items);
}

int dfa_plan_describe_forward(int32_t B, int32_t H, int32_t N, const dfa_branch_t* branches, int32_t nb,
                              const int32_t* head_offsets, int32_t* n_tiles, int32_t* n_rows, int32_t* n_segs,
                              int32_t* n_items, int32_t* tiles, int32_t* rows, int32_t* segs, int32_t* block_mult,
                              int32_t* items) {
    return describe_plan(true, B, H, N, branches, nb, head_offsets, n_tiles, n_rows, n_segs, n_items, tiles, rows, segs,
                         block_mult, items);
}

int dfa_release_plans(void) {
    std::vector<PlanRef> dropped;          // freed after the lock (each free synchronises its device)
    {
        std::lock_guard<std::mutex> lock(g_mu);
        for (auto& kv : g_lru) dropped.push_back(kv.second);
        g_lru.clear();
        g_plans.clear();
        g_cached_bytes = 0;
    }
    return DFA_OK;
}

size_t dfa_dense_unfused_workspace_bytes(int32_t B, int32_t H, int32_t N, int32_t D) {
    if (B <= 0 || H <= 0 || N <= 0 || D != DFA_HEAD_DIM) return 0;
    return align256((size_t)B * H * N * N * 2) + align256((size_t)B * H * N * D * 2);
}

int dfa_dense_unfused(const void* q, const void* k, const void* v, dfa_strides_t sq, dfa_strides_t sk,
                      dfa_strides_t sv, int32_t B, int32_t H, int32_t N, int32_t D, float scale,
                      void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !out || !workspace) return DFA_ERR_NULL;
    int rc = check_common(B, H, N, D, DFA_BF16);
    if (rc != DFA_OK) return rc;
    if (N % 256 || N > 4096) return DFA_ERR_SHAPE;       // whole 256-row tiles; a row of scores is held in registers
    if (!std::isfinite(scale) || scale <= 0.f) return DFA_ERR_SHAPE;
    if (!aligned_rows(q, sq, 2) || !aligned_rows(k, sk, 2) || !aligned_rows(v, sv, 2)) return DFA_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(out) % 16 || reinterpret_cast<uintptr_t>(workspace) % 16 ||
        (lse && reinterpret_cast<uintptr_t>(lse) % 4)) return DFA_ERR_ALIGN;
    if (sq.n <= 0 || sk.n <= 0 || sv.n <= 0 || sq.n >= ((int64_t)1 << 26) || sk.n >= ((int64_t)1 << 26)) return DFA_ERR_TOO_LARGE;
    if ((int64_t)B * H > 65535) return DFA_ERR_TOO_LARGE;
    if (workspace_bytes < dfa_dense_unfused_workspace_bytes(B, H, N, D)) return DFA_ERR_WORKSPACE;
    char* ws = static_cast<char*>(workspace);
    return launch_dense_unfused(q, k, v, sq.b, sq.n, sq.h, sk.b, sk.n, sk.h, sv.b, sv.n, sv.h, B, H, N, scale, out, lse,
                                ws, ws + align256((size_t)B * H * N * N * 2), static_cast<hipStream_t>(stream)) == hipSuccess
               ? DFA_OK : DFA_ERR_LAUNCH;
}

int dfa_forward_timed(const void* q, const void* k, const void* v, dfa_strides_t sq, dfa_strides_t sk,
                      dfa_strides_t sv, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                      float scale, const dfa_branch_t* branches, int32_t nb, const int32_t* head_offsets,
                      void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream,
                      int32_t iters, float* ms) {
    if (!ms) return DFA_ERR_NULL;
    if (iters < 1) return DFA_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // one untimed call builds the plan and surfaces argument errors
    int rc = dfa_forward(q, k, v, sq, sk, sv, B, H, N, D, dt, scale, branches, nb, head_offsets, out, lse,
                         workspace, workspace_bytes, stream);
    if (rc != DFA_OK) return rc;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return DFA_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return DFA_ERR_LAUNCH; }
    bool ok = hipEventRecord(e0, st) == hipSuccess;
    for (int i = 0; ok && i < iters && rc == DFA_OK; ++i)
        rc = dfa_forward(q, k, v, sq, sk, sv, B, H, N, D, dt, scale, branches, nb, head_offsets, out, lse,
                         workspace, workspace_bytes, stream);
    ok = ok && hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
    float total = 0.f;
    ok = ok && hipEventElapsedTime(&total, e0, e1) == hipSuccess;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != DFA_OK) return rc;
    if (!ok) return DFA_ERR_LAUNCH;
    *ms = total / iters;
    return DFA_OK;
}

}  // extern "C"
