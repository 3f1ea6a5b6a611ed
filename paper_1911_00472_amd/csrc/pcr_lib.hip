// C ABI of the PCR decode library (see include/pcr.h) and the host logic behind it: header
// validation, layout of the device buffers, the work lists that map lanes to restart
// intervals, and the kernel launches.  Everything data-dependent runs in the kernels of
// pcr_kernels.h; the host parse done in pcr_open only sizes buffers and rejects bad input early.
#include <hip/hip_runtime.h>
#include <fcntl.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/pcr.h"
#include "pcr_kernels.h"
#include "pcr_hist.h"
#include "pcr_similarity.h"
#include "pcr_encode.h"

using namespace pcr;

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return PCR_E_DEVICE; } } while (0)

namespace {

enum Kind { kDcFirst = 0, kAcFirst = 1, kAcRefine = 2, kSequential = 3, kNumKinds = 4 };
struct LevelList {
    Unit* d_units = nullptr; uint32_t n = 0; int kind = 0;
    int shape = 0;                                                               // DC first scans: dc_shape of the units
    RefineScan* d_refine = nullptr; uint32_t n_refine = 0;                      // the scans of an AC refinement launch, for its per-block kernels
    RefineTile* d_plane_tiles = nullptr; uint32_t n_plane_tiles = 0;              // k_refine_history: chunks of the padded planes of those scans
    RefineTile* d_cov_tiles = nullptr; uint32_t n_cov_tiles = 0;                  // k_refine_deal, k_refine_blocks: chunks of the blocks the images cover
    LaneJob* d_jobs = nullptr; uint32_t n_jobs = 0;                              // the same units cut into jobs of a lane-per-unit kernel
};

struct Plan {                               // launch geometry for one scan group k
    std::vector<LevelList> levels;
    ApplyUnit* d_apply = nullptr; ApplyList* d_apply_lists = nullptr; int32_t* d_list_idx = nullptr; uint32_t n_apply = 0, apply_grid_x = 0;
    bool has_ac = false;                     // some scan <= k is an AC scan (else only element 0 of every block is ever touched)
    bool had_ac = false;                     // ... some scan <= k0 (the fidelity an upgrade starts from)
    bool dc_complete = true;                 // every component of every image has its first DC scan among the scans <= k
};

// Device memory of a handle comes out of two arenas (one sized by the image and scan counts, one by the
// images themselves): a block that is handed out front to back and re-used as a whole when the handle is
// bound to another record.  An arena grows only when a record needs more than it holds, so that a loader
// that binds record after record of similar size to one handle stops allocating after the first few.
// What does not fit (work lists of a scan group first asked for when the arena is full) is allocated on
// its own and released at the next reset.
struct Arena {
    uint8_t* base = nullptr; size_t cap = 0, used = 0;
    std::vector<void*> extra;
};
constexpr size_t kArenaAlign = 256;
size_t arena_round(size_t bytes) { return (bytes + kArenaAlign - 1) / kArenaAlign * kArenaAlign; }
void arena_release_extra(Arena* a) { for (void* p : a->extra) (void)hipFree(p); a->extra.clear(); }
void arena_free(Arena* a) { arena_release_extra(a); if (a->base) (void)hipFree(a->base); a->base = nullptr; a->cap = a->used = 0; }
// Empties the arena and makes sure it holds at least `bytes`.  Nothing handed out earlier may still be in use.
int arena_reset(Arena* a, size_t bytes) {
    arena_release_extra(a);
    a->used = 0;
    if (a->cap >= bytes) return PCR_OK;
    if (a->base) (void)hipFree(a->base);
    a->base = nullptr; a->cap = 0;
    const size_t want = bytes + bytes / 8;                    // some room for the next, slightly larger record
    if (hipMalloc((void**)&a->base, want) != hipSuccess) {
        (void)hipGetLastError();
        if (hipMalloc((void**)&a->base, bytes) != hipSuccess) { (void)hipGetLastError(); return PCR_E_NOMEM; }
        a->cap = bytes;
    } else a->cap = want;
    return PCR_OK;
}
template <class T> int arena_alloc(Arena* a, T** p, size_t count) {
    *p = nullptr;
    const size_t bytes = arena_round((count ? count : 1) * sizeof(T));
    if (a->used + bytes <= a->cap) { *p = reinterpret_cast<T*>(a->base + a->used); a->used += bytes; return PCR_OK; }
    void* q = nullptr;
    if (hipMalloc(&q, bytes) != hipSuccess) { (void)hipGetLastError(); return PCR_E_NOMEM; }
    a->extra.push_back(q);
    *p = reinterpret_cast<T*>(q);
    return PCR_OK;
}
// (a synchronous copy: the data is on the device when the call returns, whatever stream uses it next)
template <class T> int arena_upload(Arena* a, T** p, const std::vector<T>& v) {
    int rc = arena_alloc(a, p, v.size());
    if (rc) return rc;
    if (!v.empty() && hipMemcpy(*p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return PCR_E_DEVICE;
    return PCR_OK;
}

}  // namespace

constexpr size_t kTimingRing = 64;
struct CallTiming {
    std::vector<hipEvent_t> ev;                // ev[0] = start of the call, ev[i] = end of interval i
    std::vector<uint8_t> stage;                // stage[i] = stage that interval (ev[i-1], ev[i]) belongs to
    size_t used = 0;                           // events recorded by the call that last used this slot
};

// Records this process has open: the default choice between the two shapes of entropy decoder looks at it (lanes_pay).
static std::atomic<int> g_open_records{0};

struct pcr_record {
    pcr_record() { g_open_records.fetch_add(1, std::memory_order_relaxed); }
    ~pcr_record() { g_open_records.fetch_sub(1, std::memory_order_relaxed); }
    pcr_record(const pcr_record&) = delete;
    pcr_record& operator=(const pcr_record&) = delete;
    int device = 0;
    size_t nbytes = 0;
    RecordHeader hdr{};
    std::vector<uint8_t> header;            // host copy of the metadata block
    std::vector<ImgDesc> img;               // host parse (sizes, validation)
    std::vector<ScanDesc> scan;
    std::vector<uint8_t> level;             // [n][G] dependency level of each scan (1-based)
    std::vector<uint64_t> out_off, coef_off, mask_off;
    std::vector<uint32_t> slot_base, slot_cnt;
    uint64_t n_masks = 0; uint32_t n_slots = 0; uint32_t max_level = 0;
    DevRecord d{};
    Arena small, big;                       // descriptor tables (sized by n and G) / everything sized by the images, and the work lists
    uint8_t* d_rec = nullptr;
    PixelTile* d_tiles = nullptr; uint32_t n_tiles = 0;
    PixelTile* d_flat_tiles = nullptr; uint32_t n_flat_tiles = 0;   // runs of 8x8 pixel cells, for decodes of DC scans only
    uint32_t flat_row_cells = 0;                                    // cells per row of the widest image
    PixelTile* d_flat_rows = nullptr; uint32_t n_flat_rows = 0;     // ... and rows of cells (none if an image is too wide for k_pixel_flat_rows)
    uint32_t* d_dims = nullptr;             // [n][2] width, height (for kernels that run without a decode before them)
    bool prebuild_tables = false;           // some AC scan has restart intervals: k_build_tables runs before the entropy kernels
    int lane_mode = 0;                      // pcr_set_lane_decoders: 0 by the number of units, 1 wherever possible, -1 never
    int last_lane_launches = 0, last_wave_launches = 0;   // AC entropy launches of the last decode call, by decoder shape
    std::vector<uint32_t> ent_off_h;        // record offset of every scan's entry points (0: none), as uploaded
    std::vector<uint32_t> unit_bits;        // records opened from host bytes: entropy-coded bits of every unit, by slot (else empty)
    // decode fused with the training tail (allocated at its first call): one tile per MCU row, the side buffer of first
    // and last pixel rows, where each image's part of it starts, pixel rows per MCU row of every image
    PixelTile* d_tail_tiles = nullptr; uint32_t n_tail_tiles = 0;
    uint8_t* d_edge = nullptr; uint64_t* d_edge_off = nullptr; uint32_t* d_mcu_px_h = nullptr;
    float2* d_ssim_part = nullptr;          // per-tile sums of the similarity kernels (allocated at their first call)
    uint8_t* d_planes = nullptr;            // rounded samples per component, for pcr_decode_batch_triangle (allocated at its first call)
    uint32_t ssim_tiles_max = 0;
    uint8_t* d_gather = nullptr; size_t gather_cap = 0;
    std::map<int, Plan> plans;
    bool timing = false;
    int resident_k = 0;                        // scan group whose planes and masks the last pixel decode left behind (0: none)
    bool borrowed = false;                  // record bytes belong to the caller (pcr_open_device)
    // stage timing: one list of events per call, the last kTimingRing calls are kept
    std::vector<CallTiming> ring;
    uint64_t timed_calls = 0;                  // calls recorded since timing was switched on
    CallTiming* cur = nullptr;                 // the call being enqueued
};

namespace {

// level[g] = 1 + max level of an earlier scan that shares a component and overlaps in band
void compute_levels(pcr_record* r) {
    const uint32_t n = r->hdr.n, G = r->hdr.G;
    r->level.assign((size_t)n * G, 0);
    r->max_level = 0;
    for (uint32_t i = 0; i < n; i++) {
        const ScanDesc* s = &r->scan[(size_t)i * G];
        for (uint32_t g = 0; g < r->img[i].nscans; g++) {
            uint32_t lv = 1;
            for (uint32_t q = 0; q < g; q++) {
                bool share = false;
                for (int a = 0; a < s[g].ns; a++) for (int b = 0; b < s[q].ns; b++) if (s[g].comp[a] == s[q].comp[b]) share = true;
                if (share && s[q].Ss <= s[g].Se && s[g].Ss <= s[q].Se) lv = std::max<uint32_t>(lv, r->level[(size_t)i * G + q] + 1u);
            }
            r->level[(size_t)i * G + g] = (uint8_t)lv;
            r->max_level = std::max(r->max_level, lv);
        }
    }
}

// Launch geometry for decoding scan groups k0+1 .. k (k0 = 0: from scratch) and turning groups 1 .. k into pixels.
int build_plan(pcr_record* r, int k0, int k, Plan** out) {
    const int key = k0 * 256 + k;
    auto it = r->plans.find(key);
    if (it != r->plans.end()) { *out = &it->second; return PCR_OK; }
    const uint32_t n = r->hdr.n, G = r->hdr.G;
    Plan plan;
    struct Item { Unit u; uint32_t bytes; uint32_t bits; };      // bytes: the scan's mean per unit; bits: the unit's own, if known
    // one list per (dependency level, kind of scan, DC decoder shape: 0 for the AC kinds)
    std::vector<std::vector<Item>> lists((size_t)r->max_level * kNumKinds * kDcShapes);
    // ... and, per list, the runs of units that belong to one scan (first item, count, the scan's mean bytes per unit):
    // ordering a list scan by scan moves whole runs, a few thousand of them, not hundreds of thousands of units
    struct Run { uint32_t first, count, bytes; };
    std::vector<std::vector<Run>> runs(lists.size());
    std::vector<std::vector<RefineScan>> rlists(r->max_level);
    std::vector<ApplyUnit> apply; uint32_t max_blk = 0;
    for (uint32_t i = 0; i < n; i++) {
        const uint32_t upto = std::min<uint32_t>(r->img[i].nscans, (uint32_t)k);
        bool refine[kMaxComp] = {false, false, false};
        uint32_t have_dc = 0;
        for (uint32_t g = 0; g < upto; g++) {
            const size_t ig = (size_t)i * G + g;
            const ScanDesc& sd = r->scan[ig];
            if (sd.Ah > 0) for (int j = 0; j < sd.ns; j++) refine[sd.comp[j]] = true;
            if (sd.Ss == 0 && sd.Ah == 0) for (int j = 0; j < sd.ns; j++) have_dc |= 1u << sd.comp[j];
            const bool seq = is_sequential_scan(sd);
            if (sd.Ss > 0 || seq) { plan.has_ac = true; if (g < (uint32_t)k0) plan.had_ac = true; }
            if (g < (uint32_t)k0) continue;                    // decoded by an earlier call
            if (sd.Ss == 0 && sd.Ah > 0) continue;             // DC refinement has no serial decode
            const int kind = seq ? kSequential : (sd.Ss == 0 ? kDcFirst : (sd.Ah == 0 ? kAcFirst : kAcRefine));
            if (kind == kAcRefine) {
                rlists[r->level[ig] - 1].push_back(RefineScan{i, g});
            }
            int shape = 0;
            if (kind == kDcFirst) {
                uint32_t hs[kMaxComp] = {1, 1, 1}, vs[kMaxComp] = {1, 1, 1};
                for (int j = 0; j < sd.ns && j < kMaxComp; j++) { hs[j] = r->img[i].hs[sd.comp[j]]; vs[j] = r->img[i].vs[sd.comp[j]]; }
                shape = dc_shape(sd.ns, hs[0], vs[0], hs[1], vs[1], hs[2], vs[2]);
            }
            const uint32_t cnt = r->slot_cnt[ig];
            const size_t li = ((size_t)(r->level[ig] - 1) * kNumKinds + kind) * kDcShapes + shape;
            if (cnt) runs[li].push_back(Run{(uint32_t)lists[li].size(), cnt, sd.data_len / cnt});
            for (uint32_t j = 0; j < cnt; j++)
                lists[li].push_back(Item{Unit{i, g, j, r->slot_base[ig]}, sd.data_len / cnt, r->unit_bits.empty() ? sd.data_len / cnt * 8 : r->unit_bits[r->slot_base[ig] + j]});
        }
        if (have_dc != (1u << r->img[i].nc) - 1u) plan.dc_complete = false;
        for (int c = 0; c < r->img[i].nc; c++) if (refine[c]) {
            apply.push_back(ApplyUnit{i, (uint32_t)c});
            max_blk = std::max<uint32_t>(max_blk, (uint32_t)r->img[i].bw[c] * r->img[i].bh[c]);
        }
    }
    for (size_t li = 0; li < lists.size(); li++) {
        if (lists[li].empty()) continue;
        std::vector<Item> l;                                          // the list with the scans of the longest units first
        {
            auto& rn = runs[li];
            std::stable_sort(rn.begin(), rn.end(), [](const Run& a, const Run& b) { return a.bytes > b.bytes; });
            l.reserve(lists[li].size());
            for (const Run& q : rn) l.insert(l.end(), lists[li].begin() + q.first, lists[li].begin() + q.first + q.count);
            std::vector<Item>().swap(lists[li]);
        }
        const int kind_of_list = (int)((li / kDcShapes) % kNumKinds);
        std::vector<LaneJob> jobs;
        if (kind_of_list == kAcFirst || kind_of_list == kAcRefine) {
            // Jobs of the lane-per-unit kernels.  A wavefront takes as long as its longest lane, and it holds kLaneTabs
            // Huffman tables: the list (scan after scan, the scans ordered by their mean unit) is cut into windows of
            // kLaneTabs scans, the units of a window are ordered by their own length, and every 64 of them are a job.
            size_t w0 = 0;
            while (w0 < l.size()) {
                LaneJob proto{}; size_t w1 = w0;
                while (w1 < l.size()) {
                    const uint32_t key = l[w1].u.img * G + l[w1].u.scan;
                    if (proto.ntab == 0 || proto.key[proto.ntab - 1] != key) {
                        if (proto.ntab == (uint32_t)kLaneTabs) break;
                        proto.key[proto.ntab++] = key;
                    }
                    w1++;
                }
                // (without the units' own lengths -- a record opened from device memory -- every unit carries its scan's mean,
                // and the scans are in that order already)
                if (!r->unit_bits.empty()) std::stable_sort(l.begin() + w0, l.begin() + w1, [](const Item& a, const Item& b) { return a.bits > b.bits; });
                for (size_t e = w0; e < w1; e += kEntropyLanes) {
                    LaneJob j = proto;
                    j.first = (uint32_t)e; j.count = (uint32_t)std::min<size_t>(kEntropyLanes, w1 - e);
                    jobs.push_back(j);
                }
                w0 = w1;
            }
        }
        std::vector<Unit> units(l.size());
        for (size_t e = 0; e < l.size(); e++) units[e] = l[e].u;
        LevelList ll; ll.n = (uint32_t)units.size(); ll.kind = kind_of_list; ll.shape = (int)(li % kDcShapes);
        int rc = arena_upload(&r->big, &ll.d_units, units); if (rc) return rc;
        if (!jobs.empty()) {
            ll.n_jobs = (uint32_t)jobs.size();
            rc = arena_upload(&r->big, &ll.d_jobs, jobs); if (rc) return rc;
        }
        if (ll.kind == kAcRefine) {
            const size_t lv = li / kDcShapes / kNumKinds;
            const auto& rl = rlists[lv];
            ll.n_refine = (uint32_t)rl.size();
            rc = arena_upload(&r->big, &ll.d_refine, rl); if (rc) return rc;
            std::vector<RefineTile> plane_tiles, cov_tiles;
            for (uint32_t e = 0; e < ll.n_refine; e++) {
                const ImgDesc& im = r->img[rl[e].img];
                const int c = r->scan[(size_t)rl[e].img * G + rl[e].scan].comp[0];
                const uint32_t plane = (uint32_t)im.bw[c] * im.bh[c], cov = (uint32_t)im.cw[c] * im.ch[c];
                for (uint32_t ch = 0; ch * 256 < plane; ch++) plane_tiles.push_back(RefineTile{e, ch});
                for (uint32_t ch = 0; ch * 256 < cov; ch++) cov_tiles.push_back(RefineTile{e, ch});
            }
            ll.n_plane_tiles = (uint32_t)plane_tiles.size(); ll.n_cov_tiles = (uint32_t)cov_tiles.size();
            if (ll.n_plane_tiles) { rc = arena_upload(&r->big, &ll.d_plane_tiles, plane_tiles); if (rc) return rc; }
            if (ll.n_cov_tiles) { rc = arena_upload(&r->big, &ll.d_cov_tiles, cov_tiles); if (rc) return rc; }
        }
        plan.levels.push_back(ll);
    }
    plan.n_apply = (uint32_t)apply.size();
    plan.apply_grid_x = (max_blk * 64 + kApplyChunk - 1) / kApplyChunk;
    if (plan.n_apply) {
        int rc = arena_upload(&r->big, &plan.d_apply, apply); if (rc) return rc;
        std::vector<int32_t> list_idx((size_t)n * kMaxComp, -1);
        for (size_t e = 0; e < apply.size(); e++) list_idx[(size_t)apply[e].img * kMaxComp + apply[e].comp] = (int32_t)e;
        rc = arena_upload(&r->big, &plan.d_list_idx, list_idx); if (rc) return rc;
        rc = arena_alloc(&r->big, &plan.d_apply_lists, apply.size()); if (rc) return rc;
    }
    auto ins = r->plans.emplace(key, plan);
    *out = &ins.first->second;
    return PCR_OK;
}

void free_plans(pcr_record* r) { r->plans.clear(); }        // (their device arrays belong to the arena)

int check_scan_group(const pcr_record* r, int k) {
    if (k < 1 || k > (int)r->hdr.G) return PCR_E_RANGE;
    if (k > (int)r->hdr.k_avail) return PCR_E_TRUNCATED;
    return PCR_OK;
}

// Stage timing.  call_begin records the start event, mark(stage) closes an interval that belongs to
// `stage` (one mark per kernel for the entropy kernels and the pixel kernel, so that a stage's time
// divided by its marks is the average duration of that kernel), call_end files the call.
void mark(pcr_record* r, int stage, hipStream_t s) {
    CallTiming* c = r->cur;
    if (!c) return;
    if (c->used == c->ev.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { r->cur = nullptr; c->used = 0; return; }
        c->ev.push_back(e); c->stage.push_back(0);
    }
    c->stage[c->used] = (uint8_t)stage;
    (void)hipEventRecord(c->ev[c->used++], s);
}
void call_begin(pcr_record* r, hipStream_t s) {
    r->cur = nullptr;
    if (!r->timing) return;
    if (r->ring.empty()) r->ring.resize(kTimingRing);
    r->cur = &r->ring[r->timed_calls % kTimingRing];
    r->cur->used = 0;
    mark(r, 0, s);
}
void call_end(pcr_record* r) { if (r->cur) { r->timed_calls++; r->cur = nullptr; } }

// adds the per-stage milliseconds and marks of one recorded call; waits for that call to finish
int add_call_times(const CallTiming& c, double* ms, uint32_t* marks) {
    if (c.used < 2) return PCR_OK;
    HIP_TRY(hipEventSynchronize(c.ev[c.used - 1]));
    for (size_t i = 1; i < c.used; i++) {
        float t = 0;
        HIP_TRY(hipEventElapsedTime(&t, c.ev[i - 1], c.ev[i]));
        ms[c.stage[i]] += t; marks[c.stage[i]]++;
    }
    return PCR_OK;
}

// One lane per unit or one wavefront per unit?  The wavefront decoders are bound by scalar instruction issue over all
// units of a launch (about 14 instructions per symbol, 256 issued per cycle), the lane decoders (pcr_lanes.h) by the
// latency of one symbol after another in the longest unit of a wavefront (about a microsecond per symbol), with a
// fifth of the instructions in total.  A launch that has the GPU to itself is therefore faster with lanes only from
// some tens of thousands of units on (measured on 1024-image records with an entry every 128 MCUs, every 64 in refinement
// scans: 53, 58 and 40 thousand units per launch, a record alone 5.4 ms against 6.6); a launch that shares the GPU with
// the decodes of other records (other streams) already from a few thousand, because what it leaves idle the others use:
// four records in flight decode twice as fast with lanes.  The library cannot see what
// else runs on the device; it takes the number of records the process has open as the sign of it.
// The lane kernels read the Huffman tables from memory: the tables must be pre-built.
constexpr uint32_t kLanesMinUnitsShared = 8192, kLanesMinUnitsAlone = 32768;
bool lanes_pay(const pcr_record* r, const LevelList& l) {
    if (!r->prebuild_tables || r->lane_mode < 0 || l.n_jobs == 0) return false;
    if (r->lane_mode > 0) return true;
    const uint32_t least = g_open_records.load(std::memory_order_relaxed) > 1 ? kLanesMinUnitsShared : kLanesMinUnitsAlone;
    return l.n >= least && l.n >= 32u * l.n_jobs;            // (jobs half full at least: few tables per 64 units)
}

// The same question for a launch of DC first scans.  A lane decodes a DC symbol with a fifth of the instructions a
// wavefront spends on it, but a launch of lanes takes as long as one unit, however few there are: it pays when the
// wavefront decoders of several records would queue for the scalar units.
constexpr uint32_t kDcLanesMinUnits = 4096;
bool dc_lanes_pay(const pcr_record* r, const LevelList& l) {
    if (r->lane_mode < 0) return false;
    if (r->lane_mode > 0) return l.n >= (uint32_t)kEntropyLanes;
    return g_open_records.load(std::memory_order_relaxed) > 1 && l.n >= kDcLanesMinUnits;
}

// Steps 1-5 of the path (index .. entropy decode + refinement) for scans 1..k.
// refine_in_memory: also run k_apply, which leaves the refined coefficients in the planes (the coefficient
// export needs that; the pixel kernel replays the refinement itself from the lists of k_apply_prep).
// k0 > 0: a fidelity upgrade -- groups 1 .. k0 are in the planes and masks already, only k0+1 .. k are decoded.
int run_entropy_stages(pcr_record* r, int k0, int k, hipStream_t s, bool refine_in_memory, Plan** plan_out) {
    Plan* plan = nullptr;
    int rc = build_plan(r, k0, k, &plan);
    if (rc) return rc;
    *plan_out = plan;
    const uint32_t n = r->hdr.n;
    call_begin(r, s);
    hipLaunchKernelGGL(k_index, dim3(k), dim3(256), 0, s, r->d, (uint32_t)k);
    hipLaunchKernelGGL(k_parse, dim3((n + 63) / 64), dim3(64), 0, s, r->d, (uint32_t)k, (uint32_t)(k0 > 0));
    r->d.tabs_prebuilt = r->prebuild_tables ? 1u : 0u;
    // (the wavefront decoders of DC first scans read pre-built tables, the lane decoder makes its own: when every launch
    // of DC first scans of this call goes to the lanes their tables are not built, and with DC first scans only, none are)
    // (decided once per call: the answer depends on how many records the process has open, which another thread may change)
    bool dc_tables = false;
    std::vector<char> dc_by_lanes(plan->levels.size(), 0);
    for (size_t li = 0; li < plan->levels.size(); li++) {
        const LevelList& l = plan->levels[li];
        if (l.kind != kDcFirst || !l.n) continue;
        dc_by_lanes[li] = dc_lanes_pay(r, l) ? 1 : 0;
        if (!dc_by_lanes[li]) dc_tables = true;
    }
    if (r->prebuild_tables && k > k0 && (dc_tables || plan->has_ac))
        hipLaunchKernelGGL(k_build_tables, dim3(n, k - k0), dim3(kEntropyLanes), 0, s, r->d, (uint32_t)k0, dc_tables ? 1u : 0u);
    mark(r, PCR_STAGE_INDEX_PARSE, s);
    if (k > k0) hipLaunchKernelGGL(k_unstuff, dim3(n, k - k0), dim3(256), 0, s, r->d, (uint32_t)k0, (uint32_t)k);
    const size_t coef_bytes = r->coef_off[n] * sizeof(int16_t);
    // AC first scans only write the coefficients they decode: everything else must read as zero.  With DC scans
    // only, the pixel kernels read nothing of the planes, so the fill is skipped (the coefficient export shows whole
    // planes and always needs it).  The mask planes need no fill: every entry a kernel reads was written earlier in
    // the same call.  An upgrade keeps the planes; when it brings the first AC scans they are cleared first.
    // The DC first scans write a compact copy of the DC coefficients (one per block), which is what every pixel kernel
    // reads; the planes get them too only for the coefficient export: 2-byte stores 128 bytes apart were measured to
    // cost the DC scan a third of its time and to slow the kernels that run beside it.
    const bool dc_to_planes = refine_in_memory;
    if (k0 == 0 ? (plan->has_ac || refine_in_memory) : (plan->has_ac && !plan->had_ac))
        hipLaunchKernelGGL(k_fill_zero, dim3(2048), dim3(256), 0, s, (uint4*)r->d.coef, coef_bytes / 16);
    if (k0 == 0 && !plan->dc_complete)                       // a component whose DC scan is not among the scans decoded reads as zero
        hipLaunchKernelGGL(k_fill_zero, dim3(256), dim3(256), 0, s, (uint4*)r->d.dc, (r->coef_off[n] / 64 * sizeof(int16_t) + 15) / 16);
    mark(r, PCR_STAGE_UNSTUFF, s);
    const uint32_t* c32 = reinterpret_cast<const uint32_t*>(r->d.clean);
    const uint64_t* h64 = r->d.masks;
    r->last_lane_launches = r->last_wave_launches = 0;
    for (size_t li = 0; li < plan->levels.size(); li++) {
        auto& l = plan->levels[li];
        const dim3 grid(l.n), block(kEntropyLanes);
        if (l.kind == kAcFirst || l.kind == kAcRefine) { if (lanes_pay(r, l)) r->last_lane_launches++; else r->last_wave_launches++; }
        if (l.kind == kDcFirst && dc_by_lanes[li]) {
            hipLaunchKernelGGL(k_dc_first_lanes, dim3((l.n + kEntropyLanes - 1) / kEntropyLanes), block, 0, s, r->d, l.d_units, l.n, c32, dc_to_planes ? 1u : 0u);
            mark(r, PCR_STAGE_DC_FIRST, s);
        }
        else if (l.kind == kDcFirst) {
            const uint32_t dcp = dc_to_planes ? 1u : 0u;
            switch (l.shape) {
                case 1: hipLaunchKernelGGL(k_dc_first<1>, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64, dcp); break;
                case 2: hipLaunchKernelGGL(k_dc_first<2>, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64, dcp); break;
                case 3: hipLaunchKernelGGL(k_dc_first<3>, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64, dcp); break;
                case 4: hipLaunchKernelGGL(k_dc_first<4>, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64, dcp); break;
                default: hipLaunchKernelGGL(k_dc_first<0>, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64, dcp); break;
            }
            mark(r, PCR_STAGE_DC_FIRST, s);
        }
        else if (l.kind == kSequential) { hipLaunchKernelGGL(k_sequential, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64); mark(r, PCR_STAGE_SEQUENTIAL, s); }
        else if (l.kind == kAcFirst) {
            if (lanes_pay(r, l)) hipLaunchKernelGGL(k_ac_first_lanes, dim3(l.n_jobs), block, 0, s, r->d, l.d_units, l.d_jobs, c32);
            else hipLaunchKernelGGL(k_ac_first, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64);
            mark(r, PCR_STAGE_AC_FIRST, s);
        }
        else if (lanes_pay(r, l)) {
            if (l.n_plane_tiles) hipLaunchKernelGGL(k_refine_history, dim3(l.n_plane_tiles), dim3(256), 0, s, r->d, l.d_refine, l.d_plane_tiles);
            mark(r, PCR_STAGE_REFINE_BLOCKS, s);
            hipLaunchKernelGGL(k_ac_refine_lanes, dim3(l.n_jobs), block, 0, s, r->d, l.d_units, l.d_jobs, c32);
            mark(r, PCR_STAGE_AC_REFINE, s);
            if (l.n_cov_tiles) hipLaunchKernelGGL(k_refine_deal, dim3(l.n_cov_tiles), dim3(256), 0, s, r->d, l.d_refine, l.d_cov_tiles);
            mark(r, PCR_STAGE_REFINE_BLOCKS, s);
        }
        else {
            hipLaunchKernelGGL(k_ac_refine, grid, block, 0, s, r->d, l.d_units, l.n, c32, h64);
            mark(r, PCR_STAGE_AC_REFINE, s);
            if (l.n_cov_tiles) hipLaunchKernelGGL(k_refine_blocks, dim3(l.n_cov_tiles), dim3(256), 0, s, r->d, l.d_refine, l.d_cov_tiles);
            mark(r, PCR_STAGE_REFINE_BLOCKS, s);
        }
    }
    if (plan->n_apply) {
        hipLaunchKernelGGL(k_apply_prep, dim3((plan->n_apply + 63) / 64), dim3(64), 0, s, r->d, plan->d_apply, plan->n_apply, (uint32_t)k, plan->d_apply_lists);
        if (refine_in_memory)
            hipLaunchKernelGGL(k_apply, dim3(plan->apply_grid_x, plan->n_apply), dim3(256), 0, s, r->d, plan->d_apply, plan->d_apply_lists);
    }
    if (plan->n_apply) mark(r, PCR_STAGE_REFINE_APPLY, s);
    if (hipGetLastError() != hipSuccess) { r->cur = nullptr; return PCR_E_DEVICE; }
    return PCR_OK;
}

}  // namespace

extern "C" {

// Host-side validation of the metadata block: region lengths must tile every available group and
// agree with the per-image scan counts.  hdr: host copy of the first header_bytes bytes.
static int validate_index(const uint8_t* hdr, const RecordHeader& h, std::vector<uint32_t>* off, std::vector<uint32_t>* len, std::vector<uint32_t>* nsc) {
    const uint32_t n = h.n, G = h.G;
    off->assign((size_t)G * n, 0); len->assign((size_t)G * n, 0); nsc->assign(n, 0);
    uint64_t start = h.header_bytes;
    for (uint32_t g = 0; g < h.k_avail; g++) {
        uint64_t pos = start;
        for (uint32_t i = 0; i < n; i++) {
            uint32_t L = ld_le32(hdr + hdr_len_pos(n, G, g, i));
            (*off)[(size_t)g * n + i] = (uint32_t)pos; (*len)[(size_t)g * n + i] = L; pos += L;
        }
        if (h.version == 2)                                       // the group's entry points lie behind its regions
            for (uint32_t i = 0; i < n; i++) pos += entry_bytes(ld_le16(hdr + hdr_ecount_pos(n, G, g, i)));
        if (pos != ld_le64(hdr + hdr_group_end_pos(g))) return PCR_E_FORMAT;
        start = pos;
    }
    for (uint32_t i = 0; i < n; i++) {
        (*nsc)[i] = ld_le32(hdr + hdr_nscans_pos(n, G, i));
        if ((*nsc)[i] == 0 || (*nsc)[i] > G) return PCR_E_FORMAT;
        for (uint32_t g = 0; g < h.k_avail; g++)
            if ((g < (*nsc)[i]) != ((*len)[(size_t)g * n + i] != 0)) return PCR_E_FORMAT;
    }
    return PCR_OK;
}

// Everything after the image/scan descriptors are known (r->img, r->scan filled, r->d.rec set):
// dependency levels, buffer layout, the buffers themselves (out of r->big), their initial contents.
// Fills are enqueued on s; the caller synchronises s before anything else uses the handle.
static int finish_open(pcr_record* r, hipStream_t s) {
    const uint32_t n = r->hdr.n, G = r->hdr.G;
    const size_t nbytes = r->nbytes;
    for (uint32_t i = 0; i < n; i++) if (r->img[i].status != kOk) return r->img[i].status;
    compute_levels(r);
    r->out_off.assign(n + 1, 0); r->coef_off.assign(n + 1, 0);
    r->mask_off.assign((size_t)n * G, 0); r->slot_base.assign((size_t)n * G, 0); r->slot_cnt.assign((size_t)n * G, 0);
    std::vector<PixelTile> tiles, flat_tiles, flat_rows;
    bool rows_fit = true;
    r->flat_row_cells = 0;
    uint64_t nm = 0; uint64_t ns = 0;
    std::vector<uint32_t> tab_idx((size_t)n * G, 0); uint32_t ntabs = 0;
    std::vector<uint32_t> dctab_idx((size_t)n * G, 0); uint32_t ndctabs = 0;
    r->prebuild_tables = false;
    // version 2: where the entry points of every scan lie (behind the regions of the scan's group)
    std::vector<uint32_t> ent_off((size_t)n * G, 0), ent_cnt((size_t)n * G, 0);
    if (r->hdr.version == 2) {
        const uint8_t* hdr = r->header.data();
        for (uint32_t g = 0; g < r->hdr.k_avail; g++) {
            uint64_t all = 0;
            for (uint32_t i = 0; i < n; i++) all += entry_bytes(ld_le16(hdr + hdr_ecount_pos(n, G, g, i)));
            uint64_t at = ld_le64(hdr + hdr_group_end_pos(g)) - all;                   // (validate_index: this is where the regions end)
            for (uint32_t i = 0; i < n; i++) {
                const uint32_t field = ld_le16(hdr + hdr_ecount_pos(n, G, g, i));
                ent_off[(size_t)i * G + g] = (uint32_t)at; ent_cnt[(size_t)i * G + g] = entry_count(field);
                at += entry_bytes(field);
            }
        }
    }
    for (uint32_t i = 0; i < n; i++) {
        const ImgDesc& d = r->img[i];
        r->out_off[i + 1] = r->out_off[i] + (uint64_t)d.W * d.H * d.nc;
        uint64_t cc = 0;
        for (int c = 0; c < d.nc; c++) {
            const uint64_t elems = (uint64_t)d.bw[c] * d.bh[c] * 64;
            if (elems >= (1ull << 32)) return PCR_E_UNSUPPORTED;       // the decoders index a plane with 32 bits
            cc += elems;
        }
        if (cc >= (1ull << 32)) return PCR_E_UNSUPPORTED;               // ... and an image's planes together
        r->coef_off[i + 1] = r->coef_off[i] + cc;
        for (uint32_t g = 0; g < d.nscans; g++) {
            const size_t ig = (size_t)i * G + g;
            const ScanDesc& sd = r->scan[ig];
            if (sd.Ss > 0) {
                r->mask_off[ig] = nm;
                nm += (uint64_t)d.bw[sd.comp[0]] * d.bh[sd.comp[0]] * (sd.Ah ? kRefWords : 0);   // one record per block of a refinement scan
                tab_idx[ig] = ntabs++;                       // (first scans use theirs only when the tables are built ahead)
            }
            uint32_t cnt = sd.ri ? (sd.mcus + sd.ri - 1) / sd.ri : 1;
            const bool serial = !(d.progressive && sd.Ss == 0 && sd.Ah > 0);          // (DC refinement is read in place, without units)
            if (sd.ri == 0 && serial && ent_cnt[ig] > 0) cnt = 1 + ent_cnt[ig];         // units start at the entry points
            else ent_off[ig] = 0;
            if (d.progressive && sd.Ss == 0 && sd.Ah == 0) { dctab_idx[ig] = ndctabs; ndctabs += kMaxComp; }
            if (cnt > 1 && (sd.Ss > 0 || d.progressive)) r->prebuild_tables = true;     // several units share a scan's tables: build them once
            r->slot_base[ig] = (uint32_t)ns; r->slot_cnt[ig] = cnt;
            ns += cnt + 1;
        }
        const uint32_t per = pixel_mcus_per_tile(d), mcus = (uint32_t)d.mcux * d.mcuy;       // runs of MCUs, one lane per block
        for (uint32_t m0 = 0; m0 < mcus; m0 += per) tiles.push_back(PixelTile{i, m0});
        for (uint32_t c0 = 0, cells = flat_cells(d.W, d.H); c0 < cells; c0 += kFlatLanes) flat_tiles.push_back(PixelTile{i, c0});
        rows_fit = rows_fit && flat_rows_fit(d.W);
        r->flat_row_cells = std::max(r->flat_row_cells, ((uint32_t)d.W + 7) >> 3);
        for (uint32_t cy = 0; cy * 8 < d.H; cy++) flat_rows.push_back(PixelTile{i, cy});
    }
    if (ns >= (1ull << 32)) return PCR_E_UNSUPPORTED;
    r->n_masks = nm; r->n_slots = (uint32_t)ns; r->n_tiles = (uint32_t)tiles.size(); r->n_flat_tiles = (uint32_t)flat_tiles.size();
    if (!rows_fit) flat_rows.clear();
    r->n_flat_rows = (uint32_t)flat_rows.size();

    DevRecord& d = r->d;
    const size_t padded = nbytes + 1024;      // slack: bit readers look ahead
    // what the buffers below take, plus room for the work lists of a few scan groups (16 bytes per unit,
    // 12 per image and component, ...): anything beyond that is allocated on its own
    size_t need = arena_round(padded) + arena_round(r->coef_off[n] * sizeof(int16_t)) + arena_round((r->coef_off[n] / 64 + 1) * sizeof(int16_t)) + arena_round((nm + 2) * sizeof(uint64_t)) +
                  arena_round((ns + 1) * sizeof(uint32_t)) + 2 * arena_round((n + 1) * sizeof(uint64_t)) +
                  4 * arena_round(((size_t)n * G + 1) * sizeof(uint64_t)) + arena_round((tiles.size() + 1) * sizeof(PixelTile)) + arena_round((flat_tiles.size() + 1) * sizeof(PixelTile)) + arena_round((flat_rows.size() + 1) * sizeof(PixelTile)) + arena_round((n + 1) * 8) +
                  arena_round(((size_t)ntabs + 1) * sizeof(AcTab)) + arena_round(((size_t)ndctabs + 1) * sizeof(DcTab)) + arena_round(((size_t)n * G + 1) * sizeof(uint32_t)) + arena_round(((size_t)n * G + 1) * sizeof(uint32_t));
    need += 8 * ((ns + (size_t)n * G) * sizeof(Unit) + (size_t)n * kMaxComp * 64) + (1u << 20);
    need += 8 * (r->coef_off[n] / 64 / 256 + (size_t)n * G) * 2 * sizeof(RefineTile);     // (the tile lists of the refinement helpers: one entry per 256 blocks)
    int rc = arena_reset(&r->big, need);
    if (!rc) rc = arena_alloc(&r->big, &d.clean, padded);
    if (!rc) rc = arena_alloc(&r->big, &d.coef, r->coef_off[n]);
    if (!rc) rc = arena_alloc(&r->big, &d.dc, r->coef_off[n] / 64 + 8);              // (+8: cleared in 16-byte units)
    if (!rc) rc = arena_alloc(&r->big, &d.masks, nm + 2);
    if (!rc) rc = arena_alloc(&r->big, &d.ivl_start, ns);
    uint64_t *d_coef_off = nullptr, *d_out_off = nullptr, *d_mask_off = nullptr; uint32_t *d_sb = nullptr, *d_sc = nullptr;
    if (!rc) rc = arena_upload(&r->big, &d_coef_off, r->coef_off);
    if (!rc) rc = arena_upload(&r->big, &d_out_off, r->out_off);
    if (!rc) rc = arena_upload(&r->big, &d_mask_off, r->mask_off);
    if (!rc) rc = arena_upload(&r->big, &d_sb, r->slot_base);
    if (!rc) rc = arena_upload(&r->big, &d_sc, r->slot_cnt);
    if (!rc) rc = arena_upload(&r->big, &r->d_tiles, tiles);
    if (!rc) rc = arena_upload(&r->big, &r->d_flat_tiles, flat_tiles);
    if (!rc) rc = arena_upload(&r->big, &r->d_flat_rows, flat_rows);
    std::vector<uint32_t> dims((size_t)n * 2);
    for (uint32_t i = 0; i < n; i++) { dims[2 * i] = (uint32_t)r->img[i].W; dims[2 * i + 1] = (uint32_t)r->img[i].H; }
    if (!rc) rc = arena_upload(&r->big, &r->d_dims, dims);
    uint32_t* d_tab_idx = nullptr;
    if (!rc) rc = arena_upload(&r->big, &d_tab_idx, tab_idx);
    uint32_t* d_dctab_idx = nullptr;
    if (!rc) rc = arena_upload(&r->big, &d_dctab_idx, dctab_idx);
    if (!rc) rc = arena_alloc(&r->big, &d.dctabs, (size_t)ndctabs);
    d.dctab_idx = d_dctab_idx;
    r->ent_off_h = ent_off; r->unit_bits.clear();
    uint32_t* d_ent_off = nullptr;
    if (!rc) rc = arena_upload(&r->big, &d_ent_off, ent_off);
    d.ent_off = d_ent_off;
    if (!rc) rc = arena_alloc(&r->big, &d.tabs, (size_t)ntabs);
    d.tab_idx = d_tab_idx;
    d.coef_off = d_coef_off; d.out_off = d_out_off; d.mask_off = d_mask_off; d.slot_base = d_sb; d.slot_cnt = d_sc;
    if (!rc && hipMemsetAsync(d.clean, 0xFF, padded, s) != hipSuccess) rc = PCR_E_DEVICE;
    // (the refinement records need no initial contents: every word a kernel reads was written earlier in the same
    // call, or by the call an upgrade builds on; consumers skip blocks outside the scans' own grids)
    if (!rc && hipMemsetAsync(d.ivl_start, 0, (ns ? ns : 1) * sizeof(uint32_t), s) != hipSuccess) rc = PCR_E_DEVICE;
    return rc;
}

// Buffers the index and parse kernels write (out of r->small); needed before the descriptors exist.
static int alloc_descriptor_buffers(pcr_record* r, hipStream_t s) {
    const uint32_t n = r->hdr.n, G = r->hdr.G;
    DevRecord& d = r->d;
    const size_t ng = (size_t)G * n;
    int rc = arena_reset(&r->small, arena_round((ng + 1) * sizeof(uint32_t)) + arena_round((n + 1) * sizeof(ImgDesc)) +
                                    arena_round((ng + 1) * sizeof(ScanDesc)) + arena_round((n + 1) * sizeof(int32_t)));
    if (!rc) rc = arena_alloc(&r->small, &d.off, ng);
    if (!rc) rc = arena_alloc(&r->small, &d.img, n);
    if (!rc) rc = arena_alloc(&r->small, &d.scan, ng);
    if (!rc) rc = arena_alloc(&r->small, &d.status, n);
    if (!rc && hipMemsetAsync(d.off, 0, ng * sizeof(uint32_t), s) != hipSuccess) rc = PCR_E_DEVICE;
    if (!rc && hipMemsetAsync(d.scan, 0, ng * sizeof(ScanDesc), s) != hipSuccess) rc = PCR_E_DEVICE;
    if (!rc && hipMemsetAsync(d.img, 0, (size_t)n * sizeof(ImgDesc), s) != hipSuccess) rc = PCR_E_DEVICE;
    d.n = n; d.G = G;
    d.len = (const uint32_t*)(d.rec + hdr_len_pos(n, G, 0, 0));
    d.nscans = (const uint32_t*)(d.rec + hdr_nscans_pos(n, G, 0));
    return rc;
}

// Entropy-coded bits of every unit, for records whose bytes the host has: the entry points say where the units of a scan
// start (the lane-per-unit kernels put units of like length into one wavefront).  Scans cut by restart markers, whose
// intervals only the unstuff kernel finds, get their mean.
static void measure_units(pcr_record* r, const uint8_t* bytes, size_t nbytes) {
    const uint32_t n = r->hdr.n, G = r->hdr.G;
    size_t slots = 0;
    for (size_t ig = 0; ig < (size_t)n * G; ig++) slots = std::max<size_t>(slots, (size_t)r->slot_base[ig] + r->slot_cnt[ig] + 1);
    r->unit_bits.assign(slots, 0);
    for (uint32_t i = 0; i < n; i++) {
        for (uint32_t g = 0; g < r->img[i].nscans && g < r->hdr.k_avail; g++) {
            const size_t ig = (size_t)i * G + g;
            const uint32_t cnt = r->slot_cnt[ig], sb = r->slot_base[ig], eo = r->ent_off_h[ig];
            const uint64_t all = (uint64_t)r->scan[ig].data_len * 8;
            const uint32_t stride = entry_stride(ld_le16(r->header.data() + hdr_ecount_pos(n, G, g, i)));
            if (eo && cnt > 1 && (size_t)eo + (size_t)stride * (cnt - 1) <= nbytes) {
                uint64_t prev = 0;
                for (uint32_t j = 0; j < cnt; j++) {
                    const uint64_t end = j + 1 < cnt ? ld_le32(bytes + eo + (size_t)stride * j + 4) : std::max<uint64_t>(all, prev);
                    r->unit_bits[sb + j] = (uint32_t)std::min<uint64_t>(end > prev ? end - prev : 0, 0xFFFFFFFFu);
                    prev = std::max(prev, end);
                }
            } else {
                for (uint32_t j = 0; j < cnt; j++) r->unit_bits[sb + j] = (uint32_t)(all / std::max<uint32_t>(cnt, 1));
            }
        }
    }
}

int pcr_open(const void* bytes_, size_t nbytes, int device_id, pcr_record** out) {
    if (!bytes_ || !out) return PCR_E_ARG;
    const uint8_t* bytes = (const uint8_t*)bytes_;
    RecordHeader h;
    int rc = parse_record_header(bytes, nbytes, &h);
    if (rc) return rc;
    if (nbytes >= (1ull << 32)) return PCR_E_UNSUPPORTED;
    if (h.k_avail == 0) return PCR_E_TRUNCATED;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device_id < 0 || device_id >= ndev) { (void)hipGetLastError(); return PCR_E_DEVICE; }
    HIP_TRY(hipSetDevice(device_id));

    pcr_record* r = new (std::nothrow) pcr_record();
    if (!r) return PCR_E_NOMEM;
    r->device = device_id; r->nbytes = nbytes; r->hdr = h;
    const uint32_t n = h.n, G = h.G;
    r->header.assign(bytes, bytes + h.header_bytes);
    std::vector<uint32_t> off, len, nsc;
    rc = validate_index(r->header.data(), h, &off, &len, &nsc);
    // host marker parse of every image: layout, work sizes, early rejection
    if (!rc) {
        r->img.resize(n); r->scan.assign((size_t)n * G, ScanDesc{});
        for (uint32_t i = 0; i < n && !rc; i++) {
            parse_image(bytes, off.data(), len.data(), n, i, nsc[i], h.k_avail, &r->img[i], &r->scan[(size_t)i * G]);
            rc = r->img[i].status;
        }
    }
    if (!rc && hipMalloc((void**)&r->d_rec, nbytes + 64) != hipSuccess) { (void)hipGetLastError(); rc = PCR_E_NOMEM; }
    if (!rc && hipMemcpy(r->d_rec, bytes, nbytes, hipMemcpyHostToDevice) != hipSuccess) rc = PCR_E_DEVICE;
    if (!rc && hipMemset(r->d_rec + nbytes, 0, 64) != hipSuccess) rc = PCR_E_DEVICE;
    if (!rc) { r->d.rec = r->d_rec; rc = alloc_descriptor_buffers(r, nullptr); }
    if (!rc) rc = finish_open(r, nullptr);
    if (!rc) measure_units(r, bytes, nbytes);
    if (!rc && hipStreamSynchronize(nullptr) != hipSuccess) rc = PCR_E_DEVICE;
    if (rc) { (void)hipGetLastError(); pcr_close(r); return rc; }
    *out = r;
    return PCR_OK;
}

// Binds handle r (fresh, or one whose earlier work has finished) to record bytes in device memory: header
// checks on the host, index and marker parse ON THE DEVICE (only the small descriptor tables come back),
// buffer layout.  Everything is enqueued on s, which is synchronised before returning.  On failure the
// handle holds no record (pcr_close is all that may follow).
static int bind_device(pcr_record* r, const void* d_bytes, size_t nbytes, hipStream_t s) {
    r->plans.clear(); r->resident_k = 0; r->hdr = RecordHeader{}; r->n_tiles = 0; r->n_flat_tiles = 0; r->n_flat_rows = 0;
    r->out_off.assign(1, 0); r->coef_off.assign(1, 0);        // until the bind succeeds the handle holds no record
    r->d_dims = nullptr; r->d_ssim_part = nullptr; r->ssim_tiles_max = 0; r->d_planes = nullptr;
    r->d_tail_tiles = nullptr; r->n_tail_tiles = 0; r->d_edge = nullptr; r->d_edge_off = nullptr; r->d_mcu_px_h = nullptr;
    // fixed part of the header, then the whole metadata block
    uint8_t fixed[24];
    HIP_TRY(hipMemcpyAsync(fixed, d_bytes, 24, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (fixed[0] != 'P' || fixed[1] != 'C' || fixed[2] != 'R' || fixed[3] != '1') return PCR_E_FORMAT;
    const uint64_t header_bytes = ld_le64(fixed + 16);
    if (header_bytes < 24 || header_bytes > (1ull << 31)) return PCR_E_FORMAT;
    if (header_bytes > nbytes) return PCR_E_TRUNCATED;
    r->header.resize(header_bytes);
    if (hipMemcpyAsync(r->header.data(), d_bytes, header_bytes, hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess) {
        (void)hipGetLastError(); return PCR_E_DEVICE;
    }
    RecordHeader h;
    int rc = parse_record_header(r->header.data(), nbytes, &h);
    if (!rc && h.k_avail == 0) rc = PCR_E_TRUNCATED;
    if (rc) return rc;
    r->nbytes = nbytes; r->hdr = h;
    const uint32_t n = h.n, G = h.G;
    std::vector<uint32_t> off, len, nsc;
    rc = validate_index(r->header.data(), h, &off, &len, &nsc);
    if (!rc) { r->d.rec = (const uint8_t*)d_bytes; rc = alloc_descriptor_buffers(r, s); }
    if (!rc) {
        hipLaunchKernelGGL(k_index, dim3(h.k_avail), dim3(256), 0, s, r->d, h.k_avail);
        hipLaunchKernelGGL(k_parse, dim3((n + 63) / 64), dim3(64), 0, s, r->d, h.k_avail, 0u);
        r->img.resize(n); r->scan.resize((size_t)n * G);
        if (hipMemcpyAsync(r->img.data(), r->d.img, n * sizeof(ImgDesc), hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipMemcpyAsync(r->scan.data(), r->d.scan, (size_t)n * G * sizeof(ScanDesc), hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) rc = PCR_E_DEVICE;
    }
    if (!rc) rc = finish_open(r, s);
    if (!rc && hipStreamSynchronize(s) != hipSuccess) rc = PCR_E_DEVICE;
    if (rc) { (void)hipGetLastError(); r->hdr = RecordHeader{}; r->n_tiles = 0; r->n_flat_tiles = 0; r->n_flat_rows = 0; }
    return rc;
}

static int check_device_bytes(const void* d_bytes, size_t nbytes, int* device) {
    if (!d_bytes) return PCR_E_ARG;
    if (((uintptr_t)d_bytes & 15) != 0) return PCR_E_ARG;              // header tables are read as aligned words
    if (nbytes < 24) return PCR_E_TRUNCATED;
    if (nbytes >= (1ull << 32)) return PCR_E_UNSUPPORTED;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, d_bytes) != hipSuccess) { (void)hipGetLastError(); return PCR_E_ARG; }
    if (attr.type != hipMemoryTypeDevice) return PCR_E_ARG;
    *device = attr.device;
    return PCR_OK;
}

int pcr_open_device(const void* d_bytes, size_t nbytes, void* stream, pcr_record** out) {
    if (!out) return PCR_E_ARG;
    int device = 0;
    int rc = check_device_bytes(d_bytes, nbytes, &device);
    if (rc) return rc;
    HIP_TRY(hipSetDevice(device));
    pcr_record* r = new (std::nothrow) pcr_record();
    if (!r) return PCR_E_NOMEM;
    r->device = device; r->borrowed = true;
    rc = bind_device(r, d_bytes, nbytes, (hipStream_t)stream);
    if (rc) { pcr_close(r); return rc; }
    *out = r;
    return PCR_OK;
}

int pcr_rebind_device(pcr_record* r, const void* d_bytes, size_t nbytes, void* stream) {
    if (!r) return PCR_E_ARG;
    int device = 0;
    int rc = check_device_bytes(d_bytes, nbytes, &device);
    if (rc) return rc;
    if (device != r->device) return PCR_E_ARG;
    HIP_TRY(hipSetDevice(device));
    if (!r->borrowed && r->d_rec) { (void)hipFree(r->d_rec); }             // the handle's own copy of its first record
    r->d_rec = nullptr; r->borrowed = true;
    return bind_device(r, d_bytes, nbytes, (hipStream_t)stream);
}

void pcr_close(pcr_record* r) {
    if (!r) return;
    (void)hipSetDevice(r->device);
    (void)hipDeviceSynchronize();
    free_plans(r);
    arena_free(&r->small); arena_free(&r->big);
    if (!r->borrowed && r->d_rec) (void)hipFree(r->d_rec);
    if (r->d_gather) (void)hipFree(r->d_gather);
    for (auto& c : r->ring) for (auto& e : c.ev) (void)hipEventDestroy(e);
    delete r;
}

int pcr_num_images(const pcr_record* r, int* n) { if (!r || !n) return PCR_E_ARG; *n = (int)r->hdr.n; return PCR_OK; }
int pcr_num_scan_groups(const pcr_record* r, int* G) { if (!r || !G) return PCR_E_ARG; *G = (int)r->hdr.G; return PCR_OK; }
int pcr_available_scan_groups(const pcr_record* r, int* k) { if (!r || !k) return PCR_E_ARG; *k = (int)r->hdr.k_avail; return PCR_OK; }

int pcr_group_end_offset(const pcr_record* r, int k, uint64_t* off) {
    if (!r || !off) return PCR_E_ARG;
    if (k < 1 || k > (int)r->hdr.G) return PCR_E_RANGE;
    *off = ld_le64(r->header.data() + hdr_group_end_pos((uint32_t)k - 1));
    return PCR_OK;
}

int pcr_image_info(const pcr_record* r, int i, int* w, int* h, int* c, int32_t* label) {
    if (!r) return PCR_E_ARG;
    if (i < 0 || i >= (int)r->hdr.n) return PCR_E_RANGE;
    if (w) *w = r->img[i].W;
    if (h) *h = r->img[i].H;
    if (c) *c = r->img[i].nc;
    if (label) *label = (int32_t)ld_le32(r->header.data() + hdr_label_pos(r->hdr.G, (uint32_t)i));
    return PCR_OK;
}

int pcr_output_layout(const pcr_record* r, uint64_t* offsets) {
    if (!r || !offsets) return PCR_E_ARG;
    if (r->out_off.size() != (size_t)r->hdr.n + 1) {           // a handle without a record (n = 0) has the one entry 0
        if (r->hdr.n) return PCR_E_ARG;
        offsets[0] = 0;
        return PCR_OK;
    }
    std::memcpy(offsets, r->out_off.data(), r->out_off.size() * sizeof(uint64_t));
    return PCR_OK;
}

int pcr_coef_layout(const pcr_record* r, uint64_t* offsets) {
    if (!r || !offsets) return PCR_E_ARG;
    if (r->coef_off.size() != (size_t)r->hdr.n + 1) {
        if (r->hdr.n) return PCR_E_ARG;
        offsets[0] = 0;
        return PCR_OK;
    }
    std::memcpy(offsets, r->coef_off.data(), r->coef_off.size() * sizeof(uint64_t));
    return PCR_OK;
}

int pcr_index(const pcr_record* r, uint64_t* off, uint32_t* len) {
    if (!r || !off || !len) return PCR_E_ARG;
    HIP_TRY(hipSetDevice(r->device));
    const uint32_t n = r->hdr.n, G = r->hdr.G, k = r->hdr.k_avail;
    hipLaunchKernelGGL(k_index, dim3(k), dim3(256), 0, 0, r->d, k);
    std::vector<uint32_t> o((size_t)G * n);
    HIP_TRY(hipMemcpy(o.data(), r->d.off, o.size() * sizeof(uint32_t), hipMemcpyDeviceToHost));
    std::vector<uint32_t> l((size_t)G * n);
    HIP_TRY(hipMemcpy(l.data(), r->d.len, l.size() * sizeof(uint32_t), hipMemcpyDeviceToHost));
    for (size_t e = 0; e < (size_t)k * n; e++) { off[e] = o[e]; len[e] = l[e]; }
    return PCR_OK;
}

int pcr_reassemble(pcr_record* r, int i, int k, uint8_t* dst, size_t cap, size_t* len) {
    if (!r || !len) return PCR_E_ARG;
    if (i < 0 || i >= (int)r->hdr.n) return PCR_E_RANGE;
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    const uint32_t n = r->hdr.n, G = r->hdr.G;
    const uint32_t ns = ld_le32(r->header.data() + hdr_nscans_pos(n, G, (uint32_t)i));
    const uint32_t have = std::min<uint32_t>(ns, (uint32_t)k);
    size_t total = 0;
    for (uint32_t g = 0; g < have; g++) total += ld_le32(r->header.data() + hdr_len_pos(n, G, g, (uint32_t)i));
    const int add_eoi = have < ns;
    total += add_eoi ? 2 : 0;
    if (!dst) { *len = total; return PCR_OK; }
    if (cap < total) return PCR_E_RANGE;
    HIP_TRY(hipSetDevice(r->device));
    if (r->gather_cap < total) {
        if (r->d_gather) (void)hipFree(r->d_gather);
        r->d_gather = nullptr; r->gather_cap = 0;
        if (hipMalloc((void**)&r->d_gather, total) != hipSuccess) return PCR_E_NOMEM;
        r->gather_cap = total;
    }
    hipLaunchKernelGGL(k_index, dim3(k), dim3(256), 0, 0, r->d, (uint32_t)k);
    hipLaunchKernelGGL(k_gather, dim3(64), dim3(256), 0, 0, r->d, (uint32_t)i, have, add_eoi, r->d_gather);
    HIP_TRY(hipMemcpy(dst, r->d_gather, total, hipMemcpyDeviceToHost));
    *len = total;
    return PCR_OK;
}

int pcr_set_lane_decoders(pcr_record* r, int mode) {
    if (!r || mode < -1 || mode > 1) return PCR_E_ARG;
    r->lane_mode = mode;
    return PCR_OK;
}

int pcr_last_decoder_shapes(pcr_record* r, int* lane_launches, int* wavefront_launches) {
    if (!r || !lane_launches || !wavefront_launches) return PCR_E_ARG;
    *lane_launches = r->last_lane_launches; *wavefront_launches = r->last_wave_launches;
    return PCR_OK;
}

int pcr_enable_stage_timing(pcr_record* r, int on) {
    if (!r) return PCR_E_ARG;
    r->timing = on != 0;
    r->timed_calls = 0;                        // switching on (again) starts a new history
    return PCR_OK;
}

int pcr_last_stage_ms(pcr_record* r, float* ms) {
    if (!r || !ms) return PCR_E_ARG;
    if (!r->timing || r->timed_calls == 0) return PCR_E_ARG;
    HIP_TRY(hipSetDevice(r->device));
    double sum[PCR_NUM_STAGES] = {}; uint32_t marks[PCR_NUM_STAGES] = {};
    int rc = add_call_times(r->ring[(r->timed_calls - 1) % kTimingRing], sum, marks);
    if (rc) return rc;
    for (int s = 0; s < PCR_NUM_STAGES; s++) ms[s] = (float)sum[s];
    return PCR_OK;
}

int pcr_stage_ms_history(pcr_record* r, double* sum_ms, uint32_t* launches, uint32_t* calls) {
    if (!r || !sum_ms || !launches || !calls) return PCR_E_ARG;
    if (!r->timing) return PCR_E_ARG;
    HIP_TRY(hipSetDevice(r->device));
    for (int s = 0; s < PCR_NUM_STAGES; s++) { sum_ms[s] = 0; launches[s] = 0; }
    const uint64_t have = r->timed_calls < kTimingRing ? r->timed_calls : kTimingRing;
    for (uint64_t j = 0; j < have; j++) {
        int rc = add_call_times(r->ring[(r->timed_calls - 1 - j) % kTimingRing], sum_ms, launches);
        if (rc) return rc;
    }
    *calls = (uint32_t)have;
    return PCR_OK;
}

int pcr_decode_coefficients(pcr_record* r, int k, int16_t* d_coef, void* stream) {
    if (!r || !d_coef) return PCR_E_ARG;
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    HIP_TRY(hipSetDevice(r->device));
    hipStream_t s = (hipStream_t)stream;
    Plan* plan = nullptr;
    r->resident_k = 0;                                       // k_apply refines the planes in place: nothing to upgrade from afterwards
    rc = run_entropy_stages(r, 0, k, s, true, &plan);
    if (rc) return rc;
    call_end(r);
    hipLaunchKernelGGL(k_export_natural, dim3(2048), dim3(256), 0, s, r->d.coef, d_coef, (size_t)r->coef_off[r->hdr.n]);
    if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
    return PCR_OK;
}

// k0 = 0: from scratch; k0 > 0: on top of the planes and masks a previous call left for scan group k0
static int decode_to_pixels(pcr_record* r, int k0, int k, uint8_t* out, size_t cap, void* stream, int32_t* d_status, const CropBox* boxes = nullptr,
                            bool smooth = false) {
    if (cap < r->out_off[r->hdr.n]) return PCR_E_RANGE;
    HIP_TRY(hipSetDevice(r->device));
    hipStream_t s = (hipStream_t)stream;
    Plan* plan = nullptr;
    r->resident_k = 0;
    int rc = run_entropy_stages(r, k0, k, s, false, &plan);
    if (rc) return rc;
    // smoothing: with DC first scans only, a kernel of its own; otherwise the predicted coefficients go into the planes
    // for the pixel kernel and are taken out again after it
    const bool smooth_flat = smooth && !plan->has_ac && !plan->n_apply && !boxes;
    if (smooth_flat) smooth = false;
    if (smooth) hipLaunchKernelGGL(k_smooth<false>, dim3(kSmoothGroups, r->hdr.n), dim3(256), 0, s, r->d);
    if (smooth_flat)
        hipLaunchKernelGGL(k_pixel_smooth_flat, dim3(r->n_flat_tiles), dim3(kFlatLanes), 0, s, r->d, r->d_flat_tiles, out);
    else if (plan->n_apply)
        hipLaunchKernelGGL((k_pixel<true, false>), dim3(r->n_tiles), dim3(kPixLanes), 0, s, r->d, r->d_tiles, out, plan->d_apply_lists, plan->d_list_idx, boxes);
    else if (plan->has_ac || smooth)
        hipLaunchKernelGGL((k_pixel<false, false>), dim3(r->n_tiles), dim3(kPixLanes), 0, s, r->d, r->d_tiles, out, (const ApplyList*)nullptr, (const int32_t*)nullptr, boxes);
    else if (r->n_flat_rows && !boxes)                       // DC scans only: every block is flat
        hipLaunchKernelGGL(k_pixel_flat_rows, dim3(r->n_flat_rows), dim3(kFlatRowLanes), flat_rows_lds(r->flat_row_cells), s, r->d, r->d_flat_rows, out, r->flat_row_cells);
    else
        hipLaunchKernelGGL(k_pixel_flat, dim3(r->n_flat_tiles), dim3(kFlatLanes), 0, s, r->d, r->d_flat_tiles, out, boxes);
    if (smooth) hipLaunchKernelGGL(k_smooth<true>, dim3(kSmoothGroups, r->hdr.n), dim3(256), 0, s, r->d);
    mark(r, PCR_STAGE_PIXEL, s);
    call_end(r);
    if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
    if (d_status) HIP_TRY(hipMemcpyAsync(d_status, r->d.status, r->hdr.n * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
    r->resident_k = k;
    return PCR_OK;
}

int pcr_decode_batch(pcr_record* r, int k, uint8_t* out, size_t cap, void* stream, int32_t* d_status) {
    if (!r || !out) return PCR_E_ARG;
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    return decode_to_pixels(r, 0, k, out, cap, stream, d_status);
}

int pcr_decode_batch_smooth(pcr_record* r, int k, uint8_t* out, size_t cap, void* stream, int32_t* d_status) {
    if (!r || !out) return PCR_E_ARG;
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    return decode_to_pixels(r, 0, k, out, cap, stream, d_status, nullptr, true);
}

int pcr_decode_batch_triangle(pcr_record* r, int k, uint8_t* out, size_t cap, void* stream, int32_t* d_status) {
    if (!r || !out) return PCR_E_ARG;
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    const uint32_t n = r->hdr.n;
    if (cap < r->out_off[n]) return PCR_E_RANGE;
    HIP_TRY(hipSetDevice(r->device));
    if (!r->d_planes) {                                      // one byte per coefficient slot
        rc = arena_alloc(&r->big, &r->d_planes, (size_t)r->coef_off[n] + 16);
        if (rc) return rc;
    }
    hipStream_t s = (hipStream_t)stream;
    Plan* plan = nullptr;
    r->resident_k = 0;
    rc = run_entropy_stages(r, 0, k, s, false, &plan);
    if (rc) return rc;
    if (plan->n_apply)
        hipLaunchKernelGGL((k_pixel<true, true>), dim3(r->n_tiles), dim3(kPixLanes), 0, s, r->d, r->d_tiles, r->d_planes, plan->d_apply_lists, plan->d_list_idx, (const CropBox*)nullptr);
    else
        hipLaunchKernelGGL((k_pixel<false, true>), dim3(r->n_tiles), dim3(kPixLanes), 0, s, r->d, r->d_tiles, r->d_planes, (const ApplyList*)nullptr, (const int32_t*)nullptr, (const CropBox*)nullptr);
    uint32_t items = 1;
    for (uint32_t i = 0; i < n; i++) items = std::max(items, (((uint32_t)r->img[i].W + 3) / 4) * (uint32_t)r->img[i].H);
    hipLaunchKernelGGL(k_triangle_rgb, dim3((items + 255) / 256, n), dim3(256), 0, s, r->d, (const uint8_t*)r->d_planes, out);
    mark(r, PCR_STAGE_PIXEL, s);
    call_end(r);
    if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
    if (d_status) HIP_TRY(hipMemcpyAsync(d_status, r->d.status, n * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
    r->resident_k = k;
    return PCR_OK;
}

int pcr_resident_scan_group(const pcr_record* r, int* k) {
    if (!r || !k) return PCR_E_ARG;
    *k = r->resident_k;
    return PCR_OK;
}

int pcr_upgrade_batch(pcr_record* r, int k, uint8_t* out, size_t cap, void* stream, int32_t* d_status) {
    if (!r || !out) return PCR_E_ARG;
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    if (r->resident_k < 1 || k < r->resident_k) return PCR_E_ARG;
    return decode_to_pixels(r, r->resident_k, k, out, cap, stream, d_status);
}

int pcr_crop_resize_batch(pcr_record* r, const uint8_t* d_pixels, const pcr_crop* d_crops, int out_h, int out_w,
                          const float* mean, const float* inv_std, void* d_out_f16, size_t out_capacity, void* stream) {
    if (!r || !d_pixels || !d_crops || !mean || !inv_std) return PCR_E_ARG;
    if (out_h < 1 || out_w < 1 || out_h > 8192 || out_w > 8192) return PCR_E_RANGE;      // (the kernel's fractions stay inside 32 bits)
    if (!d_out_f16) return PCR_E_ARG;
    const uint32_t n = r->hdr.n;
    if (n == 0 || !r->d_dims) return PCR_E_ARG;
    const int C = r->img[0].nc;
    for (uint32_t i = 1; i < n; i++) if (r->img[i].nc != C) return PCR_E_UNSUPPORTED;    // one tensor, one channel count
    if (out_capacity < (size_t)n * C * out_h * out_w * sizeof(__half)) return PCR_E_RANGE;
    HIP_TRY(hipSetDevice(r->device));
    static_assert(sizeof(pcr_crop) == sizeof(CropBox), "crop box layout");
    if (n > 65535) return PCR_E_UNSUPPORTED;                  // (images are the grid's third dimension)
    const dim3 grid(((uint32_t)out_w + 31) / 32, ((uint32_t)out_h + 7) / 8, n);
    hipLaunchKernelGGL(k_crop_resize, grid, dim3(256), 0, (hipStream_t)stream, r->d_dims, r->d.out_off, d_pixels, reinterpret_cast<const CropBox*>(d_crops),
                       out_h, out_w, C, mean[0], C > 1 ? mean[1] : 0.f, C > 2 ? mean[2] : 0.f,
                       inv_std[0], C > 1 ? inv_std[1] : 1.f, C > 2 ? inv_std[2] : 1.f, reinterpret_cast<__half*>(d_out_f16));
    if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
    return PCR_OK;
}

// Tiles, side buffer and tables of the fused decode + tail (once per bound record).
static int prepare_fused_tail(pcr_record* r) {
    if (r->d_tail_tiles) return PCR_OK;
    const uint32_t n = r->hdr.n;
    std::vector<PixelTile> tiles; std::vector<uint64_t> eoff(n + 1, 0); std::vector<uint32_t> mh(n);
    for (uint32_t i = 0; i < n; i++) {
        const ImgDesc& d = r->img[i];
        if (d.mcux > 1 && 2 * blocks_per_mcu(d) > (uint32_t)kTailLanes) return PCR_E_UNSUPPORTED;   // (a pass holds two MCUs at least)
        for (uint32_t my = 0; my < d.mcuy; my++) tiles.push_back(PixelTile{i, my * d.mcux});
        eoff[i + 1] = eoff[i] + (uint64_t)2 * d.mcuy * d.W * d.nc;
        mh[i] = 8u * d.vmax;
    }
    int rc = arena_upload(&r->big, &r->d_edge_off, eoff);
    if (!rc) rc = arena_upload(&r->big, &r->d_mcu_px_h, mh);
    if (!rc) rc = arena_alloc(&r->big, &r->d_edge, (size_t)eoff[n] + 16);
    PixelTile* dt = nullptr;
    if (!rc) rc = arena_upload(&r->big, &dt, tiles);
    if (rc) return rc;
    r->d_tail_tiles = dt; r->n_tail_tiles = (uint32_t)tiles.size();
    return PCR_OK;
}

int pcr_decode_crop_batch(pcr_record* r, int k, const pcr_crop* d_crops, uint8_t* d_pixels, size_t pixel_capacity, int out_h, int out_w,
                          const float* mean, const float* inv_std, void* d_out_f16, size_t out_capacity, void* stream, int32_t* d_status) {
    if (!r || !d_crops || !mean || !inv_std) return PCR_E_ARG;
    if (!d_pixels) {
        // No working buffer: decode and tail in one kernel, the full-resolution pixels stay on the chip.
        int rc = check_scan_group(r, k);
        if (rc) return rc;
        if (out_h < 1 || out_w < 1 || out_h > 8192 || out_w > 8192) return PCR_E_RANGE;
        if (!d_out_f16 || !r->d_dims) return PCR_E_ARG;
        const uint32_t n = r->hdr.n;
        const int C = r->img[0].nc;
        for (uint32_t i = 1; i < n; i++) if (r->img[i].nc != C) return PCR_E_UNSUPPORTED;
        if (n > 65535) return PCR_E_UNSUPPORTED;
        if (out_capacity < (size_t)n * C * out_h * out_w * sizeof(__half)) return PCR_E_RANGE;
        HIP_TRY(hipSetDevice(r->device));
        rc = prepare_fused_tail(r);
        if (rc) return rc;
        hipStream_t s = (hipStream_t)stream;
        Plan* plan = nullptr;
        r->resident_k = 0;
        rc = run_entropy_stages(r, 0, k, s, false, &plan);
        if (rc) return rc;
        TailParams P;
        P.out_h = out_h; P.out_w = out_w;
        for (int c = 0; c < 3; c++) { P.mean[c] = c < C ? mean[c] : 0.f; P.istd[c] = c < C ? inv_std[c] : 1.f; }
        static_assert(sizeof(pcr_crop) == sizeof(CropBox), "crop box layout");
        const CropBox* boxes = reinterpret_cast<const CropBox*>(d_crops);
        if (plan->n_apply)
            hipLaunchKernelGGL(k_pixel_tail<true>, dim3(r->n_tail_tiles), dim3(kTailLanes), 0, s, r->d, r->d_tail_tiles, plan->d_apply_lists, plan->d_list_idx,
                               boxes, P, reinterpret_cast<__half*>(d_out_f16), r->d_edge, r->d_edge_off);
        else
            hipLaunchKernelGGL(k_pixel_tail<false>, dim3(r->n_tail_tiles), dim3(kTailLanes), 0, s, r->d, r->d_tail_tiles, (const ApplyList*)nullptr,
                               (const int32_t*)nullptr, boxes, P, reinterpret_cast<__half*>(d_out_f16), r->d_edge, r->d_edge_off);
        hipLaunchKernelGGL(k_tail_edges, dim3((uint32_t)out_h, n), dim3(64), 0, s, r->d_dims, r->d_mcu_px_h, C, boxes, P, r->d_edge, r->d_edge_off,
                           reinterpret_cast<__half*>(d_out_f16));
        mark(r, PCR_STAGE_PIXEL, s);
        call_end(r);
        if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
        if (d_status) HIP_TRY(hipMemcpyAsync(d_status, r->d.status, n * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
        r->resident_k = k;
        return PCR_OK;
    }
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    // argument checks of the tail before anything is enqueued (it repeats them)
    if (out_h < 1 || out_w < 1 || out_h > 8192 || out_w > 8192) return PCR_E_RANGE;
    if (!d_out_f16 || !r->d_dims) return PCR_E_ARG;
    const uint32_t n = r->hdr.n;
    const int C = r->img[0].nc;
    for (uint32_t i = 1; i < n; i++) if (r->img[i].nc != C) return PCR_E_UNSUPPORTED;
    if (n > 65535) return PCR_E_UNSUPPORTED;
    if (out_capacity < (size_t)n * C * out_h * out_w * sizeof(__half)) return PCR_E_RANGE;
    rc = decode_to_pixels(r, 0, k, d_pixels, pixel_capacity, stream, d_status, reinterpret_cast<const CropBox*>(d_crops));
    if (rc) return rc;
    return pcr_crop_resize_batch(r, d_pixels, d_crops, out_h, out_w, mean, inv_std, d_out_f16, out_capacity, stream);
}

int pcr_msssim_batch(pcr_record* r, const uint8_t* d_a, const uint8_t* d_b, float* d_scores, void* stream) {
    if (!r || !d_a || !d_b || !d_scores) return PCR_E_ARG;
    const uint32_t n = r->hdr.n;
    if (n == 0 || !r->d_dims) return PCR_E_ARG;
    const int C = r->img[0].nc;
    if (C != 1 && C != 3) return PCR_E_UNSUPPORTED;
    for (uint32_t i = 1; i < n; i++) if (r->img[i].nc != C) return PCR_E_UNSUPPORTED;
    if (n > 65535) return PCR_E_UNSUPPORTED;                  // (images are the grid's second dimension)
    HIP_TRY(hipSetDevice(r->device));
    if (!r->d_ssim_part) {
        uint32_t tmax = 1;
        for (uint32_t i = 0; i < n; i++) tmax = std::max(tmax, ssim_tiles_all((uint32_t)r->img[i].W, (uint32_t)r->img[i].H));
        int rc = arena_alloc(&r->big, &r->d_ssim_part, (size_t)n * tmax);
        if (rc) return rc;
        r->ssim_tiles_max = tmax;
    }
    hipLaunchKernelGGL(k_ssim_tiles, dim3(r->ssim_tiles_max, n), dim3(256), 0, (hipStream_t)stream, r->d_dims, r->d.out_off, C, d_a, d_b,
                       r->d_ssim_part, r->ssim_tiles_max);
    hipLaunchKernelGGL(k_ssim_score, dim3(n), dim3(64), 0, (hipStream_t)stream, r->d_dims, r->d_ssim_part, r->ssim_tiles_max, d_scores);
    if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
    return PCR_OK;
}

// ---- similarity scores without any allocation ----
// The per-tile sums of the similarity kernels in a fixed array of the code object instead of the handle's
// arena, for callers that must not allocate (HIP graph capture, serving loops).  Every GPU holds its own copy
// of the array at its own address; host code never uses the array's name as an address, only the pointer
// hipGetSymbolAddress returned for that device.
constexpr size_t kStaticSsimTiles = 512 * 1024;                       // 4 MiB of float2 per device
static __device__ __align__(256) float2 scratch[kStaticSsimTiles];
constexpr int kStaticMaxDevices = 64;
static std::mutex g_scratch_mu;
static float2* g_scratch_ptr[kStaticMaxDevices] = {};

// the array's address on `device` (which must be current), looked up once per device
static int static_scratch(int device, float2** p) {
    if (device < 0 || device >= kStaticMaxDevices) return PCR_E_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) { (void)hipGetLastError(); return PCR_E_DEVICE; }
        g_scratch_ptr[device] = reinterpret_cast<float2*>(q);
    }
    *p = g_scratch_ptr[device];
    return PCR_OK;
}

int pcr_msssim_batch_static(pcr_record* r, const uint8_t* d_a, const uint8_t* d_b, float* d_scores, void* stream) {
    if (!r || !d_a || !d_b || !d_scores) return PCR_E_ARG;
    const uint32_t n = r->hdr.n;
    if (n == 0 || !r->d_dims) return PCR_E_ARG;
    const int C = r->img[0].nc;
    if (C != 1 && C != 3) return PCR_E_UNSUPPORTED;
    for (uint32_t i = 1; i < n; i++) if (r->img[i].nc != C) return PCR_E_UNSUPPORTED;
    if (n > 65535) return PCR_E_UNSUPPORTED;
    uint32_t tmax = 1;
    for (uint32_t i = 0; i < n; i++) tmax = std::max(tmax, ssim_tiles_all((uint32_t)r->img[i].W, (uint32_t)r->img[i].H));
    if ((uint64_t)n * tmax > kStaticSsimTiles) return PCR_E_RANGE;   // the record's tile sums do not fit the fixed array
    HIP_TRY(hipSetDevice(r->device));
    float2* part = nullptr;
    int rc = static_scratch(r->device, &part);
    if (rc) return rc;
    // (nothing to clear: every entry k_ssim_score reads is written by k_ssim_tiles in the same call)
    hipLaunchKernelGGL(k_ssim_tiles, dim3(tmax, n), dim3(256), 0, (hipStream_t)stream, r->d_dims, r->d.out_off, C, d_a, d_b, part, tmax);
    hipLaunchKernelGGL(k_ssim_score, dim3(n), dim3(64), 0, (hipStream_t)stream, r->d_dims, part, tmax, d_scores);
    if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
    return PCR_OK;
}

// ---- record creation (host only) ----
int pcr_scan_ends(const void* jpeg, size_t nbytes, uint64_t* ends, int max_ends, int* n_scans) {
    if (!jpeg || !ends || !n_scans || max_ends < 1) return PCR_E_ARG;
    const int s = enc::scan_ends((const uint8_t*)jpeg, nbytes, ends, max_ends);
    if (s <= 0) return PCR_E_FORMAT;
    *n_scans = s;
    return PCR_OK;
}

int pcr_record_size(const void* const* files, const size_t* sizes, uint32_t n, uint64_t* record_bytes, uint32_t* scan_groups) {
    if (!files || !sizes || !record_bytes) return PCR_E_ARG;
    enc::RecordPlan P;
    const int rc = enc::plan_record(files, sizes, n, &P);
    if (rc) return rc;
    *record_bytes = P.total;
    if (scan_groups) *scan_groups = P.G;
    return PCR_OK;
}

int pcr_record_write(const void* const* files, const size_t* sizes, const int32_t* labels, uint32_t n, void* out, size_t capacity, uint64_t* written) {
    if (!files || !sizes || !out) return PCR_E_ARG;
    enc::RecordPlan P;
    const int rc = enc::plan_record(files, sizes, n, &P);
    if (rc) return rc;
    if (written) *written = P.total;
    if (capacity < P.total) return PCR_E_RANGE;
    enc::write_record(P, files, labels, (uint8_t*)out);
    return PCR_OK;
}

int pcr_record_write_indexed(const void* const* files, const size_t* sizes, const int32_t* labels, uint32_t n, uint32_t entry_interval,
                             void* out, size_t capacity, uint64_t* written) {
    if (!files || !sizes || !out) return PCR_E_ARG;
    if (entry_interval < 1 || entry_interval > (1u << 20)) return PCR_E_RANGE;
    enc::IndexedPlan Q;
    const int rc = enc::plan_record_indexed(files, sizes, n, entry_interval, &Q);
    if (rc) return rc;
    if (written) *written = Q.P.total;
    if (capacity < Q.P.total) return PCR_E_RANGE;
    enc::write_record_indexed(Q, files, labels, (uint8_t*)out);
    return PCR_OK;
}

int pcr_transcode_progressive(const void* src_jpeg, size_t src_bytes, const int16_t* coef, size_t coef_count, uint32_t restart_interval,
                              void* out, size_t capacity, uint64_t* written) {
    if (!src_jpeg || !coef || !written) return PCR_E_ARG;
    std::vector<uint8_t> bytes;
    bytes.reserve(src_bytes + src_bytes / 4 + 1024);
    const int rc = enc::transcode_progressive((const uint8_t*)src_jpeg, src_bytes, coef, coef_count, restart_interval, &bytes);
    if (rc) return rc;
    *written = bytes.size();
    if (!out || capacity < bytes.size()) return PCR_E_RANGE;
    memcpy(out, bytes.data(), bytes.size());
    return PCR_OK;
}

int pcr_transcode_progressive_counted(const void* src_jpeg, size_t src_bytes, const int16_t* coef, size_t coef_count, uint32_t restart_interval,
                                      const uint32_t* counts, void* out, size_t capacity, uint64_t* written) {
    if (!src_jpeg || !coef || !written || !counts) return PCR_E_ARG;
    std::vector<uint8_t> bytes;
    bytes.reserve(src_bytes + src_bytes / 4 + 1024);
    const int rc = enc::transcode_progressive((const uint8_t*)src_jpeg, src_bytes, coef, coef_count, restart_interval, &bytes, counts);
    if (rc) return rc;
    *written = bytes.size();
    if (!out || capacity < bytes.size()) return PCR_E_RANGE;
    memcpy(out, bytes.data(), bytes.size());
    return PCR_OK;
}

int pcr_transcode_symbol_counts(const void* src_jpeg, size_t src_bytes, const int16_t* coef, size_t coef_count, uint32_t restart_interval,
                                uint32_t* counts) {
    if (!src_jpeg || !coef || !counts) return PCR_E_ARG;
    return enc::transcode_progressive((const uint8_t*)src_jpeg, src_bytes, coef, coef_count, restart_interval, nullptr, nullptr, counts);
}

int pcr_symbol_histograms(pcr_record* r, uint32_t restart_interval, uint32_t* d_hist, void* stream) {
    if (!r || !d_hist) return PCR_E_ARG;
    if (restart_interval > 65535) return PCR_E_RANGE;
    const int k = (int)r->hdr.k_avail;
    int rc = check_scan_group(r, k);
    if (rc) return rc;
    HIP_TRY(hipSetDevice(r->device));
    hipStream_t s = (hipStream_t)stream;
    Plan* plan = nullptr;
    r->resident_k = 0;                                       // the planes are refined in place, as for the coefficient export
    rc = run_entropy_stages(r, 0, k, s, true, &plan);
    if (rc) return rc;
    call_end(r);
    static_assert(PCR_HIST_ENTRIES == kHistPerImage, "header and kernel agree on the layout of the counts");
    hipLaunchKernelGGL(k_symbol_hist, dim3(r->hdr.n, kScriptScansMax), dim3(64), 0, s, (const ImgDesc*)r->d.img, (const int16_t*)r->d.coef, r->d.coef_off,
                       restart_interval, d_hist);
    if (hipGetLastError() != hipSuccess) return PCR_E_DEVICE;
    return PCR_OK;
}

int pcr_select_scan_group(pcr_record* r, float min_mean_score, uint8_t* d_work_a, uint8_t* d_work_b, size_t work_capacity, float* d_scores,
                          float* mean_by_group, int* scan_group, void* stream) {
    if (!r || !d_work_a || !d_work_b || !d_scores || !scan_group) return PCR_E_ARG;
    const uint32_t n = r->hdr.n;
    const int top = (int)r->hdr.k_avail;
    if (n == 0 || top < 1) return PCR_E_ARG;
    if (mean_by_group) for (int g = 0; g < (int)r->hdr.G; g++) mean_by_group[g] = -1.0f;
    int rc = pcr_decode_batch(r, top, d_work_b, work_capacity, stream, nullptr);              // the reference pictures
    if (rc) return rc;
    std::vector<float> host(n);
    *scan_group = top;
    for (int k = 1; k < top; k++) {
        rc = k == 1 ? pcr_decode_batch(r, 1, d_work_a, work_capacity, stream, nullptr) : pcr_upgrade_batch(r, k, d_work_a, work_capacity, stream, nullptr);
        if (!rc) rc = pcr_msssim_batch(r, d_work_a, d_work_b, d_scores, stream);
        if (rc) return rc;
        if (hipMemcpyAsync(host.data(), d_scores, n * sizeof(float), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess ||
            hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return PCR_E_DEVICE;
        double sum = 0; uint32_t cnt = 0;
        for (uint32_t i = 0; i < n; i++) if (host[i] == host[i]) { sum += host[i]; cnt++; }   // (images too small to score are NaN)
        const float mean = cnt ? (float)(sum / cnt) : 1.0f;
        if (mean_by_group) mean_by_group[k - 1] = mean;
        if (mean >= min_mean_score) { *scan_group = k; return PCR_OK; }
    }
    if (mean_by_group) mean_by_group[top - 1] = 1.0f;
    return PCR_OK;
}

int pcr_probe_scalar_issue_rate(int device_id, int waves_per_cu, double* ginst_per_s) {
    if (!ginst_per_s || waves_per_cu < 1 || waves_per_cu > 32) return PCR_E_ARG;
    HIP_TRY(hipSetDevice(device_id));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, device_id));
    const uint32_t grid = (uint32_t)prop.multiProcessorCount * (uint32_t)waves_per_cu, iters = 20000;
    uint32_t* d_out = nullptr;
    if (hipMalloc((void**)&d_out, grid * sizeof(uint32_t)) != hipSuccess) return PCR_E_NOMEM;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = PCR_OK;
    float ms = 0;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = PCR_E_DEVICE;
    for (int rep = 0; rep < 2 && rc == PCR_OK; rep++) {          // the first launch warms up
        (void)hipEventRecord(e0, nullptr);
        hipLaunchKernelGGL(k_probe_scalar, dim3(grid), dim3(64), 0, nullptr, d_out, iters, 1u);
        (void)hipEventRecord(e1, nullptr);
        if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = PCR_E_DEVICE;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(d_out);
    if (rc == PCR_OK) *ginst_per_s = (double)grid * iters * 16.0 / (ms * 1e-3) / 1e9;
    return rc;
}

int pcr_prefix_length(const void* first_bytes, size_t nbytes, int k, uint64_t* need) {
    if (!first_bytes || !need) return PCR_E_ARG;
    const uint8_t* b = (const uint8_t*)first_bytes;
    if (nbytes < 24) { *need = 24; return PCR_E_TRUNCATED; }
    if (b[0] != 'P' || b[1] != 'C' || b[2] != 'R' || b[3] != '1') return PCR_E_FORMAT;
    if (ld_le32(b + 4) != 1 && ld_le32(b + 4) != 2) return PCR_E_UNSUPPORTED;
    const uint32_t G = ld_le32(b + 12);
    if (k < 1 || (uint32_t)k > G) return PCR_E_RANGE;
    const size_t pos = hdr_group_end_pos((uint32_t)k - 1);
    if (nbytes < pos + 8) { *need = pos + 8; return PCR_E_TRUNCATED; }
    *need = ld_le64(b + pos);
    return PCR_OK;
}

// ---- loader: re-used pinned staging buffers, device buffers, streams and handles ----
struct pcr_loader_slot {
    void* host = nullptr; uint8_t* dev = nullptr; hipStream_t stream = nullptr; pcr_record* rec = nullptr;
};
struct pcr_loader {
    int device = 0; size_t slot_bytes = 0;
    std::vector<pcr_loader_slot> slots;
    // token bucket: `rate` bytes are granted per second, at most `burst` are saved up
    double rate = 0, burst = 0, tokens = 0;
    std::chrono::steady_clock::time_point last;
};

int pcr_loader_create(int device_id, int slots, size_t slot_bytes, pcr_loader** out) {
    if (!out || slots < 1 || slots > 16 || slot_bytes < 24 || slot_bytes >= (1ull << 32)) return PCR_E_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device_id < 0 || device_id >= ndev) { (void)hipGetLastError(); return PCR_E_DEVICE; }
    HIP_TRY(hipSetDevice(device_id));
    pcr_loader* ld = new (std::nothrow) pcr_loader();
    if (!ld) return PCR_E_NOMEM;
    ld->device = device_id; ld->slot_bytes = slot_bytes; ld->slots.resize((size_t)slots);
    ld->last = std::chrono::steady_clock::now();
    int rc = PCR_OK;
    for (auto& sl : ld->slots) {
        if (hipHostMalloc(&sl.host, slot_bytes, hipHostMallocDefault) != hipSuccess) { rc = PCR_E_NOMEM; break; }
        if (hipMalloc((void**)&sl.dev, slot_bytes + 64) != hipSuccess) { rc = PCR_E_NOMEM; break; }
        if (hipStreamCreateWithFlags(&sl.stream, hipStreamNonBlocking) != hipSuccess) { rc = PCR_E_DEVICE; break; }
    }
    if (rc) { (void)hipGetLastError(); pcr_loader_destroy(ld); return rc; }
    *out = ld;
    return PCR_OK;
}

void pcr_loader_destroy(pcr_loader* ld) {
    if (!ld) return;
    (void)hipSetDevice(ld->device);
    for (auto& sl : ld->slots) {
        if (sl.stream) (void)hipStreamSynchronize(sl.stream);
        if (sl.rec) pcr_close(sl.rec);
        if (sl.stream) (void)hipStreamDestroy(sl.stream);
        if (sl.dev) (void)hipFree(sl.dev);
        if (sl.host) (void)hipHostFree(sl.host);
    }
    delete ld;
}

static pcr_loader_slot* loader_slot(pcr_loader* ld, int slot) {
    return (ld && slot >= 0 && (size_t)slot < ld->slots.size()) ? &ld->slots[(size_t)slot] : nullptr;
}

int pcr_loader_staging(pcr_loader* ld, int slot, void** host, size_t* capacity) {
    pcr_loader_slot* sl = loader_slot(ld, slot);
    if (!sl || !host) return PCR_E_ARG;
    *host = sl->host;
    if (capacity) *capacity = ld->slot_bytes;
    return PCR_OK;
}

int pcr_loader_stream(pcr_loader* ld, int slot, void** hip_stream) {
    pcr_loader_slot* sl = loader_slot(ld, slot);
    if (!sl || !hip_stream) return PCR_E_ARG;
    *hip_stream = (void*)sl->stream;
    return PCR_OK;
}

int pcr_loader_set_rate(pcr_loader* ld, double bytes_per_second, double burst_bytes) {
    if (!ld || bytes_per_second < 0 || burst_bytes < 0) return PCR_E_ARG;
    ld->rate = bytes_per_second; ld->burst = burst_bytes; ld->tokens = 0;
    ld->last = std::chrono::steady_clock::now();
    return PCR_OK;
}

// blocks until the bucket holds `bytes` tokens (a request larger than the burst size waits for the whole amount)
static void loader_take_tokens(pcr_loader* ld, double bytes) {
    if (ld->rate <= 0) return;
    for (;;) {
        const auto now = std::chrono::steady_clock::now();
        ld->tokens += std::chrono::duration<double>(now - ld->last).count() * ld->rate;
        ld->last = now;
        const double cap = std::max(ld->burst, bytes);
        if (ld->tokens > cap) ld->tokens = cap;
        if (ld->tokens >= bytes) { ld->tokens -= bytes; return; }
        std::this_thread::sleep_for(std::chrono::duration<double>((bytes - ld->tokens) / ld->rate));
    }
}

int pcr_loader_upload(pcr_loader* ld, int slot, size_t nbytes, pcr_record** rec) {
    pcr_loader_slot* sl = loader_slot(ld, slot);
    if (!sl) return PCR_E_ARG;
    if (nbytes < 24) return PCR_E_TRUNCATED;
    if (nbytes > ld->slot_bytes) return PCR_E_RANGE;
    HIP_TRY(hipSetDevice(ld->device));
    HIP_TRY(hipStreamSynchronize(sl->stream));                // the slot's buffers and handle are free again
    loader_take_tokens(ld, (double)nbytes);
    HIP_TRY(hipMemcpyAsync(sl->dev, sl->host, nbytes, hipMemcpyHostToDevice, sl->stream));
    HIP_TRY(hipMemsetAsync(sl->dev + nbytes, 0, 64, sl->stream));
    int rc;
    if (!sl->rec) rc = pcr_open_device(sl->dev, nbytes, (void*)sl->stream, &sl->rec);
    else rc = pcr_rebind_device(sl->rec, sl->dev, nbytes, (void*)sl->stream);
    if (rc) return rc;
    if (rec) *rec = sl->rec;
    return PCR_OK;
}

// pread until `count` bytes are in or the file ends; returns the bytes read, or -1
static ssize_t read_fully(int fd, uint8_t* dst, size_t count, off_t at) {
    size_t got = 0;
    while (got < count) {
        const ssize_t r = pread(fd, dst + got, count - got, at + (off_t)got);
        if (r < 0) return -1;
        if (r == 0) break;
        got += (size_t)r;
    }
    return (ssize_t)got;
}

int pcr_loader_read_file(pcr_loader* ld, int slot, const char* path, int k, size_t* nbytes, pcr_record** rec) {
    pcr_loader_slot* sl = loader_slot(ld, slot);
    if (!sl || !path) return PCR_E_ARG;
    HIP_TRY(hipSetDevice(ld->device));
    HIP_TRY(hipStreamSynchronize(sl->stream));                // the staging buffer is free again
    const int fd = open(path, O_RDONLY | O_CLOEXEC);
    if (fd < 0) return PCR_E_ARG;
    uint8_t* host = (uint8_t*)sl->host;
    const size_t head = std::min<size_t>(24 + 8 * 64, ld->slot_bytes);
    const ssize_t got = read_fully(fd, host, head, 0);
    int rc = got < 0 ? PCR_E_ARG : PCR_OK;
    uint64_t need = 0;
    if (!rc) rc = pcr_prefix_length(host, (size_t)got, k, &need);   // (a file that ends inside its header: TRUNCATED)
    if (!rc && need > ld->slot_bytes) rc = PCR_E_RANGE;
    if (!rc && need > (uint64_t)got) {
        const ssize_t more = read_fully(fd, host + got, (size_t)(need - (uint64_t)got), (off_t)got);
        if (more < 0) rc = PCR_E_ARG;
        else if ((uint64_t)got + (uint64_t)more < need) rc = PCR_E_TRUNCATED;
    }
    (void)close(fd);
    if (rc) return rc;
    if (nbytes) *nbytes = (size_t)need;
    return pcr_loader_upload(ld, slot, (size_t)need, rec);
}

int pcr_loader_decode(pcr_loader* ld, int slot, int k, uint8_t* out, size_t cap, int32_t* d_status) {
    pcr_loader_slot* sl = loader_slot(ld, slot);
    if (!sl || !sl->rec) return PCR_E_ARG;
    return pcr_decode_batch(sl->rec, k, out, cap, (void*)sl->stream, d_status);
}

int pcr_loader_decode_crop(pcr_loader* ld, int slot, int k, const pcr_crop* d_crops, uint8_t* d_pixels, size_t pixel_capacity, int out_h, int out_w,
                           const float* mean, const float* inv_std, void* d_out_f16, size_t out_capacity, int32_t* d_status) {
    pcr_loader_slot* sl = loader_slot(ld, slot);
    if (!sl || !sl->rec) return PCR_E_ARG;
    return pcr_decode_crop_batch(sl->rec, k, d_crops, d_pixels, pixel_capacity, out_h, out_w, mean, inv_std, d_out_f16, out_capacity,
                                 (void*)sl->stream, d_status);
}

int pcr_loader_wait(pcr_loader* ld, int slot) {
    pcr_loader_slot* sl = loader_slot(ld, slot);
    if (!sl) return PCR_E_ARG;
    HIP_TRY(hipSetDevice(ld->device));
    HIP_TRY(hipStreamSynchronize(sl->stream));
    return PCR_OK;
}

const char* pcr_strerror(int code) {
    switch (code) {
        case PCR_OK: return "ok";
        case PCR_E_ARG: return "invalid argument";
        case PCR_E_FORMAT: return "malformed record or JPEG stream";
        case PCR_E_TRUNCATED: return "record bytes do not reach the requested scan group";
        case PCR_E_UNSUPPORTED: return "unsupported JPEG feature or record size";
        case PCR_E_RANGE: return "index or capacity out of range";
        case PCR_E_NOMEM: return "out of memory";
        case PCR_E_DEVICE: return "HIP device error";
        default: return "unknown error";
    }
}

}  // extern "C"
