// gfx950 kernels of the PCR decode path.  One kernel per step:
//   k_index      scan-group index (prefix sums of region lengths)
//   k_parse      JPEG marker parsing, one lane per image
//   k_unstuff    byte un-stuffing + restart-interval location, one workgroup per (image, scan)
//   k_dc_first, k_ac_first, k_ac_refine   progressive Huffman decode, one wavefront per restart
//                interval of a scan (per scan where there are no restart markers)
//   k_refine_blocks   second phase of AC refinement, one lane per block
//   k_apply      data-parallel refinement (DC bits, AC corrections and new coefficients)
//   k_pixel      de-quantise + IDCT + chroma replication + YCbCr->RGB + store
//   k_gather     materialise an image's scan prefix (parity hook)
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "pcr_common.h"
#include "pcr_format.h"
#include "pcr_entropy.h"
#include "pcr_pixel.h"

namespace pcr {

// Everything a kernel needs to find its data; passed by value.
// Wave priority.  A decode call on one record usually shares the GPU with calls on other records (other
// streams).  The AC entropy kernels then keep every SIMD busy with long-running wavefronts that issue
// scalar instructions back to back, and instruction arbitration serves the oldest wavefronts first: a short
// data-parallel kernel of another record (unstuff, fill, phase 2 of refinement, pixels) was measured to run
// 3-8 times longer than alone, holding up its record's dependency chain.  These kernels therefore raise
// their own wavefronts' issue priority (s_setprio; stream priorities are not touched); the DC first kernel,
// few and latency-bound wavefronts, takes a middle value.  The AC entropy kernels stay at the default.
PCR_D void short_kernel_priority() { __builtin_amdgcn_s_setprio(3); }
PCR_D void dc_kernel_priority() { __builtin_amdgcn_s_setprio(2); }

struct DevRecord {
    const uint8_t* rec;        // record bytes
    uint8_t* clean;            // unstuffed entropy data, same offsets as rec
    uint32_t n, G;
    uint32_t* off;             // [G][n] absolute region offsets (k_index)
    const uint32_t* len;       // [G][n] region lengths (inside rec's header)
    const uint32_t* nscans;    // [n] (inside rec's header)
    ImgDesc* img;              // [n]
    ScanDesc* scan;            // [n][G]
    const uint64_t* coef_off;  // [n+1] int16 units
    const uint64_t* out_off;   // [n+1] bytes
    const uint64_t* mask_off;  // [n][G] u64 units into masks (AC scans)
    const uint32_t* slot_base; // [n][G] first entry of the scan in ivl_start
    const uint32_t* slot_cnt;  // [n][G] intervals of the scan
    uint32_t* ivl_start;       // per scan: intervals+1 offsets into the clean segment
    int16_t* coef;
    uint64_t* masks;
    int32_t* status;           // [n]
    AcTab* tabs;               // Huffman tables of the AC scans: those of the refinement scans are written by phase 1 for phase 2;
                               // with tabs_prebuilt, k_build_tables has written all of them before the entropy kernels start
    const uint32_t* tab_idx;   // [n][G] index into tabs
    const uint32_t* ent_off;   // [n][G] record offset of the scan's entry points (0: none; then slot_cnt - 1 of them)
    uint32_t tabs_prebuilt;    // set per call by the host (records whose scans have restart intervals)
};

// segment of a scan in the clean buffer: 4-byte aligned base (big-endian words)
PCR_HD uint32_t clean_base(uint32_t data_off) { return (data_off + 3u) & ~3u; }

// --------------------------------------------------------------------------------------
// k_index: off[g][i] = start of group g + sum of len[g][j], j < i.  One workgroup per group.
// --------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_index(DevRecord R, uint32_t kmax) {
    __shared__ uint32_t part[256];
    __shared__ uint32_t carry;
    uint32_t g = blockIdx.x;
    if (g >= kmax) return;
    uint64_t hb = ld_le64(R.rec + 16);
    uint64_t start = g == 0 ? hb : ld_le64(R.rec + hdr_group_end_pos(g - 1));
    if (threadIdx.x == 0) carry = (uint32_t)start;
    __syncthreads();
    for (uint32_t base = 0; base < R.n; base += 256) {
        uint32_t i = base + threadIdx.x;
        uint32_t v = i < R.n ? R.len[(size_t)g * R.n + i] : 0;
        part[threadIdx.x] = v;
        __syncthreads();
        for (uint32_t d = 1; d < 256; d <<= 1) {           // inclusive Hillis-Steele scan
            uint32_t t = threadIdx.x >= d ? part[threadIdx.x - d] : 0;
            __syncthreads();
            part[threadIdx.x] += t;
            __syncthreads();
        }
        if (i < R.n) R.off[(size_t)g * R.n + i] = carry + part[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 255) carry += part[255];
        __syncthreads();
    }
}

// --------------------------------------------------------------------------------------
// k_parse: one lane per image walks the marker segments of its regions 1..kmax.
// --------------------------------------------------------------------------------------
// keep_status: a fidelity upgrade builds on planes decoded earlier; an image those calls found damaged stays so
__global__ void __launch_bounds__(64) k_parse(DevRecord R, uint32_t kmax, uint32_t keep_status) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= R.n) return;
    parse_image(R.rec, R.off, R.len, R.n, i, R.nscans[i], kmax, &R.img[i], &R.scan[(size_t)i * R.G]);
    if (!(keep_status && R.status[i] != kOk)) R.status[i] = R.img[i].status;
}

// --------------------------------------------------------------------------------------
// k_unstuff: per (image, scan) remove stuffed zeros, fill bytes and restart markers from the
// entropy-coded segment, stop at the first other marker, note where each restart interval
// begins.  256 lanes x 8 bytes per step, one exclusive scan per step.
// --------------------------------------------------------------------------------------
constexpr int kUnstuffPer = 8;

// grid: (images, scan groups kfrom .. kmax-1)
__global__ void __launch_bounds__(256) k_unstuff(DevRecord R, uint32_t kfrom, uint32_t kmax) {
    short_kernel_priority();
    __shared__ uint32_t part[4];
    __shared__ uint32_t s_stop;
    uint32_t i = blockIdx.x, g = kfrom + blockIdx.y;
    if (g >= kmax) return;
    const ImgDesc& img = R.img[i];
    if (img.status != kOk || g >= img.nscans) return;
    const ScanDesc& sd = R.scan[(size_t)i * R.G + g];
    const uint8_t* src = R.rec + sd.data_off;
    uint8_t* dst = R.clean + clean_base(sd.data_off);     // stored as big-endian 32-bit words: byte o goes to o ^ 3
    const uint32_t L = sd.data_len;
    const uint32_t sb = R.slot_base[(size_t)i * R.G + g], sc = R.slot_cnt[(size_t)i * R.G + g];
    uint32_t out_total = 0, rst_total = 0;
    if (threadIdx.x == 0) { s_stop = 0xFFFFFFFFu; R.ivl_start[sb] = 0; }
    __syncthreads();
    for (uint32_t base = 0; base < L; base += 256 * kUnstuffPer) {
        uint32_t p0 = base + threadIdx.x * kUnstuffPer;
        uint8_t b[kUnstuffPer + 2];                    // prev, 8 bytes, next
        for (int j = 0; j < kUnstuffPer + 2; j++) {
            uint32_t q = p0 + j;                       // index of b[j] is q - 1
            b[j] = (q >= 1 && q - 1 < L) ? src[q - 1] : 0;
        }
        if (p0 == 0) b[0] = 0;
        uint32_t keep = 0, rst = 0, stop = 0xFFFFFFFFu;
        for (int j = 0; j < kUnstuffPer; j++) {
            uint32_t q = p0 + j;
            if (q >= L) break;
            uint8_t prev = b[j], cur = b[j + 1], next = b[j + 2];
            bool last = (q + 1 >= L);
            if (cur == 0xFF) {
                bool is_rst = !last && next >= 0xD0 && next <= 0xD7;
                bool is_data = !last && next == 0x00;
                bool is_fill = !last && next == 0xFF;
                if (is_rst) rst |= 1u << j;
                else if (is_data) keep |= 1u << j;
                else if (!is_fill) { stop = q; break; }   // any other marker ends the segment
            } else if (prev == 0xFF && (cur == 0x00 || (cur >= 0xD0 && cur <= 0xD7))) {
                // stuffed zero or second byte of a restart marker: dropped
            } else keep |= 1u << j;
        }
        if (stop != 0xFFFFFFFFu) atomicMin(&s_stop, stop);
        __syncthreads();
        uint32_t stop_all = s_stop;
        // drop what lies at or after the terminating marker
        if (stop_all != 0xFFFFFFFFu) {
            for (int j = 0; j < kUnstuffPer; j++) if (p0 + j >= stop_all) { keep &= ~(1u << j); rst &= ~(1u << j); }
        }
        // prefix sums of (bytes kept | restart markers << 16) over the 256 lanes: inside each wavefront by lane
        // shuffles, then the four wavefront totals through LDS
        const uint32_t mine = (uint32_t)__builtin_popcount(keep) | ((uint32_t)__builtin_popcount(rst) << 16);
        const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        uint32_t incl = mine;
#pragma unroll
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t t = (uint32_t)__shfl_up((int)incl, d, 64);
            if (lane >= d) incl += t;
        }
        if (lane == 63) part[wave] = incl;
        __syncthreads();
        const uint32_t w0 = part[0], w1 = part[1], w2 = part[2], w3 = part[3];
        const uint32_t before = (wave > 0 ? w0 : 0) + (wave > 1 ? w1 : 0) + (wave > 2 ? w2 : 0);
        const uint32_t excl = before + incl - mine;
        uint32_t o = out_total + (excl & 0xFFFF), r = rst_total + (excl >> 16);
        for (int j = 0; j < kUnstuffPer; j++) {
            if (keep & (1u << j)) { dst[o ^ 3u] = b[j + 1]; o++; }
            if (rst & (1u << j)) { r++; if (r < sc) R.ivl_start[sb + r] = o; }
        }
        const uint32_t tot = w0 + w1 + w2 + w3;
        out_total += tot & 0xFFFF; rst_total += tot >> 16;
        __syncthreads();
        if (stop_all != 0xFFFFFFFFu) break;
    }
    if (threadIdx.x == 0) {
        // intervals whose restart marker never showed up get an empty range; the end goes last
        for (uint32_t r = rst_total + 1; r <= sc; r++) R.ivl_start[sb + r] = out_total;
        R.ivl_start[sb + sc] = out_total;
        if (rst_total + 1 != (sd.ri ? sc : 1u)) R.status[i] = kEFormat;      // (without restart intervals the units of a scan start at entry points)
        if (sd.Ss == 0 && sd.Ah != 0) {
            // DC refinement is read in place later (one bit per block): check every interval is long enough
            uint32_t bpm = 0;
            for (int q = 0; q < sd.ns; q++) bpm += sd.ns > 1 ? (uint32_t)img.hs[sd.comp[q]] * img.vs[sd.comp[q]] : 1;
            for (uint32_t r = 0; r < sc; r++) {
                uint32_t m0 = sd.ri ? r * sd.ri : 0, m1 = sd.ri ? (m0 + sd.ri < sd.mcus ? m0 + sd.ri : sd.mcus) : sd.mcus;
                uint32_t have = (R.ivl_start[sb + r + 1] - R.ivl_start[sb + r]) * 8;
                if ((m1 - m0) * bpm > have) R.status[i] = kEFormat;
            }
        }
    }
}

// --------------------------------------------------------------------------------------
// Entropy kernels: ONE WAVEFRONT PER UNIT (a restart interval of one scan of one image).
// Everything the decoder touches is a function of blockIdx.x alone, i.e. wave-uniform, so the
// compiler keeps the decoder state in scalar registers and runs it on the scalar ALU with
// native 64-bit shifts, population counts and find-first-set; the Huffman table sits in LDS.
// A serial bit-stream decoder has no use for 64 lanes, but a lone wavefront issues only about
// one instruction per ten cycles whatever its width, and packing 64 different streams into one
// wavefront makes every loop iteration pay for the union of all lanes' branches; one stream
// per wavefront costs only the branch actually taken and lets thousands of streams interleave
// on the SIMDs.  The host orders units by decreasing byte length (longest first).
// --------------------------------------------------------------------------------------
constexpr int kEntropyLanes = 64;
// clean32 and hist64 are R.clean and R.masks again, as separate restrict-qualified kernel arguments: the
// kernels only read the unstuffed data and the history planes of EARLIER scans, and knowing that nothing
// written here aliases them lets the compiler fetch them with scalar loads (straight into scalar
// registers, waited for at the first use) instead of vector loads followed by a read-first-lane.

struct UnitSetup {
    const uint32_t* words;        // segment base, unit start and length for the window readers
    uint32_t byte_off, sub_bits, nbits, pos0;
    LaneScan ls;
    int16_t* plane[kMaxComp];     // planes of the scan's components
    uint32_t plane_elems[kMaxComp];
    int16_t* base;                // the image's coefficient buffer (all planes)
    uint32_t base_elems;
    bool ok;
};

PCR_D void unit_setup(const DevRecord& R, const Unit& un, const uint32_t* __restrict__ clean32, UnitSetup* L) {
    L->ok = false;
    const ImgDesc* img = &R.img[un.img];
    if (R.status[un.img] != kOk || un.scan >= img->nscans) return;
    const size_t ig = (size_t)un.img * R.G + un.scan;
    const ScanDesc* sd = &R.scan[ig];
    if (!sd->valid) return;
    const uint32_t sb = R.slot_base[ig];
    const uint32_t ri = sd->ri, mcus = sd->mcus;
    LaneScan& ls = L->ls;
    ls.mcu_w = uni(sd->mcu_w);
    ls.pred[0] = ls.pred[1] = ls.pred[2] = 0;
    const uint32_t sc = R.slot_cnt[ig];
    if (ri == 0 && sc > 1) {
        // Units of a scan without restart markers start at the record's entry points: unit j runs from entry j-1
        // (the scan's start for j = 0) to entry j (the scan's end for the last unit).
        const uint8_t* e = R.rec + uni(R.ent_off[ig]) + (size_t)kEntryBytes * un.interval;        // entry j; entry j-1 lies 16 bytes before it
        const uint32_t total = uni(R.ivl_start[sb + sc]) * 8;                                    // bits of the scan's unstuffed data
        uint32_t m0 = 0, bit0 = 0, m1 = mcus, bit1 = total;
        if (un.interval > 0) {
            m0 = uni(ld_le32(e - 16)); bit0 = uni(ld_le32(e - 12));
            ls.pred[0] = uni((int)(int16_t)ld_le16(e - 8)); ls.pred[1] = uni((int)(int16_t)ld_le16(e - 6)); ls.pred[2] = uni((int)(int16_t)ld_le16(e - 4));
        }
        if (un.interval + 1 < sc) { m1 = uni(ld_le32(e)); bit1 = uni(ld_le32(e + 4)); }
        if (!(m0 < m1 && m1 <= mcus && bit0 <= bit1 && bit1 <= total)) { R.status[un.img] = kEFormat; return; }   // entries out of order or out of range
        ls.mcu0 = m0; ls.mcu1 = m1;
        L->byte_off = bit0 >> 3; L->sub_bits = bit0 & 7; L->nbits = bit1 - (bit0 & ~7u); L->pos0 = bit0 & ~7u;
    } else {
        const uint32_t b0 = R.ivl_start[sb + un.interval], b1 = R.ivl_start[sb + un.interval + 1];
        ls.mcu0 = uni(ri ? un.interval * ri : 0);
        ls.mcu1 = uni(ri ? (ls.mcu0 + ri < mcus ? ls.mcu0 + ri : mcus) : mcus);
        if (ls.mcu0 >= mcus) return;
        L->byte_off = uni(b0); L->sub_bits = 0; L->nbits = uni(b1 > b0 ? b1 - b0 : 0) * 8; L->pos0 = 0;
    }
    ls.Ss = uni((int)sd->Ss); ls.Se = uni((int)sd->Se); ls.Al = uni((int)sd->Al); ls.ns = uni((int)sd->ns);
    int16_t* base = R.coef + uni((uint64_t)R.coef_off[un.img]);
    size_t poff[kMaxComp + 1]; poff[0] = 0;
#pragma unroll
    for (int c = 0; c < kMaxComp; c++) poff[c + 1] = poff[c] + (c < img->nc ? (size_t)uni((uint32_t)img->bw[c]) * uni((uint32_t)img->bh[c]) * 64 : 0);
#pragma unroll
    for (int j = 0; j < kMaxComp; j++) {
        const int c = uni(j < ls.ns ? (int)sd->comp[j] : 0);
        ls.hs[j] = uni((uint32_t)img->hs[c]); ls.vs[j] = uni((uint32_t)img->vs[c]); ls.bw[j] = uni((uint32_t)img->bw[c]);
        const size_t po = c == 0 ? poff[0] : (c == 1 ? poff[1] : poff[2]);
        ls.poff[j] = (uint32_t)po;
        L->plane[j] = base + po;
        L->plane_elems[j] = (uint32_t)((c == 0 ? poff[1] : (c == 1 ? poff[2] : poff[3])) - po);
    }
    L->base = base;
    L->base_elems = (uint32_t)poff[kMaxComp];
    L->words = clean32 + (uni(clean_base(sd->data_off)) >> 2);
    L->ok = true;
}

// SHAPE: which DC decoder (dc_shape) the units of this launch take; the host sorts the units by it.
template <int SHAPE>
__global__ void __launch_bounds__(kEntropyLanes) k_dc_first(DevRecord R, const Unit* __restrict__ units, uint32_t nunits,
        const uint32_t* __restrict__ clean32, const uint64_t* __restrict__ hist64) {
    __shared__ DcTab tabs[kMaxComp];
    dc_kernel_priority();
    const Unit un = units[blockIdx.x];
    UnitSetup L;
    unit_setup(R, un, clean32, &L);
    if (!L.ok) return;
    const ScanDesc* sd = &R.scan[(size_t)un.img * R.G + un.scan];
    const uint32_t o0 = sd->dc_off[0], o1 = L.ls.ns > 1 ? sd->dc_off[1] : o0, o2 = L.ls.ns > 2 ? sd->dc_off[2] : o0;
    // distinct tables of the scan's components: slot 0 always, slot 1/2 when a component uses another one
    int tj1 = 0, tj2 = 0, ntab = 1;
    if (o1 != o0) { tj1 = 1; ntab = 2; }
    if (o2 == o1) tj2 = tj1; else if (o2 != o0) { tj2 = ntab; ntab++; }
    if (threadIdx.x == 0) dctab_build(&tabs[0], R.rec + o0);
    if (threadIdx.x == 1 && tj1 == 1) dctab_build(&tabs[1], R.rec + o1);
    if (threadIdx.x == 2 && tj2 != 0 && tj2 != tj1) dctab_build(&tabs[tj2], R.rec + o2);
    __syncthreads();
    DcWindowReader wr;                                      // tables by scan component
    wr.init(L.words, L.byte_off, L.sub_bits, L.nbits, &tabs[0], &tabs[uni(tj1)], &tabs[uni(tj2)], L.ls.ns, threadIdx.x);
    CoefSink sink;
    sink.init(L.base, L.base_elems, L.ls.Al);
    int rc = kEFormat;                                      // (a unit in the wrong launch: the descriptors disagree with the host's)
    if (dc_shape(L.ls.ns, L.ls.hs[0], L.ls.vs[0], L.ls.hs[1], L.ls.vs[1], L.ls.hs[2], L.ls.vs[2]) == SHAPE) rc = decode_dc_first_as<SHAPE>(&wr, L.ls, &sink);
    if (rc != kOk) R.status[un.img] = rc;
}

// The AC table of a unit's scan into LDS: copied from the pre-built one (k_build_tables), or built here from the
// table definition in the record by one lane and packed by all.  Call with every lane of the wavefront.
PCR_D void load_ac_table(const DevRecord& R, size_t ig, bool first, AcTab* tab) {
    if (R.tabs_prebuilt) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&R.tabs[R.tab_idx[ig]]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(tab);
        for (uint32_t e = threadIdx.x; e < sizeof(AcTab) / 4; e += kEntropyLanes) dst[e] = src[e];
        __syncthreads();
        return;
    }
    if (threadIdx.x == 0) actab_build(tab, R.rec + R.scan[ig].ac_off);
    __syncthreads();
    actab_pack(tab, first, threadIdx.x, kEntropyLanes);
    __syncthreads();
}

// One wavefront per (image, scan): the scan's AC table, built once for all its restart intervals.
// grid: (n, scans), scans k0 .. k0 + gridDim.y - 1.
__global__ void __launch_bounds__(kEntropyLanes) k_build_tables(DevRecord R, uint32_t k0) {
    __shared__ AcTab tab;
    short_kernel_priority();
    const uint32_t i = blockIdx.x, g = k0 + blockIdx.y;
    if (R.status[i] != kOk || g >= R.img[i].nscans) return;
    const size_t ig = (size_t)i * R.G + g;
    const ScanDesc* sd = &R.scan[ig];
    if (!sd->valid || sd->Ss == 0) return;                  // (DC scans and sequential scans build their own)
    if (threadIdx.x == 0) actab_build(&tab, R.rec + sd->ac_off);
    __syncthreads();
    actab_pack(&tab, sd->Ah == 0, threadIdx.x, kEntropyLanes);
    __syncthreads();
    const uint32_t* src = reinterpret_cast<const uint32_t*>(&tab);
    uint32_t* dst = reinterpret_cast<uint32_t*>(&R.tabs[R.tab_idx[ig]]);
    for (uint32_t e = threadIdx.x; e < sizeof(AcTab) / 4; e += kEntropyLanes) dst[e] = src[e];
}

__global__ void __launch_bounds__(kEntropyLanes) k_ac_first(DevRecord R, const Unit* __restrict__ units, uint32_t nunits,
        const uint32_t* __restrict__ clean32, const uint64_t* __restrict__ hist64) {
    __shared__ AcTab tab;
    const Unit un = units[blockIdx.x];
    UnitSetup L;
    unit_setup(R, un, clean32, &L);
    if (!L.ok) return;
    const size_t ig = (size_t)un.img * R.G + un.scan;
    load_ac_table(R, ig, true, &tab);
    WindowReader wr;
    wr.init(L.words, L.byte_off, L.sub_bits, L.nbits, L.pos0, &tab, true, threadIdx.x, true);
    IndexSink sink;
    sink.init(L.plane[0], L.plane_elems[0], L.ls.Al);
    int rc = decode_ac_first(&wr, L.ls, &sink);
    if (rc != kOk) R.status[un.img] = rc;
}

// Sequential (baseline) scans: the DC and AC tables of every scan component, once per distinct table.
__global__ void __launch_bounds__(kEntropyLanes) k_sequential(DevRecord R, const Unit* __restrict__ units, uint32_t nunits,
        const uint32_t* __restrict__ clean32, const uint64_t* __restrict__ hist64) {
    __shared__ DcTab dtabs[kMaxComp];
    __shared__ AcTab atabs[kMaxComp];
    const Unit un = units[blockIdx.x];
    UnitSetup L;
    unit_setup(R, un, clean32, &L);
    if (!L.ok) return;
    const ScanDesc* sd = &R.scan[(size_t)un.img * R.G + un.scan];
    if (!is_sequential_scan(*sd)) { R.status[un.img] = kEFormat; return; }      // (a unit in the wrong launch)
    const uint32_t d0 = sd->dc_off[0], d1 = L.ls.ns > 1 ? sd->dc_off[1] : d0, d2 = L.ls.ns > 2 ? sd->dc_off[2] : d0;
    const uint32_t a0 = sd->ac_offc[0], a1 = L.ls.ns > 1 ? sd->ac_offc[1] : a0, a2 = L.ls.ns > 2 ? sd->ac_offc[2] : a0;
    int dj1 = 0, dj2 = 0, nd = 1, aj1 = 0, aj2 = 0, na = 1;
    if (d1 != d0) { dj1 = 1; nd = 2; }
    if (d2 == d1) dj2 = dj1; else if (d2 != d0) { dj2 = nd; nd++; }
    if (a1 != a0) { aj1 = 1; na = 2; }
    if (a2 == a1) aj2 = aj1; else if (a2 != a0) { aj2 = na; na++; }
    if (threadIdx.x == 0) { dctab_build(&dtabs[0], R.rec + d0); actab_build(&atabs[0], R.rec + a0); }
    if (threadIdx.x == 1) {
        if (dj1 == 1) dctab_build(&dtabs[1], R.rec + d1);
        if (aj1 == 1) actab_build(&atabs[1], R.rec + a1);
    }
    if (threadIdx.x == 2) {
        if (dj2 != 0 && dj2 != dj1) dctab_build(&dtabs[dj2], R.rec + d2);
        if (aj2 != 0 && aj2 != aj1) actab_build(&atabs[aj2], R.rec + a2);
    }
    __syncthreads();
    for (int t = 0; t < na; t++) actab_pack(&atabs[t], true, threadIdx.x, kEntropyLanes);
    __syncthreads();
    SeqTables tb;
    tb.dc[0] = &dtabs[0]; tb.dc[1] = &dtabs[uni(dj1)]; tb.dc[2] = &dtabs[uni(dj2)];
    tb.ac[0] = &atabs[0]; tb.ac[1] = &atabs[uni(aj1)]; tb.ac[2] = &atabs[uni(aj2)];
    WindowReader wr;
    wr.init(L.words, L.byte_off, L.sub_bits, L.nbits, L.pos0, tb.ac[0], true, threadIdx.x, true);
    IndexSink sink;
    sink.init(L.base, L.base_elems, 0);
    const int rc = decode_sequential(&wr, L.ls, tb, &sink);
    if (rc != kOk) R.status[un.img] = rc;
}

struct ApplyUnit { uint32_t img; uint32_t comp; };

__global__ void __launch_bounds__(kEntropyLanes) k_ac_refine(DevRecord R, const Unit* __restrict__ units, uint32_t nunits,
        const uint32_t* __restrict__ clean32, const uint64_t* __restrict__ hist64) {
    __shared__ AcTab tab;
    const Unit un = units[blockIdx.x];
    UnitSetup L;
    unit_setup(R, un, clean32, &L);
    if (!L.ok) return;
    const size_t ig = (size_t)un.img * R.G + un.scan;
    const ScanDesc* sd = &R.scan[ig];
    load_ac_table(R, ig, false, &tab);
    if (un.interval == 0 && !R.tabs_prebuilt) {             // phase 2 needs the same table: keep a copy
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&tab);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&R.tabs[R.tab_idx[ig]]);
        for (uint32_t e = threadIdx.x; e < sizeof(AcTab) / 4; e += kEntropyLanes) dst[e] = src[e];
    }
    HistPlanes hp;
    hp.coef = L.plane[0];
    hp.n = sd->nhist;
#pragma unroll
    for (int q = 0; q < kMaxHist; q++) hp.p[q] = hist64 + uni((uint64_t)R.mask_off[(size_t)un.img * R.G + sd->hist[q < hp.n ? q : 0]]);
    hp.n = uni(hp.n);
    const ImgDesc* img = &R.img[un.img];
    const int c = sd->comp[0];
    const size_t plane = (size_t)uni((uint32_t)img->bw[c]) * uni((uint32_t)img->bh[c]);
    uint64_t* mk = R.masks + uni((uint64_t)R.mask_off[ig]);
    WindowReader wr;
    wr.init(L.words, L.byte_off, L.sub_bits, L.nbits, L.pos0, &tab, false, threadIdx.x, false);
    int rc = skim_ac_refine(&wr, L.ls, hp, mk);
    if (rc != kOk) R.status[un.img] = rc;
}

// Phase 2 of AC refinement: one lane per block of the scan.  grid: (ceil(max blocks / 256), scans)
struct RefineScan { uint32_t img; uint32_t scan; };

__global__ void __launch_bounds__(256) k_refine_blocks(DevRecord R, const RefineScan* rs) {
    __shared__ AcTab tab;
    short_kernel_priority();
    const RefineScan a = rs[blockIdx.y];
    if (R.status[a.img] != kOk) return;
    const ImgDesc* img = &R.img[a.img];
    const size_t ig = (size_t)a.img * R.G + a.scan;
    const ScanDesc* sd = &R.scan[ig];
    const int c = sd->comp[0];
    const uint32_t cw = img->cw[c], ncov = cw * img->ch[c];
    if (blockIdx.x * 256 >= ncov) return;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&R.tabs[R.tab_idx[ig]]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&tab);
        for (uint32_t e = threadIdx.x; e < sizeof(AcTab) / 4; e += 256) dst[e] = src[e];
    }
    __syncthreads();
    const uint32_t b = blockIdx.x * 256 + threadIdx.x;
    if (b >= ncov) return;
    const uint32_t bw = img->bw[c];
    const size_t blk = (size_t)(b / cw) * bw + (b % cw);
    const size_t plane = (size_t)bw * img->bh[c];
    uint64_t* mk = R.masks + R.mask_off[ig];
    uint64_t* rec = mk + blk * kRefWords;
    const uint64_t h = rec[kRefHist];                        // the history phase 1 worked on
    const uint32_t ivl = sd->ri ? b / sd->ri : 0;
    const uint32_t* words = reinterpret_cast<const uint32_t*>(R.clean + clean_base(sd->data_off));
    uint64_t sgn, cb;
    refine_block(words, R.ivl_start[R.slot_base[ig] + ivl], rec[kRefStart], &tab, h, rec[kRefNz], sd->Ss, sd->Se, &sgn, &cb);
    rec[kRefSign] = sgn; rec[kRefCbits] = cb;
}

// --------------------------------------------------------------------------------------
// Refinement, data-parallel.  One lane per coefficient of every block of a component
// (natural order within the block, so loads and stores are contiguous).
//   k = 0: DC refinement scans -- the block's bit sits at a position fixed by the scan's block
//          order (and restart intervals), so it is simply fetched and OR-ed in;
//   k > 0: replay the AC scans of the component in file order: first scans only extend the
//          non-zero mask, refinement scans add a correction bit or place a new +-2^Al.
// --------------------------------------------------------------------------------------
// k_apply_prep gathers, once per (image, component), the scans that matter for refinement (AC
// scans of the component in file order, DC refinement scans) into a compact list; k_apply then
// runs one lane per coefficient, a workgroup covering kApplyChunk consecutive coefficients.
struct ApplyScan { uint64_t mask_off; uint32_t slot; uint32_t data_base; uint32_t mcu_w; uint16_t ri; uint8_t Ss, Se, Ah, Al, ns, before, bpm, pad[3]; };
struct ApplyList { uint32_t n; uint32_t pad; ApplyScan sc[kApplyMaxScans]; };
constexpr uint32_t kApplyChunk = 4096;

// DC refinement of the block at (row, col) of a component with sampling hs x vs: the block's bit sits at
// a position fixed by the scan's block order and restart intervals; returns the bit (0 / 1), 0 for a block
// a non-interleaved scan does not visit.
PCR_D uint32_t dc_refinement_bit(const DevRecord& R, const ApplyScan& S, uint32_t row, uint32_t col, uint32_t hs, uint32_t vs, bool covered) {
    uint32_t m, within;
    if (S.ns > 1) { m = (row / vs) * S.mcu_w + col / hs; within = S.before + (row % vs) * hs + col % hs; }
    else { if (!covered) return 0; m = row * S.mcu_w + col; within = 0; }
    const uint32_t ivl = S.ri ? m / S.ri : 0;
    const uint32_t bit = (m - ivl * S.ri) * S.bpm + within;
    const uint32_t* words = reinterpret_cast<const uint32_t*>(R.clean + S.data_base);
    return (uint32_t)dc_refine_bit(words, R.ivl_start[S.slot + ivl], bit);
}

__global__ void __launch_bounds__(64) k_apply_prep(DevRecord R, const ApplyUnit* __restrict__ au, uint32_t nau, uint32_t kmax, ApplyList* lists) {
    const uint32_t u = blockIdx.x * 64 + threadIdx.x;
    if (u >= nau) return;
    const ApplyUnit a = au[u];
    const ImgDesc* img = &R.img[a.img];
    const int c = a.comp;
    ApplyList* L = &lists[u];
    uint32_t n = 0;
    const uint32_t upto = img->nscans < kmax ? img->nscans : kmax;
    for (uint32_t g = 0; g < upto && n < kApplyMaxScans; g++) {
        const size_t ig = (size_t)a.img * R.G + g;
        const ScanDesc* sd = &R.scan[ig];
        ApplyScan e;
        e.Ss = sd->Ss; e.Se = sd->Se; e.Ah = sd->Ah; e.Al = sd->Al; e.ns = sd->ns; e.ri = sd->ri; e.mcu_w = sd->mcu_w;
        e.mask_off = R.mask_off[ig]; e.slot = R.slot_base[ig]; e.data_base = clean_base(sd->data_off);
        e.before = 0; e.bpm = 0; e.pad[0] = e.pad[1] = e.pad[2] = 0;
        if (sd->Ss == 0) {
            if (sd->Ah == 0) continue;
            int j = -1; uint32_t before = 0, bpm = 0;
            for (int q = 0; q < sd->ns; q++) {
                const int cq = sd->comp[q];
                if (cq == c) { j = q; before = bpm; }
                bpm += sd->ns > 1 ? (uint32_t)img->hs[cq] * img->vs[cq] : 1;
            }
            if (j < 0) continue;
            e.before = (uint8_t)before; e.bpm = (uint8_t)bpm;
        } else if (sd->comp[0] != c || sd->Ah == 0) continue;  // AC first scans are in the planes already
        L->sc[n++] = e;
    }
    L->n = n;
}

__global__ void __launch_bounds__(256) k_apply(DevRecord R, const ApplyUnit* __restrict__ au, const ApplyList* __restrict__ lists) {
    __shared__ ApplyList L;
    const ApplyUnit a = au[blockIdx.y];
    const ImgDesc* img = &R.img[a.img];
    if (R.status[a.img] != kOk) return;
    const int c = a.comp;
    const uint32_t bw = img->bw[c], nblk = bw * img->bh[c];
    const uint32_t first = blockIdx.x * kApplyChunk;
    if (first >= nblk * 64) return;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&lists[blockIdx.y]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&L);
        for (uint32_t e = threadIdx.x; e < sizeof(ApplyList) / 4; e += 256) dst[e] = src[e];
    }
    __syncthreads();
    const uint32_t n = L.n;
    const uint32_t cw = img->cw[c], ch = img->ch[c], hs = img->hs[c], vs = img->vs[c];
    const size_t plane = nblk;
    int16_t* pl = R.coef + R.coef_off[a.img];
    for (int q = 0; q < c; q++) pl += (size_t)img->bw[q] * img->bh[q] * 64;
    for (uint32_t idx = first + threadIdx.x; idx < first + kApplyChunk && idx < nblk * 64; idx += 256) {
        const uint32_t b = idx >> 6; const int k = (int)(idx & 63);  // element k of a block = zig-zag position k
        const uint32_t row = b / bw, col = b % bw;
        const bool covered = row < ch && col < cw;
        const int16_t v0 = pl[idx];
        int16_t v = v0;
        for (uint32_t e = 0; e < n; e++) {
            const ApplyScan& S = L.sc[e];
            if (S.Ss == 0) {
                if (k != 0) continue;
                if (dc_refinement_bit(R, S, row, col, hs, vs, covered)) v |= (int16_t)(1 << S.Al);
            } else if (k != 0 && covered && k >= S.Ss && k <= S.Se) {
                const uint64_t* rec = R.masks + S.mask_off + (size_t)b * kRefWords;
                v = refine_apply(v, k, rec[kRefHist], rec[kRefNz], rec[kRefSign], rec[kRefCbits], S.Al);
            }
        }
        if (v != v0) pl[idx] = v;
    }
}

// Parity hook: internal planes (zig-zag order inside each block) -> natural order.
__global__ void __launch_bounds__(256) k_export_natural(const int16_t* in, int16_t* out, size_t n) {
    __shared__ uint8_t zz[64];
    if (threadIdx.x < 64) zz[threadIdx.x] = (uint8_t)zigzag_lookup(threadIdx.x);
    __syncthreads();
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) out[(i & ~(size_t)63) + zz[i & 63]] = in[i];
}

// --------------------------------------------------------------------------------------
// k_crop_resize: the training tail.  For every image one box of the decoded pixels is resized to
// out_h x out_w with bilinear interpolation on pixel centres (no anti-aliasing; samples beyond the
// box's edge repeat the edge), optionally mirrored left to right, normalised per channel and written
// as half precision, channel-planar: out[((i * C + c) * out_h + oy) * out_w + ox].
// One lane per output sample position (all channels); a workgroup covers 32 columns of 8 rows (the usual
// training sizes are multiples of 32), so a wavefront stores two runs of 64 contiguous bytes per channel.
// grid (ceil(out_w / 32), ceil(out_h / 8), n).  A box that does not lie inside its image is clamped into it.
// dims: width and height per image and out_off: byte offset of every image in `in`, both as laid down when the
// record was opened (the descriptors in device memory are only filled by a decode call).
// --------------------------------------------------------------------------------------
struct CropBox { int32_t x0, y0, w, h, flip; };

// floor(num / den) and the remainder in [0, den), den > 0, |num| < 2^31: the quotient is guessed in single
// precision (off by one at most for the quotients that occur, below 2^17) and put right with the remainder
PCR_D void floor_div(int num, int den, float inv_den, int* q, int* r) {
    int g = (int)floorf((float)num * inv_den);
    int rem = num - g * den;
    if (rem < 0) { g--; rem += den; }
    if (rem >= den) { g++; rem -= den; }
    *q = g; *r = rem;
}

__global__ void __launch_bounds__(256) k_crop_resize(const uint32_t* __restrict__ dims, const uint64_t* __restrict__ out_off,
        const uint8_t* __restrict__ in, const CropBox* __restrict__ boxes,
        int out_h, int out_w, int C, float m0, float m1, float m2, float s0, float s1, float s2, __half* __restrict__ out) {
    const uint32_t i = blockIdx.z;
    const int ox = (int)(blockIdx.x * 32 + (threadIdx.x & 31)), oy = (int)(blockIdx.y * 8 + (threadIdx.x >> 5));
    if (ox >= out_w || oy >= out_h) return;
    const int W = (int)dims[2 * i], H = (int)dims[2 * i + 1];
    if (W < 1 || H < 1) return;
    CropBox b = boxes[i];
    b.x0 = min(max(b.x0, 0), W - 1); b.y0 = min(max(b.y0, 0), H - 1);
    b.w = min(max(b.w, 1), W - b.x0); b.h = min(max(b.h, 1), H - b.y0);
    const int oxs = b.flip ? out_w - 1 - ox : ox;
    // source point relative to the box, as an exact fraction: ((2 o + 1) * size - out) / (2 * out) pixels
    const int dy = 2 * out_h, dx = 2 * out_w;
    const float inv_dy = 1.0f / (float)dy, inv_dx = 1.0f / (float)dx;
    int yl, ry, xl, rx;
    floor_div((2 * oy + 1) * b.h - out_h, dy, inv_dy, &yl, &ry);
    floor_div((2 * oxs + 1) * b.w - out_w, dx, inv_dx, &xl, &rx);
    const float fy = (float)ry * inv_dy, fx = (float)rx * inv_dx;
    const int ya = b.y0 + min(max(yl, 0), b.h - 1), yb = b.y0 + min(max(yl + 1, 0), b.h - 1);
    const int xa = b.x0 + min(max(xl, 0), b.w - 1), xb = b.x0 + min(max(xl + 1, 0), b.w - 1);
    const uint8_t* img = in + out_off[i];
    const uint8_t* paa = img + ((size_t)ya * W + xa) * C; const uint8_t* pab = img + ((size_t)ya * W + xb) * C;
    const uint8_t* pba = img + ((size_t)yb * W + xa) * C; const uint8_t* pbb = img + ((size_t)yb * W + xb) * C;
    const float mean[3] = {m0, m1, m2}, istd[3] = {s0, s1, s2};
    __half* dst = out + ((size_t)i * C * out_h + oy) * out_w + ox;
#pragma unroll
    for (int c = 0; c < 3; c++) {
        if (c < C) {
            const float top = (1.0f - fx) * (float)paa[c] + fx * (float)pab[c];
            const float bot = (1.0f - fx) * (float)pba[c] + fx * (float)pbb[c];
            const float v = (1.0f - fy) * top + fy * bot;
            dst[(size_t)c * out_h * out_w] = __float2half_rn((v * (1.0f / 255.0f) - mean[c]) * istd[c]);
        }
    }
}

// --------------------------------------------------------------------------------------
// k_pixel: one workgroup per strip of MCUs (128 pixels wide at most) of one MCU row of one image.
//   phase 1  coefficients -> LDS: every lane loads 16 contiguous bytes (8 coefficients in
//            zig-zag order), de-quantises and scatters them to their natural positions; chunks
//            that no scan <= k can have touched are not read at all; a component that only
//            has its DC gets one lane per block, which writes the flat block's value
//   phase 2  row IDCT, one lane per (block, row)
//   phase 3  column IDCT + level shift + clamp, one lane per (block, column)
//   phase 4  chroma replication + colour + store: one lane per group of 12 bytes of an output row
//            (4 RGB pixels), written as one 12-byte store that need not be aligned
// The measured limit of this kernel is vector-ALU issue, so the index arithmetic is kept off
// the lanes: components are handled one after the other (their geometry is wave-uniform),
// divisions by strip widths use a reciprocal computed once, and the zig-zag scatter offsets
// and quantiser steps come from two small LDS tables.
// --------------------------------------------------------------------------------------
constexpr int kStripPx = 128;              // strip width in pixels
constexpr int kMaxStripBlocks = 96;        // worst sampling: 16 MCUs x 6 blocks or 8 MCUs x 12 blocks (4:2:0: 48)
constexpr int kStripMcus = 8;              // MCUs per strip when the MCU is 16 pixels wide (tiles are built for this)

struct PixelTile { uint32_t img; uint16_t mcu_row; uint16_t mcu_col0; };
typedef short short8 __attribute__((ext_vector_type(8)));

// w / d as (w * recip16(d)) >> 16, exact while w * d < 65536
PCR_HD uint32_t recip16(uint32_t d) { return d ? 65536u / d + 1u : 0u; }

// Refinement is applied here, on the way in: the coefficient planes hold what the first scans wrote, and a
// lane that loads eight coefficients replays the component's refinement scans on them from the mask planes
// (exactly what k_apply does for the coefficient export, which is the only caller that still needs the
// refined values in memory).  lists / list_idx: the per-(image, component) scan lists of k_apply_prep and
// their index by image * 3 + component (-1: nothing to refine); both null if no scan <= k refines.
// kRefine = false compiles the replay out (scan groups without refinement scans: fewer registers).
// boxes (optional): one box per image; strips that do not touch their image's box are skipped altogether (their
// pixels are left as they are): for callers that go on to read only the boxes (pcr_decode_crop_batch).
template <bool kRefine>
__global__ void __launch_bounds__(256) k_pixel(DevRecord R, const PixelTile* __restrict__ tiles, uint8_t* __restrict__ out,
                                               const ApplyList* __restrict__ lists, const int32_t* __restrict__ list_idx,
                                               const CropBox* __restrict__ boxes) {
    // samples of the strip, one row-major plane per component (so that neighbouring pixels are
    // neighbouring words of LDS in phase 4); rows are one word longer than the data, which
    // spreads the rows of a block over the banks for phase 2
    __shared__ float tile[kMaxStripBlocks * 64 + 64];
    __shared__ __attribute__((aligned(16))) float qz[kMaxComp][64];       // quantiser steps, zig-zag order
    __shared__ __attribute__((aligned(16))) uint16_t zoff[kMaxComp][64];  // zig-zag index -> offset of that position from the block's corner in `tile`
    __shared__ ImgDesc img;                                // this image's descriptor, read many times below
    __shared__ ApplyList rl[kMaxComp];                     // refinement scan lists of the components (n = 0: none)
    short_kernel_priority();
    const PixelTile t = tiles[blockIdx.x];
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&R.img[t.img]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&img);
        if (threadIdx.x < sizeof(ImgDesc) / 4) dst[threadIdx.x] = src[threadIdx.x];
    }
    __syncthreads();
    const uint32_t nc = img.nc;
    const uint32_t W = img.W, H = img.H;
    uint8_t* o = out + R.out_off[t.img];
    const uint32_t hmax = img.hmax, vmax = img.vmax;
    const uint32_t mcu_px_w = 8 * hmax, mcu_px_h = 8 * vmax;
    const uint32_t per = kStripPx / mcu_px_w;              // MCUs per strip: 8 (16-px MCUs) or 16 (8-px MCUs)
    const uint32_t col0 = t.mcu_col0 * (per / kStripMcus);
    if (col0 >= img.mcux) return;                          // tiles are laid out for 8 MCUs per strip; wider strips need fewer
    const uint32_t nm = img.mcux - col0 < per ? img.mcux - col0 : per;
    const uint32_t x0 = col0 * mcu_px_w, y0 = t.mcu_row * mcu_px_h;
    const uint32_t sw = nm * mcu_px_w;                     // strip width in pixels
    const uint32_t xe = x0 + sw < W ? x0 + sw : W;         // visible part of the strip
    const uint32_t rows = y0 + mcu_px_h < H ? mcu_px_h : H - y0;
    const uint32_t row_bytes = (xe - x0) * nc;
    if (boxes) {                                            // (clamped into the image exactly as k_crop_resize clamps it)
        CropBox b = boxes[t.img];
        b.x0 = min(max(b.x0, 0), (int)W - 1); b.y0 = min(max(b.y0, 0), (int)H - 1);
        b.w = min(max(b.w, 1), (int)W - b.x0); b.h = min(max(b.h, 1), (int)H - b.y0);
        if ((int)x0 >= b.x0 + b.w || (int)xe <= b.x0 || (int)y0 >= b.y0 + b.h || (int)(y0 + rows) <= b.y0) return;
    }
    const bool dead = R.status[t.img] != kOk;
    // per component (all wave-uniform): blocks per strip row, blocks in the strip, row stride and plane
    // offset in `tile`, reciprocal of the blocks per row, first block of the strip in the coefficient buffer
    uint32_t bwc[kMaxComp], nbc[kMaxComp], pstr[kMaxComp], poff[kMaxComp], rcp[kMaxComp], first_blk[kMaxComp], bwi[kMaxComp], zmx[kMaxComp];
    bool flat[kMaxComp];
    {
        uint32_t plane0 = 0, lds = 0;
#pragma unroll
        for (uint32_t c = 0; c < kMaxComp; c++) {
            const uint32_t hs = c < nc ? img.hs[c] : 0, vs = c < nc ? img.vs[c] : 0;
            bwi[c] = c < nc ? img.bw[c] : 0;
            bwc[c] = nm * hs; nbc[c] = bwc[c] * vs; pstr[c] = bwc[c] * 8 + 1; poff[c] = lds; lds += vs * 8 * pstr[c];
            rcp[c] = recip16(bwc[c]);
            first_blk[c] = plane0 + (t.mcu_row * vs) * bwi[c] + col0 * hs;
            plane0 += c < nc ? bwi[c] * (uint32_t)img.bh[c] : 0;
            zmx[c] = c < nc ? img.zmax[c] : 0;
            flat[c] = c < nc && zmx[c] <= 1;
        }
    }
    for (uint32_t c = 0; kRefine && c < nc; c++) {
        const int32_t li = list_idx ? list_idx[t.img * kMaxComp + c] : -1;
        uint32_t* dst = reinterpret_cast<uint32_t*>(&rl[c]);
        if (li >= 0) {
            const uint32_t* src = reinterpret_cast<const uint32_t*>(&lists[li]);
            for (uint32_t e = threadIdx.x; e < sizeof(ApplyList) / 4; e += 256) dst[e] = src[e];
        } else if (threadIdx.x == 0) dst[0] = 0;           // n = 0
    }
    for (uint32_t e = threadIdx.x; e < nc * 64; e += 256) {
        const uint32_t c = e >> 6, k = e & 63;
        const uint8_t* q = R.rec + img.qoff[img.tq[c]];
        const uint32_t p = zigzag_lookup(k);
        qz[c][k] = img.qprec[img.tq[c]] ? (float)ld_be16(q + 2 * k) : (float)q[k];
        zoff[c][k] = (uint16_t)((p >> 3) * (c == 0 ? pstr[0] : (c == 1 ? pstr[1] : pstr[2])) + (p & 7));
    }
    __syncthreads();
    if (!dead) {
        const int16_t* coef = R.coef + R.coef_off[t.img];
        // phase 1: chunk = 8 consecutive coefficients (zig-zag order) of a block.  Component c starts
        // at wave c, so that the small chroma planes of a 4:2:0 strip do not all land on wave 0.
#pragma unroll
        for (uint32_t c = 0; c < kMaxComp; c++) {
            if (c >= nc) continue;
            const uint32_t tt = (threadIdx.x - 64 * c) & 255;
            const int16_t* pl = coef + (size_t)first_blk[c] * 64;
            float* plane = tile + poff[c];
            const uint32_t nref = kRefine ? rl[c].n : 0;   // scans to replay (0: the planes are final)
            const uint32_t hsc = img.hs[c], vsc = img.vs[c], cwc = img.cw[c], chc = img.ch[c];
            const uint32_t nplane = bwi[c] * (uint32_t)img.bh[c];
            if (flat[c]) {                                 // only the DC: the block is flat
                const float q0 = qz[c][0];
                for (uint32_t lb = tt; lb < nbc[c]; lb += 256) {
                    const uint32_t lrow = (lb * rcp[c]) >> 16, lcol = lb - lrow * bwc[c];
                    int dcv = pl[((size_t)lrow * bwi[c] + lcol) * 64];
                    if (kRefine && nref != 0) {
                        const uint32_t brow = t.mcu_row * vsc + lrow, bcol = col0 * hsc + lcol;
                        for (uint32_t e = 0; e < nref; e++)
                            if (rl[c].sc[e].Ss == 0 && dc_refinement_bit(R, rl[c].sc[e], brow, bcol, hsc, vsc, brow < chc && bcol < cwc)) dcv |= 1 << rl[c].sc[e].Al;
                    }
                    plane[lrow * 8 * pstr[c] + lcol * 8] = clamp255((float)dcv * q0 * 0.125f + 128.f);
                }
                continue;
            }
            for (uint32_t w = tt; w < nbc[c] * 8; w += 256) {
                const uint32_t lb = w >> 3, ch = w & 7;
                const uint32_t lrow = (lb * rcp[c]) >> 16, lcol = lb - lrow * bwc[c];
                short8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                if (ch * 8 < zmx[c]) {
                    v = *reinterpret_cast<const short8*>(pl + ((size_t)lrow * bwi[c] + lcol) * 64 + ch * 8);
                    if (kRefine && nref != 0) {
                        const uint32_t brow = t.mcu_row * vsc + lrow, bcol = col0 * hsc + lcol;
                        const bool covered = brow < chc && bcol < cwc;
                        const uint32_t b = brow * bwi[c] + bcol;       // block index in the component's plane
                        const uint32_t k0 = ch * 8;
                        for (uint32_t e = 0; e < nref; e++) {
                            const ApplyScan& S = rl[c].sc[e];
                            if (S.Ss == 0) {
                                if (k0 == 0 && dc_refinement_bit(R, S, brow, bcol, hsc, vsc, covered)) v[0] |= (short)(1 << S.Al);
                            } else if (covered && k0 <= S.Se && k0 + 7 >= S.Ss) {
                                // the eight positions k0..k0+7 as 8-bit fields of the scan's masks (all restricted to
                                // its band); the correction bit of position k0 + j is number (non-zero history
                                // positions below it) of the scan's string
                                const uint64_t* rec = R.masks + S.mask_off + (size_t)b * kRefWords;   // the block's record
                                const uint64_t hb = rec[kRefHist];
                                const uint32_t h8 = (uint32_t)(hb >> k0) & 0xFF, n8 = (uint32_t)(rec[kRefNz] >> k0) & 0xFF;
                                const uint32_t s8 = (uint32_t)(rec[kRefSign] >> k0) & 0xFF;
                                const uint32_t below = (uint32_t)__builtin_popcountll(hb & ((1ull << k0) - 1));
                                const uint32_t c8 = (uint32_t)(rec[kRefCbits] >> below) & 0xFF;
                                const int p1 = 1 << S.Al;
#pragma unroll
                                for (int j = 0; j < 8; j++) {
                                    const uint32_t bj = 1u << j;
                                    const int vj = v[j];
                                    if (h8 & bj) {
                                        if ((c8 >> __builtin_popcount(h8 & (bj - 1))) & 1) v[j] = (short)(vj > 0 ? vj + p1 : vj - p1);
                                    } else if (n8 & bj) v[j] = (short)((s8 & bj) ? p1 : -p1);
                                }
                            }
                        }
                    }
                }
                float* blk = plane + lrow * 8 * pstr[c] + lcol * 8;               // sample (0,0) of the block
                const float4 qa = *reinterpret_cast<const float4*>(&qz[c][ch * 8]), qb = *reinterpret_cast<const float4*>(&qz[c][ch * 8 + 4]);
                const uint4 zo = *reinterpret_cast<const uint4*>(&zoff[c][ch * 8]);
                blk[zo.x & 0xFFFF] = (float)v[0] * qa.x; blk[zo.x >> 16] = (float)v[1] * qa.y;
                blk[zo.y & 0xFFFF] = (float)v[2] * qa.z; blk[zo.y >> 16] = (float)v[3] * qa.w;
                blk[zo.z & 0xFFFF] = (float)v[4] * qb.x; blk[zo.z >> 16] = (float)v[5] * qb.y;
                blk[zo.w & 0xFFFF] = (float)v[6] * qb.z; blk[zo.w >> 16] = (float)v[7] * qb.w;
            }
        }
        __syncthreads();
        // phase 2: rows
#pragma unroll
        for (uint32_t c = 0; c < kMaxComp; c++) {
            if (c >= nc || flat[c]) continue;
            const uint32_t tt = (threadIdx.x - 64 * c) & 255;
            for (uint32_t w = tt; w < nbc[c] * 8; w += 256) {
                const uint32_t lb = w >> 3, v = w & 7;
                const uint32_t lrow = (lb * rcp[c]) >> 16, lcol = lb - lrow * bwc[c];
                float* rowp = tile + poff[c] + (lrow * 8 + v) * pstr[c] + lcol * 8;
                float in[8], res[8];
#pragma unroll
                for (int u = 0; u < 8; u++) in[u] = rowp[u];
                idct8(in, res);
#pragma unroll
                for (int x = 0; x < 8; x++) rowp[x] = res[x];
            }
        }
        __syncthreads();
        // phase 3: columns
#pragma unroll
        for (uint32_t c = 0; c < kMaxComp; c++) {
            if (c >= nc || flat[c]) continue;
            const uint32_t tt = (threadIdx.x - 64 * c) & 255;
            for (uint32_t w = tt; w < nbc[c] * 8; w += 256) {
                const uint32_t lb = w >> 3, x = w & 7;
                const uint32_t lrow = (lb * rcp[c]) >> 16, lcol = lb - lrow * bwc[c];
                float* colp = tile + poff[c] + (lrow * 8) * pstr[c] + lcol * 8 + x;
                float in[8], res[8];
#pragma unroll
                for (int v = 0; v < 8; v++) in[v] = colp[v * pstr[c]];
                idct8(in, res);
#pragma unroll
                for (int y = 0; y < 8; y++) colp[y * pstr[c]] = clamp255(res[y] + 128.f);
            }
        }
        __syncthreads();
    }
    // phase 4: one lane per group of 12 bytes of an output row of the strip (4 RGB pixels or 12 gray ones),
    // stored as three dwords.  Rows start wherever width x 3 puts them, so the stores are in general not
    // 4-byte aligned: global memory takes unaligned dword accesses (a store that straddles a line is split
    // by the memory pipeline), which is far cheaper than shifting every group into alignment.
    if (row_bytes == 0) return;
    const uint32_t shx0 = img.hs[0] == hmax ? 0 : 1, shy0 = img.vs[0] == vmax ? 0 : 1;     // sampling factors are 1 or 2
    const uint32_t shx1 = nc > 1 && img.hs[1] != hmax, shy1 = nc > 1 && img.vs[1] != vmax;
    const uint32_t shx2 = nc > 2 && img.hs[2] != hmax, shy2 = nc > 2 && img.vs[2] != vmax;
    const uint32_t m0 = flat[0] ? ~7u : ~0u, m1 = flat[1] ? ~7u : ~0u, m2 = flat[2] ? ~7u : ~0u;   // flat: read the block's corner
    const uint32_t groups = (row_bytes + 11) / 12;         // per row; only the last one can be partial
    const uint32_t rcpg = recip16(groups);
    for (uint32_t it = threadIdx.x; it < rows * groups; it += 256) {
        const uint32_t ly = (it * rcpg) >> 16, g = it - ly * groups;
        const uint32_t r0 = g * 12;                        // byte offset of the group in the row
        uint8_t* wp = o + ((size_t)(y0 + ly) * W + x0) * nc + r0;
        uint32_t wd[3] = {0, 0, 0};
        if (nc == 1) {
            const float* yrow = tile + poff[0] + ((ly >> shy0) & m0) * pstr[0];
#pragma unroll
            for (int j = 0; j < 12; j++) {
                const uint32_t r = r0 + j;
                const float s = (r < row_bytes && !dead) ? yrow[(r >> shx0) & m0] : 0.f;
                wd[j >> 2] |= (uint32_t)round_u8(s) << (8 * (j & 3));
            }
        } else {
            const uint32_t p0 = g * 4;                     // first of the group's four pixels
            const float* yrow = tile + poff[0] + ((ly >> shy0) & m0) * pstr[0];
            const float* brow = tile + poff[1] + ((ly >> shy1) & m1) * pstr[1];
            const float* rrow = tile + poff[2] + ((ly >> shy2) & m2) * pstr[2];
            uint32_t three[4];                             // R | G << 8 | B << 16 of the four pixels
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const uint32_t lx = p0 + q;
                uint8_t px[3] = {0, 0, 0};
                if (lx * 3 < row_bytes && !dead)
                    ycc_to_rgb(yrow[(lx >> shx0) & m0], brow[(lx >> shx1) & m1], rrow[(lx >> shx2) & m2], px);
                three[q] = (uint32_t)px[0] | ((uint32_t)px[1] << 8) | ((uint32_t)px[2] << 16);
            }
            wd[0] = three[0] | (three[1] << 24); wd[1] = (three[1] >> 8) | (three[2] << 16); wd[2] = (three[2] >> 16) | (three[3] << 8);
        }
        if (r0 + 12 <= row_bytes) {
            struct __attribute__((packed, aligned(1))) Twelve { uint32_t a, b, c; };
            Twelve tw; tw.a = wd[0]; tw.b = wd[1]; tw.c = wd[2];
            *reinterpret_cast<Twelve*>(wp) = tw;           // one (possibly unaligned) 12-byte store
        } else {
#pragma unroll
            for (int j = 0; j < 12; j++)
                if (r0 + j < row_bytes) wp[j] = (uint8_t)(wd[j >> 2] >> (8 * (j & 3)));
        }
    }
}

// --------------------------------------------------------------------------------------
// k_gather: copy regions 1..have of one image back to back, append FF D9 if asked.
// --------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_gather(DevRecord R, uint32_t i, uint32_t have, int add_eoi, uint8_t* dst) {
    uint32_t w = 0;
    for (uint32_t g = 0; g < have; g++) {
        uint32_t p = R.off[(size_t)g * R.n + i], L = R.len[(size_t)g * R.n + i];
        for (uint32_t j = blockIdx.x * 256 + threadIdx.x; j < L; j += gridDim.x * 256) dst[w + j] = R.rec[p + j];
        w += L;
    }
    if (add_eoi && blockIdx.x == 0 && threadIdx.x == 0) { dst[w] = 0xFF; dst[w + 1] = 0xD9; }
}

// --------------------------------------------------------------------------------------
// k_probe_scalar: yardstick for the entropy kernels.  Every wavefront runs `iters` times a chain of 16
// dependent scalar instructions, the same kind of work a wave-uniform decoder is made of; the host
// turns the duration into scalar instructions per second for a given number of wavefronts per CU.
// --------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_probe_scalar(uint32_t* out, uint32_t iters, uint32_t seed) {
    uint32_t a = uni(seed + blockIdx.x), b = a * 3u + 1u;
    for (uint32_t i = 0; i < iters; i++) {
        asm volatile(
            "s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n"
            "s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n"
            "s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n"
            "s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n s_add_u32 %0, %0, %1\n s_xor_b32 %1, %1, %0\n"
            : "+s"(a), "+s"(b) : : "scc");
    }
    if (threadIdx.x == 0) out[blockIdx.x] = a ^ b;
}

// zero every coefficient except element 0 of each 64-element block (n16: 16-byte units, 8 per block)
__global__ void __launch_bounds__(256) k_fill_zero_keep_dc(uint4* p, size_t n16) {
    short_kernel_priority();
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if ((i & 7) == 0) v.x = p[i].x & 0xFFFFu;          // the DC coefficient is the low half of the block's first word
        p[i] = v;
    }
}

__global__ void __launch_bounds__(256) k_fill_zero(uint4* p, size_t n16) {
    short_kernel_priority();
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace pcr
