// gfx950 kernels of the PCR decode path.  One kernel per step:
//   k_index      scan-group index (prefix sums of region lengths)
//   k_parse      JPEG marker parsing, one lane per image
//   k_unstuff    byte un-stuffing + restart-interval location, one workgroup per (image, scan)
//   k_dc_first, k_ac_first, k_ac_refine   progressive Huffman decode, one wavefront per unit: a restart
//                interval of a scan, or the stretch between two entry points of the record (the whole scan
//                where there is neither)
//   k_refine_blocks   second phase of AC refinement, one lane per block
//   k_dc_first_lanes, k_ac_first_lanes, k_ac_refine_lanes   the same scans with one LANE per unit (pcr_lanes.h), for
//                launches with very many units; k_refine_history, k_refine_deal: per-block work before and after
//   k_apply      data-parallel refinement (DC bits, AC corrections and new coefficients)
//   k_pixel      de-quantise + IDCT + chroma replication + YCbCr->RGB + store
//   k_gather     materialise an image's scan prefix (parity hook)
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "pcr_common.h"
#include "pcr_format.h"
#include "pcr_entropy.h"
#include "pcr_lanes.h"
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

// Workgroups are handed to the chip's eight dies (XCDs, each with its own L2) round-robin by their index.  Kernels whose
// neighbouring work items write neighbouring memory (the runs of MCUs of one image row, the rows of cells of one image)
// take item xcd_major(blockIdx.x, gridDim.x) instead of item blockIdx.x: every die then works through one contiguous
// eighth of the list, so the cache lines two neighbours share are completed in one L2 instead of being written back
// in parts from two.
constexpr uint32_t kXcds = 8;
PCR_D uint32_t xcd_major(uint32_t b, uint32_t n) {
    const uint32_t q = n / kXcds, r = n - q * kXcds, x = b % kXcds, i = b / kXcds;
    return x * q + (x < r ? x : r) + i;
}
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
    int16_t* dc;               // the DC coefficients, one per block in the order of the blocks of `coef` (written by the DC first scans and
                               // by sequential scans): what the pixel kernels read; element 0 of a block in `coef` holds it only for the
                               // coefficient export
    uint64_t* masks;
    int32_t* status;           // [n]
    AcTab* tabs;               // Huffman tables of the AC scans: those of the refinement scans are written by phase 1 for phase 2;
                               // with tabs_prebuilt, k_build_tables has written all of them before the entropy kernels start
    const uint32_t* tab_idx;   // [n][G] index into tabs
    DcTab* dctabs;             // with tabs_prebuilt: the DC tables of the DC first scans, three slots per scan (one per scan component)
    const uint32_t* dctab_idx; // [n][G] first slot of the scan in dctabs
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
    short_kernel_priority();
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
    short_kernel_priority();
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= R.n) return;
    parse_image(R.rec, R.off, R.len, R.n, i, R.nscans[i], kmax, &R.img[i], &R.scan[(size_t)i * R.G]);
    if (!(keep_status && R.status[i] != kOk)) R.status[i] = R.img[i].status;
}

// --------------------------------------------------------------------------------------
// k_unstuff: per (image, scan) remove stuffed zeros, fill bytes and restart markers from the
// entropy-coded segment, stop at the first other marker, note where each restart interval
// begins.  256 lanes x 8 bytes per step.  A lane classifies its eight bytes at once (one flag bit per
// byte in a 64-bit word: equal to FF, to 00, a restart marker's second byte, and the same of the byte
// that follows), squeezes out the few it drops and puts the rest, byte by byte, at their place in a ring
// in LDS; the workgroup then stores the words the step has completed, already in the big-endian order
// the decoders read (one 4-byte store per lane instead of eight single bytes).
// --------------------------------------------------------------------------------------
constexpr int kUnstuffPer = 8;
constexpr uint32_t kUnstuffRing = 4096;                    // bytes; a step adds at most 2048 to fewer than 4 left over

// 0x80 in every byte of the result whose byte in x is zero (exact, no carries between bytes)
PCR_D uint64_t zero_bytes(uint64_t x) {
    const uint64_t m = 0x7F7F7F7F7F7F7F7Full;
    return ~(((x & m) + m) | x | m);
}
// the flags (0x80 per byte) of the bytes below byte n (n >= 8: all)
PCR_D uint64_t flags_below(uint32_t n) { return n >= 8 ? 0x8080808080808080ull : ((1ull << (8 * n)) - 1) & 0x8080808080808080ull; }

// grid: (images, scan groups kfrom .. kmax-1)
__global__ void __launch_bounds__(256) k_unstuff(DevRecord R, uint32_t kfrom, uint32_t kmax) {
    short_kernel_priority();
    __shared__ uint32_t part[4];
    __shared__ uint32_t s_stop;
    __shared__ __attribute__((aligned(16))) uint32_t ring[kUnstuffRing / 4];
    uint32_t i = blockIdx.x, g = kfrom + blockIdx.y;
    if (g >= kmax) return;
    const ImgDesc& img = R.img[i];
    if (img.status != kOk || g >= img.nscans) return;
    const ScanDesc& sd = R.scan[(size_t)i * R.G + g];
    const uint8_t* src = R.rec + sd.data_off;
    uint8_t* dst = R.clean + clean_base(sd.data_off);     // stored as big-endian 32-bit words: byte o goes to o ^ 3
    const uint32_t L = sd.data_len;
    const uint32_t sb = R.slot_base[(size_t)i * R.G + g], sc = R.slot_cnt[(size_t)i * R.G + g];
    uint8_t* ringb = reinterpret_cast<uint8_t*>(ring);
    uint32_t out_total = 0, rst_total = 0;
    if (threadIdx.x == 0) { s_stop = 0xFFFFFFFFu; R.ivl_start[sb] = 0; }
    __syncthreads();
    for (uint32_t base = 0; base < L; base += 256 * kUnstuffPer) {
        const uint32_t p0 = base + threadIdx.x * kUnstuffPer;
        const uint32_t nvalid = p0 >= L ? 0u : (L - p0 < 8 ? L - p0 : 8u);
        uint64_t w = 0;                                  // byte j of the lane: bits 8j .. 8j+7
        if (nvalid == 8) {
            struct __attribute__((packed, aligned(1))) Two { uint32_t a, b; };
            const Two t = *reinterpret_cast<const Two*>(src + p0);
            w = (uint64_t)t.a | ((uint64_t)t.b << 32);
        } else for (uint32_t j = 0; j < nvalid; j++) w |= (uint64_t)src[p0 + j] << (8 * j);
        const uint32_t prevb = (p0 > 0 && p0 <= L) ? src[p0 - 1] : 0u;
        const bool has_next = p0 + 8 < L;
        const uint32_t nextb = has_next ? src[p0 + 8] : 0u;
        const uint64_t top = 0x8000000000000000ull, all = 0x8080808080808080ull;
        const uint64_t valid = flags_below(nvalid);
        const uint64_t ff = zero_bytes(~w), z0 = zero_bytes(w), rs = zero_bytes((w & 0xF8F8F8F8F8F8F8F8ull) ^ 0xD0D0D0D0D0D0D0D0ull);
        // the same of the byte that follows (none follows the segment's last byte) and of the byte before
        const uint64_t nvalid_next = (valid >> 8) | (has_next ? top : 0);
        const uint64_t nff = ((ff >> 8) | (nextb == 0xFF ? top : 0)) & nvalid_next;
        const uint64_t nz0 = ((z0 >> 8) | (nextb == 0x00 ? top : 0)) & nvalid_next;
        const uint64_t nrs = ((rs >> 8) | ((nextb & 0xF8) == 0xD0 ? top : 0)) & nvalid_next;
        const uint64_t pff = (ff << 8) | (prevb == 0xFF ? 0x80ull : 0);
        // FF: kept if a zero follows (a data byte), a restart marker if D0..D7 follows, dropped if another FF follows (fill),
        // else the marker that ends the segment.  Others: dropped if they are the second byte of FF 00 or of a restart marker.
        uint64_t keep = valid & ((all & ~ff & ~(pff & (z0 | rs))) | (ff & nz0));
        uint64_t rst = valid & ff & nrs;
        const uint64_t stopf = valid & ff & ~nrs & ~nz0 & ~nff;
        if (stopf) atomicMin(&s_stop, p0 + ((uint32_t)__builtin_ctzll(stopf) >> 3));
        __syncthreads();
        const uint32_t stop_all = s_stop;
        if (stop_all != 0xFFFFFFFFu) {                     // drop what lies at or after the terminating marker
            const uint64_t before = flags_below(stop_all > p0 ? stop_all - p0 : 0u);
            keep &= before; rst &= before;
        }
        // prefix sums of (bytes kept | restart markers << 16) over the 256 lanes: inside each wavefront by lane
        // shuffles, then the four wavefront totals through LDS
        const uint32_t nkeep = (uint32_t)__builtin_popcountll(keep);
        const uint32_t mine = nkeep | ((uint32_t)__builtin_popcountll(rst) << 16);
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
        const uint32_t o = out_total + (excl & 0xFFFF);
        if (rst) {                                         // (rare) where the next interval begins: behind the bytes kept ahead of the marker
            uint32_t r = rst_total + (excl >> 16);
            for (uint64_t m = rst; m; m &= m - 1) {
                const uint32_t j = (uint32_t)__builtin_ctzll(m) >> 3;
                r++;
                if (r < sc) R.ivl_start[sb + r] = o + (uint32_t)__builtin_popcountll(keep & flags_below(j));
            }
        }
        // squeeze the dropped bytes out (few: one step of the loop per dropped byte), then the kept ones into the ring
        uint64_t kw = w;
        for (uint64_t drop = valid & ~keep; drop; ) {
            const uint32_t j = 63u - (uint32_t)__builtin_clzll(drop);      // highest first, so that the positions below stay put
            drop &= ~(1ull << j);
            const uint32_t sh = (j >> 3) * 8;                               // first bit of the byte
            const uint64_t low = sh ? (kw & ((1ull << sh) - 1)) : 0;
            kw = low | (sh < 56 ? (kw >> (sh + 8)) << sh : 0);
        }
        for (uint32_t j = 0; j < nkeep; j++) ringb[(o + j) & (kUnstuffRing - 1)] = (uint8_t)(kw >> (8 * j));
        const uint32_t tot = w0 + w1 + w2 + w3;
        const uint32_t end = out_total + (tot & 0xFFFF);
        __syncthreads();
        for (uint32_t wi = (out_total >> 2) + threadIdx.x; wi < (end >> 2); wi += 256)      // the words complete by now
            *reinterpret_cast<uint32_t*>(dst + 4 * (size_t)wi) = __builtin_bswap32(ring[wi & (kUnstuffRing / 4 - 1)]);
        out_total = end; rst_total += tot >> 16;
        __syncthreads();
        if (stop_all != 0xFFFFFFFFu) break;
    }
    if (threadIdx.x < (out_total & 3u)) {                  // the bytes of the last, incomplete word
        const uint32_t q = (out_total & ~3u) + threadIdx.x;
        dst[q ^ 3u] = ringb[q & (kUnstuffRing - 1)];
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
// (With tens of thousands of units per launch the balance tips: see pcr_lanes.h and the kernels
// k_ac_first_lanes / k_ac_refine_lanes below, which the host takes for such launches.)
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
        const uint32_t stride = uni(entry_stride(ld_le16(R.rec + hdr_ecount_pos(R.n, R.G, un.scan, un.img))));   // 16 bytes, or 8 without DC predictions
        const uint8_t* e = R.rec + uni(R.ent_off[ig]) + (size_t)stride * un.interval;             // entry j; entry j-1 lies one stride before it
        const uint32_t total = uni(R.ivl_start[sb + sc]) * 8;                                    // bits of the scan's unstuffed data
        uint32_t m0 = 0, bit0 = 0, m1 = mcus, bit1 = total;
        if (un.interval > 0) {
            const uint8_t* p = e - stride;
            m0 = uni(ld_le32(p)); bit0 = uni(ld_le32(p + 4));
            if (stride == kEntryBytes) { ls.pred[0] = uni((int)(int16_t)ld_le16(p + 8)); ls.pred[1] = uni((int)(int16_t)ld_le16(p + 10)); ls.pred[2] = uni((int)(int16_t)ld_le16(p + 12)); }
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

PCR_D uint32_t lane_le32(const uint8_t* p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }

// The same checks and ranges as unit_setup (pcr_kernels.h), without the assumption that the unit is wave-uniform.
PCR_D void lane_unit_setup(const DevRecord& R, const Unit& un, const uint32_t* __restrict__ clean32, LaneUnit* U) {
    U->ok = false;
    const ImgDesc* img = &R.img[un.img];
    if (R.status[un.img] != kOk || un.scan >= img->nscans) return;
    const size_t ig = (size_t)un.img * R.G + un.scan;
    const ScanDesc* sd = &R.scan[ig];
    if (!sd->valid || sd->ns != 1 || sd->Ss == 0) return;
    const uint32_t sb = R.slot_base[ig], sc = R.slot_cnt[ig];
    const uint32_t ri = sd->ri, mcus = sd->mcus;
    if (ri == 0 && sc > 1) {
        const uint32_t stride = entry_stride(ld_le16(R.rec + hdr_ecount_pos(R.n, R.G, un.scan, un.img)));
        const uint8_t* e = R.rec + R.ent_off[ig] + (size_t)stride * un.interval;
        const uint32_t total = R.ivl_start[sb + sc] * 8;
        uint32_t m0 = 0, b0 = 0, m1 = mcus, b1 = total;
        if (un.interval > 0) { m0 = lane_le32(e - stride); b0 = lane_le32(e - stride + 4); }
        if (un.interval + 1 < sc) { m1 = lane_le32(e); b1 = lane_le32(e + 4); }
        if (!(m0 < m1 && m1 <= mcus && b0 <= b1 && b1 <= total)) { R.status[un.img] = kEFormat; return; }
        U->mcu0 = m0; U->mcu1 = m1; U->bit0 = b0; U->bit1 = b1;
    } else {
        const uint32_t b0 = R.ivl_start[sb + un.interval], b1 = R.ivl_start[sb + un.interval + 1];
        U->mcu0 = ri ? un.interval * ri : 0;
        U->mcu1 = ri ? (U->mcu0 + ri < mcus ? U->mcu0 + ri : mcus) : mcus;
        if (U->mcu0 >= mcus) return;
        U->bit0 = b0 * 8; U->bit1 = (b1 > b0 ? b1 : b0) * 8;
    }
    U->mcu_w = sd->mcu_w;
    if (U->mcu_w == 0) return;
    U->Ss = sd->Ss; U->Se = sd->Se; U->Al = sd->Al;
    const uint32_t c = sd->comp[0];
    size_t po = 0;
    for (uint32_t q = 0; q < c && q < kMaxComp; q++) po += (size_t)img->bw[q] * img->bh[q] * 64;
    U->bw = img->bw[c];
    U->plane = R.coef + R.coef_off[un.img] + po;
    U->plane_elems = (uint32_t)img->bw[c] * img->bh[c] * 64;
    U->words = clean32 + (clean_base(sd->data_off) >> 2);
    U->tab = nullptr;                                         // (the kernel points it at the job's copy in LDS)
    U->ok = true;
}

// One job of a lane-per-unit kernel: units [first, first + count) of the launch's list, count <= 64, and the scans they
// belong to (image * scans per image + scan), kLaneTabs at most: one Huffman table each.
constexpr int kLaneTabs = 8;
struct LaneJob { uint32_t first, count, ntab; uint32_t key[kLaneTabs]; };

// The AC tables of a job into LDS (call with every lane of the wavefront) and the slot of the table of scan `key`
// (>= kLaneTabs: not among the job's -- the host never makes such a job).
PCR_D uint32_t lane_table_slots(const DevRecord& R, const LaneJob& job, uint32_t key, bool mine, uint32_t (*tabs)[kLaneTabWords]) {
    const uint32_t t = threadIdx.x;
    uint32_t slot = ~0u;
#pragma unroll
    for (uint32_t sl = 0; sl < (uint32_t)kLaneTabs; sl++) {
        if (sl < job.ntab) {                                  // (the same for all lanes)
            const uint32_t k = job.key[sl];
            if (k < R.n * R.G) {
                const uint32_t* src = reinterpret_cast<const uint32_t*>(&R.tabs[R.tab_idx[k]]);
                for (uint32_t e = t; e < kLaneTabWords; e += kEntropyLanes) tabs[sl][e] = src[e];
                if (k == key) slot = sl;
            }
        }
    }
    __syncthreads();
    return mine ? slot : ~0u;
}

// SHAPE: which DC decoder (dc_shape) the units of this launch take; the host sorts the units by it.
template <int SHAPE>
__global__ void __launch_bounds__(kEntropyLanes) k_dc_first(DevRecord R, const Unit* __restrict__ units, uint32_t nunits,
        const uint32_t* __restrict__ clean32, const uint64_t* __restrict__ hist64, uint32_t to_planes) {
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
    if (R.tabs_prebuilt) {                                  // built once per scan by k_build_tables: copy the distinct ones
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&R.dctabs[R.dctab_idx[(size_t)un.img * R.G + un.scan]]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&tabs[0]);
        constexpr uint32_t kWords = sizeof(DcTab) / 4;
        for (uint32_t e = threadIdx.x; e < kWords; e += kEntropyLanes) {
            dst[e] = src[e];
            if (tj1 == 1) dst[kWords + e] = src[kWords + e];
            if (tj2 != 0 && tj2 != tj1) dst[(uint32_t)tj2 * kWords + e] = src[2 * kWords + e];
        }
    } else {
        if (threadIdx.x == 0) dctab_build(&tabs[0], R.rec + o0);
        if (threadIdx.x == 1 && tj1 == 1) dctab_build(&tabs[1], R.rec + o1);
        if (threadIdx.x == 2 && tj2 != 0 && tj2 != tj1) dctab_build(&tabs[tj2], R.rec + o2);
    }
    __syncthreads();
    DcWindowReader wr;                                      // tables by scan component
    wr.init(L.words, L.byte_off, L.sub_bits, L.nbits, &tabs[0], &tabs[uni(tj1)], &tabs[uni(tj2)], L.ls.ns, threadIdx.x);
    CoefSink sink;
    // (to_planes = 0: only the compact copy, one value per block -- all a decode without AC scans and refinements reads)
    sink.init(to_planes ? L.base : nullptr, L.base_elems, L.ls.Al, R.dc + (uni((uint64_t)R.coef_off[un.img]) >> 6));
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
// grid: (n, scans), scans k0 .. k0 + gridDim.y - 1.  dc_too = 0: the DC first scans of this call are all decoded by
// k_dc_first_lanes, which builds its own tables.
__global__ void __launch_bounds__(kEntropyLanes) k_build_tables(DevRecord R, uint32_t k0, uint32_t dc_too) {
    __shared__ AcTab tab;
    short_kernel_priority();
    const uint32_t i = blockIdx.x, g = k0 + blockIdx.y;
    if (R.status[i] != kOk || g >= R.img[i].nscans) return;
    const size_t ig = (size_t)i * R.G + g;
    const ScanDesc* sd = &R.scan[ig];
    if (!sd->valid) return;
    if (sd->Ss == 0) {                                      // DC first scans: the table of every scan component (sequential scans build their own)
        if (dc_too && sd->Ah == 0 && R.img[i].progressive && threadIdx.x < sd->ns)
            dctab_build(&R.dctabs[R.dctab_idx[ig] + threadIdx.x], R.rec + sd->dc_off[threadIdx.x]);
        return;
    }
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

// The same scan kind with one LANE per unit (pcr_lanes.h).  One wavefront per job: up to 64 consecutive units of the
// launch's list that use at most kLaneTabs different Huffman tables between them (the host cuts the list that way; the
// units of one scan lie together).  The tables (built by k_build_tables) are copied into LDS first: every lane looks
// its codes up in its own table, and 64 scattered reads of memory per symbol would bound the kernel by the rate at
// which the memory pipeline takes requests.
__global__ void __launch_bounds__(kEntropyLanes) k_ac_first_lanes(DevRecord R, const Unit* __restrict__ units, const LaneJob* __restrict__ jobs,
        const uint32_t* __restrict__ clean32) {
    __shared__ uint32_t tabs[kLaneTabs][kLaneTabWords];
    __shared__ LaneRing rings;
    const LaneJob job = jobs[blockIdx.x];
    const uint32_t t = threadIdx.x;
    const bool mine = t < job.count;
    Unit un = units[job.first + (mine ? t : 0u)];
    const uint32_t key = un.img * R.G + un.scan;
    const uint32_t slot = lane_table_slots(R, job, key, mine, tabs);
    LaneUnit U;
    U.ok = false;
    if (mine && slot < (uint32_t)kLaneTabs) lane_unit_setup(R, un, clean32, &U);
    if (!U.ok) return;
    U.tab = reinterpret_cast<const LaneTab*>(&tabs[slot][0]);
    const int rc = lane_decode_ac_first(U, &rings, t);
    if (rc != kOk) R.status[un.img] = rc;
}

// AC refinement scans with one lane per unit: as k_ac_first_lanes.  k_refine_history must have run for the scans of the
// launch, k_refine_deal must follow.
__global__ void __launch_bounds__(kEntropyLanes) k_ac_refine_lanes(DevRecord R, const Unit* __restrict__ units, const LaneJob* __restrict__ jobs,
        const uint32_t* __restrict__ clean32) {
    __shared__ uint32_t tabs[kLaneTabs][kLaneTabWords];
    __shared__ LaneRing rings;
    __shared__ LaneHistRing hring;
    const LaneJob job = jobs[blockIdx.x];
    const uint32_t t = threadIdx.x;
    const bool mine = t < job.count;
    Unit un = units[job.first + (mine ? t : 0u)];
    const uint32_t key = un.img * R.G + un.scan;
    const uint32_t slot = lane_table_slots(R, job, key, mine, tabs);
    LaneUnit U;
    U.ok = false;
    if (mine && slot < (uint32_t)kLaneTabs) lane_unit_setup(R, un, clean32, &U);
    if (!U.ok) return;
    U.tab = reinterpret_cast<const LaneTab*>(&tabs[slot][0]);
    const int rc = lane_decode_ac_refine(U, R.masks + R.mask_off[key], U.plane_elems >> 6, &rings, &hring, t);
    if (rc != kOk) R.status[un.img] = rc;
}

// DC first scans with one lane per unit (pcr_lanes.h: lane_decode_dc_first): 64 consecutive units of the launch's list
// per wavefront, whatever images they belong to -- every lane builds its own small tables.  The checks and ranges are
// those of unit_setup.
PCR_D __attribute__((always_inline)) void lane_dc_unit_setup(const DevRecord& R, const Unit& un, const uint32_t* __restrict__ clean32, uint32_t to_planes, LaneDcUnit* U) {
    U->ok = false;
    const ImgDesc* img = &R.img[un.img];
    if (R.status[un.img] != kOk || un.scan >= img->nscans) return;
    const size_t ig = (size_t)un.img * R.G + un.scan;
    const ScanDesc* sd = &R.scan[ig];
    if (!sd->valid || sd->Ss != 0 || sd->Ah != 0 || !img->progressive || sd->ns < 1 || sd->ns > kMaxComp) return;
    const uint32_t sb = R.slot_base[ig], sc = R.slot_cnt[ig];
    const uint32_t ri = sd->ri, mcus = sd->mcus;
    U->pred0 = U->pred1 = U->pred2 = 0;
    if (ri == 0 && sc > 1) {
        const uint32_t stride = entry_stride(ld_le16(R.rec + hdr_ecount_pos(R.n, R.G, un.scan, un.img)));
        const uint8_t* e = R.rec + R.ent_off[ig] + (size_t)stride * un.interval;
        const uint32_t total = R.ivl_start[sb + sc] * 8;
        uint32_t m0 = 0, b0 = 0, m1 = mcus, b1 = total;
        if (un.interval > 0) {
            const uint8_t* p = e - stride;
            m0 = lane_le32(p); b0 = lane_le32(p + 4);
            if (stride == kEntryBytes) { U->pred0 = (int)(int16_t)ld_le16(p + 8); U->pred1 = (int)(int16_t)ld_le16(p + 10); U->pred2 = (int)(int16_t)ld_le16(p + 12); }
        }
        if (un.interval + 1 < sc) { m1 = lane_le32(e); b1 = lane_le32(e + 4); }
        if (!(m0 < m1 && m1 <= mcus && b0 <= b1 && b1 <= total)) { R.status[un.img] = kEFormat; return; }
        U->mcu0 = m0; U->mcu1 = m1; U->bit0 = b0; U->bit1 = b1;
    } else {
        const uint32_t b0 = R.ivl_start[sb + un.interval], b1 = R.ivl_start[sb + un.interval + 1];
        U->mcu0 = ri ? un.interval * ri : 0;
        U->mcu1 = ri ? (U->mcu0 + ri < mcus ? U->mcu0 + ri : mcus) : mcus;
        if (U->mcu0 >= mcus) return;
        U->bit0 = b0 * 8; U->bit1 = (b1 > b0 ? b1 : b0) * 8;
    }
    U->mcu_w = sd->mcu_w;
    if (U->mcu_w == 0) return;
    U->ns = sd->ns; U->Al = sd->Al;
    const uint32_t nb0 = (uint32_t)img->bw[0] * img->bh[0], nb1 = img->nc > 1 ? (uint32_t)img->bw[1] * img->bh[1] : 0u, nb2 = img->nc > 2 ? (uint32_t)img->bw[2] * img->bh[2] : 0u;
    const bool one = sd->ns == 1;                               // a scan of one component goes block by block
    // scan component j is component c of the image (sampling factors are 1 or 2: the parser refuses anything else)
    auto component = [&](int j, uint32_t* hs, uint32_t* vs, uint32_t* bw, uint32_t* pblk, const uint8_t** def) {
        const int c = j < sd->ns ? (int)sd->comp[j] : 0;
        *hs = one ? 1u : (uint32_t)img->hs[c]; *vs = one ? 1u : (uint32_t)img->vs[c]; *bw = img->bw[c];
        *pblk = c == 0 ? 0u : (c == 1 ? nb0 : nb0 + nb1);
        *def = R.rec + sd->dc_off[j < sd->ns ? j : 0];
    };
    component(0, &U->hs0, &U->vs0, &U->bw0, &U->pblk0, &U->def0);
    component(1, &U->hs1, &U->vs1, &U->bw1, &U->pblk1, &U->def1);
    component(2, &U->hs2, &U->vs2, &U->bw2, &U->pblk2, &U->def2);
    U->nblocks = nb0 + nb1 + nb2;
    U->dense = R.dc + (R.coef_off[un.img] >> 6);
    U->planes = to_planes ? R.coef + R.coef_off[un.img] : nullptr;
    U->words = clean32 + (clean_base(sd->data_off) >> 2);
    U->ok = true;
}

__global__ void __launch_bounds__(kEntropyLanes) k_dc_first_lanes(DevRecord R, const Unit* __restrict__ units, uint32_t nunits,
        const uint32_t* __restrict__ clean32, uint32_t to_planes) {
    __shared__ LaneRing rings;
    __shared__ LaneDcTabs tabs;
    short_kernel_priority();
    const uint32_t t = threadIdx.x, u = blockIdx.x * kEntropyLanes + t;
    LaneDcUnit U;
    U.ok = false;
    Unit un = units[u < nunits ? u : 0u];
    if (u < nunits) lane_dc_unit_setup(R, un, clean32, to_planes, &U);
    if (!U.ok) return;
    const int rc = lane_decode_dc_first(U, &rings, &tabs, t);
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
    sink.init(L.base, L.base_elems, 0, R.dc + (uni((uint64_t)R.coef_off[un.img]) >> 6));
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
    int rc = skim_ac_refine(&wr, L.ls, hp, mk, plane);
    if (rc != kOk) R.status[un.img] = rc;
}

// Phase 2 of AC refinement: one lane per block of the scan.
struct RefineScan { uint32_t img; uint32_t scan; };
// The per-block helpers of the lane decoders take their work from a list instead: chunk `chunk` (256 blocks) of scan
// `entry` of the launch's RefineScan list -- the planes of a record differ in size by an order of magnitude (luma and
// chroma, small and large images), and a grid sized for the largest would be mostly workgroups that find nothing to do.
struct RefineTile { uint32_t entry; uint32_t chunk; };

// What the lane-per-unit refinement decoder needs before and after it, one lane per block of the scan (the grid of
// k_refine_blocks).  k_refine_history: the kRefHist word of every block -- which positions of the band are non-zero
// when the scan starts: what the AC first scans left in the coefficient plane, and what earlier refinement scans of the
// band added (their kRefNz words).  k_refine_deal: the correction bits the decoder left in reading order go to the
// history positions they belong to (kRefPlus as every consumer reads it).
PCR_D bool refine_block_of_lane(const DevRecord& R, const RefineScan& a, uint32_t chunk, size_t* ig_out, uint32_t* blk_out, uint32_t* plane_out) {
    if (R.status[a.img] != kOk) return false;
    const ImgDesc* img = &R.img[a.img];
    const size_t ig = (size_t)a.img * R.G + a.scan;
    const int c = R.scan[ig].comp[0];
    const uint32_t cw = img->cw[c], ncov = cw * img->ch[c];
    const uint32_t b = chunk * 256 + threadIdx.x;
    if (b >= ncov) return false;
    const uint32_t bw = img->bw[c];
    *ig_out = ig; *blk_out = (b / cw) * bw + (b % cw); *plane_out = bw * img->bh[c];
    return true;
}
// k_refine_history works through the padded plane (blocks the image does not cover included: they hold zeros), 64
// consecutive blocks -- 8 KB of coefficients -- per wavefront: lane i of step j loads 16-byte chunk 64 j + i of them, so
// that every load instruction reads one contiguous kilobyte, turns its eight coefficients into eight mask bits, and leaves
// the byte in LDS where the lane that owns the block picks up all eight.  grid: one workgroup per tile (chunks of the padded planes).
__global__ void __launch_bounds__(256) k_refine_history(DevRecord R, const RefineScan* __restrict__ rs, const RefineTile* __restrict__ tiles) {
    __shared__ __attribute__((aligned(8))) uint8_t bytes[4][64 * 8];
    short_kernel_priority();
    const RefineTile tile = tiles[blockIdx.x];
    const RefineScan a = rs[tile.entry];
    if (R.status[a.img] != kOk) return;
    const ImgDesc* img = &R.img[a.img];
    const size_t ig = (size_t)a.img * R.G + a.scan;
    const ScanDesc* sd = &R.scan[ig];
    const int c = sd->comp[0];
    const uint32_t plane = (uint32_t)img->bw[c] * img->bh[c];
    if (tile.chunk * 256 >= plane) return;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint32_t blk0 = tile.chunk * 256 + wave * 64, blk = blk0 + lane;
    uint64_t m = 0;
    // An earlier refinement scan of the very same band has this word already: what it started from and what it added
    // are what this scan starts from (16 bytes per block instead of the block's 128 bytes of coefficients).
    const ScanDesc* first = sd->nhist ? &R.scan[(size_t)a.img * R.G + sd->hist[0]] : sd;
    const bool from_records = sd->nhist && first->Ss == sd->Ss && first->Se == sd->Se;
    if (from_records) {
        if (blk < plane) m = R.masks[R.mask_off[(size_t)a.img * R.G + sd->hist[0]] + (size_t)kRefHist * plane + blk];
    } else {
        size_t po = 0;
        for (int q = 0; q < c; q++) po += (size_t)img->bw[q] * img->bh[q] * 64;
        const uint4* src = reinterpret_cast<const uint4*>(R.coef + R.coef_off[a.img] + po) + (size_t)blk0 * 8;
        const uint32_t chunk = lane & 7u;                     // (the same in every step: 64 is a multiple of 8)
        const bool wanted = chunk >= (uint32_t)(sd->Ss >> 3) && chunk <= (uint32_t)(sd->Se >> 3);
#pragma unroll
        for (uint32_t j = 0; j < 8; j++) {
            const uint32_t e = j * 64 + lane;                 // chunk e & 7 of block blk0 + (e >> 3)
            uint32_t bits = 0;
            if (wanted && blk0 + (e >> 3) < plane) {
                const uint4 v = src[e];
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (uint32_t q = 0; q < 4; q++) bits |= ((w[q] & 0xFFFFu) ? 1u : 0u) << (2 * q) | ((w[q] >> 16) ? 2u : 0u) << (2 * q);
            }
            bytes[wave][e] = (uint8_t)bits;
        }
    }
    __syncthreads();
    if (blk >= plane) return;
    if (!from_records) m = *reinterpret_cast<const uint64_t*>(&bytes[wave][lane * 8]);
    for (uint32_t q = 0; q < sd->nhist && q < (uint32_t)kMaxHist; q++)
        m |= R.masks[R.mask_off[(size_t)a.img * R.G + sd->hist[q]] + (size_t)kRefNz * plane + blk];
    R.masks[R.mask_off[ig] + (size_t)kRefHist * plane + blk] = m & band_mask(sd->Ss, sd->Se);
}
// grid: one workgroup per tile (chunks of the blocks the image covers)
__global__ void __launch_bounds__(256) k_refine_deal(DevRecord R, const RefineScan* __restrict__ rs, const RefineTile* __restrict__ tiles) {
    short_kernel_priority();
    const RefineTile tile = tiles[blockIdx.x];
    const RefineScan a = rs[tile.entry];
    size_t ig; uint32_t blk, plane;
    if (!refine_block_of_lane(R, a, tile.chunk, &ig, &blk, &plane)) return;
    uint64_t* rec = R.masks + R.mask_off[ig] + blk;
    rec[(size_t)kRefPlus * plane] = deal_bits(rec[(size_t)kRefPlus * plane], rec[(size_t)kRefHist * plane]);
}

__global__ void __launch_bounds__(256) k_refine_blocks(DevRecord R, const RefineScan* __restrict__ rs, const RefineTile* __restrict__ tiles) {
    __shared__ AcTab tab;
    short_kernel_priority();
    const RefineTile tile = tiles[blockIdx.x];
    const RefineScan a = rs[tile.entry];
    if (R.status[a.img] != kOk) return;
    const ImgDesc* img = &R.img[a.img];
    const size_t ig = (size_t)a.img * R.G + a.scan;
    const ScanDesc* sd = &R.scan[ig];
    const int c = sd->comp[0];
    const uint32_t cw = img->cw[c], ncov = cw * img->ch[c];
    if (tile.chunk * 256 >= ncov) return;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&R.tabs[R.tab_idx[ig]]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&tab);
        for (uint32_t e = threadIdx.x; e < sizeof(AcTab) / 4; e += 256) dst[e] = src[e];
    }
    __syncthreads();
    const uint32_t b = tile.chunk * 256 + threadIdx.x;
    if (b >= ncov) return;
    const uint32_t bw = img->bw[c];
    const size_t blk = (size_t)(b / cw) * bw + (b % cw);
    const size_t plane = (size_t)bw * img->bh[c];
    uint64_t* mk = R.masks + R.mask_off[ig];
    uint64_t* rec = mk + blk;                                // (word w of the block: rec[w * plane])
    const uint64_t h = rec[kRefHist * plane];                // the history phase 1 worked on
    const uint32_t ivl = sd->ri ? b / sd->ri : 0;
    const uint32_t* words = reinterpret_cast<const uint32_t*>(R.clean + clean_base(sd->data_off));
    uint64_t sgn, plus;
    refine_block(words, R.ivl_start[R.slot_base[ig] + ivl], rec[kRefStart * plane], &tab, h, rec[kRefNz * plane], sd->Ss, sd->Se, &sgn, &plus);
    rec[kRefSign * plane] = sgn; rec[kRefPlus * plane] = plus;
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
    if (S.ns > 1) { m = (row >> (vs - 1)) * S.mcu_w + (col >> (hs - 1)); within = S.before + (row & (vs - 1)) * hs + (col & (hs - 1)); }   // (sampling factors are 1 or 2)
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
                const uint64_t* rec = R.masks + S.mask_off + b;
                v = refine_apply(v, k, rec[kRefNz * nblk], rec[kRefSign * nblk], rec[kRefPlus * nblk], S.Al);
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

// Where output sample (oy, ox) of a resize looks: the two source rows and columns (absolute, the box's edge samples
// repeated) and the weights of the second row / column, as exact fractions of 2 * out size.
struct TailTaps { int ya, yb, xa, xb; float fy, fx; };
PCR_D void tail_rows(const CropBox& b, int oy, int out_h, int* ya, int* yb, float* fy) {
    const int dy = 2 * out_h;
    const float inv_dy = 1.0f / (float)dy;
    int yl, ry;
    floor_div((2 * oy + 1) * b.h - out_h, dy, inv_dy, &yl, &ry);
    *fy = (float)ry * inv_dy;
    *ya = b.y0 + min(max(yl, 0), b.h - 1); *yb = b.y0 + min(max(yl + 1, 0), b.h - 1);
}
PCR_D void tail_cols(const CropBox& b, int ox, int out_w, int* xa, int* xb, float* fx) {
    const int oxs = b.flip ? out_w - 1 - ox : ox;
    const int dx = 2 * out_w;
    const float inv_dx = 1.0f / (float)dx;
    int xl, rx;
    floor_div((2 * oxs + 1) * b.w - out_w, dx, inv_dx, &xl, &rx);
    *fx = (float)rx * inv_dx;
    *xa = b.x0 + min(max(xl, 0), b.w - 1); *xb = b.x0 + min(max(xl + 1, 0), b.w - 1);
}
// A box as the tail uses it: clamped into its W x H image.
PCR_D CropBox clamp_box(CropBox b, int W, int H) {
    b.x0 = min(max(b.x0, 0), W - 1); b.y0 = min(max(b.y0, 0), H - 1);
    b.w = min(max(b.w, 1), W - b.x0); b.h = min(max(b.h, 1), H - b.y0);
    return b;
}
// One channel of one output sample from its four source values (whole numbers 0..255), normalised, as half precision.
// The operations are spelled out one by one (no contraction left to the compiler), so that every kernel that
// interpolates gives the very same bits.
PCR_D __half tail_value(float aa, float ab, float ba, float bb, float fx, float fy, float mean, float istd) {
    const float gx = __fsub_rn(1.0f, fx), gy = __fsub_rn(1.0f, fy);
    const float top = __fmaf_rn(fx, ab, __fmul_rn(gx, aa));
    const float bot = __fmaf_rn(fx, bb, __fmul_rn(gx, ba));
    const float v = __fmaf_rn(fy, bot, __fmul_rn(gy, top));
    return __float2half_rn(__fmul_rn(__fsub_rn(__fmul_rn(v, 1.0f / 255.0f), mean), istd));
}

__global__ void __launch_bounds__(256) k_crop_resize(const uint32_t* __restrict__ dims, const uint64_t* __restrict__ out_off,
        const uint8_t* __restrict__ in, const CropBox* __restrict__ boxes,
        int out_h, int out_w, int C, float m0, float m1, float m2, float s0, float s1, float s2, __half* __restrict__ out) {
    const uint32_t i = blockIdx.z;
    const int ox = (int)(blockIdx.x * 32 + (threadIdx.x & 31)), oy = (int)(blockIdx.y * 8 + (threadIdx.x >> 5));
    if (ox >= out_w || oy >= out_h) return;
    const int W = (int)dims[2 * i], H = (int)dims[2 * i + 1];
    if (W < 1 || H < 1) return;
    const CropBox b = clamp_box(boxes[i], W, H);
    // source point relative to the box, as an exact fraction: ((2 o + 1) * size - out) / (2 * out) pixels
    int ya, yb, xa, xb; float fy, fx;
    tail_rows(b, oy, out_h, &ya, &yb, &fy);
    tail_cols(b, ox, out_w, &xa, &xb, &fx);
    const uint8_t* img = in + out_off[i];
    const uint8_t* paa = img + ((size_t)ya * W + xa) * C; const uint8_t* pab = img + ((size_t)ya * W + xb) * C;
    const uint8_t* pba = img + ((size_t)yb * W + xa) * C; const uint8_t* pbb = img + ((size_t)yb * W + xb) * C;
    const float mean[3] = {m0, m1, m2}, istd[3] = {s0, s1, s2};
    __half* dst = out + ((size_t)i * C * out_h + oy) * out_w + ox;
#pragma unroll
    for (int c = 0; c < 3; c++) {
        if (c < C) dst[(size_t)c * out_h * out_w] = tail_value((float)paa[c], (float)pab[c], (float)pba[c], (float)pbb[c], fx, fy, mean[c], istd[c]);
    }
}

// --------------------------------------------------------------------------------------
// k_pixel: one workgroup per run of consecutive MCUs of one image (raster order over its MCU grid, across the
// ends of MCU rows), ONE LANE PER 8x8 BLOCK.
//   phase A  the lane loads its block's 64 coefficients (eight 16-byte loads; chunks that no scan <= k can have
//            touched are not read), replays the component's refinement scans on them, de-quantises, and runs the
//            whole 8x8 inverse DCT in registers: zig-zag order becomes register naming, the row and the column
//            pass need no exchange between lanes, no LDS and no barrier.  The constant factors of the transform
//            (1/2 per pass, cos(pi/4) on terms 0 and 4) are folded into the de-quantisation table.  The clamped
//            samples stay in the lane's registers.
//   phase B  twice, for the upper and for the lower half of the pixel rows of the MCUs: the lanes put the part of
//            their block that lies in the half into LDS, MCU by MCU (per MCU the rows of each component as one small
//            row-major plane; a component that only has its DC writes one sample per block: the block is flat);
//            then chroma replication + colour + one rounding + store: one lane per group of 12 output bytes (4 RGB
//            pixels; 8 gray ones) of one pixel row of one MCU, lanes ordered along the image rows, the samples
//            read from LDS as 16- and 8-byte vectors, the group written with one (possibly unaligned) store.
// The kernel is bound by memory latency times occupancy, not by arithmetic.  Occupancy is bounded by LDS, which is
// why the samples go through it in halves (128 bytes per lane at a time: four wavefronts per SIMD instead of two,
// measured a third faster); and the chain of dependent trips to memory is kept short: the image's descriptor is read
// with scalar loads (no copy through LDS, no barrier), and the coefficient loads are issued before the tables of the
// prologue are built.  (A decode without any AC scan goes
// through k_pixel_flat instead.)
// The refinement is applied here, on the way in: the coefficient planes hold what the first scans wrote, and the
// lane replays the component's refinement scans from the records the refinement kernels left (exactly what k_apply
// does for the coefficient export, the only caller that needs the refined values in memory).  lists / list_idx:
// the per-(image, component) scan lists of k_apply_prep and their index by image * 3 + component (-1: nothing to
// refine); both null if no scan <= k refines.  kRefine = false compiles the replay out.
// boxes (optional): one box per image; runs of MCUs that do not touch their image's box are skipped altogether
// (their pixels are left as they are): for callers that go on to read only the boxes (pcr_decode_crop_batch).
// --------------------------------------------------------------------------------------
constexpr int kPixLanes = 128;             // blocks per workgroup (the samples of half a run take kPixLanes * 128 bytes of LDS)

struct PixelTile { uint32_t img; uint32_t mcu0; };          // first MCU of the run
typedef short short8 __attribute__((ext_vector_type(8)));

// w / d as (w * recip16(d)) >> 16, exact while w * d < 65536
PCR_HD uint32_t recip16(uint32_t d) { return d ? 65536u / d + 1u : 0u; }

PCR_HD uint32_t blocks_per_mcu(const ImgDesc& d) {
    uint32_t b = 0;
    for (int c = 0; c < d.nc; c++) b += (uint32_t)d.hs[c] * d.vs[c];
    return b;
}
PCR_HD uint32_t pixel_mcus_per_tile(const ImgDesc& d) { return (uint32_t)kPixLanes / blocks_per_mcu(d); }   // >= 10: an MCU has at most 12 blocks

// 8-point inverse transform with the constant factors taken out: in[u] must already carry the 1/2 of the pass and,
// for u = 0 and 4, cos(pi/4).  out[x] = sum_u in'[u] cos((2x+1) u pi / 16).
PCR_D void idct8_scaled(float& x0, float& x1, float& x2, float& x3, float& x4, float& x5, float& x6, float& x7) {
    const float c1 = 0.98078528040323044913f, c2 = 0.92387953251128675613f, c3 = 0.83146961230254523708f,
                c5 = 0.55557023301960222474f, c6 = 0.38268343236508977173f, c7 = 0.19509032201612826785f;
    const float a = x0 + x4, b = x0 - x4;
    const float p = x2 * c2 + x6 * c6, q = x2 * c6 - x6 * c2;
    const float e0 = a + p, e1 = b + q, e2 = b - q, e3 = a - p;
    const float o0 = x1 * c1 + x3 * c3 + x5 * c5 + x7 * c7;
    const float o1 = x1 * c3 - x3 * c7 - x5 * c1 - x7 * c5;
    const float o2 = x1 * c5 - x3 * c1 + x5 * c7 + x7 * c3;
    const float o3 = x1 * c7 - x3 * c5 + x5 * c3 - x7 * c1;
    x0 = e0 + o0; x7 = e0 - o0; x1 = e1 + o1; x6 = e1 - o1;
    x2 = e2 + o2; x5 = e2 - o2; x3 = e3 + o3; x4 = e3 - o3;
}
// the factor folded into the quantiser step of zig-zag position k: 1/2 per pass, cos(pi/4) for row or column 0 and 4
PCR_D float idct_fold(uint32_t k) {
    const uint32_t p = zigzag_lookup(k), u = p & 7, v = p >> 3;
    const float c4 = 0.70710678118654752440f;
    const bool a = (u & 3) == 0, b = (v & 3) == 0;
    return a && b ? 0.125f : (a || b ? 0.25f * c4 : 0.25f);            // (cos(pi/4) squared is exactly 1/2: a block with only its DC is exactly DC x step / 8)
}

// byte `which` of `word` := v rounded half up and clamped to [0, 255] (v is finite); the other bytes are kept.
// (The conversion instruction saturates and is exact on integers, which floor(v + 1/2) is.)
PCR_D uint32_t put_u8(float v, uint32_t which, uint32_t word) {
    return __builtin_amdgcn_cvt_pk_u8_f32(__builtin_floorf(v + 0.5f), which, word);
}

// a value per component, picked by a per-lane component number out of three wave-uniform ones
PCR_D uint32_t pick3(uint32_t c, uint32_t a0, uint32_t a1, uint32_t a2) { return c == 0 ? a0 : (c == 1 ? a1 : a2); }

// What the pixel kernels need to know about an image, all wave-uniform (read through a wave-uniform pointer, so
// with scalar loads): sampling, blocks per MCU, where a component's samples start inside an MCU's part of the
// sample tile (rb) and their row length there (rs), first block of its plane in the image's coefficient buffer.
struct PixGeom {
    uint32_t nc, W, H, hmax, vmax, mcux, mcuy, bpm;
    uint32_t hs[kMaxComp], vs[kMaxComp], nbl[kMaxComp], rb[kMaxComp], rs[kMaxComp], plane0[kMaxComp], npl[kMaxComp], bw[kMaxComp], zmx[kMaxComp], cw[kMaxComp], ch[kMaxComp];
    bool flat[kMaxComp];
};
PCR_D void pix_geom(const ImgDesc* ip, PixGeom* g) {
    g->nc = ip->nc; g->W = ip->W; g->H = ip->H; g->hmax = ip->hmax; g->vmax = ip->vmax; g->mcux = ip->mcux; g->mcuy = ip->mcuy;
    uint32_t bpm = 0, p0 = 0;
#pragma unroll
    for (uint32_t c = 0; c < kMaxComp; c++) {
        const bool on = c < g->nc;
        g->hs[c] = on ? ip->hs[c] : 0; g->vs[c] = on ? ip->vs[c] : 0;
        g->nbl[c] = g->hs[c] * g->vs[c]; g->rb[c] = bpm * 64; g->rs[c] = g->hs[c] * 8; bpm += g->nbl[c];
        g->bw[c] = on ? ip->bw[c] : 0;
        g->npl[c] = on ? g->bw[c] * (uint32_t)ip->bh[c] : 0;         // blocks of the component's plane
        g->plane0[c] = p0; p0 += g->npl[c];
        g->zmx[c] = on ? ip->zmax[c] : 0; g->cw[c] = on ? ip->cw[c] : 0; g->ch[c] = on ? ip->ch[c] : 0;
        g->flat[c] = on && g->zmx[c] <= 1;
    }
    g->bpm = bpm;
}

// The lane's block: component c, block (brow, bcol) of the component's plane.
struct PixBlock { uint32_t c, hs, vs, brow, bcol, b, zm, nblk; const int16_t* coef; const int16_t* dc; bool covered; };   // nblk: blocks of the component's plane;   // dc: the block's entry of the compact DC copy
// j: number of the block inside its MCU (components one after the other, each vs rows of hs blocks); (my, mx): the MCU
PCR_D void pix_block(const DevRecord& R, const PixGeom& G, uint32_t img, uint32_t j, uint32_t my, uint32_t mx, PixBlock* B, uint32_t* by_out, uint32_t* bx_out) {
    const uint32_t c = j < G.nbl[0] ? 0u : (j < G.nbl[0] + G.nbl[1] ? 1u : 2u);
    const uint32_t jj = j - pick3(c, 0u, G.nbl[0], G.nbl[0] + G.nbl[1]);
    B->c = c; B->hs = pick3(c, G.hs[0], G.hs[1], G.hs[2]); B->vs = pick3(c, G.vs[0], G.vs[1], G.vs[2]);
    const uint32_t bx = jj & (B->hs - 1), by = jj >> (B->hs - 1);                  // (sampling factors are 1 or 2)
    B->brow = my * B->vs + by; B->bcol = mx * B->hs + bx;
    B->b = B->brow * pick3(c, G.bw[0], G.bw[1], G.bw[2]) + B->bcol;
    B->zm = pick3(c, G.zmx[0], G.zmx[1], G.zmx[2]);
    B->nblk = pick3(c, G.npl[0], G.npl[1], G.npl[2]);
    B->coef = R.coef + R.coef_off[img] + ((size_t)pick3(c, G.plane0[0], G.plane0[1], G.plane0[2]) + B->b) * 64;
    B->dc = R.dc + (R.coef_off[img] >> 6) + pick3(c, G.plane0[0], G.plane0[1], G.plane0[2]) + B->b;
    B->covered = B->brow < pick3(c, G.ch[0], G.ch[1], G.ch[2]) && B->bcol < pick3(c, G.cw[0], G.cw[1], G.cw[2]);
    *by_out = by; *bx_out = bx;
}
// the block's coefficients as they lie in memory (zig-zag order), chunks beyond zm left zero; the DC coefficient comes
// from the compact copy (the planes hold it only for the coefficient export)
PCR_D void pix_load(const PixBlock& B, short8 v[8]) {
    const int16_t dc = *B.dc;
#pragma unroll
    for (int ch = 0; ch < 8; ch++) {
        v[ch] = short8{0, 0, 0, 0, 0, 0, 0, 0};
        if ((uint32_t)ch * 8 < B.zm) v[ch] = *reinterpret_cast<const short8*>(B.coef + ch * 8);
    }
    v[0][0] = dc;
}
// DC of the block after the component's DC refinement scans
template <bool kRefine>
PCR_D int pix_dc(const DevRecord& R, const PixBlock& B, int dcv, const ApplyList* rlc) {
    const uint32_t nref = kRefine ? rlc->n : 0;
    for (uint32_t e = 0; e < nref; e++)
        if (rlc->sc[e].Ss == 0 && dc_refinement_bit(R, rlc->sc[e], B.brow, B.bcol, B.hs, B.vs, B.covered)) dcv |= 1 << rlc->sc[e].Al;
    return dcv;
}
// Refinement replay, de-quantisation and the 8x8 inverse transform of the lane's block; the clamped samples are left in
// F[8 y + x].  qc: the component's folded quantiser steps (zig-zag order); rlc: its refinement scan list.
template <bool kRefine>
PCR_D void pix_samples(const DevRecord& R, const PixBlock& B, const short8 v[8], const float* qc, const ApplyList* rlc, float F[64]) {
    int ci[64];
#pragma unroll
    for (int ch = 0; ch < 8; ch++) {
#pragma unroll
        for (int q = 0; q < 8; q++) ci[ch * 8 + q] = v[ch][q];
    }
    const uint32_t nref = kRefine ? rlc->n : 0;
    for (uint32_t e = 0; e < nref; e++) {
        const ApplyScan& S = rlc->sc[e];
        if (S.Ss == 0) {
            if (dc_refinement_bit(R, S, B.brow, B.bcol, B.hs, B.vs, B.covered)) ci[0] |= 1 << S.Al;
        } else if (B.covered) {
            // the three words of the block's record: positions that become non-zero, their signs, positions
            // whose magnitude grows (all inside the scan's band)
            const uint64_t* rec = R.masks + S.mask_off + B.b;
            const uint64_t nzm = rec[kRefNz * (size_t)B.nblk], sgm = rec[kRefSign * (size_t)B.nblk], plm = rec[kRefPlus * (size_t)B.nblk];
            // A position either grows (it was non-zero: + 2^Al with its own sign) or is new (it was zero: +- 2^Al by the
            // sign bit) or stays: one step with one sign, taken from the coefficient or from the record.
            const uint64_t anym = nzm | plm, negm = nzm & ~sgm;
            const int p1 = 1 << S.Al, above = -2 * p1;       // (above: the bits over bit Al)
#pragma unroll
            for (int k = 1; k < 64; k++) {
                const uint32_t anw = k < 32 ? (uint32_t)anym : (uint32_t)(anym >> 32), ngw = k < 32 ? (uint32_t)negm : (uint32_t)(negm >> 32);
                const int bit = k & 31;
                const int neg = (ci[k] | (int)(ngw << (31 - bit))) >> 31;   // all ones where the step is negative
                const int step = (neg & above) | p1;                        // -2^Al or 2^Al
                // ... taken where the coefficient changes: bit x step + coefficient in one instruction (written out: the
                // compiler turns a product with a single bit into a mask, an `and` and an addition)
                asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(ci[k]) : "v"((anw >> bit) & 1u), "v"(step), "v"(ci[k]));
            }
        }
    }
#pragma unroll
    for (int k4 = 0; k4 < 16; k4++) {                        // natural order: F[8 v + u]
        const float4 qq = *reinterpret_cast<const float4*>(qc + 4 * k4);
        F[zigzag_lookup(4 * k4)] = (float)ci[4 * k4] * qq.x; F[zigzag_lookup(4 * k4 + 1)] = (float)ci[4 * k4 + 1] * qq.y;
        F[zigzag_lookup(4 * k4 + 2)] = (float)ci[4 * k4 + 2] * qq.z; F[zigzag_lookup(4 * k4 + 3)] = (float)ci[4 * k4 + 3] * qq.w;
    }
    // the level shift: the DC term reaches every sample with weight one (its folded factor is exactly 1/8 and the
    // transforms only add it), so 128 is added to it once instead of to the 64 samples
    F[0] += 128.f;
#pragma unroll
    for (int r = 0; r < 8; r++)
        idct8_scaled(F[8 * r], F[8 * r + 1], F[8 * r + 2], F[8 * r + 3], F[8 * r + 4], F[8 * r + 5], F[8 * r + 6], F[8 * r + 7]);
#pragma unroll
    for (int x = 0; x < 8; x++)
        idct8_scaled(F[x], F[8 + x], F[16 + x], F[24 + x], F[32 + x], F[40 + x], F[48 + x], F[56 + x]);
#pragma unroll
    for (int e = 0; e < 64; e++) F[e] = clamp255(F[e]);
}
// rows y0 .. y0 + kRows - 1 of the block's samples to dst[(y - y0) * row_len + x]
template <int y0, int kRows>
PCR_D void pix_put_rows(const float F[64], float* dst, uint32_t row_len) {
#pragma unroll
    for (int y = 0; y < kRows; y++) {
        *reinterpret_cast<float4*>(dst + y * row_len) = float4{F[8 * (y0 + y)], F[8 * (y0 + y) + 1], F[8 * (y0 + y) + 2], F[8 * (y0 + y) + 3]};
        *reinterpret_cast<float4*>(dst + y * row_len + 4) = float4{F[8 * (y0 + y) + 4], F[8 * (y0 + y) + 5], F[8 * (y0 + y) + 6], F[8 * (y0 + y) + 7]};
    }
}
// the same, with the whole block stored to dst[y * row_len + x]
template <bool kRefine>
PCR_D void pix_finish(const DevRecord& R, const PixBlock& B, const short8 v[8], const float* qc, const ApplyList* rlc, float* dst, uint32_t row_len) {
    float F[64];
    pix_samples<kRefine>(R, B, v, qc, rlc, F);
    pix_put_rows<0, 8>(F, dst, row_len);
}
// Half kHalf (0: upper, 1: lower) of the pixel rows of an MCU: the part of the lane's block that lies in it, to the
// component's rows of the half (sampling factors are 1 or 2: a block of a component with two block rows per MCU lies
// in one half whole, any other block has four sample rows in each).  dst: the block's first sample row in the half.
// A flat block (flat: only its DC) is one sample.
template <int kHalf>
PCR_D void pix_put_half(const float F[64], bool flat, uint32_t vs, uint32_t by, float* dst, uint32_t row_len) {
    if (vs == 2) {
        if (by != (uint32_t)kHalf) return;
        if (flat) dst[0] = F[0]; else pix_put_rows<0, 8>(F, dst, row_len);
    } else {
        if (flat) dst[0] = F[0]; else pix_put_rows<4 * kHalf, 4>(F, dst, row_len);
    }
}
// the component's folded quantiser steps into LDS; every lane of the workgroup calls it
PCR_D void pix_quant_table(const DevRecord& R, const ImgDesc* ip, uint32_t nc, float (*qz)[68], uint32_t tid, uint32_t nthreads) {
    for (uint32_t e = tid; e < nc * 64; e += nthreads) {
        const uint32_t c = e >> 6, k = e & 63;
        const uint32_t tq = ip->tq[c];
        const uint8_t* q = R.rec + ip->qoff[tq];
        qz[c][k] = (ip->qprec[tq] ? (float)ld_be16(q + 2 * k) : (float)q[k]) * idct_fold(k);
    }
}
// the refinement scan lists of the image's components into LDS
PCR_D void pix_lists(const ApplyList* __restrict__ lists, const int32_t* __restrict__ list_idx, uint32_t img, uint32_t nc, ApplyList* rl, uint32_t tid, uint32_t nthreads) {
    for (uint32_t c = 0; c < nc; c++) {
        const int32_t li = list_idx ? list_idx[img * kMaxComp + c] : -1;
        uint32_t* dst = reinterpret_cast<uint32_t*>(&rl[c]);
        if (li >= 0) {
            const uint32_t* src = reinterpret_cast<const uint32_t*>(&lists[li]);
            for (uint32_t e = tid; e < sizeof(ApplyList) / 4; e += nthreads) dst[e] = src[e];
        } else if (tid == 0) dst[0] = 0;                    // n = 0
    }
}

// four consecutive samples of a component for the output pixels x0 .. x0+3 of a pixel row (x0 a multiple of 4):
// row: the component's row of the MCU; sh: 1 if the component has half the horizontal resolution
PCR_D void four_samples(const float* row, uint32_t x0, uint32_t sh, float v[4]) {
    if (sh == 0) { const float4 t = *reinterpret_cast<const float4*>(row + x0); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
    else { const float2 t = *reinterpret_cast<const float2*>(row + (x0 >> 1)); v[0] = v[1] = t.x; v[2] = v[3] = t.y; }
}

// The first n (< 12) bytes of w0 w1 w2 to p with at most three stores (a row's last, narrower group: a loop over
// the bytes would cost every wavefront that holds a row end its full length)
PCR_D void store_head(uint8_t* p, uint32_t w0, uint32_t w1, uint32_t w2, uint32_t n) {
    struct __attribute__((packed, aligned(1))) U32 { uint32_t v; };
    struct __attribute__((packed, aligned(1))) U16 { uint16_t v; };
    const uint32_t words[3] = {w0, w1, w2};
    uint32_t done = 0;
    if (n >= 8) { reinterpret_cast<U32*>(p)->v = w0; reinterpret_cast<U32*>(p + 4)->v = w1; done = 8; }
    else if (n >= 4) { reinterpret_cast<U32*>(p)->v = w0; done = 4; }
    const uint32_t w = done == 8 ? words[2] : (done == 4 ? words[1] : words[0]);       // the word the rest comes from
    if (n - done >= 2) { reinterpret_cast<U16*>(p + done)->v = (uint16_t)w; if (n - done == 3) p[done + 2] = (uint8_t)(w >> 16); }
    else if (n - done == 1) p[done] = (uint8_t)w;
}

template <bool kRefine, bool kPlanes>
__global__ void __launch_bounds__(kPixLanes) k_pixel(DevRecord R, const PixelTile* __restrict__ tiles, uint8_t* __restrict__ out,
                                                     const ApplyList* __restrict__ lists, const int32_t* __restrict__ list_idx,
                                                     const CropBox* __restrict__ boxes) {
    // samples of half the pixel rows of the run: 32 per block
    __shared__ __attribute__((aligned(16))) float tile[kPixLanes * 32];
    // quantiser steps in zig-zag order times the folded transform factors; the rows of the three components start
    // four banks apart, so that lanes of different components read them without bank conflicts
    __shared__ __attribute__((aligned(16))) float qz[kMaxComp][68];
    __shared__ ApplyList rl[kRefine ? kMaxComp : 1];       // refinement scan lists of the components (n = 0: none)
    __shared__ uint32_t org[kPixLanes];                    // per MCU of the run: its first pixel, counted in pixels from the image's first (< 2^32)
    __shared__ uint16_t visw[kPixLanes], vish[kPixLanes];  // ... and how many of its pixel columns / rows lie inside the image
    short_kernel_priority();
    const uint32_t item = xcd_major(blockIdx.x, gridDim.x);
    const uint32_t timg = uni(tiles[item].img), mcu0 = uni(tiles[item].mcu0);
    const uint32_t tid = threadIdx.x;
    const ImgDesc* ip = R.img + timg;
    PixGeom G;
    pix_geom(ip, &G);
    const uint32_t nc = G.nc, W = G.W, H = G.H, mcux = G.mcux, bpm = G.bpm;
    const uint32_t mcu_px_w = 8 * G.hmax, mcu_px_h = 8 * G.vmax;
    if (bpm == 0 || bpm > 12) return;                       // (cannot happen for an image the parser accepted)
    const uint32_t per = (uint32_t)kPixLanes / bpm;
    const uint32_t total = mcux * G.mcuy;
    if (mcu0 >= total) return;
    const uint32_t nm = total - mcu0 < per ? total - mcu0 : per;      // MCUs of this run
    if (boxes) {                                            // (clamped into the image exactly as k_crop_resize clamps it)
        CropBox b = boxes[timg];
        b.x0 = min(max(b.x0, 0), (int)W - 1); b.y0 = min(max(b.y0, 0), (int)H - 1);
        b.w = min(max(b.w, 1), (int)W - b.x0); b.h = min(max(b.h, 1), (int)H - b.y0);
        const uint32_t r0 = mcu0 / mcux, r1 = (mcu0 + nm - 1) / mcux;          // MCU rows the run touches
        if ((int)(r0 * mcu_px_h) >= b.y0 + b.h || (int)((r1 + 1) * mcu_px_h) <= b.y0) return;
        if (r0 == r1) {
            const uint32_t c0 = mcu0 - r0 * mcux;
            if ((int)(c0 * mcu_px_w) >= b.x0 + b.w || (int)((c0 + nm) * mcu_px_w) <= b.x0) return;
        }
    }
    const bool dead = uni((uint32_t)(R.status[timg] != kOk)) != 0;
    // ---- phase A, first half: the lane's block and its loads ----
    const uint32_t m = (tid * recip16(bpm)) >> 16, j = tid - m * bpm;
    const bool mine = !dead && m < nm;
    PixBlock B;
    uint32_t by = 0, bx = 0;
    short8 v[8];
    if (mine) {
        const uint32_t M = mcu0 + m, my = M / mcux, mx = M - my * mcux;
        pix_block(R, G, timg, j, my, mx, &B, &by, &bx);
        if (B.zm <= 1) {
            v[0] = short8{0, 0, 0, 0, 0, 0, 0, 0};
            v[0][0] = *B.dc;
        } else pix_load(B, v);
    }
    // ---- prologue tables (the loads above are under way meanwhile) ----
    if (kRefine) pix_lists(lists, list_idx, timg, nc, rl, tid, kPixLanes);
    pix_quant_table(R, ip, nc, qz, tid, kPixLanes);
    if (tid < nm) {
        const uint32_t M = mcu0 + tid, my = M / mcux, mx = M - my * mcux;
        org[tid] = my * mcu_px_h * W + mx * mcu_px_w;
        const uint32_t x = mx * mcu_px_w, y = my * mcu_px_h;
        visw[tid] = (uint16_t)(x >= W ? 0 : (W - x < mcu_px_w ? W - x : mcu_px_w));
        vish[tid] = (uint16_t)(y >= H ? 0 : (H - y < mcu_px_h ? H - y : mcu_px_h));
    }
    __syncthreads();
    // ---- phase A, second half: the block's samples, in registers ----
    float S[64];
    const bool flatb = mine && B.zm <= 1;                   // flat: one sample stands for the block
    if (mine) {
        const ApplyList* rlc = &rl[kRefine ? B.c : 0];
        if (flatb) S[0] = clamp255((float)pix_dc<kRefine>(R, B, v[0][0], rlc) * qz[B.c][0] + 128.f);
        else pix_samples<kRefine>(R, B, v, qz[B.c], rlc, S);
    }
    if (kPlanes) {
        // Instead of pixels: the lane's block, rounded, into the component's own plane of bytes (`out`: one byte per
        // coefficient slot, so a component's plane lies where its coefficient plane lies, [rows of samples][bw * 8]),
        // for k_triangle_rgb.  A damaged image's planes are left alone; that kernel writes its pixels as zeros.
        if (mine) {
            const uint32_t pw = pick3(B.c, G.bw[0], G.bw[1], G.bw[2]) * 8;
            uint8_t* pd = out + R.coef_off[timg] + (size_t)pick3(B.c, G.plane0[0], G.plane0[1], G.plane0[2]) * 64 + (size_t)(B.brow * 8) * pw + B.bcol * 8;
#pragma unroll
            for (int y = 0; y < 8; y++) {
                uint2 w;
                if (flatb) {
                    w.x = put_u8(S[0], 0, 0); w.x = put_u8(S[0], 1, w.x); w.x = put_u8(S[0], 2, w.x); w.x = put_u8(S[0], 3, w.x);
                    w.y = w.x;
                } else {
                    w.x = put_u8(S[8 * y], 0, 0); w.x = put_u8(S[8 * y + 1], 1, w.x); w.x = put_u8(S[8 * y + 2], 2, w.x); w.x = put_u8(S[8 * y + 3], 3, w.x);
                    w.y = put_u8(S[8 * y + 4], 0, 0); w.y = put_u8(S[8 * y + 5], 1, w.y); w.y = put_u8(S[8 * y + 6], 2, w.y); w.y = put_u8(S[8 * y + 7], 3, w.y);
                }
                *reinterpret_cast<uint2*>(pd + (size_t)y * pw) = w;
            }
        }
        return;
    }
    // ---- phase B: one lane per group of output bytes of one pixel row of one MCU, the upper half of the pixel rows of
    // the MCUs first, then the lower: the samples of half a run are what the workgroup holds in LDS at a time ----
    const uint32_t shx0 = G.hs[0] == G.hmax ? 0 : 1, shy0 = G.vs[0] == G.vmax ? 0 : 1;       // sampling factors are 1 or 2
    const uint32_t shx1 = nc > 1 && G.hs[1] != G.hmax, shy1 = nc > 1 && G.vs[1] != G.vmax;
    const uint32_t shx2 = nc > 2 && G.hs[2] != G.hmax, shy2 = nc > 2 && G.vs[2] != G.vmax;
    const uint32_t ppg = nc == 1 ? 8u : 4u;                 // pixels per group: 8 gray bytes, or 12 bytes of RGB
    const uint32_t gpm = mcu_px_w / ppg;                    // groups per pixel row of an MCU: 1, 2 or 4
    const uint32_t lg = gpm == 4 ? 2u : (gpm == 2 ? 1u : 0u);
    const uint32_t half_h = mcu_px_h >> 1;                  // pixel rows of an MCU per half: 4 or 8
    const uint32_t items = nm * half_h * gpm;
    const uint32_t rcpn = nm > 1 ? 0xFFFFFFFFu / nm + 1u : 0u;       // q / nm as the high word of q * rcpn: exact while q * nm < 2^32
    const uint32_t mstride = bpm * 32;                      // samples of an MCU in one half
    // component c's four samples for pixels x0.. of row ly (counted inside the half) of MCU mm: a flat component has one per block
    auto fetch = [&](uint32_t c, uint32_t mm, uint32_t ly, uint32_t x0, uint32_t shx, uint32_t shy, float s[4]) {
        if (G.flat[c]) {
            const float f = tile[mm * mstride + (G.rb[c] >> 1) + ((x0 >> shx) >> 3) * 8];      // (a half holds one block row of the component, or half of one)
            s[0] = s[1] = s[2] = s[3] = f;
        } else four_samples(tile + mm * mstride + (G.rb[c] >> 1) + (ly >> shy) * G.rs[c], x0, shx, s);
    };
#pragma unroll
    for (int half = 0; half < 2; half++) {
        if (half) __syncthreads();                          // (the upper half has been read)
        if (mine) {
            float* const dst = tile + m * mstride + (pick3(B.c, G.rb[0], G.rb[1], G.rb[2]) >> 1) + bx * 8;
            if (half == 0) pix_put_half<0>(S, flatb, B.vs, by, dst, B.hs * 8);
            else pix_put_half<1>(S, flatb, B.vs, by, dst, B.hs * 8);
        }
        __syncthreads();
        for (uint32_t it = tid; it < items; it += kPixLanes) {
            // lanes run along the image rows: group, then MCU, then pixel row
            const uint32_t g = it & (gpm - 1), q = it >> lg;
            const uint32_t lyh = nm > 1 ? __umulhi(q, rcpn) : q, mm = q - lyh * nm;
            const uint32_t ly = lyh + half * half_h;        // the pixel row inside the MCU
            const uint32_t x0 = g * ppg, vw = visw[mm];
            if (ly >= vish[mm] || x0 >= vw) continue;
            uint8_t* wp = out + R.out_off[timg] + ((size_t)org[mm] + (size_t)ly * W + x0) * nc;
            const uint32_t left = vw - x0;                  // pixels of the group inside the image
            if (nc == 1) {
                float a[4], bq[4];
                fetch(0, mm, lyh, x0, 0, 0, a); fetch(0, mm, lyh, x0 + 4, 0, 0, bq);
                uint32_t w0 = 0, w1 = 0;
                if (!dead) {
                    w0 = put_u8(a[0], 0, w0); w0 = put_u8(a[1], 1, w0); w0 = put_u8(a[2], 2, w0); w0 = put_u8(a[3], 3, w0);
                    w1 = put_u8(bq[0], 0, w1); w1 = put_u8(bq[1], 1, w1); w1 = put_u8(bq[2], 2, w1); w1 = put_u8(bq[3], 3, w1);
                }
                if (left >= 8) {
                    struct __attribute__((packed, aligned(1))) Eight { uint32_t a, b; };
                    Eight e8; e8.a = w0; e8.b = w1;
                    *reinterpret_cast<Eight*>(wp) = e8;
                } else {
                    store_head(wp, w0, w1, 0u, left);
                }
            } else {
                float ys[4], cb[4], cr[4];
                uint32_t w0 = 0, w1 = 0, w2 = 0;
                if (!dead) {
                    fetch(0, mm, lyh, x0, shx0, shy0, ys); fetch(1, mm, lyh, x0, shx1, shy1, cb); fetch(2, mm, lyh, x0, shx2, shy2, cr);
                    float r[4], gg[4], bb[4];
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const float u = cb[i] - 128.f, w = cr[i] - 128.f;
                        r[i] = ys[i] + 1.402f * w; gg[i] = ys[i] - 0.344136f * u - 0.714136f * w; bb[i] = ys[i] + 1.772f * u;
                    }
                    w0 = put_u8(r[0], 0, w0); w0 = put_u8(gg[0], 1, w0); w0 = put_u8(bb[0], 2, w0); w0 = put_u8(r[1], 3, w0);
                    w1 = put_u8(gg[1], 0, w1); w1 = put_u8(bb[1], 1, w1); w1 = put_u8(r[2], 2, w1); w1 = put_u8(gg[2], 3, w1);
                    w2 = put_u8(bb[2], 0, w2); w2 = put_u8(r[3], 1, w2); w2 = put_u8(gg[3], 2, w2); w2 = put_u8(bb[3], 3, w2);
                }
                if (left >= 4) {
                    struct __attribute__((packed, aligned(1))) Twelve { uint32_t a, b, c; };
                    Twelve tw; tw.a = w0; tw.b = w1; tw.c = w2;
                    *reinterpret_cast<Twelve*>(wp) = tw;           // one (possibly unaligned) 12-byte store
                } else {
                    store_head(wp, w0, w1, w2, left * 3);
                }
            }
        }
    }
}

// --------------------------------------------------------------------------------------
// k_pixel_flat: the pixel stage of a decode that holds DC coefficients only (scan groups ahead of every AC scan):
// every block is flat, so an 8x8 cell of output pixels has ONE colour.  One lane per cell (runs of kFlatLanes cells in
// raster order over the image's grid of cells): it reads the DC of the block of each component that covers its cell
// from the compact DC plane (sampling factors are 1 or 2, so a cell lies inside one block of every component),
// de-quantises, converts the colour once and writes the cell's rows, 24 bytes each (8 gray bytes), with unaligned
// vector stores.  No LDS and no barrier; the work per output byte is a few instructions, which is what bounds a
// kernel whose input is 1/64 of its output.  The arithmetic is k_pixel's, so the pixels are the same.
// --------------------------------------------------------------------------------------
constexpr int kFlatLanes = 256;
PCR_HD uint32_t flat_cells(uint32_t W, uint32_t H) { return ((W + 7) >> 3) * ((H + 7) >> 3); }

// an image's descriptor through a wave-uniform pointer, as dwords
PCR_D void load_desc(const ImgDesc* ip, ImgDesc* D) {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(ip);
    uint32_t* dst = reinterpret_cast<uint32_t*>(D);
#pragma unroll
    for (uint32_t e = 0; e < sizeof(ImgDesc) / 4; e++) dst[e] = src[e];
}
// only DCs decoded for every component?  (the host launches the flat kernels only for such decodes)
PCR_D bool flat_image(const ImgDesc& D) {
    bool ok = D.nc == 1 || D.nc == 3;
    for (uint32_t c = 0; c < kMaxComp; c++) if (c < D.nc && D.zmax[c] > 1) ok = false;
    return ok;
}
// The output bytes of cell (cx, cy): four pixels as three words (w0 w1 w2; a cell row of eight pixels is w0 w1 w2 w0 w1 w2),
// for a gray image four equal bytes in each.  dcp: the image's compact DC plane.
PCR_D void flat_cell_words(const DevRecord& R, const ImgDesc& D, const int16_t* dcp, uint32_t cx, uint32_t cy, bool dead, uint32_t* w0, uint32_t* w1, uint32_t* w2) {
    float s[kMaxComp];
    uint32_t plane0 = 0;
#pragma unroll
    for (uint32_t c = 0; c < kMaxComp; c++) {
        s[c] = 128.f;
        if (c < D.nc) {
            const uint32_t bcol = (cx * D.hs[c]) >> (D.hmax - 1), brow = (cy * D.vs[c]) >> (D.vmax - 1);      // (sampling factors are 1 or 2)
            // (picked with compares: an index computed at run time would put the whole descriptor into scratch memory)
            const uint32_t tq = D.tq[c] & 3;
            const uint32_t qoff = tq == 0 ? D.qoff[0] : (tq == 1 ? D.qoff[1] : (tq == 2 ? D.qoff[2] : D.qoff[3]));
            const uint32_t qprec = tq == 0 ? D.qprec[0] : (tq == 1 ? D.qprec[1] : (tq == 2 ? D.qprec[2] : D.qprec[3]));
            const uint8_t* q = R.rec + qoff;
            const float q0 = (qprec ? (float)ld_be16(q) : (float)q[0]) * 0.125f;
            s[c] = clamp255((float)dcp[plane0 + brow * D.bw[c] + bcol] * q0 + 128.f);
            plane0 += (uint32_t)D.bw[c] * D.bh[c];
        }
    }
    if (D.nc == 1) { uint32_t g = put_u8(s[0], 0, 0); g |= g << 8; g |= g << 16; *w0 = g; *w1 = g; *w2 = g; }
    else {
        const float u = s[1] - 128.f, w = s[2] - 128.f;
        const uint32_t r = put_u8(s[0] + 1.402f * w, 0, 0), gq = put_u8(s[0] - 0.344136f * u - 0.714136f * w, 0, 0), bq = put_u8(s[0] + 1.772f * u, 0, 0);
        *w0 = r | (gq << 8) | (bq << 16) | (r << 24); *w1 = gq | (bq << 8) | (r << 16) | (gq << 24); *w2 = bq | (r << 8) | (gq << 16) | (bq << 24);
    }
    if (dead) { *w0 = 0; *w1 = 0; *w2 = 0; }
}

__global__ void __launch_bounds__(kFlatLanes) k_pixel_flat(DevRecord R, const PixelTile* __restrict__ tiles, uint8_t* __restrict__ out,
                                                           const CropBox* __restrict__ boxes) {
    short_kernel_priority();
    const uint32_t item = xcd_major(blockIdx.x, gridDim.x);
    const uint32_t timg = uni(tiles[item].img), cell0 = uni(tiles[item].mcu0);
    ImgDesc D;
    load_desc(R.img + timg, &D);
    const uint32_t nc = D.nc, W = D.W, H = D.H;
    const uint32_t cells_w = (W + 7) >> 3, total = cells_w * ((H + 7) >> 3);
    const uint32_t cell = cell0 + threadIdx.x;
    if (!flat_image(D)) return;
    if (cell >= total) return;
    // cell / cells_w as the high word of a product: exact while cell * cells_w < 2^32 (and the factor fits: cells_w > 1)
    const uint32_t cy = cells_w == 1 ? cell : ((uint64_t)total * cells_w < (1ull << 32) ? __umulhi(cell, 0xFFFFFFFFu / cells_w + 1u) : cell / cells_w);
    const uint32_t cx = cell - cy * cells_w;
    const uint32_t x = cx * 8, y = cy * 8;
    if (boxes) {                                            // (clamped into the image exactly as k_crop_resize clamps it)
        CropBox b = boxes[timg];
        b.x0 = min(max(b.x0, 0), (int)W - 1); b.y0 = min(max(b.y0, 0), (int)H - 1);
        b.w = min(max(b.w, 1), (int)W - b.x0); b.h = min(max(b.h, 1), (int)H - b.y0);
        if ((int)x >= b.x0 + b.w || (int)x + 8 <= b.x0 || (int)y >= b.y0 + b.h || (int)y + 8 <= b.y0) return;
    }
    const bool dead = uni((uint32_t)(R.status[timg] != kOk)) != 0;
    uint32_t w0, w1, w2;
    flat_cell_words(R, D, R.dc + (R.coef_off[timg] >> 6), cx, cy, dead, &w0, &w1, &w2);
    const uint32_t npx = W - x < 8 ? W - x : 8, nrows = H - y < 8 ? H - y : 8;
    const size_t pitch = (size_t)W * nc;
    uint8_t* wp = out + R.out_off[timg] + (size_t)y * pitch + (size_t)x * nc;
    struct __attribute__((packed, aligned(1))) Words2 { uint32_t a, b; };
    struct __attribute__((packed, aligned(1))) Words4 { uint32_t a, b, c, d; };
    if (npx == 8) {
        if (nc == 1) {
            Words2 e; e.a = w0; e.b = w0;
            for (uint32_t r = 0; r < nrows; r++, wp += pitch) *reinterpret_cast<Words2*>(wp) = e;
        } else {
            Words4 e; e.a = w0; e.b = w1; e.c = w2; e.d = w0;
            Words2 f; f.a = w1; f.b = w2;
            for (uint32_t r = 0; r < nrows; r++, wp += pitch) { *reinterpret_cast<Words4*>(wp) = e; *reinterpret_cast<Words2*>(wp + 16) = f; }
        }
    } else {                                                // the image's last, narrower column of cells
        const uint32_t nb = npx * nc;
        for (uint32_t r = 0; r < nrows; r++, wp += pitch)
            for (uint32_t i = 0; i < nb; i++) wp[i] = (uint8_t)((nc == 1 ? w0 : (i % 12 < 4 ? w0 : (i % 12 < 8 ? w1 : w2))) >> (8 * (i & 3)));
    }
}

// --------------------------------------------------------------------------------------
// k_pixel_flat_rows: the same pixels written as whole aligned 16-byte chunks, for images of at most kFlatRowCells
// cells per row decoded without crop boxes (the usual case; k_pixel_flat serves the rest).  One wavefront per row of
// cells (many short workgroups in flight hide the chain descriptor -> DC -> LDS -> stores better than few wide ones).  The eight pixel rows the cells cover are equal and lie one behind the other in the output, so the band is
// one run of bytes that repeats the pixel row; the lanes first make that row in LDS (one cell each), then write the
// band chunk by chunk -- a chunk is sixteen bytes of the repeated row from the chunk's distance to the band's start
// modulo the row length -- and the few bytes ahead of the first and behind the last whole chunk one by one.
// Measured on this chip, writing a decoded record's pixels this way takes 0.10 ms per 490 MB against 0.14 ms for
// 24-byte pieces at the cells' own addresses.
// --------------------------------------------------------------------------------------
constexpr int kFlatRowCells = 1024, kFlatRowLanes = 64;
PCR_HD bool flat_rows_fit(uint32_t W) { return ((W + 7) >> 3) <= (uint32_t)kFlatRowCells; }
// LDS bytes a launch needs for images of at most `cells` cells per row: 24 bytes per cell, the repeated 32 bytes, slack
PCR_HD uint32_t flat_rows_lds(uint32_t cells) { return cells * 24 + 64; }

__global__ void __launch_bounds__(kFlatRowLanes) k_pixel_flat_rows(DevRecord R, const PixelTile* __restrict__ tiles, uint8_t* __restrict__ out, uint32_t max_cells) {
    // the pixel row: 24 bytes per cell (8 for a gray image), then its first 32 bytes again so that a chunk may run past its end
    extern __shared__ __attribute__((aligned(16))) uint32_t pat[];
    short_kernel_priority();
    const uint32_t item = xcd_major(blockIdx.x, gridDim.x);
    const uint32_t timg = uni(tiles[item].img), cy = uni(tiles[item].mcu0);      // (mcu0: the row of cells)
    ImgDesc D;
    load_desc(R.img + timg, &D);
    const uint32_t nc = D.nc, W = D.W, H = D.H, tid = threadIdx.x;
    const uint32_t cells_w = (W + 7) >> 3;
    if (!flat_image(D) || cells_w > max_cells || cy * 8 >= H) return;      // (wave-uniform: no lane is left behind at a barrier)
    const bool dead = uni((uint32_t)(R.status[timg] != kOk)) != 0;
    const int16_t* dcp = R.dc + (R.coef_off[timg] >> 6);
    for (uint32_t cx = tid; cx < cells_w; cx += kFlatRowLanes) {
        uint32_t w0, w1, w2;
        flat_cell_words(R, D, dcp, cx, cy, dead, &w0, &w1, &w2);
        if (nc == 1) { pat[2 * cx] = w0; pat[2 * cx + 1] = w0; }
        else { uint32_t* d = pat + 6 * cx; d[0] = w0; d[1] = w1; d[2] = w2; d[3] = w0; d[4] = w1; d[5] = w2; }
    }
    __syncthreads();
    const uint32_t pitch = W * nc;                           // bytes of a pixel row (< 2^15 here)
    uint8_t* pb = reinterpret_cast<uint8_t*>(pat);
    uint32_t wrap = 0;
    if (tid < 32) wrap = pb[tid % pitch];
    __syncthreads();                                        // (the last cell may have written past the row's end: read first, then overwrite)
    if (tid < 32) pb[pitch + tid] = (uint8_t)wrap;
    __syncthreads();
    const uint32_t nrows = H - cy * 8 < 8 ? H - cy * 8 : 8;
    const uint32_t len = nrows * pitch;                     // bytes of the band (< 2^18)
    uint8_t* band = out + R.out_off[timg] + (size_t)cy * 8 * pitch;
    const uint32_t head = (uint32_t)((16 - (reinterpret_cast<uintptr_t>(band) & 15)) & 15);   // bytes ahead of the first aligned chunk
    const float inv_pitch = 1.0f / (float)pitch;
    // distance from the band's start -> position in the pixel row (p < 2^24: the quotient in single precision is off by at most one)
    auto in_row = [&](uint32_t p) {
        uint32_t r = (uint32_t)((float)p * inv_pitch);
        int32_t q = (int32_t)(p - r * pitch);
        if (q < 0) q += (int32_t)pitch; else if (q >= (int32_t)pitch) q -= (int32_t)pitch;
        return (uint32_t)q;
    };
    if (head >= len) {                                      // a band shorter than one chunk
        for (uint32_t p = tid; p < len; p += kFlatRowLanes) band[p] = pb[in_row(p)];
        return;
    }
    const uint32_t nchunks = (len - head) >> 4, tail0 = head + (nchunks << 4);
    for (uint32_t j = tid; j < nchunks; j += kFlatRowLanes) {
        const uint32_t p = head + (j << 4), q = in_row(p);
        const uint32_t* s = pat + (q >> 2);
        const uint32_t a = s[0], b = s[1], c = s[2], d = s[3], e = s[4], sh = q & 3;
        uint4 v;
        v.x = __builtin_amdgcn_alignbyte(b, a, sh); v.y = __builtin_amdgcn_alignbyte(c, b, sh);
        v.z = __builtin_amdgcn_alignbyte(d, c, sh); v.w = __builtin_amdgcn_alignbyte(e, d, sh);
        *reinterpret_cast<uint4*>(band + p) = v;
    }
    if (tid < head) band[tid] = pb[tid];                    // (head < 16 <= the repeated part)
    if (tid < len - tail0) band[tail0 + tid] = pb[in_row(tail0 + tid)];
}

// --------------------------------------------------------------------------------------
// k_triangle_rgb: pixels from planes of rounded samples (k_pixel<., true>) with the chroma up-sampling stock decoders
// use instead of replication: every output sample of a component at half resolution is 3/4 of the nearer and 1/4 of the
// farther sample of the component's grid, down the columns first, then along the rows; beyond the component's own
// samples (ceil(W hs / hmax) x ceil(H vs / vmax)) the nearest one stands in.  On integer samples these weights are exact
// in single precision.  One lane per four pixels of a row.  grid: (ceil(items of the largest image / 256), images).
// --------------------------------------------------------------------------------------
PCR_D float triangle_sample(const uint8_t* p, uint32_t pw, uint32_t xc, uint32_t yc, uint32_t fx, uint32_t fy, uint32_t x, uint32_t y) {
    if (fx == 1 && fy == 1) return (float)p[(size_t)y * pw + x];
    const uint32_t xi = fx == 2 ? x >> 1 : x;
    uint32_t xj = fx == 2 ? ((x & 1) ? xi + 1 : (xi ? xi - 1 : 0)) : xi;
    if (xj >= xc) xj = xc - 1;
    const uint32_t yi = fy == 2 ? y >> 1 : y;
    uint32_t yj = fy == 2 ? ((y & 1) ? yi + 1 : (yi ? yi - 1 : 0)) : yi;
    if (yj >= yc) yj = yc - 1;
    const float a0 = (float)p[(size_t)yi * pw + xi], a1 = (float)p[(size_t)yj * pw + xi];
    const float c0 = fy == 2 ? 0.75f * a0 + 0.25f * a1 : a0;
    if (fx != 2) return c0;
    const float b0 = (float)p[(size_t)yi * pw + xj], b1 = (float)p[(size_t)yj * pw + xj];
    const float c1 = fy == 2 ? 0.75f * b0 + 0.25f * b1 : b0;
    return 0.75f * c0 + 0.25f * c1;
}

__global__ void __launch_bounds__(256) k_triangle_rgb(DevRecord R, const uint8_t* __restrict__ planes, uint8_t* __restrict__ out) {
    const uint32_t img = blockIdx.y;
    ImgDesc D;
    load_desc(R.img + img, &D);
    const uint32_t W = D.W, H = D.H, nc = D.nc;
    const uint32_t gw = (W + 3) >> 2;                        // groups of four pixels per row
    const uint32_t item = blockIdx.x * 256 + threadIdx.x;
    if (item >= gw * H || (nc != 1 && nc != 3)) return;
    const uint32_t y = item / gw, x0 = (item - y * gw) * 4;
    const uint32_t npx = W - x0 < 4 ? W - x0 : 4;
    const bool dead = R.status[img] != kOk;
    float s[kMaxComp][4];
    uint32_t plane0 = 0;
#pragma unroll
    for (uint32_t c = 0; c < kMaxComp; c++) {
        if (c < nc && !dead) {
            const uint8_t* p = planes + R.coef_off[img] + (size_t)plane0 * 64;
            const uint32_t pw = (uint32_t)D.bw[c] * 8, fx = D.hmax / D.hs[c], fy = D.vmax / D.vs[c];
            const uint32_t xc = (W * D.hs[c] + D.hmax - 1) / D.hmax, yc = (H * D.vs[c] + D.vmax - 1) / D.vmax;
            for (uint32_t i = 0; i < 4; i++) s[c][i] = i < npx ? triangle_sample(p, pw, xc, yc, fx, fy, x0 + i, y) : 0.f;
        } else for (uint32_t i = 0; i < 4; i++) s[c][i] = 0.f;
        plane0 += c < nc ? (uint32_t)D.bw[c] * D.bh[c] : 0;
    }
    uint8_t* wp = out + R.out_off[img] + ((size_t)y * W + x0) * nc;
    if (nc == 1) {
        for (uint32_t i = 0; i < npx; i++) wp[i] = dead ? 0 : (uint8_t)put_u8(s[0][i], 0, 0);
        return;
    }
    uint32_t w0 = 0, w1 = 0, w2 = 0;
    if (!dead) {
        float r[4], g[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const float u = s[1][i] - 128.f, w = s[2][i] - 128.f;
            r[i] = s[0][i] + 1.402f * w; g[i] = s[0][i] - 0.344136f * u - 0.714136f * w; b[i] = s[0][i] + 1.772f * u;
        }
        w0 = put_u8(r[0], 0, w0); w0 = put_u8(g[0], 1, w0); w0 = put_u8(b[0], 2, w0); w0 = put_u8(r[1], 3, w0);
        w1 = put_u8(g[1], 0, w1); w1 = put_u8(b[1], 1, w1); w1 = put_u8(r[2], 2, w1); w1 = put_u8(g[2], 3, w1);
        w2 = put_u8(b[2], 0, w2); w2 = put_u8(r[3], 1, w2); w2 = put_u8(g[3], 2, w2); w2 = put_u8(b[3], 3, w2);
    }
    if (npx == 4) {
        struct __attribute__((packed, aligned(1))) Twelve { uint32_t a, b, c; };
        Twelve tw; tw.a = w0; tw.b = w1; tw.c = w2;
        *reinterpret_cast<Twelve*>(wp) = tw;
    } else {
        for (uint32_t i = 0; i < npx * 3; i++) wp[i] = (uint8_t)((i < 4 ? w0 : (i < 8 ? w1 : w2)) >> (8 * (i & 3)));
    }
}

// --------------------------------------------------------------------------------------
// k_smooth: the five lowest AC coefficients of every block of a component of which only the DC first scan has been
// received, predicted from the DC coefficients of the block and its eight neighbours (T.81 K.8: the coefficients of
// the quadratic surface whose means over the nine blocks are the nine DC values; what stock decoders show for the
// first scans of a progressive file).  Integer form: weights 36/256, 9/256 and 5/256 of the de-quantised DC
// differences, rounded to a multiple of the coefficient's own quantiser step, halves away from zero, limited to
// +-1023; a neighbour beyond the component's block grid is the nearest block inside it.
// kClear = false: writes the first 16-byte chunk of each such block of the coefficient planes (zig-zag positions
// 0..7: 1..5 predicted, the others zero; the pixel kernel takes position 0 from the compact DC copy) and raises the
// component's zmax to 6, so that k_pixel reads that chunk and nothing more.  kClear = true, after k_pixel: the chunks
// are zero again and zmax is 1, the state an upgrade to a higher scan group builds on.
// grid: (kSmoothGroups, images); 256 lanes, a block per lane and trip.
// --------------------------------------------------------------------------------------
constexpr uint32_t kSmoothGroups = 8;
PCR_D int smooth_predict(int64_t w, int64_t q0, int64_t delta, int64_t qz) {
    const int64_t num = w * q0 * delta, den = 256 * qz;
    int64_t v = num >= 0 ? (num + den / 2) / den : -((-num + den / 2) / den);
    v = v > 1023 ? 1023 : (v < -1023 ? -1023 : v);
    return (int)v;
}
template <bool kClear>
__global__ void __launch_bounds__(256) k_smooth(DevRecord R) {
    __shared__ uint32_t does[kMaxComp];                      // per component: 1 if it holds its DC first scan and nothing else
    __shared__ uint32_t qs[kMaxComp][6];                     // its quantiser steps of zig-zag positions 0..5
    const uint32_t img = blockIdx.y, tid = threadIdx.x;
    ImgDesc* ip = R.img + img;
    const uint32_t nc = ip->nc;
    if (ip->status != kOk || !ip->progressive || nc > kMaxComp) return;
    if (tid < kMaxComp) {
        uint32_t carried = 0, dc_first = 0, tq = 0;
        if (tid < nc) {
            tq = ip->tq[tid];
            const ScanDesc* sc = R.scan + (size_t)img * R.G;
            const uint32_t ng = ip->nscans < R.G ? ip->nscans : R.G;
            for (uint32_t g = 0; g < ng; g++)
                for (uint32_t j = 0; j < sc[g].ns && j < kMaxComp; j++)
                    if (sc[g].comp[j] == tid) { carried++; dc_first += (sc[g].Ss == 0 && sc[g].Se == 0 && sc[g].Ah == 0) ? 1u : 0u; }
        }
        const bool on = carried == 1 && dc_first == 1 && ip->qoff[tq] != 0;
        does[tid] = on ? 1u : 0u;
        if (on) {
            const uint8_t* q = R.rec + ip->qoff[tq];
            const bool wide = ip->qprec[tq] != 0;
            // (a step of zero, which the standard does not allow, predicts nothing: DC step zero makes every difference zero,
            // and a coefficient with step zero de-quantises to zero whatever it is; the divisor only must not be zero)
            for (uint32_t k = 0; k < 6; k++) { const uint32_t v = wide ? ld_be16(q + 2 * k) : q[k]; qs[tid][k] = (v || k == 0) ? v : 1u; }
        }
    }
    __syncthreads();
    uint32_t plane0 = 0;
    for (uint32_t c = 0; c < nc; c++) {
        const uint32_t bw = ip->bw[c], bh = ip->bh[c], nb = bw * bh;
        if ((uint64_t)(plane0 + nb) * 64 > R.coef_off[img + 1] - R.coef_off[img]) return;   // (cannot happen for an image the parser accepted)
        if (does[c]) {
            if (blockIdx.x == 0 && tid == 0) ip->zmax[c] = kClear ? 1 : 6;
            const int16_t* dc = R.dc + (R.coef_off[img] >> 6) + plane0;
            int16_t* planes = R.coef + R.coef_off[img] + (size_t)plane0 * 64;
            const int64_t q0 = qs[c][0], q1 = qs[c][1], q2 = qs[c][2], q3 = qs[c][3], q4 = qs[c][4], q5 = qs[c][5];
            for (uint32_t b = blockIdx.x * 256 + tid; b < nb; b += kSmoothGroups * 256) {
                short8 o = short8{0, 0, 0, 0, 0, 0, 0, 0};
                if (!kClear) {
                    const uint32_t by = b / bw, bx = b - by * bw;
                    const uint32_t xl = bx ? bx - 1 : 0, xr = bx + 1 < bw ? bx + 1 : bx, ya = by ? by - 1 : 0, yb = by + 1 < bh ? by + 1 : by;
                    const int64_t al = dc[ya * bw + xl], a = dc[ya * bw + bx], ar = dc[ya * bw + xr];
                    const int64_t l = dc[by * bw + xl], m = dc[b], r = dc[by * bw + xr];
                    const int64_t bl = dc[yb * bw + xl], be = dc[yb * bw + bx], br = dc[yb * bw + xr];
                    o[1] = (short)smooth_predict(36, q0, l - r, q1);
                    o[2] = (short)smooth_predict(36, q0, a - be, q2);
                    o[3] = (short)smooth_predict(9, q0, a + be - 2 * m, q3);
                    o[4] = (short)smooth_predict(5, q0, (al - ar) - (bl - br), q4);
                    o[5] = (short)smooth_predict(9, q0, l + r - 2 * m, q5);
                }
                *reinterpret_cast<short8*>(planes + (size_t)b * 64) = o;
            }
        }
        plane0 += nb;
    }
}

// --------------------------------------------------------------------------------------
// k_pixel_smooth_flat: the pixels of a decode that holds DC first scans only, with k_smooth's predictions, without the
// detour through the coefficient planes and the full transform: one lane per 8x8 cell of pixels, as in k_pixel_flat.
// A block with zig-zag coefficients 0..5 only is
//     f(y, x) = F00 / 8 + a (F01 c1(x) + F02 c2(x)) + a (F10 c1(y) + F20 c2(y)) + F11 c1(x) c1(y) / 4,
//     a = 1 / (4 sqrt 2),  c1(t) = cos((2t + 1) pi / 16),  c2(t) = cos((2t + 1) pi / 8),
// a sum of a function of x, a function of y and one product: per component the lane keeps the two functions of x for
// its eight pixel columns and the two of y for its eight pixel rows (a cell of a component at half resolution covers
// four of the block's sample columns or rows, each twice), and a sample costs two operations.  Clamping, colour
// conversion and rounding as everywhere.  The predictions are the same integers k_smooth writes (32-bit arithmetic when
// the quantiser table has 8-bit entries: 36 x 255 x four DC coefficients fits).  Launched by the host only when every scan decoded
// is a DC first scan; a component without its DC scan reads as zero and is not predicted.
// grid: the flat tile list (runs of kFlatLanes cells of one image).
// --------------------------------------------------------------------------------------
PCR_D int smooth_predict32(uint32_t w, uint32_t q0, int delta, uint32_t qz) {
    const uint32_t mag = (uint32_t)(delta < 0 ? -delta : delta);
    const uint32_t num = w * q0 * mag, den = 256u * qz;
    uint32_t v = (num + den / 2) / den;
    v = v > 1023u ? 1023u : v;
    return delta < 0 ? -(int)v : (int)v;
}
__global__ void __launch_bounds__(kFlatLanes) k_pixel_smooth_flat(DevRecord R, const PixelTile* __restrict__ tiles, uint8_t* __restrict__ out) {
    __shared__ uint32_t does[kMaxComp];
    short_kernel_priority();
    const uint32_t item = xcd_major(blockIdx.x, gridDim.x);
    const uint32_t timg = uni(tiles[item].img), cell0 = uni(tiles[item].mcu0);
    ImgDesc D;
    load_desc(R.img + timg, &D);
    const uint32_t nc = D.nc, W = D.W, H = D.H;
    if (!flat_image(D)) return;
    if (threadIdx.x < kMaxComp) {
        uint32_t carried = 0, dc_first = 0;
        if (threadIdx.x < nc && D.progressive) {
            const ScanDesc* sc = R.scan + (size_t)timg * R.G;
            const uint32_t ng = D.nscans < R.G ? D.nscans : R.G;
            for (uint32_t g = 0; g < ng; g++)
                for (uint32_t j = 0; j < sc[g].ns && j < kMaxComp; j++)
                    if (sc[g].comp[j] == threadIdx.x) { carried++; dc_first += (sc[g].Ss == 0 && sc[g].Se == 0 && sc[g].Ah == 0) ? 1u : 0u; }
        }
        does[threadIdx.x] = (carried == 1 && dc_first == 1) ? 1u : 0u;
    }
    __syncthreads();
    const uint32_t cells_w = (W + 7) >> 3, total = cells_w * ((H + 7) >> 3);
    const uint32_t cell = cell0 + threadIdx.x;
    if (cell >= total) return;
    const uint32_t cy = cells_w == 1 ? cell : ((uint64_t)total * cells_w < (1ull << 32) ? __umulhi(cell, 0xFFFFFFFFu / cells_w + 1u) : cell / cells_w);
    const uint32_t cx = cell - cy * cells_w;
    const uint32_t x = cx * 8, y = cy * 8;
    const bool dead = uni((uint32_t)(R.status[timg] != kOk)) != 0;
    constexpr float kC1[8] = {0.98078528f, 0.83146961f, 0.55557023f, 0.19509032f, -0.19509032f, -0.55557023f, -0.83146961f, -0.98078528f};
    constexpr float kC2[8] = {0.92387953f, 0.38268343f, -0.38268343f, -0.92387953f, -0.92387953f, -0.38268343f, 0.38268343f, 0.92387953f};
    constexpr float kA = 0.17677670f;
    // per component and pixel column: the function of x and the factor of the product; per pixel row: the same of y
    float fx[kMaxComp][8], px[kMaxComp][8], fy[kMaxComp][8], py[kMaxComp][8];
    const int16_t* dcp = R.dc + (R.coef_off[timg] >> 6);
    uint32_t plane0 = 0;
#pragma unroll
    for (uint32_t c = 0; c < kMaxComp; c++) {
#pragma unroll
        for (int t = 0; t < 8; t++) { fx[c][t] = 128.f; px[c][t] = 0.f; fy[c][t] = 0.f; py[c][t] = 0.f; }
        if (c < nc) {
            const uint32_t shx = D.hs[c] == D.hmax ? 0u : 1u, shy = D.vs[c] == D.vmax ? 0u : 1u;      // (sampling factors are 1 or 2)
            const uint32_t bcol = (cx * D.hs[c]) >> (D.hmax - 1), brow = (cy * D.vs[c]) >> (D.vmax - 1);
            const uint32_t bw = D.bw[c], bh = D.bh[c];
            const uint32_t tq = D.tq[c] & 3;
            const uint32_t qoff = tq == 0 ? D.qoff[0] : (tq == 1 ? D.qoff[1] : (tq == 2 ? D.qoff[2] : D.qoff[3]));
            const uint32_t wide = tq == 0 ? D.qprec[0] : (tq == 1 ? D.qprec[1] : (tq == 2 ? D.qprec[2] : D.qprec[3]));
            const uint8_t* q = R.rec + qoff;
            uint32_t qs[6], qd[6];                           // the steps, and the divisors (a step of zero predicts nothing)
#pragma unroll
            for (uint32_t k = 0; k < 6; k++) { qs[k] = wide ? ld_be16(q + 2 * k) : q[k]; qd[k] = qs[k] ? qs[k] : 1u; }
            const int16_t* d = dcp + plane0;
            const int m = d[brow * bw + bcol];
            int p1 = 0, p2 = 0, p3 = 0, p4 = 0, p5 = 0;
            if (does[c] && qoff != 0 && bcol < bw && brow < bh) {
                const uint32_t xl = bcol ? bcol - 1 : 0, xr = bcol + 1 < bw ? bcol + 1 : bcol, ya = brow ? brow - 1 : 0, yb = brow + 1 < bh ? brow + 1 : brow;
                const int al = d[ya * bw + xl], a = d[ya * bw + bcol], ar = d[ya * bw + xr];
                const int l = d[brow * bw + xl], r = d[brow * bw + xr];
                const int bl = d[yb * bw + xl], be = d[yb * bw + bcol], br = d[yb * bw + xr];
                if (wide) {
                    p1 = smooth_predict(36, qs[0], l - r, qd[1]); p2 = smooth_predict(36, qs[0], a - be, qd[2]);
                    p3 = smooth_predict(9, qs[0], a + be - 2 * m, qd[3]); p4 = smooth_predict(5, qs[0], (al - ar) - (bl - br), qd[4]);
                    p5 = smooth_predict(9, qs[0], l + r - 2 * m, qd[5]);
                } else {
                    p1 = smooth_predict32(36, qs[0], l - r, qd[1]); p2 = smooth_predict32(36, qs[0], a - be, qd[2]);
                    p3 = smooth_predict32(9, qs[0], a + be - 2 * m, qd[3]); p4 = smooth_predict32(5, qs[0], (al - ar) - (bl - br), qd[4]);
                    p5 = smooth_predict32(9, qs[0], l + r - 2 * m, qd[5]);
                }
            }
            const float F00 = (float)m * (float)qs[0], F01 = (float)p1 * (float)qs[1], F10 = (float)p2 * (float)qs[2];
            const float F20 = (float)p3 * (float)qs[3], F11 = (float)p4 * (float)qs[4], F02 = (float)p5 * (float)qs[5];
            // the eight sample columns and rows of the block ...
            float gx[8], hx[8], gy[8];
#pragma unroll
            for (int t = 0; t < 8; t++) {
                gx[t] = F00 * 0.125f + 128.f + kA * (F01 * kC1[t] + F02 * kC2[t]);
                hx[t] = 0.25f * F11 * kC1[t];
                gy[t] = kA * (F10 * kC1[t] + F20 * kC2[t]);
            }
            // ... and those the cell's pixel columns and rows take them from
            const bool right = shx && (cx & 1u), low = shy && (cy & 1u);
#pragma unroll
            for (int t = 0; t < 8; t++) {
                fx[c][t] = shx ? (right ? gx[4 + (t >> 1)] : gx[t >> 1]) : gx[t];
                px[c][t] = shx ? (right ? hx[4 + (t >> 1)] : hx[t >> 1]) : hx[t];
                fy[c][t] = shy ? (low ? gy[4 + (t >> 1)] : gy[t >> 1]) : gy[t];
                py[c][t] = shy ? (low ? kC1[4 + (t >> 1)] : kC1[t >> 1]) : kC1[t];
            }
            plane0 += bw * bh;
        }
    }
    const uint32_t npx = W - x < 8 ? W - x : 8, nrows = H - y < 8 ? H - y : 8;
    const size_t pitch = (size_t)W * nc;
    uint8_t* wp = out + R.out_off[timg] + (size_t)y * pitch + (size_t)x * nc;
    struct __attribute__((packed, aligned(1))) Words2 { uint32_t a, b; };
    struct __attribute__((packed, aligned(1))) Words4 { uint32_t a, b, c, d; };
    // both chroma components at half resolution both ways (4:2:0): a chroma sample serves a 2 x 2 group of pixels and is
    // evaluated once for it (the same expression on the same values as below, so the pixels do not depend on the path)
    const bool quarter = nc == 3 && D.hs[0] == D.hmax && D.vs[0] == D.vmax && D.hs[1] != D.hmax && D.vs[1] != D.vmax && D.hs[2] != D.hmax && D.vs[2] != D.vmax;
#pragma unroll
    for (int rp = 0; rp < 4; rp++) {
        float u[8], v[8];
#pragma unroll
        for (int t = 0; t < 8; t++) { u[t] = 0.f; v[t] = 0.f; }
        if (quarter && !dead && (uint32_t)(2 * rp) < nrows) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                u[2 * j] = u[2 * j + 1] = clamp255(fx[1][2 * j] + fy[1][2 * rp] + px[1][2 * j] * py[1][2 * rp]) - 128.f;
                v[2 * j] = v[2 * j + 1] = clamp255(fx[2][2 * j] + fy[2][2 * rp] + px[2][2 * j] * py[2][2 * rp]) - 128.f;
            }
        }
#pragma unroll
        for (int dr = 0; dr < 2; dr++) {
            const int r = 2 * rp + dr;
            if ((uint32_t)r >= nrows) continue;
            uint32_t w[6] = {0, 0, 0, 0, 0, 0};
            if (!dead) {
                if (nc == 3 && !quarter) {
#pragma unroll
                    for (int t = 0; t < 8; t++) {
                        u[t] = clamp255(fx[1][t] + fy[1][r] + px[1][t] * py[1][r]) - 128.f;
                        v[t] = clamp255(fx[2][t] + fy[2][r] + px[2][t] * py[2][r]) - 128.f;
                    }
                }
#pragma unroll
                for (int t = 0; t < 8; t++) {
                    const float s0 = clamp255(fx[0][t] + fy[0][r] + px[0][t] * py[0][r]);
                    if (nc == 1) w[t >> 2] = put_u8(s0, t & 3, w[t >> 2]);
                    else {
                        w[(3 * t) >> 2] = put_u8(s0 + 1.402f * v[t], (3 * t) & 3, w[(3 * t) >> 2]);
                        w[(3 * t + 1) >> 2] = put_u8(s0 - 0.344136f * u[t] - 0.714136f * v[t], (3 * t + 1) & 3, w[(3 * t + 1) >> 2]);
                        w[(3 * t + 2) >> 2] = put_u8(s0 + 1.772f * u[t], (3 * t + 2) & 3, w[(3 * t + 2) >> 2]);
                    }
                }
            }
            uint8_t* rp8 = wp + (size_t)r * pitch;
            if (npx == 8) {
                if (nc == 1) { Words2 e; e.a = w[0]; e.b = w[1]; *reinterpret_cast<Words2*>(rp8) = e; }
                else {
                    Words4 e; e.a = w[0]; e.b = w[1]; e.c = w[2]; e.d = w[3];
                    Words2 f; f.a = w[4]; f.b = w[5];
                    *reinterpret_cast<Words4*>(rp8) = e; *reinterpret_cast<Words2*>(rp8 + 16) = f;
                }
            } else {                                        // the image's last, narrower column of cells
                const uint32_t nb = npx * nc;
                for (uint32_t i = 0; i < nb; i++) {
                    const uint32_t wi = i >> 2;
                    const uint32_t word = wi == 0 ? w[0] : (wi == 1 ? w[1] : (wi == 2 ? w[2] : (wi == 3 ? w[3] : (wi == 4 ? w[4] : w[5]))));
                    rp8[i] = (uint8_t)(word >> (8 * (i & 3)));
                }
            }
        }
    }
}

// --------------------------------------------------------------------------------------
// k_pixel_tail: decode and training tail in one kernel, so that the full-resolution pixels never reach memory.
// One workgroup per MCU row of one image, one lane per block as in k_pixel; the samples of the MCU row lie in LDS as
// one row-major plane per component, kTailLanes / blocks-per-MCU MCUs at a time (42 for 4:2:0: one pass for images up
// to 672 pixels wide; a wider box is done in passes that overlap by one MCU).
// Phase B is replaced by the tail: the output samples whose two source rows both lie in this MCU row are interpolated
// from pixels computed on the fly from the samples (colour conversion and rounding exactly as k_pixel does them, since
// the tail is defined on the rounded pixels).  Output rows whose two source rows lie in two MCU rows cannot be served
// by either workgroup: every workgroup leaves its first and last pixel row (1/8 of the pixels for 16-row MCUs) in a
// side buffer, and k_tail_edges interpolates those rows from it afterwards.
//   edge: side buffer; image i's part starts at edge_off[i] and holds, per MCU row r, its first pixel row at
//         (2 r) * W * C and its last one at (2 r + 1) * W * C.
// MCU rows (and MCUs) that do not touch the image's box are not decoded at all.
// --------------------------------------------------------------------------------------
constexpr int kTailLanes = 256;
struct TailParams { int out_h, out_w; float mean[3], istd[3]; };

// the rounded pixel (x, y) of the MCU row, y counted from the MCU row's first pixel row: up to three whole numbers
struct TailView {
    const float* plane[kMaxComp]; uint32_t len[kMaxComp], shx[kMaxComp], shy[kMaxComp], fm[kMaxComp]; uint32_t nc; bool dead;
};
PCR_D void tail_pixel(const TailView& V, uint32_t x, uint32_t y, float px[3]) {
    if (V.dead) { px[0] = px[1] = px[2] = 0.f; return; }
    const float s0 = V.plane[0][((y >> V.shy[0]) & V.fm[0]) * V.len[0] + ((x >> V.shx[0]) & V.fm[0])];
    if (V.nc == 1) { px[0] = fminf(fmaxf(__builtin_floorf(s0 + 0.5f), 0.f), 255.f); px[1] = px[2] = 0.f; return; }
    const float u = V.plane[1][((y >> V.shy[1]) & V.fm[1]) * V.len[1] + ((x >> V.shx[1]) & V.fm[1])] - 128.f;
    const float w = V.plane[2][((y >> V.shy[2]) & V.fm[2]) * V.len[2] + ((x >> V.shx[2]) & V.fm[2])] - 128.f;
    px[0] = fminf(fmaxf(__builtin_floorf(s0 + 1.402f * w + 0.5f), 0.f), 255.f);
    px[1] = fminf(fmaxf(__builtin_floorf(s0 - 0.344136f * u - 0.714136f * w + 0.5f), 0.f), 255.f);
    px[2] = fminf(fmaxf(__builtin_floorf(s0 + 1.772f * u + 0.5f), 0.f), 255.f);
}

template <bool kRefine>
__global__ void __launch_bounds__(kTailLanes) k_pixel_tail(DevRecord R, const PixelTile* __restrict__ tiles, const ApplyList* __restrict__ lists,
                                                           const int32_t* __restrict__ list_idx, const CropBox* __restrict__ boxes, TailParams P,
                                                           __half* __restrict__ out, uint8_t* __restrict__ edge, const uint64_t* __restrict__ edge_off) {
    __shared__ __attribute__((aligned(16))) float tile[kTailLanes * 64];
    __shared__ __attribute__((aligned(16))) float qz[kMaxComp][68];
    __shared__ ApplyList rl[kRefine ? kMaxComp : 1];
    __shared__ uint32_t row_lo, row_hi;                    // output rows served here: [row_lo, row_hi)
    short_kernel_priority();
    const uint32_t item = xcd_major(blockIdx.x, gridDim.x);
    const uint32_t timg = uni(tiles[item].img), mcu0 = uni(tiles[item].mcu0);
    const uint32_t tid = threadIdx.x;
    const ImgDesc* ip = R.img + timg;
    PixGeom G;
    pix_geom(ip, &G);
    const uint32_t nc = G.nc, W = G.W, H = G.H, mcux = G.mcux, bpm = G.bpm;
    const uint32_t mcu_px_w = 8 * G.hmax, mcu_px_h = 8 * G.vmax;
    const uint32_t seg_m = min((uint32_t)kTailLanes / max(bpm, 1u), mcux);   // MCUs one pass holds in LDS
    if (bpm == 0 || seg_m == 0 || (seg_m < 2 && mcux > 1)) return;       // (no sampling layout this library accepts gets here)
    const uint32_t my = mcu0 / mcux;
    const uint32_t ylo = my * mcu_px_h, yhi = ylo + mcu_px_h < H ? ylo + mcu_px_h : H;   // pixel rows of this MCU row
    const CropBox b = clamp_box(boxes[timg], (int)W, (int)H);
    if ((int)ylo >= b.y0 + b.h || (int)yhi <= b.y0) return;
    const uint32_t mc0 = (uint32_t)b.x0 / mcu_px_w, mc1 = (uint32_t)(b.x0 + b.w - 1) / mcu_px_w;   // MCUs the box touches
    const bool dead = uni((uint32_t)(R.status[timg] != kOk)) != 0;
    const uint32_t ml = (tid * recip16(bpm)) >> 16, j = tid - ml * bpm;   // MCU within the pass, block within the MCU
    if (kRefine) pix_lists(lists, list_idx, timg, nc, rl, tid, kTailLanes);
    pix_quant_table(R, ip, nc, qz, tid, kTailLanes);
    if (tid == 0) { row_lo = 0xFFFFFFFFu; row_hi = 0; }
    __syncthreads();
    // output rows both of whose source rows lie in [ylo, yhi): they form one interval
    for (int oy = (int)tid; oy < P.out_h; oy += kTailLanes) {
        int ya, yb; float fy;
        tail_rows(b, oy, P.out_h, &ya, &yb, &fy);
        if (ya >= (int)ylo && yb < (int)yhi) { atomicMin(&row_lo, (uint32_t)oy); atomicMax(&row_hi, (uint32_t)oy + 1); }
    }
    TailView V;
    V.nc = nc; V.dead = dead;
#pragma unroll
    for (uint32_t c = 0; c < kMaxComp; c++) {
        V.plane[c] = tile + seg_m * G.rb[c]; V.len[c] = seg_m * G.rs[c];
        V.shx[c] = c < nc && G.hs[c] != G.hmax; V.shy[c] = c < nc && G.vs[c] != G.vmax;
        V.fm[c] = G.flat[c] ? ~7u : ~0u;
    }
    // The MCUs the box touches, seg_m at a time.  A pass serves the source columns of all its MCUs but the last one,
    // which it holds only as the right-hand neighbour (an output sample reads columns xa and xa + 1); the pass that
    // reaches the box's last MCU serves that one too.  Most images need one pass.
    for (uint32_t s0 = mc0;; s0 += seg_m - 1) {
        const uint32_t s1 = min(s0 + seg_m - 1, mc1);                   // last MCU decoded in this pass
        const bool last = s1 == mc1;
        const uint32_t m = s0 + ml;
        const bool mine = !dead && ml < seg_m && m <= s1;
        PixBlock B;
        uint32_t by = 0, bx = 0;
        short8 v[8];
        if (mine) {
            pix_block(R, G, timg, j, my, m, &B, &by, &bx);
            if (B.zm <= 1) { v[0] = short8{0, 0, 0, 0, 0, 0, 0, 0}; v[0][0] = *B.dc; }
            else pix_load(B, v);
            const ApplyList* rlc = &rl[kRefine ? B.c : 0];
            const uint32_t row_len = seg_m * B.hs * 8;
            float* dst = tile + seg_m * pick3(B.c, G.rb[0], G.rb[1], G.rb[2]) + by * 8 * row_len + (ml * B.hs + bx) * 8;
            if (B.zm <= 1) dst[0] = clamp255((float)pix_dc<kRefine>(R, B, v[0][0], rlc) * qz[B.c][0] + 128.f);
            else pix_finish<kRefine>(R, B, v, qz[B.c], rlc, dst, row_len);
        }
        __syncthreads();
        const uint32_t xorg = s0 * mcu_px_w;                            // image column of the pass's first sample
        const uint32_t xs = max((uint32_t)b.x0, xorg);                  // source columns served here: [xs, xe)
        const uint32_t xe = last ? (uint32_t)(b.x0 + b.w) : s1 * mcu_px_w;
        // the first and the last pixel row, for the output rows that need a neighbouring MCU row as well
        {
            uint8_t* e = edge + edge_off[timg] + (size_t)(2 * my) * W * nc;
            const uint32_t span = xe - xs;
            for (uint32_t it = tid; it < 2 * span; it += kTailLanes) {
                const uint32_t which = it >= span, x = xs + (which ? it - span : it);
                float px[3];
                tail_pixel(V, x - xorg, which ? yhi - 1 - ylo : 0u, px);
                uint8_t* wp = e + ((size_t)which * W + x) * nc;
                for (uint32_t c = 0; c < nc; c++) wp[c] = (uint8_t)px[c];
            }
        }
        const uint32_t lo = row_lo, hi = row_hi;
        if (lo < hi) {
            const uint32_t ow = (uint32_t)P.out_w, items = (hi - lo) * ow;
            const uint32_t rcpw = ow > 1 ? 0xFFFFFFFFu / ow + 1u : 0u;
            for (uint32_t it = tid; it < items; it += kTailLanes) {
                const uint32_t r = ow > 1 ? __umulhi(it, rcpw) : it, ox = it - r * ow, oy = lo + r;
                int ya, yb, xa, xb; float fy, fx;
                tail_cols(b, (int)ox, P.out_w, &xa, &xb, &fx);
                if ((uint32_t)xa < xs || (uint32_t)xa >= xe) continue;  // another pass's column
                tail_rows(b, (int)oy, P.out_h, &ya, &yb, &fy);
                const uint32_t ua = (uint32_t)xa - xorg, ub = (uint32_t)xb - xorg;
                float aa[3], ab[3], ba[3], bb[3];
                tail_pixel(V, ua, (uint32_t)ya - ylo, aa); tail_pixel(V, ub, (uint32_t)ya - ylo, ab);
                tail_pixel(V, ua, (uint32_t)yb - ylo, ba); tail_pixel(V, ub, (uint32_t)yb - ylo, bb);
                __half* dst = out + ((size_t)timg * nc * P.out_h + oy) * ow + ox;
#pragma unroll
                for (uint32_t c = 0; c < kMaxComp; c++)
                    if (c < nc) dst[(size_t)c * P.out_h * ow] = tail_value(aa[c], ab[c], ba[c], bb[c], fx, fy, P.mean[c], P.istd[c]);
            }
        }
        if (last) break;
        __syncthreads();                                                // the samples in LDS are replaced next
    }
}

// The output rows k_pixel_tail could not serve: their two source rows are the last pixel row of one MCU row and the first
// of the next, both in the side buffer.  One workgroup per (output row, image); rows served already leave at once.
__global__ void __launch_bounds__(64) k_tail_edges(const uint32_t* __restrict__ dims, const uint32_t* __restrict__ mcu_rows_px, int C,
                                                   const CropBox* __restrict__ boxes, TailParams P, const uint8_t* __restrict__ edge,
                                                   const uint64_t* __restrict__ edge_off, __half* __restrict__ out) {
    const uint32_t i = blockIdx.y, oy = blockIdx.x;
    const int W = (int)dims[2 * i], H = (int)dims[2 * i + 1];
    const uint32_t mh = mcu_rows_px[i];                     // pixel rows per MCU row of this image (8 or 16)
    const CropBox b = clamp_box(boxes[i], W, H);
    int ya, yb; float fy;
    tail_rows(b, (int)oy, P.out_h, &ya, &yb, &fy);
    const uint32_t ra = (uint32_t)ya / mh, rb = (uint32_t)yb / mh;
    if (ra == rb) return;                                   // both rows in one MCU row: done by k_pixel_tail
    const uint8_t* e = edge + edge_off[i];
    const uint8_t* rowa = e + (size_t)(2 * ra + 1) * W * C;  // ya is the last row of MCU row ra, yb the first of rb = ra + 1
    const uint8_t* rowb = e + (size_t)(2 * rb) * W * C;
    for (int ox = (int)threadIdx.x; ox < P.out_w; ox += 64) {
        int xa, xb; float fx;
        tail_cols(b, ox, P.out_w, &xa, &xb, &fx);
        __half* dst = out + ((size_t)i * C * P.out_h + oy) * P.out_w + ox;
        for (int c = 0; c < C; c++)
            dst[(size_t)c * P.out_h * P.out_w] = tail_value((float)rowa[xa * C + c], (float)rowa[xb * C + c], (float)rowb[xa * C + c], (float)rowb[xb * C + c],
                                                            fx, fy, P.mean[c], P.istd[c]);
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

__global__ void __launch_bounds__(256) k_fill_zero(uint4* p, size_t n16) {
    short_kernel_priority();
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace pcr
