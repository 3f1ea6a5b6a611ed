// gfx950 kernels of the PCR decode path.  One kernel per step:
//   k_index      scan-group index (prefix sums of region lengths)
//   k_parse      JPEG marker parsing, one lane per image
//   k_unstuff    byte un-stuffing + restart-interval location, one workgroup per (image, scan)
//   k_entropy    progressive Huffman decode, one lane per restart interval of a scan
//   k_apply      data-parallel part of AC refinement
//   k_pixel      de-quantise + IDCT + chroma replication + YCbCr->RGB + store
//   k_gather     materialise an image's scan prefix (parity hook)
#pragma once
#include <hip/hip_runtime.h>
#include "pcr_common.h"
#include "pcr_format.h"
#include "pcr_entropy.h"
#include "pcr_pixel.h"

namespace pcr {

// Everything a kernel needs to find its data; passed by value.
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
};

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
__global__ void __launch_bounds__(64) k_parse(DevRecord R, uint32_t kmax) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= R.n) return;
    parse_image(R.rec, R.off, R.len, R.n, i, R.nscans[i], kmax, &R.img[i], &R.scan[(size_t)i * R.G]);
    R.status[i] = R.img[i].status;
}

// --------------------------------------------------------------------------------------
// k_unstuff: per (image, scan) remove stuffed zeros, fill bytes and restart markers from the
// entropy-coded segment, stop at the first other marker, note where each restart interval
// begins.  256 lanes x 8 bytes per step, one exclusive scan per step.
// --------------------------------------------------------------------------------------
constexpr int kUnstuffPer = 8;

__global__ void __launch_bounds__(256) k_unstuff(DevRecord R, uint32_t kmax) {
    __shared__ uint32_t part[256];
    __shared__ uint32_t s_stop;
    uint32_t i = blockIdx.x, g = blockIdx.y;
    if (g >= kmax) return;
    const ImgDesc& img = R.img[i];
    if (img.status != kOk || g >= img.nscans) return;
    const ScanDesc& sd = R.scan[(size_t)i * R.G + g];
    const uint8_t* src = R.rec + sd.data_off;
    uint8_t* dst = R.clean + sd.data_off;
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
        uint32_t mine = (uint32_t)__builtin_popcount(keep) | ((uint32_t)__builtin_popcount(rst) << 16);
        part[threadIdx.x] = mine;
        __syncthreads();
        for (uint32_t d = 1; d < 256; d <<= 1) {
            uint32_t t = threadIdx.x >= d ? part[threadIdx.x - d] : 0;
            __syncthreads();
            part[threadIdx.x] += t;
            __syncthreads();
        }
        uint32_t excl = part[threadIdx.x] - mine;
        uint32_t o = out_total + (excl & 0xFFFF), r = rst_total + (excl >> 16);
        for (int j = 0; j < kUnstuffPer; j++) {
            if (keep & (1u << j)) dst[o++] = b[j + 1];
            if (rst & (1u << j)) { r++; if (r < sc) R.ivl_start[sb + r] = o; }
        }
        uint32_t tot = part[255];
        out_total += tot & 0xFFFF; rst_total += tot >> 16;
        __syncthreads();
        if (stop_all != 0xFFFFFFFFu) break;
    }
    if (threadIdx.x == 0) {
        // intervals whose restart marker never showed up get an empty range; the end goes last
        for (uint32_t r = rst_total + 1; r <= sc; r++) R.ivl_start[sb + r] = out_total;
        if (rst_total + 1 != sc) R.status[i] = kEFormat;
    }
}

// --------------------------------------------------------------------------------------
// k_entropy: one lane per unit.  Each lane builds the Huffman tables of its scan in LDS.
// --------------------------------------------------------------------------------------
constexpr int kEntropyLanes = 32;
constexpr int kTabsPerLane = 3;

__global__ void __launch_bounds__(kEntropyLanes) k_entropy(DevRecord R, const Unit* units, uint32_t nunits) {
    extern __shared__ __align__(16) uint8_t smem[];
    HuffTab* tabs = reinterpret_cast<HuffTab*>(smem) + (size_t)threadIdx.x * kTabsPerLane;
    uint8_t* zz = smem + sizeof(HuffTab) * kEntropyLanes * kTabsPerLane;
    for (int k = threadIdx.x; k < 64; k += blockDim.x) zz[k] = (uint8_t)zigzag_natural(k);
    __syncthreads();
    uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= nunits) return;
    const Unit un = units[u];
    const ImgDesc& img = R.img[un.img];
    if (R.status[un.img] != kOk || un.scan >= img.nscans) return;
    const ScanDesc& sd = R.scan[(size_t)un.img * R.G + un.scan];
    if (!sd.valid) return;
    const size_t ig = (size_t)un.img * R.G + un.scan;
    const uint32_t sb = R.slot_base[ig];
    const uint32_t b0 = R.ivl_start[sb + un.interval], b1 = R.ivl_start[sb + un.interval + 1];
    BitReader br;
    br.init(R.clean + sd.data_off + b0, b1 > b0 ? b1 - b0 : 0);
    UnitGeom ug;
    ug.mcu_w = sd.mcu_w;
    ug.mcu0 = sd.ri ? un.interval * sd.ri : 0;
    ug.mcu1 = sd.ri ? (ug.mcu0 + sd.ri < sd.mcus ? ug.mcu0 + sd.ri : sd.mcus) : sd.mcus;
    if (ug.mcu0 >= sd.mcus) return;
    int16_t* base = R.coef + R.coef_off[un.img];
    int16_t* cpl[kMaxComp];
    {
        size_t o = 0; int16_t* pl[kMaxComp];
        for (int c = 0; c < img.nc; c++) { pl[c] = base + o; o += (size_t)img.bw[c] * img.bh[c] * 64; }
        for (int j = 0; j < sd.ns; j++) cpl[j] = pl[sd.comp[j]];
    }
    int rc;
    if (sd.Ss == 0) {
        if (sd.Ah == 0) {
            const HuffTab* tp[kMaxComp];
            for (int j = 0; j < sd.ns; j++) {
                int same = -1;
                for (int q = 0; q < j; q++) if (sd.dc_off[q] == sd.dc_off[j]) same = q;
                if (same >= 0) tp[j] = tp[same];
                else { hufftab_build(&tabs[j], R.rec + sd.dc_off[j]); tp[j] = &tabs[j]; }
            }
            rc = decode_dc_first(&br, &img, &sd, &ug, tp, cpl);
        } else rc = decode_dc_refine(&br, &img, &sd, &ug, cpl);
    } else {
        hufftab_build(&tabs[0], R.rec + sd.ac_off);
        int c = sd.comp[0];
        size_t plane = (size_t)img.bw[c] * img.bh[c];
        uint64_t* mk = R.masks + R.mask_off[ig];
        if (sd.Ah == 0) rc = decode_ac_first(&br, &img, &sd, &ug, &tabs[0], zz, cpl[0], mk);
        else {
            const uint64_t* hist[kMaxHist];
            for (int q = 0; q < sd.nhist; q++) hist[q] = R.masks + R.mask_off[(size_t)un.img * R.G + sd.hist[q]];
            rc = decode_ac_refine(&br, &img, &sd, &ug, &tabs[0], hist, sd.nhist, mk, mk + plane, mk + 2 * plane);
        }
    }
    if (rc != kOk) R.status[un.img] = rc;
}

// --------------------------------------------------------------------------------------
// k_apply: for every coefficient of every block a non-interleaved scan visits, replay the AC
// scans of its component in file order: first scans only extend the non-zero mask, refinement
// scans add their correction bit or place their new +-2^Al value.
// grid: (ceil(max covered coefficients / 256), apply units)
// --------------------------------------------------------------------------------------
struct ApplyUnit { uint32_t img; uint32_t comp; };

__global__ void __launch_bounds__(256) k_apply(DevRecord R, const ApplyUnit* au, uint32_t kmax) {
    const ApplyUnit a = au[blockIdx.y];
    const ImgDesc& img = R.img[a.img];
    if (R.status[a.img] != kOk) return;
    const int c = a.comp;
    const uint32_t cw = img.cw[c], ncov = cw * img.ch[c];
    uint32_t idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= ncov * 64) return;
    const uint32_t cb = idx >> 6; const int k = idx & 63;
    const size_t blk = (size_t)(cb / cw) * img.bw[c] + (cb % cw);
    const size_t plane = (size_t)img.bw[c] * img.bh[c];
    int16_t* pl = R.coef + R.coef_off[a.img];
    for (int q = 0; q < c; q++) pl += (size_t)img.bw[q] * img.bh[q] * 64;
    int16_t* cp = pl + blk * 64 + zigzag_natural(k);
    int16_t v = *cp; const int16_t v0 = v;
    uint64_t h = 0;
    const uint32_t upto = img.nscans < kmax ? img.nscans : kmax;
    for (uint32_t g = 0; g < upto; g++) {
        const ScanDesc& sd = R.scan[(size_t)a.img * R.G + g];
        if (sd.Ss == 0 || sd.comp[0] != c) continue;
        const uint64_t* mk = R.masks + R.mask_off[(size_t)a.img * R.G + g];
        if (sd.Ah != 0 && k >= sd.Ss && k <= sd.Se)
            v = refine_apply(v, k, h & band_mask(sd.Ss, sd.Se), mk[blk], mk[plane + blk], mk[2 * plane + blk], sd.Al);
        h |= mk[blk];
    }
    if (v != v0) *cp = v;
}

// --------------------------------------------------------------------------------------
// k_pixel: one workgroup per strip of up to kStripMcus MCUs of one MCU row of one image.
// Phase 1: de-quantise + row IDCT per (block, row); phase 2: column IDCT + level shift + clamp;
// phase 3: chroma replication + colour + store.
// --------------------------------------------------------------------------------------
constexpr int kStripMcus = 8;
constexpr int kMaxBlocksPerMcu = 6;        // 4:2:0: 4 + 1 + 1

struct PixelTile { uint32_t img; uint16_t mcu_row; uint16_t mcu_col0; };

__global__ void __launch_bounds__(256) k_pixel(DevRecord R, const PixelTile* tiles, uint8_t* out) {
    __shared__ float tile[kStripMcus * kMaxBlocksPerMcu * 64];
    __shared__ float qn[kMaxComp][64];
    const PixelTile t = tiles[blockIdx.x];
    const ImgDesc& img = R.img[t.img];
    const int nc = img.nc;
    const uint32_t W = img.W, H = img.H;
    uint8_t* o = out + R.out_off[t.img];
    const uint32_t mcu_px_w = 8 * img.hmax, mcu_px_h = 8 * img.vmax;
    const uint32_t nm = (uint32_t)img.mcux - t.mcu_col0 < (uint32_t)kStripMcus ? (uint32_t)img.mcux - t.mcu_col0 : (uint32_t)kStripMcus;
    const uint32_t x0 = t.mcu_col0 * mcu_px_w, y0 = t.mcu_row * mcu_px_h;
    const uint32_t sw = nm * mcu_px_w;                     // strip width in pixels
    if (R.status[t.img] != kOk) {                          // corrupt image: zero-filled
        for (uint32_t p = threadIdx.x; p < sw * mcu_px_h; p += 256) {
            uint32_t y = y0 + p / sw, x = x0 + p % sw;
            if (x < W && y < H) for (int c = 0; c < nc; c++) o[((size_t)y * W + x) * nc + c] = 0;
        }
        return;
    }
    // quantisation tables in natural order
    for (int e = threadIdx.x; e < nc * 64; e += 256) {
        int c = e >> 6, k = e & 63;
        const uint8_t* q = R.rec + img.qoff[img.tq[c]];
        qn[c][zigzag_natural(k)] = img.qprec[img.tq[c]] ? (float)ld_be16(q + 2 * k) : (float)q[k];
    }
    __syncthreads();
    // blocks of the strip, component by component: component c contributes nm*hs rows of vs
    uint32_t cbase[kMaxComp + 1]; cbase[0] = 0;
    for (int c = 0; c < nc; c++) cbase[c + 1] = cbase[c] + nm * img.hs[c] * img.vs[c];
    const uint32_t nblk = cbase[nc];
    const int16_t* coef = R.coef + R.coef_off[t.img];
    // phase 1
    for (uint32_t w = threadIdx.x; w < nblk * 8; w += 256) {
        uint32_t b = w >> 3, v = w & 7;
        int c = 0; while (b >= cbase[c + 1]) c++;
        uint32_t lb = b - cbase[c];
        uint32_t bwc = nm * img.hs[c];                     // blocks per row of this strip in component c
        uint32_t brow = t.mcu_row * img.vs[c] + lb / bwc, bcol = t.mcu_col0 * img.hs[c] + lb % bwc;
        const int16_t* pl = coef;
        for (int q = 0; q < c; q++) pl += (size_t)img.bw[q] * img.bh[q] * 64;
        const int16_t* src = pl + ((size_t)brow * img.bw[c] + bcol) * 64 + v * 8;
        float in[8], res[8];
        for (int u = 0; u < 8; u++) in[u] = (float)src[u] * qn[c][v * 8 + u];
        idct8(in, res);
        for (int x = 0; x < 8; x++) tile[b * 64 + v * 8 + x] = res[x];
    }
    __syncthreads();
    // phase 2
    for (uint32_t w = threadIdx.x; w < nblk * 8; w += 256) {
        uint32_t b = w >> 3, x = w & 7;
        float in[8], res[8];
        for (int v = 0; v < 8; v++) in[v] = tile[b * 64 + v * 8 + x];
        idct8(in, res);
        for (int y = 0; y < 8; y++) tile[b * 64 + y * 8 + x] = clamp255(res[y] + 128.f);
    }
    __syncthreads();
    // phase 3
    for (uint32_t p = threadIdx.x; p < sw * mcu_px_h; p += 256) {
        uint32_t ly = p / sw, lx = p % sw;
        uint32_t y = y0 + ly, x = x0 + lx;
        if (x >= W || y >= H) continue;
        float s[kMaxComp];
        for (int c = 0; c < nc; c++) {
            uint32_t sx = lx * img.hs[c] / img.hmax, sy = ly * img.vs[c] / img.vmax;   // sample in the strip's plane
            uint32_t bwc = nm * img.hs[c];
            uint32_t b = cbase[c] + (sy >> 3) * bwc + (sx >> 3);
            s[c] = tile[b * 64 + (sy & 7) * 8 + (sx & 7)];
        }
        uint8_t* dst = o + ((size_t)y * W + x) * nc;
        if (nc == 1) dst[0] = round_u8(s[0]);
        else ycc_to_rgb(s[0], s[1], s[2], dst);
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

__global__ void __launch_bounds__(256) k_fill_zero(uint4* p, size_t n16) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace pcr
