// Symbol statistics for the transcode to progressive files (paper Section 5, "Encoding": every image is re-coded as
// a progressive file before its scans are grouped into a record).  An optimised Huffman table needs to know how often
// each symbol occurs in a scan; k_symbol_hist counts that on the device, from the coefficient planes a decode left
// there, for every scan of the script the transcoder writes.  One wavefront per (image, scan): 64 blocks at a time in
// scan order, a lane per block counting its own symbols into a histogram in LDS; what spans blocks -- end-of-band
// runs -- is settled from two lane masks (block emits a symbol; block ends inside a run) by wave-uniform code.
// The symbol stream is the one pcr_encode.h's ScanCoder writes (the JPEG progressive coding procedures): the two are
// compared count by count in the tests.
#pragma once
#include "pcr_common.h"

namespace pcr {

// The scan scripts stock encoders use by default: DC with one bit held back, the low luma band, chroma, the rest of
// luma, then the held-back bits plane by plane.  nc = 3: 10 scans; nc = 1: 6 scans.
struct ScriptScan { uint8_t ns, comp[kMaxComp], Ss, Se, Ah, Al; };
constexpr int kScriptScansMax = 10;
PCR_HD int script_scans(int nc) { return nc == 3 ? 10 : 6; }
PCR_HD ScriptScan script_scan(int nc, int idx) {
    if (nc == 3) {
        switch (idx) {
            case 0: return ScriptScan{3, {0, 1, 2}, 0, 0, 0, 1};
            case 1: return ScriptScan{1, {0, 0, 0}, 1, 5, 0, 2};
            case 2: return ScriptScan{1, {2, 0, 0}, 1, 63, 0, 1};
            case 3: return ScriptScan{1, {1, 0, 0}, 1, 63, 0, 1};
            case 4: return ScriptScan{1, {0, 0, 0}, 6, 63, 0, 2};
            case 5: return ScriptScan{1, {0, 0, 0}, 1, 63, 2, 1};
            case 6: return ScriptScan{3, {0, 1, 2}, 0, 0, 1, 0};
            case 7: return ScriptScan{1, {2, 0, 0}, 1, 63, 1, 0};
            case 8: return ScriptScan{1, {1, 0, 0}, 1, 63, 1, 0};
            default: return ScriptScan{1, {0, 0, 0}, 1, 63, 1, 0};
        }
    }
    switch (idx) {
        case 0: return ScriptScan{1, {0, 0, 0}, 0, 0, 0, 1};
        case 1: return ScriptScan{1, {0, 0, 0}, 1, 5, 0, 2};
        case 2: return ScriptScan{1, {0, 0, 0}, 6, 63, 0, 2};
        case 3: return ScriptScan{1, {0, 0, 0}, 1, 63, 2, 1};
        case 4: return ScriptScan{1, {0, 0, 0}, 0, 0, 1, 0};
        default: return ScriptScan{1, {0, 0, 0}, 1, 63, 1, 0};
    }
}

// counts of one image: [scan of the script][table slot][symbol]; slot 0: the scan's first (or only) table, slot 1: the
// table of the second and third component of an interleaved DC scan
constexpr uint32_t kHistPerScan = 2 * 256, kHistPerImage = kScriptScansMax * kHistPerScan;

#if defined(__HIPCC__)

PCR_D uint32_t bit_length_u32(uint32_t v) { return v ? 32u - (uint32_t)__builtin_clz(v) : 0u; }

// planes: the coefficient planes with every scan applied (element k of a block = zig-zag position k); coef_off: [n + 1]
// element offsets of the images.  restart: MCUs per restart interval of the file to be written (0: none; a scan of
// one component counts its blocks).  hist: n * kHistPerImage counters, written (not added to).
// grid: (n, kScriptScansMax), one wavefront each.
__global__ void __launch_bounds__(64) k_symbol_hist(const ImgDesc* __restrict__ imgs, const int16_t* __restrict__ planes, const uint64_t* __restrict__ coef_off,
                                                    uint32_t restart, uint32_t* __restrict__ hist) {
    __shared__ uint32_t h[kHistPerScan];
    const uint32_t img = blockIdx.x, sidx = blockIdx.y, lane = threadIdx.x;
    for (uint32_t e = lane; e < kHistPerScan; e += 64) h[e] = 0;
    __syncthreads();
    const ImgDesc* D = imgs + img;
    const uint32_t nc = D->nc;
    uint32_t* out = hist + (size_t)img * kHistPerImage + (size_t)sidx * kHistPerScan;
    const bool live = (nc == 1 || nc == 3) && (int)sidx < script_scans((int)nc);
    const ScriptScan S = script_scan((int)nc, live ? (int)sidx : 0);
    if (live && !(S.Ss == 0 && S.Ah > 0)) {                // (a DC refinement scan is raw bits: no symbols)
        const int16_t* base = planes + coef_off[img];
        uint32_t plane0[kMaxComp + 1]; plane0[0] = 0;
        for (uint32_t c = 0; c < kMaxComp; c++) plane0[c + 1] = plane0[c] + (c < nc ? (uint32_t)D->bw[c] * D->bh[c] : 0);
        if (S.Ss == 0) {
            // ---- DC first: one difference per block against the previous block of the same component in scan order ----
            uint32_t bpm = 0, first_of[kMaxComp] = {0, 0, 0};
            for (uint32_t j = 0; j < S.ns; j++) { first_of[j] = bpm; bpm += S.ns > 1 ? (uint32_t)D->hs[S.comp[j]] * D->vs[S.comp[j]] : 1u; }
            const uint32_t c0 = S.comp[0];
            const uint32_t mcus = S.ns > 1 ? (uint32_t)D->mcux * D->mcuy : (uint32_t)D->cw[c0] * D->ch[c0];
            const uint32_t mcu_w = S.ns > 1 ? D->mcux : D->cw[c0];
            const uint32_t total = mcus * bpm;
            for (uint32_t t0 = 0; t0 < total; t0 += 64) {
                const uint32_t t = t0 + lane;
                if (t < total) {
                    const uint32_t m = t / bpm, within = t - m * bpm;
                    uint32_t j = 0;
                    for (uint32_t q = 1; q < S.ns; q++) if (within >= first_of[q]) j = q;
                    const uint32_t c = S.comp[j], hs = S.ns > 1 ? D->hs[c] : 1u, vs = S.ns > 1 ? D->vs[c] : 1u, bw = D->bw[c];
                    const uint32_t w = within - first_of[j], by = w / hs, bx = w - by * hs;
                    const uint32_t my = m / mcu_w, mx = m - my * mcu_w;
                    const int16_t* pl = base + (size_t)plane0[c] * 64;
                    const int v = (int)pl[((size_t)(my * vs + by) * bw + mx * hs + bx) * 64] >> S.Al;
                    int pred = 0;
                    if (w > 0) {                            // the block before it inside the MCU
                        const uint32_t pby = bx ? by : by - 1, pbx = bx ? bx - 1 : hs - 1;
                        pred = (int)pl[((size_t)(my * vs + pby) * bw + mx * hs + pbx) * 64] >> S.Al;
                    } else if (m > 0 && !(restart && m % restart == 0)) {   // the component's last block of the MCU before
                        const uint32_t pm = m - 1, pmy = pm / mcu_w, pmx = pm - pmy * mcu_w;
                        pred = (int)pl[((size_t)(pmy * vs + vs - 1) * bw + pmx * hs + hs - 1) * 64] >> S.Al;
                    }
                    const int diff = v - pred;
                    atomicAdd(&h[(j == 0 ? 0u : 256u) + bit_length_u32((uint32_t)(diff < 0 ? -diff : diff))], 1u);
                }
            }
        } else {
            // ---- AC scans (one component): the blocks that cover the component's samples, row by row ----
            const uint32_t c = S.comp[0], cw = D->cw[c], total = cw * (uint32_t)D->ch[c], bw = D->bw[c];
            const int16_t* pl = base + (size_t)plane0[c] * 64;
            uint32_t run = 0;                               // end-of-band run carried along the blocks (wave-uniform)
            auto emit_run = [&](uint32_t r) { if (lane == 0) atomicAdd(&h[(bit_length_u32(r) - 1u) << 4], 1u); };
            for (uint32_t t0 = 0; t0 < total; t0 += 64) {
                const uint32_t t = t0 + lane;
                bool emits = false, ends = false;           // the block emits a symbol of its own; it ends inside an end-of-band run
                if (t < total) {
                    const uint32_t row = t / cw, col = t - row * cw;
                    const int16_t* b = pl + ((size_t)row * bw + col) * 64;
                    int last_new = -1;
                    if (S.Ah) for (int k = S.Ss; k <= S.Se; k++) { const int x = b[k]; if (((x < 0 ? -x : x) >> S.Al) == 1) last_new = k; }
                    uint32_t zeros = 0; bool corr = false;
                    for (int k = S.Ss; k <= S.Se; k++) {
                        const int x = b[k];
                        const uint32_t mag = (uint32_t)(x < 0 ? -x : x) >> S.Al;
                        if (mag == 0) { zeros++; continue; }
                        if (S.Ah == 0) {
                            while (zeros > 15) { atomicAdd(&h[0xF0], 1u); zeros -= 16; }
                            atomicAdd(&h[(zeros << 4) | bit_length_u32(mag)], 1u);
                            zeros = 0; emits = true;
                        } else {
                            while (zeros > 15 && k <= last_new) { atomicAdd(&h[0xF0], 1u); zeros -= 16; corr = false; emits = true; }
                            if (mag > 1) { corr = true; continue; }     // known already: a correction bit, no symbol
                            atomicAdd(&h[(zeros << 4) | 1u], 1u);
                            zeros = 0; corr = false; emits = true;
                        }
                    }
                    ends = zeros > 0 || corr;
                }
                // What spans the blocks.  In scan order: a restart boundary and a block that emits a symbol both put out the
                // pending run first; a block that ends inside a run makes it one longer, and 32767 is the longest run there is.
                const uint64_t E = __ballot(emits), N = __ballot(ends);
                uint64_t B = 0;
                if (restart) B = __ballot(t < total && t > 0 && t % restart == 0);
                uint64_t todo = E | N | B;
                while (todo) {
                    const uint32_t i = (uint32_t)__builtin_ctzll(todo);
                    todo &= todo - 1;
                    if (((B | E) >> i) & 1) { if (run) emit_run(run); run = 0; }
                    if ((N >> i) & 1) { if (++run == 0x7FFF) { emit_run(run); run = 0; } }
                }
            }
            if (run) emit_run(run);
        }
    }
    __syncthreads();
    for (uint32_t e = lane; e < kHistPerScan; e += 64) out[e] = h[e];
}

#endif  // __HIPCC__

}  // namespace pcr
