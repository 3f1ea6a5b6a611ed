// Shared definitions of the PCR decode library: descriptor structs and small helpers that are
// compiled both for the gfx950 device and for the host (PCR_HD).
#pragma once
#include <stdint.h>
#include <stddef.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define PCR_HD __host__ __device__ inline
#define PCR_D __device__ inline
#else
#define PCR_HD inline
#define PCR_D inline
#endif

namespace pcr {

// error codes of the C ABI (include/pcr.h) -- repeated as plain ints so device code can set them
enum : int { kOk = 0, kEArg = -1, kEFormat = -2, kETruncated = -3, kEUnsupported = -4, kERange = -5, kENoMem = -6, kEDevice = -7 };

constexpr int kMaxComp = 3;
constexpr int kMaxHist = 6;      // earlier AC refinement scans of the same component a refinement scan may build on
constexpr int kApplyMaxScans = 16;   // refinement scans (DC and AC together) of one component that are replayed when the
                                     // coefficients are loaded; a file with more is refused when its headers are parsed

// One image of a record (frame header + tables that hold for the whole image).
struct ImgDesc {
    uint16_t W, H;
    uint8_t nc, hmax, vmax, progressive;
    uint8_t hs[kMaxComp], vs[kMaxComp], tq[kMaxComp], cid[kMaxComp];
    uint16_t mcux, mcuy;
    uint16_t bw[kMaxComp], bh[kMaxComp];   // allocated block grid (MCU padded)
    uint16_t cw[kMaxComp], ch[kMaxComp];   // blocks covering the component's own samples
    uint32_t qoff[4];                      // absolute record offset of the 64 DQT entries (0 = undefined)
    uint8_t qprec[4];                      // 0: 8-bit entries, 1: 16-bit big endian
    int32_t status;                        // kOk or the first error found while parsing
    uint32_t nscans;                       // scans parsed
    uint8_t zmax[kMaxComp];                // per component: zig-zag positions [0, zmax) may be non-zero after the scans parsed
    uint8_t pad;
};

static_assert(sizeof(ImgDesc) % 4 == 0, "ImgDesc is copied as dwords");

// One scan of one image.
struct ScanDesc {
    uint32_t data_off;                     // absolute record offset of the entropy-coded segment
    uint32_t data_len;                     // bytes from data_off to the end of the scan's region
    uint32_t dc_off[kMaxComp];             // record offset of BITS[16] of the DC table of scan component j
    uint32_t ac_off;                       // same for the AC table (AC scans have one component)
    uint16_t ri;                           // restart interval in MCUs of this scan (0 = none)
    uint8_t ns, comp[kMaxComp];
    uint8_t Ss, Se, Ah, Al;
    uint8_t nhist, hist[kMaxHist];         // AC refinement: earlier AC REFINEMENT scans (indices) of the same component and band
    uint8_t valid;
    uint32_t mcus;                         // MCUs in this scan
    uint32_t mcu_w;                        // MCUs per row of this scan
    uint32_t ac_offc[kMaxComp];            // sequential scans: record offset of BITS[16] of the AC table of scan component j
};

// A scan of a sequential (baseline) file carries whole blocks: DC difference, then the AC run/size pairs.
PCR_HD bool is_sequential_scan(const ScanDesc& sd) { return sd.Ss == 0 && sd.Se == 63; }

struct Unit {                              // one independently decodable piece: a restart interval of a scan
    uint32_t img;
    uint32_t scan;
    uint32_t interval;
    uint32_t slot;                         // index into the interval tables
};

PCR_HD uint32_t ld_le32(const uint8_t* p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }
PCR_HD uint64_t ld_le64(const uint8_t* p) { return (uint64_t)ld_le32(p) | ((uint64_t)ld_le32(p + 4) << 32); }
PCR_HD uint32_t ld_be16(const uint8_t* p) { return ((uint32_t)p[0] << 8) | p[1]; }

// Tell the compiler a value is the same in every lane of the wavefront (it then lives in a
// scalar register).  Only used where that is true by construction.
PCR_HD uint32_t uni(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
#else
    return v;
#endif
}
PCR_HD int uni(int v) { return (int)uni((uint32_t)v); }
PCR_HD uint64_t uni(uint64_t v) { return ((uint64_t)uni((uint32_t)(v >> 32)) << 32) | uni((uint32_t)v); }
// (pointers: apply uni() to the offset and add it to a kernel-argument base pointer; a pointer
// rebuilt from integers loses its address space and loads through it count as divergent)

PCR_HD uint32_t bitrev32(uint32_t v) {
#if defined(__has_builtin)
#if __has_builtin(__builtin_bitreverse32)
    return __builtin_bitreverse32(v);
#else
    v = ((v >> 1) & 0x55555555u) | ((v & 0x55555555u) << 1);
    v = ((v >> 2) & 0x33333333u) | ((v & 0x33333333u) << 2);
    v = ((v >> 4) & 0x0F0F0F0Fu) | ((v & 0x0F0F0F0Fu) << 4);
    return __builtin_bswap32(v);
#endif
#else
    v = ((v >> 1) & 0x55555555u) | ((v & 0x55555555u) << 1);
    v = ((v >> 2) & 0x33333333u) | ((v & 0x33333333u) << 2);
    v = ((v >> 4) & 0x0F0F0F0Fu) | ((v & 0x0F0F0F0Fu) << 4);
    return __builtin_bswap32(v);
#endif
}

// zig-zag position -> natural index, by walking the anti-diagonals (row + col = d)
PCR_HD constexpr int zigzag_natural(int k) {
    int d = 0, first = 0;
    while (true) {                                   // find diagonal d holding position k
        int len = d < 8 ? d + 1 : 15 - d;
        if (k < first + len) break;
        first += len; d++;
    }
    int j = k - first;
    int lo = d < 8 ? 0 : d - 7;                      // smallest row (or col) index on this diagonal
    // even diagonals run bottom-left -> top-right (row decreasing), odd ones the other way
    int row = (d & 1) ? lo + j : (d < 8 ? d : 7) - j;
    return row * 8 + (d - row);
}

// the same as a table, filled in at compile time by the walk above (for code that looks positions up per lane)
struct ZigzagTable {
    uint8_t natural[64];
    constexpr ZigzagTable() : natural{} { for (int k = 0; k < 64; k++) natural[k] = (uint8_t)zigzag_natural(k); }
};
PCR_HD uint32_t zigzag_lookup(uint32_t k) {
    constexpr ZigzagTable t{};
    return t.natural[k];
}

// Pointer to the unstuffed entropy data as the decoders read it.  The data was written by an earlier
// kernel and is never written while a decoder runs, so on the device it is addressed as constant memory:
// loads through such a pointer at a wave-uniform address are scalar loads, which arrive straight in
// scalar registers and are only waited for at their first use.
#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) uint32_t* StreamPtr;
#else
typedef const uint32_t* StreamPtr;
#endif
PCR_HD StreamPtr stream_ptr(const uint32_t* p) { return (StreamPtr)p; }

}  // namespace pcr
