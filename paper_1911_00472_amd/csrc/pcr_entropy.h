// Progressive-JPEG entropy decoding for one independently decodable unit (a restart interval
// of one scan of one image), written so that the same code runs in a gfx950 lane and on the
// host.  Decoding follows the JPEG progressive mode (spectral selection + successive
// approximation) that the paper's records are made of (Section 2, "Progressive Image
// Compression"; Section 3: scan k of an image is usable once scans 1..k have been read).
//
// Input is the *unstuffed* entropy-coded data of the unit (FF 00 -> FF, restart markers
// removed); consuming a bit past the unit's end is a data error, never a guess.
//
// Shape of the decoders: ONE WAVEFRONT DECODES ONE UNIT.  Every value below is then the same in
// all 64 lanes, so the compiler keeps it in scalar registers and the loops run on the scalar
// ALU (native 64-bit shifts, population count, find-first-set), paying only for the branch
// actually taken.  All per-scan parameters are passed in registers (LaneScan); the Huffman
// table lives in LDS.
//
// AC refinement is decoded against a 64-bit "already non-zero" mask per block (zig-zag bit
// order) instead of against the coefficients: the serial decoder only finds where new
// coefficients go, their signs, and the string of correction bits (exactly one per already
// non-zero coefficient of the band, in zig-zag order); the arithmetic on the coefficients is
// data-parallel (refine_apply).  DC refinement needs no serial decoder at all: it is one
// bit per block at a position known in advance (dc_refine_bit).
#pragma once
#include "pcr_common.h"

namespace pcr {

// ---------------------------------------------------------------------------------------
// Huffman tables.  Codes of <= 8 bits resolve through `lut`, indexed by the next 8 bits.  In a
// canonical code the longer code words are the numerically largest ones, so all of them lie in
// [limit8, 65536) when left-aligned in 16 bits; `lut2`, indexed by the distance from limit8
// scaled to 128 entries, resolves every long code that owns at least one whole entry, and the
// canonical limits resolve the rest.  An entry is (length << 8) | symbol; 0 means "not here".
// ---------------------------------------------------------------------------------------
struct AcTab {
    uint16_t lut[256];
    uint16_t lut2[128];
    uint32_t limit[9];          // limit[L-8]: first 16-bit-left-aligned code value NOT of length <= L (L = 8..16)
    uint16_t valptr[8];         // valptr[L-9]: index in huffval of the first code of length L
    uint32_t sh2;               // lut2 index = (code16 - limit[0]) >> sh2
    uint8_t huffval[256];
    uint32_t pad;
    // the 8-bit look-up again, pre-packed for the lanes of a window reader (see packed_entry): everything
    // of a symbol's packed word that does not depend on the bits after the code
    uint32_t lutp[256];
};
static_assert(sizeof(AcTab) == 1084 + 1024, "AcTab layout");

struct DcTab {                  // DC symbols are categories 0..15
    uint8_t lut[256];           // (length << 4) | symbol for codes of <= 8 bits, 0xFF otherwise
    uint32_t limit[9];
    uint16_t valptr[8];
    uint8_t huffval[16];
};
static_assert(sizeof(DcTab) == 324, "DcTab layout");

// Build from a DHT payload: 16 counts followed by the symbols in code order.  Codes of each
// length are consecutive integers in symbol order; moving to the next length doubles the code.
PCR_HD void dctab_build(DcTab* t, const uint8_t* bits_vals) {
    for (int i = 0; i < 256; i++) t->lut[i] = 0xFF;
    uint32_t code = 0; int k = 0;
    for (int L = 1; L <= 16; L++) {
        int cnt = bits_vals[L - 1];
        if (L >= 9) t->valptr[L - 9] = (uint16_t)k;
        for (int j = 0; j < cnt; j++) {
            if (k < 16) {
                uint8_t sym = bits_vals[16 + k];
                t->huffval[k] = sym;
                if (L <= 8) {
                    uint32_t first = code << (8 - L), span = 1u << (8 - L);
                    for (uint32_t e = 0; e < span && first + e < 256; e++) t->lut[first + e] = (uint8_t)((L << 4) | (sym & 15));
                }
            }
            code++; k++;
        }
        if (L >= 8) { uint64_t lim = (uint64_t)code << (16 - L); t->limit[L - 8] = lim > 65536 ? 65536u : (uint32_t)lim; }
        code <<= 1;
    }
}

PCR_HD void actab_build(AcTab* t, const uint8_t* bits_vals) {
    for (int i = 0; i < 256; i++) t->lut[i] = 0;
    for (int i = 0; i < 128; i++) t->lut2[i] = 0;
    // pass 1: short codes, limits
    uint32_t code = 0; int k = 0;
    for (int L = 1; L <= 16; L++) {
        int cnt = bits_vals[L - 1];
        if (L >= 9) t->valptr[L - 9] = (uint16_t)k;
        for (int j = 0; j < cnt; j++) {
            if (k < 256) {
                uint8_t sym = bits_vals[16 + k];
                t->huffval[k] = sym;
                if (L <= 8) {
                    uint32_t first = code << (8 - L), span = 1u << (8 - L);
                    for (uint32_t e = 0; e < span && first + e < 256; e++) t->lut[first + e] = (uint16_t)((L << 8) | sym);
                }
            }
            code++; k++;
        }
        if (L >= 8) { uint64_t lim = (uint64_t)code << (16 - L); t->limit[L - 8] = lim > 65536 ? 65536u : (uint32_t)lim; }
        code <<= 1;
    }
    // pass 2: long codes into lut2
    const uint32_t lim8 = t->limit[0];
    const uint32_t D = 65536u - lim8;
    uint32_t sh2 = 0;
    while (D && ((D - 1) >> sh2) >= 128) sh2++;
    t->sh2 = sh2;
    code = 0; k = 0;
    for (int L = 1; L <= 16; L++) {
        int cnt = bits_vals[L - 1];
        for (int j = 0; j < cnt; j++) {
            if (L >= 9 && k < 256 && (uint32_t)(16 - L) >= sh2) {
                uint64_t c = (uint64_t)code << (16 - L);
                if (c >= lim8 && c < 65536) {
                    uint32_t first = ((uint32_t)c - lim8) >> sh2, span = 1u << (16 - L - sh2);
                    for (uint32_t e = 0; e < span && first + e < 128; e++) t->lut2[first + e] = (uint16_t)((L << 8) | bits_vals[16 + k]);
                }
            }
            code++; k++;
        }
        code <<= 1;
    }
}

// The unstuffed data of a unit is stored as big-endian 32-bit words (the unstuff step swaps the bytes of
// every aligned 4-byte group), so a word is usable as loaded.  The buffer stays readable for some bytes
// past any position a decoder can reach before it checks for an overrun.

// bits [len, len+n) of a 32-bit window (n may be 0)
PCR_HD uint32_t field(uint32_t win, int len, int n) { return n ? (win << len) >> (32 - n) : 0; }

// Hides where a value came from, so that the compiler keeps it in the register it is in instead of
// re-deriving it from other values it would then have to keep alive through a hot loop.
PCR_HD uint32_t opaque(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+s"(v));
#endif
    return v;
}
// Bits [pos, pos + width) of v with the field packed as (width << 16) | pos in a register (one instruction).
PCR_HD uint32_t bit_field(uint32_t v, uint32_t packed) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t r;
    asm("s_bfe_u32 %0, %1, %2" : "=s"(r) : "s"(v), "s"(packed) : "scc");
    return r;
#else
    return (v >> (packed & 31)) & ((1u << (packed >> 16)) - 1);
#endif
}
// The loop that follows starts on a 64-byte line of the instruction cache (a lone wavefront runs a short loop
// visibly faster when it does not straddle lines); the padding is jumped over, not executed.
PCR_HD void align_loop() {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_branch 1f\n\t.p2align 6\n1:");
#endif
}

// Resolve a code of more than 8 bits.  Returns (length << 8) | symbol, or 0 if it is no code.
PCR_HD uint32_t ac_long_code(const AcTab* t, uint32_t win) {
    const uint32_t c16 = win >> 16;
    const uint32_t lim8 = t->limit[0];
    if (c16 < lim8) return 0;
    const uint32_t i2 = (c16 - lim8) >> t->sh2;
    uint32_t e = i2 < 128 ? t->lut2[i2] : 0;
    if (e) return e;
    for (int L = 9; L <= 16; L++) {
        if (c16 < t->limit[L - 8]) {
            uint32_t idx = t->valptr[L - 9] + ((c16 - t->limit[L - 9]) >> (16 - L));
            return idx < 256 ? ((uint32_t)L << 8) | t->huffval[idx] : 0;
        }
    }
    return 0;
}
PCR_HD uint32_t ac_code(const AcTab* t, uint32_t win) {
    uint32_t e = t->lut[win >> 24];
    return e ? e : ac_long_code(t, win);
}
// DC: returns (length << 4) | category, or 0 if it is no code (a valid entry is never 0: length >= 1)
PCR_HD uint32_t dc_code(const DcTab* t, uint32_t win) {
    uint32_t e = t->lut[win >> 24];
    if (e != 0xFF) return e;
    const uint32_t c16 = win >> 16;
    if (c16 < t->limit[0]) return 0;
    for (int L = 9; L <= 16; L++) {
        if (c16 < t->limit[L - 8]) {
            uint32_t idx = t->valptr[L - 9] + ((c16 - t->limit[L - 9]) >> (16 - L));
            return idx < 16 ? ((uint32_t)L << 4) | t->huffval[idx] : 0;
        }
    }
    return 0;
}

PCR_HD int extend(uint32_t v, int s) { return (s && v < (1u << (s - 1))) ? (int)v - (1 << s) + 1 : (int)v; }

// ---------------------------------------------------------------------------------------
// Window reader for the AC scans: the 64 lanes of the wavefront look up, in parallel, the
// Huffman code that WOULD start at each of the next 64 bit offsets of the stream (which code
// starts where does not depend on the decoder's state), and pack what follows from it --
// symbol, total length with its appended bits, the appended value -- into one word per lane.
// The serial part of the decoder then only follows the chain of offsets, fetching the word of
// the offset it stands on with one cross-lane read (readlane), instead of doing a table look-up,
// field extraction, sign extension and bit-buffer refill per symbol on the scalar ALU.
// Codes longer than 8 bits are left unresolved (word 0) and decoded on the spot if the chain
// really lands on them.  The window is 96 bits of stream (w0,w1,w2): offsets 0..63 each with
// 32 bits of look-ahead; two more words are always already loaded.
//
// packed word: value (16 bits, signed) << 16 | kSymCoef | kSymEob | total bits (6) << 8 | kSymSpecial | advance (7 bits)
// (see pack_symbol).  Offsets whose code the lanes cannot resolve carry kSymMiss, a word that makes the serial
// part leave its straight line exactly as an end of band does, so that the common path tests nothing extra.
// ---------------------------------------------------------------------------------------
PCR_HD uint32_t bits_at(uint32_t w0, uint32_t w1, uint32_t w2, int j) {      // 32 bits from offset j (0..63)
    const uint32_t hi = j < 32 ? w0 : w1, lo = j < 32 ? w1 : w2;
    return (uint32_t)((((((uint64_t)hi) << 32) | lo) << (j & 31)) >> 32);
}

// e: table entry (length << 8 | symbol), non-zero.  first: AC first scan (size s = s value bits,
// sign-extended here); otherwise refinement (size 1 = one sign bit).  An end-of-band symbol
// (size 0, run r < 15) is followed by r bits of run length in both.
//
// The low 7 bits are how far the symbol moves the decoder on, counted to the position AFTER the one it
// lands on: run + 1 for a coefficient and for sixteen zeros, 65 + run ("past everything") for an end of
// band.  AC first scans add it to the position in the band, refinement scans to the index into the
// block's zero table.  kSymSpecial marks the words the straight line of a decoder cannot finish by itself:
//   kSymMiss   no code of <= 8 bits starts here (a longer code, or no code at all): length 0, advance 127;
//   in a refinement scan, sixteen zeros: it lands on a zero WITHOUT taking it, so it is given the advance
//   of an end of band (80) and redone by hand;
//   kSymInvalid  no code at all (or one that cannot occur in the scan): flags the stream as damaged.
constexpr uint32_t kSymCoef = 0x8000u, kSymEob = 0x4000u, kSymSpecial = 0x80u;
constexpr uint32_t kSymMiss = kSymSpecial | 127u;
constexpr uint32_t kSymInvalid = kSymEob | kSymSpecial | 65u;   // what the AC decoders see where no code matches: an "end of band" of
                                                             // length 0, marked special so that only the by-hand paths need to know it
constexpr uint32_t kZrlAdvance = 16;

PCR_HD uint32_t pack_symbol(uint32_t e, uint32_t win, bool first) {
    const int len = (int)(e >> 8), r = (int)((e >> 4) & 15), s = (int)(e & 15);
    const int nx = s ? (first ? s : 1) : (r != 15 ? r : 0);
    const uint32_t extra = field(win, len, nx);
    const int value = (first && s) ? extend(extra, s) : (int)extra;
    // bit 15: the symbol carries a coefficient; bit 14: it is an end-of-band symbol
    const uint32_t flags = (s ? kSymCoef : 0u) | ((s == 0 && r != 15) ? kSymEob : 0u);
    if (!first && s > 1) return kSymInvalid;                 // sizes above 1 do not exist in a refinement scan
    uint32_t adv = (uint32_t)r + 1u;
    if (flags & kSymEob) adv += 64u;
    else if (!first && s == 0) adv = kSymSpecial | (64u + kZrlAdvance);
    return ((uint32_t)(value & 0xFFFF) << 16) | flags | ((uint32_t)(len + nx) << 8) | adv;
}

// Pre-packed table entry for a symbol whose code has `len` bits: the low 16 bits are those of the packed
// word (advance, total bits, flags), bits 16..20 the code length and bits 21..24 the number of appended
// bits, which finish_packed() replaces by the appended value.  "Not in this table" is kSymMiss.
PCR_HD uint32_t packed_entry(uint32_t e, bool first) {
    if (e == 0) return kSymMiss;
    const uint32_t low = pack_symbol(e, 0, first) & 0xFFFFu;
    if (low == kSymInvalid) return kSymInvalid;               // (no appended bits: finish_packed leaves it alone)
    const uint32_t len = e >> 8, r = (e >> 4) & 15, s = e & 15;
    const uint32_t nx = s ? (first ? s : 1u) : (r != 15 ? r : 0u);
    return low | (len << 16) | (nx << 21);
}
PCR_HD uint32_t finish_packed(uint32_t p, uint32_t win, bool first) {
    const uint32_t len = (p >> 16) & 31, nx = (p >> 21) & 15;
    uint32_t x = ((win << len) >> 1) >> (31 - nx);            // the nx bits after the code (nx = 0: none)
    if (first && (p & kSymCoef)) x = (uint32_t)extend(x, (int)nx) & 0xFFFFu;
    return (p & 0xFFFFu) | (x << 16);
}
// fills lutp from lut: entry i by lane (i mod nlanes); call with every lane of the workgroup, after lut is complete
PCR_HD void actab_pack(AcTab* t, bool first, uint32_t lane, uint32_t nlanes) {
    for (uint32_t i = lane; i < 256; i += nlanes) t->lutp[i] = packed_entry(t->lut[i], first);
}

// packed DC word: difference (16 bits, signed) << 16 | total bits (6) << 8 | category (4)
PCR_HD uint32_t pack_dc(uint32_t e, uint32_t win) {          // e = (length << 4) | category, non-zero
    const int len = (int)(e >> 4), t = (int)(e & 15);
    const int diff = extend(field(win, len, t), t);
    return ((uint32_t)(diff & 0xFFFF) << 16) | ((uint32_t)(len + t) << 8) | (uint32_t)t;
}

// v[lane] = value, lane and value the same in every lane (the lane select travels in m0: a vector instruction of
// this chip reads at most one scalar register besides it)
#if defined(__HIP_DEVICE_COMPILE__)
__device__ inline void write_lane(uint32_t& v, uint32_t value, uint32_t lane) {
    asm volatile("s_mov_b32 m0, %2\n\tv_writelane_b32 %0, %1, m0" : "+v"(v) : "s"(value), "s"(lane) : "m0");
}
#endif

struct WindowReader {
    StreamPtr p;                // words after n1
    const AcTab* tab;
    uint32_t w0, w1, w2, n0, n1;
    uint32_t o;                 // offset of the next unread bit inside the window (may run past 63 until normalised)
    uint32_t wbase;             // bits of the stream before the window
    uint32_t mis_bits, total_bits;
    uint32_t lane;              // this lane's offset (device); unused on the host
    uint32_t vinfo;             // this lane's packed word (device)
    const uint32_t* g;          // p again, for the vector memory path
    uint32_t vnext;             // device: even lanes p[0], odd lanes p[1], fetched one window ahead (see slide)
    bool first;
    bool vfeed;                 // fetch the stream through the vector memory path (see fetch_next)

    // The unit starts sub_bits (0..7) bits into byte byte_off of the segment and holds nbits bits counted from that
    // byte's first bit; pos0: what position() reports for the byte's first bit (0: positions relative to the unit's
    // first byte, as for restart intervals; byte_off * 8: positions in the scan, as for units that start at entry points).
    PCR_HD void init(const uint32_t* words, uint32_t byte_off, uint32_t sub_bits, uint32_t nbits, uint32_t pos0, const AcTab* t, bool first_scan,
                     uint32_t lane_id, bool vector_feed) {
        tab = t; first = first_scan; lane = lane_id; vfeed = vector_feed;
        mis_bits = (byte_off & 3) * 8;
        p = stream_ptr(words + (byte_off >> 2));
        w0 = p[0]; w1 = p[1]; w2 = p[2]; n0 = p[3]; n1 = p[4]; p += 5;
        g = words + (byte_off >> 2) + 5;
        o = mis_bits + sub_bits; wbase = pos0; total_bits = pos0 + nbits + mis_bits;
        vnext = 0;
        fetch_next();
        fill();
    }
    // With vfeed the two words after n1 are fetched by the vector unit, one per lane parity, although they are the
    // same for all lanes: a scalar load is waited for together with the LDS look-up that follows it in fill()
    // (scalar loads and LDS share a counter and scalar loads return out of order), a window before it is needed.
    // A decoder that keeps other vector loads in flight (the refinement history) is better off with the scalar
    // load: the vector counter is in order, and the wait for these words would take the younger loads with it.
    PCR_HD void fetch_next() {
#if defined(__HIP_DEVICE_COMPILE__)
        if (vfeed) vnext = g[lane & 1];
#endif
    }
    PCR_HD void slide() {                                     // on by 64 bits
        w0 = w2; w1 = n0; w2 = n1;
#if defined(__HIP_DEVICE_COMPILE__)
        if (vfeed) { n0 = (uint32_t)__builtin_amdgcn_readlane((int)vnext, 0); n1 = (uint32_t)__builtin_amdgcn_readlane((int)vnext, 1); }
        else { n0 = p[0]; n1 = p[1]; }
#else
        n0 = p[0]; n1 = p[1];
#endif
        p += 2; g += 2; o -= 64; wbase += 64;
        fetch_next();
    }
    PCR_HD void fill() {
#if defined(__HIP_DEVICE_COMPILE__)
        const uint32_t win = bits_at(w0, w1, w2, (int)lane);
        vinfo = finish_packed(tab->lutp[win >> 24], win, first);
#endif
    }
    // packed word of the offset `off` of the window (0..63); kSymMiss where no short code starts
    PCR_HD uint32_t lookup(uint32_t off) const {
#if defined(__HIP_DEVICE_COMPILE__)
        return (uint32_t)__builtin_amdgcn_readlane((int)vinfo, (int)off);
#else
        const uint32_t win = bits_at(w0, w1, w2, (int)off);
        return finish_packed(tab->lutp[win >> 24], win, first);
#endif
    }
    // the same for an offset that lookup() answered with kSymMiss: a code longer than 8 bits, or garbage
    PCR_HD uint32_t resolve(uint32_t off) const {
        const uint32_t win = bits_at(w0, w1, w2, (int)off);
        const uint32_t e = ac_long_code(tab, win);
        return uni(e ? pack_symbol(e, win, first) : kSymInvalid);
    }
    PCR_HD bool exhausted() const { return o >= 64; }         // the next symbol starts beyond the window
    PCR_HD void refill() {
        do slide(); while (o >= 64);
        fill();
    }
    // Sequential scans switch tables between blocks: the words of the current window are looked up again.
    PCR_HD void use_table(const AcTab* t) { tab = t; fill(); }
    // Sequential scans: packed DC word (pack_dc) of the symbol at the current position, decoded on the spot;
    // 0 where the bits are no code of the table.
    PCR_HD uint32_t dc_word(const DcTab* t) const {
        const uint32_t win = bits_at(w0, w1, w2, (int)o);
        const uint32_t e = dc_code(t, win);
        return uni(e ? pack_dc(e, win) : 0u);                 // (table reads come back in vector registers)
    }
    // refill() that returns the lanes' words of the window being left (device; 0 on the host)
    PCR_HD uint32_t refill_keep() {
        const uint32_t old = vinfo;
        refill();
        return old;
    }
    // replaces the word of offset `off` (a symbol the serial part resolved by hand)
    PCR_HD void set_word(uint32_t off, uint32_t word) {
#if defined(__HIP_DEVICE_COMPILE__)
        write_lane(vinfo, word, off);
#else
        (void)off; (void)word;
#endif
    }
    PCR_HD void consume(uint32_t n) { o += n; }
    PCR_HD uint32_t position() const { return wbase + o - mis_bits; }       // bits consumed since the unit's first bit
    PCR_HD bool overrun() const { return wbase + o > total_bits; }
    PCR_HD uint32_t overrun_bit() const { return (total_bits - (wbase + o)) >> 31; }   // the same as 0 / 1, without a compare (streams are < 2^31 bits)
};

// Per-lane parameters of the unit being decoded (all in registers).
struct LaneScan {
    uint32_t mcu0, mcu1;        // MCU range [mcu0, mcu1) of the scan handled by this unit
    uint32_t mcu_w;             // MCUs per row of the scan
    int Ss, Se, Al;
    // interleaved DC scans: per scan component j
    int ns;
    uint32_t hs[kMaxComp], vs[kMaxComp], bw[kMaxComp];
    uint32_t poff[kMaxComp];   // element offset of each scan component's plane inside the image's coefficient buffer
    int pred[kMaxComp];        // DC predictions at the unit's first MCU (0 after a restart marker; an entry point brings its own)
};

// ---------------------------------------------------------------------------------------
// CoefSink: keeps memory off the serial path.  Every symbol the serial part passes goes, as (element
// index, packed word with the value in its top 16 bits), into two vector registers, in the lane whose
// number is the window offset the symbol STARTS at: symbols that start inside one window start at
// different offsets, so no counter is needed.  Each time the bit window slides the lanes whose word
// carries kSymCoef store their value, and all words are cleared.  Words without kSymCoef (an end of
// band, sixteen zeros, an unresolved code) are written too and simply never stored.  The element
// index is checked against the plane's size by the lanes, so the serial part need not clamp what a
// damaged stream makes of it.
// ---------------------------------------------------------------------------------------
struct CoefSink {
    int16_t* plane;                                           // may be null if `dense` is given: then only that copy is written
    int16_t* dense;                                           // optional second copy, one value per block: dense[element index / 64]
    uint32_t limit;                                           // elements of `plane`
    int Al;                                                   // values are stored shifted left by this
    uint32_t vidx; int vval;                                  // device: this lane's pending pair
    PCR_HD void init(int16_t* p, uint32_t elems, int al, int16_t* per_block = nullptr) { plane = p; dense = per_block; limit = elems; Al = al; vidx = 0; vval = 0; }
    // slot: window offset the symbol starts at (0..63); word: packed symbol word
    PCR_HD void emit(uint32_t slot, uint32_t elem, int word) {
#if defined(__HIP_DEVICE_COMPILE__)
        // (the lane select travels in m0: a vector instruction of this chip reads at most one scalar
        // register besides it)
        asm volatile("s_mov_b32 m0, %4\n\tv_writelane_b32 %0, %2, m0\n\tv_writelane_b32 %1, %3, m0"
                     : "+v"(vidx), "+v"(vval) : "s"(elem), "s"(word), "s"(slot) : "m0");
#else
        (void)slot;
        if (((uint32_t)word & kSymCoef) && elem < limit) { const int16_t val = (int16_t)((word >> 16) * (1 << Al)); if (plane) plane[elem] = val; if (dense) dense[elem >> 6] = val; }
#endif
    }
    PCR_HD void flush() {
#if defined(__HIP_DEVICE_COMPILE__)
        if (((uint32_t)vval & kSymCoef) && vidx < limit) {
            const int16_t val = (int16_t)((vval >> 16) * (1 << Al));
            if (plane) plane[vidx] = val;
            if (dense) dense[vidx >> 6] = val;
        }
        vval = 0;
#endif
    }
};

// IndexSink: the same for the AC first scan, with one register instead of two.  The lane of a window offset
// already holds the packed word of the symbol that starts there (the reader's look-up), so all the serial
// part has to leave in that lane is the element index; a lane stores if it was given an index and its word
// carries a coefficient.  A symbol the serial part resolved by hand is written back into the reader's words.
struct IndexSink {
    int16_t* plane;
    int16_t* dense;                                           // sequential scans: the compact copy of the DC coefficients, dense[element index / 64]
    uint32_t limit;
    int Al;
    uint32_t vidx;                                            // device: this lane's element index, ~0 = none
    PCR_HD void init(int16_t* p, uint32_t elems, int al, int16_t* per_block = nullptr) { plane = p; dense = per_block; limit = elems; Al = al; vidx = ~0u; }
    // host build: store at once (there are no lanes to hold anything back)
    PCR_HD void store_now(uint32_t elem, uint32_t word) {
        if ((word & kSymCoef) && elem < limit) {
            plane[elem] = (int16_t)(((int32_t)word >> 16) * (1 << Al));
            if (dense && (elem & 63) == 0) dense[elem >> 6] = plane[elem];
        }
    }
    // words: the lanes' packed words of the window the indices belong to
    PCR_HD void flush(uint32_t words) {
#if defined(__HIP_DEVICE_COMPILE__)
        if ((words & kSymCoef) && vidx < limit) plane[vidx] = (int16_t)(((int32_t)words >> 16) * (1 << Al));
        vidx = ~0u;
#else
        (void)words;
#endif
    }
    // the same for scans that also carry DC coefficients (element 0 of a block goes to the compact copy as well)
    PCR_HD void flush_with_dc(uint32_t words) {
#if defined(__HIP_DEVICE_COMPILE__)
        if ((words & kSymCoef) && vidx < limit) {
            const int16_t val = (int16_t)(((int32_t)words >> 16) * (1 << Al));
            plane[vidx] = val;
            if ((vidx & 63) == 0) dense[vidx >> 6] = val;
        }
        vidx = ~0u;
#else
        (void)words;
#endif
    }
};

// ---------------------------------------------------------------------------------------
// Window reader for DC first scans: as WindowReader, but an interleaved scan switches between the
// DC tables of its components, so every lane looks its offset up in the table of each scan
// component (once per distinct table) and the serial part picks the word of the component whose
// block it is decoding.  Everything is indexed by scan component with constants: a run-time index
// into the reader would pin it to memory.
// packed word: difference (16 bits, signed) << 16 | total bits (6) << 8 | category (4)
// ---------------------------------------------------------------------------------------

struct DcWindowReader {
    StreamPtr p;
    const DcTab* tab[kMaxComp];     // table of scan component j
    uint32_t w0, w1, w2, n0, n1;
    uint32_t o, wbase, mis_bits, total_bits, lane;
    uint32_t vinfo[kMaxComp];       // this lane's packed word under the table of scan component j
    uint32_t nocode;                // set when the bits at the current position are no code of the table
    int ncomp;
    const uint32_t* g;              // p again, for the vector memory path (as in WindowReader)
    uint32_t vnext;

    PCR_HD void init(const uint32_t* words, uint32_t byte_off, uint32_t sub_bits, uint32_t nbits, const DcTab* t0, const DcTab* t1, const DcTab* t2,
                     int ncomponents, uint32_t lane_id) {                  // (byte_off, sub_bits, nbits: as WindowReader::init)
        tab[0] = t0; tab[1] = t1; tab[2] = t2; ncomp = ncomponents; lane = lane_id;
        mis_bits = (byte_off & 3) * 8;
        p = stream_ptr(words + (byte_off >> 2));
        w0 = p[0]; w1 = p[1]; w2 = p[2]; n0 = p[3]; n1 = p[4]; p += 5;
        g = words + (byte_off >> 2) + 5;
        o = mis_bits + sub_bits; wbase = 0; total_bits = nbits + mis_bits; nocode = 0;
        vinfo[0] = vinfo[1] = vinfo[2] = 0;
        fetch_next();
        fill();
    }
    PCR_HD void fetch_next() {
#if defined(__HIP_DEVICE_COMPILE__)
        vnext = g[lane & 1];
#endif
    }
    PCR_HD void slide() {                                     // on by 64 bits
        w0 = w2; w1 = n0; w2 = n1;
#if defined(__HIP_DEVICE_COMPILE__)
        n0 = (uint32_t)__builtin_amdgcn_readlane((int)vnext, 0); n1 = (uint32_t)__builtin_amdgcn_readlane((int)vnext, 1);
#else
        n0 = p[0]; n1 = p[1];
#endif
        p += 2; g += 2; o -= 64; wbase += 64;
        fetch_next();
    }
    PCR_HD uint32_t word_of(const DcTab* t, uint32_t win) const { const uint32_t e = t->lut[win >> 24]; return e != 0xFF ? pack_dc(e, win) : 0; }
    PCR_HD void fill() {
#if defined(__HIP_DEVICE_COMPILE__)
        const uint32_t win = bits_at(w0, w1, w2, (int)lane);
        vinfo[0] = word_of(tab[0], win);
        if (ncomp > 1) vinfo[1] = tab[1] == tab[0] ? vinfo[0] : word_of(tab[1], win);
        if (ncomp > 2) vinfo[2] = tab[2] == tab[1] ? vinfo[1] : (tab[2] == tab[0] ? vinfo[0] : word_of(tab[2], win));
#endif
    }
    PCR_HD bool exhausted() const { return o >= 64; }
    PCR_HD void refill() {
        do slide(); while (o >= 64);
        fill();
    }
    // packed word of the symbol at the current position (inside the window) for scan component J; where the bits
    // are no code at all it returns 0 (length 0, difference 0) and raises `nocode`
    template <int J> PCR_HD uint32_t peek() {
        uint32_t info;
#if defined(__HIP_DEVICE_COMPILE__)
        info = (uint32_t)__builtin_amdgcn_readlane((int)vinfo[J], (int)o);
#else
        info = word_of(tab[J], bits_at(w0, w1, w2, (int)o));
#endif
        if (__builtin_expect(info == 0, 0)) {                // a code longer than 8 bits, or garbage
            const uint32_t win = bits_at(w0, w1, w2, (int)o);
            const uint32_t e = dc_code(tab[J], win);
            info = uni(e ? pack_dc(e, win) : 0u);            // (table reads come back in vector registers)
            nocode |= uni(e ? 0u : 1u);
        }
        return info;
    }
    PCR_HD void consume(uint32_t n) { o += n; }
    PCR_HD uint32_t overrun_bit() const { return (total_bits - (wbase + o)) >> 31; }
};

// ---------------------------------------------------------------------------------------
// DC first scan.  Non-interleaved scans visit the blocks covering the component's own
// samples, interleaved scans the MCU-padded grid, component by component inside each MCU.
// The sink's plane is the image's coefficient buffer; ls.poff[j] locates the plane of scan component j
// in it ([bh][bw][64] blocks, DC at element 0 of each block).  tj0/1/2: which of the reader's tables each
// scan component uses.
// ---------------------------------------------------------------------------------------
// One DC symbol of scan component J for the block at element e.
template <int J>
PCR_HD void dc_first_block(DcWindowReader* wr, CoefSink* sink, int* pred, uint32_t e, uint32_t* bad) {
    if (wr->exhausted()) {
        *bad |= wr->overrun_bit();                           // never walk far beyond the unit's data
        wr->refill();                                        // (before the flush: the wait for the words fetched a window ago must not include these stores)
        sink->flush();
    }
    const uint32_t info = wr->peek<J>();
    *pred += (int32_t)info >> 16;
    sink->emit(wr->o, e, (int)(((uint32_t)*pred << 16) | kSymCoef));
    wr->consume((info >> 8) & 63);
}

// The common shapes with everything about the MCU known at compile time: NS components, the first one
// HS0 x VS0 blocks per MCU, the others one block (a non-interleaved scan is NS = 1, one block per "MCU" and
// only the blocks that cover the component's samples).  Element indices run along instead of being
// recomputed per MCU.
template <int NS, int HS0, int VS0>
PCR_HD int decode_dc_first_shape(DcWindowReader* wr, const LaneScan& ls, CoefSink* sink) {
    int pred0 = ls.pred[0], pred1 = ls.pred[1], pred2 = ls.pred[2];
    const uint32_t mcu_w = ls.mcu_w;
    const uint32_t my0 = ls.mcu0 / mcu_w;
    uint32_t mx = ls.mcu0 % mcu_w;
    const uint32_t bw0 = ls.bw[0];
    uint32_t e0 = ls.poff[0] + ((my0 * VS0) * bw0 + mx * HS0) * 64;
    uint32_t e1 = NS > 1 ? ls.poff[1] + (my0 * ls.bw[1] + mx) * 64 : 0;
    uint32_t e2 = NS > 2 ? ls.poff[2] + (my0 * ls.bw[2] + mx) * 64 : 0;
    // at the end of a row of MCUs: on to the first block of the next row of MCUs
    const uint32_t wrap0 = (VS0 * bw0 - mcu_w * HS0) * 64;
    const uint32_t wrap1 = NS > 1 ? (ls.bw[1] - mcu_w) * 64 : 0, wrap2 = NS > 2 ? (ls.bw[2] - mcu_w) * 64 : 0;
    uint32_t bad = 0;
    uint32_t left = ls.mcu1 - ls.mcu0;
    while (left != 0) {
#pragma unroll
        for (int by = 0; by < VS0; by++) {
#pragma unroll
            for (int bx = 0; bx < HS0; bx++) dc_first_block<0>(wr, sink, &pred0, e0 + (by * bw0 + bx) * 64, &bad);
        }
        if (NS > 1) dc_first_block<1>(wr, sink, &pred1, e1, &bad);
        if (NS > 2) dc_first_block<2>(wr, sink, &pred2, e2, &bad);
        bad |= wr->nocode;
        e0 += HS0 * 64; e1 += 64; e2 += 64;
        if (++mx == mcu_w) { mx = 0; e0 += wrap0; e1 += wrap1; e2 += wrap2; }
        left = bad ? 0 : left - 1;
    }
    sink->flush();
    bad |= wr->overrun_bit();
    return bad ? kEFormat : kOk;
}

// Any other shape.
template <int J>
PCR_HD void dc_first_component(DcWindowReader* wr, const LaneScan& ls, CoefSink* sink, uint32_t mx, uint32_t my, int* pred, uint32_t* bad) {
    const uint32_t hs = ls.ns > 1 ? ls.hs[J] : 1, vs = ls.ns > 1 ? ls.vs[J] : 1, bw = ls.bw[J];
    uint32_t rowe = ls.poff[J] + ((my * vs) * bw + mx * hs) * 64;       // first block of this MCU in the plane
    for (uint32_t by = 0; by < vs; by++) {
        uint32_t e = rowe;
        for (uint32_t bx = 0; bx < hs; bx++) { dc_first_block<J>(wr, sink, pred, e, bad); e += 64; }
        rowe += bw * 64;
    }
}
PCR_HD int decode_dc_first_any(DcWindowReader* wr, const LaneScan& ls, CoefSink* sink) {
    int pred0 = ls.pred[0], pred1 = ls.pred[1], pred2 = ls.pred[2];
    uint32_t my = ls.mcu0 / ls.mcu_w, mx = ls.mcu0 % ls.mcu_w;
    uint32_t bad = 0;
    uint32_t m = ls.mcu0;
    while (m < ls.mcu1) {
        dc_first_component<0>(wr, ls, sink, mx, my, &pred0, &bad);
        if (ls.ns > 1) dc_first_component<1>(wr, ls, sink, mx, my, &pred1, &bad);
        if (ls.ns > 2) dc_first_component<2>(wr, ls, sink, mx, my, &pred2, &bad);
        bad |= wr->nocode;
        if (++mx == ls.mcu_w) { mx = 0; my++; }
        m = bad ? ls.mcu1 : m + 1;
    }
    sink->flush();
    bad |= wr->overrun_bit();
    return bad ? kEFormat : kOk;
}

// Which of the decoders above fits a scan: 0 = decode_dc_first_any, else an instance of decode_dc_first_shape
// (kDcShapes of them).  ns: components of the scan; hs, vs: their sampling factors in scan order (passed one by
// one: an array argument would pin the caller's copy of them to memory).
constexpr int kDcShapes = 5;
PCR_HD int dc_shape(int ns, uint32_t hs0, uint32_t vs0, uint32_t hs1, uint32_t vs1, uint32_t hs2, uint32_t vs2) {
    if (ns == 1) return 1;
    if (ns == 3 && hs1 == 1 && vs1 == 1 && hs2 == 1 && vs2 == 1) {
        if (hs0 == 2 && vs0 == 2) return 2;
        if (hs0 == 1 && vs0 == 1) return 3;
        if (hs0 == 2 && vs0 == 1) return 4;
    }
    return 0;
}
template <int SHAPE>
PCR_HD int decode_dc_first_as(DcWindowReader* wr, const LaneScan& ls, CoefSink* sink) {
    if (SHAPE == 1) return decode_dc_first_shape<1, 1, 1>(wr, ls, sink);
    if (SHAPE == 2) return decode_dc_first_shape<3, 2, 2>(wr, ls, sink);
    if (SHAPE == 3) return decode_dc_first_shape<3, 1, 1>(wr, ls, sink);
    if (SHAPE == 4) return decode_dc_first_shape<3, 2, 1>(wr, ls, sink);
    return decode_dc_first_any(wr, ls, sink);
}
PCR_HD int decode_dc_first(DcWindowReader* wr, const LaneScan& ls, CoefSink* sink) {
    switch (dc_shape(ls.ns, ls.hs[0], ls.vs[0], ls.hs[1], ls.vs[1], ls.hs[2], ls.vs[2])) {
        case 1: return decode_dc_first_as<1>(wr, ls, sink);
        case 2: return decode_dc_first_as<2>(wr, ls, sink);
        case 3: return decode_dc_first_as<3>(wr, ls, sink);
        case 4: return decode_dc_first_as<4>(wr, ls, sink);
        default: return decode_dc_first_as<0>(wr, ls, sink);
    }
}

// ---------------------------------------------------------------------------------------
// AC first scan of one component, band Ss..Se.  Writes coefficient values in ZIG-ZAG order
// inside each 64-element block (element k of a block is zig-zag position k).  Blocks skipped by
// an end-of-band run are not touched: coefficients must be zero-filled beforehand.
//
// The serial part handles one symbol per loop iteration and does no memory access: a decoded
// coefficient goes, as (element index, value), into the next free lane of two vector registers
// (CoefSink), and the lanes store them all at once each time the bit window slides.  A window
// of 64 bits holds at most 32 coefficient symbols (each is at least 2 bits long), so the 64
// lanes always suffice.  Control flow is structured -- flags and loop conditions instead of
// returns and breaks -- because the compiler turns early exits from nested loops into a state
// variable that is tested after every symbol.
// ---------------------------------------------------------------------------------------
// Non-zero mask of the band Ss..Se of one block in internal (zig-zag) order: what an AC first
// scan over that band has made non-zero.
PCR_HD uint64_t nz_mask_of_block(const int16_t* blk, int Ss, int Se) {
    uint64_t m = 0;
    for (int k = Ss; k <= Se; k++) m |= (uint64_t)(blk[k] != 0) << k;
    return m;
}

// Leaves element `elem` in the sink's lane `slot` (device), or stores the word's coefficient there at once (host).
PCR_HD void sink_index(IndexSink* sink, uint32_t slot, uint32_t elem, uint32_t word) {
#if defined(__HIP_DEVICE_COMPILE__)
    (void)word;
    write_lane(sink->vidx, elem, slot);
#else
    (void)slot;
    sink->store_now(elem, word);
#endif
}

// The symbols that start inside the current window, one straight line each: a coefficient (run r, then the
// value) and sixteen zeros (r = 15) both move on by r + 1; an end of band and an unresolved code move "past
// everything".  Every symbol leaves the element it landed on in the sink's lane of its offset.  On the device
// the loop is written out by hand: the window offset lives in m0, which is what selects the lane for the
// cross-lane read and write, so that no instruction is spent on moving it there (ten instructions per
// symbol: seven scalar, two cross-lane, the branch; 48 bytes, placed on one 64-byte line of the instruction
// cache: a lone wavefront runs a short loop visibly faster when it does not straddle lines, 10 % here).
// Returns the word of the last symbol.
PCR_HD uint32_t ac_first_symbols(WindowReader* wr, IndexSink* sink, uint32_t* kb_io, uint32_t base_b, uint32_t adv_mask, uint32_t tot_field) {
    uint32_t info, kb = *kb_io, o = wr->o;
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t t0, t1;
    asm volatile(
        "s_mov_b32 m0, %[o]\n\t"
        "s_branch 1f\n\t"                                     // (over the padding)
        ".p2align 6\n"
        "1:\n\t"
        "v_readlane_b32 %[info], %[vinfo], m0\n\t"
        "s_and_b32 %[t0], %[info], %[advm]\n\t"
        "s_bfe_u32 %[t1], %[info], %[totf]\n\t"
        "s_add_i32 %[kb], %[kb], %[t0]\n\t"
        "s_add_i32 %[t0], %[kb], %[base]\n\t"
        "v_writelane_b32 %[vidx], %[t0], m0\n\t"
        "s_add_i32 m0, m0, %[t1]\n\t"
        "s_or_b32 %[t0], m0, %[kb]\n\t"
        "s_cmp_lt_u32 %[t0], 64\n\t"
        "s_cbranch_scc1 1b\n\t"
        "s_mov_b32 %[o], m0"
        : [info] "=&s"(info), [t0] "=&s"(t0), [t1] "=&s"(t1), [kb] "+s"(kb), [vidx] "+v"(sink->vidx), [o] "+s"(o)
        : [vinfo] "v"(wr->vinfo), [base] "s"(base_b), [advm] "s"(adv_mask), [totf] "s"(tot_field)
        : "m0", "scc");
#else
    do {
        info = wr->lookup(o);
        kb += info & adv_mask;
        sink->store_now(base_b + kb, info);
        o += bit_field(info, tot_field);
    } while ((kb | o) < 64);
#endif
    wr->o = o; *kb_io = kb;
    return info;
}

PCR_HD int decode_ac_first(WindowReader* wr, const LaneScan& ls, IndexSink* sink) {
    const uint32_t Ss = (uint32_t)ls.Ss, Se = (uint32_t)ls.Se;
    const uint32_t bw = ls.bw[0], mcu_w = ls.mcu_w;
    // Positions are kept biased: kb = (zig-zag position of the next candidate) + bias with bias = 63 - Se,
    // so that "the band is complete" reads kb >= 64 whatever Se is, the same bit that says "the window
    // is used up" in the window offset.  After a symbol's advance (run + 1) kb is one past the position
    // it landed on; base_b = element index of the block - bias - 1 makes base_b + kb that element.
    const uint32_t bias = 63 - Se;
    uint32_t left = ls.mcu1 - ls.mcu0;                       // blocks of the unit not finished yet (the current one included)
    uint32_t col = ls.mcu0 % mcu_w;
    uint32_t base_b = ((ls.mcu0 / mcu_w) * bw + col) * 64 - bias - 1;
    const uint32_t row_skip = (bw - mcu_w) * 64;             // elements of the padded grid between two rows of the scan
    uint32_t kb = Ss + bias;
    uint32_t bad = 0;
    const uint32_t adv_mask = opaque(127u), tot_field = opaque((6u << 16) | 8u);
    while (left != 0) {
        if (wr->exhausted()) {
            bad |= wr->overrun_bit();                        // never walk far beyond the unit's data
            const uint32_t words = wr->refill_keep();        // (before the flush: the wait for the words fetched a window ago must not include these stores)
            sink->flush(words);
        }
        uint32_t info = opaque(ac_first_symbols(wr, sink, &kb, base_b, adv_mask, tot_field));   // (a scalar: tested on the scalar unit)
        if (kb >= 64) {                                      // the block is finished, or the lanes left the code to us
            if (info & kSymSpecial) {                        // a code longer than 8 bits (or none): the same step by hand
                kb -= kSymMiss & 127;
                info = wr->resolve(wr->o);
                if (info == kSymInvalid) bad |= 1u;          // no code at all
                kb += info & 127;
                wr->set_word(wr->o, info);                   // (the index left in this lane a moment ago is replaced too)
                sink_index(sink, wr->o, base_b + kb, info);
                wr->consume((info >> 8) & 63);
            }
            if (kb >= 64) {                                  // band complete, or end of band
                uint32_t adv = 1;                            // blocks to move on by
                if (info & kSymEob) {                        // run of 2^r + extra blocks
                    adv = (1u << ((info & 127) - 65)) + (info >> 16);
                } else {
                    bad |= ((64u - kb) >> 31) & (info >> 15);   // a coefficient beyond the band (kb > 64)
                }
                adv = adv < left ? adv : left;
                left = bad ? 0 : left - adv;                 // stop at the first damaged block
                col += adv; base_b += adv * 64; kb = Ss + bias;
                while (col >= mcu_w) { col -= mcu_w; base_b += row_skip; }
            }
        }
    }
    sink->flush(wr->vinfo);
    bad |= wr->overrun_bit();
    return bad ? kEFormat : kOk;
}

// ---------------------------------------------------------------------------------------
// Sequential (baseline) scan: every block is a DC difference followed by AC run/size pairs up to an end of
// block, the blocks of the components interleaved MCU by MCU (or one component alone).  It is read with the
// AC first scan's reader and symbol loop over the band 1..63: the lanes hold the packed AC word of every
// window offset under ONE table, that of the component being decoded; when the next block belongs to a
// component with another AC table the words of the current window are looked up again (twice per MCU of a
// colour image).  The DC symbol, one per block, is decoded by hand at its position and its word (the running
// DC value) put into the lane of its offset like any other coefficient.
// ---------------------------------------------------------------------------------------
// Tables of the scan's components (pointers into LDS on the device).
struct SeqTables { const DcTab* dc[kMaxComp]; const AcTab* ac[kMaxComp]; };

// One block at element e (its DC), coefficients in zig-zag order behind it.
PCR_HD void sequential_block(WindowReader* wr, IndexSink* sink, const DcTab* dt, const AcTab* at, int* pred, uint32_t e, uint32_t* bad,
                             uint32_t adv_mask, uint32_t tot_field) {
    if (wr->exhausted()) {
        *bad |= wr->overrun_bit();
        const uint32_t words = wr->refill_keep();
        sink->flush_with_dc(words);
    }
    if (at != wr->tab) {                                     // (what the lanes still hold goes out before their words change)
        sink->flush_with_dc(wr->vinfo);
        wr->use_table(at);
    }
    uint32_t info = wr->dc_word(dt);
    if (info == 0) *bad |= 1u;                               // no code at all
    *pred += (int32_t)info >> 16;
    const uint32_t dcw = ((uint32_t)*pred << 16) | kSymCoef;
    wr->set_word(wr->o, dcw);
    sink_index(sink, wr->o, e, dcw);
    wr->consume((info >> 8) & 63);
    // kb: one past the zig-zag position the last symbol landed on (the band 1..63 needs no bias)
    uint32_t kb = 1;
    const uint32_t base_b = e - 1;
    while (kb < 64) {
        if (wr->exhausted()) {
            *bad |= wr->overrun_bit();
            const uint32_t words = wr->refill_keep();
            sink->flush_with_dc(words);
        }
        info = opaque(ac_first_symbols(wr, sink, &kb, base_b, adv_mask, tot_field));
        if (kb >= 64) {
            if (info & kSymSpecial) {                        // a code longer than 8 bits (or none): the same step by hand
                kb -= kSymMiss & 127;
                info = wr->resolve(wr->o);
                if (info == kSymInvalid) *bad |= 1u;
                kb += info & 127u;
                wr->set_word(wr->o, info);
                sink_index(sink, wr->o, base_b + kb, info);
                wr->consume((info >> 8) & 63);
            }
            if (kb >= 64) {
                if (info & kSymEob) *bad |= ((info & 127u) != 65u) ? 1u : 0u;     // only the plain end of block exists here
                else *bad |= ((64u - kb) >> 31) & (info >> 15);                   // a coefficient beyond position 63
            }
        }
    }
}

template <int J>
PCR_HD void sequential_component(WindowReader* wr, const LaneScan& ls, const SeqTables& tb, IndexSink* sink, uint32_t mx, uint32_t my, int* pred,
                                 uint32_t* bad, uint32_t adv_mask, uint32_t tot_field) {
    const uint32_t hs = ls.ns > 1 ? ls.hs[J] : 1, vs = ls.ns > 1 ? ls.vs[J] : 1, bw = ls.bw[J];
    uint32_t rowe = ls.poff[J] + ((my * vs) * bw + mx * hs) * 64;
    for (uint32_t by = 0; by < vs; by++) {
        uint32_t e = rowe;
        for (uint32_t bx = 0; bx < hs; bx++) {
            if (!*bad) sequential_block(wr, sink, tb.dc[J], tb.ac[J], pred, e, bad, adv_mask, tot_field);      // (stop at the first damaged block)
            e += 64;
        }
        rowe += bw * 64;
    }
}

// The sink's plane is the image's coefficient buffer; ls.poff[j] locates the plane of scan component j in it.
// The reader must have been initialised with tb.ac[0] as a first-scan reader.
PCR_HD int decode_sequential(WindowReader* wr, const LaneScan& ls, const SeqTables& tb, IndexSink* sink) {
    int pred0 = ls.pred[0], pred1 = ls.pred[1], pred2 = ls.pred[2];
    uint32_t my = ls.mcu0 / ls.mcu_w, mx = ls.mcu0 % ls.mcu_w;
    uint32_t bad = 0;
    uint32_t m = ls.mcu0;
    const uint32_t adv_mask = opaque(127u), tot_field = opaque((6u << 16) | 8u);
    while (m < ls.mcu1) {
        sequential_component<0>(wr, ls, tb, sink, mx, my, &pred0, &bad, adv_mask, tot_field);
        if (ls.ns > 1) sequential_component<1>(wr, ls, tb, sink, mx, my, &pred1, &bad, adv_mask, tot_field);
        if (ls.ns > 2) sequential_component<2>(wr, ls, tb, sink, mx, my, &pred2, &bad, adv_mask, tot_field);
        if (++mx == ls.mcu_w) { mx = 0; my++; }
        m = bad ? ls.mcu1 : m + 1;
    }
    sink->flush_with_dc(wr->vinfo);
    bad |= wr->overrun_bit();
    return bad ? kEFormat : kOk;
}

// ---------------------------------------------------------------------------------------
// AC refinement scan.  hist0..: masks written by the earlier AC scans of the
// component (nhist of them).  Per block this writes
//   nzout  positions that become non-zero in this scan,
//   sign   for those positions, 1 = positive,
//   cbits  the correction bits in reading order (first bit read = bit 0).
// ---------------------------------------------------------------------------------------
PCR_HD uint64_t band_mask(int Ss, int Se) { return ((Se >= 63) ? ~0ull : ((1ull << (Se + 1)) - 1)) & ~((1ull << Ss) - 1); }

// What an AC refinement scan leaves per block: one record of kRefWords 64-bit words (zig-zag bit order),
//   [kRefNz]    positions that become non-zero in this scan (later scans need them as history)   } written by phase 1
//   [kRefSign]  signs of the kRefNz positions, 1 = positive                                       } written by
//   [kRefPlus]  positions whose correction bit is 1 (their magnitude grows by 2^Al)              } phase 2
//   [kRefStart] bit offset of the block inside its unit | end-of-band run pending at its start << 32  } written by
//   [kRefHist]  positions of the band already non-zero when the scan starts                      } phase 1
// A scan keeps one array per word, each with one entry per block of the component's plane (word w of block b lies
// at w * blocks + b): every kernel that writes a word for consecutive blocks then writes whole lines (records of five
// words per block, of which a kernel writes two or three, were measured to cost 1.7 - 2.4 times the bytes in partial
// sectors); what the consumers of a finished scan need (the replay of the refinement on the coefficients) is the first
// three words.
constexpr int kRefNz = 0, kRefSign = 1, kRefPlus = 2, kRefStart = 3, kRefHist = 4, kRefWords = 5;
PCR_HD size_t ref_word(int w, size_t blk, size_t nblk) { return (size_t)w * nblk + blk; }

// History of a refinement scan: the positions of its band that are non-zero when it starts.  What the
// AC first scans made non-zero is read back from the coefficient plane (one coefficient per lane, a ballot
// of "!= 0"); what earlier refinement scans added is in the records they wrote (p[0..n): their record arrays).
struct HistPlanes { const int16_t* coef; const uint64_t* p[kMaxHist]; int n; };

struct HistWords {                                            // one block's history, combined only when used
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t half;                                            // even lanes: low half, odd lanes: high half of what earlier refinement scans added
    int16_t mine;                                             // this lane's coefficient of the block
#else
    uint64_t a, first;
#endif
};
// On the device the record word is fetched by the vector unit (every lane one half of it) although it is the
// same for all lanes: scalar loads return out of order, so a wait for any LDS result -- there is one ahead of
// every symbol loop -- would also wait for a scalar load issued just before it for two blocks later, and expose
// a trip to memory per block.  Vector loads return in order and have a counter of their own.
PCR_HD HistWords hist_fetch(const HistPlanes& hp, uint32_t blk, uint32_t lane) {
    HistWords w;
    static_assert(kRefNz == 0, "the words that become history are a scan's first array");
    const uint32_t off = blk * 8;                             // (32-bit offsets: a plane has far fewer than 2^29 blocks)
#if defined(__HIP_DEVICE_COMPILE__)
    w.half = 0;
    if (hp.n > 0) {
        const uint32_t sel = off + (lane & 1) * 4;
        w.half = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(hp.p[0]) + sel);
        if (__builtin_expect(hp.n > 1, 0)) {                 // scripts with more than two refinement passes over a band
            for (int q = 1; q < kMaxHist; q++) if (q < hp.n) w.half |= *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(hp.p[q]) + sel);
        }
    }
    w.mine = hp.coef[(size_t)blk * 64 + lane];
#else
    (void)lane;
    w.a = 0;
    for (int q = 0; q < kMaxHist; q++) if (q < hp.n) w.a |= *reinterpret_cast<const uint64_t*>(reinterpret_cast<const char*>(hp.p[q]) + off);
    w.first = nz_mask_of_block(hp.coef + (size_t)blk * 64, 0, 63);
#endif
    return w;
}
PCR_HD uint64_t hist_combine(const HistWords& w) {
#if defined(__HIP_DEVICE_COMPILE__)
    const uint64_t a = (uint32_t)__builtin_amdgcn_readlane((int)w.half, 0) | ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)w.half, 1) << 32);
    return a | __ballot(w.mine != 0);
#else
    return w.a | w.first;
#endif
}

// Zero table of one block: entry n (n = 0, 1, ...) belongs to the n-th position of the band that is
// still zero when the scan reaches the block (zig-zag order) and holds the number of non-zero-history
// positions below it -- the correction bits a decoder has stepped over when it lands there -- plus
// kZtLast if nothing is left in the block after it (the band's last position, if it is a zero).
// Entries from number-of-zeros on are sentinels, "no such zero": all non-zero-history positions of the
// band, plus kZtLast.
// With the table the serial decoder does no bit arithmetic per symbol: a run of r zeros followed by
// a new coefficient is "index += r + 1, read the entry", and the entry is what to add to the window
// offset.  kZtLast = 64 pushes that offset past the window, so the one test "offset < 64" ends the
// symbol loop for both reasons, a used-up window and a finished block.
// The 64 lanes build the table in a handful of vector instructions (a prefix count of the two masks
// and one permute); lane i also keeps the index of ITS position so that the set of table entries
// that were taken can be turned back into a mask of positions.
constexpr uint32_t kZtLast = 64;

// v = lane's bit of the wave-uniform mask m ? a : b, without materialising the bit: the mask is used as
// the select operand of a conditional move
PCR_HD uint32_t select_by_mask(uint64_t m, uint32_t a, uint32_t b, uint32_t lane) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t r;
    (void)lane;
    asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(b), "v"(a), "s"(m));
    return r;
#else
    return ((m >> lane) & 1) ? a : b;
#endif
}

struct ZeroTable {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t ventry, vindex;                                  // lane n: entry n; lane i: table index of position i (63 if not a zero)
#else
    uint32_t entry[64], index[64];
#endif
    // top64: kZtLast in the lane of the band's last position, 0 elsewhere (the same for every block of a scan)
    PCR_HD void build(uint64_t h, uint64_t z, uint32_t nzeros, uint32_t ncorr, uint32_t lane, uint32_t top64) {
#if defined(__HIP_DEVICE_COMPILE__)
        const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(z >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)z, 0));
        const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(h >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)h, 0));
        const uint32_t data = select_by_mask(z, below + top64, ncorr + kZtLast, lane);
        const uint32_t dest = select_by_mask(z, rank, nzeros + (lane - rank), lane);       // a permutation of the 64 lanes
        ventry = (uint32_t)__builtin_amdgcn_ds_permute((int)(dest * 4), (int)data);
        vindex = select_by_mask(z, rank, 63u, lane);
#else
        (void)lane; (void)top64;
        uint32_t rank = 0, below = 0, top = 0;
        for (uint32_t i = 0; i < 64; i++) if ((z | h) >> i & 1) top = i;
        for (uint32_t i = 0; i < 64; i++) {
            const bool iz = (z >> i) & 1;
            entry[iz ? rank : nzeros + (i - rank)] = iz ? below + (i == top ? kZtLast : 0u) : ncorr + kZtLast;
            index[i] = iz ? rank : 63u;
            rank += iz; below += (h >> i) & 1;
        }
#endif
    }
    PCR_HD uint32_t at(uint32_t n) const {                    // n <= 63
#if defined(__HIP_DEVICE_COMPILE__)
        return (uint32_t)__builtin_amdgcn_readlane((int)ventry, (int)n);
#else
        return entry[n];
#endif
    }
    // taken: bit n set = a symbol landed on entry n.  Returns the positions of those entries; positions that are
    // no zeros all point at entry 63 and must be masked off by the caller.
    PCR_HD uint64_t positions_of(uint64_t taken) const {
#if defined(__HIP_DEVICE_COMPILE__)
        return __ballot(((taken >> vindex) & 1) != 0);
#else
        uint64_t m = 0;
        for (uint32_t i = 0; i < 64; i++) if ((taken >> index[i]) & 1) m |= 1ull << i;
        return m;
#endif
    }
};

// All LDS and scalar-memory results this wavefront is waiting for have arrived: stated once ahead of a
// hot loop, the wait is not repeated inside it.
PCR_HD void settle_lds() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0xC07F);                      // lgkmcnt(0), the other counters untouched
#endif
}
// sets bit n (0..63) of a wave-uniform mask: one scalar instruction
PCR_HD void set_bit(uint64_t* m, uint32_t n) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm("s_bitset1_b64 %0, %1" : "+s"(*m) : "s"(n));
#else
    *m |= 1ull << n;
#endif
}

// Phase 1 (serial, one wavefront per unit): walk the scan only as far as needed to know where
// every block starts.  For each symbol that means: the code (length, run, size), the zero the run
// ends on and the NUMBER of correction bits stepped over on the way -- both read from the block's
// zero table; the sign and correction bits themselves are not read.  Per block it writes the
// kRefNz, kRefStart and kRefHist words of the block's record.
// The history of the next block is fetched while the current one is decoded.  Conditions are kept
// as integer arithmetic and single compares: a boolean widened to an integer, or two conditions
// and-ed together, cost the compiler a detour through the vector unit or through 64-bit lane masks.
PCR_HD int skim_ac_refine(WindowReader* wr, const LaneScan& ls, const HistPlanes& hp, uint64_t* recs, size_t nblk) {     // nblk: blocks of the component's plane
    const uint32_t bw = ls.bw[0], mcu_w = ls.mcu_w;
    const uint64_t band = band_mask(ls.Ss, ls.Se);
    const uint32_t top64 = wr->lane == (uint32_t)ls.Se ? kZtLast : 0u;
    const uint32_t adv_mask = opaque(127u), tot_field = opaque((6u << 16) | 8u);   // (in registers: see decode_ac_first)
    uint32_t left = ls.mcu1 - ls.mcu0;                       // blocks still to do
    const uint32_t row_skip = bw - mcu_w;                    // blocks of the padded grid between two rows of the scan
    const uint32_t last_blk = ((ls.mcu1 - 1) / mcu_w) * bw + (ls.mcu1 - 1) % mcu_w;
    uint32_t eobrun = 0;                                     // blocks still covered by an end-of-band run
    uint32_t bad = 0;
    // The history of a block is fetched two blocks ahead (a block of a dozen symbols is shorter than a trip to
    // memory).  One cursor (fblk, fcol) walks the unit's blocks for the fetches, stopping at the last one; b0 / b1
    // remember which block the words under way in h0 / h1 belong to: the block each body works on next.
    uint32_t fcol = ls.mcu0 % mcu_w;
    uint32_t fblk = (ls.mcu0 / mcu_w) * bw + fcol;
    uint32_t b0 = fblk;
    HistWords h0 = hist_fetch(hp, b0, wr->lane);
    fblk++; if (++fcol == mcu_w) { fcol = 0; fblk += row_skip; }
    uint32_t b1 = fblk < last_blk ? fblk : last_blk;
    HistWords h1 = hist_fetch(hp, b1, wr->lane);
    ZeroTable zt;
    // One block.  hw, bcur: the block's history and index on entry; on return the fetch for the block two further on
    // is under way in hw and bcur is that block.  (Two copies of this body alternate below, each with its own
    // history registers: handing the words from one variable to the next would mean waiting for the fetch that is
    // still in flight.)
    auto one_block = [&](HistWords& hw, uint32_t& bcur) {
        const uint64_t h = hist_combine(hw) & band;           // already non-zero
        const uint64_t z = h ^ band;                         // still zero
        uint64_t* rec = recs + bcur;
        left--;
        fblk++; if (++fcol == mcu_w) { fcol = 0; fblk += row_skip; }
        bcur = fblk < last_blk ? fblk : last_blk;
        hw = hist_fetch(hp, bcur, wr->lane);
        const uint64_t start = ((uint64_t)eobrun << 32) | wr->position();
        const uint32_t ncorr = (uint32_t)__builtin_popcountll(h);
        uint64_t newm = 0;
        if (eobrun == 0) {                                   // symbols are read only outside an end-of-band run
            const uint32_t nzeros = (uint32_t)__builtin_popcountll(z);   // <= 63: a band never holds position 0
            zt.build(h, z, nzeros, ncorr, wr->lane, top64);
            uint32_t at = ~0u;                               // table index the last symbol landed on (none yet)
            uint32_t ob = wr->o;                             // window offset not counting the correction bits stepped over in this block
            uint64_t taken = 0;                              // table entries a symbol landed on
            uint32_t info, e, t;
            for (;;) {
                if (wr->exhausted()) { const uint32_t before = wr->o; wr->refill(); ob -= before - wr->o; }
                settle_lds();
                align_loop();
                do {
                    // One straight line for every symbol.  A new +-1 after r zeros: r zeros are passed, the next
                    // one is taken.  End of band: as if the run went past every zero -- the sentinel entry says
                    // "all corrections, nothing left".  Unresolved codes and sixteen-zero symbols behave like an
                    // end of band here and are redone below.
                    info = wr->lookup(wr->o);
                    t = at + (info & adv_mask);              // run + 1, or 65 + run for an end of band
                    at = t < nzeros ? t : nzeros;            // past the last zero: the sentinel
                    e = zt.at(at);
                    set_bit(&taken, at);
                    ob += bit_field(info, tot_field);        // code and sign
                    wr->o = ob + e;                          // ... the corrections passed so far, and 64 more after the block's last entry
                } while (wr->o < 64);
                if (e < kZtLast) continue;                   // the window ran out inside the block
                wr->o -= kZtLast;
                if ((info & kSymSpecial) == 0) break;        // the block is complete
                // By hand: the symbol again from where it started.
                const uint32_t prev = opaque(t) - (info & 127);   // where the symbol before it had landed
                if (info == kSymMiss) {                      // a code longer than 8 bits, or none
                    const uint32_t passed = prev == ~0u ? 0u : zt.at(prev & 63u) & 63u;
                    info = wr->resolve(ob + passed);         // (a miss has length 0: ob is still the symbol's)
                    ob += (info >> 8) & 63;
                }
                if (info == kSymInvalid) { bad |= 1u; wr->o = ob; break; }   // no code at all, or one a refinement scan cannot hold
                const uint32_t zrl = info & kSymSpecial;     // sixteen zeros: lands on a zero and leaves it zero
                t = prev + (zrl ? kZrlAdvance : (info & 127));
                at = t < nzeros ? t : nzeros;
                e = zt.at(at);
                if (!zrl) set_bit(&taken, at);
                wr->o = ob + (e & 63);
                if (e >= kZtLast) break;
            }
            if (info & kSymEob) {                            // the block ended with an end-of-band (run) symbol
                eobrun = (1u << ((info & 127) - 65)) + (info >> 16);
            }
            bad |= (info >> 15) & ((nzeros - 1 - at) >> 31);  // a new coefficient with no zero left to take (it landed on the sentinel)
            newm = zt.positions_of(taken) & z;                 // (& z: lanes that are no zeros share index 63, which the sentinel can be)
            eobrun -= eobrun ? 1u : 0u;                      // the run counted this block
        } else {
            wr->consume(ncorr);
            eobrun--;
        }
        rec[ref_word(kRefNz, 0, nblk)] = newm; rec[ref_word(kRefStart, 0, nblk)] = start; rec[ref_word(kRefHist, 0, nblk)] = h;   // (phase 2 and the refinement replay work on the same history)
        bad |= wr->overrun_bit();
        left = bad ? 0 : left;                               // stop at the first damaged block
    };
    while (left != 0) {
        one_block(h0, b0);
        if (left == 0) break;
        one_block(h1, b1);
    }
    return bad ? kEFormat : kOk;
}

// Phase 2 (data-parallel, one lane per block): decode one block completely from its start.
//   words, byte_off  the unit's unstuffed data;  st  the block's kRefStart word;  h  history mask;
//   newm  the positions phase 1 found to become non-zero (kRefNz): the j-th symbol that carries a
//         coefficient lands on the j-th of them, so no zero run has to be counted here
// Returns the sign mask (1 = positive) of the positions that become non-zero and the mask of the positions whose
// correction bit is 1.  The stream holds exactly one correction bit per history-non-zero position of the band, in
// zig-zag order; the bits read between two symbols are dealt out to the history positions passed on the way.
// The lane keeps 64 bits of the stream in a register pair and fetches a word only when 32 of them are used up
// (every lane of a wavefront reads another block: these are plain vector loads), and takes a symbol's correction
// bits out of the 32 bits it looked the symbol up in whenever they fit.

// bits (first bit read = bit 0) dealt out to the set bits of `where`, lowest position first.  The two 32-bit halves of
// `where` are dealt to separately (the low half takes the first popcount(low half) bits): 64-bit shifts and carries
// would double the work of every step.
PCR_HD uint32_t deal_bits32(uint32_t bits, uint32_t where) {
    uint32_t out = 0;
    while (where) {
        const uint32_t low = where & (0u - where);            // the lowest position left
        out |= (bits & 1u) ? low : 0u;
        where ^= low; bits >>= 1;
    }
    return out;
}
PCR_HD uint64_t deal_bits(uint64_t bits, uint64_t where) {
    const uint32_t wlo = (uint32_t)where, whi = (uint32_t)(where >> 32);
    const uint32_t nlo = (uint32_t)__builtin_popcount(wlo);
    const uint32_t lo = deal_bits32((uint32_t)bits, wlo);
    const uint32_t hi = deal_bits32((uint32_t)(nlo < 32 ? bits >> nlo : bits >> 32), whi);   // (at most 63 bits are ever dealt)
    return ((uint64_t)hi << 32) | lo;
}

// position of the n-th (n = 1, 2, ...) set bit of z, or `none` if z has fewer: a binary search on population counts
// (a loop that clears n - 1 bits costs a wavefront its full length whenever one lane needs it)
PCR_HD int nth_set_bit(uint64_t z, uint32_t n, int none) {
    if ((uint32_t)__builtin_popcountll(z) < n) return none;
    uint32_t w = (uint32_t)z, base = 0;
    uint32_t t = (uint32_t)__builtin_popcount(w);
    if (n > t) { n -= t; w = (uint32_t)(z >> 32); base = 32; }
    t = (uint32_t)__builtin_popcount(w & 0xFFFFu); if (n > t) { n -= t; w >>= 16; base += 16; }
    t = (uint32_t)__builtin_popcount(w & 0xFFu);   if (n > t) { n -= t; w >>= 8; base += 8; }
    t = (uint32_t)__builtin_popcount(w & 0xFu);    if (n > t) { n -= t; w >>= 4; base += 4; }
    t = (uint32_t)__builtin_popcount(w & 0x3u);    if (n > t) { n -= t; w >>= 2; base += 2; }
    t = w & 1u;                                     if (n > t) base += 1;
    return (int)base;
}

struct LaneBits {
    const uint32_t* words;
    uint64_t buf;                                             // words[wi] : words[wi + 1]
    uint32_t wi, pos;                                         // next unread bit: bit `pos` (0..31) of buf, counted from its top
    PCR_HD void init(const uint32_t* w, uint32_t bit) { words = w; wi = bit >> 5; pos = bit & 31; buf = ((uint64_t)words[wi] << 32) | words[wi + 1]; }
    PCR_HD uint32_t peek() const { return (uint32_t)((buf << pos) >> 32); }          // the next 32 bits
    PCR_HD void skip(uint32_t n) {
        pos += n;
        while (pos >= 32) { wi++; buf = (buf << 32) | words[wi + 1]; pos -= 32; }
    }
    PCR_HD uint64_t take_reversed(uint32_t n) {               // the next n <= 63 bits, first bit read -> bit 0
        uint64_t out = 0; uint32_t done = 0;
        while (n > 0) {
            const uint32_t t = n > 32 ? 32 : n;
            out |= (uint64_t)(bitrev32(peek()) & (t == 32 ? ~0u : (1u << t) - 1)) << done;
            skip(t); done += t; n -= t;
        }
        return out;
    }
};

PCR_HD void refine_block(const uint32_t* words, uint32_t byte_off, uint64_t st, const AcTab* tab, uint64_t h, uint64_t newm, int Ss, int Se,
                         uint64_t* sign_out, uint64_t* plus_out) {
    const uint64_t band = band_mask(Ss, Se);
    h &= band;
    LaneBits rd;
    rd.init(words, byte_off * 8 + (uint32_t)st);
    const uint32_t ncorr = (uint32_t)__builtin_popcountll(h);
    uint64_t sgn = 0;
    uint64_t corr = 0;                                       // the correction bits in reading order (dealt out to the history positions at the end, once)
    uint32_t taken = 0;                                      // correction bits read so far
    uint32_t n = ncorr;                                      // inside an end-of-band run: all of them, nothing else
    if ((uint32_t)(st >> 32) == 0) {
        uint64_t rem = newm & band;                          // positions still to receive their coefficient
        int k = Ss;                                          // first position not yet passed
        n = 0;
        while (k <= Se) {
            const uint32_t win = rd.peek();
            const uint32_t e = ac_code(tab, win);
            if (!e) break;                                   // phase 1 has already flagged the image
            const uint32_t len = e >> 8, r = (e >> 4) & 15, s = e & 15;
            uint32_t used;                                   // bits of `win` this symbol takes
            int pos;
            if (s) {                                         // code, sign bit, then the corrections passed on the way
                if (!rem) break;
                pos = __builtin_ctzll(rem); rem &= rem - 1;
                sgn |= (uint64_t)((win << len) >> 31) << pos;
                used = len + 1;
            } else if (r == 15) {                            // sixteen zeros: lands on the sixteenth zero from k, which stays zero
                used = len;
                pos = nth_set_bit(~h & band & ~((1ull << k) - 1), 16, Se);
            } else {                                         // end of band: code, run-length bits, then every correction left
                rd.skip(len + r);
                n = ncorr - taken;
                break;
            }
            const uint32_t upto = (uint32_t)__builtin_popcountll(h & ((2ull << pos) - 1));   // corrections at positions <= pos (pos itself is a zero)
            if (upto > taken) {
                const uint32_t m = upto - taken;
                uint64_t bits;
                if (used + m <= 32) {                        // they are in the window already
                    bits = bitrev32(win << used) & ((1u << m) - 1);
                    used += m;
                } else {
                    rd.skip(used); used = 0;
                    bits = rd.take_reversed(m);
                }
                corr |= bits << taken;
                taken = upto;
            }
            rd.skip(used);
            k = pos + 1;
        }
    }
    if (n) corr |= rd.take_reversed(n) << taken;             // (taken + n is at most the number of history positions, 63)
    *sign_out = sgn; *plus_out = deal_bits(corr, h);
}

// ---------------------------------------------------------------------------------------
// Data-parallel part of AC refinement for one coefficient at zig-zag position k of a block.
//   newm, sgn, plus   the block's kRefNz, kRefSign and kRefPlus words of the scan
// ---------------------------------------------------------------------------------------
PCR_HD int16_t refine_apply(int16_t v, int k, uint64_t newm, uint64_t sgn, uint64_t plus, int Al) {
    uint64_t bit = 1ull << k;
    int p = 1 << Al;
    if (plus & bit) v = (int16_t)(v > 0 ? v + p : v - p);
    else if (newm & bit) v = (int16_t)((sgn & bit) ? p : -p);
    return v;
}

// ---------------------------------------------------------------------------------------
// DC refinement: bit number `index` (0 = first bit) of an unstuffed segment.
// ---------------------------------------------------------------------------------------
// words: aligned base of the segment (big-endian words); byte_off: start of the interval in it.
PCR_HD int dc_refine_bit(const uint32_t* words, uint32_t byte_off, uint32_t index) {
    const uint32_t bit = byte_off * 8 + index;
    return (words[bit >> 5] >> (31 - (bit & 31))) & 1;
}

}  // namespace pcr
