// Decompression, fast path (COMET Sec. 3.4 / Sec. 4.1 run backwards) for planes
// up to 512 columns wide, as two streaming kernels:
//
//   k_decode_chunks: chunk-parallel Huffman decode.  A wavefront takes 64
//     consecutive chunks, copies their words global -> LDS with coalesced loads (several
//     in flight; the chunk offsets are fetched one group ahead) and
//     decodes one chunk per lane: two words of the stream and a bit position per
//     lane, one word of look-ahead from LDS so that no load sits on the critical
//     path, and a look-up table whose entries already hold the residual (code -
//     radius): 12 bits and 16-bit entries for alphabets up to 4096 bins, else 11
//     bits and 32-bit entries (8 KB of LDS either way).  Symbols are decoded in
//     pairs (one refill per pair); codes longer than the table take a
//     wavefront-uniform slow path that starts its search at the length the table
//     entry gives.  32 residuals are collected in registers and leave as int16
//     in four back-to-back 16-byte stores.  The kernel needs about 9 KB of LDS per
//     wavefront, so four wavefronts per SIMD share the issue slots.
//
//   k_scan_store: Lorenzo reconstruction -> dequantise -> verbatim values ->
//     re-zero filter -> store.  Lanes are columns (pairs of adjacent columns for even
//     widths: one load and one store per pair).  Row by row a wavefront reads 64
//     residuals or pairs (buffer loads, several rows in flight), forms the row prefix with a
//     DPP scan (no LDS, no barrier), adds it to the per-column running sum held in
//     a register (the column prefix), multiplies by 2*eb, applies the re-zero
//     filter and stores fp32 (or rounds to a 16-bit type).  Loads and stores use buffer addressing: a lane that
//     has no element gets an out-of-range offset, which the hardware ignores, so
//     the loop has no divergent branches and the compiler can count the memory
//     operations in flight instead of draining them.
// Escaped residuals (code 0) sit in the work buffer as -32768 and are replaced, in
// element order, from the outlier records (copied to LDS once per strip).
//
// This file is the body of three translation units, one per output type (k_decompress_f32.hip,
// k_decompress_f16.hip, k_decompress_bf16.hip define COMET_DEC_OUT and include it).
#include <type_traits>

#include "comet_kernels.h"

#ifndef COMET_DEC_OUT
#error "include through k_decompress_f32.hip, k_decompress_f16.hip or k_decompress_bf16.hip"
#endif

namespace comet {

namespace {

constexpr int32_t kEscape = -32768;
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x16_t __attribute__((ext_vector_type(16)));

struct DsTables {
    const uint32_t *lut;        // LDS: the 11-bit table (u32 entries) or the compact 12-bit one (u16 entries)
    const uint64_t *limit, *first;
    const uint32_t *findex;
    const uint16_t *sorted;     // global: symbols in canonical order
    const uint16_t *sub;        // LDS: second level of the compact table (sub-tables of the prefixes with longer codes), or null
    const int16_t *tail;        // LDS: residuals of the canonical indices [tail0, tail0 + tail_n), i.e. of the long codes
    uint32_t tail0, tail_n;
    uint32_t max_len, n_active;
    int32_t radius;
    int32_t escape;             // residual value that stands for the escape symbol in the work buffer
};

// Codes longer than the look-up table: canonical search by length, from the shortest length the
// table entry says this prefix can have.
__device__ inline int32_t decode_long(uint64_t win, uint32_t start, uint32_t lut_bits, const DsTables &t, uint32_t *len_out) {
    uint32_t L = start > lut_bits ? start : lut_bits + 1u;
    while (L < t.max_len && win >= t.limit[L]) ++L;
    if (L > 57u) L = 57u;
    uint64_t idx = t.findex[L] + ((win >> (64u - L)) - t.first[L]);
    if (idx >= t.n_active) idx = t.n_active - 1u;            // corrupt stream only
    *len_out = L;
    const uint32_t ti = (uint32_t)idx - t.tail0;
    if (ti < t.tail_n) return (int32_t)t.tail[ti];
    const uint32_t sym = t.sorted[idx];                      // very large alphabets only
    return sym ? (int32_t)sym - t.radius : t.escape;
}

// Bit reader of one lane: two words of the stream plus a bit position inside the
// first one, and one word of look-ahead so that no load sits on the critical
// path.  Words are read from words[min(i, last)].  Everything is branch-free
// except the wavefront-uniform test for a code longer than the look-up table.
// The position runs from 1 to 32 (32: the first word is used up, the next bit is
// the second word's first), so that the next 32 bits of the stream are always one
// funnel shift of the two words, `alignbit(hi, lo, 32 - pos)`, whose shift count
// the hardware takes modulo 32.
// C16: the compact table (12 bits, u16 entries (residual << 4) | length), else the
// general one (11 bits, u32 entries (residual << 8) | length).
// STAGED: the words lie in the wavefront's LDS region, where a read past the last word is harmless (it stays inside
// the workgroup's LDS or returns nothing) and needs no clamp.
template <bool C16, bool STAGED = false>
struct BitBuf {
    static constexpr int kBits = C16 ? kLut16Bits : kLutBits;
    const uint32_t *words;
    uint32_t last;
    uint32_t hi, lo, nw;        // the word being consumed, the next one, the one after (look-ahead)
    uint32_t pos, wp;           // bits of `hi` already consumed (1 .. 32); index of `nw`
    __device__ inline uint32_t word(uint32_t i) const { return STAGED ? words[i] : words[i < last ? i : last]; }
    __device__ inline void open(const uint32_t *w, uint32_t last_, uint32_t w0) {
        words = w; last = last_;
        hi = 0u; lo = word(w0); nw = word(w0 + 1);          // (a first word that is used up already)
        pos = 32;
        wp = w0 + 1;
    }
    static __device__ inline uint32_t look(const DsTables &t, uint64_t window) {
        const uint32_t idx = (uint32_t)(window >> (64 - kBits));
        return C16 ? (uint32_t)reinterpret_cast<const uint16_t *>(t.lut)[idx] : t.lut[idx];
    }
    static __device__ inline uint32_t look32(const DsTables &t, uint32_t window) {       // window: the next 32 bits
        const uint32_t idx = window >> (32 - kBits);
        return C16 ? (uint32_t)reinterpret_cast<const uint16_t *>(t.lut)[idx] : t.lut[idx];
    }
    static __device__ inline uint32_t len_of(uint32_t e) { return C16 ? (e & 0xfu) : (e & 0xffu); }
    static __device__ inline int32_t resid_of(uint32_t e) { return C16 ? ((int32_t)(e << 16) >> 20) : ((int32_t)e >> 8); }
    static __device__ inline uint32_t hint_of(uint32_t e) { return C16 ? (e >> 4) : (e >> 8); }
    __device__ inline void advance() { hi = lo; lo = nw; ++wp; nw = word(wp); }

    __device__ inline int32_t next(const DsTables &t) {
        const uint64_t both = (((uint64_t)hi << 32) | lo) << pos;          // the next 64 - pos bits, left-aligned
        const uint32_t e = look(t, both);
        uint32_t L = len_of(e);
        int32_t d = resid_of(e);
        if (__builtin_expect(wave_ballot(L == 0u) != 0ull, 0)) {   // some lane met a code longer than the table: rare
            if (L == 0u) {
                const uint64_t win = both | ((uint64_t)nw >> (32u - pos));
                // second level: the prefix's sub-table on the next 1, 2, 4 or 6 bits; what is longer still
                // (or has no sub-table) is searched by length
                const bool found = second_level(t, e, win, L, d);
                if (!found) d = decode_long(win, C16 ? 0u : hint_of(e), (uint32_t)kBits, t, &L);
                if (pos + L >= 64u) {            // the code runs into the look-ahead word: move one word on here
                    advance();
                    pos -= 32u;                  // (modulo 2^32; the sum below is in range again)
                }
            }
        }
        pos += L;
        // a word is used up: the next ones move in
        const bool need = pos > 32u;
        hi = need ? lo : hi;
        lo = need ? nw : lo;
        pos -= need ? 32u : 0u;
        wp += need ? 1u : 0u;
        nw = word(wp);
        return d;
    }
    // Second level of the compact table: the sub-table of the first-level entry `e` (a prefix under which
    // longer codes lie), indexed by the bits that follow the prefix in `win` (64 bits of the stream from the
    // code's first bit).  False if the prefix has no sub-table or the code is longer than its sub-table covers.
    static __device__ inline bool second_level(const DsTables &t, uint32_t e, uint64_t win, uint32_t &L, int32_t &d) {
        const uint32_t h = e >> 4;
        if (!C16 || h == 0u) return false;
        const uint32_t kb = (0x6421u >> ((h & 3u) * 4u)) & 0xfu;
        const uint32_t e2 = t.sub[((h >> 2) << 1) + (uint32_t)((win << kBits) >> (64u - kb))];
        if ((e2 & 0xfu) == 0u) return false;
        L = (uint32_t)kBits + (e2 & 0xfu);
        d = resid_of(e2);
        return true;
    }
    // 64 bits of the stream from bit p (1 .. 63) of the two words on: the look-ahead word fills the low end
    __device__ inline uint64_t window_at(uint64_t both, uint32_t p) const {
        return (both << p) | (((uint64_t)nw << 32) >> (64u - p));
    }
    // Two symbols packed as (second << 16) | (first & 0xffff).  The first code is looked up in the next 32
    // bits, the second in the same bits shifted by the first one's length (a look-up-table code is at most
    // kBits long, so 32 - kBits >= kBits of them are still there), and the words move on at most once per
    // pair.  One wavefront-uniform test per pair: if either code of any lane is longer than the table the
    // pair is finished by pair_with_long_codes.
    __device__ inline uint32_t next_pair(const DsTables &t) {
        const uint32_t top = __builtin_amdgcn_alignbit(hi, lo, 32u - pos);
        const uint32_t e0 = look32(t, top);
        const uint32_t e1 = look32(t, top << len_of(e0));
        if (__builtin_expect(wave_ballot(len_of(e0) == 0u || len_of(e1) == 0u) != 0ull, 0)) return pair_with_long_codes(t, e0);
        const uint32_t p2 = pos + len_of(e0) + len_of(e1);
        const bool need = p2 > 32u;
        hi = need ? lo : hi;
        lo = need ? nw : lo;
        pos = need ? p2 - 32u : p2;
        wp += need ? 1u : 0u;
        nw = word(wp);
        if (C16) {
            // the two entries side by side, then both residuals moved down over their lengths at once
            typedef short s16x2 __attribute__((ext_vector_type(2)));
            s16x2 two = __builtin_bit_cast(s16x2, __builtin_amdgcn_perm(e1, e0, 0x05040100u));
            two >>= (short)4;
            return __builtin_bit_cast(uint32_t, two);
        }
        return __builtin_amdgcn_perm(e1, e0, 0x06050201u);      // bytes 1, 2 of each entry: the two residuals
    }
    // The same pair when some lane has a code longer than the table.  Such a code is resolved through the
    // second level (the lanes concerned only): up to 18 bits, so the second look-up still finds its bits in the
    // two words, and the pair may use up two words instead of one.  Only a code beyond both levels makes the
    // pair start over, one symbol at a time.
    __device__ inline uint32_t pair_with_long_codes(const DsTables &t, uint32_t e0) {
        const uint64_t both = ((uint64_t)hi << 32) | lo;
        uint32_t L0 = len_of(e0);
        int32_t d0 = resid_of(e0);
        bool fail = false;
        if (L0 == 0u) fail = !second_level(t, e0, window_at(both, pos), L0, d0);
        const uint32_t p1 = pos + L0;                          // at most 32 + 18
        const uint32_t e1 = look(t, both << p1);
        uint32_t L1 = len_of(e1);
        int32_t d1 = resid_of(e1);
        if (L1 == 0u) fail = !second_level(t, e1, window_at(both, p1), L1, d1) || fail;
        if (wave_ballot(fail) != 0ull) {
            const uint32_t s0 = (uint32_t)next(t) & 0xffffu;
            const uint32_t s1 = (uint32_t)next(t);
            return (s1 << 16) | s0;
        }
        uint32_t p2 = p1 + L1;                                 // at most 32 + 36
        const bool need = p2 > 32u;
        hi = need ? lo : hi;
        lo = need ? nw : lo;
        p2 -= need ? 32u : 0u;
        wp += need ? 1u : 0u;
        nw = word(wp);
        if (p2 > 32u) { advance(); p2 -= 32u; }                 // long codes may have used up a second word
        pos = p2;
        return ((uint32_t)d1 << 16) | ((uint32_t)d0 & 0xffffu);
    }
};

// Decode the first `nsym` symbols of one chunk into dst[0 .. nsym) (int16).  Chunk sizes that are a
// multiple of 32 (dst is then 64-byte aligned) collect 32 residuals in registers and write a whole
// 64-byte sector with four back-to-back 16-byte stores: every lane keeps a line of its own open, far
// more lines than the L2 holds, and 16-byte stores spread over time reached HBM as partial
// sectors (3.4 times the bytes).  Other multiples of eight leave as single 16-byte stores.
template <bool C16>
__device__ inline void decode_chunk(const uint32_t *words, uint32_t last, uint32_t w0, uint32_t S, uint32_t nsym, const DsTables &t, int16_t *dst) {
    BitBuf<C16> bb;
    bb.open(words, last, w0);
    uint32_t k = 0;
    if ((S & 31u) == 0u) {
        uint4 *dst16 = reinterpret_cast<uint4 *>(dst);
        for (uint32_t k32 = 0; k32 < nsym / 32u; ++k32) {
            uint32_t pk[16];                 // indexed by a wavefront-uniform counter: stays in registers
#pragma unroll 4
            for (int j = 0; j < 16; ++j) pk[j] = bb.next_pair(t);
#pragma unroll
            for (int j = 0; j < 4; ++j) dst16[k32 * 4u + j] = make_uint4(pk[4 * j], pk[4 * j + 1], pk[4 * j + 2], pk[4 * j + 3]);
        }
        k = nsym & ~31u;
    } else if ((S & 7u) == 0u) {
        uint4 *dst16 = reinterpret_cast<uint4 *>(dst);
        for (uint32_t k8 = 0; k8 < nsym / 8u; ++k8) {
            uint32_t pk[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) pk[j] = bb.next_pair(t);
            dst16[k8] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
        k = nsym & ~7u;
    }
    for (; k < nsym; ++k) dst[k] = (int16_t)bb.next(t);     // chunk sizes that are no multiple of eight; the tensor's last chunk
}

// ---- DPP: value of another lane of the same 16-lane row (0 where there is none) ----
template <int CTRL, int ROW_MASK, bool BOUND>
__device__ inline int32_t dpp0(int32_t v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, BOUND);
}

// Inclusive scan over runs of lanes.  MODE 0: runs of `width` <= 16 lanes packed
// inside 16-lane rows (pos = position in the run); MODE 1: one run per 32-lane
// half; MODE 2: one run over the whole wavefront.
template <int MODE>
__device__ inline int32_t run_scan(int32_t v, uint32_t pos, uint32_t width) {
    if (MODE == 0) {
        int32_t t;
        t = dpp0<0x111, 0xf, true>(v); if (width > 1u) v += (pos >= 1u) ? t : 0;
        t = dpp0<0x112, 0xf, true>(v); if (width > 2u) v += (pos >= 2u) ? t : 0;
        t = dpp0<0x114, 0xf, true>(v); if (width > 4u) v += (pos >= 4u) ? t : 0;
        t = dpp0<0x118, 0xf, true>(v); if (width > 8u) v += (pos >= 8u) ? t : 0;
        return v;
    }
    v += dpp0<0x111, 0xf, true>(v);
    v += dpp0<0x112, 0xf, true>(v);
    v += dpp0<0x114, 0xf, true>(v);
    v += dpp0<0x118, 0xf, true>(v);
    v += dpp0<0x142, 0xa, false>(v);            // lane 15 of rows 0, 2 into rows 1, 3
    if (MODE == 2) v += dpp0<0x143, 0xc, false>(v);   // lane 31 into rows 2, 3
    return v;
}

// first record index in [lo, hi) whose key is >= target (65-ary search by one wavefront)
__device__ inline uint32_t rec_lower_bound(const uint32_t *rec, uint32_t lo, uint32_t hi, uint32_t target, uint32_t lane) {
    while (lo < hi) {
        const uint32_t step = (hi - lo + 64u) / 65u;
        const uint32_t p = lo + (lane + 1u) * step - 1u;
        const bool less = (p < hi) ? (rec[2 * (size_t)p] < target) : false;
        const uint32_t c = (uint32_t)__popcll(wave_ballot(less));
        const uint32_t pc = lo + (c + 1u) * step - 1u;
        hi = (c < (uint32_t)kWave && pc < hi) ? pc : hi;
        lo = lo + c * step;
    }
    return lo;
}

// Element type of the output: OUT = 0 fp32, 1 IEEE half, 2 bfloat16.  A 16-bit output is the fp32
// result rounded to nearest, ties to even (NaN stays NaN).
template <int OUT> __device__ inline uint32_t narrow16(float v) {
    if (OUT == 1) return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)v);
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;       // NaN: keep it one
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// buffer descriptor over [p, p + bytes): accesses at offsets >= bytes are dropped (loads give 0)
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

}  // namespace

#if COMET_DEC_OUT == 0            // (not a template: in the fp32 unit only)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kDsBlock) void k_decode_chunks(DsArgs a) {
    extern __shared__ uint32_t s_dyn_ds[];                  // kDsWaves x kDsStageWords: the words of 64 chunks per wavefront
    __shared__ uint32_t s_lut[kLutSize];
    __shared__ uint64_t s_limit[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint32_t s_findex[65];
    __shared__ int16_t s_tail[kDsTailEntries];
    __shared__ uint32_t s_sub[kSubEntries / 2u];

    if (a.ctl->status & ST_FORMAT) return;

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));

    const Header *hdr = reinterpret_cast<const Header *>(a.container);
    if (a.skip_chunk64 && hdr->chunk_syms == 64u) return;
    const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.container + hdr->off_chunk);
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(a.container + hdr->off_payload);
    const uint32_t payload_words = (uint32_t)hdr->payload_words;
    const uint32_t S = hdr->chunk_syms;
    const uint32_t n_chunks = hdr->n_chunks;
    const bool zero_chunks = hdr->version == 2u;

    const bool c16 = a.t.meta[4] != 0u;                     // the compact table exists: use it
    {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a.t.lut16);     // the compact table, or a copy of the general one: kLutSize dwords
        for (uint32_t i = tid; i < kLutSize; i += kDsBlock) s_lut[i] = src[i];
    }
    for (uint32_t i = tid; i < 65u; i += kDsBlock) { s_limit[i] = a.t.limit[i]; s_first[i] = a.t.first_code[i]; s_findex[i] = a.t.first_index[i]; }
    if (c16) for (uint32_t i = tid; i < kSubEntries / 2u; i += kDsBlock) s_sub[i] = reinterpret_cast<const uint32_t *>(a.t.sub16)[i];
    DsTables t;
    t.sub = reinterpret_cast<const uint16_t *>(s_sub);
    t.lut = s_lut; t.limit = s_limit; t.first = s_first; t.findex = s_findex; t.sorted = a.t.sorted;
    t.max_len = a.t.meta[0]; t.n_active = a.t.meta[1]; t.radius = (int32_t)(hdr->nbins / 2u);
    // residuals of the symbols whose codes are longer than the look-up table, in canonical order
    t.tail = s_tail;
    const uint32_t lut_bits = c16 ? (uint32_t)kLut16Bits : (uint32_t)kLutBits;
    t.escape = c16 ? kLut16Escape : kEscape;
    t.tail0 = (t.max_len > lut_bits) ? a.t.first_index[lut_bits + 1u] : t.n_active;
    t.tail_n = t.n_active - t.tail0 < kDsTailEntries ? t.n_active - t.tail0 : kDsTailEntries;
    for (uint32_t i = tid; i < t.tail_n; i += kDsBlock) {
        const uint32_t sym = a.t.sorted[t.tail0 + i];
        s_tail[i] = (int16_t)(sym ? (int32_t)sym - t.radius : t.escape);
    }
    __syncthreads();

    uint32_t *stage = s_dyn_ds + wave * kDsStageWords;
    const uint32_t n_groups = (n_chunks + kWave - 1u) / kWave;
    // The offsets of a group are fetched while the group before it is decoded: what is loaded after
    // the residual stores of a group completes only once those stores have.
    const uint32_t grp_step = gridDim.x * kDsWaves;
    auto offsets_of = [&](uint32_t grp, uint32_t &o_lane, uint32_t &o_end) {
        if (grp >= n_groups) return;
        const uint32_t c_lo = grp * kWave;
        const uint32_t c_hi = (n_chunks - c_lo < (uint32_t)kWave) ? n_chunks : c_lo + kWave;
        o_lane = chunk_off[c_lo + lane < c_hi ? c_lo + lane : c_lo];
        o_end = chunk_off[c_hi < n_chunks ? c_hi : c_lo];
    };
    uint32_t off_lane_next = 0, off_end_next = 0;
    offsets_of(blockIdx.x * kDsWaves + wave, off_lane_next, off_end_next);
    for (uint32_t grp = blockIdx.x * kDsWaves + wave; grp < n_groups; grp += grp_step) {
        const uint32_t c_lo = grp * kWave;
        const uint32_t c_hi = (n_chunks - c_lo < (uint32_t)kWave) ? n_chunks : c_lo + kWave;
        const uint32_t c = c_lo + lane;

        // ---- the group's words, kDsStageBatch loads in flight per lane (a loop of load, wait, LDS
        // write would spend one memory round trip per 64 words, as long as the decoding itself) ----
        const uint32_t off_lane = off_lane_next, off_end = off_end_next;
        const uint32_t my_off = (c < c_hi) ? off_lane : 0u;
        uint32_t w_end = (c_hi < n_chunks) ? off_end : payload_words;
        uint32_t w_begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)my_off);
        if (w_end > payload_words) w_end = payload_words;
        if (w_begin > w_end) w_begin = w_end;
        const uint32_t n_words = w_end - w_begin;
        const bool all_staged = n_words <= kDsStageWords;
        if (all_staged) {
            const __amdgpu_buffer_rsrc_t r_w = make_rsrc(payload + w_begin, n_words * 4u);   // loads past the end give 0
            for (uint32_t i0 = 0; i0 < n_words; i0 += kDsStageBatch * kWave) {
                uint32_t v[kDsStageBatch];
#pragma unroll
                for (uint32_t j = 0; j < kDsStageBatch; ++j)
                    v[j] = __builtin_amdgcn_raw_buffer_load_b32(r_w, (int)((i0 + j * kWave + lane) * 4u), 0, 0);
#pragma unroll
                for (uint32_t j = 0; j < kDsStageBatch; ++j) {
                    const uint32_t i = i0 + j * kWave + lane;
                    if (i < n_words) stage[i] = v[j];
                }
            }
        }
        wave_lds_fence();
        offsets_of(grp + grp_step, off_lane_next, off_end_next);

        // ---- decode, one lane per chunk ----
        // (container version 2: a chunk without words is the centre code, residual 0, throughout)
        bool no_words = false;
        if (zero_chunks) {
            const uint32_t next_off = (uint32_t)__shfl_down((int)my_off, 1, kWave);
            no_words = c < c_hi && ((c + 1u < c_hi) ? next_off : w_end) <= my_off;
        }
        if (no_words) {
            const uint64_t s0 = (uint64_t)c * S;
            const uint32_t nsym = (a.n - s0 < (uint64_t)S) ? (uint32_t)(a.n - s0) : S;
            int16_t *dst = a.resid + s0;
            uint32_t k = 0;
            for (; k + 8u <= nsym; k += 8u) *reinterpret_cast<uint4 *>(dst + k) = make_uint4(0u, 0u, 0u, 0u);
            for (; k < nsym; ++k) dst[k] = 0;
        } else if (c < c_hi && n_words) {
            uint32_t w0 = (my_off < w_begin) ? 0u : my_off - w_begin;
            const uint64_t s0 = (uint64_t)c * S;
            const uint32_t nsym = (a.n - s0 < (uint64_t)S) ? (uint32_t)(a.n - s0) : S;
            int16_t *dst = a.resid + s0;
            if (c16) {
                if (all_staged) decode_chunk<true>(stage, n_words - 1u, w0, S, nsym, t, dst);          // words in LDS
                else decode_chunk<true>(payload + w_begin, n_words - 1u, w0, S, nsym, t, dst);         // too many for LDS: read them in place
            } else {
                if (all_staged) decode_chunk<false>(stage, n_words - 1u, w0, S, nsym, t, dst);
                else decode_chunk<false>(payload + w_begin, n_words - 1u, w0, S, nsym, t, dst);
            }
        }
        wave_lds_fence();
    }
}
#endif

// ---------------------------------------------------------------------------------------------
// VEC: adjacent columns per lane (2 needs an even W and an output aligned to two elements: one load
// and one store per pair, half the memory instructions).  A row takes L = W / VEC lanes.
// NSEG: 64-lane segments per row.  MODE (how the lanes of a wavefront map to rows):
// 0: L <= 16, 16/L planes side by side in every 16-lane row; 1: L <= 32, one plane per 32-lane
// half; 2: one plane, NSEG segments.
template <int NSEG, int MODE, int OUT, int VEC>
__global__ __launch_bounds__(kDsBlock) void k_scan_store(DsArgs a) {
    constexpr uint32_t OS = OUT ? 2u : 4u;                   // bytes per output element
    extern __shared__ uint32_t s_dyn_ds[];                  // kDsWaves x kScanListWords: escape list of a wavefront's strip

    if (a.ctl->status & ST_FORMAT) return;

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));

    const Header *hdr = reinterpret_cast<const Header *>(a.container);
    if (a.skip_chunk64 && hdr->chunk_syms == 64u) return;
    const uint32_t *rec = reinterpret_cast<const uint32_t *>(a.container + hdr->off_outlier);
    const uint32_t n_rec = hdr->n_rec;
    const float eb = __uint_as_float(hdr->eb_bits);
    const float ebx2 = __uint_as_float(hdr->ebx2_bits);
    const int32_t esc_marker = a.t.meta[4] ? kLut16Escape : kEscape;   // what the decode kernel wrote for escaped residuals
    uint32_t *list = s_dyn_ds + wave * kScanListWords;       // pairs (element offset inside the strip, residual)
    constexpr uint32_t kListCap = kScanListWords / 2u;

    // ---- geometry ----
    const uint32_t W = a.W, H = a.H, P = H * W;
    const uint32_t L = W / (uint32_t)VEC;                     // lanes per row
    constexpr bool group_mode = MODE != 2;                    // small planes: groups of whole planes; else one plane in strips of rows
    // lanes -> (plane slot, position in the row).  L <= 16: 16/L slots per 16-lane row; L <= 32: one
    // slot per 32-lane half; wider: one slot, NSEG segments of 64 lanes.
    uint32_t ppi = 1, slot = 0, wl = lane;
    bool lane_on = true;
    uint64_t slot_mask = ~0ull;
    if (MODE == 0) {
        const uint32_t spr = 16u / L, r = lane & 15u, sir = fdiv(r, a.divL);
        wl = r - sir * L; lane_on = sir < spr; slot = (lane >> 4) * spr + sir; ppi = 4u * spr;
        slot_mask = ((1ull << L) - 1ull) << ((lane & ~15u) + sir * L);
    } else if (MODE == 1) {
        wl = lane & 31u; lane_on = wl < L; slot = lane >> 5; ppi = 2u;
        slot_mask = ((1ull << L) - 1ull) << (lane & 32u);
    } else if (NSEG == 1) {
        lane_on = lane < L;
    }
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    const uint32_t G = group_mode ? a.group_planes : 1u;      // planes per unit
    const uint32_t R = group_mode ? H : (kScanStripElems / W ? kScanStripElems / W : 1u);   // rows per strip
    const uint32_t n_units = (a.planes + G - 1u) / G;

    // rows handled per batch of loads: four row segments in flight per batch, two batches (eight were
    // slower on every layer: more registers, fewer wavefronts)
    constexpr uint32_t U = NSEG >= 4 ? 1u : 4u / NSEG;

    for (uint32_t unit = blockIdx.x * kDsWaves + wave; unit < n_units; unit += gridDim.x * kDsWaves) {
        const uint32_t p0 = unit * G;
        const uint32_t planes_here = (a.planes - p0 < G) ? a.planes - p0 : G;
        const uint32_t e_unit = p0 * P;
        uint32_t rpos = 0;
        if (n_rec) rpos = rec_lower_bound(rec, 0, n_rec, 2u * e_unit, lane);
        int32_t q[NSEG][VEC];                               // running column sums
#pragma unroll
        for (int s = 0; s < NSEG; ++s)
#pragma unroll
            for (int v = 0; v < VEC; ++v) q[s][v] = 0;

        for (uint32_t row0 = 0; row0 < H; row0 += R) {
            const uint32_t rows = (H - row0 < R) ? H - row0 : R;
            const uint32_t e0 = e_unit + row0 * W;
            const uint32_t e1 = group_mode ? e_unit + planes_here * P : e0 + rows * W;
            const __amdgpu_buffer_rsrc_t r_in = make_rsrc(a.resid + e0, (e1 - e0) * 2u);
            const __amdgpu_buffer_rsrc_t r_out = make_rsrc(reinterpret_cast<char *>(a.out) + (size_t)e0 * OS, (e1 - e0) * OS);

            // ---- the strip's escaped residuals, compacted into LDS ----
            const uint32_t r_begin = rpos;
            uint32_t r_end = rpos;
            uint32_t n_esc = 0;          // type-0 records of the strip
            bool esc_in_lds = true, has_verbatim = false;
            if (n_rec && rpos < n_rec) {
                const uint32_t span = 2u * (e1 - e0);             // at most two records per element
                const uint32_t hi = (n_rec - rpos < span) ? n_rec : rpos + span;
                r_end = rec_lower_bound(rec, rpos, hi, 2u * e1, lane);
                for (uint32_t base = r_begin; base < r_end; base += kWave) {
                    const uint32_t k = base + lane;
                    uint32_t key = 1u, val = 0;
                    if (k < r_end) { key = rec[2 * (size_t)k]; val = rec[2 * (size_t)k + 1]; }
                    const bool esc = k < r_end && !(key & 1u);
                    const uint64_t esc_mask = wave_ballot(esc);
                    if (wave_ballot(k < r_end && (key & 1u))) has_verbatim = true;
                    if (esc) {
                        const uint32_t pos = n_esc + (uint32_t)__popcll(esc_mask & lt_mask);
                        if (pos < kListCap) { list[2 * pos] = (key >> 1) - e0; list[2 * pos + 1] = val; }
                    }
                    n_esc += (uint32_t)__popcll(esc_mask);
                }
                rpos = r_end;
                if (n_esc > kListCap) esc_in_lds = false;
                wave_lds_fence();
            }

            // ---- scans + dequantise + store; lanes are columns ----
            const uint32_t passes = group_mode ? (planes_here + ppi - 1u) / ppi : 1u;
            for (uint32_t pass = 0; pass < passes; ++pass) {
                const uint32_t pl = pass * ppi + slot;           // plane inside the unit
                const bool slot_on = lane_on && pl < planes_here;
                const uint32_t rel0 = group_mode ? pl * P : 0u;  // my plane's first element here, relative to e0
                if (group_mode) {
#pragma unroll
                    for (int s = 0; s < NSEG; ++s)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) q[s][v] = 0;
                }
                // my cursor into the escape list: first entry at or after my plane's first element
                uint32_t cur = 0;
                if (n_esc && group_mode && esc_in_lds) {
                    const uint32_t target = slot_on ? rel0 : 0xffffffffu;
                    uint32_t lo = 0, hi = n_esc;
                    while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (list[2 * mid] < target) lo = mid + 1; else hi = mid; }
                    cur = lo;
                }
                // element offsets (relative to e0) of my first column in row 0; 0x3fffffff for "no element":
                // times 2 or 4 it still lies beyond every strip, so the access is dropped
                uint32_t col[NSEG];
#pragma unroll
                for (int s = 0; s < NSEG; ++s) {
                    const uint32_t w = wl + (uint32_t)s * kWave;
                    col[s] = (slot_on && w < L) ? rel0 + w * (uint32_t)VEC : 0x3fffffffu;
                }
                auto fetch = [&](uint32_t h, int32_t (&d)[U][NSEG][VEC]) {
#pragma unroll
                    for (uint32_t u = 0; u < U; ++u) {
                        const uint32_t roff = (h + u < rows) ? (h + u) * W : 0x3fffffffu;    // wavefront-uniform
#pragma unroll
                        for (int s = 0; s < NSEG; ++s) {
                            uint32_t off = col[s] + roff;
                            off = off > 0x3fffffffu ? 0x3fffffffu : off;
                            if (VEC == 2) {
                                const uint32_t two = __builtin_amdgcn_raw_buffer_load_b32(r_in, (int)(off * 2u), 0, 0);
                                d[u][s][0] = (int32_t)(int16_t)(two & 0xffffu);
                                d[u][s][VEC - 1] = (int32_t)two >> 16;
                            } else {
                                d[u][s][0] = (int32_t)(int16_t)__builtin_amdgcn_raw_buffer_load_b16(r_in, (int)(off * 2u), 0, 0);
                            }
                        }
                    }
                };
                // The row loop exists twice: the usual one touches no memory besides the strip
                // (so the compiler never has to drain the stores), the other one looks escaped
                // residuals up in the container when their list did not fit LDS.
                auto rows_of = [&](auto slow_tag, uint32_t h, int32_t (&dd)[U][NSEG][VEC]) {
                    constexpr bool SLOW = decltype(slow_tag)::value;
#pragma unroll
                    for (uint32_t u = 0; u < U; ++u) {
                        const uint32_t roff = (h + u < rows) ? (h + u) * W : 0x3fffffffu;
                        int32_t carry = 0;
#pragma unroll
                        for (int s = 0; s < NSEG; ++s) {
                            uint32_t off = col[s] + roff;
                            off = off > 0x3fffffffu ? 0x3fffffffu : off;
                            int32_t d[VEC];
                            bool is_esc[VEC];
                            uint64_t em[VEC], any_esc = 0ull;
#pragma unroll
                            for (int v = 0; v < VEC; ++v) {
                                d[v] = dd[u][s][v];
                                is_esc[v] = d[v] == esc_marker;
                                em[v] = wave_ballot(is_esc[v]);
                                any_esc |= em[v];
                            }
                            if (any_esc) {                            // wavefront-uniform
                                // escapes of my plane in element order: lanes, then a lane's columns
                                uint32_t before = 0, all = 0;
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
                                    const uint64_t m = em[v] & slot_mask;
                                    before += (uint32_t)__popcll(m & lt_mask);
                                    all += (uint32_t)__popcll(m);
                                }
                                uint32_t pos = cur + before;
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
                                    if (is_esc[v]) {
                                        if (SLOW) {
                                            const uint32_t key = 2u * (e0 + off + (uint32_t)v);
                                            uint32_t lo = r_begin, hi = r_end;
                                            while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (rec[2 * (size_t)mid] < key) lo = mid + 1; else hi = mid; }
                                            d[v] = (lo < r_end && rec[2 * (size_t)lo] == key) ? (int32_t)rec[2 * (size_t)lo + 1] : 0;
                                        } else {
                                            const uint32_t at = pos < kListCap ? pos : kListCap - 1u;   // beyond: corrupt container only
                                            d[v] = n_esc ? (int32_t)list[2 * at + 1] : 0;
                                        }
                                        ++pos;
                                    }
                                }
                                cur += all;
                            }
                            // row prefix: the lane's own columns, then a scan of the lanes' sums
                            int32_t mine = d[0];
#pragma unroll
                            for (int v = 1; v < VEC; ++v) mine = (int32_t)((uint32_t)mine + (uint32_t)d[v]);
                            int32_t incl = run_scan<MODE>(mine, wl, L);
                            incl = (int32_t)((uint32_t)incl + (uint32_t)carry);
                            if (NSEG > 1) carry = __builtin_amdgcn_readlane(incl, 63);
                            int32_t rp[VEC];
                            rp[VEC - 1] = incl;
#pragma unroll
                            for (int v = VEC - 2; v >= 0; --v) rp[v] = (int32_t)((uint32_t)rp[v + 1] - (uint32_t)d[v + 1]);
                            float val[VEC];
#pragma unroll
                            for (int v = 0; v < VEC; ++v) {
                                q[s][v] = (int32_t)((uint32_t)q[s][v] + (uint32_t)rp[v]);
                                val[v] = (float)q[s][v] * ebx2;
                                if (fabsf(val[v]) <= eb) val[v] = 0.0f;
                            }
                            if (OUT == 0 && VEC == 2) {
                                u32x2_t two;
                                two.x = __float_as_uint(val[0]); two.y = __float_as_uint(val[VEC - 1]);
                                __builtin_amdgcn_raw_buffer_store_b64(two, r_out, (int)(off * 4u), 0, 0);
                            } else if (OUT == 0) {
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val[0]), r_out, (int)(off * 4u), 0, 0);
                            } else if (VEC == 2) {
                                __builtin_amdgcn_raw_buffer_store_b32(narrow16<OUT>(val[0]) | (narrow16<OUT>(val[VEC - 1]) << 16), r_out, (int)(off * 2u), 0, 0);
                            } else {
                                __builtin_amdgcn_raw_buffer_store_b16((unsigned short)narrow16<OUT>(val[0]), r_out, (int)(off * 2u), 0, 0);
                            }
                        }
                    }
                };
                auto row_loop = [&](auto slow_tag) {
                    // two batches of rows alternate: the loads of one are in flight while the other is scanned
                    int32_t da[U][NSEG][VEC], db[U][NSEG][VEC];
                    fetch(0, da);
                    for (uint32_t h = 0; h < rows; h += 2u * U) {
                        fetch(h + U, db);
                        rows_of(slow_tag, h, da);
                        fetch(h + 2u * U, da);
                        rows_of(slow_tag, h + U, db);
                    }
                };
                if (!esc_in_lds) row_loop(std::true_type{});
                else row_loop(std::false_type{});
            }

            // ---- verbatim values overwrite what was just stored ----
            if (has_verbatim) {
                // the lattice values of this wavefront must have landed first (workgroup scope waits for
                // the stores; a wider scope would also write back and invalidate the L2)
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
                for (uint32_t k = r_begin + lane; k < r_end; k += kWave) {
                    const uint32_t key = rec[2 * (size_t)k];
                    if (key & 1u) {
                        float v = __uint_as_float(rec[2 * (size_t)k + 1]);
                        if (fabsf(v) <= eb) v = 0.0f;
                        const uint32_t e = key >> 1;
                        if (e >= e0 && e < e1) {
                            if (OUT == 0) static_cast<float *>(a.out)[e] = v;
                            else static_cast<unsigned short *>(a.out)[e] = (unsigned short)narrow16<OUT>(v);
                        }
                    }
                }
            }
            wave_lds_fence();
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Fused decompression for containers with 64-symbol chunks: Huffman decode, Lorenzo reconstruction,
// dequantisation, verbatim values, re-zero filter and store in one kernel; residuals never leave the
// compute unit (Sec. 3.4: "decompress ... when needed" as one pass over the container).
//
// The tensor is cut into segments of whole planes and a segment into strips: runs of whole rows whose
// elements lie inside 64 consecutive chunks (about 4032 elements).  A wavefront takes a strip:
//   1. the words of the strip's chunks come global -> LDS with coalesced loads;
//   2. every lane decodes one chunk, 64 symbols, into 32 registers (pairs of int16 residuals);
//   3. the lanes write their registers to the same LDS region, element after element
//      (the words are no longer needed: the two uses share the memory);
//   4. the lanes turn into columns and walk the strip's rows out of LDS: row prefix by a DPP scan,
//      column prefix in a register per column, * 2eb, store.  Rows that take at most 32 lanes are
//      walked several at a time (slots of lanes side by side); the column prefix then also runs
//      across the slots of a step (cross-lane permutes), and what a plane has summed up so far is
//      handed from step to step through the lanes of the last row.
// A strip need not end at a plane boundary: the column sums restart wherever a plane starts.
//
// Who takes which strip.  Planes of at most 128 lanes per row (COOP: 128 columns, 256 with two columns per lane):
// one segment per workgroup, its strips dealt to the sixteen wavefronts in turn, so the work divides evenly whatever the plane size.  A strip
// that starts inside a plane needs that plane's column sums over the rows above: every strip adds up
// the residuals of its last (unfinished) plane column by column, which after a prefix over the
// columns is what the strip contributes, adds what it received itself if the plane started earlier,
// and hands the result to the next strip through LDS (a slot and two sequence numbers per wavefront).
// That sum costs a fraction of the scan, and it is ready long before the strip's own scan is, so the
// wavefronts of a workgroup decode and scan side by side instead of one after the other.  Wider
// planes: a segment per wavefront (a.G planes), the sums stay in its registers.
//
// The re-zero filter needs no instruction here: a lattice value q * 2eb lies within eb of zero only
// for q == 0, which already gives +0.0; verbatim values are filtered where they are written.
template <int NSEG, int MODE, int OUT, int VEC>
__global__ __launch_bounds__(kFuBlock) void k_decode_scan(FuArgs a) {
    constexpr uint32_t OS = OUT ? 2u : 4u;                   // bytes per output element
    constexpr bool COOP = NSEG <= 2;                                // planes of at most 128 lanes per row
    constexpr uint32_t CW = (NSEG == 2 && VEC == 2) ? 2u * kFuCarryW : kFuCarryW;   // columns of the widest of them
    constexpr uint32_t NWG = COOP ? (uint32_t)kFuWaves : 1u;        // wavefronts that share a segment
    extern __shared__ uint32_t s_dyn_ds[];                  // per wavefront: strip (kFuStripWords), escape values (kFuEscEntries)
    __shared__ uint32_t s_lut[kLutSize];
    __shared__ uint32_t s_sub[kSubEntries / 2u];
    __shared__ uint64_t s_limit[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint32_t s_findex[65];
    __shared__ int32_t s_carry[COOP ? kFuWaves : 1][COOP ? CW : 1];   // column sums a strip hands to the next one
    __shared__ uint32_t s_ready[kFuWaves], s_acked[kFuWaves];               // strip number + 1 of the slot's content / of its last reader
    __shared__ uint32_t s_cnt[(MODE != 2) ? kFuWaves : 1][64];                // MODE 0 / 1: escapes per slot of lanes

    if (a.ctl->status & ST_FORMAT) return;

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));

    const Header *hdr = reinterpret_cast<const Header *>(a.container);
    if (hdr->chunk_syms != 64u) return;                     // another chunk size: the general kernel launched behind this one takes it
    const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.container + hdr->off_chunk);
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(a.container + hdr->off_payload);
    const uint32_t *rec = reinterpret_cast<const uint32_t *>(a.container + hdr->off_outlier);
    const uint32_t payload_words = (uint32_t)hdr->payload_words;
    const uint32_t n_chunks = hdr->n_chunks;
    const uint32_t n_rec = hdr->n_rec;
    const bool zero_chunks = hdr->version == 2u;
    const float eb = __uint_as_float(hdr->eb_bits);
    const float ebx2 = __uint_as_float(hdr->ebx2_bits);

    // ---- decode tables into LDS (every load independent of the others: one round trip) ----
    const bool c16 = a.t.meta[4] != 0u;
    {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a.t.lut16);     // the compact table, or a copy of the general one
        for (uint32_t i = tid; i < kLutSize; i += kFuBlock) s_lut[i] = src[i];
        for (uint32_t i = tid; i < kSubEntries / 2u; i += kFuBlock) s_sub[i] = reinterpret_cast<const uint32_t *>(a.t.sub16)[i];
    }
    for (uint32_t i = tid; i < 65u; i += kFuBlock) { s_limit[i] = a.t.limit[i]; s_first[i] = a.t.first_code[i]; s_findex[i] = a.t.first_index[i]; }
    if (tid < (uint32_t)kFuWaves) { s_ready[tid] = 0u; s_acked[tid] = 0u; }
    DsTables t;
    t.lut = s_lut; t.sub = reinterpret_cast<const uint16_t *>(s_sub);
    t.limit = s_limit; t.first = s_first; t.findex = s_findex; t.sorted = a.t.sorted;
    t.max_len = a.t.meta[0]; t.n_active = a.t.meta[1]; t.radius = (int32_t)(hdr->nbins / 2u);
    t.tail = nullptr; t.tail0 = 0; t.tail_n = 0;            // what neither table level resolves is rare: symbols from global memory
    t.escape = c16 ? kLut16Escape : kEscape;
    const int32_t esc_marker = t.escape;
    __syncthreads();

    uint32_t *strip = s_dyn_ds + wave * kFuRegionWords;
    int32_t *esc = reinterpret_cast<int32_t *>(strip + kFuStripWords);

    // ---- lanes -> columns (scan phase) ----
    const uint32_t W = a.W, H = a.H, P = H * W;
    const uint32_t L = W / (uint32_t)VEC;                     // lanes per row
    uint32_t K = 1, slot = 0, wl = lane;                      // rows per step; my row inside a step; my position in the row
    bool lane_on = true;
    uint32_t spr = 1;
    if (MODE == 0) {
        spr = 16u / L;
        const uint32_t r = lane & 15u, sir = fdiv(r, a.divL);
        wl = r - sir * L; lane_on = sir < spr; slot = (lane >> 4) * spr + sir; K = 4u * spr;
    } else if (MODE == 1) {
        wl = lane & 31u; lane_on = wl < L; slot = lane >> 5; K = 2u;
    } else if (NSEG == 1) {
        lane_on = lane < L;
    }
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    // kNoElem for "no element": as an element offset times 2 or 4 it lies beyond every strip, so a
    // buffer access with it is dropped
    constexpr uint32_t kNoElem = 0x1fffffffu;
    uint32_t colw[NSEG];                                      // my first column's index in its row (kNoElem if none)
#pragma unroll
    for (int s = 0; s < NSEG; ++s) {
        const uint32_t w = wl + (uint32_t)s * kWave;
        const bool on = lane_on && w < L;
        colw[s] = on ? w * (uint32_t)VEC : kNoElem;
    }
    // next strip boundary after s (a strip = whole rows inside 64 consecutive chunks), inside a segment that ends at e_end
    auto strip_end = [&](uint32_t s, uint32_t e_end) {
        const uint32_t lim = fdiv(((s >> 6) + 64u) << 6, a.divW) * W;
        return lim < e_end ? lim : e_end;
    };
    // first word and number of words of the chunks whose offsets the lanes hold (lane 0: the first chunk's; off_end: that of
    // the chunk behind the last one, c_end), clamped to the payload; uniform results
    auto words_of = [&](uint32_t off_mine, uint32_t off_end, uint32_t c_end, uint32_t &w_begin, uint32_t &n_words) {
        uint32_t w_end = (c_end < n_chunks) ? (uint32_t)__builtin_amdgcn_readfirstlane((int)off_end) : payload_words;
        w_begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)off_mine);
        if (w_end > payload_words) w_end = payload_words;
        if (w_begin > w_end) w_begin = w_end;
        n_words = w_end - w_begin;
    };
    // wait until *flag >= want (LDS; the writer is another wavefront of this workgroup working on an earlier strip)
    auto wait_for = [&](const uint32_t *flag, uint32_t want) {
        uint32_t spins = 0;
        while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < want) {
            __builtin_amdgcn_s_sleep(2);
            if (++spins > (1u << 24)) { if (lane == 0) atomicOr(&a.ctl->status, (uint32_t)ST_INTERNAL); break; }   // cannot happen: turns a hang into an error
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    };

    const uint32_t gw = COOP ? wave : 0u;                     // my place among the wavefronts of my segment
    const uint32_t n_seg = COOP ? gridDim.x : a.n_units;
    const uint32_t seg_planes = COOP ? (a.planes + gridDim.x - 1u) / gridDim.x : a.G;
    const uint32_t seg_first = COOP ? blockIdx.x : wave * gridDim.x + blockIdx.x;
    const uint32_t seg_step = COOP ? n_seg : gridDim.x * (uint32_t)kFuWaves;
    uint32_t published = 0;                                   // COOP: strip number + 1 of my last hand-over that somebody reads

    for (uint32_t seg = seg_first; seg < n_seg; seg += seg_step) {
        const uint32_t p0 = seg * seg_planes;
        if (p0 >= a.planes) break;
        const uint32_t p1 = (a.planes - p0 < seg_planes) ? a.planes : p0 + seg_planes;
        const uint32_t e_a = p0 * P, e_b = p1 * P;
        uint32_t rpos = 0;                                  // records before my current strip (only ever moves forward)
        int32_t q[NSEG][VEC];                               // MODE 2: running column sums; MODE 0 / 1: the plane's sums up to the last row of the step before
#pragma unroll
        for (int s = 0; s < NSEG; ++s)
#pragma unroll
            for (int v = 0; v < VEC; ++v) q[s][v] = 0;

        bool pf_have = false;                               // what has been asked for ahead of time for my next strip
        uint32_t pf_off_lane = 0, pf_off_end = 0;
        uint32_t pf_words[kFuPrefetch];
#pragma unroll
        for (uint32_t jj = 0; jj < kFuPrefetch; ++jj) pf_words[jj] = 0u;
        // my first strip: number gw of the segment
        uint32_t j = gw;
        uint32_t s_a = e_a;
        for (uint32_t i = 0; i < gw && s_a < e_b; ++i) s_a = strip_end(s_a, e_b);
        while (s_a < e_b) {
            const uint32_t s_b = strip_end(s_a, e_b);
            const uint32_t c0 = s_a >> 6;
            const uint32_t c1 = (s_b + 63u) >> 6;                             // <= c0 + 64
            const uint32_t rows = fdiv(s_b - s_a, a.divW);
            const uint32_t row0 = fdiv(s_a, a.divW);
            const uint32_t h0 = row0 - fdiv(row0, a.divH) * H;   // row of the strip's first row inside its plane
            // the strip's last plane: it starts at row `lastseg` of the strip, or before the strip (then `fresh` is false)
            const uint32_t h_last = (h0 + rows - 1u) - fdiv(h0 + rows - 1u, a.divH) * H;
            const bool fresh = h_last + 1u <= rows;
            const uint32_t lastseg = fresh ? rows - (h_last + 1u) : 0u;
            const bool carry_in = COOP && h0 != 0u;             // (then the strip is not the first of its segment)
            const bool hand_on = COOP && s_b < e_b && h_last + 1u != H;    // the next strip starts inside my last plane
            const uint32_t c = c0 + lane;
            const uint32_t prev_w = (wave + (uint32_t)kFuWaves - 1u) % (uint32_t)kFuWaves;

            // ---- 1. words of the chunks [c0, c1) -> LDS.  The chunk offsets and the first kFuPrefetch * 64 words were
            // asked for while the strip before this one was being worked on (pf_*). ----
            uint32_t off_lane, off_end;
            if (pf_have) { off_lane = pf_off_lane; off_end = pf_off_end; }
            else { off_lane = chunk_off[c < c1 ? c : c0]; off_end = chunk_off[c1 < n_chunks ? c1 : c0]; }
            const uint32_t my_off = (c < c1) ? off_lane : 0u;
            uint32_t w_begin, n_words;
            words_of(my_off, off_end, c1, w_begin, n_words);
            const bool all_staged = n_words <= kFuStripWords - 4u;             // (the reader looks up to two words ahead)
            if (all_staged) {
                const __amdgpu_buffer_rsrc_t r_w = make_rsrc(payload + w_begin, n_words * 4u);   // loads past the end give 0
                uint32_t i_first = 0;
                if (pf_have) {
#pragma unroll
                    for (uint32_t jj = 0; jj < kFuPrefetch; ++jj) {
                        const uint32_t i = jj * kWave + lane;
                        if (i < n_words) strip[i] = pf_words[jj];
                    }
                    i_first = kFuPrefetch * kWave;
                }
                for (uint32_t i0 = i_first; i0 < n_words; i0 += kDsStageBatch * kWave) {
                    uint32_t v[kDsStageBatch];
#pragma unroll
                    for (uint32_t jj = 0; jj < kDsStageBatch; ++jj)
                        v[jj] = __builtin_amdgcn_raw_buffer_load_b32(r_w, (int)((i0 + jj * kWave + lane) * 4u), 0, 0);
#pragma unroll
                    for (uint32_t jj = 0; jj < kDsStageBatch; ++jj) {
                        const uint32_t i = i0 + jj * kWave + lane;
                        if (i < n_words) strip[i] = v[jj];
                    }
                }
            }
            // my next strip (NWG strips on): its chunk offsets are asked for now
            uint32_t n_sa = s_b;
            for (uint32_t i = 1; i < NWG && n_sa < e_b; ++i) n_sa = strip_end(n_sa, e_b);
            const bool n_have = n_sa < e_b;
            const uint32_t n_sb = n_have ? strip_end(n_sa, e_b) : e_b;
            const uint32_t n_c0 = n_sa >> 6, n_c1 = (n_sb + 63u) >> 6;
            if (n_have) {
                pf_off_lane = chunk_off[n_c0 + lane < n_c1 ? n_c0 + lane : n_c0];
                pf_off_end = chunk_off[n_c1 < n_chunks ? n_c1 : n_c0];
            }
            // MODE 0 / 1: the strip's rows are dealt to the K slots of lanes, slot k walks rows [ra, rb) on its own
            // (MODE 2: one slot, all rows).  ha: my first row inside its plane; my last plane starts at row
            // `lastseg_l` of the strip, or before my rows (then fresh_l is false).
            uint32_t rps = rows, ra = 0u, rb = rows, ha = h0, lastseg_l = lastseg;
            bool fresh_l = fresh;
            auto slot_rows = [&](uint32_t k, uint32_t &r0, uint32_t &r1, bool &fr, uint32_t &ls) {
                r0 = k * rps; r0 = r0 < rows ? r0 : rows;
                r1 = r0 + rps; r1 = r1 < rows ? r1 : rows;
                fr = false; ls = r0;
                if (r1 > r0) {
                    const uint32_t x = h0 + r1 - 1u;
                    const uint32_t hl = x - fdiv(x, a.divH) * H;
                    fr = hl + 1u <= r1 - r0;
                    ls = fr ? r1 - (hl + 1u) : r0;
                }
            };
            if (MODE != 2) {
                rps = fdiv(rows + K - 1u, a.divK);
                slot_rows(slot, ra, rb, fresh_l, lastseg_l);
                const uint32_t x = h0 + ra;
                ha = x - fdiv(x, a.divH) * H;
            }
            const bool exchange = hand_on || MODE != 2;       // column sums go through the exchange area of LDS
            // my exchange area: free once the reader of what I handed on last has taken it; cleared for the escapes' share
            if (exchange) {
                if (published) wait_for(&s_acked[wave], published);
                for (uint32_t i = lane; i < CW; i += kWave) s_carry[wave][COOP ? i : 0u] = 0;
                if (MODE != 2) s_cnt[wave][lane] = 0u;
            }
            wave_lds_fence();

            // ---- 2. decode, one lane per chunk, into registers: two halves of sixteen pairs, each filled by
            // a loop over four groups of four pairs (a vector of 16 words indexed by a wavefront-uniform
            // counter stays in registers; an array would be placed in scratch memory) ----
            u32x16_t pa = {}, pb = {};
            {
                const uint32_t last = n_words ? n_words - 1u : 0u;
                uint32_t w0 = (my_off < w_begin) ? 0u : my_off - w_begin;
                w0 = w0 < last ? w0 : last;
                // (one call per address space of the words, so that the reader's loads are LDS or global
                // instructions, not generic ones)
                auto run = [&](auto c16_tag, auto staged_tag, auto wsrc) {
                    BitBuf<decltype(c16_tag)::value, decltype(staged_tag)::value> bb;
                    bb.open(wsrc, last, w0);
#pragma nounroll
                    for (uint32_t j4 = 0; j4 < 4u; ++j4) {
#pragma unroll
                        for (uint32_t i = 0; i < 4u; ++i) pa[4u * j4 + i] = bb.next_pair(t);
                    }
#pragma nounroll
                    for (uint32_t j4 = 0; j4 < 4u; ++j4) {
#pragma unroll
                        for (uint32_t i = 0; i < 4u; ++i) pb[4u * j4 + i] = bb.next_pair(t);
                    }
                };
                if (c < c1 && n_words) {
                    if (all_staged) {
                        if (c16) run(std::true_type{}, std::true_type{}, strip); else run(std::false_type{}, std::true_type{}, strip);
                    } else {
                        const uint32_t *gsrc = payload + w_begin;
                        if (c16) run(std::true_type{}, std::false_type{}, gsrc); else run(std::false_type{}, std::false_type{}, gsrc);
                    }
                }
                // Container version 2: a chunk without words is residual 0 throughout.  Its lane has read
                // the words of the chunk behind it (or past the end of the strip's, which is harmless) with
                // the others; what it decoded is dropped.
                if (zero_chunks && n_words) {
                    const uint32_t next_off = (uint32_t)__shfl_down((int)my_off, 1, kWave);
                    const uint32_t w_last = w_begin + n_words;
                    if (((c + 1u < c1) ? next_off : w_last) <= my_off) { pa = u32x16_t{}; pb = u32x16_t{}; }
                }
            }
            wave_lds_fence();

            // the first words of my next strip: on their way while this strip is scanned
            pf_have = false;
            if (n_have) {
                uint32_t nb, nn;
                words_of((n_c0 + lane < n_c1) ? pf_off_lane : 0u, pf_off_end, n_c1, nb, nn);
                if (nn <= kFuStripWords - 4u) {
                    const __amdgpu_buffer_rsrc_t r_n = make_rsrc(payload + nb, nn * 4u);
#pragma unroll
                    for (uint32_t jj = 0; jj < kFuPrefetch; ++jj)
                        pf_words[jj] = __builtin_amdgcn_raw_buffer_load_b32(r_n, (int)((jj * kWave + lane) * 4u), 0, 0);
                }
                pf_have = true;
            }

            // ---- 3. registers -> LDS, element after element: 32 words per chunk.  (The 16-byte writes of the 64 lanes
            // fall into the same banks, which costs a few hundred cycles per strip; a padded row per chunk would avoid
            // that, and cost every later read of the strip four instructions for its address instead of one.) ----
            {
                uint4 *row = reinterpret_cast<uint4 *>(strip + lane * 32u);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    row[i] = make_uint4(pa[4 * i], pa[4 * i + 1], pa[4 * i + 2], pa[4 * i + 3]);
                    row[4 + i] = make_uint4(pb[4 * i], pb[4 * i + 1], pb[4 * i + 2], pb[4 * i + 3]);
                }
            }

            // ---- the strip's escaped residuals: their values compacted into LDS in element order; each also goes,
            // column by column, into the exchange area of the slot whose last plane it lies in (minus the marker
            // the residual holds); per slot they are counted, for the slot's place in the list ----
            uint32_t r_begin = rpos, r_end = rpos;
            uint32_t n_esc = 0;
            bool has_verbatim = false;
            if (n_rec) {
                // (my strip before this one ended at rpos and this one starts a few strips later: its first record is
                // nearly always among the next few thousand, which two rounds of probes find; else all that is left is searched)
                {
                    const uint32_t near = (j != gw && n_rec - rpos > 65u * 64u) ? rpos + 65u * 64u : n_rec;     // (my first strip: anywhere)
                    r_begin = rec_lower_bound(rec, rpos, near, 2u * s_a, lane);
                    if (r_begin == near && near < n_rec) r_begin = rec_lower_bound(rec, near, n_rec, 2u * s_a, lane);
                }
                r_end = r_begin;
                for (uint32_t base = r_begin; base < n_rec; base += kWave) {     // until a record beyond the strip turns up
                    const uint32_t k = base + lane;
                    uint32_t key = 0xffffffffu, val = 0;
                    if (k < n_rec) { key = rec[2 * (size_t)k]; val = rec[2 * (size_t)k + 1]; }
                    const bool mine = key < 2u * s_b;
                    const uint32_t n_mine_rec = (uint32_t)__popcll(wave_ballot(mine));
                    const bool is_e = mine && !(key & 1u);
                    if (wave_ballot(mine && (key & 1u))) has_verbatim = true;
                    // Compact table: the strip holds 16-bit residuals of which the table's own take 12 bits.  An
                    // escaped residual that fits the rest of the 16-bit range goes into the strip as it is (it
                    // is a residual like any other from then on); only the others are listed.
                    const bool direct = is_e && c16 && (int32_t)val > kLut16Escape && (int32_t)val < 32768;
                    if (direct) {
                        const uint32_t rel = (key >> 1) - (c0 << 6);
                        *reinterpret_cast<int16_t *>(reinterpret_cast<char *>(strip) + (rel << 1)) = (int16_t)(int32_t)val;
                    }
                    const bool listed = is_e && !direct;
                    const uint64_t esc_mask = wave_ballot(listed);
                    if (listed) {
                        const uint32_t pos = n_esc + (uint32_t)__popcll(esc_mask & lt_mask);
                        const uint32_t e = (key >> 1) - s_a;                     // inside the strip
                        int32_t held = esc_marker;                               // what the strip holds for this residual
                        if (pos < kFuEscEntries) {
                            esc[pos] = (int32_t)val;
                            if (c16) {
                                // the place in the list goes into the strip (values below the table's escape marker
                                // are free), so that the scan finds the value without counting escapes
                                held = kLut16Escape - 1 - (int32_t)pos;
                                const uint32_t rel = e + (s_a - (c0 << 6));
                                *reinterpret_cast<int16_t *>(reinterpret_cast<char *>(strip) + (rel << 1)) = (int16_t)held;
                            }
                        }
                        if (exchange) {
                            const uint32_t r = fdiv(e, a.divW);
                            const uint32_t cw = e - r * W;
                            uint32_t ke = 0u, ls = lastseg;
                            if (MODE != 2) {
                                // r / rps for small numbers: the float quotient is off by one at most
                                ke = (uint32_t)((float)r / (float)rps);
                                if (ke * rps > r) --ke;
                                if ((ke + 1u) * rps <= r) ++ke;
                                uint32_t r0, r1; bool fr;
                                slot_rows(ke, r0, r1, fr, ls);
                                if (!c16) atomicAdd(&s_cnt[wave][ke & 63u], 1u);
                            }
                            if (r >= ls && (MODE != 2 || hand_on))
                                atomicAdd(&s_carry[wave][COOP ? (ke * W + cw) & (CW - 1u) : 0u], (int32_t)(val - (uint32_t)held));
                        }
                    }
                    n_esc += (uint32_t)__popcll(esc_mask);
                    r_end += n_mine_rec;
                    if (n_mine_rec < (uint32_t)kWave) break;
                }
                rpos = r_end;
            }
            const bool esc_in_lds = n_esc <= kFuEscEntries;
            wave_lds_fence();
            uint32_t esc_base = 0;                               // escapes of the slots in front of mine
            if (MODE != 2 && n_esc && !c16) {
                const uint32_t mine = s_cnt[wave][lane];
                const uint32_t incl = wave_incl_scan<uint32_t>(mine);
                wave_lds_fence();
                s_cnt[wave][lane] = incl - mine;
                wave_lds_fence();
                esc_base = s_cnt[wave][slot & 63u];
            }

            const uint32_t rel0 = s_a - (c0 << 6);               // the strip's first element inside its chunks
            // a strip's element `off` in LDS: byte 2 * (rel0 + off) of the strip's region
            auto lds_of = [&](uint32_t off) { return (off + rel0) << 1; };
            auto lds_read = [&](uint32_t off) -> uint32_t {      // VEC == 2: two residuals; else one (sign-extended)
                const char *p = reinterpret_cast<const char *>(strip) + lds_of(off);
                if (VEC == 2) return *reinterpret_cast<const uint32_t *>(p);
                return (uint32_t)(int32_t)*reinterpret_cast<const int16_t *>(p);
            };

            // ---- column sums above my rows.  Every slot adds up the residuals of its last (unfinished) plane column
            // by column (an escaped one counts as its marker; the difference is in the exchange area already), a
            // prefix over the columns turns that into what the slot adds to the plane's column sums; a slot then
            // collects what the slots in front of it add, back to the one its plane starts in, and what the strip
            // itself received if the plane started before the strip; the last slot hands the sums on. ----
            if (COOP) {
                int32_t tcol[NSEG][VEC];
#pragma unroll
                for (int s = 0; s < NSEG; ++s)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) tcol[s][v] = 0;
                if (exchange) {
                    int32_t dsum[NSEG][VEC];
#pragma unroll
                    for (int s = 0; s < NSEG; ++s)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) dsum[s][v] = 0;
                    // (MODE 0 / 1: a slot's last plane starts in its last H rows at the earliest, so every slot walks up
                    // from its own last row, H rows at most)
                    const uint32_t r_first = MODE == 2 ? lastseg : 0u;       // MODE 2: uniform
                    const uint32_t r_count = MODE == 2 ? rows - lastseg : (rps < H ? rps : H);
#pragma unroll 4
                    for (uint32_t ts = 0; ts < r_count; ++ts) {
                        const uint32_t r = MODE == 2 ? r_first + ts : rb - 1u - ts;   // my row inside the strip
#pragma unroll
                        for (int s = 0; s < NSEG; ++s) {
                            // (one slot: the loop's bounds are the rows that count, and what a lane without a column
                            // adds up is dropped behind the loop)
                            const bool on = MODE == 2 ? true : (colw[s] != kNoElem && ts < rb - ra && r >= lastseg_l);
                            const uint32_t raw = lds_read((MODE == 2 ? colw[s] != kNoElem : on) ? r * W + colw[s] : 0u);
                            if (VEC == 2) {
                                dsum[s][0] += on ? (int32_t)(int16_t)(raw & 0xffffu) : 0;
                                dsum[s][VEC - 1] += on ? (int32_t)raw >> 16 : 0;
                            } else {
                                dsum[s][0] += on ? (int32_t)raw : 0;
                            }
                        }
                    }
                    if (MODE == 2) {
#pragma unroll
                        for (int s = 0; s < NSEG; ++s)
#pragma unroll
                            for (int v = 0; v < VEC; ++v) dsum[s][v] = colw[s] != kNoElem ? dsum[s][v] : 0;
                    }
                    // prefix over the columns, on top of the escapes' share
                    int32_t carry = 0;
#pragma unroll
                    for (int s = 0; s < NSEG; ++s) {
                        int32_t dd[VEC];
#pragma unroll
                        for (int v = 0; v < VEC; ++v)
                            dd[v] = colw[s] != kNoElem ? (int32_t)((uint32_t)dsum[s][v] + (uint32_t)s_carry[wave][COOP ? (slot * W + colw[s] + (uint32_t)v) & (CW - 1u) : 0u]) : 0;
                        int32_t mine = dd[0];
#pragma unroll
                        for (int v = 1; v < VEC; ++v) mine = (int32_t)((uint32_t)mine + (uint32_t)dd[v]);
                        int32_t incl = run_scan<MODE>(mine, wl, L);
                        incl = (int32_t)((uint32_t)incl + (uint32_t)carry);
                        if (NSEG > 1) carry = __builtin_amdgcn_readlane(incl, 63);
                        tcol[s][VEC - 1] = incl;
#pragma unroll
                        for (int v = VEC - 2; v >= 0; --v) tcol[s][v] = (int32_t)((uint32_t)tcol[s][v + 1] - (uint32_t)dd[v + 1]);
                    }
                    wave_lds_fence();                             // everybody has read the escapes' share
                }
                // MODE 0 / 1: the slots exchange their sums
                int32_t acc[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] = 0;
                bool reached = false;                             // the slot my first row's plane starts in has been added
                if (MODE != 2) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v)
                        if (colw[0] != kNoElem) s_carry[wave][COOP ? (slot * W + colw[0] + (uint32_t)v) & (CW - 1u) : 0u] = tcol[0][v];
                    wave_lds_fence();
                    for (uint32_t dd = 1; dd < K; ++dd) {         // slots in front of mine, nearest first
                        const bool take = slot >= dd && !reached && colw[0] != kNoElem;
                        const uint32_t kk = take ? slot - dd : 0u;
                        uint32_t r0, r1, ls; bool fr;
                        slot_rows(kk, r0, r1, fr, ls);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            const int32_t tv = s_carry[wave][COOP ? (kk * W + (take ? colw[0] : 0u) + (uint32_t)v) & (CW - 1u) : 0u];
                            acc[v] = take ? (int32_t)((uint32_t)acc[v] + (uint32_t)tv) : acc[v];
                        }
                        reached = reached || (take && fr);
                    }
                    wave_lds_fence();                             // all sums read: the area may take the hand-over
                }
                // What I hand on is my last plane's column sums down to my last row.  If that plane starts inside my
                // strip it does not depend on what I receive, and goes out before I wait: otherwise every strip of the
                // segment would wait for the one before it to have waited.
                auto hand_over = [&](const int32_t (&qq)[NSEG][VEC]) {
                    const bool last_slot = MODE == 2 || (rb == rows && rb > ra);
#pragma unroll
                    for (int s = 0; s < NSEG; ++s)
#pragma unroll
                        for (int v = 0; v < VEC; ++v)
                            if (colw[s] != kNoElem && last_slot)
                                s_carry[wave][COOP ? (colw[s] + (uint32_t)v) & (CW - 1u) : 0u] = (int32_t)((uint32_t)tcol[s][v] + (fresh_l ? 0u : (uint32_t)qq[s][v]));
                    wave_lds_fence();
                    if (lane == 0) __hip_atomic_store(&s_ready[wave], j + 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                    published = j + 1u;
                };
                const bool early = hand_on && fresh;
                if (early) {
                    // (a slot whose last plane started in an earlier slot of this strip has met that slot on its way back:
                    // its sums above are those of the slots in between)
                    int32_t q0[NSEG][VEC];
#pragma unroll
                    for (int s = 0; s < NSEG; ++s)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) q0[s][v] = (MODE == 2 || ha == 0u) ? 0 : acc[v];
                    hand_over(q0);
                }
                // what the strip received
                int32_t cin[NSEG][VEC];
#pragma unroll
                for (int s = 0; s < NSEG; ++s)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) cin[s][v] = 0;
                if (carry_in) {
                    wait_for(&s_ready[prev_w], j);                // strip j - 1 has handed over
#pragma unroll
                    for (int s = 0; s < NSEG; ++s)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) cin[s][v] = colw[s] != kNoElem ? s_carry[prev_w][COOP ? (colw[s] + (uint32_t)v) & (CW - 1u) : 0u] : 0;
                    wave_lds_fence();
                    if (lane == 0) __hip_atomic_store(&s_acked[prev_w], j, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                // the sums above my first row
#pragma unroll
                for (int s = 0; s < NSEG; ++s)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        if (MODE == 2) q[s][v] = cin[s][v];
                        else q[s][v] = ha != 0u ? (int32_t)((uint32_t)acc[v] + (reached ? 0u : (uint32_t)cin[s][v])) : 0;
                    }
                if (hand_on && !early) hand_over(q);
                if (!hand_on) published = 0u;
            }

            // ---- 4. scan the rows out of LDS ----
            const __amdgpu_buffer_rsrc_t r_out = make_rsrc(reinterpret_cast<char *>(a.out) + (size_t)s_a * OS, (s_b - s_a) * OS);
            const uint32_t n_steps = MODE == 2 ? rows : rps;
            uint32_t h_row = h0;                                 // MODE 2: the step's row inside its plane (uniform)
            uint32_t h_l = ha;                                   // MODE 0 / 1: my row inside its plane
            uint32_t cur = esc_base;                             // my place in the list of escaped values
            // lanes of my slot (MODE 0 / 1: the escapes of a step are taken slot by slot)
            uint64_t slot_mask = ~0ull;
            if (MODE == 0) slot_mask = ((1ull << L) - 1ull) << ((lane & ~15u) + (slot - (lane >> 4) * spr) * L);
            if (MODE == 1) slot_mask = ((1ull << L) - 1ull) << (lane & 32u);

            uint32_t sbase[NSEG], rbase[NSEG];                   // my first column in my first row: element of the strip (kNoElem: none) / where to read it
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                sbase[s] = colw[s] != kNoElem ? ra * W + colw[s] : kNoElem;
                rbase[s] = colw[s] != kNoElem ? ra * W + colw[s] : 0u;
            }
            const uint32_t n_mine = rb - ra;                     // MODE 0 / 1: rows of my slot

            auto scan_rows = [&](auto esc_tag) {
                constexpr int ESC = decltype(esc_tag)::value;   // 0: the strip has no escape; 1: compact table, escaped residuals hold their place in the list; 2: escapes counted
                constexpr uint32_t U = 2u;                       // steps per batch of LDS reads; two batches alternate
                // Step ts: my first column is element sbase[s] + ts * W of the strip (rows I do not have: see n_mine).
                // A lane without a column reads the strip's first word (what it computes goes nowhere: it sits
                // behind the row's lanes in every scan, and its store is dropped); reads of steps past the end
                // (the batch fetched ahead) may leave the strip, which LDS tolerates.
                auto fetch = [&](uint32_t t0, uint32_t (&raw)[U][NSEG]) {
#pragma unroll
                    for (uint32_t u = 0; u < U; ++u) {
                        const uint32_t tw = (t0 + u) * W;                 // uniform
#pragma unroll
                        for (int s = 0; s < NSEG; ++s) raw[u][s] = lds_read(rbase[s] + tw);
                    }
                };
                auto steps_of = [&](uint32_t t0, const uint32_t (&raw)[U][NSEG]) {
#pragma unroll
                  for (uint32_t u = 0; u < U; ++u) {
                    const uint32_t tstep = t0 + u;
                    if (tstep >= n_steps) break;                          // uniform
                    int32_t carry = 0;
                    const uint32_t tw = tstep * W;                              // uniform
#pragma unroll
                    for (int s = 0; s < NSEG; ++s) {
                        // element offset inside the strip (kNoElem or beyond: no element, the store is dropped)
                        const uint32_t off = (MODE == 2 || tstep < n_mine) ? sbase[s] + tw : kNoElem;
                        int32_t d[VEC];
                        if (VEC == 2) {
                            d[0] = (int32_t)(int16_t)(raw[u][s] & 0xffffu);
                            d[VEC - 1] = (int32_t)raw[u][s] >> 16;
                        } else {
                            d[0] = (int32_t)raw[u][s];
                        }
                        // the value of an escaped residual, looked up in the container (the list in LDS did not hold it)
                        auto from_container = [&](uint32_t elem) -> int32_t {
                            const uint32_t key = 2u * elem;
                            uint32_t lo = r_begin, hi = r_end;
                            while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (rec[2 * (size_t)mid] < key) lo = mid + 1; else hi = mid; }
                            return (lo < r_end && rec[2 * (size_t)lo] == key) ? (int32_t)rec[2 * (size_t)lo + 1] : 0;
                        };
                        if (ESC == 1) {
                            // compact table: an escaped residual holds its place in the list (or the bare marker if the list was full)
                            const bool on = sbase[s] != kNoElem && (MODE == 2 || tstep < n_mine);
                            bool is_esc[VEC];
                            bool any = false;
#pragma unroll
                            for (int v = 0; v < VEC; ++v) { is_esc[v] = on && d[v] <= kLut16Escape; any = any || is_esc[v]; }
                            if (wave_ballot(any)) {                    // wavefront-uniform
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
                                    if (is_esc[v]) {
                                        if (d[v] == kLut16Escape) d[v] = from_container(s_a + off + (uint32_t)v);
                                        else d[v] = esc[(uint32_t)(kLut16Escape - 1 - d[v]) & (kFuEscEntries - 1u)];
                                    }
                                }
                            }
                        }
                        if (ESC == 2) {
                            const bool on = sbase[s] != kNoElem && (MODE == 2 || tstep < n_mine);
                            bool is_esc[VEC];
                            uint64_t em[VEC], any_esc = 0ull;
#pragma unroll
                            for (int v = 0; v < VEC; ++v) {
                                is_esc[v] = on && d[v] == esc_marker;
                                em[v] = wave_ballot(is_esc[v]);
                                any_esc |= em[v];
                            }
                            if (any_esc) {                            // wavefront-uniform
                                // escapes of my slot in element order: lanes, then a lane's own columns
                                uint32_t before = 0, all = 0;
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
                                    const uint64_t m = em[v] & slot_mask;
                                    before += (uint32_t)__popcll(m & lt_mask);
                                    all += (uint32_t)__popcll(m);
                                }
                                uint32_t pos = cur + before;
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
                                    if (is_esc[v]) {
                                        if (!esc_in_lds) d[v] = from_container(s_a + off + (uint32_t)v);
                                        else d[v] = esc[pos < kFuEscEntries ? pos : kFuEscEntries - 1u];   // beyond: corrupt container only
                                        ++pos;
                                    }
                                }
                                cur += all;
                            }
                        }
                        // row prefix: the lane's own columns, then a scan over the lanes of the row
                        int32_t mine = d[0];
#pragma unroll
                        for (int v = 1; v < VEC; ++v) mine = (int32_t)((uint32_t)mine + (uint32_t)d[v]);
                        int32_t incl = run_scan<MODE>(mine, wl, L);
                        incl = (int32_t)((uint32_t)incl + (uint32_t)carry);
                        if (NSEG > 1) carry = __builtin_amdgcn_readlane(incl, 63);
                        int32_t rp[VEC];
                        rp[VEC - 1] = incl;
#pragma unroll
                        for (int v = VEC - 2; v >= 0; --v) rp[v] = (int32_t)((uint32_t)rp[v + 1] - (uint32_t)d[v + 1]);
                        float val[VEC];
                        const uint32_t keep = (MODE == 2 ? h_row : h_l) ? ~0u : 0u;     // a plane starts: its column sums start over
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            q[s][v] = (int32_t)(((uint32_t)q[s][v] & keep) + (uint32_t)rp[v]);
                            val[v] = (float)q[s][v] * ebx2;
                        }
                        if (OUT == 0 && VEC == 2) {
                            u32x2_t two;
                            two.x = __float_as_uint(val[0]); two.y = __float_as_uint(val[VEC - 1]);
                            __builtin_amdgcn_raw_buffer_store_b64(two, r_out, (int)(off * 4u), 0, 0);
                        } else if (OUT == 0) {
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val[0]), r_out, (int)(off * 4u), 0, 0);
                        } else if (VEC == 2) {
                            __builtin_amdgcn_raw_buffer_store_b32(narrow16<OUT>(val[0]) | (narrow16<OUT>(val[VEC - 1]) << 16), r_out, (int)(off * 2u), 0, 0);
                        } else {
                            __builtin_amdgcn_raw_buffer_store_b16((unsigned short)narrow16<OUT>(val[0]), r_out, (int)(off * 2u), 0, 0);
                        }
                    }
                    if (MODE == 2) { ++h_row; h_row = (h_row == H) ? 0u : h_row; }
                    else { ++h_l; h_l = (h_l == H) ? 0u : h_l; }
                  }
                };
                uint32_t ra_[U][NSEG], rb_[U][NSEG];
                fetch(0, ra_);
                for (uint32_t t0 = 0; t0 < n_steps; t0 += 2u * U) {
                    fetch(t0 + U, rb_);
                    steps_of(t0, ra_);
                    fetch(t0 + 2u * U, ra_);
                    steps_of(t0 + U, rb_);
                }
            };
            if (n_esc == 0u) scan_rows(std::integral_constant<int, 0>{});
            else if (c16) scan_rows(std::integral_constant<int, 1>{});
            else scan_rows(std::integral_constant<int, 2>{});

            // ---- verbatim values overwrite what was just stored ----
            if (has_verbatim) {
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");      // the lattice values of this wavefront have landed
                for (uint32_t k = r_begin + lane; k < r_end; k += kWave) {
                    const uint32_t key = rec[2 * (size_t)k];
                    if (key & 1u) {
                        float v = __uint_as_float(rec[2 * (size_t)k + 1]);
                        if (fabsf(v) <= eb) v = 0.0f;
                        const uint32_t e = key >> 1;
                        if (e >= s_a && e < s_b) {
                            if (OUT == 0) static_cast<float *>(a.out)[e] = v;
                            else static_cast<unsigned short *>(a.out)[e] = (unsigned short)narrow16<OUT>(v);
                        }
                    }
                }
            }
            wave_lds_fence();

            s_a = n_have ? n_sa : e_b;
            j += NWG;
        }
    }
}

// One translation unit per output type (COMET_DEC_OUT: 0 fp32, 1 IEEE half, 2 bfloat16) instantiates the
// kernels; they compile side by side.
#define COMET_INST_DEC(NS, MO, VE)                                                   \
    template __global__ void k_decode_scan<NS, MO, COMET_DEC_OUT, VE>(FuArgs);       \
    template __global__ void k_scan_store<NS, MO, COMET_DEC_OUT, VE>(DsArgs);
COMET_INST_DEC(1, 0, 1) COMET_INST_DEC(1, 1, 1) COMET_INST_DEC(1, 2, 1) COMET_INST_DEC(2, 2, 1)
COMET_INST_DEC(4, 2, 1) COMET_INST_DEC(8, 2, 1) COMET_INST_DEC(1, 0, 2) COMET_INST_DEC(1, 1, 2)
COMET_INST_DEC(1, 2, 2) COMET_INST_DEC(2, 2, 2) COMET_INST_DEC(4, 2, 2)
#undef COMET_INST_DEC

}  // namespace comet
