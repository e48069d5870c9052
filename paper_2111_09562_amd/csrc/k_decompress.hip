// Fused decompression, fast path (COMET Sec. 3.4 / Sec. 4.1 run backwards) for
// planes up to 512 columns wide: chunk-parallel Huffman decode -> Lorenzo
// reconstruction -> dequantise -> verbatim values -> re-zero filter -> store.
//
// Every wavefront works on its own: it takes a unit (a group of whole planes, or
// one plane cut into strips of rows), and for every strip
//   1. copies the strip's Huffman words global -> LDS with coalesced loads;
//   2. decodes: one lane per chunk, a 64-bit bit buffer per lane refilled from
//      LDS (two words of look-ahead so that no load sits on the critical path),
//      an 11-bit look-up table whose entries already hold the residual
//      (code - radius); residuals go to an int16 tile in LDS, every chunk padded
//      by one dword so that the 64 lanes hit 64 different banks;
//   3. scans: lanes become columns.  Row by row the wavefront reads 64 residuals,
//      forms the row prefix with a DPP scan (no LDS, no barrier), adds it to the
//      per-column running sum held in a register (the column prefix), multiplies
//      by 2*eb, applies the re-zero filter and stores fp32.
// Escaped residuals (code 0) sit in the tile as -32768 and are replaced, in
// element order, from the strip's outlier records (copied to LDS once per strip).
#include <type_traits>

#include "comet_kernels.h"

namespace comet {

namespace {

constexpr int32_t kEscape = -32768;

struct DsTables {
    const uint32_t *lut;        // LDS
    const uint64_t *limit, *first;
    const uint32_t *findex;
    const uint16_t *sorted;     // global: symbols in canonical order
    const int16_t *tail;        // LDS: residuals of the canonical indices [tail0, tail0 + tail_n), i.e. of the long codes
    uint32_t tail0, tail_n;
    uint32_t max_len, n_active;
    int32_t radius;
};

// Codes longer than the look-up table: canonical search by length.
__device__ inline int32_t decode_long(uint64_t win, const DsTables &t, uint32_t *len_out) {
    uint32_t L = kLutBits + 1;
    while (L < t.max_len && win >= t.limit[L]) ++L;
    if (L > 57u) L = 57u;
    uint64_t idx = t.findex[L] + ((win >> (64u - L)) - t.first[L]);
    if (idx >= t.n_active) idx = t.n_active - 1u;            // corrupt stream only
    *len_out = L;
    const uint32_t ti = (uint32_t)idx - t.tail0;
    if (ti < t.tail_n) return (int32_t)t.tail[ti];
    const uint32_t sym = t.sorted[idx];                      // very large alphabets only
    return sym ? (int32_t)sym - t.radius : kEscape;
}

// Decode `nsym` symbols of one chunk into dst[0..nsym).  Words are read from
// words[min(i, last)]; the chunk starts at word index w0.
// Bit buffer: `buf` holds the next bits left-aligned with more than 32 of them
// valid; nw0 / nw1 are the two words after it.  Everything in the loop is
// branch-free except the wavefront-uniform test for a long code.
__device__ inline void decode_chunk(const uint32_t *words, uint32_t last, uint32_t w0, uint32_t nsym, const DsTables &t, int16_t *dst) {
    auto word = [&](uint32_t i) -> uint32_t { return words[i < last ? i : last]; };
    uint64_t buf = ((uint64_t)word(w0) << 32) | word(w0 + 1);
    uint32_t nb = 64;
    uint32_t nw0 = word(w0 + 2), nw1 = word(w0 + 3);
    uint32_t wp = w0 + 3;                       // index of nw1
    for (uint32_t k = 0; k < nsym; ++k) {
        const uint32_t e = t.lut[(uint32_t)(buf >> (64 - kLutBits))];
        uint32_t L = e & 0xffu;
        int32_t d = (int32_t)e >> 8;
        if (__builtin_expect(__ballot(e == 0u) != 0ull, 0)) {   // some lane met a code longer than the table: rare
            if (e == 0u) {
                const uint64_t win = buf | ((uint64_t)nw0 >> (nb - 32u));
                d = decode_long(win, t, &L);
                if (L >= nb) {                  // the code runs into the look-ahead word: consume it here
                    const uint32_t extra = L - nb;
                    buf = ((uint64_t)nw0 << 32) << extra;
                    nb = 32u - extra;
                    nw0 = nw1; ++wp; nw1 = word(wp);
                    L = 0;
                }
            }
        }
        dst[k] = (int16_t)d;
        buf <<= L;
        nb -= L;
        // refill: below 33 valid bits the next word moves in
        const bool need = nb <= 32u;
        const uint64_t add = (uint64_t)nw0 << ((32u - nb) & 31u);
        buf |= need ? add : 0ull;
        nb += need ? 32u : 0u;
        nw0 = need ? nw1 : nw0;
        wp += need ? 1u : 0u;
        nw1 = word(wp);
    }
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
        const uint32_t c = (uint32_t)__popcll(__ballot(less));
        const uint32_t pc = lo + (c + 1u) * step - 1u;
        hi = (c < (uint32_t)kWave && pc < hi) ? pc : hi;
        lo = lo + c * step;
    }
    return lo;
}

}  // namespace

// NSEG: 64-column segments per row.  MODE (how the lanes of a wavefront map to columns):
// 0: W <= 16, 16/W planes side by side in every 16-lane row; 1: W <= 32, one plane per 32-lane
// half; 2: one plane, columns = lanes.
template <int NSEG, int MODE>
__global__ __launch_bounds__(kDsBlock) void k_decode_scan(DsArgs a) {
    extern __shared__ uint32_t s_dyn_ds[];
    __shared__ uint32_t s_lut[kLutSize];
    __shared__ uint64_t s_limit[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint32_t s_findex[65];
    __shared__ int16_t s_tail[kDsTailEntries];

    if (a.ctl->status & ST_FORMAT) return;

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = tid / kWave;

    const Header *hdr = reinterpret_cast<const Header *>(a.container);
    const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.container + hdr->off_chunk);
    const uint32_t *rec = reinterpret_cast<const uint32_t *>(a.container + hdr->off_outlier);
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(a.container + hdr->off_payload);
    const uint32_t payload_words = (uint32_t)hdr->payload_words;
    const uint32_t n_rec = hdr->n_rec;
    const uint32_t S = hdr->chunk_syms;
    const uint32_t n_chunks = hdr->n_chunks;
    const float eb = __uint_as_float(hdr->eb_bits);
    const float ebx2 = __uint_as_float(hdr->ebx2_bits);

    for (uint32_t i = tid; i < kLutSize; i += kDsBlock) s_lut[i] = a.t.lut[i];
    for (uint32_t i = tid; i < 65u; i += kDsBlock) { s_limit[i] = a.t.limit[i]; s_first[i] = a.t.first_code[i]; s_findex[i] = a.t.first_index[i]; }
    DsTables t;
    t.lut = s_lut; t.limit = s_limit; t.first = s_first; t.findex = s_findex; t.sorted = a.t.sorted;
    t.max_len = a.t.meta[0]; t.n_active = a.t.meta[1]; t.radius = (int32_t)(hdr->nbins / 2u);
    // residuals of the symbols whose codes are longer than the look-up table, in canonical order
    t.tail = s_tail;
    t.tail0 = (t.max_len > (uint32_t)kLutBits) ? a.t.first_index[kLutBits + 1] : t.n_active;
    t.tail_n = t.n_active - t.tail0 < kDsTailEntries ? t.n_active - t.tail0 : kDsTailEntries;
    for (uint32_t i = tid; i < t.tail_n; i += kDsBlock) {
        const uint32_t sym = a.t.sorted[t.tail0 + i];
        s_tail[i] = (int16_t)(sym ? (int32_t)sym - t.radius : kEscape);
    }
    __syncthreads();

    // per-wavefront LDS: residual tile (int16), then the word stage / escape list
    uint32_t *my = s_dyn_ds + wave * (kDsTileEntries / 2u + kDsStageWords);
    int16_t *tile = reinterpret_cast<int16_t *>(my);
    uint32_t *stage = my + kDsTileEntries / 2u;

    // ---- geometry (depends on the chunk size, which only the header knows) ----
    const uint32_t W = a.W, H = a.H, P = H * W;
    const uint32_t n = (uint32_t)a.n;
    const uint32_t pitch = S + 2u;                               // tile entries per chunk
    const bool pow2 = (S & (S - 1u)) == 0u;
    const uint32_t log2S = pow2 ? (uint32_t)(31 - __clz((int)S)) : 0u;
    const uint32_t cps = kDsTileEntries / pitch;                 // chunks that fit the tile
    const uint32_t emax = cps >= 2u ? (cps - 1u) * S : 0u;       // elements per strip, whatever its alignment
    if (emax < W) { if (tid == 0) atomicOr(&a.ctl->status, (uint32_t)ST_FORMAT); return; }
    const bool group_mode = P <= emax;
    const uint32_t G = group_mode ? emax / P : 1u;               // planes per unit
    const uint32_t R = group_mode ? H : emax / W;                // rows per strip
    const uint32_t n_units = group_mode ? (a.planes + G - 1u) / G : a.planes;

    // lanes -> (plane slot, column).  W <= 16: 16/W slots per 16-lane row; W <= 32: one slot per
    // 32-lane half; wider: one slot, NSEG segments of 64 columns.
    uint32_t ppi = 1, slot = 0, wl = lane;
    bool lane_on = true;
    uint64_t slot_mask = ~0ull;
    if (MODE == 0) {
        const uint32_t spr = 16u / W, r = lane & 15u, sir = fdiv(r, a.divW);
        wl = r - sir * W; lane_on = sir < spr; slot = (lane >> 4) * spr + sir; ppi = 4u * spr;
        slot_mask = ((1ull << W) - 1ull) << ((lane & ~15u) + sir * W);
    } else if (MODE == 1) {
        wl = lane & 31u; lane_on = wl < W; slot = lane >> 5; ppi = 2u;
        slot_mask = ((1ull << W) - 1ull) << (lane & 32u);
    } else if (NSEG == 1) {
        lane_on = lane < W;
    }
    const uint64_t lt_mask = (1ull << lane) - 1ull;

    const uint32_t gw = blockIdx.x * kDsWaves + wave;
    const uint32_t n_gw = gridDim.x * kDsWaves;

    COMET_ACC_DECL;
    for (uint32_t unit = gw; unit < n_units; unit += n_gw) {
        COMET_ACC(a.ctl, 10);
        const uint32_t p0 = group_mode ? unit * G : unit;
        const uint32_t planes_here = group_mode ? ((a.planes - p0 < G) ? a.planes - p0 : G) : 1u;
        const uint32_t e_unit = p0 * P;
        uint32_t rpos = 0;
        if (n_rec) rpos = rec_lower_bound(rec, 0, n_rec, 2u * e_unit, lane);
        int32_t q[NSEG];
#pragma unroll
        for (int s = 0; s < NSEG; ++s) q[s] = 0;
        COMET_ACC(a.ctl, 11);

        for (uint32_t row0 = 0; row0 < H; row0 += R) {
            const uint32_t rows = (H - row0 < R) ? H - row0 : R;
            const uint32_t e0 = e_unit + row0 * W;
            const uint32_t e1 = group_mode ? e_unit + planes_here * P : e0 + rows * W;
            const uint32_t c_lo = e0 / S;
            uint32_t c_hi = (e1 - 1u) / S + 1u;
            if (c_hi > n_chunks) c_hi = n_chunks;

            // ---- 1. stage the strip's words (one round trip for the offsets, one for the words) ----
            uint32_t my_off = 0;                                  // word offset of chunk c_lo + lane
            if (c_lo + lane < c_hi) my_off = chunk_off[c_lo + lane];
            uint32_t w_end = (c_hi < n_chunks) ? chunk_off[c_hi] : payload_words;
            uint32_t w_begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)my_off);
            if (w_end > payload_words) w_end = payload_words;
            if (w_begin > w_end) w_begin = w_end;
            const uint32_t n_words = w_end - w_begin;
            const uint32_t n_stage = n_words < kDsStageWords ? n_words : kDsStageWords;
            for (uint32_t i = lane; i < n_stage; i += kWave) stage[i] = payload[w_begin + i];
            wave_lds_fence();
            COMET_ACC(a.ctl, 12);

            // ---- 2. decode, one lane per chunk ----
            const bool all_staged = n_words <= kDsStageWords;
            const uint32_t last = n_words ? n_words - 1u : 0u;
            if (n_words) {
                for (uint32_t c = c_lo + lane; c < c_hi; c += kWave) {
                    uint32_t w0 = (c == c_lo + lane) ? my_off : chunk_off[c];
                    w0 = (w0 < w_begin) ? 0u : w0 - w_begin;
                    const uint32_t s0 = c * S;
                    const uint32_t nsym = (n - s0 < S) ? n - s0 : S;
                    int16_t *dst = tile + (c - c_lo) * pitch;
                    if (all_staged) decode_chunk(stage, last, w0, nsym, t, dst);            // words in LDS
                    else decode_chunk(payload + w_begin, last, w0, nsym, t, dst);           // too many for LDS: read them in place
                }
            }
            wave_lds_fence();
            COMET_ACC(a.ctl, 13);

            // ---- 3. the strip's escaped residuals, compacted into LDS (reuses the stage) ----
            const uint32_t r_begin = rpos;
            uint32_t r_end = rpos;
            uint32_t n_esc = 0;          // type-0 records of the strip
            bool esc_in_lds = true, has_verbatim = false;
            if (n_rec && rpos < n_rec) {
                const uint32_t span = 2u * (e1 - e0);             // at most two records per element
                const uint32_t hi = (n_rec - rpos < span) ? n_rec : rpos + span;
                r_end = rec_lower_bound(rec, rpos, hi, 2u * e1, lane);
                uint32_t *list = stage;  // pairs (element offset from e0, value)
                for (uint32_t base = r_begin; base < r_end; base += kWave) {
                    const uint32_t k = base + lane;
                    uint32_t key = 1u, val = 0;
                    if (k < r_end) { key = rec[2 * (size_t)k]; val = rec[2 * (size_t)k + 1]; }
                    const bool esc = k < r_end && !(key & 1u);
                    const uint64_t esc_mask = __ballot(esc);
                    if (__ballot(k < r_end && (key & 1u))) has_verbatim = true;
                    if (esc) {
                        const uint32_t pos = n_esc + (uint32_t)__popcll(esc_mask & lt_mask);
                        if (pos < kDsStageWords / 2u) { list[2 * pos] = (key >> 1) - e0; list[2 * pos + 1] = val; }
                    }
                    n_esc += (uint32_t)__popcll(esc_mask);
                }
                rpos = r_end;
                if (n_esc > kDsStageWords / 2u) esc_in_lds = false;
                wave_lds_fence();
            }
            COMET_ACC(a.ctl, 14);

            // ---- 4. scans + dequantise + store; lanes are columns ----
            const uint32_t tile_e0 = c_lo * S;                   // element held by tile entry 0
            const uint32_t passes = group_mode ? (planes_here + ppi - 1u) / ppi : 1u;
            for (uint32_t pass = 0; pass < passes; ++pass) {
                const uint32_t pl = pass * ppi + slot;           // plane inside the unit
                const bool slot_on = lane_on && pl < planes_here;
                const uint32_t e_row0 = group_mode ? e_unit + pl * P : e0;   // first element of my plane's first row here
                if (group_mode) {
#pragma unroll
                    for (int s = 0; s < NSEG; ++s) q[s] = 0;
                }
                // my cursor into the escape list: first entry at or after my plane's first element
                uint32_t cur = 0;
                if (n_esc && group_mode && esc_in_lds) {
                    const uint32_t target = slot_on ? e_row0 - e0 : 0xffffffffu;
                    uint32_t lo = 0, hi = n_esc;
                    while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (stage[2 * mid] < target) lo = mid + 1; else hi = mid; }
                    cur = lo;
                }
                // The row loop exists twice: the usual one touches no global memory besides its
                // stores (so the compiler never has to wait for them), the other one looks escaped
                // residuals up in the container when their list did not fit LDS.
                auto row_loop = [&](auto slow_tag, auto pow2_tag) {
                    constexpr bool SLOW = decltype(slow_tag)::value;
                    constexpr bool POW2 = decltype(pow2_tag)::value;
                    for (uint32_t h = 0; h < rows; ++h) {
                        int32_t carry = 0;
#pragma unroll
                        for (int s = 0; s < NSEG; ++s) {
                            const uint32_t w = wl + (uint32_t)s * kWave;
                            const bool on = slot_on && w < W;
                            const uint32_t e = e_row0 + h * W + w;
                            const uint32_t ce = e - tile_e0;
                            const uint32_t entry = POW2 ? ce + ((ce >> log2S) << 1) : ce + 2u * (ce / S);
                            int32_t d = on ? (int32_t)tile[entry] : 0;
                            const bool is_esc = d == kEscape;
                            const uint64_t any_esc = __ballot(is_esc);
                            if (any_esc) {                            // wavefront-uniform
                                const uint64_t m = any_esc & slot_mask;
                                if (is_esc) {
                                    if (SLOW) {
                                        const uint32_t key = 2u * e;
                                        uint32_t lo = r_begin, hi = r_end;
                                        while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (rec[2 * (size_t)mid] < key) lo = mid + 1; else hi = mid; }
                                        d = (lo < r_end && rec[2 * (size_t)lo] == key) ? (int32_t)rec[2 * (size_t)lo + 1] : 0;
                                    } else {
                                        uint32_t pos = cur + (uint32_t)__popcll(m & lt_mask);
                                        if (pos >= kDsStageWords / 2u) pos = kDsStageWords / 2u - 1u;   // corrupt container only
                                        d = n_esc ? (int32_t)stage[2 * pos + 1] : 0;
                                    }
                                }
                                cur += (uint32_t)__popcll(m);
                            }
                            int32_t rp;
                            rp = run_scan<MODE>(d, wl, W);
                            rp = (int32_t)((uint32_t)rp + (uint32_t)carry);
                            if (NSEG > 1) carry = __builtin_amdgcn_readlane(rp, 63);
                            q[s] = (int32_t)((uint32_t)q[s] + (uint32_t)rp);
                            float v = (float)q[s] * ebx2;
                            if (fabsf(v) <= eb) v = 0.0f;
                            if (on) a.out[e] = v;
                        }
                    }
                };
                if (!esc_in_lds) row_loop(std::true_type{}, std::false_type{});
                else if (pow2) row_loop(std::false_type{}, std::true_type{});
                else row_loop(std::false_type{}, std::false_type{});
            }
            COMET_ACC(a.ctl, 15);

            // ---- 5. verbatim values overwrite what was just stored ----
            if (has_verbatim) {
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");  // the lattice values of this wavefront must have landed first
                // (workgroup scope waits for the stores; a wider scope would also write back and invalidate the L2)
                for (uint32_t k = r_begin + lane; k < r_end; k += kWave) {
                    const uint32_t key = rec[2 * (size_t)k];
                    if (key & 1u) {
                        float v = __uint_as_float(rec[2 * (size_t)k + 1]);
                        if (fabsf(v) <= eb) v = 0.0f;
                        const uint32_t e = key >> 1;
                        if (e >= e0 && e < e1) a.out[e] = v;
                    }
                }
            }
            wave_lds_fence();
            COMET_ACC(a.ctl, 16);
        }
    }
}

template __global__ void k_decode_scan<1, 0>(DsArgs);
template __global__ void k_decode_scan<1, 1>(DsArgs);
template __global__ void k_decode_scan<1, 2>(DsArgs);
template __global__ void k_decode_scan<2, 2>(DsArgs);
template __global__ void k_decode_scan<4, 2>(DsArgs);
template __global__ void k_decode_scan<8, 2>(DsArgs);

}  // namespace comet
