// Chunked Huffman encode (COMET Sec. 4.1, last step of the modified cuSZ
// pipeline), wavefront-cooperative.  A wavefront takes 256 consecutive codes per
// step, four per lane (one 8-byte load), so a chunk of 64 / 128 / 256 symbols is
// a group of 16 / 32 / 64 adjacent lanes.  Every lane looks up (code word, length)
// for its four codes; a DPP prefix sum of the lengths inside the lane group gives
// the bit position of each code word inside its chunk; the lanes OR their pieces
// into the chunk's words in LDS (most significant bit first); the words of the
// step's chunks, contiguous in the payload, leave with one coalesced store.
// No per-lane serial chain, coalesced input and output, 2 KB of LDS per wavefront.
//
// Placement is deterministic and needs no spinning: two kernels over the same
// segmentation of the chunks (one workgroup per segment).
//   k_encode_count: word count of every chunk (lengths only); per segment the
//                   exclusive scan of its counts -> chunk_off (segment-relative)
//                   and the segment's total.
//   k_encode_pack : a segment's base is the sum of the totals of the segments in
//                   front of it; chunk_off becomes absolute; the chunks are
//                   encoded and written at their final place.
// Neither kernel fences or counts finished workgroups: a device-scope release writes back and
// invalidates the L2 of the issuing XCD, which costs far more than the kernel boundary that
// orders these two kernels.  The last segment's workgroup of the pack kernel seals the container
// header: the payload size it computes decides everything the header still lacks.
// The encode table ((code << 6) | length per symbol) is cached in LDS for the
// bins around the centre; other symbols are looked up in global memory.
#include <type_traits>

#include "comet_kernels.h"
#include "comet_encode.h"

namespace comet {

namespace {

// Four consecutive codes of this lane (symbols i0 .. i0+3) as two packed words, 0 past the end
// (the caller masks those positions: every 16-bit value can be a code of the largest alphabet).
__device__ inline uint2 load4(const uint16_t *codes, uint64_t i0, uint64_t n) {
    if (i0 + 4u <= n) return *reinterpret_cast<const uint2 *>(codes + i0);
    uint32_t c[4];
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) c[j] = (i0 + j < n) ? (uint32_t)codes[i0 + j] : 0u;
    return make_uint2(c[0] | (c[1] << 16), c[2] | (c[3] << 16));
}
// The codes of kEncUnroll consecutive steps (256 symbols each) from step st0 of the segment that
// starts at chunk c_lo.  All arguments but `lane` are wavefront-uniform: the usual case, every step
// inside the segment and the tensor, is one branch and kEncUnroll plain loads.
template <int S>
__device__ inline void fetch_steps(const uint16_t *codes, uint64_t n, uint32_t c_lo, uint32_t st0, uint32_t steps, uint32_t lane,
                                   uint2 (&v)[kEncUnroll]) {
    const uint64_t e0 = (uint64_t)c_lo * S + (uint64_t)st0 * 256u;
    if (st0 + kEncUnroll <= steps && e0 + 256u * kEncUnroll <= n) {
        const uint2 *src = reinterpret_cast<const uint2 *>(codes + e0) + lane;
#pragma unroll
        for (uint32_t u = 0; u < kEncUnroll; ++u) v[u] = src[u * kWave];
    } else {
#pragma unroll
        for (uint32_t u = 0; u < kEncUnroll; ++u)
            v[u] = (st0 + u < steps) ? load4(codes, e0 + u * 256u + lane * 4u, n) : make_uint2(0, 0);
    }
}
}  // namespace

// ---------------------------------------------------------------------------
template <int S, bool FULLTBL>
__global__ __launch_bounds__(kEncBlock) void k_encode_count(EncodeArgs a) {
    constexpr int LPC = S / 4;                       // lanes per chunk
    constexpr int CPS = 256 / S;                     // chunks per wavefront step
    extern __shared__ uint64_t s_dyn_enc[];
    uint64_t *s_tbl = s_dyn_enc;                                                // a.tbl_n entries and a zero entry
    uint32_t *s_cnt = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(s_dyn_enc) + a.tbl_room);   // a.seg_chunks word counts
    __shared__ uint32_t s_part32[kEncBlock / kWave];

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));   // a scalar: what derives from it stays scalar
    // (behind the cached entries: a zero entry, or the escape symbol's if part of the table is cached)
    // Part of the table cached, symbols that occur outside it, but all of them inside the wider range of lengths
    // alone: those are cached instead (in the room of the entries; the launch has made it large enough for either).
    const bool lengths_only = !FULLTBL && a.len8 && a.tbl_n == kEncTableMax && !a.ctl->enc_in_window && a.ctl->len_in_window;
    const uint32_t lenw_n = enc_len_window(a.nbins), lenw_lo = (a.nbins - lenw_n) / 2u;
    if (lengths_only) {
        uint8_t *s_len8 = reinterpret_cast<uint8_t *>(s_tbl);
        for (uint32_t i = tid; i <= lenw_n; i += kEncBlock) s_len8[i] = (i < lenw_n) ? a.len8[lenw_lo + i] : a.len8[0];
    } else {
        for (uint32_t i = tid; i <= a.tbl_n; i += kEncBlock) s_tbl[i] = (i < a.tbl_n) ? a.enc[a.tbl_lo + i] : (FULLTBL ? 0ull : a.enc[0]);
    }
    __syncthreads();

    const uint32_t seg = blockIdx.x;
    const uint32_t c_lo = seg * a.seg_chunks;
    const uint32_t c_hi = (c_lo + a.seg_chunks < a.n_chunks) ? c_lo + a.seg_chunks : a.n_chunks;
    const uint32_t nc = c_hi - c_lo;                 // seg_chunks is a multiple of the chunks per step
    const uint32_t steps = (nc + CPS - 1u) / CPS;
    const uint32_t g = lane / LPC;                   // my chunk inside a step

    // The loop over the steps, once per way of looking a code up (the choice is the same for every thread).
    auto sweep = [&](auto tbl) {
    // kEncUnroll steps per iteration, their loads issued together
    for (uint32_t st0 = wave * kEncUnroll; st0 < steps; st0 += (kEncBlock / kWave) * kEncUnroll) {
        uint2 v[kEncUnroll];
        fetch_steps<S>(a.codes, a.n, c_lo, st0, steps, lane, v);
#pragma unroll
        for (uint32_t u = 0; u < kEncUnroll; ++u) {
            if (st0 + u >= steps) break;
            const uint32_t c0 = c_lo + (st0 + u) * CPS;
            const uint64_t e0 = (uint64_t)c0 * S;                           // first symbol of the step (uniform)
            uint32_t bits = 0;
            if (e0 + 256u <= a.n) {                                         // every symbol of the step exists (uniform)
#pragma unroll
                for (int j = 0; j < 4; ++j) bits += tbl.length(code_of(v[u], j));
            } else {
                const uint32_t left = (a.n > e0) ? (uint32_t)(a.n - e0) : 0u;
#pragma unroll
                for (int j = 0; j < 4; ++j) bits += (lane * 4u + (uint32_t)j < left) ? tbl.length(code_of(v[u], j)) : 0u;
            }
            if (a.zero_pair) {                                               // (uniform)
                const uint32_t left = (e0 + 256u <= a.n) ? 256u : ((a.n > e0) ? (uint32_t)(a.n - e0) : 0u);
                if (chunk_is_centre_only<LPC>(v[u], a.zero_pair, lane, left)) bits = 0;
            }
            const uint32_t incl = group_incl_scan<LPC>(bits);
            if ((lane % LPC) == LPC - 1 && c0 + g < c_hi) s_cnt[c0 + g - c_lo] = (incl + 31u) >> 5;
        }
    }
    };
    if (FULLTBL) sweep(TableView<1>{s_tbl, a.enc, a.tbl_lo, a.tbl_n, a.nbins});
    else if (a.ctl->enc_in_window) sweep(TableView<2>{s_tbl, a.enc, a.tbl_lo, a.tbl_n, a.nbins});
    else if (lengths_only) sweep(LengthView{reinterpret_cast<const uint8_t *>(s_tbl), lenw_lo, lenw_n});
    else sweep(TableView<0>{s_tbl, a.enc, a.tbl_lo, a.tbl_n, a.nbins});
    __syncthreads();

    // counts -> segment-relative exclusive offsets, kEncBlock consecutive chunks at a time
    uint32_t running = 0;
    for (uint32_t base = 0; base < nc; base += kEncBlock) {
        const uint32_t idx = base + tid;
        const uint32_t cnt = (idx < nc) ? s_cnt[idx] : 0u;
        uint32_t tot;
        const uint32_t ex = block_excl_scan<uint32_t, kEncBlock / kWave>(cnt, s_part32, tot);
        if (idx < nc) a.chunk_off[c_lo + idx] = running + ex;
        running += tot;
    }
    if (tid == 0) a.desc[seg] = running;             // words of this segment
}

// ---------------------------------------------------------------------------
template <int S, bool FULLTBL>
__global__ __launch_bounds__(kEncBlock) void k_encode_pack(EncodeArgs a) {
    constexpr int LPC = S / 4;
    constexpr int CPS = 256 / S;
    extern __shared__ uint64_t s_dyn_enc[];
    uint64_t *s_tbl = s_dyn_enc;                                                // a.tbl_n entries and a zero entry
    uint32_t *s_buf = reinterpret_cast<uint32_t *>(s_dyn_enc + a.tbl_n + 1u);   // one assembly buffer per wavefront
    __shared__ uint64_t s_part64[kEncBlock / kWave];

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));   // a scalar: what derives from it stays scalar
    for (uint32_t i = tid; i <= a.tbl_n; i += kEncBlock) s_tbl[i] = (i < a.tbl_n) ? a.enc[a.tbl_lo + i] : (FULLTBL ? 0ull : a.enc[0]);
    uint32_t *buf = s_buf + wave * kEncBufWords;
    for (uint32_t i = lane; i < kEncBufWords; i += kWave) buf[i] = 0;

    uint32_t *payload;
    uint64_t cap_words;
    if (a.container) {
        const uint64_t off = a.ctl->off_payload;
        payload = reinterpret_cast<uint32_t *>(a.container + off);
        cap_words = (a.capacity >= off) ? (a.capacity - off) / 4u : 0u;
    } else {
        payload = a.payload;
        cap_words = a.payload_cap_words;
    }

    const uint32_t seg = blockIdx.x;
    const uint32_t c_lo = seg * a.seg_chunks;
    const uint32_t c_hi = (c_lo + a.seg_chunks < a.n_chunks) ? c_lo + a.seg_chunks : a.n_chunks;
    const uint32_t nc = c_hi - c_lo;
    const uint32_t steps = (nc + CPS - 1u) / CPS;
    const uint32_t g = lane / LPC;

    // words of all segments in front of mine
    uint64_t sum = 0;
    for (uint32_t i0 = 0; i0 < seg; i0 += 8u * kEncBlock) {              // eight loads in flight per thread
        uint64_t v[8];
#pragma unroll
        for (uint32_t j = 0; j < 8; ++j) {
            const uint32_t idx = i0 + j * kEncBlock + tid;
            v[j] = (idx < seg) ? a.desc[idx] : 0ull;
        }
#pragma unroll
        for (uint32_t j = 0; j < 8; ++j) sum += v[j];
    }
    uint64_t base;
    (void)block_excl_scan<uint64_t, kEncBlock / kWave>(sum, s_part64, base);
    bool overflow = false;
    if (seg + 1u == gridDim.x && tid == 0) {
        const uint64_t pw = base + a.desc[seg];
        a.ctl->payload_words = pw;
        if (a.payload_words_out) *a.payload_words_out = pw;
        if (pw > 0xffffffffull) overflow = true;      // chunk offsets are 32-bit word indices
        if (a.container && a.latched) {
            // The thread that knows the payload size also seals the container header (no kernel of its
            // own for that): the only bit this kernel can raise is the capacity bit, and whether any
            // workgroup raises it follows from the size.
            Header *h = reinterpret_cast<Header *>(a.container);
            const uint64_t total = a.ctl->off_payload + 4ull * pw;
            uint32_t stt = a.ctl->status;             // what the kernels before this one raised
            if (overflow || total > a.capacity) stt |= (uint32_t)ST_CAPACITY;
            h->payload_words = pw;
            h->total_bytes = total;
            h->status = stt ? 1u : 0u;
            a.ctl->total_bytes = total;
            if (stt) atomicOr(a.latched, stt);        // folded into the context's persistent word
        }
    }
    __syncthreads();                                  // table and buffers ready

    // A wavefront handles kEncUnroll steps per iteration: their words are contiguous in the
    // payload, so they are assembled side by side in the buffer and leave together.  The codes and
    // the offset of an iteration are fetched one iteration ahead, before the stores of the current
    // one are issued: memory operations retire in order, so a load issued after a store could not
    // be consumed before that store has completed.
    auto fetch = [&](uint32_t st0, uint2 (&v)[kEncUnroll], uint32_t &off) {
        fetch_steps<S>(a.codes, a.n, c_lo, st0, steps, lane, v);
        off = a.chunk_off[c_lo + st0 * CPS];
    };
    auto flush = [&](uint64_t off0, uint32_t n_words) {
        wave_lds_fence();
        for (uint32_t k = lane; k < n_words; k += kWave) {
            const uint32_t word = buf[k];
            buf[k] = 0;
            if (off0 + k < cap_words) payload[off0 + k] = word;
            else overflow = true;
        }
        wave_lds_fence();
    };
    constexpr uint32_t kStride = (kEncBlock / kWave) * kEncUnroll;
    // The loop over the steps, once per way of looking a code up (the choice is the same for every thread), and once
    // more for the tensor's last segment: everywhere else every step has its 256 symbols, and the loop tests nothing.
    auto sweep = [&](auto tbl, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    uint32_t st0 = wave * kEncUnroll;
    uint2 v_next[kEncUnroll];
    uint32_t off_next = 0;
    if (st0 < steps) fetch(st0, v_next, off_next);
    for (; st0 < steps; st0 += kStride) {
        uint2 v[kEncUnroll];
#pragma unroll
        for (uint32_t u = 0; u < kEncUnroll; ++u) v[u] = v_next[u];
        uint64_t off0 = base + off_next;
        if (st0 + kStride < steps) fetch(st0 + kStride, v_next, off_next);
        uint32_t wpos = 0;                           // words assembled in the buffer so far
#pragma unroll
        for (uint32_t u = 0; u < kEncUnroll; ++u) {
            if (st0 + u >= steps) break;
            uint32_t left = 256u;
            if (TAIL) {
                const uint64_t e0 = (uint64_t)(c_lo + (st0 + u) * CPS) * S;    // first symbol of the step (uniform)
                left = (e0 + 256u <= a.n) ? 256u : ((a.n > e0) ? (uint32_t)(a.n - e0) : 0u);
            }
            uint64_t cw[4];
            uint32_t len[4], bits = 0;
            uint64_t acc = 0;                                // my code words one after the other (if they fit 64 bits)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint64_t e = tbl.full(code_of(v[u], j));
                if (TAIL && __builtin_expect(left < 256u, 0)) {      // wavefront-uniform; only the last step of the tensor
                    asm volatile("" ::: "memory");           // keep this a branch: as selects it would cost every step
                    e = (lane * 4u + (uint32_t)j < left) ? e : 0ull;
                }
                len[j] = (uint32_t)e & 63u;
                cw[j] = e >> 6;
                bits += len[j];
                acc = (acc << len[j]) | cw[j];
            }
            // a chunk of nothing but centre codes takes no words: its lanes place a string of no bits
            if (a.zero_pair && chunk_is_centre_only<LPC>(v[u], a.zero_pair, lane, left)) bits = 0;      // (the test on zero_pair is uniform)
            const uint32_t incl = group_incl_scan<LPC>(bits);
            // words of every chunk of the step, and where each chunk's words start inside the buffer
            uint32_t wbase = 0, total_words = 0;
#pragma unroll
            for (int k = 0; k < CPS; ++k) {
                const uint32_t wk = ((uint32_t)__builtin_amdgcn_readlane((int)incl, k * LPC + LPC - 1) + 31u) >> 5;
                if ((uint32_t)k == g) wbase = total_words;
                total_words += wk;
            }
            if (wpos + total_words + 4u > kEncBufWords) {       // only with very long code words
                flush(off0, wpos);
                off0 += wpos;
                wpos = 0;
            }
            uint32_t p = (wpos + wbase) * 32u + incl - bits;   // bit position of my first code word inside the buffer
            // A bit string of L <= 64 bits, left-aligned in t, goes to bit p of the word stream: at most
            // three words.  The second OR is unconditional (a branch around it costs more than an OR of
            // zero; the buffer has spare words behind the step), the third is rare.
            auto place = [&](uint64_t t, uint32_t L, uint32_t at) {
                const uint32_t sh = at & 31u, w = at >> 5;
                const uint64_t hi = t >> sh;
                atomicOr(&buf[w], (uint32_t)(hi >> 32));
                atomicOr(&buf[w + 1], (uint32_t)hi);
                if (L + sh > 64u) atomicOr(&buf[w + 2], (uint32_t)((t << (64u - sh)) >> 32));
            };
            if (bits <= 64u) {
                // the usual case: my four code words as one string (a shift by 64 - 0 leaves zero bits: nothing is set)
                place(bits ? acc << (64u - bits) : 0ull, bits, p);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t L = len[j];
                    if (L) place(cw[j] << (64u - L), L, p);
                    p += L;
                }
            }
            wpos += total_words;
        }
        flush(off0, wpos);
    }
    };
    const bool whole = (uint64_t)c_hi * S <= a.n;              // every chunk of my segment has all its symbols
    auto sweep_with = [&](auto tbl) {
        if (whole) sweep(tbl, std::false_type{}); else sweep(tbl, std::true_type{});
    };
    if (FULLTBL) sweep_with(TableView<1>{s_tbl, a.enc, a.tbl_lo, a.tbl_n, a.nbins});
    else if (a.ctl->enc_in_window) sweep_with(TableView<2>{s_tbl, a.enc, a.tbl_lo, a.tbl_n, a.nbins});
    else sweep_with(TableView<0>{s_tbl, a.enc, a.tbl_lo, a.tbl_n, a.nbins});
    // chunk offsets become absolute (every wavefront has consumed the relative ones of its steps
    // only after this barrier)
    __syncthreads();
    for (uint32_t idx = tid; idx < nc; idx += kEncBlock) a.chunk_off[c_lo + idx] = (uint32_t)(base + a.chunk_off[c_lo + idx]);
    if (overflow) atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);

}

// ---------------------------------------------------------------------------
// Single-pass compression, last step.  The quantise kernel has left the words of every run of
// rows in a work area, with chunk offsets relative to the run, and k_gather_records the number
// of outlier records, which decides where the payload starts.  One wavefront per run: the words
// in front of the run are added up (the counts of all runs in front of the workgroup, by the
// whole workgroup), the run's words are copied to their place and its chunk offsets made
// absolute.  The wavefront of the last run seals the header.  Nothing is copied if an earlier
// kernel of the call has raised an error.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kPlaceBlock) void k_place_payload(PlaceArgs a) {
    constexpr int kWaves = kPlaceBlock / kWave;
    __shared__ uint64_t s_part64[kWaves];
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));
    const uint32_t run0 = blockIdx.x * kWaves, run = run0 + wave;

    uint64_t sum = 0;
    for (uint32_t i0 = 0; i0 < run0; i0 += 8u * kPlaceBlock) {            // eight loads in flight per thread
        uint32_t v[8];
#pragma unroll
        for (uint32_t j = 0; j < 8; ++j) {
            const uint32_t i = i0 + j * kPlaceBlock + tid;
            v[j] = (i < run0) ? a.run_words[i] : 0u;
        }
#pragma unroll
        for (uint32_t j = 0; j < 8; ++j) sum += v[j];
    }
    uint64_t base;
    (void)block_excl_scan<uint64_t, kWaves>(sum, s_part64, base);
    uint32_t mine = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t c = (run0 + (uint32_t)w < a.n_runs) ? a.run_words[run0 + w] : 0u;
        if ((uint32_t)w < wave) base += c;
        if ((uint32_t)w == wave) mine = c;
    }
    if (run >= a.n_runs) return;

    Header *h = reinterpret_cast<Header *>(a.container);
    const uint64_t n_rec = a.ctl->n_rec;
    const uint64_t rec_end = h->off_outlier + 8ull * n_rec;
    const uint64_t off_payload = align16(rec_end);
    const uint32_t earlier = a.ctl->status;                  // what the kernels before this one raised
    const uint64_t pw_mine = base + mine;
    if (run + 1u == a.n_runs && lane == 0) {
        uint32_t stt = earlier;
        const uint64_t total = off_payload + 4ull * pw_mine;
        if (pw_mine > 0xffffffffull || total > a.capacity) stt |= (uint32_t)ST_CAPACITY;   // (chunk offsets are 32-bit word indices)
        h->n_rec = (uint32_t)n_rec;
        h->n_vrec = (uint32_t)a.ctl->n_vrec;
        h->nnz = a.ctl->nnz;
        h->off_payload = off_payload;
        h->payload_words = pw_mine;
        h->total_bytes = total;
        h->status = stt ? 1u : 0u;
        a.ctl->off_payload = off_payload;
        a.ctl->payload_words = pw_mine;
        a.ctl->total_bytes = total;
        if (off_payload <= a.capacity)
            for (uint64_t o = rec_end; o < off_payload; ++o) a.container[o] = 0;     // padding behind the records
        if (stt) {
            atomicOr(&a.ctl->status, stt);
            atomicOr(a.latched, stt);
        }
    }
    if (earlier) return;
    const uint64_t cap_words = (a.capacity >= off_payload) ? (a.capacity - off_payload) / 4u : 0u;
    const uint64_t row_lo = (uint64_t)run * a.rows_per_wave;
    uint64_t row_hi = row_lo + a.rows_per_wave;
    if (row_hi > a.rows_total) row_hi = a.rows_total;
    const uint64_t e_lo = row_lo * a.W, e_hi = row_hi * a.W;
    uint32_t *payload = reinterpret_cast<uint32_t *>(a.container + off_payload);
    const uint32_t *src = a.work_words + e_lo / 2u;
    for (uint32_t i = lane; i < mine; i += kWave)
        if (base + i < cap_words) payload[base + i] = src[i];
    uint32_t *chunk_off = reinterpret_cast<uint32_t *>(a.container + h->off_chunk);
    const uint32_t c_lo = (uint32_t)(e_lo / a.chunk_syms), c_hi = (uint32_t)((e_hi + a.chunk_syms - 1u) / a.chunk_syms);
    for (uint32_t c = c_lo + lane; c < c_hi; c += kWave) chunk_off[c] = (uint32_t)(base + chunk_off[c]);
}

#define COMET_INST_ENC(S)                                                  \
    template __global__ void k_encode_count<S, true>(EncodeArgs);          \
    template __global__ void k_encode_count<S, false>(EncodeArgs);         \
    template __global__ void k_encode_pack<S, true>(EncodeArgs);           \
    template __global__ void k_encode_pack<S, false>(EncodeArgs);
COMET_INST_ENC(64)
COMET_INST_ENC(128)
COMET_INST_ENC(256)
#undef COMET_INST_ENC

}  // namespace comet
