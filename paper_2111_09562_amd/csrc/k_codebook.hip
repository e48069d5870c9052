// Codebook kernels (COMET Sec. 4.1, "customized Huffman coding"):
//   k_codebook       histogram -> Huffman code lengths -> canonical codes -> encode
//                    table; also lays out the container (header, section offsets).
//   k_decode_tables  length table -> canonical decode tables; validates a header.
// One workgroup each: the work is a few thousand symbols at most and sits on the
// critical path between the two streaming kernels, so it is latency- not
// bandwidth-bound.  Alphabets up to kBookLdsSyms live entirely in LDS.
//
// Length rule (must give exactly one answer): leaves ordered by (frequency,
// symbol); two queues; at every step the two smallest heads are merged, the leaf
// first when a leaf and an internal node weigh the same; internal nodes are
// consumed in creation order.
#include "comet_kernels.h"

namespace comet {

namespace {

// Ascending bitonic sort of n2 (power of two) 64-bit keys by the whole workgroup.
__device__ void bitonic_sort(uint64_t *keys, uint32_t n2) {
    for (uint32_t k = 2; k <= n2; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = threadIdx.x; i < n2; i += blockDim.x) {
                const uint32_t p = i ^ j;
                if (p > i) {
                    const uint64_t x = keys[i], y = keys[p];
                    const bool asc = (i & k) == 0;
                    if ((x > y) == asc) { keys[i] = y; keys[p] = x; }
                }
            }
            __syncthreads();
        }
    }
}

__device__ inline uint32_t next_pow2(uint32_t v) {
    uint32_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Canonical first codes per length from the per-length symbol counts; returns
// false if the lengths are not a complete prefix code (or a single 1-bit code).
__device__ bool canonical_first_codes(const uint32_t *cnt, uint32_t n_active, uint64_t *first_code,
                                      uint32_t *first_index, uint32_t *max_len_out, uint32_t *min_len_out) {
    uint64_t c = 0;
    uint32_t idx = 0, max_len = 0, min_len = 0;
    bool ok = true;
    for (uint32_t L = 1; L <= 64; ++L) {
        c <<= 1;                       // first code of length L = (first of L-1 + count of L-1) * 2
        first_code[L] = c;
        first_index[L] = idx;
        if (cnt[L]) {
            if (!min_len) min_len = L;
            max_len = L;
            if (L < 64 && c + cnt[L] > (1ull << L)) ok = false;
            c += cnt[L];
            idx += cnt[L];
        }
    }
    if (idx != n_active || max_len == 0 || max_len > 57) ok = false;
    if (ok && n_active > 1) {
        // completeness: one past the last code of the longest length is 2^max_len
        uint64_t end = first_code[max_len] + cnt[max_len];
        if (end != (1ull << max_len)) ok = false;
    }
    if (ok && n_active == 1 && max_len != 1) ok = false;
    *max_len_out = max_len;
    *min_len_out = min_len;
    return ok;
}

}  // namespace

__global__ __launch_bounds__(kBookBlock) void k_codebook(BookArgs a) {
    __shared__ uint64_t s_keys[kBookLdsSyms];
    __shared__ uint64_t s_iw[kBookLdsSyms];
    __shared__ uint32_t s_lp[kBookLdsSyms];
    __shared__ uint32_t s_ip[kBookLdsSyms];
    __shared__ uint32_t s_part[kBookBlock / kWave];
    __shared__ uint32_t s_cnt[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint32_t s_findex[65];
    __shared__ uint32_t s_maxlen;

    const uint32_t tid = threadIdx.x;
    const uint32_t nbins = a.nbins;
    const bool in_lds = nbins <= kBookLdsSyms;
    uint64_t *keys = in_lds ? s_keys : a.scratch.keys;
    uint64_t *iw = in_lds ? s_iw : a.scratch.iw;
    uint32_t *leaf_parent = in_lds ? s_lp : a.scratch.leaf_parent;
    uint32_t *int_parent = in_lds ? s_ip : a.scratch.int_parent;

    if (tid < 65) s_cnt[tid] = 0;
    if (tid == 0) s_maxlen = 0;

    // ---- 1. compact the active symbols into sort keys (frequency << 16 | symbol) ----
    uint32_t m = 0;
    for (uint32_t base = 0; base < nbins; base += kBookBlock) {
        const uint32_t s = base + tid;
        const uint32_t f = (s < nbins) ? a.hist[s] : 0u;
        uint32_t tot;
        const uint32_t pos = block_excl_scan<uint32_t, kBookBlock / kWave>(f ? 1u : 0u, s_part, tot);
        if (f) keys[m + pos] = ((uint64_t)f << 16) | s;
        else if (s < nbins) {           // unused symbol: length 0 everywhere
            a.len_out[s] = 0;
            a.enc[s] = 0;
            if (a.code_out) a.code_out[s] = 0;
        }
        m += tot;
    }
    const uint32_t m2 = next_pow2(m > 1 ? m : 2);
    for (uint32_t i = m + tid; i < m2; i += kBookBlock) keys[i] = ~0ull;
    __syncthreads();

    // ---- 2. leaves in (frequency, symbol) order ----
    bitonic_sort(keys, m2);

    // ---- 3. two-queue merge (one lane; m-1 dependent steps) ----
    if (m >= 2 && tid == 0) {
        uint32_t li = 0, ii = 0, ni = 0;
        for (uint32_t step = 0; step + 1 < m; ++step) {
            uint64_t sum = 0;
#pragma unroll
            for (int pick = 0; pick < 2; ++pick) {
                bool take_leaf;
                const uint64_t lw = (li < m) ? (keys[li] >> 16) : ~0ull;
                if (li < m && ii < ni) take_leaf = (lw <= iw[ii]);
                else take_leaf = (li < m);
                if (take_leaf) { sum += lw; leaf_parent[li] = ni; ++li; }
                else { sum += iw[ii]; int_parent[ii] = ni; ++ii; }
            }
            iw[ni++] = sum;
        }
    }
    __syncthreads();

    // ---- 4. depth of every leaf: walk to the root (node m-2) ----
    for (uint32_t i = tid; i < m; i += kBookBlock) {
        const uint32_t sym = (uint32_t)(keys[i] & 0xffffu);
        uint32_t depth = 1;
        if (m >= 2) {
            uint32_t p = leaf_parent[i];
            const uint32_t root = m - 2;
            while (p != root && depth < 66u) { p = int_parent[p]; ++depth; }
        }
        keys[i] = ((uint64_t)depth << 16) | sym;     // re-keyed for the canonical order
        atomicAdd(&s_cnt[depth > 64 ? 64 : depth], 1u);
        atomicMax(&s_maxlen, depth);
    }
    __syncthreads();

    // ---- 5. canonical order (length, symbol) ----
    bitonic_sort(keys, m2);
    if (tid == 0) {
        uint32_t mx, mn;
        const bool ok = (m == 0) || canonical_first_codes(s_cnt, m, s_first, s_findex, &mx, &mn);
        if (!ok) atomicOr(&a.ctl->status, (uint32_t)ST_INTERNAL);
    }
    __syncthreads();

    // ---- 6. codes and tables ----
    for (uint32_t p = tid; p < m; p += kBookBlock) {
        const uint32_t L = (uint32_t)(keys[p] >> 16);
        const uint32_t sym = (uint32_t)(keys[p] & 0xffffu);
        const uint64_t code = s_first[L > 64 ? 64 : L] + (p - s_findex[L > 64 ? 64 : L]);
        a.len_out[sym] = (uint8_t)L;
        a.enc[sym] = (code << 6) | (uint64_t)(L & 63u);
        if (a.code_out) a.code_out[sym] = code;
    }

    // ---- 7. container layout ----
    if (tid == 0) {
        a.ctl->n_active = m;
        a.ctl->max_len = s_maxlen;
        if (a.hdr) {
            Header h = a.proto;
            h.n_active = m;
            h.max_len = s_maxlen;
            h.n_rec = (uint32_t)a.ctl->n_rec;
            h.n_vrec = (uint32_t)a.ctl->n_vrec;
            h.nnz = a.ctl->nnz;
            h.off_payload = align16(h.off_outlier + 8ull * a.ctl->n_rec);
            h.payload_words = 0;
            h.total_bytes = 0;
            h.status = 1;                      // overwritten by the encode kernel's last workgroup
            a.ctl->off_payload = h.off_payload;
            if (h.off_payload > a.capacity) atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
            *a.hdr = h;
            // zero the padding between sections
            uint8_t *base = reinterpret_cast<uint8_t *>(a.hdr);
            for (uint64_t o = h.off_len + nbins; o < h.off_chunk; ++o) base[o] = 0;
            for (uint64_t o = h.off_chunk + 4ull * h.n_chunks; o < h.off_outlier; ++o) base[o] = 0;
            if (h.off_payload <= a.capacity)
                for (uint64_t o = h.off_outlier + 8ull * a.ctl->n_rec; o < h.off_payload; ++o) base[o] = 0;
        }
    }
}

// ---------------------------------------------------------------------------
// Decode tables from a length table.  Also checks a container header against
// the shape the caller passed; any inconsistency latches ST_FORMAT, which makes
// the reconstruct kernel do nothing.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBookBlock) void k_decode_tables(TablesArgs a) {
    __shared__ uint32_t s_part[kBookBlock / kWave];
    __shared__ uint32_t s_cnt[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint64_t s_limit[65];
    __shared__ uint32_t s_findex[65];
    __shared__ uint32_t s_ok, s_maxlen, s_nbins;

    const uint32_t tid = threadIdx.x;
    if (tid == 0) {
        uint32_t ok = 1;
        s_nbins = a.nbins;
        if (a.hdr) {
            const Header h = *a.hdr;
            const Header &e = a.expect;
            const uint64_t n = (uint64_t)e.N * e.C * e.H * e.W;
            if (a.bytes < kHeaderBytes) ok = 0;
            if (h.magic != kMagic || h.version != 1u || h.status != 0u) ok = 0;
            if (h.N != e.N || h.C != e.C || h.H != e.H || h.W != e.W) ok = 0;
            if (h.nbins < 4u || h.nbins > 65536u || (h.nbins & 1u)) ok = 0;
            s_nbins = h.nbins;
            if (h.chunk_syms == 0) ok = 0;
            const float eb = __uint_as_float(h.eb_bits);
            if (!(eb >= 0x1p-100f && eb <= 0x1p100f)) ok = 0;
            if (__float_as_uint(2.0f * eb) != h.ebx2_bits) ok = 0;
            if (ok) {
                const uint64_t n_chunks = (n + h.chunk_syms - 1u) / h.chunk_syms;
                if (h.n_chunks != n_chunks) ok = 0;
                if (h.off_len != kHeaderBytes || h.off_chunk != align16(h.off_len + h.nbins) ||
                    h.off_outlier != align16(h.off_chunk + 4ull * h.n_chunks) ||
                    h.off_payload != align16(h.off_outlier + 8ull * h.n_rec) ||
                    h.total_bytes != h.off_payload + 4ull * h.payload_words || h.total_bytes > a.bytes) ok = 0;
            }
        }
        s_ok = ok;
    }
    if (tid < 65) s_cnt[tid] = 0;
    __syncthreads();
    if (!s_ok) {
        if (tid == 0) atomicOr(&a.ctl->status, (uint32_t)ST_FORMAT);
        return;
    }
    const uint32_t nbins = s_nbins;
    uint64_t *keys = a.keys;

    // symbols with a code, keyed (length << 16 | symbol)
    uint32_t m = 0;
    bool bad = false;
    for (uint32_t base = 0; base < nbins; base += kBookBlock) {
        const uint32_t s = base + tid;
        const uint32_t L = (s < nbins) ? a.len[s] : 0u;
        if (L > 57u) bad = true;
        uint32_t tot;
        const uint32_t pos = block_excl_scan<uint32_t, kBookBlock / kWave>(L ? 1u : 0u, s_part, tot);
        if (L) { keys[m + pos] = ((uint64_t)L << 16) | s; atomicAdd(&s_cnt[L > 64u ? 64u : L], 1u); }
        m += tot;
    }
    const uint32_t m2 = next_pow2(m > 1 ? m : 2);
    for (uint32_t i = m + tid; i < m2; i += kBookBlock) keys[i] = ~0ull;
    if (__syncthreads_or(bad ? 1 : 0) || m == 0) {
        if (tid == 0) atomicOr(&a.ctl->status, (uint32_t)ST_FORMAT);
        return;
    }
    bitonic_sort(keys, m2);
    if (tid == 0) {
        uint32_t mx, mn;
        const bool ok = canonical_first_codes(s_cnt, m, s_first, s_findex, &mx, &mn);
        s_maxlen = mx;
        s_ok = ok ? 1u : 0u;
        if (ok) {
            for (uint32_t L = 1; L <= 64; ++L) {
                // exclusive upper bound, left-aligned; the longest length closes the code space
                uint64_t lim = 0;
                if (L < mx) lim = (s_first[L] + s_cnt[L]) << (64u - L);
                else lim = ~0ull;
                s_limit[L] = lim;
                a.t.limit[L] = lim;
                a.t.first_code[L] = s_first[L];
                a.t.first_index[L] = s_findex[L];
            }
            a.t.limit[0] = 0; a.t.first_code[0] = 0; a.t.first_index[0] = 0;
            a.t.meta[0] = mx; a.t.meta[1] = m; a.t.meta[2] = mn;
        }
    }
    __syncthreads();
    if (!s_ok) {
        if (tid == 0) atomicOr(&a.ctl->status, (uint32_t)ST_FORMAT);
        return;
    }
    for (uint32_t p = tid; p < m; p += kBookBlock) a.t.sorted[p] = (uint16_t)(keys[p] & 0xffffu);
    // look-up table on the next kLutBits bits
    const uint32_t mx = s_maxlen;
    for (uint32_t e = tid; e < kLutSize; e += kBookBlock) {
        const uint64_t v = (uint64_t)e << (64 - kLutBits);
        uint32_t entry = 0;
        const uint32_t top = mx < (uint32_t)kLutBits ? mx : (uint32_t)kLutBits;
        for (uint32_t L = 1; L <= top; ++L) {
            if (s_cnt[L] && (v < s_limit[L] || L == mx)) {
                uint64_t off = (v >> (64u - L)) - s_first[L];
                if (off >= s_cnt[L]) off = s_cnt[L] - 1u;      // only reachable with an invalid stream
                const uint32_t sym = (uint32_t)(keys[s_findex[L] + off] & 0xffffu);
                entry = (sym << 8) | L;
                break;
            }
        }
        a.t.lut[e] = entry;
    }
}

}  // namespace comet
