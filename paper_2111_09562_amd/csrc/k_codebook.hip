// Codebook kernels (COMET Sec. 4.1, "customized Huffman coding"):
//   k_codebook       histogram -> Huffman code lengths -> canonical codes -> encode
//                    table; also lays out the container (header, section offsets).
//   k_decode_tables  length table -> canonical decode tables; validates a header.
// One workgroup each: the work is a few thousand symbols at most and sits on the
// critical path between the two streaming kernels, so it is latency- not
// bandwidth-bound.  Alphabets up to kBookLdsSyms live entirely in LDS.  Larger ones:
//   k_book_sort_tiles, k_book_merge  the leaves in (frequency, symbol) order, by as many
//                    workgroups as the alphabet has tiles of 1024 symbols (a merge sort:
//                    tiles sorted in registers, then runs merged pairwise by ranking);
//                    k_codebook then merges in global memory while many items wait and
//                    finishes in LDS.
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

// Ascending bitonic sort of one key per lane over the first n2 (power of two,
// <= blockDim) lanes of the workgroup; keys stay in registers, partners closer
// than a wavefront are reached by shuffles, the others through LDS.
__device__ inline uint64_t bitonic_sort_regs(uint64_t key, uint64_t *s_x, uint32_t n2) {
    const uint32_t i = threadIdx.x;
    for (uint32_t k = 2; k <= n2; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            uint64_t other;
            if (j < (uint32_t)kWave) other = __shfl_xor(key, (int)j, kWave);
            else {
                s_x[i] = key;
                __syncthreads();
                other = s_x[i ^ j];
                __syncthreads();
            }
            const bool keep_min = ((i & k) == 0) == ((i & j) == 0);
            const uint64_t lo = key < other ? key : other, hi = key < other ? other : key;
            key = keep_min ? lo : hi;
        }
    }
    return key;
}

// arr[begin, end) is non-decreasing in (arr[i] >> shift); number of entries <= t
// (or < t when strict).  Gallops from the front: the answer is usually small.
__device__ inline uint32_t count_below(const uint64_t *arr, uint32_t begin, uint32_t end, uint64_t t, int shift, bool strict) {
    const uint32_t n = end - begin;
    uint32_t pos = 0, step = 1;
    auto ok = [&](uint32_t idx) { const uint64_t w = arr[begin + idx] >> shift; return strict ? (w < t) : (w <= t); };
    while (pos + step <= n && ok(pos + step - 1)) { pos += step; step <<= 1; }
    uint32_t lo = pos, hi = (pos + step - 1 < n) ? pos + step - 1 : n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (ok(mid)) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__device__ inline uint32_t next_pow2(uint32_t v) {
    uint32_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

__device__ inline uint64_t lane_value64_any(uint64_t v, uint32_t src) {      // src: wavefront-uniform
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, (int)src);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), (int)src);
    return ((uint64_t)hi << 32) | lo;
}

// Canonical first codes per length from the per-length symbol counts (cnt[1 .. 64]; 64 stands for
// every length the container cannot hold); returns false if the lengths are not a complete prefix
// code (or a single 1-bit code).  By one whole wavefront: every lane of it must call, the results
// are wavefront-uniform.  The first code of length L is (first code of L-1 + count of L-1) * 2,
// i.e. the sum over k < L of cnt[k] * 2^(L-k): lane L holds the count of length L and the first
// codes are an exclusive scan of the counts in units of 2^-57.  A table is a valid code exactly
// if no length above 57 is used, the Kraft sum does not exceed one, and it equals one unless the
// code has a single symbol (of length 1).
__device__ inline bool canonical_first_codes_wave(const uint32_t *cnt, uint32_t n_active, uint64_t *first_code,
                                                  uint32_t *first_index, uint32_t *max_len_out, uint32_t *min_len_out) {
    const uint32_t L = (uint32_t)lane_id();                  // lane 0 stands for no length; length 64 is looked at apart
    const uint32_t c = L ? cnt[L] : 0u;
    const uint32_t c64 = cnt[64];
    const uint64_t used = wave_ballot(c != 0u);
    // a count above 2^L alone breaks the Kraft inequality (and would overflow the sum below)
    const bool too_many = L && L < 17u && c > (1u << L);
    const bool too_long = (L > 57u && c != 0u);
    const bool broken = wave_ballot(too_many || too_long) != 0ull || c64 != 0u;
    const uint64_t term = (L && L <= 57u && !too_many) ? (uint64_t)c << (57u - L) : 0ull;
    const uint64_t incl = wave_incl_scan<uint64_t>(term);
    const uint32_t idx_incl = wave_incl_scan<uint32_t>(c);
    const uint64_t excl = incl - term;
    if (L) {
        first_code[L] = (L <= 57u) ? excl >> (57u - L) : excl << (L - 57u);
        first_index[L] = idx_incl - c;
    }
    const uint64_t kraft = lane_value64_any(incl, 63);       // in units of 2^-57
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)idx_incl, 63);
    if (L == 0u) { first_code[64] = lane_value64_any(excl, 63) << 7; first_index[64] = total; }   // (length 64 is never valid)
    const uint32_t max_len = c64 ? 64u : (used ? 63u - (uint32_t)__builtin_clzll(used) : 0u);
    const uint32_t min_len = used ? (uint32_t)__builtin_ctzll(used) : (c64 ? 64u : 0u);
    bool ok = !broken && total + c64 == n_active && max_len != 0u && max_len <= 57u && kraft <= (1ull << 57);
    if (ok && n_active > 1u && kraft != (1ull << 57)) ok = false;
    if (ok && n_active == 1u && max_len != 1u) ok = false;
    *max_len_out = max_len;
    *min_len_out = min_len;
    return ok;
}

}  // namespace


// The merge rounds.  NT lanes take part (a whole workgroup, or one wavefront when
// the arrays are in LDS and the rounds are short); `sync` is the barrier that
// matches NT.
//
// State: leaves [li, m) and internal nodes [ii, ni) not yet merged.  With t the sum
// of the two smallest heads, every new node weighs at least t, so every waiting item
// of weight <= t is merged before any node created now: those items, taken in merged
// order (leaf before node on equal weight) and paired consecutively, are exactly the
// next steps of the sequential two-queue construction.  An odd item out waits for the
// next round.  iw[0, m) must be zero on entry.
// Same count, by one whole wavefront probing 64 consecutive entries per step
// (the entries are sorted, so the lanes that pass form a prefix).
__device__ inline uint32_t count_below_wave(const uint64_t *arr, uint32_t begin, uint32_t end, uint64_t t, int shift) {
    uint32_t cnt = 0;
    const uint32_t lane = (uint32_t)lane_id();
    while (true) {
        const uint32_t idx = begin + cnt + lane;
        const bool ok = idx < end && (arr[idx] >> shift) <= t;
        const uint64_t mask = __ballot(ok);
        const uint32_t c = (~mask == 0ull) ? 64u : (uint32_t)(__ffsll((unsigned long long)~mask) - 1);
        cnt += c;
        if (c < 64u) break;
    }
    return cnt;
}

// The same count by a whole workgroup of kBookBlock threads (every thread must call; arrays in global memory):
// every thread probes one entry per step, kBookBlock entries evenly spread over what is left of the range, so
// two steps (two memory round trips) settle a range of a million entries, where the galloping search of one
// thread takes two dependent loads per bit of the answer.
__device__ inline uint32_t count_below_block(const uint64_t *arr, uint32_t begin, uint32_t end, uint64_t t, int shift) {
    uint32_t lo = begin, hi = end;                   // the first entry above t lies in [lo, hi]
    while (true) {
        const uint32_t n = hi - lo;
        if (n == 0u) return lo - begin;
        const uint32_t stride = (n + (uint32_t)kBookBlock - 1u) / (uint32_t)kBookBlock;
        const uint32_t p = lo + (threadIdx.x + 1u) * stride - 1u;         // my probe: the last entry of my piece
        const bool ok = p < hi && (arr[p] >> shift) <= t;                 // (the probes that pass are the first ones)
        const uint32_t c = (uint32_t)__syncthreads_count(ok ? 1 : 0);
        const uint32_t new_lo = lo + c * stride;
        if (stride == 1u) return new_lo - begin;
        const uint32_t next_probe = new_lo + stride - 1u;                 // the first probe that failed, or beyond the range
        hi = next_probe < hi ? next_probe : hi;
        lo = new_lo;
    }
}

// One round, control part: how many leaves (nl) and internal nodes (nn) are merged now.  Uniform
// over the callers; WAVE: the counts are taken by a whole wavefront probing 64 entries per step;
// BLOCK: by the whole workgroup (every thread of it calls).
template <bool WAVE, bool BLOCK = false>
__device__ inline void round_control(const uint64_t *keys, const uint64_t *iw, uint32_t m, uint32_t li, uint32_t ii, uint32_t ni,
                                     uint32_t *nl_out, uint32_t *nn_out) {
    const uint64_t inf = ~0ull;
    const uint64_t a0 = li < m ? keys[li] >> 16 : inf, a1 = li + 1 < m ? keys[li + 1] >> 16 : inf;
    const uint64_t b0 = ii < ni ? iw[ii] : inf, b1 = ii + 1 < ni ? iw[ii + 1] : inf;
    uint64_t s0, s1;
    if (a0 <= b0) { s0 = a0; s1 = (a1 <= b0) ? a1 : b0; }
    else { s0 = b0; s1 = (a0 <= b1) ? a0 : b1; }
    const uint64_t t = s0 + s1;
    uint32_t nl = BLOCK ? count_below_block(keys, li, m, t, 16) : (WAVE ? count_below_wave(keys, li, m, t, 16) : count_below(keys, li, m, t, 16, false));
    uint32_t nn = BLOCK ? count_below_block(iw, ii, ni, t, 0) : (WAVE ? count_below_wave(iw, ii, ni, t, 0) : count_below(iw, ii, ni, t, 0, false));
    if ((nl + nn) & 1u) {
        const uint64_t la = nl ? keys[li + nl - 1] >> 16 : 0, lb = nn ? iw[ii + nn - 1] : 0;
        if (nn && (!nl || la <= lb)) --nn; else --nl;
    }
    *nl_out = nl; *nn_out = nn;
}

// One round, the items: lane `lane` of `nlanes` takes every nlanes-th of the nl + nn items.
// ITEMS: items a lane works on side by side (arrays in global memory: every item is a chain of dependent loads).
template <uint32_t ITEMS = 1>
__device__ inline void round_items(const uint64_t *keys, uint64_t *iw, uint32_t *leaf_parent, uint32_t *int_parent,
                                   uint32_t li, uint32_t ii, uint32_t ni, uint32_t nl, uint32_t nn, uint32_t lane, uint32_t nlanes) {
    if (ITEMS > 1) {
        for (uint32_t idx0 = lane; idx0 < nl + nn; idx0 += ITEMS * nlanes) {
            uint64_t w[ITEMS];
            bool on[ITEMS], leaf[ITEMS];
            // the item's weight, then its rank among the items of the other kind (both loops: ITEMS loads in flight)
#pragma unroll
            for (uint32_t k = 0; k < ITEMS; ++k) {
                const uint32_t idx = idx0 + k * nlanes;
                on[k] = idx < nl + nn;
                leaf[k] = idx < nl;
                w[k] = !on[k] ? 0ull : (leaf[k] ? keys[li + idx] >> 16 : iw[ii + (idx - nl)]);
            }
            uint32_t rank[ITEMS];
#pragma unroll
            for (uint32_t k = 0; k < ITEMS; ++k) {
                const uint32_t idx = idx0 + k * nlanes;
                rank[k] = 0;
                if (on[k]) rank[k] = leaf[k] ? idx + count_below(iw, ii, ii + nn, w[k], 0, true)
                                             : (idx - nl) + count_below(keys, li, li + nl, w[k], 16, false);
            }
#pragma unroll
            for (uint32_t k = 0; k < ITEMS; ++k) {
                const uint32_t idx = idx0 + k * nlanes;
                if (on[k]) {
                    if (leaf[k]) leaf_parent[li + idx] = ni + (rank[k] >> 1);
                    else int_parent[ii + (idx - nl)] = ni + (rank[k] >> 1);
                    atomicAdd(reinterpret_cast<unsigned long long *>(&iw[ni + (rank[k] >> 1)]), (unsigned long long)w[k]);
                }
            }
        }
        return;
    }
    for (uint32_t idx = lane; idx < nl + nn; idx += nlanes) {
        uint64_t w;
        uint32_t rank;
        if (idx < nl) {
            w = keys[li + idx] >> 16;
            rank = idx + count_below(iw, ii, ii + nn, w, 0, true);
            leaf_parent[li + idx] = ni + (rank >> 1);
        } else {
            const uint32_t b = idx - nl;
            w = iw[ii + b];
            rank = b + count_below(keys, li, li + nl, w, 16, false);
            int_parent[ii + b] = ni + (rank >> 1);
        }
        atomicAdd(reinterpret_cast<unsigned long long *>(&iw[ni + (rank >> 1)]), (unsigned long long)w);
    }
}

// Rounds while more than `stop` items wait; the state is handed back.
template <bool WAVE, typename Sync>
__device__ inline void huffman_rounds(const uint64_t *keys, uint64_t *iw, uint32_t *leaf_parent, uint32_t *int_parent,
                                      uint32_t m, uint32_t lane, uint32_t nlanes, Sync sync, uint32_t stop,
                                      uint32_t &li, uint32_t &ii, uint32_t &ni) {
    li = 0; ii = 0; ni = 0;
    while ((m - li) + (ni - ii) > stop) {
        uint32_t nl, nn;
        round_control<WAVE, !WAVE>(keys, iw, m, li, ii, ni, &nl, &nn);     // (not WAVE: the whole workgroup is here)
        round_items<WAVE ? 1u : 4u>(keys, iw, leaf_parent, int_parent, li, ii, ni, nl, nn, lane, nlanes);
        sync();
        li += nl; ii += nn; ni += (nl + nn) >> 1;
    }
}

__device__ inline uint64_t lane_value64(uint64_t v, uint32_t src) { return lane_value64_any(v, src); }

// The same rounds for arrays in LDS, by the whole workgroup.  The first wavefront runs the rounds of
// at most 64 items alone and in registers: lane l holds the l-th waiting leaf and the l-th waiting
// node, the counts of a round are two ballots (the queues are sorted, so the items merged now are
// a prefix of each), and the merged order of the items comes from a short counting loop or from
// one bitonic merge across the lanes instead of a binary search in LDS per item.  A round with more items is shared by all
// wavefronts through the general routines (every wavefront works out the round's counts for
// itself).  state: three words of LDS.  n_wait: nodes that wait already, iw[0, n_wait) (a
// construction that was begun elsewhere); iw beyond them must be zero on entry.
__device__ inline void huffman_rounds_lds(const uint64_t *keys, uint64_t *iw, uint32_t *leaf_parent, uint32_t *int_parent,
                                          uint32_t m, uint32_t tid, uint32_t nthreads, uint32_t *state, uint32_t n_wait = 0) {
    uint32_t li = 0, ii = 0, ni = n_wait;
    const uint32_t lane = tid & (uint32_t)(kWave - 1);
    const uint64_t inf = ~0ull;
    while (true) {
        if (tid < (uint32_t)kWave) {
            while ((m - li) + (ni - ii) > 1u) {
                const uint64_t A = li + lane < m ? keys[li + lane] >> 16 : inf;      // waiting leaves
                const uint64_t B = ii + lane < ni ? iw[ii + lane] : inf;             // waiting nodes
                const uint64_t a0 = lane_value64(A, 0), a1 = lane_value64(A, 1), b0 = lane_value64(B, 0), b1 = lane_value64(B, 1);
                uint64_t s0, s1;
                if (a0 <= b0) { s0 = a0; s1 = (a1 <= b0) ? a1 : b0; }
                else { s0 = b0; s1 = (a0 <= b1) ? a0 : b1; }
                const uint64_t t = s0 + s1;
                uint32_t nl = (uint32_t)__popcll(wave_ballot(A != inf && A <= t));
                uint32_t nn = (uint32_t)__popcll(wave_ballot(B != inf && B <= t));
                if (nl == (uint32_t)kWave || nn == (uint32_t)kWave) break;   // there may be more beyond the window: everybody's round
                if ((nl + nn) & 1u) {
                    const uint64_t la = nl ? lane_value64(A, nl - 1u) : 0, lb = nn ? lane_value64(B, nn - 1u) : 0;
                    if (nn && (!nl || la <= lb)) --nn; else --nl;
                }
                if (nl + nn > (uint32_t)kWave) break;        // more items than lanes: everybody's round
                if ((nl < nn ? nl : nn) <= 8u) {
                    // A short queue: an item's rank in the other queue is counted in a loop over the shorter
                    // one (one broadcast and one comparison per step): my leaf counts the merged nodes lighter
                    // than it, my node the merged leaves not heavier than it.
                    uint32_t before_leaf = 0, before_node = 0;
                    if (nn <= nl) {
                        for (uint32_t k = 0; k < nn; ++k) {
                            const uint64_t bk = lane_value64(B, k);
                            before_leaf += (bk < A) ? 1u : 0u;
                            const uint32_t c = (uint32_t)__popcll(wave_ballot(lane < nl && A <= bk));
                            before_node = (lane == k) ? c : before_node;
                        }
                    } else {
                        for (uint32_t k = 0; k < nl; ++k) {
                            const uint64_t ak = lane_value64(A, k);
                            before_node += (ak <= B) ? 1u : 0u;
                            const uint32_t c = (uint32_t)__popcll(wave_ballot(lane < nn && B < ak));
                            before_leaf = (lane == k) ? c : before_leaf;
                        }
                    }
                    if (lane < nl) {
                        const uint32_t parent = ni + ((lane + before_leaf) >> 1);
                        leaf_parent[li + lane] = parent;
                        atomicAdd(reinterpret_cast<unsigned long long *>(&iw[parent]), (unsigned long long)A);
                    }
                    if (lane < nn) {
                        const uint32_t parent = ni + ((lane + before_node) >> 1);
                        int_parent[ii + lane] = parent;
                        atomicAdd(reinterpret_cast<unsigned long long *>(&iw[parent]), (unsigned long long)B);
                    }
                } else {
                    // Merged order of the round's items: the leaves ascending from lane 0, the nodes descending
                    // from lane 63 and infinity between them are a bitonic sequence, which six compare-exchange
                    // steps sort.  Key = (weight, node after leaf, position in its queue): the order of the
                    // sequential construction, and no two keys are equal (weights stay below 2^57: at most
                    // 65536 counts of 32 bits).
                    const uint64_t Brev = __shfl(B, (int)(kWave - 1u - lane), kWave);
                    uint64_t key = inf;
                    if (lane < nl) key = (A << 7) | lane;
                    else if ((uint32_t)kWave - 1u - lane < nn) key = (Brev << 7) | 64u | ((uint32_t)kWave - 1u - lane);
#pragma unroll
                    for (uint32_t j = kWave / 2; j > 0; j >>= 1) {
                        const uint64_t other = __shfl_xor(key, (int)j, kWave);
                        const uint64_t lo = key < other ? key : other, hi = key < other ? other : key;
                        key = (lane & j) ? hi : lo;
                    }
                    // lane r now holds the item of rank r: items 2j and 2j+1 become node ni + j
                    const uint64_t w = key >> 7;
                    const uint64_t w_next = __shfl_xor(w, 1, kWave);
                    if (lane < nl + nn) {
                        const uint32_t parent = ni + (lane >> 1);
                        const uint32_t pos = (uint32_t)key & 63u;
                        if (key & 64u) int_parent[ii + pos] = parent;
                        else leaf_parent[li + pos] = parent;
                        if ((lane & 1u) == 0u) iw[parent] = w + w_next;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
                __builtin_amdgcn_wave_barrier();
                li += nl; ii += nn; ni += (nl + nn) >> 1;
            }
            if (lane == 0) { state[0] = li; state[1] = ii; state[2] = ni; }
        }
        __syncthreads();
        li = state[0]; ii = state[1]; ni = state[2];
        if ((m - li) + (ni - ii) <= 1u) break;
        uint32_t nl, nn;
        round_control<true>(keys, iw, m, li, ii, ni, &nl, &nn);
        round_items(keys, iw, leaf_parent, int_parent, li, ii, ni, nl, nn, tid, nthreads);
        __syncthreads();
        li += nl; ii += nn; ni += (nl + nn) >> 1;
    }
}

// Everything between the histogram and the tables, on storage that is either LDS
// (LDS == true: the pointers are the workgroup's own __shared__ arrays, so the
// compiler emits ds_* instructions) or global scratch for large alphabets.
// l_keys .. l_ip: the workgroup's LDS arrays of kBookLdsSyms entries (the same pointers as keys .. int_parent when LDS).
template <bool LDS>
__device__ inline void codebook_body(const BookArgs &a, uint32_t m, uint64_t *keys, uint64_t *iw, uint32_t *leaf_parent,
                                     uint32_t *int_parent, uint64_t *l_keys, uint64_t *l_iw, uint32_t *l_lp, uint32_t *l_ip,
                                     uint64_t *s_x, uint32_t *s_part, uint32_t *s_cnt,
                                     uint64_t *s_first, uint32_t *s_findex, uint32_t *s_maxlen, uint32_t *s_wc) {
    const uint32_t tid = threadIdx.x;
    const uint32_t nbins = a.nbins;
    // ---- 1. compact the active symbols into sort keys (frequency << 16 | symbol) ----
    // (code book reuse: the given length takes the place of the frequency, so the keys are already
    // those of step 5 and steps 2-4 are skipped)
    const bool given = a.given_len != nullptr;
    // presorted: the sort kernels have left the leaves in order in keys[0, m) (large alphabets built from a histogram)
    const bool presorted = !LDS && !given && a.presorted != 0u;
    if (presorted) {
        for (uint32_t s = tid; s < nbins; s += kBookBlock)
            if (a.hist[s] == 0u) {
                a.len_out[s] = 0;
                a.enc[s] = 0;
                if (a.code_out) a.code_out[s] = 0;
            }
    } else {
        uint32_t done = 0;
        for (uint32_t base = 0; base < nbins; base += kBookBlock) {
            const uint32_t s = base + tid;
            const uint32_t f = (s < nbins) ? (given ? (uint32_t)a.given_len[s] : a.hist[s]) : 0u;
            uint32_t tot;
            const uint32_t pos = block_excl_scan<uint32_t, kBookBlock / kWave>(f ? 1u : 0u, s_part, tot);
            if (f) keys[done + pos] = ((uint64_t)f << 16) | s;
            else if (s < nbins) {           // unused symbol: length 0 everywhere
                a.len_out[s] = 0;
                a.enc[s] = 0;
                if (a.code_out) a.code_out[s] = 0;
            }
            done += tot;
        }
    }
    const uint32_t m2 = next_pow2(m > 1 ? m : 2);
    if (!presorted) for (uint32_t i = m + tid; i < m2; i += kBookBlock) keys[i] = ~0ull;
    for (uint32_t i = tid; i < m; i += kBookBlock) iw[i] = 0;
    __syncthreads();

    const bool reg_sort = LDS && m2 <= (uint32_t)kBookBlock;
    // Canonical order without a second sort: the lengths are scattered into a by-symbol table (in the
    // sort's exchange buffer, free after step 2) and the symbols are then visited in increasing order.
    // The by-symbol table of an alphabet built in global memory is the length table itself (a sort of
    // that many keys by one workgroup would cost more than visiting every symbol).
    const bool by_symbol = !LDS || nbins <= (uint32_t)kBookBySymbolMax;
    uint8_t *s_depth = LDS ? reinterpret_cast<uint8_t *>(s_x) : a.len_out;
    if (given) {
        // lengths per symbol are known: count them; a length the container cannot hold spoils the count
        // of length 64, which the completeness test below then rejects
        if (by_symbol && LDS) {
            for (uint32_t i = tid; i < nbins; i += kBookBlock) s_depth[i] = 0;
            __syncthreads();
        }
        for (uint32_t i = tid; i < m; i += kBookBlock) {
            const uint32_t depth = (uint32_t)(keys[i] >> 16);
            atomicAdd(&s_cnt[depth > 57 ? 64 : depth], 1u);
            atomicMax(s_maxlen, depth);
            if (by_symbol) s_depth[(uint32_t)(keys[i] & 0xffffu)] = (uint8_t)(depth > 57 ? 64 : depth);
        }
        __syncthreads();
    } else {
    // ---- 2. leaves in (frequency, symbol) order ----
    if (reg_sort) {
        uint64_t key = tid < m2 ? keys[tid] : ~0ull;
        key = bitonic_sort_regs(key, s_x, m2);
        if (tid < m2) keys[tid] = key;
        __syncthreads();
    } else if (!presorted) {
        bitonic_sort(keys, m2);
    }

    // ---- 3. two-queue merge in rounds ----
    if (m >= 2) {
        if (LDS) {
            huffman_rounds_lds(keys, iw, leaf_parent, int_parent, m, tid, (uint32_t)kBookBlock, s_part);
        } else {
            // The first rounds merge thousands of light leaves each: in global memory, by everybody.  Most
            // rounds come later, with few items each: once the L leaves and N nodes that wait make at most
            // kBookLdsSyms / 2 items, they move to LDS (L + 2N - 1 nodes at the end, which fit), the rounds
            // are finished there, and the parents go back with the offset of the first node moved.
            uint32_t li, ii, ni;
            huffman_rounds<false>(keys, iw, leaf_parent, int_parent, m, tid, (uint32_t)kBookBlock, [] { __syncthreads(); },
                                  kBookLdsSyms / 2u, li, ii, ni);
            const uint32_t L = m - li, N = ni - ii;
            if (L + N > 1u) {
                for (uint32_t j = tid; j < L; j += kBookBlock) l_keys[j] = keys[li + j];
                for (uint32_t k = tid; k < kBookLdsSyms; k += kBookBlock) l_iw[k] = k < N ? iw[ii + k] : 0ull;
                __syncthreads();
                huffman_rounds_lds(l_keys, l_iw, l_lp, l_ip, L, tid, (uint32_t)kBookBlock, s_part, N);
                __syncthreads();
                for (uint32_t j = tid; j < L; j += kBookBlock) leaf_parent[li + j] = ii + l_lp[j];
                for (uint32_t k = tid; k + 1u < L + 2u * N - 1u; k += kBookBlock) int_parent[ii + k] = ii + l_ip[k];   // (the last node is the root)
            }
        }
    }
    __syncthreads();

    if (by_symbol && LDS) {
        for (uint32_t i = tid; i < nbins; i += kBookBlock) s_depth[i] = 0;
        __syncthreads();
    }
    // ---- 4. depth of every leaf: walk to the root (node m-2) ----
    // (four leaves per thread at a time: a walk is a chain of dependent loads, in global memory for a large
    // alphabet, and four chains wait side by side)
    constexpr uint32_t kWalks = 4;
    for (uint32_t i0 = tid; i0 < m; i0 += kWalks * kBookBlock) {
        uint32_t p[kWalks], depth[kWalks];
        const uint32_t root = m >= 2 ? m - 2 : 0u;
#pragma unroll
        for (uint32_t k = 0; k < kWalks; ++k) {
            const uint32_t i = i0 + k * kBookBlock;
            depth[k] = 1;
            p[k] = (m >= 2 && i < m) ? leaf_parent[i] : root;
        }
        bool more = true;
        while (more) {
            more = false;
#pragma unroll
            for (uint32_t k = 0; k < kWalks; ++k) {
                const bool go = p[k] != root && depth[k] < 66u;
                const uint32_t q = go ? int_parent[p[k]] : root;
                p[k] = go ? q : p[k];
                depth[k] += go ? 1u : 0u;
                more = more || go;
            }
        }
#pragma unroll
        for (uint32_t k = 0; k < kWalks; ++k) {
            const uint32_t i = i0 + k * kBookBlock;
            if (i < m) {
                const uint32_t sym = (uint32_t)(keys[i] & 0xffffu);
                keys[i] = ((uint64_t)depth[k] << 16) | sym;     // re-keyed for the canonical order
                atomicAdd(&s_cnt[depth[k] > 64 ? 64 : depth[k]], 1u);
                atomicMax(s_maxlen, depth[k]);
                if (by_symbol) s_depth[sym] = (uint8_t)(depth[k] > 64 ? 64 : depth[k]);
            }
        }
    }
    __syncthreads();
    }   // !given

    // ---- 5. canonical order (length, symbol) ----
    if (!by_symbol) {
        if (reg_sort) {
            uint64_t key = tid < m2 ? keys[tid] : ~0ull;
            key = bitonic_sort_regs(key, s_x, m2);
            if (tid < m2) keys[tid] = key;
            __syncthreads();
        } else {
            bitonic_sort(keys, m2);
        }
    }
    bool ok = true;
    if (tid < (uint32_t)kWave) {
        uint32_t mx, mn;
        ok = (m == 0 && !given) || (m != 0 && canonical_first_codes_wave(s_cnt, m, s_first, s_findex, &mx, &mn));
        if (!ok && tid == 0) atomicOr(&a.ctl->status, given ? (uint32_t)ST_CODEBOOK : (uint32_t)ST_INTERNAL);   // a given table must be a complete code
    }
    ok = __syncthreads_and(ok ? 1 : 0) != 0;

    // ---- 6. codes and tables ----
    if (!by_symbol) {
        for (uint32_t p = tid; p < m; p += kBookBlock) {
            const uint32_t L = (uint32_t)(keys[p] >> 16);
            const uint32_t sym = (uint32_t)(keys[p] & 0xffffu);
            const uint64_t code = s_first[L > 64 ? 64 : L] + (p - s_findex[L > 64 ? 64 : L]);
            a.len_out[sym] = (uint8_t)L;
            a.enc[sym] = (code << 6) | (uint64_t)(L & 63u);
            if (a.code_out) a.code_out[sym] = code;
        }
        return;
    }
    // The symbols in increasing order: the code of a symbol is the first code of its length plus the
    // number of smaller symbols of the same length (per wavefront the lanes of one length are found
    // with a ballot per length that occurs, then a prefix over the wavefronts in front).
    const uint32_t lane = tid & (uint32_t)(kWave - 1), wave = tid / (uint32_t)kWave;
    constexpr uint32_t kWaves = kBookBlock / kWave;
    uint32_t *s_run = s_wc + kWaves * 64u;                   // symbols per length in front of the current 1024 symbols
    for (uint32_t i = tid; i < 65u; i += kBookBlock) s_run[i] = 0;
    for (uint32_t base = 0; base < nbins; base += kBookBlock) {
        for (uint32_t i = tid; i < kWaves * 64u; i += kBookBlock) s_wc[i] = 0;
        __syncthreads();
        const uint32_t sym = base + tid;
        const uint32_t L = (sym < nbins) ? s_depth[sym] : 0u;
        uint32_t in_wave = 0;
        uint64_t todo = wave_ballot(L != 0u);
        while (todo) {                                       // one step per length that occurs in the wavefront
            const uint32_t Lc = (uint32_t)__builtin_amdgcn_readlane((int)L, __builtin_ctzll(todo));
            const uint64_t same = wave_ballot(L == Lc);
            if (L == Lc) in_wave = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
            if (lane == 0) s_wc[wave * 64u + (Lc & 63u)] = (uint32_t)__popcll(same);
            todo &= ~same;
        }
        __syncthreads();
        if (L) {
            uint32_t before = s_run[L & 63u];
            for (uint32_t w = 0; w < wave; ++w) before += s_wc[w * 64u + (L & 63u)];
            const uint64_t code = s_first[L] + before + in_wave;
            a.len_out[sym] = (uint8_t)L;
            a.enc[sym] = (code << 6) | (uint64_t)(L & 63u);
            if (a.code_out) a.code_out[sym] = code;
        }
        __syncthreads();
        if (tid < 64u) {
            uint32_t add = 0;
            for (uint32_t w = 0; w < kWaves; ++w) add += s_wc[w * 64u + tid];
            s_run[tid] += add;
        }
        __syncthreads();                                     // the counts are cleared for the next 1024 symbols
    }
}

// ---------------------------------------------------------------------------
// Leaves of a large alphabet in (frequency, symbol) order.  One key per symbol: (frequency, symbol), or
// a key above all of those for a symbol that does not occur (each its own, so that no two keys are
// equal).  k_book_sort_tiles: one tile of kBookBlock symbols per workgroup, sorted in registers; the
// grid's tiles are a power of two and cover the alphabet.  It also counts the symbols that occur.
// k_book_merge: runs of `run` keys merged pairwise; a key's place is its rank in its own run plus the
// number of smaller keys in the other one (binary search); one key per thread.  Alphabets whose
// occurring symbols fit LDS are built there from the histogram: the merges then have nothing to do.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBookBlock) void k_book_sort_tiles(const uint32_t *hist, uint32_t nbins, uint64_t *keys, Control *ctl) {
    __shared__ uint64_t s_x[kBookBlock];
    const uint32_t s = blockIdx.x * (uint32_t)kBookBlock + threadIdx.x;
    const uint32_t f = s < nbins ? hist[s] : 0u;
    const uint32_t cnt = (uint32_t)__syncthreads_count(f != 0u);
    if (threadIdx.x == 0 && cnt) atomicAdd(&ctl->n_active, cnt);
    uint64_t key = f ? (((uint64_t)f << 16) | s) : ((1ull << 63) | s);
    key = bitonic_sort_regs(key, s_x, (uint32_t)kBookBlock);
    keys[s] = key;
}

__global__ __launch_bounds__(kBookMergeBlock) void k_book_merge(const uint64_t *src, uint64_t *dst, uint32_t run, const Control *ctl) {
    if (ctl->n_active <= kBookLdsSyms) return;
    const uint32_t i = blockIdx.x * (uint32_t)kBookMergeBlock + threadIdx.x;
    const uint64_t key = src[i];
    const uint32_t r = i / run, own = i - r * run;           // run: a power of two
    const uint64_t *other = src + (size_t)(r ^ 1u) * run;
    uint32_t lo = 0, hi = run;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (other[mid] < key) lo = mid + 1; else hi = mid;
    }
    dst[(size_t)(r & ~1u) * run + own + lo] = key;
}

__global__ __launch_bounds__(kBookBlock) void k_codebook(BookArgs a) {
    // One workgroup on the critical path of its stream, often next to the streaming kernels of
    // other streams: its wavefronts go first whenever they are ready to issue.
    __builtin_amdgcn_s_setprio(3);
    __shared__ uint64_t s_keys[kBookLdsSyms];
    __shared__ uint64_t s_iw[kBookLdsSyms];
    __shared__ uint32_t s_lp[kBookLdsSyms];
    __shared__ uint32_t s_ip[kBookLdsSyms];
    __shared__ uint64_t s_x[kBookBlock];
    __shared__ uint32_t s_part[kBookBlock / kWave];
    __shared__ uint32_t s_cnt[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint32_t s_findex[65];
    __shared__ uint32_t s_maxlen;
    __shared__ uint32_t s_wc[(kBookBlock / kWave) * 64 + 65];      // canonical order: symbols per (wavefront, length), and per length so far

    const uint32_t tid = threadIdx.x;
    const uint32_t nbins = a.nbins;
    if (tid < 65) s_cnt[tid] = 0;
    if (tid == 0) s_maxlen = 0;

    uint32_t m = 0;
    // (and: does every symbol that occurs, but for the escape symbol, lie in the part of the encode table that the
    // encoders keep in LDS?)
    const uint32_t win_n = nbins < kEncTableMax ? nbins : kEncTableMax, win_lo = (nbins - win_n) / 2u;
    const uint32_t lenw_n = enc_len_window(nbins), lenw_lo = (nbins - lenw_n) / 2u;
    int outside = 0;
    for (uint32_t base = 0; base < nbins; base += kBookBlock) {
        const uint32_t s = base + tid;
        const bool occurs = (s < nbins) && (a.given_len ? a.given_len[s] != 0 : a.hist[s] != 0u);
        m += __syncthreads_count(occurs);
        outside |= (occurs && s != 0u && s - win_lo >= win_n) ? 1 : 0;
        outside |= (occurs && s != 0u && s - lenw_lo >= lenw_n) ? 2 : 0;
    }
    outside = (__syncthreads_or(outside & 1) ? 1 : 0) | (__syncthreads_or(outside & 2) ? 2 : 0);
    if (m <= kBookLdsSyms)
        codebook_body<true>(a, m, s_keys, s_iw, s_lp, s_ip, s_keys, s_iw, s_lp, s_ip, s_x, s_part, s_cnt, s_first, s_findex, &s_maxlen, s_wc);
    else
        codebook_body<false>(a, m, a.scratch.keys, a.scratch.iw, a.scratch.leaf_parent, a.scratch.int_parent, s_keys, s_iw, s_lp, s_ip,
                             s_x, s_part, s_cnt, s_first, s_findex, &s_maxlen, s_wc);

    // ---- 7. container layout ----
    if (tid == 0) {
        a.ctl->n_active = m;
        a.ctl->max_len = s_maxlen;
        a.ctl->enc_in_window = (outside & 1) ? 0u : 1u;
        a.ctl->len_in_window = (outside & 2) ? 0u : 1u;
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
    __builtin_amdgcn_s_setprio(3);                  // as k_codebook: a single workgroup others wait for
    __shared__ uint32_t s_cnt[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint64_t s_limit[65];
    __shared__ uint32_t s_findex[65];
    __shared__ uint32_t s_ok, s_maxlen, s_nbins, s_chunk;
    __shared__ uint16_t s_sorted[kBookBlock * 2];                   // symbols in canonical order (alphabets up to this size)
    __shared__ uint32_t s_wc[(kBookBlock / kWave) * 64];            // symbols per (wavefront, length) of the current 1024 symbols
    __shared__ uint32_t s_run[65];                                  // symbols per length in front of them
    __shared__ uint32_t s_scan[kBookBlock / kWave];
    __shared__ uint16_t s_ent[kLut16Size];                          // first level of the compact table
    __shared__ uint16_t s_owner[kSubEntries];                       // second level: the prefix every entry belongs to

    const uint32_t tid = threadIdx.x;
    if (a.reset_ctl && tid < sizeof(Control) / 4u) reinterpret_cast<uint32_t *>(a.ctl)[tid] = 0u;   // before the first barrier: nothing has raised a bit yet
    auto raise_format = [&]() {                     // thread 0 only
        atomicOr(&a.ctl->status, (uint32_t)ST_FORMAT);
        if (a.latched) atomicOr(a.latched, (uint32_t)ST_FORMAT);
        if (a.status_out) *a.status_out = -3;
    };
    if (tid == 0) {
        if (a.status_out) *a.status_out = 0;
        uint32_t ok = 1;
        s_nbins = a.nbins;
        s_chunk = 64u;
        if (a.hdr) {
            const Header h = *a.hdr;
            const Header &e = a.expect;
            const uint64_t n = (uint64_t)e.N * e.C * e.H * e.W;
            if (a.bytes < kHeaderBytes) ok = 0;
            if (h.magic != kMagic || (h.version != 1u && h.version != 2u) || h.status != 0u) ok = 0;
            if (h.N != e.N || h.C != e.C || h.H != e.H || h.W != e.W) ok = 0;
            if (h.nbins < 4u || h.nbins > 65536u || (h.nbins & 1u)) ok = 0;
            s_nbins = h.nbins;
            if (h.chunk_syms == 0) ok = 0;
            s_chunk = h.chunk_syms;
            const float eb = __uint_as_float(h.eb_bits);
            if (!(eb >= 0x1p-100f && eb <= 0x1p100f)) ok = 0;
            if (__float_as_uint(2.0f * eb) != h.ebx2_bits) ok = 0;
            if (__float_as_uint((float)(1.0 / (double)(2.0f * eb))) != h.r_bits) ok = 0;
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
        if (tid == 0) raise_format();
        return;
    }
    const uint32_t nbins = s_nbins;

    // ---- symbols per length ----
    uint32_t m = 0;
    bool bad = false;
    for (uint32_t base = 0; base < nbins; base += kBookBlock) {
        const uint32_t s = base + tid;
        const uint32_t L = (s < nbins) ? a.len[s] : 0u;
        if (L > 57u) bad = true;
        if (L) atomicAdd(&s_cnt[L > 64u ? 64u : L], 1u);
        m += __syncthreads_count(L != 0u);
    }
    if (__syncthreads_or(bad ? 1 : 0) || m == 0) {
        if (tid == 0) raise_format();
        return;
    }
    if (tid < (uint32_t)kWave) {
        uint32_t mx, mn;
        const bool ok = canonical_first_codes_wave(s_cnt, m, s_first, s_findex, &mx, &mn);
        if (tid == 0) { s_maxlen = mx; s_ok = ok ? 1u : 0u; }
        if (ok) {
            wave_lds_fence();                                // the first codes of the other lengths
            const uint32_t L = tid ? tid : 64u;              // one length per lane
            // exclusive upper bound, left-aligned; the longest length closes the code space
            uint64_t lim = 0;
            if (L < mx) lim = (s_first[L] + s_cnt[L]) << (64u - L);
            else lim = ~0ull;
            s_limit[L] = lim;
            a.t.limit[L] = lim;
            a.t.first_code[L] = s_first[L];
            a.t.first_index[L] = s_findex[L];
            if (tid == 0) {
                a.t.limit[0] = 0; a.t.first_code[0] = 0; a.t.first_index[0] = 0;
                a.t.meta[0] = mx; a.t.meta[1] = m; a.t.meta[2] = mn;
            }
        }
    }
    __syncthreads();
    if (!s_ok) {
        if (tid == 0) raise_format();
        return;
    }
    // ---- canonical order: by length, then by symbol.  The symbols are visited in increasing order,
    // so the place of a symbol is the first index of its length plus the number of smaller symbols of
    // the same length: a counting sort (per wavefront the lanes of one length are found with a ballot
    // per length that occurs, then a prefix over the wavefronts in front). ----
    const bool small = m <= (uint32_t)kBookBlock * 2u;
    uint16_t *sorted = small ? s_sorted : a.t.sorted;
    {
        const uint32_t lane = tid & (uint32_t)(kWave - 1), wave = tid / (uint32_t)kWave;
        constexpr uint32_t kWaves = kBookBlock / kWave;
        for (uint32_t i = tid; i < 65u; i += kBookBlock) s_run[i] = 0;
        for (uint32_t base = 0; base < nbins; base += kBookBlock) {
            for (uint32_t i = tid; i < kWaves * 64u; i += kBookBlock) s_wc[i] = 0;
            __syncthreads();
            const uint32_t s = base + tid;
            const uint32_t L = (s < nbins) ? a.len[s] : 0u;  // 1 .. 57 here
            uint32_t in_wave = 0;
            uint64_t todo = wave_ballot(L != 0u);
            while (todo) {                                   // one step per length that occurs in the wavefront
                const uint32_t Lc = (uint32_t)__builtin_amdgcn_readlane((int)L, __builtin_ctzll(todo));
                const uint64_t same = wave_ballot(L == Lc);
                if (L == Lc) in_wave = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
                if (lane == 0) s_wc[wave * 64u + Lc] = (uint32_t)__popcll(same);
                todo &= ~same;
            }
            __syncthreads();
            if (L) {
                uint32_t before = s_run[L];
                for (uint32_t w = 0; w < wave; ++w) before += s_wc[w * 64u + L];
                sorted[s_findex[L] + before + in_wave] = (uint16_t)s;
            }
            __syncthreads();
            if (tid < 64u && tid) {                          // symbols of each length so far
                uint32_t add = 0;
                for (uint32_t w = 0; w < kWaves; ++w) add += s_wc[w * 64u + tid];
                s_run[tid] += add;
            }
            __syncthreads();                                 // the counts are cleared for the next 1024 symbols
        }
    }
    if (small) {
        for (uint32_t p = tid; p < m; p += kBookBlock) a.t.sorted[p] = sorted[p];
    }

    // look-up table on the next kLutBits bits; entries carry the residual, not the symbol
    const uint32_t mx = s_maxlen;
    // Length of the code a left-aligned bit pattern v starts with, searched in [lo, hi]: the smallest L with
    // v below the upper bound of the codes of length L (the bounds do not decrease with L, and the longest
    // length closes the code space); 0 if the code is longer than hi.  A handful of LDS reads.
    auto code_length = [&](uint64_t v, uint32_t lo, uint32_t hi) -> uint32_t {
        if (hi > mx) hi = mx;
        if (lo > hi) return 0u;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (mid >= mx || v < s_limit[mid]) hi = mid; else lo = mid + 1u;
        }
        return (lo >= mx || v < s_limit[lo]) && s_cnt[lo] ? lo : 0u;
    };
    const int32_t radius = (int32_t)(nbins / 2u);
    const bool compact = nbins <= kLut16MaxBins;
    const bool skip_general = compact && a.compact_only && !(a.general_unless_chunk64 && s_chunk != 64u);
    for (uint32_t e = tid; e < (skip_general ? 0u : kLutSize); e += kBookBlock) {
        const uint64_t v = (uint64_t)e << (64 - kLutBits);
        uint32_t entry = 0;
        {
            const uint32_t L = code_length(v, 1u, (uint32_t)kLutBits);
            if (L) {
                uint64_t off = (v >> (64u - L)) - s_first[L];
                if (off >= s_cnt[L]) off = s_cnt[L] - 1u;      // only reachable with an invalid stream
                const uint32_t sym = sorted[s_findex[L] + off];
                const int32_t d = sym ? (int32_t)sym - radius : -32768;
                entry = ((uint32_t)d << 8) | L;
            }
        }
        if (entry == 0) {
            // no code of at most kLutBits bits starts here: length byte 0, and in the residual field the
            // shortest length a code with this prefix can have (where the decoder's search starts)
            uint32_t L = code_length(v, (uint32_t)kLutBits + 1u, mx);
            if (L == 0u) L = mx;
            entry = L << 8;
        }
        a.t.lut[e] = entry;
        if (!compact) reinterpret_cast<uint32_t *>(a.t.lut16)[e] = entry;    // the chunk decoders load their table from one place
    }
    // The compact table on the next kLut16Bits bits, for alphabets whose residuals fit 12 signed bits, and
    // its second level.  A prefix of kLut16Bits bits under which longer codes lie gets a sub-table indexed by
    // the next 1, 2, 4 or 6 bits (enough for the longest code under the prefix, 6 at most): its entries are
    // (residual << 4) | (length - kLut16Bits), or 0 for a code that is longer still.  The first-level entry of
    // such a prefix is ((offset / 2) << 2 | width code) << 4 with a zero length; offset 0 is never given out,
    // so an all-zero entry means "no sub-table" (the sub-tables filled their array: search by length).
    if (compact) {
        constexpr uint32_t kPer = kLut16Size / kBookBlock;          // consecutive first-level entries per thread
        uint32_t ent[kPer], kbits[kPer], need = 0;
        for (uint32_t j = 0; j < kPer; ++j) {
            const uint32_t e = tid * kPer + j;
            const uint64_t v = (uint64_t)e << (64 - kLut16Bits);
            uint32_t entry = 0;
            {
                const uint32_t L = code_length(v, 1u, (uint32_t)kLut16Bits);
                if (L) {
                    uint64_t off = (v >> (64u - L)) - s_first[L];
                    if (off >= s_cnt[L]) off = s_cnt[L] - 1u;      // only reachable with an invalid stream
                    const uint32_t sym = sorted[s_findex[L] + off];
                    const int32_t d = sym ? (int32_t)sym - radius : kLut16Escape;
                    entry = (((uint32_t)d & 0xfffu) << 4) | L;
                }
            }
            ent[j] = entry;
            kbits[j] = 0;
            if (entry == 0) {
                // the longest code under this prefix is the one its last bit pattern belongs to
                const uint64_t v_hi = v | ((1ull << (64 - kLut16Bits)) - 1ull);
                uint32_t L = code_length(v_hi, (uint32_t)kLut16Bits + 1u, mx);
                if (L == 0u) L = mx;
                const uint32_t k = L - (uint32_t)kLut16Bits;
                kbits[j] = k <= 1u ? 1u : (k <= 2u ? 2u : (k <= 4u ? 4u : 6u));
                need += 1u << kbits[j];
            }
        }
        uint32_t total;
        uint32_t at = 2u + block_excl_scan<uint32_t, kBookBlock / kWave>(need, s_scan, total);
        // first-level entries; every sub-table entry learns which prefix it belongs to
        for (uint32_t j = 0; j < kPer; ++j) {
            const uint32_t e = tid * kPer + j;
            if (kbits[j]) {
                const uint32_t kb = kbits[j], size = 1u << kb;
                if (at + size <= kSubEntries) {
                    const uint32_t kcode = kb == 1u ? 0u : (kb == 2u ? 1u : (kb == 4u ? 2u : 3u));
                    ent[j] = (((at >> 1) << 2) | kcode) << 4;
                    for (uint32_t i = 0; i < size; ++i) s_owner[at + i] = (uint16_t)e;
                }
                at += size;
            }
            s_ent[e] = (uint16_t)ent[j];
            a.t.lut16[e] = (uint16_t)ent[j];
        }
        __syncthreads();
        // the sub-table entries, one thread each
        const uint32_t used = (2u + total < kSubEntries) ? 2u + total : kSubEntries;
        for (uint32_t x = tid; x < used; x += kBookBlock) {
            uint32_t entry = 0;
            if (x >= 2u) {
                const uint32_t e = s_owner[x] & (kLut16Size - 1u);      // (an entry past the last sub-table that fitted holds anything)
                const uint32_t pe = s_ent[e];
                const uint32_t kb = (0x6421u >> (((pe >> 4) & 3u) * 4u)) & 0xfu;
                const uint32_t first = (pe >> 6) << 1;
                if (pe != 0u && (pe & 0xfu) == 0u && x >= first && x - first < (1u << kb)) {       // (always, for an entry inside an allocated sub-table)
                    const uint64_t v = ((uint64_t)e << (64 - kLut16Bits)) | ((uint64_t)(x - first) << (64 - kLut16Bits - kb));
                    const uint32_t L = code_length(v, (uint32_t)kLut16Bits + 1u, (uint32_t)kLut16Bits + kb);
                    if (L) {
                        uint64_t off = (v >> (64u - L)) - s_first[L];
                        if (off >= s_cnt[L]) off = s_cnt[L] - 1u;  // only reachable with an invalid stream
                        const uint32_t sym = sorted[s_findex[L] + off];
                        const int32_t d = sym ? (int32_t)sym - radius : kLut16Escape;
                        entry = (((uint32_t)d & 0xfffu) << 4) | (L - (uint32_t)kLut16Bits);
                    }
                }
            }
            a.t.sub16[x] = (uint16_t)entry;
        }
    }
    if (tid == 0) { a.t.meta[3] = (uint32_t)radius; a.t.meta[4] = compact ? 1u : 0u; }
}

}  // namespace comet
