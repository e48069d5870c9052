// Shared device-side definitions of libcomet: container header, per-call control
// block, wavefront/block scans and the single-pass chained scan used to place
// variable-size output (outlier records, Huffman words) deterministically.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace comet {

constexpr uint32_t kMagic = 0x31544D43u;   // bytes 'C','M','T','1'
constexpr uint32_t kHeaderBytes = 128u;
constexpr int kWave = 64;                   // CDNA wavefront width

// device-side status bits, latched in Control::status
enum : uint32_t { ST_CAPACITY = 1u, ST_FORMAT = 2u, ST_INTERNAL = 4u, ST_CODEBOOK = 8u };

// Container header.  Field order is the on-disk order (little-endian).
struct Header {
    uint32_t magic, version, status, N, C, H, W, nbins;
    uint32_t chunk_syms, n_chunks, eb_bits, ebx2_bits, r_bits, n_active, max_len, n_rec;
    uint64_t nnz, payload_words, total_bytes, off_len, off_chunk, off_outlier, off_payload;
    uint32_t n_vrec, zero;
};
static_assert(sizeof(Header) == kHeaderBytes, "header layout");

// Per-call control block in the workspace; zeroed (with the histogram and the
// scan descriptors that follow it) by one memset before every call.
struct Control {
    uint32_t ticket_q;      // next tile of the quantise kernel
    uint32_t ticket_e;      // next tile of the encode kernel
    uint32_t done_e;        // encode workgroups that have finished
    uint32_t status;        // ST_* bits of this call
    uint64_t n_rec;         // all outlier records
    uint64_t n_vrec;        // verbatim (type 1) records
    uint64_t nnz;           // non-zero inputs
    uint64_t payload_words;
    uint64_t off_payload;   // byte offset of the payload section (known once the records are counted)
    uint64_t total_bytes;
    uint32_t n_active;
    uint32_t max_len;
    uint32_t enc_in_window;  // k_codebook: every symbol with a code word, but for the escape symbol, lies in the part of the encode table the encoders cache in LDS
    uint32_t len_in_window;  // k_codebook: ... in the (wider) part whose lengths the count kernel caches
};

// Orders the LDS accesses of the lanes of one wavefront (writes before, reads after).  Only the
// LDS counter is waited for: a fence over all address spaces would also wait for every global
// load and store in flight, which turns a streaming loop into one memory round trip per step.
__device__ inline void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup", "local");
    __builtin_amdgcn_wave_barrier();
}

// Lanes of the wavefront for which `p` holds.  (The HIP __ballot takes an int: its bool -> int -> compare
// round trip costs two extra vector instructions per call.)
__device__ inline uint64_t wave_ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

__host__ __device__ inline uint64_t align16(uint64_t v) { return (v + 15u) & ~(uint64_t)15u; }

// ---------------------------------------------------------------------------
// exact unsigned division of 32-bit values by a runtime constant:
// floor(x / d) = mulhi64(x, ceil(2^64 / d)) for every x < 2^32, d >= 2
// (error term x * (d*M - 2^64) < 2^32 * d <= 2^64).  d == 1 is the identity.
// ---------------------------------------------------------------------------
struct FastDiv {
    uint64_t magic;
    uint32_t d;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    f.magic = (d <= 1u) ? 0ull : (~0ull / d + 1ull);
    return f;
}
__device__ inline uint32_t fdiv(uint32_t x, const FastDiv &f) {
    return (f.d <= 1u) ? x : (uint32_t)__umul64hi((uint64_t)x, f.magic);
}

// ---------------------------------------------------------------------------
// wavefront / block scans
// ---------------------------------------------------------------------------
__device__ inline int lane_id() { return (int)__lane_id(); }

template <typename T>
__device__ inline T wave_incl_scan(T v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

template <typename T>
__device__ inline T wave_sum(T v) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

// Exclusive scan over the block; `total` receives the block sum.  s_part must
// hold one T per wavefront.  Contains two barriers.
template <typename T, int NWAVES>
__device__ inline T block_excl_scan(T v, T *s_part, T &total) {
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    T incl = wave_incl_scan(v);
    if (lane == kWave - 1) s_part[wave] = incl;
    __syncthreads();
    T off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {
        T t = s_part[w];
        if (w < wave) off += t;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return off + incl - v;
}

// ---------------------------------------------------------------------------
// Chained scan (single pass, decoupled look-back) over tiles taken in ticket
// order.  One 64-bit descriptor per tile: the top two bits say whether the low
// 62 bits hold nothing yet (0), the tile's own aggregate (1) or the inclusive
// prefix up to and including the tile (2).  A tile only ever waits for tiles
// with smaller tickets, and a ticket is taken before its tile is touched, so
// the tile with the smallest unfinished ticket is always running: every wait
// ends.  The whole state of a tile is one word, so relaxed agent-scope atomics
// are enough.  Must be called by all 64 lanes of one wavefront; returns the
// exclusive prefix of `tile`.  A bounded spin turns a broken invariant into an
// error flag instead of a hang.
// ---------------------------------------------------------------------------
constexpr uint64_t kDescAgg = 1ull << 62;
constexpr uint64_t kDescIncl = 2ull << 62;
constexpr uint64_t kDescMask = (1ull << 62) - 1ull;

__device__ inline uint64_t desc_load(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void desc_store(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline uint64_t chained_scan_wave(uint64_t *desc, uint32_t tile, uint64_t aggregate, uint32_t *status) {
    const int lane = lane_id();
    if (tile == 0) {
        if (lane == 0) desc_store(&desc[0], kDescIncl | aggregate);
        return 0;
    }
    if (lane == 0) desc_store(&desc[tile], kDescAgg | aggregate);
    uint64_t excl = 0;
    int64_t window_end = (int64_t)tile - 1;
    bool failed = false;
    while (true) {
        const int64_t idx = window_end - lane;
        uint64_t v = kDescIncl;            // virtual tiles before tile 0: inclusive prefix 0
        if (idx >= 0) {
            uint32_t spins = 0;
            do {
                v = desc_load(&desc[idx]);
                if ((v >> 62) != 0) break;
                __builtin_amdgcn_s_sleep(1);
            } while (++spins < (1u << 22));
            if ((v >> 62) == 0) { failed = true; v = kDescIncl; }
        }
        const uint64_t incl_mask = __ballot((v >> 62) == 2);
        if (incl_mask) {
            const int first = __ffsll((unsigned long long)incl_mask) - 1;
            excl += wave_sum<uint64_t>(lane <= first ? (v & kDescMask) : 0ull);
            break;
        }
        excl += wave_sum<uint64_t>(v & kDescMask);
        window_end -= kWave;
    }
    if (__ballot(failed) && lane == 0) atomicOr(status, (uint32_t)ST_INTERNAL);
    if (lane == 0) desc_store(&desc[tile], kDescIncl | ((excl + aggregate) & kDescMask));
    return excl;
}

}  // namespace comet
