// Host side of libcomet: context / workspace, argument checks, launch geometry
// and the extern "C" entry points declared in include/comet.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <numeric>
#include <new>
#include <vector>

#include "../../include/comet.h"
#include "comet_kernels.h"

using namespace comet;

namespace {

thread_local char g_hip_msg[256] = "no HIP error recorded";

int hip_fail(hipError_t e, const char *what) {
    snprintf(g_hip_msg, sizeof(g_hip_msg), "%s: %s", what, hipGetErrorString(e));
    return COMET_ERR_HIP;
}
#define HIP_TRY(expr)                                                   \
    do {                                                                \
        hipError_t e_ = (expr);                                         \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);               \
    } while (0)

constexpr uint64_t kMaxElems = (1ull << 31) - 1ull;
constexpr uint32_t kMaxW = 8192;
constexpr uint32_t kMaxBins = 65536;

inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

bool valid_eb(float eb) { return std::isfinite(eb) && eb >= 0x1p-100f && eb <= 0x1p100f; }
bool valid_nbins(uint32_t nb) { return nb >= 4u && nb <= kMaxBins && (nb & 1u) == 0u; }
bool valid_chunk(uint32_t s) { return s == 64u || s == 128u || s == 256u; }

bool shape_elems(comet_shape s, uint64_t *n) {
    if (!s.n || !s.c || !s.h || !s.w) return false;
    const uint64_t a = (uint64_t)s.n * s.c, b = (uint64_t)s.h * s.w;
    if (a > kMaxElems || b > kMaxElems) return false;
    const uint64_t t = a * b;
    if (t > kMaxElems) return false;
    *n = t;
    return true;
}

uint32_t ilog2(uint32_t v) { uint32_t l = 0; while ((1u << l) < v) ++l; return l; }

}  // namespace

// Persistent device words followed by the per-call control block.
struct DevState {
    uint32_t latched;      // first-come device errors since the last synchronising call
    uint32_t pad[3];
    Control ctl;
};

struct comet_ctx {
    int device = 0;
    int num_cu = 0;
    uint64_t max_elems = 0;
    uint32_t max_nbins = 0;
    uint32_t chunk_syms = COMET_DEFAULT_CHUNK_SYMS;
    uint32_t zero_chunks = 0;                       // containers of version 2: chunks of nothing but centre codes take no words
    // device memory
    DevState *state = nullptr;       // latched + Control, then histogram + descriptors (zero region)
    uint8_t *zero_region = nullptr;  // == (uint8_t*)&state->ctl
    uint64_t zero_cap = 0;
    uint16_t *codes = nullptr;
    uint32_t *rec_stage = nullptr;   // row-walking quantise kernel: staging area of every run's outlier records
    uint32_t *run_count = nullptr;   //   and per run: record count, non-zero inputs, verbatim records
    uint64_t max_runs = 0;
    uint64_t *enc = nullptr;
    BookScratch book{};
    DecodeTables tables{};
    void *tables_blob = nullptr;
    // pinned host
    DevState *host_state = nullptr;
    Header *host_hdr = nullptr;
    // occupancy (workgroups per CU) measured once
    double *stats = nullptr;      // kStatsPartialMax partial sums and, behind them, the mean
    int occ_quant = 1;
    // optional per-kernel timing
    struct Timed { uint32_t id; hipEvent_t a, b; };
    bool profiling = false;
    std::vector<Timed> pool;      // pre-created event pairs
    size_t used = 0;
};

namespace {

struct ZeroLayout {          // sub-allocation of the zero region for one call
    uint64_t off_hist, off_parts, off_desc_q, off_desc_e, bytes;
};

// partial histograms of the row-walking quantise kernel for an alphabet of nbins
uint32_t hist_copies(uint32_t nbins) {
    const uint32_t c = kQuantHistPartsWords / (nbins ? nbins : 1u);
    return c < 1u ? 1u : (c > kQuantHistCopiesMax ? kQuantHistCopiesMax : c);
}

// nbins_hist: entries of the histogram itself (0 if the caller brings its own), nbins_parts: alphabet
// the partial histograms are for (0: none)
ZeroLayout zero_layout(uint32_t nbins_hist, uint32_t nbins_parts, uint64_t tiles_q, uint64_t tiles_e) {
    ZeroLayout z;
    uint64_t o = align_up(sizeof(Control), 256);
    z.off_desc_q = o; o += align_up(8 * tiles_q, 256);
    z.off_desc_e = o; o += align_up(8 * tiles_e, 256);
    z.off_hist = o; o += align_up(4ull * nbins_hist, 256);
    z.off_parts = o; o += align_up(4ull * nbins_parts * hist_copies(nbins_parts), 256);
    z.bytes = o;
    return z;
}

int status_to_error(uint32_t st) {
    if (st & ST_INTERNAL) return COMET_ERR_INTERNAL;
    if (st & ST_CODEBOOK) return COMET_ERR_CODEBOOK;
    if (st & ST_FORMAT) return COMET_ERR_FORMAT;
    if (st & ST_CAPACITY) return COMET_ERR_CAPACITY;
    return COMET_OK;
}

// Clears the zero region of a call (control block, descriptors, histograms): one launch, and a plain
// kernel rather than a memset node for callers that capture the call in a graph.  n16: 16-byte words.
__global__ __launch_bounds__(256) void k_clear(uint4 *p, uint32_t n16) {
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ void k_latch(DevState *s) {           // fold this call's status into the persistent word
    if (s->ctl.status) atomicOr(&s->latched, s->ctl.status);
}

// Brackets a kernel launch with two events when profiling is on.
struct TimedScope {
    comet_ctx *c; hipStream_t st; comet_ctx::Timed *t = nullptr;
    TimedScope(comet_ctx *ctx, hipStream_t s, uint32_t id) : c(ctx), st(s) {
        if (c && c->profiling && c->used < c->pool.size()) {
            t = &c->pool[c->used++];
            t->id = id;
            (void)hipEventRecord(t->a, st);
        }
    }
    ~TimedScope() { if (t) (void)hipEventRecord(t->b, st); }
};

struct ReconGeometry { uint32_t planes_per_unit, tile_rows, n_units, pitch, use_carry; size_t lds; };

bool recon_geometry(comet_shape s, ReconGeometry *g) {
    const uint64_t planes = (uint64_t)s.n * s.c;
    const uint64_t P = (uint64_t)s.h * s.w;
    g->pitch = s.w | 1u;
    if (P <= kDecTileElems) {
        uint64_t G = kDecTileElems / P;
        if (G > planes) G = planes;
        g->planes_per_unit = (uint32_t)G;
        g->tile_rows = (uint32_t)(G * s.h);
        g->n_units = (uint32_t)((planes + G - 1) / G);
        g->use_carry = 0;
    } else {
        uint32_t R = kDecTileElems / s.w;
        if (R < 1) R = 1;
        if (R > s.h) R = s.h;
        g->planes_per_unit = 1;
        g->tile_rows = R;
        g->n_units = (uint32_t)planes;
        g->use_carry = 1;
    }
    g->lds = (size_t)g->tile_rows * g->pitch * 4u + (g->use_carry ? (size_t)s.w * 4u : 0u);
    return g->lds <= 96u * 1024u;
}

int fused_opt_in();          // k_decode_scan: opt in to its dynamic LDS size (defined with the decompression)
// segments of the encode kernel: (chunks per segment, number of segments)
void encode_geometry(const comet_ctx *ctx, uint64_t n_chunks, uint32_t *seg_chunks, uint32_t *n_seg);
// Work split of the quantise kernel.  rows: the row-walking kernel (planes up to kQuantRowsMaxW
// columns) with `grid` workgroups of four wavefronts, each wavefront on rows_per_wave consecutive
// rows; otherwise the flat-tile kernel with `grid` segments of tiles.
// vec: columns per lane of the row-walking kernel (2 if W is even and the input is 8-byte aligned).
// chunk_align: if not 0, every run is a whole number of chunks of that many symbols (single-pass compression).
struct QuantGeom { bool rows; uint32_t grid, rows_per_wave, rows_per_step, vec; };
// nbins: the alphabet (its histogram window decides how many workgroups a compute unit holds at once).
QuantGeom quantize_geometry(const comet_ctx *ctx, comet_shape s, uint64_t n, const void *x, uint32_t nbins, uint32_t elem_bytes = 4, uint32_t chunk_align = 0);

// Single-pass compression with a given code book: what the quantise kernel needs to encode its own codes.
struct SinglePass {
    const uint64_t *enc;       // encode table of the given lengths (k_codebook has run)
    uint32_t chunk_syms, zero_pair;
    uint32_t *chunk_off;       // chunk table of the container
    uint32_t *run_words;       // one entry per run
    uint32_t *work_words;      // n / 2 words
};

// reuse_len: code book reuse (device u8[nbins], row-walking kernel only, with sp); else null
// in_type: element type of x (0 fp32, COMET_F16, COMET_BF16; the 16-bit types: row-walking kernel only, no reuse)
int launch_quantize(comet_ctx *ctx, const void *x, comet_shape s, uint64_t n, float eb, uint32_t nbins,
                    hipStream_t st, uint16_t *codes, uint32_t *hist, uint32_t *hist_parts, uint32_t *rec, uint64_t rec_cap,
                    uint64_t *desc, const uint8_t *reuse_len = nullptr, int in_type = 0, const SinglePass *sp = nullptr) {
    if (in_type != 0 && (reuse_len || s.w > kQuantRowsMaxW)) return COMET_ERR_INVALID;
    if ((reuse_len != nullptr) != (sp != nullptr)) return COMET_ERR_INVALID;
    QuantArgs a{};
    a.x = x; a.n = n;
    a.divW = make_fastdiv(s.w); a.divH = make_fastdiv(s.h);
    a.eb = eb; a.ebx2 = 2.0f * eb; a.r = (float)(1.0 / (double)a.ebx2);
    a.radius = (int32_t)(nbins / 2u); a.nbins = nbins;
    a.win_n = nbins < kHistWindowMax ? nbins : kHistWindowMax;
    a.win_lo = (nbins - a.win_n) / 2u;
    a.n_tiles = (uint32_t)((n + kQuantTile - 1) / kQuantTile);
    a.codes = codes; a.hist = hist; a.rec = rec; a.rec_cap = rec_cap; a.desc = desc; a.ctl = &ctx->state->ctl;
    const QuantGeom g = quantize_geometry(ctx, s, n, x, nbins, in_type ? 2u : 4u, sp ? sp->chunk_syms : 0u);
    const uint32_t grid = g.grid;
    if (g.rows) {
        a.rows_total = (uint32_t)((uint64_t)s.n * s.c * s.h);
        a.rows_per_wave = g.rows_per_wave;
        a.rows_per_step = g.rows_per_step;
        if ((uint64_t)grid * (kQuantBlock / kWave) > ctx->max_runs) return COMET_ERR_INTERNAL;
        a.stage = ctx->rec_stage;
        a.run_count = ctx->run_count;
        a.hist_parts = hist_parts;
        a.hist_copies = hist_copies(nbins);
        a.hist_shift = a.win_n <= 2048u ? 2u : 0u;            // four copies while they fit 32 KB
        const bool full = a.win_n == nbins;
        const size_t lds = (((size_t)a.win_n << a.hist_shift) + kQuantBlock) * 4u + (full ? 0u : (size_t)(kQuantBlock / kWave) * kQuantOowList * 2u);
#define COMET_LAUNCH_QR_IN(VEC, NSEG, MULTI, IN)                                                                       \
        do {                                                                                                           \
            {                                                                                                          \
                TimedScope ts(ctx, st, COMET_KERNEL_QUANTIZE);                                                         \
                if (full) hipLaunchKernelGGL((k_quantize_rows<VEC, NSEG, MULTI, true, false, IN>), dim3(grid), dim3(kQuantBlock), lds, st, a);   \
                else hipLaunchKernelGGL((k_quantize_rows<VEC, NSEG, MULTI, false, false, IN>), dim3(grid), dim3(kQuantBlock), lds, st, a);       \
            }                                                                                                          \
            TimedScope ts(ctx, st, COMET_KERNEL_GATHER);                                                               \
            hipLaunchKernelGGL((k_gather_records<VEC, NSEG, MULTI, false, IN>), dim3(grid), dim3(kQuantBlock), 0, st, a); \
        } while (0)
#define COMET_LAUNCH_QR(VEC, NSEG, MULTI)                                                                              \
        do {                                                                                                           \
            if (in_type == COMET_F16) { COMET_LAUNCH_QR_IN(VEC, NSEG, MULTI, 1); break; }                              \
            if (in_type == COMET_BF16) { COMET_LAUNCH_QR_IN(VEC, NSEG, MULTI, 2); break; }                             \
            if (!reuse_len) { COMET_LAUNCH_QR_IN(VEC, NSEG, MULTI, 0); break; }                                        \
            {                                                                                                          \
                TimedScope ts(ctx, st, COMET_KERNEL_QUANTIZE);                                                         \
                if (a.enc_n == nbins) hipLaunchKernelGGL((k_quantize_rows<VEC, NSEG, MULTI, true, true>), dim3(grid), dim3(kQuantBlock), lds_single, st, a); \
                else hipLaunchKernelGGL((k_quantize_rows<VEC, NSEG, MULTI, false, true>), dim3(grid), dim3(kQuantBlock), lds_single, st, a);                 \
            }                                                                                                          \
            TimedScope ts(ctx, st, COMET_KERNEL_GATHER);                                                               \
            hipLaunchKernelGGL((k_gather_records<VEC, NSEG, MULTI, true>), dim3(grid), dim3(kQuantBlock), lds_reuse, st, a); \
        } while (0)
        a.reuse_len = reuse_len;
        const size_t lds_reuse = ((size_t)nbins + 7u) & ~(size_t)7u;    // the given length table, one byte per bin
        size_t lds_single = 0;
        if (sp) {
            // the kernel encodes its own codes: part of the encode table, a ring of codes and an assembly buffer per wavefront
            a.enc = sp->enc;
            a.enc_n = nbins < kEncTableMax ? nbins : kEncTableMax;
            a.enc_lo = (nbins - a.enc_n) / 2u;
            a.chunk_syms = sp->chunk_syms; a.zero_pair = sp->zero_pair;
            a.chunk_off = sp->chunk_off; a.run_words = sp->run_words; a.work_words = sp->work_words;
            lds_single = (a.enc_n == nbins ? 0u : lds_reuse) + ((size_t)a.enc_n + 1u) * 8u +
                         (size_t)(kQuantBlock / kWave) * ((kEncRingSyms + 4u) * 2u + kEncRunBufWords * 4u);
        }
        const uint32_t lanes_per_row = s.w / g.vec;
        if (g.vec == 2u) {
            if (lanes_per_row <= 32u) COMET_LAUNCH_QR(2, 1, true);
            else if (lanes_per_row <= 64u) COMET_LAUNCH_QR(2, 1, false);
            else if (lanes_per_row <= 128u) COMET_LAUNCH_QR(2, 2, false);
            else COMET_LAUNCH_QR(2, 4, false);
        } else {
            if (lanes_per_row <= 32u) COMET_LAUNCH_QR(1, 1, true);
            else if (lanes_per_row <= 64u) COMET_LAUNCH_QR(1, 1, false);
            else if (lanes_per_row <= 128u) COMET_LAUNCH_QR(1, 2, false);
            else if (lanes_per_row <= 256u) COMET_LAUNCH_QR(1, 4, false);
            else COMET_LAUNCH_QR(1, 8, false);
        }
#undef COMET_LAUNCH_QR
#undef COMET_LAUNCH_QR_IN
    } else {
        if (reuse_len) return COMET_ERR_INVALID;          // the flat-tile kernel has no code book reuse
        // one segment of consecutive tiles per workgroup, about as many workgroups as fit the chip at once
        a.tiles_per_seg = (a.n_tiles + grid - 1) / grid;
        a.rec_lds = kQuantRecLds;
        const size_t lds = (size_t)a.win_n * 4u + (size_t)kQuantRecLds * 8u;
        TimedScope ts(ctx, st, COMET_KERNEL_QUANTIZE);
        if (a.win_n == nbins) hipLaunchKernelGGL(k_quantize<true>, dim3(grid), dim3(kQuantBlock), lds, st, a);
        else hipLaunchKernelGGL(k_quantize<false>, dim3(grid), dim3(kQuantBlock), lds, st, a);
    }
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

// The code book kernel, behind the sort kernels that an alphabet too large for LDS needs.  b.ctl->n_active
// must be zero on entry (the call's control block has just been cleared).
int launch_codebook(comet_ctx *ctx, BookArgs &b, hipStream_t st) {
    TimedScope ts(ctx, st, COMET_KERNEL_CODEBOOK);
    // (up to kBookBySymbolMax bins the occurring symbols mostly fit LDS, and the launches would cost more than
    // the kernel's own sort does when they do not)
    if (!b.given_len && b.nbins > kBookBySymbolMax) {
        uint32_t tiles = 1;
        while (tiles * (uint32_t)kBookBlock < b.nbins) tiles <<= 1;
        const uint32_t total = tiles * (uint32_t)kBookBlock;          // <= kMaxBins: what the scratch arrays hold
        uint64_t *src = b.scratch.keys, *dst = b.scratch.iw;
        hipLaunchKernelGGL(k_book_sort_tiles, dim3(tiles), dim3(kBookBlock), 0, st, b.hist, b.nbins, src, b.ctl);
        for (uint32_t run = (uint32_t)kBookBlock; run < total; run <<= 1) {
            hipLaunchKernelGGL(k_book_merge, dim3(total / (uint32_t)kBookMergeBlock), dim3(kBookMergeBlock), 0, st, src, dst, run, b.ctl);
            uint64_t *t = src; src = dst; dst = t;
        }
        b.scratch.keys = src; b.scratch.iw = dst;
        b.presorted = 1u;
    }
    hipLaunchKernelGGL(k_codebook, dim3(1), dim3(kBookBlock), 0, st, b);
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

int launch_encode(comet_ctx *ctx, const uint16_t *codes, uint64_t n, uint32_t nbins, uint32_t chunk_syms,
                  hipStream_t st, uint32_t *chunk_off, uint8_t *container, uint64_t capacity,
                  uint32_t *payload, uint64_t payload_cap, uint64_t *payload_words_out, uint64_t *desc) {
    EncodeArgs a{};
    a.len8 = container ? container + kHeaderBytes : nullptr;      // the length section k_codebook has written
    a.codes = codes; a.n = n; a.chunk_syms = chunk_syms;
    a.zero_pair = ctx->zero_chunks ? ((nbins / 2u) << 16) | (nbins / 2u) : 0u;
    a.n_chunks = (uint32_t)((n + chunk_syms - 1) / chunk_syms);
    a.enc = ctx->enc; a.nbins = nbins;
    a.tbl_n = nbins < kEncTableMax ? nbins : kEncTableMax;
    a.tbl_lo = (nbins - a.tbl_n) / 2u;
    uint32_t seg, grid;
    encode_geometry(ctx, a.n_chunks, &seg, &grid);
    a.seg_chunks = seg;
    // table and a zero entry (or, for a large alphabet, the lengths of enc_len_window() symbols: whichever is larger), word counts
    const size_t lenw = enc_len_window(nbins) + 8u;
    const size_t tbl_bytes = ((size_t)a.tbl_n + 1u) * 8u;
    a.tbl_room = (uint32_t)((a.tbl_n < nbins && lenw > tbl_bytes ? lenw : tbl_bytes) + 7u) & ~7u;
    const size_t lds_count = (size_t)a.tbl_room + (size_t)seg * 4u;
    const size_t lds_pack = ((size_t)a.tbl_n + 1u) * 8u + (size_t)(kEncBlock / kWave) * kEncBufWords * 4u;
    a.chunk_off = chunk_off; a.container = container; a.capacity = capacity;
    a.payload = payload; a.payload_cap_words = payload_cap; a.payload_words_out = payload_words_out;
    a.desc = desc; a.ctl = &ctx->state->ctl;
    a.latched = container ? &ctx->state->latched : nullptr;
    const bool full = (a.tbl_n == nbins);
#define COMET_LAUNCH_ENC(S)                                                                                            \
    do {                                                                                                               \
        {                                                                                                              \
            TimedScope ts(ctx, st, COMET_KERNEL_ENCODE_COUNT);                                                         \
            if (full) hipLaunchKernelGGL((k_encode_count<S, true>), dim3(grid), dim3(kEncBlock), lds_count, st, a);    \
            else hipLaunchKernelGGL((k_encode_count<S, false>), dim3(grid), dim3(kEncBlock), lds_count, st, a);        \
        }                                                                                                              \
        TimedScope ts(ctx, st, COMET_KERNEL_ENCODE);                                                                   \
        if (full) hipLaunchKernelGGL((k_encode_pack<S, true>), dim3(grid), dim3(kEncBlock), lds_pack, st, a);          \
        else hipLaunchKernelGGL((k_encode_pack<S, false>), dim3(grid), dim3(kEncBlock), lds_pack, st, a);              \
    } while (0)
    if (chunk_syms == 64u) COMET_LAUNCH_ENC(64);
    else if (chunk_syms == 128u) COMET_LAUNCH_ENC(128);
    else COMET_LAUNCH_ENC(256);
#undef COMET_LAUNCH_ENC
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

void encode_geometry(const comet_ctx *ctx, uint64_t n_chunks, uint32_t *seg_chunks, uint32_t *n_seg) {
    // one segment of consecutive chunks per workgroup: about as many segments as workgroups fit the chip
    const uint64_t want = (uint64_t)ctx->num_cu * 6u;
    uint64_t seg = (n_chunks + want - 1) / want;
    seg = (seg + 3u) & ~(uint64_t)3u;
    if (seg < 4u) seg = 4u;
    if (seg > kEncSegChunksMax) seg = kEncSegChunksMax;
    *seg_chunks = (uint32_t)seg;
    *n_seg = (uint32_t)((n_chunks + seg - 1) / seg);
}

QuantGeom quantize_geometry(const comet_ctx *ctx, comet_shape s, uint64_t n, const void *x, uint32_t nbins, uint32_t elem_bytes, uint32_t chunk_align) {
    QuantGeom g{};
    g.vec = 1;
    if (s.w <= kQuantRowsMaxW) {
        g.rows = true;
        const uint64_t rows_total = (uint64_t)s.n * s.c * s.h;
        // two columns per lane: every row then starts at an even element, so pairs are aligned to their size
        if ((s.w & 1u) == 0u && ((uintptr_t)x & (2u * elem_bytes - 1u)) == 0u) g.vec = 2;
        const uint32_t lanes_per_row = s.w / g.vec;
        const uint32_t K = lanes_per_row <= 32u ? (uint32_t)kWave / lanes_per_row : 1u;
        g.rows_per_step = K;
        // runs of whole steps; single-pass compression: and of whole chunks (chunk sizes are powers of two)
        uint32_t unit = K;
        if (chunk_align) {
            uint32_t rows_per_chunk = chunk_align;               // rows after which a chunk boundary is a row boundary
            for (uint32_t w = s.w; (w & 1u) == 0u && rows_per_chunk > 1u; w >>= 1) rows_per_chunk >>= 1;
            unit = K / std::gcd(K, rows_per_chunk) * rows_per_chunk;
        }
        // a few wavefronts per SIMD, but runs of at least 2048 elements (every run re-reads one row)
        // All runs should be resident at once: a run that has to wait for a place makes the launch take two rounds.
        // A workgroup is one wavefront per SIMD; how many a compute unit holds follows from the LDS they need (the
        // histogram window of a large alphabet leaves room for three; the encoder's ring and tables of the single-pass
        // compression for four).
        uint32_t runs_per_simd = chunk_align ? kQuantRunsPerSimdSingle : kQuantRunsPerSimd;
        if (!chunk_align) {
            const uint32_t win_n = nbins < kHistWindowMax ? nbins : kHistWindowMax;
            const size_t lds = (((size_t)win_n << (win_n <= 2048u ? 2u : 0u)) + kQuantBlock) * 4u + kQuantStaticLds +
                               (win_n < nbins ? (size_t)(kQuantBlock / kWave) * kQuantOowList * 2u : 0u);
            const uint32_t fit = (uint32_t)(kLdsPerCu / lds);
            if (fit < runs_per_simd) runs_per_simd = fit ? fit : 1u;
        }
        const uint64_t want = (uint64_t)ctx->num_cu * 4u * runs_per_simd;
        uint64_t per = (rows_total + want - 1) / want;
        const uint64_t min_rows = (2048u + s.w - 1u) / s.w;
        if (per < min_rows) per = min_rows;
        per = (per + unit - 1) / unit * unit;
        if (per > rows_total) per = (rows_total + unit - 1) / unit * unit;
        // a run must stay below 2^28 elements (buffer offsets): cannot be exceeded, rows_total * w < 2^31 and
        // the run count is in the thousands unless the tensor itself is small
        const uint64_t waves = (rows_total + per - 1) / per;
        g.rows_per_wave = (uint32_t)per;
        g.grid = (uint32_t)((waves + (kQuantBlock / kWave) - 1) / (kQuantBlock / kWave));
        return g;
    }
    const uint64_t n_tiles = (n + kQuantTile - 1) / kQuantTile;
    uint64_t grid = (uint64_t)ctx->num_cu * (uint64_t)ctx->occ_quant;
    if (grid > n_tiles) grid = n_tiles;
    const uint64_t per = (n_tiles + grid - 1) / grid;
    g.grid = (uint32_t)((n_tiles + per - 1) / per);
    return g;
}

}  // namespace

extern "C" {

int comet_create(comet_ctx **out, uint64_t max_elems, uint32_t max_nbins) {
    if (!out || max_elems == 0 || max_elems > kMaxElems || !valid_nbins(max_nbins)) return COMET_ERR_INVALID;
    comet_ctx *c = new (std::nothrow) comet_ctx();
    if (!c) return COMET_ERR_NOMEM;
    c->max_elems = max_elems;
    c->max_nbins = max_nbins;
    int rc = COMET_OK;
    auto fail = [&](int code) { comet_destroy(c); return code; };
    hipError_t e;
    if ((e = hipGetDevice(&c->device)) != hipSuccess) return fail(hip_fail(e, "hipGetDevice"));
    hipDeviceProp_t prop;
    if ((e = hipGetDeviceProperties(&prop, c->device)) != hipSuccess) return fail(hip_fail(e, "hipGetDeviceProperties"));
    c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // scan descriptors: one per segment of the quantise / encode kernels (worst case over chunk sizes)
    const uint64_t tiles_q = (uint64_t)c->num_cu * 16u + 16u;
    const uint64_t tiles_e = (uint64_t)c->num_cu * 8u + max_elems / 64u / kEncSegChunksMax + 16u;
    const ZeroLayout z = zero_layout(kMaxBins, kMaxBins, tiles_q, tiles_e);   // the partial histograms take up to 2 MB
    c->zero_cap = z.bytes;
    const uint64_t state_bytes = offsetof(DevState, ctl) + z.bytes;
    if ((e = hipMalloc((void **)&c->state, state_bytes)) != hipSuccess) return fail(COMET_ERR_NOMEM);
    if ((e = hipMemset(c->state, 0, state_bytes)) != hipSuccess) return fail(hip_fail(e, "hipMemset"));
    c->zero_region = reinterpret_cast<uint8_t *>(&c->state->ctl);
    if ((e = hipMalloc((void **)&c->codes, align_up(2 * max_elems + 64, 256))) != hipSuccess) return fail(COMET_ERR_NOMEM);
    if ((e = hipMalloc((void **)&c->enc, 8ull * kMaxBins)) != hipSuccess) return fail(COMET_ERR_NOMEM);
    if ((e = hipMalloc((void **)&c->stats, 8ull * (kStatsPartialMax + 1u))) != hipSuccess) return fail(COMET_ERR_NOMEM);
    c->max_runs = (uint64_t)c->num_cu * 4u * kQuantRunsPerSimd + 8u;
    if ((e = hipMalloc((void **)&c->rec_stage, c->max_runs * kQuantRecRun * 8ull)) != hipSuccess) return fail(COMET_ERR_NOMEM);
    // (a fourth array of one entry per run: the words of every run of the single-pass compression)
    if ((e = hipMalloc((void **)&c->run_count, 4ull * c->max_runs * 4ull)) != hipSuccess) return fail(COMET_ERR_NOMEM);
    {
        // one blob: book scratch + decode tables
        uint64_t o = 0;
        const uint64_t o_keys = o; o += 8ull * kMaxBins;
        const uint64_t o_iw = o; o += 8ull * kMaxBins;
        const uint64_t o_lp = o; o += 4ull * kMaxBins;
        const uint64_t o_ip = o; o += 4ull * kMaxBins;
        const uint64_t o_limit = o; o += 8ull * 72;
        const uint64_t o_first = o; o += 8ull * 72;
        const uint64_t o_findex = o; o += 4ull * 72;
        const uint64_t o_lut = o; o += 4ull * kLutSize;
        const uint64_t o_lut16 = o; o += 2ull * kLut16Size;
        const uint64_t o_sub16 = o; o += 2ull * kSubEntries;
        const uint64_t o_meta = o; o += 64;
        const uint64_t o_sorted = o; o += 2ull * kMaxBins;
        uint8_t *blob = nullptr;
        if ((e = hipMalloc((void **)&blob, align_up(o, 256))) != hipSuccess) return fail(COMET_ERR_NOMEM);
        c->tables_blob = blob;
        c->book.keys = (uint64_t *)(blob + o_keys); c->book.iw = (uint64_t *)(blob + o_iw);
        c->book.leaf_parent = (uint32_t *)(blob + o_lp); c->book.int_parent = (uint32_t *)(blob + o_ip);
        c->tables.limit = (uint64_t *)(blob + o_limit); c->tables.first_code = (uint64_t *)(blob + o_first);
        c->tables.first_index = (uint32_t *)(blob + o_findex); c->tables.lut = (uint32_t *)(blob + o_lut);
        c->tables.meta = (uint32_t *)(blob + o_meta); c->tables.sorted = (uint16_t *)(blob + o_sorted);
        c->tables.lut16 = (uint16_t *)(blob + o_lut16);
        c->tables.sub16 = (uint16_t *)(blob + o_sub16);
    }
    if ((e = hipHostMalloc((void **)&c->host_state, sizeof(DevState) + sizeof(Header), hipHostMallocDefault)) != hipSuccess)
        return fail(COMET_ERR_NOMEM);
    c->host_hdr = reinterpret_cast<Header *>(reinterpret_cast<uint8_t *>(c->host_state) + sizeof(DevState));

    // kernels that need more than 64 KB of dynamic LDS must opt in
    if ((e = hipFuncSetAttribute((const void *)k_reconstruct<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024)) != hipSuccess)
        return fail(hip_fail(e, "hipFuncSetAttribute(k_reconstruct<0>)"));
    if ((e = hipFuncSetAttribute((const void *)k_reconstruct<1>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024)) != hipSuccess)
        return fail(hip_fail(e, "hipFuncSetAttribute(k_reconstruct<1>)"));
    if (fused_opt_in() != COMET_OK) return fail(COMET_ERR_HIP);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&c->occ_quant, k_quantize<true>, kQuantBlock, 4096 + kQuantRecLds * 8) != hipSuccess || c->occ_quant < 1) c->occ_quant = 4;
    (void)rc;
    *out = c;
    return COMET_OK;
}

void comet_destroy(comet_ctx *c) {
    if (!c) return;
    if (c->state) (void)hipFree(c->state);
    if (c->codes) (void)hipFree(c->codes);
    if (c->stats) (void)hipFree(c->stats);
    if (c->rec_stage) (void)hipFree(c->rec_stage);
    if (c->run_count) (void)hipFree(c->run_count);
    if (c->enc) (void)hipFree(c->enc);
    if (c->tables_blob) (void)hipFree(c->tables_blob);
    if (c->host_state) (void)hipHostFree(c->host_state);
    for (auto &t : c->pool) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
    delete c;
}

int comet_set_zero_chunks(comet_ctx *ctx, int enable) {
    if (!ctx) return COMET_ERR_INVALID;
    ctx->zero_chunks = enable ? 1u : 0u;
    return COMET_OK;
}

int comet_set_chunk_syms(comet_ctx *ctx, uint32_t chunk_syms) {
    if (!ctx || !valid_chunk(chunk_syms)) return COMET_ERR_INVALID;
    ctx->chunk_syms = chunk_syms;
    return COMET_OK;
}

uint64_t comet_compress_bound(comet_shape s, uint32_t nbins, uint32_t chunk_syms) {
    uint64_t n;
    if (!shape_elems(s, &n) || !valid_nbins(nbins) || chunk_syms == 0) return 0;
    const uint64_t n_chunks = (n + chunk_syms - 1) / chunk_syms;
    uint64_t sz = kHeaderBytes;
    sz = align16(sz + nbins);
    sz = align16(sz + 4 * n_chunks);
    sz = align16(sz + 16 * n);                          // every element both escaped and verbatim
    sz += 4 * ((17 * n + 31) / 32 + n_chunks);         // an optimal code averages < log2(nbins) + 1 <= 17 bits
    return sz;
}

namespace {
int compress_impl(comet_ctx *ctx, const void *dev_in, int in_type, comet_shape s, float eb, uint32_t nbins, const uint8_t *dev_len,
                  void *stream, void *dev_out, uint64_t capacity, uint64_t *bytes_out);
}

int comet_compress(comet_ctx *ctx, const float *dev_in, comet_shape s, float eb, uint32_t nbins,
                   void *stream, void *dev_out, uint64_t capacity, uint64_t *bytes_out) {
    return compress_impl(ctx, dev_in, 0, s, eb, nbins, nullptr, stream, dev_out, capacity, bytes_out);
}

int comet_compress_16(comet_ctx *ctx, const void *dev_in, int dtype, comet_shape s, float eb, uint32_t nbins,
                      void *stream, void *dev_out, uint64_t capacity, uint64_t *bytes_out) {
    if ((dtype != COMET_F16 && dtype != COMET_BF16) || s.w > kQuantRowsMaxW) return COMET_ERR_INVALID;
    return compress_impl(ctx, dev_in, dtype, s, eb, nbins, nullptr, stream, dev_out, capacity, bytes_out);
}

int comet_compress_with_codebook(comet_ctx *ctx, const float *dev_in, comet_shape s, float eb, uint32_t nbins,
                                 const uint8_t *dev_len, void *stream, void *dev_out, uint64_t capacity,
                                 uint64_t *bytes_out) {
    if (!dev_len || nbins > kQuantReuseMaxBins || s.w > kQuantRowsMaxW) return COMET_ERR_INVALID;
    return compress_impl(ctx, dev_in, 0, s, eb, nbins, dev_len, stream, dev_out, capacity, bytes_out);
}

namespace {
int compress_impl(comet_ctx *ctx, const void *dev_in, int in_type, comet_shape s, float eb, uint32_t nbins, const uint8_t *dev_len,
                  void *stream, void *dev_out, uint64_t capacity, uint64_t *bytes_out) {
    uint64_t n;
    if (!ctx || !dev_in || !dev_out || !shape_elems(s, &n) || !valid_eb(eb) || !valid_nbins(nbins) ||
        s.w > kMaxW || ((uintptr_t)dev_out & 15u) || ((uintptr_t)dev_in & 15u)) return COMET_ERR_INVALID;
    if (n > ctx->max_elems || nbins > ctx->max_nbins) return COMET_ERR_NOMEM;
    hipStream_t st = (hipStream_t)stream;
    const uint32_t S = ctx->chunk_syms;
    const uint64_t n_chunks = (n + S - 1) / S;
    uint32_t e_seg, e_grid;
    encode_geometry(ctx, n_chunks, &e_seg, &e_grid);
    const uint64_t tiles_q = quantize_geometry(ctx, s, n, dev_in, nbins, in_type ? 2u : 4u, dev_len ? S : 0u).grid;
    const uint64_t tiles_e = e_grid;

    Header proto{};
    proto.magic = kMagic; proto.version = ctx->zero_chunks ? 2u : 1u; proto.N = s.n; proto.C = s.c; proto.H = s.h; proto.W = s.w;
    proto.nbins = nbins; proto.chunk_syms = S; proto.n_chunks = (uint32_t)n_chunks;
    const float ebx2 = 2.0f * eb;
    const float r = (float)(1.0 / (double)ebx2);
    memcpy(&proto.eb_bits, &eb, 4); memcpy(&proto.ebx2_bits, &ebx2, 4); memcpy(&proto.r_bits, &r, 4);
    proto.off_len = kHeaderBytes;
    proto.off_chunk = align16(proto.off_len + nbins);
    proto.off_outlier = align16(proto.off_chunk + 4 * n_chunks);
    if (proto.off_outlier > capacity) return COMET_ERR_CAPACITY;

    const ZeroLayout z = zero_layout(nbins, nbins, tiles_q, tiles_e);
    if (z.bytes > ctx->zero_cap) return COMET_ERR_NOMEM;
    {
        const uint32_t n16 = (uint32_t)(z.bytes / 16u);      // the layout is made of 256-byte pieces
        hipLaunchKernelGGL(k_clear, dim3((n16 + 255u) / 256u), dim3(256), 0, st, reinterpret_cast<uint4 *>(ctx->zero_region), n16);
        HIP_TRY(hipGetLastError());
    }
    uint32_t *hist = reinterpret_cast<uint32_t *>(ctx->zero_region + z.off_hist);
    uint32_t *hist_parts = reinterpret_cast<uint32_t *>(ctx->zero_region + z.off_parts);
    uint64_t *desc_q = reinterpret_cast<uint64_t *>(ctx->zero_region + z.off_desc_q);
    uint64_t *desc_e = reinterpret_cast<uint64_t *>(ctx->zero_region + z.off_desc_e);
    uint8_t *out = static_cast<uint8_t *>(dev_out);

    BookArgs b{};
    b.hist = hist; b.given_len = dev_len; b.nbins = nbins; b.len_out = out + proto.off_len; b.code_out = nullptr; b.enc = ctx->enc;
    b.scratch = ctx->book; b.ctl = &ctx->state->ctl; b.hdr = reinterpret_cast<Header *>(out); b.proto = proto; b.capacity = capacity;
    uint32_t *rec = reinterpret_cast<uint32_t *>(out + proto.off_outlier);
    const uint64_t rec_cap = (capacity - proto.off_outlier) / 8u;
    uint32_t *chunk_off = reinterpret_cast<uint32_t *>(out + proto.off_chunk);
    int rc;
    if (dev_len) {
        // Single pass over the input: the code book first (header, length section, encode table), then the quantise
        // kernel encodes its own codes into the work area, then the words of every run move to their place.
        if ((rc = launch_codebook(ctx, b, st))) return rc;
        const QuantGeom g = quantize_geometry(ctx, s, n, dev_in, nbins, 4u, S);
        SinglePass sp{};
        sp.enc = ctx->enc; sp.chunk_syms = S;
        sp.zero_pair = ctx->zero_chunks ? ((nbins / 2u) << 16) | (nbins / 2u) : 0u;
        sp.chunk_off = chunk_off;
        sp.run_words = ctx->run_count + 3u * ctx->max_runs;
        sp.work_words = reinterpret_cast<uint32_t *>(ctx->codes);
        if ((rc = launch_quantize(ctx, dev_in, s, n, eb, nbins, st, nullptr, hist, hist_parts, rec, rec_cap, desc_q, dev_len, 0, &sp))) return rc;
        PlaceArgs p{};
        p.run_words = sp.run_words;
        p.rows_per_wave = g.rows_per_wave; p.rows_total = (uint32_t)((uint64_t)s.n * s.c * s.h); p.W = s.w;
        p.n_runs = (p.rows_total + g.rows_per_wave - 1u) / g.rows_per_wave;
        p.chunk_syms = S; p.work_words = sp.work_words; p.container = out; p.capacity = capacity;
        p.ctl = &ctx->state->ctl; p.latched = &ctx->state->latched;
        constexpr uint32_t per_wg = (uint32_t)(kPlaceBlock / kWave);
        TimedScope ts(ctx, st, COMET_KERNEL_ENCODE);
        hipLaunchKernelGGL(k_place_payload, dim3((p.n_runs + per_wg - 1u) / per_wg), dim3(kPlaceBlock), 0, st, p);
        HIP_TRY(hipGetLastError());
    } else {
        if ((rc = launch_quantize(ctx, dev_in, s, n, eb, nbins, st, ctx->codes, hist, hist_parts, rec, rec_cap, desc_q, nullptr, in_type))) return rc;
        if ((rc = launch_codebook(ctx, b, st))) return rc;
        if ((rc = launch_encode(ctx, ctx->codes, n, nbins, S, st, chunk_off, out, capacity, nullptr, 0, nullptr, desc_e))) return rc;
    }
    if (bytes_out) {
        HIP_TRY(hipMemcpyAsync(ctx->host_state, ctx->state, sizeof(DevState), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        // this call's own bits, and whatever earlier asynchronous calls on this context have latched
        const uint32_t own = ctx->host_state->ctl.status;
        const uint32_t stt = own | ctx->host_state->latched;
        if (!own) *bytes_out = ctx->host_state->ctl.total_bytes;
        if (stt) {
            HIP_TRY(hipMemsetAsync(&ctx->state->latched, 0, 4, st));
            HIP_TRY(hipStreamSynchronize(st));
            return status_to_error(stt);
        }
    }
    return COMET_OK;
}
}  // namespace

namespace {
// What a decompression needs beyond its input and its output: the control block, the decode tables and the
// residual work buffer, in a context's workspace or in the library's static scratch array.
struct DecompWs {
    DevState *state;
    DecodeTables tables;
    int16_t *resid;            // one int16 per element, max_elems of them
    uint64_t max_elems;
    int num_cu;
    uint32_t chunk_syms;       // chunk size the launch geometry is estimated with
    comet_ctx *prof;           // per-kernel timing, or null
    int32_t *dev_status;       // if set, the tables kernel stores 0 or COMET_ERR_FORMAT there
};
int decompress_impl(const DecompWs &ws, const void *dev_in, uint64_t bytes, comet_shape s, void *stream, void *dev_out, int out_type);
DecompWs ctx_ws(comet_ctx *ctx) {
    DecompWs ws{};
    ws.state = ctx->state; ws.tables = ctx->tables; ws.resid = reinterpret_cast<int16_t *>(ctx->codes);
    ws.max_elems = ctx->max_elems; ws.num_cu = ctx->num_cu; ws.chunk_syms = ctx->chunk_syms; ws.prof = ctx; ws.dev_status = nullptr;
    return ws;
}
}

int comet_decompress(comet_ctx *ctx, const void *dev_in, uint64_t bytes, comet_shape s, void *stream, float *dev_out) {
    if (!ctx) return COMET_ERR_INVALID;
    return decompress_impl(ctx_ws(ctx), dev_in, bytes, s, stream, dev_out, 0);
}

int comet_decompress_16(comet_ctx *ctx, const void *dev_in, uint64_t bytes, comet_shape s, int dtype, void *stream, void *dev_out) {
    if (!ctx || (dtype != COMET_F16 && dtype != COMET_BF16)) return COMET_ERR_INVALID;
    return decompress_impl(ctx_ws(ctx), dev_in, bytes, s, stream, dev_out, dtype);
}

namespace {
constexpr size_t kFuLdsBytes = (size_t)kFuWaves * kFuRegionWords * 4u;

// instantiation of k_decode_scan for (64-lane segments per row, lane mapping, output type, columns per lane)
const void *fused_kernel(int nseg, int mode, int out, int vec) {
#define COMET_FU(NS, MO, OU, VE) if (nseg == NS && mode == MO && out == OU && vec == VE) return (const void *)k_decode_scan<NS, MO, OU, VE>;
#define COMET_FU_OUT(OU)                                                                     \
    COMET_FU(1, 0, OU, 1) COMET_FU(1, 1, OU, 1) COMET_FU(1, 2, OU, 1) COMET_FU(2, 2, OU, 1) \
    COMET_FU(4, 2, OU, 1) COMET_FU(8, 2, OU, 1) COMET_FU(1, 0, OU, 2) COMET_FU(1, 1, OU, 2) \
    COMET_FU(1, 2, OU, 2) COMET_FU(2, 2, OU, 2) COMET_FU(4, 2, OU, 2)
    COMET_FU_OUT(0) COMET_FU_OUT(1) COMET_FU_OUT(2)
#undef COMET_FU_OUT
#undef COMET_FU
    return nullptr;
}

// every instantiation needs more than 64 KB of dynamic LDS: opt in once per device
int fused_opt_in() {
    static const int nsegs[] = {1, 2, 4, 8};
    for (int out = 0; out < 3; ++out)
        for (int vec = 1; vec <= 2; ++vec)
            for (int mode = 0; mode < 3; ++mode)
                for (int ns : nsegs) {
                    const void *fn = fused_kernel(ns, mode, out, vec);
                    if (fn) HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFuLdsBytes));
                }
    return COMET_OK;
}

// Work split of k_decode_scan: units of G whole planes, one wavefront per unit at a time.  A unit costs as
// many strips (decode phases of 64 symbols per lane) as its elements take at about 4032 per strip, and the
// launch takes as long as its busiest wavefront: G minimises (units per wavefront) * (strips per unit).
struct FusedGeom { uint32_t G, n_units, grid; };
FusedGeom fused_geometry(int num_cu, comet_shape s) {
    const uint64_t planes = (uint64_t)s.n * s.c, P = (uint64_t)s.h * s.w;
    const uint64_t waves = (uint64_t)num_cu * kFuWaves;
    auto strips_of = [&](uint64_t G) {                       // a unit that starts on a chunk boundary
        uint64_t a = 0, cnt = 0;
        const uint64_t end = G * P;
        while (a < end) {
            uint64_t lim = ((a >> 6) + 64u) * 64u / s.w * s.w;
            a = lim < end ? lim : end;
            ++cnt;
        }
        return cnt;
    };
    uint64_t g_max = 2u * ((planes + waves - 1) / waves) + 2u * (4096u / P) + 2u;
    if (g_max > planes) g_max = planes;
    uint64_t best_g = 1, best_cost = ~0ull;
    for (uint64_t G = 1; G <= g_max; ++G) {
        const uint64_t units = (planes + G - 1) / G;
        const uint64_t cost = ((units + waves - 1) / waves) * strips_of(G);
        if (cost < best_cost) { best_cost = cost; best_g = G; }
    }
    FusedGeom f;
    f.G = (uint32_t)best_g;
    f.n_units = (uint32_t)((planes + best_g - 1) / best_g);
    f.grid = (uint32_t)(f.n_units < (uint64_t)num_cu ? f.n_units : (uint64_t)num_cu);
    return f;
}

int decompress_impl(const DecompWs &ws, const void *dev_in, uint64_t bytes, comet_shape s, void *stream, void *dev_out, int out_type) {
    uint64_t n;
    if (!dev_in || !dev_out || !shape_elems(s, &n) || s.w > kMaxW || ((uintptr_t)dev_in & 15u)) return COMET_ERR_INVALID;
    if (bytes < kHeaderBytes) return COMET_ERR_FORMAT;
    if (n > ws.max_elems) return COMET_ERR_NOMEM;        // the work buffer holds one residual per element of the context's size
    hipStream_t st = (hipStream_t)stream;
    ReconGeometry g;
    if (!recon_geometry(s, &g)) return COMET_ERR_INVALID;
    const uint8_t *in = static_cast<const uint8_t *>(dev_in);
    // scan kernel: two adjacent columns per lane if every pair is aligned in the output; a row then takes
    // lpr lanes, and ppi planes lie side by side in a wavefront
    const uint32_t out_elem = out_type ? 2u : 4u;
    const uint32_t vec = ((s.w & 1u) == 0u && ((uintptr_t)dev_out & (2u * out_elem - 1u)) == 0u) ? 2u : 1u;
    const uint32_t lpr = s.w / vec;
    const uint32_t ppi = lpr <= 16u ? 4u * (16u / lpr) : (lpr <= 32u ? 2u : 1u);
    const bool fast_path = s.w <= kDsMaxW && (uint64_t)ppi * s.h * s.w < (1ull << 28);
    if (out_type != 0 && !fast_path) return COMET_ERR_INVALID;       // 16-bit outputs: planes of at most kDsMaxW columns
    // Chunks of 64 symbols (what the caller's context compresses with tells what to expect) go through the
    // single fused kernel; it leaves a container with another chunk size alone, and the kernels launched
    // behind it, which take any chunk size, leave one with 64 alone.
    const bool fused = fast_path && ws.chunk_syms == 64u;
    {
        TablesArgs t{};
        t.len = in + kHeaderBytes; t.nbins = 0; t.t = ws.tables; t.ctl = &ws.state->ctl;
        t.hdr = reinterpret_cast<const Header *>(in);
        t.expect.N = s.n; t.expect.C = s.c; t.expect.H = s.h; t.expect.W = s.w; t.bytes = bytes;
        t.compact_only = fast_path ? 1u : 0u;
        t.general_unless_chunk64 = (fused && out_type == 0) ? 1u : 0u;   // the kernel behind k_decode_scan reads the general table
        // the only kernel of a decompression that raises status bits: it clears the call's control block itself
        // and latches what it raises, so the call needs neither a fill before nor a kernel after
        t.reset_ctl = 1u; t.latched = &ws.state->latched; t.status_out = ws.dev_status;
        {
            TimedScope ts(ws.prof, st, COMET_KERNEL_TABLES);
            hipLaunchKernelGGL(k_decode_tables, dim3(1), dim3(kBookBlock), 0, st, t);
        }
        HIP_TRY(hipGetLastError());
    }
    if (fused) {
        FuArgs f{};
        f.container = in; f.t = ws.tables; f.n = n; f.planes = s.n * s.c; f.H = s.h; f.W = s.w;
        f.divW = make_fastdiv(s.w); f.divH = make_fastdiv(s.h); f.divL = make_fastdiv(lpr);
        f.divSpr = make_fastdiv(lpr <= 16u ? 16u / lpr : 1u);
        f.divK = make_fastdiv(lpr <= 16u ? 4u * (16u / lpr) : (lpr <= 32u ? 2u : 1u));
        f.out = dev_out; f.ctl = &ws.state->ctl;
        const int mode = lpr <= 16u ? 0 : (lpr <= 32u ? 1 : 2);
        const int nseg = lpr <= 64u ? 1 : (lpr <= 128u ? 2 : (lpr <= 256u ? 4 : 8));
        // planes of at most 128 lanes per row: one segment of planes per workgroup, its strips dealt to all its
        // wavefronts; wider planes: units of whole planes per wavefront
        const bool coop = nseg <= 2;
        FusedGeom fg = fused_geometry(ws.num_cu, s);
        if (coop) {
            const uint64_t planes = (uint64_t)s.n * s.c;
            fg.grid = (uint32_t)(planes < (uint64_t)ws.num_cu ? planes : (uint64_t)ws.num_cu);
        }
        f.G = fg.G; f.n_units = fg.n_units;
        const void *fn = fused_kernel(nseg, mode, out_type, (int)vec);
        if (!fn) return COMET_ERR_INTERNAL;
        void *kargs[] = {&f};
        TimedScope ts(ws.prof, st, COMET_KERNEL_FUSED);
        HIP_TRY(hipLaunchKernel(fn, dim3(fg.grid), dim3(kFuBlock), kargs, kFuLdsBytes, st));
    }
    if (fused && out_type == 0) {
        // any other chunk size: the general kernel, on a small grid (it is rarely needed)
        ReconArgs a{};
        a.container = in; a.t = ws.tables; a.n = n; a.planes = s.n * s.c; a.H = s.h; a.W = s.w; a.divW = make_fastdiv(s.w);
        a.planes_per_unit = g.planes_per_unit; a.tile_rows = g.tile_rows; a.n_units = g.n_units; a.pitch = g.pitch; a.use_carry = g.use_carry;
        a.out = static_cast<float *>(dev_out); a.ctl = &ws.state->ctl; a.skip_chunk64 = 1u;
        uint32_t grid = g.n_units;
        const uint32_t cap = (uint32_t)ws.num_cu * 4u;
        if (grid > cap) grid = cap;
        hipLaunchKernelGGL(k_reconstruct<0>, dim3(grid), dim3(kDecBlock), g.lds, st, a);
    } else if (fast_path) {
        // Huffman decode into int16 residuals (the code buffer of the context doubles as
        // the work buffer), then scans and stores
        DsArgs d{};
        d.skip_chunk64 = fused ? 1u : 0u;
        d.container = in; d.t = ws.tables; d.n = n; d.planes = s.n * s.c; d.H = s.h; d.W = s.w; d.divW = make_fastdiv(s.w); d.divL = make_fastdiv(lpr);
        d.resid = ws.resid; d.out = dev_out; d.ctl = &ws.state->ctl;
        {
            // groups of 64 chunks, one per wavefront at a time; the same number of groups for every
            // wavefront of a grid that is resident at once (estimated with the context's chunk size)
            const uint64_t groups = (n + (uint64_t)ws.chunk_syms * kWave - 1) / ((uint64_t)ws.chunk_syms * kWave);
            const uint64_t resident = (uint64_t)ws.num_cu * 4u * kDsWaves;
            const uint64_t per_wave = (groups + resident - 1) / resident;
            const uint64_t waves = (groups + per_wave - 1) / per_wave;
            const uint32_t grid = (uint32_t)((waves + kDsWaves - 1) / kDsWaves);
            TimedScope ts(ws.prof, st, COMET_KERNEL_DECODE);
            hipLaunchKernelGGL(k_decode_chunks, dim3(grid), dim3(kDsBlock), (size_t)kDsWaves * kDsStageWords * 4u, st, d);
        }
        HIP_TRY(hipGetLastError());
        // small planes: a unit of work is a group of whole planes, `passes` times the planes that sit side by
        // side in a wavefront: about kScanStripElems elements, fewer if that leaves the chip short of wavefronts
        const uint64_t P = (uint64_t)s.h * s.w;
        uint64_t G = 1;
        if (lpr <= 32u) {
            uint64_t passes = kScanStripElems / (ppi * P);
            const uint64_t spread = (uint64_t)d.planes / ((uint64_t)ppi * ws.num_cu * 32u);
            if (passes > spread) passes = spread;
            G = ppi * (passes ? passes : 1u);
        }
        d.group_planes = (uint32_t)G;
        const uint64_t units = ((uint64_t)d.planes + G - 1) / G;
        uint64_t grid = (units + kDsWaves - 1) / kDsWaves;
        const uint64_t cap = (uint64_t)ws.num_cu * 8u;
        if (grid > cap) grid = cap;
        const size_t lds = (size_t)kDsWaves * kScanListWords * 4u;
        TimedScope ts(ws.prof, st, COMET_KERNEL_RECONSTRUCT);
        const dim3 g3((uint32_t)grid), b3(kDsBlock);
#define COMET_LAUNCH_SCAN(OUT)                                                                           \
        do {                                                                                             \
            if (vec == 2u) {                                                                             \
                if (lpr <= 16u) hipLaunchKernelGGL((k_scan_store<1, 0, OUT, 2>), g3, b3, lds, st, d);    \
                else if (lpr <= 32u) hipLaunchKernelGGL((k_scan_store<1, 1, OUT, 2>), g3, b3, lds, st, d); \
                else if (lpr <= 64u) hipLaunchKernelGGL((k_scan_store<1, 2, OUT, 2>), g3, b3, lds, st, d); \
                else if (lpr <= 128u) hipLaunchKernelGGL((k_scan_store<2, 2, OUT, 2>), g3, b3, lds, st, d); \
                else hipLaunchKernelGGL((k_scan_store<4, 2, OUT, 2>), g3, b3, lds, st, d);               \
            } else {                                                                                     \
                if (lpr <= 16u) hipLaunchKernelGGL((k_scan_store<1, 0, OUT, 1>), g3, b3, lds, st, d);    \
                else if (lpr <= 32u) hipLaunchKernelGGL((k_scan_store<1, 1, OUT, 1>), g3, b3, lds, st, d); \
                else if (lpr <= 64u) hipLaunchKernelGGL((k_scan_store<1, 2, OUT, 1>), g3, b3, lds, st, d); \
                else if (lpr <= 128u) hipLaunchKernelGGL((k_scan_store<2, 2, OUT, 1>), g3, b3, lds, st, d); \
                else if (lpr <= 256u) hipLaunchKernelGGL((k_scan_store<4, 2, OUT, 1>), g3, b3, lds, st, d); \
                else hipLaunchKernelGGL((k_scan_store<8, 2, OUT, 1>), g3, b3, lds, st, d);               \
            }                                                                                            \
        } while (0)
        if (out_type == COMET_F16) COMET_LAUNCH_SCAN(1);
        else if (out_type == COMET_BF16) COMET_LAUNCH_SCAN(2);
        else COMET_LAUNCH_SCAN(0);
#undef COMET_LAUNCH_SCAN
    } else {
        ReconArgs a{};
        a.container = in; a.t = ws.tables; a.n = n; a.planes = s.n * s.c; a.H = s.h; a.W = s.w; a.divW = make_fastdiv(s.w);
        a.planes_per_unit = g.planes_per_unit; a.tile_rows = g.tile_rows; a.n_units = g.n_units; a.pitch = g.pitch; a.use_carry = g.use_carry;
        a.out = static_cast<float *>(dev_out); a.ctl = &ws.state->ctl;
        uint32_t grid = g.n_units;
        const uint32_t cap = (uint32_t)ws.num_cu * 32u;
        if (grid > cap) grid = cap;
        TimedScope ts(ws.prof, st, COMET_KERNEL_RECONSTRUCT);
        hipLaunchKernelGGL(k_reconstruct<0>, dim3(grid), dim3(kDecBlock), g.lds, st, a);
    }
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}
}  // namespace

// ---------------------------------------------------------------------------
// decompression without a context, for callers that cannot allocate
// ---------------------------------------------------------------------------
namespace {
constexpr uint64_t kStaticMaxElems = COMET_STATIC_MAX_ELEMS;
// layout of the static scratch array: control block | decode tables | residual work buffer
constexpr size_t kSsState = 0;
constexpr size_t kSsLimit = 512;
constexpr size_t kSsFirst = kSsLimit + 8 * 72;
constexpr size_t kSsFindex = kSsFirst + 8 * 72;
constexpr size_t kSsMeta = kSsFindex + 4 * 72 + 32;          // 16-byte aligned
constexpr size_t kSsLut = kSsMeta + 64;
constexpr size_t kSsLut16 = kSsLut + 4 * kLutSize;
constexpr size_t kSsSub16 = kSsLut16 + 2 * kLut16Size;
constexpr size_t kSsSorted = kSsSub16 + 2 * kSubEntries;
constexpr size_t kSsResid = (kSsSorted + 2 * (size_t)kMaxBins + 255) / 256 * 256;
constexpr size_t kSsBytes = kSsResid + 2 * (size_t)kStaticMaxElems + 256;
static_assert(sizeof(DevState) <= kSsLimit && kSsMeta % 16 == 0 && kSsLut % 16 == 0, "scratch layout");
constexpr int kStaticMaxDevices = 64;
struct StaticDev { void *ptr; int num_cu; };
StaticDev g_static_dev[kStaticMaxDevices];       // filled once per device, under the lock
bool g_static_ready[kStaticMaxDevices];
std::mutex g_static_lock;
}  // namespace

// Device memory of comet_decompress_static: every GPU the library runs on holds its own copy until
// the process ends.  In host code this name is a stand-in, not a device address; the address comes
// from hipGetSymbolAddress (static_scratch below).
static __device__ __align__(256) unsigned char scratch[kSsBytes];

namespace {
// The current device's copy of `scratch` (looked up once per device, with that device current).
int static_scratch(StaticDev *out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return COMET_ERR_INVALID;
    std::lock_guard<std::mutex> guard(g_static_lock);
    if (!g_static_ready[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return COMET_ERR_HIP;
        int cus = 0;
        HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        // the kernel for planes wider than 512 columns needs more than 64 KB of dynamic LDS
        HIP_TRY(hipFuncSetAttribute((const void *)k_reconstruct<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
        {
            const int rc = fused_opt_in();
            if (rc) return rc;
        }
        g_static_dev[dev].ptr = ptr;
        g_static_dev[dev].num_cu = cus > 0 ? cus : 256;
        g_static_ready[dev] = true;
    }
    *out = g_static_dev[dev];
    return COMET_OK;
}
}  // namespace

int comet_decompress_static(const void *dev_in, uint64_t bytes, comet_shape s, void *stream, float *dev_out, int32_t *dev_status) {
    uint64_t n;
    if (!shape_elems(s, &n)) return COMET_ERR_INVALID;
    if (n > kStaticMaxElems) return COMET_ERR_NOMEM;         // the static work buffer holds COMET_STATIC_MAX_ELEMS residuals
    StaticDev sd{};
    const int rc = static_scratch(&sd);
    if (rc) return rc;
    uint8_t *base = static_cast<uint8_t *>(sd.ptr);
    DecompWs ws{};
    ws.state = reinterpret_cast<DevState *>(base + kSsState);
    ws.tables.limit = reinterpret_cast<uint64_t *>(base + kSsLimit);
    ws.tables.first_code = reinterpret_cast<uint64_t *>(base + kSsFirst);
    ws.tables.first_index = reinterpret_cast<uint32_t *>(base + kSsFindex);
    ws.tables.meta = reinterpret_cast<uint32_t *>(base + kSsMeta);
    ws.tables.lut = reinterpret_cast<uint32_t *>(base + kSsLut);
    ws.tables.lut16 = reinterpret_cast<uint16_t *>(base + kSsLut16);
    ws.tables.sub16 = reinterpret_cast<uint16_t *>(base + kSsSub16);
    ws.tables.sorted = reinterpret_cast<uint16_t *>(base + kSsSorted);
    ws.resid = reinterpret_cast<int16_t *>(base + kSsResid);
    ws.max_elems = kStaticMaxElems; ws.num_cu = sd.num_cu; ws.chunk_syms = COMET_DEFAULT_CHUNK_SYMS;
    ws.prof = nullptr; ws.dev_status = dev_status;
    // Nothing in the array has to start at zero: the tables kernel clears the control block and stores
    // the status, every table entry and residual that is read has been written by this call.
    return decompress_impl(ws, dev_in, bytes, s, stream, dev_out, 0);
}

int comet_sync(comet_ctx *ctx, void *stream) {
    if (!ctx) return COMET_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(ctx->host_state, ctx->state, sizeof(DevState), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    const uint32_t latched = ctx->host_state->latched;
    if (latched) {
        HIP_TRY(hipMemsetAsync(&ctx->state->latched, 0, 4, st));
        HIP_TRY(hipStreamSynchronize(st));
    }
    return status_to_error(latched);
}

int comet_peek(comet_ctx *ctx, const void *dev_in, uint64_t bytes, void *stream, comet_info *info) {
    if (!ctx || !dev_in || !info) return COMET_ERR_INVALID;
    if (bytes < kHeaderBytes) return COMET_ERR_FORMAT;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(ctx->host_hdr, dev_in, sizeof(Header), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    const Header &h = *ctx->host_hdr;
    comet_shape s{h.N, h.C, h.H, h.W};
    uint64_t n;
    if (h.magic != kMagic || (h.version != 1 && h.version != 2) || h.status != 0 || !shape_elems(s, &n) || !valid_nbins(h.nbins) ||
        h.chunk_syms == 0 || h.total_bytes > bytes || h.total_bytes != h.off_payload + 4 * h.payload_words) return COMET_ERR_FORMAT;
    info->shape = s; info->nbins = h.nbins; info->chunk_syms = h.chunk_syms; info->n_chunks = h.n_chunks;
    info->n_active = h.n_active; info->max_len = h.max_len; info->n_outlier_records = h.n_rec; info->n_value_records = h.n_vrec;
    memcpy(&info->eb, &h.eb_bits, 4);
    info->nnz = h.nnz; info->payload_words = h.payload_words; info->total_bytes = h.total_bytes;
    return COMET_OK;
}

void comet_adapt_defaults(comet_adapt_cfg *cfg) {
    if (!cfg) return;
    cfg->a = 0.32; cfg->sigma_frac = 0.01; cfg->eb_min = 0x1p-100f; cfg->eb_max = 0x1p100f;
}

int comet_adapt_eb(const comet_layer_stats *s, const comet_adapt_cfg *cfg_in, float *eb_out) {
    if (!s || !eb_out) return COMET_ERR_INVALID;
    comet_adapt_cfg cfg;
    if (cfg_in) cfg = *cfg_in; else comet_adapt_defaults(&cfg);
    if (!std::isfinite(s->momentum_abs_mean) || !std::isfinite(s->loss_grad_mean) || !std::isfinite(s->nonzero_ratio) ||
        !std::isfinite(cfg.a) || !std::isfinite(cfg.sigma_frac)) return COMET_ERR_INVALID;
    if (s->momentum_abs_mean < 0.0 || s->loss_grad_mean < 0.0 || s->nonzero_ratio < 0.0 || s->nonzero_ratio > 1.0 ||
        s->batch == 0 || !(cfg.a > 0.0) || !(cfg.sigma_frac > 0.0) || !(cfg.eb_min > 0.0f) || !(cfg.eb_max >= cfg.eb_min)) return COMET_ERR_INVALID;
    if (s->loss_grad_mean == 0.0 || s->nonzero_ratio == 0.0) { *eb_out = cfg.eb_max; return COMET_OK; }
    const double sigma = cfg.sigma_frac * s->momentum_abs_mean;                                 // Sec. 3.2
    const double eb = sigma / (cfg.a * s->loss_grad_mean * std::sqrt((double)s->batch * s->nonzero_ratio));   // Sec. 3.3
    float e = (float)eb;
    if (!(e >= cfg.eb_min)) e = cfg.eb_min;
    if (e > cfg.eb_max) e = cfg.eb_max;
    *eb_out = e;
    return COMET_OK;
}

// ---------------------------------------------------------------------------
// controller glue (Sec. 3.1)
// ---------------------------------------------------------------------------

int comet_abs_mean(comet_ctx *ctx, const float *dev_in, uint64_t n, void *stream, double *mean_out) {
    if (!ctx || !dev_in || !mean_out || n == 0) return COMET_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    // a slice of at least 16384 values per workgroup, a few workgroups per CU at most
    uint64_t grid = (n + 16383u) / 16384u;
    const uint64_t cap = (uint64_t)ctx->num_cu * 8u < kStatsPartialMax ? (uint64_t)ctx->num_cu * 8u : kStatsPartialMax;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL(k_abs_sum, dim3((uint32_t)grid), dim3(kStatsBlock), 0, st, dev_in, n, ctx->stats);
    hipLaunchKernelGGL(k_abs_mean_final, dim3(1), dim3(kWave), 0, st, ctx->stats, (uint32_t)grid, n, ctx->stats + kStatsPartialMax);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpyAsync(mean_out, ctx->stats + kStatsPartialMax, 8, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return COMET_OK;
}

int comet_controller_init(comet_controller *c, uint32_t w_default) {
    if (!c) return COMET_ERR_INVALID;
    c->w_default = w_default ? w_default : 1000u;
    c->w = c->w_default;
    c->since = 0;
    return COMET_OK;
}

int comet_controller_tick(comet_controller *c, int *collect) {
    if (!c || !collect || c->w == 0) return COMET_ERR_INVALID;
    *collect = 0;
    if (++c->since >= c->w) { c->since = 0; *collect = 1; }
    return COMET_OK;
}

int comet_controller_update(comet_controller *c, const float *eb_old, const float *eb_new, uint32_t n_layers) {
    if (!c || !eb_old || !eb_new || n_layers == 0 || c->w == 0) return COMET_ERR_INVALID;
    bool moved = false;                                   // some layer's bound changed by more than 2x, up or down
    for (uint32_t l = 0; l < n_layers; ++l) {
        const double a = (double)eb_old[l], b = (double)eb_new[l];
        if (!(a > 0.0) || !(b > 0.0) || !std::isfinite(a) || !std::isfinite(b)) return COMET_ERR_INVALID;
        if (a > 2.0 * b || b > 2.0 * a) moved = true;
    }
    if (moved) c->w = c->w > 1u ? c->w / 2u : 1u;
    else c->w = c->w_default;
    return COMET_OK;
}

// ---------------------------------------------------------------------------
// stage-level entry points
// ---------------------------------------------------------------------------

int comet_stage_quantize(comet_ctx *ctx, const float *dev_in, comet_shape s, float eb, uint32_t nbins, void *stream,
                         uint16_t *dev_codes, uint32_t *dev_hist, uint32_t *dev_records, uint64_t rec_capacity,
                         uint64_t *dev_counts) {
    uint64_t n;
    if (!ctx || !dev_in || !dev_codes || !dev_hist || !dev_counts || (rec_capacity && !dev_records) ||
        !shape_elems(s, &n) || !valid_eb(eb) || !valid_nbins(nbins) || s.w > kMaxW || ((uintptr_t)dev_in & 15u) ||
        ((uintptr_t)dev_codes & 7u) || ((uintptr_t)dev_records & 7u)) return COMET_ERR_INVALID;
    if (n > ctx->max_elems) return COMET_ERR_NOMEM;
    hipStream_t st = (hipStream_t)stream;
    const uint64_t tiles_q = quantize_geometry(ctx, s, n, dev_in, nbins).grid;
    const ZeroLayout z = zero_layout(0, nbins, tiles_q, 1);
    if (z.bytes > ctx->zero_cap) return COMET_ERR_NOMEM;
    HIP_TRY(hipMemsetAsync(ctx->zero_region, 0, z.bytes, st));
    HIP_TRY(hipMemsetAsync(dev_hist, 0, 4ull * nbins, st));
    uint64_t *desc_q = reinterpret_cast<uint64_t *>(ctx->zero_region + z.off_desc_q);
    uint32_t *hist_parts = reinterpret_cast<uint32_t *>(ctx->zero_region + z.off_parts);
    int rc = launch_quantize(ctx, dev_in, s, n, eb, nbins, st, dev_codes, dev_hist, hist_parts, dev_records, rec_capacity, desc_q);
    if (rc) return rc;
    HIP_TRY(hipMemcpyAsync(dev_counts, &ctx->state->ctl.n_rec, 24, hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(k_latch, dim3(1), dim3(1), 0, st, ctx->state);
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

int comet_stage_codebook(comet_ctx *ctx, const uint32_t *dev_hist, uint32_t nbins, void *stream, uint8_t *dev_len, uint64_t *dev_code) {
    if (!ctx || !dev_hist || !dev_len || nbins == 0 || nbins > kMaxBins) return COMET_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemsetAsync(ctx->zero_region, 0, sizeof(Control), st));
    BookArgs b{};
    b.hist = dev_hist; b.nbins = nbins; b.len_out = dev_len; b.code_out = dev_code; b.enc = ctx->enc;
    b.scratch = ctx->book; b.ctl = &ctx->state->ctl; b.hdr = nullptr; b.capacity = 0;
    const int rc = launch_codebook(ctx, b, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_latch, dim3(1), dim3(1), 0, st, ctx->state);
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

int comet_stage_encode(comet_ctx *ctx, const uint16_t *dev_codes, uint64_t n, uint32_t nbins, uint32_t chunk_syms, void *stream,
                       uint32_t *dev_chunk_off, uint32_t *dev_payload, uint64_t payload_capacity_words, uint64_t *dev_payload_words) {
    if (!ctx || !dev_codes || !dev_chunk_off || !dev_payload_words || (payload_capacity_words && !dev_payload) ||
        n == 0 || n > kMaxElems || nbins == 0 || nbins > kMaxBins || !valid_chunk(chunk_syms) || ((uintptr_t)dev_codes & 15u)) return COMET_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    const uint64_t n_chunks = (n + chunk_syms - 1) / chunk_syms;
    uint32_t e_seg, e_grid;
    encode_geometry(ctx, n_chunks, &e_seg, &e_grid);
    const uint64_t tiles_e = e_grid;
    const ZeroLayout z = zero_layout(0, 0, 1, tiles_e);
    if (z.bytes > ctx->zero_cap) return COMET_ERR_NOMEM;
    HIP_TRY(hipMemsetAsync(ctx->zero_region, 0, z.bytes, st));
    uint64_t *desc_e = reinterpret_cast<uint64_t *>(ctx->zero_region + z.off_desc_e);
    int rc = launch_encode(ctx, dev_codes, n, nbins, chunk_syms, st, dev_chunk_off, nullptr, 0, dev_payload, payload_capacity_words,
                           dev_payload_words, desc_e);
    if (rc) return rc;
    hipLaunchKernelGGL(k_latch, dim3(1), dim3(1), 0, st, ctx->state);
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

int comet_stage_decode(comet_ctx *ctx, const uint8_t *dev_len, uint32_t nbins, const uint32_t *dev_chunk_off, const uint32_t *dev_payload,
                       uint64_t payload_words, uint64_t n, uint32_t chunk_syms, void *stream, uint16_t *dev_codes_out) {
    if (!ctx || !dev_len || !dev_chunk_off || !dev_codes_out || (payload_words && !dev_payload) || n == 0 || n > kMaxElems ||
        nbins == 0 || nbins > kMaxBins || chunk_syms == 0) return COMET_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemsetAsync(ctx->zero_region, 0, sizeof(Control), st));
    TablesArgs t{};
    t.len = dev_len; t.nbins = nbins; t.t = ctx->tables; t.ctl = &ctx->state->ctl; t.hdr = nullptr;
    hipLaunchKernelGGL(k_decode_tables, dim3(1), dim3(kBookBlock), 0, st, t);
    HIP_TRY(hipGetLastError());
    ReconArgs a{};
    a.chunk_off = dev_chunk_off; a.payload = dev_payload; a.payload_words = payload_words; a.chunk_syms = chunk_syms;
    a.n_chunks = (uint32_t)((n + chunk_syms - 1) / chunk_syms); a.t = ctx->tables; a.n = n; a.codes_out = dev_codes_out; a.ctl = &ctx->state->ctl;
    a.zero_chunks = ctx->zero_chunks;
    uint32_t grid = (a.n_chunks + kDecBlock - 1) / kDecBlock;
    const uint32_t cap = (uint32_t)ctx->num_cu * 32u;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL(k_decode_only, dim3(grid), dim3(kDecBlock), 0, st, a);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(k_latch, dim3(1), dim3(1), 0, st, ctx->state);
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

int comet_stage_reconstruct(comet_ctx *ctx, const uint16_t *dev_codes, const uint32_t *dev_records, uint64_t n_records, comet_shape s,
                            uint32_t nbins, float eb, void *stream, float *dev_out) {
    uint64_t n;
    if (!ctx || !dev_codes || !dev_out || (n_records && !dev_records) || !shape_elems(s, &n) || !valid_nbins(nbins) || !valid_eb(eb) ||
        s.w > kMaxW) return COMET_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    ReconGeometry g;
    if (!recon_geometry(s, &g)) return COMET_ERR_INVALID;
    ReconArgs a{};
    a.codes_in = dev_codes; a.rec = dev_records; a.n_rec = n_records; a.n = n; a.planes = s.n * s.c; a.H = s.h; a.W = s.w;
    a.divW = make_fastdiv(s.w); a.radius = (int32_t)(nbins / 2u); a.eb = eb; a.ebx2 = 2.0f * eb;
    a.planes_per_unit = g.planes_per_unit; a.tile_rows = g.tile_rows; a.n_units = g.n_units; a.pitch = g.pitch; a.use_carry = g.use_carry;
    a.out = dev_out; a.ctl = &ctx->state->ctl; a.chunk_syms = 1;
    uint32_t grid = g.n_units;
    const uint32_t cap = (uint32_t)ctx->num_cu * 32u;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL(k_reconstruct<1>, dim3(grid), dim3(kDecBlock), g.lds, st, a);
    HIP_TRY(hipGetLastError());
    return COMET_OK;
}

int comet_profile_enable(comet_ctx *ctx, int enable) {
    if (!ctx) return COMET_ERR_INVALID;
    if (enable && ctx->pool.empty()) {
        ctx->pool.reserve(16384);
        for (int i = 0; i < 16384; ++i) {
            comet_ctx::Timed t{};
            HIP_TRY(hipEventCreate(&t.a));
            HIP_TRY(hipEventCreate(&t.b));
            ctx->pool.push_back(t);
        }
    }
    ctx->profiling = enable != 0;
    return COMET_OK;
}

int comet_profile_reset(comet_ctx *ctx) {
    if (!ctx) return COMET_ERR_INVALID;
    ctx->used = 0;
    return COMET_OK;
}

int comet_profile_read(comet_ctx *ctx, uint32_t kernel_id, uint32_t *launches, double *total_ms) {
    if (!ctx || !launches || !total_ms || kernel_id >= COMET_KERNEL_COUNT) return COMET_ERR_INVALID;
    uint32_t cnt = 0;
    double sum = 0.0;
    for (size_t i = 0; i < ctx->used; ++i) {
        const comet_ctx::Timed &t = ctx->pool[i];
        if (t.id != kernel_id) continue;
        HIP_TRY(hipEventSynchronize(t.b));
        float ms = 0.0f;
        HIP_TRY(hipEventElapsedTime(&ms, t.a, t.b));
        sum += ms;
        ++cnt;
    }
    *launches = cnt;
    *total_ms = sum;
    return COMET_OK;
}

const char *comet_strerror(int code) {
    switch (code) {
        case COMET_OK: return "ok";
        case COMET_ERR_INVALID: return "invalid argument";
        case COMET_ERR_CAPACITY: return "container does not fit the output buffer";
        case COMET_ERR_FORMAT: return "malformed container or shape mismatch";
        case COMET_ERR_HIP: return g_hip_msg;
        case COMET_ERR_NOMEM: return "out of memory, or request larger than the context was created for";
        case COMET_ERR_INTERNAL: return "device-side consistency check failed";
        case COMET_ERR_CODEBOOK: return "the given code lengths are no complete prefix code, or lack a code word for an escape the tensor needs";
        default: return "unknown error code";
    }
}

}  // extern "C"
