// Kernel argument blocks and launch constants shared by the host API and the
// kernel translation units.
#pragma once
#include "comet_dev.h"

namespace comet {

// ---- quantise (prequantise + Lorenzo + codes + histogram + records) ----------
constexpr int kQuantBlock = 256;
constexpr int kQuantTile = 4096;           // elements per tile: 256 lanes x 4 iterations x float4
constexpr uint32_t kHistWindowMax = 8192;  // LDS-private histogram bins per workgroup

struct QuantArgs {
    const void *x;             // fp32; the row-walking kernels also take IEEE half or bfloat16 (template parameter IN)
    uint64_t n;
    FastDiv divW, divH;        // plane width / height
    float r, ebx2, eb;
    int32_t radius;
    uint32_t nbins;
    uint32_t win_lo, win_n;    // histogram bins [win_lo, win_lo + win_n) are counted in LDS
    uint32_t n_tiles;
    uint32_t tiles_per_seg;    // consecutive tiles per workgroup (one segment each)
    uint32_t rec_lds;          // records the LDS buffer of a workgroup can hold
    uint32_t rows_total;       // row-walking kernel: planes * H rows of W elements
    uint32_t rows_per_wave;    //   consecutive rows per wavefront (a multiple of rows_per_step)
    uint32_t rows_per_step;    //   rows a wavefront covers per step (64 / lanes per row if a row takes at most 32 lanes, else 1)
    uint32_t hist_shift;       //   log2 of the copies of the LDS histogram window (lane & (copies - 1) picks one)
    uint32_t *stage;           //   staging area: kQuantRecRun (key, payload) pairs per run
    uint32_t *run_count;       //   three arrays of one entry per run: records, non-zero inputs, verbatim records
    const uint8_t *reuse_len;  //   code book reuse (REUSE kernels): u8[nbins] code lengths; a code of length 0 becomes an escape; no histogram
    uint32_t *hist_parts;      //   hist_copies partial histograms of nbins entries, zeroed: workgroup b adds to copy b % hist_copies
    uint32_t hist_copies;      //   (k_gather_records adds them up into hist)
    // single-pass compression (REUSE kernels): the codes are encoded by the wavefront that makes them
    const uint64_t *enc;       //   encode table of the given lengths: (code << 6) | length per symbol
    uint32_t enc_lo, enc_n;    //   table entries [enc_lo, enc_lo + enc_n) are cached in LDS
    uint32_t chunk_syms;       //   64, 128 or 256; a run is a whole number of chunks
    uint32_t zero_pair;        //   container version 2: (centre << 16) | centre, else 0
    uint32_t *chunk_off;       //   chunk table of the container: offsets relative to the run (k_place_payload makes them absolute)
    uint32_t *run_words;       //   words of every run
    uint32_t *work_words;      //   work area: the words of the run that starts at element e at word e / 2
    uint16_t *codes;
    uint32_t *hist;            // u32[nbins], zeroed
    uint32_t *rec;             // (key, payload) pairs
    uint64_t rec_cap;          // capacity in records
    uint64_t *desc;            // chained-scan descriptors, one per segment, zeroed
    Control *ctl;
};
constexpr uint32_t kEncRingSyms = 1024;    // single-pass compression: codes a wavefront keeps in LDS between quantisation and encoding (a batch of at most 512, and less than 256 not yet encoded)
constexpr uint32_t kEncRunBufWords = 476;  //   its assembly buffer: the words of one step of 256 symbols (at most 456 of code words of 57 bits, two more touched) and slack
constexpr uint32_t kQuantRecLds = 3072;   // outlier records buffered in LDS per workgroup (24 KB)
template <bool FULLWIN> __global__ void k_quantize(QuantArgs a);   // flat tiles, any plane width; FULLWIN: every bin is in the LDS window
constexpr uint32_t kQuantRowsMaxW = 512;  // widest plane of the row-walking kernel
constexpr uint32_t kQuantRecRun = 768;    // outlier records staged per run (one run of rows per wavefront)
constexpr uint32_t kQuantRecLds2 = 256;   // records a wavefront buffers in LDS before it writes them to the staging area in bulk
constexpr uint32_t kQuantRunsPerSimd = 5; // runs the launch aims at, per SIMD
constexpr uint32_t kQuantOowList = 512;   // codes outside the LDS histogram window a wavefront lists before it adds them to the global histogram
constexpr uint32_t kQuantStaticLds = 8448; // static LDS of k_quantize_rows (the record buffers of its four wavefronts and a few words), rounded up
constexpr uint32_t kLdsPerCu = 160u * 1024u;
constexpr uint32_t kQuantRunsPerSimdSingle = 4;   //   ... of the single-pass compression (all of them resident at once)
constexpr uint32_t kQuantHistCopiesMax = 32;        // partial histograms the workgroups spread their flushes over
constexpr uint32_t kQuantHistPartsWords = 8u * 65536u;    // all copies together have at most this many entries (2 MB: eight copies of the largest alphabet)
// VEC adjacent columns per lane (2 needs an even W and 8-byte aligned input), NSEG segments of 64 lanes per row,
// MULTI: several rows per step
// REUSE: code book reuse: escapes follow the given length table, no histogram (FULLWIN is then true and unused)
// IN: element type of x (0 fp32, 1 IEEE half, 2 bfloat16; 16-bit inputs are widened exactly as they are loaded;
// VEC = 2 then needs 4-byte aligned input)
template <int VEC, int NSEG, bool MULTI, bool FULLWIN, bool REUSE = false, int IN = 0> __global__ void k_quantize_rows(QuantArgs a);
template <int VEC, int NSEG, bool MULTI, bool REUSE = false, int IN = 0> __global__ void k_gather_records(QuantArgs a);
constexpr uint32_t kQuantReuseMaxBins = 8192;   // largest alphabet whose length table the REUSE kernels keep in LDS

// ---- statistics ---------------------------------------------------------------
constexpr int kStatsBlock = 256;
constexpr uint32_t kStatsPartialMax = 4096;     // workgroups of k_abs_sum at most (one partial sum each)
__global__ void k_abs_sum(const float *x, uint64_t n, double *partial);
__global__ void k_abs_mean_final(const double *partial, uint32_t n_partial, uint64_t n, double *mean_out);

// ---- codebook -----------------------------------------------------------------
constexpr int kBookBlock = 1024;
constexpr uint32_t kBookLdsSyms = 2048;    // alphabets up to this size are built entirely in LDS
constexpr uint32_t kBookBySymbolMax = 8192; // nbins up to which the code lengths also fit LDS by symbol (one byte each)

struct BookScratch {                        // global scratch for large alphabets (>= 65536 entries each)
    uint64_t *keys;        // sort keys
    uint64_t *iw;          // internal-node weights
    uint32_t *leaf_parent;
    uint32_t *int_parent;
};

struct BookArgs {
    const uint32_t *hist;
    const uint8_t *given_len;  // code book reuse: take these lengths instead of building them from hist (which is then unused)
    uint32_t nbins;
    uint8_t *len_out;          // u8[nbins]
    uint64_t *code_out;        // u64[nbins] or null (stage output)
    uint64_t *enc;             // u64[nbins]: (code << 6) | len, 0 for unused symbols
    BookScratch scratch;
    uint32_t presorted;        // scratch.keys holds the leaves in (frequency, symbol) order (k_book_sort_tiles, k_book_merge) if more than kBookLdsSyms symbols occur
    Control *ctl;
    // container finalisation (null header = stage call)
    Header *hdr;
    Header proto;              // host-filled fields
    uint64_t capacity;
};
__global__ void k_codebook(BookArgs a);
constexpr int kBookMergeBlock = 256;
__global__ void k_book_sort_tiles(const uint32_t *hist, uint32_t nbins, uint64_t *keys, Control *ctl);
__global__ void k_book_merge(const uint64_t *src, uint64_t *dst, uint32_t run, const Control *ctl);

// ---- encode -------------------------------------------------------------------
constexpr int kEncBlock = 256;             // four wavefronts, each encodes 256 symbols per step cooperatively
constexpr uint32_t kEncTableMax = 2048;    // table entries cached in LDS
// Code lengths (one byte each) the count kernel caches in LDS instead of part of the encode table, if every symbol that
// occurs lies among them: 16384 around the centre (the room of the table's cached part), 32768 for the largest alphabets
// (whose symbols spread wider; twice the LDS, which costs the smaller ones more than it gains them).
__host__ __device__ inline uint32_t enc_len_window(uint32_t nbins) { return nbins <= 16384u ? nbins : (nbins <= 32768u ? 16384u : 32768u); }
constexpr uint32_t kEncSegChunksMax = 4096;   // chunks per workgroup segment (their word counts live in LDS)

struct EncodeArgs {
    const uint16_t *codes;
    uint64_t n;
    uint32_t chunk_syms;       // 64, 128 or 256
    uint32_t n_chunks;
    uint32_t seg_chunks;       // chunks per segment (one segment per workgroup)
    const uint64_t *enc;
    const uint8_t *len8;       // device u8[nbins]: the code lengths alone (the container's length section), or null
    uint32_t nbins;
    uint32_t tbl_lo, tbl_n;    // table entries [tbl_lo, tbl_lo + tbl_n) are cached in LDS
    uint32_t tbl_room;         // count kernel: bytes of LDS in front of the word counts (the table, or the lengths of a large alphabet)
    uint32_t *chunk_off;
    uint8_t *container;        // product path: payload position comes from ctl->off_payload
    uint64_t capacity;
    uint32_t *payload;         // stage path: explicit payload buffer
    uint64_t payload_cap_words;
    uint64_t *payload_words_out;   // stage path
    uint64_t *desc;            // words of every segment (written by the count kernel, read by the pack kernel)
    Control *ctl;
    uint32_t *latched;         // product path: the context's persistent status word (the pack kernel seals the header); else null
    uint32_t zero_pair;        // container version 2: (centre << 16) | centre, a chunk of nothing but centre codes takes no words; else 0
};
// single-pass compression: the words of every run from the work area to the payload
struct PlaceArgs {
    const uint32_t *run_words;     // words of every run
    uint32_t n_runs;               // runs that hold rows (the arrays have an entry for every wavefront of the grid)
    uint32_t rows_per_wave, rows_total, W;
    uint32_t chunk_syms;
    const uint32_t *work_words;    // the run that starts at element e has its words from word e / 2 on
    uint8_t *container;
    uint64_t capacity;
    Control *ctl;
    uint32_t *latched;             // the context's persistent status word
};
constexpr int kPlaceBlock = 256;
__global__ void k_place_payload(PlaceArgs a);

constexpr uint32_t kEncUnroll = 4;         // steps of 256 symbols a wavefront handles per iteration
constexpr uint32_t kEncStepWordsMax = 468; // 256 code words of up to 58 bits, in 32-bit words, plus slack
constexpr uint32_t kEncBufWords = 640;     // assembly buffer of a wavefront (ordinary code books fill a fraction of it)
// S: symbols per chunk (64, 128, 256); FULLTBL: the whole encode table is in LDS
template <int S, bool FULLTBL> __global__ void k_encode_count(EncodeArgs a);
template <int S, bool FULLTBL> __global__ void k_encode_pack(EncodeArgs a);

// ---- decode tables ------------------------------------------------------------
constexpr int kLutBits = 11;
constexpr uint32_t kLutSize = 1u << kLutBits;
// Alphabets of at most kLut16MaxBins bins (residuals fit 12 signed bits) also get a compact table on
// the next 12 bits: same 8 KB of LDS, half as many codes too long for it.
constexpr int kLut16Bits = 12;
constexpr uint32_t kLut16Size = 1u << kLut16Bits;
constexpr uint32_t kLut16MaxBins = 4096;
constexpr int32_t kLut16Escape = -2048;    // residual value that stands for the escape symbol in the compact table
constexpr uint32_t kSubEntries = 2048;     // second level of the compact table: entries of all sub-tables together

struct DecodeTables {          // all in the workspace (global memory)
    uint32_t *lut;             // kLutSize entries: (residual << 8) | length with residual = symbol - radius
                               // (-32768 for the escape symbol 0); length 0 = code longer than kLutBits, the
                               // residual field then holds the shortest length a code with this prefix can have
    uint64_t *limit;           // [65]: left-aligned exclusive upper bound of the codes of each length
    uint64_t *first_code;      // [65]
    uint32_t *first_index;     // [65]: position of the first symbol of each length in `sorted`
    uint16_t *lut16;           // (if the alphabet is too large for the compact table: a copy of `lut`, so that the chunk decoders
                               // always load from here; meta[4] tells which it is)
                               // kLut16Size entries: (residual << 4) | length, residual in 12 signed bits (kLut16Escape for
                               // the escape symbol); length 0 = longer code: the upper 12 bits are (offset / 2) << 2 | width
                               // code of the prefix's sub-table in sub16 (width 1, 2, 4, 6 bits), all zero if it has none
    uint16_t *sub16;           // kSubEntries entries: (residual << 4) | (length - kLut16Bits), 0 = longer still
    uint16_t *sorted;          // symbols in canonical (length, symbol) order
    uint32_t *meta;            // [0] max_len, [1] n_active, [2] min_len, [3] radius, [4] 1 if lut16 is valid
};

struct TablesArgs {
    const uint8_t *len;        // u8[nbins]
    uint32_t nbins;
    DecodeTables t;
    uint32_t compact_only;     // 1: the caller decodes with kernels that use the compact table whenever it
                               //    exists, so the general table need not be filled in that case
    uint32_t general_unless_chunk64;   // 1: ... except for a container whose chunks are not 64 symbols (its kernel reads the general table)
    Control *ctl;
    uint32_t reset_ctl;        // 1: this kernel is the first of its call and clears *ctl itself (no separate fill before it)
    uint32_t *latched;         // if set, a status bit raised here also goes into this persistent word (no separate kernel after the call)
    int32_t *status_out;       // if set: receives 0, or -3 (the library's code for a malformed container) if the header or the table is refused
    // container validation (null = stage call)
    const Header *hdr;
    Header expect;             // shape the caller passed
    uint64_t bytes;
};
__global__ void k_decode_tables(TablesArgs a);

// ---- decode + reconstruct -----------------------------------------------------
constexpr int kDecBlock = 64;
constexpr uint32_t kDecTileElems = 8192;   // elements per strip held in LDS

struct ReconArgs {
    // source: a container (product) or explicit arrays (stage calls)
    const uint8_t *container;
    const uint16_t *codes_in;      // stage reconstruct: codes come from memory
    const uint32_t *chunk_off;
    const uint32_t *payload;
    uint64_t payload_words;
    const uint32_t *rec;
    uint64_t n_rec;
    uint32_t chunk_syms, log2_chunk, n_chunks;
    DecodeTables t;
    uint64_t n;
    uint32_t planes, H, W;
    FastDiv divW;
    int32_t radius;
    float eb, ebx2;
    // strip geometry
    uint32_t planes_per_unit;      // >= 1 when a unit is a group of whole planes
    uint32_t rows_per_strip;       // rows of one strip when a plane is cut into strips
    uint32_t n_units;
    uint32_t pitch;                // LDS row pitch (odd)
    uint32_t tile_rows;            // rows held in LDS
    uint32_t use_carry;            // 1 if planes are cut into strips (column carry in LDS)
    float *out;
    uint32_t skip_chunk64;         // 1: do nothing for a container with chunks of 64 symbols (k_decode_scan has handled it)
    uint16_t *codes_out;           // stage decode: write codes instead of reconstructing
    uint32_t zero_chunks;          // stage decode: a chunk without words is the centre code throughout (a container says so in its version)
    Control *ctl;
};
template <int MODE> __global__ void k_reconstruct(ReconArgs a);   // 0 container, 1 codes from memory
__global__ void k_decode_only(ReconArgs a);

// ---- decode + reconstruct, fast path (planes up to 512 columns): two kernels ------
constexpr int kDsWaves = 4;                           // wavefronts per workgroup, each working on its own
constexpr int kDsBlock = kDsWaves * kWave;
constexpr uint32_t kDsStageWords = 1536u;             // decode: Huffman words of 64 chunks per wavefront (LDS)
constexpr uint32_t kDsStageBatch = 8u;                // decode: loads in flight per lane while those words are fetched
constexpr uint32_t kDsMaxW = 512u;
constexpr uint32_t kDsTailEntries = 1024u;            // decode: residuals of long codes kept in LDS
constexpr uint32_t kScanListWords = 1024u;            // scan: escape list of a strip per wavefront (pairs) (LDS)
constexpr uint32_t kScanStripElems = 4096u;           // scan: elements per strip (unit of the escape list)

struct DsArgs {
    const uint8_t *container;
    DecodeTables t;
    uint64_t n;
    uint32_t planes, H, W;
    uint32_t group_planes;     // scan kernel, planes of at most 32 columns: whole planes per unit of work (a multiple of the planes side by side in a wavefront)
    FastDiv divW;
    FastDiv divL;              // scan kernel: lanes per row (W / columns per lane)
    uint32_t skip_chunk64;     // 1: do nothing for a container with chunks of 64 symbols (k_decode_scan has handled it)
    int16_t *resid;            // work buffer: one int16 residual per element (-32768 = escaped)
    void *out;                 // fp32, or IEEE half / bfloat16 (template parameter OUT of the scan kernel)
    Control *ctl;
};
__global__ void k_decode_chunks(DsArgs a);
// NSEG = ceil(lanes per row / 64) rounded up to 1, 2, 4, 8; OUT: element type of the output (0 fp32, 1 IEEE half, 2 bfloat16:
// the fp32 result rounded to nearest even)
// VEC: adjacent columns per lane (2: even W, output aligned to two elements); the lane mapping follows W / VEC
template <int NSEG, int MODE, int OUT = 0, int VEC = 1> __global__ void k_scan_store(DsArgs a);

// ---- decode + reconstruct in one kernel (planes up to 512 columns, chunks of 64 symbols) ----------
constexpr int kFuWaves = 16;                          // wavefronts per workgroup, each working on its own; one workgroup per CU
constexpr int kFuBlock = kFuWaves * kWave;
constexpr uint32_t kFuStripWords = 64u * 32u;         // a strip's residuals, element after element (64 chunks of 64 int16); before that, the words of its chunks
constexpr uint32_t kFuEscEntries = 32u;               // values of a strip's escaped residuals kept in LDS
constexpr uint32_t kFuRegionWords = kFuStripWords + kFuEscEntries;
constexpr uint32_t kFuPrefetch = 20u;                 // words per lane (of a strip's chunks) loaded while the strip before is scanned
constexpr uint32_t kFuCarryW = 128u;                  // widest plane whose strips are dealt to all wavefronts of a workgroup (column sums handed on through LDS), one column per lane; twice that with two

struct FuArgs {
    const uint8_t *container;
    DecodeTables t;
    uint64_t n;
    uint32_t planes, H, W;
    uint32_t G;                // whole planes per unit of work (one wavefront walks a unit)
    uint32_t n_units;
    FastDiv divW, divH;
    FastDiv divL;              // lanes per row (W / columns per lane)
    FastDiv divSpr;            // rows of at most 16 lanes: rows side by side in 16 lanes
    FastDiv divK;              // rows per step
    void *out;                 // fp32, or IEEE half / bfloat16 (template parameter OUT)
    Control *ctl;
};
// NSEG, MODE, OUT, VEC as for k_scan_store; MODE 0 / 1 walk several consecutive rows per step
template <int NSEG, int MODE, int OUT = 0, int VEC = 1> __global__ void k_decode_scan(FuArgs a);

}  // namespace comet
