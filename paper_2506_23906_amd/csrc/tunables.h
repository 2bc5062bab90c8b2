// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// Build-time tunables, constants of the tile layout and of the workspace, and the parameter block of the
// single-pass kernel.
#pragma once

namespace {

// Tunables (the defaults are the measured best on MI355X; -D overrides are for experiments).
#ifndef MMV_WAVES
#define MMV_WAVES 8      // waves per workgroup (int8)
#endif
#ifndef MMV_WAVES_F16
#define MMV_WAVES_F16 8
#endif
#ifndef MMV_WAVES_F32
#define MMV_WAVES_F32 8
#endif
#ifndef MMV_WAVES_SPMV
#define MMV_WAVES_SPMV 8
#endif
#ifndef MMV_CPW_I8
#define MMV_CPW_I8 4     // most chunks per wave, int8 inputs (6 spills registers)
#endif
#ifndef MMV_CPW_X8_MFMA
#define MMV_CPW_X8_MFMA 2   // ... bytes under exclusive or on the matrix cores (4 spills registers)
#endif
#ifndef MMV_CPW_F16
#define MMV_CPW_F16 2    // most chunks per wave, 16-bit inputs (4 spills registers)
#endif
#ifndef MMV_CPW_F32
#define MMV_CPW_F32 1    // most chunks per wave, fp32 inputs (2 spills registers)
#endif
// The scan without a flag vector (mmv_scan): every tile waits for the carry of the tiles before, so longer tiles
// pay.  n = 2^28, % of peak: 16-bit inputs 3 chunks 70.8, 2 chunks 67 (4 spill); fp32 2 chunks 70.5 (shuffle 73.6)
// although 24 bytes per lane spill, 1 chunk 60.6 (62.1); bytes: 5 or 6 chunks 66.7 against 74.5 with 4.
// With flags the longer tiles lose (16-bit 78.5 -> 72 %; fp32 72 -> 62 %, 88 bytes spilled).
#ifndef MMV_CPW_F16_SCAN
#define MMV_CPW_F16_SCAN 3
#endif
#ifndef MMV_CPW_F32_SCAN
#define MMV_CPW_F32_SCAN 2
#endif
// Segmented sum of fp32 values without the matrix cores: two chunks per wave fit the registers (111) and halve the
// tickets, barriers and look-backs per element: n = 2^28 52 -> 73 % of peak.  On the matrix cores two chunks spill
// (the three-way split of a chunk and its 16 accumulators beside the other chunk's 32 registers: 40 to 144 bytes
// per lane however the loops are shaped) and end at 46 to 50 %, so that variant keeps one.
#ifndef MMV_CPW_F32_SUM_SHUFFLE
#define MMV_CPW_F32_SUM_SHUFFLE 2
#endif
#ifndef MMV_CPW_SPMV
#define MMV_CPW_SPMV 1
#endif
#ifndef MMV_UNROLL_CHUNKS
#define MMV_UNROLL_CHUNKS 1   // 1: the chunk loops of the sum / SpMV kernels are unrolled (see kUnrollChunks)
#endif
#ifndef MMV_MIN_WAVES_PER_SIMD
#define MMV_MIN_WAVES_PER_SIMD 4   // register budget: 512 / 4 = 128 VGPRs per lane
#endif
#ifndef MMV_SPMV_STAGGER_US
#define MMV_SPMV_STAGGER_US 15   // SpMV: start times of the first round spread over this many microseconds
#endif
#ifndef MMV_KEEP_ROWS
#define MMV_KEEP_ROWS 1   // 1: single-chunk waves of the matrix-core variant keep their row scans in LDS (see kKeepRows)
#endif
#ifndef MMV_DPP_SCAN
#define MMV_DPP_SCAN 1   // 1: the sum-type kernels exchange lanes with DPP moves and v_permlane32_swap, 0: with lane shuffles through the LDS hardware
#endif
#ifndef MMV_DENSE_SHORTCUT
#define MMV_DENSE_SHORTCUT 1   // 1: fp32 scans store a chunk whose positions all start segments straight from its registers
#endif
#ifndef MMV_ROLL_STEP
#define MMV_ROLL_STEP 2
#endif
#ifndef MMV_LOAD_PRIO
#define MMV_LOAD_PRIO 1   // wave priority while a workgroup takes its ticket and issues its loads (0: off)
#endif
// Scan kernels, tiles without any flag: 0 = the aggregate is published after phase A, as for every other tile;
// 1 = the plain sum is published as soon as the tile's loads have landed; 2 = and the wave that publishes it looks
// back for the carry at once; 3 = that wave asks for the descriptors of the tiles before when its phase A is done and
// looks at them after the barrier (the look-back takes 3 to 4 us whoever has published what, so it pays to have the
// poll under way early; 2 makes the wave late for the barrier).  Per input width (measured best on MI355X; 32-bit inputs
// on the matrix cores: 3 makes the vector without flags 5 % faster and every vector with flags 2 % slower; without the
// matrix cores it costs the vectors with flags nothing: MMV_EARLY_F32_SHUFFLE).
#ifndef MMV_EARLY_I8
#define MMV_EARLY_I8 3
#endif
#ifndef MMV_EARLY_F16
#define MMV_EARLY_F16 3
#endif
#ifndef MMV_EARLY_F32
#define MMV_EARLY_F32 0
#endif
#ifndef MMV_EARLY_F32_SHUFFLE
#define MMV_EARLY_F32_SHUFFLE 3   // 32-bit inputs without the matrix cores: one segment of 2^28 values 57 -> 64 % of peak, and
                                  // nothing lost with flags (every flag set 78 -> 79.5 %, lengths U{1..64} 72 %): 2^30 stress 73 -> 75.3 %
#endif
#ifndef MMV_EARLY_F32_SCAN
#define MMV_EARLY_F32_SCAN 3   // mmv_scan of 32-bit inputs: no tile has a flag, so nothing is there to lose
#endif
#ifndef MMV_EXACT_STARTS
#define MMV_EXACT_STARTS 1   // 1: fp32 scans give a position that starts a segment its input bit for bit
#endif
#ifndef MMV_POLL_WINDOWS
#define MMV_POLL_WINDOWS 1   // windows of 64 tile descriptors that a look-back started ahead of time asks for at once (2 and 4: 3 to 5 % slower, the descriptor loads compete with the streams)
#endif
#ifndef MMV_CHUNK_SUM
#define MMV_CHUNK_SUM 1   // 1: the segmented sum of 8- and 16-bit inputs on long vectors speculates over whole chunks
#endif
#ifndef MMV_SHORT_SUMS_ROW_FORM
#define MMV_SHORT_SUMS_ROW_FORM 1   // 1: sums that fit one round of workgroups use the scan's tile body (see tile_plan)
#endif
#ifndef MMV_SUM_CPW_I8
#define MMV_SUM_CPW_I8 8    // most chunks per wave of the chunk-speculating segmented sum, 8-bit inputs
#endif
#ifndef MMV_SUM_CPW_F16
#define MMV_SUM_CPW_F16 16  // ... 16-bit inputs: two workgroups per compute unit instead of four, and longer tiles pay
                            // (n = 2^28, density 0.1 / 1 %, % of peak: 4 chunks 58 / 54, 8: 65 / 60, 16: 69 / 61.5, 32: 68 / 63;
                            // n = 2^26 and 2^27: 16 as good as or better than the shorter ones)
#endif
#ifndef MMV_SUM_WAVES_PER_SIMD_I8
#define MMV_SUM_WAVES_PER_SIMD_I8 8   // register budget of the segmented sum of 8-bit inputs: 512 / 8 = 64 VGPRs per lane (four workgroups per compute unit)
#endif
#ifndef MMV_SUM_LOAD_DEPTH_I8
#define MMV_SUM_LOAD_DEPTH_I8 2   // chunks of a wave of that sum whose loads are in flight at once, 8-bit inputs (3: 73 registers, 4: spills at 80)
#endif
#ifndef MMV_SUM_LOAD_DEPTH_F16
#define MMV_SUM_LOAD_DEPTH_F16 2   // ... 16-bit inputs
#endif
#ifndef MMV_MIN_TILES
#define MMV_MIN_TILES 512   // workgroups resident at once: 2 per compute unit (LDS)
#endif

constexpr int kS = 32;                          // row length = MFMA tile edge
constexpr int kRowsPerChunk = 64;               // a chunk = 64 rows, one per lane = two 32x32 tiles
constexpr int kChunkElems = kS * kRowsPerChunk; // 2048
constexpr int kRowStride = 36;                  // dwords per LDS row: 4 meta + 32 values
constexpr int kSlotF = 0;                       // flag word of the row
constexpr int kSlotPrefix = 1;                  // (segmented sum) sum of the rows of the chunk before this one
constexpr int kSlotNegCarry = 2;                // minus the carry into the row
constexpr int kSlotZero = 3;                    // x-bar(-1) = 0
constexpr int kRowData = 4;

constexpr uint32_t kHdrTicket = 0;              // workspace header words
constexpr uint32_t kHdrError = 1;
constexpr uint32_t kErrLookback = 1, kErrNotPrepared = 2;   // values of the status word
constexpr uint32_t kHdrHints = 32;              // first of the words the SpMV kernels read as hints (a cache line of
                                                // their own: the line of the ticket is busy with atomics):
constexpr uint32_t kHdrEmptyRows = 32;          // CSR SpMV: set when some row of the matrix has no entries
constexpr uint32_t kHdrColumnRuns = 33;         // SpMV: set when neighbouring entries mostly have consecutive columns
constexpr uint32_t kHdrPrepared = 34;         // SpMV in two steps: what the preparing call left for this matrix (0: nothing)
constexpr size_t kHdrBytes = 256;

constexpr uint64_t kStatusInvalid = 0;          // descriptor not written yet
constexpr uint64_t kStatusAggregate = 1;        // payload = aggregate of a tile without any flag
constexpr uint64_t kStatusPrefix = 2;           // payload = carry out of the tile, look-back stops here
constexpr uint32_t kMaxSpins = 1u << 20;        // bounded wait, then the status word is set

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef short v8s __attribute__((ext_vector_type(8)));

// What a kernel instantiation computes (values match mmv_op where there is one):
//   kScan       segmented inclusive scan
//   kSum        segmented sum (one output per segment, index = number of segment ends before it)
//   kSpmv       row-sorted COO SpMV: products val * x[col], sums scattered to y[row]
//   kPlainScan  unsegmented inclusive scan (no flag vector: every row aggregate is carried on)
//   kSpmvCsr    CSR SpMV: as kSpmv, but the sum of the k-th segment goes to y[rowmap[k]]
enum Op { kScan = 0, kSum = 1, kSpmv = 2, kPlainScan = 3, kSpmvCsr = 7 };

// The tiles of one launch, as up to kMaxRegions runs of equally long tiles: a long vector starts with tiles
// of growing length (the workgroups of the first round then finish at different times and the stores of
// the short ones begin while the long ones still load), continues with tiles of the full length and ends
// with tiles of shrinking length (the workgroups of the last round finish together).  The length of a tile
// is its number of chunks per wave.
constexpr int kMaxRegions = 8;
struct TileRegions {
    uint64_t base[kMaxRegions];    // first element of the region
    uint32_t first[kMaxRegions];   // first tile of the region (first[0] = 0)
    uint32_t cpw[kMaxRegions];     // chunks per wave of its tiles
    uint32_t count;                // regions in use
    uint32_t num_tiles;
};
struct TileSpan {
    uint64_t base;   // first element of the tile
    uint32_t cpw;    // its chunks per wave
};
// Where tile `tile` lies (`unit` = elements of one chunk per wave: waves x 2048).  With a uniform tile number
// everything here stays in scalar registers.
__host__ __device__ __forceinline__ TileSpan tile_span(const TileRegions &R, uint32_t tile, uint32_t unit) {
    uint64_t base = R.base[0];
    uint32_t first = 0, cpw = R.cpw[0];
#pragma unroll
    for (int i = 1; i < kMaxRegions; ++i)
        if (i < (int)R.count && tile >= R.first[i]) {
            base = R.base[i];
            first = R.first[i];
            cpw = R.cpw[i];
        }
    return {base + (uint64_t)(tile - first) * cpw * unit, cpw};
}
// The tile that holds element e.
__host__ __device__ __forceinline__ uint32_t tile_of_element(const TileRegions &R, uint64_t e, uint32_t unit) {
    uint64_t base = R.base[0];
    uint32_t first = 0, cpw = R.cpw[0];
#pragma unroll
    for (int i = 1; i < kMaxRegions; ++i)
        if (i < (int)R.count && e >= R.base[i]) {
            base = R.base[i];
            first = R.first[i];
            cpw = R.cpw[i];
        }
    return first + (uint32_t)((e - base) / ((uint64_t)cpw * unit));
}

struct Params {
    const void *x;          // values (scan, sum) / val (spmv)
    const uint32_t *fw;     // packed flag words (scan, sum)
    uint64_t n;             // elements / nnz
    void *z;                // scan output
    void *out;              // sum output
    uint64_t out_cap;
    uint64_t *nseg;
    const int32_t *row;     // spmv (coo)
    const uint32_t *rowmap; // spmv (csr): row index of the k-th non-empty row
    uint32_t first_one;     // plain scan of a flag vector: element 0 counts as 1 whatever it holds
    const int32_t *col;
    const float *xv;
    float *y;
    uint32_t *hdr;          // workspace header
    uint64_t *desc_v;       // value descriptors, one per tile
    const uint32_t *tile_count;  // sum: segment starts per tile (position 0 not counted), or ...
    uint32_t count_is_prefix;    // ... their exclusive prefix sums already (long vectors)
    const uint32_t *span_count;  // sum of 8- and 16-bit inputs: segment starts per wave span (kWaves of them per tile)
    uint32_t num_tiles;
    TileRegions reg;        // which elements a tile covers
    uint32_t prepared;      // SpMV in two steps: the mark the preparing call must have left in the header (0: not asked for)
    uint32_t first_round;   // workgroups [0, first_round) are resident together from the start and take the tile
                            // of their own index; the others take tickets
    uint32_t stagger_wgs;   // workgroups [0, stagger_wgs) start after a delay of up to ...
    uint32_t stagger_ticks; // ... this many ticks of the 100 MHz clock, spread evenly over them
};

}  // namespace
