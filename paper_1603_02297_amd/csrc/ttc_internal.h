// Internal declarations shared by the host planner (ttc_plan.cpp) and the device side
// (ttc_device.hip).  Nothing here is part of the C ABI.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "ttc.h"
#include "ttc_aux.h"

namespace ttc {

constexpr int kMaxDim = TTC_MAX_DIM;
constexpr int kWave = 64;                 // CDNA wavefront
constexpr int kMaxThreads = 512;          // launch bound of every kernel
constexpr int kMaxLdsBytes = 160 * 1024;  // per workgroup: all of a CU's LDS (gfx950); smaller tiles let several workgroups share it

// Exact unsigned division by a run-time constant d >= 1 for any 32-bit x whose
// quotient sum does not overflow (x < 2^31 is enough):
//   q = (mulhi(x, mul) + x) >> shift,   mul = floor(2^32 (2^shift - d) / d) + 1,  shift = ceil(log2 d).
struct FastDiv {
    uint32_t mul;
    uint32_t shift;
    uint32_t div;
};
FastDiv make_fastdiv(uint32_t d);

constexpr int kBoxDims = 4;               // a box spans at most this many indices
constexpr int kMaxIters = 2048;           // sub-box positions per tile and walk (size of the position table)
constexpr int kMaxDigitExtent = 32000;    // flat extent of one digit of a walk: coordinates are compared 16 bits at a time

// A box spans at most kBoxDims indices of the tensor; "slot" j is the j-th of them in A order.
// Each walk ("side") sees the box as up to kBoxDims digits.  A digit is one index, or -- when
// the leading indices of the walk's tensor lie whole inside the box -- the chain of those
// indices merged into one flat index (the tile-level form of the paper's index fusion): the
// flat digit is contiguous in memory over the whole chain.  Digits are stored at the slot of
// the chain's outermost index, the only one the tensor's edge can cut; a slot whose index is
// an inner member of a chain holds an empty digit (tile = 1).
struct Digit {
    int32_t  tile;                   // flat extent of the digit inside the box
    int32_t  lane;                   // flat extent of the sub-box the 64 lanes cover
    int32_t  iters;                  // ceil(tile / lane): sub-box positions along the digit
    int32_t  lane_mul;               // flat elements per lane step: vec on the vector digit, else 1
    int32_t  slot_mul;               // flat elements per step of the slot's index (product of merged inner extents)
    int32_t  lstride;                // LDS element stride of one flat step
    int32_t  ragged;                 // 1: lane does not divide tile (the last sub-box position overhangs)
    int32_t  pad;
    FastDiv  lane_below, lane_cnt;   // lane id -> lane coordinate: (lane / below) % cnt
    FastDiv  iter_below, iter_cnt;   // position id -> position digit
    int64_t  gstride;                // element stride of one flat step in the tensor the walk follows
    int64_t  g2stride;               // direct kernel: element stride in B
};

struct Side {
    int32_t  vec;                    // elements per lane per access, along the walk's first digit
    int32_t  lanes;                  // active lanes of a wavefront
    int32_t  n_iter;                 // sub-box positions per tile = prod(iters)
    int32_t  vec_lds_stride;         // LDS element stride between the vec elements of one lane
    int32_t  exact;                  // 1: lane divides tile on every digit (no ragged sub-boxes)
    int32_t  chunk;                  // positions per wavefront, rounded up: ceil(n_iter / waves)
    int32_t  chunk_rem;              // wavefronts that really have `chunk` positions (the others have one less)
    int32_t  partial;                // 1: the first digit's extent is not a multiple of vec: the last vector of a run is cut
    int32_t  vec_slot;               // slot (0..3) that holds the walk's first digit, the one vectors run along
    FastDiv  chunk_div;
    Digit    d[kBoxDims];
};

struct Slot {
    int32_t  tile;                   // box extent along the slot's index
    int32_t  pad;
    int64_t  size;                   // extent of the index in the tensor
    FastDiv  tile_below, tile_cnt;   // tile id -> tile coordinate along this index
};

// The micro-tile kernel: a tile spans ta columns and tb rows and nothing else.  The column index is A's stride-1
// index (index 0), or A's indices 0 and 1 taken as one index where rows are short (together they are one contiguous
// run of A, and a column's place in B follows from its two parts); the row index is B's stride-1 index (A's index
// p0), or B's first two indices taken as one.  Lanes load 16-byte vectors along the columns and park them in LDS with
// one 128-bit write; after the barrier a lane reads the vec x vec block it owns with vec 128-bit reads, transposes
// it in registers and stores vec 16-byte vectors along the rows.  Rows of the LDS tile are `pitch`
// 16-byte chunks long (a multiple of eight); chunk c of row r sits at chunk position c ^ ((r / vec) & 7), which
// makes both the writes (lanes along c) and the reads (lanes along r in steps of vec) free of bank conflicts.
struct MicroParams {
    int32_t  ta, tb;                 // tile extents along the column index and along the row index (multiples of vec)
    int32_t  p0;                     // the index of A that is B's stride-1 index
    int32_t  merged_a, merged_b;     // 1: the column index is A's indices 0 and 1 taken as one (contiguous in A), the row
                                     // index B's first two indices taken as one (contiguous in B); 0: one index each
    int32_t  vec, vec_log;           // elements in 16 bytes, and its log2
    int32_t  la, lb;                 // ta / vec and tb / vec: vectors per row of the tile, blocks per column
    int32_t  pitch;                  // 16-byte chunks per row of the LDS tile: la rounded up to a multiple of 8
    uint32_t swizzle;                // 7: chunk c of row r sits at c ^ ((r / vec) & 7); 0: rows laid out plainly (measurement aid)
    int32_t  loads;                  // vectors a lane loads per tile: ceil(la * tb / threads)
    int32_t  blocks;                 // vec x vec blocks a lane owns: ceil(la * lb / threads)
    FastDiv  la_div, lb_div;
    int64_t  size_a0, size_p0;       // extents of the column index and of the row index (the product where two are merged)
    // A column x sits at element x of A's run and at (x % in) * stride_in + (x / in) * stride_out in B, where `in`
    // is the extent of A's index 0; a row likewise with the tensors exchanged.  Not merged: x / in is always 0.
    FastDiv  col_in_div, row_in_div;
    int64_t  col_b_in, col_b_out;    // element strides in B of the column index's inner and outer part
    int64_t  row_a_in, row_a_out;    // element strides in A of the row index's inner and outer part
};

// Everything a kernel launch needs; passed by value as the kernel argument.
struct KernelParams {
    int32_t  n;                      // fused number of indices
    int32_t  xcd_remap;              // how tile ids map to the 8 XCDs: 0 round robin, 1 one contiguous range each,
                                     // k >= 2: chunks of 2^k consecutive tiles dealt round robin
    uint32_t num_tiles;
    uint32_t tiles_per_xcd;          // num_tiles / 8
    uint32_t tiles_rem_xcd;          // num_tiles % 8
    uint32_t grid;                   // workgroups launched (filled at launch; <= num_tiles)
    uint32_t grid_per_xcd;           // grid / 8
    uint32_t grid_rem_xcd;           // grid % 8
    uint32_t xcd_tiles[8];           // chunked mapping: tiles of each XCD
    int32_t  lds_data_off;           // byte offset of the first data buffer in dynamic LDS
    int32_t  lds_tile_elems;         // elements per LDS data buffer (padded tile)
    int32_t  lds_buffers;            // 2: tile buffers alternate, one barrier per tile; 1: one buffer, two barriers
    int32_t  nt_a;                   // 1: loads of A carry the non-temporal hint (streamed, not kept in cache)
    int32_t  nslots;                 // indices the box spans
    int32_t  nt_b;                   // 1: stores to B, and loads of B when beta != 0, carry the non-temporal hint
    Slot     slot[kBoxDims];
    int32_t  tile[kMaxDim];          // box extent per fused index of A (1 = index not blocked)
    FastDiv  tile_below[kMaxDim];    // prod of tile counts of the indices that vary faster in the tile order
    FastDiv  tile_cnt[kMaxDim];      // ceil(size[k] / tile[k])
    int64_t  stride_a[kMaxDim];      // element stride of fused index k in A
    int64_t  stride_b[kMaxDim];      // element stride of fused index k in B
    Side     a;                      // load walk (A order)
    Side     b;                      // store walk (B order); unused by the direct kernel
    double   alpha[2];               // re, im (im = 0 for real types)
    double   beta[2];
    int32_t  debug_stop;             // measurement aid: 1 = every workgroup returns after its set-up (micro-tile kernel: 2 = after its loads)
    int32_t  pad_end;
    MicroParams micro;               // micro-tile kernel only
};

// The micro-tile kernel's whole argument: what it needs of KernelParams and nothing else, seven 64-byte lines
// instead of twenty-six.  Every workgroup reads its arguments through the scalar cache before it can issue a
// load, and that shows: a copy kernel that first reads 1.6 KB of arguments takes 0.9 us longer per launch than the
// same kernel with 24 bytes (8 MB: 3.8 against 2.9 us; 32 MB: 8.3 against 7.2 us).  Built from the candidate at
// launch (micro_args()), so that the tile mapping and the streaming hints are the plan's current ones.
struct MicroArgs {
    int32_t  xcd_remap;              // the fields of KernelParams that tile_sequence() reads, under the same names
    uint32_t num_tiles, tiles_per_xcd, tiles_rem_xcd;
    uint32_t grid, grid_per_xcd, grid_rem_xcd;
    uint32_t xcd_tiles[8];
    int32_t  nt_a, nt_b;
    int32_t  debug_stop;
    int32_t  col_pos, row_pos;       // where the column index and the row index stand in the tile order
    int32_t  pad;
    FastDiv  cnt[kMaxDim];           // tile id -> tile coordinates, mixed radix in tile order: tiles along the i-th index of the order
    int64_t  step_a[kMaxDim];        // element offset in A, and in B, of one tile step along it (the column index: its place
    int64_t  step_b[kMaxDim];        // in A's run only; the row index: its place in B's run only; see MicroTile)
    double   alpha[2], beta[2];
    MicroParams micro;
};

// Parameters of the row kernel (stride-1 index fixed: rows are contiguous in both tensors).  B is walked in
// the order of its multi-index, so the writes of consecutive workgroups are consecutive in memory.
struct RowsParams {
    int32_t  n;                      // fused number of indices; index 0 is the row
    int32_t  vec;                    // elements per lane and access
    int32_t  unroll;                 // accesses a lane keeps in flight
    int32_t  overlap;                // 1: rows are not a multiple of vec: the last vector of a row is moved back to end with it
    uint32_t row;                    // extent of index 0
    uint32_t slots;                  // vectors per row: ceil(row / vec)
    uint32_t chunk;                  // vectors a workgroup moves: threads * unroll
    int32_t  nt_a, nt_b;             // non-temporal accesses per side
    int32_t  pad;
    FastDiv  slot_div;               // x / slots
    FastDiv  size_div[kMaxDim];      // extent of B's index d, d = 1 .. n-1 (entry 0 unused)
    int64_t  stride_a[kMaxDim];      // element stride in A of B's index d
    int64_t  stride_b[kMaxDim];      // element stride in B of B's index d
    int64_t  vectors;                // rows * slots
    double   alpha[2];
    double   beta[2];
};

// One candidate launch configuration ("candidate" in the paper's Section 3).
struct Candidate {
    int      kernel_class;           // TTC_KERNEL_*
    int      threads;
    int      wg_per_cu;              // workgroups launched per compute unit (each walks several tiles)
    int      lds_bytes;              // dynamic LDS per workgroup: shared tile records, spare slots, position tables, one or two tile buffers
    int      tile_order[kMaxDim];
    int      tile[kMaxDim], lds_stride[kMaxDim];   // by fused index of A
    int      digits_a, digits_b;                   // digits of each walk, in the walk's own order:
    int      dtile_a[kBoxDims], dlane_a[kBoxDims]; //   flat extent and lane sub-box extent
    int      dtile_b[kBoxDims], dlane_b[kBoxDims];
    int      lds_conflict_a, lds_conflict_b;
    double   score;                  // heuristic cost, smaller is better
    float    tuned_ms;
    KernelParams kp;                 // box kernels (staged and direct); the streaming flags and the tile mapping of every class
    RowsParams rows;                 // row kernel
};

// Element kinds of one tensor (the two tensors of a mixed-precision problem differ).
enum { kKindF32 = 0, kKindF64 = 1, kKindC64 = 2, kKindC128 = 3 };

struct Problem {
    int      dtype;                  // TTC_* code the plan was created with
    int      kind_a, kind_b;         // element kind of A and of B
    int      eb_a, eb_b;             // element bytes of A (also the LDS tile's) and of B
    int      epilogue;               // TTC_EPI_*
    int      ndim;                   // fused
    int64_t  size[kMaxDim];
    int      perm[kMaxDim];
    int64_t  stride_a[kMaxDim];      // by fused index of A; from the leading dimensions, dense if none were given
    int64_t  stride_b[kMaxDim];      // by fused index of A (stride it has in B)
    int64_t  elements;
    int64_t  span_a, span_b;         // elements from the first to the last element of each (sub-)tensor, inclusive
    double   alpha[2], beta[2];
};

}  // namespace ttc

struct ttc_plan_s {
    ttc::Problem prob;
    std::vector<ttc::Candidate> cands;     // complete: candidate 0 is ttc_plan_create's choice, the others follow ranked
                                           // by the heuristic cost; not complete: only that choice
    int selected;
    bool complete;
};

namespace ttc {

// Host planner.  Returns TTC_OK and fills *out, or a status.
int build_plan(int dtype, int ndim, const int64_t* sizes, const int* perm, const int64_t* lda, const int64_t* ldb,
               const void* alpha, const void* beta, ttc_plan_s* out);
int complete_plan(ttc_plan_s* plan);
void set_last_status(int status);
bool verbose();
// Plan store (ttc_cache.cpp).
int cache_store(const ttc_plan_s* plan, const char* path);
int cache_lookup(ttc_plan_s* plan, const char* path);
// Workgroups to launch for a candidate on a device with `cus` compute units.
uint32_t launch_grid(const Candidate& c, int cus);
void set_grid(KernelParams* kp, uint32_t grid);
// tile ids -> XCDs: 0 round robin, 1 one contiguous range per XCD, 2..10: chunks of 2^mode tiles dealt in turn
// mode -1: the default, chunks of 32 tiles; round robin below 2048 tiles
constexpr int kDefaultTileMapping = -1;
bool set_tile_mapping(KernelParams* kp, int mode);
void default_streaming(const Problem& P, Candidate* c);
MicroArgs micro_args(const Candidate& c);

}  // namespace ttc
