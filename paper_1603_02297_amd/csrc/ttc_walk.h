// Index arithmetic of a tile walk, shared by the device kernels and by the host-side bounds
// checker (ttc_debug_emulate_map), so that what the checker proves in bounds is the code the
// GPU runs.
//
// A walk covers the tile with copies of one fixed sub-box.  Two small tables make a step of
// the walk cost a handful of instructions whatever the number of indices:
//   * per lane (vector registers, built once per workgroup): where the lane sits inside the
//     sub-box -- its offset in the tensor, its offset in the LDS tile, its coordinates;
//   * per sub-box position (LDS, built once per workgroup, the same for every tile): where
//     the sub-box sits inside the tile -- the same three things.
// A memory access of the walk is then  tile base + position entry + lane entry.
#pragma once

#include "ttc_internal.h"

#if defined(__HIPCC__)
#define TTC_HD __host__ __device__ __forceinline__
#else
#define TTC_HD inline
#endif

namespace ttc {

TTC_HD uint32_t fdiv(uint32_t x, const FastDiv& d)
{
    return ((uint32_t)(((uint64_t)x * d.mul) >> 32) + x) >> d.shift;
}
TTC_HD uint32_t fdigit(uint32_t x, const FastDiv& below, const FastDiv& cnt)
{
    const uint32_t q = fdiv(x, below);
    return q - fdiv(q, cnt) * cnt.div;
}

// ---- row kernel: where a logical element of B (position in the order of B's multi-index) lies ----------
// `row_index` counts rows in B's order (all indices but the first), `col` is the position inside the row.
struct RowPlace { int64_t a, b; };

TTC_HD RowPlace rows_place(const RowsParams& p, uint32_t row_index, uint32_t col)
{
    RowPlace r;
    r.a = col; r.b = col;
    uint32_t rest = row_index;
#pragma unroll
    for (int d = 1; d < kMaxDim; ++d) {             // unused indices: extent 1, stride 0
        const uint32_t q = fdiv(rest, p.size_div[d]);
        const uint32_t j = rest - q * p.size_div[d].div;
        r.a += (int64_t)j * p.stride_a[d];
        r.b += (int64_t)j * p.stride_b[d];
        rest = q;
    }
    return r;
}

// One access of the row kernel: `k` is the number of its vector inside the workgroup's chunk, which starts at
// vector `base` = row `row0`, slot `slot0` (a row holds `slots` vectors; where the row is not a multiple of the
// vector, the last one is moved back so that it ends with the row and repeats elements of its neighbour).
// (slot0 + k stays far below 2^31: rows are shorter than 2^30 elements and a chunk holds at most 2^20 vectors.)
struct RowAccess { RowPlace at; bool valid; };

TTC_HD RowAccess rows_access(const RowsParams& p, int64_t base, uint32_t row0, uint32_t slot0, uint32_t k)
{
    const uint32_t x = slot0 + k;
    const uint32_t rl = fdiv(x, p.slot_div);
    const uint32_t sl = x - rl * p.slots;
    uint32_t c = sl * (uint32_t)p.vec;
    if (c + (uint32_t)p.vec > p.row) c = p.row - (uint32_t)p.vec;      // only with overlap: the last slot of a row
    RowAccess r;
    r.valid = (base + (int64_t)k < p.vectors);
    r.at = rows_place(p, r.valid ? row0 + rl : 0u, r.valid ? c : 0u);  // past the end: the first vector, never stored
    return r;
}

// ---- which tiles a workgroup walks ---------------------------------------------------------
// Consecutive workgroup ids land on consecutive XCDs (8 of them, each with its own L2).  Every
// XCD owns one contiguous range of tile ids; its workgroups take the tiles of that range round
// robin, so tiles that are neighbours in memory are in flight on the same XCD at the same time.
// A workgroup walks positions first, first + step, ... < end of its XCD's sequence of tiles; tile_of() turns a
// position into a tile id.  Three mappings: plain round robin over all workgroups (one window that advances
// through the tensor: the lowest memory latency when tiles share no cache lines); one contiguous range of
// tile ids per XCD (neighbouring tiles always meet in one L2); and chunks of 2^k consecutive tiles dealt to the
// XCDs in turn (neighbours inside a chunk share an L2 and the window still advances as one).
struct TileSeq { uint32_t first, end, step, base, xcd, chunk_log; };

template <typename Params>       // KernelParams, or the micro-tile kernel's MicroArgs
TTC_HD TileSeq tile_sequence(const Params& p, uint32_t wg)
{
    TileSeq s;
    s.base = 0; s.xcd = 0; s.chunk_log = 0;
    if (!p.xcd_remap || p.grid < 8u) {
        s.first = wg; s.end = p.num_tiles; s.step = p.grid;
        return s;
    }
    const uint32_t x = wg & 7u, slot = wg >> 3;
    s.first = slot;
    s.step = p.grid_per_xcd + (x < p.grid_rem_xcd ? 1u : 0u);
    if (p.xcd_remap == 1) {
        s.base = x * p.tiles_per_xcd + (x < p.tiles_rem_xcd ? x : p.tiles_rem_xcd);
        s.end = p.tiles_per_xcd + (x < p.tiles_rem_xcd ? 1u : 0u);
    } else {
        s.xcd = x;
        s.chunk_log = (uint32_t)p.xcd_remap;
        s.end = p.xcd_tiles[x];
    }
    return s;
}

TTC_HD uint32_t tile_of(const TileSeq& s, uint32_t q)
{
    if (s.chunk_log == 0) return s.base + q;
    return ((s.xcd + 8u * (q >> s.chunk_log)) << s.chunk_log) + (q & ((1u << s.chunk_log) - 1u));
}

// tile id -> element offsets of the box origin in A and in B
struct TileBase { int64_t a, b; };
// what one wavefront works out for the others about a tile (two of these sit at the start of LDS)
// (per walk: the tile's limits in the walk's digits, packed for the bounds test, and whether the walk has to
// test its positions in this tile, so that the other wavefronts read all of it instead of deriving it again)
struct alignas(16) SideShare { int32_t lim[kBoxDims]; uint32_t t01, t23, dynamic, pad; };
struct alignas(16) TileShare { int64_t a, b; SideShare sa, sb; };
constexpr int kTileShareBytes = 2 * (int)sizeof(TileShare);
// after them: one spare slot of 16 bytes per lane of a wavefront, where lanes outside a tile park what they loaded
constexpr int kSpareBytes = 64 * 16;
constexpr int kTablesOff = kTileShareBytes + kSpareBytes;

TTC_HD TileBase tile_base(const KernelParams& p, uint32_t tile)
{
    TileBase t;
    t.a = 0; t.b = 0;
    // straight-line over all kMaxDim entries: unused ones hold neutral values (one tile, stride 0), and code
    // without branches lets the compiler fetch every parameter in one batch instead of index by index
#pragma unroll
    for (int k = 0; k < kMaxDim; ++k) {
        const int64_t origin = (int64_t)fdigit(tile, p.tile_below[k], p.tile_cnt[k]) * p.tile[k];
        t.a += origin * p.stride_a[k];
        t.b += origin * p.stride_b[k];
    }
    return t;
}

// How much of the box lies inside the tensor along each slot.  whole: nothing is cut off.
struct TileLim { int32_t lim[kBoxDims]; bool whole; };

TTC_HD TileLim tile_lim(const KernelParams& p, uint32_t tile)
{
    TileLim t;
    t.whole = true;
#pragma unroll
    for (int j = 0; j < kBoxDims; ++j) {            // unused slots: extent 1, size 1, one tile
        const Slot& sl = p.slot[j];
        const int64_t origin = (int64_t)fdigit(tile, sl.tile_below, sl.tile_cnt) * sl.tile;
        const int64_t left = sl.size - origin;
        t.lim[j] = (int32_t)(left < (int64_t)sl.tile ? left : (int64_t)sl.tile);
        t.whole = t.whole && (t.lim[j] == sl.tile);
    }
    return t;
}

// The same limits in the flat units of one walk's digits, and packed for the bounds test.
//
// The test "coordinate of the lane + coordinate of the sub-box < limit" runs on all four digits
// at once, 16 bits per digit: with g = 0x8000 a guard bit per field,
//     x = (g + limit - 1)  -  position  -  lane        (field by field; no field can borrow from its
//                                                      neighbour because extents stay below 32000)
// keeps its guard bit exactly where the element lies inside the limit.
constexpr uint32_t kGuard = 0x80008000u;
struct SideLim { int32_t lim[kBoxDims]; uint32_t t01, t23; };

TTC_HD SideLim side_lim(const Side& s, const TileLim& t)
{
    SideLim r;
#pragma unroll
    for (int j = 0; j < kBoxDims; ++j) r.lim[j] = t.lim[j] * s.d[j].slot_mul;
    r.t01 = (kGuard + (uint32_t)(r.lim[0] - 1)) + ((uint32_t)(r.lim[1] - 1) << 16);
    r.t23 = (kGuard + (uint32_t)(r.lim[2] - 1)) + ((uint32_t)(r.lim[3] - 1) << 16);
    return r;
}

// ---- micro-tile kernel -----------------------------------------------------------------------
// Where a tile lies and how much of it is inside the tensor along its two indices.  A remainder tile that holds
// less than one vector along an index is moved back along it until it holds one (the elements it shares with its
// neighbour are then written twice, with the same value), so lim_a and lim_b are at least vec.
// a, b: element offsets in A and B of everything but the tile's two indices, plus (a) the first column's place in A's
// run and (b) the first row's place in B's run; col0, row0: the tile's first column and row (where a column lies in
// B and a row in A follows from those, see micro_col_b / micro_row_a).
// own_a, own_b: the first column and row that are this tile's own (not 0 where the tile was moved back over its neighbour).
struct MicroTile { int64_t a, b; uint32_t col0, row0, lim_a, lim_b, own_a, own_b; };

TTC_HD MicroTile micro_tile(const MicroArgs& p, uint32_t tile)
{
    const MicroParams& m = p.micro;
    // mixed radix in tile order; straight-line over all kMaxDim places (unused ones hold one tile and no step).
    // The steps leave out what depends on the column in B and on the row in A.
    struct { int64_t a, b; } t = {0, 0};
    uint32_t rest = tile, da = 0, db = 0;
#pragma unroll
    for (int i = 0; i < kMaxDim; ++i) {
        const uint32_t next = fdiv(rest, p.cnt[i]);
        const uint32_t d = rest - next * p.cnt[i].div;
        rest = next;
        t.a += (int64_t)d * p.step_a[i];
        t.b += (int64_t)d * p.step_b[i];
        if (i == p.col_pos) da = d;
        if (i == p.row_pos) db = d;
    }
    const int64_t oa = (int64_t)da * m.ta, ob = (int64_t)db * m.tb;
    int64_t lim_a = m.size_a0 - oa < (int64_t)m.ta ? m.size_a0 - oa : (int64_t)m.ta;
    int64_t lim_b = m.size_p0 - ob < (int64_t)m.tb ? m.size_p0 - ob : (int64_t)m.tb;
    const int64_t back_a = lim_a < m.vec ? m.vec - lim_a : 0, back_b = lim_b < m.vec ? m.vec - lim_b : 0;
    MicroTile r;
    r.a = t.a - back_a;
    r.b = t.b - back_b;
    r.col0 = (uint32_t)(oa - back_a);
    r.row0 = (uint32_t)(ob - back_b);
    r.own_a = (uint32_t)back_a;
    r.own_b = (uint32_t)back_b;
    r.lim_a = (uint32_t)(lim_a + back_a);
    r.lim_b = (uint32_t)(lim_b + back_b);
    return r;
}

// Element offset in B of column x (of the whole tensor), and in A of row y.
TTC_HD int64_t micro_col_b(const MicroParams& m, uint32_t x)
{
    const uint32_t out = fdiv(x, m.col_in_div);
    return (int64_t)(x - out * m.col_in_div.div) * m.col_b_in + (int64_t)out * m.col_b_out;
}

TTC_HD int64_t micro_row_a(const MicroParams& m, uint32_t y)
{
    const uint32_t out = fdiv(y, m.row_in_div);
    return (int64_t)(y - out * m.row_in_div.div) * m.row_a_in + (int64_t)out * m.row_a_out;
}

// Where the vector (or block side) that nominally starts at x really starts in a tile holding lim (at least vec)
// elements along that index: the last one is moved back so that it ends with the tile.  Both phases apply the same
// rule, so the LDS slot of lane (row, lane_a) holds the same columns for its writer and its readers.
TTC_HD uint32_t micro_back(uint32_t x, uint32_t lim, uint32_t vec) { return x + vec > lim ? lim - vec : x; }

// The 16-byte LDS slot of row `row` of the tile, column group `lane_c`.
TTC_HD uint32_t micro_slot(const MicroParams& m, uint32_t row, uint32_t lane_c)
{
    return row * (uint32_t)m.pitch + (lane_c ^ ((row >> m.vec_log) & m.swizzle));
}

// Load walk: vector k of lane `tid` (vectors are numbered row by row, so consecutive lanes load consecutive
// vectors of a row).  row runs along A's index p0 (B's stride-1 index), col along A's index 0; chunk is the
// 16-byte slot of the LDS tile the vector is parked in.  valid: the vector is one of the tile's.
struct MicroLoad { uint32_t row, col, chunk; bool valid; };

TTC_HD MicroLoad micro_load(const MicroParams& m, uint32_t threads, uint32_t tid, uint32_t k)
{
    const uint32_t g = tid + k * threads;
    MicroLoad r;
    r.row = fdiv(g, m.la_div);
    const uint32_t lane_a = g - r.row * (uint32_t)m.la;
    r.col = lane_a << m.vec_log;
    r.chunk = micro_slot(m, r.row, lane_a);
    r.valid = r.row < (uint32_t)m.tb;
    return r;
}

// Store walk: block b of lane `tid` (blocks are numbered along B's stride-1 index first): vec rows x vec columns
// nominally starting at (row, col).  Row r of the tile, column group lane_c, sits in LDS slot micro_slot(m, r, lane_c).
struct MicroBlock { uint32_t row, col, lane_c; bool valid; };

TTC_HD MicroBlock micro_block(const MicroParams& m, uint32_t threads, uint32_t tid, uint32_t b)
{
    const uint32_t h = tid + b * threads;
    MicroBlock r;
    r.lane_c = fdiv(h, m.lb_div);
    const uint32_t lane_r = h - r.lane_c * (uint32_t)m.lb;
    r.row = lane_r << m.vec_log;
    r.col = r.lane_c << m.vec_log;
    r.valid = r.lane_c < (uint32_t)m.la;
    return r;
}

// ---- lane entry ------------------------------------------------------------------------------
// Offsets are in BYTES.  A walk has three element sizes: of the tensor it follows (g), of B in
// the direct kernel (g2), and of the LDS tile, which holds elements of A (l).
struct Scales { int32_t g, g2, l; };

struct LaneState {
    int64_t g;                 // byte offset into the tensor the walk follows
    int64_t g2;                // direct kernel: byte offset into B
    int32_t l;                 // byte offset into the LDS tile
    uint32_t c01, c23;         // flat coordinate along each digit, in elements, 16 bits per digit
    bool    active;
};

template <bool DIRECT>
TTC_HD LaneState lane_setup(const Side& s, uint32_t lane, const Scales& scale)
{
    LaneState L;
    L.g = 0; L.g2 = 0; L.l = 0;
    L.active = lane < (uint32_t)s.lanes;
    uint32_t cs[kBoxDims];
#pragma unroll
    for (int j = 0; j < kBoxDims; ++j) {            // empty digits: one lane step, stride 0
        const Digit& d = s.d[j];
        const int32_t c = (int32_t)fdigit(lane, d.lane_below, d.lane_cnt) * d.lane_mul;
        cs[j] = (uint32_t)c;
        L.g += (int64_t)c * d.gstride;
        if (DIRECT) L.g2 += (int64_t)c * d.g2stride;
        else L.l += c * d.lstride;
    }
    L.g *= scale.g; L.g2 *= scale.g2; L.l *= scale.l;
    L.c01 = cs[0] | (cs[1] << 16);
    L.c23 = cs[2] | (cs[3] << 16);
    return L;
}

// ---- position entry --------------------------------------------------------------------------
// 16 + 8 bytes per sub-box position: offsets of the sub-box origin, and its coordinates inside
// the tile packed 16 bits per digit (flat extents of a digit stay below 32000).
struct alignas(16) PosEntry {
    int64_t g;                 // byte offset in the tensor the walk follows
    int64_t l_or_g2;           // staged kernel: LDS byte offset; direct kernel: byte offset in B
};
struct alignas(8) PosCoord { uint32_t c01, c23; };

template <bool DIRECT>
TTC_HD void make_position(const Side& s, uint32_t it, const Scales& scale, PosEntry* e, PosCoord* c)
{
    int64_t g = 0, x = 0;
    uint32_t pc[kBoxDims];
#pragma unroll
    for (int i = 0; i < kBoxDims; ++i) {            // digits with one position contribute 0
        const Digit& d = s.d[i];
        const uint32_t q = fdigit(it, d.iter_below, d.iter_cnt) * (uint32_t)d.lane;
        pc[i] = q;
        g += (int64_t)q * d.gstride;
        x += (int64_t)q * (DIRECT ? d.g2stride : (int64_t)d.lstride);
    }
    e->g = g * scale.g;
    e->l_or_g2 = x * (DIRECT ? scale.g2 : scale.l);
    c->c01 = pc[0] | (pc[1] << 16);
    c->c23 = pc[2] | (pc[3] << 16);
}

// Limits of one tile as one lane sees them: the lane's own coordinates already taken off.
struct LaneLim { uint32_t x01, x23; };

TTC_HD LaneLim lane_lim(const LaneState& L, const SideLim& lim)
{
    LaneLim r;
    r.x01 = lim.t01 - L.c01;
    r.x23 = lim.t23 - L.c23;
    return r;
}

// does this lane's element (the first one of its vector) at this sub-box position lie inside the
// box and the tensor?
TTC_HD bool lane_valid(const LaneLim& x, const PosCoord& pc)
{
    return (((x.x01 - pc.c01) & (x.x23 - pc.c23)) & kGuard) == kGuard;
}

// Vectors of V elements along the walk's first digit whose extent is not a multiple of V: by how many
// elements must the lane's vector move back so that it ends inside the limit?  0 .. V-1, or -1 if not
// even its first element lies inside (the limit is at least V, so a moved vector never starts before 0).
template <int V>
TTC_HD int lane_back(const LaneLim& x, const PosCoord& pc, int vec_slot)
{
    const uint32_t a = x.x01 - pc.c01, b = x.x23 - pc.c23;
    if (((a & b) & kGuard) != kGuard) return -1;
    const uint32_t w = (vec_slot & 2) ? b : a;
    const uint32_t f = (vec_slot & 1) ? (w >> 16) : w;
    const int left = (int)(f & 0x7fffu) + 1;          // the field holds limit - 1 - coordinate
    return left < V ? V - left : 0;
}

// Which sub-box positions a wavefront takes, and where their table entries sit.  Wavefront w of
// nwave takes positions w, w + nwave, w + 2 nwave, ...; the tables are stored wave-major, the
// k-th position of wavefront w at index w * chunk + k, so that a wavefront reads consecutive
// entries.
TTC_HD uint32_t wave_positions(const Side& s, uint32_t wave)
{
    return (uint32_t)s.chunk - (wave >= (uint32_t)s.chunk_rem ? 1u : 0u);
}

// How a group of positions treats the bounds: no test at all, whole vectors tested, or vectors
// that are moved back where the run ends inside them.
enum { kWalkFull = 0, kWalkMasked = 1, kWalkPartial = 2 };

// U positions at a time: stage1 for all U (issue the loads), then stage2 for all U (consume
// them), so that U memory instructions are in flight per wavefront.  stage(u, entry, back, ok):
// u = slot 0..U-1, back = elements the lane's vector is moved back by (0 unless the walk is partial),
// ok = the lane's element lies inside the tile.  Stages run for every lane: a lane that is not ok must
// do something harmless (load the tile's first vector, write to a spare LDS slot, skip a global store),
// so that no load sits inside divergent control flow, where it would be waited for on the spot.
template <int U, int V, int MODE, class Stage1, class Stage2>
TTC_HD void walk_group(const LaneLim& x, int vec_slot, const PosEntry* e_ptr, const PosCoord* c_ptr,
                       Stage1&& stage1, Stage2&& stage2)
{
    PosEntry e[U];
    int back[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        e[u] = e_ptr[u];
        if (MODE == kWalkFull) back[u] = 0;
        else if (MODE == kWalkMasked) back[u] = lane_valid(x, c_ptr[u]) ? 0 : -1;
        else back[u] = lane_back<V>(x, c_ptr[u], vec_slot);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        stage1(u, e[u], (MODE == kWalkPartial && back[u] > 0) ? back[u] : 0, MODE == kWalkFull ? true : back[u] >= 0);
#pragma unroll
    for (int u = 0; u < U; ++u)
        stage2(u, e[u], (MODE == kWalkPartial && back[u] > 0) ? back[u] : 0, MODE == kWalkFull ? true : back[u] >= 0);
}

// What a walk has to test per lane in one tile.  Digits with a single sub-box position are
// tested once per tile (lane_ok); only digits that step AND are cut by the tensor's edge or
// overhang the tile need the test at every position (dynamic, wave-uniform).
struct WalkMask { bool lane_ok; bool dynamic; };

// bit j: digit j has a single sub-box position (the same for every tile)
TTC_HD uint32_t single_digits(const Side& s)
{
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < kBoxDims; ++j) m |= (s.d[j].iters == 1 ? 1u : 0u) << j;
    return m;
}

// the wave-uniform half: does the walk have to test its positions in this tile?
TTC_HD bool walk_dynamic(const Side& s, const SideLim& lim)
{
    bool dynamic = (s.partial != 0);
#pragma unroll
    for (int j = 0; j < kBoxDims; ++j) {
        const Digit& d = s.d[j];
        if (d.iters != 1) dynamic = dynamic | (lim.lim[j] != d.tile) | (d.ragged != 0);
    }
    return dynamic;
}

// the per-lane half: is the lane inside the tile along the digits that do not step?
TTC_HD bool lane_inside(uint32_t single, const LaneState& L, const SideLim& lim)
{
    bool ok = L.active;
#pragma unroll
    for (int j = 0; j < kBoxDims; ++j) {
        const int32_t c = (int32_t)(((j & 2) ? L.c23 : L.c01) >> ((j & 1) ? 16 : 0)) & 0xffff;
        if ((single >> j) & 1u) ok = ok & (c < lim.lim[j]);
    }
    return ok;
}

// one walk's part of the shared tile record
TTC_HD SideShare make_side_share(const Side& s, const TileLim& tl)
{
    const SideLim sl = side_lim(s, tl);
    SideShare v;
    v.lim[0] = sl.lim[0]; v.lim[1] = sl.lim[1]; v.lim[2] = sl.lim[2]; v.lim[3] = sl.lim[3];
    v.t01 = sl.t01; v.t23 = sl.t23;
    v.dynamic = walk_dynamic(s, sl) ? 1u : 0u;
    v.pad = 0;
    return v;
}

TTC_HD WalkMask walk_mask(const Side& s, const LaneState& L, const SideLim& lim)
{
    WalkMask m;
    m.lane_ok = lane_inside(single_digits(s), L, lim);
    m.dynamic = walk_dynamic(s, lim);
    return m;
}

template <int U, int V, int MODE, class Stage1, class Stage2>
TTC_HD void walk_mode(const LaneLim& x, int vec_slot, const PosEntry* my, const PosCoord* myc, uint32_t cnt,
                      Stage1&& stage1, Stage2&& stage2)
{
    uint32_t k = 0;
    for (; k + U <= cnt; k += U) walk_group<U, V, MODE>(x, vec_slot, my + k, myc + k, stage1, stage2);
    for (; k < cnt; ++k) walk_group<1, V, MODE>(x, vec_slot, my + k, myc + k, stage1, stage2);
}

// Drive one wavefront through its share of a walk with V elements per lane and access.
template <int U, int V, class Stage1, class Stage2>
TTC_HD void walk(const Side& s, const LaneState& L, const SideLim& lim, const WalkMask& m, const PosEntry* tab,
                 const PosCoord* tabc, uint32_t wave, Stage1&& stage1, Stage2&& stage2)
{
    if (!m.lane_ok) return;
    const uint32_t cnt = wave_positions(s, wave);
    const PosEntry* my = tab + wave * (uint32_t)s.chunk;
    const PosCoord* myc = tabc + wave * (uint32_t)s.chunk;
    const LaneLim x = lane_lim(L, lim);
    if (!m.dynamic) walk_mode<U, V, kWalkFull>(x, 0, my, myc, cnt, stage1, stage2);
    else if (V == 1 || !s.partial) walk_mode<U, V, kWalkMasked>(x, 0, my, myc, cnt, stage1, stage2);
    else walk_mode<U, V, kWalkPartial>(x, s.vec_slot, my, myc, cnt, stage1, stage2);
}

// Fill the two tables of one walk (all threads of the workgroup take part).
template <bool DIRECT>
TTC_HD void build_tables(const Side& s, uint32_t nwave, uint32_t thread, uint32_t nthreads, const Scales& scale,
                         PosEntry* tab, PosCoord* tabc)
{
    const uint32_t total = nwave * (uint32_t)s.chunk;
    for (uint32_t j = thread; j < total; j += nthreads) {
        const uint32_t w = fdiv(j, s.chunk_div);
        const uint32_t it = w + (j - w * (uint32_t)s.chunk) * nwave;
        if (it < (uint32_t)s.n_iter) make_position<DIRECT>(s, it, scale, &tab[j], &tabc[j]);
    }
}

}  // namespace ttc
