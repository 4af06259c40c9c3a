// Host planner: validation, size-1 removal, index fusion (paper Section 3, stage (1)),
// case split (Section 3.1), candidate enumeration with a heuristic ranking (Sections 3.2,
// 3.3 and the candidate queue of Section 3).  Pure host C++: no device is touched here.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <unordered_map>

#include "ttc_internal.h"
#include "ttc_walk.h"

namespace ttc {

static thread_local int g_last_status = TTC_OK;
void set_last_status(int status) { g_last_status = status; }

// TTC_VERBOSE=1 in the environment: one line on stderr per plan, per completed candidate list and per search
bool verbose()
{
    static const bool on = [] { const char* e = std::getenv("TTC_VERBOSE"); return e && *e && *e != '0'; }();
    return on;
}

FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    if (d <= 1) { f.div = 1; f.shift = 0; f.mul = 1; return f; }      // (x * 1 >> 32) + x >> 0 = x for x < 2^32
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    f.div = d;
    f.shift = s;
    f.mul = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << s) - d)) / d + 1);
    return f;
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t round_up(int64_t a, int64_t m) { return ceil_div(a, m) * m; }

// ---------------------------------------------------------------------------------
// Normalisation: element kinds, strides from the leading dimensions, drop extents of 1, merge
// indices that stay adjacent and in order and are contiguous in both tensors.
// ---------------------------------------------------------------------------------
static int kind_bytes(int kind) { return kind == kKindF32 ? 4 : (kind == kKindC128 ? 16 : 8); }

static bool dtype_kinds(int dtype, int* ka, int* kb)
{
    switch (dtype) {
    case TTC_F32:      *ka = kKindF32;  *kb = kKindF32;  return true;
    case TTC_F64:      *ka = kKindF64;  *kb = kKindF64;  return true;
    case TTC_C64:      *ka = kKindC64;  *kb = kKindC64;  return true;
    case TTC_C128:     *ka = kKindC128; *kb = kKindC128; return true;
    case TTC_F32_F64:  *ka = kKindF32;  *kb = kKindF64;  return true;
    case TTC_F64_F32:  *ka = kKindF64;  *kb = kKindF32;  return true;
    case TTC_C64_C128: *ka = kKindC64;  *kb = kKindC128; return true;
    case TTC_C128_C64: *ka = kKindC128; *kb = kKindC64;  return true;
    default: return false;
    }
}

static int normalise(int dtype, int ndim, const int64_t* sizes, const int* perm, const int64_t* lda,
                     const int64_t* ldb, const void* alpha, const void* beta, Problem* P)
{
    if (!sizes || !perm) return TTC_ERR_NULL_POINTER;
    int ka, kb;
    if (!dtype_kinds(dtype, &ka, &kb)) return TTC_ERR_UNSUPPORTED_DTYPE;
    if (ndim < 1 || ndim > kMaxDim) return TTC_ERR_INVALID_VALUE;
    bool seen[kMaxDim] = {false};
    for (int j = 0; j < ndim; ++j) {
        if (perm[j] < 0 || perm[j] >= ndim || seen[perm[j]]) return TTC_ERR_INVALID_PERM;
        seen[perm[j]] = true;
    }
    int64_t total = 1, alloc_a = 1, alloc_b = 1;
    for (int k = 0; k < ndim; ++k)
        if (sizes[k] < 1) return TTC_ERR_INVALID_VALUE;
    for (int k = 0; k < ndim; ++k) {
        const int64_t la = lda ? lda[k] : sizes[k], lb = ldb ? ldb[k] : sizes[perm[k]];
        if (la < sizes[k] || lb < sizes[perm[k]]) return TTC_ERR_INVALID_VALUE;
        if (total > (INT64_MAX / 16) / sizes[k]) return TTC_ERR_OVERFLOW;
        if (alloc_a > (INT64_MAX / 16) / la || alloc_b > (INT64_MAX / 16) / lb) return TTC_ERR_OVERFLOW;
        total *= sizes[k];
        alloc_a *= la;
        alloc_b *= lb;
    }
    // strides in the caller's index space (paper Table 1, --lda / --ldb: the tensor may be a part of
    // a larger one whose extents are the leading dimensions)
    int64_t sa[kMaxDim], sb[kMaxDim];          // sa by index of A; sb by index (position) of B
    sa[0] = 1; sb[0] = 1;
    for (int k = 1; k < ndim; ++k) {
        sa[k] = sa[k - 1] * (lda ? lda[k - 1] : sizes[k - 1]);
        sb[k] = sb[k - 1] * (ldb ? ldb[k - 1] : sizes[perm[k - 1]]);
    }
    int64_t span_a = 1, span_b = 1;
    for (int k = 0; k < ndim; ++k) {
        span_a += (sizes[k] - 1) * sa[k];
        span_b += (sizes[perm[k]] - 1) * sb[k];
    }

    // 1. drop size-1 extents (they contribute offset 0 on both sides)
    int newidx[kMaxDim], m = 0;
    int64_t s1[kMaxDim], sa1[kMaxDim];
    for (int k = 0; k < ndim; ++k) {
        newidx[k] = -1;
        if (sizes[k] > 1) { newidx[k] = m; s1[m] = sizes[k]; sa1[m] = sa[k]; ++m; }
    }
    int p1[kMaxDim], mp = 0;
    int64_t sb1[kMaxDim];                      // by kept position of B
    for (int j = 0; j < ndim; ++j)
        if (sizes[perm[j]] > 1) { p1[mp] = newidx[perm[j]]; sb1[mp] = sb[j]; ++mp; }
    if (m == 0) { m = 1; s1[0] = 1; p1[0] = 0; sa1[0] = 1; sb1[0] = 1; }

    // 2. merge: B positions j, j+1 holding A indices a, a+1 form one index if the pair is contiguous in
    //    both tensors: ld(i_{m+1}) = size(i_m) * ld(i_m), the condition of the footnote in Section 3.
    int group_start[kMaxDim], group_len[kMaxDim], group_pos[kMaxDim], ng = 0;     // groups in B order
    for (int j = 0; j < m;) {
        int len = 1;
        while (j + len < m && p1[j + len] == p1[j + len - 1] + 1 &&
               sa1[p1[j + len]] == sa1[p1[j + len - 1]] * s1[p1[j + len - 1]] &&
               sb1[j + len] == sb1[j + len - 1] * s1[p1[j + len - 1]]) ++len;
        group_start[ng] = p1[j];
        group_len[ng] = len;
        group_pos[ng] = j;
        ++ng;
        j += len;
    }
    // fused index of A = rank of the group's first A index
    int rank_of_group[kMaxDim];
    for (int g = 0; g < ng; ++g) {
        int r = 0;
        for (int h = 0; h < ng; ++h) if (group_start[h] < group_start[g]) ++r;
        rank_of_group[g] = r;
    }
    P->dtype = dtype;
    P->kind_a = ka; P->kind_b = kb;
    P->eb_a = kind_bytes(ka); P->eb_b = kind_bytes(kb);
    P->ndim = ng;
    P->elements = total;
    P->span_a = span_a; P->span_b = span_b;
    for (int k = 0; k < kMaxDim; ++k) { P->size[k] = 0; P->perm[k] = 0; P->stride_a[k] = 0; P->stride_b[k] = 0; }
    for (int g = 0; g < ng; ++g) {
        int64_t sz = 1;
        for (int i = 0; i < group_len[g]; ++i) sz *= s1[group_start[g] + i];
        const int r = rank_of_group[g];
        P->size[r] = sz;
        P->perm[g] = r;
        P->stride_a[r] = sa1[group_start[g]];
        P->stride_b[r] = sb1[group_pos[g]];
    }

    // scalars (defaults of the paper's Table 1: alpha = 1, beta = 0), in the precision the arithmetic
    // runs in: the data type's, or double for mixed precision
    const bool wide = (ka == kKindF64 || ka == kKindC128 || kb == kKindF64 || kb == kKindC128);
    const bool cplx = (ka == kKindC64 || ka == kKindC128);
    auto read = [&](const void* src, double* dst) {
        if (wide) { dst[0] = ((const double*)src)[0]; dst[1] = cplx ? ((const double*)src)[1] : 0.0; }
        else      { dst[0] = ((const float*)src)[0];  dst[1] = cplx ? ((const float*)src)[1] : 0.0; }
    };
    P->alpha[0] = 1.0; P->alpha[1] = 0.0; P->beta[0] = 0.0; P->beta[1] = 0.0;
    if (alpha) read(alpha, P->alpha);
    if (beta) read(beta, P->beta);
    const bool beta0 = (P->beta[0] == 0.0 && P->beta[1] == 0.0);
    const bool alpha1 = (P->alpha[0] == 1.0 && P->alpha[1] == 0.0);
    P->epilogue = beta0 ? (alpha1 ? TTC_EPI_COPY : TTC_EPI_SCALE) : TTC_EPI_AXPBY;
    return TTC_OK;
}

// ---------------------------------------------------------------------------------
// Tile (box) construction
// ---------------------------------------------------------------------------------

// Extent near `want` along an index of size s, a multiple of mult (s % mult == 0).
// Divisors of s are preferred (no remainder tiles: the second rule of the paper's blocking
// heuristic, Section 3.2); otherwise the index is cut into equal pieces.
static int pick_extent(int64_t s, int64_t want, int mult, int style = 0, int nice = 1)
{
    if (want < mult) want = mult;
    if (want >= s) return (int)s;
    if (style == 1) {
        // cache-line friendly: a multiple of `nice` elements (64 bytes) even if that leaves a remainder tile
        const int64_t unit = std::max<int64_t>(nice, mult);
        for (int64_t t = round_up(want, unit); t <= std::min<int64_t>(s, 2 * want); t += unit)
            if (s % t == 0) return (int)t;
        const int64_t t = round_up(want, unit);
        if (t < s) return (int)t;
    }
    for (int64_t t = round_up(want, mult); t <= std::min<int64_t>(s, 2 * want); t += mult)
        if (s % t == 0) return (int)t;
    for (int64_t t = (want / mult) * mult; t >= mult && 4 * t >= 3 * want; t -= mult)
        if (s % t == 0) return (int)t;
    const int64_t parts = ceil_div(s, want);
    int64_t t = round_up(ceil_div(s, parts), mult);
    return (int)std::min<int64_t>(t, s);
}

// Leading indices of one tensor, in that tensor's order, until the contiguous run they
// span reaches `target` elements.  All but the last are taken whole.
static void build_group(const Problem& P, const int* order, int eb, int64_t target, int vec, int max_dims, int* t,
                        int style = 0)
{
    for (int k = 0; k < kMaxDim; ++k) t[k] = 1;
    int64_t run = 1;
    for (int i = 0; i < P.ndim && i < max_dims; ++i) {
        const int k = order[i];
        const int64_t need = ceil_div(target, run);
        if (need <= 1) break;
        const int mult = (i == 0) ? vec : 1;
        int ext;
        if (P.size[k] <= need + need / 2) ext = (int)P.size[k];
        else ext = pick_extent(P.size[k], need, mult, style, std::max(1, 64 / eb));
        t[k] = ext;
        run *= ext;
        if (ext < P.size[k]) break;
    }
}

// ---------------------------------------------------------------------------------
// Walks: how each side sees the box
// ---------------------------------------------------------------------------------
struct DigitSpec {
    int first_dim;      // innermost index of the chain (the stride-1 end)
    int outer_dim;      // outermost index of the chain: the only one the tensor's edge can cut
    int tile;           // flat extent inside the box
    int inner;          // product of the box extents of the chain's inner indices
    int lane;           // flat extent of the lane sub-box (filled by choose_lanes)
};
struct WalkSpec { int nd; DigitSpec d[kBoxDims]; };

// Digits of one walk in the walk's own order.  With `merge`, the leading indices that lie whole
// inside the box fuse with their successor into one flat digit (tile-level index fusion); an
// index whose bit is set in `no_tail` may not be appended to a chain.
static bool build_walk(const Problem& P, const int* order, const int64_t* stride, const int* t, bool merge,
                       unsigned no_tail, WalkSpec* w)
{
    w->nd = 0;
    bool leading = true;
    for (int i = 0; i < P.ndim; ++i) {
        const int k = order[i];
        if (t[k] <= 1) { leading = false; continue; }
        if (merge && leading && w->nd == 1) {
            DigitSpec& d = w->d[0];
            const int prev = d.outer_dim;
            if (i > 0 && order[i - 1] == prev && t[prev] == P.size[prev] && !(no_tail & (1u << k)) &&
                stride[k] == stride[prev] * P.size[prev] && (int64_t)d.tile * t[k] <= kMaxDigitExtent) {
                d.inner = d.tile;
                d.tile *= t[k];
                d.outer_dim = k;
                continue;
            }
        }
        if (w->nd >= 1) leading = false;
        if (w->nd == kBoxDims) return false;
        DigitSpec& d = w->d[w->nd++];
        d.first_dim = d.outer_dim = k;
        d.tile = t[k];
        d.inner = 1;
        d.lane = 1;
        if (t[k] > kMaxDigitExtent) return false;
    }
    return w->nd >= 1;
}

// Largest vector width (elements) for a walk: vectors lie along the first digit and must not
// straddle its end, in whole tiles and in the tiles the tensor's edge cuts.
// A limit above 16 also admits vectors that do not divide the run (*partial = true): the last vector of every
// run is then moved back to end with the run and overlaps its neighbour.  That needs every run, also the
// shortened ones of the tiles the tensor's edge cuts, to hold at least one vector, and pays only for runs of
// several vectors.
static int walk_vec(const Problem& P, const WalkSpec& w, const int* t, int limit, int eb, bool unit_stride,
                    bool* partial)
{
    *partial = false;
    if (!unit_stride) return 1;      // a dropped size-1 index with a padded leading dimension: no stride-1 index
    const int widest = std::max(1, std::min(std::min(limit, 16), std::max(1, 16 / eb)));
    const DigitSpec& d = w.d[0];
    const int64_t rest = P.size[d.outer_dim] % t[d.outer_dim];
    int v = widest;
    while (v > 1 && (d.tile % v != 0 || (rest * d.inner) % v != 0)) v /= 2;
    v = std::max(v, 1);
    if (limit > 16 && v < widest && d.tile >= 4 * widest && (rest == 0 || rest * d.inner >= widest)) {
        *partial = true;
        return widest;
    }
    return v;
}

// Lane mapping: which sub-box of the tile one wavefront instruction covers.
static void choose_lanes(const Problem& P, WalkSpec* w, int vec, int eb, int* n_iter_out, int* lanes_out)
{
    int best_lane[kBoxDims] = {1, 1, 1, 1};
    int64_t best_cost = INT64_MAX;
    int best_iter = 1, best_lanes = 1;
    const int t0 = w->d[0].tile;
    std::vector<int> opts;
    const int cap = (int)std::min<int64_t>(round_up(t0, vec), kWave * vec);
    for (int l = vec; l <= cap; l += vec)
        if (t0 % l == 0 || l == cap) opts.push_back(l);
    if (opts.empty()) opts.push_back(vec);
    for (int l0 : opts) {
        int lane[kBoxDims] = {1, 1, 1, 1};
        lane[0] = l0;
        int lanes = l0 / vec;
        int rem = kWave / std::max(lanes, 1);
        int64_t iters = ceil_div(t0, l0);
        bool ragged = (t0 % l0) != 0;
        for (int i = 1; i < w->nd; ++i) {
            const int ti = w->d[i].tile;
            int l = 1;
            if (rem > 1) {
                l = std::min(rem, ti);
                // prefer a divisor of the extent if it costs at most one position in four
                int div = l;
                while (div > 1 && ti % div != 0) --div;
                if (4 * ceil_div(ti, div) <= 5 * ceil_div(ti, l)) l = div;
                else l = (int)ceil_div(ti, ceil_div(ti, l));      // same count, less ragged
                rem /= l;
                lanes *= l;
            }
            lane[i] = l;
            iters *= ceil_div(ti, l);
            if (ti % l != 0) ragged = true;
        }
        // short segments along the stride-1 index cost coalescing: ask for a 128-byte line unless the tile is
        // shorter; an overhanging sub-box makes every position test its bounds
        const bool short_seg = (l0 < t0) && (l0 * eb < 128);
        const int64_t cost = iters * (short_seg ? 8 : 4) * (ragged ? 5 : 4);
        if (cost < best_cost || (cost == best_cost && l0 > best_lane[0])) {
            best_cost = cost;
            for (int i = 0; i < kBoxDims; ++i) best_lane[i] = lane[i];
            best_iter = (int)std::min<int64_t>(iters, INT32_MAX);
            best_lanes = lanes;
        }
    }
    for (int i = 0; i < w->nd; ++i) w->d[i].lane = best_lane[i];
    *n_iter_out = best_iter;
    *lanes_out = best_lanes;
}

// Lay one walk out for the kernel: digits go to the slot of their outermost index.
static bool fill_side(const Problem& P, const WalkSpec& w, int vec, const int* slot_of_dim,
                      const int* lds_stride, bool follows_b, Side* s)
{
    std::memset(s, 0, sizeof(*s));
    s->vec = vec;
    s->exact = 1;
    for (int j = 0; j < kBoxDims; ++j) {
        Digit& d = s->d[j];
        d.tile = 1; d.lane = 1; d.iters = 1; d.lane_mul = 1; d.slot_mul = 1;
        d.lane_below = d.lane_cnt = d.iter_below = d.iter_cnt = make_fastdiv(1);
    }
    uint32_t lane_below = 1, iter_below = 1;
    int64_t n_iter = 1;
    for (int i = 0; i < w.nd; ++i) {
        const DigitSpec& ds = w.d[i];
        const int j = slot_of_dim[ds.outer_dim];
        if (j < 0 || j >= kBoxDims) return false;
        Digit& d = s->d[j];
        const int mul = (i == 0) ? vec : 1;
        if (ds.lane % mul != 0) return false;
        const int cnt = ds.lane / mul;
        const int its = (int)ceil_div(ds.tile, ds.lane);
        d.tile = ds.tile;
        d.lane = ds.lane;
        d.iters = its;
        d.lane_mul = mul;
        d.slot_mul = ds.inner;
        d.lane_below = make_fastdiv(lane_below);
        d.lane_cnt = make_fastdiv((uint32_t)cnt);
        d.iter_below = make_fastdiv(iter_below);
        d.iter_cnt = make_fastdiv((uint32_t)its);
        d.gstride = follows_b ? P.stride_b[ds.first_dim] : P.stride_a[ds.first_dim];
        d.g2stride = P.stride_b[ds.first_dim];
        d.lstride = lds_stride ? lds_stride[ds.first_dim] : 0;
        d.ragged = (ds.tile % ds.lane != 0) ? 1 : 0;
        if (d.ragged) s->exact = 0;
        lane_below *= (uint32_t)cnt;
        iter_below *= (uint32_t)its;
        n_iter *= its;
        if (n_iter > kMaxIters || lane_below > (uint32_t)kWave) return false;
    }
    s->lanes = (int)lane_below;
    s->n_iter = (int)n_iter;
    s->vec_lds_stride = lds_stride ? lds_stride[w.d[0].first_dim] : 0;
    s->vec_slot = slot_of_dim[w.d[0].outer_dim];
    return true;
}

// ---------------------------------------------------------------------------------
// LDS layout.  Indices that a walk merged into one flat digit must be affine in LDS as well:
// stride(next) = extent(cur) * stride(cur).  These links form chains; the chain holding A's
// stride-1 index comes first, the others follow, each chain head on a small pad chosen by
// simulating which banks the 64 lanes of one LDS instruction touch.
// ---------------------------------------------------------------------------------
// Lane coordinates of one walk, per digit slot, in flat elements: what the bank simulation needs besides the
// LDS strides (computed once per layout search; the strides change from one trial layout to the next).
struct LaneCoords { int lanes, vec; int c[kWave][kBoxDims]; };

static void lane_coords(const Side& s, LaneCoords* out)
{
    out->lanes = s.lanes;
    out->vec = s.vec;
    for (int lane = 0; lane < s.lanes; ++lane)
        for (int i = 0; i < kBoxDims; ++i) {
            const Digit& d = s.d[i];
            out->c[lane][i] = (int)((lane / d.lane_below.div) % d.lane_cnt.div) * d.lane_mul;
        }
}

// Worst number of distinct addresses that the lanes of one LDS instruction send to one bank, relative to the
// unavoidable number (ceil(addresses / banks)), for 32 and for 64 banks; the two are added (2 = conflict-free).
static int bank_multiplicity(const LaneCoords& lc, const int* lstride /* per slot */, int vec_stride, int words)
{
    int worst32 = 1, worst64 = 1;
    int64_t base[kWave], addr[kWave];
    for (int lane = 0; lane < lc.lanes; ++lane) {
        int64_t a = 0;
        for (int i = 0; i < kBoxDims; ++i) a += (int64_t)lc.c[lane][i] * lstride[i];
        base[lane] = a;
    }
    for (int j = 0; j < lc.vec; ++j) {
        int n = lc.lanes;
        for (int lane = 0; lane < n; ++lane) addr[lane] = (base[lane] + (int64_t)j * vec_stride) * words;
        // distinct word addresses per bank (same address = broadcast, no conflict)
        std::sort(addr, addr + n);
        n = (int)(std::unique(addr, addr + n) - addr);
        int cnt32[32] = {0}, cnt64[64] = {0};
        for (int i = 0; i < n; ++i)
            for (int w = 0; w < words; ++w) {
                const uint64_t x = (uint64_t)(addr[i] + w);
                cnt32[x & 31u]++;
                cnt64[x & 63u]++;
            }
        int mx32 = 0, mx64 = 0;
        for (int b = 0; b < 32; ++b) mx32 = std::max(mx32, cnt32[b]);
        for (int b = 0; b < 64; ++b) mx64 = std::max(mx64, cnt64[b]);
        const int ideal32 = std::max(1, (int)ceil_div((int64_t)n * words, 32));
        const int ideal64 = std::max(1, (int)ceil_div((int64_t)n * words, 64));
        worst32 = std::max(worst32, (int)ceil_div(mx32, ideal32));
        worst64 = std::max(worst64, (int)ceil_div(mx64, ideal64));
    }
    return worst32 + worst64;
}

struct LdsLayout { int stride[kMaxDim]; int elems; int conflict_a, conflict_b; };

static LdsLayout choose_lds_layout(const Problem& P, const int* t, const int* slot_of_dim,
                                   const WalkSpec& wa, const WalkSpec& wb, int va, int vb,
                                   const int* next_in_chain /* by dim, -1 = chain end */,
                                   const bool* is_head /* by dim */)
{
    LdsLayout best;
    best.elems = 0; best.conflict_a = best.conflict_b = 1 << 20;
    // chain heads in layout order: the chain of index 0 first, then by index
    int heads[kMaxDim], nh = 0;
    for (int k = 0; k < P.ndim; ++k) if (t[k] > 1 && is_head[k]) heads[nh++] = k;
    // TTC_LDS_PAD=0 in the environment lays every tile out without pads (the ablation of the studies)
    const char* pad_env = std::getenv("TTC_LDS_PAD");
    const bool pads = !(pad_env && pad_env[0] == '0');
    const int npad = pads ? std::max(0, std::min(nh - 1, 3)) : 0;
    // the walks' lane mappings do not depend on the LDS strides: lay the sides out once
    Side sa, sb;
    const int zero[kMaxDim] = {0, 0, 0, 0, 0, 0};
    if (!fill_side(P, wa, va, slot_of_dim, zero, false, &sa)) return best;
    if (!fill_side(P, wb, vb, slot_of_dim, zero, true, &sb)) return best;
    LaneCoords la, lb;
    lane_coords(sa, &la);
    lane_coords(sb, &lb);
    int dim_of_slot_a[kBoxDims] = {-1, -1, -1, -1}, dim_of_slot_b[kBoxDims] = {-1, -1, -1, -1};
    for (int i = 0; i < wa.nd; ++i) dim_of_slot_a[slot_of_dim[wa.d[i].outer_dim]] = wa.d[i].first_dim;
    for (int i = 0; i < wb.nd; ++i) dim_of_slot_b[slot_of_dim[wb.d[i].outer_dim]] = wb.d[i].first_dim;
    const int words = P.eb_a / 4;               // the LDS tile holds elements of A
    int64_t best_cost = INT64_MAX;
    const int combos = 1 << (2 * npad);
    for (int c = 0; c < combos; ++c) {
        LdsLayout L;
        for (int k = 0; k < kMaxDim; ++k) L.stride[k] = 0;
        int64_t run = 1;
        for (int h = 0; h < nh; ++h) {
            if (h >= 1 && h - 1 < npad) run += (c >> (2 * (h - 1))) & 3;
            for (int k = heads[h]; k >= 0; k = next_in_chain[k]) {
                L.stride[k] = (int)run;
                run *= t[k];
            }
        }
        L.elems = (int)run;
        if ((int64_t)L.elems * P.eb_a > kMaxLdsBytes) continue;
        int ls_a[kBoxDims], ls_b[kBoxDims];
        for (int j = 0; j < kBoxDims; ++j) {
            ls_a[j] = dim_of_slot_a[j] >= 0 ? L.stride[dim_of_slot_a[j]] : 0;
            ls_b[j] = dim_of_slot_b[j] >= 0 ? L.stride[dim_of_slot_b[j]] : 0;
        }
        L.conflict_a = bank_multiplicity(la, ls_a, L.stride[wa.d[0].first_dim], words);
        L.conflict_b = bank_multiplicity(lb, ls_b, L.stride[wb.d[0].first_dim], words);
        const int64_t cost = ((int64_t)(L.conflict_a + L.conflict_b) << 24) + L.elems;
        if (cost < best_cost) { best_cost = cost; best = L; }
        if (L.conflict_a + L.conflict_b == 4) break;             // conflict-free under both bank counts
    }
    return best;
}

// ---------------------------------------------------------------------------------
// Candidate assembly
// ---------------------------------------------------------------------------------
// The LDS layout depends on the box and the walks only, not on the launch shape or the tile
// order: candidates that differ only in those share one layout search.
struct LayoutKey {
    int t[kMaxDim]; int vec_limit; bool merge_a, merge_b;
    bool operator==(const LayoutKey& o) const
    {
        for (int k = 0; k < kMaxDim; ++k) if (t[k] != o.t[k]) return false;
        return vec_limit == o.vec_limit && merge_a == o.merge_a && merge_b == o.merge_b;
    }
};
struct LayoutCache { std::vector<std::pair<LayoutKey, LdsLayout>> items; };

static bool make_candidate(const Problem& P, const int* t_in, int vec_limit, bool direct, int threads,
                           int wg_per_cu, const int* tile_order, int xcd_remap, Candidate* out,
                           bool merge_a = true, bool merge_b = true, LayoutCache* cache = nullptr, int nbuf = 2)
{
    Candidate C;
    std::memset(&C, 0, sizeof(C));
    int t[kMaxDim];
    for (int k = 0; k < kMaxDim; ++k) t[k] = (k < P.ndim) ? t_in[k] : 1;
    int order_a[kMaxDim], order_b[kMaxDim];
    for (int k = 0; k < kMaxDim; ++k) { order_a[k] = k; order_b[k] = (k < P.ndim) ? P.perm[k] : k; }

    KernelParams& kp = C.kp;
    kp.n = P.ndim;
    int64_t ntiles = 1;
    for (int k = 0; k < kMaxDim; ++k) {
        kp.stride_a[k] = (k < P.ndim) ? P.stride_a[k] : 0;
        kp.stride_b[k] = (k < P.ndim) ? P.stride_b[k] : 0;
        kp.tile[k] = t[k];
        kp.tile_below[k] = make_fastdiv(1);
        kp.tile_cnt[k] = make_fastdiv(1);
    }
    for (int i = 0; i < P.ndim; ++i) {
        const int k = tile_order[i];
        const int64_t cnt = ceil_div(P.size[k], t[k]);
        if (ntiles > INT32_MAX / 2 || cnt > INT32_MAX / 2) return false;
        kp.tile_below[k] = make_fastdiv((uint32_t)ntiles);
        kp.tile_cnt[k] = make_fastdiv((uint32_t)cnt);
        ntiles *= cnt;
        if (ntiles > INT32_MAX / 2) return false;
        C.tile_order[i] = k;
    }
    kp.num_tiles = (uint32_t)ntiles;
    kp.tiles_per_xcd = kp.num_tiles / 8;
    kp.tiles_rem_xcd = kp.num_tiles % 8;
    if (!set_tile_mapping(&kp, xcd_remap)) return false;
    kp.alpha[0] = P.alpha[0]; kp.alpha[1] = P.alpha[1];
    kp.beta[0] = P.beta[0];   kp.beta[1] = P.beta[1];

    // slots: the indices the box spans, in A order
    int slot_of_dim[kMaxDim];
    int nslots = 0;
    for (int k = 0; k < kMaxDim; ++k) {
        slot_of_dim[k] = -1;
        if (k < P.ndim && t[k] > 1) {
            if (nslots == kBoxDims) return false;
            Slot& sl = kp.slot[nslots];
            sl.tile = t[k];
            sl.size = P.size[k];
            sl.tile_below = kp.tile_below[k];
            sl.tile_cnt = kp.tile_cnt[k];
            slot_of_dim[k] = nslots++;
        }
    }
    for (int j = nslots; j < kBoxDims; ++j) {
        kp.slot[j].tile = 1; kp.slot[j].size = 1;
        kp.slot[j].tile_below = kp.slot[j].tile_cnt = make_fastdiv(1);
    }
    kp.nslots = nslots;
    if (nslots == 0) {                      // a one-element tensor: give the walks one trivial digit
        kp.nslots = 1;
        slot_of_dim[0] = 0;
    }

    for (int k = 0; k < kMaxDim; ++k) { C.tile[k] = t[k]; C.lds_stride[k] = 0; }
    WalkSpec wa, wb;
    auto trivial_walk = [&](WalkSpec* w) {
        w->nd = 1;
        w->d[0].first_dim = w->d[0].outer_dim = 0;
        w->d[0].tile = 1; w->d[0].inner = 1; w->d[0].lane = 1;
    };
    if (direct) {
        if (nslots == 0) trivial_walk(&wa);
        else if (!build_walk(P, order_a, P.stride_a, t, false, 0u, &wa)) return false;
        const int eb_max = std::max(P.eb_a, P.eb_b);        // every lane stores what it loaded: one width for both
        // overlapping vectors would read elements of B that a neighbour may already have updated
        if (P.epilogue == TTC_EPI_AXPBY) vec_limit = std::min(vec_limit, 16);
        bool part = false;
        const int v = (nslots == 0) ? 1 : walk_vec(P, wa, t, vec_limit, eb_max,
                                                  P.stride_a[wa.d[0].first_dim] == 1 && P.stride_b[wa.d[0].first_dim] == 1,
                                                  &part);
        int n_iter, lanes;
        choose_lanes(P, &wa, v, eb_max, &n_iter, &lanes);
        if (!fill_side(P, wa, v, slot_of_dim, nullptr, false, &kp.a)) return false;
        kp.a.partial = part ? 1 : 0;
        kp.b = kp.a;
        wb = wa;
        C.kernel_class = TTC_KERNEL_DIRECT;
        C.lds_bytes = (int)round_up(24 * (int64_t)kp.a.n_iter, 16);
        kp.lds_data_off = C.lds_bytes;
        kp.lds_tile_elems = 0;
        kp.lds_buffers = 1;
        C.lds_conflict_a = C.lds_conflict_b = 0;
    } else {
        if (nslots == 0) return false;
        if (!build_walk(P, order_a, P.stride_a, t, merge_a, 0u, &wa)) return false;
        // LDS chains from A's merged digit; B may chain its own leading indices only where that
        // does not give an index a second predecessor or a second successor
        int next_in_chain[kMaxDim];
        bool is_head[kMaxDim];
        unsigned in_a_chain = 0, a_nonlast = 0;
        for (int k = 0; k < kMaxDim; ++k) { next_in_chain[k] = -1; is_head[k] = true; }
        if (wa.d[0].first_dim != wa.d[0].outer_dim)
            for (int k = wa.d[0].first_dim; k <= wa.d[0].outer_dim; ++k) {      // A's chain is consecutive indices
                in_a_chain |= 1u << k;
                if (k < wa.d[0].outer_dim) { next_in_chain[k] = k + 1; is_head[k + 1] = false; a_nonlast |= 1u << k; }
            }
        const bool b_may_merge = merge_b && !(a_nonlast & (1u << order_b[0]));
        if (!build_walk(P, order_b, P.stride_b, t, b_may_merge, in_a_chain, &wb)) return false;
        if (wb.d[0].first_dim != wb.d[0].outer_dim) {
            int prev = -1;
            for (int i = 0; i < P.ndim; ++i) {
                const int k = order_b[i];
                if (prev >= 0) { next_in_chain[prev] = k; is_head[k] = false; }
                prev = k;
                if (k == wb.d[0].outer_dim) break;
            }
        }
        bool part_a = false, part_b = false;
        const int va = walk_vec(P, wa, t, vec_limit, P.eb_a, P.stride_a[wa.d[0].first_dim] == 1, &part_a);
        const int vb = walk_vec(P, wb, t, P.epilogue == TTC_EPI_AXPBY ? std::min(vec_limit, 16) : vec_limit, P.eb_b,
                                P.stride_b[wb.d[0].first_dim] == 1, &part_b);     // see the direct case
        int ia, la_, ib, lb_;
        choose_lanes(P, &wa, va, P.eb_a, &ia, &la_);
        choose_lanes(P, &wb, vb, P.eb_b, &ib, &lb_);
        LdsLayout L;
        bool cached = false;
        LayoutKey key;
        for (int k = 0; k < kMaxDim; ++k) key.t[k] = t[k];
        key.vec_limit = vec_limit; key.merge_a = merge_a; key.merge_b = merge_b;
        if (cache)
            for (const auto& it : cache->items) if (it.first == key) { L = it.second; cached = true; break; }
        if (!cached) {
            L = choose_lds_layout(P, t, slot_of_dim, wa, wb, va, vb, next_in_chain, is_head);
            if (cache) cache->items.emplace_back(key, L);
        }
        if (L.elems == 0) return false;
        for (int k = 0; k < kMaxDim; ++k) C.lds_stride[k] = L.stride[k];
        if (!fill_side(P, wa, va, slot_of_dim, L.stride, false, &kp.a)) return false;
        if (!fill_side(P, wb, vb, slot_of_dim, L.stride, true, &kp.b)) return false;
        kp.a.partial = part_a ? 1 : 0;
        kp.b.partial = part_b ? 1 : 0;
        C.kernel_class = TTC_KERNEL_LDS;
        kp.lds_data_off = (int)round_up(24 * (int64_t)(kp.a.n_iter + kp.b.n_iter), 16);
        kp.lds_tile_elems = (int)round_up(L.elems, std::max(1, 16 / P.eb_a));
        kp.lds_buffers = nbuf;
        C.lds_bytes = kp.lds_data_off + nbuf * kp.lds_tile_elems * P.eb_a;
        if (C.lds_bytes > kMaxLdsBytes) return false;
        C.lds_conflict_a = L.conflict_a;
        C.lds_conflict_b = L.conflict_b;
    }
    C.digits_a = wa.nd;
    C.digits_b = wb.nd;
    for (int i = 0; i < kBoxDims; ++i) {
        C.dtile_a[i] = i < wa.nd ? wa.d[i].tile : 0;  C.dlane_a[i] = i < wa.nd ? wa.d[i].lane : 0;
        C.dtile_b[i] = i < wb.nd ? wb.d[i].tile : 0;  C.dlane_b[i] = i < wb.nd ? wb.d[i].lane : 0;
    }
    C.threads = threads;
    const int nwave = threads / kWave;
    auto set_chunks = [&](Side* sd) {
        sd->chunk = (int)ceil_div(sd->n_iter, nwave);
        sd->chunk_rem = sd->n_iter - (sd->chunk - 1) * nwave;
        sd->chunk_div = make_fastdiv((uint32_t)sd->chunk);
    };
    set_chunks(&kp.a);
    set_chunks(&kp.b);
    const int64_t tab_entries = (int64_t)nwave * (kp.a.chunk + (direct ? 0 : kp.b.chunk));
    const int tab_bytes = (int)round_up(kTablesOff + 24 * tab_entries, 16);
    C.lds_bytes += tab_bytes - kp.lds_data_off;
    kp.lds_data_off = tab_bytes;
    if (C.lds_bytes > kMaxLdsBytes) return false;
    // wg_per_cu <= 0: as many workgroups as a compute unit holds at once (LDS in granules of 1280 bytes, 32
    // wavefronts, 16 workgroups that need a barrier), so that every workgroup is resident from the start and its
    // set-up is paid once per slot instead of once per round
    if (wg_per_cu <= 0) {
        const int by_lds = (int)(kMaxLdsBytes / round_up(std::max(C.lds_bytes, 1), 1280));
        const int by_waves = 32 / nwave;
        wg_per_cu = std::max(1, std::min(std::min(by_lds, by_waves), nwave > 1 ? 16 : 32));
    }
    C.wg_per_cu = wg_per_cu;
    set_grid(&kp, launch_grid(C, 256));
    C.tuned_ms = 0.f;
    *out = C;
    return true;
}

// The micro-tile kernel's candidate: a tile of ta columns x tb rows.  The column index is A's index 0, or A's
// indices 0 and 1 taken as one (merge_a: together they are one contiguous run of A); the row index is B's
// stride-1 index p0, or B's first two indices taken as one (merge_b).  Needs one element type of 4 or 8 bytes on
// both sides, indices contiguous in their tensor, four different indices where both sides merge, both (merged)
// extents at least one 16-byte vector, ta and tb multiples of the vector, a tile of at most 64 KB.  Extents that
// are not multiples of the vector make some elements be moved twice; where B is updated (beta != 0) the kernel
// writes such an element once, from the block that owns it.
static bool make_micro_candidate(const Problem& P, int ta, int tb, int threads, const int* tile_order, bool merge_a, bool merge_b,
                                 Candidate* out)
{
    if (P.ndim < 2 || P.perm[0] == 0 || P.kind_a != P.kind_b || (P.eb_a != 4 && P.eb_a != 8)) return false;
    const int p0 = P.perm[0], vec = 16 / P.eb_a;
    const int a1 = 1, p1 = P.ndim >= 2 ? P.perm[1] : -1;         // the second index of A and of B
    if (P.stride_a[0] != 1 || P.stride_b[p0] != 1) return false;
    if (merge_a && (P.ndim < 3 || a1 == p0 || P.stride_a[a1] != P.size[0] || (merge_b && a1 == p1))) return false;
    if (merge_b && (P.ndim < 3 || p1 == 0 || P.stride_b[p1] != P.size[p0] || (merge_a && p1 == a1))) return false;
    const int64_t cols = merge_a ? P.size[0] * P.size[a1] : P.size[0], rows = merge_b ? P.size[p0] * P.size[p1] : P.size[p0];
    if (cols >= (int64_t(1) << 31) || rows >= (int64_t(1) << 31)) return false;
    if (cols < vec || rows < vec || ta % vec != 0 || tb % vec != 0 || ta < vec || tb < vec) return false;
    const int la = ta / vec, lb = tb / vec;
    const int pitch = (la + 7) / 8 * 8;
    if ((int64_t)tb * pitch * 16 > 64 * 1024) return false;
    const int loads = (int)ceil_div((int64_t)la * tb, threads), blocks = (int)ceil_div((int64_t)la * lb, threads);
    if (blocks > 8) return false;
    Candidate C;
    std::memset(&C, 0, sizeof(C));
    C.kernel_class = TTC_KERNEL_MICRO;
    C.threads = threads;
    C.wg_per_cu = 0;                   // one tile per workgroup
    C.lds_bytes = tb * pitch * 16;
    KernelParams& kp = C.kp;
    kp.n = P.ndim;
    int64_t ntiles = 1;
    // what the tile decode sees: the (merged) column index in the place of index 0, the row index in the place of
    // p0, an index merged into one of them as a single tile that contributes nothing, every other index one
    // element per tile.  The decode adds the column's place in A and the row's place in B (stride 1); where the
    // column lies in B and the row in A depends on more than a stride and is left to the kernel.
    int64_t extent[kMaxDim];
    for (int k = 0; k < kMaxDim; ++k) {
        extent[k] = (k < P.ndim) ? P.size[k] : 1;
        C.tile[k] = 1;
        kp.stride_a[k] = (k < P.ndim) ? P.stride_a[k] : 0;
        kp.stride_b[k] = (k < P.ndim) ? P.stride_b[k] : 0;
        kp.tile_below[k] = kp.tile_cnt[k] = make_fastdiv(1);
    }
    extent[0] = cols; C.tile[0] = ta; kp.stride_a[0] = 1; kp.stride_b[0] = 0;
    extent[p0] = rows; C.tile[p0] = tb; kp.stride_a[p0] = 0; kp.stride_b[p0] = 1;
    if (merge_a) { extent[a1] = 1; kp.stride_a[a1] = kp.stride_b[a1] = 0; }
    if (merge_b) { extent[p1] = 1; kp.stride_a[p1] = kp.stride_b[p1] = 0; }
    for (int k = 0; k < kMaxDim; ++k) kp.tile[k] = C.tile[k];
    uint32_t ordered = 0;                        // the order has to name every index of the problem once
    for (int i = 0; i < P.ndim; ++i) if (tile_order[i] >= 0 && tile_order[i] < P.ndim) ordered |= 1u << tile_order[i];
    if (ordered != (1u << P.ndim) - 1u) return false;
    for (int i = 0; i < P.ndim; ++i) {
        const int k = tile_order[i];
        const int64_t cnt = ceil_div(extent[k], C.tile[k]);
        if (cnt > INT32_MAX / 2 || ntiles > INT32_MAX / 2) return false;
        kp.tile_below[k] = make_fastdiv((uint32_t)ntiles);
        kp.tile_cnt[k] = make_fastdiv((uint32_t)cnt);
        ntiles *= cnt;
        if (ntiles > INT32_MAX / 2) return false;
        C.tile_order[i] = k;
    }
    kp.num_tiles = (uint32_t)ntiles;
    kp.tiles_per_xcd = kp.num_tiles / 8;
    kp.tiles_rem_xcd = kp.num_tiles % 8;
    if (!set_tile_mapping(&kp, kDefaultTileMapping)) return false;
    set_grid(&kp, kp.num_tiles);
    kp.alpha[0] = P.alpha[0]; kp.alpha[1] = P.alpha[1];
    kp.beta[0] = P.beta[0];   kp.beta[1] = P.beta[1];
    kp.a.vec = kp.b.vec = vec;
    kp.lds_buffers = 1;
    kp.lds_tile_elems = ta * tb;
    for (int j = 0; j < kBoxDims; ++j) {            // the box kernels' slots, so that shared helpers see neutral values
        kp.slot[j].tile = 1; kp.slot[j].size = 1;
        kp.slot[j].tile_below = kp.slot[j].tile_cnt = make_fastdiv(1);
    }
    MicroParams& m = kp.micro;
    m.ta = ta; m.tb = tb; m.p0 = p0; m.vec = vec;
    m.merged_a = merge_a ? 1 : 0; m.merged_b = merge_b ? 1 : 0;
    m.la = la; m.lb = lb; m.pitch = pitch; m.loads = loads; m.blocks = blocks;
    {   // TTC_LDS_PAD=0 in the environment: no swizzle either (the ablation of the studies)
        const char* pad_env = std::getenv("TTC_LDS_PAD");
        m.swizzle = (pad_env && pad_env[0] == '0') ? 0u : 7u;
    }
    m.la_div = make_fastdiv((uint32_t)la); m.lb_div = make_fastdiv((uint32_t)lb);
    m.vec_log = (vec == 4) ? 2 : 1;
    m.size_a0 = cols; m.size_p0 = rows;
    m.col_in_div = make_fastdiv((uint32_t)P.size[0]);
    m.row_in_div = make_fastdiv((uint32_t)P.size[p0]);
    m.col_b_in = P.stride_b[0];  m.col_b_out = merge_a ? P.stride_b[a1] : 0;
    m.row_a_in = P.stride_a[p0]; m.row_a_out = merge_b ? P.stride_a[p1] : 0;
    // the tile per index of A, as the plan reports it: a merged index takes what the tile spans of it
    if (merge_a) { C.tile[0] = (int)std::min<int64_t>(ta, P.size[0]); C.tile[a1] = (int)std::min<int64_t>(ceil_div(ta, P.size[0]), P.size[a1]); }
    if (merge_b) { C.tile[p0] = (int)std::min<int64_t>(tb, P.size[p0]); C.tile[p1] = (int)std::min<int64_t>(ceil_div(tb, P.size[p0]), P.size[p1]); }
    C.digits_a = C.digits_b = 2;
    C.dtile_a[0] = ta; C.dtile_a[1] = tb; C.dlane_a[0] = std::min(ta, kWave * vec); C.dlane_a[1] = std::max(1, kWave / la);
    C.dtile_b[0] = tb; C.dtile_b[1] = ta; C.dlane_b[0] = std::min(tb, kWave * vec); C.dlane_b[1] = std::max(1, kWave / lb) * vec;
    C.dlane_a[2] = m.merged_a; C.dlane_b[2] = m.merged_b;       // part of what names the configuration
    C.lds_conflict_a = C.lds_conflict_b = 2;       // conflict-free by construction (the value the bank model gives such a layout)
    C.lds_stride[0] = 1;
    C.lds_stride[p0] = pitch * vec;
    *out = C;
    return true;
}

// The micro-tile kernel's argument block from a candidate as it stands (tile mapping, streaming hints and grid are
// the plan's current ones).
MicroArgs micro_args(const Candidate& c)
{
    const KernelParams& kp = c.kp;
    MicroArgs a;
    std::memset(&a, 0, sizeof(a));
    a.xcd_remap = kp.xcd_remap;
    a.num_tiles = kp.num_tiles; a.tiles_per_xcd = kp.tiles_per_xcd; a.tiles_rem_xcd = kp.tiles_rem_xcd;
    a.grid = kp.grid; a.grid_per_xcd = kp.grid_per_xcd; a.grid_rem_xcd = kp.grid_rem_xcd;
    for (int x = 0; x < 8; ++x) a.xcd_tiles[x] = kp.xcd_tiles[x];
    a.nt_a = kp.nt_a; a.nt_b = kp.nt_b;
    a.debug_stop = 0;
    a.col_pos = a.row_pos = -1;
    for (int i = 0; i < kMaxDim; ++i) {
        a.cnt[i] = make_fastdiv(1);
        a.step_a[i] = a.step_b[i] = 0;
    }
    for (int i = 0; i < kp.n && i < kMaxDim; ++i) {
        const int k = c.tile_order[i];
        a.cnt[i] = kp.tile_cnt[k];
        a.step_a[i] = (int64_t)kp.tile[k] * kp.stride_a[k];
        a.step_b[i] = (int64_t)kp.tile[k] * kp.stride_b[k];
        if (k == 0) a.col_pos = i;
        if (k == kp.micro.p0) a.row_pos = i;
    }
    a.alpha[0] = kp.alpha[0]; a.alpha[1] = kp.alpha[1];
    a.beta[0] = kp.beta[0];   a.beta[1] = kp.beta[1];
    a.micro = kp.micro;
    return a;
}

// The row kernel's candidate: B walked front to back, `vec` elements per lane and access.  Needs rows that are
// contiguous in both tensors and hold at least one vector, fewer than 2^31 rows, rows shorter than 2^30.
static bool make_rows_candidate(const Problem& P, int vec, int unroll, Candidate* out)
{
    if (P.perm[0] != 0 || P.stride_a[0] != 1 || P.stride_b[0] != 1) return false;
    const int64_t row = P.size[0], rows = P.elements / P.size[0];
    if (row < vec || row >= (int64_t(1) << 30) || rows >= (int64_t(1) << 31)) return false;
    // rows that are not a multiple of the vector: their last vector overlaps its neighbour, which is only
    // harmless where B is not read
    if (row % vec != 0 && P.epilogue == TTC_EPI_AXPBY) return false;
    Candidate C;
    std::memset(&C, 0, sizeof(C));
    C.kernel_class = TTC_KERNEL_ROWS;
    C.threads = 256;
    C.wg_per_cu = 0;                   // one-shot workgroups: nothing to choose
    C.lds_bytes = 0;
    RowsParams& r = C.rows;
    r.n = P.ndim;
    r.vec = vec;
    r.unroll = unroll;
    r.row = (uint32_t)row;
    r.slots = (uint32_t)ceil_div(row, vec);
    r.chunk = (uint32_t)(C.threads * r.unroll);
    r.overlap = (row % vec != 0) ? 1 : 0;
    r.slot_div = make_fastdiv(r.slots);
    r.vectors = rows * (int64_t)r.slots;
    for (int d = 0; d < kMaxDim; ++d) {
        r.size_div[d] = make_fastdiv(1);
        r.stride_a[d] = 0;
        r.stride_b[d] = 0;
        if (d >= 1 && d < P.ndim) {
            const int k = P.perm[d];                       // B's index d is A's index k
            r.size_div[d] = make_fastdiv((uint32_t)P.size[k]);
            r.stride_a[d] = P.stride_a[k];
            r.stride_b[d] = P.stride_b[k];
        }
    }
    r.alpha[0] = P.alpha[0]; r.alpha[1] = P.alpha[1];
    r.beta[0] = P.beta[0];   r.beta[1] = P.beta[1];
    // what the other kernels' fields say about this one
    KernelParams& kp = C.kp;
    kp.n = P.ndim;
    kp.a.vec = vec; kp.b.vec = vec;
    kp.lds_buffers = 1;
    const int64_t grid = ceil_div(r.vectors, r.chunk);
    if (grid > INT32_MAX / 2) return false;
    kp.a.partial = kp.b.partial = r.overlap;
    kp.num_tiles = (uint32_t)grid;
    kp.grid = (uint32_t)grid;
    for (int k = 0; k < kMaxDim; ++k) {
        C.tile[k] = (k == 0) ? (int)row : 1;
        C.tile_order[k] = (k < P.ndim) ? P.perm[k] : k;
        kp.tile[k] = C.tile[k];
        kp.tile_below[k] = kp.tile_cnt[k] = make_fastdiv(1);
        kp.stride_a[k] = (k < P.ndim) ? P.stride_a[k] : 0;
        kp.stride_b[k] = (k < P.ndim) ? P.stride_b[k] : 0;
    }
    C.digits_a = C.digits_b = 1;
    C.dtile_a[0] = C.dtile_b[0] = (int)row;
    C.dlane_a[0] = C.dlane_b[0] = (int)std::min<int64_t>(row, (int64_t)kWave * vec);
    *out = C;
    return true;
}

bool set_tile_mapping(KernelParams* kp, int mode)
{
    if (mode == kDefaultTileMapping) {
        mode = kp->num_tiles >= 2048u ? 5 : 0;      // few tiles (a workgroup gets one or two): round robin spreads them best
    }
    if (mode < 0 || mode > 10) return false;
    kp->xcd_remap = mode;
    for (int x = 0; x < 8; ++x) kp->xcd_tiles[x] = 0;
    if (mode >= 2) {
        const uint32_t C = 1u << mode;
        const uint32_t chunks = (kp->num_tiles + C - 1) / C;             // the last one may be partial
        for (uint32_t x = 0; x < 8; ++x) {
            const uint32_t mine = chunks > x ? (chunks - x + 7) / 8 : 0;
            kp->xcd_tiles[x] = mine * C;
            if (mine > 0 && (chunks - 1) % 8 == x) kp->xcd_tiles[x] -= chunks * C - kp->num_tiles;
        }
    }
    return true;
}

uint32_t launch_grid(const Candidate& c, int cus)
{
    if (c.kernel_class == TTC_KERNEL_MICRO || c.kernel_class == TTC_KERNEL_ROWS) return c.kp.num_tiles;    // one-shot workgroups
    const uint64_t want = (uint64_t)std::max(cus, 1) * (uint64_t)std::max(c.wg_per_cu, 1);
    return (uint32_t)std::min<uint64_t>(want, c.kp.num_tiles);
}

void set_grid(KernelParams* kp, uint32_t grid)
{
    kp->grid = grid;
    kp->grid_per_xcd = grid / 8;
    kp->grid_rem_xcd = grid % 8;
}

// Heuristic cost of a candidate (smaller is better).  It plays the role of the paper's cost
// estimate that admits candidates to the bounded queue; the paper does not define one, this
// one prices coalescing (length and alignment of the contiguous runs on both sides),
// remainder tiles, tile size, lane use and vector width.
// How a candidate touches memory, in bytes per side: the contiguous run the tile spans, the
// contiguous piece one wavefront instruction covers, and the power of two (up to 128) that
// divides the byte offset of every run start.
struct AccessShape { int run[2], seg[2], align[2]; };

static int segment_elems(const Side& s, bool second)
{
    struct Item { int64_t stride; int lane, tile; } it[kBoxDims];
    int n = 0;
    for (int j = 0; j < kBoxDims; ++j)
        if (s.d[j].tile > 1) { it[n].stride = second ? s.d[j].g2stride : s.d[j].gstride; it[n].lane = s.d[j].lane; it[n].tile = s.d[j].tile; ++n; }
    std::sort(it, it + n, [](const Item& x, const Item& y) { return x.stride < y.stride; });
    int64_t seg = 1, expect = 1;
    for (int i = 0; i < n; ++i) {
        if (it[i].stride != expect) break;
        seg *= it[i].lane;
        if (it[i].lane < it[i].tile) break;
        expect = it[i].stride * it[i].tile;
    }
    return (int)std::min<int64_t>(seg, 1 << 20);
}

static AccessShape access_shape(const Problem& P, const Candidate& C)
{
    AccessShape r;
    const bool direct = (C.kernel_class == TTC_KERNEL_DIRECT);
    for (int side = 0; side < 2; ++side) {
        int order[kMaxDim];
        for (int k = 0; k < kMaxDim; ++k) order[k] = side ? ((k < P.ndim) ? P.perm[k] : k) : k;
        const int64_t* stride = side ? P.stride_b : P.stride_a;
        const int eb = side ? P.eb_b : P.eb_a;
        int64_t run = 1, g = 0;
        bool open = true;
        for (int i = 0; i < P.ndim; ++i) {
            const int k = order[i];
            if (open && stride[k] != run) open = false;
            if (open) {
                run *= C.kp.tile[k];
                if (C.kp.tile[k] < P.size[k]) open = false;
            } else if (P.size[k] > 1) {
                int64_t a = stride[k] * eb, b = g;
                while (b) { const int64_t t = a % b; a = b; b = t; }
                g = a;
            }
        }
        int64_t a = run * eb, b = g;
        while (b) { const int64_t t = a % b; a = b; b = t; }
        int al = 1;
        while (al < 128 && a % (2 * al) == 0) al *= 2;
        r.run[side] = (int)std::min<int64_t>(run * eb, INT32_MAX);
        r.align[side] = al;
        const Side& s = (side && !direct) ? C.kp.b : C.kp.a;
        r.seg[side] = segment_elems(s, side && direct) * eb;
    }
    return r;
}

// The row kernel against the tiled kernels: measured on 384^3, 376^3, 374^3 (0,2,1) and 4-D to 6-D problems with
// the stride-1 index fixed (fp32, fp64, complex64).  Long rows gathered whole are what it is good at (87-94 % of a
// copy where the tiled kernels reach 75-90 %); short rows leave it with sub-line pieces of A that a tile spanning
// A's next index reads as one run (53-62 % against 71-81 %).
static double rows_cost(const Problem& P, const Candidate& C)
{
    const double row_bytes = (double)P.size[0] * P.eb_a;
    auto oct_below = [](double x, double ref) { return x < ref ? std::log2(ref / x) : 0.0; };
    double e = -0.30;
    e += 0.60 * oct_below(row_bytes, 512.0);                            // 576-byte rows: 94 % of a copy; 340-byte rows: 62 %
    if (std::fmod(row_bytes, 128.0) != 0.0) e += 0.04;                  // rows that share lines with their neighbours
    if (C.rows.overlap) e += 0.02;                                      // the last vector of every row repeats part of its neighbour
    // Access width and bytes a lane keeps in flight (loads of B count when beta != 0), measured on 384^3, 374^3,
    // 917x374x153, 208x115x63x35 and 72^4 fp64: 16-byte accesses with 16 to 32 bytes in flight reach 94-97 % of a
    // copy (4 to 8 KB per workgroup); every doubling beyond costs about 4 %, 8 bytes in flight reach 70 %,
    // 8-byte accesses trail 16-byte ones by 5 %, 4-byte accesses stop at 62 %.
    const int access = C.rows.vec * std::max(P.eb_a, P.eb_b);
    if (access < 8) e += 0.40;
    else if (access < 16) e += 0.05;
    const double in_flight = (double)access * C.rows.unroll * (P.epilogue == TTC_EPI_AXPBY ? 2.0 : 1.0);
    if (in_flight > 32.0) e += 0.045 * std::log2(in_flight / 32.0);
    if (in_flight < 16.0) e += 0.30 * std::log2(16.0 / in_flight);
    // small problems: a chunk is 4 to 32 KB, and too few of them leave compute units idle (the same guard rails as for tiles)
    const double tiles_wanted = std::min(2048.0, std::max(1.0, (double)P.elements * P.eb_a / 8192.0));
    if (C.kp.num_tiles < tiles_wanted) e += 1.28 * (tiles_wanted - C.kp.num_tiles) / 2048.0;
    const double cus_wanted = std::min(256.0, std::max(1.0, (double)P.elements * P.eb_a / 4096.0));
    if (C.kp.num_tiles < cus_wanted) e += 1.5 * (cus_wanted - C.kp.num_tiles) / 256.0;
    return std::exp(e);
}

// The micro-tile kernel's ranking model: log-linear like the box kernels' below, with the family's own features
// (it has no tables, no barriers per walk, no bank conflicts).  Weights fitted to the timings of every micro-tile
// candidate of 68 problems (the 57-case benchmark and the search study's 30, the suite included; weighted least
// squares, penalties constrained to be penalties, checked by holding problems out: the first candidate reaches
// 93.8 % of the family's best on problems the fit has not seen, the first ten 98.5 %) and rounded; the offset
// against the box kernels' model is the one that makes the first candidate of the joint ranking best on the same
// problems.  Guard rails for small problems as below.
static double micro_cost(const Problem& P, const Candidate& C)
{
    auto below = [](double x, double ref) { return x < ref ? std::log2(ref / x) : 0.0; };
    auto above = [](double x, double ref) { return x > ref ? std::log2(x / ref) : 0.0; };
    const MicroParams& m = C.kp.micro;
    const double run_a = (double)m.ta * P.eb_a, run_b = (double)m.tb * P.eb_a;
    const int64_t line = 128 / P.eb_a;
    const bool un_a = m.size_a0 % line != 0 || m.ta % line != 0;          // runs of A start inside lines
    const bool un_b = m.size_p0 % line != 0 || m.tb % line != 0;
    double e = -0.22;
    e += 0.05 * below(run_a, 128.0) + 0.012 * below(run_b, 128.0);
    e += -0.01 * above(run_a, 1024.0) - 0.03 * above(run_b, 1024.0);
    const double padded = ((double)ceil_div(m.size_a0, m.ta) * m.ta / (double)m.size_a0) *
                          ((double)ceil_div(m.size_p0, m.tb) * m.tb / (double)m.size_p0);
    e += 0.11 * (padded - 1.0);                                          // idle lanes in the remainder tiles
    if (un_a) e += 0.028 * below(run_a, 512.0);                          // the shorter the run, the larger the share of split lines
    if (un_b) e += 0.072 * below(run_b, 512.0);
    if (C.threads == 128) e += 0.04; else if (C.threads == 64) e += 0.068;
    bool b_order = true;
    for (int i = 0; i < P.ndim; ++i) if (C.tile_order[i] != P.perm[i]) b_order = false;
    if (!b_order) e += 0.054;
    e += 0.009 * std::log2((double)std::max(1, m.blocks));
    e += 0.114 * (double)C.lds_bytes / 65536.0;                          // fewer workgroups per compute unit
    if (m.merged_a) e += 0.006;
    if (m.merged_b) e += 0.011;
    e += 0.27 * (1.0 - (double)m.la * m.lb / ((double)m.blocks * C.threads));   // lanes without a block
    const double tiles_wanted = std::min(2048.0, std::max(1.0, (double)P.elements * P.eb_a / 8192.0));
    if (C.kp.num_tiles < tiles_wanted) e += 1.28 * (tiles_wanted - C.kp.num_tiles) / 2048.0;
    const double cus_wanted = std::min(256.0, std::max(1.0, (double)P.elements * P.eb_a / 4096.0));
    if (C.kp.num_tiles < cus_wanted) e += 1.5 * (cus_wanted - C.kp.num_tiles) / 256.0;
    return std::exp(e);
}

static double heuristic_cost(const Problem& P, const Candidate& C)
{
    if (C.kernel_class == TTC_KERNEL_ROWS) return rows_cost(P, C);
    if (C.kernel_class == TTC_KERNEL_MICRO) return micro_cost(P, C);
    // Weights fitted to timings of every candidate of 105 problems on MI355X (the benchmark workloads, 3-D and
    // 5-D problems with odd extents, a 57-case benchmark drawn by the paper's rules, power-of-two shapes): log-linear least
    // squares weighted towards the fast candidates, penalties constrained to be penalties, a small ridge term,
    // checked by holding problems out; rounded, with guard rails outside the measured range (runs under 64
    // bytes, small problems).
    const KernelParams& kp = C.kp;
    const double eb_a = P.eb_a, eb_b = P.eb_b;
    const bool direct = (C.kernel_class == TTC_KERNEL_DIRECT);
    const bool reads_b = (P.epilogue == TTC_EPI_AXPBY);
    auto oct_below = [](double x, double ref) { return x < ref ? std::log2(ref / x) : 0.0; };
    double volume = 1, padded = 1;
    for (int k = 0; k < P.ndim; ++k) {
        volume *= kp.tile[k];
        padded *= (double)ceil_div(P.size[k], kp.tile[k]) * kp.tile[k] / (double)P.size[k];
    }
    const double tile_bytes = volume * eb_a;
    const AccessShape sh = access_shape(P, C);
    const double run_a = sh.run[0], run_b = sh.run[1], seg_a = sh.seg[0], seg_b = sh.seg[1];
    const int vec_b = direct ? kp.a.vec : kp.b.vec;
    bool b_order = true, a_order = true;
    for (int i = 0; i < P.ndim; ++i) {
        if (C.tile_order[i] != P.perm[i]) b_order = false;
        if (C.tile_order[i] != i) a_order = false;
    }
    const bool order_a = !b_order && a_order, order_mixed = !b_order && !a_order;
    double e = 0.0;
    // coalescing: the contiguous run per tile and the contiguous piece per wavefront instruction; where runs
    // are whole lines their length counts for more (nothing is shared with a neighbour that could hide it)
    e += 0.002 * oct_below(run_a, 1024.0) + 0.016 * oct_below(run_b, 1024.0);
    e += 0.15 * oct_below(run_a, 64.0) + 0.20 * oct_below(run_b, 64.0);
    e += 0.015 * oct_below(seg_a, 256.0) + 0.025 * oct_below(seg_b, 256.0);
    e += 0.066 * oct_below(seg_a, 64.0) + 0.10 * oct_below(seg_b, 64.0);
    if (sh.align[0] >= 128) e += 0.026 * oct_below(run_a, 1024.0) - 0.004 * oct_below(run_a, 256.0);
    if (sh.align[1] >= 128) e += 0.007 * oct_below(run_b, 2048.0);
    // runs that start or end inside a line: lines_shared = what a run shares with its neighbours per 128
    // bytes it moves; requests = line (A) or 64-byte write (B) requests per line or 64 bytes moved, minus one.
    // On the B side both cost more when the tiles that share the line run far apart in time (tile ids in
    // A's order).
    const double lines_shared_a = (1.0 - sh.align[0] / 128.0) * 128.0 / run_a;
    const double requests_a = ((run_a + 128.0 - std::min(sh.align[0], 128)) / 128.0) * 128.0 / run_a - 1.0;
    const double lines_shared = (1.0 - sh.align[1] / 128.0) * 128.0 / run_b;
    const double requests = ((run_b + 64.0 - std::min(sh.align[1], 64)) / 64.0) * 64.0 / run_b - 1.0;
    e += 0.014 * lines_shared_a + 0.014 * requests_a + 0.0705 * requests;
    if (order_a) e += 0.002 + 0.065 * lines_shared + 0.124 * requests;
    if (order_mixed) e += -0.010 + 0.021 * lines_shared;
    e -= 0.0568 * (kp.nt_a + kp.nt_b);                                  // sides that stream (whole lines only)
    e += (kp.a.vec * eb_a >= 16 ? 0.0 : (kp.a.vec * eb_a >= 8 ? 0.037 : 0.057));
    e += (vec_b * eb_b >= 8 ? 0.0 : 0.005);
    if (!direct && kp.b.partial) e -= 0.016;
    e += 0.214 * (padded - 1.0);                                        // lanes idle in remainder tiles
    // tile size and occupancy
    e += 0.2035 * oct_below(tile_bytes, 8192.0);
    if (tile_bytes > 16384.0) e -= 0.0626 * std::log2(tile_bytes / 16384.0);
    if (tile_bytes > 32768.0) e += 0.0629 * std::log2(tile_bytes / 32768.0);
    const double lane_a = (double)kp.a.n_iter * kWave * kp.a.vec / volume;
    e += 0.052 * (lane_a - 1.0);
    double groups = 16.0, resident_waves = 32.0;
    if (direct) {
        // no regrouping through LDS: every instruction's piece meets memory as it is
        e += 0.0436 + 0.0555 * ((1.0 - sh.align[0] / 128.0) * 128.0 / seg_a + (1.0 - sh.align[1] / 128.0) * 128.0 / seg_b);
    } else {
        groups = std::min(16.0, std::floor(160.0 * 1024 / C.lds_bytes));
        resident_waves = std::min(32.0, groups * (C.threads / kWave));
        if (kp.lds_buffers == 1) e += reads_b ? 0.005 : 0.002;
        const double lane_b = (double)kp.b.n_iter * kWave * kp.b.vec / volume;
        e += 0.006 * (lane_b - 1.0);
    }
    if (resident_waves < 16.0) e += 0.233 * (16.0 - resident_waves) / 16.0;
    if (resident_waves < 8.0) e += 0.277 * (8.0 - resident_waves) / 8.0;
    if (groups < 4.0) e += 0.061 * (4.0 - groups) / 4.0;
    // launch shape: measured preference
    if (C.threads == 128) e -= reads_b ? 0.0744 : 0.0259;
    else if (C.threads == 512) e += 0.0285;
    if (C.wg_per_cu == 4) e += 0.022;
    else if (C.wg_per_cu == 8) e += 0.0225;
    // too few tiles to fill the chip (a problem too small for 2048 tiles of 8 KB is not pushed below 8 KB)
    const double tiles_wanted = std::min(2048.0, std::max(1.0, (double)P.elements * eb_a / 8192.0));
    if (kp.num_tiles < tiles_wanted) e += 1.28 * (tiles_wanted - kp.num_tiles) / 2048.0;
    // small problems (outside the fitted range): a tile per compute unit comes before large tiles
    const double cus_wanted = std::min(256.0, std::max(1.0, (double)P.elements * eb_a / 4096.0));
    if (kp.num_tiles < cus_wanted) e += 1.5 * (cus_wanted - kp.num_tiles) / 256.0;
    return std::exp(e);
}

static bool same_config(const Candidate& x, const Candidate& y)
{
    if (x.kernel_class != y.kernel_class || x.threads != y.threads || x.wg_per_cu != y.wg_per_cu) return false;
    if (x.rows.unroll != y.rows.unroll) return false;
    if (x.kp.a.vec != y.kp.a.vec || x.kp.b.vec != y.kp.b.vec || x.kp.lds_buffers != y.kp.lds_buffers) return false;
    for (int k = 0; k < kMaxDim; ++k) {
        if (x.tile[k] != y.tile[k]) return false;
        if (x.kp.tile_below[k].div != y.kp.tile_below[k].div) return false;
    }
    for (int i = 0; i < kBoxDims; ++i)
        if (x.dlane_a[i] != y.dlane_a[i] || x.dlane_b[i] != y.dlane_b[i] || x.dtile_a[i] != y.dtile_a[i] ||
            x.dtile_b[i] != y.dtile_b[i]) return false;
    return true;
}

// Non-temporal hints by rule: a side streams if all its runs are whole 128-byte lines.  Then no line is
// shared with a neighbouring tile, and keeping it in cache would only displace lines that are.  (The timed
// search tries the other settings on its finalists.)
void default_streaming(const Problem& P, Candidate* c)
{
    if (c->kernel_class == TTC_KERNEL_ROWS) {      // B is written front to back and A's rows are read once: stream both
        c->kp.nt_a = c->kp.nt_b = 1;
        return;
    }
    const AccessShape sh = access_shape(P, *c);
    c->kp.nt_a = (sh.align[0] >= 128) ? 1 : 0;
    c->kp.nt_b = (sh.align[1] >= 128) ? 1 : 0;
    if (c->kernel_class == TTC_KERNEL_MICRO && P.epilogue == TTC_EPI_AXPBY && sh.align[0] >= 32 && sh.align[1] >= 32) {
        // B is read and written by the same lane within a few hundred cycles, and runs that start on 32-byte
        // boundaries split no memory transaction with a neighbour: with both sides streamed 72^4 fp64 (rows of 576
        // bytes) runs at 98-105 % of a copy against 77-88 % by the rule above.  (Runs that start anywhere,
        // 24x20x16x18x22x17 with its 68-byte steps in B, lose up to 20 % that way and keep the rule.)
        c->kp.nt_a = c->kp.nt_b = 1;
    }
    if (c->kernel_class == TTC_KERNEL_DIRECT) c->kp.nt_a = c->kp.nt_b = (c->kp.nt_a && c->kp.nt_b) ? 1 : 0;   // both or neither
}

// what same_config() compares, folded into one number: candidates are looked up by it instead of being
// compared with every earlier one
static uint64_t config_hash(const Candidate& c)
{
    uint64_t h = 1469598103934665603ull;
    auto mix = [&](int64_t x) { h = (h ^ (uint64_t)x) * 1099511628211ull; };
    mix(c.kernel_class); mix(c.threads); mix(c.wg_per_cu); mix(c.rows.unroll);
    mix(c.kp.a.vec); mix(c.kp.b.vec); mix(c.kp.lds_buffers);
    for (int k = 0; k < kMaxDim; ++k) { mix(c.tile[k]); mix(c.kp.tile_below[k].div); }
    for (int i = 0; i < kBoxDims; ++i) { mix(c.dlane_a[i]); mix(c.dlane_b[i]); mix(c.dtile_a[i]); mix(c.dtile_b[i]); }
    return h;
}

struct CandidateList {
    std::vector<Candidate>& v;
    std::unordered_multimap<uint64_t, size_t> seen;
    explicit CandidateList(std::vector<Candidate>& out) : v(out) {}
};

static void add_candidate(const Problem& P, CandidateList& L, const Candidate& c)
{
    const uint64_t h = config_hash(c);
    const auto range = L.seen.equal_range(h);
    for (auto it = range.first; it != range.second; ++it)
        if (same_config(L.v[it->second], c)) return;
    L.seen.emplace(h, L.v.size());
    L.v.push_back(c);
    default_streaming(P, &L.v.back());
    L.v.back().score = heuristic_cost(P, L.v.back());
}

static int max_vec(int eb, int64_t extent)
{
    int v = std::max(1, 16 / eb);
    while (v > 1 && extent % v != 0) v /= 2;
    return v;
}

// Launch shapes tried for every tile shape: workgroup size and workgroups per compute unit.
struct LaunchShape { int threads, wg_per_cu; };
static const LaunchShape kLaunchShapes[] = {{256, 16}, {128, 8}, {256, 8}, {128, 16}, {256, 4}, {512, 8}, {64, 32},
                                            {256, 0}, {128, 0}, {512, 0}};      // 0: what a compute unit holds at once

// Different run-length targets often ask for the same box: each (box, vector rule, kernel family) is expanded once.
struct ShapesSeen {
    struct Key { int t[kMaxDim]; int vec, family; };
    std::vector<Key> keys;
    bool first_time(const int* t, int vec, int family)
    {
        for (const Key& k : keys) {
            bool same = (k.vec == vec && k.family == family);
            for (int i = 0; same && i < kMaxDim; ++i) same = (k.t[i] == t[i]);
            if (same) return false;
        }
        Key k;
        for (int i = 0; i < kMaxDim; ++i) k.t[i] = t[i];
        k.vec = vec; k.family = family;
        keys.push_back(k);
        return true;
    }
};

// quick: only the variants the ranking prefers (both walks merged, the two favoured launch shapes) -- what
// ttc_plan_create pays for; the full list is built when something first asks for it.
static void enumerate(const Problem& P, std::vector<Candidate>& out_list, bool quick)
{
    out_list.reserve(quick ? 2048 : 16384);      // a candidate is a few KB: no regrowth copies
    CandidateList out(out_list);
    ShapesSeen shapes;
    LayoutCache cache;
    const int n = P.ndim;
    const int eb = std::max(P.eb_a, P.eb_b);
    int order_a[kMaxDim], order_b[kMaxDim];
    for (int k = 0; k < kMaxDim; ++k) { order_a[k] = k; order_b[k] = (k < n) ? P.perm[k] : k; }
    const bool stride1_fixed = (P.perm[0] == 0);
    // Tile orders (which index varies fastest from one tile id to the next): B's index order, A's, and the
    // two mixed ones that put the other tensor's stride-1 index first, so that tiles sharing a cache line
    // at the end of a run are in flight together on BOTH sides.
    int order_ab[kMaxDim], order_ba[kMaxDim];
    {
        int na = 0, nb = 0;
        order_ab[na++] = 0;
        for (int i = 0; i < kMaxDim; ++i) if (order_b[i] != 0) order_ab[na++] = order_b[i];
        order_ba[nb++] = order_b[0];
        for (int i = 0; i < kMaxDim; ++i) if (order_a[i] != order_b[0]) order_ba[nb++] = order_a[i];
    }
    const int* orders[4] = {order_b, order_a, order_ab, order_ba};
    const int norders = stride1_fixed ? 2 : 4;
    const int nshapes = quick ? 2 : (int)(sizeof(kLaunchShapes) / sizeof(kLaunchShapes[0]));

    // -- the row kernel: only when the stride-1 index keeps its place (or there is one index only)
    if (stride1_fixed) {
        const int vwide = std::max(1, 16 / eb);
        for (int v = vwide; v >= 1; v /= 2) {
            for (int unroll : {2, 4, 1, 8}) {
                Candidate c;
                if (make_rows_candidate(P, v, unroll, &c)) add_candidate(P, out, c);
                if (quick) break;
            }
        }
    }

    // -- direct candidates: only when the stride-1 index keeps its place.  The box takes leading
    //    indices of A and of B so that both sides move a few long contiguous chunks per tile.
    if (stride1_fixed) {
        const int vfull = max_vec(eb, P.size[0]);
        const int64_t chunk_bytes[7] = {16384, 4096, 32768, 8192, 2048, 65536, 1024};
        const int vwide = std::max(1, 16 / eb);
        for (int vsel = 0; vsel < 3; ++vsel) {
            if (vsel == 1 && vfull == 1) continue;
            if (vsel == 2 && (vfull == vwide || P.stride_a[0] != 1 || P.stride_b[0] != 1)) continue;
            // 0: the widest vector that divides the rows; 1: scalar; 2: the widest vector, cut at the end of a run
            const int v = vsel == 0 ? vfull : (vsel == 1 ? 1 : 32);
            const int vmult = vsel == 0 ? vfull : 1;
            for (int style = 0; style < 2; ++style)
            for (int64_t ra : chunk_bytes)
                for (int64_t rb : chunk_bytes) {
                    int ta[kMaxDim], tb[kMaxDim], t[kMaxDim];
                    build_group(P, order_a, P.eb_a, ra / P.eb_a, vmult, kBoxDims, ta, style);
                    build_group(P, order_b, P.eb_b, rb / P.eb_b, vmult, kBoxDims, tb, style);
                    int64_t vol = 1;
                    int spanned = 0;
                    for (int k = 0; k < kMaxDim; ++k) t[k] = std::max(ta[k], tb[k]);
                    for (int k = 0; k < n; ++k) { vol *= t[k]; spanned += (t[k] > 1); }
                    if (spanned > kBoxDims || vol * eb > 128 * 1024) continue;
                    if (vol * eb < 4096 && vol < P.elements) continue;
                    if (!shapes.first_time(t, v, 0)) continue;
                    for (int o = 0; o < norders; ++o)
                        for (int li = 0; li < nshapes; ++li) {
                            const LaunchShape& ls = kLaunchShapes[li];
                            Candidate c;
                            if (make_candidate(P, t, v, true, ls.threads, ls.wg_per_cu, orders[o], kDefaultTileMapping, &c))
                                add_candidate(P, out, c);
                        }
                }
        }
    }

    // -- the micro-tile kernel: a tile over the two stride-1 indices.  Tile extents in vectors: powers of two, and
    // the divisors of the extent (no remainder tiles)
    if (!stride1_fixed && n >= 2) {
        const int vec = std::max(1, 16 / P.eb_a);
        auto extents = [&](int64_t size, bool divisors, std::vector<int>* v) {
            const int64_t whole = size / vec;
            for (int l = 8; l <= 64; l *= 2) if (l <= 2 * whole) v->push_back(l);
            if (size % vec == 0 && divisors)
                for (int l = 6; l <= 96; ++l)
                    if (whole % l == 0 && (l & (l - 1)) != 0) v->push_back(l);
            if (whole >= 1 && whole < 8) v->push_back((int)ceil_div(size, vec));
            if (size % vec != 0 && whole >= 8) {               // the whole extent in one tile, or in two: no run shared between tiles
                const int64_t all = ceil_div(size, vec);
                if (all <= 96) v->push_back((int)all);
                if (all >= 16 && ceil_div(all, 2) <= 96) v->push_back((int)ceil_div(all, 2));
            }
        };
        // the column index: A's index 0, or (short rows) indices 0 and 1 as one; the row index likewise on B's side
        const int p0 = P.perm[0], p1 = P.perm[1];
        for (int merge_a = 0; merge_a < 2; ++merge_a)
            for (int merge_b = 0; merge_b < 2; ++merge_b) {
                if (merge_a && (n < 3 || P.size[0] * P.eb_a > 1024 || p0 == 1)) continue;
                if (merge_b && (n < 3 || P.size[p0] * P.eb_a > 1024 || p1 == 0)) continue;
                if (merge_a && merge_b && p1 == 1) continue;
                const int64_t cols = merge_a ? P.size[0] * P.size[1] : P.size[0], rows = merge_b ? P.size[p0] * P.size[p1] : P.size[p0];
                std::vector<int> las, lbs;
                extents(cols, !(quick && merge_a), &las);       // the short list: a merged index is cut at powers of two and whole rows only
                extents(rows, !(quick && merge_b), &lbs);
                // whole rows of the inner index: tiles that end where a run of the other tensor ends
                if (merge_a) for (int64_t k = 1; k * P.size[0] <= 96 * vec && k <= P.size[1]; ++k) if (k * P.size[0] % vec == 0) las.push_back((int)(k * P.size[0] / vec));
                if (merge_b) for (int64_t k = 1; k * P.size[p0] <= 96 * vec && k <= P.size[p1]; ++k) if (k * P.size[p0] % vec == 0) lbs.push_back((int)(k * P.size[p0] / vec));
                for (int threads : {256, 128, 64}) {
                    if (quick && threads == 64) continue;          // the model ranks one-wavefront workgroups behind the others
                    for (int la : las)
                        for (int lb : lbs) {
                            const int64_t blocks = ceil_div((int64_t)la * lb, threads);
                            if (blocks > 6 || (int64_t)la * lb * 5 < blocks * threads * 4) continue;      // lanes mostly busy
                            for (int o = 0; o < (quick ? 1 : 2); ++o) {       // the mixed orders, and the indices outside the tile first, time the same (384^3, 72^4, 6-D reversals)
                                Candidate c;
                                if (make_micro_candidate(P, la * vec, lb * vec, threads, orders[o], merge_a != 0, merge_b != 0, &c))
                                    add_candidate(P, out, c);
                            }
                        }
                }
            }
    }

    // -- staged candidates: a box spanning the leading indices of A and of B
    if (n >= 2) {
        const int p0 = P.perm[0];
        const int va_full = max_vec(P.eb_a, P.size[0]);
        const int vb_full = max_vec(P.eb_b, P.size[p0]);
        const int64_t run_bytes[8] = {256, 512, 128, 1024, 64, 2048, 4096, 8192};
        const bool odd_rows = va_full < std::max(1, 16 / P.eb_a) || vb_full < std::max(1, 16 / P.eb_b);
        for (int vsel = 0; vsel < 3; ++vsel) {
            if (vsel == 2 && !odd_rows) continue;
            // 0: the widest vectors that divide the runs; 1: scalar; 2: the widest vectors, cut at the end of a run
            const int va = vsel == 0 ? va_full : 1;       // multiples the group builder keeps on the stride-1 extents
            const int vb = vsel == 0 ? vb_full : 1;
            const int vec_limit = vsel == 0 ? 16 : (vsel == 1 ? 1 : 32);
            for (int md = 3; md >= 1; --md)
              for (int style = 0; style < 2; ++style)
                for (int64_t ra : run_bytes)
                    for (int64_t rb : run_bytes) {
                        int ta[kMaxDim], tb[kMaxDim], t[kMaxDim];
                        build_group(P, order_a, P.eb_a, std::max<int64_t>(1, ra / P.eb_a), va, md, ta, style);
                        build_group(P, order_b, P.eb_b, std::max<int64_t>(1, rb / P.eb_b), vb, md, tb, style);
                        int64_t vol = 1;
                        int spanned = 0;
                        for (int k = 0; k < kMaxDim; ++k) t[k] = std::max(ta[k], tb[k]);
                        for (int k = 0; k < n; ++k) { vol *= t[k]; spanned += (t[k] > 1); }
                        if (spanned > kBoxDims) continue;
                        if (vol * P.eb_a > kMaxLdsBytes - 2048) continue;
                        if (vol * eb < 2048 && md > 1 && vol < P.elements) continue;
                        if (!shapes.first_time(t, vec_limit, 1)) continue;
                        for (int nbuf = 2; nbuf >= 1; --nbuf) {
                            if (nbuf == 1 && vol * eb < 8192) continue;     // small tiles can afford two buffers
                            for (int mg = 0; mg < (quick ? 1 : 4); ++mg)
                                for (int o = 0; o < norders; ++o)
                                    for (int li = 0; li < nshapes; ++li) {
                                        const LaunchShape& ls = kLaunchShapes[li];
                                        Candidate c;
                                        if (make_candidate(P, t, vec_limit, false, ls.threads, ls.wg_per_cu, orders[o], kDefaultTileMapping,
                                                           &c, (mg & 1) == 0, (mg & 2) == 0, &cache, nbuf))
                                            add_candidate(P, out, c);
                                    }
                        }
                    }
        }
    }

    // -- last resort so that every problem has a candidate: scalar direct walk in A order
    if (out_list.empty() || n == 1) {
        int t[kMaxDim];
        build_group(P, order_a, P.eb_a, 16384 / eb, 1, kBoxDims, t);
        Candidate c;
        if (make_candidate(P, t, 1, true, 256, 8, order_a, kDefaultTileMapping, &c)) add_candidate(P, out, c);
    }
}

int build_plan(int dtype, int ndim, const int64_t* sizes, const int* perm, const int64_t* lda, const int64_t* ldb,
               const void* alpha, const void* beta, ttc_plan_s* plan)
{
    Problem& P = plan->prob;
    int st = normalise(dtype, ndim, sizes, perm, lda, ldb, alpha, beta, &P);
    if (st != TTC_OK) return st;
    std::vector<Candidate> quick;
    enumerate(P, quick, true);
    if (quick.empty()) enumerate(P, quick, false);
    if (quick.empty()) return TTC_ERR_OVERFLOW;
    size_t best = 0;
    for (size_t i = 1; i < quick.size(); ++i) if (quick[i].score < quick[best].score) best = i;
    plan->cands.assign(1, quick[best]);
    plan->selected = 0;
    plan->complete = false;
    if (verbose()) {
        const Candidate& c = plan->cands[0];
        std::fprintf(stderr, "ttc: plan dtype %d, %d fused indices, %s kernel, tile", P.dtype, P.ndim,
                     c.kernel_class == TTC_KERNEL_DIRECT ? "direct" : (c.kernel_class == TTC_KERNEL_ROWS ? "row" : (c.kernel_class == TTC_KERNEL_MICRO ? "micro-tile" : "staged")));
        for (int k = 0; k < P.ndim; ++k) std::fprintf(stderr, " %d", c.tile[k]);
        size_t per_class[4] = {0, 0, 0, 0};
        for (const Candidate& q : quick) if (q.kernel_class >= 0 && q.kernel_class < 4) ++per_class[q.kernel_class];
        std::fprintf(stderr, ", vectors %d/%d, %d threads, %d B LDS, cost %.4f (best of %zu candidates of the short list: %zu direct, %zu staged, %zu row, %zu micro-tile)\n",
                     c.kp.a.vec, c.kp.b.vec, c.threads, c.lds_bytes, c.score, quick.size(), per_class[0], per_class[1], per_class[2], per_class[3]);
    }
    return TTC_OK;
}

// The ranked list of all candidates, built on first use.  Candidate 0 stays what ttc_plan_create chose (with
// whatever the caller has set on it since); the others follow in the order of the heuristic cost.
int complete_plan(ttc_plan_s* plan)
{
    if (plan->complete) return TTC_OK;
    const Candidate first = plan->cands[plan->selected];
    std::vector<Candidate> all;
    enumerate(plan->prob, all, false);
    std::stable_sort(all.begin(), all.end(), [](const Candidate& x, const Candidate& y) { return x.score < y.score; });
    std::vector<Candidate> ranked;
    ranked.reserve(all.size() + 1);
    ranked.push_back(first);
    for (const Candidate& c : all) if (!same_config(c, first)) ranked.push_back(c);
    plan->cands.swap(ranked);
    plan->selected = 0;
    plan->complete = true;
    if (verbose()) std::fprintf(stderr, "ttc: %zu candidates ranked\n", plan->cands.size());
    return TTC_OK;
}

}  // namespace ttc

// Nothing may throw across the C boundary: allocation failures and anything unexpected become status codes.
template <class F> static int guarded(F&& body)
{
    try { return body(); }
    catch (const std::bad_alloc&) { return TTC_ERR_ALLOC; }
    catch (...) { return TTC_ERR_INTERNAL; }
}

// The kernels instantiate a walk for a compile-time vector width; the replay picks the same one.
template <class S1, class S2>
static void emu_walk(const ttc::Side& s, const ttc::LaneState& L, const ttc::SideLim& lim, const ttc::WalkMask& m,
                     const ttc::PosEntry* tab, const ttc::PosCoord* tabc, uint32_t wave, S1&& s1, S2&& s2)
{
    switch (s.vec) {
    case 1: ttc::walk<4, 1>(s, L, lim, m, tab, tabc, wave, s1, s2); break;
    case 2: ttc::walk<4, 2>(s, L, lim, m, tab, tabc, wave, s1, s2); break;
    default: ttc::walk<4, 4>(s, L, lim, m, tab, tabc, wave, s1, s2); break;
    }
}

// ---------------------------------------------------------------------------------
// Host-only part of the C ABI
// ---------------------------------------------------------------------------------
extern "C" {

ttc_plan_t ttc_plan_create(int dtype, int ndim, const int64_t* sizes, const int* perm,
                           const void* alpha, const void* beta)
{
    return ttc_plan_create_ex(dtype, ndim, sizes, perm, nullptr, nullptr, alpha, beta);
}

ttc_plan_t ttc_plan_create_ex(int dtype, int ndim, const int64_t* sizes, const int* perm,
                              const int64_t* lda, const int64_t* ldb, const void* alpha, const void* beta)
{
    ttc_plan_s* plan = new (std::nothrow) ttc_plan_s();
    if (!plan) { ttc::set_last_status(TTC_ERR_ALLOC); return nullptr; }
    int st;
    try {
        st = ttc::build_plan(dtype, ndim, sizes, perm, lda, ldb, alpha, beta, plan);
    } catch (const std::bad_alloc&) {
        st = TTC_ERR_ALLOC;
    } catch (...) {
        st = TTC_ERR_INVALID_VALUE;
    }
    ttc::set_last_status(st);
    if (st != TTC_OK) { delete plan; return nullptr; }
    return plan;
}

int ttc_plan_destroy(ttc_plan_t plan)
{
    delete plan;
    return TTC_OK;
}

int ttc_last_status(void) { return ttc::g_last_status; }

const char* ttc_status_string(int status)
{
    switch (status) {
    case TTC_OK: return "ok";
    case TTC_ERR_INVALID_VALUE: return "invalid value";
    case TTC_ERR_INVALID_PERM: return "perm is not a permutation";
    case TTC_ERR_UNSUPPORTED_DTYPE: return "unsupported data type";
    case TTC_ERR_NULL_POINTER: return "null pointer";
    case TTC_ERR_ALIAS: return "A and B overlap";
    case TTC_ERR_OVERFLOW: return "size overflow";
    case TTC_ERR_HIP: return "HIP runtime error";
    case TTC_ERR_ALLOC: return "allocation failed";
    case TTC_ERR_MISALIGNED: return "pointer not aligned to the element size";
    case TTC_ERR_INTERNAL: return "internal error: a candidate's walk is not a bijection in bounds";
    case TTC_ERR_NOT_FOUND: return "no stored plan for this problem";
    case TTC_ERR_IO: return "the plan store could not be written";
    default: return "unknown status";
    }
}

int ttc_plan_get_info(ttc_plan_t plan, ttc_plan_info_t* out)
{
    if (!plan || !out) return TTC_ERR_NULL_POINTER;
    return guarded([&]() -> int {
    const ttc::Problem& P = plan->prob;
    const ttc::Candidate& C = plan->cands[plan->selected];
    std::memset(out, 0, sizeof(*out));
    out->dtype = P.dtype;
    out->ndim = P.ndim;
    for (int k = 0; k < P.ndim; ++k) {
        out->sizes[k] = P.size[k];
        out->perm[k] = P.perm[k];
        out->tile[k] = C.tile[k];
        out->tile_order[k] = C.tile_order[k];
        out->lds_stride[k] = C.lds_stride[k];
    }
    out->digits_a = C.digits_a;
    out->digits_b = C.digits_b;
    for (int i = 0; i < ttc::kBoxDims; ++i) {
        out->digit_tile_a[i] = C.dtile_a[i];  out->digit_lane_a[i] = C.dlane_a[i];
        out->digit_tile_b[i] = C.dtile_b[i];  out->digit_lane_b[i] = C.dlane_b[i];
    }
    out->stride1_fixed = (P.perm[0] == 0) ? 1 : 0;
    out->kernel_class = C.kernel_class;
    out->epilogue = P.epilogue;
    out->vec_a = C.kp.a.vec;
    out->vec_b = C.kp.b.vec;
    out->partial_a = C.kp.a.partial;
    out->partial_b = C.kp.b.partial;
    out->threads = C.threads;
    out->wg_per_cu = C.wg_per_cu;
    out->xcd_remap = C.kp.xcd_remap;
    out->lds_bytes = C.lds_bytes;
    out->lds_buffers = C.kp.lds_buffers;
    out->nt_a = C.kp.nt_a;
    out->nt_b = C.kp.nt_b;
    out->lds_conflict_a = C.lds_conflict_a;
    out->lds_conflict_b = C.lds_conflict_b;
    {
        const ttc::AccessShape sh = ttc::access_shape(P, C);
        out->run_bytes_a = sh.run[0]; out->run_bytes_b = sh.run[1];
        out->seg_bytes_a = sh.seg[0]; out->seg_bytes_b = sh.seg[1];
        out->align_a = sh.align[0];   out->align_b = sh.align[1];
    }
    out->num_tiles = C.kp.num_tiles;
    out->elements = P.elements;
    out->bytes_moved = P.elements * (P.eb_a + (P.epilogue == TTC_EPI_AXPBY ? 2 : 1) * P.eb_b);
    out->span_a = P.span_a;
    out->span_b = P.span_b;
    for (int k = 0; k < P.ndim; ++k) { out->stride_a[k] = P.stride_a[k]; out->stride_b[k] = P.stride_b[k]; }
    out->candidate_index = plan->selected;
    out->candidate_count = (int)plan->cands.size();
    out->tuned_ms = C.tuned_ms;
    out->heuristic_cost = C.score;
    out->merged = C.kernel_class == TTC_KERNEL_MICRO ? (C.kp.micro.merged_a | (C.kp.micro.merged_b << 1)) : 0;
    out->unroll = C.kernel_class == TTC_KERNEL_ROWS ? C.rows.unroll : (C.kernel_class == TTC_KERNEL_MICRO ? C.kp.micro.blocks : 0);
    return TTC_OK;
    });
}

int ttc_plan_set_streaming(ttc_plan_t plan, int stream_a, int stream_b)
{
    if (!plan) return TTC_ERR_NULL_POINTER;
    if (stream_a < -1 || stream_a > 1 || stream_b < -1 || stream_b > 1) return TTC_ERR_INVALID_VALUE;
    return guarded([&]() -> int {
        ttc::Candidate& C = plan->cands[plan->selected];
        ttc::Candidate rule = C;
        ttc::default_streaming(plan->prob, &rule);
        C.kp.nt_a = stream_a < 0 ? rule.kp.nt_a : stream_a;
        C.kp.nt_b = stream_b < 0 ? rule.kp.nt_b : stream_b;
        if (C.kernel_class == TTC_KERNEL_DIRECT) C.kp.nt_a = C.kp.nt_b = (C.kp.nt_a && C.kp.nt_b) ? 1 : 0;
        return TTC_OK;
    });
}

int ttc_plan_set_tile_mapping(ttc_plan_t plan, int mode)
{
    if (!plan) return TTC_ERR_NULL_POINTER;
    if (mode < -1 || mode > 10) return TTC_ERR_INVALID_VALUE;
    ttc::Candidate& C = plan->cands[plan->selected];
    return ttc::set_tile_mapping(&C.kp, mode) ? TTC_OK : TTC_ERR_INVALID_VALUE;
}

int ttc_plan_candidate_count(ttc_plan_t plan)
{
    if (!plan) return -TTC_ERR_NULL_POINTER;
    const int st = guarded([&] { return ttc::complete_plan(plan); });
    return st == TTC_OK ? (int)plan->cands.size() : -st;
}

int ttc_plan_select_candidate(ttc_plan_t plan, int index)
{
    if (!plan) return TTC_ERR_NULL_POINTER;
    if (index < 0) return TTC_ERR_INVALID_VALUE;
    if (index == 0 && plan->selected == 0) return TTC_OK;          // the choice of ttc_plan_create: no list needed
    const int st = guarded([&] { return ttc::complete_plan(plan); });
    if (st != TTC_OK) return st;
    if (index >= (int)plan->cands.size()) return TTC_ERR_INVALID_VALUE;
    plan->selected = index;
    return TTC_OK;
}

// Host-side bounds checker: replays the selected candidate's walk (the same index code the
// kernels run) lane by lane and records, for every offset of B, the offset of A that lands
// there.  Fails on any access outside the (sub-)tensors or the LDS tile, any access that is
// not element-aligned, any element of B written twice or never, and any LDS slot read before
// it was written.
static int emulate_map(ttc_plan_t plan, int64_t* b_from_a);

int ttc_debug_emulate_map(ttc_plan_t plan, int64_t* b_from_a)
{
    if (!plan || !b_from_a) return TTC_ERR_NULL_POINTER;
    return guarded([&] { return emulate_map(plan, b_from_a); });
}

}  // extern "C"

// Replay of the row kernel: every workgroup, every lane, the index code the kernel runs.
static int emulate_rows(const ttc::Problem& P, const ttc::Candidate& C, int64_t* b_from_a)
{
    using namespace ttc;
    const RowsParams& p = C.rows;
    for (int64_t i = 0; i < P.span_b; ++i) b_from_a[i] = -1;
    const int64_t rows = P.elements / P.size[0];
    if ((p.vec != 1 && p.vec != 2 && p.vec != 4) || (p.unroll != 1 && p.unroll != 2 && p.unroll != 4 && p.unroll != 8) || C.threads != 256 ||
        p.chunk != (uint32_t)(C.threads * p.unroll) || p.row < (uint32_t)p.vec || p.row != (uint32_t)P.size[0] ||
        p.slots != (p.row + (uint32_t)p.vec - 1) / (uint32_t)p.vec || p.vectors != rows * (int64_t)p.slots ||
        p.overlap != (P.size[0] % p.vec != 0 ? 1 : 0) || (p.overlap && P.epilogue == TTC_EPI_AXPBY) ||
        P.size[0] >= (int64_t(1) << 30) || rows >= (int64_t(1) << 31))
        return TTC_ERR_INTERNAL;
    auto inside = [&](int64_t off, const int64_t* stride, bool b_side) {
        if (off < 0) return false;
        for (int i = P.ndim - 1; i >= 0; --i) {
            const int k = b_side ? P.perm[i] : i;
            const int64_t c = off / stride[k];
            if (c >= P.size[k]) return false;
            off -= c * stride[k];
        }
        return off == 0;
    };
    int64_t written = 0;
    bool bad = false;
    const int64_t grid = (p.vectors + p.chunk - 1) / p.chunk;
    for (int64_t wg = 0; wg < grid && !bad; ++wg) {
        const int64_t base = wg * (int64_t)p.chunk;
        const int64_t row0_wide = base / (int64_t)p.slots;
        const uint32_t row0 = (uint32_t)row0_wide, slot0 = (uint32_t)(base - row0_wide * (int64_t)p.slots);
        for (int u = 0; u < p.unroll && !bad; ++u)
            for (uint32_t tid = 0; tid < (uint32_t)C.threads && !bad; ++tid) {
                const RowAccess x = rows_access(p, base, row0, slot0, (uint32_t)u * (uint32_t)C.threads + tid);
                for (int j = 0; j < p.vec; ++j) {            // loads happen for every lane: they must stay inside
                    const int64_t ea = x.at.a + j, eo = x.at.b + j;
                    if (!inside(ea, P.stride_a, false) || !inside(eo, P.stride_b, true)) { bad = true; break; }
                    if (!x.valid) continue;
                    // an overlapping vector repeats its neighbour's elements: same source
                    if (b_from_a[eo] != -1 && (b_from_a[eo] != ea || !p.overlap)) { bad = true; break; }
                    if (b_from_a[eo] == -1) ++written;
                    b_from_a[eo] = ea;
                }
            }
    }
    return (bad || written != P.elements) ? TTC_ERR_INTERNAL : TTC_OK;
}

// Replay of the micro-tile kernel: every workgroup, every lane, the index code the kernel runs; every LDS slot
// must be written before it is read, inside the tile buffer.
static int emulate_micro(const ttc::Problem& P, const ttc::Candidate& C, int64_t* b_from_a)
{
    using namespace ttc;
    const MicroArgs p = micro_args(C);          // what the launch hands to the kernel
    const MicroParams& m = p.micro;
    for (int64_t i = 0; i < P.span_b; ++i) b_from_a[i] = -1;
    const uint32_t threads = (uint32_t)C.threads;
    const int vec = m.vec;
    if (p.col_pos < 0 || p.row_pos < 0 || p.col_pos == p.row_pos) return TTC_ERR_INTERNAL;
    if ((vec != 2 && vec != 4) || vec * P.eb_a != 16 || P.eb_a != P.eb_b ||
        (threads != 64 && threads != 128 && threads != 256) || m.ta != vec * m.la || m.tb != vec * m.lb ||
        m.la < 1 || m.lb < 1 || m.pitch < m.la || (m.pitch & 7) || (m.swizzle != 7u && m.swizzle != 0u) || m.la_div.div != (uint32_t)m.la || m.lb_div.div != (uint32_t)m.lb ||
        (int64_t)m.loads * threads < (int64_t)m.la * m.tb || (int64_t)m.blocks * threads < (int64_t)m.la * m.lb ||
        (1 << m.vec_log) != vec || C.lds_bytes != m.tb * m.pitch * 16 || C.lds_bytes > 64 * 1024 || p.grid != p.num_tiles ||
        m.p0 != P.perm[0] || m.p0 == 0 || P.ndim < 2 || P.stride_a[0] != 1 || P.stride_b[m.p0] != 1 ||
        (m.merged_a != 0 && m.merged_a != 1) || (m.merged_b != 0 && m.merged_b != 1))
        return TTC_ERR_INTERNAL;
    const int a1 = 1, p1 = P.perm[1];
    if (m.merged_a && (P.ndim < 3 || a1 == m.p0 || P.stride_a[a1] != P.size[0] || (m.merged_b && a1 == p1))) return TTC_ERR_INTERNAL;
    if (m.merged_b && (P.ndim < 3 || p1 == 0 || P.stride_b[p1] != P.size[m.p0] || (m.merged_a && p1 == a1))) return TTC_ERR_INTERNAL;
    const int64_t cols = m.merged_a ? P.size[0] * P.size[a1] : P.size[0], rows = m.merged_b ? P.size[m.p0] * P.size[p1] : P.size[m.p0];
    if (m.size_a0 != cols || m.size_p0 != rows || cols < vec || rows < vec || cols >= (int64_t(1) << 31) || rows >= (int64_t(1) << 31) ||
        m.col_in_div.div != (uint32_t)P.size[0] || m.row_in_div.div != (uint32_t)P.size[m.p0] ||
        m.col_b_in != P.stride_b[0] || m.col_b_out != (m.merged_a ? P.stride_b[a1] : 0) ||
        m.row_a_in != P.stride_a[m.p0] || m.row_a_out != (m.merged_b ? P.stride_a[p1] : 0))
        return TTC_ERR_INTERNAL;
    const bool whole = cols % vec == 0 && rows % vec == 0;                   // else some elements are written twice ...
    const bool update = P.epilogue == TTC_EPI_AXPBY;                         // ... unless B is read as well: then blocks write only their own
    auto inside = [&](int64_t off, const int64_t* stride, bool b_side) {
        if (off < 0) return false;
        for (int i = P.ndim - 1; i >= 0; --i) {
            const int k = b_side ? P.perm[i] : i;
            const int64_t c = off / stride[k];
            if (c >= P.size[k]) return false;
            off -= c * stride[k];
        }
        return off == 0;
    };
    const int64_t slots = (int64_t)m.tb * m.pitch;              // 16-byte slots of the tile buffer
    std::vector<int64_t> lds((size_t)(slots * vec));
    std::vector<char> seen(p.num_tiles, 0);
    int64_t written = 0;
    for (uint32_t wg = 0; wg < p.grid; ++wg) {
        const TileSeq seq = tile_sequence(p, wg);
        for (uint32_t q = seq.first; q < seq.end; q += seq.step) {
            const uint32_t tile = tile_of(seq, q);
            if (tile >= p.num_tiles || seen[tile]) return TTC_ERR_INTERNAL;
            seen[tile] = 1;
            const MicroTile t = micro_tile(p, tile);
            if (t.lim_a < (uint32_t)vec || t.lim_b < (uint32_t)vec || t.lim_a > (uint32_t)m.ta || t.lim_b > (uint32_t)m.tb) return TTC_ERR_INTERNAL;
            if (whole && (t.lim_a % vec || t.lim_b % vec)) return TTC_ERR_INTERNAL;
            std::fill(lds.begin(), lds.end(), (int64_t)-1);
            for (int i = 0; i < vec; ++i)                         // lanes outside load the tile's first vector or block
                for (int j = 0; j < vec; ++j)
                    if (!inside(t.a + micro_row_a(m, t.row0 + (uint32_t)i) + j, P.stride_a, false) ||
                        !inside(t.b + micro_col_b(m, t.col0 + (uint32_t)j) + i, P.stride_b, true))
                        return TTC_ERR_INTERNAL;
            for (uint32_t tid = 0; tid < threads; ++tid)
                for (int k = 0; k < (m.loads + 3) / 4 * 4; ++k) { // the kernel walks its loads four at a time
                    const MicroLoad x = micro_load(m, threads, tid, (uint32_t)k);
                    if (!x.valid) continue;
                    if (x.chunk >= (uint64_t)slots) return TTC_ERR_INTERNAL;
                    const bool ok = x.row < t.lim_b && x.col < t.lim_a;
                    const uint32_t col = ok ? micro_back(x.col, t.lim_a, (uint32_t)vec) : 0u;
                    for (int j = 0; j < vec; ++j) {
                        int64_t src = -2;                         // parked by a lane outside the tensor: must never be read
                        if (ok) {
                            src = t.a + micro_row_a(m, t.row0 + x.row) + col + j;
                            if (!inside(src, P.stride_a, false)) return TTC_ERR_INTERNAL;
                        }
                        if (lds[(size_t)x.chunk * vec + j] != -1) return TTC_ERR_INTERNAL;       // every slot has one writer
                        lds[(size_t)x.chunk * vec + j] = src;
                    }
                }
            for (uint32_t tid = 0; tid < threads; ++tid)
                for (int b = 0; b < m.blocks; ++b) {
                    const MicroBlock x = micro_block(m, threads, tid, (uint32_t)b);
                    if (!(x.valid && x.row < t.lim_b && x.col < t.lim_a)) continue;
                    const uint32_t row = micro_back(x.row, t.lim_b, (uint32_t)vec), col = micro_back(x.col, t.lim_a, (uint32_t)vec);
                    const bool edge = update && (row != x.row || col != x.col || x.row < t.own_b || x.col < t.own_a);
                    const uint32_t first_row = std::max(x.row, t.own_b), first_col = std::max(x.col, t.own_a);
                    for (int i = 0; i < vec; ++i) {
                        const uint64_t chunk = micro_slot(m, row + (uint32_t)i, x.lane_c);
                        if (chunk >= (uint64_t)slots) return TTC_ERR_INTERNAL;
                        for (int j = 0; j < vec; ++j) {
                            const int64_t src = lds[(size_t)chunk * vec + j];
                            const int64_t dst = t.b + micro_col_b(m, t.col0 + col + (uint32_t)j) + row + i;
                            // what sits in the slot must be the element of the tile at (row + i, col + j)
                            if (src != t.a + micro_row_a(m, t.row0 + row + (uint32_t)i) + col + j) return TTC_ERR_INTERNAL;
                            if (!inside(dst, P.stride_b, true)) return TTC_ERR_INTERNAL;
                            if (edge && !(col + (uint32_t)j >= first_col && row + (uint32_t)i >= first_row)) continue;   // not this block's to update
                            if (b_from_a[dst] == -1) ++written;
                            else if (whole || update || b_from_a[dst] != src) return TTC_ERR_INTERNAL;   // a second write brings the same element
                            b_from_a[dst] = src;
                        }
                    }
                }
        }
    }
    return written == P.elements ? TTC_OK : TTC_ERR_INTERNAL;
}

static int emulate_map(ttc_plan_t plan, int64_t* b_from_a)
{
    using namespace ttc;
    const Problem& P = plan->prob;
    const Candidate& C = plan->cands[plan->selected];
    if (C.kernel_class == TTC_KERNEL_ROWS) return emulate_rows(P, C, b_from_a);
    if (C.kernel_class == TTC_KERNEL_MICRO) return emulate_micro(P, C, b_from_a);
    KernelParams p = C.kp;
    set_grid(&p, launch_grid(C, 256));
    const int32_t eba = P.eb_a, ebb = P.eb_b;
    for (int64_t i = 0; i < P.span_b; ++i) b_from_a[i] = -1;
    const uint32_t nwave = (uint32_t)C.threads / kWave;
    if (nwave < 1 || C.threads % kWave) return TTC_ERR_INTERNAL;
    const bool direct = (C.kernel_class == TTC_KERNEL_DIRECT);
    if ((p.lds_buffers != 1 && p.lds_buffers != 2) ||
        p.lds_data_off + p.lds_buffers * (int64_t)p.lds_tile_elems * eba != C.lds_bytes || C.lds_bytes > kMaxLdsBytes)
        return TTC_ERR_INTERNAL;
    // is this element offset an element of the sub-tensor?  (decode by strides, slowest index first)
    auto inside = [&](int64_t off, const int64_t* stride, bool b_side) {
        if (off < 0) return false;
        for (int i = P.ndim - 1; i >= 0; --i) {
            const int k = b_side ? P.perm[i] : i;
            const int64_t c = off / stride[k];
            if (c >= P.size[k]) return false;
            off -= c * stride[k];
        }
        return off == 0;
    };
    // position tables, as a workgroup builds them
    const uint32_t ta = nwave * (uint32_t)p.a.chunk, tbn = direct ? 0u : nwave * (uint32_t)p.b.chunk;
    if (kTablesOff + (int64_t)24 * (ta + tbn) > p.lds_data_off) return TTC_ERR_INTERNAL;
    if (p.a.chunk_rem < 1 || p.a.chunk_rem > (int)nwave || (p.a.chunk - 1) * (int)nwave + p.a.chunk_rem != p.a.n_iter)
        return TTC_ERR_INTERNAL;
    if (!direct && (p.b.chunk_rem < 1 || p.b.chunk_rem > (int)nwave ||
                    (p.b.chunk - 1) * (int)nwave + p.b.chunk_rem != p.b.n_iter)) return TTC_ERR_INTERNAL;
    const Scales sc_a = {eba, ebb, eba};       // walk over A (direct: g2 addresses B)
    const Scales sc_b = {ebb, ebb, eba};       // walk over B of the staged kernel
    std::vector<PosEntry> tab_a(ta), tab_b(tbn);
    std::vector<PosCoord> tabc_a(ta), tabc_b(tbn);
    for (uint32_t th = 0; th < (uint32_t)C.threads; ++th) {
        if (direct) build_tables<true>(p.a, nwave, th, (uint32_t)C.threads, sc_a, tab_a.data(), tabc_a.data());
        else {
            build_tables<false>(p.a, nwave, th, (uint32_t)C.threads, sc_a, tab_a.data(), tabc_a.data());
            build_tables<false>(p.b, nwave, th, (uint32_t)C.threads, sc_b, tab_b.data(), tabc_b.data());
        }
    }

    const int64_t lds_bytes = (int64_t)p.lds_tile_elems * eba;
    std::vector<int64_t> lds((size_t)p.lds_tile_elems);          // which element offset of A each slot holds
    std::vector<char> seen(p.num_tiles, 0);
    bool bad = false;
    int fail_line = 0;
    auto fail_at = [&](int line) { if (!bad) fail_line = line; bad = true; };
#define fail() fail_at(__LINE__)
    auto nop = [](int, const PosEntry&, int, bool) {};
    const bool axpby = (P.epilogue == TTC_EPI_AXPBY);
    std::vector<int64_t> writer((size_t)P.span_b, -1);      // which instruction wrote an element of B
    int64_t written = 0;
    for (uint32_t wg = 0; wg < p.grid && !bad; ++wg) {
        const TileSeq seq = tile_sequence(p, wg);
        for (uint32_t q = seq.first; q < seq.end && !bad; q += seq.step) {
            const uint32_t tile = tile_of(seq, q);
            if (tile >= p.num_tiles || seen[tile]) return TTC_ERR_INTERNAL;
            seen[tile] = 1;
            const TileBase tb = tile_base(p, tile);
            const int64_t base_a = tb.a * eba, base_b = tb.b * ebb;
            const TileLim tl = tile_lim(p, tile);
            const SideLim la = side_lim(p.a, tl);
            // lanes outside the tile load the tile's first vector instead (and read the LDS tile's first slots)
            for (int j = 0; j < p.a.vec; ++j) if (!inside(tb.a + j, P.stride_a, false)) return TTC_ERR_INTERNAL;
            for (int j = 0; j < (direct ? p.a.vec : p.b.vec); ++j)
                if (!inside(tb.b + j, P.stride_b, true)) return TTC_ERR_INTERNAL;
            if (!direct && (int64_t)(p.b.vec - 1) * p.b.vec_lds_stride >= p.lds_tile_elems) return TTC_ERR_INTERNAL;
            if (direct) {
                for (uint32_t wave = 0; wave < nwave; ++wave)
                    for (uint32_t lane = 0; lane < (uint32_t)kWave; ++lane) {
                        const LaneState L = lane_setup<true>(p.a, lane, sc_a);
                        const WalkMask wm = walk_mask(p.a, L, la);
                        auto st = [&](int, const PosEntry& e, int back, bool ok) {
                            if (!ok) return;
                            const int64_t oa = base_a + e.g + L.g, ob = base_b + e.l_or_g2 + L.g2;
                            if (oa % eba || ob % ebb || back < 0 || back >= p.a.vec) return fail();
                            const int64_t who = ((int64_t)tile << 32) | (wave << 16) | (uint32_t)(&e - tab_a.data());
                            for (int j = -back; j < p.a.vec - back; ++j) {
                                const int64_t ea = oa / eba + j, eo = ob / ebb + j;
                                if (!inside(ea, P.stride_a, false) || !inside(eo, P.stride_b, true)) return fail();
                                // a moved-back vector repeats its neighbour's elements: same source, same instruction
                                // if B is read as well as written
                                if (b_from_a[eo] != -1 && (b_from_a[eo] != ea || (axpby && writer[eo] != who))) return fail();
                                if (b_from_a[eo] == -1) ++written;
                                b_from_a[eo] = ea;
                                writer[eo] = who;
                            }
                        };
                        emu_walk(p.a, L, la, wm, tab_a.data(), tabc_a.data(), wave, st, nop);
                    }
                continue;
            }
            std::fill(lds.begin(), lds.end(), (int64_t)-1);
            for (uint32_t wave = 0; wave < nwave; ++wave)
                for (uint32_t lane = 0; lane < (uint32_t)kWave; ++lane) {
                    const LaneState L = lane_setup<false>(p.a, lane, sc_a);
                    const WalkMask wm = walk_mask(p.a, L, la);
                    auto st = [&](int, const PosEntry& e, int back, bool ok) {
                        if (!ok) return;
                        const int64_t oa = base_a + e.g + L.g;
                        const int64_t lo = (int64_t)(int32_t)e.l_or_g2 + L.l;
                        if (oa % eba || lo % eba || back < 0 || back >= p.a.vec) return fail();
                        if (lo < 0 || lo >= lds_bytes) return fail();
                        for (int j = -back; j < p.a.vec - back; ++j) {
                            const int64_t ea = oa / eba + j;
                            if (!inside(ea, P.stride_a, false)) return fail();
                            const int64_t li = lo / eba + (int64_t)j * p.a.vec_lds_stride;
                            if (li < 0 || li >= p.lds_tile_elems) return fail();
                            if (lds[li] != -1 && lds[li] != ea) return fail();
                            lds[li] = ea;
                        }
                    };
                    emu_walk(p.a, L, la, wm, tab_a.data(), tabc_a.data(), wave, st, nop);
                }
            const SideLim lb = side_lim(p.b, tl);
            for (uint32_t wave = 0; wave < nwave; ++wave)
                for (uint32_t lane = 0; lane < (uint32_t)kWave; ++lane) {
                    const LaneState L = lane_setup<false>(p.b, lane, sc_b);
                    const WalkMask wm = walk_mask(p.b, L, lb);
                    auto st = [&](int, const PosEntry& e, int back, bool ok) {
                        if (!ok) return;
                        const int64_t ob = base_b + e.g + L.g;
                        const int64_t lo = (int64_t)(int32_t)e.l_or_g2 + L.l;
                        if (ob % ebb || lo % eba || back < 0 || back >= p.b.vec) return fail();
                        const int64_t who = ((int64_t)tile << 32) | (wave << 16) | (uint32_t)(&e - tab_b.data());
                        for (int j = -back; j < p.b.vec - back; ++j) {
                            const int64_t eo = ob / ebb + j;
                            if (!inside(eo, P.stride_b, true)) return fail();
                            const int64_t li = lo / eba + (int64_t)j * p.b.vec_lds_stride;
                            if (li < 0 || li >= p.lds_tile_elems) return fail();
                            if (lds[li] == -1) return fail();
                            if (b_from_a[eo] != -1 && (b_from_a[eo] != lds[li] || (axpby && writer[eo] != who))) return fail();
                            if (b_from_a[eo] == -1) ++written;
                            b_from_a[eo] = lds[li];
                            writer[eo] = who;
                        }
                    };
                    emu_walk(p.b, L, lb, wm, tab_b.data(), tabc_b.data(), wave, st, nop);
                }
        }
    }
#undef fail
    if (bad || written != P.elements) {
        if (std::getenv("TTC_EMU_DEBUG")) std::fprintf(stderr, "ttc_debug_emulate_map: check at line %d failed, %lld of %lld elements written\n", fail_line, (long long)written, (long long)P.elements);
        return TTC_ERR_INTERNAL;
    }
    return TTC_OK;
}
