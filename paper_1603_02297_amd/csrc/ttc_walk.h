// Index arithmetic of a tile walk, shared by the device kernels and by the host-side
// bounds checker (ttc_debug_emulate_map), so that what the checker proves in bounds is
// the code the GPU runs.
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

// workgroup id -> tile id.  Consecutive workgroup ids land on consecutive XCDs; every XCD gets
// one contiguous range of tiles so that neighbouring tiles share its L2.
TTC_HD uint32_t tile_of_workgroup(const KernelParams& p, uint32_t wg)
{
    if (!p.xcd_remap) return wg;
    const uint32_t x = wg & 7u, slot = wg >> 3;
    return x * p.tiles_per_xcd + (x < p.tiles_rem_xcd ? x : p.tiles_rem_xcd) + slot;
}

// tile id -> base offsets of the box in A and B and the part of the box inside the tensor
struct TilePos { int64_t base_a, base_b; int32_t lim[kMaxDim]; };

TTC_HD TilePos tile_pos(const KernelParams& p, uint32_t tile)
{
    TilePos t;
    t.base_a = 0; t.base_b = 0;
#pragma unroll
    for (int k = 0; k < kMaxDim; ++k) {
        t.lim[k] = 1;
        if (k < p.n) {
            const int64_t origin = (int64_t)fdigit(tile, p.tile_below[k], p.tile_cnt[k]) * p.tile[k];
            t.base_a += origin * p.stride_a[k];
            t.base_b += origin * p.stride_b[k];
            const int64_t left = p.size[k] - origin;
            t.lim[k] = (int32_t)(left < (int64_t)p.tile[k] ? left : (int64_t)p.tile[k]);
        }
    }
    return t;
}

// What one lane keeps for a walk: its fixed coordinates inside the wavefront's sub-box.
struct LaneState {
    int64_t g;                 // offset (elements) into the tensor the walk follows
    int64_t g2;                // direct kernel: offset into B
    int32_t l;                 // offset into the LDS tile
    int32_t c[kMaxDim];        // coordinate along each index, in elements
    bool    active;
};

template <bool DIRECT>
TTC_HD LaneState lane_setup(const KernelParams& p, const Side& s, const int64_t* stride, uint32_t lane)
{
    LaneState L;
    L.g = 0; L.g2 = 0; L.l = 0;
    L.active = lane < (uint32_t)s.lanes;
#pragma unroll
    for (int k = 0; k < kMaxDim; ++k) {
        L.c[k] = 0;
        if (k < p.n && s.lane[k] > 1) {
            const int32_t c = (int32_t)fdigit(lane, s.lane_below[k], s.lane_cnt[k]) * s.lane_mul[k];
            L.c[k] = c;
            L.g += (int64_t)c * stride[k];
            if (DIRECT) L.g2 += (int64_t)c * p.stride_b[k];
            else L.l += c * p.lds_stride[k];
        }
    }
    return L;
}

// Position of the wavefront's sub-box for iteration `it` of a walk (wave-uniform), and whether
// this lane's element(s) fall inside the tile and the tensor.
struct IterPos { int64_t g, g2; int32_t l; bool valid; };

template <bool DIRECT>
TTC_HD IterPos iter_pos(const KernelParams& p, const Side& s, const int64_t* stride, const int32_t* lim,
                        const LaneState& L, uint32_t it)
{
    IterPos r;
    r.g = 0; r.g2 = 0; r.l = 0;
    r.valid = L.active;
#pragma unroll
    for (int k = 0; k < kMaxDim; ++k) {
        if (k < p.n && p.tile[k] > 1) {
            int32_t base = 0;
            if (s.iters[k].div > 1) {
                base = (int32_t)fdigit(it, s.iter_below[k], s.iters[k]) * s.lane[k];
                r.g += (int64_t)base * stride[k];
                if (DIRECT) r.g2 += (int64_t)base * p.stride_b[k];
                else r.l += base * p.lds_stride[k];
            }
            r.valid = r.valid && (L.c[k] < lim[k] - base);
        }
    }
    return r;
}

}  // namespace ttc
