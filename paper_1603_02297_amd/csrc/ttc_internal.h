// Internal declarations shared by the host planner (ttc_plan.cpp) and the device side
// (ttc_device.hip).  Nothing here is part of the C ABI.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "ttc.h"

namespace ttc {

constexpr int kMaxDim = TTC_MAX_DIM;
constexpr int kWave = 64;                 // CDNA wavefront
constexpr int kMaxThreads = 512;          // launch bound of every kernel
constexpr int kMaxLdsBytes = 64 * 1024;   // per workgroup; several workgroups share a CU's 160 KB

// Exact unsigned division by a run-time constant d >= 1 for any 32-bit x whose
// quotient sum does not overflow (x < 2^31 is enough):
//   q = (mulhi(x, mul) + x) >> shift,   mul = floor(2^32 (2^shift - d) / d) + 1,  shift = ceil(log2 d).
struct FastDiv {
    uint32_t mul;
    uint32_t shift;
    uint32_t div;
};
FastDiv make_fastdiv(uint32_t d);

// One way of walking the tile ("box"): which sub-box the 64 lanes of a wavefront cover
// with one memory instruction, and how many such instructions cover the box.  All arrays
// are indexed by fused index of A.  An index k outside the box has lane=1, iters=1.
struct Side {
    int32_t  vec;                    // elements per lane per access along vec_dim
    int32_t  lanes;                  // active lanes = prod(lane[k]) / vec
    int32_t  n_iter;                 // prod(iters[k])
    int32_t  vec_lds_stride;         // LDS stride (elements) between the vec elements of one lane
    int32_t  lane[kMaxDim];          // lane sub-box extent (elements); multiple of vec on vec_dim
    int32_t  lane_mul[kMaxDim];      // elements per lane step: vec on vec_dim, else 1
    FastDiv  lane_below[kMaxDim];    // prod of lane counts of the digits below k in this side's order
    FastDiv  lane_cnt[kMaxDim];      // lane count along k (lane[k] / lane_mul[k])
    FastDiv  iter_below[kMaxDim];    // prod of iters of the digits below k in this side's order
    FastDiv  iters[kMaxDim];         // ceil(tile[k] / lane[k])
};

// Everything a kernel launch needs; passed by value as the kernel argument.
struct KernelParams {
    int32_t  n;                      // fused number of indices
    int32_t  xcd_remap;
    uint32_t num_tiles;
    uint32_t tiles_per_xcd;          // num_tiles / 8
    uint32_t tiles_rem_xcd;          // num_tiles % 8
    int64_t  size[kMaxDim];          // fused extents
    int64_t  stride_a[kMaxDim];      // element stride of fused index k in A
    int64_t  stride_b[kMaxDim];      // element stride of fused index k in B
    int32_t  tile[kMaxDim];          // box extent (1 = index not blocked)
    int32_t  lds_stride[kMaxDim];    // element stride of index k in the LDS tile
    FastDiv  tile_below[kMaxDim];    // prod of tile counts of the indices that vary faster in the tile order
    FastDiv  tile_cnt[kMaxDim];      // ceil(size[k] / tile[k])
    Side     a;                      // load side (A order)
    Side     b;                      // store side (B order); unused by the direct kernel
    double   alpha[2];               // re, im (im = 0 for real types)
    double   beta[2];
};

// One candidate launch configuration ("candidate" in the paper's Section 3).
struct Candidate {
    int      kernel_class;           // TTC_KERNEL_*
    int      threads;
    int      lds_bytes;
    int      tile_order[kMaxDim];
    int      lds_conflict_a, lds_conflict_b;
    double   score;                  // heuristic cost, smaller is better
    float    tuned_ms;
    KernelParams kp;
};

struct Problem {
    int      dtype;
    int      elem_bytes;
    int      epilogue;               // TTC_EPI_*
    int      ndim;                   // fused
    int64_t  size[kMaxDim];
    int      perm[kMaxDim];
    int64_t  stride_a[kMaxDim];      // by fused index of A
    int64_t  stride_b[kMaxDim];      // by fused index of A (stride it has in B)
    int64_t  elements;
    double   alpha[2], beta[2];
};

}  // namespace ttc

struct ttc_plan_s {
    ttc::Problem prob;
    std::vector<ttc::Candidate> cands;     // ranked, best first
    int selected;
    int fallback;                          // index of a candidate with vec_a = vec_b = 1
};

namespace ttc {

// Host planner.  Returns TTC_OK and fills *out, or a status.
int build_plan(int dtype, int ndim, const int64_t* sizes, const int* perm,
               const void* alpha, const void* beta, ttc_plan_s* out);
void set_last_status(int status);

}  // namespace ttc
