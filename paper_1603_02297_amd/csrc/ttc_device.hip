// Device side of the library for gfx950 (MI355X): launch dispatch, the timed search over candidates
// and the measurement helpers.  The tile ("box") kernels live in ttc_kernels.h.
//
// One kernel template serves both cases of the paper's Section 3.1.
//   * staged (stride-1 index changes):  a workgroup owns one box of the tensor that spans the
//     leading indices of A *and* of B.  Wavefronts walk the box in A order with vector loads
//     (lanes along A's stride-1 index), park it in LDS, and after one barrier walk it again in B
//     order (lanes along B's stride-1 index), apply the alpha/beta epilogue and store vectors.
//   * direct (stride-1 index fixed, or 1-D):  the same walk, but every lane stores what it
//     loaded; no LDS, no barrier.
// A walk is factorised CDNA-style: the 64 lanes of a wavefront cover a fixed sub-box (lane
// offsets are computed once and live in VGPRs), and the position of that sub-box inside the
// tile is wave-uniform, so the per-instruction index arithmetic runs on the scalar unit.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <new>
#include <cstring>
#include <vector>

#include "ttc_internal.h"
#include "ttc_walk.h"

namespace ttc {

// One launcher per group of element types, each in its own translation unit (ttc_launch_*.hip).
hipError_t launch_f32(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s);
hipError_t launch_f64(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s);
hipError_t launch_c64(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s);
hipError_t launch_c128(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s);
hipError_t launch_mixed_real(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s);
hipError_t launch_mixed_complex(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s);

static hipError_t launch(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s)
{
    if (c.threads < kWave || c.threads > kMaxThreads || (c.threads % kWave) != 0) return hipErrorInvalidValue;
    if (c.lds_bytes < 0 || c.lds_bytes > kMaxLdsBytes) return hipErrorInvalidValue;
    switch (P.dtype) {
    case TTC_F32:      return launch_f32(P, c, A, B, s);
    case TTC_F64:      return launch_f64(P, c, A, B, s);
    case TTC_C64:      return launch_c64(P, c, A, B, s);
    case TTC_C128:     return launch_c128(P, c, A, B, s);
    case TTC_F32_F64:
    case TTC_F64_F32:  return launch_mixed_real(P, c, A, B, s);
    case TTC_C64_C128:
    case TTC_C128_C64: return launch_mixed_complex(P, c, A, B, s);
    default: return hipErrorInvalidValue;
    }
}

static int check_buffers(const ttc_plan_s* plan, const void* A, const void* B)
{
    if (!plan || !A || !B) return TTC_ERR_NULL_POINTER;
    const Problem& P = plan->prob;
    const uintptr_t a = (uintptr_t)A, b = (uintptr_t)B;
    // element alignment; complex64 pairs move as 8-byte units, complex128 as two of them
    if (a % (uintptr_t)std::min(P.eb_a, 8) || b % (uintptr_t)std::min(P.eb_b, 8)) return TTC_ERR_MISALIGNED;
    const uintptr_t bytes_a = (uintptr_t)P.span_a * P.eb_a, bytes_b = (uintptr_t)P.span_b * P.eb_b;
    if (a < b + bytes_b && b < a + bytes_a) return TTC_ERR_ALIAS;
    return TTC_OK;
}

// ---------------------------------------------------------------------------------
// Ceiling kernels
// ---------------------------------------------------------------------------------
// Both copies are persistent: a workgroup moves 16 KB (four 16-byte accesses per lane in flight, no bounds test
// except in the last, partial chunk), then takes the chunk one grid further on.  Measured 4-15 % faster than
// one chunk per workgroup.
template <bool NT>
__device__ __forceinline__ void copy_chunks(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n)
{
    typedef uint32_t W __attribute__((ext_vector_type(4)));
    const W* s4 = reinterpret_cast<const W*>(src);
    W* d4 = reinterpret_cast<W*>(dst);
    const int64_t chunk = 256 * 4;
    for (int64_t c0 = (int64_t)blockIdx.x * chunk; c0 < n; c0 += (int64_t)gridDim.x * chunk) {
        const int64_t base = c0 + threadIdx.x;
        W r[4];
        if (c0 + chunk <= n) {
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] = NT ? __builtin_nontemporal_load(s4 + base + u * 256) : s4[base + u * 256];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (NT) __builtin_nontemporal_store(r[u], d4 + base + u * 256); else d4[base + u * 256] = r[u];
            }
        } else {
            for (int u = 0; u < 4; ++u)
                if (base + u * 256 < n) d4[base + u * 256] = s4[base + u * 256];
        }
    }
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n)
{
    copy_chunks<false>(src, dst, n);
}

// the same copy with the non-temporal hint on both sides (a copy reuses nothing)
__global__ __launch_bounds__(256) void copy_stream_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n)
{
    copy_chunks<true>(src, dst, n);
}

// one 16-byte access per lane, one 4 KB chunk per workgroup, non-temporal: nothing persistent, the hardware deals
// the chunks (the launch shape of the row kernel); the faster copy on the largest tensors
__global__ __launch_bounds__(256) void copy_oneshot_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n)
{
    typedef uint32_t W __attribute__((ext_vector_type(4)));
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const W*>(src) + i), reinterpret_cast<W*>(dst) + i);
}

// dst <- 0.75 * src + 1.25 * dst with non-temporal accesses, one 16-byte access per lane and side, one 4 KB chunk
// per one-shot workgroup (the launch shape of the fastest copy)
__global__ __launch_bounds__(256) void axpby_oneshot_kernel(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n)
{
    typedef float W __attribute__((ext_vector_type(4)));
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) {
        const W r = __builtin_nontemporal_load(reinterpret_cast<const W*>(src) + i);
        const W w = __builtin_nontemporal_load(reinterpret_cast<const W*>(dst) + i);
        W o;
        o.x = __builtin_fmaf(0.75f, r.x, 1.25f * w.x);
        o.y = __builtin_fmaf(0.75f, r.y, 1.25f * w.y);
        o.z = __builtin_fmaf(0.75f, r.z, 1.25f * w.z);
        o.w = __builtin_fmaf(0.75f, r.w, 1.25f * w.w);
        __builtin_nontemporal_store(o, reinterpret_cast<W*>(dst) + i);
    }
}

__global__ __launch_bounds__(256) void axpby_kernel(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n)
{
    const int64_t chunk = 256 * 4;
    auto fused = [](const float4& r, const float4& w) {
        float4 o;
        o.x = __builtin_fmaf(0.75f, r.x, 1.25f * w.x);
        o.y = __builtin_fmaf(0.75f, r.y, 1.25f * w.y);
        o.z = __builtin_fmaf(0.75f, r.z, 1.25f * w.z);
        o.w = __builtin_fmaf(0.75f, r.w, 1.25f * w.w);
        return o;
    };
    for (int64_t c0 = (int64_t)blockIdx.x * chunk; c0 < n; c0 += (int64_t)gridDim.x * chunk) {
        const int64_t base = c0 + threadIdx.x;
        if (c0 + chunk <= n) {
            float4 r[4], w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { r[u] = src[base + u * 256]; w[u] = dst[base + u * 256]; }
#pragma unroll
            for (int u = 0; u < 4; ++u) dst[base + u * 256] = fused(r[u], w[u]);
        } else {
            for (int u = 0; u < 4; ++u)
                if (base + u * 256 < n) dst[base + u * 256] = fused(src[base + u * 256], dst[base + u * 256]);
        }
    }
}

struct EventPair {
    hipEvent_t start = nullptr, stop = nullptr;
    bool ok = false;
    EventPair() { ok = hipEventCreate(&start) == hipSuccess && hipEventCreate(&stop) == hipSuccess; }
    ~EventPair() { if (start) (void)hipEventDestroy(start); if (stop) (void)hipEventDestroy(stop); }
};

}  // namespace ttc

// ---------------------------------------------------------------------------------
// Device part of the C ABI
// ---------------------------------------------------------------------------------
extern "C" {

int ttc_execute(ttc_plan_t plan, const void* A, void* B, void* stream)
{
    const int st = ttc::check_buffers(plan, A, B);
    if (st != TTC_OK) return st;
    const ttc::Candidate& c = plan->cands[plan->selected];
    return ttc::launch(plan->prob, c, A, B, (hipStream_t)stream) == hipSuccess ? TTC_OK : TTC_ERR_HIP;
}

static int tune_pairs(ttc_plan_t plan, int npairs, const void* const* A_list, void* const* B_list,
                      void* stream, int max_candidates);

int ttc_plan_tune_pairs(ttc_plan_t plan, int npairs, const void* const* A_list, void* const* B_list,
                        void* stream, int max_candidates)
{
    try { return tune_pairs(plan, npairs, A_list, B_list, stream, max_candidates); }
    catch (const std::bad_alloc&) { return TTC_ERR_ALLOC; }
    catch (...) { return TTC_ERR_INTERNAL; }
}

static int tune_pairs(ttc_plan_t plan, int npairs, const void* const* A_list, void* const* B_list,
                      void* stream, int max_candidates)
{
    if (!plan || !A_list || !B_list) return TTC_ERR_NULL_POINTER;
    if (npairs < 1) return TTC_ERR_INVALID_VALUE;
    for (int i = 0; i < npairs; ++i) {
        const int st = ttc::check_buffers(plan, A_list[i], B_list[i]);
        if (st != TTC_OK) return st;
    }
    hipStream_t s = (hipStream_t)stream;
    int cap = max_candidates;
    if (cap == 0) {
        const char* e = std::getenv("TTC_MAX_CANDIDATES");
        cap = e ? std::atoi(e) : 200;
        if (cap == 0) cap = 200;
    }
    if (cap == 1) return ttc_plan_select_candidate(plan, 0);         // the heuristic's choice, nothing timed
    const int st_list = ttc::complete_plan(plan);
    if (st_list != TTC_OK) return st_list;
    const int total = (int)plan->cands.size();
    if (cap < 0 || cap > total) cap = total;
    const char* store = std::getenv("TTC_PLAN_CACHE");
    if (store && *store && ttc::cache_lookup(plan, store) == TTC_OK) return TTC_OK;     // solved before
    ttc::EventPair ev;
    if (!ev.ok) return TTC_ERR_HIP;
    int turn = 0;
    // one launch configuration, timed: `warm` untimed launches, then the mean of `reps`
    auto time_one = [&](const ttc::Candidate& c, int warm, int reps, float* ms_out) -> int {
        for (int r = 0; r < warm; ++r, ++turn)
            if (ttc::launch(plan->prob, c, A_list[turn % npairs], B_list[turn % npairs], s) != hipSuccess) return TTC_ERR_HIP;
        if (hipEventRecord(ev.start, s) != hipSuccess) return TTC_ERR_HIP;
        for (int r = 0; r < reps; ++r, ++turn)
            if (ttc::launch(plan->prob, c, A_list[turn % npairs], B_list[turn % npairs], s) != hipSuccess) return TTC_ERR_HIP;
        if (hipEventRecord(ev.stop, s) != hipSuccess) return TTC_ERR_HIP;
        if (hipEventSynchronize(ev.stop) != hipSuccess) return TTC_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev.start, ev.stop) != hipSuccess) return TTC_ERR_HIP;
        *ms_out = ms / reps;
        return TTC_OK;
    };
    // pass 1: every candidate briefly; pass 2: the fastest few again, longer, to beat the noise.  Launches of a
    // few microseconds are repeated more often: both passes time at least 0.2 ms and 1 ms of work.
    float first_ms = 0.f;
    const int st0 = time_one(plan->cands[0], 2, 3, &first_ms);
    if (st0 != TTC_OK) return st0;
    const float unit = first_ms > 1e-4f ? first_ms : 1e-4f;
    {   // a GPU that has been idle runs its first milliseconds at low clocks (short launches measured 3-4x
        // slower there): keep it busy for about 3 ms before anything is compared
        float ignored = 0.f;
        const int st_warm = time_one(plan->cands[0], std::min(2000, std::max(1, (int)std::ceil(3.0f / unit))), 1, &ignored);
        if (st_warm != TTC_OK) return st_warm;
    }
    const int reps1 = std::min(40, std::max(3, (int)std::ceil(0.2f / unit)));
    const int reps2 = std::min(200, std::max(12, (int)std::ceil(1.0f / unit)));
    // What is timed: the `cap` best-ranked candidates; a fifth of the places goes to the best-ranked micro-tile
    // candidates over single indices, and another fifth to those over merged indices, where the ranking would have
    // left them out (the families are ranked by separate models, each good at ordering its own family and only
    // roughly calibrated against the others)
    std::vector<int> chosen;
    for (int i = 0; i < cap; ++i) chosen.push_back(i);
    if (cap >= 10 && cap < total) {
        auto family = [&](int i) {
            const ttc::Candidate& c = plan->cands[i];
            if (c.kernel_class != TTC_KERNEL_MICRO) return 0;
            return (c.kp.micro.merged_a || c.kp.micro.merged_b) ? 2 : 1;
        };
        std::vector<int> extra;
        for (int fam = 1; fam <= 2; ++fam) {
            int seen = 0;
            for (int i = 0; i < total && seen < cap / 5; ++i)
                if (family(i) == fam) {
                    ++seen;
                    if (i >= cap) extra.push_back(i);
                }
        }
        for (int k = cap - 1; k >= 1 && !extra.empty(); --k)
            if (family(chosen[k]) == 0) {
                chosen[k] = extra.back();
                extra.pop_back();
            }
    }
    std::vector<std::pair<float, int>> timed;
    for (int i : chosen) {
        ttc::Candidate& c = plan->cands[i];
        float ms = 0.f;
        const int st1 = time_one(c, 1, reps1, &ms);
        if (st1 != TTC_OK) return st1;
        // the streaming hints can be worth more than the choice of the tile (72^4 fp64 with beta != 0: 77 % of a copy
        // by the rule, 100 % with both sides streamed; 85^4: 66 % against 48 %): a candidate is ranked by the better
        // of the rule's hints and both sides streamed, so that pass 2 sees the right finalists
        if (!(c.kp.nt_a == 1 && c.kp.nt_b == 1)) {
            const int rule_a = c.kp.nt_a, rule_b = c.kp.nt_b;
            c.kp.nt_a = c.kp.nt_b = 1;
            float ms_nt = 0.f;
            const int st1b = time_one(c, 1, reps1, &ms_nt);
            c.kp.nt_a = rule_a; c.kp.nt_b = rule_b;
            if (st1b != TTC_OK) return st1b;
            if (ms_nt < ms) ms = ms_nt;
        }
        c.tuned_ms = ms;
        timed.emplace_back(ms, i);
    }
    std::sort(timed.begin(), timed.end());
    int best = -1;
    float best_ms = 0.f;
    const int finalists = std::min<int>(8, (int)timed.size());
    for (int k = 0; k < finalists; ++k) {
        const int i = timed[k].second;
        ttc::Candidate& c = plan->cands[i];
        // the rule's streaming hints, then none, all, and one side only (the direct kernel streams both sides or
        // neither): keep what is fastest for this candidate
        const int rule_a = c.kp.nt_a, rule_b = c.kp.nt_b;
        const int variants[5][2] = {{rule_a, rule_b}, {0, 0}, {1, 1}, {1, 0}, {0, 1}};
        const int nvariants = c.kernel_class == TTC_KERNEL_DIRECT ? 3 : 5;
        float cand_ms = 0.f;
        int keep_a = rule_a, keep_b = rule_b;
        for (int v = 0; v < nvariants; ++v) {
            if (v > 0 && variants[v][0] == rule_a && variants[v][1] == rule_b) continue;
            c.kp.nt_a = variants[v][0];
            c.kp.nt_b = variants[v][1];
            float ms = 0.f;
            const int st2 = time_one(c, 2, reps2, &ms);
            if (st2 != TTC_OK) { c.kp.nt_a = rule_a; c.kp.nt_b = rule_b; return st2; }
            if (v == 0 || ms < cand_ms) { cand_ms = ms; keep_a = variants[v][0]; keep_b = variants[v][1]; }
        }
        c.kp.nt_a = keep_a;
        c.kp.nt_b = keep_b;
        // the same for the mapping of tiles to XCDs: the default (chunks of 32 if there are enough tiles), one
        // range per XCD, chunks of 8
        const int mapping0 = c.kp.xcd_remap;
        int keep_map = mapping0;
        for (int mode : {1, 3}) {
            if (c.kernel_class == TTC_KERNEL_ROWS) break;           // no tiles to deal
            if (mode == mapping0 || !ttc::set_tile_mapping(&c.kp, mode)) continue;
            float ms = 0.f;
            const int st3 = time_one(c, 2, reps2, &ms);
            if (st3 != TTC_OK) { (void)ttc::set_tile_mapping(&c.kp, mapping0); return st3; }
            if (ms < cand_ms) { cand_ms = ms; keep_map = mode; }
        }
        (void)ttc::set_tile_mapping(&c.kp, keep_map);
        c.tuned_ms = cand_ms;
        if (best < 0 || cand_ms < best_ms) { best = i; best_ms = cand_ms; }
    }
    if (best >= 0) plan->selected = best;
    if (ttc::verbose())
        std::fprintf(stderr, "ttc: search timed %d of %d candidates, selected %d (%.4f ms)\n", cap, total, plan->selected, best_ms);
    if (store && *store) (void)ttc::cache_store(plan, store);       // a store that cannot be written costs a later search, no more
    return TTC_OK;
}

int ttc_plan_tune(ttc_plan_t plan, const void* A, void* B, void* stream, int max_candidates)
{
    return ttc_plan_tune_pairs(plan, 1, &A, &B, stream, max_candidates);
}

int ttc_time_execute(ttc_plan_t plan, int npairs, const void* const* A_list, void* const* B_list,
                     void* stream, int warmup, int iters, float* ms_per_launch)
{
    if (!plan || !A_list || !B_list || !ms_per_launch) return TTC_ERR_NULL_POINTER;
    if (npairs < 1 || warmup < 0 || iters < 1) return TTC_ERR_INVALID_VALUE;
    for (int i = 0; i < npairs; ++i) {
        const int st = ttc::check_buffers(plan, A_list[i], B_list[i]);
        if (st != TTC_OK) return st;
    }
    hipStream_t s = (hipStream_t)stream;
    ttc::EventPair ev;
    if (!ev.ok) return TTC_ERR_HIP;
    for (int i = 0; i < warmup; ++i) {
        const int st = ttc_execute(plan, A_list[i % npairs], B_list[i % npairs], stream);
        if (st != TTC_OK) return st;
    }
    if (hipEventRecord(ev.start, s) != hipSuccess) return TTC_ERR_HIP;
    for (int i = 0; i < iters; ++i) {
        const int st = ttc_execute(plan, A_list[(warmup + i) % npairs], B_list[(warmup + i) % npairs], stream);
        if (st != TTC_OK) return st;
    }
    if (hipEventRecord(ev.stop, s) != hipSuccess) return TTC_ERR_HIP;
    if (hipEventSynchronize(ev.stop) != hipSuccess) return TTC_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ev.start, ev.stop) != hipSuccess) return TTC_ERR_HIP;
    *ms_per_launch = ms / iters;
    return TTC_OK;
}

int ttc_time_ceiling(int kind, int64_t bytes, int npairs, const void* const* src_list, void* const* dst_list,
                     void* stream, int warmup, int iters, float* ms_per_launch)
{
    if (!src_list || !dst_list || !ms_per_launch) return TTC_ERR_NULL_POINTER;
    if (kind < 0 || kind > 5 || bytes < 16 || (bytes % 16) != 0 || npairs < 1 || warmup < 0 || iters < 1)
        return TTC_ERR_INVALID_VALUE;
    for (int i = 0; i < npairs; ++i) {
        if (!src_list[i] || !dst_list[i]) return TTC_ERR_NULL_POINTER;
        const uintptr_t a = (uintptr_t)src_list[i], b = (uintptr_t)dst_list[i];
        if (a % 16 || b % 16) return TTC_ERR_MISALIGNED;
        if (a < b + (uintptr_t)bytes && b < a + (uintptr_t)bytes) return TTC_ERR_ALIAS;
    }
    hipStream_t s = (hipStream_t)stream;
    ttc::EventPair ev;
    if (!ev.ok) return TTC_ERR_HIP;
    const int64_t n = bytes / 16;
    const int64_t grid64 = (n + 1023) / 1024;
    if (grid64 > INT32_MAX) return TTC_ERR_OVERFLOW;
    const uint32_t grid = (uint32_t)grid64;
    const uint32_t copy_grid = std::min<uint32_t>(grid, 8192u);       // the copies loop over their chunks
    auto one = [&](int i) -> hipError_t {
        const void* src = src_list[i % npairs];
        void* dst = dst_list[i % npairs];
        if (kind == 0) {
            hipLaunchKernelGGL(ttc::copy_kernel, dim3(copy_grid), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
            return hipGetLastError();
        }
        if (kind == 1) return hipMemcpyAsync(dst, src, (size_t)bytes, hipMemcpyDeviceToDevice, s);
        if (kind == 3) {
            hipLaunchKernelGGL(ttc::copy_stream_kernel, dim3(copy_grid), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
            return hipGetLastError();
        }
        if (kind == 4) {
            const int64_t g = (n + 255) / 256;
            if (g > INT32_MAX) return hipErrorInvalidValue;
            hipLaunchKernelGGL(ttc::copy_oneshot_kernel, dim3((uint32_t)g), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
            return hipGetLastError();
        }
        if (kind == 5) {
            const int64_t g = (n + 255) / 256;
            if (g > INT32_MAX) return hipErrorInvalidValue;
            hipLaunchKernelGGL(ttc::axpby_oneshot_kernel, dim3((uint32_t)g), dim3(256), 0, s, (const float4*)src, (float4*)dst, n);
            return hipGetLastError();
        }
        hipLaunchKernelGGL(ttc::axpby_kernel, dim3(copy_grid), dim3(256), 0, s, (const float4*)src, (float4*)dst, n);
        return hipGetLastError();
    };
    for (int i = 0; i < warmup; ++i) if (one(i) != hipSuccess) return TTC_ERR_HIP;
    if (hipEventRecord(ev.start, s) != hipSuccess) return TTC_ERR_HIP;
    for (int i = 0; i < iters; ++i) if (one(warmup + i) != hipSuccess) return TTC_ERR_HIP;
    if (hipEventRecord(ev.stop, s) != hipSuccess) return TTC_ERR_HIP;
    if (hipEventSynchronize(ev.stop) != hipSuccess) return TTC_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ev.start, ev.stop) != hipSuccess) return TTC_ERR_HIP;
    *ms_per_launch = ms / iters;
    return TTC_OK;
}

}  // extern "C"
