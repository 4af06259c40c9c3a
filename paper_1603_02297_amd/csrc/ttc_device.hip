// Device side of the library for gfx950 (MI355X): the tile ("box") kernels, their launch,
// the timed search over candidates and the measurement helpers.
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
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ttc_internal.h"
#include "ttc_walk.h"

namespace ttc {

// ---------------------------------------------------------------------------------
// Element types and the alpha/beta epilogue (fixed evaluation order; built with
// -ffp-contract=off so the only fused operations are the ones written here).
//   real:    copy: r = a | scale: r = alpha*a | axpby: t = beta*b, r = fma(alpha, a, t)
//   complex: product z = s*x as z.re = fma(s.re, x.re, -(s.im*x.im)), z.im = fma(s.re, x.im, s.im*x.re);
//            scale: r = alpha*a | axpby: r = alpha*a + beta*b componentwise
// Mixed precision (A and B of different precision): elements are widened to double, the same
// formulas run in double, the result is rounded once (to nearest even) to B's type.
// ---------------------------------------------------------------------------------
struct alignas(8) cfloat { float re, im; };
struct alignas(8) cdouble { double re, im; };

// Global vectors are only guaranteed element alignment (gfx950 global dwordx2/x4 accesses need
// no more); the hardware runs them at full rate at any 4-byte boundary.
template <typename T, int V> struct alignas(alignof(T)) Pack { T v[V]; };

template <typename To, typename From> struct Convert;
template <typename T> struct Convert<T, T> { __device__ static __forceinline__ T go(T x) { return x; } };
template <> struct Convert<double, float> { __device__ static __forceinline__ double go(float x) { return (double)x; } };
template <> struct Convert<float, double> { __device__ static __forceinline__ float go(double x) { return (float)x; } };
template <> struct Convert<cdouble, cfloat> {
    __device__ static __forceinline__ cdouble go(cfloat x) { cdouble r; r.re = (double)x.re; r.im = (double)x.im; return r; }
};
template <> struct Convert<cfloat, cdouble> {
    __device__ static __forceinline__ cfloat go(cdouble x) { cfloat r; r.re = (float)x.re; r.im = (float)x.im; return r; }
};

__device__ __forceinline__ float fused(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fused(double a, double b, double c) { return __builtin_fma(a, b, c); }

// the arithmetic, in the type it runs in
template <typename C, int MODE> struct Core {                    // C = float or double
    C al, be;
    __device__ explicit Core(const KernelParams& p) : al((C)p.alpha[0]), be((C)p.beta[0]) {}
    __device__ __forceinline__ C operator()(C a, C b) const
    {
        if (MODE == TTC_EPI_COPY) return a;
        if (MODE == TTC_EPI_SCALE) return al * a;
        const C t = be * b;
        return fused(al, a, t);
    }
};

template <typename Z, typename R, int MODE> struct ComplexCore {  // Z = cfloat / cdouble over R = float / double
    R ar, ai, br, bi;
    __device__ explicit ComplexCore(const KernelParams& p)
        : ar((R)p.alpha[0]), ai((R)p.alpha[1]), br((R)p.beta[0]), bi((R)p.beta[1]) {}
    __device__ __forceinline__ Z operator()(Z a, Z b) const
    {
        if (MODE == TTC_EPI_COPY) return a;
        Z p;
        p.re = fused(ar, a.re, -(ai * a.im));
        p.im = fused(ar, a.im, ai * a.re);
        if (MODE == TTC_EPI_SCALE) return p;
        Z q;
        q.re = fused(br, b.re, -(bi * b.im));
        q.im = fused(br, b.im, bi * b.re);
        Z r;
        r.re = p.re + q.re;
        r.im = p.im + q.im;
        return r;
    }
};
template <int MODE> struct Core<cfloat, MODE> : ComplexCore<cfloat, float, MODE> { using ComplexCore<cfloat, float, MODE>::ComplexCore; };
template <int MODE> struct Core<cdouble, MODE> : ComplexCore<cdouble, double, MODE> { using ComplexCore<cdouble, double, MODE>::ComplexCore; };

// type the arithmetic runs in: the common type, or the double-precision one when they differ
template <typename TA, typename TB> struct Wider;
template <typename T> struct Wider<T, T> { using type = T; };
template <> struct Wider<float, double> { using type = double; };
template <> struct Wider<double, float> { using type = double; };
template <> struct Wider<cfloat, cdouble> { using type = cdouble; };
template <> struct Wider<cdouble, cfloat> { using type = cdouble; };

template <typename TA, typename TB, int MODE> struct Epilogue {
    using C = typename Wider<TA, TB>::type;
    Core<C, MODE> core;
    __device__ explicit Epilogue(const KernelParams& p) : core(p) {}
    __device__ __forceinline__ TB operator()(TA a, TB b) const
    {
        return Convert<TB, C>::go(core(Convert<C, TA>::go(a), Convert<C, TB>::go(b)));
    }
};

// ---------------------------------------------------------------------------------
// The kernel.  Dynamic LDS: [two shared tile records][position tables of both walks][tile buffer 0][tile buffer 1].
// Cut vectors: where a run is not a multiple of the vector width, the lane that would overhang moves its
// vector back so that it ends with the run (`back` elements, handed to the stages).  It then repeats what
// its neighbour does for those elements, with the same values, so nothing diverges and every access stays a
// full vector.
// A workgroup walks several tiles; with two tile buffers one barrier per tile is enough: a
// wavefront can only start filling buffer (t+1)%2 after it passed the barrier of tile t, and
// every wavefront reached that barrier after it had finished reading that buffer for tile t-1.
// ---------------------------------------------------------------------------------
// memory instructions a wavefront keeps in flight per walk step: four 16-byte accesses per lane, more of the
// narrow ones (the bytes in flight per wavefront are what hides the memory latency)
template <typename T, int V> struct Unroll { static constexpr int value = (V * sizeof(T) >= 16) ? 4 : 8; };

__device__ __forceinline__ int64_t uniform64(int64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <typename T, int V>
__device__ __forceinline__ Pack<T, V> load_pack(const unsigned char* base, int64_t off)
{
    return *reinterpret_cast<const Pack<T, V>*>(base + off);
}

template <typename TA, typename TB, int MODE, int VA, int VB, bool DIRECT>
__global__ __launch_bounds__(kMaxThreads) void box_kernel(const KernelParams p, const TA* __restrict__ A,
                                                          TB* __restrict__ B)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int32_t kScaleA = (int32_t)sizeof(TA), kScaleB = (int32_t)sizeof(TB);
    const Scales sc_a = {kScaleA, kScaleB, kScaleA};     // walk over A; the LDS tile holds elements of A
    const Scales sc_b = {kScaleB, kScaleB, kScaleA};     // walk over B
    const uint32_t nwave = blockDim.x >> 6;
    const uint32_t n_a = nwave * (uint32_t)p.a.chunk, n_b = DIRECT ? 0u : nwave * (uint32_t)p.b.chunk;
    TileShare* share = reinterpret_cast<TileShare*>(smem);            // two slots, kTileShareBytes in all
    PosEntry* tab_a = reinterpret_cast<PosEntry*>(smem + kTileShareBytes);
    PosEntry* tab_b = tab_a + n_a;
    PosCoord* tabc_a = reinterpret_cast<PosCoord*>(tab_b + n_b);
    PosCoord* tabc_b = tabc_a + n_a;

    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    build_tables<DIRECT>(p.a, nwave, threadIdx.x, blockDim.x, sc_a, tab_a, tabc_a);
    if (!DIRECT) build_tables<false>(p.b, nwave, threadIdx.x, blockDim.x, sc_b, tab_b, tabc_b);
    const LaneState LA = lane_setup<DIRECT>(p.a, lane, sc_a);
    const LaneState LB = DIRECT ? LA : lane_setup<false>(p.b, lane, sc_b);
    const Epilogue<TA, TB, MODE> epi(p);
    const TileSeq seq = tile_sequence(p, blockIdx.x);

    // Staged kernel: the last wavefront works out where a tile lies (scalar divisions and
    // multiplications) one tile ahead and leaves the result in LDS; the barrier that already
    // separates the two walks of the current tile publishes it to the other wavefronts.
    auto publish = [&](uint32_t tile, uint32_t slot) {
        const TileBase tb = tile_base(p, tile);
        const TileLim tl = tile_lim(p, tile);
        TileShare v;
        v.a = tb.a; v.b = tb.b;
        v.lim[0] = tl.lim[0]; v.lim[1] = tl.lim[1]; v.lim[2] = tl.lim[2]; v.lim[3] = tl.lim[3];
        share[slot] = v;
    };
    if (!DIRECT && wave == nwave - 1 && seq.first < seq.end) publish(seq.first, 0);
    __syncthreads();

    uint32_t parity = 0;
    for (uint32_t tile = seq.first; tile < seq.end; tile += seq.step) {
        TileBase tb;
        TileLim tl;
        if (DIRECT) {
            tb = tile_base(p, tile);
            tl = tile_lim(p, tile);
        } else {
            const TileShare v = share[parity];
            tb.a = uniform64(v.a); tb.b = uniform64(v.b);
            tl.lim[0] = __builtin_amdgcn_readfirstlane(v.lim[0]); tl.lim[1] = __builtin_amdgcn_readfirstlane(v.lim[1]);
            tl.lim[2] = __builtin_amdgcn_readfirstlane(v.lim[2]); tl.lim[3] = __builtin_amdgcn_readfirstlane(v.lim[3]);
            tl.whole = false;
        }
        const unsigned char* At = reinterpret_cast<const unsigned char*>(A + tb.a);
        unsigned char* Bt = reinterpret_cast<unsigned char*>(B + tb.b);
        const SideLim sla = side_lim(p.a, tl);
        const WalkMask wma = walk_mask(p.a, LA, sla);
        if (DIRECT) {
            constexpr int kUnroll = Unroll<TA, VA>::value;
            Pack<TA, VA> ra[kUnroll];
            Pack<TB, VA> rb[kUnroll];
            auto load = [&](int u, const PosEntry& e, int back) {
                ra[u] = load_pack<TA, VA>(At, e.g + LA.g - back * kScaleA);
                if (MODE == TTC_EPI_AXPBY) rb[u] = load_pack<TB, VA>(Bt, e.l_or_g2 + LA.g2 - back * kScaleB);
            };
            auto store = [&](int u, const PosEntry& e, int back) {
                Pack<TB, VA> out;
#pragma unroll
                for (int j = 0; j < VA; ++j) {
                    TB old = TB();
                    if (MODE == TTC_EPI_AXPBY) old = rb[u].v[j];
                    out.v[j] = epi(ra[u].v[j], old);
                }
                *reinterpret_cast<Pack<TB, VA>*>(Bt + (e.l_or_g2 + LA.g2 - back * kScaleB)) = out;
            };
            walk<kUnroll, VA>(p.a, LA, sla, wma, tab_a, tabc_a, wave, load, store);
            continue;
        }

        unsigned char* lds = smem + p.lds_data_off +
                             (parity & (uint32_t)(p.lds_buffers - 1)) * (uint32_t)(p.lds_tile_elems * kScaleA);
        parity ^= 1u;
        // ---- walk 1: A order, global -> LDS
        {
            const int32_t vs = p.a.vec_lds_stride;
            constexpr int kUnroll = Unroll<TA, VA>::value;
            Pack<TA, VA> ra[kUnroll];
            auto load = [&](int u, const PosEntry& e, int back) { ra[u] = load_pack<TA, VA>(At, e.g + LA.g - back * kScaleA); };
            auto park = [&](int u, const PosEntry& e, int back) {
                TA* dst = reinterpret_cast<TA*>(lds + ((int32_t)e.l_or_g2 + LA.l - back * vs * kScaleA));
#pragma unroll
                for (int j = 0; j < VA; ++j) dst[j * vs] = ra[u].v[j];
            };
            walk<kUnroll, VA>(p.a, LA, sla, wma, tab_a, tabc_a, wave, load, park);
        }
        if (wave == nwave - 1 && tile + seq.step < seq.end) publish(tile + seq.step, parity);   // parity already flipped
        __syncthreads();
        // ---- walk 2: B order, LDS -> epilogue -> global
        {
            const SideLim slb = side_lim(p.b, tl);
            const WalkMask wmb = walk_mask(p.b, LB, slb);
            const int32_t vs = p.b.vec_lds_stride;
            constexpr int kUnroll = Unroll<TB, VB>::value;
            Pack<TB, VB> rb[kUnroll];
            Pack<TA, VB> rl[kUnroll];
            auto load = [&](int u, const PosEntry& e, int back) {
                if (MODE == TTC_EPI_AXPBY) rb[u] = load_pack<TB, VB>(Bt, e.g + LB.g - back * kScaleB);
                const TA* src = reinterpret_cast<const TA*>(lds + ((int32_t)e.l_or_g2 + LB.l - back * vs * kScaleA));
#pragma unroll
                for (int j = 0; j < VB; ++j) rl[u].v[j] = src[j * vs];
            };
            auto store = [&](int u, const PosEntry& e, int back) {
                Pack<TB, VB> out;
#pragma unroll
                for (int j = 0; j < VB; ++j) {
                    TB old = TB();
                    if (MODE == TTC_EPI_AXPBY) old = rb[u].v[j];
                    out.v[j] = epi(rl[u].v[j], old);
                }
                *reinterpret_cast<Pack<TB, VB>*>(Bt + (e.g + LB.g - back * kScaleB)) = out;
            };
            walk<kUnroll, VB>(p.b, LB, slb, wmb, tab_b, tabc_b, wave, load, store);
        }
        if (p.lds_buffers == 1) __syncthreads();      // the one buffer is refilled by the next tile
    }
}

// Compute units of the current device (256 on MI355X), asked once per process and device.
static int device_cus()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

// ---------------------------------------------------------------------------------
// Dispatch
// ---------------------------------------------------------------------------------
using KernelFn = void (*)(const KernelParams, const void*, void*);

template <typename TA, typename TB, int MODE, int VA, int VB, bool DIRECT>
static hipError_t launch_one(const KernelParams& kp, const void* A, void* B, uint32_t grid, int threads,
                             int lds_bytes, hipStream_t stream)
{
    if (grid != kp.grid || grid < 1 || grid > kp.num_tiles) return hipErrorInvalidValue;
    hipLaunchKernelGGL((box_kernel<TA, TB, MODE, VA, VB, DIRECT>), dim3(grid), dim3(threads), (size_t)lds_bytes, stream,
                       kp, static_cast<const TA*>(A), static_cast<TB*>(B));
    return hipGetLastError();
}

// VMAXA / VMAXB: elements of each type in 16 bytes
template <typename TA, typename TB, int MODE, int VMAXA, int VMAXB>
static hipError_t launch_vec(const Candidate& c, const void* A, void* B, hipStream_t s)
{
    KernelParams kp = c.kp;
    const uint32_t grid = launch_grid(c, device_cus());
    set_grid(&kp, grid);
    const int va = kp.a.vec, vb = kp.b.vec;
    constexpr int VD = VMAXA < VMAXB ? VMAXA : VMAXB;      // direct kernel: one width for both sides
    if (c.kernel_class == TTC_KERNEL_DIRECT) {
        if (va == 1) return launch_one<TA, TB, MODE, 1, 1, true>(kp, A, B, grid, c.threads, c.lds_bytes, s);
        if (va == 2 && VD >= 2) return launch_one<TA, TB, MODE, (VD >= 2 ? 2 : 1), (VD >= 2 ? 2 : 1), true>(kp, A, B, grid, c.threads, c.lds_bytes, s);
        if (va == 4 && VD >= 4) return launch_one<TA, TB, MODE, (VD >= 4 ? 4 : 1), (VD >= 4 ? 4 : 1), true>(kp, A, B, grid, c.threads, c.lds_bytes, s);
        return hipErrorInvalidValue;
    }
#define TTC_CASE(VA_, VB_)                                                                                   \
    if (va == VA_ && vb == VB_ && VA_ <= VMAXA && VB_ <= VMAXB)                                              \
        return launch_one<TA, TB, MODE, (VA_ <= VMAXA ? VA_ : 1), (VB_ <= VMAXB ? VB_ : 1), false>(          \
            kp, A, B, grid, c.threads, c.lds_bytes, s);
    TTC_CASE(1, 1) TTC_CASE(1, 2) TTC_CASE(2, 1) TTC_CASE(2, 2)
    TTC_CASE(1, 4) TTC_CASE(2, 4) TTC_CASE(4, 1) TTC_CASE(4, 2) TTC_CASE(4, 4)
#undef TTC_CASE
    return hipErrorInvalidValue;
}

template <typename TA, typename TB, int VMAXA, int VMAXB>
static hipError_t launch_mode(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s)
{
    switch (P.epilogue) {
    case TTC_EPI_COPY:  return launch_vec<TA, TB, TTC_EPI_COPY, VMAXA, VMAXB>(c, A, B, s);
    case TTC_EPI_SCALE: return launch_vec<TA, TB, TTC_EPI_SCALE, VMAXA, VMAXB>(c, A, B, s);
    default:            return launch_vec<TA, TB, TTC_EPI_AXPBY, VMAXA, VMAXB>(c, A, B, s);
    }
}

static hipError_t launch(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s)
{
    if (c.threads < kWave || c.threads > kMaxThreads || (c.threads % kWave) != 0) return hipErrorInvalidValue;
    if (c.lds_bytes > kMaxLdsBytes) return hipErrorInvalidValue;
    switch (P.dtype) {
    case TTC_F32:      return launch_mode<float, float, 4, 4>(P, c, A, B, s);
    case TTC_F64:      return launch_mode<double, double, 2, 2>(P, c, A, B, s);
    case TTC_C64:      return launch_mode<cfloat, cfloat, 2, 2>(P, c, A, B, s);
    case TTC_C128:     return launch_mode<cdouble, cdouble, 1, 1>(P, c, A, B, s);
    case TTC_F32_F64:  return launch_mode<float, double, 4, 2>(P, c, A, B, s);
    case TTC_F64_F32:  return launch_mode<double, float, 2, 4>(P, c, A, B, s);
    case TTC_C64_C128: return launch_mode<cfloat, cdouble, 2, 1>(P, c, A, B, s);
    case TTC_C128_C64: return launch_mode<cdouble, cfloat, 1, 2>(P, c, A, B, s);
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

static const Candidate& pick_candidate(const ttc_plan_s* plan, const void* A, const void* B)
{
    (void)A; (void)B;
    return plan->cands[plan->selected];
}

// ---------------------------------------------------------------------------------
// Ceiling kernels
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n)
{
    const int64_t base = (int64_t)blockIdx.x * (256 * 4) + threadIdx.x;
    uint4 r[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) if (base + u * 256 < n) r[u] = src[base + u * 256];
#pragma unroll
    for (int u = 0; u < 4; ++u) if (base + u * 256 < n) dst[base + u * 256] = r[u];
}

__global__ __launch_bounds__(256) void axpby_kernel(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n)
{
    const int64_t base = (int64_t)blockIdx.x * (256 * 4) + threadIdx.x;
    float4 r[4], w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) if (base + u * 256 < n) { r[u] = src[base + u * 256]; w[u] = dst[base + u * 256]; }
#pragma unroll
    for (int u = 0; u < 4; ++u) if (base + u * 256 < n) {
        float4 o;
        o.x = __builtin_fmaf(0.75f, r[u].x, 1.25f * w[u].x);
        o.y = __builtin_fmaf(0.75f, r[u].y, 1.25f * w[u].y);
        o.z = __builtin_fmaf(0.75f, r[u].z, 1.25f * w[u].z);
        o.w = __builtin_fmaf(0.75f, r[u].w, 1.25f * w[u].w);
        dst[base + u * 256] = o;
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
    const ttc::Candidate& c = ttc::pick_candidate(plan, A, B);
    return ttc::launch(plan->prob, c, A, B, (hipStream_t)stream) == hipSuccess ? TTC_OK : TTC_ERR_HIP;
}

int ttc_plan_tune_pairs(ttc_plan_t plan, int npairs, const void* const* A_list, void* const* B_list,
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
    const int total = (int)plan->cands.size();
    if (cap < 0 || cap > total) cap = total;
    if (cap == 1) { plan->selected = 0; return TTC_OK; }
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
    // pass 1: every candidate briefly; pass 2: the fastest few again, longer, to beat the noise
    std::vector<std::pair<float, int>> timed;
    for (int i = 0; i < cap; ++i) {
        float ms = 0.f;
        const int st1 = time_one(plan->cands[i], 1, 3, &ms);
        if (st1 != TTC_OK) return st1;
        plan->cands[i].tuned_ms = ms;
        timed.emplace_back(ms, i);
    }
    std::sort(timed.begin(), timed.end());
    int best = -1;
    float best_ms = 0.f;
    const int finalists = std::min<int>(8, (int)timed.size());
    for (int k = 0; k < finalists; ++k) {
        const int i = timed[k].second;
        float ms = 0.f;
        const int st2 = time_one(plan->cands[i], 2, 12, &ms);
        if (st2 != TTC_OK) return st2;
        plan->cands[i].tuned_ms = ms;
        if (best < 0 || ms < best_ms) { best = i; best_ms = ms; }
    }
    if (best >= 0) plan->selected = best;
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
    if (kind < 0 || kind > 2 || bytes < 16 || (bytes % 16) != 0 || npairs < 1 || warmup < 0 || iters < 1)
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
    auto one = [&](int i) -> hipError_t {
        const void* src = src_list[i % npairs];
        void* dst = dst_list[i % npairs];
        if (kind == 0) {
            hipLaunchKernelGGL(ttc::copy_kernel, dim3(grid), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
            return hipGetLastError();
        }
        if (kind == 1) return hipMemcpyAsync(dst, src, (size_t)bytes, hipMemcpyDeviceToDevice, s);
        hipLaunchKernelGGL(ttc::axpby_kernel, dim3(grid), dim3(256), 0, s, (const float4*)src, (float4*)dst, n);
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
