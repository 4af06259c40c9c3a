// The tile ("box") kernels for gfx950 (MI355X) and their launch templates.  Included by one
// translation unit per group of element types (ttc_launch_*.hip), so that the groups compile in parallel.
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
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <climits>
#include <cstdlib>
#include <type_traits>

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
    __device__ Core(const double* alpha, const double* beta) : al((C)alpha[0]), be((C)beta[0]) {}
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
    __device__ ComplexCore(const double* alpha, const double* beta)
        : ar((R)alpha[0]), ai((R)alpha[1]), br((R)beta[0]), bi((R)beta[1]) {}
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
    __device__ Epilogue(const double* alpha, const double* beta) : core(alpha, beta) {}
    __device__ __forceinline__ TB operator()(TA a, TB b) const
    {
        return Convert<TB, C>::go(core(Convert<C, TA>::go(a), Convert<C, TB>::go(b)));
    }
};

// ---------------------------------------------------------------------------------
// The kernel.  Dynamic LDS: [two shared tile records][spare slots][position tables of both walks][tile buffer 0][tile buffer 1].
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

// Non-temporal accesses (the paper's streaming stores, Table 1 / Section 3.4, and their load counterpart):
// data that is touched once need not displace what neighbouring tiles will share.  The hint is a compile-time
// property of an access; a walk exists in both forms and the (wave-uniform) flag picks one per tile.
template <int N> struct Words;
template <> struct Words<1> { typedef uint32_t type; };
template <> struct Words<2> { typedef uint32_t type __attribute__((ext_vector_type(2), aligned(4))); };
template <> struct Words<4> { typedef uint32_t type __attribute__((ext_vector_type(4), aligned(4))); };
template <> struct Words<8> { typedef uint32_t type __attribute__((ext_vector_type(8), aligned(4))); };

template <typename T, int V, bool NT>
__device__ __forceinline__ Pack<T, V> load_pack(const unsigned char* base, int64_t off)
{
    typedef typename Words<V * sizeof(T) / 4>::type W;
    if (NT) {
        union { W w; Pack<T, V> p; } u;
        u.w = __builtin_nontemporal_load(reinterpret_cast<const W*>(base + off));
        return u.p;
    }
    return *reinterpret_cast<const Pack<T, V>*>(base + off);
}

template <typename T, int V, bool NT>
__device__ __forceinline__ void store_pack(unsigned char* base, int64_t off, const Pack<T, V>& v)
{
    typedef typename Words<V * sizeof(T) / 4>::type W;
    if (NT) {
        union { W w; Pack<T, V> p; } u;
        u.p = v;
        __builtin_nontemporal_store(u.w, reinterpret_cast<W*>(base + off));
    } else {
        *reinterpret_cast<Pack<T, V>*>(base + off) = v;
    }
}

// what one wavefront left in LDS about a tile and a walk, as the (wave-uniform) limits and the lane's own verdict
__device__ __forceinline__ void take_side(const SideShare& v, uint32_t single, const LaneState& L, SideLim* sl, WalkMask* wm)
{
    sl->lim[0] = __builtin_amdgcn_readfirstlane(v.lim[0]); sl->lim[1] = __builtin_amdgcn_readfirstlane(v.lim[1]);
    sl->lim[2] = __builtin_amdgcn_readfirstlane(v.lim[2]); sl->lim[3] = __builtin_amdgcn_readfirstlane(v.lim[3]);
    sl->t01 = __builtin_amdgcn_readfirstlane(v.t01); sl->t23 = __builtin_amdgcn_readfirstlane(v.t23);
    wm->dynamic = __builtin_amdgcn_readfirstlane(v.dynamic) != 0;
    wm->lane_ok = lane_inside(single, L, *sl);
}

template <typename TA, typename TB, int MODE, int VA, int VB, bool DIRECT>
__global__ __launch_bounds__(kMaxThreads) void box_kernel(const KernelParams params_by_value, const TA* __restrict__ A,
                                                          TB* __restrict__ B)
{
    // The parameter block is read where the launch put it, at the start of the kernel-argument segment (constant
    // memory, scalar loads).  Reading the by-value argument instead leaves it to the optimiser to see through the
    // copy the language asks for, and past a certain number of uses it keeps the copy: 1.4 KB of scratch per lane.
    const KernelParams& p = *reinterpret_cast<const KernelParams*>((const void*)__builtin_amdgcn_kernarg_segment_ptr());
    extern __shared__ __align__(16) unsigned char smem[];
    {   // Bring the whole parameter block into the scalar cache at once (read-only scalar loads of one word per
        // 64-byte line): the set-up code below reads it piece by piece, and each piece would otherwise be a miss.
        typedef const uint32_t __attribute__((address_space(4))) ConstWord;
        const ConstWord* args = (const ConstWord*)__builtin_amdgcn_kernarg_segment_ptr();
        uint32_t touched = 0;
#pragma unroll
        for (int i = 0; i < (int)(sizeof(KernelParams) / 64); ++i) touched ^= args[i * 16];
        asm volatile("" :: "s"(touched));
    }
    constexpr int32_t kScaleA = (int32_t)sizeof(TA), kScaleB = (int32_t)sizeof(TB);
    const Scales sc_a = {kScaleA, kScaleB, kScaleA};     // walk over A; the LDS tile holds elements of A
    const Scales sc_b = {kScaleB, kScaleB, kScaleA};     // walk over B
    const uint32_t nwave = blockDim.x >> 6;
    const uint32_t n_a = nwave * (uint32_t)p.a.chunk, n_b = DIRECT ? 0u : nwave * (uint32_t)p.b.chunk;
    TileShare* share = reinterpret_cast<TileShare*>(smem);            // two slots, kTileShareBytes in all
    PosEntry* tab_a = reinterpret_cast<PosEntry*>(smem + kTablesOff);
    PosEntry* tab_b = tab_a + n_a;
    PosCoord* tabc_a = reinterpret_cast<PosCoord*>(tab_b + n_b);
    PosCoord* tabc_b = tabc_a + n_a;

    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    build_tables<DIRECT>(p.a, nwave, threadIdx.x, blockDim.x, sc_a, tab_a, tabc_a);
    if (!DIRECT) build_tables<false>(p.b, nwave, threadIdx.x, blockDim.x, sc_b, tab_b, tabc_b);
    const LaneState LA = lane_setup<DIRECT>(p.a, lane, sc_a);
    const LaneState LB = DIRECT ? LA : lane_setup<false>(p.b, lane, sc_b);
    const Epilogue<TA, TB, MODE> epi(p.alpha, p.beta);
    const bool nt_a = p.nt_a != 0, nt_b = p.nt_b != 0;
    unsigned char* spare = smem + kTileShareBytes + lane * 16;      // where this lane parks what it must not keep
    const TileSeq seq = tile_sequence(p, blockIdx.x);

    // Staged kernel: the last wavefront works out where a tile lies (scalar divisions and
    // multiplications) one tile ahead and leaves the result in LDS; the barrier that already
    // separates the two walks of the current tile publishes it to the other wavefronts.
    auto publish = [&](uint32_t tile, uint32_t slot) __attribute__((always_inline)) {     // (not inlined, it would need the parameter block in memory)
        const TileBase tb = tile_base(p, tile);
        const TileLim tl = tile_lim(p, tile);
        TileShare v;
        v.a = tb.a; v.b = tb.b;
        v.sa = make_side_share(p.a, tl);
        v.sb = make_side_share(p.b, tl);
        share[slot] = v;
    };
    const uint32_t single_a = single_digits(p.a), single_b = DIRECT ? 0u : single_digits(p.b);
    if (!DIRECT && wave == nwave - 1 && seq.first < seq.end) publish(tile_of(seq, seq.first), 0);
    __syncthreads();
    if (p.debug_stop) return;

    uint32_t parity = 0;
    for (uint32_t q = seq.first; q < seq.end; q += seq.step) {
        const uint32_t tile = tile_of(seq, q);
        TileBase tb;
        SideLim sla, slb;
        WalkMask wma, wmb;
        if (DIRECT) {
            tb = tile_base(p, tile);
            const TileLim tl = tile_lim(p, tile);
            sla = side_lim(p.a, tl);
            wma = walk_mask(p.a, LA, sla);
            slb = sla; wmb = wma;
        } else {
            const TileShare v = share[parity];
            tb.a = uniform64(v.a); tb.b = uniform64(v.b);
            take_side(v.sa, single_a, LA, &sla, &wma);
            take_side(v.sb, single_b, LB, &slb, &wmb);
        }
        const unsigned char* At = reinterpret_cast<const unsigned char*>(A + tb.a);
        unsigned char* Bt = reinterpret_cast<unsigned char*>(B + tb.b);
        if (DIRECT) {
            auto run = [&](auto stream) {            // the direct kernel streams both tensors or neither
                constexpr bool NT = decltype(stream)::value;
                constexpr int kUnroll = Unroll<TA, VA>::value;
                Pack<TA, VA> ra[kUnroll];
                Pack<TB, VA> rb[kUnroll];
                auto load = [&](int u, const PosEntry& e, int back, bool ok) {
                    ra[u] = load_pack<TA, VA, NT>(At, ok ? e.g + LA.g - back * kScaleA : 0);
                    if (MODE == TTC_EPI_AXPBY) rb[u] = load_pack<TB, VA, NT>(Bt, ok ? e.l_or_g2 + LA.g2 - back * kScaleB : 0);
                };
                auto store = [&](int u, const PosEntry& e, int back, bool ok) {
                    if (!ok) return;
                    Pack<TB, VA> out;
#pragma unroll
                    for (int j = 0; j < VA; ++j) {
                        TB old = TB();
                        if (MODE == TTC_EPI_AXPBY) old = rb[u].v[j];
                        out.v[j] = epi(ra[u].v[j], old);
                    }
                    store_pack<TB, VA, NT>(Bt, e.l_or_g2 + LA.g2 - back * kScaleB, out);
                };
                walk<kUnroll, VA>(p.a, LA, sla, wma, tab_a, tabc_a, wave, load, store);
            };
            if (nt_a && nt_b) run(std::true_type()); else run(std::false_type());
            continue;
        }

        unsigned char* lds = smem + p.lds_data_off +
                             (parity & (uint32_t)(p.lds_buffers - 1)) * (uint32_t)(p.lds_tile_elems * kScaleA);
        parity ^= 1u;
        // ---- walk 1: A order, global -> LDS
        {
            auto run = [&](auto stream) {
                constexpr bool NT = decltype(stream)::value;
                const int32_t vs = p.a.vec_lds_stride;
                constexpr int kUnroll = Unroll<TA, VA>::value;
                Pack<TA, VA> ra[kUnroll];
                auto load = [&](int u, const PosEntry& e, int back, bool ok) {
                    ra[u] = load_pack<TA, VA, NT>(At, ok ? e.g + LA.g - back * kScaleA : 0);
                };
                auto park = [&](int u, const PosEntry& e, int back, bool ok) {
                    unsigned char* dst = lds + ((int32_t)e.l_or_g2 + LA.l - back * vs * kScaleA);
#pragma unroll
                    for (int j = 0; j < VA; ++j)
                        *reinterpret_cast<TA*>(ok ? dst + j * vs * kScaleA : spare) = ra[u].v[j];
                };
                walk<kUnroll, VA>(p.a, LA, sla, wma, tab_a, tabc_a, wave, load, park);
            };
            if (nt_a) run(std::true_type()); else run(std::false_type());
        }
        if (wave == nwave - 1 && q + seq.step < seq.end) publish(tile_of(seq, q + seq.step), parity);   // parity already flipped
        __syncthreads();
        // ---- walk 2: B order, LDS -> epilogue -> global
        {
            auto run = [&](auto stream) {
                constexpr bool NT = decltype(stream)::value;
                const int32_t vs = p.b.vec_lds_stride;
                constexpr int kUnroll = Unroll<TB, VB>::value;
                Pack<TB, VB> rb[kUnroll];
                Pack<TA, VB> rl[kUnroll];
                auto load = [&](int u, const PosEntry& e, int back, bool ok) {
                    if (MODE == TTC_EPI_AXPBY) rb[u] = load_pack<TB, VB, NT>(Bt, ok ? e.g + LB.g - back * kScaleB : 0);
                    const TA* src = reinterpret_cast<const TA*>(lds + (ok ? (int32_t)e.l_or_g2 + LB.l - back * vs * kScaleA : 0));
#pragma unroll
                    for (int j = 0; j < VB; ++j) rl[u].v[j] = src[j * vs];
                };
                auto store = [&](int u, const PosEntry& e, int back, bool ok) {
                    if (!ok) return;
                    Pack<TB, VB> out;
#pragma unroll
                    for (int j = 0; j < VB; ++j) {
                        TB old = TB();
                        if (MODE == TTC_EPI_AXPBY) old = rb[u].v[j];
                        out.v[j] = epi(rl[u].v[j], old);
                    }
                    store_pack<TB, VB, NT>(Bt, e.g + LB.g - back * kScaleB, out);
                };
                walk<kUnroll, VB>(p.b, LB, slb, wmb, tab_b, tabc_b, wave, load, store);
            };
            if (nt_b) run(std::true_type()); else run(std::false_type());
        }
        if (p.lds_buffers == 1) __syncthreads();      // the one buffer is refilled by the next tile
    }
}

// ---------------------------------------------------------------------------------
// The row kernel, for the case where the stride-1 index keeps its place and rows are contiguous in both tensors
// (paper Section 3.1, case 1: the first column is copied, inside loops over the other indices).  B is walked in the order of its
// multi-index: workgroup w moves the `chunk` vectors that start at vector w * chunk, so consecutive
// workgroups write consecutive memory (a dense B is written front to back like a copy), and every lane gathers
// its vectors from the rows of A.  No tiles, no LDS, no tables: a lane finds its row by one division and the
// row's place in both tensors by one division per index.  Where rows are not a multiple of the vector, the last
// vector of a row is moved back to end with the row and repeats up to V-1 elements of its neighbour with the same
// values (only where B is not read: with beta != 0 the planner picks a vector that divides the row).
// ---------------------------------------------------------------------------------
constexpr int kRowsThreads = 256;

template <typename TA, typename TB, int MODE, int V, int U>
__global__ __launch_bounds__(kRowsThreads) void rows_kernel(const RowsParams p, const TA* __restrict__ A, TB* __restrict__ B)
{
    constexpr int32_t kScaleA = (int32_t)sizeof(TA), kScaleB = (int32_t)sizeof(TB);
    const Epilogue<TA, TB, MODE> epi(p.alpha, p.beta);
    const int64_t base = (int64_t)blockIdx.x * (int64_t)p.chunk;
    const int64_t row0_wide = base / (int64_t)p.slots;                  // wave-uniform: once per workgroup
    const uint32_t row0 = (uint32_t)row0_wide;
    const uint32_t slot0 = (uint32_t)(base - row0_wide * (int64_t)p.slots);
    const unsigned char* Ab = reinterpret_cast<const unsigned char*>(A);
    unsigned char* Bb = reinterpret_cast<unsigned char*>(B);
    auto run = [&](auto stream_a, auto stream_b) {
        constexpr bool NTA = decltype(stream_a)::value, NTB = decltype(stream_b)::value;
        Pack<TA, V> ra[U];
        Pack<TB, V> rb[U];
        int64_t to[U];
        bool valid[U];
        // a lane past the end of the tensor loads the first vector instead and stores nothing, so that no load
        // sits in divergent control flow
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const RowAccess x = rows_access(p, base, row0, slot0, (uint32_t)u * kRowsThreads + threadIdx.x);
            valid[u] = x.valid;
            to[u] = x.at.b * kScaleB;
            ra[u] = load_pack<TA, V, NTA>(Ab, x.at.a * kScaleA);
            if (MODE == TTC_EPI_AXPBY) rb[u] = load_pack<TB, V, NTB>(Bb, to[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!valid[u]) continue;
            Pack<TB, V> out;
#pragma unroll
            for (int j = 0; j < V; ++j) {
                TB old = TB();
                if (MODE == TTC_EPI_AXPBY) old = rb[u].v[j];
                out.v[j] = epi(ra[u].v[j], old);
            }
            store_pack<TB, V, NTB>(Bb, to[u], out);
        }
    };
    if (p.nt_a) { if (p.nt_b) run(std::true_type(), std::true_type()); else run(std::true_type(), std::false_type()); }
    else        { if (p.nt_b) run(std::false_type(), std::true_type()); else run(std::false_type(), std::false_type()); }
}

// ---------------------------------------------------------------------------------
// The micro-tile kernel (the paper's w x w in-register transposition, Section 3.2, in its gfx950 form): a tile over
// the two stride-1 indices only (each possibly merged with the index next to it in its tensor, see MicroParams),
// every access 128 bits wide.  Lanes load 16-byte vectors along A's stride-1 index and park each with one 128-bit
// LDS write; after the barrier a lane reads the V x V block it owns with V 128-bit LDS reads (rows of the tile are
// XOR-swizzled at 16-byte granularity: neither phase has bank conflicts), transposes it in registers -- no
// cross-lane traffic: row i of the block is one register quad, column j is element j of each -- and stores V
// 16-byte vectors along B's stride-1 index.  Extents need not be multiples of V: the last vector of a row and the
// last block of a column are moved back to end with the tensor (micro_back), and where B is updated as well a
// moved block writes only what is its own.  Both tensors have one element type of 4 or 8 bytes.
// ---------------------------------------------------------------------------------
template <typename T, int MODE, int V>
__global__ __launch_bounds__(256) void micro_kernel(const MicroArgs args_by_value, const T* __restrict__ A, T* __restrict__ B)
{
    static_assert(V * sizeof(T) == 16, "one 16-byte vector");
    const MicroArgs& p = *reinterpret_cast<const MicroArgs*>((const void*)__builtin_amdgcn_kernarg_segment_ptr());
    extern __shared__ __align__(16) unsigned char smem[];
    typedef uint32_t Quad __attribute__((ext_vector_type(4)));
    Quad* lds = reinterpret_cast<Quad*>(smem);
    constexpr int U = 4;                                       // loads a lane keeps in flight (eight: 0-5 % slower on the suite)
    constexpr int32_t kScale = (int32_t)sizeof(T);
    const MicroParams& m = p.micro;
    const Epilogue<T, T, MODE> epi(p.alpha, p.beta);
    const uint32_t tid = threadIdx.x, threads = blockDim.x;
    const uint32_t loads = (uint32_t)m.loads, blocks = (uint32_t)m.blocks;
    const TileSeq seq = tile_sequence(p, blockIdx.x);
    for (uint32_t q = seq.first; q < seq.end; q += seq.step) {
        const MicroTile t = micro_tile(p, tile_of(seq, q));
        if (p.debug_stop == 1) return;                        // measurement aid: launch, parameters and tile decode only
        const unsigned char* At = reinterpret_cast<const unsigned char*>(A + t.a);
        unsigned char* Bt = reinterpret_cast<unsigned char*>(B + t.b);
        auto run = [&](auto stream_a, auto stream_b) {
            constexpr bool NTA = decltype(stream_a)::value, NTB = decltype(stream_b)::value;
            union Vec { Pack<T, V> p; Quad q; };
            // ---- A order: global -> LDS, U vectors at a time.  A lane whose vector lies outside the tensor loads the
            // tile's first vector instead (no load in divergent control flow); what it parks nobody reads.
            for (uint32_t k0 = 0; k0 < loads; k0 += U) {
                Vec in[U];
                MicroLoad x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    x[u] = micro_load(m, threads, tid, k0 + (uint32_t)u);
                    const bool ok = x[u].valid && x[u].row < t.lim_b && x[u].col < t.lim_a;
                    const uint32_t col = ok ? micro_back(x[u].col, t.lim_a, V) : 0u;
                    in[u].p = load_pack<T, V, NTA>(At, (micro_row_a(m, t.row0 + (ok ? x[u].row : 0u)) + (int64_t)col) * kScale);
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (x[u].valid) lds[x[u].chunk] = in[u].q;
            }
            __syncthreads();
            if (p.debug_stop == 2) return;                     // measurement aid: ... and the loads of A into LDS
            // ---- B order: LDS -> registers (V x V block) -> epilogue -> global
            for (uint32_t b = 0; b < blocks; ++b) {
                const MicroBlock x = micro_block(m, threads, tid, b);
                const bool ok = x.valid && x.row < t.lim_b && x.col < t.lim_a;
                const uint32_t row = ok ? micro_back(x.row, t.lim_b, V) : 0u, col = ok ? micro_back(x.col, t.lim_a, V) : 0u;
                const uint32_t lane_c = ok ? x.lane_c : 0u;
                int64_t to[V];                                  // byte offsets of the block's V columns in B
#pragma unroll
                for (int j = 0; j < V; ++j) to[j] = (micro_col_b(m, t.col0 + col + (uint32_t)j) + (int64_t)row) * kScale;
                Pack<T, V> old[V];
                if (MODE == TTC_EPI_AXPBY) {
#pragma unroll
                    for (int j = 0; j < V; ++j) old[j] = load_pack<T, V, NTB>(Bt, to[j]);
                }
                Vec blk[V];
#pragma unroll
                for (int i = 0; i < V; ++i) blk[i].q = lds[micro_slot(m, row + (uint32_t)i, lane_c)];
                // Where B is read as well as written an element must be updated once: a block that was moved back, or
                // lies in a tile that was, updates only what is its own (from its nominal place on, and not the
                // neighbouring tile's elements), element by element.  Such blocks exist at the tensor's edge only.
                const bool edge = MODE == TTC_EPI_AXPBY && ok && (row != x.row || col != x.col || x.row < t.own_b || x.col < t.own_a);
                if (MODE == TTC_EPI_AXPBY && edge) {
                    const uint32_t first_row = x.row > t.own_b ? x.row : t.own_b, first_col = x.col > t.own_a ? x.col : t.own_a;
#pragma unroll
                    for (int j = 0; j < V; ++j)
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            if (col + (uint32_t)j >= first_col && row + (uint32_t)i >= first_row) {
                                T* pb = reinterpret_cast<T*>(Bt + to[j]) + i;
                                *pb = epi(blk[i].p.v[j], *pb);
                            }
                } else if (ok) {
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        Pack<T, V> out;
#pragma unroll
                        for (int i = 0; i < V; ++i) {
                            T b_old = T();
                            if (MODE == TTC_EPI_AXPBY) b_old = old[j].v[i];
                            out.v[i] = epi(blk[i].p.v[j], b_old);
                        }
                        store_pack<T, V, NTB>(Bt, to[j], out);
                    }
                }
            }
        };
        if (p.nt_a) { if (p.nt_b) run(std::true_type(), std::true_type()); else run(std::true_type(), std::false_type()); }
        else        { if (p.nt_b) run(std::false_type(), std::true_type()); else run(std::false_type(), std::false_type()); }
        __syncthreads();                                       // the tile buffer is refilled by the next tile
    }
}

template <typename TA, typename TB, int MODE>
inline hipError_t launch_micro(const Candidate& c, const void* A, void* B, hipStream_t stream)
{
    if constexpr (std::is_same<TA, TB>::value && (sizeof(TA) == 4 || sizeof(TA) == 8)) {
        constexpr int V = 16 / (int)sizeof(TA);
        const KernelParams& kp = c.kp;
        const MicroParams& m = kp.micro;
        const uint32_t grid = kp.num_tiles;                    // one tile per workgroup: the hardware deals them
        const int64_t th = c.threads;
        if (m.vec != V || (1 << m.vec_log) != V || (th != 64 && th != 128 && th != 256) || m.la < 1 || m.lb < 1 ||
            m.ta != m.la * V || m.tb != m.lb * V || m.pitch < m.la || (m.pitch & 7) || (m.swizzle != 7u && m.swizzle != 0u) || m.la_div.div != (uint32_t)m.la ||
            m.lb_div.div != (uint32_t)m.lb || (int64_t)m.loads * th < (int64_t)m.la * m.tb || (int64_t)m.blocks * th < (int64_t)m.la * m.lb ||
            (int64_t)(m.loads + 4) * th >= (int64_t(1) << 31) ||
            c.lds_bytes != m.tb * m.pitch * 16 || c.lds_bytes > 64 * 1024 || grid < 1 || grid != kp.grid ||
            m.size_a0 < V || m.size_p0 < V || m.size_a0 >= (int64_t(1) << 31) || m.size_p0 >= (int64_t(1) << 31) ||
            m.col_in_div.div < 1 || m.row_in_div.div < 1)
            return hipErrorInvalidValue;
        const void* fn = reinterpret_cast<const void*>(&micro_kernel<TA, MODE, V>);
        const TA* a = static_cast<const TA*>(A);
        TA* b = static_cast<TA*>(B);
        // TTC_DEBUG_STOP=1 or 2 in the environment: workgroups return early (how the parts of a launch were timed)
        static const int stop = std::getenv("TTC_DEBUG_STOP") ? std::atoi(std::getenv("TTC_DEBUG_STOP")) : 0;
        MicroArgs ready = micro_args(c);
        ready.debug_stop = stop;
        void* args[] = {&ready, &a, &b};
        return hipLaunchKernel(fn, dim3(grid), dim3(c.threads), args, (size_t)c.lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

// Compute units of the current device (256 on MI355X), asked once per process and device.
inline int device_cus()
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
template <typename TA, typename TB, int MODE, int VA, int VB, bool DIRECT>
inline hipError_t launch_one(const KernelParams& kp, const void* A, void* B, uint32_t grid, int threads,
                             int lds_bytes, hipStream_t stream)
{
    if (grid != kp.grid || grid < 1 || grid > kp.num_tiles) return hipErrorInvalidValue;
    const void* fn = reinterpret_cast<const void*>(&box_kernel<TA, TB, MODE, VA, VB, DIRECT>);
    // more than 64 KB of dynamic LDS has to be asked for, once per kernel and device (a CU of gfx950 has 160 KB)
    if (lds_bytes > 64 * 1024) {
        static std::atomic<uint64_t> raised{0};                 // bit d: done on device d
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        if (!((raised.load(std::memory_order_acquire) >> dev) & 1u)) {
            const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
            if (e != hipSuccess) return e;
            raised.fetch_or(uint64_t(1) << dev, std::memory_order_release);
        }
    }
    const TA* a = static_cast<const TA*>(A);
    TB* b = static_cast<TB*>(B);
    void* args[] = {const_cast<KernelParams*>(&kp), &a, &b};
    // the launch's own status: an error left behind by an earlier, unrelated call on this thread is not ours
    return hipLaunchKernel(fn, dim3(grid), dim3(threads), args, (size_t)lds_bytes, stream);
}

template <typename TA, typename TB, int MODE, int V, int U>
inline hipError_t launch_rows_unrolled(const Candidate& c, const void* A, void* B, hipStream_t stream)
{
    RowsParams rp = c.rows;
    rp.nt_a = c.kp.nt_a;
    rp.nt_b = c.kp.nt_b;
    if (rp.vec != V || rp.unroll != U || c.threads != kRowsThreads || rp.chunk != (uint32_t)(kRowsThreads * U) ||
        rp.row < (uint32_t)V || rp.slots != (rp.row + V - 1) / V || rp.vectors < 1 || (MODE == TTC_EPI_AXPBY && rp.overlap)) return hipErrorInvalidValue;
    const int64_t grid = (rp.vectors + rp.chunk - 1) / rp.chunk;
    if (grid < 1 || grid > INT32_MAX) return hipErrorInvalidValue;
    const TA* a = static_cast<const TA*>(A);
    TB* b = static_cast<TB*>(B);
    void* args[] = {&rp, &a, &b};
    return hipLaunchKernel(reinterpret_cast<const void*>(&rows_kernel<TA, TB, MODE, V, U>), dim3((uint32_t)grid), dim3(kRowsThreads), args, 0, stream);
}

template <typename TA, typename TB, int MODE, int V>
inline hipError_t launch_rows_one(const Candidate& c, const void* A, void* B, hipStream_t stream)
{
    switch (c.rows.unroll) {
    case 1: return launch_rows_unrolled<TA, TB, MODE, V, 1>(c, A, B, stream);
    case 2: return launch_rows_unrolled<TA, TB, MODE, V, 2>(c, A, B, stream);
    case 4: return launch_rows_unrolled<TA, TB, MODE, V, 4>(c, A, B, stream);
    case 8: return launch_rows_unrolled<TA, TB, MODE, V, 8>(c, A, B, stream);
    default: return hipErrorInvalidValue;
    }
}

// VMAXA / VMAXB: elements of each type in 16 bytes
template <typename TA, typename TB, int MODE, int VMAXA, int VMAXB>
inline hipError_t launch_vec(const Candidate& c, const void* A, void* B, hipStream_t s)
{
    constexpr int VD = VMAXA < VMAXB ? VMAXA : VMAXB;      // direct and row kernel: one width for both sides
    if (c.kernel_class == TTC_KERNEL_MICRO) return launch_micro<TA, TB, MODE>(c, A, B, s);
    if (c.kernel_class == TTC_KERNEL_ROWS) {
        const int v = c.rows.vec;
        if (v == 1) return launch_rows_one<TA, TB, MODE, 1>(c, A, B, s);
        if (v == 2 && VD >= 2) return launch_rows_one<TA, TB, MODE, (VD >= 2 ? 2 : 1)>(c, A, B, s);
        if (v == 4 && VD >= 4) return launch_rows_one<TA, TB, MODE, (VD >= 4 ? 4 : 1)>(c, A, B, s);
        return hipErrorInvalidValue;
    }
    // the candidate's parameter block is launch-ready for a device of 256 compute units (every MI355X); it is
    // copied and re-gridded only for another device, or for the set-up measurement (TTC_DEBUG_STOP in the
    // environment: every workgroup returns after its set-up)
    static const bool stop = std::getenv("TTC_DEBUG_STOP") != nullptr;
    const uint32_t grid = launch_grid(c, device_cus());
    KernelParams other;
    const KernelParams* ready = &c.kp;
    if (grid != c.kp.grid || stop) {
        other = c.kp;
        set_grid(&other, grid);
        other.debug_stop = stop ? 1 : 0;
        ready = &other;
    }
    const KernelParams& kp = *ready;
    const int va = kp.a.vec, vb = kp.b.vec;
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
inline hipError_t launch_mode(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s)
{
    switch (P.epilogue) {
    case TTC_EPI_COPY:  return launch_vec<TA, TB, TTC_EPI_COPY, VMAXA, VMAXB>(c, A, B, s);
    case TTC_EPI_SCALE: return launch_vec<TA, TB, TTC_EPI_SCALE, VMAXA, VMAXB>(c, A, B, s);
    default:            return launch_vec<TA, TB, TTC_EPI_AXPBY, VMAXA, VMAXB>(c, A, B, s);
    }
}

}  // namespace ttc
