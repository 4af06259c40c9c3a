/*
 * ttc.h -- C ABI of the MI355X tensor-transposition library.
 *
 * The operation (paper Eq. 1), out of place, on dense column-major tensors
 * (leftmost index has stride 1; paper Section 1):
 *
 *     B[Pi(i_0..i_{N-1})]  <-  alpha * A[i_0..i_{N-1}]  +  beta * B[Pi(i_0..i_{N-1})]
 *
 * perm[j] is the index of A that becomes index j of B (the capital-Pi list of Eq. 1:
 * Pi(i1,i2,i3) = (i2,i3,i1) is perm = {1,2,0}); B's extents are sizes[perm[j]].
 *
 * All functions return integer status codes; nothing throws or aborts across this
 * boundary.  Plan objects live in host memory and are owned by the library.  Tensor
 * pointers are DEVICE pointers owned by the caller.  No function here synchronises
 * the device unless its comment says so.
 */
#ifndef TTC_H_
#define TTC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TTC_MAX_DIM 6

typedef struct ttc_plan_s* ttc_plan_t;

/* Element types (paper Table 1, --dataType s d c z and the mixed-precision sd ds cz zc, where the
 * first letter is A's type and the second B's).  Complex elements are interleaved (re, im). */
enum { TTC_F32 = 0, TTC_F64 = 1, TTC_C64 = 2, TTC_C128 = 3,
       TTC_F32_F64 = 4, TTC_F64_F32 = 5, TTC_C64_C128 = 6, TTC_C128_C64 = 7 };

enum {
    TTC_OK = 0,
    TTC_ERR_INVALID_VALUE = 1,     /* ndim outside 1..6, an extent < 1, bad candidate index, ... */
    TTC_ERR_INVALID_PERM = 2,      /* perm is not a permutation of 0..ndim-1 */
    TTC_ERR_UNSUPPORTED_DTYPE = 3,
    TTC_ERR_NULL_POINTER = 4,
    TTC_ERR_ALIAS = 5,             /* A and B overlap: the operation is out of place */
    TTC_ERR_OVERFLOW = 6,          /* element or byte count does not fit */
    TTC_ERR_HIP = 7,               /* a HIP runtime call failed */
    TTC_ERR_ALLOC = 8,
    TTC_ERR_MISALIGNED = 9,        /* pointer not aligned to the element size */
    TTC_ERR_INTERNAL = 10,         /* a candidate failed the host-side bounds check */
    TTC_ERR_NOT_FOUND = 11,        /* the plan store holds no usable entry for this problem */
    TTC_ERR_IO = 12                /* the plan store could not be written */
};

/* Kernel families (paper Section 3.1: the stride-1 index keeps its place, or not). */
enum { TTC_KERNEL_DIRECT = 0 /* tiles, no staging: stride-1 index fixed */, TTC_KERNEL_LDS = 1 /* tile staged through LDS */,
       TTC_KERNEL_ROWS = 2 /* stride-1 index fixed: B walked front to back, rows gathered from A */,
       TTC_KERNEL_MICRO = 3 /* tile over the two stride-1 indices only (each possibly merged with the index next to it in
                               its tensor): 128-bit LDS accesses, XOR-swizzled rows, register transposes of 4x4 (2x2)
                               blocks; one precision of 4- or 8-byte elements */ };
/* Epilogues chosen from alpha, beta. */
enum { TTC_EPI_COPY = 0 /* alpha=1, beta=0 */, TTC_EPI_SCALE = 1 /* beta=0: B never read */, TTC_EPI_AXPBY = 2 };

/*
 * What a plan decided.  "Fused" quantities are after size-1 extents were dropped and
 * adjacent indices that stay adjacent and in order in B were merged (paper Section 3,
 * stage (1)).  Arrays are indexed by fused index of A, entries past ndim are 0.
 */
typedef struct {
    int     dtype;
    int     ndim;                          /* fused number of indices, >= 1 */
    int64_t sizes[TTC_MAX_DIM];            /* fused extents of A */
    int     perm[TTC_MAX_DIM];             /* fused permutation */
    int     stride1_fixed;                 /* 1: paper's case pi(i1)=i1 (or 1-D axpby), 0: stride-1 index changes */
    int     kernel_class;                  /* TTC_KERNEL_* of the selected candidate */
    int     epilogue;                      /* TTC_EPI_* */
    int     tile[TTC_MAX_DIM];             /* extent of the tile (box) along each fused index; 1 = not blocked */
    int     digits_a, digits_b;            /* digits of the load walk (A order) and of the store walk (B order): a digit
                                              is one index, or the leading indices of that tensor that lie whole inside
                                              the tile merged into one flat, contiguous index */
    int     digit_tile_a[4], digit_lane_a[4]; /* per digit of the load walk, in its order: flat extent inside the tile,
                                              and extent of the sub-box one wavefront instruction covers */
    int     digit_tile_b[4], digit_lane_b[4]; /* the same for the store walk */
    int     tile_order[TTC_MAX_DIM];       /* fused indices from fastest to slowest in the workgroup-id -> tile map */
    int     lds_stride[TTC_MAX_DIM];       /* element stride of each fused index inside the LDS tile (0 = unused) */
    int     vec_a, vec_b;                  /* elements per lane per global access on the A side / B side */
    int     partial_a, partial_b;          /* 1: runs are not a multiple of the vector: the last vector of a run is moved
                                              back to end with the run and overlaps its neighbour */
    int     threads;                       /* workgroup size */
    int     wg_per_cu;                     /* workgroups launched per compute unit; each walks several tiles (row kernel: 0,
                                              its workgroups move one chunk each) */
    int     xcd_remap;                     /* tiles -> XCDs: 0 round robin, 1 a contiguous range each, k >= 2: chunks of 2^k tiles in turn */
    int     lds_bytes;                     /* dynamic LDS per workgroup: position tables + tile buffer(s) */
    int     lds_buffers;                   /* 2: tile buffers alternate (one barrier per tile), 1: one buffer (two barriers) */
    int     nt_a, nt_b;                    /* 1: loads of A / stores to B (and loads of B if beta != 0) carry the
                                              non-temporal hint (the paper's streaming stores, and their load counterpart) */
    int     lds_conflict_a, lds_conflict_b;/* modelled worst bank multiplicity of the LDS write / read instructions */
    int     run_bytes_a, run_bytes_b;      /* contiguous bytes the tile spans in A / in B */
    int     seg_bytes_a, seg_bytes_b;      /* contiguous bytes one wavefront instruction covers in A / in B */
    int     align_a, align_b;              /* power of two (<= 128) dividing the byte offset of every run start */
    int64_t num_tiles;                     /* tiles the tensor is cut into */
    int64_t elements;                      /* prod(sizes) */
    int64_t bytes_moved;                   /* bytes of A read + bytes of B written (+ bytes of B read iff beta != 0; paper Eq. 2) */
    int64_t span_a, span_b;                /* elements from the first to the last element of A / of B, inclusive (= elements if dense) */
    int64_t stride_a[TTC_MAX_DIM];         /* element stride of each fused index in A ... */
    int64_t stride_b[TTC_MAX_DIM];         /* ... and in B */
    int     candidate_index;               /* which candidate is selected */
    int     candidate_count;               /* how many the plan holds: 1 until the ranked list has been built (ttc_plan_create),
                                              then all of them: candidate 0 as created, the others by heuristic cost */
    float   tuned_ms;                      /* time of the selected candidate in the last ttc_plan_tune, else 0 */
    double  heuristic_cost;                /* the ranking key: modelled relative cost, smaller is better */
    int     unroll;                        /* row kernel: vectors a lane keeps in flight (1, 2, 4 or 8); micro-tile kernel: blocks a lane owns
                                              (1 to 6); 0 for the box kernels */
    int     merged;                        /* micro-tile kernel: bit 0: the tile's column index is A's indices 0 and 1 taken as one,
                                              bit 1: its row index is B's first two indices taken as one; else 0 */
} ttc_plan_info_t;

/*
 * Create a plan for one transposition (paper Eq. 1; defaults of Table 1).
 *   dtype       any TTC_* element type; for the mixed-precision pairs see ttc_plan_create_ex.
 *   ndim        1..TTC_MAX_DIM.
 *   sizes, perm HOST arrays of length ndim, copied; every extent >= 1.
 *   alpha, beta HOST pointers to one scalar of dtype (float, double, float[2], double[2]; double or
 *               double[2] for the mixed-precision pairs); NULL means alpha = 1, beta = 0.  Copied.
 * Touches no device.  Returns NULL on error; ttc_last_status() says why.
 * Only the heuristic's choice (candidate 0: tile shape, vector widths, lane mapping, tile order) is
 * laid out here; the ranked list of all candidate launch configurations is built when something
 * first asks for it (ttc_plan_candidate_count, ttc_plan_select_candidate, the search, the plan store).
 */
ttc_plan_t ttc_plan_create(int dtype, int ndim, const int64_t* sizes, const int* perm,
                           const void* alpha, const void* beta);

/*
 * The same for tensors that are parts of larger ones, and for every data type of Table 1.
 *   lda   HOST array of length ndim or NULL: lda[k] >= sizes[k] is the extent of the enclosing tensor
 *         along index k of A (Table 1, --lda), so A's element
 *         strides are 1, lda[0], lda[0]*lda[1], ...  NULL = dense.  The sub-tensor starts at the pointer
 *         later given to ttc_execute (the caller adds the offset of its corner).
 *   ldb   likewise for B: ldb[j] >= sizes[perm[j]] belongs to index j of B.
 * Two indices are merged only if they are contiguous in both tensors (footnote of Section 3, stage (1):
 * ld(i_{m+1}) = size(i_m) * ld(i_m)).  Elements of B outside the sub-tensor are neither read nor written.
 * Mixed precision (TTC_F32_F64 ...; the paper names the feature and no more): alpha and beta are HOST
 * doubles (double[2] for the complex pairs), every element is widened to double, the arithmetic of the
 * data type's epilogue runs in double, and the result is rounded once to B's precision.
 * For the single types alpha and beta are one scalar of that type, as in ttc_plan_create.
 */
ttc_plan_t ttc_plan_create_ex(int dtype, int ndim, const int64_t* sizes, const int* perm,
                              const int64_t* lda, const int64_t* ldb, const void* alpha, const void* beta);

/*
 * Run the plan: B <- alpha * permute(A) + beta * B (paper Eq. 1).
 *   A, B    DEVICE pointers to the first element of each tensor: prod(sizes) elements, dense and
 *           column-major, or span_a / span_b elements for sub-tensors (ttc_plan_create_ex).
 *           Aligned to the size of their real type (vector accesses need no more than that).
 *           The two ranges must not overlap (TTC_ERR_ALIAS).
 *   stream  hipStream_t passed as void*; NULL is the default stream.
 * Asynchronous: enqueues one kernel on `stream`, allocates nothing, never synchronises.
 * With beta == 0, B is never read.  Returns the launch status.
 */
int ttc_execute(ttc_plan_t plan, const void* A, void* B, void* stream);

/* Free a plan.  NULL is a no-op.  Returns TTC_OK. */
int ttc_plan_destroy(ttc_plan_t plan);

/* Why the last ttc_plan_create on this thread returned NULL (TTC_OK if it did not). */
int ttc_last_status(void);
const char* ttc_status_string(int status);

/* Fill *out with the decisions of the selected candidate.  Host only. */
int ttc_plan_get_info(ttc_plan_t plan, ttc_plan_info_t* out);

/* Number of candidates the plan holds, or a negative status. */
int ttc_plan_candidate_count(ttc_plan_t plan);
/* Select candidate `index` (0 = heuristic best) for later ttc_execute calls.  Host only. */
int ttc_plan_select_candidate(ttc_plan_t plan, int index);

/*
 * Non-temporal ("streaming") accesses of the selected candidate (paper Table 1, --no-streaming-stores, here
 * for loads as well): stream_a for the loads of A, stream_b for the stores to B and the loads of B when
 * beta != 0.  1 = on, 0 = off, -1 = the planner's rule (a side streams if all its runs are whole 128-byte
 * lines).  The direct kernel streams both sides or neither.  Host only.
 */
int ttc_plan_set_streaming(ttc_plan_t plan, int stream_a, int stream_b);

/*
 * How the selected candidate deals its tiles to the 8 XCDs (each has its own L2): the MI355X form of the
 * paper's loop-order question (Section 3.3) one level up.  mode 0: tile ids round robin over all workgroups;
 * 1: one contiguous range of tile ids per XCD; 2..10: chunks of 2^mode consecutive tile ids dealt to the
 * XCDs in turn; -1: the default (chunks of 32; round robin below 2048 tiles).  Reported as xcd_remap by ttc_plan_get_info.  The search
 * times its finalists with modes 1 and 3 as well.  Host only.
 */
int ttc_plan_set_tile_mapping(ttc_plan_t plan, int mode);

/*
 * Search (paper Section 3: candidates are timed and the fastest becomes the solution;
 * Table 1 --maxImplementations).  Times at most max_candidates candidates, in heuristic
 * rank order (up to two fifths of the places are kept for the best-ranked candidates of
 * the micro-tile kernel, over single and over merged indices, whose ranking is a model
 * of its own), on the caller's buffers and stream (HIP events, a few launches each, more
 * of them if a launch takes only microseconds, after about 3 ms of untimed launches that
 * bring an idle GPU up to its clocks), each with the non-temporal hints of the rule and
 * with both sides streamed, and selects the fastest; the best few are timed again, with
 * every setting of the hints and with the other tile mappings.
 * max_candidates: 0 = environment TTC_MAX_CANDIDATES or 200,
 * 1 = keep the heuristic choice without timing, -1 = all candidates.
 * A_scratch / B_scratch are DEVICE buffers of prod(sizes) elements; B_scratch is
 * overwritten.  SYNCHRONISES the stream.
 */
int ttc_plan_tune(ttc_plan_t plan, const void* A_scratch, void* B_scratch, void* stream,
                  int max_candidates);

/*
 * The same search over `npairs` buffer pairs (HOST arrays of DEVICE pointers) used in rotation,
 * launch after launch, so that a last-level cache as large as a tensor cannot hold the working
 * set and flatter some candidates.  Every B_list[i] is overwritten.  SYNCHRONISES the stream.
 */
int ttc_plan_tune_pairs(ttc_plan_t plan, int npairs, const void* const* A_list, void* const* B_list,
                        void* stream, int max_candidates);

/*
 * Persistent store of search results (paper Section 3: solutions of previous searches are kept in a
 * local database and returned without a new search).  `path` names a text file, one line per problem;
 * the key is the fused problem (data type, extents, permutation, strides, whether beta is 0) on gfx950.
 *   ttc_plan_cache_store   appends the plan's selected candidate (normally after ttc_plan_tune).
 *   ttc_plan_cache_lookup  selects the stored candidate if the file has one for this problem and the
 *                          library still builds that configuration: TTC_OK; otherwise TTC_ERR_NOT_FOUND
 *                          and the plan is unchanged.  A missing file is "not found", not an error.
 * Host only.  When the environment variable TTC_PLAN_CACHE names a file, ttc_plan_tune and
 * ttc_plan_tune_pairs look the problem up there first (a hit skips the search) and store what a
 * search selects.
 */
int ttc_plan_cache_store(ttc_plan_t plan, const char* path);
int ttc_plan_cache_lookup(ttc_plan_t plan, const char* path);

#ifdef __cplusplus
}
#endif
#endif /* TTC_H_ */
