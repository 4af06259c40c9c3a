/*
 * ttc_aux.h -- measurement and test aids of the MI355X tensor-transposition library.
 *
 * None of these is part of the transposition path (include/ttc.h is): the timing helpers serve
 * bench.py and the studies, the host replay serves the CPU tests of the planner.
 */
#ifndef TTC_AUX_H_
#define TTC_AUX_H_

#include "ttc.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement helper: enqueue `warmup` untimed and `iters` timed ttc_execute calls on
 * `stream`, launch i using the buffer pair (A_list[i % npairs], B_list[i % npairs])
 * (HOST arrays of DEVICE pointers; rotating pairs keeps the last-level cache from holding
 * the working set), bracket the timed launches with HIP events recorded on `stream`, wait
 * for them, and return the mean milliseconds per launch in *ms_per_launch.  SYNCHRONISES.
 */
int ttc_time_execute(ttc_plan_t plan, int npairs, const void* const* A_list, void* const* B_list,
                     void* stream, int warmup, int iters, float* ms_per_launch);

/*
 * Bandwidth ceilings measured the same way (the role of the STREAM/SAXPY lines in the
 * paper's Section 4).  kind 0: dst <- src with a 128-bit-per-lane copy kernel (1 read, 1
 * write); kind 1: hipMemcpyAsync device-to-device; kind 2: dst <- 0.75*src + 1.25*dst as
 * fp32 (2 reads, 1 write); kind 3: the copy kernel of kind 0 with non-temporal loads and stores; kind 4: a non-temporal copy of one
 * 16-byte access per lane and one 4 KB chunk per one-shot workgroup; kind 5: the update of kind 2 in the launch shape of kind 4,
 * non-temporal.  `bytes` must be a multiple of 16 and the pointers 16-byte
 * aligned.  Buffer pairs rotate as in ttc_time_execute.  SYNCHRONISES.
 */
int ttc_time_ceiling(int kind, int64_t bytes, int npairs, const void* const* src_list,
                     void* const* dst_list, void* stream, int warmup, int iters,
                     float* ms_per_launch);

/*
 * Host-side bounds checker for the planner and the kernels' index arithmetic; it is a test
 * aid, never part of ttc_execute.  Replays the walk of the selected candidate lane by lane on
 * the host, with the index code the kernels are compiled from, and writes to b_from_a[o]
 * (HOST array of span_b entries, see ttc_plan_info_t; prod(sizes) for dense tensors) the element
 * offset of A that the candidate moves to element offset o of B (the element map of paper Eq. 1),
 * -1 where B is not written.  Returns TTC_ERR_INTERNAL if any access would leave the (sub-)tensors
 * or the LDS tile, or an element of B would not be written at all or be written twice from different
 * sources (overlapping vectors write an element twice with the same value; if beta != 0 they must
 * belong to one instruction).  Cost grows with prod(sizes).
 */
int ttc_debug_emulate_map(ttc_plan_t plan, int64_t* b_from_a);

#ifdef __cplusplus
}
#endif
#endif /* TTC_AUX_H_ */
