/*
 * libdip developer tools: launch-shape overrides, the switch between the one-launch and the
 * two-launch form of a pruning point, and per-kernel timing.  Unlike the calls of dip.h these
 * keep PROCESS-WIDE host state (no device state): they are meant for a single benchmarking or
 * test thread and are not thread-safe against concurrent launches.
 */
#ifndef DIP_DEVTOOLS_H_
#define DIP_DEVTOOLS_H_

#include "dip.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launch-shape override for the gathered GEMV kernels, for tuning sweeps.  0 restores the
 * built-in choice for that parameter.  Host-side, process-wide, not thread-safe against
 * concurrent launches.
 *   lanes_per_row  8, 16, 32 or 64 lanes cooperate on one stored row (16 bytes per lane)
 *   waves          wavefronts per workgroup: 2, 4, 8 or 16
 *   ksplit         workgroups that share one output strip (partial sums reduced in fixed order)
 *   unroll         rows in flight per lane group: 1, 2, 4 or 8
 */
int32_t dip_tune_gemv(int32_t lanes_per_row, int32_t waves, int32_t ksplit, int32_t unroll);

/*
 * The launch shape the gathered GEMV would use for matrix w and k selected rows, for
 * reports: shape_out (host, 4 ints) = {lanes_per_row, waves, ksplit, unroll}.
 * bundled != 0 asks for the up/gate kernel of dip_swiglu_mlp_forward (w = the bundled
 * matrix, two output halves per workgroup), 0 for the plain kernel.
 */
int32_t dip_gemv_launch_shape(const dip_weight* w, int32_t k, int32_t bundled, int32_t* shape_out);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel the library launches is
 * bracketed by a pair of HIP events bound to that dispatch (its own begin/end timestamps,
 * no extra work on the stream), up to max_launches launches; later launches are not timed.
 * The events are host objects; no device memory is allocated.  dip_profile_read() waits
 * for the recorded events and returns the summed duration and the number of launches of
 * one kernel kind.  Process-wide and not thread-safe: meant for a single benchmarking
 * thread.
 */
#define DIP_KERNEL_SELECT_IN 0   /* scores + top-K + cache update at pruning point 1       */
#define DIP_KERNEL_GEMV_UPGATE 1 /* gathered up/gate GEMV + SwiGLU                          */
#define DIP_KERNEL_SELECT_MID 2  /* scores + top-K + cache update at pruning point 2       */
#define DIP_KERNEL_GEMV_DOWN 3   /* gathered down GEMV (also dip_gathered_gemv)             */
#define DIP_KERNEL_GEMV_DENSE 4  /* dense first product of gate / up pruning                */
#define DIP_KERNEL_ROWDOT 5      /* row-gathered dot products                               */
#define DIP_KERNEL_TIER_FILL 6   /* host -> HBM copies of the columns a cache update inserted  */
#define DIP_KERNEL_CACHE_UPDATE 7 /* a cache update launched on its own (end of a forward call) */
#define DIP_KERNEL_STREAM_READ 8  /* dip_stream_read                                            */
#define DIP_KERNEL_KINDS 9
int32_t dip_profile_enable(int32_t max_launches);
int32_t dip_profile_read(int32_t kind, double* total_ms /* host */, int32_t* launches /* host */);
int32_t dip_profile_disable(void);

/*
 * Form of a pruning point in the forward calls.  1 (the default): the gathered product runs
 * the scores and the top-K of Alg. 1 at its own head, one launch per pruning point, where a
 * kernel covers the shape; 0: selection and product are always launched apart (two launches
 * per pruning point).  Masks, index lists and cache states are the same either way; sums
 * differ by rounding only when the two forms use different launch shapes.
 */
int32_t dip_set_fusion(int32_t on);

/*
 * shape_out (host, 4 ints) = {lanes_per_row, waves, ksplit, unroll} of the one-launch form for
 * a product over matrix w with k selected rows (bundled as in dip_gemv_launch_shape); returns
 * DIP_ERR_UNSUPPORTED when the forward calls would launch selection and product apart.
 */
int32_t dip_fused_launch_shape(const dip_weight* w, int32_t k, int32_t bundled, int32_t* shape_out);

/*
 * A plain streaming read of `bytes` bytes of device memory (16-byte aligned, a multiple of
 * 16; the contents must not xor to 0x9e3779b9), timed as kind DIP_KERNEL_STREAM_READ: the
 * bandwidth a kernel that only loads gets on this machine, to set beside the gathered products.
 *   src   device buffer       sink   one device word (written only in the excluded case)
 */
int32_t dip_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DIP_DEVTOOLS_H_ */
