/*
 * slide_prof.h - measurement hooks of libslide (used by bench.py and the profiling tools; not part of the step's
 * interface in slide.h).  Same conventions as slide.h.
 */
#ifndef SLIDE_PROF_H_
#define SLIDE_PROF_H_

#include "slide.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-launch timing.  Between slide_prof_begin and slide_prof_end every launch of the kernel family `kernel_id`
 * (SLIDE_PROF_ALL: of every family) is bracketed by a pair of HIP events recorded on the launch's own stream
 * (events are created by the library on first use; at most SLIDE_PROF_MAX launches are recorded, later ones run
 * unrecorded).  slide_prof_end synchronises on the recorded events and returns the summed duration (milliseconds),
 * the number of launches recorded and the FLOPs / algorithmic bytes those launches were asked to do (host
 * pointers; any may be NULL).  slide_prof_family returns the same four figures for one family of the last
 * recording.  Families are numbered 0 .. as slide_kernel_name enumerates them. */
#define SLIDE_PROF_MAX 4096
#define SLIDE_PROF_ALL (-1)
int         slide_prof_begin(slide_ctx* ctx, int kernel_id);
int         slide_prof_end(slide_ctx* ctx, double* total_ms, int* launches, double* flops, double* bytes);
int         slide_prof_family(const slide_ctx* ctx, int kernel_id, double* total_ms, int* launches, double* flops,
                              double* bytes);
const char* slide_kernel_name(int kernel_id);  /* NULL past the last id */

/* A plain device-to-device copy kernel (calib_copy_k) of `bytes` bytes (a multiple of 16; dst and src 16-byte
 * aligned device pointers, not overlapping).  It moves a known number of bytes, which is what the hardware traffic
 * counters of the other kernels are scaled with. */
int  slide_calib_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIDE_PROF_H_ */
