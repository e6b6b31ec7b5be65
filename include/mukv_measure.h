/*
 * libmukv -- measurement aids.  NOT part of the method's interface (that is
 * mukv.h): the hooks a benchmark uses to time the library's kernels with HIP
 * events on the stream they are launched on, and a plain copy kernel that
 * hardware traffic counters are calibrated against.  Exported by the same
 * shared library.
 */
#ifndef MUKV_MEASURE_H
#define MUKV_MEASURE_H

#include "mukv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel families timed by the profiling hooks below. */
typedef enum mukv_kernel_id {
    MUKV_K_ATT = 0,     /* Eq. 1 attention signal                              */
    MUKV_K_FREQ = 1,    /* Eq. 2-3 frequency signal                            */
    MUKV_K_SELECT = 2,  /* Eq. 4 fusion, keep, Eq. 5 frame / super-patch keys  */
    MUKV_K_REFINE = 3,  /* fp64 re-scoring of near-tie frames (three kernels)  */
    MUKV_K_COMPACT = 4, /* copy of kept rows of all layers + segment keys      */
    MUKV_K_POOLQ = 5,   /* Eq. 6                                               */
    MUKV_K_SCORE = 6,   /* Eq. 7                                               */
    MUKV_K_RERANK = 7,  /* top-k selections and Eq. 8                          */
    MUKV_K_GATHER = 8,  /* Sec. 3.5 gather                                     */
    MUKV_K_COPY_FREQ = 9, /* overlap_copy: copy of the previous batch's kept rows and
                             Eq. 2-3 of the new batch in one launch                */
    MUKV_K_CHAIN = 10,  /* overlap_copy with the matrix-core attention: that copy, Eq. 2-3
                             and Eq. 1 of the new batch in one launch              */
    MUKV_K_COUNT = 11
} mukv_kernel_id;

typedef struct mukv_profile {
    double ms[MUKV_K_COUNT];        /* summed HIP-event time of the family's launches */
    int64_t launches[MUKV_K_COUNT]; /* number of timed launches                        */
} mukv_profile;

/*
 * Measurement hooks (for benchmarks; not part of the method).  Between
 * mukv_profile_begin and mukv_profile_end every kernel the library enqueues is
 * bracketed by a pair of HIP events recorded on the caller's stream;
 * mukv_profile_end waits for those events (this is the one call that blocks
 * on the device), adds up the elapsed times per kernel family into *out and
 * releases the events.  Not allowed inside a stream capture.
 */
int mukv_profile_begin(mukv_ctx *ctx);
int mukv_profile_end(mukv_ctx *ctx, mukv_profile *out);

/* Measurement aid: a plain 16-bytes-per-thread device copy of `bytes` bytes (a
 * multiple of 16; both pointers 16-byte aligned) on `stream`.  Used to calibrate
 * hardware traffic counters against a kernel whose HBM traffic is known. */
int mukv_plain_copy(void *dst, const void *src, int64_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MUKV_MEASURE_H */
