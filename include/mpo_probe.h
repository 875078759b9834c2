/*
 * mpo_probe — measuring aids that go with libmpo (libmpo_probe.so): the memory traffic of the
 * split-precision optimizer step (arXiv 2309.12381, Section 3.1: 26 bytes per parameter for
 * Adam) with the arithmetic taken out, plain streams, and a search for where to put the
 * optimizer state in the device memory.  Nothing here is part of the method and libmpo.so
 * does not depend on it.
 *
 * All pointers are DEVICE pointers on the current HIP device unless said otherwise, 16-byte
 * aligned.  `stream` is a hipStream_t passed as void* (NULL = default stream).  Return value:
 * 0, or -1 for a bad argument, or the hipError_t of a HIP call that failed.  The probes
 * overwrite the arrays they are given.
 */
#ifndef MPO_PROBE_H
#define MPO_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per parameter: reads hi, res, grad (2 bytes each) and m, v (4 bytes each) and writes hi,
 * res, m, v back in place, over the first n - n % 4096 parameters, in the launch shape of the
 * step kernel's long chunks.  v may be NULL: the 18-byte traffic of SGD with momentum.
 * Asynchronous on `stream`. */
int mpo_probe_stream(void *hi, void *res, const void *grad, void *m, void *v, long long n, void *stream);

/* The Adam-shaped traffic with one choice of the launch shape changed (lane width, cache
 * policy, rows in flight, chunk length, row order, persistent workgroups, software
 * pipelining, workgroup size, chunk order); variant 0 is mpo_probe_stream's shape.  Runs over
 * the first n - n % 131072 parameters; `compute_units` sizes the grid of the persistent
 * variant. */
int mpo_probe_num_variants(void);
const char *mpo_probe_variant_name(int variant);
int mpo_probe_variant(int variant, void *hi, void *res, const void *grad, void *m, void *v, long long n,
                      int compute_units, void *stream);

/* k (1 to 8) arrays (`arrays`: a HOST array of k device pointers) of `bytes` bytes each (the
 * first bytes - bytes % 16384 are used) walked in lock step: mode 0 reads them, 1 writes
 * them, 2 reads them and writes them back.  `sink`: 4 bytes of device memory. */
int mpo_probe_plain(int mode, void *const *arrays, int k, unsigned long long bytes, void *sink, void *stream);

/* Where to put res, v and the gradient buffer, given hi and m: for callers that do not go
 * through the Python package (whose placement.py does the same search on torch tensors).
 *
 * On MI355X the device memory behaves as three regions of 96 GiB, and a step whose written
 * arrays all lie in one region runs about 13 % slower than one whose written arrays are
 * divided between two; allocations made one after the other in a fresh process all land in
 * the first region.  This call allocates (hipMalloc) up to 8 candidate blocks one after the
 * other, at least 16 GiB apart (filler blocks between small ones; nothing is freed during
 * the search, because freed memory comes back in any order), each laid out as
 *     res at offset 0, v at *v_offset, grad at *grad_offset (multiples of 256 bytes),
 * times the probe on windows of 2^26 parameters at four matching positions of hi, m, res and
 * v (the way the step walks them), and stops at the first candidate that is faster than the
 * one-region reference (every window but hi's taken from inside m) by 7 % on average and by
 * 4 % at each position.  The fastest candidate is returned in *block (free it with hipFree or
 * mpo_place_free); the others and the fillers are freed.  It knows no physical addresses:
 * every decision is a measurement, reported in *report.
 *
 *   hi, hi_bytes     the 16-bit weights (at least 2^27 bytes); the windows the probe
 *                    overwrites are saved and restored when keep_hi != 0.
 *   m, m_bytes       the fp32 first moments (at least 6 * 2^27 bytes), allocated right after
 *                    hi; OVERWRITTEN: clear it afterwards.
 *   res_bytes, v_bytes, grad_bytes   sizes of the three parts of the block (res at least 2^27
 *                    bytes, v at least 2^28; grad may be 0 or small: the probe then reads its
 *                    gradient window from a part of m, where read-only data lie does not matter).
 *   max_transient_bytes  most the search may hold beyond the block it returns; 0 = half of
 *                    the free device memory at entry.
 * Arrays below the sizes above are not probed: the block is allocated plainly and
 * report->split is 0.  The call synchronises with the device. */
typedef struct {
    int32_t split;                 /* 1: the returned block shows the gain of a second region */
    int32_t candidates;            /* blocks tried */
    int32_t chosen;                /* index of the one returned */
    int32_t reserved;
    double one_region_GBps[4];     /* the reference at the four positions */
    double chosen_GBps[4];         /* the returned block at the four positions */
    uint64_t peak_transient_bytes; /* most that was held beyond the returned block */
    uint64_t max_transient_bytes;  /* the bound that applied */
    uint64_t block_bytes;          /* size of the block */
    uint64_t v_offset, grad_offset;
} mpo_place_report;

int mpo_place_second(void *hi, uint64_t hi_bytes, void *m, uint64_t m_bytes, uint64_t res_bytes, uint64_t v_bytes,
                     uint64_t grad_bytes, uint64_t max_transient_bytes, int keep_hi, void **block,
                     mpo_place_report *report, void *stream);
int mpo_place_free(void *block);

#ifdef __cplusplus
}
#endif
#endif /* MPO_PROBE_H */
