/* libopal: the five bandwidth-bound streaming vector kernels that the paper uses
 * as its small, memory-bound optimisation subjects (Table 1: Copy, Mul, Add,
 * Triad, Dot; Section 5.2), as hand-written HIP kernels for one MI355X
 * (CDNA4, gfx950) behind a C ABI.
 *
 * Common rules for every call
 *   Pointers   Every array pointer is DEVICE memory owned by the caller; the
 *              library never allocates, frees, copies to the host or keeps a
 *              pointer after the call returns.  Arrays are dense, contiguous
 *              and hold n elements of the type named by `dtype`.
 *   Alignment  An array pointer only has to be a multiple of its element size
 *              (8 for OPAL_F64, 4 for OPAL_F32); anything else is
 *              OPAL_ERR_ALIGN.  Arrays that are 1 KiB aligned, or that all
 *              share one misalignment, run on the fastest path.
 *   Aliasing   An output array must not overlap an input array of the same
 *              call (not checked; the result would be undefined).
 *   Stream     `stream` is a hipStream_t passed as void* (NULL = the default
 *              stream).  Every call only enqueues work on that stream and
 *              returns; it never synchronises.
 *   Scalar     `s` crosses the interface as double.  For OPAL_F32 it is rounded
 *              once, on the host, to float, and the kernel multiplies by that.
 *   Rounding   Elementwise results are the IEEE-754 round-to-nearest-even
 *              result of each single operation in the array's own type; Triad
 *              rounds the product and then the sum (it is never fused).  They
 *              are bit-identical to a plain CPU loop compiled without
 *              floating-point contraction.
 *   Errors     Only the return value reports errors; nothing is printed or
 *              thrown.  Argument errors are found on the host before any GPU
 *              work is enqueued, and then nothing is enqueued.  n == 0 is
 *              valid: nothing is launched (opal_dot still stores 0.0).
 *   Sizes      n is a size_t element count; arrays larger than 2 GiB are fine.  A
 *              dispatch holds at most 2^31 work-items, so a very large elementwise
 *              call is issued as several launches (one per 32 GiB of an array with
 *              fp64 or fp32 elements) on the same stream; only an n whose byte count
 *              does not fit half the address space is refused (OPAL_ERR_SIZE).
 *   Runtime    The library links the HIP runtime it finds at load time.  A process
 *              must use ONE copy of that runtime: streams and device pointers made
 *              by another copy (for instance the one a Python package ships, when
 *              the library was bound to the system's) are foreign to it.  Load the
 *              library after the module that owns the streams and pointers.
 */
#ifndef OPAL_H
#define OPAL_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Status codes (returned as int). */
enum {
  OPAL_OK = 0,
  OPAL_ERR_NULL = 1,      /* a required pointer is NULL while n > 0 (or result/workspace is NULL) */
  OPAL_ERR_DTYPE = 2,     /* dtype is neither OPAL_F64 nor OPAL_F32 */
  OPAL_ERR_ALIGN = 3,     /* a pointer is not a multiple of its element size (workspace/result: 8) */
  OPAL_ERR_WORKSPACE = 4, /* workspace_bytes < opal_dot_workspace_bytes(n, dtype) */
  OPAL_ERR_LAUNCH = 5,    /* the HIP runtime refused a query or a kernel launch */
  OPAL_ERR_SIZE = 6       /* n * element size does not fit an address, an LDS call's n is not a whole number
                             of tiles, or a tuning value is out of range */
};

/* Element types (passed as int). */
enum { OPAL_F64 = 0, OPAL_F32 = 1 };

/* Copy (Table 1):  c[i] = a[i],  0 <= i < n.
 * a: device, read, n elements.  c: device, written, n elements. */
int opal_copy(const void* a, void* c, size_t n, int dtype, void* stream);

/* Mul (Table 1; "scale" here):  b[i] = s * c[i].
 * c: device, read.  b: device, written.  One rounded multiply per element. */
int opal_scale(void* b, const void* c, double s, size_t n, int dtype, void* stream);

/* Add (Table 1):  c[i] = a[i] + b[i].
 * a, b: device, read.  c: device, written.  One rounded add per element. */
int opal_add(const void* a, const void* b, void* c, size_t n, int dtype, void* stream);

/* Triad (Table 1):  a[i] = b[i] + s * c[i], the product rounded first, then the sum.
 * b, c: device, read.  a: device, written. */
int opal_triad(void* a, const void* b, const void* c, double s, size_t n, int dtype, void* stream);

/* Bytes of device workspace opal_dot needs for n elements of `dtype`: room for one
 * fp64 partial sum per workgroup of its first pass.  A pure host function of its
 * arguments (no GPU call), at most 64 KiB, and 0 for an unknown dtype. */
size_t opal_dot_workspace_bytes(size_t n, int dtype);

/* Dot (Table 1):  *result = sum_{i<n} a[i] * b[i].
 * a, b: device, read.  workspace: device, 8-byte aligned, at least
 * opal_dot_workspace_bytes(n, dtype) bytes, overwritten.  result: device, one
 * fp64 (also for OPAL_F32), 8-byte aligned, written.
 * Two kernels on `stream`: each workgroup of the first writes one fp64 partial
 * sum to the workspace, the second adds the partials in a fixed order.  No
 * atomics: for given (pointers' alignment, n, dtype, device, pacing setting) the
 * result is bit-reproducible from run to run.  OPAL_F64 accumulates in fp64 throughout
 * (with fused multiply-adds); OPAL_F32 accumulates in fp32 within a thread and
 * a wavefront and in fp64 from there on.
 * Calls that share a workspace must be ordered (same stream, or synchronised).
 * n == 0 stores 0.0; result and workspace must still be valid pointers (a NULL
 * workspace is OPAL_ERR_NULL also for n == 0: the check does not depend on n). */
int opal_dot(const void* a, const void* b, size_t n, int dtype,
             void* workspace, size_t workspace_bytes, double* result, void* stream);

/* opal_dot for callers that cannot allocate device memory or pass a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation).
 * Same kernels, same result bits as opal_dot for the same (a, b, n, dtype, device);
 * the first pass writes its partial sums into a fixed 64 KiB array that lives in the
 * library's device image (one copy per GPU, held until the process ends) instead of a
 * caller workspace.  The call itself never allocates or frees; the array's device
 * address is looked up once per device, on the first call made with that device current.
 * opal_dot_static_scratch_bytes() is that array's size, the largest workspace any n
 * needs; a call whose first pass would need more is refused with OPAL_ERR_WORKSPACE
 * and enqueues nothing.  a, b, result, stream and every other rule are as for opal_dot.
 * All calls on one GPU share the one array, which keeps the previous call's partial
 * sums (every slot that is read is rewritten first, so nothing needs clearing):
 * calls that may overlap on one GPU (different streams, no ordering between them)
 * race and must be serialised by the caller. */
size_t opal_dot_static_scratch_bytes(void);
int opal_dot_static(const void* a, const void* b, size_t n, int dtype, double* result, void* stream);

/* Launch shapes for arrays far beyond the caches ("paced" shapes).  For large arrays on an
 * MI355X (from 768 MiB per array for Copy and Mul, 512 MiB for Add and Triad, 384 MiB for Dot)
 * the five kernels run as persistent wavefronts that issue their loads and stores in bursts on a
 * common timetable read off the chip-wide constant-rate counter, so that HBM sees one stream and
 * one direction at a time (2-3 % more bytes per second for the elementwise kernels, 3-4 % for
 * Dot, than workgroups handed out in index order; Add and Triad load their second input in the
 * order that suits where the two inputs lie relative to each other, see csrc/launch_plan.hpp).  Results are the
 * same bits either way.  The timetable keeps a few device words of feedback inside the library's
 * device image (one copy per GPU); calls that overlap on one GPU share them, which can only cost
 * speed.  opal_set_pacing(0) switches to index-ordered workgroups for every size, 1 (the
 * default) uses the paced shapes from the sizes above on, 2 uses them for every array that holds at
 * least 16 chunks of the timetable (128 MiB for Copy and Mul; for measurements and tests).  The
 * environment variable OPAL_PACING=0|1|2 sets the same before the first call; opal_get_pacing()
 * returns the current mode.  Process-wide, not per stream. */
void opal_set_pacing(int mode);
int opal_get_pacing(void);

/* The order in which the paced Add and Triad load the runs of their second input.  By default it is one of
 * two orders that match the first input's memory-channel classes (csrc/launch_plan.hpp, matched_run); which
 * of the two suits a pair of arrays depends on address bits a kernel cannot see, so the kernels time
 * themselves: of every 128 launches with the same two inputs and n, the first four alternate between the
 * two orders and the others use the faster one (csrc/pacing.hpp).  What was learnt lives in a few device
 * words inside the library's device image (one copy per GPU, 64 pairs; pairs that collide, and calls that
 * overlap on one GPU, learn nothing or the wrong order: slower, same results).
 * opal_set_matched_order: 0 loads the second input in the same order as the first (no matching), 2 times
 * the other of the two orders first, any other value restores the default; every call starts the learning
 * afresh.  For measurements and tests; same results whatever the value; process-wide, call it while no
 * other thread is inside the library.
 * opal_matched_order_state: what has been learnt for the pair of inputs a paced Add or Triad call with these
 * arguments would use (out: the call's output array; host pointer state[4] receives: launches so far, the
 * shortest duration in ticks of the 100 MHz counter with order 0 and with order 1 (0xFFFFFFFF: none yet),
 * the order the next launch will use).  Synchronous: it copies from the device with hipMemcpy, which waits
 * for the work queued on the default stream only; synchronise any other stream the calls in question
 * went to before asking.  For tests and diagnosis.  Errors: OPAL_ERR_DTYPE, OPAL_ERR_NULL, OPAL_ERR_LAUNCH. */
void opal_set_matched_order(int on);
int opal_matched_order_state(const void* out, const void* in0, const void* in1, size_t n, int dtype,
                             unsigned state[4]);

/* Tuning hook for the timetable of one kind of paced kernel (0: Copy and Mul, 1: Add and Triad,
 * 2: Dot): the rate the timetable asks of memory in TB/s (1 TB = 1e12 B), where in the period the
 * store burst goes (fraction in [0,1); 0 = as soon as the data has arrived), for Dot how long
 * after the burst of `a` the burst of `b` goes (fraction of the period; for Add and Triad the
 * same for their second input), how far apart the accesses of one burst are spread (fraction of
 * the period, below 0.25; 0 = all at once), how many ticks late a
 * wavefront has to be before the timetable is pushed back, whether lateness is fed back at
 * all, and which bit of the workgroup index splits the wavefronts into the two sets (0..8; 3 puts
 * whole compute units into one set).  Defaults are the measured optimum on MI355X; a timetable that asks too much degrades to
 * unordered traffic, it never affects results.  OPAL_ERR_SIZE for a value out of range.
 * Like opal_set_pacing it changes process-wide state that every launch reads: call it while no
 * other thread is inside the library. */
int opal_pacing_configure(int kind, double terabytes_per_second, double store_at, double second_input_at,
                          double gap, unsigned tolerance_ticks, int feedback, unsigned set_bit);

/* LDS streaming microkernel: the analogue, for this chip's 160 KiB local data share, of the
 * shared-memory benchmark the paper lists beside the five kernels (Table 1: the Shmembench row,
 * parameter rep = kernel repetition count, 300..1500, default 600; Section 5.2 says it exercises
 * shared memory).  The paper gives no definition, so this one is the library's own:
 *
 *   The arrays are cut into tiles of OPAL_LDS_TILE_VECTORS (1024) 16-byte vectors (2048 fp64
 *   or 4096 fp32 elements).  A tile is loaded into the LDS and then goes through `rep` rounds;
 *   in one round every vector j of the tile becomes  x'[j] = x[(j + 1) mod 1024] + c  (the
 *   tile rotates by one vector and c is added to every element, one rounded add), each round
 *   reading what the previous one wrote through the LDS.  After the last round the tile is
 *   stored to `out`.  So  out = rotate_by_rep(in) with c added rep times, tile by tile.
 *
 * in: device, read, n elements; out: device, written, n elements, must not overlap in.  Both
 * 16-byte aligned (else OPAL_ERR_ALIGN).  n must be a multiple of opal_lds_tile_elements(dtype)
 * (else OPAL_ERR_SIZE).  rep = 0 copies.  LDS traffic: 32 bytes per vector per round. */
#define OPAL_LDS_TILE_VECTORS 1024
size_t opal_lds_tile_elements(int dtype);   /* 2048 (fp64), 4096 (fp32), 0 for an unknown dtype */
int opal_lds_stream(const void* in, void* out, double c, size_t n, unsigned rep, int dtype, void* stream);

/* Static, NUL-terminated description of a status code (never NULL). */
const char* opal_status_string(int status);

/* Name of the last HIP runtime error the calling thread met inside this library
 * ("hipSuccess" if none): the detail behind an OPAL_ERR_LAUNCH.  Static string. */
const char* opal_last_hip_error(void);

/* Algorithmic bytes per element: every input read once and every output written
 * once (16/16/24/24/16 for fp64, half that for fp32).  kernel: 0 copy, 1 scale,
 * 2 add, 3 triad, 4 dot.  Returns 0 for an unknown kernel or dtype. */
size_t opal_bytes_per_element(int kernel, int dtype);

#ifdef __cplusplus
}
#endif

#endif /* OPAL_H */
