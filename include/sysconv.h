/*
 * sysconv.h -- C ABI of libsysconv: 1-D and 2-D fp32 "valid" convolution run as
 * a software systolic array inside the 64-lane wavefronts of an AMD MI355X
 * (gfx950).
 *
 * The operations are the ones the paper "Systolic Computing on GPUs for
 * Productive Performance" (arXiv 2010.15884) uses as its examples:
 *
 *   1-D, Eq. 2 (Section 3.1):  y[c]    = sum_q         x[c+q]      * w[q]
 *   2-D, Eq. 3 (Section 5):    y[r][c] = sum_p sum_q   x[r+p][c+q] * f[p][q]
 *
 * (also at stride 2, sys_conv1d_strided / sys_conv2d_strided, and for 1-D designs given as
 * data, sys_conv1d_stt)
 *
 * No filter flip, no padding: n inputs and k taps give n-k+1 outputs.  The
 * paper's systolic (fast) axis c,q is the column of a row-major image.
 * Data and arithmetic are fp32 (the paper's SIMD8 float vectors, Section 6);
 * the order of the k (or kh*kw) fused multiply-adds depends on the projection,
 * so projections agree with each other to rounding, not bit for bit.
 *
 * A "projection" is one of the space-time mappings of Section 3.1 / Table 2,
 * named (input, weight, partial sum) with B = broadcast, F = forwarded from
 * PE to PE, S = stays, M = migrates, S = sediments:
 *
 *   FBS  partial sums and weights stay in registers, inputs move one PE per
 *        time step (Table 2, row 3 left).  PE = output position; here four
 *        consecutive PEs share a lane, so three of four hand-overs are
 *        register renames and the fourth is a one-lane DPP move.
 *   SBM  inputs stay, partial sums move one PE per step, results appear k-1
 *        PEs further on (Section 3.1, the paper's worked example).
 *   BFS  partial sums stay, each input is broadcast to every PE that needs
 *        it while the weights move past (Table 2, row 2 left).  Here the PE
 *        array runs along the per-lane registers (1-D: consecutive outputs of
 *        one lane; 2-D: consecutive output rows of one lane).
 *   BSM, FSM, FFS (1-D only)  the remaining designs of Table 2, one PE per lane:
 *        BSM and FSM arrays are k lanes long (PE = tap; weights stay; partial sums
 *        move up resp. down; inputs are broadcast resp. move at half speed), FFS
 *        arrays are 16 PEs long (PE = output; inputs and weights both move).  The
 *        paper measures them as inferior; they are provided to reproduce that
 *        ranking, and run several times slower than FBS / SBM / BFS.
 *
 * Conventions common to every entry point
 *   - d_* pointers are DEVICE memory on the current HIP device; h_* pointers
 *     are HOST memory.  The caller owns all of them.  The library allocates
 *     nothing on the device and keeps no state between calls.
 *   - Host taps are copied into the kernel-argument block before the call
 *     returns; the caller may free or change them immediately.
 *   - Calls are asynchronous: work is enqueued on `stream` (0 = the null
 *     stream) and the call returns without synchronising.
 *   - A call enqueues kernels and nothing else (no allocation, no memset, no copy, no
 *     synchronisation), so it may be recorded into a HIP graph by stream capture; a
 *     replay then uses the taps of the recorded call, which travel in the kernel
 *     arguments.
 *   - Device buffers need only 4-byte alignment; 16-byte aligned bases and
 *     pitches that are multiples of 4 elements are fastest.
 *   - Arguments are validated before any HIP call is made.  Nothing aborts:
 *     every failure is an integer status and no kernel is launched.
 *   - Input and output ranges must not overlap (SYS_ERR_ALIAS).
 */
#ifndef SYSCONV_H
#define SYSCONV_H

#include <stddef.h>

#ifdef SYSCONV_NO_HIP_HEADER
typedef struct ihipStream_t *hipStream_t;
#else
#include <hip/hip_runtime_api.h>
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SYS_OK = 0,
    SYS_ERR_NULL = 1,         /* a required pointer is NULL                          */
    SYS_ERR_SIZE = 2,         /* k < 1, k > n, pitch < width, empty output, ...      */
    SYS_ERR_ALIAS = 3,        /* input and output byte ranges overlap                */
    SYS_ERR_UNSUPPORTED = 4,  /* size beyond the limits below / unknown projection /
                                 projection not built for this filter size          */
    SYS_ERR_HIP = 5,          /* a HIP call failed; see sys_last_hip_error()         */
    SYS_ERR_DESIGN = 6        /* a space-time design breaks the recurrences or the
                                 conditions of Section 2.2 (see sys_stt_check)       */
} sys_status_t;

typedef enum {
    SYS_PROJ_AUTO = 0,        /* the fastest projection available for the size       */
    SYS_PROJ_FBS = 1,
    SYS_PROJ_BFS = 2,
    SYS_PROJ_SBM = 3,
    SYS_PROJ_BSM = 4,         /* 1-D only */
    SYS_PROJ_FSM = 5,         /* 1-D only */
    SYS_PROJ_FFS = 6,         /* 1-D only */
    SYS_PROJ_MFMA = 7         /* 2-D only, never chosen by AUTO: see sys_conv2d          */
} sys_projection_t;

/* Limits.  Larger filters return SYS_ERR_UNSUPPORTED. */
#define SYS_MAX_K1D 64        /* taps of a 1-D filter                                */
#define SYS_MAX_K2D 15        /* rows and columns of a 2-D filter                    */

/*
 * 1-D valid convolution, Eq. 2:  d_y[c] = sum_{q<k} d_x[c+q] * h_w[q],  c < n-k+1.
 *   d_x   device, n floats (read only)
 *   h_w   host, k floats, 1 <= k <= min(n, SYS_MAX_K1D)
 *   d_y   device, n-k+1 floats (written; nothing else is touched)
 *   projection  a sys_projection_t; every projection accepts every k in range
 *         (sys_conv1d_has reports it).  SYS_PROJ_AUTO is FBS, and BFS from 36 taps on
 *         or for n >= 2^29, where BFS measures faster on MI355X.
 */
int sys_conv1d(const float *d_x, size_t n,
               const float *h_w, int k,
               float *d_y,
               int projection, hipStream_t stream);

/*
 * Strided 1-D valid convolution:  d_y[c] = sum_{q<k} d_x[stride*c+q] * h_w[q],
 * c < (n-k)/stride + 1  (integer division).  This is what the stride-2 FBS design of
 * Table 2 (row 3 right) computes: its hand-over X(c,q) = X(c+1,q-2) is the identity
 * x(2c+q) = x(2(c+1)+q-2); the cell's printed "x(c+q)" is read as x(2c+q).
 *   stride 1  identical to sys_conv1d (every projection).
 *   stride 2  FBS only (SYS_PROJ_AUTO or SYS_PROJ_FBS); any 1 <= k <= min(n, SYS_MAX_K1D).
 *   other strides, or other projections at stride 2: SYS_ERR_UNSUPPORTED
 *             (sys_conv1d_strided_has reports it); stride < 1: SYS_ERR_SIZE.
 *   d_x   device, n floats (read only);  d_y  device, (n-k)/stride + 1 floats (written).
 */
int sys_conv1d_strided(const float *d_x, size_t n,
                       const float *h_w, int k, int stride,
                       float *d_y,
                       int projection, hipStream_t stream);

/* 1 if sys_conv1d_strided(projection) is built for a k-tap filter at this stride, else 0. */
int sys_conv1d_strided_has(int projection, int k, int stride);

/*
 * A 1-D systolic design in the paper's terms (Section 2.2, Section 3.1, Table 2) over the
 * iteration space z = (c, q), output position c and tap q:
 *   alloc  P:  processing element  = alloc[0]*c + alloc[1]*q
 *   sched  s:  time step           = sched[0]*c + sched[1]*q
 *   X, the input x(c+q): loaded by every PE that needs it (x_passed = 0), or handed on,
 *      X(z) = X(z - dep_x) wherever z - dep_x lies in the PE array's chunk of outputs;
 *      dep_x = (a, -a), a != 0, since both points must read the same input.
 *   W, the tap w(q): w_passed = 0, or W(z) = W(z - dep_w) with dep_w = (a, 0), a != 0.
 *   Z, the partial sum: Z(z) = Z(z - dep_z) + X(z)*W(z), dep_z = (0, 1) (taps ascending)
 *      or (0, -1) (descending); the output leaves where that chain ends.
 * SBM is {P=(1,1), s=(0,1), dep_x=(-1,1), W loaded, dep_z=(0,1)}; the rows of Table 2 are
 * written the same way.
 */
typedef struct {
    int alloc[2];
    int sched[2];
    int x_passed;
    int dep_x[2];
    int w_passed;
    int dep_w[2];
    int dep_z[2];
} sys_stt_design_t;

/*
 * Check a design for a k-tap filter without running anything:
 *   SYS_OK               it can be run by sys_conv1d_stt
 *   SYS_ERR_DESIGN       it is not a valid systolic design: a dependence vector does not
 *                        fit the recurrences above, the transform is singular (two
 *                        iteration points on one PE at one time), or a passed value
 *                        would be needed before it exists (s.e < 1; Section 2.2)
 *   SYS_ERR_UNSUPPORTED  valid, but beyond this kernel: |det(P; s)| != 1, a value that
 *                        travels more than one PE per hand-over (|P.e| > 1) or more than
 *                        3 time steps (s.e > 3), coefficients beyond +-64, or a PE vector
 *                        that does not fit 64 lanes for this k
 *   SYS_ERR_NULL / SYS_ERR_SIZE  design == NULL / k outside 1..SYS_MAX_K1D
 */
int sys_stt_check(const sys_stt_design_t *design, int k);

/*
 * 1-D valid convolution (Eq. 2, as sys_conv1d) executed by the general form of the
 * paper's generated code (Section 4.1) for the given design: one PE per lane, per-PE
 * histories as deep as each variable's time distance, the transform inverted at every
 * step.  Every design that passes sys_stt_check gives the result of sys_conv1d to
 * rounding; it runs several times slower than the hand-laid projections and exists to
 * try designs, not to serve them.  Arguments and errors as sys_conv1d, plus those of
 * sys_stt_check.
 */
int sys_conv1d_stt(const float *d_x, size_t n,
                   const float *h_w, int k,
                   float *d_y,
                   const sys_stt_design_t *design, hipStream_t stream);

/*
 * 2-D valid convolution, Eq. 3, single channel, row-major:
 *   d_y[r*y_pitch + c] = sum_{p<kh} sum_{q<kw} d_x[(r+p)*x_pitch + c+q] * h_f[p*kw+q]
 * for r < h-kh+1, c < w-kw+1.
 *   d_x      device, h rows of w floats, row stride x_pitch elements (>= w)
 *   h_f      host, kh*kw floats row-major, 1 <= kh <= min(h, SYS_MAX_K2D), same for kw / w
 *   d_y      device, h-kh+1 rows of w-kw+1 floats, row stride y_pitch elements
 *            (>= w-kw+1); elements between rows are left untouched
 *   projection  AUTO and FBS accept every filter in range (AUTO, from measurements: square
 *            filters up to 6x6 run FBS, or BFS where x_pitch * 4 is a power of two of at most
 *            16 KB; 7x7 .. 11x11 run SBM; everything else FBS); BFS and SBM are built
 *            for SQUARE filters 2x2 .. 11x11 only (sys_conv2d_has) and return
 *            SYS_ERR_UNSUPPORTED otherwise; BSM, FSM and FFS are 1-D only.  FBS runs
 *            kernels specialised at compile time for every filter of up to 11 rows and
 *            columns whose smaller side is at most 7 (square or not; this includes single
 *            rows and columns, 1 x k and k x 1: the two passes of a
 *            separable filter, which run at the rate of a plain copy), and a kernel with
 *            run-time filter sizes otherwise.
 *   h, w     at most INT_MAX - 2048 (SYS_ERR_UNSUPPORTED beyond; pitches at most 2^31).
 *
 * SYS_PROJ_MFMA (opt-in; any filter with kh, kw <= 13, square or not) leaves the paper's
 * software arrays for the matrix cores: Section 6.2 / Table 5 observe that 2-D throughput
 * collapses as the filter grows, and here an 11x11 filter is bound by the vector ALUs, not by
 * memory.  Inputs and taps are split into two fp16 numbers each (hi + lo, 22 significant
 * bits), three of the four partial products are accumulated in fp32 by
 * v_mfma_f32_16x16x32_f16, and the result is fp32.  What the caller must know:
 *   - every input must satisfy |x| < 8 (inputs are scaled by 2^13 before the split; a
 *     larger value becomes infinite and turns the outputs it feeds into inf / NaN);
 *     the taps are scaled by a power of two that the library derives from the largest
 *     |f|, which must be 0 or lie within [1e-30, 1e30] (SYS_ERR_UNSUPPORTED otherwise);
 *   - each input is represented to 2^-22 relative; inputs below 2^-27 (7.5e-9) in magnitude
 *     count as zero, and so do taps below 2^-28 of the largest tap.  On data spread over
 *     [0, 1] or [-1, 1] the results agree with the fp64 definition to about 1e-7 of
 *     sum |f||x| (better than an fp32 chain of 121 multiply-adds).  The input range is a
 *     promise the library cannot check, which is why AUTO never picks this path;
 *   - a non-finite input (or tap) also spoils outputs outside its window, up to 18 rows
 *     above / 3 below and 15 columns left / 3 right of it (0 * inf inside the blocked sums).
 */
int sys_conv2d(const float *d_x, int h, int w, size_t x_pitch,
               const float *h_f, int kh, int kw,
               float *d_y, size_t y_pitch,
               int projection, hipStream_t stream);

/*
 * Strided 2-D valid convolution, the same stride on both axes:
 *   d_y[r*y_pitch + c] = sum_{p<kh} sum_{q<kw} d_x[(stride*r+p)*x_pitch + stride*c+q] * h_f[p*kw+q]
 * for r < (h-kh)/stride + 1, c < (w-kw)/stride + 1 (integer divisions).  The paper's
 * experiment (Section 6) runs its convolutions at stride 1 or 2 and gives the stride-2
 * design for one axis (Table 2, row 3 right); applying it along the columns and taking
 * every second row is this library's reading for two axes.
 *   stride 1  identical to sys_conv2d (every projection).
 *   stride 2  FBS only (SYS_PROJ_AUTO or SYS_PROJ_FBS); any filter up to SYS_MAX_K2D.
 *   other strides, or other projections at stride 2: SYS_ERR_UNSUPPORTED
 *             (sys_conv2d_strided_has reports it); stride < 1: SYS_ERR_SIZE.
 * Arguments as sys_conv2d; d_y has (h-kh)/stride + 1 rows of (w-kw)/stride + 1 floats.
 */
int sys_conv2d_strided(const float *d_x, int h, int w, size_t x_pitch,
                       const float *h_f, int kh, int kw, int stride,
                       float *d_y, size_t y_pitch,
                       int projection, hipStream_t stream);

/* 1 if sys_conv2d_strided(projection) is built for a kh x kw filter at this stride, else 0. */
int sys_conv2d_strided_has(int projection, int kh, int kw, int stride);

/* 1 if sys_conv1d(projection) is built for a k-tap filter, else 0. */
int sys_conv1d_has(int projection, int k);

/* 1 if sys_conv2d(projection) is built for a kh x kw filter, else 0. */
int sys_conv2d_has(int projection, int kh, int kw);

/*
 * Plain device-to-device copy of n floats with 16-byte accesses.  It is the
 * yard-stick the benchmark prints beside every convolution ("what the memory
 * system gives a streaming kernel of this footprint") and the kernel of known
 * traffic that hardware byte counters are calibrated against.
 */
int sys_copy_f32(const float *d_src, float *d_dst, size_t n, hipStream_t stream);

/*
 * The vector-ALU counterpart of sys_copy_f32: a register-only loop of fp32 multiply-adds (taps in
 * scalar registers, as in the convolution kernels), `workgroups` x 256 lanes x `trips` x 256
 * multiply-adds.  The benchmark prints its rate beside the ALU-bound 11x11 row: what the vector
 * ALUs of this part sustain with one v_fmac_f32 per lane and clock.
 *   d_out  device, workgroups * 256 floats (written: one value per lane)
 * Returns the number of multiply-adds enqueued, or minus a sys_status_t on error
 * (workgroups and trips must lie in 1 .. 2^20).
 */
long long sys_alu_yardstick_f32(float *d_out, int workgroups, int trips, hipStream_t stream);

const char *sys_status_string(int status);
const char *sys_projection_name(int projection);

/* hipError_t (as int) behind the calling thread's most recent SYS_ERR_HIP; 0 if this thread
 * has never seen one.  Later successful calls do not clear it. */
int sys_last_hip_error(void);

/* major*10000 + minor*100 + patch */
int sys_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SYSCONV_H */
