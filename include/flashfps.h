/*
 * flashfps.h -- C ABI of the MI355X (gfx950) farthest-point-sampling library.
 *
 * The library computes farthest point sampling (FPS) as the FlashFPS paper
 * states it: exact FPS (Sec. 3.1, Eq. 1), FPS-Prune (Sec. 3.2; Alg. 1,
 * layer 1) and the hierarchical stage chain with or without FPS-Cache
 * (Sec. 3.3; Alg. 1, layers 2..L).
 *
 * Conventions shared by every entry point
 *   - "d_" arguments are DEVICE pointers, everything else is host data.
 *   - Clouds are fp32 array-of-structs: d_xyz[b][i][0..2], b < B, i < N,
 *     densely packed ([B][N][3]); coordinates must be finite.
 *   - Indices are int32 positions in [0, N) of the caller's cloud, also for
 *     pruned and chained variants.
 *   - Distance is the squared Euclidean distance ((dx*dx)+(dy*dy))+(dz*dz)
 *     with every operation rounded to fp32 and no fused multiply-add; the
 *     running minimum starts at +inf; the argmax runs over all points and a
 *     tie goes to the lowest index.  With these rules the result is unique,
 *     independent of the launch shape, and identical from run to run.
 *   - Ownership: the caller owns every buffer.  The library allocates no
 *     device memory and keeps no state besides a per-device note of facts that
 *     never change (device kind, CU count); calls on different streams are
 *     independent provided they use different workspaces.
 *   - Asynchrony: work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and the call returns without
 *     synchronising.  Outputs are valid once the stream has been synchronised.
 *     A call only enqueues kernel launches (no host round trip, no memset, no
 *     allocation), so it may be recorded into a HIP graph by stream capture;
 *     the buffers and the workspace then belong to that graph's replays.
 *   - Errors: 0 on success, a negative FFPS_ERR_* code otherwise.  Arguments
 *     are validated on the host before anything is enqueued, so an invalid
 *     call has no effect on the device.
 */
#ifndef FLASHFPS_H
#define FLASHFPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FFPS_OK 0
#define FFPS_ERR_INVALID_ARG (-1)         /* null pointer, size out of range, M > N, bad ratio ... */
#define FFPS_ERR_WORKSPACE_TOO_SMALL (-2) /* ws_bytes < ffps_workspace_bytes(...)                  */
#define FFPS_ERR_UNSUPPORTED_DEVICE (-3)  /* current device is not gfx950                          */
#define FFPS_ERR_LAUNCH_FAILED (-4)       /* a HIP call failed                                     */
#define FFPS_ERR_TIMEOUT (-5)             /* a kernel gave up waiting for another workgroup        */
#define FFPS_ERR_UNSUPPORTED_SIZE (-6)    /* the requested kernel variant cannot hold this N       */
#define FFPS_ERR_INTERNAL (-7)            /* a kernel found its own intermediate results inconsistent */

/* FPS-Prune switches (Alg. 1, layer 1). */
#define FFPS_FLAG_CP 1u /* candidate pruning: FPS sees only N' = ceil(N * keep) points      */
#define FFPS_FLAG_IP 2u /* iteration pruning: FPS stops after k = ceil(M * keep) picks       */
#define FFPS_FLAG_PERM 4u /* seeded random sub-sample and fill instead of the strided ones    */

/* How layers 2..L of a stage chain are produced. */
#define FFPS_MODE_CACHED 0 /* FPS-Cache: prefixes of layer 1 (Alg. 1, layers 2..L)           */
#define FFPS_MODE_CHAIN 1  /* every layer runs its own FPS on the previous layer (Sec. 3.3)  */

/* Kernel variant; AUTO picks by (B, N). */
#define FFPS_VARIANT_AUTO 0
#define FFPS_VARIANT_WG 1     /* one workgroup per cloud, points resident in registers       */
#define FFPS_VARIANT_GRID 2   /* each cloud across many CUs, points resident in registers    */
#define FFPS_VARIANT_STREAM 3 /* one cloud across all CUs, points streamed from HBM per pass */
/* Benchmarking knob: cap on the picks accepted per round, i.e. per pass over the
 * points (1 = one pick per pass; 0 = library default).  The result never
 * depends on it. */
#define FFPS_VARIANT_WITH_PICKS(variant, picks) ((variant) | ((picks) << 8))
/* Test knob for the error path: a workgroup of the GRID kernel that does not find
 * the records of all other workgroups at its first look gives up at once instead
 * of after the library's bound on waiting.  Every workgroup then leaves the
 * kernel in the ordinary way and the status word reads FFPS_ERR_TIMEOUT; the
 * outputs of such a call are unspecified. */
#define FFPS_VARIANT_TEST_NO_WAIT (1 << 16)

/* Library version: major * 10000 + minor * 100 + patch.  Host only. */
int ffps_version(void);

/* Static, NUL-terminated description of an FFPS_* code.  Host only. */
const char *ffps_strerror(int code);

/*
 * Sizes of FPS-Prune for pruning ratio p, given as keep_num/keep_den = 1 - p
 * (Alg. 1: N' = (1-p) N, k = (1-p) M1, p M1 fill picks; both products are
 * rounded up, in 64-bit integers):
 *   *Nc = candidate count N' (N when FFPS_FLAG_CP is off)
 *   *k  = FPS picks          (M when FFPS_FLAG_IP is off)
 *   *R  = M - k fill picks
 * Host only.  FFPS_ERR_INVALID_ARG unless 0 < keep_num <= keep_den,
 * 1 <= M <= N and 1 <= k <= N'.
 */
int ffps_prune_sizes(int N, int M, int keep_num, int keep_den, unsigned flags, int *Nc, int *k,
                     int *R);

/*
 * Upper bound, in bytes, of the device workspace any entry point below needs
 * for B clouds of N points and at most M samples per cloud.  Host only.
 * The workspace needs 256-byte alignment and no initialisation.
 */
int ffps_workspace_bytes(int B, int N, int M, size_t *bytes);

/*
 * Exact FPS (Sec. 3.1, Eq. 1).
 *   d_xyz      in   [B][N][3] fp32
 *   M          samples per cloud, 1 <= M <= N
 *   start_idx  index of the first sample (the fixed seed point of Sec. 1), in [0, N)
 *   variant    FFPS_VARIANT_*
 *   d_idx      out  [B][M] int32; d_idx[b][0] = start_idx, then the picks in order
 *   d_maxdist  out  [B][M] fp32 or NULL: squared minimum distance each pick had
 *                   when it was chosen; entry 0 is +inf
 *   d_ws       workspace of ws_bytes >= ffps_workspace_bytes(B, N, M)
 */
int ffps_exact(const float *d_xyz, int B, int N, int M, int start_idx, int variant,
               int32_t *d_idx, float *d_maxdist, void *d_ws, size_t ws_bytes, void *stream);

/*
 * ffps_exact for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): takes
 * no workspace and allocates nothing.  What the kernels need besides inputs and
 * outputs (the status block and the exchange areas of one launch, 12 MiB + 256
 * bytes) lives in an array inside the library's device image; every GPU the
 * library runs on holds its copy until the process ends.
 *   arguments   as ffps_exact, without d_ws / ws_bytes
 *   d_status    out  int32[2] on the device, or NULL: {status word, rounds} of
 *                    this call, readable through ffps_last_status(d_status, stream)
 *                    and ffps_last_rounds(d_status, stream)
 * Limit: clouds must fit the register-resident kernels, N <= 12288 points per CU
 * (3,145,728 on MI355X); beyond that, or with FFPS_VARIANT_STREAM, the call
 * returns FFPS_ERR_UNSUPPORTED_SIZE and enqueues nothing.  B is not limited.
 * All calls on one GPU share that GPU's array (each call clears what it needs
 * at the start): calls that may run at the same time on one GPU, on whatever
 * streams, race and must be serialised by the caller.  The outputs equal
 * ffps_exact's bit for bit.
 */
int ffps_exact_noalloc(const float *d_xyz, int B, int N, int M, int start_idx, int variant,
                       int32_t *d_idx, float *d_maxdist, int32_t *d_status, void *stream);

/*
 * FPS-Prune (Sec. 3.2; Alg. 1, layer 1).  With (N', k, R) = ffps_prune_sizes:
 *   candidates  the N' indices sort{ (start_idx + floor(j*N/N')) mod N : j < N' }
 *               (an index-uniform subsample that contains start_idx);
 *   FPS part    d_idx[b][0..k)  = exact FPS over the candidates, first sample
 *               start_idx, ties to the lowest index, mapped to indices of the
 *               full cloud, in FPS order;
 *   fill part   d_idx[b][k..M)  = free[floor(j*(N-k)/R)], j < R, where free is
 *               the ascending list of the N-k indices the FPS part did not pick
 *               (drawn from the full cloud, not from the candidates).
 * keep = 1/1 (p = 0) gives exactly ffps_exact.  k_out_host (may be NULL)
 * receives k.  Other arguments as ffps_exact; B <= 65535.
 *
 * With FFPS_FLAG_PERM the two deterministic strided rules are replaced by the
 * literal random draws of Alg. 1, made reproducible by `seed` (cloud b uses
 * seed + b).  Let perm_s be the seeded bijection of [0, N): a 4-round Feistel
 * network over 2h bits (2^(2h) >= N, h >= 1) on the halves (l, r) of the argument,
 *   f = mix(r ^ (key[round & 1] + 0x9E3779B9 * (round + 1))) & (2^h - 1),
 *   (l, r) <- (r, l ^ f),   key = {low, high 32 bits of s},
 *   mix(x): x ^= x >> 16; x *= 0x85EBCA6B; x ^= x >> 13; x *= 0xC2B2AE35; x ^= x >> 16,
 * repeated until the value is below N.  Then
 *   candidates  sort{ perm_seed(j) : j < N' }, with perm_seed(N'-1) replaced by
 *               start_idx when start_idx is not among them;
 *   fill part   the first R values of perm_(seed ^ 0xD1B54A32D192ED03)(0), (1), ...
 *               that the FPS part did not pick, in that order.
 * `seed` is ignored without FFPS_FLAG_PERM.
 */
int ffps_prune(const float *d_xyz, int B, int N, int M, int start_idx, int keep_num,
               int keep_den, unsigned flags, uint64_t seed, int variant, int32_t *d_idx,
               int *k_out_host, void *d_ws, size_t ws_bytes, void *stream);

/*
 * Hierarchical stage chain (Alg. 1; Sec. 3.3).
 *   L, M_stages  host array of L sample counts, N >= M_stages[0] >= ... >= M_stages[L-1] >= 1
 *   layer 1      ffps_prune with M = M_stages[0] and the same keep, flags, seed
 *                (exact FPS when keep = 1/1)
 *   FFPS_MODE_CACHED  layer l = first M_stages[l] entries of layer 1
 *   FFPS_MODE_CHAIN   layer l = exact FPS over the points of layer l-1 taken in
 *                     sample order, started at its first point, M_stages[l]
 *                     picks, mapped back to indices of the full cloud
 *   d_idx        out [B][S], S = sum of M_stages; layer l of cloud b starts at
 *                d_idx[b*S + M_stages[0] + ... + M_stages[l-1]]
 *   d_ws         workspace of ws_bytes >= ffps_workspace_bytes(B, N, M_stages[0])
 * B <= 65535.
 */
int ffps_cached_stages(const float *d_xyz, int B, int N, int L, const int *M_stages,
                       int start_idx, int keep_num, int keep_den, unsigned flags, uint64_t seed,
                       int mode, int variant, int32_t *d_idx, void *d_ws, size_t ws_bytes,
                       void *stream);

/*
 * What the layer after a sampling stage consumes (Sec. 1: each stage samples,
 * then aggregates features around the samples): the rows of a per-point fp32
 * array at the sampled indices, in sample order.
 *   d_rows  in  [B][N][C] fp32 (C = 3 for coordinates, or any feature width)
 *   d_idx   in  int32, S indices per cloud, cloud b at d_idx + b * idx_stride
 *               (a stage of ffps_cached_stages: pass its offset and the row
 *               length sum(M_stages) as idx_stride); every index in [0, N)
 *   d_out   out [B][S][C]
 * B <= 65535.  Needs no workspace.
 */
int ffps_gather_rows(const float *d_rows, int B, int N, int C, const int32_t *d_idx, long idx_stride,
                     int S, float *d_out, void *stream);

/*
 * Status word the kernels of the last call on this workspace left behind:
 * synchronises `stream`, copies one int from the workspace and returns it
 * (FFPS_OK; FFPS_ERR_TIMEOUT when a workgroup stopped waiting for another;
 * FFPS_ERR_INTERNAL when a round of a multi-pick kernel named no pick, which
 * the method rules out, and the kernel went on only in order to end; the
 * outputs of such a call are undefined).
 */
int ffps_last_status(const void *d_ws, void *stream);

/*
 * Largest number of rounds any cloud took in a multi-pick kernel of the last
 * call on this workspace (each round delivers one or more picks), or a
 * negative status as ffps_last_status.  0 if no such kernel ran (clouds of at
 * most 256 points use a one-pick kernel).  Synchronises `stream`.  Diagnostic:
 * for a single ffps_exact launch, (M - 1) / rounds = picks per round.
 */
int ffps_last_rounds(const void *d_ws, void *stream);

/*
 * How a call on B clouds of N points would be laid over a device with num_cu
 * compute units (256 on MI355X), without touching any device.  Host only.
 *   *kernel              FFPS_VARIANT_WG / _GRID / _STREAM that `variant`
 *                        (AUTO or explicit) resolves to
 *   *wg_per_cloud        workgroups that share one cloud (1 for WG)
 *   *units_per_cloud     reporting units of a round (0 for the one-pick kernel
 *                        that serves clouds of at most 256 points, and clouds
 *                        beyond 4608 points when WG is forced)
 *   *clouds_per_launch   clouds one kernel launch carries
 * Any output pointer may be NULL.  FFPS_ERR_INVALID_ARG for B, N, num_cu < 1,
 * FFPS_ERR_UNSUPPORTED_SIZE when the requested variant cannot hold N.
 */
int ffps_describe_plan(int B, int N, int variant, int num_cu, int *kernel, int *wg_per_cloud,
                       int *units_per_cloud, int *clouds_per_launch);

/*
 * Reference measurement for the multi-workgroup kernels: runs `iters`
 * (1 .. 2^20) plain grid barriers (one device-scope atomic arrive plus a spin
 * on the counter each) over one workgroup per CU, the launch shape of the GRID
 * and STREAM variants, and stores the mean time of one barrier in
 * microseconds to *us_per_barrier (host).  Synchronises `stream`.  d_ws as for
 * the other calls (ffps_workspace_bytes(1, 1, 1) suffices).
 */
int ffps_barrier_probe(int iters, void *d_ws, size_t ws_bytes, void *stream, float *us_per_barrier);

/*
 * Diagnostic for benchmarks, not part of the sampling path: the sustained rate
 * of individually rounded fp32 vector operations (subtract, multiply, add,
 * minimum: the arithmetic of one distance update of Eq. 1, no FMA, no memory
 * traffic) with waves_per_cu waves of 64 lanes resident on every compute unit
 * (1 .. 32), each lane working on 16 independent values for `iters` rounds.
 * Creates two events, launches two kernels and waits for them.
 *   d_ws / ws_bytes  a workspace of at least ffps_workspace_bytes(1, 1, 1); its
 *                    exchange area takes one word per wave
 *   ops_per_s        out (host): operations per second over all lanes
 * Returns FFPS_OK or FFPS_ERR_INVALID_ARG / WORKSPACE_TOO_SMALL / LAUNCH_FAILED.
 */
int ffps_alu_probe(int waves_per_cu, int iters, void *d_ws, size_t ws_bytes, void *stream,
                   double *ops_per_s);

#ifdef __cplusplus
}
#endif
#endif /* FLASHFPS_H */
