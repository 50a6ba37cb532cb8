// Host-side launch interface between the C-ABI layer (api.hip) and the kernel
// translation units.  Plain pointers and sizes only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ffps {

#ifndef FFPS_MAX_PICKS
#define FFPS_MAX_PICKS 192
#endif
constexpr int kMaxPicksPerRound = FFPS_MAX_PICKS;  // picks one round may deliver
// Status words the kernels write themselves (the C interface's FFPS_ERR_TIMEOUT
// and FFPS_ERR_INTERNAL).
constexpr int kErrGaveUp = -5;
constexpr int kErrInconsistent = -7;

// ---- fps_wg.hip: one workgroup per cloud ------------------------------------
int wg_capacity();   // largest N the single-workgroup kernels hold
int wgm_capacity();  // largest N of the multi-pick single-workgroup kernel
int wg_units(int N);  // reporting units of the kernel that serves N points (0: one-pick kernel)
int stream_workgroups(int N, int num_cu);  // workgroups the streaming kernel spreads N points over
int stream_capacity();  // largest N the streaming kernel takes (its 32-bit point counters must not wrap)
// In all FPS launchers `start_dev`, when not null, is a device array with one
// start index per cloud that overrides `start` (read by the kernel).
// `max_picks` caps the picks one pass over the points may deliver (0: no cap
// beyond kMaxPicksPerRound); the result does not depend on it.  status[1]
// receives the largest number of passes any cloud took (multi-pick kernel only).
hipError_t launch_fps_wg(const float *xyz, int B, int N, int M, int start, const int *start_dev,
                         int32_t *idx, long idx_stride, float *md, long md_stride, int max_picks,
                         int *status, hipStream_t s);

// ---- fps_grid.hip: clouds spread over the whole device, resident in registers ----
constexpr int kMaxGridWG = 256;      // workgroups (one per CU) a launch may use
// bytes of one cloud's exchange area: two buffers of four 16-byte chunks for each of 256 units
constexpr size_t kExchangeBytesPerCloud = 2 * 6 * (size_t)kMaxGridWG * 16;
size_t grid_exchange_bytes_per_cloud();  // the same value, as the kernels' own headers derive it
long grid_capacity(int num_cu);          // largest N the register-resident grid kernel holds
// How B clouds of N points are laid over the device: workgroups per cloud, and
// how many clouds one launch carries (each cloud on its own cluster of workgroups).
struct GridPlan {
    int wg_per_cloud;
    int clouds_per_launch;
    int units_per_cloud;  // reporting units of a round
};
GridPlan plan_fps_grid(int B, int N, int num_cu);
// `clouds` clouds (densely packed, outputs idx_stride / md_stride apart) in one
// launch.  `exchange` needs clouds * grid_exchange_bytes_per_cloud() bytes, cleared
// (all zero) on the same stream.  status[0] receives an error code if a
// workgroup gives up, status[1] the largest number of exchange rounds a cloud took.
hipError_t launch_fps_grid(const float *xyz, int clouds, int N, int M, int start,
                           const int *start_dev, int32_t *idx, long idx_stride, float *md,
                           long md_stride, void *exchange, int *status, int wg_per_cloud,
                           int max_picks, int spin_limit, hipStream_t s);  // spin_limit < 0: the default

// ---- fps_stream.hip: one cloud over the whole device, streamed from HBM ------
// `mind` is an [N] fp32 scratch array; `exchange` and `status` as for the grid kernel.
hipError_t launch_fps_stream(const float *xyz, float *mind, int N, int M, int start,
                             const int *start_dev, int32_t *idx, float *md, void *exchange,
                             int *status, int num_cu, int max_picks, hipStream_t s);

// ---- aux.hip: small helper kernels -------------------------------------------
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);
// `iters` grid barriers over num_wg co-resident workgroups; *counter must be zero
hipError_t launch_barrier_probe(unsigned *counter, int *status, int num_wg, int iters, hipStream_t s);
hipError_t launch_alu_probe(float *sink, int num_wg, int waves_per_wg, int iters, hipStream_t s);
// cxyz[b][i] = xyz[b][cand(i)], cand = the sorted strided candidate list (see flashfps.h)
hipError_t launch_gather_candidates(const float *xyz, int B, int N, int Nc, int start,
                                    float *cxyz, hipStream_t s);
// idx[b][j] = cand(loc[b][j]) for j < k
hipError_t launch_map_candidates(const int32_t *loc, long loc_stride, int B, int N, int Nc,
                                 int start, int k, int32_t *idx, long idx_stride, hipStream_t s);
// idx[b][k + j] = j-th strided rank of the indices not in idx[b][0..k)
hipError_t launch_fill(int B, int N, int k, int R, int32_t *idx, long idx_stride,
                       uint32_t *bitmap, hipStream_t s);
// Seeded random candidate set of cloud b (seed + b): ascending list cand[b][0..Nc),
// its coordinates cxyz[b][0..Nc), and spos[b] = position of `start` in the list.
hipError_t launch_perm_candidates(const float *xyz, int B, int N, int Nc, int start, uint64_t seed,
                                  uint32_t *bitmap, int32_t *cand, float *cxyz, int *spos,
                                  hipStream_t s);
// idx[b][k + r], r < R = first R indices, in the order of a second seeded permutation,
// that are not in idx[b][0..k)
hipError_t launch_fill_perm(int B, int N, int k, int R, uint64_t seed, int32_t *idx, long idx_stride,
                            uint32_t *bitmap, hipStream_t s);
// dst[b][j] = xyz[b][sel[b][j]] for j < S
hipError_t launch_gather_points(const float *xyz, int B, int N, const int32_t *sel,
                                long sel_stride, int S, float *dst, hipStream_t s);
// out[b][j][0..C) = rows[b][sel[b][j]][0..C) for j < S
hipError_t launch_gather_rows(const float *rows, int B, int N, int C, const int32_t *sel,
                              long sel_stride, int S, float *out, hipStream_t s);
// out[b][j] = prev[b][loc[b][j]] for j < S
hipError_t launch_compose(const int32_t *prev, long prev_stride, const int32_t *loc,
                          long loc_stride, int B, int S, int32_t *out, long out_stride,
                          hipStream_t s);
// out[b][j] = src[b][j] for j < S
hipError_t launch_copy_prefix(const int32_t *src, long src_stride, int B, int S, int32_t *out,
                              long out_stride, hipStream_t s);

}  // namespace ffps
