// C-ABI layer: argument validation, workspace carving and kernel dispatch.
// Every step of the sampling path runs in the kernels of this library; the
// host side only validates, sizes and enqueues.
#include <hip/hip_runtime.h>
#include <string.h>

#include <mutex>

#include "../../include/flashfps.h"
#include "fps_launch.h"

static_assert(ffps::kErrGaveUp == FFPS_ERR_TIMEOUT && ffps::kErrInconsistent == FFPS_ERR_INTERNAL,
              "the kernels write these codes into the status word");

namespace {

using namespace ffps;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Workspace {  // byte offsets into the caller's workspace
    size_t status, exchange, cxyz, loc, bitmap, mind, cand, spos, total;
};

Workspace carve(int B, int N, int M) {
    Workspace w;
    size_t o = 0;
    w.status = o;   o += kAlign;
    w.exchange = o; o += align_up((size_t)kMaxGridWG * grid_exchange_bytes_per_cloud());
    w.cxyz = o;     o += align_up((size_t)B * N * 3 * sizeof(float));
    w.loc = o;      o += align_up((size_t)B * M * sizeof(int32_t));
    w.bitmap = o;   o += align_up((size_t)B * ((N + 31) / 32) * sizeof(uint32_t));
    w.mind = o;     o += align_up((size_t)B * N * sizeof(float));
    w.cand = o;     o += align_up((size_t)B * N * sizeof(int32_t));
    w.spos = o;     o += align_up((size_t)B * sizeof(int));
    w.total = o;
    return w;
}

struct Device {
    int ok;      // FFPS_OK or an error code
    int num_cu;
};

// Facts about a device that never change while the process lives (is it a
// gfx950, how many CUs), looked up once per device: the full property query is
// far dearer than a small launch.  This cache is the library's only state.
constexpr int kMaxDevices = 64;
std::mutex g_device_mutex;
bool g_device_known[kMaxDevices];
Device g_device[kMaxDevices];

// Device memory of the allocation-free entry point: the status block and the
// exchange areas of one launch, i.e. everything exact FPS needs besides its
// inputs and outputs as long as the clouds fit in registers.  Every device the
// library runs on holds its own copy of this array until the process ends.  In
// host code the name is only a handle: the array's address on a device comes
// from hipGetSymbolAddress, asked once per device with that device current.
constexpr size_t kScratchBytes = kAlign + (size_t)kMaxGridWG * kExchangeBytesPerCloud;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
char *g_scratch_ptr[kMaxDevices];  // address of `scratch` on each device, null until asked

Device query_device_uncached(int dev) {
    Device d{FFPS_ERR_LAUNCH_FAILED, 0};
    hipDeviceProp_t p;
    if (hipGetDeviceProperties(&p, dev) != hipSuccess) return d;
    if (strncmp(p.gcnArchName, "gfx950", 6) != 0) {
        d.ok = FFPS_ERR_UNSUPPORTED_DEVICE;
        return d;
    }
    d.ok = FFPS_OK;
    d.num_cu = p.multiProcessorCount;
    return d;
}

// Properties of the current device.
Device query_device(int *dev_out = nullptr) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return Device{FFPS_ERR_LAUNCH_FAILED, 0};
    if (dev_out) *dev_out = dev;
    if (dev < 0 || dev >= kMaxDevices) return query_device_uncached(dev);
    std::lock_guard<std::mutex> lock(g_device_mutex);
    if (!g_device_known[dev]) {
        g_device[dev] = query_device_uncached(dev);
        // a failed query is tried again by the next call
        g_device_known[dev] = g_device[dev].ok != FFPS_ERR_LAUNCH_FAILED;
    }
    return g_device[dev];
}

// Address of `scratch` on the current device (number `dev`), or null.
char *scratch_of_current_device(int dev) {
    if (dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_device_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = (char *)p;
    }
    return g_scratch_ptr[dev];
}

inline int hip_rc(hipError_t e) { return e == hipSuccess ? FFPS_OK : FFPS_ERR_LAUNCH_FAILED; }

int check_common(const void *xyz, int B, int N, int M, int start, const void *idx) {
    if (!xyz || !idx) return FFPS_ERR_INVALID_ARG;
    if (B < 1 || N < 1 || M < 1 || M > N) return FFPS_ERR_INVALID_ARG;
    if (start < 0 || start >= N) return FFPS_ERR_INVALID_ARG;
    if ((long)B * N > (1L << 31) - 1) return FFPS_ERR_INVALID_ARG;
    return FFPS_OK;
}

// The helper kernels of FPS-Prune and of the stage chain put the cloud number
// in gridDim.y, which the hardware limits to 65535.
constexpr int kMaxBatchHelpers = 65535;

// `variant` carries the kernel choice in its low byte and the optional
// picks-per-round cap above it (FFPS_VARIANT_WITH_PICKS).
inline int variant_kind(int variant) { return variant & 0xff; }
inline int variant_picks(int variant) {
    int p = (variant >> 8) & 0xff;
    return p == 0 ? kMaxPicksPerRound : p;
}
int check_variant(int variant) {
    if (variant < 0 || (variant >> 17) != 0) return FFPS_ERR_INVALID_ARG;
    int v = variant_kind(variant);
    return (v >= FFPS_VARIANT_AUTO && v <= FFPS_VARIANT_STREAM) ? FFPS_OK : FFPS_ERR_INVALID_ARG;
}

// The status word is cleared once per call; the exchange area before every
// grid launch (its tags restart at 1 in each launch).
int clear_status(char *ws, const Workspace &w, hipStream_t s) {
    return hip_rc(launch_fill_zero(ws + w.status, kAlign, s));
}
int clear_exchange(char *ws, const Workspace &w, int clouds, hipStream_t s) {
    return hip_rc(launch_fill_zero(ws + w.exchange, (size_t)clouds * grid_exchange_bytes_per_cloud(), s));
}

// Kernel variant that will run for clouds of N points, or a negative error.
int resolve_variant(int B, int N, int variant, const Device &dev) {
    int v = variant_kind(variant);
    if (v == FFPS_VARIANT_AUTO) {
        // Clouds that fit the multi-pick single-workgroup kernel run there, larger
        // ones on clusters of workgroups, those beyond the registers of the
        // device are streamed.
        if (N <= wgm_capacity())
            v = FFPS_VARIANT_WG;
        else if (N <= grid_capacity(dev.num_cu))
            v = FFPS_VARIANT_GRID;
        else
            v = FFPS_VARIANT_STREAM;
    }
    if (v == FFPS_VARIANT_WG && N > wg_capacity()) return FFPS_ERR_UNSUPPORTED_SIZE;
    if (v == FFPS_VARIANT_GRID && N > grid_capacity(dev.num_cu)) return FFPS_ERR_UNSUPPORTED_SIZE;
    if (v == FFPS_VARIANT_STREAM && N > stream_capacity()) return FFPS_ERR_UNSUPPORTED_SIZE;
    return v;
}

// Exact FPS of B clouds [N] into idx (row stride idx_stride).  Arguments are
// already validated.
int run_exact(const float *xyz, int B, int N, int M, int start, const int *start_dev, int variant,
              int32_t *idx, long idx_stride, float *md, long md_stride, char *ws,
              const Workspace &w, const Device &dev, hipStream_t s) {
    int v = resolve_variant(B, N, variant, dev);
    if (v < 0) return v;
    if (v == FFPS_VARIANT_WG)
        return hip_rc(launch_fps_wg(xyz, B, N, M, start, start_dev, idx, idx_stride, md, md_stride,
                                    variant_picks(variant), (int *)(ws + w.status), s));
    if (v == FFPS_VARIANT_GRID) {
        const GridPlan plan = plan_fps_grid(B, N, dev.num_cu);
        for (int b = 0; b < B; b += plan.clouds_per_launch) {
            const int clouds = B - b < plan.clouds_per_launch ? B - b : plan.clouds_per_launch;
            int rc = clear_exchange(ws, w, clouds, s);
            if (rc) return rc;
            hipError_t e = launch_fps_grid(xyz + (size_t)b * N * 3, clouds, N, M, start,
                                           start_dev ? start_dev + b : nullptr,
                                           idx + b * idx_stride, idx_stride,
                                           md ? md + b * md_stride : nullptr, md_stride,
                                           ws + w.exchange, (int *)(ws + w.status),
                                           plan.wg_per_cloud, variant_picks(variant),
                                           (variant & FFPS_VARIANT_TEST_NO_WAIT) ? 0 : -1, s);
            if (e != hipSuccess) return FFPS_ERR_LAUNCH_FAILED;
        }
        return FFPS_OK;
    }
    if (v == FFPS_VARIANT_STREAM) {
        for (int b = 0; b < B; ++b) {
            int rc = clear_exchange(ws, w, 1, s);
            if (rc) return rc;
            hipError_t e = launch_fps_stream(xyz + (size_t)b * N * 3, (float *)(ws + w.mind) + (size_t)b * N,
                                             N, M, start, start_dev ? start_dev + b : nullptr,
                                             idx + b * idx_stride,
                                             md ? md + b * md_stride : nullptr, ws + w.exchange,
                                             (int *)(ws + w.status), dev.num_cu,
                                             variant_picks(variant), s);
            if (e != hipSuccess) return FFPS_ERR_LAUNCH_FAILED;
        }
        return FFPS_OK;
    }
    return FFPS_ERR_UNSUPPORTED_SIZE;
}

int run_prune(const float *xyz, int B, int N, int M, int start, int keep_num, int keep_den,
              unsigned flags, uint64_t seed, int variant, int32_t *idx, long idx_stride, char *ws,
              const Workspace &w, const Device &dev, hipStream_t s) {
    int Nc, k, R;
    int rc = ffps_prune_sizes(N, M, keep_num, keep_den, flags, &Nc, &k, &R);
    if (rc) return rc;
    const bool perm = (flags & FFPS_FLAG_PERM) != 0;
    uint32_t *bitmap = (uint32_t *)(ws + w.bitmap);
    if (Nc < N) {
        float *cxyz = (float *)(ws + w.cxyz);
        int32_t *loc = (int32_t *)(ws + w.loc);
        if (perm) {
            int32_t *cand = (int32_t *)(ws + w.cand);
            int *spos = (int *)(ws + w.spos);
            rc = hip_rc(launch_perm_candidates(xyz, B, N, Nc, start, seed, bitmap, cand, cxyz, spos, s));
            if (rc) return rc;
            rc = run_exact(cxyz, B, Nc, k, 0, spos, variant, loc, k, nullptr, 0, ws, w, dev, s);
            if (rc) return rc;
            rc = hip_rc(launch_compose(cand, Nc, loc, k, B, k, idx, idx_stride, s));
        } else {
            rc = hip_rc(launch_gather_candidates(xyz, B, N, Nc, start, cxyz, s));
            if (rc) return rc;
            long j0 = (((long)N - start) * Nc + N - 1) / N;  // where the strided list wraps
            if (j0 > Nc) j0 = Nc;
            int spos = (int)((Nc - j0) % Nc);  // position of start_idx in the sorted list
            rc = run_exact(cxyz, B, Nc, k, spos, nullptr, variant, loc, k, nullptr, 0, ws, w, dev, s);
            if (rc) return rc;
            rc = hip_rc(launch_map_candidates(loc, k, B, N, Nc, start, k, idx, idx_stride, s));
        }
        if (rc) return rc;
    } else {
        rc = run_exact(xyz, B, N, k, start, nullptr, variant, idx, idx_stride, nullptr, 0, ws, w, dev, s);
        if (rc) return rc;
    }
    if (perm) return hip_rc(launch_fill_perm(B, N, k, R, seed, idx, idx_stride, bitmap, s));
    return hip_rc(launch_fill(B, N, k, R, idx, idx_stride, bitmap, s));
}

}  // namespace

extern "C" {

int ffps_version(void) { return 100; }

const char *ffps_strerror(int code) {
    switch (code) {
        case FFPS_OK: return "success";
        case FFPS_ERR_INVALID_ARG: return "invalid argument";
        case FFPS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case FFPS_ERR_UNSUPPORTED_DEVICE: return "device is not gfx950";
        case FFPS_ERR_LAUNCH_FAILED: return "HIP call failed";
        case FFPS_ERR_TIMEOUT: return "a workgroup stopped waiting for another";
        case FFPS_ERR_UNSUPPORTED_SIZE: return "kernel variant cannot hold this cloud size";
        case FFPS_ERR_INTERNAL: return "a kernel found its own intermediate results inconsistent";
        default: return "unknown error code";
    }
}

int ffps_prune_sizes(int N, int M, int keep_num, int keep_den, unsigned flags, int *Nc, int *k,
                     int *R) {
    if (!Nc || !k || !R) return FFPS_ERR_INVALID_ARG;
    if (N < 1 || M < 1 || M > N) return FFPS_ERR_INVALID_ARG;
    if (keep_num < 1 || keep_den < 1 || keep_num > keep_den) return FFPS_ERR_INVALID_ARG;
    if (flags & ~(FFPS_FLAG_CP | FFPS_FLAG_IP | FFPS_FLAG_PERM)) return FFPS_ERR_INVALID_ARG;
    long nc = (flags & FFPS_FLAG_CP) ? ((long)N * keep_num + keep_den - 1) / keep_den : N;
    long kk = (flags & FFPS_FLAG_IP) ? ((long)M * keep_num + keep_den - 1) / keep_den : M;
    if (kk < 1 || kk > nc) return FFPS_ERR_INVALID_ARG;
    *Nc = (int)nc;
    *k = (int)kk;
    *R = M - (int)kk;
    return FFPS_OK;
}

int ffps_workspace_bytes(int B, int N, int M, size_t *bytes) {
    if (!bytes || B < 1 || N < 1 || M < 1 || M > N) return FFPS_ERR_INVALID_ARG;
    if ((long)B * N > (1L << 31) - 1) return FFPS_ERR_INVALID_ARG;
    *bytes = carve(B, N, M).total;
    return FFPS_OK;
}

int ffps_exact(const float *d_xyz, int B, int N, int M, int start_idx, int variant, int32_t *d_idx,
               float *d_maxdist, void *d_ws, size_t ws_bytes, void *stream) {
    int rc = d_ws ? check_common(d_xyz, B, N, M, start_idx, d_idx) : FFPS_ERR_INVALID_ARG;
    if (rc) return rc;
    if ((rc = check_variant(variant))) return rc;
    Workspace w = carve(B, N, M);
    if (ws_bytes < w.total) return FFPS_ERR_WORKSPACE_TOO_SMALL;
    Device dev = query_device();
    if (dev.ok) return dev.ok;
    if ((rc = resolve_variant(B, N, variant, dev)) < 0) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = clear_status((char *)d_ws, w, s))) return rc;
    return run_exact(d_xyz, B, N, M, start_idx, nullptr, variant, d_idx, M, d_maxdist, M,
                     (char *)d_ws, w, dev, s);
}

int ffps_exact_noalloc(const float *d_xyz, int B, int N, int M, int start_idx, int variant,
                       int32_t *d_idx, float *d_maxdist, int32_t *d_status, void *stream) {
    int dev_no = 0;
    int rc = check_common(d_xyz, B, N, M, start_idx, d_idx);
    if (rc) return rc;
    if ((rc = check_variant(variant))) return rc;
    Device dev = query_device(&dev_no);
    if (dev.ok) return dev.ok;
    if ((rc = resolve_variant(B, N, variant, dev)) < 0) return rc;
    // the streaming kernel needs N running distances per cloud: beyond this array
    if (rc == FFPS_VARIANT_STREAM) return FFPS_ERR_UNSUPPORTED_SIZE;
    char *ws = scratch_of_current_device(dev_no);
    if (!ws) return FFPS_ERR_LAUNCH_FAILED;
    Workspace w;
    const size_t none = ~(size_t)0;
    w.status = 0; w.exchange = kAlign; w.total = kScratchBytes;
    w.cxyz = w.loc = w.bitmap = w.mind = w.cand = w.spos = none;  // not part of this path
    hipStream_t s = (hipStream_t)stream;
    if ((rc = clear_status(ws, w, s))) return rc;
    rc = run_exact(d_xyz, B, N, M, start_idx, nullptr, variant, d_idx, M, d_maxdist, M, ws, w, dev, s);
    if (rc) return rc;
    if (d_status)
        rc = hip_rc(launch_copy_prefix((const int32_t *)(ws + w.status), 2, 1, 2, d_status, 2, s));
    return rc;
}

int ffps_prune(const float *d_xyz, int B, int N, int M, int start_idx, int keep_num, int keep_den,
               unsigned flags, uint64_t seed, int variant, int32_t *d_idx, int *k_out_host,
               void *d_ws, size_t ws_bytes, void *stream) {
    int rc = d_ws ? check_common(d_xyz, B, N, M, start_idx, d_idx) : FFPS_ERR_INVALID_ARG;
    if (rc) return rc;
    if (B > kMaxBatchHelpers) return FFPS_ERR_INVALID_ARG;
    if ((rc = check_variant(variant))) return rc;
    int Nc, k, R;
    if ((rc = ffps_prune_sizes(N, M, keep_num, keep_den, flags, &Nc, &k, &R))) return rc;
    Workspace w = carve(B, N, M);
    if (ws_bytes < w.total) return FFPS_ERR_WORKSPACE_TOO_SMALL;
    Device dev = query_device();
    if (dev.ok) return dev.ok;
    if ((rc = resolve_variant(B, Nc, variant, dev)) < 0) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = clear_status((char *)d_ws, w, s))) return rc;
    if (k_out_host) *k_out_host = k;
    return run_prune(d_xyz, B, N, M, start_idx, keep_num, keep_den, flags, seed, variant, d_idx, M,
                     (char *)d_ws, w, dev, s);
}

int ffps_cached_stages(const float *d_xyz, int B, int N, int L, const int *M_stages, int start_idx,
                       int keep_num, int keep_den, unsigned flags, uint64_t seed, int mode,
                       int variant, int32_t *d_idx, void *d_ws, size_t ws_bytes, void *stream) {
    if (!M_stages || L < 1) return FFPS_ERR_INVALID_ARG;
    int rc = d_ws ? check_common(d_xyz, B, N, M_stages[0], start_idx, d_idx) : FFPS_ERR_INVALID_ARG;
    if (rc) return rc;
    if (B > kMaxBatchHelpers) return FFPS_ERR_INVALID_ARG;
    if ((rc = check_variant(variant))) return rc;
    if (mode != FFPS_MODE_CACHED && mode != FFPS_MODE_CHAIN) return FFPS_ERR_INVALID_ARG;
    long S = M_stages[0];
    for (int l = 1; l < L; ++l) {
        if (M_stages[l] < 1 || M_stages[l] > M_stages[l - 1]) return FFPS_ERR_INVALID_ARG;
        S += M_stages[l];
    }
    int Nc, k, R;
    if ((rc = ffps_prune_sizes(N, M_stages[0], keep_num, keep_den, flags, &Nc, &k, &R))) return rc;
    Workspace w = carve(B, N, M_stages[0]);
    if (ws_bytes < w.total) return FFPS_ERR_WORKSPACE_TOO_SMALL;
    Device dev = query_device();
    if (dev.ok) return dev.ok;
    if ((rc = resolve_variant(B, Nc, variant, dev)) < 0) return rc;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)d_ws;
    if ((rc = clear_status(ws, w, s))) return rc;

    rc = run_prune(d_xyz, B, N, M_stages[0], start_idx, keep_num, keep_den, flags, seed, variant,
                   d_idx, S, ws, w, dev, s);
    if (rc) return rc;
    long off = M_stages[0];
    const int32_t *prev = d_idx;
    for (int l = 1; l < L; ++l) {
        int32_t *cur = d_idx + off;
        if (mode == FFPS_MODE_CACHED) {
            rc = hip_rc(launch_copy_prefix(d_idx, S, B, M_stages[l], cur, S, s));
        } else {
            float *pxyz = (float *)(ws + w.cxyz);
            int32_t *loc = (int32_t *)(ws + w.loc);
            rc = hip_rc(launch_gather_points(d_xyz, B, N, prev, S, M_stages[l - 1], pxyz, s));
            if (rc) return rc;
            rc = run_exact(pxyz, B, M_stages[l - 1], M_stages[l], 0, nullptr, variant, loc,
                           M_stages[l], nullptr, 0, ws, w, dev, s);
            if (rc) return rc;
            rc = hip_rc(launch_compose(prev, S, loc, M_stages[l], B, M_stages[l], cur, S, s));
        }
        if (rc) return rc;
        prev = cur;
        off += M_stages[l];
    }
    return FFPS_OK;
}

int ffps_describe_plan(int B, int N, int variant, int num_cu, int *kernel, int *wg_per_cloud,
                       int *units_per_cloud, int *clouds_per_launch) {
    if (B < 1 || N < 1 || num_cu < 1 || check_variant(variant)) return FFPS_ERR_INVALID_ARG;
    Device dev{FFPS_OK, num_cu};
    const int v = resolve_variant(B, N, variant, dev);
    if (v < 0) return v;
    int wg = 1, units = 0, clouds = B;
    if (v == FFPS_VARIANT_WG) {
        units = wg_units(N);
    } else if (v == FFPS_VARIANT_GRID) {
        const GridPlan plan = plan_fps_grid(B, N, num_cu);
        wg = plan.wg_per_cloud;
        units = plan.units_per_cloud;
        clouds = plan.clouds_per_launch;
    } else {
        wg = stream_workgroups(N, num_cu);
        units = wg;
        clouds = 1;
    }
    if (kernel) *kernel = v;
    if (wg_per_cloud) *wg_per_cloud = wg;
    if (units_per_cloud) *units_per_cloud = units;
    if (clouds_per_launch) *clouds_per_launch = clouds;
    return FFPS_OK;
}

int ffps_last_status(const void *d_ws, void *stream) {
    if (!d_ws) return FFPS_ERR_INVALID_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return FFPS_ERR_LAUNCH_FAILED;
    int st = 0;
    if (hipMemcpy(&st, d_ws, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess)
        return FFPS_ERR_LAUNCH_FAILED;
    return st;
}

int ffps_gather_rows(const float *d_rows, int B, int N, int C, const int32_t *d_idx, long idx_stride,
                     int S, float *d_out, void *stream) {
    if (!d_rows || !d_idx || !d_out) return FFPS_ERR_INVALID_ARG;
    if (B < 1 || B > kMaxBatchHelpers || N < 1 || C < 1 || S < 1 || idx_stride < S) return FFPS_ERR_INVALID_ARG;
    Device dev = query_device();
    if (dev.ok) return dev.ok;
    return hip_rc(launch_gather_rows(d_rows, B, N, C, d_idx, idx_stride, S, d_out, (hipStream_t)stream));
}

int ffps_barrier_probe(int iters, void *d_ws, size_t ws_bytes, void *stream, float *us_per_barrier) {
    if (!d_ws || !us_per_barrier || iters < 1 || iters > (1 << 20)) return FFPS_ERR_INVALID_ARG;
    Workspace w = carve(1, 1, 1);
    if (ws_bytes < w.total) return FFPS_ERR_WORKSPACE_TOO_SMALL;
    Device dev = query_device();
    if (dev.ok) return dev.ok;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)d_ws;
    int rc = clear_status(ws, w, s);
    if (rc) return rc;
    if ((rc = clear_exchange(ws, w, 1, s))) return rc;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return FFPS_ERR_LAUNCH_FAILED;
    int G = dev.num_cu < kMaxGridWG ? dev.num_cu : kMaxGridWG;
    hipError_t e = hipEventRecord(e0, s);
    if (e == hipSuccess)
        e = launch_barrier_probe((unsigned *)(ws + w.exchange), (int *)(ws + w.status), G, iters, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    float ms = 0.f;
    if (e != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
        rc = FFPS_ERR_LAUNCH_FAILED;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    *us_per_barrier = ms * 1000.f / (float)iters;
    int st = 0;
    if (hipMemcpy(&st, ws + w.status, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess)
        return FFPS_ERR_LAUNCH_FAILED;
    return st;
}

int ffps_alu_probe(int waves_per_cu, int iters, void *d_ws, size_t ws_bytes, void *stream,
                   double *ops_per_s) {
    if (!d_ws || !ops_per_s || iters < 1 || iters > (1 << 20) || waves_per_cu < 1 || waves_per_cu > 32)
        return FFPS_ERR_INVALID_ARG;
    Workspace w = carve(1, 1, 1);
    if (ws_bytes < w.total) return FFPS_ERR_WORKSPACE_TOO_SMALL;
    Device dev = query_device();
    if (dev.ok) return dev.ok;
    hipStream_t s = (hipStream_t)stream;
    // up to 16 waves in a workgroup; more waves per CU as two workgroups per CU
    const int per_wg = waves_per_cu > 16 ? (waves_per_cu + 1) / 2 : waves_per_cu;
    const int num_wg = dev.num_cu * (waves_per_cu > 16 ? 2 : 1);
    if ((size_t)num_wg * per_wg * sizeof(float) > kExchangeBytesPerCloud) return FFPS_ERR_INVALID_ARG;
    float *sink = (float *)((char *)d_ws + w.exchange);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return FFPS_ERR_LAUNCH_FAILED;
    int rc = FFPS_OK;
    hipError_t e = launch_alu_probe(sink, num_wg, per_wg, 16, s);  // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = launch_alu_probe(sink, num_wg, per_wg, iters, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    float ms = 0.f;
    if (e != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
        rc = FFPS_ERR_LAUNCH_FAILED;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    // 16 values x 4 operations per lane and iteration
    *ops_per_s = (double)num_wg * per_wg * 64.0 * 16.0 * 4.0 * (double)iters / ((double)ms * 1e-3);
    return FFPS_OK;
}

int ffps_last_rounds(const void *d_ws, void *stream) {
    if (!d_ws) return FFPS_ERR_INVALID_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return FFPS_ERR_LAUNCH_FAILED;
    int st[2] = {0, 0};
    if (hipMemcpy(st, d_ws, sizeof(st), hipMemcpyDeviceToHost) != hipSuccess)
        return FFPS_ERR_LAUNCH_FAILED;
    return st[0] < 0 ? st[0] : st[1];
}

}  // extern "C"
