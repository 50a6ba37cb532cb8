// k_fps_wg: exact FPS (Sec. 3.1, Eq. 1), one workgroup per cloud.
//
// The whole cloud lives in registers for the duration of the call: thread t
// holds points [t*P, t*P+P) and their running minimum distances, so lane order,
// wave order and index order coincide and "lowest index wins a tie" becomes
// "lowest lane / lowest wave wins".  Per pick: P distance updates per lane, a
// per-lane argmax, a DPP max across the wave, one LDS exchange across waves
// (double-buffered, so a single s_barrier per pick).  Nothing is re-read from
// HBM after the initial load.
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

struct WaveSlot {  // what one wave reports per pick
    uint32_t dbits;
    int idx;
    float x, y, z;
    uint32_t pad[3];
};

template <int NT, int P>
__global__ __launch_bounds__(NT) void k_fps_wg(const float *__restrict__ xyz_all, int N, int M,
                                               int start_in, const int *__restrict__ start_dev,
                                               int32_t *__restrict__ idx_all,
                                               long idx_stride, float *__restrict__ md_all,
                                               long md_stride) {
    constexpr int NW = NT / kWave;
    __shared__ WaveSlot slots[2][NW > 1 ? NW : 1];

    const int b = blockIdx.x;
    const int start = start_dev ? start_dev[b] : start_in;
    const float *xyz = xyz_all + (size_t)b * N * 3;
    int32_t *idx_out = idx_all + (size_t)b * idx_stride;
    float *md_out = md_all ? md_all + (size_t)b * md_stride : nullptr;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int base = tid * P;

    float x[P], y[P], z[P], m[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        int i = base + j;
        bool ok = i < N;
        x[j] = ok ? xyz[3 * (size_t)i + 0] : 0.f;
        y[j] = ok ? xyz[3 * (size_t)i + 1] : 0.f;
        z[j] = ok ? xyz[3 * (size_t)i + 2] : 0.f;
        // padding lanes hold distance 0 forever: they cannot beat a real point,
        // and they sit at the highest indices, so they lose every tie as well
        m[j] = ok ? __builtin_inff() : 0.f;
    }

    float lx = xyz[3 * (size_t)start + 0];
    float ly = xyz[3 * (size_t)start + 1];
    float lz = xyz[3 * (size_t)start + 2];
    if (tid == 0) {
        idx_out[0] = start;
        if (md_out) md_out[0] = __builtin_inff();
    }

    for (int k = 1; k < M; ++k) {
        // distance update + per-lane argmax (ascending j, strict >)
        float bd = 0.f;
        int bj = 0;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            float d = sqdist(x[j], y[j], z[j], lx, ly, lz);
            m[j] = fminf(m[j], d);
            if (j == 0) {
                bd = m[0];
            } else if (m[j] > bd) {
                bd = m[j];
                bj = j;
            }
        }
        // wave argmax: max of the bits, then the lowest lane that holds it
        uint32_t wbits = wave_max_u32(f2u(bd));
        int wl = first_lane(f2u(bd) == wbits);
        int wj = readlane_i(bj, wl);
        float wx, wy, wz;
        pick_xyz<P>(x, y, z, wj, wl, wx, wy, wz);
        int widx = (wave * kWave + wl) * P + wj;

        if constexpr (NW == 1) {
            lx = wx; ly = wy; lz = wz;
            if (tid == 0) {
                idx_out[k] = widx;
                if (md_out) md_out[k] = u2f(wbits);
            }
        } else {
            WaveSlot *buf = slots[k & 1];
            if (lane == 0) {
                buf[wave].dbits = wbits;
                buf[wave].idx = widx;
                buf[wave].x = wx;
                buf[wave].y = wy;
                buf[wave].z = wz;
            }
            __syncthreads();
            // every wave reduces the NW slots on its own: lowest wave wins a tie
            uint32_t sb = lane < NW ? buf[lane].dbits : 0u;
            uint32_t gb = (uint32_t)__builtin_amdgcn_readlane((int)row16_max_u32(sb), 15);
            int ww = first_lane(lane < NW && sb == gb);
            lx = buf[ww].x;
            ly = buf[ww].y;
            lz = buf[ww].z;
            if (tid == 0) {
                idx_out[k] = buf[ww].idx;
                if (md_out) md_out[k] = u2f(gb);
            }
        }
    }
}

template <int NT, int P>
static hipError_t launch_wg_t(const float *xyz, int B, int N, int M, int start, const int *start_dev,
                              int32_t *idx, long idx_stride, float *md, long md_stride,
                              hipStream_t s) {
    hipLaunchKernelGGL((k_fps_wg<NT, P>), dim3(B), dim3(NT), 0, s, xyz, N, M, start, start_dev, idx,
                       idx_stride, md, md_stride);
    return hipGetLastError();
}

int wg_capacity() { return 1024 * 24; }

// Shapes are ordered by capacity; the first one that holds N is used.
hipError_t launch_fps_wg(const float *xyz, int B, int N, int M, int start, const int *start_dev,
                         int32_t *idx, long idx_stride, float *md, long md_stride, hipStream_t s) {
#define FFPS_WG_CASE(NT, P)         \
    if (N <= (NT) * (P))            \
        return launch_wg_t<NT, P>(xyz, B, N, M, start, start_dev, idx, idx_stride, md, md_stride, s);
    FFPS_WG_CASE(64, 4)
    FFPS_WG_CASE(256, 2)
    FFPS_WG_CASE(256, 4)
    FFPS_WG_CASE(256, 8)
    FFPS_WG_CASE(256, 16)
    FFPS_WG_CASE(1024, 8)
    FFPS_WG_CASE(1024, 16)
    FFPS_WG_CASE(1024, 24)
#undef FFPS_WG_CASE
    return hipErrorInvalidValue;
}

}  // namespace ffps
