// Exact FPS (Sec. 3.1, Eq. 1) with one workgroup per cloud: k_fps_wg takes one
// pick per pass over the points, k_fps_wgm many (further down).
//
// k_fps_wg: the whole cloud lives in registers for the duration of the call: thread t
// holds points [t*P, t*P+P) and their running minimum distances, so lane order,
// wave order and index order coincide and "lowest index wins a tie" becomes
// "lowest lane / lowest wave wins".  Per pick: P distance updates per lane, a
// per-lane argmax, a DPP max across the wave, one LDS exchange across waves
// (double-buffered, so a single s_barrier per pick).  Nothing is re-read from
// HBM after the initial load.
#include "fps_exchange.h"

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


// ---------------------------------------------------------------------------
// k_fps_wgm: one workgroup per cloud, MANY picks per pass over the points.
//
// The workgroup is one REPLAY wave (wave 0) plus seven worker waves that own the
// points (point i belongs to worker lane i mod NTW).  Per round every worker
// lane reports the two best of its own points and the value of its third best
// (one 16-byte LDS record); the replay wave takes the 2 * NTW reported points as
// candidates and, together with the worker waves, replays the greedy rule of
// Eq. 1 on them alone (fps_exchange.h) for as long as the best candidate stays
// strictly above every lane's third-best value, since no unreported point can
// then be the maximum.  The picks of a round go to the workers through LDS
// together.  A round delivers some tens of picks, so nothing is reduced over
// the whole workgroup per pick: the lanes' reports need no cross-lane step at
// all.
struct WgmArgs {
    const float *xyz;
    int N, M, start;
    const int *start_dev;
    int32_t *idx_out;
    long idx_stride;
    float *md_out;
    long md_stride;
    int max_picks;
    int *status;  // status[1] receives the largest number of rounds any cloud took
};

__host__ __device__ constexpr int wgm_waves(int nwk) { return nwk + 1; }

template <int NWK, int P>
__global__ __launch_bounds__(kWave *wgm_waves(NWK)) void k_fps_wgm(WgmArgs a) {
    static_assert(NWK == 7, "eight waves in all: two per SIMD");
    constexpr int NTW = NWK * kWave;  // worker lanes = reporting units
    constexpr int KR = NWK;           // records per lane of the replay wave
    constexpr int KC = 2 * KR;        // candidates per lane of the replay wave
    __shared__ float4 sxyz[NTW * P];  // coordinates by point index
    __shared__ u32x4 rec[NTW];        // {best value, second value, third value, j1 | j2 << 16}
    __shared__ RoundLds L;
    // {batch id, picks emitted in total once that batch is complete}, one 8-byte word
    __shared__ __attribute__((aligned(8))) uint32_t fin[2];

    const int cloud = blockIdx.x;
    a.xyz += (size_t)cloud * a.N * 3;
    a.idx_out += cloud * a.idx_stride;
    if (a.md_out) a.md_out += cloud * a.md_stride;
    if (a.start_dev) a.start = a.start_dev[cloud];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;

    const uint32_t pk_off = lds_offset(L.pk);
    const uint32_t fin_off = lds_offset(fin);

    if (wave == 0) {
        // batch 0 is the seed point alone; other slots start with an impossible seq
        u32x4 s;
        s.x = f2u(a.xyz[3 * (size_t)a.start + 0]);
        s.y = f2u(a.xyz[3 * (size_t)a.start + 1]);
        s.z = f2u(a.xyz[3 * (size_t)a.start + 2]);
        for (int c = lane; c < kMaxPicksPerRound + 8; c += kWave) {
            s.w = c == 0 ? 0u : 0xffffffffu;
            lds_write16(pk_off + c * 16, s);
        }
        if (lane == 0) {
            u32x2 f;
            f.x = 0u; f.y = 1u;
            lds_write8(fin_off, f);
            a.idx_out[0] = a.start;
            if (a.md_out) a.md_out[0] = __builtin_inff();
        }
    }

    if (wave != 0) {
        // =============================== worker ===============================
        const int wk = wave - 1;          // 0 .. NWK-1
        const int t = wk * kWave + lane;  // worker lane number
        // element j of this lane is point j * NTW + t: ascending in j
        float x[P], y[P], z[P], m[P];
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int i = j * NTW + t;
            const bool ok = i < a.N;
            x[j] = ok ? a.xyz[3 * (size_t)i + 0] : 0.f;
            y[j] = ok ? a.xyz[3 * (size_t)i + 1] : 0.f;
            z[j] = ok ? a.xyz[3 * (size_t)i + 2] : 0.f;
            // padding: value 0 and an index beyond every real one, never preferred
            m[j] = ok ? __builtin_inff() : 0.f;
            sxyz[i] = make_float4(x[j], y[j], z[j], 0.f);
        }
        __syncthreads();  // pick slots and coordinates in place
        int applied = 0;  // picks applied so far
        for (;;) {
            // ---- the picks of the round (first the seed point), which are all in place
            //      by now: {round, picks so far} says how many.  Eight slots per step;
            //      the slots behind the last pick of the round hold picks of earlier
            //      rounds (or the seed point), which every value reflects already. ----
            const u32x2 f = lds_read8(fin_off);
            const int upto = __builtin_amdgcn_readfirstlane((int)f.y);
            for (int c0 = 0; c0 < upto - applied; c0 += 8) {
                u32x4 sl[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) sl[e] = L.pk[c0 + e];
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float lx = u2f(sl[e].x), ly = u2f(sl[e].y), lz = u2f(sl[e].z);
                    const float kx = u2f(sl[e + 1].x), ky = u2f(sl[e + 1].y), kz = u2f(sl[e + 1].z);
#pragma unroll
                    for (int j = 0; j < P; ++j)
                        m[j] = min3_dist(m[j], sqdist(x[j], y[j], z[j], lx, ly, lz),
                                         sqdist(x[j], y[j], z[j], kx, ky, kz));
                }
            }
            applied = upto;
            if (applied >= a.M) break;
            // ---- the lane's top three values (element numbers for the first two) ----
            float a1 = m[0], a2 = 0.f, a3 = 0.f;
            int j1 = 0, j2 = 0;
#pragma unroll
            for (int j = 1; j < P; ++j) {
                float v = m[j];
                bool g1 = v > a1, g2 = v > a2;  // strict: the earlier (lower) j keeps a tie
                a3 = fmaxf(a3, fminf(v, a2));
                j2 = g1 ? j1 : (g2 ? j : j2);
                a2 = fmaxf(a2, fminf(v, a1));
                j1 = g1 ? j : j1;
                a1 = fmaxf(a1, v);
            }
            u32x4 r;
            r.x = f2u(a1); r.y = f2u(a2); r.z = f2u(a3);
            r.w = (uint32_t)j1 | ((uint32_t)j2 << 16);
            rec[t] = r;
            __syncthreads();  // records ready for the replay wave
            team_barrier();   // which has the candidates in place
            team_matrix(L, lane, wave, NWK + 1);
            team_barrier();   // masks complete
            team_barrier();   // picks of the round in place
        }
        return;
    }

    // ============================== replay wave ==============================
    team_barrier();  // coordinates and pick slots in place
    int npicked = 1;
    int round = 0;
    RoundProf *prof = nullptr;
#ifdef FFPS_PROFILE
    RoundProf prof_store = {};
    if (cloud == 0) prof = &prof_store;
    prof_store.last = wall_clock64();
    const uint64_t prof_w0 = prof_store.last, prof_c0 = clock64();
#endif
    while (npicked < a.M) {
        ++round;
        FFPS_STAMP(prof, 0);
        __syncthreads();  // workers have applied every pick so far and written rec
        FFPS_STAMP(prof, 1);
        uint32_t cv[KC], ci[KC], lb = 0u;
        float cx[KC], cy[KC], cz[KC];
#pragma unroll
        for (int q = 0; q < KR; ++q) {
            const int t = q * kWave + lane;
            const u32x4 r = rec[t];
            cv[2 * q] = r.x;
            cv[2 * q + 1] = r.y;
            lb = umax(lb, r.z);
            ci[2 * q] = (r.w & 0xffffu) * NTW + t;
            ci[2 * q + 1] = (r.w >> 16) * NTW + t;
        }
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            const float4 v = sxyz[ci[c]];
            cx[c] = v.x; cy[c] = v.y; cz[c] = v.z;
        }
        const int cap = __builtin_amdgcn_readfirstlane(min(a.max_picks, a.M - npicked));
        FFPS_STAMP(prof, 2);
        // a round of a cloud this small ends after a few tens of picks: about 64 live
        // candidates are enough, and the pairwise work grows with their square
        const RoundResult res = replay_round<KC>(L, lane, cv, ci, cx, cy, cz, lb, npicked, cap, prof,
                                                       NWK + 1, kSets, 64);
        // release the workers first, then note the picks
        if (lane == 0) {
            u32x2 f;
            f.x = (uint32_t)round; f.y = (uint32_t)(npicked + res.cnt);
            lds_write8(fin_off, f);
        }
        team_barrier();  // the workers wait here for the picks
        if (res.stuck && lane == 0) note_inconsistent(a.status, round);
        record_picks(L, lane, res, npicked, a.idx_out, a.md_out);
        npicked += res.cnt;
        FFPS_STAMP(prof, 4);
    }
    if (lane == 0) {
        __hip_atomic_fetch_max(a.status + 1, round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#ifdef FFPS_PROFILE
        if (cloud == 0) {
            for (int i = 0; i < 8; ++i) a.status[8 + i] = (int)prof_store.acc[i];
            for (int i = 0; i < 4; ++i) a.status[20 + i] = (int)prof_store.loop[i];
            for (int i = 0; i < 4; ++i) a.status[24 + i] = (int)prof_store.sub[i];
            a.status[16] = (int)(wall_clock64() - prof_w0);    // 10 ns units
            a.status[17] = (int)((clock64() - prof_c0) >> 4);  // shader cycles / 16
        }
#endif
    }
}

template <int NWK, int P>
static hipError_t launch_wgm_t(const WgmArgs &a, int B, hipStream_t s) {
    hipLaunchKernelGGL((k_fps_wgm<NWK, P>), dim3(B), dim3(kWave * wgm_waves(NWK)), 0, s, a);
    return hipGetLastError();
}

int wg_capacity() { return 1024 * 24; }

int wgm_capacity() { return 4608; }  // <= 7 * 64 * 11

int wg_units(int N) {
    if (N <= 64 * 4 || N > wgm_capacity()) return 0;
    return 7 * kWave;  // one reporting unit per worker lane
}

// Very small clouds (one wave holds them) and clouds beyond the multi-pick
// kernel's capacity use the one-pick kernel, the others the multi-pick kernel.
// Shapes are ordered by capacity; the first one that holds N is used.
hipError_t launch_fps_wg(const float *xyz, int B, int N, int M, int start, const int *start_dev,
                         int32_t *idx, long idx_stride, float *md, long md_stride, int max_picks,
                         int *status, hipStream_t s) {
#define FFPS_WG_CASE(NT, P) \
    if (N <= (NT) * (P))    \
        return launch_wg_t<NT, P>(xyz, B, N, M, start, start_dev, idx, idx_stride, md, md_stride, s);
    FFPS_WG_CASE(64, 4)
    if (N <= wgm_capacity()) {
        WgmArgs a;
        a.xyz = xyz; a.N = N; a.M = M; a.start = start; a.start_dev = start_dev;
        a.idx_out = idx; a.idx_stride = idx_stride;
        a.md_out = md; a.md_stride = md_stride;
        a.status = status;
        a.max_picks = max_picks < 1 ? kMaxPicksPerRound
                                    : (max_picks > kMaxPicksPerRound ? kMaxPicksPerRound : max_picks);
#define FFPS_WGM_CASE(NWK, P) \
    if (N <= (NWK) * kWave * (P)) return launch_wgm_t<NWK, P>(a, B, s);
        FFPS_WGM_CASE(7, 1)
        FFPS_WGM_CASE(7, 2)
        FFPS_WGM_CASE(7, 3)
        FFPS_WGM_CASE(7, 4)
        FFPS_WGM_CASE(7, 6)
        FFPS_WGM_CASE(7, 8)
        FFPS_WGM_CASE(7, 11)
#undef FFPS_WGM_CASE
    }
    FFPS_WG_CASE(1024, 8)
    FFPS_WG_CASE(1024, 16)
    FFPS_WG_CASE(1024, 24)
#undef FFPS_WG_CASE
    return hipErrorInvalidValue;
}

}  // namespace ffps
