// k_fps_stream: exact FPS (Sec. 3.1, Eq. 1) of ONE cloud spread over all CUs,
// points and running minimum distances streamed from HBM.
//
// For clouds that do not fit in registers.  G co-resident workgroups own
// contiguous slices.  Per ROUND (fps_exchange.h) every workgroup makes ONE pass
// over its slice: each point's coordinates (12 B) and minimum distance (4 B) are
// read, all picks of the previous round are applied, the minimum distance is
// written back (4 B), and the pass keeps the slice's two best points and the
// bound on the rest.  Since a round delivers several picks, the 20 bytes per
// point are paid once per round, not once per pick.
//
// Lanes take groups of four consecutive points (three 16-byte loads of
// coordinates, one of distances); slices stay contiguous so that every load of
// a wave is coalesced.
#include "fps_exchange.h"

namespace ffps {

namespace {

constexpr int kStreamThreads = 1024;

struct StreamArgs {
    const float *xyz;
    float *mind;  // [N] running minimum squared distance (workspace; written before read)
    int N, M, start;
    const int *start_dev;  // start index overriding `start`, or null
    int chunk;  // points per workgroup, a multiple of 4
    int32_t *idx_out;
    float *md_out;
    char *exchange;
    int *status;
    int max_picks;
    int aligned16;  // xyz is 16-byte aligned
};

__global__ __launch_bounds__(kStreamThreads) void k_fps_stream(StreamArgs a) {
    if (a.start_dev) a.start = a.start_dev[0];
    constexpr int NT = kStreamThreads, NW = NT / kWave;
    __shared__ RoundLds L;
    __shared__ TopK<2> wtop[NW];
    __shared__ int s_cnt, s_abort;

    const int G = gridDim.x;
    const int w = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int lo = w * a.chunk;
    const int hi = min(a.N, lo + a.chunk);
    const uint32_t pk_off = lds_offset(L.pk);

    if (tid < kWave) {
        // every pick slot starts as the seed point: the replay may read slots behind
        // the picks of a round, and a point picked earlier changes nothing
        u32x4 s;
        s.x = f2u(a.xyz[3 * (size_t)a.start + 0]);
        s.y = f2u(a.xyz[3 * (size_t)a.start + 1]);
        s.z = f2u(a.xyz[3 * (size_t)a.start + 2]);
        for (int c = tid; c < kMaxPicksPerRound + 8; c += kWave) {
            s.w = c == 0 ? 0u : 0xffffffffu;
            lds_write16(pk_off + c * 16, s);
        }
    }
    if (tid == 0) {
        s_cnt = 1;
        s_abort = 0;
        if (w == 0) {
            a.idx_out[0] = a.start;
            if (a.md_out) a.md_out[0] = __builtin_inff();
        }
    }
    __syncthreads();

    int npicked = 1;
    uint32_t round = 0;
    while (npicked < a.M) {
        ++round;
        const int cnt_prev = s_cnt;
        const bool first_pass = round == 1;  // minimum distances start at +inf, nothing to read
        // ---- 1. one pass over the slice ----
        // running top three of this lane; -1 sorts below every distance
        float t1 = -1.f, t2 = -1.f, t3 = -1.f;
        uint32_t j1 = 0xffffffffu, j2 = 0xffffffffu;
        auto track = [&](float v, uint32_t i) {
            const bool g1 = v > t1, g2 = v > t2;  // strict: this lane visits indices in ascending order
            t3 = fmaxf(t3, fminf(v, t2));
            j2 = g1 ? j1 : (g2 ? i : j2);
            t2 = fmaxf(t2, fminf(v, t1));
            j1 = g1 ? i : j1;
            t1 = fmaxf(t1, v);
        };
        // Two groups of four points per step: all eight 16-byte loads are issued
        // before either group is worked on, which doubles the bytes in flight.
        struct Group {
            float px[4], py[4], pz[4], pm[4];
        };
        auto load = [&](Group &gp, int g) {
            const bool full = g + 4 <= hi;
            if (full && a.aligned16) {
                const float4 *src = reinterpret_cast<const float4 *>(a.xyz + 3 * (size_t)g);
                const float4 q0 = src[0], q1 = src[1], q2 = src[2];
                gp.px[0] = q0.x; gp.py[0] = q0.y; gp.pz[0] = q0.z;
                gp.px[1] = q0.w; gp.py[1] = q1.x; gp.pz[1] = q1.y;
                gp.px[2] = q1.z; gp.py[2] = q1.w; gp.pz[2] = q2.x;
                gp.px[3] = q2.y; gp.py[3] = q2.z; gp.pz[3] = q2.w;
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool ok = g + k < hi;
                    gp.px[k] = ok ? a.xyz[3 * (size_t)(g + k) + 0] : 0.f;
                    gp.py[k] = ok ? a.xyz[3 * (size_t)(g + k) + 1] : 0.f;
                    gp.pz[k] = ok ? a.xyz[3 * (size_t)(g + k) + 2] : 0.f;
                }
            }
            if (first_pass) {
#pragma unroll
                for (int k = 0; k < 4; ++k) gp.pm[k] = __builtin_inff();
            } else if (full) {
                const float4 mm = *reinterpret_cast<const float4 *>(a.mind + g);
                gp.pm[0] = mm.x; gp.pm[1] = mm.y; gp.pm[2] = mm.z; gp.pm[3] = mm.w;
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) gp.pm[k] = g + k < hi ? a.mind[g + k] : 0.f;
            }
        };
        auto finish = [&](Group &gp, int g) {
            if (g + 4 <= hi) {
                *reinterpret_cast<float4 *>(a.mind + g) =
                    make_float4(gp.pm[0], gp.pm[1], gp.pm[2], gp.pm[3]);
#pragma unroll
                for (int k = 0; k < 4; ++k) track(gp.pm[k], (uint32_t)(g + k));
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (g + k < hi) {
                        a.mind[g + k] = gp.pm[k];
                        track(gp.pm[k], (uint32_t)(g + k));
                    }
            }
        };
        for (int g = lo + tid * 4; g < hi; g += 2 * NT * 4) {
            const int g2 = g + NT * 4;
            const bool two = g2 < hi;
            Group A, B;
            load(A, g);
            if (two) load(B, g2);
            for (int q = 0; q < cnt_prev; ++q) {
                const u32x4 s = lds_read16(pk_off + q * 16);
                const float lx = u2f(s.x), ly = u2f(s.y), lz = u2f(s.z);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    A.pm[k] = fminf(A.pm[k], sqdist(A.px[k], A.py[k], A.pz[k], lx, ly, lz));
                    if (two) B.pm[k] = fminf(B.pm[k], sqdist(B.px[k], B.py[k], B.pz[k], lx, ly, lz));
                }
            }
            finish(A, g);  // group A's indices precede group B's: ascending order is kept
            if (two) finish(B, g2);
        }
        // ---- 1b. wave top two + bound (value ties broken on the index) ----
        TopK<2> mine;
        mine.v[0] = f2u(fmaxf(t1, 0.f)); mine.v[1] = f2u(fmaxf(t2, 0.f)); mine.v[2] = f2u(fmaxf(t3, 0.f));
        mine.i[0] = j1; mine.i[1] = j2;
        int src[2], ent[2];
        const TopK<2> wt = merge_topk<2>(mine, true, lane, [](uint32_t v) { return wave_max_u32(v); },
                                         [](uint32_t v) { return wave_min_u32(v); }, src, ent);
        if (lane == 0) wtop[wave] = wt;
        __syncthreads();  // wave tops visible; every wave is done with the picks in L.pk

        if (wave == 0) {
            // ---- 2a. workgroup top two + bound ----
            const bool act = lane < NW;
            const TopK<2> g3 = merge_topk<2>(wtop[act ? lane : 0], act, lane,
                                             [](uint32_t v) { return row_max_uniform(v); },
                                             [](uint32_t v) { return row_min_uniform(v); }, src, ent);
            // an index that does not exist (slice of one point) has value 0
            RoundInput<2> in;
            in.bound = g3.v[2];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const uint32_t ir = g3.i[r];
                const bool e = ir < (uint32_t)a.N;
                in.v[r] = g3.v[r];
                in.i[r] = e ? ir : kNoIndex;
                in.x[r] = e ? a.xyz[3 * (size_t)(e ? ir : 0) + 0] : 0.f;
                in.y[r] = e ? a.xyz[3 * (size_t)(e ? ir : 0) + 1] : 0.f;
                in.z[r] = e ? a.xyz[3 * (size_t)(e ? ir : 0) + 2] : 0.f;
            }
            const int cap = __builtin_amdgcn_readfirstlane(min(a.max_picks, a.M - npicked));
            const RoundResult res = exchange_round<2, 2>(L, a.exchange, G, w, 1, lane, round, in,
                                                            npicked, cap, a.status, nullptr, NW);
            if (res.cnt < 0) {
                // gave up before the replay: the other waves wait for it at two barriers
                if (lane == 0) lds_write4(lds_offset(&L.team_total), 0u);
                team_barrier();
                team_barrier();
            }
            if (lane == 0) {
                s_cnt = res.cnt < 0 ? 0 : res.cnt;
                if (res.cnt < 0) s_abort = 1;
            }
            if (res.cnt > 0 && res.stuck && lane == 0) note_inconsistent(a.status, (int)round);
            if (w == 0 && res.cnt > 0) record_picks(L, lane, res, npicked, a.idx_out, a.md_out);
        } else {
            // ---- 2b. help with the replay of the round ----
            team_barrier();  // wave 0 has the candidates in place
            team_matrix(L, lane, wave, NW);
            team_barrier();  // masks complete
        }
        team_barrier();  // picks of this round visible to all waves
        if (s_abort) return;
        npicked += s_cnt;
    }
    if (w == 0 && tid == 0)
        __hip_atomic_fetch_max(a.status + 1, (int)round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace

// A lane's position advances by 8192 points per step and a slice end is
// computed as slice begin + slice length, both in 32-bit integers.
int stream_capacity() { return 0x7fffffff - 2 * kStreamThreads * 4 - 4 * kMaxGridWG; }

int stream_workgroups(int N, int num_cu) {
    int maxG = num_cu < kMaxGridWG ? num_cu : kMaxGridWG;
    // a workgroup pass covers 4096 points per step; do not spread thinner than that
    int G = (N + 4095) / 4096;
    if (G > maxG) G = maxG;
    return G < 1 ? 1 : G;
}

hipError_t launch_fps_stream(const float *xyz, float *mind, int N, int M, int start,
                             const int *start_dev, int32_t *idx, float *md, void *exchange,
                             int *status, int num_cu, int max_picks, hipStream_t s) {
    const int G = stream_workgroups(N, num_cu);
    StreamArgs a;
    a.xyz = xyz; a.mind = mind; a.N = N; a.M = M; a.start = start; a.start_dev = start_dev;
    a.chunk = ((N + G - 1) / G + 3) / 4 * 4;
    a.idx_out = idx; a.md_out = md;
    a.exchange = (char *)exchange; a.status = status;
    a.max_picks = max_picks < 1 ? 1 : (max_picks > kMaxPicksPerRound ? kMaxPicksPerRound : max_picks);
    a.aligned16 = ((uintptr_t)xyz & 15) == 0;
    void *params[] = {&a};
    return hipLaunchCooperativeKernel((const void *)k_fps_stream, dim3(G), dim3(kStreamThreads),
                                      params, 0, s);
}

}  // namespace ffps
