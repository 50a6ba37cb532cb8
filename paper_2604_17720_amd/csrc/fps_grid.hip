// k_fps_grid: exact FPS (Sec. 3.1, Eq. 1) of ONE cloud spread over all CUs,
// points resident in registers.
//
// Each of G co-resident workgroups keeps every G-th point of the cloud (point i
// belongs to workgroup i mod G) and its running minimum distance in registers
// for the whole call.  The strided assignment spreads any run of consecutive
// indices over all workgroups, so an input that is already in farthest-point
// order (a layer of a stage chain) yields as many picks per round as any other.
// A workgroup is one COMMUNICATION wave (wave 0) plus NWK = 7 WORKER waves that
// own the points: eight waves, two per SIMD (waves i and i+4 share one).
//
// Workgroups meet once per ROUND (fps_exchange.h), and a round can deliver many
// picks.  The workers apply the picks of a round to their points, all of which
// are in LDS by then, reduce their slice to its three best points and an upper
// bound on every other point (the fourth-best value), and help the communication
// wave with the pairwise work of the replay.  The communication wave merges the
// worker waves' results into the workgroup's report, or, when workgroups x
// worker waves fit the exchange area, passes every wave's result on as a report
// of its own (more reporting units, more picks per round), exchanges reports
// with the other workgroups and settles the picks of the round.  The picks are
// exactly those of the one-pick-per-pass loop.
//
// With `overlap` (clouds spread over whole workgroups) the communication wave
// does not wait for the workers' report: the workers first update the three
// points of their last report with the new picks, which is quick, and the
// communication wave builds the next round on those while the workers apply the
// picks to everything else and make their next report.  Five workgroup barriers
// per round then, four without.
//
// Exit: every wait is bounded or ends when the communication wave says so; a
// workgroup that gives up sets the status word and leaves, and the others then
// run into their own bound.
#include "fps_exchange.h"

namespace ffps {

namespace {

// Candidates a reporting unit contributes to a round.  With two a round is
// cheaper (smaller records, fewer candidates to count and compact) but delivers
// about 40 % fewer picks.
constexpr int kT = 3;

struct WaveTop {  // a worker wave's kT best points and the bound on its others
    TopK<kT> t;
    float x[kT], y[kT], z[kT];
};

struct GridArgs {  // pointers are those of the first cloud of the launch
    const float *xyz;
    int N, M, start;
    const int *start_dev;  // per-cloud start indices overriding `start`, or null
    int wg_per_cloud;  // the grid holds (clouds of this launch) x wg_per_cloud workgroups
    int wave_units;    // 1: every worker wave reports on its own; 0: the workgroup reports as one
    int overlap;       // 1: a round is built while the picks of the one before are applied; 0: after
    int32_t *idx_out;
    long idx_stride;   // elements between the outputs of consecutive clouds
    float *md_out;
    long md_stride;
    char *exchange;    // per cloud: two buffers of buf_bytes(kT)
    int *status;
    int max_picks;
    int spin_limit;    // polls a workgroup makes for the records of a round before it gives up
};

// Number of waves a workgroup with NWK worker waves launches: wave 0
// communicates, the others work.
__host__ __device__ constexpr int grid_waves(int nwk) { return nwk + 1; }

template <int NWK, int P>
__global__ __launch_bounds__(kWave *grid_waves(NWK)) void k_fps_grid(GridArgs a_in) {
    static_assert(NWK == 3 || NWK == 7, "four or eight waves in all");
    // reports of the worker waves, two buffers: the communication wave reads one while the
    // workers fill the other
    __shared__ WaveTop wtop[2][NWK];
    // the values of a report's kT candidates after the picks of the round that followed it
    __shared__ uint32_t wupd[NWK][kT];
    __shared__ RoundLds L;
    // {batch id, picks emitted in total once that batch is complete}, one 8-byte word
    __shared__ __attribute__((aligned(8))) uint32_t fin[2];
    __shared__ int s_abort;

    // A launch may carry several clouds: each gets a cluster of wg_per_cloud
    // consecutive workgroups with its own exchange area; clusters never interact.
    GridArgs a = a_in;
    const int G = a.wg_per_cloud;
    const int cloud = blockIdx.x / G;
    const int w = blockIdx.x - cloud * G;
    a.xyz += (size_t)cloud * a.N * 3;
    a.idx_out += cloud * a.idx_stride;
    if (a.md_out) a.md_out += cloud * a.md_stride;
    a.exchange += (size_t)cloud * 2 * buf_bytes(kT);
    if (a.start_dev) a.start = a.start_dev[cloud];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;

    // One pick handed from the communication wave to the workers is a single
    // 16-byte LDS word {x, y, z, seq}: written and read by one instruction each, so
    // a reader that sees the expected seq also sees its coordinates.
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
            s_abort = 0;
            if (w == 0) {
                a.idx_out[0] = a.start;
                if (a.md_out) a.md_out[0] = __builtin_inff();
            }
        }
    }
    __syncthreads();

    if (wave != 0) {
        // =============================== worker ===============================
        const int wk = wave - 1;  // 0 .. NWK-1
        constexpr int NTW = NWK * kWave;
        const int t = wk * kWave + lane;      // worker thread number
        // element j of this lane is point (j * NTW + t) * G + w: ascending in j
        auto index_of = [&](int j) { return (uint32_t)((j * NTW + t) * G + w); };
        float x[P], y[P], z[P], m[P];
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const uint32_t i = index_of(j);
            const bool ok = i < (uint32_t)a.N;
            x[j] = ok ? a.xyz[3 * (size_t)i + 0] : 0.f;
            y[j] = ok ? a.xyz[3 * (size_t)i + 1] : 0.f;
            z[j] = ok ? a.xyz[3 * (size_t)i + 2] : 0.f;
            // padding: value 0 and an index beyond every real one, never preferred
            m[j] = ok ? __builtin_inff() : 0.f;
        }
        int applied = 0;  // picks applied so far
        int buf = 1;      // buffer that holds this wave's last report
        bool first = true;
        for (;;) {
            // {round, picks so far}: the picks of the last round are all in L.pk by now
            const u32x2 f = lds_read8(fin_off);
            const int upto = __builtin_amdgcn_readfirstlane((int)f.y);
            if (s_abort || upto >= a.M) break;  // the picks of the last round need not be applied
            if (upto > applied) {
            if (!first && a.overlap) {
                // ---- 1z. first of all, what those picks do to the kT points of this wave's
                //      last report (a few picks per lane), for the communication wave, which
                //      builds the next round on them while the rest of this wave's points
                //      follow ----
                const WaveTop &o = wtop[buf][wk];
                float qx[kT], qy[kT], qz[kT];
                uint32_t qv[kT];
#pragma unroll
                for (int r = 0; r < kT; ++r) {
                    qx[r] = o.x[r]; qy[r] = o.y[r]; qz[r] = o.z[r];
                    qv[r] = lane == 0 ? o.t.v[r] : 0xffffffffu;
                }
                for (int c = lane; c < upto - applied; c += kWave) {
                    const u32x4 pk = L.pk[c];
#pragma unroll
                    for (int r = 0; r < kT; ++r)
                        qv[r] = umin(qv[r], f2u(sqdist(qx[r], qy[r], qz[r], u2f(pk.x), u2f(pk.y), u2f(pk.z))));
                }
#pragma unroll
                for (int r = 0; r < kT; ++r) qv[r] = wave_min_u32(qv[r]);
                if (lane == 0) {
#pragma unroll
                    for (int r = 0; r < kT; ++r) wupd[wk][r] = qv[r];
                }
                team_barrier();  // the communication wave waits here for all worker waves' updates
            }
            // ---- 1a. the picks of the round (first the seed point).  Eight slots per
            //      step; the slots behind the last pick of the round hold picks of
            //      earlier rounds (or the seed point), which every value reflects
            //      already, so applying those again changes nothing.  Meanwhile the
            //      communication wave is already at work on the next round: it brings
            //      this wave's previous report up to date itself. ----
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
            // ---- 1b. the lane's kT + 1 largest values (element numbers for the first kT) ----
            float top[kT + 1];
            int tj[kT];
            top[0] = m[0];
#pragma unroll
            for (int r = 1; r <= kT; ++r) top[r] = 0.f;
#pragma unroll
            for (int r = 0; r < kT; ++r) tj[r] = 0;
#pragma unroll
            for (int j = 1; j < P; ++j) {
                const float v = m[j];
                bool g[kT + 1];  // strict: the earlier (lower) j keeps a tie
#pragma unroll
                for (int r = 0; r <= kT; ++r) g[r] = v > top[r];
#pragma unroll
                for (int r = kT; r >= 1; --r) {
                    top[r] = fmaxf(top[r], fminf(v, top[r - 1]));
                    if (r < kT) tj[r] = g[r - 1] ? tj[r - 1] : (g[r] ? j : tj[r]);
                }
                tj[0] = g[0] ? j : tj[0];
                top[0] = fmaxf(top[0], v);
            }
            // ---- 1c. the wave's kT best + bound (equal values: lowest index first) ----
            TopK<kT> mine;
#pragma unroll
            for (int r = 0; r <= kT; ++r) mine.v[r] = f2u(top[r]);
#pragma unroll
            for (int r = 0; r < kT; ++r) mine.i[r] = index_of(tj[r]);
            int src[kT], ent[kT];
            const TopK<kT> wt = merge_topk<kT>(mine, true, lane, [](uint32_t v) { return wave_max_u32(v); },
                                               [](uint32_t v) { return wave_min_u32(v); }, src, ent);
            float wx[kT], wy[kT], wz[kT];
#pragma unroll
            for (int r = 0; r < kT; ++r) {
                int ej = tj[0];  // element number of this lane's ent[r]-th entry
#pragma unroll
                for (int e = 1; e < kT; ++e) ej = ent[r] == e ? tj[e] : ej;
                pick_xyz<P>(x, y, z, readlane_i(ej, src[r]), src[r], wx[r], wy[r], wz[r]);
            }
            buf = a.overlap ? buf ^ 1 : 0;
            if (lane == 0) {
                WaveTop &o = wtop[buf][wk];
                o.t = wt;
#pragma unroll
                for (int r = 0; r < kT; ++r) {
                    o.x[r] = wx[r]; o.y[r] = wy[r]; o.z[r] = wz[r];
                }
            }
            }  // picks applied, report made
            if (first || !a.overlap) {
                // the first report (without overlap: every report) is in place before the
                // communication wave reads it
                __syncthreads();
                first = false;
            }
            // ---- 1d. help with the replay of the round ----
            team_barrier();  // the communication wave has the candidates in place, every report is made
            team_matrix(L, lane, wave, NWK + 1);
            team_barrier();  // masks complete
            team_barrier();  // picks of the round in place
        }
        return;
    }

    // ========================== communication wave ==========================
    // it shares its SIMD with worker waves and sets the pace: it goes first
    __builtin_amdgcn_s_setprio(3);
    int npicked = 1;
    uint32_t round = 0;
    RoundProf *prof = nullptr;
#ifdef FFPS_PROFILE
    RoundProf prof_store = {};
    if (w == 0 && cloud == 0) prof = &prof_store;
    prof_store.last = wall_clock64();
    const uint64_t prof_w0 = prof_store.last, prof_c0 = clock64();
#endif
    // The rounds overlap.  When a round's picks are in L.pk the workers first work out
    // what they do to the kT points of their own last report (buffer cur), which takes
    // a few picks per lane, and then apply them to all their points and make their next
    // report.  Meanwhile this wave builds the next round on the updated last reports:
    // merge, publish, gather, compaction.  The candidates' values are exact that way;
    // the bounds (each wave's fourth value) are one round old, which only makes them
    // larger than need be.  What such a report cannot promise is that the best point of
    // all is a candidate: a round in which no candidate is above the bounds makes no
    // pick then (replay_round, fresh = false), and the next one starts from reports
    // that reflect every pick.
    int cur = 0, pend = 0;
    if (a.M > 1 && a.overlap) __syncthreads();  // the workers' first report (the seed point applied) is in place
    const int cs = lane % NWK;  // the worker wave whose report this lane holds
    while (npicked < a.M) {
        ++round;
        FFPS_STAMP(prof, 0);
        if (!a.overlap) __syncthreads();  // the workers have applied every pick so far and made their reports
        // ---- 2a. the report of worker wave cs, brought up to date ----
        uint32_t cv[kT], ci[kT], cbound;
        float cx[kT], cy[kT], cz[kT];
        {
            const WaveTop o = wtop[cur][cs];
#pragma unroll
            for (int r = 0; r < kT; ++r) {
                cv[r] = o.t.v[r]; ci[r] = o.t.i[r];
                cx[r] = o.x[r]; cy[r] = o.y[r]; cz[r] = o.z[r];
            }
            cbound = o.t.v[kT];
        }
        if (pend > 0) {
            // the workers work out first what the pending picks do to these candidates
            team_barrier();
#pragma unroll
            for (int r = 0; r < kT; ++r) cv[r] = wupd[cs][r];
        }
        FFPS_STAMP(prof, 1);
        RoundInput<kT> in;
        RoundResult res;
        const int cap = __builtin_amdgcn_readfirstlane(min(a.max_picks, a.M - npicked));
        const bool fresh = pend == 0;
        if (a.wave_units) {
            // ---- 2a'. every worker wave is a unit of its own: lane s reports wave s ----
#pragma unroll
            for (int r = 0; r < kT; ++r) {
                in.v[r] = cv[r]; in.i[r] = ci[r];
                in.x[r] = cx[r]; in.y[r] = cy[r]; in.z[r] = cz[r];
            }
            in.bound = cbound;
            // ---- 2b/2c/3. publish, gather, replay (picks go to L.pk as they are found) ----
            res = exchange_round<kT>(L, a.exchange, G * NWK, w * NWK, NWK, lane, round, in, npicked,
                                           cap, a.status, prof, NWK + 1, 0, a.spin_limit, fresh);
        } else {
            // ---- 2a'. the workgroup's kT best + bound from the worker waves'.  The values
            //      have changed, so each wave's three go back into order first (value
            //      descending, index ascending). ----
            static_assert(kT == 3, "a sorting network for three");
            auto exchange = [&](int p, int q) {
                const bool sw = cv[q] > cv[p] || (cv[q] == cv[p] && ci[q] < ci[p]);
                const uint32_t tv = cv[p], ti = ci[p];
                const float tx = cx[p], ty = cy[p], tz = cz[p];
                cv[p] = sw ? cv[q] : tv; ci[p] = sw ? ci[q] : ti;
                cx[p] = sw ? cx[q] : tx; cy[p] = sw ? cy[q] : ty; cz[p] = sw ? cz[q] : tz;
                cv[q] = sw ? tv : cv[q]; ci[q] = sw ? ti : ci[q];
                cx[q] = sw ? tx : cx[q]; cy[q] = sw ? ty : cy[q]; cz[q] = sw ? tz : cz[q];
            };
            exchange(0, 1); exchange(1, 2); exchange(0, 1);
            const bool act = lane < NWK;
            int src[kT], ent[kT];
            TopK<kT> own;
#pragma unroll
            for (int r = 0; r < kT; ++r) {
                own.v[r] = cv[r]; own.i[r] = ci[r];
            }
            own.v[kT] = cbound;
            const TopK<kT> g3 = merge_topk<kT>(own, act, lane,
                                               [](uint32_t v) { return row_max_uniform(v); },
                                               [](uint32_t v) { return row_min_uniform(v); }, src, ent);
#pragma unroll
            for (int r = 0; r < kT; ++r) {
                in.v[r] = g3.v[r]; in.i[r] = g3.i[r];
                // entry r is wave src[r]'s ent[r]-th
                const float ex = ent[r] == 0 ? cx[0] : ent[r] == 1 ? cx[1] : cx[2];
                const float ey = ent[r] == 0 ? cy[0] : ent[r] == 1 ? cy[1] : cy[2];
                const float ez = ent[r] == 0 ? cz[0] : ent[r] == 1 ? cz[1] : cz[2];
                in.x[r] = u2f((uint32_t)readlane_i((int)f2u(ex), src[r]));
                in.y[r] = u2f((uint32_t)readlane_i((int)f2u(ey), src[r]));
                in.z[r] = u2f((uint32_t)readlane_i((int)f2u(ez), src[r]));
            }
            // what is left of the lists, and every wave's own (older) bound, which a
            // wave whose candidates are not used up keeps behind them
            in.bound = umax(g3.v[kT], row_max_uniform(act ? cbound : 0u));
            // ---- 2b/2c/3. publish, gather, replay (picks go to L.pk as they are found) ----
            res = exchange_round<kT>(L, a.exchange, G, w, 1, lane, round, in, npicked, cap,
                                           a.status, prof, NWK + 1, 0, a.spin_limit, fresh);
        }
        const int cnt = res.cnt;
        if (cnt < 0) {
            // the workers wait for the ranking: let them through with nothing to do
            if (lane == 0) lds_write4(lds_offset(&L.team_total), 0u);
            team_barrier();
            team_barrier();
#ifdef FFPS_PROFILE
            if (prof && lane == 0)
        #endif
            if (lane == 0) {
                s_abort = 1;
                u32x2 f;
                f.x = round; f.y = 0u;
                lds_write8(fin_off, f);  // no new picks; the workers then see s_abort
            }
            team_barrier();
            return;
        }
        // release the workers first, then note the picks (workgroup 0 only)
        if (lane == 0) {
            u32x2 f;
            f.x = round; f.y = (uint32_t)(npicked + cnt);
            lds_write8(fin_off, f);
        }
        team_barrier();  // the workers wait here for the picks
        if (res.stuck && lane == 0) note_inconsistent(a.status, (int)round);
        if (w == 0) record_picks(L, lane, res, npicked, a.idx_out, a.md_out);
        npicked += cnt;
        if (pend > 0) cur ^= 1;  // the workers have made a new report meanwhile
        pend = a.overlap ? cnt : 0;
        FFPS_STAMP(prof, 4);
    }
    if (w == 0 && lane == 0) {
        // exchange rounds this launch took (the largest count among its clouds)
        __hip_atomic_fetch_max(a.status + 1, (int)round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#ifdef FFPS_PROFILE
        if (cloud == 0) {
        for (int i = 0; i < 8; ++i) a.status[8 + i] = (int)prof_store.acc[i];
        for (int i = 0; i < 4; ++i) a.status[20 + i] = (int)prof_store.loop[i];
        for (int i = 0; i < 4; ++i) a.status[24 + i] = (int)prof_store.sub[i];
        for (int i = 0; i < 4; ++i) a.status[28 + i] = (int)prof_store.ev[i];
        for (int i = 0; i < 6; ++i) a.status[32 + i] = (int)prof_store.ord[i];
        a.status[16] = (int)(wall_clock64() - prof_w0);       // 10 ns units
        a.status[17] = (int)((clock64() - prof_c0) >> 4);     // shader cycles / 16
        }
#endif
    }
}

template <int NWK, int P>
hipError_t launch_t(GridArgs &a, int num_wg, hipStream_t s) {
    void *params[] = {&a};
    return hipLaunchCooperativeKernel((const void *)k_fps_grid<NWK, P>, dim3(num_wg),
                                      dim3(kWave * grid_waves(NWK)), params, 0, s);
}

// Kernel shapes (worker waves, points per worker lane), ordered by capacity; a
// workgroup's slice runs on the first shape that holds it.  Eight waves per
// workgroup: two per SIMD issue plain fp32 instructions at nearly twice the rate
// of one, all eight share the pairwise work of a round, and with 256 registers
// per lane neither the worker waves (four registers per point) nor the
// communication wave spill.
#define FFPS_GRID_SHAPES(X)                                                               \
    X(7, 1) X(7, 2) X(7, 3) X(7, 4) X(7, 5) X(7, 6) X(7, 8) X(7, 10) X(7, 12) X(7, 16) X(7, 20) \
    X(7, 24) X(7, 28)

constexpr int kMaxPointsPerWG = 12 * kWave * 16;  // 12288 <= 7 * 64 * 28

// Worker waves of the shape that holds per_wg points (0 if none does).
int shape_waves(int per_wg) {
#define X(NWK, P) \
    if (per_wg <= (NWK) * kWave * (P)) return NWK;
    FFPS_GRID_SHAPES(X)
#undef X
    return 0;
}

// Reporting units of a cloud on g workgroups: every worker wave when that many
// records fit the exchange area, else one per workgroup.
int units_of(int N, int g) {
    const int nwk = shape_waves((N + g - 1) / g);
    return nwk > 0 && g * nwk <= kMaxUnits ? g * nwk : g;
}

}  // namespace

static_assert(kExchangeBytesPerCloud == 2 * buf_bytes(kT), "exchange area as the host side sizes it");
size_t grid_exchange_bytes_per_cloud() { return 2 * buf_bytes(kT); }  // the streaming kernel reports two as well

long grid_capacity(int num_cu) {
    int G = num_cu < kMaxGridWG ? num_cu : kMaxGridWG;
    return (long)G * kMaxPointsPerWG;
}

GridPlan plan_fps_grid(int B, int N, int num_cu) {
    const int maxG = num_cu < kMaxGridWG ? num_cu : kMaxGridWG;
    // at least 128 points per workgroup before another CU is worth a record ...
    int want = (N + 127) / 128;
    if (want > maxG) want = maxG;
    // ... but rather all clouds in one launch than few clouds on many workgroups
    int share = maxG / (B < maxG ? B : maxG);
    if (share < 1) share = 1;
    int g = want < share ? want : share;
    const int need = (N + kMaxPointsPerWG - 1) / kMaxPointsPerWG;  // registers must hold the cloud
    if (g < need) g = need;
    // The picks a round delivers grow with the number of reporting units, and
    // fewer workgroups whose waves report one by one can give more units than
    // many workgroups that report as a whole: take the count with the most units.
    int best = g, best_units = units_of(N, g);
    for (int c = g - 1; c >= need && c >= 1; --c) {
        const int u = units_of(N, c);
        if (u > best_units) {
            best = c;
            best_units = u;
        }
    }
    GridPlan p;
    p.units_per_cloud = best_units;
    p.wg_per_cloud = best;
    p.clouds_per_launch = maxG / best < 1 ? 1 : maxG / best;
    if (p.clouds_per_launch > B) p.clouds_per_launch = B;
    return p;
}

hipError_t launch_fps_grid(const float *xyz, int clouds, int N, int M, int start,
                           const int *start_dev, int32_t *idx, long idx_stride, float *md,
                           long md_stride, void *exchange, int *status, int wg_per_cloud,
                           int max_picks, int spin_limit, hipStream_t s) {
    const int G = wg_per_cloud;
    GridArgs a;
    a.xyz = xyz; a.N = N; a.M = M; a.start = start; a.start_dev = start_dev;
    a.wg_per_cloud = G;
    a.idx_out = idx; a.idx_stride = idx_stride;
    a.md_out = md; a.md_stride = md_stride;
    a.exchange = (char *)exchange; a.status = status;
    a.max_picks = max_picks < 1 ? 1 : (max_picks > kMaxPicksPerRound ? kMaxPicksPerRound : max_picks);
    a.spin_limit = spin_limit < 0 ? kSpinLimit : spin_limit;
    const int per_wg = (N + G - 1) / G;  // most points any workgroup holds
    const int num_wg = clouds * G;
    a.wave_units = units_of(N, G) > G ? 1 : 0;
    // Rounds of small clouds (every wave a unit) deliver few picks, and applying them is
    // short work: nothing to hide a round's exchange behind, and reports that are one
    // round old cost picks.  Those launches take one round after the other.
    a.overlap = a.wave_units ? 0 : 1;
#define X(NWK, P) \
    if (per_wg <= (NWK) * kWave * (P)) return launch_t<NWK, P>(a, num_wg, s);
    FFPS_GRID_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace ffps
