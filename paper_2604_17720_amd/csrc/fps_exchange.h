// Cross-workgroup exchange and candidate replay shared by the multi-workgroup
// FPS kernels (register-resident and HBM-streaming).
//
// The points of a cloud are divided among U <= 256 reporting UNITS (a whole
// workgroup, or each worker wave of a workgroup).  Once per ROUND every unit
// contributes its two best points and an upper bound on all its other points
// (its third-best value).  One wave per workgroup publishes the records of its
// units as four 16-byte chunks each, every chunk closed by a checksum that also
// encodes the round, gathers the chunks of all U units with coalesced
// device-scope loads (the only cross-workgroup step: no counters, no fences, no
// separate barrier), and replays the greedy rule of Eq. 1 on the 2U published
// candidates: the best candidate is the next pick as long as its value is
// strictly above B = max of all bounds, because no unpublished point can then
// reach it; picking it lowers the other candidates' values by the same distance
// rule, and the replay continues until the test fails.  The first pick of a
// round never needs the test: the global best point (largest value, lowest
// index among equals) is the best of its own unit, hence published.
// Every workgroup replays the same arithmetic on the same records, so all agree
// on the picks without further communication.
//
// "Best" always means largest value, then lowest point index.  Points may be
// assigned to units in any way; candidates carry their indices, and equal
// values are detected and resolved on the index wherever they can occur.
#pragma once
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

constexpr int kMaxUnits = kMaxGridWG;     // reporting units of a cloud
constexpr int kRPL = kMaxUnits / kWave;   // unit records per lane of the gathering wave
constexpr int kSpinLimit = 1 << 19;
constexpr uint32_t kNoIndex = 0x7fffffffu;  // index of a candidate that does not exist

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Exchange area: two buffers (round parity); each holds one array of 256 slots
// x 16 bytes per chunk of a record.  A record of T candidates is, in chunks of
// three words plus a check word,
//   T = 2: {v0, v1, bound} {x0, y0, z0} {x1, y1, z1} {i0, i1, 0}
//   T = 3: {v0, v1, v2} {x0, y0, z0} {x1, y1, z1} {x2, y2, z2} {i0, i1, i2} {bound, 0, 0}.
// Unit u uses slot u, and lane L of a gathering wave reads slots L, L + 64,
// L + 128, L + 192: each 16-byte load per lane touches one contiguous KiB, and
// units with consecutive numbers, which hold consecutive point indices, land in
// different lanes.
__host__ __device__ constexpr int chunks_of(int T) { return T == 2 ? 4 : 6; }
constexpr size_t kChunkBytes = (size_t)kMaxUnits * 16;
__host__ __device__ constexpr size_t buf_bytes(int T) { return chunks_of(T) * kChunkBytes; }

// A chunk is valid for a round when its last word equals this value.  Memory
// cleared to zero never validates (the round term is non-zero for round >= 1),
// a chunk of round-2 in the same buffer does not validate, and a read that
// mixed old and new words fails the test and is simply polled again.
__device__ __forceinline__ uint32_t chunk_check(uint32_t a, uint32_t b, uint32_t c, uint32_t round,
                                                uint32_t which) {
    uint32_t m = a ^ ((b << 11) | (b >> 21)) ^ ((c << 22) | (c >> 10));
    return m ^ (round * 0x9E3779B1u + which * 0x85EBCA6Bu);
}
__device__ __forceinline__ bool chunk_ok(const u32x4 &c, uint32_t round, uint32_t which) {
    return c.w == chunk_check(c.x, c.y, c.z, round, which);
}

// Device-scope (all XCDs) 16-byte store and loads.  The compiler offers atomics
// up to 8 bytes only, so these are spelled out; sc1 is the device-scope cache
// policy the compiler itself uses for agent-scope atomics on this target.
__device__ __forceinline__ void store_chunk(void *p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}
// r[c][q] = 16 bytes at p + c * kChunkBytes + q * 1024, q < 4: all loads are
// issued before the single wait, so a poll costs one round trip.
__device__ __forceinline__ void load_chunks(const char *p, u32x4 (&r)[4][kRPL]) {
    static_assert(kRPL == 4, "four slots per lane");
    const char *pa = p, *pb = p + kChunkBytes, *pc = p + 2 * kChunkBytes, *pd = p + 3 * kChunkBytes;
    asm volatile(
        "global_load_dwordx4 %0, %16, off sc1\n\t"
        "global_load_dwordx4 %1, %16, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %16, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %16, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %4, %17, off sc1\n\t"
        "global_load_dwordx4 %5, %17, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %6, %17, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %7, %17, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %8, %18, off sc1\n\t"
        "global_load_dwordx4 %9, %18, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %10, %18, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %11, %18, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %12, %19, off sc1\n\t"
        "global_load_dwordx4 %13, %19, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %14, %19, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %15, %19, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(r[0][0]), "=&v"(r[0][1]), "=&v"(r[0][2]), "=&v"(r[0][3]), "=&v"(r[1][0]),
          "=&v"(r[1][1]), "=&v"(r[1][2]), "=&v"(r[1][3]), "=&v"(r[2][0]), "=&v"(r[2][1]),
          "=&v"(r[2][2]), "=&v"(r[2][3]), "=&v"(r[3][0]), "=&v"(r[3][1]), "=&v"(r[3][2]),
          "=&v"(r[3][3])
        : "v"(pa), "v"(pb), "v"(pc), "v"(pd)
        : "memory");
}
__device__ __forceinline__ void load_chunks(const char *p, u32x4 (&r)[6][kRPL]) {
    static_assert(kRPL == 4, "four slots per lane");
    const char *pa = p, *pb = p + kChunkBytes, *pc = p + 2 * kChunkBytes, *pd = p + 3 * kChunkBytes,
               *pe = p + 4 * kChunkBytes, *pf = p + 5 * kChunkBytes;
    asm volatile(
        "global_load_dwordx4 %0, %24, off sc1\n\t"
        "global_load_dwordx4 %1, %24, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %24, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %24, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %4, %25, off sc1\n\t"
        "global_load_dwordx4 %5, %25, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %6, %25, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %7, %25, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %8, %26, off sc1\n\t"
        "global_load_dwordx4 %9, %26, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %10, %26, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %11, %26, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %12, %27, off sc1\n\t"
        "global_load_dwordx4 %13, %27, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %14, %27, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %15, %27, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %16, %28, off sc1\n\t"
        "global_load_dwordx4 %17, %28, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %18, %28, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %19, %28, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %20, %29, off sc1\n\t"
        "global_load_dwordx4 %21, %29, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %22, %29, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %23, %29, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(r[0][0]), "=&v"(r[0][1]), "=&v"(r[0][2]), "=&v"(r[0][3]), "=&v"(r[1][0]),
          "=&v"(r[1][1]), "=&v"(r[1][2]), "=&v"(r[1][3]), "=&v"(r[2][0]), "=&v"(r[2][1]),
          "=&v"(r[2][2]), "=&v"(r[2][3]), "=&v"(r[3][0]), "=&v"(r[3][1]), "=&v"(r[3][2]),
          "=&v"(r[3][3]), "=&v"(r[4][0]), "=&v"(r[4][1]), "=&v"(r[4][2]), "=&v"(r[4][3]),
          "=&v"(r[5][0]), "=&v"(r[5][1]), "=&v"(r[5][2]), "=&v"(r[5][3])
        : "v"(pa), "v"(pb), "v"(pc), "v"(pd), "v"(pe), "v"(pf)
        : "memory");
}

// 16-byte LDS accesses as single instructions (a compiler-generated access of
// a 16-byte vector may be split, which would let a reader see half of a slot).
__device__ __forceinline__ uint32_t lds_offset(const void *p) { return (uint32_t)(uintptr_t)p; }
__device__ __forceinline__ void lds_write16(uint32_t off, u32x4 v) {
    asm volatile("ds_write_b128 %0, %1" : : "v"(off), "v"(v) : "memory");
}
__device__ __forceinline__ u32x4 lds_read16(uint32_t off) {
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(off) : "memory");
    return r;
}

// The same read in two halves, so that work can overlap its latency: r is not
// valid before lds_wait16(r) has run.
__device__ __forceinline__ void lds_issue16(u32x4 &r, uint32_t off) {
    asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(off) : "memory");
}
__device__ __forceinline__ void lds_wait16(u32x4 &r) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r) : : "memory");
}
// 8-byte LDS word written and read by one instruction each.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void lds_write8(uint32_t off, u32x2 v) {
    asm volatile("ds_write_b64 %0, %1" : : "v"(off), "v"(v) : "memory");
}
__device__ __forceinline__ u32x2 lds_read8(uint32_t off) {
    u32x2 r;
    asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(off) : "memory");
    return r;
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) { return ~wave_max_u32(~v); }
// Reductions over lanes 0..15 only (other lanes must pass the identity), wave-uniform.
__device__ __forceinline__ uint32_t row_max_uniform(uint32_t v) {
    return (uint32_t)readlane_i((int)row16_max_u32(v), 15);
}
__device__ __forceinline__ uint32_t row_min_uniform(uint32_t v) { return ~row_max_uniform(~v); }

// Lane that holds the best of the pairs (value v, index i): largest value, then
// lowest index.  `vmax` is the (uniform) largest value; the index reduction is
// only paid when several lanes hold it.
template <typename MINF>
__device__ __forceinline__ int best_lane(uint32_t v, uint32_t i, uint32_t vmax, MINF minf) {
    const uint64_t tied = __builtin_amdgcn_ballot_w64(v == vmax);
    if (__builtin_popcountll(tied) == 1) return (int)__builtin_ctzll(tied);
    const uint32_t imin = minf(v == vmax ? i : 0xffffffffu);
    return first_lane(v == vmax && i == imin);
}

// The K best (value, index) pairs of a set and the value that follows them,
// in (value descending, index ascending) order.
template <int K>
struct TopK {
    uint32_t v[K + 1];
    uint32_t i[K];
};

// Merge the TopK of the participating lanes (`act`) into one.  src[r] receives
// the lane that supplied entry r and ent[r] which of that lane's entries it
// was.  MAXF / MINF reduce over the participating lanes and return wave-uniform
// values.
template <int K, typename MAXF, typename MINF>
__device__ __forceinline__ TopK<K> merge_topk(const TopK<K> &t, bool act, int lane, MAXF maxf,
                                              MINF minf, int (&src)[K], int (&ent)[K]) {
    TopK<K> r;
    int cur = 0;  // entries of this lane already taken
    uint32_t hv = act ? t.v[0] : 0u, hi = act ? t.i[0] : 0xffffffffu;  // this lane's next entry
#pragma unroll
    for (int k = 0; k < K; ++k) {
        r.v[k] = maxf(hv);
        const int l = best_lane(hv, hi, r.v[k], minf);
        r.i[k] = (uint32_t)readlane_i((int)hi, l);
        src[k] = l;
        ent[k] = readlane_i(cur, l);
        if (lane == l) {
            ++cur;
            hv = t.v[K];
            hi = 0xffffffffu;
#pragma unroll
            for (int e = 1; e < K; ++e) {
                hv = cur == e ? t.v[e] : hv;
                hi = cur == e ? t.i[e] : hi;
            }
        }
    }
    r.v[K] = maxf(hv);
    return r;
}

// What a reporting unit contributes to a round: its T best points (any order)
// with their current values and indices, and the bound on its other points.
// A candidate that does not exist has value 0 and index kNoIndex.
template <int T>
struct RoundInput {
    uint32_t v[T], bound;
    float x[T], y[T], z[T];
    uint32_t i[T];
};

// LDS used by the wave that runs exchange_round.
struct RoundLds {
    __attribute__((aligned(16))) u32x4 pk[kMaxPicksPerRound];  // picks of the round: {x, y, z, seq}
    uint32_t pk_idx[kMaxPicksPerRound];  // index of each pick of the round
    uint32_t pk_val[kMaxPicksPerRound];  // and the value it was picked with
    uint32_t pk_key[kMaxPicksPerRound];  // winning key of each pick (packed replay loops)
    uint32_t tab_idx[2 * kWave];         // point index by candidate code (packed replay loops)
    __attribute__((aligned(16))) u32x4 cmp_a[2 * kWave];  // compacted live candidates: {value, index, x, y}
    float cmp_z[2 * kWave];                               // and z
};

// Counters of a profiling build (workgroup 0 only).
struct RoundProf {
    uint32_t acc[8];   // 100 MHz ticks per phase; [5], [6]: rounds on the packed paths; [7]: polls
    uint32_t loop[4];  // shader cycles and picks inside the two packed loops
    uint32_t sub[4];   // shader cycles of the replay set-up: bounds, counting, compaction
    uint64_t last;
};
#ifdef FFPS_PROFILE
#define FFPS_STAMP(P, i)                                 \
    do {                                                 \
        if ((P) != nullptr) {                            \
            uint64_t now_ = wall_clock64();              \
            (P)->acc[i] += (uint32_t)(now_ - (P)->last); \
            (P)->last = now_;                            \
        }                                                \
    } while (0)
#else
#define FFPS_STAMP(P, i) \
    do {                 \
    } while (0)
#endif

// Replay of the greedy rule of Eq. 1 on KC candidates per lane of ONE full wave
// (value bits cv, point index ci, coordinates cx/cy/cz; a candidate that does
// not exist has value 0 and index kNoIndex), given lb = the lane's share of the
// bounds on all points that are not candidates.  Pick number c of the round is
// written as {x, y, z, npicked + c} to L.pk[c] (16-byte LDS writes, in pick
// order, so other waves may consume them while the replay is still running),
// and what record_picks needs to name its index and value is left in L.
// Returns the number of picks (1 .. cap) and how they were noted.  The
// candidate arrays are used up.
struct RoundResult {
    int cnt;        // picks of the round, or -1 when the round failed
    bool by_key;    // picks noted as keys (L.pk_key, L.tab_idx) rather than in L.pk_idx / L.pk_val
    uint32_t T;     // threshold the keys are relative to
};

// Writes index (and value) of the picks of a round to the outputs; run by the
// wave that ran the round, in one workgroup of the cloud.
__device__ __forceinline__ void record_picks(const RoundLds &L, int lane, const RoundResult &r,
                                             int npicked, int32_t *idx_out, float *md_out);

template <int KC>
__device__ __forceinline__ RoundResult replay_round(RoundLds &L, int lane, uint32_t (&cv)[KC],
                                            uint32_t (&ci)[KC], float (&cx)[KC], float (&cy)[KC],
                                            float (&cz)[KC], uint32_t lb, int npicked, int cap,
                                            RoundProf *prof) {
    const uint32_t pk_off = lds_offset(L.pk);
#ifdef FFPS_PROFILE
    uint64_t sc = clock64();
#define FFPS_SUB(i)                              \
    do {                                         \
        if (prof) {                              \
            uint64_t n_ = clock64();             \
            prof->sub[i] += (uint32_t)(n_ - sc); \
            sc = n_;                             \
        }                                        \
    } while (0)
#else
#define FFPS_SUB(i) \
    do {            \
    } while (0)
#endif
    const uint32_t Bound = wave_max_u32(lb);
    // Hand pick number c of this round to the other waves (one 16-byte LDS write)
    // and note its index and value; `mine` holds in exactly one lane.
    auto emit = [&](bool mine, int c, uint32_t idx, uint32_t vbits, float ex, float ey, float ez) {
        if (mine) {
            u32x4 s;
            s.x = f2u(ex); s.y = f2u(ey); s.z = f2u(ez); s.w = (uint32_t)(npicked + c);
            lds_write16(pk_off + c * 16, s);
            L.pk_idx[c] = idx;
            L.pk_val[c] = vbits;
        }
    };
    auto lane_best = [&](uint32_t &bv, uint32_t &bi, int &bq) {
        bv = cv[0]; bi = ci[0]; bq = 0;
#pragma unroll
        for (int q = 1; q < KC; ++q) {
            const bool better = cv[q] > bv || (cv[q] == bv && ci[q] < bi);
            bv = better ? cv[q] : bv;
            bi = better ? ci[q] : bi;
            bq = better ? q : bq;
        }
    };
    auto wmin = [](uint32_t v) { return wave_min_u32(v); };
    uint32_t lv = cv[0];
#pragma unroll
    for (int q = 1; q < KC; ++q) lv = umax(lv, cv[q]);
    uint32_t V = wave_max_u32(lv);  // best candidate value
    int cnt = 0;
    int pl;
    float px, py, pz;
    // Only candidates above the bound can be picked after the first pick, and
    // when the best candidate is above it the first pick is one of them too:
    // compact them (in any order).  Any threshold T >= Bound serves as well (the
    // round then ends when the best candidate is no longer above T), so when more
    // than 128 candidates are above the bound T is raised to the largest
    // third-best candidate value of any lane, which leaves at most two per lane.
    uint32_t T = Bound;
    int total = 0, before = 0;
    FFPS_SUB(0);
    if (V > Bound && cap > 1) {
        // total = live candidates of the wave, before = those of lower lanes: the
        // per-lane count goes through one ballot per bit of it
        auto count_live = [&]() {
            uint32_t c = 0u;
#pragma unroll
            for (int q = 0; q < KC; ++q) c += cv[q] > T ? 1u : 0u;
            total = 0;
            before = 0;
#pragma unroll
            for (int bit = 0; (1 << bit) <= KC; ++bit) {
                const uint64_t mk = __builtin_amdgcn_ballot_w64((c >> bit) & 1u);
                total += __builtin_popcountll(mk) << bit;
                before += (int)__builtin_amdgcn_mbcnt_hi(
                              (uint32_t)(mk >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mk, 0u))
                          << bit;
            }
        };
        count_live();
        if (total > 2 * kWave) {
            uint32_t t1 = 0u, t2 = 0u, t3 = 0u;
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                const uint32_t v = cv[q];
                t3 = umax(t3, v < t2 ? v : t2);
                t2 = umax(t2, v < t1 ? v : t1);
                t1 = umax(t1, v);
            }
            T = umax(Bound, wave_max_u32(t3));
            count_live();
        }
    }
    // With at most 128 live candidates whose values lie within 2^24 ulps above
    // the threshold, value and position fit one 32-bit key
    //   key = (value_bits - threshold_bits) << 7 | position,
    // and a single wave-wide max yields the best value and a lane that holds it.
    // Values at or below the threshold saturate to 0 and end the round.  Whether other
    // candidates hold the same value costs one ballot; only then is the index
    // compared.
    const bool packed = total >= 1 && total <= 2 * kWave && V - T < (1u << 24);
    FFPS_SUB(1);
#ifdef FFPS_PROFILE
    if (prof && packed) prof->acc[total <= kWave ? 5 : 6] += 1;
#endif
    if (packed) {
        int pos = before;
#pragma unroll
        for (int q = 0; q < KC; ++q) {
            if (cv[q] > T) {
                u32x4 r;
                r.x = cv[q]; r.y = ci[q]; r.z = f2u(cx[q]); r.w = f2u(cy[q]);
                L.cmp_a[pos] = r;
                L.cmp_z[pos] = cz[q];
                ++pos;
            }
        }
        // the same wave wrote and now reads: LDS keeps its accesses in order
        FFPS_SUB(2);
        // In both loops below the key of a candidate is (value - T) << 7 | code,
        // where the 7-bit code names the candidate (its entry in L.tab_idx).  The
        // wave-wide max K names a best candidate.  Another lane holds the same value
        // exactly when its key differs from K in the code bits alone, i.e. when
        // (key ^ K) - 1 < 127: one compare and a branch on the lane mask.  Each pick
        // is handed over as {x, y, z, seq} by every lane at once (the data are
        // wave-uniform, so no lane has to be singled out), and K itself is noted:
        // it holds the pick's value and, through the code, its index.
        auto hand_over = [&](int c, uint32_t K) {
            u32x4 s;
            s.x = f2u(px); s.y = f2u(py); s.z = f2u(pz); s.w = (uint32_t)(npicked + c);
            lds_write16(pk_off + c * 16, s);
            L.pk_key[c] = K;
        };
        // The wave-wide max of the next keys with the hand-over of pick c written
        // between its steps: a DPP step must wait two issue slots for the result of
        // the one before, and the hand-over's independent moves and writes fill them.
        auto max_and_hand_over = [&](uint32_t key, int c, uint32_t Kc) {
            uint32_t v = key;
            u32x4 s;
            v = umax(v, dpp_or_zero<kDppRowShr1>(v));
            s.x = f2u(px); s.y = f2u(py);
            v = umax(v, dpp_or_zero<kDppRowShr2>(v));
            s.z = f2u(pz); s.w = (uint32_t)(npicked + c);
            v = umax(v, dpp_or_zero<kDppRowShr4>(v));
            const uint32_t at = pk_off + c * 16;
            v = umax(v, dpp_or_zero<kDppRowShr8>(v));
            lds_write16(at, s);
            v = umax(v, dpp_or_zero<kDppRowBcast15, 0xa>(v));
            L.pk_key[c] = Kc;
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
            return lo > hi ? lo : hi;
        };
        if (total <= kWave) {
            // one candidate per lane: lane L takes position L, code = L
            const bool h = lane < total;
            const u32x4 r0 = L.cmp_a[lane];
            uint32_t v0 = h ? r0.x : 0u;
            const uint32_t i0 = h ? r0.y : kNoIndex;
            const float x0 = h ? u2f(r0.z) : 0.f, y0 = h ? u2f(r0.w) : 0.f,
                        z0 = h ? L.cmp_z[lane] : 0.f;
            L.tab_idx[lane] = i0;
#ifdef FFPS_PROFILE
            const uint64_t lc0 = clock64();
#endif
            // the first pick of the round is never below the threshold
            uint32_t d = __builtin_elementwise_sub_sat(v0, T);
            uint32_t key = (d << 7) | (uint32_t)lane;
            uint32_t K = wave_max_u32(key);
            while (true) {
                pl = (int)(K & 127u);
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(((key ^ K) - 1u) < 127u) != 0, 0)) {
                    // several candidates share the best value: the lowest index wins
                    const uint32_t imin = wave_min_u32(d == (K >> 7) ? i0 : 0xffffffffu);
                    pl = first_lane(d == (K >> 7) && i0 == imin);
                    K = (K & ~127u) | (uint32_t)pl;
                }
                px = readlane_f(x0, pl);
                py = readlane_f(y0, pl);
                pz = readlane_f(z0, pl);
                const int c = cnt++;
                if (cnt >= cap) {
                    hand_over(c, K);
                    break;
                }
                v0 = f2u(min_dist(u2f(v0), sqdist(x0, y0, z0, px, py, pz)));
                d = __builtin_elementwise_sub_sat(v0, T);
                key = (d << 7) | (uint32_t)lane;
                K = max_and_hand_over(key, c, K);
                if ((K >> 7) == 0) break;
            }
#ifdef FFPS_PROFILE
            if (prof) {
                prof->loop[0] += (uint32_t)(clock64() - lc0);
                prof->loop[1] += cnt;
            }
#endif
        } else {
            // two candidates per lane (positions L and L + 64), the lower index first,
            // so that a lane whose two values tie puts forward the right one;
            // code = 2 L + (0 for the first, 1 for the second)
            const int p1 = lane + kWave;
            const bool h1 = p1 < total;  // position L itself is always taken here
            const u32x4 r0 = L.cmp_a[lane], r1 = L.cmp_a[p1];
            uint32_t v0 = r0.x, v1 = h1 ? r1.x : 0u;
            uint32_t i0 = r0.y, i1 = h1 ? r1.y : kNoIndex;
            float x0 = u2f(r0.z), y0 = u2f(r0.w), z0 = L.cmp_z[lane];
            float x1 = h1 ? u2f(r1.z) : 0.f, y1 = h1 ? u2f(r1.w) : 0.f, z1 = h1 ? L.cmp_z[p1] : 0.f;
            if (i1 < i0) {
                uint32_t tu;
                float tf;
                tu = v0; v0 = v1; v1 = tu;
                tu = i0; i0 = i1; i1 = tu;
                tf = x0; x0 = x1; x1 = tf;
                tf = y0; y0 = y1; y1 = tf;
                tf = z0; z0 = z1; z1 = tf;
            }
            L.tab_idx[2 * lane] = i0;
            L.tab_idx[2 * lane + 1] = i1;
#ifdef FFPS_PROFILE
            const uint64_t lc0 = clock64();
#endif
            uint32_t bd, key;
            float bx, by, bz;
            bool sec;
            auto keys_of_lane = [&]() {
                const uint32_t d0 = __builtin_elementwise_sub_sat(v0, T);
                const uint32_t d1 = __builtin_elementwise_sub_sat(v1, T);
                sec = d1 > d0;  // strict: equal values put the lower index forward
                bx = sec ? x1 : x0; by = sec ? y1 : y0; bz = sec ? z1 : z0;
                bd = sec ? d1 : d0;
                key = (bd << 7) | ((uint32_t)lane << 1) | (sec ? 1u : 0u);
            };
            keys_of_lane();
            uint32_t K = wave_max_u32(key);  // the first pick is never below the threshold
            while (true) {
                pl = (int)((K >> 1) & 63u);
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(((key ^ K) - 1u) < 127u) != 0, 0)) {
                    const uint32_t bidx = sec ? i1 : i0;
                    const uint32_t imin = wave_min_u32(bd == (K >> 7) ? bidx : 0xffffffffu);
                    pl = first_lane(bd == (K >> 7) && bidx == imin);
                    K = (K & ~127u) | (uint32_t)readlane_i((int)(key & 127u), pl);
                }
                px = readlane_f(bx, pl);
                py = readlane_f(by, pl);
                pz = readlane_f(bz, pl);
                const int c = cnt++;
                if (cnt >= cap) {
                    hand_over(c, K);
                    break;
                }
                v0 = f2u(min_dist(u2f(v0), sqdist(x0, y0, z0, px, py, pz)));
                v1 = f2u(min_dist(u2f(v1), sqdist(x1, y1, z1, px, py, pz)));
                keys_of_lane();
                K = max_and_hand_over(key, c, K);
                if ((K >> 7) == 0) break;
            }
#ifdef FFPS_PROFILE
            if (prof) {
                prof->loop[2] += (uint32_t)(clock64() - lc0);
                prof->loop[3] += cnt;
            }
#endif
        }
    } else {
        // a single pick (best candidate not above the bound, or cap 1), or values
        // spread too far above the threshold for the packed key: work on all
        // candidates of every lane
        while (true) {
            uint32_t bv, bi;
            int bq;
            lane_best(bv, bi, bq);
            V = wave_max_u32(bv);
            if (cnt > 0 && !(V > Bound)) break;
            pl = best_lane(bv, bi, V, wmin);
            const int pq = readlane_i(bq, pl);
            pick_xyz<KC>(cx, cy, cz, pq, pl, px, py, pz);
            emit(lane == pl, cnt, bi, V, px, py, pz);
            if (++cnt >= cap) break;
#pragma unroll
            for (int q = 0; q < KC; ++q)
                cv[q] = f2u(fminf(u2f(cv[q]), sqdist(cx[q], cy[q], cz[q], px, py, pz)));
        }
    }
    RoundResult res;
    res.cnt = cnt;
    res.by_key = packed;
    res.T = T;
    return res;
}

__device__ __forceinline__ void record_picks(const RoundLds &L, int lane, const RoundResult &r,
                                             int npicked, int32_t *idx_out, float *md_out) {
    for (int c = lane; c < r.cnt; c += kWave) {
        uint32_t idx, val;
        if (r.by_key) {
            // the key holds the pick's value above the threshold and the code of its candidate
            const uint32_t K = L.pk_key[c];
            idx = L.tab_idx[K & 127u];
            val = (K >> 7) + r.T;
        } else {
            idx = L.pk_idx[c];
            val = L.pk_val[c];
        }
        idx_out[npicked + c] = (int32_t)idx;
        if (md_out) md_out[npicked + c] = u2f(val);
    }
}

// One round, run by ONE full wave of a workgroup.  The cloud has U reporting
// units (a whole workgroup, or each of its worker waves); lanes 0 .. nsub-1 of
// this wave publish `in` as unit unit0 + lane.  The wave then gathers all U
// records, replays, writes each pick as {x, y, z, npicked + c} to L.pk[c]
// (16-byte LDS writes, in pick order, so other waves may consume them while
// the replay is still running).  Returns the picks of the round (1 .. cap; see
// record_picks), or a count of -1 after setting *status when another unit's
// record never arrived.
template <int T>
__device__ __forceinline__ RoundResult exchange_round(RoundLds &L, char *exchange, int U, int unit0,
                                                      int nsub, int lane, uint32_t round,
                                                      const RoundInput<T> &in, int npicked, int cap,
                                                      int *status, RoundProf *prof) {
    static_assert(T == 2 || T == 3, "two or three candidates per unit");
    constexpr int NCH = chunks_of(T);
    constexpr int KC = T * kRPL;  // candidates per lane before compaction
    // ---- publish ----
    char *buf = exchange + (size_t)(round & 1) * buf_bytes(T);
    if (lane < nsub) {
        uint32_t d[NCH][3] = {};
#pragma unroll
        for (int t = 0; t < T; ++t) {
            d[0][t] = in.v[t];
            d[1 + t][0] = f2u(in.x[t]); d[1 + t][1] = f2u(in.y[t]); d[1 + t][2] = f2u(in.z[t]);
            d[T + 1][t] = in.i[t];
        }
        if (T == 2) d[0][2] = in.bound; else d[NCH - 1][0] = in.bound;
        const size_t so = (size_t)(unit0 + lane) * 16;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            u32x4 ch;
            ch.x = d[c][0]; ch.y = d[c][1]; ch.z = d[c][2];
            ch.w = chunk_check(ch.x, ch.y, ch.z, round, (uint32_t)c);
            store_chunk(buf + c * kChunkBytes + so, ch);
        }
    }
    FFPS_STAMP(prof, 2);
    // ---- gather: lane L reads slots (= units) q*64+L ----
    u32x4 r[NCH][kRPL];
    bool gave_up = false;
    for (int spin = 0;; ++spin) {
        load_chunks(buf + (size_t)lane * 16, r);
        bool all = true;
#pragma unroll
        for (int q = 0; q < kRPL; ++q) {
            bool ok = true;
#pragma unroll
            for (int c = 0; c < NCH; ++c) ok = ok && chunk_ok(r[c][q], round, (uint32_t)c);
            all = all && (ok || q * kWave + lane >= U);
        }
#ifdef FFPS_PROFILE
        if (prof) ++prof->acc[7];
#endif
        if (__builtin_amdgcn_ballot_w64(!all) == 0) break;
        if (spin >= kSpinLimit) {
            gave_up = true;
            break;
        }
    }
    FFPS_STAMP(prof, 3);
    if (gave_up) {
        if (lane == 0) __hip_atomic_store(status, -5, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        RoundResult failed;
        failed.cnt = -1;
        failed.by_key = false;
        failed.T = 0u;
        return failed;
    }
    // candidate c = T q + t of this lane: unit q*64 + lane, its t-th entry
    uint32_t cv[KC], ci[KC], lb = 0u;
    float cx[KC], cy[KC], cz[KC];
#pragma unroll
    for (int q = 0; q < kRPL; ++q) {
        const bool present = q * kWave + lane < U;  // absent records: value 0, bound 0
        const uint32_t vals[3] = {r[0][q].x, r[0][q].y, r[0][q].z};
        const uint32_t idxs[3] = {r[T + 1][q].x, r[T + 1][q].y, r[T + 1][q].z};
#pragma unroll
        for (int t = 0; t < T; ++t) {
            cv[T * q + t] = present ? vals[t] : 0u;
            ci[T * q + t] = present ? idxs[t] : kNoIndex;
            cx[T * q + t] = u2f(r[1 + t][q].x);
            cy[T * q + t] = u2f(r[1 + t][q].y);
            cz[T * q + t] = u2f(r[1 + t][q].z);
        }
        const uint32_t bnd = T == 2 ? r[0][q].z : r[NCH - 1][q].x;
        lb = umax(lb, present ? bnd : 0u);
    }
    return replay_round<KC>(L, lane, cv, ci, cx, cy, cz, lb, npicked, cap, prof);
}

}  // namespace ffps
