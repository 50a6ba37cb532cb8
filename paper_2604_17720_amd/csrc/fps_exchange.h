// The round shared by the multi-pick FPS kernels: cross-workgroup exchange of
// candidate records and the replay of the greedy rule on them.
//
// The points of a cloud are divided among reporting UNITS (up to 256 across
// workgroups: a whole workgroup, or each worker wave of a workgroup; or the
// worker lanes of a single workgroup).  Once per ROUND every unit contributes
// its T best points (two or three) and an upper bound on all its other points
// (the next value).  Across workgroups one wave per workgroup publishes the
// records of its units as 16-byte chunks, every chunk closed by a checksum that
// also encodes the round, and gathers the chunks of all units with coalesced
// device-scope loads (the only cross-workgroup step: no counters, no fences, no
// separate barrier).  The greedy rule of Eq. 1 is then replayed on the
// published candidates: the best candidate is the next pick as long as its
// value is strictly above B = max of all bounds, because no unpublished point
// can then reach it; picking it lowers the other candidates' values by the same
// distance rule, and the replay continues until the test fails.  The first pick
// of a round never needs the test: the global best point (largest value, lowest
// index among equals) is the best of its own unit, hence published.  Every
// workgroup replays the same arithmetic on the same records, so all agree on
// the picks without further communication.
//
// The replay (replay_round) is done by the whole workgroup at once, through
// pairwise bit masks over the live candidates (team_matrix and the settle
// step); only rounds that can deliver a single pick, or whose candidates do not
// fit, are replayed pick after pick by one wave.
//
// "Best" always means largest value, then lowest point index.  Points may be
// assigned to units in any way; candidates carry their indices, and equal
// values are resolved on the index wherever they can occur.
#pragma once
#include <type_traits>
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

constexpr int kMaxUnits = kMaxGridWG;     // reporting units of a cloud
constexpr int kRPL = kMaxUnits / kWave;   // unit records per lane of the gathering wave
constexpr int kSpinLimit = 1 << 19;
constexpr uint32_t kNoIndex = 0x7fffffffu;  // index of a candidate that does not exist
constexpr int kSets = 3;                    // a replay takes up to kSets * 64 live candidates
constexpr int kMaxLive = kSets * kWave;
static_assert(kMaxPicksPerRound <= kMaxLive && kMaxLive <= 256, "a round picks live candidates only");

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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
// mixed old and new words (the hardware does not tear an aligned 16-byte access)
// would pass only if the words it got wrong happened to leave the XOR unchanged;
// it is simply polled again otherwise.  Kept to three instructions per chunk: the
// gathering wave checks 24 chunks per lane on the critical path of every round.
__device__ __forceinline__ uint32_t chunk_check(uint32_t a, uint32_t b, uint32_t c, uint32_t round,
                                                uint32_t which) {
    return a ^ b ^ c ^ (round * 0x9E3779B1u + which * 0x85EBCA6Bu);
}
__device__ __forceinline__ bool chunk_ok(const u32x4 &c, uint32_t round, uint32_t which) {
    return c.w == chunk_check(c.x, c.y, c.z, round, which);
}

// Device-scope (all XCDs) 16-byte store and loads.  The compiler offers atomics
// up to 8 bytes only, so these are spelled out; sc1 is the device-scope cache
// policy the compiler itself uses for agent-scope atomics on this target.
// A vector-memory store of more than 8 bytes reads its data registers a few
// cycles after it issues, and a vector instruction that overwrites them right
// behind it changes what is stored.  The compiler keeps the distance for its
// own stores but cannot see into this text, hence the two idle cycles.
__device__ __forceinline__ void store_chunk(void *p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
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

// The records of three candidates and the complements of their indices, all reads in flight together.
__device__ __forceinline__ void lds_read_own_keys(u32x4 (&c)[3], uint32_t (&k)[3], const uint32_t (&a_c)[3],
                                                  const uint32_t (&a_k)[3]) {
    asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %7\n\tds_read_b128 %2, %8\n\t"
                 "ds_read_b32 %3, %9\n\tds_read_b32 %4, %10\n\tds_read_b32 %5, %11\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(c[0]), "=&v"(c[1]), "=&v"(c[2]), "=&v"(k[0]), "=&v"(k[1]), "=&v"(k[2])
                 : "v"(a_c[0]), "v"(a_c[1]), "v"(a_c[2]), "v"(a_k[0]), "v"(a_k[1]), "v"(a_k[2])
                 : "memory");
}
__device__ __forceinline__ void lds_write4(uint32_t off, uint32_t v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(off), "v"(v) : "memory");
}
// 8-byte LDS word written and read by one instruction each.
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
    // picks of the round: {x, y, z, seq}; spare slots that are never picks (they
    // keep the seed point), so that readers may read a few slots past the last pick
    __attribute__((aligned(16))) u32x4 pk[kMaxPicksPerRound + 8];
    uint32_t pk_idx[kMaxPicksPerRound];  // index of each pick of the round (pick-after-pick loop)
    uint32_t pk_val[kMaxPicksPerRound];  // and the value it was picked with
    // live candidates in compaction order; behind each array 64 entries, one per
    // lane, take what the compaction discards (one common entry would make every
    // such write a 64-way bank conflict)
    __attribute__((aligned(16))) u32x4 cand[kMaxLive + 4 + kWave];   // {x, y, z, value}
    __attribute__((aligned(16))) uint32_t nidx[kMaxLive + 4 + kWave];  // complement of the index: {value, nidx} compares as the order does
    // replay by the whole workgroup: number of live candidates (0: nothing to do this
    // round) and the threshold, then for every candidate b three bit masks over the
    // candidates a, in slices of 16: a lowers b to the threshold or below / a lowers b
    // / a comes before b in the order; the first two only where a comes before b
    __attribute__((aligned(8))) uint32_t team_total, team_T;
    __attribute__((aligned(8))) uint16_t mask[3][kMaxLive][kMaxLive / 16];
};
constexpr uint32_t kMaskRow = (kMaxLive / 16) * 2;        // bytes of one candidate's mask
constexpr uint32_t kMaskPlane = kMaxLive * kMaskRow;     // bytes of one of the three masks
static_assert(kMaskRow == 24, "a mask row is read as three 8-byte words");

// Counters of a profiling build (workgroup 0 only).
struct RoundProf {
    uint32_t acc[8];   // 100 MHz ticks per phase; [5], [6]: rounds replayed by the workgroup with up to 64 / more live candidates; [7]: polls
    uint32_t loop[4];  // [1], [3]: picks of those rounds, by the same split
    uint32_t sub[4];   // shader cycles inside the replay: bounds, counting, compaction, work of the whole workgroup
    uint32_t ev[4];    // [0]: live candidates; [2]: rounds ended by a lowered candidate
    uint32_t ord[6];   // shader cycles of that work: own candidates back from LDS, first barrier, share of the masks, second barrier, settling
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

// Workgroup barrier for LDS traffic issued by the assembly helpers of this file,
// which the compiler does not know about and therefore does not wait for.
__device__ __forceinline__ void team_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
    __syncthreads();
}

__device__ __forceinline__ void lds_write2b(uint32_t off, uint32_t v) {
    asm volatile("ds_write_b16 %0, %1" : : "v"(off), "v"(v) : "memory");
}

// What the picks of a round do to each other, worked out by all W waves of a
// workgroup (the wave that replays and the worker waves, which have nothing
// else to do at that point).  L.cand[0 .. total) holds the live candidates
// {x, y, z, value} in any order and L.nidx the complements of their indices,
// followed by at least 15 entries of value 0.  For candidates a and b let d be their squared
// distance (the individually rounded operations of sqdist, which give the same
// bits either way round) and let "a before b" mean that a precedes b in the
// order (value descending, index ascending).  A task takes a slice of 16
// candidates a and a set of 64 candidates b, one per lane, and writes 16 bits of
// each of b's masks: a before b; that and d <= T (picking a would put b out of
// this round); that and d < value of b (picking a would lower b).  Bit 31 - (a mod 32) of 32-bit
// word a / 32 stands for a.  Slices are dealt out to the waves in turn.  Called by
// every wave between two workgroup barriers.
__device__ __forceinline__ void team_matrix(RoundLds &L, int lane, int wv_in, int W) {
    const u32x2 hdr = lds_read8(lds_offset(&L.team_total));
    const int total = __builtin_amdgcn_readfirstlane((int)hdr.x);
    if (total == 0) return;
    const uint32_t T = (uint32_t)__builtin_amdgcn_readfirstlane((int)hdr.y);
    const int nsl = (total + 15) >> 4, nsets = (total + kWave - 1) / kWave;
    const uint32_t mask_off = lds_offset(L.mask);
    // One task: candidates a = 16 sl .. 16 sl + 15 (records ra, keys ka2; sl may differ
    // from lane to lane) against candidate b of this lane.
    auto task = [&](const u32x4 (&ra)[16], const u32x4 (&na)[4], int sl, int b, bool write) {
        const u32x4 cb = L.cand[b];
        const uint32_t nb = L.nidx[b];
        const float xb = u2f(cb.x), yb = u2f(cb.y), zb = u2f(cb.z);
        const uint64_t kb = ((uint64_t)cb.w << 32) | nb;
        uint32_t mk = 0u, ml = 0u, mb = 0u;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const uint64_t ka = ((uint64_t)ra[e].w << 32) | na[e >> 2][e & 3];
            const uint32_t d = f2u(sqdist(xb, yb, zb, u2f(ra[e].x), u2f(ra[e].y), u2f(ra[e].z)));
            // a before b: the sign of the 64-bit difference of the keys (both below 2^63)
            mb = __builtin_amdgcn_alignbit(mb, (uint32_t)((kb - ka) >> 32), 31);
            // values are bit patterns of non-negative numbers: the sign of a difference is
            // the comparison, and it goes into the mask (built from its most significant
            // end: m = 2 m + bit) with one funnel shift
            mk = __builtin_amdgcn_alignbit(mk, T - d, 31);        // T < d, turned round below
            ml = __builtin_amdgcn_alignbit(ml, d - cb.w, 31);     // d < value of b
        }
        // the first two masks are only wanted where a comes before b
        mk = ~mk & mb;
        ml &= mb;
        // two slices share a 32-bit word, the earlier one in its upper half
        const uint32_t at = mask_off + (uint32_t)b * kMaskRow + (uint32_t)(sl ^ 1) * 2;
        if (write) {
            lds_write2b(at, mk);
            lds_write2b(at + kMaskPlane, ml);
            lds_write2b(at + 2 * kMaskPlane, mb);
        }
    };
    // When the last set holds no more than 16 (32) candidates, a task against it would
    // leave three quarters (half) of the lanes idle: such a set is taken by groups of
    // 4 (2) slices instead, each row of 16 (32) lanes with a slice of its own.
    const int tail = total - (nsets - 1) * kWave;
    const int pack = tail <= 16 ? 4 : tail <= 32 ? 2 : 1;
    const int nmain = pack > 1 ? nsets - 1 : nsets;  // sets taken slice by slice
    const int wv = __builtin_amdgcn_readfirstlane(wv_in);
    // Plain loads, all of a task's up front, so that they are in flight together (the
    // arrays were written before the barrier).  A wave takes slices wv, wv + W, ...
    // and does all (full) sets of a slice, whose 16 candidates it then reads only once.
    if (nmain > 0) {
        for (int sl = wv; sl < nsl; sl += W) {
            u32x4 ra[16], na[4];
#pragma unroll
            for (int e = 0; e < 16; ++e) ra[e] = L.cand[sl * 16 + e];  // the same address in all lanes
#pragma unroll
            for (int e = 0; e < 4; ++e) na[e] = *reinterpret_cast<const u32x4 *>(&L.nidx[sl * 16 + 4 * e]);
#pragma unroll 1
            for (int set = 0; set < nmain; ++set) task(ra, na, sl, set * kWave + lane, true);
        }
    }
    if (pack > 1) {
        // groups of slices, dealt out from the last wave downwards (the first waves
        // have the most slices above)
        const int rows = kWave / pack, rsh = pack == 4 ? 4 : 5;  // lanes per slice, and its log2
        const int ngroups = (nsl + pack - 1) / pack;
#pragma unroll 1
        for (int g = W - 1 - wv; g < ngroups; g += W) {
            const int sl = g * pack + (lane >> rsh);
            const bool ok = sl < nsl;
            const int sr = ok ? sl : nsl - 1;
            u32x4 ra[16], na[4];
#pragma unroll
            for (int e = 0; e < 16; ++e) ra[e] = L.cand[sr * 16 + e];
#pragma unroll
            for (int e = 0; e < 4; ++e) na[e] = *reinterpret_cast<const u32x4 *>(&L.nidx[sr * 16 + 4 * e]);
            task(ra, na, sr, (nsets - 1) * kWave + (lane & (rows - 1)), ok);
        }
    }
}

// Replay of the greedy rule of Eq. 1 on KC candidates per lane of ONE full wave
// (value bits cv, point index ci, coordinates cx/cy/cz; a candidate that does
// not exist has value 0 and index kNoIndex), given lb = the lane's share of the
// bounds on all points that are not candidates.  Pick number c of the round is
// written as {x, y, z, npicked + c} to L.pk[c] (16-byte LDS writes), and what
// record_picks needs to name its index and value is left in the lanes or in L.
// Returns the number of picks (1 .. cap) and how they were noted.  The
// candidate arrays are used up.
struct RoundResult {
    int cnt;        // picks of the round, or -1 when the round failed
    bool stuck;     // the pairwise masks named no pick at all, which cannot happen while
                    // they are consistent; cnt is 1 then so that the kernel still ends,
                    // and the caller reports kErrInconsistent in the status word
    bool by_lane;   // picks noted in the lanes (below) rather than in L.pk_idx / L.pk_val
    // by_lane: what this lane's live candidates became: pick number within the
    // round (-1: not picked), point index, value when picked
    int pc[kSets];
    uint32_t pi[kSets], pv[kSets];
};

// Writes index (and value) of the picks of a round to the outputs; run by the
// wave that ran the round, in one workgroup of the cloud.
__device__ __forceinline__ void record_picks(const RoundLds &L, int lane, const RoundResult &r,
                                             int npicked, int32_t *idx_out, float *md_out);

// The other team_waves - 1 waves of the workgroup take part in the replay: they
// wait at a workgroup barrier after handing in their reports, call team_matrix
// and pass a second barrier, every round; this function passes the same two
// barriers exactly once, whatever path the round takes.  MAXS (1 .. kSets) is the
// largest number of sets of 64 live candidates the caller wants code for.  live_sets (1 .. kSets)
// limits the live candidates to that many per lane: the pairwise work grows with
// the square of their number, and where a round ends after a few tens of picks
// anyway (small clouds) the candidates further down the order are not reached.
// live_target > 0 asks for about that many live candidates in all, for the same
// reason.
template <int KC, int MAXS = kSets>
__device__ __forceinline__ RoundResult replay_round(RoundLds &L, int lane, uint32_t (&cv)[KC],
                                            uint32_t (&ci)[KC], float (&cx)[KC], float (&cy)[KC],
                                            float (&cz)[KC], uint32_t lb, int npicked, int cap,
                                            RoundProf *prof, int team_waves, int live_sets = MAXS,
                                            int live_target = 0, bool fresh = true) {
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
#ifdef FFPS_PROFILE
    uint64_t oc = 0;
#define FFPS_ORD(i)                              \
    do {                                         \
        if (prof) {                              \
            uint64_t n_ = clock64();             \
            prof->ord[i] += (uint32_t)(n_ - oc); \
            oc = n_;                             \
        }                                        \
    } while (0)
#else
#define FFPS_ORD(i) \
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
    // than kMaxLive candidates are above the bound T is raised to the largest
    // value that is number kSets + 1 in its lane, which leaves at most kSets per lane.
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
        // about `aim` candidates, taking their values as evenly spread between the
        // threshold and the best one (any threshold above the bound will do)
        auto thin_out = [&](int aim) {
            const uint32_t span = V - T;
            T = V - (uint32_t)(((uint64_t)span * (uint32_t)aim) / (uint32_t)total);
            count_live();
        };
        if (live_target > 0 && total > live_target + live_target / 4) thin_out(live_target);
        // more than fit: aim a little below the limit, twice if need be, before falling
        // back on a threshold that is certain to fit but usually leaves far fewer
        const int limit = live_sets * kWave;
        if (total > limit) thin_out(limit - limit / 16);
        if (total > limit) thin_out(limit - limit / 16);
        if (total > limit) {
            // the largest value that is only number live_sets + 1 in its lane
            uint32_t t[kSets + 1] = {};
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                const uint32_t v = cv[q];
#pragma unroll
                for (int r = kSets; r >= 1; --r) t[r] = umax(t[r], v < t[r - 1] ? v : t[r - 1]);
                t[0] = umax(t[0], v);
            }
            T = umax(T, wave_max_u32(live_sets == 1 ? t[1] : live_sets == 2 ? t[2] : t[kSets]));
            static_assert(MAXS >= 1 && MAXS <= kSets, "sets of 64 live candidates");
            count_live();
        }
    }
    // With at most MAXS * 64 live candidates the replay needs no argmax per pick.  Take
    // the candidates in the order (value descending, index ascending).  The first
    // one is the next pick.  Picking a point can only lower other values, so the
    // next candidate in that order is the following pick as long as its own value
    // has not been lowered by a pick of this round: everything behind it started
    // no higher and has not grown, candidates ahead of it are picked or out of
    // the round, and unreported points are at or below the threshold.  A candidate
    // whose value has been lowered to the threshold or below is out of this
    // round and is passed over; one that has been lowered but is still above the
    // threshold belongs further back in the order, at its new value, and the
    // round ends where the order reaches that value (the next round sees the
    // candidate again).  All of this is decided for all candidates at once from
    // pairwise bit masks (further down).
    const bool ordered = total >= 1 && total <= MAXS * kWave;
    FFPS_SUB(1);
#ifdef FFPS_PROFILE
    if (prof && ordered) prof->acc[total <= kWave ? 5 : 6] += 1;
#endif
    RoundResult res;
    res.stuck = false;
#pragma unroll
    for (int s = 0; s < kSets; ++s) {
        res.pc[s] = -1;
        res.pi[s] = kNoIndex;
        res.pv[s] = 0u;
    }
    if (ordered) {
        const uint32_t cand_off = lds_offset(L.cand), nidx_off = lds_offset(L.nidx);
        // compaction without branches (predicated writes by the live lanes alone were
        // slower): a candidate that is not live goes to the lane's own slot behind the
        // live ones, which nobody reads
        {
            const uint32_t dump = (uint32_t)(kMaxLive + 4 + lane);
            uint32_t pos = (uint32_t)before;
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                const bool live = cv[q] > T;
                u32x4 r;
                r.x = f2u(cx[q]); r.y = f2u(cy[q]); r.z = f2u(cz[q]); r.w = cv[q];
                lds_write16(cand_off + (live ? pos : dump) * 16, r);
                lds_write4(nidx_off + (live ? pos : dump) * 4, ~ci[q]);
                pos += live ? 1u : 0u;
            }
        }
        // the same wave wrote and now reads: LDS keeps its accesses in order
        FFPS_SUB(2);
#ifdef FFPS_PROFILE
        oc = clock64();
#endif
        // ---- every lane takes the candidates at positions lane, lane + 64, ... back
        //      from LDS (sets 0, 1, ...); they are in no particular order yet ----
        const int nsets = (total + kWave - 1) / kWave;  // sets in use
        bool h[kSets];          // this lane has a candidate in set s
        uint32_t a_c[kSets], a_k[kSets];  // where to read it (position 0 if it has none)
#pragma unroll
        for (int s = 0; s < kSets; ++s) {
            const int p = lane + s * kWave;
            h[s] = p < total;
            const uint32_t q = h[s] ? (uint32_t)p : 0u;
            a_c[s] = cand_off + q * 16; a_k[s] = nidx_off + q * 4;
        }
        u32x4 c[kSets];
        uint32_t ix[kSets], o[kSets];  // index; value at the start of the round
        lds_read_own_keys(c, ix, a_c, a_k);
#pragma unroll
        for (int s = 0; s < kSets; ++s) ix[s] = ~ix[s];
#pragma unroll
        for (int s = 0; s < kSets; ++s) o[s] = h[s] ? c[s].w : 0u;
        FFPS_ORD(0);
        {
            // ---- replay by the whole workgroup: no order, no pick after pick.  The
            //      other waves work out, for every pair of live candidates, which one
            //      comes first and what picking it does to the other (team_matrix).
            //      Candidate b is a pick of this round when no pick before it lowers
            //      it.  Which candidates are picks follows from the candidates before
            //      them alone, so starting from "all of them" and applying the rule to
            //      every candidate at once settles one more candidate of the order per
            //      pass at least, and in practice all of them after a few passes.
            //      What becomes of the lowered candidates, and where the round ends
            //      because of them, is worked out afterwards (further down). ----
            if (lane < 16) {
                // entries of value 0 behind the last candidate: they come after every
                // live one, which keeps their bits out of the masks
                u32x4 zr;
                zr.x = 0u; zr.y = 0u; zr.z = 0u; zr.w = 0u;
                lds_write16(cand_off + (uint32_t)(total + lane) * 16, zr);
                lds_write4(nidx_off + (uint32_t)(total + lane) * 4, 0u);
            }
            if (lane == 0) {
                u32x2 hd;
                hd.x = (uint32_t)total; hd.y = T;
                lds_write8(lds_offset(&L.team_total), hd);
            }
            team_barrier();
            FFPS_ORD(1);
            team_matrix(L, lane, 0, team_waves);
            FFPS_ORD(2);
            team_barrier();
            FFPS_ORD(3);
            // The rest for NS sets in use (known when compiling, so that every loop
            // below is unrolled and the words of the sets not in use are not touched).
            bool ended = false;
            auto settle = [&](auto ns_tag) {
                constexpr int NS = decltype(ns_tag)::value;
                constexpr int NW = 2 * NS;
                // this lane's masks (plain loads, all in flight together; written by the
                // other waves before the barrier)
                uint32_t KB[NS][6], LB[NS][6], BB[NS][6];
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const int b = lane + s * kWave;
#pragma unroll
                    for (int wd = 0; wd < NW; wd += 2) {
                        const u32x2 k2 = *reinterpret_cast<const u32x2 *>(&L.mask[0][b][2 * wd]);
                        const u32x2 l2 = *reinterpret_cast<const u32x2 *>(&L.mask[1][b][2 * wd]);
                        const u32x2 b2 = *reinterpret_cast<const u32x2 *>(&L.mask[2][b][2 * wd]);
                        KB[s][wd] = k2.x; KB[s][wd + 1] = k2.y;
                        LB[s][wd] = l2.x; LB[s][wd + 1] = l2.y;
                        BB[s][wd] = b2.x; BB[s][wd + 1] = b2.y;
                    }
                }
                // a set of candidates as mask words (bit 31 - (a mod 32) of word a / 32)
                auto to_words = [&](const uint64_t (&m)[NS], uint32_t (&wds)[NW]) {
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        wds[2 * s] = __builtin_bitreverse32((uint32_t)m[s]);
                        wds[2 * s + 1] = __builtin_bitreverse32((uint32_t)(m[s] >> 32));
                    }
                };
                auto hits = [&](const uint32_t (&m)[6], const uint32_t (&wds)[NW]) {
                    uint32_t acc = 0u;
#pragma unroll
                    for (int wd = 0; wd < NW; ++wd) acc |= m[wd] & wds[wd];
                    return acc != 0u;
                };
                uint64_t pm[NS];
                uint32_t P[NW];
                bool pk[NS];
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    pk[s] = h[s];
                    pm[s] = __builtin_amdgcn_ballot_w64(h[s]);
                }
                to_words(pm, P);
                for (int pass = 0; pass <= total; ++pass) {
                    uint32_t Q[NW];
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        pk[s] = h[s] && !hits(LB[s], P);
                        pm[s] = __builtin_amdgcn_ballot_w64(pk[s]);
                    }
                    to_words(pm, Q);
                    bool same = true;
#pragma unroll
                    for (int wd = 0; wd < NW; ++wd) {
                        same = same && Q[wd] == P[wd];
                        P[wd] = Q[wd];
                    }
                    if (same) break;
                }
                // A candidate that a pick lowers is not a pick of this round.  If the pick
                // takes it to the threshold or below it is simply out of the round.
                // Otherwise it is still live at a lower value, and it would be the next
                // pick as soon as the candidates left in the order are no higher than
                // that value: its new value is the smallest distance to the picks before
                // it that lower it (few, and named by its mask), the largest such value
                // over all lowered candidates is where the round ends, and the picks are
                // the candidates strictly above it.
                bool wounded[NS];
                uint64_t any_w = 0;
                uint32_t F[NW];
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    wounded[s] = h[s] && !pk[s] && !hits(KB[s], P);
                    any_w |= __builtin_amdgcn_ballot_w64(wounded[s]);
                }
                ended = any_w != 0;
                if (ended) {
                    uint32_t vstar = 0u;
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        uint32_t vp = 0xffffffffu;
                        const float xb = u2f(c[s].x), yb = u2f(c[s].y), zb = u2f(c[s].z);
#pragma unroll
                        for (int wd = 0; wd < NW; ++wd) {
                            uint32_t m = wounded[s] ? (LB[s][wd] & P[wd]) : 0u;
                            while (__builtin_amdgcn_ballot_w64(m != 0u) != 0) {
                                const bool act = m != 0u;
                                const int lz = __builtin_clz(m | 1u);  // the first candidate left in the word
                                m &= ~(0x80000000u >> lz);
                                const u32x4 ra = lds_read16(cand_off + (act ? (uint32_t)(wd * 32 + lz) : 0u) * 16);
                                const uint32_t d = f2u(sqdist(xb, yb, zb, u2f(ra.x), u2f(ra.y), u2f(ra.z)));
                                vp = act && d < vp ? d : vp;
                            }
                        }
                        vstar = umax(vstar, wounded[s] ? vp : 0u);
                    }
                    vstar = wave_max_u32(vstar);
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        pk[s] = pk[s] && o[s] > vstar;
                        pm[s] = __builtin_amdgcn_ballot_w64(pk[s]);
                    }
                }
                to_words(pm, F);
                int npk = 0;
#pragma unroll
                for (int s = 0; s < NS; ++s) npk += __builtin_popcountll(pm[s]);
                cnt = npk < cap ? npk : cap;
                // a pick's number within the round: the picks before it
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    int ord = 0;
#pragma unroll
                    for (int wd = 0; wd < NW; ++wd) ord += __builtin_popcount(BB[s][wd] & F[wd]);
                    const bool sel = pk[s] && ord < cap;
                    if (sel) {
                        u32x4 rec = c[s];
                        rec.w = (uint32_t)(npicked + ord);
                        lds_write16(pk_off + (uint32_t)ord * 16, rec);
                    }
                    res.pc[s] = sel ? ord : -1;
                    res.pi[s] = ix[s];
                    res.pv[s] = o[s];
                }
            };
            static_assert(kSets == 3, "one case per number of sets");
            if (nsets == 1 || MAXS == 1) settle(std::integral_constant<int, 1>{});
            else if (nsets == 2 || MAXS == 2) settle(std::integral_constant<int, 2>{});
            else if constexpr (MAXS >= 3) settle(std::integral_constant<int, 3>{});
            if (cnt == 0) {
                // The first candidate of the order is always a pick.  Every round must
                // make progress for the kernel to end, whatever went wrong.
                cnt = 1;
                res.stuck = true;
            }
            FFPS_ORD(4);
            FFPS_SUB(3);
#ifdef FFPS_PROFILE
            if (prof) {
                prof->ev[0] += (uint32_t)total;
                prof->ev[2] += ended ? 1u : 0u;
                prof->loop[total <= kWave ? 1 : 3] += cnt;
            }
#endif
        }
    } else {
        // a single pick (best candidate not above the bound, or cap 1), or more
        // live candidates than fit above every threshold tried: this wave works
        // pick after pick on all candidates of every lane.  The other waves wait at
        // the two barriers of the replay: nothing for them to do.
        if (lane == 0) lds_write4(lds_offset(&L.team_total), 0u);
        team_barrier();
        team_barrier();
        // Not fresh: the candidates' values are exact but the caller cannot promise that
        // the best point of all is among them, so nothing may be picked on the strength
        // of being the best candidate alone: the first pick, too, must be above the
        // bound.  If it is not the round is empty (cnt = 0) and the caller sees to it
        // that the next one is fresh.
        while (true) {
            uint32_t bv, bi;
            int bq;
            lane_best(bv, bi, bq);
            V = wave_max_u32(bv);
            if ((cnt > 0 || !fresh) && !(V > Bound)) break;
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
    res.cnt = cnt;
    res.by_lane = ordered;
    return res;
}

// Status word for a round whose masks named no pick (FFPS_ERR_INTERNAL of the C
// interface, kErrInconsistent); status[2] = the round.  Called by one lane.
__device__ __forceinline__ void note_inconsistent(int *status, int round) {
    int expected = 0;
    if (__hip_atomic_compare_exchange_strong(status, &expected, kErrInconsistent, __ATOMIC_RELAXED,
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        status[2] = round;
}

__device__ __forceinline__ void record_picks(const RoundLds &L, int lane, const RoundResult &r,
                                             int npicked, int32_t *idx_out, float *md_out) {
    if (r.by_lane) {
#pragma unroll
        for (int e = 0; e < kSets; ++e) {
            if (r.pc[e] >= 0) {
                idx_out[npicked + r.pc[e]] = (int32_t)r.pi[e];
                if (md_out) md_out[npicked + r.pc[e]] = u2f(r.pv[e]);
            }
        }
        return;
    }
    for (int c = lane; c < r.cnt; c += kWave) {
        idx_out[npicked + c] = (int32_t)L.pk_idx[c];
        if (md_out) md_out[npicked + c] = u2f(L.pk_val[c]);
    }
}

// One round, run by ONE full wave of a workgroup.  The cloud has U reporting
// units (a whole workgroup, or each of its worker waves); lanes 0 .. nsub-1 of
// this wave publish `in` as unit unit0 + lane.  The wave then gathers all U
// records and replays with the help of the workgroup's other team_waves - 1 waves
// (replay_round), which leaves each pick as {x, y, z, npicked + c} in L.pk[c].
// Returns the picks of the round (1 .. cap; see record_picks), or a count of -1
// after setting *status when another unit's record never arrived (the two
// barriers of the replay have not been passed then).
template <int T, int MAXS = kSets>
__device__ __forceinline__ RoundResult exchange_round(RoundLds &L, char *exchange, int U, int unit0,
                                                      int nsub, int lane, uint32_t round,
                                                      const RoundInput<T> &in, int npicked, int cap,
                                                      int *status, RoundProf *prof, int team_waves,
                                                      int live_target = 0, int spin_limit = kSpinLimit,
                                                      bool fresh = true) {
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
        if (spin >= spin_limit) {
            gave_up = true;
            break;
        }
    }
    FFPS_STAMP(prof, 3);
    if (gave_up) {
        // the first workgroup to give up notes what it was waiting for: status[2] =
        // round, status[3] = lowest unit whose record had not arrived, status[4] = its own unit
        int missing = 0x7fffffff;
#pragma unroll
        for (int q = kRPL - 1; q >= 0; --q) {
            bool ok = true;
#pragma unroll
            for (int c = 0; c < NCH; ++c) ok = ok && chunk_ok(r[c][q], round, (uint32_t)c);
            if (!ok && q * kWave + lane < U) missing = q * kWave + lane;
        }
        missing = (int)wave_min_u32((uint32_t)missing);
        if (lane == 0) {
            int expected = 0;
            if (__hip_atomic_compare_exchange_strong(status, &expected, kErrGaveUp, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                status[2] = (int)round;
                status[3] = missing;
                status[4] = unit0;
            }
        }
        RoundResult failed = {};
        failed.cnt = -1;
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
    return replay_round<KC, MAXS>(L, lane, cv, ci, cx, cy, cz, lb, npicked, cap, prof, team_waves, MAXS,
                                        live_target, fresh);
}

}  // namespace ffps
