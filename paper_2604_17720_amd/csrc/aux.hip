// Index bookkeeping around the FPS loop: candidate pruning and the fill of
// FPS-Prune (Alg. 1, layer 1), and the gathers / prefix copies of the stage
// chain (Alg. 1, layers 2..L; Sec. 3.3).  All O(N) integer work.
#include "fps_device.h"
#include "fps_launch.h"

namespace ffps {

namespace {

constexpr int kT = 256;

inline int blocks_for(size_t n, int per_block = kT, int cap = 4096) {
    size_t b = (n + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > (size_t)cap) b = cap;
    return (int)b;
}

__global__ void k_fill_zero(uint32_t *p, size_t words) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < words;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

// Position i of the ascending candidate list.  The raw list
// raw[j] = (start + floor(j*N/Nc)) mod N wraps once, at j0; the sorted list is
// the wrapped tail followed by the unwrapped head, i.e. raw[(i + j0) mod Nc].
__device__ __forceinline__ int cand_at(int i, int N, int Nc, int start, int j0) {
    long j = (long)i + j0;
    if (j >= Nc) j -= Nc;
    return (int)(((long)start + (j * (long)N) / Nc) % N);
}

__global__ void k_gather_candidates(const float *__restrict__ xyz, int N, int Nc, int start, int j0,
                                    float *__restrict__ cxyz) {
    const int b = blockIdx.y;
    const float *src = xyz + (size_t)b * N * 3;
    float *dst = cxyz + (size_t)b * Nc * 3;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < Nc; i += gridDim.x * blockDim.x) {
        int c = cand_at(i, N, Nc, start, j0);
        dst[3 * (size_t)i + 0] = src[3 * (size_t)c + 0];
        dst[3 * (size_t)i + 1] = src[3 * (size_t)c + 1];
        dst[3 * (size_t)i + 2] = src[3 * (size_t)c + 2];
    }
}

__global__ void k_map_candidates(const int32_t *__restrict__ loc, long loc_stride, int N, int Nc,
                                 int start, int j0, int k, int32_t *__restrict__ idx,
                                 long idx_stride) {
    const int b = blockIdx.y;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < k; j += gridDim.x * blockDim.x)
        idx[b * idx_stride + j] = cand_at(loc[b * loc_stride + j], N, Nc, start, j0);
}

// One workgroup per cloud: bitmap of the k FPS picks, ranks of the free
// indices by popcount + scan, then every free index decides on its own whether
// some j maps to its rank: fill[j] = free[floor(j*F/R)], F = N - k.  Since
// F >= R the ranks floor(j*F/R) are distinct, and rank r is hit exactly by
// j = ceil(r*R/F) when floor(j*F/R) == r.
__global__ __launch_bounds__(1024) void k_fill(int N, int k, int R, int32_t *__restrict__ idx_all,
                                               long idx_stride, uint32_t *__restrict__ bitmap_all) {
    __shared__ int part[1024];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int words = (N + 31) / 32;
    uint32_t *bm = bitmap_all + (size_t)b * words;
    int32_t *idx = idx_all + b * idx_stride;

    for (int i = tid; i < words; i += 1024) bm[i] = 0u;
    __syncthreads();
    for (int j = tid; j < k; j += 1024) {
        int v = idx[j];
        atomicOr(&bm[v >> 5], 1u << (v & 31));
    }
    __syncthreads();

    const int per = (words + 1023) / 1024;
    const int w0 = tid * per;
    const int w1 = min(words, w0 + per);
    int cnt = 0;
    for (int wd = w0; wd < w1; ++wd) {
        uint32_t valid = (wd == words - 1 && (N & 31)) ? ((1u << (N & 31)) - 1u) : 0xffffffffu;
        cnt += __popc(~bm[wd] & valid);
    }
    part[tid] = cnt;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {  // inclusive scan
        int v = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    // Rank r is taken by fill slot j = ceil(r*R/F) iff floor(j*F/R) == r, i.e. iff
    // acc = j*F - r*R lies in [0, R).  One division finds j for the thread's first
    // rank; from rank to rank acc drops by R and, when it goes negative, j steps up.
    long r = part[tid] - cnt;  // rank of this thread's first free index
    const long F = (long)N - k;
    long j = (r * R + F - 1) / F;
    long acc = j * F - r * R;
    for (int wd = w0; wd < w1; ++wd) {
        uint32_t valid = (wd == words - 1 && (N & 31)) ? ((1u << (N & 31)) - 1u) : 0xffffffffu;
        uint32_t free_bits = ~bm[wd] & valid;
        while (free_bits) {
            int bit = __ffs(free_bits) - 1;
            free_bits &= free_bits - 1;
            if (acc < R && j < R) idx[k + j] = wd * 32 + bit;
            acc -= R;
            if (acc < 0) {
                ++j;
                acc += F;
            }
        }
    }
}

__global__ void k_gather_points(const float *__restrict__ xyz, int N, const int32_t *__restrict__ sel,
                                long sel_stride, int S, float *__restrict__ dst) {
    const int b = blockIdx.y;
    const float *src = xyz + (size_t)b * N * 3;
    float *out = dst + (size_t)b * S * 3;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < S; j += gridDim.x * blockDim.x) {
        int c = sel[b * sel_stride + j];
        out[3 * (size_t)j + 0] = src[3 * (size_t)c + 0];
        out[3 * (size_t)j + 1] = src[3 * (size_t)c + 1];
        out[3 * (size_t)j + 2] = src[3 * (size_t)c + 2];
    }
}

// out[b][j][0..C) = rows[b][sel[b][j]][0..C): one thread per output float, so
// consecutive threads write consecutive addresses.
__global__ void k_gather_rows(const float *__restrict__ rows, int N, int C,
                              const int32_t *__restrict__ sel, long sel_stride, int S,
                              float *__restrict__ out) {
    const int b = blockIdx.y;
    const float *src = rows + (size_t)b * N * C;
    float *dst = out + (size_t)b * S * C;
    const size_t total = (size_t)S * C;
    for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const size_t j = e / C;
        const int c = (int)(e - j * C);
        dst[e] = src[(size_t)sel[b * sel_stride + j] * C + c];
    }
}

__global__ void k_compose(const int32_t *__restrict__ prev, long prev_stride,
                          const int32_t *__restrict__ loc, long loc_stride, int S,
                          int32_t *__restrict__ out, long out_stride) {
    const int b = blockIdx.y;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < S; j += gridDim.x * blockDim.x)
        out[b * out_stride + j] = prev[b * prev_stride + loc[b * loc_stride + j]];
}

__global__ void k_copy_prefix(const int32_t *__restrict__ src, long src_stride, int S,
                              int32_t *__restrict__ out, long out_stride) {
    const int b = blockIdx.y;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < S; j += gridDim.x * blockDim.x)
        out[b * out_stride + j] = src[b * src_stride + j];
}

// ---- seeded random select / fill --------------------------------------------
// Seeded bijection of [0, N): a 4-round Feistel network over 2h bits,
// 2^(2h) >= N, with a 32-bit integer mixer as round function, walked until the
// value falls below N.  Stateless: every element is computed on its own.
struct Perm {
    uint32_t n, mask, k0, k1;
    int h;
};
__host__ __device__ inline Perm make_perm(int N, uint64_t seed) {
    Perm p;
    p.n = (uint32_t)N;
    p.h = 1;
    while ((1ull << (2 * p.h)) < (unsigned long long)N) ++p.h;
    p.mask = (1u << p.h) - 1u;
    p.k0 = (uint32_t)seed;
    p.k1 = (uint32_t)(seed >> 32);
    return p;
}
__device__ __forceinline__ uint32_t perm_mix(uint32_t x) {
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint32_t perm_at(const Perm &p, uint32_t j) {
    uint32_t x = j;
    do {
        uint32_t l = (x >> p.h) & p.mask, r = x & p.mask;
#pragma unroll
        for (uint32_t round = 0; round < 4; ++round) {
            uint32_t f = perm_mix(r ^ (((round & 1) ? p.k1 : p.k0) + 0x9E3779B9u * (round + 1))) & p.mask;
            uint32_t t = l ^ f;
            l = r;
            r = t;
        }
        x = (l << p.h) | r;
    } while (x >= p.n);
    return x;
}
constexpr uint64_t kFillSeedXor = 0xD1B54A32D192ED03ull;

// bitmap[b] |= { perm_{seed+b}(j) : j < Nc }   (bitmap cleared beforehand)
__global__ void k_perm_mark(int N, int Nc, uint64_t seed, uint32_t *__restrict__ bitmap_all) {
    const int b = blockIdx.y;
    uint32_t *bm = bitmap_all + (size_t)b * ((N + 31) / 32);
    const Perm p = make_perm(N, seed + (uint64_t)b);
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < Nc; j += gridDim.x * blockDim.x) {
        uint32_t t = perm_at(p, (uint32_t)j);
        atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
}

// One workgroup per cloud: force `start` into the candidate set (in place of
// the last drawn candidate), then list the set in ascending order with the
// candidates' coordinates, and report the position of `start` in it.
__global__ __launch_bounds__(1024) void k_perm_compact(const float *__restrict__ xyz_all, int N, int Nc,
                                                       int start, uint64_t seed,
                                                       uint32_t *__restrict__ bitmap_all,
                                                       int32_t *__restrict__ cand_all,
                                                       float *__restrict__ cxyz_all,
                                                       int *__restrict__ spos_all) {
    __shared__ int part[1024];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int words = (N + 31) / 32;
    uint32_t *bm = bitmap_all + (size_t)b * words;
    const float *xyz = xyz_all + (size_t)b * N * 3;
    int32_t *cand = cand_all + (size_t)b * Nc;
    float *cxyz = cxyz_all + (size_t)b * Nc * 3;
    if (tid == 0 && !((bm[start >> 5] >> (start & 31)) & 1u)) {
        const uint32_t last = perm_at(make_perm(N, seed + (uint64_t)b), (uint32_t)(Nc - 1));
        bm[last >> 5] &= ~(1u << (last & 31));
        bm[start >> 5] |= 1u << (start & 31);
    }
    __syncthreads();
    const int per = (words + 1023) / 1024;
    const int w0 = tid * per, w1 = min(words, w0 + per);
    int cnt = 0;
    for (int wd = w0; wd < w1; ++wd) cnt += __popc(bm[wd]);
    part[tid] = cnt;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {  // inclusive scan
        int v = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int r = part[tid] - cnt;
    for (int wd = w0; wd < w1; ++wd) {
        uint32_t bits = bm[wd];
        while (bits) {
            const int i = wd * 32 + __ffs(bits) - 1;
            bits &= bits - 1;
            cand[r] = i;
            cxyz[3 * (size_t)r + 0] = xyz[3 * (size_t)i + 0];
            cxyz[3 * (size_t)r + 1] = xyz[3 * (size_t)i + 1];
            cxyz[3 * (size_t)r + 2] = xyz[3 * (size_t)i + 2];
            if (i == start) spos_all[b] = r;
            ++r;
        }
    }
}

// One workgroup per cloud: idx[k + r] = r-th index, in the order of a second
// permutation of [0, N), that is not among idx[0..k); r < R.
__global__ __launch_bounds__(1024) void k_fill_perm(int N, int k, int R, uint64_t seed,
                                                    int32_t *__restrict__ idx_all, long idx_stride,
                                                    uint32_t *__restrict__ bitmap_all) {
    __shared__ int part[1024];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int words = (N + 31) / 32;
    uint32_t *bm = bitmap_all + (size_t)b * words;
    int32_t *idx = idx_all + b * idx_stride;
    for (int i = tid; i < words; i += 1024) bm[i] = 0u;
    __syncthreads();
    for (int j = tid; j < k; j += 1024) {
        int v = idx[j];
        atomicOr(&bm[v >> 5], 1u << (v & 31));
    }
    __syncthreads();
    const Perm p = make_perm(N, (seed + (uint64_t)b) ^ kFillSeedXor);
    const int per = (N + 1023) / 1024;
    const int j0 = tid * per, j1 = min(N, j0 + per);
    int cnt = 0;
    for (int j = j0; j < j1; ++j) {
        const uint32_t t = perm_at(p, (uint32_t)j);
        cnt += !((bm[t >> 5] >> (t & 31)) & 1u);
    }
    part[tid] = cnt;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        int v = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int r = part[tid] - cnt;
    for (int j = j0; j < j1 && r < R; ++j) {
        const uint32_t t = perm_at(p, (uint32_t)j);
        if (!((bm[t >> 5] >> (t & 31)) & 1u)) idx[k + r++] = (int32_t)t;
    }
}

// Reference point for the multi-workgroup kernels: `iters` plain grid barriers
// (one device-scope atomic arrive + a bounded spin on the counter per barrier).
__global__ __launch_bounds__(256) void k_barrier_probe(unsigned *counter, int iters, int *status) {
    const unsigned G = gridDim.x;
    for (int it = 1; it <= iters; ++it) {
        __syncthreads();
        if (threadIdx.x == 0) {
            __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            int spin = 0;
            while (__hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < G * (unsigned)it) {
                if (++spin > (1 << 22)) {
                    __hip_atomic_store(status, -5, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
        }
        __syncthreads();
        if (__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    }
}

inline int wrap_point(int N, int Nc, int start) {
    // smallest j with start + floor(j*N/Nc) >= N, capped at Nc (no wrap)
    long j0 = (((long)N - start) * Nc + N - 1) / N;
    return (int)(j0 > Nc ? Nc : j0);
}

}  // namespace

// Diagnostic: sustained rate of the arithmetic of a distance update.  Every lane
// keeps 16 independent values and applies subtract, multiply, add, minimum to
// each of them `iters` times: individually rounded fp32 operations with no
// memory traffic, the mix of Eq. 1's inner loop.  One word per wave goes to
// `sink` so that the work cannot be dropped.
__global__ __launch_bounds__(1024) void k_alu_probe(int iters, float seed, float *sink) {
    constexpr int CH = 16;
    float a[CH];
    const float b = seed + (float)threadIdx.x * 1e-3f, c = 0.999f;
#pragma unroll
    for (int i = 0; i < CH; ++i) a[i] = (float)(i + (int)threadIdx.x);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            a[i] = __fsub_rn(a[i], b);
            a[i] = __fmul_rn(a[i], c);
            a[i] = __fadd_rn(a[i], b);
            a[i] = fminf(a[i], 1e30f);
        }
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < CH; ++i) t += a[i];
    if ((threadIdx.x & 63) == 0) sink[(blockIdx.x * blockDim.x + threadIdx.x) >> 6] = t;
}

hipError_t launch_alu_probe(float *sink, int num_wg, int waves_per_wg, int iters, hipStream_t s) {
    k_alu_probe<<<dim3(num_wg), dim3(64 * waves_per_wg), 0, s>>>(iters, 1.0f, sink);
    return hipGetLastError();
}

hipError_t launch_barrier_probe(unsigned *counter, int *status, int num_wg, int iters, hipStream_t s) {
    void *params[] = {&counter, &iters, &status};
    return hipLaunchCooperativeKernel((const void *)k_barrier_probe, dim3(num_wg), dim3(256), params,
                                      0, s);
}

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
    size_t words = bytes / 4;
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks_for(words)), dim3(kT), 0, s, (uint32_t *)p, words);
    return hipGetLastError();
}

hipError_t launch_gather_candidates(const float *xyz, int B, int N, int Nc, int start, float *cxyz,
                                    hipStream_t s) {
    hipLaunchKernelGGL(k_gather_candidates, dim3(blocks_for(Nc), B), dim3(kT), 0, s, xyz, N, Nc,
                       start, wrap_point(N, Nc, start), cxyz);
    return hipGetLastError();
}

hipError_t launch_map_candidates(const int32_t *loc, long loc_stride, int B, int N, int Nc,
                                 int start, int k, int32_t *idx, long idx_stride, hipStream_t s) {
    hipLaunchKernelGGL(k_map_candidates, dim3(blocks_for(k), B), dim3(kT), 0, s, loc, loc_stride, N,
                       Nc, start, wrap_point(N, Nc, start), k, idx, idx_stride);
    return hipGetLastError();
}

hipError_t launch_fill(int B, int N, int k, int R, int32_t *idx, long idx_stride, uint32_t *bitmap,
                       hipStream_t s) {
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill, dim3(B), dim3(1024), 0, s, N, k, R, idx, idx_stride, bitmap);
    return hipGetLastError();
}

hipError_t launch_perm_candidates(const float *xyz, int B, int N, int Nc, int start, uint64_t seed,
                                  uint32_t *bitmap, int32_t *cand, float *cxyz, int *spos,
                                  hipStream_t s) {
    const size_t words = (size_t)B * ((N + 31) / 32);
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks_for(words)), dim3(kT), 0, s, bitmap, words);
    hipLaunchKernelGGL(k_perm_mark, dim3(blocks_for(Nc), B), dim3(kT), 0, s, N, Nc, seed, bitmap);
    hipLaunchKernelGGL(k_perm_compact, dim3(B), dim3(1024), 0, s, xyz, N, Nc, start, seed, bitmap, cand,
                       cxyz, spos);
    return hipGetLastError();
}

hipError_t launch_fill_perm(int B, int N, int k, int R, uint64_t seed, int32_t *idx, long idx_stride,
                            uint32_t *bitmap, hipStream_t s) {
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_perm, dim3(B), dim3(1024), 0, s, N, k, R, seed, idx, idx_stride, bitmap);
    return hipGetLastError();
}

hipError_t launch_gather_points(const float *xyz, int B, int N, const int32_t *sel, long sel_stride,
                                int S, float *dst, hipStream_t s) {
    hipLaunchKernelGGL(k_gather_points, dim3(blocks_for(S), B), dim3(kT), 0, s, xyz, N, sel,
                       sel_stride, S, dst);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const float *rows, int B, int N, int C, const int32_t *sel,
                              long sel_stride, int S, float *out, hipStream_t s) {
    hipLaunchKernelGGL(k_gather_rows, dim3(blocks_for((size_t)S * C), B), dim3(kT), 0, s, rows, N, C,
                       sel, sel_stride, S, out);
    return hipGetLastError();
}

hipError_t launch_compose(const int32_t *prev, long prev_stride, const int32_t *loc, long loc_stride,
                          int B, int S, int32_t *out, long out_stride, hipStream_t s) {
    hipLaunchKernelGGL(k_compose, dim3(blocks_for(S), B), dim3(kT), 0, s, prev, prev_stride, loc,
                       loc_stride, S, out, out_stride);
    return hipGetLastError();
}

hipError_t launch_copy_prefix(const int32_t *src, long src_stride, int B, int S, int32_t *out,
                              long out_stride, hipStream_t s) {
    hipLaunchKernelGGL(k_copy_prefix, dim3(blocks_for(S), B), dim3(kT), 0, s, src, src_stride, S,
                       out, out_stride);
    return hipGetLastError();
}

}  // namespace ffps
