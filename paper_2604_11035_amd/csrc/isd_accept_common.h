// Device helpers shared by the acceptance kernels (gfx950): slice statistics of a logit row, the
// streaming row-statistics kernel, Philox4x32-10, the uniform / Gumbel maps and the 64-bit arg-max key.
#pragma once
#include "idlm_common.h"
#include <limits.h>

namespace idlm {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// Sums of exponentials of a row at temperature T are kept in base 2: with k = log2(e) / T,
// z = sum 2^(l*k - ref_k(m, k)) = sum exp((l - m) / T).  k = kLog2e is T = 1.
__device__ __forceinline__ float ref_k(float m, float k)
{
#pragma clang fp contract(off)
    return (m == -INFINITY) ? 0.f : m * k;
}

__device__ __forceinline__ float rescale_k(float m_old, float r_new, float k)
{
#pragma clang fp contract(off)
    return (m_old == -INFINITY) ? 0.f : fast_exp2(m_old * k - r_new);
}

struct RowPartial {   // statistics of one slice of one logit row
    float m;          // maximum (true value, compared exactly)
    float z;          // sum of 2^(l*k - ref_k(m, k))
    int arg;          // lowest index attaining m (INT_MAX if the slice is empty)
    float m2;         // a value attained by an element other than `arg`, or -inf: the largest of the other
                      // threads' maxima, a lower bound of the second-largest logit that costs nothing per element
};

// (m, m2) of the union of two disjoint element sets, to be called before m is updated
__device__ __forceinline__ float combine_second(float m, float m2, float mo, float m2o)
{
    return fmaxf(fmaxf(m2, m2o), fminf(m, mo));
}

// Best (score, index) of a sampled row as one 64-bit key whose unsigned order is "higher score
// first, then lower index": workgroups of a row combine with a single atomic max, no fences.
__device__ __forceinline__ unsigned long long sample_key(float score, int idx)
{
    const uint32_t bits = __float_as_uint(score);
    const uint32_t ordered = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    return ((unsigned long long)ordered << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)idx);
}

// ---- reductions ---------------------------------------------------------------------------

__device__ __forceinline__ void combine_stats(float& m, float& z, int& a, float m2, float z2, int a2, float k = kLog2e)
{
    const float mm = fmaxf(m, m2);
    const float r = ref_k(mm, k);
    z = z * rescale_k(m, r, k) + z2 * rescale_k(m2, r, k);
    a = (m2 > m) ? a2 : ((m > m2) ? a : min(a, a2));
    m = mm;
}

__device__ __forceinline__ void combine_best(float& s, int& i, float s2, int i2)
{
    if (s2 > s || (s2 == s && i2 < i)) { s = s2; i = i2; }
}

// ---- logit rows in fp32 or bf16 --------------------------------------------------------------
// A row is streamed in 16-byte vectors: 4 fp32 values, or 8 bf16 values that widen to fp32 exactly
// (a bf16 is the upper half of the fp32 with the same value).

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <bool BF16> struct LogitVec;

template <> struct LogitVec<false> {
    static constexpr int N = 4;
    typedef f32x4 raw;
    __device__ static __forceinline__ void unpack(const raw& r, float (&v)[4])
    {
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    }
    __device__ static __forceinline__ raw minus_inf() { return raw{-INFINITY, -INFINITY, -INFINITY, -INFINITY}; }
    __device__ static __forceinline__ float element(const void* base, size_t i)
    {
        return static_cast<const float*>(base)[i];
    }
};

template <> struct LogitVec<true> {
    static constexpr int N = 8;
    typedef u32x4 raw;
    __device__ static __forceinline__ void unpack(const raw& r, float (&v)[8])
    {
        v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xFFFF0000u);
        v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xFFFF0000u);
        v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xFFFF0000u);
        v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
    __device__ static __forceinline__ raw minus_inf() { return raw{0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u}; }
    __device__ static __forceinline__ float element(const void* base, size_t i)
    {
        return __uint_as_float((uint32_t)static_cast<const uint16_t*>(base)[i] << 16);
    }
};

// ---- pass 1: row statistics ---------------------------------------------------------------

template <int UNROLL, bool BF16 = false>
__global__ __launch_bounds__(256) void isd_row_stats_kernel(const void* __restrict__ logits, int V,
                                                            int chunk, int nsplit, int S,
                                                            RowPartial* __restrict__ stats, float k)
{
    typedef LogitVec<BF16> LV;
    typedef typename LV::raw raw_t;
    constexpr int N = LV::N;
    const int row = blockIdx.x / nsplit;
    const int c = blockIdx.x - row * nsplit;
    const int tid = threadIdx.x;
    const raw_t* __restrict__ pv = reinterpret_cast<const raw_t*>(
        static_cast<const char*>(logits) + (size_t)row * V * (16 / N));
    const int fbeg = (c * chunk) / N;
    const int fend = min(V, (c + 1) * chunk) / N;

    float m = -INFINITY;   // running maximum of this thread's elements
    float z = 0.f;         // sum of 2^(l*k - ref_k(m, k))
    int argv = -1;         // index of the vector that holds the first occurrence of m

    // One batch of UNROLL vectors per thread, all loads issued before the first use.  The last batch
    // of a slice is ragged: its missing vectors read as -inf, which changes neither the maximum nor
    // the sum (2^-inf = 0), so the tail keeps as many loads in flight as the body.
    int f = fbeg + tid;
    auto batch = [&](const bool full) {
        raw_t v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            v[u] = (full || f + u * 256 < fend) ? __builtin_nontemporal_load(pv + f + u * 256) : LV::minus_inf();
        float newm = m;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float e[N];
            LV::unpack(v[u], e);
            float bm = e[0];
#pragma unroll
            for (int i = 1; i < N; ++i) bm = fmaxf(bm, e[i]);
            if (bm > newm) { newm = bm; argv = f + u * 256; }
        }
        const float r = ref_k(newm, k);
        float acc = z * rescale_k(m, r, k);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            // bf16: unpacked again from the loaded vector (two instructions per pair) rather than kept
            // from the maximum loop, which would double the registers and cost two waves per SIMD
            if constexpr (BF16) asm volatile("" : "+v"(v[u]));
            float e[N];
            LV::unpack(v[u], e);
#pragma unroll
            for (int i = 0; i < N; ++i) acc += fast_exp2(fmaf(e[i], k, -r));
        }
        z = acc;
        m = newm;
    };
    for (; f + (UNROLL - 1) * 256 < fend; f += UNROLL * 256) batch(true);
    if (f < fend) batch(false);

    // which component of that vector was first to reach m
    int arg = INT_MAX;
    if (argv >= 0) {
        float e[N];
        LV::unpack(pv[argv], e);
        int lane = N - 1;
#pragma unroll
        for (int i = N - 2; i >= 0; --i) lane = (e[i] == m) ? i : lane;
        arg = argv * N + lane;
    }

    // wavefront reduction, then the four wavefronts through LDS
    float second = -INFINITY;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float mo = __shfl_xor(m, off);
        const float zo = __shfl_xor(z, off);
        const int ao = __shfl_xor(arg, off);
        const float so = __shfl_xor(second, off);
        second = combine_second(m, second, mo, so);
        combine_stats(m, z, arg, mo, zo, ao, k);
    }
    __shared__ float sm[4], sz[4], ss[4];
    __shared__ int sa[4];
    const int w = tid >> 6;
    if ((tid & 63) == 0) { sm[w] = m; sz[w] = z; sa[w] = arg; ss[w] = second; }
    __syncthreads();
    if (tid == 0) {
        for (int q = 1; q < 4; ++q) {
            second = combine_second(m, second, sm[q], ss[q]);
            combine_stats(m, z, arg, sm[q], sz[q], sa[q], k);
        }
        RowPartial out;
        out.m = m; out.z = z; out.arg = arg; out.m2 = second;
        stats[(size_t)row * nsplit + c] = out;
    }
}

// ---- counter-based random numbers (Philox4x32-10, Salmon et al. SC'11) --------------------

__device__ __forceinline__ uint4 philox4x32_10(uint4 ctr, uint2 key)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        // one 32 x 32 -> 64 bit multiply-add instruction per product instead of separate high and low multiplies
        const unsigned long long p0 = (unsigned long long)0xD2511F53u * ctr.x;
        const unsigned long long p1 = (unsigned long long)0xCD9E8D57u * ctr.z;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        ctr = make_uint4(hi1 ^ ctr.y ^ key.x, lo1, hi0 ^ ctr.w ^ key.y, lo0);
        key.x += 0x9E3779B9u;
        key.y += 0xBB67AE85u;
    }
    return ctr;
}

// 32 bits -> u = (2*(x>>9)+1) * 2^-24: an odd 24-bit numerator, exact in fp32, inside (0,1)
__device__ __forceinline__ float unit_uniform(uint32_t x)
{
    return (float)(2u * (x >> 9) + 1u) * 5.9604644775390625e-8f;
}

// g = -ln(-ln u).  The inner logarithm must be accurate relative to its result for u close to 1
// (the large noise values that decide the arg-max), so it is the library logf; the outer one only
// needs absolute accuracy and is the hardware log2.
__device__ __forceinline__ float gumbel(uint32_t x)
{
    const float t = -logf(unit_uniform(x));
    return -0.69314718056f * __builtin_amdgcn_logf(t);
}

// Pruning of the Gumbel-max, exact.  Let c be a score that the winner is known to reach (a "floor").
// Element i wins only if l_i + g_i > c, i.e. -ln u_i < e^(l_i - c), which needs 1 - u_i < e^(l_i - c)
// (because e^-x >= 1 - x).  1 - u_i is exact for the 24-bit uniform, so an element whose 1 - u_i is not
// below e^(l_i - c) (taken 0.7 % larger: covers the rounding of the exponential, of the noise and of the
// sums) is dropped before its two logarithms; on average only e^(LSE - c) = O(1) elements of a row
// survive.  Before even drawing the Philox block of four elements: the noise lies in
// [-ln(-ln 2^-24), -ln(-ln(1 - 2^-24))] = [-2.8115, 16.6355], so four logits all more than 16.7 below the
// floor (a score) cannot win whatever their uniforms are.
// The floor starts as the score of the row's arg-max element (computed by the chain kernel with the same
// arithmetic), or, when the arg-max is the excluded token (the usual rejection), as m2 - 2.82 with m2 the
// value of another element that the row-statistics pass brings along (RowPartial::m2), and rises with the
// thread's own best.  Every dropped element would have failed the comparison it skips, so the sequence
// of updates, and with it the result, is that of the full evaluation.
constexpr float kNoiseMax = 16.7f;
constexpr float kGumbelMin = -2.82f;

// 1 - u for u = (2*(x >> 9) + 1) * 2^-24: again an odd 24-bit numerator, exact in fp32
__device__ __forceinline__ float one_minus_uniform(uint32_t x)
{
    return (float)(2u * (0x7FFFFFu - (x >> 9)) + 1u) * 5.9604644775390625e-8f;
}

// ---- launch shapes shared by the acceptance entry points (host) ---------------------------------

struct AcceptPlan {
    int chunk;    // vocabulary elements per workgroup in pass 1 (multiple of 1024)
    int nsplit;   // slices per row in pass 1
    int gchunk;   // vocabulary elements per workgroup in the Gumbel pass (multiple of 1024)
    int nsb;      // workgroups per sequence in pass 2
};

static inline AcceptPlan make_plan(int32_t B, int32_t S, int32_t V)
{
    AcceptPlan p;
    const int64_t rows = (int64_t)B * S;
    // One round of about two workgroups per compute unit (512 on this part) is what streams fastest: a
    // workgroup keeps 64 KB in flight, every further slice of a row costs a block reduction, and a launch
    // of more workgroups than can be resident ends in a round of stragglers.  So a workgroup streams a
    // whole row from about 400 rows on, and fewer rows are cut into round(512 / rows) slices (measured on
    // 152K-element rows: 512 rows 54 us whole against 65 us in eight slices; 1024 rows 100 against 112 us
    // in four; 128 rows best in four slices, 256 rows in two).
    int64_t nsplit = rows > 0 ? (512 + rows / 2) / rows : 1;
    int64_t max_split = ((int64_t)V + 4095) / 4096;
    if (nsplit > max_split) nsplit = max_split;
    if (nsplit < 1) nsplit = 1;
    int64_t chunk = (((int64_t)V + nsplit - 1) / nsplit + 1023) / 1024 * 1024;
    p.chunk = (int)chunk;
    p.nsplit = (int)(((int64_t)V + chunk - 1) / chunk);
    int64_t nsb = ((int64_t)V + 4095) / 4096;     // 4K elements of Philox + logs per workgroup
    if (nsb > 64) nsb = 64;
    int64_t gchunk = (((int64_t)V + nsb - 1) / nsb + 1023) / 1024 * 1024;
    p.gchunk = (int)gchunk;
    p.nsb = (int)(((int64_t)V + gchunk - 1) / gchunk);
    return p;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace idlm
