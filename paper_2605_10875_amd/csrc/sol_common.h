// Device-side helpers shared by the gfx950 kernels: bf16 <-> fp32, element I/O, wave / block
// reductions, exact k-th-largest selection (radix select on order-preserving keys) and the
// per-token fake-quantiser.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sol {

typedef uint16_t bf16_t;   // raw bfloat16 bits

// Per-row decoded action (one 16-byte load per kernel that needs it).
struct RowAct {
    uint32_t keep_num, keep_den;  // attention keep fraction
    int32_t  m;                   // MLP channels kept = ceil(rho * d_ff), in [1, d_ff]
    int32_t  bits;                // activation bit-width; >= 16 bypasses the quantiser
};

enum { FLAG_BAD_ACTION = 1, FLAG_CACHE_OVERFLOW = 2, FLAG_BAD_TOKEN = 4 };

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest, ties to even (v_cvt_pk_bf16_f32 on gfx950)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
// two values -> one dword, `a` in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ float ld(const float *p) { return *p; }
__device__ __forceinline__ float ld(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st(float *p, float v) { *p = v; }
__device__ __forceinline__ void st(bf16_t *p, float v) { *p = f32_to_bf16(v); }
// value after a round trip through the storage type
__device__ __forceinline__ float rnd(float v, const float *) { return v; }
__device__ __forceinline__ float rnd(float v, const bf16_t *) { return bf16_to_f32(f32_to_bf16(v)); }

// 16-byte vector of elements: 4 floats or 8 bf16
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    float4 raw;
    __device__ __forceinline__ void load(const float *p) { raw = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ void store(float *p) const { *reinterpret_cast<float4 *>(p) = raw; }
    __device__ __forceinline__ float get(int i) const { return i == 0 ? raw.x : i == 1 ? raw.y : i == 2 ? raw.z : raw.w; }
    __device__ __forceinline__ void unpack(float *f) const { f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w; }
    __device__ __forceinline__ void pack(const float *f) { raw = make_float4(f[0], f[1], f[2], f[3]); }
};
template <> struct Vec16<bf16_t> {
    static constexpr int N = 8;
    uint4 raw;
    __device__ __forceinline__ void load(const bf16_t *p) { raw = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void store(bf16_t *p) const { *reinterpret_cast<uint4 *>(p) = raw; }
    __device__ __forceinline__ void unpack(float *f) const
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i]     = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ __forceinline__ void pack(const float *f)
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)f32_to_bf16(f[2 * i]) | ((uint32_t)f32_to_bf16(f[2 * i + 1]) << 16);
        raw = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// ---- reductions (fixed shuffle pattern => deterministic) -----------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ int wave_sum_i(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Block-wide sum / max. `red` is LDS scratch of at least BLOCK/64 floats. All threads get the
// result. Contains two barriers, so `red` may be reused right after the call.
template <int BLOCK> __device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < BLOCK / 64; ++i) t += red[i];
    __syncthreads();
    return t;
}
template <int BLOCK> __device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int i = 1; i < BLOCK / 64; ++i) t = fmaxf(t, red[i]);
    __syncthreads();
    return t;
}

// ---- order-preserving integer keys ----------------------------------------------------------
// float -> uint32 such that a < b  <=>  key(a) < key(b)   (-0 and +0 map to neighbouring keys;
// scores are compared as IEEE values by the definition, so fold -0 into +0 first)
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t u = __float_as_uint(s + 0.0f);      // -0 + 0 = +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
// |a| as key: non-negative floats order like their bit patterns
__device__ __forceinline__ uint32_t mag_key(float a) { return __float_as_uint(a) & 0x7FFFFFFFu; }

// ---- exact k-th largest of n keys -----------------------------------------------------------
// keyfn(i) yields key i (i in [0,n)). 1 <= k <= n. On return (uniform across the block):
//   thr   = the k-th largest key,
//   quota = how many of the keys equal to thr belong to the k largest (>= 1),
//   n_eq  = how many keys equal thr in total.
// hist: LDS int[256]; sh: LDS int[4]. Every thread of the block must call it.
template <int BLOCK, typename KeyFn>
__device__ __forceinline__ void block_radix_select(KeyFn keyfn, int n, int k, int *hist, int *sh,
                                                   uint32_t &thr, int &quota, int &n_eq)
{
    const int tid = threadIdx.x;
    uint32_t prefix = 0, mask = 0;
    int remaining = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = tid; i < 256; i += BLOCK) hist[i] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += BLOCK) {
            const uint32_t u = keyfn(i);
            if ((u & mask) == prefix) atomicAdd(&hist[(u >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns bins 255-4l .. 252-4l; scan from the largest digit downwards
            const int b0 = 255 - 4 * tid;
            const int c0 = hist[b0], c1 = hist[b0 - 1], c2 = hist[b0 - 2], c3 = hist[b0 - 3];
            const int s = c0 + c1 + c2 + c3;
            int incl = s;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o, 64);
                if (tid >= o) incl += t;
            }
            const int excl = incl - s;
            if (excl < remaining && remaining <= incl) {
                const int r = remaining - excl;
                int bin, above, cnt;
                if (r <= c0) { bin = b0; above = 0; cnt = c0; }
                else if (r <= c0 + c1) { bin = b0 - 1; above = c0; cnt = c1; }
                else if (r <= c0 + c1 + c2) { bin = b0 - 2; above = c0 + c1; cnt = c2; }
                else { bin = b0 - 3; above = c0 + c1 + c2; cnt = c3; }
                sh[0] = bin;
                sh[1] = r - above;
                sh[2] = cnt;
            }
        }
        __syncthreads();
        prefix |= ((uint32_t)sh[0]) << shift;
        mask |= 0xFFu << shift;
        remaining = sh[1];
        n_eq = sh[2];
        __syncthreads();
    }
    thr = prefix;
    quota = remaining;
}

// Among the keys equal to thr, the `quota` of lowest index win. Returns the largest index J such
// that exactly `quota` keys equal to thr have index <= J (uniform across the block).
// Only needed when quota < n_eq. wcnt: LDS int[BLOCK/64]; sh: LDS int[4].
template <int BLOCK, typename KeyFn>
__device__ __forceinline__ int block_tie_cutoff(KeyFn keyfn, int n, uint32_t thr, int quota, int *wcnt, int *sh)
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int taken = 0;
    if (tid == 0) sh[3] = n - 1;
    __syncthreads();
    for (int base = 0; base < n; base += BLOCK) {
        const int i = base + tid;
        const bool tie = (i < n) && (keyfn(i) == thr);
        const unsigned long long bal = __ballot(tie);
        const int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wcnt[w] = __popcll(bal);
        __syncthreads();
        int wave_off = 0, total = 0;
#pragma unroll
        for (int j = 0; j < BLOCK / 64; ++j) {
            const int c = wcnt[j];
            if (j < w) wave_off += c;
            total += c;
        }
        if (tie && taken + wave_off + before + 1 == quota) sh[3] = i;
        __syncthreads();
        taken += total;
        if (taken >= quota) break;     // uniform
    }
    __syncthreads();
    return sh[3];
}

// ---- wave-wide reductions on DPP (no LDS traffic); all 64 lanes must be active -------------------
// quad swaps, half-mirror and mirror reduce each row of 16 lanes; row_bcast15 / row_bcast31 fold
// the four rows into lane 63, which is broadcast through a scalar register.
#define SOL_DPP(T, x, ident, ctrl, rmask)                                                                       \
    __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, ident), __builtin_bit_cast(int, x), \
                                                      ctrl, rmask, 0xF, false))
template <typename T, typename Op> __device__ __forceinline__ T wave_reduce_dpp(T v, T ident, Op op)
{
    v = op(v, SOL_DPP(T, v, ident, 0xB1, 0xF));     // quad_perm [1,0,3,2]
    v = op(v, SOL_DPP(T, v, ident, 0x4E, 0xF));     // quad_perm [2,3,0,1]
    v = op(v, SOL_DPP(T, v, ident, 0x141, 0xF));    // row_half_mirror
    v = op(v, SOL_DPP(T, v, ident, 0x140, 0xF));    // row_mirror
    v = op(v, SOL_DPP(T, v, ident, 0x142, 0xA));    // row_bcast15 into rows 1 and 3
    v = op(v, SOL_DPP(T, v, ident, 0x143, 0xC));    // row_bcast31 into rows 2 and 3
    return __builtin_bit_cast(T, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
struct OpMaxU { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };
struct OpMinU { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a < b ? a : b; } };
struct OpAddF { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) { return wave_reduce_dpp<uint32_t>(v, 0u, OpMaxU()); }
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) { return wave_reduce_dpp<uint32_t>(v, 0xFFFFFFFFu, OpMinU()); }
__device__ __forceinline__ float wave_sum_dpp(float v) { return wave_reduce_dpp<float>(v, 0.f, OpAddF()); }

// inverse of score_key
__device__ __forceinline__ float score_unkey(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// Keys equal to thr: the first `quota` of them in column order (column = 256*j + 4*lane + e) stay, the
// others are overwritten with 0 so that afterwards  kept <=> key >= thr. Returns the number of keys
// equal to thr that this wave held (before the overwrite).
template <int SLOTS>
__device__ __forceinline__ int wave_tie_fixup(uint32_t (&key)[SLOTS], int n, uint32_t thr, int quota, int lane)
{
    constexpr int NJ = SLOTS / 4;
    (void)lane;
    int total = 0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (256 * j < n) {
            int below = 0, here = 0;                    // ties in lower lanes of this j / in all lanes
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned long long bal = __ballot(key[4 * j + e] == thr);
                below = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, below));
                here += __popcll(bal);
            }
            int mine = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool tie = key[4 * j + e] == thr;
                if (tie && below + mine >= quota) key[4 * j + e] = 0u;     // loses the tie
                mine += tie;
            }
            total += here;
            quota = quota > here ? quota - here : 0;
        }
        __builtin_amdgcn_sched_barrier(0);              // keep the slot groups sequential: low register pressure
    }
    return total;
}

// 64-bit lane mask of (key >= pivot) into a scalar register pair of the compiler's choice: unlike the
// default VCC form, several of these can be in flight before the first population count reads one
__device__ __forceinline__ unsigned long long mask_ge_u32(uint32_t key, uint32_t pivot)
{
    unsigned long long m;
    asm("v_cmp_ge_u32_e64 %0, %1, %2" : "=s"(m) : "v"(key), "s"(pivot));
    return m;
}

// number of keys >= pivot in the first NG groups of 256 columns (columns >= n carry key 0 and pivot >= 1)
template <int SLOTS, int NG>
__device__ __forceinline__ int wave_count_ge_g(const uint32_t (&key)[SLOTS], uint32_t pivot)
{
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < NG; ++j) {
        const unsigned long long m0 = mask_ge_u32(key[4 * j + 0], pivot), m1 = mask_ge_u32(key[4 * j + 1], pivot);
        const unsigned long long m2 = mask_ge_u32(key[4 * j + 2], pivot), m3 = mask_ge_u32(key[4 * j + 3], pivot);
        cnt += (__popcll(m0) + __popcll(m1)) + (__popcll(m2) + __popcll(m3));
    }
    return cnt;
}

// number of keys >= pivot held by the wave (pivot wave-uniform)
template <int SLOTS>
__device__ __forceinline__ int wave_count_ge(const uint32_t (&key)[SLOTS], int n, uint32_t pivot)
{
    pivot = (uint32_t)__builtin_amdgcn_readfirstlane((int)pivot);
    constexpr int NJ = SLOTS / 4;
    const int ng = (n + 255) >> 8;
    if constexpr (NJ <= 4) {
        if (ng <= 1) return wave_count_ge_g<SLOTS, 1>(key, pivot);
        if constexpr (NJ >= 2) if (ng == 2) return wave_count_ge_g<SLOTS, 2>(key, pivot);
        if constexpr (NJ >= 3) if (ng == 3) return wave_count_ge_g<SLOTS, 3>(key, pivot);
        return wave_count_ge_g<SLOTS, NJ>(key, pivot);
    } else {
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            if (256 * j < n) {
                const unsigned long long m0 = mask_ge_u32(key[4 * j + 0], pivot), m1 = mask_ge_u32(key[4 * j + 1], pivot);
                const unsigned long long m2 = mask_ge_u32(key[4 * j + 2], pivot), m3 = mask_ge_u32(key[4 * j + 3], pivot);
                cnt += (__popcll(m0) + __popcll(m1)) + (__popcll(m2) + __popcll(m3));
            }
        return cnt;
    }
}

// the same for two rows with their own pivots, interleaved
template <int SLOTS, int NG>
__device__ __forceinline__ void wave_count_ge2_g(const uint32_t (&keya)[SLOTS], const uint32_t (&keyb)[SLOTS], uint32_t pa,
                                                 uint32_t pb, int &ca, int &cb)
{
    ca = 0; cb = 0;
#pragma unroll
    for (int j = 0; j < NG; ++j) {
        const unsigned long long a0 = mask_ge_u32(keya[4 * j + 0], pa), a1 = mask_ge_u32(keya[4 * j + 1], pa);
        const unsigned long long b0 = mask_ge_u32(keyb[4 * j + 0], pb), b1 = mask_ge_u32(keyb[4 * j + 1], pb);
        const unsigned long long a2 = mask_ge_u32(keya[4 * j + 2], pa), a3 = mask_ge_u32(keya[4 * j + 3], pa);
        const unsigned long long b2 = mask_ge_u32(keyb[4 * j + 2], pb), b3 = mask_ge_u32(keyb[4 * j + 3], pb);
        ca += (__popcll(a0) + __popcll(a1)) + (__popcll(a2) + __popcll(a3));
        cb += (__popcll(b0) + __popcll(b1)) + (__popcll(b2) + __popcll(b3));
    }
}

// ---- wave-level exact top-b (keys in registers) ---------------------------------------------------
// A wave holds SLOTS keys per lane; element (j, e) of lane l is column 256*j + 4*l + e (j < SLOTS/4,
// e < 4). Columns >= n carry key 0, which is below the key of every real score. Finds the b largest
// (1 <= b < n), equal keys going to the lower columns, and returns a threshold `thr` such that after
// the call   kept  <=>  key >= thr   (keys equal to thr that lose the tie are overwritten with 0).
// kmin / kmax: smallest / largest valid key of the row (wave-uniform).
// The search bisects [kmin, kmax] counting with ballots and stops as soon as exactly b keys lie at
// or above the pivot, about log2 of the key range over the gap at the threshold steps.
template <int SLOTS>
__device__ __forceinline__ uint32_t wave_select_topk(uint32_t (&key)[SLOTS], int n_in, int b_in, uint32_t kmin,
                                                     uint32_t kmax, int lane)
{
    // every search variable is wave-uniform: scalar registers, scalar control flow around ballots
    const int n = __builtin_amdgcn_readfirstlane(n_in), b = __builtin_amdgcn_readfirstlane(b_in);
    uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)kmin);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)kmax);
    // invariant: count(key >= lo) >= b  and  count(key >= hi + 1) < b
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo + 1u) >> 1);
        const int cnt = wave_count_ge<SLOTS>(key, n, mid);
        if (cnt == b) return mid;                       // exactly b keys at or above the pivot
        if (cnt > b) lo = mid; else hi = mid - 1u;
    }
    const uint32_t thr = lo;                            // the b-th largest key; ties decide the rest
    const int n_gt = (thr == 0xFFFFFFFFu) ? 0 : wave_count_ge<SLOTS>(key, n, thr + 1u);
    wave_tie_fixup<SLOTS>(key, n, thr, b - n_gt, lane);
    return thr;
}

// Two rows searched in one loop: while both searches are open every step counts both rows, so the two
// ballot -> count -> compare chains overlap. Leaves each row's bracket [lo, hi] (invariant of
// wave_select_topk) and whether it stopped with exactly b keys at or above lo (then lo is the threshold).
template <int SLOTS>
__device__ __forceinline__ void wave_bisect2(const uint32_t (&keya)[SLOTS], const uint32_t (&keyb)[SLOTS], int na_in, int nb_in,
                                             int ba_in, int bb_in, uint32_t &lo_a, uint32_t &hi_a, uint32_t &lo_b,
                                             uint32_t &hi_b, bool &exact_a, bool &exact_b)
{
    constexpr int NJ = SLOTS / 4;
    const int na = __builtin_amdgcn_readfirstlane(na_in), nb = __builtin_amdgcn_readfirstlane(nb_in);
    const int ba = __builtin_amdgcn_readfirstlane(ba_in), bb = __builtin_amdgcn_readfirstlane(bb_in);
    const int nm = na > nb ? na : nb;
    uint32_t loa = (uint32_t)__builtin_amdgcn_readfirstlane((int)lo_a), hia = (uint32_t)__builtin_amdgcn_readfirstlane((int)hi_a);
    uint32_t lob = (uint32_t)__builtin_amdgcn_readfirstlane((int)lo_b), hib = (uint32_t)__builtin_amdgcn_readfirstlane((int)hi_b);
    exact_a = exact_b = false;
    const int ng = (nm + 255) >> 8;
    while (loa < hia && lob < hib) {
        const uint32_t mida = loa + ((hia - loa + 1u) >> 1), midb = lob + ((hib - lob + 1u) >> 1);
        int ca, cb;
        if constexpr (NJ <= 4) {
            if (ng <= 1) wave_count_ge2_g<SLOTS, 1>(keya, keyb, mida, midb, ca, cb);
            else if (NJ >= 2 && ng == 2) wave_count_ge2_g<SLOTS, NJ >= 2 ? 2 : NJ>(keya, keyb, mida, midb, ca, cb);
            else if (NJ >= 3 && ng == 3) wave_count_ge2_g<SLOTS, NJ >= 3 ? 3 : NJ>(keya, keyb, mida, midb, ca, cb);
            else wave_count_ge2_g<SLOTS, NJ>(keya, keyb, mida, midb, ca, cb);
        } else {
            ca = wave_count_ge<SLOTS>(keya, na, mida);
            cb = wave_count_ge<SLOTS>(keyb, nb, midb);
        }
        if (ca == ba) { loa = hia = mida; exact_a = true; } else if (ca > ba) loa = mida; else hia = mida - 1u;
        if (cb == bb) { lob = hib = midb; exact_b = true; } else if (cb > bb) lob = midb; else hib = midb - 1u;
    }
    lo_a = loa; hi_a = hia; lo_b = lob; hi_b = hib;
}

// ---- per-token symmetric fake-quantiser ------------------------------------------------------
// q_max = 2^(bits-1)-1, s = absmax / q_max, z_hat = clamp(rint(z / s), -q_max, q_max) * s,
// all in IEEE fp32 (true division, round half to even).
__device__ __forceinline__ float fq_qmax(int bits) { return (float)((1 << (bits - 1)) - 1); }
__device__ __forceinline__ float fq_code(float z, float s, float qmax)
{
    float c = rintf(z / s);
    c = fminf(fmaxf(c, -qmax), qmax);
    return c;
}

__device__ __forceinline__ int budget_ceil(uint32_t num, uint32_t den, int n)
{
    const unsigned long long x = (unsigned long long)num * (unsigned long long)n + den - 1ull;
    // the 32-bit quotient is an order of magnitude fewer instructions than the 64-bit one
    unsigned long long b = (x >> 32) == 0ull ? (unsigned long long)((uint32_t)x / den) : x / den;
    if (b < 1ull) b = 1ull;
    if (b > (unsigned long long)n) b = (unsigned long long)n;
    return (int)b;
}

}  // namespace sol
