// Attention with per-query budgeted key selection.
//
// k_attn_rows: one workgroup per (query row, group of HPB query heads that share a KV head).
//   1. scores s_j = (q . k_j) / sqrt(dh) over the allowed cache positions j in [0, pos]   -> LDS (fp32)
//   2. budget b = ceil(kappa * n); b < n: exact b-th largest score by radix select, ties to the
//      lower position; b = n: dense
//   3. softmax over the kept keys (dropped keys contribute exp(-inf) = 0)
//   4. o = sum_j p_j v_j, reading only V rows kept by at least one of the HPB heads
// K is streamed once per workgroup (HPB heads share it), V rows are gathered. This is the any-shape /
// fp32 path, and the only one that knows the other key-selection rules of the method (Appendix "Quest
// masking"):
//   - sink / window keys: the first n_sink and the last n_window allowed keys are always kept and
//     count against the budget (the selection sees them with the largest possible key);
//   - pages of S > 1 contiguous keys: a page's score is the upper bound sum_c max(q_c max_c, q_c min_c)
//     over the channel-wise extremes of its allowed keys; the top ceil(b / S) pages are kept whole
//     (ties to the lower page) together with the forced keys.
#include <type_traits>
#include "sol_internal.h"

namespace sol {

struct ScoreKeyLds {
    const float *row;
    __device__ __forceinline__ uint32_t operator()(int i) const { return score_key(row[i]); }
};

// selection key of key j when keys [0, sink_end) and [win_begin, n) are forced
struct ForcedKeyLds {
    const float *row;
    int sink_end, win_begin;
    __device__ __forceinline__ uint32_t operator()(int i) const
    {
        return (i < sink_end || i >= win_begin) ? 0xFFFFFFFFu : score_key(row[i]);
    }
};

template <typename T, int HPB, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
k_attn_rows(const T *__restrict__ q, const T *__restrict__ kc, const T *__restrict__ vc, float *__restrict__ o32,
            const RowAct *__restrict__ ra, const int32_t *__restrict__ pos0, int Tn, int L_max, int Hq, int Hkv,
            int dh, int lpad, float scale, int *flags, AttnOpts opt, int ppad)
{
    constexpr int VEC = Vec16<T>::N;
    constexpr int NW = BLOCK / 64;
    extern __shared__ float smem[];
    float *sc = smem;                               // [HPB][lpad]
    float *ored = smem + (size_t)HPB * lpad;        // [NW][HPB][dh]
    float *pgs = ored + (size_t)NW * HPB * dh;      // [HPB][ppad] page scores (page size > 1 only)
    __shared__ int hist[256];
    __shared__ int sh[4];
    __shared__ int wcnt[NW];
    __shared__ float red[NW];

    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const int s = (int)(r / Tn), i = (int)(r % Tn);
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) {               // the sequence does not fit its cache: skipped
        if (tid == 0) atomicOr(flags, FLAG_CACHE_OVERFLOW);
        return;
    }
    const int n = p0 + i + 1;                       // allowed keys 0..pos, self included
    const int h0 = blockIdx.x * HPB;
    const int kvh = h0 / (Hq / Hkv);
    const T *kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * dh;
    const T *vbase = vc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * dh;
    const int lpk = dh / VEC;                       // lanes per key (power of two, <= 64)
    const int kpi = BLOCK / lpk;                    // keys per block iteration
    const int ks = tid / lpk, cs = tid - ks * lpk;

    // ---- 1. scores -------------------------------------------------------------------------
    float qf[HPB][VEC];
#pragma unroll
    for (int h = 0; h < HPB; ++h) {
        Vec16<T> v;
        v.load(q + r * (int64_t)(Hq * dh) + (int64_t)(h0 + h) * dh + cs * VEC);
        v.unpack(qf[h]);
    }
    for (int j0 = 0; j0 < n; j0 += kpi) {
        const int j = j0 + ks;
        float part[HPB];
#pragma unroll
        for (int h = 0; h < HPB; ++h) part[h] = 0.f;
        if (j < n) {
            Vec16<T> kv;
            kv.load(kbase + (int64_t)j * dh + cs * VEC);
            float kf[VEC];
            kv.unpack(kf);
#pragma unroll
            for (int h = 0; h < HPB; ++h)
#pragma unroll
                for (int e = 0; e < VEC; ++e) part[h] = fmaf(qf[h][e], kf[e], part[h]);
        }
        for (int o = lpk >> 1; o > 0; o >>= 1)
#pragma unroll
            for (int h = 0; h < HPB; ++h) part[h] += __shfl_xor(part[h], o, 64);
        if (cs == 0 && j < n)
#pragma unroll
            for (int h = 0; h < HPB; ++h) sc[h * lpad + j] = part[h] * scale;
    }
    const RowAct act = ra[r];
    const int b = budget_ceil(act.keep_num, act.keep_den, n);
    const int S = opt.page;
    const int n_pages = (n + S - 1) / S;
    if (S > 1 && b < n) {
        // ---- 1b. page bounds: a group of lpk lanes walks the allowed keys of one page --------------
        for (int u0 = 0; u0 < n_pages; u0 += kpi) {
            const int u = u0 + ks;
            float part[HPB];
#pragma unroll
            for (int h = 0; h < HPB; ++h) part[h] = 0.f;
            if (u < n_pages) {
                const int j0 = u * S, j1 = (j0 + S < n) ? j0 + S : n;
                float kmx[VEC], kmn[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) { kmx[e] = -INFINITY; kmn[e] = INFINITY; }
                for (int j = j0; j < j1; ++j) {
                    Vec16<T> kv;
                    kv.load(kbase + (int64_t)j * dh + cs * VEC);
                    float kf[VEC];
                    kv.unpack(kf);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) { kmx[e] = fmaxf(kmx[e], kf[e]); kmn[e] = fminf(kmn[e], kf[e]); }
                }
#pragma unroll
                for (int h = 0; h < HPB; ++h)
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        part[h] = fmaf(qf[h][e], qf[h][e] >= 0.f ? kmx[e] : kmn[e], part[h]);
            }
            for (int o = lpk >> 1; o > 0; o >>= 1)
#pragma unroll
                for (int h = 0; h < HPB; ++h) part[h] += __shfl_xor(part[h], o, 64);
            if (cs == 0 && u < n_pages)
#pragma unroll
                for (int h = 0; h < HPB; ++h) pgs[h * ppad + u] = part[h];
        }
    }
    __syncthreads();

    // ---- 2 + 3. selection and softmax numerators, head by head ------------------------------
    // forced keys: [0, sink_end) and [win_begin, n)
    const int sink_end = opt.n_sink < n ? opt.n_sink : n;
    int win_begin = n - opt.n_window;
    win_begin = win_begin < sink_end ? sink_end : win_begin;
    const int forced = sink_end + (n - win_begin);
    float inv_den[HPB];
#pragma unroll
    for (int h = 0; h < HPB; ++h) {
        float *row = sc + h * lpad;
        uint32_t thr = 0u; int J = n;                // by key (S = 1) or by page (S > 1): kept if above thr, or tied and <= J
        if (b < n) {
            int quota, n_eq;
            if (S > 1) {
                ScoreKeyLds kf{pgs + h * ppad};
                int np = (b + S - 1) / S;
                np = np < n_pages ? np : n_pages;
                J = n_pages;
                if (np < n_pages) {
                    block_radix_select<BLOCK>(kf, n_pages, np, hist, sh, thr, quota, n_eq);
                    if (quota < n_eq) J = block_tie_cutoff<BLOCK>(kf, n_pages, thr, quota, wcnt, sh);
                }
            } else if (forced == 0) {
                ScoreKeyLds kf{row};
                block_radix_select<BLOCK>(kf, n, b, hist, sh, thr, quota, n_eq);
                if (quota < n_eq) J = block_tie_cutoff<BLOCK>(kf, n, thr, quota, wcnt, sh);
            } else if (forced < n) {                 // forced keys rank first; the rest of the budget goes by score
                ForcedKeyLds kf{row, sink_end, win_begin};
                const int bb = b > forced ? b : forced;
                block_radix_select<BLOCK>(kf, n, bb, hist, sh, thr, quota, n_eq);
                if (quota < n_eq) J = block_tie_cutoff<BLOCK>(kf, n, thr, quota, wcnt, sh);
            }
        }
        auto kept = [&](int j, float sv) -> bool {
            if (b >= n) return true;
            const bool f = j < sink_end || j >= win_begin;
            if (S > 1) {
                const int u = j / S;
                const uint32_t key = score_key(pgs[h * ppad + u]);
                return f || key > thr || (key == thr && u <= J);
            }
            const uint32_t key = f ? 0xFFFFFFFFu : score_key(sv);
            return key > thr || (key == thr && j <= J);
        };
        float mx = -INFINITY;                        // over the kept keys (the best key may be dropped with its page)
        for (int j = tid; j < n; j += BLOCK) {
            const float sv = row[j];
            if (kept(j, sv)) mx = fmaxf(mx, sv);
        }
        mx = block_max<BLOCK>(mx, red);
        float den = 0.f;
        for (int j = tid; j < n; j += BLOCK) {
            const float sv = row[j];
            const float p = kept(j, sv) ? expf(sv - mx) : 0.f;
            row[j] = p;
            den += p;
        }
        den = block_sum<BLOCK>(den, red);
        inv_den[h] = 1.0f / den;
    }
    __syncthreads();

    // ---- 4. o = sum p_j v_j over rows any head kept --------------------------------------------
    float acc[HPB][VEC];
#pragma unroll
    for (int h = 0; h < HPB; ++h)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[h][e] = 0.f;
    for (int j = ks; j < n; j += kpi) {
        float p[HPB];
        bool any = false;
#pragma unroll
        for (int h = 0; h < HPB; ++h) { p[h] = sc[h * lpad + j]; any |= (p[h] != 0.f); }
        if (!any) continue;
        Vec16<T> vv;
        vv.load(vbase + (int64_t)j * dh + cs * VEC);
        float vf[VEC];
        vv.unpack(vf);
#pragma unroll
        for (int h = 0; h < HPB; ++h)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[h][e] = fmaf(p[h], vf[e], acc[h][e]);
    }
    // reduce over the key slots of a wave (lanes with equal cs), then across waves in fixed order
    for (int o = lpk; o < 64; o <<= 1)
#pragma unroll
        for (int h = 0; h < HPB; ++h)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[h][e] += __shfl_xor(acc[h][e], o, 64);
    const int w = tid >> 6, lane = tid & 63;
    if (lane < lpk) {
#pragma unroll
        for (int h = 0; h < HPB; ++h)
#pragma unroll
            for (int e = 0; e < VEC; ++e) ored[((size_t)w * HPB + h) * dh + lane * VEC + e] = acc[h][e];
    }
    __syncthreads();
    for (int idx = tid; idx < HPB * dh; idx += BLOCK) {
        const int h = idx / dh;
        float t = 0.f;
        for (int ww = 0; ww < NW; ++ww) t += ored[(size_t)ww * HPB * dh + idx];
        float id = inv_den[0];
#pragma unroll
        for (int hh = 1; hh < HPB; ++hh) if (h == hh) id = inv_den[hh];
        o32[r * (int64_t)(Hq * dh) + (int64_t)h0 * dh + idx] = t * id;
    }
}

template <typename T, int HPB, int BLOCK>
static bool launch_attn_rows_t(const void *q, const void *kc, const void *vc, float *o32, const RowAct *ra,
                               const int32_t *pos0, int n_seq, int Tn, int L_max, int Hq, int Hkv, int dh, int lpad,
                               size_t lds, int *flags, AttnOpts opt, int ppad, hipStream_t st)
{
    auto kern = k_attn_rows<T, HPB, BLOCK>;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return false;
    }
    const float scale = 1.0f / sqrtf((float)dh);
    hipLaunchKernelGGL(kern, dim3(Hq / HPB, (unsigned)((int64_t)n_seq * Tn)), dim3(BLOCK), lds, st, (const T *)q,
                       (const T *)kc, (const T *)vc, o32, ra, pos0, Tn, L_max, Hq, Hkv, dh, lpad, scale, flags, opt, ppad);
    return true;
}

bool launch_attn_rows(const void *q, const void *k_cache, const void *v_cache, int dtype, float *o32,
                      const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh,
                      int *flags, hipStream_t st, AttnOpts opt)
{
    if ((int64_t)n_seq * T <= 0) return true;
    if (opt.page < 1 || opt.n_sink < 0 || opt.n_window < 0) return false;
    const int vec = dtype == 0 ? 4 : 8;
    if (dh % vec) return false;
    const int lpk = dh / vec;
    if (lpk > 64 || (lpk & (lpk - 1))) return false;
    const int g = Hq / Hkv;
    const int lpad = (L_max + 63) & ~63;
    // long caches (decode) get 1024-thread workgroups: more loads in flight per CU
    const int block = (L_max >= 2048) ? 1024 : 256;
    const size_t budget = 150 * 1024;
    const int ppad = opt.page > 1 ? (L_max + opt.page - 1) / opt.page : 0;
    int hpb = 4;
    while (hpb > 1 && (g % hpb != 0 ||
                       (size_t)hpb * (lpad + ppad) * 4 + (size_t)(block / 64) * hpb * dh * 4 > budget)) hpb >>= 1;
    const size_t lds = (size_t)hpb * (lpad + ppad) * 4 + (size_t)(block / 64) * hpb * dh * 4;
    if (lds > budget) return false;
#define SOL_ATTN_CASE(TT, H, B)                                                                                     \
    return launch_attn_rows_t<TT, H, B>(q, k_cache, v_cache, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, dh, lpad, lds, \
                                        flags, opt, ppad, st)
    if (dtype == 0) {
        if (block == 256) { if (hpb == 4) SOL_ATTN_CASE(float, 4, 256); if (hpb == 2) SOL_ATTN_CASE(float, 2, 256); SOL_ATTN_CASE(float, 1, 256); }
        else { if (hpb == 4) SOL_ATTN_CASE(float, 4, 1024); if (hpb == 2) SOL_ATTN_CASE(float, 2, 1024); SOL_ATTN_CASE(float, 1, 1024); }
    } else {
        if (block == 256) { if (hpb == 4) SOL_ATTN_CASE(bf16_t, 4, 256); if (hpb == 2) SOL_ATTN_CASE(bf16_t, 2, 256); SOL_ATTN_CASE(bf16_t, 1, 256); }
        else { if (hpb == 4) SOL_ATTN_CASE(bf16_t, 4, 1024); if (hpb == 2) SOL_ATTN_CASE(bf16_t, 2, 1024); SOL_ATTN_CASE(bf16_t, 1, 1024); }
    }
#undef SOL_ATTN_CASE
    return false;
}


typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_a;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_a;
typedef uint32_t u32x4_a __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_a __attribute__((ext_vector_type(2)));
typedef float f32x4_a __attribute__((ext_vector_type(4)));

// =================================================================================================
// Batched bf16 attention in two kernels.
//
//   k_attn_select   per (sequence, query head, BQ query rows): all causal scores of the rows by MFMA into
//                   LDS as fp32, then per row the row maximum and -- when the budget is below the row
//                   length -- the exact threshold of the b largest scores (wave bisection on ballots).
//                   Output per (row, head): { thr, max, jstar }: a key is kept iff
//                   s > thr  or  (s == thr and key index <= jstar).
//   k_attn_pv       per (sequence, KV head, 32 query rows), one wave per query head of the group: streams
//                   K and V^T chunks through LDS once for all heads of the group, recomputes the scores
//                   with the same MFMA sequence (bit-identical to the first kernel's), applies the
//                   threshold, and accumulates softmax numerators times V flash-style with scores and
//                   probabilities never leaving registers (the row maximum is already known, so there
//                   is no running rescale).
// Both compute a score tile as S^T = K Q^T, so a lane owns one query and four keys per tile; in
// k_attn_pv the keys of a 32-key chunk are assigned to MFMA rows such that each lane group ends up
// with 8 consecutive keys, which is exactly the A operand of the P V product.
// =================================================================================================
struct __align__(16) SelRow { float thr, mx; int jstar; int pad; };
__host__ __device__ __forceinline__ int attn_lpad64(int L_max) { return (L_max + 63) & ~63; }

// column (256*j + 4*lane + e order) of the quota-th key equal to thr; quota >= 1 and at most the
// number of such keys
template <int SLOTS>
__device__ __forceinline__ int wave_tie_last(const float (&key)[SLOTS], int n, float thr, int quota, int lane)
{
    int result = 0x7FFFFFFF;
    bool found = false;
#pragma unroll
    for (int j = 0; j < SLOTS / 4; ++j) {
        if (256 * j < n && !found) {
            int below = 0, here = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned long long bal = __ballot(key[4 * j + e] == thr);
                below = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, below));
                here += __popcll(bal);
            }
            if (quota <= here) {                         // the quota-th tie sits in this group of 256 columns
                int mine = 0, col = -1;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool tie = key[4 * j + e] == thr;
                    if (tie && below + mine == quota - 1) col = 256 * j + 4 * lane + e;
                    mine += tie;
                }
                const unsigned long long who = __ballot(col >= 0);          // exactly one lane
                result = __builtin_amdgcn_readlane(col, (int)__builtin_ctzll(who));
                found = true;
            } else {
                quota -= here;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    return result;
}

// number of scores >= pivot, the pivot in a vector register (the same value in every lane). NG > 0: the first NG groups of
// 256 columns; NG == 0: every group that starts below n. The row is held as the scores themselves (-inf past its end)
// and compared as floats: that counts what comparing order-preserving keys counts (-0 and +0 are one value either way,
// subnormals are not flushed, there are no NaNs), and the row needs no conversion when it is loaded.
template <int SLOTS, int NG>
__device__ __forceinline__ int wave_count_ge_v(const float (&key)[SLOTS], int n, float pivot)
{
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < (NG ? NG : SLOTS / 4); ++j)
        if (NG || 256 * j < n) {
            unsigned long long m[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) asm("v_cmp_ge_f32_e64 %0, %1, %2" : "=s"(m[e]) : "v"(key[4 * j + e]), "v"(pivot));
            cnt += (__popcll(m[0]) + __popcll(m[1])) + (__popcll(m[2]) + __popcll(m[3]));
        }
    return cnt;
}

// the same count with one dispatch per call on the row's number of 256-column groups ng = ceil(n / 256), for a search
// loop that exists once (the variant with a side job): long rows only
template <int SLOTS>
__device__ __forceinline__ int wave_count_ge_sw(const float (&key)[SLOTS], int n, int ng, float pivot)
{
    static_assert(SLOTS == 20 || SLOTS == 32 || SLOTS == 64, "long-row variants");
    if constexpr (SLOTS == 20) {
        return ng == 5 ? wave_count_ge_v<SLOTS, 5>(key, n, pivot) : wave_count_ge_v<SLOTS, 0>(key, n, pivot);
    } else if constexpr (SLOTS == 32) {
        switch (ng) {
        case 8: return wave_count_ge_v<SLOTS, 8>(key, n, pivot);
        case 7: return wave_count_ge_v<SLOTS, 7>(key, n, pivot);
        case 6: return wave_count_ge_v<SLOTS, 6>(key, n, pivot);
        case 5: return wave_count_ge_v<SLOTS, 5>(key, n, pivot);
        default: return wave_count_ge_v<SLOTS, 0>(key, n, pivot);
        }
    } else {
        switch (ng) {
        case 16: return wave_count_ge_v<SLOTS, 16>(key, n, pivot);
        case 15: return wave_count_ge_v<SLOTS, 15>(key, n, pivot);
        case 14: return wave_count_ge_v<SLOTS, 14>(key, n, pivot);
        case 13: return wave_count_ge_v<SLOTS, 13>(key, n, pivot);
        case 12: return wave_count_ge_v<SLOTS, 12>(key, n, pivot);
        case 11: return wave_count_ge_v<SLOTS, 11>(key, n, pivot);
        case 10: return wave_count_ge_v<SLOTS, 10>(key, n, pivot);
        case 9: return wave_count_ge_v<SLOTS, 9>(key, n, pivot);
        default: return wave_count_ge_v<SLOTS, 0>(key, n, pivot);
        }
    }
}

// One row's search from the bracket [lo, hi] (count(key >= lo) >= b, count(key >= hi + 1) < b): returns the bracket
// closed on the threshold key (lo == hi), or exact = true and a pivot with exactly b keys at or above it.
// With g(x) = #(key >= x) - b + 1/2, g(lo) > 0 > g(hi + 1). The pivot is the zero of the straight line through the
// two ends in the score domain (regula falsi with the Illinois correction: an end that stays put twice in a row has
// its weight halved), clamped into (lo, hi] so that every step shrinks the bracket; on smooth score distributions
// this lands between the b-th and (b+1)-th largest score in about 6 steps where bisection of the key needs about
// 14. From the 13th step on the pivot is the midpoint of the key range, which bounds the worst case.
// The bracket and the line live in vector registers and are updated by selects although every lane holds the same
// values: the loop is bound by the scalar unit, which already counts the compare masks, and a CU has four vector
// pipes to its one scalar pipe.
// side: called once per step, after the count: work of the caller's that does not depend on the search and that the
// steps' vector and scalar instructions can hide (k_attn_select: the score tiles of the workgroup's next block)
struct NoSide { __device__ __forceinline__ void operator()() const {} };
template <int SLOTS, int NG, class Side>
__device__ __forceinline__ uint32_t wave_search_thr(const float (&key)[SLOTS], int n, int b, uint32_t lo_s, uint32_t hi_s,
                                                    bool &exact, Side &side)
{
    uint32_t lo = lo_s, hi = hi_s;
    asm volatile("" : "+v"(lo), "+v"(hi));               // from here on the compiler treats the bracket as per-lane data
    // counts enter the line as log-odds, t(c) = log2((c + 1/2) / (n - c + 1/2)) - t(b - 1/2): for bell-shaped score
    // distributions t is close to linear in the score where the count itself is S-shaped
    // uniform and fixed over the loop: kept in scalar registers (the vector registers are what limits the kernel's occupancy)
    const float nh = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int((float)n + 0.5f)));
    const float t_b = __int_as_float(__builtin_amdgcn_readfirstlane(
        __float_as_int(__builtin_amdgcn_logf((float)b * __builtin_amdgcn_rcpf((float)(n - b) + 1.0f)))));
    float flo = score_unkey(lo), fhi = score_unkey(hi);
    float glo = __builtin_amdgcn_logf(nh * 2.0f) - t_b, ghi = -__builtin_amdgcn_logf(nh * 2.0f) - t_b;
    float w_up = 1.0f, w_dn = 1.0f;                      // what the end that stays put is scaled by if the step goes up / down
    exact = false;
    for (int it = 0; __ballot(lo < hi) != 0ull; ++it) {
        const float fp = __builtin_fmaf(fhi - flo, glo * __builtin_amdgcn_rcpf(glo - ghi), flo);
        const uint32_t ufp = __float_as_uint(fp);         // as score_key; which of the two zeros' keys a pivot takes is immaterial
        uint32_t mid = ufp ^ ((uint32_t)((int32_t)ufp >> 31) | 0x80000000u);
        mid = __builtin_elementwise_max(mid, lo + 1u);
        mid = __builtin_elementwise_min(mid, hi);
        if (__builtin_amdgcn_readfirstlane(it) >= 12) {   // a branch that is hardly ever taken, not five instructions per step
            mid = lo + ((hi - lo + 1u) >> 1);
            asm volatile("" : "+v"(mid));
        }
        // score_unkey as a shift and one three-input bit operation (the sign mask passes through an empty asm, or the
        // compiler turns it back into a compare and a select)
        int32_t sgn = (int32_t)mid >> 31;
        asm("" : "+v"(sgn));
        const float fmid = __uint_as_float(mid ^ (~(uint32_t)sgn | 0x80000000u));
        int cnt;
        if constexpr (NG < 0) cnt = wave_count_ge_sw<SLOTS>(key, n, (n + 255) >> 8, fmid);
        else cnt = wave_count_ge_v<SLOTS, NG>(key, n, fmid);
        side();
        if (cnt == b) { exact = true; lo = mid; break; }
        const float cf = (float)cnt;
        const float g = __builtin_amdgcn_logf((cf + 0.5f) * __builtin_amdgcn_rcpf(nh - cf)) - t_b;
        const bool up = cnt > b;                          // the pivot becomes the lower end, else pivot - 1 the upper
        const float glo_w = glo * w_dn, ghi_w = ghi * w_up;
        lo = up ? mid : lo;
        hi = up ? hi : mid - 1u;
        flo = up ? fmid : flo;
        fhi = up ? fhi : fmid;
        glo = up ? g : glo_w;
        ghi = up ? ghi_w : g;
        w_up = up ? 0.5f : 1.0f;
        w_dn = up ? 1.0f : 0.5f;
    }
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)lo);
}

// finishes one row's search from the bracket [lo, hi] (see wave_select_topk): returns the threshold key
// and the index of the last kept key among those equal to it (INT_MAX when all of them are kept)
template <int SLOTS, class Side>
__device__ __forceinline__ uint32_t wave_select_thr(const float (&key)[SLOTS], int n_in, int b_in, uint32_t lo_in,
                                                    uint32_t hi_in, int lane, int &jstar, Side &side)
{
    const int n = __builtin_amdgcn_readfirstlane(n_in), b = __builtin_amdgcn_readfirstlane(b_in);
    const uint32_t lo0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)lo_in);
    const uint32_t hi0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)hi_in);
    jstar = 0x7FFFFFFF;
    bool exact;
    uint32_t lo;
    if constexpr (!std::is_same<Side, NoSide>::value && SLOTS > 16) {
        lo = wave_search_thr<SLOTS, -1, Side>(key, n, b, lo0, hi0, exact, side);   // the side job's code exists once
    } else if constexpr (SLOTS <= 16) {                  // one copy of the loop per row length in groups: no per-step dispatch
        const int ng = (n + 255) >> 8;
        if (ng <= 1) lo = wave_search_thr<SLOTS, 1, Side>(key, n, b, lo0, hi0, exact, side);
        else if (SLOTS >= 8 && ng == 2) lo = wave_search_thr<SLOTS, (SLOTS >= 8 ? 2 : 1), Side>(key, n, b, lo0, hi0, exact, side);
        else if (SLOTS >= 12 && ng == 3) lo = wave_search_thr<SLOTS, (SLOTS >= 12 ? 3 : 1), Side>(key, n, b, lo0, hi0, exact, side);
        else lo = wave_search_thr<SLOTS, SLOTS / 4, Side>(key, n, b, lo0, hi0, exact, side);
    } else if constexpr (SLOTS == 20) {                  // rows of 1025..1280 keys (a 1024-token prefix plus a short episode)
        if (((n + 255) >> 8) == 5) lo = wave_search_thr<SLOTS, 5, Side>(key, n, b, lo0, hi0, exact, side);
        else lo = wave_search_thr<SLOTS, 0, Side>(key, n, b, lo0, hi0, exact, side);
    } else if constexpr (SLOTS == 32) {                  // rows of 1025..2048 keys: 5..8 groups (shorter ones take the general loop)
        const int ng = (n + 255) >> 8;
        if (ng == 8) lo = wave_search_thr<SLOTS, 8, Side>(key, n, b, lo0, hi0, exact, side);
        else if (ng == 7) lo = wave_search_thr<SLOTS, 7, Side>(key, n, b, lo0, hi0, exact, side);
        else if (ng == 6) lo = wave_search_thr<SLOTS, 6, Side>(key, n, b, lo0, hi0, exact, side);
        else if (ng == 5) lo = wave_search_thr<SLOTS, 5, Side>(key, n, b, lo0, hi0, exact, side);
        else lo = wave_search_thr<SLOTS, 0, Side>(key, n, b, lo0, hi0, exact, side);
    } else if constexpr (SLOTS == 64) {                  // rows of 2049..4096 keys: 9..16 groups
        const int ng = (n + 255) >> 8;
        switch (ng) {
        case 16: lo = wave_search_thr<SLOTS, 16, Side>(key, n, b, lo0, hi0, exact, side); break;
        case 15: lo = wave_search_thr<SLOTS, 15, Side>(key, n, b, lo0, hi0, exact, side); break;
        case 14: lo = wave_search_thr<SLOTS, 14, Side>(key, n, b, lo0, hi0, exact, side); break;
        case 13: lo = wave_search_thr<SLOTS, 13, Side>(key, n, b, lo0, hi0, exact, side); break;
        case 12: lo = wave_search_thr<SLOTS, 12, Side>(key, n, b, lo0, hi0, exact, side); break;
        case 11: lo = wave_search_thr<SLOTS, 11, Side>(key, n, b, lo0, hi0, exact, side); break;
        case 10: lo = wave_search_thr<SLOTS, 10, Side>(key, n, b, lo0, hi0, exact, side); break;
        case 9: lo = wave_search_thr<SLOTS, 9, Side>(key, n, b, lo0, hi0, exact, side); break;
        default: lo = wave_search_thr<SLOTS, 0, Side>(key, n, b, lo0, hi0, exact, side); break;
        }
    } else {
        lo = wave_search_thr<SLOTS, 0, Side>(key, n, b, lo0, hi0, exact, side);
    }
    if (exact) return lo;
    float flo = score_unkey(lo), fnext = score_unkey(lo + 1u);
    asm volatile("" : "+v"(flo), "+v"(fnext));           // vector registers, as the counting compare takes them
    const int n_ge = wave_count_ge_v<SLOTS, 0>(key, n, flo);
    if (n_ge > b) {                                      // more keys equal to the threshold than the budget has room for
        const int n_gt = (lo == 0xFFFFFFFFu) ? 0 : wave_count_ge_v<SLOTS, 0>(key, n, fnext);
        jstar = wave_tie_last<SLOTS>(key, n, flo, b - n_gt, lane);
    }
    return lo;
}

template <int SLOTS>
__device__ __forceinline__ uint32_t wave_select_thr(const float (&key)[SLOTS], int n_in, int b_in, uint32_t lo_in,
                                                    uint32_t hi_in, int lane, int &jstar)
{
    NoSide none;
    return wave_select_thr<SLOTS, NoSide>(key, n_in, b_in, lo_in, hi_in, lane, jstar, none);
}

// loads a score row from LDS as it is (-inf for columns >= n: below every pivot of the search); the row's maximum and
// minimum come back as order-preserving keys (-0.0 counts as +0.0), the bracket the search starts from
template <int SLOTS>
__device__ __forceinline__ void sel_row_load(const float *row, int n, int lane, float (&key)[SLOTS], uint32_t &kmax_out,
                                             uint32_t &kmin_out)
{
    // score_key as shift / or / xor; the extremes are taken on the floats (three-input max and min), which order like the keys
    auto to_key = [](float v) {
        const uint32_t u = __float_as_uint(v + 0.0f);      // -0 + 0 = +0
        return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
    };
    float fmax = -__builtin_inff(), fmin = __builtin_inff();
#pragma unroll
    for (int j = 0; j < SLOTS / 4; ++j) {
        if (256 * (j + 1) <= n) {                          // every column of the group is a key of the row
            const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * j + e] = v[e];
            fmax = __builtin_fmaxf(__builtin_fmaxf(fmax, v[0]), v[1]);
            fmax = __builtin_fmaxf(__builtin_fmaxf(fmax, v[2]), v[3]);
            fmin = __builtin_fminf(__builtin_fminf(fmin, v[0]), v[1]);
            fmin = __builtin_fminf(__builtin_fminf(fmin, v[2]), v[3]);
        } else if (256 * j < n) {
            const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool valid = 256 * j + 4 * lane + e < n;
                key[4 * j + e] = valid ? v[e] : -__builtin_inff();
                fmax = valid ? __builtin_fmaxf(fmax, v[e]) : fmax;
                fmin = valid ? __builtin_fminf(fmin, v[e]) : fmin;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * j + e] = -__builtin_inff();
        }
    }
    kmax_out = wave_max_u32(to_key(fmax));                 // a lane without a valid column holds -inf / +inf: below / above every score
    kmin_out = wave_min_u32(to_key(fmin));
}

// ---- pieces of k_attn_select's score phase; they expand where qf, kbase, kdelta, pv, sc, scale, lane, l16, lg, w and
// n_kt (key tiles of the block) are in scope: the kernel itself and SelSide below ----
    // K tile KT_ (clamped to the last tile / key of the block) into SET_[U_]: lane (l16, lg) gets 8 channels at 8*lg of
    // key 16*tile + l16 for every 32-channel piece
#define SOL_SEL_LOADK(SET_, U_, KT_, KEY0_, NKEYS_)                                                        \
    {   /* addresses as a uniform base plus a 32-bit byte offset per lane: one address register per load, no 64-bit sums */ \
        const char *kb_ = reinterpret_cast<const char *>(kbase);                                           \
        if constexpr (KF && PRE) {      /* prefix tiles from the operand-order copy, own tiles from the own cache */ \
            int kt_ = (KT_);                                                                               \
            if (kt_ * 16 >= (NKEYS_)) kt_ = ((NKEYS_) - 1) >> 4;                                           \
            const bool in_pre = kt_ * 16 < pv.P;            /* wave-uniform; pv.P is a multiple of 64 */   \
            int key = kt_ * 16 + l16;                                                                      \
            if (key >= (NKEYS_)) key = (NKEYS_) - 1;                                                       \
            const uint32_t off = in_pre ? (uint32_t)kt_ * (uint32_t)(KK * 512) + (uint32_t)(lane * 8)      \
                                        : kdelta + (uint32_t)key * (uint32_t)DH + (uint32_t)(lg * 8);      \
            const uint32_t step = in_pre ? 1024u : 64u;                                                    \
            _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                              \
                SET_[U_][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(kb_ + (off * 2u + kk * step))); \
        } else if constexpr (KF) {                                                                         \
            int kt_ = (KT_);                                                                               \
            if (kt_ * 16 >= (NKEYS_)) kt_ = ((NKEYS_) - 1) >> 4;                                           \
            const uint32_t fo = ((uint32_t)kt_ * (uint32_t)(KK * 512) + (uint32_t)((KEY0_) * 8)) * 2u;     \
            _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                              \
                SET_[U_][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(kb_ + fo + kk * 1024)); \
        } else {                                                                                           \
            int key = (KEY0_) + (U_) * NW * 16;                                                            \
            if (key >= (NKEYS_)) key = (NKEYS_) - 1;                                                       \
            uint32_t ko = (uint32_t)key * (uint32_t)DH + (uint32_t)(lg * 8);                               \
            if constexpr (PRE) ko += key >= pv.P ? kdelta : 0u;                                            \
            ko *= 2u;                                                                                      \
            _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                              \
                SET_[U_][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(kb_ + ko + kk * 64)); \
        }                                                                                                  \
    }
    // group of UH tiles from this wave's tile T0_ on (stride NW), if the group has a tile below the block's last key.
    // EACH_: tiles past the last key are not loaded (the prefetch of the next block, issued before a long search);
    // otherwise they re-read the last tile, which keeps the loads of a group free of branches.
#define SOL_SEL_LOADG(SET_, T0_, NKEYS_, EACH_)                                                            \
    if ((T0_) * 16 < (NKEYS_)) {                                                                           \
        int key0_ = KF ? lane : (T0_) * 16 + l16;                                                          \
        asm volatile("" : "+v"(key0_));   /* recomputed per group: hoisted copies of all the indices spill */ \
        _Pragma("unroll") for (int u = 0; u < UH; ++u) {                                                   \
            if (!(EACH_) || ((T0_) + u * NW) * 16 < (NKEYS_)) SOL_SEL_LOADK(SET_, u, (T0_) + u * NW, key0_, NKEYS_) \
        }                                                                                                  \
    }
    // q fragments and the first two groups of K tiles of query block QB_
#define SOL_SEL_LOAD(QB_)                                                                                  \
    {                                                                                                      \
        const int q0_ = q_lo + (QB_) * BQ;                                                                 \
        const int nmax_ = p0 + (q_hi < q0_ + BQ ? q_hi : q0_ + BQ);                                        \
        _Pragma("unroll") for (int rt = 0; rt < RT; ++rt) {                                                \
            int qr = q0_ + rt * 16 + l16;                                                                  \
            if (qr >= Tn) qr = Tn - 1;                                                                     \
            const uint32_t qo = ((uint32_t)qr * (uint32_t)(Hq * DH) + (uint32_t)(lg * 8)) * 2u;            \
            _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                              \
                qf[rt][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(              \
                                                    reinterpret_cast<const char *>(qbase) + qo + kk * 64)); \
        }                                                                                                  \
        SOL_SEL_LOADG(ka, w, nmax_, true)                                                                  \
        if constexpr (DB) SOL_SEL_LOADG(kb, w + UH * NW, nmax_, true)                                      \
    }
    // S^T tile = K tile (rows) x Q^T (columns): lane (l16, lg) gets keys 4*lg..4*lg+3 of query l16
#define SOL_SEL_MFMA(SET_, U_, KT_)                                                                        \
    _Pragma("unroll") for (int rt = 0; rt < RT; ++rt) {                                                    \
        floatx4_a acc = {0.f, 0.f, 0.f, 0.f};                                                              \
        _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                                  \
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(SET_[U_][kk], qf[rt][kk], acc, 0, 0, 0);         \
        const int row = rt * 16 + l16;                                                                     \
        if (row < BQ)                                                                                      \
            *reinterpret_cast<f32x4_a *>(sc + row * LS + (KT_) * 16 + 4 * lg) =                            \
                f32x4_a{acc[0] * scale, acc[1] * scale, acc[2] * scale, acc[3] * scale};                   \
    }
#define SOL_SEL_MFMAG(SET_, T0_)                                                                           \
    _Pragma("unroll") for (int u = 0; u < UH; ++u) {                                                       \
        const int kt = (T0_) + u * NW;                                                                     \
        if (kt < n_kt) { SOL_SEL_MFMA(SET_, u, kt); }                                                      \
    }


// The score phase of k_attn_select as a side job of the threshold search (long rows): the fragments in registers and
// what the macros above refer to, under the same names. One call multiplies the next two groups of key tiles of the
// block [n_max keys, n_kt tiles] (one per register set) into the LDS rows sc and requests the two groups after them;
// nothing once the block's tiles are through (tcur >= n_kt).
template <int BQ, int SLOTS, int DH, int NW, bool PRE, bool KF> struct SelSide {
    static constexpr int LPAD = SLOTS * 64, LS = LPAD + 4; // row stride = 4 mod 64 floats: the 16 query rows of a
                                                           // 128-bit store hit 16 different bank groups
    static constexpr int RT = (BQ + 15) / 16, KK = DH / 32;
    // key tiles held per wave. Head size 128, rows up to 2048 keys: 2, with which the kernel fits 128 registers and a
    // second workgroup fits the CU (4 tiles: 168 registers, one workgroup; 1.28 -> 0.83 ms for the 1025..2048-key rows
    // of 4096-token sequences at the 8B shape). The 20-slot variant at head size 64 likewise: 80 registers and 41 KB
    // of LDS, so three workgroups share a CU (episode pass, 16 rows per sequence on a 1024-token prefix: 272 -> 199 us
    // per launch; on long walks, rows of 1025..1280 keys at C3, it gains nothing over the 32-slot variant)
    static constexpr int UA = (SLOTS <= 16 && DH <= 64) ? 8 : ((SLOTS <= 32 && DH > 64) || SLOTS == 20) ? 2 : 4;
    // Rows longer than what the waves hold at once (SLOTS > 16): two register sets of UH key tiles each, one in flight
    // while the other is multiplied. Shorter rows: one set, all of it loaded while the block before is searched.
    static constexpr bool DB = SLOTS > 16;
    static constexpr int UH = DB ? UA / 2 : UA;
    static constexpr int GS = UH * NW;                     // tiles per group over the workgroup
    bf16x8_a qf[RT][KK], ka[UH][KK], kb[DB ? UH : 1][KK];
    const bf16_t *kbase;
    uint32_t kdelta;
    PrefixView pv;
    float *sc;
    float scale;
    int lane, l16, lg, w;
    int n_max, n_kt, tcur;
    __device__ __forceinline__ void operator()()
    {
        if (tcur < n_kt) {
            SOL_SEL_MFMAG(ka, tcur)
            SOL_SEL_LOADG(ka, tcur + 2 * GS, n_max, false)
            if (tcur + GS < n_kt) {
                SOL_SEL_MFMAG(kb, tcur + GS)
                SOL_SEL_LOADG(kb, tcur + 3 * GS, n_max, false)
            }
            tcur += 2 * GS;
        }
    }
};

// A workgroup walks several blocks of BQ query rows of one (sequence, head): while the waves search the
// thresholds of one block, the q and K fragments of the next are already on their way into registers,
// so the global-load latency of the score phase is hidden. Blocks are dealt to the nb workgroups of a
// (sequence, head) in zigzag order (k-th visit: block nb*k + bi for even k, nb*k + nb-1-bi for odd k),
// which gives every workgroup the same number of causal keys.
// PRE: keys [0, pv.P) of sequence s are read from the prefix cache of input s / pv.K (shared by the pv.K schedules
// of that input), keys from pv.P on from the sequence's own cache kc, which holds positions pv.P.. only
// ([n_seq][Hkv][crows][DH]); pv.P is a multiple of 64 and the two caches lie less than 2^31 elements apart.
// KF: kc (with PRE: pv.kf, for the prefix keys) is the copy of the K cache in MFMA operand order written by k_frag_k,
// in which the 16 bytes a lane feeds to one MFMA are contiguous over the lanes: a fragment load reads 1 KB in a row
// (8 full cache lines) where the same load from the cache itself picks 64-byte pieces out of 16 rows. The values in
// the registers are the same either way. With PRE the sequence's own keys (positions pv.P..) still come from its cache.
template <int BQ, int SLOTS, int DH, int NW, bool PRE, bool KF>
__global__ void __launch_bounds__(NW * 64)
__attribute__((amdgpu_waves_per_eu(SLOTS == 20 && DH <= 64 ? 6 : SLOTS <= 32 ? 4 : 2, SLOTS <= 16 ? 4 : 8)))
k_attn_select(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc, SelRow *__restrict__ sel,
              const RowAct *__restrict__ ra, const int32_t *__restrict__ pos0, int Tn, int L_max, int Hq, int Hkv,
              float scale, int nb, PrefixView pv, int n_lo, int n_hi)
{
    using Frags = SelSide<BQ, SLOTS, DH, NW, PRE, KF>;
    constexpr int LS = Frags::LS, RT = Frags::RT, KK = Frags::KK, UH = Frags::UH, GS = Frags::GS;
    constexpr bool DB = Frags::DB;
    extern __shared__ __align__(16) float sc[];            // [BQ][LS]
    __shared__ int next_row;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bi = blockIdx.x, h = blockIdx.y, s = blockIdx.z;
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) return;                 // flagged by the projection kernel; sequence skipped
    // this launch takes the rows whose key count n = p0 + row + 1 lies in (n_lo, n_hi]: rows [q_lo, q_hi) of the sequence
    // (long sequences are split by row length over the kernel's variants; the blocks of BQ rows count from q_lo)
    const int q_lo = n_lo - p0 < 0 ? 0 : (n_lo - p0 > Tn ? Tn : n_lo - p0);
    const int q_hi = n_hi - p0 < 0 ? 0 : (n_hi - p0 > Tn ? Tn : n_hi - p0);
    if (q_hi <= q_lo) return;                              // whole workgroup, before any barrier
    const int n_qb = (q_hi - q_lo + BQ - 1) / BQ;
    const int kvh = h / (Hq / Hkv);
    // wave-uniform bases + 32-bit per-lane offsets: one address register per load instead of two
    const bf16_t *kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)(KF ? attn_lpad64(L_max) : L_max) * DH;
    uint32_t kdelta = 0u;                                   // PRE: offset of the own cache (minus P rows) from the prefix cache
    if constexpr (PRE) {
        const bf16_t *own = kc + ((int64_t)s * Hkv + kvh) * (int64_t)pv.crows * DH - (int64_t)pv.P * DH;
        kbase = (KF ? pv.kf : pv.k) + ((int64_t)(s / pv.K) * Hkv + kvh) * (int64_t)pv.P * DH;
        kdelta = (uint32_t)__builtin_amdgcn_readfirstlane((int)(own - kbase));
    }
    const bf16_t *qbase = q + (int64_t)s * Tn * (int64_t)(Hq * DH) + (int64_t)h * DH;
    const int l16 = lane & 15, lg = lane >> 4;

    Frags fr;                                              // the fragments, and the score phase as the search's side job
    auto &qf = fr.qf;
    auto &ka = fr.ka;
    auto &kb = fr.kb;
    fr.kbase = kbase, fr.kdelta = kdelta, fr.pv = pv, fr.sc = sc, fr.scale = scale;
    fr.lane = lane, fr.l16 = l16, fr.lg = lg, fr.w = w;
    fr.n_max = 0, fr.n_kt = 0, fr.tcur = 0;
    int visit = 0, qb = bi;
    if (qb >= n_qb) return;
    SOL_SEL_LOAD(qb);
    if constexpr (DB) {
        // Long rows, one row per wave. The score phase is bound by what the CU's L1 delivers and the search by the
        // vector and scalar pipes, so a wave does both at once: while it searches its row of block k (in registers; the
        // LDS rows are free once every wave has taken its own) each step of the search also multiplies one group of key
        // tiles of block k + 1 into LDS and requests the group after the next. What the search leaves over is done behind
        // it. The barriers wait for LDS only (s_waitcnt lgkmcnt): global loads and the result's store stay in flight.
        static_assert(BQ == NW, "one row per wave");
#define SOL_SEL_BARRIER asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")
        {                                                   // scores of the workgroup's first block
            const int q0 = q_lo + qb * BQ;
            const int rows = (q_hi - q0 < BQ) ? (q_hi - q0) : BQ;
            const int n_max = p0 + q0 + rows;
            const int n_kt = (n_max + 15) >> 4;
            for (int t0 = w;; t0 += 2 * GS) {
                SOL_SEL_MFMAG(ka, t0)
                SOL_SEL_LOADG(ka, t0 + 2 * GS, n_max, false)
                if (t0 + GS >= n_kt) break;
                SOL_SEL_MFMAG(kb, t0 + GS)
                SOL_SEL_LOADG(kb, t0 + 3 * GS, n_max, false)
                if (t0 + 2 * GS >= n_kt) break;
            }
        }
        while (true) {
            const int q0 = q_lo + qb * BQ;
            const int rows = (q_hi - q0 < BQ) ? (q_hi - q0) : BQ;
            ++visit;
            const int qb_next = nb * visit + ((visit & 1) ? nb - 1 - bi : bi);
            const bool more = qb_next < n_qb;
            const bool have = w < rows;                     // this wave's row of the block
            const int n = p0 + q0 + w + 1;
            RowAct act = RowAct();
            if (have) act = ra[(int64_t)s * Tn + q0 + w];
            fr.n_max = 0, fr.n_kt = 0;                      // the next block's
            if (more) {
                SOL_SEL_LOAD(qb_next);
                const int q0n = q_lo + qb_next * BQ;
                fr.n_max = p0 + (q_hi < q0n + BQ ? q_hi : q0n + BQ);
                fr.n_kt = (fr.n_max + 15) >> 4;
            }
            SOL_SEL_BARRIER;                                // the block's scores are complete
            float key[SLOTS];
            uint32_t kmax = 0u, kmin = 0u;
            if (have) sel_row_load<SLOTS>(sc + w * LS, n, lane, key, kmax, kmin);
            SOL_SEL_BARRIER;                                // every row is in registers: LDS may be overwritten
            fr.tcur = w;
            if (have) {
                const int b = budget_ceil(act.keep_num, act.keep_den, n);
                uint32_t thr = 0u;                          // key 0: below every score, everything kept
                int js = 0x7FFFFFFF;
                if (b < n) thr = wave_select_thr<SLOTS>(key, n, b, kmin, kmax, lane, js, fr);
                if (lane == 0)
                    sel[((int64_t)s * Tn + q0 + w) * Hq + h] =
                        SelRow{thr ? score_unkey(thr) : -__builtin_inff(), score_unkey(kmax), js, 0};
            }
            if (!more) break;
            while (fr.tcur < fr.n_kt) fr();
            qb = qb_next;
        }
#undef SOL_SEL_BARRIER
    } else {
    while (true) {
        const int q0 = q_lo + qb * BQ;
        const int rows = (q_hi - q0 < BQ) ? (q_hi - q0) : BQ;
        const int n_max = p0 + q0 + rows;
        const int n_kt = (n_max + 15) >> 4;
        // ---- scores of this block into LDS: the loads of a group of tiles go out while the group before it is multiplied ----
        SOL_SEL_MFMAG(ka, w)
        for (int t0 = w + GS; t0 < n_kt; t0 += GS) {
            SOL_SEL_LOADG(ka, t0, n_max, false)
            SOL_SEL_MFMAG(ka, t0)
        }
        if (tid == 0) next_row = NW;
        __syncthreads();
        // ---- next block's fragments on their way while this block's rows are searched ----
        ++visit;
        const int qb_next = nb * visit + ((visit & 1) ? nb - 1 - bi : bi);
        const bool more = qb_next < n_qb;
        if (more) SOL_SEL_LOAD(qb_next);
        // ---- per row: maximum, and the threshold when the budget is below the row length ----
        // the first NW rows go one to each wave, the others to whichever wave is free first
        for (int r = w; r < rows;) {
            const int n = p0 + q0 + r + 1;
            const RowAct act = ra[(int64_t)s * Tn + q0 + r];
            const int b = budget_ceil(act.keep_num, act.keep_den, n);
            float key[SLOTS];
            uint32_t kmax, kmin;
            sel_row_load<SLOTS>(sc + r * LS, n, lane, key, kmax, kmin);
            uint32_t thr = 0u;                             // key 0: below every score, everything kept
            int js = 0x7FFFFFFF;
            if (b < n) thr = wave_select_thr<SLOTS>(key, n, b, kmin, kmax, lane, js);
            int r_next = 0;
            if (lane == 0) {
                sel[((int64_t)s * Tn + q0 + r) * Hq + h] =
                    SelRow{thr ? score_unkey(thr) : -__builtin_inff(), score_unkey(kmax), js, 0};
                r_next = atomicAdd(&next_row, 1);
            }
            r = __builtin_amdgcn_readfirstlane(r_next);
        }
        if (!more) break;
        __syncthreads();                                   // every row is in registers or done: LDS may be overwritten
        qb = qb_next;
    }
    }
#undef SOL_SEL_LOADK
#undef SOL_SEL_LOADG
#undef SOL_SEL_LOAD
#undef SOL_SEL_MFMA
#undef SOL_SEL_MFMAG
}

// Unit hook: the row stage of k_attn_select (keys from an fp32 score row in LDS, threshold search, tie index) on caller
// rows, one wave per row; keep[r][j] = 1 for the kept columns, by the same rule k_attn_pv applies to {thr, jstar}.
template <int SLOTS>
__global__ void __launch_bounds__(64) k_test_select_rows(const float *__restrict__ scores, int n_cols, const int32_t *__restrict__ n_valid,
                                                         const int32_t *__restrict__ kk, uint8_t *__restrict__ keep)
{
    extern __shared__ __align__(16) float sc[];              // [SLOTS * 64]
    const int lane = threadIdx.x, r = blockIdx.x;
    const float *row = scores + (int64_t)r * n_cols;
    const int n = n_valid[r], b = kk[r];
    for (int j = lane; j < SLOTS * 64; j += 64) sc[j] = j < n ? row[j] : 0.f;
    __syncthreads();
    float key[SLOTS];
    uint32_t kmax, kmin;
    sel_row_load<SLOTS>(sc, n, lane, key, kmax, kmin);
    uint32_t thr = 0u;
    int js = 0x7FFFFFFF;
    if (b < n) thr = wave_select_thr<SLOTS>(key, n, b, kmin, kmax, lane, js);
    const float fthr = thr ? score_unkey(thr) : -__builtin_inff();
    for (int j = lane; j < n_cols; j += 64) {
        const float sv = j < n ? sc[j] : 0.f;
        keep[(int64_t)r * n_cols + j] = (j < n && (sv > fthr || (sv == fthr && j <= js))) ? 1 : 0;
    }
}

bool launch_test_attn_threshold(const float *scores, int rows, int n_cols, const int32_t *n_valid, const int32_t *k,
                                uint8_t *keep_out, hipStream_t st)
{
    if (n_cols > 4096) return false;
#define SOL_TSEL(SL)                                                                                                 \
    hipLaunchKernelGGL((k_test_select_rows<SL>), dim3(rows), dim3(64), (size_t)(SL) * 64 * 4, st, scores, n_cols, n_valid, k, \
                       keep_out)
    if (n_cols <= 256) SOL_TSEL(4);                          // the variants of launch_attn_tile
    else if (n_cols <= 1024) SOL_TSEL(16);
    else if (n_cols <= 1280) SOL_TSEL(20);
    else if (n_cols <= 2048) SOL_TSEL(32);
    else SOL_TSEL(64);
#undef SOL_TSEL
    return true;
}

// ---- k_attn_pv -------------------------------------------------------------------------------------
// LDS chunk layouts (bf16, 16-byte pieces XOR-swizzled so that the 128-bit fragment reads of 16 lanes
// hit 16 different bank groups):
//   K chunk   [64 keys][DH]      piece' = piece ^ swzK(key row)
//   V^T chunk [DH][64 keys]      piece' = piece ^ ((d >> 1) & 7)
template <int DH> __device__ __forceinline__ int pv_swz_k(int row)
{
    if constexpr (DH == 64) return ((row >> 1) & 1) | (((row >> 3) & 3) << 1);   // rows {0-3, 8-11, 16-19, 24-27} (+4)
    else return (row & 3) | (((row >> 3) & 3) << 2);
}

// softmax numerators of one 32-key sub-chunk for one query tile, as the A operand (hi and lo bf16
// halves) of the P V product. st[kt][r] is the score of key  kbase + 8*lg + 4*kt + r.
template <bool MASK, bool TIES>
__device__ __forceinline__ void pv_probs(const floatx4_a (&st)[2], float scale, float thr, float mxl, int jstar, int pos,
                                         int kfirst, float &den, bf16x8_a &phi, bf16x8_a &plo)
{
    float p[8];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float sv = st[kt][r] * scale;
            const int j = kfirst + 4 * kt + r;
            bool keep = sv >= thr;
            if (TIES) keep = sv > thr || (sv == thr && j <= jstar);
            if (MASK) keep = keep && j <= pos;
            const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(sv, 1.44269504088896341f, -mxl));
            p[4 * kt + r] = keep ? e : 0.f;
            den += p[4 * kt + r];
        }
    u32x4_a hi, lo;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        hi[i] = pack_bf16x2(p[2 * i], p[2 * i + 1]);
        lo[i] = pack_bf16x2(p[2 * i] - __uint_as_float(hi[i] << 16), p[2 * i + 1] - __uint_as_float(hi[i] & 0xFFFF0000u));
    }
    phi = __builtin_bit_cast(bf16x8_a, hi);
    plo = __builtin_bit_cast(bf16x8_a, lo);
}

// PRE: as in k_attn_select; vt then is the transposed copy of the own cache ([n_seq][Hkv][DH][lpadv], positions
// pv.P..) and pv.vt that of the prefix cache ([inputs][Hkv][DH][pv.lpadv]); 64-key chunks never straddle pv.P.
// NQT: query tiles of 16 rows per workgroup (2; 1 for passes of at most 16 rows per sequence).
// Occupancy floors (4+ heads per group): four waves per SIMD at head size 64 (128 registers; the 18 values that do not
// fit are spilled outside the chunk loop), two at head size 128 (256 registers, no spills). Left alone the compiler takes
// 186 and 328 registers, and with one wave per SIMD the softmax's exp / pack chains and the MFMAs have nothing to
// overlap with: 2.90 -> 1.81 ms per launch at the 8B shape with 4096-token sequences.
template <int DH, int G, bool PRE, int NQT>
__global__ void __launch_bounds__(G * 64) __attribute__((amdgpu_waves_per_eu(DH == 64 && G >= 4 ? 4 : (DH == 128 && G >= 4 ? 2 : 1), 8)))
k_attn_pv(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc, const bf16_t *__restrict__ vt,
          const SelRow *__restrict__ sel, float *__restrict__ o32, const int32_t *__restrict__ pos0, int Tn, int L_max, int Hq,
          int Hkv, int lpadv, float scale, PrefixView pv)
{
    constexpr int NT = G * 64, KK = DH / 32, DT = DH / 16, KC = 64, QT = 16 * NQT;
    constexpr int KP = DH / 8;                              // 16-byte pieces per K row
    constexpr int K_PIECES = KC * KP / NT, V_PIECES = DH * (KC / 8) / NT;
    constexpr int K_BYTES = KC * DH * 2, STAGE = 2 * K_BYTES;
    static_assert(KC * KP % NT == 0 && DH * (KC / 8) % NT == 0, "chunk / thread mismatch");
    extern __shared__ __align__(16) unsigned char pvl[];   // 2 stages of { K chunk, V^T chunk }

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups go to the 8 XCDs round-robin in launch order; the gridDim.x workgroups of a (sequence, KV head) read the
    // same K and V, so they are renumbered to share an XCD (and its L2): of 8 * gridDim.x consecutive workgroups, those
    // with the same launch index modulo 8 form one group.
    int bx = blockIdx.x, kvh = blockIdx.y, s = blockIdx.z;
    {
        const int nbx = gridDim.x, n_grp = (int)(gridDim.y * gridDim.z);
        if (n_grp % 8 == 0) {
            const int id = bx + nbx * (kvh + (int)gridDim.y * s), chunk = id / (8 * nbx), within = id - chunk * (8 * nbx);
            const int g = chunk * 8 + (within & 7);
            bx = within >> 3;
            kvh = g % (int)gridDim.y;
            s = g / (int)gridDim.y;
        }
    }
    const int h = kvh * G + w;
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) return;
    // A workgroup takes query blocks n_qb - 1 - x and x: every workgroup streams the same number of causal keys.
    // With one block per workgroup the lifetimes differ by a factor of up to n_qb, and slots freed by the short
    // workgroups of a launch were seen to stay empty until the long ones around them had ended.
    const int n_qb = (Tn + QT - 1) / QT;
    for (int pass = 0; pass < 2; ++pass) {
    const int qb = pass == 0 ? n_qb - 1 - bx : bx;
    if (pass == 1 && qb >= n_qb - 1 - bx) break;            // the middle block of an odd count is its own partner
    const int q0 = qb * QT;
    const int rows = (Tn - q0 < QT) ? (Tn - q0) : QT;
    const int n_max = p0 + q0 + rows;                      // keys seen by the block's last live row
    const int n_chunks = (n_max + KC - 1) / KC;
    const bf16_t *kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    const bf16_t *vbase = vt + ((int64_t)s * Hkv + kvh) * (int64_t)DH * lpadv;
    const bf16_t *kpre = nullptr, *vpre = nullptr;
    if constexpr (PRE) {                                    // own segment addressed by absolute key: bases minus P keys
        kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)pv.crows * DH - (int64_t)pv.P * DH;
        vbase = vbase - pv.P;
        kpre = pv.k + ((int64_t)(s / pv.K) * Hkv + kvh) * (int64_t)pv.P * DH;
        vpre = pv.vt + ((int64_t)(s / pv.K) * Hkv + kvh) * (int64_t)DH * pv.lpadv;
    }

    // per-lane query state: lane l16 of every lane group owns query q0 + 16*qt + l16
    bf16x8_a qf[NQT][KK];
    float thr[NQT], mxl[NQT], den[NQT];
    int jstar[NQT], pos[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        den[qt] = 0.f;
        const int qi = q0 + 16 * qt + l16;
        const bool live = qi < Tn;
        const int qr = live ? qi : Tn - 1;
        const bf16_t *qp = q + ((int64_t)s * Tn + qr) * (int64_t)(Hq * DH) + (int64_t)h * DH + lg * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            qf[qt][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(qp + kk * 32));
        const SelRow sr = sel[((int64_t)s * Tn + qr) * Hq + h];
        thr[qt] = live ? sr.thr : __builtin_inff();        // dead rows of a ragged block keep nothing
        mxl[qt] = sr.mx * 1.44269504088896341f;
        jstar[qt] = sr.jstar;
        pos[qt] = p0 + qi;
    }
    const bool any_ties = __ballot(jstar[0] != 0x7FFFFFFF || jstar[NQT - 1] != 0x7FFFFFFF) != 0ull;

    floatx4_a oacc[NQT][DT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) oacc[qt][dt] = floatx4_a{0.f, 0.f, 0.f, 0.f};

    // staging: global -> registers -> LDS, one chunk ahead
    u32x4_a kreg0[K_PIECES], vreg0[V_PIECES];
#define SOL_PV_GLOAD(KR, VR, CH_)                                                                                  \
    {                                                                                                      \
        const int key0_ = (CH_) * KC;                                                                      \
        const bool pre_ = PRE && key0_ < pv.P;              /* chunk-uniform: P is a multiple of the chunk */ \
        const bf16_t *kb_ = pre_ ? kpre : kbase, *vb_ = pre_ ? vpre : vbase;                               \
        const int64_t vs_ = pre_ ? pv.lpadv : lpadv;                                                       \
        _Pragma("unroll") for (int i = 0; i < K_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, row = pc / KP, piece = pc - row * KP;                             \
            int key = key0_ + row;                                                                         \
            if (key >= n_max) key = n_max - 1;              /* never used unmasked: beyond every row */     \
            KR[i] = *reinterpret_cast<const u32x4_a *>(kb_ + (int64_t)key * DH + piece * 8);               \
        }                                                                                                  \
        _Pragma("unroll") for (int i = 0; i < V_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, d = pc >> 3, piece = pc & 7;                                      \
            VR[i] = *reinterpret_cast<const u32x4_a *>(vb_ + (int64_t)d * vs_ + key0_ + piece * 8);        \
        }                                                                                                  \
    }
#define SOL_PV_LSTORE(KR, VR, STG_)                                                                                \
    {                                                                                                      \
        unsigned char *kb_ = pvl + (STG_) * STAGE, *vb_ = kb_ + K_BYTES;                                   \
        _Pragma("unroll") for (int i = 0; i < K_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, row = pc / KP, piece = pc - row * KP;                             \
            *reinterpret_cast<u32x4_a *>(kb_ + row * (DH * 2) + ((piece ^ pv_swz_k<DH>(row)) << 4)) = KR[i]; \
        }                                                                                                  \
        _Pragma("unroll") for (int i = 0; i < V_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, d = pc >> 3, piece = pc & 7;                                      \
            *reinterpret_cast<u32x4_a *>(vb_ + d * (KC * 2) + ((piece ^ ((d >> 1) & 7)) << 4)) = VR[i];    \
        }                                                                                                  \
    }

    // chunk ch is multiplied out of LDS stage ch % 2 while chunk ch + 1 (fetched one iteration ago) moves from
    // registers into the other stage and chunk ch + 2 is fetched: global latency has a whole iteration to hide in
    SOL_PV_GLOAD(kreg0, vreg0, 0);
    SOL_PV_LSTORE(kreg0, vreg0, 0);
    if (1 < n_chunks) SOL_PV_GLOAD(kreg0, vreg0, 1);
    __syncthreads();
    for (int ch = 0; ch < n_chunks; ++ch) {
        const int stg = ch & 1;
        // one register set: what was fetched an iteration ago goes to LDS, then the set is requested again
        if (ch + 1 < n_chunks) SOL_PV_LSTORE(kreg0, vreg0, stg ^ 1);
        if (ch + 2 < n_chunks) SOL_PV_GLOAD(kreg0, vreg0, ch + 2);
        const unsigned char *kb = pvl + stg * STAGE, *vb = kb + K_BYTES;
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
            const int kb32 = ch * KC + cc * 32;             // first key of this 32-key sub-chunk
            if (kb32 < n_max) {
                // scores: MFMA row m of tile kt is key  kb32 + 8*(m >> 2) + 4*kt + (m & 3)
                floatx4_a st[NQT][2];                         // [qt][kt]
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    const int krow = cc * 32 + 8 * (l16 >> 2) + 4 * kt + (l16 & 3);
                    bf16x8_a kf[KK];
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk)
                        kf[kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(
                            kb + krow * (DH * 2) + (((kk * 4 + lg) ^ pv_swz_k<DH>(krow)) << 4)));
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt) {
                        floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int kk = 0; kk < KK; ++kk)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kk], qf[qt][kk], acc, 0, 0, 0);
                        st[qt][kt] = acc;
                    }
                }
                bf16x8_a phi[NQT], plo[NQT];
                const int kfirst = kb32 + 8 * lg;
                const bool diag = kb32 + 31 > p0 + q0;      // some key of the sub-chunk is beyond some query
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt) {
                    if (any_ties) pv_probs<true, true>(st[qt], scale, thr[qt], mxl[qt], jstar[qt], pos[qt], kfirst, den[qt], phi[qt], plo[qt]);
                    else if (diag) pv_probs<true, false>(st[qt], scale, thr[qt], mxl[qt], jstar[qt], pos[qt], kfirst, den[qt], phi[qt], plo[qt]);
                    else pv_probs<false, false>(st[qt], scale, thr[qt], mxl[qt], jstar[qt], pos[qt], kfirst, den[qt], phi[qt], plo[qt]);
                }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const int d = dt * 16 + l16;
                    const bf16x8_a vf = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(
                        vb + d * (KC * 2) + (((cc * 4 + lg) ^ ((d >> 1) & 7)) << 4)));
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt) {
                        oacc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo[qt], vf, oacc[qt][dt], 0, 0, 0);
                        oacc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi[qt], vf, oacc[qt][dt], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();                                   // also frees both stages for the workgroup's next block
    }
#undef SOL_PV_GLOAD
#undef SOL_PV_LSTORE

    // ---- normalise and store: accumulator lane (l16, lg) register r is query 4*lg + r, column 16*dt + l16 ----
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        float dsum = den[qt];
        dsum += __shfl_xor(dsum, 16);
        dsum += __shfl_xor(dsum, 32);
        const float inv = dsum > 0.f ? 1.0f / dsum : 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float iv = __shfl(inv, 4 * lg + r);
            const int qi = q0 + 16 * qt + 4 * lg + r;
            if (qi < Tn) {
                float *op = o32 + ((int64_t)s * Tn + qi) * (int64_t)(Hq * DH) + (int64_t)h * DH + l16;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) op[dt * 16] = oacc[qt][dt][r] * iv;
            }
        }
    }
    }   // pass
}

// =================================================================================================
// Decode attention (one query per sequence, bf16, HBM-bound): one workgroup of 16 waves per
// (sequence, KV head) serves the HPB = 4 query heads that share that KV head, so K is streamed from
// HBM once and V rows are fetched once if any of the four heads kept them.
//   1. scores on MFMA: A = a tile of 16 keys (each lane loads 16 contiguous bytes of a K row straight
//      from global memory, four tiles in flight per wave), B = the query heads as columns; fp32 scores
//      of all four heads go to LDS.
//   2. selection: the 4 waves of a head hold a quarter of the row each in registers and bisect the
//      key range together, exchanging their ballot counts through LDS once per step.
//   3. softmax numerators back to LDS, 4. V rows gathered where any head kept the key.
// =================================================================================================
constexpr int DEC_WAVES = 16, DEC_BLOCK = DEC_WAVES * 64, DEC_HPB = 4, DEC_GW = DEC_WAVES / DEC_HPB;
// The last phases of the decode kernels: sc holds the softmax numerators of the HPB heads ([HPB][lpad], 0 for
// dropped keys), s_den the per-wave partial denominators ([head][DEC_GW]); o_row receives HPB * DH outputs.
//   4. o = sum_j p_j v_j, reading only V rows kept by at least one head; 5. reduction over lanes and waves.
template <int DH>
__device__ __forceinline__ void decode_pv_tail(float *sc, int lpad, int n, const bf16_t *__restrict__ vbase,
                                               const float *s_den, float *__restrict__ o_row)
{
    constexpr int VEC = 8, LPK = DH / VEC, KPI = DEC_BLOCK / LPK;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // ---- 4. o = sum p_j v_j over rows any head kept ---------------------------------------------------
    const int ks = tid / LPK, cs = tid - ks * LPK;
    float acc[DEC_HPB][VEC];
#pragma unroll
    for (int hh = 0; hh < DEC_HPB; ++hh)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[hh][e] = 0.f;
    constexpr int UV = 4;
    for (int j0 = ks; j0 < n; j0 += KPI * UV) {
        float p[UV][DEC_HPB];
        u32x4_a vv[UV];
        bool any[UV];
#pragma unroll
        for (int u = 0; u < UV; ++u) {
            const int j = j0 + u * KPI;
            any[u] = false;
#pragma unroll
            for (int hh = 0; hh < DEC_HPB; ++hh) {
                p[u][hh] = (j < n) ? sc[hh * lpad + j] : 0.f;
                any[u] |= p[u][hh] != 0.f;
            }
            vv[u] = u32x4_a{0u, 0u, 0u, 0u};
            if (any[u]) vv[u] = *reinterpret_cast<const u32x4_a *>(vbase + (int64_t)j * DH + cs * VEC);
        }
#pragma unroll
        for (int u = 0; u < UV; ++u) {
            if (any[u]) {
#pragma unroll
                for (int wi = 0; wi < 4; ++wi) {
                    const float v0 = __uint_as_float(vv[u][wi] << 16), v1 = __uint_as_float(vv[u][wi] & 0xFFFF0000u);
#pragma unroll
                    for (int hh = 0; hh < DEC_HPB; ++hh) {
                        acc[hh][2 * wi] = fmaf(p[u][hh], v0, acc[hh][2 * wi]);
                        acc[hh][2 * wi + 1] = fmaf(p[u][hh], v1, acc[hh][2 * wi + 1]);
                    }
                }
            }
        }
    }
    // Reduce over the key slots of a wave (lanes with equal cs) by halving butterflies: at each step a lane
    // keeps one half of its values and hands the other half to its partner, so the 4 * VEC values per lane
    // end as 4 * VEC * LPK / 64 fully reduced ones; then across waves in fixed order.
    float *accf = &acc[0][0];
    int fbase = 0;                                             // first flattened (head, element) index this lane keeps
    {
        int nv = DEC_HPB * VEC;
#pragma unroll
        for (int o = LPK; o < 64; o <<= 1) {
            nv >>= 1;
            const bool up = (lane & o) != 0;
#pragma unroll
            for (int i = 0; i < DEC_HPB * VEC / 2; ++i) {
                if (i < nv) {
                    const float keep = up ? accf[i + nv] : accf[i];
                    const float send = up ? accf[i] : accf[i + nv];
                    accf[i] = keep + __shfl_xor(send, o, 64);
                }
            }
            fbase += up ? nv : 0;
        }
    }
    constexpr int NKEEP = DEC_HPB * VEC * LPK / 64;            // 4 (head_dim 64) or 8 (head_dim 128)
    __syncthreads();                                           // all reads of the numerators are done
    float *ored = sc;                                          // [DEC_WAVES][HPB][DH]
    {
        const int hh = fbase / VEC, e0 = fbase - hh * VEC;     // NKEEP values of one head, elements e0..e0+NKEEP-1
        float *dst = ored + ((size_t)w * DEC_HPB + hh) * DH + (lane & (LPK - 1)) * VEC + e0;
#pragma unroll
        for (int i = 0; i < NKEEP; i += 4)
            *reinterpret_cast<f32x4_a *>(dst + i) = f32x4_a{accf[i], accf[i + 1], accf[i + 2], accf[i + 3]};
    }
    __syncthreads();
    for (int idx = tid; idx < DEC_HPB * DH; idx += DEC_BLOCK) {
        const int hh = idx / DH;
        float t = 0.f, dsum = 0.f;
#pragma unroll
        for (int ww = 0; ww < DEC_WAVES; ++ww) t += ored[(size_t)ww * DEC_HPB * DH + idx];
#pragma unroll
        for (int i = 0; i < DEC_GW; ++i) dsum += s_den[hh * DEC_GW + i];
        o_row[idx] = t / dsum;
    }
}

template <int DH, int SLOTS>
__global__ void __launch_bounds__(DEC_BLOCK)
k_attn_decode(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc, const bf16_t *__restrict__ vc,
              float *__restrict__ o32, const RowAct *__restrict__ ra, const int32_t *__restrict__ cache_len,
              const int32_t *__restrict__ seq_order, int L_max, int Hq, int Hkv, float scale, int *flags)
{
    constexpr int KK = DH / 32, SLICE = SLOTS * 64, LPAD = SLICE * DEC_GW, NJ = SLOTS / 4;
    extern __shared__ __align__(16) float sc[];               // [DEC_HPB][LPAD]; later partial O [DEC_WAVES][HPB][DH]
    __shared__ int s_cnt[2][DEC_WAVES];
    __shared__ uint32_t s_min[DEC_WAVES], s_max[DEC_WAVES];
    __shared__ int s_done[2][DEC_HPB];
    __shared__ int s_gt[DEC_WAVES];
    __shared__ float s_den[DEC_WAVES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kvh = blockIdx.x;
    // Longest sequences first: workgroups are handed to compute units in launch order, one per CU, so with
    // mixed cache lengths the last round would otherwise wait for a long row that started late. seq_order
    // (k_seq_order, once per decode step) lists the sequences by decreasing cache length.
    int s = seq_order ? seq_order[blockIdx.y] : (int)blockIdx.y;
    s = __builtin_amdgcn_readfirstlane(s);
    const int p0 = __builtin_amdgcn_readfirstlane(cache_len[s]);
    if (p0 < 0 || p0 + 1 > L_max) {
        if (tid == 0) atomicOr(flags, FLAG_CACHE_OVERFLOW);
        return;
    }
    const int n = p0 + 1;                                      // keys 0..p0 (the new token's key included)
    const int h0 = kvh * DEC_HPB;
    const bf16_t *kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    const bf16_t *vbase = vc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    const int l16 = lane & 15, lg = lane >> 4;

    // ---- 1. scores -----------------------------------------------------------------------------
    {
        bf16x8_a qf[KK];                                       // B operand: column = head (l16 < HPB), zero elsewhere
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            u32x4_a v = {0u, 0u, 0u, 0u};
            if (l16 < DEC_HPB)
                v = *reinterpret_cast<const u32x4_a *>(q + (int64_t)s * (Hq * DH) + (int64_t)(h0 + l16) * DH + kk * 32 + lg * 8);
            qf[kk] = __builtin_bit_cast(bf16x8_a, v);
        }
        const int n_kt = (n + 15) >> 4;
        // two register sets of key tiles: the loads of the next group are in flight while this group is multiplied
        constexpr int U = DH == 64 ? 4 : 2, STEP = DEC_WAVES * U;
        bf16x8_a kfa[U][KK], kfb[U][KK];
#define SOL_DEC_LOADK(KF, KT0_)                                                                            \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                        \
        int key = ((KT0_) + u * DEC_WAVES) * 16 + l16;                                                     \
        if (key >= n) key = n - 1;                                                                         \
        const bf16_t *kp = kbase + (int64_t)key * DH + lg * 8;                                             \
        _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                                  \
            KF[u][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(kp + kk * 32));    \
    }
#define SOL_DEC_MMAK(KF, KT0_)                                                                             \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                        \
        const int kt = (KT0_) + u * DEC_WAVES;                                                             \
        if (kt < n_kt) {                                                                                   \
            floatx4_a acc = {0.f, 0.f, 0.f, 0.f};                                                          \
            _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                              \
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(KF[u][kk], qf[kk], acc, 0, 0, 0);            \
            if (l16 < DEC_HPB) {                                                                           \
                _Pragma("unroll") for (int r = 0; r < 4; ++r) sc[l16 * LPAD + kt * 16 + lg * 4 + r] = acc[r] * scale; \
            }                                                                                              \
        }                                                                                                  \
    }
        int kt0 = w;
        if (kt0 < n_kt) SOL_DEC_LOADK(kfa, kt0);
        for (; kt0 < n_kt; kt0 += 2 * STEP) {
            if (kt0 + STEP < n_kt) SOL_DEC_LOADK(kfb, kt0 + STEP);
            SOL_DEC_MMAK(kfa, kt0);
            if (kt0 + 2 * STEP < n_kt) SOL_DEC_LOADK(kfa, kt0 + 2 * STEP);
            if (kt0 + STEP < n_kt) SOL_DEC_MMAK(kfb, kt0 + STEP);
        }
#undef SOL_DEC_LOADK
#undef SOL_DEC_MMAK
    }
    __syncthreads();

    // ---- 2. selection: DEC_GW waves per head, each with SLICE columns in registers --------------
    const int head = w / DEC_GW, wg = w - head * DEC_GW;
    const int base = wg * SLICE;
    int n_loc = n - base;
    n_loc = n_loc < 0 ? 0 : (n_loc > SLICE ? SLICE : n_loc);   // valid columns held by this wave
    float *row = sc + head * LPAD + base;
    uint32_t key[SLOTS];                                        // the score itself is recovered from its key
    uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (256 * j < n_loc) {
            const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool valid = 256 * j + 4 * lane + e < n_loc;
                const uint32_t kv = valid ? score_key(v[e]) : 0u;
                key[4 * j + e] = kv;
                kmax = kv > kmax ? kv : kmax;
                kmin = (valid && kv < kmin) ? kv : kmin;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * j + e] = 0u;
        }
    }
    kmax = wave_max_u32(kmax);
    kmin = wave_min_u32(kmin);
    if (lane == 0) { s_max[w] = kmax; s_min[w] = kmin; }
    __syncthreads();
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int i = 0; i < DEC_GW; ++i) {
        const uint32_t a = s_min[head * DEC_GW + i], c = s_max[head * DEC_GW + i];
        lo = a < lo ? a : lo;
        hi = c > hi ? c : hi;
    }
    // values read back from LDS are wave-uniform: move them to scalar registers so that the search
    // below is scalar control flow
    lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)lo);
    hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)hi);
    const float mx = score_unkey(hi);                          // the head's best score, always kept
    const RowAct act = ra[s];
    const int b = __builtin_amdgcn_readfirstlane(budget_ceil(act.keep_num, act.keep_den, n));   // 64-bit divide runs on the VALU
    uint32_t thr = 1u;                                         // budget keeps all: every valid key passes
    bool done = b >= n, exact = true;
    // invariant while searching: count(key >= lo) >= b, count(key >= hi + 1) < b. Pivots by regula falsi on
    // g(x) = count(key >= x) - b + 1/2 in the score domain with the Illinois correction (about 7 counting
    // rounds, each a workgroup barrier, instead of about 15 for bisection of the key); after 12 rounds, or when
    // the guess leaves (lo, hi], the midpoint of the key range takes over, which bounds the search.
    float flo = score_unkey(lo), fhi = score_unkey(hi), glo = (float)(n - b) + 0.5f, ghi = 0.5f - (float)b;
    int side = 0;
    for (int it = 0; it < 48; ++it) {
        const int par = it & 1;
        uint32_t mid = 0u;
        if (!done) {
            const float fp = __builtin_fmaf(fhi - flo, glo * __builtin_amdgcn_rcpf(glo - ghi), flo);
            mid = (uint32_t)__builtin_amdgcn_readfirstlane((int)score_key(fp));
            if (it >= 12 || !(mid > lo && mid <= hi)) mid = lo + ((hi - lo + 1u) >> 1);
            const int c = lo < hi ? wave_count_ge<SLOTS>(key, n_loc, mid) : 0;
            if (lane == 0) s_cnt[par][w] = c;
        }
        if (wg == 0 && lane == 0) s_done[par][head] = done || lo >= hi;
        __syncthreads();
        if (!done) {
            if (lo >= hi) { thr = lo; exact = false; done = true; }
            else {
                int cnt = 0;
#pragma unroll
                for (int i = 0; i < DEC_GW; ++i) cnt += s_cnt[par][head * DEC_GW + i];
                cnt = __builtin_amdgcn_readfirstlane(cnt);
                const float g = (float)(cnt - b) + 0.5f;
                if (cnt == b) { thr = mid; done = true; }
                else if (cnt > b) {
                    lo = mid; flo = score_unkey(mid); glo = g;
                    if (side > 0) ghi *= 0.5f;
                    side = 1;
                } else {
                    hi = mid - 1u; fhi = score_unkey(hi); ghi = g;
                    if (side < 0) glo *= 0.5f;
                    side = -1;
                }
            }
        }
        const bool all_done =
            __builtin_amdgcn_readfirstlane(s_done[par][0] & s_done[par][1] & s_done[par][2] & s_done[par][3]) != 0;
        if (all_done) break;                                   // uniform: every wave reads the same flags
    }
    // Ties at the threshold go to the lower columns. Rare for fp32 scores, so the fix-up is a plain
    // loop by the first wave of the head over the row in LDS: tied keys beyond the quota get -inf.
    {
        const bool need = (b < n) && !exact;
        int gt = 0;
        if (need) {
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) gt += __popcll(__ballot(key[i] > thr));
        }
        if (lane == 0) s_gt[w] = gt;
        __syncthreads();
        if (need && wg == 0) {
            int quota = b;
#pragma unroll
            for (int i = 0; i < DEC_GW; ++i) quota -= s_gt[head * DEC_GW + i];
            quota = __builtin_amdgcn_readfirstlane(quota);      // >= 1 tied keys stay
            float *hrow = sc + head * LPAD;
            int taken = 0;
            for (int c0 = 0; c0 < n; c0 += 64) {
                const int col = c0 + lane;
                const bool tie = col < n && score_key(hrow[col]) == thr;
                const unsigned long long bal = __ballot(tie);
                const int rank = taken + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
                if (tie && rank >= quota) hrow[col] = -INFINITY;
                taken += __popcll(bal);
            }
        }
        __syncthreads();
    }

    // ---- 3. softmax numerators back to LDS ----------------------------------------------------------
    // The scores are still in registers (as keys); only a row the tie fix-up rewrote is read back.
    float den = 0.f;
    const bool reread = (b < n) && !exact;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (256 * j < n_loc) {
            f32x4_a v = {0.f, 0.f, 0.f, 0.f};
            if (reread) v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
            f32x4_a p;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t kv = reread ? score_key(v[e]) : key[4 * j + e];
                const float sv = reread ? v[e] : score_unkey(key[4 * j + e]);
                const bool on = (256 * j + 4 * lane + e < n_loc) && kv >= thr;
                p[e] = on ? __expf(sv - mx) : 0.f;
                den += p[e];
            }
            *reinterpret_cast<f32x4_a *>(row + 256 * j + 4 * lane) = p;
        }
    }
    den = wave_sum_dpp(den);
    if (lane == 0) s_den[w] = den;
    __syncthreads();

    decode_pv_tail<DH>(sc, LPAD, n, vbase, s_den, o32 + (int64_t)s * (Hq * DH) + (int64_t)h0 * DH);
}

template <int DH, int SLOTS>
static bool launch_attn_decode_t(const void *q, const void *kc, const void *vc, float *o32, const RowAct *ra,
                                 const int32_t *cache_len, const int32_t *seq_order, int B, int L_max, int Hq, int Hkv,
                                 int *flags, hipStream_t st)
{
    auto kern = k_attn_decode<DH, SLOTS>;
    const size_t lds = (size_t)DEC_HPB * SLOTS * 64 * DEC_GW * 4;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return false;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(Hkv, B), dim3(DEC_BLOCK), lds, st, (const bf16_t *)q, (const bf16_t *)kc,
                       (const bf16_t *)vc, o32, ra, cache_len, seq_order, L_max, Hq, Hkv, 1.0f / sqrtf((float)DH), flags);
    return true;
}

// order[r] = the sequence with the r-th longest cache (equal lengths in index order); identity beyond 1024
// sequences. One workgroup; the lengths are the same for every layer of a decode step.
__global__ void __launch_bounds__(1024)
k_seq_order(const int32_t *__restrict__ len, int n, int32_t *__restrict__ order)
{
    __shared__ int s_len[1024];
    const int tid = threadIdx.x;
    if (n > 1024) {
        for (int i = tid; i < n; i += 1024) order[i] = i;
        return;
    }
    const int my_len = tid < n ? len[tid] : 0;
    s_len[tid] = my_len;
    __syncthreads();
    if (tid < n) {
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const int lj = s_len[j];
            rank += (lj > my_len || (lj == my_len && j < tid)) ? 1 : 0;
        }
        order[rank] = tid;
    }
}

void launch_seq_order(const int32_t *cache_len, int B, int32_t *order, hipStream_t st)
{
    if (B > 0) hipLaunchKernelGGL(k_seq_order, dim3(1), dim3(1024), 0, st, cache_len, B, order);
}

// One query per sequence (T = 1), bf16, 4 query heads per KV head, head_dim 64 / 128, L_max <= 9216.
// seq_order: sequences by decreasing cache length (launch_seq_order), or null for launch order.
bool launch_attn_decode(const void *q, const void *k_cache, const void *v_cache, float *o32, const RowAct *ra,
                        const int32_t *cache_len, const int32_t *seq_order, int B, int L_max, int Hq, int Hkv, int dh,
                        int *flags, hipStream_t st)
{
    if (B <= 0) return true;
    if (!cache_len || Hq != DEC_HPB * Hkv || (dh != 64 && dh != 128) || L_max > 9216) return false;
    const size_t red = (size_t)DEC_WAVES * DEC_HPB * dh * 4;
#define SOL_DEC(SL)                                                                                             \
    if ((size_t)DEC_HPB * SL * 64 * DEC_GW * 4 >= red)                                                           \
        return dh == 64 ? launch_attn_decode_t<64, SL>(q, k_cache, v_cache, o32, ra, cache_len, seq_order, B, L_max, Hq, Hkv, flags, st) \
                        : launch_attn_decode_t<128, SL>(q, k_cache, v_cache, o32, ra, cache_len, seq_order, B, L_max, Hq, Hkv, flags, st)
    if (L_max <= 1024) { SOL_DEC(4); }
    if (L_max <= 2048) { SOL_DEC(8); }
    if (L_max <= 4096) { SOL_DEC(16); }
    if (L_max <= 8192) { SOL_DEC(32); }
    SOL_DEC(36);                                   // 9216 columns: an 8192-token cache plus the tokens being decoded
#undef SOL_DEC
    return false;
}

// =================================================================================================
// Decode attention under the page rule (Appendix "Quest masking", page size S > 1), bf16.
//
// Page metadata: for every page of S contiguous keys of a (sequence, KV head) one row of 2 * dh bf16 values,
// [channel-wise maximum | channel-wise minimum] over the keys of the page written so far. The caller owns
// the buffer ([n_seq][Hkv][ceil(L_max / S)][2 * dh]); k_page_meta_build fills it from a cache,
// k_page_meta_update folds in the key a decode step has just written. With it the page bound
//   sum_c max(q_c max_c, q_c min_c) = [max(q, 0) | min(q, 0)] . [max | min]
// is a dot product of length 2 * dh, i.e. the score kernel's MFMA loop run over metadata rows, and a decode
// step reads 2 / S of K for the bounds plus the K and V rows of the pages it keeps, not all of K.
// =================================================================================================
template <int DH>
__global__ void __launch_bounds__(256)
k_page_meta_build(const bf16_t *__restrict__ kc, const int32_t *__restrict__ len, bf16_t *__restrict__ meta, int S,
                  int L_max, int P_max, int Hkv, const int32_t *__restrict__ first, int extra)
{
    constexpr int LPK = DH / 8, PPB = 256 / LPK;               // lanes per page row, pages per workgroup
    const int s = blockIdx.z, kvh = blockIdx.y;
    const int u = blockIdx.x * PPB + threadIdx.x / LPK, cs = threadIdx.x % LPK;
    int n = len[s] + extra;
    n = n < 0 ? 0 : (n > L_max ? L_max : n);
    const int j0 = u * S;
    if (u >= P_max || j0 >= n) return;
    if (first && j0 + S <= first[s]) return;                   // page wholly before the rewritten keys
    const int j1 = j0 + S < n ? j0 + S : n;
    const bf16_t *kb = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH + cs * 8;
    float mx[8], mn[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { mx[e] = -INFINITY; mn[e] = INFINITY; }
    for (int j = j0; j < j1; ++j) {
        const u32x4_a v = *reinterpret_cast<const u32x4_a *>(kb + (int64_t)j * DH);
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            const float a = __uint_as_float(v[wi] << 16), b = __uint_as_float(v[wi] & 0xFFFF0000u);
            mx[2 * wi] = fmaxf(mx[2 * wi], a); mn[2 * wi] = fminf(mn[2 * wi], a);
            mx[2 * wi + 1] = fmaxf(mx[2 * wi + 1], b); mn[2 * wi + 1] = fminf(mn[2 * wi + 1], b);
        }
    }
    bf16_t *mrow = meta + (((int64_t)s * Hkv + kvh) * P_max + u) * (2 * DH) + cs * 8;
    u32x4_a omx, omn;                                          // extremes of bf16 values are bf16 values: exact
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {
        omx[wi] = (__float_as_uint(mx[2 * wi]) >> 16) | (__float_as_uint(mx[2 * wi + 1]) & 0xFFFF0000u);
        omn[wi] = (__float_as_uint(mn[2 * wi]) >> 16) | (__float_as_uint(mn[2 * wi + 1]) & 0xFFFF0000u);
    }
    *reinterpret_cast<u32x4_a *>(mrow) = omx;
    *reinterpret_cast<u32x4_a *>(mrow + DH) = omn;
}

// the key at position pos[s] (just written) joins its page: first key of a page initialises the row
template <int DH>
__global__ void __launch_bounds__(64)
k_page_meta_update(const bf16_t *__restrict__ kc, const int32_t *__restrict__ pos, bf16_t *__restrict__ meta, int S,
                   int L_max, int P_max, int Hkv)
{
    constexpr int LPK = DH / 8;
    const int s = blockIdx.y, kvh = blockIdx.x, cs = threadIdx.x;
    const int p = pos[s];
    if (cs >= LPK || p < 0 || p >= L_max) return;
    const int u = p / S;
    const u32x4_a v = *reinterpret_cast<const u32x4_a *>(kc + (((int64_t)s * Hkv + kvh) * L_max + p) * DH + cs * 8);
    bf16_t *mrow = meta + (((int64_t)s * Hkv + kvh) * P_max + u) * (2 * DH) + cs * 8;
    u32x4_a omx = v, omn = v;
    if (p != u * S) {
        const u32x4_a amx = *reinterpret_cast<const u32x4_a *>(mrow), amn = *reinterpret_cast<const u32x4_a *>(mrow + DH);
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            const float a = __uint_as_float(v[wi] << 16), b = __uint_as_float(v[wi] & 0xFFFF0000u);
            const float xa = fmaxf(a, __uint_as_float(amx[wi] << 16)), xb = fmaxf(b, __uint_as_float(amx[wi] & 0xFFFF0000u));
            const float na = fminf(a, __uint_as_float(amn[wi] << 16)), nb = fminf(b, __uint_as_float(amn[wi] & 0xFFFF0000u));
            omx[wi] = (__float_as_uint(xa) >> 16) | (__float_as_uint(xb) & 0xFFFF0000u);
            omn[wi] = (__float_as_uint(na) >> 16) | (__float_as_uint(nb) & 0xFFFF0000u);
        }
    }
    *reinterpret_cast<u32x4_a *>(mrow) = omx;
    *reinterpret_cast<u32x4_a *>(mrow + DH) = omn;
}

bool launch_page_meta_build(const void *k_cache, const int32_t *len, void *meta, int n_seq, int L_max, int Hkv, int dh,
                            int S, hipStream_t st, const int32_t *first, int extra)
{
    if (n_seq <= 0) return true;
    if (S < 2 || (dh != 64 && dh != 128)) return false;
    const int P_max = (L_max + S - 1) / S;
    const int ppb = 256 / (dh / 8);
    const dim3 grid((unsigned)((P_max + ppb - 1) / ppb), Hkv, n_seq);
    if (dh == 64) hipLaunchKernelGGL(k_page_meta_build<64>, grid, dim3(256), 0, st, (const bf16_t *)k_cache, len, (bf16_t *)meta, S, L_max, P_max, Hkv, first, extra);
    else hipLaunchKernelGGL(k_page_meta_build<128>, grid, dim3(256), 0, st, (const bf16_t *)k_cache, len, (bf16_t *)meta, S, L_max, P_max, Hkv, first, extra);
    return true;
}

bool launch_page_meta_update(const void *k_cache, const int32_t *pos, void *meta, int n_seq, int L_max, int Hkv, int dh,
                             int S, hipStream_t st)
{
    if (n_seq <= 0) return true;
    if (S < 2 || (dh != 64 && dh != 128)) return false;
    const int P_max = (L_max + S - 1) / S;
    if (dh == 64) hipLaunchKernelGGL(k_page_meta_update<64>, dim3(Hkv, n_seq), dim3(64), 0, st, (const bf16_t *)k_cache, pos, (bf16_t *)meta, S, L_max, P_max, Hkv);
    else hipLaunchKernelGGL(k_page_meta_update<128>, dim3(Hkv, n_seq), dim3(64), 0, st, (const bf16_t *)k_cache, pos, (bf16_t *)meta, S, L_max, P_max, Hkv);
    return true;
}

// [max(q, 0) | min(q, 0)] of a pair of packed bf16 values: element e of the doubled query row
__device__ __forceinline__ uint32_t q_split_pair(uint32_t x, bool neg_half)
{
    const bool nlo = (x & 0x8000u) != 0u, nhi = (x & 0x80000000u) != 0u;
    const uint32_t lo = (nlo == neg_half) ? (x & 0xFFFFu) : 0u;
    const uint32_t hi = (nhi == neg_half) ? (x & 0xFFFF0000u) : 0u;
    return lo | hi;
}

// One workgroup of 16 waves per (sequence, KV head), the 4 query heads of the group together:
//   1. page bounds on MFMA from the metadata rows (fp32, to LDS);
//   2. per head, the threshold of the top ceil(b / S) bounds (same joint search as the per-key kernel, over
//      pages), ties to the lower page; the kept pages of the 4 heads as bit flags in LDS;
//   3. scores of the keys of kept pages and of the sink / window keys (K tiles no head needs are skipped),
//      -inf elsewhere;  4. softmax numerators;  5. V rows gathered where any head kept the key.
template <int DH, int SLOTS>
__global__ void __launch_bounds__(DEC_BLOCK)
k_attn_decode_paged(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc, const bf16_t *__restrict__ vc,
                    const bf16_t *__restrict__ meta, float *__restrict__ o32, const RowAct *__restrict__ ra,
                    const int32_t *__restrict__ cache_len, const int32_t *__restrict__ seq_order, int L_max, int P_max,
                    int lpad, int Hq, int Hkv, float scale, AttnOpts opt, int *flags)
{
    constexpr int KK = DH / 32, KK2 = 2 * KK, SLICE = SLOTS * 64, PPAD = SLICE * DEC_GW, NJ = SLOTS / 4;
    extern __shared__ __align__(16) float sc[];               // page bounds [HPB][PPAD], then scores [HPB][lpad], then partial O
    __shared__ int s_pk[PPAD];                                 // bit h: head h keeps the page
    __shared__ int s_cnt[2][DEC_WAVES];
    __shared__ uint32_t s_min[DEC_WAVES], s_max[DEC_WAVES];
    __shared__ int s_done[2][DEC_HPB];
    __shared__ int s_gt[DEC_WAVES];
    __shared__ float s_den[DEC_WAVES], s_mx[DEC_WAVES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kvh = blockIdx.x;
    const int s = __builtin_amdgcn_readfirstlane(seq_order ? seq_order[blockIdx.y] : (int)blockIdx.y);
    const int p0 = __builtin_amdgcn_readfirstlane(cache_len[s]);
    if (p0 < 0 || p0 + 1 > L_max) {
        if (tid == 0) atomicOr(flags, FLAG_CACHE_OVERFLOW);
        return;
    }
    const int n = p0 + 1;
    const int S = opt.page;
    const int n_pages = (n + S - 1) / S;
    const int h0 = kvh * DEC_HPB;
    const bf16_t *kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    const bf16_t *vbase = vc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    const bf16_t *mbase = meta + ((int64_t)s * Hkv + kvh) * (int64_t)P_max * (2 * DH);
    const int l16 = lane & 15, lg = lane >> 4;
    const RowAct act = ra[s];
    const int b = __builtin_amdgcn_readfirstlane(budget_ceil(act.keep_num, act.keep_den, n));
    int np = (b + S - 1) / S;
    np = np < n_pages ? np : n_pages;
    const bool all_pages = b >= n || np >= n_pages;            // every page (or, b >= n, every key) is kept
    const bool dense = b >= n;
    const int head = w / DEC_GW, wg = w - head * DEC_GW;

    for (int u = tid; u < PPAD; u += DEC_BLOCK) s_pk[u] = 0;

    // the query heads as MFMA B operand (column = head)
    u32x4_a qraw[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        qraw[kk] = u32x4_a{0u, 0u, 0u, 0u};
        if (l16 < DEC_HPB)
            qraw[kk] = *reinterpret_cast<const u32x4_a *>(q + (int64_t)s * (Hq * DH) + (int64_t)(h0 + l16) * DH + kk * 32 + lg * 8);
    }

    if (!all_pages) {
        // ---- 1. page bounds ---------------------------------------------------------------------
        bf16x8_a qq[KK2];                                      // [max(q, 0) | min(q, 0)], 2 * DH long
#pragma unroll
        for (int kk = 0; kk < KK2; ++kk) {
            u32x4_a v;
#pragma unroll
            for (int wi = 0; wi < 4; ++wi) v[wi] = q_split_pair(qraw[kk % KK][wi], kk >= KK);
            qq[kk] = __builtin_bit_cast(bf16x8_a, v);
        }
        const int n_pt = (n_pages + 15) >> 4;
        constexpr int U = 2;
        for (int pt0 = w; pt0 < n_pt; pt0 += DEC_WAVES * U) {
            bf16x8_a mf[U][KK2];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int pg = (pt0 + u * DEC_WAVES) * 16 + l16;
                if (pg >= n_pages) pg = n_pages - 1;
                const bf16_t *mp = mbase + (int64_t)pg * (2 * DH) + lg * 8;
#pragma unroll
                for (int kk = 0; kk < KK2; ++kk)
                    mf[u][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(mp + kk * 32));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int pt = pt0 + u * DEC_WAVES;
                if (pt < n_pt) {
                    floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < KK2; ++kk)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mf[u][kk], qq[kk], acc, 0, 0, 0);
                    if (l16 < DEC_HPB) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) sc[l16 * PPAD + pt * 16 + lg * 4 + r] = acc[r];
                    }
                }
            }
        }
        __syncthreads();

        // ---- 2. the np best pages of each head ------------------------------------------------------
        const int base = wg * SLICE;
        int n_loc = n_pages - base;
        n_loc = n_loc < 0 ? 0 : (n_loc > SLICE ? SLICE : n_loc);
        float *row = sc + head * PPAD + base;
        uint32_t key[SLOTS];
        uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (256 * j < n_loc) {
                const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool valid = 256 * j + 4 * lane + e < n_loc;
                    const uint32_t kv = valid ? score_key(v[e]) : 0u;
                    key[4 * j + e] = kv;
                    kmax = kv > kmax ? kv : kmax;
                    kmin = (valid && kv < kmin) ? kv : kmin;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) key[4 * j + e] = 0u;
            }
        }
        kmax = wave_max_u32(kmax);
        kmin = wave_min_u32(kmin);
        if (lane == 0) { s_max[w] = kmax; s_min[w] = kmin; }
        __syncthreads();
        uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
        for (int i = 0; i < DEC_GW; ++i) {
            const uint32_t a = s_min[head * DEC_GW + i], c = s_max[head * DEC_GW + i];
            lo = a < lo ? a : lo;
            hi = c > hi ? c : hi;
        }
        lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)lo);
        hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)hi);
        uint32_t thr = 1u;
        bool done = false, exact = true;
        // invariant: count(key >= lo) >= np, count(key >= hi + 1) < np; regula falsi with the Illinois correction
        // on g(x) = count(key >= x) - np + 1/2, the midpoint of the key range after 12 rounds or a bad guess
        float flo = score_unkey(lo), fhi = score_unkey(hi), glo = (float)(n_pages - np) + 0.5f, ghi = 0.5f - (float)np;
        int side = 0;
        for (int it = 0; it < 48; ++it) {
            const int par = it & 1;
            uint32_t mid = 0u;
            if (!done) {
                const float fp = __builtin_fmaf(fhi - flo, glo * __builtin_amdgcn_rcpf(glo - ghi), flo);
                mid = (uint32_t)__builtin_amdgcn_readfirstlane((int)score_key(fp));
                if (it >= 12 || !(mid > lo && mid <= hi)) mid = lo + ((hi - lo + 1u) >> 1);
                const int c = lo < hi ? wave_count_ge<SLOTS>(key, n_loc, mid) : 0;
                if (lane == 0) s_cnt[par][w] = c;
            }
            if (wg == 0 && lane == 0) s_done[par][head] = done || lo >= hi;
            __syncthreads();
            if (!done) {
                if (lo >= hi) { thr = lo; exact = false; done = true; }
                else {
                    int cnt = 0;
#pragma unroll
                    for (int i = 0; i < DEC_GW; ++i) cnt += s_cnt[par][head * DEC_GW + i];
                    cnt = __builtin_amdgcn_readfirstlane(cnt);
                    const float g = (float)(cnt - np) + 0.5f;
                    if (cnt == np) { thr = mid; done = true; }
                    else if (cnt > np) {
                        lo = mid; flo = score_unkey(mid); glo = g;
                        if (side > 0) ghi *= 0.5f;
                        side = 1;
                    } else {
                        hi = mid - 1u; fhi = score_unkey(hi); ghi = g;
                        if (side < 0) glo *= 0.5f;
                        side = -1;
                    }
                }
            }
            const bool all_done =
                __builtin_amdgcn_readfirstlane(s_done[par][0] & s_done[par][1] & s_done[par][2] & s_done[par][3]) != 0;
            if (all_done) break;
        }
        // ties at the threshold go to the lower pages: the first wave of the head walks the row
        {
            const bool need = !exact;
            int gt = 0;
            if (need) {
#pragma unroll
                for (int i = 0; i < SLOTS; ++i) gt += __popcll(__ballot(key[i] > thr));
            }
            if (lane == 0) s_gt[w] = gt;
            __syncthreads();
            if (need && wg == 0) {
                int quota = np;
#pragma unroll
                for (int i = 0; i < DEC_GW; ++i) quota -= s_gt[head * DEC_GW + i];
                quota = __builtin_amdgcn_readfirstlane(quota);
                float *hrow = sc + head * PPAD;
                int taken = 0;
                for (int c0 = 0; c0 < n_pages; c0 += 64) {
                    const int col = c0 + lane;
                    const bool tie = col < n_pages && score_key(hrow[col]) == thr;
                    const unsigned long long bal = __ballot(tie);
                    const int rank = taken + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
                    if (tie && rank >= quota) hrow[col] = -INFINITY;
                    taken += __popcll(bal);
                }
            }
            __syncthreads();
        }
        // kept pages of this head -> flags
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (256 * j < n_loc) {
                const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int u = 256 * j + 4 * lane + e;
                    if (u < n_loc && score_key(v[e]) >= thr) atomicOr(&s_pk[base + u], 1 << head);
                }
            }
        }
    }
    __syncthreads();                                           // flags complete; the page bounds in sc are dead

    // ---- 3. scores of the kept keys ---------------------------------------------------------------
    const int sink_end = opt.n_sink < n ? opt.n_sink : n;
    int win_begin = n - opt.n_window;
    win_begin = win_begin < sink_end ? sink_end : win_begin;
    {
        bf16x8_a qf[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[kk] = __builtin_bit_cast(bf16x8_a, qraw[kk]);
        const int n_kt = (n + 15) >> 4;
        constexpr int U = 4;
        for (int kt0 = w; kt0 < n_kt; kt0 += DEC_WAVES * U) {
            bf16x8_a kf[U][KK];
            bool need[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kt = kt0 + u * DEC_WAVES;
                const int j0 = kt * 16, j1 = j0 + 15 < n - 1 ? j0 + 15 : n - 1;
                bool nd = false;
                if (kt < n_kt) {
                    nd = all_pages || j0 < sink_end || j1 >= win_begin;
                    if (!nd)
                        for (int pg = j0 / S; pg <= j1 / S; ++pg) nd |= s_pk[pg] != 0;
                }
                need[u] = __builtin_amdgcn_readfirstlane((int)nd) != 0;
                if (need[u]) {
                    int key = j0 + l16;
                    if (key >= n) key = n - 1;
                    const bf16_t *kp = kbase + (int64_t)key * DH + lg * 8;
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk)
                        kf[u][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(kp + kk * 32));
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kt = kt0 + u * DEC_WAVES;
                if (kt < n_kt) {
                    floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
                    if (need[u]) {
#pragma unroll
                        for (int kk = 0; kk < KK; ++kk)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[u][kk], qf[kk], acc, 0, 0, 0);
                    }
                    if (l16 < DEC_HPB) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int j = kt * 16 + lg * 4 + r;
                            bool kept = false;
                            if (need[u] && j < n)
                                kept = dense || j < sink_end || j >= win_begin || all_pages || ((s_pk[j / S] >> l16) & 1) != 0;
                            sc[l16 * lpad + j] = kept ? acc[r] * scale : -INFINITY;
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- 4. softmax numerators over the kept keys ---------------------------------------------------
    {
        float *row = sc + head * lpad;
        float mx = -INFINITY;
        for (int j0 = wg * 256; j0 < n; j0 += DEC_GW * 256) {
            const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + j0 + 4 * lane);
#pragma unroll
            for (int e = 0; e < 4; ++e) mx = (j0 + 4 * lane + e < n) ? fmaxf(mx, v[e]) : mx;
        }
        mx = wave_reduce_dpp<float>(mx, -INFINITY, [](float x, float y) { return fmaxf(x, y); });
        if (lane == 0) s_mx[w] = mx;
        __syncthreads();
        mx = s_mx[head * DEC_GW];
#pragma unroll
        for (int i = 1; i < DEC_GW; ++i) mx = fmaxf(mx, s_mx[head * DEC_GW + i]);
        float den = 0.f;
        for (int j0 = wg * 256; j0 < n; j0 += DEC_GW * 256) {
            const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + j0 + 4 * lane);
            f32x4_a p;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                p[e] = (j0 + 4 * lane + e < n) ? __expf(v[e] - mx) : 0.f;     // exp(-inf) = 0 for dropped keys
                den += p[e];
            }
            *reinterpret_cast<f32x4_a *>(row + j0 + 4 * lane) = p;
        }
        den = wave_sum_dpp(den);
        if (lane == 0) s_den[w] = den;
        __syncthreads();
    }
    decode_pv_tail<DH>(sc, lpad, n, vbase, s_den, o32 + (int64_t)s * (Hq * DH) + (int64_t)h0 * DH);
}

template <int DH, int SLOTS>
static bool launch_attn_decode_paged_t(const void *q, const void *kc, const void *vc, const void *meta, float *o32,
                                       const RowAct *ra, const int32_t *cache_len, const int32_t *seq_order, int B,
                                       int L_max, int P_max, int lpad, int Hq, int Hkv, AttnOpts opt, int *flags,
                                       hipStream_t st)
{
    auto kern = k_attn_decode_paged<DH, SLOTS>;
    size_t lds = (size_t)DEC_HPB * lpad * 4;
    const size_t pg = (size_t)DEC_HPB * SLOTS * 64 * DEC_GW * 4, red = (size_t)DEC_WAVES * DEC_HPB * DH * 4;
    lds = lds < pg ? pg : lds;
    lds = lds < red ? red : lds;
    if (lds + (size_t)SLOTS * 64 * DEC_GW * 4 + 1024 > 160 * 1024) return false;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                150 * 1024) != hipSuccess)
            return false;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(Hkv, B), dim3(DEC_BLOCK), lds, st, (const bf16_t *)q, (const bf16_t *)kc,
                       (const bf16_t *)vc, (const bf16_t *)meta, o32, ra, cache_len, seq_order, L_max, P_max, lpad, Hq, Hkv,
                       1.0f / sqrtf((float)DH), opt, flags);
    return true;
}

// One query per sequence under the page rule, with caller-kept page metadata (page_meta_build / _update).
// bf16, 4 query heads per KV head, head_dim 64 / 128, at most 3072 pages and about 9000 keys.
bool launch_attn_decode_paged(const void *q, const void *k_cache, const void *v_cache, const void *meta, float *o32,
                              const RowAct *ra, const int32_t *cache_len, const int32_t *seq_order, int B, int L_max, int Hq,
                              int Hkv, int dh, AttnOpts opt, int *flags, hipStream_t st)
{
    if (B <= 0) return true;
    if (!cache_len || !meta || opt.page < 2 || Hq != DEC_HPB * Hkv || (dh != 64 && dh != 128)) return false;
    const int P_max = (L_max + opt.page - 1) / opt.page;
    const int lpad = (L_max + 1023) & ~1023;                   // rows are walked in steps of 4 waves x 256 columns
    if ((size_t)DEC_HPB * lpad * 4 > 148 * 1024) return false;
#define SOL_DECP(SL)                                                                                            \
    if (P_max <= SL * 64 * DEC_GW)                                                                              \
        return dh == 64 ? launch_attn_decode_paged_t<64, SL>(q, k_cache, v_cache, meta, o32, ra, cache_len, seq_order, B, \
                                                             L_max, P_max, lpad, Hq, Hkv, opt, flags, st)       \
                        : launch_attn_decode_paged_t<128, SL>(q, k_cache, v_cache, meta, o32, ra, cache_len, seq_order, B, \
                                                              L_max, P_max, lpad, Hq, Hkv, opt, flags, st)
    SOL_DECP(4);
    SOL_DECP(8);
    SOL_DECP(12);
#undef SOL_DECP
    return false;
}

// V cache [s][kvh][key][dh] -> vt [s][kvh][dh][lpadv] for keys < pos0[s] + Tn, zero beyond (lpadv a multiple of 64).
// 16 bytes per lane on both sides of memory: 8 channels of a key in, 8 keys of a channel out; the tile's LDS rows are
// DH + 2 elements apart (an odd number of words), which puts the 8 keys a lane gathers for its output, and the lanes
// of a wave, on different banks.
template <int DH>
__global__ void __launch_bounds__(256)
k_transpose_v(const bf16_t *__restrict__ vc, bf16_t *__restrict__ vt, const int32_t *__restrict__ pos0, int Tn, int L_max,
              int Hkv, int lpadv)
{
    constexpr int KP = DH / 8;                               // 16-byte pieces per key
    __shared__ __align__(4) bf16_t tile[64][DH + 2];
    const int kb = blockIdx.x * 64, kvh = blockIdx.y, s = blockIdx.z;
    const int p0 = pos0 ? pos0[s] : 0;
    int len = p0 + Tn;
    if (p0 < 0 || len > L_max) len = 0;
    const bf16_t *src = vc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    bf16_t *dst = vt + ((int64_t)s * Hkv + kvh) * (int64_t)DH * lpadv;
    for (int idx = threadIdx.x; idx < 64 * KP; idx += 256) {
        const int k = idx / KP, p = idx - k * KP;
        u32x4_a v = {0u, 0u, 0u, 0u};
        if (kb + k < len) v = *reinterpret_cast<const u32x4_a *>(src + (int64_t)(kb + k) * DH + p * 8);
        uint32_t *row = reinterpret_cast<uint32_t *>(&tile[k][p * 8]);
#pragma unroll
        for (int e = 0; e < 4; ++e) row[e] = v[e];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < DH * 8; idx += 256) {
        const int d = idx >> 3, kp = idx & 7;                // channel d, keys kb + 8 * kp .. + 7
        if (kb + kp * 8 < lpadv) {
            u32x4_a o;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = (uint32_t)tile[kp * 8 + 2 * e][d] | ((uint32_t)tile[kp * 8 + 2 * e + 1][d] << 16);
            *reinterpret_cast<u32x4_a *>(dst + (int64_t)d * lpadv + kb + kp * 8) = o;
        }
    }
}

// K cache [s][kvh][key][dh] -> kfr [s][kvh][tile of 16 keys][dh / 32][64 lanes][8]: lane (l16, lg) of piece kk holds
// channels 32*kk + 8*lg .. + 7 of key 16*tile + l16, the A operand of mfma_f32_16x16x32_bf16 for that tile; keys from
// pos0[s] + Tn on are zero. attn_lpad64(L_max) keys per (s, kvh).
template <int DH>
__global__ void __launch_bounds__(256)
k_frag_k(const bf16_t *__restrict__ kc, bf16_t *__restrict__ kfr, const int32_t *__restrict__ pos0, int Tn, int L_max, int Hkv,
         int lpad)
{
    constexpr int KP = DH / 8, KK = DH / 32;                // 16-byte pieces per key
    const int kb = blockIdx.x * 64, kvh = blockIdx.y, s = blockIdx.z;
    const int p0 = pos0 ? pos0[s] : 0;
    int len = p0 + Tn;
    if (p0 < 0 || len > L_max) len = 0;
    const bf16_t *src = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    bf16_t *dst = kfr + ((int64_t)s * Hkv + kvh) * (int64_t)lpad * DH;
    for (int idx = threadIdx.x; idx < 64 * KP; idx += 256) {
        const int key = kb + idx / KP, p = idx % KP;
        if (key >= lpad) break;
        u32x4_a v = {0u, 0u, 0u, 0u};
        if (key < len) v = *reinterpret_cast<const u32x4_a *>(src + (int64_t)key * DH + p * 8);
        const int tile = key >> 4, l16 = key & 15, kk = p >> 2, lg = p & 3;
        *reinterpret_cast<u32x4_a *>(dst + ((int64_t)(tile * KK + kk) * 64 + lg * 16 + l16) * 8) = v;
    }
}

// rows whose key count lies in (n_lo, n_hi] (all rows by default); SLOTS * 64 >= min(n_hi, L_max) is the caller's business
template <int BQ, int SLOTS, int DH, int NW, bool PRE = false, bool KF = false>
static bool launch_attn_select_t(const void *q, const void *kc, SelRow *sel, const RowAct *ra, const int32_t *pos0,
                                 int n_seq, int Tn, int L_max, int Hq, int Hkv, hipStream_t st, PrefixView pv = PrefixView(),
                                 int n_lo = 0, int n_hi = 1 << 30)
{
    auto kern = k_attn_select<BQ, SLOTS, DH, NW, PRE, KF>;
    const size_t lds = (size_t)BQ * (SLOTS * 64 + 4) * 4;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return false;
        attr_done = true;
    }
    // workgroups per (sequence, head): enough to fill the chip about eight times over, at most one per block
    int t_range = (n_hi < L_max ? n_hi : L_max) - n_lo;     // no sequence has more rows than that in the range
    if (t_range > Tn) t_range = Tn;
    if (t_range <= 0) return true;
    const int n_qb = (t_range + BQ - 1) / BQ;
    int nb = (int)((4096 + (int64_t)Hq * n_seq - 1) / ((int64_t)Hq * n_seq));
    if (nb > n_qb) nb = n_qb;
    if (nb < 1) nb = 1;
    hipLaunchKernelGGL(kern, dim3(nb, Hq, n_seq), dim3(NW * 64), lds, st, (const bf16_t *)q, (const bf16_t *)kc, sel, ra,
                       pos0, Tn, L_max, Hq, Hkv, 1.0f / sqrtf((float)DH), nb, pv, n_lo, n_hi);
    return true;
}

template <int DH, int G, bool PRE = false>
static bool launch_attn_pv_t(const void *q, const void *kc, const void *vt, const SelRow *sel, float *o32,
                             const int32_t *pos0, int n_seq, int Tn, int L_max, int Hq, int Hkv, int lpadv, hipStream_t st,
                             PrefixView pv = PrefixView())
{
    const size_t lds = 4 * (size_t)64 * DH * 2;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(k_attn_pv<DH, G, PRE, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(k_attn_pv<DH, G, PRE, 2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return false;
        attr_done = true;
    }
    if (Tn <= 16)                                            // one tile of 16 query rows per workgroup
        hipLaunchKernelGGL((k_attn_pv<DH, G, PRE, 1>), dim3(1, Hkv, n_seq), dim3(G * 64), lds, st, (const bf16_t *)q,
                           (const bf16_t *)kc, (const bf16_t *)vt, sel, o32, pos0, Tn, L_max, Hq, Hkv, lpadv,
                           1.0f / sqrtf((float)DH), pv);
    else
        hipLaunchKernelGGL((k_attn_pv<DH, G, PRE, 2>), dim3(((Tn + 31) / 32 + 1) / 2, Hkv, n_seq), dim3(G * 64), lds, st,
                           (const bf16_t *)q, (const bf16_t *)kc, (const bf16_t *)vt, sel, o32, pos0, Tn, L_max, Hq, Hkv, lpadv,
                           1.0f / sqrtf((float)DH), pv);
    return true;
}

// =================================================================================================
// Batched bf16 attention under the page rule (page size S a power of two, 4 <= S <= 64), sink / window keys.
//   k_page_prefix_meta : pm[j] = channel-wise [max | min] over the keys of j's page up to j (2 * dh values per key).
//                        The last key of a full page carries the page's extremes; row p is the partial page of the
//                        query at position p.
//   k_attn_select_pages: per (16 query rows, head): page bounds [max(q,0) | min(q,0)] . pm on MFMA (full pages as one
//                        tile product, the partial page of every query as the diagonal of one more tile), then per
//                        row the top ceil(b / S) bounds, ties to the lower page -> a bit mask of kept pages.
//   k_attn_pv_pages    : k_attn_pv with the mask (and the forced keys) as keep rule and a running maximum, since the
//                        largest kept score is not known beforehand.
// =================================================================================================
template <int DH>
__global__ void __launch_bounds__(256)
k_page_prefix_meta(const bf16_t *__restrict__ kc, const int32_t *__restrict__ pos0, bf16_t *__restrict__ pm, int Tn, int S,
                   int L_max, int Hkv)
{
    constexpr int LPK = DH / 8, PPB = 256 / LPK;
    const int s = blockIdx.z, kvh = blockIdx.y;
    const int u = blockIdx.x * PPB + threadIdx.x / LPK, cs = threadIdx.x % LPK;
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) return;
    const int n = p0 + Tn, j0 = u * S;
    if (j0 >= n) return;
    const int j1 = j0 + S < n ? j0 + S : n;
    const bf16_t *kb = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH + cs * 8;
    bf16_t *pb = pm + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * (2 * DH) + cs * 8;
    float mx[8], mn[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { mx[e] = -INFINITY; mn[e] = INFINITY; }
    for (int j = j0; j < j1; ++j) {
        const u32x4_a v = *reinterpret_cast<const u32x4_a *>(kb + (int64_t)j * DH);
        u32x4_a omx, omn;
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            const float a = __uint_as_float(v[wi] << 16), b = __uint_as_float(v[wi] & 0xFFFF0000u);
            mx[2 * wi] = fmaxf(mx[2 * wi], a); mn[2 * wi] = fminf(mn[2 * wi], a);
            mx[2 * wi + 1] = fmaxf(mx[2 * wi + 1], b); mn[2 * wi + 1] = fminf(mn[2 * wi + 1], b);
            omx[wi] = (__float_as_uint(mx[2 * wi]) >> 16) | (__float_as_uint(mx[2 * wi + 1]) & 0xFFFF0000u);
            omn[wi] = (__float_as_uint(mn[2 * wi]) >> 16) | (__float_as_uint(mn[2 * wi + 1]) & 0xFFFF0000u);
        }
        *reinterpret_cast<u32x4_a *>(pb + (int64_t)j * (2 * DH)) = omx;
        *reinterpret_cast<u32x4_a *>(pb + (int64_t)j * (2 * DH) + DH) = omn;
    }
}

// PRE (shared prefix, as in k_attn_select): pm holds the metadata rows of the sequence's own keys (positions pv.P..,
// [n_seq][Hkv][pv.crows][2 * DH]), pv.pm those of the prefix keys of input s / pv.K ([inputs][Hkv][pv.P][2 * DH]);
// pv.P is a multiple of 16 pages, so a tile of 16 pages lies on one side.
template <int DH, int W, bool PRE>
__global__ void __launch_bounds__(256)
k_attn_select_pages(const bf16_t *__restrict__ q, const bf16_t *__restrict__ pm, unsigned long long *__restrict__ selp,
                    const RowAct *__restrict__ ra, const int32_t *__restrict__ pos0, int Tn, int L_max, int Hq, int Hkv,
                    int log2S, PrefixView pv)
{
    constexpr int KK = DH / 32, KK2 = 2 * KK, PS = 64 * W + 4, BQ = 16;
    __shared__ float sb[BQ][PS];                             // bounds of the full pages, [query][page]
    __shared__ float sd[BQ];                                 // bound of each query's own (partial) page
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q0 = blockIdx.x * BQ, h = blockIdx.y, s = blockIdx.z;
    const int kvh = h / (Hq / Hkv);
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) return;
    const int S = 1 << log2S;
    const int q_last = (q0 + BQ - 1 < Tn ? q0 + BQ - 1 : Tn - 1);
    const int u_max = (p0 + q_last) >> log2S;                // last page any query of the block touches
    const bf16_t *pmb = pm + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * (2 * DH);
    const bf16_t *pmb_pre = nullptr;
    if constexpr (PRE) {                                     // own rows addressed by absolute key: base minus P rows
        pmb = pm + ((int64_t)s * Hkv + kvh) * (int64_t)pv.crows * (2 * DH) - (int64_t)pv.P * (2 * DH);
        pmb_pre = pv.pm + ((int64_t)(s / pv.K) * Hkv + kvh) * (int64_t)pv.P * (2 * DH);
    }

    // queries as MFMA B operand: column l16 = query q0 + l16, doubled row [max(q, 0) | min(q, 0)]
    bf16x8_a qq[KK2];
    {
        const int qi = q0 + l16 < Tn ? q0 + l16 : Tn - 1;
        const bf16_t *qp = q + ((int64_t)s * Tn + qi) * (int64_t)(Hq * DH) + (int64_t)h * DH + lg * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const u32x4_a raw = *reinterpret_cast<const u32x4_a *>(qp + kk * 32);
            u32x4_a a, b;
#pragma unroll
            for (int wi = 0; wi < 4; ++wi) { a[wi] = q_split_pair(raw[wi], false); b[wi] = q_split_pair(raw[wi], true); }
            qq[kk] = __builtin_bit_cast(bf16x8_a, a);
            qq[KK + kk] = __builtin_bit_cast(bf16x8_a, b);
        }
    }
    // full pages: tile pt holds pages 16 pt .. 16 pt + 15; page u is read from the row of its last key
    const int n_pt = (u_max + 16) >> 4;
    for (int pt = w; pt < n_pt; pt += 4) {
        int j = (((pt * 16 + l16) + 1) << log2S) - 1;
        j = j < L_max ? j : L_max - 1;                       // pages past the live keys are masked below
        const bf16_t *mp = ((PRE && ((pt * 16) << log2S) < pv.P) ? pmb_pre : pmb) + (int64_t)j * (2 * DH) + lg * 8;
        floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK2; ++kk) {
            const bf16x8_a mf = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(mp + kk * 32));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mf, qq[kk], acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) sb[l16][pt * 16 + lg * 4 + r] = acc[r];
    }
    if (w == 3) {                                            // the queries' own pages: row m = the key of query m; diagonal
        int j = p0 + q0 + l16;
        j = j < p0 + Tn ? j : p0 + Tn - 1;
        const bf16_t *mp = pmb + (int64_t)j * (2 * DH) + lg * 8;
        floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK2; ++kk) {
            const bf16x8_a mf = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(mp + kk * 32));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mf, qq[kk], acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (lg * 4 + r == l16) sd[l16] = acc[r];
    }
    __syncthreads();

    // ---- per query row: the top ceil(b / S) pages ------------------------------------------------
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int i = 4 * w; i < 4 * w + 4; ++i) {
        const int qi = q0 + i;
        if (qi >= Tn) break;                                 // uniform
        const int p = p0 + qi, n = p + 1, u_p = p >> log2S, npg = u_p + 1;
        const RowAct act = ra[(int64_t)s * Tn + qi];
        const int b = __builtin_amdgcn_readfirstlane(budget_ceil(act.keep_num, act.keep_den, n));
        int np = (b + S - 1) >> log2S;
        np = np < npg ? np : npg;
        unsigned long long mask[W];
        if (b >= n || np >= npg) {
#pragma unroll
            for (int ww = 0; ww < W; ++ww) mask[ww] = ~0ull;
        } else {
            uint32_t key[W];
            uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
#pragma unroll
            for (int ww = 0; ww < W; ++ww) {
                const int u = 64 * ww + lane;
                const float v = u < u_p ? sb[i][u] : sd[i];
                key[ww] = u <= u_p ? score_key(v) : 0u;
                if (u <= u_p) { kmax = key[ww] > kmax ? key[ww] : kmax; kmin = key[ww] < kmin ? key[ww] : kmin; }
            }
            uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_min_u32(kmin));
            uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_max_u32(kmax));
            auto count_ge = [&](uint32_t t) -> int {
                int c = 0;
#pragma unroll
                for (int ww = 0; ww < W; ++ww) c += __popcll(__ballot(key[ww] >= t));
                return c;
            };
            bool exact = false;                              // invariant: count(key >= lo) >= np, count(key >= hi + 1) < np
            while (lo < hi) {
                const uint32_t mid = lo + ((hi - lo + 1u) >> 1);
                const int c = count_ge(mid);
                if (c == np) { lo = mid; exact = true; break; }
                if (c > np) lo = mid; else hi = mid - 1u;
            }
            const uint32_t thr = lo;
            int quota = 64 * W;                              // tied pages kept, lowest pages first
            if (!exact) {
                const int n_ge = count_ge(thr);
                if (n_ge > np) quota = np - (thr == 0xFFFFFFFFu ? 0 : count_ge(thr + 1u));
            }
#pragma unroll
            for (int ww = 0; ww < W; ++ww) {
                const bool tie = key[ww] == thr && 64 * ww + lane <= u_p;
                const unsigned long long bal = __ballot(tie);
                const bool keep = key[ww] > thr || (tie && __popcll(bal & lt_mask) < quota);
                mask[ww] = __ballot(keep);
                const int total = __popcll(bal);
                quota = quota > total ? quota - total : 0;
            }
        }
        if (lane == 0) {
            unsigned long long *o = selp + (((int64_t)s * Tn + qi) * Hq + h) * W;
#pragma unroll
            for (int ww = 0; ww < W; ++ww) o[ww] = mask[ww];
        }
    }
}

// maximum over the four lanes l16, l16 + 16, l16 + 32, l16 + 48 with the gfx950 lane-swap instructions (vector ALU
// only: v_permlane32_swap exchanges the upper half of one operand with the lower half of the other,
// v_permlane16_swap the odd rows of 16 lanes of one with the even rows of the other)
typedef uint32_t u32x2_a __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_over_lane_groups(float v)
{
    const u32x2_a a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const u32x2_a b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// PRE: two-segment addressing as in k_attn_pv. NQT: query tiles of 16 rows per workgroup (2; 1 for passes of at most
// 16 rows per sequence, where a second tile would be all dead rows).
template <int DH, int G, int W, bool PRE, int NQT>
// (head size 64: a floor of 3 / 4 waves per SIMD caps the registers at 168 / 128; left alone the compiler takes 218 and
// 138 and the exp / pack chains of the softmax have nothing to overlap with: 0.94 -> 0.74 ms at C2 under the paper's
// configuration; head size 128 with 4+ heads per group: 2 waves per SIMD, 256 registers instead of 410, 4.51 -> 2.44 ms
// at the 8B shape with 4096-token sequences)
__global__ void __launch_bounds__(G * 64) __attribute__((amdgpu_waves_per_eu(DH == 64 ? (NQT == 1 ? 4 : 3) : (G >= 4 ? 2 : 1), 8)))
k_attn_pv_pages(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc, const bf16_t *__restrict__ vt,
                const unsigned long long *__restrict__ selp, float *__restrict__ o32, const int32_t *__restrict__ pos0, int Tn,
                int L_max, int Hq, int Hkv, int lpadv, float scale, int log2S, int n_sink, int n_window, PrefixView pv)
{
    constexpr int NT = G * 64, KK = DH / 32, DT = DH / 16, KC = 64, QT = 16 * NQT;
    constexpr int KP = DH / 8;
    constexpr int K_PIECES = KC * KP / NT, V_PIECES = DH * (KC / 8) / NT;
    constexpr int K_BYTES = KC * DH * 2, STAGE = 2 * K_BYTES;
    static_assert(KC * KP % NT == 0 && DH * (KC / 8) % NT == 0, "chunk / thread mismatch");
    extern __shared__ __align__(16) unsigned char pvl[];

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kvh = blockIdx.y, s = blockIdx.z, h = kvh * G + w;
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) return;
    const int n_qb = (Tn + QT - 1) / QT;
    for (int pass = 0; pass < 2; ++pass) {                  // query blocks n_qb - 1 - x and x, as in k_attn_pv
    const int qb = pass == 0 ? n_qb - 1 - (int)blockIdx.x : (int)blockIdx.x;
    if (pass == 1 && qb >= n_qb - 1 - (int)blockIdx.x) break;
    const int q0 = qb * QT;
    const int rows = (Tn - q0 < QT) ? (Tn - q0) : QT;
    const int n_max = p0 + q0 + rows;
    const int n_chunks = (n_max + KC - 1) / KC;
    const bf16_t *kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    const bf16_t *vbase = vt + ((int64_t)s * Hkv + kvh) * (int64_t)DH * lpadv;
    const bf16_t *kpre = nullptr, *vpre = nullptr;
    if constexpr (PRE) {                                    // own segment addressed by absolute key: bases minus P keys
        kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)pv.crows * DH - (int64_t)pv.P * DH;
        vbase = vbase - pv.P;
        kpre = pv.k + ((int64_t)(s / pv.K) * Hkv + kvh) * (int64_t)pv.P * DH;
        vpre = pv.vt + ((int64_t)(s / pv.K) * Hkv + kvh) * (int64_t)DH * pv.lpadv;
    }
    const float sl2 = scale * 1.44269504088896341f;          // scores in the log2 domain

    bf16x8_a qf[NQT][KK];
    unsigned long long mask[NQT][W];
    float m_run[NQT], den[NQT];
    int pos[NQT], sink_end[NQT], win_begin[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        m_run[qt] = -INFINITY;
        den[qt] = 0.f;
        const int qi = q0 + 16 * qt + l16;
        const bool live = qi < Tn;
        const int qr = live ? qi : Tn - 1;
        const bf16_t *qp = q + ((int64_t)s * Tn + qr) * (int64_t)(Hq * DH) + (int64_t)h * DH + lg * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            qf[qt][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(qp + kk * 32));
#pragma unroll
        for (int ww = 0; ww < W; ++ww)                      // no masks at all: every page of every row is kept
            mask[qt][ww] = selp ? selp[(((int64_t)s * Tn + qr) * Hq + h) * W + ww] : ~0ull;
        pos[qt] = live ? p0 + qi : -1;                      // dead rows of a ragged block keep nothing
        const int n = p0 + qi + 1;
        sink_end[qt] = n_sink < n ? n_sink : n;
        win_begin[qt] = n - n_window > sink_end[qt] ? n - n_window : sink_end[qt];
    }

    floatx4_a oacc[NQT][DT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) oacc[qt][dt] = floatx4_a{0.f, 0.f, 0.f, 0.f};

    u32x4_a kreg0[K_PIECES], vreg0[V_PIECES];
#define SOL_PV_GLOAD(KR, VR, CH_)                                                                                  \
    {                                                                                                      \
        const int key0_ = (CH_) * KC;                                                                      \
        const bool pre_ = PRE && key0_ < pv.P;              /* chunk-uniform: P is a multiple of the chunk */ \
        const bf16_t *kb_ = pre_ ? kpre : kbase, *vb_ = pre_ ? vpre : vbase;                               \
        const int64_t vs_ = pre_ ? pv.lpadv : lpadv;                                                       \
        _Pragma("unroll") for (int i = 0; i < K_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, row = pc / KP, piece = pc - row * KP;                             \
            int key = key0_ + row;                                                                         \
            if (key >= n_max) key = n_max - 1;                                                             \
            KR[i] = *reinterpret_cast<const u32x4_a *>(kb_ + (int64_t)key * DH + piece * 8);               \
        }                                                                                                  \
        _Pragma("unroll") for (int i = 0; i < V_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, d = pc >> 3, piece = pc & 7;                                      \
            VR[i] = *reinterpret_cast<const u32x4_a *>(vb_ + (int64_t)d * vs_ + key0_ + piece * 8);        \
        }                                                                                                  \
    }
#define SOL_PV_LSTORE(KR, VR, STG_)                                                                                \
    {                                                                                                      \
        unsigned char *kb_ = pvl + (STG_) * STAGE, *vb_ = kb_ + K_BYTES;                                   \
        _Pragma("unroll") for (int i = 0; i < K_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, row = pc / KP, piece = pc - row * KP;                             \
            *reinterpret_cast<u32x4_a *>(kb_ + row * (DH * 2) + ((piece ^ pv_swz_k<DH>(row)) << 4)) = KR[i]; \
        }                                                                                                  \
        _Pragma("unroll") for (int i = 0; i < V_PIECES; ++i) {                                             \
            const int pc = i * NT + tid, d = pc >> 3, piece = pc & 7;                                      \
            *reinterpret_cast<u32x4_a *>(vb_ + d * (KC * 2) + ((piece ^ ((d >> 1) & 7)) << 4)) = VR[i];    \
        }                                                                                                  \
    }
    SOL_PV_GLOAD(kreg0, vreg0, 0);
    SOL_PV_LSTORE(kreg0, vreg0, 0);
    if (1 < n_chunks) SOL_PV_GLOAD(kreg0, vreg0, 1);
    __syncthreads();
    for (int ch = 0; ch < n_chunks; ++ch) {
        const int stg = ch & 1;
        // one register set: what was fetched an iteration ago goes to LDS, then the set is requested again
        if (ch + 1 < n_chunks) SOL_PV_LSTORE(kreg0, vreg0, stg ^ 1);
        if (ch + 2 < n_chunks) SOL_PV_GLOAD(kreg0, vreg0, ch + 2);
        const unsigned char *kb = pvl + stg * STAGE, *vb = kb + K_BYTES;
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
            const int kb32 = ch * KC + cc * 32;
            if (kb32 < n_max) {
                floatx4_a st[NQT][2];
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    const int krow = cc * 32 + 8 * (l16 >> 2) + 4 * kt + (l16 & 3);
                    bf16x8_a kf[KK];
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk)
                        kf[kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(
                            kb + krow * (DH * 2) + (((kk * 4 + lg) ^ pv_swz_k<DH>(krow)) << 4)));
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt) {
                        floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int kk = 0; kk < KK; ++kk)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kk], qf[qt][kk], acc, 0, 0, 0);
                        st[qt][kt] = acc;
                    }
                }
                // keep rule, running maximum (log2 domain), numerators as hi + lo bf16 pairs
                bf16x8_a phi[NQT], plo[NQT];                    // numerators as hi + lo bf16 pairs (single bf16 numerators cost
                float fac[NQT];                               // ~1e-2 of a short row: measured, not taken)
                bool grew = false;
                const int kfirst = kb32 + 8 * lg;
                // sub-chunks wholly before every query of the block and free of sink / window keys need the page
                // bit only (one test per 4 keys, folded into the scaling as an additive 0 / -inf)
                const bool plain = kb32 + 31 <= p0 + q0 && kb32 >= n_sink && kb32 + 31 < p0 + q0 + 1 - n_window;
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt) {
                    float x[8];
                    float m_loc = -INFINITY;
#pragma unroll
                    for (int kt = 0; kt < 2; ++kt) {
                        const int j0 = kfirst + 4 * kt;      // 4 consecutive keys of one page (S >= 4)
                        const int u = j0 >> log2S;
                        unsigned long long word = mask[qt][0];
#pragma unroll
                        for (int ww = 1; ww < W; ++ww) word = (u >> 6) == ww ? mask[qt][ww] : word;
                        const bool bit = ((word >> (u & 63)) & 1ull) != 0ull;
                        if (plain) {
                            const float off = bit ? 0.f : -INFINITY;
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                x[4 * kt + r] = __builtin_fmaf(st[qt][kt][r], sl2, off);
                                m_loc = fmaxf(m_loc, x[4 * kt + r]);
                            }
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int j = j0 + r;
                                const bool keep = (bit || j < sink_end[qt] || j >= win_begin[qt]) && j <= pos[qt];
                                x[4 * kt + r] = keep ? st[qt][kt][r] * sl2 : -INFINITY;
                                m_loc = fmaxf(m_loc, x[4 * kt + r]);
                            }
                        }
                    }
                    m_loc = max_over_lane_groups(m_loc);
                    const float m_new = fmaxf(m_run[qt], m_loc);
                    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                    grew |= m_new > m_run[qt];
                    fac[qt] = __builtin_amdgcn_exp2f(m_run[qt] - m_safe);     // exp2(-inf) = 0 before the first kept key
                    m_run[qt] = m_new;
                    float p[8], psum = 0.f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) { p[i] = __builtin_amdgcn_exp2f(x[i] - m_safe); psum += p[i]; }
                    den[qt] = den[qt] * fac[qt] + psum;
                    u32x4_a hi, lo;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        hi[i] = pack_bf16x2(p[2 * i], p[2 * i + 1]);
                        lo[i] = pack_bf16x2(p[2 * i] - __uint_as_float(hi[i] << 16), p[2 * i + 1] - __uint_as_float(hi[i] & 0xFFFF0000u));
                    }
                    phi[qt] = __builtin_bit_cast(bf16x8_a, hi);
                    plo[qt] = __builtin_bit_cast(bf16x8_a, lo);
                }
                if (__ballot(grew) != 0ull) {                // some row's maximum moved: rescale what is accumulated
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float fo = __shfl(fac[qt], 4 * lg + r);    // accumulator register r is query 4 lg + r
#pragma unroll
                            for (int dt = 0; dt < DT; ++dt) oacc[qt][dt][r] *= fo;
                        }
                }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const int d = dt * 16 + l16;
                    const bf16x8_a vf = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(
                        vb + d * (KC * 2) + (((cc * 4 + lg) ^ ((d >> 1) & 7)) << 4)));
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt) {
                        oacc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo[qt], vf, oacc[qt][dt], 0, 0, 0);
                        oacc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi[qt], vf, oacc[qt][dt], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();
    }
#undef SOL_PV_GLOAD
#undef SOL_PV_LSTORE
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        float dsum = den[qt];
        dsum += __shfl_xor(dsum, 16);
        dsum += __shfl_xor(dsum, 32);
        const float inv = dsum > 0.f ? 1.0f / dsum : 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float iv = __shfl(inv, 4 * lg + r);
            const int qi = q0 + 16 * qt + 4 * lg + r;
            if (qi < Tn) {
                float *op = o32 + ((int64_t)s * Tn + qi) * (int64_t)(Hq * DH) + (int64_t)h * DH + l16;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) op[dt * 16] = oacc[qt][dt][r] * iv;
            }
        }
    }
    }   // pass
}

int attn_tile_lpadv(int L_max) { return attn_lpad64(L_max); }
size_t attn_tile_sel_bytes(int64_t rows, int Hq) { return (size_t)rows * Hq * sizeof(SelRow); }

bool launch_attn_frag_k(const void *k_cache, void *kfr, const int32_t *pos0, int n_seq, int T, int L_max, int Hkv, int dh,
                        hipStream_t st)
{
    if ((dh != 64 && dh != 128) || n_seq <= 0 || T <= 0 || L_max <= 0) return false;
    const int lpad = attn_lpad64(L_max);
    const dim3 tg(lpad / 64, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL((k_frag_k<64>), tg, dim3(256), 0, st, (const bf16_t *)k_cache, (bf16_t *)kfr, pos0, T, L_max, Hkv, lpad);
    else
        hipLaunchKernelGGL((k_frag_k<128>), tg, dim3(256), 0, st, (const bf16_t *)k_cache, (bf16_t *)kfr, pos0, T, L_max, Hkv, lpad);
    return true;
}

bool launch_attn_tile(const void *q, const void *k_cache, const void *v_cache, void *vt, void *kfr, void *sel_ws, float *o32,
                      const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh,
                      hipStream_t st)
{
    if ((int64_t)n_seq * T <= 0) return true;
    const int G = Hkv > 0 ? Hq / Hkv : 0;
    if ((dh != 64 && dh != 128) || L_max > 4096 || T < 16 || G * Hkv != Hq || (G != 1 && G != 2 && G != 4 && G != 8))
        return false;
    const int lpadv = attn_tile_lpadv(L_max);
    SelRow *sel = (SelRow *)sel_ws;
    const dim3 tg((lpadv + 63) / 64, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL((k_transpose_v<64>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
    else
        hipLaunchKernelGGL((k_transpose_v<128>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
    // K in MFMA operand order for the threshold kernel, which reads all causal keys once per block of 8 or 16 query rows
    // (up to 256 keys the copy does not pay)
    const bool frag = L_max > 256;
    if (frag && !launch_attn_frag_k(k_cache, kfr, pos0, n_seq, T, L_max, Hkv, dh, st)) return false;
    // score rows of a workgroup stay in LDS: 16 rows x 1024 keys (66 KB) lets two workgroups share a CU. A launch per
    // class of row lengths: the rows of a long sequence that see at most 1024 (2048) keys go to the variant for that
    // length, with its larger blocks and higher occupancy, not to the one the sequence's last row needs.
    bool ok;
#define SOL_SEL(BQ, SL, KF, LO, HI)                                                                                  \
    ok = dh == 64 ? launch_attn_select_t<BQ, SL, 64, 8, false, KF>(q, KF ? kfr : k_cache, sel, ra, pos0, n_seq, T, L_max, Hq, Hkv, st, PrefixView(), LO, HI)  \
                  : launch_attn_select_t<BQ, SL, 128, 8, false, KF>(q, KF ? kfr : k_cache, sel, ra, pos0, n_seq, T, L_max, Hq, Hkv, st, PrefixView(), LO, HI)
    constexpr int ALL = 1 << 30;
    if (L_max <= 256) { SOL_SEL(32, 4, false, 0, ALL); }
    else if (L_max <= 1024) { SOL_SEL(16, 16, true, 0, ALL); }
    else {
        SOL_SEL(16, 16, true, 0, 1024);
        if (ok && L_max <= 1280) { SOL_SEL(8, 20, true, 1024, ALL); }       // a 1024-token prefix plus a short episode
        else if (ok && L_max <= 2048) { SOL_SEL(8, 32, true, 1024, ALL); }
        else if (ok) {
            SOL_SEL(8, 32, true, 1024, 2048);
            if (ok) { SOL_SEL(8, 64, true, 2048, ALL); }
        }
    }
#undef SOL_SEL
    if (!ok) return false;
#define SOL_PV(G_)                                                                                                   \
    return dh == 64 ? launch_attn_pv_t<64, G_>(q, k_cache, vt, sel, o32, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, st)  \
                    : launch_attn_pv_t<128, G_>(q, k_cache, vt, sel, o32, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, st)
    if (G == 1) { SOL_PV(1); }
    if (G == 2) { SOL_PV(2); }
    if (G == 4) { SOL_PV(4); }
    SOL_PV(8);
#undef SOL_PV
}

// launch_attn_tile for sequences that share prefix caches (PrefixView): k_cache / v_cache hold positions pv.P.. only
// ([n_seq][Hkv][pv.crows][dh]), vt is scratch for their transposed copy ([n_seq][Hkv][dh][attn_tile_lpadv(pv.crows)]);
// every sequence's T rows sit at positions pv.P .. pv.P + T - 1. Returns false (nothing launched) outside the shapes
// of launch_attn_tile, if pv.P is not a multiple of 64 or the caches lie 2^31 elements or more apart.
// shape and address limits of launch_attn_tile_prefix (only differences of the pointers are looked at)
bool attn_tile_prefix_ok(const void *k_cache, int n_seq, int T, int Hq, int Hkv, int dh, const PrefixView &pv)
{
    const int G = Hkv > 0 ? Hq / Hkv : 0, L_max = pv.P + T;
    if ((dh != 64 && dh != 128) || L_max > 4096 || T < 16 || G * Hkv != Hq || (G != 1 && G != 2 && G != 4 && G != 8))
        return false;
    if (pv.P <= 0 || pv.P % 64 || pv.K < 1 || T > pv.crows) return false;
    // the threshold kernel reaches a sequence's own keys as a 32-bit element offset from its input's prefix cache:
    // (own cache of (s, kvh), minus P rows) - (prefix cache of (s / K, kvh)) must lie in [0, 2^31 - a row span) for
    // every (s, kvh); the difference is linear in input, schedule and head, so the corners decide
    if (n_seq % pv.K) return false;
    // (the same from the prefix's copy in operand order, when the view has one: same shape, same strides)
    for (const bf16_t *pre : {pv.k, pv.kf}) {
        if (!pre) continue;
        const int64_t base = (const bf16_t *)k_cache - pre - (int64_t)pv.P * dh;
        for (int c = 0; c < 8; ++c) {
            const int64_t b = (c & 1) ? n_seq / pv.K - 1 : 0, k = (c & 2) ? pv.K - 1 : 0, kv = (c & 4) ? Hkv - 1 : 0;
            const int64_t diff = base + ((b * pv.K + k) * Hkv + kv) * (int64_t)pv.crows * dh - (b * Hkv + kv) * (int64_t)pv.P * dh;
            if (diff < 0 || diff >= (1ll << 31) - (int64_t)(L_max + 1) * dh) return false;
        }
    }
    return true;
}

bool launch_attn_tile_prefix(const void *q, const void *k_cache, const void *v_cache, void *vt, void *sel_ws, float *o32,
                             const RowAct *ra, const int32_t *pos0, int n_seq, int T, int Hq, int Hkv, int dh, PrefixView pv,
                             hipStream_t st)
{
    if ((int64_t)n_seq * T <= 0) return true;
    if (pv.kf && !attn_tile_prefix_ok(k_cache, n_seq, T, Hq, Hkv, dh, pv)) pv.kf = nullptr;   // copy out of reach: do without
    if (!pv.k || !pv.vt || !attn_tile_prefix_ok(k_cache, n_seq, T, Hq, Hkv, dh, pv)) return false;
    const int G = Hq / Hkv, L_max = pv.P + T;
    const int lpadv = attn_tile_lpadv(pv.crows);
    SelRow *sel = (SelRow *)sel_ws;
    const dim3 tg((lpadv + 63) / 64, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL((k_transpose_v<64>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt,
                           (const int32_t *)nullptr, T, pv.crows, Hkv, lpadv);
    else
        hipLaunchKernelGGL((k_transpose_v<128>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt,
                           (const int32_t *)nullptr, T, pv.crows, Hkv, lpadv);
    bool ok;
    // rows longer than 1024 keys read the prefix keys from their copy in operand order, if the view has one
#define SOL_SEL(BQ, SL, KF)                                                                                          \
    ok = dh == 64 ? launch_attn_select_t<BQ, SL, 64, 8, true, KF>(q, k_cache, sel, ra, pos0, n_seq, T, L_max, Hq, Hkv, st, pv) \
                  : launch_attn_select_t<BQ, SL, 128, 8, true, KF>(q, k_cache, sel, ra, pos0, n_seq, T, L_max, Hq, Hkv, st, pv)
    if (L_max <= 256) { SOL_SEL(32, 4, false); }
    else if (L_max <= 1024) { SOL_SEL(16, 16, false); }
    else if (!pv.kf) {
        if (L_max <= 1280) { SOL_SEL(8, 20, false); }
        else if (L_max <= 2048) { SOL_SEL(8, 32, false); }
        else { SOL_SEL(8, 64, false); }
    }
    else if (L_max <= 1280) { SOL_SEL(8, 20, true); }
    else if (L_max <= 2048) { SOL_SEL(8, 32, true); }
    else { SOL_SEL(8, 64, true); }
#undef SOL_SEL
    if (!ok) return false;
#define SOL_PV(G_)                                                                                                   \
    return dh == 64 ? launch_attn_pv_t<64, G_, true>(q, k_cache, vt, sel, o32, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, st, pv)  \
                    : launch_attn_pv_t<128, G_, true>(q, k_cache, vt, sel, o32, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, st, pv)
    if (G == 1) { SOL_PV(1); }
    if (G == 2) { SOL_PV(2); }
    if (G == 4) { SOL_PV(4); }
    SOL_PV(8);
#undef SOL_PV
}

// PRE: kc / vt / pm belong to the sequences' own keys (pv.crows rows each, positions pv.P..), L_max = pv.P + T.
template <int DH, int W, bool PRE = false>
static bool launch_attn_tile_pages_t(const void *q, const void *kc, const void *vt, void *pm, void *selp, float *o32,
                                     const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv,
                                     int lpadv, int log2S, AttnOpts opt, hipStream_t st, PrefixView pv = PrefixView())
{
    const int S = 1 << log2S, G = Hq / Hkv;
    constexpr int ppb = 256 / (DH / 8);
    if (PRE)   // metadata of the own keys, by local row (pages do not straddle pv.P)
        hipLaunchKernelGGL(k_page_prefix_meta<DH>, dim3(((pv.crows + S - 1) / S + ppb - 1) / ppb, Hkv, n_seq), dim3(256), 0,
                           st, (const bf16_t *)kc, (const int32_t *)nullptr, (bf16_t *)pm, T, S, pv.crows, Hkv);
    else
        hipLaunchKernelGGL(k_page_prefix_meta<DH>, dim3(((L_max + S - 1) / S + ppb - 1) / ppb, Hkv, n_seq), dim3(256), 0, st,
                           (const bf16_t *)kc, pos0, (bf16_t *)pm, T, S, L_max, Hkv);
    hipLaunchKernelGGL((k_attn_select_pages<DH, W, PRE>), dim3((T + 15) / 16, Hq, n_seq), dim3(256), 0, st, (const bf16_t *)q,
                       (const bf16_t *)pm, (unsigned long long *)selp, ra, pos0, T, L_max, Hq, Hkv, log2S, pv);
    const size_t lds = 4 * (size_t)64 * DH * 2;
    const float scale = 1.0f / sqrtf((float)DH);
#define SOL_PVP(G_, NQT_)                                                                                            \
    {                                                                                                                \
        auto kern = k_attn_pv_pages<DH, G_, W, PRE, NQT_>;                                                           \
        static bool attr_done = false;                                                                               \
        if (!attr_done) {                                                                                            \
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    (int)lds) != hipSuccess)                                                         \
                return false;                                                                                        \
            attr_done = true;                                                                                        \
        }                                                                                                            \
        hipLaunchKernelGGL(kern, dim3(((T + 16 * NQT_ - 1) / (16 * NQT_) + 1) / 2, Hkv, n_seq), dim3(G_ * 64), lds, st, (const bf16_t *)q, \
                           (const bf16_t *)kc, (const bf16_t *)vt, (const unsigned long long *)selp, o32, pos0, T, L_max, Hq, \
                           Hkv, lpadv, scale, log2S, opt.n_sink, opt.n_window, pv);                                  \
        return true;                                                                                                 \
    }
    if (T <= 16) {                                           // one tile of 16 query rows per workgroup
        if (G == 1) SOL_PVP(1, 1)
        if (G == 2) SOL_PVP(2, 1)
        if (G == 4) SOL_PVP(4, 1)
        SOL_PVP(8, 1)
    }
    if (G == 1) SOL_PVP(1, 2)
    if (G == 2) SOL_PVP(2, 2)
    if (G == 4) SOL_PVP(4, 2)
    SOL_PVP(8, 2)
#undef SOL_PVP
}

// Dense causal attention for rows that keep every key (prefill, cache refresh): the flash-style kernel alone, with
// its running maximum, no threshold pass. Shapes of launch_attn_tile.
bool launch_attn_tile_dense(const void *q, const void *k_cache, const void *v_cache, void *vt, float *o32,
                            const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh, hipStream_t st)
{
    if ((int64_t)n_seq * T <= 0) return true;
    const int G = Hkv > 0 ? Hq / Hkv : 0;
    if ((dh != 64 && dh != 128) || L_max > 4096 || T < 16 || G * Hkv != Hq || (G != 1 && G != 2 && G != 4 && G != 8) || !vt)
        return false;
    const int lpadv = attn_tile_lpadv(L_max);
    const dim3 tg((lpadv + 63) / 64, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL((k_transpose_v<64>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
    else
        hipLaunchKernelGGL((k_transpose_v<128>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
    const size_t lds = 4 * (size_t)64 * dh * 2;
    const float scale = 1.0f / sqrtf((float)dh);
#define SOL_PVD2(DH_, G_, NQT_)                                                                                      \
    {                                                                                                                \
        auto kern = k_attn_pv_pages<DH_, G_, 1, false, NQT_>;                                                        \
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,    \
                                (int)lds) != hipSuccess)                                                             \
            return false;                                                                                            \
        hipLaunchKernelGGL(kern, dim3(((T + 16 * NQT_ - 1) / (16 * NQT_) + 1) / 2, Hkv, n_seq), dim3(G_ * 64), lds, st, (const bf16_t *)q, \
                           (const bf16_t *)k_cache, (const bf16_t *)vt, (const unsigned long long *)nullptr, o32, pos0, T, \
                           L_max, Hq, Hkv, lpadv, scale, 6, 0, 0, PrefixView());                                     \
        return true;                                                                                                 \
    }
#define SOL_PVD(DH_, G_) { if (T <= 16) SOL_PVD2(DH_, G_, 1) SOL_PVD2(DH_, G_, 2) }
    if (dh == 64) {
        if (G == 1) SOL_PVD(64, 1)
        if (G == 2) SOL_PVD(64, 2)
        if (G == 4) SOL_PVD(64, 4)
        SOL_PVD(64, 8)
    }
    if (G == 1) SOL_PVD(128, 1)
    if (G == 2) SOL_PVD(128, 2)
    if (G == 4) SOL_PVD(128, 4)
    SOL_PVD(128, 8)
#undef SOL_PVD
#undef SOL_PVD2
}

size_t attn_tile_pages_meta_bytes(int64_t n_seq, int Hkv, int L_max, int dh) { return (size_t)n_seq * Hkv * L_max * 2 * dh * 2; }
size_t attn_tile_pages_sel_bytes(int64_t rows, int Hq, int L_max, int S) { return (size_t)rows * Hq * (((L_max + S - 1) / S + 63) / 64) * 8; }

// Batched bf16 attention under the page rule: page size a power of two in [4, 64], at most 256 pages, the limits of
// launch_attn_tile otherwise. pm: attn_tile_pages_meta_bytes of scratch, selp: attn_tile_pages_sel_bytes.
bool launch_attn_tile_pages(const void *q, const void *k_cache, const void *v_cache, void *vt, void *pm, void *selp,
                            float *o32, const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv,
                            int dh, AttnOpts opt, hipStream_t st)
{
    if ((int64_t)n_seq * T <= 0) return true;
    const int G = Hkv > 0 ? Hq / Hkv : 0, S = opt.page;
    if ((dh != 64 && dh != 128) || L_max > 4096 || T < 16 || G * Hkv != Hq || (G != 1 && G != 2 && G != 4 && G != 8))
        return false;
    if (S < 4 || S > 64 || (S & (S - 1)) || !pm || !vt) return false;
    int log2S = 0;
    while ((1 << log2S) < S) ++log2S;
    const int n_words = ((L_max + S - 1) / S + 63) / 64;
    if (n_words > 4) return false;
    const int lpadv = attn_tile_lpadv(L_max);
    const dim3 tg((lpadv + 63) / 64, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL((k_transpose_v<64>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
    else
        hipLaunchKernelGGL((k_transpose_v<128>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
#define SOL_TP(W_)                                                                                                   \
    return dh == 64 ? launch_attn_tile_pages_t<64, W_>(q, k_cache, vt, pm, selp, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, log2S, opt, st) \
                    : launch_attn_tile_pages_t<128, W_>(q, k_cache, vt, pm, selp, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, log2S, opt, st)
    if (n_words == 1) { SOL_TP(1); }
    if (n_words == 2) { SOL_TP(2); }
    SOL_TP(4);
#undef SOL_TP
}

// Prefix side of the shared-prefix variant: the metadata rows of the prefix keys, once per input and layer.
bool launch_page_prefix_meta(const void *k_cache, void *pm, int n_seq, int P, int Hkv, int dh, int S, hipStream_t st)
{
    if ((int64_t)n_seq * P <= 0) return true;
    if ((dh != 64 && dh != 128) || S < 4 || S > 64 || (S & (S - 1)) || !pm) return false;
    const int ppb = 256 / (dh / 8);
    const dim3 grid(((P + S - 1) / S + ppb - 1) / ppb, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL(k_page_prefix_meta<64>, grid, dim3(256), 0, st, (const bf16_t *)k_cache, (const int32_t *)nullptr,
                           (bf16_t *)pm, P, S, P, Hkv);
    else
        hipLaunchKernelGGL(k_page_prefix_meta<128>, grid, dim3(256), 0, st, (const bf16_t *)k_cache, (const int32_t *)nullptr,
                           (bf16_t *)pm, P, S, P, Hkv);
    return true;
}

// shapes launch_attn_tile_pages_prefix takes
bool attn_tile_pages_prefix_ok(int n_seq, int T, int Hq, int Hkv, int dh, int S, const PrefixView &pv)
{
    const int G = Hkv > 0 ? Hq / Hkv : 0, L_max = pv.P + T;
    if ((dh != 64 && dh != 128) || L_max > 4096 || T < 16 || G * Hkv != Hq || (G != 1 && G != 2 && G != 4 && G != 8))
        return false;
    if (S < 4 || S > 64 || (S & (S - 1)) || ((L_max + S - 1) / S + 63) / 64 > 4) return false;
    // chunks of 64 keys and tiles of 16 pages must lie on one side of the prefix boundary
    return pv.P > 0 && pv.P % 64 == 0 && pv.P % (16 * S) == 0 && pv.K >= 1 && n_seq % pv.K == 0 && T <= pv.crows;
}

// launch_attn_tile_pages for sequences that share prefix caches (PrefixView: pv.k, pv.vt and pv.pm of the input's
// prefix, written by the prefix pass and launch_page_prefix_meta); k_cache / v_cache / vt / pm hold the sequences'
// own pv.crows positions from pv.P on.
bool launch_attn_tile_pages_prefix(const void *q, const void *k_cache, const void *v_cache, void *vt, void *pm, void *selp,
                                   float *o32, const RowAct *ra, const int32_t *pos0, int n_seq, int T, int Hq, int Hkv,
                                   int dh, AttnOpts opt, PrefixView pv, hipStream_t st)
{
    if ((int64_t)n_seq * T <= 0) return true;
    const int S = opt.page;
    if (!pv.k || !pv.vt || !pv.pm || !pm || !vt || !attn_tile_pages_prefix_ok(n_seq, T, Hq, Hkv, dh, S, pv)) return false;
    const int L_max = pv.P + T;
    int log2S = 0;
    while ((1 << log2S) < S) ++log2S;
    const int n_words = ((L_max + S - 1) / S + 63) / 64;
    const int lpadv = attn_tile_lpadv(pv.crows);
    const dim3 tg((lpadv + 63) / 64, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL((k_transpose_v<64>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt,
                           (const int32_t *)nullptr, T, pv.crows, Hkv, lpadv);
    else
        hipLaunchKernelGGL((k_transpose_v<128>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt,
                           (const int32_t *)nullptr, T, pv.crows, Hkv, lpadv);
#define SOL_TPP(W_)                                                                                                  \
    return dh == 64 ? launch_attn_tile_pages_t<64, W_, true>(q, k_cache, vt, pm, selp, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, log2S, opt, st, pv) \
                    : launch_attn_tile_pages_t<128, W_, true>(q, k_cache, vt, pm, selp, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, log2S, opt, st, pv)
    if (n_words == 1) { SOL_TPP(1); }
    if (n_words == 2) { SOL_TPP(2); }
    SOL_TPP(4);
#undef SOL_TPP
}

}  // namespace sol
