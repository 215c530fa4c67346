// Attention with per-query budgeted key selection.
//
// k_attn_rows: one workgroup per (query row, group of HPB query heads that share a KV head).
//   1. scores s_j = (q . k_j) / sqrt(dh) over the allowed cache positions j in [0, pos]   -> LDS (fp32)
//   2. budget b = ceil(kappa * n); b < n: exact b-th largest score by radix select, ties to the
//      lower position; b = n: dense
//   3. softmax over the kept keys (dropped keys contribute exp(-inf) = 0)
//   4. o = sum_j p_j v_j, reading only V rows kept by at least one of the HPB heads
// K is streamed once per workgroup (HPB heads share it), V rows are gathered. This is the decode
// kernel (one query per sequence, HBM-bound) and the any-shape / fp32 path of the batched pass.
#include "sol_internal.h"

namespace sol {

struct ScoreKeyLds {
    const float *row;
    __device__ __forceinline__ uint32_t operator()(int i) const { return score_key(row[i]); }
};

template <typename T, int HPB, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
k_attn_rows(const T *__restrict__ q, const T *__restrict__ kc, const T *__restrict__ vc, float *__restrict__ o32,
            const RowAct *__restrict__ ra, const int32_t *__restrict__ pos0, int Tn, int L_max, int Hq, int Hkv,
            int dh, int lpad, float scale, int *flags)
{
    constexpr int VEC = Vec16<T>::N;
    constexpr int NW = BLOCK / 64;
    extern __shared__ float smem[];
    float *sc = smem;                               // [HPB][lpad]
    float *ored = smem + (size_t)HPB * lpad;        // [NW][HPB][dh]
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
    __syncthreads();

    // ---- 2 + 3. selection and softmax numerators, head by head ------------------------------
    const RowAct act = ra[r];
    const int b = budget_ceil(act.keep_num, act.keep_den, n);
    float inv_den[HPB];
#pragma unroll
    for (int h = 0; h < HPB; ++h) {
        float *row = sc + h * lpad;
        uint32_t thr = 0u; int J = n;
        if (b < n) {
            ScoreKeyLds kf{row};
            int quota, n_eq;
            block_radix_select<BLOCK>(kf, n, b, hist, sh, thr, quota, n_eq);
            if (quota < n_eq) J = block_tie_cutoff<BLOCK>(kf, n, thr, quota, wcnt, sh);
        }
        float mx = -INFINITY;
        for (int j = tid; j < n; j += BLOCK) mx = fmaxf(mx, row[j]);   // the best key is always kept
        mx = block_max<BLOCK>(mx, red);
        float den = 0.f;
        for (int j = tid; j < n; j += BLOCK) {
            const float sv = row[j];
            const uint32_t key = score_key(sv);
            const bool keep = key > thr || (key == thr && j <= J);
            const float p = keep ? expf(sv - mx) : 0.f;
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

size_t attn_rows_lds_bytes(int L_max, int hpb, int block)
{
    const size_t lpad = ((size_t)L_max + 63) & ~(size_t)63;
    return (size_t)hpb * lpad * sizeof(float);      // + ored, added by the launcher (needs dh)
}

template <typename T, int HPB, int BLOCK>
static bool launch_attn_rows_t(const void *q, const void *kc, const void *vc, float *o32, const RowAct *ra,
                               const int32_t *pos0, int n_seq, int Tn, int L_max, int Hq, int Hkv, int dh, int lpad,
                               size_t lds, int *flags, hipStream_t st)
{
    auto kern = k_attn_rows<T, HPB, BLOCK>;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return false;
    }
    const float scale = 1.0f / sqrtf((float)dh);
    hipLaunchKernelGGL(kern, dim3(Hq / HPB, (unsigned)((int64_t)n_seq * Tn)), dim3(BLOCK), lds, st, (const T *)q,
                       (const T *)kc, (const T *)vc, o32, ra, pos0, Tn, L_max, Hq, Hkv, dh, lpad, scale, flags);
    return true;
}

bool launch_attn_rows(const void *q, const void *k_cache, const void *v_cache, int dtype, float *o32,
                      const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh,
                      int *flags, hipStream_t st)
{
    if ((int64_t)n_seq * T <= 0) return true;
    const int vec = dtype == 0 ? 4 : 8;
    if (dh % vec) return false;
    const int lpk = dh / vec;
    if (lpk > 64 || (lpk & (lpk - 1))) return false;
    const int g = Hq / Hkv;
    const int lpad = (L_max + 63) & ~63;
    // long caches (decode) get 1024-thread workgroups: more loads in flight per CU
    const int block = (L_max >= 2048) ? 1024 : 256;
    const size_t budget = 150 * 1024;
    int hpb = 4;
    while (hpb > 1 && (g % hpb != 0 ||
                       (size_t)hpb * lpad * 4 + (size_t)(block / 64) * hpb * dh * 4 > budget)) hpb >>= 1;
    const size_t lds = (size_t)hpb * lpad * 4 + (size_t)(block / 64) * hpb * dh * 4;
    if (lds > budget) return false;
#define SOL_ATTN_CASE(TT, H, B)                                                                                     \
    return launch_attn_rows_t<TT, H, B>(q, k_cache, v_cache, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, dh, lpad, lds, \
                                        flags, st)
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

}  // namespace sol
