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


// =================================================================================================
// Tiled attention for the batched (teacher-forced) pass, bf16.
//
// One workgroup (8 waves) per (sequence, query head, block of BQ consecutive query positions):
//   A. S = Q K^T on MFMA (16x16x32 tiles, fp32 accumulate), waves striding over key tiles; the scaled
//      fp32 scores of the whole block go to LDS, one padded row per query (selection needs the exact
//      fp32 value of every causal score, so rows stay on chip instead of a 2 GB HBM round trip).
//   B. One wave per row, scores in registers: budget b = ceil(kappa * n); if b < n the threshold of
//      the b largest scores is found by bisection on order-preserving integer keys between the
//      row's min and max, counting with ballots and stopping as soon as exactly b scores lie above
//      the pivot (about log2(n) steps); equal scores at the threshold go to the lower positions.
//      Softmax numerators of the kept keys are written back over the row as a pair of bf16 halves
//      (p = hi + lo, zeros elsewhere), which fits the 4 bytes per key the fp32 score occupied.
//   C. O = P V on MFMA with V read K-contiguous from a transposed copy, waves striding over key
//      chunks, partial sums reduced through LDS in wave order, scaled by 1 / sum(p).
// Rows whose budget keeps every key skip B's search. LDS: BQ * (Lpad + 4) * 4 bytes.
// =================================================================================================
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_a;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_a;
typedef uint32_t u32x4_a __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_a __attribute__((ext_vector_type(2)));
typedef float f32x4_a __attribute__((ext_vector_type(4)));


#ifdef SOL_ATTN_TIMING   // probe builds only: per-phase s_memtime stamps of wave 0 of every workgroup
__device__ unsigned long long *g_attn_stamps;
#define AT_STAMP(i)                                                                                  \
    if (threadIdx.x == 0 && g_attn_stamps)                                                           \
        g_attn_stamps[((size_t)(blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 8 + (i)] = __builtin_readcyclecounter()
#else
#define AT_STAMP(i)
#endif

template <int BQ, int SLOTS, int DH, int AT_WAVES>
__global__ void __launch_bounds__(AT_WAVES * 64)
k_attn_tile(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc, const bf16_t *__restrict__ vt,
            float *__restrict__ o32, const RowAct *__restrict__ ra, const int32_t *__restrict__ pos0, int Tn, int L_max,
            int Hq, int Hkv, int lpadv, float scale)
{
    constexpr int AT_BLOCK = AT_WAVES * 64;
    constexpr int LPAD = SLOTS * 64, LS = LPAD + 4;
    constexpr int RT = (BQ + 15) / 16, KK = DH / 32, DT = DH / 16, NJ = SLOTS / 4;
    constexpr int UA = (SLOTS <= 16) ? 8 : 4;              // key tiles in flight per wave in phase A
    constexpr int UC = (SLOTS <= 16) ? 4 : 2;                                  // key chunks in flight per wave in phase C
    extern __shared__ __align__(16) float sc[];            // [BQ][LS] scores, then P (hi | lo bf16) in place, then partial O
    __shared__ float inv_den[BQ];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index, scalar
    const int nqb = gridDim.x;
    const int qb = nqb - 1 - (int)blockIdx.x;              // heaviest blocks first
    const int h = blockIdx.y, s = blockIdx.z;
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) return;                 // flagged by the projection kernel; sequence skipped
    const int q0 = qb * BQ;
    const int rows = (Tn - q0 < BQ) ? (Tn - q0) : BQ;      // live rows of this block
    const int n_max = p0 + q0 + rows;                      // keys seen by the block's last row
    const int kvh = h / (Hq / Hkv);
    const bf16_t *kbase = kc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    const bf16_t *vbase = vt + ((int64_t)s * Hkv + kvh) * (int64_t)DH * lpadv;
    const int l16 = lane & 15, lg = lane >> 4;

    AT_STAMP(0);
    // ---- A. scores ---------------------------------------------------------------------------
    {
        bf16x8_a qf[RT][KK];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            int qr = q0 + rt * 16 + l16;
            if (qr >= Tn) qr = Tn - 1;
            const bf16_t *qp = q + ((int64_t)s * Tn + qr) * (int64_t)(Hq * DH) + (int64_t)h * DH + lg * 8;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                qf[rt][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(qp + kk * 32));
        }
        const int n_kt = (n_max + 15) >> 4;
        for (int kt0 = w; kt0 < n_kt; kt0 += AT_WAVES * UA) {
            bf16x8_a kf[UA][KK];
#pragma unroll
            for (int u = 0; u < UA; ++u) {                 // issue every load of the group before the first MFMA
                int key = (kt0 + u * AT_WAVES) * 16 + l16;
                if (key >= n_max) key = n_max - 1;
                const bf16_t *kp = kbase + (int64_t)key * DH + lg * 8;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk)
                    kf[u][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(kp + kk * 32));
            }
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                const int kt = kt0 + u * AT_WAVES;
                if (kt < n_kt) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int kk = 0; kk < KK; ++kk)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[rt][kk], kf[u][kk], acc, 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int row = rt * 16 + lg * 4 + r;
                            if (row < BQ) sc[row * LS + kt * 16 + l16] = acc[r] * scale;
                        }
                    }
                }
            }
        }
    }
    __syncthreads();
    AT_STAMP(1);

    // ---- B. selection + softmax numerators, one wave per row --------------------------------------
    for (int r = w; r < BQ; r += AT_WAVES) {
        float *row = sc + r * LS;
        uint32_t *prow = reinterpret_cast<uint32_t *>(row);           // P as bf16 pairs, in place
        if (r >= rows) {                                              // dead row of a ragged block: P = 0
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                *reinterpret_cast<u32x2_a *>(prow + (256 * j + 4 * lane) / 2) = u32x2_a{0u, 0u};
                *reinterpret_cast<u32x2_a *>(prow + (LPAD + 256 * j + 4 * lane) / 2) = u32x2_a{0u, 0u};
            }
            if (lane == 0) inv_den[r] = 0.f;
            continue;
        }
        const int n = p0 + q0 + r + 1;                                // wave-uniform
        const RowAct act = ra[(int64_t)s * Tn + q0 + r];
        const int b = budget_ceil(act.keep_num, act.keep_den, n);
        float sv[SLOTS];
        uint32_t key[SLOTS];
        uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (256 * j < n) {
                const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool valid = 256 * j + 4 * lane + e < n;
                    const uint32_t kv = valid ? score_key(v[e]) : 0u;   // 0 is below every real score
                    sv[4 * j + e] = v[e];
                    key[4 * j + e] = kv;
                    kmax = kv > kmax ? kv : kmax;
                    kmin = (valid && kv < kmin) ? kv : kmin;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) { sv[4 * j + e] = 0.f; key[4 * j + e] = 0u; }
            }
        }
        kmax = wave_max_u32(kmax);
        const float mx = score_unkey(kmax);                           // the best key is always kept
        uint32_t thr = 1u;                                            // budget keeps all: every valid key passes
        if (b < n) {
            kmin = wave_min_u32(kmin);
            thr = wave_select_topk<SLOTS>(key, n, b, kmin, kmax, lane);
        }
        float den = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float p[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                p[e] = key[4 * j + e] >= thr ? __expf(sv[4 * j + e] - mx) : 0.f;
                den += p[e];
            }
            // p = hi + lo with both halves bf16: the MFMA product with bf16 V is then exact to ~2^-17
            u32x2_a pk, pl;
            pk[0] = pack_bf16x2(p[0], p[1]);
            pk[1] = pack_bf16x2(p[2], p[3]);
            pl[0] = pack_bf16x2(p[0] - __uint_as_float(pk[0] << 16), p[1] - __uint_as_float(pk[0] & 0xFFFF0000u));
            pl[1] = pack_bf16x2(p[2] - __uint_as_float(pk[1] << 16), p[3] - __uint_as_float(pk[1] & 0xFFFF0000u));
            *reinterpret_cast<u32x2_a *>(prow + (256 * j + 4 * lane) / 2) = pk;
            *reinterpret_cast<u32x2_a *>(prow + (LPAD + 256 * j + 4 * lane) / 2) = pl;
        }
        den = wave_sum_dpp(den);
        if (lane == 0) inv_den[r] = 1.0f / den;
    }
    AT_STAMP(2);
    __syncthreads();
    AT_STAMP(3);

    // ---- C. O = P V --------------------------------------------------------------------------------
    floatx4_a oacc[RT][DT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) oacc[rt][dt] = floatx4_a{0.f, 0.f, 0.f, 0.f};
    {
        const int n_ch = (n_max + 31) >> 5;
        for (int c0 = w; c0 < n_ch; c0 += AT_WAVES * UC) {
            bf16x8_a vf[UC][DT];
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                int c = c0 + u * AT_WAVES;
                if (c >= n_ch) c = n_ch - 1;               // re-read the last chunk; its product is not used
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const bf16_t *vp = vbase + (int64_t)(dt * 16 + l16) * lpadv + c * 32 + lg * 8;
                    vf[u][dt] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(vp));
                }
            }
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                const int c = c0 + u * AT_WAVES;
                if (c < n_ch) {
                    bf16x8_a pf[RT], pl[RT];
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        int pr = rt * 16 + l16;
                        if (pr >= BQ) pr = BQ - 1;
                        const unsigned char *pp =
                            reinterpret_cast<const unsigned char *>(sc + pr * LS) + (c * 32 + lg * 8) * 2;
                        pf[rt] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(pp));
                        pl[rt] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(pp + 2 * LPAD));
                    }
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) {
                            oacc[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pl[rt], vf[u][dt], oacc[rt][dt], 0, 0, 0);
                            oacc[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf[rt], vf[u][dt], oacc[rt][dt], 0, 0, 0);
                        }
                }
            }
        }
    }
    AT_STAMP(4);
    __syncthreads();                                          // every wave is done reading P
    float *red = sc;                                          // [AT_WAVES][BQ][DH]
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = rt * 16 + lg * 4 + r;
                if (row < BQ) red[((size_t)w * BQ + row) * DH + dt * 16 + l16] = oacc[rt][dt][r];
            }
    __syncthreads();
    for (int idx = tid; idx < rows * DH; idx += AT_BLOCK) {
        const int row = idx / DH, d = idx - row * DH;
        float t = 0.f;
#pragma unroll
        for (int ww = 0; ww < AT_WAVES; ++ww) t += red[((size_t)ww * BQ + row) * DH + d];
        o32[((int64_t)s * Tn + q0 + row) * (int64_t)(Hq * DH) + (int64_t)h * DH + d] = t * inv_den[row];
    }
    AT_STAMP(5);
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

template <int DH, int SLOTS>
__global__ void __launch_bounds__(DEC_BLOCK)
k_attn_decode(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc, const bf16_t *__restrict__ vc,
              float *__restrict__ o32, const RowAct *__restrict__ ra, const int32_t *__restrict__ cache_len, int L_max,
              int Hq, int Hkv, float scale, int *flags)
{
    constexpr int KK = DH / 32, SLICE = SLOTS * 64, LPAD = SLICE * DEC_GW, NJ = SLOTS / 4;
    constexpr int VEC = 8, LPK = DH / VEC, KPI = DEC_BLOCK / LPK;
    extern __shared__ __align__(16) float sc[];               // [DEC_HPB][LPAD]; later partial O [DEC_WAVES][HPB][DH]
    __shared__ int s_cnt[2][DEC_WAVES];
    __shared__ uint32_t s_min[DEC_WAVES], s_max[DEC_WAVES];
    __shared__ int s_done[2][DEC_HPB];
    __shared__ int s_gt[DEC_WAVES];
    __shared__ float s_den[DEC_WAVES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kvh = blockIdx.x, s = blockIdx.y;
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
        constexpr int U = 4;
        for (int kt0 = w; kt0 < n_kt; kt0 += DEC_WAVES * U) {
            bf16x8_a kf[U][KK];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int key = (kt0 + u * DEC_WAVES) * 16 + l16;
                if (key >= n) key = n - 1;
                const bf16_t *kp = kbase + (int64_t)key * DH + lg * 8;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk)
                    kf[u][kk] = __builtin_bit_cast(bf16x8_a, *reinterpret_cast<const u32x4_a *>(kp + kk * 32));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kt = kt0 + u * DEC_WAVES;
                if (kt < n_kt) {
                    floatx4_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[u][kk], qf[kk], acc, 0, 0, 0);
                    if (l16 < DEC_HPB) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) sc[l16 * LPAD + kt * 16 + lg * 4 + r] = acc[r] * scale;
                    }
                }
            }
        }
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
    // invariant while searching: count(key >= lo) >= b, count(key >= hi + 1) < b
    for (int it = 0; it < 34; ++it) {
        const int par = it & 1;
        uint32_t mid = 0u;
        if (!done) {
            mid = lo + ((hi - lo + 1u) >> 1);
            const int c = wave_count_ge<SLOTS>(key, n_loc, mid);
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
                if (cnt == b) { thr = mid; done = true; }
                else if (cnt > b) lo = mid; else hi = mid - 1u;
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
    float den = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (256 * j < n_loc) {
            const f32x4_a v = *reinterpret_cast<const f32x4_a *>(row + 256 * j + 4 * lane);
            f32x4_a p;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool on = (256 * j + 4 * lane + e < n_loc) && score_key(v[e]) >= thr;
                p[e] = on ? __expf(v[e] - mx) : 0.f;
                den += p[e];
            }
            *reinterpret_cast<f32x4_a *>(row + 256 * j + 4 * lane) = p;
        }
    }
    den = wave_sum_dpp(den);
    if (lane == 0) s_den[w] = den;
    __syncthreads();

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
                p[u][hh] = (j < n) ? sc[hh * LPAD + j] : 0.f;
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
    // reduce over the key slots of a wave (lanes with equal cs), then across waves in fixed order
    for (int o = LPK; o < 64; o <<= 1)
#pragma unroll
        for (int hh = 0; hh < DEC_HPB; ++hh)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[hh][e] += __shfl_xor(acc[hh][e], o, 64);
    __syncthreads();                                           // all reads of the numerators are done
    float *ored = sc;                                          // [DEC_WAVES][HPB][DH]
    if (lane < LPK) {
#pragma unroll
        for (int hh = 0; hh < DEC_HPB; ++hh)
#pragma unroll
            for (int e = 0; e < VEC; ++e) ored[((size_t)w * DEC_HPB + hh) * DH + lane * VEC + e] = acc[hh][e];
    }
    __syncthreads();
    for (int idx = tid; idx < DEC_HPB * DH; idx += DEC_BLOCK) {
        const int hh = idx / DH;
        float t = 0.f, dsum = 0.f;
        for (int ww = 0; ww < DEC_WAVES; ++ww) t += ored[(size_t)ww * DEC_HPB * DH + idx];
#pragma unroll
        for (int i = 0; i < DEC_GW; ++i) dsum += s_den[hh * DEC_GW + i];
        o32[(int64_t)s * (Hq * DH) + (int64_t)h0 * DH + idx] = t / dsum;
    }
}

template <int DH, int SLOTS>
static bool launch_attn_decode_t(const void *q, const void *kc, const void *vc, float *o32, const RowAct *ra,
                                 const int32_t *cache_len, int B, int L_max, int Hq, int Hkv, int *flags, hipStream_t st)
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
                       (const bf16_t *)vc, o32, ra, cache_len, L_max, Hq, Hkv, 1.0f / sqrtf((float)DH), flags);
    return true;
}

// One query per sequence (T = 1), bf16, 4 query heads per KV head, head_dim 64 / 128, L_max <= 9216.
bool launch_attn_decode(const void *q, const void *k_cache, const void *v_cache, float *o32, const RowAct *ra,
                        const int32_t *cache_len, int B, int L_max, int Hq, int Hkv, int dh, int *flags, hipStream_t st)
{
    if (B <= 0) return true;
    if (!cache_len || Hq != DEC_HPB * Hkv || (dh != 64 && dh != 128) || L_max > 9216) return false;
    const size_t red = (size_t)DEC_WAVES * DEC_HPB * dh * 4;
#define SOL_DEC(SL)                                                                                             \
    if ((size_t)DEC_HPB * SL * 64 * DEC_GW * 4 >= red)                                                           \
        return dh == 64 ? launch_attn_decode_t<64, SL>(q, k_cache, v_cache, o32, ra, cache_len, B, L_max, Hq, Hkv, flags, st) \
                        : launch_attn_decode_t<128, SL>(q, k_cache, v_cache, o32, ra, cache_len, B, L_max, Hq, Hkv, flags, st)
    if (L_max <= 1024) { SOL_DEC(4); }
    if (L_max <= 2048) { SOL_DEC(8); }
    if (L_max <= 4096) { SOL_DEC(16); }
    if (L_max <= 8192) { SOL_DEC(32); }
    SOL_DEC(36);                                   // 9216 columns: an 8192-token cache plus the tokens being decoded
#undef SOL_DEC
    return false;
}

// V cache [s][kvh][key][dh] -> vt [s][kvh][dh][lpadv] for keys < pos0[s] + Tn, zero beyond.
template <int DH>
__global__ void __launch_bounds__(256)
k_transpose_v(const bf16_t *__restrict__ vc, bf16_t *__restrict__ vt, const int32_t *__restrict__ pos0, int Tn, int L_max,
              int Hkv, int lpadv)
{
    __shared__ bf16_t tile[64][DH + 2];
    const int kb = blockIdx.x * 64, kvh = blockIdx.y, s = blockIdx.z;
    const int p0 = pos0 ? pos0[s] : 0;
    int len = p0 + Tn;
    if (p0 < 0 || len > L_max) len = 0;
    const bf16_t *src = vc + ((int64_t)s * Hkv + kvh) * (int64_t)L_max * DH;
    bf16_t *dst = vt + ((int64_t)s * Hkv + kvh) * (int64_t)DH * lpadv;
    for (int idx = threadIdx.x; idx < 64 * DH; idx += 256) {
        const int k = idx / DH, d = idx - k * DH;
        tile[k][d] = (kb + k < len) ? src[(int64_t)(kb + k) * DH + d] : (bf16_t)0;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < 64 * DH; idx += 256) {
        const int d = idx >> 6, k = idx & 63;
        if (kb + k < lpadv) dst[(int64_t)d * lpadv + kb + k] = tile[k][d];
    }
}

template <int BQ, int SLOTS, int DH, int AT_WAVES>
static bool launch_attn_tile_t(const void *q, const void *kc, const void *vt, float *o32, const RowAct *ra,
                               const int32_t *pos0, int n_seq, int Tn, int L_max, int Hq, int Hkv, int lpadv,
                               hipStream_t st)
{
    constexpr int AT_BLOCK = AT_WAVES * 64;
    auto kern = k_attn_tile<BQ, SLOTS, DH, AT_WAVES>;
    const size_t score_bytes = (size_t)BQ * (SLOTS * 64 + 4) * 4;
    const size_t red_bytes = (size_t)AT_WAVES * BQ * DH * 4;
    const size_t lds = score_bytes > red_bytes ? score_bytes : red_bytes;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return false;
        attr_done = true;
    }
    const float scale = 1.0f / sqrtf((float)DH);
    hipLaunchKernelGGL(kern, dim3((Tn + BQ - 1) / BQ, Hq, n_seq), dim3(AT_BLOCK), lds, st, (const bf16_t *)q,
                       (const bf16_t *)kc, (const bf16_t *)vt, o32, ra, pos0, Tn, L_max, Hq, Hkv, lpadv, scale);
    return true;
}

int attn_tile_lpadv(int L_max) { return (L_max + 63) & ~63; }

bool launch_attn_tile(const void *q, const void *k_cache, const void *v_cache, void *vt, float *o32, const RowAct *ra,
                      const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh, hipStream_t st)
{
    if ((int64_t)n_seq * T <= 0) return true;
    if ((dh != 64 && dh != 128) || L_max > 4096 || T < 16) return false;
    const int lpadv = attn_tile_lpadv(L_max);
    const dim3 tg((lpadv + 63) / 64, Hkv, n_seq);
    if (dh == 64)
        hipLaunchKernelGGL((k_transpose_v<64>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
    else
        hipLaunchKernelGGL((k_transpose_v<128>), tg, dim3(256), 0, st, (const bf16_t *)v_cache, (bf16_t *)vt, pos0, T,
                           L_max, Hkv, lpadv);
#define SOL_AT(BQ, SL, NW)                                                                                                  \
    return dh == 64 ? launch_attn_tile_t<BQ, SL, 64, NW>(q, k_cache, vt, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, st) \
                    : launch_attn_tile_t<BQ, SL, 128, NW>(q, k_cache, vt, o32, ra, pos0, n_seq, T, L_max, Hq, Hkv, lpadv, st)
    if (L_max <= 256) { SOL_AT(32, 4, 8); }
    // 16 rows keep the score rows of two workgroups resident per CU (2 x 66 KB of LDS), so one
    // workgroup's load / MFMA phases overlap the other's selection phase: measured 3.1 ms against
    // 4.7 ms for one 32-row workgroup per CU on the 32 x 1024-token layer
    if (L_max <= 1024) { SOL_AT(16, 16, 8); }
    if (L_max <= 2048) { SOL_AT(16, 32, 8); }
    SOL_AT(8, 64, 8);
#undef SOL_AT
}

}  // namespace sol
