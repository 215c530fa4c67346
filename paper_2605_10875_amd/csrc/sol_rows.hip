// Row-wise kernels (one workgroup per token row): action decode + bucketing, RMSNorm with the
// fake-quantise epilogue, magnitude pruning + quantise, rotary/scatter, residuals, NLL rows and
// the unit hooks. All HBM-bound; rows are contiguous, so accesses are coalesced.
#include "sol_internal.h"

namespace sol {

// ------------------------------------------------------------------------------------------------
// action decode (Method, "Actions and controlled compute": a -> (kappa, rho, q))
// ------------------------------------------------------------------------------------------------
__global__ void k_prepare_rows(const int32_t *__restrict__ ids, const ActionDev *__restrict__ table, int n_actions,
                               int d_ff /* width of the pruned vector */, int64_t M, RowAct *__restrict__ ra, int32_t *__restrict__ row_bucket,
                               int *flags)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= M) return;
    const int id = ids[r];
    RowAct a;
    int bucket = 0;
    if (id < 0 || id >= n_actions) {
        atomicOr(flags, FLAG_BAD_ACTION);
        a.keep_num = 1; a.keep_den = 1; a.m = d_ff; a.bits = 16;
        bucket = 0;
    } else {
        const ActionDev t = table[id];
        a.keep_num = t.keep_num; a.keep_den = t.keep_den;
        a.m = budget_ceil(t.mlp_keep_num, t.mlp_keep_den, d_ff);
        a.bits = (int)t.bits;
        bucket = t.bucket;
    }
    ra[r] = a;
    row_bucket[r] = bucket;
}

// dst [N][Hkv][L_dst][dh] <- src [N / K][Hkv][P][dh] for positions < P (16-byte pieces): the K schedules of an
// input start from the same prefix cache
__global__ void __launch_bounds__(256)
k_bcast_prefix(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int K, int Hkv, int P, int L_dst, int row16, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % row16);
    int64_t t = i / row16;
    const int j = (int)(t % P); t /= P;
    const int h = (int)(t % Hkv);
    const int64_t n = t / Hkv;
    dst[((n * Hkv + h) * L_dst + j) * row16 + c] = src[(((n / K) * Hkv + h) * P + j) * row16 + c];
}

void launch_bcast_prefix(const void *src, void *dst, int64_t N, int K, int Hkv, int P, int L_dst, int dh, size_t esize,
                         hipStream_t st)
{
    const int row16 = (int)(dh * esize / 16);
    const int64_t total = N * Hkv * P * row16;
    if (total <= 0) return;
    hipLaunchKernelGGL(k_bcast_prefix, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint4 *)src,
                       (uint4 *)dst, K, Hkv, P, L_dst, row16, total);
}

__global__ void k_fill_i32(int32_t *p, int v, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

void launch_fill_i32(int32_t *p, int v, int64_t n, hipStream_t st)
{
    if (n > 0) hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
}

// every row under the dense action: keep all keys, all `width` channels, quantiser bypassed
__global__ void k_dense_rows(int width, int64_t M, RowAct *__restrict__ ra, int32_t *__restrict__ row_bucket)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= M) return;
    RowAct a;
    a.keep_num = 1; a.keep_den = 1; a.m = width; a.bits = 16;
    ra[r] = a;
    row_bucket[r] = 0;
}

void launch_dense_rows(int width, int64_t M, RowAct *ra, int32_t *row_bucket, hipStream_t st)
{
    if (M <= 0) return;
    hipLaunchKernelGGL(k_dense_rows, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, st, width, M, ra, row_bucket);
}

void launch_prepare_rows(const int32_t *action_ids, const ActionDev *table, int n_actions, int d_ff, int64_t M,
                         RowAct *ra, int32_t *row_bucket, int *flags, hipStream_t st)
{
    if (M <= 0) return;
    hipLaunchKernelGGL(k_prepare_rows, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, st, action_ids, table,
                       n_actions, d_ff, M, ra, row_bucket, flags);
}

// ------------------------------------------------------------------------------------------------
// stable counting sort of rows by MLP bucket (one workgroup; M is at most a few 10^5 rows)
// ------------------------------------------------------------------------------------------------
constexpr int SORT_BLOCK = 1024;
constexpr int SORT_GROUP = 8;

__global__ void __launch_bounds__(SORT_BLOCK)
k_bucket_sort(const int32_t *__restrict__ row_bucket, int64_t M, int n_buckets, int32_t *__restrict__ perm,
              int32_t *__restrict__ bucket_off)
{
    __shared__ int wtot[SORT_BLOCK / 64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t seg = (M + SORT_BLOCK - 1) / SORT_BLOCK;
    const int64_t r0 = (int64_t)tid * seg;
    const int64_t r1 = (r0 + seg < M) ? r0 + seg : M;
    int base = 0;
    for (int g0 = 0; g0 < n_buckets; g0 += SORT_GROUP) {
        int cnt[SORT_GROUP];
#pragma unroll
        for (int b = 0; b < SORT_GROUP; ++b) cnt[b] = 0;
        for (int64_t r = r0; r < r1; ++r) {
            const int b = row_bucket[r] - g0;
#pragma unroll
            for (int bb = 0; bb < SORT_GROUP; ++bb) cnt[bb] += (b == bb);
        }
        int start[SORT_GROUP];
#pragma unroll
        for (int b = 0; b < SORT_GROUP; ++b) {
            int incl = cnt[b];
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o, 64);
                if (lane >= o) incl += t;
            }
            if (lane == 63) wtot[w] = incl;
            __syncthreads();
            int woff = 0, total = 0;
#pragma unroll
            for (int j = 0; j < SORT_BLOCK / 64; ++j) {
                const int c = wtot[j];
                if (j < w) woff += c;
                total += c;
            }
            __syncthreads();
            start[b] = base + woff + incl - cnt[b];
            if (tid == 0 && g0 + b < n_buckets) bucket_off[g0 + b] = base;
            base += total;
        }
        for (int64_t r = r0; r < r1; ++r) {
            const int b = row_bucket[r] - g0;
#pragma unroll
            for (int bb = 0; bb < SORT_GROUP; ++bb)
                if (b == bb) perm[start[bb]++] = (int32_t)r;
        }
    }
    if (tid == 0) bucket_off[n_buckets] = base;
}

void launch_bucket_sort(const int32_t *row_bucket, int64_t M, int n_buckets, int32_t *perm, int32_t *bucket_off,
                        hipStream_t st)
{
    if (M <= 0) return;
    hipLaunchKernelGGL(k_bucket_sort, dim3(1), dim3(SORT_BLOCK), 0, st, row_bucket, M, n_buckets, perm, bucket_off);
}

// ------------------------------------------------------------------------------------------------
// RMSNorm (+ optional residual add) + per-token fake-quantise epilogue
// ------------------------------------------------------------------------------------------------
constexpr int ROW_BLOCK = 256;

template <typename TX, typename TW, typename TH>
__global__ void __launch_bounds__(ROW_BLOCK)
k_rmsnorm_fq(const TX *__restrict__ x, const float *__restrict__ add, int nsplit, int64_t split_stride,
             float *__restrict__ xsum, const TW *__restrict__ w, TH *__restrict__ h, const RowAct *__restrict__ ra,
             int quant, int d, float eps)
{
    extern __shared__ float row[];
    __shared__ float red[ROW_BLOCK / 64];
    const int64_t r = blockIdx.x;
    const int tid = threadIdx.x;
    const TX *xr = x + r * d;
    float ss = 0.f;
    for (int j = tid; j < d; j += ROW_BLOCK) {
        float v = ld(xr + j);
        if (add) {
            float t = 0.f;
            for (int sp = 0; sp < nsplit; ++sp) t += add[sp * split_stride + r * d + j];   // fixed split order
            v += t;
        }
        if (xsum) xsum[r * d + j] = v;
        row[j] = v;
        ss += v * v;
    }
    ss = block_sum<ROW_BLOCK>(ss, red);
    const float rinv = 1.0f / sqrtf(ss / (float)d + eps);
    float amax = 0.f;
    for (int j = tid; j < d; j += ROW_BLOCK) {
        const float v = row[j] * rinv * ld(w + j);
        row[j] = v;
        amax = fmaxf(amax, fabsf(v));
    }
    const int bits = (quant && ra) ? ra[r].bits : 16;
    TH *hr = h + r * d;
    if (bits < 16) {
        amax = block_max<ROW_BLOCK>(amax, red);
        if (amax > 0.f) {
            const float qmax = fq_qmax(bits);
            const float s = amax / qmax;
            for (int j = tid; j < d; j += ROW_BLOCK) st(hr + j, fq_code(row[j], s, qmax) * s);
            return;
        }
    }
    for (int j = tid; j < d; j += ROW_BLOCK) st(hr + j, row[j]);
}

// One wave per row, the row in registers (d = CH * 512: lane l holds elements [c*512 + 8*l, +8) of every chunk
// c), 16-byte accesses, reductions on DPP: the layer's bf16 pass, where x is bf16 (layer input) or fp32 (the
// residual stream inside the layer), the gain and the output are bf16 and there is nothing to add.
typedef uint32_t u32x4_w __attribute__((ext_vector_type(4)));
typedef float f32x4_w __attribute__((ext_vector_type(4)));

// Keeps the m entries of largest magnitude of a row held by one wave (lane l holds elements
// (c * 64 + l) * 8 .. + 8 of chunk c) and zeroes the rest; equal magnitudes go to the lower channel.
// |x| of an fp32 orders like its bit pattern, so the m-th largest magnitude is found on integer keys: pivots
// by regula falsi (Illinois) on g(t) = #(|x| >= t) - m + 1/2 in the value domain, the midpoint of the key range
// after 12 steps or a guess outside the bracket.
template <int CH>
__device__ __forceinline__ void wave_keep_topm(float (&v)[CH][8], int m, int lane)
{
    constexpr int D = CH * 512;
    auto count_ge = [&](uint32_t t) -> int {
        int cnt = 0;
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) cnt += __popcll(__ballot((__float_as_uint(v[c][e]) & 0x7FFFFFFFu) >= t));
        return cnt;
    };
    uint32_t kmax = 0u;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t k = __float_as_uint(v[c][e]) & 0x7FFFFFFFu;
            kmax = k > kmax ? k : kmax;
        }
    uint32_t lo = 0u, hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_max_u32(kmax));
    // invariant: count(key >= lo) >= m, count(key >= hi + 1) < m
    float glo = (float)(D - m) + 0.5f, ghi = 0.5f - (float)m;
    int side = 0;
    bool exact = false;
    for (int it = 0; lo < hi; ++it) {
        const float flo = __uint_as_float(lo), fhi = __uint_as_float(hi);
        const float fp = __builtin_fmaf(fhi - flo, glo * __builtin_amdgcn_rcpf(glo - ghi), flo);
        uint32_t mid = (uint32_t)__builtin_amdgcn_readfirstlane((int)(__float_as_uint(fp) & 0x7FFFFFFFu));
        if (it >= 12 || !(mid > lo && mid <= hi)) mid = lo + ((hi - lo + 1u) >> 1);
        const int cnt = count_ge(mid);
        if (cnt == m) { lo = mid; exact = true; break; }
        const float g = (float)(cnt - m) + 0.5f;
        if (cnt > m) {
            lo = mid; glo = g;
            if (side > 0) ghi *= 0.5f;
            side = 1;
        } else {
            hi = mid - 1u; ghi = g;
            if (side < 0) glo *= 0.5f;
            side = -1;
        }
    }
    const uint32_t thr = lo;
    int quota = D;                                           // ties kept, in channel order
    if (!exact) {
        const int n_ge = count_ge(thr);
        if (n_ge > m) quota = m - count_ge(thr + 1u);
    }
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        int before = 0, total = 0;                           // ties in lower lanes / in the whole chunk
        bool tie[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            tie[e] = (__float_as_uint(v[c][e]) & 0x7FFFFFFFu) == thr;
            const unsigned long long bal = __ballot(tie[e]);
            before += __popcll(bal & lt_mask);
            total += __popcll(bal);
        }
        int mine = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t k = __float_as_uint(v[c][e]) & 0x7FFFFFFFu;
            const bool keep = k > thr || (tie[e] && before + mine < quota);
            mine += tie[e];
            if (!keep) v[c][e] = 0.f;
        }
        quota = quota > total ? quota - total : 0;
    }
}

template <typename TX, int CH, bool ADD>
__global__ void __launch_bounds__(256)
k_rmsnorm_fq_wave(const TX *__restrict__ x, const float *__restrict__ add, int nsplit, int64_t split_stride,
                  float *__restrict__ xsum, const bf16_t *__restrict__ w, bf16_t *__restrict__ h,
                  const RowAct *__restrict__ ra, int quant, int64_t M, float eps, int prune)
{
    constexpr int D = CH * 512;
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);   // 4 rows per workgroup, or 1 (few rows)
    if (r >= M) return;                                      // whole wave
    float v[CH][8];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        if constexpr (sizeof(TX) == 2) {
            const u32x4_w t = *reinterpret_cast<const u32x4_w *>(x + r * D + c * 512 + lane * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[c][2 * e] = __uint_as_float(t[e] << 16); v[c][2 * e + 1] = __uint_as_float(t[e] & 0xFFFF0000u); }
        } else {
            const f32x4_w t0 = *reinterpret_cast<const f32x4_w *>(x + r * D + c * 512 + lane * 8);
            const f32x4_w t1 = *reinterpret_cast<const f32x4_w *>(x + r * D + c * 512 + lane * 8 + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[c][e] = t0[e]; v[c][4 + e] = t1[e]; }
        }
    }
    if constexpr (ADD) {                                     // x + K-split partial sums (folded in split order), kept as xsum
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float t[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
            for (int sp = 0; sp < nsplit; ++sp) {           // unrolled: the loads of all splits go out together
                const float *ap = add + sp * split_stride + r * D + c * 512 + lane * 8;
                const f32x4_w a0 = *reinterpret_cast<const f32x4_w *>(ap), a1 = *reinterpret_cast<const f32x4_w *>(ap + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) { t[e] += a0[e]; t[4 + e] += a1[e]; }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) v[c][e] += t[e];
            float *xp = xsum + r * D + c * 512 + lane * 8;
            *reinterpret_cast<f32x4_w *>(xp) = f32x4_w{v[c][0], v[c][1], v[c][2], v[c][3]};
            *reinterpret_cast<f32x4_w *>(xp + 4) = f32x4_w{v[c][4], v[c][5], v[c][6], v[c][7]};
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += v[c][e] * v[c][e];
    ss = wave_sum_dpp(ss);
    const float rinv = 1.0f / sqrtf(ss / (float)D + eps);
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const u32x4_w t = *reinterpret_cast<const u32x4_w *>(w + c * 512 + lane * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[c][2 * e] = v[c][2 * e] * rinv * __uint_as_float(t[e] << 16);
            v[c][2 * e + 1] = v[c][2 * e + 1] * rinv * __uint_as_float(t[e] & 0xFFFF0000u);
            amax = fmaxf(amax, fmaxf(fabsf(v[c][2 * e]), fabsf(v[c][2 * e + 1])));
        }
    }
    if (prune) {                                             // pruning at the MLP input: ra.m of the D channels stay
        const int m = __builtin_amdgcn_readfirstlane(ra[r].m);
        if (m < D) wave_keep_topm<CH>(v, m, lane);           // (the largest magnitude stays, so amax is unchanged)
    }
    const int bits = (quant && ra) ? ra[r].bits : 16;
    if (bits < 16) {
        amax = __uint_as_float(wave_max_u32(__float_as_uint(amax)));     // non-negative floats order like their bits
        if (amax > 0.f) {
            const float qmax = fq_qmax(bits), s = amax / qmax;
#pragma unroll
            for (int c = 0; c < CH; ++c)
#pragma unroll
                for (int e = 0; e < 8; ++e) v[c][e] = fq_code(v[c][e], s, qmax) * s;
        }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        u32x4_w o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = pack_bf16x2(v[c][2 * e], v[c][2 * e + 1]);
        *reinterpret_cast<u32x4_w *>(h + r * D + c * 512 + lane * 8) = o;
    }
}

// the same layout for the row-wise fake-quantiser of an fp32 matrix into bf16
template <int CH>
__global__ void __launch_bounds__(256)
k_fq_rows_wave(const float *__restrict__ in, bf16_t *__restrict__ out, const RowAct *__restrict__ ra, int quant, int64_t M)
{
    constexpr int D = CH * 512;
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    float v[CH][8];
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const f32x4_w t0 = *reinterpret_cast<const f32x4_w *>(in + r * D + c * 512 + lane * 8);
        const f32x4_w t1 = *reinterpret_cast<const f32x4_w *>(in + r * D + c * 512 + lane * 8 + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[c][e] = t0[e]; v[c][4 + e] = t1[e]; amax = fmaxf(amax, fmaxf(fabsf(t0[e]), fabsf(t1[e]))); }
    }
    const int bits = (quant && ra) ? ra[r].bits : 16;
    if (bits < 16) {
        amax = __uint_as_float(wave_max_u32(__float_as_uint(amax)));
        if (amax > 0.f) {
            const float qmax = fq_qmax(bits), s = amax / qmax;
#pragma unroll
            for (int c = 0; c < CH; ++c)
#pragma unroll
                for (int e = 0; e < 8; ++e) v[c][e] = fq_code(v[c][e], s, qmax) * s;
        }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        u32x4_w o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = pack_bf16x2(v[c][2 * e], v[c][2 * e + 1]);
        *reinterpret_cast<u32x4_w *>(out + r * D + c * 512 + lane * 8) = o;
    }
}

// xsum = x + the K-split partial sums (folded in split order): what k_rmsnorm_fq_wave<.., true> computes in its first
// step, as a kernel of its own with one thread per 4 elements, for the short batches of a decode step whose rows each
// come with hundreds of KB of partial sums (the norm reads a row's sums with one wave)
template <typename TX>
__global__ void __launch_bounds__(256)
k_fold_resid(const TX *__restrict__ x, const float *__restrict__ add, int nsplit, int64_t split_stride,
             float *__restrict__ xsum, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    float t[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int sp = 0; sp < nsplit; ++sp) {
        const f32x4_w a = *reinterpret_cast<const f32x4_w *>(add + sp * split_stride + 4 * i);
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] += a[e];
    }
    f32x4_w v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = ld(x + 4 * i + e) + t[e];
    *reinterpret_cast<f32x4_w *>(xsum + 4 * i) = v;
}

template <typename TX, typename TW, typename TH>
static void rmsnorm_dispatch3(const void *x, const float *add, int nsplit, float *xsum, const void *w, void *h,
                              const RowAct *ra, bool quant, int64_t M, int d, float eps, hipStream_t st)
{
    hipLaunchKernelGGL((k_rmsnorm_fq<TX, TW, TH>), dim3((unsigned)M), dim3(ROW_BLOCK), (size_t)d * sizeof(float), st,
                       (const TX *)x, add, nsplit, M * (int64_t)d, xsum, (const TW *)w, (TH *)h, ra, quant ? 1 : 0, d, eps);
}

bool launch_rmsnorm_fq(const void *x, int x_dtype, const float *add, float *xsum, const void *w, int w_dtype, void *h,
                       int h_dtype, const RowAct *ra, bool quant, int64_t M, int d, float eps, hipStream_t st, int nsplit,
                       bool prune)
{
    if (M <= 0) return true;
    if (w_dtype == 1 && h_dtype == 1 && (d == 2048 || d == 4096) && (add != nullptr) == (xsum != nullptr)) {
        const int rpw = M <= 512 ? 1 : 4;                        // a decode step's few rows: one per workgroup, on as many CUs
        const dim3 grid((unsigned)((M + rpw - 1) / rpw)), block(64 * rpw);
        const int64_t ss = M * (int64_t)d;
        if (add && rpw == 1 && (int64_t)nsplit * 4 * d > (128 << 10)) {   // a row's partial sums: too much for one wave to
            const int64_t n4 = ss / 4;                           // read in a row (35 us for 256 KB); fold with the whole chip first
            const dim3 fg((unsigned)((n4 + 255) / 256));
            if (x_dtype == 1) hipLaunchKernelGGL((k_fold_resid<bf16_t>), fg, dim3(256), 0, st, (const bf16_t *)x, add, nsplit, ss, xsum, n4);
            else hipLaunchKernelGGL((k_fold_resid<float>), fg, dim3(256), 0, st, (const float *)x, add, nsplit, ss, xsum, n4);
            x = xsum, x_dtype = 0, add = nullptr, xsum = nullptr, nsplit = 1;
        }
#define SOL_NORM_WAVE(TX, CH)                                                                                   \
    if (add)                                                                                                    \
        hipLaunchKernelGGL((k_rmsnorm_fq_wave<TX, CH, true>), grid, block, 0, st, (const TX *)x, add, nsplit, ss, \
                           xsum, (const bf16_t *)w, (bf16_t *)h, ra, quant ? 1 : 0, M, eps, prune ? 1 : 0);     \
    else                                                                                                        \
        hipLaunchKernelGGL((k_rmsnorm_fq_wave<TX, CH, false>), grid, block, 0, st, (const TX *)x, add, nsplit, ss, \
                           xsum, (const bf16_t *)w, (bf16_t *)h, ra, quant ? 1 : 0, M, eps, prune ? 1 : 0)
        if (x_dtype == 1) { if (d == 2048) { SOL_NORM_WAVE(bf16_t, 4); } else { SOL_NORM_WAVE(bf16_t, 8); } }
        else { if (d == 2048) { SOL_NORM_WAVE(float, 4); } else { SOL_NORM_WAVE(float, 8); } }
#undef SOL_NORM_WAVE
        return true;
    }
    if (prune) return false;                                 // the caller prunes with the row kernels instead
    const int key = (x_dtype << 2) | (w_dtype << 1) | h_dtype;
    switch (key) {
    case 0: rmsnorm_dispatch3<float, float, float>(x, add, nsplit, xsum, w, h, ra, quant, M, d, eps, st); break;
    case 7: rmsnorm_dispatch3<bf16_t, bf16_t, bf16_t>(x, add, nsplit, xsum, w, h, ra, quant, M, d, eps, st); break;
    case 3: rmsnorm_dispatch3<float, bf16_t, bf16_t>(x, add, nsplit, xsum, w, h, ra, quant, M, d, eps, st); break;
    case 6: rmsnorm_dispatch3<bf16_t, bf16_t, float>(x, add, nsplit, xsum, w, h, ra, quant, M, d, eps, st); break;
    case 2: rmsnorm_dispatch3<float, bf16_t, float>(x, add, nsplit, xsum, w, h, ra, quant, M, d, eps, st); break;
    default: break;   // no other combination is ever requested by the host code
    }
    return true;
}

// ------------------------------------------------------------------------------------------------
// row-wise fake-quantise of an fp32 matrix into the storage type (attention output -> o-proj input)
// ------------------------------------------------------------------------------------------------
template <typename TO>
__global__ void __launch_bounds__(ROW_BLOCK)
k_fq_rows(const float *__restrict__ in, TO *__restrict__ out, const RowAct *__restrict__ ra, int quant, int n)
{
    __shared__ float red[ROW_BLOCK / 64];
    const int64_t r = blockIdx.x;
    const int tid = threadIdx.x;
    const float *ir = in + r * n;
    TO *orow = out + r * n;
    const int bits = (quant && ra) ? ra[r].bits : 16;
    if (bits < 16) {
        float amax = 0.f;
        for (int j = tid; j < n; j += ROW_BLOCK) amax = fmaxf(amax, fabsf(ir[j]));
        amax = block_max<ROW_BLOCK>(amax, red);
        if (amax > 0.f) {
            const float qmax = fq_qmax(bits);
            const float s = amax / qmax;
            for (int j = tid; j < n; j += ROW_BLOCK) st(orow + j, fq_code(ir[j], s, qmax) * s);
            return;
        }
    }
    for (int j = tid; j < n; j += ROW_BLOCK) st(orow + j, ir[j]);
}

void launch_fq_rows(const float *in, void *out, int out_dtype, const RowAct *ra, bool quant, int64_t M, int n,
                    hipStream_t st)
{
    if (M <= 0) return;
    if (out_dtype == 1 && (n == 2048 || n == 4096)) {
        const dim3 grid((unsigned)((M + 3) / 4));
        if (n == 2048) hipLaunchKernelGGL((k_fq_rows_wave<4>), grid, dim3(256), 0, st, in, (bf16_t *)out, ra, quant ? 1 : 0, M);
        else hipLaunchKernelGGL((k_fq_rows_wave<8>), grid, dim3(256), 0, st, in, (bf16_t *)out, ra, quant ? 1 : 0, M);
        return;
    }
    if (out_dtype == 0)
        hipLaunchKernelGGL((k_fq_rows<float>), dim3((unsigned)M), dim3(ROW_BLOCK), 0, st, in, (float *)out, ra,
                           quant ? 1 : 0, n);
    else
        hipLaunchKernelGGL((k_fq_rows<bf16_t>), dim3((unsigned)M), dim3(ROW_BLOCK), 0, st, in, (bf16_t *)out, ra,
                           quant ? 1 : 0, n);
}

// ------------------------------------------------------------------------------------------------
// rotary embedding (rotate-half pairs (c, c + dh/2)) and scatter of q, k, v
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
k_rope_store(const float *__restrict__ qkv, int nsplit, int64_t split_stride, T *__restrict__ q, T *__restrict__ kc,
             T *__restrict__ vc, const float2 *__restrict__ rope, const int32_t *__restrict__ pos0, int Tn, int L_max,
             int Hq, int Hkv, int dh, int *flags, int crows)
{
    auto val = [&](const float *p) {                       // folds K-split partial sums in split order
        float t = 0.f;
#pragma unroll 8
        for (int sp = 0; sp < nsplit; ++sp) t += p[sp * split_stride];
        return t;
    };
    // grid: (row, head slot) with head slots 0..Hq-1 = q heads, then the K heads, then the V heads; a
    // workgroup of dh / 2 threads handles one head of one row, so all loads of a row are in flight at once
    const int64_t r = blockIdx.x;
    const int slot = blockIdx.y;
    const int s = (int)(r / Tn), i = (int)(r % Tn);
    const int p0 = pos0 ? pos0[s] : 0;
    if (p0 < 0 || p0 + Tn > L_max) {
        if (threadIdx.x == 0 && slot == 0) atomicOr(flags, FLAG_CACHE_OVERFLOW);
        return;
    }
    const int pos = p0 + i, half = dh >> 1;
    const int ncol = (Hq + 2 * Hkv) * dh;
    const float *in = qkv + r * ncol + (int64_t)slot * dh;
    const int c = threadIdx.x;                             // < half
    if (slot < Hq + Hkv) {                                 // q or k head: rotate the pair (c, c + half)
        const float x0 = val(in + c), x1 = val(in + c + half);
        const float2 t = rope[(int64_t)pos * half + c];
        T *dst = slot < Hq ? q + r * (int64_t)(Hq * dh) + slot * dh
                           : kc + (((int64_t)s * Hkv + (slot - Hq)) * crows + pos) * dh;
        st(dst + c, x0 * t.x - x1 * t.y);
        st(dst + c + half, x1 * t.x + x0 * t.y);
    } else {
        T *dst = vc + (((int64_t)s * Hkv + (slot - Hq - Hkv)) * crows + pos) * dh;
        st(dst + c, val(in + c));
        st(dst + c + half, val(in + c + half));
    }
}

void launch_rope_store(const float *qkv32, void *q, void *k_cache, void *v_cache, int dtype, const float2 *rope,
                       const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh, int *flags,
                       hipStream_t st, int nsplit, int cache_rows)
{
    const int64_t M = (int64_t)n_seq * T;
    if (M <= 0) return;
    const int crows = cache_rows > 0 ? cache_rows : L_max;
    const int64_t ss = M * (int64_t)((Hq + 2 * Hkv) * dh);
    if (dtype == 0)
        hipLaunchKernelGGL((k_rope_store<float>), dim3((unsigned)M, Hq + 2 * Hkv), dim3(dh / 2), 0, st, qkv32, nsplit, ss, (float *)q,
                           (float *)k_cache, (float *)v_cache, rope, pos0, T, L_max, Hq, Hkv, dh, flags, crows);
    else
        hipLaunchKernelGGL((k_rope_store<bf16_t>), dim3((unsigned)M, Hq + 2 * Hkv), dim3(dh / 2), 0, st, qkv32, nsplit, ss, (bf16_t *)q,
                           (bf16_t *)k_cache, (bf16_t *)v_cache, rope, pos0, T, L_max, Hq, Hkv, dh, flags, crows);
}

// ------------------------------------------------------------------------------------------------
// SwiGLU elementwise: a = g * sigmoid(g) * u
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float silu_mul(float g, float u) { return (g / (1.0f + expf(-g))) * u; }

template <typename T>
__global__ void k_silu_mul(const float *__restrict__ gu, int nsplit, T *__restrict__ a, int64_t M, int dff)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= M * dff) return;
    const int64_t r = idx / dff;
    const int c = (int)(idx - r * dff);
    float g = 0.f, u = 0.f;
#pragma unroll 8
    for (int sp = 0; sp < nsplit; ++sp) {                  // K-split partial sums, fixed order
        g += gu[(sp * M + r) * 2 * dff + c];
        u += gu[(sp * M + r) * 2 * dff + dff + c];
    }
    st(a + idx, silu_mul(g, u));
}

void launch_silu_mul(const float *gu32, void *a, int dtype, int64_t M, int dff, hipStream_t st, int nsplit)
{
    const int64_t n = M * dff;
    if (n <= 0) return;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (dtype == 0) hipLaunchKernelGGL((k_silu_mul<float>), dim3(grid), dim3(256), 0, st, gu32, nsplit, (float *)a, M, dff);
    else hipLaunchKernelGGL((k_silu_mul<bf16_t>), dim3(grid), dim3(256), 0, st, gu32, nsplit, (bf16_t *)a, M, dff);
}

// ------------------------------------------------------------------------------------------------
// per-token magnitude pruning + fake-quantise, in place (down-projection input)
// ------------------------------------------------------------------------------------------------
struct MagKeyLds {
    const float *row;
    __device__ __forceinline__ uint32_t operator()(int i) const { return mag_key(row[i]); }
};

template <typename T>
__global__ void __launch_bounds__(ROW_BLOCK)
k_prune_fq(T *__restrict__ a, const RowAct *__restrict__ ra, const int32_t *__restrict__ perm, int quant, int prune,
           int dff)
{
    extern __shared__ float row[];
    __shared__ int hist[256];
    __shared__ int sh[4];
    __shared__ int wcnt[ROW_BLOCK / 64];
    __shared__ float red[ROW_BLOCK / 64];
    const int64_t r = perm ? perm[blockIdx.x] : (int64_t)blockIdx.x;
    const RowAct act = ra[r];
    const int bits = quant ? act.bits : 16;
    const int m = prune ? act.m : dff;
    if (m >= dff && bits >= 16) return;          // dense bucket: the row is already final
    const int tid = threadIdx.x;
    T *ar = a + r * dff;
    float amax = 0.f;
    for (int j = tid; j < dff; j += ROW_BLOCK) {
        const float v = ld(ar + j);
        row[j] = v;
        amax = fmaxf(amax, fabsf(v));
    }
    __syncthreads();
    if (m < dff) {
        MagKeyLds kf{row};
        uint32_t thr; int quota, n_eq;
        block_radix_select<ROW_BLOCK>(kf, dff, m, hist, sh, thr, quota, n_eq);
        int J = dff;
        if (quota < n_eq) J = block_tie_cutoff<ROW_BLOCK>(kf, dff, thr, quota, wcnt, sh);
        for (int j = tid; j < dff; j += ROW_BLOCK) {
            const uint32_t key = mag_key(row[j]);
            const bool keep = key > thr || (key == thr && j <= J);
            if (!keep) row[j] = 0.f;
        }
    }
    if (bits < 16) {
        amax = block_max<ROW_BLOCK>(amax, red);   // the largest magnitude is always kept
        if (amax > 0.f) {
            const float qmax = fq_qmax(bits);
            const float s = amax / qmax;
            for (int j = tid; j < dff; j += ROW_BLOCK) st(ar + j, fq_code(row[j], s, qmax) * s);
            return;
        }
    }
    for (int j = tid; j < dff; j += ROW_BLOCK) st(ar + j, row[j]);
}

// bf16 rows whose length is a multiple of 512: one WAVE per row, the whole row in registers as packed
// bf16 pairs (lane l holds elements (c*64 + l)*8 .. +8 of chunk c), no LDS, no barriers.
//   - |a| of a bf16 is a 15-bit integer key, so the m-th largest magnitude is found by bisecting at
//     most 15 times; a pass counts keys below the pivot two at a time (packed 16-bit subtract, sign
//     bits, popcount) and reduces over the wave on DPP.
//   - bf16 magnitudes collide all the time (about 20 channels share the threshold value at
//     d_ff = 8192), so the tie rule (lower channel wins) always runs: ballots per element slot give
//     each tied channel its rank in channel order.
//   - the quantiser then works on the kept values in fp32 with true IEEE division.
typedef uint32_t u32x4_r __attribute__((ext_vector_type(4)));
typedef short i16x2_r __attribute__((ext_vector_type(2)));

// NWV waves share a row (NWV = 1: one wave per row, for many rows; NWV = 4: a workgroup per row, for the few
// rows of a decode step, where the latency of one row's search is what counts). Wave v holds chunks
// [v * CW, (v + 1) * CW) of 512 channels each; counts are combined through LDS.
// The row takes 4 registers per chunk; without a floor on the waves per SIMD the compiler spreads the unrolled passes
// over the whole register file (256 registers, one wave per SIMD) and nothing hides the latency of the DPP
// reductions and ballots: the floor caps the registers at 128 for up to 16 chunks per wave (at 16 chunks 24 values
// spill; three waves per SIMD without spills measure the same). Rows of more than 16 chunks are shared by four (or
// two) waves also when there are many rows: one wave per row at 28 chunks either spills 196 values (three waves per
// SIMD) or takes 256 registers; 0.99 / 0.71 / 0.65 ms for 32768 rows of 14336 (one wave spilling / one wave / four).
template <int CHUNKS, int NWV>
__global__ void __launch_bounds__(64 * NWV)
__attribute__((amdgpu_waves_per_eu(CHUNKS / NWV <= 16 ? 4 : 2, 8)))
k_prune_fq_wave(bf16_t *__restrict__ a, const RowAct *__restrict__ ra, const int32_t *__restrict__ perm, int quant,
                int prune, int64_t M)
{
    constexpr int DFF = CHUNKS * 512, CW = CHUNKS / NWV;
    static_assert(CHUNKS % NWV == 0, "chunks must split evenly over the waves");
    __shared__ uint32_t s_x[2][NWV];                         // per-wave partial results, double-buffered
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t slot = blockIdx.x;
    if (slot >= M) return;
    const int64_t r = perm ? perm[slot] : slot;
    const RowAct act = ra[r];
    const int bits = __builtin_amdgcn_readfirstlane(quant ? act.bits : 16);
    const int m = __builtin_amdgcn_readfirstlane(prune ? act.m : DFF);
    if (m >= DFF && bits >= 16) return;                      // dense bucket: the row is already final (whole workgroup)
    bf16_t *ar = a + r * DFF + (int64_t)wv * CW * 512;
    u32x4_r d[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) d[c] = *reinterpret_cast<const u32x4_r *>(ar + (c * 64 + lane) * 8);
    int xpar = 0;
    // sum (or maximum) of a wave-uniform value over the waves of the row
#define SOL_ROW_COMBINE(V_, IS_MAX_)                                                                       \
    if constexpr (NWV > 1) {                                                                               \
        if (lane == 0) s_x[xpar][wv] = (V_);                                                               \
        __syncthreads();                                                                                   \
        uint32_t t_ = 0u;                                                                                  \
        _Pragma("unroll") for (int i_ = 0; i_ < NWV; ++i_) {                                               \
            const uint32_t y_ = s_x[xpar][i_];                                                             \
            t_ = (IS_MAX_) ? (y_ > t_ ? y_ : t_) : t_ + y_;                                                \
        }                                                                                                  \
        (V_) = (uint32_t)__builtin_amdgcn_readfirstlane((int)t_);                                          \
        xpar ^= 1;                                                                                         \
    }

    // largest magnitude key of the row
    uint32_t kmax = 0u;
#pragma unroll
    for (int c = 0; c < CW; ++c)
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            const uint32_t k2 = d[c][wi] & 0x7FFF7FFFu;
            const uint32_t lo16 = k2 & 0xFFFFu, hi16 = k2 >> 16;
            kmax = lo16 > kmax ? lo16 : kmax;
            kmax = hi16 > kmax ? hi16 : kmax;
        }
    kmax = wave_max_u32(kmax);
    SOL_ROW_COMBINE(kmax, true);

    if (m < DFF) {
        // invariant: count(key >= lo) >= m, count(key >= hi + 1) < m. Pivots by regula falsi on
        // g(x) = count(key >= x) - m + 1/2 in the value domain (the key is the bf16 bit pattern of |a|) with the Illinois
        // correction, the midpoint of the key range after 10 steps or a guess outside (lo, hi]: about 9 counting passes
        // where bisection of the key takes 14-15.
        uint32_t lo = 0u, hi = kmax;
        float glo = (float)(DFF - m) + 0.5f, ghi = 0.5f - (float)m;
        int side = 0;
        for (int it = 0; lo < hi; ++it) {
            const float flo = __uint_as_float(lo << 16), fhi = __uint_as_float(hi << 16);
            const float fp = __builtin_fmaf(fhi - flo, glo * __builtin_amdgcn_rcpf(glo - ghi), flo);
            uint32_t mid = (uint32_t)__builtin_amdgcn_readfirstlane((int)((__float_as_uint(fp) >> 16) & 0x7FFFu));
            if (it >= 10 || !(mid > lo && mid <= hi)) mid = lo + ((hi - lo + 1u) >> 1);
            const uint32_t mid2 = mid | (mid << 16);
            uint32_t below = 0u;                             // keys < mid held by this lane
#pragma unroll
            for (int c = 0; c < CW; ++c)
#pragma unroll
                for (int wi = 0; wi < 4; ++wi) {
                    const i16x2_r diff = __builtin_bit_cast(i16x2_r, d[c][wi] & 0x7FFF7FFFu) - __builtin_bit_cast(i16x2_r, mid2);
                    below += __popc(__builtin_bit_cast(uint32_t, diff) & 0x80008000u);
                }
            uint32_t below_row = wave_reduce_dpp<uint32_t>(below, 0u, [](uint32_t x, uint32_t y) { return x + y; });
            SOL_ROW_COMBINE(below_row, false);
            const int cnt = DFF - (int)below_row;
            const float g = (float)(cnt - m) + 0.5f;
            if (cnt >= m) {
                lo = mid; glo = g;
                if (side > 0) ghi *= 0.5f;
                side = 1;
            } else {
                hi = mid - 1u; ghi = g;
                if (side < 0) glo *= 0.5f;
                side = -1;
            }
        }
        const uint32_t thr = lo, thr2 = thr | (thr << 16);
        // keys above the threshold, then ties in channel order until the quota is used up
        uint32_t above = 0u, ties = 0u;
#pragma unroll
        for (int c = 0; c < CW; ++c)
#pragma unroll
            for (int wi = 0; wi < 4; ++wi) {
                const uint32_t k2 = d[c][wi] & 0x7FFF7FFFu;
                const i16x2_r diff = __builtin_bit_cast(i16x2_r, thr2) - __builtin_bit_cast(i16x2_r, k2);
                above += __popc(__builtin_bit_cast(uint32_t, diff) & 0x80008000u);      // thr < key
                if constexpr (NWV > 1) ties += ((k2 & 0xFFFFu) == thr) + ((k2 >> 16) == thr);
            }
        uint32_t above_row = wave_reduce_dpp<uint32_t>(above, 0u, [](uint32_t x, uint32_t y) { return x + y; });
        SOL_ROW_COMBINE(above_row, false);
        int quota = m - (int)above_row;
        if constexpr (NWV > 1) {                             // ties held by the waves before this one come first
            const uint32_t ties_w = wave_reduce_dpp<uint32_t>(ties, 0u, [](uint32_t x, uint32_t y) { return x + y; });
            if (lane == 0) s_x[xpar][wv] = ties_w;
            __syncthreads();
            int before_w = 0;
#pragma unroll
            for (int i = 0; i < NWV; ++i) before_w += i < wv ? (int)s_x[xpar][i] : 0;
            xpar ^= 1;
            quota -= __builtin_amdgcn_readfirstlane(before_w);
            if (quota < 0) quota = 0;
        }
        const unsigned long long lt_mask = (1ull << lane) - 1ull;
#pragma unroll
        for (int c = 0; c < CW; ++c) {
            int before = 0, total = 0;                       // ties in lower lanes / in the whole chunk
            bool tie[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t k = (e & 1) ? ((d[c][e >> 1] >> 16) & 0x7FFFu) : (d[c][e >> 1] & 0x7FFFu);
                tie[e] = k == thr;
                const unsigned long long bal = __ballot(tie[e]);
                before += __popcll(bal & lt_mask);
                total += __popcll(bal);
            }
            int mine = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t k = (e & 1) ? ((d[c][e >> 1] >> 16) & 0x7FFFu) : (d[c][e >> 1] & 0x7FFFu);
                const bool keep = k > thr || (tie[e] && before + mine < quota);
                mine += tie[e];
                if (!keep) d[c][e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
            }
            quota = quota > total ? quota - total : 0;
            __builtin_amdgcn_sched_barrier(0);               // one chunk's ballots at a time
        }
    }
#undef SOL_ROW_COMBINE
    if (bits < 16 && kmax != 0u) {
        const float qmax = fq_qmax(bits);
        const float s = __uint_as_float(kmax << 16) / qmax;  // the largest magnitude is always kept
#pragma unroll
        for (int c = 0; c < CW; ++c)
#pragma unroll
            for (int wi = 0; wi < 4; ++wi) {
                const float v0 = __uint_as_float(d[c][wi] << 16), v1 = __uint_as_float(d[c][wi] & 0xFFFF0000u);
                d[c][wi] = pack_bf16x2(fq_code(v0, s, qmax) * s, fq_code(v1, s, qmax) * s);
                if (wi & 1) __builtin_amdgcn_sched_barrier(0);   // four divisions in flight are enough: more only cost registers
            }
    }
#pragma unroll
    for (int c = 0; c < CW; ++c) *reinterpret_cast<u32x4_r *>(ar + (c * 64 + lane) * 8) = d[c];
}

static bool prune_wave_case(int dtype, int dff)
{
    if (dtype != 1 || dff % 512) return false;
    const int c = dff / 512;
    return c == 2 || c == 4 || c == 8 || c == 16 || c == 22 || c == 28;
}

// The one-row-per-workgroup kernel wants rows of one action next to each other (workgroups of a CU then
// run the same number of search steps); the one-row-per-wave kernel has no use for the order.
bool prune_fq_wants_order(int dtype, int dff) { return !prune_wave_case(dtype, dff); }

void launch_prune_fq(void *a, int dtype, const RowAct *ra, const int32_t *perm, bool quant, int64_t M, int dff,
                     hipStream_t st, bool prune)
{
    if (M <= 0) return;
    if (prune_wave_case(dtype, dff)) {
        perm = nullptr;
        const dim3 grid((unsigned)M);
        const bool few = M <= 512 && (dff / 512) % 4 == 0;  // a decode step: four waves per row
#define SOL_PRUNE_CASE(C)                                                                                       \
    case C:                                                                                                     \
        if (few) hipLaunchKernelGGL((k_prune_fq_wave<C, (C % 4 == 0 ? 4 : 1)>), grid, dim3(C % 4 == 0 ? 256 : 64), 0, st, \
                                    (bf16_t *)a, ra, perm, quant ? 1 : 0, prune ? 1 : 0, M);                    \
        else hipLaunchKernelGGL((k_prune_fq_wave<C, (C > 16 ? (C % 4 == 0 ? 4 : 2) : 1)>), grid, dim3(64 * (C > 16 ? (C % 4 == 0 ? 4 : 2) : 1)), 0, st, (bf16_t *)a, ra, \
                                perm, quant ? 1 : 0, prune ? 1 : 0, M);       /* rows of more than 16 chunks: four (two) waves */ \
        return;
        switch (dff / 512) {
            SOL_PRUNE_CASE(2) SOL_PRUNE_CASE(4) SOL_PRUNE_CASE(8) SOL_PRUNE_CASE(16) SOL_PRUNE_CASE(22)
            SOL_PRUNE_CASE(28)
        default: break;
        }
#undef SOL_PRUNE_CASE
    }
    const size_t lds = (size_t)dff * sizeof(float);
    if (dtype == 0)
        hipLaunchKernelGGL((k_prune_fq<float>), dim3((unsigned)M), dim3(ROW_BLOCK), lds, st, (float *)a, ra, perm,
                           quant ? 1 : 0, prune ? 1 : 0, dff);
    else
        hipLaunchKernelGGL((k_prune_fq<bf16_t>), dim3((unsigned)M), dim3(ROW_BLOCK), lds, st, (bf16_t *)a, ra, perm,
                           quant ? 1 : 0, prune ? 1 : 0, dff);
}

// ------------------------------------------------------------------------------------------------
// residual add into the output type; embedding gather
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_resid_out(const float *__restrict__ x2, const float *__restrict__ z, int nsplit, T *__restrict__ out,
                            int64_t n)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    float t = 0.f;
#pragma unroll 8
    for (int sp = 0; sp < nsplit; ++sp) t += z[sp * n + idx];
    st(out + idx, x2[idx] + t);
}

void launch_resid_out(const float *x2, const float *z, void *out, int dtype, int64_t M, int d, hipStream_t st, int nsplit)
{
    const int64_t n = M * d;
    if (n <= 0) return;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (dtype == 0) hipLaunchKernelGGL((k_resid_out<float>), dim3(grid), dim3(256), 0, st, x2, z, nsplit, (float *)out, n);
    else hipLaunchKernelGGL((k_resid_out<bf16_t>), dim3(grid), dim3(256), 0, st, x2, z, nsplit, (bf16_t *)out, n);
}

// out = x2 + FQ(z, bits): the quantiser on the MLP block's output (the paper's own site, Appendix
// "Activation quantization"), one workgroup per row, the row of z in LDS.
template <typename T>
__global__ void __launch_bounds__(ROW_BLOCK)
k_resid_out_fq(const float *__restrict__ x2, const float *__restrict__ z, int nsplit, int64_t split_stride,
               T *__restrict__ out, const RowAct *__restrict__ ra, int d)
{
    extern __shared__ float row[];
    __shared__ float red[ROW_BLOCK / 64];
    const int64_t r = blockIdx.x;
    const int tid = threadIdx.x;
    const int bits = ra[r].bits;
    float amax = 0.f;
    for (int j = tid; j < d; j += ROW_BLOCK) {
        float t = 0.f;
        for (int sp = 0; sp < nsplit; ++sp) t += z[sp * split_stride + r * d + j];   // K-split partial sums, fixed order
        row[j] = t;
        amax = fmaxf(amax, fabsf(t));
    }
    amax = block_max<ROW_BLOCK>(amax, red);        // (its barriers also publish row[])
    const bool q = bits < 16 && amax > 0.f;
    const float qmax = q ? fq_qmax(bits) : 1.f;
    const float s = q ? amax / qmax : 1.f;
    for (int j = tid; j < d; j += ROW_BLOCK) {
        const float zz = q ? fq_code(row[j], s, qmax) * s : row[j];
        st(out + r * d + j, x2[r * d + j] + zz);
    }
}

// bf16 rows of 2048 / 4096: one workgroup of four waves per row, wave v holding chunks v, v + 4, .. of 512 values
// in registers (the K-split partial sums of a decode step are many: four waves keep four times the loads in flight)
template <int CH>
__global__ void __launch_bounds__(256)
k_resid_out_fq_wave(const float *__restrict__ x2, const float *__restrict__ z, int nsplit, int64_t split_stride,
                    bf16_t *__restrict__ out, const RowAct *__restrict__ ra, int64_t M)
{
    constexpr int D = CH * 512, CW = CH / 4;
    __shared__ float s_amax[4];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t r = blockIdx.x;
    float v[CW][8];
    float amax = 0.f;
#pragma unroll
    for (int cc = 0; cc < CW; ++cc) {
        const int c = wv + 4 * cc;
        float t[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int sp = 0; sp < nsplit; ++sp) {               // K-split partial sums, fixed order
            const float *zp = z + sp * split_stride + r * D + c * 512 + lane * 8;
            const f32x4_w a0 = *reinterpret_cast<const f32x4_w *>(zp), a1 = *reinterpret_cast<const f32x4_w *>(zp + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { t[e] += a0[e]; t[4 + e] += a1[e]; }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { v[cc][e] = t[e]; amax = fmaxf(amax, fabsf(t[e])); }
    }
    const int bits = ra[r].bits;
    if (bits < 16) {                                         // uniform over the workgroup
        amax = __uint_as_float(wave_max_u32(__float_as_uint(amax)));
        if (lane == 0) s_amax[wv] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(s_amax[0], s_amax[1]), fmaxf(s_amax[2], s_amax[3]));
        if (amax > 0.f) {
            const float qmax = fq_qmax(bits), s = amax / qmax;
#pragma unroll
            for (int cc = 0; cc < CW; ++cc)
#pragma unroll
                for (int e = 0; e < 8; ++e) v[cc][e] = fq_code(v[cc][e], s, qmax) * s;
        }
    }
#pragma unroll
    for (int cc = 0; cc < CW; ++cc) {
        const int c = wv + 4 * cc;
        const float *xp = x2 + r * D + c * 512 + lane * 8;
        const f32x4_w x0 = *reinterpret_cast<const f32x4_w *>(xp), x1 = *reinterpret_cast<const f32x4_w *>(xp + 4);
        u32x4_w o;
        o[0] = pack_bf16x2(x0[0] + v[cc][0], x0[1] + v[cc][1]);
        o[1] = pack_bf16x2(x0[2] + v[cc][2], x0[3] + v[cc][3]);
        o[2] = pack_bf16x2(x1[0] + v[cc][4], x1[1] + v[cc][5]);
        o[3] = pack_bf16x2(x1[2] + v[cc][6], x1[3] + v[cc][7]);
        *reinterpret_cast<u32x4_w *>(out + r * D + c * 512 + lane * 8) = o;
    }
}

void launch_resid_out_fq(const float *x2, const float *z, void *out, int dtype, const RowAct *ra, int64_t M, int d,
                         hipStream_t st, int nsplit)
{
    if (M <= 0) return;
    if (dtype == 1 && (d == 2048 || d == 4096)) {
        const dim3 grid((unsigned)M);
        if (d == 2048) hipLaunchKernelGGL((k_resid_out_fq_wave<4>), grid, dim3(256), 0, st, x2, z, nsplit, M * (int64_t)d, (bf16_t *)out, ra, M);
        else hipLaunchKernelGGL((k_resid_out_fq_wave<8>), grid, dim3(256), 0, st, x2, z, nsplit, M * (int64_t)d, (bf16_t *)out, ra, M);
        return;
    }
    const size_t lds = (size_t)d * sizeof(float);
    if (dtype == 0)
        hipLaunchKernelGGL((k_resid_out_fq<float>), dim3((unsigned)M), dim3(ROW_BLOCK), lds, st, x2, z, nsplit,
                           M * (int64_t)d, (float *)out, ra, d);
    else
        hipLaunchKernelGGL((k_resid_out_fq<bf16_t>), dim3((unsigned)M), dim3(ROW_BLOCK), lds, st, x2, z, nsplit,
                           M * (int64_t)d, (bf16_t *)out, ra, d);
}

template <typename T>
__global__ void k_embed(const T *__restrict__ embed, const int32_t *__restrict__ tokens, T *__restrict__ x, int G,
                        int Tn, int d, int vocab, int *__restrict__ flags)
{
    const int64_t r = blockIdx.x;                 // row = (b*G + g)*T + t
    const int t = (int)(r % Tn);
    const int b = (int)(r / ((int64_t)G * Tn));
    int tok = tokens[(int64_t)b * Tn + t];
    if (tok < 0 || tok >= vocab) {                 // outside the vocabulary: clamped, and reported through the sticky flag
        if (threadIdx.x == 0) atomicOr(flags, FLAG_BAD_TOKEN);
        tok = tok < 0 ? 0 : vocab - 1;
    }
    for (int j = threadIdx.x; j < d; j += blockDim.x) x[r * d + j] = embed[(int64_t)tok * d + j];
}

void launch_embed(const void *embed, const int32_t *tokens, void *x, int dtype, int B, int G, int T, int d, int vocab,
                  int *flags, hipStream_t st)
{
    const int64_t M = (int64_t)B * G * T;
    if (M <= 0) return;
    if (dtype == 0)
        hipLaunchKernelGGL((k_embed<float>), dim3((unsigned)M), dim3(256), 0, st, (const float *)embed, tokens,
                           (float *)x, G, T, d, vocab, flags);
    else
        hipLaunchKernelGGL((k_embed<bf16_t>), dim3((unsigned)M), dim3(256), 0, st, (const bf16_t *)embed, tokens,
                           (bf16_t *)x, G, T, d, vocab, flags);
}

// ------------------------------------------------------------------------------------------------
// NLL of materialised logits rows: logsumexp(l) - l[target]   (Method, Eq. 1, negated)
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(ROW_BLOCK)
k_nll_rows(const float *__restrict__ logits, int V, const int32_t *__restrict__ targets, int64_t row0, int G, int Tn,
           int broadcast_g, float *__restrict__ nll, int *__restrict__ flags)
{
    __shared__ float red[ROW_BLOCK / 64];
    const int64_t lr = blockIdx.x, r = row0 + lr;
    const float *l = logits + lr * V;
    float mx = -INFINITY;
    for (int v = threadIdx.x; v < V; v += ROW_BLOCK) mx = fmaxf(mx, l[v]);
    mx = block_max<ROW_BLOCK>(mx, red);
    float se = 0.f;
    for (int v = threadIdx.x; v < V; v += ROW_BLOCK) se += expf(l[v] - mx);
    se = block_sum<ROW_BLOCK>(se, red);
    if (threadIdx.x == 0) {
        const int64_t ti = broadcast_g ? (r / ((int64_t)G * Tn)) * Tn + (r % Tn) : r;
        int tg = targets[ti];
        if (tg < 0 || tg >= V) {                   // outside the vocabulary: clamped, and reported through the sticky flag
            atomicOr(flags, FLAG_BAD_TOKEN);
            tg = tg < 0 ? 0 : V - 1;
        }
        nll[r] = (mx + logf(se)) - l[tg];
    }
}

void launch_nll_rows(const float *logits, int64_t rows, int V, const int32_t *targets, int64_t row0, int G, int T,
                     bool broadcast_g, float *nll, int *flags, hipStream_t st)
{
    if (rows <= 0) return;
    hipLaunchKernelGGL(k_nll_rows, dim3((unsigned)rows), dim3(ROW_BLOCK), 0, st, logits, V, targets, row0, G, T,
                       broadcast_g ? 1 : 0, nll, flags);
}

// ------------------------------------------------------------------------------------------------
// unit hooks
// ------------------------------------------------------------------------------------------------
struct ScoreKeyGlobal {
    const float *row;
    __device__ __forceinline__ uint32_t operator()(int i) const { return score_key(row[i]); }
};
struct MagKeyGlobal {
    const float *row;
    __device__ __forceinline__ uint32_t operator()(int i) const { return mag_key(row[i]); }
};

template <typename KeyFn>
__device__ __forceinline__ void select_row_to_mask(KeyFn kf, int n_valid, int n_cols, int k, uint8_t *keep)
{
    __shared__ int hist[256];
    __shared__ int sh[4];
    __shared__ int wcnt[ROW_BLOCK / 64];
    const int tid = threadIdx.x;
    if (k >= n_valid) {
        for (int j = tid; j < n_cols; j += ROW_BLOCK) keep[j] = j < n_valid;
        return;
    }
    if (k <= 0) {
        for (int j = tid; j < n_cols; j += ROW_BLOCK) keep[j] = 0;
        return;
    }
    uint32_t thr; int quota, n_eq;
    block_radix_select<ROW_BLOCK>(kf, n_valid, k, hist, sh, thr, quota, n_eq);
    int J = n_valid;
    if (quota < n_eq) J = block_tie_cutoff<ROW_BLOCK>(kf, n_valid, thr, quota, wcnt, sh);
    for (int j = tid; j < n_cols; j += ROW_BLOCK) {
        uint8_t kp = 0;
        if (j < n_valid) {
            const uint32_t key = kf(j);
            kp = key > thr || (key == thr && j <= J);
        }
        keep[j] = kp;
    }
}

// the wave-level selection used by the tiled attention kernel: one wave per row, n_cols <= 64*SLOTS
template <int SLOTS>
__global__ void __launch_bounds__(64)
k_test_topk_wave(const float *__restrict__ scores, int n_cols, const int32_t *__restrict__ n_valid,
                 const int32_t *__restrict__ k, uint8_t *__restrict__ keep)
{
    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x;
    int nv = n_valid[r];
    nv = nv < 0 ? 0 : (nv > n_cols ? n_cols : nv);
    const int kk = k[r];
    uint32_t key[SLOTS];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int j = 0; j < SLOTS / 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int col = 256 * j + 4 * lane + e;
            const uint32_t kv = col < nv ? score_key(scores[r * n_cols + col]) : 0u;
            key[4 * j + e] = kv;
            kmax = kv > kmax ? kv : kmax;
            kmin = (col < nv && kv < kmin) ? kv : kmin;
        }
    kmax = wave_max_u32(kmax);
    kmin = wave_min_u32(kmin);
    uint32_t thr = 1u;                                   // keeps every valid key
    if (kk <= 0) thr = 0xFFFFFFFFu;
    else if (kk < nv) thr = wave_select_topk<SLOTS>(key, nv, kk, kmin, kmax, lane);
#pragma unroll
    for (int j = 0; j < SLOTS / 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int col = 256 * j + 4 * lane + e;
            if (col < n_cols) keep[r * n_cols + col] = (col < nv) && (kk > 0) && key[4 * j + e] >= thr;
        }
}

__global__ void __launch_bounds__(ROW_BLOCK)
k_test_topk(const float *__restrict__ scores, int n_cols, const int32_t *__restrict__ n_valid,
            const int32_t *__restrict__ k, uint8_t *__restrict__ keep)
{
    const int64_t r = blockIdx.x;
    int nv = n_valid[r];
    nv = nv < 0 ? 0 : (nv > n_cols ? n_cols : nv);
    ScoreKeyGlobal kf{scores + r * n_cols};
    select_row_to_mask(kf, nv, n_cols, k[r], keep + r * n_cols);
}

__global__ void __launch_bounds__(ROW_BLOCK)
k_test_prune(const float *__restrict__ a, int n, const int32_t *__restrict__ m, uint8_t *__restrict__ keep)
{
    const int64_t r = blockIdx.x;
    MagKeyGlobal kf{a + r * n};
    select_row_to_mask(kf, n, n, m[r], keep + r * n);
}

__global__ void __launch_bounds__(ROW_BLOCK)
k_test_quant(const float *__restrict__ z, int n, const int32_t *__restrict__ bits, int32_t *__restrict__ codes,
             float *__restrict__ scale, float *__restrict__ zhat)
{
    __shared__ float red[ROW_BLOCK / 64];
    const int64_t r = blockIdx.x;
    const int tid = threadIdx.x;
    const float *zr = z + r * n;
    const int b = bits[r];
    float amax = 0.f;
    for (int j = tid; j < n; j += ROW_BLOCK) amax = fmaxf(amax, fabsf(zr[j]));
    amax = block_max<ROW_BLOCK>(amax, red);
    if (b >= 16 || !(amax > 0.f)) {
        for (int j = tid; j < n; j += ROW_BLOCK) { codes[r * n + j] = 0; zhat[r * n + j] = zr[j]; }
        if (tid == 0) scale[r] = 0.f;
        return;
    }
    const float qmax = fq_qmax(b);
    const float s = amax / qmax;
    if (tid == 0) scale[r] = s;
    for (int j = tid; j < n; j += ROW_BLOCK) {
        const float c = fq_code(zr[j], s, qmax);
        codes[r * n + j] = (int32_t)c;
        zhat[r * n + j] = c * s;
    }
}

__global__ void k_fill_rowact(const int32_t *__restrict__ m, const int32_t *__restrict__ bits, RowAct *__restrict__ ra, int rows)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) ra[r] = RowAct{1u, 1u, m[r], bits[r]};
}

void launch_test_prune_quant(void *a, int dtype, int rows, int n, const int32_t *m, const int32_t *bits, void *scratch,
                             hipStream_t st)
{
    if (rows <= 0 || n <= 0) return;
    RowAct *ra = (RowAct *)scratch;
    hipLaunchKernelGGL(k_fill_rowact, dim3((rows + 255) / 256), dim3(256), 0, st, m, bits, ra, rows);
    launch_prune_fq(a, dtype, ra, nullptr, true, rows, n, st);
}

void launch_test_topk(const float *scores, int rows, int n_cols, const int32_t *n_valid, const int32_t *k,
                      uint8_t *keep, hipStream_t st)
{
    if (rows <= 0 || n_cols <= 0) return;
    // rows that fit a wave's registers go through the wave-level search of the tiled attention
    // kernel, longer rows through the workgroup-level radix select of the row / decode kernel
    if (n_cols <= 1024)
        hipLaunchKernelGGL((k_test_topk_wave<16>), dim3(rows), dim3(64), 0, st, scores, n_cols, n_valid, k, keep);
    else if (n_cols <= 4096)
        hipLaunchKernelGGL((k_test_topk_wave<64>), dim3(rows), dim3(64), 0, st, scores, n_cols, n_valid, k, keep);
    else
        hipLaunchKernelGGL(k_test_topk, dim3(rows), dim3(ROW_BLOCK), 0, st, scores, n_cols, n_valid, k, keep);
}
void launch_test_prune(const float *a, int rows, int n, const int32_t *m, uint8_t *keep, hipStream_t st)
{
    if (rows <= 0 || n <= 0) return;
    hipLaunchKernelGGL(k_test_prune, dim3(rows), dim3(ROW_BLOCK), 0, st, a, n, m, keep);
}
void launch_test_quant(const float *z, int rows, int n, const int32_t *bits, int32_t *codes, float *scale,
                       float *zhat, hipStream_t st)
{
    if (rows <= 0 || n <= 0) return;
    hipLaunchKernelGGL(k_test_quant, dim3(rows), dim3(ROW_BLOCK), 0, st, z, n, bits, codes, scale, zhat);
}

}  // namespace sol
