// bf16 MFMA GEMM for gfx950 with fused epilogues:  C[M][Nv] = A[M][K] * Wv[Nv][K]^T, fp32 accumulate.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants for A and B
// alike (each lane supplies 8 consecutive k of one row / one column). "Nv" is a virtual column
// space: a column maps to a row of one of up to three weight matrices (q|k|v stacked, or gate and
// up interleaved in 64-column halves so that SiLU(gate)*up is formed inside one wave tile).
//
// Tiling: workgroup tile BM x BN, K step 64; waves in a (BM/WM) x (BN/WN) grid, each wave owning
// WM x WN = (WM/32) x (WN/32) MFMA tiles of 32x32 in accumulator registers. A and B K-slices are
// staged through LDS (two stages, XOR-swizzled 16-byte chunks so that the 128-bit fragment reads
// are bank-conflict free) with the next slice prefetched into registers while the MFMAs of the
// current slice issue. Workgroups are mapped to tiles XCD-aware: each of the 8 XCDs walks its own
// contiguous band of the tile grid in groups of GROUP_M tile rows, so the tiles resident on an
// XCD at any time share A rows and B columns in that XCD's L2.
//
// Epilogue: accumulators are spilled 32 rows at a time through LDS into row-contiguous order and
// handed to an epilogue functor 4 columns per lane (rotary + cache write, residual add,
// SiLU(gate)*up, plain store).
#include "sol_internal.h"

namespace sol {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // native 16-byte vector (stays in registers)

constexpr int BK = 64;               // K step (bf16 elements); one LDS row = 128 bytes = 8 chunks of 16 B
constexpr int GROUP_M = 8;           // tile rows walked together by an XCD
// LDS has 64 banks of 4 bytes (256 B per clock): two 128-byte rows share one bank row, so the
// 16-byte chunk index is XOR-ed with bits 1..3 of the row. Measured SQ_LDS_BANK_CONFLICT drops 32x
// against swizzling with bits 0..2.
#ifndef SOL_SWZ
#define SOL_SWZ(r) (((r) >> 1) & 7)
#endif

struct BMap {                        // virtual column -> weight row
    const bf16_t *base[3];
    int seg_end[3];                  // mode 0: virtual columns [seg_end[i-1], seg_end[i]) belong to base[i]
    int mode;                        // 0 = stacked segments, 1 = gate/up interleaved in halves of `half`
    int half;
    int64_t ld;
    __device__ __forceinline__ const bf16_t *row(int v) const
    {
        if (mode == 0) {
            if (v < seg_end[0]) return base[0] + (int64_t)v * ld;
            if (v < seg_end[1]) return base[1] + (int64_t)(v - seg_end[0]) * ld;
            return base[2] + (int64_t)(v - seg_end[1]) * ld;
        }
        const int blk = v / (2 * half), w = v - blk * 2 * half;
        const int r = blk * half + (w < half ? w : w - half);
        return (w < half ? base[0] : base[1]) + (int64_t)r * ld;
    }
};

// ------------------------------------------------------------------------------------------------
// epilogues: apply(row, vcol0, lc, lrow) handles local columns [lc, lc+4) of a wave-tile row whose
// first virtual column is vcol0; lrow points at the fp32 row in LDS (WN floats).
// ------------------------------------------------------------------------------------------------
struct EpiStoreF32 {
    float *C; int64_t ldc;
    template <int WN> __device__ __forceinline__ void apply(int64_t row, int vcol0, int lc, const float *lrow) const
    {
        *reinterpret_cast<float4 *>(C + row * ldc + vcol0 + lc) = *reinterpret_cast<const float4 *>(lrow + lc);
    }
};

// x2 = resid + acc  (fp32 out), resid in bf16
struct EpiResidF32 {
    const bf16_t *resid; float *out; int64_t ld;
    template <int WN> __device__ __forceinline__ void apply(int64_t row, int vcol0, int lc, const float *lrow) const
    {
        const float4 v = *reinterpret_cast<const float4 *>(lrow + lc);
        const uint2 r = *reinterpret_cast<const uint2 *>(resid + row * ld + vcol0 + lc);
        float4 o;
        o.x = v.x + __uint_as_float(r.x << 16);
        o.y = v.y + __uint_as_float(r.x & 0xFFFF0000u);
        o.z = v.z + __uint_as_float(r.y << 16);
        o.w = v.w + __uint_as_float(r.y & 0xFFFF0000u);
        *reinterpret_cast<float4 *>(out + row * ld + vcol0 + lc) = o;
    }
};

// out = bf16(x2 + acc), x2 in fp32
struct EpiResidOut {
    const float *x2; bf16_t *out; int64_t ld;
    template <int WN> __device__ __forceinline__ void apply(int64_t row, int vcol0, int lc, const float *lrow) const
    {
        const float4 v = *reinterpret_cast<const float4 *>(lrow + lc);
        const float4 r = *reinterpret_cast<const float4 *>(x2 + row * ld + vcol0 + lc);
        uint2 o;
        o.x = pack_bf16x2(v.x + r.x, v.y + r.y);
        o.y = pack_bf16x2(v.z + r.z, v.w + r.w);
        *reinterpret_cast<uint2 *>(out + row * ld + vcol0 + lc) = o;
    }
};

// a = bf16(silu(gate) * up); the wave tile's first WN/2 columns are gate, the rest the matching up
struct EpiSiluMul {
    bf16_t *a; int64_t ld;   // [M][d_ff]
    template <int WN> __device__ __forceinline__ void apply(int64_t row, int vcol0, int lc, const float *lrow) const
    {
        if (lc >= WN / 2) return;
        const float4 g = *reinterpret_cast<const float4 *>(lrow + lc);
        const float4 u = *reinterpret_cast<const float4 *>(lrow + WN / 2 + lc);
        // g * sigmoid(g) * u with the hardware exp2 / reciprocal (about 1 ulp each, far below the
        // bf16 rounding that follows)
        const float a0 = g.x * __frcp_rn(1.0f + __expf(-g.x)) * u.x, a1 = g.y * __frcp_rn(1.0f + __expf(-g.y)) * u.y;
        const float a2 = g.z * __frcp_rn(1.0f + __expf(-g.z)) * u.z, a3 = g.w * __frcp_rn(1.0f + __expf(-g.w)) * u.w;
        uint2 o;
        o.x = pack_bf16x2(a0, a1);
        o.y = pack_bf16x2(a2, a3);
        *reinterpret_cast<uint2 *>(a + row * ld + (vcol0 / WN) * (WN / 2) + lc) = o;
    }
};

// rotary embedding on q and k heads (pairs (c, c + dh/2)), q -> [M][nq], k/v -> caches
struct EpiQkvRope {
    bf16_t *q, *kc, *vc;
    const float2 *rope; const int32_t *pos0;
    int Tn, L_max, Hq, Hkv, dh; int *flags;
    template <int WN> __device__ __forceinline__ void apply(int64_t row, int vcol0, int lc, const float *lrow) const
    {
        const int s = (int)(row / Tn), i = (int)(row - (int64_t)s * Tn);
        const int p0 = pos0 ? pos0[s] : 0;
        if (p0 < 0 || p0 + Tn > L_max) { if (lc == 0 && vcol0 == 0 && i == 0) atomicOr(flags, FLAG_CACHE_OVERFLOW); return; }
        const int pos = p0 + i, half = dh >> 1;
        const int v = vcol0 + lc;                       // virtual column of the first of 4 values
        const int nq = Hq * dh, nkv = Hkv * dh;
        const float4 x = *reinterpret_cast<const float4 *>(lrow + lc);
        float o[4] = {x.x, x.y, x.z, x.w};
        if (v < nq + nkv) {                             // q or k: rotate
            const int c = v % dh;                       // position inside the head (4 values stay in one half)
            const bool lo = c < half;
            const float4 y = *reinterpret_cast<const float4 *>(lrow + lc + (lo ? half : -half));
            const float yy[4] = {y.x, y.y, y.z, y.w};
            const float2 *cs = rope + (int64_t)pos * half + (lo ? c : c - half);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float2 t = cs[e];
                o[e] = lo ? (o[e] * t.x - yy[e] * t.y) : (o[e] * t.x + yy[e] * t.y);
            }
        }
        uint2 pk;
        pk.x = pack_bf16x2(o[0], o[1]);
        pk.y = pack_bf16x2(o[2], o[3]);
        bf16_t *dst;
        if (v < nq) dst = q + row * (int64_t)nq + v;
        else if (v < nq + nkv) { const int w = v - nq; dst = kc + (((int64_t)s * Hkv + w / dh) * L_max + pos) * dh + w % dh; }
        else { const int w = v - nq - nkv; dst = vc + (((int64_t)s * Hkv + w / dh) * L_max + pos) * dh + w % dh; }
        *reinterpret_cast<uint2 *>(dst) = pk;
    }
};

// ------------------------------------------------------------------------------------------------
// the kernel
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, class Epi>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64) __attribute__((amdgpu_waves_per_eu(1, 1)))
k_gemm_mfma(const bf16_t *__restrict__ A, int64_t lda, BMap bmap, int64_t M, int Nv, int K, int tiles_m, int tiles_n,
            Epi epi)
{
    constexpr int NWM = BM / WM, NWN = BN / WN, NT = NWM * NWN * 64;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWS_PER_PASS = NT / 8;                 // 8 threads (16-byte chunks) per 128-byte row
    constexpr int A_PASSES = BM / ROWS_PER_PASS, B_PASSES = BN / ROWS_PER_PASS;
    constexpr int STAGE_BYTES = (BM + BN) * 128;
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile / thread mismatch");
    extern __shared__ __align__(16) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / NWN, wn = wave - wm * NWN;

    // ---- XCD-aware tile mapping: workgroup b runs on XCD b % 8; XCD x owns a contiguous band ----
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + 7) / 8;
    const int lin = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (lin >= n_tiles) return;
    const int group_sz = GROUP_M * tiles_n;
    const int grp = lin / group_sz, in_grp = lin - grp * group_sz;
    const int rows_here = (tiles_m - grp * GROUP_M) < GROUP_M ? (tiles_m - grp * GROUP_M) : GROUP_M;
    const int tm = grp * GROUP_M + in_grp % rows_here, tn = in_grp / rows_here;
    const int64_t m0 = (int64_t)tm * BM;
    const int n0 = tn * BN;

    // ---- per-thread global sources and LDS destinations of the staged K slices ----
    const int chunk = tid & 7, r_in_pass = tid >> 3;
    const bf16_t *a_src[A_PASSES];
    const bf16_t *b_src[B_PASSES];
    int a_dst[A_PASSES], b_dst[B_PASSES];
#pragma unroll
    for (int p = 0; p < A_PASSES; ++p) {
        const int rl = p * ROWS_PER_PASS + r_in_pass;
        int64_t gr = m0 + rl;
        if (gr >= M) gr = M - 1;                            // ragged last tile: re-read the last row, never stored
        a_src[p] = A + gr * lda + chunk * 8;
        a_dst[p] = rl * 128 + ((chunk ^ SOL_SWZ(rl)) << 4);
    }
#pragma unroll
    for (int p = 0; p < B_PASSES; ++p) {
        const int rl = p * ROWS_PER_PASS + r_in_pass;
        b_src[p] = bmap.row(n0 + rl) + chunk * 8;
        b_dst[p] = BM * 128 + rl * 128 + ((chunk ^ SOL_SWZ(rl)) << 4);
    }

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Software pipeline, three K slices deep: LDS holds slices kt and kt+1, one register set holds
    // slice kt+2 (loaded one full iteration ago, so HBM latency is covered by two iterations of
    // MFMAs), the other register set is being loaded with slice kt+3. One barrier per iteration:
    // after it, slice kt's LDS stage is free and takes slice kt+2.
    // (macros, not lambdas: register arrays captured by reference would be demoted to scratch)
    u32x4_t ra0[A_PASSES], rb0[B_PASSES], ra1[A_PASSES], rb1[B_PASSES];
    const int KT = K / BK;
#define SOL_G_LOAD(RA, RB, KT_)                                                                            \
    {                                                                                                      \
        const int koff_ = ((KT_) < KT ? (KT_) : KT - 1) * BK; /* past the end: re-read the last slice */   \
        _Pragma("unroll") for (int p = 0; p < A_PASSES; ++p)                                               \
            RA[p] = *reinterpret_cast<const u32x4_t *>(a_src[p] + koff_);                                  \
        _Pragma("unroll") for (int p = 0; p < B_PASSES; ++p)                                               \
            RB[p] = *reinterpret_cast<const u32x4_t *>(b_src[p] + koff_);                                  \
    }
#define SOL_L_STORE(RA, RB, STAGE_)                                                                        \
    {                                                                                                      \
        _Pragma("unroll") for (int p = 0; p < A_PASSES; ++p)                                               \
            *reinterpret_cast<u32x4_t *>((STAGE_) + a_dst[p]) = RA[p];                                     \
        _Pragma("unroll") for (int p = 0; p < B_PASSES; ++p)                                               \
            *reinterpret_cast<u32x4_t *>((STAGE_) + b_dst[p]) = RB[p];                                     \
    }
    // fragment read offsets (row = lane % 32 of the MFMA tile, k chunk = 2*kk + lane/32)
    const int frow = lane & 31, fk = lane >> 5, fsw = SOL_SWZ(frow);
    const int a_frag0 = (wm * WM + frow) * 128;
    const int b_frag0 = BM * 128 + (wn * WN + frow) * 128;
#define SOL_COMPUTE(CUR_)                                                                                  \
    _Pragma("unroll") for (int kk = 0; kk < BK / 16; ++kk)                                                 \
    {                                                                                                      \
        const int coff = (((kk * 2 + fk) ^ fsw) << 4);                                                     \
        bf16x8_t af[TM], bfr[TN];                                                                          \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) af[i] = __builtin_bit_cast(                         \
            bf16x8_t, *reinterpret_cast<const u32x4_t *>((CUR_) + a_frag0 + i * 32 * 128 + coff));         \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) bfr[j] = __builtin_bit_cast(                        \
            bf16x8_t, *reinterpret_cast<const u32x4_t *>((CUR_) + b_frag0 + j * 32 * 128 + coff));         \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)      \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);        \
    }

    SOL_G_LOAD(ra0, rb0, 0);
    SOL_G_LOAD(ra1, rb1, 1);
    SOL_L_STORE(ra0, rb0, lds);
    SOL_L_STORE(ra1, rb1, lds + STAGE_BYTES);
    SOL_G_LOAD(ra0, rb0, 2);
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {                    // KT is even (K is a multiple of 128)
        // even step: stage 0 holds slice kt; set 0 holds slice kt+2; load slice kt+3 into set 1
        SOL_G_LOAD(ra1, rb1, kt + 3);
        SOL_COMPUTE(lds);
        __syncthreads();
        SOL_L_STORE(ra0, rb0, lds);
        // odd step: stage 1 holds slice kt+1; set 1 holds slice kt+3; load slice kt+4 into set 0
        SOL_G_LOAD(ra0, rb0, kt + 4);
        SOL_COMPUTE(lds + STAGE_BYTES);
        __syncthreads();
        SOL_L_STORE(ra1, rb1, lds + STAGE_BYTES);
    }
    __syncthreads();
#undef SOL_G_LOAD
#undef SOL_L_STORE
#undef SOL_COMPUTE

    // ---- epilogue: 32 rows x WN columns per wave at a time through LDS ----
    constexpr int LROW = WN + 4;                           // padded fp32 row
    float *stage = reinterpret_cast<float *>(lds) + (size_t)wave * 32 * LROW;
    constexpr int LPR = WN / 4;                            // lanes per row when each lane takes 4 columns
    constexpr int RPP = 64 / LPR;                          // rows per pass
    const int e_row = lane / LPR, e_col = (lane - e_row * LPR) * 4;
    const int vcol0 = n0 + wn * WN;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                stage[rr * LROW + j * 32 + (lane & 31)] = acc[i][j][r];
            }
        __syncthreads();
#pragma unroll
        for (int ps = 0; ps < 32 / RPP; ++ps) {
            const int rr = ps * RPP + e_row;
            const int64_t grow = m0 + wm * WM + i * 32 + rr;
            if (grow < M) epi.template apply<WN>(grow, vcol0, e_col, stage + rr * LROW);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, class Epi>
static bool launch_mfma(const bf16_t *A, int64_t lda, const BMap &bmap, int64_t M, int Nv, int K, const Epi &epi,
                        hipStream_t st)
{
    if (M <= 0) return true;
    if (Nv % BN || K % (2 * BK) || K < 2 * BK) return false;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr size_t lds_main = 2 * (size_t)(BM + BN) * 128;
    constexpr size_t lds_epi = (size_t)(NT / 64) * 32 * (WN + 4) * 4;
    constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
    auto kern = k_gemm_mfma<BM, BN, WM, WN, Epi>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return false;
        attr_done = true;
    }
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = Nv / BN;
    const int n_tiles = tiles_m * tiles_n;
    const int grid = ((n_tiles + 7) / 8) * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st, A, lda, bmap, M, Nv, K, tiles_m, tiles_n, epi);
    return true;
}

// Tile configurations of the fused layer GEMMs: 256 x 256 workgroup tiles, 8 waves (two per SIMD, so
// one wave's LDS / barrier waits hide under the other's MFMAs). Wave tile 128 x 64 measured fastest;
// the q/k/v epilogue needs a whole head (up to 128 columns) inside one wave tile, hence 64 x 128.
#define SOL_TILE 256, 256, 128, 64
#define SOL_TILE_QKV 256, 256, 64, 128

bool launch_gemm_qkv_rope(const void *h, const void *wq, const void *wk, const void *wv, void *q, void *kc, void *vc,
                          const float2 *rope, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh,
                          int d, int *flags, hipStream_t st)
{
    const int nq = Hq * dh, nkv = Hkv * dh;
    if (dh > 128 || 128 % dh || nq % 256 || nkv % 256) return false;      // heads must not straddle wave tiles
    BMap bm{};
    bm.base[0] = (const bf16_t *)wq; bm.base[1] = (const bf16_t *)wk; bm.base[2] = (const bf16_t *)wv;
    bm.seg_end[0] = nq; bm.seg_end[1] = nq + nkv; bm.seg_end[2] = nq + 2 * nkv;
    bm.mode = 0; bm.half = 0; bm.ld = d;
    EpiQkvRope epi{(bf16_t *)q, (bf16_t *)kc, (bf16_t *)vc, rope, pos0, T, L_max, Hq, Hkv, dh, flags};
    return launch_mfma<SOL_TILE_QKV>((const bf16_t *)h, d, bm, (int64_t)n_seq * T, nq + 2 * nkv, d, epi, st);
}

bool launch_gemm_resid_f32(const void *a, const void *w, const void *resid, float *out, int64_t M, int N, int K,
                           hipStream_t st)
{
    BMap bm{};
    bm.base[0] = (const bf16_t *)w; bm.seg_end[0] = bm.seg_end[1] = bm.seg_end[2] = N; bm.mode = 0; bm.ld = K;
    EpiResidF32 epi{(const bf16_t *)resid, out, N};
    return launch_mfma<SOL_TILE>((const bf16_t *)a, K, bm, M, N, K, epi, st);
}

bool launch_gemm_gateup_silu(const void *h, const void *wg, const void *wu, void *a, int64_t M, int dff, int d,
                             hipStream_t st)
{
    if (dff % 128) return false;
    BMap bm{};
    bm.base[0] = (const bf16_t *)wg; bm.base[1] = (const bf16_t *)wu; bm.mode = 1; bm.half = 32; bm.ld = d;   // half = WN / 2
    EpiSiluMul epi{(bf16_t *)a, dff};
    return launch_mfma<SOL_TILE>((const bf16_t *)h, d, bm, M, 2 * dff, d, epi, st);
}

bool launch_gemm_resid_out(const void *a, const void *w, const float *x2, void *out, int64_t M, int N, int K,
                           hipStream_t st)
{
    BMap bm{};
    bm.base[0] = (const bf16_t *)w; bm.seg_end[0] = bm.seg_end[1] = bm.seg_end[2] = N; bm.mode = 0; bm.ld = K;
    EpiResidOut epi{x2, (bf16_t *)out, N};
    return launch_mfma<SOL_TILE>((const bf16_t *)a, K, bm, M, N, K, epi, st);
}

bool launch_gemm_f32(const void *a, const void *w, float *C, int64_t ldc, int64_t M, int N, int K, hipStream_t st)
{
    BMap bm{};
    bm.base[0] = (const bf16_t *)w; bm.seg_end[0] = bm.seg_end[1] = bm.seg_end[2] = N; bm.mode = 0; bm.ld = K;
    EpiStoreF32 epi{C, ldc};
    return launch_mfma<SOL_TILE>((const bf16_t *)a, K, bm, M, N, K, epi, st);
}


// =================================================================================================
// Skinny GEMM for the decode step: out[M][Nv] = x[M][K] * Wv[Nv][K]^T with M <= 64 tokens.
// HBM-bound: every weight byte is read exactly once, by exactly one wave. A wave owns 32 weight
// rows (they are the MFMA's "A" rows) and streams them straight from global memory in 128-byte
// pieces (lane (r, h) takes the 64 contiguous bytes of half h of row r, so every fetched line is
// fully used); the activations are the "B" operand, staged per workgroup in LDS in K chunks of 512.
// Since the same k-to-lane assignment is used for A and B the MFMA sum is exact. The K range may be
// split over gridDim.y workgroups; partial sums go to fp32 partial[split][M][Nv] and are folded by
// the consumer kernel in split order (fixed split count per shape => deterministic).
// =================================================================================================
constexpr int SK_KC = 512;                 // K chunk staged in LDS
constexpr int SK_XROW = SK_KC * 2 + 16;    // padded LDS row of activations (bytes): rows shift 4 banks

template <int MT>                           // MT tiles of 32 tokens (1: M <= 32, 2: M <= 64)
__global__ void __launch_bounds__(256)
k_gemm_skinny(const bf16_t *__restrict__ x, int64_t ldx, BMap bmap, int M, int Nv, int K, int k_per_split,
              float *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char xs[];      // [MT*32][SK_XROW]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n0 = (blockIdx.x * 4 + wave) * 32;
    const int split = blockIdx.y;
    const int k_begin = split * k_per_split;
    const int k_end = (k_begin + k_per_split < K) ? k_begin + k_per_split : K;
    const int r = lane & 31, h = lane >> 5;
    const bool live = n0 < Nv;                                // whole wave
    int nrow = n0 + r;
    if (nrow >= Nv) nrow = Nv - 1;
    const bf16_t *wrow = bmap.row(nrow) + h * 32;             // this lane's 64-byte half of each 128-byte piece
    floatx16_t acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    for (int kc = k_begin; kc < k_end; kc += SK_KC) {
        const int kw = (k_end - kc < SK_KC) ? (k_end - kc) : SK_KC;   // multiple of 64
        __syncthreads();                                              // previous chunk fully consumed
        // stage x[0..MT*32)[kc .. kc+kw) into LDS, 16 bytes per thread per step (rows >= M: zeros)
        const int pieces = kw / 8;
        for (int idx = tid; idx < MT * 32 * pieces; idx += 256) {
            const int m = idx / pieces, p = idx - m * pieces;
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (m < M) v = *reinterpret_cast<const u32x4_t *>(x + (int64_t)m * ldx + kc + p * 8);
            *reinterpret_cast<u32x4_t *>(xs + m * SK_XROW + p * 16) = v;
        }
        __syncthreads();
        if (live) {
            constexpr int UK = 4;                                       // 64-wide K blocks in flight per wave
            for (int kb = 0; kb < kw; kb += 64 * UK) {
                u32x4_t wa[UK][4];
#pragma unroll
                for (int u = 0; u < UK; ++u) {
                    const int ko = (kb + u * 64 < kw) ? kb + u * 64 : kb;   // ragged tail: re-read, not used
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        wa[u][j] = *reinterpret_cast<const u32x4_t *>(wrow + kc + ko + j * 8);
                }
#pragma unroll
                for (int u = 0; u < UK; ++u) {
                    if (kb + u * 64 < kw) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const bf16x8_t af = __builtin_bit_cast(bf16x8_t, wa[u][j]);
#pragma unroll
                            for (int t = 0; t < MT; ++t) {
                                const unsigned char *xp = xs + (t * 32 + r) * SK_XROW + (kb + u * 64 + h * 32 + j * 8) * 2;
                                const bf16x8_t bfr = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>(xp));
                                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[t], 0, 0, 0);
                            }
                        }
                    }
                }
            }
        }
    }
    if (!live) return;
    // acc[t][i]: weight row n0 + 8*(i/4) + 4*h + (i%4), token t*32 + r
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = t * 32 + r;
        if (m < M) {
            float *dst = partial + ((int64_t)split * M + m) * Nv + n0 + 4 * h;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (n0 + 8 * g + 4 * h + 3 < Nv) {
                    const float4 v = make_float4(acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]);
                    *reinterpret_cast<float4 *>(dst + 8 * g) = v;
                }
            }
        }
    }
}

// Number of K splits for the skinny kernel: enough waves to cover the chip, partial-sum traffic kept
// below about a quarter of the weight traffic.
int skinny_splits(int M, int Nv, int K)
{
    const int tiles = (Nv + 31) / 32;
    int want = (1024 + tiles - 1) / tiles;
    int cap = K / (8 * (M > 0 ? M : 1));
    if (cap < 1) cap = 1;
    int s = want < cap ? want : cap;
    if (s < 1) s = 1;
    while (s > 1 && (K / 64) % s != 0) --s;                 // every split gets a whole number of 64-wide blocks
    return s;
}

static bool launch_skinny(const bf16_t *x, int64_t ldx, const BMap &bm, int M, int Nv, int K, float *partial, int nsplit,
                          hipStream_t st)
{
    if (M <= 0) return true;
    if (M > 64 || Nv % 4 || K % 64) return false;
    const int k_per_split = K / nsplit;
    if (k_per_split % 64) return false;
    const dim3 grid((Nv + 127) / 128, nsplit);
    static bool attr_done = false;
    const size_t lds = (size_t)64 * SK_XROW;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(k_gemm_skinny<2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess) return false;
        attr_done = true;
    }
    if (M <= 32)
        hipLaunchKernelGGL((k_gemm_skinny<1>), grid, dim3(256), (size_t)32 * SK_XROW, st, x, ldx, bm, M, Nv, K, k_per_split, partial);
    else
        hipLaunchKernelGGL((k_gemm_skinny<2>), grid, dim3(256), lds, st, x, ldx, bm, M, Nv, K, k_per_split, partial);
    return true;
}

// partial[nsplit][M][N] = x * [w0; w1; w2]^T  (rows of up to three stacked weight matrices)
bool launch_gemm_skinny(const void *x, int64_t ldx, const void *w0, int n0, const void *w1, int n1, const void *w2,
                        int n2, int M, int K, float *partial, int nsplit, hipStream_t st)
{
    BMap bm{};
    bm.base[0] = (const bf16_t *)w0; bm.base[1] = (const bf16_t *)w1; bm.base[2] = (const bf16_t *)w2;
    bm.seg_end[0] = n0; bm.seg_end[1] = n0 + n1; bm.seg_end[2] = n0 + n1 + n2;
    bm.mode = 0; bm.half = 0; bm.ld = K;
    return launch_skinny((const bf16_t *)x, ldx, bm, M, n0 + n1 + n2, K, partial, nsplit, st);
}

}  // namespace sol
