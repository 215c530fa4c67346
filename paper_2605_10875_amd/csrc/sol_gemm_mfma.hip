// bf16 MFMA GEMM for gfx950 with fused epilogues:  C[M][Nv] = A[M][K] * Wv[Nv][K]^T, fp32 accumulate.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants for A and B
// alike (each lane supplies 8 consecutive k of one row / one column). "Nv" is a virtual column
// space: a column maps to a row of one of up to three weight matrices (q|k|v stacked, or gate and
// up interleaved in 64-column halves so that SiLU(gate)*up is formed inside one wave tile).
//
// Tiling: workgroup tile BM x BN, K step 64; waves in a (BM/WM) x (BN/WN) grid, each wave owning
// WM x WN = (WM/32) x (WN/32) MFMA tiles of 32x32 in accumulator registers. A and B K-slices go
// from global memory straight into LDS (LDS-direct loads; two stages, XOR-swizzled 16-byte chunks
// so that the 128-bit fragment reads are bank-conflict free): the slice after next is requested
// while the MFMAs of the current slice's last k-group issue. Workgroups are mapped to tiles
// XCD-aware: each of the 8 XCDs walks its own contiguous band of the tile grid in groups of
// GROUP_M tile rows, so the tiles resident on an XCD at any time share A rows and B columns in
// that XCD's L2; with several tiles per CU one persistent workgroup per CU walks its share of the
// band and the load pipeline runs across tile boundaries.
//
// Epilogue: functors consume the accumulators in their MFMA register layout, two rows at a time
// (rotary + cache write, residual add, SiLU(gate)*up, plain store); bf16 outputs are paired up across
// neighbouring lanes into 4-byte stores.
#include "sol_internal.h"

namespace sol {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // native 16-byte vector (stays in registers)
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int BK = 64;               // K step (bf16 elements); one LDS row = 128 bytes = 8 chunks of 16 B
constexpr int GROUP_M = 4;           // tile rows walked together by an XCD: its 32 CUs then hold 4 x 8 tiles (measured on the
                                     // 16 x 2048-token stack: 2, 4 within 1 %; 8: 2 - 4 % slower; 16: 4 - 8 % slower)
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
// Epilogues work on the accumulator layout of v_mfma_f32_32x32x16 directly: for one (row-tile, register
// pair) a lane holds, for two consecutive rows, the TN values at columns  c + 32*j  (c = lane % 32) of
// the wave tile. An epilogue has two halves so that the kernel can issue every global read of a 32-row
// tile before the first store (the compiler must assume that stores alias later loads):
//   preload(row0, row1, ok0, ok1, vcol0, c, aux)      reads what the row pair needs from memory into aux
//                                                     (row0 / row1 clamped to existing rows: no branches)
//   rows2(row0, ok0, ok1, vcol0, c, v0, v1, aux)      combines and stores
// row0 / row0 + 1 are the global rows, ok0 / ok1 say whether they exist (every lane still runs the code:
// bf16 outputs exchange values between neighbouring lanes), vcol0 is the wave tile's first virtual column.
// ------------------------------------------------------------------------------------------------

// Two rows of bf16 outputs at column c: neighbouring lanes pair up so that every lane stores one 4-byte
// pair: even lanes (row0, columns c, c+1), odd lanes (row1, columns c-1, c).
__device__ __forceinline__ void store_bf16_rows2(bf16_t *p0, bf16_t *p1, bool ok0, bool ok1, int c, float x0, float x1)
{
    const float t0 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x0), 0xB1, 0xF, 0xF, false));
    const float t1 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x1), 0xB1, 0xF, 0xF, false));
    const bool even = (c & 1) == 0;
    const uint32_t pk = even ? pack_bf16x2(x0, t0) : pack_bf16x2(t1, x1);
    bf16_t *dst = even ? p0 + c : p1 + (c - 1);
    if (even ? ok0 : ok1) *reinterpret_cast<uint32_t *>(dst) = pk;
}

struct NoAux {};

struct EpiStoreF32 {
    static constexpr bool persistent_walk = true;
    float *C; int64_t ldc;
    template <int TN> using Aux = NoAux;
    template <int TN> __device__ __forceinline__ void preload0(int64_t, int64_t, NoAux &) const {}
    template <int TN> __device__ __forceinline__ void preload(int64_t, int64_t, bool, bool, int, int, NoAux &) const {}
    template <int TN>
    __device__ __forceinline__ void rows2(int64_t row0, bool ok0, bool ok1, int vcol0, int c, const float (&v0)[TN],
                                          const float (&v1)[TN], const NoAux &) const
    {
        float *p0 = C + row0 * ldc + vcol0 + c, *p1 = p0 + ldc;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (ok0) p0[32 * j] = v0[j];
            if (ok1) p1[32 * j] = v1[j];
        }
    }
};

template <int TN> struct AuxRows { float a0[TN], a1[TN]; };

// x2 = resid + acc  (fp32 out), resid in bf16
struct EpiResidF32 {
    static constexpr bool persistent_walk = false;   // measured: 0.30 -> 0.42 ms for the C2 o-projection under the persistent walk
    const bf16_t *resid; float *out; int64_t ld;
    template <int TN> using Aux = AuxRows<TN>;
    template <int TN> __device__ __forceinline__ void preload0(int64_t, int64_t, AuxRows<TN> &) const {}
    template <int TN>
    __device__ __forceinline__ void preload(int64_t row0, int64_t row1, bool, bool, int vcol0, int c, AuxRows<TN> &x) const
    {
        const int64_t o0 = row0 * ld + vcol0 + c, o1 = row1 * ld + vcol0 + c;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            x.a0[j] = bf16_to_f32(resid[o0 + 32 * j]);
            x.a1[j] = bf16_to_f32(resid[o1 + 32 * j]);
        }
    }
    template <int TN>
    __device__ __forceinline__ void rows2(int64_t row0, bool ok0, bool ok1, int vcol0, int c, const float (&v0)[TN],
                                          const float (&v1)[TN], const AuxRows<TN> &x) const
    {
        const int64_t o0 = row0 * ld + vcol0 + c, o1 = o0 + ld;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (ok0) out[o0 + 32 * j] = v0[j] + x.a0[j];
            if (ok1) out[o1 + 32 * j] = v1[j] + x.a1[j];
        }
    }
};

// out = bf16(x2 + acc), x2 in fp32
struct EpiResidOut {
    static constexpr bool persistent_walk = true;
    const float *x2; bf16_t *out; int64_t ld;
    template <int TN> using Aux = AuxRows<TN>;
    template <int TN> __device__ __forceinline__ void preload0(int64_t, int64_t, AuxRows<TN> &) const {}
    template <int TN>
    __device__ __forceinline__ void preload(int64_t row0, int64_t row1, bool, bool, int vcol0, int c, AuxRows<TN> &x) const
    {
        const int64_t o0 = row0 * ld + vcol0 + c, o1 = row1 * ld + vcol0 + c;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            x.a0[j] = x2[o0 + 32 * j];
            x.a1[j] = x2[o1 + 32 * j];
        }
    }
    template <int TN>
    __device__ __forceinline__ void rows2(int64_t row0, bool ok0, bool ok1, int vcol0, int c, const float (&v0)[TN],
                                          const float (&v1)[TN], const AuxRows<TN> &x) const
    {
        const int64_t o0 = row0 * ld + vcol0, o1 = o0 + ld;
#pragma unroll
        for (int j = 0; j < TN; ++j)
            store_bf16_rows2(out + o0 + 32 * j, out + o1 + 32 * j, ok0, ok1, c, v0[j] + x.a0[j], v1[j] + x.a1[j]);
    }
};

// a = bf16(silu(gate) * up); the wave tile's first WN/2 columns are gate, the rest the matching up
struct EpiSiluMul {
    static constexpr bool persistent_walk = true;
    bf16_t *a; int64_t ld;   // [M][d_ff]
    template <int TN> using Aux = NoAux;
    template <int TN> __device__ __forceinline__ void preload0(int64_t, int64_t, NoAux &) const {}
    template <int TN> __device__ __forceinline__ void preload(int64_t, int64_t, bool, bool, int, int, NoAux &) const {}
    static __device__ __forceinline__ float silu_mul(float g, float u)
    {
        // g * sigmoid(g) * u with the hardware exp2 / reciprocal instructions (about 1 ulp each, far below the
        // bf16 rounding that follows). v_rcp_f32 itself: a correctly rounded reciprocal is an eleven-instruction
        // division sequence, a third of this epilogue's vector instructions.
        return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
    }
    template <int TN>
    __device__ __forceinline__ void rows2(int64_t row0, bool ok0, bool ok1, int vcol0, int c, const float (&v0)[TN],
                                          const float (&v1)[TN], const NoAux &) const
    {
        constexpr int WN = TN * 32;
        bf16_t *p0 = a + row0 * ld + (vcol0 / WN) * (WN / 2), *p1 = p0 + ld;
#pragma unroll
        for (int j = 0; j < TN / 2; ++j)
            store_bf16_rows2(p0 + 32 * j, p1 + 32 * j, ok0, ok1, c, silu_mul(v0[j], v0[j + TN / 2]),
                             silu_mul(v1[j], v1[j + TN / 2]));
    }
};

// rotary embedding on q and k heads (pairs (c, c + dh/2)), q -> [M][nq], k/v -> caches.
// row_sp[row] = (sequence, absolute position) of the row, position -1 if its sequence does not fit the
// cache (written by k_row_positions before the GEMM).
template <int TN> struct AuxRope { float2 t0[TN], t1[TN]; int2 sp0, sp1; };

template <int DHT>                                      // head size: 64 or 128
struct EpiQkvRope {
    static constexpr bool persistent_walk = true;
    bf16_t *q, *kc, *vc;
    const float2 *rope; const int2 *row_sp;
    int L_max, Hq, Hkv;
    const int *only_if_flagged;                          // not null: the kernel runs only if a sequence has been flagged (see EpiQkvRopeTile)
    __device__ __forceinline__ bool run() const { return !only_if_flagged || (*only_if_flagged & FLAG_CACHE_OVERFLOW) != 0; }
    template <int TN> using Aux = AuxRope<TN>;
    template <int TN> __device__ __forceinline__ void preload0(int64_t row0, int64_t row1, AuxRope<TN> &x) const
    {
        x.sp0 = row_sp[row0];
        x.sp1 = row_sp[row1];
    }
    template <int TN>
    __device__ __forceinline__ void preload(int64_t, int64_t, bool, bool, int vcol0, int c, AuxRope<TN> &x) const
    {
        constexpr int dh = DHT, half = DHT / 2;
        if (vcol0 < (Hq + Hkv) * dh) {                   // q or k: cos / sin of the two positions
            const int pa = x.sp0.y < 0 ? 0 : x.sp0.y, pb = x.sp1.y < 0 ? 0 : x.sp1.y;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int cj = (32 * j + c) & (dh - 1);  // position inside the head
                const int ci = cj < half ? cj : cj - half;
                x.t0[j] = rope[(int64_t)pa * half + ci];
                x.t1[j] = rope[(int64_t)pb * half + ci];
            }
        }
    }
    template <int TN>
    __device__ __forceinline__ void rows2(int64_t row0, bool ok0, bool ok1, int vcol0, int c, const float (&v0)[TN],
                                          const float (&v1)[TN], const AuxRope<TN> &x) const
    {
        constexpr int dh = DHT, half = DHT / 2;
        const int nq = Hq * dh, nkv = Hkv * dh;
        ok0 = ok0 && x.sp0.y >= 0;
        ok1 = ok1 && x.sp1.y >= 0;
        // the wave tile (128 columns, heads of 64 or 128) lies inside one of q / k / v
        const int seg = vcol0 < nq ? 0 : (vcol0 < nq + nkv ? 1 : 2);
        const int w0 = vcol0 - (seg == 0 ? 0 : (seg == 1 ? nq : nq + nkv));   // column inside the segment
        bf16_t *d0, *d1;                                 // destination of the wave tile's first column, rows 0 / 1
        if (seg == 0) { d0 = q + row0 * (int64_t)nq + w0; d1 = d0 + nq; }
        else {
            bf16_t *cache = seg == 1 ? kc : vc;
            const int hd = w0 / dh, wi = w0 - hd * dh;
            d0 = cache + (((int64_t)x.sp0.x * Hkv + hd) * L_max + x.sp0.y) * dh + wi;
            d1 = cache + (((int64_t)x.sp1.x * Hkv + hd) * L_max + x.sp1.y) * dh + wi;
        }
        const int hstep = (seg == 0 || dh >= TN * 32) ? 0 : (int)((int64_t)L_max * dh) - dh;   // next head inside the tile (dh = 64)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            float o0 = v0[j], o1 = v1[j];
            if (seg < 2) {                               // q or k: rotate
                const bool lo = ((32 * j) & (dh - 1)) < half;                 // the same for every c < 32
                const int jp = lo ? j + half / 32 : j - half / 32;            // tile of the partner column
                const float y0 = v0[jp], y1 = v1[jp];
                o0 = lo ? (o0 * x.t0[j].x - y0 * x.t0[j].y) : (o0 * x.t0[j].x + y0 * x.t0[j].y);
                o1 = lo ? (o1 * x.t1[j].x - y1 * x.t1[j].y) : (o1 * x.t1[j].x + y1 * x.t1[j].y);
            }
            const int hj = (32 * j) / dh;                // head inside the tile of column 32*j + c
            const int64_t off = (seg == 0) ? 32 * j : (int64_t)hj * hstep + 32 * j;
            store_bf16_rows2(d0 + off, d1 + off, ok0, ok1, c, o0, o1);
        }
    }
};

// The same epilogue for whole wave tiles whose 128 consecutive rows touch at most two sequences (Tn >= 128, M a
// multiple of the tile height). EpiQkvRope reads a row's (sequence, position) and then, at an address that depends on
// it, its cos / sin pairs: two exposed load latencies per block of 32 rows, about 16 us per tile under the GEMM's own
// traffic, as long as the MFMA part of a K = 2048 tile. Here the positions come from arithmetic on the tile's first
// row (two scalar loads of pos0 per tile), so every table load can be issued at once, and they run two groups of four
// rows ahead of the rotation and the stores. Values and destinations are those of EpiQkvRope.
template <int DHT>
struct EpiQkvRopeTile {
    static constexpr bool persistent_walk = false;       // inside the persistent walk, next to the held fragments, it spills
    static constexpr bool whole_tile = true;
    bf16_t *q, *kc, *vc;
    const float2 *rope; const int32_t *pos0;
    int Tn, L_max, Hq, Hkv, n_seq;                       // L_max: rows of a cache slab
    const int *flags;
    // flags not null: the kernel runs only while no sequence of the call has been flagged (k_row_positions, just before
    // it, flags those that do not fit their cache): then every store is unconditional. Otherwise the launcher's second
    // kernel, with EpiQkvRope and its per-row predicates, does the work (both versions in one kernel spill the
    // accumulators). Without per-sequence start positions the host has checked that T rows fit: flags is null.
    __device__ __forceinline__ bool run() const { return !flags || (*flags & FLAG_CACHE_OVERFLOW) == 0; }
    template <int TM, int TN>
    __device__ __forceinline__ void tile(const floatx16_t (&acc)[TM][TN], int64_t row_w, int vcol_w, int lane) const
    {
        // the wave tile's corner is the same in every lane; said so, what follows from it (segment, bases, positions)
        // stays in scalar registers and the segment tests become branches instead of selects per value
        const int vcol_u = __builtin_amdgcn_readfirstlane(vcol_w);
        const int64_t row_u = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(row_w >> 32)) << 32) |
                                        (uint32_t)__builtin_amdgcn_readfirstlane((int)row_w));
        // rows row_u + k, k < 128: sequence s0 up to its end, then s0 + 1
        const int s0 = (int)(row_u / Tn), t0 = (int)(row_u - (int64_t)s0 * Tn);
        const int pa = pos0 ? pos0[s0] : 0;
        const int pb = (pos0 && s0 + 1 < n_seq) ? pos0[s0 + 1] : 0;
        tile_rows<TM, TN>(acc, row_u, vcol_u, lane, s0, t0, pa, pb);
    }
    // Destinations are a uniform base per 32-column tile plus a 32-bit byte offset per lane. Of a pair of rows a lane
    // stores one (even columns the first, odd columns the second: two bf16 of that row, its own and its neighbour's),
    // so it needs the destination of that row only; the cos / sin pairs it needs for both.
    template <int TM, int TN>
    __device__ __forceinline__ void tile_rows(const floatx16_t (&acc)[TM][TN], int64_t row_w, int vcol_w, int lane, int s0,
                                              int t0, int pa, int pb) const
    {
        constexpr int dh = DHT, half = DHT / 2, ND = DHT / 64;   // ND: table columns a lane needs per row (c, c + 32, ..)
        static_assert(TN * 32 == 128 && TM * 32 == 128, "128 x 128 wave tiles");
        const int c = lane & 31, rg = lane >> 5;
        const bool odd = (c & 1) != 0;
        const int nq = Hq * dh, nkv = Hkv * dh;
        const int seg = vcol_w < nq ? 0 : (vcol_w < nq + nkv ? 1 : 2);        // the wave tile lies inside one of q / k / v
        const int w0 = vcol_w - (seg == 0 ? 0 : (seg == 1 ? nq : nq + nkv));  // column inside the segment
        const int hd = w0 / dh, wi = w0 - hd * dh;
        const int hstep = (seg == 0 || dh >= TN * 32) ? 0 : (int)((int64_t)L_max * dh) - dh;   // next head inside the tile (dh = 64)
        // row k of the tile lies (k < kx ? ca : cb) + k rows of rs bytes behind `base` (q: the tile's first row; caches:
        // the slab of (s0, head hd), that of s0 + 1 being Hkv * L_max rows further on)
        const int kx = Tn - t0;
        char *base;
        int ca, cb;
        uint32_t rs;
        if (seg == 0) { base = reinterpret_cast<char *>(q + row_w * (int64_t)nq + w0); ca = cb = 0; rs = (uint32_t)nq * 2u; }
        else {
            base = reinterpret_cast<char *>((seg == 1 ? kc : vc) + ((int64_t)s0 * Hkv + hd) * (int64_t)L_max * dh + wi);
            ca = pa + t0; cb = Hkv * L_max + pb - kx; rs = (uint32_t)dh * 2u;
        }
        char *bj[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) bj[j] = base + (32 * j + ((32 * j) / dh) * hstep) * 2;
        const uint32_t lane_col = (uint32_t)(c - (odd ? 1 : 0)) * 2u;
        const int ta = pa + t0, tb = pb - kx;                    // position of row k: (k < kx ? ta : tb) + k
        const char *const tbase = reinterpret_cast<const char *>(rope);
        constexpr int NCH = TM * 4;                              // groups of four rows (registers 4g .. 4g + 3 of block i)
        float2 cs[3][4][ND];
        auto load_group = [&](int n, float2 (&x)[4][ND]) {
            if (seg < 2) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = (n >> 2) * 32 + 8 * (n & 3) + 4 * rg + e;
                    const bool a = k < kx;
                    const int pos = (a ? ta : tb) + k;
                    const uint32_t to = ((uint32_t)pos * (uint32_t)half + (uint32_t)c) * 8u;
#pragma unroll
                    for (int dd = 0; dd < ND; ++dd) x[e][dd] = *reinterpret_cast<const float2 *>(tbase + to + dd * 256);
                }
            }
        };
        load_group(0, cs[0]);
        load_group(1, cs[1]);
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            if (n + 2 < NCH) load_group(n + 2, cs[(n + 2) % 3]);
            const int i = n >> 2, g4 = n & 3;
#pragma unroll
            for (int e = 0; e < 4; e += 2) {                     // rows in pairs
                const int ko = i * 32 + 8 * g4 + 4 * rg + e + (odd ? 1 : 0);   // the row of the pair this lane stores
                const bool a = ko < kx;
                const uint32_t roff = (uint32_t)((a ? ca : cb) + ko) * rs + lane_col;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int r = 4 * g4 + e;
                    float o0 = acc[i][j][r], o1 = acc[i][j][r + 1];
                    if (seg < 2) {                               // q or k: rotate
                        const int cj0 = (32 * j) & (dh - 1);     // the tile's first column inside its head
                        const bool lo = cj0 < half;
                        const int jp = lo ? j + half / 32 : j - half / 32;   // tile of the partner column
                        const int dd = (cj0 & (half - 1)) / 32;
                        const float y0 = acc[i][jp][r], y1 = acc[i][jp][r + 1];
                        const float2 a0 = cs[n % 3][e][dd], a1 = cs[n % 3][e + 1][dd];
                        o0 = lo ? (o0 * a0.x - y0 * a0.y) : (o0 * a0.x + y0 * a0.y);
                        o1 = lo ? (o1 * a1.x - y1 * a1.y) : (o1 * a1.x + y1 * a1.y);
                    }
                    // the neighbour's values of both rows (lanes c ^ 1); even columns store (own, neighbour's) of the
                    // first row, odd columns (neighbour's, own) of the second
                    const float n0 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, o0), 0xB1, 0xF, 0xF, false));
                    const float n1 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, o1), 0xB1, 0xF, 0xF, false));
                    const uint32_t pk = pack_bf16x2(odd ? n1 : o0, odd ? o1 : n0);
                    *reinterpret_cast<uint32_t *>(bj[j] + roff) = pk;
                }
                __builtin_amdgcn_sched_barrier(0);               // one pair at a time: hoisted accumulator reads would spill
            }
        }
    }
};

// row -> (sequence, absolute position), position -1 (and the overflow flag) if the sequence does not fit
__global__ void __launch_bounds__(256)
k_row_positions(const int32_t *__restrict__ pos0, int64_t M, int Tn, int L_max, int2 *__restrict__ row_sp, int *flags)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= M) return;
    const int s = (int)(row / Tn), i = (int)(row - (int64_t)s * Tn);
    const int p0 = pos0 ? pos0[s] : 0;
    const bool bad = p0 < 0 || p0 + Tn > L_max;
    if (bad && i == 0) atomicOr(flags, FLAG_CACHE_OVERFLOW);
    row_sp[row] = make_int2(s, bad ? -1 : p0 + i);
}

// LM head with the logits never written: per (token, tile of 128 vocabulary entries) the maximum and the sum of
// exp(logit - maximum); k_nll_finish_cols folds the tiles of a token into  logsumexp(logits) - logits[target]
// (Method, Eq. 1, negated), the target's logit coming from k_target_logit.
// target token of every row (teacher-forced rows (b, g, t) share the targets of input b when broadcast_g)
__global__ void __launch_bounds__(256)
k_row_targets(const int32_t *__restrict__ targets, int64_t M, int G, int Tn, int broadcast_g, int V, int32_t *__restrict__ row_tgt,
              int *__restrict__ flags)
{
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= M) return;
    const int64_t ti = broadcast_g ? (r / ((int64_t)G * Tn)) * Tn + (r % Tn) : r;
    int tg = targets[ti];
    if (tg < 0 || tg >= V) {                       // outside the vocabulary: clamped, and reported through the sticky flag
        atomicOr(flags, FLAG_BAD_TOKEN);
        tg = tg < 0 ? 0 : V - 1;
    }
    row_tgt[r] = tg;
}

// The product's rows are the vocabulary entries (A = the head's weights), its columns the tokens (B = the hidden
// states, padded with zero rows to a multiple of the tile). A lane of the
// accumulator layout then holds, for each of its TN tokens, 16 * TM logits of that token (the wave tile's 128 vocabulary
// rows are split between the two halves of the wave), so the maximum and the sum of exponentials per (token, tile) are
// sums over the lane's own registers plus ONE exchange with lane ^ 32 (with tokens as rows a lane holds one column
// and every row costs two five-step butterflies), and the big operand (525 MB of weights at the Llama vocabulary) is
// the one that each XCD streams once, while the hidden states, which the memory-side cache holds, are the ones read
// again. part: [V / 128][Mp] (token fastest: a half-wave stores 32 consecutive entries; Mp = padded token count).
// What a token gets does not depend on the other tokens of the call. The target's logit comes from k_target_logit,
// since a lane would have to search its registers for it.
__device__ __forceinline__ float swap_halves(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, v)));
}
struct EpiNllCols {
    static constexpr bool persistent_walk = true;
    static constexpr bool whole_tile = true;
    float2 *part;               // [V / 128][Mp]
    int64_t M;                  // Mp: tokens, padded to the tile
    template <int TM, int TN>
    __device__ __forceinline__ void tile(const floatx16_t (&acc)[TM][TN], int64_t vrow_w, int tcol_w, int lane) const
    {
        constexpr float LOG2E = 1.44269504088896341f;
        float2 *dst = part + (vrow_w / (TM * 32)) * M + tcol_w + (lane & 31);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            float m = acc[0][j][0];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) m = fmaxf(m, acc[i][j][r]);
            m = fmaxf(m, swap_halves(m, lane));
            const float ml = m * LOG2E;
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][r], LOG2E, -ml));
                    s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][r + 1], LOG2E, -ml));
                }
            float se = s0 + s1;
            se += swap_halves(se, lane);
            if (lane < 32) dst[32 * j] = make_float2(m, se);
        }
    }
};

// logit of each row's target: one wave per row, hf[r] . lm_head[target(r)] in fp32
__global__ void __launch_bounds__(256)
k_target_logit(const bf16_t *__restrict__ hf, const bf16_t *__restrict__ lm_head, const int32_t *__restrict__ row_tgt, int64_t M,
               int K, float *__restrict__ tgt_logit)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    const bf16_t *a = hf + r * K, *b = lm_head + (int64_t)row_tgt[r] * K;
    float acc = 0.f;
    for (int k = lane * 8; k < K; k += 512) {
        const uint4 x = *reinterpret_cast<const uint4 *>(a + k), y = *reinterpret_cast<const uint4 *>(b + k);
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = __builtin_fmaf(__uint_as_float(xs[e] << 16), __uint_as_float(ys[e] << 16), acc);
            acc = __builtin_fmaf(__uint_as_float(xs[e] & 0xFFFF0000u), __uint_as_float(ys[e] & 0xFFFF0000u), acc);
        }
    }
    acc = wave_sum_dpp(acc);
    if (lane == 0) tgt_logit[r] = acc;
}

// nll = max + log(sum_t s_t * exp(m_t - max)) - target logit over part [n_wt][Mp]. A workgroup takes 64 rows; wave q
// folds the tiles t = q, q + 16, ... of its 64 rows with a running maximum (a wave reads 64 consecutive entries of a
// tile), then the 16 partial results of a row are folded in wave order: the same sequence of operations for every
// row, whatever the batch.
constexpr int NLL_FIN_WAVES = 16;
__global__ void __launch_bounds__(NLL_FIN_WAVES * 64)
k_nll_finish_cols(const float2 *__restrict__ part, const float *__restrict__ tgt_logit, int n_wt, int64_t M, int64_t Mp,
                  float *__restrict__ nll)
{
    __shared__ float2 fold[NLL_FIN_WAVES][64];
    const int rl = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * 64 + rl;       // r < Mp: the grid covers ceil(M / 64) * 64 <= Mp rows
    float mx = -INFINITY, se = 0.f;
    for (int t = q; t < n_wt; t += NLL_FIN_WAVES) {
        const float2 v = part[(int64_t)t * Mp + r];
        const float m2 = fmaxf(mx, v.x);
        se = se * expf(mx - m2) + v.y * expf(v.x - m2);
        mx = m2;
    }
    fold[q][rl] = make_float2(mx, se);
    __syncthreads();
    if (q != 0 || r >= M) return;
    for (int i = 1; i < NLL_FIN_WAVES; ++i) {
        const float2 v = fold[i][rl];
        if (v.x == -INFINITY) continue;                    // a wave without tiles (fewer than 16 tiles)
        const float m2 = fmaxf(mx, v.x);
        se = se * expf(mx - m2) + v.y * expf(v.x - m2);
        mx = m2;
    }
    nll[r] = (mx + logf(se)) - tgt_logit[r];
}

// Register r of accumulator tile (i, j) is row 32*i + 8*(r/4) + 4*(lane/32) + r%4, column 32*j + lane%32
// of the wave tile (row_w already holds the wave tile's first row + 4*(lane/32)). Per 32-row tile all
// global reads of the epilogue are issued first, then the row pairs are combined and stored.
template <class E, class = void> struct epi_gated { static constexpr bool value = false; };
template <class E> struct epi_gated<E, decltype((void)&E::run)> { static constexpr bool value = true; };
template <class E, class = void> struct epi_whole_tile { static constexpr bool value = false; };
template <class E> struct epi_whole_tile<E, decltype((void)E::whole_tile)> { static constexpr bool value = E::whole_tile; };

template <bool FULL, int TM, int TN, class Epi>
__device__ __forceinline__ void gemm_epilogue(const floatx16_t (&acc)[TM][TN], const Epi &epi, int64_t row_w, int64_t M,
                                              int vcol0, int c)
{
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        typename Epi::template Aux<TN> aux[8];
#pragma unroll
        for (int rp = 0; rp < 8; ++rp) {
            const int64_t row0 = row_w + i * 32 + 8 * (rp >> 1) + 2 * (rp & 1);
            const bool ok0 = FULL || row0 < M, ok1 = FULL || row0 + 1 < M;
            epi.template preload0<TN>(ok0 ? row0 : M - 1, ok1 ? row0 + 1 : M - 1, aux[rp]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int rp = 0; rp < 8; ++rp) {
            const int64_t row0 = row_w + i * 32 + 8 * (rp >> 1) + 2 * (rp & 1);
            const bool ok0 = FULL || row0 < M, ok1 = FULL || row0 + 1 < M;
            epi.template preload<TN>(ok0 ? row0 : M - 1, ok1 ? row0 + 1 : M - 1, ok0, ok1, vcol0, c, aux[rp]);
        }
        __builtin_amdgcn_sched_barrier(0);                // keep the reads up here: sunk next to their uses they serialise
#pragma unroll
        for (int rp = 0; rp < 8; ++rp) {
            const int r = 2 * rp;                         // registers r, r + 1: two consecutive rows
            const int64_t row0 = row_w + i * 32 + 8 * (r >> 2) + (r & 3);
            float v0[TN], v1[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) { v0[j] = acc[i][j][r]; v1[j] = acc[i][j][r + 1]; }
            epi.template rows2<TN>(row0, FULL || row0 < M, FULL || row0 + 1 < M, vcol0, c, v0, v1, aux[rp]);
        }
    }
}

// 16 bytes per lane from global memory (wave-uniform base + 32-bit byte offset per lane) straight into LDS: lane l's
// piece lands at lds_addr + 16 * l (M0 holds the wave's LDS byte address; one wait state between writing M0 and the
// load). Written as inline assembly because the compiler, which sees an LDS write it cannot place, would wait for
// the load before the next LDS read of any stage. The kernel therefore owns the waits: vm_wait<0>() before the
// barrier that publishes a stage, and before a workgroup ends. The kernel must have no static LDS (the dynamic
// segment then starts at LDS address 0).
__device__ __forceinline__ void dtl16(const bf16_t *base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "memory", "m0");
}
// s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the expcnt and lgkmcnt fields at "no wait")
template <int N> __device__ __forceinline__ void vm_wait()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt(((N >> 4) << 14) | 0x0F70 | (N & 15));
}

// EpiResidF32 for whole tiles of a kernel that is not persistent (its two LDS stages are dead once the K loop is
// over). In the accumulator layout a lane holds one column of four consecutive rows, so the plain epilogue issues a
// 4-byte store and a 2-byte residual load per element: 1024 store and 1024 load instructions per tile through the
// CU's one memory pipeline, which takes them at a few tens of cycles each whatever their size. Here the wave passes
// its tile, 64 rows at a time, through its own quarter of the LDS and takes it back row-wise: a lane then owns four
// consecutive columns of a row, reads the residual as 8 bytes and stores 16 (two whole 512-byte rows of the wave tile
// per instruction): 64 + 64 instructions per wave tile instead of 256 + 256. Same values as EpiResidF32.
struct EpiResidF32Tile {
    static constexpr bool persistent_walk = false;
    static constexpr bool whole_tile = true;
    const bf16_t *resid; float *out; int64_t ld;
    template <int TM, int TN>
    __device__ __forceinline__ void tile(const floatx16_t (&acc)[TM][TN], int64_t row_w, int vcol_w, int lane) const
    {
        static_assert(TM * 32 == 128 && TN * 32 == 128, "128 x 128 wave tiles: 64 rows of fp32 fill the wave's 32 KB");
        extern __shared__ __align__(16) unsigned char lds_all[];          // the kernel's dynamic segment (128 KB)
        const int vcol_u = __builtin_amdgcn_readfirstlane(vcol_w);
        const int64_t row_u = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(row_w >> 32)) << 32) |
                                        (uint32_t)__builtin_amdgcn_readfirstlane((int)row_w));
        const int wave_u = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const int c = lane & 31, rg = lane >> 5;
        unsigned char *const lw = lds_all + (uint32_t)wave_u * 32768u;    // [64 rows][128 fp32]
        const char *const rbase = reinterpret_cast<const char *>(resid + row_u * ld + vcol_u);
        char *const obase = reinterpret_cast<char *>(out + row_u * ld + vcol_u);
        const uint32_t ld_u = (uint32_t)ld;                      // a wave tile spans 128 rows: offsets far below 2^32
        // row-wise pass: instruction t of a half covers rows 2t and 2t + 1; this lane: row 2t + rg, columns 4c .. 4c + 3
        const uint32_t el0 = (uint32_t)rg * ld_u + (uint32_t)c * 4u;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            u32x2_t rv[32];                                      // the half's residual, requested before the LDS round trip
#pragma unroll
            for (int t = 0; t < 32; ++t)
                rv[t] = *reinterpret_cast<const u32x2_t *>(rbase + (el0 + (uint32_t)(hf * 64 + 2 * t) * ld_u) * 2u);
#pragma unroll
            for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = ii * 32 + 8 * (r >> 2) + (r & 3);   // row of the half, less the lane's 4 * rg
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        *reinterpret_cast<float *>(lw + (uint32_t)(k + 4 * rg) * 512u + (uint32_t)(c + 32 * j) * 4u) = acc[hf * 2 + ii][j][r];
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own writes, read back by the wave: no barrier
#pragma unroll
            for (int t = 0; t < 32; ++t) {
                const f32x4_t v = *reinterpret_cast<const f32x4_t *>(lw + (uint32_t)(2 * t + rg) * 512u + (uint32_t)c * 16u);
                const f32x4_t o = {v[0] + __uint_as_float(rv[t][0] << 16), v[1] + __uint_as_float(rv[t][0] & 0xFFFF0000u),
                                   v[2] + __uint_as_float(rv[t][1] << 16), v[3] + __uint_as_float(rv[t][1] & 0xFFFF0000u)};
                *reinterpret_cast<f32x4_t *>(obase + (el0 + (uint32_t)(hf * 64 + 2 * t) * ld_u) * 4u) = o;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the reads are over before the next half overwrites the rows
        }
    }
};

// PERSIST: one workgroup per CU walks every tile of its slot in the XCD's band (tile index + workgroups per XCD) and
// the pipeline runs across the tile boundary: the last two K steps of a tile request the first two slices of the next
// one, so only a workgroup's first tile starts cold. (The pipeline's state between steps is LDS only, no registers,
// so the epilogue in between costs it nothing.)
template <int BM, int BN, int WM, int WN, class Epi, bool PERSIST>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64) __attribute__((amdgpu_waves_per_eu(1, 1)))
k_gemm_mfma(const bf16_t *__restrict__ A, int64_t lda, BMap bmap, int64_t M, int Nv, int K, int tiles_m, int tiles_n,
            Epi epi)
{
    constexpr int NWM = BM / WM, NWN = BN / WN, NT = NWM * NWN * 64;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWS_PER_PASS = NT / 8;                 // 8 threads (16-byte chunks) per 128-byte row
    constexpr int A_PASSES = BM / ROWS_PER_PASS, B_PASSES = BN / ROWS_PER_PASS;
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile / thread mismatch");
    extern __shared__ __align__(16) unsigned char lds[];

    if constexpr (epi_gated<Epi>::value) {
        if (!epi.run()) return;                            // the whole grid, before any barrier
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / NWN, wn = wave - wm * NWN;

    // ---- XCD-aware tile mapping: workgroup b runs on XCD b % 8; XCD x owns a contiguous band ----
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + 7) / 8;
    const int band_end = ((int)(blockIdx.x & 7) + 1) * per_xcd < n_tiles ? ((int)(blockIdx.x & 7) + 1) * per_xcd : n_tiles;
    const int lin_step = (int)(gridDim.x >> 3);             // PERSIST: workgroups per XCD
    int lin = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (lin >= band_end) return;
    const int group_sz = GROUP_M * tiles_n;

    // ---- per-thread global sources and LDS destinations of the staged K slices ----
    // A pass covers ROWS_PER_PASS rows (8 threads x 16 bytes per 128-byte row). Sources are wave-uniform
    // bases (scalar registers) plus one 32-bit lane offset each; the LDS swizzle does not depend on the
    // pass (ROWS_PER_PASS is a multiple of 16), so one destination offset serves all passes.
    static_assert(ROWS_PER_PASS % 16 == 0, "swizzle must repeat from pass to pass");
    const int chunk = tid & 7, r_in_pass = tid >> 3;
    const bf16_t *a_base;                                   // uniform
    uint32_t a_off[A_PASSES];
    const bf16_t *b_base[B_PASSES];                         // uniform: first weight row of each pass
    // sources of tile LIN_, its first row and first virtual column
#define SOL_TILE_SRC(LIN_, M0_, N0_)                                                                       \
    {                                                                                                      \
        const int grp_ = (LIN_) / group_sz, in_grp_ = (LIN_) - grp_ * group_sz;                            \
        const int rows_here_ = (tiles_m - grp_ * GROUP_M) < GROUP_M ? (tiles_m - grp_ * GROUP_M) : GROUP_M; \
        M0_ = (int64_t)(grp_ * GROUP_M + in_grp_ % rows_here_) * BM;                                       \
        N0_ = (in_grp_ / rows_here_) * BN;                                                                 \
        a_base = A + M0_ * lda;                                                                            \
        _Pragma("unroll") for (int p = 0; p < A_PASSES; ++p) {                                             \
            int64_t rl = p * ROWS_PER_PASS + r_in_pass;                                                    \
            if (M0_ + rl >= M) rl = M - 1 - M0_;   /* ragged last tile: re-read the last row, never stored */ \
            a_off[p] = ((uint32_t)(rl * lda) + (uint32_t)((chunk ^ SOL_SWZ(r_in_pass)) * 8)) * 2u;   /* bytes; lane = LDS slot */ \
        }                                                                                                  \
        _Pragma("unroll") for (int p = 0; p < B_PASSES; ++p) b_base[p] = bmap.row(N0_ + p * ROWS_PER_PASS); \
    }
    int64_t m0, m0_next = 0;
    int n0, n0_next = 0;
    SOL_TILE_SRC(lin, m0, n0);
    const uint32_t b_off = ((uint32_t)r_in_pass * (uint32_t)bmap.ld + (uint32_t)((chunk ^ SOL_SWZ(r_in_pass)) * 8)) * 2u;

    floatx16_t acc[TM][TN];
#define SOL_ACC_ZERO                                                                                       \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)          \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    SOL_ACC_ZERO;

    // Two LDS stages filled by LDS-direct loads: slice kt+2 is requested into the stage of slice kt right after the
    // barrier that ends the reads of slice kt, and must have landed by the next step's barrier.
    bf16x8_t fa0[TM], fb0[TN], fa1[TM], fb1[TN], fa2[TM], fb2[TN], fa3[TM], fb3[TN];   // one set per k-group of a step
    const int KT = K / BK;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int frow = lane & 31, fk = lane >> 5, fsw = SOL_SWZ(frow);
    const int a_frag0 = (wm * WM + frow) * 128;
    const int b_frag0 = BM * 128 + (wn * WN + frow) * 128;
#define SOL_F_READ(FA, FB, STAGE_, KK_)                                                                    \
    {                                                                                                      \
        const int coff = ((((KK_) * 2 + fk) ^ fsw) << 4);                                                  \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) FA[i] = __builtin_bit_cast(                         \
            bf16x8_t, *reinterpret_cast<const u32x4_t *>((STAGE_) + a_frag0 + i * 32 * 128 + coff));       \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) FB[j] = __builtin_bit_cast(                         \
            bf16x8_t, *reinterpret_cast<const u32x4_t *>((STAGE_) + b_frag0 + j * 32 * 128 + coff));       \
    }
#define SOL_MMA(FA, FB)                                                                                    \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)          \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[i], FB[j], acc[i][j], 0, 0, 0);
#define SOL_FENCE __builtin_amdgcn_sched_barrier(0)
#define SOL_ORDER_RM                                                                                       \
    _Pragma("unroll") for (int i_ = 0; i_ < TM + TN; ++i_) {                                               \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                 \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                 \
    }                                                                                                      \
    __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN), 0);
    // all passes of slice KT_ into the stage at LDS byte offset STG_
#define SOL_DTL_ONE(P_, KT_, STG_)                                                                         \
    {                                                                                                      \
        const int koff_ = ((KT_) < KT ? (KT_) : KT - 1) * BK;                                              \
        if ((P_) < A_PASSES) dtl16(a_base + koff_, a_off[(P_)], (uint32_t)((STG_) + (P_) * ROWS_PER_PASS * 128 + wave_u * 1024)); \
        else dtl16(b_base[(P_) - A_PASSES] + koff_, b_off, (uint32_t)((STG_) + BM * 128 + ((P_) - A_PASSES) * ROWS_PER_PASS * 128 + wave_u * 1024)); \
    }
    static_assert(TM * TN == A_PASSES + B_PASSES && ROWS_PER_PASS == 32, "one LDS-direct load per MFMA of a k-group");
    // one k-group of the second half of a step, in issue order: behind each MFMA one fragment read (the first TM + TN
    // MFMAs: k-group KK_ of the next slice into the set (FRA, FRB)) and behind every second MFMA one LDS-direct
    // request (passes P0_ .. P0_ + 7 of slice KT_LOAD_ into the stage that was just read out)
#define SOL_MMA_DTL(FA, FB, FRA, FRB, STG_, KK_, P0_, KT_LOAD_, CURO_)                                     \
    {                                                                                                      \
        const int coff_ = ((((KK_) * 2 + fk) ^ fsw) << 4);                                                 \
        _Pragma("unroll") for (int m = 0; m < TM * TN; ++m) {                                              \
            acc[m / TN][m % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[m / TN], FB[m % TN],          \
                                                                         acc[m / TN][m % TN], 0, 0, 0);    \
            if (m < TM) FRA[m] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>(          \
                            (STG_) + a_frag0 + m * 32 * 128 + coff_));                                     \
            else if (m < TM + TN) FRB[m - TM] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>( \
                            (STG_) + b_frag0 + (m - TM) * 32 * 128 + coff_));                              \
            if (m & 1) SOL_DTL_ONE((P0_) + m / 2, KT_LOAD_, CURO_);                                        \
            SOL_FENCE;                                                                                     \
        }                                                                                                  \
    }
    // One step. Fragments are read two k-groups ahead (four register sets), so the reads of the current stage are
    // over after the second k-group: the barrier sits there, and the second half of the step requests slice
    // KT_LOAD_ into the stage just read out (CURO_ = its LDS byte offset) while it reads the first two k-groups of
    // the next stage. The requests of the previous step must have landed before the barrier publishes their stage.
#define SOL_STEP(CUR_, NXT_, CURO_, KT_LOAD_)                                                              \
    SOL_F_READ(fa2, fb2, CUR_, 2); SOL_MMA(fa0, fb0); SOL_ORDER_RM; SOL_FENCE;                             \
    SOL_F_READ(fa3, fb3, CUR_, 3); SOL_MMA(fa1, fb1); SOL_ORDER_RM; SOL_FENCE;                             \
    vm_wait<0>();                                                                                          \
    __syncthreads();                                                                                       \
    SOL_FENCE;                                                                                             \
    SOL_MMA_DTL(fa2, fb2, fa0, fb0, NXT_, 0, 0, KT_LOAD_, CURO_);                                          \
    SOL_MMA_DTL(fa3, fb3, fa1, fb1, NXT_, 1, (A_PASSES + B_PASSES) / 2, KT_LOAD_, CURO_);

    constexpr int STAGE_BYTES2 = (BM + BN) * 128;
    unsigned char *const stage0 = lds, *const stage1 = lds + STAGE_BYTES2;
#pragma unroll
    for (int p = 0; p < A_PASSES + B_PASSES; ++p) SOL_DTL_ONE(p, 0, 0);
#pragma unroll
    for (int p = 0; p < A_PASSES + B_PASSES; ++p) SOL_DTL_ONE(p, 1, STAGE_BYTES2);
    vm_wait<0>();
    __syncthreads();
    SOL_F_READ(fa0, fb0, stage0, 0);
    SOL_F_READ(fa1, fb1, stage0, 1);
    const int vcol_w = wn * WN;
    const int64_t row_w = wm * WM + 4 * (lane >> 5);
    if constexpr (!PERSIST) {
        for (int kt = 0; kt < KT; kt += 2) {                // KT is even (K is a multiple of 128)
            SOL_STEP(stage0, stage1, 0, kt + 2);
            SOL_STEP(stage1, stage0, STAGE_BYTES2, kt + 3);
        }
        vm_wait<0>();
        __syncthreads();
    } else {
        for (;;) {
            const bool more = lin + lin_step < band_end;
            for (int kt = 0; kt < KT - 2; kt += 2) {
                SOL_STEP(stage0, stage1, 0, kt + 2);
                SOL_STEP(stage1, stage0, STAGE_BYTES2, kt + 3);
            }
            // the last two steps request slices 0 and 1 of the next tile (of this tile again after the last one:
            // never used)
            SOL_TILE_SRC(more ? lin + lin_step : lin, m0_next, n0_next);
            SOL_STEP(stage0, stage1, 0, 0);
            SOL_STEP(stage1, stage0, STAGE_BYTES2, 1);
            // stage 0 holds the next tile's slice 0 and its first fragments are in registers; slice 1 is on its way
            // into stage 1 and is waited for in the next tile's first step
            if constexpr (epi_whole_tile<Epi>::value) epi.template tile<TM, TN>(acc, m0 + wm * WM, n0 + vcol_w, lane);
            else gemm_epilogue<true, TM, TN>(acc, epi, m0 + row_w, M, n0 + vcol_w, lane & 31);   // M % BM == 0 (launcher): with
            if (!more) break;                               // both epilogue versions in the loop the compiler spills the accumulators
            SOL_ACC_ZERO;
            lin += lin_step; m0 = m0_next; n0 = n0_next;
        }
        vm_wait<0>();                                       // no LDS-direct load outlives its workgroup
        return;
    }
#undef SOL_F_READ
#undef SOL_MMA
#undef SOL_STEP
#undef SOL_MMA_DTL
#undef SOL_ORDER_RM
#undef SOL_FENCE
#undef SOL_DTL_ONE
#undef SOL_TILE_SRC
#undef SOL_ACC_ZERO

    // ---- epilogue straight from the accumulators (tiles that lie wholly inside the matrix take the
    // version without row checks) ----
    if constexpr (epi_whole_tile<Epi>::value) {             // (the launcher admits whole tiles only)
        epi.template tile<TM, TN>(acc, m0 + wm * WM, n0 + vcol_w, lane);
    } else {
        if (m0 + BM <= M) gemm_epilogue<true, TM, TN>(acc, epi, m0 + row_w, M, n0 + vcol_w, lane & 31);
        else gemm_epilogue<false, TM, TN>(acc, epi, m0 + row_w, M, n0 + vcol_w, lane & 31);
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
// compute units of the current device (one persistent workgroup each), 0 if the query fails
static int device_cus()
{
    static int cus[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (!cus[dev]) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cus[dev] = n;
    }
    return cus[dev];
}

#ifndef SOL_GEMM_PERSIST
#define SOL_GEMM_PERSIST 1
#endif

template <int BM, int BN, int WM, int WN, class Epi>
static bool launch_mfma(const bf16_t *A, int64_t lda, const BMap &bmap, int64_t M, int Nv, int K, const Epi &epi,
                        hipStream_t st)
{
    if (M <= 0) return true;
    if (Nv % BN || K % (2 * BK) || K < 2 * BK) return false;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr size_t lds = 2 * (size_t)(BM + BN) * 128;
    auto kern = k_gemm_mfma<BM, BN, WM, WN, Epi, false>;
    auto kern_p = k_gemm_mfma<BM, BN, WM, WN, Epi, true>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern_p), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return false;
        attr_done = true;
    }
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = Nv / BN;
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + 7) / 8;
    // several tiles per CU and no ragged tile: the persistent walk, one workgroup per CU (CUs / 8 per XCD)
    const int wg_xcd = device_cus() / 8;
    if (SOL_GEMM_PERSIST && Epi::persistent_walk && wg_xcd > 0 && per_xcd > wg_xcd && M % BM == 0) {
        hipLaunchKernelGGL(kern_p, dim3(wg_xcd * 8), dim3(NT), lds, st, A, lda, bmap, M, Nv, K, tiles_m, tiles_n, epi);
        return true;
    }
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(NT), lds, st, A, lda, bmap, M, Nv, K, tiles_m, tiles_n, epi);
    return true;
}

// Tile configuration of the fused layer GEMMs: 256 x 256 workgroup tiles, 4 waves (one per SIMD) with
// 128 x 128 wave tiles: 256 accumulator registers per lane, the smallest LDS read traffic per MFMA
// (128 KB per K slice), and latency hidden by the software pipeline rather than by a second wave.
// The q/k/v epilogue needs a whole head (up to 128 columns) inside one wave tile.
constexpr int SOL_WN = 128;
#define SOL_TILE 256, 256, 128, SOL_WN
#define SOL_TILE_QKV 256, 256, 128, SOL_WN

bool launch_gemm_qkv_rope(const void *h, const void *wq, const void *wk, const void *wv, void *q, void *kc, void *vc,
                          const float2 *rope, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh,
                          int d, int *flags, void *row_sp_ws, hipStream_t st, int cache_rows)
{
    const int nq = Hq * dh, nkv = Hkv * dh;
    if ((dh != 64 && dh != 128) || nq % 256 || nkv % 256) return false;      // heads must not straddle wave tiles
    const int crows = cache_rows > 0 ? cache_rows : L_max;                    // rows of a (sequence, KV head) in the caches
    const int64_t M = (int64_t)n_seq * T;
    if (M <= 0) return true;
    if (d % (2 * BK) || d < 2 * BK) return false;
    BMap bm{};
    bm.base[0] = (const bf16_t *)wq; bm.base[1] = (const bf16_t *)wk; bm.base[2] = (const bf16_t *)wv;
    bm.seg_end[0] = nq; bm.seg_end[1] = nq + nkv; bm.seg_end[2] = nq + 2 * nkv;
    bm.mode = 0; bm.half = 0; bm.ld = d;
    int2 *row_sp = (int2 *)row_sp_ws;
    // whole tiles of at most two sequences each: positions by arithmetic (the epilogue's 32-bit byte offsets span two
    // cache slabs, 128 rows of q, and the cos / sin table); it runs unless k_row_positions has flagged a sequence, in
    // which case the general kernel behind it does
    const bool tiles = M % 256 == 0 && T >= 128 && (int64_t)(Hkv + 1) * crows * dh * 2 < (1ll << 31) &&
                       (int64_t)L_max * dh * 4 < (1ll << 31);
    const bool sure = pos0 == nullptr && T <= L_max;          // every sequence starts at 0 and fits: nothing to flag
    int *gate = sure ? nullptr : flags;
    if (!(tiles && sure))                                     // the rows' (sequence, position) table, and the flags
        hipLaunchKernelGGL(k_row_positions, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, st, pos0, M, T, L_max, row_sp, flags);
    if (dh == 64) {
        if (tiles) {
            EpiQkvRopeTile<64> te{(bf16_t *)q, (bf16_t *)kc, (bf16_t *)vc, rope, pos0, T, crows, Hq, Hkv, n_seq, gate};
            if (!launch_mfma<SOL_TILE_QKV>((const bf16_t *)h, d, bm, M, nq + 2 * nkv, d, te, st)) return false;
            if (sure) return true;
        }
        EpiQkvRope<64> epi{(bf16_t *)q, (bf16_t *)kc, (bf16_t *)vc, rope, row_sp, crows, Hq, Hkv, tiles ? flags : nullptr};
        return launch_mfma<SOL_TILE_QKV>((const bf16_t *)h, d, bm, M, nq + 2 * nkv, d, epi, st);
    }
    if (tiles) {
        EpiQkvRopeTile<128> te{(bf16_t *)q, (bf16_t *)kc, (bf16_t *)vc, rope, pos0, T, crows, Hq, Hkv, n_seq, gate};
        if (!launch_mfma<SOL_TILE_QKV>((const bf16_t *)h, d, bm, M, nq + 2 * nkv, d, te, st)) return false;
        if (sure) return true;
    }
    EpiQkvRope<128> epi{(bf16_t *)q, (bf16_t *)kc, (bf16_t *)vc, rope, row_sp, crows, Hq, Hkv, tiles ? flags : nullptr};
    return launch_mfma<SOL_TILE_QKV>((const bf16_t *)h, d, bm, M, nq + 2 * nkv, d, epi, st);
}

bool launch_gemm_resid_f32(const void *a, const void *w, const void *resid, float *out, int64_t M, int N, int K,
                           hipStream_t st)
{
    BMap bm{};
    bm.base[0] = (const bf16_t *)w; bm.seg_end[0] = bm.seg_end[1] = bm.seg_end[2] = N; bm.mode = 0; bm.ld = K;
    if (M % 256 == 0) {                                   // whole tiles
        EpiResidF32Tile te{(const bf16_t *)resid, out, N};
        return launch_mfma<SOL_TILE>((const bf16_t *)a, K, bm, M, N, K, te, st);
    }
    EpiResidF32 epi{(const bf16_t *)resid, out, N};
    return launch_mfma<SOL_TILE>((const bf16_t *)a, K, bm, M, N, K, epi, st);
}

bool launch_gemm_gateup_silu(const void *h, const void *wg, const void *wu, void *a, int64_t M, int dff, int d,
                             hipStream_t st)
{
    if (dff % (SOL_WN / 2)) return false;
    BMap bm{};
    bm.base[0] = (const bf16_t *)wg; bm.base[1] = (const bf16_t *)wu; bm.mode = 1; bm.half = SOL_WN / 2; bm.ld = d;
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


static int64_t nll_pad_rows(int64_t M) { return (M + 255) / 256 * 256; }
int64_t gemm_nll_hf_rows(int64_t M) { return nll_pad_rows(M); }
size_t gemm_nll_scratch_bytes(int64_t M, int V) { return (size_t)nll_pad_rows(M) * ((size_t)(V / SOL_WN) * sizeof(float2) + 8); }

// nll[r] = logsumexp(hf[r] . lm_head^T) - (hf[r] . lm_head[target(r)]) without materialising the logits.
// hf: [gemm_nll_hf_rows(M)][K], the first M rows filled (the padding rows are cleared here); scratch:
// gemm_nll_scratch_bytes(M, V) bytes. Returns false (nothing launched) if the shape does not tile.
bool launch_gemm_nll(void *hf, const void *lm_head, const int32_t *targets, int G, int T, bool broadcast_g,
                     float *nll, void *scratch, int64_t M, int V, int K, int *flags, hipStream_t st)
{
    if (M <= 0) return true;
    const int64_t Mp = nll_pad_rows(M);
    if (V % 256 || K % (2 * BK) || K < 2 * BK || Mp >= (1ll << 31)) return false;
    const int n_wt = V / SOL_WN;
    float2 *part = (float2 *)scratch;
    float *tgt_logit = (float *)(part + (size_t)Mp * n_wt);
    int32_t *row_tgt = (int32_t *)(tgt_logit + Mp);
    hipLaunchKernelGGL(k_row_targets, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, st, targets, M, G, T,
                       broadcast_g ? 1 : 0, V, row_tgt, flags);
    if (Mp > M) launch_fill_i32((int32_t *)((bf16_t *)hf + M * K), 0, (Mp - M) * K / 2, st);   // K is even
    BMap bt{};
    bt.base[0] = (const bf16_t *)hf; bt.seg_end[0] = bt.seg_end[1] = bt.seg_end[2] = (int)Mp; bt.mode = 0; bt.ld = K;
    EpiNllCols epc{part, Mp};
    if (!launch_mfma<SOL_TILE>((const bf16_t *)lm_head, K, bt, V, (int)Mp, K, epc, st)) return false;
    hipLaunchKernelGGL(k_target_logit, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, (const bf16_t *)hf,
                       (const bf16_t *)lm_head, row_tgt, M, K, tgt_logit);
    hipLaunchKernelGGL(k_nll_finish_cols, dim3((unsigned)((M + 63) / 64)), dim3(NLL_FIN_WAVES * 64), 0, st, part, tgt_logit, n_wt,
                       M, Mp, nll);
    return true;
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
              float *__restrict__ partial, int xrow)
{
    extern __shared__ __align__(16) unsigned char xs[];      // [MT*32][xrow]: xrow = padded bytes of a staged row (the
                                                             // chunk is no longer than a split: short splits leave room
                                                             // for more workgroups per CU)
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

    // The split's K range is walked in 64-wide blocks, UK blocks per batch, two batches per LDS chunk of
    // activations. Weight loads run one batch ahead of the MFMAs (two register sets), and the first batch
    // of a chunk is already in flight while the chunk's activations are staged, so a workgroup pays the
    // global-memory latency about once instead of once per batch.
    constexpr int UK = 4;                                             // 64-wide K blocks per batch
    static_assert(SK_KC == 2 * UK * 64, "two batches per staged chunk");
    const int nblk = (k_end - k_begin) / 64;
    u32x4_t wa0[UK][4], wa1[UK][4];
#define SOL_SK_LOADW(WA, B0_)                                                                              \
    _Pragma("unroll") for (int u = 0; u < UK; ++u) {                                                       \
        const int blk_ = ((B0_) + u < nblk) ? (B0_) + u : nblk - 1;     /* ragged tail: re-read, not used */ \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                      \
            WA[u][j] = *reinterpret_cast<const u32x4_t *>(wrow + k_begin + blk_ * 64 + j * 8);             \
    }
#define SOL_SK_MMA(WA, B0_, KOFF_)          /* KOFF_: offset of the batch inside the staged chunk */          \
    _Pragma("unroll") for (int u = 0; u < UK; ++u) {                                                       \
        if ((B0_) + u < nblk) {                                                                            \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                \
                const bf16x8_t af = __builtin_bit_cast(bf16x8_t, WA[u][j]);                                \
                _Pragma("unroll") for (int t = 0; t < MT; ++t) {                                           \
                    const unsigned char *xp = xs + (t * 32 + r) * xrow + ((KOFF_) + u * 64 + h * 32 + j * 8) * 2; \
                    const bf16x8_t bfr = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>(xp)); \
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[t], 0, 0, 0);            \
                }                                                                                          \
            }                                                                                              \
        }                                                                                                  \
    }
    if (live) SOL_SK_LOADW(wa0, 0);
    for (int b0 = 0; b0 < nblk; b0 += 2 * UK) {
        const int kc = k_begin + b0 * 64;
        const int kw = (k_end - kc < SK_KC) ? (k_end - kc) : SK_KC;   // multiple of 64
        __syncthreads();                                              // previous chunk fully consumed
        // stage x[0..MT*32)[kc .. kc+kw) into LDS, 16 bytes per thread per step (rows >= M: zeros)
        const int pieces = kw / 8;
        for (int idx = tid; idx < MT * 32 * pieces; idx += 256) {
            const int m = idx / pieces, p = idx - m * pieces;
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (m < M) v = *reinterpret_cast<const u32x4_t *>(x + (int64_t)m * ldx + kc + p * 8);
            *reinterpret_cast<u32x4_t *>(xs + m * xrow + p * 16) = v;
        }
        __syncthreads();
        if (live) {
            if (b0 + UK < nblk) SOL_SK_LOADW(wa1, b0 + UK);
            SOL_SK_MMA(wa0, b0, 0);
            if (b0 + 2 * UK < nblk) SOL_SK_LOADW(wa0, b0 + 2 * UK);
            if (b0 + UK < nblk) SOL_SK_MMA(wa1, b0 + UK, UK * 64);
        }
    }
#undef SOL_SK_LOADW
#undef SOL_SK_MMA
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
    int want = (2048 + tiles - 1) / tiles;
    int cap = K / (4 * (M > 0 ? M : 1));
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
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(k_gemm_skinny<2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)((size_t)64 * SK_XROW)) != hipSuccess) return false;
        attr_done = true;
    }
    const int xrow = (k_per_split < SK_KC ? k_per_split : SK_KC) * 2 + 16;
    if (M <= 32)
        hipLaunchKernelGGL((k_gemm_skinny<1>), grid, dim3(256), (size_t)32 * xrow, st, x, ldx, bm, M, Nv, K, k_per_split, partial, xrow);
    else
        hipLaunchKernelGGL((k_gemm_skinny<2>), grid, dim3(256), (size_t)64 * xrow, st, x, ldx, bm, M, Nv, K, k_per_split, partial, xrow);
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
