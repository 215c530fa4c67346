// Reward reduction after the teacher-forced pass (Method, "Actions and controlled compute", Eqs. 2-5, and
// "GRPO with per-sequence budget sampling"): from the NLL tensor [B][K][T] and the action ids to
//   - the realised compute averages of each schedule over its effective steps, the squared-hinge penalty,
//   - the discounted return-to-go of the task reward r_t = -nll_t, the signal r_t = G_t - C,
//   - advantages: mean-centred over the K schedules of an input at fixed t, whitened over the batch.
// Tiny and latency-bound: three short kernels, sums that decide the whitening in fp64 and in a fixed order.
#include "sol_internal.h"

namespace sol {

constexpr int RW_BLOCK = 256;

__device__ __forceinline__ double block_sum_f64(double v, double *red)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if (lane == 0) red[w] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int i = 0; i < RW_BLOCK / 64; ++i) t += red[i];
    __syncthreads();
    return t;
}

// One workgroup per schedule (b, k). Return-to-go: every thread scans a contiguous chunk of steps backwards from
// a zero carry, thread 0 chains the chunk carries (G at a chunk's first step is its local value plus gamma^len
// times the carry of the chunk after it), then every thread adds gamma^(steps to the chunk end) times its carry.
__global__ void __launch_bounds__(RW_BLOCK)
k_reward_rows(const float *__restrict__ nll, const int32_t *__restrict__ ids, const ActionDev *__restrict__ table,
              int n_actions, const int32_t *__restrict__ eff, const float *__restrict__ targets, RewardCfg rc, int K, int T,
              float *__restrict__ avg_out, float *__restrict__ pen_out, float *__restrict__ ret_out,
              float *__restrict__ signal, int *flags)
{
    __shared__ double red[RW_BLOCK / 64];
    __shared__ float s_first[RW_BLOCK], s_decay[RW_BLOCK], s_carry[RW_BLOCK];
    const int k = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int64_t row = ((int64_t)b * K + k) * T;
    // ---- realised averages over the effective steps, penalty -------------------------------------
    double sk = 0.0, sr = 0.0, se = 0.0, sn = 0.0;
    bool bad = false;
    for (int t = tid; t < T; t += RW_BLOCK) {
        const int e = eff ? (eff[(int64_t)b * T + t] != 0) : 1;
        int id = ids[row + t];
        if (id < 0 || id >= n_actions) { bad = true; id = 0; }
        const ActionDev a = table[id];
        if (e) {
            sk += (double)a.keep_num / (double)a.keep_den;
            sr += (double)a.mlp_keep_num / (double)a.mlp_keep_den;
            se += (double)(a.bits < 16u ? a.bits : 16u) / 16.0;
            sn += 1.0;
        }
    }
    if (bad) atomicOr(flags, FLAG_BAD_ACTION);
    sk = block_sum_f64(sk, red); sr = block_sum_f64(sr, red); se = block_sum_f64(se, red); sn = block_sum_f64(sn, red);
    const float ck = targets[b * 3 + 0], cr = targets[b * 3 + 1], ce = targets[b * 3 + 2];
    const float ak = sn > 0.0 ? (float)(sk / sn) : ck, ar = sn > 0.0 ? (float)(sr / sn) : cr, ae = sn > 0.0 ? (float)(se / sn) : ce;
    auto psi = [&](float d) { const float x = fmaxf(0.f, fabsf(d) - rc.tau); return x * x; };
    const float pen = rc.alpha_kappa * psi(ak - ck) + rc.alpha_rho * psi(ar - cr) + rc.alpha_eta * psi(ae - ce);
    if (tid == 0) {
        if (avg_out) { float *o = avg_out + ((int64_t)b * K + k) * 3; o[0] = ak; o[1] = ar; o[2] = ae; }
        if (pen_out) pen_out[(int64_t)b * K + k] = pen;
    }
    // ---- return-to-go ---------------------------------------------------------------------------
    const int len = (T + RW_BLOCK - 1) / RW_BLOCK;
    const int t0 = tid * len, t1 = (t0 + len < T) ? t0 + len : T;   // this thread's steps [t0, t1)
    float g = 0.f, decay = 1.f;
    for (int t = t1 - 1; t >= t0; --t) { g = -nll[row + t] + rc.gamma * g; decay *= rc.gamma; }
    s_first[tid] = g;                                               // local G at t0 (0 for an empty chunk)
    s_decay[tid] = decay;                                           // gamma^(t1 - t0)
    __syncthreads();
    if (tid == 0) {
        float carry = 0.f;                                          // G at the first step after the chunk
        for (int i = RW_BLOCK - 1; i >= 0; --i) {
            s_carry[i] = carry;
            carry = s_first[i] + s_decay[i] * carry;
        }
    }
    __syncthreads();
    const float carry = s_carry[tid];
    g = 0.f;
    float w = rc.gamma;                                             // gamma^(t1 - t)
    for (int t = t1 - 1; t >= t0; --t) {
        g = -nll[row + t] + rc.gamma * g;
        const float G = g + w * carry;
        w *= rc.gamma;
        if (ret_out) ret_out[row + t] = G;
        signal[row + t] = G - pen;
    }
}

// mean over the K schedules of an input at fixed t; writes the centred signal and per-workgroup partial sums
__global__ void __launch_bounds__(RW_BLOCK)
k_reward_center(const float *__restrict__ signal, int K, int T, float *__restrict__ adv, double *__restrict__ partial)
{
    __shared__ double red[RW_BLOCK / 64];
    const int b = blockIdx.y, t = blockIdx.x * RW_BLOCK + threadIdx.x;
    double s1 = 0.0, s2 = 0.0;
    if (t < T) {
        const float *p = signal + (int64_t)b * K * T + t;
        double m = 0.0;
        for (int k = 0; k < K; ++k) m += (double)p[(int64_t)k * T];
        m /= (double)K;
        for (int k = 0; k < K; ++k) {
            const double c = (double)p[(int64_t)k * T] - m;
            adv[(int64_t)b * K * T + (int64_t)k * T + t] = (float)c;
            s1 += c; s2 += c * c;
        }
    }
    s1 = block_sum_f64(s1, red); s2 = block_sum_f64(s2, red);
    if (threadIdx.x == 0) {
        double *o = partial + 2 * ((int64_t)blockIdx.y * gridDim.x + blockIdx.x);
        o[0] = s1; o[1] = s2;
    }
}

// every workgroup folds the partial sums in the same fixed order, then whitens its share
__global__ void __launch_bounds__(RW_BLOCK)
k_reward_whiten(float *__restrict__ adv, const double *__restrict__ partial, int n_partial, int64_t n, float eps)
{
    __shared__ double red[RW_BLOCK / 64];
    double s1 = 0.0, s2 = 0.0;
    for (int i = threadIdx.x; i < n_partial; i += RW_BLOCK) { s1 += partial[2 * i]; s2 += partial[2 * i + 1]; }
    s1 = block_sum_f64(s1, red); s2 = block_sum_f64(s2, red);
    const double mean = s1 / (double)n;
    double var = s2 / (double)n - mean * mean;
    var = var > 0.0 ? var : 0.0;
    const float mu = (float)mean, inv = (float)(1.0 / (sqrt(var) + (double)eps));
    for (int64_t i = (int64_t)blockIdx.x * RW_BLOCK + threadIdx.x; i < n; i += (int64_t)gridDim.x * RW_BLOCK)
        adv[i] = (adv[i] - mu) * inv;
}

size_t reward_scratch_bytes(int B, int T) { return (size_t)B * ((T + RW_BLOCK - 1) / RW_BLOCK) * 2 * sizeof(double) + 64; }

void launch_reward(const float *nll, const int32_t *ids, const ActionDev *table, int n_actions, const int32_t *eff,
                   const float *targets, const RewardCfg &rc, int B, int K, int T, float *avg_out, float *pen_out,
                   float *ret_out, float *signal, float *adv, void *scratch, int *flags, hipStream_t st)
{
    if ((int64_t)B * K * T <= 0) return;
    double *partial = (double *)scratch;
    const int tb = (T + RW_BLOCK - 1) / RW_BLOCK;
    hipLaunchKernelGGL(k_reward_rows, dim3(K, B), dim3(RW_BLOCK), 0, st, nll, ids, table, n_actions, eff, targets, rc, K, T,
                       avg_out, pen_out, ret_out, signal, flags);
    hipLaunchKernelGGL(k_reward_center, dim3(tb, B), dim3(RW_BLOCK), 0, st, signal, K, T, adv, partial);
    const int64_t n = (int64_t)B * K * T;
    int grid = (int)((n + RW_BLOCK * 4 - 1) / (RW_BLOCK * 4));
    grid = grid < 1 ? 1 : (grid > 1024 ? 1024 : grid);
    hipLaunchKernelGGL(k_reward_whiten, dim3(grid), dim3(RW_BLOCK), 0, st, adv, partial, tb * B, n, rc.eps);
}

}  // namespace sol
