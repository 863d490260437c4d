// Rewards of the two stages and their online normalisation, computed on the device so that a batch
// of verifier outcomes can go straight into the value update.
//   Stage 1 (Sec. 3.3): +1 if the candidate is feasible, -1 otherwise.
//   Stage 2 (Sec. 3.4): -1 if infeasible, else tanh(log b - log l), b the best latency so far, l the
//   measured one (App. A: tanh(log rho), rho the speed-up ratio).
//   Normalisation (Sec. 3.4, App. A "Stability of Online Normalization"): sample t becomes
//   (r_t - mu_{t-1}) / max(sigma_{t-1}, sigma_min), optionally clipped, with mu, sigma the running
//   mean and population deviation of the raw rewards BEFORE it; the statistics (count, sum, sum of
//   squares, fp64) persist in the handle's workspace.
// The dependence of sample t on all earlier ones is a prefix sum: one workgroup walks the batch in
// pieces of 1024 samples, scans (r, r^2) within the piece (wavefront shuffles, then the 16 wavefront
// totals) and carries the totals to the next piece.  All arithmetic in fp64; outputs fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evk {

__device__ __forceinline__ double wave_inclusive_sum_d(double x, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double y = __shfl_up(x, o, 64);
        if (lane >= o) x += y;
    }
    return x;
}

__global__ __launch_bounds__(1024) void k_shape_rewards(int stage, const unsigned char* __restrict__ feasible,
                                                        const float* __restrict__ latency, const float* __restrict__ best,
                                                        int64_t M, int normalise, double sigma_min, double clip,
                                                        double* __restrict__ state, float* __restrict__ out) {
    __shared__ double wave_s[16], wave_q[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double n0 = state[0], s0 = state[1], q0 = state[2];          // statistics before the current piece
    for (int64_t base = 0; base < M; base += 1024) {
        const int64_t j = base + tid;
        const bool live = j < M;
        double raw = 0.0;
        if (live) {
            if (!feasible[j]) raw = -1.0;
            else if (stage == 0) raw = 1.0;
            else raw = tanh(log((double)best[j]) - log((double)latency[j]));
        }
        double r = raw;
        if (normalise) {                                             // uniform
            const double is = wave_inclusive_sum_d(raw, lane), iq = wave_inclusive_sum_d(raw * raw, lane);
            if (lane == 63) { wave_s[wave] = is; wave_q[wave] = iq; }
            __syncthreads();
            double before_s = 0.0, before_q = 0.0, piece_s = 0.0, piece_q = 0.0;
#pragma unroll
            for (int w = 0; w < 16; ++w) {
                if (w < wave) { before_s += wave_s[w]; before_q += wave_q[w]; }
                piece_s += wave_s[w];
                piece_q += wave_q[w];
            }
            __syncthreads();
            const double n = n0 + (double)tid;                       // samples before this one
            const double sum = s0 + before_s + (is - raw), sq = q0 + before_q + (iq - raw * raw);
            const double mu = n > 0.0 ? sum / n : 0.0;
            const double var = n > 0.0 ? sq / n - mu * mu : 0.0;
            const double sigma = var > 0.0 ? sqrt(var) : 0.0;
            r = (raw - mu) / (sigma > sigma_min ? sigma : sigma_min);
            if (clip > 0.0) r = r > clip ? clip : (r < -clip ? -clip : r);
            const int64_t left = M - base;
            n0 += (double)(left < 1024 ? left : 1024);
            s0 += piece_s;
            q0 += piece_q;
        }
        if (live) out[j] = (float)r;
    }
    if (normalise && tid == 0) { state[0] = n0; state[1] = s0; state[2] = q0; }
}

}  // namespace evk
