// Sequence-level step that follows the row path: per-token importance weights
// pi_train^mp / pi_infer^mp from the two sides' constrained log-probabilities
// (App. A, protocol item 4: the log-probabilities are formed independently and
// their difference is exponentiated), the cumulative log mismatch Delta_y of
// every sampled sequence (Thm. 4.1) and the token veto (App. A, item 5: a
// sequence with a token of weight below the threshold is discarded).
//
// A segmented reduction over [N] with sequence offsets: one workgroup per
// sequence, sums in double precision in a fixed order (run-to-run identical).
#include "dvp_device.h"
#include "dvp_internal.h"

namespace dvp {

constexpr int kSeqThreads = 1024;

__global__ __launch_bounds__(kSeqThreads) void sequence_kernel(const SequenceArgs a)
{
    constexpr int NW = kSeqThreads / kWave;
    __shared__ double lds_sum[NW];
    __shared__ float lds_min[NW];
    __shared__ int lds_flag[2 * NW];
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    int64_t t0 = a.offsets[s], t1 = a.offsets[s + 1];
    // offsets live in device memory and cannot be checked by the host: tokens outside [0, N) are ignored
    if (t0 < 0) t0 = 0;
    if (t1 > a.n_tokens) t1 = a.n_tokens;

    double sum = 0.0;
    float wmin = INFINITY;
    int veto = 0, saw_nan = 0;
    for (int64_t t = t0 + tid; t < t1; t += kSeqThreads) {
        const float lt = a.logp_train[t], li = a.logp_infer[t];
        // a token with zero constrained training probability has weight zero (Sec. 5.3), whatever li is
        const float l = (lt == -INFINITY) ? -INFINITY : lt - li;      // one fp32 rounding
        const float w = __expf(l);
        if (a.weight) a.weight[t] = w;
        sum += (double)l;
        if (w != w) saw_nan = 1; else wmin = fminf(wmin, w);
        // w < threshold, decided in log space on the fp32 difference; NaN and +inf veto as well
        if (l < a.log_threshold || l != l || l == INFINITY) veto = 1;
    }
    // wavefront, then workgroup reduction in a fixed order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        sum += __shfl_xor(sum, off, kWave);
        wmin = fminf(wmin, __shfl_xor(wmin, off, kWave));
        veto |= __shfl_xor(veto, off, kWave);
        saw_nan |= __shfl_xor(saw_nan, off, kWave);
    }
    if ((tid & (kWave - 1)) == 0) {
        const int w = tid / kWave;
        lds_sum[w] = sum; lds_min[w] = wmin; lds_flag[w] = veto; lds_flag[NW + w] = saw_nan;
    }
    __syncthreads();
    if (tid == 0) {
        double tot = lds_sum[0];
        float mn = lds_min[0];
        int v = lds_flag[0], nn = lds_flag[NW];
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            tot += lds_sum[w]; mn = fminf(mn, lds_min[w]); v |= lds_flag[w]; nn |= lds_flag[NW + w];
        }
        a.seq_log_ratio[s] = (float)tot;
        if (a.seq_min_weight) a.seq_min_weight[s] = nn ? __uint_as_float(0x7fc00000u) : mn;
        a.seq_veto[s] = (uint8_t)v;
    }
}

hipError_t launch_sequences(const SequenceArgs &a, hipStream_t stream)
{
    if (a.n_seq == 0) return hipSuccess;
    const int64_t max_grid = 0x7fffffff;
    for (int64_t s0 = 0; s0 < a.n_seq; s0 += max_grid) {
        SequenceArgs b = a;
        b.n_seq = a.n_seq - s0 < max_grid ? a.n_seq - s0 : max_grid;
        b.offsets = a.offsets + s0;
        b.seq_log_ratio = a.seq_log_ratio + s0;
        b.seq_min_weight = a.seq_min_weight ? a.seq_min_weight + s0 : nullptr;
        b.seq_veto = a.seq_veto + s0;
        hipLaunchKernelGGL(sequence_kernel, dim3((unsigned)b.n_seq), dim3(kSeqThreads), 0, stream, b);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace dvp
