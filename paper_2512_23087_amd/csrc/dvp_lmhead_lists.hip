// LM-head variant, gradient through per-row lists (Prop. 5.4: dz is zero outside
// the safe set, so a row with a short safe set has a short gradient).
//
// Pass B's epilogue has appended every safe token of a row to that row's list in
// arrival order, with exp(z - m).  Here each list is sorted by token and turned
// into gradient entries, dH = dz W is summed per row in token order, the lists
// are copied into column-major order (a counting sort whose positions do not
// depend on the launch order) and dW = dz^T H is summed per token in row order:
// every sum has a fixed order, results are run-to-run identical.  No matrix
// product is involved: the work is |lists| x d multiply-adds.
#include "dvp_lmhead_internal.h"

namespace dvp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr int kWave = 64;

__device__ __forceinline__ void fma8(float (&acc)[8], float v, const u32x4 w)
{
    const uint32_t x[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc[2 * i] += v * __uint_as_float(x[i] << 16);
        acc[2 * i + 1] += v * __uint_as_float(x[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void store8(float *dst, const float (&acc)[8])
{
    *(float4 *)dst = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *(float4 *)(dst + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
}

__device__ __forceinline__ int effective_len(const LmListArgs &a, int row)
{
    return (a.row_flags[row] & DVP_ROW_GRAD_OVERFLOW) ? 0 : a.grad_len[row];
}

// One workgroup per token row: flags and length, the list sorted by token, values turned into dz,
// and the row of dH.
__global__ __launch_bounds__(kThreads) void lm_lists_finish_kernel(const LmListArgs a)
{
    __shared__ unsigned long long key[kLmListMax];
    __shared__ uint32_t tok[kLmListMax];
    __shared__ float val[kLmListMax];
    const int i = blockIdx.x, tid = threadIdx.x;
    const int c = a.safe_count[i];
    const uint32_t fl = a.row_flags[i];
    const bool y_safe = (fl & DVP_ROW_Y_IN_TRAIN_SAFE) != 0;
    const bool overflow = y_safe && c > a.list_cap;
    const int len = (y_safe && !overflow) ? c : 0;     // <= list_cap <= kLmListMax
    if (tid == 0) {
        a.grad_len[i] = y_safe ? c : 0;
        if (overflow) a.row_flags[i] = (uint8_t)(fl | DVP_ROW_GRAD_OVERFLOW);
    }
    float *dh = a.d_hidden + (int64_t)i * a.ld_h;
    if (len == 0) {                                    // zero gradient, or left to the caller
        const float zero[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        for (int j0 = tid * 8; j0 < a.d; j0 += kThreads * 8) store8(dh + j0, zero);
        return;
    }
    dvp_grad_entry *list = a.entries + (int64_t)i * a.list_cap;
    int pow2 = 1;
    while (pow2 < len) pow2 <<= 1;
    for (int p = tid; p < pow2; p += kThreads) {
        unsigned long long k = ~0ull;
        if (p < len) k = ((unsigned long long)list[p].index << 32) | (unsigned long long)__float_as_uint(list[p].value);
        key[p] = k;
    }
    for (int k = 2; k <= pow2; k <<= 1) {              // bitonic sort, ascending
        for (int j = k >> 1; j > 0; j >>= 1) {
            __syncthreads();
            for (int p = tid; p < pow2; p += kThreads) {
                const int q = p ^ j;
                if (q > p) {
                    const unsigned long long x = key[p], y = key[q];
                    const bool up = (p & k) == 0;
                    if ((x > y) == up) { key[p] = y; key[q] = x; }
                }
            }
        }
    }
    __syncthreads();
    const uint32_t y = (uint32_t)a.ids[i];             // in range: the row's sampled token is safe
    const float qy = a.coef[i], s = a.scale[i];
    for (int p = tid; p < len; p += kThreads) {
        const uint32_t t = (uint32_t)(key[p] >> 32);
        const float e = __uint_as_float((uint32_t)key[p]);
        const float g = t == y ? qy : s * e;           // Prop. 5.4, the sampled token's entry formed as c (1 - p_y)
        tok[p] = t; val[p] = g;
        list[p].index = t; list[p].value = g;
    }
    __syncthreads();
    for (int j0 = tid * 8; j0 < a.d; j0 += kThreads * 8) {
        float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        for (int p = 0; p < len; ++p)
            fma8(acc, val[p], *(const u32x4 *)(a.W + (int64_t)tok[p] * a.ld_w + j0));
        store8(dh + j0, acc);
    }
}

__global__ void lm_zero_i32_kernel(int32_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// blk_cnt[b][t] = number of rows of row block b whose list holds token t
__global__ __launch_bounds__(kThreads) void lm_csc_count_kernel(const LmListArgs a)
{
    const int b = blockIdx.x, wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int r0 = b * a.rows_per_blk;
    const int r1 = (r0 + a.rows_per_blk) < a.n ? (r0 + a.rows_per_blk) : a.n;
    int32_t *cnt = a.blk_cnt + (int64_t)b * a.v;
    for (int r = r0 + wave; r < r1; r += kThreads / kWave) {
        const int len = effective_len(a, r);
        const dvp_grad_entry *list = a.entries + (int64_t)r * a.list_cap;
        for (int p = lane; p < len; p += kWave) atomicAdd(cnt + list[p].index, 1);
    }
}

// Inclusive scan of one value per thread over a 256-thread workgroup, through LDS.
__device__ __forceinline__ int block_scan_inclusive(int x, int *part, int tid)
{
    part[tid] = x;
    __syncthreads();
    for (int off = 1; off < kThreads; off <<= 1) {
        const int add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    return part[tid];
}

// per token: counts of the row blocks -> exclusive prefix over the blocks; the token's total is scanned
// within the workgroup's 256 tokens (col_start[t] = entries of the workgroup's earlier tokens) and the
// workgroup's total goes to grp_total
__global__ __launch_bounds__(kThreads) void lm_csc_prefix_kernel(const LmListArgs a, int32_t *grp_total)
{
    __shared__ int part[kThreads];
    const int tid = threadIdx.x, t = blockIdx.x * kThreads + tid;
    int run = 0;
    if (t < a.v) {
        for (int b = 0; b < a.n_blk; ++b) {
            int32_t *c = a.blk_cnt + (int64_t)b * a.v + t;
            const int here = *c;
            *c = run;
            run += here;
        }
    }
    const int incl = block_scan_inclusive(run, part, tid);
    if (t < a.v) a.col_start[t] = incl - run;
    if (tid == kThreads - 1) grp_total[blockIdx.x] = incl;
}

// grp_total[0 .. n_grp): totals -> exclusive prefix sums in place, grand total to grp_total[n_grp];
// one workgroup, a contiguous chunk per thread (n_grp = ceil(v / 256) <= 2^14)
__global__ __launch_bounds__(kThreads) void lm_csc_scan_kernel(int32_t *grp_total, int n_grp)
{
    __shared__ int part[kThreads];
    const int tid = threadIdx.x;
    const int per = (n_grp + kThreads - 1) / kThreads;
    const int g0 = tid * per < n_grp ? tid * per : n_grp, g1 = (g0 + per) < n_grp ? (g0 + per) : n_grp;
    int sum = 0;
    for (int g = g0; g < g1; ++g) sum += grp_total[g];
    const int incl = block_scan_inclusive(sum, part, tid);
    int run = incl - sum;
    for (int g = g0; g < g1; ++g) {
        const int here = grp_total[g];
        grp_total[g] = run;
        run += here;
    }
    if (tid == kThreads - 1) grp_total[n_grp] = incl;
}

// col_start[t] += entries of the earlier workgroups' tokens; col_start[v] = all entries
__global__ __launch_bounds__(kThreads) void lm_csc_offset_kernel(int32_t *col_start, const int32_t *grp_total, int v, int n_grp)
{
    const int t = blockIdx.x * kThreads + threadIdx.x;
    if (t < v) col_start[t] += grp_total[blockIdx.x];
    if (t == v) col_start[v] = grp_total[n_grp];
}

// One wavefront per row block walks its rows in order; entry (r, t) goes to position
// col_start[t] + (rows before r that hold t): earlier blocks from the prefix, earlier rows of this
// block from the running counter, which only this wavefront touches.
__global__ __launch_bounds__(kWave) void lm_csc_fill_kernel(const LmListArgs a)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int r0 = b * a.rows_per_blk;
    const int r1 = (r0 + a.rows_per_blk) < a.n ? (r0 + a.rows_per_blk) : a.n;
    int32_t *cnt = a.blk_cnt + (int64_t)b * a.v;
    for (int r = r0; r < r1; ++r) {
        const int len = effective_len(a, r);
        const dvp_grad_entry *list = a.entries + (int64_t)r * a.list_cap;
        for (int p = lane; p < len; p += kWave) {       // tokens of one row are distinct
            const dvp_grad_entry e = list[p];
            const int pos = a.col_start[e.index] + atomicAdd(cnt + e.index, 1);
            a.csc_row[pos] = r;
            a.csc_val[pos] = e.value;
        }
    }
}

// One workgroup per token: dW[t, :] = sum over the token's entries, in row order, of dz * H[row, :]
__global__ __launch_bounds__(kThreads) void lm_dw_gather_kernel(const LmListArgs a)
{
    const int t = blockIdx.x, tid = threadIdx.x;
    const int q0 = a.col_start[t], q1 = a.col_start[t + 1];
    float *dw = a.d_w + (int64_t)t * a.ld_w;
    for (int j0 = tid * 8; j0 < a.d; j0 += kThreads * 8) {
        float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        for (int q = q0; q < q1; ++q)
            fma8(acc, a.csc_val[q], *(const u32x4 *)(a.H + (int64_t)a.csc_row[q] * a.ld_h + j0));
        store8(dw + j0, acc);
    }
}

// zy_low[i]: a value below the logit of row i's sampled token as the matrix cores will form it, hence
// below the row maximum.  The two are the same dot product of exactly representable terms summed in fp32
// in different orders: each is within K 2^-24 sum|terms| of the exact value (K terms), so twice that, plus a
// relative 2^-20 for the scale of an 8-bit engine, is taken off.  One wavefront per row.
template <bool BYTES>
__global__ __launch_bounds__(kWave) void lm_zy_low_kernel(const uint16_t *H, int64_t ld_h, const uint16_t *W, int64_t ld_w,
                                                          const int64_t *ids, float *zy_low, int d, int v, float scale8)
{
    const int i = blockIdx.x, lane = threadIdx.x;
    const int64_t y = ids[i];
    if (y < 0 || y >= (int64_t)v) {
        if (lane == 0) zy_low[i] = -INFINITY;
        return;
    }
    const uint16_t *h = H + (int64_t)i * ld_h, *w = W + y * ld_w;
    float acc = 0.0f, mag = 0.0f;     // the dot product and the sum of its terms' magnitudes
    for (int j0 = lane * 8; j0 < d; j0 += kWave * 8) {
        const u32x4 a = *(const u32x4 *)(h + j0), b = *(const u32x4 *)(w + j0);
        const uint32_t x[4] = {a.x, a.y, a.z, a.w}, u[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if constexpr (BYTES) {      // four E4M3 codes per word, widened exactly by the hardware converter
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                const f32x2 xl = __builtin_amdgcn_cvt_pk_f32_fp8((int)x[k], false), xh = __builtin_amdgcn_cvt_pk_f32_fp8((int)x[k], true);
                const f32x2 ul = __builtin_amdgcn_cvt_pk_f32_fp8((int)u[k], false), uh = __builtin_amdgcn_cvt_pk_f32_fp8((int)u[k], true);
                const float t[4] = {xl.x * ul.x, xl.y * ul.y, xh.x * uh.x, xh.y * uh.y};
#pragma unroll
                for (int q = 0; q < 4; ++q) { acc += t[q]; mag += fabsf(t[q]); }
            } else {
                const float t0 = __uint_as_float(x[k] << 16) * __uint_as_float(u[k] << 16);
                const float t1 = __uint_as_float(x[k] & 0xffff0000u) * __uint_as_float(u[k] & 0xffff0000u);
                acc += t0; acc += t1;
                mag += fabsf(t0) + fabsf(t1);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        acc += __shfl_xor(acc, off, kWave);
        mag += __shfl_xor(mag, off, kWave);
    }
    const float terms = (float)(BYTES ? 2 * d : d);
    float low = acc - 0x1p-23f * terms * mag;
    if constexpr (BYTES) low = low * scale8 - 0x1p-20f * fabsf(low * scale8);
    if (lane == 0) zy_low[i] = low - 1e-6f;
}

// One workgroup per token row: the candidates at or above the final threshold are the safe set.
// Sorted by token, so the sum has a fixed order whatever the arrival order was.
__global__ __launch_bounds__(kThreads) void lm_candidates_finish_kernel(const LmCandArgs a)
{
    __shared__ unsigned long long key[kLmCandMax];
    __shared__ float part[kThreads];
    __shared__ int n_safe;
    const int i = blockIdx.x, tid = threadIdx.x;
    const int nc = a.cand_count[i];
    // The candidates are a superset of the safe set only if the bound they were collected with really
    // lies at or below the sampled token's logit as the matrix cores delivered it.  It is built to (twice
    // the fp32 accumulation bound below a plain dot product); should it ever fail, the row takes the
    // second pass over its logits like a row with too many candidates, instead of losing safe tokens.
    const int64_t y0 = a.ids[i];
    const bool bound_broken = y0 >= 0 && y0 < (int64_t)a.v && a.zy[i] < a.zy_low[i];
    const bool redo = nc > kLmCandMax || bound_broken;
    if (tid == 0) a.overflow[i] = redo ? 1 : 0;
    if (redo) return;                                  // this row goes through a second pass over its logits
    const float m = a.m[i], tau = a.tau[i];
    const dvp_grad_entry *cand = a.cand + (int64_t)i * kLmCandMax;
    int pow2 = 1;
    while (pow2 < nc) pow2 <<= 1;
    if (tid == 0) n_safe = 0;
    int mine = 0;
    for (int p = tid; p < pow2; p += kThreads) {
        unsigned long long k = ~0ull;
        if (p < nc) {
            const dvp_grad_entry e = cand[p];
            if (e.value >= tau) { k = ((unsigned long long)e.index << 32) | (unsigned long long)__float_as_uint(e.value); ++mine; }
        }
        key[p] = k;
    }
    for (int k = 2; k <= pow2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            __syncthreads();
            for (int p = tid; p < pow2; p += kThreads) {
                const int q = p ^ j;
                if (q > p) {
                    const unsigned long long x = key[p], y = key[q];
                    const bool up = (p & k) == 0;
                    if ((x > y) == up) { key[p] = y; key[q] = x; }
                }
            }
        }
    }
    __syncthreads();
    if (mine) atomicAdd(&n_safe, mine);
    __syncthreads();
    const int c = n_safe;                              // the safe tokens are key[0 .. c), by token
    float s = 0.0f;
    for (int p = tid; p < c; p += kThreads) s += __expf(__uint_as_float((uint32_t)key[p]) - m);
    part[tid] = s;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if (tid < off) part[tid] += part[tid + off];
        __syncthreads();
    }
    const float sum = part[0];
    if (a.entries && c <= a.list_cap) {
        dvp_grad_entry *list = a.entries + (int64_t)i * a.list_cap;
        for (int p = tid; p < c; p += kThreads) {
            list[p].index = (uint32_t)(key[p] >> 32);
            list[p].value = __expf(__uint_as_float((uint32_t)key[p]) - m);
        }
    }
    if (tid != 0) return;
    const float log_s = logf(sum);
    const int64_t y = a.ids[i];
    const bool y_ok = y >= 0 && y < (int64_t)a.v;
    const float zy = a.zy[i];
    const bool y_safe = y_ok && zy >= tau;
    if (a.side == 0) {
        const float c_i = !y_safe ? 0.0f : (a.grad_out ? a.grad_out[i] : 0.0f);
        a.coef[i] = c_i != 0.0f ? c_i * (1.0f - __expf(zy - m) / sum) : 0.0f;
        a.scale[i] = -c_i / sum;
    }
    if (a.out.row_max) a.out.row_max[i] = m;
    if (a.out.lse_safe) a.out.lse_safe[i] = m + log_s;
    if (a.out.safe_count) a.out.safe_count[i] = c;
    if (a.out.logp) a.out.logp[i] = !y_ok ? __uint_as_float(0x7fc00000u) : (y_safe ? (zy - m) - log_s : -INFINITY);
    if (a.row_flags) {
        uint32_t fl = a.side == 0 ? (y_ok ? 0u : (uint32_t)DVP_ROW_ID_OUT_OF_RANGE) : a.row_flags[i];
        if (y_safe) fl |= a.side == 0 ? DVP_ROW_Y_IN_TRAIN_SAFE : DVP_ROW_Y_IN_INFER_SAFE;
        a.row_flags[i] = (uint8_t)fl;
    }
}

// One workgroup: the flagged rows in row order (a contiguous chunk of rows per thread, a scan of the
// chunk counts, then each thread writes its chunk's rows).
constexpr int kCompactThreads = 1024;
__global__ __launch_bounds__(kCompactThreads) void lm_subset_compact_kernel(const LmSubsetArgs a)
{
    __shared__ int part[kCompactThreads];
    const int tid = threadIdx.x;
    const int per = (a.n + kCompactThreads - 1) / kCompactThreads;
    const int r0 = tid * per < a.n ? tid * per : a.n, r1 = (r0 + per) < a.n ? (r0 + per) : a.n;
    int cnt = 0;
    for (int r = r0; r < r1; ++r) cnt += a.overflow[r] != 0;
    part[tid] = cnt;
    __syncthreads();
    for (int off = 1; off < kCompactThreads; off <<= 1) {
        const int add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int at = part[tid] - cnt;
    for (int r = r0; r < r1; ++r)
        if (a.overflow[r] != 0) a.rowmap[at++] = r;
    if (tid == kCompactThreads - 1) {
        *a.n_sub = part[tid];
        *a.n_report = part[tid];
    }
}

// One wavefront per position of the subset (launched for every row; positions past the subset exit)
__global__ __launch_bounds__(kWave) void lm_subset_gather_kernel(const LmSubsetArgs a)
{
    const int j = blockIdx.x, lane = threadIdx.x;
    if (j >= *a.n_sub) return;
    const int r = a.rowmap[j];
    const uint16_t *src = a.H + (int64_t)r * a.ld_h;
    uint16_t *dst = a.Hc + (int64_t)j * a.d;
    for (int j0 = lane * 8; j0 < a.d; j0 += kWave * 8) *(u32x4 *)(dst + j0) = *(const u32x4 *)(src + j0);
    if (lane == 0) { a.m_sub[j] = a.m[r]; a.tau_sub[j] = a.tau[r]; }
}

// One wavefront per position of the subset
__global__ __launch_bounds__(kWave) void lm_rows_gather_kernel(const LmRowsArgs a)
{
    const int j = blockIdx.x, lane = threadIdx.x;
    if (a.n_dev && j >= *a.n_dev) return;
    const int r = a.rows[j];
    const bool ok = r >= 0 && r < a.n;
    uint16_t *dst = a.Hc + (int64_t)j * a.d;
    const uint16_t *src = a.H + (int64_t)(ok ? r : 0) * a.ld_h;
    for (int j0 = lane * 8; j0 < a.d; j0 += kWave * 8) *(u32x4 *)(dst + j0) = *(const u32x4 *)(src + j0);
    if (lane == 0) {
        a.ids_c[j] = ok ? a.ids[r] : -1;
        a.g_c[j] = ok ? a.grad_out[r] : 0.0f;
    }
}

__global__ __launch_bounds__(kWave) void lm_rows_scatter_kernel(const LmRowsArgs a)
{
    const int j = blockIdx.x, lane = threadIdx.x;
    if (a.n_dev && j >= *a.n_dev) return;
    const int r = a.rows[j];
    if (r < 0 || r >= a.n) return;
    const float *src = a.dHc + (int64_t)j * a.d;
    float *dst = a.d_hidden + (int64_t)r * a.ld_h;
    for (int j0 = lane * 4; j0 < a.d; j0 += kWave * 4) *(float4 *)(dst + j0) = *(const float4 *)(src + j0);
}

// One workgroup: the rows whose flags meet the mask, in row order (a contiguous chunk of rows per thread, a
// scan of the chunk counts, then each thread writes its chunk's rows); what is left of rows[] becomes -1.
__global__ __launch_bounds__(kCompactThreads) void lm_select_rows_kernel(const uint8_t *row_flags, uint32_t mask, int64_t n,
                                                                         int32_t *rows, int64_t max_rows, int32_t *n_sub,
                                                                         int32_t *n_flagged)
{
    __shared__ int part[kCompactThreads];
    const int tid = threadIdx.x;
    const int64_t per = (n + kCompactThreads - 1) / kCompactThreads;
    const int64_t r0 = tid * per < n ? tid * per : n, r1 = (r0 + per) < n ? (r0 + per) : n;
    int cnt = 0;
    for (int64_t r = r0; r < r1; ++r) cnt += (row_flags[r] & mask) != 0;
    part[tid] = cnt;
    __syncthreads();
    for (int off = 1; off < kCompactThreads; off <<= 1) {
        const int add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    const int total = part[kCompactThreads - 1];
    int64_t pos = part[tid] - cnt;                       // rows flagged before this thread's chunk
    for (int64_t r = r0; r < r1; ++r) {
        if ((row_flags[r] & mask) != 0) {
            if (pos < max_rows) rows[pos] = (int32_t)r;
            ++pos;
        }
    }
    const int64_t used = total < max_rows ? total : max_rows;
    for (int64_t q = used + tid; q < max_rows; q += kCompactThreads) rows[q] = -1;
    if (tid == 0) {
        *n_sub = (int32_t)used;
        if (n_flagged) *n_flagged = total;
    }
}

}  // namespace

hipError_t launch_lmhead_select_rows(const uint8_t *row_flags, uint32_t mask, int64_t n, int32_t *rows, int64_t max_rows,
                                     int32_t *n_sub, int32_t *n_flagged, hipStream_t stream)
{
    hipLaunchKernelGGL(lm_select_rows_kernel, dim3(1), dim3(kCompactThreads), 0, stream, row_flags, mask, n, rows, max_rows,
                       n_sub, n_flagged);
    return hipGetLastError();
}

hipError_t launch_lmhead_rows_gather(const LmRowsArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(lm_rows_gather_kernel, dim3((unsigned)a.n_sub), dim3(kWave), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_lmhead_rows_scatter(const LmRowsArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(lm_rows_scatter_kernel, dim3((unsigned)a.n_sub), dim3(kWave), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_lmhead_subset(const LmSubsetArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(lm_subset_compact_kernel, dim3(1), dim3(kCompactThreads), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lm_subset_gather_kernel, dim3((unsigned)a.n), dim3(kWave), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_lmhead_zy_low(const uint16_t *H, int64_t ld_h, const uint16_t *W, int64_t ld_w, const int64_t *ids,
                                float *zy_low, int n, int d, int v, float scale8, hipStream_t stream)
{
    if (scale8 > 0.0f)
        hipLaunchKernelGGL(lm_zy_low_kernel<true>, dim3((unsigned)n), dim3(kWave), 0, stream, H, ld_h, W, ld_w, ids, zy_low, d, v, scale8);
    else
        hipLaunchKernelGGL(lm_zy_low_kernel<false>, dim3((unsigned)n), dim3(kWave), 0, stream, H, ld_h, W, ld_w, ids, zy_low, d, v, 0.0f);
    return hipGetLastError();
}

hipError_t launch_lmhead_candidates_finish(const LmCandArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(lm_candidates_finish_kernel, dim3((unsigned)a.n), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_lmhead_lists_backward(const LmListArgs &a, hipStream_t stream)
{
#define DVP_LAUNCHED() do { hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return e_; } while (0)
    hipLaunchKernelGGL(lm_lists_finish_kernel, dim3((unsigned)a.n), dim3(kThreads), 0, stream, a);
    DVP_LAUNCHED();
    const int64_t cells = (int64_t)a.n_blk * a.v;
    const int64_t zero_grid = (cells + 256 * 16 - 1) / (256 * 16);
    hipLaunchKernelGGL(lm_zero_i32_kernel, dim3((unsigned)(zero_grid < 4096 ? (zero_grid < 1 ? 1 : zero_grid) : 4096)), dim3(256),
                       0, stream, a.blk_cnt, cells);
    DVP_LAUNCHED();
    hipLaunchKernelGGL(lm_csc_count_kernel, dim3((unsigned)a.n_blk), dim3(kThreads), 0, stream, a);
    DVP_LAUNCHED();
    const int n_grp = (a.v + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(lm_csc_prefix_kernel, dim3((unsigned)n_grp), dim3(kThreads), 0, stream, a, a.grp_total);
    DVP_LAUNCHED();
    hipLaunchKernelGGL(lm_csc_scan_kernel, dim3(1), dim3(kThreads), 0, stream, a.grp_total, n_grp);
    DVP_LAUNCHED();
    hipLaunchKernelGGL(lm_csc_offset_kernel, dim3((unsigned)(a.v / kThreads + 1)), dim3(kThreads), 0, stream, a.col_start,
                       (const int32_t *)a.grp_total, a.v, n_grp);
    DVP_LAUNCHED();
    hipLaunchKernelGGL(lm_csc_fill_kernel, dim3((unsigned)a.n_blk), dim3(kWave), 0, stream, a);
    DVP_LAUNCHED();
    hipLaunchKernelGGL(lm_dw_gather_kernel, dim3((unsigned)a.v), dim3(kThreads), 0, stream, a);
    DVP_LAUNCHED();
#undef DVP_LAUNCHED
    return hipSuccess;
}

}  // namespace dvp
