// Row kernels of the DVP hot path for gfx950.
//
// Per token row (Def. 5.1, Def. 5.2, Prop. 5.4 of the paper):
//   m = max_k z_k;  tau = fl32(m + log_rho);  safe_k = [z_k >= tau];
//   S = sum_{safe} exp(z_k - m);  lse_safe = m + log S;
//   logp = (z_y - m) - log S  (or -inf when y is pruned);
//   dz_k = g * (delta_ky - exp((z_k - m) - log S)) on the safe set, 0 elsewhere.
//
// Membership needs the final row maximum, so a row has to be looked at twice.
// The resident kernel keeps the whole row in the workgroup's vector registers
// (one V = 151936 bf16 row is 297 KB; a CU's register file is 512 KB) so HBM
// sees every logit once; the streaming kernel re-reads the row per phase and
// takes any shape or alignment.
#include "dvp_device.h"
#include "dvp_internal.h"

namespace dvp {

// ---------------------------------------------------------------------------
// resident kernel: NT threads hold NV 16-byte vectors each
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ u32x4 load_tail_vector(const T *p, int n_valid)
{
    // fewer than one vector of valid elements at the end of a row: fetch them
    // one by one and fill the rest with -inf
    constexpr int EPV = elem_traits<T>::kPerVec;
    float x[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) x[e] = (e < n_valid) ? load_elem(p + e) : -INFINITY;
    if constexpr (EPV == 4) {
        return pack(x, float());
    } else {
        u32x4 v;   // exact: the values are bf16 already, truncation keeps them
        v.x = (float_to_bits(x[0]) >> 16) | (float_to_bits(x[1]) & 0xffff0000u);
        v.y = (float_to_bits(x[2]) >> 16) | (float_to_bits(x[3]) & 0xffff0000u);
        v.z = (float_to_bits(x[4]) >> 16) | (float_to_bits(x[5]) & 0xffff0000u);
        v.w = (float_to_bits(x[6]) >> 16) | (float_to_bits(x[7]) & 0xffff0000u);
        return v;
    }
}

// Compiler fences with no run-time cost.  The row lives in registers across
// three phases; without them the optimiser keeps every phase's unpacked copy
// of the row (and every per-vector index and predicate) alive from one phase
// to the next, which overflows the register file.
__device__ __forceinline__ void keep_packed(u32x4 &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ int fresh(int v) { asm volatile("" : "+v"(v)); return v; }

template <typename T, int NV, int NT, int MINW>
__global__ __launch_bounds__(NT, MINW) void rows_resident_kernel(const RowArgs a)
{
    using TR = elem_traits<T>;
    constexpr int EPV = TR::kPerVec;
    constexpr int NW = NT / kWave;
    __shared__ float lds_max[NW];
    __shared__ float lds_f[2 * NW];
    __shared__ int lds_i[NW];

    const int tid = threadIdx.x;
    const int V = a.vocab;
    const int nvec = V / EPV;              // whole vectors in a row
    const int tail = V - nvec * EPV;       // elements in the ragged last vector
    const int nfull = nvec / NT;           // register slots that hold a whole vector in every thread
    const float log_rho = a.log_rho;
    const bool want_bwd = a.grad_out != nullptr;
    const int bits_words = (V + 31) / 32;

    for (int64_t row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        const int64_t y = a.ids[row];
        const bool y_ok = (y >= 0) && (y < (int64_t)V);
        uint32_t flags = y_ok ? 0u : (uint32_t)DVP_ROW_ID_OUT_OF_RANGE;

        for (int side = a.n_sides - 1; side >= 0; --side) {   // inference row first, training row last
            const T *zrow = (const T *)a.z[side] + row * a.ld[side];
            const u32x4 *zvec = (const u32x4 *)zrow;
            const SideOut &out = a.out[side];
            const bool want_full = out.lse_full != nullptr;
            uint8_t *bits_row = out.safe_bits
                ? (uint8_t *)(out.safe_bits + row * (int64_t)bits_words) : nullptr;

            // ---- the row enters the register file: its only trip from HBM.
            // Slots past the end of the row hold -inf: they never win the max,
            // add exp(-inf) = 0 to the sums, and are safe only when tau = -inf.
            u32x4 r[NV];
            {
                const int t = fresh(tid);
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    if (j < nfull) {
                        r[j] = __builtin_nontemporal_load(zvec + (j * NT + t));
                    } else {
                        const int idx = j * NT + t;
                        if (idx < nvec) {
                            r[j] = __builtin_nontemporal_load(zvec + idx);
                        } else if (idx == nvec && tail) {
                            r[j] = load_tail_vector(zrow + (int64_t)nvec * EPV, tail);
                        } else {
                            r[j] = (u32x4){TR::kPadWord, TR::kPadWord, TR::kPadWord, TR::kPadWord};
                        }
                    }
                }
            }
            const float zy = y_ok ? load_elem(zrow + y) : 0.0f;

            // ---- row maximum (Def. 5.1) ----
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                float x[EPV];
                unpack(r[j], x, T());
#pragma unroll
                for (int e = 0; e < EPV; ++e) m = fmaxf(m, x[e]);
            }
            m = block_max<NT>(m, lds_max);
#pragma unroll
            for (int j = 0; j < NV; ++j) keep_packed(r[j]);

            // ---- threshold, membership, size, masked sum (Def. 5.1 / 5.2) ----
            const float tau = m + log_rho;   // one fp32 rounding
            RowSums acc = {0.0f, 0.0f, 0};
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                float x[EPV];
                unpack(r[j], x, T());
                uint32_t mask = 0;
#pragma unroll
                for (int e = 0; e < EPV; ++e) mask |= (x[e] >= tau ? 1u : 0u) << e;
                acc.count += __popc(mask);
                if (want_full) {
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const float ex = __expf(x[e] - m);
                        acc.s_full += ex;
                        acc.s_safe += ((mask >> e) & 1u) ? ex : 0.0f;
                    }
                } else if (__any(mask != 0u)) {   // wavefront-uniform: skip the exps of all-pruned vectors
#pragma unroll
                    for (int e = 0; e < EPV; ++e)
                        acc.s_safe += ((mask >> e) & 1u) ? __expf(x[e] - m) : 0.0f;
                }
                if (bits_row) {
                    const int idx = j * NT + fresh(tid);
                    const uint32_t valid = idx < nvec ? ((1u << EPV) - 1u)
                                                      : (idx == nvec ? (1u << tail) - 1u : 0u);
                    mask &= valid;
                    if constexpr (EPV == 8) {
                        if (idx < 4 * bits_words) bits_row[idx] = (uint8_t)mask;
                    } else {
                        const uint32_t other = __shfl_xor(mask, 1, kWave);
                        if (!(idx & 1) && (idx >> 1) < 4 * bits_words)
                            bits_row[idx >> 1] = (uint8_t)(mask | (other << 4));
                    }
                }
            }
            acc = block_sums<NT>(acc, lds_f, lds_i);
            if (tau == -INFINITY) acc.count = V;   // nothing pruned; do not count the -inf padding

            const float log_s = logf(acc.s_safe);
            const bool y_safe = y_ok && (zy >= tau);
            if (y_safe) flags |= (side == 0 ? DVP_ROW_Y_IN_TRAIN_SAFE : DVP_ROW_Y_IN_INFER_SAFE);
            if (tid == 0) {
                if (out.row_max) out.row_max[row] = m;
                if (out.lse_safe) out.lse_safe[row] = m + log_s;
                if (out.lse_full) out.lse_full[row] = m + logf(acc.s_full);
                if (out.safe_count) out.safe_count[row] = acc.count;
                if (out.logp)
                    out.logp[row] = !y_ok ? __uint_as_float(0x7fc00000u)
                                          : (y_safe ? (zy - m) - log_s : -INFINITY);
            }

            // ---- gradient of the training row (Prop. 5.4), straight from the registers ----
            if (side == 0 && want_bwd) {
                T *dzrow = (T *)a.dz + row * a.ld_grad;
                u32x4 *dzvec = (u32x4 *)dzrow;
                const float g = a.grad_out[row];
                const int t = fresh(tid);
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    keep_packed(r[j]);
                    const int idx = j * NT + t;
                    u32x4 o = {0u, 0u, 0u, 0u};
                    if (y_safe) {
                        float x[EPV];
                        unpack(r[j], x, T());
                        bool any_safe = false;
#pragma unroll
                        for (int e = 0; e < EPV; ++e) any_safe |= (x[e] >= tau);
                        if (__any(any_safe)) {
                            float d[EPV];
                            const int64_t k0 = (int64_t)idx * EPV;
#pragma unroll
                            for (int e = 0; e < EPV; ++e) {
                                const float p = __expf((x[e] - m) - log_s);
                                const float onehot = (k0 + e == y) ? 1.0f : 0.0f;
                                d[e] = (x[e] >= tau) ? g * (onehot - p) : 0.0f;
                            }
                            o = pack(d, T());
                        }
                    }
                    if (j < nfull) {
                        __builtin_nontemporal_store(o, dzvec + idx);
                    } else if (idx < nvec) {
                        __builtin_nontemporal_store(o, dzvec + idx);
                    } else if (idx == nvec && tail) {   // ragged last vector: element stores
                        float d[EPV];
                        unpack(o, d, T());
                        for (int e = 0; e < tail; ++e) store_elem(dzrow + (int64_t)nvec * EPV + e, d[e]);
                    }
                }
            }
        }
        if (tid == 0 && a.row_flags) a.row_flags[row] = (uint8_t)flags;
    }
}

// ---------------------------------------------------------------------------
// streaming kernel: any V, any stride, any alignment; re-reads the row per phase
// ---------------------------------------------------------------------------
template <typename T, int NT>
__global__ __launch_bounds__(NT) void rows_streaming_kernel(const RowArgs a)
{
    constexpr int NW = NT / kWave;
    __shared__ float lds_max[NW];
    __shared__ float lds_f[2 * NW];
    __shared__ int lds_i[NW];

    const int tid = threadIdx.x;
    const int V = a.vocab;
    const int v_round = (V + NT - 1) / NT * NT;
    const float log_rho = a.log_rho;
    const bool want_bwd = a.grad_out != nullptr;
    const int bits_words = (V + 31) / 32;

    for (int64_t row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        const int64_t y = a.ids[row];
        const bool y_ok = (y >= 0) && (y < (int64_t)V);
        uint32_t flags = y_ok ? 0u : (uint32_t)DVP_ROW_ID_OUT_OF_RANGE;

        for (int side = a.n_sides - 1; side >= 0; --side) {
            const T *zrow = (const T *)a.z[side] + row * a.ld[side];
            const SideOut &out = a.out[side];
            const bool want_full = out.lse_full != nullptr;
            uint32_t *bits_row = out.safe_bits ? out.safe_bits + row * (int64_t)bits_words : nullptr;
            const float zy = y_ok ? load_elem(zrow + y) : 0.0f;

            float m = -INFINITY;
            for (int k = tid; k < V; k += NT) m = fmaxf(m, load_elem(zrow + k));
            m = block_max<NT>(m, lds_max);

            const float tau = m + log_rho;
            RowSums acc = {0.0f, 0.0f, 0};
            for (int k = tid; k < v_round; k += NT) {   // uniform trip count: ballot below needs every lane
                const bool in = k < V;
                const float x = in ? load_elem(zrow + k) : -INFINITY;
                const bool safe = in && (x >= tau);
                acc.count += safe ? 1 : 0;
                if (want_full) {
                    const float ex = in ? __expf(x - m) : 0.0f;
                    acc.s_full += ex;
                    acc.s_safe += safe ? ex : 0.0f;
                } else if (safe) {
                    acc.s_safe += __expf(x - m);
                }
                if (bits_row) {
                    const unsigned long long b = __ballot(safe);
                    if ((tid & (kWave - 1)) == 0) {
                        const int w = k >> 5;   // k is a multiple of 64 on lane 0
                        if (w < bits_words) bits_row[w] = (uint32_t)b;
                        if (w + 1 < bits_words) bits_row[w + 1] = (uint32_t)(b >> 32);
                    }
                }
            }
            acc = block_sums<NT>(acc, lds_f, lds_i);

            const float log_s = logf(acc.s_safe);
            const bool y_safe = y_ok && (zy >= tau);
            if (y_safe) flags |= (side == 0 ? DVP_ROW_Y_IN_TRAIN_SAFE : DVP_ROW_Y_IN_INFER_SAFE);
            if (tid == 0) {
                if (out.row_max) out.row_max[row] = m;
                if (out.lse_safe) out.lse_safe[row] = m + log_s;
                if (out.lse_full) out.lse_full[row] = m + logf(acc.s_full);
                if (out.safe_count) out.safe_count[row] = acc.count;
                if (out.logp)
                    out.logp[row] = !y_ok ? __uint_as_float(0x7fc00000u)
                                          : (y_safe ? (zy - m) - log_s : -INFINITY);
            }

            if (side == 0 && want_bwd) {
                T *dzrow = (T *)a.dz + row * a.ld_grad;
                const float g = a.grad_out[row];
                for (int k = tid; k < V; k += NT) {
                    const float x = load_elem(zrow + k);
                    float d = 0.0f;
                    if (y_safe && x >= tau) {
                        const float p = __expf((x - m) - log_s);
                        d = g * (((int64_t)k == y ? 1.0f : 0.0f) - p);
                    }
                    store_elem(dzrow + k, d);
                }
            }
        }
        if (tid == 0 && a.row_flags) a.row_flags[row] = (uint8_t)flags;
    }
}

// ---------------------------------------------------------------------------
// stand-alone backward: one pass over the training row with the forward's
// row_max / lse_safe / flags (Prop. 5.4; the set is a constant of the backward)
// ---------------------------------------------------------------------------
template <typename T, int NT, bool VEC>
__global__ __launch_bounds__(NT) void backward_kernel(const BackwardArgs a)
{
    using TR = elem_traits<T>;
    constexpr int EPV = TR::kPerVec;
    const int tid = threadIdx.x;
    const int V = a.vocab;

    for (int64_t row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        const T *zrow = (const T *)a.z + row * a.ld;
        T *dzrow = (T *)a.dz + row * a.ld_grad;
        const float m = a.row_max[row];
        const float log_s = a.lse_safe[row] - m;
        const float tau = m + a.log_rho;      // same fp32 add as the forward
        const float g = a.grad_out[row];
        const int64_t y = a.ids[row];
        const bool y_safe = (a.row_flags[row] & DVP_ROW_Y_IN_TRAIN_SAFE) != 0;
        int k_scalar = 0;
        if constexpr (VEC) {
            const int nvec = V / EPV;
            const u32x4 *zvec = (const u32x4 *)zrow;
            u32x4 *dzvec = (u32x4 *)dzrow;
            const u32x4 zero = {0u, 0u, 0u, 0u};
            const int nvec_round = (nvec + NT - 1) / NT * NT;
            for (int idx = tid; idx < nvec_round; idx += NT) {
                const bool in = idx < nvec;
                u32x4 o = zero;
                if (y_safe) {
                    float x[EPV];
                    const u32x4 v = in ? __builtin_nontemporal_load(zvec + idx)
                                       : (u32x4){TR::kPadWord, TR::kPadWord, TR::kPadWord, TR::kPadWord};
                    unpack(v, x, T());
                    bool any_safe = false;
#pragma unroll
                    for (int e = 0; e < EPV; ++e) any_safe |= (x[e] >= tau);
                    if (__any(any_safe)) {
                        float d[EPV];
                        const int64_t k0 = (int64_t)idx * EPV;
#pragma unroll
                        for (int e = 0; e < EPV; ++e) {
                            const float p = __expf((x[e] - m) - log_s);
                            const float onehot = (k0 + e == y) ? 1.0f : 0.0f;
                            d[e] = (x[e] >= tau) ? g * (onehot - p) : 0.0f;
                        }
                        o = pack(d, T());
                    }
                }
                if (in) __builtin_nontemporal_store(o, dzvec + idx);
            }
            k_scalar = nvec * EPV;
        }
        for (int k = k_scalar + tid; k < V; k += NT) {
            float d = 0.0f;
            if (y_safe) {
                const float x = load_elem(zrow + k);
                if (x >= tau) {
                    const float p = __expf((x - m) - log_s);
                    d = g * (((int64_t)k == y ? 1.0f : 0.0f) - p);
                }
            }
            store_elem(dzrow + k, d);
        }
    }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
static int device_cu_count()
{
    static int cached = 0;
    if (cached == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cached = n;
        else
            return 256;
    }
    return cached;
}

template <typename Kernel>
static int blocks_per_cu(Kernel k, int threads)
{
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k, threads, 0) != hipSuccess || nb < 1) nb = 1;
    return nb;
}

template <typename T, int NV, int NT, int MINW>
static hipError_t launch_resident_inst(const RowArgs &a, hipStream_t stream)
{
    static int per_cu = 0;
    if (per_cu == 0) per_cu = blocks_per_cu(rows_resident_kernel<T, NV, NT, MINW>, NT);
    int64_t grid = (int64_t)device_cu_count() * per_cu;
    if (grid > a.n_rows) grid = a.n_rows;
    hipLaunchKernelGGL((rows_resident_kernel<T, NV, NT, MINW>), dim3((unsigned)grid), dim3(NT), 0, stream, a);
    return hipGetLastError();
}

// vectors per thread the resident kernel is built for: 256-thread groups for
// short rows (several groups share a CU), 1024-thread groups for long rows
// (one group owns the CU's register file)
template <typename T>
static hipError_t launch_resident_t(const RowArgs &a, hipStream_t stream)
{
    const int epv = elem_traits<T>::kPerVec;
    const int64_t slots = ((int64_t)a.vocab + epv - 1) / epv;
    if (slots <= 256 * 4)   return launch_resident_inst<T, 4, 256, 8>(a, stream);
    if (slots <= 256 * 8)   return launch_resident_inst<T, 8, 256, 6>(a, stream);
    if (slots <= 256 * 16)  return launch_resident_inst<T, 16, 256, 4>(a, stream);
    if (slots <= 1024 * 8)  return launch_resident_inst<T, 8, 1024, 4>(a, stream);
    if (slots <= 1024 * 12) return launch_resident_inst<T, 12, 1024, 4>(a, stream);
    if (slots <= 1024 * 16) return launch_resident_inst<T, 16, 1024, 4>(a, stream);
    if (slots <= 1024 * 19) return launch_resident_inst<T, 19, 1024, 4>(a, stream);
    if (slots <= 1024 * 20) return launch_resident_inst<T, 20, 1024, 4>(a, stream);
    return hipErrorInvalidValue;
}

bool row_fits_resident(int dtype, int64_t vocab)
{
    const int epv = dtype == DVP_BF16 ? 8 : 4;
    return (vocab + epv - 1) / epv <= 1024 * 20;
}

hipError_t launch_rows_resident(int dtype, const RowArgs &a, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    return dtype == DVP_BF16 ? launch_resident_t<bf16_t>(a, stream) : launch_resident_t<float>(a, stream);
}

hipError_t launch_rows_streaming(int dtype, const RowArgs &a, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    constexpr int NT = 512;
    int64_t grid = (int64_t)device_cu_count() * 4;
    if (grid > a.n_rows) grid = a.n_rows;
    if (dtype == DVP_BF16)
        hipLaunchKernelGGL((rows_streaming_kernel<bf16_t, NT>), dim3((unsigned)grid), dim3(NT), 0, stream, a);
    else
        hipLaunchKernelGGL((rows_streaming_kernel<float, NT>), dim3((unsigned)grid), dim3(NT), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_backward(int dtype, const BackwardArgs &a, bool vector_ok, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    constexpr int NT = 512;
    int64_t grid = (int64_t)device_cu_count() * 8;
    if (grid > a.n_rows) grid = a.n_rows;
    const dim3 g((unsigned)grid), b(NT);
    if (dtype == DVP_BF16) {
        if (vector_ok) hipLaunchKernelGGL((backward_kernel<bf16_t, NT, true>), g, b, 0, stream, a);
        else           hipLaunchKernelGGL((backward_kernel<bf16_t, NT, false>), g, b, 0, stream, a);
    } else {
        if (vector_ok) hipLaunchKernelGGL((backward_kernel<float, NT, true>), g, b, 0, stream, a);
        else           hipLaunchKernelGGL((backward_kernel<float, NT, false>), g, b, 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace dvp
