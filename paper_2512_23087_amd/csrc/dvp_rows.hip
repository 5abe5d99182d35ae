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
#include <atomic>

#include "dvp_device.h"
#include "dvp_internal.h"

namespace dvp {

// ---------------------------------------------------------------------------
// resident kernel: NT threads hold NV 16-byte vectors each
// ---------------------------------------------------------------------------
// Compiler fences with no run-time cost.  The row lives in registers across
// three phases; without them the optimiser keeps every phase's unpacked copy
// of the row (and every per-slot index and predicate) alive from one phase to
// the next, which overflows the register file.
__device__ __forceinline__ void keep_packed(u32x4 &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ int fresh(int v) { asm volatile("" : "+v"(v)); return v; }
__device__ __forceinline__ bool opaque_true()
{
    int one;
    asm volatile("s_mov_b32 %0, 1" : "=s"(one));
    return one != 0;
}

// Register slot j of thread t holds vector (j * NT + t) of the row.  Slots
// below NVFULL hold a whole vector in every thread of every row the
// instantiation is launched for; the others may lie past the end of the row
// and then hold -inf: they never win the max, add exp(-inf) = 0 to the sums,
// and pass the threshold only when it is -inf itself.
template <typename T, int NT, int NVFULL>
__device__ __forceinline__ u32x4 load_slot(const T *zrow, int j, int t, int nvec)
{
    using TR = elem_traits<T>;
    const u32x4 *zvec = (const u32x4 *)zrow;
    const int idx = j * NT + t;
    if (j < NVFULL) return __builtin_nontemporal_load(zvec + idx);
    // the load runs under the lane mask and lands on top of the padding value:
    // nothing has to wait for it here
    u32x4 v = (u32x4){TR::kPadWord, TR::kPadWord, TR::kPadWord, TR::kPadWord};
    if (idx < nvec) v = __builtin_nontemporal_load(zvec + idx);
    return v;
}

// Unpack part `part` of a slot (a slot is read in kParts pieces so that no
// more than 8 widened elements are live at a time).  Formats with a -inf
// encoding pad the slots past the end of the row with it at load time; 8-bit
// E4M3 has none, so those elements are replaced here (only the slots that can
// lie past the end pay for the test).
template <typename T, int NT, int NVFULL>
__device__ __forceinline__ void unpack_part(const u32x4 v, float (&x)[elem_traits<T>::kPerPart], int part, int j,
                                            int tid, int nvec)
{
    unpack(v, x, part, T());
    if constexpr (!elem_traits<T>::kHasNegInf) {
        if (j >= NVFULL && j * NT + tid >= nvec) {
#pragma unroll
            for (int e = 0; e < elem_traits<T>::kPerPart; ++e) x[e] = -INFINITY;
        }
    }
}

// Single elements fetched ahead of time stay in their stored form until they
// are used: converting right after the load would make the wavefront wait for
// the memory round trip on the spot.
__device__ __forceinline__ uint32_t load_raw(const float *p) { return __float_as_uint(*p); }
__device__ __forceinline__ uint32_t load_raw(const bf16_t *p) { return p->bits; }
__device__ __forceinline__ uint32_t load_raw(const f8_t *p) { return p->bits; }
__device__ __forceinline__ float from_raw(uint32_t u, float) { return __uint_as_float(u); }
__device__ __forceinline__ float from_raw(uint32_t u, bf16_t) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float from_raw(uint32_t u, f8_t)    // bit 8 set: no element here
{
    return (u & 0x100u) ? -INFINITY : e4m3_to_float(u);
}
template <typename T> __device__ __forceinline__ uint32_t raw_neg_inf()
{
    return sizeof(T) == 1 ? 0x100u : (sizeof(T) == 2 ? 0xff80u : 0xff800000u);
}

// Append the (index, value) pairs of the lanes with `take` set to a row's
// list; `counter` is a workgroup-wide cursor in LDS.  Wavefront-uniform call.
__device__ __forceinline__ void list_append(uint2 *list, int *counter, bool take, uint32_t k, float d)
{
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(take);
    if (bal == 0) return;
    int base = 0;
    if ((threadIdx.x & (kWave - 1)) == 0) base = atomicAdd(counter, (int)__builtin_popcountll(bal));
    base = __builtin_amdgcn_readfirstlane(base);
    if (take) {
        const int pos = base + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                              __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
        list[pos] = make_uint2(k, __float_as_uint(d));
    }
}

// gradient values of one vector -> storage format
__device__ __forceinline__ u32x4 pack_grad(const float (&d)[4], float) { return pack(d, float()); }
__device__ __forceinline__ u32x4 pack_grad(const float (&d)[8], bf16_t)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    u32x4 v;   // hardware pack-convert, round to nearest even
    bf16x2 b;
    b = __builtin_convertvector((f32x2){d[0], d[1]}, bf16x2); v.x = __builtin_bit_cast(uint32_t, b);
    b = __builtin_convertvector((f32x2){d[2], d[3]}, bf16x2); v.y = __builtin_bit_cast(uint32_t, b);
    b = __builtin_convertvector((f32x2){d[4], d[5]}, bf16x2); v.z = __builtin_bit_cast(uint32_t, b);
    b = __builtin_convertvector((f32x2){d[6], d[7]}, bf16x2); v.w = __builtin_bit_cast(uint32_t, b);
    return v;
}

// What a workgroup carries from one task (one side of one row) to the next.
struct TaskState {
    int64_t row;
    int side;            // 1 = inference row, 0 = training row
    int64_t y;
    bool y_ok;
    float g;
    uint32_t zy_raw;     // the sampled token's logit (stored form)
    uint32_t xt_raw;     // this thread's element of the ragged end (stored form), or -inf
    uint32_t flags;
    bool dense_hint;     // the task before this one had more safe tokens than a list holds (see NL below)
};

// One task: everything one side of one row needs, from the registers.
//   TS / NVS / NVFULL_S   element type of this task's row, the register slots it
//                         occupies and how many of them are full in every thread
//   TN / NVN / NVFULL_N   the same for the task after it, whose vectors are
//                         loaded into the slots as this task lets go of them
// Returns false after the workgroup's last task.
//   OVF                   the row is longer than the slots hold: vectors from NT * NVS on are
//                         re-read from memory in every phase (all slots are then full, and both
//                         tasks have the same type)
//   NL                    slots of the next row that may be fetched ahead into LDS (lds_pf, NL * NT * 16
//                         bytes): the LAST NL of its slots.  A densely written training row keeps every
//                         register slot until its gradient vector is stored, so without this nothing
//                         could be in flight during its sum phase, and the loads of the next row would
//                         all be issued during the last phase, the last of them right before the next
//                         task needs it.  With it those vectors are copied straight into LDS while the
//                         sum phase runs and move to the registers at the end of the last phase; the
//                         other slots are refilled from memory before them, so every load has been on
//                         its way for a while when the phase ends.  Used when the task before was dense
//                         (for a training row that is the same row's inference side, whose safe set is
//                         about the same); rows with short safe sets free their slots early anyway.
//   ALLSAFE               the build for log_rho = -inf (nothing is pruned: plain log-softmax and its
//                         gradient): every token passes the threshold, so the per-token comparisons,
//                         the counting and the selects are left out (the safe-set size is V)
template <typename TS, int NVS, int NVFULL_S, typename TN, int NVN, int NVFULL_N, int NV, int NT, int EXTRAS,
          bool CAN_BWD, bool OVF = false, int NL = 0, bool ALLSAFE = false>
__device__ __forceinline__ bool row_task(const RowArgs &a, TaskState &s, u32x4 (&r)[NV], float *lds_max,
                                         float *lds_f, int *lds_i, int *lds_list_count, uint8_t *lds_pf = nullptr)
{
    using TR = elem_traits<TS>;
    constexpr int EPV = TR::kPerVec;
    constexpr int EPP = TR::kPerPart;      // elements widened at a time
    constexpr int PARTS = EPV / EPP;
    constexpr int EPV_N = elem_traits<TN>::kPerVec;
    constexpr int NW = NT / kWave;
    static_assert(NVS <= NV && NVN <= NV, "slots");
    static_assert(!CAN_BWD || PARTS == 1, "gradient rows are widened whole");
    static_assert(!OVF || (PARTS == 1 && NVFULL_S == NVS && NVS == NVN), "overflow builds: full slots, one type");
    static_assert(NL <= NVN && (NL == 0 || (!OVF && CAN_BWD && NVS == NVN)), "slots fetched ahead into LDS: rows of one type that fit the registers");
    constexpr int L0 = NVN - NL;           // first slot that can be fetched ahead
    constexpr int FIRST_OVF = NT * NVS;    // first vector that lives outside the registers (OVF)
    constexpr int OVF_BATCH = 4;           // vectors a thread has in flight while it walks that part

    const int tid = threadIdx.x;
    const int V = a.vocab;
    const int nvec = V / EPV;              // whole vectors in this task's row
    const int tail = V - nvec * EPV;       // elements in its ragged end
    const int nvec_n = V / EPV_N;          // the same for the next task's row
    const int tail_n = V - nvec_n * EPV_N;
    const float log_rho = a.log_rho;
    const bool want_bwd = CAN_BWD && a.grad_out != nullptr;
    const int bits_words = (V + 31) / 32;
    const int first_side = a.n_sides - 1;  // inference row first, training row last

    const int64_t row = s.row;
    const int side = s.side;
    const int64_t y = s.y;
    const bool y_ok = s.y_ok;
    const float g = s.g;
    uint32_t flags = s.flags;

    // ---- the task after this one (its loads are issued during this task's last phase) ----
    int64_t nrow = row, ny = y;
    int nside = side - 1;
    if (nside < 0) { nrow = row + gridDim.x; nside = first_side; }
    const bool has_next = nrow < a.n_rows;
    float ng = g;
    if (has_next && nrow != row) {
        ny = a.ids[nrow];
        if (a.grad_out != nullptr) ng = a.grad_out[nrow];
    }
    const bool ny_ok = (ny >= 0) && (ny < (int64_t)V);
    const TN *znext = (const TN *)a.z[has_next ? nside : side] + (has_next ? nrow : row) * a.ld[has_next ? nside : side];
    uint32_t nzy_raw = 0, nxt_raw = raw_neg_inf<TN>();
    const float xt = from_raw(s.xt_raw, TS());
    const float zy = from_raw(s.zy_raw, TS());

    // slots this task's row does not reach are free for the next row from the start
    if constexpr (NVN > NVS) {
        if (has_next) {
#pragma unroll
            for (int j = NVS; j < NVN; ++j) r[j] = load_slot<TN, NT, NVFULL_N>(znext, j, fresh(tid), nvec_n);
        }
    }

    const SideOut &out = a.out[side];
    const bool want_ent = EXTRAS == 2 && out.entropy != nullptr;
    const bool want_full = EXTRAS && (out.lse_full != nullptr || want_ent);   // every exponential is taken
    uint8_t *bits_row = (EXTRAS && out.safe_bits)
        ? (uint8_t *)(out.safe_bits + row * (int64_t)bits_words) : nullptr;
    const bool bwd_here = want_bwd && side == 0;
    // OVF: the part of the row beyond the slots; the vector after the last whole one takes part in the
    // uniform loops when it has to carry the ragged end's membership bits
    const u32x4 *zovf = (const u32x4 *)((const TS *)a.z[side] + row * a.ld[side]) + FIRST_OVF;
    const int novf = OVF ? nvec - FIRST_OVF : 0;
    const int novf_round = (novf + (tail ? 1 : 0) + NT * OVF_BATCH - 1) / (NT * OVF_BATCH) * (NT * OVF_BATCH);
    const u32x4 pad_vec = {TR::kPadWord, TR::kPadWord, TR::kPadWord, TR::kPadWord};

    // ---- row maximum (Def. 5.1) ----
    float m = xt;
#pragma unroll
    for (int j = 0; j < NVS; ++j) {
#pragma unroll
        for (int part = 0; part < PARTS; ++part) {
            float x[EPP];
            unpack_part<TS, NT, NVFULL_S>(r[j], x, part, j, tid, nvec);
#pragma unroll
            for (int e = 0; e < EPP; ++e) m = fmaxf(m, x[e]);
        }
    }
    if constexpr (OVF) {
        for (int q0 = tid; q0 < novf_round; q0 += NT * OVF_BATCH) {
            u32x4 v[OVF_BATCH];
#pragma unroll
            for (int u = 0; u < OVF_BATCH; ++u)    // plain loads: these lines are read again in the next phase
                v[u] = q0 + u * NT < novf ? zovf[q0 + u * NT] : pad_vec;
#pragma unroll
            for (int u = 0; u < OVF_BATCH; ++u) {
                float x[EPV];
                unpack(v[u], x, TS());
#pragma unroll
                for (int e = 0; e < EPV; ++e) m = fmaxf(m, x[e]);
            }
        }
    }
    m = block_max<NT>(m, lds_max);
#pragma unroll
    for (int j = 0; j < NVS; ++j) keep_packed(r[j]);
    // every wavefront is past the previous row's appends (it reached the barrier
    // above) and the next appends come after one more barrier
    if (tid == 0) *lds_list_count = 0;

    // ---- threshold, membership, size, masked sum (Def. 5.1 / 5.2) ----
    const float tau = m + log_rho;   // one fp32 rounding

    float s_safe = 0.0f, s_full = 0.0f;
    float s_ent = 0.0f;              // sum over the safe set of exp(z - m) (z - m): entropy (EXTRAS builds)
    int wave_count = 0;              // wavefront-uniform: lanes are counted with scalar popcounts
    uint32_t any_mask = 0;           // bit j: some lane of this wavefront has a safe token in slot j
    // A training row that is going to be written densely holds every slot until the gradient phase: the
    // next row's first NL vectors per thread start their way into LDS now (workgroup-uniform decision).
    [[maybe_unused]] bool ahead = false;
    if constexpr (NL > 0) {
        // (a task without gradient phase refills its slots during this phase: the same holds for it when
        // the exponentials make the phase long, which is when the row before was dense)
        ahead = !a.sparse_only && has_next && (ALLSAFE || s.dense_hint);
        if (ahead) {
            // this wavefront's earlier reads of these LDS bytes fed registers the max phase has consumed
            const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
            const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds_pf + wave * 1024;
            const uint8_t *src = (const uint8_t *)znext + wave * 1024;
            const uint32_t lane_off = (uint32_t)(fresh(tid) & (kWave - 1)) * 16u;
#pragma unroll
            for (int j = L0; j < NVN; ++j) {
                // (a lane past the end of the row copies nothing; its LDS bytes are not read either)
                if (j < NVFULL_N || j * NT + fresh(tid) < nvec_n)
                    copy16_to_lds(src + (size_t)j * NT * 16, lane_off, lds_base + (j - L0) * NT * 16);
            }
        }
    }
    // slot j of the next row out of LDS (padding where the row has ended, as load_slot gives it)
    [[maybe_unused]] auto take_ahead = [&](int j, int t) {
        u32x4 v = {elem_traits<TN>::kPadWord, elem_traits<TN>::kPadWord, elem_traits<TN>::kPadWord, elem_traits<TN>::kPadWord};
        if (j < NVFULL_N || j * NT + t < nvec_n) v = *(const u32x4 *)(lds_pf + (size_t)(j - L0) * NT * 16 + (size_t)t * 16);
        return v;
    };
    if (has_next) {   // the next task's single elements, fetched early and left in stored form
        if (ny_ok) nzy_raw = load_raw(znext + ny);
        if (tid < tail_n) nxt_raw = load_raw(znext + (int64_t)nvec_n * EPV_N + tid);
    }
    {   // ragged end: one element per thread
        const unsigned long long tail_ballot = __builtin_amdgcn_ballot_w64(xt >= tau);
        wave_count += __builtin_popcountll(tail_ballot);
        if constexpr (EXTRAS != 0 && !OVF) {
            // The ragged end's membership bits travel with the slot after the last whole vector.  A row
            // whose whole vectors fill every slot has no such slot: its last bitmask word then holds the
            // ragged end alone (NT * NVS vectors are a multiple of 32 tokens) and is written from here.
            if (bits_row && tail && nvec == NT * NVS && tid == 0)
                ((uint32_t *)bits_row)[(int64_t)nvec * EPV / 32] = (uint32_t)tail_ballot & ((1u << tail) - 1u);
        }
        const float ex = __expf(xt - m);
        s_safe += (xt >= tau) ? ex : 0.0f;
        if (want_full) s_full += ex;
        if (want_ent && xt >= tau && ex > 0.0f) s_ent += ex * (xt - m);   // 0 log 0 = 0 (also the -inf padding when tau = -inf)
    }
#pragma unroll
    for (int j = 0; j < NVS; ++j) {
        bool any = false;
        uint32_t mask = 0;
#pragma unroll
        for (int part = 0; part < PARTS; ++part) {
            float x[EPP];
            unpack_part<TS, NT, NVFULL_S>(r[j], x, part, j, tid, nvec);
            const int before = wave_count;
            if constexpr (!ALLSAFE) {
#pragma unroll
                for (int e = 0; e < EPP; ++e)
                    wave_count += __builtin_popcountll(__builtin_amdgcn_ballot_w64(x[e] >= tau));
            }
            // (ALLSAFE: always true, but through a scalar register the optimiser cannot see through, so
            // that each slot keeps its own wavefront-uniform branch: as one straight block the 19 slots
            // are widened together and the row no longer fits the registers)
            const bool any_part = ALLSAFE ? opaque_true() : wave_count != before;
            any |= any_part;
            if (want_full) {
#pragma unroll
                for (int e = 0; e < EPP; ++e) {
                    const float ex = __expf(x[e] - m);
                    s_full += ex;
                    s_safe += (x[e] >= tau) ? ex : 0.0f;
                    if (want_ent) s_ent += (x[e] >= tau && ex > 0.0f) ? ex * (x[e] - m) : 0.0f;
                }
            } else if (any_part) {   // wavefront-uniform: all-pruned vectors cost no exp
#pragma unroll
                for (int e = 0; e < EPP; ++e) s_safe += (ALLSAFE || x[e] >= tau) ? __expf(x[e] - m) : 0.0f;
            }
            if (EXTRAS && bits_row) {
                const int idx = j * NT + fresh(tid);
                if (idx == nvec && tail) {   // the slot after the last whole vector carries the ragged end's bits
                    const TS *zrow = (const TS *)a.z[side] + row * a.ld[side] + (int64_t)nvec * EPV;
#pragma unroll
                    for (int e = 0; e < EPP; ++e)
                        x[e] = part * EPP + e < tail ? load_elem(zrow + part * EPP + e) : -INFINITY;
                }
#pragma unroll
                for (int e = 0; e < EPP; ++e) mask |= (x[e] >= tau ? 1u : 0u) << (part * EPP + e);
            }
        }
        if (any) any_mask |= 1u << j;
        if (EXTRAS && bits_row) {
            const int idx = j * NT + fresh(tid);
            mask &= idx < nvec ? ((1u << EPV) - 1u) : (idx == nvec ? (1u << tail) - 1u : 0u);
            if constexpr (EPV == 16) {
                if (idx < 2 * bits_words) ((uint16_t *)bits_row)[idx] = (uint16_t)mask;
            } else if constexpr (EPV == 8) {
                if (idx < 4 * bits_words) bits_row[idx] = (uint8_t)mask;
            } else {
                const uint32_t other = __shfl_xor(mask, 1, kWave);
                if (!(idx & 1) && (idx >> 1) < 4 * bits_words)
                    bits_row[idx >> 1] = (uint8_t)(mask | (other << 4));
            }
        }
        // a slot the gradient phase will not read again (no safe token in this
        // wavefront's part of it) is refilled right away
        if (j < NVN && has_next && (!bwd_here || !any) && !(NL > 0 && ahead && j >= L0))
            r[j] = load_slot<TN, NT, NVFULL_N>(znext, j, fresh(tid), nvec_n);
    }
    if constexpr (NL > 0) {
        if (ahead && !bwd_here) {
            // younger than the copies into LDS are only this loop's refills of the other slots, the last of
            // them issued NL slots of work ago
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int j = L0; j < NVN; ++j) r[j] = take_ahead(j, fresh(tid));
        }
    }
    if constexpr (OVF) {
        for (int q0 = tid; q0 < novf_round; q0 += NT * OVF_BATCH) {   // uniform trip count: the ballots need every lane
            u32x4 v[OVF_BATCH];
#pragma unroll
            for (int u = 0; u < OVF_BATCH; ++u) v[u] = q0 + u * NT < novf ? zovf[q0 + u * NT] : pad_vec;
#pragma unroll
            for (int u = 0; u < OVF_BATCH; ++u) {
                const int idx = FIRST_OVF + q0 + u * NT;
                float x[EPV];
                unpack(v[u], x, TS());
                const int before = wave_count;
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    wave_count += __builtin_popcountll(__builtin_amdgcn_ballot_w64(x[e] >= tau));
                if (want_full) {
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const float ex = __expf(x[e] - m);
                        s_full += ex;
                        s_safe += (x[e] >= tau) ? ex : 0.0f;
                        if (want_ent) s_ent += (x[e] >= tau && ex > 0.0f) ? ex * (x[e] - m) : 0.0f;
                    }
                } else if (wave_count != before) {
#pragma unroll
                    for (int e = 0; e < EPV; ++e) s_safe += (x[e] >= tau) ? __expf(x[e] - m) : 0.0f;
                }
                if (EXTRAS && bits_row) {
                    if (idx == nvec && tail) {
                        const TS *zrow = (const TS *)a.z[side] + row * a.ld[side] + (int64_t)nvec * EPV;
#pragma unroll
                        for (int e = 0; e < EPV; ++e) x[e] = e < tail ? load_elem(zrow + e) : -INFINITY;
                    }
                    uint32_t mask = 0;
#pragma unroll
                    for (int e = 0; e < EPV; ++e) mask |= (x[e] >= tau ? 1u : 0u) << e;
                    mask &= idx < nvec ? ((1u << EPV) - 1u) : (idx == nvec ? (1u << tail) - 1u : 0u);
                    if constexpr (EPV == 8) {
                        if (idx < 4 * bits_words) bits_row[idx] = (uint8_t)mask;
                    } else {
                        const uint32_t other = __shfl_xor(mask, 1, kWave);
                        if (!(idx & 1) && (idx >> 1) < 4 * bits_words)
                            bits_row[idx >> 1] = (uint8_t)(mask | (other << 4));
                    }
                }
            }
        }
    }
    s_safe = wave_sum(s_safe);
    if (want_full) s_full = wave_sum(s_full);
    if (want_ent) s_ent = wave_sum(s_ent);
    if ((tid & (kWave - 1)) == 0) {
        const int w = tid / kWave;
        lds_f[w] = s_safe;
        lds_f[NW + w] = s_full;
        if (EXTRAS == 2) lds_f[2 * NW + w] = s_ent;
        lds_i[w] = wave_count;
    }
    __syncthreads();
    RowSums acc = {lds_f[0], lds_f[NW], lds_i[0]};
    float ent_sum = EXTRAS == 2 ? lds_f[2 * NW] : 0.0f;
#pragma unroll
    for (int w = 1; w < NW; ++w) {   // fixed order: results are run-to-run identical
        acc.s_safe += lds_f[w];
        acc.s_full += lds_f[NW + w];
        if (EXTRAS == 2) ent_sum += lds_f[2 * NW + w];
        acc.count += lds_i[w];
    }
    if (tau == -INFINITY) acc.count = V;   // nothing pruned; do not count the -inf padding

    const float log_s = logf(acc.s_safe);
    const bool y_safe = y_ok && (zy >= tau);
    if (y_safe) flags |= (side == 0 ? DVP_ROW_Y_IN_TRAIN_SAFE : DVP_ROW_Y_IN_INFER_SAFE);
    if (side == 0 && acc.count <= DVP_SHORT_SAFE_SET_MAX) flags |= DVP_ROW_SHORT_SAFE_SET;
    // list-only output: a safe set longer than the list's capacity is reported, not written
    const bool overflow = a.sparse_only && bwd_here && y_safe && acc.count > a.list_cap;
    if (overflow) flags |= DVP_ROW_GRAD_OVERFLOW;
    if (tid == 0) {
        if (bwd_here && a.grad_len) a.grad_len[row] = y_safe ? acc.count : 0;
        if (out.row_max) out.row_max[row] = m;
        if (out.lse_safe) out.lse_safe[row] = m + log_s;
        if (EXTRAS && out.lse_full) out.lse_full[row] = m + logf(acc.s_full);
        // H = -sum pi log pi with log pi = (z - m) - log S  =>  H = log S - (sum e^{z-m} (z-m)) / S
        if (want_ent) out.entropy[row] = log_s - ent_sum / acc.s_safe;
        if (out.safe_count) out.safe_count[row] = acc.count;
        if (out.logp)
            out.logp[row] = !y_ok ? __uint_as_float(0x7fc00000u)
                                  : (y_safe ? (zy - m) - log_s : -INFINITY);
        if (side == 0 && a.row_flags) a.row_flags[row] = (uint8_t)flags;
    }

    // ---- gradient of the training row (Prop. 5.4), straight from the registers.
    // Dense rows are written here.  In split mode a row with a short safe set
    // (or a pruned sampled token: all zero) only leaves its (index, value)
    // pairs at the start of the gradient row; the fill kernel writes the row
    // afterwards, so this kernel's memory traffic stays (almost) read-only.
    if constexpr (CAN_BWD) {
    if (bwd_here) {
        const bool dense_out = !a.sparse_only;
        TS *dzrow = (TS *)a.dz + (dense_out ? row * a.ld_grad : 0);
        u32x4 *dzvec = (u32x4 *)dzrow;
        uint2 *list = dense_out ? (uint2 *)dzrow : (uint2 *)a.dz + row * (int64_t)a.list_cap;
        const bool listed = a.split_grad && !(y_safe && acc.count > a.list_cap);
        const bool grad_row = y_safe && !overflow;     // an overflowing row is only walked to refill its slots
        const float neg_g = -g;
        // exp((x - m) - log S) for a gradient stored as bf16: the exact difference x - m, then one fused
        // multiply-add and one exp2, exp2((x - m) log2(e) - log S log2(e)); rounding the constant moves the
        // result by |log S| 2^-24 relative (log S <= log V), far below half a unit of a bf16 value
        constexpr bool FOLD = sizeof(TS) == 2;
        constexpr float kLog2e = 1.4426950408889634f;
        const float fold_s = -log_s * kLog2e;
        const int t = fresh(tid);
        const int64_t y_slot = grad_row ? (y / EPV) : -1;
        if constexpr (NL > 0) {
            // The copies into LDS were issued a whole sum phase ago and nothing younger is in flight on a
            // dense row (its slots are all still taken): waiting here, before this phase's stores are issued,
            // costs nothing then (a wait further down, where the slots are taken out of LDS, would also wait
            // for those stores).
            if (ahead) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        {   // ragged end
            const int64_t k = (int64_t)nvec * EPV + t;
            const bool safe = grad_row && t < tail && xt >= tau;
            float d = 0.0f;
            if (safe) d = neg_g * __expf((xt - m) - log_s) - (k == y ? neg_g : 0.0f);
            if (listed) list_append(list, lds_list_count, safe, (uint32_t)k, d);
            else if (t < tail && dense_out) store_elem(dzrow + k, d);
        }
#pragma unroll
        for (int j = 0; j < NVS; ++j) {
            const int idx = j * NT + t;
            u32x4 o = {0u, 0u, 0u, 0u};
            if (grad_row && ((any_mask >> j) & 1u)) {   // wavefront-uniform
                float x[EPV], d[EPV];
                keep_packed(r[j]);
                unpack(r[j], x, TS());
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    d[e] = (ALLSAFE || x[e] >= tau) ? neg_g * (FOLD ? __builtin_amdgcn_exp2f(fmaf(x[e] - m, kLog2e, fold_s)) : __expf((x[e] - m) - log_s)) : 0.0f;
                if ((int64_t)idx == y_slot) {          // the sampled token: g * (1 - p)
                    const int ey = (int)(y - (int64_t)idx * EPV);
#pragma unroll
                    for (int e = 0; e < EPV; ++e)
                        if (e == ey) d[e] -= neg_g;
                }
                if (listed) {
                    const bool real = j < NVFULL_S || idx < nvec;   // padding slots pass a -inf threshold
#pragma unroll
                    for (int e = 0; e < EPV; ++e)
                        list_append(list, lds_list_count, real && x[e] >= tau, (uint32_t)(idx * EPV + e), d[e]);
                } else {
                    o = pack_grad(d, TS());
                }
            }
            if (!listed && dense_out && (j < NVFULL_S || idx < nvec)) __builtin_nontemporal_store(o, dzvec + idx);
            if (NL > 0 && ahead && j >= L0) {
                r[j] = take_ahead(j, t);
            } else if (j < NVN && has_next && ((any_mask >> j) & 1u)) {
                r[j] = load_slot<TN, NT, NVFULL_N>(znext, j, t, nvec_n);
            }
        }
        if constexpr (OVF) {
            // the part beyond the slots, read once more; a listed row without gradient has nothing to add
            if (!listed || grad_row) {
                for (int q0 = t; q0 < novf_round; q0 += NT * OVF_BATCH) {
                    u32x4 v[OVF_BATCH];
#pragma unroll
                    for (int u = 0; u < OVF_BATCH; ++u)
                        v[u] = (grad_row && q0 + u * NT < novf) ? zovf[q0 + u * NT] : pad_vec;
#pragma unroll
                    for (int u = 0; u < OVF_BATCH; ++u) {
                        const int idx = FIRST_OVF + q0 + u * NT;
                        const bool in = q0 + u * NT < novf;
                        u32x4 o = {0u, 0u, 0u, 0u};
                        float x[EPV], d[EPV];
                        unpack(v[u], x, TS());
                        bool mine = false;
#pragma unroll
                        for (int e = 0; e < EPV; ++e) mine |= x[e] >= tau;
                        mine &= in && grad_row;                 // (padding passes a -inf threshold)
                        if (__builtin_amdgcn_ballot_w64(mine) != 0) {
#pragma unroll
                            for (int e = 0; e < EPV; ++e)
                                d[e] = (mine && x[e] >= tau) ? neg_g * __expf((x[e] - m) - log_s) : 0.0f;
                            if ((int64_t)idx == y_slot) {
                                const int ey = (int)(y - (int64_t)idx * EPV);
#pragma unroll
                                for (int e = 0; e < EPV; ++e)
                                    if (e == ey) d[e] -= neg_g;
                            }
                            if (listed) {
#pragma unroll
                                for (int e = 0; e < EPV; ++e)
                                    list_append(list, lds_list_count, mine && x[e] >= tau, (uint32_t)(idx * EPV + e), d[e]);
                            } else {
                                o = pack_grad(d, TS());
                            }
                        }
                        if (!listed && dense_out && in) __builtin_nontemporal_store(o, dzvec + idx);
                    }
                }
            }
        }
    }
    }

    if (!has_next) return false;
    if (nrow != row) flags = ny_ok ? 0u : (uint32_t)DVP_ROW_ID_OUT_OF_RANGE;
    s.row = nrow; s.side = nside; s.y = ny; s.y_ok = ny_ok; s.g = ng; s.zy_raw = nzy_raw; s.xt_raw = nxt_raw;
    s.flags = flags;
    s.dense_hint = acc.count > a.list_cap;
    return true;
}

// The workgroup walks a list of tasks: for each of its rows, the inference
// side then the training side.  While the last phase of a task consumes the
// registers, each freed slot is refilled with the next task's vector, so the
// CU keeps loads in flight while it computes.  The ragged end of a row (fewer
// than one vector) is held one element per thread in threads 0..tail-1.
// EXTRAS builds also produce lse_full and the membership bitmask (1), and the entropy on top (2).
// OVF builds take rows longer than the registers hold: the first NT * NV vectors are resident, the rest
// is re-read in every phase (from the last-level cache when the workgroups' rows fit it).
// NL > 0: NL * NT * 16 bytes of dynamic LDS hold vectors of the next row fetched ahead (see row_task).
template <typename T, int NV, int NVFULL, int NT, int MINW, int EXTRAS, bool OVF = false, int NL = 0, bool ALLSAFE = false>
__global__ __launch_bounds__(NT, MINW) void rows_resident_kernel(const RowArgs a)
{
    using TR = elem_traits<T>;
    constexpr int EPV = TR::kPerVec;
    constexpr int NW = NT / kWave;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds_ahead[];
    __shared__ float lds_max[NW];
    __shared__ float lds_f[3 * NW];
    __shared__ int lds_i[NW];
    __shared__ int lds_list_count;

    const int tid = threadIdx.x;
    const int V = a.vocab;
    const int nvec = V / EPV;              // whole vectors in a row (>= 1, checked by the launcher)
    const int tail = V - nvec * EPV;       // elements in the ragged end
    if ((int64_t)blockIdx.x >= a.n_rows) return;

    TaskState s;
    s.row = blockIdx.x;
    s.side = a.n_sides - 1;                // inference row first, training row last
    s.y = a.ids[s.row];
    s.y_ok = (s.y >= 0) && (s.y < (int64_t)V);
    s.g = a.grad_out ? a.grad_out[s.row] : 0.0f;
    s.xt_raw = raw_neg_inf<T>();
    s.zy_raw = 0;
    s.flags = s.y_ok ? 0u : (uint32_t)DVP_ROW_ID_OUT_OF_RANGE;
    s.dense_hint = false;
    u32x4 r[NV];
    {
        const T *zrow = (const T *)a.z[s.side] + s.row * a.ld[s.side];
        const int t = fresh(tid);
#pragma unroll
        for (int j = 0; j < NV; ++j) r[j] = load_slot<T, NT, NVFULL>(zrow, j, t, nvec);
        if (t < tail) s.xt_raw = load_raw(zrow + (int64_t)nvec * EPV + t);
        if (s.y_ok) s.zy_raw = load_raw(zrow + s.y);
    }
    while (row_task<T, NV, NVFULL, T, NV, NVFULL, NV, NT, EXTRAS, true, OVF, NL, ALLSAFE>(a, s, r, lds_max, lds_f, lds_i,
                                                                                         &lds_list_count, lds_ahead)) {}
}

// The same walk when the inference logits are stored as 8-bit E4M3 codes: an
// inference row then takes half the register slots of a training row and half
// the HBM bytes.  Always two sides; tasks alternate between the two types.
template <typename T, int NV, int NVFULL, int NT, int MINW, int EXTRAS>
__global__ __launch_bounds__(NT, MINW) void rows_resident_f8infer_kernel(const RowArgs a)
{
    constexpr int NVI = (NV + 1) / 2, NVFULL_I = NVFULL / 2;
    constexpr int EPV_I = elem_traits<f8_t>::kPerVec;
    constexpr int NW = NT / kWave;
    __shared__ float lds_max[NW];
    __shared__ float lds_f[3 * NW];
    __shared__ int lds_i[NW];
    __shared__ int lds_list_count;

    const int tid = threadIdx.x;
    const int V = a.vocab;
    const int nvec_i = V / EPV_I;
    const int tail_i = V - nvec_i * EPV_I;
    if ((int64_t)blockIdx.x >= a.n_rows) return;

    TaskState s;
    s.row = blockIdx.x;
    s.side = 1;
    s.y = a.ids[s.row];
    s.y_ok = (s.y >= 0) && (s.y < (int64_t)V);
    s.g = a.grad_out ? a.grad_out[s.row] : 0.0f;
    s.xt_raw = raw_neg_inf<f8_t>();
    s.zy_raw = 0;
    s.flags = s.y_ok ? 0u : (uint32_t)DVP_ROW_ID_OUT_OF_RANGE;
    s.dense_hint = false;
    u32x4 r[NV];
    {
        const f8_t *zrow = (const f8_t *)a.z[1] + s.row * a.ld[1];
        const int t = fresh(tid);
#pragma unroll
        for (int j = 0; j < NVI; ++j) r[j] = load_slot<f8_t, NT, NVFULL_I>(zrow, j, t, nvec_i);
        if (t < tail_i) s.xt_raw = load_raw(zrow + (int64_t)nvec_i * EPV_I + t);
        if (s.y_ok) s.zy_raw = load_raw(zrow + s.y);
    }
    for (;;) {
        row_task<f8_t, NVI, NVFULL_I, T, NV, NVFULL, NV, NT, EXTRAS, false>(a, s, r, lds_max, lds_f, lds_i, &lds_list_count);
        if (!row_task<T, NV, NVFULL, f8_t, NVI, NVFULL_I, NV, NT, EXTRAS, true>(a, s, r, lds_max, lds_f, lds_i, &lds_list_count))
            break;
    }
}

// ---------------------------------------------------------------------------
// streaming kernel: any V, any stride, any alignment; re-reads the row per phase
// ---------------------------------------------------------------------------
// TI is the element type of the inference rows (T, or 8-bit E4M3 codes).
template <typename T, typename TI, int NT>
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
            const T *zrow = (const T *)a.z[0] + row * a.ld[0];
            const TI *zrow_i = (const TI *)a.z[1] + (side == 1 ? row * a.ld[1] : 0);
            auto logit = [&](int64_t k) { return side == 1 ? load_elem(zrow_i + k) : load_elem(zrow + k); };
            const SideOut &out = a.out[side];
            const bool want_ent = out.entropy != nullptr;
            const bool want_full = out.lse_full != nullptr || want_ent;
            uint32_t *bits_row = out.safe_bits ? out.safe_bits + row * (int64_t)bits_words : nullptr;
            const float zy = y_ok ? logit(y) : 0.0f;

            float m = -INFINITY;
            for (int k = tid; k < V; k += NT) m = fmaxf(m, logit(k));
            m = block_max<NT>(m, lds_max);

            float tau = m + log_rho;
            if (a.finite_mask) tau = storage_rounded(tau, T());   // both sides share T in that variant
            RowSums acc = {0.0f, 0.0f, 0};
            float s_ent = 0.0f;
            for (int k = tid; k < v_round; k += NT) {   // uniform trip count: ballot below needs every lane
                const bool in = k < V;
                const float x = in ? logit(k) : -INFINITY;
                const bool safe = in && (x >= tau);
                acc.count += safe ? 1 : 0;
                if (want_full) {
                    const float ex = in ? __expf(x - m) : 0.0f;
                    acc.s_full += ex;
                    acc.s_safe += safe ? ex : 0.0f;
                    if (want_ent && safe && ex > 0.0f) s_ent += ex * (x - m);   // 0 log 0 = 0
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
            float ent_sum = 0.0f;
            if (want_ent) {      // workgroup-uniform; lds_max is free again (a barrier has passed since its reads)
                s_ent = wave_sum(s_ent);
                if ((tid & (kWave - 1)) == 0) lds_max[tid / kWave] = s_ent;
                __syncthreads();
#pragma unroll
                for (int w = 0; w < NW; ++w) ent_sum += lds_max[w];
                __syncthreads();
            }

            // Exact rule: log S over the safe set.  Finite-mask variant (Sec. 5.5): every pruned token
            // also counts, with the logit mask_value; sums are rebased to ref = max(m, mask_value).
            float ref = m, log_s = logf(acc.s_safe);
            if (a.finite_mask) {
                ref = fmaxf(m, a.mask_value);
                log_s = logf(acc.s_safe * __expf(m - ref) + (float)(V - acc.count) * __expf(a.mask_value - ref));
            }
            const bool y_safe = y_ok && (zy >= tau);
            if (y_safe) flags |= (side == 0 ? DVP_ROW_Y_IN_TRAIN_SAFE : DVP_ROW_Y_IN_INFER_SAFE);
            if (side == 0 && acc.count <= DVP_SHORT_SAFE_SET_MAX) flags |= DVP_ROW_SHORT_SAFE_SET;
            if (tid == 0) {
                if (out.row_max) out.row_max[row] = m;
                if (out.lse_safe) out.lse_safe[row] = ref + log_s;
                if (out.lse_full) out.lse_full[row] = m + logf(acc.s_full);
                if (want_ent) out.entropy[row] = log_s - ent_sum / acc.s_safe;
                if (out.safe_count) out.safe_count[row] = acc.count;
                if (out.logp) {
                    float lp = y_safe ? (zy - ref) - log_s : -INFINITY;
                    if (a.finite_mask && !y_safe) lp = (a.mask_value - ref) - log_s;   // finite: the mask's own log-prob
                    out.logp[row] = !y_ok ? __uint_as_float(0x7fc00000u) : lp;
                }
            }

            if (side == 0 && want_bwd) {
                T *dzrow = (T *)a.dz + row * a.ld_grad;
                const float g = a.grad_out[row];
                // finite-mask variant: a pruned sampled token still pushes the safe logits down
                const bool grad_row = a.finite_mask ? y_ok : y_safe;
                for (int k = tid; k < V; k += NT) {
                    const float x = load_elem(zrow + k);
                    float d = 0.0f;
                    if (grad_row && x >= tau) {
                        const float p = __expf((x - ref) - log_s);
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
// Which rows the zero kernel writes when the call is split (a.split): the rows without a gradient and
// the rows whose safe set is short.  Both kernels derive it from the same flags.
__device__ __forceinline__ bool backward_has_gradient(const BackwardArgs &a, uint32_t fl)
{
    // "gradient row": the sampled token is safe; in the finite-mask variant, any id in range
    return a.finite_mask ? (fl & DVP_ROW_ID_OUT_OF_RANGE) == 0 : (fl & DVP_ROW_Y_IN_TRAIN_SAFE) != 0;
}
__device__ __forceinline__ bool backward_row_is_zero_filled(const BackwardArgs &a, uint32_t fl)
{
    return a.split && (!backward_has_gradient(a, fl) || (fl & DVP_ROW_SHORT_SAFE_SET) != 0);
}

constexpr int kBwdZeroThreads = 256, kBwdZeroVecs = 1;     // see the zero kernel of the gradient fill
template <typename T, bool VEC>
__global__ __launch_bounds__(kBwdZeroThreads) void backward_zero_kernel(const BackwardArgs a, int chunks_per_row)
{
    constexpr int EPV = elem_traits<T>::kPerVec;
    const int64_t row = blockIdx.x / chunks_per_row;
    const int chunk = blockIdx.x - (int)(row * chunks_per_row);
    if (!backward_row_is_zero_filled(a, a.row_flags[row])) return;
    T *dzrow = (T *)a.dz + row * a.ld_grad;
    const int V = a.vocab;
    if constexpr (VEC) {
        const int nvec = V / EPV;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < kBwdZeroVecs; ++u) {
            const int idx = (chunk * kBwdZeroVecs + u) * kBwdZeroThreads + threadIdx.x;
            if (idx < nvec) __builtin_nontemporal_store(zero, (u32x4 *)dzrow + idx);
        }
        if (chunk == chunks_per_row - 1) {
            const int k = nvec * EPV + threadIdx.x;
            if (k < V) store_elem(dzrow + k, 0.0f);
        }
    } else {
        const int per = kBwdZeroThreads * kBwdZeroVecs * EPV;   // elements per workgroup
        for (int k = chunk * per + threadIdx.x; k < (chunk + 1) * per && k < V; k += kBwdZeroThreads)
            store_elem(dzrow + k, 0.0f);
    }
}

template <typename T, int NT, bool VEC>
__global__ __launch_bounds__(NT) void backward_kernel(const BackwardArgs a)
{
    using TR = elem_traits<T>;
    constexpr int EPV = TR::kPerVec;
    const int tid = threadIdx.x;
    const int V = a.vocab;

    for (int64_t row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        const uint32_t fl = a.row_flags[row];
        if (a.only_flagged && !(fl & a.only_flagged)) continue;   // workgroup-uniform
        const bool y_safe = backward_has_gradient(a, fl);
        const bool zeroed = backward_row_is_zero_filled(a, fl);     // the zero kernel has written this row
        if (zeroed && !y_safe) continue;                            // ... and it has no gradient: not even read
        const T *zrow = (const T *)a.z + row * a.ld;
        T *dzrow = (T *)a.dz + row * a.ld_grad;
        const float m = a.row_max[row];
        const float log_s = a.lse_safe[row] - m;
        float tau = m + a.log_rho;            // same fp32 add as the forward
        if (a.finite_mask) tau = storage_rounded(tau, T());
        const float g = a.grad_out[row];
        const int64_t y = a.ids[row];
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
                bool any_safe = false;
                if (y_safe) {
                    float x[EPV];
                    const u32x4 v = in ? __builtin_nontemporal_load(zvec + idx)
                                       : (u32x4){TR::kPadWord, TR::kPadWord, TR::kPadWord, TR::kPadWord};
                    unpack(v, x, T());
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
                // a zero-filled row takes only the vectors that hold a safe token (a -inf threshold makes the
                // padding lanes pass: they are not in the row)
                if (in && (!zeroed || any_safe)) __builtin_nontemporal_store(o, dzvec + idx);
            }
            k_scalar = nvec * EPV;
        }
        for (int k = k_scalar + tid; k < V; k += NT) {
            float d = 0.0f;
            bool safe = false;
            if (y_safe) {
                const float x = load_elem(zrow + k);
                if (x >= tau) {
                    const float p = __expf((x - m) - log_s);
                    d = g * (((int64_t)k == y ? 1.0f : 0.0f) - p);
                    safe = true;
                }
            }
            if (!zeroed || safe) store_elem(dzrow + k, d);
        }
    }
}

// ---------------------------------------------------------------------------
// gradient fill: finishes the rows the resident kernel left as lists.
//   zero kernel     one workgroup per 4 KB chunk of a row, in memory order:
//                   writes zeros everywhere except over the row's list.  Apart
//                   from two words per chunk it only writes, so HBM sees one
//                   long burst of stores instead of stores mixed into reads.
//   scatter kernel  one workgroup per row: reads the list, zeroes the bytes it
//                   occupied, drops the values in place.
// Shape of the zero kernels (this one, backward_zero_kernel, lists_zero_kernel): 256 threads, one
// nontemporal 16-byte store each.  How fast a write-only kernel drains depends on how its stores are paced,
// not only on how many there are: with 8 small workgroups per CU, each waiting for its row's information
// (about a microsecond) before its single store, stores are issued at about the rate HBM takes them.
// Measured on 32768 x 151936 bf16 (9.96 GB), stand-alone, same row lookup: 256 x 1 nontemporal 1.44 ms
// (6.9 TB/s), 512 x 1 nontemporal 1.55, 1024 x 2 nontemporal 1.67, 1024 x 2 plain stores 1.75 (what this
// kernel used first), 256 x 1 plain stores 2.1; in the fused call 4.56 ms against 4.80 ms.  The price: a
// row the row kernel wrote itself now costs 75 workgroups that look it up and leave instead of 10
// (+3 % on a call whose rows are all dense).
// ---------------------------------------------------------------------------
constexpr int kZeroThreads = 256;
constexpr int kFillVecPerThread = 1;
constexpr int kFillChunk = kZeroThreads * kFillVecPerThread;   // vectors per workgroup
constexpr int kFillThreads = 256;      // scatter kernel

__device__ __forceinline__ bool row_is_listed(const FillArgs &a, int64_t row, int &len)
{
    const bool y_safe = (a.row_flags[row] & DVP_ROW_Y_IN_TRAIN_SAFE) != 0;
    const int count = a.safe_count[row];
    len = y_safe ? count : 0;
    return !(y_safe && count > a.list_cap);     // same test as in the row kernel
}

template <typename T>
__global__ __launch_bounds__(kZeroThreads) void grad_zero_kernel(const FillArgs a, int chunks_per_row)
{
    using TR = elem_traits<T>;
    constexpr int EPV = TR::kPerVec;
    const int64_t row = blockIdx.x / chunks_per_row;
    const int chunk = blockIdx.x - (int)(row * chunks_per_row);
    int len;
    if (!row_is_listed(a, row, len)) return;    // dense row: the row kernel wrote it
    const int V = a.vocab;
    const int nvec = V / EPV;
    const int first = (len * 8 + 15) / 16;      // vectors covered by the list: left to the scatter kernel
    T *dzrow = (T *)a.dz + row * a.ld_grad;
    u32x4 *dzvec = (u32x4 *)dzrow;
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < kFillVecPerThread; ++u) {
        const int idx = chunk * kFillChunk + u * kZeroThreads + threadIdx.x;
        if (idx >= first && idx < nvec) __builtin_nontemporal_store(zero, dzvec + idx);
    }
    if (chunk == chunks_per_row - 1) {          // ragged end of the row (a list never reaches the last 16 bytes)
        const int k = nvec * EPV + threadIdx.x;
        if (k < V) store_elem(dzrow + k, 0.0f);
    }
}

template <typename T>
__global__ __launch_bounds__(kFillThreads) void grad_scatter_kernel(const FillArgs a)
{
    __shared__ uint2 lds_list[kListMax];
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    int len;
    if (!row_is_listed(a, row, len) || len == 0) return;
    T *dzrow = (T *)a.dz + row * a.ld_grad;
    const uint2 *list = (const uint2 *)dzrow;
    for (int i = tid; i < len; i += kFillThreads) lds_list[i] = list[i];
    __syncthreads();                            // the list is in LDS before its bytes are cleared
    // the whole vectors the list touched (the zero kernel skipped exactly these)
    const int stop = (len * 8 + 15) / 16 * elem_traits<T>::kPerVec;
    for (int k = tid; k < stop; k += kFillThreads) store_elem(dzrow + k, 0.0f);
    // the zeros must have reached the L2 before another thread writes a value on top
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int i = tid; i < len; i += kFillThreads) {
        const uint2 e = lds_list[i];
        store_elem(dzrow + e.x, __uint_as_float(e.y));
    }
}

// ---------------------------------------------------------------------------
// dense gradient from lists: dz[i, index] = scale_i * value for row i's entries, zero elsewhere.  Two
// write-only kernels: zeros over every row that has a list (rows flagged as overflowing are left to
// the caller of the launcher), then one workgroup per row drops the scaled values in place.
// ---------------------------------------------------------------------------
constexpr int kListsZeroThreads = 256, kListsZeroVecs = 1;   // see the zero kernel of the gradient fill
template <typename T, bool VEC>
__global__ __launch_bounds__(kListsZeroThreads) void lists_zero_kernel(const ListsArgs a, int chunks_per_row)
{
    constexpr int EPV = elem_traits<T>::kPerVec;
    const int64_t row = blockIdx.x / chunks_per_row;
    const int chunk = blockIdx.x - (int)(row * chunks_per_row);
    if (a.row_flags[row] & DVP_ROW_GRAD_OVERFLOW) return;
    T *dzrow = (T *)a.dz + row * a.ld_grad;
    const int V = a.vocab;
    if constexpr (VEC) {
        const int nvec = V / EPV;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < kListsZeroVecs; ++u) {
            const int idx = (chunk * kListsZeroVecs + u) * kListsZeroThreads + threadIdx.x;
            if (idx < nvec) __builtin_nontemporal_store(zero, (u32x4 *)dzrow + idx);
        }
        if (chunk == chunks_per_row - 1) {
            const int k = nvec * EPV + threadIdx.x;
            if (k < V) store_elem(dzrow + k, 0.0f);
        }
    } else {
        const int per = kListsZeroThreads * kListsZeroVecs * EPV;   // elements per workgroup
        for (int k = chunk * per + threadIdx.x; k < (chunk + 1) * per && k < V; k += kListsZeroThreads)
            store_elem(dzrow + k, 0.0f);
    }
}

constexpr int kListsScatterThreads = 64;
template <typename T>
__global__ __launch_bounds__(kListsScatterThreads) void lists_scatter_kernel(const ListsArgs a)
{
    const int64_t row = blockIdx.x;
    if (a.row_flags[row] & DVP_ROW_GRAD_OVERFLOW) return;
    int len = a.grad_len[row];
    if (len > a.list_cap) len = a.list_cap;
    const uint2 *list = (const uint2 *)a.entries + row * (int64_t)a.list_cap;
    const float g = a.scale ? a.scale[row] : 1.0f;
    T *dzrow = (T *)a.dz + row * a.ld_grad;
    for (int i = threadIdx.x; i < len; i += kListsScatterThreads) {
        const uint2 e = list[i];
        if (e.x < (uint32_t)a.vocab) store_elem(dzrow + e.x, g * __uint_as_float(e.y));
    }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
// Compute units of the first device asked about, cached for the process (and so is the occupancy below):
// the kernels walk their rows from any grid size, so on another device the figure only costs speed.
static std::atomic<int> g_cu_count{0};   // callers may come from several host threads
static hipError_t prepare_cu_count()
{
    int dev = 0, n = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess && n > 0) g_cu_count.store(n, std::memory_order_relaxed);
    return e;
}
static PrepareRegistrar g_cu_count_registrar(&prepare_cu_count);
static int device_cu_count()
{
    if (g_cu_count.load(std::memory_order_relaxed) == 0 && prepare_cu_count() != hipSuccess) return 256;
    const int n = g_cu_count.load(std::memory_order_relaxed);
    return n > 0 ? n : 256;
}

// One build of the resident kernel and how many of its workgroups a CU holds (queried once).
// NOPRUNE: the build for log_rho = -inf.  Every row is then written densely, so it fetches slots of the
// next row ahead into LDS (as many 16 KB slots as the LDS holds beside the reduction scratch; its
// workgroup owns the CU) and leaves the threshold tests out.  The other builds keep the LDS free: on rows
// with short safe sets the fetch-ahead code costs more than it brings (measured: 1.5 % on the row kernel).
template <typename T, bool F8_INFER, int NV, int NVFULL, int NT, int MINW, int EXTRAS, bool OVF, bool NOPRUNE>
struct ResidentBuild {
    typedef void (*Kernel)(const RowArgs);
    static_assert(!NOPRUNE || (!F8_INFER && !OVF && NT == 1024 && EXTRAS == 0), "the no-pruning build");
    static constexpr int NL = NOPRUNE ? (NV < 9 ? NV : 9) : 0;
    static constexpr int kDynLds = NL * NT * 16;
    static Kernel kernel()
    {
        if constexpr (F8_INFER) return rows_resident_f8infer_kernel<T, NV, NVFULL, NT, MINW, EXTRAS>;
        else                    return rows_resident_kernel<T, NV, NVFULL, NT, MINW, EXTRAS, OVF, NL, NOPRUNE>;
    }
    static inline std::atomic<int> per_cu{0};
    static inline std::atomic<uint64_t> configured{0};   // bit d: device d allows this build its dynamic LDS
    static hipError_t prepare()
    {
        if (kDynLds > 0) {      // more than 64 KB of LDS per workgroup has to be asked for, once per device
            int dev = 0;
            hipError_t e = hipGetDevice(&dev);
            if (e == hipSuccess) e = hipFuncSetAttribute((const void *)kernel(), hipFuncAttributeMaxDynamicSharedMemorySize, kDynLds);
            if (e != hipSuccess) return e;
            if (dev >= 0 && dev < 64) configured.fetch_or(1ull << dev, std::memory_order_release);
        }
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel(), NT, kDynLds) != hipSuccess || nb < 1) nb = 1;
        per_cu.store(nb, std::memory_order_relaxed);
        return hipSuccess;
    }
    static inline PrepareRegistrar registrar{&prepare};
};

template <typename T, bool F8_INFER, int NV, int NVFULL, int NT, int MINW, int EXTRAS, bool OVF = false, bool NOPRUNE = false>
static hipError_t launch_resident_inst(const RowArgs &a, hipStream_t stream)
{
    typedef ResidentBuild<T, F8_INFER, NV, NVFULL, NT, MINW, EXTRAS, OVF, NOPRUNE> Build;
    (void)&Build::registrar;             // instantiates the registration of this build
    bool ready = Build::per_cu.load(std::memory_order_relaxed) != 0;
    if (ready && Build::kDynLds > 0) {
        int dev = 0;
        ready = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64 &&
                (Build::configured.load(std::memory_order_acquire) & (1ull << dev));
    }
    if (!ready) {
        const hipError_t e = Build::prepare();
        if (e != hipSuccess) return e;
    }
    int64_t grid = (int64_t)device_cu_count() * Build::per_cu.load(std::memory_order_relaxed);
    if (grid > a.n_rows) grid = a.n_rows;
    hipLaunchKernelGGL(Build::kernel(), dim3((unsigned)grid), dim3(NT), Build::kDynLds, stream, a);
    return hipGetLastError();
}

// Register slots per thread the resident kernel is built for: 256-thread
// groups for short rows (several groups share a CU), 1024-thread groups for
// long rows (one group owns the CU's register file).  Each build covers row
// lengths from its NVFULL (exclusive) to its NV (inclusive) slots per thread.
template <typename T, bool F8_INFER, int EXTRAS>
static hipError_t launch_resident_t(const RowArgs &a, hipStream_t stream)
{
    const int epv = elem_traits<T>::kPerVec;
    const int64_t slots = (int64_t)a.vocab / epv;   // whole vectors; the ragged end lives outside the slots
    if (slots <= 256 * 4)   return launch_resident_inst<T, F8_INFER, 4, 0, 256, 4, EXTRAS>(a, stream);
    if (slots <= 256 * 8)   return launch_resident_inst<T, F8_INFER, 8, 4, 256, 6, EXTRAS>(a, stream);
    if (slots <= 256 * 16)  return launch_resident_inst<T, F8_INFER, 16, 8, 256, 4, EXTRAS>(a, stream);
    if constexpr (!F8_INFER && EXTRAS == 0) {
        // nothing pruned and a dense gradient matrix: the build without threshold tests, with LDS fetch-ahead
        if (a.log_rho == -INFINITY && !a.sparse_only && a.grad_out != nullptr) {
            if (slots <= 1024 * 8)  return launch_resident_inst<T, false, 8, 4, 1024, 5, 0, false, true>(a, stream);
            if (slots <= 1024 * 12) return launch_resident_inst<T, false, 12, 8, 1024, 4, 0, false, true>(a, stream);
            if (slots <= 1024 * 16) return launch_resident_inst<T, false, 16, 12, 1024, 4, 0, false, true>(a, stream);
            if (slots <= 1024 * 19) return launch_resident_inst<T, false, 19, 16, 1024, 4, 0, false, true>(a, stream);
            if (slots <= 1024 * 20) return launch_resident_inst<T, false, 20, 19, 1024, 4, 0, false, true>(a, stream);
        }
    }
    if (slots <= 1024 * 8)  return launch_resident_inst<T, F8_INFER, 8, 4, 1024, 5, EXTRAS>(a, stream);
    if (slots <= 1024 * 12) return launch_resident_inst<T, F8_INFER, 12, 8, 1024, 4, EXTRAS>(a, stream);
    if (slots <= 1024 * 16) return launch_resident_inst<T, F8_INFER, 16, 12, 1024, 4, EXTRAS>(a, stream);
    if (slots <= 1024 * 19) return launch_resident_inst<T, F8_INFER, 19, 16, 1024, 4, EXTRAS>(a, stream);
    if (slots <= 1024 * 20) return launch_resident_inst<T, F8_INFER, 20, 19, 1024, 4, EXTRAS>(a, stream);
    if constexpr (!F8_INFER) return launch_resident_inst<T, false, 16, 16, 1024, 4, EXTRAS, true>(a, stream);
    return hipErrorInvalidValue;
}

bool row_fits_resident(int dtype, int dtype_infer, int64_t vocab)
{
    const int epv = dtype == DVP_BF16 ? 8 : 4;
    if (dtype_infer == DVP_F8E4M3)    // bf16 training rows that fit the registers only
        return dtype == DVP_BF16 && vocab >= 16 && vocab / epv <= 1024 * 20;
    return vocab >= epv;              // longer rows: resident up to 1024 * 20 vectors, the rest re-read
}

hipError_t launch_rows_resident(int dtype, int dtype_infer, const RowArgs &a, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    const bool two = a.n_sides == 2;
    const bool ent = a.out[0].entropy || (two && a.out[1].entropy);
    const bool extras = a.out[0].lse_full || a.out[0].safe_bits || (two && (a.out[1].lse_full || a.out[1].safe_bits));
    const int level = ent ? 2 : (extras ? 1 : 0);
    if (two && dtype_infer == DVP_F8E4M3) {
        if (dtype != DVP_BF16) return hipErrorInvalidValue;
        return level == 2 ? launch_resident_t<bf16_t, true, 2>(a, stream)
             : level == 1 ? launch_resident_t<bf16_t, true, 1>(a, stream) : launch_resident_t<bf16_t, true, 0>(a, stream);
    }
    if (dtype == DVP_BF16)
        return level == 2 ? launch_resident_t<bf16_t, false, 2>(a, stream)
             : level == 1 ? launch_resident_t<bf16_t, false, 1>(a, stream) : launch_resident_t<bf16_t, false, 0>(a, stream);
    return level == 2 ? launch_resident_t<float, false, 2>(a, stream)
         : level == 1 ? launch_resident_t<float, false, 1>(a, stream) : launch_resident_t<float, false, 0>(a, stream);
}

hipError_t launch_grad_fill(int dtype, const FillArgs &a, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    const int epv = dtype == DVP_BF16 ? 8 : 4;
    const int64_t nvec = a.vocab / epv;
    const int chunks = (int)((nvec + kFillChunk - 1) / kFillChunk > 0 ? (nvec + kFillChunk - 1) / kFillChunk : 1);
    const int64_t max_rows = 0x7fffffff / chunks;        // one launch covers this many rows
    for (int64_t r0 = 0; r0 < a.n_rows; r0 += max_rows) {
        FillArgs b = a;
        b.n_rows = a.n_rows - r0 < max_rows ? a.n_rows - r0 : max_rows;
        b.dz = (char *)a.dz + r0 * a.ld_grad * (dtype == DVP_BF16 ? 2 : 4);
        b.row_flags = a.row_flags + r0;
        b.safe_count = a.safe_count + r0;
        const dim3 gz((unsigned)(b.n_rows * chunks)), gs((unsigned)b.n_rows);
        const dim3 bz(kZeroThreads), blk(kFillThreads);
        if (dtype == DVP_BF16) {
            hipLaunchKernelGGL((grad_zero_kernel<bf16_t>), gz, bz, 0, stream, b, chunks);
            hipLaunchKernelGGL((grad_scatter_kernel<bf16_t>), gs, blk, 0, stream, b);
        } else {
            hipLaunchKernelGGL((grad_zero_kernel<float>), gz, bz, 0, stream, b, chunks);
            hipLaunchKernelGGL((grad_scatter_kernel<float>), gs, blk, 0, stream, b);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_rows_streaming(int dtype, int dtype_infer, const RowArgs &a, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    constexpr int NT = 512;
    int64_t grid = (int64_t)device_cu_count() * 4;
    if (grid > a.n_rows) grid = a.n_rows;
    const dim3 g((unsigned)grid), b(NT);
    const bool f8 = a.n_sides == 2 && dtype_infer == DVP_F8E4M3;
    if (dtype == DVP_BF16) {
        if (f8) hipLaunchKernelGGL((rows_streaming_kernel<bf16_t, f8_t, NT>), g, b, 0, stream, a);
        else    hipLaunchKernelGGL((rows_streaming_kernel<bf16_t, bf16_t, NT>), g, b, 0, stream, a);
    } else {
        if (f8) hipLaunchKernelGGL((rows_streaming_kernel<float, f8_t, NT>), g, b, 0, stream, a);
        else    hipLaunchKernelGGL((rows_streaming_kernel<float, float, NT>), g, b, 0, stream, a);
    }
    return hipGetLastError();
}

hipError_t launch_lists_to_dense(int dtype, const ListsArgs &a, bool vector_ok, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    const int epv = dtype == DVP_BF16 ? 8 : 4;
    const int64_t per = (int64_t)kListsZeroThreads * kListsZeroVecs * epv;
    const int chunks = (int)((a.vocab + per - 1) / per);
    const int64_t max_rows = 0x7fffffff / chunks;
    for (int64_t r0 = 0; r0 < a.n_rows; r0 += max_rows) {
        ListsArgs b = a;
        b.n_rows = a.n_rows - r0 < max_rows ? a.n_rows - r0 : max_rows;
        b.entries = (const char *)a.entries + r0 * a.list_cap * 8;
        b.grad_len = a.grad_len + r0;
        b.row_flags = a.row_flags + r0;
        b.scale = a.scale ? a.scale + r0 : nullptr;
        b.dz = (char *)a.dz + r0 * a.ld_grad * (dtype == DVP_BF16 ? 2 : 4);
        const dim3 gz((unsigned)(b.n_rows * chunks)), bz(kListsZeroThreads);
        const dim3 gs((unsigned)b.n_rows), bs(kListsScatterThreads);
        if (dtype == DVP_BF16) {
            if (vector_ok) hipLaunchKernelGGL((lists_zero_kernel<bf16_t, true>), gz, bz, 0, stream, b, chunks);
            else           hipLaunchKernelGGL((lists_zero_kernel<bf16_t, false>), gz, bz, 0, stream, b, chunks);
            hipLaunchKernelGGL((lists_scatter_kernel<bf16_t>), gs, bs, 0, stream, b);
        } else {
            if (vector_ok) hipLaunchKernelGGL((lists_zero_kernel<float, true>), gz, bz, 0, stream, b, chunks);
            else           hipLaunchKernelGGL((lists_zero_kernel<float, false>), gz, bz, 0, stream, b, chunks);
            hipLaunchKernelGGL((lists_scatter_kernel<float>), gs, bs, 0, stream, b);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_backward(int dtype, const BackwardArgs &a, bool vector_ok, hipStream_t stream)
{
    if (a.n_rows == 0) return hipSuccess;
    if (a.split) {      // zeros over the rows without gradient or with a short safe set: write-only, before any read
        const int epv = dtype == DVP_BF16 ? 8 : 4;
        const int64_t per = (int64_t)kBwdZeroThreads * kBwdZeroVecs * epv;
        const int chunks = (int)((a.vocab + per - 1) / per);
        const int64_t max_rows = 0x7fffffff / chunks;
        for (int64_t r0 = 0; r0 < a.n_rows; r0 += max_rows) {
            BackwardArgs b = a;
            b.n_rows = a.n_rows - r0 < max_rows ? a.n_rows - r0 : max_rows;
            b.row_flags = a.row_flags + r0;
            b.dz = (char *)a.dz + r0 * a.ld_grad * (dtype == DVP_BF16 ? 2 : 4);
            const dim3 gz((unsigned)(b.n_rows * chunks)), bz(kBwdZeroThreads);
            if (dtype == DVP_BF16) {
                if (vector_ok) hipLaunchKernelGGL((backward_zero_kernel<bf16_t, true>), gz, bz, 0, stream, b, chunks);
                else           hipLaunchKernelGGL((backward_zero_kernel<bf16_t, false>), gz, bz, 0, stream, b, chunks);
            } else {
                if (vector_ok) hipLaunchKernelGGL((backward_zero_kernel<float, true>), gz, bz, 0, stream, b, chunks);
                else           hipLaunchKernelGGL((backward_zero_kernel<float, false>), gz, bz, 0, stream, b, chunks);
            }
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
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
