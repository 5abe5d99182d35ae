// Device-side helpers shared by the DVP kernels: 16-byte vector access,
// bf16 <-> fp32 bit conversions, wavefront (64 lanes) and workgroup reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dvp {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };   // storage-only tag type for bf16 rows
struct f8_t { uint8_t bits; };      // storage-only tag type for 8-bit E4M3 rows (OCP: bias 7, no infinity, max 448)

template <typename T> struct elem_traits;
template <> struct elem_traits<float> {
    static constexpr int kPerVec = 4;
    static constexpr int kPerPart = 4;
    static constexpr uint32_t kPadWord = 0xff800000u;   // -inf
    static constexpr bool kHasNegInf = true;
};
template <> struct elem_traits<bf16_t> {
    static constexpr int kPerVec = 8;
    static constexpr int kPerPart = 8;
    static constexpr uint32_t kPadWord = 0xff80ff80u;   // two bf16 -inf
    static constexpr bool kHasNegInf = true;
};
template <> struct elem_traits<f8_t> {
    static constexpr int kPerVec = 16;
    static constexpr int kPerPart = 8;                  // widened half a vector at a time
    static constexpr uint32_t kPadWord = 0u;            // the format has no -inf: readers mask by index
    static constexpr bool kHasNegInf = false;
};

__device__ __forceinline__ float bits_to_float(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t float_to_bits(float f) { return __float_as_uint(f); }

// fp32 -> bf16 bits, round to nearest even (finite inputs and infinities).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = float_to_bits(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// widen the elements of one 16-byte vector to fp32, memory order
__device__ __forceinline__ void unpack(const u32x4 v, float (&x)[4], float)
{
    x[0] = bits_to_float(v.x); x[1] = bits_to_float(v.y);
    x[2] = bits_to_float(v.z); x[3] = bits_to_float(v.w);
}
__device__ __forceinline__ void unpack(const u32x4 v, float (&x)[8], bf16_t)
{
    x[0] = bits_to_float(v.x << 16); x[1] = bits_to_float(v.x & 0xffff0000u);
    x[2] = bits_to_float(v.y << 16); x[3] = bits_to_float(v.y & 0xffff0000u);
    x[4] = bits_to_float(v.z << 16); x[5] = bits_to_float(v.z & 0xffff0000u);
    x[6] = bits_to_float(v.w << 16); x[7] = bits_to_float(v.w & 0xffff0000u);
}

// 8-bit E4M3 -> fp32 with the hardware converter (exact: every code is an fp32 value)
__device__ __forceinline__ float e4m3_to_float(uint32_t byte) { return __builtin_amdgcn_cvt_f32_fp8((int)byte, 0); }
__device__ __forceinline__ void unpack(const u32x4 v, float (&x)[8], int part, f8_t)   // bytes 8*part .. 8*part+7
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const uint32_t w[2] = {part == 0 ? v.x : v.z, part == 0 ? v.y : v.w};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
        const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
        x[4 * i + 0] = lo.x; x[4 * i + 1] = lo.y; x[4 * i + 2] = hi.x; x[4 * i + 3] = hi.y;
    }
}
__device__ __forceinline__ void unpack(const u32x4 v, float (&x)[4], int, float) { unpack(v, x, float()); }
__device__ __forceinline__ void unpack(const u32x4 v, float (&x)[8], int, bf16_t) { unpack(v, x, bf16_t()); }

__device__ __forceinline__ u32x4 pack(const float (&d)[4], float)
{
    u32x4 v;
    v.x = float_to_bits(d[0]); v.y = float_to_bits(d[1]);
    v.z = float_to_bits(d[2]); v.w = float_to_bits(d[3]);
    return v;
}
__device__ __forceinline__ u32x4 pack(const float (&d)[8], bf16_t)
{
    u32x4 v;
    v.x = f32_to_bf16_rne(d[0]) | (f32_to_bf16_rne(d[1]) << 16);
    v.y = f32_to_bf16_rne(d[2]) | (f32_to_bf16_rne(d[3]) << 16);
    v.z = f32_to_bf16_rne(d[4]) | (f32_to_bf16_rne(d[5]) << 16);
    v.w = f32_to_bf16_rne(d[6]) | (f32_to_bf16_rne(d[7]) << 16);
    return v;
}

__device__ __forceinline__ float load_elem(const float *p) { return *p; }
__device__ __forceinline__ float load_elem(const bf16_t *p)
{
    return bits_to_float((uint32_t)p->bits << 16);
}
__device__ __forceinline__ float load_elem(const f8_t *p) { return e4m3_to_float(p->bits); }
__device__ __forceinline__ void store_elem(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(bf16_t *p, float v)
{
    p->bits = (uint16_t)f32_to_bf16_rne(v);
}

// Threshold of the finite-mask variant: the fp32 sum rounded to the logits' storage type, as a
// tensor-plus-scalar add in that type delivers it on a GPU (Sec. 5.5, App. A).
__device__ __forceinline__ float storage_rounded(float t, float) { return t; }
__device__ __forceinline__ float storage_rounded(float t, bf16_t) { return bits_to_float(f32_to_bf16_rne(t) << 16); }

// Asynchronous copy from global memory straight into LDS, no register staging: lane l moves the 16
// bytes at gbase + voff (per lane) to LDS byte lds_addr + 16 l (gbase and lds_addr wavefront-uniform).
// The compiler's wait-count bookkeeping does not see these copies: whoever reads the LDS bytes waits for
// them explicitly (s_waitcnt vmcnt) first.
__device__ __forceinline__ void copy16_to_lds(const void *gbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
}

// ---- wavefront reductions (all 64 lanes end with the result) ----
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// ---- workgroup reductions through LDS: one barrier each.  `slot` must hold
// NT/64 entries and must not be reused before another barrier has passed. ----
template <int NT>
__device__ __forceinline__ float block_max(float v, float *slot)
{
    constexpr int NW = NT / kWave;
    v = wave_max(v);
    if ((threadIdx.x & (kWave - 1)) == 0) slot[threadIdx.x / kWave] = v;
    __syncthreads();
    float r = slot[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = fmaxf(r, slot[w]);
    return r;
}

struct RowSums { float s_safe; float s_full; int count; };

template <int NT>
__device__ __forceinline__ RowSums block_sums(RowSums v, float *slot_f, int *slot_i)
{
    constexpr int NW = NT / kWave;
    v.s_safe = wave_sum(v.s_safe);
    v.s_full = wave_sum(v.s_full);
    v.count = wave_sum(v.count);
    if ((threadIdx.x & (kWave - 1)) == 0) {
        const int w = threadIdx.x / kWave;
        slot_f[w] = v.s_safe;
        slot_f[NW + w] = v.s_full;
        slot_i[w] = v.count;
    }
    __syncthreads();
    RowSums r = {slot_f[0], slot_f[NW], slot_i[0]};
#pragma unroll
    for (int w = 1; w < NW; ++w) {   // fixed order: results are run-to-run identical
        r.s_safe += slot_f[w];
        r.s_full += slot_f[NW + w];
        r.count += slot_i[w];
    }
    return r;
}

}  // namespace dvp
