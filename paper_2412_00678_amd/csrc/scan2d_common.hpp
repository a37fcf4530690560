// Shared device helpers of the gfx950 2D selective scan kernels: storage types, wide loads
// with 4-byte alignment, bf16 conversion, DPP lane movement and the wave-level scan of
// (decay-product, state) pairs.  Device code only; nothing here is used by the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace scan2d {

constexpr float kLog2e = 1.4426950408889634f;


struct bf16_t { uint16_t bits; };   // storage tag: upper half of an IEEE fp32

template <typename T> struct Elem;
template <> struct Elem<float>  { static constexpr int kBytes = 4; };
template <> struct Elem<bf16_t> { static constexpr int kBytes = 2; };

// 32-bit words that hold K consecutive elements of T (K is a multiple of 4).
template <typename T, int K> constexpr int words_of() { return K * Elem<T>::kBytes / 4; }

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef u32x4_t u32x4_a4 __attribute__((aligned(4)));
typedef u32x2_t u32x2_a4 __attribute__((aligned(4)));

// Load WORDS consecutive dwords from a 4-byte aligned address with the widest instructions.
template <int WORDS>
__device__ __forceinline__ void load_words(const uint32_t* __restrict__ p, uint32_t* r) {
    int w = 0;
#pragma unroll
    for (; w + 4 <= WORDS; w += 4) {
        const u32x4_a4 v = *reinterpret_cast<const u32x4_a4*>(p + w);
        r[w] = v.x; r[w + 1] = v.y; r[w + 2] = v.z; r[w + 3] = v.w;
    }
#pragma unroll
    for (; w + 2 <= WORDS; w += 2) {
        const u32x2_a4 v = *reinterpret_cast<const u32x2_a4*>(p + w);
        r[w] = v.x; r[w + 1] = v.y;
    }
#pragma unroll
    for (; w < WORDS; ++w) r[w] = p[w];
}

// The same from any byte address (global memory only: flat and global loads of gfx950 accept
// unaligned addresses, buffer loads do not).
typedef u32x4_t u32x4_a1 __attribute__((aligned(1)));
typedef u32x2_t u32x2_a1 __attribute__((aligned(1)));
typedef uint32_t u32_a1 __attribute__((aligned(1)));
template <int WORDS>
__device__ __forceinline__ void load_words_any(const void* __restrict__ q, uint32_t* r) {
    const unsigned char* p = static_cast<const unsigned char*>(q);
    int w = 0;
#pragma unroll
    for (; w + 4 <= WORDS; w += 4) {
        const u32x4_a1 v = *reinterpret_cast<const u32x4_a1*>(p + 4 * w);
        r[w] = v.x; r[w + 1] = v.y; r[w + 2] = v.z; r[w + 3] = v.w;
    }
#pragma unroll
    for (; w + 2 <= WORDS; w += 2) {
        const u32x2_a1 v = *reinterpret_cast<const u32x2_a1*>(p + 4 * w);
        r[w] = v.x; r[w + 1] = v.y;
    }
#pragma unroll
    for (; w < WORDS; ++w) r[w] = *reinterpret_cast<const u32_a1*>(p + 4 * w);
}

template <int WORDS>
__device__ __forceinline__ void store_words_any(void* __restrict__ q, const uint32_t* r) {
    unsigned char* p = static_cast<unsigned char*>(q);
    int w = 0;
#pragma unroll
    for (; w + 4 <= WORDS; w += 4) {
        u32x4_a1 v; v.x = r[w]; v.y = r[w + 1]; v.z = r[w + 2]; v.w = r[w + 3];
        *reinterpret_cast<u32x4_a1*>(p + 4 * w) = v;
    }
#pragma unroll
    for (; w + 2 <= WORDS; w += 2) {
        u32x2_a1 v; v.x = r[w]; v.y = r[w + 1];
        *reinterpret_cast<u32x2_a1*>(p + 4 * w) = v;
    }
#pragma unroll
    for (; w < WORDS; ++w) *reinterpret_cast<u32_a1*>(p + 4 * w) = r[w];
}

template <int WORDS>
__device__ __forceinline__ void store_words(uint32_t* __restrict__ p, const uint32_t* r) {
    int w = 0;
#pragma unroll
    for (; w + 4 <= WORDS; w += 4) {
        u32x4_a4 v; v.x = r[w]; v.y = r[w + 1]; v.z = r[w + 2]; v.w = r[w + 3];
        *reinterpret_cast<u32x4_a4*>(p + w) = v;
    }
#pragma unroll
    for (; w + 2 <= WORDS; w += 2) {
        u32x2_a4 v; v.x = r[w]; v.y = r[w + 1];
        *reinterpret_cast<u32x2_a4*>(p + w) = v;
    }
#pragma unroll
    for (; w < WORDS; ++w) p[w] = r[w];
}

// Buffer addressing: a wave-uniform base in a resource descriptor (scalar registers), a 32-bit
// byte offset per lane and a 32-bit uniform byte offset (the row), which the memory instruction
// adds itself - no 64-bit vector address arithmetic per load.  Spans are below 2^31 bytes.
// `bytes` is what remains of the tensor behind `base`: a load that reaches past it returns 0
// instead of touching memory, so a lane may read its K elements across the end of the last row.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
    const int records = bytes > (size_t)0x7fffffff ? 0x7fffffff : (int)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, records, 0x00020000);
}
template <int WORDS>
__device__ __forceinline__ void buffer_load_words(rsrc_t rs, uint32_t lane_bytes, uint32_t uniform_bytes, uint32_t* r) {
    int w = 0;
#pragma unroll
    for (; w + 4 <= WORDS; w += 4) {
        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_bytes + 4 * w, uniform_bytes, 0);
        r[w] = v.x; r[w + 1] = v.y; r[w + 2] = v.z; r[w + 3] = v.w;
    }
#pragma unroll
    for (; w + 2 <= WORDS; w += 2) {
        const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(rs, lane_bytes + 4 * w, uniform_bytes, 0);
        r[w] = v.x; r[w + 1] = v.y;
    }
#pragma unroll
    for (; w < WORDS; ++w) r[w] = __builtin_amdgcn_raw_buffer_load_b32(rs, lane_bytes + 4 * w, uniform_bytes, 0);
}

__device__ __forceinline__ uint32_t elem_bits(const float* p)  { return __float_as_uint(*p); }
__device__ __forceinline__ uint32_t elem_bits(const bf16_t* p) { return p->bits; }

template <typename T, int K>
__device__ __forceinline__ void put_elem(uint32_t* r, int j, uint32_t bits) {
    if constexpr (Elem<T>::kBytes == 4) r[j] = bits;
    else r[j >> 1] |= bits << (16 * (j & 1));
}

// The K elements [col0, col0+K) of one row (global memory); columns >= W read as +0 and are never
// touched in memory (identity padding: delta = 0 gives a = 1, x = B = C = 0 gives u = 0).  A lane whose
// K columns all exist reads them with wide loads whatever the address alignment (vec_ok: the address
// is known to be 4-byte aligned); only a lane across the row end goes element by element.
template <typename T, int K>
__device__ __forceinline__ void load_row(const T* __restrict__ rowp, int col0, int W, bool vec_ok,
                                         uint32_t* r) {
    if (col0 + K <= W) {
        if (vec_ok) load_words<words_of<T, K>()>(reinterpret_cast<const uint32_t*>(rowp + col0), r);
        else load_words_any<words_of<T, K>()>(rowp + col0, r);
    } else {
#pragma unroll
        for (int w = 0; w < words_of<T, K>(); ++w) r[w] = 0u;
#pragma unroll
        for (int j = 0; j < K; ++j)
            if (col0 + j < W) put_elem<T, K>(r, j, elem_bits(rowp + col0 + j));
    }
}

// K mask bytes packed 4 per word; columns >= W read as 0 (not background).
template <int K>
__device__ __forceinline__ void load_mask(const uint8_t* __restrict__ rowp, int col0, int W, bool vec_ok,
                                          uint32_t* m) {
    if (col0 + K <= W) {
        if (vec_ok) load_words<K / 4>(reinterpret_cast<const uint32_t*>(rowp + col0), m);
        else load_words_any<K / 4>(rowp + col0, m);
    } else {
#pragma unroll
        for (int w = 0; w < K / 4; ++w) m[w] = 0u;
#pragma unroll
        for (int j = 0; j < K; ++j)
            if (col0 + j < W) m[j >> 2] |= static_cast<uint32_t>(rowp[col0 + j]) << (8 * (j & 3));
    }
}

template <int K>
__device__ __forceinline__ bool mask_bit(const uint32_t* m, int j) {
    return ((m[j >> 2] >> (8 * (j & 3))) & 0xffu) != 0u;
}

template <typename T, int K>
__device__ __forceinline__ float get_elem(const uint32_t* r, int j) {
    if constexpr (Elem<T>::kBytes == 4) return __uint_as_float(r[j]);
    else return (j & 1) ? __uint_as_float(r[j >> 1] & 0xffff0000u) : __uint_as_float(r[j >> 1] << 16);
}

// fp32 -> bf16 bits, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? ((u >> 16) | 0x40u) : r;
}

template <typename T> __device__ __forceinline__ uint32_t to_elem_bits(float f) {
    if constexpr (Elem<T>::kBytes == 4) return __float_as_uint(f);
    else return f32_to_bf16_bits(f);
}

__device__ __forceinline__ void store_elem(float* p, float f)  { *p = f; }
__device__ __forceinline__ void store_elem(bf16_t* p, float f) { p->bits = static_cast<uint16_t>(f32_to_bf16_bits(f)); }

// Write v[0..K) to columns [col0, col0+K) of a row, skipping columns >= W.
template <typename T, int K>
__device__ __forceinline__ void store_row(T* __restrict__ rowp, int col0, int W, bool vec_ok, const float* v) {
    if (col0 + K <= W) {                      // wide stores at any alignment (vec_ok: known to be 4-byte aligned)
        uint32_t r[words_of<T, K>()];
#pragma unroll
        for (int w = 0; w < words_of<T, K>(); ++w) r[w] = 0u;
#pragma unroll
        for (int j = 0; j < K; ++j) put_elem<T, K>(r, j, to_elem_bits<T>(v[j]));
        if (vec_ok) store_words<words_of<T, K>()>(reinterpret_cast<uint32_t*>(rowp + col0), r);
        else store_words_any<words_of<T, K>()>(rowp + col0, r);
    } else {
#pragma unroll
        for (int j = 0; j < K; ++j)
            if (col0 + j < W) store_elem(rowp + col0 + j, v[j]);
    }
}

// softplus(t) = log(1 + exp(t)) (2DMamba Eq. 3: the step is the softplus of its projection), through
// v_exp_f32 / v_log_f32 (base 2).  Beyond t = 15 the result is t to fp32 precision.  For very negative t
// the sum 1 + exp(t) loses the low digits of exp(t): the absolute error of the step stays below 1e-7, far
// inside the tolerance of everything computed from it (the step itself is then below 1e-4).
__device__ __forceinline__ float softplus_f32(float t) {
    const float lp = __builtin_amdgcn_logf(1.0f + __builtin_amdgcn_exp2f(t * kLog2e)) * 0.6931471805599453f;
    return t > 15.0f ? t : lp;
}
// d softplus(t) / dt = 1 / (1 + exp(-t))
__device__ __forceinline__ float logistic_f32(float t) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-t * kLog2e));
}

// h = a * h + add with h updated in place.  The compiler would pick the two-operand
// v_fmac_f32, whose destination is the addend, and then move the result back into the register
// that carries h into the next row: one extra instruction per state and column.  The
// three-operand form writes h directly.
__device__ __forceinline__ void fma_inplace(float& h, float a, float add) {
    asm("v_fma_f32 %0, %1, %0, %2" : "+v"(h) : "v"(a), "v"(add));
}

// ----------------------------------------------------------------------------- DPP
// dpp_ctrl names of gfx9 used below: row_shr:n / row_shl:n shift inside a row of 16 lanes,
// wave_shr:1 / wave_shl:1 shift across the whole wavefront, row_bcast:15 copies lane 15 of
// each row to the next row, row_bcast:31 copies lane 31 to rows 2 and 3.
// ------------------------------------------------------------------ group scan (rightwards)
// Inclusive scan, over the LG lanes of a lane group, of the linear recurrence h <- P*h_in + H.
// In : per lane, P = product of the decays of its K columns, H = its last local state
//      computed with zero carry-in.
// Out: H = state at the lane's last column including everything to its left in the group;
//      C = that value of the lane to the left (0 for the group's first lane), i.e. the carry
//      entering this lane.  P is consumed (afterwards: the product of the decays up to and
//      including this lane inside its DPP row).
// A lane whose source lane does not exist (or whose row is switched off by row_mask) is not
// written by a DPP instruction, which is exactly the identity element of the recurrence.  The
// copy that fetches the carry sets bound_ctrl instead: such a lane then reads 0, so C needs no
// initial value.
// Each step is H += P * H[lane-d]; P *= P[lane-d], written as VOP2 instructions with a DPP
// source so that the lane movement costs no extra instruction.  S independent recurrences
// are interleaved in one block: that keeps the two wait states the hardware requires between
// a VALU write of a VGPR and a DPP read of it (explicit s_nop where S is too small).
#define SCAN2D_SHR(n) " row_shr:" #n " row_mask:0xf bank_mask:0xf\n\t"
#define SCAN2D_BC15 " row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
#define SCAN2D_BC31 " row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
#define SCAN2D_CIN16 " row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0\n\t"
#define SCAN2D_CIN64 " wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0\n\t"

#define SCAN2D_S1_STEP(M) "v_fmac_f32_dpp %0, %0, %1" M "v_mul_f32_dpp %1, %1, %1" M "s_nop 0\n\t"
#define SCAN2D_S1_LAST(M) "v_fmac_f32_dpp %0, %0, %1" M "s_nop 1\n\t"
#define SCAN2D_S2_STEP(M) "v_fmac_f32_dpp %0, %0, %2" M "v_fmac_f32_dpp %1, %1, %3" M \
                          "v_mul_f32_dpp %2, %2, %2" M "v_mul_f32_dpp %3, %3, %3" M
#define SCAN2D_S2_LAST(M) "v_fmac_f32_dpp %0, %0, %2" M "v_fmac_f32_dpp %1, %1, %3" M "s_nop 0\n\t"
#define SCAN2D_S4_STEP(M) "v_fmac_f32_dpp %0, %0, %4" M "v_fmac_f32_dpp %1, %1, %5" M \
                          "v_fmac_f32_dpp %2, %2, %6" M "v_fmac_f32_dpp %3, %3, %7" M \
                          "v_mul_f32_dpp %4, %4, %4" M "v_mul_f32_dpp %5, %5, %5" M   \
                          "v_mul_f32_dpp %6, %6, %6" M "v_mul_f32_dpp %7, %7, %7" M
#define SCAN2D_S4_LAST(M) "v_fmac_f32_dpp %0, %0, %4" M "v_fmac_f32_dpp %1, %1, %5" M \
                          "v_fmac_f32_dpp %2, %2, %6" M "v_fmac_f32_dpp %3, %3, %7" M

template <int LG>
__device__ __forceinline__ void group_scan1(float& P0, float& H0, float& C0) {
    if constexpr (LG == 32) {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S1_STEP(SCAN2D_SHR(1)) SCAN2D_S1_STEP(SCAN2D_SHR(2))
                     SCAN2D_S1_STEP(SCAN2D_SHR(4)) SCAN2D_S1_STEP(SCAN2D_SHR(8))
                     SCAN2D_S1_LAST(SCAN2D_BC15)
                     "v_mov_b32_dpp %2, %0" SCAN2D_CIN64
                     : "+v"(H0), "+v"(P0), "=&v"(C0));
    } else if constexpr (LG == 16) {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S1_STEP(SCAN2D_SHR(1)) SCAN2D_S1_STEP(SCAN2D_SHR(2))
                     SCAN2D_S1_STEP(SCAN2D_SHR(4)) SCAN2D_S1_LAST(SCAN2D_SHR(8))
                     "v_mov_b32_dpp %2, %0" SCAN2D_CIN16
                     : "+v"(H0), "+v"(P0), "=&v"(C0));
    } else {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S1_STEP(SCAN2D_SHR(1)) SCAN2D_S1_STEP(SCAN2D_SHR(2))
                     SCAN2D_S1_STEP(SCAN2D_SHR(4)) SCAN2D_S1_STEP(SCAN2D_SHR(8))
                     SCAN2D_S1_STEP(SCAN2D_BC15) SCAN2D_S1_LAST(SCAN2D_BC31)
                     "v_mov_b32_dpp %2, %0" SCAN2D_CIN64
                     : "+v"(H0), "+v"(P0), "=&v"(C0));
    }
}

template <int LG>
__device__ __forceinline__ void group_scan2(float& P0, float& P1, float& H0, float& H1, float& C0, float& C1) {
    if constexpr (LG == 32) {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S2_STEP(SCAN2D_SHR(1)) SCAN2D_S2_STEP(SCAN2D_SHR(2))
                     SCAN2D_S2_STEP(SCAN2D_SHR(4)) SCAN2D_S2_STEP(SCAN2D_SHR(8))
                     SCAN2D_S2_LAST(SCAN2D_BC15)
                     "v_mov_b32_dpp %4, %0" SCAN2D_CIN64 "v_mov_b32_dpp %5, %1" SCAN2D_CIN64
                     : "+v"(H0), "+v"(H1), "+v"(P0), "+v"(P1), "=&v"(C0), "=&v"(C1));
    } else if constexpr (LG == 16) {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S2_STEP(SCAN2D_SHR(1)) SCAN2D_S2_STEP(SCAN2D_SHR(2))
                     SCAN2D_S2_STEP(SCAN2D_SHR(4)) SCAN2D_S2_LAST(SCAN2D_SHR(8))
                     "v_mov_b32_dpp %4, %0" SCAN2D_CIN16 "v_mov_b32_dpp %5, %1" SCAN2D_CIN16
                     : "+v"(H0), "+v"(H1), "+v"(P0), "+v"(P1), "=&v"(C0), "=&v"(C1));
    } else {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S2_STEP(SCAN2D_SHR(1)) SCAN2D_S2_STEP(SCAN2D_SHR(2))
                     SCAN2D_S2_STEP(SCAN2D_SHR(4)) SCAN2D_S2_STEP(SCAN2D_SHR(8))
                     SCAN2D_S2_STEP(SCAN2D_BC15) SCAN2D_S2_LAST(SCAN2D_BC31)
                     "v_mov_b32_dpp %4, %0" SCAN2D_CIN64 "v_mov_b32_dpp %5, %1" SCAN2D_CIN64
                     : "+v"(H0), "+v"(H1), "+v"(P0), "+v"(P1), "=&v"(C0), "=&v"(C1));
    }
}

template <int LG>
__device__ __forceinline__ void group_scan4(float& P0, float& P1, float& P2, float& P3,
                                            float& H0, float& H1, float& H2, float& H3,
                                            float& C0, float& C1, float& C2, float& C3) {
    if constexpr (LG == 32) {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S4_STEP(SCAN2D_SHR(1)) SCAN2D_S4_STEP(SCAN2D_SHR(2))
                     SCAN2D_S4_STEP(SCAN2D_SHR(4)) SCAN2D_S4_STEP(SCAN2D_SHR(8))
                     SCAN2D_S4_LAST(SCAN2D_BC15)
                     "v_mov_b32_dpp %8, %0" SCAN2D_CIN64 "v_mov_b32_dpp %9, %1" SCAN2D_CIN64
                     "v_mov_b32_dpp %10, %2" SCAN2D_CIN64 "v_mov_b32_dpp %11, %3" SCAN2D_CIN64
                     : "+v"(H0), "+v"(H1), "+v"(H2), "+v"(H3), "+v"(P0), "+v"(P1), "+v"(P2), "+v"(P3),
                       "=&v"(C0), "=&v"(C1), "=&v"(C2), "=&v"(C3));
    } else if constexpr (LG == 16) {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S4_STEP(SCAN2D_SHR(1)) SCAN2D_S4_STEP(SCAN2D_SHR(2))
                     SCAN2D_S4_STEP(SCAN2D_SHR(4)) SCAN2D_S4_LAST(SCAN2D_SHR(8))
                     "v_mov_b32_dpp %8, %0" SCAN2D_CIN16 "v_mov_b32_dpp %9, %1" SCAN2D_CIN16
                     "v_mov_b32_dpp %10, %2" SCAN2D_CIN16 "v_mov_b32_dpp %11, %3" SCAN2D_CIN16
                     : "+v"(H0), "+v"(H1), "+v"(H2), "+v"(H3), "+v"(P0), "+v"(P1), "+v"(P2), "+v"(P3),
                       "=&v"(C0), "=&v"(C1), "=&v"(C2), "=&v"(C3));
    } else {
        asm volatile("s_nop 1\n\t"
                     SCAN2D_S4_STEP(SCAN2D_SHR(1)) SCAN2D_S4_STEP(SCAN2D_SHR(2))
                     SCAN2D_S4_STEP(SCAN2D_SHR(4)) SCAN2D_S4_STEP(SCAN2D_SHR(8))
                     SCAN2D_S4_STEP(SCAN2D_BC15) SCAN2D_S4_LAST(SCAN2D_BC31)
                     "v_mov_b32_dpp %8, %0" SCAN2D_CIN64 "v_mov_b32_dpp %9, %1" SCAN2D_CIN64
                     "v_mov_b32_dpp %10, %2" SCAN2D_CIN64 "v_mov_b32_dpp %11, %3" SCAN2D_CIN64
                     : "+v"(H0), "+v"(H1), "+v"(H2), "+v"(H3), "+v"(P0), "+v"(P1), "+v"(P2), "+v"(P3),
                       "=&v"(C0), "=&v"(C1), "=&v"(C2), "=&v"(C3));
    }
}

// Scan S (1, 2 or 4) recurrences held in arrays.  LG = 32 (half a wavefront): the first lane of
// the upper half must not take the carry of the lower half.
template <int LG, int S>
__device__ __forceinline__ void group_scan(float* P, float* H, float* C) {
    if constexpr (S == 1) group_scan1<LG>(P[0], H[0], C[0]);
    else if constexpr (S == 2) group_scan2<LG>(P[0], P[1], H[0], H[1], C[0], C[1]);
    else group_scan4<LG>(P[0], P[1], P[2], P[3], H[0], H[1], H[2], H[3], C[0], C[1], C[2], C[3]);
    if constexpr (LG == 32) {
        const bool first = (threadIdx.x & 31u) == 0u;
#pragma unroll
        for (int t = 0; t < S; ++t) C[t] = first ? 0.0f : C[t];
    }
}

// The same scans without the copy of the left neighbour's state: for callers that apply the carry with the
// lane movement inside the multiply-add (DPP source).  C is only written for half-wave groups, which keep
// the plain form.  The trailing s_nop of the one-state form covers the DPP read that follows.
template <int LG, int S>
__device__ __forceinline__ void group_scan_nocarry(float* P, float* H, float* C) {
    if constexpr (LG == 32) {
        group_scan<LG, S>(P, H, C);
    } else if constexpr (S == 1) {
        if constexpr (LG == 16)
            asm volatile("s_nop 1\n\t"
                         SCAN2D_S1_STEP(SCAN2D_SHR(1)) SCAN2D_S1_STEP(SCAN2D_SHR(2))
                         SCAN2D_S1_STEP(SCAN2D_SHR(4)) SCAN2D_S1_LAST(SCAN2D_SHR(8))
                         : "+v"(H[0]), "+v"(P[0]));
        else
            asm volatile("s_nop 1\n\t"
                         SCAN2D_S1_STEP(SCAN2D_SHR(1)) SCAN2D_S1_STEP(SCAN2D_SHR(2))
                         SCAN2D_S1_STEP(SCAN2D_SHR(4)) SCAN2D_S1_STEP(SCAN2D_SHR(8))
                         SCAN2D_S1_STEP(SCAN2D_BC15) SCAN2D_S1_LAST(SCAN2D_BC31)
                         : "+v"(H[0]), "+v"(P[0]));
    } else if constexpr (S == 2) {
        if constexpr (LG == 16)
            asm volatile("s_nop 1\n\t"
                         SCAN2D_S2_STEP(SCAN2D_SHR(1)) SCAN2D_S2_STEP(SCAN2D_SHR(2))
                         SCAN2D_S2_STEP(SCAN2D_SHR(4)) SCAN2D_S2_LAST(SCAN2D_SHR(8))
                         : "+v"(H[0]), "+v"(H[1]), "+v"(P[0]), "+v"(P[1]));
        else
            asm volatile("s_nop 1\n\t"
                         SCAN2D_S2_STEP(SCAN2D_SHR(1)) SCAN2D_S2_STEP(SCAN2D_SHR(2))
                         SCAN2D_S2_STEP(SCAN2D_SHR(4)) SCAN2D_S2_STEP(SCAN2D_SHR(8))
                         SCAN2D_S2_STEP(SCAN2D_BC15) SCAN2D_S2_LAST(SCAN2D_BC31)
                         : "+v"(H[0]), "+v"(H[1]), "+v"(P[0]), "+v"(P[1]));
    } else {
        if constexpr (LG == 16)
            asm volatile("s_nop 1\n\t"
                         SCAN2D_S4_STEP(SCAN2D_SHR(1)) SCAN2D_S4_STEP(SCAN2D_SHR(2))
                         SCAN2D_S4_STEP(SCAN2D_SHR(4)) SCAN2D_S4_LAST(SCAN2D_SHR(8))
                         : "+v"(H[0]), "+v"(H[1]), "+v"(H[2]), "+v"(H[3]), "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]));
        else
            asm volatile("s_nop 1\n\t"
                         SCAN2D_S4_STEP(SCAN2D_SHR(1)) SCAN2D_S4_STEP(SCAN2D_SHR(2))
                         SCAN2D_S4_STEP(SCAN2D_SHR(4)) SCAN2D_S4_STEP(SCAN2D_SHR(8))
                         SCAN2D_S4_STEP(SCAN2D_BC15) SCAN2D_S4_LAST(SCAN2D_BC31)
                         : "+v"(H[0]), "+v"(H[1]), "+v"(H[2]), "+v"(H[3]), "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]));
    }
}

// ------------------------------------------------------------------ group scan (leftwards)
// Mirror image for the reverse row scan of the backward pass: q <- Q + P * q_in where q_in
// comes from the lane to the RIGHT.  Out: C = the value at the first column of the lane to the
// right, including everything further right in the group (0 for the group's last lane), i.e.
// the carry entering this lane.  P and Q are consumed.  Inside a DPP row the steps use row_shl.  A wavefront has no leftward
// counterpart of row_bcast, so for LG = 64 the pairs are mirrored across the wave with
// ds_bpermute (LDS crossbar, no VALU slot), scanned rightwards, and the carry mirrored back.
#define SCAN2D_SHL(n) " row_shl:" #n " row_mask:0xf bank_mask:0xf\n\t"

__device__ __forceinline__ void row_scan_left1(float& P0, float& H0, float& C0) {
    C0 = 0.0f;
    asm volatile("s_nop 1\n\t"
                 SCAN2D_S1_STEP(SCAN2D_SHL(1)) SCAN2D_S1_STEP(SCAN2D_SHL(2))
                 SCAN2D_S1_STEP(SCAN2D_SHL(4)) SCAN2D_S1_LAST(SCAN2D_SHL(8))
                 "v_mov_b32_dpp %2, %0" SCAN2D_SHL(1)
                 : "+v"(H0), "+v"(P0), "+v"(C0));
}
__device__ __forceinline__ void row_scan_left2(float& P0, float& P1, float& H0, float& H1, float& C0, float& C1) {
    C0 = 0.0f; C1 = 0.0f;
    asm volatile("s_nop 1\n\t"
                 SCAN2D_S2_STEP(SCAN2D_SHL(1)) SCAN2D_S2_STEP(SCAN2D_SHL(2))
                 SCAN2D_S2_STEP(SCAN2D_SHL(4)) SCAN2D_S2_LAST(SCAN2D_SHL(8))
                 "v_mov_b32_dpp %4, %0" SCAN2D_SHL(1) "v_mov_b32_dpp %5, %1" SCAN2D_SHL(1)
                 : "+v"(H0), "+v"(H1), "+v"(P0), "+v"(P1), "+v"(C0), "+v"(C1));
}
__device__ __forceinline__ void row_scan_left4(float& P0, float& P1, float& P2, float& P3,
                                               float& H0, float& H1, float& H2, float& H3,
                                               float& C0, float& C1, float& C2, float& C3) {
    C0 = 0.0f; C1 = 0.0f; C2 = 0.0f; C3 = 0.0f;
    asm volatile("s_nop 1\n\t"
                 SCAN2D_S4_STEP(SCAN2D_SHL(1)) SCAN2D_S4_STEP(SCAN2D_SHL(2))
                 SCAN2D_S4_STEP(SCAN2D_SHL(4)) SCAN2D_S4_LAST(SCAN2D_SHL(8))
                 "v_mov_b32_dpp %8, %0" SCAN2D_SHL(1) "v_mov_b32_dpp %9, %1" SCAN2D_SHL(1)
                 "v_mov_b32_dpp %10, %2" SCAN2D_SHL(1) "v_mov_b32_dpp %11, %3" SCAN2D_SHL(1)
                 : "+v"(H0), "+v"(H1), "+v"(H2), "+v"(H3), "+v"(P0), "+v"(P1), "+v"(P2), "+v"(P3),
                   "+v"(C0), "+v"(C1), "+v"(C2), "+v"(C3));
}

__device__ __forceinline__ float wave_mirror(float v) {
    const int lane = (int)(threadIdx.x & 63u);
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((63 - lane) << 2, __builtin_bit_cast(int, v)));
}

template <int LG, int S>
__device__ __forceinline__ void group_scan_left(float* P, float* Q, float* C) {
    if constexpr (LG == 16) {
        if constexpr (S == 1) row_scan_left1(P[0], Q[0], C[0]);
        else if constexpr (S == 2) row_scan_left2(P[0], P[1], Q[0], Q[1], C[0], C[1]);
        else row_scan_left4(P[0], P[1], P[2], P[3], Q[0], Q[1], Q[2], Q[3], C[0], C[1], C[2], C[3]);
    } else {
        float Pm[S], Qm[S], Cm[S];
#pragma unroll
        for (int t = 0; t < S; ++t) { Pm[t] = wave_mirror(P[t]); Qm[t] = wave_mirror(Q[t]); }
        group_scan<64, S>(Pm, Qm, Cm);
#pragma unroll
        for (int t = 0; t < S; ++t) C[t] = wave_mirror(Cm[t]);
    }
}

// Value held by the lane to the right inside the lane group (0 for the group's last lane).
template <int LG>
__device__ __forceinline__ float from_right(float v) {
    float r = 0.0f;
    if constexpr (LG == 64) asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 wave_shl:1 row_mask:0xf bank_mask:0xf" : "+v"(r) : "v"(v));
    else asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 row_shl:1 row_mask:0xf bank_mask:0xf" : "+v"(r) : "v"(v));
    return r;
}

// Sum over the 16 lanes of a DPP row (every lane of the row gets the total).
__device__ __forceinline__ float row_sum16(float v) {
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_ror:1 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_ror:2 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_ror:4 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
                 : "+v"(v));
    return v;
}

}  // namespace scan2d
