// Shared device-side definitions for the gfx950 kernels (wave64, bf16 MFMA, 160 KB LDS).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// The kernels are templates over the head dimension D (64, 128 or 256).  A row of D bf16 is
// D/8 16-byte chunks; LDS tiles are unpadded and keep chunk c of row r at position c ^ (r & kSwz<D>)
// (see the kernels), where the mask is the row's chunk count minus one, capped at 15.
template <int D> constexpr int kChunks = D / 8;                            // 16-byte chunks per row
template <int D> constexpr int kSwz = (D / 8 < 16 ? D / 8 : 16) - 1;       // chunk permutation mask
template <int D> constexpr int kRowsPerLoad = 512 / D;                     // rows one 1 KB wave-wide load covers
constexpr float kLog2e = 1.4426950408889634f;

// One q-block row.  Queries: first token of the block (index into Q and O) and the number of
// valid tokens in it (1..128).  I = the block's index within its sequence, i.e. its index within
// the query chunk plus the KV prefix in blocks; its causal key blocks are J <= I.  Keys: the
// sequence's first token (index into K and V), one past its last, the first row of its pooled
// keys in the workspace and the number of its key blocks.
struct __attribute__((aligned(16))) RowRec {
    int q_tok0, q_len, I, kb_row0;
    int k_tok0, k_end, n_kb, pad1;
};
// One key block: first token and number of valid tokens.
typedef int2 KeyBlockRec;

#define FP_LDS(T) __attribute__((address_space(3))) T

__device__ __forceinline__ float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// v_mfma_f32_32x32x16_bf16: A is 32x16 (lane l holds row l%32, k = 8*(l/32)..+7), B is 16x32
// (lane l holds column l%32, same k), the 32x32 result keeps column l%32 in lane l and row
// 8*(r/4) + 4*(l/32) + r%4 in register r.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Combine each lane's value with that of lane l ^ 32 through the register swap between the two
// halves of the wave (v_permlane32_swap exchanges the upper half of its first operand with the
// lower half of its second): applied to two copies of x, one register ends up with x[l % 32] and
// the other with x[32 + l % 32] in every lane.  Unlike a shuffle through the LDS crossbar this
// leaves the LDS queue alone, so no wait on outstanding fragment reads is needed around it.
// Written as inline assembly because the compiler's builtin folds the two results into one when
// both inputs are the same value; the s_nop covers the wait states the instruction needs after
// a VALU write of its operands.
__device__ __forceinline__ void halves_swap(float x, float &lo, float &hi) {
    lo = x;
    hi = x;
    asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
}
__device__ __forceinline__ float halves_max(float x) {
    float a, b;
    halves_swap(x, a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float halves_sum(float x) {
    float a, b;
    halves_swap(x, a, b);
    return a + b;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max of three.  The device code is compiled with NaNs not honoured (see build.py), so this
// becomes one v_max3_f32 instead of three canonicalising v_max_f32 plus the max itself.  It must
// stay a compiler-visible instruction: the wait states the hardware needs between an MFMA and a
// VALU read of its result are inserted by the compiler, and inline assembly would not get them.
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// 16 bytes per lane, global -> LDS, no register staging: lane i's 16 bytes, fetched from
// sbase + voff, land at LDS byte address lds_addr + 16 i (lds_addr is wave-uniform and goes to
// M0).  Written as inline assembly on purpose: the compiler then neither tracks these loads in
// vmcnt nor orders LDS reads after them (it would wait for *all* outstanding loads before the
// first LDS read of every step, which defeats the prefetch).  Completion is waited for
// explicitly with FP_WAIT_VMCNT followed by a workgroup barrier.
// M0 is named as clobbered so that the compiler does not keep a value of its own in it across
// the statement; it answers with a warning that it will not save and restore a reserved register
// for us, which is what is wanted here (no code in these kernels needs M0 otherwise).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds(const char *sbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

// s_waitcnt vmcnt(n) alone (expcnt and lgkmcnt left at "no wait"), n < 64: the count's low four
// bits sit in bits 3:0 of the immediate, its high two in bits 15:14
#define FP_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))

}  // namespace fp
