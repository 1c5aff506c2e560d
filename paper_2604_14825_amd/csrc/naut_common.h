// naut_common.h -- device-side pieces shared by the attention kernels of this library (gfx950).
#ifndef NAUT_COMMON_H
#define NAUT_COMMON_H
#include <hip/hip_runtime.h>

#include <type_traits>

#include <cstdint>

#include "naut_attn.h"

namespace naut {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x2_t __attribute__((ext_vector_type(2)));
typedef short i16x4_t __attribute__((ext_vector_type(4)));

#define NAUT_LDS __attribute__((address_space(3)))

// ---- hand-made synchronisation, and the build that checks it -----------------------------------------
// The kernels publish direct-to-LDS tile loads with bare s_barrier instructions, count their own loads in
// flight (s_waitcnt vmcnt(n)) and owe a few wait states around instructions written as asm.  A library built
// with -DNAUT_SAFE_SYNC=1 replaces all of that by the most conservative form: every such barrier first waits
// for every memory operation of the wavefront and is a full __syncthreads(); every counted wait is a wait for
// all loads; tile loads are issued, awaited and published before the step that issued them computes anything
// (nothing is in flight during compute: single-stage); and every owed wait state is paid several times over.
// The arithmetic and its order are the same, so the two builds must agree bit for bit; a difference is a race
// or a missing wait in the fast build (tests/test_safe_sync_gpu.py compares them).
#ifndef NAUT_SAFE_SYNC
#define NAUT_SAFE_SYNC 0
#endif
constexpr bool SAFE_SYNC = NAUT_SAFE_SYNC != 0;
#if NAUT_SAFE_SYNC
#define NAUT_NOP_SHORT "s_nop 7\n\t"                         /* in place of the 1 or 2 wait states owed */
#define NAUT_NOP_AFTER_MFMA "\n\ts_nop 15\n\ts_nop 15"         /* 32 wait states behind every asm MFMA */
#define NAUT_NOP_SETTLE "s_nop 15\n\ts_nop 15"
#else
#define NAUT_NOP_SHORT "s_nop 1\n\t"
#define NAUT_NOP_AFTER_MFMA ""
#define NAUT_NOP_SETTLE "s_nop 11"
#endif

// The barrier that publishes tile loads (the loads to be published have been awaited by their wavefronts).
__device__ __forceinline__ void tile_barrier()
{
    if constexpr (SAFE_SYNC) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
    } else {
        asm volatile("s_barrier" ::: "memory");
    }
}
// Waits until at most N of this wavefront's vector memory operations are still in flight.
template <int N>
__device__ __forceinline__ void wait_loads()
{
    static_assert(N >= 0 && N < 64, "vmcnt field");
    if constexpr (SAFE_SYNC)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// One 1 KB direct global->LDS load: lane i's 16 bytes from `base` + `off` land at LDS address `dst` + 16 i.
// asm, so that the compiler does not make every later LDS read wait for these loads; their completion is
// awaited explicitly (wait_loads) before the barrier that publishes the tile.
__device__ __forceinline__ void load_to_lds(unsigned dst, int off, const unsigned char* base)
{
#if NAUT_SAFE_SYNC
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 7\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"(off), "s"(base) : "memory", "m0");
#else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"(off), "s"(base) : "memory", "m0");
#endif
}

// f(integral_constant<int, I>) for I = I0 .. N-1, unrolled at compile time
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// ---- per-dtype pieces ------------------------------------------------------

template <int DT>
struct In;

template <>
struct In<NAUT_BF16> {
    static __device__ __forceinline__ f32x16_t mfma(i32x4_t a, i32x4_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ int pack2(float lo, float hi)
    {
        f32x2_t f = {lo, hi};
        return __builtin_bit_cast(int, __builtin_convertvector(f, bf16x2_t));
    }
    // acc + the two 16-bit values of `packed`, in fp32 (v_dot2c_f32_bf16 against a pair of ones)
    static __device__ __forceinline__ float add_pair(int packed, float acc)
    {
        const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, packed), ones, acc, false);
    }
    // a block's row sum of P above this moves the reference maximum (P itself must stay representable)
    static constexpr float P_LIMIT = 1073741824.0f;  // 2^30
};

template <>
struct In<NAUT_F16> {
    static __device__ __forceinline__ f32x16_t mfma(i32x4_t a, i32x4_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ int pack2(float lo, float hi)
    {
        f32x2_t f = {lo, hi};
        return __builtin_bit_cast(int, __builtin_convertvector(f, f16x2_t));
    }
    static __device__ __forceinline__ float add_pair(int packed, float acc)
    {
        const f16x2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, packed), ones, acc, false);
    }
    static constexpr float P_LIMIT = 1024.0f;  // f16 ends at 65504
};

// ---- LDS layouts -------------------------------------------------------------
// Both tiles hold BN rows of D 16-bit values.  Addresses are byte offsets inside
// one tile; `c` counts 16-byte chunks inside a row.
//
// K is read as the MFMA A operand: 32 lanes read the same chunk of 32
// consecutive rows, so the chunk position is XOR-ed with the 256-byte line
// number to spread those reads over all banks.
template <int D>
__device__ __forceinline__ int k_off(int row, int c)
{
    constexpr int CPR = D / 8;  // chunks per row
    const int L = row * CPR + c;
    const int line = L >> 4, pos = L & 15;
    // A 512-byte row (D = 256) spans two lines: the key is the row number there, so that 16 consecutive
    // rows still take 16 different positions.
    const int key = CPR > 16 ? line >> 1 : line;
    return (line << 8) + ((pos ^ (key & 15)) << 4);
}

// V is read transposed: one wavefront-wide read touches 8 consecutive rows x 64
// bytes, so the 64-byte quarter of the 256-byte line is XOR-ed with the row
// number to put the rows of one read in different quarters.
template <int D>
__device__ __forceinline__ int v_off(int row, int c)
{
    if constexpr (D >= 128)
        return row * (D * 2) + ((c ^ ((row & 3) << 2)) << 4);
    else
        return row * 128 + ((c ^ (((row >> 1) & 1) << 2)) << 4);
}

// 8 values V[key(slot)][d] for the MFMA A operand of the P.V product.
// The lane owns output row d = 32*db + lane%32 and k-slots 8h..8h+7 (h = lane/32),
// which stand for keys kbase + 4h + {0..3} and kbase + 8 + 4h + {0..3}.
// ds_read_b64_tr_b16: within each 16-lane group, lane i supplies the address of 4 consecutive d of
// key (i/4) and receives the 4 keys of d = i.
template <int D>
__device__ __forceinline__ i32x4_t load_vt_frag(const unsigned char* vt, int kbase, int db, int lane)
{
    const int h = lane >> 5;
    const int i16 = lane & 15;
    const int d = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
    const int key = kbase + 4 * h + (i16 >> 2);
    const int a0 = v_off<D>(key, d >> 3) + (d & 7) * 2;
    const int a1 = v_off<D>(key + 8, d >> 3) + (d & 7) * 2;
    i16x4_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((NAUT_LDS i16x4_t*)(vt + a0));
    i16x4_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((NAUT_LDS i16x4_t*)(vt + a1));
    i32x2_t lo = __builtin_bit_cast(i32x2_t, r0);
    i32x2_t hi = __builtin_bit_cast(i32x2_t, r1);
    i32x4_t out = {lo.x, lo.y, hi.x, hi.y};
    return out;
}

// max over the two 32-lane halves.  v_permlane32_swap exchanges the upper 32 lanes of its first
// operand with the lower 32 lanes of its second, so afterwards (a, b) = (x[lane%32], x[lane%32+32])
// in every lane.  Written as inline asm: the compiler folds the two results of the corresponding
// builtin into one.
__device__ __forceinline__ float half_max(float x)
{
    float a = x, b = x;
    asm volatile(NAUT_NOP_SHORT "v_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return fmaxf(a, b);
}

// ---- FP8 (E4M3) pieces shared by the prefill and the decode kernel ----------------------------

typedef int i32x8_t __attribute__((ext_vector_type(8)));

// K tile: 64 rows of D bytes; the 16-byte chunks of a row are XOR-ed with (row/2), so that the 32 lanes
// that read the same chunk of 32 consecutive rows cover all banks (measured: no bank conflicts).
template <int D>
__device__ __forceinline__ int k8_off(int row, int c16)
{
    constexpr int CPR = D / 16;
    return row * D + ((c16 ^ ((row >> 1) & (CPR - 1))) << 4);
}
// V tile: rows of D bytes in 32-byte chunks.  One transposed read touches, per half of the wavefront, 8
// rows (r0 + {0,1,2,3,8,9,10,11}) x 32 bytes = 256 bytes, one access per bank if the 8 rows land in 8
// different bank groups: row parity gives two (128-byte rows) and the chunk position is XOR-ed with bits
// 1 and 3 of the row number for the other four (D = 64: 64-byte rows, bits 0..1 give four, bit 3 the rest).
template <int D>
__device__ __forceinline__ int v8_off(int row, int c32)
{
    const int key = D == 128 ? (((row >> 1) & 1) | (((row >> 3) & 1) << 1)) : ((row >> 3) & 1);
    return row * D + ((c32 ^ key) << 5);
}

// Four floats to four E4M3 bytes.  The conversion writes one 16-bit half of its destination and keeps the
// other; `old` is whatever the register held (both halves get written, so it only saves the instruction
// that would clear it).
__device__ __forceinline__ int pack4_fp8(float x0, float x1, float x2, float x3, int old)
{
    const int w = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, old, false);
    return __builtin_amdgcn_cvt_pk_fp8_f32(x2, x3, w, true);
}

// ---- host side: the calling thread's last error (defined next to the C ABI entry points) ----
extern thread_local char g_err[256];
int fail(int code, const char* msg);   // records msg, returns code
int fail_launch(hipError_t e);         // records the HIP error text, returns NAUT_ERR_HIP

}  // namespace naut

#endif  // NAUT_COMMON_H
