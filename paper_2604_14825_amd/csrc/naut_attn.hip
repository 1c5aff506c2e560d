// naut_attn.hip -- fused attention forward for gfx950 (MI355X) and its C ABI.
//
// One kernel computes O = softmax(scale * Q K^T + causal mask) V for a
// (batch, head, 128-query tile) per work-group.  The reductions over the key
// axis (row max, row sum, weighted sum of V) are fused with the rolling-update
// scheme of Section 4.2/4.3 of the paper: a running maximum m and running sum l
// are kept per query, and whenever m grows the partial results are repaired by
// the factor exp2(m_old - m_new).  The S x S scores never leave registers.
// Hand-applied rewrites (table of Section 5): scale*log2(e) folded into one
// constant, exp -> exp2, and a single division by l in the epilogue instead of
// one per step.
//
// Work decomposition (bi-level tiling, Section 4.2): outer loops (batch, head,
// query tile) -> work-groups; inner tile = 128 queries x 64 keys.  A work-group
// has 4 wavefronts, each owning 32 queries.  Per key tile and wavefront:
//
//   S^T[key][query] = K_tile . Q^T     v_mfma_f32_32x32x16 (A = K from LDS, B = Q in registers)
//   online softmax over keys           each lane owns ONE query (column) and 16 keys per 32-key block,
//                                      so row max / row sum are in-lane plus one exchange between the
//                                      two 32-lane halves
//   O^T[d][query] += V^T . P^T         A = V^T (LDS transpose read), B = P^T taken straight from the
//                                      S^T accumulator registers (no shuffle: the MFMA k-slot <-> key
//                                      assignment is chosen to match the accumulator layout)
//
// K and V tiles are double-buffered in LDS (global -> registers -> LDS, one
// barrier per step).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "naut_attn.h"

namespace {

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

constexpr int BM = 128;  // queries per work-group
constexpr int BN = 64;   // keys per step
constexpr int NWAVES = 4;
constexpr int NTHREADS = NWAVES * 64;
constexpr float RESCALE_TAU = 6.0f;  // log2 units

struct Params {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    float* lse;
    int B, Hq, Hkv, S;
    int nqt;       // number of query tiles = ceil(S / BM)
    float c;       // scale * log2(e), > 0
};

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
    return (line << 8) + ((pos ^ (line & 15)) << 4);
}

// V is read transposed: one wavefront-wide read touches 8 consecutive rows x 64
// bytes, so the 64-byte quarter of the 256-byte line is XOR-ed with the row
// number to put the rows of one read in different quarters.
template <int D>
__device__ __forceinline__ int v_off(int row, int c)
{
    if constexpr (D == 128)
        return row * 256 + ((c ^ ((row & 3) << 2)) << 4);
    else
        return row * 128 + ((c ^ (((row >> 1) & 1) << 2)) << 4);
}

// 8 values V[key(slot)][d] for the MFMA A operand of the P.V product.
// The lane owns output row d = 32*db + lane%32 and k-slots 8h..8h+7 (h = lane/32),
// which stand for keys kbase + 4h + {0..3} and kbase + 8 + 4h + {0..3}.
template <int D, bool VTR>
__device__ __forceinline__ i32x4_t load_vt_frag(const unsigned char* vt, int kbase, int db, int lane)
{
    const int h = lane >> 5;
    if constexpr (VTR) {
        // ds_read_b64_tr_b16: within each 16-lane group, lane i supplies the address of 4 consecutive
        // d of key (i/4) and receives the 4 keys of d = i.
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
    } else {
        const int d = 32 * db + (lane & 31);
        unsigned short e[8];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int key = kbase + 8 * a + 4 * h + i;
                e[4 * a + i] = *(const unsigned short*)(vt + v_off<D>(key, d >> 3) + (d & 7) * 2);
            }
        i32x4_t out = {(int)(e[0] | ((unsigned)e[1] << 16)), (int)(e[2] | ((unsigned)e[3] << 16)),
                       (int)(e[4] | ((unsigned)e[5] << 16)), (int)(e[6] | ((unsigned)e[7] << 16))};
        return out;
    }
}

// max over the two 32-lane halves.  v_permlane32_swap exchanges the upper 32 lanes of its first
// operand with the lower 32 lanes of its second, so afterwards (a, b) = (x[lane%32], x[lane%32+32])
// in every lane.  Written as inline asm: the compiler folds the two results of the corresponding
// builtin into one.
__device__ __forceinline__ float half_max(float x)
{
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return fmaxf(a, b);
}

// ---- the kernel ------------------------------------------------------------------

template <int D, int DT_IN, int DT_OUT, bool CAUSAL, bool VTR>
__global__ __launch_bounds__(NTHREADS, 2) void naut_fwd_kernel(const Params p)
{
    using T = In<DT_IN>;
    constexpr int ROWB = D * 2;              // bytes per K/V row
    constexpr int TILEB = BN * ROWB;         // bytes per K or V tile
    constexpr int CPR = D / 8;               // 16-byte chunks per row
    constexpr int LD_PER_T = BN * CPR / NTHREADS;  // chunks per thread per tile
    constexpr int KS = D / 16;               // MFMA k-steps of Q.K^T
    constexpr int DB = D / 32;               // 32-row blocks of O^T
    constexpr int KB = BN / 32;              // 32-key blocks of S^T

    __shared__ __attribute__((aligned(256))) unsigned char smem[4 * TILEB];  // K0 V0 K1 V1

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // Tile scheduler: heaviest (last) query tiles first; consecutive block ids walk the
    // (batch, head) axis so that each XCD (block id mod 8) keeps to a fixed subset of heads.
    const int nbh = p.B * p.Hq;
    const int bid = blockIdx.x;
    const int qt = p.nqt - 1 - bid / nbh;
    const int bh = bid % nbh;
    const int b = bh / p.Hq;
    const int hq = bh % p.Hq;
    const int hk = hq / (p.Hq / p.Hkv);
    const int S = p.S;

    const unsigned char* qg = (const unsigned char*)p.q + (size_t)bh * S * ROWB;
    const unsigned char* kg = (const unsigned char*)p.k + (size_t)(b * p.Hkv + hk) * S * ROWB;
    const unsigned char* vg = (const unsigned char*)p.v + (size_t)(b * p.Hkv + hk) * S * ROWB;

    const int q_wave0 = qt * BM + wave * 32;  // first query of this wavefront
    const int my_q = q_wave0 + l32;           // the query this lane owns
    const int my_q_ld = my_q < S ? my_q : S - 1;

    // Q^T fragments (MFMA B operand): lane holds q[my_q][16*ks + 8*h .. +8].
    i32x4_t qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        qf[ks] = *(const i32x4_t*)(qg + (size_t)my_q_ld * ROWB + ks * 32 + h * 16);
    // Keep Q resident: without this the compiler re-issues the global loads inside the key loop.
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        asm volatile("" : "+v"(qf[ks]));

    const int kv_end = CAUSAL ? (S < (qt + 1) * BM ? S : (qt + 1) * BM) : S;
    const int ntiles = (kv_end + BN - 1) / BN;

    // global -> register staging of one K and one V tile
    i32x4_t kst[LD_PER_T], vst[LD_PER_T];
    auto g_load = [&](int tile) {
#pragma unroll
        for (int i = 0; i < LD_PER_T; ++i) {
            const int L = tid + NTHREADS * i;
            int row = tile * BN + L / CPR;
            row = row < S ? row : S - 1;
            const size_t off = (size_t)row * ROWB + (L % CPR) * 16;
            kst[i] = *(const i32x4_t*)(kg + off);
            vst[i] = *(const i32x4_t*)(vg + off);
        }
    };
    auto s_store = [&](int buf) {
        unsigned char* kt = smem + buf * 2 * TILEB;
        unsigned char* vt = kt + TILEB;
#pragma unroll
        for (int i = 0; i < LD_PER_T; ++i) {
            const int L = tid + NTHREADS * i;
            *(i32x4_t*)(kt + k_off<D>(L / CPR, L % CPR)) = kst[i];
            *(i32x4_t*)(vt + v_off<D>(L / CPR, L % CPR)) = vst[i];
        }
    };

    f32x16_t oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            oacc[db][r] = 0.f;
    float m_run = -INFINITY;  // running max, in the exp2 domain (already times c)
    float l_run = 0.f;        // this lane's share of the running sum (its 16 of every 32 keys)
    const float c = p.c;

    g_load(0);
    s_store(0);
    __syncthreads();

    for (int j = 0; j < ntiles; ++j) {
        const int buf = j & 1;
        const unsigned char* kt = smem + buf * 2 * TILEB;
        const unsigned char* vt = kt + TILEB;
        const int kv0 = j * BN;
        if (j + 1 < ntiles)
            g_load(j + 1);

        // Causal block skipping per wavefront: nothing to do if every key of the tile lies
        // beyond this wavefront's last query.
        const bool active = !CAUSAL || kv0 <= q_wave0 + 31;
        if (active) {
            f32x16_t sacc[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    sacc[kb][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const i32x4_t kf = *(const i32x4_t*)(kt + k_off<D>(kb * 32 + l32, ks * 2 + h));
                    sacc[kb] = T::mfma(kf, qf[ks], sacc[kb]);
                }
            }
            // Mask only where the tile straddles the diagonal or the end of the sequence.
            const bool need_mask = (CAUSAL && kv0 + BN - 1 > q_wave0) || (kv0 + BN > S);
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kv0 + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        const bool dead = (CAUSAL && key > my_q) || key >= S;
                        sacc[kb][r] = dead ? -INFINITY : sacc[kb][r];
                    }
            }
            // running max over keys: in-lane, then across the two 32-lane halves
            float mx = sacc[0][0];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    mx = fmaxf(mx, sacc[kb][r]);
            mx = half_max(mx);
            // The reference maximum only has to be *a* bound shared by l and O, not the exact running
            // maximum: it is moved (and the partial sums repaired) only when some query of this
            // wavefront exceeds it by more than 2^RESCALE_TAU, which keeps every P below that factor.
            const float m_cand = mx * c;
            const bool grow = m_cand > m_run + RESCALE_TAU;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float m_new = fmaxf(m_run, m_cand);
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // repair factor
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        oacc[db][r] *= alpha;
            }
            const float m_new = m_run;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][r], c, -m_new));
                    sacc[kb][r] = pv;
                    psum += pv;
                }
            l_run += psum;
            // O^T += V^T . P^T, 16 keys per MFMA
#pragma unroll
            for (int t = 0; t < BN / 16; ++t) {
                const int kb = t >> 1, r0 = (t & 1) * 8;
                i32x4_t pb = {T::pack2(sacc[kb][r0 + 0], sacc[kb][r0 + 1]), T::pack2(sacc[kb][r0 + 2], sacc[kb][r0 + 3]),
                              T::pack2(sacc[kb][r0 + 4], sacc[kb][r0 + 5]), T::pack2(sacc[kb][r0 + 6], sacc[kb][r0 + 7])};
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const i32x4_t vf = load_vt_frag<D, VTR>(vt, t * 16, db, lane);
                    oacc[db] = T::mfma(vf, pb, oacc[db]);
                }
            }
        }
        if (j + 1 < ntiles)
            s_store(buf ^ 1);
        __syncthreads();
    }

    // Epilogue: one division by l (the per-step divide/multiply pairs telescope away), lse, store.
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv_l = 1.0f / l_tot;
    if (my_q < S) {
        if (p.lse != nullptr && h == 0)
            p.lse[(size_t)bh * S + my_q] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
        constexpr int OUTB = DT_OUT == NAUT_F32 ? 4 : 2;
        unsigned char* og = (unsigned char*)p.o + ((size_t)bh * S + my_q) * D * OUTB;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * db + 8 * g + 4 * h;
                const float x0 = oacc[db][4 * g + 0] * inv_l, x1 = oacc[db][4 * g + 1] * inv_l;
                const float x2 = oacc[db][4 * g + 2] * inv_l, x3 = oacc[db][4 * g + 3] * inv_l;
                if constexpr (DT_OUT == NAUT_F32) {
                    f32x4_t w = {x0, x1, x2, x3};
                    *(f32x4_t*)(og + d * 4) = w;
                } else {
                    i32x2_t w = {In<DT_OUT>::pack2(x0, x1), In<DT_OUT>::pack2(x2, x3)};
                    *(i32x2_t*)(og + d * 2) = w;
                }
            }
    }
}

// ---- host side ---------------------------------------------------------------------

thread_local char g_err[256] = "";

int fail(int code, const char* msg)
{
    snprintf(g_err, sizeof g_err, "%s", msg);
    return code;
}

bool use_vtr()
{
    const char* e = getenv("NAUT_ATTN_VTR");
    return e == nullptr || e[0] != '0';
}

template <int D, int DT_IN, int DT_OUT>
int launch(const Params& p, int causal, hipStream_t stream)
{
    const long long nblocks = (long long)p.nqt * p.B * p.Hq;
    if (nblocks > 0x7fffffffLL)
        return fail(NAUT_ERR_UNSUPPORTED, "B*Hq*ceil(S/128) exceeds the 1-D grid limit");
    const dim3 grid((unsigned)nblocks), block(NTHREADS);
    const bool vtr = use_vtr();
    if (causal) {
        if (vtr)
            hipLaunchKernelGGL((naut_fwd_kernel<D, DT_IN, DT_OUT, true, true>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((naut_fwd_kernel<D, DT_IN, DT_OUT, true, false>), grid, block, 0, stream, p);
    } else {
        if (vtr)
            hipLaunchKernelGGL((naut_fwd_kernel<D, DT_IN, DT_OUT, false, true>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((naut_fwd_kernel<D, DT_IN, DT_OUT, false, false>), grid, block, 0, stream, p);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_err, sizeof g_err, "kernel launch failed: %s", hipGetErrorString(e));
        return NAUT_ERR_HIP;
    }
    return NAUT_OK;
}

bool dtype_pair_ok(int in_dtype, int out_dtype)
{
    if (in_dtype != NAUT_BF16 && in_dtype != NAUT_F16)
        return false;
    return out_dtype == in_dtype || out_dtype == NAUT_F32;
}

}  // namespace

extern "C" {

int naut_attn_fwd_dt(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                     int S, int D, int causal, float scale, void* stream, int in_dtype, int out_dtype)
{
    if (!q || !k || !v || !o)
        return fail(NAUT_ERR_NULL, "q, k, v and o must be non-NULL device pointers");
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || S <= 0 || D <= 0)
        return fail(NAUT_ERR_SHAPE, "B, Hq, Hkv, S and D must be positive");
    if (Hq % Hkv != 0)
        return fail(NAUT_ERR_SHAPE, "Hq must be a multiple of Hkv");
    if (!std::isfinite(scale))
        return fail(NAUT_ERR_SHAPE, "scale must be finite");
    if (scale < 0.f)
        return fail(NAUT_ERR_UNSUPPORTED, "negative scale is not supported");
    if (D != 64 && D != 128)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be 64 or 128");
    if (!dtype_pair_ok(in_dtype, out_dtype))
        return fail(NAUT_ERR_UNSUPPORTED, "supported dtypes: q/k/v bf16 or f16; o of the same type or f32");
    if ((long long)B * Hq > 0x7fffffffLL || (long long)B * Hkv > 0x7fffffffLL)
        return fail(NAUT_ERR_UNSUPPORTED, "B*Hq too large");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15u)
        return fail(NAUT_ERR_ALIGN, "q, k, v and o must be 16-byte aligned");
    if ((uintptr_t)lse & 3u)
        return fail(NAUT_ERR_ALIGN, "lse must be 4-byte aligned");

    Params p;
    p.q = q;
    p.k = k;
    p.v = v;
    p.o = o;
    p.lse = lse;
    p.B = B;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.S = S;
    p.nqt = (S + BM - 1) / BM;
    // exp(x) = exp2(log2(e) x); the constant is hoisted out of the key loop.  A zero scale is
    // replaced by the smallest useful positive constant so that masked scores (-inf) stay -inf.
    const float c = scale * 1.4426950408889634f;
    p.c = c > 0.f ? c : 1e-30f;
    hipStream_t st = (hipStream_t)stream;

#define NAUT_DISPATCH(DD, IN, OUT)                         \
    if (D == DD && in_dtype == IN && out_dtype == OUT)    \
        return launch<DD, IN, OUT>(p, causal, st);
    NAUT_DISPATCH(128, NAUT_BF16, NAUT_BF16)
    NAUT_DISPATCH(64, NAUT_BF16, NAUT_BF16)
    NAUT_DISPATCH(128, NAUT_BF16, NAUT_F32)
    NAUT_DISPATCH(64, NAUT_BF16, NAUT_F32)
    NAUT_DISPATCH(128, NAUT_F16, NAUT_F16)
    NAUT_DISPATCH(64, NAUT_F16, NAUT_F16)
    NAUT_DISPATCH(128, NAUT_F16, NAUT_F32)
    NAUT_DISPATCH(64, NAUT_F16, NAUT_F32)
#undef NAUT_DISPATCH
    return fail(NAUT_ERR_UNSUPPORTED, "no kernel for this (D, dtype) combination");
}

int naut_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int S,
                  int D, int causal, float scale, void* stream)
{
    return naut_attn_fwd_dt(q, k, v, o, lse, B, Hq, Hkv, S, D, causal, scale, stream, NAUT_BF16, NAUT_BF16);
}

const char* naut_last_error_string(void) { return g_err; }

int naut_version(void) { return 100; }

const char* naut_attn_variant_name(int S, int D, int causal, int in_dtype, int out_dtype)
{
    (void)S;
    (void)causal;
    if ((D != 64 && D != 128) || !dtype_pair_ok(in_dtype, out_dtype))
        return nullptr;
    return D == 128 ? "fwd_d128_bm128_bn64_w4" : "fwd_d64_bm128_bn64_w4";
}

}  // extern "C"
