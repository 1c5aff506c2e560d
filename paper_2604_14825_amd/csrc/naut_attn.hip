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
#include <type_traits>

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
    int nqt;       // number of 128-query tiles = ceil(S / BM)
    int nqt2;      // number of 256-query tiles
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

// ---- kernel 2: 64 queries per wavefront, software-pipelined over 32-key blocks -------------
//
// A work-group owns 256 queries (4 wavefronts x 64); each lane owns two queries (one in each
// 32-query half, "A" and "B").  Every K fragment and every V^T fragment read from LDS feeds two
// MFMAs (half A and half B), which halves LDS traffic per FLOP compared with 32 queries per
// wavefront.  With one wavefront per SIMD, matrix and vector work overlap inside the wavefront:
// the key axis is processed in 32-key blocks and stage k issues
//
//     MFMA:  Y(k-1) = O^T += V^T . P^T of block k-1      VALU:  SM(k) = online softmax of block k
//            X(k+1) = S^T of block k+1
//
// so the MFMAs of a stage never depend on its vector work.  K and V tiles (64 keys) are
// triple-buffered in LDS and filled by direct global->LDS loads, one barrier per tile.

constexpr int BM2 = 256;
constexpr int NBUF = 3;

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// sum over the two 32-lane halves (same exchange as half_max)
__device__ __forceinline__ float half_sum(float x)
{
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}

template <int D, int DT_IN, int DT_OUT, bool CAUSAL>
__global__ __launch_bounds__(NTHREADS, 1) void naut_fwd_kernel_v2(const Params p)
{
    using T = In<DT_IN>;
    constexpr int ROWB = D * 2;
    constexpr int TILEB = BN * ROWB;           // one 64-key K or V tile
    constexpr int CPR = D / 8;
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int LD_PER_W = TILEB / 1024 / NWAVES;  // direct loads per wavefront per tile (1 KB each)

    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * NBUF * TILEB];  // K0 K1 K2 V0 V1 V2
    unsigned char* const k_lds = smem;
    unsigned char* const v_lds = smem + NBUF * TILEB;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    const int nbh = p.B * p.Hq;
    const int bid = blockIdx.x;
    const int qt = p.nqt2 - 1 - bid / nbh;   // heaviest query tiles first
    const int bh = bid % nbh;
    const int b = bh / p.Hq;
    const int hq = bh % p.Hq;
    const int hk = hq / (p.Hq / p.Hkv);
    const int S = p.S;
    const float c = p.c;

    const unsigned char* qg = (const unsigned char*)p.q + (size_t)bh * S * ROWB;
    const unsigned char* kg = (const unsigned char*)p.k + (size_t)(b * p.Hkv + hk) * S * ROWB;
    const unsigned char* vg = (const unsigned char*)p.v + (size_t)(b * p.Hkv + hk) * S * ROWB;

    const int Q0 = qt * BM2 + wave * 64;  // first query of this wavefront
    const int qa = Q0 + l32, qb = Q0 + 32 + l32;

    // Q^T fragments of both halves (MFMA B operands), resident for the whole kernel.
    i32x4_t qfa[KS], qfb[KS];
    {
        const int qa_ld = qa < S ? qa : S - 1, qb_ld = qb < S ? qb : S - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qfa[ks] = *(const i32x4_t*)(qg + (size_t)qa_ld * ROWB + ks * 32 + h * 16);
            qfb[ks] = *(const i32x4_t*)(qg + (size_t)qb_ld * ROWB + ks * 32 + h * 16);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            asm volatile("" : "+v"(qfa[ks]));
            asm volatile("" : "+v"(qfb[ks]));
        }
    }

    // Key blocks (32 keys) this wavefront / this work-group has to visit.
    const int kv_end_wg = CAUSAL ? (S < (qt + 1) * BM2 ? S : (qt + 1) * BM2) : S;
    const int kv_end_w = Q0 >= S ? 0 : (CAUSAL ? (S < Q0 + 64 ? S : Q0 + 64) : S);
    const int nb_w = (kv_end_w + 31) >> 5;
    const int nb_wg = (kv_end_wg + 31) >> 5;
    const int ntiles = (kv_end_wg + BN - 1) / BN;
    const int niter = (nb_wg + 2) >> 1;  // stages 0..nb_wg, two per iteration

    // Direct global->LDS tile loads.  Each instruction moves 1 KB: lane i fills physical chunk i of
    // the block, so the lane fetches the logical chunk that the swizzle maps there.
    int k_goff[LD_PER_W], v_goff[LD_PER_W], k_grow[LD_PER_W], v_grow[LD_PER_W];
#pragma unroll
    for (int i = 0; i < LD_PER_W; ++i) {
        const int P = (wave * LD_PER_W + i) * 64 + lane;  // physical chunk index in the tile
        {
            const int line = P >> 4, pos = P & 15;
            const int L = (line << 4) + (pos ^ (line & 15));
            k_grow[i] = L / CPR;
            k_goff[i] = (L % CPR) * 16;
        }
        if constexpr (D == 128) {
            const int row = P >> 4, cc = P & 15;
            v_grow[i] = row;
            v_goff[i] = (cc ^ ((row & 3) << 2)) * 16;
        } else {
            const int row = P >> 3, cc = P & 7;
            v_grow[i] = row;
            v_goff[i] = (cc ^ (((row >> 1) & 1) << 2)) * 16;
        }
    }
    auto load_tile = [&](const unsigned char* g, unsigned char* lds_tiles, int tile, const int* grow, const int* goff) {
        unsigned char* dst = lds_tiles + (tile % NBUF) * TILEB + wave * LD_PER_W * 1024;
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i) {
            int row = tile * BN + grow[i];
            row = row < S ? row : S - 1;
            const unsigned char* src = g + (size_t)row * ROWB + goff[i];
            // Written as asm so that the compiler does not make every later LDS read wait for these
            // loads; completion is awaited explicitly (vmcnt) before the barrier that publishes the tile.
            const unsigned lds_addr = (unsigned)(uintptr_t)(NAUT_LDS unsigned char*)(dst + i * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :
                         : "s"(lds_addr), "v"(src)
                         : "memory", "m0");
        }
    };

    f32x16_t oa[DB], ob[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            oa[db][r] = 0.f;
            ob[db][r] = 0.f;
        }
    float ma = -INFINITY, mb = -INFINITY, la = 0.f, lb = 0.f;

    // ---- pipeline pieces ----
    // X(kblk): S^T of 32-key block kblk for both halves.
    auto stage_x = [&](int kblk, f32x16_t& sa, f32x16_t& sb) {
        const unsigned char* kt = k_lds + ((kblk >> 1) % NBUF) * TILEB;
        const int row = (kblk & 1) * 32 + l32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            sa[r] = 0.f;
            sb[r] = 0.f;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const i32x4_t kf = *(const i32x4_t*)(kt + k_off<D>(row, ks * 2 + h));
            sa = T::mfma(kf, qfa[ks], sa);
            sb = T::mfma(kf, qfb[ks], sb);
        }
    };
    // Y(kblk): O^T += V^T . P^T over the 32 keys of block kblk.
    auto stage_y = [&](int kblk, const i32x4_t (&pa)[2], const i32x4_t (&pb)[2]) {
        const unsigned char* vt = v_lds + ((kblk >> 1) % NBUF) * TILEB;
        const int kbase = (kblk & 1) * 32;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const i32x4_t vf = load_vt_frag<D, true>(vt, kbase + 16 * t, db, lane);
                oa[db] = T::mfma(vf, pa[t], oa[db]);
                ob[db] = T::mfma(vf, pb[t], ob[db]);
            }
    };
    // SM(kblk), first part: masking (if asked) and the new reference maxima / repair factors.
    auto mask_block = [&](int kblk, f32x16_t& sa, f32x16_t& sb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kblk * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            const bool oob = key >= kv_end_w;  // beyond the sequence, or beyond this wavefront's last block
            sa[r] = (oob || (CAUSAL && key > qa)) ? -INFINITY : sa[r];
            sb[r] = (oob || (CAUSAL && key > qb)) ? -INFINITY : sb[r];
        }
    };
    auto row_max16 = [&](const f32x16_t& s) {
        float m0 = fmaxf(s[0], s[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2)
            m0 = fmaxf(m0, fmaxf(s[r], s[r + 1]));
        return half_max(m0);
    };
    // exponentials, row sums and the packed P^T operands of one half
    auto exp_pack = [&](f32x16_t& s, float m_new, float& psum, i32x4_t (&pp)[2]) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -m_new));
            psum += s[r];
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            i32x4_t w = {T::pack2(s[8 * t + 0], s[8 * t + 1]), T::pack2(s[8 * t + 2], s[8 * t + 3]),
                         T::pack2(s[8 * t + 4], s[8 * t + 5]), T::pack2(s[8 * t + 6], s[8 * t + 7])};
            pp[t] = w;
        }
    };

    // One pipeline stage k: Y(k-1) and X(k+1) on the matrix pipe, SM(k) on the vector ALU.  Every
    // wavefront runs every stage: Y(-1) is issued with P = 0, X past the last block computes scores
    // nobody reads, and SM of a block past this wavefront's last one is fully masked (P = 0, no
    // change of m or l), so one straight-line body serves every k and the loop has a single path.
    //
    // The body is written as 2*KS "units" of two MFMAs (one LDS fragment feeding half A and half B),
    // alternating Y and X units, each followed by a slice of the softmax arithmetic; scheduling
    // fences between units keep that interleaving (and keep LDS reads just two units ahead of their
    // use, which bounds the registers they occupy).
    auto stage = [&](int k, bool masked, f32x16_t& sa_cur, f32x16_t& sb_cur, f32x16_t& sa_nxt, f32x16_t& sb_nxt,
                     const i32x4_t (&pa_in)[2], const i32x4_t (&pb_in)[2], i32x4_t (&pa_out)[2],
                     i32x4_t (&pb_out)[2]) {
        if (masked)
            mask_block(k, sa_cur, sb_cur);
        constexpr int NU = 2 * KS;       // units: even = Y (V^T fragment), odd = X (K fragment)
        constexpr int NYU = 2 * DB;      // Y units that exist (== KS for D = 128 and D = 64)
        static_assert(NYU == KS, "Y and X units must pair up");
        int ky = k > 0 ? k - 1 : 0;       // stage 0 has P = 0; past the end P = 0 as well
        ky = ky < nb_wg ? ky : nb_wg - 1;  // stay on a V tile that is resident
        const unsigned char* vt = v_lds + ((ky >> 1) % NBUF) * TILEB;
        const int vkbase = (ky & 1) * 32;
        const unsigned char* kt = k_lds + (((k + 1) >> 1) % NBUF) * TILEB;
        const int krow = ((k + 1) & 1) * 32 + l32;
        i32x4_t frag[NU];
        auto issue = [&](auto U) {
            constexpr int u = decltype(U)::value;
            if constexpr (u % 2 == 0) {
                constexpr int i = u / 2;
                frag[u] = load_vt_frag<D, true>(vt, vkbase + 16 * (i / DB), i % DB, lane);
            } else {
                constexpr int ks = u / 2;
                frag[u] = *(const i32x4_t*)(kt + k_off<D>(krow, ks * 2 + h));
            }
        };
        float mxa = 0.f, mxb = 0.f, ca = 0.f, cb = 0.f, ma_new = 0.f, mb_new = 0.f, psa = 0.f, psb = 0.f;
        bool any = false;
        const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // softmax slices: 4 for the maxima, the rest for the 32 exponentials (16 per half)
        constexpr int NEXPU = NU - 4;
        auto exp_one = [&](f32x16_t& s_, float m_new, float& psum, i32x4_t (&pp)[2], int e) {
            s_[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_[e], c, -m_new));
            psum += s_[e];
            if (e & 1) {
                int w = T::pack2(s_[e - 1], s_[e]);
                // anchor: keeps this slice of the softmax inside its unit (the optimiser would
                // otherwise sink it to the first use of P, after the last MFMA of the stage)
                asm volatile("" : "+v"(w), "+v"(psum));
                pp[e >> 3][(e >> 1) & 3] = w;
            }
        };
        auto valu = [&](auto U) {
            constexpr int u = decltype(U)::value;
            if constexpr (u == 0) {
                mxa = fmaxf(sa_cur[0], sa_cur[1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2)
                    mxa = fmaxf(mxa, fmaxf(sa_cur[r], sa_cur[r + 1]));
            } else if constexpr (u == 1) {
                mxb = fmaxf(sb_cur[0], sb_cur[1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2)
                    mxb = fmaxf(mxb, fmaxf(sb_cur[r], sb_cur[r + 1]));
            } else if constexpr (u == 2) {
                ca = half_max(mxa) * c;
                cb = half_max(mxb) * c;
            } else if constexpr (u == 3) {
                const bool grow = (ca > ma + RESCALE_TAU) || (cb > mb + RESCALE_TAU);
                any = __builtin_amdgcn_ballot_w64(grow) != 0;
                ma_new = any ? fmaxf(ma, ca) : ma;
                mb_new = any ? fmaxf(mb, cb) : mb;
            } else {
                constexpr int i = u - 4;
                constexpr int e0 = i * 32 / NEXPU, e1 = (i + 1) * 32 / NEXPU;
#pragma unroll
                for (int e = e0; e < e1; ++e) {
                    if (e < 16)
                        exp_one(sa_cur, ma_new, psa, pa_out, e);
                    else
                        exp_one(sb_cur, mb_new, psb, pb_out, e - 16);
                }
            }
        };
        issue(std::integral_constant<int, 0>{});
        issue(std::integral_constant<int, 1>{});
        static_for<0, NU>([&](auto U) {
            constexpr int u = decltype(U)::value;
            if constexpr (u + 2 < NU)
                issue(std::integral_constant<int, u + 2>{});
            if constexpr (u % 2 == 0) {
                constexpr int i = u / 2, t = i / DB, db = i % DB;
                oa[db] = T::mfma(frag[u], pa_in[t], oa[db]);
                ob[db] = T::mfma(frag[u], pb_in[t], ob[db]);
            } else {
                constexpr int ks = u / 2;
                sa_nxt = T::mfma(frag[u], qfa[ks], ks == 0 ? zero16 : sa_nxt);
                sb_nxt = T::mfma(frag[u], qfb[ks], ks == 0 ? zero16 : sb_nxt);
            }
            valu(U);
            __builtin_amdgcn_sched_barrier(0);
        });
        if (any) {
            // repair factors; applied after Y(k-1), whose P was formed against the old maxima
            const float aa = __builtin_amdgcn_exp2f(ma - ma_new), ab = __builtin_amdgcn_exp2f(mb - mb_new);
            la *= aa;
            lb *= ab;
            // One accumulator block at a time; each block is pinned back into the accumulation
            // registers right away so that O never lives in ordinary vector registers in the loop.
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    oa[db][r] *= aa;
                asm volatile("" : "+a"(oa[db]));
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    ob[db][r] *= ab;
                asm volatile("" : "+a"(ob[db]));
            }
            ma = ma_new;
            mb = mb_new;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
            asm volatile("" : "+a"(oa[db]), "+a"(ob[db]));
        la += psa;
        lb += psb;
    };
    auto needs_mask = [&](int k) { return (CAUSAL && 32 * k + 31 > Q0) || 32 * k + 32 > kv_end_w; };

    // ---- prologue: K tiles 0 and 1, V tile 0; S of block 0 ----
    load_tile(kg, k_lds, 0, k_grow, k_goff);
    load_tile(vg, v_lds, 0, v_grow, v_goff);
    if (ntiles > 1)
        load_tile(kg, k_lds, 1, k_grow, k_goff);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    f32x16_t s0a, s0b, s1a, s1b;
    i32x4_t pea[2], peb[2], poa[2], pob[2];  // P of the last even / odd block
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        pea[t] = i32x4_t{0, 0, 0, 0};
        peb[t] = i32x4_t{0, 0, 0, 0};
        poa[t] = i32x4_t{0, 0, 0, 0};
        pob[t] = i32x4_t{0, 0, 0, 0};
    }
    stage_x(0, s0a, s0b);

    for (int j = 0; j < niter; ++j) {
        if (j + 2 < ntiles)
            load_tile(kg, k_lds, j + 2, k_grow, k_goff);
        if (j + 1 < ntiles)
            load_tile(vg, v_lds, j + 1, v_grow, v_goff);

        const int ke = 2 * j, ko = 2 * j + 1;
        stage(ke, needs_mask(ke), s0a, s0b, s1a, s1b, poa, pob, pea, peb);
        stage(ko, needs_mask(ko), s1a, s1b, s0a, s0b, pea, peb, poa, pob);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- epilogue ----
    if (Q0 >= S)
        return;
    const float lta = half_sum(la), ltb = half_sum(lb);
    constexpr int OUTB = DT_OUT == NAUT_F32 ? 4 : 2;
    auto store_half = [&](int q, float m, float lt, const f32x16_t (&o)[DB]) {
        if (q >= S)
            return;
        const float inv_l = 1.0f / lt;
        if (p.lse != nullptr && h == 0)
            p.lse[(size_t)bh * S + q] = (m + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f;
        unsigned char* og = (unsigned char*)p.o + ((size_t)bh * S + q) * D * OUTB;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * db + 8 * g + 4 * h;
                const float x0 = o[db][4 * g + 0] * inv_l, x1 = o[db][4 * g + 1] * inv_l;
                const float x2 = o[db][4 * g + 2] * inv_l, x3 = o[db][4 * g + 3] * inv_l;
                if constexpr (DT_OUT == NAUT_F32) {
                    f32x4_t w = {x0, x1, x2, x3};
                    *(f32x4_t*)(og + d * 4) = w;
                } else {
                    i32x2_t w = {In<DT_OUT>::pack2(x0, x1), In<DT_OUT>::pack2(x2, x3)};
                    *(i32x2_t*)(og + d * 2) = w;
                }
            }
    };
    store_half(qa, ma, lta, oa);
    store_half(qb, mb, ltb, ob);
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

int kernel_choice()
{
    const char* e = getenv("NAUT_ATTN_KERNEL");
    return e == nullptr ? 2 : atoi(e);
}

template <int D, int DT_IN, int DT_OUT>
int launch(const Params& p, int causal, hipStream_t stream)
{
    const long long nblocks = (long long)p.nqt * p.B * p.Hq;
    if (nblocks > 0x7fffffffLL)
        return fail(NAUT_ERR_UNSUPPORTED, "B*Hq*ceil(S/128) exceeds the 1-D grid limit");
    const dim3 grid((unsigned)nblocks), block(NTHREADS);
    const bool vtr = use_vtr();
    if (kernel_choice() == 2) {
        const dim3 grid2((unsigned)((long long)p.nqt2 * p.B * p.Hq));
        if (causal)
            hipLaunchKernelGGL((naut_fwd_kernel_v2<D, DT_IN, DT_OUT, true>), grid2, block, 0, stream, p);
        else
            hipLaunchKernelGGL((naut_fwd_kernel_v2<D, DT_IN, DT_OUT, false>), grid2, block, 0, stream, p);
    } else if (causal) {
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
    p.nqt2 = (S + BM2 - 1) / BM2;
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
