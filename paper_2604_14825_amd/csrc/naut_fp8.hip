// naut_fp8.hip -- fused attention forward on FP8 (OCP E4M3) inputs for gfx950 (MI355X).
//
// The second precision of the paper's experiments (Section 6: every workload is run in FP16 and FP8).
// Q, K and V are E4M3 bytes with one scale per tensor (real value = descale * decoded); both matrix
// products run on the 32x32x64 FP8 MFMA with fp32 accumulation, the softmax in fp32, O is written as
// bf16.  Same formulation as the 16-bit kernels: scores are held transposed (S^T = K.Q^T, a lane owns
// one query), the online softmax keeps a lazily moved reference maximum, and P, converted to E4M3, is
// used straight from the score registers as the B operand of O^T += V^T.P^T.
//
// What is specific to 8-bit operands (layouts verified with a probe on the device):
//   - the MFMA takes 32 consecutive k-values per lane: lane l holds row l%32, k = 32*(l/32) .. +31;
//   - one instruction covers 64 keys of P.V, so the key axis is processed 64 keys (two 32-key score
//     blocks) at a time, and k-slot 16*blk + r of a lane half stands for the key of score register r of
//     block blk -- P needs no shuffle, its 32 bytes are the two blocks' registers in order;
//   - V^T fragments come from ds_read_b64_tr_b8: within 16 lanes, lane i supplies the address of 8
//     bytes X_i, lane j < 8 receives byte j of X_0, X_2, .., X_14 and lane 8+j byte j of X_1, X_3, ..,
//     X_15.  With X_2e = V[key_e][d0 .. d0+7] and X_2e+1 = V[key_e][d0+8 .. d0+15] a group of 16 lanes
//     gets, for 16 consecutive d, the same 8 keys each;
//   - P is scaled by 2^7 before the conversion (E4M3 has 3 fraction bits and loses everything below
//     2^-9): with the reference maximum at most one binade below the true one P*2^7 <= 256 < 448, and
//     the factor cancels in O / l.  The conversion does not saturate (it makes NaN), hence the bound.
//
// Work decomposition as the 128-query kernel of naut_attn_kernels.h: 4 wavefronts x 32 queries per
// work-group, 64-key tiles.  K and V tiles go straight from global memory to LDS (global_load_lds_dwordx4,
// the swizzle of the LDS layouts applied to the source address), F8_NBUF - 1 tiles ahead over a ring of
// F8_NBUF buffers per operand: every wavefront waits for its own loads of the tile about to be used (vmcnt),
// one barrier publishes them, and the buffer read in the previous step is refilled right after it.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <type_traits>

#include "naut_attn.h"
#include "naut_common.h"

namespace {

using namespace naut;

constexpr int F8_BM = 128;
constexpr int F8_BN = 64;
constexpr int F8_WAVES = 4;
constexpr int F8_THREADS = F8_WAVES * 64;
#ifndef NAUT_F8_NBUF
#define NAUT_F8_NBUF 3
#endif
constexpr int F8_NBUF = NAUT_F8_NBUF;  // LDS buffers per operand: tiles are requested F8_NBUF - 1 steps ahead
constexpr float F8_TAU = 1.0f;      // the reference maximum moves when a row exceeds it by more than 2^1
constexpr float F8_P_SHIFT = 7.0f;  // P is formed as exp2(.. + 7): <= 2^(1+7) = 256, inside E4M3's range
constexpr float F8_M_INIT = -1.0e30f;

struct Fp8Params {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    float* lse;
    int B, Hq, Hkv, S;
    int nqt;        // ceil(S / 128)
    float c;        // scale * descale_q * descale_k * log2(e), > 0
    float dv;       // descale_v
    // byte strides of batch, head and sequence position (the D axis is contiguous; q, k, v: 1 byte per
    // element, o: 2)
    long long q_bs, q_hs, k_bs, k_hs, v_bs, v_hs, o_bs, o_hs;
    int q_rs, k_rs, v_rs, o_rs;
    // The kernels are compiled for D = 64 or 128; a narrower head runs on the next wider one (strided
    // instantiation only): cpr16 16-byte chunks of every row are real, the chunks of Q beyond them read as
    // zero, those of K and V repeat a real chunk (they meet zeros of Q, or end in columns of O that are
    // not stored).
    int cpr16;
};

// STRIDED = false: contiguous [B][H][S][D] tensors, every stride a compile-time constant (the launch
// parameters' strides are not read); true: strides from the launch parameters.
template <int D, bool CAUSAL, bool STRIDED>
__global__ __launch_bounds__(F8_THREADS, 2) void naut_fwd_kernel_fp8(const Fp8Params p)
{
    constexpr int TILEB = F8_BN * D;            // bytes per K or V tile
    constexpr int CPR16 = D / 16;               // 16-byte chunks per row
    constexpr int NLDW = TILEB / 1024 / F8_WAVES;  // 1 KB direct loads per wavefront, tile and operand
    constexpr int LA = F8_NBUF - 1;               // tiles in flight ahead of the one in use
    constexpr int KS = D / 64;                  // MFMA k-steps of Q.K^T (64 d-values each)
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    static_assert(NLDW >= 1, "every wavefront takes part in the tile loads");
    static_assert(LA >= 1 && LA * 2 * NLDW < 64, "vmcnt field");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[F8_NBUF * 2 * TILEB];  // K0 V0 K1 V1 ...

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    const int nbh = p.B * p.Hq;
    const int bid = blockIdx.x;
    const int qt = p.nqt - 1 - bid / nbh;  // heaviest query tiles first
    const int bh = bid % nbh;
    const int b = bh / p.Hq;
    const int hq = bh % p.Hq;
    const int hk = hq / (p.Hq / p.Hkv);
    const int S = p.S;
    const float c = p.c;

    const int q_rs = STRIDED ? p.q_rs : D, k_rs = STRIDED ? p.k_rs : D, v_rs = STRIDED ? p.v_rs : D;
    const int o_rs = STRIDED ? p.o_rs : D * 2;
    const int cpr16 = STRIDED ? p.cpr16 : CPR16;  // real 16-byte chunks per row
    const unsigned char* qg = (const unsigned char*)p.q + (STRIDED ? b * p.q_bs + hq * p.q_hs : (long long)bh * S * D);
    const unsigned char* kg =
        (const unsigned char*)p.k + (STRIDED ? b * p.k_bs + hk * p.k_hs : (long long)(b * p.Hkv + hk) * S * D);
    const unsigned char* vg =
        (const unsigned char*)p.v + (STRIDED ? b * p.v_bs + hk * p.v_hs : (long long)(b * p.Hkv + hk) * S * D);

    const int q_wave0 = qt * F8_BM + wave * 32;
    const int my_q = q_wave0 + l32;
    const int my_q_ld = my_q < S ? my_q : S - 1;

    // Q^T fragments (MFMA B operand): lane holds q[my_q][64*ks + 32*h .. +32]
    i32x8_t qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int c0 = ks * 4 + h * 2;  // this lane's two 16-byte chunks of the row
        i32x4_t lo = *(const i32x4_t*)(qg + (size_t)my_q_ld * q_rs + (c0 < cpr16 ? c0 : 0) * 16);
        i32x4_t hi = *(const i32x4_t*)(qg + (size_t)my_q_ld * q_rs + (c0 + 1 < cpr16 ? c0 + 1 : 0) * 16);
        if (STRIDED && c0 >= cpr16)
            lo = i32x4_t{0, 0, 0, 0};
        if (STRIDED && c0 + 1 >= cpr16)
            hi = i32x4_t{0, 0, 0, 0};
        qf[ks] = i32x8_t{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        asm volatile("" : "+v"(qf[ks]));

    const int kv_end = CAUSAL ? (S < (qt + 1) * F8_BM ? S : (qt + 1) * F8_BM) : S;
    const int ntiles = (kv_end + F8_BN - 1) / F8_BN;

    // Direct global->LDS tile loads.  Load n of a tile fills its physical 16-byte chunks 64n .. 64n+63, lane i
    // the chunk 64n+i, so the lane fetches the logical chunk that k8_off / v8_off place there; wavefront w
    // issues loads w*NLDW .. of both operands.  The tile's base is wave-uniform (a scalar), the lane's byte
    // offset inside the tile is fixed; only the last tile of the sequence can be ragged: its offsets re-read
    // the last row, chosen by a uniform branch.
    int k_row[NLDW], k_col[NLDW], v_row[NLDW], v_col[NLDW];
#pragma unroll
    for (int i = 0; i < NLDW; ++i) {
        const int P = (wave * NLDW + i) * 64 + lane;
        const int r = P / CPR16, pc = P % CPR16;
        const int kc = pc ^ ((r >> 1) & (CPR16 - 1));  // the inverse of k8_off
        const int key = D == 128 ? (((r >> 1) & 1) | (((r >> 3) & 1) << 1)) : ((r >> 3) & 1);
        const int vc = (((pc >> 1) ^ key) << 1) + (pc & 1);  // the inverse of v8_off (32-byte chunks, two halves)
        k_row[i] = v_row[i] = r;
        k_col[i] = (kc < cpr16 ? kc : cpr16 - 1) * 16;
        v_col[i] = (vc < cpr16 ? vc : cpr16 - 1) * 16;
    }
    const unsigned smem_base = (unsigned)(uintptr_t)(NAUT_LDS unsigned char*)smem;
    const unsigned ld_dst = smem_base + (unsigned)(wave * NLDW * 1024);
    const int last_tile = (S + F8_BN - 1) / F8_BN - 1;
    const int rows_last = S - last_tile * F8_BN;  // rows of the sequence's last tile, >= 1
    auto issue_tile = [&](int tile, auto BUFC) {
        constexpr unsigned KB_OFF = decltype(BUFC)::value * 2 * TILEB;
        const unsigned char* kp = kg + (size_t)tile * F8_BN * k_rs;
        const unsigned char* vp = vg + (size_t)tile * F8_BN * v_rs;
        if (tile == last_tile) {
#pragma unroll
            for (int i = 0; i < NLDW; ++i) {
                const int rl = k_row[i] < rows_last ? k_row[i] : rows_last - 1;
                load_to_lds(ld_dst + KB_OFF + i * 1024, rl * k_rs + k_col[i], kp);
                load_to_lds(ld_dst + KB_OFF + TILEB + i * 1024, rl * v_rs + v_col[i], vp);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NLDW; ++i) {
                load_to_lds(ld_dst + KB_OFF + i * 1024, k_row[i] * k_rs + k_col[i], kp);
                load_to_lds(ld_dst + KB_OFF + TILEB + i * 1024, v_row[i] * v_rs + v_col[i], vp);
            }
        }
    };

    // lane-constant parts of the transposed V reads (see the file header): key index e and byte offset
    const int i16 = lane & 15;
    const int v_e = i16 >> 1;                                      // which of the 8 keys of a read this lane addresses
    const int v_key = 4 * h + (v_e & 3) + ((v_e >> 2) << 3);       // + base(t): keys {0,1,2,3,8,9,10,11} + 4h
    const int v_byte = 16 * ((lane >> 4) & 1) + 8 * (i16 & 1);     // inside the 32-byte chunk of block db
    // fixed LDS addresses of this lane's fragment reads in buffer 0 (K: per k-step and 16-byte half; V:
    // per 32-row block of O^T and group of 8 keys); buffer and key-block offsets are immediates
    int rd_k[KS][2], rd_v[DB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            rd_k[ks][u] = (int)smem_base + k8_off<D>(l32, ks * 4 + h * 2 + u);
            asm volatile("" : "+v"(rd_k[ks][u]));
        }
    // (adding 16 or 32 to a row changes neither swizzle key, so those steps are plain byte offsets)
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        rd_v[db] = (int)smem_base + v8_off<D>(v_key, db) + v_byte;
        asm volatile("" : "+v"(rd_v[db]));
    }

    f32x16_t oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            oacc[db][r] = 0.f;
    float m_run = F8_M_INIT;
    float l_run = 0.f;
    i32x8_t pb = {0, 0, 0, 0, 0, 0, 0, 0};  // P of the current tile as the B operand (lives across tiles, see pack4_fp8)

    // prologue: the first LA tiles
    static_for<0, LA>([&](auto T) {
        if (decltype(T)::value < ntiles)
            issue_tile(decltype(T)::value, T);
    });

    // one key tile; BUFC = j % F8_NBUF as a constant (the driver loop below is unrolled over the buffers)
    auto step = [&](auto BUFC, int j) {
        constexpr int BUF = decltype(BUFC)::value;
        constexpr int KT = BUF * 2 * TILEB, VT = KT + TILEB;  // byte offsets of this step's K and V tiles
        const int kv0 = j * F8_BN;
        // Tile j must have landed.  Loads complete in order, so with the tiles j+1 .. j+LA-1 requested after it
        // this wavefront may leave their loads in flight; near the end fewer were requested and it waits for all.
        if (j + LA - 1 < ntiles)
            wait_loads<(LA - 1) * 2 * NLDW>();
        else
            wait_loads<0>();
        tile_barrier();  // publishes tile j; every wavefront is done with the buffer of tile j-1, refilled next
        if (j + LA < ntiles)
            issue_tile(j + LA, std::integral_constant<int, (BUF + LA) % F8_NBUF>{});
        if constexpr (SAFE_SYNC) {  // checking build: nothing in flight while a step computes
            wait_loads<0>();
            tile_barrier();
        }

        const bool active = !CAUSAL || kv0 <= q_wave0 + 31;
        if (active) {
            f32x16_t sacc[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    sacc[kb][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const i32x4_t lo = *(const NAUT_LDS i32x4_t*)(uintptr_t)(rd_k[ks][0] + KT + kb * 32 * D);
                    const i32x4_t hi = *(const NAUT_LDS i32x4_t*)(uintptr_t)(rd_k[ks][1] + KT + kb * 32 * D);
                    const i32x8_t kf = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    sacc[kb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf, qf[ks], sacc[kb], 0, 0, 0, 0, 0, 0);
                }
            }
            const bool need_mask = (CAUSAL && kv0 + F8_BN - 1 > q_wave0) || (kv0 + F8_BN > S);
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kv0 + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        const bool dead = (CAUSAL && key > my_q) || key >= S;
                        sacc[kb][r] = dead ? -INFINITY : sacc[kb][r];
                    }
            }
            float mx = sacc[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    mx = fmaxf(mx, sacc[kb][r]);
            mx = half_max(mx);
            const float m_cand = mx * c;
            if (__builtin_amdgcn_ballot_w64(m_cand > m_run + F8_TAU) != 0) {
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
            const float shift = F8_P_SHIFT - m_run;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][r], c, shift));
                    sacc[kb][r] = pv;
                    psum = (kb | r) == 0 ? pv : psum + pv;
                }
            l_run += psum;
            // P as the B operand: k-slot 16*kb + r of this lane half is score register r of block kb
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                const int kb = w >> 2, r0 = (w & 3) * 4;
                pb[w] = pack4_fp8(sacc[kb][r0 + 0], sacc[kb][r0 + 1], sacc[kb][r0 + 2], sacc[kb][r0 + 3], pb[w]);
            }
            // O^T += V^T . P^T, all 64 keys of the tile in one MFMA per 32 rows of O^T
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                i32x8_t vf;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const i32x2_t x = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                        (NAUT_LDS i32x2_t*)(uintptr_t)(rd_v[db] + VT + (32 * (t >> 1) + 16 * (t & 1)) * D));
                    vf[2 * t] = x.x;
                    vf[2 * t + 1] = x.y;
                }
                oacc[db] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf, pb, oacc[db], 0, 0, 0, 0, 0, 0);
            }
        }
    };
    for (int j = 0; j < ntiles; j += F8_NBUF)
        static_for<0, F8_NBUF>([&](auto B_) {
            if (j + decltype(B_)::value < ntiles)
                step(B_, j + decltype(B_)::value);
        });
    __syncthreads();  // the tiles are dead from here on: the epilogue stages O in them

    // Epilogue: one division by l (the 2^7 of P cancels), times descale_v; lse undoes the shift.
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv_l = p.dv / l_tot;
    if (my_q < S && p.lse != nullptr && h == 0)
        p.lse[(size_t)bh * S + my_q] = (m_run - F8_P_SHIFT + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    // O leaves through LDS in whole rows: a lane owns 4 consecutive d of one query (8 bytes, 32 different
    // rows per store instruction); after the exchange D/8 lanes write one row with 16 bytes each.  The tiles
    // are dead after the loop's last barrier; each wavefront stages its 32 rows in its own quarter of them.
    {
        constexpr int ROWB_O = D * 2, CPRO = D / 8, R256 = ROWB_O >= 256 ? 1 : 256 / ROWB_O;
        static_assert(F8_WAVES * 32 * ROWB_O <= F8_NBUF * 2 * TILEB, "staging rows must fit the tile buffers");
        // Every address below derives from this copy of the lane id, which exists only from here on: nothing
        // of the epilogue can be computed before the key loop and held in registers across it.
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int l32e = ln & 31, he = ln >> 5;
        unsigned char* const stg = smem + wave * 32 * ROWB_O;
        auto staged = [&](int r, int ch) {  // swizzled so that neither the writes nor the reads conflict
            return stg + r * ROWB_O + ((ch ^ ((r / R256) & (CPRO - 1))) << 4);
        };
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * db + 8 * g + 4 * he;
                const i32x2_t w = {In<NAUT_BF16>::pack2(oacc[db][4 * g + 0] * inv_l, oacc[db][4 * g + 1] * inv_l),
                                   In<NAUT_BF16>::pack2(oacc[db][4 * g + 2] * inv_l, oacc[db][4 * g + 3] * inv_l)};
                *(i32x2_t*)(staged(l32e, d >> 3) + (d & 7) * 2) = w;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int RPI = 64 / CPRO;  // rows per store instruction
        typedef i32x4_t __attribute__((aligned(8))) i32x4_a8;  // O rows are 8-byte aligned, not more
        unsigned char* const o_bh =
            (unsigned char*)p.o + (STRIDED ? b * p.o_bs + hq * p.o_hs : (long long)bh * S * D * 2);
        i32x4_t rows[32 / RPI];
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i)
            rows[i] = *(const i32x4_t*)staged(i * RPI + ln / CPRO, ln % CPRO);
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int q = q_wave0 + i * RPI + ln / CPRO;
            if (q < S && (ln % CPRO) < 2 * cpr16)  // 16 bytes of bf16 O are 8 columns: two per real input chunk
                *(i32x4_a8*)(o_bh + (size_t)q * o_rs + (ln % CPRO) * 16) = rows[i];
        }
    }
}

}  // namespace

extern "C" {

int naut_attn_fwd_fp8_strided(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                              int S, int D, int causal, float scale, float descale_q, float descale_k,
                              float descale_v, void* stream, const naut_strides* st)
{
    if (!q || !k || !v || !o)
        return fail(NAUT_ERR_NULL, "q, k, v and o must be non-NULL device pointers");
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || S <= 0 || D <= 0)
        return fail(NAUT_ERR_SHAPE, "B, Hq, Hkv, S and D must be positive");
    if (Hq % Hkv != 0)
        return fail(NAUT_ERR_SHAPE, "Hq must be a multiple of Hkv");
    if (!std::isfinite(scale) || !std::isfinite(descale_q) || !std::isfinite(descale_k) || !std::isfinite(descale_v))
        return fail(NAUT_ERR_SHAPE, "scale and the three descale factors must be finite");
    if (scale < 0.f || descale_q <= 0.f || descale_k <= 0.f || descale_v <= 0.f)
        return fail(NAUT_ERR_UNSUPPORTED, "scale must be >= 0 and the descale factors > 0");
    if (D % 16 != 0 || D > 128)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be a multiple of 16, at most 128");
    const int DK = D <= 64 ? 64 : 128;  // width the kernels are compiled for
    const long long nblocks = (long long)B * Hq * ((S + F8_BM - 1) / F8_BM);
    if ((long long)B * Hq > 0x7fffffffLL || nblocks > 0x7fffffffLL)
        return fail(NAUT_ERR_UNSUPPORTED, "B*Hq*ceil(S/128) exceeds the 1-D grid limit");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15u)
        return fail(NAUT_ERR_ALIGN, "q, k, v and o must be 16-byte aligned");
    if ((uintptr_t)lse & 3u)
        return fail(NAUT_ERR_ALIGN, "lse must be 4-byte aligned");

    naut_strides cs;  // contiguous [B][H][S][D]
    cs.q_s = cs.k_s = cs.v_s = cs.o_s = D;
    cs.q_h = cs.o_h = cs.k_h = cs.v_h = (long long)S * D;
    cs.q_b = cs.o_b = (long long)Hq * S * D;
    cs.k_b = cs.v_b = (long long)Hkv * S * D;
    if (!st)
        st = &cs;
    const long long in_strides[9] = {st->q_b, st->q_h, st->q_s, st->k_b, st->k_h, st->k_s, st->v_b, st->v_h, st->v_s};
    for (long long x : in_strides)
        if (x < 0 || x % 16 != 0)
            return fail(NAUT_ERR_ALIGN, "q/k/v strides must be non-negative multiples of 16 elements (16 bytes)");
    if (st->o_b <= 0 || st->o_h <= 0 || st->o_s <= 0 || st->o_b % 4 != 0 || st->o_h % 4 != 0 || st->o_s % 4 != 0)
        return fail(NAUT_ERR_ALIGN, "o strides must be positive multiples of 4 elements");
    if (st->q_s < D || st->k_s < D || st->v_s < D || st->o_s < D)
        return fail(NAUT_ERR_SHAPE, "a sequence stride is smaller than D: rows would overlap");
    const long long max_rs = 1LL << 23;  // elements: keeps 64 rows of byte offsets inside 32 bits
    if (st->q_s > max_rs || st->k_s > max_rs || st->v_s > max_rs || st->o_s > max_rs)
        return fail(NAUT_ERR_UNSUPPORTED, "sequence stride too large");

    Fp8Params p;
    p.q_bs = st->q_b;
    p.q_hs = st->q_h;
    p.q_rs = (int)st->q_s;
    p.k_bs = st->k_b;
    p.k_hs = st->k_h;
    p.k_rs = (int)st->k_s;
    p.v_bs = st->v_b;
    p.v_hs = st->v_h;
    p.v_rs = (int)st->v_s;
    p.o_bs = st->o_b * 2;
    p.o_hs = st->o_h * 2;
    p.o_rs = (int)(st->o_s * 2);
    p.q = q;
    p.k = k;
    p.v = v;
    p.o = o;
    p.lse = lse;
    p.B = B;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.S = S;
    p.nqt = (S + F8_BM - 1) / F8_BM;
    const float c = scale * descale_q * descale_k * 1.4426950408889634f;
    p.c = c > 0.f ? c : 1e-30f;
    p.dv = descale_v;
    p.cpr16 = D / 16;
    const dim3 grid((unsigned)nblocks);
    hipStream_t hs = (hipStream_t)stream;
    // contiguous tensors (whoever says so) take the instantiation with compile-time strides
    const bool strided = D != DK || st->q_b != cs.q_b || st->q_h != cs.q_h || st->q_s != cs.q_s || st->k_b != cs.k_b ||
                         st->k_h != cs.k_h || st->k_s != cs.k_s || st->v_b != cs.v_b || st->v_h != cs.v_h ||
                         st->v_s != cs.v_s || st->o_b != cs.o_b || st->o_h != cs.o_h || st->o_s != cs.o_s;
#define NAUT_F8_LAUNCH(DD, CC, SS)                                                          \
    if (DK == DD && (causal != 0) == CC && strided == SS)                                   \
        hipLaunchKernelGGL((naut_fwd_kernel_fp8<DD, CC, SS>), grid, dim3(F8_THREADS), 0, hs, p);
    NAUT_F8_LAUNCH(128, true, false)
    NAUT_F8_LAUNCH(128, false, false)
    NAUT_F8_LAUNCH(64, true, false)
    NAUT_F8_LAUNCH(64, false, false)
    NAUT_F8_LAUNCH(128, true, true)
    NAUT_F8_LAUNCH(128, false, true)
    NAUT_F8_LAUNCH(64, true, true)
    NAUT_F8_LAUNCH(64, false, true)
#undef NAUT_F8_LAUNCH
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_launch(e);
    return NAUT_OK;
}

int naut_attn_fwd_fp8(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int S,
                      int D, int causal, float scale, float descale_q, float descale_k, float descale_v, void* stream)
{
    return naut_attn_fwd_fp8_strided(q, k, v, o, lse, B, Hq, Hkv, S, D, causal, scale, descale_q, descale_k, descale_v,
                                     stream, nullptr);
}

}  // extern "C"
