// naut_attn_kernels.h -- the fused attention forward kernels for gfx950 (MI355X) and their launcher.
//
// Included by naut_attn.hip (the C ABI, which only declares the launcher instantiations) and by
// naut_attn_inst.hip (compiled once per storage-type pair, which defines them): splitting the
// instantiations over translation units lets them compile in parallel.
//
// One kernel computes O = softmax(scale * Q K^T + causal mask) V for a
// (batch, head, query tile) per work-group; three variants share the formulation
// below and are picked per shape (pick_variant): kernel 1 (128 queries per
// work-group; also the D = 256 instantiation) and kernel 2 (256 queries,
// software-pipelined over 32-key blocks, in two shapes).  The reductions over the key
// axis (row max, row sum, weighted sum of V) are fused with the rolling-update
// scheme of Section 4.2/4.3 of the paper: a running maximum m and running sum l
// are kept per query, and whenever m grows the partial results are repaired by
// the factor exp2(m_old - m_new).  The S x S scores never leave registers.
// Hand-applied rewrites (table of Section 5): scale*log2(e) folded into one
// constant, exp -> exp2, and a single division by l in the epilogue instead of
// one per step.
//
// Work decomposition (bi-level tiling, Section 4.2): outer loops (batch, head,
// query tile) -> work-groups; inner tile = 128 or 256 queries x 64 keys.  A
// wavefront owns 32 (or 64) queries.  Per key tile and wavefront:
//
//   S^T[key][query] = K_tile . Q^T     v_mfma_f32_32x32x16 (A = K from LDS, B = Q in registers)
//   online softmax over keys           each lane owns ONE query (column) and 16 keys per 32-key block,
//                                      so row max / row sum are in-lane plus one exchange between the
//                                      two 32-lane halves
//   O^T[d][query] += V^T . P^T         A = V^T (LDS transpose read), B = P^T taken straight from the
//                                      S^T accumulator registers (no shuffle: the MFMA k-slot <-> key
//                                      assignment is chosen to match the accumulator layout)
//
// K and V tiles are multi-buffered in LDS, one barrier per tile, and go straight from
// global memory into LDS (global_load_lds_dwordx4, the swizzle applied to the source
// address): one tile ahead over two buffers in kernel 1, three tiles ahead over four
// buffers in kernel 2 and in the D = 256 instantiation.
#ifndef NAUT_ATTN_KERNELS_H
#define NAUT_ATTN_KERNELS_H
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "naut_attn.h"
#include "naut_common.h"

#ifndef NAUT_KPF
#define NAUT_KPF 2
#endif
#ifndef NAUT_K1_NBUF
#define NAUT_K1_NBUF 2
#endif

namespace naut_k {

using namespace naut;


constexpr int BM = 128;  // queries per work-group
constexpr int BN = 64;   // keys per step
constexpr int NWAVES = 4;
constexpr int NTHREADS = NWAVES * 64;
constexpr float RESCALE_TAU = 6.0f;  // log2 units
constexpr float P_LIMIT = 1024.0f;   // a block's per-lane row sum above this moves the reference maximum

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
    // Byte strides of batch, head and sequence position (the D axis is contiguous).  The kernels are
    // compiled for D = 64 or 128; a smaller head dimension runs on the next wider one: cpr 16-byte
    // chunks of every row are real, the chunks of Q beyond them read as zero, those of K and V repeat
    // a real chunk (they meet zeros of Q, or end in columns of O that are not stored).
    long long q_bs, q_hs, k_bs, k_hs, v_bs, v_hs, o_bs, o_hs;
    int q_rs, k_rs, v_rs, o_rs;
    int cpr;       // real 16-byte chunks per row = head dimension / 8
    int hao;       // kernel 1: (batch, head) pairs an XCD works on at a time (0: all of its share at once)
};

// S^T MFMAs of the variants that need more than 256 registers per lane (64 queries per wavefront in
// kernel 2, D = 256 in kernel 1), written as asm so that their accumulator is an ordinary vector
// register tuple while O and Q live in the accumulation registers (the compiler's own MFMA form
// would then put the scores there too and copy each one out for the softmax).  The compiler's hazard handling does not look inside asm, so the wait states the
// hardware does not interlock are owed by hand:
//   - a vector instruction that writes an MFMA source (the register allocator may route a
//     fragment through a copy) must be 2 wait states ahead of the MFMA: each asm starts with them;
//   - an MFMA result may be read by a vector instruction only 11 wait states after the issue of
//     this 8-pass MFMA: see `settle` and the guard at the start of kernel 2's `stage`.
// Everything that fits the ordinary vector registers uses the compiler's MFMA throughout.
template <int DT>
struct XMfma;
// Puts every later reader of an asm MFMA's result `d` the owed wait states behind that MFMA.
__device__ __forceinline__ void settle(f32x16_t& d) { asm volatile(NAUT_NOP_SETTLE : "+v"(d)); }
template <>
struct XMfma<NAUT_BF16> {
    static __device__ __forceinline__ void first(f32x16_t& d, i32x4_t a, i32x4_t b)
    {
        asm volatile(NAUT_NOP_SHORT "v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" NAUT_NOP_AFTER_MFMA : "=&v"(d) : "v"(a), "a"(b));
    }
    static __device__ __forceinline__ void acc(f32x16_t& d, i32x4_t a, i32x4_t b)
    {
        asm volatile(NAUT_NOP_SHORT "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" NAUT_NOP_AFTER_MFMA : "+v"(d) : "v"(a), "a"(b));
    }
};
template <>
struct XMfma<NAUT_F16> {
    static __device__ __forceinline__ void first(f32x16_t& d, i32x4_t a, i32x4_t b)
    {
        asm volatile(NAUT_NOP_SHORT "v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" NAUT_NOP_AFTER_MFMA : "=&v"(d) : "v"(a), "a"(b));
    }
    static __device__ __forceinline__ void acc(f32x16_t& d, i32x4_t a, i32x4_t b)
    {
        asm volatile(NAUT_NOP_SHORT "v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" NAUT_NOP_AFTER_MFMA : "+v"(d) : "v"(a), "a"(b));
    }
};

// ---- kernel 1: 128 queries per work-group, 4 wavefronts x 32 queries ----
// Two work-groups per CU (four at D = 64) and 64 keys per step for D <= 128.  D = 256 doubles the O accumulator and the
// Q fragments of a lane (192 registers between them), so it runs one work-group per CU on the full
// 512-register budget, 32 keys per step (the four tile buffers then still fill 64 KB).

template <int D, int DT_IN, int DT_OUT, bool CAUSAL>
__global__ __launch_bounds__(NTHREADS, D > 128 ? 1 : 2) void naut_fwd_kernel_bm128(const Params p)
{
    using T = In<DT_IN>;
    constexpr int BN = D > 128 ? 32 : 64;    // keys per step (hides the file-scope value used by kernel 2)
    constexpr int ROWB = D * 2;              // bytes per K/V row
    constexpr int TILEB = BN * ROWB;         // bytes per K or V tile
    constexpr int CPR = D / 8;               // 16-byte chunks per row
    constexpr int KS = D / 16;               // MFMA k-steps of Q.K^T
    constexpr int DB = D / 32;               // 32-row blocks of O^T
    constexpr int KB = BN / 32;              // 32-key blocks of S^T

    // Tiles are filled by direct global->LDS loads, each wavefront its share of every tile.  D = 256: four K
    // buffers, then four V buffers, filled three steps ahead (one wavefront per SIMD has nothing else to
    // hide the load latency behind).  D <= 128: K0 V0 K1 V1 ..., a ring of NB2 buffers filled NB2 - 1 steps
    // ahead (the key loop is unrolled over the ring, so a tile's LDS offsets are instruction immediates).
    constexpr bool WIDE = D > 128;
    constexpr int NB = 4;                          // buffers per operand (wide)
    constexpr int NB2 = NAUT_K1_NBUF;              // buffers per operand (D <= 128)
    constexpr int LDW = TILEB / 1024 / NWAVES;     // direct loads (1 KB each) per wavefront per tile
    static_assert(LDW >= 1 && (NB2 - 1) * 2 * LDW < 64, "every wavefront loads; vmcnt field");
    __shared__ __attribute__((aligned(1024))) unsigned char smem[(WIDE ? 2 * NB : 2 * NB2) * TILEB];
    __shared__ float dl_lds[NTHREADS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: it feeds scalar operands of the tile loads
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // Tile scheduler: heaviest (last) query tiles first; consecutive block ids walk the
    // (batch, head) axis so that each XCD (block id mod 8) keeps to a fixed subset of heads.
    const int nbh = p.B * p.Hq;
    const int bid = blockIdx.x;
    int qt, bh;
    if (p.hao > 0 && (nbh & 7) == 0) {
        // Long key ranges: an XCD takes a contiguous run of heads and works on p.hao of them at a
        // time, so that the K/V tiles its work-groups stream stay in its L2.
        const int xcd = bid & 7, s = bid >> 3;
        const int hpx = nbh >> 3;
        const int G = hpx < p.hao ? hpx : p.hao;
        const int per_group = p.nqt * G;
        const int g = s / per_group, sg = s % per_group;
        const int ng = hpx - g * G < G ? hpx - g * G : G;
        bh = xcd * hpx + g * G + sg % ng;
        qt = p.nqt - 1 - sg / ng;
    } else {
        qt = p.nqt - 1 - bid / nbh;
        bh = bid % nbh;
    }
    const int b = bh / p.Hq;
    const int hq = bh % p.Hq;
    const int hk = hq / (p.Hq / p.Hkv);
    const int S = p.S;

    const unsigned char* qg = (const unsigned char*)p.q + b * p.q_bs + hq * p.q_hs;
    const unsigned char* kg = (const unsigned char*)p.k + b * p.k_bs + hk * p.k_hs;
    const unsigned char* vg = (const unsigned char*)p.v + b * p.v_bs + hk * p.v_hs;
    const int cpr = p.cpr;

    const int q_wave0 = qt * BM + wave * 32;  // first query of this wavefront
    const int my_q = q_wave0 + l32;           // the query this lane owns
    const int my_q_ld = my_q < S ? my_q : S - 1;

    // Q^T fragments (MFMA B operand): lane holds q[my_q][16*ks + 8*h .. +8].
    i32x4_t qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        // Unconditional, from a chunk that exists (a load under a condition becomes a branch); the padding
        // chunks of a narrower head are zeroed when Q is pinned.
        const int ch = ks * 2 + h < cpr ? ks * 2 + h : cpr - 1;
        qf[ks] = *(const i32x4_t*)(qg + (size_t)my_q_ld * p.q_rs + ch * 16);
    }
    // Keep Q resident: without this the compiler re-issues the global loads inside the key loop.
    // The wide instantiation keeps it, and O, in the accumulation registers.  D <= 128 pins it only
    // after the first tile's loads are out, so that the two share one round trip to memory.
    auto pin_acc = [](f32x16_t& x) {
        if constexpr (WIDE)
            asm volatile("" : "+a"(x));
    };
    auto pin_q = [&](int cpr_now) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks * 2 + h >= cpr_now)
                qf[ks] = i32x4_t{0, 0, 0, 0};
            if constexpr (WIDE)
                asm volatile("" : "+a"(qf[ks]));
            else
                asm volatile("" : "+v"(qf[ks]));
        }
    };
    if constexpr (WIDE)
        pin_q(cpr);

    const int kv_end = CAUSAL ? (S < (qt + 1) * BM ? S : (qt + 1) * BM) : S;
    const int ntiles = (kv_end + BN - 1) / BN;

    // Lane i of direct load n fills physical chunk P = (wave*LDW + n)*64 + i of the tile, so it fetches the
    // logical (row, chunk) that k_off / v_off place there (chunks beyond a narrower head repeat a real one).
    auto source_of = [&](int n, int& krow, int& kcol, int& vrow, int& vcol) {
        const int P = (wave * LDW + n) * 64 + lane;
        int kc, vc;
        if constexpr (WIDE) {
            const int line = P >> 4;
            krow = line >> 1;
            kc = ((line & 1) << 4) | ((P & 15) ^ (krow & 15));
            vrow = P >> 5;
            vc = (P & 31) ^ ((vrow & 3) << 2);
        } else {
            const int line = P >> 4, pos = P & 15;
            const int off = ((line << 4) + (pos ^ (line & 15))) * 16;  // the inverse of k_off: byte offset in a dense tile
            krow = off / ROWB;
            kc = off % ROWB / 16;
            vrow = P / CPR;                                              // the inverse of v_off
            vc = D == 128 ? (P % CPR) ^ ((vrow & 3) << 2) : (P % CPR) ^ (((vrow >> 1) & 1) << 2);
        }
        kcol = (kc < cpr ? kc : cpr - 1) * 16;
        vcol = (vc < cpr ? vc : cpr - 1) * 16;
    };
    // wide: (row, byte in the row) per load; D <= 128: the byte offset inside a whole tile
    int wk_row[LDW], wk_col[LDW], wv_row[LDW], wv_col[LDW];
    const unsigned smem_base = (unsigned)(uintptr_t)(NAUT_LDS unsigned char*)smem;
#pragma unroll
    for (int n = 0; n < LDW; ++n) {
        source_of(n, wk_row[n], wk_col[n], wv_row[n], wv_col[n]);
        if constexpr (!WIDE) {
            wk_col[n] += wk_row[n] * p.k_rs;
            wv_col[n] += wv_row[n] * p.v_rs;
        }
    }
    const int last_tile = (S + BN - 1) / BN - 1;  // of the sequence: the only one that can be ragged
    // The address of a load is the tile's base, a 64-bit wave-uniform pointer, plus a 32-bit lane offset inside
    // the tile (at most BN rows of the largest row stride the entry point admits); rows beyond the end of the
    // sequence re-read its last row.
    // (D <= 128: `buf`, the tile's place in the ring, is a constant at every call)
    auto issue_tile = [&](int tile, int buf = 0) {
        const unsigned kd = smem_base + (unsigned)((WIDE ? (tile % NB) * TILEB : buf * 2 * TILEB) + wave * LDW * 1024);
        const unsigned vd = kd + (WIDE ? NB * TILEB : TILEB);
        const unsigned char* const kt = kg + (size_t)tile * BN * p.k_rs;
        const unsigned char* const vt = vg + (size_t)tile * BN * p.v_rs;
        const int last_row = S - 1 - tile * BN;  // of this tile, counted from its first row; >= 0
        if constexpr (WIDE) {
#pragma unroll
            for (int n = 0; n < LDW; ++n) {
                const int row = wk_row[n] < last_row ? wk_row[n] : last_row;
                const int off = row * p.k_rs + wk_col[n];
                load_to_lds(kd + n * 1024, off, kt);
            }
#pragma unroll
            for (int n = 0; n < LDW; ++n) {
                const int row = wv_row[n] < last_row ? wv_row[n] : last_row;
                const int off = row * p.v_rs + wv_col[n];
                load_to_lds(vd + n * 1024, off, vt);
            }
        } else if (tile == last_tile) {  // once per work-group: the offsets of the ragged tile are formed on the spot
#pragma unroll
            for (int n = 0; n < LDW; ++n) {
                int kr, kcol, vr, vcol;
                source_of(n, kr, kcol, vr, vcol);
                load_to_lds(kd + n * 1024, (kr < last_row ? kr : last_row) * p.k_rs + kcol, kt);
                load_to_lds(vd + n * 1024, (vr < last_row ? vr : last_row) * p.v_rs + vcol, vt);
            }
        } else {
#pragma unroll
            for (int n = 0; n < LDW; ++n) {
                load_to_lds(kd + n * 1024, wk_col[n], kt);
                load_to_lds(vd + n * 1024, wv_col[n], vt);
            }
        }
    };
    // Waits until at most `ahead` later tiles of this wavefront's loads are still in flight.
    auto wait_tiles = [&](int ahead) {
        if (ahead >= 2)
            wait_loads<WIDE ? 2 * 2 * LDW : 0>();
        else if (ahead == 1)
            wait_loads<WIDE ? 2 * LDW : 0>();
        else
            wait_loads<0>();
    };

    // fixed LDS addresses of this lane's fragment reads in buffer 0 (K: per k-step; V: per 32-row block
    // of O^T, first of the two transposed reads); buffer, key-block and key-step offsets are immediates
    // (adding 8, 16 or 32 to a row changes no swizzle key)
    int rd_k[KS], rd_v[DB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        rd_k[ks] = (int)smem_base + k_off<D>(l32, ks * 2 + h);
        asm volatile("" : "+v"(rd_k[ks]));
    }
    {
        const int i16 = lane & 15;
        const int key = 4 * h + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int d = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
            rd_v[db] = (int)smem_base + v_off<D>(key, d >> 3) + (d & 7) * 2;
            asm volatile("" : "+v"(rd_v[db]));
        }
    }

    f32x16_t oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            oacc[db][r] = 0.f;
    float m_run = -INFINITY;  // running max, in the exp2 domain (already times c)
    float l_run = 0.f;        // this lane's share of the running sum (its 16 of every 32 keys)
    // What the sum of P as rounded for the second product, the divisor of O, has over l (this lane's share; see
    // "the two sums" in kernel 2).  It is touched only in rare blocks and in the epilogue, so it lives in a word
    // of LDS per lane instead of a register: the D = 64 instantiation fits four wavefronts per SIMD on exactly
    // 128 registers.
    // (its index is re-derived from the hardware lane count where it is used: no register holds it either)
    auto dl_slot = [&]() -> float& {
        const int ln = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        return dl_lds[wave * 64 + ln];
    };
    dl_slot() = 0.f;
    const float c = p.c;

    if constexpr (WIDE) {
        // Q must be in its registers before the tile loads start: the compiler's own wait for Q would
        // otherwise also wait for every tile load issued before it.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        for (int t = 0; t < NB - 1 && t < ntiles; ++t)
            issue_tile(t);
        wait_tiles(ntiles - 1);
        tile_barrier();
    } else {
        static_for<0, NB2 - 1>([&](auto TC) {
            if (decltype(TC)::value < ntiles)
                issue_tile(decltype(TC)::value, decltype(TC)::value);
        });
        int cpr_late = cpr;
        asm volatile("" : "+s"(cpr_late));  // ordered after the asm of the tile loads: so is everything that uses it
        pin_q(cpr_late);                    // Q and the first tiles share one round trip to memory
    }

    // One key tile.  D <= 128: UC = j & 1 as a constant -- the driver loop below is unrolled over the two
    // LDS buffers, so the tile's LDS offsets are immediates.  D = 256 keeps one copy of its (long) body
    // and adds the buffer offset at run time.
    constexpr int NU = WIDE ? 1 : NB2;
    auto step = [&](auto UC, int j) {
        constexpr int U = decltype(UC)::value;
        const int KT = WIDE ? (j % NB) * TILEB : U * 2 * TILEB;   // byte offset of this step's K tile
        const int VT = WIDE ? KT + NB * TILEB : KT + TILEB;
        const int kv0 = j * BN;
        if constexpr (WIDE) {
            // buffer (j + NB - 1) % NB was last read in step j - 1, which every wavefront has left
            if (j + NB - 1 < ntiles)
                issue_tile(j + NB - 1);
            if constexpr (SAFE_SYNC)
                tile_barrier();  // checking build: nothing in flight while the step computes
        } else {
            // Tile j must have landed.  Loads complete in order, so with the tiles j+1 .. j+NB2-2 requested after
            // it this wavefront may leave theirs in flight; near the end fewer were requested and it waits for all.
            if (j + NB2 - 2 < ntiles)
                wait_loads<(NB2 - 2) * 2 * LDW>();
            else
                wait_loads<0>();
            tile_barrier();  // publishes tile j; every wavefront has left step j-1, whose buffer is refilled next
            if (j + NB2 - 1 < ntiles)
                issue_tile(j + NB2 - 1, (U + NB2 - 1) % NB2);
            if constexpr (SAFE_SYNC) {  // checking build: nothing in flight while the step computes
                wait_loads<0>();
                tile_barrier();
            }
        }

        // Causal block skipping per wavefront: nothing to do if every key of the tile lies
        // beyond this wavefront's last query.
        const bool active = !CAUSAL || kv0 <= q_wave0 + 31;
        if (active) {
            f32x16_t sacc[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                if constexpr (WIDE) {
                    // The compiler moves nothing across the asm MFMAs, so the fragment reads are put
                    // KPF MFMAs ahead of their use by hand.  Measured at S = 16384: reading each fragment
                    // right before its MFMA exposes the LDS latency 16 times per step (714 TFLOP/s), one
                    // ahead 829, two 850, three 846, four 843, six 839, eight 835, twelve 825, sixteen 812:
                    // two reads in flight cover the latency, more only lengthen the wait before the first
                    // MFMA of the step.
                    constexpr int KPF = NAUT_KPF;
                    i32x4_t kf[KS];
#pragma unroll
                    for (int ks = 0; ks < KPF; ++ks)
                        kf[ks] = *(const NAUT_LDS i32x4_t*)(uintptr_t)(rd_k[ks] + KT + kb * 32 * ROWB);
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        if (ks + KPF < KS)
                            kf[ks + KPF] = *(const NAUT_LDS i32x4_t*)(uintptr_t)(rd_k[ks + KPF] + KT + kb * 32 * ROWB);
                        if (ks == 0)
                            XMfma<DT_IN>::first(sacc[kb], kf[ks], qf[ks]);
                        else
                            XMfma<DT_IN>::acc(sacc[kb], kf[ks], qf[ks]);
                    }
                    settle(sacc[kb]);
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        sacc[kb][r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const i32x4_t kf = *(const NAUT_LDS i32x4_t*)(uintptr_t)(rd_k[ks] + KT + kb * 32 * ROWB);
                        sacc[kb] = T::mfma(kf, qf[ks], sacc[kb]);
                    }
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
                dl_slot() *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    pin_acc(oacc[db]);  // the copy into vector registers for the multiply starts here, not at the loop top
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        oacc[db][r] *= alpha;
                    pin_acc(oacc[db]);
                }
            }
#pragma unroll
            for (int db = 0; db < DB; ++db)
                pin_acc(oacc[db]);
            const float m_new = m_run;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][r], c, -m_new));
                    sacc[kb][r] = pv;
                    psum = (kb | r) == 0 ? pv : psum + pv;
                }
            // O^T += V^T . P^T, 16 keys per MFMA
#pragma unroll
            for (int t = 0; t < BN / 16; ++t) {
                const int kb = t >> 1, r0 = (t & 1) * 8;
                i32x4_t pb = {T::pack2(sacc[kb][r0 + 0], sacc[kb][r0 + 1]), T::pack2(sacc[kb][r0 + 2], sacc[kb][r0 + 3]),
                              T::pack2(sacc[kb][r0 + 4], sacc[kb][r0 + 5]), T::pack2(sacc[kb][r0 + 6], sacc[kb][r0 + 7])};
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int a = rd_v[db] + VT + t * 16 * ROWB;
                    const i16x4_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((NAUT_LDS i16x4_t*)(uintptr_t)a);
                    const i16x4_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((NAUT_LDS i16x4_t*)(uintptr_t)(a + 8 * ROWB));
                    const i32x2_t lo = __builtin_bit_cast(i32x2_t, r0), hi = __builtin_bit_cast(i32x2_t, r1);
                    const i32x4_t vf = {lo.x, lo.y, hi.x, hi.y};
                    oacc[db] = T::mfma(vf, pb, oacc[db]);
                }
            }
            // The divisor of O takes the sum of P as rounded for the second product only for a tile that at least
            // doubles some row's running sum (see "the two sums" in kernel 2); elsewhere the unrounded sum stands
            // in for it.  The test sits at the end of the tile, where it splits no schedule; a tile that passes
            // it rounds its P, still in their registers, once more (the pairs in the other order -- the sum does
            // not care -- so that these packs are not merged with those of the product loop above).
            if (__builtin_amdgcn_ballot_w64(psum > l_run) != 0) {
                float prsum = -psum;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; r += 2)
                        prsum = T::add_pair(T::pack2(sacc[kb][r + 1], sacc[kb][r]), prsum);
                dl_slot() += prsum;
            }
            l_run += psum;
        }
        if constexpr (WIDE) {
            // Tile j + 1 must have landed; the tiles after it may fly on.  A bare barrier: every LDS
            // read of this step has been consumed by its MFMA, and the fence of __syncthreads()
            // would wait for all tile loads in flight.
            wait_tiles(ntiles - 2 - j);
            tile_barrier();
        }
    };
    for (int j0 = 0; j0 < ntiles; j0 += NU) {
        static_for<0, NU>([&](auto UC) {
            const int j = j0 + decltype(UC)::value;
            if (j < ntiles)  // uniform over the work-group
                step(UC, j);
        });
    }

    if constexpr (!WIDE)
        __syncthreads();  // every wavefront has left the last step: the tiles are dead, the epilogue stages O in them
    // Epilogue: one division by l (the per-step divide/multiply pairs telescope away), lse, store.
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float dl_run = dl_slot();
    const float inv_l = 1.0f / (l_tot + (dl_run + __shfl_xor(dl_run, 32)));
    if (my_q < S && p.lse != nullptr && h == 0)
        p.lse[(size_t)bh * S + my_q] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    unsigned char* const o_bh = (unsigned char*)p.o + b * p.o_bs + hq * p.o_hs;
    if constexpr (DT_OUT != NAUT_F32) {
        // 16-bit O leaves through LDS in whole rows: a lane owns 4 consecutive d of one query (8 bytes, 32
        // different rows per store instruction); after the exchange D/8 lanes write one row with 16 bytes
        // each.  The tiles are dead after the loop's last barrier (every tile load has landed, every
        // fragment has been consumed); each wavefront stages its 32 rows in its own part of them.
        constexpr int CPRO = D / 8, R256 = ROWB >= 256 ? 1 : 256 / ROWB;
        static_assert(NWAVES * 32 * ROWB <= (int)sizeof(smem), "staging rows must fit the tile buffers");
        // Every address below derives from this copy of the lane id, which exists only from here on: nothing
        // of the epilogue can be computed before the key loop and held in registers across it.
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int l32e = ln & 31, he = ln >> 5;
        unsigned char* const stg = smem + wave * 32 * ROWB;
        auto staged = [&](int r, int ch) {  // swizzled so that neither the writes nor the reads conflict
            return stg + r * ROWB + ((ch ^ ((r / R256) & (CPRO - 1))) << 4);
        };
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * db + 8 * g + 4 * he;
                const i32x2_t w = {In<DT_OUT>::pack2(oacc[db][4 * g + 0] * inv_l, oacc[db][4 * g + 1] * inv_l),
                                   In<DT_OUT>::pack2(oacc[db][4 * g + 2] * inv_l, oacc[db][4 * g + 3] * inv_l)};
                *(i32x2_t*)(staged(l32e, d >> 3) + (d & 7) * 2) = w;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int RPI = 64 / CPRO;    // rows per store instruction
        constexpr int BATCH = 8 < 32 / RPI ? 8 : 32 / RPI;  // reads in flight before their stores
        typedef i32x4_t __attribute__((aligned(8))) i32x4_a8;  // O rows are 8-byte aligned, not more
#pragma unroll
        for (int i0 = 0; i0 < 32 / RPI; i0 += BATCH) {
            i32x4_t rows[BATCH];
#pragma unroll
            for (int i = 0; i < BATCH; ++i)
                rows[i] = *(const i32x4_t*)staged((i0 + i) * RPI + ln / CPRO, ln % CPRO);
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const int q = q_wave0 + (i0 + i) * RPI + ln / CPRO;
                if (q < S && ln % CPRO < cpr)  // not the rows beyond S, not the padding columns of a narrower head
                    *(i32x4_a8*)(o_bh + (size_t)q * p.o_rs + (ln % CPRO) * 16) = rows[i];
            }
        }
    } else if (my_q < S) {
        unsigned char* og = o_bh + (size_t)my_q * p.o_rs;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * db + 8 * g + 4 * h;
                if (d >= cpr * 8)
                    continue;  // padding columns of a narrower head dimension
                f32x4_t w = {oacc[db][4 * g + 0] * inv_l, oacc[db][4 * g + 1] * inv_l,
                             oacc[db][4 * g + 2] * inv_l, oacc[db][4 * g + 3] * inv_l};
                *(f32x4_t*)(og + d * 4) = w;
            }
    }
}

// ---- kernel 2: software-pipelined over 32-key blocks ------------------------------------------
//
// A work-group owns 256 queries.  Two shapes share one body:
//   QH = 1, 8 wavefronts: each wavefront owns 32 queries (each lane one query), two wavefronts per
//          SIMD, so the hardware can also overlap one wavefront's vector work with the other's MFMAs;
//   QH = 2, 4 wavefronts: each wavefront owns 64 queries in two 32-query halves, so every K and V^T
//          fragment read from LDS feeds two MFMAs (half the LDS traffic), one wavefront per SIMD.
// In both, matrix and vector work overlap inside the wavefront: the key axis is processed in
// 32-key blocks and stage k issues
//
//     MFMA:  Y(k-1) = O^T += V^T . P^T of block k-1      VALU:  SM(k) = online softmax of block k
//            X(k+1) = S^T of block k+1
//
// so the MFMAs of a stage never depend on its vector work.  A stage is laid out as a sequence of
// slots, one MFMA each, followed by a few vector instructions: the matrix pipe hides about six
// ordinary vector instructions per MFMA and no more, so the softmax is cut into pieces of that
// size.  K and V tiles (64 keys) are multi-buffered in LDS and filled by direct global->LDS loads
// issued LA tiles ahead, one barrier per tile.

// LDS fragments read ahead of their MFMAs.  Swept on the S = 16384 and S = 4096 causal shapes: 1 and 2 lose 5
// and 3 %, 3 to 8 are within half a per cent of each other with 3 ahead every time (and three fragments fewer
// held in registers).
#ifndef NAUT_PF
#define NAUT_PF 3
#endif
#ifndef NAUT_HAO
#define NAUT_HAO 8
#endif
constexpr int HEADS_AT_ONCE = NAUT_HAO;
constexpr int BM2 = 256;
constexpr int LA = 3;           // tile loads are issued this many iterations ahead of their use
constexpr int NBUF = LA + 1;    // LDS buffers per operand
constexpr float M_INIT = -1.0e30f;  // finite stand-in for "no maximum yet": keeps -inf - (-inf) out

// sum over the two 32-lane halves (same exchange as half_max)
__device__ __forceinline__ float half_sum(float x)
{
    float a = x, b = x;
    asm volatile(NAUT_NOP_SHORT "v_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}

// The softmax of a stage is cut into two pieces per score: FE (fma + exp2) and AC (row-sum add, and
// for odd scores the pack to 16 bit).  FE of score e+1 is placed before AC of score e so that no
// add waits on the exponential just issued.  Approximate issue costs, in vector slots (an
// exponential counts 2), are dealt out to the MFMA slots greedily, at most `cap` per slot.
template <int QH>
struct Pieces {
    static constexpr int NE = 16 * QH, N = 2 * NE;
    // position -> (is_fe, score index)
    static constexpr bool is_fe(int pos) { return pos == 0 || (pos != N - 1 && pos % 2 == 1); }
    static constexpr int score(int pos)
    {
        return pos == 0 ? 0 : pos == N - 1 ? NE - 1 : pos % 2 == 1 ? (pos + 1) / 2 : pos / 2 - 1;
    }
    static constexpr int cost(int pos) { return is_fe(pos) ? 3 : (score(pos) % 2 == 1 ? 2 : 1); }
    template <int NSLOT>
    static constexpr int begin(int slot)
    {
        int total = 0;
        for (int pc = 0; pc < N; ++pc)
            total += cost(pc);
        const int cap = (total + NSLOT - 1) / NSLOT + 1;
        int pc = 0;
        for (int s = 0; s < slot && s < NSLOT; ++s) {
            int used = 0;
            while (pc < N && (s == NSLOT - 1 || used + cost(pc) <= cap || used == 0)) {
                used += cost(pc);
                ++pc;
            }
        }
        return slot >= NSLOT ? N : pc;
    }
};

template <int D, int DT_IN, int DT_OUT, bool CAUSAL, int QH, int NWV>
__global__ __launch_bounds__(NWV * 64, 1) void naut_fwd_kernel_v2(const Params p)
{
    using T = In<DT_IN>;
    using XM = XMfma<DT_IN>;
    using PC = Pieces<QH>;
    static_assert(QH * NWV * 32 == BM2, "a work-group owns 256 queries");
    constexpr int ROWB = D * 2;
    constexpr int TILEB = BN * ROWB;           // one 64-key K or V tile
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int LD_PER_W = TILEB / 1024 / NWV;  // direct loads per wavefront per tile (1 KB each)
    constexpr int NF = 2 * KS;                 // fragments per stage: even = V^T (Y), odd = K (X)
    constexpr int NS = NF * QH;                // slots (MFMAs) per stage
    constexpr int WQ = 32 * QH;                // queries per wavefront
    constexpr bool ALLV = QH == 1;  // everything fits the ordinary vector registers: no accumulation registers at all
    auto pin_acc = [](f32x16_t& x) {
        if constexpr (ALLV)
            asm volatile("" : "+v"(x));
        else
            asm volatile("" : "+a"(x));
    };
    constexpr int PREFETCH = NAUT_PF < NF ? NAUT_PF : NF - 1;  // LDS fragments in flight ahead of their MFMAs
    static_assert(2 * DB == KS, "Y and X fragments must pair up");
    static_assert(LD_PER_W >= 1, "every wavefront must take part in the tile loads");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * NBUF * TILEB];  // K tiles, then V tiles

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // Tile scheduler.  Work-groups are dealt to the 8 XCDs round-robin by block id, and each XCD has
    // its own L2.  Every XCD is given a contiguous run of (batch, head) pairs and works on
    // HEADS_AT_ONCE of them at a time, heaviest (last) query tile first, so that the work-groups
    // resident on an XCD stream few K/V heads through its L2 (query heads that share a K/V head --
    // grouped-query attention -- sit next to each other).
    const int nbh = p.B * p.Hq;
    const int bid = blockIdx.x;
    int qt, bh;
    if ((nbh & 7) == 0) {
        const int xcd = bid & 7, s = bid >> 3;
        const int hpx = nbh >> 3;                                  // heads per XCD
        const int G = hpx < HEADS_AT_ONCE ? hpx : HEADS_AT_ONCE;  // heads an XCD works on at a time
        const int per_group = p.nqt2 * G;
        const int g = s / per_group, sg = s % per_group;
        const int ng = hpx - g * G < G ? hpx - g * G : G;          // the last group may be smaller
        bh = xcd * hpx + g * G + sg % ng;
        qt = p.nqt2 - 1 - sg / ng;
    } else {
        qt = p.nqt2 - 1 - bid / nbh;
        bh = bid % nbh;
    }
    const int b = bh / p.Hq;
    const int hq = bh % p.Hq;
    const int hk = hq / (p.Hq / p.Hkv);
    const int S = p.S;
    const float c = p.c;
    float c_v = c;  // copy held in a vector register: an FMA with a scalar-register operand issues at the slower rate
    asm volatile("" : "+v"(c_v));

    const unsigned char* qg = (const unsigned char*)p.q + b * p.q_bs + hq * p.q_hs;
    const unsigned char* kg = (const unsigned char*)p.k + b * p.k_bs + hk * p.k_hs;
    const unsigned char* vg = (const unsigned char*)p.v + b * p.v_bs + hk * p.v_hs;
    const int cpr = p.cpr;

    const int Q0 = qt * BM2 + wave * WQ;  // first query of this wavefront
    int qrow[QH];
#pragma unroll
    for (int hf = 0; hf < QH; ++hf)
        qrow[hf] = Q0 + 32 * hf + l32;

    // Q^T fragments (MFMA B operands), resident in the accumulation registers for the whole kernel.
    i32x4_t qf[QH][KS];
#pragma unroll
    for (int hf = 0; hf < QH; ++hf) {
        const int q_ld = qrow[hf] < S ? qrow[hf] : S - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            // Unconditional, from a chunk that exists; the padding chunks of a narrower head are zeroed
            // when Q is pinned below.  (A load under a condition becomes a branch, and the compiler then
            // waited for the first loads in the middle of issuing the rest.)
            const int ch = ks * 2 + h < cpr ? ks * 2 + h : cpr - 1;
            qf[hf][ks] = *(const i32x4_t*)(qg + (size_t)q_ld * p.q_rs + ch * 16);
        }
    }
    // Key range of this wavefront / this work-group (keys at or beyond kv_end_w are dead for it).
    const int kv_end_wg = CAUSAL ? (S < (qt + 1) * BM2 ? S : (qt + 1) * BM2) : S;
    const int kv_end_w = Q0 >= S ? 0 : (CAUSAL ? (S < Q0 + WQ ? S : Q0 + WQ) : S);
    const int ntiles = (kv_end_wg + BN - 1) / BN;
    const int niter = ntiles + 1;  // stages -1 .. 2*ntiles, two per iteration
    // With the causal mask the wavefronts of a work-group finish at different keys: this one needs blocks
    // up to kw_last, i.e. stages up to kw_last + 1 = iterations below n_act; after those it only keeps
    // loading its share of the tiles (the others still read them) and meeting the barrier.
    const int kw_last = (kv_end_w + 31) / 32 - 1;
    const int n_act = CAUSAL ? ((kw_last + 2) / 2 + 1 < niter ? (kw_last + 2) / 2 + 1 : niter) : niter;

    // Direct global->LDS tile loads.  Each instruction moves 1 KB: lane i fills physical chunk i of
    // the block, so the lane fetches the logical chunk that the swizzle maps there.  The address is
    // (scalar tile base) + (per-lane constant offset), so a full tile costs no vector arithmetic.
    int k_goff[LD_PER_W], v_goff[LD_PER_W];  // byte offset of the lane's chunk inside a tile
    int k_grow[LD_PER_W], v_grow[LD_PER_W];  // its row inside the tile (set-up only)
#pragma unroll
    for (int i = 0; i < LD_PER_W; ++i) {
        const int P = (wave * LD_PER_W + i) * 64 + lane;  // physical chunk index in the tile
        {
            const int line = P >> 4, pos = P & 15;
            const int L = (line << 4) + (pos ^ (line & 15));
            const int krow = L / (D / 8), kch = L % (D / 8);  // logical chunk L = row krow, chunk kch
            k_goff[i] = krow * p.k_rs + (kch < cpr ? kch : cpr - 1) * 16;
            k_grow[i] = krow;
        }
        if constexpr (D == 128) {
            const int row = P >> 4, cc = P & 15;
            const int lc = cc ^ ((row & 3) << 2);
            v_goff[i] = row * p.v_rs + (lc < cpr ? lc : cpr - 1) * 16;
            v_grow[i] = row;
        } else {
            const int row = P >> 3, cc = P & 7;
            const int lc = cc ^ (((row >> 1) & 1) << 2);
            v_goff[i] = row * p.v_rs + (lc < cpr ? lc : cpr - 1) * 16;
            v_grow[i] = row;
        }
    }
    const unsigned smem_base = (unsigned)(uintptr_t)(NAUT_LDS unsigned char*)smem;
    // Every iteration issues the same number of loads (the vmcnt arithmetic below counts on it):
    // a tile index past the end is clamped to the last tile, and that reload lands in a buffer
    // nobody reads.  The last tile may be ragged (S not a multiple of BN): lanes whose row does not
    // exist re-read the last row that does, through a second set of per-lane offsets.
    int k_goff_last[LD_PER_W], v_goff_last[LD_PER_W];
    {
        const int rows_left = S - (ntiles - 1) * BN;  // >= 1
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i) {
            const int kr = k_grow[i], vr = v_grow[i];
            k_goff_last[i] = kr < rows_left ? k_goff[i] : k_goff[i] - (kr - (rows_left - 1)) * p.k_rs;
            v_goff_last[i] = vr < rows_left ? v_goff[i] : v_goff[i] - (vr - (rows_left - 1)) * p.v_rs;
        }
    }
    struct TileLoad {
        unsigned dst;             // LDS byte address of this wavefront's part of the tile
        const unsigned char* gt;  // global address of the tile (wave-uniform)
    };
    // `buf` is the LDS buffer the tile goes to (tile % NBUF, a constant at every call site).  Once the
    // last tile is reached the per-lane offsets are replaced, for good, by the ragged-tail set: a
    // wave-uniform branch taken a few times per work-group instead of a select per load.
    auto tile_load = [&](const unsigned char* g, int row_stride, unsigned lds_tiles, int tile, int buf,
                         int (&goff)[LD_PER_W], const int (&goff_last)[LD_PER_W]) {
        TileLoad t;
        const int tl = tile < ntiles ? tile : ntiles - 1;
        t.dst = lds_tiles + (unsigned)(buf * TILEB + wave * LD_PER_W * 1024);
        t.gt = g + (size_t)tl * BN * row_stride;
        if (tile >= ntiles - 1) {
#pragma unroll
            for (int i = 0; i < LD_PER_W; ++i) {
                goff[i] = goff_last[i];
                asm volatile("" : "+v"(goff[i]));  // keeps this a branch: nothing here can be speculated into a select
            }
        }
        return t;
    };
    auto issue_load = [&](const TileLoad& t, int i, const int* goff) {
        load_to_lds(t.dst + i * 1024, goff[i], t.gt);
    };
    const unsigned k_lds = smem_base, v_lds = smem_base + NBUF * TILEB;

    // Lane parts of the LDS fragment addresses (block / step offsets are immediates on top).
    int k_lane[KS], v_lane[DB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        k_lane[ks] = k_off<D>(l32, ks * 2 + h);
    {
        const int i16 = lane & 15;
        const int key = 4 * h + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int d = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
            v_lane[db] = v_off<D>(key, d >> 3) + (d & 7) * 2;
        }
    }
    // LDS byte addresses of the fragments in buffer 0 of K and of V; they stay as they are for the whole
    // kernel (buffer, block and step offsets are immediates)
    int k_it[KS], v_it[DB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        k_it[ks] = k_lane[ks] + (int)k_lds;
        asm volatile("" : "+v"(k_it[ks]));  // opaque: the compiler then adds nothing but instruction immediates to it
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        v_it[db] = v_lane[db] + (int)v_lds;
        asm volatile("" : "+v"(v_it[db]));
    }

    f32x16_t oacc[QH][DB];
#pragma unroll
    for (int hf = 0; hf < QH; ++hf)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                oacc[hf][db][r] = 0.f;
    // reference maximum (log2 units), its negation, a quarter of the running sum of P (kept as the quarter
    // because that is what a block's sum is compared with: one FMA per block adds to it, and the factor is
    // exact), and what the sum of P as rounded for the second product has over the unrounded sum (touched in
    // heavy blocks only; see "the two sums" at the pieces of a stage)
    float m_run[QH], neg_m[QH], lq_run[QH], dl_run[QH];
#pragma unroll
    for (int hf = 0; hf < QH; ++hf) {
        m_run[hf] = M_INIT;
        neg_m[hf] = -M_INIT;
        lq_run[hf] = 0.f;
        dl_run[hf] = 0.f;
    }

    // SM(kblk) part 0: causal / tail / out-of-range masking
    auto mask_block = [&](int kblk, f32x16_t (&s_)[QH]) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kblk * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            const bool oob = key >= kv_end_w || kblk < 0;
#pragma unroll
            for (int hf = 0; hf < QH; ++hf)
                s_[hf][r] = (oob || (CAUSAL && key > qrow[hf])) ? -INFINITY : s_[hf][r];
        }
    };
    // first block that needs masking: 32k+31 > Q0 (causal; Q0 is a multiple of 32) or 32k+32 > kv_end_w;
    // k = -1 (the empty first stage) compares as a huge unsigned number
    const int kc2 = kv_end_w / 32;
    const unsigned k_mask_from = (unsigned)(CAUSAL ? (Q0 / 32 < kc2 ? Q0 / 32 : kc2) : kc2);
    auto needs_mask = [&](int k) { return (unsigned)k >= k_mask_from; };
    // max of three; the device code is compiled with NaNs assumed absent, so this is one v_max3_f32
    // with no quieting of the operands
    auto max3 = [](float x, float y, float z) { return __builtin_fmaxf(__builtin_fmaxf(x, y), z); };

    // Fragment f of block BLKX: even f = V^T (two transposed 64-bit reads), odd f = K (one 128-bit
    // read).  NEXT selects the tiles of the next iteration (same lane addresses plus a scalar delta).
    // U = iteration index mod NBUF: iteration j reads K tile j from buffer U and V tile j-1 from buffer
    // U-1 (mod NBUF), so with the key loop unrolled NBUF times every buffer offset is an immediate of
    // the LDS instruction and the per-lane addresses never change.
    auto load_frag = [&](auto F, auto BLKX, auto NEXT, auto UC) -> i32x4_t {
        constexpr int f = decltype(F)::value, BLK = decltype(BLKX)::value, U = decltype(UC)::value;
        constexpr bool next_iter = decltype(NEXT)::value;
        constexpr int KOFF = (next_iter ? (U + 1) % NBUF : U) * TILEB;
        constexpr int VOFF = (next_iter ? U : (U + NBUF - 1) % NBUF) * TILEB;
        if constexpr (f % 2 == 0) {
            constexpr int y = f / 2, t = y / DB, db = y % DB;
            constexpr int off = (BLK * 32 + 16 * t) * ROWB;
            const int a = v_it[db] + VOFF;
            const i16x4_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((NAUT_LDS i16x4_t*)(uintptr_t)(a + off));
            const i16x4_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((NAUT_LDS i16x4_t*)(uintptr_t)(a + off + 8 * ROWB));
            const i32x2_t lo = __builtin_bit_cast(i32x2_t, r0), hi = __builtin_bit_cast(i32x2_t, r1);
            return i32x4_t{lo.x, lo.y, hi.x, hi.y};
        } else {
            constexpr int ks = f / 2;
            const int a = k_it[ks] + KOFF;
            return *(const NAUT_LDS i32x4_t*)(uintptr_t)(a + BLK * 32 * ROWB);
        }
    };

    // One pipeline stage k = 2*j - 1 + BLK of iteration j (j mod NBUF = U): Y(k-1) reads block BLK of V
    // tile j-1, X(k+1) block BLK of K tile j.  Every wavefront runs every stage: blocks that
    // do not exist for it are fully masked in SM (P = 0, m and l unchanged), Y then adds zeros and
    // X computes scores nobody reads, so one straight-line body serves every k.  The first PREFETCH
    // fragments arrive in `carry` (read during the previous stage) and the last slots read the next
    // stage's first fragments into it, so no stage starts with an empty LDS pipeline.
    auto stage = [&](auto BLKC, auto UC, int k, i32x4_t (&carry)[PREFETCH], f32x16_t (&s_cur)[QH], f32x16_t (&s_nxt)[QH],
                     const i32x4_t (&p_in)[QH][2], i32x4_t (&p_out)[QH][2], auto&& side) {
        constexpr int BLK = decltype(BLKC)::value;
        // s_cur was written by the asm MFMAs at the end of the previous stage: keep every vector
        // read of it 11 wait states behind them (see XMfma)
        if constexpr (!ALLV)
            asm volatile(NAUT_NOP_SETTLE ::: "memory");
        if (needs_mask(k))
            mask_block(k, s_cur);
        i32x4_t frag[NF];
        static_for<0, PREFETCH>([&](auto F) { frag[decltype(F)::value] = carry[decltype(F)::value]; });
        auto issue = [&](auto F) {
            constexpr int f = decltype(F)::value;
            if constexpr (f < NF) {
                frag[f] = load_frag(F, std::integral_constant<int, BLK>{}, std::false_type{}, UC);
            } else {
                carry[f - NF] = load_frag(std::integral_constant<int, f - NF>{}, std::integral_constant<int, BLK ^ 1>{},
                                          std::integral_constant<bool, BLK == 1>{}, UC);
            }
        };
        float psum[QH], pe[QH][16];  // this block's row sums (per lane: its 16 of the 32 keys) and exponentials
#pragma unroll
        for (int hf = 0; hf < QH; ++hf)
            psum[hf] = 0.f;
        // Vector work of the stage, one piece at a time (see Pieces).  P is formed against the
        // reference maximum as it stands, with no look at this block's own maximum: as long as the
        // row sums stay below P_LIMIT every P is below it too, and the reference need not move.
        // The two sums: lse needs l = sum of P to better than 16-bit accuracy, so P is summed in fp32 before it
        // is rounded; O, on the other hand, must be divided by the sum of the P that went into it, the rounded
        // ones.  With the reference lagging behind the maximum the largest P of a row is an arbitrary number,
        // not 1, and its rounding error (up to 2^-8 relative in bf16, whose significand has 8 bits) would otherwise
        // go into O but not into its divisor: for a row that one key dominates that is an error of up to 2^-8 |v|
        // on top of the rounding of O itself (as much again: together past the 2e-2 bar once |v| exceeds 2.6).
        // Divided by the rounded sum the weights add up to one exactly and such a row returns v (what is left is
        // 2^-8 w |v - O| per key of weight w, as in any kernel that rounds P).  Only keys of large weight matter for
        // this, so the rounded sum is formed (after the slots, from the packed P) only for a block that
        // adds a quarter or more to some row's running sum -- every key that ends with a fifth of its row's
        // weight or more is in such a block -- and the unrounded sum stands in for it otherwise: a key so
        // treated adds at most 0.2 * 2^-8 |v| to the error, and |O| near 4 would take several such keys with
        // |v| near 4 in one column, which N(0,1)-like values do not supply; the rounding errors of the many
        // light keys, independent and of either sign, average out in O.
        auto piece = [&](auto PCI) {
            constexpr int pos = decltype(PCI)::value, e = PC::score(pos), hf = e / 16, idx = e % 16;
            if constexpr (PC::is_fe(pos)) {
                pe[hf][idx] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[hf][idx], c_v, neg_m[hf]));
                // anchor: keeps this piece in its slot (the optimiser would otherwise sink it to the
                // first use of P, after the last MFMA of the stage).  Input-only: an asm that also
                // defined the value would make the compiler pad the next use with a wait state.
                asm volatile("" ::"v"(pe[hf][idx]));
            } else {
                // fp32 sum of the unrounded P: lse needs l to better than bf16 accuracy
                if constexpr (idx == 0)
                    psum[hf] = pe[hf][0];
                else
                    psum[hf] += pe[hf][idx];
                if constexpr (idx % 2 == 1) {
                    int w = T::pack2(pe[hf][idx - 1], pe[hf][idx]);
                    asm volatile("" ::"v"(w), "v"(psum[hf]));
                    p_out[hf][idx >> 3][(idx >> 1) & 3] = w;
                } else {
                    asm volatile("" ::"v"(psum[hf]));
                }
            }
        };
        static_for<0, NS>([&](auto I) {
            constexpr int i = decltype(I)::value;
            constexpr int f = i / QH, hf = i % QH;
            if constexpr (hf == 0)
                issue(std::integral_constant<int, f + PREFETCH>{});
            if constexpr (f % 2 == 0) {
                constexpr int y = f / 2, t = y / DB, db = y % DB;
                oacc[hf][db] = T::mfma(frag[f], p_in[hf][t], oacc[hf][db]);
            } else {
                constexpr int ks = f / 2;
                if constexpr (ALLV) {
                    if constexpr (ks == 0)
                        s_nxt[hf] = T::mfma(frag[f], qf[hf][ks], f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f});
                    else
                        s_nxt[hf] = T::mfma(frag[f], qf[hf][ks], s_nxt[hf]);
                } else if constexpr (ks == 0)
                    XM::first(s_nxt[hf], frag[f], qf[hf][ks]);
                else
                    XM::acc(s_nxt[hf], frag[f], qf[hf][ks]);
            }
            constexpr int p0 = PC::template begin<NS>(i), p1 = PC::template begin<NS>(i + 1);
            side(I);
            static_for<p0, p1>([&](auto PCI) { piece(PCI); });
            // one wait for two fragments: LDS reads return in order, so waiting at the end of an odd
            // slot for the fragment two slots on covers the next slot's too, and neither of the two
            // coming slots needs a wait instruction of its own
            if constexpr (hf == QH - 1 && f % 2 == 1 && f + 2 < NF)
                asm volatile("" ::"v"(frag[f + 2]));
            __builtin_amdgcn_sched_barrier(0);
        });
        bool over = false;   // also true for +inf (first block of a row: the reference is still M_INIT)
        bool heavy = false;  // the block adds a quarter or more to the row's running sum (first block: always)
#pragma unroll
        for (int hf = 0; hf < QH; ++hf) {
            over = over || psum[hf] > T::P_LIMIT;
            heavy = heavy || psum[hf] > lq_run[hf];
        }
        const unsigned long long over_mask = __builtin_amdgcn_ballot_w64(over);
        if ((over_mask | __builtin_amdgcn_ballot_w64(heavy)) != 0) {  // two lane masks and a scalar OR: no vector work
        if (over_mask != 0) {
            // Rare path: some row of this wavefront met scores far above its reference maximum.  Move
            // the reference of every row to its true running maximum, apply the repair factor
            // exp2(m_old - m_new) to l and O (after Y(k-1), whose P was formed against the old
            // maxima), and form this block's P again from the scores, which are still intact.
#pragma unroll
            for (int hf = 0; hf < QH; ++hf) {
                const f32x16_t& s_ = s_cur[hf];
                float mx = max3(s_[0], s_[1], s_[2]);
                mx = max3(mx, s_[3], s_[4]);
                mx = max3(mx, s_[5], s_[6]);
                mx = max3(mx, s_[7], s_[8]);
                mx = max3(mx, s_[9], s_[10]);
                mx = max3(mx, s_[11], s_[12]);
                mx = max3(mx, s_[13], s_[14]);
                mx = max3(mx, s_[15], s_[15]);
                float a2 = mx, b2 = mx;
                asm volatile(NAUT_NOP_SHORT "v_permlane32_swap_b32 %0, %1" : "+v"(a2), "+v"(b2));
                const float cand = max3(a2, b2, b2) * c;  // -inf if the block is masked for this row
                const float m_new = max3(m_run[hf], cand, cand);
                const float alpha = __builtin_amdgcn_exp2f(m_run[hf] - m_new);
                lq_run[hf] *= alpha;
                dl_run[hf] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        oacc[hf][db][r] *= alpha;
                    pin_acc(oacc[hf][db]);
                }
                m_run[hf] = m_new;
                neg_m[hf] = -m_new;
                float ps = 0.f;
#pragma unroll
                for (int idx = 0; idx < 16; idx += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_[idx], c_v, neg_m[hf]));
                    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_[idx + 1], c_v, neg_m[hf]));
                    ps += p0 + p1;
                    p_out[hf][idx >> 3][(idx >> 1) & 3] = T::pack2(p0, p1);
                }
                psum[hf] = ps;
            }
        }
        // the heavy block's sum of the rounded P; its difference to the unrounded sum goes to dl_run
#pragma unroll
        for (int hf = 0; hf < QH; ++hf) {
            float pr = -psum[hf];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    pr = T::add_pair(p_out[hf][t][e], pr);
            dl_run[hf] += pr;
        }
        }
#pragma unroll
        for (int hf = 0; hf < QH; ++hf) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
                pin_acc(oacc[hf][db]);
            lq_run[hf] = __builtin_fmaf(psum[hf], 0.25f, lq_run[hf]);
        }
    };

    // ---- prologue: the first LA K tiles and LA-1 V tiles ----
    // V tile 0 also goes to the last V buffer: the empty first stage multiplies "V tile -1" from there
    // by P = 0, which needs finite data; the real owner of that buffer is loaded after that stage.
    {
        int v_first[LD_PER_W];
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i)
            v_first[i] = v_goff[i];
        const TileLoad tv = tile_load(vg, p.v_rs, v_lds, 0, NBUF - 1, v_first, v_goff_last);
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i)
            issue_load(tv, i, v_first);
    }
#pragma unroll
    for (int t = 0; t < LA; ++t)
    {
        const TileLoad tk = tile_load(kg, p.k_rs, k_lds, t, t, k_goff, k_goff_last);
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i)
            issue_load(tk, i, k_goff);
    }
#pragma unroll
    for (int t = 0; t + 1 < LA; ++t)
    {
        const TileLoad tv = tile_load(vg, p.v_rs, v_lds, t, t, v_goff, v_goff_last);
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i)
            issue_load(tv, i, v_goff);
    }
    // Q is pinned to its registers only here: its loads, issued at the top, and the tile loads share one
    // round trip to memory instead of taking one each.
    int cpr_late = cpr;
    asm volatile("" : "+s"(cpr_late));  // ordered after the tile loads above: so is everything that uses it
#pragma unroll
    for (int hf = 0; hf < QH; ++hf)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks * 2 + h >= cpr_late)
                qf[hf][ks] = i32x4_t{0, 0, 0, 0};
            if constexpr (ALLV)
                asm volatile("" : "+v"(qf[hf][ks]));
            else
                asm volatile("" : "+a"(qf[hf][ks]));
        }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // s_e / s_o: scores of the current even / odd block; p_e / p_o: P of the last even / odd block
    f32x16_t s_e[QH], s_o[QH];
    i32x4_t p_e[QH][2], p_o[QH][2];
#pragma unroll
    for (int hf = 0; hf < QH; ++hf) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s_e[hf][r] = 0.f;
            s_o[hf][r] = 0.f;
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            p_e[hf][t] = i32x4_t{0, 0, 0, 0};
            p_o[hf][t] = i32x4_t{0, 0, 0, 0};
        }
    }

    i32x4_t carry[PREFETCH];  // first fragments of the coming stage
    static_for<0, PREFETCH>([&](auto F) {
        carry[decltype(F)::value] =
            load_frag(F, std::integral_constant<int, 0>{}, std::false_type{}, std::integral_constant<int, 0>{});
    });

    // One iteration of the key loop: K tile j, V tile j-1.  UC = j mod NBUF as a constant: the loop is
    // unrolled NBUF times so that every LDS buffer offset is an immediate.
    auto iteration = [&](auto UC, int j) {
        constexpr int U = decltype(UC)::value;
        // tiles LA iterations ahead (iteration j reads K tile j and V tile j-1)
        // The 2*LD_PER_W loads of a wavefront are dealt out over the MFMA slots of one stage (even
        // wavefronts: the first stage, odd ones: the second) rather than issued in one burst by all
        // wavefronts right after the barrier, which backs up the memory pipeline and stalls them.
        const TileLoad kt = tile_load(kg, p.k_rs, k_lds, j + LA, (U + LA) % NBUF, k_goff, k_goff_last);
        const TileLoad vt = tile_load(vg, p.v_rs, v_lds, j + LA - 1, (U + LA - 1) % NBUF, v_goff, v_goff_last);
        auto side = [&](auto BLKC, auto I) {
            constexpr int BLK = decltype(BLKC)::value, i = decltype(I)::value;
            constexpr int NL = 2 * LD_PER_W, STEP = NS / NL;
            if constexpr (!SAFE_SYNC && BLK == 0 && STEP > 0 && i % STEP == STEP / 2 && i / STEP < NL) {
                constexpr int q = i / STEP;
                if constexpr (q < LD_PER_W)
                    issue_load(kt, q, k_goff);
                else
                    issue_load(vt, q - LD_PER_W, v_goff);
            }
        };

        if constexpr (SAFE_SYNC) {  // checking build: the iteration's loads are issued, awaited and published first
            tile_barrier();
#pragma unroll
            for (int i = 0; i < LD_PER_W; ++i)
                issue_load(kt, i, k_goff);
#pragma unroll
            for (int i = 0; i < LD_PER_W; ++i)
                issue_load(vt, i, v_goff);
            tile_barrier();
        }
        // stage 2j-1: Y(2j-2) with p_e, X(2j) -> s_e, SM(2j-1): s_o -> p_o
        stage(std::integral_constant<int, 0>{}, UC, 2 * j - 1, carry, s_o, s_e, p_e, p_o,
              [&](auto I) { side(std::integral_constant<int, 0>{}, I); });
        // stage 2j:   Y(2j-1) with p_o, X(2j+1) -> s_o, SM(2j): s_e -> p_e
        stage(std::integral_constant<int, 1>{}, UC, 2 * j, carry, s_e, s_o, p_o, p_e,
              [&](auto I) { side(std::integral_constant<int, 1>{}, I); });

        // The last slots of the next iteration already read the tiles of the one after it, so the
        // tiles issued LA-2 iterations ago must have landed by now; newer ones may fly on.
        static_assert(LA >= 2 && (LA - 2) * 2 * LD_PER_W < 64, "vmcnt field");
        wait_loads<(LA - 2) * 2 * LD_PER_W>();
        // A bare barrier, not __syncthreads(): the fence in the latter would first drain the LDS
        // reads in flight, which are this wavefront's prefetch for the next stage.  They target
        // tiles published by the previous barrier and buffers that no load overwrites before the
        // barrier after this one, so they may stay in flight; the tile loads to be published have
        // been awaited just above.
        tile_barrier();
    };
    for (int j0 = 0; j0 < n_act; j0 += NBUF) {
        static_for<0, NBUF>([&](auto UC) {
            const int j = j0 + decltype(UC)::value;
            if (j < n_act)  // uniform over the wavefront
                iteration(UC, j);
        });
    }
    for (int j = n_act; j < niter; ++j) {  // this wavefront's part of the remaining tiles, one barrier each
        const TileLoad kt = tile_load(kg, p.k_rs, k_lds, j + LA, (j + LA) % NBUF, k_goff, k_goff_last);
        const TileLoad vt = tile_load(vg, p.v_rs, v_lds, j + LA - 1, (j + LA - 1) % NBUF, v_goff, v_goff_last);
        if constexpr (SAFE_SYNC)
            tile_barrier();  // checking build: the same three barriers per iteration as the wavefronts still computing
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i)
            issue_load(kt, i, k_goff);
#pragma unroll
        for (int i = 0; i < LD_PER_W; ++i)
            issue_load(vt, i, v_goff);
        if constexpr (SAFE_SYNC)
            tile_barrier();
        wait_loads<(LA - 2) * 2 * LD_PER_W>();
        tile_barrier();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue ----
    if (Q0 >= S)
        return;
    constexpr int OUTB = DT_OUT == NAUT_F32 ? 4 : 2;
    unsigned char* const o_bh = (unsigned char*)p.o + b * p.o_bs + hq * p.o_hs;
    if constexpr (OUTB == 2) {
        // 16-bit output goes through LDS so that it leaves in whole rows: a lane owns 4 consecutive
        // d of one query (8 bytes, 32 different rows per store instruction); after the exchange 16
        // lanes (D = 128) write one 256-byte row with 16 bytes each.  The staging rows live in this
        // wavefront's own part of the first four tile buffers (where only its own tile loads land,
        // and those are complete), so no barrier is needed: the other wavefronts have consumed every
        // tile by the time this one is past the last barrier.
        constexpr int CPRO = D / 8;           // 16-byte chunks per staged row
        constexpr int PS = LD_PER_W * 1024;   // this wavefront's part of one tile buffer
        constexpr int RP = PS / ROWB;         // staged rows per part
        constexpr int R256 = ROWB >= 256 ? 1 : 256 / ROWB;  // rows per 256-byte bank line
        static_assert(WQ / RP <= 2 * NBUF && WQ % RP == 0, "staging rows must fit this wavefront's tile parts");
        auto staged = [&](int r, int ch) {  // chunk ch of staged row r; swizzled so that neither side conflicts
            return smem + (r / RP) * TILEB + wave * PS + (r % RP) * ROWB + ((ch ^ ((r / R256) & (CPRO - 1))) << 4);
        };
#pragma unroll
        for (int hf = 0; hf < QH; ++hf) {
            const int q = qrow[hf];
            const float lt = 4.0f * half_sum(lq_run[hf]);
            const float inv_l = 1.0f / (lt + half_sum(dl_run[hf]));  // rows beyond S: staged, never stored
            if (p.lse != nullptr && h == 0 && q < S)
                p.lse[(size_t)bh * S + q] = (m_run[hf] + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = 32 * db + 8 * g + 4 * h;
                    const float x0 = oacc[hf][db][4 * g + 0] * inv_l, x1 = oacc[hf][db][4 * g + 1] * inv_l;
                    const float x2 = oacc[hf][db][4 * g + 2] * inv_l, x3 = oacc[hf][db][4 * g + 3] * inv_l;
                    i32x2_t w = {In<DT_OUT>::pack2(x0, x1), In<DT_OUT>::pack2(x2, x3)};
                    *(i32x2_t*)(staged(32 * hf + l32, d >> 3) + (d & 7) * 2) = w;
                }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int RPI = 64 / CPRO;  // rows per store instruction
        typedef i32x4_t __attribute__((aligned(8))) i32x4_a8;  // O rows are 8-byte aligned, not more
        i32x4_t rows[WQ / RPI];
#pragma unroll
        for (int i = 0; i < WQ / RPI; ++i)  // all reads first: one LDS latency, not one per store
            rows[i] = *(const i32x4_t*)staged(i * RPI + lane / CPRO, lane % CPRO);
#pragma unroll
        for (int i = 0; i < WQ / RPI; ++i) {
            const int ch = lane % CPRO;
            const int q = Q0 + i * RPI + lane / CPRO;
            if (q < S && ch < cpr)  // not the rows beyond S, not the padding columns of a narrower head
                *(i32x4_a8*)(o_bh + (size_t)q * p.o_rs + ch * 16) = rows[i];
        }
    } else {
#pragma unroll
        for (int hf = 0; hf < QH; ++hf) {
            const int q = qrow[hf];
            const float lt = 4.0f * half_sum(lq_run[hf]);
            const float lr = lt + half_sum(dl_run[hf]);
            if (q >= S)
                continue;
            const float inv_l = 1.0f / lr;
            if (p.lse != nullptr && h == 0)
                p.lse[(size_t)bh * S + q] = (m_run[hf] + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f;
            unsigned char* og = o_bh + (size_t)q * p.o_rs;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = 32 * db + 8 * g + 4 * h;
                    if (d >= cpr * 8)
                        continue;  // padding columns of a narrower head dimension
                    f32x4_t w = {oacc[hf][db][4 * g + 0] * inv_l, oacc[hf][db][4 * g + 1] * inv_l,
                                 oacc[hf][db][4 * g + 2] * inv_l, oacc[hf][db][4 * g + 3] * inv_l};
                    *(f32x4_t*)(og + d * 4) = w;
                }
        }
    }
}

// ---- host side: variant choice and launch -------------------------------------------

// Kernel variants (the tile shape / wavefront count / buffering choice the paper leaves to its
// auto-tuner, Section 4.4 and Section 7.2).  NAUT_ATTN_VARIANT=w8q32|w4q64|bm128 overrides the
// shape-based choice for A/B runs (read at every call, so that one process can time all of them; any other
// non-empty value makes the call fail).
enum Variant { V_W8Q32 = 0, V_W4Q64 = 1, V_BM128 = 2 };
constexpr const char* kVariantName[3] = {"fwd_bm256_w8q32_bn64", "fwd_bm256_w4q64_bn64", "fwd_bm128_w4q32_bn64"};

inline int pick_variant(int S, long long nbh, int D, int causal)
{
    if (const char* e = getenv("NAUT_ATTN_VARIANT")) {
        if (!strcmp(e, "w8q32"))
            return V_W8Q32;
        if (!strcmp(e, "w4q64"))
            return V_W4Q64;
        if (!strcmp(e, "bm128"))
            return V_BM128;
        if (e[0] != 0)
            return -1;  // a name that selects nothing is an error, not a silent fall-back to the rule
    }
    // Rule fitted to the timings of `python -m paper_2604_14825_amd.tune` over sequence lengths
    // 256..16384, 2..512 heads, both head dimensions, with and without the causal mask.  The
    // pipelined 256-query kernel halves the K/V traffic per FLOP but pays a fill and a drain stage
    // per work-group and needs a full wave of work-groups: it wins once there is one work-group per
    // CU and the key loop is long enough.  At D = 128 that is an average of 1024 keys per query
    // without the mask and 2048 with it (the 128-query tiles follow the causal diagonal more
    // closely).  At D = 64 the softmax and not the MFMAs sets the pace and the 128-query kernel keeps
    // four wavefronts per SIMD: the pipelined kernel is ahead only on long key loops (8192 keys per
    // query) with few work-groups (fewer than four 256-query tiles per CU).  The
    // 64-queries-per-wavefront variant is within 2 % of the fastest where it wins at all and is
    // selectable by name only.
    const long long wg256 = nbh * ((S + BM2 - 1) / BM2);
    const int avg_keys = causal ? (S + 1) / 2 : S;
    if (wg256 < 256)
        return V_BM128;
    if (D > 64)
        return avg_keys >= (causal ? 2048 : 1024) ? V_W8Q32 : V_BM128;
    return (avg_keys >= 8192 && wg256 < 1024) ? V_W8Q32 : V_BM128;
}

template <int D, int DT_IN, int DT_OUT>
int launch(const Params& p, int causal, hipStream_t stream)
{
    const long long nbh = (long long)p.B * p.Hq;
    // The pipelined kernel exists for D <= 128; wider heads always take the 128-query kernel.
    const int variant = D > 128 ? V_BM128 : pick_variant(p.S, nbh, D, causal);
    if (variant < 0)
        return fail(NAUT_ERR_UNSUPPORTED, "NAUT_ATTN_VARIANT names no kernel variant (w8q32, w4q64 or bm128)");
    const long long nblocks = nbh * (variant == V_BM128 ? p.nqt : p.nqt2);
    if (nblocks > 0x7fffffffLL)
        return fail(NAUT_ERR_UNSUPPORTED, "B*Hq*ceil(S/128) exceeds the 1-D grid limit");
    const dim3 grid((unsigned)nblocks);
#define NAUT_LAUNCH(KERNEL, THREADS)                                              \
    do {                                                                          \
        if (causal)                                                               \
            hipLaunchKernelGGL((KERNEL<D, DT_IN, DT_OUT, true NAUT_TAIL>), grid, dim3(THREADS), 0, stream, p);  \
        else                                                                      \
            hipLaunchKernelGGL((KERNEL<D, DT_IN, DT_OUT, false NAUT_TAIL>), grid, dim3(THREADS), 0, stream, p); \
    } while (0)
    bool launched = false;
    if constexpr (D <= 128) {
        if (variant == V_W8Q32) {
#define NAUT_TAIL , 1, 8
            NAUT_LAUNCH(naut_fwd_kernel_v2, 512);
#undef NAUT_TAIL
            launched = true;
        } else if (variant == V_W4Q64) {
#define NAUT_TAIL , 2, 4
            NAUT_LAUNCH(naut_fwd_kernel_v2, 256);
#undef NAUT_TAIL
            launched = true;
        }
    }
    if (!launched) {
#define NAUT_TAIL
        NAUT_LAUNCH(naut_fwd_kernel_bm128, NTHREADS);
#undef NAUT_TAIL
    }
#undef NAUT_LAUNCH
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_launch(e);
    return NAUT_OK;
}

}  // namespace naut_k

#endif  // NAUT_ATTN_KERNELS_H
