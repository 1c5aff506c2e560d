// naut_decode.hip -- decode-time attention for gfx950 (MI355X): a few new query positions per head
// against a long key/value cache (the paper's second workload, "DC", Section 6).
//
// The work is bound by reading K and V once from HBM, not by the matrix pipes, so the key axis is
// split across work-groups (and again across the four wavefronts of a work-group): every wavefront
// streams its own 32-key blocks of K and V through a private double buffer in LDS with direct
// global->LDS loads (no work-group barrier in the loop), runs the same transposed MFMA formulation
// as the prefill kernels on them (S^T = K.Q^T, online softmax with a lazily moved reference maximum,
// O^T += V^T.P^T), and the partial (O, m, l) triples are merged with the split-merge identity of
// softmax, first across the wavefronts through LDS, then across the splits by a second small kernel
// that reads them from a caller-provided workspace.
//
// Query heads that share a K/V head (grouped-query attention) and the Sq positions of each form the
// rows of one MFMA tile: for a fixed (batch, K/V head) the Hq/Hkv * Sq query rows are contiguous in
// memory, so they are simply rows 0..R-1 of a [R][D] matrix, taken 32 at a time.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdio>

#include "naut_attn.h"
#include "naut_common.h"

namespace {

using namespace naut;

#ifndef NAUT_DEC_WAVES
#define NAUT_DEC_WAVES 4
#endif
constexpr int DEC_WAVES = NAUT_DEC_WAVES;  // wavefronts of the split kernel, each with a private 4-block LDS region
constexpr int DEC_THREADS = DEC_WAVES * 64;
constexpr int MRG_WAVES = 4;               // wavefronts of the merge kernel
constexpr int MRG_THREADS = MRG_WAVES * 64;
constexpr int DEC_ROWS = 32;               // query rows per work-group (one MFMA tile)
constexpr int DEC_BLK = 32;                // keys per block
// The reference maximum of the 16-bit kernel moves whenever a row's maximum grows: the largest P of a row is
// then exactly 1 and carries no rounding error into O (with a reference that lags, the largest P is an
// arbitrary number whose rounding to 16 bit, up to 2^-8 relative in bf16, goes into O but not into l).  The
// rescaling this costs is vector work that a kernel bound by reading the cache has to spare.
constexpr float DEC_TAU = 0.0f;
constexpr float DEC_M_INIT = -1.0e30f;     // finite stand-in for "no maximum yet"
#ifndef NAUT_DEC_TARGET
#define NAUT_DEC_TARGET 256
#endif
constexpr int DEC_TARGET_WGS = NAUT_DEC_TARGET;  // one work-group per CU: only one is resident at a time (LDS), and a single round measured fastest (256..1024 tried)

struct DecodeParams {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    float* lse;
    float* ws;     // workspace: partial O [nparts][32][D], then m [nparts][32], then l [nparts][32]
    int B, Hq, Hkv, Sq, Sk;
    int R;         // query rows per (batch, K/V head) = Hq/Hkv * Sq
    int nchunks;   // ceil(R / 32)
    int nsplit;    // splits of the key axis
    int bps;       // 32-key blocks per split (a multiple of 4)
    int causal;
    float c;       // scale * log2(e) (FP8: times descale_q * descale_k), > 0
    float dv;      // factor on O: 1 (16-bit inputs) or descale_v (FP8)
    // byte strides of batch, head and sequence position (the D axis is contiguous)
    long long q_bs, q_hs, k_bs, k_hs, v_bs, v_hs, o_bs, o_hs;
    int q_rs, k_rs, v_rs, o_rs;
    // The kernels are compiled for D = 64, 128 or 256 (FP8: 64 or 128); a smaller head dimension runs on the next wider one:
    // cpr 16-byte chunks of every row are real, the chunks of Q beyond them read as zero, those of K and
    // V repeat a real chunk (they meet zeros of Q, or end in columns of O that are not stored).
    int cpr;
};

__device__ __forceinline__ float half_sum_f(float x)
{
    float a = x, b = x;
    asm volatile(NAUT_NOP_SHORT "v_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}

// Tail of a split kernel: the four wavefronts' partial (O, m, l) are merged through LDS (each wavefront
// reuses its own, now idle, region of REGION bytes) and the work-group's partial goes to the workspace.
// m is the reference maximum the wavefront's l and O are relative to (log2 units).
template <int D, int REGION, int NW>
__device__ __forceinline__ void merge_wavefronts(unsigned char* smem, const f32x16_t (&oacc)[D / 32], float m_run,
                                                 float l_run, const DecodeParams& p, int bhk, int chunk, int split)
{
    constexpr int DB = D / 32;
    constexpr int OSTRIDE = D + 4;  // floats per row of the partial O in LDS (padded against bank conflicts)
    static_assert(DEC_ROWS * OSTRIDE * 4 + 2 * DEC_ROWS * 4 <= REGION, "the wavefront's partial fits its LDS region");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;
    unsigned char* my_lds = smem + wave * REGION;
    // ---- merge the four wavefronts through LDS (each reuses its own, now idle, region) ----
    float* my_o = (float*)my_lds;                          // [32][OSTRIDE]
    float* my_ml = my_o + DEC_ROWS * OSTRIDE;              // m[32], l[32]
    const float l_tot = half_sum_f(l_run);
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int d = 32 * db + 8 * gq + 4 * h;
            const f32x4_t w = {oacc[db][4 * gq + 0], oacc[db][4 * gq + 1], oacc[db][4 * gq + 2], oacc[db][4 * gq + 3]};
            *(f32x4_t*)(my_o + l32 * OSTRIDE + d) = w;
        }
    if (h == 0) {
        my_ml[l32] = m_run;
        my_ml[DEC_ROWS + l32] = l_tot;
    }
    __syncthreads();

    // (row, D/8 consecutive d) items, dealt to the threads; partial written to the workspace
    constexpr int DPT = D / 8;  // floats per item: 32 (D = 256), 16 (D = 128) or 8 (D = 64)
    const size_t nparts = (size_t)p.B * p.Hkv * p.nchunks * p.nsplit;
    const size_t part = ((size_t)bhk * p.nchunks + chunk) * p.nsplit + split;
#pragma unroll
    for (int item = tid; item < DEC_ROWS * 8; item += NW * 64) {
    const int r_out = item >> 3, d0 = (item & 7) * DPT;
    float mw[NW], lw[NW];
    float M = DEC_M_INIT;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const float* ml = (const float*)(smem + w * REGION) + DEC_ROWS * OSTRIDE;
        mw[w] = ml[r_out];
        lw[w] = ml[DEC_ROWS + r_out];
        M = fmaxf(M, mw[w]);
    }
    float L = 0.f;
    f32x4_t acc[DPT / 4];
#pragma unroll
    for (int i = 0; i < DPT / 4; ++i)
        acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const float f = __builtin_amdgcn_exp2f(mw[w] - M);
        L += f * lw[w];
        const float* ow = (const float*)(smem + w * REGION) + r_out * OSTRIDE + d0;
#pragma unroll
        for (int i = 0; i < DPT / 4; ++i) {
            const f32x4_t x = *(const f32x4_t*)(ow + 4 * i);
            acc[i] += x * f;
        }
    }
    if (chunk * DEC_ROWS + r_out >= p.R)
        continue;  // rows past the last one are padding: nobody reads their partials
    float* ws_o = p.ws + (part * DEC_ROWS + r_out) * D + d0;
#pragma unroll
    for (int i = 0; i < DPT / 4; ++i)
        *(f32x4_t*)(ws_o + 4 * i) = acc[i];
    if ((item & 7) == 0) {
        float* ws_m = p.ws + nparts * DEC_ROWS * D;
        float* ws_l = ws_m + nparts * DEC_ROWS;
        ws_m[part * DEC_ROWS + r_out] = M;
        ws_l[part * DEC_ROWS + r_out] = L;
    }
    }
}

// wavefronts of the 16-bit split kernel: the four LDS blocks of a wavefront are 64 KB at D = 256
constexpr int dec_waves(int D) { return D > 128 ? 2 : DEC_WAVES; }

template <int D, int DT_IN>
__global__ __launch_bounds__(dec_waves(D) * 64, 1) void naut_decode_split_kernel(const DecodeParams p)
{
    using T = In<DT_IN>;
    constexpr int NW = dec_waves(D);
    constexpr int ROWB = D * 2;
    constexpr int BLKB = DEC_BLK * ROWB;   // one 32-key block of K or V
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int NLD = BLKB / 1024;       // direct loads (1 KB each) per block and operand

    __shared__ __attribute__((aligned(1024))) unsigned char smem[NW * 4 * BLKB];  // per wavefront: K0 V0 K1 V1

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    const int split = blockIdx.x, chunk = blockIdx.y, bhk = blockIdx.z;
    const int b = bhk / p.Hkv, hk = bhk % p.Hkv;
    const int g = p.Hq / p.Hkv;
    const int Sk = p.Sk;
    const float c = p.c;

    // The R rows of this (batch, K/V head): row r is position r % Sq of query head hk*g + r / Sq.
    const unsigned char* qg = (const unsigned char*)p.q + b * p.q_bs + (long long)(hk * g) * p.q_hs;
    const unsigned char* kg = (const unsigned char*)p.k + b * p.k_bs + hk * p.k_hs;
    const unsigned char* vg = (const unsigned char*)p.v + b * p.v_bs + hk * p.v_hs;

    const int row = chunk * DEC_ROWS + l32;                 // the query row this lane owns
    const int row_ld = row < p.R ? row : p.R - 1;
    // last key this row may see: the Sq queries are the last positions of a sequence of Sk
    const int lim = p.causal ? Sk - p.Sq + (row_ld % p.Sq) : Sk - 1;

    i32x4_t qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        qf[ks] = ks * 2 + h < p.cpr
                     ? *(const i32x4_t*)(qg + (row_ld / p.Sq) * p.q_hs + (long long)(row_ld % p.Sq) * p.q_rs + ks * 32 + h * 16)
                     : i32x4_t{0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        asm volatile("" : "+v"(qf[ks]));

    // Direct global->LDS loads: instruction n fills physical chunks 64n..64n+63 of the block, lane i
    // the chunk 64n+i, so the lane fetches the logical chunk that the swizzle maps there.
    // (row of the block, byte inside the row) of that logical chunk:
    int k_row[NLD], k_col[NLD], v_row[NLD], v_col[NLD];
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
        const int P = n * 64 + lane;
        {
            const int line = P >> 4, pos = P & 15;
            const int key = D > 128 ? line >> 1 : line;                // the inverse of k_off
            const int off = ((line << 4) + (pos ^ (key & 15))) * 16;   // byte offset in a dense [32][D] block
            k_row[n] = off / ROWB;
            const int kc = off % ROWB / 16;
            k_col[n] = (kc < p.cpr ? kc : p.cpr - 1) * 16;
        }
        if constexpr (D >= 128) {
            const int r = P / (D / 8), cc = P % (D / 8);
            const int vc = cc ^ ((r & 3) << 2);
            v_row[n] = r;
            v_col[n] = (vc < p.cpr ? vc : p.cpr - 1) * 16;
        } else {
            const int r = P >> 3, cc = P & 7;
            const int vc = cc ^ (((r >> 1) & 1) << 2);
            v_row[n] = r;
            v_col[n] = (vc < p.cpr ? vc : p.cpr - 1) * 16;
        }
    }
    const unsigned lds0 = (unsigned)(uintptr_t)(NAUT_LDS unsigned char*)smem + (unsigned)(wave * 4 * BLKB);
    unsigned char* my_lds = smem + wave * 4 * BLKB;

    const int nblk = (Sk + DEC_BLK - 1) / DEC_BLK;
    const int blk_begin = split * p.bps;
    const int blk_end = blk_begin + p.bps < nblk ? blk_begin + p.bps : nblk;

    auto issue = [&](int blk, int buf) {
        const unsigned char* kp = kg + (size_t)blk * DEC_BLK * p.k_rs;
        const unsigned char* vp = vg + (size_t)blk * DEC_BLK * p.v_rs;
        const int rows_left = Sk - blk * DEC_BLK;  // >= 1
        const unsigned dst = lds0 + (unsigned)(buf * 2 * BLKB);
#pragma unroll
        for (int n = 0; n < NLD; ++n) {
            int kr = k_row[n], vr = v_row[n];
            if (rows_left < DEC_BLK) {  // ragged last block: re-read the last row instead of running past the end
                kr = kr < rows_left ? kr : rows_left - 1;
                vr = vr < rows_left ? vr : rows_left - 1;
            }
            const int ko = kr * p.k_rs + k_col[n], vo = vr * p.v_rs + v_col[n];
            load_to_lds(dst + n * 1024, ko, kp);
            load_to_lds(dst + BLKB + n * 1024, vo, vp);
        }
    };

    f32x16_t oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            oacc[db][r] = 0.f;
    float m_run = DEC_M_INIT;  // reference maximum, log2 units (already times c)
    float l_run = 0.f;         // this lane's share of the running sum (its 16 of every 32 keys)

    // This wavefront's blocks: blk_begin + wave, + NW, ...  Block n+1 is in flight while block n is used.
    static_assert(2 * NLD < 64, "vmcnt field");
    int blk = blk_begin + wave;
    if (blk < blk_end)
        issue(blk, 0);
    for (int it = 0; blk < blk_end; blk += NW, ++it) {
        const int buf = it & 1;
        const bool more = blk + NW < blk_end;
        if (more) {
            issue(blk + NW, buf ^ 1);
            wait_loads<2 * NLD>();
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        const unsigned char* kt = my_lds + buf * 2 * BLKB;
        const unsigned char* vt = kt + BLKB;

        f32x16_t s_;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s_[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const i32x4_t kf = *(const i32x4_t*)(kt + k_off<D>(l32, ks * 2 + h));
            s_ = T::mfma(kf, qf[ks], s_);
        }
        const int key0 = blk * DEC_BLK;
        if (key0 + DEC_BLK - 1 > Sk - p.Sq || key0 + DEC_BLK > Sk) {  // some row's limit may fall inside the block
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + 8 * (r >> 2) + 4 * h + (r & 3);
                s_[r] = key > lim ? -INFINITY : s_[r];
            }
        }
        float mx = s_[0];
#pragma unroll
        for (int r = 1; r < 16; ++r)
            mx = fmaxf(mx, s_[r]);
        mx = half_max(mx);
        const float m_cand = mx * c;  // -inf if the whole block is masked for this row
        if (__builtin_amdgcn_ballot_w64(m_cand > m_run + DEC_TAU) != 0) {
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
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s_[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_[r], c, -m_run));
            psum = r == 0 ? s_[r] : psum + s_[r];
        }
        l_run += psum;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int r0 = t * 8;
            const i32x4_t pb = {T::pack2(s_[r0 + 0], s_[r0 + 1]), T::pack2(s_[r0 + 2], s_[r0 + 3]),
                                T::pack2(s_[r0 + 4], s_[r0 + 5]), T::pack2(s_[r0 + 6], s_[r0 + 7])};
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const i32x4_t vf = load_vt_frag<D>(vt, t * 16, db, lane);
                oacc[db] = T::mfma(vf, pb, oacc[db]);
            }
        }
    }

    merge_wavefronts<D, 4 * BLKB, NW>(smem, oacc, m_run, l_run, p, bhk, chunk, split);
}

// The same split kernel on FP8 (E4M3) Q, K and V: 64-key blocks (one 32x32x64 MFMA covers 64 keys of
// P.V), the LDS layouts, transposed byte reads and the 2^7 scaling of P of the FP8 prefill kernel, the
// blocks dealt to the wavefronts and double-buffered in LDS exactly as above; strides and narrower heads
// as above too, in 16-byte chunks of 16 values (p.cpr counts 8 values: two per chunk here).
// bps counts 64-key blocks here.  The partial's reference maximum is stored as m - 7, which makes its l
// and O (both carry the factor 2^7) relative to it in the plain sense the merge kernel expects.
constexpr int DEC8_BLK = 64;
constexpr float DEC8_TAU = 1.0f;      // P * 2^7 <= 2^(1+7) = 256 < 448, the largest E4M3 value
constexpr float DEC8_P_SHIFT = 7.0f;

template <int D>
__global__ __launch_bounds__(DEC_THREADS, 1) void naut_decode_split_fp8_kernel(const DecodeParams p)
{
    constexpr int BLKB = DEC8_BLK * D;     // bytes of one 64-key block of K or V
    constexpr int KS = D / 64;
    constexpr int DB = D / 32;
    constexpr int CPR = D / 16;            // 16-byte chunks per row
    constexpr int NLD = BLKB / 1024;       // direct loads (1 KB each) per block and operand

    __shared__ __attribute__((aligned(1024))) unsigned char smem[DEC_WAVES * 4 * BLKB];  // per wavefront: K0 V0 K1 V1

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    const int split = blockIdx.x, chunk = blockIdx.y, bhk = blockIdx.z;
    const int b = bhk / p.Hkv, hk = bhk % p.Hkv;
    const int g = p.Hq / p.Hkv;
    const int Sk = p.Sk;
    const float c = p.c;

    // The R rows of this (batch, K/V head): row r is position r % Sq of query head hk*g + r / Sq.
    const unsigned char* qg = (const unsigned char*)p.q + b * p.q_bs + (long long)(hk * g) * p.q_hs;
    const unsigned char* kg = (const unsigned char*)p.k + b * p.k_bs + hk * p.k_hs;
    const unsigned char* vg = (const unsigned char*)p.v + b * p.v_bs + hk * p.v_hs;
    const int cpr16 = p.cpr >> 1;  // real 16-byte chunks per row

    const int row = chunk * DEC_ROWS + l32;                 // the query row this lane owns
    const int row_ld = row < p.R ? row : p.R - 1;
    const int lim = p.causal ? Sk - p.Sq + (row_ld % p.Sq) : Sk - 1;  // last key this row may see

    // Q^T fragments (MFMA B operand): lane holds q[row][64*ks + 32*h .. +32]
    i32x8_t qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const unsigned char* qrow = qg + (row_ld / p.Sq) * p.q_hs + (long long)(row_ld % p.Sq) * p.q_rs;
        const int c0 = ks * 4 + h * 2;  // this lane's two 16-byte chunks of the row
        const i32x4_t lo = c0 < cpr16 ? *(const i32x4_t*)(qrow + c0 * 16) : i32x4_t{0, 0, 0, 0};
        const i32x4_t hi = c0 + 1 < cpr16 ? *(const i32x4_t*)(qrow + c0 * 16 + 16) : i32x4_t{0, 0, 0, 0};
        qf[ks] = i32x8_t{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        asm volatile("" : "+v"(qf[ks]));

    // Direct global->LDS loads: instruction n fills physical 16-byte chunks 64n..64n+63 of the block, lane i
    // the chunk 64n+i, so the lane fetches the logical chunk that k8_off / v8_off place there.
    int k_row[NLD], k_col[NLD], v_row[NLD], v_col[NLD];
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
        const int P = n * 64 + lane;
        const int r = P / CPR, pc = P % CPR;
        k_row[n] = r;
        const int kc = pc ^ ((r >> 1) & (CPR - 1));  // logical chunk that k8_off places at position pc
        k_col[n] = (kc < cpr16 ? kc : cpr16 - 1) * 16;
        const int key = D == 128 ? (((r >> 1) & 1) | (((r >> 3) & 1) << 1)) : ((r >> 3) & 1);
        v_row[n] = r;
        const int vc = (((pc >> 1) ^ key) << 1) + (pc & 1);  // likewise for v8_off (32-byte chunks, two halves)
        v_col[n] = (vc < cpr16 ? vc : cpr16 - 1) * 16;
    }
    const unsigned lds0 = (unsigned)(uintptr_t)(NAUT_LDS unsigned char*)smem + (unsigned)(wave * 4 * BLKB);
    unsigned char* my_lds = smem + wave * 4 * BLKB;

    const int nblk = (Sk + DEC8_BLK - 1) / DEC8_BLK;
    const int blk_begin = split * p.bps;
    const int blk_end = blk_begin + p.bps < nblk ? blk_begin + p.bps : nblk;

    auto issue = [&](int blk, int buf) {
        const unsigned char* kp = kg + (size_t)blk * DEC8_BLK * p.k_rs;
        const unsigned char* vp = vg + (size_t)blk * DEC8_BLK * p.v_rs;
        const int rows_left = Sk - blk * DEC8_BLK;  // >= 1
        const unsigned dst = lds0 + (unsigned)(buf * 2 * BLKB);
#pragma unroll
        for (int n = 0; n < NLD; ++n) {
            int kr = k_row[n], vr = v_row[n];
            if (rows_left < DEC8_BLK) {  // ragged last block: re-read the last row instead of running past the end
                kr = kr < rows_left ? kr : rows_left - 1;
                vr = vr < rows_left ? vr : rows_left - 1;
            }
            const int ko = kr * p.k_rs + k_col[n], vo = vr * p.v_rs + v_col[n];
            load_to_lds(dst + n * 1024, ko, kp);
            load_to_lds(dst + BLKB + n * 1024, vo, vp);
        }
    };

    // lane-constant parts of the transposed V reads (as in the FP8 prefill kernel)
    const int i16 = lane & 15;
    const int v_e = i16 >> 1;
    const int v_key = 4 * h + (v_e & 3) + ((v_e >> 2) << 3);
    const int v_byte = 16 * ((lane >> 4) & 1) + 8 * (i16 & 1);

    f32x16_t oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            oacc[db][r] = 0.f;
    float m_run = DEC_M_INIT;
    float l_run = 0.f;
    i32x8_t pb = {0, 0, 0, 0, 0, 0, 0, 0};

    static_assert(2 * NLD < 64, "vmcnt field");
    int blk = blk_begin + wave;
    if (blk < blk_end)
        issue(blk, 0);
    for (int it = 0; blk < blk_end; blk += DEC_WAVES, ++it) {
        const int buf = it & 1;
        const bool more = blk + DEC_WAVES < blk_end;
        if (more) {
            issue(blk + DEC_WAVES, buf ^ 1);
            wait_loads<2 * NLD>();
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        const unsigned char* kt = my_lds + buf * 2 * BLKB;
        const unsigned char* vt = kt + BLKB;

        f32x16_t sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                sacc[kb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int rw = kb * 32 + l32, c0 = ks * 4 + h * 2;
                const i32x4_t lo = *(const i32x4_t*)(kt + k8_off<D>(rw, c0));
                const i32x4_t hi = *(const i32x4_t*)(kt + k8_off<D>(rw, c0 + 1));
                const i32x8_t kf = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                sacc[kb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf, qf[ks], sacc[kb], 0, 0, 0, 0, 0, 0);
            }
        }
        const int key0 = blk * DEC8_BLK;
        if (key0 + DEC8_BLK - 1 > Sk - p.Sq || key0 + DEC8_BLK > Sk) {  // some row's limit may fall inside the block
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    sacc[kb][r] = key > lim ? -INFINITY : sacc[kb][r];
                }
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                mx = fmaxf(mx, sacc[kb][r]);
        mx = half_max(mx);
        const float m_cand = mx * c;  // -inf if the whole block is masked for this row
        if (__builtin_amdgcn_ballot_w64(m_cand > m_run + DEC8_TAU) != 0) {
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
        const float shift = DEC8_P_SHIFT - m_run;
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
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const int kb = w >> 2, r0 = (w & 3) * 4;
            pb[w] = pack4_fp8(sacc[kb][r0 + 0], sacc[kb][r0 + 1], sacc[kb][r0 + 2], sacc[kb][r0 + 3], pb[w]);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            i32x8_t vf;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int key = 32 * (t >> 1) + 16 * (t & 1) + v_key;
                const i32x2_t x = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                    (NAUT_LDS i32x2_t*)(vt + v8_off<D>(key, db) + v_byte));
                vf[2 * t] = x.x;
                vf[2 * t + 1] = x.y;
            }
            oacc[db] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf, pb, oacc[db], 0, 0, 0, 0, 0, 0);
        }
    }
    merge_wavefronts<D, 4 * BLKB, DEC_WAVES>(smem, oacc, m_run - DEC8_P_SHIFT, l_run, p, bhk, chunk, split);
}

// One work-group (four wavefronts) per query row: merges the nsplit partials of the row, divides by l
// once, stores O and lse.  Wavefront w takes splits w, w+4, ...; lanes run over D.
template <int D, int DT_OUT>
__global__ __launch_bounds__(MRG_THREADS) void naut_decode_merge_kernel(const DecodeParams p)
{
    __shared__ float red_m[MRG_WAVES];
    __shared__ float red_l[MRG_WAVES];
    __shared__ float red_o[MRG_WAVES][D];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = blockIdx.x;    // row inside the (batch, K/V head): 0 .. R-1
    const int bhk = blockIdx.y;
    const int chunk = r / DEC_ROWS, rr = r % DEC_ROWS;
    const size_t nparts = (size_t)p.B * p.Hkv * p.nchunks * p.nsplit;
    const size_t part0 = ((size_t)bhk * p.nchunks + chunk) * p.nsplit;
    const float* ws_m = p.ws + nparts * DEC_ROWS * D + part0 * DEC_ROWS + rr;   // stride DEC_ROWS per split
    const float* ws_l = ws_m + nparts * DEC_ROWS;
    const float* ws_o = p.ws + (part0 * DEC_ROWS + rr) * D;                      // stride DEC_ROWS*D per split

    // pass 1: the maximum over all splits (every thread takes a strided share, then LDS)
    float M = DEC_M_INIT;
    for (int s = tid; s < p.nsplit; s += MRG_THREADS)
        M = fmaxf(M, ws_m[(size_t)s * DEC_ROWS]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        M = fmaxf(M, __shfl_xor(M, off));
    if (lane == 0)
        red_m[wave] = M;
    __syncthreads();
    M = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));

    // pass 2: weighted sums
    constexpr int EPT = D / 64;  // elements per lane
    float acc[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e)
        acc[e] = 0.f;
    float L = 0.f;
#pragma unroll 4
    for (int s = wave; s < p.nsplit; s += MRG_WAVES) {
        const float f = __builtin_amdgcn_exp2f(ws_m[(size_t)s * DEC_ROWS] - M);
        L += f * ws_l[(size_t)s * DEC_ROWS];
        const float* po = ws_o + (size_t)s * DEC_ROWS * D + lane * EPT;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            acc[e] += f * po[e];
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e)
        red_o[wave][lane * EPT + e] = acc[e];
    if (lane == 0)
        red_l[wave] = L;
    __syncthreads();
    if (wave != 0)
        return;
    L = red_l[0] + red_l[1] + red_l[2] + red_l[3];
#pragma unroll
    for (int e = 0; e < EPT; ++e)
        acc[e] = red_o[0][lane * EPT + e] + red_o[1][lane * EPT + e] + red_o[2][lane * EPT + e] + red_o[3][lane * EPT + e];
    const float inv_l = p.dv / L;
    // lse is dense [B][Hq][Sq]: the R rows of (batch, K/V head) bhk are contiguous there
    if (p.lse != nullptr && lane == 0)
        p.lse[(size_t)bhk * p.R + r] = (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f;
    const int b = bhk / p.Hkv, hk = bhk % p.Hkv;
    const int head = hk * (p.Hq / p.Hkv) + r / p.Sq, pos = r % p.Sq;
    unsigned char* orow = (unsigned char*)p.o + b * p.o_bs + head * p.o_hs + (long long)pos * p.o_rs;
    if (lane * EPT >= p.cpr * 8)
        return;  // padding columns of a narrower head dimension
    if constexpr (DT_OUT == NAUT_F32) {
        float* og = (float*)orow + lane * EPT;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            og[e] = acc[e] * inv_l;
    } else if constexpr (EPT == 4) {
        i32x2_t* og = (i32x2_t*)(orow + lane * EPT * 2);
        *og = i32x2_t{In<DT_OUT>::pack2(acc[0] * inv_l, acc[1] * inv_l), In<DT_OUT>::pack2(acc[2] * inv_l, acc[3] * inv_l)};
    } else if constexpr (EPT == 2) {
        int* og = (int*)(orow + lane * EPT * 2);
        *og = In<DT_OUT>::pack2(acc[0] * inv_l, acc[1] * inv_l);
    } else {
        unsigned short* og = (unsigned short*)orow + lane;
        *og = (unsigned short)(In<DT_OUT>::pack2(acc[0] * inv_l, 0.f) & 0xffff);
    }
}

struct Plan {
    int nchunks, nsplit, bps;
    size_t ws_bytes;
};

// Scratch of naut_attn_decode_static: the split partials live in this file-scope device array instead of a
// caller-provided workspace.  Every GPU the library runs on holds its own copy at its own address for the
// life of the process.  In host code the array's name is only a handle for hipGetSymbolAddress: the device
// address it returns (taken once per device, with that device current) is what kernels and copies get.
constexpr size_t DEC_STATIC_BYTES = 16u << 20;
static __device__ __align__(256) unsigned char scratch[DEC_STATIC_BYTES];
constexpr int DEC_MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[DEC_MAX_DEVICES];

// Device address of `scratch` on the current device (NULL and an error message on failure).
void* static_scratch(int* err)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        *err = fail_launch(e);
        return nullptr;
    }
    if (dev < 0 || dev >= DEC_MAX_DEVICES) {
        *err = fail(NAUT_ERR_UNSUPPORTED, "device ordinal beyond the library's per-device table");
        return nullptr;
    }
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            snprintf(g_err, sizeof g_err, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
            *err = NAUT_ERR_HIP;
            return nullptr;
        }
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // every thread computes the same value
    }
    return ptr;
}

// D: the width the kernels are compiled for (64, 128 or 256)
bool make_plan(int B, int Hq, int Hkv, int Sq, int Sk, int D, Plan* pl)
{
    const int W = dec_waves(D);
    const long long R = (long long)(Hq / Hkv) * Sq;
    const long long nchunks = (R + DEC_ROWS - 1) / DEC_ROWS;
    const long long nblk = ((long long)Sk + DEC_BLK - 1) / DEC_BLK;
    const long long base = (long long)B * Hkv * nchunks;
    long long nsplit = (DEC_TARGET_WGS + base - 1) / base;
    const long long max_split = (nblk + 2 * W - 1) / (2 * W);  // at least two blocks per wavefront
    nsplit = nsplit > max_split ? max_split : nsplit;
    nsplit = nsplit < 1 ? 1 : nsplit;
    long long bps = (nblk + nsplit - 1) / nsplit;
    bps = (bps + W - 1) / W * W;
    nsplit = (nblk + bps - 1) / bps;
    if (nchunks > 65535 || (long long)B * Hkv > 65535 || nsplit > 0x7fffffffLL || R > 0x7fffffffLL)
        return false;
    pl->nchunks = (int)nchunks;
    pl->nsplit = (int)nsplit;
    pl->bps = (int)bps;
    pl->ws_bytes = (size_t)(base * nsplit) * DEC_ROWS * (D + 2) * sizeof(float);
    return true;
}

template <int D, int DT_IN, int DT_OUT>
int launch_decode(const DecodeParams& p, hipStream_t stream)
{
    const dim3 g1((unsigned)p.nsplit, (unsigned)p.nchunks, (unsigned)(p.B * p.Hkv));
    hipLaunchKernelGGL((naut_decode_split_kernel<D, DT_IN>), g1, dim3(dec_waves(D) * 64), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_launch(e);
    const dim3 g2((unsigned)p.R, (unsigned)(p.B * p.Hkv));
    hipLaunchKernelGGL((naut_decode_merge_kernel<D, DT_OUT>), g2, dim3(MRG_THREADS), 0, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess)
        return fail_launch(e);
    return NAUT_OK;
}

}  // namespace

extern "C" {

size_t naut_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int Sq, int Sk, int D)
{
    Plan pl;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Sk <= 0 || Hq % Hkv != 0 || D <= 0 || D % 8 != 0 || D > 256 ||
        !make_plan(B, Hq, Hkv, Sq, Sk, D <= 64 ? 64 : D <= 128 ? 128 : 256, &pl))
        return 0;
    return pl.ws_bytes;
}

}  // extern "C"

namespace {

// The 16-bit decode path behind naut_attn_decode[_dt|_strided] and naut_attn_decode_static.  With
// `use_static` the split partials go to the library's static device array instead of `workspace`; its
// address is taken only after every argument check has passed (no HIP call before that).
int decode_16bit(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                 int Sq, int Sk, int D, int causal, float scale, void* workspace, size_t workspace_bytes,
                 bool use_static, void* stream, int in_dtype, int out_dtype, const naut_strides* st)
{
    if (!q || !k || !v || !o)
        return fail(NAUT_ERR_NULL, "q, k, v and o must be non-NULL device pointers");
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Sk <= 0 || D <= 0)
        return fail(NAUT_ERR_SHAPE, "B, Hq, Hkv, Sq, Sk and D must be positive");
    if (Hq % Hkv != 0)
        return fail(NAUT_ERR_SHAPE, "Hq must be a multiple of Hkv");
    if (causal && Sk < Sq)
        return fail(NAUT_ERR_SHAPE, "with the causal mask the Sq queries are the last positions of Sk: Sk >= Sq");
    if (!std::isfinite(scale))
        return fail(NAUT_ERR_SHAPE, "scale must be finite");
    if (scale < 0.f)
        return fail(NAUT_ERR_UNSUPPORTED, "negative scale is not supported");
    if (D % 8 != 0 || D > 256)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be a multiple of 8, at most 256");
    const int DK = D <= 64 ? 64 : D <= 128 ? 128 : 256;  // width the kernels are compiled for
    if ((in_dtype != NAUT_BF16 && in_dtype != NAUT_F16) || (out_dtype != in_dtype && out_dtype != NAUT_F32))
        return fail(NAUT_ERR_UNSUPPORTED, "supported dtypes: q/k/v bf16 or f16; o of the same type or f32");
    Plan pl;
    if (!make_plan(B, Hq, Hkv, Sq, Sk, DK, &pl))
        return fail(NAUT_ERR_UNSUPPORTED, "shape exceeds the grid limits");
    if (use_static)
        workspace = nullptr;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o | (uintptr_t)workspace) & 15)
        return fail(NAUT_ERR_ALIGN, "q, k, v, o and workspace must be 16-byte aligned");
    if ((uintptr_t)lse & 3)
        return fail(NAUT_ERR_ALIGN, "lse must be 4-byte aligned");
    if (use_static) {
        if (pl.ws_bytes > DEC_STATIC_BYTES) {
            snprintf(g_err, sizeof g_err,
                     "these sizes need %zu bytes of split partials, more than the %zu-byte static scratch of "
                     "naut_attn_decode_static: use naut_attn_decode with a workspace",
                     pl.ws_bytes, DEC_STATIC_BYTES);
            return NAUT_ERR_UNSUPPORTED;
        }
    } else {
        if (!workspace)
            return fail(NAUT_ERR_NULL, "workspace must be a non-NULL device pointer");
        if (workspace_bytes < pl.ws_bytes)
            return fail(NAUT_ERR_SHAPE, "workspace is smaller than naut_attn_decode_workspace_bytes()");
    }

    naut_strides cs;  // contiguous q, o [B][Hq][Sq][D] and k, v [B][Hkv][Sk][D]
    cs.q_s = cs.k_s = cs.v_s = cs.o_s = D;
    cs.q_h = cs.o_h = (long long)Sq * D;
    cs.k_h = cs.v_h = (long long)Sk * D;
    cs.q_b = cs.o_b = (long long)Hq * Sq * D;
    cs.k_b = cs.v_b = (long long)Hkv * Sk * D;
    if (!st)
        st = &cs;
    const long long in_strides[9] = {st->q_b, st->q_h, st->q_s, st->k_b, st->k_h, st->k_s, st->v_b, st->v_h, st->v_s};
    for (long long x : in_strides)
        if (x < 0 || x % 8 != 0)
            return fail(NAUT_ERR_ALIGN, "q/k/v strides must be non-negative multiples of 8 elements (16 bytes)");
    if (st->o_b <= 0 || st->o_h <= 0 || st->o_s <= 0 || st->o_b % 4 != 0 || st->o_h % 4 != 0 || st->o_s % 4 != 0)
        return fail(NAUT_ERR_ALIGN, "o strides must be positive multiples of 4 elements");
    if (st->q_s < D || st->k_s < D || st->v_s < D || st->o_s < D)
        return fail(NAUT_ERR_SHAPE, "a sequence stride is smaller than D: rows would overlap");
    const long long max_rs = 1LL << 23;  // elements: keeps 32 rows of byte offsets inside 32 bits
    if (st->q_s > max_rs || st->k_s > max_rs || st->v_s > max_rs || st->o_s > max_rs)
        return fail(NAUT_ERR_UNSUPPORTED, "sequence stride too large");
    const int out_b = out_dtype == NAUT_F32 ? 4 : 2;

    if (use_static) {  // every host-side check has passed: the first HIP calls of this path
        int err = NAUT_OK;
        workspace = static_scratch(&err);
        if (workspace == nullptr)
            return err;
    }
    DecodeParams p;
    p.q = q;
    p.k = k;
    p.v = v;
    p.o = o;
    p.lse = lse;
    p.ws = (float*)workspace;
    p.B = B;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.Sq = Sq;
    p.Sk = Sk;
    p.R = Hq / Hkv * Sq;
    p.nchunks = pl.nchunks;
    p.nsplit = pl.nsplit;
    p.bps = pl.bps;
    p.causal = causal ? 1 : 0;
    const float cc = scale * 1.4426950408889634f;
    p.c = cc > 0.f ? cc : 1.0e-30f;  // scale == 0: every score becomes (almost exactly) 0, the softmax uniform
    p.dv = 1.0f;
    p.q_bs = st->q_b * 2;
    p.q_hs = st->q_h * 2;
    p.q_rs = (int)(st->q_s * 2);
    p.k_bs = st->k_b * 2;
    p.k_hs = st->k_h * 2;
    p.k_rs = (int)(st->k_s * 2);
    p.v_bs = st->v_b * 2;
    p.v_hs = st->v_h * 2;
    p.v_rs = (int)(st->v_s * 2);
    p.o_bs = st->o_b * out_b;
    p.o_hs = st->o_h * out_b;
    p.o_rs = (int)(st->o_s * out_b);
    p.cpr = D / 8;
    hipStream_t hs = (hipStream_t)stream;
#define NAUT_DEC(DD, IN, OUT)                                  \
    if (DK == DD && in_dtype == IN && out_dtype == OUT)        \
        return launch_decode<DD, IN, OUT>(p, hs);
    NAUT_DEC(256, NAUT_BF16, NAUT_BF16)
    NAUT_DEC(256, NAUT_BF16, NAUT_F32)
    NAUT_DEC(256, NAUT_F16, NAUT_F16)
    NAUT_DEC(256, NAUT_F16, NAUT_F32)
    NAUT_DEC(128, NAUT_BF16, NAUT_BF16)
    NAUT_DEC(128, NAUT_BF16, NAUT_F32)
    NAUT_DEC(128, NAUT_F16, NAUT_F16)
    NAUT_DEC(128, NAUT_F16, NAUT_F32)
    NAUT_DEC(64, NAUT_BF16, NAUT_BF16)
    NAUT_DEC(64, NAUT_BF16, NAUT_F32)
    NAUT_DEC(64, NAUT_F16, NAUT_F16)
    NAUT_DEC(64, NAUT_F16, NAUT_F32)
#undef NAUT_DEC
    return fail(NAUT_ERR_UNSUPPORTED, "no kernel for this (D, dtype) combination");
}

}  // namespace

extern "C" {

int naut_attn_decode_strided(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                             int Sq, int Sk, int D, int causal, float scale, void* workspace, size_t workspace_bytes,
                             void* stream, int in_dtype, int out_dtype, const naut_strides* st)
{
    return decode_16bit(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, causal, scale, workspace, workspace_bytes, false, stream,
                        in_dtype, out_dtype, st);
}

int naut_attn_decode_fp8_strided(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq,
                                 int Hkv, int Sq, int Sk, int D, int causal, float scale, float descale_q,
                                 float descale_k, float descale_v, void* workspace, size_t workspace_bytes, void* stream,
                                 const naut_strides* st)
{
    if (!q || !k || !v || !o)
        return fail(NAUT_ERR_NULL, "q, k, v and o must be non-NULL device pointers");
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Sk <= 0 || D <= 0)
        return fail(NAUT_ERR_SHAPE, "B, Hq, Hkv, Sq, Sk and D must be positive");
    if (Hq % Hkv != 0)
        return fail(NAUT_ERR_SHAPE, "Hq must be a multiple of Hkv");
    if (causal && Sk < Sq)
        return fail(NAUT_ERR_SHAPE, "with the causal mask the Sq queries are the last positions of Sk: Sk >= Sq");
    if (!std::isfinite(scale) || !std::isfinite(descale_q) || !std::isfinite(descale_k) || !std::isfinite(descale_v))
        return fail(NAUT_ERR_SHAPE, "scale and the three descale factors must be finite");
    if (scale < 0.f || descale_q <= 0.f || descale_k <= 0.f || descale_v <= 0.f)
        return fail(NAUT_ERR_UNSUPPORTED, "scale must be >= 0 and the descale factors > 0");
    if (D % 16 != 0 || D > 128)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be a multiple of 16, at most 128");
    const int DK = D <= 64 ? 64 : 128;  // width the kernels are compiled for
    Plan pl;  // over 64-key blocks: the plan of a cache half as long in 32-key blocks
    if (!make_plan(B, Hq, Hkv, Sq, (Sk + 1) / 2, DK, &pl))
        return fail(NAUT_ERR_UNSUPPORTED, "shape exceeds the grid limits");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o | (uintptr_t)workspace) & 15)
        return fail(NAUT_ERR_ALIGN, "q, k, v, o and workspace must be 16-byte aligned");
    if ((uintptr_t)lse & 3)
        return fail(NAUT_ERR_ALIGN, "lse must be 4-byte aligned");
    if (!workspace)
        return fail(NAUT_ERR_NULL, "workspace must be a non-NULL device pointer");
    if (workspace_bytes < pl.ws_bytes)
        return fail(NAUT_ERR_SHAPE, "workspace is smaller than naut_attn_decode_workspace_bytes()");

    naut_strides cs;  // contiguous q, o [B][Hq][Sq][D] and k, v [B][Hkv][Sk][D]
    cs.q_s = cs.k_s = cs.v_s = cs.o_s = D;
    cs.q_h = cs.o_h = (long long)Sq * D;
    cs.k_h = cs.v_h = (long long)Sk * D;
    cs.q_b = cs.o_b = (long long)Hq * Sq * D;
    cs.k_b = cs.v_b = (long long)Hkv * Sk * D;
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

    DecodeParams p;
    p.q = q;
    p.k = k;
    p.v = v;
    p.o = o;
    p.lse = lse;
    p.ws = (float*)workspace;
    p.B = B;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.Sq = Sq;
    p.Sk = Sk;
    p.R = Hq / Hkv * Sq;
    p.nchunks = pl.nchunks;
    p.nsplit = pl.nsplit;
    p.bps = pl.bps;
    p.causal = causal ? 1 : 0;
    const float cc = scale * descale_q * descale_k * 1.4426950408889634f;
    p.c = cc > 0.f ? cc : 1.0e-30f;
    p.dv = descale_v;
    // q, k, v: one byte per element; o: bf16
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
    p.cpr = D / 8;
    hipStream_t hs = (hipStream_t)stream;
    const dim3 g1((unsigned)p.nsplit, (unsigned)p.nchunks, (unsigned)(p.B * p.Hkv));
    const dim3 g2((unsigned)p.R, (unsigned)(p.B * p.Hkv));
    if (DK == 128) {
        hipLaunchKernelGGL((naut_decode_split_fp8_kernel<128>), g1, dim3(DEC_THREADS), 0, hs, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return fail_launch(e);
        hipLaunchKernelGGL((naut_decode_merge_kernel<128, NAUT_BF16>), g2, dim3(MRG_THREADS), 0, hs, p);
    } else {
        hipLaunchKernelGGL((naut_decode_split_fp8_kernel<64>), g1, dim3(DEC_THREADS), 0, hs, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return fail_launch(e);
        hipLaunchKernelGGL((naut_decode_merge_kernel<64, NAUT_BF16>), g2, dim3(MRG_THREADS), 0, hs, p);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_launch(e);
    return NAUT_OK;
}

int naut_attn_decode_fp8(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                         int Sq, int Sk, int D, int causal, float scale, float descale_q, float descale_k,
                         float descale_v, void* workspace, size_t workspace_bytes, void* stream)
{
    if (D > 0 && D != 64 && D != 128)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be 64 or 128 (naut_attn_decode_fp8_strided takes other head dimensions)");
    return naut_attn_decode_fp8_strided(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, causal, scale, descale_q, descale_k,
                                        descale_v, workspace, workspace_bytes, stream, nullptr);
}

int naut_attn_decode_static(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                              int Sq, int Sk, int D, int causal, float scale, void* stream)
{
    if (D > 0 && D != 64 && D != 128)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be 64 or 128");
    return decode_16bit(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, causal, scale, nullptr, 0, true, stream, NAUT_BF16,
                        NAUT_BF16, nullptr);
}

int naut_attn_decode_dt(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                        int Sq, int Sk, int D, int causal, float scale, void* workspace, size_t workspace_bytes,
                        void* stream, int in_dtype, int out_dtype)
{
    if (D > 0 && D != 64 && D != 128)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be 64 or 128 (naut_attn_decode_strided takes other head dimensions)");
    return naut_attn_decode_strided(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, causal, scale, workspace, workspace_bytes,
                                    stream, in_dtype, out_dtype, nullptr);
}

int naut_attn_decode(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int Sq,
                     int Sk, int D, int causal, float scale, void* workspace, size_t workspace_bytes, void* stream)
{
    return naut_attn_decode_dt(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, causal, scale, workspace, workspace_bytes, stream,
                               NAUT_BF16, NAUT_BF16);
}

}  // extern "C"
