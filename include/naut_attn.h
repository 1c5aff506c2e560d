/*
 * naut_attn.h -- C ABI of the fused attention forward for AMD MI355X (gfx950).
 *
 * The operation is the one the paper's auto-scheduler exists to speed up
 * (Section 1: attention given as two matrix products around a softmax; operator table of
 * Section 6: Global, Causal and Grouped-Query attention): for every batch b,
 * query head h and query position i
 *
 *     s_ij = scale * sum_d q[b,h,i,d] * k[b,hk,j,d]            j in J_i
 *     P_ij = exp(s_ij - m_i) / l_i,  m_i = max_j s_ij,  l_i = sum_j exp(s_ij - m_i)
 *     o[b,h,i,:] = sum_j P_ij * v[b,hk,j,:]
 *     lse[b,h,i] = m_i + ln l_i                                 (natural log)
 *
 * with J_i = {0..S-1}, or {0..i} when `causal` is non-zero (the diagonal is
 * kept), and hk = h / (Hq/Hkv): consecutive query heads share a key/value head.
 * It is computed in ONE kernel: the reductions over j are fused with the
 * rolling-update ("online") scheme of Section 4.2/4.3, so the S x S score
 * matrix never reaches memory; the running maximum introduces the repair factor
 * exp(m_old - m_new).  The three rewrites of the expression-rewriting table of
 * Section 5 are applied by hand: `scale` is hoisted out of the loop into one
 * constant, the per-step division by l is replaced by one division at the end,
 * and exp(x) is evaluated as exp2(log2(e) * x).
 *
 * Memory: every pointer is DEVICE memory owned by the caller, contiguous and
 * row-major with D innermost:
 *     q, o : [B][Hq][S][D]      k, v : [B][Hkv][S][D]      lse : [B][Hq][S] (fp32)
 * q/k/v/o must be 16-byte aligned, lse 4-byte aligned.  `lse` may be NULL (not
 * written then).  The library allocates nothing, keeps no state between calls
 * and never frees.  `stream` is a hipStream_t passed as void* (NULL = the
 * default stream).  Calls are asynchronous: work is enqueued on `stream` and the
 * call returns without synchronising.
 *
 * Errors: every argument is validated on the host before any HIP call; a
 * negative naut_status is returned and naut_last_error_string() explains it.
 * Nothing aborts or throws across this boundary.
 */
#ifndef NAUT_ATTN_H
#define NAUT_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NAUT_OK = 0,
    NAUT_ERR_NULL = -1,        /* q, k, v, o or a required workspace is NULL */
    NAUT_ERR_SHAPE = -2,       /* a size <= 0, Hq % Hkv != 0, scale not finite, rows that overlap, workspace too small */
    NAUT_ERR_UNSUPPORTED = -3, /* a head dimension the entry point does not take (each one states its set), unknown
                                  dtype pair, scale < 0, sizes or strides beyond the 32-bit limits of a kernel */
    NAUT_ERR_ALIGN = -4,       /* a pointer or stride off the alignment the entry point states */
    NAUT_ERR_HIP = -5          /* the launch failed; see naut_last_error_string() */
} naut_status;

typedef enum {
    NAUT_BF16 = 0,
    NAUT_F16 = 1,
    NAUT_F32 = 2 /* output only */
} naut_dtype;

/*
 * Fused attention forward, bf16 q/k/v -> bf16 o (round to nearest even), fp32 lse.
 * Arguments: device pointers as described above; B batch, Hq query heads, Hkv
 * key/value heads (Hq % Hkv == 0), S sequence length (queries and keys), D head
 * dimension (64, 128 or 256); causal != 0 selects J_i = {0..i}; scale >= 0 multiplies
 * the scores (typically 1/sqrt(D)); stream as above.  Any S >= 1 is handled
 * (ragged tails are masked inside the kernel).
 * Returns NAUT_OK or a negative naut_status.
 */
int naut_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                  int B, int Hq, int Hkv, int S, int D, int causal, float scale, void* stream);

/*
 * Same computation with explicit storage types.  in_dtype is the type of q, k
 * and v (NAUT_BF16 or NAUT_F16); out_dtype the type of o (in_dtype, or
 * NAUT_F32 for an unrounded fp32 output).  The matrix products run in in_dtype
 * with fp32 accumulation; the softmax runs in fp32.
 */
int naut_attn_fwd_dt(const void* q, const void* k, const void* v, void* o, float* lse,
                     int B, int Hq, int Hkv, int S, int D, int causal, float scale, void* stream,
                     int in_dtype, int out_dtype);

/*
 * Element strides of the batch, head and sequence axes of q, k, v and o (the D axis is contiguous).
 * [B][H][S][D] has {H*S*D, S*D, D}; [B][S][H][D], the layout most frameworks produce, {S*H*D, D, H*D}.
 */
typedef struct {
    long long q_b, q_h, q_s;
    long long k_b, k_h, k_s;
    long long v_b, v_h, v_s;
    long long o_b, o_h, o_s;
} naut_strides;

/*
 * The same operator on strided tensors and on other head dimensions (the paper's evaluation spans
 * models with less common head sizes, Section 7.1): D any multiple of 8 up to 256 -- a head runs on
 * the next of the 64-, 128- and 256-wide kernels with the missing columns of Q read as zero.  `st` gives
 * element strides as above (NULL = contiguous [B][H][S][D]); q/k/v strides must be non-negative
 * multiples of 8 (16 bytes; 0 broadcasts a tensor along that axis), o strides positive multiples of 4,
 * every sequence stride at least D and at most 2^23.  lse stays contiguous [B][Hq][S].  Everything else
 * as naut_attn_fwd_dt, which is this call with st = NULL and D restricted to 64, 128 or 256.
 */
int naut_attn_fwd_strided(const void* q, const void* k, const void* v, void* o, float* lse,
                          int B, int Hq, int Hkv, int S, int D, int causal, float scale, void* stream,
                          int in_dtype, int out_dtype, const naut_strides* st);

/*
 * The same operator on FP8 inputs, the second precision of the paper's experiments (Section 6): q, k, v
 * are OCP E4M3 bytes (1 sign, 4 exponent bits with bias 7, 3 fraction bits; 0x7f/0xff are NaN and must not
 * occur), contiguous [B][H][S][D] like the 16-bit entry points, each with one scale per tensor: the real
 * tensors are descale_q * q, descale_k * k, descale_v * v (all descale factors > 0).  o is bf16, lse fp32.
 * Both products run on the FP8 matrix instructions with fp32 accumulation; P is rounded to E4M3 for the
 * second product (that rounding, relative 2^-4, is what the accuracy of this entry point is bound by).
 * D is a multiple of 16, at most 128 (a head narrower than 64 or 128 runs on the next wider kernel: the
 * missing columns of Q read as zero and those of O are not stored).  Everything else as naut_attn_fwd.
 */
int naut_attn_fwd_fp8(const void* q, const void* k, const void* v, void* o, float* lse,
                      int B, int Hq, int Hkv, int S, int D, int causal, float scale,
                      float descale_q, float descale_k, float descale_v, void* stream);

/*
 * The same on strided tensors (e.g. sequence-major [B][S][H][D], the layout FP8 attention is usually fed):
 * `st` as in naut_attn_fwd_strided, in elements, except that q/k/v strides must be multiples of 16 (their
 * elements are bytes and rows are read 16 bytes at a time); o is bf16, its strides multiples of 4.  D as in
 * naut_attn_fwd_fp8.  st = NULL means contiguous, which is what naut_attn_fwd_fp8 passes.
 */
int naut_attn_fwd_fp8_strided(const void* q, const void* k, const void* v, void* o, float* lse,
                              int B, int Hq, int Hkv, int S, int D, int causal, float scale,
                              float descale_q, float descale_k, float descale_v, void* stream,
                              const naut_strides* st);

/* Message for the last non-OK status returned on the calling thread ("" if none). Never NULL. */
const char* naut_last_error_string(void);

/* Library version, major*10000 + minor*100 + patch. */
int naut_version(void);

/*
 * Name of the kernel variant naut_attn_fwd_dt would launch for these arguments (a static string
 * such as "fwd_bm256_w8q32_bn64": 256-query work-group tile, 8 wavefronts of 32 queries, 64-key
 * steps), or NULL if the arguments are unsupported.  The choice of tile shape per workload is the
 * knob the paper leaves to its auto-tuner (Section 4.4; Section 7.2 reports 64x128 tiles with 4
 * warps on short sequences against 128x128 with 8); here it is a fixed rule on the number of
 * work-groups and the length of the key loop, fitted to timings of every variant over a grid of
 * shapes (python -m paper_2604_14825_amd.tune prints that table and flags where the rule loses), and
 * overridable with the environment variable NAUT_ATTN_VARIANT=w8q32|w4q64|bm128.
 * Host only; used by the benchmark to match profiler rows to launches.
 */
const char* naut_attn_variant_name(int B, int Hq, int S, int D, int causal, int in_dtype, int out_dtype);

/*
 * Decode-time attention (the paper's second workload, "DC", Section 6: decoding with a key/value
 * cache): Sq new query positions per head, taken to be the LAST Sq positions of a sequence of Sk,
 * attend to all Sk cached keys.  Same operator as above with
 *     q, o : [B][Hq][Sq][D]     k, v : [B][Hkv][Sk][D]     lse : [B][Hq][Sq] (fp32, may be NULL)
 * and J_i = {0..Sk-1}, or {0..Sk-Sq+i} when `causal` is non-zero (then Sk >= Sq is required; Sq == Sk
 * gives the causal self-attention of naut_attn_fwd).  bf16 in and out.  The work is bound by reading
 * K and V once, so the key axis is split over work-groups and the partial results are merged by the
 * split-merge identity of softmax (the rolling update of Section 4.2/4.3 applied across splits
 * instead of across steps); the partials live in `workspace`, DEVICE memory owned by the caller, 16-byte
 * aligned, of at least naut_attn_decode_workspace_bytes(...) bytes, which the call overwrites and
 * which must not be shared by calls that may overlap.  Two kernels are enqueued on `stream`; nothing
 * is allocated, nothing is synchronised.  Errors as above (a NULL workspace is NAUT_ERR_NULL, a short one
 * NAUT_ERR_SHAPE).
 */
int naut_attn_decode(const void* q, const void* k, const void* v, void* o, float* lse,
                     int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, float scale,
                     void* workspace, size_t workspace_bytes, void* stream);

/* The same with explicit storage types (see naut_attn_fwd_dt). */
int naut_attn_decode_dt(const void* q, const void* k, const void* v, void* o, float* lse,
                        int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, float scale,
                        void* workspace, size_t workspace_bytes, void* stream, int in_dtype, int out_dtype);

/*
 * The same on strided tensors: `st` gives element strides of the batch, head and sequence axes (the D axis
 * is contiguous) of q and o, indexed [B][Hq][Sq][D], and of k and v, indexed [B][Hkv][Sk][D] -- e.g. a
 * sequence-major K/V cache [B][Sk][Hkv][D] has {Sk*Hkv*D, D, Hkv*D}.  Same rules as naut_attn_fwd_strided
 * (q/k/v strides non-negative multiples of 8, o strides positive multiples of 4, sequence strides between D
 * and 2^23); st = NULL means contiguous, which is what naut_attn_decode_dt passes.  lse stays dense.
 * D may be any multiple of 8 up to 256 here (a head narrower than 64, 128 or 256 runs on the next wider
 * kernel, as in naut_attn_fwd_strided); naut_attn_decode and naut_attn_decode_dt keep D = 64 or 128.
 */
int naut_attn_decode_strided(const void* q, const void* k, const void* v, void* o, float* lse,
                             int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, float scale,
                             void* workspace, size_t workspace_bytes, void* stream, int in_dtype, int out_dtype,
                             const naut_strides* st);

/*
 * Decode-time attention on an FP8 (E4M3) K/V cache, the setting in which the cache is the traffic that
 * matters: q, k, v are E4M3 bytes with one scale per tensor as in naut_attn_fwd_fp8, contiguous
 * [B][H][S][D]; o is bf16, lse fp32.  D is 64 or 128.  Workspace, masks and everything else as
 * naut_attn_decode; a workspace of naut_attn_decode_workspace_bytes(...) of the same sizes is large enough.
 */
int naut_attn_decode_fp8(const void* q, const void* k, const void* v, void* o, float* lse,
                         int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, float scale,
                         float descale_q, float descale_k, float descale_v,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same on strided tensors, e.g. a sequence-major FP8 cache [B][Sk][Hkv][D]: `st` as in
 * naut_attn_decode_strided, in elements, with the FP8 rules of naut_attn_fwd_fp8_strided (q/k/v strides
 * multiples of 16, o strides multiples of 4, sequence strides between D and 2^23).  D may be any multiple
 * of 16 up to 128 here.  st = NULL means contiguous, which is what naut_attn_decode_fp8 passes.
 */
int naut_attn_decode_fp8_strided(const void* q, const void* k, const void* v, void* o, float* lse,
                                 int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, float scale,
                                 float descale_q, float descale_k, float descale_v,
                                 void* workspace, size_t workspace_bytes, void* stream, const naut_strides* st);

/*
 * naut_attn_decode for callers that cannot allocate or pass a workspace: code recorded under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * naut_attn_decode (bf16 in and out, D = 64 or 128) without `workspace`: the split partials go to a
 * 16 MiB array in the library's own static device memory, which every GPU the library runs on holds until
 * the process ends.  Sizes whose partials (naut_attn_decode_workspace_bytes) exceed 16 MiB are rejected
 * with NAUT_ERR_UNSUPPORTED and a message that names both numbers.  The call allocates and frees nothing;
 * its first use on a device looks up the array's device address (hipGetSymbolAddress, once per device), so
 * make that first call outside a graph capture.  All calls on one GPU share the one array, which keeps the
 * last call's partials (every call overwrites all it reads, nothing needs clearing): calls that may overlap
 * on one GPU -- different streams, or a graph replay beside eager calls -- race on it and must use
 * naut_attn_decode with workspaces of their own.
 */
int naut_attn_decode_static(const void* q, const void* k, const void* v, void* o, float* lse,
                            int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, float scale, void* stream);

/* Bytes of workspace naut_attn_decode[_dt|_strided] needs for these sizes; 0 if they are unsupported.  Host only. */
size_t naut_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int Sq, int Sk, int D);

/*
 * Measurement aid, not part of the attention path (the paper's evaluation, Section 6, reports throughput
 * against the hardware's capability; this gives the capability of the box at hand): a register-only loop of
 * the matrix instruction the bf16 kernels use (v_mfma_f32_32x32x16_bf16), `work_groups` work-groups of 8
 * wavefronts, each issuing trips * 16 of them = trips * 16 * 32768 FLOP per wavefront, with no LDS, memory
 * or vector work beside them.  kind 0: all operands zero; kind 1: operands with random signs, fractions and
 * a few binades of exponent, a fresh A operand every instruction -- the switching activity of real data,
 * which decides how far the chip lowers its clock under sustained matrix load.  `out` (device memory,
 * work_groups * 512 floats, overwritten) only keeps the loop alive.  Asynchronous on `stream`.
 */
int naut_probe_mfma(float* out, size_t out_floats, int work_groups, int trips, int kind, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NAUT_ATTN_H */
