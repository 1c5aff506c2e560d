// naut_attn.hip -- the C ABI of the fused attention forward (gfx950, MI355X): argument checks, launch
// parameters, dispatch on head dimension and storage types.  The kernels and their launcher live in
// naut_attn_kernels.h; their instantiations are compiled in naut_attn_inst.hip, one translation unit per
// storage-type pair.
#include "naut_attn_kernels.h"

namespace naut {

thread_local char g_err[256] = "";

int fail(int code, const char* msg)
{
    snprintf(g_err, sizeof g_err, "%s", msg);
    return code;
}

int fail_launch(hipError_t e)
{
    snprintf(g_err, sizeof g_err, "kernel launch failed: %s", hipGetErrorString(e));
    return NAUT_ERR_HIP;
}

}  // namespace naut

namespace naut_k {

// defined in naut_attn_inst.hip
extern template int launch<64, NAUT_BF16, NAUT_BF16>(const Params&, int, hipStream_t);
extern template int launch<128, NAUT_BF16, NAUT_BF16>(const Params&, int, hipStream_t);
extern template int launch<256, NAUT_BF16, NAUT_BF16>(const Params&, int, hipStream_t);
extern template int launch<64, NAUT_BF16, NAUT_F32>(const Params&, int, hipStream_t);
extern template int launch<128, NAUT_BF16, NAUT_F32>(const Params&, int, hipStream_t);
extern template int launch<256, NAUT_BF16, NAUT_F32>(const Params&, int, hipStream_t);
extern template int launch<64, NAUT_F16, NAUT_F16>(const Params&, int, hipStream_t);
extern template int launch<128, NAUT_F16, NAUT_F16>(const Params&, int, hipStream_t);
extern template int launch<256, NAUT_F16, NAUT_F16>(const Params&, int, hipStream_t);
extern template int launch<64, NAUT_F16, NAUT_F32>(const Params&, int, hipStream_t);
extern template int launch<128, NAUT_F16, NAUT_F32>(const Params&, int, hipStream_t);
extern template int launch<256, NAUT_F16, NAUT_F32>(const Params&, int, hipStream_t);

}  // namespace naut_k

namespace {

using namespace naut;
using namespace naut_k;

bool dtype_pair_ok(int in_dtype, int out_dtype)
{
    if (in_dtype != NAUT_BF16 && in_dtype != NAUT_F16)
        return false;
    return out_dtype == in_dtype || out_dtype == NAUT_F32;
}

}  // namespace

extern "C" {

int naut_attn_fwd_strided(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                          int S, int D, int causal, float scale, void* stream, int in_dtype, int out_dtype,
                          const naut_strides* st)
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
    if (D % 8 != 0 || D > 256)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be a multiple of 8, at most 256");
    if (!dtype_pair_ok(in_dtype, out_dtype))
        return fail(NAUT_ERR_UNSUPPORTED, "supported dtypes: q/k/v bf16 or f16; o of the same type or f32");
    if ((long long)B * Hq > 0x7fffffffLL || (long long)B * Hkv > 0x7fffffffLL)
        return fail(NAUT_ERR_UNSUPPORTED, "B*Hq too large");
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
        if (x < 0 || x % 8 != 0)
            return fail(NAUT_ERR_ALIGN, "q/k/v strides must be non-negative multiples of 8 elements (16 bytes)");
    if (st->o_b <= 0 || st->o_h <= 0 || st->o_s <= 0 || st->o_b % 4 != 0 || st->o_h % 4 != 0 || st->o_s % 4 != 0)
        return fail(NAUT_ERR_ALIGN, "o strides must be positive multiples of 4 elements");
    if (st->q_s < D || st->k_s < D || st->v_s < D || st->o_s < D)
        return fail(NAUT_ERR_SHAPE, "a sequence stride is smaller than D: rows would overlap");
    const long long max_rs = 1LL << 23;  // elements: keeps 64 rows of byte offsets inside 32 bits
    if (st->q_s > max_rs || st->k_s > max_rs || st->v_s > max_rs || st->o_s > max_rs)
        return fail(NAUT_ERR_UNSUPPORTED, "sequence stride too large");

    const int out_b = out_dtype == NAUT_F32 ? 4 : 2;
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
    // D = 256: the K/V of one head is twice as large and every 128-query work-group streams it, so an XCD
    // is kept to two heads at a time (measured: +2..5 % over all of its heads at once; no gain for D <= 128)
    p.hao = D > 128 ? 2 : 0;
    hipStream_t st_ = (hipStream_t)stream;
    const int DK = D <= 64 ? 64 : D <= 128 ? 128 : 256;  // width the kernel is compiled for

#define NAUT_DISPATCH(DD, IN, OUT)                         \
    if (DK == DD && in_dtype == IN && out_dtype == OUT)   \
        return launch<DD, IN, OUT>(p, causal, st_);
    NAUT_DISPATCH(128, NAUT_BF16, NAUT_BF16)
    NAUT_DISPATCH(64, NAUT_BF16, NAUT_BF16)
    NAUT_DISPATCH(128, NAUT_BF16, NAUT_F32)
    NAUT_DISPATCH(64, NAUT_BF16, NAUT_F32)
    NAUT_DISPATCH(128, NAUT_F16, NAUT_F16)
    NAUT_DISPATCH(64, NAUT_F16, NAUT_F16)
    NAUT_DISPATCH(128, NAUT_F16, NAUT_F32)
    NAUT_DISPATCH(64, NAUT_F16, NAUT_F32)
    NAUT_DISPATCH(256, NAUT_BF16, NAUT_BF16)
    NAUT_DISPATCH(256, NAUT_BF16, NAUT_F32)
    NAUT_DISPATCH(256, NAUT_F16, NAUT_F16)
    NAUT_DISPATCH(256, NAUT_F16, NAUT_F32)
#undef NAUT_DISPATCH
    return fail(NAUT_ERR_UNSUPPORTED, "no kernel for this (D, dtype) combination");
}

int naut_attn_fwd_dt(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv,
                     int S, int D, int causal, float scale, void* stream, int in_dtype, int out_dtype)
{
    if (D > 0 && D != 64 && D != 128 && D != 256)
        return fail(NAUT_ERR_UNSUPPORTED, "D must be 64, 128 or 256 (naut_attn_fwd_strided takes other head dimensions)");
    return naut_attn_fwd_strided(q, k, v, o, lse, B, Hq, Hkv, S, D, causal, scale, stream, in_dtype, out_dtype, nullptr);
}

int naut_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int B, int Hq, int Hkv, int S,
                  int D, int causal, float scale, void* stream)
{
    return naut_attn_fwd_dt(q, k, v, o, lse, B, Hq, Hkv, S, D, causal, scale, stream, NAUT_BF16, NAUT_BF16);
}

const char* naut_last_error_string(void) { return g_err; }

int naut_version(void) { return 100; }

const char* naut_attn_variant_name(int B, int Hq, int S, int D, int causal, int in_dtype, int out_dtype)
{
    if (B <= 0 || Hq <= 0 || S <= 0 || (D != 64 && D != 128 && D != 256) || !dtype_pair_ok(in_dtype, out_dtype))
        return nullptr;
    if (D == 256)
        return "fwd_bm128_w4q32_bn32";
    const int variant = pick_variant(S, (long long)B * Hq, D, causal);
    return variant < 0 ? nullptr : kVariantName[variant];
}

}  // extern "C"
