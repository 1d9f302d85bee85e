// C-ABI entry points: argument validation and dispatch to the kernel launchers.
// See include/sb_attn.h for the contract of every call.
#include "../../include/sb_attn.h"
#include "../../include/sb_diag.h"
#include "sb_kernels.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(int B, int H, int T, int d)
{
    if (B < 1 || H < 1 || T < 1) return SB_ERR_SHAPE;
    if (d != 32 && d != 64 && d != 128) return SB_ERR_UNSUPPORTED;
    const double elems = (double)B * H * (double)T * d;
    if (elems >= 1099511627776.0 /* 2^40 */ || (double)B * H > 2147483647.0) return SB_ERR_SHAPE;
    return SB_OK;
}

}  // namespace

extern "C" {

int sb_attn_fwd_train(const void* q, const void* k, const void* v, void* o, float* m,
                      int B, int H, int T, int d, void* stream);

int sb_attn_fwd(const void* q, const void* k, const void* v, void* o,
                int B, int H, int T, int d, void* stream)
{
    if (!q || !k || !v || !o) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_bf16(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                       static_cast<const uint16_t*>(v), nullptr, static_cast<uint16_t*>(o),
                                       nullptr, B, H, H, T, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_attn_fwd_gqa(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                    int B, int H, int Hkv, int T, int d, void* stream)
{
    if (!q || !k || !v || !o) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (Hkv < 1 || H % Hkv != 0) return SB_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(r) || !aligned16(o) || !aligned16(m))
        return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_bf16(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                       static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(r),
                                       static_cast<uint16_t*>(o), m, B, H, Hkv, T, d,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_attn_fwd_rb(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                   int B, int H, int T, int d, void* stream)
{
    if (!r) return SB_ERR_NULL;
    return sb_attn_fwd_gqa(q, k, v, r, o, m, B, H, H, T, d, stream);
}

int sb_attn_fwd_halt(const void* q, const void* k, const void* v, void* o,
                     float eps, unsigned long long* tile_counts,
                     int B, int H, int T, int d, void* stream)
{
    if (!q || !k || !v || !o) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (!(eps > 0.0f && eps < 1.0f)) return SB_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(tile_counts))
        return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_bf16_halt(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                            static_cast<const uint16_t*>(v), static_cast<uint16_t*>(o),
                                            eps, tile_counts, B, H, T, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_attn_fwd_train(const void* q, const void* k, const void* v, void* o, float* m,
                      int B, int H, int T, int d, void* stream)
{
    if (!q || !k || !v || !o || !m) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(m))
        return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_bf16(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                       static_cast<const uint16_t*>(v), nullptr, static_cast<uint16_t*>(o),
                                       m, B, H, H, T, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_attn_fwd_f32(const float* q, const float* k, const float* v, float* o, float* m,
                    int B, int H, int T, int d, void* stream)
{
    if (!q || !k || !v || !o) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || (m && !aligned16(m)))
        return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_f32(q, k, v, o, m, B, H, T, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

size_t sb_attn_bwd_workspace_bytes(int B, int H, int T, int d)
{
    if (check_shape(B, H, T, d) != SB_OK) return 0;
    return sb::bwd_workspace_bytes(B, H, T, d);
}

}  // extern "C"

namespace {

int bwd_checked(const void* q, const void* k, const void* v, const void* r, const float* m, const void* dout,
                float* dq, float* dk, float* dv, float* dr, void* workspace, size_t workspace_bytes,
                int B, int H, int Hkv, int T, int d, int passes, void* stream)
{
    if (!q || !k || !v || !dout) return SB_ERR_NULL;
    if ((r == nullptr) != (dr == nullptr)) return SB_ERR_NULL;
    if ((passes & 1) && (!m || !dq)) return SB_ERR_NULL;
    if ((passes & 2) && (!dk || !dv)) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (Hkv < 1 || H % Hkv != 0) return SB_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(m) || !aligned16(dout) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv) || !aligned16(workspace) ||
        !aligned16(r) || !aligned16(dr))
        return SB_ERR_ALIGN;
    if (!workspace || workspace_bytes < sb::bwd_workspace_bytes(B, H, T, d)) return SB_ERR_WORKSPACE;
    hipError_t e = sb::launch_bwd_bf16(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                       static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(r), m,
                                       static_cast<const uint16_t*>(dout), dq, dk, dv, dr,
                                       static_cast<float*>(workspace),
                                       B, H, Hkv, T, d, passes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int sb_attn_bwd(const void* q, const void* k, const void* v, const float* m, const void* dout,
                float* dq, float* dk, float* dv, void* workspace, size_t workspace_bytes,
                int B, int H, int T, int d, void* stream)
{
    return bwd_checked(q, k, v, nullptr, m, dout, dq, dk, dv, nullptr, workspace, workspace_bytes,
                       B, H, H, T, d, 3, stream);
}

int sb_attn_bwd_rb(const void* q, const void* k, const void* v, const void* r, const float* m,
                   const void* dout, float* dq, float* dk, float* dv, float* dr,
                   void* workspace, size_t workspace_bytes, int B, int H, int T, int d, void* stream)
{
    if (!r || !dr) return SB_ERR_NULL;
    return bwd_checked(q, k, v, r, m, dout, dq, dk, dv, dr, workspace, workspace_bytes, B, H, H, T, d, 3, stream);
}

int sb_attn_bwd_gqa(const void* q, const void* k, const void* v, const void* r, const float* m,
                    const void* dout, float* dq, float* dk, float* dv, float* dr,
                    void* workspace, size_t workspace_bytes, int B, int H, int Hkv, int T, int d, void* stream)
{
    return bwd_checked(q, k, v, r, m, dout, dq, dk, dv, dr, workspace, workspace_bytes, B, H, Hkv, T, d, 3, stream);
}

int sb_attn_bwd_dq(const void* q, const void* k, const void* v, const float* m, const void* dout,
                   float* dq, void* workspace, size_t workspace_bytes,
                   int B, int H, int T, int d, void* stream)
{
    return bwd_checked(q, k, v, nullptr, m, dout, dq, nullptr, nullptr, nullptr, workspace, workspace_bytes,
                       B, H, H, T, d, 1, stream);
}

int sb_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dout,
                     float* dk, float* dv, void* workspace, size_t workspace_bytes,
                     int B, int H, int T, int d, void* stream)
{
    return bwd_checked(q, k, v, nullptr, nullptr, dout, nullptr, dk, dv, nullptr, workspace, workspace_bytes,
                       B, H, H, T, d, 2, stream);
}

namespace {
int check_varlen(int nseq, int H, int Hkv, int Ttot, int max_T, int d)
{
    if (nseq < 1 || H < 1 || Hkv < 1 || H % Hkv != 0 || Ttot < 1 || max_T < 1 || max_T > Ttot) return SB_ERR_SHAPE;
    if (d != 32 && d != 64 && d != 128) return SB_ERR_UNSUPPORTED;
    if ((double)H * Ttot * d >= 1099511627776.0 || (double)nseq * H > 2147483647.0) return SB_ERR_SHAPE;
    return SB_OK;
}
}  // namespace

int sb_attn_varlen_fwd(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                       const int* cu_seqlens, int nseq, int H, int Hkv, int Ttot, int max_T, int d, void* stream)
{
    if (!q || !k || !v || !o || !cu_seqlens) return SB_ERR_NULL;
    if (int rc = check_varlen(nseq, H, Hkv, Ttot, max_T, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(r) || !aligned16(o) || !aligned16(m))
        return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_bf16_varlen(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                              static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(r),
                                              static_cast<uint16_t*>(o), m, cu_seqlens, nseq, H, Hkv, Ttot, max_T, d,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

size_t sb_attn_varlen_bwd_workspace_bytes(int nseq, int H, int Ttot, int max_T, int d)
{
    if (check_varlen(nseq, H, H, Ttot, max_T, d) != SB_OK) return 0;
    return sb::bwd_varlen_workspace_bytes(nseq, H, Ttot, max_T, d);
}

int sb_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* r, const float* m,
                       const void* dout, float* dq, float* dk, float* dv, float* dr,
                       const int* cu_seqlens, int nseq, int H, int Hkv, int Ttot, int max_T, int d,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k || !v || !m || !dout || !dq || !dk || !dv || !cu_seqlens) return SB_ERR_NULL;
    if ((r == nullptr) != (dr == nullptr)) return SB_ERR_NULL;
    if (int rc = check_varlen(nseq, H, Hkv, Ttot, max_T, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(m) || !aligned16(dout) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv) || !aligned16(workspace) ||
        !aligned16(r) || !aligned16(dr))
        return SB_ERR_ALIGN;
    if (!workspace || workspace_bytes < sb::bwd_varlen_workspace_bytes(nseq, H, Ttot, max_T, d))
        return SB_ERR_WORKSPACE;
    hipError_t e = sb::launch_bwd_bf16_varlen(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                              static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(r), m,
                                              static_cast<const uint16_t*>(dout), dq, dk, dv, dr,
                                              static_cast<float*>(workspace), cu_seqlens, nseq, H, Hkv,
                                              Ttot, max_T, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

namespace {
int check_decode(int B, int H, int Hkv, int T, int Tcap, int d)
{
    if (B < 1 || H < 1 || Hkv < 1 || H % Hkv != 0 || T < 1 || Tcap < T) return SB_ERR_SHAPE;
    if (d != 32 && d != 64 && d != 128) return SB_ERR_UNSUPPORTED;
    if (T > sb::decode_max_T() || (double)B * Hkv > 65535.0 || (double)B * H * (double)Tcap * d >= 1099511627776.0)
        return SB_ERR_SHAPE;
    return SB_OK;
}
}  // namespace

size_t sb_attn_decode_workspace_bytes(int B, int H, int T, int d)
{
    if (check_decode(B, H, H, T, T, d) != SB_OK) return 0;
    return sb::decode_workspace_bytes(B, H, T, d);
}

int sb_attn_decode(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                   void* workspace, size_t workspace_bytes,
                   int B, int H, int Hkv, int T, int Tcap, int d, void* stream)
{
    if (!q || !k || !v || !o) return SB_ERR_NULL;
    if (int rc = check_decode(B, H, Hkv, T, Tcap, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(r) || !aligned16(o) || !aligned16(m) ||
        !aligned16(workspace))
        return SB_ERR_ALIGN;
    if (!workspace || workspace_bytes < sb::decode_workspace_bytes(B, H, T, d)) return SB_ERR_WORKSPACE;
    hipError_t e = sb::launch_decode(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                     static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(r),
                                     static_cast<uint16_t*>(o), m, static_cast<float*>(workspace),
                                     B, H, Hkv, T, Tcap, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_attn_decode_static(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                          int B, int H, int Hkv, int T, int Tcap, int d, void* stream)
{
    if (!q || !k || !v || !o) return SB_ERR_NULL;
    if (int rc = check_decode(B, H, Hkv, T, Tcap, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(r) || !aligned16(o) || !aligned16(m))
        return SB_ERR_ALIGN;
    if (sb::decode_workspace_bytes(B, H, T, d) > sb::decode_static_bytes()) return SB_ERR_WORKSPACE;
    float* scratch = nullptr;
    if (sb::decode_static_scratch(&scratch) != hipSuccess) return SB_ERR_LAUNCH;
    hipError_t e = sb::launch_decode(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                     static_cast<const uint16_t*>(v), static_cast<const uint16_t*>(r),
                                     static_cast<uint16_t*>(o), m, scratch,
                                     B, H, Hkv, T, Tcap, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_diag_mfma_rate(const void* operands, size_t operand_bytes, int iters, unsigned long long* ticks,
                      double* flop, void* stream)
{
    if (!operands || !ticks || !flop) return SB_ERR_NULL;
    if (operand_bytes < (1u << 20) || iters < 1) return SB_ERR_SHAPE;
    if (!aligned16(operands) || !aligned16(ticks)) return SB_ERR_ALIGN;
    *flop = sb::diag_mfma_flop(iters);
    hipError_t e = sb::launch_diag_mfma(operands, iters, ticks, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_diag_stream_read(const void* data, size_t bytes, unsigned int* sink, void* stream)
{
    if (!data || !sink) return SB_ERR_NULL;
    if (bytes < (1u << 20) || bytes % 16 != 0) return SB_ERR_SHAPE;
    if (!aligned16(data)) return SB_ERR_ALIGN;
    hipError_t e = sb::launch_diag_stream(data, bytes, sink, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_diag_fwd_clock(const void* q, const void* k, const void* v, void* o, float* m,
                      int B, int H, int T, int d, unsigned long long* clocks, void* stream)
{
    if (!q || !k || !v || !o || !m || !clocks) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(m) || !aligned16(clocks))
        return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_bf16(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                       static_cast<const uint16_t*>(v), nullptr, static_cast<uint16_t*>(o),
                                       m, B, H, H, T, d, static_cast<hipStream_t>(stream), clocks);
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

int sb_diag_fwd_tri(const void* q, const void* k, const void* v, void* o, float* m,
                    int B, int H, int T, int d, void* stream)
{
    if (!q || !k || !v || !o || !m) return SB_ERR_NULL;
    if (int rc = check_shape(B, H, T, d)) return rc;
    if (d != 128) return SB_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(m)) return SB_ERR_ALIGN;
    hipError_t e = sb::launch_fwd_bf16_tri(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                                           static_cast<const uint16_t*>(v), static_cast<uint16_t*>(o), m,
                                           B, H, T, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SB_OK : SB_ERR_LAUNCH;
}

const char* sb_status_string(int status)
{
    switch (status) {
    case SB_OK: return "ok";
    case SB_ERR_NULL: return "null pointer";
    case SB_ERR_SHAPE: return "bad shape";
    case SB_ERR_UNSUPPORTED: return "unsupported head dimension (need 32, 64 or 128)";
    case SB_ERR_ALIGN: return "pointer not 16-byte aligned";
    case SB_ERR_LAUNCH: return "kernel launch failed";
    case SB_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
    }
}

int sb_version(void) { return 100; }

}  // extern "C"
