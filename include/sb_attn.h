/*
 * sb_attn.h -- C ABI of the stick-breaking attention library for MI355X (gfx950).
 *
 * The operation (paper section 2, Eq. 1), per batch b and head h, 0-based rows:
 *
 *     z[i,j] = q_j . k_i / sqrt(d)                       logits
 *     A[i,j] = sigma(z[i,j]) * prod_{i<k<j} (1 - sigma(z[k,j]))      for i < j
 *     o_j    = sum_{i<j} A[i,j] v_i                      (o_0 = 0: empty sum)
 *
 * evaluated in the log-space form of section 4 (Eq. 2) with a sweep over key
 * tiles from the diagonal towards key 0 that carries, per query row, the running
 * sum of softplus(z) (Algorithm 1).  The backward is Eq. 4 / Algorithm 2.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library
 *     never allocates, frees or keeps device memory and holds no state.
 *   - Layout [B, H, T, d], contiguous, d fastest.  `m` is [B, H, T].
 *   - d is 32, 64 or 128; B, H, T >= 1 (any T, not only multiples of the tile);
 *     B*H*T*d must be below 2^40 elements.
 *   - Every tensor pointer must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void*; NULL means the default stream.
 *   - Calls only enqueue work: they return after the launch, without a device
 *     synchronisation.  The return value is an sb_status (0 = ok, negative =
 *     error, nothing was enqueued).  Nothing is thrown across the boundary.
 *   - Outputs are written for every row, including the all-zero row j = 0.
 */
#ifndef SB_ATTN_H
#define SB_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SB_OK = 0,
    SB_ERR_NULL = -1,        /* a required pointer is NULL */
    SB_ERR_SHAPE = -2,       /* B, H or T < 1, or the tensor is too large */
    SB_ERR_UNSUPPORTED = -3, /* d is not 32, 64 or 128 */
    SB_ERR_ALIGN = -4,       /* a pointer is not 16-byte aligned */
    SB_ERR_LAUNCH = -5,      /* the HIP launch reported an error */
    SB_ERR_WORKSPACE = -6    /* workspace missing or too small */
} sb_status;

/*
 * Forward, Eq. 1 via Algorithm 1.  q, k, v, o: bf16 (16-bit brain float).
 * Logits, softplus, the carried sums and the output accumulator are fp32; the
 * weights are rounded to bf16 only as matrix-core operands; o is rounded to
 * bf16 (nearest even) on store.
 */
int sb_attn_fwd(const void* q, const void* k, const void* v, void* o,
                int B, int H, int T, int d, void* stream);

/*
 * Inference forward with early halt (the paper's "conditional computation",
 * section 4.1): as sb_attn_fwd, but a block of 128 query rows stops sweeping keys
 * once every one of its rows has less than eps of its stick left
 * (prod (1 - beta) < eps over the keys swept so far).  No skipped key can weigh more
 * than what is left, so |o_j - exact o_j| <= eps * max_i |v_i| per component.
 * 0 < eps < 1 (SB_ERR_SHAPE otherwise).  How much is skipped depends on the data.
 * tile_counts: optional (may be NULL) device pointer to 2 x u64, 16-byte aligned;
 * the call ADDS to [0] the 64-key tiles swept beyond the diagonal band and to [1]
 * the tiles a full sweep would take (per 128-row block), for reporting.
 */
int sb_attn_fwd_halt(const void* q, const void* k, const void* v, void* o,
                     float eps, unsigned long long* tile_counts,
                     int B, int H, int T, int d, void* stream);

/*
 * Training forward: as sb_attn_fwd, and also writes m[b,h,j] (fp32) =
 * -sum_{i<j} softplus(z[i,j]) = log(1 - sum_i A[i,j]), the vector that
 * Algorithm 1 stores at its end and Algorithm 2 reads back.  m[.,.,0] = 0.
 */
int sb_attn_fwd_train(const void* q, const void* k, const void* v, void* o, float* m,
                      int B, int H, int T, int d, void* stream);

/*
 * fp32 forward (fp32 q, k, v, o, optional m; all arithmetic fp32 on the vector
 * ALU).  m may be NULL.
 */
int sb_attn_fwd_f32(const float* q, const float* k, const float* v, float* o, float* m,
                    int B, int H, int T, int d, void* stream);

/*
 * Backward, Eq. 4 with the per-tile steps of Algorithm 2 (dV = A^T dO,
 * dK = dZ^T Q / sqrt(d), dQ = dZ K / sqrt(d)).
 * q, k, v, dout: bf16.  m: fp32 from sb_attn_fwd_train.  dq, dk, dv: fp32,
 * fully overwritten (no need to clear them).
 * workspace: caller-owned device scratch of at least
 * sb_attn_bwd_workspace_bytes(B,H,T,d) bytes, 16-byte aligned; its contents on
 * entry do not matter and are garbage afterwards.  It holds two floats per
 * (query row, 32-key strip), one int per 128-row block of queries and of keys and
 * d floats per 128-row block (partial sums of sb_attn_bwd_rb's dr):
 * B*H*(8*T*ceil(T/32) + (8 + 4*d)*ceil(T/128)) bytes.  SB_ERR_WORKSPACE if it is NULL or
 * too small.  sb_attn_bwd_workspace_bytes returns 0 for a bad shape.
 * The carried sums make the workspace grow with T^2 (T^2/4 bytes per head: 4 MiB at
 * T = 4096, 64 MiB at T = 16384, 1 GiB at T = 65536), where Algorithm 2 itself keeps O(T):
 * that is the price of writing dK and dV without atomics.  Heads are independent, so a caller
 * short of memory at long T runs the backward on groups of heads (or batch entries) with one
 * smaller workspace, one call after the other.
 * m is required (SB_ERR_NULL otherwise): it is what the training forward of the same step
 * leaves behind, and rebuilding it here would cost a forward sweep (two of the backward's
 * seven contractions) that no caller of a backward has reason to pay.
 * No atomics are used: results are bit-reproducible from run to run.
 */
size_t sb_attn_bwd_workspace_bytes(int B, int H, int T, int d);
int sb_attn_bwd(const void* q, const void* k, const void* v, const float* m, const void* dout,
                float* dq, float* dk, float* dv, void* workspace, size_t workspace_bytes,
                int B, int H, int T, int d, void* stream);

/*
 * The two passes of sb_attn_bwd on their own (same arguments, same workspace, which
 * carries the per-strip sums from the first to the second):
 *   sb_attn_bwd_dq    query-stationary pass of Algorithm 2: dq, and the carries.
 *   sb_attn_bwd_dkdv  key-stationary pass: dk, dv from the carries; must follow
 *                     sb_attn_bwd_dq on the same inputs and workspace.
 * sb_attn_bwd is exactly the first followed by the second.
 */
int sb_attn_bwd_dq(const void* q, const void* k, const void* v, const float* m, const void* dout,
                   float* dq, void* workspace, size_t workspace_bytes,
                   int B, int H, int T, int d, void* stream);
int sb_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dout,
                     float* dk, float* dv, void* workspace, size_t workspace_bytes,
                     int B, int H, int T, int d, void* stream);

/*
 * Remainder bias (Appendix C, the output equation with the remainder term): the part
 * of the stick that no key took, 1 - sum_i A[i,j] = exp(m_j), goes to a learned
 * embedding r of the head,  o_j = sum_{i<j} A[i,j] v_i + exp(m_j) r_h.
 * r: bf16 [H, d] (one embedding per head, shared by the batch), device, 16-byte aligned.
 *   sb_attn_fwd_rb  as sb_attn_fwd_train with the extra term; m may be NULL (inference).
 *                   Row 0 has nothing to attend to: o_0 = r_h.
 *   sb_attn_bwd_rb  as sb_attn_bwd for that forward (m from sb_attn_fwd_rb, same
 *                   workspace rules); dZ gains -beta[i,j] exp(m_j) (dO_j . r_h), and
 *                   dr [H, d] fp32 (fully overwritten) = sum over the batch and the rows
 *                   of exp(m_j) dO_j, added in a fixed order (bit-reproducible).
 */
int sb_attn_fwd_rb(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                   int B, int H, int T, int d, void* stream);
int sb_attn_bwd_rb(const void* q, const void* k, const void* v, const void* r, const float* m,
                   const void* dout, float* dq, float* dk, float* dv, float* dr,
                   void* workspace, size_t workspace_bytes, int B, int H, int T, int d, void* stream);

/*
 * Grouped kv heads (the paper's larger models pair 12 query heads with 4 kv heads;
 * Appendix C, model table): q, o, dout, dq are [B, H, T, d], k, v, dk, dv are
 * [B, Hkv, T, d], H a multiple of Hkv (SB_ERR_SHAPE otherwise); query head h attends to
 * kv head h / (H / Hkv).  These are the general forms of the calls above:
 *   sb_attn_fwd_gqa  forward; r (remainder bias, [H, d] bf16) and m may each be NULL.
 *   sb_attn_bwd_gqa  backward; r and dr both NULL or both given; dk, dv are summed over
 *                    the query heads of each group inside one workgroup's registers (no
 *                    atomics, bit-reproducible).  Workspace as for sb_attn_bwd with the
 *                    number of query heads: sb_attn_bwd_workspace_bytes(B, H, T, d).
 */
int sb_attn_fwd_gqa(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                    int B, int H, int Hkv, int T, int d, void* stream);
int sb_attn_bwd_gqa(const void* q, const void* k, const void* v, const void* r, const float* m,
                    const void* dout, float* dq, float* dk, float* dv, float* dr,
                    void* workspace, size_t workspace_bytes, int B, int H, int Hkv, int T, int d, void* stream);

/*
 * Packed variable-length batches (the paper trains padding-free): the sequences of a batch
 * lie one after the other along T and attend only inside themselves.
 * q, o, dout, dq: [H, Ttot, d]; k, v, dk, dv: [Hkv, Ttot, d]; m: [H, Ttot] fp32;
 * r (optional), dr: [H, d].  cu_seqlens: nseq + 1 ints on the DEVICE, cu[0] = 0,
 * non-decreasing, cu[nseq] = Ttot; sequence s is rows cu[s] .. cu[s+1]-1 (empty
 * sequences allowed).  max_T: an upper bound of the longest sequence, 1 <= max_T <= Ttot;
 * it sizes the launch and the workspace, so a tight bound is cheaper.  The library cannot
 * read cu_seqlens on the host: rows of a sequence beyond max_T, or beyond Ttot, are left
 * unwritten rather than touched out of bounds; other malformed offsets give undefined
 * values in o / the gradients of the affected sequences.
 * The first row of every sequence has nothing to attend to (o = 0, or r with the bias).
 * Otherwise exactly sb_attn_fwd_gqa / sb_attn_bwd_gqa per sequence, in one launch each;
 * dr adds up over all sequences in a fixed order.
 * Workspace: sb_attn_varlen_bwd_workspace_bytes(nseq, H, Ttot, max_T, d) bytes
 * = 8*H*Ttot*ceil(max_T/32) + nseq*H*(8 + 4*d)*ceil(max_T/128).
 */
int sb_attn_varlen_fwd(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                       const int* cu_seqlens, int nseq, int H, int Hkv, int Ttot, int max_T, int d, void* stream);
size_t sb_attn_varlen_bwd_workspace_bytes(int nseq, int H, int Ttot, int max_T, int d);
int sb_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* r, const float* m,
                       const void* dout, float* dq, float* dk, float* dv, float* dr,
                       const int* cu_seqlens, int nseq, int H, int Hkv, int Ttot, int max_T, int d,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Single-token decode (inference on a key/value cache; the paper's long-context
 * evaluation regime): one new query per (batch entry, head) against T cached keys and
 * values, all visible - the last row of Eq. 1 on the sequence extended by the new position.
 * q, o: bf16 [B, H, d].  k, v: bf16 [B, Hkv, Tcap, d], rows 0..T-1 valid, 1 <= T <= Tcap
 * (Tcap = allocated rows per head).  r: optional remainder bias [H, d] bf16 (NULL = none).
 * m: optional fp32 [B, H], log of the stick left over (NULL = not wanted).
 * One pass over K and V (bound by HBM bandwidth), split over the keys; partial results are
 * combined in a fixed order (bit-reproducible).  T <= 524288 (SB_ERR_SHAPE beyond),
 * B*Hkv <= 65535.  workspace: sb_attn_decode_workspace_bytes(B, H, T, d) bytes of device
 * scratch, 16-byte aligned (at most 4*B*H*256*(d+1) bytes); SB_ERR_WORKSPACE if NULL or too
 * small.
 */
size_t sb_attn_decode_workspace_bytes(int B, int H, int T, int d);
int sb_attn_decode(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                   void* workspace, size_t workspace_bytes,
                   int B, int H, int Hkv, int T, int Tcap, int d, void* stream);

/*
 * sb_attn_decode for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and kernels as sb_attn_decode, minus the workspace: the partial results
 * of the key chunks go to a scratch array of SB_DECODE_STATIC_BYTES that is part of the
 * library's device image (every GPU the library runs on holds its own copy until the process
 * ends).  The call allocates and frees nothing; the first call on a device looks up the
 * array's device address (hipGetSymbolAddress) and keeps it.
 * Limit: sb_attn_decode_workspace_bytes(B, H, T, d) <= SB_DECODE_STATIC_BYTES, otherwise
 * SB_ERR_WORKSPACE and nothing is enqueued (B*H*min(ceil(T/64), 256)*(d+1)*4 bytes: e.g.
 * B*H = 128 heads of d = 128 at any T, or 256 heads up to T = 8192).
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 * (different streams, or different host threads) race on it.  Calls on one stream are safe
 * back to back; every element a call reads it has written itself, so nothing needs clearing.
 */
#define SB_DECODE_STATIC_BYTES ((size_t)33554432)
int sb_attn_decode_static(const void* q, const void* k, const void* v, const void* r, void* o, float* m,
                          int B, int H, int Hkv, int T, int Tcap, int d, void* stream);

/* Human-readable name of a status code (static storage). */
const char* sb_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int sb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SB_ATTN_H */
