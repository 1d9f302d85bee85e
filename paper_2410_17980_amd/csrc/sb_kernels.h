// Internal launcher declarations shared by the C-ABI translation unit and the
// kernel translation units.  Not part of the public interface.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sb {

// Each launcher validates nothing (the C-ABI layer did) and returns the HIP
// error of the launch.
hipError_t launch_fwd_f32(const float* q, const float* k, const float* v, float* o, float* m,
                          int B, int H, int T, int d, hipStream_t stream);

// rb: remainder-bias embeddings [H][d] bf16, or nullptr; m: nullptr when not wanted.
// H query heads, Hkv kv heads (H a multiple of Hkv): k, v are [B][Hkv][T][d].
// clocks: nullptr, or 4 x u64 on the device that receive the shader-clock and 100 MHz reference
// counters at the start ([0], [1]) and the end ([2], [3]) of the launch's first workgroup.
hipError_t launch_fwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                           uint16_t* o, float* m, int B, int H, int Hkv, int T, int d, hipStream_t stream,
                           unsigned long long* clocks = nullptr);

// measurement variant of the d = 128 training forward: in-tile cumulative sum by triangular MFMA
hipError_t launch_fwd_bf16_tri(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o, float* m,
                               int B, int H, int T, hipStream_t stream);

// forward that stops sweeping a query block once every row has less than eps of its stick left
hipError_t launch_fwd_bf16_halt(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o,
                                float eps, unsigned long long* tile_counts,
                                int B, int H, int T, int d, hipStream_t stream);

// workspace: bwd_workspace_bytes(B, H, T, d) bytes of device memory, 16-byte aligned.
// passes: bit 0 = query-stationary pass (dq and the carries in the workspace; with rb
// also drb [H][d]), bit 1 = key-stationary pass (dk, dv from the carries).
// rb, drb: remainder-bias embeddings and their gradient, both nullptr without the bias.
// H query heads, Hkv kv heads: k, v, dk, dv are [B][Hkv][T][d].
size_t bwd_workspace_bytes(int B, int H, int T, int d);
hipError_t launch_bwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                           const float* m, const uint16_t* dout, float* dq, float* dk, float* dv,
                           float* drb, float* workspace,
                           int B, int H, int Hkv, int T, int d, int passes, hipStream_t stream);

// Packed variable-length batches: tensors [H][Ttot][d] ([Hkv][Ttot][d] for k, v, dk, dv), m
// [H][Ttot]; cu: nseq + 1 ints on the device, cu[0] = 0 <= ... <= cu[nseq] = Ttot; max_T: an
// upper bound of the longest sequence (sizes the grid and the workspace).
hipError_t launch_fwd_bf16_varlen(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                                  uint16_t* o, float* m, const int* cu, int nseq, int H, int Hkv,
                                  int Ttot, int max_T, int d, hipStream_t stream);
size_t bwd_varlen_workspace_bytes(int nseq, int H, int Ttot, int max_T, int d);
hipError_t launch_bwd_bf16_varlen(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                                  const float* m, const uint16_t* dout, float* dq, float* dk, float* dv,
                                  float* drb, float* workspace, const int* cu, int nseq, int H, int Hkv,
                                  int Ttot, int max_T, int d, hipStream_t stream);

// Single-token decode: q, o [B][H][d], k, v [B][Hkv][Tcap][d] of which the first T rows are
// valid, m [B][H] or nullptr, rb [H][d] or nullptr; workspace: decode_workspace_bytes bytes.
int decode_max_T();
size_t decode_workspace_bytes(int B, int H, int T, int d);
hipError_t launch_decode(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                         uint16_t* o, float* m, float* workspace,
                         int B, int H, int Hkv, int T, int Tcap, int d, hipStream_t stream);

// The library's own decode scratch (a file-scope device array, one copy per GPU): its size,
// and its device address on the current device (looked up on the first call per device).
size_t decode_static_bytes();
hipError_t decode_static_scratch(float** out);

// MFMA-only diagnostic: operands = at least 1 MiB of bf16 on the device, ticks = 3 x u64 on the device
hipError_t launch_diag_mfma(const void* operands, int iters, unsigned long long* ticks, hipStream_t stream);
double diag_mfma_flop(int iters);
// read-only streaming diagnostic: every 16-byte word of [data, data + bytes) is loaded once
hipError_t launch_diag_stream(const void* data, size_t bytes, unsigned int* sink, hipStream_t stream);

}  // namespace sb
