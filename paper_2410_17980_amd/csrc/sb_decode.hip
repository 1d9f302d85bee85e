// Single-token decode: one new query per (batch entry, head) against a cache of T keys
// and values, all of them visible (the last row of Eq. 1 on the extended sequence).
//
// The work is one pass over K and V (2*T*d*2 bytes per kv head) with ~1 FLOP per byte:
// bound by HBM bandwidth, so it runs on the vector ALU with coalesced 16-byte loads and
// is split over the keys to fill the chip ("split-KV").  Stick-breaking partial results
// combine without any rescaling by a maximum: a chunk of keys processed on its own gives
//     O_s = sum_i A_s[i] v_i   with the chunk-local weights A_s (Eq. 2 inside the chunk),
//     a_s = sum_i softplus(z_i)                      (minus the log of what the chunk leaves),
// and the exact output is  sum_s exp(-sum_{s' nearer than s} a_s') O_s  (the farther
// chunk's log-weights are shifted by what the nearer chunks took; Eq. 2).
//
//   decode_partial_kernel  grid (chunk, kv head, block of query heads).  Logits for the
//       chunk (a row of K is read once for all query heads of the group), base-2
//       softplus, suffix sums over the chunk, weights, weighted sum of the V rows.
//   decode_combine_kernel  one workgroup per (batch entry, query head): suffix sums of the
//       a_s over the chunks, O = sum_s 2^-A_s O_s, optional remainder bias, store.
#include <mutex>
#include <type_traits>

#include "../../include/sb_attn.h"
#include "sb_kernels.h"
#include "sb_mma.h"

namespace sb {
namespace {

constexpr int DEC_THREADS = 256;
constexpr int DEC_MAXCHUNKS = 256;     // chunks per head: the combine kernel gives each a thread
constexpr int DEC_CMAX = 2048;         // keys per chunk at most (logits of a chunk live in LDS)
constexpr int DEC_GT = 4;              // query heads of a group handled by one workgroup

__device__ __forceinline__ float bf_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

// sum of v over the aligned group of N lanes (N = 4, 8 or 16) this lane belongs to, in every
// lane of the group, with data-parallel-primitive adds (no LDS traffic): neighbours inside
// quads, then the mirrored half row and the mirrored row (all lanes of a quad already hold
// the same value then, so mirroring reaches the other quads' sum)
template <int N> __device__ __forceinline__ float group_sum(float v)
{
    auto dpp = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x),
                                                                     decltype(ctrl)::value, 0xf, 0xf, false));
    };
    v += dpp(v, std::integral_constant<int, 0xB1>{});              // quad_perm [1,0,3,2]
    v += dpp(v, std::integral_constant<int, 0x4E>{});              // quad_perm [2,3,0,1]
    if (N >= 8) v += dpp(v, std::integral_constant<int, 0x141>{}); // row_half_mirror
    if (N >= 16) v += dpp(v, std::integral_constant<int, 0x140>{}); // row_mirror
    return v;
}

// sum over the 256 threads' values v of all threads with a HIGHER thread index (exclusive
// suffix sum), and the total in `total`.  red: 4 floats of LDS; contains a barrier.
__device__ __forceinline__ float block_suffix_excl(float v, float* red, float& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float y = __shfl_down(inc, off);
        if (lane + off < 64) inc += y;
    }
    __syncthreads();                       // red may still be read from the call before
    if (lane == 0) red[wave] = inc;        // the wave's total
    __syncthreads();
    float above = 0.0f, tot = 0.0f;
#pragma unroll
    for (int w = 0; w < DEC_THREADS / 64; ++w) {
        const float t = red[w];
        tot += t;
        if (w > wave) above += t;
    }
    total = tot;
    return inc - v + above;
}

template <int D, int GT>
__global__ void __launch_bounds__(DEC_THREADS)
decode_partial_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                      const uint16_t* __restrict__ v, float* __restrict__ part_o, float* __restrict__ part_a,
                      int T, int Tcap, int H, int G, int C, int nchunk)
{
    constexpr int LPR = D / 8;             // lanes per row (16 B each)
    constexpr int RPI = 64 / LPR;          // rows per wave-wide load
    constexpr int RSTEP = RPI * (DEC_THREADS / 64);
    constexpr int U = 4;                   // rows in flight per lane
    extern __shared__ float zs[];          // [GT][C]: logits (base 2), then weights
    __shared__ float red[DEC_THREADS / 64];
    __shared__ float ored[DEC_THREADS / 64][GT][D];

    const int chunk = blockIdx.x;
    const int bkv = blockIdx.y;            // batch entry * Hkv + kv head
    const int g0 = blockIdx.z * GT;        // first query head (inside the group) of this workgroup
    const int Hkv = H / G;
    const int b = bkv / Hkv, hkv = bkv % Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPR, rw = lane / LPR;
    const int k0 = chunk * C, k1 = min(T, k0 + C), n = k1 - k0;
    const long kvbase = (long)bkv * Tcap * D;
    const float c2 = SB_LOG2E / sqrtf((float)D);

    // ---- logits: z[g][key] = q_g . k_key * log2(e) / sqrt(d)
    float qf[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        const bool live = g0 + g < G;
        const long hq = (long)b * H + hkv * G + min(g0 + g, G - 1);
        const u32x4 w = *reinterpret_cast<const u32x4*>(q + hq * D + 8 * sub);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            qf[g][2 * e] = live ? bf_lo(w[e]) * c2 : 0.0f;
            qf[g][2 * e + 1] = live ? bf_hi(w[e]) * c2 : 0.0f;
        }
    }
    for (int r0 = wave * RPI + rw; r0 < n; r0 += U * RSTEP) {
        u32x4 kw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = k0 + min(r0 + u * RSTEP, n - 1);
            kw[u] = *reinterpret_cast<const u32x4*>(k + kvbase + (long)row * D + 8 * sub);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) { kf[2 * e] = bf_lo(kw[u][e]); kf[2 * e + 1] = bf_hi(kw[u][e]); }
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) s += qf[g][e] * kf[e];
                s = group_sum<LPR>(s);
                if (sub == 0 && r0 + u * RSTEP < n) zs[g * C + r0 + u * RSTEP] = s;
            }
        }
    }
    __syncthreads();

    // ---- weights inside the chunk: w[i] = 2^(x_i - sum_{i' >= i} sp2(x_i'))  (Eq. 2).
    // Two sweeps over consecutive keys per thread: totals, a suffix scan of the totals over
    // the threads, then the weights (the softplus is evaluated again rather than kept).
    // With one query head the whole workgroup scans; with GT = 4 each wave takes one head
    // and no barrier is needed in between.
    {
        const int nthr = GT == 1 ? DEC_THREADS : 64;           // threads that share one head's scan
        const int g = GT == 1 ? 0 : wave;
        const int t = GT == 1 ? tid : lane;
        const int E = (C + nthr - 1) / nthr;                   // consecutive keys per thread
        float* z = zs + g * C;
        float mine = 0.0f;
        for (int e = 0; e < E; ++e) {
            const int i = t * E + e;
            if (i < n) mine += sp2(z[i]);
        }
        float total, run;
        if constexpr (GT == 1) {
            run = block_suffix_excl(mine, red, total);         // sp2 of all keys after this thread's
        } else {
            float inc = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float y = __shfl_down(inc, off);
                if (lane + off < 64) inc += y;
            }
            total = __shfl(inc, 0);
            run = inc - mine;
        }
        for (int e = E - 1; e >= 0; --e) {
            const int i = t * E + e;
            if (i < n) {
                const float x = z[i];
                run += sp2(x);
                z[i] = fast_exp2(x - run);
            }
        }
        if (t == 0 && g0 + g < G) {
            const long hq = (long)b * H + hkv * G + g0 + g;
            part_a[hq * nchunk + chunk] = total;
        }
    }
    __syncthreads();

    // ---- O_s[g][c] = sum_key w[g][key] V[key][c]
    float acc[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.0f;
    for (int r0 = wave * RPI + rw; r0 < n; r0 += U * RSTEP) {
        u32x4 vw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = k0 + min(r0 + u * RSTEP, n - 1);
            vw[u] = *reinterpret_cast<const u32x4*>(v + kvbase + (long)row * D + 8 * sub);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = r0 + u * RSTEP;
            float vf[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) { vf[2 * e] = bf_lo(vw[u][e]); vf[2 * e + 1] = bf_hi(vw[u][e]); }
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const float w = i < n ? zs[g * C + i] : 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] += w * vf[e];
            }
        }
    }
    // the lanes of a wave that hold the same columns, then the four waves
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float s = acc[g][e];
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) s += __shfl_xor(s, off);
            if (rw == 0) ored[wave][g][8 * sub + e] = s;
        }
    __syncthreads();
    for (int idx = tid; idx < GT * D; idx += DEC_THREADS) {
        const int g = idx / D, c = idx % D;
        if (g0 + g < G) {
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < DEC_THREADS / 64; ++w) s += ored[w][g][c];
            const long hq = (long)b * H + hkv * G + g0 + g;
            part_o[(hq * nchunk + chunk) * D + c] = s;
        }
    }
}

template <int D>
__global__ void __launch_bounds__(DEC_THREADS)
decode_combine_kernel(const float* __restrict__ part_o, const float* __restrict__ part_a,
                      const uint16_t* __restrict__ rb, uint16_t* __restrict__ o, float* __restrict__ m,
                      int H, int nchunk)
{
    constexpr int NV = D / 4;              // a thread adds four columns of every NG-th chunk
    constexpr int NG = DEC_THREADS / NV;
    __shared__ float red[DEC_THREADS / 64];
    __shared__ float ws[DEC_MAXCHUNKS];
    __shared__ float ored[NG][D];
    const long bh = blockIdx.x;
    const int tid = threadIdx.x;
    // chunk `tid` is shifted by everything the nearer (higher) chunks took
    const float a = tid < nchunk ? part_a[bh * nchunk + tid] : 0.0f;
    float total;
    const float above = block_suffix_excl(a, red, total);
    ws[tid] = fast_exp2(-above);
    __syncthreads();
    const int c4 = tid % NV, grp = tid / NV;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    const float4* po = reinterpret_cast<const float4*>(part_o + bh * (long)nchunk * D) + c4;
#pragma unroll 4
    for (int ch = grp; ch < nchunk; ch += NG) {
        const float4 p = po[(long)ch * NV];
        const float w = ws[ch];
        s0 += w * p.x; s1 += w * p.y; s2 += w * p.z; s3 += w * p.w;
    }
    ored[grp][4 * c4] = s0; ored[grp][4 * c4 + 1] = s1; ored[grp][4 * c4 + 2] = s2; ored[grp][4 * c4 + 3] = s3;
    __syncthreads();
    if (tid < D) {
        float r = 0.0f;
#pragma unroll
        for (int g = 0; g < NG; ++g) r += ored[g][tid];
        // remainder bias (Appendix C): what no key took goes to the head's embedding
        if (rb) r += fast_exp2(-total) * bf_lo((uint32_t)rb[(bh % H) * D + tid]);
        const __bf16 val = (__bf16)r;
        o[bh * D + tid] = __builtin_bit_cast(uint16_t, val);
    }
    if (m && tid == 0) m[bh] = -total * SB_LN2;
}

template <int D>
hipError_t launch_d(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                    uint16_t* o, float* m, float* workspace, int B, int H, int Hkv, int T, int Tcap,
                    int C, int nchunk, hipStream_t stream)
{
    const int G = H / Hkv;
    float* part_a = workspace;
    float* part_o = workspace + (((long)B * H * nchunk + 3) & ~3L);
    const dim3 grid((unsigned)nchunk, (unsigned)(B * Hkv), (unsigned)((G + DEC_GT - 1) / DEC_GT));
    if (G == 1)
        hipLaunchKernelGGL((decode_partial_kernel<D, 1>), dim3((unsigned)nchunk, (unsigned)(B * Hkv), 1u),
                           dim3(DEC_THREADS), sizeof(float) * C, stream, q, k, v, part_o, part_a, T, Tcap, H, G, C, nchunk);
    else
        hipLaunchKernelGGL((decode_partial_kernel<D, DEC_GT>), grid, dim3(DEC_THREADS), sizeof(float) * DEC_GT * C, stream,
                           q, k, v, part_o, part_a, T, Tcap, H, G, C, nchunk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((decode_combine_kernel<D>), dim3((unsigned)(B * H)), dim3(DEC_THREADS), 0, stream,
                       part_o, part_a, rb, o, m, H, nchunk);
    return hipGetLastError();
}

// keys per chunk: as few as keep the chunk count within the combine kernel's reach; larger
// while the launch would still have more than a thousand workgroups (measured: the fixed
// cost per workgroup outweighs finer balance beyond that)
int chunk_keys(int BHkv, int T)
{
    int C = 64;
    while ((T + C - 1) / C > DEC_MAXCHUNKS) C *= 2;
    while ((long)((T + C - 1) / C) * BHkv > 1024 && C < 1024) C *= 2;
    return C;
}

// Scratch of the entry point that allocates nothing: every GPU the library runs on holds its
// own copy of this array, at its own address, until the process ends.  Host code never uses
// the array's name as a pointer: the device address is looked up once per device.
constexpr size_t DEC_STATIC_BYTES = SB_DECODE_STATIC_BYTES;
static __device__ __align__(256) unsigned char scratch[DEC_STATIC_BYTES];

constexpr int DEC_MAX_DEVICES = 64;
std::mutex scratch_lock;
void* scratch_ptr[DEC_MAX_DEVICES];        // device address of `scratch`, per device, once known

}  // namespace

int decode_max_T() { return DEC_MAXCHUNKS * DEC_CMAX; }

size_t decode_static_bytes() { return DEC_STATIC_BYTES; }

hipError_t decode_static_scratch(float** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= DEC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(scratch_lock);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *out = static_cast<float*>(scratch_ptr[dev]);
    return hipSuccess;
}

size_t decode_workspace_bytes(int B, int H, int T, int d)
{
    // the chunk count depends on the kv head count only through chunk_keys' second loop,
    // which can only lower it: size for the largest
    const int C = chunk_keys(1, T);
    const size_t nchunk = (size_t)(T + C - 1) / C;
    return sizeof(float) * ((((size_t)B * H * nchunk + 3) & ~(size_t)3) + (size_t)B * H * nchunk * d);
}

hipError_t launch_decode(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                         uint16_t* o, float* m, float* workspace,
                         int B, int H, int Hkv, int T, int Tcap, int d, hipStream_t stream)
{
    if (B * Hkv > 65535) return hipErrorInvalidValue;
    const int C = chunk_keys(B * Hkv, T);
    if (C > DEC_CMAX) return hipErrorInvalidValue;
    const int nchunk = (T + C - 1) / C;
    if (d == 32) return launch_d<32>(q, k, v, rb, o, m, workspace, B, H, Hkv, T, Tcap, C, nchunk, stream);
    if (d == 64) return launch_d<64>(q, k, v, rb, o, m, workspace, B, H, Hkv, T, Tcap, C, nchunk, stream);
    return launch_d<128>(q, k, v, rb, o, m, workspace, B, H, Hkv, T, Tcap, C, nchunk, stream);
}

}  // namespace sb
