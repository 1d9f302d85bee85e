// bf16 backward of causal stick-breaking attention on the gfx950 matrix cores
// (Eq. 4 evaluated tile by tile as in Algorithm 2).
//
// A workgroup (4 wavefronts) owns 128 query rows of one (batch, head), each
// wavefront 32 of them, and sweeps the key tiles from key 0 towards the
// diagonal.  Per query row it carries
//   a2 : sum of sp2 = log2(1+2^x) over the keys from the current position to
//        the query (starts at -m/ln2, the total saved by the forward, and is
//        reduced tile by tile: Algorithm 2's "a <- a - sum L"), and
//   b  : sum of G = A * (dO . v) over the keys already passed (Algorithm 2's b).
//
// Per 32-key subtile, in the same transposed register layout as the forward
// (a lane owns one query column and 16 consecutive keys):
//   S^T = K Q^T, P^T = V dO^T                      (MFMA, K and V rows from LDS)
//   A   = 2^(x - cumsum<- sp2 - carry)             (as the forward)
//   G   = A * P
//   dZ  = G - sigma(z) * (cumsum-> G + b),  sigma(z) = 2^(x - sp2(x))
//   dQ += (dZ/sqrt d) K                            (MFMA, dZ from registers, K through
//                                                   the transposing LDS load)
//   dV_tile = A^T dO, dK_tile = (dZ/sqrt d)^T Q    (MFMA; A and dZ are turned into
//                                                   A-operand layout through a small per-wave
//                                                   LDS scratch: written row-wise, read back with
//                                                   the transposing load)
// and the dK/dV tiles are added to HBM with fp32 atomics, since every later
// query block contributes to the same key rows.
#include "sb_kernels.h"

namespace sb {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define SB_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int BQ = 128;
constexpr int BK = 64;
constexpr int NTHREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;

template <int D> struct BwdCfg {
    static constexpr int ROWB = D * 2 + 16;            // padded row, K / V / Q / dO tiles
    static constexpr int TROW = 80;                    // scratch row: 32 bf16 + pad
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = K_OFF + BK * ROWB;
    static constexpr int Q_OFF = V_OFF + BK * ROWB;
    static constexpr int G_OFF = Q_OFF + BQ * ROWB;    // dO block
    static constexpr int T_OFF = G_OFF + BQ * ROWB;    // per-wave transposition scratch
    static constexpr int T_WAVE = 2 * 32 * TROW;
    static constexpr int LDS_BYTES = T_OFF + 4 * T_WAVE;
    static constexpr int CHUNKS_PER_ROW = D / 8;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float sp2(float x)
{
    // log2(1 + 2^x); where 2^x overflows the value is x itself (median picks it)
    return __builtin_amdgcn_fmed3f(fast_log2(1.0f + fast_exp2(x)), x, 128.0f);
}

__device__ __forceinline__ bf16x8 tr_pair(const char* p, int row_bytes4)
{
    // two transposing loads: K-dim elements 0..3 from p, 4..7 from four rows further
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SB_LDS(s16x4, p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SB_LDS(s16x4, p + row_bytes4));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__global__ void __launch_bounds__(256) fill_zero_kernel(float4* p, long n4)
{
    const long stride = (long)gridDim.x * blockDim.x;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

template <int D>
__global__ void __launch_bounds__(NTHREADS, 1)
bwd_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                const uint16_t* __restrict__ v, const float* __restrict__ m,
                const uint16_t* __restrict__ dout, float* __restrict__ dq,
                float* __restrict__ dk, float* __restrict__ dv, int T, int BH, int nqb)
{
    using C = BwdCfg<D>;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const long bh = xcd + 8L * (slot / nqb);
    const int qb = nqb - 1 - (slot % nqb);
    if (bh >= BH) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int gg = lane >> 4, li = lane & 15;
    const int q0 = qb * BQ + wave * 32;
    const bool wave_live = q0 < T;

    const long base = bh * (long)T * D;
    const uint16_t* Qg = q + base;
    const uint16_t* Kg = k + base;
    const uint16_t* Vg = v + base;
    const uint16_t* Gg = dout + base;

    // ---- the workgroup's Q and dO rows into LDS (rows past T: Q clamped, dO zero)
    for (int id = tid; id < BQ * C::CHUNKS_PER_ROW; id += NTHREADS) {
        const int row = id / C::CHUNKS_PER_ROW, c = id % C::CHUNKS_PER_ROW;
        const int j = qb * BQ + row;
        const long gr = min(j, T - 1);
        u32x4 qv = *reinterpret_cast<const u32x4*>(Qg + gr * D + c * 8);
        u32x4 gv = *reinterpret_cast<const u32x4*>(Gg + gr * D + c * 8);
        if (j >= T) gv = u32x4{0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(smem + C::Q_OFF + row * C::ROWB + c * 16) = qv;
        *reinterpret_cast<u32x4*>(smem + C::G_OFF + row * C::ROWB + c * 16) = gv;
    }

    // ---- B operands held in registers: Q and dO rows of this lane's query
    bf16x8 qf[D / 16], gf[D / 16];
    {
        const int j = q0 + n;
        const long jq = min(j, T - 1);
        const u32x4* qs = reinterpret_cast<const u32x4*>(Qg + jq * D + 8 * hh);
        const u32x4* gs = reinterpret_cast<const u32x4*>(Gg + jq * D + 8 * hh);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            u32x4 a = qs[2 * s], g = gs[2 * s];
            if (j >= T) g = u32x4{0u, 0u, 0u, 0u};
            qf[s] = __builtin_bit_cast(bf16x8, a);
            gf[s] = __builtin_bit_cast(bf16x8, g);
        }
    }

    // ---- per-lane LDS byte offsets
    const int key_l = 16 * ((n >> 2) & 1) + 4 * (n >> 3) + (n & 3);     // LDS row feeding MFMA row n
    const int a_off = key_l * C::ROWB + hh * 16;                        // A-operand reads of K / V rows
    const int tr_col = (16 * (gg & 1) + 4 * (li & 3)) * 2;
    const int kt_off = (16 * (gg >> 1) + (li >> 2)) * C::ROWB + tr_col; // transposing reads of the K tile
    const int qt_off = (32 * wave + 8 * (gg >> 1) + (li >> 2)) * C::ROWB + tr_col;   // ... of Q / dO rows
    char* const scr = smem + C::T_OFF + wave * C::T_WAVE;               // [2][32][TROW]
    const int sw_off = n * C::TROW + 32 * hh;                           // scratch write (row = query)
    const int st_off = (8 * (gg >> 1) + (li >> 2)) * C::TROW + tr_col;  // scratch transposing read

    f32x16 dqacc[D / 32];
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) dqacc[b][r] = 0.0f;

    const float c2 = LOG2E / sqrtf((float)D);
    const float scale = 1.0f / sqrtf((float)D);
    // a2: sum of sp2 over the keys from the sweep position up to the query
    float a2 = -m[bh * (long)T + min(q0 + n, T - 1)] * LOG2E;
    float bsum = 0.0f;

    float* const dKg = dk + base;
    float* const dVg = dv + base;

    auto subtile = [&](int kbase, int u, bool diag) {
        const char* kb = smem + C::K_OFF + u * 32 * C::ROWB;
        const char* vb = smem + C::V_OFF + u * 32 * C::ROWB;
        f32x16 sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[r] = 0.0f; pacc[r] = 0.0f; }
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            const u32x4 kw = *reinterpret_cast<const u32x4*>(kb + a_off + s * 32);
            const u32x4 vw = *reinterpret_cast<const u32x4*>(vb + a_off + s * 32);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kw), qf[s], sacc, 0, 0, 0);
            pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw), gf[s], pacc, 0, 0, 0);
        }
        // element (r): key kbase + 32u + 16hh + r, query q0 + n
        float x[16], sp[16], cs[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = sacc[r] * c2;
        if (diag) {
#pragma unroll
            for (int r = 0; r < 16; ++r) x[r] = (16 * hh + r < n) ? x[r] : -INFINITY;
        }
        float run = 0.0f;
#pragma unroll
        for (int r = 15; r >= 0; --r) {
            sp[r] = sp2(x[r]);
            run += sp[r];
            cs[r] = run;
        }
        auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(int, run), __builtin_bit_cast(int, run), false, false);
        const float tot_lo = __builtin_bit_cast(float, (int)sw[0]);
        const float tot_hi = __builtin_bit_cast(float, (int)sw[1]);
        a2 -= tot_lo + tot_hi;                               // now: keys right of this subtile
        const float off = a2 + (hh == 0 ? tot_hi : 0.0f);
        float g[16], pre[16];
        bf16x8 pa[2], pz[2];
        float grun = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float w = fast_exp2((x[r] - off) - cs[r]);  // A
            pa[r >> 3][r & 7] = (__bf16)w;
            g[r] = w * pacc[r];                               // G = A * (dO . v)
            grun += g[r];
            pre[r] = grun;                                    // inclusive prefix inside the lane
        }
        auto gw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(int, grun), __builtin_bit_cast(int, grun), false, false);
        const float g_lo = __builtin_bit_cast(float, (int)gw[0]);
        const float g_hi = __builtin_bit_cast(float, (int)gw[1]);
        const float boff = bsum + (hh == 1 ? g_lo : 0.0f);
        bsum += g_lo + g_hi;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float beta = fast_exp2(x[r] - sp[r]);       // sigma(z)
            const float dz = g[r] - beta * (pre[r] + boff);
            pz[r >> 3][r & 7] = (__bf16)(dz * scale);
        }

        // ---- dQ += dZ K : A operand from registers, K through the transposing load
#pragma unroll
        for (int b = 0; b < D / 32; ++b) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 kf = tr_pair(kb + (8 * s) * C::ROWB + b * 64 + kt_off, 4 * C::ROWB);
                dqacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pz[s], kf, dqacc[b], 0, 0, 0);
            }
        }

        // ---- A and dZ into A-operand layout [key][query] through the wave's scratch
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        *reinterpret_cast<bf16x8*>(scr + sw_off) = pa[0];
        *reinterpret_cast<bf16x8*>(scr + sw_off + 16) = pa[1];
        *reinterpret_cast<bf16x8*>(scr + 32 * C::TROW + sw_off) = pz[0];
        *reinterpret_cast<bf16x8*>(scr + 32 * C::TROW + sw_off + 16) = pz[1];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        bf16x8 at[2], zt[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            at[s2] = tr_pair(scr + (16 * s2) * C::TROW + st_off, 4 * C::TROW);
            zt[s2] = tr_pair(scr + (32 + 16 * s2) * C::TROW + st_off, 4 * C::TROW);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

        // ---- dV_tile = A^T dO, dK_tile = dZ^T Q ; rows = keys, added to HBM
        const int key0 = kbase + 32 * u;
#pragma unroll
        for (int b = 0; b < D / 32; ++b) {
            f32x16 va, ka;
#pragma unroll
            for (int r = 0; r < 16; ++r) { va[r] = 0.0f; ka[r] = 0.0f; }
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const bf16x8 gop = tr_pair(smem + C::G_OFF + (16 * s2) * C::ROWB + b * 64 + qt_off, 4 * C::ROWB);
                const bf16x8 qop = tr_pair(smem + C::Q_OFF + (16 * s2) * C::ROWB + b * 64 + qt_off, 4 * C::ROWB);
                va = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[s2], gop, va, 0, 0, 0);
                ka = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zt[s2], qop, ka, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                if (key < T) {
                    const long idx = (long)key * D + 32 * b + n;
                    atomicAdd(dVg + idx, va[r]);
                    atomicAdd(dKg + idx, ka[r]);
                }
            }
        }
    };

    // ---- sweep over key tiles, left to right
    const int jmax = min(T, qb * BQ + BQ) - 1;
    const int ntile = (jmax + BK - 1) / BK;
    for (int kt = 0; kt < ntile; ++kt) {
        __syncthreads();                                   // previous tile fully consumed
        for (int id = tid; id < BK * C::CHUNKS_PER_ROW; id += NTHREADS) {
            const int row = id / C::CHUNKS_PER_ROW, c = id % C::CHUNKS_PER_ROW;
            const long gr = min(kt * BK + row, T - 1);
            *reinterpret_cast<u32x4*>(smem + C::K_OFF + row * C::ROWB + c * 16) =
                *reinterpret_cast<const u32x4*>(Kg + gr * D + c * 8);
            *reinterpret_cast<u32x4*>(smem + C::V_OFF + row * C::ROWB + c * 16) =
                *reinterpret_cast<const u32x4*>(Vg + gr * D + c * 8);
        }
        __syncthreads();
        const int k0 = kt * BK;
        if (wave_live && k0 <= q0) subtile(k0, 0, k0 == q0);
        if (wave_live && k0 + 32 <= q0) subtile(k0, 1, k0 + 32 == q0);
    }

    // ---- dQ store: dqacc[b][r] is query row 8*(r/4) + 4*hh + r%4, column 32b + n
    if (wave_live) {
        float* dQg = dq + base;
#pragma unroll
        for (int b = 0; b < D / 32; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = q0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                if (row < T) dQg[(long)row * D + 32 * b + n] = dqacc[b][r];
            }
        }
    }
}

template <int D>
hipError_t launch_one(const uint16_t* q, const uint16_t* k, const uint16_t* v, const float* m,
                      const uint16_t* dout, float* dq, float* dk, float* dv,
                      int BH, int T, hipStream_t stream)
{
    using C = BwdCfg<D>;
    auto kern = bwd_bf16_kernel<D>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    // dk and dv are accumulated with atomics: clear them first (a kernel, not a
    // memset node, so the call stays safe under graph capture)
    const long n4 = (long)BH * T * D / 4;
    const int zb = (int)((n4 + 255) / 256 < 4096 ? (n4 + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(zb), dim3(256), 0, stream, reinterpret_cast<float4*>(dk), n4);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(zb), dim3(256), 0, stream, reinterpret_cast<float4*>(dv), n4);
    const int nqb = (T + BQ - 1) / BQ;
    const long blocks = 8L * ((BH + 7) / 8) * nqb;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), C::LDS_BYTES, stream,
                       q, k, v, m, dout, dq, dk, dv, T, BH, nqb);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, const float* m,
                           const uint16_t* dout, float* dq, float* dk, float* dv,
                           int B, int H, int T, int d, hipStream_t stream)
{
    const int BH = B * H;
    if (d == 64) return launch_one<64>(q, k, v, m, dout, dq, dk, dv, BH, T, stream);
    return launch_one<128>(q, k, v, m, dout, dq, dk, dv, BH, T, stream);
}

}  // namespace sb
