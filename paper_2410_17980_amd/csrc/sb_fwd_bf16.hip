// bf16 forward of causal stick-breaking attention on the gfx950 matrix cores.
//
// Work split.  A workgroup (4 wavefronts) owns 128 query rows of one (batch,
// head); each wavefront owns 32 of them.  Key/value tiles of 64 rows are staged
// in LDS (double buffered) and swept from the diagonal towards key 0, which is
// the order Algorithm 1 prescribes: the weight of key i needs the sum of
// softplus(z) over the keys between i and the query (Eq. 2), so that sum is
// carried per query row from tile to tile (the vector `a` of Algorithm 1).
//
// Layout inside a wavefront.  Logits are formed transposed, S^T = K Q^T, with
// the 32x32x16 bf16 MFMA: A operand = 32 key rows from LDS, B operand = the
// wave's 32 query rows held in registers for the whole kernel.  In the MFMA
// accumulator a lane then owns ONE query column (lane % 32) and 16 key rows.
// The LDS row fed to MFMA row rho is chosen so that those 16 keys are
// consecutive: lanes 0-31 hold keys 0..15 of the 32-key subtile, lanes 32-63
// keys 16..31.  The right-to-left cumulative sum of softplus is therefore a
// serial add inside the lane plus one exchange with the partner lane
// (v_permlane32_swap), and the row total for the carry falls out of the scan.
// The weights feed the second MFMA (O += A V) straight from registers: the
// accumulator's per-lane key order is also a valid K-dimension order for the
// A operand, and V is read from LDS with the transposing load
// (ds_read_b64_tr_b16) in that same key order.
//
// Arithmetic.  Everything between the two MFMAs is fp32 in the base-2 domain:
// x = z*log2(e), sp2(x) = log2(1 + 2^x) (v_exp_f32 / v_log_f32 are base 2),
// A = 2^(x - cumsum sp2 - carry).  log(1-sigma(z)) = -softplus(z) and
// log(sigma(z)) = z - softplus(z), so no product of probabilities is ever
// formed.  Where 2^x overflows fp32 (x > 128) softplus is x itself; see sp2().
#include "sb_kernels.h"

namespace sb {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define SB_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int BQ = 128;          // query rows per workgroup
constexpr int BK = 64;           // key rows per LDS tile
constexpr int NTHREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

template <int D> struct FwdCfg {
    static constexpr int KROW = D * 2;          // bytes per K row in LDS (xor-swizzled 16 B chunks)
    static constexpr int VROW = D * 2 + 64;     // bytes per V row in LDS (padded: rows 16 banks apart)
    static constexpr int KTILE = BK * KROW;
    static constexpr int VTILE = BK * VROW;
    static constexpr int STAGE = KTILE + VTILE; // one buffer
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int CHUNKS_PER_ROW = D / 8;                 // 16 B chunks
    static constexpr int CHUNKS_PER_THREAD = BK * CHUNKS_PER_ROW / NTHREADS;
};

// xor mask for the 16 B chunk index of K row `key`: makes the 16 rows that one
// quarter-wave reads (keys {0..7} and {16..23} (+8) of a subtile) hit 16
// different 4-bank groups.
template <int D> __device__ __forceinline__ int k_swizzle(int key)
{
    if (D == 128) return (key & 7) | (((key >> 4) & 1) << 3);
    return ((key >> 1) & 3) | (((key >> 4) & 1) << 2);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// log2(1 + 2^x).  For x > 128 the power overflows to +inf and so does the log;
// the true value is then x itself to fp32 precision, and the median of
// (log, x, 128) picks it.  Below that the log lies between x and 128 and wins.
__device__ __forceinline__ float sp2(float x)
{
    return __builtin_amdgcn_fmed3f(fast_log2(1.0f + fast_exp2(x)), x, 128.0f);
}

template <int D, bool WRITE_M>
__global__ void __launch_bounds__(NTHREADS, 2)
fwd_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ m,
                int T, int BH, int nqb)
{
    using C = FwdCfg<D>;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // workgroup -> (head, query block).  Consecutive workgroup ids go round the 8
    // XCDs, so give every XCD its own heads (K/V of a head stay in one L2) and
    // walk a head's query blocks longest-first.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const long bh = xcd + 8L * (slot / nqb);
    const int qb = nqb - 1 - (slot % nqb);
    if (bh >= BH) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31;          // query column inside the wave / MFMA row index
    const int hh = lane >> 5;         // which half of the wave
    const int q0 = qb * BQ + wave * 32;
    const bool wave_live = q0 < T;

    const uint16_t* Qg = q + bh * (long)T * D;
    const uint16_t* Kg = k + bh * (long)T * D;
    const uint16_t* Vg = v + bh * (long)T * D;

    // ---- B operand of S^T = K Q^T: Q[q0+n][16s + 8hh .. +7], s = 0..D/16-1
    bf16x8 qf[D / 16];
    {
        const int jq = min(q0 + n, T - 1);
        const u32x4* src = reinterpret_cast<const u32x4*>(Qg + (long)jq * D + 8 * hh);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            u32x4 w = src[2 * s];
            qf[s] = __builtin_bit_cast(bf16x8, w);
        }
    }

    // ---- per-lane LDS byte offsets
    // K (A operand): MFMA row rho = n must carry key 16*((rho>>2)&1) + 4*(rho>>3) + (rho&3)
    const int key_l = 16 * ((n >> 2) & 1) + 4 * (n >> 3) + (n & 3);
    int koff[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
        koff[s] = key_l * C::KROW + (((2 * s + hh) ^ k_swizzle<D>(key_l)) << 4);
    // V (B operand through the transposing load): quarter-wave gg = lane/16 reads
    // rows 16*(gg>>1) + (i>>2), columns 16*(gg&1) + 4*(i&3), i = lane%16
    const int gg = lane >> 4, li = lane & 15;
    const int voff = (16 * (gg >> 1) + (li >> 2)) * C::VROW + (16 * (gg & 1) + 4 * (li & 3)) * 2;

    // ---- staging map: thread -> CHUNKS_PER_THREAD 16 B chunks of the K tile and of the V tile
    u32x4 kst[C::CHUNKS_PER_THREAD], vst[C::CHUNKS_PER_THREAD];
    auto stage_load = [&](int kt) {
#pragma unroll
        for (int i = 0; i < C::CHUNKS_PER_THREAD; ++i) {
            const int id = tid + i * NTHREADS;
            const int row = id / C::CHUNKS_PER_ROW, c = id % C::CHUNKS_PER_ROW;
            const long gr = min(kt * BK + row, T - 1);
            kst[i] = *reinterpret_cast<const u32x4*>(Kg + gr * D + c * 8);
            vst[i] = *reinterpret_cast<const u32x4*>(Vg + gr * D + c * 8);
        }
    };
    auto stage_store = [&](int buf) {
        char* kb = smem + buf * C::STAGE;
        char* vb = kb + C::KTILE;
#pragma unroll
        for (int i = 0; i < C::CHUNKS_PER_THREAD; ++i) {
            const int id = tid + i * NTHREADS;
            const int row = id / C::CHUNKS_PER_ROW, c = id % C::CHUNKS_PER_ROW;
            *reinterpret_cast<u32x4*>(kb + row * C::KROW + ((c ^ k_swizzle<D>(row)) << 4)) = kst[i];
            *reinterpret_cast<u32x4*>(vb + row * C::VROW + (c << 4)) = vst[i];
        }
    };

    f32x16 oacc[D / 32];
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[b][r] = 0.0f;
    float a = 0.0f;   // carried sum of sp2 over all keys right of the current subtile (this lane's query)

    const float c2 = LOG2E / sqrtf((float)D);

    // one 32-key subtile: logits, weights, accumulate
    auto subtile = [&](const char* kb, const char* vb, int u, bool diag) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(kb + u * 32 * C::KROW + koff[s]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), qf[s], acc, 0, 0, 0);
        }
        // acc[r] <-> key (tile base) + 32u + 16hh + r, query q0 + n
        float x[16], cs[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = acc[r] * c2;
        if (diag) {
            // same 32-row block on both axes: key index 16hh + r is valid iff < n
#pragma unroll
            for (int r = 0; r < 16; ++r) x[r] = (16 * hh + r < n) ? x[r] : -INFINITY;
        }
        float run = 0.0f;
#pragma unroll
        for (int r = 15; r >= 0; --r) {
            run += sp2(x[r]);
            cs[r] = run;                       // sum over this lane's keys r..15
        }
        // totals of both half-waves for this query: lanes < 32 get (own, partner), lanes >= 32 (partner, own)
        auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(int, run), __builtin_bit_cast(int, run), false, false);
        const float tot_lo = __builtin_bit_cast(float, (int)sw[0]);
        const float tot_hi = __builtin_bit_cast(float, (int)sw[1]);
        const float off = a + (hh == 0 ? tot_hi : 0.0f);
        a += tot_lo + tot_hi;
        bf16x8 pa[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float w = fast_exp2((x[r] - off) - cs[r]);
            pa[r >> 3][r & 7] = (__bf16)w;
        }
        // O[q][dcol] += sum_keys A[q][key] V[key][dcol]; K-dim index 8g+e <-> key 16g + 8s + e
#pragma unroll
        for (int b = 0; b < D / 32; ++b) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const char* vp = vb + (u * 32 + 8 * s) * C::VROW + b * 64 + voff;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SB_LDS(s16x4, vp));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SB_LDS(s16x4, vp + 4 * C::VROW));
                const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa[s], vf, oacc[b], 0, 0, 0);
            }
        }
    };

    // ---- sweep over key tiles, right to left
    const int jmax = min(T, qb * BQ + BQ) - 1;          // last live query row of the workgroup
    const int ntile = (jmax + BK - 1) / BK;              // tiles covering keys 0 .. jmax-1
    if (ntile > 0) {
        stage_load(ntile - 1);
        stage_store(0);
    }
    __syncthreads();
    for (int it = 0; it < ntile; ++it) {
        const int kt = ntile - 1 - it;
        const int buf = it & 1;
        const char* kb = smem + buf * C::STAGE;
        const char* vb = kb + C::KTILE;
        const bool more = it + 1 < ntile;
        if (more) stage_load(kt - 1);
        {
            const int k0 = kt * BK + 32;
            if (wave_live && k0 <= q0) subtile(kb, vb, 1, k0 == q0);
        }
        if (more) stage_store(buf ^ 1);
        {
            const int k0 = kt * BK;
            if (wave_live && k0 <= q0) subtile(kb, vb, 0, k0 == q0);
        }
        __syncthreads();
    }

    // ---- store.  oacc[b][r] is query row 8*(r/4) + 4*hh + r%4, column 32b + n.
    if (wave_live) {
        uint16_t* Og = o + bh * (long)T * D;
#pragma unroll
        for (int b = 0; b < D / 32; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = q0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                if (row < T) {
                    const __bf16 val = (__bf16)oacc[b][r];
                    Og[(long)row * D + 32 * b + n] = __builtin_bit_cast(uint16_t, val);
                }
            }
        }
        if (WRITE_M && hh == 0 && q0 + n < T) m[bh * (long)T + q0 + n] = -a * LN2;
    }
}

template <int D, bool WRITE_M>
hipError_t launch_one(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o, float* m,
                      int BH, int T, hipStream_t stream)
{
    using C = FwdCfg<D>;
    auto kern = fwd_bf16_kernel<D, WRITE_M>;
    static bool attr_done = false;   // the attribute is per function, set once per process
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int nqb = (T + BQ - 1) / BQ;
    const long blocks = 8L * ((BH + 7) / 8) * nqb;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), C::LDS_BYTES, stream,
                       q, k, v, o, m, T, BH, nqb);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o,
                           float* m, int B, int H, int T, int d, hipStream_t stream)
{
    const int BH = B * H;
    if (d == 64)
        return m ? launch_one<64, true>(q, k, v, o, m, BH, T, stream)
                 : launch_one<64, false>(q, k, v, o, m, BH, T, stream);
    return m ? launch_one<128, true>(q, k, v, o, m, BH, T, stream)
             : launch_one<128, false>(q, k, v, o, m, BH, T, stream);
}

}  // namespace sb
