// bf16 backward of causal stick-breaking attention on the gfx950 matrix cores
// (Eq. 4 evaluated tile by tile; the per-tile steps are those of Algorithm 2).
//
// Two kernels instead of Algorithm 2's single query-stationary kernel with
// atomic adds into dK and dV.  The dependency that forces the paper's atomics is
// the cumulative sum over keys inside each query row; it is cut by saving, per
// query row and per 32-key subtile, the two carried scalars
//     ca = sum of sp2 over the keys to the right of the subtile (up to the query),
//     cb = sum of G = A*(dO.v) over the keys to the left of the subtile,
// (2 floats per 32x1 strip of the attention matrix).  With them any subtile can
// be recomputed on its own, so dK and dV are accumulated by a key-stationary
// kernel in registers and written once, with no atomics and no zero fill, and
// the result is bit-reproducible.
//
//   bwd_dq_kernel  (query-stationary, 128 query rows per workgroup, sweep from
//                   key 0 to the diagonal as Algorithm 2): recomputes A from m,
//                   forms G and dZ, accumulates dQ += (dZ/sqrt d) K, stores ca, cb.
//   bwd_dkv_kernel (key-stationary, 128 key rows per workgroup = 32 per wave,
//                   K and V rows held in registers, sweep over query blocks from
//                   the diagonal to the end): recomputes A, G, dZ from ca, cb and
//                   accumulates dV += A^T dO, dK += (dZ/sqrt d)^T Q.
//
// Register layout is the forward's: S^T = K Q^T and P^T = V dO^T with the
// 32x32x16 bf16 MFMA, a lane owns one query column and 16 consecutive keys, so
// both cumulative sums are serial inside the lane plus one exchange between the
// half-waves.  A and dZ feed the "query-major" product (dQ) straight from
// registers; for the "key-major" products (dK, dV) they are written to a small
// per-wave LDS scratch row-wise and read back with the transposing load.
#include "sb_kernels.h"
#include "sb_mma.h"

namespace sb {
namespace {

constexpr int NTHREADS = 256;
constexpr int BQ = 128;      // dq kernel: query rows per workgroup
constexpr int BK = 64;       // dq kernel: key rows per LDS tile
constexpr int BKW = 128;     // dkv kernel: key rows per workgroup (32 per wave)
constexpr int TROW = 80;     // scratch row: 32 bf16 + pad (rows stay 16 B aligned)

// ------------------------------------------------------------------ element-wise core
// One 32x32 subtile in the lane layout (query n; keys 16hh + r).
struct SubtileOut {
    bf16x8 pa[2];    // A, as MFMA operand (K-dim element e of half s <-> key 16hh + 8s + e)
    bf16x8 pz[2];    // dZ / sqrt(d), same layout
    float ca_right;  // sum of sp2 over the keys right of the subtile
    float g_tot;     // sum of G over the subtile's 32 keys
};

// sacc: q.k accumulator, pacc: dO.v accumulator.  cb: sum of G over the keys left
// of the subtile.  ca: sum of sp2 over the keys right of the subtile, or, with
// CA_INCLUDES_SUBTILE, over the subtile's own keys as well (Algorithm 2 carries
// that and subtracts the subtile's total before use).
template <bool CA_INCLUDES_SUBTILE>
__device__ __forceinline__ SubtileOut subtile_math(const f32x16& sacc, const f32x16& pacc, float ca,
                                                   float cb, float c2, float scale, int n, int hh, bool diag)
{
    SubtileOut out;
    float x[16], sp[16], cs[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = sacc[r] * c2;
    if (diag) {
        // same 32 rows on both axes: key 16hh + r is visible to query n iff it is smaller
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = (16 * hh + r < n) ? x[r] : -INFINITY;
    }
    float run = 0.0f;
#pragma unroll
    for (int r = 15; r >= 0; --r) {
        sp[r] = sp2(x[r]);
        run += sp[r];
        cs[r] = run;                                       // keys r..15 of this lane
    }
    float tot_lo, tot_hi;
    both_halves(run, tot_lo, tot_hi);
    const float car = CA_INCLUDES_SUBTILE ? ca - (tot_lo + tot_hi) : ca;
    out.ca_right = car;
    const float off = car + (hh == 0 ? tot_hi : 0.0f);
    float g[16], pre[16];
    float grun = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float w = fast_exp2((x[r] - off) - cs[r]);   // A (Eq. 2)
        out.pa[r >> 3][r & 7] = (__bf16)w;
        g[r] = w * pacc[r];                                // dL/dlogA = A * dL/dA
        grun += g[r];
        pre[r] = grun;                                     // inclusive prefix inside the lane
    }
    float g_lo, g_hi;
    both_halves(grun, g_lo, g_hi);
    out.g_tot = g_lo + g_hi;
    const float boff = cb + (hh == 1 ? g_lo : 0.0f);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float beta = fast_exp2(x[r] - sp[r]);        // sigma(z)
        const float dz = g[r] - beta * (pre[r] + boff);    // Eq. 4
        out.pz[r >> 3][r & 7] = (__bf16)(dz * scale);
    }
    return out;
}

// ------------------------------------------------------------------ dQ kernel
template <int D> struct DqCfg {
    static constexpr int ROW = D * 2;
    static constexpr int TILE = BK * ROW;
    static constexpr int STAGE = 2 * TILE;           // K tile + V tile
    static constexpr int LDS_BYTES = 2 * STAGE;      // double buffered
    static constexpr int CPR = D / 8;                // 16 B chunks per row
    static constexpr int CPT = BK * CPR / NTHREADS;  // chunks per thread per tile
};

template <int D>
__global__ void __launch_bounds__(NTHREADS, 2)
bwd_dq_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
              const uint16_t* __restrict__ v, const float* __restrict__ m,
              const uint16_t* __restrict__ dout, float* __restrict__ dq,
              float* __restrict__ ca, float* __restrict__ cb, int T, int BH, int nqb, int nt32)
{
    using C = DqCfg<D>;
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
    const int jq = min(q0 + n, T - 1);

    const long base = bh * (long)T * D;
    const uint16_t* Kg = k + base;
    const uint16_t* Vg = v + base;

    // B operands: this lane's query row of Q and dO (dO = 0 past T: such rows contribute nothing)
    bf16x8 qf[D / 16], gf[D / 16];
    {
        const u32x4* qs = reinterpret_cast<const u32x4*>(q + base + (long)jq * D + 8 * hh);
        const u32x4* gs = reinterpret_cast<const u32x4*>(dout + base + (long)jq * D + 8 * hh);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            u32x4 a = qs[2 * s], g = gs[2 * s];
            if (q0 + n >= T) g = u32x4{0u, 0u, 0u, 0u};
            qf[s] = __builtin_bit_cast(bf16x8, a);
            gf[s] = __builtin_bit_cast(bf16x8, g);
        }
    }

    // per-lane LDS offsets inside a tile
    const int key_l = perm_row(n);
    int aoff[D / 16];                       // A-operand reads (K rows for S^T, V rows for P^T)
#pragma unroll
    for (int s = 0; s < D / 16; ++s) aoff[s] = tile_off_perm<D>(key_l, 2 * s + hh);
    int ktr[D / 32][2];                     // transposing reads of K for dQ = dZ K
    {
        const int row_l = 16 * (gg >> 1) + (li >> 2);
        const int cl = 2 * (gg & 1) + ((li & 3) >> 1);
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                ktr[b][t] = tile_off_perm<D>(row_l + 4 * t, 4 * b + cl) + 8 * (li & 1);
    }

    u32x4 kst[C::CPT], vst[C::CPT];
    auto stage_load = [&](int kt) {
#pragma unroll
        for (int i = 0; i < C::CPT; ++i) {
            const int id = tid + i * NTHREADS;
            const int row = id / C::CPR, c = id % C::CPR;
            const long gr = min(kt * BK + row, T - 1);
            kst[i] = *reinterpret_cast<const u32x4*>(Kg + gr * D + c * 8);
            vst[i] = *reinterpret_cast<const u32x4*>(Vg + gr * D + c * 8);
        }
    };
    auto stage_store = [&](int buf) {
        char* kb = smem + buf * C::STAGE;
#pragma unroll
        for (int i = 0; i < C::CPT; ++i) {
            const int id = tid + i * NTHREADS;
            const int row = id / C::CPR, c = id % C::CPR;
            const int off = tile_off_perm<D>(row, c);
            *reinterpret_cast<u32x4*>(kb + off) = kst[i];
            *reinterpret_cast<u32x4*>(kb + C::TILE + off) = vst[i];
        }
    };

    f32x16 dqacc[D / 32];
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) dqacc[b][r] = 0.0f;

    const float scale = 1.0f / sqrtf((float)D);
    const float c2 = SB_LOG2E * scale;
    float a2 = -m[bh * (long)T + jq] * SB_LOG2E;   // sum of sp2 from the sweep position up to the query
    float bsum = 0.0f;                             // sum of G over the keys already passed
    float* const cag = ca + bh * (long)nt32 * T;
    float* const cbg = cb + bh * (long)nt32 * T;

    // ---- sweep over key tiles, left to right
    const int jmax = min(T, qb * BQ + BQ) - 1;
    const int ntile = (jmax + BK - 1) / BK;
    if (ntile > 0) {
        stage_load(0);
        stage_store(0);
    }
    __syncthreads();
    for (int kt = 0; kt < ntile; ++kt) {
        const int buf = kt & 1;
        const char* kb = smem + buf * C::STAGE;
        const bool more = kt + 1 < ntile;
        if (more) stage_load(kt + 1);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int key0 = kt * BK + 32 * u;
            if (wave_live && key0 <= q0) {
                const char* ktile = kb + u * 32 * C::ROW;
                const char* vtile = ktile + C::TILE;
                f32x16 sacc, pacc;
#pragma unroll
                for (int r = 0; r < 16; ++r) { sacc[r] = 0.0f; pacc[r] = 0.0f; }
#pragma unroll
                for (int s = 0; s < D / 16; ++s) {
                    const u32x4 kw = *reinterpret_cast<const u32x4*>(ktile + aoff[s]);
                    const u32x4 vw = *reinterpret_cast<const u32x4*>(vtile + aoff[s]);
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kw), qf[s], sacc, 0, 0, 0);
                    pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw), gf[s], pacc, 0, 0, 0);
                }
                const SubtileOut so = subtile_math<true>(sacc, pacc, a2, bsum, c2, scale, n, hh, key0 == q0);
                // carries of this (subtile, query) for the key-stationary kernel
                if (hh == 0 && q0 + n < T) {
                    const long ci = (long)(key0 >> 5) * T + q0 + n;
                    cag[ci] = so.ca_right;
                    cbg[ci] = bsum;
                }
                a2 = so.ca_right;
                bsum += so.g_tot;
                // dQ += dZ K: dZ from registers, K (rows = keys) through the transposing load
#pragma unroll
                for (int b = 0; b < D / 32; ++b) {
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const char* p = ktile + (8 * s) * C::ROW;
                        const bf16x8 kf = tr_pair(p + ktr[b][0], p + ktr[b][1]);
                        dqacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(so.pz[s], kf, dqacc[b], 0, 0, 0);
                    }
                }
            }
            if (u == 0 && more) stage_store(buf ^ 1);
        }
        __syncthreads();
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

// ------------------------------------------------------------------ dK / dV kernel
template <int D> struct DkvCfg {
    static constexpr int ROW = D * 2;
    static constexpr int TILE = 32 * ROW;            // 32 query rows
    static constexpr int STAGE = 2 * TILE;           // Q tile + dO tile
    static constexpr int T_OFF = 2 * STAGE;          // after the double buffer
    static constexpr int T_WAVE = 2 * 32 * TROW;     // A and dZ scratch of one wave
    static constexpr int LDS_BYTES = T_OFF + 4 * T_WAVE;
    static constexpr int CPR = D / 8;
    static constexpr int CPT = (32 * CPR + NTHREADS - 1) / NTHREADS;
};

template <int D>
__global__ void __launch_bounds__(NTHREADS, 1)
bwd_dkv_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
               const uint16_t* __restrict__ v, const uint16_t* __restrict__ dout,
               const float* __restrict__ ca, const float* __restrict__ cb,
               float* __restrict__ dk, float* __restrict__ dv, int T, int BH, int nkb, int nt32)
{
    using C = DkvCfg<D>;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const long bh = xcd + 8L * (slot / nkb);
    const int kb = slot % nkb;                      // small kb = most later queries = first
    if (bh >= BH) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int gg = lane >> 4, li = lane & 15;
    const int k0 = kb * BKW + wave * 32;            // this wave's 32 keys
    const int kt32 = k0 >> 5;
    const bool wave_live = k0 < T;

    const long base = bh * (long)T * D;
    const uint16_t* Qg = q + base;
    const uint16_t* Gg = dout + base;

    // A operands held for the whole kernel: this wave's K and V rows (MFMA row n <- key perm_row(n))
    bf16x8 kf[D / 16], vf[D / 16];
    {
        const long kr = min(k0 + perm_row(n), T - 1);
        const u32x4* ks = reinterpret_cast<const u32x4*>(k + base + kr * D + 8 * hh);
        const u32x4* vs = reinterpret_cast<const u32x4*>(v + base + kr * D + 8 * hh);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            kf[s] = __builtin_bit_cast(bf16x8, ks[2 * s]);
            vf[s] = __builtin_bit_cast(bf16x8, vs[2 * s]);
        }
    }

    // per-lane LDS offsets inside a 32-row Q / dO tile (natural row order)
    int boff[D / 16];                       // B-operand reads: row = query n
#pragma unroll
    for (int s = 0; s < D / 16; ++s) boff[s] = tile_off_nat<D>(n, 2 * s + hh);
    int qtr[D / 32][2];                     // transposing reads (K-dim = queries)
    {
        const int row_l = 8 * (gg >> 1) + (li >> 2);
        const int cl = 2 * (gg & 1) + ((li & 3) >> 1);
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                qtr[b][t] = tile_off_nat<D>(row_l + 4 * t, 4 * b + cl) + 8 * (li & 1);
    }
    char* const scr = smem + C::T_OFF + wave * C::T_WAVE;                 // [2][32][TROW]
    const int sw_off = n * TROW + 32 * hh;                                // scratch write: row = query n
    const int st_off = (8 * (gg >> 1) + (li >> 2)) * TROW + (16 * (gg & 1) + 4 * (li & 3)) * 2;

    u32x4 qst[C::CPT], gst[C::CPT];
    auto stage_load = [&](int qs) {
#pragma unroll
        for (int i = 0; i < C::CPT; ++i) {
            const int id = tid + i * NTHREADS;
            if (id < 32 * C::CPR) {
                const int row = id / C::CPR, c = id % C::CPR;
                const int j = qs * 32 + row;
                const long gr = min(j, T - 1);
                qst[i] = *reinterpret_cast<const u32x4*>(Qg + gr * D + c * 8);
                gst[i] = *reinterpret_cast<const u32x4*>(Gg + gr * D + c * 8);
                if (j >= T) gst[i] = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    auto stage_store = [&](int buf) {
        char* qb = smem + buf * C::STAGE;
#pragma unroll
        for (int i = 0; i < C::CPT; ++i) {
            const int id = tid + i * NTHREADS;
            if (id < 32 * C::CPR) {
                const int row = id / C::CPR, c = id % C::CPR;
                const int off = tile_off_nat<D>(row, c);
                *reinterpret_cast<u32x4*>(qb + off) = qst[i];
                *reinterpret_cast<u32x4*>(qb + C::TILE + off) = gst[i];
            }
        }
    };

    f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dkacc[b][r] = 0.0f; dvacc[b][r] = 0.0f; }

    const float scale = 1.0f / sqrtf((float)D);
    const float c2 = SB_LOG2E * scale;
    const float* const cag = ca + (bh * (long)nt32 + kt32) * T;
    const float* const cbg = cb + (bh * (long)nt32 + kt32) * T;

    // ---- sweep over 32-row query blocks, from the workgroup's diagonal to the end
    const int qs_begin = kb * (BKW / 32);
    if (qs_begin < nt32) {
        stage_load(qs_begin);
        stage_store(0);
    }
    __syncthreads();
    for (int qs = qs_begin; qs < nt32; ++qs) {
        const int buf = (qs - qs_begin) & 1;
        const char* qtile = smem + buf * C::STAGE;
        const char* gtile = qtile + C::TILE;
        const bool more = qs + 1 < nt32;
        if (more) stage_load(qs + 1);
        if (wave_live && qs >= kt32) {
            f32x16 sacc, pacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) { sacc[r] = 0.0f; pacc[r] = 0.0f; }
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                const u32x4 qw = *reinterpret_cast<const u32x4*>(qtile + boff[s]);
                const u32x4 gw = *reinterpret_cast<const u32x4*>(gtile + boff[s]);
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], __builtin_bit_cast(bf16x8, qw), sacc, 0, 0, 0);
                pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], __builtin_bit_cast(bf16x8, gw), pacc, 0, 0, 0);
            }
            const int j = qs * 32 + n;
            const int jc = min(j, T - 1);
            const float car = cag[jc];
            const float cbl = (j < T) ? cbg[jc] : 0.0f;    // rows past T must give dZ = 0
            const SubtileOut so = subtile_math<false>(sacc, pacc, car, cbl, c2, scale, n, hh, qs == kt32);

            // A and dZ into [key][query] operand layout through the wave's scratch
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            *reinterpret_cast<bf16x8*>(scr + sw_off) = so.pa[0];
            *reinterpret_cast<bf16x8*>(scr + sw_off + 16) = so.pa[1];
            *reinterpret_cast<bf16x8*>(scr + 32 * TROW + sw_off) = so.pz[0];
            *reinterpret_cast<bf16x8*>(scr + 32 * TROW + sw_off + 16) = so.pz[1];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            bf16x8 at[2], zt[2];
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const char* pa = scr + (16 * s2) * TROW + st_off;
                const char* pz = pa + 32 * TROW;
                at[s2] = tr_pair(pa, pa + 4 * TROW);
                zt[s2] = tr_pair(pz, pz + 4 * TROW);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

            // dV += A^T dO, dK += dZ^T Q: K-dim = the 32 queries, B operands through the transposing load
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const int ro = (16 * s2) * C::ROW;
                    const bf16x8 gop = tr_pair(gtile + ro + qtr[b][0], gtile + ro + qtr[b][1]);
                    const bf16x8 qop = tr_pair(qtile + ro + qtr[b][0], qtile + ro + qtr[b][1]);
                    dvacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[s2], gop, dvacc[b], 0, 0, 0);
                    dkacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zt[s2], qop, dkacc[b], 0, 0, 0);
                }
            }
        }
        if (more) stage_store(buf ^ 1);
        __syncthreads();
    }

    // ---- store: acc[b][r] is key row k0 + 8*(r/4) + 4*hh + r%4, column 32b + n
    if (wave_live) {
        float* dKg = dk + base;
        float* dVg = dv + base;
#pragma unroll
        for (int b = 0; b < D / 32; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = k0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                if (key < T) {
                    dKg[(long)key * D + 32 * b + n] = dkacc[b][r];
                    dVg[(long)key * D + 32 * b + n] = dvacc[b][r];
                }
            }
        }
    }
}

template <int D>
hipError_t launch_one(const uint16_t* q, const uint16_t* k, const uint16_t* v, const float* m,
                      const uint16_t* dout, float* dq, float* dk, float* dv, float* workspace,
                      int BH, int T, hipStream_t stream)
{
    auto kq = bwd_dq_kernel<D>;
    auto kkv = bwd_dkv_kernel<D>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kq),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, DqCfg<D>::LDS_BYTES);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kkv),
                            hipFuncAttributeMaxDynamicSharedMemorySize, DkvCfg<D>::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int nt32 = (T + 31) / 32;
    float* ca = workspace;
    float* cb = workspace + (long)BH * nt32 * T;
    const int nqb = (T + BQ - 1) / BQ;
    const int nkb = (T + BKW - 1) / BKW;
    const long bq = 8L * ((BH + 7) / 8) * nqb;
    const long bk = 8L * ((BH + 7) / 8) * nkb;
    if (bq > 0x7fffffffL || bk > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kq, dim3((unsigned)bq), dim3(NTHREADS), DqCfg<D>::LDS_BYTES, stream,
                       q, k, v, m, dout, dq, ca, cb, T, BH, nqb, nt32);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kkv, dim3((unsigned)bk), dim3(NTHREADS), DkvCfg<D>::LDS_BYTES, stream,
                       q, k, v, dout, ca, cb, dk, dv, T, BH, nkb, nt32);
    return hipGetLastError();
}

}  // namespace

size_t bwd_workspace_bytes(int B, int H, int T)
{
    const size_t nt32 = (size_t)(T + 31) / 32;
    return 2 * sizeof(float) * (size_t)B * H * nt32 * T;
}

hipError_t launch_bwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, const float* m,
                           const uint16_t* dout, float* dq, float* dk, float* dv, float* workspace,
                           int B, int H, int T, int d, hipStream_t stream)
{
    const int BH = B * H;
    if (d == 64) return launch_one<64>(q, k, v, m, dout, dq, dk, dv, workspace, BH, T, stream);
    return launch_one<128>(q, k, v, m, dout, dq, dk, dv, workspace, BH, T, stream);
}

}  // namespace sb
