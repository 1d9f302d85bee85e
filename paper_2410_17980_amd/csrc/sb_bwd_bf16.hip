// bf16 backward of causal stick-breaking attention on the gfx950 matrix cores
// (Eq. 4 evaluated tile by tile; the per-tile steps are those of Algorithm 2).
//
// Two kernels instead of Algorithm 2's single query-stationary kernel with
// atomic adds into dK and dV.  The dependency that forces the paper's atomics is
// the cumulative sum over keys inside each query row; it is cut by saving, per
// query row and per 32-key subtile, the two carried scalars
//     ca = sum of sp2 over the keys to the right of the subtile (up to the query),
//     cb = sum of G = A*(dO.v) over the keys to the left of the subtile,
// (2 floats per 32x1 strip of the attention matrix; sp2 = base-2 softplus).  With
// them any subtile can be recomputed on its own, so dK and dV are accumulated by a
// key-stationary kernel in registers and written once, with no atomics and no
// zero fill, and the result is bit-reproducible.
//
//   bwd_dq_kernel  (query-stationary, 128 query rows per block, sweep from key 0
//                   to the diagonal as Algorithm 2): recomputes A from m, forms G
//                   and dZ, accumulates dQ += dZ K, stores ca, cb.
//   bwd_dkv_kernel (key-stationary, 128 key rows per block = 32 per wave, K and V
//                   rows held in registers, sweep over query tiles from the
//                   diagonal to the end): recomputes A, G, dZ from ca, cb and
//                   accumulates dV += A^T dO, dK += dZ^T Q.
// The element-wise arithmetic runs in the linear domain inside a lane (one exponential
// and one reciprocal per element, see subtile_stage1/2); where its running product
// leaves the fp32 range (sharp logits) the kernel only records that in a per-block
// flag, and a second launch of the same kernel in its log-domain variant (SLOW)
// redoes exactly the flagged blocks and returns at once for the others.  Keeping the
// overflow-proof form out of the fast kernels keeps them within their register budget.
// Both kernels give a workgroup two blocks, p and n-1-p, whose causal costs add up
// to the same total for every p, and stage their streamed tiles with direct
// global->LDS loads, double buffered, one barrier per 64-row tile.  The 1/sqrt(d)
// of dQ and dK is applied once, to the accumulators, on store.
//
// Register layout is the forward's: S^T = K Q^T and P^T = V dO^T with the
// 32x32x16 bf16 MFMA, a lane owns one query column and 16 consecutive keys, so
// both cumulative quantities are serial inside the lane plus one exchange between
// the half-waves.  dZ feeds the "query-major" product (dQ) straight from
// registers; for the "key-major" products (dK, dV) A and dZ are written to a small
// per-wave LDS scratch row-wise and read back with the transposing load.
#include <type_traits>

#include "sb_kernels.h"
#include "sb_mma.h"

namespace sb {
namespace {

constexpr int NTHREADS = 256;
constexpr int NW = 4;        // wavefronts per workgroup
constexpr int BQ = 128;      // dq kernel: query rows per block
constexpr int BKW = 128;     // dkv kernel: key rows per block (32 per wave)
constexpr int TK = 64;       // rows per staged tile (keys in the dq kernel, queries in the dkv kernel)
constexpr int SCR_MAT = 32 * 64;   // one 32x32 bf16 matrix of the A / dZ transposition scratch

// Byte offset of 16-byte chunk c (0..3) of row `row` of a scratch matrix.  16-byte LDS writes
// are taken eight lanes at a time (measured: 8 cycles per conflict-free ds_write_b128), so the
// eight rows 8i .. 8i+7 that write the same chunk together must land in eight different 16-byte
// slots of a 128-byte window: the chunk index is xor-ed with bits 1-2 of the row (rows 2j and
// 2j+1 already differ by 64 bytes).  The transposing reads take four whole rows at a time and
// do not care how a row's chunks are permuted.  Counters: no bank conflicts either way (the
// same layout with bits 2-3 of the row costs 8 conflict cycles per write).
__device__ __forceinline__ int scr_off(int row, int c)
{
    return row * 64 + ((c ^ ((row >> 1) & 3)) << 4);
}

template <bool B> using bc = std::integral_constant<bool, B>;

#ifndef SB_SIGMA_DQ
#define SB_SIGMA_DQ 2
#endif
#ifndef SB_SIGMA_DKV
#define SB_SIGMA_DKV 2
#endif
constexpr int SIGMA_DQ = SB_SIGMA_DQ;     // how each pass forms sigma (see subtile_stage1)
constexpr int SIGMA_DKV = SB_SIGMA_DKV;

// ------------------------------------------------------------------ element-wise core
// One 32x32 subtile in the lane layout (query n; keys 16hh + r).
struct SubtileOut {
    bf16x8 pa[2];    // A, as MFMA operand (K-dim element e of half s <-> key 16hh + 8s + e)
    bf16x8 pz[2];    // dZ (without the 1/sqrt(d)), same layout
    float ca_right;  // sum of sp2 over the keys right of the subtile
    float g_tot;     // sum of G over the subtile's 32 keys
};

// Log-domain form (Eq. 2 / Eq. 4 as printed), overflow-proof; used only where the
// linear-domain chain of subtile_math leaves its range.
template <bool CA_INCLUDES_SUBTILE, bool MASK>
__device__ __forceinline__ void subtile_math_log(SubtileOut& out, const f32x16& sacc, const f32x16& pacc,
                                              float ca, float cb, float c2, int n, int hh)
{
    float x[16], sp[16], cs[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = sacc[r] * c2;
    if (MASK) {
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
        out.pz[r >> 3][r & 7] = (__bf16)dz;
    }
}

// The same in the linear domain inside the lane, as in the forward: with e_r = 2^{x_r}
// the chain t_r = W_r e_r, W_{r+1} = W_r + t_r over ascending keys gives
// A[r] = t_r / W_16 * 2^-(sp2 total of all nearer keys), and sigma = e / (1 + e):
// one exponential and one reciprocal per element instead of three exponentials and
// a logarithm.  W_0 = 2^-60; a chain that gets beyond 2^80 (or overflows) makes the
// caller redo the subtile with subtile_math_log.  Two stages, so that the dO.v
// accumulator need not be live during the first:
//   stage 1 (logits only): sigma, chain.  Returns false in a lane whose chain left its range.
//   stage 2 (needs dO.v): A, G, dZ.
// sacc: q.k accumulator, pacc: dO.v accumulator.  cb: sum of G over the keys left
// of the subtile.  ca: sum of sp2 over the keys right of the subtile, or, with
// CA_INCLUDES_SUBTILE, over the subtile's own keys as well (Algorithm 2 carries
// that and subtracts the subtile's total before use).  With MASK, key 16hh + r is
// visible to query n iff 16hh + r < n (the subtile on the diagonal).
struct Chain {
    float be[16];    // sigma(z)
    float t[16];     // chain terms, later G
    float W;         // end of the chain
};

// How sigma = e / (1 + e) is formed (SIGMA):
//   0  e * rcp(1 + e): independent of the chain, an add and a reciprocal per element;
//   1  t_r * rcp(W_{r+1}): one add fewer, but the reciprocal waits for the chain;
//   2  t_r * (1 / W_{r+1}) with the 16 reciprocals from ONE reciprocal and a second chain run
//      backwards, 1/W_r = 1/W_{r+1} * (1 + e_r): a fused multiply-add per element in place of
//      the reciprocal (a transcendental, about twice the cost of a plain instruction here).
template <bool MASK, int SIGMA = 0>
__device__ __forceinline__ bool subtile_stage1(Chain& ch, const f32x16& sacc, float c2, int n, int hh)
{
    float W = 0x1p-60f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        float e = fast_exp2(sacc[r] * c2);
        if (MASK) e = (16 * hh + r < n) ? e : 0.0f;
        ch.t[r] = W * e;
        W += ch.t[r];
        if (SIGMA == 0) ch.be[r] = e * __builtin_amdgcn_rcpf(1.0f + e);
        else if (SIGMA == 1) ch.be[r] = ch.t[r] * __builtin_amdgcn_rcpf(W);
        else ch.be[r] = e;                                 // kept for the backward chain below
    }
    ch.W = W;
    if (SIGMA == 2) {
        float inv = __builtin_amdgcn_rcpf(W);              // 1 / W_16; 0 where the chain overflowed
#pragma unroll
        for (int r = 15; r >= 0; --r) {
            const float e = ch.be[r];
            ch.be[r] = ch.t[r] * inv;                      // t_r / W_{r+1}
            inv = __builtin_fmaf(inv, e, inv);             // 1 / W_r
        }
    }
    return W < 0x1p80f;                                    // false: this lane's chain left its range
}

template <bool CA_INCLUDES_SUBTILE, bool NEED_A>
__device__ __forceinline__ void subtile_stage2(SubtileOut& out, Chain& ch, const f32x16& pacc,
                                               float ca, float cb, int hh)
{
    const float l = fast_log2(ch.W) + 60.0f;               // sp2 total of this lane's 16 keys
    float l_lo, l_hi;
    both_halves(l, l_lo, l_hi);
    const float car = CA_INCLUDES_SUBTILE ? ca - (l_lo + l_hi) : ca;
    out.ca_right = car;
    // keys 16..31 (hh = 1) are nearer to the query than keys 0..15
    const float kf = fast_exp2(60.0f - (car + l_hi + (hh == 0 ? l_lo : 0.0f)));
    // dZ = G - sigma * (prefix of G + boff), boff = cb + the partner half's total for the
    // nearer half: the part that needs boff is added once boff is known
    float grun = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float w = ch.t[r] * kf;                      // A
        if (NEED_A) out.pa[r >> 3][r & 7] = (__bf16)w;
        const float g = w * pacc[r];                       // G = dL/dlogA = A * dL/dA
        grun += g;                                         // inclusive prefix inside the lane
        ch.t[r] = g - ch.be[r] * grun;
    }
    float g_lo, g_hi;
    both_halves(grun, g_lo, g_hi);
    out.g_tot = g_lo + g_hi;
    const float boff = cb + (hh == 1 ? g_lo : 0.0f);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float dz = ch.t[r] - ch.be[r] * boff;        // Eq. 4
        out.pz[r >> 3][r & 7] = (__bf16)dz;
    }
}

// ------------------------------------------------------------------ staging
// Direct global -> LDS staging of 64-row tiles of two [T][D] matrices (X then Y in
// one stage).  One instruction moves 16 B per lane to 1 KB of consecutive LDS; the
// swizzle is applied on the global side.  PERM selects the swizzle (see sb_mma.h).
template <int D> struct StageCfg {
    static constexpr int ROW = D * 2;
    static constexpr int TILE = TK * ROW;               // one 64-row tile
    static constexpr int STAGE = 2 * TILE;
    static constexpr int CPR = ROW / 16;
    static constexpr int BLK_ROWS = 1024 / ROW;
    static constexpr int NPW = TILE / 1024 / NW;        // loads per wave per tile
};

// goff[i]: byte offset inside a tile of the 16 B this lane fetches with its i-th load
template <int D, bool PERM>
__device__ __forceinline__ void stage_offsets(int (&goff)[StageCfg<D>::NPW], int wave, int lane)
{
    using C = StageCfg<D>;
#pragma unroll
    for (int i = 0; i < C::NPW; ++i) {
        const int row = (wave * C::NPW + i) * C::BLK_ROWS + lane / C::CPR;
        const int swz = PERM ? swz_perm<D>(row) : swz_nat<D>(row);
        goff[i] = (row * D + (((lane % C::CPR) ^ swz) << 3)) * 2;
    }
}

template <int D, bool PERM>
__device__ __forceinline__ void stage_tile(const uint16_t* X, const uint16_t* Y, int jt, int T, char* sp,
                                           const int (&goff)[StageCfg<D>::NPW], int wave, int lane)
{
    using C = StageCfg<D>;
    if ((jt + 1) * TK <= T) {                           // all 64 rows exist
        const uint16_t* xb = X + (long)jt * TK * D;
        const uint16_t* yb = Y + (long)jt * TK * D;
#pragma unroll
        for (int i = 0; i < C::NPW; ++i) dma16_to_lds_saddr(xb, goff[i], sp + (wave * C::NPW + i) * 1024);
#pragma unroll
        for (int i = 0; i < C::NPW; ++i) dma16_to_lds_saddr(yb, goff[i], sp + C::TILE + (wave * C::NPW + i) * 1024);
    } else {                                            // rows past T are clamped (their results are masked)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const uint16_t* G = m == 0 ? X : Y;
#pragma unroll
            for (int i = 0; i < C::NPW; ++i) {
                const int row = (wave * C::NPW + i) * C::BLK_ROWS + lane / C::CPR;
                const int swz = PERM ? swz_perm<D>(row) : swz_nat<D>(row);
                const int c = (lane % C::CPR) ^ swz;
                const long gr = min(jt * TK + row, T - 1);
                dma16_to_lds(G + gr * D + c * 8, sp + m * C::TILE + (wave * C::NPW + i) * 1024);
            }
        }
    }
}

// ------------------------------------------------------------------ dQ kernel
// VL (both kernels): packed variable-length batch, tensors [H][Ttot][D] ([H/G][Ttot][D] for
// k, v, dk, dv) with sequence s at rows cu[s] .. cu[s+1]-1.  BH counts (sequence, head)
// pairs; T_arg and the block counts describe the longest sequence (they size the grid, the
// flag arrays and the carries, which are then laid out [head][strip][Ttot]); a workgroup
// whose blocks lie beyond its own sequence's end returns at once.
template <int D, bool SLOW, bool RB, bool VL>
__global__ void __launch_bounds__(NTHREADS, SLOW ? 1 : 2)
bwd_dq_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
              const uint16_t* __restrict__ v, const uint16_t* __restrict__ rb,
              const float* __restrict__ m,
              const uint16_t* __restrict__ dout, float* __restrict__ dq,
              float* __restrict__ ca, float* __restrict__ cb, int* __restrict__ flags,
              int T_arg, int BH, int H, int G, int nqb_arg, int nt32, const int* __restrict__ cu, int Ttot)
{
    using C = StageCfg<D>;
    __shared__ __attribute__((aligned(1024))) char smem[2 * C::STAGE];
    __shared__ int s_dirty;

    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const int npair = (nqb_arg + 1) >> 1;
    const long bh = xcd + 8L * (slot / npair);
    const int pidx = slot % npair;
    if (bh >= BH) return;
    int T = T_arg, nqb = nqb_arg;
    long row0, kvrow0, cbase, cstride;      // first q / k row of this head; carries: base and strip stride
    int head;
    if constexpr (VL) {
        const int seq = (int)(bh / H);
        head = (int)(bh % H);
        const int c0 = cu[seq];
        T = min(min(cu[seq + 1], Ttot) - c0, T_arg);      // never past the packed rows or the stated maximum
        if (c0 < 0) return;
        nqb = (T + BQ - 1) / BQ;
        if (pidx >= ((nqb + 1) >> 1)) return;
        row0 = (long)head * Ttot + c0;
        kvrow0 = (long)(head / G) * Ttot + c0;
        cbase = (long)head * nt32 * Ttot + c0;
        cstride = Ttot;
    } else {
        // grouped kv heads: G consecutive query heads read the same K and V
        head = (int)(bh % H);
        row0 = bh * (long)T;
        kvrow0 = (G == 1 ? bh : (bh / H) * (H / G) + (bh % H) / G) * (long)T;
        cbase = bh * (long)nt32 * T;
        cstride = T;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;
    const int gg = lane >> 4, li = lane & 15;

    const long base = row0 * D;
    const long kvbase = kvrow0 * D;
    const uint16_t* Kg = k + kvbase;
    const uint16_t* Vg = v + kvbase;

    // Per-lane LDS offsets inside a 32-row subtile.  The swizzle xors the chunk index, and the
    // chunk indices a lane reads differ in bits the swizzle leaves alone, so one offset per
    // access pattern is kept and the others follow by xor with a constant:
    //   A-operand read of chunk pair s (K rows for S^T, V rows for P^T):  aoff0 ^ (s << 5)
    //   transposing read of K, column block b, row group t (dQ = dZ K):    ktr0[t] ^ (b << 6)
    const uint32_t aoff0 = tile_off_perm<D>(perm_row(n), hh);
    uint32_t ktr0[2];
    {
        const int row_l = 16 * (gg >> 1) + (li >> 2);
        const int cl = 2 * (gg & 1) + ((li & 3) >> 1);
#pragma unroll
        for (int t = 0; t < 2; ++t) ktr0[t] = tile_off_perm<D>(row_l + 4 * t, cl) + 8 * (li & 1);
    }
    const uint32_t smem0 = lds_offset(smem);
    int goff[C::NPW];
    stage_offsets<D, true>(goff, wave, lane);

    const float scale = 1.0f / sqrtf((float)D);
    const float c2 = SB_LOG2E * scale;
    float* const cag = ca + cbase;
    float* const cbg = cb + cbase;

    bf16x8 qf[D / 16], gf[D / 16];          // B operands: this lane's query row of Q and dO
    f32x16 dqacc[D / 32];
    float a2 = 0.0f;                        // sum of sp2 from the sweep position up to the query
    float bsum = 0.0f;                      // sum of G over the keys already passed
    int q0 = 0;
    bool dirty = false;                     // a chain of this lane left its range (fast variant)

    // one 32-key subtile at keys key0 .. key0+31
    // ktile: LDS address of the subtile's K rows (its V rows lie C::TILE further)
    auto subtile = [&](auto mask_c, uint32_t ktile, int key0) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_c)::value;
        const uint32_t ka = ktile + aoff0;
        // the operand reads of a product are issued before its first MFMA: the LDS latency
        // is then paid once per product, not once per MFMA
        auto s_mfma = [&]() __attribute__((always_inline)) {
            u32x4 kw[D / 16];
#pragma unroll
            for (int s = 0; s < D / 16; ++s) kw[s] = lds_load16(ka ^ (s << 5));
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kw[s]), qf[s], acc, 0, 0, 0);
            return acc;
        };
        auto p_mfma = [&]() __attribute__((always_inline)) {
            u32x4 vw[D / 16];
#pragma unroll
            for (int s = 0; s < D / 16; ++s) vw[s] = lds_load16((ka ^ (s << 5)) + C::TILE);
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw[s]), gf[s], acc, 0, 0, 0);
            return acc;
        };
        SubtileOut so;
        if constexpr (SLOW) {
            const f32x16 sacc = s_mfma();
            const f32x16 pacc = p_mfma();
            subtile_math_log<true, MASK>(so, sacc, pacc, a2, bsum, c2, n, hh);
        } else {
            Chain ch;
            const f32x16 sacc = s_mfma();
            dirty |= !subtile_stage1<MASK, SIGMA_DQ>(ch, sacc, c2, n, hh);
            const f32x16 pacc = p_mfma();
            subtile_stage2<true, false>(so, ch, pacc, a2, bsum, hh);
        }
        // carries of this (subtile, query) for the key-stationary kernel
        if (hh == 0 && q0 + n < T) {
            const long ci = (long)(key0 >> 5) * cstride + q0 + n;
            cag[ci] = so.ca_right;
            cbg[ci] = bsum;
        }
        a2 = so.ca_right;
        bsum += so.g_tot;
        // dQ += dZ K: dZ from registers, K (rows = keys) through the transposing load
        bf16x8 kt[D / 16];
        const uint32_t k0a = ktile + ktr0[0], k1a = ktile + ktr0[1];
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int ro = (8 * s) * C::ROW;
                kt[2 * b + s] = tr_pair_at((k0a ^ (b << 6)) + ro, (k1a ^ (b << 6)) + ro);
            }
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                dqacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(so.pz[s], kt[2 * b + s], dqacc[b], 0, 0, 0);
    };

    for (int part = 0; part < 2; ++part) {
        const int qb = part == 0 ? nqb - 1 - pidx : pidx;
        if (part == 1 && 2 * pidx == nqb - 1) break;     // odd block count: the middle block is alone
        if (SLOW && flags[bh * nqb_arg + qb] == 0) continue;  // only the blocks the fast variant flagged
        const int Q0 = qb * BQ;
        q0 = Q0 + wave * 32;
        const bool wave_live = q0 < T;
        const int jq = min(q0 + n, T - 1);
        if (tid == 0) s_dirty = 0;
        dirty = false;
        barrier_nofence();                               // everyone is done with the stages of the block before
        {
            const u32x4* qs = reinterpret_cast<const u32x4*>(q + base + (long)jq * D + 8 * hh);
            const u32x4* gs = reinterpret_cast<const u32x4*>(dout + base + (long)jq * D + 8 * hh);
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                u32x4 a = qs[2 * s], g = gs[2 * s];
                if (q0 + n >= T) g = u32x4{0u, 0u, 0u, 0u};   // rows past T contribute nothing
                qf[s] = __builtin_bit_cast(bf16x8, a);
                gf[s] = __builtin_bit_cast(bf16x8, g);
            }
        }
        a2 = -m[row0 + jq] * SB_LOG2E;
        bsum = 0.0f;
        if constexpr (RB) {
            // remainder bias (Appendix C): the unused stick exp(m) acts like one more weight
            // in front of key 0, with "value" r_head: the cumulative sum of G starts at
            // exp(m_j) (dO_j . r_head)
            const u32x4* rs = reinterpret_cast<const u32x4*>(rb + head * D + 8 * hh);
            float dot = 0.0f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                const bf16x8 rr = __builtin_bit_cast(bf16x8, rs[2 * s]);
#pragma unroll
                for (int e = 0; e < 8; ++e) dot += (float)gf[s][e] * (float)rr[e];
            }
            float d_lo, d_hi;
            both_halves(dot, d_lo, d_hi);
            bsum = fast_exp2(-a2) * (d_lo + d_hi);
        }
        // wait for these loads (and the first block's stores) once, before the staging
        // loads, which are counted in the same counter behind the compiler's back
#pragma unroll
        for (int s = 0; s < D / 16; ++s) { asm volatile("" :: "v"(qf[s])); asm volatile("" :: "v"(gf[s])); }
        asm volatile("" :: "v"(a2));
        asm volatile("" :: "v"(bsum));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) dqacc[b][r] = 0.0f;

        // ---- sweep over 64-key tiles, left to right; iteration it handles tile it in buffer it & 1
        const int kmax = min(T, Q0 + BQ) - 1;            // keys 0 .. kmax-1 are visible to some row
        const int ntile = (kmax + TK - 1) / TK;
        const int nclean = min(ntile, Q0 / TK);          // tiles entirely left of the block's rows
        stage_tile<D, true>(Kg, Vg, 0, T, smem, goff, wave, lane);
        auto begin_iter = [&](int it) __attribute__((always_inline)) {
            dma_wait<0>();                               // this wave's share of tile `it` has landed
            barrier_nofence();                           // ... everyone's has, and tile it-1 is no longer read
            // past the end tile 0 is loaded once more into the buffer nobody reads
            stage_tile<D, true>(Kg, Vg, it + 1 < ntile ? it + 1 : 0, T, smem + ((it + 1) & 1) * C::STAGE, goff, wave, lane);
            return smem0 + (it & 1) * C::STAGE;
        };
        int it = 0;
        for (; it < nclean; ++it) {                      // fully visible tiles
            const uint32_t sp = begin_iter(it);
            subtile(bc<false>{}, sp, it * TK);
            subtile(bc<false>{}, sp + 32 * C::ROW, it * TK + 32);
        }
        for (; it < ntile; ++it) {                       // tiles that touch the diagonal band
            const uint32_t sp = begin_iter(it);
            if (wave_live) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int key0 = it * TK + 32 * u;
                    if (key0 == q0) subtile(bc<true>{}, sp + u * 32 * C::ROW, key0);
                    else if (key0 < q0) subtile(bc<false>{}, sp + u * 32 * C::ROW, key0);
                }
            }
        }
        dma_wait<0>();

        // ---- dQ store: dqacc[b][r] is query row 8*(r/4) + 4*hh + r%4, column 32b + n
        if (wave_live) {
            float* dQg = dq + base;
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = q0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (row < T) dQg[(long)row * D + 32 * b + n] = dqacc[b][r] * scale;
                }
            }
        }
        if constexpr (!SLOW) {
            if (__builtin_amdgcn_ballot_w64(dirty) != 0 && lane == 0) atomicOr(&s_dirty, 1);
            __syncthreads();
            if (tid == 0) flags[bh * nqb_arg + qb] = s_dirty;
        }
    }
}

// Where a kv head's rows and its query heads' rows and carries live (key-stationary kernels).
// bh counts kv heads (B * H / G of them); its G query heads are qh0 .. qh0+G-1.  Returns
// false when the workgroup has nothing to do (packed batch: blocks beyond its sequence).
struct KvHead {
    int T, nkb;                             // rows and 128-key blocks of this head's sequence
    long base;                              // first element of the kv head's K / V / dK / dV rows
    long qrow0, qrow_step;                  // first Q / dO row of query head qh0, step to the next head
    long cbase, cbase_step, cstride;        // carries: start for head qh0, step per head, strip stride
};

template <int D, bool VL>
__device__ __forceinline__ bool kv_head(KvHead& kh, long bh, int pidx, int T_arg, int nkb_arg, int H, int G,
                                        int nt32, const int* __restrict__ cu, int Ttot)
{
    const int Hkv = H / G;
    if constexpr (VL) {
        const int seq = (int)(bh / Hkv);
        const int hkv = (int)(bh % Hkv);
        const int c0 = cu[seq];
        kh.T = min(min(cu[seq + 1], Ttot) - c0, T_arg);   // never past the packed rows or the stated maximum
        if (c0 < 0) return false;
        kh.nkb = (kh.T + BKW - 1) / BKW;
        if (pidx >= ((kh.nkb + 1) >> 1)) return false;
        kh.base = ((long)hkv * Ttot + c0) * D;
        kh.qrow0 = (long)hkv * G * Ttot + c0;
        kh.qrow_step = Ttot;
        kh.cbase = (long)hkv * G * nt32 * Ttot + c0;
        kh.cbase_step = (long)nt32 * Ttot;
        kh.cstride = Ttot;
    } else {
        const long qh0 = G == 1 ? bh : (bh / Hkv) * H + (bh % Hkv) * G;
        kh.T = T_arg;
        kh.nkb = nkb_arg;
        kh.base = bh * (long)T_arg * D;
        kh.qrow0 = qh0 * (long)T_arg;
        kh.qrow_step = T_arg;
        kh.cbase = qh0 * (long)nt32 * T_arg;
        kh.cbase_step = (long)nt32 * T_arg;
        kh.cstride = T_arg;
    }
    return true;
}

// ------------------------------------------------------------------ dK / dV kernel
template <int D> struct DkvCfg {
    static constexpr int T_OFF = 2 * StageCfg<D>::STAGE;   // after the double buffer
    static constexpr int T_WAVE = 2 * SCR_MAT;             // A and dZ scratch of one wave
    static constexpr int LDS_BYTES = T_OFF + NW * T_WAVE;
};

template <int D, bool SLOW, bool GQA, bool VL>
__global__ void __launch_bounds__(NTHREADS, (D == 128 || SLOW) ? 1 : 2)
bwd_dkv_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
               const uint16_t* __restrict__ v, const uint16_t* __restrict__ dout,
               const float* __restrict__ ca, const float* __restrict__ cb,
               float* __restrict__ dk, float* __restrict__ dv, int* __restrict__ flags,
               int T_arg, int BH, int H, int G_arg, int nkb_arg, int nt32, const int* __restrict__ cu, int Ttot)
{
    using C = StageCfg<D>;
    using CK = DkvCfg<D>;
    const int G = GQA ? G_arg : 1;                      // query heads per kv head
    __shared__ __attribute__((aligned(1024))) char smem[CK::LDS_BYTES];
    __shared__ int s_dirty;

    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const int npair = (nkb_arg + 1) >> 1;
    const long bh = xcd + 8L * (slot / npair);
    const int pidx = slot % npair;
    if (bh >= BH) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;
    const int gg = lane >> 4, li = lane & 15;

    // bh counts kv heads here (BH = B * H / G of them)
    KvHead kh;
    if (!kv_head<D, VL>(kh, bh, pidx, T_arg, nkb_arg, H, G, nt32, cu, Ttot)) return;
    const int T = kh.T, nkb = kh.nkb;
    const long base = kh.base, qrow0 = kh.qrow0, qrow_step = kh.qrow_step;
    const long cbase = kh.cbase, cbase_step = kh.cbase_step, cstride = kh.cstride;
    const uint16_t* Qg = nullptr;
    const uint16_t* Gg = nullptr;

    // per-lane LDS offsets inside a 32-row Q / dO subtile (natural row order)
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
    int goff[C::NPW];
    stage_offsets<D, false>(goff, wave, lane);
    char* const scr = smem + CK::T_OFF + wave * CK::T_WAVE;               // [A, dZ][32 rows of 64 B]
    const int sw_off = scr_off(n, 2 * hh);                                // scratch write: row = query n; second chunk: ^ 16
    int st_off[2];                                                        // transposing reads, rows 8h + li/4 (+ 4t)
#pragma unroll
    for (int t = 0; t < 2; ++t)
        st_off[t] = scr_off(8 * (gg >> 1) + (li >> 2) + 4 * t, 2 * (gg & 1) + ((li & 3) >> 1)) + 8 * (li & 1);

    const float scale = 1.0f / sqrtf((float)D);
    const float c2 = SB_LOG2E * scale;

    bf16x8 kf[D / 16], vf[D / 16];          // A operands: this wave's K and V rows (MFMA row n <- key perm_row(n))
    f32x16 dkacc[D / 32], dvacc[D / 32];
    const float* cag = nullptr;
    const float* cbg = nullptr;
    bool dirty = false;                     // a chain of this lane left its range (fast variant)

    // one 32-query subtile at query rows j0 .. j0+31
    // the steps of one 32-query subtile (Q rows at qtile, dO rows C::TILE further).  All
    // operand reads of a step are issued before its first MFMA, so that the LDS latency
    // is paid once per step and not once per MFMA.
    // S^T = K Q^T and P^T = V dO^T (two independent accumulation chains, interleaved)
    auto sp_mfma = [&](const char* qtile, f32x16& sacc, f32x16& pacc) __attribute__((always_inline)) {
        const char* gtile = qtile + C::TILE;
        u32x4 qw[D / 16], gw[D / 16];
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            qw[s] = *reinterpret_cast<const u32x4*>(qtile + boff[s]);
            gw[s] = *reinterpret_cast<const u32x4*>(gtile + boff[s]);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[r] = 0.0f; pacc[r] = 0.0f; }
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], __builtin_bit_cast(bf16x8, qw[s]), sacc, 0, 0, 0);
            pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], __builtin_bit_cast(bf16x8, gw[s]), pacc, 0, 0, 0);
        }
    };
    // A and dZ into [key][query] operand layout through the wave's scratch
    auto transpose = [&](const SubtileOut& so, bf16x8 (&at)[2], bf16x8 (&zt)[2]) __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        *reinterpret_cast<bf16x8*>(scr + sw_off) = so.pa[0];
        *reinterpret_cast<bf16x8*>(scr + (sw_off ^ 16)) = so.pa[1];
        *reinterpret_cast<bf16x8*>(scr + SCR_MAT + sw_off) = so.pz[0];
        *reinterpret_cast<bf16x8*>(scr + SCR_MAT + (sw_off ^ 16)) = so.pz[1];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const char* pa = scr + (16 * s2) * 64;         // rows 16 s2 + ..: same swizzle as rows 0..15
            const char* pz = pa + SCR_MAT;
            at[s2] = tr_pair(pa + st_off[0], pa + st_off[1]);
            zt[s2] = tr_pair(pz + st_off[0], pz + st_off[1]);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    };
    // dV += A^T dO, dK += dZ^T Q: K-dim = the 32 queries, B operands through the transposing load
    auto mm2_fetch = [&](const char* qtile, bf16x8 (&gop)[D / 16], bf16x8 (&qop)[D / 16]) __attribute__((always_inline)) {
        const char* gtile = qtile + C::TILE;
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const int ro = (16 * s2) * C::ROW;
                gop[2 * b + s2] = tr_pair(gtile + ro + qtr[b][0], gtile + ro + qtr[b][1]);
                qop[2 * b + s2] = tr_pair(qtile + ro + qtr[b][0], qtile + ro + qtr[b][1]);
            }
    };
    auto mm2 = [&](const bf16x8 (&gop)[D / 16], const bf16x8 (&qop)[D / 16], const bf16x8 (&at)[2], const bf16x8 (&zt)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                dvacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[s2], gop[2 * b + s2], dvacc[b], 0, 0, 0);
                dkacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zt[s2], qop[2 * b + s2], dkacc[b], 0, 0, 0);
            }
    };
    // one 32-query subtile, start to end
    auto subtile = [&](auto mask_c, const char* qtile, float car, float cbl) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_c)::value;
        if (MASK && n == 0) {
            // The first query of the diagonal subtile sees none of its keys, and where that
            // query is the last row of the sequence the query-stationary pass never visits
            // this subtile: its carries may be unwritten memory.  They multiply zeros, so
            // any finite value will do.
            car = 0.0f;
            cbl = 0.0f;
        }
        SubtileOut so;
        f32x16 sacc, pacc;
        sp_mfma(qtile, sacc, pacc);
        bf16x8 gop[D / 16], qop[D / 16];
        mm2_fetch(qtile, gop, qop);                          // lands during the element-wise work
        if constexpr (SLOW) {
            subtile_math_log<false, MASK>(so, sacc, pacc, car, cbl, c2, n, hh);
        } else {
            Chain ch;
            dirty |= !subtile_stage1<MASK, SIGMA_DKV>(ch, sacc, c2, n, hh);
            subtile_stage2<false, true>(so, ch, pacc, car, cbl, hh);
        }
        bf16x8 at[2], zt[2];
        transpose(so, at, zt);
        mm2(gop, qop, at, zt);
    };

    for (int part = 0; part < 2; ++part) {
        const int kb = part == 0 ? pidx : nkb - 1 - pidx;    // small kb = most later queries = first
        if (part == 1 && 2 * pidx == nkb - 1) break;
        if (SLOW && flags[bh * nkb_arg + kb] == 0) continue; // only the blocks the fast variant flagged
        const int K0 = kb * BKW;
        const int k0 = K0 + wave * 32;                       // this wave's 32 keys
        const int kt32 = k0 >> 5;
        const bool wave_live = k0 < T;
        if (tid == 0) s_dirty = 0;
        dirty = false;
        barrier_nofence();                                   // everyone is done with the stages of the block before
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
#pragma unroll
        for (int s = 0; s < D / 16; ++s) { asm volatile("" :: "v"(kf[s])); asm volatile("" :: "v"(vf[s])); }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) { dkacc[b][r] = 0.0f; dvacc[b][r] = 0.0f; }
        // the query heads of the group one after the other, into the same accumulators
        for (int g = 0; g < G; ++g) {
        Qg = q + (qrow0 + g * qrow_step) * D;
        Gg = dout + (qrow0 + g * qrow_step) * D;
        cag = ca + cbase + g * cbase_step + kt32 * cstride;
        cbg = cb + cbase + g * cbase_step + kt32 * cstride;
        if (g > 0) barrier_nofence();                        // everyone is done with the stages of the head before

        // ---- sweep over 64-row query tiles, from the block's diagonal to the end;
        // iteration it handles tile jt0 + it in buffer it & 1.  The carries of a tile are
        // fetched one iteration ahead, and BEFORE the staging loads of that iteration are
        // issued: vector memory operations complete in order, so a wait for a carry
        // issued after the staging loads would wait for those as well.
        const int jt0 = K0 / TK;
        const int ntile = max((T + TK - 1) / TK - jt0, 0);
        const int ndiag = min(ntile, BKW / TK);              // tiles that touch the diagonal band
        float cn[2][2];                                      // [subtile][ca, cb] of the next tile
        auto load_carries = [&](int jt) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int j = jt * TK + 32 * u + n;
                // rows past T: an infinite carry gives A = 0 and G = 0, and with cb = 0 also dZ = 0
                cn[u][0] = (j < T && wave_live) ? cag[j] : INFINITY;   // a dead wave's rows lie outside the arrays
                cn[u][1] = (j < T && wave_live) ? cbg[j] : 0.0f;
            }
        };
        if (ntile > 0) {
            load_carries(jt0);
            stage_tile<D, false>(Qg, Gg, jt0, T, smem, goff, wave, lane);
        }
        float cc[2][2];
        auto begin_iter = [&](int it) __attribute__((always_inline)) {
            dma_wait<0>();
            barrier_nofence();
#pragma unroll
            for (int u = 0; u < 2; ++u) { cc[u][0] = cn[u][0]; cc[u][1] = cn[u][1]; }
            if (it + 1 < ntile) load_carries(jt0 + it + 1);
            stage_tile<D, false>(Qg, Gg, it + 1 < ntile ? jt0 + it + 1 : jt0, T, smem + ((it + 1) & 1) * C::STAGE, goff, wave, lane);
            return (const char*)(smem + (it & 1) * C::STAGE);
        };
        int it = 0;
        for (; it < ndiag; ++it) {
            const char* sp = begin_iter(it);
            if (wave_live) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int j0 = (jt0 + it) * TK + 32 * u;
                    if (j0 == k0) subtile(bc<true>{}, sp + u * 32 * C::ROW, cc[u][0], cc[u][1]);
                    else if (j0 > k0 && j0 < T) subtile(bc<false>{}, sp + u * 32 * C::ROW, cc[u][0], cc[u][1]);
                }
            }
        }
        for (; it < ntile; ++it) {
            const char* sp = begin_iter(it);
            if (wave_live) {
                const int j0 = (jt0 + it) * TK;
                subtile(bc<false>{}, sp, cc[0][0], cc[0][1]);
                if (j0 + 32 < T) subtile(bc<false>{}, sp + 32 * C::ROW, cc[1][0], cc[1][1]);
            }
        }
        dma_wait<0>();
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
                        dKg[(long)key * D + 32 * b + n] = dkacc[b][r] * scale;
                        dVg[(long)key * D + 32 * b + n] = dvacc[b][r];
                    }
                }
            }
        }
        if constexpr (!SLOW) {
            if (__builtin_amdgcn_ballot_w64(dirty) != 0 && lane == 0) atomicOr(&s_dirty, 1);
            __syncthreads();
            if (tid == 0) flags[bh * nkb_arg + kb] = s_dirty;
        }
    }
}

// ------------------------------------------------------------------ dK / dV kernel, paired waves
// The same computation with eight waves per workgroup, two per 32-key strip, for d = 128.
// There one wave that holds both accumulators (128 registers) and both stationary operands
// (64) fills a SIMD's register file alone, and a lone wave cannot hide its own latencies.
// Here the two waves of a strip split the work so that each needs one accumulator only:
//   - "front": each takes one 32-query subtile of every 64-row tile through S^T, P^T and the
//     element-wise path and writes A and dZ (bf16) row-wise into the strip's LDS scratch;
//   - "back": role 0 accumulates dV += A^T dO and role 1 accumulates dK += dZ^T Q over both
//     subtiles, reading the transposed operands from the scratch.
// No arithmetic is duplicated.  The back of a tile is taken one barrier interval after its
// front, together with the front of the next tile: one workgroup barrier per tile, and in the
// steady state a wave's interval is one block of code in which the matrix instructions of the
// back are issued between the vector instructions of the front's element-wise path (step()).
// Price: the Q/dO tile of the interval before must stay in LDS (three tile buffers) and the
// A/dZ scratch is double buffered; with compact scratch rows (64 B, xor-swizzled) that is
// exactly the 160 KB of a CU at d = 128.  Two waves per SIMD.
// The steady-state intervals run in a loop of their own in which LDS addresses rotate through
// registers and global pointers advance by constants: with one barrier per interval all eight
// waves do their loop bookkeeping at the same time, and a hundred dependent scalar instructions
// there cost about 500 clocks per interval.
// Measured against the predecessor of this kernel (front and back as two phases with a
// barrier each, padded scratch rows): 1.35 -> 1.29 ms at B8 H16 T4096, 1.20 with the
// steady-state loop.  Also measured:
// the two roles taking front and back in opposite order within an interval (so that one
// wave of a SIMD is in its vector phase while the other is in its matrix phase) is slower,
// 1.47 ms: the compiler then copies the accumulator (64 registers) on every switch.
constexpr int NW2 = 8;
constexpr int NTHREADS2 = 64 * NW2;

template <int D> struct Dkv3Cfg {
    static constexpr int NBUF = 3;
    static constexpr int T_OFF = NBUF * StageCfg<D>::STAGE;  // after the tile buffers
    static constexpr int M_BYTES = 32 * 64;                  // one 32x32 bf16 matrix
    static constexpr int W_BYTES = 2 * M_BYTES;              // A and dZ of one wave's subtile
    static constexpr int SCR_BUF = NW2 * W_BYTES;            // the eight waves' subtiles of one tile
    static constexpr int LDS_BYTES = T_OFF + 2 * SCR_BUF;
    static constexpr int LOADS = StageCfg<D>::TILE / 1024;
    static constexpr int NPW = (LOADS + NW2 - 1) / NW2;
};

template <int D, bool SLOW, bool GQA, bool VL>
__global__ void __launch_bounds__(NTHREADS2, 1)
bwd_dkv_pair_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                    const uint16_t* __restrict__ v, const uint16_t* __restrict__ dout,
                    const float* __restrict__ ca, const float* __restrict__ cb,
                    float* __restrict__ dk, float* __restrict__ dv, int* __restrict__ flags,
                    int T_arg, int BH, int H, int G_arg, int nkb_arg, int nt32, const int* __restrict__ cu, int Ttot)
{
    using C = StageCfg<D>;
    using CK = Dkv3Cfg<D>;
    static_assert(CK::LDS_BYTES <= 160 * 1024, "LDS budget");
    const int G = GQA ? G_arg : 1;                      // query heads per kv head
    __shared__ __attribute__((aligned(1024))) char smem[CK::LDS_BYTES];

    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const int npair = (nkb_arg + 1) >> 1;
    const long bh = xcd + 8L * (slot / npair);
    const int pidx = slot % npair;
    if (bh >= BH) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int strip = wave & 3;             // which 32 keys of the block
    const int role = wave >> 2;             // the subtile of every tile this wave fronts; 0 accumulates dV, 1 dK
    const int n = lane & 31, hh = lane >> 5;
    const int gg = lane >> 4, li = lane & 15;

    KvHead kh;
    if (!kv_head<D, VL>(kh, bh, pidx, T_arg, nkb_arg, H, G, nt32, cu, Ttot)) return;
    const int T = kh.T, nkb = kh.nkb;
    const long base = kh.base, qrow0 = kh.qrow0, qrow_step = kh.qrow_step;
    const long cbase = kh.cbase, cbase_step = kh.cbase_step, cstride = kh.cstride;
    const uint16_t* Qg = nullptr;
    const uint16_t* Gg = nullptr;

    // Per-lane LDS offsets inside a 32-row Q / dO subtile.  The swizzle xors the chunk index,
    // and the chunk indices a lane reads differ in bits the swizzle leaves alone, so one
    // offset per access pattern is kept and the others follow by xor with a constant:
    //   B-operand read of chunk pair s (row = query n):        boff0 ^ (s << 5)
    //   transposing read of column block b, row group t:       qtr0[t] ^ (b << 6)
    const uint32_t boff0 = tile_off_nat<D>(n, hh);
    uint32_t qtr0[2];
    {
        const int row_l = 8 * (gg >> 1) + (li >> 2);
        const int cl = 2 * (gg & 1) + ((li & 3) >> 1);
#pragma unroll
        for (int t = 0; t < 2; ++t) qtr0[t] = tile_off_nat<D>(row_l + 4 * t, cl) + 8 * (li & 1);
    }
    int goff[CK::NPW];
#pragma unroll
    for (int i = 0; i < CK::NPW; ++i) {
        const int row = (wave + NW2 * i) * C::BLK_ROWS + lane / C::CPR;
        goff[i] = (row * D + (((lane % C::CPR) ^ swz_nat<D>(row)) << 3)) * 2;
    }
    const uint32_t smem0 = lds_offset(smem);
    auto stage = [&](int jt, char* sp) __attribute__((always_inline)) {
        if ((jt + 1) * TK <= T) {                           // all 64 rows exist
            const uint16_t* xb = Qg + (long)jt * TK * D;
            const uint16_t* yb = Gg + (long)jt * TK * D;
#pragma unroll
            for (int i = 0; i < CK::NPW; ++i)
                if (wave + NW2 * i < CK::LOADS) {
                    dma16_to_lds_saddr(xb, goff[i], sp + (wave + NW2 * i) * 1024);
                    dma16_to_lds_saddr(yb, goff[i], sp + C::TILE + (wave + NW2 * i) * 1024);
                }
        } else {                                            // rows past T are clamped (their results are masked)
#pragma unroll
            for (int i = 0; i < CK::NPW; ++i)
                if (wave + NW2 * i < CK::LOADS) {
                    const int row = (wave + NW2 * i) * C::BLK_ROWS + lane / C::CPR;
                    const int c = (lane % C::CPR) ^ swz_nat<D>(row);
                    const long gr = min(jt * TK + row, T - 1);
                    dma16_to_lds(Qg + gr * D + c * 8, sp + (wave + NW2 * i) * 1024);
                    dma16_to_lds(Gg + gr * D + c * 8, sp + C::TILE + (wave + NW2 * i) * 1024);
                }
        }
    };
    // scratch: [tile parity][strip][subtile][A, dZ][32 rows of 64 B]
    const uint32_t scr = smem0 + CK::T_OFF + strip * 2 * CK::W_BYTES;
    const uint32_t sw_off = scr_off(n, 2 * hh);                                  // writes: row = query n; second chunk: ^ 16
    uint32_t st_off[2];                                                          // transposing reads
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int row = 8 * (gg >> 1) + (li >> 2) + 4 * t;
        st_off[t] = scr_off(row, 2 * (gg & 1) + ((li & 3) >> 1)) + 8 * (li & 1);
    }

    const float scale = 1.0f / sqrtf((float)D);
    const float c2 = SB_LOG2E * scale;

    bf16x8 kf[D / 16], vf[D / 16];          // A operands: the strip's K and V rows (MFMA row n <- key perm_row(n))
    f32x16 acc[D / 32];                     // dV (role 0) or dK (role 1) of the strip's 32 keys
    const float* cag = nullptr;
    const float* cbg = nullptr;
    bool dirty = false;                     // a chain of this lane left its range (fast variant)

    // this wave's subtile of a tile: logits, dO.v, element-wise path; A and dZ to the scratch
    // qtile: LDS address of the subtile's Q rows (its dO rows lie C::TILE further); sc: LDS
    // address of this strip's scratch for the tile
    auto front = [&](auto mask_c, uint32_t qtile, uint32_t sc, float car, float cbl) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_c)::value;
        if (MASK && n == 0) {               // sees none of the subtile's keys; its carries may be unwritten
            car = 0.0f;
            cbl = 0.0f;
        }
        const uint32_t qa = qtile + boff0;
        u32x4 qw[D / 16], gw[D / 16];
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            qw[s] = lds_load16(qa ^ (s << 5));
            gw[s] = lds_load16((qa ^ (s << 5)) + C::TILE);
        }
        f32x16 sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[r] = 0.0f; pacc[r] = 0.0f; }
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], __builtin_bit_cast(bf16x8, qw[s]), sacc, 0, 0, 0);
            pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], __builtin_bit_cast(bf16x8, gw[s]), pacc, 0, 0, 0);
        }
        SubtileOut so;
        if constexpr (SLOW) {
            subtile_math_log<false, MASK>(so, sacc, pacc, car, cbl, c2, n, hh);
        } else {
            Chain ch;
            dirty |= !subtile_stage1<MASK, SIGMA_DKV>(ch, sacc, c2, n, hh);
            subtile_stage2<false, true>(so, ch, pacc, car, cbl, hh);
        }
        const uint32_t w = sc + role * CK::W_BYTES + sw_off;
        lds_store16(w, so.pa[0]);
        lds_store16(w ^ 16, so.pa[1]);
        lds_store16(w + CK::M_BYTES, so.pz[0]);
        lds_store16((w ^ 16) + CK::M_BYTES, so.pz[1]);
    };
    // this wave's accumulator += (A or dZ of subtile u)^T (dO or Q rows of subtile u);
    // tile, sc: LDS addresses of the tile buffer and of this strip's scratch for the tile
    auto back = [&](uint32_t tile, uint32_t sc, int u) __attribute__((always_inline)) {
        const uint32_t m = sc + u * CK::W_BYTES + role * CK::M_BYTES;
        const uint32_t x = tile + (role == 0 ? C::TILE : 0) + u * 32 * C::ROW;
        const uint32_t x0 = x + qtr0[0], x1 = x + qtr0[1];
        bf16x8 mt[2], op[D / 16];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) mt[s2] = tr_pair_at(m + st_off[0] + (16 * s2) * 64, m + st_off[1] + (16 * s2) * 64);
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const int ro = (16 * s2) * C::ROW;
                op[2 * b + s2] = tr_pair_at((x0 ^ (b << 6)) + ro, (x1 ^ (b << 6)) + ro);
            }
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mt[s2], op[2 * b + s2], acc[b], 0, 0, 0);
    };

    // front of this wave's subtile (Q rows at qtile) and back of the tile before (buffer ptile,
    // scratch scp), unmasked and complete, written as one block so that the matrix
    // instructions of one part can be issued between the vector instructions of the other.
    // xn, yn: Q and dO rows of the tile to stage meanwhile, spn: its LDS buffer.
    // The wave's priority falls from part to part: of the two waves of a SIMD the one that is
    // behind wins the arbitration, so they reach the barrier closer together.
    auto step = [&](uint32_t qtile, uint32_t sc, uint32_t ptile, uint32_t scp, float car, float cbl,
                    const uint16_t* xn, const uint16_t* yn, const char* spn) __attribute__((always_inline)) {
        const uint32_t qa = qtile + boff0;
        // part A: logits
        __builtin_amdgcn_s_setprio(3);
        u32x4 qw[D / 16], gw[D / 16];
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qw[s] = lds_load16(qa ^ (s << 5));
        f32x16 sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[r] = 0.0f; pacc[r] = 0.0f; }
        // the staging loads go out between the matrix instructions
        static_assert(CK::LOADS == 2 * NW2, "two staging loads per wave and matrix");
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], __builtin_bit_cast(bf16x8, qw[s]), sacc, 0, 0, 0);
            if (s == 0) dma16_to_lds_saddr(xn, goff[0], spn + wave * 1024);
            if (s == 2) dma16_to_lds_saddr(yn, goff[0], spn + C::TILE + wave * 1024);
            if (s == 4) dma16_to_lds_saddr(xn, goff[1], spn + (wave + NW2) * 1024);
            if (s == 6) dma16_to_lds_saddr(yn, goff[1], spn + C::TILE + (wave + NW2) * 1024);
        }
#pragma unroll
        for (int s = 0; s < D / 16; ++s) gw[s] = lds_load16((qa ^ (s << 5)) + C::TILE);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(2);
        // part B: the chain of the logits (vector) beside dO.v and the back of subtile 0 (matrix)
        Chain ch;
        dirty |= !subtile_stage1<false, SIGMA_DKV>(ch, sacc, c2, n, hh);
#pragma unroll
        for (int s = 0; s < D / 16; ++s)
            pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], __builtin_bit_cast(bf16x8, gw[s]), pacc, 0, 0, 0);
        back(ptile, scp, 0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
        // part C: A, G, dZ (vector) beside the back of subtile 1 (matrix)
        SubtileOut so;
        subtile_stage2<false, true>(so, ch, pacc, car, cbl, hh);
        back(ptile, scp, 1);
        const uint32_t w = sc + role * CK::W_BYTES + sw_off;
        lds_store16(w, so.pa[0]);
        lds_store16(w ^ 16, so.pa[1]);
        lds_store16(w + CK::M_BYTES, so.pz[0]);
        lds_store16((w ^ 16) + CK::M_BYTES, so.pz[1]);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
    };

    for (int part = 0; part < 2; ++part) {
        const int kb = part == 0 ? pidx : nkb - 1 - pidx;    // small kb = most later queries = first
        if (part == 1 && 2 * pidx == nkb - 1) break;
        if (SLOW && flags[bh * nkb_arg + kb] == 0) continue; // only the blocks the fast variant flagged
        const int K0 = kb * BKW;
        const int k0 = K0 + strip * 32;                      // the strip's 32 keys
        const int kt32 = k0 >> 5;
        const bool live = k0 < T;
        dirty = false;
        barrier_lds();                                       // everyone is done with the LDS of the block before
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
#pragma unroll
        for (int s = 0; s < D / 16; ++s) { asm volatile("" :: "v"(kf[s])); asm volatile("" :: "v"(vf[s])); }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;

        // the query heads of the group one after the other, into the same accumulators
        for (int g = 0; g < G; ++g) {
        Qg = q + (qrow0 + g * qrow_step) * D;
        Gg = dout + (qrow0 + g * qrow_step) * D;
        cag = ca + cbase + g * cbase_step + kt32 * cstride;
        cbg = cb + cbase + g * cbase_step + kt32 * cstride;
        if (g > 0) barrier_lds();                            // everyone is done with the LDS of the head before

        // ---- sweep over 64-row query tiles, from the block's diagonal to the end.  Interval
        // `it` (between two barriers) holds the front of tile jt0 + it (buffer it % 3, scratch
        // it & 1) and the back of tile jt0 + it - 1; the staging loads of tile jt0 + it + 1 are
        // issued at its start, after the carries of that tile (vector memory operations
        // complete in order, so the carries must not queue behind the staging loads).
        const int jt0 = K0 / TK;
        const int ntile = max((T + TK - 1) / TK - jt0, 0);
        const int ndiag = min(ntile, BKW / TK);              // tiles that touch the diagonal band
        float cn0 = INFINITY, cn1 = 0.0f;                    // ca, cb of this wave's subtile of the next tile
        auto load_carries = [&](int jt) __attribute__((always_inline)) {
            const int j = jt * TK + 32 * role + n;
            // rows past T: an infinite carry gives A = 0 and G = 0, and with cb = 0 also dZ = 0
            cn0 = (j < T && live) ? cag[j] : INFINITY;       // a dead strip's rows lie outside the arrays
            cn1 = (j < T && live) ? cbg[j] : 0.0f;
        };
        if (ntile > 0) {
            load_carries(jt0);
            stage(jt0, smem);
        }
        // steady state (the intervals hot_begin .. hot_end - 1): the strip is live, tile `it` is past
        // the diagonal band and complete, and the next tile is complete or does not exist
        const int nfull = max(T / TK - jt0, 0);
        const int hot_begin = ndiag + 1;
        const int hot_end = (SLOW || !live) ? 0 : (nfull == ntile ? ntile : nfull - 1);
        int it = 0;
        while (it <= ntile) {
            if (it == hot_begin && it < hot_end) {
                // LDS addresses of the tile buffers of tiles it, it - 1, it + 1 and of the scratch
                // of tiles it, it - 1; they rotate, nothing is recomputed.  The tile staged in an
                // interval is tile it + 1, or, after the last one, that tile once more (never read).
                uint32_t a_cur = smem0 + (it % 3) * C::STAGE, a_prev = smem0 + ((it + 2) % 3) * C::STAGE;
                uint32_t a_next = smem0 + ((it + 1) % 3) * C::STAGE;
                uint32_t s_cur = scr + (it & 1) * CK::SCR_BUF, s_prev = scr + ((it + 1) & 1) * CK::SCR_BUF;
                const int tn = min(it + 1, ntile - 1);
                const uint16_t* xn = Qg + (long)(jt0 + tn) * TK * D;
                const uint16_t* yn = Gg + (long)(jt0 + tn) * TK * D;
                const float* cap = cag + (jt0 + tn) * TK + 32 * role + n;
                const float* cbp = cbg + (jt0 + tn) * TK + 32 * role + n;
                for (; it < hot_end; ++it) {
                    dma_wait<0>();
                    barrier_lds();
                    const float car = cn0, cbl = cn1;
                    cn0 = *cap;
                    cn1 = *cbp;
                    step(a_cur + role * 32 * C::ROW, s_cur, a_prev, s_prev, car, cbl, xn, yn, smem + (a_next - smem0));
                    const int adv = it + 2 < ntile ? TK : 0;
                    xn += adv * D;
                    yn += adv * D;
                    cap += adv;
                    cbp += adv;
                    const uint32_t t = a_prev;
                    a_prev = a_cur;
                    a_cur = a_next;
                    a_next = t;
                    const uint32_t u = s_prev;
                    s_prev = s_cur;
                    s_cur = u;
                }
                continue;
            }
            const int bcur = it % 3, bprev = (it + 2) % 3, bnext = (it + 1) % 3;   // buffers of tiles it, it - 1, it + 1
            dma_wait<0>();
            barrier_lds();        // tile `it` has landed, the scratch of tile it-1 is complete, tile it-2 is free
            const float car = cn0, cbl = cn1;
            if (it + 1 < ntile) {
                load_carries(jt0 + it + 1);
                stage(jt0 + it + 1, smem + bnext * C::STAGE);
            }
            const int jbase = (jt0 + it) * TK;
            const uint32_t qt = smem0 + bcur * C::STAGE + role * 32 * C::ROW;
            const uint32_t sc = scr + (it & 1) * CK::SCR_BUF;
            const uint32_t spp = smem0 + bprev * C::STAGE;
            const uint32_t scp = scr + ((it + 1) & 1) * CK::SCR_BUF;
            const int j0 = jbase + 32 * role;
            if (it < ntile && live && j0 < T) {
                if (it < ndiag) {
                    if (j0 == k0) front(bc<true>{}, qt, sc, car, cbl);
                    else if (j0 > k0) front(bc<false>{}, qt, sc, car, cbl);
                } else {
                    front(bc<false>{}, qt, sc, car, cbl);
                }
            }
            if (it >= 1 && live) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int ju = jbase - TK + 32 * u;
                    if (ju >= k0 && ju < T) back(spp, scp, u);
                }
            }
            ++it;
        }
        }

        // ---- store: acc[b][r] is key row k0 + 8*(r/4) + 4*hh + r%4, column 32b + n
        if (live) {
            float* out = (role == 0 ? dv : dk) + base;
            const float f = role == 0 ? 1.0f : scale;
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = k0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (key < T) out[(long)key * D + 32 * b + n] = acc[b][r] * f;
                }
            }
        }
        if constexpr (!SLOW) {
            // the block's flag: any chain of any wave out of range.  The tile buffers are free by now.
            int* s_dirty = reinterpret_cast<int*>(smem);
            barrier_lds();
            if (tid == 0) *s_dirty = 0;
            __syncthreads();
            if (__builtin_amdgcn_ballot_w64(dirty) != 0 && lane == 0) atomicOr(s_dirty, 1);
            __syncthreads();
            if (tid == 0) flags[bh * nkb_arg + kb] = *s_dirty;
        }
    }
}

// ------------------------------------------------------------------ gradient of the remainder bias
// dr[h][c] = sum over the batch and the rows j of exp(m_j) dO[j][c] (Appendix C: the
// output holds (stick left of row j) * r_h).  Two deterministic steps: per (batch entry,
// head, 128-row chunk) partial sums, then one thread per (h, c) adds them in a fixed order.
constexpr int DR_ROWS = 128;

template <int D, bool VL>
__global__ void __launch_bounds__(NTHREADS)
bwd_drb_partial_kernel(const float* __restrict__ m, const uint16_t* __restrict__ dout,
                       float* __restrict__ part, int T_arg, int nchunk, int H,
                       const int* __restrict__ cu, int Ttot)
{
    constexpr int CP = D / 2;                 // column pairs
    constexpr int RG = NTHREADS / CP;         // row groups
    __shared__ float red[RG][D];
    const long bh = blockIdx.x / nchunk;      // one grid dimension: no 65535 limit on the heads
    const int chunk = blockIdx.x % nchunk;
    const int cp = threadIdx.x % CP, rg = threadIdx.x / CP;
    int T = T_arg;
    long row0 = bh * (long)T;
    if constexpr (VL) {                       // bh = sequence * H + head; chunks past the sequence's end give 0
        const int c0 = cu[bh / H];
        T = c0 < 0 ? 0 : min(min(cu[bh / H + 1], Ttot) - c0, T_arg);
        row0 = (bh % H) * (long)Ttot + c0;
    }
    const int j1 = min(T, (chunk + 1) * DR_ROWS);
    float a0 = 0.0f, a1 = 0.0f;
    for (int j = chunk * DR_ROWS + rg; j < j1; j += RG) {
        const float w = __expf(m[row0 + j]);
        const uint32_t g = *reinterpret_cast<const uint32_t*>(dout + (row0 + j) * D + 2 * cp);
        a0 += w * __builtin_bit_cast(float, g << 16);
        a1 += w * __builtin_bit_cast(float, g & 0xffff0000u);
    }
    red[rg][2 * cp] = a0;
    red[rg][2 * cp + 1] = a1;
    __syncthreads();
    if (threadIdx.x < D) {
        float s = 0.0f;
#pragma unroll
        for (int g = 0; g < RG; ++g) s += red[g][threadIdx.x];
        part[(bh * nchunk + chunk) * D + threadIdx.x] = s;
    }
}

template <int D>
__global__ void __launch_bounds__(D)
bwd_drb_sum_kernel(const float* __restrict__ part, float* __restrict__ drb, int B, int H, int nchunk)
{
    const int h = blockIdx.x, c = threadIdx.x;
    float s = 0.0f;
    for (int b = 0; b < B; ++b) {
        const float* p = part + ((long)(b * (long)H + h) * nchunk) * D + c;
        float sb = 0.0f;
        for (int ch = 0; ch < nchunk; ++ch) sb += p[(long)ch * D];
        s += sb;
    }
    drb[h * D + c] = s;
}

// workspace layout: ca[BH][nt32][T], cb[BH][nt32][T] (fp32; [H][nt32][Ttot] for a packed
// batch), then the per-block flags of the two kernels (int): [BH][nqb], [BH][nkb], then the
// partial sums of the remainder-bias gradient (fp32): [BH][nchunk][D].  B, T: batch size and
// length, or for a packed batch (VL) the number of sequences and the longest length.
template <int D, bool VL>
hipError_t launch_one(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                      const float* m, const uint16_t* dout, float* dq, float* dk, float* dv,
                      float* drb, float* workspace, int B, int H, int Hkv, int T, int passes, hipStream_t stream,
                      const int* cu, int Ttot)
{
    const int BH = B * H;
    const int BHkv = B * Hkv;
    const int G = H / Hkv;
    const int nt32 = (T + 31) / 32;
    const int nqb = (T + BQ - 1) / BQ;
    const int nkb = (T + BKW - 1) / BKW;
    const long ncarry = VL ? (long)H * nt32 * Ttot : (long)BH * nt32 * T;
    float* ca = workspace;
    float* cb = ca + ncarry;
    int* fq = reinterpret_cast<int*>(cb + ncarry);
    int* fk = fq + (long)BH * nqb;
    float* part = reinterpret_cast<float*>(fk + (long)BH * nkb);
    const int nchunk = (T + DR_ROWS - 1) / DR_ROWS;
    const long bq = 8L * ((BH + 7) / 8) * ((nqb + 1) / 2);
    const long bk = 8L * ((BHkv + 7) / 8) * ((nkb + 1) / 2);
    // checked before the first launch, so that an error leaves nothing enqueued
    if (bq > 0x7fffffffL || bk > 0x7fffffffL || nchunk * (long)BH > 0x7fffffffL) return hipErrorInvalidValue;
    if (bq == 0) return hipSuccess;
    hipError_t e = hipSuccess;
#define SB_DQ(SLOWV, RBV)                                                                                       \
    hipLaunchKernelGGL((bwd_dq_kernel<D, SLOWV, RBV, VL>), dim3((unsigned)bq), dim3(NTHREADS), 0, stream,       \
                       q, k, v, rb, m, dout, dq, ca, cb, fq, T, BH, H, G, nqb, nt32, cu, Ttot);                 \
    if ((e = hipGetLastError()) != hipSuccess) return e
// d = 128 takes the paired-wave kernel (two waves per SIMD instead of one); smaller head
// dimensions leave room for two workgroups of the one-wave-per-strip kernel per CU, which
// is faster there (measured).
#define SB_DKV(SLOWV, GQAV)                                                                                     \
    if constexpr (D == 128)                                                                                     \
        hipLaunchKernelGGL((bwd_dkv_pair_kernel<D, SLOWV, GQAV, VL>), dim3((unsigned)bk), dim3(NTHREADS2), 0,   \
                           stream, q, k, v, dout, ca, cb, dk, dv, fk, T, BHkv, H, G, nkb, nt32, cu, Ttot);      \
    else                                                                                                        \
        hipLaunchKernelGGL((bwd_dkv_kernel<D, SLOWV, GQAV, VL>), dim3((unsigned)bk), dim3(NTHREADS), 0,         \
                           stream, q, k, v, dout, ca, cb, dk, dv, fk, T, BHkv, H, G, nkb, nt32, cu, Ttot);      \
    if ((e = hipGetLastError()) != hipSuccess) return e
    if (passes & 1) {
        if (rb) { SB_DQ(false, true); SB_DQ(true, true); }
        else    { SB_DQ(false, false); SB_DQ(true, false); }
        if (drb) {
            hipLaunchKernelGGL((bwd_drb_partial_kernel<D, VL>), dim3((unsigned)(nchunk * (long)BH)), dim3(NTHREADS), 0,
                               stream, m, dout, part, T, nchunk, H, cu, Ttot);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            hipLaunchKernelGGL((bwd_drb_sum_kernel<D>), dim3((unsigned)H), dim3(D), 0, stream,
                               part, drb, B, H, nchunk);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
    }
    if (passes & 2) {
        // a packed batch always takes the grouped variant (a group of one included)
        if (VL || G > 1) { SB_DKV(false, true); SB_DKV(true, true); }
        else             { SB_DKV(false, false); SB_DKV(true, false); }
    }
#undef SB_DQ
#undef SB_DKV
    return e;
}

}  // namespace

size_t bwd_workspace_bytes(int B, int H, int T, int d)
{
    const size_t nt32 = (size_t)(T + 31) / 32;
    const size_t nblk = (size_t)(T + BQ - 1) / BQ + (size_t)(T + BKW - 1) / BKW;
    const size_t nchunk = (size_t)(T + DR_ROWS - 1) / DR_ROWS;
    return (2 * sizeof(float) * nt32 * T + sizeof(int) * nblk + sizeof(float) * nchunk * d) * (size_t)B * H;
}

size_t bwd_varlen_workspace_bytes(int nseq, int H, int Ttot, int max_T, int d)
{
    const size_t nt32 = (size_t)(max_T + 31) / 32;
    const size_t nblk = (size_t)(max_T + BQ - 1) / BQ + (size_t)(max_T + BKW - 1) / BKW;
    const size_t nchunk = (size_t)(max_T + DR_ROWS - 1) / DR_ROWS;
    return 2 * sizeof(float) * nt32 * (size_t)Ttot * H +
           (sizeof(int) * nblk + sizeof(float) * nchunk * d) * (size_t)nseq * H;
}

hipError_t launch_bwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                           const float* m, const uint16_t* dout, float* dq, float* dk, float* dv,
                           float* drb, float* workspace,
                           int B, int H, int Hkv, int T, int d, int passes, hipStream_t stream)
{
#define SB_BWD(DD) launch_one<DD, false>(q, k, v, rb, m, dout, dq, dk, dv, drb, workspace, B, H, Hkv, T, passes, stream, nullptr, 0)
    if (d == 32) return SB_BWD(32);
    if (d == 64) return SB_BWD(64);
    return SB_BWD(128);
#undef SB_BWD
}

hipError_t launch_bwd_bf16_varlen(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                                  const float* m, const uint16_t* dout, float* dq, float* dk, float* dv,
                                  float* drb, float* workspace, const int* cu, int nseq, int H, int Hkv,
                                  int Ttot, int max_T, int d, hipStream_t stream)
{
#define SB_BWD(DD) launch_one<DD, true>(q, k, v, rb, m, dout, dq, dk, dv, drb, workspace, nseq, H, Hkv, max_T, 3, stream, cu, Ttot)
    if (d == 32) return SB_BWD(32);
    if (d == 64) return SB_BWD(64);
    return SB_BWD(128);
#undef SB_BWD
}

}  // namespace sb
