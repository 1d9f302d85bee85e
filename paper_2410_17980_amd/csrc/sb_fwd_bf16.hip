// bf16 forward of causal stick-breaking attention on the gfx950 matrix cores.
//
// Work split.  A workgroup (4 wavefronts) owns 128*NG query rows of one (batch,
// head); each wavefront owns NG groups of 32 of them and keeps their Q fragments
// in registers (NG = 2 at d = 128: every K / V fragment read from LDS then feeds
// two MFMAs, and the wave has two independent element-wise streams to interleave
// with the matrix pipe; the 512-register budget of one wave per SIMD holds it).
// Keys are swept in 32-row subtiles from the diagonal towards key 0, the order
// Algorithm 1 prescribes: the weight of key i needs the sum of softplus(z) over
// the keys between i and the query (Eq. 2), so that sum is carried per query row
// from subtile to subtile (the vector `a` of Algorithm 1).
//
// Layout inside a wavefront.  Logits are formed transposed, S^T = K Q^T, with
// the 32x32x16 bf16 MFMA: A operand = 32 key rows from LDS, B operand = the
// wave's 32 query rows.  In the accumulator a lane owns ONE query column
// (lane % 32) and 16 key rows; the LDS row fed to MFMA row rho is perm_row(rho),
// which makes those 16 keys consecutive (lanes 0-31: keys 0..15 of the subtile,
// lanes 32-63: keys 16..31).  The right-to-left cumulative sum of softplus is
// then a serial add inside the lane plus one exchange with the partner lane, and
// the row total for the carry falls out of the scan.  The weights feed the
// second MFMA (O += A V) straight from registers: the accumulator's per-lane key
// order is a valid K-dimension order for the A operand, and V is read from LDS
// with the transposing load in that same key order.
//
// Software pipeline.  Step t of a wave runs, in one straight-line block,
//     MFMA : O += A(t-1) V(t-1)   and   S(t+1) = K(t+1) Q^T
//     VALU : A(t) from S(t)       (softplus, scan, exp2, bf16 convert)
// so the matrix pipe works on the neighbours of the subtile whose element-wise
// path is on the vector pipe; the instruction streams are interleaved with
// scheduling barriers.  K and V subtiles are brought in by direct global->LDS
// loads into four-slot rings (subtile j lives in slot j&3), two steps ahead of
// their use: step t issues the loads of K(t+3) and V(t+1) and, before its closing
// barrier, waits only for the loads issued in step t-1 (K(t+2), V(t)), so a load
// has two full steps to land.
//
// Arithmetic.  Everything between the two MFMAs is fp32 in the base-2 domain:
// x = z*log2(e), sp2(x) = log2(1 + 2^x), A = 2^(x - cumsum sp2 - carry); see
// sb_mma.h.  No product of probabilities is formed.
#include <cstdlib>
#include <type_traits>

#include "sb_kernels.h"
#include "sb_mma.h"

namespace sb {
namespace {

constexpr int NTHREADS = 256;

template <int D> struct FwdCfg {
    static constexpr int ROW = D * 2;                   // bytes per tile row (unpadded, swizzled)
    static constexpr int SUB = 32 * ROW;                // one 32-row subtile
    static constexpr int NSLOT = 4;                     // ring depth (subtile j in slot j & 3)
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = NSLOT * SUB;
    static constexpr int LDS_BYTES = 2 * NSLOT * SUB;
    static constexpr int CPR = ROW / 16;                // 16 B chunks per row
    static constexpr int BLK_ROWS = 1024 / ROW;         // rows written by one wave-wide 16 B/lane load
    static constexpr int NI = SUB / 1024 / 4;           // such loads per wave per subtile
};

template <bool B> using bc = std::integral_constant<bool, B>;
template <int I> using ic = std::integral_constant<int, I>;

template <int D, int NG, bool WRITE_M>
__global__ void __launch_bounds__(NTHREADS, NG == 1 ? 2 : 1)
fwd_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ m,
                int T, int BH, int nqb)
{
    using C = FwdCfg<D>;
    constexpr int BQ = 128 * NG;                        // query rows per workgroup
    constexpr int WQ = 32 * NG;                         // query rows per wave
    __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];

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
    const int n = lane & 31;          // query column inside the wave
    const int hh = lane >> 5;         // half-wave: keys 16*hh .. 16*hh+15 of a subtile
    const int gg = lane >> 4, li = lane & 15;
    const int q0 = qb * BQ + wave * WQ;
    const bool wave_live = q0 < T;

    const uint16_t* Qg = q + bh * (long)T * D;
    const uint16_t* Kg = k + bh * (long)T * D;
    const uint16_t* Vg = v + bh * (long)T * D;

    // ---- B operand of S^T = K Q^T: Q[q0 + 32g + n][16s + 8hh .. +7], s = 0..D/16-1
    bf16x8 qf[NG][D / 16];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int jq = min(q0 + 32 * g + n, T - 1);
        const u32x4* src = reinterpret_cast<const u32x4*>(Qg + (long)jq * D + 8 * hh);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qf[g][s] = __builtin_bit_cast(bf16x8, src[2 * s]);
    }
    // Make the compiler wait for the Q loads here, once: the staging loads below are
    // issued behind its back, and a wait for "all my loads" placed inside the loop
    // would also wait for those.
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int s = 0; s < D / 16; ++s) asm volatile("" :: "v"(qf[g][s]));

    // ---- per-lane LDS byte offsets inside a subtile
    int aoff[D / 16];                       // K rows as A operand: row perm_row(n), chunk 2s + hh
    {
        const int key_l = perm_row(n);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) aoff[s] = tile_off_perm<D>(key_l, 2 * s + hh);
    }
    int vtr[D / 32][2];                     // V through the transposing load: rows 16g + li/4 (+4t, +8s)
    {
        const int row_l = 16 * (gg >> 1) + (li >> 2);
        const int cl = 2 * (gg & 1) + ((li & 3) >> 1);
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                vtr[b][t] = tile_off_perm<D>(row_l + 4 * t, 4 * b + cl) + 8 * (li & 1);
    }

    // ---- direct global -> LDS staging of one 32-row subtile of K or V.
    // One instruction moves 16 B per lane to 1 KB of consecutive LDS; the swizzle is
    // applied on the global side: the lane whose LDS position is (row, physical chunk)
    // fetches the logical chunk that belongs there.  The per-lane byte offset inside
    // the subtile never changes, so the loop only moves a scalar base address.
    int goff[C::NI];
#pragma unroll
    for (int i = 0; i < C::NI; ++i) {
        const int row = (wave * C::NI + i) * C::BLK_ROWS + lane / C::CPR;
        goff[i] = (row * D + (((lane % C::CPR) ^ swz_perm<D>(row)) << 3)) * 2;
    }
    const int top_sub = (min(T, qb * BQ + BQ) - 1 + 31) / 32 - 1;   // topmost staged subtile (may be ragged)
    auto stage = [&](const uint16_t* g, int sidx, char* slot_ptr) __attribute__((always_inline)) {
        if (sidx != top_sub) {                      // all 32 rows exist
            const uint16_t* base = g + (long)sidx * 32 * D;
#pragma unroll
            for (int i = 0; i < C::NI; ++i)
                dma16_to_lds_saddr(base, goff[i], slot_ptr + (wave * C::NI + i) * 1024);
        } else {                                    // rows past T are clamped (they are masked by causality)
#pragma unroll
            for (int i = 0; i < C::NI; ++i) {
                const int row = (wave * C::NI + i) * C::BLK_ROWS + lane / C::CPR;
                const int c = (lane % C::CPR) ^ swz_perm<D>(row);
                const long gr = min(sidx * 32 + row, T - 1);
                dma16_to_lds(g + gr * D + c * 8, slot_ptr + (wave * C::NI + i) * 1024);
            }
        }
    };

    f32x16 oacc[NG][D / 32];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[g][b][r] = 0.0f;
    // pipeline registers: sbuf[0] = logits of subtile t, sbuf[1] = of subtile t+1;
    // pbuf[0] = weights of subtile t-1, pbuf[1] = of subtile t (as MFMA operands).
    // A step with static phase and odd parity uses them with the roles swapped.
    f32x16 sbuf[2][NG];
    bf16x8 pbuf[2][NG][2];
    float a[NG];                     // carried sum of sp2 over all keys right of the current subtile
#pragma unroll
    for (int g = 0; g < NG; ++g) a[g] = 0.0f;

    const float c2 = SB_LOG2E / sqrtf((float)D);

    // Element-wise path of one 32x32 subtile of group g: logits sin -> weights pout,
    // carry a_g updated.  Returns this lane's sum of sp2 (+inf / NaN if a 2^x overflowed
    // with SAFE = false).  With MASK, key 16hh + r is visible iff 16hh + r < lim.
    auto ew_group = [&](auto mask_c, auto safe_c, const f32x16& sin, bf16x8 (&pout)[2], float& a_g, int lim) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_c)::value, SAFE = decltype(safe_c)::value;
        float y[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) y[r] = sin[r] * c2;
        if constexpr (MASK) {
#pragma unroll
            for (int r = 0; r < 16; ++r) y[r] = (16 * hh + r < lim) ? y[r] : -INFINITY;
        }
        float run = 0.0f;
#pragma unroll
        for (int r = 15; r >= 0; --r) {
            run += SAFE ? sp2(y[r]) : sp2_fast(y[r]);
            y[r] -= run;                           // x - (sum of sp2 over this lane's keys r..15)
        }
        float tot_lo, tot_hi;
        both_halves(run, tot_lo, tot_hi);
        const float off = a_g + (hh == 0 ? tot_hi : 0.0f);
        a_g += tot_lo + tot_hi;
#pragma unroll
        for (int r = 0; r < 16; ++r) pout[r >> 3][r & 7] = (__bf16)fast_exp2(y[r] - off);
        return run;
    };

    // One pipeline step.  HAS_S: form S(t+1); HAS_PV: accumulate A(t-1) V(t-1);
    // HAS_EW: turn S(t) into A(t).  With MASK, key 16hh + r of the subtile is
    // visible to the lane's query of group g iff 16hh + r < lim0 + 32g.
    // PHASE = (t+1)&3 fixes the ring slots (and register roles) at compile time;
    // PHASE = -1 takes them from t and rotates the pipeline registers at the end.
    auto step = [&](auto has_pv, auto has_ew, auto has_s, auto mask, auto phase_c, int t, int lim0) __attribute__((always_inline)) {
        constexpr bool HAS_PV = decltype(has_pv)::value, HAS_EW = decltype(has_ew)::value;
        constexpr bool HAS_S = decltype(has_s)::value, MASK = decltype(mask)::value;
        constexpr int PHASE = decltype(phase_c)::value;
        constexpr int Q = PHASE < 0 ? 0 : (PHASE & 1);              // register parity
        const char* kslot = smem + C::K_OFF + (PHASE < 0 ? ((t + 1) & 3) : PHASE) * C::SUB;        // K(t+1)
        const char* vslot = smem + C::V_OFF + (PHASE < 0 ? ((t - 1) & 3) : ((PHASE + 2) & 3)) * C::SUB;   // V(t-1)
        f32x16 (&s_in)[NG] = sbuf[Q];
        f32x16 (&s_out)[NG] = sbuf[Q ^ 1];
        bf16x8 (&p_in)[NG][2] = pbuf[Q];
        bf16x8 (&p_out)[NG][2] = pbuf[Q ^ 1];

        if constexpr (HAS_S) {
            f32x16 acc[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[g][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(kslot + aoff[s]);
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), qf[g][s], acc[g], 0, 0, 0);
            }
#pragma unroll
            for (int g = 0; g < NG; ++g) s_out[g] = acc[g];
        }
        if constexpr (HAS_PV) {
            // O[q][dcol] += sum_keys A[q][key] V[key][dcol]; K-dim index 8h+e <-> key 16h + 8s + e
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const char* p = vslot + (8 * s) * C::ROW;
                    const bf16x8 vf = tr_pair(p + vtr[b][0], p + vtr[b][1]);
#pragma unroll
                    for (int g = 0; g < NG; ++g)
                        oacc[g][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_in[g][s], vf, oacc[g][b], 0, 0, 0);
                }
            }
        }
        if constexpr (HAS_EW) {
#pragma unroll
            for (int g = 0; g < NG; ++g) ew_group(bc<MASK>{}, bc<true>{}, s_in[g], p_out[g], a[g], lim0 + 32 * g);
            if constexpr (HAS_PV || HAS_S) {
                // interleave: one MFMA, then a slice of the element-wise stream
                constexpr int NMFMA = NG * ((HAS_PV ? D / 16 : 0) + (HAS_S ? D / 16 : 0));
                constexpr int SLICE = (130 * NG) / NMFMA;
#pragma unroll
                for (int i = 0; i < NMFMA; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x402, SLICE, 0);   // VALU incl. transcendental
                }
            }
        }
        if constexpr (PHASE < 0) {
            // rotate the pipeline registers
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if constexpr (HAS_S) sbuf[0][g] = sbuf[1][g];
                if constexpr (HAS_EW) { pbuf[0][g][0] = pbuf[1][g][0]; pbuf[0][g][1] = pbuf[1][g][1]; }
            }
        }
    };

    // ---- the steady-state step, scheduled by hand (one query group per wave).
    // The same work as step(PV, EW, S) above, laid out as 2*D/16 slots: each slot
    // issues the LDS reads of the MFMA two slots ahead, one MFMA (S and PV products
    // alternate, so consecutive links of the S accumulation chain are a slot
    // apart), and one or two chunks of the element-wise stream.  The element-wise
    // stream is ordered stage by stage over all 16 elements of the lane (scale,
    // 2^x, +1, log2, guarded scan, shift, 2^x, convert) rather than element by
    // element, so that no instruction waits on the one just before it; scheduling
    // barriers keep the compiler from folding it back.
    auto hot_step = [&](int t) __attribute__((always_inline)) {
        static_assert(NG == 1 || NG == 2, "");
        constexpr int NM = D / 16;                 // MFMAs of each product
        constexpr int NSLOT = 2 * NM;
        const char* kslot = smem + C::K_OFF + ((t + 1) & 3) * C::SUB;     // K(t+1)
        const char* vslot = smem + C::V_OFF + ((t - 1) & 3) * C::SUB;     // V(t-1)
        const f32x16& s_in = sbuf[0][0];
        bf16x8 (&p_in)[2] = pbuf[0][0];
        bf16x8 (&p_out)[2] = pbuf[1][0];

        u32x4 kop[NM];
        bf16x8 vop[NM];
        auto fetch = [&](auto ic_i) __attribute__((always_inline)) {
            constexpr int i = decltype(ic_i)::value;
            if constexpr (i < NSLOT) {
                if constexpr ((i & 1) == 0) {
                    kop[i / 2] = *reinterpret_cast<const u32x4*>(kslot + aoff[i / 2]);
                } else {
                    constexpr int j = i / 2, b = j / 2, sh = j % 2;
                    const char* p = vslot + (8 * sh) * C::ROW;
                    vop[j] = tr_pair(p + vtr[b][0], p + vtr[b][1]);
                }
            }
        };
        f32x16 acc;
        float x[16], w[16];
        float run = 0.0f, off = 0.0f;
        auto mfma = [&](auto ic_i) __attribute__((always_inline)) {
            constexpr int i = decltype(ic_i)::value;
            if constexpr ((i & 1) == 0) {
                constexpr int sI = i / 2;
                if constexpr (sI == 0) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kop[0]), qf[0][0], z, 0, 0, 0);
                } else {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kop[sI]), qf[0][sI], acc, 0, 0, 0);
                }
            } else {
                constexpr int j = i / 2, b = j / 2, sh = j % 2;
                oacc[0][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_in[sh], vop[j], oacc[0][b], 0, 0, 0);
            }
        };
        auto chunk = [&](auto ic_c) __attribute__((always_inline)) {
            constexpr int c = decltype(ic_c)::value;
            if constexpr (c == 0) {
#pragma unroll
                for (int r = 0; r < 16; ++r) x[r] = s_in[r] * c2;
            } else if constexpr (c == 1) {
#pragma unroll
                for (int r = 15; r >= 10; --r) w[r] = fast_exp2(x[r]);
            } else if constexpr (c == 2) {
#pragma unroll
                for (int r = 9; r >= 4; --r) w[r] = fast_exp2(x[r]);
            } else if constexpr (c == 3) {
#pragma unroll
                for (int r = 3; r >= 0; --r) w[r] = fast_exp2(x[r]);
#pragma unroll
                for (int r = 15; r >= 8; --r) w[r] += 1.0f;
            } else if constexpr (c == 4) {
#pragma unroll
                for (int r = 7; r >= 0; --r) w[r] += 1.0f;
#pragma unroll
                for (int r = 15; r >= 13; --r) w[r] = fast_log2(w[r]);
            } else if constexpr (c == 5) {
#pragma unroll
                for (int r = 12; r >= 7; --r) w[r] = fast_log2(w[r]);
            } else if constexpr (c == 6) {
#pragma unroll
                for (int r = 6; r >= 0; --r) w[r] = fast_log2(w[r]);
            } else if constexpr (c == 7 || c == 8 || c == 9) {
                constexpr int hi = c == 7 ? 15 : (c == 8 ? 10 : 5), lo = c == 7 ? 11 : (c == 8 ? 6 : 0);
#pragma unroll
                for (int r = hi; r >= lo; --r) w[r] = __builtin_amdgcn_fmed3f(w[r], x[r], 128.0f);   // sp2, overflow-proof
#pragma unroll
                for (int r = hi; r >= lo; --r) {
                    run += w[r];
                    x[r] -= run;                   // x - (sum of sp2 over this lane's keys r..15)
                }
            } else if constexpr (c == 10) {
                float tot_lo, tot_hi;
                both_halves(run, tot_lo, tot_hi);
                off = a[0] + (hh == 0 ? tot_hi : 0.0f);
                a[0] += tot_lo + tot_hi;
#pragma unroll
                for (int r = 0; r < 16; ++r) x[r] -= off;
            } else if constexpr (c == 11) {
#pragma unroll
                for (int r = 0; r < 6; ++r) w[r] = fast_exp2(x[r]);
            } else if constexpr (c == 12) {
#pragma unroll
                for (int r = 6; r < 12; ++r) w[r] = fast_exp2(x[r]);
            } else if constexpr (c == 13) {
#pragma unroll
                for (int r = 12; r < 16; ++r) w[r] = fast_exp2(x[r]);
#pragma unroll
                for (int r = 0; r < 8; ++r) p_out[0][r] = (__bf16)w[r];
            } else if constexpr (c == 14) {
#pragma unroll
                for (int r = 8; r < 16; ++r) p_out[1][r & 7] = (__bf16)w[r];
            }
        };

        fetch(ic<0>{});
        fetch(ic<1>{});
        __builtin_amdgcn_sched_barrier(0);
        auto slot_body = [&](auto ic_i) __attribute__((always_inline)) {
            constexpr int i = decltype(ic_i)::value;
            fetch(ic<i + 2>{});
            mfma(ic<i>{});
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NSLOT == 16) {
                chunk(ic<i>{});
            } else {
                chunk(ic<2 * i>{});
                __builtin_amdgcn_sched_barrier(0);
                chunk(ic<2 * i + 1>{});
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        slot_body(ic<0>{}); slot_body(ic<1>{}); slot_body(ic<2>{}); slot_body(ic<3>{});
        slot_body(ic<4>{}); slot_body(ic<5>{}); slot_body(ic<6>{}); slot_body(ic<7>{});
        if constexpr (NSLOT == 16) {
            slot_body(ic<8>{}); slot_body(ic<9>{}); slot_body(ic<10>{}); slot_body(ic<11>{});
            slot_body(ic<12>{}); slot_body(ic<13>{}); slot_body(ic<14>{}); slot_body(ic<15>{});
        }
        // rotate the pipeline registers
        sbuf[0][0] = acc;
        pbuf[0][0][0] = pbuf[1][0][0];
        pbuf[0][0][1] = pbuf[1][0][1];
    };

    // ---- the sweep
    const int jmax = min(T, qb * BQ + BQ) - 1;          // last live query row of the workgroup
    const int nsub = (jmax + 31) >> 5;                   // subtiles covering keys 0 .. jmax-1
    // this wave's subtiles: from the diagonal of its last group (or the last staged one) down to 0
    const int nw = wave_live ? min((q0 >> 5) + NG, nsub) : 0;
    const int t0w = nsub - nw;                           // global step of the wave's first subtile
    // from this step on every live wave is past its diagonals (wave 0 is the last to get there)
    const int t_clean = nsub - min(((qb * BQ) >> 5) + NG, nsub) + NG;

    // subtile handled at step j is number nsub-1-j (counted from key 0); past the end re-load
    // subtile 0 into a slot nobody reads, which keeps the number of loads per step constant
    auto stage_step = [&](int t) __attribute__((always_inline)) {
        stage(Kg, max(nsub - 1 - (t + 3), 0), smem + C::K_OFF + ((t + 3) & 3) * C::SUB);
        stage(Vg, max(nsub - 1 - (t + 1), 0), smem + C::V_OFF + ((t + 1) & 3) * C::SUB);
    };
    auto end_step = [&]() __attribute__((always_inline)) {
        dma_wait<2 * C::NI>();       // everything but this step's own 2*NI loads has landed
        barrier_nofence();
    };
    // a step whose variant depends on where this wave is in its own pipeline
    auto generic_step = [&](int t) __attribute__((always_inline)) {
        stage_step(t);
        const int tau = t - t0w;                         // the wave's own step index
        if (nw > 0 && tau >= -1) {
            // key 32*sidx + 16hh + r is visible to query q0 + 32g + n iff it is smaller
            const int lim0 = q0 + n - 32 * (nsub - 1 - t);
            if (tau == -1) step(bc<false>{}, bc<false>{}, bc<true>{}, bc<false>{}, ic<-1>{}, t, 0);
            else if (tau == 0) step(bc<false>{}, bc<true>{}, bc<true>{}, bc<true>{}, ic<-1>{}, t, lim0);
            else if (tau < NG) step(bc<true>{}, bc<true>{}, bc<true>{}, bc<true>{}, ic<-1>{}, t, lim0);
            else step(bc<true>{}, bc<true>{}, bc<true>{}, bc<false>{}, ic<-1>{}, t, 0);
        }
        end_step();
    };
    if (nsub > 0) {
        stage(Kg, max(nsub - 1, 0), smem + C::K_OFF);                  // K(0)
        stage(Kg, max(nsub - 2, 0), smem + C::K_OFF + C::SUB);         // K(1)
    }
    dma_wait<0>();
    barrier_nofence();

    int t = -1;
    // ramp: waves enter their pipelines one after the other and pass their diagonals
    for (; t < min(t_clean, nsub); ++t) generic_step(t);
    // steady state: every live wave runs the full step
    for (; t < nsub; ++t) {                              // the last step forms an S that is never used
        stage_step(t);
        if (nw > 0) {
            if constexpr (NG == 1) hot_step(t);
            else step(bc<true>{}, bc<true>{}, bc<true>{}, bc<false>{}, ic<-1>{}, t, 0);
        }
        end_step();
    }
    if (nw > 0) step(bc<true>{}, bc<false>{}, bc<false>{}, bc<false>{}, ic<-1>{}, t, 0);   // drain: O += A(last) V(last)
    dma_wait<0>();                                       // the trailing re-loads

    // ---- store.  oacc[g][b][r] is query row 32g + 8*(r/4) + 4*hh + r%4, column 32b + n.
    if (wave_live) {
        uint16_t* Og = o + bh * (long)T * D;
        const bool full = q0 + WQ <= T;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = q0 + 32 * g + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (full || row < T) {
                        const __bf16 val = (__bf16)oacc[g][b][r];
                        Og[(long)row * D + 32 * b + n] = __builtin_bit_cast(uint16_t, val);
                    }
                }
            }
            if (WRITE_M && hh == 0 && q0 + 32 * g + n < T) m[bh * (long)T + q0 + 32 * g + n] = -a[g] * SB_LN2;
        }
    }
}

template <int D, int NG, bool WRITE_M>
hipError_t launch_one(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o, float* m,
                      int BH, int T, hipStream_t stream)
{
    constexpr int BQ = 128 * NG;
    const int nqb = (T + BQ - 1) / BQ;
    const long blocks = 8L * ((BH + 7) / 8) * nqb;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((fwd_bf16_kernel<D, NG, WRITE_M>), dim3((unsigned)blocks), dim3(NTHREADS), 0, stream,
                       q, k, v, o, m, T, BH, nqb);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o,
                           float* m, int B, int H, int T, int d, hipStream_t stream)
{
    const int BH = B * H;
    if (d == 64)
        return m ? launch_one<64, 1, true>(q, k, v, o, m, BH, T, stream)
                 : launch_one<64, 1, false>(q, k, v, o, m, BH, T, stream);
    static const int ng = getenv("SB_FWD_NG") ? atoi(getenv("SB_FWD_NG")) : 1;   // tuning knob (temporary)
    if (ng == 1)
        return m ? launch_one<128, 1, true>(q, k, v, o, m, BH, T, stream)
                 : launch_one<128, 1, false>(q, k, v, o, m, BH, T, stream);
    return m ? launch_one<128, 2, true>(q, k, v, o, m, BH, T, stream)
             : launch_one<128, 2, false>(q, k, v, o, m, BH, T, stream);
}

}  // namespace sb
