// bf16 forward of causal stick-breaking attention on the gfx950 matrix cores.
//
// Work split.  A query block is 128 rows of one (batch, head); each of the 4
// wavefronts of a workgroup owns 32 of them and keeps their Q fragments in
// registers.  A workgroup processes TWO query blocks one after the other, block p
// and block nqb-1-p of the same head: with causal skipping their costs add up to
// the same total for every p, so all workgroups run equally long.  Two workgroups
// share a CU (two wavefronts per SIMD).
//
// Keys are swept in 64-row tiles (two 32-row subtiles each) from the diagonal
// towards key 0, the order Algorithm 1 prescribes: the weight of key i needs the
// total of softplus(z) over the keys between i and the query (Eq. 2), so that total
// is carried per query row from subtile to subtile (the vector `a` of Algorithm 1).
// K and V tiles are brought into LDS by direct global->LDS loads, double buffered,
// one workgroup barrier per tile; tiles above the diagonal are never touched.
//
// Layout inside a wavefront.  Logits are formed transposed, S^T = K Q^T, with the
// 32x32x16 bf16 MFMA: A operand = 32 key rows from LDS, B operand = the wave's 32
// query rows.  In the accumulator a lane owns ONE query column (lane % 32) and 16
// key rows; the LDS row fed to MFMA row rho is perm_row(rho), which makes those 16
// keys consecutive (lanes 0-31: keys 0..15 of the subtile, lanes 32-63: keys
// 16..31).  The running product along the keys is then a serial chain inside the
// lane plus one exchange with the partner lane.  The weights feed the second MFMA
// (O += A V) straight from registers: the accumulator's per-lane key order is a
// valid K-dimension order for the A operand, and V is read from LDS with the
// transposing load in that same key order.
//
// Arithmetic between the two MFMAs (fp32): Eq. 1's product is evaluated in the
// linear domain inside a lane's 16 keys and in the log domain across lanes,
// subtiles and tiles.  With x = z*log2(e) and e_r = 2^{x_r} = beta_r / (1 - beta_r):
//     A[r] = beta_r * prod_{r' > r} (1 - beta_r') * 2^{-carry}
//          = e_r * prod_{r' < r} (1 + e_r') / prod_{all r'} (1 + e_r') * 2^{-carry},
// carry = sum over all nearer keys of log2(1 + e) (the base-2 softplus, i.e. Eq. 2's
// running sum).  That costs one exponential and four multiply/adds per weight; the
// log form of Eq. 2/3 needs three transcendentals.  Where the in-lane product could
// overflow, the wave falls back to the log form for that subtile (see ew()).
//
// Early halt (HALT variant, inference forward without m; the paper's "conditional
// computation", section 4.1): the carry of a row is -log2 of the stick it has left, and
// no weight of a farther key can exceed that.  Once every row of a query block has less
// than eps left, the block stops sweeping: the error of o_j is at most eps * max|v|.
#include <type_traits>

#include "sb_kernels.h"
#include "sb_mma.h"

namespace sb {
namespace {

constexpr int NW = 4;                                   // wavefronts per workgroup
constexpr int BQ = 32 * NW;                             // query rows per block
constexpr int NS = 2;                                   // staging buffers (tiles in LDS)

template <int D> struct FwdCfg {
    static constexpr int ROW = D * 2;                   // bytes per tile row (unpadded, swizzled)
    static constexpr int TK = 64;                       // keys per staged tile
    static constexpr int KT_BYTES = TK * ROW;           // one K (or V) tile
    static constexpr int STAGE = 2 * KT_BYTES;          // K tile then V tile
    static constexpr int CPR = ROW / 16;                // 16 B chunks per row
    static constexpr int BLK_ROWS = 1024 / ROW;         // rows moved by one wave-wide 16 B/lane load
    static constexpr int NPW = KT_BYTES / 1024 / NW;    // such loads per wave per K (or V) tile
};

template <bool B> using bc = std::integral_constant<bool, B>;

// VL: packed variable-length batch.  The tensors are [H][Ttot][D] ([H/G][Ttot][D] for k, v),
// sequence s occupies rows cu[s] .. cu[s+1]-1, BH counts (sequence, head) pairs and T_arg,
// nqb_arg describe the longest sequence (they size the grid); a workgroup whose pair of
// blocks lies beyond its own sequence's end returns at once.
// TRI: measurement variant of the element-wise path.  The in-tile reverse cumulative sum of
// Algorithm 1 is taken on the matrix pipe, as a product with a triangular matrix of ones,
// instead of the in-lane chain (see ew_tri()); everything else is the same kernel.
template <int D, bool WRITE_M, bool HALT, bool RB, bool VL, bool TRI = false>
__global__ void __launch_bounds__(64 * NW, D == 128 ? 2 : (D == 64 ? 3 : 4))
fwd_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                const uint16_t* __restrict__ v, const uint16_t* __restrict__ rb,
                uint16_t* __restrict__ o, float* __restrict__ m,
                int T_arg, int BH, int H, int G, int nqb_arg, float halt_carry,
                unsigned long long* __restrict__ tile_counts, const int* __restrict__ cu, int Ttot)
{
    using C = FwdCfg<D>;
    constexpr int NPW = C::NPW;
    static_assert(!(HALT && WRITE_M), "a halted sweep does not know m");
    __shared__ __attribute__((aligned(1024))) char smem[NS * C::STAGE];
    __shared__ int s_halt[2][NW];                       // per iteration parity and wave: all rows exhausted
    __shared__ __attribute__((aligned(16))) char s_tri[TRI ? 2 * 64 * 16 : 16];   // triangular operand, per lane

    // workgroup -> (head, pair of query blocks).  Consecutive workgroup ids go round
    // the 8 XCDs, so every XCD gets its own heads and K/V of a head stay in one L2.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const int npair = (nqb_arg + 1) >> 1;
    const long bh = xcd + 8L * (slot / npair);
    const int pidx = slot % npair;
    if (bh >= BH) return;
    int T = T_arg, nqb = nqb_arg;
    long row0, kvrow0;                                  // first row of this head's q / k rows
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
    } else {
        // grouped kv heads: G consecutive query heads read the same K and V
        head = (int)(bh % H);
        row0 = bh * (long)T;
        kvrow0 = (G == 1 ? bh : (bh / H) * (H / G) + (bh % H) / G) * (long)T;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if constexpr (!HALT) {
        // measurement aid: with a non-null tile_counts the first workgroup leaves the shader
        // clock counter and the 100 MHz reference counter at its start ([0], [1]) and at its end
        // ([2], [3]); their ratio is the clock the chip sustained while this kernel ran
        if (tile_counts && wg == 0 && tid == 0) {
            tile_counts[0] = (unsigned long long)clock64();
            tile_counts[1] = (unsigned long long)wall_clock64();
        }
    }
    const int n = lane & 31;          // query column inside the wave
    const int hh = lane >> 5;         // half-wave: keys 16*hh .. 16*hh+15 of a subtile
    const int gg = lane >> 4, li = lane & 15;
    if constexpr (TRI) {
        // A operand of C^T = U L^T, U[key][key'] = 1 for key' >= key (keys of one 32-key subtile).
        // MFMA row rho stands for key perm_row(rho) (the accumulator layout of the logits), and
        // K-dim element 8h + e of MFMA s stands for key 16h + 8s + e (the order in which a lane
        // holds its 16 values).  Every wave writes the same words: benign.
        const int key_out = perm_row(n);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 u;
#pragma unroll
            for (int e = 0; e < 8; ++e) u[e] = (16 * hh + 8 * s + e >= key_out) ? (__bf16)1.0f : (__bf16)0.0f;
            *reinterpret_cast<bf16x8*>(s_tri + (s * 64 + lane) * 16) = u;
        }
        __syncthreads();
    }

    const uint16_t* Qg = q + row0 * D;
    const uint16_t* Kg = k + kvrow0 * D;
    const uint16_t* Vg = v + kvrow0 * D;

    // ---- per-lane LDS byte addresses inside the first 32-row subtile of the first staging
    // buffer; every other subtile, matrix and buffer is a compile-time constant further on
    const uint32_t smem0 = lds_offset(smem);
    uint32_t aoff[D / 16];                  // K rows as A operand: row perm_row(n), chunk 2s + hh
    {
        const int key_l = perm_row(n);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) aoff[s] = smem0 + tile_off_perm<D>(key_l, 2 * s + hh);
    }
    uint32_t vtr[D / 32][2];                // V through the transposing load: rows 16hh + li/4 (+4t, +8s)
    {
        const int row_l = 16 * (gg >> 1) + (li >> 2);
        const int cl = 2 * (gg & 1) + ((li & 3) >> 1);
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                vtr[b][t] = smem0 + tile_off_perm<D>(row_l + 4 * t, 4 * b + cl) + 8 * (li & 1);
    }

    // ---- direct global -> LDS staging of one 64-row tile of K and of V.
    // One instruction moves 16 B per lane to 1 KB of consecutive LDS; the swizzle is
    // applied on the global side: the lane whose LDS position is (row, physical chunk)
    // fetches the logical chunk that belongs there.  Instruction i of this wave covers
    // tile rows (wave*NPW + i)*BLK_ROWS + lane/CPR.
    int goff[NPW];
#pragma unroll
    for (int i = 0; i < NPW; ++i) {
        const int row = (wave * NPW + i) * C::BLK_ROWS + lane / C::CPR;
        goff[i] = (row * D + (((lane % C::CPR) ^ swz_perm<D>(row)) << 3)) * 2;
    }
    auto stage_tile = [&](int jt, int st) __attribute__((always_inline)) {
        char* sp = smem + st * C::STAGE;
        if ((jt + 1) * C::TK <= T) {                    // all 64 rows exist
            const uint16_t* kb = Kg + (long)jt * C::TK * D;
            const uint16_t* vb = Vg + (long)jt * C::TK * D;
#pragma unroll
            for (int i = 0; i < NPW; ++i) dma16_to_lds_saddr(kb, goff[i], sp + (wave * NPW + i) * 1024);
#pragma unroll
            for (int i = 0; i < NPW; ++i) dma16_to_lds_saddr(vb, goff[i], sp + C::KT_BYTES + (wave * NPW + i) * 1024);
        } else {                                        // rows past T are clamped (causality masks them)
#pragma unroll
            for (int i = 0; i < NPW; ++i) {
                const int row = (wave * NPW + i) * C::BLK_ROWS + lane / C::CPR;
                const int c = (lane % C::CPR) ^ swz_perm<D>(row);
                const long gr = min(jt * C::TK + row, T - 1);
                dma16_to_lds(Kg + gr * D + c * 8, sp + (wave * NPW + i) * 1024);
            }
#pragma unroll
            for (int i = 0; i < NPW; ++i) {
                const int row = (wave * NPW + i) * C::BLK_ROWS + lane / C::CPR;
                const int c = (lane % C::CPR) ^ swz_perm<D>(row);
                const long gr = min(jt * C::TK + row, T - 1);
                dma16_to_lds(Vg + gr * D + c * 8, sp + C::KT_BYTES + (wave * NPW + i) * 1024);
            }
        }
    };

    f32x16 oacc[D / 32];
    float a = 0.0f;                   // carry: sum of log2(1 + e) over all keys already swept (nearer keys)
    bf16x8 qf[D / 16];                // B operand of S^T = K Q^T: Q[q0 + n][16s + 8hh .. +7]
    const float c2 = SB_LOG2E / sqrtf((float)D);

    // operand fetches from LDS, kept apart from the MFMAs that use them so that they
    // can be issued a phase ahead
    // kslot / vslot: byte offset of the subtile's K / V rows from the start of the LDS tile
    // array; a compile-time constant in the unrolled sweep (it then rides in the instruction's
    // offset field), a runtime value in the diagonal band
    auto k_fetch = [&](uint32_t kslot, u32x4 (&kop)[D / 16]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < D / 16; ++s) kop[s] = lds_load16(aoff[s] + kslot);
    };
    auto v_fetch = [&](uint32_t vslot, bf16x8 (&vop)[D / 16]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const uint32_t pp = vslot + (8 * s) * C::ROW;
                vop[2 * b + s] = tr_pair_at(vtr[b][0] + pp, vtr[b][1] + pp);
            }
    };
    // S^T = K Q^T
    auto s_mfma = [&](const u32x4 (&kop)[D / 16]) __attribute__((always_inline)) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
        for (int s = 0; s < D / 16; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kop[s]), qf[s], acc, 0, 0, 0);
        return acc;
    };
    // O[q][dcol] += sum_keys A[q][key] V[key][dcol]; K-dim index 8h+e <-> key 16h + 8s + e
    auto pv_mfma = [&](const bf16x8 (&vop)[D / 16], const bf16x8 (&p)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p[s], vop[2 * b + s], oacc[b], 0, 0, 0);
    };

    // Element-wise path of one 32x32 subtile: logits -> weights (as MFMA operands).
    // Inside the lane the chain  t_r = W_r e_r,  W_{r+1} = W_r + t_r  runs over the 16
    // keys in ascending order, so W_r = W_0 prod_{r' < r} (1 + e_r') and the weight of
    // key r is t_r / W_16 * 2^-(carry from all nearer keys).  log2(W_16 / W_0) is this
    // lane's contribution to the carry.  W_0 = 2^-60 keeps the chain inside fp32 for
    // in-lane products up to 2^140; weights below 2^-66 are flushed to zero.  If a chain
    // still gets beyond 2^80 (sharp logits: softplus summing to more than 97 nats over
    // 16 keys) or overflows, the wave redoes the subtile in the log form of Eq. 2 with
    // the overflow-proof base-2 softplus.
    // With MASK (the subtile on the diagonal) key 16hh + r is visible to query n iff
    // 16hh + r < n.
    auto ew = [&](auto mask_c, const f32x16& sin, bf16x8 (&pout)[2]) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_c)::value;
        float g[16];
        float W = 0x1p-60f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float e = fast_exp2(sin[r] * c2);
            if constexpr (MASK) e = (16 * hh + r < n) ? e : 0.0f;
            g[r] = W * e;
            W += g[r];
        }
        const bool bad = !(W < 0x1p80f);
        if (__builtin_amdgcn_ballot_w64(bad) == 0) {
            const float l = fast_log2(W) + 60.0f;        // log2 of the lane's prod (1 + e)
            float l_lo, l_hi;
            both_halves(l, l_lo, l_hi);
            // keys 16..31 (hh = 1) are nearer to the query than keys 0..15
            const float kf = fast_exp2(60.0f - (a + l_hi + (hh == 0 ? l_lo : 0.0f)));
            a += l_lo + l_hi;
#pragma unroll
            for (int r = 0; r < 16; ++r) pout[r >> 3][r & 7] = (__bf16)(g[r] * kf);
        } else {
            float y[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                y[r] = sin[r] * c2;
                if constexpr (MASK) y[r] = (16 * hh + r < n) ? y[r] : -INFINITY;
            }
            float run = 0.0f;
#pragma unroll
            for (int r = 15; r >= 0; --r) {
                run += sp2(y[r]);
                y[r] -= run;                           // x - (sum of sp2 over this lane's keys r..15)
            }
            float t_lo, t_hi;
            both_halves(run, t_lo, t_hi);
            const float off = a + (hh == 0 ? t_hi : 0.0f);
            a += t_lo + t_hi;
#pragma unroll
            for (int r = 0; r < 16; ++r) pout[r >> 3][r & 7] = (__bf16)fast_exp2(y[r] - off);
        }
    };

    // The same step in the log form of Eq. 2 with Algorithm 1's in-tile cumulative sum on the
    // matrix pipe (unmasked subtiles only).  L = sp2(x) per element (two transcendentals); the
    // inclusive sums over the keys from a lane's own key to the subtile's last key, both
    // half-waves at once, are C^T = U L^T with L split into a bf16 head and a bf16 remainder
    // (one bf16 alone would leave 2^-9 of up to 32 summands in the exponent): four MFMAs.  The
    // weight is 2^(x - C - carry), a third transcendental.
    auto ew_tri = [&](const f32x16& sin, bf16x8 (&pout)[2]) __attribute__((always_inline)) {
        float y[16];
        bf16x8 lh[2], ll[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            y[r] = sin[r] * c2;
            const float L = sp2(y[r]);
            const __bf16 h = (__bf16)L;
            lh[r >> 3][r & 7] = h;
            ll[r >> 3][r & 7] = (__bf16)(L - (float)h);
        }
        const bf16x8 u0 = *reinterpret_cast<const bf16x8*>(s_tri + lane * 16);
        const bf16x8 u1 = *reinterpret_cast<const bf16x8*>(s_tri + (64 + lane) * 16);
        f32x16 c;
#pragma unroll
        for (int r = 0; r < 16; ++r) c[r] = 0.0f;
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u0, lh[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u1, lh[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u0, ll[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u1, ll[1], c, 0, 0, 0);
        float t_lo, t_hi;
        both_halves(c[0], t_lo, t_hi);                 // key 0's sum (lanes 0-31) is the subtile's total
#pragma unroll
        for (int r = 0; r < 16; ++r) pout[r >> 3][r & 7] = (__bf16)fast_exp2((y[r] - c[r]) - a);
        a += t_lo;
    };

    // one 32-key subtile, start to end (tiles that touch the diagonal band)
    auto subtile = [&](auto mask_c, uint32_t stage_off, int sub) __attribute__((always_inline)) {
        const uint32_t kslot = stage_off + sub * 32 * C::ROW;
        const uint32_t vslot = stage_off + C::KT_BYTES + sub * 32 * C::ROW;
        u32x4 kop[D / 16];
        bf16x8 vop[D / 16];
        k_fetch(kslot, kop);
        const f32x16 s = s_mfma(kop);
        v_fetch(vslot, vop);
        bf16x8 p[2];
        ew(mask_c, s, p);
        pv_mfma(vop, p);
    };
    // a full tile, upper subtile first, written so that the operand fetches of a phase
    // can be issued during the phase before it
    auto hot_tile = [&](uint32_t sp) __attribute__((always_inline)) {
        u32x4 kop[D / 16];
        bf16x8 vop[D / 16];
        bf16x8 p[2];
        k_fetch(sp + 32 * C::ROW, kop);
        f32x16 s = s_mfma(kop);
        v_fetch(sp + C::KT_BYTES + 32 * C::ROW, vop);
        if constexpr (TRI) ew_tri(s, p); else ew(bc<false>{}, s, p);
        k_fetch(sp, kop);
        pv_mfma(vop, p);
        s = s_mfma(kop);
        v_fetch(sp + C::KT_BYTES, vop);
        if constexpr (TRI) ew_tri(s, p); else ew(bc<false>{}, s, p);
        pv_mfma(vop, p);
    };

    for (int part = 0; part < 2; ++part) {
        const int qb = part == 0 ? nqb - 1 - pidx : pidx;
        if (part == 1 && 2 * pidx == nqb - 1) break;     // odd block count: the middle block is alone
        const int Q0 = qb * BQ;
        const int q0 = Q0 + wave * 32;                   // this wave's first query row
        const bool wave_live = q0 < T;
        if (part == 1) barrier_nofence();                // everyone is done with the stages of the first block
        {
            const int jq = min(q0 + n, T - 1);
            const u32x4* src = reinterpret_cast<const u32x4*>(Qg + (long)jq * D + 8 * hh);
#pragma unroll
            for (int s = 0; s < D / 16; ++s) qf[s] = __builtin_bit_cast(bf16x8, src[2 * s]);
        }
        // Wait for the Q loads (and the first block's stores) here, once: the staging
        // loads below are issued behind the compiler's back, and a wait for "all my
        // loads" placed inside the loop would also wait for those.
#pragma unroll
        for (int s = 0; s < D / 16; ++s) asm volatile("" :: "v"(qf[s]));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[b][r] = 0.0f;
        a = 0.0f;

        // ---- the sweep over 64-key tiles, from the diagonal down to key 0
        const int kmax = min(T, Q0 + BQ) - 1;                // keys 0 .. kmax-1 are visible to some row
        const int ntile = (kmax + C::TK - 1) / C::TK;
        const int ndiag = min(ntile, ntile - Q0 / C::TK);    // leading tiles that touch the diagonal band

        // iteration `it` handles tile ntile-1-it, staged in buffer it % NS.  Past the end
        // tile 0 is loaded again into a buffer nobody reads, which keeps the number of
        // outstanding loads per iteration constant.
        stage_tile(max(ntile - 1, 0), 0);
        auto begin_iter = [&](int it) __attribute__((always_inline)) {
            dma_wait<0>();                                   // this wave's share of tile `it` has landed
            // ... everyone's has, and tile it-1 is no longer read.  The halting variant also
            // publishes its flags through LDS here: their writes must have completed first,
            // or the waves of a workgroup could disagree about leaving the loop.
            if constexpr (HALT) barrier_lds(); else barrier_nofence();
            stage_tile(max(ntile - 2 - it, 0), (it + 1) % NS);
            return (uint32_t)((it % NS) * C::STAGE);
        };
        int it = 0;
        for (; it < ndiag; ++it) {                           // tiles that touch the diagonal band
            const uint32_t sp = begin_iter(it);
            const int jt = ntile - 1 - it;
            if (wave_live) {
#pragma unroll
                for (int sub = 1; sub >= 0; --sub) {
                    const int k0 = jt * C::TK + 32 * sub;    // subtiles and wave rows are both 32-aligned
                    if (k0 == q0) subtile(bc<true>{}, sp, sub);
                    else if (k0 < q0) subtile(bc<false>{}, sp, sub);
                }
            }
        }
        if constexpr (HALT) {
            if (lane == 0) { s_halt[0][wave] = 0; s_halt[1][wave] = 0; }   // read only after later barriers
        }
        if constexpr (!HALT) {
            // Tiles fully visible to every row, two per trip with the staging buffer a
            // compile-time constant, so that every LDS read of the sweep is a precomputed
            // register plus an immediate: no address arithmetic in the loop.
            static_assert(NS == 2, "the unrolled sweep alternates two buffers");
            if ((it & 1) && it < ntile) { hot_tile(begin_iter(it)); ++it; }
            for (; it + 1 < ntile; it += 2) {
                begin_iter(it);
                hot_tile(0u);
                begin_iter(it + 1);
                hot_tile((uint32_t)C::STAGE);
            }
        }
        for (; it < ntile; ++it) {                           // tiles fully visible to every row
            const uint32_t sp = begin_iter(it);
            if constexpr (HALT) {
                // flags of the previous iteration, written before the barrier just passed; all
                // waves read the same four words, so they leave the loop together
                const int* f = s_halt[(it + 1) & 1];
                if (it > ndiag && (f[0] & f[1] & f[2] & f[3])) break;
            }
            hot_tile(sp);
            if constexpr (HALT) {
                // both half-waves hold the same carry; rows past T repeat row T-1
                const int done = __builtin_amdgcn_ballot_w64(a < halt_carry) == 0;
                if (lane == 0) s_halt[it & 1][wave] = done;
            }
        }
        if constexpr (HALT) {
            if (tile_counts && tid == 0) {
                atomicAdd(&tile_counts[0], (unsigned long long)it);        // tiles swept
                atomicAdd(&tile_counts[1], (unsigned long long)ntile);     // tiles of the full sweep
            }
        }
        dma_wait<0>();                                       // the trailing re-load

        // ---- store.  oacc[b][r] is query row 8*(r/4) + 4*hh + r%4, column 32b + n.
        if (wave_live) {
            if constexpr (RB) {
                // remainder bias (Appendix C): o_j += (stick left of row j) * r_head.  The
                // lanes n of both half-waves hold the carry of row q0 + n.
                const float rem = fast_exp2(-a);
                const uint16_t* rh = rb + head * D;
                float rc[D / 32];
#pragma unroll
                for (int b = 0; b < D / 32; ++b)
                    rc[b] = __builtin_bit_cast(float, (uint32_t)rh[32 * b + n] << 16);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float rr = __shfl(rem, 8 * (r >> 2) + 4 * hh + (r & 3));
#pragma unroll
                    for (int b = 0; b < D / 32; ++b) oacc[b][r] += rr * rc[b];
                }
            }
            uint16_t* Og = o + row0 * D;
            const bool full = q0 + 32 <= T;
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = q0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (full || row < T) {
                        const __bf16 val = (__bf16)oacc[b][r];
                        Og[(long)row * D + 32 * b + n] = __builtin_bit_cast(uint16_t, val);
                    }
                }
            }
            if (WRITE_M && hh == 0 && q0 + n < T) m[row0 + q0 + n] = -a * SB_LN2;
        }
    }
    if constexpr (!HALT) {
        if (tile_counts && wg == 0 && tid == 0) {
            tile_counts[2] = (unsigned long long)clock64();
            tile_counts[3] = (unsigned long long)wall_clock64();
        }
    }
}

template <int D, bool WRITE_M, bool HALT, bool RB, bool VL = false, bool TRI = false>
hipError_t launch_one(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                      uint16_t* o, float* m, int BH, int H, int G, int T, float halt_carry,
                      unsigned long long* tile_counts, hipStream_t stream,
                      const int* cu = nullptr, int Ttot = 0)
{
    const int nqb = (T + BQ - 1) / BQ;
    const long blocks = 8L * ((BH + 7) / 8) * ((nqb + 1) / 2);
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL((fwd_bf16_kernel<D, WRITE_M, HALT, RB, VL, TRI>), dim3((unsigned)blocks), dim3(64 * NW), 0, stream,
                       q, k, v, rb, o, m, T, BH, H, G, nqb, halt_carry, tile_counts, cu, Ttot);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                           uint16_t* o, float* m, int B, int H, int Hkv, int T, int d, hipStream_t stream,
                           unsigned long long* clocks)
{
    const int BH = B * H;
    const int G = H / Hkv;
#define SB_FWD(DD, WM, RBV) launch_one<DD, WM, false, RBV>(q, k, v, rb, o, m, BH, H, G, T, 0.0f, clocks, stream)
    if (d == 32) {
        if (rb) return m ? SB_FWD(32, true, true) : SB_FWD(32, false, true);
        return m ? SB_FWD(32, true, false) : SB_FWD(32, false, false);
    }
    if (d == 64) {
        if (rb) return m ? SB_FWD(64, true, true) : SB_FWD(64, false, true);
        return m ? SB_FWD(64, true, false) : SB_FWD(64, false, false);
    }
    if (rb) return m ? SB_FWD(128, true, true) : SB_FWD(128, false, true);
    return m ? SB_FWD(128, true, false) : SB_FWD(128, false, false);
#undef SB_FWD
}

hipError_t launch_fwd_bf16_tri(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o, float* m,
                               int B, int H, int T, hipStream_t stream)
{
    return launch_one<128, true, false, false, false, true>(q, k, v, nullptr, o, m, B * H, H, 1, T, 0.0f, nullptr, stream);
}

hipError_t launch_fwd_bf16_varlen(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* rb,
                                  uint16_t* o, float* m, const int* cu, int nseq, int H, int Hkv,
                                  int Ttot, int max_T, int d, hipStream_t stream)
{
    const int BH = nseq * H;
    const int G = H / Hkv;
#define SB_FWD(DD, WM, RBV) \
    launch_one<DD, WM, false, RBV, true>(q, k, v, rb, o, m, BH, H, G, max_T, 0.0f, nullptr, stream, cu, Ttot)
    if (d == 32) {
        if (rb) return m ? SB_FWD(32, true, true) : SB_FWD(32, false, true);
        return m ? SB_FWD(32, true, false) : SB_FWD(32, false, false);
    }
    if (d == 64) {
        if (rb) return m ? SB_FWD(64, true, true) : SB_FWD(64, false, true);
        return m ? SB_FWD(64, true, false) : SB_FWD(64, false, false);
    }
    if (rb) return m ? SB_FWD(128, true, true) : SB_FWD(128, false, true);
    return m ? SB_FWD(128, true, false) : SB_FWD(128, false, false);
#undef SB_FWD
}

hipError_t launch_fwd_bf16_halt(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* o,
                                float eps, unsigned long long* tile_counts,
                                int B, int H, int T, int d, hipStream_t stream)
{
    const int BH = B * H;
    const float halt_carry = -log2f(eps);               // carry = -log2(stick left)
    if (d == 32)
        return launch_one<32, false, true, false>(q, k, v, nullptr, o, nullptr, BH, H, 1, T, halt_carry, tile_counts, stream);
    if (d == 64)
        return launch_one<64, false, true, false>(q, k, v, nullptr, o, nullptr, BH, H, 1, T, halt_carry, tile_counts, stream);
    return launch_one<128, false, true, false>(q, k, v, nullptr, o, nullptr, BH, H, 1, T, halt_carry, tile_counts, stream);
}

}  // namespace sb
