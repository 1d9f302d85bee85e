// fp32 forward of causal stick-breaking attention on the vector ALU.
//
// One wavefront per block of 64 query rows, one lane per query row.  The lane
// keeps its q row and its output row in registers and walks the keys from j-1
// down to 0 (the sweep direction of Algorithm 1 at a tile width of one key),
// carrying s = sum of softplus(z) over the keys already passed, so that the
// weight of key i is exp(z_i - s) with s including key i (Eq. 2).  K and V tiles
// are staged in LDS and read as broadcasts: every lane looks at the same key at
// the same time, masked by i < j.
//
// This path exists for full-precision checks (every operation is fp32 with
// correctly rounded library exp / log1p); the bf16 matrix-core kernel is the
// fast path.
#include "sb_kernels.h"

namespace sb {
namespace {

constexpr int F32_BQ = 64;   // query rows per workgroup (one per lane)
constexpr int F32_BK = 32;   // keys per LDS tile

__device__ __forceinline__ float softplus_f32(float z)
{
    // log(1 + e^z) = max(z, 0) + log1p(e^{-|z|}): no overflow on either side
    return fmaxf(z, 0.0f) + log1pf(expf(-fabsf(z)));
}

template <int D>
__global__ void __launch_bounds__(F32_BQ)
fwd_f32_kernel(const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
               float* __restrict__ o, float* __restrict__ m, int T, int nqb)
{
    __shared__ float4 Ks[F32_BK * D / 4];
    __shared__ float4 Vs[F32_BK * D / 4];

    const long bh = blockIdx.x / nqb;
    const int qb = nqb - 1 - (int)(blockIdx.x % nqb);   // longest rows first
    const int t = threadIdx.x;
    const int j = qb * F32_BQ + t;
    const bool live = j < T;
    const float scale = 1.0f / sqrtf((float)D);

    const float* Q = q + bh * (long)T * D;
    const float* K = k + bh * (long)T * D;
    const float* V = v + bh * (long)T * D;

    float4 qr[D / 4], acc[D / 4];
    {
        const float4* qrow = reinterpret_cast<const float4*>(Q + (long)(live ? j : T - 1) * D);
#pragma unroll
        for (int c = 0; c < D / 4; ++c) {
            qr[c] = qrow[c];
            acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    float s = 0.0f;   // sum of softplus(z) over the keys i' with i <= i' < j passed so far

    // largest live query row of this block; it needs keys 0 .. jmax-1
    const int jmax = min(T, qb * F32_BQ + F32_BQ) - 1;
    const int ntile = (jmax + F32_BK - 1) / F32_BK;

    for (int kt = ntile - 1; kt >= 0; --kt) {
        __syncthreads();
        for (int idx = t; idx < F32_BK * D / 4; idx += F32_BQ) {
            const int row = idx / (D / 4), c4 = idx % (D / 4);
            const int gr = min(kt * F32_BK + row, T - 1);
            Ks[idx] = reinterpret_cast<const float4*>(K + (long)gr * D)[c4];
            Vs[idx] = reinterpret_cast<const float4*>(V + (long)gr * D)[c4];
        }
        __syncthreads();
        for (int kk = F32_BK - 1; kk >= 0; --kk) {
            const int i = kt * F32_BK + kk;
            if (i >= jmax) continue;                    // no row of this block sees key i
            const float4* kr = &Ks[kk * (D / 4)];
            float z0 = 0.f, z1 = 0.f, z2 = 0.f, z3 = 0.f;
#pragma unroll
            for (int c = 0; c < D / 4; ++c) {
                const float4 kv = kr[c];
                z0 = fmaf(qr[c].x, kv.x, z0);
                z1 = fmaf(qr[c].y, kv.y, z1);
                z2 = fmaf(qr[c].z, kv.z, z2);
                z3 = fmaf(qr[c].w, kv.w, z3);
            }
            const float z = ((z0 + z1) + (z2 + z3)) * scale;
            if (live && i < j) {
                s += softplus_f32(z);
                const float a = expf(z - s);
                const float4* vr = &Vs[kk * (D / 4)];
#pragma unroll
                for (int c = 0; c < D / 4; ++c) {
                    const float4 vv = vr[c];
                    acc[c].x = fmaf(a, vv.x, acc[c].x);
                    acc[c].y = fmaf(a, vv.y, acc[c].y);
                    acc[c].z = fmaf(a, vv.z, acc[c].z);
                    acc[c].w = fmaf(a, vv.w, acc[c].w);
                }
            }
        }
    }

    if (live) {
        float4* orow = reinterpret_cast<float4*>(o + (bh * (long)T + j) * D);
#pragma unroll
        for (int c = 0; c < D / 4; ++c) orow[c] = acc[c];
        if (m) m[bh * (long)T + j] = -s;
    }
}

}  // namespace

hipError_t launch_fwd_f32(const float* q, const float* k, const float* v, float* o, float* m,
                          int B, int H, int T, int d, hipStream_t stream)
{
    const int nqb = (T + F32_BQ - 1) / F32_BQ;
    const long blocks = (long)B * H * nqb;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(F32_BQ);
    if (d == 32)
        hipLaunchKernelGGL(fwd_f32_kernel<32>, grid, block, 0, stream, q, k, v, o, m, T, nqb);
    else if (d == 64)
        hipLaunchKernelGGL(fwd_f32_kernel<64>, grid, block, 0, stream, q, k, v, o, m, T, nqb);
    else
        hipLaunchKernelGGL(fwd_f32_kernel<128>, grid, block, 0, stream, q, k, v, o, m, T, nqb);
    return hipGetLastError();
}

}  // namespace sb
