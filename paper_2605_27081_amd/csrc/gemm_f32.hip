// Grouped expert GEMMs in fp32 (vector FMA), the reference-precision path of fp32 layers.
//
// Same contract and tile list as the bf16 kernels:
//   mode 0:  h   = silu(X_e W_gate[e]^T) * (X_e W_up[e]^T)
//   mode 1:  out = (h_e W_down[e]^T) * gate weight of the row
// One workgroup of 16 x 16 threads owns a 64 x 64 output block (4 x 4 per thread) of one half of a
// 128-row tile and walks the reduction in LDS-staged slices of 16.  Every load is bounds-checked,
// so any H, I are accepted.  This path exists for correctness at small fp32 shapes, not for speed.
#include "common.h"

namespace remoe {

namespace {

constexpr int F_BM = 64, F_BN = 64, F_BK = 16;

struct FArgs {
    const float *a;
    int64_t lda;
    const int32_t *row_gather;
    const float *b0;
    const float *b1;
    int k_dim;
    int n_out;
    const int32_t *tile_expert, *tile_row0, *tile_rows, *n_tiles;
    int dense_rows;
    int tile_m;
    const float *row_scale;
    float *c;
    int64_t ldc;
    int64_t c_row_offset;
};

template <int MODE>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(const FArgs p)
{
    __shared__ float As[F_BK][F_BM + 1];
    __shared__ float B0s[F_BK][F_BN + 1];
    __shared__ float B1s[(MODE == 0) ? F_BK : 1][F_BN + 1];

    const int halves = p.tile_m / F_BM;
    const int mt = blockIdx.y / halves, half = blockIdx.y % halves;
    const int n_mt = p.tile_expert ? *p.n_tiles : (p.dense_rows + p.tile_m - 1) / p.tile_m;
    if (mt >= n_mt) return;
    int expert = 0, row0 = mt * p.tile_m, rows = p.dense_rows - row0;
    if (p.tile_expert) {
        expert = p.tile_expert[mt];
        row0 = p.tile_row0[mt];
        rows = p.tile_rows[mt];
    }
    if (rows > p.tile_m) rows = p.tile_m;
    const int m_base = half * F_BM;
    if (m_base >= rows) return;
    const int n_base = blockIdx.x * F_BN;

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t estride = (int64_t)p.n_out * p.k_dim;
    const float *b0 = p.b0 + expert * estride;
    const float *b1 = (MODE == 0) ? p.b1 + expert * estride : nullptr;

    float acc0[4][4] = {}, acc1[4][4] = {};
    for (int k0 = 0; k0 < p.k_dim; k0 += F_BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = tid + 256 * i, r = q >> 4, kk = q & 15;
            const int m = m_base + r, k = k0 + kk;
            float av = 0.f;
            if (m < rows && k < p.k_dim) {
                int64_t arow = row0 + m;
                if (p.row_gather) arow = p.row_gather[arow];
                av = p.a[arow * p.lda + k];
            }
            As[kk][r] = av;
            const int n = n_base + r;
            float bv0 = 0.f, bv1 = 0.f;
            if (n < p.n_out && k < p.k_dim) {
                bv0 = b0[(int64_t)n * p.k_dim + k];
                if (MODE == 0) bv1 = b1[(int64_t)n * p.k_dim + k];
            }
            B0s[kk][r] = bv0;
            if (MODE == 0) B1s[kk][r] = bv1;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < F_BK; ++kk) {
            float av[4], bv0[4], bv1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bv0[j] = B0s[kk][tx * 4 + j];
                bv1[j] = (MODE == 0) ? B1s[kk][tx * 4 + j] : 0.f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[i][j] = fmaf(av[i], bv0[j], acc0[i][j]);
                    if (MODE == 0) acc1[i][j] = fmaf(av[i], bv1[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m_base + ty * 4 + i;
        if (m >= rows) continue;
        const int64_t crow = (p.c_row_offset + row0 + m) * p.ldc;
        const float sc = (MODE == 1 && p.row_scale) ? p.row_scale[row0 + m] : 1.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n_base + tx * 4 + j;
            if (n >= p.n_out) continue;
            if (MODE == 0) {
                const float g = acc0[i][j], u = acc1[i][j];
                p.c[crow + n] = g / (1.0f + expf(-g)) * u;
            } else {
                p.c[crow + n] = acc0[i][j] * sc;
            }
        }
    }
}

}  // namespace

remoe_status launch_grouped_gemm_f32(int mode, const GroupedGemmArgs &g, hipStream_t stream)
{
    if (g.max_tiles <= 0) return REMOE_OK;
    FArgs p;
    p.a = static_cast<const float *>(g.a);
    p.lda = g.lda;
    p.row_gather = g.row_gather;
    p.b0 = static_cast<const float *>(g.b0);
    p.b1 = static_cast<const float *>(g.b1);
    p.k_dim = g.k_dim;
    p.n_out = g.n_out;
    p.tile_expert = g.tile_expert;
    p.tile_row0 = g.tile_row0;
    p.tile_rows = g.tile_rows;
    p.n_tiles = g.n_tiles;
    p.dense_rows = (int)g.dense_rows;
    p.tile_m = gemm_tile_m();
    p.row_scale = g.row_scale;
    p.c = static_cast<float *>(g.c);
    p.ldc = g.ldc;
    p.c_row_offset = g.c_row_offset;
    const int64_t gy = (int64_t)g.max_tiles * (p.tile_m / F_BM);
    if (gy > 65535) return fail(REMOE_E_UNSUPPORTED, "fp32 path: too many row tiles (%lld)", (long long)gy);
    const dim3 grid((unsigned)ceil_div(g.n_out, F_BN), (unsigned)gy), block(256);
    if (mode == 0)
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<0>, grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<1>, grid, block, 0, stream, p);
    return check_hip(hipGetLastError(), "grouped_gemm_f32 launch");
}

}  // namespace remoe
