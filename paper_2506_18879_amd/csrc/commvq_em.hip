// libcommvq: EM-like learner of the RoPE-commutative key codebook (Sec. 4.2, Algorithm 1; App. A.2),
// one iteration for J independent 2-D sub-spaces, hand-written for gfx950.
//
// A sub-space has N_c' parameter pairs phi = (x_l, y_l) and N_c'^2 clustering centres
// c_ab = (x_a - y_b, y_a + x_b) (Eq. def_center).  One iteration:
//   E step   W_i,ab = softmax_ab(-D_i,ab / T), D the Euclidean distance of point i to centre ab
//            (soft assignment with temperature, Eq. W);
//   M step   the minimiser of sum_ab N_ab ||c_ab(phi) - m_ab||^2 with N_ab = sum_i W_i,ab and m_ab the
//            weighted mean of the points of centre ab.  The paper writes it with a constant matrix T as
//            phi* = (T^T S T)^-1 T^T S m; T^T S T and T^T S m are formed here directly from their
//            entries (derivatives of the objective with respect to x_a and y_a):
//              A[x_a][x_a] = A[y_a][y_a] = sum_b (N_ab + N_ba)
//              A[x_a][y_b] = A[y_b][x_a] = N_ba - N_ab
//              rhs[x_a] = sum_b (Sx_ab + Sy_ba),   rhs[y_a] = sum_b (Sy_ab - Sx_ba)
//            with (Sx, Sy)_ab = sum_i W_i,ab k_i = N_ab m_ab, and solved by Cholesky factorisation.
// Three kernels: k_em_norm (per point: nearest distance and softmax denominator), k_em_accum (per centre:
// N_ab and S_ab, points streamed through LDS, summed in a fixed order), k_em_solve (one workgroup per
// sub-space, the 2 N_c' x 2 N_c' system in LDS).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "commvq.h"

namespace {

constexpr int kEmMaxNc = 64;
constexpr int kEmTile = 1024;  // points per LDS tile in k_em_accum
constexpr float kLog2eEm = 1.4426950408889634f;

inline size_t em_align(size_t v) { return (v + 255) / 256 * 256; }

// dmin[j][i] = min_ab D_i,ab ;  zsum[j][i] = sum_ab exp(-(D_i,ab - dmin) / T)
__global__ __launch_bounds__(256) void k_em_norm(const float2 *__restrict__ data, const float2 *__restrict__ phi,
                                                 float *__restrict__ dmin, float *__restrict__ zsum, int N, int Nc, float inv_t)
{
    __shared__ float2 ph[kEmMaxNc];
    const int j = blockIdx.y;
    if (threadIdx.x < Nc) ph[threadIdx.x] = phi[(size_t)j * Nc + threadIdx.x];
    __syncthreads();
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    const float2 k = data[(size_t)j * N + i];
    // one pass with a running minimum: when a nearer centre turns up the partial sum is rescaled
    float dm = INFINITY, z = 0.f;
    for (int a = 0; a < Nc; ++a)
        for (int b = 0; b < Nc; ++b) {
            const float ex = k.x - (ph[a].x - ph[b].y), ey = k.y - (ph[a].y + ph[b].x);
            const float d = __builtin_sqrtf(ex * ex + ey * ey);
            if (d < dm) {
                z *= __builtin_amdgcn_exp2f(-(dm - d) * inv_t * kLog2eEm);  // dm = inf the first time: z stays 0
                dm = d;
            }
            z += __builtin_amdgcn_exp2f(-(d - dm) * inv_t * kLog2eEm);
        }
    dmin[(size_t)j * N + i] = dm;
    zsum[(size_t)j * N + i] = z;
}

// One thread per centre ab of sub-space j; all points pass by in LDS tiles, in index order.
__global__ __launch_bounds__(256) void k_em_accum(const float2 *__restrict__ data, const float2 *__restrict__ phi,
                                                  const float *__restrict__ dmin, const float *__restrict__ zsum,
                                                  float *__restrict__ nab, float2 *__restrict__ sab, int N, int Nc, float inv_t)
{
    __shared__ float2 pts[kEmTile];
    __shared__ float2 nz[kEmTile];  // (dmin, 1 / zsum) of the tile's points
    const int j = blockIdx.y;
    const int ab = blockIdx.x * 256 + threadIdx.x;
    const bool live = ab < Nc * Nc;
    float cx = 0.f, cy = 0.f;
    if (live) {
        const float2 pa = phi[(size_t)j * Nc + ab / Nc], pb = phi[(size_t)j * Nc + ab % Nc];
        cx = pa.x - pb.y;
        cy = pa.y + pb.x;
    }
    float n = 0.f, sx = 0.f, sy = 0.f;
    for (int t0 = 0; t0 < N; t0 += kEmTile) {
        const int cnt = min(kEmTile, N - t0);
        __syncthreads();
        for (int x = threadIdx.x; x < cnt; x += 256) {
            pts[x] = data[(size_t)j * N + t0 + x];
            nz[x] = make_float2(dmin[(size_t)j * N + t0 + x], 1.f / zsum[(size_t)j * N + t0 + x]);
        }
        __syncthreads();
        if (live) {
#pragma unroll 4
            for (int x = 0; x < cnt; ++x) {
                const float2 k = pts[x];
                const float ex = k.x - cx, ey = k.y - cy;
                const float w = __builtin_amdgcn_exp2f(-(__builtin_sqrtf(ex * ex + ey * ey) - nz[x].x) * inv_t * kLog2eEm) * nz[x].y;
                n += w;
                sx = __builtin_fmaf(w, k.x, sx);
                sy = __builtin_fmaf(w, k.y, sy);
            }
        }
    }
    if (live) {
        nab[(size_t)j * Nc * Nc + ab] = n;
        sab[(size_t)j * Nc * Nc + ab] = make_float2(sx, sy);
    }
}

// One workgroup per sub-space: build the 2Nc x 2Nc normal equations, Cholesky, two triangular solves.
__global__ __launch_bounds__(256) void k_em_solve(const float *__restrict__ nab, const float2 *__restrict__ sab,
                                                  float2 *__restrict__ phi, int Nc)
{
    extern __shared__ float em_lds[];
    const int n2 = 2 * Nc;
    float *A = em_lds;                 // [n2][n2 + 1]: padded rows
    float *rhs = A + n2 * (n2 + 1);    // [n2]
    const int ld = n2 + 1;
    const int j = blockIdx.x, tid = threadIdx.x;
    const float *Nj = nab + (size_t)j * Nc * Nc;
    const float2 *Sj = sab + (size_t)j * Nc * Nc;
    for (int x = tid; x < n2 * ld; x += 256) A[x] = 0.f;
    __syncthreads();
    // off-diagonal blocks: A[x_a][y_b] = A[y_b][x_a] = N_ba - N_ab  (unknown order x_0, y_0, x_1, y_1, ...)
    for (int x = tid; x < Nc * Nc; x += 256) {
        const int a = x / Nc, b = x % Nc;
        const float v = Nj[b * Nc + a] - Nj[a * Nc + b];
        A[(2 * a) * ld + 2 * b + 1] = v;
        A[(2 * b + 1) * ld + 2 * a] = v;
    }
    __syncthreads();
    if (tid < Nc) {
        const int a = tid;
        float d = 0.f, rx = 0.f, ry = 0.f;
        for (int b = 0; b < Nc; ++b) {
            d += Nj[a * Nc + b] + Nj[b * Nc + a];
            rx += Sj[a * Nc + b].x + Sj[b * Nc + a].y;
            ry += Sj[a * Nc + b].y - Sj[b * Nc + a].x;
        }
        A[(2 * a) * ld + 2 * a] = d;
        A[(2 * a + 1) * ld + 2 * a + 1] = d;
        rhs[2 * a] = rx;
        rhs[2 * a + 1] = ry;
    }
    __syncthreads();
    // right-looking Cholesky A = L L^T in place (lower triangle)
    for (int k = 0; k < n2; ++k) {
        if (tid == 0) A[k * ld + k] = __builtin_sqrtf(A[k * ld + k]);
        __syncthreads();
        const float dk = A[k * ld + k];
        for (int r = k + 1 + tid; r < n2; r += 256) A[r * ld + k] /= dk;
        __syncthreads();
        const int m = n2 - k - 1;
        for (int x = tid; x < m * m; x += 256) {
            const int r = k + 1 + x / m, c = k + 1 + x % m;
            if (c <= r) A[r * ld + c] -= A[r * ld + k] * A[c * ld + k];
        }
        __syncthreads();
    }
    // L z = rhs, then L^T phi = z (column-oriented substitutions)
    for (int k = 0; k < n2; ++k) {
        const float zk = rhs[k] / A[k * ld + k];
        __syncthreads();
        if (tid == 0) rhs[k] = zk;
        for (int r = k + 1 + tid; r < n2; r += 256) rhs[r] -= A[r * ld + k] * zk;
        __syncthreads();
    }
    for (int k = n2 - 1; k >= 0; --k) {
        const float pk = rhs[k] / A[k * ld + k];
        __syncthreads();
        if (tid == 0) rhs[k] = pk;
        for (int r = tid; r < k; r += 256) rhs[r] -= A[k * ld + r] * pk;
        __syncthreads();
    }
    if (tid < Nc) phi[(size_t)j * Nc + tid] = make_float2(rhs[2 * tid], rhs[2 * tid + 1]);
}

}  // namespace

extern "C" {

commvq_status commvq_em_workspace_bytes(int32_t n_subspaces, int32_t n_points, int32_t n_centres, size_t *bytes)
{
    if (!bytes) return COMMVQ_ERR_NULL;
    if (n_subspaces < 1 || n_points < 1 || n_centres < 1 || n_centres > kEmMaxNc) return COMMVQ_ERR_SHAPE;
    const size_t pts = (size_t)n_subspaces * n_points, cen = (size_t)n_subspaces * n_centres * n_centres;
    *bytes = 2 * em_align(pts * 4) + em_align(cen * 4) + em_align(cen * 8);
    return COMMVQ_OK;
}

commvq_status commvq_em_step(const float *data, int32_t n_subspaces, int32_t n_points, int32_t n_centres,
                             float temperature, float *phi, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!data || !phi || !workspace) return COMMVQ_ERR_NULL;
    size_t need = 0;
    commvq_status st = commvq_em_workspace_bytes(n_subspaces, n_points, n_centres, &need);
    if (st != COMMVQ_OK) return st;
    if (!(temperature > 0.f)) return COMMVQ_ERR_CONFIG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need) return COMMVQ_ERR_WORKSPACE;
    const size_t pts = (size_t)n_subspaces * n_points, cen = (size_t)n_subspaces * n_centres * n_centres;
    char *w = static_cast<char *>(workspace);
    float *dmin = reinterpret_cast<float *>(w);
    float *zsum = reinterpret_cast<float *>(w + em_align(pts * 4));
    float *nab = reinterpret_cast<float *>(w + 2 * em_align(pts * 4));
    float2 *sab = reinterpret_cast<float2 *>(w + 2 * em_align(pts * 4) + em_align(cen * 4));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const float inv_t = 1.f / temperature;
    const float2 *d2 = reinterpret_cast<const float2 *>(data);
    float2 *p2 = reinterpret_cast<float2 *>(phi);
    hipLaunchKernelGGL(k_em_norm, dim3((unsigned)((n_points + 255) / 256), (unsigned)n_subspaces), dim3(256), 0, s, d2, p2,
                       dmin, zsum, n_points, n_centres, inv_t);
    if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
    hipLaunchKernelGGL(k_em_accum, dim3((unsigned)((n_centres * n_centres + 255) / 256), (unsigned)n_subspaces), dim3(256), 0, s,
                       d2, p2, dmin, zsum, nab, sab, n_points, n_centres, inv_t);
    if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
    const int n2 = 2 * n_centres;
    const int lds = (n2 * (n2 + 1) + n2) * 4;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_em_solve), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (2 * kEmMaxNc * (2 * kEmMaxNc + 1) + 2 * kEmMaxNc) * 4) != hipSuccess)
            return COMMVQ_ERR_LAUNCH;
        attr_set = true;
    }
    hipLaunchKernelGGL(k_em_solve, dim3((unsigned)n_subspaces), dim3(256), lds, s, nab, sab, p2, n_centres);
    return hipGetLastError() == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

}  // extern "C"
