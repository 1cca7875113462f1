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
#include "commvq_launch.hpp"

namespace {

constexpr int kEmMaxNc = 64;
constexpr int kEmTile = 1024;  // points per LDS tile in k_em_accum
constexpr float kLog2eEm = 1.4426950408889634f;

inline size_t em_align(size_t v) { return (v + 255) / 256 * 256; }

// v_sqrt_f32 as it is (1 ulp): the library square root adds a scaling and a correction step per call, and the
// E step takes one per (point, centre) pair.
__device__ __forceinline__ float em_sqrt(float v) { return __builtin_amdgcn_sqrtf(v); }

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
    // two sweeps over the centres: the nearest squared distance first (no square root, no exponential), then the
    // denominator -- one v_sqrt_f32 and one v_exp_f32 per pair, the quarter-rate instructions that bound this kernel
    // (a single sweep with a running minimum computes a second exponential per pair for the rescaling)
    float dm2 = INFINITY;
    for (int a = 0; a < Nc; ++a)
        for (int b = 0; b < Nc; ++b) {
            const float ex = k.x - (ph[a].x - ph[b].y), ey = k.y - (ph[a].y + ph[b].x);
            dm2 = fminf(dm2, ex * ex + ey * ey);
        }
    const float dm = em_sqrt(dm2), sc = inv_t * kLog2eEm;
    float z = 0.f;
    for (int a = 0; a < Nc; ++a)
        for (int b = 0; b < Nc; ++b) {
            const float ex = k.x - (ph[a].x - ph[b].y), ey = k.y - (ph[a].y + ph[b].x);
            z += __builtin_amdgcn_exp2f((dm - em_sqrt(ex * ex + ey * ey)) * sc);
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
    const float sc = inv_t * kLog2eEm;
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
                const float w = __builtin_amdgcn_exp2f((nz[x].x - em_sqrt(ex * ex + ey * ey)) * sc) * nz[x].y;
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

// Blocked Cholesky A = L L^T in place (lower triangle of A [np][ld] in LDS; np a multiple of 16, the rows and
// columns past the system's size n hold the identity), 16 columns per step.  The 16 x 16 diagonal block is
// factored by wavefront 0 with a row per lane, columns exchanged through v_readlane (constant lanes: scalar
// broadcasts, no LDS round trips); the same lanes then invert the triangular block, so that everything below --
// the panel's rows here, the right-hand sides in em_substitute -- is a product with inv(L_kk) by independent
// threads instead of a 16-step chain per thread.  Dinv [np / 16][16][16] receives the inverses.
constexpr int kEmNb = 16;
__device__ __forceinline__ int em_pad(int n) { return (n + kEmNb - 1) / kEmNb * kEmNb; }
__device__ __forceinline__ float em_lane(float v, int l)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ float em_rcp(float d)
{
    const float x = __builtin_amdgcn_rcpf(d);
    return x * (2.f - d * x);
}
template <int NT>
__device__ __forceinline__ void em_cholesky(float *A, int ld, int np, float *Dinv, int tid)
{
    for (int k0 = 0; k0 < np; k0 += kEmNb) {
        float *Di = Dinv + (k0 / kEmNb) * (kEmNb * kEmNb);
        if (tid < 64) {
            const int t = tid & (kEmNb - 1);  // lanes 16..63 repeat lanes 0..15 and store nothing
            float row[kEmNb], isd[kEmNb];
#pragma unroll
            for (int c = 0; c < kEmNb; ++c) row[c] = c <= t ? A[(k0 + t) * ld + k0 + c] : 0.f;
#pragma unroll
            for (int c = 0; c < kEmNb; ++c) {
                const float d = __builtin_sqrtf(em_lane(row[c], c));
                isd[c] = em_rcp(d);
                row[c] = t == c ? d : row[c] * isd[c];  // entries above the diagonal are never read
#pragma unroll
                for (int cc = c + 1; cc < kEmNb; ++cc) row[cc] -= row[c] * em_lane(row[c], cc);  // L[t][c] L[cc][c]
            }
            // column t of X = inv(L_kk):  X[i][t] = (delta_it - sum_{k < i} L[i][k] X[k][t]) / L[i][i]
            float x[kEmNb];
#pragma unroll
            for (int i = 0; i < kEmNb; ++i) {
                float v = i == t ? 1.f : 0.f;
#pragma unroll
                for (int k = 0; k < i; ++k) v -= em_lane(row[k], i) * x[k];
                x[i] = i >= t ? v * isd[i] : 0.f;
            }
            if (tid < kEmNb) {
#pragma unroll
                for (int c = 0; c < kEmNb; ++c) {
                    if (c <= t) A[(k0 + t) * ld + k0 + c] = row[c];
                    Di[c * kEmNb + t] = x[c];
                }
            }
        }
        __syncthreads();
        for (int r = k0 + kEmNb + tid; r < np; r += NT) {  // x L_kk^T = a for the rows below: x = a inv(L_kk)^T
            float av[kEmNb], xv[kEmNb];
#pragma unroll
            for (int e = 0; e < kEmNb; ++e) av[e] = A[r * ld + k0 + e];
#pragma unroll
            for (int c = 0; c < kEmNb; ++c) {
                float v = 0.f;
#pragma unroll
                for (int e = 0; e <= c; ++e) v += av[e] * Di[c * kEmNb + e];
                xv[c] = v;
            }
#pragma unroll
            for (int c = 0; c < kEmNb; ++c) A[r * ld + k0 + c] = xv[c];
        }
        __syncthreads();
        // rest -= panel panel^T (lower triangle): 32 lanes walk a row's columns, the row's panel entries in registers
        for (int r = k0 + kEmNb + tid / 32; r < np; r += NT / 32) {
            float pr[kEmNb];
#pragma unroll
            for (int e = 0; e < kEmNb; ++e) pr[e] = A[r * ld + k0 + e];
            for (int cc = k0 + kEmNb + tid % 32; cc <= r; cc += 32) {
                float sum = 0.f;
#pragma unroll
                for (int e = 0; e < kEmNb; ++e) sum += pr[e] * A[cc * ld + k0 + e];
                A[r * ld + cc] -= sum;
            }
        }
        __syncthreads();
    }
}

// L Z = R, then L^T X = Z, for the nr columns of R [np][nr] in LDS (16 nr <= NT), blocked like em_cholesky: thread
// (c, j) forms entry c of a block's solution for column j as a product with the inverted diagonal block, then
// every thread takes one (row, column) of what remains and subtracts the block's contribution.
template <int NT>
__device__ __forceinline__ void em_substitute(const float *A, int ld, int np, const float *Dinv, float *R, int nr, int tid)
{
    const bool act = tid < kEmNb * nr;
    const int c = tid / nr, j = tid % nr;
    for (int k0 = 0; k0 < np; k0 += kEmNb) {
        const float *Di = Dinv + (k0 / kEmNb) * (kEmNb * kEmNb);
        float v = 0.f;
        if (act) {
#pragma unroll
            for (int e = 0; e < kEmNb; ++e)
                if (e <= c) v += Di[c * kEmNb + e] * R[(k0 + e) * nr + j];
        }
        __syncthreads();
        if (act) R[(k0 + c) * nr + j] = v;
        __syncthreads();
        for (int x = tid; x < (np - k0 - kEmNb) * nr; x += NT) {
            const int r = k0 + kEmNb + x / nr, jj = x % nr;
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < kEmNb; ++e) sum += A[r * ld + k0 + e] * R[(k0 + e) * nr + jj];
            R[r * nr + jj] -= sum;
        }
        __syncthreads();
    }
    for (int k0 = np - kEmNb; k0 >= 0; k0 -= kEmNb) {
        const float *Di = Dinv + (k0 / kEmNb) * (kEmNb * kEmNb);
        float v = 0.f;
        if (act) {
#pragma unroll
            for (int e = 0; e < kEmNb; ++e)
                if (e >= c) v += Di[e * kEmNb + c] * R[(k0 + e) * nr + j];  // inv(L_kk)^T
        }
        __syncthreads();
        if (act) R[(k0 + c) * nr + j] = v;
        __syncthreads();
        for (int x = tid; x < k0 * nr; x += NT) {
            const int r = x / nr, jj = x % nr;
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < kEmNb; ++e) sum += A[(k0 + e) * ld + r] * R[(k0 + e) * nr + jj];
            R[r * nr + jj] -= sum;
        }
        __syncthreads();
    }
}

// One workgroup per sub-space: build the 2Nc x 2Nc normal equations, Cholesky, two triangular solves.
__global__ __launch_bounds__(256) void k_em_solve(const float *__restrict__ nab, const float2 *__restrict__ sab,
                                                  float2 *__restrict__ phi, int Nc)
{
    extern __shared__ float em_lds[];
    const int n2 = 2 * Nc, np = em_pad(n2);
    float *A = em_lds;                 // [np][np + 1]: padded rows; identity past n2
    float *rhs = A + np * (np + 1);    // [np]
    float *Dinv = rhs + np;            // [np / 16][16][16]
    const int ld = np + 1;
    const int j = blockIdx.x, tid = threadIdx.x;
    const float *Nj = nab + (size_t)j * Nc * Nc;
    const float2 *Sj = sab + (size_t)j * Nc * Nc;
    for (int x = tid; x < np * ld; x += 256) A[x] = 0.f;
    if (tid < np) rhs[tid] = 0.f;
    __syncthreads();
    if (tid >= n2 && tid < np) A[tid * ld + tid] = 1.f;
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
    em_cholesky<256>(A, ld, np, Dinv, tid);
    em_substitute<256>(A, ld, np, Dinv, rhs, 1, tid);
    if (tid < Nc) phi[(size_t)j * Nc + tid] = make_float2(rhs[2 * tid], rhs[2 * tid + 1]);
}

// ------------------------------------------------------------------ one code shared by a group of sub-spaces
// Sec. 4.2 groups g consecutive sub-spaces under one quantized value, so a clustering centre is the pair (a, b)
// applied in all g sub-spaces and the E step weighs whole vectors:  D_i,ab^2 = sum_j ||k_i^j - c_ab^j||^2
//   = ||k_i||^2 + (N_a - 2 P_i[a]) + (N_b - 2 Q_i[b]) + X_ab,   P_i[a] = k_i . C[a],  Q_i[b] = k_i . (i C[b]),
//   N_a = ||C[a]||^2,  X_ab = 2 C[a] . (i C[b])     (C[a] = the row (x_a^j, y_a^j)_j; i C = (-y, x) per sub-space)
// -- the tables of the key encoder.  The M step is App. A.2's closed form in every sub-space with the common W:
// one matrix T^T S T (it only holds N_ab = sum_i W_i,ab) and one right-hand side per sub-space, which needs
// only the marginals of W:  rhs_j[x_a] = sum_i k_i^jx Wa_i[a] + k_i^jy Wb_i[a],  rhs_j[y_a] = sum_i k_i^jy Wa_i[a] -
// k_i^jx Wb_i[a],  Wa_i[a] = sum_b W_i,ab,  Wb_i[a] = sum_b W_i,ba.
constexpr int kEmsPts = 32;     // points per workgroup of k_ems_assign
constexpr int kEmsSplits = 16;  // point ranges whose right-hand-side partials are summed in a fixed order

// X_ab and N_a of the current codebook (one thread per (a, b)).
__global__ __launch_bounds__(256) void k_ems_tables(const float2 *__restrict__ phi, float *__restrict__ xab, float *__restrict__ nn,
                                                    int J, int Nc)
{
    const int ab = blockIdx.x * 256 + threadIdx.x;
    if (ab >= Nc * Nc) return;
    const int a = ab / Nc, b = ab % Nc;
    float x = 0.f, n = 0.f;
    for (int j = 0; j < J; ++j) {
        const float2 pa = phi[(size_t)j * Nc + a], pb = phi[(size_t)j * Nc + b];
        x += pa.y * pb.x - pa.x * pb.y;
        n += pa.x * pa.x + pa.y * pa.y;
    }
    xab[ab] = 2.f * x;
    if (b == 0) nn[a] = n;
}

// Workgroup = 32 points.  LDS: the codebook (later overwritten by X), the points, u = N_a - 2 P[a] and
// v = N_b - 2 Q[b] per point.
// 1. P, Q by plain FMAs (thread = point x eighth of the rows);  2. per point, eight lanes sweep the Nc^2 centres
// twice: nearest distance, then the softmax denominator;  3. per centre pair, four lanes sweep the 32 points:
// N_ab partial of the workgroup and the marginal Wa (first index fixed), then again transposed for Wb.
__global__ __launch_bounds__(256) void k_ems_assign(const float2 *__restrict__ data, const float2 *__restrict__ phi,
                                                    const float *__restrict__ xab_g, const float *__restrict__ nn_g,
                                                    float *__restrict__ nab_part, float *__restrict__ wa_g, float *__restrict__ wb_g,
                                                    int N, int J, int Nc, float c)
{
    extern __shared__ __attribute__((aligned(16))) float ems_lds[];
    const int JS = J + 1, NS = Nc + 1;                      // padded strides
    const int r0 = (max(J * Nc * 2, Nc * Nc) + 1) & ~1;     // floats (even) of the region that holds phi, then X
    float2 *ph = reinterpret_cast<float2 *>(ems_lds);       // [J][Nc]      (step 1)
    float *xs = ems_lds;                                    // [Nc][Nc]     (steps 2 and 3)
    float2 *pts = reinterpret_cast<float2 *>(ems_lds + r0); // [32][J + 1]
    float *u = reinterpret_cast<float *>(pts + kEmsPts * JS);  // [32][Nc + 1]
    float *v = u + kEmsPts * NS;                            // [32][Nc + 1]
    float *kk = v + kEmsPts * NS;                           // [32] ||k||^2
    float *dmin = kk + kEmsPts;                             // [32]
    float *rz = dmin + kEmsPts;                             // [32] 1 / softmax denominator
    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * kEmsPts;
    const int cnt = min(kEmsPts, N - i0);
    for (int x = tid; x < J * Nc; x += 256) ph[x] = phi[x];
    for (int x = tid; x < kEmsPts * J; x += 256) {
        const int i = x / J, j = x % J;
        pts[i * JS + j] = i < cnt ? data[(size_t)(i0 + i) * J + j] : make_float2(0.f, 0.f);
    }
    __syncthreads();
    {   // 1. thread = (point i, rows a = ag, ag + 8, ...)
        const int i = tid & (kEmsPts - 1), ag = tid / kEmsPts;
        for (int a = ag; a < Nc; a += 256 / kEmsPts) {
            float P = 0.f, Q = 0.f;
            for (int j = 0; j < J; ++j) {
                const float2 k = pts[i * JS + j], r = ph[j * Nc + a];
                P += k.x * r.x + k.y * r.y;
                Q += k.y * r.x - k.x * r.y;
            }
            const float na = nn_g[a];
            u[i * NS + a] = na - 2.f * P;
            v[i * NS + a] = na - 2.f * Q;
        }
        if (ag == 0) {
            float s = 0.f;
            for (int j = 0; j < J; ++j) { const float2 k = pts[i * JS + j]; s += k.x * k.x + k.y * k.y; }
            kk[i] = s;
        }
    }
    __syncthreads();  // phi is no longer read: X takes its place
    for (int x = tid; x < Nc * Nc; x += 256) xs[x] = xab_g[x];
    __syncthreads();
    {   // 2. lane (n, q) of wavefront w: point 8 w + n, first indices a = q, q + 8, ...
        const int n = tid & 7, q = (tid >> 3) & 7, i = (tid >> 6) * 8 + n;
        const float ki = kk[i];
        float d2m = INFINITY;
        for (int a = q; a < Nc; a += 8) {
            const float ua = ki + u[i * NS + a];
            for (int b = 0; b < Nc; ++b) d2m = fminf(d2m, ua + (v[i * NS + b] + xs[a * Nc + b]));
        }
        d2m = fminf(d2m, __shfl_xor(d2m, 8));
        d2m = fminf(d2m, __shfl_xor(d2m, 16));
        d2m = fminf(d2m, __shfl_xor(d2m, 32));
        const float dm = em_sqrt(fmaxf(d2m, 0.f));
        float z = 0.f;
        for (int a = q; a < Nc; a += 8) {
            const float ua = ki + u[i * NS + a];
#pragma unroll 4
            for (int b = 0; b < Nc; ++b) {
                const float d = em_sqrt(fmaxf(ua + (v[i * NS + b] + xs[a * Nc + b]), 0.f));
                z += __builtin_amdgcn_exp2f(-(d - dm) * c);
            }
        }
        z += __shfl_xor(z, 8);
        z += __shfl_xor(z, 16);
        z += __shfl_xor(z, 32);
        if (q == 0) { dmin[i] = dm; rz[i] = 1.f / z; }
    }
    __syncthreads();
    // 3. thread = (first index f = tid / 4, second indices s = tid % 4, + 4, ...); tr = 1: the same with the
    // roles of the two indices exchanged (marginal over the first index)
    const int f = tid >> 2, sq = tid & 3;
    for (int tr = 0; tr < 2; ++tr) {
        float nacc[kEmMaxNc / 4], xr[kEmMaxNc / 4];
#pragma unroll
        for (int e = 0; e < kEmMaxNc / 4; ++e) {
            nacc[e] = 0.f;
            const int s2 = sq + 4 * e;
            xr[e] = (f < Nc && s2 < Nc) ? (tr == 0 ? xs[f * Nc + s2] : xs[s2 * Nc + f]) : 0.f;
        }
        const float *mine = tr == 0 ? u : v, *other = tr == 0 ? v : u;
        float *marg = tr == 0 ? wa_g : wb_g;
        for (int i = 0; i < cnt; ++i) {
            float w = 0.f;
            if (f < Nc) {
                const float base = kk[i] + mine[i * NS + f];
                const float dm = dmin[i], r = rz[i];
#pragma unroll
                for (int e = 0; e < kEmMaxNc / 4; ++e) {
                    const int s2 = sq + 4 * e;
                    if (s2 < Nc) {
                        const float d = em_sqrt(fmaxf(base + (other[i * NS + s2] + xr[e]), 0.f));
                        const float wi = __builtin_amdgcn_exp2f(-(d - dm) * c) * r;
                        nacc[e] += wi;
                        w += wi;
                    }
                }
            }
            w += __shfl_xor(w, 1);
            w += __shfl_xor(w, 2);
            if (f < Nc && sq == 0) marg[(size_t)(i0 + i) * Nc + f] = w;
        }
        if (tr == 0 && f < Nc) {
#pragma unroll
            for (int e = 0; e < kEmMaxNc / 4; ++e) {
                const int s2 = sq + 4 * e;
                if (s2 < Nc) nab_part[(size_t)blockIdx.x * Nc * Nc + f * Nc + s2] = nacc[e];
            }
        }
    }
}

// N_ab = sum of the workgroups' partials in a fixed order: 16 lanes per centre pair take every 16th workgroup,
// then a butterfly over the 16 lanes.
__global__ __launch_bounds__(256) void k_ems_reduce(const float *__restrict__ nab_part, float *__restrict__ nab, int n_wg, int Nc)
{
    const int ab = blockIdx.x * 16 + (threadIdx.x >> 4), l = threadIdx.x & 15;
    float s = 0.f;
    if (ab < Nc * Nc)
        for (int w = l; w < n_wg; w += 16) s += nab_part[(size_t)w * Nc * Nc + ab];
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    s += __shfl_xor(s, 4);
    s += __shfl_xor(s, 8);
    if (ab < Nc * Nc && l == 0) nab[ab] = s;
}

// Right-hand sides: workgroup = (sub-space j, range of points), thread = a.
__global__ __launch_bounds__(kEmMaxNc) void k_ems_rhs(const float2 *__restrict__ data, const float *__restrict__ wa_g,
                                                     const float *__restrict__ wb_g, float2 *__restrict__ rhs_part, int N, int J, int Nc)
{
    const int j = blockIdx.x, sp = blockIdx.y, a = threadIdx.x;
    const int per = (N + kEmsSplits - 1) / kEmsSplits;
    const int i0 = sp * per, i1 = min(N, i0 + per);
    float rx = 0.f, ry = 0.f;
    if (a < Nc) {
#pragma unroll 4
        for (int i = i0; i < i1; ++i) {
            const float2 k = data[(size_t)i * J + j];
            const float wa = wa_g[(size_t)i * Nc + a], wb = wb_g[(size_t)i * Nc + a];
            rx += k.x * wa + k.y * wb;
            ry += k.y * wa - k.x * wb;
        }
        rhs_part[((size_t)sp * J + j) * Nc + a] = make_float2(rx, ry);
    }
}

// The common 2Nc x 2Nc matrix, its Cholesky factor, and the right-hand sides of the J sub-spaces side by side.
// The factorisation is a chain of dependent steps that one workgroup runs as fast as sixteen, while the
// right-hand sides are independent: workgroup w repeats the (cheap) factorisation and substitutes for the
// kEmsSolveCols sub-spaces w * kEmsSolveCols ... only.
constexpr int kEmsSolveThreads = 1024;
constexpr int kEmsSolveCols = 4;
__global__ __launch_bounds__(kEmsSolveThreads) void k_ems_solve(const float *__restrict__ nab, const float2 *__restrict__ rhs_part,
                                                   float2 *__restrict__ phi, int J, int Nc)
{
    extern __shared__ float em_lds[];
    const int n2 = 2 * Nc, np = em_pad(n2), ld = np + 1;
    const int tid = threadIdx.x;
    const int j0 = blockIdx.x * kEmsSolveCols, jn = min(kEmsSolveCols, J - j0);
    float *A = em_lds;                 // [np][np + 1]; identity past n2
    float *R = A + np * ld;            // [np][jn]
    float *Dinv = R + np * kEmsSolveCols;  // [np / 16][16][16]
    for (int x = tid; x < np * ld; x += kEmsSolveThreads) A[x] = 0.f;
    for (int x = tid; x < np * jn; x += kEmsSolveThreads) R[x] = 0.f;
    __syncthreads();
    if (tid >= n2 && tid < np) A[tid * ld + tid] = 1.f;
    for (int x = tid; x < Nc * Nc; x += kEmsSolveThreads) {
        const int a = x / Nc, b = x % Nc;
        const float v = nab[b * Nc + a] - nab[a * Nc + b];
        A[(2 * a) * ld + 2 * b + 1] = v;
        A[(2 * b + 1) * ld + 2 * a] = v;
    }
    for (int x = tid; x < Nc * jn; x += kEmsSolveThreads) {
        const int a = x / jn, j = x % jn;
        float rx = 0.f, ry = 0.f;
        for (int sp = 0; sp < kEmsSplits; ++sp) {
            const float2 p = rhs_part[((size_t)sp * J + j0 + j) * Nc + a];
            rx += p.x;
            ry += p.y;
        }
        R[(2 * a) * jn + j] = rx;
        R[(2 * a + 1) * jn + j] = ry;
    }
    __syncthreads();
    if (tid < Nc) {
        float d = 0.f;
        for (int b = 0; b < Nc; ++b) d += nab[tid * Nc + b] + nab[b * Nc + tid];
        A[(2 * tid) * ld + 2 * tid] = d;
        A[(2 * tid + 1) * ld + 2 * tid + 1] = d;
    }
    __syncthreads();
    em_cholesky<kEmsSolveThreads>(A, ld, np, Dinv, tid);
    em_substitute<kEmsSolveThreads>(A, ld, np, Dinv, R, jn, tid);
    for (int x = tid; x < jn * Nc; x += kEmsSolveThreads) {
        const int j = x / Nc, a = x % Nc;
        phi[(size_t)j0 * Nc + x] = make_float2(R[(2 * a) * jn + j], R[(2 * a + 1) * jn + j]);
    }
}

struct EmsLayout {
    size_t xab, nn, wa, wb, nab_part, nab, rhs_part, bytes;
    int n_wg;
};
inline EmsLayout ems_layout(int J, int N, int Nc)
{
    EmsLayout l;
    l.n_wg = (N + kEmsPts - 1) / kEmsPts;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += em_align(bytes); return at; };
    l.xab = take((size_t)Nc * Nc * 4);
    l.nn = take((size_t)Nc * 4);
    l.wa = take((size_t)N * Nc * 4);
    l.wb = take((size_t)N * Nc * 4);
    l.nab_part = take((size_t)l.n_wg * Nc * Nc * 4);
    l.nab = take((size_t)Nc * Nc * 4);
    l.rhs_part = take((size_t)kEmsSplits * J * Nc * 8);
    l.bytes = off;
    return l;
}

}  // namespace

extern "C" {

commvq_status commvq_em_workspace_bytes(int32_t n_subspaces, int32_t n_points, int32_t n_centres, size_t *bytes)
{
    if (!bytes) return COMMVQ_ERR_NULL;
    // sub-spaces are the y dimension of the launch grids (at most 65535); point indices are 32-bit
    if (n_subspaces < 1 || n_subspaces > 65535 || n_points < 1 || n_points > (1 << 24) || n_centres < 1 || n_centres > kEmMaxNc)
        return COMMVQ_ERR_SHAPE;
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
    const int np = (2 * n_centres + 15) / 16 * 16;  // the system padded to whole 16-column blocks
    const int lds = (np * (np + 1) + np + np * 16) * 4;
    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(&k_em_solve, (2 * kEmMaxNc * (2 * kEmMaxNc + 1) + 2 * kEmMaxNc + 2 * kEmMaxNc * 16) * 4, lds_ok) != hipSuccess)
        return COMMVQ_ERR_LAUNCH;
    hipLaunchKernelGGL(k_em_solve, dim3((unsigned)n_subspaces), dim3(256), lds, s, nab, sab, p2, n_centres);
    return hipGetLastError() == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

commvq_status commvq_em_shared_workspace_bytes(int32_t group, int32_t n_points, int32_t n_centres, size_t *bytes)
{
    if (!bytes) return COMMVQ_ERR_NULL;
    if (group < 1 || group > 64 || n_points < 1 || n_points > (1 << 24) || n_centres < 1 || n_centres > kEmMaxNc) return COMMVQ_ERR_SHAPE;
    *bytes = ems_layout(group, n_points, n_centres).bytes;
    return COMMVQ_OK;
}

commvq_status commvq_em_step_shared(const float *data, int32_t group, int32_t n_points, int32_t n_centres, float temperature,
                                    float *phi, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!data || !phi || !workspace) return COMMVQ_ERR_NULL;
    size_t need = 0;
    commvq_status st = commvq_em_shared_workspace_bytes(group, n_points, n_centres, &need);
    if (st != COMMVQ_OK) return st;
    if (!(temperature > 0.f)) return COMMVQ_ERR_CONFIG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need) return COMMVQ_ERR_WORKSPACE;
    const int J = group, N = n_points, Nc = n_centres;
    const EmsLayout l = ems_layout(J, N, Nc);
    char *w = static_cast<char *>(workspace);
    float *xab = reinterpret_cast<float *>(w + l.xab), *nn = reinterpret_cast<float *>(w + l.nn);
    float *wa = reinterpret_cast<float *>(w + l.wa), *wb = reinterpret_cast<float *>(w + l.wb);
    float *nab_part = reinterpret_cast<float *>(w + l.nab_part), *nab = reinterpret_cast<float *>(w + l.nab);
    float2 *rhs_part = reinterpret_cast<float2 *>(w + l.rhs_part);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const float2 *d2 = reinterpret_cast<const float2 *>(data);
    float2 *p2 = reinterpret_cast<float2 *>(phi);
    const unsigned cgrid = (unsigned)((Nc * Nc + 255) / 256);
    hipLaunchKernelGGL(k_ems_tables, dim3(cgrid), dim3(256), 0, s, p2, xab, nn, J, Nc);
    if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
    const int lds_a = ((((J * Nc * 2 > Nc * Nc ? J * Nc * 2 : Nc * Nc) + 1) & ~1) + kEmsPts * (J + 1) * 2 + 2 * kEmsPts * (Nc + 1) + 3 * kEmsPts) * 4;
    const int np_s = (2 * Nc + 15) / 16 * 16;
    const int lds_s = (np_s * (np_s + 1) + np_s * kEmsSolveCols + np_s * 16) * 4;
    static std::atomic<uint64_t> lds_ok_a{0}, lds_ok_s{0};
    const int max_a = (64 * 64 * 2 + kEmsPts * 65 * 2 + 2 * kEmsPts * 65 + 3 * kEmsPts) * 4;
    const int max_s = (128 * 129 + 128 * kEmsSolveCols + 128 * 16) * 4;
    if (allow_dynamic_lds(&k_ems_assign, max_a, lds_ok_a) != hipSuccess || allow_dynamic_lds(&k_ems_solve, max_s, lds_ok_s) != hipSuccess)
        return COMMVQ_ERR_LAUNCH;
    hipLaunchKernelGGL(k_ems_assign, dim3((unsigned)l.n_wg), dim3(256), lds_a, s, d2, p2, xab, nn, nab_part, wa, wb, N, J, Nc,
                       kLog2eEm / temperature);
    if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
    hipLaunchKernelGGL(k_ems_reduce, dim3((unsigned)((Nc * Nc + 15) / 16)), dim3(256), 0, s, nab_part, nab, l.n_wg, Nc);
    if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
    hipLaunchKernelGGL(k_ems_rhs, dim3((unsigned)J, (unsigned)kEmsSplits), dim3(kEmMaxNc), 0, s, d2, wa, wb, rhs_part, N, J, Nc);
    if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
    hipLaunchKernelGGL(k_ems_solve, dim3((unsigned)((J + kEmsSolveCols - 1) / kEmsSolveCols)), dim3(kEmsSolveThreads), lds_s, s, nab,
                       rhs_part, p2, J, Nc);
    return hipGetLastError() == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

}  // extern "C"
