// The compression step on the GPU (paper Sec. 3.1: low-rank SVD of the head-merged cache; Alg. 1,
// compress step; the appendix's implementation details name randomized SVD).
//
// ap_compute_bases: decompression matrix D [r, HD] of X [n, HD], rows = approximate leading right
// singular vectors in decreasing order of singular value, by the published randomized range-finder
// scheme run on the ROW space with l = r + oversampling vectors, the start block given by the caller:
//
//     P <- Omega [l, HD]
//     power_iters + 1 times:   Yt = P X^T   [l, n]      matrix cores (compact_gemm.hip), 16-bit out
//                              M  = Yt X    [l, HD]     matrix cores, fp32 out (X^T from transpose16)
//                              P  = rows of M made orthonormal: S = M M^T in fp64 (gram_f64),
//                                   S = L L^T (chol_update / chol_panel, panels of 32 columns),
//                                   P = L^-1 M (tri_inverse, gemm_nn; fp64 accumulation)
//     Rayleigh-Ritz:           Zt = P X^T [l, n] fp32,  S = Zt Zt^T [l, l]  (= P X^T X P^T)
//                              S = J Lambda J^T by one-sided Jacobi on the rows of S (jacobi_block)
//                              D = (J^T P)[:r] in decreasing order of Lambda,  sigma = sqrt(Lambda)
//
// The matrices that lose information when rounded (M, whose singular values span the square of the
// cache's spectrum, and the small Gram matrices) stay in fp32 / fp64; what goes back into the matrix
// cores as a 16-bit operand is either the cache itself (exact) or a block with orthonormal rows.
//
// ap_decompress: Alg. 1 "retrieve cache" as a matrix, Xtilde[t] = C[t, :rank_t] D[:rank_t]: what the
// periodic re-compression decomposes again (next to the uncompressed tail).
#include "ap_common.hpp"
#include "lane_ops.hpp"

namespace ap {
namespace {

__device__ __forceinline__ double wave_sum_d(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// ---- out[c][r] = in[r][c] for 16-bit elements; columns rows .. ld_out-1 of out are zero-filled.
//      grid (ceil(ld_out / 64), ceil(cols / 64), batch), 256 threads.
__global__ void __launch_bounds__(256)
transpose16(const uint16_t* __restrict__ in, int64_t in_bstride, int ld_in, uint16_t* __restrict__ out,
            int64_t out_bstride, int ld_out, int rows, int cols) {
  __shared__ uint16_t tile[64][66];
  const int tid = threadIdx.x, r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  in += (size_t)blockIdx.z * in_bstride;
  out += (size_t)blockIdx.z * out_bstride;
  for (int e = tid; e < 64 * 64; e += 256) {
    const int rr = e >> 6, cc = e & 63;
    const int r = r0 + rr, c = c0 + cc;
    tile[rr][cc] = (r < rows && c < cols) ? in[(size_t)r * ld_in + c] : (uint16_t)0;
  }
  __syncthreads();
  for (int e = tid; e < 64 * 64; e += 256) {
    const int cc = e >> 6, rr = e & 63;
    const int r = r0 + rr, c = c0 + cc;
    if (c < cols && r < ld_out) out[(size_t)c * ld_out + r] = tile[rr][cc];
  }
}

// ---- zero the columns n .. ld-1 of a 16-bit [rows][ld] matrix.  grid (rows, batch), 64 threads.
__global__ void fill_pad16(uint16_t* __restrict__ a, int64_t bstride, int ld, int n) {
  uint16_t* row = a + (size_t)blockIdx.y * bstride + (size_t)blockIdx.x * ld;
  for (int c = n + threadIdx.x; c < ld; c += 64) row[c] = 0;
}

// ---- C̃[t, j] = j < rank[t] ? C[t, j] : 0 (16-bit).  grid (ceil(T / 4), batch), 256 threads.
__global__ void __launch_bounds__(256)
mask_coeffs(const uint16_t* __restrict__ C, int64_t c_bstride, const int32_t* __restrict__ rank, int64_t r_bstride,
            uint16_t* __restrict__ out, int64_t o_bstride, int T, int r) {
  const int b = blockIdx.y;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const int rk = rank[(size_t)b * r_bstride + t];
  const uint16_t* src = C + (size_t)b * c_bstride + (size_t)t * r;
  uint16_t* dst = out + (size_t)b * o_bstride + (size_t)t * r;
  for (int j = threadIdx.x & 63; j < r; j += 64) dst[j] = j < rk ? src[j] : (uint16_t)0;
}

// ---- S = A A^T in fp64 for A [l][lda] fp32 (m columns used).  32 x 32 tiles of the lower
//      triangle, mirrored on the way out.  grid (ceil(l/32), ceil(l/32), batch), 256 threads.
__global__ void __launch_bounds__(256)
gram_f64(const float* __restrict__ A, int64_t a_bstride, int lda, double* __restrict__ S, int64_t s_bstride,
         int l, int m) {
  if (blockIdx.x > blockIdx.y) return;
  __shared__ float As[32][33], Bs[32][33];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;
  A += (size_t)blockIdx.z * a_bstride;
  S += (size_t)blockIdx.z * s_bstride;
  double acc[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
  for (int k0 = 0; k0 < m; k0 += 32) {
    for (int e = tid; e < 1024; e += 256) {
      const int rr = e >> 5, kk = e & 31;
      const bool kin = k0 + kk < m;
      As[rr][kk] = (kin && i0 + rr < l) ? A[(size_t)(i0 + rr) * lda + k0 + kk] : 0.f;
      Bs[rr][kk] = (kin && j0 + rr < l) ? A[(size_t)(j0 + rr) * lda + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < 32; ++kk) {
      const double a0 = As[2 * ty][kk], a1 = As[2 * ty + 1][kk];
      const double b0 = Bs[2 * tx][kk], b1 = Bs[2 * tx + 1][kk];
      acc[0][0] = fma(a0, b0, acc[0][0]);
      acc[0][1] = fma(a0, b1, acc[0][1]);
      acc[1][0] = fma(a1, b0, acc[1][0]);
      acc[1][1] = fma(a1, b1, acc[1][1]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const int i = i0 + 2 * ty + u, j = j0 + 2 * tx + v;
      if (i < l && j < l) {
        S[(size_t)i * l + j] = acc[u][v];
        S[(size_t)j * l + i] = acc[u][v];
      }
    }
}

// ---- Cholesky S = L L^T in place (the lower triangle of S becomes L), fp64, in panels of 32
//      columns.  Per panel two launches:
//   chol_update   rows c0 .. l-1 of the panel minus the contribution of the columns left of it:
//                 S[i][c] -= sum_{j < c0} L[i][j] L[c][j]; a workgroup per 32 x 32 tile
//   chol_panel    one workgroup per matrix: the 32 x 32 diagonal block is factored in LDS, then
//                 every row below solves its 32 unknowns against it (a thread per row)
//      A pivot below 1e-13 of the largest diagonal entry (dmax) marks a direction that the rows
//      do not span: its column of L and its diagonal entry are zero, its row of L^-1 is zero,
//      so the corresponding row of P = L^-1 M is zero and drops out later.
__global__ void __launch_bounds__(256)
diag_max(const double* __restrict__ S, int64_t s_bstride, int l, double* __restrict__ dmax) {
  const double* Sb = S + (size_t)blockIdx.x * s_bstride;
  __shared__ double red[4];
  double m = 0.0;
  for (int i = threadIdx.x; i < l; i += 256) m = fmax(m, Sb[(size_t)i * l + i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmax(m, __shfl_xor(m, o));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) dmax[blockIdx.x] = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
}

// grid (ceil((l - c0) / 32), batch), 256 threads = 16 x 16, 2 x 2 results each
__global__ void __launch_bounds__(256)
chol_update(double* __restrict__ S, int64_t s_bstride, int l, int c0) {
  __shared__ double As[32][33], Bs[32][33];
  double* L = S + (size_t)blockIdx.y * s_bstride;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int i0 = c0 + blockIdx.x * 32;
  double acc[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
  for (int k0 = 0; k0 < c0; k0 += 32) {              // c0 is a multiple of 32
    for (int e = tid; e < 1024; e += 256) {
      const int rr = e >> 5, kk = e & 31;
      As[rr][kk] = i0 + rr < l ? L[(size_t)(i0 + rr) * l + k0 + kk] : 0.0;
      Bs[rr][kk] = c0 + rr < l ? L[(size_t)(c0 + rr) * l + k0 + kk] : 0.0;
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < 32; ++kk) {
      const double a0 = As[2 * ty][kk], a1 = As[2 * ty + 1][kk];
      const double b0 = Bs[2 * tx][kk], b1 = Bs[2 * tx + 1][kk];
      acc[0][0] = fma(a0, b0, acc[0][0]);
      acc[0][1] = fma(a0, b1, acc[0][1]);
      acc[1][0] = fma(a1, b0, acc[1][0]);
      acc[1][1] = fma(a1, b1, acc[1][1]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const int i = i0 + 2 * ty + u, c = c0 + 2 * tx + v;
      if (i < l && c < l) L[(size_t)i * l + c] -= acc[u][v];
    }
}

// grid (batch), 256 threads
__global__ void __launch_bounds__(256)
chol_panel(double* __restrict__ S, int64_t s_bstride, int l, int c0, const double* __restrict__ dmax) {
  __shared__ double Dg[32][33];
  double* L = S + (size_t)blockIdx.x * s_bstride;
  const int tid = threadIdx.x;
  const int nb = l - c0 < 32 ? l - c0 : 32;
  const double tol = dmax[blockIdx.x] * 1e-13;
  for (int e = tid; e < 1024; e += 256) {
    const int rr = e >> 5, cc = e & 31;
    Dg[rr][cc] = (rr < nb && cc < nb && cc <= rr) ? L[(size_t)(c0 + rr) * l + c0 + cc] : 0.0;
  }
  __syncthreads();
  // unblocked Cholesky of the diagonal block (right-looking, 32 short steps)
  for (int k = 0; k < nb; ++k) {
    const double piv = Dg[k][k];
    const bool dead = !(piv > tol);
    const double d = dead ? 0.0 : sqrt(piv), inv = dead ? 0.0 : 1.0 / d;
    __syncthreads();
    if (tid == 0) Dg[k][k] = d;
    if (tid > k && tid < nb) Dg[tid][k] *= inv;
    __syncthreads();
    for (int e = tid; e < 1024; e += 256) {
      const int i = e >> 5, j = e & 31;
      if (i > k && j > k && j <= i && i < nb) Dg[i][j] -= Dg[i][k] * Dg[j][k];
    }
    __syncthreads();
  }
  for (int e = tid; e < 1024; e += 256) {
    const int rr = e >> 5, cc = e & 31;
    if (rr < nb && cc < nb) L[(size_t)(c0 + rr) * l + c0 + cc] = cc <= rr ? Dg[rr][cc] : 0.0;
  }
  // rows below the block: x Dg^T = t, forward substitution, a thread per row
  for (int i = c0 + 32 + tid; i < l; i += 256) {
    double* row = L + (size_t)i * l + c0;
    double x[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) x[c] = row[c];
#pragma unroll
    for (int c = 0; c < 32; ++c) {
      double v = x[c];
#pragma unroll
      for (int j = 0; j < 32; ++j)
        if (j < c) v = fma(-x[j], Dg[c][j], v);
      const double d = Dg[c][c];
      x[c] = d == 0.0 ? 0.0 : v / d;
    }
#pragma unroll
    for (int c = 0; c < 32; ++c) row[c] = x[c];
  }
}

// X = L^-1 (lower triangular, fp64) by forward substitution, a wave per column j: the column's
// entries found so far sit in LDS, row i's dot product with them is spread over the lanes.  Rows
// of a dead pivot stay zero.  grid (ceil(l / 4), batch), 256 threads; dynamic LDS 4 * l doubles.
__global__ void __launch_bounds__(256)
tri_inverse(const double* __restrict__ S, int64_t s_bstride, double* __restrict__ X, int64_t x_bstride, int l) {
  extern __shared__ double xcol[];                      // [4][l]
  const double* L = S + (size_t)blockIdx.y * s_bstride;
  double* Li = X + (size_t)blockIdx.y * x_bstride;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int j = blockIdx.x * 4 + w;
  if (j >= l) return;
  double* x = xcol + (size_t)w * l;
  for (int i = lane; i < j; i += 64) Li[(size_t)i * l + j] = 0.0;     // above the diagonal
  for (int i = j; i < l; ++i) {
    const double* rowi = L + (size_t)i * l;
    double s = 0.0;
    for (int k = j + lane; k < i; k += 64) s = fma(rowi[k], x[k], s);
    s = wave_sum_d(s);
    const double dii = rowi[i];
    const double v = dii == 0.0 ? 0.0 : ((i == j ? 1.0 : 0.0) - s) / dii;
    if (lane == 0) {
      x[i] = v;
      Li[(size_t)i * l + j] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// ---- C = A B with A [M][K] fp64, B [K][N] fp32, fp64 accumulation; C as fp32 and / or in 16-bit
//      storage.  lower: A is lower triangular (blocks above the diagonal are skipped).
//      64 x 64 tiles, 256 threads x (4 x 4).  grid (ceil(N/64), ceil(M/64), batch).
template <class Tag>
__global__ void __launch_bounds__(256)
gemm_nn(const double* __restrict__ A, int64_t a_bstride, int lda, const float* __restrict__ Bm, int64_t b_bstride,
        int ldb, float* __restrict__ C32, int64_t c32_bstride, uint16_t* __restrict__ C16, int64_t c16_bstride,
        int ldc, int M, int N, int K, int lower) {
  __shared__ double As[16][65];
  __shared__ float Bs[16][68];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  A += (size_t)blockIdx.z * a_bstride;
  Bm += (size_t)blockIdx.z * b_bstride;
  double acc[4][4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
  const int kend = lower ? (m0 + 64 < K ? m0 + 64 : K) : K;
  for (int k0 = 0; k0 < kend; k0 += 16) {
    for (int e = tid; e < 1024; e += 256) {
      const int mm = e >> 4, kk = e & 15;
      As[kk][mm] = (m0 + mm < M && k0 + kk < K) ? A[(size_t)(m0 + mm) * lda + k0 + kk] : 0.0;
      const int kb = e >> 6, nn = e & 63;
      Bs[kb][nn] = (k0 + kb < K && n0 + nn < N) ? Bm[(size_t)(k0 + kb) * ldb + n0 + nn] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      double a[4], bv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) a[u] = As[kk][4 * ty + u];
#pragma unroll
      for (int v = 0; v < 4; ++v) bv[v] = (double)Bs[kk][4 * tx + v];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fma(a[u], bv[v], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = m0 + 4 * ty + u;
    if (i >= M) continue;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int j = n0 + 4 * tx + v;
      if (j >= N) continue;
      const float f = (float)acc[u][v];
      if (C32) C32[(size_t)blockIdx.z * c32_bstride + (size_t)i * ldc + j] = f;
      if (C16) C16[(size_t)blockIdx.z * c16_bstride + (size_t)i * ldc + j] = f32_to_bits(f, Tag{});
    }
  }
}

// ---- fp64 -> fp32 copy of n values per batch item.
__global__ void to_f32(const double* __restrict__ in, float* __restrict__ out, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = (float)in[i];
}

// ---- One-sided Jacobi on the rows of W [l][l] (fp32), block version.  The rows are cut into blocks
//      of BS; one launch takes disjoint pairs of blocks (round-robin over the blocks), a workgroup
//      per pair: its 2 BS rows come into LDS, one cyclic sweep over all their row pairs runs there
//      (2 BS - 1 steps of BS disjoint pairs, each rotated in its plane so that the two rows become
//      orthogonal), and the rows go back.  For a symmetric positive semi-definite W = S the rows
//      converge to lambda_i j_i^T, the eigenvectors scaled by their eigenvalues.
//      state[b]: [0] rotations in this sweep, [1] done.  grid (pairs, batch), 1024 threads.
template <int BS>
__global__ void __launch_bounds__(1024)
jacobi_block(float* __restrict__ W, int64_t w_bstride, int l, int nblk, int step, float tol, int* __restrict__ state) {
  extern __shared__ float rows_lds[];                   // [2 BS][l + 1]
  constexpr int TPP = 1024 / BS;                        // threads per row pair (32 or 64: within one wave)
  constexpr int NC = BS == 32 ? 19 : 16;                // a thread's columns of a row: l <= 599 / l <= 1024
  const int b = blockIdx.y, tid = threadIdx.x;
  if (state[2 * b + 1]) return;
  // round-robin over nblk blocks (nblk even; a block index >= the real count is an empty block)
  const int k = blockIdx.x, nm1 = nblk - 1;
  int ba, bb;
  if (k == 0) { ba = nm1; bb = step; }
  else { ba = (step + k) % nm1; bb = (step + nm1 - k) % nm1; }
  const int pitch = l + 1;
  float* Wb = W + (size_t)b * w_bstride;
  const int nreal = (l + BS - 1) / BS;
  if (ba >= nreal && bb >= nreal) return;
  for (int e = tid; e < 2 * BS * l; e += 1024) {
    const int rr = e / l, c = e - rr * l;
    const int gr = (rr < BS ? ba * BS + rr : bb * BS + rr - BS);
    const bool real = (rr < BS ? ba : bb) < nreal && gr < l;
    rows_lds[rr * pitch + c] = real ? Wb[(size_t)gr * l + c] : 0.f;
  }
  __syncthreads();
  const int pr = tid / TPP, sub = tid - pr * TPP;
  int nrot = 0;
  constexpr int N2 = 2 * BS;
  for (int s2 = 0; s2 < N2 - 1; ++s2) {
    int ia, ib;
    if (pr == 0) { ia = N2 - 1; ib = s2; }
    else { ia = (s2 + pr) % (N2 - 1); ib = (s2 + N2 - 1 - pr) % (N2 - 1); }
    float* ra = rows_lds + ia * pitch;
    float* rb = rows_lds + ib * pitch;
    // the pair's two rows stay in registers between the three dot products and the rotation
    // (one LDS read of each element per step), and the sums cross the pair's lanes on the DPP path
    float x[NC], y[NC];
    float al = 0.f, be = 0.f, ga = 0.f;
#pragma unroll
    for (int k = 0; k < NC; ++k) {
      const int c = sub + k * TPP;
      const bool in = c < l;
      x[k] = in ? ra[c] : 0.f;
      y[k] = in ? rb[c] : 0.f;
      al = fmaf(x[k], x[k], al);
      be = fmaf(y[k], y[k], be);
      ga = fmaf(x[k], y[k], ga);
    }
    al = group_sum<32>(al);
    be = group_sum<32>(be);
    ga = group_sum<32>(ga);
    if (TPP == 64) {
      al += __shfl_xor(al, 32);
      be += __shfl_xor(be, 32);
      ga += __shfl_xor(ga, 32);
    }
    if (fabsf(ga) > tol * sqrtf(al * be)) {               // the same decision in all lanes of the pair
      const float zeta = (be - al) / (2.f * ga);
      const float t = (zeta >= 0.f ? 1.f : -1.f) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta));
      const float cs = 1.f / sqrtf(1.f + t * t), sn = cs * t;
#pragma unroll
      for (int k = 0; k < NC; ++k) {
        const int c = sub + k * TPP;
        if (c < l) {
          ra[c] = cs * x[k] - sn * y[k];
          rb[c] = sn * x[k] + cs * y[k];
        }
      }
      if (sub == 0) ++nrot;
    }
    __syncthreads();
  }
  for (int e = tid; e < 2 * BS * l; e += 1024) {
    const int rr = e / l, c = e - rr * l;
    const int gr = (rr < BS ? ba * BS + rr : bb * BS + rr - BS);
    const bool real = (rr < BS ? ba : bb) < nreal && gr < l;
    if (real) Wb[(size_t)gr * l + c] = rows_lds[rr * pitch + c];
  }
  if (nrot) atomicAdd(&state[2 * b], nrot);
}

// after a sweep: a matrix without a rotation is done
__global__ void jacobi_sweep_end(int* __restrict__ state, int batch) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b < batch) {
    if (state[2 * b] == 0) state[2 * b + 1] = 1;
    state[2 * b] = 0;
  }
}
__global__ void jacobi_reset(int* __restrict__ state, int batch) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b < batch) { state[2 * b] = 0; state[2 * b + 1] = 0; }
}

// ---- eigenvalues = row norms, sorted in decreasing order (ties by row index); the r leading rows,
//      normalised, become R [r][l] (fp64) and sigma[i] = sqrt(lambda_i).  One workgroup per matrix.
__global__ void __launch_bounds__(1024)
eig_select(const float* __restrict__ W, int64_t w_bstride, int l, int r, double* __restrict__ R, int64_t r_bstride,
           float* __restrict__ sigma, int64_t sig_bstride) {
  __shared__ double lam[1024];
  __shared__ int pos[1024];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const float* Wb = W + (size_t)b * w_bstride;
  for (int i = w; i < l; i += 16) {
    double s = 0.0;
    for (int c = lane; c < l; c += 64) { const double v = Wb[(size_t)i * l + c]; s = fma(v, v, s); }
    s = wave_sum_d(s);
    if (lane == 0) lam[i] = sqrt(s);
  }
  __syncthreads();
  for (int i = tid; i < l; i += 1024) {
    int p = 0;
    const double li = lam[i];
    for (int j = 0; j < l; ++j) p += (lam[j] > li || (lam[j] == li && j < i)) ? 1 : 0;
    pos[i] = p;
    if (p < r && sigma) sigma[(size_t)b * sig_bstride + p] = (float)sqrt(li);
  }
  __syncthreads();
  for (int i = w; i < l; i += 16) {
    const int p = pos[i];
    if (p >= r) continue;
    const double inv = lam[i] > 0.0 ? 1.0 / lam[i] : 0.0;
    for (int c = lane; c < l; c += 64) R[(size_t)b * r_bstride + (size_t)p * l + c] = (double)Wb[(size_t)i * l + c] * inv;
  }
}

constexpr int kJacobiSweeps = 12;      // at most; a matrix without a rotation in a sweep is done
constexpr float kJacobiTol = 1e-5f;    // |a.b| <= tol |a||b|: far below what 16-bit storage of the result keeps

struct BasesLayout {
  size_t xt, yt, m32, p16, p32, zt, s64, linv, w32, rsel, state, dmax, total;
  int n_pad;
};
BasesLayout bases_layout(int B, int n, int HD, int l, int r) {
  BasesLayout w;
  w.n_pad = (n + 63) / 64 * 64;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += round_up(bytes, 256); return at; };
  w.xt = take((size_t)B * HD * w.n_pad * 2);
  w.yt = take((size_t)B * l * w.n_pad * 2);
  w.m32 = take((size_t)B * l * HD * 4);
  w.p16 = take((size_t)B * l * HD * 2);
  w.p32 = take((size_t)B * l * HD * 4);
  w.zt = take((size_t)B * l * w.n_pad * 4);
  w.s64 = take((size_t)B * l * l * 8);
  w.linv = take((size_t)B * l * l * 8);
  w.w32 = take((size_t)B * l * l * 4);
  w.rsel = take((size_t)B * r * l * 8);
  w.state = take((size_t)B * 2 * 4);
  w.dmax = take((size_t)B * 8);
  w.total = off;
  return w;
}

template <class Tag>
void launch_gemm_nn(const double* A, int64_t a_bs, int lda, const float* Bm, int64_t b_bs, int ldb, float* C32,
                    int64_t c32_bs, uint16_t* C16, int64_t c16_bs, int ldc, int M, int N, int K, int lower, int batch,
                    hipStream_t st) {
  hipLaunchKernelGGL((gemm_nn<Tag>), dim3((N + 63) / 64, (M + 63) / 64, batch), dim3(256), 0, st, A, a_bs, lda, Bm,
                     b_bs, ldb, C32, c32_bs, C16, c16_bs, ldc, M, N, K, lower);
}

template <class Tag>
ap_status run_bases(const BasesArgs& a) {
  const int B = a.B, n = a.n, HD = a.HD, r = a.r, l = a.r + a.oversample;
  const BasesLayout w = bases_layout(B, n, HD, l, r);
  char* ws = (char*)a.workspace;
  uint16_t* Xt = (uint16_t*)(ws + w.xt);
  uint16_t* Yt = (uint16_t*)(ws + w.yt);
  float* M32 = (float*)(ws + w.m32);
  uint16_t* P16 = (uint16_t*)(ws + w.p16);
  float* P32 = (float*)(ws + w.p32);
  float* Zt = (float*)(ws + w.zt);
  double* S = (double*)(ws + w.s64);
  double* Linv = (double*)(ws + w.linv);
  float* W = (float*)(ws + w.w32);
  double* Rsel = (double*)(ws + w.rsel);
  int* state = (int*)(ws + w.state);
  double* dmax = (double*)(ws + w.dmax);
  hipStream_t st = a.stream;
  const int np = w.n_pad;
  const ap_dtype dt = a.dt;

  hipLaunchKernelGGL(transpose16, dim3(np / 64, (HD + 63) / 64, B), dim3(256), 0, st, (const uint16_t*)a.X,
                     (int64_t)n * HD, HD, Xt, (int64_t)HD * np, np, n, HD);
  if (np > n) hipLaunchKernelGGL(fill_pad16, dim3(l, B), dim3(64), 0, st, Yt, (int64_t)l * np, np, n);
  const void* Pcur = a.Omega;
  int64_t p_bs = a.omega_batch_stride;
  ap_status s;
  for (int it = 0; it <= a.power_iters; ++it) {
    // Yt = P X^T  [l, n]
    NtGemmArgs g1{Pcur, p_bs, HD, a.X, (int64_t)n * HD, HD, Yt, (int64_t)l * np, np, nullptr, 0, B, l, n, HD, dt, 0, st};
    if ((s = launch_gemm_nt(g1)) != AP_OK) return s;
    // M = Yt X  [l, HD]  (X^T supplies rows that are contiguous along the token axis)
    NtGemmArgs g2{Yt, (int64_t)l * np, np, Xt, (int64_t)HD * np, np, M32, (int64_t)l * HD, HD, nullptr, 0, B, l, HD, np, dt, 2, st};
    if ((s = launch_gemm_nt(g2)) != AP_OK) return s;
    // rows of M made orthonormal
    hipLaunchKernelGGL(gram_f64, dim3((l + 31) / 32, (l + 31) / 32, B), dim3(256), 0, st, M32, (int64_t)l * HD, HD, S,
                       (int64_t)l * l, l, HD);
    hipLaunchKernelGGL(diag_max, dim3(B), dim3(256), 0, st, S, (int64_t)l * l, l, dmax);
    for (int c0 = 0; c0 < l; c0 += 32) {
      if (c0 > 0)
        hipLaunchKernelGGL(chol_update, dim3((l - c0 + 31) / 32, B), dim3(256), 0, st, S, (int64_t)l * l, l, c0);
      hipLaunchKernelGGL(chol_panel, dim3(B), dim3(256), 0, st, S, (int64_t)l * l, l, c0, dmax);
    }
    hipLaunchKernelGGL(tri_inverse, dim3((l + 3) / 4, B), dim3(256), (size_t)4 * l * 8, st, S, (int64_t)l * l, Linv, (int64_t)l * l, l);
    launch_gemm_nn<Tag>(Linv, (int64_t)l * l, l, M32, (int64_t)l * HD, HD, P32, (int64_t)l * HD, P16, (int64_t)l * HD,
                        HD, l, HD, l, 1, B, st);
    Pcur = P16;
    p_bs = (int64_t)l * HD;
  }
  // Rayleigh-Ritz in the span of P
  NtGemmArgs g4{P16, (int64_t)l * HD, HD, a.X, (int64_t)n * HD, HD, Zt, (int64_t)l * np, np, nullptr, 0, B, l, n, HD, dt, 2, st};
  if ((s = launch_gemm_nt(g4)) != AP_OK) return s;
  hipLaunchKernelGGL(gram_f64, dim3((l + 31) / 32, (l + 31) / 32, B), dim3(256), 0, st, Zt, (int64_t)l * np, np, S,
                     (int64_t)l * l, l, n);
  const size_t nel = (size_t)B * l * l;
  hipLaunchKernelGGL(to_f32, dim3((unsigned)((nel + 255) / 256)), dim3(256), 0, st, S, W, nel);
  hipLaunchKernelGGL(jacobi_reset, dim3((B + 63) / 64), dim3(64), 0, st, state, B);
  {
    // blocks of 32 rows while two of them fit the LDS next to each other, else 16
    const bool big = (size_t)64 * (l + 1) * 4 <= 150 * 1024;
    const int bs = big ? 32 : 16;
    int nblk = (l + bs - 1) / bs;
    nblk += nblk & 1;                                    // an even number of blocks (the last may be empty)
    const size_t lds = (size_t)2 * bs * (l + 1) * 4;
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e1 = hipFuncSetAttribute((const void*)jacobi_block<32>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      hipError_t e2 = hipFuncSetAttribute((const void*)jacobi_block<16>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e1 != hipSuccess || e2 != hipSuccess) {
        set_error("hipFuncSetAttribute: %s", hipGetErrorString(e1 != hipSuccess ? e1 : e2));
        return AP_ERR_HIP;
      }
      attr_set = true;
    }
    for (int sweep = 0; sweep < kJacobiSweeps; ++sweep) {
      for (int step = 0; step < nblk - 1; ++step) {
        if (big)
          hipLaunchKernelGGL(jacobi_block<32>, dim3(nblk / 2, B), dim3(1024), lds, st, W, (int64_t)l * l, l, nblk, step, kJacobiTol, state);
        else
          hipLaunchKernelGGL(jacobi_block<16>, dim3(nblk / 2, B), dim3(1024), lds, st, W, (int64_t)l * l, l, nblk, step, kJacobiTol, state);
      }
      hipLaunchKernelGGL(jacobi_sweep_end, dim3((B + 63) / 64), dim3(64), 0, st, state, B);
    }
  }
  hipLaunchKernelGGL(eig_select, dim3(B), dim3(1024), 0, st, W, (int64_t)l * l, l, r, Rsel, (int64_t)r * l, a.sigma,
                     (int64_t)r);
  // D = R P  [r, HD]
  launch_gemm_nn<Tag>(Rsel, (int64_t)r * l, l, P32, (int64_t)l * HD, HD, nullptr, 0, (uint16_t*)a.Bm, (int64_t)r * HD,
                      HD, r, HD, l, 0, B, st);
  return check_launch("ap_compute_bases");
}

}  // namespace

size_t bases_workspace(int B, int n, int HD, int r, int oversample) {
  return bases_layout(B, n, HD, r + oversample, r).total;
}

ap_status launch_compute_bases(const BasesArgs& a) {
  return a.dt == AP_F16 ? run_bases<F16Tag>(a) : run_bases<BF16Tag>(a);
}

size_t decompress_workspace(int B, int T, int HD, int r, bool ranks) {
  return round_up((size_t)B * HD * r * 2, 256) + (ranks ? round_up((size_t)B * T * r * 2, 256) : 0);
}

// Xtilde[b, t, :] = C[b, t, :rank] D[b][:rank]  (16-bit in and out, fp32 accumulation)
ap_status launch_decompress(const void* C, const void* Bm, int64_t bstride, const int32_t* rank, void* X, int B, int T,
                            int T_cap, int HD, int r, ap_dtype dt, void* workspace, hipStream_t st) {
  uint16_t* Dt = (uint16_t*)workspace;                                     // [B or 1][HD][r]
  const int nb = bstride ? B : 1;
  hipLaunchKernelGGL(transpose16, dim3((r + 63) / 64, (HD + 63) / 64, nb), dim3(256), 0, st, (const uint16_t*)Bm,
                     bstride, HD, Dt, (int64_t)HD * r, r, r, HD);
  const void* A = C;
  int64_t a_bs = (int64_t)T_cap * r;
  if (rank) {
    uint16_t* Cm = (uint16_t*)((char*)workspace + round_up((size_t)B * HD * r * 2, 256));
    hipLaunchKernelGGL(mask_coeffs, dim3((T + 3) / 4, B), dim3(256), 0, st, (const uint16_t*)C, (int64_t)T_cap * r, rank,
                       (int64_t)T, Cm, (int64_t)T * r, T, r);
    A = Cm;
    a_bs = (int64_t)T * r;
  }
  NtGemmArgs g{A, a_bs, r, Dt, bstride ? (int64_t)HD * r : 0, r, X, (int64_t)T * HD, HD, nullptr, 0, B, T, HD, r, dt, 0, st};
  ap_status s = launch_gemm_nt(g);
  return s != AP_OK ? s : check_launch("ap_decompress");
}

}  // namespace ap
