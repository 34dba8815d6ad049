// Kernels of the step-by-step path (one or more launches per entry point of indexmem.h).
// gfx950, wave64.  All index arithmetic that can exceed 2^31 is done in size_t.
#pragma once
#include "im_device.h"

// ------------------------------------------------------------------------------------------
// workspace clear (status word + counters); a kernel so that callers may capture the stream
// ------------------------------------------------------------------------------------------
__global__ void k_fill_i32(int32_t* p, int n, int32_t v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ------------------------------------------------------------------------------------------
// measurement only: a plain streaming read of `n16` 16-byte pieces (the ceiling the decode step's
// stream kernel is compared with).  Every thread keeps 8 loads with the streaming hint in flight and
// folds what arrives into one word; the word is stored only if it equals `never` (the benchmark
// passes a value the data cannot produce), so the loads stay and nothing is written.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_stream_read(const uint4* __restrict__ src, size_t n16,
                                                     uint32_t never, uint32_t* __restrict__ sink) {
  typedef unsigned int u4 __attribute__((ext_vector_type(4)));
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u4 v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = __builtin_nontemporal_load((const u4*)src + i + k * stride);
#pragma unroll
    for (int k = 0; k < 8; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  }
  for (; i < n16; i += stride) {
    const u4 v = __builtin_nontemporal_load((const u4*)src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == never) sink[0] = acc;
}

// ------------------------------------------------------------------------------------------
// helper: append rows
// ------------------------------------------------------------------------------------------
// A "set" is what shares one slot order: lengths, positions, indexer keys, lists and the memory
// state are kept per set.  H_set KV heads form a set: 1 (a set per (batch, KV head) unit) or H_kv
// (one set per sequence: every KV head of the layer holds the same tokens in the same slots).
// grid (ceil(n_new*16/256), units); one thread moves one 16-byte chunk of a K row and of a V row
__global__ __launch_bounds__(256) void k_append_rows(bf16_t* __restrict__ K, bf16_t* __restrict__ V,
                                                     int32_t* __restrict__ pos,
                                                     const int32_t* __restrict__ len,
                                                     const bf16_t* __restrict__ k_new,
                                                     const bf16_t* __restrict__ v_new,
                                                     const int32_t* __restrict__ pos_new, int n_new,
                                                     int H_kv, int H_set, int C) {
  const int unit = blockIdx.y, set = unit / H_set;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int row = idx >> 4, ch = idx & 15;
  if (row >= n_new) return;
  const int n = len[set];
  if (n + n_new > C) return;  // dropped; k_append_len raises the status bit
  if (k_new) {   // (NULL: the rows are already in place, only positions and lengths follow)
    const size_t src = ((size_t)unit * n_new + row) * IM_D + ch * 8;
    const size_t dst = ((size_t)unit * C + n + row) * IM_D + ch * 8;
    *(uint4*)(K + dst) = *(const uint4*)(k_new + src);
    *(uint4*)(V + dst) = *(const uint4*)(v_new + src);
  }
  if (ch == 0 && unit % H_set == 0) pos[(size_t)set * C + n + row] = pos_new[(size_t)(unit / H_kv) * n_new + row];
}

// Indexer keys of n_new appended tokens from their hidden states (one key per token, shared by all
// heads: Section 3.1 "Architecture", k_t = Norm(U_k X_t)): y[b][row][0..15] holds U_k X in fp64;
// the rows get RMSNorm over their 16 values and go, in bf16, to slots len[b] .. of sequence b.
// grid (ceil(n_new/16), B), 256 threads = 16 rows x 16 dims.  Runs before k_append_len.
__global__ __launch_bounds__(256) void k_store_hidden_keys(const double* __restrict__ y,
                                                           bf16_t* __restrict__ Kidx,
                                                           const int32_t* __restrict__ len,
                                                           int32_t* __restrict__ n_projected,
                                                           const bf16_t* __restrict__ norm_w, int n_new,
                                                           int C, float rms_eps) {
  const int b = blockIdx.y, row = blockIdx.x * 16 + (threadIdx.x >> 4), d = threadIdx.x & 15;
  const int n = len[b];
  if (n + n_new > C) return;
  if (blockIdx.x == 0 && threadIdx.x == 0) n_projected[b] = n + n_new;
  if (row >= n_new) return;
  const double* yr = y + ((size_t)b * n_new + row) * 16;
  double ss = 0.0;
#pragma unroll
  for (int e = 0; e < 16; ++e) ss = fma(yr[e], yr[e], ss);
  const double rr = sqrt(ss / 16.0 + (double)rms_eps);
  const double w = norm_w ? (double)bf2f(norm_w[d]) : 1.0;
  Kidx[((size_t)b * C + n + row) * 16 + d] = d2bf_rne(yr[d] / rr * w);
}

__global__ void k_append_len(int32_t* __restrict__ len, int n_units, int n_new, int C,
                             int32_t* __restrict__ status) {
  int u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= n_units) return;
  int n = len[u];
  if (n + n_new > C)
    atomicOr(status, 1);
  else
    len[u] = n + n_new;
}

// ------------------------------------------------------------------------------------------
// a1 (i): indexer keys of the slots not yet projected:  Kidx = bf16(RMSNorm(Uk K_slot)), fp64
// ------------------------------------------------------------------------------------------
// grid (tiles of 64 rows, units), 4 waves; wave w projects rows 16 w .. 16 w + 15 of the tile on the
// fp64 matrix cores: U[key][c] = sum_d K[key][d] Uk[c][d] as 4 column blocks x 32 steps of the
// 16x16x4 product (lane (l16, kq) supplies A[row l16][k = kq] and B[k = kq][column l16]; step m of
// this kernel covers dims 32 kq + m; result register r of the lane is row 4 r + kq, column l16).
typedef double im_v4d __attribute__((ext_vector_type(4)));

template <int N>
__device__ __forceinline__ double row16_ror_d(double v) {   // value of the lane N to the right in its 16-lane row
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), 0x120 + N, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), 0x120 + N, 0xF, 0xF, false);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// sum over the 16 lanes of a row, in every lane (rotations of 1, 2, 4, 8)
__device__ __forceinline__ double row16_sum_d(double v) {
  v += row16_ror_d<1>(v);
  v += row16_ror_d<2>(v);
  v += row16_ror_d<4>(v);
  v += row16_ror_d<8>(v);
  return v;
}

// LDS of the key projection: a 16 x 64 output tile per wave, and the few-row path's raw outputs
struct ProjectSmem {
  __attribute__((aligned(16))) bf16_t outs[4][16][IM_DI + 8];
  double ys[4][IM_DI];
};

// One wave: rows row0 .. row0 + 15 of the unit (those below n) on the fp64 matrix cores.
__device__ __forceinline__ void project_keys_tile(const bf16_t* __restrict__ K, bf16_t* __restrict__ Kidx,
                                                  const bf16_t* __restrict__ Uk,
                                                  const bf16_t* __restrict__ norm_w, int C, float rms_eps,
                                                  int unit, int row0, int n, ProjectSmem& sm) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, kq = lane >> 4;
  const int rows = min(16, n - row0);
  const size_t krow = ((size_t)unit * C + row0 + min(l16, rows - 1)) * IM_D;   // rows past the end repeat the last
  uint4 ka[4], ub[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) ka[i] = *(const uint4*)(K + krow + 32 * kq + 8 * i);
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int i = 0; i < 4; ++i) ub[cb][i] = *(const uint4*)(Uk + (16 * cb + l16) * IM_D + 32 * kq + 8 * i);
  im_v4d acc[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) acc[cb] = im_v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float fa[8] = {bf_lo(ka[i].x), bf_hi(ka[i].x), bf_lo(ka[i].y), bf_hi(ka[i].y),
                         bf_lo(ka[i].z), bf_hi(ka[i].z), bf_lo(ka[i].w), bf_hi(ka[i].w)};
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      const uint4 u = ub[cb][i];
      const float fb[8] = {bf_lo(u.x), bf_hi(u.x), bf_lo(u.y), bf_hi(u.y),
                           bf_lo(u.z), bf_hi(u.z), bf_lo(u.w), bf_hi(u.w)};
#pragma unroll
      for (int e = 0; e < 8; ++e)
        acc[cb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)fa[e], (double)fb[e], acc[cb], 0, 0, 0);
    }
  }
  // RMSNorm over the 64 outputs of a row: this lane's 4 columns, then the 16 lanes of its row
  double wn[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) wn[cb] = norm_w ? (double)bf2f(norm_w[16 * cb + l16]) : 1.0;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    double ss = 0.0;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) ss = fma(acc[cb][r], acc[cb][r], ss);
    ss = row16_sum_d(ss);
    const double rr = sqrt(ss / (double)IM_DI + (double)rms_eps);
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) sm.outs[w][4 * r + kq][16 * cb + l16] = d2bf_rne(acc[cb][r] / rr * wn[cb]);
  }
  // the wave's own 16 x 64 tile goes out in 16-byte pieces (LDS operations of one wave complete in order)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int idx = lane + 64 * k, r = idx >> 3, ch = idx & 7;
    if (r < rows)
      *(uint4*)(Kidx + ((size_t)unit * C + row0 + r) * IM_DI + 8 * ch) = *(const uint4*)&sm.outs[w][r][8 * ch];
  }
  // (the next tile of this wave may overwrite the staging rows only after these reads)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// One workgroup: rows np .. n - 1 of the unit, at most 4 of them (a decode step appends one), with plain
// fp64 FMAs: 4 lanes per output column, 32 dims each.  (Products of bf16 values summed in fp64 are exact
// at these sizes, so the order of the sum is immaterial and the rows equal the matrix-core ones.)
__device__ __forceinline__ void project_keys_few(const bf16_t* __restrict__ K, bf16_t* __restrict__ Kidx,
                                                 const bf16_t* __restrict__ Uk,
                                                 const bf16_t* __restrict__ norm_w, int C, float rms_eps,
                                                 int unit, int np, int n, ProjectSmem& sm) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int nr = n - np, c = tid >> 2, q4 = tid & 3;
  uint4 ub[4], ka[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) ub[i] = *(const uint4*)(Uk + c * IM_D + 32 * q4 + 8 * i);
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int i = 0; i < 4; ++i)
      ka[r][i] = *(const uint4*)(K + ((size_t)unit * C + np + min(r, nr - 1)) * IM_D + 32 * q4 + 8 * i);
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint4 u = ub[i];
    const float fb[8] = {bf_lo(u.x), bf_hi(u.x), bf_lo(u.y), bf_hi(u.y),
                         bf_lo(u.z), bf_hi(u.z), bf_lo(u.w), bf_hi(u.w)};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint4 v = ka[r][i];
      const float fa[8] = {bf_lo(v.x), bf_hi(v.x), bf_lo(v.y), bf_hi(v.y),
                           bf_lo(v.z), bf_hi(v.z), bf_lo(v.w), bf_hi(v.w)};
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[r] = fma((double)fa[e], (double)fb[e], acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    acc[r] += __shfl_xor(acc[r], 1, 64);
    acc[r] += __shfl_xor(acc[r], 2, 64);
    if (q4 == 0) sm.ys[r][c] = acc[r];
  }
  __syncthreads();
  if (w < nr) {   // wave w: row w, lane = column
    const double y = sm.ys[w][lane];
    const double ss = wave_sum_d(y * y);
    const double rr = sqrt(ss / (double)IM_DI + (double)rms_eps);
    const double wn1 = norm_w ? (double)bf2f(norm_w[lane]) : 1.0;
    Kidx[((size_t)unit * C + np + w) * IM_DI + lane] = d2bf_rne(y / rr * wn1);
  }
}

// grid (tiles of 64 rows, units), 4 waves; wave w projects rows 16 w .. 16 w + 15 of the tile
__global__ __launch_bounds__(256) void k_project_keys(const bf16_t* __restrict__ K,
                                                      bf16_t* __restrict__ Kidx,
                                                      const int32_t* __restrict__ len,
                                                      const int32_t* __restrict__ n_projected,
                                                      const bf16_t* __restrict__ Uk,
                                                      const bf16_t* __restrict__ norm_w, int C,
                                                      int max_live, float rms_eps,
                                                      int32_t* __restrict__ status) {
  __shared__ ProjectSmem sm;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6;
  int n = len[unit];
  if (n > max_live) {
    if (tid == 0 && blockIdx.x == 0) atomicOr(status, IM_STATUS_LIVE_EXCEEDED_BIT);
    n = max_live;
  }
  const int np = n_projected[unit];
  if (n - np <= 4) {   // (uniform per workgroup)
    if (blockIdx.x == 0 && n > np) project_keys_few(K, Kidx, Uk, norm_w, C, rms_eps, unit, np, n, sm);
    return;
  }
  const int row0 = np + blockIdx.x * 64 + 16 * w;
  if (row0 >= n) return;                       // wave-uniform; no workgroup barrier below
  project_keys_tile(K, Kidx, Uk, norm_w, C, rms_eps, unit, row0, n, sm);
}

// ------------------------------------------------------------------------------------------
// a1 (ii): query side.  C[m][n] = sum_k A[m][k] B[n][k], bf16 inputs, fp64 accumulate/output.
// ------------------------------------------------------------------------------------------
// Tiled version for many rows (prefill events).  grid (ceil(N/64), ceil(M/64)); K % 16 == 0.
__global__ __launch_bounds__(256) void k_gemm_nt_f64(const bf16_t* __restrict__ A,
                                                     const bf16_t* __restrict__ B,
                                                     double* __restrict__ Cm, int M, int N, int Kd) {
  __shared__ double As[16][64 + 2];
  __shared__ double Bs[16][64 + 2];
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int lr = tid >> 2, lc = (tid & 3) * 4;  // loader: row lr of the tile, k offset lc..lc+3
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  for (int k0 = 0; k0 < Kd; k0 += 16) {
    uint2 a = make_uint2(0, 0), b = make_uint2(0, 0);
    if (m0 + lr < M) a = *(const uint2*)(A + (size_t)(m0 + lr) * Kd + k0 + lc);
    if (n0 + lr < N) b = *(const uint2*)(B + (size_t)(n0 + lr) * Kd + k0 + lc);
    __syncthreads();
    As[lc + 0][lr] = (double)bf_lo(a.x); As[lc + 1][lr] = (double)bf_hi(a.x);
    As[lc + 2][lr] = (double)bf_lo(a.y); As[lc + 3][lr] = (double)bf_hi(a.y);
    Bs[lc + 0][lr] = (double)bf_lo(b.x); Bs[lc + 1][lr] = (double)bf_hi(b.x);
    Bs[lc + 2][lr] = (double)bf_lo(b.y); Bs[lc + 3][lr] = (double)bf_hi(b.y);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      double av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fma(av[i], bv[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < N) Cm[(size_t)m * N + n] = acc[i][j];
    }
  }
}

// The same product on the fp64 matrix cores, for Kd % 32 == 0.  A workgroup is 2 x 2 waves; a wave
// owns TM x TN tiles of 16 x 16 outputs and streams its 16 TM rows of A and 16 TN rows of B from
// L2 in 32-wide chunks (lane (l16, kq) loads the 8 values k = 32 c + 8 kq .. + 7 of row l16 of a
// tile; step e of the chunk contracts k = 32 c + 8 kq + e over the 4 kq).  Result register r of
// lane (l16, kq) is C[row 4 r + kq of the A tile][row l16 of the B tile].
// grid (ceil(N / (32 TN)), ceil(M / (32 TM))).
template <int TM, int TN>
__global__ __launch_bounds__(256) void k_gemm_nt_mfma(const bf16_t* __restrict__ A,
                                                      const bf16_t* __restrict__ B,
                                                      double* __restrict__ Cm, int M, int N, int Kd) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l16 = lane & 15, kq = lane >> 4;
  const int m0 = (blockIdx.y * 2 + (w >> 1)) * 16 * TM, n0 = (blockIdx.x * 2 + (w & 1)) * 16 * TN;
  if (m0 >= M || n0 >= N) return;   // wave-uniform; no barrier in this kernel
  const bf16_t* ap[TM];
  const bf16_t* bp[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) ap[i] = A + (size_t)min(m0 + 16 * i + l16, M - 1) * Kd + 8 * kq;
#pragma unroll
  for (int j = 0; j < TN; ++j) bp[j] = B + (size_t)min(n0 + 16 * j + l16, N - 1) * Kd + 8 * kq;
  im_v4d acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = im_v4d{0.0, 0.0, 0.0, 0.0};
  for (int k0 = 0; k0 < Kd; k0 += 64) {
    uint4 au[2][TM], bu[2][TN];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int k = (k0 + 32 * c < Kd) ? k0 + 32 * c : k0;   // an absent second chunk repeats the first, unused
#pragma unroll
      for (int i = 0; i < TM; ++i) au[c][i] = *(const uint4*)(ap[i] + k);
#pragma unroll
      for (int j = 0; j < TN; ++j) bu[c][j] = *(const uint4*)(bp[j] + k);
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if (k0 + 32 * c < Kd) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          double av[TM], bv[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            const uint32_t wd = (e < 2) ? au[c][i].x : (e < 4) ? au[c][i].y : (e < 6) ? au[c][i].z : au[c][i].w;
            av[i] = (double)((e & 1) ? bf_hi(wd) : bf_lo(wd));
          }
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const uint32_t wd = (e < 2) ? bu[c][j].x : (e < 4) ? bu[c][j].y : (e < 6) ? bu[c][j].z : bu[c][j].w;
            bv[j] = (double)((e & 1) ? bf_hi(wd) : bf_lo(wd));
          }
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + 16 * i + 4 * r + kq, n = n0 + 16 * j + l16;
        if (m < M && n < N) Cm[(size_t)m * N + n] = acc[i][j][r];
      }
}

// The same for small products: ONE 16 x 16 output tile per workgroup, its 4 waves take a quarter of
// the contraction each (Kd % 128 == 0) and meet in LDS.  grid (ceil(N / 16), ceil(M / 16)).
__global__ __launch_bounds__(256) void k_gemm_nt_mfma_k4(const bf16_t* __restrict__ A,
                                                         const bf16_t* __restrict__ B,
                                                         double* __restrict__ Cm, int M, int N, int Kd) {
  __shared__ double red[3][64][4];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l16 = lane & 15, kq = lane >> 4;
  const int m0 = blockIdx.y * 16, n0 = blockIdx.x * 16, kw = Kd / 4;
  const bf16_t* ap = A + (size_t)min(m0 + l16, M - 1) * Kd + w * kw + 8 * kq;
  const bf16_t* bp = B + (size_t)min(n0 + l16, N - 1) * Kd + w * kw + 8 * kq;
  im_v4d acc = {0.0, 0.0, 0.0, 0.0};
  for (int k0 = 0; k0 < kw; k0 += 128) {      // 4 chunks of 32 in flight
    uint4 au[4], bu[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int k = (k0 + 32 * c < kw) ? k0 + 32 * c : k0;
      au[c] = *(const uint4*)(ap + k);
      bu[c] = *(const uint4*)(bp + k);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (k0 + 32 * c < kw) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t wa = (e < 2) ? au[c].x : (e < 4) ? au[c].y : (e < 6) ? au[c].z : au[c].w;
          const uint32_t wb = (e < 2) ? bu[c].x : (e < 4) ? bu[c].y : (e < 6) ? bu[c].z : bu[c].w;
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64((double)((e & 1) ? bf_hi(wa) : bf_lo(wa)),
                                                     (double)((e & 1) ? bf_hi(wb) : bf_lo(wb)), acc, 0, 0, 0);
        }
      }
    }
  }
  if (w > 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[w - 1][lane][r] = acc[r];
  }
  __syncthreads();
  if (w == 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = m0 + 4 * r + kq, n = n0 + l16;
      if (m < M && n < N) Cm[(size_t)m * N + n] = ((acc[r] + red[0][lane][r]) + red[1][lane][r]) + red[2][lane][r];
    }
  }
}

// Few rows (decode): every workgroup owns 2 rows of B and streams them once for all M rows of A.
// Kd % 8 == 0.  Rows n0, n0 + 1 of B against all M rows of A (8 at a time), fp64 accumulation; the 16
// wave sums of a round as one butterfly of half and row swaps.
__device__ __forceinline__ void gemv_nt_rows(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                             double* __restrict__ Cm, int M, int N, int Kd, int n0,
                                             double (*red)[16]) {
  const int tid = threadIdx.x, w = tid >> 6;
  const int r1 = (n0 + 1 < N) ? n0 + 1 : n0;   // an absent second row repeats the first (result unused)
  for (int mb = 0; mb < M; mb += 8) {
    double acc[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i][0] = acc[i][1] = 0.0;
    // a round covers two 2048-wide chunks of the contraction; the loads of both go out before the arithmetic
    // (an absent second chunk repeats the first, unused; rows past M repeat the last row, unused)
    for (int k0 = tid * 8; k0 < Kd; k0 += 2 * 2048) {
      uint4 bu[2][2], au[2][8];
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int k = (k0 + it * 2048 < Kd) ? k0 + it * 2048 : k0;
        bu[it][0] = *(const uint4*)(B + (size_t)n0 * Kd + k);
        bu[it][1] = *(const uint4*)(B + (size_t)r1 * Kd + k);
#pragma unroll
        for (int i = 0; i < 8; ++i) au[it][i] = *(const uint4*)(A + (size_t)min(mb + i, M - 1) * Kd + k);
      }
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        if (k0 + it * 2048 < Kd) {
          const uint4 u0 = bu[it][0], u1 = bu[it][1];
          const float b0[8] = {bf_lo(u0.x), bf_hi(u0.x), bf_lo(u0.y), bf_hi(u0.y),
                               bf_lo(u0.z), bf_hi(u0.z), bf_lo(u0.w), bf_hi(u0.w)};
          const float b1[8] = {bf_lo(u1.x), bf_hi(u1.x), bf_lo(u1.y), bf_hi(u1.y),
                               bf_lo(u1.z), bf_hi(u1.z), bf_lo(u1.w), bf_hi(u1.w)};
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            if (mb + i < M) {
              const uint4 u = au[it][i];
              const float av[8] = {bf_lo(u.x), bf_hi(u.x), bf_lo(u.y), bf_hi(u.y),
                                   bf_lo(u.z), bf_hi(u.z), bf_lo(u.w), bf_hi(u.w)};
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                acc[i][0] = fma((double)av[e], (double)b0[e], acc[i][0]);
                acc[i][1] = fma((double)av[e], (double)b1[e], acc[i][1]);
              }
            }
          }
        }
      }
    }
    // value 2 i + r (row mb + i of A, row n0 + r of B): lane 15 of row rho of register j holds the
    // wave's sum of value 4 j + 2 (rho & 1) + (rho >> 1)
    double ws[4];
    wave_sums_butterfly_d<16>(&acc[0][0], ws);
    __syncthreads();
    if ((tid & 15) == 15) {
      const int rho = (tid >> 4) & 3;
#pragma unroll
      for (int j = 0; j < 4; ++j) red[w][4 * j + 2 * (rho & 1) + (rho >> 1)] = ws[j];
    }
    __syncthreads();
    if (tid < 16) {
      const int i = tid >> 1, r = tid & 1;
      if (mb + i < M && n0 + r < N)
        Cm[(size_t)(mb + i) * N + n0 + r] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
    }
  }
}

// grid (ceil(N/2))
__global__ __launch_bounds__(256) void k_gemv_nt_f64(const bf16_t* __restrict__ A,
                                                     const bf16_t* __restrict__ B,
                                                     double* __restrict__ Cm, int M, int N, int Kd) {
  __shared__ double red[4][16];
  gemv_nt_rows(A, B, Cm, M, N, Kd, blockIdx.x * 2, red);
}

// The query side of a decode-size scoring call in one launch: the two products (query projection, head
// gate) and, in the per-unit layout, the indexer keys of the rows not yet projected (IM_PROJ_WGS workgroups
// per unit walk over the unit's tiles of 64 rows; a few rows go through the plain-FMA path).
// grid (n_proj_units * IM_PROJ_WGS + ceil(N1/2) + ceil(N2/2))
#define IM_PROJ_WGS 4
__global__ __launch_bounds__(256) void k_query_side_few(
    const bf16_t* __restrict__ A1, const bf16_t* __restrict__ B1, double* __restrict__ C1, int N1, int K1,
    const bf16_t* __restrict__ A2, const bf16_t* __restrict__ B2, double* __restrict__ C2, int N2, int K2, int M,
    int n_proj_units, const bf16_t* __restrict__ K, bf16_t* __restrict__ Kidx, const int32_t* __restrict__ len,
    const int32_t* __restrict__ n_projected, const bf16_t* __restrict__ Uk, const bf16_t* __restrict__ norm_k_w,
    int C, int max_live, float rms_eps, int32_t* __restrict__ status) {
  __shared__ union { ProjectSmem proj; double red[4][16]; } sm;
  const int np_blocks = n_proj_units * IM_PROJ_WGS;
  if ((int)blockIdx.x < np_blocks) {
    const int unit = blockIdx.x / IM_PROJ_WGS, pb = blockIdx.x % IM_PROJ_WGS, tid = threadIdx.x, w = tid >> 6;
    int n = len[unit];
    if (n > max_live) {
      if (tid == 0 && pb == 0) atomicOr(status, IM_STATUS_LIVE_EXCEEDED_BIT);
      n = max_live;
    }
    const int np = n_projected[unit];
    if (n - np <= 4) {   // (uniform per workgroup)
      if (pb == 0 && n > np) project_keys_few(K, Kidx, Uk, norm_k_w, C, rms_eps, unit, np, n, sm.proj);
      return;
    }
    for (int row0 = np + pb * 64 + 16 * w; row0 < n; row0 += IM_PROJ_WGS * 64)   // wave-uniform; no workgroup barrier
      project_keys_tile(K, Kidx, Uk, norm_k_w, C, rms_eps, unit, row0, n, sm.proj);
    return;
  }
  const int g = (int)blockIdx.x - np_blocks, nb1 = (N1 + 1) / 2;
  if (g < nb1) gemv_nt_rows(A1, B1, C1, M, N1, K1, g * 2, sm.red);
  else gemv_nt_rows(A2, B2, C2, M, N2, K2, (g - nb1) * 2, sm.red);
}

// RMSNorm of every indexer query head in place: y[m][j][0..di-1] -> fp32-rounded q, kept as fp64.
// One wave per (m, j), di <= 64.  grid (ceil(rows/4)) with rows = M * H_idx.
__global__ __launch_bounds__(256) void k_qnorm(double* __restrict__ y, int rows, int di,
                                               const bf16_t* __restrict__ norm_w, float rms_eps) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const bool on = lane < di;
  const double v = on ? y[(size_t)row * di + lane] : 0.0;
  const double ss = wave_sum_d(v * v);
  const double rr = sqrt(ss / (double)di + (double)rms_eps);
  const double w = (norm_w && on) ? (double)bf2f(norm_w[lane]) : 1.0;
  if (on) y[(size_t)row * di + lane] = (double)(float)(v / rr * w);
}

// alpha = fp32(G x / sqrt(H_idx d_idx)), kept as fp64
__global__ void k_alpha_scale(double* __restrict__ a, int n, double denom) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) a[i] = (double)(float)(a[i] / denom);
}

// Both of the above in one launch (few rows: a decode-size scoring call).  grid (ceil(rows/4) + ceil(n/256))
__global__ __launch_bounds__(256) void k_qnorm_alpha(double* __restrict__ y, int rows, int di,
                                                     const bf16_t* __restrict__ norm_w, float rms_eps,
                                                     double* __restrict__ a, int n, double denom) {
  const int nbq = (rows + 3) / 4;
  if ((int)blockIdx.x >= nbq) {
    const int i = ((int)blockIdx.x - nbq) * 256 + threadIdx.x;
    if (i < n) a[i] = (double)(float)(a[i] / denom);
    return;
  }
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const bool on = lane < di;
  const double v = on ? y[(size_t)row * di + lane] : 0.0;
  const double ss = wave_sum_d(v * v);
  const double rr = sqrt(ss / (double)di + (double)rms_eps);
  const double w = (norm_w && on) ? (double)bf2f(norm_w[lane]) : 1.0;
  if (on) y[(size_t)row * di + lane] = (double)(float)(v / rr * w);
}

// ------------------------------------------------------------------------------------------
// a1 (iii): scores on the fp64 matrix cores.  imp[key] = max over the queries that may see the key
// of sum_j alpha[s][j] ReLU(q[s][j] . k[key]).
// ------------------------------------------------------------------------------------------
// grid (ceil(max_live / (64 TPW)), units) read as one list of (tile, unit) pairs, 4 waves; a wave owns
// TPW tiles of 16 rows (TPW = 4 for long caches, 1 when that gives too few workgroups; the A operand,
// kept in registers as packed bf16) and walks over the queries 16 at a time.  One pass of the
// 16x16x4 product (DI / 4 steps over the DI dims) takes ONE indexer head of 16 queries as its 16
// columns, so a lane's result registers belong to one query and the gated ReLU terms of the heads
// are added in place, head after head, with no cross-lane step; after the last head the block's
// scores go into the running maximum under the position mask.  The maxima of the 16 query columns
// meet once, at the end.
// DI (64 or 16) is the indexer head dim: a lane holds DI / 4 dims of its row, packed in DI / 8 words.
template <int TPW, int DI>
__global__ __launch_bounds__(256) void k_score(const bf16_t* __restrict__ Kidx,
                                               const int32_t* __restrict__ pos,
                                               const int32_t* __restrict__ len,
                                               int32_t* __restrict__ n_projected,
                                               const double* __restrict__ qhat,
                                               const double* __restrict__ alpha,
                                               const int32_t* __restrict__ q_pos, int n_q, int H_kv,
                                               int C, int H_idx, int max_live,
                                               float* __restrict__ scores, int q_per_group) {
  // grid z: groups of q_per_group queries (a multiple of 16), each with workgroups of its own; with
  // more than one group, group g writes its maxima to scores + g * units * C and k_score_max
  // folds the groups
  __shared__ int s_min[4];
  __shared__ int s_first[4];
  // tiles of low slots see the most queries in a prefill event: they are dispatched first, for
  // every unit, so the launch does not end on a few long workgroups
  const int units = gridDim.y, bid = blockIdx.y * gridDim.x + blockIdx.x;
  const int unit = bid % units, tile = bid / units;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, kq = lane >> 4;
  const int b = unit / H_kv;
  const int n = min(len[unit], max_live);
  if (tile == 0 && blockIdx.z == 0 && tid == 0) n_projected[unit] = n;  // the projection kernel ran before
  const int t0 = tile * (64 * TPW);
  if (t0 >= n) return;
  const int kbase = t0 + 16 * TPW * w;
  // A operands: lane (row l16, kq) holds dims 16 kq .. 16 kq + 15 of its row in each of the tiles
  // (rows past the end repeat the last live one; their scores are never written)
  constexpr int WPL = DI / 8, DPL = DI / 4;
  uint32_t ka[TPW][WPL];
  int posk[TPW][4];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const size_t row = (size_t)unit * C + min(kbase + 16 * t + l16, n - 1);
    if constexpr (DI == 64) {
      const uint4 u0 = *(const uint4*)(Kidx + row * DI + DPL * kq);
      const uint4 u1 = *(const uint4*)(Kidx + row * DI + DPL * kq + 8);
      ka[t][0] = u0.x; ka[t][1] = u0.y; ka[t][2] = u0.z; ka[t][3] = u0.w;
      ka[t][4] = u1.x; ka[t][5] = u1.y; ka[t][6] = u1.z; ka[t][7] = u1.w;
    } else {
      static_assert(DI == 16, "indexer head dim 64 or 16");
      const uint2 u0 = *(const uint2*)(Kidx + row * DI + DPL * kq);
      ka[t][0] = u0.x; ka[t][1] = u0.y;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {   // positions of the keys of this lane's result registers
      const int key = kbase + 16 * t + 4 * r + kq;
      const int p = pos[(size_t)unit * C + min(key, n - 1)];
      posk[t][r] = (key < n) ? p : INT_MAX;
    }
  }
  // smallest key position of the workgroup's tile, and the first query that sees it: the walk over
  // the queries starts there (visibility is decided per key further down)
  int mn = INT_MAX;
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) mn = min(mn, posk[t][r]);
  mn = (int)(wave_min_u((uint32_t)mn ^ 0x80000000u) ^ 0x80000000u);
  if (lane == 0) s_min[w] = mn;
  __syncthreads();
  const int tile_min = min(min(s_min[0], s_min[1]), min(s_min[2], s_min[3]));
  const int32_t* qp_b = q_pos + (size_t)b * n_q;
  int first = n_q;
  for (int i = tid; i < n_q; i += 256)
    if (qp_b[i] >= tile_min) { first = i; break; }
  first = (int)wave_min_u((uint32_t)first);
  if (lane == 0) s_first[w] = first;
  __syncthreads();
  first = min(min(s_first[0], s_first[1]), min(s_first[2], s_first[3]));
  float imp[TPW][4];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) imp[t][r] = -INFINITY;
  const int q_lo = blockIdx.z * q_per_group, q_hi = min(n_q, q_lo + q_per_group);
  scores += (size_t)blockIdx.z * units * C;
#pragma unroll 1
  for (int s0 = max(first & ~15, q_lo); s0 < q_hi; s0 += 16) {
    // this lane's query column; columns past the end repeat the last query and are masked
    const int s = min(s0 + l16, n_q - 1);
    const bool sv = s0 + l16 < q_hi;
    const int qp = qp_b[s];
    double acc[TPW][4];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[t][r] = 0.0;
#pragma unroll 1
    for (int j = 0; j < H_idx; ++j) {
      // B operand: lane (column l16 = query s, kq) holds dims DPL kq .. DPL kq + DPL - 1 of head j
      double qd[DPL];
      {
        const uint4* src = (const uint4*)(qhat + (((size_t)b * n_q + s) * H_idx + j) * DI + DPL * kq);
#pragma unroll
        for (int m = 0; m < DPL / 2; ++m) {
          const uint4 u = src[m];
          qd[2 * m] = __longlong_as_double(((long long)u.y << 32) | u.x);
          qd[2 * m + 1] = __longlong_as_double(((long long)u.w << 32) | u.z);
        }
      }
      const double al = alpha[((size_t)b * n_q + s) * H_idx + j];
      // keep the A operand packed: converted to fp64 ahead of the loop it would take 32 registers
      // per tile and halve the occupancy; the conversions hide under the matrix cores
#pragma unroll
      for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int i = 0; i < WPL; ++i) __asm__ volatile("" : "+v"(ka[t][i]));
      im_v4d z[TPW];
#pragma unroll
      for (int t = 0; t < TPW; ++t) z[t] = im_v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int m = 0; m < DPL; ++m) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
          const uint32_t wd = ka[t][m >> 1];
          const float f = (m & 1) ? bf_hi(wd) : bf_lo(wd);
          z[t] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)f, qd[m], z[t], 0, 0, 0);
        }
      }
#pragma unroll
      for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = fma(al, fmax(z[t][r], 0.0), acc[t][r]);
    }
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool vis = sv && posk[t][r] <= qp;     // key row 4 r + kq of tile t, query s
        imp[t][r] = vis ? fmaxf(imp[t][r], (float)acc[t][r]) : imp[t][r];
      }
  }
  // the 16 query columns' maxima meet in lane 15 of each row, which writes the keys of its register rows
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float v = imp[t][r];
      v = fmaxf(v, dpp_keep_f<0x111, 0xF>(v));
      v = fmaxf(v, dpp_keep_f<0x112, 0xF>(v));
      v = fmaxf(v, dpp_keep_f<0x114, 0xF>(v));
      v = fmaxf(v, dpp_keep_f<0x118, 0xF>(v));
      const int key = kbase + 16 * t + 4 * r + kq;
      if (l16 == 15 && key < n) scores[(size_t)unit * C + key] = v;
    }
  }
}

// a1 (iii) for a few queries (a decode step: fewer queries than indexer heads; Section 3.1, Eq. (5)).
// Here the 16 columns of the 16x16x4 product are the indexer HEADS of one query (H_idx <= 16; absent
// heads carry a zero gate), so one pass over the DI dims gives a tile of 16 keys its similarities to
// all heads; the gated ReLU terms of a key then sit in the 16 lanes of a row and meet by four
// rotations.  grid (ceil(max_live / 64), units), 4 waves, one tile of 16 keys per wave.
template <int DI>
__global__ __launch_bounds__(256) void k_score_few(const bf16_t* __restrict__ Kidx,
                                                   const int32_t* __restrict__ pos,
                                                   const int32_t* __restrict__ len,
                                                   int32_t* __restrict__ n_projected,
                                                   const double* __restrict__ qhat,
                                                   const double* __restrict__ alpha,
                                                   const int32_t* __restrict__ q_pos, int n_q, int H_kv,
                                                   int C, int H_idx, int max_live,
                                                   float* __restrict__ scores) {
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, kq = lane >> 4;
  const int b = unit / H_kv;
  const int n = min(len[unit], max_live);
  if (blockIdx.x == 0 && tid == 0) n_projected[unit] = n;  // the projection kernel ran before
  const int kbase = blockIdx.x * 64 + 16 * w;
  if (kbase >= n) return;
  constexpr int WPL = DI / 8, DPL = DI / 4;
  // A operand: lane (row l16, kq) holds dims DPL kq .. DPL kq + DPL - 1 of key kbase + l16 (rows past the
  // end repeat the last live one; their scores are never written)
  uint32_t ka[WPL];
  {
    const size_t row = (size_t)unit * C + min(kbase + l16, n - 1);
    if constexpr (DI == 64) {
      const uint4 u0 = *(const uint4*)(Kidx + row * DI + DPL * kq);
      const uint4 u1 = *(const uint4*)(Kidx + row * DI + DPL * kq + 8);
      ka[0] = u0.x; ka[1] = u0.y; ka[2] = u0.z; ka[3] = u0.w;
      ka[4] = u1.x; ka[5] = u1.y; ka[6] = u1.z; ka[7] = u1.w;
    } else {
      static_assert(DI == 16, "indexer head dim 64 or 16");
      const uint2 u0 = *(const uint2*)(Kidx + row * DI + DPL * kq);
      ka[0] = u0.x; ka[1] = u0.y;
    }
  }
  int posk[4];   // positions of the keys of this lane's result registers (row 4 r + kq)
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int key = kbase + 4 * r + kq;
    const int p = pos[(size_t)unit * C + min(key, n - 1)];
    posk[r] = (key < n) ? p : INT_MAX;
  }
  const bool hv = l16 < H_idx;
  const int jh = hv ? l16 : 0;
  float imp[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll 1
  for (int s = 0; s < n_q; ++s) {
    // B operand: lane (column l16 = head, kq) holds dims DPL kq .. of head l16 of query s
    double qd[DPL];
    {
      const uint4* src = (const uint4*)(qhat + (((size_t)b * n_q + s) * H_idx + jh) * DI + DPL * kq);
#pragma unroll
      for (int m = 0; m < DPL / 2; ++m) {
        const uint4 u = src[m];
        qd[2 * m] = __longlong_as_double(((long long)u.y << 32) | u.x);
        qd[2 * m + 1] = __longlong_as_double(((long long)u.w << 32) | u.z);
      }
    }
    const double al_in = alpha[((size_t)b * n_q + s) * H_idx + jh];
    const int qp = q_pos[(size_t)b * n_q + s];
    const double al = hv ? al_in : 0.0;   // (an absent head's column repeats head 0 and is gated off)
    im_v4d z = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int m = 0; m < DPL; ++m) {
      const uint32_t wd = ka[m >> 1];
      const float f = (m & 1) ? bf_hi(wd) : bf_lo(wd);
      z = __builtin_amdgcn_mfma_f64_16x16x4f64((double)f, qd[m], z, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const double sum = row16_sum_d(al * fmax(z[r], 0.0));   // over the heads, in every lane of the row
      imp[r] = (posk[r] <= qp) ? fmaxf(imp[r], (float)sum) : imp[r];
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int key = kbase + 4 * r + kq;
    if (l16 == 0 && key < n) scores[(size_t)unit * C + key] = imp[r];
  }
}

// scores[unit][key] = max over the query groups' partial maxima.  grid (ceil(max_live/256), units)
__global__ __launch_bounds__(256) void k_score_max(const float* __restrict__ part, int groups,
                                                   const int32_t* __restrict__ len, int C, int max_live,
                                                   float* __restrict__ scores) {
  const int unit = blockIdx.y, units = gridDim.y, key = blockIdx.x * 256 + threadIdx.x;
  if (key >= min(len[unit], max_live)) return;
  float v = -INFINITY;
  for (int g = 0; g < groups; ++g) v = fmaxf(v, part[((size_t)g * units + unit) * C + key]);
  scores[(size_t)unit * C + key] = v;
}

// ------------------------------------------------------------------------------------------
// a2: per-unit top-B by radix selection on (score key, position), then an ordered emission
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned block_excl_scan_1024(bool flag, unsigned* wsum, unsigned& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(flag);
  const unsigned inwave = __popcll(bal & ((1ull << lane) - 1ull));
  if (lane == 0) wsum[w] = __popcll(bal);
  __syncthreads();
  unsigned off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const unsigned v = wsum[i];
    if (i < w) off += v;
    tot += v;
  }
  __syncthreads();
  total = tot;
  return off + inwave;
}

// Of 256 bins, the first one (from bin 255 downwards if DESC, else from bin 0 upwards) at which the running
// count reaches rem (1 <= rem <= the total): its index, the count before it, and its own count, left in
// sh[0..2].  A scan by the first 4 waves of the workgroup (a serial walk over the bins by one thread cost
// ~10 us per radix pass).  All threads of the workgroup call it.
template <bool DESC>
__device__ __forceinline__ void select_pick_bin(const unsigned* hist, unsigned rem, unsigned* wtot, unsigned* sh) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int bin = DESC ? 255 - tid : tid;
  unsigned v = 0, incl = 0;
  if (tid < 256) {
    v = hist[bin];
    incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned t = __shfl_up(incl, o, 64);
      if (lane >= o) incl += t;
    }
    if (lane == 63) wtot[w] = incl;
  }
  __syncthreads();
  if (tid < 256) {
    for (int i = 0; i < w; ++i) incl += wtot[i];
    if (incl >= rem && incl - v < rem) { sh[0] = (unsigned)bin; sh[1] = incl - v; sh[2] = v; }
  }
  __syncthreads();
}

// grid (units), 1024 threads
__global__ __launch_bounds__(1024) void k_select(const float* __restrict__ scores,
                                                 const int32_t* __restrict__ pos,
                                                 const int32_t* __restrict__ len, int C, int max_live,
                                                 int budget, int n_sink, int n_recent,
                                                 int32_t* __restrict__ keep_idx,
                                                 int32_t* __restrict__ evict_idx,
                                                 int32_t* __restrict__ n_keep,
                                                 int32_t* __restrict__ n_evict,
                                                 int32_t* __restrict__ status) {
  __shared__ unsigned hist[256];
  __shared__ unsigned sh_prefix, sh_rem, sh_cnt, sh_pick[3];
  __shared__ int sh_red[16];
  __shared__ unsigned wsum[16];
  const int unit = blockIdx.x, tid = threadIdx.x;
  const int n_true = len[unit];
  const int n = min(n_true, max_live);
  const float* sc = scores + (size_t)unit * C;
  const int32_t* ps = pos + (size_t)unit * C;
  int32_t* keep = keep_idx + (size_t)unit * C;
  int32_t* evict = evict_idx + (size_t)unit * C;
  // A unit longer than the caller's promise is flagged and evicts nothing: its lists keep the first
  // max_live slots, so the memory update skips it, and the compaction (which sees the same length)
  // leaves it as it is.
  const bool over = n_true > max_live;
  if (over && tid == 0) atomicOr(status, IM_STATUS_LIVE_EXCEEDED_BIT);
  const int k = over ? n : min(budget, n);

  int maxpos = INT_MIN;
  if (n_recent > 0) {
    int m = INT_MIN;
    for (int i = tid; i < n; i += 1024) m = max(m, ps[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, 64));
    if ((tid & 63) == 0) sh_red[tid >> 6] = m;
    __syncthreads();
    for (int i = 0; i < 16; ++i) maxpos = max(maxpos, sh_red[i]);
    __syncthreads();
  }
  auto key_of = [&](int i) -> uint32_t {
    const int p = ps[i];
    const bool forced = (p < n_sink) || (n_recent > 0 && (long long)p > (long long)maxpos - n_recent);
    return forced ? IM_KEY_PINF : score_key(sc[i]);
  };

  if (k == n - 1 && n >= 2) {
    // One entry leaves (a decode step): it is the one ranked last: smallest score key, then largest
    // position, then largest slot.  One reduction instead of the radix passes; the lists follow from it.
    unsigned long long best = ~0ull;   // (key << 32) | ~position key: its minimum is the last-ranked (score, position)
    int bslot = -1;
    for (int i = tid; i < n; i += 1024) {
      const unsigned long long c = ((unsigned long long)key_of(i) << 32) | (uint32_t)(~((uint32_t)ps[i] ^ 0x80000000u));
      if (c <= best) { best = c; bslot = i; }   // ascending slots: <= keeps the largest
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const unsigned long long ob = __shfl_xor(best, o, 64);
      const int os = __shfl_xor(bslot, o, 64);
      if (os >= 0 && (bslot < 0 || ob < best || (ob == best && os > bslot))) { best = ob; bslot = os; }
    }
    __shared__ unsigned long long sh_b[16];
    if ((tid & 63) == 0) { sh_b[tid >> 6] = best; sh_red[tid >> 6] = bslot; }
    __syncthreads();
    for (int i = 0; i < 16; ++i) {
      const unsigned long long ob = sh_b[i];
      const int os = sh_red[i];
      if (os >= 0 && (bslot < 0 || ob < best || (ob == best && os > bslot))) { best = ob; bslot = os; }
    }
    const int e = bslot;
    for (int i = tid; i < n - 1; i += 1024) keep[i] = (i < e) ? i : i + 1;
    if (tid == 0) { evict[0] = e; n_keep[unit] = n - 1; n_evict[unit] = 1; }
    return;
  }
  // mode: 0 = keep all, 1 = keep none, 2 = threshold
  uint32_t T = 0, P = 0xffffffffu;
  unsigned rem2 = 0;
  bool all_ties = true;
  const int mode = (k >= n) ? 0 : (k == 0 ? 1 : 2);
  if (mode == 2) {
    // k-th largest score key
    if (tid == 0) { sh_prefix = 0; sh_rem = (unsigned)k; }
    uint32_t mask = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      const uint32_t prefix = sh_prefix;
      for (int i = tid; i < n; i += 1024) {
        const uint32_t key = key_of(i);
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      const unsigned rem = sh_rem;
      select_pick_bin<true>(hist, rem, wsum, sh_pick);
      if (tid == 0) {
        sh_prefix = prefix | (sh_pick[0] << shift);
        sh_rem = rem - sh_pick[1];
        sh_cnt = sh_pick[2];
      }
      mask |= 255u << shift;
      __syncthreads();
    }
    T = sh_prefix;
    const unsigned rem = sh_rem, cnt = sh_cnt;  // take `rem` of the `cnt` entries with key == T
    __syncthreads();
    if (rem < cnt) {
      // rem-th smallest position among the ties
      all_ties = false;
      if (tid == 0) { sh_prefix = 0; sh_rem = rem; }
      mask = 0;
      for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh_prefix;
        for (int i = tid; i < n; i += 1024) {
          if (key_of(i) != T) continue;
          const uint32_t pk = (uint32_t)ps[i] ^ 0x80000000u;
          if ((pk & mask) == prefix) atomicAdd(&hist[(pk >> shift) & 255u], 1u);
        }
        __syncthreads();
        const unsigned r = sh_rem;
        select_pick_bin<false>(hist, r, wsum, sh_pick);
        if (tid == 0) {
          sh_prefix = prefix | (sh_pick[0] << shift);
          sh_rem = r - sh_pick[1];
        }
        mask |= 255u << shift;
        __syncthreads();
      }
      P = sh_prefix;
      rem2 = sh_rem;  // take the first rem2 (in slot order) of the entries equal in score and position
      __syncthreads();
    }
  }

  // ordered emission
  unsigned kb = 0, eb = 0, qb = 0;
  for (int base = 0; base < n; base += 1024) {
    const int i = base + tid;
    const bool in = i < n;
    bool f = false, eq = false;
    if (in) {
      if (mode == 0) f = true;
      else if (mode == 2) {
        const uint32_t key = key_of(i);
        if (key > T) f = true;
        else if (key == T) {
          if (all_ties) f = true;
          else {
            const uint32_t pk = (uint32_t)ps[i] ^ 0x80000000u;
            if (pk < P) f = true;
            else if (pk == P) eq = true;
          }
        }
      }
    }
    if (mode == 2 && !all_ties) {  // uniform branch
      unsigned tot;
      const unsigned r = block_excl_scan_1024(eq, wsum, tot);
      if (eq && qb + r < rem2) f = true;
      qb += tot;
    }
    unsigned tot;
    const unsigned r = block_excl_scan_1024(f, wsum, tot);
    if (in) {
      if (f) keep[kb + r] = i;
      else evict[eb + (unsigned)tid - r] = i;
    }
    kb += tot;
    eb += (unsigned)min(1024, n - base) - tot;
  }
  if (tid == 0) { n_keep[unit] = (int)kb; n_evict[unit] = (int)eb; }
}

// ------------------------------------------------------------------------------------------
// a3: latent-memory write.  Partial sums over a split of the evicted rows on the matrix cores,
// then the decayed update (deterministic: splits are added in order).
// ------------------------------------------------------------------------------------------
#define IM_MEM_TOK 32  // evicted rows per MFMA tile (a sub-tile of the fold block)
#define IM_MEM_FEW 4   // up to this many evicted rows (a decode step evicts one) k_mem_finalize does the whole
                       // update in fp32 FMAs by itself and the partial kernels return at once

typedef short im_v4s __attribute__((ext_vector_type(4)));
typedef float im_v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int im_mem_blocks_per_split(int ne, int fold_block, int n_split) {
  const int blocks = (ne + fold_block - 1) / fold_block;
  return (blocks + n_split - 1) / n_split;
}

// grid (n_split, units), 4 waves.  Two chained bf16 MFMA products per tile of 32 evicted rows:
//   Phi^T[c][i] = sum_d W[c][d] K_i[d]            (wave w owns memory rows c = 32 w .. 32 w + 31)
//   M[c][d]    += sum_i Phi[i][c] V_i[d]          (Phi split into hi + lo bf16 parts, so the
//                                                  product carries 16 mantissa bits of Phi)
// 32x32x8 operand layout: lane l supplies row / column l % 32 and k = 4 (l / 32) .. + 3; result
// register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32.
__global__ __launch_bounds__(256) void k_mem_partial(const bf16_t* __restrict__ K,
                                                     const bf16_t* __restrict__ V,
                                                     const int32_t* __restrict__ evict_idx,
                                                     const int32_t* __restrict__ n_evict,
                                                     const bf16_t* __restrict__ Wtheta, int C,
                                                     int fold_block, int n_split,
                                                     float* __restrict__ part) {
  __shared__ float Ps[IM_DM][IM_MEM_TOK + 1];                                  // Phi^T [c][row]
  __shared__ __attribute__((aligned(16))) bf16_t Vs[IM_MEM_TOK][IM_D + 8];     // V rows of the tile
  const int unit = blockIdx.y, split = blockIdx.x, tid = threadIdx.x;
  const int ne = n_evict[unit];
  if (ne <= IM_MEM_FEW) return;
  const int bps = im_mem_blocks_per_split(ne, fold_block, n_split);
  const int i0 = split * bps * fold_block;
  const int i1 = min(ne, i0 + bps * fold_block);
  if (i0 >= i1) return;
  const int w = tid >> 6, lane = tid & 63, l32 = lane & 31, kh = lane >> 5;
  // W rows of this wave as the A operand of the first product: k-step ks covers dims 8 ks .. 8 ks + 7
  im_v4s wa[16];
#pragma unroll
  for (int ks = 0; ks < 16; ++ks)
    wa[ks] = *(const im_v4s*)(Wtheta + (32 * w + l32) * IM_D + 8 * ks + 4 * kh);
  im_v16f macc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) macc[db][r] = 0.f;
  float bsum[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) bsum[r] = 0.f;
  const int32_t* ev = evict_idx + (size_t)unit * C;
  // Software pipeline: the rows of tile t + 1 and the list entries of tile t + 2 are in flight while
  // tile t is in the matrix cores.  Entries past the end of the split repeat its last one and are
  // zeroed after the load.  This thread's rows: l32 for the K operand, vr0 / vr0 + 16 for V staging.
  const int vr0 = tid >> 4, vc16 = tid & 15;
  auto list_at = [&](int t) { return ev[min(t, i1 - 1)]; };
  int ek_n = list_at(i0 + l32), ev0_n = list_at(i0 + vr0), ev1_n = list_at(i0 + vr0 + 16);   // tile 0
  im_v4s kb[16], kb_n[16];
  uint4 vv0, vv1, vv0_n, vv1_n;
  {
    const bf16_t* kr = K + ((size_t)unit * C + ek_n) * IM_D + 4 * kh;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) kb_n[ks] = *(const im_v4s*)(kr + 8 * ks);
    vv0_n = *(const uint4*)(V + ((size_t)unit * C + ev0_n) * IM_D + vc16 * 8);
    vv1_n = *(const uint4*)(V + ((size_t)unit * C + ev1_n) * IM_D + vc16 * 8);
  }
  ek_n = list_at(i0 + IM_MEM_TOK + l32);                                                     // tile 1
  ev0_n = list_at(i0 + IM_MEM_TOK + vr0);
  ev1_n = list_at(i0 + IM_MEM_TOK + vr0 + 16);
#pragma unroll 1
  for (int t0 = i0; t0 < i1; t0 += IM_MEM_TOK) {
    // rotate: the prefetched rows become this tile's; issue the next tile's rows and the list
    // entries of the tile after it
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) kb[ks] = kb_n[ks];
    vv0 = vv0_n; vv1 = vv1_n;
    {
      const bf16_t* kr = K + ((size_t)unit * C + ek_n) * IM_D + 4 * kh;
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) kb_n[ks] = *(const im_v4s*)(kr + 8 * ks);
      vv0_n = *(const uint4*)(V + ((size_t)unit * C + ev0_n) * IM_D + vc16 * 8);
      vv1_n = *(const uint4*)(V + ((size_t)unit * C + ev1_n) * IM_D + vc16 * 8);
    }
    ek_n = list_at(t0 + 2 * IM_MEM_TOK + l32);
    ev0_n = list_at(t0 + 2 * IM_MEM_TOK + vr0);
    ev1_n = list_at(t0 + 2 * IM_MEM_TOK + vr0 + 16);
    if (t0 + l32 >= i1) {
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) kb[ks] = im_v4s{0, 0, 0, 0};
    }
    if (t0 + vr0 >= i1) vv0 = make_uint4(0, 0, 0, 0);
    if (t0 + vr0 + 16 >= i1) vv1 = make_uint4(0, 0, 0, 0);
    __syncthreads();   // the previous tile's LDS reads are done
    *(uint4*)&Vs[vr0][vc16 * 8] = vv0;
    *(uint4*)&Vs[vr0 + 16][vc16 * 8] = vv1;
    im_v16f ph;
#pragma unroll
    for (int r = 0; r < 16; ++r) ph[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) ph = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(wa[ks], kb[ks], ph, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      Ps[32 * w + 8 * (r >> 2) + 4 * kh + (r & 3)][l32] = ph[r];
      bsum[r] = fmaf(ph[r], ph[r], bsum[r]);
    }
    __syncthreads();
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {   // k-step kt covers rows 8 kt .. 8 kt + 7 of the tile
      im_v4s ah, al;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float p = Ps[32 * w + l32][8 * kt + 4 * kh + e];
        const bf16_t hi = f2bf_rne(p);
        const bf16_t lo = f2bf_rne(p - bf2f(hi));
        ah[e] = (short)hi;
        al[e] = (short)lo;
      }
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        im_v4s vb;
#pragma unroll
        for (int e = 0; e < 4; ++e) vb[e] = (short)Vs[8 * kt + 4 * kh + e][32 * db + l32];
        macc[db] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(ah, vb, macc[db], 0, 0, 0);
        macc[db] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(al, vb, macc[db], 0, 0, 0);
      }
    }
  }
  float* out = part + ((size_t)unit * n_split + split) * (IM_DM * IM_D + IM_DM);
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      out[(32 * w + 8 * (r >> 2) + 4 * kh + (r & 3)) * IM_D + 32 * db + l32] = macc[db][r];
  // sum_i Phi[i][c]^2: every lane holds the partial of its row position; add the 32 positions
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16; ++r) Ps[32 * w + 8 * (r >> 2) + 4 * kh + (r & 3)][l32] = bsum[r];
  __syncthreads();
  if (tid < IM_DM) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < IM_MEM_TOK; ++i) t += Ps[tid][i];
    out[IM_DM * IM_D + tid] = t;
  }
}

// The same for a set of H_set KV heads with one memory (Algorithm 1, `mem_write`: the evicted rows
// are summed across heads per token): Phi^T = sum_h W K_h and M += sum_h Phi V_h by linearity, so
// the sums over heads are taken inside the two products' accumulators and no summed row is ever
// rounded.  K, V are per unit (set * H_set + head); lists, counts and the partials per set.
// grid (n_split, sets), 4 waves.
__global__ __launch_bounds__(256) void k_mem_partial_sets(const bf16_t* __restrict__ K,
                                                          const bf16_t* __restrict__ V,
                                                          const int32_t* __restrict__ evict_idx,
                                                          const int32_t* __restrict__ n_evict,
                                                          const bf16_t* __restrict__ Wtheta, int C,
                                                          int H_set, int fold_block, int n_split,
                                                          float* __restrict__ part) {
  __shared__ float Ps[IM_DM][IM_MEM_TOK + 1];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[IM_MEM_TOK][IM_D + 8];
  const int set = blockIdx.y, split = blockIdx.x, tid = threadIdx.x;
  const int ne = n_evict[set];
  if (ne <= IM_MEM_FEW) return;
  const int bps = im_mem_blocks_per_split(ne, fold_block, n_split);
  const int i0 = split * bps * fold_block;
  const int i1 = min(ne, i0 + bps * fold_block);
  if (i0 >= i1) return;
  const int w = tid >> 6, lane = tid & 63, l32 = lane & 31, kh = lane >> 5;
  im_v4s wa[16];
#pragma unroll
  for (int ks = 0; ks < 16; ++ks)
    wa[ks] = *(const im_v4s*)(Wtheta + (32 * w + l32) * IM_D + 8 * ks + 4 * kh);
  im_v16f macc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) macc[db][r] = 0.f;
  float bsum[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) bsum[r] = 0.f;
  const int32_t* ev = evict_idx + (size_t)set * C;
  const int vr0 = tid >> 4, vc16 = tid & 15;
  // Software pipeline over (tile, head): while one head's rows are in the matrix cores the next head's
  // rows are in flight (K rows during the first product, V rows during the second; the last V phase of a
  // tile fetches the first K rows of the next tile), and a tile's list entries are read one tile ahead.
  // Entries past the end of the split repeat its last one; their rows are zeroed after the load.
  auto list_at = [&](int t) { return ev[min(t, i1 - 1)]; };
  auto load_k = [&](int hh, int slot, im_v4s* dst) {
    const bf16_t* kr = K + ((size_t)(set * H_set + hh) * C + slot) * IM_D + 4 * kh;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) dst[ks] = *(const im_v4s*)(kr + 8 * ks);
  };
  int ek = list_at(i0 + l32), ev0 = list_at(i0 + vr0), ev1 = list_at(i0 + vr0 + 16);
  im_v4s kb_n[16];
  load_k(0, ek, kb_n);
#pragma unroll 1
  for (int t0 = i0; t0 < i1; t0 += IM_MEM_TOK) {
    const int ek_n = list_at(t0 + IM_MEM_TOK + l32);
    const int ev0_n = list_at(t0 + IM_MEM_TOK + vr0), ev1_n = list_at(t0 + IM_MEM_TOK + vr0 + 16);
    const bool k_on = t0 + l32 < i1, v0_on = t0 + vr0 < i1, v1_on = t0 + vr0 + 16 < i1;
    im_v16f ph;
#pragma unroll
    for (int r = 0; r < 16; ++r) ph[r] = 0.f;
    uint4 vv0_n = make_uint4(0, 0, 0, 0), vv1_n = vv0_n;
#pragma unroll 1
    for (int hh = 0; hh < H_set; ++hh) {
      im_v4s kb[16];
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) kb[ks] = k_on ? kb_n[ks] : im_v4s{0, 0, 0, 0};
      if (hh + 1 < H_set) {
        load_k(hh + 1, ek, kb_n);
      } else {   // the first head's V rows of this tile
        const size_t ub = (size_t)(set * H_set) * C;
        vv0_n = *(const uint4*)(V + (ub + ev0) * IM_D + vc16 * 8);
        vv1_n = *(const uint4*)(V + (ub + ev1) * IM_D + vc16 * 8);
      }
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) ph = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(wa[ks], kb[ks], ph, 0, 0, 0);
    }
    __syncthreads();   // the previous tile's reads of Ps are done
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      Ps[32 * w + 8 * (r >> 2) + 4 * kh + (r & 3)][l32] = ph[r];
      bsum[r] = fmaf(ph[r], ph[r], bsum[r]);
    }
    __syncthreads();
    im_v4s ah[4], al[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float p = Ps[32 * w + l32][8 * kt + 4 * kh + e];
        const bf16_t hi = f2bf_rne(p);
        const bf16_t lo = f2bf_rne(p - bf2f(hi));
        ah[kt][e] = (short)hi;
        al[kt][e] = (short)lo;
      }
#pragma unroll 1
    for (int hh = 0; hh < H_set; ++hh) {
      const uint4 vv0 = v0_on ? vv0_n : make_uint4(0, 0, 0, 0);
      const uint4 vv1 = v1_on ? vv1_n : make_uint4(0, 0, 0, 0);
      if (hh + 1 < H_set) {
        const size_t ub = (size_t)(set * H_set + hh + 1) * C;
        vv0_n = *(const uint4*)(V + (ub + ev0) * IM_D + vc16 * 8);
        vv1_n = *(const uint4*)(V + (ub + ev1) * IM_D + vc16 * 8);
      } else {   // the first head's K rows of the next tile (of the last entry again, unused, after the last tile)
        load_k(0, ek_n, kb_n);
      }
      __syncthreads();   // the previous head's reads of Vs are done
      *(uint4*)&Vs[vr0][vc16 * 8] = vv0;
      *(uint4*)&Vs[vr0 + 16][vc16 * 8] = vv1;
      __syncthreads();
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          im_v4s vb;
#pragma unroll
          for (int e = 0; e < 4; ++e) vb[e] = (short)Vs[8 * kt + 4 * kh + e][32 * db + l32];
          macc[db] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(ah[kt], vb, macc[db], 0, 0, 0);
          macc[db] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(al[kt], vb, macc[db], 0, 0, 0);
        }
    }
    ek = ek_n; ev0 = ev0_n; ev1 = ev1_n;
  }
  float* out = part + ((size_t)set * n_split + split) * (IM_DM * IM_D + IM_DM);
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      out[(32 * w + 8 * (r >> 2) + 4 * kh + (r & 3)) * IM_D + 32 * db + l32] = macc[db][r];
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16; ++r) Ps[32 * w + 8 * (r >> 2) + 4 * kh + (r & 3)][l32] = bsum[r];
  __syncthreads();
  if (tid < IM_DM) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < IM_MEM_TOK; ++i) t += Ps[tid][i];
    out[IM_DM * IM_D + tid] = t;
  }
}

// grid (ceil((DM*D + DM)/256), sets): a workgroup owns two rows of M, the last one owns b.
// With at most IM_MEM_FEW evicted rows there are no partials: the workgroup sums the rows over the set's
// heads (fp32), takes Phi = W k for its own rows of W and applies the update itself.
__global__ __launch_bounds__(256) void k_mem_finalize(float* __restrict__ M, float* __restrict__ bvec,
                                                      const int32_t* __restrict__ n_evict,
                                                      const float* __restrict__ part, int fold_block,
                                                      int n_split, float lambda, float eta,
                                                      const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                                                      const int32_t* __restrict__ evict_idx,
                                                      const bf16_t* __restrict__ Wtheta, int C, int H_set) {
  const int unit = blockIdx.y;
  const int ne = n_evict[unit];
  if (ne <= 0) return;
  if (ne <= IM_MEM_FEW) {
    __shared__ float ks[IM_MEM_FEW][IM_D], vs[IM_MEM_FEW][IM_D], red[IM_MEM_FEW][4];
    const int tid = threadIdx.x, w = tid >> 6;
    const bool bblock = blockIdx.x == IM_DM * IM_D / 256;   // the workgroup of the 128 entries of b
    // this thread's weight and old entry of M depend on nothing: their loads go out with the list's
    float wv = 0.f, mold = 0.f;
    float* mdst = M + (size_t)unit * IM_DM * IM_D + (blockIdx.x * 2 + (tid >> 7)) * IM_D + (tid & 127);
    if (!bblock) {
      wv = bf2f(Wtheta[(blockIdx.x * 2 + (tid >> 7)) * IM_D + (tid & 127)]);
      mold = *mdst;
    }
    for (int idx = tid; idx < ne * IM_D; idx += 256) {
      const int i = idx >> 7, d = idx & 127;
      const int slot = evict_idx[(size_t)unit * C + i];
      float kk = 0.f, vv = 0.f;
      for (int hh = 0; hh < H_set; ++hh) {
        const size_t row = ((size_t)(unit * H_set + hh) * C + slot) * IM_D + d;
        kk += bf2f(K[row]);
        if (!bblock) vv += bf2f(V[row]);
      }
      ks[i][d] = kk;
      vs[i][d] = vv;
    }
    __syncthreads();
    if (bblock) {
      if (tid < IM_DM) {
        const uint4* wp = (const uint4*)(Wtheta + tid * IM_D);
        float ph[IM_MEM_FEW];
#pragma unroll
        for (int i = 0; i < IM_MEM_FEW; ++i) ph[i] = 0.f;
#pragma unroll 4
        for (int g = 0; g < 16; ++g) {
          const uint4 u = wp[g];
          const float wr[8] = {bf_lo(u.x), bf_hi(u.x), bf_lo(u.y), bf_hi(u.y),
                               bf_lo(u.z), bf_hi(u.z), bf_lo(u.w), bf_hi(u.w)};
#pragma unroll
          for (int i = 0; i < IM_MEM_FEW; ++i)
            if (i < ne) {
#pragma unroll
              for (int e = 0; e < 8; ++e) ph[i] = fmaf(wr[e], ks[i][8 * g + e], ph[i]);
            }
        }
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < IM_MEM_FEW; ++i)
          if (i < ne) s = fmaf(ph[i], ph[i], s);
        float* dst = bvec + (size_t)unit * IM_DM + tid;
        *dst = fmaf(lambda, *dst, eta * s);
      }
      return;
    }
    const int d = tid & 127;
    for (int i = 0; i < ne; ++i) {
      const float t = wave_sum_f(wv * ks[i][d]);
      if ((tid & 63) == 0) red[i][w] = t;
    }
    __syncthreads();
    float s = 0.f;
    for (int i = 0; i < ne; ++i) s = fmaf(red[i][w & 2] + red[i][(w & 2) + 1], vs[i][d], s);
    *mdst = fmaf(lambda, mold, eta * s);
    return;
  }
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= IM_DM * IM_D + IM_DM) return;
  const int bps = im_mem_blocks_per_split(ne, fold_block, n_split);
  const int active = ((ne + fold_block - 1) / fold_block + bps - 1) / bps;
  float s = 0.f;
  for (int sp = 0; sp < active; ++sp)
    s += part[((size_t)unit * n_split + sp) * (IM_DM * IM_D + IM_DM) + e];
  float* dst = (e < IM_DM * IM_D) ? (M + (size_t)unit * IM_DM * IM_D + e)
                                  : (bvec + (size_t)unit * IM_DM + (e - IM_DM * IM_D));
  *dst = fmaf(lambda, *dst, eta * s);
}

// ------------------------------------------------------------------------------------------
// a4: in-place compaction by hole filling.  One wave moves one entry (K, V, Kidx rows and pos).
// ------------------------------------------------------------------------------------------
// grid (gx, units): every KV head of a set applies the set's lists to its own K / V rows; the first
// head of the set also moves the set's indexer-key rows (di values each) and positions
__global__ __launch_bounds__(256) void k_compact(bf16_t* __restrict__ K, bf16_t* __restrict__ V,
                                                 bf16_t* __restrict__ Kidx, int32_t* __restrict__ pos,
                                                 int32_t* __restrict__ len,
                                                 int32_t* __restrict__ n_projected,
                                                 const int32_t* __restrict__ keep_idx,
                                                 const int32_t* __restrict__ n_keep,
                                                 const int32_t* __restrict__ evict_idx,
                                                 const int32_t* __restrict__ n_evict, int C, int H_set,
                                                 int di, int max_live, int32_t* __restrict__ status) {
  const int unit = blockIdx.y, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int set = unit / H_set;
  const bool lead = unit % H_set == 0;
  // a set longer than the caller's promise is flagged and left as it is (its lists cover only the
  // first max_live slots: applying them would drop the rest without a trace in the memory)
  if (len[set] > max_live) {
    if (lead && blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, IM_STATUS_LIVE_EXCEEDED_BIT);
    return;
  }
  const int nk = n_keep[set], ne = n_evict[set];
  const int32_t* keep = keep_idx + (size_t)set * C;
  const int32_t* evict = evict_idx + (size_t)set * C;
  // p = number of kept slots below nk = nk - number of evicted slots below nk (both lists ascend, and
  // together they hold every live slot once): found in the shorter list, one probe for a single eviction
  int p;
  if (ne < nk) {
    int lo = 0, hi = ne;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (evict[mid] < nk) lo = mid + 1; else hi = mid;
    }
    p = nk - lo;
  } else {
    int lo = 0, hi = nk;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (keep[mid] < nk) lo = mid + 1; else hi = mid;
    }
    p = lo;
  }
  const int n_moves = nk - p;
  for (int j = blockIdx.x * 4 + w; j < n_moves; j += gridDim.x * 4) {
    const int ss = keep[p + j], ds = evict[j];
    const size_t src = (size_t)unit * C + ss, dst = (size_t)unit * C + ds;
    const size_t isrc = (size_t)set * C + ss, idst = (size_t)set * C + ds;
    if (lane < 16) *(uint4*)(K + dst * IM_D + lane * 8) = *(const uint4*)(K + src * IM_D + lane * 8);
    else if (lane < 32) *(uint4*)(V + dst * IM_D + (lane - 16) * 8) = *(const uint4*)(V + src * IM_D + (lane - 16) * 8);
    else if (lane < 32 + di / 8) {
      if (lead) *(uint4*)(Kidx + idst * di + (lane - 32) * 8) = *(const uint4*)(Kidx + isrc * di + (lane - 32) * 8);
    } else if (lane == 40 && lead) pos[idst] = pos[isrc];
  }
  if (lead && blockIdx.x == 0 && threadIdx.x == 0) { len[set] = nk; n_projected[set] = nk; }
}

// The same Gather out of place: the kept entries of a source state go to the slots the in-place
// hole filling would leave them in, but of a destination state with its own capacity Cd (kept entry j of
// the ascending keep list: slot keep[j] if that is below n_keep, else the (j - p)-th evicted slot, p =
// number of kept slots below n_keep); the memory state is copied along; the destination's lengths are
// set.  The source is only read.  grid (gx, units), one wave per entry.
__global__ __launch_bounds__(256) void k_gather_kept(const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                                                     const bf16_t* __restrict__ Kidx,
                                                     const int32_t* __restrict__ pos,
                                                     const int32_t* __restrict__ len,
                                                     const float* __restrict__ M, const float* __restrict__ bvec,
                                                     bf16_t* __restrict__ Kd, bf16_t* __restrict__ Vd,
                                                     bf16_t* __restrict__ Kidxd, int32_t* __restrict__ posd,
                                                     int32_t* __restrict__ lend, int32_t* __restrict__ nprojd,
                                                     float* __restrict__ Md, float* __restrict__ bd,
                                                     const int32_t* __restrict__ keep_idx,
                                                     const int32_t* __restrict__ n_keep,
                                                     const int32_t* __restrict__ evict_idx, int C, int Cd,
                                                     int H_set, int di, int max_live,
                                                     int32_t* __restrict__ status) {
  const int unit = blockIdx.y, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int set = unit / H_set;
  const bool lead = unit % H_set == 0;
  const int nk = n_keep[set];
  // a set longer than the caller's promise has lists that cover only its first max_live slots, and a
  // kept set that does not fit the destination cannot be gathered: flagged, destination untouched
  if (len[set] > max_live || nk > Cd) {
    if (lead && blockIdx.x == 0 && threadIdx.x == 0)
      atomicOr(status, len[set] > max_live ? IM_STATUS_LIVE_EXCEEDED_BIT : IM_STATUS_APPEND_OVERFLOW_BIT);
    return;
  }
  const int32_t* keep = keep_idx + (size_t)set * C;
  const int32_t* evict = evict_idx + (size_t)set * C;
  int lo = 0, hi = nk;   // p = number of kept slots below nk (keep is ascending)
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (keep[mid] < nk) lo = mid + 1; else hi = mid;
  }
  const int p = lo;
  for (int j = blockIdx.x * 4 + w; j < nk; j += gridDim.x * 4) {
    const int ss = keep[j], ds = (j < p) ? ss : evict[j - p];
    const size_t src = (size_t)unit * C + ss, dst = (size_t)unit * Cd + ds;
    const size_t isrc = (size_t)set * C + ss, idst = (size_t)set * Cd + ds;
    if (lane < 16) *(uint4*)(Kd + dst * IM_D + lane * 8) = *(const uint4*)(K + src * IM_D + lane * 8);
    else if (lane < 32) *(uint4*)(Vd + dst * IM_D + (lane - 16) * 8) = *(const uint4*)(V + src * IM_D + (lane - 16) * 8);
    else if (lane < 32 + di / 8) {
      if (lead) *(uint4*)(Kidxd + idst * di + (lane - 32) * 8) = *(const uint4*)(Kidx + isrc * di + (lane - 32) * 8);
    } else if (lane == 40 && lead) posd[idst] = pos[isrc];
  }
  if (lead) {
    const float* Ms = M + (size_t)set * IM_DM * IM_D;
    float* Mo = Md + (size_t)set * IM_DM * IM_D;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < IM_DM * IM_D / 4; i += gridDim.x * 256)
      ((float4*)Mo)[i] = ((const float4*)Ms)[i];
    if (blockIdx.x == 0 && threadIdx.x < IM_DM) bd[(size_t)set * IM_DM + threadIdx.x] = bvec[(size_t)set * IM_DM + threadIdx.x];
    if (blockIdx.x == 0 && threadIdx.x == 0) { lend[set] = nk; nprojd[set] = nk; }
  }
}

// ------------------------------------------------------------------------------------------
// a5: split-K decode attention, then the combine with the gated memory readout
// ------------------------------------------------------------------------------------------
#define IM_ATT_CHUNK 128   // keys per workgroup: 32 per wave
#define IM_ATT_REC (IM_D + 2)  // partial record: running max, denominator, 128 numerators
#define IM_COMB_LDS 512        // chunks whose maxima and denominators the combine stages in LDS

// grid (chunks, units), 4 waves; wave w owns keys 32 w .. 32 w + 31 of the chunk as 2 tiles of 16.
// Logits on the bf16 matrix cores: S[key][head] = K_tile Q^T, 16x16x16, fp32 accumulation (operand lane
// (l16, kq): row l16, k = 4 kq .. 4 kq + 3 of a 16-wide step; a 32-dim chunk c of the rows gives two steps,
// lane (l16, kq) holding dims 32 c + 8 kq .. + 7 of row l16; result register r of the lane is key 4 kq + r,
// head l16).  Softmax statistics per wave (relative to the maximum of the wave's own 32 keys), the
// probabilities through LDS, P V with 16 lanes sharing a V row (8 dims each); the 4 waves' partials are
// rescaled to the chunk's maximum at the end.
typedef short im_att_v4s __attribute__((ext_vector_type(4)));
typedef float im_att_v4f __attribute__((ext_vector_type(4)));

template <int G>
__global__ __launch_bounds__(256) void k_attn_partial(const bf16_t* __restrict__ K,
                                                      const bf16_t* __restrict__ V,
                                                      const int32_t* __restrict__ len,
                                                      const bf16_t* __restrict__ q, int H, int H_kv,
                                                      int H_set, int C, int max_live, float scale,
                                                      float* __restrict__ part, int n_chunks,
                                                      int32_t* __restrict__ status) {
  __shared__ float s_ml[4][G][2];
  __shared__ float s_acc[4][G][IM_D];
  __shared__ float pl[IM_ATT_CHUNK][8];   // probabilities [key][head]
  const int unit = blockIdx.y, chunk = blockIdx.x;
  const int b = unit / H_kv, h = unit % H_kv;
  const int n_true = len[unit / H_set];
  const int n = min(n_true, max_live);
  if (n_true > max_live && chunk == 0 && threadIdx.x == 0) atomicOr(status, IM_STATUS_LIVE_EXCEEDED_BIT);
  const int k0 = chunk * IM_ATT_CHUNK;
  if (k0 >= n) return;
  const int nk = min(IM_ATT_CHUNK, n - k0);
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, kq = lane >> 4, l16 = lane & 15;
  const bf16_t* Kb = K + ((size_t)unit * C + k0) * IM_D;
  const bf16_t* Vb = V + ((size_t)unit * C + k0) * IM_D;
  // every load first (rows past the end of the chunk repeat its last row: finite values, masked below)
  uint4 kf[2][4], qf[4], vf[2][4];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int kr = min(16 * (2 * w + tt) + l16, nk - 1);
#pragma unroll
    for (int c = 0; c < 4; ++c) kf[tt][c] = load_stream16(Kb + (size_t)kr * IM_D + 32 * c + 8 * kq);
  }
  {
    const int jq = min(l16, G - 1);   // lanes past the group read its last head; zeroed where used
#pragma unroll
    for (int c = 0; c < 4; ++c) qf[c] = *(const uint4*)(q + ((size_t)b * H + h * G + jq) * IM_D + 32 * c + 8 * kq);
  }
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int vr = min(16 * (2 * w + tt) + 4 * i + kq, nk - 1);
      vf[tt][i] = load_stream16(Vb + (size_t)vr * IM_D + 8 * l16);
    }
  __asm__ volatile("" ::: "memory");   // keep the loads above the arithmetic, in this order
  float sreg[2][4];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    im_att_v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint4 ka = kf[tt][c], qb = (l16 < G) ? qf[c] : make_uint4(0, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(im_att_v4s, make_uint2(ka.x, ka.y)),
                                                      __builtin_bit_cast(im_att_v4s, make_uint2(qb.x, qb.y)), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(im_att_v4s, make_uint2(ka.z, ka.w)),
                                                      __builtin_bit_cast(im_att_v4s, make_uint2(qb.z, qb.w)), acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)   // this lane: head l16, key 16 (2 w + tt) + 4 kq + r
      sreg[tt][r] = (16 * (2 * w + tt) + 4 * kq + r < nk) ? acc[r] * scale : -INFINITY;
  }
  float lmax = fmaxf(fmaxf(fmaxf(sreg[0][0], sreg[0][1]), fmaxf(sreg[0][2], sreg[0][3])),
                     fmaxf(fmaxf(sreg[1][0], sreg[1][1]), fmaxf(sreg[1][2], sreg[1][3])));
  lmax = rows_max_f(lmax);   // over the wave's 32 keys, per head (lane column)
  const float mw = (lmax == -INFINITY) ? -1e30f : lmax;
  float lsum = 0.f;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float p = (sreg[tt][r] == -INFINITY) ? 0.f : __expf(sreg[tt][r] - mw);
      lsum += p;
      if (l16 < 8) pl[16 * (2 * w + tt) + 4 * kq + r][l16] = p;
    }
  lsum = rows_sum_f(lsum);
  if (kq == 0 && l16 < G) { s_ml[w][l16][0] = mw; s_ml[w][l16][1] = lsum; }
  // the probabilities just written are this wave's own keys: read back without a workgroup barrier
  // (LDS operations of one wave complete in order)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  float acc[G][8];
#pragma unroll
  for (int j = 0; j < G; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[j][e] = 0.f;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kl = 16 * (2 * w + tt) + 4 * i + kq;
      float pv[8];
      *(float4*)&pv[0] = *(const float4*)&pl[kl][0];
      if (G > 4) *(float4*)&pv[4] = *(const float4*)&pl[kl][4];
      const uint4 u = vf[tt][i];
      const float v[8] = {bf_lo(u.x), bf_hi(u.x), bf_lo(u.y), bf_hi(u.y),
                          bf_lo(u.z), bf_hi(u.z), bf_lo(u.w), bf_hi(u.w)};
#pragma unroll
      for (int j = 0; j < G; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[j][e] = fmaf(pv[j], v[e], acc[j][e]);
    }
  // the wave's 4 key streams (the same lane of the four 16-lane rows) share the wave's maximum: plain sums
#pragma unroll
  for (int j = 0; j < G; ++j) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[j][e] = rows_sum_f(acc[j][e]);
    if (kq == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s_acc[w][j][l16 * 8 + e] = acc[j][e];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * IM_D; idx += 256) {
    const int j = idx >> 7, d = idx & 127;
    float m = fmaxf(fmaxf(s_ml[0][j][0], s_ml[1][j][0]), fmaxf(s_ml[2][j][0], s_ml[3][j][0]));
    float o = 0.f, l = 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
      const float sc = __expf(s_ml[ww][j][0] - m);
      o = fmaf(sc, s_acc[ww][j][d], o);
      l = fmaf(sc, s_ml[ww][j][1], l);
    }
    float* rec = part + (((size_t)b * H + h * G + j) * n_chunks + chunk) * IM_ATT_REC;
    rec[2 + d] = o;
    if (d == 0) { rec[0] = m; rec[1] = l; }
  }
}

// grid (B*H), 128 threads (thread = output dim)
__global__ __launch_bounds__(128) void k_attn_combine(const float* __restrict__ part, int n_chunks,
                                                      const int32_t* __restrict__ len,
                                                      const bf16_t* __restrict__ q,
                                                      const bf16_t* __restrict__ Wtheta,
                                                      const bf16_t* __restrict__ wg, float cg,
                                                      const float* __restrict__ M,
                                                      const float* __restrict__ bvec, int H, int H_kv,
                                                      int H_set, int max_live, float mem_eps,
                                                      bf16_t* __restrict__ out,
                                                      float* __restrict__ readout_dbg) {
  __shared__ float qs[IM_D];
  __shared__ float phi[IM_DM];
  __shared__ float red[2][2];
  const int bh = blockIdx.x, tid = threadIdx.x;
  const int b = bh / H, j = bh % H, G = H / H_kv, h = j / G;
  const int unit = (b * H_kv + h) / H_set;   // the set: it owns the length and the memory state
  const int n = min(len[unit], max_live);
  const int nch = min((n + IM_ATT_CHUNK - 1) / IM_ATT_CHUNK, n_chunks);
  const float* rec = part + (size_t)bh * n_chunks * IM_ATT_REC;
  // the loads that depend on nothing go out first: q, this thread's row of W_theta, b, w_g
  const float qd = bf2f(q[(size_t)bh * IM_D + tid]);
  uint4 wrow[16];
  {
    const uint4* wr = (const uint4*)(Wtheta + tid * IM_D);
#pragma unroll
    for (int i = 0; i < 16; ++i) wrow[i] = wr[i];
  }
  const float bv = bvec[(size_t)unit * IM_DM + tid];
  const float wgv = bf2f(wg[tid]);
  // ... and this thread's column of the memory (row c of M is 512 contiguous bytes across the threads): 128
  // independent loads here instead of 8 dependent batches of 16 at the end
  float mcol[IM_DM];
  {
    const float* Mu = M + (size_t)unit * IM_DM * IM_D + tid;
#pragma unroll
    for (int c = 0; c < IM_DM; ++c) mcol[c] = Mu[c * IM_D];
  }
  float m = -1e30f, o = 0.f, l = 0.f;
  if (nch <= IM_COMB_LDS) {
    // thread c brings in chunk c's maximum and denominator (one round trip for all of them), the scale
    // factors are made once, and the numerators follow with 8 loads in flight; same sums in the same order
    // as the plain loops below
    __shared__ float cm[IM_COMB_LDS], cl[IM_COMB_LDS];
    for (int c = tid; c < nch; c += 128) {
      cm[c] = rec[(size_t)c * IM_ATT_REC];
      cl[c] = rec[(size_t)c * IM_ATT_REC + 1];
    }
    __syncthreads();
    for (int c = 0; c < nch; ++c) m = fmaxf(m, cm[c]);
    __syncthreads();
    for (int c = tid; c < nch; c += 128) cm[c] = __expf(cm[c] - m);
    __syncthreads();
#pragma unroll 8
    for (int c = 0; c < nch; ++c) {
      o = fmaf(cm[c], rec[(size_t)c * IM_ATT_REC + 2 + tid], o);
      l = fmaf(cm[c], cl[c], l);
    }
  } else {
#pragma unroll 4
    for (int c = 0; c < nch; ++c) m = fmaxf(m, rec[(size_t)c * IM_ATT_REC]);
#pragma unroll 4
    for (int c = 0; c < nch; ++c) {
      const float sc = __expf(rec[(size_t)c * IM_ATT_REC] - m);
      o = fmaf(sc, rec[(size_t)c * IM_ATT_REC + 2 + tid], o);
      l = fmaf(sc, rec[(size_t)c * IM_ATT_REC + 1], l);
    }
  }
  const float o_attn = (nch > 0) ? o / l : 0.f;
  // memory readout
  qs[tid] = qd;
  __syncthreads();
  float ph = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const uint4 u = wrow[i];
    ph = fmaf(bf_lo(u.x), qs[8 * i + 0], ph); ph = fmaf(bf_hi(u.x), qs[8 * i + 1], ph);
    ph = fmaf(bf_lo(u.y), qs[8 * i + 2], ph); ph = fmaf(bf_hi(u.y), qs[8 * i + 3], ph);
    ph = fmaf(bf_lo(u.z), qs[8 * i + 4], ph); ph = fmaf(bf_hi(u.z), qs[8 * i + 5], ph);
    ph = fmaf(bf_lo(u.w), qs[8 * i + 6], ph); ph = fmaf(bf_hi(u.w), qs[8 * i + 7], ph);
  }
  phi[tid] = ph;
  float den = wave_sum_f(ph * ph * bv);
  float gz = wave_sum_f(wgv * qd);
  if ((tid & 63) == 0) { red[tid >> 6][0] = den; red[tid >> 6][1] = gz; }
  __syncthreads();
  den = red[0][0] + red[1][0] + mem_eps;
  gz = red[0][1] + red[1][1] + cg;
  const float gate = 1.f / (1.f + __expf(-gz));
  float mr = 0.f;
#pragma unroll
  for (int c = 0; c < IM_DM; ++c) mr = fmaf(phi[c], mcol[c], mr);
  const float res = gate * (mr / den);
  out[(size_t)bh * IM_D + tid] = f2bf_rne(o_attn + res);
  if (readout_dbg) readout_dbg[(size_t)bh * IM_D + tid] = res;
}
