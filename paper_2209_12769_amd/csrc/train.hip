// Supervised training of the fused-op estimator (Sec. 3.3.3) on gfx950, fp32.
//
// One pass = forward with the activations of every layer kept, the loss of Eq. (1) read as the
// mean squared difference of logarithms, and the reverse pass of exactly the forward formulas:
//     y = z2.w3 + b3,  z2 = ReLU(z1 W2 + b2),  z1 = ReLU(r W1 + b1),  r = sum of h_L over the
//     ops of the fused op (Secs. 3.3.1, 3.3.2),
//     h_{l+1} = ReLU([h_l | mean over predecessors | mean over successors] W_l + b_l).
// Dense products run on the fp32 matrix cores (32x32x2): forward and the data gradients through the
// layer update kernel, the weight gradients through wgrad_kernel below, whose contraction
// index is the row of the batch (transposed-A product, split over slabs of rows, partial
// results reduced in a fixed order, so a pass is bit-reproducible).  Everything else is
// bandwidth-bound and done by plain grid-stride kernels.  Adam as published by Kingma & Ba.
#include "common.h"

namespace dc {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

// ---- sample of each row: largest g with node_off[g] <= v (graphs may be empty) ----
__global__ __launch_bounds__(256) void gid_kernel(const int* __restrict__ node_off, int B, int* __restrict__ gid,
                                                  const int* __restrict__ status) {
  if (status[0] != 0) return;
  const long long ntot = node_off[B];
  for (long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x; v < ntot;
       v += (long long)gridDim.x * blockDim.x) {
    int lo = 0, hi = B;                 // invariant: node_off[lo] <= v < node_off[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (node_off[mid] <= v) lo = mid; else hi = mid;
    }
    gid[v] = lo;
  }
}

// ---- r[g] = sum over the rows of graph g, fp64 in ascending row order ----
__global__ __launch_bounds__(256) void readout_kernel(const float* __restrict__ h, int H,
                                                      const int* __restrict__ node_off, int B,
                                                      float* __restrict__ R, const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int cpr = H / 4;
  const long long total = (long long)B * cpr;
  const float4* __restrict__ h4 = reinterpret_cast<const float4*>(h);
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int g = (int)(idx / cpr), ch = (int)(idx - (long long)g * cpr);
    double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    for (int v = node_off[g]; v < node_off[g + 1]; ++v) {
      const float4 x = h4[(size_t)v * cpr + ch];
      a0 += x.x; a1 += x.y; a2 += x.z; a3 += x.w;
    }
    reinterpret_cast<float4*>(R)[idx] = make_float4((float)a0, (float)a1, (float)a2, (float)a3);
  }
}

// ---- per sample: y, the loss term and dL/dy; one wave per sample ----
__global__ __launch_bounds__(256) void loss_kernel(const float* __restrict__ Z2, int H, const float* __restrict__ w3b3,
                                                   const float* __restrict__ target, int B, float floor_,
                                                   float* __restrict__ y, float* __restrict__ dy,
                                                   double* __restrict__ lterm, float* __restrict__ pred,
                                                   int* __restrict__ status) {
  if (status[0] != 0) return;
  const int lane = threadIdx.x & 63;
  const int wpb = blockDim.x >> 6;
  for (int g = blockIdx.x * wpb + (threadIdx.x >> 6); g < B; g += gridDim.x * wpb) {
    // a profiled time is positive and finite: anything else has no logarithm, and the call is refused
    // (every later kernel of the call sees the status word and leaves its outputs alone)
    const float tg = target[g];
    if (!(tg > 0.f) || tg > 3.0e38f) {
      if (lane == 0) set_error(status, DC_ERR_INVALID_ARG);
      continue;
    }
    double s = 0.0;
    for (int j = lane; j < H; j += 64) s += (double)Z2[(size_t)g * H + j] * (double)w3b3[j];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) {
      const float yf = (float)(s + (double)w3b3[H]);
      const double yc = yf > floor_ ? (double)yf : (double)floor_;
      const double dl = log(yc) - log((double)tg);
      y[g] = yf;
      if (pred) pred[g] = yf;
      lterm[g] = dl * dl;
      dy[g] = yf > floor_ ? (float)(2.0 / (double)B * dl / yc) : 0.f;
    }
  }
}

// ---- loss = mean of the terms; one workgroup, fixed order ----
__global__ __launch_bounds__(1024) void loss_reduce_kernel(const double* __restrict__ lterm, int B,
                                                           float* __restrict__ loss,
                                                           const int* __restrict__ status) {
  if (status[0] != 0) return;
  __shared__ double red[1024];
  double s = 0.0;
  for (int g = threadIdx.x; g < B; g += 1024) s += lterm[g];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = B > 0 ? (float)(red[0] / (double)B) : 0.f;
}

// ---- dz2[g][j] = dy[g] w3[j] where z2 > 0 ----
__global__ __launch_bounds__(256) void dz2_kernel(const float* __restrict__ Z2, const float* __restrict__ dy,
                                                  const float* __restrict__ w3, int H, int B,
                                                  float* __restrict__ dZ2, const int* __restrict__ status) {
  if (status[0] != 0) return;
  const long long total = (long long)B * H;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int g = (int)(i / H), j = (int)(i - (long long)g * H);
    dZ2[i] = Z2[i] > 0.f ? dy[g] * w3[j] : 0.f;
  }
}

// ---- x = 0 where the activation is not positive (ReLU'), rows from a device count ----
__global__ __launch_bounds__(256) void relu_mask_kernel(float* __restrict__ x, const float* __restrict__ act,
                                                        const int* __restrict__ nrows, int H,
                                                        const int* __restrict__ status) {
  if (status[0] != 0) return;
  const long long total = (long long)nrows[0] * H;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x)
    if (!(act[i] > 0.f)) x[i] = 0.f;
}

// ---- gradient at the last layer's pre-activations: every op of a fused op receives dr ----
__global__ __launch_bounds__(256) void top_kernel(const float* __restrict__ dR, const int* __restrict__ gid,
                                                  const float* __restrict__ hL, const int* __restrict__ nrows, int H,
                                                  float* __restrict__ dZ, const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int cpr = H / 4;
  const long long total = (long long)nrows[0] * cpr;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const long long v = i / cpr;
    const int ch = (int)(i - v * cpr);
    const float4 g = reinterpret_cast<const float4*>(dR)[(size_t)gid[v] * cpr + ch];
    const float4 a = reinterpret_cast<const float4*>(hL)[i];
    reinterpret_cast<float4*>(dZ)[i] = make_float4(a.x > 0.f ? g.x : 0.f, a.y > 0.f ? g.y : 0.f,
                                                   a.z > 0.f ? g.z : 0.f, a.w > 0.f ? g.w : 0.f);
  }
}

// ---- WT [N, M] = transpose of W [M, N] ----
__global__ __launch_bounds__(256) void transpose_kernel(const float* __restrict__ W, int M, int N,
                                                        float* __restrict__ WT, const int* __restrict__ status) {
  if (status[0] != 0) return;
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  const int tm = (M + 31) / 32, tn = (N + 31) / 32;
  for (int t = blockIdx.x; t < tm * tn; t += gridDim.x) {
    const int m0 = (t / tn) * 32, n0 = (t % tn) * 32;
    for (int r = ty; r < 32; r += 8)
      tile[r][tx] = (m0 + r < M && n0 + tx < N) ? W[(size_t)(m0 + r) * N + n0 + tx] : 0.f;
    __syncthreads();
    for (int r = ty; r < 32; r += 8)
      if (n0 + r < N && m0 + tx < M) WT[(size_t)(n0 + r) * M + m0 + tx] = tile[tx][r];
    __syncthreads();
  }
}

// ---- reverse of the two neighbour means, plus the node's own block, then ReLU' of the layer below ----
// dA [rows, 3d] = dZ W^T holds per row v the gradient at [h[v] | mean over pred(v) | mean over succ(v)].
// h[u] enters the predecessor mean of each successor v with weight 1/indeg(v), and the successor
// mean of each predecessor v with weight 1/outdeg(v).
__global__ __launch_bounds__(256) void gather_back_kernel(const float* __restrict__ dA, int d,
                                                          const int* __restrict__ in_rp, const int* __restrict__ in_ci,
                                                          const int* __restrict__ out_rp,
                                                          const int* __restrict__ out_ci,
                                                          const float* __restrict__ h, const int* __restrict__ nrows,
                                                          float* __restrict__ dZ, const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int cpr = d / 4;
  const long long total = (long long)nrows[0] * cpr;
  const float4* __restrict__ A4 = reinterpret_cast<const float4*>(dA);
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const long long u = i / cpr;
    const int ch = (int)(i - u * cpr);
    float4 acc = A4[(size_t)u * 3 * cpr + ch];
    for (int k = out_rp[u]; k < out_rp[u + 1]; ++k) {
      const int v = out_ci[k];
      const float sc = 1.0f / (float)(in_rp[v + 1] - in_rp[v]);
      const float4 x = A4[(size_t)v * 3 * cpr + cpr + ch];
      acc.x += x.x * sc; acc.y += x.y * sc; acc.z += x.z * sc; acc.w += x.w * sc;
    }
    for (int k = in_rp[u]; k < in_rp[u + 1]; ++k) {
      const int v = in_ci[k];
      const float sc = 1.0f / (float)(out_rp[v + 1] - out_rp[v]);
      const float4 x = A4[(size_t)v * 3 * cpr + 2 * cpr + ch];
      acc.x += x.x * sc; acc.y += x.y * sc; acc.z += x.z * sc; acc.w += x.w * sc;
    }
    const float4 a = reinterpret_cast<const float4*>(h)[i];
    reinterpret_cast<float4*>(dZ)[i] = make_float4(a.x > 0.f ? acc.x : 0.f, a.y > 0.f ? acc.y : 0.f,
                                                   a.z > 0.f ? acc.z : 0.f, a.w > 0.f ? acc.w : 0.f);
  }
}

// ---- weight gradients: C [M, N] = sum over rows r of A[r][:]^T B[r][:], M = nseg * d ----
// One workgroup = one 256 x 128 tile of C over one slab of rows; 8 waves of 64 x 64 (4 accumulator
// blocks of 32 x 32 each; four waves per SIMD at two workgroups per CU).  The contraction index is the batch row: chunks of 16 rows of both
// operands are staged in LDS exactly as they lie in memory (row-major, 16-byte loads, each line read
// once per workgroup), double-buffered, with the next chunk's global loads in flight while the
// current one multiplies.  An MFMA block is free to take any 32 columns: block i of a wave takes
// columns 2*l + i of its 64 (l = lane mod 32), so one 8-byte LDS read feeds a lane's two A operands
// and another its two B operands.  The column sums of B (bias gradients) ride
// along in the waves of the first row of tiles.
constexpr int kTM = 256, kTN = 128, kRC = 16;
__device__ __forceinline__ float4 keep4(bool c, float4 x) {
  return make_float4(c ? x.x : 0.f, c ? x.y : 0.f, c ? x.z : 0.f, c ? x.w : 0.f);
}
__global__ __launch_bounds__(512) void wgrad_kernel(const float* __restrict__ A0, const float* __restrict__ A1,
                                                    const float* __restrict__ A2, int d, int nseg,
                                                    const float* __restrict__ Bm, int ldb, int N,
                                                    const int* __restrict__ nrows, float* __restrict__ part,
                                                    long long part_stride, int S, const int* __restrict__ status) {
  if (status[0] != 0) return;
  __shared__ __attribute__((aligned(16))) float As[2][kRC][kTM];
  __shared__ __attribute__((aligned(16))) float Bs[2][kRC][kTN];
  const int M = nseg * d;
  const int tiles_n = (N + kTN - 1) / kTN, tiles_m = (M + kTM - 1) / kTM;
  const int ntile = tiles_m * tiles_n;
  // Workgroups go round-robin to the 8 XCDs, each with an L2 of its own: workgroup b becomes work
  // item (b % 8) * (grid / 8) + b / 8, so that the tiles of one slab, which read the same rows, run
  // on one XCD (the grid is ntile * S with S a multiple of 8).
  const int per_xcd = gridDim.x >> 3;
  const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  const int tile = item % ntile, slab = item / ntile;
  if (slab >= S) return;
  const int m0 = (tile / tiles_n) * kTM, n0 = (tile % tiles_n) * kTN;
  const int rows = nrows[0];
  const int per = (rows + S - 1) / S;
  const long long r0 = (long long)slab * per;
  const long long r1 = r0 + per < rows ? r0 + per : rows;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, lh = lane >> 5;

  // loader roles: A rows arow + 8u (u < 2), 4 columns from am; B row brow, 4 columns from bn
  const int ac4 = t & 63, arow = t >> 6;                 // arow 0..7
  const int am = m0 + ac4 * 4;
  const bool aok = am < M;                               // M is a multiple of 4: all four columns or none
  const int aseg = aok ? am / d : 0;
  const float* pa = (aseg == 0 ? A0 : (aseg == 1 ? A1 : A2)) + (aok ? am - aseg * d : 0);
  const int bc4 = t & 31, brow = t >> 5;                 // brow 0..15
  const int bn = n0 + bc4 * 4;
  const bool bvec = (N & 3) == 0 && (ldb & 3) == 0;      // 16-byte loads of B are possible
  // Straight-line loads: a row past the slab's end re-reads the slab's last row (in bounds) and a column
  // past the matrix re-reads column 0; both are stored to LDS as zeros.
  const int bnc = bn < N ? bn : 0;
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 ra0 = zero4, ra1 = zero4, rb0 = zero4;
  const int ir1 = (int)r1, last = ir1 - 1;               // row counts fit an int
  auto fetch = [&](int rbase) {
    const int a0r = rbase + arow, a1r = a0r + 8, br = rbase + brow;
    ra0 = *reinterpret_cast<const float4*>(pa + (size_t)(a0r < ir1 ? a0r : last) * d);
    ra1 = *reinterpret_cast<const float4*>(pa + (size_t)(a1r < ir1 ? a1r : last) * d);
    const float* q = Bm + (size_t)(br < ir1 ? br : last) * ldb;
    if (bvec) {
      rb0 = *reinterpret_cast<const float4*>(q + bnc);
    } else {
      rb0 = zero4;
      if (bn < N) rb0.x = q[bn];
      if (bn + 1 < N) rb0.y = q[bn + 1];
      if (bn + 2 < N) rb0.z = q[bn + 2];
      if (bn + 3 < N) rb0.w = q[bn + 3];
    }
  };
  auto stash = [&](int buf, int rbase) {
    const int a0r = rbase + arow, a1r = a0r + 8, br = rbase + brow;
    *reinterpret_cast<float4*>(&As[buf][arow][ac4 * 4]) = keep4(aok && a0r < ir1, ra0);
    *reinterpret_cast<float4*>(&As[buf][arow + 8][ac4 * 4]) = keep4(aok && a1r < ir1, ra1);
    *reinterpret_cast<float4*>(&Bs[buf][brow][bc4 * 4]) = keep4(bn < N && br < ir1, rb0);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  float bsum[2] = {0.f, 0.f};

  const int nchunk = r1 > r0 ? (int)((r1 - r0 + kRC - 1) / kRC) : 0;       // the same for the whole workgroup
  if (nchunk > 0) {
    fetch((int)r0);
    stash(0, (int)r0);
  }
  __syncthreads();
  for (int c = 0; c < nchunk; ++c) {
    const int buf = c & 1;
    if (c + 1 < nchunk) fetch((int)r0 + (c + 1) * kRC);
    __builtin_amdgcn_sched_barrier(0);       // keep the global loads ahead of this chunk's products
#pragma unroll
    for (int ks = 0; ks < kRC / 2; ++ks) {
      const float2 a2 = *reinterpret_cast<const float2*>(&As[buf][2 * ks + lh][wm * 64 + l32 * 2]);
      const float2 b2 = *reinterpret_cast<const float2*>(&Bs[buf][2 * ks + lh][wn * 64 + l32 * 2]);
      const float a[2] = {a2.x, a2.y};
      const float b[2] = {b2.x, b2.y};
      bsum[0] += b2.x;
      bsum[1] += b2.y;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (c + 1 < nchunk) stash(buf ^ 1, (int)r0 + (c + 1) * kRC);   // buffer last read one iteration ago, before that barrier
    __syncthreads();
  }

  float* P = part + (size_t)slab * (size_t)part_stride;
  // accumulator register v of lane (l32, lh) holds row 8*(v/4) + 4*lh + (v%4), column l32 of its 32 x 32
  // block; block (i, j) row R is tile column 2R + i of the wave's 64, block column l is 2l + j of its 64
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + l32 * 2 + j;
    if (n >= N) continue;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 64 + (8 * (v >> 2) + 4 * lh + (v & 3)) * 2 + i;
        if (m < M) P[(size_t)m * N + n] = acc[i][j][v];
      }
  }
  if (m0 == 0 && wm == 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float tot = bsum[j] + __shfl_xor(bsum[j], 32, 64);
      const int n = n0 + wn * 64 + l32 * 2 + j;
      if (lh == 0 && n < N) P[(size_t)M * N + n] = tot;
    }
  }
}

// ---- the same product with the operands moved into LDS by DMA (global_load_lds_dwordx4) ----
// For d a multiple of 256, N a multiple of 128 and 16-byte aligned rows of B: a tile's 256 columns
// of A lie in one operand, so one wave instruction moves one row of the A chunk (64 lanes x 16
// bytes = its 256 floats) or two rows of the B chunk straight into the layout the products read,
// with no registers, LDS stores or selects in between.  Three chunk buffers: the DMA of chunk c+2
// is issued when chunk c starts, so a load has two chunks' products to land.  The compiler does
// not see these loads; the waits for them are placed by hand (loads return in issue order, so
// "at most three newer outstanding" means the chunk before the newest has landed).  Rows that do
// not fill a chunk at the end of a slab go through registers with zero fill.
typedef __attribute__((address_space(3))) char lds_char;
constexpr int kWgradRing = 3;
constexpr int kWgradLds = kWgradRing * kRC * (kTM + kTN) * 4;       // 73728
extern __shared__ __attribute__((aligned(1024))) char dc_wgrad_smem[];
__device__ __forceinline__ void dma16_to_lds(const void* gaddr, unsigned lds_base) {
  // lane l writes lds_base + 16 * l
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gaddr), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  // s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  asm volatile("s_waitcnt %0" : : "n"((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14)) : "memory");
}

__global__ __launch_bounds__(512) void wgrad_dma_kernel(const float* __restrict__ A0, const float* __restrict__ A1,
                                                        const float* __restrict__ A2, int d, int nseg,
                                                        const float* __restrict__ Bm, int ldb, int N,
                                                        const int* __restrict__ nrows, float* __restrict__ part,
                                                        long long part_stride, int S,
                                                        const int* __restrict__ status) {
  if (status[0] != 0) return;
  // dynamic LDS (72 KB, above the static limit): the A ring, then the B ring
  typedef float AChunk[kRC][kTM];
  typedef float BChunk[kRC][kTN];
  AChunk* As = reinterpret_cast<AChunk*>(dc_wgrad_smem);
  BChunk* Bs = reinterpret_cast<BChunk*>(dc_wgrad_smem + kWgradRing * sizeof(AChunk));
  constexpr int kRing = kWgradRing;
  const int M = nseg * d;                                // a multiple of kTM, N a multiple of kTN (host)
  const int tiles_n = N / kTN, tiles_m = M / kTM;
  const int ntile = tiles_m * tiles_n;
  const int per_xcd = gridDim.x >> 3;                    // see wgrad_kernel
  const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  const int tile = item % ntile, slab = item / ntile;
  if (slab >= S) return;
  const int m0 = (tile / tiles_n) * kTM, n0 = (tile % tiles_n) * kTN;
  const int rows = nrows[0];
  const int per = (rows + S - 1) / S;
  const long long r0l = (long long)slab * per;
  const int r0 = (int)(r0l < rows ? r0l : rows);
  const int r1 = r0 + per < rows ? r0 + per : rows;
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, lh = lane >> 5;
  const int aseg = m0 / d;                               // the tile's columns lie in one operand
  const float* Aseg = (aseg == 0 ? A0 : (aseg == 1 ? A1 : A2)) + (m0 - aseg * d);
  const unsigned ldsA = (unsigned)(size_t)((lds_char*)dc_wgrad_smem);
  const unsigned ldsB = ldsA + (unsigned)(kWgradRing * sizeof(AChunk));
  constexpr unsigned kABuf = kRC * kTM * 4, kBBuf = kRC * kTN * 4;   // bytes per ring slot
  const int nfull = (r1 - r0) / kRC;                     // chunks moved by DMA; the same for the whole workgroup

  // wave w moves rows 2w and 2w+1 of the A chunk (one instruction each) and rows 2w, 2w+1 of the B
  // chunk (one instruction: lanes 0-31 the first, lanes 32-63 the second): three per wave and chunk
  auto dma_chunk = [&](int c) {
    const int slot = c % kRing;
    const size_t row = (size_t)(r0 + c * kRC + 2 * wave);           // < r1 - 1: the chunk is full
    dma16_to_lds(Aseg + row * d + lane * 4, ldsA + slot * kABuf + (2 * wave) * (kTM * 4));
    dma16_to_lds(Aseg + (row + 1) * d + lane * 4, ldsA + slot * kABuf + (2 * wave + 1) * (kTM * 4));
    dma16_to_lds(Bm + (row + lh) * ldb + n0 + l32 * 4, ldsB + slot * kBBuf + (2 * wave) * (kTN * 4));
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  float bsum[2] = {0.f, 0.f};
  auto multiply = [&](int slot) {
    // the operands of the next row pair are requested before the products of the current one
    float2 a2 = *reinterpret_cast<const float2*>(&As[slot][lh][wm * 64 + l32 * 2]);
    float2 b2 = *reinterpret_cast<const float2*>(&Bs[slot][lh][wn * 64 + l32 * 2]);
#pragma unroll
    for (int ks = 0; ks < kRC / 2; ++ks) {
      float2 an = a2, bn = b2;
      if (ks + 1 < kRC / 2) {
        an = *reinterpret_cast<const float2*>(&As[slot][2 * ks + 2 + lh][wm * 64 + l32 * 2]);
        bn = *reinterpret_cast<const float2*>(&Bs[slot][2 * ks + 2 + lh][wn * 64 + l32 * 2]);
      }
      __builtin_amdgcn_sched_barrier(0);
      bsum[0] += b2.x;
      bsum[1] += b2.y;
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.x, b2.x, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.x, b2.y, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.y, b2.x, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.y, b2.y, acc[1][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      a2 = an;
      b2 = bn;
    }
  };

  if (nfull > 0) dma_chunk(0);
  if (nfull > 1) dma_chunk(1);
  for (int c = 0; c < nfull; ++c) {
    // this wave's part of chunk c has landed (newer: chunk c+1's three, if it exists) ...
    if (c + 1 < nfull) wait_vmcnt<3>(); else wait_vmcnt<0>();
    // ... and so has everybody's; all waves are also done with chunk c-1, whose slot chunk c+2 takes
    __syncthreads();
    if (c + 2 < nfull) dma_chunk(c + 2);
    multiply(c % kRing);
  }
  if (r0 + nfull * kRC < r1) {
    // the rows left over: through registers, zero-filled, into the slot after the last chunk's
    // (last read two chunks ago; no DMA is outstanding)
    const int slot = nfull % kRing;
    const int rbase = r0 + nfull * kRC;
    const int ac4 = t & 63, arow = t >> 6, bc4 = t & 31, brow = t >> 5;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int r = rbase + arow + 8 * u;
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < r1) x = *reinterpret_cast<const float4*>(Aseg + (size_t)r * d + ac4 * 4);
      *reinterpret_cast<float4*>(&As[slot][arow + 8 * u][ac4 * 4]) = x;
    }
    {
      const int r = rbase + brow;
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < r1) x = *reinterpret_cast<const float4*>(Bm + (size_t)r * ldb + n0 + bc4 * 4);
      *reinterpret_cast<float4*>(&Bs[slot][brow][bc4 * 4]) = x;
    }
    __syncthreads();
    multiply(slot);
  }

  float* P = part + (size_t)slab * (size_t)part_stride;
  // same block-to-column assignment as wgrad_kernel
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + l32 * 2 + j;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 64 + (8 * (v >> 2) + 4 * lh + (v & 3)) * 2 + i;
        P[(size_t)m * N + n] = acc[i][j][v];
      }
  }
  if (m0 == 0 && wm == 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float tot = bsum[j] + __shfl_xor(bsum[j], 32, 64);
      const int n = n0 + wn * 64 + l32 * 2 + j;
      if (lh == 0) P[(size_t)M * N + n] = tot;
    }
  }
}

// gW [M*N] and gb [N] = sums of the slabs' partial results, fp64, ascending slab order
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part, long long part_stride,
                                                           int S, long long MN, int N, float* __restrict__ gW,
                                                           float* __restrict__ gb, const int* __restrict__ status) {
  if (status[0] != 0) return;
  const long long total = MN + (gb ? N : 0);
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    double s = 0.0;
    for (int k = 0; k < S; ++k) s += (double)part[(size_t)k * (size_t)part_stride + i];
    if (i < MN) gW[i] = (float)s; else gb[i - MN] = (float)s;
  }
}

__global__ void set_count_kernel(int* cnt, int n) {
  cnt[0] = 0;
  cnt[1] = n;
}

__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ theta, const float* __restrict__ g,
                                                   float* __restrict__ m, float* __restrict__ v, long long n,
                                                   float lr, float beta1, float beta2, float eps, float c1, float c2,
                                                   const int* __restrict__ status) {
  if (status[0] != 0) return;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (long long)gridDim.x * blockDim.x) {
    const float gi = g[i];
    const float mi = beta1 * m[i] + (1.f - beta1) * gi;
    const float vi = beta2 * v[i] + (1.f - beta2) * gi * gi;
    m[i] = mi;
    v[i] = vi;
    theta[i] -= lr * (mi * c1) / (sqrtf(vi * c2) + eps);      // c1 = 1/(1-beta1^t), c2 = 1/(1-beta2^t)
  }
}

int grid_for(long long items, int n_cu) {
  long long g = (items + 255) / 256;
  const long long cap = (long long)n_cu * 16;
  if (g > cap) g = cap;
  return g < 1 ? 1 : (int)g;
}

// slabs of a product with ntile tiles: one round of workgroups at two per CU, a multiple of 8
int slabs_for(int ntile, int n_cu, int cap) {
  int S = ((2 * n_cu) / ntile) & ~7;
  if (S > cap) S = cap;
  return S < 8 ? 8 : S;
}

// C = sum over rows of [A0|A1|A2]^T B into gW (and column sums of B into gb)
void weight_gradient(const TrainPass& t, const float* A0, const float* A1, const float* A2, int d, int nseg,
                     const float* Bm, int ldb, int N, const int* nrows, float* gW, float* gb, hipStream_t s) {
  const int M = nseg * d;
  const int ntile = ((M + kTM - 1) / kTM) * ((N + kTN - 1) / kTN);
  const int S = slabs_for(ntile, t.n_cu, t.slabs);
  const long long stride = (long long)M * N + N;
  static bool lds_ok = false, lds_tried = false;
  if (!lds_tried) {
    lds_tried = true;
    lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad_dma_kernel),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, kWgradLds) == hipSuccess;
  }
  if (lds_ok && d % kTM == 0 && N % kTN == 0 && ldb % 4 == 0)
    hipLaunchKernelGGL(wgrad_dma_kernel, dim3(ntile * S), dim3(512), kWgradLds, s, A0, A1, A2, d, nseg, Bm, ldb, N, nrows,
                       t.part, stride, S, t.status);
  else
    hipLaunchKernelGGL(wgrad_kernel, dim3(ntile * S), dim3(512), 0, s, A0, A1, A2, d, nseg, Bm, ldb, N, nrows,
                       t.part, stride, S, t.status);
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(grid_for(stride, t.n_cu)), dim3(256), 0, s, t.part, stride, S,
                     (long long)M * N, N, gW, gb, t.status);
}

}  // namespace

int train_slabs(int n_cu, int F, int H) {
  // the largest slab count weight_gradient() uses (the partial-result buffer is sized for it)
  (void)n_cu;
  (void)F;
  (void)H;
  return 128;
}

hipError_t launch_train_pass(const TrainPass& t, Profiler* prof, hipStream_t s) {
  auto begin = [&](int fam) { if (prof) prof->begin(fam, s); };
  auto end = [&]() { if (prof) prof->end(s); };
  const int B = t.n_samples, H = t.H, F = t.F, L = t.L;
  const size_t HH = (size_t)H * H;
  const int* nrows = t.node_off + B;          // device-resident row count
  GnnArgs g{};
  g.n_cand = B;
  g.node_off = t.node_off;
  g.out_rowptr = t.out_rowptr;
  g.out_col = t.out_col;
  g.in_rowptr = t.in_rowptr;
  g.in_col = t.in_col;
  g.H = H;
  g.bf16 = 0;
  g.status = t.status;
  g.n_cu = t.n_cu;
  GnnArgs gh = g;                              // the regression network: one row per sample
  gh.n_cand = 1;
  gh.node_off = t.cnt;
  const long long rows_cap = t.max_rows;
  const size_t dmax = (size_t)(F > H ? F : H);
  const float* W1 = t.head;
  const float* b1 = W1 + HH;
  const float* W2 = b1 + H;
  const float* b2 = W2 + HH;
  const float* w3 = b2 + H;                    // followed by b3
  // gradient vector: W_layers | b_layers | W1 b1 W2 b2 w3 b3
  size_t nW = 0;
  for (int l = 0; l < L; ++l) nW += (size_t)3 * (l == 0 ? F : H) * H;
  float* gWl = t.grad;
  float* gbl = t.grad + nW;
  float* gW1 = gbl + (size_t)L * H;
  float* gb1 = gW1 + HH;
  float* gW2 = gb1 + H;
  float* gb2 = gW2 + HH;
  float* gw3 = gb2 + H;
  float* gb3 = gw3 + H;

  hipLaunchKernelGGL(set_count_kernel, dim3(1), dim3(1), 0, s, t.cnt, B);
  hipLaunchKernelGGL(gid_kernel, dim3(grid_for(rows_cap, t.n_cu)), dim3(256), 0, s, t.node_off, B, t.gid, t.status);

  // ---- forward, every layer's output kept ----
  const float* hcur = t.X;
  int d = F;
  const float* Wl = t.W;
  const float* bl = t.b;
  for (int l = 0; l < L; ++l) {
    float* hn = t.hs + (size_t)l * rows_cap * H;
    float* mp = t.means + (size_t)(2 * l) * rows_cap * dmax;      // both means are kept for the reverse pass
    float* ms = mp + (size_t)rows_cap * dmax;
    begin(kFamTrainAggregate);
    launch_mean_aggregate(g, hcur, d, mp, ms, s);
    end();
    begin(kFamTrainUpdate);
    launch_dense_update(g, hcur, mp, ms, d, 3, Wl, bl, hn, s);
    end();
    Wl += (size_t)3 * d * H;
    bl += H;
    hcur = hn;
    d = H;
  }
  begin(kFamTrainHead);
  hipLaunchKernelGGL(readout_kernel, dim3(grid_for((long long)B * (H / 4), t.n_cu)), dim3(256), 0, s, hcur, H,
                     t.node_off, B, t.R, t.status);
  launch_dense_update(gh, t.R, nullptr, nullptr, H, 1, W1, b1, t.Z1, s);
  launch_dense_update(gh, t.Z1, nullptr, nullptr, H, 1, W2, b2, t.Z2, s);
  hipLaunchKernelGGL(loss_kernel, dim3(grid_for((long long)B * 64, t.n_cu)), dim3(256), 0, s, t.Z2, H, w3, t.target, B,
                     t.floor, t.y, t.dy, t.lterm, t.pred, t.status);
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, t.lterm, B, t.loss, t.status);
  if (!t.grad) {
    end();
    return hipGetLastError();
  }

  // ---- regression network, reverse ----
  const int* nB = t.cnt + 1;
  weight_gradient(t, t.Z2, nullptr, nullptr, H, 1, t.dy, 1, 1, nB, gw3, gb3, s);
  hipLaunchKernelGGL(dz2_kernel, dim3(grid_for((long long)B * H, t.n_cu)), dim3(256), 0, s, t.Z2, t.dy, w3, H, B,
                     t.dZ2, t.status);
  weight_gradient(t, t.Z1, nullptr, nullptr, H, 1, t.dZ2, H, H, nB, gW2, gb2, s);
  hipLaunchKernelGGL(transpose_kernel, dim3(64), dim3(256), 0, s, W2, H, H, t.WT, t.status);
  launch_dense_update(gh, t.dZ2, nullptr, nullptr, H, 1, t.WT, nullptr, t.dZ1, s);
  hipLaunchKernelGGL(relu_mask_kernel, dim3(grid_for((long long)B * H, t.n_cu)), dim3(256), 0, s, t.dZ1, t.Z1, nB, H,
                     t.status);
  weight_gradient(t, t.R, nullptr, nullptr, H, 1, t.dZ1, H, H, nB, gW1, gb1, s);
  hipLaunchKernelGGL(transpose_kernel, dim3(64), dim3(256), 0, s, W1, H, H, t.WT, t.status);
  launch_dense_update(gh, t.dZ1, nullptr, nullptr, H, 1, t.WT, nullptr, t.dR, s);

  // ---- graph layers, reverse ----
  float* dZ = t.dZ[0];
  float* dZn = t.dZ[1];
  hipLaunchKernelGGL(top_kernel, dim3(grid_for(rows_cap * (H / 4), t.n_cu)), dim3(256), 0, s, t.dR, t.gid, hcur, nrows,
                     H, dZ, t.status);
  end();
  GnnArgs g3 = g;
  g3.H = 3 * H;                                // dA = dZ W^T is [rows, 3H] for the layers above the first
  for (int l = L - 1; l >= 0; --l) {
    const int dl = l == 0 ? F : H;
    const float* hl = l == 0 ? t.X : t.hs + (size_t)(l - 1) * rows_cap * H;
    size_t woff = 0;
    for (int k = 0; k < l; ++k) woff += (size_t)3 * (k == 0 ? F : H) * H;
    const float* mp = t.means + (size_t)(2 * l) * rows_cap * dmax;
    const float* ms = mp + (size_t)rows_cap * dmax;
    begin(kFamTrainWgrad);
    weight_gradient(t, hl, mp, ms, dl, 3, dZ, H, H, nrows, gWl + woff, gbl + (size_t)l * H, s);
    end();
    if (l == 0) break;
    begin(kFamTrainDgrad);
    hipLaunchKernelGGL(transpose_kernel, dim3(128), dim3(256), 0, s, t.W + woff, 3 * H, H, t.WT, t.status);
    launch_dense_update(g3, dZ, nullptr, nullptr, H, 1, t.WT, nullptr, t.dA, s);
    end();
    begin(kFamTrainGatherBack);
    hipLaunchKernelGGL(gather_back_kernel, dim3(grid_for(rows_cap * (H / 4), t.n_cu)), dim3(256), 0, s, t.dA, H,
                       t.in_rowptr, t.in_col, t.out_rowptr, t.out_col, hl, nrows, dZn, t.status);
    end();
    float* tmp = dZ;
    dZ = dZn;
    dZn = tmp;
  }
  return hipGetLastError();
}

hipError_t launch_adam(float* theta, const float* grad, float* m, float* v, long long n, float lr, float beta1,
                       float beta2, float eps, double c1, double c2, const int* status, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(adam_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, theta, grad, m, v, n, lr, beta1, beta2,
                     eps, (float)c1, (float)c2, status);
  return hipGetLastError();
}

}  // namespace dc
