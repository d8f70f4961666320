// MV-RNN level kernel for gfx950, d = 64.
//
// Per node with left child (a, A) and right child (b, B):
//   p = tanh(W [B a ; A b]),   P = W_M [A ; B]          (W, W_M: [64,128])
// The two child matrices (16 KB each) are per-instance operands - this is the cell that
// multiplies two activations (section 7.2) - while W and W_M are shared by every node of
// every level (parameter reuse, section 5.1).  Children are read where they live: an
// internal child from the arena, a leaf child straight from the embedding tables (gather
// fusion, section 5.2; no copies of leaf embeddings, section 7.4).
//
// One workgroup (4 wavefronts) handles one node at a time and strides over the level, so
// the shared weights are loaded into registers once per workgroup:
//  * P (97 % of the flops) is a [64x128]x[128x64] product on the fp32 matrix cores.
//    Wavefront (mb, kh) owns output rows 32*mb..+31 and the k half kh (kh = 0: W_M[:, :64]
//    times A, kh = 1: W_M[:, 64:] times B).  W_M is the A operand and stays in 32 registers
//    for the whole launch.  The child matrix is the B operand and is loaded from global
//    memory directly in operand layout: lane l reads the two adjacent columns 2*(l%32),
//    2*(l%32)+1 of row 2s + l/32 (one 8-byte load, 256 contiguous bytes per half
//    wavefront); the even columns feed one accumulator block and the odd columns another,
//    so every lane ends up with adjacent output columns and stores them as one float2.
//    The two k halves are summed through LDS.
//  * the three small mat-vecs run on the vector ALUs: four lanes per output row, 16-wide
//    partial dot products, quad reduction with lane shuffles.
#include "cell_kernels.h"

namespace acrobat {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kD = 64;
constexpr int kDD = kD * kD;

__device__ __forceinline__ float fast_tanh(float x) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(__expf(2.0f * x) + 1.0f);
}

__device__ __forceinline__ float quad_sum(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

__global__ __launch_bounds__(256) void mvrnn_level_kernel(const MvrnnLevelArgs a) {
  __shared__ float s_ab[2 * kD];  // a | b
  __shared__ float s_v[2 * kD];   // B a | A b
  __shared__ float s_red[2][32 * 64];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mb = wave & 1, kh = wave >> 1;
  const int lcol = lane & 31, lhi = lane >> 5;

  // shared weights -> registers, once per workgroup
  float wm[32];  // W_M[32*mb + lcol][64*kh + 2s + lhi]
#pragma unroll
  for (int s = 0; s < 32; ++s) wm[s] = a.WM[(mb * 32 + lcol) * (2 * kD) + kh * kD + 2 * s + lhi];
  const int vr = tid >> 2, vq = tid & 3;  // mat-vec: output row, quarter of the columns
  floatx4 wv[8];                          // W[vr][32*vq .. +31]
#pragma unroll
  for (int k = 0; k < 8; ++k)
    wv[k] = *reinterpret_cast<const floatx4*>(a.W + vr * (2 * kD) + vq * 32 + k * 4);

  for (int node = blockIdx.x; node < a.n; node += gridDim.x) {
    const int ls = a.lsrc[node], rs = a.rsrc[node];
    const size_t orow = (size_t)a.out_rows[node];
    const float* va = ls >= 0 ? a.vec + (size_t)ls * kD : a.vec_tab + (size_t)(-(ls + 1)) * kD;
    const float* mA = ls >= 0 ? a.mat + (size_t)ls * kDD : a.mat_tab + (size_t)(-(ls + 1)) * kDD;
    const float* vb = rs >= 0 ? a.vec + (size_t)rs * kD : a.vec_tab + (size_t)(-(rs + 1)) * kD;
    const float* mB = rs >= 0 ? a.mat + (size_t)rs * kDD : a.mat_tab + (size_t)(-(rs + 1)) * kDD;

    // ---- matrix path: issue the operand loads first, they are the long latency
    const float* X = (kh ? mB : mA) + lhi * kD + 2 * lcol;
    floatx2 x[32];
#pragma unroll
    for (int s = 0; s < 32; ++s) x[s] = *reinterpret_cast<const floatx2*>(X + 2 * s * kD);

    // ---- vector path
    if (tid < kD) s_ab[tid] = va[tid];
    else if (tid < 2 * kD) s_ab[tid] = vb[tid - kD];
    __syncthreads();
    float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const floatx4 rb = *reinterpret_cast<const floatx4*>(mB + vr * kD + vq * 16 + k * 4);
      const floatx4 ra = *reinterpret_cast<const floatx4*>(mA + vr * kD + vq * 16 + k * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s0 += rb[e] * s_ab[vq * 16 + k * 4 + e];
        s1 += ra[e] * s_ab[kD + vq * 16 + k * 4 + e];
      }
    }
    s0 = quad_sum(s0);
    s1 = quad_sum(s1);
    if (vq == 0) {
      s_v[vr] = s0;
      s_v[kD + vr] = s1;
    }
    __syncthreads();
    float t = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
      for (int e = 0; e < 4; ++e) t += wv[k][e] * s_v[vq * 32 + k * 4 + e];
    t = quad_sum(t);
    if (vq == 0) a.vec[orow * kD + vr] = fast_tanh(t);

    // ---- matrix path: 32 k-steps of two 32x32 blocks (even / odd output columns)
    floatx16 acc_e, acc_o;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_e[v] = acc_o[v] = 0.0f;
#pragma unroll
    for (int s = 0; s < 32; ++s) {
      acc_e = __builtin_amdgcn_mfma_f32_32x32x2f32(wm[s], x[s][0], acc_e, 0, 0, 0);
      acc_o = __builtin_amdgcn_mfma_f32_32x32x2f32(wm[s], x[s][1], acc_o, 0, 0, 0);
    }
    if (kh == 1) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        s_red[mb][(2 * v) * 64 + lane] = acc_e[v];
        s_red[mb][(2 * v + 1) * 64 + lane] = acc_o[v];
      }
    }
    __syncthreads();
    if (kh == 0) {
      float* P = a.mat + orow * kDD;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = mb * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3);
        floatx2 o;
        o[0] = acc_e[v] + s_red[mb][(2 * v) * 64 + lane];
        o[1] = acc_o[v] + s_red[mb][(2 * v + 1) * 64 + lane];
        *reinterpret_cast<floatx2*>(P + i * kD + 2 * lcol) = o;
      }
    }
    __syncthreads();  // s_ab / s_v / s_red are reused by the next node
  }
}

__global__ __launch_bounds__(256) void mvrnn_leaf_copy_kernel(int n, const int32_t* out_rows,
                                                              const int32_t* token,
                                                              const float* vec_tab,
                                                              const float* mat_tab, float* vec,
                                                              float* mat) {
  const int tid = threadIdx.x;
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    const size_t src = (size_t)token[i], dst = (size_t)out_rows[i];
    const floatx4* ms = reinterpret_cast<const floatx4*>(mat_tab + src * kDD);
    floatx4* md = reinterpret_cast<floatx4*>(mat + dst * kDD);
#pragma unroll
    for (int k = 0; k < 4; ++k) md[tid + 256 * k] = ms[tid + 256 * k];
    if (tid < kD) vec[dst * kD + tid] = vec_tab[src * kD + tid];
  }
}

}  // namespace

hipError_t launch_mvrnn_level(const MvrnnLevelArgs& a, hipStream_t stream, int32_t* tile) {
  if (tile) *tile = 1;
  if (a.n <= 0) return hipSuccess;
  const int grid = a.n < 512 ? a.n : 512;  // two resident workgroups per compute unit, each strides over the level
  hipLaunchKernelGGL(mvrnn_level_kernel, dim3(grid), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_mvrnn_leaf_copy(int32_t n, const int32_t* out_rows, const int32_t* token,
                                  const float* vec_tab, const float* mat_tab, float* vec, float* mat,
                                  hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int grid = n < 2048 ? n : 2048;
  hipLaunchKernelGGL(mvrnn_leaf_copy_kernel, dim3(grid), dim3(256), 0, stream, n, out_rows, token,
                     vec_tab, mat_tab, vec, mat);
  return hipGetLastError();
}

}  // namespace acrobat
