// Gather-fused cell kernels for gfx950 (TreeLSTM leaf / internal level, LSTM input
// transform and step).
//
// One launch executes one depth level of the schedule (section 4.1).  The kernel reads the
// level's operand rows straight from the arena through index lists instead of from a
// gathered contiguous copy (gather fusion, section 5.2), contracts them with the shared
// weight matrix once for all gates (parameter reuse, section 5.1; horizontal fusion,
// appendix B.3) on the fp32 matrix cores and applies the gate non-linearities and the state
// update before anything is written back (vertical fusion, section 7.5).
//
// Tiling.  A workgroup of four wavefronts owns BM = 32*WM nodes and 32 hidden units j, and
// for those it computes ALL G gates: the weight tile is made of G row blocks of the weight
// matrix (rows g*H + j0 .. +31), so no packing of the weights is needed and the epilogue
// finds every gate of a (node, j) pair in the same lane and register slot.  The k loop
// streams 32-column slabs of both operands through LDS with a register prefetch of the
// next slab.  Wavefronts are arranged WM (node blocks) x WK (k split inside a slab); small
// levels use WK > 1 so that all four matrix pipes of the CU work on a 32-node tile.
//
// Matrix instruction: v_mfma_f32_32x32x2_f32.  Lane l supplies A[i = l%32][k = l/32] and
// B[k = l/32][j = l%32]; the 16 result registers of lane l hold column j = l%32 and rows
// i = 8*(v/4) + 4*(l/32) + v%4.  Rows are nodes, columns are hidden units, so stores are
// 128-byte contiguous per half wavefront.  Each lane fetches four consecutive k of its row
// with one 16-byte LDS read and feeds them to four instructions; lanes 32..63 take the
// upper four k of an 8-k group, which is just a permutation of the summation order applied
// to both operands alike.
#include "cell_kernels.h"

namespace acrobat {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;        // k columns per slab
constexpr int kLdT = kBK + 4;  // LDS row stride (floats): 16-byte aligned, conflict-free b128 reads
constexpr int kThreads = 256;

__device__ __forceinline__ float fast_sigmoid(float x) {
  return __builtin_amdgcn_rcpf(1.0f + __expf(-x));  // exp -> inf gives 0, exp -> 0 gives 1
}
__device__ __forceinline__ float fast_tanh(float x) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(__expf(2.0f * x) + 1.0f);  // saturates to +-1
}

template <int EPI>
__device__ __forceinline__ constexpr int gate_row(int g) {
  // row block (in units of H) of computed gate g inside the weight matrix
  return EPI == EPI_TREE_LEAF ? (g == 0 ? 0 : g + 2) : g;  // leaf: i, o, u = blocks 0, 3, 4
}

template <int G, int EPI, int WM, int WK>
__global__ __launch_bounds__(kThreads) void cell_level_kernel(const CellLevelArgs a) {
  static_assert(WM * WK == 4, "four wavefronts per workgroup");
  constexpr int BM = 32 * WM;
  constexpr int BROWS = 32 * G;
  constexpr int TILE_FLOATS = (BM + BROWS) * kLdT;
  constexpr int RED_FLOATS = WK > 1 ? WM * G * 16 * 64 : 0;
  constexpr int SMEM_FLOATS = TILE_FLOATS > RED_FLOATS ? TILE_FLOATS : RED_FLOATS;
  __shared__ __attribute__((aligned(16))) float smem[SMEM_FLOATS];
  float* As = smem;
  float* Bs = smem + BM * kLdT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wk = wave / WM;
  const int H = a.H, n = a.n;
  const int n_jt = H >> 5;
  const int jt = blockIdx.x % n_jt, mt = blockIdx.x / n_jt;
  const int j0 = jt * 32, m0 = mt * BM;

  // ---- global -> LDS staging assignment: 16-byte chunk `tid & 7` of tile row `tid >> 3` (+32 i)
  const int lrow = tid >> 3, lpart = (tid & 7) * 4;
  const float* aptr0[WM];
  const float* aptr1[WM];
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    int node = m0 + lrow + 32 * i;
    node = node < n ? node : n - 1;  // tail rows re-read the last node; never stored
    aptr0[i] = aptr1[i] = nullptr;
    if (a.nseg > 0) {
      const size_t r0 = a.idx0 ? (size_t)a.idx0[node] : (size_t)node;
      aptr0[i] = a.src0 + r0 * (size_t)a.ld0 + lpart;
    }
    if (a.nseg > 1) {
      const size_t r1 = a.idx1 ? (size_t)a.idx1[node] : (size_t)node;
      aptr1[i] = a.src1 + r1 * (size_t)a.ld1 + lpart;
    }
  }
  const float* bptr[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    bptr[g] = a.W + (size_t)(gate_row<EPI>(g) * H + j0 + lrow) * (size_t)a.ldw + lpart;

  floatx16 acc[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[g][v] = 0.0f;

  const int slabs_per_seg = a.kseg / kBK;
  const int n_slabs = a.nseg * slabs_per_seg;

  floatx4 ra[WM], rb[G];
  auto load_slab = [&](int kb) {
    const int seg = kb >= slabs_per_seg;
    const int koff = (kb - (seg ? slabs_per_seg : 0)) * kBK;
#pragma unroll
    for (int i = 0; i < WM; ++i)
      ra[i] = *reinterpret_cast<const floatx4*>((seg ? aptr1[i] : aptr0[i]) + koff);
#pragma unroll
    for (int g = 0; g < G; ++g) rb[g] = *reinterpret_cast<const floatx4*>(bptr[g] + kb * kBK);
  };
  auto store_slab = [&]() {
#pragma unroll
    for (int i = 0; i < WM; ++i)
      *reinterpret_cast<floatx4*>(&As[(lrow + 32 * i) * kLdT + lpart]) = ra[i];
#pragma unroll
    for (int g = 0; g < G; ++g)
      *reinterpret_cast<floatx4*>(&Bs[(lrow + 32 * g) * kLdT + lpart]) = rb[g];
  };

  if (n_slabs > 0) {
    load_slab(0);
    store_slab();
    __syncthreads();
    const int frag = (lane & 31) * kLdT + (lane >> 5) * 4;
    for (int kb = 0; kb < n_slabs; ++kb) {
      if (kb + 1 < n_slabs) load_slab(kb + 1);
#pragma unroll
      for (int q = 0; q < 4 / WK; ++q) {
        const int kk = wk * (4 / WK) + q;  // 8-k group of the slab handled by this wavefront
        const floatx4 av = *reinterpret_cast<const floatx4*>(&As[wm * 32 * kLdT + frag + kk * 8]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const floatx4 bv = *reinterpret_cast<const floatx4*>(&Bs[g * 32 * kLdT + frag + kk * 8]);
#pragma unroll
          for (int s = 0; s < 4; ++s)
            acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s], bv[s], acc[g], 0, 0, 0);
        }
      }
      __syncthreads();  // everyone is done reading this slab
      if (kb + 1 < n_slabs) {
        store_slab();
        __syncthreads();
      }
    }
  }

  // ---- sum the k-split partial tiles into the wk == 0 wavefront of each node block
  if constexpr (WK > 1) {
    float* red = smem + wm * (G * 16 * 64);
    for (int r = 1; r < WK; ++r) {
      __syncthreads();
      if (wk == r) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int v = 0; v < 16; ++v) red[(g * 16 + v) * 64 + lane] = acc[g][v];
      }
      __syncthreads();
      if (wk == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[g][v] += red[(g * 16 + v) * 64 + lane];
      }
    }
    if (wk != 0) return;
  }

  // ---- fused epilogue: bias, gates, state update, scatter to the arena
  const int j = j0 + (lane & 31);
  float bz[G];
#pragma unroll
  for (int g = 0; g < G; ++g) bz[g] = a.bias ? a.bias[gate_row<EPI>(g) * H + j] : 0.0f;

#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int node = m0 + wm * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
    if (node >= n) continue;
    const size_t orow = a.out_rows ? (size_t)a.out_rows[node] : (size_t)node;
    float z[G];
#pragma unroll
    for (int g = 0; g < G; ++g) z[g] = acc[g][v] + bz[g];

    if constexpr (EPI == EPI_STORE_Z) {
#pragma unroll
      for (int g = 0; g < G; ++g) a.zout[orow * (size_t)(G * H) + g * H + j] = z[g];
    } else if constexpr (EPI == EPI_TREE_LEAF) {
      const float c = fast_sigmoid(z[0]) * fast_tanh(z[2]);
      a.c[orow * H + j] = c;
      a.h[orow * H + j] = fast_sigmoid(z[1]) * fast_tanh(c);
    } else if constexpr (EPI == EPI_TREE_INTERNAL) {
      const float cl = a.cprev_src[(size_t)a.idx0[node] * H + j];
      const float cr = a.cprev_src[(size_t)a.idx1[node] * H + j];
      const float c = fast_sigmoid(z[0]) * fast_tanh(z[4]) + fast_sigmoid(z[1]) * cl +
                      fast_sigmoid(z[2]) * cr;
      a.c[orow * H + j] = c;
      a.h[orow * H + j] = fast_sigmoid(z[3]) * fast_tanh(c);
    } else {  // EPI_LSTM_STEP
#pragma unroll
      for (int g = 0; g < G; ++g) z[g] += a.zadd[orow * (size_t)(G * H) + g * H + j];
      const float cp = a.cprev_src ? a.cprev_src[(size_t)a.idx0[node] * H + j] : 0.0f;
      const float c = fast_sigmoid(z[1]) * cp + fast_sigmoid(z[0]) * fast_tanh(z[3]);
      a.c[orow * H + j] = c;
      a.h[orow * H + j] = fast_sigmoid(z[2]) * fast_tanh(c);
    }
  }
}

template <int G, int EPI>
hipError_t launch_shape(const CellLevelArgs& a, hipStream_t stream) {
  const int n_jt = a.H / 32;
  // largest node tile that still gives the 256 compute units at least one workgroup each
  auto wgs = [&](int bm) { return (long)((a.n + bm - 1) / bm) * n_jt; };
  if (wgs(128) >= 256) {
    hipLaunchKernelGGL((cell_level_kernel<G, EPI, 4, 1>), dim3((unsigned)wgs(128)), dim3(kThreads), 0,
                       stream, a);
  } else if (wgs(64) >= 256) {
    hipLaunchKernelGGL((cell_level_kernel<G, EPI, 2, 2>), dim3((unsigned)wgs(64)), dim3(kThreads), 0,
                       stream, a);
  } else {
    hipLaunchKernelGGL((cell_level_kernel<G, EPI, 1, 4>), dim3((unsigned)wgs(32)), dim3(kThreads), 0,
                       stream, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_cell_level(CellEpilogue epi, const CellLevelArgs& a, hipStream_t stream) {
  if (a.n <= 0) return hipSuccess;
  switch (epi) {
    case EPI_TREE_LEAF: return launch_shape<3, EPI_TREE_LEAF>(a, stream);
    case EPI_TREE_INTERNAL: return launch_shape<5, EPI_TREE_INTERNAL>(a, stream);
    case EPI_LSTM_STEP: return launch_shape<4, EPI_LSTM_STEP>(a, stream);
    case EPI_STORE_Z: return launch_shape<4, EPI_STORE_Z>(a, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace acrobat
