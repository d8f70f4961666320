// Gather-fused cell kernels for gfx950 (TreeLSTM leaf / internal level, LSTM and RNN input
// transform and step, RNN output layer).
//
// One launch executes one depth level of the schedule (section 4.1).  The kernel reads the
// level's operand rows straight from the arena through index lists instead of from a
// gathered contiguous copy (gather fusion, section 5.2), contracts them with the shared
// weight matrix once for all gates (parameter reuse, section 5.1; horizontal fusion,
// appendix "Exploiting Data Reuse") on the fp32 matrix cores and applies the gate non-linearities and the state
// update before anything is written back (vertical fusion, Evaluation, "Benefits of Optimizations").
//
// Tiling.  A workgroup of four wavefronts owns BM = 32*WM nodes and 32 hidden units j, and
// for those it computes ALL G gates: the weight tile is made of G row blocks of the weight
// matrix (rows g*H + j0 .. +31), so no packing of the weights is needed and the epilogue
// finds every gate of a (node, j) pair in the same lane and register slot.  The k loop
// streams 32-column slabs of both operands through LDS with a register prefetch of the
// next slab.  Wavefronts are arranged WM (node blocks) x WK (k split inside a slab); small
// levels use WK > 1 so that all four matrix pipes of the CU work on a 32-node tile.
//
// Latency-bound levels (few nodes) go to cell_tiny_kernel further down.  Mid-size levels
// cannot fill 256 compute units with (node tile, j tile) pairs alone, so the
// k range is additionally split over `ksplit` workgroups.  Each writes its partial tile to
// a workspace; a second, small kernel launched behind it sums the partial tiles in fixed
// order and runs the epilogue.
//
// Matrix instruction: v_mfma_f32_32x32x2_f32.  Lane l supplies A[i = l%32][k = l/32] and
// B[k = l/32][j = l%32]; the 16 result registers of lane l hold column j = l%32 and rows
// i = 8*(v/4) + 4*(l/32) + v%4.  Rows are nodes, columns are hidden units, so stores are
// 128-byte contiguous per half wavefront.  Each lane fetches four consecutive k of its row
// with one 16-byte LDS read and feeds them to four instructions; lanes 32..63 take the
// upper four k of an 8-k group, which is just a permutation of the summation order applied
// to both operands alike.
//
// Workgroup order: the j tile is the fastest index of the linear workgroup id.  Workgroups
// go round-robin to the 8 XCDs, so with 8 or 16 j tiles every XCD only ever touches the
// weight rows of one or two j tiles and keeps them in its own L2 for the whole level.
#include "cell_kernels.h"

#include "agent_access.h"

#include <algorithm>
#include <atomic>
#include <type_traits>

namespace acrobat {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;        // k columns per slab
constexpr int kThreads = 256;
constexpr int kBlockFloats = 16 * 64;  // one 32x32 accumulator block of one wavefront

// The kernels for small levels number their workgroups (node tile, unit tile) with the unit tile fastest and pad
// the number of unit tiles to a multiple of 8: workgroup ids go round-robin to the 8 XCDs, so every node tile of a
// unit tile then runs on the same XCD and finds that tile's weight rows in its L2.  With fewer than 8 unit tiles
// the padding would leave XCDs empty, so there is none.
__host__ __device__ constexpr int padded_unit_tiles(int n_jt) { return n_jt >= 8 ? (n_jt + 7) & ~7 : n_jt; }

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

// Fused epilogue of one lane: bias, gates, state update, scatter to the arena, for NV
// accumulator rows (node_of(v)) of hidden unit j; acc(g, v) is the pre-activation of gate g.
// Two stages.  epilogue_fetch reads the indices and then every gathered operand (all loads of a
// pass in flight together instead of one dependent chain per row); it depends on nothing the
// contraction computes, so a kernel may run it ahead of its k loop.  epilogue_apply does the
// arithmetic and the stores (the stores may alias the loads as far as the compiler can tell,
// which would otherwise serialise the rows).
//
// `sidx` (may be null) is the tile's index table in LDS, [3][bm]: arena row written, first and
// second operand row of tile row r = node - m0, as staged by the contraction kernel's prologue
// (tail rows hold the entries of node n - 1); without it the indices come from global memory.
template <int G, int EPI, int NV>
struct EpilogueOperands {
  float bz[G];
  size_t orow[NV];
  bool live[NV];
  float p0[NV], p1[NV];                        // gathered state: c of the two children / previous c / hoisted z (RNN)
  float zx[EPI == EPI_LSTM_STEP ? G : 1][NV];  // hoisted input transform of an LSTM step
};

template <int G, int EPI, int NV, class NodeOf>
__device__ __forceinline__ void epilogue_fetch(const CellLevelArgs& a, const int j, NodeOf&& node_of,
                                               EpilogueOperands<G, EPI, NV>& o, const int* sidx = nullptr, const int bm = 0,
                                               const int m0 = 0) {
  const int H = a.H, n = a.n;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    if constexpr (EPI == EPI_RELU_OUT) o.bz[g] = a.bias && j < a.n_cols ? a.bias[j] : 0.0f;
    else o.bz[g] = a.bias ? a.bias[gate_row<EPI>(g) * H + j] : 0.0f;
  }
  int ia[NV], ib[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int node = node_of(v);
    o.live[v] = node < n;
    const int nd = o.live[v] ? node : n - 1;  // tail rows read what the last node reads, store nothing
    ia[v] = ib[v] = 0;
    if (sidx) {
      const int r = node - m0;
      o.orow[v] = (size_t)sidx[r];
      if constexpr (EPI == EPI_TREE_INTERNAL || EPI == EPI_LSTM_STEP) ia[v] = sidx[bm + r];
      if constexpr (EPI == EPI_TREE_INTERNAL) ib[v] = sidx[2 * bm + r];
    } else {
      o.orow[v] = a.out_rows ? (size_t)a.out_rows[nd] : (size_t)nd;
      if constexpr (EPI == EPI_TREE_INTERNAL) {
        ia[v] = a.idx0[nd];
        ib[v] = a.idx1[nd];
      }
      if constexpr (EPI == EPI_LSTM_STEP) {
        if (a.cprev_src) ia[v] = a.idx0[nd];
      }
    }
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    o.p0[v] = o.p1[v] = 0.0f;
    if constexpr (EPI == EPI_TREE_INTERNAL) {
      o.p0[v] = a.cprev_src[(size_t)ia[v] * H + j];
      o.p1[v] = a.cprev_src[(size_t)ib[v] * H + j];
    } else if constexpr (EPI == EPI_RNN_STEP) {
      o.p0[v] = a.zadd ? a.zadd[o.orow[v] * (size_t)H + j] : 0.0f;
    } else if constexpr (EPI == EPI_LSTM_STEP) {
      o.p0[v] = a.cprev_src ? a.cprev_src[(size_t)ia[v] * H + j] : 0.0f;
#pragma unroll
      for (int g = 0; g < G; ++g) o.zx[g][v] = a.zadd[o.orow[v] * (size_t)(G * H) + g * H + j];
    }
  }
}

template <int G, int EPI, int NV, class Acc>
__device__ __forceinline__ void epilogue_apply(const CellLevelArgs& a, const int j, Acc&& acc,
                                               const EpilogueOperands<G, EPI, NV>& o) {
  const int H = a.H;
  const float* bz = o.bz;
  if constexpr (EPI == EPI_STORE_Z) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      if (!o.live[v]) continue;
#pragma unroll
      for (int g = 0; g < G; ++g) a.zout[o.orow[v] * (size_t)(G * H) + g * H + j] = acc(g, v) + bz[g];
    }
  } else if constexpr (EPI == EPI_TREE_LEAF) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      if (!o.live[v]) continue;
      const float c = fast_sigmoid(acc(0, v) + bz[0]) * fast_tanh(acc(2, v) + bz[2]);
      a.c[o.orow[v] * H + j] = c;
      a.h[o.orow[v] * H + j] = fast_sigmoid(acc(1, v) + bz[1]) * fast_tanh(c);
    }
  } else if constexpr (EPI == EPI_TREE_INTERNAL) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      if (!o.live[v]) continue;
      const float c = fast_sigmoid(acc(0, v) + bz[0]) * fast_tanh(acc(4, v) + bz[4]) +
                      fast_sigmoid(acc(1, v) + bz[1]) * o.p0[v] + fast_sigmoid(acc(2, v) + bz[2]) * o.p1[v];
      a.c[o.orow[v] * H + j] = c;
      a.h[o.orow[v] * H + j] = fast_sigmoid(acc(3, v) + bz[3]) * fast_tanh(c);
    }
  } else if constexpr (EPI == EPI_RNN_STEP) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      if (!o.live[v]) continue;
      a.h[o.orow[v] * H + j] = fast_sigmoid(acc(0, v) + o.p0[v] + bz[0]);
    }
  } else if constexpr (EPI == EPI_RELU_OUT) {
    if (j < a.n_cols) {
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        if (!o.live[v]) continue;
        a.y[o.orow[v] * (size_t)a.ldo + j] = fmaxf(acc(0, v) + bz[0], 0.0f);
      }
    }
  } else {  // EPI_LSTM_STEP
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      if (!o.live[v]) continue;
      const float c = fast_sigmoid(acc(1, v) + o.zx[1][v] + bz[1]) * o.p0[v] +
                      fast_sigmoid(acc(0, v) + o.zx[0][v] + bz[0]) * fast_tanh(acc(3, v) + o.zx[3][v] + bz[3]);
      a.c[o.orow[v] * H + j] = c;
      a.h[o.orow[v] * H + j] = fast_sigmoid(acc(2, v) + o.zx[2][v] + bz[2]) * fast_tanh(c);
    }
  }
}

template <int G, int EPI, int NV, class Acc, class NodeOf>
__device__ __forceinline__ void cell_epilogue(const CellLevelArgs& a, const int j, Acc&& acc, NodeOf&& node_of,
                                              const int* sidx = nullptr, const int bm = 0, const int m0 = 0) {
  EpilogueOperands<G, EPI, NV> o;
  epilogue_fetch<G, EPI, NV>(a, j, node_of, o, sidx, bm, m0);
  epilogue_apply<G, EPI, NV>(a, j, acc, o);
}

// LDS of one workgroup of the tiled kernels: slab buffers (reused by the reduction over the k-split
// wavefronts) and the tile's index table [3][BM] behind them.
template <int G, int WM, int WK>
struct TileLds {
  static constexpr int BM = 32 * WM;
  static constexpr int Q = 4 / WK;  // 8-k groups of a slab handled by one wavefront
  static constexpr int TILE_FLOATS = (BM + 32 * G) * kBK;
  static constexpr int RED_FLOATS = WM * (WK - 1) * G * kBlockFloats;
  static constexpr int NBUF = Q == 1 ? 3 : 2;  // slab buffers (see the pipeline in contract_tile)
  static constexpr int SMEM_FLOATS = NBUF * TILE_FLOATS > RED_FLOATS ? NBUF * TILE_FLOATS : RED_FLOATS;
  static constexpr int TOTAL_FLOATS = SMEM_FLOATS + 3 * BM;
  static constexpr int NV = 4 * (4 / WK);  // accumulator rows a lane owns after the reduction over wk
};

// Contraction of one tile (BM nodes from m0, hidden units j0 .. j0 + 31, all G gates) over the slabs
// [slab0, slab0 + my_slabs) of the k range.  On return own[g][v] holds this wavefront's share of the
// result (accumulator row acc_row(v), see tile_acc_row) and sidx the tile's index table.
// `early()` runs once the index table is complete and the first slabs are on their way: the place to request
// whatever the epilogue gathers (epilogue_fetch), so that it has arrived when the contraction is through.
template <int G, int EPI, int WM, int WK, class Early>
__device__ __forceinline__ void contract_tile(const CellLevelArgs& a, const int m0, const int j0, const int slab0,
                                              const int my_slabs, float* const smem, int* const sidx,
                                              float (&own)[G][TileLds<G, WM, WK>::NV], Early&& early) {
  static_assert(WM * WK == 4, "four wavefronts per workgroup");
  using L = TileLds<G, WM, WK>;
  constexpr int BM = L::BM;
  constexpr int Q = L::Q;
  constexpr int TILE_FLOATS = L::TILE_FLOATS;
  constexpr int NBUF = L::NBUF;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wk = wave / WM;
  const int H = a.H, n = a.n;

  // ---- global -> LDS staging assignment: 16-byte chunk `tid & 7` of tile row `tid >> 3` (+32 i)
  const int lrow = tid >> 3, lpart = (tid & 7) * 4;
  // The tile's indices are read once: for the operand row pointers below and, through LDS, for
  // the epilogue (which then starts with an LDS read instead of a dependent global load).
  int row0[WM], row1[WM];
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    int node = m0 + lrow + 32 * i;
    node = node < n ? node : n - 1;  // tail rows re-read the last node; never stored
    row0[i] = a.idx0 ? a.idx0[node] : node;
    row1[i] = a.idx1 ? a.idx1[node] : node;
    if ((tid & 7) == 2) sidx[lrow + 32 * i] = a.out_rows ? a.out_rows[node] : node;
  }
  // weights: one per-lane offset; gate and slab offsets are uniform (fit 32 bits: host-checked)
  // (RELU_OUT: rows past the last weight row re-read it; their columns are never stored)
  const int wrow = EPI == EPI_RELU_OUT ? (j0 + lrow < a.n_cols ? j0 + lrow : a.n_cols - 1) : j0 + lrow;
  const unsigned boff = (unsigned)wrow * (unsigned)a.ldw + (unsigned)lpart;
  const unsigned gate_stride = (unsigned)H * (unsigned)a.ldw;

  floatx16 acc[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[g][v] = 0.0f;

  const int slabs_per_seg = a.kseg / kBK;

  // Software pipeline, written so that one wavefront per SIMD can keep the matrix pipe busy
  // and two workgroups fit a compute unit (<= 80 KB LDS, <= 256 registers):
  //  * global -> registers: NS staging sets hold slabs in flight;
  //  * registers -> LDS: slab buffers of 32 floats per row without padding; the 16-byte chunk
  //    c of row r sits at chunk position c ^ ((r >> 1) & 7), which makes both the row-wise
  //    stores and the column-wise 16-byte operand reads free of bank conflicts;
  //  * LDS -> operand registers: two fragment sets, the fragments of the next 8-k group are
  //    read while the matrix instructions of the current group issue.
  // Q == 1 (each wavefront has one group per slab): three buffers - read / complete / being
  // filled - and one barrier at the end of a slab.  Q >= 2: two buffers; slab kb+1 is written
  // during the first group of slab kb, the barrier sits before the LAST group of slab kb, and
  // that group's shadow hides the first operand read of slab kb+1.
  // Inside a group none of the memory instructions depends on the matrix instructions, and
  // the scheduling hints interleave them one to one.  Slab indices past the end are clamped:
  // the last slab is fetched again into a buffer nothing reads, so the loop has no branches.
  constexpr int NS = WM == 1 ? 4 : 2;
  constexpr int AHEAD = Q == 1 ? 2 : 1;  // a slab is stored to LDS AHEAD iterations before its use
  floatx4 ra[NS][WM], rb[NS][G];
  floatx4 fa[2], fb[2][G];
  const float* aptr0[WM];
  const float* aptr1[WM];
  auto load_slab_b = [&](int set, int i) {
    const int kb = slab0 + (i < my_slabs ? i : my_slabs - 1);
#pragma unroll
    for (int g = 0; g < G; ++g)
      rb[set][g] = *reinterpret_cast<const floatx4*>(a.W + (gate_row<EPI>(g) * gate_stride + kb * kBK) + boff);
  };
  auto load_slab_a = [&](int set, int i) {
    const int kb = slab0 + (i < my_slabs ? i : my_slabs - 1);
    const int seg = kb >= slabs_per_seg;
    const int koff = (kb - (seg ? slabs_per_seg : 0)) * kBK;
#pragma unroll
    for (int r = 0; r < WM; ++r)
      ra[set][r] = *reinterpret_cast<const floatx4*>((seg ? aptr1[r] : aptr0[r]) + koff);
  };
  auto load_slab = [&](int set, int i) {
    load_slab_a(set, i);
    load_slab_b(set, i);
  };
  const int st_off = lrow * kBK + (((tid & 7) ^ ((lrow >> 1) & 7)) << 2);
  auto store_slab = [&](int set, int buf) {
    float* As = smem + buf * TILE_FLOATS;
    float* Bs = As + BM * kBK;
#pragma unroll
    for (int r = 0; r < WM; ++r) *reinterpret_cast<floatx4*>(&As[32 * r * kBK + st_off]) = ra[set][r];
#pragma unroll
    for (int g = 0; g < G; ++g) *reinterpret_cast<floatx4*>(&Bs[32 * g * kBK + st_off]) = rb[set][g];
  };
  int fr_off[Q];  // operand fragment of group q: row lane%32, chunk 2*(wk*Q + q) + lane/32
#pragma unroll
  for (int q = 0; q < Q; ++q)
    fr_off[q] = (lane & 31) * kBK + (((2 * (wk * Q + q) + (lane >> 5)) ^ (((lane & 31) >> 1) & 7)) << 2);
  auto read_frag = [&](int fset, int buf, int q) {
    const float* As = smem + buf * TILE_FLOATS;
    const float* Bs = As + BM * kBK;
    fa[fset] = *reinterpret_cast<const floatx4*>(&As[wm * 32 * kBK + fr_off[q]]);
#pragma unroll
    for (int g = 0; g < G; ++g) fb[fset][g] = *reinterpret_cast<const floatx4*>(&Bs[g * 32 * kBK + fr_off[q]]);
  };
  auto mfma_group = [&](int fset) {
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int g = 0; g < G; ++g)  // G independent accumulators between dependent issues
        acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[fset][s], fb[fset][g][s], acc[g], 0, 0, 0);
  };
  // one slab; `set` = (kb + AHEAD) % NS is the staging set that holds slab kb + AHEAD,
  // `par` = kb & 1 the fragment set when Q == 1, `bc` = kb % NBUF the buffer of slab kb
  auto iteration = [&](int kb, int set, int par, int bc) {
    const int b_next = bc + 1 == NBUF ? 0 : bc + 1;
    const int b_fill = Q == 1 ? (bc == 0 ? 2 : bc - 1) : b_next;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const int fcur = Q == 1 ? par : (q & 1);
      if (Q > 1 && q == Q - 1) __syncthreads();  // slab kb + 1 is complete in b_next
      if (q + 1 < Q) read_frag(fcur ^ 1, bc, q + 1);
      else read_frag(fcur ^ 1, b_next, 0);
      if (q == 0) {
        store_slab(set, b_fill);  // slab kb + AHEAD
        load_slab(set, kb + AHEAD + NS);
      }
      mfma_group(fcur);
      // interleave: one memory instruction after each matrix instruction
      constexpr int n_mfma = 4 * G, n_rd = 1 + G, n_st = WM + G;
      // the stores and the loads of a slab each get at most half of the slots left by the reads
      constexpr int half = (n_mfma - n_rd) / 2;
      constexpr int w = (n_st + half - 1) / half;
#pragma unroll
      for (int i = 0; i < n_rd; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
      }
      if (q == 0) {
#pragma unroll
        for (int i = 0; i < (n_st + w - 1) / w; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x200, w, 0);  // DS write
        }
#pragma unroll
        for (int i = 0; i < (n_st + w - 1) / w; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, w, 0);  // VMEM read
        }
      }
      constexpr int rest0 = n_mfma - n_rd - 2 * ((n_st + w - 1) / w), rest = n_mfma - n_rd;
      static_assert(rest0 >= 0, "more memory slots than matrix instructions");
      if (q == 0) {
        if (rest0 > 0) __builtin_amdgcn_sched_group_barrier(0x008, rest0, 0);  // the remaining MFMAs
      } else {
        __builtin_amdgcn_sched_group_barrier(0x008, rest, 0);
      }
    }
    if (Q == 1) __syncthreads();
  };

  // The weight slabs do not depend on the indices: they are requested first, the gathered rows as
  // soon as the indices have arrived.
  if (my_slabs > 0) {
#pragma unroll
    for (int i = 0; i < NS; ++i) load_slab_b(i, i);
  }
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    aptr0[i] = a.nseg > 0 ? a.src0 + (size_t)row0[i] * (size_t)a.ld0 + lpart : nullptr;
    aptr1[i] = a.nseg > 1 ? a.src1 + (size_t)row1[i] * (size_t)a.ld1 + lpart : nullptr;
    if ((tid & 7) == 0) sidx[BM + lrow + 32 * i] = row0[i];
    if ((tid & 7) == 1) sidx[2 * BM + lrow + 32 * i] = row1[i];
  }
  if (my_slabs > 0) {
    // all NS staging sets are requested at once (slab i -> set i); slabs 0 .. AHEAD-1 then go
    // to LDS and their sets are refilled with slabs NS .. NS+AHEAD-1
#pragma unroll
    for (int i = 0; i < NS; ++i) load_slab_a(i, i);
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) {
      store_slab(i, i);
      load_slab(i, NS + i);
    }
    __syncthreads();
    read_frag(0, 0, 0);
    early();
    int kb = 0, bc = 0;
    for (; kb + NS <= my_slabs; kb += NS) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        iteration(kb + i, (i + AHEAD) % NS, i & 1, bc);
        bc = bc + 1 == NBUF ? 0 : bc + 1;
      }
    }
#pragma unroll
    for (int i = 0; i < NS - 1; ++i) {
      if (kb + i < my_slabs) {
        iteration(kb + i, (i + AHEAD) % NS, i & 1, bc);
        bc = bc + 1 == NBUF ? 0 : bc + 1;
      }
    }
    if (Q > 1) __syncthreads();  // the last group's barrier pairs: LDS is reused by the reductions
  } else {
    __syncthreads();  // no contraction (first step of a recurrence): publish the index table
    early();
  }

  // The WK wavefronts of a node block hold partial sums over their share of k.  They are added
  // by a reduce-scatter through LDS: wavefront wk ends up with the complete sums of the QPW = 4/WK
  // accumulator quads v4 = wk*QPW .. wk*QPW + QPW-1 (8 nodes each) and every wavefront runs the
  // epilogue for the rows it owns, so the gate arithmetic is spread over all four SIMDs.  Each
  // quad is summed in ascending wk order, whoever owns it.
  constexpr int QPW = 4 / WK;  // quads owned per wavefront
  if constexpr (WK == 1) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int v = 0; v < 16; ++v) own[g][v] = acc[g][v];
  } else {
    // inbox of wavefront (wm, o): (WK-1) senders x G gates x QPW quads, one float4 per lane each
    floatx4* red = reinterpret_cast<floatx4*>(smem);
    auto inbox = [&](int o, int sender, int g, int qi) {
      const int slot = sender < o ? sender : sender - 1;
      return ((((wm * WK + o) * (WK - 1) + slot) * G + g) * QPW + qi) * 64 + lane;
    };
    __syncthreads();
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
      const int o = v4 / QPW, qi = v4 % QPW;
      if (o != wk) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          floatx4 q;
#pragma unroll
          for (int e = 0; e < 4; ++e) q[e] = acc[g][v4 * 4 + e];
          red[inbox(o, wk, g, qi)] = q;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int qi = 0; qi < QPW; ++qi) {
        floatx4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int src = 0; src < WK; ++src) {  // ascending wk, own contribution in its place
          floatx4 q;
          if (src == wk) {
#pragma unroll
            for (int o = 0; o < WK; ++o)
              if (o == wk) {
#pragma unroll
                for (int e = 0; e < 4; ++e) q[e] = acc[g][(o * QPW + qi) * 4 + e];
              }
          } else {
            q = red[inbox(wk, src, g, qi)];
          }
          sum += q;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) own[g][qi * 4 + e] = sum[e];
      }
  }
}

// accumulator row of a lane's owned row v: quad wk * QPW + v / 4, element v % 4
template <int WK>
__device__ __forceinline__ int tile_acc_row(int wk, int v) { return (wk * (4 / WK) + (v >> 2)) * 4 + (v & 3); }

// fused epilogue of a contracted tile (accumulator row r of a lane: node = m0 + 32 wm + 8 (r / 4) + 4 (lane / 32) + r % 4),
// in its two stages
template <int G, int EPI, int WM, int WK>
using TileEpilogueOperands = EpilogueOperands<G, EPI, TileLds<G, WM, WK>::NV>;

template <int G, int EPI, int WM, int WK>
__device__ __forceinline__ void tile_epilogue_fetch(const CellLevelArgs& a, const int m0, const int j0, const int* sidx,
                                                    TileEpilogueOperands<G, EPI, WM, WK>& eo) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave % WM, wk = wave / WM;
  epilogue_fetch<G, EPI, TileLds<G, WM, WK>::NV>(
      a, j0 + (lane & 31),
      [&](int v) {
        const int r = tile_acc_row<WK>(wk, v);
        return m0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
      },
      eo, sidx, 32 * WM, m0);
}
template <int G, int EPI, int WM, int WK>
__device__ __forceinline__ void tile_epilogue_apply(const CellLevelArgs& a, const int j0,
                                                    const float (&own)[G][TileLds<G, WM, WK>::NV],
                                                    const TileEpilogueOperands<G, EPI, WM, WK>& eo) {
  epilogue_apply<G, EPI, TileLds<G, WM, WK>::NV>(
      a, j0 + (int)(threadIdx.x & 31), [&](int g, int v) { return own[g][v]; }, eo);
}

template <int G, int EPI, int WM, int WK>
__global__ __launch_bounds__(kThreads, 2) void cell_level_kernel(const CellLevelPair pr, const int ksplit,
                                                                 float* __restrict__ partial) {
  const bool second = blockIdx.x >= (unsigned)pr.split;  // which of the two batches (uniform)
  const CellLevelArgs& a = pr.a[second];
  const int bid = (int)blockIdx.x - (second ? pr.split : 0);
  using L = TileLds<G, WM, WK>;
  __shared__ __attribute__((aligned(16))) float smem[L::TOTAL_FLOATS];
  int* const sidx = reinterpret_cast<int*>(smem + L::SMEM_FLOATS);  // the tile's index table, see cell_epilogue

  const int n_jt = a.H >> 5;
  int jt, mt, ks = 0;
  if (ksplit == 0) {
    // Unsplit level, XCD-aware order (workgroup id % 8 is the XCD): XCD x runs the unit tiles x % 4 + 4 i of the
    // node tiles 2 i' + x / 4, so it keeps a quarter of the weight rows in its L2 and streams half of the node
    // rows, instead of an eighth of the weights and every node row.
    const int x = bid & 7, q = bid >> 3, jq = n_jt >> 2;
    jt = (x & 3) + 4 * (q % jq);
    mt = 2 * (q / jq) + (x >> 2);
    if (mt * L::BM >= a.n) return;  // padding of an odd number of node tiles
  } else {
    jt = bid % n_jt;
    const int rest = bid / n_jt;
    ks = rest % ksplit;
    mt = rest / ksplit;
  }
  const int j0 = jt * 32, m0 = mt * L::BM;
  const int my_slabs = (a.nseg * (a.kseg / kBK)) / (ksplit ? ksplit : 1);  // host guarantees divisibility
  float own[G][L::NV];
  TileEpilogueOperands<G, EPI, WM, WK> eo;
  // (the 32-node tile has no registers to spare during its k loop: it fetches behind the loop)
  constexpr bool kEarly = WM == 2;
  contract_tile<G, EPI, WM, WK>(a, m0, j0, ks * my_slabs, my_slabs, smem, sidx, own, [&] {
    if (kEarly && ksplit <= 1) tile_epilogue_fetch<G, EPI, WM, WK>(a, m0, j0, sidx, eo);
  });

  // ---- k split over workgroups: store the partial tile in register layout and stop; the
  // reduction kernel that follows on the stream adds the partial tiles and runs the epilogue
  if (ksplit > 1) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WM, wk = wave / WM;
    const int tile = mt * n_jt + jt;
    float* mine = partial + ((size_t)(tile * ksplit + ks) * WM + wm) * (G * kBlockFloats);
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int v = 0; v < L::NV; ++v) mine[(g * 16 + tile_acc_row<WK>(wk, v)) * 64 + lane] = own[g][v];
    return;
  }
  if (!kEarly) tile_epilogue_fetch<G, EPI, WM, WK>(a, m0, j0, sidx, eo);
  tile_epilogue_apply<G, EPI, WM, WK>(a, j0, own, eo);
}

// ---- even split of a level over the chip ("stream-k") ---------------------------------------------------
// A level of T tiles is T * n_slabs units of work (one unit = one 32-k slab of one tile) in the order
// (tile, slab).  With fewer tiles than the chip has room for, whole tiles leave compute units idle for a
// good part of the level (208 tiles on 256 units: the level takes as long as 256 tiles would).  Here the
// unit range is cut into P equal contiguous shares, one per workgroup, so a share is the tail of one tile,
// some whole tiles and the head of another.  A workgroup finishes the whole tiles itself.  For a piece of a
// tile it stores its partial sums to the workspace (write-through), completes those stores and counts
// itself in at the tile's counter; whoever counts in last adds the pieces - all of them read back from the
// workspace, in ascending order of k, so the sum does not depend on who came last - and runs the epilogue.
// Nobody waits for anybody, so nothing here can hang and no workgroup needs another to be resident.  No
// fence is involved (a release / acquire pair at agent scope costs several microseconds on this part, see
// persistent_kernels.hip): the pieces are stored with agent-scope atomic stores and read with agent-scope
// atomic loads.  A workgroup's share touches at most two tiles partially (its first and its last), hence
// two workspace slots per workgroup.  The last arriver resets the counter for the next launch.
struct StreamKArgs {
  CellLevelArgs a;
  int32_t n_wg;        // P, at most the number of units
  float* partial;      // [P][2][WM][G][4 quads][64 lanes][4 rows]
  uint32_t partial_bytes;
  unsigned* counters;  // [tiles], zero at launch and again at exit
};

template <int G, int EPI, int WM, int WK>
__global__ __launch_bounds__(kThreads, 1) void cell_streamk_kernel(const StreamKArgs sk) {
  const CellLevelArgs& a = sk.a;
  using L = TileLds<G, WM, WK>;
  __shared__ __attribute__((aligned(16))) float smem[L::TOTAL_FLOATS];
  __shared__ int s_last;
  int* const sidx = reinterpret_cast<int*>(smem + L::SMEM_FLOATS);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave % WM, wk = wave / WM;
  const int n_jt = a.H >> 5;
  // all of this fits 32 bits: the host admits at most 8192 tiles and 512 workgroups, and a k range of 2^16 slabs
  // would be a contraction over two million columns
  const int n_slabs = a.nseg * (a.kseg / kBK);
  const int n_mt = (a.n + L::BM - 1) / L::BM;
  const int tiles = n_mt * n_jt;
  const unsigned U = (unsigned)tiles * (unsigned)n_slabs, P = (unsigned)sk.n_wg;
  auto start_of = [&](unsigned p) { return (unsigned)((unsigned long long)p * U / P); };               // first unit of workgroup p
  auto owner_of = [&](unsigned x) { return (unsigned)(((unsigned long long)(x + 1) * P - 1) / U); };  // whose share holds unit x
  constexpr int QPW = 4 / WK;  // accumulator quads (4 rows each) a wavefront owns per gate
  // byte offset in the workspace of the slot where workgroup p parks its piece of `tile` (this wavefront's node block)
  auto slot_of = [&](unsigned p, int tile) {
    return (unsigned)(((2 * p + ((int)(start_of(p) / n_slabs) == tile ? 0 : 1)) * WM + wm) * (G * kBlockFloats) * sizeof(float));
  };
  auto quad_off = [&](int g, int qi) { return (unsigned)((((g * 4 + wk * QPW + qi) * 64) + lane) * 4 * sizeof(float)); };
  const __amdgpu_buffer_rsrc_t ws_rsrc = agent_buffer(sk.partial, sk.partial_bytes);
  // XCD-aware placement (workgroup id % 8 is the XCD): the shares of one XCD are contiguous, and with the node
  // tile as the fastest index of a tile number an XCD's range of tiles is all node tiles of an eighth of the unit
  // tiles - it keeps that eighth of the weight rows in its L2, and the pieces of a tile are parked and read back
  // within one XCD.  (Any bijection would do for correctness; P is a multiple of 8 whenever it is the number of
  // compute units.)
  const unsigned p = (P & 7) == 0 ? (blockIdx.x & 7) * (P >> 3) + (blockIdx.x >> 3) : blockIdx.x;
  const unsigned u1 = start_of(p + 1);
  bool first = true;
  for (unsigned u = start_of(p); u < u1; first = false) {
    const int tile = (int)(u / n_slabs);
    const int s0 = (int)(u - (unsigned)tile * n_slabs);
    const int cnt = (n_slabs - s0 < (int)(u1 - u)) ? n_slabs - s0 : (int)(u1 - u);
    u += cnt;
    const int mt = tile % n_mt, jt = tile / n_mt;
    const int j0 = jt * 32, m0 = mt * L::BM;
    if (!first) __syncthreads();  // the previous tile's epilogue is through with the index table and the slabs
    float own[G][L::NV];
    TileEpilogueOperands<G, EPI, WM, WK> eo;
    contract_tile<G, EPI, WM, WK>(a, m0, j0, s0, cnt, smem, sidx, own, [&] {
      if (cnt == n_slabs) tile_epilogue_fetch<G, EPI, WM, WK>(a, m0, j0, sidx, eo);  // a whole tile
    });
    if (cnt < n_slabs) {  // a piece: park it, count in, and leave unless last
      // 16 bytes per lane and access: the four rows of accumulator quad (wk * QPW + qi) of gate g
      const unsigned mine = slot_of(p, tile);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int qi = 0; qi < QPW; ++qi) {
          const agent_f4 v = {own[g][4 * qi], own[g][4 * qi + 1], own[g][4 * qi + 2], own[g][4 * qi + 3]};
          store_agent_f4(ws_rsrc, mine + quad_off(g, qi), v);
        }
      wait_stores_done();  // this wavefront's stores have completed
      __syncthreads();     // ... and so have the other wavefronts'
      const unsigned first_wg = owner_of((unsigned)tile * n_slabs), last_wg = owner_of((unsigned)tile * n_slabs + n_slabs - 1);
      if (threadIdx.x == 0) {
        const unsigned arrived = __hip_atomic_fetch_add(sk.counters + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = arrived == last_wg - first_wg;
        if (last) __hip_atomic_store(sk.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = last ? 1 : 0;
      }
      __syncthreads();
      if (!s_last) continue;
      // the pieces in ascending order of k, this workgroup's own from its registers (the same bits it parked)
      tile_epilogue_fetch<G, EPI, WM, WK>(a, m0, j0, sidx, eo);
      float sum[G][L::NV];
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int v = 0; v < L::NV; ++v) sum[g][v] = 0.0f;
      for (unsigned q = first_wg; q <= last_wg; ++q) {
        if (q == p) {
#pragma unroll
          for (int g = 0; g < G; ++g)
#pragma unroll
            for (int v = 0; v < L::NV; ++v) sum[g][v] += own[g][v];
          continue;
        }
        const unsigned theirs = slot_of(q, tile);
        agent_f4 piece[G][QPW];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int qi = 0; qi < QPW; ++qi) piece[g][qi] = load_agent_f4(ws_rsrc, theirs + quad_off(g, qi));
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int qi = 0; qi < QPW; ++qi)
#pragma unroll
            for (int e = 0; e < 4; ++e) sum[g][4 * qi + e] += piece[g][qi][e];
      }
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int v = 0; v < L::NV; ++v) own[g][v] = sum[g][v];
    }
    tile_epilogue_apply<G, EPI, WM, WK>(a, j0, own, eo);
  }
}

// Second half of a level whose k range was split over `ksplit` workgroups: one wavefront per
// (tile, node block, accumulator row v) adds the partial tiles in fixed order and runs the fused
// epilogue.  The kernel boundary between the two launches is the only synchronisation: a
// device-wide fence inside a kernel costs far more on this part (about 15 us with 256
// workgroups) than a launch (about 3 us).
template <int G, int EPI>
__global__ __launch_bounds__(64) void cell_splitk_reduce_kernel(const CellLevelArgs a, const int ksplit, const int wm_count,
                                                                const float* __restrict__ partial) {
  const int lane = threadIdx.x;
  const int v = blockIdx.x & 15;
  const int rest = blockIdx.x >> 4;
  const int wm = rest % wm_count, tile = rest / wm_count;
  const int n_jt = a.H >> 5;
  const int jt = tile % n_jt, mt = tile / n_jt;
  float acc[G];
#pragma unroll
  for (int g = 0; g < G; ++g) acc[g] = 0.0f;
#pragma unroll 4
  for (int s = 0; s < ksplit; ++s) {
    const float* p = partial + ((size_t)(tile * ksplit + s) * wm_count + wm) * (G * kBlockFloats) + v * 64 + lane;
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] += p[g * kBlockFloats];
  }
  const int node = mt * 32 * wm_count + wm * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
  cell_epilogue<G, EPI, 1>(
      a, jt * 32 + (lane & 31), [&](int g, int) { return acc[g]; }, [&](int) { return node; });
}

// Latency-bound levels.  With few nodes a level is a skinny product: the time goes into streaming the
// weight rows and into the chain of dependent steps, not into arithmetic.  This kernel therefore
//  * gives a workgroup 32 nodes x JW hidden units x all G gates, the G*JW <= 32 columns c = g*JW + jj
//    packed into ONE 32-column block (JW = 6 for five gates, else 8; the last tile may be partial):
//    four to five times as many workgroups as 32-unit tiles, each streaming only G*JW weight rows,
//    and no k split across workgroups, hence no second launch;
//  * moves U 32-k slabs per step with one barrier per step (U = 8: 4 steps for K = 1024) and keeps
//    two steps (up to 128 KB) in flight in registers, double buffered in LDS;
//  * splits every slab's k over the four wavefronts as the large kernel does, publishes the four
//    partial tiles in LDS and lets thread t add them (ascending wavefront order) for node t / 8,
//    unit t % 8 and run the epilogue for that one element.
// LDS layout of a slab and the operand fragments are those of cell_level_kernel.
template <int G>
constexpr int tiny_jw() { return G >= 5 ? 6 : 8; }

template <int G, int EPI, int U>
__global__ __launch_bounds__(kThreads) void cell_tiny_kernel(const CellLevelPair pr) {
  const bool second = blockIdx.x >= (unsigned)pr.split;  // which of the two batches (uniform)
  const CellLevelArgs& a = pr.a[second];
  const int bid = (int)blockIdx.x - (second ? pr.split : 0);
  constexpr int JW = tiny_jw<G>();
  static_assert(G * JW <= 32 && JW <= 8, "one column block, one epilogue element per thread");
  constexpr int SLAB = 64 * kBK;  // floats: tile rows 0..31 = nodes, 32..63 = columns
  constexpr int ZLD = 32 + 8;
  static_assert(4 * 32 * ZLD <= 2 * U * SLAB, "the partial tiles reuse the slab buffers");
  extern __shared__ __attribute__((aligned(16))) float tiny_smem[];  // [2 buffers][U][SLAB], index table [3][32]
  float* const smem = tiny_smem;
  int* const sidx = reinterpret_cast<int*>(tiny_smem + 2 * U * SLAB);

  const int tid = threadIdx.x, lane = tid & 63, wk = tid >> 6;
  const int H = a.H, n = a.n;
  const int hlim = EPI == EPI_RELU_OUT ? a.n_cols : H;  // hidden units that exist
  // the launcher pads the number of unit tiles (padded_unit_tiles): every node tile of a unit tile then runs on the
  // same XCD (workgroup id % 8) and finds that tile's weight rows in its L2 instead of fetching them again
  const int n_jt = (hlim + JW - 1) / JW, n_jt_padded = padded_unit_tiles(n_jt);
  const int jt = bid % n_jt_padded, mt = bid / n_jt_padded;
  if (jt >= n_jt) return;
  const int j0 = jt * JW, m0 = mt * 32;

  const int lrow = tid >> 3, lpart = (tid & 7) * 4;
  int node = m0 + lrow;
  node = node < n ? node : n - 1;  // tail rows re-read the last node; never stored
  const int row0 = a.idx0 ? a.idx0[node] : node;
  const int row1 = a.idx1 ? a.idx1[node] : node;
  if ((tid & 7) == 2) sidx[lrow] = a.out_rows ? a.out_rows[node] : node;
  // tile row 32 + lrow is column c = lrow: gate c / JW, unit j0 + c % JW; columns and units past the
  // end repeat the last valid one and are never read back
  unsigned boff;
  {
    const int c = lrow < G * JW ? lrow : G * JW - 1;
    int j = j0 + c % JW;
    j = j < hlim ? j : hlim - 1;
    int grow = 0;
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (c / JW == g) grow = gate_row<EPI>(g);
    boff = ((unsigned)grow * (unsigned)H + (unsigned)j) * (unsigned)a.ldw + (unsigned)lpart;
  }

  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  // the element this thread finishes (node row tid / 8, unit tid % 8 of the tile); its gathered operands are
  // requested as soon as the index table is in LDS, long before the contraction is through
  const int erow = tid >> 3, ejj = tid & 7;
  const bool finisher = ejj < JW && j0 + ejj < hlim;
  EpilogueOperands<G, EPI, 1> eo;
  // (an LSTM step gathers five values per element; requested early they cost the k loop more than they save:
  // 11.2 instead of 10.7 us at 250 rows)
  constexpr bool kEarly = EPI != EPI_LSTM_STEP;

  const int slabs_per_seg = a.kseg / kBK;
  const int S = a.nseg * slabs_per_seg;
  const int steps = (S + U - 1) / U;
  const float* aptr0 = nullptr;
  const float* aptr1 = nullptr;
  floatx4 ra[2][U], rb[2][U];
  auto load_b = [&](int slot, int s) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int kb = s * U + u;
      kb = kb < S ? kb : S - 1;  // past the end: fetched again, never multiplied
      rb[slot][u] = *reinterpret_cast<const floatx4*>(a.W + boff + kb * kBK);
    }
  };
  auto load_a = [&](int slot, int s) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int kb = s * U + u;
      kb = kb < S ? kb : S - 1;
      const int seg = kb >= slabs_per_seg;
      ra[slot][u] = *reinterpret_cast<const floatx4*>((seg ? aptr1 : aptr0) + (kb - (seg ? slabs_per_seg : 0)) * kBK);
    }
  };
  const int st_off = lrow * kBK + (((tid & 7) ^ ((lrow >> 1) & 7)) << 2);
  auto store_step = [&](int slot, int buf) {
    float* base = smem + buf * (U * SLAB);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      *reinterpret_cast<floatx4*>(&base[u * SLAB + st_off]) = ra[slot][u];
      *reinterpret_cast<floatx4*>(&base[u * SLAB + 32 * kBK + st_off]) = rb[slot][u];
    }
  };
  // wavefront wk multiplies the 8-k group wk of every slab
  const int fr_off = (lane & 31) * kBK + (((2 * wk + (lane >> 5)) ^ (((lane & 31) >> 1) & 7)) << 2);
  auto compute_step = [&](int buf, int s) {
    const float* base = smem + buf * (U * SLAB);
    floatx4 fa[U], fb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      fa[u] = *reinterpret_cast<const floatx4*>(&base[u * SLAB + fr_off]);
      fb[u] = *reinterpret_cast<const floatx4*>(&base[u * SLAB + 32 * kBK + fr_off]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (s * U + u < S) {
#pragma unroll
        for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[u][t], fb[u][t], acc, 0, 0, 0);
      }
    }
  };

  if (S > 0) {
    // the weight slabs do not depend on the indices: requested first
    load_b(0, 0);
    if (steps > 1) load_b(1, 1);
    aptr0 = a.src0 + (size_t)row0 * (size_t)a.ld0 + lpart;
    aptr1 = a.nseg > 1 ? a.src1 + (size_t)row1 * (size_t)a.ld1 + lpart : aptr0;
    if ((tid & 7) == 0) sidx[32 + lrow] = row0;
    if ((tid & 7) == 1) sidx[64 + lrow] = row1;
    load_a(0, 0);
    if (steps > 1) load_a(1, 1);
    store_step(0, 0);
    if (steps > 2) {
      load_a(0, 2);
      load_b(0, 2);
    }
    __syncthreads();
    if (kEarly && finisher) epilogue_fetch<G, EPI, 1>(a, j0 + ejj, [&](int) { return m0 + erow; }, eo, sidx, 32, m0);
    // invariant at the top: buffer 0 holds step s, slot 1 step s + 1, slot 0 step s + 2
    for (int s = 0; s < steps; s += 2) {
      if (s + 1 < steps) {
        store_step(1, 1);
        if (s + 3 < steps) {
          load_a(1, s + 3);
          load_b(1, s + 3);
        }
      }
      compute_step(0, s);
      __syncthreads();
      if (s + 1 < steps) {
        if (s + 2 < steps) {
          store_step(0, 0);
          if (s + 4 < steps) {
            load_a(0, s + 4);
            load_b(0, s + 4);
          }
        }
        compute_step(1, s + 1);
        __syncthreads();
      }
    }
  } else {
    if ((tid & 7) == 0) sidx[32 + lrow] = row0;
    if ((tid & 7) == 1) sidx[64 + lrow] = row1;
    __syncthreads();
    if (kEarly && finisher) epilogue_fetch<G, EPI, 1>(a, j0 + ejj, [&](int) { return m0 + erow; }, eo, sidx, 32, m0);
  }

  // partial tiles z[wk][node row][column], then one epilogue element per thread
  float* z = smem;
#pragma unroll
  for (int v = 0; v < 16; ++v)
    z[(wk * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * ZLD + (lane & 31)] = acc[v];
  __syncthreads();
  if (!finisher) return;
  if (!kEarly) epilogue_fetch<G, EPI, 1>(a, j0 + ejj, [&](int) { return m0 + erow; }, eo, sidx, 32, m0);
  float zs[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float sum = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) sum += z[(w * 32 + erow) * ZLD + g * JW + ejj];
    zs[g] = sum;
  }
  epilogue_apply<G, EPI, 1>(a, j0 + ejj, [&](int g, int) { return zs[g]; }, eo);
}

template <int G, int EPI, int U>
hipError_t launch_tiny(const CellLevelPair& pr, unsigned grid, hipStream_t stream, const LaunchEvents& ev) {
  constexpr size_t bytes = (size_t)(2 * U * 64 * kBK + 96) * sizeof(float);
  // More than 64 KB of dynamic LDS has to be asked for once per device.  One bit per device id; two
  // threads that both find the bit clear both set the attribute, which is harmless.
  static std::atomic<uint64_t> configured{0};
  int dev = 0;
  if (const hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (dev >= 64 || !(configured.load(std::memory_order_acquire) & bit)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&cell_tiny_kernel<G, EPI, U>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    if (dev < 64) configured.fetch_or(bit, std::memory_order_release);
  }
  launch_with_events((cell_tiny_kernel<G, EPI, U>), dim3(grid), dim3(kThreads), bytes, stream, ev.start, ev.stop, 
                        pr);
  return hipGetLastError();
}

// ---- small levels straight from global memory to the matrix cores --------------------------------------
// cell_tiny_kernel walks its k range in steps (global -> registers -> LDS -> barrier -> operand registers), and
// a level with few nodes is as long as that chain of dependent steps.  This kernel has no steps: a workgroup
// owns 16 nodes x JW hidden units x all G gates (G * JW <= 16 columns, one 16x16 block of
// v_mfma_f32_16x16x4_f32), wavefront w takes the 16-k groups w, w + 4, ... of the k range, and every lane
// requests ALL of its operand pieces - 16 bytes of its node row and 16 bytes of its weight row per group -
// before the first matrix instruction; lane l supplies A[node l % 16][k] and B[k][column l % 16] for the four
// k = 16 group + 4 (l / 16) + e, one instruction per e (a permutation of the summation order applied to both
// operands).  The only dependent chain left is index -> rows -> matrix instructions -> four-way sum through
// LDS -> gate arithmetic, and the gathered operands of the gate arithmetic are requested right behind the
// rows.  Column c of a workgroup is gate c / JW of unit j0 + c % JW.  The launcher pads the number of unit
// tiles (padded_unit_tiles) so that all node tiles of a unit tile run on the same XCD and find its weight
// rows in that XCD's L2.
template <int G>
constexpr int direct_jw() { return 16 / G; }
constexpr int kDirectGroups = 16;  // 16-k groups of a wavefront in flight at once (K = 1024: all of them)

template <int G, int EPI>
__global__ __launch_bounds__(kThreads, 3) void cell_direct_kernel(const CellLevelPair pr) {
  const bool second = blockIdx.x >= (unsigned)pr.split;  // which of the two batches (uniform)
  const CellLevelArgs& a = pr.a[second];
  const int bid = (int)blockIdx.x - (second ? pr.split : 0);
  constexpr int JW = direct_jw<G>(), NC = G * JW;
  __shared__ float z[4][16][17];
  __shared__ int sidx[3 * 16];  // the tile's index table, see epilogue_fetch

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int li = lane & 15, kq = lane >> 4;
  const int H = a.H, n = a.n;
  const int hlim = EPI == EPI_RELU_OUT ? a.n_cols : H;  // hidden units that exist
  const int n_jt = (hlim + JW - 1) / JW, n_jt_padded = padded_unit_tiles(n_jt);
  const int jt = bid % n_jt_padded, mt = bid / n_jt_padded;
  if (jt >= n_jt) return;  // padding of the grid
  const int j0 = jt * JW, m0 = mt * 16;

  // operand node of this lane, and the element this thread finishes: node m0 + tid / JW, unit j0 + tid % JW
  int node = m0 + li;
  node = node < n ? node : n - 1;  // tail rows re-read the last node; never stored
  const int row0 = a.idx0 ? a.idx0[node] : node;
  const int row1 = a.idx1 ? a.idx1[node] : node;
  const int orow = a.out_rows ? a.out_rows[node] : node;
  const int er = tid / JW, ej = j0 + tid % JW;
  const bool finisher = tid < 16 * JW && ej < hlim;

  // weight row of column li (columns past the last repeat it and are never read back)
  const float* bptr;
  {
    const int c = li < NC ? li : NC - 1;
    int j = j0 + c % JW;
    j = j < hlim ? j : hlim - 1;
    int grow = 0;
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (c / JW == g) grow = gate_row<EPI>(g);
    bptr = a.W + ((size_t)grow * (size_t)H + (size_t)j) * (size_t)a.ldw + 4 * kq;
  }

  const int groups_per_seg = a.kseg / 16;
  const int n_groups = a.nseg * groups_per_seg;
  const int mine = n_groups > w ? (n_groups - w + 3) / 4 : 0;  // groups w, w + 4, ...
  floatx4 acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
  EpilogueOperands<G, EPI, 1> eo;
  for (int base = 0; base < mine || base == 0; base += kDirectGroups) {
    floatx4 rb[kDirectGroups], ra[kDirectGroups];
#pragma unroll
    for (int t = 0; t < kDirectGroups; ++t)
      if (base + t < mine) rb[t] = *reinterpret_cast<const floatx4*>(bptr + 16 * (4 * (base + t) + w));
    const float* aptr0 = a.nseg > 0 ? a.src0 + (size_t)row0 * (size_t)a.ld0 + 4 * kq : nullptr;
    const float* aptr1 = a.nseg > 1 ? a.src1 + (size_t)row1 * (size_t)a.ld1 + 4 * kq : aptr0;
#pragma unroll
    for (int t = 0; t < kDirectGroups; ++t)
      if (base + t < mine) {
        const int grp = 4 * (base + t) + w;
        const bool seg = grp >= groups_per_seg;
        ra[t] = *reinterpret_cast<const floatx4*>((seg ? aptr1 : aptr0) + 16 * (grp - (seg ? groups_per_seg : 0)));
      }
    if (base == 0) {  // the gate arithmetic's own operands, right behind the rows
      if (tid < 16) {
        sidx[li] = orow;
        sidx[16 + li] = row0;
        sidx[32 + li] = row1;
      }
      __syncthreads();
      if (finisher) epilogue_fetch<G, EPI, 1>(a, ej, [&](int) { return m0 + er; }, eo, sidx, 16, m0);
    }
#pragma unroll
    for (int t = 0; t < kDirectGroups; ++t)
      if (base + t < mine) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (t & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[t][e], rb[t][e], acc1, 0, 0, 0);
          else acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[t][e], rb[t][e], acc0, 0, 0, 0);
        }
      }
  }
  // result register v of lane l: node 4 (l / 16) + v, column l % 16
#pragma unroll
  for (int v = 0; v < 4; ++v) z[w][4 * kq + v][li] = acc0[v] + acc1[v];
  __syncthreads();
  if (!finisher || m0 + er >= n) return;
  float zs[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float sum = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) sum += z[q][er][g * JW + tid % JW];
    zs[g] = sum;
  }
  epilogue_apply<G, EPI, 1>(a, ej, [&](int g, int) { return zs[g]; }, eo);
}

template <int G>
unsigned direct_grid(const CellLevelArgs& a, bool relu_out) {
  const int hlim = relu_out ? a.n_cols : a.H;
  const int n_jt = (hlim + direct_jw<G>() - 1) / direct_jw<G>();
  return (unsigned)((long)((a.n + 15) / 16) * padded_unit_tiles(n_jt));
}

struct Shape {
  int bm, ksplit;  // bm == 6 stands for cell_tiny_kernel (ksplit then carries its slabs per step, 0 = automatic)
  int streamk_wgs = 0;  // > 0: the level is split evenly over this many workgroups in one launch (ksplit is 1)
};

// Workgroups for the even split of a level, 0 if the level cannot be split that way.
template <int G>
int streamk_workgroups(const CellLevelArgs& a, const SplitKWorkspace& ws, int bm) {
  const long n_slabs = (long)a.nseg * (a.kseg / kBK);
  const long tiles = (long)((a.n + bm - 1) / bm) * (a.H / 32);
  if (n_slabs < 4 || ws.n_cu <= 0 || !ws.counters || tiles > ws.n_counters) return 0;
  // a share is at least a quarter of a tile's k range: at most five pieces per tile, at least one unit per workgroup
  const long wgs = std::min<long>(ws.n_cu, 4 * tiles);  // two per compute unit measured slower (65 vs 61 us at 288 tiles)
  const size_t floats = (size_t)wgs * 2 * (bm / 32) * G * kBlockFloats;
  if (floats > ws.partial_floats || floats * sizeof(float) >= ((size_t)1 << 32)) return 0;
  return (int)wgs;
}

// Picks the node-tile height and the k split for a level from a small cost model.
template <int G>
Shape pick_shape(const CellLevelArgs& a, const SplitKWorkspace& ws) {
  const int n_jt = a.H / 32;
  const int n_slabs = a.nseg * (a.kseg / kBK);
  auto fits = [&](int bm, int s) {
    if (s < 1 || s > 32 || (s & (s - 1))) return false;
    if (s == 1) return true;
    if (n_slabs == 0 || n_slabs % s != 0) return false;
    const long tiles = (long)((a.n + bm - 1) / bm) * n_jt;
    return (size_t)tiles * s * (bm / 32) * G * kBlockFloats <= ws.partial_floats;
  };
  if (ws.force_bm == 6) return Shape{6, ws.force_ksplit == 4 || ws.force_ksplit == 8 ? ws.force_ksplit : 0};
  if (ws.force_bm == 16) return Shape{16, 1};
  if (ws.force_bm == 65 || ws.force_bm == 33) {  // tuning override: even split with 64- or 32-node tiles
    const int bm = ws.force_bm - 1;
    const int wgs = streamk_workgroups<G>(a, ws, bm);
    if (wgs > 0) return Shape{bm, 1, wgs};
  }
  if (ws.force_bm == 64 || ws.force_bm == 32) {  // tuning override
    Shape f{ws.force_bm, ws.force_ksplit > 0 ? ws.force_ksplit : 1};
    if (fits(f.bm, f.ksplit)) return f;
  }
  // Rules fitted to sweeps on MI355X (TreeLSTM H = 512 and 256, LSTM H = 512):
  //  * 64-node tiles for all but the smallest levels (32-node tiles re-read the weights too often;
  //    a 128-node tile was measured and dropped: at the level sizes of these workloads it leaves
  //    too few workgroups and turns 2.1 rounds into 3);
  //  * one compute unit streams its operand slabs at only ~40 GB/s, so a level with fewer
  //    tiles than compute units is latency bound: split k until about 256 workgroups exist
  //    (at least 2 slabs each, at most 8 ways - the reduction kernel costs a launch, ~3 us,
  //    and reads ksplit partial tiles);
  //  * slightly more tiles than compute units: split in two for balance.
  //  * latency-bound levels (n x K up to about 256 000) run cell_tiny_kernel: one launch, no k split;
  //  * cell_direct_kernel (no steps at all, but every workgroup pulls its 16 node rows and 16 weight rows through
  //    the L2 on its own) while all its workgroups are resident at once and together request at most 24 MiB.
  //    Measured against the stepwise kernel: five-gate tree level, K = 1024, up to 16 nodes 5.6-6.8 instead of
  //    9.6-10.0 us (36 nodes: 13.5 instead of 10.4); K = 512, up to 64 nodes 4.5-6.7 instead of 6.6-7.1 (88 nodes:
  //    8.7 instead of 7.1); LSTM step, K = 512, up to 30 rows 5.2 instead of 6.8; single-gate recurrent step,
  //    K = 256, 128 rows 4.4 instead of 6.9.
  const int hlim = a.n_cols > 0 ? a.n_cols : a.H;
  const long direct_jt = (hlim + direct_jw<G>() - 1) / direct_jw<G>(), direct_mt = (a.n + 15) / 16;
  const long direct_wgs = direct_mt * direct_jt;                                      // those that have a tile
  const long direct_rows = direct_wgs * (G * direct_jw<G>()) + direct_jt * (long)a.n;  // weight rows + node rows requested
  //    A single-gate cell leaves the other kernels little to work with (a quarter of the stepwise kernel's matrix
  //    columns, 32-column tiles with one accumulator block), so there the limit is 64 MiB and the rule applies
  //    whatever n x K: recurrent cell of the tree generator, H = 512, K = 1024, 165-244 rows (two cells per launch)
  //    12.4-16.8 us against 22-30 us (stepwise) and 12.2-21 us (32-node tiles); 587 rows go to the tiled kernel.
  const long direct_cap = G == 1 ? (64L << 20) : (24L << 20);
  const bool direct_ok = ws.n_cu > 0 && direct_wgs <= 2L * ws.n_cu &&
                         direct_rows * n_slabs * kBK * (long)sizeof(float) <= direct_cap;
  if (G == 1 && direct_ok) return Shape{16, 1};
  if ((long)a.n * n_slabs * kBK <= 256000) return direct_ok ? Shape{16, 1} : Shape{6, 0};
  //  * a narrow output layer (at most 8 unit tiles of the direct kernel, e.g. 16 output units) gives the tiled
  //    kernels one unit tile, i.e. few workgroups however many rows it has: 1 299 rows x 16 units, K = 1024,
  //    9.3 us as 21 tiles split eight ways plus the reduction launch;
  if (direct_ok && direct_jt <= 8) return Shape{16, 1};
  //  * levels whose 32-node tiles all fit the chip at once (one workgroup per compute unit) run them
  //    unsplit: 29-30 us at 286 / 399 nodes against 32-33 us for 64-node tiles split in two;
  const long tiles32 = (long)((a.n + 31) / 32) * n_jt;
  //    (single-gate cells too: 603 rows, H = 256, 9.0 instead of 12.4 us; 587 rows, H = 512, 17.5 instead of 18.6)
  if (tiles32 <= 256 && (G >= 4 || G == 1)) return Shape{32, 1};
  Shape best{a.n > 128 ? 64 : 32, 1};
  const long tiles = (long)((a.n + best.bm - 1) / best.bm) * n_jt;
  //  * up to two rounds of 64-node tiles: whole tiles leave compute units idle for part of the level (144 or
  //    208 tiles take as long as 256, 288 nearly as long as 512).  Cutting the level into equal shares, one
  //    per compute unit, inside one launch (cell_streamk_kernel) evens that out but costs about 12 us of its
  //    own (a second prologue, parking and adding the pieces).  Fitted on H = 512: a slab of a five-gate
  //    tile takes 1.4 us on a compute unit, two co-resident tiles 1.87 times one; measured 61 instead of
  //    74 us at 288 tiles, 39 instead of 44 at 144, but 49 instead of 45 at 208 and 90 instead of 85 at 448.
  if (best.bm == 64 && tiles <= 2L * ws.n_cu && ws.n_cu > 0) {
    const double full = 0.28 * G * n_slabs;  // one whole tile on a compute unit of its own, us
    const double plain = tiles <= ws.n_cu ? full : 1.87 * full;
    const double even = (double)tiles / ws.n_cu * full + 12.0;
    if (even < 0.95 * plain) {
      const int wgs = streamk_workgroups<G>(a, ws, 64);
      if (wgs > 0) return Shape{64, 1, wgs};
    }
  }
  int s = 1;
  while (s * 2 <= 8 && tiles * s * 2 <= 256 && n_slabs % (s * 2) == 0 && n_slabs / (s * 2) >= 2) s *= 2;
  //  * the reduction kernel adds about 4.4 us to the level's dependent chain while one workgroup
  //    streams about 50 KB/us: splitting must take at least that much streaming time off the
  //    workgroup, or the level runs unsplit (single-gate RNN steps, narrow LSTMs).
  const double wg_kb = (double)(32 * G + best.bm) * n_slabs * kBK * sizeof(float) / 1024.0;
  if (s > 1 && wg_kb * (1.0 - 1.0 / s) < 4.4 * 50.0) s = 1;
  //    (only where two workgroups fill a compute unit: single-gate tiles fit five to a unit and run such a level
  //    unsplit in one round - 22 instead of 38 us for the two input projections of 1 299 rows, H = 512)
  if (s == 1 && G >= 3 && tiles > 256 && tiles <= 384 && n_slabs % 2 == 0 && n_slabs >= 8) s = 2;
  if (fits(best.bm, s)) best.ksplit = s;
  return best;
}

template <int G>
long tiny_live_workgroups(const CellLevelArgs& a, bool relu_out) {  // workgroups of tiny_grid that have a tile
  const int hlim = relu_out ? a.n_cols : a.H;
  return (long)((a.n + 31) / 32) * ((hlim + tiny_jw<G>() - 1) / tiny_jw<G>());
}

template <int G>
unsigned tiny_grid(const CellLevelArgs& a, bool relu_out) {
  const int hlim = relu_out ? a.n_cols : a.H;
  return (unsigned)((long)((a.n + 31) / 32) * padded_unit_tiles((hlim + tiny_jw<G>() - 1) / tiny_jw<G>()));
}

// `b` (may be null) is a second, independent batch for the same launch.
template <int G, int EPI>
hipError_t launch_shape(const CellLevelArgs& a, const CellLevelArgs* b, hipStream_t stream, const SplitKWorkspace& ws,
                        int32_t* tile, int32_t* ksplit, const LaunchEvents& ev) {
  const Shape sh = pick_shape<G>(a, ws);
  if (b) {
    const Shape sh2 = pick_shape<G>(*b, ws);
    const bool shareable = sh.bm == sh2.bm && sh.streamk_wgs == 0 && sh2.streamk_wgs == 0 &&
                           (sh.bm == 6 ? sh.ksplit == sh2.ksplit : (sh.ksplit == 1 && sh2.ksplit == 1));

    if (!shareable) {  // two launches in a row, bracketed as one: first kernel's begin .. last kernel's end
      LaunchEvents e0, e1;
      e0.start = ev.start;
      if (sh2.bm != 6 && sh2.ksplit > 1 && sh2.streamk_wgs == 0) e1.reduce_stop = ev.stop;
      else e1.stop = ev.stop;
      const hipError_t err = launch_shape<G, EPI>(a, nullptr, stream, ws, tile, nullptr, e0);
      if (err != hipSuccess) return err;
      if (ksplit) *ksplit = 1;
      return launch_shape<G, EPI>(*b, nullptr, stream, ws, nullptr, nullptr, e1);
    }
  }
  if (tile) *tile = sh.bm;
  if (ksplit) *ksplit = sh.ksplit;
  CellLevelPair pr;
  pr.a[0] = a;
  pr.a[1] = b ? *b : a;
  if (sh.bm == 6) {
    const unsigned g0 = tiny_grid<G>(a, EPI == EPI_RELU_OUT), g1 = b ? tiny_grid<G>(*b, EPI == EPI_RELU_OUT) : 0;
    pr.split = (int32_t)g0;
    // 8 slabs per step need 128 KB of LDS, one workgroup per compute unit: only while all fit at once
    const long live = tiny_live_workgroups<G>(a, EPI == EPI_RELU_OUT) + (b ? tiny_live_workgroups<G>(*b, EPI == EPI_RELU_OUT) : 0);
    const int u = sh.ksplit ? sh.ksplit : (live <= 256 ? 8 : 4);
    if (ksplit) *ksplit = 1;
    return u == 8 ? launch_tiny<G, EPI, 8>(pr, g0 + g1, stream, ev) : launch_tiny<G, EPI, 4>(pr, g0 + g1, stream, ev);
  }
  if (sh.bm == 16) {
    const unsigned g0 = direct_grid<G>(a, EPI == EPI_RELU_OUT), g1 = b ? direct_grid<G>(*b, EPI == EPI_RELU_OUT) : 0;
    pr.split = (int32_t)g0;  // (a multiple of 8 where the unit tiles are padded: the second batch keeps its XCD assignment)
    launch_with_events((cell_direct_kernel<G, EPI>), dim3(g0 + g1), dim3(kThreads), 0, stream, ev.start, ev.stop, pr);
    return hipGetLastError();
  }
  if (sh.streamk_wgs > 0) {
    StreamKArgs sk{a, sh.streamk_wgs, ws.partial,
                   (uint32_t)((size_t)sh.streamk_wgs * 2 * (sh.bm / 32) * G * kBlockFloats * sizeof(float)), ws.counters};
    if (ksplit) *ksplit = 0;  // reported as 0: cut into equal shares, not into a fixed number of k ranges per tile
    if (sh.bm == 64) {
      launch_with_events((cell_streamk_kernel<G, EPI, 2, 2>), dim3((unsigned)sh.streamk_wgs), dim3(kThreads), 0, stream,
                         ev.start, ev.stop, sk);
    } else {
      launch_with_events((cell_streamk_kernel<G, EPI, 1, 4>), dim3((unsigned)sh.streamk_wgs), dim3(kThreads), 0, stream,
                         ev.start, ev.stop, sk);
    }
    return hipGetLastError();
  }
  const int n_jt = a.H / 32;
  const long n_mt = (a.n + sh.bm - 1) / sh.bm;
  // An unsplit single batch runs in the XCD-aware order (kernel argument 0) where that saves bytes: every XCD
  // then fetches a quarter of the weights and half of the node rows (2 W + 4 A in all) instead of an eighth and
  // all of them (W + 8 A), which is less once the node rows outweigh a quarter of the weights.
  const double a_bytes = (double)a.n * a.nseg * a.kseg, w_bytes = (double)G * a.H * a.nseg * a.kseg;
  const bool xcd_order = !b && sh.ksplit == 1 && n_jt % 4 == 0 && n_mt >= 2 && ws.force_bm == 0 && 4.0 * a_bytes > w_bytes;
  const unsigned g0 = xcd_order ? (unsigned)(2 * n_jt * ((n_mt + 1) / 2)) : (unsigned)(n_mt * n_jt * sh.ksplit);
  const unsigned g1 = b ? (unsigned)((long)((b->n + sh.bm - 1) / sh.bm) * (b->H / 32)) : 0;
  pr.split = (int32_t)g0;
  const unsigned grid = g0 + g1;
  const int ks_arg = xcd_order ? 0 : sh.ksplit;
  if (sh.bm == 64) {
    launch_with_events((cell_level_kernel<G, EPI, 2, 2>), dim3(grid), dim3(kThreads), 0, stream, ev.start,
                          ev.stop, pr, ks_arg, ws.partial);
  } else {
    launch_with_events((cell_level_kernel<G, EPI, 1, 4>), dim3(grid), dim3(kThreads), 0, stream, ev.start,
                          ev.stop, pr, ks_arg, ws.partial);
  }
  if (sh.ksplit > 1) {
    const int wm_count = sh.bm / 32;
    const unsigned rgrid = (unsigned)((long)((a.n + sh.bm - 1) / sh.bm) * n_jt * wm_count * 16);
    launch_with_events((cell_splitk_reduce_kernel<G, EPI>), dim3(rgrid), dim3(64), 0, stream, ev.reduce_start,
                          ev.reduce_stop, a, sh.ksplit, wm_count, (const float*)ws.partial);
  }
  return hipGetLastError();
}

// one wavefront per (operand list, row): a contiguous 16-byte-vector copy of the row
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(const GatherArgs g) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int vec = g.width >> 2;
  for (long r = (long)blockIdx.x * 4 + wave; r < (long)g.n * g.count; r += (long)gridDim.x * 4) {
    const int k = (int)(r / g.n), i = (int)(r % g.n);
    const floatx4* s = reinterpret_cast<const floatx4*>(g.src[k] + (size_t)g.idx[k][i] * g.width);
    floatx4* d = reinterpret_cast<floatx4*>(g.dst[k] + (size_t)i * g.width);
    for (int c = lane; c < vec; c += 64) d[c] = s[c];
  }
}

template <class F>
hipError_t dispatch_epilogue(CellEpilogue epi, F&& f) {
  switch (epi) {
    case EPI_TREE_LEAF: return f(std::integral_constant<int, 3>(), std::integral_constant<int, EPI_TREE_LEAF>());
    case EPI_TREE_INTERNAL: return f(std::integral_constant<int, 5>(), std::integral_constant<int, EPI_TREE_INTERNAL>());
    case EPI_LSTM_STEP: return f(std::integral_constant<int, 4>(), std::integral_constant<int, EPI_LSTM_STEP>());
    case EPI_STORE_Z: return f(std::integral_constant<int, 4>(), std::integral_constant<int, EPI_STORE_Z>());
    case EPI_STORE_Z1: return f(std::integral_constant<int, 1>(), std::integral_constant<int, EPI_STORE_Z>());
    case EPI_RNN_STEP: return f(std::integral_constant<int, 1>(), std::integral_constant<int, EPI_RNN_STEP>());
    case EPI_RELU_OUT: return f(std::integral_constant<int, 1>(), std::integral_constant<int, EPI_RELU_OUT>());
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_cell_level(CellEpilogue epi, const CellLevelArgs& a, hipStream_t stream,
                             const SplitKWorkspace& ws, int32_t* tile, int32_t* ksplit, const LaunchEvents& ev) {
  if (a.n <= 0) return hipSuccess;
  return dispatch_epilogue(epi, [&](auto g, auto e) {
    return launch_shape<decltype(g)::value, decltype(e)::value>(a, nullptr, stream, ws, tile, ksplit, ev);
  });
}

hipError_t launch_cell_level_pair(CellEpilogue epi, const CellLevelArgs& a0, const CellLevelArgs& a1, hipStream_t stream,
                                  const SplitKWorkspace& ws, int32_t* tile, int32_t* ksplit, const LaunchEvents& ev) {
  if (a0.n <= 0) return launch_cell_level(epi, a1, stream, ws, tile, ksplit, ev);
  if (a1.n <= 0) return launch_cell_level(epi, a0, stream, ws, tile, ksplit, ev);
  return dispatch_epilogue(epi, [&](auto g, auto e) {
    return launch_shape<decltype(g)::value, decltype(e)::value>(a0, &a1, stream, ws, tile, ksplit, ev);
  });
}

hipError_t launch_gather_rows(const GatherArgs& g, hipStream_t stream, const LaunchEvents& ev) {
  if (g.n <= 0 || g.count <= 0) return hipSuccess;
  if (g.count > 4 || g.width % 4) return hipErrorInvalidValue;
  const long rows = (long)g.n * g.count;
  const unsigned grid = (unsigned)((rows + 3) / 4 < 4096 ? (rows + 3) / 4 : 4096);
  launch_with_events(gather_rows_kernel, dim3(grid), dim3(kThreads), 0, stream, ev.start, ev.stop, g);
  return hipGetLastError();
}

}  // namespace acrobat
