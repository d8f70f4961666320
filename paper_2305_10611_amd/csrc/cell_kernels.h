// Launch interface of the gather-fused cell kernels (device code in cell_kernels.hip,
// mvrnn_kernels.hip).  Plain structs and functions only; no HIP types besides hipStream_t.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>

namespace acrobat {

enum CellEpilogue : int {
  EPI_TREE_LEAF = 0,      // gates (i, o, u): c = s(i) tanh(u), h = s(o) tanh(c)
  EPI_TREE_INTERNAL = 1,  // gates (i, f_l, f_r, o, u) + gathered child c rows
  EPI_LSTM_STEP = 2,      // gates (i, f, o, u) + precomputed input transform + previous c
  EPI_STORE_Z = 3,        // plain pre-activation store (hoisted input transform), 4 gates
  EPI_RNN_STEP = 4,       // single gate: h = s(z + precomputed input transform)
  EPI_RELU_OUT = 5,       // single gate: y = relu(z + bias), n_cols <= H valid columns
  EPI_STORE_Z1 = 6,       // EPI_STORE_Z with a single gate
};

// One batch (one depth level) of a cell whose contraction is
//   z[node, g*H + j] = sum_k in[node, k] * W[(gate_row[g]*H + j) * ldw + k]
// where in[node, :] is the concatenation of `nseg` row segments of length kseg, segment s
// being row idx_s[node] (or `node` itself when idx_s is null) of the matrix src_s.
struct CellLevelArgs {
  int32_t n;     // nodes in this batch (> 0)
  int32_t H;     // hidden size (multiple of 32)
  int32_t nseg;  // 0 (no contraction), 1 or 2
  int32_t kseg;  // columns per segment (multiple of 32)
  const float* src0; const int32_t* idx0; int32_t ld0;
  const float* src1; const int32_t* idx1; int32_t ld1;
  const float* W; int32_t ldw;  // weight rows are contiguous in k
  const float* bias;            // indexed like W's rows, or null
  const int32_t* out_rows;      // [n] arena row written by each node, null = node index
  float* h; float* c;           // arena [rows, H]
  const float* cprev_src;       // tree/LSTM: c rows gathered with idx0 (and idx1); null = zero state
  const float* zadd;            // LSTM / RNN step: [rows, G*H] pre-activations added to z (row = out row); RNN step: may be null
  float* zout;                  // STORE_Z: [rows, G*H]
  // RELU_OUT only: the weight matrix has n_cols <= H rows (H = n_cols rounded up to 32 sizes the
  // grid), y[row * ldo + j] is written for j < n_cols.  0 elsewhere (= H).
  int32_t n_cols;
  float* y; int32_t ldo;
};

// Device workspace for levels whose k range is split over several workgroups: partial
// accumulator tiles, written by the contraction kernel and summed by the reduction kernel
// that follows it on the stream.
struct SplitKWorkspace {
  float* partial = nullptr;
  size_t partial_floats = 0;
  // tile counters of the levels that are split evenly over the chip inside one launch (zero whenever no such
  // launch is in flight), and the number of compute units the split is made for
  unsigned* counters = nullptr;
  int32_t n_counters = 0;
  int32_t n_cu = 0;
  int32_t force_bm = 0, force_ksplit = 0;  // tuning override, 0 = automatic
};

// Optional events handed to the launches themselves: the runtime stamps them with the kernel's
// own begin and end, so their elapsed time is the kernel's execution time without the idle gaps
// that events recorded on the stream add around a launch.  Null = plain launch.
struct LaunchEvents {
  hipEvent_t start = nullptr, stop = nullptr;                // the level kernel
  hipEvent_t reduce_start = nullptr, reduce_stop = nullptr;  // the reduction kernel of a k-split level
};

// Two independent batches of the same cell type (the two directions of a bidirectional recurrence)
// can share one launch when both are handled by the same kernel variant without a k split:
// workgroups [0, split) execute a[0], the others a[1].
struct CellLevelPair {
  CellLevelArgs a[2];
  int32_t split;
};

// One launch: with events through the extended launch call (which stamps them), without events
// through the plain one (which, unlike the extended call, can be recorded by a stream capture).
template <class Kernel, class... Args>
inline void launch_with_events(Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, hipEvent_t start,
                               hipEvent_t stop, Args... args) {
  if (start || stop) hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, start, stop, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
}

// Launches the kernel for one level; picks the node-tile height and k split from the level's
// size and reports them in *tile / *ksplit (may be null).  Returns hipGetLastError().
hipError_t launch_cell_level(CellEpilogue epi, const CellLevelArgs& a, hipStream_t stream,
                             const SplitKWorkspace& ws, int32_t* tile, int32_t* ksplit,
                             const LaunchEvents& ev = LaunchEvents());

// MV-RNN level: for each of the n nodes at list positions [0,n):
//   p = tanh(W [B a ; A b]),  P = W_M [A ; B]  with (a,A) / (b,B) the left / right child state.
// A child source code s >= 0 means arena row s of (vec, mat); s < 0 means table row -(s+1).
struct MvrnnLevelArgs {
  int32_t n;
  int32_t d;        // 64 or 128
  int32_t variant;  // 0 = default kernel (d = 64: register-resident, d = 128: four workgroups per node), 1 = streaming kernel
  const int32_t* out_rows;  // [n]
  const int32_t* lsrc;      // [n] encoded left child source
  const int32_t* rsrc;      // [n]
  const float* vec_tab; const float* mat_tab;
  const float* W; const float* WM;  // [d,2d] each
  float* vec; float* mat;           // arena [rows,d], [rows,d,d]
  // launch_mvrnn_dataflow only: four words per arena row, word q set to `epoch` by workgroup q of the node that owns
  // the row once its part of the state has been stored (d = 64 without quarters: one word per row); the status word and the bound of every wait as for the other persistent kernels
  unsigned* flags; unsigned epoch;
  unsigned* status; int32_t max_polls;
};
// Same for two independent batches: one shared launch where the variants agree (then *tile / *ksplit
// describe it and ev brackets it), else two launches in a row on the stream (ev.start on the first,
// ev.stop on the second; *tile / *ksplit describe the first).
hipError_t launch_cell_level_pair(CellEpilogue epi, const CellLevelArgs& a0, const CellLevelArgs& a1, hipStream_t stream,
                                  const SplitKWorkspace& ws, int32_t* tile, int32_t* ksplit,
                                  const LaunchEvents& ev = LaunchEvents());

// Explicit gather (only for the unfused-gather ablation, section 5.2 / 7.5): copies rows idx[k][i] of
// src[k] (row stride = width floats) to row i of dst[k], for up to four operand lists in one launch.
struct GatherArgs {
  int32_t n, width, count;
  const int32_t* idx[4];
  const float* src[4];
  float* dst[4];
};
hipError_t launch_gather_rows(const GatherArgs& g, hipStream_t stream, const LaunchEvents& ev = LaunchEvents());

hipError_t launch_mvrnn_level(const MvrnnLevelArgs& a, hipStream_t stream, int32_t* tile,
                              const LaunchEvents& ev = LaunchEvents());

// All internal levels of an MV-RNN batch in ONE launch: the lists hold every internal node in schedule
// order; a node waits for its own two children only (a.flags / a.epoch), never for a whole level.  `quarters`
// (d = 64 only; d = 128 always works that way): four workgroups per node, each a quarter of the node's matrix
// product, for batches of narrow levels, where a node's latency is what counts; otherwise one workgroup per node.
// a.flags needs four words per arena row (one per workgroup of a node; d = 64 without quarters uses the first
// word per row of a [rows] array).
// mvrnn_dataflow_workgroups: how many workgroups such a launch may have so that all are resident at once on the
// current device (0: not available for this d); launch with exactly that many (d = 64 without quarters: or fewer).
int mvrnn_dataflow_workgroups(int32_t d, int32_t n, bool quarters);
hipError_t launch_mvrnn_dataflow(const MvrnnLevelArgs& a, int workgroups, bool quarters, hipStream_t stream,
                                 const LaunchEvents& ev = LaunchEvents());

// Copies table rows `token[i]` into arena rows out_rows[i] (vector and matrix), i in [0,n).
hipError_t launch_mvrnn_leaf_copy(int32_t n, int32_t d, const int32_t* out_rows, const int32_t* token,
                                  const float* vec_tab, const float* mat_tab, float* vec, float* mat,
                                  hipStream_t stream, const LaunchEvents& ev = LaunchEvents());

}  // namespace acrobat
