// MV-RNN level kernels for gfx950 (d = 64: register-resident kernel, one workgroup per node, and for single
// launches over narrow levels a kernel with four workgroups per node; d = 128: four workgroups per node; d = 64 or
// 128: streaming kernel, kept as a tuning alternative).
//
// Per node with left child (a, A) and right child (b, B):
//   p = tanh(W [B a ; A b]),   P = W_M [A ; B]          (W, W_M: [64,128])
// The two child matrices (16 KB each) are per-instance operands - this is the cell that
// multiplies two activations (Evaluation, "Overall Performance") - while W and W_M are shared by every node of
// every level (parameter reuse, section 5.1).  Children are read where they live: an
// internal child from the arena, a leaf child straight from the embedding tables (gather
// fusion, section 5.2; no copies of leaf embeddings, Evaluation, "Overall Performance").
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
//  * B a and A b reuse the same registers: a wavefront holds its whole child matrix (64
//    registers x 64 lanes), multiplies its two columns per row by the other child's vector
//    and sums over the 32 lanes of a half wavefront with a reduce-scatter butterfly (16 rows
//    per wavefront -> 16 exchanges instead of 16 x 5).  W [B a ; A b] runs on the vector
//    ALUs, four lanes per output row.
//  * the loop is software pipelined over nodes: the next node's indices and matrix loads
//    are issued before the current node's matrix instructions.
#include "cell_kernels.h"

#include "agent_access.h"

#include <algorithm>

namespace acrobat {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kD = 64;
constexpr int kDD = kD * kD;
constexpr int kWld = 2 * kD + 4;  // LDS row stride of W

__device__ __forceinline__ float fast_tanh(float x) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(__expf(2.0f * x) + 1.0f);
}

__device__ __forceinline__ float quad_sum(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

// 8-byte agent-scope accesses (see agent_access.h): one relaxed atomic each
__device__ __forceinline__ floatx2 load_agent_f2(const float* p) {
  const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return __builtin_bit_cast(floatx2, u);
}
__device__ __forceinline__ void store_agent_f2(float* p, floatx2 v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}

struct NodeRef {  // where one node's operands live and where its results go
  const float* mat;  // this wavefront's child matrix (left child for kh = 0, right for kh = 1)
  const float* vec;  // the OTHER child's vector
  size_t orow;
};

// DF (dataflow): ONE launch for all internal levels.  The list then holds every internal node in schedule
// order, workgroup w takes list positions w, w + grid, ..., and a node waits only for its own two children:
// every finished node announces itself in a flag word (the call's epoch number), the parent's workgroup polls
// the two words, bounded, before it requests the operands.  No level boundary, no barrier among workgroups: a
// batch takes (height of the tallest tree) x (one node's latency) instead of (levels) x (one launch).  Nothing
// can deadlock as long as all workgroups are resident (the host checks): the earliest unfinished list position
// only waits for earlier positions.  Children's states are stored write-through and read with agent-scope
// loads, as everything that workgroups of one kernel hand to each other (agent_access.h).
template <bool DF>
__global__ __launch_bounds__(256, 2) void mvrnn_level_kernel(const MvrnnLevelArgs a) {
  __shared__ float s_v[2 * kD];  // B a | A b
  __shared__ int s_go;
  __shared__ float s_red[2][2][16 * 64];  // [row block][k half of the writer][8 rows x even/odd x lane]
  __shared__ __attribute__((aligned(16))) float s_W[kD * kWld];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mb = wave & 1, kh = wave >> 1;
  const int lcol = lane & 31, lhi = lane >> 5;

  const int vr = tid >> 2, vq = tid & 3;  // p = tanh(W v): output row, quarter of the columns
  float wm[32];  // W_M[32*mb + lcol][64*kh + 2s + lhi], in registers for the whole launch (loaded below)

  struct RawIdx { int ls, rs, orow; };
  // the index lists are only read in this kernel and `node` is uniform in the workgroup
  const int32_t* __restrict__ lsrc = a.lsrc;
  const int32_t* __restrict__ rsrc = a.rsrc;
  const int32_t* __restrict__ orows = a.out_rows;
  auto load_idx = [&](int node) {
    const int u = __builtin_amdgcn_readfirstlane(node);
    RawIdx r;
    r.ls = lsrc[u];
    r.rs = rsrc[u];
    r.orow = orows[u];
    return r;
  };
  auto resolve = [&](const RawIdx& i) {
    const int ms = kh ? i.rs : i.ls, vs = kh ? i.ls : i.rs;
    NodeRef r;
    r.mat = ms >= 0 ? a.mat + (size_t)ms * kDD : a.mat_tab + (size_t)(-(ms + 1)) * kDD;
    r.vec = vs >= 0 ? a.vec + (size_t)vs * kD : a.vec_tab + (size_t)(-(vs + 1)) * kD;
    r.orow = (size_t)i.orow;
    return r;
  };
  auto load_node = [&](const NodeRef& r, floatx2 (&x)[32], floatx2& vv) {
    const float* X = r.mat + lhi * kD + 2 * lcol;
    if constexpr (DF) {  // a child may have been written by another workgroup of this launch
#pragma unroll
      for (int s = 0; s < 32; ++s) x[s] = load_agent_f2(X + 2 * s * kD);
      vv = load_agent_f2(r.vec + 2 * lcol);
    } else {
#pragma unroll
      for (int s = 0; s < 32; ++s) x[s] = *reinterpret_cast<const floatx2*>(X + 2 * s * kD);
      vv = *reinterpret_cast<const floatx2*>(r.vec + 2 * lcol);
    }
  };
  // DF: have both children of the node announced themselves?  (wave-uniform; leaves are table rows: always)
  auto children_done = [&](const RawIdx& i) {
    // (both words requested before either is looked at: one round trip, not two)
    const unsigned l = i.ls >= 0 ? load_agent(a.flags + i.ls) : a.epoch;
    const unsigned r = i.rs >= 0 ? load_agent(a.flags + i.rs) : a.epoch;
    return l == a.epoch && r == a.epoch;
  };

  // one node: `x`, `vv` hold its operands; `xn`, `vvn` receive the next node's, whose indices
  // (`raw`) were fetched one iteration ago; the indices of the node after that are fetched now
  // DF only: `cur_raw` names the current node's children, `have` says whether its operands were already
  // requested (a wavefront requests the next node's operands early only if both children are done by then)
  auto process = [&](int node, NodeRef& cur, RawIdx& raw, floatx2 (&x)[32], floatx2& vv, floatx2 (&xn)[32],
                     floatx2& vvn, RawIdx& cur_raw, bool& have) -> bool {
    if constexpr (DF) {
      if (tid == 0) {
        int polls = 0;
        bool ok = true;
        if (a.max_polls == 0) {  // test hook: every wait gives up at once, whether or not it would have had to wait
          raise_status(a.status);
          ok = false;
        }
        while (ok && !children_done(cur_raw)) {
          if (++polls > a.max_polls) {
            raise_status(a.status);
            ok = false;
            break;
          }
          if ((polls & 255) == 0 && status_raised(a.status)) { ok = false; break; }
          __builtin_amdgcn_s_sleep(1);
        }
        s_go = ok ? 1 : 0;
      }
      __syncthreads();
      if (!s_go) return false;  // a wait ran out here or elsewhere: drain
      if (!have) load_node(cur, x, vv);
    }
    // (indices past the end are clamped to the last node: a harmless re-read keeps the loop body
    // free of branches, so the compiler can leave these loads in flight)
    const int next2 = min(node + 2 * (int)gridDim.x, a.n - 1);
    // (opaque to the optimiser: nothing derived from these indices may be computed, and so
    // waited for, before this point - they were requested a whole iteration ago)
    asm volatile("" : "+v"(raw.ls), "+v"(raw.rs), "+v"(raw.orow));
    const NodeRef nxt = resolve(raw);
    const RawIdx nxt_raw = raw;
    raw = load_idx(next2);

    // ---- mat-vec rows 2*(16 mb + i) + lhi, i < 16: partial over this lane's two columns,
    // then reduce-scatter over the 32 lanes of the half wavefront
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const floatx2 xi = mb ? x[16 + i] : x[i];  // (a select, not a runtime register index)
      v[i] = xi[0] * vv[0] + xi[1] * vv[1];
    }
#pragma unroll
    for (int half = 8, bit = 16; half >= 1; half >>= 1, bit >>= 1) {
      const bool up = (lcol & bit) != 0;  // upper lanes keep the upper half of the rows
#pragma unroll
      for (int i = 0; i < half; ++i) {
        const float send = up ? v[i] : v[i + half];
        const float keep = up ? v[i + half] : v[i];
        v[i] = keep + __shfl_xor(send, bit);
      }
    }
    v[0] += __shfl_xor(v[0], 1);  // lanes 2i, 2i+1 both hold row i's sum now
    if ((lcol & 1) == 0) s_v[(kh ? 0 : kD) + 2 * (16 * mb + (lcol >> 1)) + lhi] = v[0];

    // ---- next node's operands: in flight during this node's matrix instructions
    bool have_next = true;
    if constexpr (DF) have_next = node + (int)gridDim.x < a.n && children_done(nxt_raw);
    if (have_next) load_node(nxt, xn, vvn);

    // ---- P: 32 k-steps of two 32x32 blocks (even / odd output columns)
    floatx16 acc_e, acc_o;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc_e[q] = acc_o[q] = 0.0f;
#pragma unroll
    for (int s = 0; s < 32; ++s) {
      acc_e = __builtin_amdgcn_mfma_f32_32x32x2f32(wm[s], x[s][0], acc_e, 0, 0, 0);
      acc_o = __builtin_amdgcn_mfma_f32_32x32x2f32(wm[s], x[s][1], acc_o, 0, 0, 0);
    }
    // the 33 operand loads of the next node go out first, one per matrix instruction
#pragma unroll
    for (int i = 0; i < 33; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 31, 0);
    // the two k halves exchange half of their accumulator rows through LDS (kh = 0 hands over
    // rows q >= 8, kh = 1 rows q < 8), so both finish and store 8 rows: the same number of
    // stores on every wavefront keeps the memory counters of the two paths alike
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int qs = kh ? q : q + 8;
      s_red[mb][kh][(2 * q) * 64 + lane] = kh ? acc_e[q] : acc_e[q + 8];
      s_red[mb][kh][(2 * q + 1) * 64 + lane] = kh ? acc_o[q] : acc_o[q + 8];
      (void)qs;
    }
    __syncthreads();  // s_v and s_red complete

    // ---- p = tanh(W [B a ; A b])
    float t = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const floatx4 wk4 = *reinterpret_cast<const floatx4*>(&s_W[vr * kWld + vq * 32 + k * 4]);
#pragma unroll
      for (int e = 0; e < 4; ++e) t += wk4[e] * s_v[vq * 32 + k * 4 + e];
    }
    t = quad_sum(t);
    if (vq == 0) {
      if constexpr (DF) __hip_atomic_store(a.vec + cur.orow * kD + vr, fast_tanh(t), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else a.vec[cur.orow * kD + vr] = fast_tanh(t);
    }

    {
      float* P = a.mat + cur.orow * kDD;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int qq = kh ? q + 8 : q;  // accumulator row finished by this wavefront
        const int i = mb * 32 + (qq >> 2) * 8 + lhi * 4 + (qq & 3);
        const float mine_e = kh ? acc_e[q + 8] : acc_e[q], mine_o = kh ? acc_o[q + 8] : acc_o[q];
        const float other_e = s_red[mb][kh ^ 1][(2 * q) * 64 + lane];
        const float other_o = s_red[mb][kh ^ 1][(2 * q + 1) * 64 + lane];
        floatx2 o;  // always (k half 0) + (k half 1)
        o[0] = kh ? other_e + mine_e : mine_e + other_e;
        o[1] = kh ? other_o + mine_o : mine_o + other_o;
        if constexpr (DF) store_agent_f2(P + i * kD + 2 * lcol, o);
        else *reinterpret_cast<floatx2*>(P + i * kD + 2 * lcol) = o;
      }
    }
    if constexpr (DF) wait_stores_done();  // this wavefront's part of the node's state has been written through
    __syncthreads();  // s_v / s_red are reused by the next node (DF: every wavefront's stores have completed)
    if constexpr (DF) {
      if (tid == 0) __hip_atomic_store(a.flags + cur.orow, a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      cur_raw = nxt_raw;
      have = have_next;
    }
    cur = nxt;
    return true;
  };

  int node = blockIdx.x;
  if (node >= a.n) return;
  // The first node's indices head the longest dependent chain (indices -> operands -> matrix
  // instructions), so they are requested before anything else.  The shared weights depend on
  // nothing and follow as a few wide, coalesced loads: vector memory instructions issue in order,
  // so anything slow to issue here (W_M fetched element by element in its operand layout was: 32
  // loads per lane, each touching 32 lines) would hold back the operand loads behind it.
  RawIdx raw = load_idx(node);
  RawIdx raw_next = load_idx(min(node + (int)gridDim.x, a.n - 1));
  // both weight matrices: coalesced 16-byte loads, 8 per thread each
  constexpr int kWVec = kD * 2 * kD / 4 / 256;
  floatx4 wmst[kWVec], wst[kWVec];
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    wmst[k] = *reinterpret_cast<const floatx4*>(a.WM + (i >> 5) * (2 * kD) + (i & 31) * 4);
  }
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    wst[k] = *reinterpret_cast<const floatx4*>(a.W + (i >> 5) * (2 * kD) + (i & 31) * 4);
  }
  NodeRef cur = resolve(raw);
  RawIdx cur_raw = raw;
  raw = raw_next;
  floatx2 x0[32], x1[32], vv0, vv1;
  bool have = !DF;  // DF: the first node's operands are requested once its children are known to be done
  if (have) load_node(cur, x0, vv0);
  // W_M goes through the LDS buffer of W first: every wavefront picks its operand registers
  // (row 32 mb + lcol, columns 64 kh + 2 s + lhi) out of it, then W takes the buffer over
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    *reinterpret_cast<floatx4*>(&s_W[(i >> 5) * kWld + (i & 31) * 4]) = wmst[k];
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < 32; ++s) wm[s] = s_W[(mb * 32 + lcol) * kWld + kh * kD + 2 * s + lhi];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    *reinterpret_cast<floatx4*>(&s_W[(i >> 5) * kWld + (i & 31) * 4]) = wst[k];
  }
  while (true) {
    if (!process(node, cur, raw, x0, vv0, x1, vv1, cur_raw, have)) break;
    node += gridDim.x;
    if (node >= a.n) break;
    if (!process(node, cur, raw, x1, vv1, x0, vv0, cur_raw, have)) break;
    node += gridDim.x;
    if (node >= a.n) break;
  }
}

// d = 64, dataflow launches, FOUR workgroups per node.  With one workgroup per node the 64 dependent matrix
// instructions of a wavefront (1.7 us) are a third of what a node of a narrow level takes, and the narrow levels
// near the roots are most of a small batch's time.  Here workgroup (node, q) computes the 32 x 32 block of P with
// rows 32 (q / 2) .. and columns 32 (q % 2) .., and rows 16 q .. 16 q + 15 of p:
//  * wavefront (kh, kq) takes rows 32 kq .. 32 kq + 31 of child kh (kh = 0: A, kh = 1: B), ALL columns: lane l
//    holds columns l % 32 and l % 32 + 32 of rows 32 kq + 2 s + l / 32, s < 16.  That is a quarter of the k range of
//    P = W_M [A ; B]: 16 v_mfma_f32_32x32x2_f32 on the workgroup's column half (0.43 us), the four partial blocks
//    summed through LDS in ascending wavefront order;
//  * the same registers give this wavefront's 32 rows of B a or A b (reduce-scatter butterfly over the 32 lanes
//    of a half wavefront, as in mvrnn_level_kernel), so every workgroup forms the whole [B a ; A b] for itself
//    and no workgroup waits for another one of its node;
//  * every workgroup reads both child matrices whole (4 x the requests of the one-workgroup kernel; the four
//    workgroups of a node are 8 ids apart and share an XCD, so HBM sees them once);
//  * a node has four flag words, one per workgroup; a parent's workgroups each wait for all eight words of the two
//    children (as mvrnn_rows_kernel<true> does for d = 128).
__global__ __launch_bounds__(256, 3) void mvrnn_quarter_kernel(const MvrnnLevelArgs a) {
  constexpr int kRows = 16;  // rows of p, and of W, per workgroup
  __shared__ float s_v[2 * kD];  // B a | A b
  __shared__ __attribute__((aligned(16))) float s_red[4][16 * 64];  // [wavefront][accumulator register][lane]
  __shared__ __attribute__((aligned(16))) float s_W[kRows * kWld];
  __shared__ int s_go;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kh = wave >> 1, kq = wave & 1;
  const int lcol = lane & 31, lhi = lane >> 5;
  const int q4 = (blockIdx.x >> 3) & 3, mb = q4 >> 1, ch = q4 & 1;
  int slot = 8 * (blockIdx.x >> 5) + (blockIdx.x & 7);
  const int nslots = 8 * (gridDim.x >> 5);  // the grid is a multiple of 32 workgroups
  if (slot >= a.n) return;

  struct RawIdx { int ls, rs, orow; };
  const int32_t* __restrict__ lsrc = a.lsrc;
  const int32_t* __restrict__ rsrc = a.rsrc;
  const int32_t* __restrict__ orows = a.out_rows;
  auto load_idx = [&](int node) {
    const int u = __builtin_amdgcn_readfirstlane(node);
    RawIdx r;
    r.ls = lsrc[u];
    r.rs = rsrc[u];
    r.orow = orows[u];
    return r;
  };
  auto resolve = [&](const RawIdx& i) {
    const int ms = kh ? i.rs : i.ls, vs = kh ? i.ls : i.rs;
    NodeRef r;
    r.mat = ms >= 0 ? a.mat + (size_t)ms * kDD : a.mat_tab + (size_t)(-(ms + 1)) * kDD;
    r.vec = vs >= 0 ? a.vec + (size_t)vs * kD : a.vec_tab + (size_t)(-(vs + 1)) * kD;
    r.orow = (size_t)i.orow;
    return r;
  };
  auto load_f = [](const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
  auto load_node = [&](const NodeRef& r, float (&x)[16][2], float (&vv)[2]) {
    const float* X = r.mat + (32 * kq + lhi) * kD + lcol;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      x[s][0] = load_f(X + 2 * s * kD);
      x[s][1] = load_f(X + 2 * s * kD + 32);
    }
    vv[0] = load_f(r.vec + lcol);
    vv[1] = load_f(r.vec + lcol + 32);
  };
  auto children_done = [&](const RawIdx& i) {
    // (all eight words requested before any is looked at: one round trip, not eight)
    unsigned l[4], r[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      l[q] = i.ls >= 0 ? load_agent(a.flags + 4 * (size_t)i.ls + q) : a.epoch;
      r[q] = i.rs >= 0 ? load_agent(a.flags + 4 * (size_t)i.rs + q) : a.epoch;
    }
    bool ok = true;
#pragma unroll
    for (int q = 0; q < 4; ++q) ok = ok && l[q] == a.epoch && r[q] == a.epoch;
    return ok;
  };

  float wm[16];  // W_M[32 mb + lcol][64 kh + 32 kq + 2 s + lhi], in registers for the whole launch (loaded below)

  // one node, as in mvrnn_level_kernel<true>: `x`, `vv` hold (or receive, if !have) its operands, `xn`, `vvn` the
  // next node's if its children are done by the time this node's operands have been consumed
  auto process = [&](int node, NodeRef& cur, RawIdx& raw, float (&x)[16][2], float (&vv)[2], float (&xn)[16][2],
                     float (&vvn)[2], RawIdx& cur_raw, bool& have) -> bool {
    if (tid == 0) {
      int polls = 0;
      bool ok = true;
      if (a.max_polls == 0) {  // test hook: every wait gives up at once, whether or not it would have had to wait
        raise_status(a.status);
        ok = false;
      }
      while (ok && !children_done(cur_raw)) {
        if (++polls > a.max_polls) {
          raise_status(a.status);
          ok = false;
          break;
        }
        if ((polls & 255) == 0 && status_raised(a.status)) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      s_go = ok ? 1 : 0;
    }
    __syncthreads();
    if (!s_go) return false;  // a wait ran out here or elsewhere: drain
    if (!have) load_node(cur, x, vv);
    const int next2 = min(node + 2 * nslots, a.n - 1);
    asm volatile("" : "+v"(raw.ls), "+v"(raw.rs), "+v"(raw.orow));  // (requested a whole iteration ago)
    const NodeRef nxt = resolve(raw);
    const RawIdx nxt_raw = raw;
    raw = load_idx(next2);

    // ---- mat-vec rows 32 kq + 2 i + lhi, i < 16: partial over this lane's two columns, then reduce-scatter
    // over the 32 lanes of the half wavefront
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = x[i][0] * vv[0] + x[i][1] * vv[1];
#pragma unroll
    for (int half = 8, bit = 16; half >= 1; half >>= 1, bit >>= 1) {
      const bool up = (lcol & bit) != 0;  // upper lanes keep the upper half of the rows
#pragma unroll
      for (int i = 0; i < half; ++i) {
        const float send = up ? v[i] : v[i + half];
        const float keep = up ? v[i + half] : v[i];
        v[i] = keep + __shfl_xor(send, bit);
      }
    }
    v[0] += __shfl_xor(v[0], 1);  // lanes 2i, 2i+1 both hold row i's sum now
    if ((lcol & 1) == 0) s_v[(kh ? 0 : kD) + 2 * (16 * kq + (lcol >> 1)) + lhi] = v[0];

    // ---- P: this wavefront's 16 two-row steps on the workgroup's column half
    floatx16 acc;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.0f;
#pragma unroll
    for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wm[s], ch ? x[s][1] : x[s][0], acc, 0, 0, 0);

    // ---- next node's operands, if its children are done: in flight during the rest of this node
    const bool have_next = node + nslots < a.n && children_done(nxt_raw);
    if (have_next) load_node(nxt, xn, vvn);

#pragma unroll
    for (int q = 0; q < 16; ++q) s_red[wave][q * 64 + lane] = acc[q];
    __syncthreads();  // s_v and s_red complete

    // ---- p = tanh(W [B a ; A b]), rows 16 q4 .. 16 q4 + 15: 16 threads per row, 8 columns each
    {
      const int pr = tid >> 4, part = tid & 15;
      float t = 0.0f;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const floatx4 wk4 = *reinterpret_cast<const floatx4*>(&s_W[pr * kWld + part * 8 + k * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) t += wk4[e] * s_v[part * 8 + k * 4 + e];
      }
      t += __shfl_xor(t, 1);
      t += __shfl_xor(t, 2);
      t += __shfl_xor(t, 4);
      t += __shfl_xor(t, 8);
      if (part == 0) __hip_atomic_store(a.vec + cur.orow * kD + kRows * q4 + pr, fast_tanh(t), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // ---- accumulator registers 4 wave .. 4 wave + 3 are finished here: rows 32 mb + 8 wave + 4 lhi + (q & 3)
    {
      float* P = a.mat + cur.orow * kDD + (size_t)(32 * mb + 8 * wave + 4 * lhi) * kD + 32 * ch + lcol;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int q = 4 * wave + e;
        const float sum = ((s_red[0][q * 64 + lane] + s_red[1][q * 64 + lane]) + s_red[2][q * 64 + lane]) + s_red[3][q * 64 + lane];
        __hip_atomic_store(P + e * kD, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    wait_stores_done();  // this wavefront's part of the node's state has been written through
    __syncthreads();     // ... and so has every other wavefront's; s_v / s_red are reused by the next node
    if (tid == 0) __hip_atomic_store(a.flags + 4 * cur.orow + q4, a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    cur_raw = nxt_raw;
    have = have_next;
    cur = nxt;
    return true;
  };

  RawIdx raw = load_idx(slot);
  RawIdx raw_next = load_idx(min(slot + nslots, a.n - 1));
  // this workgroup's 32 rows of W_M go through s_red (32 x 128 floats) into the operand registers; its 16 rows of W
  // stay in LDS
  floatx4 wmst[4], wst[2];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = tid + 256 * k;
    wmst[k] = *reinterpret_cast<const floatx4*>(a.WM + (size_t)(32 * mb + (i >> 5)) * (2 * kD) + (i & 31) * 4);
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int i = tid + 256 * k;
    wst[k] = *reinterpret_cast<const floatx4*>(a.W + (size_t)(kRows * q4 + (i >> 5)) * (2 * kD) + (i & 31) * 4);
  }
  NodeRef cur = resolve(raw);
  RawIdx cur_raw = raw;
  raw = raw_next;
  float* const stage = &s_red[0][0];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = tid + 256 * k;
    *reinterpret_cast<floatx4*>(&stage[(i >> 5) * (2 * kD) + (i & 31) * 4]) = wmst[k];
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int i = tid + 256 * k;
    *reinterpret_cast<floatx4*>(&s_W[(i >> 5) * kWld + (i & 31) * 4]) = wst[k];
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < 16; ++s) wm[s] = stage[lcol * (2 * kD) + 64 * kh + 32 * kq + 2 * s + lhi];
  __syncthreads();  // s_red is free for the partial blocks
  float x0[16][2], x1[16][2], vv0[2], vv1[2];
  bool have = false;  // the first node's operands are requested once its children are known to be done
  while (true) {
    if (!process(slot, cur, raw, x0, vv0, x1, vv1, cur_raw, have)) break;
    slot += nslots;
    if (slot >= a.n) break;
    if (!process(slot, cur, raw, x1, vv1, x0, vv0, cur_raw, have)) break;
    slot += nslots;
    if (slot >= a.n) break;
  }
}

// Streaming variant, any D in {64, 128}: P = W_M [A ; B] with v_mfma_f32_16x16x4_f32.
// Lane l = 16 r4 + c loads 16 bytes: columns 4c..4c+3 (of a 64-column group) of row 4s + r4 of
// the stacked child matrices - exactly the B-operand layout of the instruction (k = l/16,
// n = l%16) for four output column blocks at once, block e taking column 4c + e, so a lane
// ends up with four adjacent output columns per accumulator row and stores them as one float4.
// Wavefront w owns output rows [D/4 * w, D/4 * (w+1)) and streams ALL rows of [A ; B] through
// a ring of PF load slots (the four wavefronts read the same lines; no reduction through LDS
// is needed).  Its rows of W_M are the A operand and stay in registers for the whole launch.
// B a and A b are formed from the streamed rows (wavefront w takes the steps s = w mod 4) and
// summed over the 16 lanes of a row group with a reduce-scatter butterfly.  The ring runs
// across node boundaries: the first PF steps of the next node are requested while the
// current node's last matrix instructions issue.
template <int D>
__global__ __launch_bounds__(256, D == 64 ? 2 : 1) void mvrnn_stream_kernel(const MvrnnLevelArgs a) {
  constexpr int CG = D / 64;     // 64-column groups
  constexpr int MB = D / 64;     // 16-row output blocks per wavefront
  constexpr int S = 2 * D / 4;   // 4-row steps over [A ; B]
  constexpr int SA = D / 4;      // steps inside A
  constexpr int PF = 8;          // load slots in flight
  constexpr int NV = S / 4;      // mat-vec rows groups handled by one wavefront
  constexpr int WLD = 2 * D + 4; // LDS row stride of W
  constexpr int LPR = 256 / D;   // lanes per output row of p = tanh(W v)
  constexpr int DD = D * D;
  __shared__ float s_v[2 * D];  // B a | A b
  __shared__ __attribute__((aligned(16))) float s_W[D * WLD];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, r4 = lane >> 4;

  float wm[MB][S];  // W_M[16 (MB w + mb) + c][4 s + r4]
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int s = 0; s < S; ++s) wm[mb][s] = a.WM[(size_t)(16 * (MB * w + mb) + c) * (2 * D) + 4 * s + r4];
  for (int i = tid; i < D * 2 * D / 4; i += 256) {
    const int r = i / (2 * D / 4), c4 = i % (2 * D / 4);
    *reinterpret_cast<floatx4*>(&s_W[r * WLD + c4 * 4]) = *reinterpret_cast<const floatx4*>(a.W + (size_t)r * (2 * D) + c4 * 4);
  }

  const int32_t* __restrict__ lsrc = a.lsrc;
  const int32_t* __restrict__ rsrc = a.rsrc;
  const int32_t* __restrict__ orows = a.out_rows;
  struct Raw { int ls, rs, orow; };
  struct Ref { const float* mA; const float* mB; const float* va; const float* vb; size_t orow; };
  auto load_idx = [&](int node) {
    Raw r;
    r.ls = lsrc[node];
    r.rs = rsrc[node];
    r.orow = orows[node];
    return r;
  };
  auto resolve = [&](const Raw& i) {
    Ref r;
    r.mA = i.ls >= 0 ? a.mat + (size_t)i.ls * DD : a.mat_tab + (size_t)(-(i.ls + 1)) * DD;
    r.va = i.ls >= 0 ? a.vec + (size_t)i.ls * D : a.vec_tab + (size_t)(-(i.ls + 1)) * D;
    r.mB = i.rs >= 0 ? a.mat + (size_t)i.rs * DD : a.mat_tab + (size_t)(-(i.rs + 1)) * DD;
    r.vb = i.rs >= 0 ? a.vec + (size_t)i.rs * D : a.vec_tab + (size_t)(-(i.rs + 1)) * D;
    r.orow = (size_t)i.orow;
    return r;
  };
  floatx4 ring[PF][CG];
  auto load_step = [&](const Ref& r, int s, int slot) {  // s, slot: compile-time at every call site
    const float* base = (s < SA ? r.mA + (size_t)(4 * s + r4) * D : r.mB + (size_t)(4 * (s - SA) + r4) * D) + 4 * c;
#pragma unroll
    for (int g = 0; g < CG; ++g) ring[slot][g] = *reinterpret_cast<const floatx4*>(base + 64 * g);
  };

  int node = blockIdx.x;
  if (node >= a.n) return;
  Raw raw = load_idx(node);
  Ref cur = resolve(raw);
  raw = load_idx(min(node + (int)gridDim.x, a.n - 1));
#pragma unroll
  for (int s = 0; s < PF; ++s) load_step(cur, s, s);

  for (; node < a.n; node += gridDim.x) {
    asm volatile("" : "+v"(raw.ls), "+v"(raw.rs), "+v"(raw.orow));  // fetched one node ago; consumed here
    const Ref nxt = resolve(raw);
    raw = load_idx(min(node + 2 * (int)gridDim.x, a.n - 1));
    floatx4 va4[CG], vb4[CG];  // the children's vectors, this lane's columns
#pragma unroll
    for (int g = 0; g < CG; ++g) {
      va4[g] = *reinterpret_cast<const floatx4*>(cur.va + 64 * g + 4 * c);
      vb4[g] = *reinterpret_cast<const floatx4*>(cur.vb + 64 * g + 4 * c);
    }

    floatx4 acc[MB][CG][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[mb][g][e] = floatx4{0.f, 0.f, 0.f, 0.f};
    float mv[NV];

#pragma unroll
    for (int s = 0; s < S; ++s) {
      floatx4 x[CG];
#pragma unroll
      for (int g = 0; g < CG; ++g) x[g] = ring[s % PF][g];
      if (s + PF < S) load_step(cur, s + PF, s % PF);
      else load_step(nxt, s + PF - S, s % PF);  // next node (a re-read of the last node at the very end)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            acc[mb][g][e] = __builtin_amdgcn_mfma_f32_16x16x4f32(wm[mb][s], x[g][e], acc[mb][g][e], 0, 0, 0);
      // mat-vec partial of rows 4s + r4 (every wavefront computes it, wavefront s % 4 keeps it)
      float d = 0.0f;
#pragma unroll
      for (int g = 0; g < CG; ++g) {
        const floatx4 v4 = s < SA ? vb4[g] : va4[g];  // A rows meet b, B rows meet a
#pragma unroll
        for (int e = 0; e < 4; ++e) d += x[g][e] * v4[e];
      }
      if ((s & 3) == 0) mv[s >> 2] = d;
      else mv[s >> 2] = (s & 3) == w ? d : mv[s >> 2];
    }
    // mv[i] belongs to step s = 4 i + w for w > 0 ... and to s = 4 i for w == 0 (set first, kept)
    // reduce over the 16 lanes of a row group
    int nv = NV;
#pragma unroll
    for (int bit = 8; bit >= 1; bit >>= 1) {
      if (nv > 1) {
        const int half = nv / 2;
        const bool up = (c & bit) != 0;
#pragma unroll
        for (int i = 0; i < NV / 2; ++i) {
          if (i < half) {
            const float send = up ? mv[i] : mv[i + half];
            const float keep = up ? mv[i + half] : mv[i];
            mv[i] = keep + __shfl_xor(send, bit);
          }
        }
        nv = half;
      } else {
        mv[0] += __shfl_xor(mv[0], bit);
      }
    }
    {
      // value index held by this lane: the bits of c at which a halving took place
      constexpr int HALVINGS = NV >= 16 ? 4 : NV >= 8 ? 3 : NV >= 4 ? 2 : 1;
      const int idx = c >> (4 - HALVINGS);
      const bool writer = (c & ((1 << (4 - HALVINGS)) - 1)) == 0;
      const int s = 4 * idx + w;
      const int row = 4 * s + r4;  // row of [A ; B]
      if (writer) s_v[row < D ? D + row : row - D] = mv[0];  // A b goes below B a
    }
    __syncthreads();

    // p = tanh(W [B a ; A b])
    {
      const int pr = tid / LPR, pq = tid % LPR;
      constexpr int COLS = 2 * D / LPR;
      float t = 0.0f;
#pragma unroll
      for (int k = 0; k < COLS / 4; ++k) {
        const floatx4 w4 = *reinterpret_cast<const floatx4*>(&s_W[pr * WLD + pq * COLS + k * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) t += w4[e] * s_v[pq * COLS + k * 4 + e];
      }
#pragma unroll
      for (int bit = 1; bit < LPR; bit <<= 1) t += __shfl_xor(t, bit);
      if (pq == 0) a.vec[cur.orow * D + pr] = fast_tanh(t);
    }
    // P rows 16 (MB w + mb) + 4 r4 + v, columns 64 g + 4 c .. +3
    float* P = a.mat + cur.orow * DD;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          floatx4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = acc[mb][g][e][v];
          *reinterpret_cast<floatx4*>(P + (size_t)(16 * (MB * w + mb) + 4 * r4 + v) * D + 64 * g + 4 * c) = o;
        }
    __syncthreads();  // s_v is reused by the next node
    cur = nxt;
  }
}

// d = 128, four workgroups per node: workgroup (node, r) computes rows 32 r .. 32 r + 31 of P and
// of p.  It needs a quarter of W_M and of W (32 KB each instead of 128 KB: loaded once per launch,
// W_M into 64 registers per lane, W into LDS) and streams both child matrices whole; B a and A b
// fall out of the streamed registers, so each of the four workgroups forms them for itself and no
// workgroup waits for another.  A node occupies four compute units for a quarter of the time,
// which is what the narrow levels near the roots need: one node per compute unit costs 14 us of
// matrix instructions however few nodes the level has.
//  * wavefront (ch, kh): output columns 64 ch .. 64 ch + 63 (even / odd columns in two
//    accumulator blocks, as in the d = 64 kernel), k half kh (kh = 0: W_M[:, :128] times A,
//    kh = 1: W_M[:, 128:] times B): 64 two-row steps of two `v_mfma_f32_32x32x2_f32` each;
//  * the child matrix streams through a ring of 32 eight-byte load slots per lane that runs
//    across node boundaries;
//  * the workgroups of one node are 8 ids apart, 8 consecutive ids being spread over the 8 XCDs:
//    the four readers of a child matrix share one L2.
//
// DF (dataflow): one launch for all internal levels, as mvrnn_level_kernel<true> does for d = 64.  A node has four
// flag words here, one per workgroup (row quarter) that writes a part of its state; the four workgroups of the
// parent each wait for all eight words of the two children.  The ring only runs on into the next node when a
// wavefront finds that node's children complete at that point; otherwise it is refilled after the wait.
template <bool DF>
__global__ __launch_bounds__(256, 2) void mvrnn_rows_kernel(const MvrnnLevelArgs a) {
  constexpr int D = 128, DD = D * D;
  constexpr int S = 64;            // two-row steps over one child matrix
  constexpr int RING = 32;         // load slots in flight
  constexpr int WLD = 2 * D + 4;   // LDS row stride of the weight rows
  constexpr int RB = 32;           // output rows per workgroup
  __shared__ float s_vp[2][2 * D];        // [column half of the writer][B a | A b], partial sums
  __shared__ float s_red[2][2][16 * 64];  // [column half][k half of the writer][8 rows x even/odd x lane]
  __shared__ __attribute__((aligned(16))) float s_W[RB * WLD];
  __shared__ int s_go;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (uniform: base addresses stay in scalar registers)
  const int ch = wave & 1, kh = wave >> 1;
  const int lcol = lane & 31, lhi = lane >> 5;
  const int r = (blockIdx.x >> 3) & 3;
  int slot = 8 * (blockIdx.x >> 5) + (blockIdx.x & 7);
  const int nslots = 8 * (gridDim.x >> 5);  // the grid is a multiple of 32 workgroups
  if (slot >= a.n) return;

  struct RawIdx { int ls, rs, orow; };
  const int32_t* __restrict__ lsrc = a.lsrc;
  const int32_t* __restrict__ rsrc = a.rsrc;
  const int32_t* __restrict__ orows = a.out_rows;
  auto load_idx = [&](int node) {
    const int u = __builtin_amdgcn_readfirstlane(node);
    RawIdx i;
    i.ls = lsrc[u];
    i.rs = rsrc[u];
    i.orow = orows[u];
    return i;
  };
  auto resolve = [&](const RawIdx& i) {
    const int ms = __builtin_amdgcn_readfirstlane(kh ? i.rs : i.ls), vs = __builtin_amdgcn_readfirstlane(kh ? i.ls : i.rs);
    NodeRef n;
    n.mat = ms >= 0 ? a.mat + (size_t)ms * DD : a.mat_tab + (size_t)(-(ms + 1)) * DD;
    n.vec = vs >= 0 ? a.vec + (size_t)vs * D : a.vec_tab + (size_t)(-(vs + 1)) * D;
    n.orow = (size_t)i.orow;
    return n;
  };
  floatx2 ring[RING];
  // DF: a child may have been written by another workgroup of this launch: agent-scope loads, through a buffer
  // resource over the child's matrix (its base is wave-uniform) so that the step offset is a scalar
  const unsigned lane_off = (unsigned)((lhi * D + 64 * ch + 2 * lcol) * sizeof(float));
  auto load_step = [&](const NodeRef& n, int s, int k) {  // s, k: compile-time at every call site
    if constexpr (DF) {
      const floatx2 v = load_agent_f2_at(agent_buffer(n.mat, DD * sizeof(float)), lane_off, (unsigned)(2 * s * D * sizeof(float)));
      ring[k] = v;
    } else {
      ring[k] = *reinterpret_cast<const floatx2*>(n.mat + (size_t)(2 * s + lhi) * D + 64 * ch + 2 * lcol);
    }
  };
  auto load_vec = [&](const NodeRef& n) {
    if constexpr (DF) return load_agent_f2(n.vec + 64 * ch + 2 * lcol);
    else return *reinterpret_cast<const floatx2*>(n.vec + 64 * ch + 2 * lcol);
  };
  // DF: have all four parts of both children been announced?  (leaves are table rows: always)
  auto children_done = [&](const RawIdx& i) {
    // (all eight words requested before any is looked at: one round trip, not eight)
    unsigned l[4], r[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      l[q] = i.ls >= 0 ? load_agent(a.flags + 4 * (size_t)i.ls + q) : a.epoch;
      r[q] = i.rs >= 0 ? load_agent(a.flags + 4 * (size_t)i.rs + q) : a.epoch;
    }
    bool ok = true;
#pragma unroll
    for (int q = 0; q < 4; ++q) ok = ok && l[q] == a.epoch && r[q] == a.epoch;
    return ok;
  };
  // DF: thread 0 waits, bounded, for the children of the node; false = a wait ran out here or elsewhere: drain
  auto wait_children = [&](const RawIdx& i) {
    if (tid == 0) {
      int polls = 0;
      bool ok = true;
      if (a.max_polls == 0) {  // test hook: every wait gives up at once
        raise_status(a.status);
        ok = false;
      }
      while (ok && !children_done(i)) {
        if (++polls > a.max_polls) {
          raise_status(a.status);
          ok = false;
          break;
        }
        if ((polls & 255) == 0 && status_raised(a.status)) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      s_go = ok ? 1 : 0;
    }
    __syncthreads();
    return s_go != 0;
  };

  // indices first (they head the dependent chain), then the weight rows as coalesced 16-byte loads
  RawIdx raw = load_idx(slot);
  RawIdx raw_next = load_idx(min(slot + nslots, a.n - 1));
  constexpr int kWVec = RB * 2 * D / 4 / 256;  // 8
  floatx4 wmst[kWVec], wst[kWVec];
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    wmst[k] = *reinterpret_cast<const floatx4*>(a.WM + (size_t)(RB * r + (i >> 6)) * (2 * D) + (i & 63) * 4);
  }
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    wst[k] = *reinterpret_cast<const floatx4*>(a.W + (size_t)(RB * r + (i >> 6)) * (2 * D) + (i & 63) * 4);
  }
  NodeRef cur = resolve(raw);
  RawIdx cur_raw = raw;  // DF: the children the current node waits for
  raw = raw_next;
  bool have = !DF;       // DF: whether this wavefront has already requested the current node's first ring of rows
  floatx2 vv;
  if constexpr (!DF) {
#pragma unroll
    for (int s = 0; s < RING; ++s) load_step(cur, s, s);
    vv = load_vec(cur);
  }

  // W_M's rows pass through the LDS buffer of W: each wavefront picks its operand registers
  // (row 32 r + lcol, columns 128 kh + 2 s + lhi), then W's rows take the buffer over
  float wm[S];
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    *reinterpret_cast<floatx4*>(&s_W[(i >> 6) * WLD + (i & 63) * 4]) = wmst[k];
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < S; ++s) wm[s] = s_W[lcol * WLD + D * kh + 2 * s + lhi];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kWVec; ++k) {
    const int i = tid + 256 * k;
    *reinterpret_cast<floatx4*>(&s_W[(i >> 6) * WLD + (i & 63) * 4]) = wst[k];
  }

  const int pr = tid >> 3, pq = tid & 7;  // p = tanh(W v): output row of this workgroup, eighth of the columns
  while (true) {
    if constexpr (DF) {
      if (!wait_children(cur_raw)) return;
      if (!have) {
#pragma unroll
        for (int s = 0; s < RING; ++s) load_step(cur, s, s);
        vv = load_vec(cur);
      }
    }
    // (opaque to the optimiser: nothing derived from these indices may be computed, and so waited
    // for, before this point - they were requested a whole node ago)
    asm volatile("" : "+v"(raw.ls), "+v"(raw.rs), "+v"(raw.orow));
    const NodeRef nxt = resolve(raw);
    const RawIdx nxt_raw = raw;
    bool pre = true;  // DF: run the ring on into the next node?
    // (past the end the last node is read again: harmless, and the loop body stays free of branches)
    raw = load_idx(min(slot + 2 * nslots, a.n - 1));

    floatx16 acc_e, acc_o;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc_e[q] = acc_o[q] = 0.0f;
    float vp[16];
    floatx2 vv_next;
    // one two-row step: two matrix instructions and the step's share of (child matrix) x (other child's vector)
    auto consume = [&](int s) {  // s: compile-time at every call site (the loops below are fully unrolled)
      const floatx2 x = ring[s % RING];
      acc_e = __builtin_amdgcn_mfma_f32_32x32x2f32(wm[s], x[0], acc_e, 0, 0, 0);
      acc_o = __builtin_amdgcn_mfma_f32_32x32x2f32(wm[s], x[1], acc_o, 0, 0, 0);
      vp[s % 16] = x[0] * vv[0] + x[1] * vv[1];  // rows 2 s + lhi of (child matrix) x (other child's vector)
      if (s % 16 == 15) {
        // sum over the 32 lanes of the half wavefront: a reduce-scatter butterfly over four lane
        // bits, after which lanes 2 i and 2 i + 1 hold the two halves of step 16 (s / 16) + i
#pragma unroll
        for (int half = 8, bit = 16; half >= 1; half >>= 1, bit >>= 1) {
          const bool up = (lcol & bit) != 0;
#pragma unroll
          for (int i = 0; i < half; ++i) {
            float lo = vp[i], hi = vp[i + half];
            // (keeps these two selects of values: folded into one select of the array index, the
            // whole butterfly turns into compare chains over a register array indexed per lane)
            asm("" : "+v"(lo), "+v"(hi));
            const float send = up ? lo : hi;
            const float keep = up ? hi : lo;
            vp[i] = keep + __shfl_xor(send, bit);
          }
        }
        vp[0] += __shfl_xor(vp[0], 1);
        if ((lcol & 1) == 0) s_vp[ch][(kh ? 0 : D) + 2 * (16 * (s / 16) + (lcol >> 1)) + lhi] = vp[0];
      }
    };
    // first half: the slot just consumed takes the step 32 ahead, still of this node
#pragma unroll
    for (int s = 0; s < S - RING; ++s) {
      consume(s);
      load_step(cur, s + RING, s % RING);
    }
    // second half: the ring runs on into the next node.  DF: only if this wavefront finds that node's children
    // complete now (a wavefront-uniform decision; past the end of the list there is no next node)
    if constexpr (DF) pre = slot + nslots < a.n && __all(children_done(nxt_raw));
    if (pre) vv_next = load_vec(nxt);
#pragma unroll
    for (int s = S - RING; s < S; ++s) {
      consume(s);
      if (pre) load_step(nxt, s + RING - S, s % RING);
    }
    // the two k halves exchange half of their accumulator rows through LDS (kh = 0 hands over
    // rows q >= 8, kh = 1 rows q < 8), so every wavefront finishes and stores 8 rows
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      s_red[ch][kh][(2 * q) * 64 + lane] = kh ? acc_e[q] : acc_e[q + 8];
      s_red[ch][kh][(2 * q + 1) * 64 + lane] = kh ? acc_o[q] : acc_o[q + 8];
    }
    __syncthreads();  // s_vp and s_red complete (and, for the first node, W's rows in s_W)

    // ---- p = tanh(W [B a ; A b]), rows 32 r .. 32 r + 31
    {
      float t = 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const floatx4 wk4 = *reinterpret_cast<const floatx4*>(&s_W[pr * WLD + pq * 32 + k * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) t += wk4[e] * (s_vp[0][pq * 32 + k * 4 + e] + s_vp[1][pq * 32 + k * 4 + e]);
      }
      t += __shfl_xor(t, 1);
      t += __shfl_xor(t, 2);
      t += __shfl_xor(t, 4);
      if (pq == 0) {
        if constexpr (DF) __hip_atomic_store(a.vec + cur.orow * D + RB * r + pr, fast_tanh(t), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else a.vec[cur.orow * D + RB * r + pr] = fast_tanh(t);
      }
    }
    {
      float* P = a.mat + cur.orow * DD + (size_t)(RB * r) * D + 64 * ch + 2 * lcol;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int qq = kh ? q + 8 : q;  // accumulator row finished by this wavefront
        const int i = (qq >> 2) * 8 + lhi * 4 + (qq & 3);
        const float mine_e = kh ? acc_e[q + 8] : acc_e[q], mine_o = kh ? acc_o[q + 8] : acc_o[q];
        const float other_e = s_red[ch][kh ^ 1][(2 * q) * 64 + lane];
        const float other_o = s_red[ch][kh ^ 1][(2 * q + 1) * 64 + lane];
        floatx2 o;  // always (k half 0) + (k half 1)
        o[0] = kh ? other_e + mine_e : mine_e + other_e;
        o[1] = kh ? other_o + mine_o : mine_o + other_o;
        if constexpr (DF) store_agent_f2(P + i * D, o);
        else *reinterpret_cast<floatx2*>(P + i * D) = o;
      }
    }
    if constexpr (DF) {
      // this workgroup's quarter of the node is complete once every wavefront's stores are: announce it
      wait_stores_done();
      __syncthreads();
      if (tid == 0) __hip_atomic_store(a.flags + 4 * cur.orow + r, a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    slot += nslots;
    if (slot >= a.n) break;
    if constexpr (!DF) __syncthreads();  // s_vp / s_red are reused by the next node
    cur = nxt;
    cur_raw = nxt_raw;
    have = pre;
    vv = vv_next;
  }
}

__global__ __launch_bounds__(256) void mvrnn_leaf_copy_kernel(int n, int d, const int32_t* out_rows,
                                                              const int32_t* token, const float* vec_tab,
                                                              const float* mat_tab, float* vec, float* mat) {
  const int tid = threadIdx.x;
  const int dd4 = d * d / 4;
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    const size_t src = (size_t)token[i], dst = (size_t)out_rows[i];
    const floatx4* ms = reinterpret_cast<const floatx4*>(mat_tab + src * d * d);
    floatx4* md = reinterpret_cast<floatx4*>(mat + dst * d * d);
    for (int k = tid; k < dd4; k += 256) md[k] = ms[k];
    if (tid < d) vec[dst * d + tid] = vec_tab[src * d + tid];
  }
}

}  // namespace

hipError_t launch_mvrnn_level(const MvrnnLevelArgs& a, hipStream_t stream, int32_t* tile, const LaunchEvents& ev) {
  if (tile) *tile = 1;
  if (a.n <= 0) return hipSuccess;
  const int grid = a.n < 512 ? a.n : 512;  // two resident workgroups per compute unit, each strides over the level
  if (a.d == 128 && a.variant == 1) {
    launch_with_events(mvrnn_stream_kernel<128>, dim3(a.n < 256 ? a.n : 256), dim3(256), 0, stream, ev.start, ev.stop, a);
  } else if (a.d == 128) {
    // four workgroups per node slot, slots in groups of 8; 512 resident workgroups = 128 slots
    const int slots = a.n < 128 ? (a.n + 7) / 8 * 8 : 128;
    launch_with_events(mvrnn_rows_kernel<false>, dim3(4 * slots), dim3(256), 0, stream, ev.start, ev.stop, a);
  } else if (a.variant == 1) {
    launch_with_events(mvrnn_stream_kernel<64>, dim3(grid), dim3(256), 0, stream, ev.start, ev.stop, a);
  } else {
    launch_with_events(mvrnn_level_kernel<false>, dim3(grid), dim3(256), 0, stream, ev.start, ev.stop, a);
  }
  return hipGetLastError();
}

int mvrnn_dataflow_workgroups(int32_t d, int32_t n, bool quarters) {
  if ((d != 64 && d != 128) || n <= 0) return 0;
  int dev = 0, per_cu = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (d == 64 && !quarters) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mvrnn_level_kernel<true>, 256, 0) != hipSuccess) return 0;
    const long resident = (long)per_cu * cus;
    return (int)(n < resident ? n : resident);
  }
  // four workgroups per node slot, slots in groups of 8 (see mvrnn_quarter_kernel, mvrnn_rows_kernel)
  const hipError_t e = d == 64 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mvrnn_quarter_kernel, 256, 0)
                               : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mvrnn_rows_kernel<true>, 256, 0);
  if (e != hipSuccess) return 0;
  const long resident_slots = (long)per_cu * cus / 32 * 8;
  const long slots = std::min<long>((n + 7) / 8 * 8, resident_slots);
  return (int)(4 * slots);
}

hipError_t launch_mvrnn_dataflow(const MvrnnLevelArgs& a, int workgroups, bool quarters, hipStream_t stream, const LaunchEvents& ev) {
  if (a.n <= 0) return hipSuccess;
  if ((a.d != 64 && a.d != 128) || workgroups <= 0 || !a.flags || !a.status) return hipErrorInvalidValue;
  if (a.d == 64 && !quarters) {
    launch_with_events(mvrnn_level_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, stream, ev.start, ev.stop, a);
    return hipGetLastError();
  }
  if (workgroups % 32) return hipErrorInvalidValue;
  if (a.d == 128) {
    launch_with_events(mvrnn_rows_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, stream, ev.start, ev.stop, a);
  } else {
    launch_with_events(mvrnn_quarter_kernel, dim3((unsigned)workgroups), dim3(256), 0, stream, ev.start, ev.stop, a);
  }
  return hipGetLastError();
}

hipError_t launch_mvrnn_leaf_copy(int32_t n, int32_t d, const int32_t* out_rows, const int32_t* token,
                                  const float* vec_tab, const float* mat_tab, float* vec, float* mat,
                                  hipStream_t stream, const LaunchEvents& ev) {
  if (n <= 0) return hipSuccess;
  const int grid = n < 2048 ? n : 2048;
  launch_with_events(mvrnn_leaf_copy_kernel, dim3(grid), dim3(256), 0, stream, ev.start, ev.stop, n, d,
                        out_rows, token, vec_tab, mat_tab, vec, mat);
  return hipGetLastError();
}

}  // namespace acrobat
