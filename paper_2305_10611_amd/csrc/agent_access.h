// Device-side helpers for data that workgroups of one kernel hand to each other (gfx950).
//
// Workgroups on different XCDs do not share an L2.  The language-level way to pass data is an agent-scope
// release / acquire pair, which on this part writes back and invalidates the whole L2 of the XCD: several
// microseconds per pair once a few hundred workgroups do it (measured by acrobat_sync_probe).  The helpers
// below are what such a pair is made of, minus the cache-wide operations: stores that are written through at
// agent scope, a wait for their completion, and loads that are coherent at agent scope.  They are enough when
// everything a consumer reads was stored this way: producer = store_agent*, wait_stores_done() in every
// wavefront, workgroup barrier, relaxed agent-scope atomic on a flag or counter; consumer = sees the flag,
// workgroup barrier, load_agent*.
#pragma once
#include <hip/hip_runtime.h>

namespace acrobat {

typedef float agent_f4 __attribute__((ext_vector_type(4)));
typedef unsigned agent_u4 __attribute__((ext_vector_type(4)));

constexpr int kRsrcFlags = 0x00020000;  // raw buffer resource, 32-bit data format (gfx9)
constexpr int kAuxAgentScope = 16;      // cache policy sc1: coherent at agent scope

// Buffer resource over [base, base + bytes), bytes < 2^32.  Offsets past the end read zero / store nothing.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t agent_buffer(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, kRsrcFlags);
}
__device__ __forceinline__ agent_f4 load_agent_f4(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_off) {
  return __builtin_bit_cast(agent_f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_off, 0, kAuxAgentScope));
}
__device__ __forceinline__ void store_agent_f4(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_off, agent_f4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(agent_u4, v), rsrc, (int)byte_off, 0, kAuxAgentScope);
}
// 8-byte load at (resource base + per-lane byte offset + wave-uniform byte offset): the uniform part travels in a
// scalar register, so a ring of such loads in flight needs no address registers of its own
typedef float agent_f2 __attribute__((ext_vector_type(2)));
typedef unsigned agent_u2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ agent_f2 load_agent_f2_at(__amdgpu_buffer_rsrc_t rsrc, unsigned lane_off, unsigned uniform_off) {
  return __builtin_bit_cast(agent_f2, __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_off, (int)uniform_off, kAuxAgentScope));
}
__device__ __forceinline__ unsigned load_agent(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The status word of the kernels that wait for other workgroups lives in pinned host memory: it is only written
// when a wait runs out and only read by workgroups that have been polling for a while, so the host sees it
// without any copy and the ordinary case never touches it.
__device__ __forceinline__ void raise_status(unsigned* status) {
  __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ bool status_raised(const unsigned* status) {
  return __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0;
}
// s_waitcnt vmcnt(0) (gfx9 encoding, the other counters at their maximum): every vector memory operation of
// this wavefront, stores included, has completed.
__device__ __forceinline__ void wait_stores_done() { __builtin_amdgcn_s_waitcnt(0x0F70); }

}  // namespace acrobat
