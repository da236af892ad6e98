// Cross-workgroup hand-off without cache-wide fences.
//
// The split-K and split-KV fix-ups pass small partial results between workgroups that may run
// on different XCDs (each XCD has its own L2).  A full agent-scope fence would write back and
// invalidate a whole L2 per call.  Instead the partial data itself is moved with agent-scope
// (device-coherent) stores and loads, the producer waits until its stores have completed before
// it bumps the arrival counter (a device-scope atomic), and the consumer reads only after it has
// seen the final count.  No spinning anywhere: the last workgroup to arrive does the merge.
//
// What this rests on: the atomics are relaxed (no release on the counter, no acquire before the partial loads);
// the order comes from the explicit wait for the stores' completion (wait_vmem_done) in front of the counter
// increment, from the barrier between the increment's return and the partial loads, and from agent-scope
// accesses going past the per-XCD L2s.  That is how hipcc of ROCm 7.2 (AMD clang 22.0.0git, roc-7.2.0) lowers these builtins for
// gfx950; a compiler that moved the loads above the barrier or dropped the scope bits would break it without a
// diagnostic.  The guard is tests/test_gpu_bf16.py::test_fresh_contexts_give_identical_bits (identical bits from
// separate contexts through every K-slice and key-split hand-off) together with the oracle parity tests.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ inline void st_agent_f32(float* p, float v) {
    __hip_atomic_store((uint32_t*)p, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float ld_agent_f32(const float* p) {
    return __uint_as_float(__hip_atomic_load((const uint32_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ inline void st_agent_i32(int32_t* p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline int32_t arrive_agent(int32_t* counter) {
    return __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 8 bytes per lane with the same agent scope (the widest the compiler's atomics offer; it keeps the wait
// counts itself, unlike a hand-written 16-byte load, whose destination registers it would feel free to move
// before the data has arrived)
__device__ inline void st_agent_f32x2(float* p, float a, float b) {
    __hip_atomic_store((uint64_t*)p, (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void ld_agent_f32x2(const float* p, float& a, float& b) {
    const uint64_t v = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    a = __uint_as_float((uint32_t)v); b = __uint_as_float((uint32_t)(v >> 32));
}
// all earlier vector-memory operations of this wave (the agent-scope stores above) have completed
__device__ inline void wait_vmem_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
