// Device-side helpers shared by the libpk kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pk.h"

namespace pk {

#define PK_LDS __attribute__((address_space(3)))
#define PK_GLOBAL __attribute__((address_space(1)))

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// s_waitcnt immediate for "vmcnt(0)" with the other counters left alone (gfx9 encoding:
// vmcnt = bits [3:0] and [15:14], expcnt = [6:4], lgkmcnt = [11:8]).
#define PK_WAIT_VMCNT0 0x0F70

constexpr uint32_t kWallClockTicksPerUs = 100;   // wall_clock64() runs at 100 MHz

// Paper appendix C, `signal`: make the data written before this call visible at device scope, then
// publish the flag.  One producer owns each flag, so a store of the epoch replaces the atomic add.
__device__ __forceinline__ void flag_signal(uint32_t* flag, uint32_t epoch) {
    __hip_atomic_store(flag, epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ bool flag_ready(const uint32_t* flag, uint32_t epoch) {
    uint32_t v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return (int32_t)(v - epoch) >= 0;
}

// Paper appendix C, `wait`: poll with relaxed loads until the flag reaches the expected value.
// Bounded: returns false once `timeout_ticks` of the 100 MHz wall clock have passed.
// The caller issues the acquire fence (after its workgroup barrier).
__device__ __forceinline__ bool flag_wait(const uint32_t* flag, uint32_t epoch, uint64_t timeout_ticks) {
    if (flag_ready(flag, epoch)) return true;
    const uint64_t t0 = wall_clock64();
    for (;;) {
        __builtin_amdgcn_s_sleep(8);
        if (flag_ready(flag, epoch)) return true;
        if (wall_clock64() - t0 > timeout_ticks) return false;
    }
}

__device__ __forceinline__ void report_timeout(uint32_t* status, uint32_t index, uint32_t phase) {
    if (atomicCAS(&status[0], 0u, (uint32_t)PK_ERR_TIMEOUT) == 0u) {
        status[1] = index;
        status[2] = phase;
    }
}

// 16-byte-per-lane direct-to-LDS load: lane l's 16 bytes from (sbase + voff) land at LDS byte address lds_addr + 16*l.
// Written as inline assembly on purpose: for the builtin form the compiler cannot tell which LDS bytes the load
// writes and makes every later LDS read wait for it (vmcnt(0)), which serialises the pipeline.  The kernel waits
// for these loads itself (s_waitcnt vmcnt + workgroup barrier) before any wave reads what they wrote.
__device__ __forceinline__ void dma_load16(const char* sbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "m0");
}

// 16-byte store that writes through to memory (system-coherent cache policy, streaming).  Together with an
// explicit wait for the stores to complete (s_waitcnt vmcnt(0)) this is the "release" half of a signal without
// the L2 write-back of a release fence: nothing dirty is left behind in the XCD's L2.  Inline assembly because
// the cache-policy bits are not reachable from a plain store.
__device__ __forceinline__ void store16_writethrough(void* p, i32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(p), "v"(v) : "memory");
}

// Publish a flag whose data was written with store16_writethrough and has completed (every wave waited on its
// stores and passed a workgroup barrier): a relaxed device-scope store is then enough.
__device__ __forceinline__ void flag_publish(uint32_t* flag, uint32_t epoch) {
    __hip_atomic_store(flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void acquire_agent() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }
__device__ __forceinline__ void release_agent() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }

}  // namespace pk
