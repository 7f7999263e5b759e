// Device-side building blocks of the bandwidth-bound streaming kernels (decode attention and
// decode-shape round scores): the per-workgroup table of round segments, the lane layout that
// reads K/V rows with full 16-byte-per-lane coalescing, and the wavefront-level reductions.
//
// Lane layout inside a 64-wide wavefront: the wave is four rows of 16 lanes.  Row `grp` works on
// one token at a time and lane `sub` of the row owns d/16 consecutive channels of that token, so
// one load instruction of the wave covers four consecutive token rows (1 KB for bf16, d = 128).
// A dot product is finished with four DPP adds inside the 16-lane row; nothing goes through LDS.
#pragma once

#include "common.hpp"

namespace ra {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float as_f32(uint32_t x) { return __builtin_bit_cast(float, x); }
__device__ __forceinline__ uint32_t as_u32(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return as_f32((uint32_t)__builtin_amdgcn_update_dpp(0, (int)as_u32(v), CTRL, 0xf, 0xf, false));
}
// Sum over the 16 lanes of a DPP row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);  // row_half_mirror
    v += dpp_mov<0x140>(v);  // row_mirror
    return v;
}
// Maxima are ordinary float code on purpose.  The compiler inserts the wait states that the hardware leaves to
// software (a vector instruction that reads the result of a matrix-core product still in flight, a DPP or lane-swap
// instruction that reads a register just written), and it does so only for instructions it can see: an asm
// statement with v_max_f32 inside gets none.  Such a statement here once read the previous tile's logits (on a
// wave's first tile: whatever the registers held before) whenever the scheduler happened to put it within a few
// instructions of the products: a reference logit that was still valid but differed from launch to launch, and with
// it the last bits of the outputs.  The price is a few copies that quiet signalling NaNs in front of some maxima.
__device__ __forceinline__ float vmax(float a, float b) { return __builtin_fmaxf(a, b); }
// Reductions over the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48); every lane ends with the
// result.  v_permlane16_swap / v_permlane32_swap applied to two copies of a value hand each lane the values of
// both rows of a pair (of both halves of the wave), so the exchange stays in the vector ALU.
__device__ __forceinline__ float xrow_max4(float v) {
    auto a = __builtin_amdgcn_permlane16_swap(as_u32(v), as_u32(v), false, false);
    v = vmax(as_f32(a[0]), as_f32(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(as_u32(v), as_u32(v), false, false);
    return vmax(as_f32(b[0]), as_f32(b[1]));
}
__device__ __forceinline__ float xrow_sum4(float v) {
    auto a = __builtin_amdgcn_permlane16_swap(as_u32(v), as_u32(v), false, false);
    v = as_f32(a[0]) + as_f32(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(as_u32(v), as_u32(v), false, false);
    return as_f32(b[0]) + as_f32(b[1]);
}

// Element-type specific pieces.  A lane's share of one K or V row is WORDS 32-bit words.
struct F32 {};
struct BF16 {};
template <typename T, int EPL>
struct RowOps;

template <int EPL>
struct RowOps<F32, EPL> {
    static constexpr int WORDS = EPL;
    static constexpr int ELEM_BYTES = 4;
    __device__ static __forceinline__ float dot(const uint32_t* k, const uint32_t* q) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < WORDS; ++e) acc = __builtin_fmaf(as_f32(k[e]), as_f32(q[e]), acc);
        return acc;
    }
    __device__ static __forceinline__ void widen(const uint32_t* w, float* f) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) f[e] = as_f32(w[e]);
    }
};

template <int EPL>
struct RowOps<BF16, EPL> {
    static constexpr int WORDS = EPL / 2;
    static constexpr int ELEM_BYTES = 2;
    // Both operands are bf16, so every product is exact in fp32; accumulation is fp32.
    __device__ static __forceinline__ float dot(const uint32_t* k, const uint32_t* q) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < WORDS; ++e)
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k[e]), __builtin_bit_cast(bf16x2_t, q[e]),
                                                  acc, false);
        return acc;
    }
    __device__ static __forceinline__ void widen(const uint32_t* w, float* f) {
#pragma unroll
        for (int e = 0; e < WORDS; ++e) {
            f[2 * e] = as_f32(w[e] << 16);
            f[2 * e + 1] = as_f32(w[e] & 0xffff0000u);
        }
    }
};

// Loads of data that a kernel reads exactly once, marked non-temporal so that the lines do not displace anything
// in the caches on their way through.  It pays where one load instruction of a wave covers whole cache lines: a
// plain read of 4 GiB reaches 7.0-7.1 TB/s this way against 5.9-6.2 TB/s with ordinary loads on the same MI355X (each
// wave streaming its own span, 16- or 8-byte loads, 512 or 1024 contiguous bytes per instruction), and the decode
// kernel's value tiles, which have that shape, took it from 212 to 194 microseconds on the large paged workload.
// It does not pay for key tiles read in the operand layout of the matrix cores (16 rows x 64 bytes per instruction,
// two instructions to a cache line): no change in the decode kernel, 738 -> 878 microseconds in the score kernel, which
// reads nothing else.  The score kernel therefore loads its keys as whole rows (four rows, eight cache lines per
// instruction) and turns them into the operand layout through LDS: 738 -> 732 microseconds for itself, and the
// kernels that follow find their tables still in the caches (decode at 6 % kept 95 -> 85 microseconds, the whole
// small-batch step 70 -> 66).  And the hint must not sit behind a run-time condition: written as `flag ? load_once(p) : *p`
// the decode kernel ran at 320 instead of 212 microseconds (the loads of a tile then sit in separate branches, and
// the two tiles the kernel keeps in flight no longer overlap).
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_once(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 load_once(const uint2* p) {
    const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
    return make_uint2(v.x, v.y);
}

template <int WORDS>
struct Frag {
    uint32_t w[WORDS];
};

template <int WORDS>
__device__ __forceinline__ Frag<WORDS> load_frag(const char* p) {
    Frag<WORDS> f;
    if constexpr (WORDS == 2) {
        uint2 t = *reinterpret_cast<const uint2*>(p);
        f.w[0] = t.x;
        f.w[1] = t.y;
    } else {
#pragma unroll
        for (int i = 0; i < WORDS / 4; ++i) {
            uint4 t = reinterpret_cast<const uint4*>(p)[i];
            f.w[4 * i + 0] = t.x;
            f.w[4 * i + 1] = t.y;
            f.w[4 * i + 2] = t.z;
            f.w[4 * i + 3] = t.w;
        }
    }
    return f;
}

// ---- per-workgroup table of the round segments it may touch ------------------------------------
// slot i < n_hist is a history round, slot n_hist (if present) is the current round.  `cum` is the
// exclusive prefix sum of the segments' unit counts (a unit = 16 tokens, never crossing a segment).
struct SlotTable {
    long long* off_k;  // [cap]   segment start: tokens (contiguous) or block-table slots (paged)
    long long* off_v;  // [cap]
    int* len;          // [cap]
    int* cum;          // [cap + 1]
    __host__ __device__ static size_t bytes(int cap) { return (size_t)cap * 24 + 4; }
    __device__ void carve(char* smem, int cap) {
        off_k = reinterpret_cast<long long*>(smem);
        off_v = off_k + cap;
        len = reinterpret_cast<int*>(off_v + cap);
        cum = len + cap;
    }
};

// The table is built once per call and sequence by a small planning kernel and kept in global memory
// (header, then the four arrays with `cap` entries each, cum with cap + 1); the streaming kernels
// copy it to LDS with independent loads, so their workgroups start after a single memory round trip.
struct PlanHeader {
    int n_slots, n_hist, U, S_eff;  // U = total work units, S_eff = pieces the sequence is cut into
};
__host__ __device__ inline size_t plan_stride(int cap) { return (sizeof(PlanHeader) + SlotTable::bytes(cap) + 15) & ~(size_t)15; }

__device__ __forceinline__ PlanHeader load_plan(const char* plan_b, int cap, SlotTable& tab) {
    const PlanHeader hdr = *reinterpret_cast<const PlanHeader*>(plan_b);
    const long long* g_off_k = reinterpret_cast<const long long*>(plan_b + sizeof(PlanHeader));
    const long long* g_off_v = g_off_k + cap;
    const int* g_len = reinterpret_cast<const int*>(g_off_v + cap);
    const int* g_cum = g_len + cap;
    for (int i = threadIdx.x; i < cap; i += blockDim.x) {  // entries past n_slots are zero and unused
        tab.off_k[i] = g_off_k[i];
        tab.off_v[i] = g_off_v[i];
        tab.len[i] = g_len[i];
        tab.cum[i] = g_cum[i];
    }
    if (threadIdx.x == 0) tab.cum[cap] = g_cum[cap];
    return hdr;
}

// Exclusive prefix sum, in place, of cum[0..n) by the first wavefront; cum[n] receives the total.
// Must be called by all threads of the workgroup (it synchronises).
__device__ inline void exclusive_scan_units(int* cum, int n) {
    __syncthreads();
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const int per = (n + 63) >> 6;
        const int base = lane * per;
        int sum = 0;
        for (int j = 0; j < per; ++j)
            if (base + j < n) sum += cum[base + j];
        int incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int t = __shfl_up(incl, off, 64);
            if (lane >= off) incl += t;
        }
        int excl = incl - sum;
        for (int j = 0; j < per; ++j)
            if (base + j < n) {
                int u = cum[base + j];
                cum[base + j] = excl;
                excl += u;
            }
        if (lane == 63) cum[n] = incl;
    }
    __syncthreads();
}

// ---- loads from global memory straight into LDS -----------------------------------------------------
typedef void __attribute__((address_space(3)))* lptr_t;
// 16 bytes per lane from global memory straight into LDS (global_load_lds_dwordx4): lane L's piece lands at
// lds + 16 * L, `lds` being an LDS byte address that is the same in all lanes (it travels in M0).  Written as
// instructions of their own because the compiler, given its builtin for them, makes every later LDS read wait for
// the load to land (it cannot tell the two tile buffers apart), which exposes the whole memory latency once per
// tile (measured: 180 against 157 microseconds); here the one wait sits where it belongs, before the barrier that
// publishes the buffer (wait_for_direct_loads).  The compiler's own vector-memory counts do not see these loads,
// which can only make one of its waits longer, never shorter: loads complete in order.
// An asm statement is opaque to the compiler's hazard handling, so the wait states the hardware leaves to software
// are written out here: a scalar write of M0 needs one before an instruction that takes its LDS address from M0
// (the compiler puts the same s_nop behind its own M0 writes), and an SGPR written by a vector instruction
// (v_readfirstlane, or v_readlane when the compiler reloads a spilled SGPR) needs five before a vector-memory
// instruction reads it as its base address: the form with a uniform base therefore waits s_nop 3, which with the
// M0 write makes five whatever came right before the statement.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // M0 is named as clobbered; the compiler sets it anew before each of its own uses
__device__ __forceinline__ void load_to_lds(const void* src, unsigned lds) {  // per-lane 64-bit address
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds) : "memory", "m0");
}
__device__ __forceinline__ void load_to_lds(const char* base, unsigned off, unsigned lds) {  // uniform base + lane offset
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 3\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(base), "s"(lds) : "memory", "m0");
}
// s_waitcnt vmcnt(0) (the other counters at their maxima: expcnt 7, lgkmcnt 15)
__device__ __forceinline__ void wait_for_direct_loads() { __builtin_amdgcn_s_waitcnt(0x0f70); }
// The same wait, for a load that is issued only on some paths and used after they meet.  Left to the compiler, the
// wait lands after the join and is a wait for everything (with a conditional load in between, the number of younger
// loads is no constant), on every pass; written into the branch, right behind the load, it is paid only there.
__device__ __forceinline__ void wait_for_loads_so_far() { __builtin_amdgcn_s_waitcnt(0x0f70); }
#pragma clang diagnostic pop

// ---- balanced schedule of a whole batch ------------------------------------------------------------
// Every workgroup of a persistent attention launch derives the same schedule from the per-sequence
// unit counts U_b the planning kernel left in the plan headers: sequence b is cut into
//   n_b = clamp(ceil(U_b / T), 1, S)   pieces,   T = max(min_units, ceil(sum_b U_b / slots)),
// so that pieces have about equal size whatever the selection sizes are, and the batch has about
// `slots` pieces in total.  sU[b] = U_b, sps = exclusive prefix of n_b (sps[B] = number of pieces).
// Must be called by all threads of the workgroup.
// Same, from unit counts already in sU[0..B) (written by all threads before the call, no barrier needed).
__device__ inline int schedule_from_counts(int B, int S, int min_units, long long slots, int* sU, int* sps);

__device__ inline int build_schedule(const char* plan, int cap, int B, int S, int min_units, long long slots,
                                     int* sU, int* sps) {
    const size_t stride = plan_stride(cap);
    for (int b = threadIdx.x; b < B; b += blockDim.x)
        sU[b] = reinterpret_cast<const PlanHeader*>(plan + (size_t)b * stride)->U;
    return schedule_from_counts(B, S, min_units, slots, sU, sps);
}

__device__ inline int schedule_from_counts(int B, int S, int min_units, long long slots, int* sU, int* sps) {
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) sps[b] = sU[b];
    exclusive_scan_units(sps, B);
    const long long total = sps[B];
    long long T = (total + slots - 1) / (slots > 0 ? slots : 1);
    if (T < min_units) T = min_units;
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        long long nb = (sU[b] + T - 1) / T;
        sps[b] = (int)(nb < 1 ? 1 : (nb > S ? S : nb));
    }
    exclusive_scan_units(sps, B);
    return sps[B];
}

// Largest slot with cum[slot] <= u, for 0 <= u < cum[n].
template <typename T>
__device__ __forceinline__ int find_slot(const T* cum, int n, T u) {
    int lo = 0, hi = n;  // invariant: cum[lo] <= u < cum[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (cum[mid] <= u) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace ra
