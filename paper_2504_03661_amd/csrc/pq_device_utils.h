// Device-side helpers shared by the decode kernels (gfx950): LDS pointer types, wave-wide
// reductions by DPP, the LDS work counter, the code-block loader.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x2 lds_u32x2;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

constexpr float NEG_BIG = -1.0e30f;  // "no score yet": finite so that differences stay finite

template <typename T> struct elem;
template <> struct elem<__half> {
    static __device__ float ld(const void *p, int64_t i) { return __half2float(((const __half *)p)[i]); }
};
template <> struct elem<float> {
    static __device__ float ld(const void *p, int64_t i) { return ((const float *)p)[i]; }
};

template <int CTRL> __device__ inline float dpp_move(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// maximum over the 64 lanes, same value returned to every lane (wave-uniform)
__device__ inline float wave_max(float x)
{
    x = fmaxf(x, dpp_move<0xB1>(x));   // quad_perm [1,0,3,2]
    x = fmaxf(x, dpp_move<0x4E>(x));   // quad_perm [2,3,0,1]
    x = fmaxf(x, dpp_move<0x141>(x));  // row_half_mirror
    x = fmaxf(x, dpp_move<0x140>(x));  // row_mirror
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// sum over the 64 lanes in a fixed order, wave-uniform result
__device__ inline float wave_sum(float x)
{
    x += dpp_move<0xB1>(x);
    x += dpp_move<0x4E>(x);
    x += dpp_move<0x141>(x);
    x += dpp_move<0x140>(x);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 48));
    return (r0 + r1) + (r2 + r3);
}

// Zero in a vector register, opaque to the compiler: added to a wave-uniform index it keeps a
// load a vector load that can stay in flight, where the compiler would otherwise issue a scalar
// read and wait for it at once.
__device__ inline int lane_zero()
{
    int z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

// ---------------------------------------------------------------------------------------------------
// Exchange of split partials between the workgroups of one output row.  Every workgroup of the row
//   1. publishes its partial with relaxed atomic stores at agent scope: on gfx942 / gfx950 the compiler emits
//      these as write-through stores (sc1) that are performed in the memory all XCDs share, not left dirty in
//      the XCD's own L2;
//   2. waits until those stores have completed (s_waitcnt vmcnt(0): the counter falls only when the memory
//      system has acknowledged the store at the scope it was issued with);
//   3. takes a ticket: a relaxed atomic add at agent scope on the row's counter — all of a row's tickets are
//      totally ordered on that one location;
// and the workgroup that draws the last ticket
//   4. loads all partials with relaxed atomic loads at agent scope (sc1: not served from a line its own L2
//      might hold), issued after its ticket has returned, merges them and puts the counter back to zero.
// Steps 2 and 4 stand where a release fence and an acquire fence would stand.  The code sequences the AMDGPU
// backend documents for those fences at agent scope are "write back the L2, then s_waitcnt vmcnt(0)" and
// "invalidate the caches"; the write-back and the invalidate exist for earlier plain stores and later plain
// loads, which may live in the non-coherent L2 — every store and load of this exchange is itself an
// agent-scope atomic access and bypasses that cache, so only the wait remains.  (The fences were measured:
// about 1.8 us per workgroup for the release, 3 us with the acquire, on a 33 us kernel.)  The counter is put
// back by the one workgroup that has seen every other ticket of the launch; nobody touches it again before
// the next launch, which the kernel boundary orders after this one: calls on a context must be
// stream-ordered.
// ---------------------------------------------------------------------------------------------------
__device__ inline void publish(float *p, float x, float y)
{
    const uint64_t bits = (uint64_t)__float_as_uint(x) | ((uint64_t)__float_as_uint(y) << 32);
    __hip_atomic_store((uint64_t *)p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// all stores this wavefront has issued are complete
__device__ inline void publish_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ inline float2 fetch(const float *p)
{
    const uint64_t bits = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((uint32_t)bits), __uint_as_float((uint32_t)(bits >> 32)));
}

__device__ inline void ticket_reset(unsigned int *ticket)
{
    __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline uint32_t comp(const uint4 &v, int r)
{
    return r == 0 ? v.x : r == 1 ? v.y : r == 2 ? v.z : v.w;
}

// Takes the next unowned block of the workgroup's split from a counter in LDS.  One lane adds
// 1; the execution mask is narrowed to that lane inside the assembly block, so no branch
// appears in the scan loop (the compiler's wait-count analysis turns conservative at
// control-flow joins) and the atomic unit serves one lane, not sixty-four on one address.
__device__ inline int lds_grab(uint32_t lds_addr)
{
    uint32_t r;
    uint64_t saved_exec;
    const uint32_t one = 1;
    asm volatile("s_mov_b64 %1, exec\n\t"
                 "s_mov_b64 exec, 1\n\t"
                 "ds_add_rtn_u32 %0, %2, %3\n\t"
                 "s_mov_b64 exec, %1\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r), "=&s"(saved_exec)
                 : "v"(lds_addr), "v"(one)
                 : "memory");
    return __builtin_amdgcn_readfirstlane((int)r);
}


// Which (unit, split) a workgroup owns; unit = a (sequence, head or head group).  Workgroups are dealt round-robin
// to the 8 XCDs; they are un-dealt so that all splits of a unit — and neighbouring units: the heads of a KV group,
// the same KV head of other sequences — sit on one XCD and share its L2.  Where every XCD gets whole units, its
// workgroups are numbered SPLIT-major: the first splits of all its units come first.  With unit-major numbering the
// live workgroups of an oversubscribed grid whose surplus splits leave at once (8 launched splits, 1 live) sit 8
// apart, and the dispatcher, which deals consecutive workgroups to the shader engines in turn, put them all on one
// engine's compute units: 8 x 32 heads x 32K with 8 launched splits took 483 us instead of 165.
__device__ inline void unit_and_split(uint32_t bid, uint32_t grid, uint32_t S, uint32_t &unit, uint32_t &split)
{
    const uint32_t n_units = grid / S;
    if ((n_units & 7u) == 0) {
        const uint32_t per_xcd = n_units >> 3, xcd = bid & 7u, local = bid >> 3;
        split = local / per_xcd;
        uint32_t j = local - split * per_xcd;
        // ... and where the XCD's unit count is a power of two, the units are visited in a scrambled order (low 3
        // bits XOR the next 3): the long sequences of a ragged batch sit at a fixed stride in the unit numbering
        // (unit = head x batch + sequence), which met the same engine every time
        if (per_xcd >= 16u && (per_xcd & (per_xcd - 1u)) == 0u)
            j ^= (j >> 3) & 7u;
        unit = xcd * per_xcd + j;
    } else {
        const uint32_t logical = (grid & 7u) == 0 ? (bid & 7u) * (grid >> 3) + (bid >> 3) : bid;
        unit = logical / S;
        split = logical - unit * S;
    }
}

// Sum over the batch of (cached tokens + recent rows), each clamped like the sequence's own lengths: lane l adds
// sequences l, l + 64, ...; the loads go out with the workgroup's own lengths.  Only batches need it (the live
// split count of a sequence follows its share of the batch's work).
// (a float: 64 sequences of 2^24 tokens already exceed an int, and every workgroup adds in the same order)
template <typename A> __device__ inline float batch_work_lane(const A &a, bool has_recent, int lane)
{
    float w = 0.f;
    for (int b2 = lane; b2 < a.B; b2 += 64) {
        int n2 = a.ctx_len[b2];
        n2 = n2 < 0 ? 0 : (n2 > a.max_context ? a.max_context : n2);
        int r2 = has_recent ? a.recent_len[b2] : 0;
        r2 = r2 < 0 ? 0 : (r2 > a.max_recent ? a.max_recent : r2);
        w += (float)(n2 + r2);
    }
    return w;
}

// The live splits of a sequence in a batch: no more than its share of the compute units — n_cu x (its work) /
// (workgroups per split x the batch's work) — so that in an oversubscribed grid (explicit n_splits on a large
// batch: a cache that must serve ragged batches) the splits go to the long sequences and a batch of equal lengths
// runs one split per sequence, as if none had been asked for.  Every workgroup of the row computes the same number
// from the same lengths.
template <typename A> __device__ inline uint32_t live_split_cap(const A &a, int units, int own_work, float w_lane)
{
    float total = w_lane;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        total += __shfl_xor(total, o);
    total = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(total)));
    const float share = (float)a.n_cu * (float)own_work / ((float)units * (total > 0.f ? total : 1.f));
    return share >= 1.f ? (share < 64.f ? (uint32_t)share : 64u) : 1u;
}

// 16 code bytes of one lane.  Codes that are read once per launch are loaded with the
// non-temporal hint: the stream then does not displace the tables and each other's lines in L2
// and the memory-side cache, and HBM delivers markedly more (measured on the 8 x 32 heads x 32K
// workload: 192 us with plain loads, 164 us with the hint; a kernel that only reads shows the same).
template <bool READ_ONCE> __device__ inline uint4 load_codes(const u32x4 *p)
{
    const u32x4 t = READ_ONCE ? __builtin_nontemporal_load(p) : *p;
    return make_uint4(t.x, t.y, t.z, t.w);
}

// (d, c) <- the smaller of (d, c) and (od, oc) in the order (distance, index)
__device__ inline void argmin_take(double &d, int &c, const double od, const int oc)
{
    const bool take = od < d || (od == d && oc < c);
    d = take ? od : d;
    c = take ? oc : c;
}

template <int CTRL> __device__ inline void argmin_dpp(double &d, int &c)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(d), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(d), CTRL, 0xf, 0xf, true);
    const int oc = __builtin_amdgcn_update_dpp(0, c, CTRL, 0xf, 0xf, true);
    argmin_take(d, c, __hiloint2double(hi, lo), oc);
}

// minimum over the 64 lanes, the same in every lane: lane exchanges inside a row of 16 by DPP (vector-ALU
// speed; a shuffle goes through the LDS crossbar), then the 4 rows' results
__device__ inline void wave_argmin(double &d, int &c)
{
    argmin_dpp<0xB1>(d, c);   // quad_perm [1,0,3,2]
    argmin_dpp<0x4E>(d, c);   // quad_perm [2,3,0,1]
    argmin_dpp<0x141>(d, c);  // row_half_mirror
    argmin_dpp<0x140>(d, c);  // row_mirror
    double rd[4];
    int rc[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        rd[r] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(d), 16 * r),
                                 __builtin_amdgcn_readlane(__double2loint(d), 16 * r));
        rc[r] = __builtin_amdgcn_readlane(c, 16 * r);
    }
    d = rd[0];
    c = rc[0];
#pragma unroll
    for (int r = 1; r < 4; ++r)
        argmin_take(d, c, rd[r], rc[r]);
}


}  // namespace
