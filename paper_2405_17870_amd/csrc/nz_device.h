// Device code of the allreduce reduction engine (gfx950, wave64): the fused
// N-way reduce + broadcast, the ring reduce-scatter / allgather step, the
// direct allgather and the segment copy, with the argument blocks they read.
// Included by nz_host.hip only.
//
// Nezha (arXiv 2405.17870): the aggregation phase of the allreduce (Sec. 4.2),
// run per rail on that rail's slice (Sec. 3.4, 4.1), with the ring schedule of
// Sec. 2.1.1 / Eq. 1, and the staging copies of Sec. 3.2.
//
// Everything here is bound by HBM bandwidth (about 0.25 flop per byte), so
// there is no matrix-core work: the kernels are built around 16-byte
// coalesced accesses on a 16-byte grid that is common to every buffer (all
// bases are 256-byte aligned and all nodes use the same element offsets),
// per-element handling of the few bytes where a segment boundary falls inside
// a 16-byte vector, and a cross-lane exchange only in the copy kernel, the one
// place where source and destination can be misaligned relative to each other.
//
// All per-call tables (node pointers, rail geometry, copy descriptors) travel
// in the kernel-argument block: no device workspace, no allocation, no
// host-to-device copy, and a call can be captured in a HIP graph as it is.
#ifndef NZ_DEVICE_H
#define NZ_DEVICE_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "nz_internal.h"

namespace {

typedef uint32_t u32;
typedef uint64_t u64;

constexpr int kThreads = 256;  // four wave64 per workgroup

// Kernel-argument blocks are read where they already are: in the kernarg
// segment (constant address space), through scalar loads, with no private copy
// even when a table in them is indexed with a run-time value.  Each kernel has
// its argument struct as its only parameter, so the struct starts the segment.
#define NZ_KARG __attribute__((address_space(4)))
#define NZ_GLOBAL __attribute__((address_space(1)))

template <class A>
__device__ __forceinline__ const NZ_KARG A &kernel_args()
{
    return *(const NZ_KARG A *)__builtin_amdgcn_kernarg_segment_ptr();
}

// ---------------------------------------------------------------------------
// Rail / segment geometry, as seen by the kernels
// ---------------------------------------------------------------------------

// Everything a workgroup needs to find its (rail, segment, tile).  Segment j
// of rail k covers elements [off[k] + j*q[k] + min(j, rem[k]), +q[k] + (j < rem[k])).
struct RailGeom {
    u64 off[NZ_MAX_RAILS + 1];   // rail boundaries, in elements
    u64 q[NZ_MAX_RAILS];         // short segment length of the rail
    u32 rem[NZ_MAX_RAILS];       // number of segments that are one element longer
    u32 tile0[NZ_MAX_RAILS + 1]; // first workgroup of each rail
    u32 tps[NZ_MAX_RAILS];       // workgroups reserved per segment of the rail
    u32 n_rails;
    u32 n_nodes;
    u64 win_off, win_len;        // the piece of every segment this launch works on (elements)
};

// Work of one workgroup: a run of 16-byte vectors of one segment.
struct SegTile {
    u64 b0, b1;         // byte range of the whole segment
    u64 vec_lo, vec_hi; // this workgroup's vectors (global 16-byte vector indices), may be empty
    u64 tile_base;      // first vector of the aligned tile the run lies in
};

// Workgroup number -> (rail, index, tile): a rail's workgroups walk through
// one index's tiles before the next index.
__device__ __forceinline__ void decode_block(const NZ_KARG RailGeom &g, u32 block, u32 &rail, u32 &idx,
                                             u32 &tile)
{
    // tile0 never decreases, so the rail is the number of later rails that start at or before
    // this workgroup; counted without a loop so that the loads do not wait for one another.
    u32 k = 0;
#pragma unroll
    for (u32 i = 1; i < NZ_MAX_RAILS; ++i) k += (i < g.n_rails && block >= g.tile0[i]) ? 1u : 0u;
    const u32 local = block - g.tile0[k];
    rail = k;
    idx = local / g.tps[k];
    tile = local - idx * g.tps[k];
}

// Tiles lie on a grid of TILE_VECS vectors that is global to the buffers, so a
// workgroup's accesses are aligned to the tile size wherever the segment
// boundary is; the first and last tile of a segment are simply shorter.
template <int TILE_VECS>
__device__ __forceinline__ SegTile segment_tile(const NZ_KARG RailGeom &g, u32 rail, u32 seg, u32 tile,
                                                u32 elem_shift, u64 win_off, u64 win_len)
{
    SegTile t;
    const u32 rem = g.rem[rail];
    u64 beg = g.off[rail] + seg * g.q[rail] + (seg < rem ? seg : rem);
    u64 len = g.q[rail] + (seg < rem ? 1u : 0u);
    const u64 skip = len < win_off ? len : win_off;
    beg += skip;
    len = (len - skip) < win_len ? (len - skip) : win_len;
    t.b0 = beg << elem_shift;
    t.b1 = (beg + len) << elem_shift;
    const u64 v0 = t.b0 >> 4;
    const u64 v1 = (t.b1 + 15) >> 4;
    t.tile_base = (v0 / TILE_VECS + tile) * TILE_VECS;
    t.vec_lo = t.tile_base > v0 ? t.tile_base : v0;
    const u64 end = t.tile_base + TILE_VECS;
    t.vec_hi = end < v1 ? end : v1;
    if (len == 0) t.vec_hi = t.vec_lo;
    return t;
}

// The same for the window the launch as a whole works on.
template <int TILE_VECS>
__device__ __forceinline__ SegTile segment_tile(const NZ_KARG RailGeom &g, u32 rail, u32 seg, u32 tile,
                                                u32 elem_shift)
{
    return segment_tile<TILE_VECS>(g, rail, seg, tile, elem_shift, g.win_off, g.win_len);
}

// ---------------------------------------------------------------------------
// Element types
// ---------------------------------------------------------------------------

typedef u32 vec16 __attribute__((ext_vector_type(4)));  // one 16-byte access
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ vec16 vec16_of(u32 x, u32 y, u32 z, u32 w)
{
    vec16 v = {x, y, z, w};
    return v;
}
__device__ __forceinline__ float as_f32(u32 u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ u32 as_u32(float f) { return __builtin_bit_cast(u32, f); }

// Each type describes how a 16-byte vector (four 32-bit words) and a single
// element are widened to the accumulator type and narrowed back.  Narrowing
// rounds to nearest, ties to even, once.
struct TF32 {
    typedef float acc_t;
    typedef u32 elem_t;
    static constexpr int kShift = 2, kLanes = 4;
    static __device__ __forceinline__ void widen(const vec16 &v, acc_t (&a)[kLanes])
    {
        a[0] = as_f32(v.x); a[1] = as_f32(v.y); a[2] = as_f32(v.z); a[3] = as_f32(v.w);
    }
    static __device__ __forceinline__ vec16 narrow(const acc_t (&a)[kLanes])
    {
        return vec16_of(as_u32(a[0]), as_u32(a[1]), as_u32(a[2]), as_u32(a[3]));
    }
    static __device__ __forceinline__ acc_t lane(const vec16 &v, int l) { return as_f32(v[l]); }
    static __device__ __forceinline__ acc_t widen1(elem_t e) { return as_f32(e); }
    static __device__ __forceinline__ elem_t narrow1(acc_t a) { return as_u32(a); }
};

struct TI32 {
    typedef u32 acc_t;  // wrapping two's-complement add
    typedef u32 elem_t;
    static constexpr int kShift = 2, kLanes = 4;
    static __device__ __forceinline__ void widen(const vec16 &v, acc_t (&a)[kLanes])
    {
        a[0] = v.x; a[1] = v.y; a[2] = v.z; a[3] = v.w;
    }
    static __device__ __forceinline__ vec16 narrow(const acc_t (&a)[kLanes])
    {
        return vec16_of(a[0], a[1], a[2], a[3]);
    }
    static __device__ __forceinline__ acc_t lane(const vec16 &v, int l) { return v[l]; }
    static __device__ __forceinline__ acc_t widen1(elem_t e) { return e; }
    static __device__ __forceinline__ elem_t narrow1(acc_t a) { return a; }
};

struct TBF16 {
    typedef float acc_t;
    typedef unsigned short elem_t;
    static constexpr int kShift = 1, kLanes = 8;
    // bfloat16 is the upper half of a binary32: widening is a shift or a mask.
    static __device__ __forceinline__ void widen(const vec16 &v, acc_t (&a)[kLanes])
    {
        a[0] = as_f32(v.x << 16); a[1] = as_f32(v.x & 0xffff0000u);
        a[2] = as_f32(v.y << 16); a[3] = as_f32(v.y & 0xffff0000u);
        a[4] = as_f32(v.z << 16); a[5] = as_f32(v.z & 0xffff0000u);
        a[6] = as_f32(v.w << 16); a[7] = as_f32(v.w & 0xffff0000u);
    }
    static __device__ __forceinline__ u32 pair(float lo, float hi)
    {
        f32x2 f = {lo, hi};
        return __builtin_bit_cast(u32, __builtin_convertvector(f, bf16x2));  // v_cvt_pk_bf16_f32
    }
    static __device__ __forceinline__ vec16 narrow(const acc_t (&a)[kLanes])
    {
        return vec16_of(pair(a[0], a[1]), pair(a[2], a[3]), pair(a[4], a[5]), pair(a[6], a[7]));
    }
    static __device__ __forceinline__ acc_t lane(const vec16 &v, int l)
    {
        return as_f32((l & 1) ? (v[l >> 1] & 0xffff0000u) : (v[l >> 1] << 16));
    }
    static __device__ __forceinline__ acc_t widen1(elem_t e) { return as_f32((u32)e << 16); }
    static __device__ __forceinline__ elem_t narrow1(acc_t a)
    {
        return __builtin_bit_cast(unsigned short, (__bf16)a);
    }
};

struct TF16 {
    typedef float acc_t;
    typedef unsigned short elem_t;
    static constexpr int kShift = 1, kLanes = 8;
    static __device__ __forceinline__ void widen2(u32 w, float &lo, float &hi)
    {
        f16x2 h = __builtin_bit_cast(f16x2, w);
        lo = (float)h.x;
        hi = (float)h.y;
    }
    static __device__ __forceinline__ void widen(const vec16 &v, acc_t (&a)[kLanes])
    {
        widen2(v.x, a[0], a[1]); widen2(v.y, a[2], a[3]);
        widen2(v.z, a[4], a[5]); widen2(v.w, a[6], a[7]);
    }
    static __device__ __forceinline__ u32 pair(float lo, float hi)
    {
        f16x2 h = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(u32, h);
    }
    static __device__ __forceinline__ vec16 narrow(const acc_t (&a)[kLanes])
    {
        return vec16_of(pair(a[0], a[1]), pair(a[2], a[3]), pair(a[4], a[5]), pair(a[6], a[7]));
    }
    static __device__ __forceinline__ acc_t lane(const vec16 &v, int l)
    {
        const u32 w = v[l >> 1];
        const unsigned short h = (unsigned short)((l & 1) ? (w >> 16) : (w & 0xffffu));
        return (float)__builtin_bit_cast(_Float16, h);
    }
    static __device__ __forceinline__ acc_t widen1(elem_t e)
    {
        return (float)__builtin_bit_cast(_Float16, e);
    }
    static __device__ __forceinline__ elem_t narrow1(acc_t a)
    {
        return __builtin_bit_cast(unsigned short, (_Float16)a);
    }
};

// A "packet" is what one thread carries per node: either a whole 16-byte
// vector (the body of a segment) or a single element (the few bytes where a
// segment boundary falls inside a vector).  Both go through the same
// summation code, so an element's sum does not depend on which path took it.
template <class T>
struct VecPacket {
    typedef vec16 raw_t;
    static constexpr int kLanes = T::kLanes;
    static __device__ __forceinline__ raw_t load(const void *base, u64 byte_off)
    {
        return __builtin_nontemporal_load(
            (const NZ_GLOBAL vec16 *)(static_cast<const char *>(base) + byte_off));
    }
    static __device__ __forceinline__ void store(void *base, u64 byte_off, const raw_t &v)
    {
        __builtin_nontemporal_store(v, (NZ_GLOBAL vec16 *)(static_cast<char *>(base) + byte_off));
    }
    // Ordinary (cache-allocating) forms, for data the next launch reads again.
    static __device__ __forceinline__ raw_t load_again(const void *base, u64 byte_off)
    {
        return *(const NZ_GLOBAL vec16 *)(static_cast<const char *>(base) + byte_off);
    }
    static __device__ __forceinline__ void store_for_reuse(void *base, u64 byte_off, const raw_t &v)
    {
        *(NZ_GLOBAL vec16 *)(static_cast<char *>(base) + byte_off) = v;
    }
    static __device__ __forceinline__ void widen(const raw_t &r, typename T::acc_t (&a)[kLanes])
    {
        T::widen(r, a);
    }
    // Lane l (a compile-time constant after unrolling) of the vector, widened.
    static __device__ __forceinline__ typename T::acc_t lane(const raw_t &r, int l)
    {
        return T::lane(r, l);
    }
    static __device__ __forceinline__ raw_t narrow(const typename T::acc_t (&a)[kLanes])
    {
        return T::narrow(a);
    }
};

template <class T>
struct ElemPacket {
    typedef typename T::elem_t raw_t;
    static constexpr int kLanes = 1;
    static __device__ __forceinline__ raw_t load(const void *base, u64 byte_off)
    {
        return *(const NZ_GLOBAL raw_t *)(static_cast<const char *>(base) + byte_off);
    }
    static __device__ __forceinline__ void store(void *base, u64 byte_off, const raw_t &v)
    {
        *(NZ_GLOBAL raw_t *)(static_cast<char *>(base) + byte_off) = v;
    }
    static __device__ __forceinline__ raw_t load_again(const void *base, u64 byte_off)
    {
        return load(base, byte_off);
    }
    static __device__ __forceinline__ void store_for_reuse(void *base, u64 byte_off, const raw_t &v)
    {
        store(base, byte_off, v);
    }
    static __device__ __forceinline__ void widen(const raw_t &r, typename T::acc_t (&a)[1])
    {
        a[0] = T::widen1(r);
    }
    static __device__ __forceinline__ typename T::acc_t lane(const raw_t &r, int) { return T::widen1(r); }
    static __device__ __forceinline__ raw_t narrow(const typename T::acc_t (&a)[1])
    {
        return T::narrow1(a[0]);
    }
};

// ---------------------------------------------------------------------------
// Fused N-way reduce + broadcast
// ---------------------------------------------------------------------------

// A table of node buffer addresses inside a kernel-argument block.
typedef const void *NodePtr;
typedef const NZ_KARG NodePtr *NodeTable;
typedef void *OutPtr;
typedef const NZ_KARG OutPtr *OutTable;

struct FusedArgs {
    RailGeom g;
    u32 n_out;       // distinct output buffers (broadcast form)
    u32 owner_only;  // reduce-scatter form: segment j is stored to out[(j - 1) mod N] alone
    const void *in[NZ_MAX_NODES];
    void *out[NZ_MAX_NODES];
};

// Sum of one packet position over all nodes, in a fixed order that depends on
// the node count alone:
//   - nodes are taken in blocks of eight consecutive indices; the values of a
//     block are added as a balanced binary tree (an operand that does not
//     exist is skipped, never replaced by zero);
//   - block sums go round-robin into four running sums (block b into b mod 4);
//   - the running sums are added as (s0 + s1) + (s2 + s3).
// With N <= 128 no value passes through more than 3 + 3 + 2 roundings, so the
// fp32 error stays below 8 * 2^-24 * sum|x|, and the eight loads of a block
// are independent and in flight together.
// Sum of a full block of eight nodes starting at node m0: a balanced tree.
template <class T, class P, bool CACHED>
__device__ __forceinline__ void block_sum8(NodeTable in, u32 m0, u64 byte_off,
                                           typename T::acc_t (&s)[P::kLanes])
{
    typename P::raw_t r[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        r[i] = CACHED ? P::load_again(in[m0 + i], byte_off) : P::load(in[m0 + i], byte_off);
#pragma unroll
    for (int l = 0; l < P::kLanes; ++l)
        s[l] = ((P::lane(r[0], l) + P::lane(r[1], l)) + (P::lane(r[2], l) + P::lane(r[3], l))) +
               ((P::lane(r[4], l) + P::lane(r[5], l)) + (P::lane(r[6], l) + P::lane(r[7], l)));
}

// Sum of a partial block of NB nodes (1 <= NB <= 7): the same tree with the
// missing leaves left out, and no load for them either.
template <class T, class P, bool CACHED, int NB>
__device__ __forceinline__ void block_sum_part(NodeTable in, u32 m0, u64 byte_off,
                                               typename T::acc_t (&s)[P::kLanes])
{
    typedef typename T::acc_t acc_t;
    typename P::raw_t r[7];
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        if (i < NB) r[i] = CACHED ? P::load_again(in[m0 + i], byte_off) : P::load(in[m0 + i], byte_off);
    }
#pragma unroll
    for (int l = 0; l < P::kLanes; ++l) {
        // r[i] with i >= NB is never read: each use below is guarded by the same comparison
        const acc_t p0 = NB > 1 ? P::lane(r[0], l) + P::lane(r[1 < NB ? 1 : 0], l) : P::lane(r[0], l);
        const acc_t p1 = NB > 3 ? P::lane(r[2], l) + P::lane(r[3 < NB ? 3 : 0], l) : P::lane(r[2 < NB ? 2 : 0], l);
        const acc_t p2 = NB > 5 ? P::lane(r[4], l) + P::lane(r[5 < NB ? 5 : 0], l) : P::lane(r[4 < NB ? 4 : 0], l);
        const acc_t p3 = P::lane(r[6 < NB ? 6 : 0], l);
        const acc_t lo = NB > 2 ? p0 + p1 : p0;
        const acc_t hi = NB > 6 ? p2 + p3 : p2;
        s[l] = NB > 4 ? lo + hi : lo;
    }
}

// The last, partial block of a sum (1 <= nb <= 7 nodes, the same for every
// thread of the launch).
template <class T, class P, bool CACHED>
__device__ __forceinline__ void block_sum_tail(NodeTable in, u32 m0, u32 nb, u64 byte_off,
                                               typename T::acc_t (&s)[P::kLanes])
{
    switch (nb) {
    case 1: block_sum_part<T, P, CACHED, 1>(in, m0, byte_off, s); break;
    case 2: block_sum_part<T, P, CACHED, 2>(in, m0, byte_off, s); break;
    case 3: block_sum_part<T, P, CACHED, 3>(in, m0, byte_off, s); break;
    case 4: block_sum_part<T, P, CACHED, 4>(in, m0, byte_off, s); break;
    case 5: block_sum_part<T, P, CACHED, 5>(in, m0, byte_off, s); break;
    case 6: block_sum_part<T, P, CACHED, 6>(in, m0, byte_off, s); break;
    default: block_sum_part<T, P, CACHED, 7>(in, m0, byte_off, s); break;
    }
}

// How many nodes a kernel instantiation is built for.  The order of additions
// is the same in all three; what differs is how many partial sums have to be
// kept, i.e. registers, i.e. waves per SIMD (a message small enough to be
// bound by latency, and the copy part of the staged kernel, want many).
enum NodeClass {
    kUpTo8 = 0,   // a single block: no running sums
    kUpTo32 = 1,  // at most four blocks: each running sum is one block sum, so the
                  // final tree (s0 + s1) + (s2 + s3) is built as the blocks arrive
    kAnyN = 2     // the general form
};

// One block's sum, full or partial: block number blk of n_full full blocks.
template <class T, class P, bool CACHED>
__device__ __forceinline__ void block_sum(NodeTable in, u32 blk, u32 n_full, u32 n_tail, u64 byte_off,
                                          typename T::acc_t (&s)[P::kLanes])
{
    if (blk < n_full)
        block_sum8<T, P, CACHED>(in, blk * 8, byte_off, s);
    else
        block_sum_tail<T, P, CACHED>(in, blk * 8, n_tail, byte_off, s);
}

// The sum at one packet position, narrowed to the storage type.  CACHED: the
// job is small enough to live in the last-level cache (the gradients were
// just written by the kernels before, the sums are read by the kernels after),
// so ordinary cache-allocating accesses are used instead of streaming ones.
template <class T, class P, int CLASS, bool CACHED>
__device__ __forceinline__ typename P::raw_t reduce_at(NodeTable in, u32 N, u64 byte_off)
{
    typedef typename T::acc_t acc_t;
    constexpr int L = P::kLanes;
    acc_t res[L];
    if (CLASS == kUpTo8) {
        if (N == 8)
            block_sum8<T, P, CACHED>(in, 0, byte_off, res);
        else
            block_sum_tail<T, P, CACHED>(in, 0, N, byte_off, res);
        return P::narrow(res);
    }
    if (CLASS == kUpTo32) {
        const u32 n_full = N >> 3, n_tail = N & 7u, n_blocks = n_full + (n_tail ? 1u : 0u);
        block_sum<T, P, CACHED>(in, 0, n_full, n_tail, byte_off, res);
        if (n_blocks > 1) {
            acc_t s[L];
            block_sum<T, P, CACHED>(in, 1, n_full, n_tail, byte_off, s);
#pragma unroll
            for (int l = 0; l < L; ++l) res[l] = res[l] + s[l];
        }
        if (n_blocks > 2) {
#pragma unroll
            for (int l = 0; l < L; ++l) asm volatile("" : "+v"(res[l]) : : "memory");
            acc_t u[L];
            block_sum<T, P, CACHED>(in, 2, n_full, n_tail, byte_off, u);
            if (n_blocks > 3) {
#pragma unroll
                for (int l = 0; l < L; ++l) asm volatile("" : "+v"(u[l]) : : "memory");
                acc_t s[L];
                block_sum<T, P, CACHED>(in, 3, n_full, n_tail, byte_off, s);
#pragma unroll
                for (int l = 0; l < L; ++l) u[l] = u[l] + s[l];
            }
#pragma unroll
            for (int l = 0; l < L; ++l) res[l] = res[l] + u[l];
        }
        return P::narrow(res);
    }
    const u32 n_full = N >> 3, n_tail = N & 7u;
    acc_t run[4][L];
    for (u32 b = 0; b < n_full; b += 4) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (b + c >= n_full) break;
            acc_t s[L];
            block_sum8<T, P, CACHED>(in, (b + c) * 8, byte_off, s);
#pragma unroll
            for (int l = 0; l < L; ++l) run[c][l] = (b == 0) ? s[l] : run[c][l] + s[l];
            // One block's eight loads in flight at a time: the running sum is
            // pinned here and no memory access may cross, otherwise the loads of
            // all four blocks are hoisted to the top, which triples the registers
            // and costs the waves per SIMD that the copy part of the staged
            // kernel needs.
#pragma unroll
            for (int l = 0; l < L; ++l) asm volatile("" : "+v"(run[c][l]) : : "memory");
        }
    }
    if (n_tail) {
        // The partial block is block number n_full: it goes to running sum n_full mod 4.
        acc_t s[L];
        block_sum_tail<T, P, CACHED>(in, n_full * 8, n_tail, byte_off, s);
        const u32 slot = n_full & 3u;
        const bool first = n_full < 4;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (slot == (u32)c) {
#pragma unroll
                for (int l = 0; l < L; ++l) run[c][l] = first ? s[l] : run[c][l] + s[l];
            }
    }
#pragma unroll
    for (int l = 0; l < L; ++l) {
        acc_t t = run[0][l];
        if (N > 8) t = t + run[1][l];
        if (N > 16) {
            acc_t u = run[2][l];
            if (N > 24) u = u + run[3][l];
            t = t + u;
        }
        res[l] = t;
    }
    return P::narrow(res);
}

// Store one reduced packet to out[out_begin .. out_end).  The stores start at
// a buffer that depends on the workgroup, so that workgroups running at the
// same time write to different buffers.
template <class P, bool CACHED>
__device__ __forceinline__ void bcast_at(OutTable out, u64 byte_off, u32 out_begin, u32 out_end,
                                         typename P::raw_t packed)
{
    const u32 K = out_end - out_begin;
    u32 o = out_begin + blockIdx.x % K;
    for (u32 i = 0; i < K; ++i) {
        if (CACHED)
            P::store_for_reuse(out[o], byte_off, packed);
        else
            P::store(out[o], byte_off, packed);
        if (++o == out_end) o = out_begin;
    }
}

template <class T, class P, int CLASS, bool CACHED>
__device__ __forceinline__ void reduce_bcast_at(const NZ_KARG FusedArgs &a, u64 byte_off, u32 out_begin,
                                                u32 out_end)
{
    bcast_at<P, CACHED>(a.out, byte_off, out_begin, out_end,
                        reduce_at<T, P, CLASS, CACHED>(a.in, a.g.n_nodes, byte_off));
}

// The segment-wise form: the reduce-scatter half (segment j goes to its owner
// alone) and allreduces over some of the rails only.  The grid has two kinds
// of workgroups.  The first g.tile0[n_rails] of them each take one aligned
// tile of 256 vectors of one segment and handle the vectors that lie wholly
// inside it.  They are followed by one workgroup per (rail, segment) for the
// elements that share a 16-byte vector with a neighbouring segment or with
// the end of the buffer: one thread per element.
template <class T, int CLASS, bool CACHED>
__global__ __launch_bounds__(kThreads) void nz_fused_reduce_bcast(const FusedArgs)
{
    const NZ_KARG FusedArgs &a = kernel_args<FusedArgs>();
    const u32 n_tiles = a.g.tile0[a.g.n_rails];
    if (blockIdx.x < n_tiles) {
        u32 rail, seg, tile;
        decode_block(a.g, blockIdx.x, rail, seg, tile);
        const SegTile t = segment_tile<kThreads>(a.g, rail, seg, tile, T::kShift);
        const u64 full_lo = (t.b0 + 15) >> 4, full_hi = t.b1 >> 4;
        const u64 lo = t.vec_lo > full_lo ? t.vec_lo : full_lo;
        const u64 hi = t.vec_hi < full_hi ? t.vec_hi : full_hi;
        const u64 vec = t.tile_base + threadIdx.x;
        const u32 owner = (seg == 0 ? a.g.n_nodes : seg) - 1;
        const u32 o0 = a.owner_only ? owner : 0, o1 = a.owner_only ? owner + 1 : a.n_out;
        if (vec >= lo && vec < hi) reduce_bcast_at<T, VecPacket<T>, CLASS, CACHED>(a, vec << 4, o0, o1);
        return;
    }
    const u32 e = blockIdx.x - n_tiles;
    const u32 rail = e / a.g.n_nodes, seg = e - rail * a.g.n_nodes;
    const SegTile t = segment_tile<kThreads>(a.g, rail, seg, 0, T::kShift);
    if (t.b0 == t.b1) return;
    const u64 full_lo = (t.b0 + 15) >> 4, full_hi = t.b1 >> 4;
    const u64 head_end = (full_lo << 4) < t.b1 ? (full_lo << 4) : t.b1;
    u64 tail_beg = full_hi << 4;
    if (tail_beg < head_end) tail_beg = head_end;
    // threads 0..7 take the head elements, threads 64..71 the tail elements
    const u32 lane = threadIdx.x & 63u, part = threadIdx.x >> 6;
    const u64 eoff = (u64)lane << T::kShift;
    const u32 owner = (seg == 0 ? a.g.n_nodes : seg) - 1;
    const u32 o0 = a.owner_only ? owner : 0, o1 = a.owner_only ? owner + 1 : a.n_out;
    if (part == 0 && t.b0 + eoff < head_end) reduce_bcast_at<T, ElemPacket<T>, CLASS, CACHED>(a, t.b0 + eoff, o0, o1);
    if (part == 1 && tail_beg + eoff < t.b1)
        reduce_bcast_at<T, ElemPacket<T>, CLASS, CACHED>(a, tail_beg + eoff, o0, o1);
}

// The allreduce over the whole message in one launch.  Every element's sum
// goes to every output, so nothing here depends on where rails and segments
// begin: a workgroup takes VPT x 256 consecutive vectors of the buffers, and
// the last vector, if the message ends inside it, is done element by element.
// VPT, vectors per thread: with few nodes a thread has few loads of its own
// to keep in flight, so it takes several vectors and issues the loads of all
// of them before the first store (used for jobs that run out of the
// last-level cache, where latency is what bounds them; a job that streams
// from HBM is no faster for it).
struct FlatArgs {
    u64 bytes;  // of every buffer
    u32 n_nodes, n_out;
    const void *in[NZ_MAX_NODES];
    void *out[NZ_MAX_NODES];
};

template <class T, int CLASS, bool CACHED, int VPT>
__global__ __launch_bounds__(kThreads) void nz_fused_flat(const FlatArgs)
{
    const NZ_KARG FlatArgs &a = kernel_args<FlatArgs>();
    typename VecPacket<T>::raw_t packed[VPT];
#pragma unroll
    for (int it = 0; it < VPT; ++it) {
        const u64 b0 = (((u64)blockIdx.x * VPT + it) * kThreads + threadIdx.x) << 4;
        if (b0 + 16 <= a.bytes) packed[it] = reduce_at<T, VecPacket<T>, CLASS, CACHED>(a.in, a.n_nodes, b0);
    }
#pragma unroll
    for (int it = 0; it < VPT; ++it) {
        const u64 b0 = (((u64)blockIdx.x * VPT + it) * kThreads + threadIdx.x) << 4;
        if (b0 + 16 <= a.bytes) {
            bcast_at<VecPacket<T>, CACHED>(a.out, b0, 0, a.n_out, packed[it]);
        } else if (b0 < a.bytes) {
            for (u64 b = b0; b < a.bytes; b += sizeof(typename T::elem_t))
                bcast_at<ElemPacket<T>, CACHED>(a.out, b, 0, a.n_out,
                                                reduce_at<T, ElemPacket<T>, CLASS, CACHED>(a.in, a.n_nodes, b));
        }
    }
}

// ---------------------------------------------------------------------------
// Fused reduce + broadcast of a large message, staged through one output
// ---------------------------------------------------------------------------
//
// Writing K output streams at once from every workgroup is what the memory
// system likes least: with all buffers in one region of HBM the single-pass
// kernel above reaches 60-67 % of peak, while one write stream at a time
// reaches 85 %.  For large messages the work is therefore cut into pieces of
// a rail (kStagePieceBytes each) and issued as a short pipeline of launches;
// launch c holds two kinds of workgroups:
//   - "reduce": piece c is read once from all N nodes, summed as above and
//     stored (streaming) to the first distinct output buffer only;
//   - "spread": piece c - 1, finished by the previous launch, is copied from
//     that buffer to every other output buffer, one buffer after the other
//     (buffer index slowest in the grid).  The first pass over the piece
//     brings it into the L2 caches, the other K - 2 passes read it there.
// A piece is sized so that the share of it that one XCD's L2 sees (workgroup
// b runs on XCD b mod 8, and the tile a workgroup copies depends on b mod 8
// alone because all counts are padded to multiples of 8) stays below the L2
// capacity of 4 MB.  Every sum is still read once per node, computed once in
// registers and written once per output; the extra traffic is one cached
// re-read of the result.
constexpr u64 kStagePieceBytes = 24ull << 20;
#ifndef NZ_STAGE_COPY_ITERS
#define NZ_STAGE_COPY_ITERS 1
#endif
constexpr int kStageCopyIters = NZ_STAGE_COPY_ITERS;  // vectors per thread of the spread part

struct StageArgs {
    u64 a_lo, a_hi;   // bytes [a_lo, a_hi) of every buffer reduced by this launch; a_lo is a multiple of 16
    u64 b_lo, b_hi;   // bytes copied from out[0] to out[1 .. n_out) by this launch; b_lo likewise
    u32 n_a_blocks;   // workgroups of the reduce part (a multiple of 8)
    u32 b_tiles;      // workgroups per output buffer of the spread part (a multiple of 8),
                      // kStageCopyIters * 256 vectors each
    u32 n_nodes, n_out;
    const void *in[NZ_MAX_NODES];
    void *out[NZ_MAX_NODES];
};

template <class T, int CLASS>
__global__ __launch_bounds__(kThreads) void nz_fused_stage(const StageArgs)
{
    const NZ_KARG StageArgs &a = kernel_args<StageArgs>();
    if (blockIdx.x < a.n_a_blocks) {
        const u64 b0 = a.a_lo + (((u64)blockIdx.x * kThreads + threadIdx.x) << 4);
        if (b0 + 16 <= a.a_hi) {
            VecPacket<T>::store(a.out[0], b0, reduce_at<T, VecPacket<T>, CLASS, false>(a.in, a.n_nodes, b0));
        } else if (b0 < a.a_hi) {
            // the end of the message inside a vector: element by element
            for (u64 b = b0; b < a.a_hi; b += sizeof(typename T::elem_t))
                ElemPacket<T>::store(a.out[0], b, reduce_at<T, ElemPacket<T>, CLASS, false>(a.in, a.n_nodes, b));
        }
        return;
    }
    const u32 bb = blockIdx.x - a.n_a_blocks;
    const u32 pass = bb / a.b_tiles, tile = bb - pass * a.b_tiles;
    const void *src = a.out[0];
    void *dst = a.out[1 + pass];
    u64 b0[kStageCopyIters];
    vec16 v[kStageCopyIters];
#pragma unroll
    for (int it = 0; it < kStageCopyIters; ++it) {
        b0[it] = a.b_lo + ((((u64)tile * kStageCopyIters + it) * kThreads + threadIdx.x) << 4);
        if (b0[it] + 16 <= a.b_hi) v[it] = VecPacket<T>::load_again(src, b0[it]);
    }
#pragma unroll
    for (int it = 0; it < kStageCopyIters; ++it) {
        if (b0[it] + 16 <= a.b_hi) {
            VecPacket<T>::store(dst, b0[it], v[it]);
        } else if (b0[it] < a.b_hi) {
            for (u64 b = b0[it]; b < a.b_hi; b += sizeof(typename T::elem_t))
                ElemPacket<T>::store(dst, b, ElemPacket<T>::load(src, b));
        }
    }
}

// ---------------------------------------------------------------------------
// Ring steps
// ---------------------------------------------------------------------------

struct RingArgs {
    RailGeom g;
    u32 step;        // s = 0 .. N-2
    u32 elem_shift;
    const void *in[NZ_MAX_NODES];
    void *out[NZ_MAX_NODES];
};

// Reduce-scatter step s: node r sends segment (r - s) mod N to node d = r + 1;
// d stores dtype(fp32(received) + fp32(own)).  What r sends is its own input
// in step 0 and the partial it stored in step s - 1 afterwards.
// Allgather step s: node r sends the complete segment (r + 1 - s) mod N; d
// overwrites its copy.
//
// What a step stores is what the next step sends.  REUSE = the bytes of one
// step fit the last-level cache: they are stored and re-read with ordinary,
// cache-allocating accesses; otherwise they stream past the caches.
template <class T, class P, bool GATHER, bool REUSE>
__device__ __forceinline__ void ring_at(const void *sent, const void *own, void *dst, u64 byte_off)
{
    const typename P::raw_t rs = REUSE ? P::load_again(sent, byte_off) : P::load(sent, byte_off);
    typename P::raw_t result = rs;
    if (!GATHER) {
        typename T::acc_t x[P::kLanes], y[P::kLanes];
        const typename P::raw_t ro = P::load(own, byte_off);
        // Both loads are issued before either value is touched (left alone, the
        // scheduler starts widening the first operand and only then issues the
        // second load: two memory round trips instead of one).
        __builtin_amdgcn_sched_barrier(0);
        P::widen(rs, x);
        P::widen(ro, y);
#pragma unroll
        for (int l = 0; l < P::kLanes; ++l) x[l] = x[l] + y[l];
        result = P::narrow(x);
    }
    if (REUSE)
        P::store_for_reuse(dst, byte_off, result);
    else
        P::store(dst, byte_off, result);
}

// One workgroup's share of ring step `step`: tile `tile` of the piece
// [win_off, win_off + g.win_len) of the segment node r of rail `rail` sends in
// that step.
template <class T, int ITERS, bool GATHER, bool REUSE>
__device__ __forceinline__ void ring_tile(const NZ_KARG RingArgs &a, u32 rail, u32 r, u32 tile, u32 step,
                                          u64 win_off)
{
    constexpr int TILE = ITERS * kThreads;
    const u32 N = a.g.n_nodes;
    const u32 d = (r + 1 == N) ? 0 : r + 1;
    const u32 seg = GATHER ? (r + 1 + N - step) % N : (r + N - step) % N;
    const SegTile t = segment_tile<TILE>(a.g, rail, seg, tile, T::kShift, win_off, a.g.win_len);
    if (t.vec_lo >= t.vec_hi) return;

    const void *sent = (GATHER || step > 0) ? a.out[r] : a.in[r];
    const void *own = a.in[d];
    void *dst = a.out[d];

    const u64 full_lo = (t.b0 + 15) >> 4, full_hi = t.b1 >> 4;
    const u64 lo = t.vec_lo > full_lo ? t.vec_lo : full_lo;
    const u64 hi = t.vec_hi < full_hi ? t.vec_hi : full_hi;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const u64 vec = t.tile_base + (u64)it * kThreads + threadIdx.x;
        if (vec >= lo && vec < hi) ring_at<T, VecPacket<T>, GATHER, REUSE>(sent, own, dst, vec << 4);
    }
    const u64 head_end = (full_lo << 4) < t.b1 ? (full_lo << 4) : t.b1;
    u64 tail_beg = full_hi << 4;
    if (tail_beg < head_end) tail_beg = head_end;
    const u64 eoff = (u64)threadIdx.x << T::kShift;
    if (t.vec_lo == (t.b0 >> 4) && t.b0 + eoff < head_end)
        ring_at<T, ElemPacket<T>, GATHER, REUSE>(sent, own, dst, t.b0 + eoff);
    if (t.vec_hi == ((t.b1 + 15) >> 4) && tail_beg + eoff < t.b1)
        ring_at<T, ElemPacket<T>, GATHER, REUSE>(sent, own, dst, tail_beg + eoff);
}

// One ring step over all rails and nodes (the piece the launch works on is in
// the geometry).
template <class T, int ITERS, bool GATHER, bool REUSE>
__global__ __launch_bounds__(kThreads) void nz_ring_step(const RingArgs)
{
    const NZ_KARG RingArgs &a = kernel_args<RingArgs>();
    u32 rail, r, tile;
    decode_block(a.g, blockIdx.x, rail, r, tile);
    ring_tile<T, ITERS, GATHER, REUSE>(a, rail, r, tile, a.step, a.g.win_off);
}

// Ring_Chunked as a pipeline: the 2 (N - 1) steps of the ring are numbered
// u = 0 .. 2N - 3 (reduce-scatter steps first), a segment transfer is cut into
// pieces, and launch number w handles, for every piece c it has, step
// u = w - c of that piece: piece 0 is one step ahead of piece 1, which is one
// step ahead of piece 2, and so on -- what a pipeline of pieces looks like at
// one moment.  Pieces cover disjoint elements, so the piece-steps of one
// launch are independent, and a piece's step u runs one launch after its step
// u - 1.  A rail with shorter segments has fewer pieces; the launch holds
// workgroups only for the pieces a rail really has: rail k contributes pieces
// piece_lo[k] .. piece_lo[k] + n - 1, n following from block0, with
// N * g.tps[k] workgroups per piece (node, then tile) -- except the rail's
// last piece, which is as short as it happens to be and gets
// N * tps_last[k] workgroups, placed after those of the full pieces.
struct RingWaveArgs {
    RingArgs ring;                    // ring.step and ring.g.tile0 are not used
    u32 wave;                         // w
    u32 piece_lo[NZ_MAX_RAILS];       // first piece of each rail in this launch
    u32 block0[NZ_MAX_RAILS + 1];     // first workgroup of each rail in this launch
    u32 full_blocks[NZ_MAX_RAILS];    // workgroups of the rail's full-size pieces in this launch
    u32 last_piece[NZ_MAX_RAILS];     // index of the rail's last piece
    u32 tps_last[NZ_MAX_RAILS];       // tiles per segment of that piece
};

template <class T, int ITERS, bool REUSE>
__global__ __launch_bounds__(kThreads) void nz_ring_wave(const RingWaveArgs)
{
    const NZ_KARG RingWaveArgs &w = kernel_args<RingWaveArgs>();
    const NZ_KARG RingArgs &a = w.ring;
    u32 rail = 0;  // block0 never decreases: count the later rails that start at or before this workgroup
#pragma unroll
    for (u32 i = 1; i < NZ_MAX_RAILS; ++i) rail += (i < a.g.n_rails && blockIdx.x >= w.block0[i]) ? 1u : 0u;
    const u32 N = a.g.n_nodes;
    u32 rest = blockIdx.x - w.block0[rail];
    u32 tile, r, piece;
    if (rest < w.full_blocks[rail]) {
        const u32 tps = a.g.tps[rail];
        tile = rest % tps;
        rest /= tps;
        r = rest % N;
        piece = w.piece_lo[rail] + rest / N;
    } else {
        rest -= w.full_blocks[rail];
        const u32 tps = w.tps_last[rail];
        tile = rest % tps;
        r = rest / tps;
        piece = w.last_piece[rail];
    }
    const u32 u = w.wave - piece, half = N - 1;
    const u64 win_off = (u64)piece * a.g.win_len;
    if (u < half)
        ring_tile<T, ITERS, false, REUSE>(a, rail, r, tile, u, win_off);
    else
        ring_tile<T, ITERS, true, REUSE>(a, rail, r, tile, u - half, win_off);
}

// Direct allgather: every segment is read from the node that owns it after a
// reduce-scatter, node (j - 1) mod N for segment j, and stored to the other
// N - 1 nodes' buffers.  Two kernels.
//
// nz_gather_range (segments of at least one tile): one destination buffer
// after the other, because one write stream at a time is what the memory
// system handles best.  A rail's range is worked on in pieces small enough
// for the L2 caches, whatever segments they span: for every piece, for every
// destination d, the piece is copied into d's buffer from the owners of the
// segments it covers (d keeps the segment it owns).  The first destination's
// pass brings the piece into L2, the other passes read it there; a piece has
// a multiple of 8 workgroups, so that a tile is always copied by the same
// XCD.  Workgroup order within a rail: piece, destination, tile.  A tile is
// shorter than a segment, so it meets at most one segment boundary, which the
// workgroup locates once; a vector that the boundary (or the end of the
// message) cuts is copied element by element.
struct GatherRangeArgs {
    RailGeom g;                     // tps = workgroups per piece, win_* unused
    u32 pieces[NZ_MAX_RAILS];       // pieces per rail
    void *buf[NZ_MAX_NODES];
};

template <class T, int ITERS>
__global__ __launch_bounds__(kThreads) void nz_gather_range(const GatherRangeArgs)
{
    const NZ_KARG GatherRangeArgs &a = kernel_args<GatherRangeArgs>();
    constexpr int TILE = ITERS * kThreads;
    typedef typename T::elem_t elem_t;
    const u32 N = a.g.n_nodes;
    u32 rail = 0;  // tile0 never decreases: count the later rails that start at or before this workgroup
#pragma unroll
    for (u32 i = 1; i < NZ_MAX_RAILS; ++i) rail += (i < a.g.n_rails && blockIdx.x >= a.g.tile0[i]) ? 1u : 0u;
    const u32 tps = a.g.tps[rail];
    u32 rest = blockIdx.x - a.g.tile0[rail];
    const u32 tile = rest % tps;
    rest /= tps;
    const u32 d = rest % N, piece = rest / N;
    const u64 r0 = a.g.off[rail] << T::kShift, r1 = a.g.off[rail + 1] << T::kShift;  // the rail in bytes
    const u64 v0 = (r0 >> 4) + ((u64)piece * tps + tile) * TILE;
    if ((v0 << 4) >= r1) return;

    // The segment the tile starts in, and where the next one begins (elements).
    const u64 q = a.g.q[rail], rem = a.g.rem[rail];
    const u64 x_rel = ((v0 << 4) - r0) >> T::kShift, longer = rem * (q + 1);
    const u32 j0 = (u32)(x_rel < longer ? x_rel / (q + 1) : rem + (x_rel - longer) / q);
    const u64 bnd = a.g.off[rail] + (u64)(j0 + 1) * q + (j0 + 1 < rem ? j0 + 1 : rem);
    const u32 keeps = d + 1 == N ? 0 : d + 1;  // the segment destination d owns
    const void *src0 = a.buf[(j0 == 0 ? N : j0) - 1];
    const void *src1 = a.buf[j0];              // owner of segment j0 + 1
    void *dst = a.buf[d];

    vec16 v[ITERS];
    u32 how[ITERS];  // 0 nothing, 1 whole vector from src0, 2 whole vector from src1, 3 element by element
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const u64 b = (v0 + (u64)it * kThreads + threadIdx.x) << 4;
        const u64 x0 = b >> T::kShift, x1 = (b + 16) >> T::kShift;
        how[it] = 0;
        if (b >= r1) continue;
        if (b + 16 > r1 || (x0 < bnd && x1 > bnd))
            how[it] = 3;
        else if (x0 >= bnd)
            how[it] = (j0 + 1 == keeps) ? 0 : 2;
        else
            how[it] = (j0 == keeps) ? 0 : 1;
        if (how[it] == 1) v[it] = VecPacket<T>::load_again(src0, b);
        if (how[it] == 2) v[it] = VecPacket<T>::load_again(src1, b);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const u64 b = (v0 + (u64)it * kThreads + threadIdx.x) << 4;
        if (how[it] == 1 || how[it] == 2) {
            VecPacket<T>::store(dst, b, v[it]);
        } else if (how[it] == 3) {
            const u64 end = b + 16 < r1 ? b + 16 : r1;
            for (u64 e = b; e < end; e += sizeof(elem_t)) {
                const bool second = (e >> T::kShift) >= bnd;
                if ((second ? j0 + 1 : j0) != keeps)
                    ElemPacket<T>::store(dst, e, ElemPacket<T>::load(second ? src1 : src0, e));
            }
        }
    }
}

// nz_gather_bcast (any segment length; used when segments are shorter than a
// tile): one workgroup reads a tile of a segment once and stores it to all
// N - 1 destinations.  Same tiling as a ring step.  A pure copy, so T only
// fixes the element size of the edge path.
struct GatherArgs {
    RailGeom g;
    void *buf[NZ_MAX_NODES];
};

template <class P>
__device__ __forceinline__ void gather_at(const NZ_KARG GatherArgs &a, u32 owner, u64 byte_off)
{
    const typename P::raw_t v = P::load(a.buf[owner], byte_off);
    for (u32 m = 0; m < a.g.n_nodes; ++m)
        if (m != owner) P::store(a.buf[m], byte_off, v);
}

template <class T, int ITERS>
__global__ __launch_bounds__(kThreads) void nz_gather_bcast(const GatherArgs)
{
    const NZ_KARG GatherArgs &a = kernel_args<GatherArgs>();
    constexpr int TILE = ITERS * kThreads;
    u32 rail, seg, tile;
    decode_block(a.g, blockIdx.x, rail, seg, tile);
    const SegTile t = segment_tile<TILE>(a.g, rail, seg, tile, T::kShift);
    if (t.vec_lo >= t.vec_hi) return;
    const u32 owner = (seg == 0 ? a.g.n_nodes : seg) - 1;

    const u64 full_lo = (t.b0 + 15) >> 4, full_hi = t.b1 >> 4;
    const u64 lo = t.vec_lo > full_lo ? t.vec_lo : full_lo;
    const u64 hi = t.vec_hi < full_hi ? t.vec_hi : full_hi;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const u64 vec = t.tile_base + (u64)it * kThreads + threadIdx.x;
        if (vec >= lo && vec < hi) gather_at<VecPacket<T>>(a, owner, vec << 4);
    }
    const u64 head_end = (full_lo << 4) < t.b1 ? (full_lo << 4) : t.b1;
    u64 tail_beg = full_hi << 4;
    if (tail_beg < head_end) tail_beg = head_end;
    const u64 eoff = (u64)threadIdx.x << T::kShift;
    if (t.vec_lo == (t.b0 >> 4) && t.b0 + eoff < head_end) gather_at<ElemPacket<T>>(a, owner, t.b0 + eoff);
    if (t.vec_hi == ((t.b1 + 15) >> 4) && tail_beg + eoff < t.b1)
        gather_at<ElemPacket<T>>(a, owner, tail_beg + eoff);
}

// ---------------------------------------------------------------------------
// Segment copy (pack / unpack)
// ---------------------------------------------------------------------------

constexpr int kCopyMaxRuns = 64;  // runs per launch; longer lists take several launches

// One run: len bytes from src_off in every source buffer to dst_off in the
// matching destination buffer.  All three are multiples of the element size.
struct CopyArgs {
    u64 src_off[kCopyMaxRuns];
    u64 dst_off[kCopyMaxRuns];
    u64 len[kCopyMaxRuns];
    u32 tile0[kCopyMaxRuns + 1];  // first workgroup (per node) of each run
    u32 n_runs;
    u32 elem_bytes;
    u32 n_nodes;
    u32 node_major;  // workgroup order: 1 = one node's runs after the other, 0 = node index fastest
    const void *src[NZ_MAX_NODES];
    void *dst[NZ_MAX_NODES];
};

template <class E>
__device__ __forceinline__ void copy_elem(char *dst, const char *src)
{
    *(NZ_GLOBAL E *)dst = *(const NZ_GLOBAL E *)src;
}

// Tiles lie on the destination's 16-byte grid, so every store is an aligned
// 16-byte store.  When the source of a run sits at another offset within its
// 16 bytes (shift != 0), each lane loads the aligned source vector that holds
// the first bytes it needs, takes the following vector from the next lane
// through the LDS crossbar (ds_bpermute: no LDS memory, no barrier; the last
// lane of a wave loads its second vector itself) and assembles its
// destination vector with byte-align operations.  With shift == 0 it is a
// plain vector copy.  Bytes of the run outside whole destination vectors, and
// destination vectors whose two source vectors are not both inside the run,
// are copied element by element, so no access ever leaves [off, off + len) of
// either buffer.
//
// ALIGNED_ONLY: the host saw that every run of the launch has shift == 0 (a
// whole rail always has); the exchange path is then compiled out.  ITERS:
// 256-vector sub-tiles per workgroup.
//
// Workgroup order.  Node-major: the chip works through one node's buffers at a
// time, one read stream and one write stream, which is what the memory system
// handles best when all buffers lie close together.  Node index fastest: the
// workgroups in flight cover the same tiles of many nodes' buffers; better
// when the destinations are spread over the memory regions and the sources
// are not, because the writes then load all regions at once.
template <bool ALIGNED_ONLY, int ITERS>
__global__ __launch_bounds__(kThreads) void nz_segment_copy(const CopyArgs)
{
    const NZ_KARG CopyArgs &a = kernel_args<CopyArgs>();
    constexpr int kCopyIters = ITERS;

    u32 node, per_node;
    if (a.node_major) {
        const u32 per_node_total = a.tile0[a.n_runs];
        node = blockIdx.x / per_node_total;
        per_node = blockIdx.x - node * per_node_total;
    } else {
        per_node = blockIdx.x / a.n_nodes;
        node = blockIdx.x - per_node * a.n_nodes;
    }
    u32 run = 0;
    for (u32 span = a.n_runs; span > 1;) {  // last run whose first workgroup is <= per_node
        const u32 half = span >> 1;
        if (per_node >= a.tile0[run + half]) {
            run += half;
            span -= half;
        } else {
            span = half;
        }
    }
    const u32 tile = per_node - a.tile0[run];

    const char *src = static_cast<const char *>(a.src[node]);
    char *dst = static_cast<char *>(a.dst[node]);
    const u64 S = a.src_off[run], D = a.dst_off[run], L = a.len[run];
    const u64 d_end = D + L;
    const u64 full_lo = (D + 15) >> 4, full_hi = d_end >> 4;  // whole destination vectors
    const u32 shift = ALIGNED_ONLY ? 0u : (u32)((S - D) & 15);
    // Aligned source vectors that lie wholly inside the run.
    const long long src_full_lo = (long long)((S + 15) >> 4), src_full_hi = (long long)((S + L) >> 4);
    const u32 lane = threadIdx.x & 63u;

    constexpr int TILE = kCopyIters * kThreads;
    const u64 tile_base = ((D >> 4) / TILE + tile) * (u64)TILE;

    if (shift == 0) {
        // One sub-tile at a time: load, store, next (measured faster than batching the loads).
#pragma unroll 1
        for (int it = 0; it < kCopyIters; ++it) {
            const u64 w = tile_base + (u64)it * kThreads + threadIdx.x;  // destination vector
            if (w >= full_lo && w < full_hi) {
                const u64 sb = (w << 4) - D + S;
                const vec16 v = __builtin_nontemporal_load((const NZ_GLOBAL vec16 *)(src + sb));
                __builtin_nontemporal_store(v, (NZ_GLOBAL vec16 *)(dst + (w << 4)));
            }
        }
    }
#pragma unroll 1
    for (int it = 0; it < (!ALIGNED_ONLY && shift != 0 ? kCopyIters : 0); ++it) {
        const u64 w = tile_base + (u64)it * kThreads + threadIdx.x;  // destination vector
        const bool whole = (w >= full_lo && w < full_hi);
        // Source position of this destination vector; its first byte lies in
        // aligned source vector sv, its last in sv + 1.  (For the first tile the
        // position can lie in front of the buffer, hence signed arithmetic; only
        // vectors wholly inside the run are loaded.)
        const long long s_pos = (long long)(w << 4) - (long long)D + (long long)S;
        const long long sv = (s_pos - (long long)shift) >> 4;  // exact: s_pos = shift mod 16
        vec16 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
        if (sv >= src_full_lo && sv < src_full_hi)
            lo = __builtin_nontemporal_load((const NZ_GLOBAL vec16 *)(src + (sv << 4)));
        // Every lane takes part in the exchange, whatever it loaded.
        hi.x = __shfl_down(lo.x, 1);
        hi.y = __shfl_down(lo.y, 1);
        hi.z = __shfl_down(lo.z, 1);
        hi.w = __shfl_down(lo.w, 1);
        const bool both = whole && sv >= src_full_lo && sv + 1 < src_full_hi;
        if (lane == 63 && both) hi = __builtin_nontemporal_load((const NZ_GLOBAL vec16 *)(src + ((sv + 1) << 4)));
        if (both) {
            const u32 word[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            const u32 sh = shift & 3;  // 0 or 2 bytes
            vec16 v;
            switch (shift >> 2) {  // uniform
            case 0:  // shift == 2
                v.x = __builtin_amdgcn_alignbyte(word[1], word[0], sh);
                v.y = __builtin_amdgcn_alignbyte(word[2], word[1], sh);
                v.z = __builtin_amdgcn_alignbyte(word[3], word[2], sh);
                v.w = __builtin_amdgcn_alignbyte(word[4], word[3], sh);
                break;
            case 1:
                v.x = __builtin_amdgcn_alignbyte(word[2], word[1], sh);
                v.y = __builtin_amdgcn_alignbyte(word[3], word[2], sh);
                v.z = __builtin_amdgcn_alignbyte(word[4], word[3], sh);
                v.w = __builtin_amdgcn_alignbyte(word[5], word[4], sh);
                break;
            case 2:
                v.x = __builtin_amdgcn_alignbyte(word[3], word[2], sh);
                v.y = __builtin_amdgcn_alignbyte(word[4], word[3], sh);
                v.z = __builtin_amdgcn_alignbyte(word[5], word[4], sh);
                v.w = __builtin_amdgcn_alignbyte(word[6], word[5], sh);
                break;
            default:
                v.x = __builtin_amdgcn_alignbyte(word[4], word[3], sh);
                v.y = __builtin_amdgcn_alignbyte(word[5], word[4], sh);
                v.z = __builtin_amdgcn_alignbyte(word[6], word[5], sh);
                v.w = __builtin_amdgcn_alignbyte(word[7], word[6], sh);
                break;
            }
            __builtin_nontemporal_store(v, (NZ_GLOBAL vec16 *)(dst + (w << 4)));
        } else if (whole) {
            // A whole destination vector at the very edge of the run's source.
            const u64 sb = (w << 4) - D + S;
            if (a.elem_bytes == 4) {
                for (int i = 0; i < 4; ++i) copy_elem<u32>(dst + (w << 4) + 4 * i, src + sb + 4 * i);
            } else {
                for (int i = 0; i < 8; ++i) copy_elem<unsigned short>(dst + (w << 4) + 2 * i, src + sb + 2 * i);
            }
        }
    }

    // Bytes of the run that are not in a whole destination vector.
    const u64 head_end = (full_lo << 4) < d_end ? (full_lo << 4) : d_end;
    u64 tail_beg = full_hi << 4;
    if (tail_beg < head_end) tail_beg = head_end;
    const u64 eoff = (u64)threadIdx.x * a.elem_bytes;
    const u64 first_tile_base = ((D >> 4) / TILE) * (u64)TILE;
    const u64 last_tile_base = (((d_end + 15) >> 4) - 1) / TILE * (u64)TILE;
    if (tile_base == first_tile_base && D + eoff < head_end) {
        if (a.elem_bytes == 4)
            copy_elem<u32>(dst + D + eoff, src + S + eoff);
        else
            copy_elem<unsigned short>(dst + D + eoff, src + S + eoff);
    }
    if (tile_base == last_tile_base && tail_beg + eoff < d_end) {
        const u64 sb = tail_beg + eoff - D + S;
        if (a.elem_bytes == 4)
            copy_elem<u32>(dst + tail_beg + eoff, src + sb);
        else
            copy_elem<unsigned short>(dst + tail_beg + eoff, src + sb);
    }
}

}  // namespace

#endif  // NZ_DEVICE_H
