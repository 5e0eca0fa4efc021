// libdear: HIP kernels (gfx950) and context for DeAR's decoupled gradient aggregation.
//
// All three phases are HBM-bandwidth bound (about 0.2 flop per byte), so the kernels are
// plain streaming kernels: 16-byte vector accesses, one workgroup per tile of one
// layer/shard run, many independent loads in flight per lane, no matrix cores.
//
// Packing (copy into the fusion buffer, paper Sec. IV-A / V-A) is never materialised:
// a host-built tile table maps every run of bucket positions to (layer, element range,
// owning shard, shard-buffer offset), and the reduce-scatter reads the per-layer tensors
// directly while the all-gather writes them directly.
//
// Alignment: layer tensors start 16-byte aligned, so 16-byte vectors counted from the
// tensor start are always aligned on the tensor side (for all P replicas alike).  Layers
// are packed densely in a bucket, so the matching shard-buffer addresses are only
// 4-byte aligned; those accesses are issued as 16-byte accesses with 4-byte alignment,
// which global memory instructions allow for dword-aligned addresses.
//
// Bit-exactness: fp32 adds in the ring order of the owning shard, one rounding per
// operation, no contraction (file compiled with -ffp-contract=off, and see the pragma).
#include <hip/hip_runtime.h>

#include <memory>
#include <new>
#include <vector>

#include "dear_internal.h"

#pragma clang fp contract(off)

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef f4 f4_dword_aligned __attribute__((aligned(4)));  // 16-byte access, 4-byte alignment

struct dear_ctx_impl {
    int32_t L = 0, B = 0, P = 0, g = 0;
    int device = 0;
    int32_t max_workgroups = 0;  // 0: one workgroup per work item
    int32_t wave_priority = 0;   // wave priority (0..3) of bounded-grid kernels
    int64_t row_len = 0;
    std::vector<int64_t> bucket_shard_len, bucket_shard_base;
    std::vector<int64_t> tile_begin;  // [B+1] range of bucket b's tiles in the tile table
    dear_tile *d_tiles = nullptr;
    const void **d_grad = nullptr;    // [P*L] device pointers
    float **d_param = nullptr;        // [P*L] device pointers
};

// ------------------------------------------------------------------------------- kernels

// Launch-shape and cache-hint choices, fixed at build time (measured on MI355X; the
// defaults are the fastest found).  *_U = 16-byte vectors per lane; a tile of
// DEAR_TILE_ELEMS is shared by TILE_VECS / (U * DEAR_BLOCK) workgroups.
#ifndef DEAR_RS_U_F32
#define DEAR_RS_U_F32 1
#endif
#ifndef DEAR_RS_U_BF16
#define DEAR_RS_U_BF16 2
#endif
#ifndef DEAR_RS_NT_LOAD
#define DEAR_RS_NT_LOAD 1
#endif
#ifndef DEAR_RS_NT_STORE
#define DEAR_RS_NT_STORE 1
#endif
#ifndef DEAR_AG_U
#define DEAR_AG_U 1
#endif
#ifndef DEAR_AG_NT_LOAD
#define DEAR_AG_NT_LOAD 0
#endif
#ifndef DEAR_AG_CHUNK_BYTES
#define DEAR_AG_CHUNK_BYTES (16 << 20)  // shard bytes whose P copies are written back to back
#endif
#ifndef DEAR_AG_NT_STORE
#define DEAR_AG_NT_STORE 1
#endif
#ifndef DEAR_UPD_U
#define DEAR_UPD_U 1
#endif
#ifndef DEAR_UPD_NT_LOAD
#define DEAR_UPD_NT_LOAD 1
#endif
#ifndef DEAR_UPD_NT_STORE
#define DEAR_UPD_NT_STORE 1
#endif

// Pointers read from the pointer tables are generic; every tensor lives in global
// memory, and saying so lets the compiler use global_load / global_store.
#define DEAR_GLOBAL __attribute__((address_space(1)))
typedef const DEAR_GLOBAL u4 *global_u4_in;
typedef DEAR_GLOBAL f4 *global_f4_out;
typedef const DEAR_GLOBAL f4_dword_aligned *global_f4u_in;
typedef DEAR_GLOBAL f4_dword_aligned *global_f4u_out;

template <bool NT, class Ptr>
__device__ __forceinline__ auto load_vec(Ptr p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <bool NT, class Ptr, class V>
__device__ __forceinline__ void store_vec(Ptr p, V v)
{
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// 16-byte accesses to shard buffers, whose addresses are only 4-byte aligned.
template <bool NT>
__device__ __forceinline__ f4 load_f4_dword_aligned(const float *p)
{
    global_f4u_in q = (global_f4u_in)p;
    if (NT) return __builtin_nontemporal_load(q);
    return *q;
}

template <bool NT>
__device__ __forceinline__ void store_f4_dword_aligned(float *p, f4 v)
{
    global_f4u_out q = (global_f4u_out)p;
    if (NT)
        __builtin_nontemporal_store(v, q);
    else
        *q = v;
}

__device__ __forceinline__ int ring_worker(int start, int k, int P)
{
    int p = start + k;  // start < P and k < P, so one wrap suffices
    return p >= P ? p - P : p;
}

template <bool BF16>
__device__ __forceinline__ float grad_elem(const void *base, int64_t i)
{
    if (BF16) {
        uint32_t h = ((const DEAR_GLOBAL uint16_t *)base)[i];
        return __uint_as_float(h << 16);
    }
    return ((const DEAR_GLOBAL float *)base)[i];
}

// acc += the VE gradient elements held in one 16-byte vector (bf16 widens exactly).
template <bool BF16, int VE>
__device__ __forceinline__ void add_vector(float (&acc)[VE], const u4 r)
{
    if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[2 * j] = acc[2 * j] + __uint_as_float(r[j] << 16);
            acc[2 * j + 1] = acc[2 * j + 1] + __uint_as_float(r[j] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = acc[j] + __uint_as_float(r[j]);
    }
}

// Launch width.  By default every work item (a part of a tile, a block of update vectors)
// gets a workgroup of its own: BOUNDED = false, the grid equals the item count and the
// hardware's in-order workgroup dispatch paces the memory streams.  A context may bound the
// grid (dear_ctx_set_max_workgroups): BOUNDED = true, each workgroup strides over the items.
// That is for running beside compute kernels on the same GPU: a few hundred resident
// workgroups with many loads in flight each disturb a GEMM's memory latency far less than
// a full grid.  `prio` (dear_ctx_set_wave_priority) raises the wave priority of such a
// kernel: its wavefronts then win instruction issue against an MFMA-saturated neighbour,
// which makes the aggregation faster and the neighbour slower.
template <bool BOUNDED, class Body>
__device__ __forceinline__ void for_each_item(unsigned n_items, int prio, Body body)
{
    if (!BOUNDED) {
        body(blockIdx.x);
    } else {
        if (prio == 1)
            __builtin_amdgcn_s_setprio(1);
        else if (prio == 2)
            __builtin_amdgcn_s_setprio(2);
        else if (prio == 3)
            __builtin_amdgcn_s_setprio(3);
        for (unsigned item = blockIdx.x; item < n_items; item += gridDim.x) body(item);
    }
}

// Orders LDS traffic among the lanes of ONE wavefront (each wavefront of the reduce-scatter
// owns its own staging area, so no other wavefront is involved): the hardware performs a
// wavefront's LDS operations in issue order, so all that is needed is that the compiler
// keeps the stores before and the loads after this point.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Where a reduce-scatter result goes.  Plain: gbar is stored to the gradient shard buffer.
// FUSED: the SGD-momentum update of the slot is applied at once (v = mu*v + gbar;
// w = w - lr*v, the same four separately rounded operations as shard_update_kernel) and gbar
// is never written, which saves its 4-byte write and 4-byte re-read per element.
template <bool FUSED>
struct rs_sink {
    float *__restrict__ g;  // plain: gradient shards
    float *__restrict__ w;  // fused: parameter shards
    float *__restrict__ v;  // fused: momentum shards
    float lr, mu;
};

__device__ __forceinline__ void sgd_momentum(float gbar, float &w, float &v, float lr, float mu)
{
    const float t1 = mu * v;
    v = t1 + gbar;
    const float t2 = lr * v;
    w = w - t2;
}

// One 16-byte piece of results at shard-buffer element index `idx` (4-byte aligned).
// FUSED callers pass the slot's w and v, loaded early so the loads overlap the gradient loads.
template <bool FUSED>
__device__ __forceinline__ void emit_piece(const rs_sink<FUSED> &o, int64_t idx, f4 gbar, f4 w, f4 v)
{
    if (!FUSED) {
        store_f4_dword_aligned<DEAR_RS_NT_STORE>(o.g + idx, gbar);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float wj = w[j], vj = v[j];
            sgd_momentum(gbar[j], wj, vj, o.lr, o.mu);
            w[j] = wj;
            v[j] = vj;
        }
        store_f4_dword_aligned<DEAR_RS_NT_STORE>(o.v + idx, v);
        store_f4_dword_aligned<DEAR_RS_NT_STORE>(o.w + idx, w);
    }
}

template <bool FUSED>
__device__ __forceinline__ void emit_elem(const rs_sink<FUSED> &o, int64_t idx, float gbar)
{
    if (!FUSED) {
        o.g[idx] = gbar;
    } else {
        float w = o.w[idx], v = o.v[idx];
        sgd_momentum(gbar, w, v, o.lr, o.mu);
        o.v[idx] = v;
        o.w[idx] = w;
    }
}

// Body of the reduce-scatter for one workgroup's part of a tile.  ALL_FULL: the tile is a
// whole, aligned DEAR_TILE_ELEMS run, so no lane needs an edge check.  CH replicas are
// loaded per lane and vector before they are added; TAIL says P is not a multiple of CH.
template <bool BF16, int U, int CH, bool TAIL, bool ALL_FULL, bool FUSED>
__device__ __forceinline__ void reduce_scatter_tile(const dear_tile &t, int part,
                                                    const void *const *__restrict__ grad_tab, int L,
                                                    int P, float inv_P, const rs_sink<FUSED> &o)
{
    constexpr int VE = BF16 ? 8 : 4;  // elements per 16-byte vector
    constexpr int PIECES = VE / 4;     // 16-byte result pieces per lane and vector
    // bf16, whole tile: a lane's 8 results are 32 bytes, so storing them directly would
    // leave each store instruction half dense (16 of every 32 bytes) and HBM would see
    // partial lines.  Each wavefront turns its 512 results through its own 2 KiB of LDS
    // so that both store instructions write 64 consecutive 16-byte pieces.
    constexpr bool TURN = BF16 && ALL_FULL;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int64_t a = t.src_begin, c = a + t.count;
    const int64_t v_first = a / VE + (int64_t)part * (U * DEAR_BLOCK);
    if (!ALL_FULL && v_first * VE >= c) return;
    const int start = t.shard + 1 >= P ? 0 : t.shard + 1;

    int64_t vi[U];
    bool full[U];
    int64_t piece_idx[U][PIECES];  // shard-buffer element index of each result piece
    float acc[U][VE];
    f4 w_old[U][PIECES] = {}, v_old[U][PIECES] = {};  // only the fused sink reads them
#pragma unroll
    for (int u = 0; u < U; ++u) {
        vi[u] = v_first + u * DEAR_BLOCK + tid;
        const int64_t e0 = vi[u] * VE;
        full[u] = ALL_FULL || (e0 >= a && e0 + VE <= c);
#pragma unroll
        for (int j = 0; j < VE; ++j) acc[u][j] = -0.0f;
#pragma unroll
        for (int h = 0; h < PIECES; ++h) {
            if (TURN)  // piece h of the wave's 512-element run, lane-th 16 bytes of it
                piece_idx[u][h] = t.dst_begin + (v_first + u * DEAR_BLOCK + wave * 64) * VE - a + 256 * h + 4 * lane;
            else
                piece_idx[u][h] = t.dst_begin + (e0 - a) + 4 * h;
            if (FUSED && full[u]) {
                w_old[u][h] = load_f4_dword_aligned<DEAR_RS_NT_LOAD>(o.w + piece_idx[u][h]);
                v_old[u][h] = load_f4_dword_aligned<DEAR_RS_NT_LOAD>(o.v + piece_idx[u][h]);
            }
        }
    }

    for (int k0 = 0; k0 < P; k0 += CH) {
        global_u4_in src[CH];
#pragma unroll
        for (int kk = 0; kk < CH; ++kk) {
            const int k = (!TAIL || k0 + kk < P) ? k0 + kk : 0;
            src[kk] = (global_u4_in)grad_tab[(size_t)ring_worker(start, k, P) * L + t.layer];
        }
        u4 raw[U][CH];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (full[u]) {
#pragma unroll
                for (int kk = 0; kk < CH; ++kk)
                    if (!TAIL || k0 + kk < P) raw[u][kk] = load_vec<DEAR_RS_NT_LOAD>(src[kk] + vi[u]);
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (full[u]) {
#pragma unroll
                for (int kk = 0; kk < CH; ++kk)
                    if (!TAIL || k0 + kk < P) add_vector<BF16, VE>(acc[u], raw[u][kk]);
            }
    }

    if constexpr (TURN) {
        __shared__ float stage[DEAR_BLOCK / 64][64 * 8];
        float *sw = stage[wave];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            f4 lo, hi;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                lo[j] = acc[u][j] * inv_P;
                hi[j] = acc[u][4 + j] * inv_P;
            }
            *reinterpret_cast<f4 *>(sw + 8 * lane) = lo;
            *reinterpret_cast<f4 *>(sw + 8 * lane + 4) = hi;
            wave_lds_sync();
            const f4 o0 = *reinterpret_cast<const f4 *>(sw + 4 * lane);
            const f4 o1 = *reinterpret_cast<const f4 *>(sw + 256 + 4 * lane);
            wave_lds_sync();
            emit_piece<FUSED>(o, piece_idx[u][0], o0, w_old[u][0], v_old[u][0]);
            emit_piece<FUSED>(o, piece_idx[u][PIECES - 1], o1, w_old[u][PIECES - 1], v_old[u][PIECES - 1]);
        }
        return;
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t e0 = vi[u] * VE;
        if (full[u]) {
#pragma unroll
            for (int h = 0; h < PIECES; ++h) {
                f4 r;
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = acc[u][4 * h + j] * inv_P;
                emit_piece<FUSED>(o, piece_idx[u][h], r, w_old[u][h], v_old[u][h]);
            }
        } else if (e0 < c) {  // edge vector of the run: element by element
            for (int j = 0; j < VE; ++j) {
                const int64_t e = e0 + j;
                if (e < a || e >= c) continue;
                float s = -0.0f;
                for (int k = 0; k < P; ++k)
                    s = s + grad_elem<BF16>(grad_tab[(size_t)ring_worker(start, k, P) * L + t.layer], e);
                emit_elem<FUSED>(o, t.dst_begin + (e - a), s * inv_P);
            }
        }
    }
}

// Reduce-scatter (paper Sec. III-A; Eq. 2 for the 1/P).  SPLIT workgroups share a tile.
// Summation starts at worker s+1 and ends with worker s, the order in which the ring
// delivers the partial sums of chunk s to its owner.  The accumulator starts as -0.0f,
// the additive identity that keeps the first addend's bits (including a -0.0f).
template <bool BF16, int U, int CH, bool TAIL, bool FUSED, bool BOUNDED>
__global__ __launch_bounds__(DEAR_BLOCK) void reduce_scatter_kernel(
    const dear_tile *__restrict__ tiles, const void *const *__restrict__ grad_tab, int L, int P,
    float inv_P, const rs_sink<FUSED> o, unsigned n_items, int prio)
{
    constexpr int SPLIT = DEAR_TILE_ELEMS / ((BF16 ? 8 : 4) * DEAR_BLOCK * U);
    static_assert(SPLIT >= 1 && (SPLIT & (SPLIT - 1)) == 0, "U must divide the tile");
    for_each_item<BOUNDED>(n_items, prio, [&](unsigned item) {
        const dear_tile t = tiles[item / SPLIT];
        const int part = item % SPLIT;
        if (t.layer < 0) {  // padding slots: gbar = +0
            for (int i = part * DEAR_BLOCK + threadIdx.x; i < t.count; i += SPLIT * DEAR_BLOCK)
                emit_elem<FUSED>(o, t.dst_begin + i, 0.0f);
        } else if (t.count == DEAR_TILE_ELEMS) {
            reduce_scatter_tile<BF16, U, CH, TAIL, true, FUSED>(t, part, grad_tab, L, P, inv_P, o);
        } else {
            reduce_scatter_tile<BF16, U, CH, TAIL, false, FUSED>(t, part, grad_tab, L, P, inv_P, o);
        }
    });
}

// SGD with momentum on contiguous shard slots (paper Eq. 1-2): v = mu*v + g; w = w - lr*v.
// blockIdx.y selects the row (worker); each row segment is `vecs` 16-byte vectors long.
constexpr int UPD_U = DEAR_UPD_U;      // vectors per lane, one workgroup per item
constexpr int UPD_U_BOUNDED = 4;       // bounded grid: more loads in flight per lane
template <int U, bool BOUNDED>
__global__ __launch_bounds__(DEAR_BLOCK) void shard_update_kernel(
    const float *__restrict__ g, float *__restrict__ w, float *__restrict__ v, int64_t row_stride,
    int64_t base, int64_t vecs, float lr, float mu, unsigned blocks_per_row, unsigned n_items, int prio)
{
    for_each_item<BOUNDED>(n_items, prio, [&](unsigned item) {
        const unsigned row = item / blocks_per_row, bx = item - row * blocks_per_row;
        const int64_t off = (int64_t)row * row_stride + base;
        const f4 *__restrict__ g4 = reinterpret_cast<const f4 *>(g + off);
        f4 *__restrict__ w4 = reinterpret_cast<f4 *>(w + off);
        f4 *__restrict__ v4 = reinterpret_cast<f4 *>(v + off);
        const int64_t first = (int64_t)bx * (U * DEAR_BLOCK) + threadIdx.x;
        f4 gg[U], ww[U], vv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = first + u * DEAR_BLOCK;
            if (i < vecs) {
                gg[u] = load_vec<DEAR_UPD_NT_LOAD>(g4 + i);
                ww[u] = load_vec<DEAR_UPD_NT_LOAD>(w4 + i);
                vv[u] = load_vec<DEAR_UPD_NT_LOAD>(v4 + i);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = first + u * DEAR_BLOCK;
            if (i < vecs) {
                f4 nv, nw;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float t1 = mu * vv[u][j];
                    nv[j] = t1 + gg[u][j];
                    const float t2 = lr * nv[j];
                    nw[j] = ww[u][j] - t2;
                }
                store_vec<DEAR_UPD_NT_STORE>(v4 + i, nv);
                store_vec<DEAR_UPD_NT_STORE>(w4 + i, nw);
            }
        }
    });
}

// All-gather with the copy-back to the layer tensors folded in (paper Sec. III-A, IV-A).
//
// One workgroup copies one part of one tile to ONE replica.  Workgroups are ordered
// (chunk, replica, part): the hardware starts workgroups in index order, so at any moment
// the chip writes a long sequential run of one or two replicas instead of P interleaved
// streams, which HBM sustains markedly better; the chunk's shard values
// (DEAR_AG_CHUNK_BYTES: 16 MiB, i.e. 2 MiB in each XCD's 4 MiB L2, since a part is always read
// by the same XCD) are re-read for replicas 1..P-1 from L2, not HBM.
template <int U, bool ALL_FULL>
__device__ __forceinline__ void all_gather_tile(const dear_tile &t, int part, DEAR_GLOBAL float *out,
                                                const float *__restrict__ src)
{
    constexpr int VE = 4;
    const int tid = threadIdx.x;
    const int64_t a = t.src_begin, c = a + t.count;
    const int64_t v_first = a / VE + (int64_t)part * (U * DEAR_BLOCK);
    if (!ALL_FULL && v_first * VE >= c) return;
    int64_t vi[U];
    bool full[U];
    f4 val[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {  // all loads first, so they are in flight together
        vi[u] = v_first + u * DEAR_BLOCK + tid;
        const int64_t e0 = vi[u] * VE;
        full[u] = ALL_FULL || (e0 >= a && e0 + VE <= c);
        if (full[u]) val[u] = load_f4_dword_aligned<DEAR_AG_NT_LOAD>(src + (e0 - a));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t e0 = vi[u] * VE;
        if (full[u]) {
            store_vec<DEAR_AG_NT_STORE>((global_f4_out)out + vi[u], val[u]);
        } else if (e0 < c) {
            for (int j = 0; j < VE; ++j) {
                const int64_t e = e0 + j;
                if (e >= a && e < c) out[e] = src[e - a];
            }
        }
    }
}

constexpr int AG_U = DEAR_AG_U;   // vectors per lane, one workgroup per item

// n_parts = tiles * SPLIT; replicas p_first .. p_first+n_p-1 receive; there are
// n_parts * n_p work items.
template <int U, bool BOUNDED>
__global__ __launch_bounds__(DEAR_BLOCK) void all_gather_kernel(
    const dear_tile *__restrict__ tiles, float *const *__restrict__ param_tab, int L, int p_first,
    int n_p, const float *__restrict__ shard_param, unsigned n_parts, unsigned n_items)
{
    constexpr int SPLIT = DEAR_TILE_ELEMS / (4 * DEAR_BLOCK * U);
    static_assert(SPLIT >= 1 && (SPLIT & (SPLIT - 1)) == 0, "U must divide the tile");
    constexpr unsigned CHUNK = DEAR_AG_CHUNK_BYTES / (16 * DEAR_BLOCK * U);  // parts per chunk
    const unsigned per_chunk = CHUNK * (unsigned)n_p;
    for_each_item<BOUNDED>(n_items, 0, [&](unsigned item) {
        // item -> (chunk, replica, part within chunk); the last chunk may be short
        const unsigned chunk = item / per_chunk;
        const unsigned r = item - chunk * per_chunk;
        const unsigned first = chunk * CHUNK;
        const unsigned len = n_parts - first < CHUNK ? n_parts - first : CHUNK;
        const unsigned q = r / len;
        const unsigned id = first + (r - q * len);
        const unsigned p = (unsigned)p_first + q;

        const dear_tile t = tiles[id / SPLIT];
        const int part = id % SPLIT;
        if (t.layer < 0) return;
        const float *__restrict__ src = shard_param + t.dst_begin;
        DEAR_GLOBAL float *out = (DEAR_GLOBAL float *)param_tab[(size_t)p * L + t.layer];
        if (t.count == DEAR_TILE_ELEMS)
            all_gather_tile<U, true>(t, part, out, src);
        else
            all_gather_tile<U, false>(t, part, out, src);
    });
}

// Bounded-grid form of the all-gather: one item is a whole tile, read once and stored to all
// receiving replicas by the same workgroup.  Beside a GEMM the grid is too narrow to be
// bandwidth-bound, so what counts is bytes in flight per workgroup (4 loads, then 4 stores
// per replica), not the replica-sequential order of the full-grid kernel.
template <bool ALL_FULL>
__device__ __forceinline__ void all_gather_tile_all_replicas(const dear_tile &t,
                                                             float *const *__restrict__ param_tab, int L,
                                                             int p_first, int n_p,
                                                             const float *__restrict__ src)
{
    constexpr int VE = 4, U = DEAR_TILE_ELEMS / (VE * DEAR_BLOCK);
    const int tid = threadIdx.x;
    const int64_t a = t.src_begin, c = a + t.count;
    const int64_t v_first = a / VE;
    int64_t vi[U];
    bool full[U];
    f4 val[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        vi[u] = v_first + u * DEAR_BLOCK + tid;
        const int64_t e0 = vi[u] * VE;
        full[u] = ALL_FULL || (e0 >= a && e0 + VE <= c);
        if (full[u]) val[u] = load_f4_dword_aligned<DEAR_AG_NT_LOAD>(src + (e0 - a));
    }
    for (int q = 0; q < n_p; ++q) {
        DEAR_GLOBAL float *out = (DEAR_GLOBAL float *)param_tab[(size_t)(p_first + q) * L + t.layer];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e0 = vi[u] * VE;
            if (full[u]) {
                store_vec<DEAR_AG_NT_STORE>((global_f4_out)out + vi[u], val[u]);
            } else if (e0 < c) {
                for (int j = 0; j < VE; ++j) {
                    const int64_t e = e0 + j;
                    if (e >= a && e < c) out[e] = src[e - a];
                }
            }
        }
    }
}

__global__ __launch_bounds__(DEAR_BLOCK) void all_gather_bounded_kernel(
    const dear_tile *__restrict__ tiles, float *const *__restrict__ param_tab, int L, int p_first,
    int n_p, const float *__restrict__ shard_param, unsigned n_tiles, int prio)
{
    for_each_item<true>(n_tiles, prio, [&](unsigned item) {
        const dear_tile t = tiles[item];
        if (t.layer < 0) return;
        const float *__restrict__ src = shard_param + t.dst_begin;
        if (t.count == DEAR_TILE_ELEMS)
            all_gather_tile_all_replicas<true>(t, param_tab, L, p_first, n_p, src);
        else
            all_gather_tile_all_replicas<false>(t, param_tab, L, p_first, n_p, src);
    });
}

// Update and all-gather of a bucket in one kernel: a workgroup takes one tile, applies the
// SGD-momentum update to the tile's slots (the same four separately rounded operations as
// shard_update_kernel), stores the new w and v to the shard buffers and the new w to all
// receiving replicas' layer tensors.  The updated value has to reach every replica from the
// workgroup that computed it, so the stores go to all replicas at once (P interleaved write
// streams) instead of replica by replica as in all_gather_kernel.
template <bool ALL_FULL>
__device__ __forceinline__ void update_gather_tile(const dear_tile &t, float *const *__restrict__ param_tab, int L,
                                                   int P, const float *__restrict__ g, float *__restrict__ w,
                                                   float *__restrict__ v, float lr, float mu)
{
    constexpr int VE = 4, U = DEAR_TILE_ELEMS / (VE * DEAR_BLOCK);
    const int tid = threadIdx.x;
    const int64_t a = t.src_begin, c = a + t.count;
    const int64_t v_first = a / VE;
    int64_t vi[U];
    bool full[U];
    f4 gg[U], ww[U], vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        vi[u] = v_first + u * DEAR_BLOCK + tid;
        const int64_t e0 = vi[u] * VE;
        full[u] = ALL_FULL || (e0 >= a && e0 + VE <= c);
        if (full[u]) {
            const int64_t slot = t.dst_begin + (e0 - a);
            gg[u] = load_f4_dword_aligned<DEAR_UPD_NT_LOAD>(g + slot);
            ww[u] = load_f4_dword_aligned<DEAR_UPD_NT_LOAD>(w + slot);
            vv[u] = load_f4_dword_aligned<DEAR_UPD_NT_LOAD>(v + slot);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t e0 = vi[u] * VE;
        if (full[u]) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float wj = ww[u][j], vj = vv[u][j];
                sgd_momentum(gg[u][j], wj, vj, lr, mu);
                ww[u][j] = wj;
                vv[u][j] = vj;
            }
            const int64_t slot = t.dst_begin + (e0 - a);
            store_f4_dword_aligned<DEAR_UPD_NT_STORE>(v + slot, vv[u]);
            store_f4_dword_aligned<DEAR_UPD_NT_STORE>(w + slot, ww[u]);
        } else if (e0 < c) {  // edge vector of the run: element by element, all replicas
            for (int j = 0; j < VE; ++j) {
                const int64_t e = e0 + j;
                if (e < a || e >= c) continue;
                const int64_t slot = t.dst_begin + (e - a);
                float wj = w[slot], vj = v[slot];
                sgd_momentum(g[slot], wj, vj, lr, mu);
                v[slot] = vj;
                w[slot] = wj;
                for (int q = 0; q < P; ++q)
                    ((DEAR_GLOBAL float *)param_tab[(size_t)q * L + t.layer])[e] = wj;
            }
        }
    }
    for (int q = 0; q < P; ++q) {
        DEAR_GLOBAL float *out = (DEAR_GLOBAL float *)param_tab[(size_t)q * L + t.layer];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (full[u]) store_vec<DEAR_AG_NT_STORE>((global_f4_out)out + vi[u], ww[u]);
    }
}

template <bool BOUNDED>
__global__ __launch_bounds__(DEAR_BLOCK) void update_all_gather_kernel(
    const dear_tile *__restrict__ tiles, float *const *__restrict__ param_tab, int L, int P,
    const float *__restrict__ g, float *__restrict__ w, float *__restrict__ v, float lr, float mu,
    unsigned n_tiles, int prio)
{
    for_each_item<BOUNDED>(n_tiles, prio, [&](unsigned item) {
        const dear_tile t = tiles[item];
        if (t.layer < 0) {  // padding slots are updated like any other (their averaged gradient is +0)
            for (int i = threadIdx.x; i < t.count; i += DEAR_BLOCK) {
                const int64_t slot = t.dst_begin + i;
                float wj = w[slot], vj = v[slot];
                sgd_momentum(g[slot], wj, vj, lr, mu);
                v[slot] = vj;
                w[slot] = wj;
            }
        } else if (t.count == DEAR_TILE_ELEMS) {
            update_gather_tile<true>(t, param_tab, L, P, g, w, v, lr, mu);
        } else {
            update_gather_tile<false>(t, param_tab, L, P, g, w, v, lr, mu);
        }
    });
}

// Inverse of the all-gather for one worker: layer tensors -> owned shard slots.
__global__ __launch_bounds__(DEAR_BLOCK) void scatter_params_kernel(
    const dear_tile *__restrict__ tiles, float *const *__restrict__ param_tab, int L, int worker,
    float *__restrict__ shard_param)
{
    constexpr int VE = 4;
    constexpr int U = DEAR_TILE_ELEMS / (VE * DEAR_BLOCK);
    const dear_tile t = tiles[blockIdx.x];
    const int tid = threadIdx.x;
    float *__restrict__ dst = shard_param + t.dst_begin;
    if (t.layer < 0) {
        for (int i = tid; i < t.count; i += DEAR_BLOCK) dst[i] = 0.0f;
        return;
    }
    const DEAR_GLOBAL float *in = (const DEAR_GLOBAL float *)param_tab[(size_t)worker * L + t.layer];
    const int64_t a = t.src_begin, c = a + t.count;
    const int64_t v_first = a / VE;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v_first + u * DEAR_BLOCK + tid;
        const int64_t e0 = v * VE;
        if (e0 >= a && e0 + VE <= c) {
            *(global_f4u_out)(dst + (e0 - a)) = ((const DEAR_GLOBAL f4 *)in)[v];
        } else if (e0 < c) {
            for (int j = 0; j < VE; ++j) {
                const int64_t e = e0 + j;
                if (e >= a && e < c) dst[e - a] = in[e];
            }
        }
    }
}

// ------------------------------------------------------------------------------- host side

inline bool misaligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_call(const dear_ctx_impl *c, int32_t bucket)
{
    if (!c) return DEAR_EINVAL;
    if (bucket < -1 || bucket >= c->B) return DEAR_ERANGE;
    int dev = -1;  // the tables live on the device that was current at dear_ctx_create
    if (hipGetDevice(&dev) != hipSuccess) return DEAR_EHIP;
    if (dev != c->device) return DEAR_EINVAL;
    return DEAR_OK;
}

int check_shard_buffer(const void *p)
{
    if (!p) return DEAR_EINVAL;
    if (misaligned(p, 256)) return DEAR_EALIGN;
    return DEAR_OK;
}

void tile_range(const dear_ctx_impl *c, int32_t bucket, int64_t &first, int64_t &count)
{
    if (bucket < 0) {
        first = 0;
        count = c->tile_begin[c->B];
    } else {
        first = c->tile_begin[bucket];
        count = c->tile_begin[bucket + 1] - first;
    }
}

int launch_status() { return hipGetLastError() == hipSuccess ? DEAR_OK : DEAR_EHIP; }

unsigned grid_width(int32_t max_workgroups, int64_t n_items)
{
    if (max_workgroups > 0 && n_items > max_workgroups) return static_cast<unsigned>(max_workgroups);
    return static_cast<unsigned>(n_items);
}

// tiles, grad_tab: device tables (a context's, or the static scratch's).
template <bool BF16, bool FUSED>
void rs_launch(int P, int L, const void *const *grad_tab, int32_t max_workgroups, int prio, int64_t n_tiles,
               hipStream_t st, const dear_tile *tiles, const rs_sink<FUSED> &o)
{
    constexpr int U = BF16 ? DEAR_RS_U_BF16 : DEAR_RS_U_F32;
    constexpr int SPLIT = DEAR_TILE_ELEMS / ((BF16 ? 8 : 4) * DEAR_BLOCK * U);
    const unsigned n_items = static_cast<unsigned>(n_tiles * SPLIT);
    const dim3 grid(grid_width(max_workgroups, n_items)), block(DEAR_BLOCK);
    const bool bounded = grid.x < n_items;
    const float inv_P = 1.0f / static_cast<float>(P);
#define RS_LAUNCH(CH, TAIL)                                                                              \
    do {                                                                                                 \
        if (bounded)                                                                                     \
            reduce_scatter_kernel<BF16, U, CH, TAIL, FUSED, true><<<grid, block, 0, st>>>(              \
                tiles, grad_tab, L, P, inv_P, o, n_items, prio);                                         \
        else                                                                                             \
            reduce_scatter_kernel<BF16, U, CH, TAIL, FUSED, false><<<grid, block, 0, st>>>(             \
                tiles, grad_tab, L, P, inv_P, o, n_items, 0);                                            \
    } while (0)
    // replicas per load batch: the largest of 8/4/2/1 that divides P without a tail when
    // P is small or a multiple of 4; otherwise batches of 8 with a predicated tail
    if (P % 8 == 0)
        RS_LAUNCH(8, false);
    else if (P % 4 == 0)
        RS_LAUNCH(4, false);
    else if (P == 2)
        RS_LAUNCH(2, false);
    else if (P == 1)
        RS_LAUNCH(1, false);
    else
        RS_LAUNCH(8, true);
#undef RS_LAUNCH
}

}  // namespace

struct dear_ctx_s : dear_ctx_impl {};

extern "C" int dear_ctx_create(const dear_plan_t *plan, int32_t grad_dtype,
                               const void *const *grad_ptrs, float *const *param_ptrs,
                               dear_ctx_t **out)
{
    if (!plan || !grad_ptrs || !param_ptrs || !out) return DEAR_EINVAL;
    if (grad_dtype != DEAR_F32 && grad_dtype != DEAR_BF16) return DEAR_EINVAL;
    if ((grad_dtype == DEAR_F32 ? 4 : 2) != plan->g) return DEAR_EINVAL;
    const size_t n_ptr = static_cast<size_t>(plan->P) * plan->L;
    for (size_t i = 0; i < n_ptr; ++i) {
        if (!grad_ptrs[i] || !param_ptrs[i]) return DEAR_EINVAL;
        if (misaligned(grad_ptrs[i], 16) || misaligned(param_ptrs[i], 16)) return DEAR_EALIGN;
    }
    std::unique_ptr<dear_ctx_s> c;
    std::vector<dear_tile> tiles;
    try {
        c.reset(new dear_ctx_s);
        c->L = plan->L;
        c->B = plan->B;
        c->P = plan->P;
        c->g = plan->g;
        c->row_len = plan->row_len;
        c->bucket_shard_len = plan->bucket_shard_len;
        c->bucket_shard_base = plan->bucket_shard_base;
        dear_build_tiles(*plan, tiles, c->tile_begin);
    } catch (const std::bad_alloc &) {
        return DEAR_ENOMEM;
    }
    if (tiles.size() > 0x7fffffffu / 16) return DEAR_EINVAL;  // grid.x limit, up to 16 workgroups a tile
    if (hipGetDevice(&c->device) != hipSuccess) return DEAR_EHIP;

    const size_t tile_bytes = tiles.size() * sizeof(dear_tile), ptr_bytes = n_ptr * sizeof(void *);
    bool ok = hipMalloc(reinterpret_cast<void **>(&c->d_tiles), tile_bytes) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&c->d_grad), ptr_bytes) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&c->d_param), ptr_bytes) == hipSuccess;
    int rc = DEAR_OK;
    if (!ok) {
        rc = DEAR_ENOMEM;
        (void)hipGetLastError();
    } else if (hipMemcpy(c->d_tiles, tiles.data(), tile_bytes, hipMemcpyHostToDevice) != hipSuccess ||
               hipMemcpy(c->d_grad, grad_ptrs, ptr_bytes, hipMemcpyHostToDevice) != hipSuccess ||
               hipMemcpy(c->d_param, param_ptrs, ptr_bytes, hipMemcpyHostToDevice) != hipSuccess) {
        rc = DEAR_EHIP;
        (void)hipGetLastError();
    }
    if (rc != DEAR_OK) {
        dear_ctx_destroy(c.release());
        return rc;
    }
    *out = c.release();
    return DEAR_OK;
}

extern "C" int dear_ctx_set_max_workgroups(dear_ctx_t *c, int32_t max_workgroups)
{
    if (!c || max_workgroups < 0) return DEAR_EINVAL;
    c->max_workgroups = max_workgroups;
    return DEAR_OK;
}

extern "C" int dear_ctx_set_wave_priority(dear_ctx_t *c, int32_t priority)
{
    if (!c || priority < 0 || priority > 3) return DEAR_EINVAL;
    c->wave_priority = priority;
    return DEAR_OK;
}

extern "C" void dear_ctx_destroy(dear_ctx_t *c)
{
    if (!c) return;
    (void)hipDeviceSynchronize();
    if (c->d_tiles) (void)hipFree(c->d_tiles);
    if (c->d_grad) (void)hipFree(c->d_grad);
    if (c->d_param) (void)hipFree(c->d_param);
    delete c;
}

extern "C" int dear_reduce_scatter(dear_ctx_t *c, int32_t bucket, float *shard_grad, void *hip_stream)
{
    int rc = check_call(c, bucket);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_grad);
    if (rc != DEAR_OK) return rc;
    int64_t first, count;
    tile_range(c, bucket, first, count);
    if (count == 0) return DEAR_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const rs_sink<false> o{shard_grad, nullptr, nullptr, 0.0f, 0.0f};
    if (c->g == 2)
        rs_launch<true, false>(c->P, c->L, c->d_grad, c->max_workgroups, c->wave_priority, count, st, c->d_tiles + first, o);
    else
        rs_launch<false, false>(c->P, c->L, c->d_grad, c->max_workgroups, c->wave_priority, count, st, c->d_tiles + first, o);
    return launch_status();
}

extern "C" int dear_reduce_scatter_update(dear_ctx_t *c, int32_t bucket, float *shard_param,
                                         float *shard_mom, float lr, float momentum, void *hip_stream)
{
    int rc = check_call(c, bucket);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_param);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_mom);
    if (rc != DEAR_OK) return rc;
    if (shard_param == shard_mom) return DEAR_EINVAL;
    int64_t first, count;
    tile_range(c, bucket, first, count);
    if (count == 0) return DEAR_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const rs_sink<true> o{nullptr, shard_param, shard_mom, lr, momentum};
    if (c->g == 2)
        rs_launch<true, true>(c->P, c->L, c->d_grad, c->max_workgroups, c->wave_priority, count, st, c->d_tiles + first, o);
    else
        rs_launch<false, true>(c->P, c->L, c->d_grad, c->max_workgroups, c->wave_priority, count, st, c->d_tiles + first, o);
    return launch_status();
}

extern "C" int dear_shard_update(dear_ctx_t *c, int32_t bucket, const float *shard_grad,
                                 float *shard_param, float *shard_mom, float lr, float momentum,
                                 void *hip_stream)
{
    int rc = check_call(c, bucket);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_grad);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_param);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_mom);
    if (rc != DEAR_OK) return rc;
    if (shard_grad == shard_param || shard_grad == shard_mom || shard_param == shard_mom) return DEAR_EINVAL;
    // All buckets: the P rows are back to back, so the whole buffer is one run.
    int64_t base = 0, elems = c->row_len * c->P;
    unsigned rows = 1;
    if (bucket >= 0) {
        base = c->bucket_shard_base[bucket];
        elems = c->bucket_shard_len[bucket];
        rows = static_cast<unsigned>(c->P);
    }
    const int64_t vecs = elems / 4;  // shard lengths are multiples of DEAR_SHARD_ALIGN
    if (vecs == 0) return DEAR_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool bounded = c->max_workgroups > 0 &&
                         (vecs + UPD_U_BOUNDED * DEAR_BLOCK - 1) / (UPD_U_BOUNDED * DEAR_BLOCK) * rows > c->max_workgroups;
    const int64_t per_block = static_cast<int64_t>(bounded ? UPD_U_BOUNDED : UPD_U) * DEAR_BLOCK;
    const int64_t blocks = (vecs + per_block - 1) / per_block;
    const int64_t n_items = blocks * rows;
    if (n_items > 0x7fffffff) return DEAR_EINVAL;
    if (bounded)
        shard_update_kernel<UPD_U_BOUNDED, true><<<dim3(c->max_workgroups), dim3(DEAR_BLOCK), 0, st>>>(
            shard_grad, shard_param, shard_mom, c->row_len, base, vecs, lr, momentum,
            static_cast<unsigned>(blocks), static_cast<unsigned>(n_items), c->wave_priority);
    else
        shard_update_kernel<UPD_U, false><<<dim3(static_cast<unsigned>(n_items)), dim3(DEAR_BLOCK), 0, st>>>(
            shard_grad, shard_param, shard_mom, c->row_len, base, vecs, lr, momentum,
            static_cast<unsigned>(blocks), static_cast<unsigned>(n_items), 0);
    return launch_status();
}

extern "C" int dear_update_all_gather(dear_ctx_t *c, int32_t bucket, const float *shard_grad,
                                      float *shard_param, float *shard_mom, float lr, float momentum,
                                      void *hip_stream)
{
    int rc = check_call(c, bucket);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_grad);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_param);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_mom);
    if (rc != DEAR_OK) return rc;
    if (shard_grad == shard_param || shard_grad == shard_mom || shard_param == shard_mom) return DEAR_EINVAL;
    int64_t first, count;
    tile_range(c, bucket, first, count);
    if (count == 0) return DEAR_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const unsigned width = grid_width(c->max_workgroups, count);
    if (width < count)
        update_all_gather_kernel<true><<<dim3(width), dim3(DEAR_BLOCK), 0, st>>>(
            c->d_tiles + first, c->d_param, c->L, c->P, shard_grad, shard_param, shard_mom, lr, momentum,
            static_cast<unsigned>(count), c->wave_priority);
    else
        update_all_gather_kernel<false><<<dim3(width), dim3(DEAR_BLOCK), 0, st>>>(
            c->d_tiles + first, c->d_param, c->L, c->P, shard_grad, shard_param, shard_mom, lr, momentum,
            static_cast<unsigned>(count), 0);
    return launch_status();
}

extern "C" int dear_all_gather_workers(dear_ctx_t *c, int32_t bucket, const float *shard_param,
                                       int32_t first_worker, int32_t n_workers, void *hip_stream)
{
    int rc = check_call(c, bucket);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_param);
    if (rc != DEAR_OK) return rc;
    if (first_worker < 0 || n_workers < 1 || first_worker > c->P - n_workers) return DEAR_ERANGE;
    int64_t first, count;
    tile_range(c, bucket, first, count);
    if (count == 0) return DEAR_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    constexpr int64_t split_free = DEAR_TILE_ELEMS / (4 * DEAR_BLOCK * AG_U);
    if (count * split_free * n_workers > 0x7fffffff) return DEAR_EINVAL;
    if (c->max_workgroups > 0 && count * split_free * n_workers > c->max_workgroups) {
        // the bounded form strides over whole tiles, so its grid is at most the tile count
        const unsigned width = grid_width(c->max_workgroups, count);
        all_gather_bounded_kernel<<<dim3(width), dim3(DEAR_BLOCK), 0, st>>>(
            c->d_tiles + first, c->d_param, c->L, first_worker, n_workers, shard_param,
            static_cast<unsigned>(count), c->wave_priority);
    } else {
        const int64_t n_parts = count * split_free, n_items = n_parts * n_workers;
        all_gather_kernel<AG_U, false><<<dim3(static_cast<unsigned>(n_items)), dim3(DEAR_BLOCK), 0, st>>>(
            c->d_tiles + first, c->d_param, c->L, first_worker, n_workers, shard_param,
            static_cast<unsigned>(n_parts), static_cast<unsigned>(n_items));
    }
    return launch_status();
}

extern "C" int dear_all_gather(dear_ctx_t *c, int32_t bucket, const float *shard_param, void *hip_stream)
{
    if (!c) return DEAR_EINVAL;
    return dear_all_gather_workers(c, bucket, shard_param, 0, c->P, hip_stream);
}

extern "C" int dear_scatter_params(dear_ctx_t *c, int32_t worker, float *shard_param, void *hip_stream)
{
    int rc = check_call(c, -1);
    if (rc != DEAR_OK) return rc;
    if (worker < 0 || worker >= c->P) return DEAR_ERANGE;
    rc = check_shard_buffer(shard_param);
    if (rc != DEAR_OK) return rc;
    const int64_t count = c->tile_begin[c->B];
    if (count == 0) return DEAR_OK;
    scatter_params_kernel<<<dim3(static_cast<unsigned>(count)), dim3(DEAR_BLOCK), 0,
                            static_cast<hipStream_t>(hip_stream)>>>(c->d_tiles, c->d_param, c->L, worker,
                                                                    shard_param);
    return launch_status();
}

// ------------------------------------------------------------- entry point without allocation
//
// dear_reduce_scatter needs a context, and creating one allocates device memory for the tile
// table and the pointer table its kernel reads.  For callers that cannot allocate, the same
// kernel reads both tables from this file-scope device array instead.  Layout: gradient
// pointer table first, tile table behind it.  Every GPU the library runs on holds its own copy
// of the array until the process ends.
namespace {

constexpr size_t STATIC_MAX_PTRS = DEAR_STATIC_MAX_POINTERS;
constexpr size_t STATIC_MAX_TILES = DEAR_STATIC_MAX_TILES;
constexpr size_t STATIC_PTR_BYTES = STATIC_MAX_PTRS * sizeof(void *);
constexpr size_t STATIC_TILE_BYTES = STATIC_MAX_TILES * sizeof(dear_tile);
static_assert(STATIC_PTR_BYTES % 256 == 0, "the tile table must start aligned");

__device__ __align__(256) unsigned char scratch[STATIC_PTR_BYTES + STATIC_TILE_BYTES];

// Host staging of the two tables (pageable, file scope: no heap use on this path).
unsigned char host_stage[STATIC_PTR_BYTES + STATIC_TILE_BYTES];

constexpr int MAX_DEVICES = 64;
unsigned char *scratch_of_device[MAX_DEVICES];  // device address of `scratch`, per GPU

// `scratch` names a host-side stand-in in host code; the device address has to be asked for,
// once per device, with that device current.
int static_scratch(int device, unsigned char **out)
{
    if (device < 0 || device >= MAX_DEVICES) return DEAR_EINVAL;
    if (!scratch_of_device[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return DEAR_EHIP;
        }
        scratch_of_device[device] = static_cast<unsigned char *>(p);
    }
    *out = scratch_of_device[device];
    return DEAR_OK;
}

}  // namespace

extern "C" int dear_reduce_scatter_static(const dear_plan_t *plan, int32_t grad_dtype,
                                          const void *const *grad_ptrs, int32_t bucket, float *shard_grad,
                                          void *hip_stream)
{
    if (!plan || !grad_ptrs) return DEAR_EINVAL;
    if (grad_dtype != DEAR_F32 && grad_dtype != DEAR_BF16) return DEAR_EINVAL;
    if ((grad_dtype == DEAR_F32 ? 4 : 2) != plan->g) return DEAR_EINVAL;
    if (bucket < -1 || bucket >= plan->B) return DEAR_ERANGE;
    int rc = check_shard_buffer(shard_grad);
    if (rc != DEAR_OK) return rc;
    const size_t n_ptr = static_cast<size_t>(plan->P) * plan->L;
    if (n_ptr > STATIC_MAX_PTRS) return DEAR_ETOOBIG;
    const int32_t b_first = bucket < 0 ? 0 : bucket, b_last = bucket < 0 ? plan->B : bucket + 1;
    // only the gradient tensors of the buckets processed are dereferenced, but the whole table is checked
    for (size_t i = 0; i < n_ptr; ++i) {
        if (!grad_ptrs[i]) return DEAR_EINVAL;
        if (misaligned(grad_ptrs[i], 16)) return DEAR_EALIGN;
    }
    dear_tile *host_tiles = reinterpret_cast<dear_tile *>(host_stage + STATIC_PTR_BYTES);
    const int64_t n_tiles = dear_emit_tiles(*plan, b_first, b_last, host_tiles, STATIC_MAX_TILES, nullptr);
    if (n_tiles > static_cast<int64_t>(STATIC_MAX_TILES)) return DEAR_ETOOBIG;
    if (n_tiles == 0) return DEAR_OK;

    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return DEAR_EHIP;
    unsigned char *dev = nullptr;
    rc = static_scratch(device, &dev);
    if (rc != DEAR_OK) return rc;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    for (size_t i = 0; i < n_ptr; ++i) reinterpret_cast<const void **>(host_stage)[i] = grad_ptrs[i];
    // Stream-ordered uploads: earlier kernels of this stream that still read the scratch finish
    // first.  The staging memory is pageable and is reused by the next call, so the stream is
    // drained before returning to the point where the copies have been taken.
    if (hipMemcpyAsync(dev, host_stage, n_ptr * sizeof(void *), hipMemcpyHostToDevice, st) != hipSuccess ||
        hipMemcpyAsync(dev + STATIC_PTR_BYTES, host_tiles, static_cast<size_t>(n_tiles) * sizeof(dear_tile),
                       hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        (void)hipGetLastError();
        return DEAR_EHIP;
    }
    const void *const *grad_tab = reinterpret_cast<const void *const *>(dev);
    const dear_tile *tiles = reinterpret_cast<const dear_tile *>(dev + STATIC_PTR_BYTES);
    const rs_sink<false> o{shard_grad, nullptr, nullptr, 0.0f, 0.0f};
    if (plan->g == 2)
        rs_launch<true, false>(plan->P, plan->L, grad_tab, 0, 0, n_tiles, st, tiles, o);
    else
        rs_launch<false, false>(plan->P, plan->L, grad_tab, 0, 0, n_tiles, st, tiles, o);
    return launch_status();
}
