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
    int64_t row_len = 0;
    std::vector<int64_t> bucket_shard_len, bucket_shard_base;
    std::vector<int64_t> tile_begin;  // [B+1] range of bucket b's tiles in the tile table
    dear_tile *d_tiles = nullptr;
    const void **d_grad = nullptr;    // [P*L] device pointers
    float **d_param = nullptr;        // [P*L] device pointers
};

// ------------------------------------------------------------------------------- kernels

// Pointers read from the pointer tables are generic; every tensor lives in global
// memory, and saying so lets the compiler use global_load / global_store.
#define DEAR_GLOBAL __attribute__((address_space(1)))
typedef const DEAR_GLOBAL u4 *global_u4_in;
typedef DEAR_GLOBAL f4 *global_f4_out;
typedef const DEAR_GLOBAL f4_dword_aligned *global_f4u_in;
typedef DEAR_GLOBAL f4_dword_aligned *global_f4u_out;

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

// Body of the reduce-scatter for one tile.  ALL_FULL: the tile is a whole, aligned
// DEAR_TILE_ELEMS run, so no lane needs an edge check.  CH replicas are loaded per lane
// and vector before they are added; TAIL says P is not a multiple of CH.
template <bool BF16, int CH, bool TAIL, bool ALL_FULL>
__device__ __forceinline__ void reduce_scatter_tile(const dear_tile &t, const void *const *__restrict__ grad_tab,
                                                    int L, int P, float inv_P, float *__restrict__ dst)
{
    constexpr int VE = BF16 ? 8 : 4;                       // elements per 16-byte vector
    constexpr int U = DEAR_TILE_ELEMS / (VE * DEAR_BLOCK);  // vectors per lane
    const int tid = threadIdx.x;
    const int64_t a = t.src_begin, c = a + t.count;
    const int64_t v_first = a / VE;
    const int start = t.shard + 1 >= P ? 0 : t.shard + 1;

    int64_t vi[U];
    bool full[U];
    float acc[U][VE];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        vi[u] = v_first + u * DEAR_BLOCK + tid;
        const int64_t e0 = vi[u] * VE;
        full[u] = ALL_FULL || (e0 >= a && e0 + VE <= c);
#pragma unroll
        for (int j = 0; j < VE; ++j) acc[u][j] = -0.0f;
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
                    if (!TAIL || k0 + kk < P) raw[u][kk] = __builtin_nontemporal_load(src[kk] + vi[u]);
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (full[u]) {
#pragma unroll
                for (int kk = 0; kk < CH; ++kk)
                    if (!TAIL || k0 + kk < P) add_vector<BF16, VE>(acc[u], raw[u][kk]);
            }
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t e0 = vi[u] * VE;
        if (full[u]) {
            float *out = dst + (e0 - a);
#pragma unroll
            for (int h = 0; h < VE / 4; ++h) {
                f4 r;
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = acc[u][4 * h + j] * inv_P;
                *(global_f4u_out)(out + 4 * h) = r;
            }
        } else if (e0 < c) {  // edge vector of the run: element by element
            for (int j = 0; j < VE; ++j) {
                const int64_t e = e0 + j;
                if (e < a || e >= c) continue;
                float s = -0.0f;
                for (int k = 0; k < P; ++k)
                    s = s + grad_elem<BF16>(grad_tab[(size_t)ring_worker(start, k, P) * L + t.layer], e);
                dst[e - a] = s * inv_P;
            }
        }
    }
}

// Reduce-scatter of one tile per workgroup (paper Sec. III-A; Eq. 2 for the 1/P).
// Summation starts at worker s+1 and ends with worker s, the order in which the ring
// delivers the partial sums of chunk s to its owner.  The accumulator starts as -0.0f,
// the additive identity that keeps the first addend's bits (including a -0.0f).
template <bool BF16, int CH, bool TAIL>
__global__ __launch_bounds__(DEAR_BLOCK) void reduce_scatter_kernel(
    const dear_tile *__restrict__ tiles, const void *const *__restrict__ grad_tab, int L, int P,
    float inv_P, float *__restrict__ shard_grad)
{
    const dear_tile t = tiles[blockIdx.x];
    float *__restrict__ dst = shard_grad + t.dst_begin;
    if (t.layer < 0) {  // padding slots reduce to +0
        for (int i = threadIdx.x; i < t.count; i += DEAR_BLOCK) dst[i] = 0.0f;
        return;
    }
    if (t.count == DEAR_TILE_ELEMS)
        reduce_scatter_tile<BF16, CH, TAIL, true>(t, grad_tab, L, P, inv_P, dst);
    else
        reduce_scatter_tile<BF16, CH, TAIL, false>(t, grad_tab, L, P, inv_P, dst);
}

// SGD with momentum on contiguous shard slots (paper Eq. 1-2): v = mu*v + g; w = w - lr*v.
// blockIdx.y selects the row (worker); each row segment is `vecs` 16-byte vectors long.
constexpr int UPD_U = 4;
__global__ __launch_bounds__(DEAR_BLOCK) void shard_update_kernel(
    const float *__restrict__ g, float *__restrict__ w, float *__restrict__ v, int64_t row_stride,
    int64_t base, int64_t vecs, float lr, float mu)
{
    const int64_t off = (int64_t)blockIdx.y * row_stride + base;
    const f4 *__restrict__ g4 = reinterpret_cast<const f4 *>(g + off);
    f4 *__restrict__ w4 = reinterpret_cast<f4 *>(w + off);
    f4 *__restrict__ v4 = reinterpret_cast<f4 *>(v + off);
    const int64_t first = (int64_t)blockIdx.x * (UPD_U * DEAR_BLOCK) + threadIdx.x;
    f4 gg[UPD_U], ww[UPD_U], vv[UPD_U];
#pragma unroll
    for (int u = 0; u < UPD_U; ++u) {
        const int64_t i = first + u * DEAR_BLOCK;
        if (i < vecs) {
            gg[u] = __builtin_nontemporal_load(g4 + i);
            ww[u] = __builtin_nontemporal_load(w4 + i);
            vv[u] = __builtin_nontemporal_load(v4 + i);
        }
    }
#pragma unroll
    for (int u = 0; u < UPD_U; ++u) {
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
            v4[i] = nv;
            w4[i] = nw;
        }
    }
}

// All-gather of one tile per workgroup with the copy-back to the layer tensors folded in
// (paper Sec. III-A, IV-A): each shard value is read once and stored to all P replicas.
template <bool ALL_FULL>
__device__ __forceinline__ void all_gather_tile(const dear_tile &t, float *const *__restrict__ param_tab,
                                                int L, int P, const float *__restrict__ src)
{
    constexpr int VE = 4;
    constexpr int U = DEAR_TILE_ELEMS / (VE * DEAR_BLOCK);
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
        if (full[u]) val[u] = __builtin_nontemporal_load((global_f4u_in)(src + (e0 - a)));
    }
    for (int p = 0; p < P; ++p) {
        global_f4_out out = (global_f4_out)param_tab[(size_t)p * L + t.layer];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (full[u]) __builtin_nontemporal_store(val[u], out + vi[u]);
    }
    if (ALL_FULL) return;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t e0 = vi[u] * VE;
        if (!full[u] && e0 < c) {
            for (int j = 0; j < VE; ++j) {
                const int64_t e = e0 + j;
                if (e < a || e >= c) continue;
                const float x = src[e - a];
                for (int p = 0; p < P; ++p) ((DEAR_GLOBAL float *)param_tab[(size_t)p * L + t.layer])[e] = x;
            }
        }
    }
}

__global__ __launch_bounds__(DEAR_BLOCK) void all_gather_kernel(
    const dear_tile *__restrict__ tiles, float *const *__restrict__ param_tab, int L, int P,
    const float *__restrict__ shard_param)
{
    const dear_tile t = tiles[blockIdx.x];
    if (t.layer < 0) return;
    const float *__restrict__ src = shard_param + t.dst_begin;
    if (t.count == DEAR_TILE_ELEMS)
        all_gather_tile<true>(t, param_tab, L, P, src);
    else
        all_gather_tile<false>(t, param_tab, L, P, src);
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

template <bool BF16>
void rs_launch_dtype(int P, dim3 grid, dim3 block, hipStream_t st, const dear_tile *tiles,
                     const void *const *grad_tab, int L, float inv_P, float *shard_grad)
{
    // replicas per load batch: the largest of 8/4/2/1 that divides P without a tail when
    // P is small or a multiple of 4; otherwise batches of 8 with a predicated tail
    if (P % 8 == 0)
        reduce_scatter_kernel<BF16, 8, false><<<grid, block, 0, st>>>(tiles, grad_tab, L, P, inv_P, shard_grad);
    else if (P % 4 == 0)
        reduce_scatter_kernel<BF16, 4, false><<<grid, block, 0, st>>>(tiles, grad_tab, L, P, inv_P, shard_grad);
    else if (P == 2)
        reduce_scatter_kernel<BF16, 2, false><<<grid, block, 0, st>>>(tiles, grad_tab, L, P, inv_P, shard_grad);
    else if (P == 1)
        reduce_scatter_kernel<BF16, 1, false><<<grid, block, 0, st>>>(tiles, grad_tab, L, P, inv_P, shard_grad);
    else
        reduce_scatter_kernel<BF16, 8, true><<<grid, block, 0, st>>>(tiles, grad_tab, L, P, inv_P, shard_grad);
}

void rs_launch(bool bf16, int P, dim3 grid, dim3 block, hipStream_t st, const dear_tile *tiles,
               const void *const *grad_tab, int L, float inv_P, float *shard_grad)
{
    if (bf16)
        rs_launch_dtype<true>(P, grid, block, st, tiles, grad_tab, L, inv_P, shard_grad);
    else
        rs_launch_dtype<false>(P, grid, block, st, tiles, grad_tab, L, inv_P, shard_grad);
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
    if (tiles.size() > 0x7fffffffu) return DEAR_EINVAL;  // grid.x limit
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
    const float inv_P = 1.0f / static_cast<float>(c->P);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid(static_cast<unsigned>(count)), block(DEAR_BLOCK);
    rs_launch(c->g == 2, c->P, grid, block, st, c->d_tiles + first, c->d_grad, c->L, inv_P, shard_grad);
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
    const int64_t per_block = static_cast<int64_t>(UPD_U) * DEAR_BLOCK;
    const int64_t blocks = (vecs + per_block - 1) / per_block;
    if (blocks == 0) return DEAR_OK;
    if (blocks > 0x7fffffff || rows > 65535u) return DEAR_EINVAL;
    shard_update_kernel<<<dim3(static_cast<unsigned>(blocks), rows), dim3(DEAR_BLOCK), 0,
                          static_cast<hipStream_t>(hip_stream)>>>(shard_grad, shard_param, shard_mom,
                                                                  c->row_len, base, vecs, lr, momentum);
    return launch_status();
}

extern "C" int dear_all_gather(dear_ctx_t *c, int32_t bucket, const float *shard_param, void *hip_stream)
{
    int rc = check_call(c, bucket);
    if (rc == DEAR_OK) rc = check_shard_buffer(shard_param);
    if (rc != DEAR_OK) return rc;
    int64_t first, count;
    tile_range(c, bucket, first, count);
    if (count == 0) return DEAR_OK;
    all_gather_kernel<<<dim3(static_cast<unsigned>(count)), dim3(DEAR_BLOCK), 0,
                        static_cast<hipStream_t>(hip_stream)>>>(c->d_tiles + first, c->d_param, c->L, c->P,
                                                                shard_param);
    return launch_status();
}

extern "C" int dear_scatter_params(dear_ctx_t *c, int32_t worker, float *shard_param, void *hip_stream)
{
    if (!c) return DEAR_EINVAL;
    if (worker < 0 || worker >= c->P) return DEAR_ERANGE;
    int rc = check_shard_buffer(shard_param);
    if (rc != DEAR_OK) return rc;
    const int64_t count = c->tile_begin[c->B];
    if (count == 0) return DEAR_OK;
    scatter_params_kernel<<<dim3(static_cast<unsigned>(count)), dim3(DEAR_BLOCK), 0,
                            static_cast<hipStream_t>(hip_stream)>>>(c->d_tiles, c->d_param, c->L, worker,
                                                                    shard_param);
    return launch_status();
}
