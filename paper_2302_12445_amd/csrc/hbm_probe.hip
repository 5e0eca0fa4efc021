// libdear_probe: bare HBM traffic patterns of the aggregation kernels (see dear_probe.h).
// 256-thread workgroups, one 16-byte vector per lane and stream, non-temporal accesses:
// the same access width and cache hints as the real kernels, nothing else.
#include <hip/hip_runtime.h>

#include <vector>

#include "dear_probe.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
#define PROBE_GLOBAL __attribute__((address_space(1)))
constexpr int BLOCK = 256;
constexpr int MAX_K = 64;

struct stream_table {
    void *ptr[MAX_K];
};

// k inputs -> 1 output.  IN_HALF: inputs are 2-byte elements, so one 16-byte input vector
// yields two 16-byte output vectors.
template <bool IN_HALF>
__global__ __launch_bounds__(BLOCK) void read_k_write_1(stream_table in, int k, f4 *__restrict__ out, int64_t in_vecs)
{
    const int64_t i = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i >= in_vecs) return;
    f4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < k; k0 += 8) {
        u4 raw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (k0 + j < k) raw[j] = __builtin_nontemporal_load((const PROBE_GLOBAL u4 *)in.ptr[k0 + j] + i);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (k0 + j < k) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (IN_HALF) {
                        lo[c] += __uint_as_float(raw[j][c] << 16);
                        hi[c] += __uint_as_float(raw[j][c] & 0xffff0000u);
                    } else {
                        lo[c] += __uint_as_float(raw[j][c]);
                    }
                }
            }
    }
    if (IN_HALF) {
        __builtin_nontemporal_store(lo, (PROBE_GLOBAL f4 *)out + 2 * i);
        __builtin_nontemporal_store(hi, (PROBE_GLOBAL f4 *)out + 2 * i + 1);
    } else {
        __builtin_nontemporal_store(lo, (PROBE_GLOBAL f4 *)out + i);
    }
}

__global__ __launch_bounds__(BLOCK) void read_1_write_k(const f4 *__restrict__ in, stream_table out, int k, int64_t vecs)
{
    const int64_t i = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i >= vecs) return;
    const f4 v = in[i];
    for (int j = 0; j < k; ++j) __builtin_nontemporal_store(v, (PROBE_GLOBAL f4 *)out.ptr[j] + i);
}

// workgroup -> (chunk, stream, part): the chip writes one stream's chunk at a time
__global__ __launch_bounds__(BLOCK) void read_1_write_k_chunked(const f4 *__restrict__ in, stream_table out, int k,
                                                                int64_t vecs, int64_t chunk_blocks)
{
    const int64_t per_chunk = chunk_blocks * k;
    const int64_t chunk = blockIdx.x / per_chunk;
    const int64_t r = blockIdx.x - chunk * per_chunk;
    const int64_t total_blocks = (vecs + BLOCK - 1) / BLOCK;
    const int64_t first = chunk * chunk_blocks;
    const int64_t len = total_blocks - first < chunk_blocks ? total_blocks - first : chunk_blocks;
    const int64_t j = r / len;
    const int64_t i = (first + (r - j * len)) * BLOCK + threadIdx.x;
    if (j >= k || i >= vecs) return;
    __builtin_nontemporal_store(in[i], (PROBE_GLOBAL f4 *)out.ptr[j] + i);
}

__global__ __launch_bounds__(BLOCK) void read_3_write_2(const f4 *__restrict__ a, f4 *__restrict__ b, f4 *__restrict__ c,
                                                        int64_t vecs)
{
    const int64_t i0 = (int64_t)blockIdx.x * (2 * BLOCK) + threadIdx.x;
    f4 x[2], y[2], z[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int64_t i = i0 + u * BLOCK;
        if (i < vecs) {
            x[u] = __builtin_nontemporal_load(a + i);
            y[u] = __builtin_nontemporal_load(b + i);
            z[u] = __builtin_nontemporal_load(c + i);
        }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int64_t i = i0 + u * BLOCK;
        if (i < vecs) {
            __builtin_nontemporal_store(x[u] + z[u], c + i);
            __builtin_nontemporal_store(y[u] + x[u], b + i);
        }
    }
}

struct buffers {
    std::vector<void *> all;
    ~buffers()
    {
        for (void *p : all) (void)hipFree(p);
    }
    // `lead` unused bytes in front: stream j of a pattern starts j*skew into its allocation
    void *get(size_t bytes, size_t lead = 0)
    {
        void *p = nullptr;
        if (hipMalloc(&p, bytes + lead) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        all.push_back(p);
        if (hipMemset(p, 0, bytes + lead) != hipSuccess) return nullptr;
        return static_cast<unsigned char *>(p) + lead;
    }
};

}  // namespace

extern "C" int dear_probe_streams(int32_t pattern, int32_t k, int64_t bytes_per_stream, int64_t chunk_bytes,
                                  int32_t elem_bytes_in, int64_t skew_bytes, int32_t reps, double *gbytes_per_s,
                                  double *avg_ms)
{
    if (skew_bytes < 0 || skew_bytes % 256 || skew_bytes > (1 << 26)) return -1;
    if (!gbytes_per_s || reps < 1 || bytes_per_stream < 4096 || bytes_per_stream % 4096) return -1;
    if (pattern < DEAR_PROBE_READ_K_WRITE_1 || pattern > DEAR_PROBE_READ_3_WRITE_2) return -1;
    if (pattern != DEAR_PROBE_READ_3_WRITE_2 && (k < 1 || k > MAX_K)) return -1;
    if (elem_bytes_in != 4 && !(elem_bytes_in == 2 && pattern == DEAR_PROBE_READ_K_WRITE_1)) return -1;
    if (pattern == DEAR_PROBE_READ_1_WRITE_K_CHUNKED && (chunk_bytes < 4096 || chunk_bytes % 4096)) return -1;
    const int64_t vecs = bytes_per_stream / 16;
    const int64_t blocks = (vecs + BLOCK - 1) / BLOCK;
    if (blocks * (pattern == DEAR_PROBE_READ_1_WRITE_K_CHUNKED ? k : 1) > 0x7fffffff) return -1;

    buffers mem;
    stream_table tab = {};
    double bytes_moved = 0;
    void *single = nullptr;
    if (pattern == DEAR_PROBE_READ_3_WRITE_2) {
        for (int j = 0; j < 3; ++j)
            if (!(tab.ptr[j] = mem.get(bytes_per_stream))) return -2;
        bytes_moved = 5.0 * bytes_per_stream;
    } else {
        for (int j = 0; j < k; ++j)
            if (!(tab.ptr[j] = mem.get(bytes_per_stream, static_cast<size_t>(j) * skew_bytes))) return -2;
        const int64_t single_bytes = (pattern == DEAR_PROBE_READ_K_WRITE_1 && elem_bytes_in == 2) ? 2 * bytes_per_stream
                                                                                                    : bytes_per_stream;
        if (!(single = mem.get(single_bytes))) return -2;
        bytes_moved = (double)k * bytes_per_stream + single_bytes;
    }

    auto launch = [&]() {
        switch (pattern) {
        case DEAR_PROBE_READ_K_WRITE_1:
            if (elem_bytes_in == 2)
                read_k_write_1<true><<<dim3((unsigned)blocks), dim3(BLOCK)>>>(tab, k, (f4 *)single, vecs);
            else
                read_k_write_1<false><<<dim3((unsigned)blocks), dim3(BLOCK)>>>(tab, k, (f4 *)single, vecs);
            break;
        case DEAR_PROBE_READ_1_WRITE_K:
            read_1_write_k<<<dim3((unsigned)blocks), dim3(BLOCK)>>>((const f4 *)single, tab, k, vecs);
            break;
        case DEAR_PROBE_READ_1_WRITE_K_CHUNKED:
            read_1_write_k_chunked<<<dim3((unsigned)(blocks * k)), dim3(BLOCK)>>>((const f4 *)single, tab, k, vecs,
                                                                                 chunk_bytes / (16 * BLOCK));
            break;
        default:
            read_3_write_2<<<dim3((unsigned)((vecs + 2 * BLOCK - 1) / (2 * BLOCK))), dim3(BLOCK)>>>(
                (const f4 *)tab.ptr[0], (f4 *)tab.ptr[1], (f4 *)tab.ptr[2], vecs);
        }
    };

    hipEvent_t t0 = nullptr, t1 = nullptr;
    if (hipEventCreate(&t0) != hipSuccess || hipEventCreate(&t1) != hipSuccess) return -3;
    int rc = 0;
    float ms = 0.f;
    launch();
    launch();
    if (hipDeviceSynchronize() != hipSuccess || hipGetLastError() != hipSuccess) rc = -3;
    if (rc == 0) {
        (void)hipEventRecord(t0, nullptr);
        for (int r = 0; r < reps; ++r) launch();
        (void)hipEventRecord(t1, nullptr);
        if (hipEventSynchronize(t1) != hipSuccess || hipGetLastError() != hipSuccess ||
            hipEventElapsedTime(&ms, t0, t1) != hipSuccess)
            rc = -3;
    }
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (rc != 0) return rc;
    const double per_launch_ms = ms / reps;
    *gbytes_per_s = bytes_moved / (per_launch_ms * 1e-3) / 1e9;
    if (avg_ms) *avg_ms = per_launch_ms;
    return 0;
}
