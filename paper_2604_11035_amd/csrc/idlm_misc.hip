// Error strings, version, and two plain streaming kernels used to calibrate byte counters and
// to measure the bandwidth a pure copy / pure read reaches on the device.
#include "idlm_common.h"
#include "isd_accept_common.h"

namespace idlm {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// One workgroup per 64 KB: sixteen independent 16-byte loads per lane, all in flight at once.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink)
{
    const size_t base = (size_t)blockIdx.x * 4096 + threadIdx.x;
    u32x4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const size_t i = base + (size_t)u * 256;
        v[u] = (i < n16) ? __builtin_nontemporal_load(src + i) : u32x4{0u, 0u, 0u, 0u};
    }
    uint32_t acc = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    // fold the wavefront's words and let one lane per wavefront touch the sink: keeps every load alive
    for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0 && acc == 0x9E3779B9u) atomicXor(sink, acc);
}

// The uniform and the Gumbel noise that element i of logit row row0 + r draws under a stream tag:
// the same device functions the acceptance kernels call, written out for inspection.
__global__ __launch_bounds__(256) void rng_dump_kernel(uint2 key, uint32_t offset, uint32_t stream_tag, uint32_t row0,
                                                        int V, float* __restrict__ uniforms, float* __restrict__ gumbels)
{
    const int r = blockIdx.y;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < V; i += gridDim.x * 256) {
        const uint4 w = philox4x32_10(make_uint4((uint32_t)i >> 2, row0 + (uint32_t)r, stream_tag, offset), key);
        const uint32_t word = (i & 3) == 0 ? w.x : (i & 3) == 1 ? w.y : (i & 3) == 2 ? w.z : w.w;
        if (uniforms) uniforms[(size_t)r * V + i] = unit_uniform(word);
        if (gumbels) gumbels[(size_t)r * V + i] = gumbel(word);
    }
}

}  // namespace idlm

using namespace idlm;

extern "C" int idlm_isd_rng_dump(uint64_t rng_seed, uint32_t rng_offset, int32_t stream_tag, int32_t row0, int32_t n_rows,
                                 int32_t V, float* uniforms, float* gumbels, void* stream)
{
    if (n_rows < 0 || n_rows > 65535 || V < 1 || row0 < 0 || stream_tag < 0 || (int64_t)row0 + n_rows > INT32_MAX)
        return IDLM_ERR_SHAPE;
    if (n_rows == 0) return IDLM_OK;
    if (!uniforms && !gumbels) return IDLM_ERR_NULL;
    (void)hipGetLastError();
    const int64_t blocks = ((int64_t)V + 255) / 256;
    const unsigned gx = (unsigned)(blocks < 1024 ? blocks : 1024);
    hipLaunchKernelGGL(rng_dump_kernel, dim3(gx, (unsigned)n_rows), dim3(256), 0, static_cast<hipStream_t>(stream),
                       make_uint2((uint32_t)rng_seed, (uint32_t)(rng_seed >> 32)), rng_offset, (uint32_t)stream_tag,
                       (uint32_t)row0, V, uniforms, gumbels);
    return launch_status();
}

extern "C" const char* idlm_strerror(int code)
{
    switch (code) {
        case IDLM_OK: return "ok";
        case IDLM_ERR_NULL: return "a required pointer is NULL";
        case IDLM_ERR_SHAPE: return "a size is outside the supported range";
        case IDLM_ERR_DTYPE: return "unknown dtype or unsupported dtype/shape combination";
        case IDLM_ERR_ALIGN: return "a pointer or stride is not aligned as required";
        case IDLM_ERR_WORKSPACE: return "workspace missing or too small";
        case IDLM_ERR_LAUNCH: return "the HIP runtime refused the launch";
        case IDLM_ERR_CONTENT: return "a device array breaks a precondition (see the report of idlm_isd_validate)";
        default: return "unknown idlm error code";
    }
}

extern "C" int idlm_version(void) { return IDLM_VERSION; }

namespace idlm {

__global__ void validate_clear_kernel(int32_t* report)
{
    if (threadIdx.x < 4) report[threadIdx.x] = threadIdx.x == 1 ? INT32_MAX : 0;
}

// One wavefront per sequence: its length, the page ids it will read, its draft count and draft ids.
__global__ __launch_bounds__(64) void validate_kernel(const int32_t* __restrict__ block_table,
                                                     const int32_t* __restrict__ ctx_lens, int S, int B, int P,
                                                     int num_pages, int max_pages,
                                                     const int32_t* __restrict__ draft_tokens,
                                                     const int32_t* __restrict__ n_draft, int n_draft_uniform, int V,
                                                     int32_t* report)
{
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    int bad = 0;
    if (ctx_lens) {
        const int ctx = ctx_lens[b];
        if (ctx < S) bad |= IDLM_BAD_CTX_SHORT;
        if (block_table && (int64_t)ctx > (int64_t)max_pages * P) bad |= IDLM_BAD_CTX_LONG;
        if (block_table && ctx > 0) {
            const int npages = (int)min((int64_t)max_pages, ((int64_t)ctx + P - 1) / P);
            for (int pg = lane; pg < npages; pg += 64) {
                const int id = block_table[(size_t)b * max_pages + pg];
                if (id < 0 || id >= num_pages) bad |= IDLM_BAD_PAGE_ID;
            }
        }
    }
    int nd = n_draft ? n_draft[b] : n_draft_uniform;
    if (nd < 0 || nd > S - 1) { bad |= IDLM_BAD_N_DRAFT; nd = max(0, min(nd, S - 1)); }
    if (draft_tokens && lane < nd) {
        const int x = draft_tokens[(size_t)b * (S - 1) + lane];
        if (x < 0 || x >= V) bad |= IDLM_BAD_DRAFT_ID;
    }
    if (bad) {
        atomicOr(&report[0], bad);
        atomicMin(&report[1], b);
    }
}

}  // namespace idlm

extern "C" int idlm_isd_validate(const int32_t* block_table, const int32_t* ctx_lens, int32_t S, int32_t B, int32_t P,
                                 int32_t num_pages, int32_t max_pages_per_seq, const int32_t* draft_tokens,
                                 const int32_t* n_draft, int32_t n_draft_uniform, int32_t V, int32_t* report,
                                 int32_t* host_report, void* stream)
{
    if (B < 0 || S < 1 || S > 64 || P < 1 || num_pages < 0 || max_pages_per_seq < 0 || V < 1) return IDLM_ERR_SHAPE;
    if (!report) return IDLM_ERR_NULL;
    if (B == 0) {
        if (host_report) { host_report[0] = 0; host_report[1] = -1; host_report[2] = host_report[3] = 0; }
        return IDLM_OK;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    hipLaunchKernelGGL(idlm::validate_clear_kernel, dim3(1), dim3(64), 0, st, report);
    hipLaunchKernelGGL(idlm::validate_kernel, dim3((unsigned)B), dim3(64), 0, st, block_table, ctx_lens, S, B, P, num_pages,
                       max_pages_per_seq, draft_tokens, n_draft, n_draft_uniform, V, report);
    int32_t host[4] = {0, 0, 0, 0};
    if (hipMemcpyAsync(host, report, sizeof host, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess)
        return IDLM_ERR_LAUNCH;
    if (host[1] == INT32_MAX) host[1] = -1;
    if (host_report) { host_report[0] = host[0]; host_report[1] = host[1]; host_report[2] = host[2]; host_report[3] = host[3]; }
    return host[0] ? IDLM_ERR_CONTENT : IDLM_OK;
}

extern "C" int idlm_stream_copy(const void* src, void* dst, size_t n_bytes, void* stream)
{
    if (n_bytes == 0) return IDLM_OK;
    if (!src || !dst) return IDLM_ERR_NULL;
    if (n_bytes % 16) return IDLM_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 16)) return IDLM_ERR_ALIGN;
    const size_t n16 = n_bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    (void)hipGetLastError();
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
    return launch_status();
}

extern "C" int idlm_stream_read(const void* src, size_t n_bytes, uint32_t* sink, void* stream)
{
    if (n_bytes == 0) return IDLM_OK;
    if (!src || !sink) return IDLM_ERR_NULL;
    if (n_bytes % 16) return IDLM_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(sink, 4)) return IDLM_ERR_ALIGN;
    const size_t n16 = n_bytes / 16;
    const size_t blocks = (n16 + 4095) / 4096;
    if (blocks > 0x7fffffffu) return IDLM_ERR_SHAPE;
    (void)hipGetLastError();
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), n16, sink);
    return launch_status();
}
