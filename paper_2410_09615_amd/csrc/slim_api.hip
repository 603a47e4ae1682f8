// Host-only parts of the boundary: status text, size queries, workspace plan.
#include "slim_internal.h"

#include <atomic>
#include <mutex>

namespace slim {

static size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

DeviceInfo device_info()
{
    constexpr int kSlots = 64;
    static DeviceInfo table[kSlots];
    static std::atomic<int> known[kSlots];
    const DeviceInfo nominal{256, (size_t)160 * 1024};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kSlots) {
        (void)hipGetLastError();         // no device: the error must not surface in a later call
        return nominal;
    }
    if (known[dev].load(std::memory_order_acquire)) return table[dev];
    static std::mutex mu;
    std::lock_guard<std::mutex> lock(mu);
    if (!known[dev].load(std::memory_order_acquire)) {
        DeviceInfo d = nominal;
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) {
            if (prop.multiProcessorCount > 0) d.cus = prop.multiProcessorCount;
            // the kernels are laid out for at most 160 KiB per workgroup
            const size_t lds = prop.maxSharedMemoryPerMultiProcessor;
            if (lds >= 64 * 1024 && lds < d.lds) d.lds = lds;
        } else {
            (void)hipGetLastError();
        }
        table[dev] = d;
        known[dev].store(1, std::memory_order_release);
    }
    return table[dev];
}

static std::atomic<int> g_decode_path{-1};
static std::atomic<int> g_decode_lds_kb{0};
int decode_path_override() { return g_decode_path.load(std::memory_order_relaxed); }
size_t decode_lds_limit() { return (size_t)g_decode_lds_kb.load(std::memory_order_relaxed) * 1024; }

int gemm_t_splits(int32_t m, int32_t rank_pad, int32_t k);   // slim_gemm.hip

WorkspacePlan plan_workspace(int32_t n, int32_t k, int32_t rank_pad, int32_t m, bool q4)
{
    WorkspacePlan p{};
    p.dec_off = 0;
    p.t16_off = p.dec_off + 256 + 2 * round256((size_t)16 * rank_pad * sizeof(float));
    p.dec_bytes = p.t16_off + round256((size_t)4 * 16 * (rank_pad / 4) * 16) - p.dec_off;
    p.t_off = p.dec_off + p.dec_bytes;
    p.t_bytes = m > 16 ? round256((size_t)m * rank_pad * sizeof(uint16_t)) : 0;
    p.acc_off = p.t_off + p.t_bytes;
    p.acc_bytes = m <= 16 ? round256((size_t)plan_decode(n, k, rank_pad, m).slots * m * n * sizeof(float)) : 0;
    p.part_off = p.acc_off + p.acc_bytes;
    p.splits = rank_pad > 0 ? gemm_t_splits(m, rank_pad, k) : 1;
    p.part_bytes = p.splits > 1 ? round256((size_t)p.splits * m * rank_pad * sizeof(float)) : 0;
    p.exp_off = p.part_off + p.part_bytes;
    // (the prefill kernels read the 4-bit codes themselves; the two-launch decode kernels read fp16)
    p.exp_bytes = q4 && rank_pad > 0 && m <= 16 ? round256(tl_bytes(n, rank_pad)) + round256(tl_bytes(rank_pad, k)) : 0;
    p.total = p.exp_off + p.exp_bytes;
    if (p.total < 256) p.total = 256;
    return p;
}

void launch_q4_expand(const uint8_t *codes, const half_t *scales, int rows, int K, int rows_t, int cols_t, half_t *out,
                      hipStream_t st);   // slim_adapters_q4.hip

int expand_q4_adapters(const slim_layer *layer, const WorkspacePlan &w, char *ws, slim_layer *out, hipStream_t st)
{
    const slim_shape s = layer->shape;
    const int rp = layer->rank_pad;
    half_t *Lx = reinterpret_cast<half_t *>(ws + w.exp_off);
    half_t *Rx = reinterpret_cast<half_t *>(ws + w.exp_off + round256(tl_bytes(s.n, rp)));
    launch_q4_expand(layer->Lq, reinterpret_cast<const half_t *>(layer->Ls), s.n, s.rank, (int)tl_rows(s.n), (int)tl_cols(rp), Lx, st);
    launch_q4_expand(layer->Rq, reinterpret_cast<const half_t *>(layer->Rs), s.rank, s.k, (int)tl_rows(rp), (int)tl_cols(s.k), Rx, st);
    *out = *layer;
    out->L = reinterpret_cast<const slim_half *>(Lx);
    out->R = reinterpret_cast<const slim_half *>(Rx);
    out->adapter_bits = 16;
    return hip_status(hipGetLastError());
}

}  // namespace slim

using namespace slim;

extern "C" const char *slim_status_string(int status)
{
    switch (status) {
        case SLIM_OK: return "ok";
        case SLIM_ERR_NULL: return "a required pointer is NULL";
        case SLIM_ERR_SHAPE: return "a dimension is outside the supported range";
        case SLIM_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case SLIM_ERR_WORKSPACE: return "workspace is NULL or too small";
        case SLIM_ERR_HIP: return "a HIP runtime call failed";
        case SLIM_ERR_WAIT: return "a decode call gave up waiting for its own intermediate result";
        default: return "unknown status";
    }
}

extern "C" int slim_decode_override(int32_t path, int32_t lds_kb)
{
    if (path < -1 || path > 3) return SLIM_ERR_SHAPE;
    if (lds_kb != 0 && (lds_kb < 16 || lds_kb > 160)) return SLIM_ERR_SHAPE;
    g_decode_path.store(path, std::memory_order_relaxed);
    g_decode_lds_kb.store(lds_kb, std::memory_order_relaxed);
    return SLIM_OK;
}

extern "C" int slim_workspace_check(void *workspace, void *stream)
{
    char *ws = static_cast<char *>(workspace);
    if (!ws) {
        void *own = nullptr;
        const int rc = scratch_of_current_device(&own);
        if (rc != SLIM_OK) return rc;
        ws = static_cast<char *>(own);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned flag = 0;
    if (hipMemcpyAsync(&flag, ws + 8, sizeof(flag), hipMemcpyDeviceToHost, st) != hipSuccess) return SLIM_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return SLIM_ERR_HIP;
    if (!flag) return SLIM_OK;
    flag = 0;
    if (hipMemcpyAsync(ws + 8, &flag, sizeof(flag), hipMemcpyHostToDevice, st) != hipSuccess) return SLIM_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return SLIM_ERR_HIP;
    return SLIM_ERR_WAIT;
}

extern "C" int32_t slim_rank_pad(int32_t rank) { return rank <= 0 ? 0 : (rank + 31) / 32 * 32; }

extern "C" int slim_packed_sizes(slim_shape shape, size_t *qvals_bytes, size_t *meta_bytes, size_t *scale_bytes,
                                 int32_t *rank_pad, size_t *L_bytes, size_t *R_bytes)
{
    if (shape.n < 1 || shape.k < 8 || shape.k % 8 || shape.rank < 0) return SLIM_ERR_SHAPE;
    int32_t rp = slim_rank_pad(shape.rank);
    if (qvals_bytes) *qvals_bytes = pk_qbytes(shape.n, shape.k);
    if (meta_bytes) *meta_bytes = pk_mbytes(shape.n, shape.k);
    if (scale_bytes) *scale_bytes = (size_t)shape.n * sizeof(float);
    if (rank_pad) *rank_pad = rp;
    if (L_bytes) *L_bytes = rp ? tl_bytes(shape.n, rp) : 0;
    if (R_bytes) *R_bytes = rp ? tl_bytes(rp, shape.k) : 0;
    return SLIM_OK;
}

extern "C" int slim_workspace_bytes(const slim_layer *layer, int32_t m, size_t *bytes)
{
    if (!layer || !bytes) return SLIM_ERR_NULL;
    const slim_shape s = layer->shape;
    if (s.n < 1 || s.k < 8 || s.k % 8 || s.rank < 0 || m < 1) return SLIM_ERR_SHAPE;
    if (layer->rank_pad != slim_rank_pad(s.rank)) return SLIM_ERR_SHAPE;
    *bytes = plan_workspace(s.n, s.k, layer->rank_pad, m, layer->adapter_bits == 4).total;
    return SLIM_OK;
}
