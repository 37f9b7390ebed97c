// C-ABI entry points of libitq3s: argument validation on the host, then launches.  See
// include/itq3s.h for the contract of every call (include/itq3s_bench.h for the measurement aids).
#include "../../include/itq3s.h"
#include "../../include/itq3s_bench.h"
#include "itq3s_kernels.h"

#include <atomic>
#include <mutex>

// Scratch of itq3s_matmul_static: one array per device the library runs on, held until the process
// ends.  The name below is a host-side stand-in for the symbol; device code gets the address that
// hipGetSymbolAddress returns for the current device (scratch_of_current_device).
static __device__ __align__(256) unsigned char scratch[ITQ3S_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Address of `scratch` on the current device (looked up once per device), or null.
void* scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p != nullptr) return p;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return nullptr;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    return p;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int pad_m(int64_t M) {
    int mp = 1;
    while (mp < M) mp <<= 1;
    return mp;
}

struct WorkspacePlan {
    size_t xt_bytes, s_bytes, flag_bytes, partial_bytes, total;
};

// N = the largest tensor of the call (sizes the split-K shares of the tiled path)
constexpr int64_t kChunkedMaxM = 2 * itq3s::kGemvMaxM;  // up to here M > 16 runs as passes of the streaming kernel
constexpr int64_t kSubStreamingMaxM = 64;               // sub-block variant: up to here passes of four rows, the tiled weight-side kernel above

WorkspacePlan plan_workspace(int64_t M, int64_t N, int64_t K) {
    if (M > itq3s::kGemvMaxM && M <= kChunkedMaxM) return plan_workspace(itq3s::kGemvMaxM, N, K);
    WorkspacePlan p;
    if (M <= itq3s::kGemvFusedMaxM) {  // the streaming kernel rotates the activations itself: nothing to park
        p.xt_bytes = p.s_bytes = p.flag_bytes = p.partial_bytes = 0;
        p.total = 256;
        return p;
    }
    const int64_t rows = M <= itq3s::kGemvMaxM ? pad_m(M) : M;
    p.xt_bytes = round_up((size_t)rows * (size_t)K * 2, 256);
    // streaming path with a rotation launch: two sums per (block, row), see launch_rotate_frag
    p.s_bytes = M <= itq3s::kGemvMaxM ? round_up((size_t)rows * (size_t)(K / 256) * 8, 256) : 0;
    // tiled path: split-K flags, then the shares (layout: rotated activations | flags | shares)
    p.flag_bytes = M <= itq3s::kGemvMaxM ? 0 : 512;
    p.partial_bytes = M <= itq3s::kGemvMaxM ? 0 : round_up(itq3s::gemm_partial_bytes(M, N, K), 256);
    p.total = p.xt_bytes + p.s_bytes + p.flag_bytes + p.partial_bytes + 256;
    return p;
}

}  // namespace

namespace {
// a call with a pair of events armed for the contraction kernel's dispatch, then a wait
template <typename Call>
int timed(float* kernel_ms, Call call) {
    if (!kernel_ms) return ITQ3S_ERR_NULL;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return ITQ3S_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return ITQ3S_ERR_LAUNCH;
    }
    itq3s::set_launch_timing(e0, e1);
    int rc = call();
    const bool taken = itq3s::take_launch_timing().start == nullptr;  // (also disarms if validation returned before any launch)
    if (rc == ITQ3S_OK && taken) {
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(kernel_ms, e0, e1) != hipSuccess) rc = ITQ3S_ERR_LAUNCH;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
}  // namespace

extern "C" {

size_t itq3s_codes_bytes(int64_t N, int64_t K) {
    if (N <= 0 || K <= 0 || K % 256 != 0) return 0;
    return (size_t)((N + 15) / 16) * (size_t)(K / 256) * 1536u;
}

size_t itq3s_scales_bytes(int64_t N, int64_t K) {
    if (N <= 0 || K <= 0 || K % 256 != 0) return 0;
    return (size_t)((N + 15) / 16) * (size_t)(K / 256) * 64u;
}

size_t itq3s_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0 || K % 256 != 0) return 256;
    return plan_workspace(M, N, K).total;
}

int itq3s_quantize(const float* W, int64_t N, int64_t K, int64_t ldw, uint32_t* codes, uint32_t* scales, uint32_t* status_flags,
                   void* stream) {
    if (!W || !codes || !scales) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || K % 256 != 0 || ldw < K) return ITQ3S_ERR_SHAPE;
    if (((N + 15) / 16) * (K / 256) > 0x3fffffffLL) return ITQ3S_ERR_SHAPE;  // two workgroups per tile, 32-bit grid
    if (!aligned(W, 16) || ldw % 4 != 0 || !aligned(codes, 16) || !aligned(scales, 16) || (status_flags && !aligned(status_flags, 4)))
        return ITQ3S_ERR_ALIGN;
    return itq3s::launch_quantize(W, N, K, ldw, codes, scales, nullptr, status_flags, static_cast<hipStream_t>(stream));
}

int itq3s_roundtrip(const float* W, int64_t N, int64_t K, int64_t ldw, int block_size, uint8_t* codes_out, uint32_t* scales_out,
                    float* W_hat, int64_t ldo, double* err2, uint32_t* status_flags, void* stream) {
    if (!W) return ITQ3S_ERR_NULL;
    if (block_size != 32 && block_size != 64 && block_size != 128 && block_size != 256 && block_size != 512) return ITQ3S_ERR_SHAPE;
    if (N <= 0 || K <= 0 || K % block_size != 0 || ldw < K || (W_hat && ldo < K)) return ITQ3S_ERR_SHAPE;
    if (N > 0x7fffffffLL / ((K + 1023) / 1024)) return ITQ3S_ERR_SHAPE;  // one wavefront per 1024 channels of a row
    if (!aligned(W, 16) || ldw % 4 != 0 || (codes_out && !aligned(codes_out, 16)) || (scales_out && !aligned(scales_out, 4)) ||
        (W_hat && (!aligned(W_hat, 16) || ldo % 4 != 0)) || (err2 && !aligned(err2, 8)) || (status_flags && !aligned(status_flags, 4)))
        return ITQ3S_ERR_ALIGN;
    return itq3s::launch_roundtrip(W, N, K, ldw, block_size, codes_out, scales_out, W_hat, ldo, err2, status_flags,
                                   static_cast<hipStream_t>(stream));
}

int itq3s_dequantize(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, void* W_out, int out_dtype, int64_t ldo,
                     uint32_t* status_flags, void* stream) {
    if (!codes || !scales || !W_out) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || K % 256 != 0 || ldo < K) return ITQ3S_ERR_SHAPE;
    if (((N + 15) / 16) * (K / 256) > 0x7fffffffLL) return ITQ3S_ERR_SHAPE;
    if (out_dtype != ITQ3S_F32 && out_dtype != ITQ3S_F16) return ITQ3S_ERR_DTYPE;
    if (!aligned(W_out, 16) || ldo % 4 != 0 || !aligned(codes, 16) || !aligned(scales, 16) || (status_flags && !aligned(status_flags, 4)))
        return ITQ3S_ERR_ALIGN;
    return itq3s::launch_dequantize(codes, scales, nullptr, N, K, W_out, out_dtype == ITQ3S_F16, ldo, status_flags, static_cast<hipStream_t>(stream));
}

int itq3s_matmul_grouped(const itq3s_weight* w, int count, int64_t K, const void* X, int64_t M, int64_t ldx, int y_dtype, void* workspace,
                         size_t workspace_bytes, uint32_t* status_flags, void* stream) {
    if (!w || !X) return ITQ3S_ERR_NULL;
    if (count < 1 || count > ITQ3S_MAX_GROUP) return ITQ3S_ERR_SHAPE;
    if (K <= 0 || M <= 0 || K % 256 != 0 || ldx < K) return ITQ3S_ERR_SHAPE;
    if (y_dtype != ITQ3S_F32 && y_dtype != ITQ3S_F16) return ITQ3S_ERR_DTYPE;
    if (M > 0x7fffffffLL / (K / 256)) return ITQ3S_ERR_SHAPE;
    if (M > itq3s::kGemvMaxM && K > (1LL << 22)) return ITQ3S_ERR_SHAPE;  // the tiled kernel's 32-bit byte offsets
    if (K > (1LL << 28) || (M <= itq3s::kGemvFusedMaxM && (M - 1) * ldx + K > (1LL << 29))) return ITQ3S_ERR_SHAPE;  // 32-bit byte offsets of the streaming kernel
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        if (!w[i].codes || !w[i].scales || !w[i].Y) return ITQ3S_ERR_NULL;
        if (w[i].N <= 0 || w[i].ldy < w[i].N || (w[i].N + 15) / 16 > 0x7fffffffLL / (K / 256)) return ITQ3S_ERR_SHAPE;
        if (!aligned(w[i].codes, 16) || !aligned(w[i].scales, 16) || !aligned(w[i].Y, y_dtype == ITQ3S_F16 ? 2 : 4)) return ITQ3S_ERR_ALIGN;
        const size_t need_i = itq3s_matmul_workspace_bytes(M, w[i].N, K);
        if (need_i > need) need = need_i;
    }
    if (!aligned(X, 16) || ldx % 8 != 0 || (status_flags && !aligned(status_flags, 4))) return ITQ3S_ERR_ALIGN;
    if (!workspace || workspace_bytes < need) return ITQ3S_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return ITQ3S_ERR_ALIGN;

    hipStream_t st = static_cast<hipStream_t>(stream);
    if (M > itq3s::kGemvMaxM && M <= kChunkedMaxM) {
        // A few rows more than the streaming kernel takes at once: two passes of it over the weights
        // are still faster than the tiled kernel, whose 128-row tiles would be mostly empty.
        const size_t y_bytes = y_dtype == ITQ3S_F16 ? 2 : 4;
        for (int64_t m0 = 0; m0 < M; m0 += itq3s::kGemvMaxM) {
            itq3s_weight part[ITQ3S_MAX_GROUP];
            for (int i = 0; i < count; ++i) {
                part[i] = w[i];
                part[i].Y = static_cast<unsigned char*>(w[i].Y) + (size_t)m0 * (size_t)w[i].ldy * y_bytes;
            }
            const int64_t rows = M - m0 < itq3s::kGemvMaxM ? M - m0 : itq3s::kGemvMaxM;
            const int rc = itq3s_matmul_grouped(part, count, K, static_cast<const _Float16*>(X) + m0 * ldx, rows, ldx, y_dtype, workspace,
                                                workspace_bytes, status_flags, stream);
            if (rc != 0) return rc;
        }
        return ITQ3S_OK;
    }
    const WorkspacePlan p = plan_workspace(M, w[0].N, K);  // (the parts in front of the split-K shares do not depend on N)
    _Float16* Xt = static_cast<_Float16*>(workspace);
    const _Float16* Xh = static_cast<const _Float16*>(X);
    const int y_f16 = y_dtype == ITQ3S_F16;
    if (M <= itq3s::kGemvMaxM) {
        itq3s::GemvWeight gw[ITQ3S_MAX_GROUP];
        for (int i = 0; i < count; ++i) gw[i] = itq3s::GemvWeight{w[i].codes, w[i].scales, w[i].N, w[i].Y, w[i].ldy};
        if (M <= itq3s::kGemvFusedMaxM) return itq3s::launch_gemv(gw, count, K, Xh, ldx, M, y_f16, status_flags, st);
        const int MP = pad_m(M) < 8 ? 8 : pad_m(M);
        float* S = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + p.xt_bytes);
        int rc = itq3s::launch_rotate_frag(Xh, M, K, ldx, MP, Xt, S, status_flags, st);
        if (rc != 0) return rc;
        return itq3s::launch_gemv_rows(gw, count, K, Xt, S, M, MP, y_f16, status_flags, st);
    }
    // tiled path: one rotation, then one contraction launch per tensor
    unsigned char* const base = static_cast<unsigned char*>(workspace);
    uint32_t* zflags = reinterpret_cast<uint32_t*>(base + p.xt_bytes);
    float* partial = reinterpret_cast<float*>(base + p.xt_bytes + p.flag_bytes);
    const size_t partial_room = workspace_bytes - p.xt_bytes - p.flag_bytes;  // (checked above: every tensor's shares fit)
    static_assert(itq3s::kGemmFlagWords * 4 <= 512, "flag words fit their slot");
    int rc = itq3s::launch_rotate_rowmajor(Xh, M, K, ldx, Xt, zflags, itq3s::kGemmFlagWords, status_flags, st);
    for (int i = 0; i < count && rc == 0; ++i) {
        rc = itq3s::launch_gemm(w[i].codes, w[i].scales, w[i].N, K, Xt, Xh, ldx, M, w[i].Y, y_f16, w[i].ldy, partial, partial_room, zflags,
                                status_flags, st);
        // (the tensors of a group share the flag words: a flag left by an earlier tensor only costs the
        // later one a needless scan of its scale words)
    }
    return rc;
}

int itq3s_matmul(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const void* X, int64_t M, int64_t ldx, void* Y,
                 int y_dtype, int64_t ldy, void* workspace, size_t workspace_bytes, uint32_t* status_flags, void* stream) {
    if (!codes || !scales || !X || !Y) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || M <= 0 || K % 256 != 0 || ldx < K || ldy < N) return ITQ3S_ERR_SHAPE;
    const itq3s_weight w = {codes, scales, N, Y, ldy};
    return itq3s_matmul_grouped(&w, 1, K, X, M, ldx, y_dtype, workspace, workspace_bytes, status_flags, stream);
}

// ---- the sub-block-scale variant of the format (116 bytes per block)

size_t itq3s_subscales_bytes(int64_t N, int64_t K) {
    if (N <= 0 || K <= 0 || K % 256 != 0) return 0;
    return (size_t)((N + 15) / 16) * (size_t)(K / 256) * 256u;
}

int itq3s_quantize_sub(const float* W, int64_t N, int64_t K, int64_t ldw, uint32_t* codes, uint32_t* scales, uint32_t* subscales,
                       uint32_t* status_flags, void* stream) {
    if (!subscales) return ITQ3S_ERR_NULL;
    if (!aligned(subscales, 16)) return ITQ3S_ERR_ALIGN;
    if (!W || !codes || !scales) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || K % 256 != 0 || ldw < K) return ITQ3S_ERR_SHAPE;
    if (((N + 15) / 16) * (K / 256) > 0x3fffffffLL) return ITQ3S_ERR_SHAPE;
    if (!aligned(W, 16) || ldw % 4 != 0 || !aligned(codes, 16) || !aligned(scales, 16) || (status_flags && !aligned(status_flags, 4)))
        return ITQ3S_ERR_ALIGN;
    return itq3s::launch_quantize(W, N, K, ldw, codes, scales, subscales, status_flags, static_cast<hipStream_t>(stream));
}

int itq3s_dequantize_sub(const uint32_t* codes, const uint32_t* scales, const uint32_t* subscales, int64_t N, int64_t K, void* W_out,
                         int out_dtype, int64_t ldo, uint32_t* status_flags, void* stream) {
    if (!codes || !scales || !subscales || !W_out) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || K % 256 != 0 || ldo < K) return ITQ3S_ERR_SHAPE;
    if (((N + 15) / 16) * (K / 256) > 0x7fffffffLL) return ITQ3S_ERR_SHAPE;
    if (out_dtype != ITQ3S_F32 && out_dtype != ITQ3S_F16) return ITQ3S_ERR_DTYPE;
    if (!aligned(W_out, 16) || ldo % 4 != 0 || !aligned(codes, 16) || !aligned(scales, 16) || !aligned(subscales, 16) ||
        (status_flags && !aligned(status_flags, 4)))
        return ITQ3S_ERR_ALIGN;
    return itq3s::launch_dequantize(codes, scales, subscales, N, K, W_out, out_dtype == ITQ3S_F16, ldo, status_flags, static_cast<hipStream_t>(stream));
}

int itq3s_matmul_sub(const uint32_t* codes, const uint32_t* scales, const uint32_t* subscales, int64_t N, int64_t K, const void* X, int64_t M,
                     int64_t ldx, void* Y, int y_dtype, int64_t ldy, void* workspace, size_t workspace_bytes, uint32_t* status_flags, void* stream) {
    if (!codes || !scales || !subscales || !X || !Y) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || M <= 0 || K % 256 != 0 || ldx < K || ldy < N) return ITQ3S_ERR_SHAPE;
    if (K > (1LL << 28) || 3 * ldx + K > (1LL << 29) || (N + 15) / 16 > 0x7fffffffLL / (K / 256)) return ITQ3S_ERR_SHAPE;
    if (y_dtype != ITQ3S_F32 && y_dtype != ITQ3S_F16) return ITQ3S_ERR_DTYPE;
    if (!aligned(X, 16) || ldx % 8 != 0 || !aligned(codes, 16) || !aligned(scales, 16) || !aligned(subscales, 16) ||
        !aligned(Y, y_dtype == ITQ3S_F16 ? 2 : 4) || (status_flags && !aligned(status_flags, 4)))
        return ITQ3S_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int y_f16 = y_dtype == ITQ3S_F16;
    // many rows: the tiled kernel that reconstructs weight tiles on chip (one pass over the weights per 512 rows)
    if (M > kSubStreamingMaxM) {
        if ((M + 511) / 512 > 65535) return ITQ3S_ERR_SHAPE;
        return itq3s::launch_gemm_weight_side(codes, scales, subscales, N, K, static_cast<const _Float16*>(X), ldx, M, Y, y_f16, ldy, status_flags, st);
    }
    // the streaming kernel: passes of up to 16 rows; a pass of up to four rows rotates the activations
    // itself, a longer one takes them from a rotation launch through the workspace
    const WorkspacePlan p = plan_workspace(M < itq3s::kGemvMaxM ? M : itq3s::kGemvMaxM, N, K);
    if (M > itq3s::kGemvFusedMaxM) {
        if (!workspace || workspace_bytes < p.total) return ITQ3S_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return ITQ3S_ERR_ALIGN;
    }
    const size_t y_bytes = y_f16 ? 2 : 4;
    for (int64_t m0 = 0; m0 < M; m0 += itq3s::kGemvMaxM) {
        const int64_t rows = M - m0 < itq3s::kGemvMaxM ? M - m0 : itq3s::kGemvMaxM;
        const _Float16* Xh = static_cast<const _Float16*>(X) + m0 * ldx;
        itq3s::GemvWeight gw{codes, scales, N, static_cast<unsigned char*>(Y) + (size_t)m0 * (size_t)ldy * y_bytes, ldy, subscales};
        int rc;
        if (rows <= itq3s::kGemvFusedMaxM) {
            rc = itq3s::launch_gemv(&gw, 1, K, Xh, ldx, rows, y_f16, status_flags, st);
        } else {
            const int MP = pad_m(rows) < 8 ? 8 : pad_m(rows);
            _Float16* Xt = static_cast<_Float16*>(workspace);
            float* S = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + p.xt_bytes);
            rc = itq3s::launch_rotate_frag(Xh, rows, K, ldx, MP, Xt, S, status_flags, st);
            if (rc == 0) rc = itq3s::launch_gemv_rows(&gw, 1, K, Xt, S, rows, MP, y_f16, status_flags, st);
        }
        if (rc != 0) return rc;
    }
    return ITQ3S_OK;
}

int itq3s_matmul_static(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const void* X, int64_t M, int64_t ldx, void* Y,
                        int y_dtype, int64_t ldy, uint32_t* status_flags, void* stream) {
    if (!codes || !scales || !X || !Y) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || M <= 0 || K % 256 != 0 || ldx < K || ldy < N) return ITQ3S_ERR_SHAPE;
    if (itq3s_matmul_workspace_bytes(M, N, K) > (size_t)ITQ3S_STATIC_SCRATCH_BYTES) return ITQ3S_ERR_WORKSPACE;
    void* ws = scratch_of_current_device();
    if (ws == nullptr) return ITQ3S_ERR_LAUNCH;
    return itq3s_matmul(codes, scales, N, K, X, M, ldx, Y, y_dtype, ldy, ws, (size_t)ITQ3S_STATIC_SCRATCH_BYTES, status_flags, stream);
}

int itq3s_matmul_weight_side(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const void* X, int64_t M, int64_t ldx,
                             void* Y, int y_dtype, int64_t ldy, uint32_t* status_flags, void* stream) {
    if (!codes || !scales || !X || !Y) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || M <= 0 || K % 256 != 0 || ldx < K || ldy < N) return ITQ3S_ERR_SHAPE;
    if ((N + 15) / 16 > 0x7fffffffLL / (K / 256) || (M + 511) / 512 > 65535) return ITQ3S_ERR_SHAPE;
    if (y_dtype != ITQ3S_F32 && y_dtype != ITQ3S_F16) return ITQ3S_ERR_DTYPE;
    if (!aligned(X, 16) || ldx % 8 != 0 || !aligned(codes, 16) || !aligned(scales, 16) || !aligned(Y, y_dtype == ITQ3S_F16 ? 2 : 4) ||
        (status_flags && !aligned(status_flags, 4)))
        return ITQ3S_ERR_ALIGN;
    return itq3s::launch_gemm_weight_side(codes, scales, nullptr, N, K, static_cast<const _Float16*>(X), ldx, M, Y, y_dtype == ITQ3S_F16, ldy, status_flags,
                                          static_cast<hipStream_t>(stream));
}

// ---- measurement aids (include/itq3s_bench.h): the same calls with a pair of events armed for the
// contraction kernel's dispatch, then a wait


int itq3s_matmul_weight_side_timed(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const void* X, int64_t M, int64_t ldx,
                                   void* Y, int y_dtype, int64_t ldy, uint32_t* status_flags, void* stream, float* kernel_ms) {
    return timed(kernel_ms, [&] { return itq3s_matmul_weight_side(codes, scales, N, K, X, M, ldx, Y, y_dtype, ldy, status_flags, stream); });
}

int itq3s_matmul_grouped_timed(const itq3s_weight* w, int count, int64_t K, const void* X, int64_t M, int64_t ldx, int y_dtype,
                               void* workspace, size_t workspace_bytes, uint32_t* status_flags, void* stream, float* kernel_ms) {
    return timed(kernel_ms, [&] { return itq3s_matmul_grouped(w, count, K, X, M, ldx, y_dtype, workspace, workspace_bytes, status_flags, stream); });
}

int itq3s_matmul_timed(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const void* X, int64_t M, int64_t ldx,
                       void* Y, int y_dtype, int64_t ldy, void* workspace, size_t workspace_bytes, uint32_t* status_flags, void* stream,
                       float* kernel_ms) {
    if (!codes || !scales || !X || !Y) return ITQ3S_ERR_NULL;
    if (N <= 0 || K <= 0 || M <= 0 || K % 256 != 0 || ldx < K || ldy < N) return ITQ3S_ERR_SHAPE;
    const itq3s_weight w = {codes, scales, N, Y, ldy};
    return itq3s_matmul_grouped_timed(&w, 1, K, X, M, ldx, y_dtype, workspace, workspace_bytes, status_flags, stream, kernel_ms);
}

const char* itq3s_strerror(int status) {
    switch (status) {
        case ITQ3S_OK: return "ok";
        case ITQ3S_ERR_NULL: return "a required pointer is NULL";
        case ITQ3S_ERR_SHAPE: return "bad shape: sizes must be positive, K a multiple of 256, leading dimensions large enough";
        case ITQ3S_ERR_ALIGN: return "pointer or leading dimension not aligned as required";
        case ITQ3S_ERR_DTYPE: return "dtype must be ITQ3S_F32 or ITQ3S_F16";
        case ITQ3S_ERR_WORKSPACE: return "workspace missing or smaller than itq3s_matmul_workspace_bytes()";
        case ITQ3S_ERR_LAUNCH: return "HIP refused the kernel launch";
    }
    return "unknown status";
}

int itq3s_version(void) { return 100; }

}  // extern "C"
