// The graph layer around graph self-attention, forward (Sec. 3.1 and Sec. 3.3, the update of the graph):
//   Z = norm(X + [head_1 .. head_H] Wo),   Y = norm(Z + max(0, Z W1 + b1) W2 + b2)
// for all 2n-1 nodes.  The dense maps are plain library GEMMs (rocBLAS, bf16 operands, fp32
// accumulation); attention is this library's own forward on the [B][N][H][64] layout the
// projections produce (no transposes); residual + bias + layer normalisation and bias + ReLU are
// the two small kernels below.
#include <hip/hip_runtime.h>
#include <rocblas/rocblas.h>

#include <mutex>

#include "bpt_internal.h"

namespace bpt {
namespace {

typedef uint16_t bf16_t;
constexpr int kLnMaxChunks = 4;   // 8-element chunks per lane: d <= 2048

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f); }

// y = norm(x + a + bias) * gain + beta, one wavefront per row; x bf16, a fp32 (the GEMM result of the
// sublayer), bias fp32 or null; the row stays in registers between the two passes (mean, then variance
// of the centred values: Ba et al., biased variance).
__global__ void __launch_bounds__(256) residual_layer_norm_kernel(const bf16_t* __restrict__ x, const float* __restrict__ a,
                                                                  const float* __restrict__ bias, const float* __restrict__ gain,
                                                                  const float* __restrict__ beta, bf16_t* __restrict__ y,
                                                                  int64_t rows, int d, float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int nchunk = d >> 3;
    float v[kLnMaxChunks][8];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxChunks; ++i) {
        const int c = lane + 64 * i;
        if (c < nchunk) {
            const uint4 xw = *reinterpret_cast<const uint4*>(x + row * d + c * 8);
            const float4 a0 = *reinterpret_cast<const float4*>(a + row * d + c * 8);
            const float4 a1 = *reinterpret_cast<const float4*>(a + row * d + c * 8 + 4);
            const uint32_t w[4] = {xw.x, xw.y, xw.z, xw.w};
            const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float xv = (e & 1) ? __uint_as_float(w[e >> 1] & 0xFFFF0000u) : bf16_to_f32(w[e >> 1] & 0xFFFFu);
                v[i][e] = xv + av[e] + (bias ? bias[c * 8 + e] : 0.f);
                sum += v[i][e];
            }
        }
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) sum += __shfl_xor(sum, s);
    const float mean = sum / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxChunks; ++i)
        if (lane + 64 * i < nchunk)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[i][e] -= mean;
                sq += v[i][e] * v[i][e];
            }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) sq += __shfl_xor(sq, s);
    const float inv = rsqrtf(sq / (float)d + eps);
#pragma unroll
    for (int i = 0; i < kLnMaxChunks; ++i) {
        const int c = lane + 64 * i;
        if (c < nchunk) {
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float y0 = v[i][e] * inv * gain[c * 8 + e] + beta[c * 8 + e];
                const float y1 = v[i][e + 1] * inv * gain[c * 8 + e + 1] + beta[c * 8 + e + 1];
                o[e >> 1] = f32_to_bf16(y0) | (f32_to_bf16(y1) << 16);
            }
            *reinterpret_cast<uint4*>(y + row * d + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

// f = max(0, f + b) in place on [rows][cols] bf16, 8 values per thread (cols a multiple of 8)
__global__ void __launch_bounds__(256) bias_relu_kernel(bf16_t* __restrict__ f, const float* __restrict__ b, int64_t chunks,
                                                        int cols) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const int col = (int)((i * 8) % cols);
    uint4 w = *reinterpret_cast<uint4*>(f + i * 8);
    uint32_t x[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = fmaxf(bf16_to_f32(x[e] & 0xFFFFu) + b[col + 2 * e], 0.f);
        const float hi = fmaxf(__uint_as_float(x[e] & 0xFFFF0000u) + b[col + 2 * e + 1], 0.f);
        x[e] = f32_to_bf16(lo) | (f32_to_bf16(hi) << 16);
    }
    *reinterpret_cast<uint4*>(f + i * 8) = make_uint4(x[0], x[1], x[2], x[3]);
}

// one rocBLAS handle per device, created on first use
rocblas_handle blas_handle(int device) {
    static std::mutex mu;
    static rocblas_handle handles[64] = {};
    std::lock_guard<std::mutex> lock(mu);
    if (device < 0 || device >= 64) return nullptr;
    if (!handles[device] && rocblas_create_handle(&handles[device]) != rocblas_status_success) handles[device] = nullptr;
    return handles[device];
}

// C[M][N] = A[M][K] B[K][N], row-major, bf16 operands, fp32 accumulation; C bf16 or fp32.
// rocBLAS is column-major: C^T = B^T A^T with the same buffers.
int gemm_rm(rocblas_handle h, int64_t M, int N, int K, const void* A, const void* B, void* C, bool c_fp32) {
    const float one = 1.f, zero = 0.f;
    const rocblas_datatype ct = c_fp32 ? rocblas_datatype_f32_r : rocblas_datatype_bf16_r;
    const rocblas_status st =
        rocblas_gemm_ex(h, rocblas_operation_none, rocblas_operation_none, N, (rocblas_int)M, K, &one, B, rocblas_datatype_bf16_r, N,
                        A, rocblas_datatype_bf16_r, K, &zero, C, ct, N, C, ct, N, rocblas_datatype_f32_r, rocblas_gemm_algo_standard,
                        0, 0);
    return st == rocblas_status_success ? BPT_OK : BPT_ERR_LAUNCH;
}

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct LayerBuffers {
    size_t q, k, v, o, lse, acc, z, f1, attn, total;
};
LayerBuffers layer_buffers(const bpt_graph* g, int B, int H, int d_ff, size_t attn_ws) {
    const size_t rows = (size_t)B * g->num_nodes, d = (size_t)H * kD;
    LayerBuffers L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes);
        return at;
    };
    L.q = take(rows * d * 2);
    L.k = take(rows * d * 2);
    L.v = take(rows * d * 2);
    L.o = take(rows * d * 2);
    L.lse = take((size_t)B * H * g->num_nodes * 4);
    L.acc = take(rows * d * 4);      // W^O and W_2 results, fp32
    L.z = take(rows * d * 2);
    L.f1 = take(rows * (size_t)d_ff * 2);
    L.attn = take(attn_ws);
    L.total = off;
    return L;
}

bpt_shape_t attn_shape(const bpt_graph* g, int B, int H, float scale, const int32_t* seq_len) {
    bpt_shape_t s = {};
    s.B = B;
    s.H = H;
    s.D = kD;
    s.dtype = BPT_BF16;
    s.stride_n = (int64_t)H * kD;              // [B][N][H][64]: the heads of a node are adjacent
    s.stride_h = kD;
    s.stride_b = (int64_t)g->num_nodes * H * kD;
    s.scale = scale;
    s.seq_len = seq_len;
    return s;
}

}  // namespace
}  // namespace bpt

using namespace bpt;

extern "C" {

size_t bpt_layer_fwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff) {
    if (!g || B < 1 || H < 1 || d_ff < 8) return 0;
    const bpt_shape_t s = attn_shape(g, B, H, 0.f, nullptr);
    return layer_buffers(g, B, H, d_ff, bpt_attn_fwd_workspace(g, &s)).total;
}

int bpt_layer_fwd(const bpt_graph_t* g, int32_t B, int32_t H, float scale, const int32_t* seq_len, const void* rel,
                  const void* X, const bpt_layer_params_t* p, void* Y, void* workspace, size_t workspace_bytes, void* stream) {
    if (!g || !rel || !X || !p || !Y || B < 1 || H < 1) return BPT_ERR_INVALID_ARG;
    if (!p->Wq || !p->Wk || !p->Wv || !p->Wo || !p->W1 || !p->W2 || !p->b1 || !p->b2 || !p->g1 || !p->beta1 || !p->g2 || !p->beta2)
        return BPT_ERR_INVALID_ARG;
    const int d = H * kD, d_ff = p->d_ff;
    if (d > 8 * 64 * kLnMaxChunks || d_ff < 8 || (d_ff & 7)) return BPT_ERR_UNSUPPORTED;
    const int64_t rows = (int64_t)B * g->num_nodes;
    if (rows > INT32_MAX) return BPT_ERR_UNSUPPORTED;
    const bpt_shape_t s = attn_shape(g, B, H, scale, seq_len);
    const size_t attn_ws = bpt_attn_fwd_workspace(g, &s);
    const LayerBuffers L = layer_buffers(g, B, H, d_ff, attn_ws);
    if (L.total > workspace_bytes || (L.total && !workspace)) return BPT_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rocblas_handle h = blas_handle(g->device);
    if (!h || rocblas_set_stream(h, st) != rocblas_status_success) return BPT_ERR_LAUNCH;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    void *q = ws + L.q, *k = ws + L.k, *v = ws + L.v, *o = ws + L.o, *z = ws + L.z, *f1 = ws + L.f1;
    float* lse = reinterpret_cast<float*>(ws + L.lse);
    float* acc = reinterpret_cast<float*>(ws + L.acc);
    const float eps = p->eps > 0.f ? p->eps : 1e-5f;
    int rc;
    // Q, K, V = X Wq, X Wk, X Wv for all nodes: [B][N][H][64], the layout the attention reads through its strides
    if ((rc = gemm_rm(h, rows, d, d, X, p->Wq, q, false)) || (rc = gemm_rm(h, rows, d, d, X, p->Wk, k, false)) ||
        (rc = gemm_rm(h, rows, d, d, X, p->Wv, v, false)))
        return rc;
    if ((rc = bpt_attn_fwd(g, &s, q, k, v, rel, o, lse, ws + L.attn, attn_ws, stream))) return rc;
    // Z = norm(X + O Wo)
    if ((rc = gemm_rm(h, rows, d, d, o, p->Wo, acc, true))) return rc;
    const unsigned ln_blocks = (unsigned)((rows + 3) / 4);
    BPT_LAUNCH("residual_layer_norm_kernel", residual_layer_norm_kernel, dim3(ln_blocks), dim3(256), 0, st,
               static_cast<const bf16_t*>(X), acc, static_cast<const float*>(nullptr), p->g1, p->beta1, static_cast<bf16_t*>(z), rows,
               d, eps);
    BPT_HIP(hipGetLastError());
    // Y = norm(Z + max(0, Z W1 + b1) W2 + b2)
    if ((rc = gemm_rm(h, rows, d_ff, d, z, p->W1, f1, false))) return rc;
    const int64_t chunks = rows * d_ff / 8;
    BPT_LAUNCH("bias_relu_kernel", bias_relu_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
               static_cast<bf16_t*>(f1), p->b1, chunks, d_ff);
    BPT_HIP(hipGetLastError());
    if ((rc = gemm_rm(h, rows, d, d_ff, f1, p->W2, acc, true))) return rc;
    BPT_LAUNCH("residual_layer_norm_kernel", residual_layer_norm_kernel, dim3(ln_blocks), dim3(256), 0, st,
               static_cast<const bf16_t*>(z), acc, p->b2, p->g2, p->beta2, static_cast<bf16_t*>(Y), rows, d, eps);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

}  // extern "C"
