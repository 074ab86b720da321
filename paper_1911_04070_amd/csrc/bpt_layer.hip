// The graph layer around graph self-attention (Sec. 3.1 and Sec. 3.3, the update of the graph):
//   Z = norm(X + [head_1 .. head_H] Wo),   Y = norm(Z + max(0, Z W1 + b1) W2 + b2)
// for all 2n-1 nodes, forward and backward, and the loop over layers from the initial states
// (embeddings on the token rows, zero on the span rows) to the root or token rows of the last
// layer.  The dense maps are plain library GEMMs (hipBLASLt, rocBLAS for the weight gradients;
// bf16 operands, fp32 accumulation); attention is this library's own forward and backward on the
// [B][N][H][64] layout the projections produce (no transposes); residual + bias + layer
// normalisation, bias + ReLU, their backward counterparts and the fixed-order column sums are
// the small kernels below.
#include <hip/hip_runtime.h>
#include <hipblaslt/hipblaslt.h>
#include <rocblas/rocblas.h>

#include <algorithm>
#include <cstdlib>
#include <string>
#include <vector>

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
                                                                  float2* __restrict__ stats, int64_t rows, int d, float eps) {
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
    if (lane == 0) stats[row] = make_float2(mean, inv);   // what the backward normalises the row with
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

// first token of a node of the tree over n = 2^lg tokens (ids are level-major)
__device__ __forceinline__ int first_token_of(int id, int lg) {
    const int x = (2 << lg) - id;
    const int level = lg - (31 - __clz(x - 1));
    return (((2 << lg) >> level) - x) << level;
}

// Backward of y = norm(s) * gain + beta with s = x + a + bias (as residual_layer_norm_kernel formed it;
// `stats` = its (mean, 1/deviation) per row):  dxh = dy * gain,
//   ds = (dxh - mean(dxh) - xh * mean(dxh * xh)) / deviation,   xh = (s - mean) / deviation,
// with dy = dy_b (bf16) + dy_f (fp32, may be null).  ds is written in bf16.  A wavefront walks rows
// `wave, wave + waves, ...` and keeps the column sums of dy * xh (gain), dy (beta) and ds (the bias
// inside s) of its rows in registers; the four wavefronts of a workgroup add theirs in a fixed order
// and the workgroup writes one row of `partials` [gridDim.x][3][d].  With seq_len, rows of nodes the
// sequence does not keep count as dy = 0.
template <int CHUNKS>   // 8-element chunks per lane: d <= 512 * CHUNKS
__global__ void __launch_bounds__(256) layer_norm_bwd_kernel(const bf16_t* __restrict__ dy_b, const float* __restrict__ dy_f,
                                                             const bf16_t* __restrict__ x, const float* __restrict__ a,
                                                             const float* __restrict__ bias, const float* __restrict__ gain,
                                                             const float2* __restrict__ stats, bf16_t* __restrict__ ds,
                                                             float* __restrict__ partials, int64_t rows, int d,
                                                             const int32_t* __restrict__ seq_len, int N, int lg) {
    extern __shared__ float red_s[];   // wavefronts 1..3: [wavefront - 1][sum][d columns]
    auto red = [&](int w, int which, int col) -> float& { return red_s[(w * 3 + which) * d + col]; };
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nchunk = d >> 3;
    float sg[CHUNKS][8], sb[CHUNKS][8], ss[CHUNKS][8];
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) sg[i][e] = sb[i][e] = ss[i][e] = 0.f;
    const int64_t stride = (int64_t)gridDim.x * 4;
    for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < rows; row += stride) {
        bool kept = true;
        if (seq_len) {
            const int b = (int)(row / N), node = (int)(row - (int64_t)b * N);
            kept = first_token_of(node, lg) < min(max(seq_len[b], 0), 1 << lg);
        }
        const float2 st = stats[row];
        float xh[CHUNKS][8], dxh[CHUNKS][8];
        float m1 = 0.f, m2 = 0.f;
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) {
            const int c = lane + 64 * i;
            if (c < nchunk) {
                const int64_t at = row * d + c * 8;
                const uint4 xw = *reinterpret_cast<const uint4*>(x + at);
                const uint4 gw = *reinterpret_cast<const uint4*>(dy_b + at);
                const float4 a0 = *reinterpret_cast<const float4*>(a + at), a1 = *reinterpret_cast<const float4*>(a + at + 4);
                float4 f0 = make_float4(0.f, 0.f, 0.f, 0.f), f1 = f0;
                if (dy_f) {
                    f0 = *reinterpret_cast<const float4*>(dy_f + at);
                    f1 = *reinterpret_cast<const float4*>(dy_f + at + 4);
                }
                const uint32_t xv[4] = {xw.x, xw.y, xw.z, xw.w}, gv[4] = {gw.x, gw.y, gw.z, gw.w};
                const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                const float fv[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float xe = (e & 1) ? __uint_as_float(xv[e >> 1] & 0xFFFF0000u) : bf16_to_f32(xv[e >> 1] & 0xFFFFu);
                    const float ge = (e & 1) ? __uint_as_float(gv[e >> 1] & 0xFFFF0000u) : bf16_to_f32(gv[e >> 1] & 0xFFFFu);
                    const float dye = kept ? ge + fv[e] : 0.f;
                    const float s = xe + av[e] + (bias ? bias[c * 8 + e] : 0.f);
                    xh[i][e] = (s - st.x) * st.y;
                    dxh[i][e] = dye * gain[c * 8 + e];
                    m1 += dxh[i][e];
                    m2 += dxh[i][e] * xh[i][e];
                    sg[i][e] += dye * xh[i][e];
                    sb[i][e] += dye;
                }
            }
        }
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            m1 += __shfl_xor(m1, s);
            m2 += __shfl_xor(m2, s);
        }
        m1 /= (float)d;
        m2 /= (float)d;
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) {
            const int c = lane + 64 * i;
            if (c < nchunk) {
                uint32_t o[4];
                float r[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    r[e] = st.y * (dxh[i][e] - m1 - xh[i][e] * m2);
                    ss[i][e] += r[e];
                }
#pragma unroll
                for (int e = 0; e < 8; e += 2) o[e >> 1] = f32_to_bf16(r[e]) | (f32_to_bf16(r[e + 1]) << 16);
                *reinterpret_cast<uint4*>(ds + row * d + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    }
    // wavefronts 1..3 hand their sums to wavefront 0, which adds them in order and writes the workgroup's row
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const int c = lane + 64 * i;
        if (c < nchunk && wave > 0)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                red(wave - 1, 0, c * 8 + e) = sg[i][e];
                red(wave - 1, 1, c * 8 + e) = sb[i][e];
                red(wave - 1, 2, c * 8 + e) = ss[i][e];
            }
    }
    __syncthreads();
    if (wave == 0) {
        float* out = partials + (int64_t)blockIdx.x * 3 * d;
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) {
            const int c = lane + 64 * i;
            if (c < nchunk)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int col = c * 8 + e;
                    out[col] = ((sg[i][e] + red(0, 0, col)) + red(1, 0, col)) + red(2, 0, col);
                    out[d + col] = ((sb[i][e] + red(0, 1, col)) + red(1, 1, col)) + red(2, 1, col);
                    out[2 * d + col] = ((ss[i][e] + red(0, 2, col)) + red(1, 2, col)) + red(2, 2, col);
                }
        }
    }
}

// Backward of f = max(0, h): df *= (f > 0) in place on [rows][cols] bf16 (f is the stored output of
// bias_relu_kernel), and the column sums of the result (the gradient of the bias) of the rows
// `blockIdx.x, blockIdx.x + gridDim.x, ...` into partials[gridDim.x][cols].  A thread owns up to
// kReluChunks chunks of 8 columns.
constexpr int kReluChunks = 4;   // cols <= 8 * 256 * 4
__global__ void __launch_bounds__(256) relu_bwd_kernel(bf16_t* __restrict__ df, const bf16_t* __restrict__ f,
                                                       float* __restrict__ partials, int64_t rows, int cols) {
    const int nchunk = cols >> 3;
    float acc[kReluChunks][8];
#pragma unroll
    for (int i = 0; i < kReluChunks; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
#pragma unroll
        for (int i = 0; i < kReluChunks; ++i) {
            const int c = threadIdx.x + 256 * i;
            if (c < nchunk) {
                const int64_t at = row * cols + c * 8;
                const uint4 gw = *reinterpret_cast<const uint4*>(df + at);
                const uint4 fw = *reinterpret_cast<const uint4*>(f + at);
                uint32_t gv[4] = {gw.x, gw.y, gw.z, gw.w};
                const uint32_t fv[4] = {fw.x, fw.y, fw.z, fw.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // the stored activations are >= 0: positive iff the bits below the sign are not all zero
                    if ((fv[e] & 0x7FFFu) == 0u) gv[e] &= 0xFFFF0000u;
                    if ((fv[e] & 0x7FFF0000u) == 0u) gv[e] &= 0x0000FFFFu;
                    acc[i][2 * e] += bf16_to_f32(gv[e] & 0xFFFFu);
                    acc[i][2 * e + 1] += __uint_as_float(gv[e] & 0xFFFF0000u);
                }
                *reinterpret_cast<uint4*>(df + at) = make_uint4(gv[0], gv[1], gv[2], gv[3]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kReluChunks; ++i) {
        const int c = threadIdx.x + 256 * i;
        if (c < nchunk) {
            float* out = partials + (int64_t)blockIdx.x * cols + c * 8;
            *reinterpret_cast<float4*>(out) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
            *reinterpret_cast<float4*>(out + 4) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
        }
    }
}

// Column sums of partials[num_parts][cols] in a fixed order: a workgroup takes 64 columns, its 16
// wavefronts each sum the rows `w, w + 16, ...` (lane = column, four sums in flight) and the 16 results
// are added in a fixed tree.  Column c goes to out[c / cols_each][c % cols_each] (up to three outputs
// whose partial sums sit side by side in a row; a null output is skipped).
struct ColumnSumOut {
    float* out[3];
    int cols_each;
};
__global__ void __launch_bounds__(1024) column_sum_kernel(const float* __restrict__ partials, int num_parts, int cols,
                                                          const ColumnSumOut o) {
    __shared__ float s[16][64];
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (c < cols) {
        const float* src = partials + c;
        int p = grp;
        for (; p + 48 < num_parts; p += 64) {
            s0 += src[(int64_t)p * cols];
            s1 += src[(int64_t)(p + 16) * cols];
            s2 += src[(int64_t)(p + 32) * cols];
            s3 += src[(int64_t)(p + 48) * cols];
        }
        for (; p < num_parts; p += 16) s0 += src[(int64_t)p * cols];
    }
    s[grp][lane] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    for (int w = 8; w > 0; w >>= 1) {
        if (grp < w) s[grp][lane] += s[grp + w][lane];
        __syncthreads();
    }
    if (grp == 0 && c < cols && o.out[c / o.cols_each]) o.out[c / o.cols_each][c % o.cols_each] = s[0][lane];
}

// out[i] = sum over s of slices[s][i] in slice order, 4 values per thread: the partial products of a
// GEMM whose contraction was cut into slices.  Element i belongs to row i / cols; its columns go to
// out[col / cols_each] (row pitch cols_each): up to three matrices computed side by side.
__global__ void __launch_bounds__(256) sum_slices_kernel(const float* __restrict__ slices, int num_slices, int64_t elems,
                                                         int cols, const ColumnSumOut o) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= elems) return;
    float4 acc = *reinterpret_cast<const float4*>(slices + i);
    for (int sl = 1; sl < num_slices; ++sl) {
        const float4 x = *reinterpret_cast<const float4*>(slices + (int64_t)sl * elems + i);
        acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    const int64_t row = i / cols;
    const int col = (int)(i - row * cols);
    *reinterpret_cast<float4*>(o.out[col / o.cols_each] + row * o.cols_each + col % o.cols_each) = acc;
}

// dst (bf16) [d][3 d] = Wq | Wk | Wv ([d][d] each) side by side, 8 values per thread; blockIdx.y picks the matrix.
// One projection X [Wq | Wk | Wv] then reads X once and gives the three results side by side.
struct PackArgs {
    const bf16_t* src[3];
    bf16_t* dst;
};
__global__ void __launch_bounds__(256) pack_qkv_weights_kernel(const PackArgs t, int64_t chunks, int d) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const int64_t row = (i * 8) / d;
    const int col = (int)(i * 8 - row * d);
    *reinterpret_cast<uint4*>(t.dst + row * 3 * d + (int64_t)blockIdx.y * d + col) =
        *reinterpret_cast<const uint4*>(t.src[blockIdx.y] + i * 8);
}

// y (bf16) = x (bf16) + a (fp32), 8 values per thread
__global__ void __launch_bounds__(256) add_cast_kernel(const bf16_t* __restrict__ x, const float* __restrict__ a,
                                                       bf16_t* __restrict__ y, int64_t chunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const uint4 xw = *reinterpret_cast<const uint4*>(x + i * 8);
    const float4 a0 = *reinterpret_cast<const float4*>(a + i * 8), a1 = *reinterpret_cast<const float4*>(a + i * 8 + 4);
    const uint32_t w[4] = {xw.x, xw.y, xw.z, xw.w};
    const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        o[e] = f32_to_bf16(bf16_to_f32(w[e] & 0xFFFFu) + av[2 * e]) |
               (f32_to_bf16(__uint_as_float(w[e] & 0xFFFF0000u) + av[2 * e + 1]) << 16);
    *reinterpret_cast<uint4*>(y + i * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// Sec. 3.3, the states before the first layer: token nodes start from their embeddings, span nodes from
// zero.  e: [B][n][d], h: [B][N][d], 8 values per thread.
__global__ void __launch_bounds__(256) initial_states_kernel(const bf16_t* __restrict__ e, bf16_t* __restrict__ h, int64_t chunks,
                                                             int n, int N, int row_chunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const int64_t row = i / row_chunks;
    const int c = (int)(i - row * row_chunks), v = (int)(row % N);
    const int64_t b = row / N;
    uint4 x = make_uint4(0u, 0u, 0u, 0u);
    if (v < n) x = *reinterpret_cast<const uint4*>(e + ((b * n + v) * row_chunks + c) * 8);
    *reinterpret_cast<uint4*>(h + i * 8) = x;
}

// Sec. 3.3, the output: the roots' rows and / or the token rows of h [B][N][d], to root [B][R][d] and tokens
// [B][n][d] (either may be null).  One thread per 8 values of the rows that are read.  A tree has one root, its
// last row (R = 1, root_row null); the graph of a packed batch has one per sequence, root_row[r] (-1: an empty
// sequence, whose output is zero).
__global__ void __launch_bounds__(256) readout_kernel(const bf16_t* __restrict__ h, bf16_t* __restrict__ root,
                                                      bf16_t* __restrict__ tokens, int64_t chunks, int n, int N, int row_chunks,
                                                      int R, const int32_t* __restrict__ root_row) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const int64_t row = i / row_chunks;   // over [B][n + R]: the tokens, then the roots
    const int c = (int)(i - row * row_chunks), v = (int)(row % (n + R));
    const int64_t b = row / (n + R);
    bf16_t* dst = v < n ? tokens : root;
    if (!dst) return;
    const int src = v < n ? v : root_row ? root_row[v - n] : N - 1;
    uint4 x = make_uint4(0u, 0u, 0u, 0u);
    if (src >= 0) x = *reinterpret_cast<const uint4*>(h + ((b * N + src) * row_chunks + c) * 8);
    *reinterpret_cast<uint4*>(dst + ((v < n ? b * n + v : b * R + (v - n)) * row_chunks + c) * 8) = x;
}

// the reverse: the gradient with respect to the last states is d_tokens on the token rows, d_root on the
// root's row (a null one counts as zero) and zero on every other row
// (first_root: the first root row -- N - 1 for a tree; root_seq: for the graph of a packed batch, the sequence of
// every row from first_root on, else null)
__global__ void __launch_bounds__(256) readout_bwd_kernel(const bf16_t* __restrict__ d_root, const bf16_t* __restrict__ d_tokens,
                                                          bf16_t* __restrict__ dh, int64_t chunks, int n, int N, int row_chunks,
                                                          int R, int first_root, const int32_t* __restrict__ root_seq) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const int64_t row = i / row_chunks;
    const int c = (int)(i - row * row_chunks), v = (int)(row % N);
    const int64_t b = row / N;
    uint4 x = make_uint4(0u, 0u, 0u, 0u);
    if (v < n && d_tokens) x = *reinterpret_cast<const uint4*>(d_tokens + ((b * n + v) * row_chunks + c) * 8);
    if (v >= first_root && d_root) {
        const int r = root_seq ? root_seq[v - first_root] : 0;
        x = *reinterpret_cast<const uint4*>(d_root + ((b * R + r) * row_chunks + c) * 8);
    }
    *reinterpret_cast<uint4*>(dh + i * 8) = x;
}

// one rocBLAS handle per host thread and device, created on first use and kept: a handle carries the
// stream of the call in progress, so two host threads must not share one
rocblas_handle blas_handle(int device) {
    thread_local rocblas_handle handles[64] = {};
    if (device < 0 || device >= 64) return nullptr;
    if (!handles[device] && rocblas_create_handle(&handles[device]) != rocblas_status_success) handles[device] = nullptr;
    return handles[device];
}

// C[M][N] = beta C + op(A) op(B), row-major, bf16 operands, fp32 accumulation; C bf16 or fp32.
// op(A) is [M][K]: A is stored [M][K], or [K][M] with ta; op(B) is [K][N]: B is stored [K][N], or [N][K]
// with tb.  rocBLAS is column-major: C^T = op(B)^T op(A)^T with the same buffers, a row-major
// [r][c] buffer being the column-major c x r matrix with leading dimension c.
int gemm_rm(rocblas_handle h, int64_t M, int64_t N, int64_t K, const void* A, bool ta, const void* B, bool tb, void* C,
            bool c_fp32, float beta = 0.f, int64_t lda = 0, int64_t ldc = 0) {   // lda, ldc: elements between rows of A, C as stored (0: dense)
    const float one = 1.f;
    const rocblas_datatype ct = c_fp32 ? rocblas_datatype_f32_r : rocblas_datatype_bf16_r;
    const rocblas_int ldc_ = (rocblas_int)(ldc ? ldc : N);
    const rocblas_status st = rocblas_gemm_ex(
        h, tb ? rocblas_operation_transpose : rocblas_operation_none, ta ? rocblas_operation_transpose : rocblas_operation_none,
        (rocblas_int)N, (rocblas_int)M, (rocblas_int)K, &one, B, rocblas_datatype_bf16_r, (rocblas_int)(tb ? K : N), A,
        rocblas_datatype_bf16_r, (rocblas_int)(lda ? lda : (ta ? M : K)), &beta, C, ct, ldc_, C, ct, ldc_,
        rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    return st == rocblas_status_success ? BPT_OK : BPT_ERR_LAUNCH;
}

// The same product through hipBLASLt, whose epilogue can add a bias row and apply the ReLU while the sums are
// still fp32 in registers (Sec. 3.1 eq. (3): max(0, Z W1 + b1) without a pass of its own), and whose kernel
// choice for the tall products of the layer (65 532 x 512..2048) is 5-15 % faster than the one behind
// rocblas_gemm_ex.  A plan (descriptor, layouts, algorithm) per distinct product, made on first use and kept,
// per host thread and device like the rocBLAS handle; the first use of a product must therefore lie outside a
// stream capture.  A product hipBLASLt has no algorithm for reports false and the caller takes the rocBLAS path.
struct LtPlan {
    int64_t M, N, K, lda, ldc;
    bool ta, tb, c_fp32, bias_relu, add;
    hipblasLtMatmulDesc_t desc;
    hipblasLtMatrixLayout_t la, lb, lc;
    hipblasLtMatmulAlgo_t algo;
    size_t ws_bytes;
};
struct LtContext {
    hipblasLtHandle_t handle = nullptr;
    void* ws = nullptr;               // the algorithms' scratch memory, kept until the process ends
    std::vector<LtPlan> plans;
    bool failed = false;
};
constexpr size_t kLtWorkspace = (size_t)32 << 20;
constexpr int kLtCandidates = 12, kLtTimedRuns = 3;
LtContext* lt_context(int device) {
    thread_local LtContext ctx[64];
    if (device < 0 || device >= 64) return nullptr;
    LtContext& c = ctx[device];
    if (c.failed) return nullptr;
    if (!c.handle) {
        if (hipblasLtCreate(&c.handle) != HIPBLAS_STATUS_SUCCESS || hipMalloc(&c.ws, kLtWorkspace) != hipSuccess) {
            c.failed = true;
            (void)hipGetLastError();
            return nullptr;
        }
    }
    return &c;
}
// C[M][N] = op(A) op(B) (+ bias[N], then max(0, .) with bias_relu; + add[M][N], of C's type and row stride, with add:
// the sum is formed in fp32 and rounded once), arguments as gemm_rm's with beta = 0
bool gemm_lt(int device, hipStream_t st, int64_t M, int64_t N, int64_t K, const void* A, bool ta, const void* B, bool tb, void* C,
             bool c_fp32, int64_t lda, int64_t ldc, const float* bias_relu, const void* add) {
    LtContext* c = lt_context(device);
    if (!c) return false;
    const int64_t lda_ = lda ? lda : (ta ? M : K), ldc_ = ldc ? ldc : N;
    LtPlan* plan = nullptr;
    for (LtPlan& q : c->plans)
        if (q.M == M && q.N == N && q.K == K && q.lda == lda_ && q.ldc == ldc_ && q.ta == ta && q.tb == tb && q.c_fp32 == c_fp32 &&
            q.bias_relu == (bias_relu != nullptr) && q.add == (add != nullptr)) {
            plan = &q;
            break;
        }
    if (!plan) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return false;
        LtPlan q = {M, N, K, lda_, ldc_, ta, tb, c_fp32, bias_relu != nullptr, add != nullptr, nullptr, nullptr, nullptr, nullptr, {}, 0};
        // column-major view: C^T [N x M] = op(B)^T [N x K] op(A)^T [K x M] on the same buffers
        const hipblasOperation_t op_first = tb ? HIPBLAS_OP_T : HIPBLAS_OP_N, op_second = ta ? HIPBLAS_OP_T : HIPBLAS_OP_N;
        const hipDataType ctype = c_fp32 ? HIP_R_32F : HIP_R_16BF;
        bool ok = hipblasLtMatmulDescCreate(&q.desc, HIPBLAS_COMPUTE_32F, HIP_R_32F) == HIPBLAS_STATUS_SUCCESS;
        ok = ok && hipblasLtMatmulDescSetAttribute(q.desc, HIPBLASLT_MATMUL_DESC_TRANSA, &op_first, sizeof(op_first)) == HIPBLAS_STATUS_SUCCESS;
        ok = ok && hipblasLtMatmulDescSetAttribute(q.desc, HIPBLASLT_MATMUL_DESC_TRANSB, &op_second, sizeof(op_second)) == HIPBLAS_STATUS_SUCCESS;
        if (ok && bias_relu) {
            const hipblasLtEpilogue_t epi = HIPBLASLT_EPILOGUE_RELU_BIAS;
            const hipDataType btype = HIP_R_32F;
            ok = hipblasLtMatmulDescSetAttribute(q.desc, HIPBLASLT_MATMUL_DESC_EPILOGUE, &epi, sizeof(epi)) == HIPBLAS_STATUS_SUCCESS &&
                 hipblasLtMatmulDescSetAttribute(q.desc, HIPBLASLT_MATMUL_DESC_BIAS_DATA_TYPE, &btype, sizeof(btype)) == HIPBLAS_STATUS_SUCCESS &&
                 hipblasLtMatmulDescSetAttribute(q.desc, HIPBLASLT_MATMUL_DESC_BIAS_POINTER, &bias_relu, sizeof(bias_relu)) == HIPBLAS_STATUS_SUCCESS;
        }
        ok = ok && hipblasLtMatrixLayoutCreate(&q.la, HIP_R_16BF, tb ? K : N, tb ? N : K, tb ? K : N) == HIPBLAS_STATUS_SUCCESS;
        ok = ok && hipblasLtMatrixLayoutCreate(&q.lb, HIP_R_16BF, ta ? M : K, ta ? K : M, lda_) == HIPBLAS_STATUS_SUCCESS;
        ok = ok && hipblasLtMatrixLayoutCreate(&q.lc, ctype, N, M, ldc_) == HIPBLAS_STATUS_SUCCESS;
        hipblasLtMatmulPreference_t pref = nullptr;
        ok = ok && hipblasLtMatmulPreferenceCreate(&pref) == HIPBLAS_STATUS_SUCCESS;
        ok = ok && hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &kLtWorkspace, sizeof(kLtWorkspace)) == HIPBLAS_STATUS_SUCCESS;
        hipblasLtMatmulHeuristicResult_t res[kLtCandidates];
        int found = 0;
        ok = ok && hipblasLtMatmulAlgoGetHeuristic(c->handle, q.desc, q.la, q.lb, q.lc, q.lc, pref, kLtCandidates, res, &found) ==
                       HIPBLAS_STATUS_SUCCESS;
        if (pref) hipblasLtMatmulPreferenceDestroy(pref);
        // the library's candidates, timed on the caller's own buffers (beta = 0: what they write is overwritten by
        // the product proper); the fastest is kept for this process
        int best = -1;
        float best_ms = 0.f;
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (ok && found > 1 && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) found = 1;
        const float one = 1.f, beta = add ? 1.f : 0.f;
        const void* cin = add ? add : C;
        for (int i = 0; ok && i < found; ++i) {
            if (res[i].state != HIPBLAS_STATUS_SUCCESS || res[i].workspaceSize > kLtWorkspace) continue;
            if (found == 1) {
                best = i;
                break;
            }
            bool ran = true;
            for (int rep = 0; rep < kLtTimedRuns + 1 && ran; ++rep) {   // the first run is not timed
                if (rep == 1) ran = hipEventRecord(e0, st) == hipSuccess;
                ran = ran && hipblasLtMatmul(c->handle, q.desc, &one, B, q.la, A, q.lb, &beta, cin, q.lc, C, q.lc, &res[i].algo, c->ws,
                                             kLtWorkspace, st) == HIPBLAS_STATUS_SUCCESS;
            }
            float ms = 0.f;
            ran = ran && hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                  hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
            if (ran && (best < 0 || ms < best_ms)) {
                best = i;
                best_ms = ms;
            }
        }
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        ok = ok && best >= 0;
        if (ok) {
            q.algo = res[best].algo;
            q.ws_bytes = res[best].workspaceSize;
        } else {   // remembered as a product to leave to rocBLAS
            if (q.lc) hipblasLtMatrixLayoutDestroy(q.lc);
            if (q.lb) hipblasLtMatrixLayoutDestroy(q.lb);
            if (q.la) hipblasLtMatrixLayoutDestroy(q.la);
            if (q.desc) hipblasLtMatmulDescDestroy(q.desc);
            q.desc = nullptr;
        }
        c->plans.push_back(q);
        plan = &c->plans.back();
    }
    if (!plan->desc) return false;
    if (bias_relu && hipblasLtMatmulDescSetAttribute(plan->desc, HIPBLASLT_MATMUL_DESC_BIAS_POINTER, &bias_relu, sizeof(bias_relu)) !=
                         HIPBLAS_STATUS_SUCCESS)
        return false;
    const float one = 1.f, beta = add ? 1.f : 0.f;
    return hipblasLtMatmul(c->handle, plan->desc, &one, B, plan->la, A, plan->lb, &beta, add ? add : C, plan->lc, C, plan->lc,
                           &plan->algo, c->ws, kLtWorkspace, st) == HIPBLAS_STATUS_SUCCESS;
}

// the dense products of the layer: hipBLASLt where it has an algorithm (always, with the bias + ReLU epilogue or
// without), else rocBLAS (and the caller's own bias + ReLU kernel: *fused says which).  BPT_LAYER_BLAS=rocblas in
// the environment keeps everything on rocBLAS (for comparisons).
struct Blas {
    rocblas_handle h;
    int device;
    hipStream_t st;
};
bool lt_enabled() {   // read at every call: a process can compare the two paths
    const char* e = getenv("BPT_LAYER_BLAS");
    return !(e && std::string(e) == "rocblas");
}
int gemm(const Blas& b, int64_t M, int64_t N, int64_t K, const void* A, bool ta, const void* B, bool tb, void* C, bool c_fp32,
         int64_t lda = 0, int64_t ldc = 0, const float* bias_relu = nullptr, bool* fused = nullptr) {
    if (fused) *fused = false;
    if (lt_enabled() && gemm_lt(b.device, b.st, M, N, K, A, ta, B, tb, C, c_fp32, lda, ldc, bias_relu, nullptr)) {
        if (fused) *fused = true;
        return BPT_OK;
    }
    return gemm_rm(b.h, M, N, K, A, ta, B, tb, C, c_fp32, 0.f, lda, ldc);
}
// C (bf16) = add (bf16) + op(A) op(B) in one product where hipBLASLt has it; else false and nothing is written
bool gemm_add(const Blas& b, int64_t M, int64_t N, int64_t K, const void* A, bool ta, const void* B, bool tb, void* C,
              const void* add, int64_t lda = 0) {
    return lt_enabled() && gemm_lt(b.device, b.st, M, N, K, A, ta, B, tb, C, false, lda, 0, nullptr, add);
}

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
// the kernels here move 16 bytes per lane: every tensor has to start on a 16-byte boundary (null passes: optional
// arguments are checked where they are used)
template <typename... P>
bool any_misaligned(P... p) {
    const uintptr_t bits = (... | reinterpret_cast<uintptr_t>(static_cast<const void*>(p)));
    return (bits & 15u) != 0;
}

struct LayerBuffers {
    size_t qkvo, wqkv, lse, acc1, acc2, st1, st2, z, f1, attn, total;
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
    L.qkvo = take(rows * 4 * d * 2);   // [rows][Q | K | V | O]: the projections side by side, then the attention's output
    L.wqkv = take(d * 3 * d * 2);      // [d][Wq | Wk | Wv]
    L.lse = take((size_t)B * H * g->num_nodes * 4);
    L.acc1 = take(rows * d * 4);     // W^O result, fp32
    L.acc2 = take(rows * d * 4);     // W_2 result, fp32
    L.st1 = take(rows * sizeof(float2));   // (mean, 1/deviation) of the two normalisations
    L.st2 = take(rows * sizeof(float2));
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
    // Q, K, V and the attention's output of a node sit side by side, [B][N][Q | K | V | O][H][64] (one projection
    // writes the first three); the gradients of the backward use the same layout with dO in the fourth place
    s.stride_n = (int64_t)4 * H * kD;
    s.stride_h = kD;
    s.stride_b = (int64_t)g->num_nodes * 4 * H * kD;
    s.grad_dtype = BPT_BF16;                   // dQ, dK, dV feed bf16 GEMMs
    s.scale = scale;
    s.seq_len = seq_len;
    return s;
}

// slices of the contraction over K for an M x N result: enough to give every compute unit a tile
int pick_slices(int M, int N, int64_t K) {
    const int64_t tiles = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
    const int64_t want = (512 + tiles - 1) / tiles;
    return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, 16), K / 2048));
}

constexpr int kColumnSumBlocks = 2048;   // workgroups (= partial rows) of the kernels that sum over rows

struct LayerBwdBuffers {
    size_t ds2, dh, t, ds1, dqkvo, part, gw, attn, total;
};
LayerBwdBuffers layer_bwd_buffers(const bpt_graph* g, int B, int H, int d_ff, size_t attn_ws) {
    const size_t rows = (size_t)B * g->num_nodes, d = (size_t)H * kD;
    LayerBwdBuffers L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes);
        return at;
    };
    L.ds2 = take(rows * d * 2);              // gradient of the second pre-normalisation sum, bf16
    L.dh = take(rows * (size_t)d_ff * 2);    // gradient of the hidden FFN activations, bf16
    L.t = take(rows * d * 4);                // fp32 GEMM results: dH W1^T, later dQ Wq^T + dK Wk^T + dV Wv^T
    L.ds1 = take(rows * d * 2);
    L.dqkvo = take(rows * 4 * d * 2);        // [rows][dQ | dK | dV | dO] bf16: the attention's gradients, rounded to bf16 by its
                                             // backward, next to the gradient of its output -- the forward's layout
    L.part = take((size_t)kColumnSumBlocks * std::max<size_t>(3 * d, (size_t)d_ff) * 4);
    // partial products of the weight gradients (contraction over the rows, cut into slices)
    const size_t gw_qkv = (size_t)pick_slices((int)d, (int)(3 * d), (int64_t)rows) * d * 3 * d;
    const size_t gw_ffn = (size_t)pick_slices((int)d, d_ff, (int64_t)rows) * d * (size_t)d_ff;
    const size_t gw_o = (size_t)pick_slices((int)d, (int)d, (int64_t)rows) * d * d;
    L.gw = take(std::max(gw_qkv, std::max(gw_ffn, gw_o)) * 4);
    L.attn = take(attn_ws);
    L.total = off;
    return L;
}

// column sums of partials[parts][cols]; the columns are `cols / cols_each` outputs side by side
template <int CHUNKS>
int launch_ln_bwd_as(int blocks, hipStream_t st, const bf16_t* dy_b, const float* dy_f, const bf16_t* x, const float* a,
                     const float* bias, const float* gain, const float2* stats, bf16_t* ds, float* partials, int64_t rows, int d,
                     const int32_t* seq_len, int N, int lg) {
    const size_t lds = (size_t)9 * d * sizeof(float);
    if (lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(layer_norm_bwd_kernel<CHUNKS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    BPT_LAUNCH("layer_norm_bwd_kernel", layer_norm_bwd_kernel<CHUNKS>, dim3(blocks), dim3(256), lds, st, dy_b, dy_f, x, a, bias,
               gain, stats, ds, partials, rows, d, seq_len, N, lg);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}
template <typename... Args>
int launch_ln_bwd(int d, Args... args) {
    if (d <= 512) return launch_ln_bwd_as<1>(args...);
    if (d <= 1024) return launch_ln_bwd_as<2>(args...);
    return launch_ln_bwd_as<kLnMaxChunks>(args...);
}

int column_sum(const float* partials, int parts, int cols, int cols_each, float* o0, float* o1, float* o2, hipStream_t st) {
    const ColumnSumOut o = {{o0, o1, o2}, cols_each};
    BPT_LAUNCH("column_sum_kernel", column_sum_kernel, dim3((cols + 63) / 64), dim3(1024), 0, st, partials, parts, cols, o);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

// C[M][N] (fp32) = A^T B with A stored [K][M], B stored [K][N], bf16, K long and M x N small: the
// contraction is cut into `slices` equal parts that run as one strided-batched GEMM into
// `partials` [slices][M][N] (plus the few left-over rows of K into the first part), and the parts
// are added in slice order by sum_slices_kernel.  The N columns are N / n_each matrices side by
// side that go to out0..out2 (each [M][n_each]).
int gemm_at_b_sliced(rocblas_handle h, int M, int N, int64_t K, const void* A, const void* B, int ldb_cols, float* partials,
                     int slices, int n_each, float* out0, float* out1, float* out2, hipStream_t st, int lda_cols = 0) {
    const float one = 1.f, zero = 0.f;
    const int lda = lda_cols ? lda_cols : M;   // elements between rows of A as stored
    const int64_t ks = K / slices;
    if (ks < 1) return BPT_ERR_INVALID_ARG;
    // column-major view: C^T (N x M) = B^T-as-stored (N x K, ld = ldb_cols) times A (K x M) given as its transpose
    rocblas_status rs = rocblas_gemm_strided_batched_ex(
        h, rocblas_operation_none, rocblas_operation_transpose, N, M, (rocblas_int)ks, &one, B, rocblas_datatype_bf16_r, ldb_cols,
        ks * ldb_cols, A, rocblas_datatype_bf16_r, lda, ks * (int64_t)lda, &zero, partials, rocblas_datatype_f32_r, N, (int64_t)M * N,
        partials, rocblas_datatype_f32_r, N, (int64_t)M * N, slices, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    if (rs != rocblas_status_success) return BPT_ERR_LAUNCH;
    const int64_t done = ks * slices;
    if (done < K) {
        rs = rocblas_gemm_ex(h, rocblas_operation_none, rocblas_operation_transpose, N, M, (rocblas_int)(K - done), &one,
                             static_cast<const bf16_t*>(B) + done * ldb_cols, rocblas_datatype_bf16_r, ldb_cols,
                             static_cast<const bf16_t*>(A) + done * lda, rocblas_datatype_bf16_r, lda, &one, partials,
                             rocblas_datatype_f32_r, N, partials, rocblas_datatype_f32_r, N, rocblas_datatype_f32_r,
                             rocblas_gemm_algo_standard, 0, 0);
        if (rs != rocblas_status_success) return BPT_ERR_LAUNCH;
    }
    const ColumnSumOut o = {{out0, out1, out2}, n_each};
    const int64_t elems = (int64_t)M * N;
    BPT_LAUNCH("sum_slices_kernel", sum_slices_kernel, dim3((unsigned)((elems / 4 + 255) / 256)), dim3(256), 0, st, partials,
               slices, elems, N, o);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

// Workspace of the stack's forward: the states H^0 .. H^layers, then one layer workspace per layer.
struct StackBuffers {
    size_t state_bytes, layer_bytes, layers_at, total;
};
StackBuffers stack_buffers(const bpt_graph* g, int B, int H, int d_ff, int num_layers) {
    const bpt_shape_t s = attn_shape(g, B, H, 0.f, nullptr);
    StackBuffers S;
    S.state_bytes = align_up((size_t)B * g->num_nodes * H * kD * 2);
    const size_t attn_ws = bpt_attn_fwd_workspace(g, &s);
    S.layer_bytes = align_up(layer_buffers(g, B, H, d_ff, attn_ws == SIZE_MAX ? 0 : attn_ws).total);
    S.layers_at = S.state_bytes * ((size_t)num_layers + 1);
    S.total = S.layers_at + S.layer_bytes * (size_t)num_layers;
    return S;
}
constexpr int kMaxStackLayers = 256;

}  // namespace
}  // namespace bpt

using namespace bpt;

extern "C" {

size_t bpt_layer_fwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff) {
    if (!g || B < 1 || H < 1 || d_ff < 8) return 0;
    const bpt_shape_t s = attn_shape(g, B, H, 0.f, nullptr);
    const size_t attn_ws = bpt_attn_fwd_workspace(g, &s);
    if (attn_ws == SIZE_MAX) return SIZE_MAX;   // the attention calls refuse this graph and shape
    return layer_buffers(g, B, H, d_ff, attn_ws).total;
}

int bpt_layer_fwd(const bpt_graph_t* g, int32_t B, int32_t H, float scale, const int32_t* seq_len, const void* rel,
                  const void* X, const bpt_layer_params_t* p, void* Y, void* workspace, size_t workspace_bytes, void* stream) {
    if (!g || !rel || !X || !p || !Y || B < 1 || H < 1) return BPT_ERR_INVALID_ARG;
    if (!p->Wq || !p->Wk || !p->Wv || !p->Wo || !p->W1 || !p->W2 || !p->b1 || !p->b2 || !p->g1 || !p->beta1 || !p->g2 || !p->beta2)
        return BPT_ERR_INVALID_ARG;
    if (any_misaligned(X, Y, workspace, p->Wq, p->Wk, p->Wv, p->Wo, p->W1, p->W2, p->b1, p->b2, p->g1, p->beta1, p->g2, p->beta2))
        return BPT_ERR_INVALID_ARG;
    const int d = H * kD, d_ff = p->d_ff;
    if (d > 8 * 64 * kLnMaxChunks || d_ff < 8 || (d_ff & 7)) return BPT_ERR_UNSUPPORTED;
    const int64_t rows = (int64_t)B * g->num_nodes;
    if (rows > INT32_MAX) return BPT_ERR_UNSUPPORTED;
    const bpt_shape_t s = attn_shape(g, B, H, scale, seq_len);
    const size_t attn_ws = bpt_attn_fwd_workspace(g, &s);
    if (attn_ws == SIZE_MAX) return BPT_ERR_UNSUPPORTED;
    const LayerBuffers L = layer_buffers(g, B, H, d_ff, attn_ws);
    if (L.total > workspace_bytes || (L.total && !workspace)) return BPT_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rocblas_handle h = blas_handle(g->device);
    if (!h || rocblas_set_stream(h, st) != rocblas_status_success) return BPT_ERR_LAUNCH;
    const Blas bl = {h, g->device, st};
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    bf16_t* qkvo = reinterpret_cast<bf16_t*>(ws + L.qkvo);
    bf16_t* wqkv = reinterpret_cast<bf16_t*>(ws + L.wqkv);
    void *q = qkvo, *k = qkvo + d, *v = qkvo + 2 * d, *o = qkvo + 3 * d, *z = ws + L.z, *f1 = ws + L.f1;
    float* lse = reinterpret_cast<float*>(ws + L.lse);
    float* acc1 = reinterpret_cast<float*>(ws + L.acc1);
    float* acc2 = reinterpret_cast<float*>(ws + L.acc2);
    float2* st1 = reinterpret_cast<float2*>(ws + L.st1);
    float2* st2 = reinterpret_cast<float2*>(ws + L.st2);
    const float eps = p->eps > 0.f ? p->eps : 1e-5f;
    int rc;
    // [Q | K | V] = X [Wq | Wk | Wv] for all nodes in one product that reads X once: rows of [Q | K | V | O][H][64],
    // the layout the attention reads and writes through its strides (the packed weights stay in the workspace for
    // the backward)
    const PackArgs pa = {{static_cast<const bf16_t*>(p->Wq), static_cast<const bf16_t*>(p->Wk), static_cast<const bf16_t*>(p->Wv)}, wqkv};
    const int64_t wchunks = (int64_t)d * d / 8;
    BPT_LAUNCH("pack_qkv_weights_kernel", pack_qkv_weights_kernel, dim3((unsigned)((wchunks + 255) / 256), 3), dim3(256), 0, st, pa,
               wchunks, d);
    BPT_HIP(hipGetLastError());
    if ((rc = gemm(bl, rows, 3 * d, d, X, false, wqkv, false, qkvo, false, 0, 4 * d))) return rc;
    if ((rc = bpt_attn_fwd(g, &s, q, k, v, rel, o, lse, ws + L.attn, attn_ws, stream))) return rc;
    // Z = norm(X + O Wo)
    if ((rc = gemm(bl, rows, d, d, o, false, p->Wo, false, acc1, true, 4 * d))) return rc;
    const unsigned ln_blocks = (unsigned)((rows + 3) / 4);
    BPT_LAUNCH("residual_layer_norm_kernel", residual_layer_norm_kernel, dim3(ln_blocks), dim3(256), 0, st,
               static_cast<const bf16_t*>(X), acc1, static_cast<const float*>(nullptr), p->g1, p->beta1, static_cast<bf16_t*>(z),
               st1, rows, d, eps);
    BPT_HIP(hipGetLastError());
    // Y = norm(Z + max(0, Z W1 + b1) W2 + b2)
    bool fused = false;   // bias + ReLU in the product's epilogue, on the fp32 sums
    if ((rc = gemm(bl, rows, d_ff, d, z, false, p->W1, false, f1, false, 0, 0, p->b1, &fused))) return rc;
    if (!fused) {
        const int64_t chunks = rows * d_ff / 8;
        BPT_LAUNCH("bias_relu_kernel", bias_relu_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
                   static_cast<bf16_t*>(f1), p->b1, chunks, d_ff);
        BPT_HIP(hipGetLastError());
    }
    if ((rc = gemm(bl, rows, d, d_ff, f1, false, p->W2, false, acc2, true))) return rc;
    BPT_LAUNCH("residual_layer_norm_kernel", residual_layer_norm_kernel, dim3(ln_blocks), dim3(256), 0, st,
               static_cast<const bf16_t*>(z), acc2, p->b2, p->g2, p->beta2, static_cast<bf16_t*>(Y), st2, rows, d, eps);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

size_t bpt_layer_bwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff) {
    if (!g || B < 1 || H < 1 || d_ff < 8) return 0;
    const bpt_shape_t s = attn_shape(g, B, H, 0.f, nullptr);
    const size_t attn_ws = bpt_attn_bwd_workspace(g, &s);
    if (attn_ws == SIZE_MAX) return SIZE_MAX;
    return layer_bwd_buffers(g, B, H, d_ff, attn_ws).total;
}

int bpt_layer_bwd(const bpt_graph_t* g, int32_t B, int32_t H, float scale, const int32_t* seq_len, const void* rel,
                  const void* X, const bpt_layer_params_t* p, const void* fwd_workspace, size_t fwd_workspace_bytes,
                  const void* dY, void* dX, float* d_rel, const bpt_layer_grads_t* gr, void* workspace,
                  size_t workspace_bytes, void* stream) {
    if (!g || !rel || !X || !p || !fwd_workspace || !dY || !dX || !d_rel || !gr || B < 1 || H < 1) return BPT_ERR_INVALID_ARG;
    if (!p->Wq || !p->Wk || !p->Wv || !p->Wo || !p->W1 || !p->W2 || !p->b1 || !p->b2 || !p->g1 || !p->beta1 || !p->g2 || !p->beta2)
        return BPT_ERR_INVALID_ARG;
    if (!gr->dWq || !gr->dWk || !gr->dWv || !gr->dWo || !gr->dW1 || !gr->db1 || !gr->dW2 || !gr->db2 || !gr->dg1 ||
        !gr->dbeta1 || !gr->dg2 || !gr->dbeta2)
        return BPT_ERR_INVALID_ARG;
    if (any_misaligned(X, fwd_workspace, dY, dX, d_rel, workspace, p->Wq, p->Wk, p->Wv, p->Wo, p->W1, p->W2, p->b1, p->b2, p->g1,
                       p->beta1, p->g2, p->beta2, gr->dWq, gr->dWk, gr->dWv, gr->dWo, gr->dW1, gr->db1, gr->dW2, gr->db2, gr->dg1,
                       gr->dbeta1, gr->dg2, gr->dbeta2))
        return BPT_ERR_INVALID_ARG;
    const int d = H * kD, d_ff = p->d_ff;
    if (d > 8 * 64 * kLnMaxChunks || d_ff < 8 || (d_ff & 7) || d_ff > 8 * 256 * kReluChunks) return BPT_ERR_UNSUPPORTED;
    const int64_t rows = (int64_t)B * g->num_nodes;
    if (rows > INT32_MAX) return BPT_ERR_UNSUPPORTED;
    const bpt_shape_t s = attn_shape(g, B, H, scale, seq_len);
    const size_t attn_fws = bpt_attn_fwd_workspace(g, &s);
    const size_t attn_ws = bpt_attn_bwd_workspace(g, &s);
    if (attn_fws == SIZE_MAX || attn_ws == SIZE_MAX) return BPT_ERR_UNSUPPORTED;
    const LayerBuffers F = layer_buffers(g, B, H, d_ff, attn_fws);
    if (F.total > fwd_workspace_bytes) return BPT_ERR_INVALID_ARG;
    const LayerBwdBuffers L = layer_bwd_buffers(g, B, H, d_ff, attn_ws);
    if (L.total > workspace_bytes || !workspace) return BPT_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rocblas_handle h = blas_handle(g->device);
    if (!h || rocblas_set_stream(h, st) != rocblas_status_success) return BPT_ERR_LAUNCH;
    const Blas bl = {h, g->device, st};
    const unsigned char* fw = static_cast<const unsigned char*>(fwd_workspace);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const bf16_t* qkvo = reinterpret_cast<const bf16_t*>(fw + F.qkvo);
    const bf16_t* wqkv = reinterpret_cast<const bf16_t*>(fw + F.wqkv);
    const void *q = qkvo, *k = qkvo + d, *v = qkvo + 2 * d, *o = qkvo + 3 * d;
    const bf16_t* z = reinterpret_cast<const bf16_t*>(fw + F.z);
    const bf16_t* f1 = reinterpret_cast<const bf16_t*>(fw + F.f1);
    const float* lse = reinterpret_cast<const float*>(fw + F.lse);
    const float *acc1 = reinterpret_cast<const float*>(fw + F.acc1), *acc2 = reinterpret_cast<const float*>(fw + F.acc2);
    const float2 *st1 = reinterpret_cast<const float2*>(fw + F.st1), *st2 = reinterpret_cast<const float2*>(fw + F.st2);
    bf16_t *ds2 = reinterpret_cast<bf16_t*>(ws + L.ds2), *dh = reinterpret_cast<bf16_t*>(ws + L.dh);
    bf16_t *ds1 = reinterpret_cast<bf16_t*>(ws + L.ds1), *dqkvo = reinterpret_cast<bf16_t*>(ws + L.dqkvo);
    bf16_t* da = dqkvo + 3 * d;
    float *t = reinterpret_cast<float*>(ws + L.t), *part = reinterpret_cast<float*>(ws + L.part);
    float* gw = reinterpret_cast<float*>(ws + L.gw);
    const int lg = 31 - __builtin_clz((unsigned)g->n);
    const int ln_blocks = (int)std::min<int64_t>(kColumnSumBlocks, (rows + 3) / 4);
    const bf16_t* Xb = static_cast<const bf16_t*>(X);
    int rc;

    // second normalisation: dS2 (= the gradient of Z's residual branch, of the FFN output and of b2), dg2, dbeta2
    if ((rc = launch_ln_bwd(d, ln_blocks, st, static_cast<const bf16_t*>(dY), static_cast<const float*>(nullptr), z, acc2, p->b2,
                            p->g2, st2, ds2, part, rows, d, seq_len, g->num_nodes, lg)))
        return rc;
    if ((rc = column_sum(part, ln_blocks, 3 * d, d, gr->dg2, gr->dbeta2, gr->db2, st))) return rc;
    // FFN: dW2 = F^T dS2, dH = (dS2 W2^T) where the hidden unit was active, db1, dW1 = Z^T dH
    if ((rc = gemm_at_b_sliced(h, d_ff, d, rows, f1, ds2, d, gw, pick_slices(d, d_ff, rows), d, gr->dW2, nullptr, nullptr, st)))
        return rc;
    if ((rc = gemm(bl, rows, d_ff, d, ds2, false, p->W2, true, dh, false))) return rc;
    const int relu_blocks = (int)std::min<int64_t>(kColumnSumBlocks, rows);
    BPT_LAUNCH("relu_bwd_kernel", relu_bwd_kernel, dim3(relu_blocks), dim3(256), 0, st, dh, f1, part, rows, d_ff);
    BPT_HIP(hipGetLastError());
    if ((rc = column_sum(part, relu_blocks, d_ff, d_ff, gr->db1, nullptr, nullptr, st))) return rc;
    if ((rc = gemm_at_b_sliced(h, d, d_ff, rows, z, dh, d_ff, gw, pick_slices(d, d_ff, rows), d_ff, gr->dW1, nullptr, nullptr, st)))
        return rc;
    // first normalisation with dZ = dS2 + dH W1^T: dS1 (= the gradient of X's residual branch and of the
    // attention sublayer's output), dg1, dbeta1 (the third column sum, that of dS1, belongs to no parameter).
    // dZ is one product with dS2 as its addend (bf16, in the first half of t); without hipBLASLt the product
    // stays fp32 and the kernel adds
    bf16_t* dz = reinterpret_cast<bf16_t*>(t);
    const bool dz_joined = gemm_add(bl, rows, d, d_ff, dh, false, p->W1, true, dz, ds2);
    if (!dz_joined && (rc = gemm(bl, rows, d, d_ff, dh, false, p->W1, true, t, true))) return rc;
    if ((rc = launch_ln_bwd(d, ln_blocks, st, dz_joined ? static_cast<const bf16_t*>(dz) : static_cast<const bf16_t*>(ds2),
                            dz_joined ? static_cast<const float*>(nullptr) : static_cast<const float*>(t), Xb, acc1,
                            static_cast<const float*>(nullptr), p->g1, st1, ds1, part, rows, d,
                            static_cast<const int32_t*>(nullptr), g->num_nodes, lg)))
        return rc;
    if ((rc = column_sum(part, ln_blocks, 3 * d, d, gr->dg1, gr->dbeta1, nullptr, st))) return rc;
    // attention sublayer: dWo = O^T dS1, dO = dS1 Wo^T, then the attention's own backward
    if ((rc = gemm_at_b_sliced(h, d, d, rows, o, ds1, d, gw, pick_slices(d, d, rows), d, gr->dWo, nullptr, nullptr, st, 4 * d)))
        return rc;
    if ((rc = gemm(bl, rows, d, d, ds1, false, p->Wo, true, da, false, 0, 4 * d))) return rc;
    // dQ, dK, dV leave the attention's backward rounded to bf16, side by side next to dO: no cast pass
    if ((rc = bpt_attn_bwd(g, &s, q, k, v, rel, lse, da, dqkvo, dqkvo + d, dqkvo + 2 * d, d_rel, ws + L.attn, attn_ws, stream)))
        return rc;
    const int64_t chunks = rows * d / 8;
    // projections, one product each: [dWq | dWk | dWv] = X^T [dQ | dK | dV], dX = dS1 + [dQ | dK | dV] [Wq | Wk | Wv]^T
    if ((rc = gemm_at_b_sliced(h, d, 3 * d, rows, X, dqkvo, 4 * d, gw, pick_slices(d, 3 * d, rows), d, gr->dWq, gr->dWk, gr->dWv,
                               st)))
        return rc;
    // (the residual branch's gradient dS1 enters as the product's addend: one rounding, no pass of its own)
    if (gemm_add(bl, rows, d, 3 * d, dqkvo, false, wqkv, true, dX, ds1, 4 * d)) return BPT_OK;
    if ((rc = gemm(bl, rows, d, 3 * d, dqkvo, false, wqkv, true, t, true, 4 * d))) return rc;
    BPT_LAUNCH("add_cast_kernel", add_cast_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
               static_cast<const bf16_t*>(ds1), static_cast<const float*>(t), static_cast<bf16_t*>(dX), chunks);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

size_t bpt_stack_fwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff, int32_t num_layers) {
    if (!g || B < 1 || H < 1 || d_ff < 8 || num_layers < 1 || num_layers > kMaxStackLayers) return 0;
    if (g->batch > 0 && B != 1) return SIZE_MAX;   // the graph of a packed batch is the whole batch
    if (bpt_layer_fwd_workspace(g, B, H, d_ff) == SIZE_MAX) return SIZE_MAX;
    return stack_buffers(g, B, H, d_ff, num_layers).total;
}

int bpt_stack_fwd(const bpt_graph_t* g, int32_t B, int32_t H, int32_t num_layers, float scale, const int32_t* seq_len,
                  const void* const* rel, const void* E, const bpt_layer_params_t* p, void* root, void* tokens, void* workspace,
                  size_t workspace_bytes, void* stream) {
    if (!g || !rel || !E || !p || (!root && !tokens) || !workspace || B < 1 || H < 1 || num_layers < 1)
        return BPT_ERR_INVALID_ARG;
    if (num_layers > kMaxStackLayers) return BPT_ERR_UNSUPPORTED;
    if (g->batch > 0 && (B != 1 || seq_len)) return BPT_ERR_INVALID_ARG;   // the graph of a packed batch is the whole batch
    for (int l = 0; l < num_layers; ++l) {
        if (!rel[l]) return BPT_ERR_INVALID_ARG;
        if (p[l].d_ff != p[0].d_ff) return BPT_ERR_UNSUPPORTED;   // one workspace size serves every layer
    }
    if (p[0].d_ff < 8) return BPT_ERR_UNSUPPORTED;
    if (any_misaligned(E, root, tokens, workspace)) return BPT_ERR_INVALID_ARG;
    const StackBuffers S = stack_buffers(g, B, H, p[0].d_ff, num_layers);
    if (S.total > workspace_bytes) return BPT_ERR_INVALID_ARG;
    const int64_t rows = (int64_t)B * g->num_nodes;
    if (rows > INT32_MAX) return BPT_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const int row_chunks = H * kD / 8;
    const int64_t chunks = rows * row_chunks;
    BPT_LAUNCH("initial_states_kernel", initial_states_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
               static_cast<const bf16_t*>(E), reinterpret_cast<bf16_t*>(ws), chunks, g->n_tokens, g->num_nodes, row_chunks);
    BPT_HIP(hipGetLastError());
    for (int l = 0; l < num_layers; ++l) {
        const int rc = bpt_layer_fwd(g, B, H, scale, seq_len, rel[l], ws + S.state_bytes * l, &p[l], ws + S.state_bytes * (l + 1),
                                     ws + S.layers_at + S.layer_bytes * l, S.layer_bytes, stream);
        if (rc) return rc;
    }
    // a tree has one root, its last row; the graph of a packed batch one per sequence
    const int roots = g->batch > 0 ? g->batch : 1;
    const int64_t out_chunks = (int64_t)B * (g->n_tokens + roots) * row_chunks;
    BPT_LAUNCH("readout_kernel", readout_kernel, dim3((unsigned)((out_chunks + 255) / 256)), dim3(256), 0, st,
               reinterpret_cast<const bf16_t*>(ws + S.state_bytes * num_layers), static_cast<bf16_t*>(root),
               static_cast<bf16_t*>(tokens), out_chunks, g->n_tokens, g->num_nodes, row_chunks, roots,
               static_cast<const int32_t*>(g->batch > 0 ? g->d_root_row : nullptr));
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

size_t bpt_stack_bwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff) {
    if (!g || B < 1 || H < 1 || d_ff < 8) return 0;
    if (g->batch > 0 && B != 1) return SIZE_MAX;
    const size_t layer = bpt_layer_bwd_workspace(g, B, H, d_ff);
    if (layer == SIZE_MAX) return SIZE_MAX;
    return layer ? 2 * align_up((size_t)B * g->num_nodes * H * kD * 2) + layer : 0;
}

int bpt_stack_bwd(const bpt_graph_t* g, int32_t B, int32_t H, int32_t num_layers, float scale, const int32_t* seq_len,
                  const void* const* rel, const bpt_layer_params_t* p, const void* fwd_workspace, size_t fwd_workspace_bytes,
                  const void* d_root, const void* d_tokens, void* dE, float* const* d_rel, const bpt_layer_grads_t* grads,
                  void* workspace, size_t workspace_bytes, void* stream) {
    if (!g || !rel || !p || !fwd_workspace || (!d_root && !d_tokens) || !dE || !d_rel || !grads || !workspace || B < 1 ||
        H < 1 || num_layers < 1)
        return BPT_ERR_INVALID_ARG;
    if (num_layers > kMaxStackLayers) return BPT_ERR_UNSUPPORTED;
    if (g->batch > 0 && (B != 1 || seq_len)) return BPT_ERR_INVALID_ARG;
    for (int l = 0; l < num_layers; ++l) {
        if (!rel[l] || !d_rel[l]) return BPT_ERR_INVALID_ARG;
        if (p[l].d_ff != p[0].d_ff) return BPT_ERR_UNSUPPORTED;
    }
    if (p[0].d_ff < 8) return BPT_ERR_UNSUPPORTED;
    if (any_misaligned(fwd_workspace, d_root, d_tokens, dE, workspace)) return BPT_ERR_INVALID_ARG;
    const StackBuffers S = stack_buffers(g, B, H, p[0].d_ff, num_layers);
    if (S.total > fwd_workspace_bytes) return BPT_ERR_INVALID_ARG;
    const size_t need = bpt_stack_bwd_workspace(g, B, H, p[0].d_ff);
    if (need == SIZE_MAX) return BPT_ERR_UNSUPPORTED;
    if (!need || need > workspace_bytes) return BPT_ERR_INVALID_ARG;
    const int64_t rows = (int64_t)B * g->num_nodes;
    if (rows > INT32_MAX) return BPT_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned char* fw = static_cast<const unsigned char*>(fwd_workspace);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    unsigned char* dh[2] = {ws, ws + S.state_bytes};   // gradients with respect to the states, alternating
    unsigned char* layer_ws = ws + 2 * S.state_bytes;
    const int row_chunks = H * kD / 8;
    const int64_t chunks = rows * row_chunks;
    BPT_LAUNCH("readout_bwd_kernel", readout_bwd_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
               static_cast<const bf16_t*>(d_root), static_cast<const bf16_t*>(d_tokens), reinterpret_cast<bf16_t*>(dh[0]), chunks,
               g->n_tokens, g->num_nodes, row_chunks, g->batch > 0 ? g->batch : 1, g->batch > 0 ? g->first_root : g->num_nodes - 1,
               static_cast<const int32_t*>(g->batch > 0 ? g->d_root_seq : nullptr));
    BPT_HIP(hipGetLastError());
    int cur = 0;
    for (int l = num_layers - 1; l >= 0; --l, cur ^= 1) {
        const int rc = bpt_layer_bwd(g, B, H, scale, seq_len, rel[l], fw + S.state_bytes * l, &p[l],
                                     fw + S.layers_at + S.layer_bytes * l, S.layer_bytes, dh[cur], dh[cur ^ 1], d_rel[l], &grads[l],
                                     layer_ws, workspace_bytes - 2 * S.state_bytes, stream);
        if (rc) return rc;
    }
    // the embeddings are the token rows of the first states; the zero rows of the spans have no parameter behind them
    const int64_t out_chunks = (int64_t)B * (g->n_tokens + 1) * row_chunks;
    BPT_LAUNCH("readout_kernel", readout_kernel, dim3((unsigned)((out_chunks + 255) / 256)), dim3(256), 0, st,
               reinterpret_cast<const bf16_t*>(dh[cur]), static_cast<bf16_t*>(nullptr), static_cast<bf16_t*>(dE), out_chunks,
               g->n_tokens, g->num_nodes, row_chunks, 1, static_cast<const int32_t*>(nullptr));
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

}  // extern "C"
