// np_sparse_adagrad: row-wise Adagrad on exactly the rows of the key list, in place in HBM (Section IV-B:
// gradients are applied directly to the vectors of the active buffer; Eq. (2): every other row keeps its
// bits).  One fused read-modify-write pass: an LPR-lane group owns a row, reads the gradient row
// (streamed) and the table row (random 16-byte loads from consecutive lanes), reduces the squared
// gradient across the group with a fixed butterfly, updates the one-float row state and writes the row.
#include "np_common.hpp"

namespace np {

#ifndef NP_ADAGRAD_MAX_GRID
#define NP_ADAGRAD_MAX_GRID 1048576  // one row per group up to 16 M rows of 64 floats (1.61 -> 1.59 ms against 65536 blocks)
#endif
constexpr int64_t kAdagradMaxGrid = NP_ADAGRAD_MAX_GRID;

template <int LPR, int NV, typename TabT>
__global__ void __launch_bounds__(256)
adagrad_kernel(TabT* __restrict__ table, float* __restrict__ state, int dim, const int64_t* __restrict__ list_keys,
               const float* __restrict__ grads, const int32_t* __restrict__ d_num_list, int cap, float lr, float eps, float inv_dim) {
    constexpr int GPB = 256 / LPR;
    const int r = threadIdx.x % LPR;
    const int words = dim / 4;
    const int L = device_count(d_num_list, cap);
    for (int64_t p = static_cast<int64_t>(blockIdx.x) * GPB + threadIdx.x / LPR; p < L; p += static_cast<int64_t>(gridDim.x) * GPB) {
        const int64_t key = list_keys[p];
        const float4* gsrc = reinterpret_cast<const float4*>(grads + static_cast<size_t>(p) * dim);
        TabT* wrow = table + static_cast<size_t>(key) * dim;
        float4 g[NV], w[NV];
        float ss = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            g[v] = make_float4(0.f, 0.f, 0.f, 0.f);
            w[v] = g[v];
            if (wv < words) {
                g[v] = load_stream(gsrc + wv);
                w[v] = load_word(wrow, wv);
            }
            ss += sumsq4(g[v]);
        }
        const float s_old = state[key];
#pragma unroll
        for (int d = LPR / 2; d > 0; d >>= 1) ss += __shfl_xor(ss, d, kWave);
        const float G = adagrad_state(s_old, ss, inv_dim);
        const float denom = sqrtf(G) + eps;
        if (r == 0) state[key] = G;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int wv = r + v * LPR;
            if (wv < words) {
                adagrad_step4(w[v], g[v], lr, denom);
                store_word_stream(wrow, wv, w[v]);  // a bf16 row is rounded to nearest even here
            }
        }
    }
}

template <int LPR, int NV, typename TabT>
void adagrad_launch(TabT* table, float* state, int dim, const int64_t* list_keys, const float* grads,
                    const int32_t* d_num_list, int cap, float lr, float eps, hipStream_t stream) {
    constexpr int GPB = 256 / LPR;
    int64_t want = (static_cast<int64_t>(cap) + GPB - 1) / GPB;
    const unsigned grid = static_cast<unsigned>(want < kAdagradMaxGrid ? want : kAdagradMaxGrid);
    NP_LAUNCH("sparse_adagrad", (adagrad_kernel<LPR, NV, TabT>), dim3(grid), dim3(256), 0, stream, table, state, dim, list_keys,
              grads, d_num_list, cap, lr, eps, 1.0f / static_cast<float>(dim));
}

template <typename TabT>
void adagrad_dispatch(TabT* table, float* state, int dim, const int64_t* list_keys, const float* grads, const int32_t* d_num_list,
                      int cap, float lr, float eps, hipStream_t s) {
    const int words = dim / 4;
    if (words <= 4) adagrad_launch<4, 1>(table, state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else if (words <= 8) adagrad_launch<8, 1>(table, state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else if (words <= 16) adagrad_launch<16, 1>(table, state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else if (words <= 32) adagrad_launch<32, 1>(table, state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else if (words <= 64) adagrad_launch<64, 1>(table, state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else if (words <= 128) adagrad_launch<64, 2>(table, state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else adagrad_launch<64, 4>(table, state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
}

}  // namespace np

extern "C" {

int np_sparse_adagrad_t(void* table, int32_t table_dtype, float* state, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                        const float* grads, const int32_t* d_num_list, int32_t cap, float lr, float eps, void* stream) {
    if (!table || !state || num_rows < 1 || cap < 0 || !d_num_list) return NP_ERR_INVALID_ARG;
    if (table_dtype != NP_F32 && table_dtype != NP_BF16 && table_dtype != NP_F16) return NP_ERR_INVALID_ARG;
    if (dim < 4 || dim % 4 != 0 || dim > NP_MAX_DIM) return NP_ERR_UNSUPPORTED;
    if (cap == 0) return NP_OK;
    if (!list_keys || !grads || !np::aligned(table, table_dtype == NP_F32 ? 16 : 8) || !np::aligned(grads, 16))
        return NP_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (table_dtype == NP_BF16)
        np::adagrad_dispatch(static_cast<uint16_t*>(table), state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else if (table_dtype == NP_F16)
        np::adagrad_dispatch(static_cast<__half*>(table), state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    else
        np::adagrad_dispatch(static_cast<float*>(table), state, dim, list_keys, grads, d_num_list, cap, lr, eps, s);
    return np::launch_status();
}

int np_sparse_adagrad(float* table, float* state, int64_t num_rows, int32_t dim, const int64_t* list_keys,
                      const float* grads, const int32_t* d_num_list, int32_t cap, float lr, float eps, void* stream) {
    return np_sparse_adagrad_t(table, NP_F32, state, num_rows, dim, list_keys, grads, d_num_list, cap, lr, eps, stream);
}

}  // extern "C"
