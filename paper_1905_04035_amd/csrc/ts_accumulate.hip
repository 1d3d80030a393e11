// ts_accumulate: the paper's two accumulation rules (arXiv 1905.04035, Section 3,
// Algorithm 1 and Section 6, Algorithm 2) for the gradients one variable receives.
//
// The rule picks a branch on the host; the branches are
//   reduce            sum_kernel: dense tensors added in list order, one streaming pass
//   convert + reduce  the dense tensor (or sum_kernel's sum of several) becomes dense_in of
//                     ts_densify_multi, which converts the slice gradients and adds them
//   gather            concat: every gradient as slices, laid end to end -- ids_kernel writes
//                     ids 0 .. V-1 for a dense tensor, copy kernels move ids and value rows
// This file sits on top of the public entry points; it shares no state with them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ts_densify.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kMaxDense = 16;     // dense tensors summed by one launch

struct DenseList {
    int32_t m;
    const float* src[kMaxDense];
};

// out[i] = ((src0[i] + src1[i]) + src2[i]) + ...   16 bytes per lane, grid-stride
__global__ __launch_bounds__(256) void sum_kernel(DenseList l, float* out, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        f4 acc = __builtin_nontemporal_load(reinterpret_cast<const f4*>(l.src[0]) + i);
        for (int j = 1; j < l.m; ++j) acc += __builtin_nontemporal_load(reinterpret_cast<const f4*>(l.src[j]) + i);
        __builtin_nontemporal_store(acc, reinterpret_cast<f4*>(out) + i);
    }
}

__global__ __launch_bounds__(256) void copy_f4_kernel(const float* src, float* dst, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const f4*>(src) + i),
                                    reinterpret_cast<f4*>(dst) + i);
}

// ids: copied from src, or 0 .. n-1 when src is NULL (a dense tensor taken as slices)
__global__ __launch_bounds__(256) void ids_kernel(const int32_t* src, int32_t* dst, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src ? src[i] : (int32_t)i;
}

unsigned grid_for(int64_t items)
{
    const int64_t wgs = (items + 255) / 256;
    return (unsigned)(wgs < 1 ? 1 : (wgs > 16384 ? 16384 : wgs));
}

int strategy_of(const ts_grad* grads, int32_t m, int32_t rule)
{
    if (m < 2) return TS_ACC_PASS_THROUGH;
    bool all_dense = true, any_dense = false;
    for (int i = 0; i < m; ++i) {
        if (grads[i].kind == TS_GRAD_DENSE) any_dense = true;
        else all_dense = false;
    }
    if (all_dense) return TS_ACC_REDUCE;
    if (rule == TS_RULE_PROPOSED && any_dense) return TS_ACC_DENSIFY_REDUCE;
    return TS_ACC_GATHER;
}

int check_list(const ts_grad* grads, int32_t m, int32_t rule)
{
    if (!grads) return TS_ERR_NULL;
    if (m < 1 || (rule != TS_RULE_TF && rule != TS_RULE_PROPOSED)) return TS_ERR_SHAPE;
    for (int i = 0; i < m; ++i) {
        const ts_grad& g = grads[i];
        if (g.kind != TS_GRAD_DENSE && g.kind != TS_GRAD_SLICES) return TS_ERR_SHAPE;
        if (g.kind == TS_GRAD_SLICES && g.n < 0) return TS_ERR_SHAPE;
        const bool empty = g.kind == TS_GRAD_SLICES && g.n == 0;
        if (!empty && !g.values) return TS_ERR_NULL;
        if (g.kind == TS_GRAD_SLICES && g.n > 0 && !g.ids) return TS_ERR_NULL;
        if ((uintptr_t)g.values & 15u) return TS_ERR_ALIGN;
    }
    return TS_OK;
}

}  // namespace

extern "C" {

int ts_accumulate_strategy(const ts_grad* grads, int32_t m, int32_t rule, int32_t* strategy_out)
{
    if (!strategy_out) return TS_ERR_NULL;
    const int rc = check_list(grads, m, rule);
    if (rc != TS_OK) return rc;
    *strategy_out = strategy_of(grads, m, rule);
    return TS_OK;
}

int ts_accumulate(const ts_grad* grads, int32_t m, int32_t rule, int32_t d, int32_t V, float* dense_out,
                  int32_t* ids_out, float* rows_out, int64_t slice_capacity, int64_t* n_slices_out,
                  int32_t* strategy_out, void* stream_v)
{
    int rc = check_list(grads, m, rule);
    if (rc != TS_OK) return rc;
    if (V <= 0 || d <= 0 || (d % 4) != 0) return TS_ERR_SHAPE;
    hipStream_t stream = (hipStream_t)stream_v;
    const int st = strategy_of(grads, m, rule);
    if (strategy_out) *strategy_out = st;
    const int64_t vd4 = (int64_t)V * d / 4;

    const bool dense_result = st == TS_ACC_REDUCE || st == TS_ACC_DENSIFY_REDUCE ||
                              (st == TS_ACC_PASS_THROUGH && grads[0].kind == TS_GRAD_DENSE);
    if (dense_result) {
        if (!dense_out) return TS_ERR_NULL;
        if ((uintptr_t)dense_out & 15u) return TS_ERR_ALIGN;
        // the dense tensors, in list order
        DenseList l;
        l.m = 0;
        for (int i = 0; i < m; ++i)
            if (grads[i].kind == TS_GRAD_DENSE) {
                if (l.m == kMaxDense) return TS_ERR_SHAPE;
                l.src[l.m++] = grads[i].values;
            }
        for (int j = l.m; j < kMaxDense; ++j) l.src[j] = nullptr;
        if (st != TS_ACC_DENSIFY_REDUCE) {
            if (l.m == 1 && l.src[0] == dense_out) return TS_OK;       // passed through in place
            hipLaunchKernelGGL(sum_kernel, dim3(grid_for(vd4)), dim3(256), 0, stream, l, dense_out, vd4);
            return hipGetLastError() == hipSuccess ? TS_OK : TS_ERR_HIP;
        }
        // Algorithm 2, added branch: one dense tensor is the dense operand of the conversion as
        // it is; several are summed into dense_out first and the conversion adds in place
        const float* dense_in = l.src[0];
        if (l.m > 1) {
            hipLaunchKernelGGL(sum_kernel, dim3(grid_for(vd4)), dim3(256), 0, stream, l, dense_out, vd4);
            if (hipGetLastError() != hipSuccess) return TS_ERR_HIP;
            dense_in = dense_out;
        }
        const int32_t* ids_k[TS_MAX_SHARDS];
        const void* rows_k[TS_MAX_SHARDS];
        int64_t n_k[TS_MAX_SHARDS];
        int k = 0;
        for (int i = 0; i < m; ++i)
            if (grads[i].kind == TS_GRAD_SLICES) {
                if (k == TS_MAX_SHARDS) return TS_ERR_SHAPE;
                ids_k[k] = grads[i].ids;
                rows_k[k] = grads[i].values;
                n_k[k] = grads[i].n;
                ++k;
            }
        return ts_densify_multi(ids_k, rows_k, n_k, k, TS_ROW_FP32, d, V, dense_in, dense_out, stream);
    }

    // slices result: gather, or one slices gradient passed through
    int64_t total = 0;
    for (int i = 0; i < m; ++i) {
        total += grads[i].kind == TS_GRAD_DENSE ? (int64_t)V : grads[i].n;
        if (total >= ((int64_t)1 << 31)) return TS_ERR_OVERFLOW;
    }
    if (!n_slices_out) return TS_ERR_NULL;
    if (total > slice_capacity) return TS_ERR_CAPACITY;
    if (total > 0 && (!ids_out || !rows_out)) return TS_ERR_NULL;
    if ((uintptr_t)rows_out & 15u) return TS_ERR_ALIGN;
    *n_slices_out = total;
    int64_t at = 0;
    for (int i = 0; i < m; ++i) {
        const bool dense = grads[i].kind == TS_GRAD_DENSE;
        const int64_t n = dense ? (int64_t)V : grads[i].n;
        if (n == 0) continue;
        hipLaunchKernelGGL(ids_kernel, dim3(grid_for(n)), dim3(256), 0, stream, dense ? nullptr : grads[i].ids,
                           ids_out + at, n);
        const int64_t n4 = n * d / 4;
        hipLaunchKernelGGL(copy_f4_kernel, dim3(grid_for(n4)), dim3(256), 0, stream, grads[i].values,
                           rows_out + at * d, n4);
        at += n;
    }
    return hipGetLastError() == hipSuccess ? TS_OK : TS_ERR_HIP;
}

}  // extern "C"
