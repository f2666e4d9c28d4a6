// MLP passes reduced to tiled matrix products (section 2 of the paper):
//   forward  (equation 1)  Z_l = A_{l-1} W_l,  A_l = sigmoid(Z_l)  (sigmoid fused into the product's epilogue)
//   backward (equation 4)  D_{l-1} = (D_l W_l^T) * A_{l-1} * (1 - A_{l-1})   (derivative fused likewise)
//            (equation 3)  dW_l = A_{l-1}^T D_l
//   update                 W_l <- W_l - lr dW_l   (the dW product's epilogue writes straight into W_l)
// plus one row-wise kernel for softmax, cross-entropy and the output error D_L.
// Every product goes through the same tile GEMM kernel as tgemm_run, with tile size T.
#include <math.h>
#include <string.h>

#include <chrono>
#include <vector>

#include "common.h"
#include "gemm_kernel.h"

struct tgemm_mlp {
    tgemm_ctx* ctx = nullptr;
    int n_layers = 0;
    std::vector<int64_t> dims;
    std::vector<float*> W;
    int32_t T = 0;
    size_t budget = 0;
    int64_t cap_batch = 0;        // batch the workspaces were sized for
    int64_t batch = 0;            // batch of the last forward (0: none yet)
    const float* X = nullptr;     // input of the last forward (caller owned)
    std::vector<float*> act;      // act[l], l = 1..L-1 : batch x dims[l]
    std::vector<float*> delta;    // delta[l], l = 1..L : batch x dims[l]
    float* logits = nullptr;      // batch x dims[L]
    float* row_loss = nullptr;    // batch
    bool have_delta = false;
};

namespace tg {
namespace {

__device__ inline float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One workgroup per row of the logits.  P = softmax(z) with the row maximum subtracted;
// row_loss = -log P[label]; delta = (P - onehot(label)) * inv_batch.  probs / delta may be NULL.
__global__ __launch_bounds__(256) void softmax_xent_rows(const float* __restrict__ logits, int64_t ld, int n,
                                                         const int32_t* __restrict__ labels, float inv_batch,
                                                         float* __restrict__ delta, float* __restrict__ probs,
                                                         float* __restrict__ row_loss)
{
    __shared__ float red[4];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* z = logits + (int64_t)row * ld;
    float m = -INFINITY;
    for (int c = tid; c < n; c += 256) m = fmaxf(m, z[c]);
    m = wave_max(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float s = 0.f;
    for (int c = tid; c < n; c += 256) s += expf(z[c] - m);
    s = wave_sum(s);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    s = (red[0] + red[1]) + (red[2] + red[3]);
    const int y = labels[row];
    const float inv = 1.f / s;
    for (int c = tid; c < n; c += 256) {
        const float p = expf(z[c] - m) * inv;
        if (probs) probs[(int64_t)row * ld + c] = p;
        if (delta) delta[(int64_t)row * ld + c] = (p - (c == y ? 1.f : 0.f)) * inv_batch;
    }
    if (tid == 0) row_loss[row] = (y >= 0 && y < n) ? (logf(s) + m - z[y]) : NAN;
}

double now_ms()
{
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

void free_workspaces(tgemm_mlp* m)
{
    for (auto& p : m->act) { if (p) (void)hipFree(p); p = nullptr; }
    for (auto& p : m->delta) { if (p) (void)hipFree(p); p = nullptr; }
    if (m->logits) (void)hipFree(m->logits);
    if (m->row_loss) (void)hipFree(m->row_loss);
    m->logits = nullptr; m->row_loss = nullptr;
    m->cap_batch = 0; m->batch = 0; m->have_delta = false;
}

int ensure_workspaces(tgemm_mlp* m, int64_t batch)
{
    if (batch <= m->cap_batch) return TGEMM_OK;
    free_workspaces(m);
    const int L = m->n_layers;
    size_t total = (size_t)batch * 4;
    for (int l = 1; l <= L; ++l) total += (size_t)batch * m->dims[l] * 4 * 2;
    if (m->budget && total > m->budget)
        return fail(TGEMM_EBUDGET, "mlp: activations and errors for batch %lld need %zu bytes, hbm_budget is %zu",
                    (long long)batch, total, m->budget);
    auto alloc = [&](float** p, size_t bytes) -> bool {
        if (hipMalloc((void**)p, bytes) != hipSuccess) { (void)hipGetLastError(); *p = nullptr; return false; }
        return true;
    };
    bool ok = alloc(&m->row_loss, (size_t)batch * 4) && alloc(&m->logits, (size_t)batch * m->dims[L] * 4);
    for (int l = 1; l <= L && ok; ++l) {
        if (l < L) ok = ok && alloc(&m->act[l], (size_t)batch * m->dims[l] * 4);
        ok = ok && alloc(&m->delta[l], (size_t)batch * m->dims[l] * 4);
    }
    if (!ok) {
        free_workspaces(m);
        return fail(TGEMM_ENOMEM, "mlp: device allocation of %zu workspace bytes failed", total);
    }
    m->cap_batch = batch;
    return TGEMM_OK;
}

int launch(tgemm_mlp* m, GemmDesc& d)
{
    d.T = m->T;
    d.config = m->ctx->opts.kernel_config;
    hipError_t e = launch_tile_gemm_f32(d, m->ctx->streams[0]);
    if (e != hipSuccess) return fail(TGEMM_EHIP, "mlp: tile GEMM launch failed: %s", hipGetErrorString(e));
    m->ctx->stats.kernel_launches++;
    m->ctx->stats.n_tile_gemms += ((d.M + d.T - 1) / d.T) * ((d.N + d.T - 1) / d.T) * ((d.K + d.T - 1) / d.T);
    return TGEMM_OK;
}

// equation 1 for every layer
int forward(tgemm_mlp* m, const float* X, int64_t batch)
{
    const int L = m->n_layers;
    const float* in = X;
    for (int l = 1; l <= L; ++l) {
        GemmDesc d;
        memset(&d, 0, sizeof d);
        d.A = in; d.lda = m->dims[l - 1]; d.a_kcontig = 1;              // A_{l-1}: batch x n_{l-1}
        d.B = m->W[l - 1]; d.ldb = m->dims[l]; d.b_kcontig = 0;          // W_l: n_{l-1} x n_l
        d.C = (l < L) ? m->act[l] : m->logits; d.ldc = m->dims[l];
        d.M = batch; d.N = m->dims[l]; d.K = m->dims[l - 1];
        d.epilogue = (l < L) ? EPI_SIGMOID : EPI_AXPBY;
        d.alpha = 1.f; d.beta = 0.f;
        const int rc = launch(m, d);
        if (rc != TGEMM_OK) return rc;
        in = d.C;
    }
    m->X = X;
    m->batch = batch;
    m->have_delta = false;
    return TGEMM_OK;
}

int softmax(tgemm_mlp* m, const int32_t* labels, float* probs, bool want_delta)
{
    const int L = m->n_layers;
    const int64_t n = m->dims[L];
    hipLaunchKernelGGL(softmax_xent_rows, dim3((unsigned)m->batch), dim3(256), 0, m->ctx->streams[0],
                       m->logits, n, (int)n, labels, 1.f / (float)m->batch,
                       want_delta ? m->delta[L] : nullptr, probs, m->row_loss);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TGEMM_EHIP, "mlp: softmax launch failed: %s", hipGetErrorString(e));
    return TGEMM_OK;
}

int read_loss(tgemm_mlp* m, float* loss)
{
    hipStream_t st = m->ctx->streams[0];
    std::vector<float> rows((size_t)m->batch);
    TG_HIP(hipMemcpyAsync(rows.data(), m->row_loss, (size_t)m->batch * 4, hipMemcpyDeviceToHost, st));
    TG_HIP(hipStreamSynchronize(st));
    double s = 0.0;
    for (float v : rows) s += v;
    if (loss) *loss = (float)(s / (double)m->batch);
    return TGEMM_OK;
}

// equations 4 and 3 for every layer, last to first.  update: W_l <- W_l - lr dW_l in place of
// storing dW_l; dW: optional destinations for the plain gradients.
int backward(tgemm_mlp* m, void* const* dW, bool update, float lr)
{
    const int L = m->n_layers;
    const int64_t batch = m->batch;
    for (int l = L; l >= 1; --l) {
        const float* a_prev = (l == 1) ? m->X : m->act[l - 1];
        if (l > 1) {
            // D_{l-1} = (D_l W_l^T) * A_{l-1} * (1 - A_{l-1}); reads W_l before it is updated below
            GemmDesc d;
            memset(&d, 0, sizeof d);
            d.A = m->delta[l]; d.lda = m->dims[l]; d.a_kcontig = 1;          // D_l: batch x n_l
            d.B = m->W[l - 1]; d.ldb = m->dims[l]; d.b_kcontig = 1;          // W_l stored n_{l-1} x n_l = N x K
            d.C = m->delta[l - 1]; d.ldc = m->dims[l - 1];
            d.aux = a_prev; d.ldaux = m->dims[l - 1];
            d.M = batch; d.N = m->dims[l - 1]; d.K = m->dims[l];
            d.epilogue = EPI_DSIGMOID; d.alpha = 1.f; d.beta = 0.f;
            const int rc = launch(m, d);
            if (rc != TGEMM_OK) return rc;
        }
        if (update || (dW && dW[l - 1])) {
            // dW_l = A_{l-1}^T D_l
            GemmDesc d;
            memset(&d, 0, sizeof d);
            d.A = a_prev; d.lda = m->dims[l - 1]; d.a_kcontig = 0;           // stored K x M (batch x n_{l-1})
            d.B = m->delta[l]; d.ldb = m->dims[l]; d.b_kcontig = 0;          // batch x n_l
            d.M = m->dims[l - 1]; d.N = m->dims[l]; d.K = batch;
            d.ldc = m->dims[l];
            d.epilogue = EPI_AXPBY;
            if (update) { d.C = m->W[l - 1]; d.alpha = -lr; d.beta = 1.f; }
            else { d.C = (float*)dW[l - 1]; d.alpha = 1.f; d.beta = 0.f; }
            const int rc = launch(m, d);
            if (rc != TGEMM_OK) return rc;
        }
    }
    return TGEMM_OK;
}

int check_batch(tgemm_mlp* m, const void* X, int64_t batch)
{
    if (!m) return fail(TGEMM_EARG, "mlp: object is NULL");
    if (!X || batch <= 0 || batch > ((int64_t)1 << 30)) return fail(TGEMM_EARG, "mlp: bad input or batch %lld", (long long)batch);
    if (classify_pointer(X, m->ctx->device) != PTR_DEVICE) return fail(TGEMM_EARG, "mlp: X must be a device pointer");
    return TGEMM_OK;
}

}  // namespace
}  // namespace tg

using namespace tg;

extern "C" {

int mlp_create(tgemm_ctx* ctx, tgemm_mlp** out, int32_t n_layers, const int64_t* dims, void* const* W,
               int32_t dtype, int32_t T, size_t hbm_budget)
{
    if (!out) return fail(TGEMM_EARG, "mlp_create: out is NULL");
    *out = nullptr;
    if (!ctx || !dims || !W || n_layers < 1 || n_layers > 64 || T <= 0)
        return fail(TGEMM_EARG, "mlp_create: bad argument");
    if (dtype != TGEMM_F32) return fail(TGEMM_EARG, "mlp_create: only TGEMM_F32 is built so far");
    for (int l = 0; l <= n_layers; ++l)
        if (dims[l] <= 0 || dims[l] > ((int64_t)1 << 30)) return fail(TGEMM_EARG, "mlp_create: dims[%d] = %lld", l, (long long)dims[l]);
    TG_HIP(hipSetDevice(ctx->device));
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l]) return fail(TGEMM_EARG, "mlp_create: W[%d] is NULL", l);
        const PtrKind k = classify_pointer(W[l], ctx->device);
        if (k == PTR_PAGEABLE) return fail(TGEMM_EUNPINNED, "mlp_create: W[%d] is pageable host memory", l);
        if (k != PTR_DEVICE) return fail(TGEMM_EARG, "mlp_create: host-resident weights (out-of-core MLP) are not built yet");
    }
    tgemm_mlp* m = new (std::nothrow) tgemm_mlp();
    if (!m) return fail(TGEMM_ENOMEM, "mlp_create: host allocation failed");
    m->ctx = ctx;
    m->n_layers = n_layers;
    m->dims.assign(dims, dims + n_layers + 1);
    for (int l = 0; l < n_layers; ++l) m->W.push_back((float*)W[l]);
    m->T = T;
    m->budget = hbm_budget;
    m->act.assign(n_layers + 1, nullptr);
    m->delta.assign(n_layers + 1, nullptr);
    *out = m;
    return TGEMM_OK;
}

int mlp_destroy(tgemm_mlp* m)
{
    if (!m) return TGEMM_OK;
    (void)hipSetDevice(m->ctx->device);
    (void)hipStreamSynchronize(m->ctx->streams[0]);
    free_workspaces(m);
    delete m;
    return TGEMM_OK;
}

int mlp_forward(tgemm_mlp* m, const void* X, int64_t batch, float* probs)
{
    int rc = check_batch(m, X, batch);
    if (rc != TGEMM_OK) return rc;
    const double t0 = now_ms();
    memset(&m->ctx->stats, 0, sizeof m->ctx->stats);
    TG_HIP(hipSetDevice(m->ctx->device));
    if ((rc = ensure_workspaces(m, batch)) != TGEMM_OK) return rc;
    if ((rc = forward(m, (const float*)X, batch)) != TGEMM_OK) return rc;
    if (probs) {
        // softmax needs labels only for the loss; a zero label vector is not available here, so
        // the probabilities are produced by the same kernel with the row-loss output ignored
        TG_HIP(hipMemsetAsync(m->row_loss, 0, (size_t)batch * 4, m->ctx->streams[0]));
        if ((rc = softmax(m, (const int32_t*)m->row_loss, probs, false)) != TGEMM_OK) return rc;
    }
    TG_HIP(hipStreamSynchronize(m->ctx->streams[0]));
    m->ctx->stats.in_core = 1;
    m->ctx->stats.wall_ms = now_ms() - t0;
    return TGEMM_OK;
}

int mlp_backward(tgemm_mlp* m, const int32_t* labels, void* const* dW, float* loss)
{
    if (!m || !labels) return fail(TGEMM_EARG, "mlp_backward: NULL argument");
    if (m->batch <= 0) return fail(TGEMM_ESTATE, "mlp_backward: no forward pass precedes");
    const double t0 = now_ms();
    memset(&m->ctx->stats, 0, sizeof m->ctx->stats);
    TG_HIP(hipSetDevice(m->ctx->device));
    int rc;
    if ((rc = softmax(m, labels, nullptr, true)) != TGEMM_OK) return rc;
    if ((rc = backward(m, dW, false, 0.f)) != TGEMM_OK) return rc;
    if ((rc = read_loss(m, loss)) != TGEMM_OK) return rc;
    m->have_delta = true;
    m->ctx->stats.in_core = 1;
    m->ctx->stats.wall_ms = now_ms() - t0;
    return TGEMM_OK;
}

int mlp_step(tgemm_mlp* m, const void* X, const int32_t* labels, int64_t batch, float lr, float* loss)
{
    int rc = check_batch(m, X, batch);
    if (rc != TGEMM_OK) return rc;
    if (!labels) return fail(TGEMM_EARG, "mlp_step: labels is NULL");
    const double t0 = now_ms();
    memset(&m->ctx->stats, 0, sizeof m->ctx->stats);
    TG_HIP(hipSetDevice(m->ctx->device));
    if ((rc = ensure_workspaces(m, batch)) != TGEMM_OK) return rc;
    if ((rc = forward(m, (const float*)X, batch)) != TGEMM_OK) return rc;
    if ((rc = softmax(m, labels, nullptr, true)) != TGEMM_OK) return rc;
    if ((rc = backward(m, nullptr, true, lr)) != TGEMM_OK) return rc;
    if ((rc = read_loss(m, loss)) != TGEMM_OK) return rc;
    m->have_delta = true;
    m->ctx->stats.in_core = 1;
    m->ctx->stats.wall_ms = now_ms() - t0;
    return TGEMM_OK;
}

int mlp_read(tgemm_mlp* m, int32_t what, int32_t layer, void* dst, size_t bytes)
{
    if (!m || !dst) return fail(TGEMM_EARG, "mlp_read: NULL argument");
    if (m->batch <= 0) return fail(TGEMM_ESTATE, "mlp_read: no forward pass precedes");
    const int L = m->n_layers;
    const float* src = nullptr;
    size_t have = 0;
    if (what == 0 && layer >= 1 && layer < L) { src = m->act[layer]; have = (size_t)m->batch * m->dims[layer] * 4; }
    else if (what == 1) { src = m->logits; have = (size_t)m->batch * m->dims[L] * 4; }
    else if (what == 2 && layer >= 1 && layer <= L) {
        if (!m->have_delta) return fail(TGEMM_ESTATE, "mlp_read: no backward pass precedes");
        src = m->delta[layer]; have = (size_t)m->batch * m->dims[layer] * 4;
    }
    if (!src) return fail(TGEMM_EARG, "mlp_read: what=%d layer=%d", what, layer);
    if (bytes > have) return fail(TGEMM_EARG, "mlp_read: %zu bytes requested, matrix has %zu", bytes, have);
    TG_HIP(hipSetDevice(m->ctx->device));
    TG_HIP(hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost));
    return TGEMM_OK;
}

}  // extern "C"
