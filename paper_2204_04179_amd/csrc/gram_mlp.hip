// Two-layer stand-in for the content encoder (bf16 features and weights):
//   z = x . W1        a = max(z, 0), kept in bf16        h = a . W2
// Eq. 4 of the paper takes any encoder and its Proposition holds for any f; the hidden
// activation a is what has to be kept for the backward pass, and under GRAM it is kept once
// per unique item instead of once per interaction (the paper's section on GPU memory
// consumption).  Both contractions run in the kernels of the linear encoder (gram_gemm.hip);
// the rectifier and its gate are applied by those kernels as they store (epilogue modes); this
// file adds the one remaining element-wise kernel and the order of the launches.
#include "gram_internal.h"

namespace gram {

typedef float f32x4 __attribute__((ext_vector_type(4)));
// out = bf16(in) for the first *n_dev rows of `cols4` float4 columns (round to nearest even).
__global__ __launch_bounds__(kBlock) void k_to_bf16(const f32x4* __restrict__ in,
                                                    const int* __restrict__ n_dev, int cols4,
                                                    uint2* __restrict__ out)
{
    const int64_t total = (int64_t)*n_dev * cols4;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const f32x4 v = in[i];
        out[i] = make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
    }
}

static unsigned blocks_for(int64_t rows_max, int cols4)
{
    int64_t b = (rows_max * cols4 + kBlock - 1) / kBlock;
    if (b > 4096) b = 4096;
    return (unsigned)(b < 1 ? 1 : b);
}

bool mlp_forward(Ctx* c, const void* X, const void* W1, const void* W2, const int* uniq, const int* u_dev,
                 int64_t rows_max, void* A1, float* E, hipStream_t s, void* H_scatter, bool caller_wants_E)
{
    if (rows_max <= 0) return false;
    const int d_in = c->cfg.d_in, dh = c->cfg.d_hidden, d = c->cfg.d;
    void* a1 = A1 ? A1 : c->A1_ws;
    // the contraction kernels read the weights as the caller holds them where they can; otherwise a
    // transposed copy is made first
    const bool plain1 = gemm_reads_plain_b(c, rows_max, c->cfg.vocab_n, d_in, dh, kEpiReluBf16);
    if (!plain1) transpose_weight(c, W1, d_in, dh, c->W1t, s);
    // the first contraction stores a = bf16(max(z, 0)) directly: z itself is never written
    gemm_rows_bf16(c, X, c->cfg.vocab_n, d_in, uniq, c->cfg.pad_id, u_dev, rows_max, c->W1t, dh,
                   static_cast<float*>(a1), s, nullptr, true, kEpiReluBf16, nullptr, plain1 ? W1 : nullptr);
    const bool plain2 = gemm_reads_plain_b(c, rows_max, rows_max, dh, d, kEpiPlain);
    if (!plain2) transpose_weight(c, W2, dh, d, c->W2t, s);
    // rows of A1 are in the order of uniq: the identity list stands in for the gather, and no row is
    // "padding" by its index (the padding item's activation row is zero already)
    return gemm_rows_bf16(c, a1, rows_max, dh, c->iota, -1, u_dev, rows_max, c->W2t, d, E, s, H_scatter,
                          caller_wants_E, kEpiPlain, nullptr, plain2 ? W2 : nullptr);
}

int64_t mlp_batch_bytes(const Ctx* c, int64_t n)
{
    const int64_t dh = c->cfg.d_hidden, d = c->cfg.d;
    auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
    return up(n * dh * 4) + up(n * dh * 2) + up(n * d * 4) + up(n * d * 2);
}

void mlp_backward(Ctx* c, const void* X, const void* W1, const void* W2, const int* ids, const float* rows,
                  const float* Ht, int64_t n, void* work, float* dW1, float* dW2, bool accumulate,
                  double* loss_dev, hipStream_t s)
{
    const int d_in = c->cfg.d_in, dh = c->cfg.d_hidden, d = c->cfg.d;
    auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
    char* w = static_cast<char*>(work);
    float* Z = reinterpret_cast<float*>(w);                  // [n, dh] dL/dz
    void* A1 = w + up(n * dh * 4);                           // [n, dh] bf16 activations
    float* R = reinterpret_cast<float*>(w + up(n * dh * 4) + up(n * dh * 2));          // [n, d]
    void* Rb = w + up(n * dh * 4) + up(n * dh * 2) + up(n * d * 4);                    // [n, d] bf16
    const int* n_dev = c->scal + kSChunkN;

    chunk_ids_prepare(c, ids, n, s);
    if (n > 0) {
        const bool plain1 = gemm_reads_plain_b(c, n, c->cfg.vocab_n, d_in, dh, kEpiReluBf16);
        if (!plain1) transpose_weight(c, W1, d_in, dh, c->W1t, s);
        gemm_rows_bf16(c, X, c->cfg.vocab_n, d_in, c->chunk_ids, c->cfg.pad_id, n_dev, n, c->W1t, dh,
                       static_cast<float*>(A1), s, nullptr, true, kEpiReluBf16, nullptr, plain1 ? W1 : nullptr);
    }
    const float* Rsrc = rows;
    if (Ht) {
        // Algorithm 1 step 4 as a regression: output at the current weights minus the stored target
        if (n > 0) {
            const bool plain2 = gemm_reads_plain_b(c, n, n, dh, d, kEpiPlain);
            if (!plain2) transpose_weight(c, W2, dh, d, c->W2t, s);
            gemm_rows_bf16(c, A1, n, dh, c->iota, -1, n_dev, n, c->W2t, d, R, s, nullptr, true, kEpiPlain, nullptr,
                           plain2 ? W2 : nullptr);
        }
        // the miss kernel also leaves the bf16 copy of the miss that the dA contraction reads
        pseudo_miss(c, R, Ht, n, loss_dev, s, Rb);
        Rsrc = R;
    }
    // dW2 = A1^T R: the kept activations play the part of the features, row j with row j
    const WgradRows top = {nullptr, Rsrc, n_dev, n, n > 0 ? n : 1, dh, d, -1};
    encoder_wgrad(c, A1, dW2, s, 0, n, accumulate, &top);
    if (n > 0) {
        // dA = R . W2^T: W2 [dh, d] is already the K-contiguous second operand of that product; gradient
        // rows handed in by the caller are rounded to bf16 here (with targets the miss kernel did it)
        if (!Ht)
            launch(c, KID_MLP_TO_BF16, k_to_bf16, dim3(blocks_for(n, d / 4)), dim3(kBlock), s,
                   reinterpret_cast<const f32x4*>(Rsrc), n_dev, d / 4, reinterpret_cast<uint2*>(Rb));
        // the gate of the rectifier is applied as the product is stored: dZ = dA where the kept
        // activation is positive, so forward and backward agree on which units are active
        gemm_rows_bf16(c, Rb, n, d, c->iota, -1, n_dev, n, W2, dh, Z, s, nullptr, true, kEpiGate, A1);
    }
    // dW1 = X[ids]^T dZ
    const WgradRows bottom = {c->chunk_ids, Z, n_dev, n, c->cfg.vocab_n, d_in, dh, c->cfg.pad_id};
    encoder_wgrad(c, X, dW1, s, 0, n, accumulate, &bottom);
}

}  // namespace gram
