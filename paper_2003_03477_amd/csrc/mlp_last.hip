// The one-unit output layer of the top MLP for the bf16 paths (gfx950): a matrix-vector
// product per sample, far too thin for the matrix cores, so it runs on the vector units fused
// with what surrounds it -- forward with the mean log-loss and dL/dlogit (Section 4,
// "Evaluation Metrics": the loss whose normalised form is NE), backward with the weight, bias
// and data gradients in one pass.  Operands are rounded to bfloat16 exactly as the MFMA
// kernels round theirs; sums are fp32.
#include "ss_internal.h"

namespace ss {

namespace {
__device__ __forceinline__ uint16_t to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float((uint32_t)h << 16);
}
}  // namespace

// Last top layer (one output unit) fused with the loss: logit_b = <q(x_b), q(w)> + bias,
// mean log-loss max(l,0) - l*y + log1p(exp(-|l|)) accumulated into *loss (zeroed earlier in
// the step), dlogit_b = (sigmoid(l) - y)/B.  16 lanes per sample.
__global__ __launch_bounds__(256) void last_layer_fwd_loss_kernel(
    const uint16_t* __restrict__ X, int ldx, const float* __restrict__ w,
    const float* __restrict__ bias, const float* __restrict__ y, int B, int in,
    float* __restrict__ logits, float* __restrict__ dlogit, float* __restrict__ loss) {
  __shared__ float part[16];
  const int sub = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int b = blockIdx.x * 16 + sl;
  float s = 0.f;
  if (b < B) {
    const uint16_t* xr = X + (size_t)b * ldx;
    for (int k = sub * 8; k < in; k += 128) {
      if (k + 8 <= in && ((((uintptr_t)(xr + k)) & 15) == 0)) {
        const uint4 xv = *(const uint4*)(xr + k);
        const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float xf = bf16_to_f32((uint16_t)(xw[j >> 1] >> ((j & 1) * 16)));
          s += xf * bf16_to_f32(to_bf16(w[k + j]));
        }
      } else {
        for (int j = 0; j < 8 && k + j < in; ++j)
          s += bf16_to_f32(xr[k + j]) * bf16_to_f32(to_bf16(w[k + j]));
      }
    }
  }
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) s += __shfl_xor(s, off);
  float lossv = 0.f;
  const float invB = 1.0f / (float)B;
  if (b < B && sub == 0) {
    const float l = s + bias[0], t = y[b];
    const float ex = expf(-fabsf(l));
    lossv = fmaxf(l, 0.f) - l * t + log1pf(ex);
    const float p = (l >= 0.f) ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
    logits[b] = l;
    if (dlogit) dlogit[b] = (p - t) * invB;
  }
  if (sub == 0) part[sl] = lossv;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) tot += part[i];
    atomicAdd(loss, tot * invB);
  }
}

void launch_last_layer_fwd_loss(const uint16_t* X, int ldx, const float* w, const float* bias,
                                const float* y, int B, int in, float* logits, float* dlogit,
                                float* loss, hipStream_t s) {
  hipLaunchKernelGGL(last_layer_fwd_loss_kernel, dim3(ceil_div(B, 16)), dim3(256), 0, s, X, ldx, w,
                     bias, y, B, in, logits, dlogit, loss);
}

// Training step.  Forward as above plus the layer's whole backward in the same launch:
// dX[b,k] = q(dlogit_b) q(w_k), stored as bf16 and gated by X[b,k] > 0 when X is the output of
// a hidden layer (dX), or as fp32 without a gate when X is the interaction output (dX32; a
// model without hidden top layer); gW[k] += sum_b q(dlogit_b) X[b,k], gb += sum_b dlogit_b.
constexpr int LAST_ROWS_PB = 32;
// A block owns LAST_ROWS_PB samples: 8 lanes per sample compute the logit, the loss term and
// dL/dlogit, which stay in LDS for the block's backward pass over the same (cache-resident)
// rows of X.
__global__ __launch_bounds__(256) void last_layer_train_kernel(
    const uint16_t* __restrict__ X, int ldx, const float* __restrict__ w,
    const float* __restrict__ bias, const float* __restrict__ y, int B, int in,
    float* __restrict__ logits, float* __restrict__ dlogit, float* __restrict__ loss,
    uint16_t* __restrict__ dX, int lddx, float* __restrict__ dX32, int lddx32,
    float* __restrict__ gpart, int gstride) {
  static_assert(LAST_ROWS_PB * 8 == 256, "8 lanes per sample");
  __shared__ float dl[LAST_ROWS_PB], dlq[LAST_ROWS_PB], lossv[LAST_ROWS_PB];
  const int b0 = blockIdx.x * LAST_ROWS_PB;
  const int nb = min(LAST_ROWS_PB, B - b0);
  {
    const int sub = threadIdx.x & 7, sl = threadIdx.x >> 3;
    const int b = b0 + sl;
    float s = 0.f;
    if (sl < nb) {
      const uint16_t* xr = X + (size_t)b * ldx;
      for (int k = sub * 8; k < in; k += 64) {
        if (k + 8 <= in && ((((uintptr_t)(xr + k)) & 15) == 0)) {
          const uint4 xv = *(const uint4*)(xr + k);
          const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float xf = bf16_to_f32((uint16_t)(xw[j >> 1] >> ((j & 1) * 16)));
            s += xf * bf16_to_f32(to_bf16(w[k + j]));
          }
        } else {
          for (int j = 0; j < 8 && k + j < in; ++j)
            s += bf16_to_f32(xr[k + j]) * bf16_to_f32(to_bf16(w[k + j]));
        }
      }
    }
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) s += __shfl_xor(s, off);
    if (sub == 0) {
      float lv = 0.f, d = 0.f;
      if (sl < nb) {
        const float invB = 1.0f / (float)B;
        const float l = s + bias[0], t = y[b];
        const float ex = expf(-fabsf(l));
        lv = fmaxf(l, 0.f) - l * t + log1pf(ex);
        const float p = (l >= 0.f) ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
        d = (p - t) * invB;
        logits[b] = l;
        dlogit[b] = d;
      }
      lossv[sl] = lv;
      dl[sl] = d;
      dlq[sl] = bf16_to_f32(to_bf16(d));
    }
  }
  __syncthreads();
  float* const gcopy = gpart + (size_t)(blockIdx.x % LAST_GRAD_COPIES) * gstride;
  for (int k = threadIdx.x; k < in; k += 256) {
    const float wq = bf16_to_f32(to_bf16(w[k]));
    float acc = 0.f;
    // eight rows' loads in flight at a time (the rows are summed in ascending order all the same)
    for (int r0 = 0; r0 < nb; r0 += 8) {
      uint16_t xb[8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        xb[i] = (r0 + i < nb) ? X[(size_t)(b0 + r0 + i) * ldx + k] : (uint16_t)0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = r0 + i;
        if (r < nb) {
          const float d = dlq[r];
          acc += d * bf16_to_f32(xb[i]);
          if (dX32) dX32[(size_t)(b0 + r) * lddx32 + k] = d * wq;
          else dX[(size_t)(b0 + r) * lddx + k] = ((int16_t)xb[i] > 0) ? to_bf16(d * wq) : (uint16_t)0;
        }
      }
    }
    atomicAdd(gcopy + k, acc);
  }
  if (threadIdx.x == 0) {
    float sb = 0.f, tot = 0.f;
    for (int r = 0; r < nb; ++r) { sb += dl[r]; tot += lossv[r]; }
    atomicAdd(gcopy + in, sb);
    atomicAdd(loss, tot * (1.0f / (float)B));
  }
}

void launch_last_layer_train(const uint16_t* X, int ldx, const float* w, const float* bias,
                             const float* y, int B, int in, float* logits, float* dlogit,
                             float* loss, uint16_t* dX, int lddx, float* dX32, int lddx32,
                             float* gpart, int gstride, hipStream_t s) {
  hipLaunchKernelGGL(last_layer_train_kernel, dim3(ceil_div(B, LAST_ROWS_PB)), dim3(256), 0, s, X,
                     ldx, w, bias, y, B, in, logits, dlogit, loss, dX, lddx, dX32, lddx32, gpart,
                     gstride);
}

}  // namespace ss
