// HBM-bound helpers: the standalone online-softmax merge (forward algorithm),
// D = rowsum(dO o O) (Alg. 2), and fills.  One lane moves 16 or 32 bytes per tensor; the
// lanes of one row sit next to each other in one wave, so every row is read and written as
// whole contiguous head_dim vectors.
#include "common.hpp"
#include "kernels.hpp"

namespace burst {

static int grid_for(int64_t total) {
  const int64_t blocks = (total + 255) / 256;
  return (int)(blocks < 256 * 32 ? blocks : 256 * 32);
}

__device__ __forceinline__ f32x4 load4(const TensorDev& t, int64_t off) {
  if (t.is_f32) return *reinterpret_cast<const f32x4*>((const float*)t.ptr + off);
  bf16x4 x = *reinterpret_cast<const bf16x4*>((const __bf16*)t.ptr + off);
  return f32x4{(float)x[0], (float)x[1], (float)x[2], (float)x[3]};
}

__global__ __launch_bounds__(256) void lse_merge_kernel(MergeParams p) {
  const int d4 = p.head_dim / 4;
  const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * d4;
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int c = i % d4;
    int64_t rest = i / d4;
    const int hq = rest % p.q_heads;
    rest /= p.q_heads;
    const int row = rest % p.sq;
    const int b = rest / p.sq;
    float* lse_ptr = p.lse_acc.ptr + b * p.lse_acc.sb + hq * p.lse_acc.sh + row;
    const float a = *lse_ptr;
    const float bcur = p.lse_part.ptr[b * p.lse_part.sb + hq * p.lse_part.sh + row];
    const float mm = fmaxf(a, bcur);
    float w_old = 0.f, w_cur = 0.f, lse_new = -INFINITY;
    if (mm != -INFINITY) {
      const float e_old = __expf(a - mm), e_cur = __expf(bcur - mm);
      const float tot = e_old + e_cur;
      lse_new = mm + __logf(tot);
      w_old = e_old / tot;
      w_cur = e_cur / tot;
    }
    const int64_t off_acc = b * p.o_acc.sb + (int64_t)row * p.o_acc.ss + hq * p.o_acc.sh + c * 4;
    const int64_t off_part = b * p.o_part.sb + (int64_t)row * p.o_part.ss + hq * p.o_part.sh + c * 4;
    f32x4 oa = *reinterpret_cast<const f32x4*>((const float*)p.o_acc.ptr + off_acc);
    f32x4 op = load4(p.o_part, off_part);
    f32x4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // a weight of 0 must also silence a non-finite partner (0 * inf)
      float x = (w_cur != 0.f ? w_cur * op[e] : 0.f) + (w_old != 0.f ? w_old * oa[e] : 0.f);
      out[e] = x;
    }
    *reinterpret_cast<f32x4*>((float*)p.o_acc.ptr + off_acc) = out;
    if (p.o_out.ptr) {
      const int64_t off_out = b * p.o_out.sb + (int64_t)row * p.o_out.ss + hq * p.o_out.sh + c * 4;
      bf16x4 y = {(__bf16)out[0], (__bf16)out[1], (__bf16)out[2], (__bf16)out[3]};
      *reinterpret_cast<bf16x4*>((__bf16*)p.o_out.ptr + off_out) = y;
    }
    // all lanes of this row are in this wave and have already loaded lse_acc above
    if (c == 0) *lse_ptr = lse_new;
  }
}

hipError_t launch_lse_merge(const MergeParams& p, hipStream_t stream) {
  const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * (p.head_dim / 4);
  const int grid = grid_for(total);
  hipLaunchKernelGGL(lse_merge_kernel, dim3(grid), dim3(256), 0, stream, p);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void preprocess_bwd_kernel(PreParams p) {
  const int d8 = p.head_dim / 8;   // lanes per row: 8 (D=64) or 16 (D=128)
  const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * d8;
  const int64_t padded = (total + 255) / 256 * 256;   // whole waves run the shuffles
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < padded; i += (int64_t)gridDim.x * 256) {
    const bool live = i < total;
    const int64_t ii = live ? i : total - 1;
    const int c = ii % d8;
    int64_t rest = ii / d8;
    const int hq = rest % p.q_heads;
    rest /= p.q_heads;
    const int row = rest % p.sq;
    const int b = rest / p.sq;
    const int64_t off_o = b * p.o.sb + (int64_t)row * p.o.ss + hq * p.o.sh + c * 8;
    const int64_t off_do = b * p.d_o.sb + (int64_t)row * p.d_o.ss + hq * p.d_o.sh + c * 8;
    f32x4 o0 = load4(p.o, off_o), o1 = load4(p.o, off_o + 4);
    f32x4 g0 = load4(p.d_o, off_do), g1 = load4(p.d_o, off_do + 4);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc += o0[e] * g0[e] + o1[e] * g1[e];
    for (int s = 1; s < d8; s <<= 1) acc += __shfl_xor(acc, s, 64);
    if (live && c == 0) p.d.ptr[b * p.d.sb + hq * p.d.sh + row] = acc;
  }
}

hipError_t launch_preprocess_bwd(const PreParams& p, hipStream_t stream) {
  const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * (p.head_dim / 8);
  const int grid = grid_for(total);
  hipLaunchKernelGGL(preprocess_bwd_kernel, dim3(grid), dim3(256), 0, stream, p);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_empty_fwd_kernel(FwdParams p) {
  const int d4 = p.head_dim / 4;
  const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * d4;
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int c = i % d4;
    int64_t rest = i / d4;
    const int hq = rest % p.q_heads;
    rest /= p.q_heads;
    const int row = rest % p.sq;
    const int b = rest / p.sq;
    const int64_t off = b * p.o_part.sb + (int64_t)row * p.o_part.ss + hq * p.o_part.sh + c * 4;
    if (p.o_part.is_f32) {
      *reinterpret_cast<f32x4*>((float*)p.o_part.ptr + off) = f32x4{0.f, 0.f, 0.f, 0.f};
    } else {
      *reinterpret_cast<bf16x4*>((__bf16*)p.o_part.ptr + off) = bf16x4{(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
    }
    if (c == 0) p.lse_part.ptr[b * p.lse_part.sb + hq * p.lse_part.sh + row] = -INFINITY;
  }
}

hipError_t launch_fill_empty_fwd(const FwdParams& p, hipStream_t stream) {
  const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * (p.head_dim / 4);
  const int grid = grid_for(total);
  hipLaunchKernelGGL(fill_empty_fwd_kernel, dim3(grid), dim3(256), 0, stream, p);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void zero_tensor_kernel(TensorDev t, int batch, int rows, int heads, int head_dim) {
  const int d4 = head_dim / 4;
  const int64_t total = (int64_t)batch * rows * heads * d4;
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int c = i % d4;
    int64_t rest = i / d4;
    const int hh = rest % heads;
    rest /= heads;
    const int row = rest % rows;
    const int b = rest / rows;
    *reinterpret_cast<f32x4*>((float*)t.ptr + b * t.sb + (int64_t)row * t.ss + hh * t.sh + c * 4) =
        f32x4{0.f, 0.f, 0.f, 0.f};
  }
}

hipError_t launch_zero_tensor(const TensorDev& t, int32_t batch, int32_t rows, int32_t heads, int32_t head_dim,
                              hipStream_t stream) {
  const int64_t total = (int64_t)batch * rows * heads * (head_dim / 4);
  if (total == 0) return hipSuccess;
  const int grid = grid_for(total);
  hipLaunchKernelGGL(zero_tensor_kernel, dim3(grid), dim3(256), 0, stream, t, batch, rows, heads, head_dim);
  return hipGetLastError();
}

// Diagnostic: back-to-back independent bf16 MFMAs from registers, two waves per SIMD on every CU.
// With constant operands the chip holds its top clock; with random operands the same instruction
// stream runs at the clock the power limit allows, which is the ceiling an attention kernel with
// real data can reach.
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* sink, int iters, int random_operands) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t u = (threadIdx.x * 97u + e * 131u + blockIdx.x * 7u) * 2654435761u;
    const uint16_t wa = 0x3c00u | ((u >> 9) & 0x83ffu), wb = 0x3c00u | ((u >> 3) & 0x83ffu);   // |x| in [0.0078, 2)
    a[e] = random_operands ? __builtin_bit_cast(__bf16, wa) : (__bf16)1.0f;
    b[e] = random_operands ? __builtin_bit_cast(__bf16, wb) : (__bf16)0.5f;
  }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int v = 0; v < 16; ++v) c0[v] = c1[v] = c2[v] = c3[v] = 0.f;
  for (int i = 0; i < iters; ++i) {
    c0 = mfma32(a, b, c0);
    c1 = mfma32(a, b, c1);
    c2 = mfma32(a, b, c2);
    c3 = mfma32(a, b, c3);
    if ((i & 1023) == 1023) {   // keep the accumulators finite
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        c0[v] *= 1e-30f;
        c1[v] *= 1e-30f;
        c2[v] *= 1e-30f;
        c3[v] *= 1e-30f;
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
  if (sink && s == 12345.678f) sink[0] = s;   // never true in practice; keeps the loop alive
}

hipError_t launch_mfma_probe(float* sink, int iters, int random_operands, int64_t* flops, hipStream_t stream) {
  const int blocks = 512;   // 256 CUs x 2 work-groups x 4 waves
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, stream, sink, iters, random_operands);
  if (flops) *flops = (int64_t)blocks * 4 * iters * 4 * 32768;
  return hipGetLastError();
}

}  // namespace burst
