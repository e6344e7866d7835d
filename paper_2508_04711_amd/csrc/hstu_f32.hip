// fp32 jagged HSTU attention (forward, dk/dv pass, dq pass): the all-fp32 data type of the
// library, computed on the vector ALUs with IEEE division and the precise exponential so that
// results stay within 1e-5 of a double-precision evaluation of the section 2.1 equation.
//
// Same schedule items as the bf16 kernels.  A workgroup of 256 threads owns a tile of 64 rows,
// four adjacent lanes per row; lane c of a row holds elements c, c+4, c+8, ... of the row's
// vectors, so a dot product is a per-lane partial sum plus two cross-lane adds.  The other
// side's rows are staged through LDS 64 at a time and visited one by one.
#include "hstu_common.h"

namespace hstu {

namespace {

constexpr int TILE = 64;     // owner rows per item
constexpr int ST = 64;       // streamed rows per LDS tile
constexpr int THREADS = 256;

template <int SIDE>
__device__ __forceinline__ void visible_range(const Item& it, int g, int causal, int& beg, int& end) {
  beg = 0;
  end = it.seg_len[g];
  if (causal) {
    if (SIDE == 0) {
      const int e = it.pos0 + it.nrows - it.seg_pos0[g];
      end = e < 0 ? 0 : (e < end ? e : end);
    } else {
      const int b = it.pos0 - it.seg_pos0[g];
      beg = b < 0 ? 0 : (b < end ? b : end);
    }
  }
}

__device__ __forceinline__ bool fetch_item(const Plan& plan, int slot, Item& it) {
  if (slot >= plan.header[0]) return false;
  it = plan.items[plan.order[slot]];
  return it.nrows > 0;
}

// Sum over the four lanes of a row.
__device__ __forceinline__ float row_sum(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

// Copy `valid` rows (zero beyond) of a [*, H, D] fp32 tensor's head slice into a dense LDS tile.
template <int D>
__device__ __forceinline__ void stage(float* tile, const float* base, int64_t row_stride, int valid,
                                      int tid) {
  constexpr int V4 = D / 4;
  for (int c = tid; c < ST * V4; c += THREADS) {
    const int row = c / V4, col = (c % V4) * 4;
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < valid) x = *(const float4*)(base + row * row_stride + col);
    *(float4*)(tile + row * D + col) = x;
  }
}

template <int D>
__device__ __forceinline__ void load_part(float (&part)[D / 4], const float* row, bool valid, int c) {
#pragma unroll
  for (int i = 0; i < D / 4; ++i) part[i] = valid ? row[4 * i + c] : 0.f;
}

template <int D>
__device__ __forceinline__ float dot_part(const float (&part)[D / 4], const float* row, int c) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < D / 4; ++i) s = fmaf(part[i], row[4 * i + c], s);
  return s;
}

template <int D>
__device__ __forceinline__ void axpy_part(float (&acc)[D / 4], float w, const float* row, int c) {
#pragma unroll
  for (int i = 0; i < D / 4; ++i) acc[i] = fmaf(w, row[4 * i + c], acc[i]);
}

template <int D>
__device__ __forceinline__ void store_part(float* row, const float (&acc)[D / 4], float scale,
                                           int accumulate, int c) {
#pragma unroll
  for (int i = 0; i < D / 4; ++i) {
    float x = acc[i] * scale;
    if (accumulate) x += row[4 * i + c];
    row[4 * i + c] = x;
  }
}

__device__ __forceinline__ float sigmoid_precise(float x) { return 1.0f / (1.0f + expf(-x)); }

// Timestamp bias of one pair (0 without bias): the table entry of the bucket of the two rows'
// timestamp difference; `bucket` receives the bucket.
__device__ __forceinline__ float pair_bias(const AttnArgs& a, int t_own, int64_t streamed_row, int& bucket) {
  bucket = 0;
  if (!a.ts_rec) return 0.f;
  bucket = bias_bucket(abs_diff(t_own, a.ts_rec[streamed_row].ts), a.nb, a.fbits);
  return a.ts_w[bucket];
}
__device__ __forceinline__ int own_timestamp(const AttnArgs& a, int64_t row, bool on) {
  return (a.ts_rec && on) ? a.ts_rec_own[row].ts : 0;
}

// ---------------------------------------------------------------------------------------------
template <int DQK, int DV>
__global__ void __launch_bounds__(THREADS) hstu_fwd_f32(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) float kt[ST * DQK];
  __shared__ __attribute__((aligned(16))) float vt[ST * DV];
  const int H = a.num_heads;
  const int slot = blockIdx.x / H, h = blockIdx.x % H;
  Item it;
  if (!fetch_item(a.plan, slot, it)) return;
  const int tid = threadIdx.x, r = tid >> 2, c = tid & 3;
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const bool on = r < it.nrows;
  float qp[DQK / 4], op[DV / 4];
  load_part<DQK>(qp, (const float*)a.q + ((int64_t)it.row0 + r) * sq + h * DQK, on, c);
#pragma unroll
  for (int i = 0; i < DV / 4; ++i) op[i] = 0.f;
  const int qpos = it.pos0 + r;
  const int t_own = own_timestamp(a, (int64_t)it.row0 + r, on);

  for (int g = 0; g < it.nseg; ++g) {
    int beg, end;
    visible_range<0>(it, g, a.causal, beg, end);
    for (int t0 = beg; t0 < end; t0 += ST) {
      const int valid = end - t0 < ST ? end - t0 : ST;
      __syncthreads();
      stage<DQK>(kt, (const float*)a.k + ((int64_t)it.seg_row0[g] + t0) * sq + h * DQK, sq, valid, tid);
      stage<DV>(vt, (const float*)a.v + ((int64_t)it.seg_row0[g] + t0) * sv + h * DV, sv, valid, tid);
      __syncthreads();
      for (int j = 0; j < valid; ++j) {
        int bucket;
        const float s = row_sum(dot_part<DQK>(qp, kt + j * DQK, c)) +
                        pair_bias(a, t_own, (int64_t)it.seg_row0[g] + t0 + j, bucket);
        const float x = a.alpha * s;
        float p = x * sigmoid_precise(x);
        const int kpos = it.seg_pos0[g] + t0 + j;
        if (a.causal && kpos > qpos) p = 0.f;
        axpy_part<DV>(op, p, vt + j * DV, c);
      }
    }
  }
  if (on)
    store_part<DV>((float*)a.o + ((int64_t)it.row0 + r) * sv + h * DV, op, a.inv_n, a.accumulate, c);
}

// ---------------------------------------------------------------------------------------------
template <int DQK, int DV>
__global__ void __launch_bounds__(THREADS) hstu_dkdv_f32(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) float qt[ST * DQK];
  __shared__ __attribute__((aligned(16))) float gt[ST * DV];
  const int H = a.num_heads;
  const int slot = blockIdx.x / H, h = blockIdx.x % H;
  Item it;
  if (!fetch_item(a.plan, slot, it)) return;
  const int tid = threadIdx.x, r = tid >> 2, c = tid & 3;
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const bool on = r < it.nrows;
  float kp[DQK / 4], vp[DV / 4], dkp[DQK / 4], dvp[DV / 4];
  load_part<DQK>(kp, (const float*)a.k + ((int64_t)it.row0 + r) * sq + h * DQK, on, c);
  load_part<DV>(vp, (const float*)a.v + ((int64_t)it.row0 + r) * sv + h * DV, on, c);
#pragma unroll
  for (int i = 0; i < DQK / 4; ++i) dkp[i] = 0.f;
#pragma unroll
  for (int i = 0; i < DV / 4; ++i) dvp[i] = 0.f;
  const int kpos = it.pos0 + r;
  const int t_own = own_timestamp(a, (int64_t)it.row0 + r, on);

  for (int g = 0; g < it.nseg; ++g) {
    int beg, end;
    visible_range<1>(it, g, a.causal, beg, end);
    for (int t0 = beg; t0 < end; t0 += ST) {
      const int valid = end - t0 < ST ? end - t0 : ST;
      __syncthreads();
      stage<DQK>(qt, (const float*)a.q + ((int64_t)it.seg_row0[g] + t0) * sq + h * DQK, sq, valid, tid);
      stage<DV>(gt, (const float*)a.d_o + ((int64_t)it.seg_row0[g] + t0) * sv + h * DV, sv, valid, tid);
      __syncthreads();
      for (int i = 0; i < valid; ++i) {
        int bucket;
        const float s = row_sum(dot_part<DQK>(kp, qt + i * DQK, c)) +
                        pair_bias(a, t_own, (int64_t)it.seg_row0[g] + t0 + i, bucket);
        const float dp = row_sum(dot_part<DV>(vp, gt + i * DV, c));
        const float x = a.alpha * s;
        const float sg = sigmoid_precise(x);
        float p = x * sg;
        float ds = dp * sg * (1.0f + x * (1.0f - sg));
        const int qpos = it.seg_pos0[g] + t0 + i;
        if (a.causal && kpos > qpos) { p = 0.f; ds = 0.f; }
        axpy_part<DV>(dvp, p, gt + i * DV, c);
        axpy_part<DQK>(dkp, ds, qt + i * DQK, c);
      }
    }
  }
  if (on) {
    store_part<DQK>((float*)a.dk + ((int64_t)it.row0 + r) * sq + h * DQK, dkp, a.alpha * a.inv_n,
                    a.accumulate, c);
    store_part<DV>((float*)a.dv + ((int64_t)it.row0 + r) * sv + h * DV, dvp, a.inv_n, a.accumulate, c);
  }
}

// ---------------------------------------------------------------------------------------------
template <int DQK, int DV>
__global__ void __launch_bounds__(THREADS) hstu_dq_f32(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) float kt[ST * DQK];
  __shared__ __attribute__((aligned(16))) float vt[ST * DV];
  __shared__ unsigned long long dwl[MAX_TS_BUCKETS];  // the workgroup's sums of dS per bucket (fixed point)
  const int H = a.num_heads;
  const int slot = blockIdx.x / H, h = blockIdx.x % H;
  Item it;
  if (!fetch_item(a.plan, slot, it)) return;
  const int tid = threadIdx.x, r = tid >> 2, c = tid & 3;
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const bool on = r < it.nrows;
  const bool want_dw = a.ts_rec && a.d_ts_acc;
  if (want_dw)
    for (int i = tid; i < a.nb; i += THREADS) dwl[i] = 0ull;  // (the loop's first barrier orders this)
  float qp[DQK / 4], gp[DV / 4], dqp[DQK / 4];
  load_part<DQK>(qp, (const float*)a.q + ((int64_t)it.row0 + r) * sq + h * DQK, on, c);
  load_part<DV>(gp, (const float*)a.d_o + ((int64_t)it.row0 + r) * sv + h * DV, on, c);
#pragma unroll
  for (int i = 0; i < DQK / 4; ++i) dqp[i] = 0.f;
  const int qpos = it.pos0 + r;
  const int t_own = own_timestamp(a, (int64_t)it.row0 + r, on);

  for (int g = 0; g < it.nseg; ++g) {
    int beg, end;
    visible_range<0>(it, g, a.causal, beg, end);
    for (int t0 = beg; t0 < end; t0 += ST) {
      const int valid = end - t0 < ST ? end - t0 : ST;
      __syncthreads();
      stage<DQK>(kt, (const float*)a.k + ((int64_t)it.seg_row0[g] + t0) * sq + h * DQK, sq, valid, tid);
      stage<DV>(vt, (const float*)a.v + ((int64_t)it.seg_row0[g] + t0) * sv + h * DV, sv, valid, tid);
      __syncthreads();
      for (int j = 0; j < valid; ++j) {
        int bucket;
        const float s = row_sum(dot_part<DQK>(qp, kt + j * DQK, c)) +
                        pair_bias(a, t_own, (int64_t)it.seg_row0[g] + t0 + j, bucket);
        const float dp = row_sum(dot_part<DV>(gp, vt + j * DV, c));
        const float x = a.alpha * s;
        const float sg = sigmoid_precise(x);
        float ds = dp * sg * (1.0f + x * (1.0f - sg));
        const int kpos = it.seg_pos0[g] + t0 + j;
        if (a.causal && kpos > qpos) ds = 0.f;
        axpy_part<DQK>(dqp, ds, kt + j * DQK, c);
        // one of the row's four lanes adds the pair's dS to its bucket (rows without an owner
        // have dS = 0: their q and d_o parts are zero)
        if (want_dw && c == 0 && ds != 0.f) atomicAdd(dwl + bucket, dw_to_fixed(ds));
      }
    }
  }
  if (want_dw) {
    __syncthreads();
    for (int i = tid; i < a.nb; i += THREADS)
      if (dwl[i] != 0ull) atomicAdd(a.d_ts_acc + i, dw_from_fixed(dwl[i]));
  }
  if (on)
    store_part<DQK>((float*)a.dq + ((int64_t)it.row0 + r) * sq + h * DQK, dqp, a.alpha * a.inv_n,
                    a.accumulate, c);
}

}  // namespace

int tile_rows_f32(int /*pass*/) { return TILE; }

#define HSTU_DISPATCH_F32(KERNEL)                                                          \
  do {                                                                                     \
    const dim3 grid((unsigned)((int64_t)a.max_items * a.num_heads)), block(THREADS);       \
    if (d_qk == 128 && d_v == 128) hipLaunchKernelGGL((KERNEL<128, 128>), grid, block, 0, stream, a); \
    else if (d_qk == 64 && d_v == 64) hipLaunchKernelGGL((KERNEL<64, 64>), grid, block, 0, stream, a); \
    else if (d_qk == 32 && d_v == 32) hipLaunchKernelGGL((KERNEL<32, 32>), grid, block, 0, stream, a); \
    else if (d_qk == 128 && d_v == 64) hipLaunchKernelGGL((KERNEL<128, 64>), grid, block, 0, stream, a); \
    else if (d_qk == 64 && d_v == 128) hipLaunchKernelGGL((KERNEL<64, 128>), grid, block, 0, stream, a); \
    else if (d_qk == 128 && d_v == 32) hipLaunchKernelGGL((KERNEL<128, 32>), grid, block, 0, stream, a); \
    else if (d_qk == 32 && d_v == 128) hipLaunchKernelGGL((KERNEL<32, 128>), grid, block, 0, stream, a); \
    else if (d_qk == 64 && d_v == 32) hipLaunchKernelGGL((KERNEL<64, 32>), grid, block, 0, stream, a); \
    else if (d_qk == 32 && d_v == 64) hipLaunchKernelGGL((KERNEL<32, 64>), grid, block, 0, stream, a); \
    else return hipErrorInvalidValue;                                                      \
    return hipGetLastError();                                                              \
  } while (0)

hipError_t launch_fwd_f32(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  HSTU_DISPATCH_F32(hstu_fwd_f32);
}
hipError_t launch_dkdv_f32(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  HSTU_DISPATCH_F32(hstu_dkdv_f32);
}
hipError_t launch_dq_f32(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  HSTU_DISPATCH_F32(hstu_dq_f32);
}

}  // namespace hstu
