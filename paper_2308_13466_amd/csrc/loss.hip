// Gradient of the local loss (Eq. 4 with softmax cross-entropy as Loss):
// dH = (softmax(H^(L)) - onehot(y)) / n over the partition's local nodes, and
// optionally the mean loss itself. One wavefront per node (eight nodes one after
// another, their rows requested together); classes are spread over the 64 lanes
// and reduced with lane-xor shuffles. The loss is summed in
// two fixed-order stages (per block into the workspace, then one block), so
// it is identical from run to run.
#include <math.h>

#include <mutex>
#include <type_traits>

#include "sat_internal.h"

namespace {

using sat::kWave;
constexpr int kRowsPerWave = 8;    // nodes a wavefront holds in registers at a time
constexpr int kRounds = 4;         // such batches per wavefront (fewer, longer-lived workgroups)
constexpr int kRowsPerBlock = 4 * kRowsPerWave * kRounds;

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// element access for fp32 (ES = 4) or bf16 (ES = 2) rows; bf16 stores round to nearest-even
template <int ES>
__device__ __forceinline__ float ld_elem(const void* row, int c) {
  if constexpr (ES == 4) return static_cast<const float*>(row)[c];
  else return __builtin_bit_cast(float, static_cast<uint32_t>(static_cast<const uint16_t*>(row)[c]) << 16);
}
template <int ES>
__device__ __forceinline__ void st_elem(void* row, int c, float x) {
  if constexpr (ES == 4) {
    static_cast<float*>(row)[c] = x;
  } else {
    static_cast<__bf16*>(row)[c] = static_cast<__bf16>(x);
  }
}

// NV > 0: at most 64 NV classes; a lane keeps its NV elements of each of the wavefront's
// rows in registers, and the rows of all kRowsPerWave nodes are requested before the first
// is used. NV = 0: any number of classes, the row is re-read for each of the three sweeps.
template <int ES, int NV>
__global__ __launch_bounds__(256) void xent_grad_kernel(const unsigned char* __restrict__ HL,
                                                        int64_t ld_hl, int64_t n, int32_t C,
                                                        const int32_t* __restrict__ y,
                                                        unsigned char* __restrict__ dH,
                                                        int64_t ld_dh,
                                                        float* __restrict__ block_loss) {
  __shared__ float wave_loss[4];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const float inv_n = 1.0f / static_cast<float>(n);
  const int64_t first0 = (static_cast<int64_t>(blockIdx.x) * 4 + wave) * kRowsPerWave * kRounds;
  float nll = 0.f;
  if constexpr (NV > 0) {
    for (int rd = 0; rd < kRounds; ++rd) {
      const int64_t first = first0 + rd * kRowsPerWave;
      if (first >= n) break;
      // every load of the batch is requested before anything is looked at (a bf16 element is
      // widened only in the second loop)
      typedef typename std::conditional<ES == 4, float, uint16_t>::type RawT;
      RawT raw[kRowsPerWave][NV];
      int32_t label[kRowsPerWave];
#pragma unroll
      for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int64_t row = first + rr < n ? first + rr : n - 1;   // past the end: the last row again
        const RawT* h = reinterpret_cast<const RawT*>(HL + row * ld_hl * ES);
        label[rr] = y[row];
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          const int c = lane + kWave * k;
          raw[rr][k] = h[c < C ? c : 0];      // lanes past the last class: discarded below
        }
      }
#pragma unroll
      for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int64_t row = first + rr;
        if (row >= n) break;
        const int32_t lab = label[rr];
        float v[NV], own = 0.f;               // own: the logit of the label, on the lane that holds it
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          const int c = lane + kWave * k;
          if constexpr (ES == 4) v[k] = raw[rr][k];
          else v[k] = __builtin_bit_cast(float, static_cast<uint32_t>(raw[rr][k]) << 16);
          if (c == lab) own = v[k];
          if (c >= C) v[k] = -INFINITY;
        }
        float mx = v[0];
#pragma unroll
        for (int k = 1; k < NV; ++k) mx = fmaxf(mx, v[k]);
        mx = wave_max(mx);
        float p[NV], se = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          p[k] = __expf(v[k] - mx);      // exp(-inf) = 0 for the lanes past the last class
          se += p[k];
        }
        se = wave_sum(se);
        const float inv_se = 1.0f / se;
        unsigned char* g = dH + row * ld_dh * ES;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          const int c = lane + kWave * k;
          if (c < C) st_elem<ES>(g, c, (p[k] * inv_se - (c == lab ? 1.f : 0.f)) * inv_n);
        }
        if (lab >= 0 && lab < C) {
          // the label is the same on every lane: its logit is read from the lane that holds it
          nll += logf(se) + mx - __shfl(own, lab & (kWave - 1));
        }
      }
    }
  } else {
    for (int rr = 0; rr < kRowsPerWave * kRounds; ++rr) {
      const int64_t row = first0 + rr;
      if (row >= n) break;
      const unsigned char* h = HL + row * ld_hl * ES;
      float mx = -INFINITY;
      for (int c = lane; c < C; c += kWave) mx = fmaxf(mx, ld_elem<ES>(h, c));
      mx = wave_max(mx);
      float se = 0.f;
      for (int c = lane; c < C; c += kWave) se += __expf(ld_elem<ES>(h, c) - mx);
      se = wave_sum(se);
      const int32_t label = y[row];
      unsigned char* g = dH + row * ld_dh * ES;
      for (int c = lane; c < C; c += kWave) {
        const float p = __expf(ld_elem<ES>(h, c) - mx) / se;
        st_elem<ES>(g, c, (p - (c == label ? 1.f : 0.f)) * inv_n);
      }
      if (label >= 0 && label < C) nll += logf(se) + mx - ld_elem<ES>(h, label);
    }
  }
  if (block_loss) {
    if (lane == 0) wave_loss[wave] = nll;
    __syncthreads();
    if (threadIdx.x == 0)
      block_loss[blockIdx.x] = (wave_loss[0] + wave_loss[1]) + (wave_loss[2] + wave_loss[3]);
  }
}

// Rows that start on 16-byte boundaries (ld a multiple of 16 / ES elements): a lane holds NQ
// groups of 4 consecutive classes (classes 4 (lane + 64 q) .. + 3), read and written with one
// 8- or 16-byte access each; at most 256 NQ classes.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef float f32x2v __attribute__((ext_vector_type(2)));

// four elements as loaded (nothing may look at them before all rows of a batch have been
// requested, or every load is waited for on its own), and widened to fp32
template <int ES>
struct RawQuad {
  typedef f32x4 T;
};
template <>
struct RawQuad<2> {
  typedef u32x2 T;
};
template <int ES>
__device__ __forceinline__ f32x4 widen_quad(typename RawQuad<ES>::T w) {
  if constexpr (ES == 4) {
    return w;
  } else {
    const uint32_t w0 = w.x, w1 = w.y;
    f32x4 r;
    r.x = __builtin_bit_cast(float, w0 << 16);
    r.y = __builtin_bit_cast(float, w0 & 0xffff0000u);
    r.z = __builtin_bit_cast(float, w1 << 16);
    r.w = __builtin_bit_cast(float, w1 & 0xffff0000u);
    return r;
  }
}
template <int ES>
__device__ __forceinline__ void st_quad(unsigned char* p, f32x4 v) {
  if constexpr (ES == 4) {
    *reinterpret_cast<f32x4*>(p) = v;
  } else {
    const f32x2v lo = {v.x, v.y}, hi = {v.z, v.w};
    u32x2 w;
    w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2v));
    w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2v));
    *reinterpret_cast<u32x2*>(p) = w;
  }
}

template <int ES, int NQ>
__global__ __launch_bounds__(256) void xent_grad_quad_kernel(const unsigned char* __restrict__ HL,
                                                             int64_t ld_hl, int64_t n, int32_t C,
                                                             const int32_t* __restrict__ y,
                                                             unsigned char* __restrict__ dH,
                                                             int64_t ld_dh,
                                                             float* __restrict__ block_loss) {
  __shared__ float wave_loss[4];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const float inv_n = 1.0f / static_cast<float>(n);
  const int64_t first0 = (static_cast<int64_t>(blockIdx.x) * 4 + wave) * kRowsPerWave * kRounds;
  float nll = 0.f;
  for (int rd = 0; rd < kRounds; ++rd) {
    const int64_t first = first0 + rd * kRowsPerWave;
    if (first >= n) break;
    // every load of the batch is requested before anything is looked at
    typename RawQuad<ES>::T raw[kRowsPerWave][NQ];
    int32_t label[kRowsPerWave];
#pragma unroll
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
      const int64_t row = first + rr < n ? first + rr : n - 1;   // past the end: the last row again
      const unsigned char* h = HL + row * ld_hl * ES;
      label[rr] = y[row];
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        // lanes past the last class re-read the row's first group; it is discarded below
        const int c0 = 4 * (lane + kWave * q);
        raw[rr][q] = *reinterpret_cast<const typename RawQuad<ES>::T*>(
            h + static_cast<int64_t>(c0 < C ? c0 : 0) * ES);
      }
    }
#pragma unroll
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
      const int64_t row = first + rr;
      if (row >= n) break;
      const int32_t lab = label[rr];
      float mx = -INFINITY, own = 0.f;     // own: the logit of the label, on the lane that holds it
      f32x4 v[NQ];
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int c0 = 4 * (lane + kWave * q);
        v[q] = widen_quad<ES>(raw[rr][q]);
        if (c0 == (lab & ~3)) {
          const int j = lab & 3;
          own = j == 0 ? v[q].x : (j == 1 ? v[q].y : (j == 2 ? v[q].z : v[q].w));
        }
        // classes past C (inside the last group: padding of the row) do not take part
        if (c0 >= C) v[q].x = -INFINITY;
        if (c0 + 1 >= C) v[q].y = -INFINITY;
        if (c0 + 2 >= C) v[q].z = -INFINITY;
        if (c0 + 3 >= C) v[q].w = -INFINITY;
        mx = fmaxf(fmaxf(mx, fmaxf(v[q].x, v[q].y)), fmaxf(v[q].z, v[q].w));
      }
      mx = wave_max(mx);
      f32x4 p[NQ];
      float se = 0.f;
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        p[q].x = __expf(v[q].x - mx);
        p[q].y = __expf(v[q].y - mx);
        p[q].z = __expf(v[q].z - mx);
        p[q].w = __expf(v[q].w - mx);
        se += (p[q].x + p[q].y) + (p[q].z + p[q].w);
      }
      se = wave_sum(se);
      const float inv_se = 1.0f / se;
      unsigned char* g = dH + row * ld_dh * ES;
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int c0 = 4 * (lane + kWave * q);
        if (c0 >= C) continue;
        f32x4 o;
        o.x = (p[q].x * inv_se - (c0 == lab ? 1.f : 0.f)) * inv_n;
        o.y = (p[q].y * inv_se - (c0 + 1 == lab ? 1.f : 0.f)) * inv_n;
        o.z = (p[q].z * inv_se - (c0 + 2 == lab ? 1.f : 0.f)) * inv_n;
        o.w = (p[q].w * inv_se - (c0 + 3 == lab ? 1.f : 0.f)) * inv_n;
        if (c0 + 3 < C) {
          st_quad<ES>(g + static_cast<int64_t>(c0) * ES, o);
        } else {
          st_elem<ES>(g, c0, o.x);
          if (c0 + 1 < C) st_elem<ES>(g, c0 + 1, o.y);
          if (c0 + 2 < C) st_elem<ES>(g, c0 + 2, o.z);
        }
      }
      if (lab >= 0 && lab < C) {
        // the label is the same on every lane: its logit is read from the lane that holds it
        const float at_label = __shfl(own, (lab >> 2) & (kWave - 1));
        nll += logf(se) + mx - at_label;
      }
    }
  }
  if (block_loss) {
    if (lane == 0) wave_loss[wave] = nll;
    __syncthreads();
    if (threadIdx.x == 0)
      block_loss[blockIdx.x] = (wave_loss[0] + wave_loss[1]) + (wave_loss[2] + wave_loss[3]);
  }
}

// Single block: loss = (sum of m partials, fixed strided order + tree) / n.
__global__ __launch_bounds__(256) void loss_finish_kernel(const float* __restrict__ part,
                                                          int64_t m, int64_t n,
                                                          float* __restrict__ loss) {
  __shared__ float sh[256];
  float s = 0.f;
  for (int64_t i = threadIdx.x; i < m; i += 256) s += part[i];
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (static_cast<int>(threadIdx.x) < w) sh[threadIdx.x] += sh[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = sh[0] / static_cast<float>(n);
}

}  // namespace

extern "C" int64_t sat_loss_workspace_bytes(int64_t n) {
  if (n <= 0) return 0;
  return ((n + kRowsPerBlock - 1) / kRowsPerBlock) * static_cast<int64_t>(sizeof(float));
}

namespace {

// Argument checks shared by the two entry points (everything but the scratch).
sat_status loss_grad_check(const void* HL, int64_t ld_hl, int64_t n, int32_t n_classes,
                           const int32_t* y, int32_t dtype, const void* dH, int64_t ld_dh) {
  if (n < 0 || n_classes <= 0) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  if (n == 0) return SAT_OK;
  if (!HL || !y || !dH || ld_hl < n_classes || ld_dh < n_classes) return SAT_EINVAL;
  if ((n + kRowsPerBlock - 1) / kRowsPerBlock > INT32_MAX) return SAT_EUNSUPPORTED;
  return SAT_OK;
}

// Enqueues the kernels. partials: device floats, one per block, every one of them written by
// the first kernel before the second reads it (nothing has to be cleared); only used when
// loss != NULL. Arguments have been checked and n > 0.
sat_status loss_grad_launch(const void* HL, int64_t ld_hl, int64_t n, int32_t n_classes,
                            const int32_t* y, int32_t dtype, void* dH, int64_t ld_dh, float* loss,
                            float* partials, void* stream) {
  const int64_t blocks = (n + kRowsPerBlock - 1) / kRowsPerBlock;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned char* hl = static_cast<const unsigned char*>(HL);
  unsigned char* dh = static_cast<unsigned char*>(dH);
  float* bl = loss ? partials : nullptr;
  const dim3 grid(static_cast<unsigned>(blocks)), block(256);
  const int es_b = dtype == SAT_BF16 ? 2 : 4;
  // (with few classes the groups of 4 would leave most lanes idle: one class per lane then)
  const bool quads = n_classes >= 2 * kWave && n_classes <= 16 * kWave && (ld_hl * es_b) % 16 == 0 && (ld_dh * es_b) % 16 == 0 &&
                     sat::aligned16(HL) && sat::aligned16(dH);
  if (quads) {   // the library's own buffers: rows start on 16-byte boundaries
    const int nq = (n_classes + 4 * kWave - 1) / (4 * kWave);
#define SAT_XENT_Q(ES, NQ) \
  xent_grad_quad_kernel<ES, NQ><<<grid, block, 0, s>>>(hl, ld_hl, n, n_classes, y, dh, ld_dh, bl)
    if (dtype == SAT_BF16) {
      switch (nq) {
        case 1: SAT_XENT_Q(2, 1); break;
        case 2: SAT_XENT_Q(2, 2); break;
        case 3: SAT_XENT_Q(2, 3); break;
        default: SAT_XENT_Q(2, 4); break;
      }
    } else {
      switch (nq) {
        case 1: SAT_XENT_Q(4, 1); break;
        case 2: SAT_XENT_Q(4, 2); break;
        case 3: SAT_XENT_Q(4, 3); break;
        default: SAT_XENT_Q(4, 4); break;
      }
    }
#undef SAT_XENT_Q
    sat_status stq = sat::check_launch();
    if (stq != SAT_OK || !loss) return stq;
    loss_finish_kernel<<<dim3(1), dim3(256), 0, s>>>(bl, blocks, n, loss);
    return sat::check_launch();
  }
  const int nv = n_classes <= 4 * kWave ? (n_classes + kWave - 1) / kWave : 0;
#define SAT_XENT(ES, NV) xent_grad_kernel<ES, NV><<<grid, block, 0, s>>>(hl, ld_hl, n, n_classes, y, dh, ld_dh, bl)
  if (dtype == SAT_BF16) {
    switch (nv) {
      case 1: SAT_XENT(2, 1); break;
      case 2: SAT_XENT(2, 2); break;
      case 3: SAT_XENT(2, 3); break;
      case 4: SAT_XENT(2, 4); break;
      default: SAT_XENT(2, 0); break;
    }
  } else {
    switch (nv) {
      case 1: SAT_XENT(4, 1); break;
      case 2: SAT_XENT(4, 2); break;
      case 3: SAT_XENT(4, 3); break;
      case 4: SAT_XENT(4, 4); break;
      default: SAT_XENT(4, 0); break;
    }
  }
#undef SAT_XENT
  sat_status st = sat::check_launch();
  if (st != SAT_OK || !loss) return st;
  loss_finish_kernel<<<dim3(1), dim3(256), 0, s>>>(bl, blocks, n, loss);
  return sat::check_launch();
}

}  // namespace

extern "C" sat_status sat_loss_grad(const void* HL, int64_t ld_hl, int64_t n, int32_t n_classes,
                                    const int32_t* y, int32_t dtype, void* dH, int64_t ld_dh,
                                    float* loss, void* workspace, int64_t workspace_bytes,
                                    void* stream) {
  const sat_status st = loss_grad_check(HL, ld_hl, n, n_classes, y, dtype, dH, ld_dh);
  if (st != SAT_OK || n == 0) return st;
  if (loss && (!workspace || workspace_bytes < sat_loss_workspace_bytes(n))) return SAT_EWORKSPACE;
  return loss_grad_launch(HL, ld_hl, n, n_classes, y, dtype, dH, ld_dh, loss,
                          static_cast<float*>(workspace), stream);
}

// ---- the same call for callers that cannot allocate: the per-block partial sums of the loss
// live in a file-scope device array instead of a caller's workspace.
namespace {

constexpr int64_t kStaticPartials = 262144;          // floats: 1 MiB per GPU the library runs on
constexpr int kMaxDevices = 64;
__device__ __align__(256) float scratch[kStaticPartials];

// Device address of `scratch` on each GPU (every GPU holds its own copy of the array at its
// own address). In host code the array's name is not that address: it is looked up once per
// device with that device current, and only the looked-up pointer is handed to kernels.
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

sat_status static_partials(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    sat::set_last_hip_error(e);
    return SAT_EHIP;
  }
  if (dev < 0 || dev >= kMaxDevices) return SAT_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      sat::set_last_hip_error(e);
      return SAT_EHIP;
    }
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return SAT_OK;
}

}  // namespace

extern "C" int64_t sat_loss_grad_static_max_rows(void) { return kStaticPartials * kRowsPerBlock; }

extern "C" sat_status sat_loss_grad_static(const void* HL, int64_t ld_hl, int64_t n,
                                           int32_t n_classes, const int32_t* y, int32_t dtype,
                                           void* dH, int64_t ld_dh, float* loss, void* stream) {
  const sat_status st = loss_grad_check(HL, ld_hl, n, n_classes, y, dtype, dH, ld_dh);
  if (st != SAT_OK || n == 0) return st;
  if (n > sat_loss_grad_static_max_rows()) return SAT_EUNSUPPORTED;
  float* partials = nullptr;
  if (loss) {
    const sat_status sp = static_partials(&partials);
    if (sp != SAT_OK) return sp;
  }
  return loss_grad_launch(HL, ld_hl, n, n_classes, y, dtype, dH, ld_dh, loss, partials, stream);
}
