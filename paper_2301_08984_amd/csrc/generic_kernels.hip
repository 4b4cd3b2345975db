// Plain (non-MFMA) attention kernels: fp32 arithmetic on the vector ALUs, one
// wavefront per row of the score matrix.  They cover every dtype / head size /
// bias / mask combination the C ABI accepts (D <= 256) and are the kernels used
// for fp32 tensors, where products must not be rounded to bf16.
#include "kparams.h"

namespace ssa {
namespace {

constexpr int WAVES = 4;       // wavefronts per work-group, one score row each
constexpr int TILE = 256;      // score-row elements handled per step (4 per lane)
constexpr int MAXD = 256;

struct bf16_t { uint16_t u; };

__device__ inline float ldf(const float* p) { return *p; }
__device__ inline float ldf(const bf16_t* p) { return __uint_as_float(((uint32_t)p->u) << 16); }
__device__ inline float rnd(float v, const float*) { return v; }
__device__ inline float rnd(float v, const bf16_t*) {  // value after rounding to bf16 (nearest even)
  uint32_t u = __float_as_uint(v);
  u += 0x7fffu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xffff0000u);
}
__device__ inline void stf(float* p, float v) { *p = v; }
__device__ inline void stf(bf16_t* p, float v) { p->u = (uint16_t)(__float_as_uint(rnd(v, p)) >> 16); }

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__device__ inline const T* act(const void* base, const KP& p, int b, int s, int h) {
  return (const T*)base + (int64_t)b * p.sb + (int64_t)s * p.ss + (int64_t)h * p.sh;
}
template <typename T>
__device__ inline T* actw(void* base, const KP& p, int b, int s, int h) {
  return (T*)base + (int64_t)b * p.sb + (int64_t)s * p.ss + (int64_t)h * p.sh;
}
template <typename T>
__device__ inline const T* dorow(const KP& p, int b, int s, int h) {
  return (const T*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)s * p.do_ss + (int64_t)(h - p.do_h0) * p.do_sh;
}

__device__ inline bool is_masked(const KP& p, int b, int i, int j) {
  if (p.mask_kind == 1) return j > i;
  if (p.mask_kind == 2) {
    const int32_t* r = p.region + (int64_t)(b % p.mask_period) * p.S;
    return r[i] != r[j];
  }
  return false;
}
__device__ inline float bias_at(const KP& p, int h, int i, int j) {
  if (p.bias_kind == 0) return 0.f;
  int64_t off;
  if (p.bias_kind == 1) {
    off = ((int64_t)h * p.S + i) * p.S + j;
  } else {
    int yi = i / p.win_w, xi = i - yi * p.win_w, yj = j / p.win_w, xj = j - yj * p.win_w;
    int r = (yi - yj + p.win_h - 1) * (2 * p.win_w - 1) + (xi - xj + p.win_w - 1);
    off = (int64_t)h * ((2 * p.win_h - 1) * (2 * p.win_w - 1)) + r;
  }
  return p.bias_bf16 ? ldf((const bf16_t*)p.bias + off) : ((const float*)p.bias)[off];
}

template <typename T>
__device__ inline float dot_lds(const float* a, const T* g, int D) {
  float acc = 0.f;
#pragma unroll 4
  for (int d = 0; d < D; ++d) acc = fmaf(a[d], ldf(g + d), acc);
  return acc;
}

// ---------------------------------------------------------------------------
// forward / recompute: one wavefront per query row i
// ---------------------------------------------------------------------------
template <typename T, bool RECOMP>
__global__ __launch_bounds__(WAVES * 64) void generic_fwd_kernel(KP p) {
  __shared__ float qrow[WAVES][MAXD];
  __shared__ float pbuf[WAVES][TILE];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int iraw = blockIdx.x * WAVES + w;
  const bool live = iraw < p.S;
  const int i = live ? iraw : p.S - 1;
  const int h = p.h0 + blockIdx.y, b = p.b0 + blockIdx.z;
  const T* q = act<T>(p.Q, p, b, i, h);
  for (int d = lane; d < p.D; d += 64) qrow[w][d] = ldf(q + d);
  __syncthreads();
  float m = -INFINITY, l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 < p.S; j0 += TILE) {
    float s[4], tmax = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int j = j0 + lane + 64 * t;
      s[t] = -INFINITY;
      if (j < p.S && !is_masked(p, b, i, j))
        s[t] = p.scale * dot_lds(qrow[w], act<T>(p.K, p, b, j, h), p.D) + bias_at(p, h, i, j);
      tmax = fmaxf(tmax, s[t]);
    }
    tmax = wave_max(tmax);
    const float mn = fmaxf(m, tmax);
    const float alpha = (mn == -INFINITY) ? 1.f : expf(m - mn);
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float e = (s[t] == -INFINITY) ? 0.f : expf(s[t] - mn);
      pbuf[w][lane + 64 * t] = e;
      psum += e;
    }
    l = l * alpha + wave_sum(psum);
    m = mn;
    __syncthreads();
    const int jn = min(TILE, p.S - j0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < p.D) {
        float acc = o[t] * alpha;
        const T* v = act<T>(p.V, p, b, j0, h) + d;
        for (int jj = 0; jj < jn; ++jj) acc = fmaf(pbuf[w][jj], ldf(v + (int64_t)jj * p.ss), acc);
        o[t] = acc;
      }
    }
    __syncthreads();
  }
  const float inv = 1.f / l;
  const float lse = m + logf(l);
  if (!RECOMP) {
    if (live) {
      T* y = actw<T>(p.Y, p, b, i, h);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int d = lane + 64 * t;
        if (d < p.D) {
          float v = o[t] * inv;
          if (p.gated) v *= 1.f / (1.f + expf(-ldf(act<T>(p.G, p, b, i, h) + d)));
          stf(y + d, v);
        }
      }
      if (p.lse_out && lane == 0) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + i] = lse;
    }
  } else {
    float part = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < p.D) {
        const float ov = o[t] * inv;
        float go = ldf(act<T>(p.dY, p, b, i, h) + d);
        if (p.gated) {
          const float g = 1.f / (1.f + expf(-ldf(act<T>(p.G, p, b, i, h) + d)));
          if (live) stf(actw<T>(p.dG, p, b, i, h) + d, go * ov * g * (1.f - g));
          go = rnd(go * g, (const T*)nullptr);
          if (live)
            stf((T*)p.dO_out + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)i * p.do_ss + (int64_t)(h - p.do_h0) * p.do_sh + d, go);
        }
        part = fmaf(go, ov, part);
      }
    }
    part = wave_sum(part);
    if (live && lane == 0) {
      p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + i] = part;
      if (p.lse_out) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + i] = lse;
    }
  }
}

// ---------------------------------------------------------------------------
// dQ: one wavefront per query row i
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(WAVES * 64) void generic_dq_kernel(KP p) {
  __shared__ float qrow[WAVES][MAXD];
  __shared__ float grow[WAVES][MAXD];
  __shared__ float dsbuf[WAVES][TILE];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int iraw = blockIdx.x * WAVES + w;
  const bool live = iraw < p.S;
  const int i = live ? iraw : p.S - 1;
  const int h = p.h0 + blockIdx.y, b = p.b0 + blockIdx.z;
  const T* q = act<T>(p.Q, p, b, i, h);
  const T* go = dorow<T>(p, b, i, h);
  for (int d = lane; d < p.D; d += 64) { qrow[w][d] = ldf(q + d); grow[w][d] = ldf(go + d); }
  __syncthreads();
  const float lse = p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + i];
  const float delta = p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + i];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 < p.S; j0 += TILE) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int j = j0 + lane + 64 * t;
      float ds = 0.f;
      if (j < p.S && !is_masked(p, b, i, j)) {
        const float s = p.scale * dot_lds(qrow[w], act<T>(p.K, p, b, j, h), p.D) + bias_at(p, h, i, j);
        const float pr = expf(s - lse);
        const float dp = dot_lds(grow[w], act<T>(p.V, p, b, j, h), p.D);
        ds = pr * (dp - delta);
      }
      dsbuf[w][lane + 64 * t] = ds;
    }
    __syncthreads();
    const int jn = min(TILE, p.S - j0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < p.D) {
        float a = acc[t];
        const T* kk = act<T>(p.K, p, b, j0, h) + d;
        for (int jj = 0; jj < jn; ++jj) a = fmaf(dsbuf[w][jj], ldf(kk + (int64_t)jj * p.ss), a);
        acc[t] = a;
      }
    }
    __syncthreads();
  }
  if (live) {
    T* out = actw<T>(p.dQ, p, b, i, h);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < p.D) stf(out + d, p.scale * acc[t]);
    }
  }
}

// ---------------------------------------------------------------------------
// dK, dV: one wavefront per key row j
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(WAVES * 64) void generic_dkdv_kernel(KP p) {
  __shared__ float krow[WAVES][MAXD];
  __shared__ float vrow[WAVES][MAXD];
  __shared__ float pbuf[WAVES][TILE];
  __shared__ float dsbuf[WAVES][TILE];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int jraw = blockIdx.x * WAVES + w;
  const bool live = jraw < p.S;
  const int j = live ? jraw : p.S - 1;
  const int h = p.h0 + blockIdx.y, b = p.b0 + blockIdx.z;
  const T* kk = act<T>(p.K, p, b, j, h);
  const T* vv = act<T>(p.V, p, b, j, h);
  for (int d = lane; d < p.D; d += 64) { krow[w][d] = ldf(kk + d); vrow[w][d] = ldf(vv + d); }
  __syncthreads();
  float dk[4] = {0.f, 0.f, 0.f, 0.f}, dv[4] = {0.f, 0.f, 0.f, 0.f};
  for (int i0 = 0; i0 < p.S; i0 += TILE) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int i = i0 + lane + 64 * t;
      float pr = 0.f, ds = 0.f;
      if (i < p.S && !is_masked(p, b, i, j)) {
        const float s = p.scale * dot_lds(krow[w], act<T>(p.Q, p, b, i, h), p.D) + bias_at(p, h, i, j);
        pr = expf(s - p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + i]);
        const float dp = dot_lds(vrow[w], dorow<T>(p, b, i, h), p.D);
        ds = pr * (dp - p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + i]);
      }
      pbuf[w][lane + 64 * t] = pr;
      dsbuf[w][lane + 64 * t] = ds;
    }
    __syncthreads();
    const int in = min(TILE, p.S - i0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < p.D) {
        float a = dv[t], c = dk[t];
        const T* go = dorow<T>(p, b, i0, h) + d;
        const T* q = act<T>(p.Q, p, b, i0, h) + d;
        for (int ii = 0; ii < in; ++ii) {
          a = fmaf(pbuf[w][ii], ldf(go + (int64_t)ii * p.do_ss), a);
          c = fmaf(dsbuf[w][ii], ldf(q + (int64_t)ii * p.ss), c);
        }
        dv[t] = a;
        dk[t] = c;
      }
    }
    __syncthreads();
  }
  if (live) {
    T* ok = actw<T>(p.dK, p, b, j, h);
    T* ov = actw<T>(p.dV, p, b, j, h);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < p.D) { stf(ok + d, p.scale * dk[t]); stf(ov + d, dv[t]); }
    }
  }
}

// ---------------------------------------------------------------------------
// dense bias gradient: thread (h,i,j) sums dS over the chunk's rows b in order,
// continuing from the value already stored when this is not the first chunk
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void generic_dbias_kernel(KP p) {
  __shared__ float qrow[MAXD];
  __shared__ float grow[MAXD];
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int i = blockIdx.y;
  const int h = p.h0 + blockIdx.z;
  const bool live = j < p.S;
  const int jc = live ? j : p.S - 1;
  float* dst = p.dbias_acc + ((int64_t)h * p.S + i) * p.S + jc;
  float acc = (p.dbias_accumulate && live) ? *dst : 0.f;
  const float bias = bias_at(p, h, i, jc);
  for (int b = p.b0; b < p.b1; ++b) {
    __syncthreads();
    const T* q = act<T>(p.Q, p, b, i, h);
    const T* go = dorow<T>(p, b, i, h);
    for (int d = threadIdx.x; d < p.D; d += 256) { qrow[d] = ldf(q + d); grow[d] = ldf(go + d); }
    __syncthreads();
    if (!is_masked(p, b, i, jc)) {
      const float s = p.scale * dot_lds(qrow, act<T>(p.K, p, b, jc, h), p.D) + bias;
      const float pr = expf(s - p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + i]);
      const float dp = dot_lds(grow, act<T>(p.V, p, b, jc, h), p.D);
      acc += pr * (dp - p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + i]);
    }
  }
  if (live) *dst = acc;
}

// table[h][r] = sum of dense[h][i][j] over the (i, j) pairs of the window whose relative position is
// r.  One wavefront per table entry: lane l takes the pairs l, l + 64, ... (numbered in (y, x) order
// of the query) and the lanes are summed with a fixed butterfly, so the result does not depend on
// anything but the values.
__global__ __launch_bounds__(256) void relpos_reduce_kernel(const float* dense, float* table, int h0,
                                                            int nh, int S, int win_h, int win_w) {
  const int R = (2 * win_h - 1) * (2 * win_w - 1);
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= nh * R) return;  // uniform over the wavefront
  const int h = h0 + t / R, r = t % R;
  const int dy = r / (2 * win_w - 1) - (win_h - 1), dx = r % (2 * win_w - 1) - (win_w - 1);
  // queries (yi, xi) with a partner inside the window: yi in [ylo, yhi), xi in [xlo, xhi)
  const int ylo = max(dy, 0), yhi = min(win_h + dy, win_h), xlo = max(dx, 0), xhi = min(win_w + dx, win_w);
  const int nx = xhi - xlo, n = (yhi - ylo) * nx;
  float v = 0.f;
  for (int i = lane; i < n; i += 64) {  // one pass for windows of up to 64 positions
    const int yi = ylo + i / nx, xi = xlo + i % nx;
    v += dense[((int64_t)h * S + (yi * win_w + xi)) * S + ((yi - dy) * win_w + (xi - dx))];
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  if (lane == 0) table[(int64_t)h * R + r] = v;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* p, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t step = (size_t)gridDim.x * 256;
  for (; i < n; i += step) p[i] = 0.f;
}

inline dim3 row_grid(const KP& p) {
  return dim3((p.S + WAVES - 1) / WAVES, p.h1 - p.h0, p.b1 - p.b0);
}

}  // namespace

hipError_t launch_generic_fwd(const KP& p, bool bf16, bool recompute, hipStream_t st) {
  dim3 g = row_grid(p), blk(WAVES * 64);
  if (bf16) {
    if (recompute) generic_fwd_kernel<bf16_t, true><<<g, blk, 0, st>>>(p);
    else generic_fwd_kernel<bf16_t, false><<<g, blk, 0, st>>>(p);
  } else {
    if (recompute) generic_fwd_kernel<float, true><<<g, blk, 0, st>>>(p);
    else generic_fwd_kernel<float, false><<<g, blk, 0, st>>>(p);
  }
  return hipGetLastError();
}
hipError_t launch_generic_dq(const KP& p, bool bf16, hipStream_t st) {
  dim3 g = row_grid(p), blk(WAVES * 64);
  if (bf16) generic_dq_kernel<bf16_t><<<g, blk, 0, st>>>(p);
  else generic_dq_kernel<float><<<g, blk, 0, st>>>(p);
  return hipGetLastError();
}
hipError_t launch_generic_dkdv(const KP& p, bool bf16, hipStream_t st) {
  dim3 g = row_grid(p), blk(WAVES * 64);
  if (bf16) generic_dkdv_kernel<bf16_t><<<g, blk, 0, st>>>(p);
  else generic_dkdv_kernel<float><<<g, blk, 0, st>>>(p);
  return hipGetLastError();
}
hipError_t launch_generic_dbias(const KP& p, bool bf16, hipStream_t st) {
  dim3 g((p.S + 255) / 256, p.S, p.h1 - p.h0), blk(256);
  if (bf16) generic_dbias_kernel<bf16_t><<<g, blk, 0, st>>>(p);
  else generic_dbias_kernel<float><<<g, blk, 0, st>>>(p);
  return hipGetLastError();
}
hipError_t launch_relpos_reduce(const float* dense, float* table, int h0, int h1, int S, int win_h,
                                int win_w, hipStream_t st) {
  const int R = (2 * win_h - 1) * (2 * win_w - 1);
  const int n = (h1 - h0) * R;
  relpos_reduce_kernel<<<(n + 3) / 4, 256, 0, st>>>(dense, table, h0, h1 - h0, S, win_h, win_w);
  return hipGetLastError();
}
hipError_t launch_fill_zero(float* ptr, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  fill_zero_kernel<<<(unsigned)blocks, 256, 0, st>>>(ptr, n);
  return hipGetLastError();
}

}  // namespace ssa
