// HIP kernels for gfx950 (CDNA4, wave64).
//
//  * gemm_mfma: bf16 x bf16 -> fp32 contraction on v_mfma_f32_32x32x16_bf16 with runtime M/N/K,
//    two-level batch strides, LDS double buffering and a fused epilogue
//    (scale, bias, activation, residual, activation, strided store).  The A operand comes from a
//    loader object: a strided matrix (MatMul) or an NHWC im2col address generator (Conv), so the
//    convolution is an implicit GEMM on the same main loop.  Tile shape is a template parameter
//    over a small fixed set (the fat / regular / skinny versions of Section 4.4.2); nothing is
//    compiled per shape.
//  * gemm_simple: any dtype, any strides, plain FMA tiles (fp32 graphs, odd layouts).
//  * conv_stem_kernel: convolutions with fewer than 8 input channels and 64 output channels.
//  * gemv_f32_kernel: fp32 contractions with at most 8 rows (the gate networks).
//  * row kernels: LayerNorm and softmax with one wavefront per row, 16-byte loads, wave shuffles.
//  * reduce_mean (plain and wide), maxpool, elementwise chains (Fig. 4).
//  * gather, cache append, arg-max; NonZero, ScatterRows, wide row gather (batch compaction);
//    nearest-neighbour Resize and Concat along the last dim.
// The direct-to-LDS contraction, its split-K pass and the skinny bf16 kernels are in gemm.hip, the
// fused attention kernels in attention.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "device_common.hpp"
#define SOD2_BF16_TAG 1

namespace sod2 {

// ---------------------------------------------------------------------------------------------
// A-operand loaders: 8 consecutive k of one row, zero outside the matrix
// ---------------------------------------------------------------------------------------------
struct MatA {
  const bf16_t* p;
  long long sm, sk;
  int M, K, vec;
  __device__ __forceinline__ void row_setup(int, int&, int&, long long&) const {}
  __device__ __forceinline__ uint4 load(int m, int k) const {
    if (vec) return (m < M && k < K) ? *(const uint4*)(p + (long long)m * sm + k) : zero4();
    V16 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v.h[i] = (m < M && k + i < K) ? p[(long long)m * sm + (long long)(k + i) * sk] : (bf16_t)0;
    return v.u;
  }
};
struct ConvA {                      // x[nb, ih, iw, c], k = (kh * KW + kw) * C + c
  const bf16_t* p;
  int H, W, C, KW, stride, pad, OH, OW, M, K, vec;
  __device__ __forceinline__ uint4 load(int m, int k) const {
    if (m >= M || k >= K) return zero4();
    int ow = m % OW, t = m / OW;
    int oh = t % OH, nb = t / OH;
    int ih0 = oh * stride - pad, iw0 = ow * stride - pad;
    const bf16_t* img = p + (long long)nb * H * W * C;
    if (vec) {
      int c = k % C, kk = k / C;
      int ih = ih0 + kk / KW, iw = iw0 + kk % KW;
      if (ih < 0 || ih >= H || iw < 0 || iw >= W) return zero4();
      return *(const uint4*)(img + ((long long)ih * W + iw) * C + c);
    }
    V16 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int ke = k + i;
      bf16_t x = 0;
      if (ke < K) {
        int c = ke % C, kk = ke / C;
        int ih = ih0 + kk / KW, iw = iw0 + kk % KW;
        if (ih >= 0 && ih < H && iw >= 0 && iw < W) x = img[((long long)ih * W + iw) * C + c];
      }
      v.h[i] = x;
    }
    return v.u;
  }
};

// ---------------------------------------------------------------------------------------------
// MFMA contraction
// ---------------------------------------------------------------------------------------------
template <class AL, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_mfma(AL al, GemmArgs g) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64, LDK = BK + 8, KV = BK / 8;
  constexpr int AV = BM * KV / 256, BV = BN * KV / 256;
  static_assert(WM * WN == 4 && AV >= 1 && BV >= 1, "four waves per workgroup");
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDK];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int tiles_m = (g.M + BM - 1) / BM;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int b0 = blockIdx.y / g.nb1, b1 = blockIdx.y % g.nb1;
  const int m0 = tm * BM, n0 = tn * BN;

  al.p += b0 * g.a_sb0 + b1 * g.a_sb1;
  const bf16_t* Bp = (const bf16_t*)g.B + b0 * g.b_sb0 + b1 * g.b_sb1;

  uint4 ra[AV], rb[BV];
  auto gload = [&](int kt) {
    const int k0 = kt * BK;
#pragma unroll
    for (int i = 0; i < AV; ++i) {
      int v = tid + i * 256;
      ra[i] = al.load(m0 + v / KV, k0 + (v % KV) * 8);
    }
    if (g.b_mode == 0) {
#pragma unroll
      for (int i = 0; i < BV; ++i) {
        int v = tid + i * 256;
        int n = n0 + v / KV, k = k0 + (v % KV) * 8;
        rb[i] = (n < g.N && k < g.K) ? *(const uint4*)(Bp + (long long)n * g.b_sn + k) : zero4();
      }
    } else if (g.b_mode == 1) {
#pragma unroll
      for (int i = 0; i < BV; ++i) {
        int v = tid + i * 256;
        int k = k0 + v / (BN / 8), n = n0 + (v % (BN / 8)) * 8;
        rb[i] = (n < g.N && k < g.K) ? *(const uint4*)(Bp + (long long)k * g.b_sk + n) : zero4();
      }
    } else {
#pragma unroll
      for (int i = 0; i < BV; ++i) {
        int v = tid + i * 256;
        int n = n0 + v / KV, k = k0 + (v % KV) * 8;
        V16 t;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          t.h[e] = (n < g.N && k + e < g.K) ? Bp[(long long)n * g.b_sn + (long long)(k + e) * g.b_sk] : (bf16_t)0;
        rb[i] = t.u;
      }
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < AV; ++i) {
      int v = tid + i * 256;
      *(uint4*)&As[buf][(v / KV) * LDK + (v % KV) * 8] = ra[i];
    }
    if (g.b_mode != 1) {
#pragma unroll
      for (int i = 0; i < BV; ++i) {
        int v = tid + i * 256;
        *(uint4*)&Bs[buf][(v / KV) * LDK + (v % KV) * 8] = rb[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < BV; ++i) {
        int v = tid + i * 256;
        int k = v / (BN / 8), n = (v % (BN / 8)) * 8;
        V16 t;
        t.u = rb[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) Bs[buf][(n + e) * LDK + k] = t.h[e];
      }
    }
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (g.K + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  const int arow = (wm * TM * 32 + (lane & 31)) * LDK + (lane >> 5) * 8;
  const int brow = (wn * TN * 32 + (lane & 31)) * LDK + (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      V16 af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i].u = *(const uint4*)&As[buf][arow + i * 32 * LDK + ks * 16];
#pragma unroll
      for (int j = 0; j < TN; ++j) bf[j].u = *(const uint4*)&Bs[buf][brow + j * 32 * LDK + ks * 16];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i].b, bf[j].b, acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(buf ^ 1);
    __syncthreads();
  }

  // epilogue: lane holds column (lane & 31); rows 8*(r/4) + 4*(lane>>5) + r%4 of each 32x32 tile
  bf16_t* Cp = (bf16_t*)g.C + b0 * g.c_sb0 + b1 * g.c_sb1;
  const bf16_t* Rp = g.res ? (const bf16_t*)g.res + b0 * g.r_sb0 + b1 * g.r_sb1 : nullptr;
  const bf16_t* bias = (const bf16_t*)g.bias;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn * TN * 32 + j * 32 + (lane & 31);
    if (col >= g.N) continue;
    const float bv = bias ? bf2f(bias[col]) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * TM * 32 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (row >= g.M) continue;
        float v = acc[i][j][r] * g.scale + bv;
        v = apply_act(v, g.act1);
        if (Rp) v += bf2f(Rp[(long long)row * g.r_sm + (long long)col * g.r_sn]);
        v = apply_act(v, g.act2);
        Cp[(long long)row * g.c_sm + (long long)col * g.c_sn] = f2bf(v);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Plain FMA contraction for any dtype and any strides
// ---------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void gemm_simple(GemmArgs g) {
  constexpr int BT = 64, BK = 32, PT = BT * BK / 256;   // PT elements of each operand tile per thread
  __shared__ float As[BK][BT + 1];
  __shared__ float Bs[BK][BT + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int tiles_m = (g.M + BT - 1) / BT;
  const int m0 = (blockIdx.x % tiles_m) * BT, n0 = (blockIdx.x / tiles_m) * BT;
  const int b0 = blockIdx.y / g.nb1, b1 = blockIdx.y % g.nb1;
  const T* A = (const T*)g.A + b0 * g.a_sb0 + b1 * g.a_sb1;
  const T* B = (const T*)g.B + b0 * g.b_sb0 + b1 * g.b_sb1;
  float acc[4][4] = {};
  // the next k-tile's 8 elements are requested before the current tile is multiplied (otherwise every
  // k-tile costs a full memory round trip with nothing to hide it)
  float pa[PT], pb[PT];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int e = tid + i * 256;
      const int r = e / BK, k = e % BK;                  // 64 rows x BK k
      const int m = m0 + r, n = n0 + r, kk = k0 + k;
      pa[i] = (m < g.M && kk < g.K) ? to_f<T>(A[(long long)m * g.a_sm + (long long)kk * g.a_sk]) : 0.f;
      pb[i] = (n < g.N && kk < g.K) ? to_f<T>(B[(long long)kk * g.b_sk + (long long)n * g.b_sn]) : 0.f;
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < g.K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int e = tid + i * 256;
      As[e % BK][e / BK] = pa[i];
      Bs[e % BK][e / BK] = pb[i];
    }
    __syncthreads();
    if (k0 + BK < g.K) fetch(k0 + BK);
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  T* C = (T*)g.C + b0 * g.c_sb0 + b1 * g.c_sb1;
  const T* R = g.res ? (const T*)g.res + b0 * g.r_sb0 + b1 * g.r_sb1 : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = m0 + ty * 4 + i;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int col = n0 + tx * 4 + j;
      if (col >= g.N) continue;
      float v = acc[i][j] * g.scale + (g.bias ? to_f<T>(((const T*)g.bias)[col]) : 0.f);
      v = apply_act(v, g.act1);
      if (R) v += to_f<T>(R[(long long)row * g.r_sm + (long long)col * g.r_sn]);
      v = apply_act(v, g.act2);
      C[(long long)row * g.c_sm + (long long)col * g.c_sn] = from_f<T>(v);
    }
  }
}

// direct convolution for any dtype (fp32 graphs): one thread per output element
template <class T>
__global__ void conv_simple(ConvArgs c) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  long long total = (long long)c.NB * c.OH * c.OW * c.O;
  if (idx >= total) return;
  int o = idx % c.O;
  long long m = idx / c.O;
  int ow = m % c.OW;
  long long t = m / c.OW;
  int oh = t % c.OH, nb = t / c.OH;
  const T* x = (const T*)c.x + (long long)nb * c.H * c.W * c.C;
  const T* w = (const T*)c.w + (long long)o * c.KH * c.KW * c.C;
  float acc = 0.f;
  for (int kh = 0; kh < c.KH; ++kh) {
    int ih = oh * c.stride - c.pad + kh;
    if (ih < 0 || ih >= c.H) continue;
    for (int kw = 0; kw < c.KW; ++kw) {
      int iw = ow * c.stride - c.pad + kw;
      if (iw < 0 || iw >= c.W) continue;
      const T* xp = x + ((long long)ih * c.W + iw) * c.C;
      const T* wp = w + (kh * c.KW + kw) * c.C;
      for (int ch = 0; ch < c.C; ++ch) acc = fmaf(to_f<T>(xp[ch]), to_f<T>(wp[ch]), acc);
    }
  }
  float v = acc + (c.bias ? to_f<T>(((const T*)c.bias)[o]) : 0.f);
  v = apply_act(v, c.act1);
  if (c.res) v += to_f<T>(((const T*)c.res)[idx]);
  v = apply_act(v, c.act2);
  ((T*)c.y)[idx] = from_f<T>(v);
}

// ---------------------------------------------------------------------------------------------
// Row kernels: one wavefront per row
// ---------------------------------------------------------------------------------------------
template <class T> struct Vec;      // 16-byte vector of T
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const bf16_t* p, float* f) {
    V16 v; v.u = *(const uint4*)p;
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = bf2f(v.h[i]);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* f) {
    V16 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v.h[i] = f2bf(f[i]);
    *(uint4*)p = v.u;
  }
};
template <> struct Vec<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float* p, float* f) {
    float4 v = *(const float4*)p; f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* f) {
    *(float4*)p = make_float4(f[0], f[1], f[2], f[3]);
  }
};

// MODE 0: LayerNorm (biased variance, two passes over registers); MODE 1: softmax (max-subtracted).
// VEC: rows are 16-byte aligned and cols % Vec::N == 0 and cols <= 64 * Vec::N * MAXV.
template <class T, int MODE, bool VEC>
__global__ __launch_bounds__(256) void row_kernel(RowArgs a) {
  constexpr int VN = Vec<T>::N, MAXV = 4;
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.rows) return;
  const T* x = (const T*)a.x + row * a.x_stride;
  T* y = (T*)a.y + row * a.y_stride;
  int valid = a.cols;                                  // softmax with a causal mask: columns < valid
  if (MODE == 1 && a.causal) {
    int i = (int)(row % a.lq);
    valid = min(a.cols, i + (a.cols - a.lq) + 1);
  }
  if (VEC) {
    float v[MAXV][VN];
    const int nvec = a.cols / VN;
#pragma unroll
    for (int q = 0; q < MAXV; ++q) {
      int vi = lane + q * 64;
      if (vi < nvec) Vec<T>::load(x + vi * VN, v[q]);
    }
    if (MODE == 0) {
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < MAXV; ++q)
        if (lane + q * 64 < nvec)
#pragma unroll
          for (int e = 0; e < VN; ++e) s += v[q][e];
      const float mean = wave_sum(s) / a.cols;
      float ss = 0.f;
#pragma unroll
      for (int q = 0; q < MAXV; ++q)
        if (lane + q * 64 < nvec)
#pragma unroll
          for (int e = 0; e < VN; ++e) { float d = v[q][e] - mean; ss += d * d; }
      const float rstd = rsqrtf(wave_sum(ss) / a.cols + a.eps);
#pragma unroll
      for (int q = 0; q < MAXV; ++q) {
        int vi = lane + q * 64;
        if (vi < nvec) {
          float gm[VN], bt[VN], o[VN];
          Vec<T>::load((const T*)a.gamma + vi * VN, gm);
          Vec<T>::load((const T*)a.beta + vi * VN, bt);
#pragma unroll
          for (int e = 0; e < VN; ++e) o[e] = (v[q][e] - mean) * rstd * gm[e] + bt[e];
          Vec<T>::store(y + vi * VN, o);
        }
      }
    } else {
      float mx = -INFINITY;
#pragma unroll
      for (int q = 0; q < MAXV; ++q)
        if (lane + q * 64 < nvec)
#pragma unroll
          for (int e = 0; e < VN; ++e)
            if ((lane + q * 64) * VN + e < valid) mx = fmaxf(mx, v[q][e]);
      mx = wave_max(mx);
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < MAXV; ++q)
        if (lane + q * 64 < nvec)
#pragma unroll
          for (int e = 0; e < VN; ++e) {
            float p = ((lane + q * 64) * VN + e < valid) ? __expf(v[q][e] - mx) : 0.f;
            v[q][e] = p;
            s += p;
          }
      const float inv = 1.f / wave_sum(s);
#pragma unroll
      for (int q = 0; q < MAXV; ++q) {
        int vi = lane + q * 64;
        if (vi < nvec) {
          float o[VN];
#pragma unroll
          for (int e = 0; e < VN; ++e) o[e] = v[q][e] * inv;
          Vec<T>::store(y + vi * VN, o);
        }
      }
    }
  } else {
    if (MODE == 0) {
      float s = 0.f;
      for (int c = lane; c < a.cols; c += 64) s += to_f<T>(x[c]);
      const float mean = wave_sum(s) / a.cols;
      float ss = 0.f;
      for (int c = lane; c < a.cols; c += 64) { float d = to_f<T>(x[c]) - mean; ss += d * d; }
      const float rstd = rsqrtf(wave_sum(ss) / a.cols + a.eps);
      for (int c = lane; c < a.cols; c += 64)
        y[c] = from_f<T>((to_f<T>(x[c]) - mean) * rstd * to_f<T>(((const T*)a.gamma)[c]) + to_f<T>(((const T*)a.beta)[c]));
    } else {
      float mx = -INFINITY;
      for (int c = lane; c < valid; c += 64) mx = fmaxf(mx, to_f<T>(x[c]));
      mx = wave_max(mx);
      float s = 0.f;
      for (int c = lane; c < valid; c += 64) s += __expf(to_f<T>(x[c]) - mx);
      const float inv = 1.f / wave_sum(s);
      for (int c = lane; c < a.cols; c += 64)
        y[c] = from_f<T>(c < valid ? __expf(to_f<T>(x[c]) - mx) * inv : 0.f);
    }
  }
}

// y[b, c] = mean_r x[b, r, c]; 64 columns per workgroup, 4 row groups of 64 lanes... one column per
// lane keeps loads coalesced; rows are split over the 4 waves and combined through LDS.
template <class TI, class TO>
__global__ __launch_bounds__(256) void reduce_mean_kernel(ReduceArgs a) {
  __shared__ float part[4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane, b = blockIdx.y;
  float s = 0.f;
  if (c < a.C) {
    const TI* x = (const TI*)a.x + (long long)b * a.R * a.C + c;
    for (long long r0 = w; r0 < a.R; r0 += 4 * 8) {          // 8 rows in flight per lane, added in row order
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (r0 + 4 * u < a.R) ? to_f<TI>(x[(r0 + 4 * u) * a.C]) : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
  }
  part[w][lane] = s;
  __syncthreads();
  if (w == 0 && c < a.C) {
    float t = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
    ((TO*)a.y)[(long long)b * a.C + c] = from_f<TO>(t / (float)a.R);
  }
}

// The same for bf16 rows with 16 waves splitting the rows.  A lane owns CPL consecutive channels (8: 16-byte loads, a workgroup
// covers 512 channels; 2: 4-byte loads, 128 channels per workgroup, for when 512-channel workgroups
// would be too few to pull the rows through more than a couple of CUs).
template <class TO, int CPL>
__global__ __launch_bounds__(1024) void reduce_mean_bf16_wide_kernel(ReduceArgs a) {
  __shared__ float part[16][64 * CPL];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c0 = (blockIdx.x * 64 + lane) * CPL, b = blockIdx.y;
  float s[CPL];
#pragma unroll
  for (int e = 0; e < CPL; ++e) s[e] = 0.f;
  if (c0 < a.C) {
    const bf16_t* x = (const bf16_t*)a.x + (long long)b * a.R * a.C + c0;
    // 8 rows in flight per lane (a loop over the run-time row count would wait for each load in turn); rows are
    // added in the same order as one by one
    for (long long r0 = w; r0 < a.R; r0 += 16 * 8) {
      if (CPL == 8) {
        V16 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u].u = (r0 + 16 * u < a.R) ? *(const uint4*)(x + (r0 + 16 * u) * a.C) : zero4();
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int e = 0; e < CPL; ++e) s[e] += bf2f(v[u].h[e]);
      } else {
        uint32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (r0 + 16 * u < a.R) ? *(const uint32_t*)(x + (r0 + 16 * u) * a.C) : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          s[0] += __uint_as_float(v[u] << 16);
          s[CPL - 1] += __uint_as_float(v[u] & 0xffff0000u);
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < CPL; ++e) part[w][lane * CPL + e] = s[e];
  __syncthreads();
  const int t = threadIdx.x, c = blockIdx.x * 64 * CPL + t;
  if (t < 64 * CPL && c < a.C) {
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) tot += part[k][t];
    ((TO*)a.y)[(long long)b * a.C + c] = from_f<TO>(tot / (float)a.R);
  }
}

template <class T>
__global__ void maxpool_kernel(PoolArgs p) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  long long total = (long long)p.NB * p.OH * p.OW * p.C;
  if (idx >= total) return;
  int c = idx % p.C;
  long long m = idx / p.C;
  int ow = m % p.OW;
  long long t = m / p.OW;
  int oh = t % p.OH, nb = t / p.OH;
  const T* x = (const T*)p.x + (long long)nb * p.H * p.W * p.C;
  float best = -INFINITY, sum = 0.f;
  int cnt = 0;
  for (int i = 0; i < p.k; ++i) {
    int ih = oh * p.stride - p.pad + i;
    if (ih < 0 || ih >= p.H) continue;
    for (int j = 0; j < p.k; ++j) {
      int iw = ow * p.stride - p.pad + j;
      if (iw < 0 || iw >= p.W) continue;
      const float v = to_f<T>(x[((long long)ih * p.W + iw) * p.C + c]);
      best = fmaxf(best, v);
      sum += v;
      ++cnt;
    }
  }
  ((T*)p.y)[idx] = from_f<T>(p.avg ? sum / (float)cnt : best);      // (pad < k: every window holds an input position)
}

// bf16 with C % 8 == 0 and a K x K window known at compile time: a thread owns 8 consecutive channels of one output
// position; the K * K rows of the window are requested together (16-byte loads) and then compared (AVG: summed in
// window order and divided by the number of positions inside the input).
template <int K, bool AVG>
__global__ __launch_bounds__(256) void maxpool_bf16x8_kernel(PoolArgs p) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const int cv = p.C >> 3;
  const long long total = (long long)p.NB * p.OH * p.OW * cv;
  if (idx >= total) return;
  const int c8 = (int)(idx % cv);
  long long m = idx / cv;
  const int ow = (int)(m % p.OW);
  m /= p.OW;
  const int oh = (int)(m % p.OH), nb = (int)(m / p.OH);
  const bf16_t* x = (const bf16_t*)p.x + (long long)nb * p.H * p.W * p.C + c8 * 8;
  V16 v[K * K];
  bool ok[K * K];
#pragma unroll
  for (int i = 0; i < K; ++i)
#pragma unroll
    for (int j = 0; j < K; ++j) {
      const int ih = oh * p.stride - p.pad + i, iw = ow * p.stride - p.pad + j;
      ok[i * K + j] = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
      v[i * K + j].u = ok[i * K + j] ? *(const uint4*)(x + ((long long)ih * p.W + iw) * p.C) : zero4();
    }
  float best[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = AVG ? 0.f : -INFINITY;
  int cnt = 0;
#pragma unroll
  for (int q = 0; q < K * K; ++q)
    if (ok[q]) {
      ++cnt;
#pragma unroll
      for (int e = 0; e < 8; ++e) best[e] = AVG ? best[e] + bf2f(v[q].h[e]) : fmaxf(best[e], bf2f(v[q].h[e]));
    }
  V16 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o.h[e] = f2bf(AVG ? best[e] / (float)cnt : best[e]);
  *(uint4*)((bf16_t*)p.y + idx * 8) = o.u;
}

template <class TO>
__global__ void eltwise_kernel(EltArgs a) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= a.total) return;
  long long off[5] = {0, 0, 0, 0, 0};
  long long rem = idx;
  for (int d = a.rank - 1; d >= 0; --d) {
    long long i = rem % a.dims[d];
    rem /= a.dims[d];
    for (int k = 0; k < a.n_in; ++k) off[k] += i * a.stride[k][d];
  }
  float in[5];
  for (int k = 0; k < a.n_in; ++k)
    in[k] = a.in_bf16[k] ? bf2f(((const bf16_t*)a.in[k])[off[k]]) : ((const float*)a.in[k])[off[k]];
  float v = in[0];
  for (int o = 0; o < a.n_ops; ++o) {
    float x = a.src[o] == 5 ? a.imm[o] : (a.src[o] >= 0 ? in[a.src[o]] : 0.f);
    switch (a.op[o]) {
      case E_ADD: v += x; break;
      case E_MUL: v *= x; break;
      case E_RELU: v = fmaxf(v, 0.f); break;
      case E_GELU: v = apply_act(v, ACT_GELU); break;
      case E_SIGMOID: v = apply_act(v, ACT_SIGMOID); break;
      case E_ROUND: v = rintf(v); break;                 // halves to the even integer
      case E_CAST_BF16: v = bf2f(f2bf(v)); break;
      default: break;
    }
  }
  ((TO*)a.out)[idx] = from_f<TO>(v);
}

// ---------------------------------------------------------------------------------------------
// Embedding gather (+ add), KV-cache append, arg-max
// ---------------------------------------------------------------------------------------------
template <class T, class I>
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
  const long long r = blockIdx.x;
  const I* idx = (const I*)((const char*)a.idx + (a.step ? *a.step * a.idx_step : 0));
  long long id = (long long)idx[r];
  id = id < 0 ? 0 : (id >= a.table_rows ? a.table_rows - 1 : id);
  const T* src = (const T*)a.table + id * a.cols;
  const T* add = a.add ? (const T*)a.add + r * a.add_stride : nullptr;
  T* dst = (T*)a.y + r * a.cols;
  for (int c = threadIdx.x; c < a.cols; c += 256) {
    float v = to_f<T>(src[c]);
    if (add) v += to_f<T>(add[c]);
    dst[c] = from_f<T>(v);
  }
}

template <class I>
__global__ void gather_rows16_kernel(GatherArgs a, long long row_units);    // wide rows, defined with ScatterRows below

template <class T>
__global__ __launch_bounds__(256) void append_kernel(AppendArgs a) {
  const long long r = blockIdx.x;
  const T* src = (const T*)a.x + r * a.x_stride;
  const long long past = a.past + (a.step ? *a.step * a.past_step : 0);
  T* dst = (T*)a.cache + (past + r) * a.cols;
  for (int c = threadIdx.x; c < a.cols; c += 256) dst[c] = src[c];
}

template <class T>
__global__ __launch_bounds__(256) void argmax_kernel(ArgmaxArgs a) {
  __shared__ float bv[4];
  __shared__ int bi[4];
  const long long r = blockIdx.x;
  const int stp = a.step ? *a.step : 0;
  const T* x = (const T*)((const char*)a.x + stp * a.x_step) + r * a.x_stride;
  float best = -INFINITY;
  int at = 0x7fffffff;
  for (int c = threadIdx.x; c < a.cols; c += 256) {      // ascending c per thread: '>' keeps the lowest index
    float v = to_f<T>(x[c]);
    if (v > best || at == 0x7fffffff) { best = v; at = c; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(best, o, 64);
    int oi = __shfl_xor(at, o, 64);
    if (ov > best || (ov == best && oi < at)) { best = ov; at = oi; }
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) { bv[w] = best; bi[w] = at; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 4; ++k)
      if (bv[k] > best || (bv[k] == best && bi[k] < at)) { best = bv[k]; at = bi[k]; }
    char* y = (char*)a.y + stp * a.y_step;
    if (a.out_i32) ((int*)y)[r] = at;
    else ((long long*)y)[r] = at;
  }
}

// bf16 rows read in 16-byte chunks by 16 waves: every load of a thread is in flight at once for the
// row lengths met here (a vocabulary of 32 000 is 4 chunks per thread)
__global__ __launch_bounds__(1024) void argmax_bf16x8_kernel(ArgmaxArgs a) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  const long long r = blockIdx.x;
  const int stp = a.step ? *a.step : 0;
  const bf16_t* x = (const bf16_t*)((const char*)a.x + stp * a.x_step) + r * a.x_stride;
  float best = -INFINITY;
  int at = 0x7fffffff;
  const int nchunk = a.cols >> 3;
  for (int c = threadIdx.x; c < nchunk; c += 1024) {     // ascending indices per thread: '>' keeps the lowest
    V16 v; v.u = *(const uint4*)(x + c * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float f = bf2f(v.h[e]);
      if (f > best || at == 0x7fffffff) { best = f; at = c * 8 + e; }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(best, o, 64);
    int oi = __shfl_xor(at, o, 64);
    if (ov > best || (ov == best && oi < at)) { best = ov; at = oi; }
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) { bv[w] = best; bi[w] = at; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 16; ++k)
      if (bv[k] > best || (bv[k] == best && bi[k] < at)) { best = bv[k]; at = bi[k]; }
    char* y = (char*)a.y + stp * a.y_step;
    if (a.out_i32) ((int*)y)[r] = at;
    else ((long long*)y)[r] = at;
  }
}

__global__ void step_set_kernel(int* step, int value) { *step = value; }
__global__ void step_advance_kernel(int* step) { *step += 1; }
hipError_t launch_step_set(int* step, int value, hipStream_t s) {
  hipLaunchKernelGGL(step_set_kernel, dim3(1), dim3(1), 0, s, step, value);
  return hipGetLastError();
}
hipError_t launch_step_advance(int* step, hipStream_t s) {
  hipLaunchKernelGGL(step_advance_kernel, dim3(1), dim3(1), 0, s, step);
  return hipGetLastError();
}

hipError_t launch_gather(const Launch& L, const GatherArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  const long long row_bytes = (long long)a.cols * (L.in_dtype == SOD2_BF16_TAG ? 2 : 4);
  if (!a.add && !a.step && row_bytes >= 4096 && row_bytes % 16 == 0 && (((uintptr_t)a.table | (uintptr_t)a.y) & 15) == 0) {
    const long long units = row_bytes / 16;
    dim3 wide((unsigned)std::min<long long>((units + 255) / 256, 64), (unsigned)a.rows);
    if (a.idx_i32) hipLaunchKernelGGL(gather_rows16_kernel<int>, wide, dim3(256), 0, s, a, units);
    else hipLaunchKernelGGL(gather_rows16_kernel<long long>, wide, dim3(256), 0, s, a, units);
    return hipGetLastError();
  }
  dim3 grid((unsigned)a.rows);
  if (L.in_dtype == SOD2_BF16_TAG) {
    if (a.idx_i32) hipLaunchKernelGGL((gather_kernel<bf16_t, int>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((gather_kernel<bf16_t, long long>), grid, dim3(256), 0, s, a);
  } else {
    if (a.idx_i32) hipLaunchKernelGGL((gather_kernel<float, int>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((gather_kernel<float, long long>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// NonZero and ScatterRows (execution-determined batch compaction)
// ---------------------------------------------------------------------------------------------
template <int KIND>
__device__ inline bool is_nonzero(const void* x, long long i) {
  if (KIND == 0) return ((const float*)x)[i] != 0.0f;
  if (KIND == 1) return (((const unsigned short*)x)[i] & 0x7fff) != 0;     // +0 and -0 are zero
  if (KIND == 2) return ((const long long*)x)[i] != 0;
  return ((const int*)x)[i] != 0;
}

// One workgroup of 256: a counting pass, then a compaction pass in element order (deterministic:
// positions come from prefix counts, no atomics).
template <int KIND>
__global__ __launch_bounds__(256) void nonzero_kernel(NonzeroArgs a) {
  __shared__ long long wave_n[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  long long mine = 0;
  for (long long i = tid; i < a.n; i += 256) mine += is_nonzero<KIND>(a.x, i) ? 1 : 0;
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
  if (lane == 0) wave_n[wave] = mine;
  __syncthreads();
  const long long total = wave_n[0] + wave_n[1] + wave_n[2] + wave_n[3];
  __syncthreads();
  long long run = 0;                                  // non-zeros before the current chunk
  for (long long c = 0; c < a.n; c += 256) {
    const long long i = c + tid;
    const bool f = i < a.n && is_nonzero<KIND>(a.x, i);
    const unsigned long long m = __ballot(f);
    if (lane == 0) wave_n[wave] = __popcll(m);
    __syncthreads();
    long long pos = run + __popcll(m & ((1ull << lane) - 1));
    for (int w = 0; w < wave; ++w) pos += wave_n[w];
    if (f) {
      long long rem = i;
      for (int r = a.rank - 1; r >= 0; --r) {
        a.out[(long long)r * total + pos] = rem % a.dims[r];
        rem /= a.dims[r];
      }
    }
    run += wave_n[0] + wave_n[1] + wave_n[2] + wave_n[3];
    __syncthreads();
  }
  if (tid == 0) *a.count = total;
}

hipError_t launch_nonzero(const NonzeroArgs& a, hipStream_t s) {
  switch (a.x_kind) {
    case 0: hipLaunchKernelGGL(nonzero_kernel<0>, dim3(1), dim3(256), 0, s, a); break;
    case 1: hipLaunchKernelGGL(nonzero_kernel<1>, dim3(1), dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL(nonzero_kernel<2>, dim3(1), dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL(nonzero_kernel<3>, dim3(1), dim3(256), 0, s, a); break;
  }
  return hipGetLastError();
}

// Non-maximum suppression.  One workgroup of 16 waves: (1) a bitonic sort in LDS of 64-bit keys (score, made
// decreasing, above the box index, so equal scores keep the index order); (2) the boxes copied to LDS in that order;
// (3) the greedy walk, 64 boxes at a time: the waves compute which box of the block suppresses which later box of
// the block (a 64 x 64 bit matrix, one ballot per row); every wave then resolves the block on its own with scalar
// bit operations (a box still alive is kept and clears the boxes its row names), wave 0 writes the kept indices,
// and all threads test the boxes behind the block against the block's kept boxes.  Two barriers per block.
// The overlap test is taken with separately rounded fp32 operations (no fused multiply-add), as the operator's
// definition states it: a kept box i suppresses j when inter > iou * ((area_i + area_j) - inter).
constexpr int NMS_THREADS = 1024;
__device__ inline bool nms_overlaps(const float4 bi, const float4 bj, float iou) {
#pragma clang fp contract(off)
  const float iw = fmaxf(0.f, fminf(bi.z, bj.z) - fmaxf(bi.x, bj.x));
  const float ih = fmaxf(0.f, fminf(bi.w, bj.w) - fmaxf(bi.y, bj.y));
  const float inter = iw * ih;
  const float area_i = (bi.z - bi.x) * (bi.w - bi.y);
  const float area_j = (bj.z - bj.x) * (bj.w - bj.y);
  const float uni = (area_i + area_j) - inter;
  return inter > iou * uni;
}
__global__ __launch_bounds__(NMS_THREADS) void nms_kernel(NmsArgs a) {
  __shared__ unsigned long long key[NMS_MAX_BOXES];
  __shared__ float4 box[NMS_MAX_BOXES];
  __shared__ unsigned char alive[NMS_MAX_BOXES];
  __shared__ unsigned long long rowmask[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int P = 1;
  while (P < a.n) P <<= 1;
  for (int i = tid; i < P; i += NMS_THREADS) {
    unsigned long long k = ~0ull;                      // padding sorts behind every box
    if (i < a.n) {
      unsigned u = __float_as_uint(a.scores[i] + 0.f); // (-0 becomes +0: the two are one score)
      u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // increasing with the score
      k = ((unsigned long long)(~u) << 32) | (unsigned)i;
    }
    key[i] = k;
  }
  __syncthreads();
  for (int size = 2; size <= P; size <<= 1)
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < P / 2; t += NMS_THREADS) {
        const int lo = 2 * t - (t & (stride - 1)), hi = lo + stride;
        const bool up = (lo & size) == 0;
        const unsigned long long x = key[lo], y = key[hi];
        if ((x > y) == up) { key[lo] = y; key[hi] = x; }
      }
      __syncthreads();
    }
  for (int i = tid; i < a.n; i += NMS_THREADS) {
    box[i] = *(const float4*)(a.boxes + 4ll * (unsigned)key[i]);
    alive[i] = 1;
  }
  __syncthreads();
  int count = 0;
  for (int b0 = 0; b0 < a.n; b0 += 64) {
    const int nb = min(64, a.n - b0);
    // which box of the block suppresses which later box of the block: wave w owns rows 4 w .. 4 w + 3, a lane a column
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = wave * 4 + q;
      bool bit = false;
      if (r < nb && lane < nb && lane > r) bit = nms_overlaps(box[b0 + r], box[b0 + lane], a.iou);
      const unsigned long long m = __ballot(bit);
      if (lane == 0) rowmask[r] = m;
    }
    __syncthreads();
    // every wave resolves the block (the same scalar walk in each: nothing to broadcast)
    const unsigned long long mine = rowmask[lane];
    const int mlo = (int)(unsigned)mine, mhi = (int)(unsigned)(mine >> 32);
    unsigned long long live = __ballot(lane < nb && alive[b0 + lane] != 0);
    unsigned long long kept = 0;
    int cnt = count;
#pragma unroll
    for (int r = 0; r < 64; ++r) {
      const unsigned long long m = (unsigned long long)(unsigned)__builtin_amdgcn_readlane(mlo, r) |
                                   ((unsigned long long)(unsigned)__builtin_amdgcn_readlane(mhi, r) << 32);
      if (((live >> r) & 1) && !(a.max_out > 0 && cnt >= a.max_out)) {
        kept |= 1ull << r;
        ++cnt;
        live &= ~m;
      }
    }
    if (wave == 0 && ((kept >> lane) & 1))
      a.out[count + __popcll(kept & ((1ull << lane) - 1))] = (long long)(unsigned)key[b0 + lane];
    count = cnt;
    if (a.max_out > 0 && count >= a.max_out) break;    // (the same in every thread)
    // the block's kept boxes against everything behind the block
    for (int j = b0 + 64 + tid; j < a.n; j += NMS_THREADS) {
      if (!alive[j]) continue;
      const float4 bj = box[j];
      for (unsigned long long m = kept; m; m &= m - 1)
        if (nms_overlaps(box[b0 + (int)__builtin_ctzll(m)], bj, a.iou)) { alive[j] = 0; break; }
    }
    __syncthreads();
  }
  if (tid == 0) *a.count = count;
}

// The same result from three kernels, for many boxes and a workspace to hold the suppression matrix: the pair tests
// are spread over the chip instead of running on one CU.  Workspace: the boxes in visiting order, their indices, and
// the matrix as 64 x 64-bit tiles, stored by column: word c of tile (rb, cb) = which of the 64 boxes of row block rb
// suppress box c of column block cb (only cb >= rb is written and read); for the diagonal tiles also by row
// (word r = which boxes of the block box r suppresses), which is what resolving a block needs.
constexpr long long NMS_WS_BOX = 0, NMS_WS_IDX = 64 << 10, NMS_WS_OWN = 96 << 10, NMS_WS_MASK = 128 << 10;
constexpr long long NMS_WS_BYTES = NMS_WS_MASK + (long long)NMS_MAX_BOXES * (NMS_MAX_BOXES / 64) * 8;
static_assert(NMS_WS_BYTES <= WS_BYTES, "the suppression matrix must fit the workspace");

__global__ __launch_bounds__(NMS_THREADS) void nms_sort_kernel(NmsArgs a) {
  __shared__ unsigned long long key[NMS_MAX_BOXES];
  const int tid = threadIdx.x;
  int P = 1;
  while (P < a.n) P <<= 1;
  for (int i = tid; i < P; i += NMS_THREADS) {
    unsigned long long k = ~0ull;
    if (i < a.n) {
      unsigned u = __float_as_uint(a.scores[i] + 0.f);
      u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      k = ((unsigned long long)(~u) << 32) | (unsigned)i;
    }
    key[i] = k;
  }
  __syncthreads();
  for (int size = 2; size <= P; size <<= 1)
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < P / 2; t += NMS_THREADS) {
        const int lo = 2 * t - (t & (stride - 1)), hi = lo + stride;
        const bool up = (lo & size) == 0;
        const unsigned long long x = key[lo], y = key[hi];
        if ((x > y) == up) { key[lo] = y; key[hi] = x; }
      }
      __syncthreads();
    }
  float4* sbox = (float4*)(a.ws + NMS_WS_BOX);
  unsigned* sidx = (unsigned*)(a.ws + NMS_WS_IDX);
  for (int i = tid; i < a.n; i += NMS_THREADS) {
    const unsigned id = (unsigned)key[i];
    sbox[i] = *(const float4*)(a.boxes + 4ll * id);
    sidx[i] = id;
  }
}

// grid (column block, row block), 64 threads: thread t owns column cb * 64 + t of the tile (and, on the diagonal,
// row rb * 64 + t as well)
__global__ __launch_bounds__(64) void nms_mask_kernel(NmsArgs a) {
  __shared__ float4 rbox[64];
  const int cb = blockIdx.x, rb = blockIdx.y, t = threadIdx.x;
  if (cb < rb) return;
  const float4* sbox = (const float4*)(a.ws + NMS_WS_BOX);
  const int W = (a.n + 63) >> 6;
  const int ir = rb * 64 + t, j = cb * 64 + t;
  rbox[t] = ir < a.n ? sbox[ir] : make_float4(0.f, 0.f, 0.f, 0.f);
  __syncthreads();
  const int r_end = min(64, a.n - rb * 64);
  unsigned long long word = 0;
  if (j < a.n) {
    const float4 bj = sbox[j];
    for (int r = 0; r < r_end; ++r)
      if (rb * 64 + r < j && nms_overlaps(rbox[r], bj, a.iou)) word |= 1ull << r;
  }
  ((unsigned long long*)(a.ws + NMS_WS_MASK))[((long long)rb * W + cb) * 64 + t] = word;
  if (cb == rb) {                                      // by row: the boxes of the block that box t suppresses
    unsigned long long own = 0;
    if (ir < a.n) {
      const float4 bi = rbox[t];
      for (int c = t + 1; c < r_end; ++c)
        if (nms_overlaps(bi, rbox[c], a.iou)) own |= 1ull << c;
    }
    ((unsigned long long*)(a.ws + NMS_WS_OWN))[ir] = own;
  }
}

// One workgroup of 4 waves walks the blocks in order; dead[w] = the boxes of block w suppressed so far.  Per block:
// wave 0 decides with scalar operations which boxes are kept (a box not yet dead is kept and kills what its own row
// names) and writes their indices; then every wave, for its share of the column blocks behind, turns the block's
// column words into the newly suppressed boxes with one ballot each (box c dies when a kept box is among the rows
// its word names).  The column words of the next block are requested before the current one is resolved.
constexpr int NMS_SCAN_THREADS = 256, NMS_SCAN_WAVES = NMS_SCAN_THREADS / 64, NMS_SCAN_PT = 64 / NMS_SCAN_WAVES;
__global__ __launch_bounds__(NMS_SCAN_THREADS) void nms_scan_kernel(NmsArgs a) {
  __shared__ unsigned long long dead[64];
  __shared__ unsigned long long kept_s;
  __shared__ int stop;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int W = (a.n + 63) >> 6;
  const unsigned long long* mask = (const unsigned long long*)(a.ws + NMS_WS_MASK);
  const unsigned long long* ownm = (const unsigned long long*)(a.ws + NMS_WS_OWN);
  const unsigned* sidx = (const unsigned*)(a.ws + NMS_WS_IDX);
  unsigned long long cur[NMS_SCAN_PT], nxt[NMS_SCAN_PT], own_nxt = 0;
  unsigned idx_nxt = 0;
  auto fetch = [&](int b) {                            // column words of tiles (b, w), w = b + wave, b + wave + 4, ...
#pragma unroll
    for (int u = 0; u < NMS_SCAN_PT; ++u) {
      const int w = b + wave + u * NMS_SCAN_WAVES;
      nxt[u] = (b < W && w < W) ? mask[((long long)b * W + w) * 64 + lane] : 0ull;
    }
    if (wave == 0 && b < W) {
      own_nxt = ownm[b * 64 + lane];
      idx_nxt = b * 64 + lane < a.n ? sidx[b * 64 + lane] : 0u;
    }
  };
  if (tid < 64) dead[tid] = 0;
  if (tid == 0) stop = 0;
  int count = 0;
  fetch(0);
  __syncthreads();
  for (int b = 0; b < W; ++b) {
#pragma unroll
    for (int u = 0; u < NMS_SCAN_PT; ++u) cur[u] = nxt[u];
    const unsigned long long own = own_nxt;
    const unsigned my_idx = idx_nxt;
    fetch(b + 1);
    if (wave == 0) {
      const int nb = min(64, a.n - b * 64);
      const int olo = (int)(unsigned)own, ohi = (int)(unsigned)(own >> 32);
      // (scalar values throughout: read through lane 0 so that the compiler keeps the walk on the scalar unit, and
      //  without branches: a taken branch costs more than the few operations it would skip)
      const unsigned long long d0 = dead[b];
      unsigned long long gone = (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)d0) |
                                ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(d0 >> 32)) << 32);
      if (nb < 64) gone |= ~0ull << nb;                // positions behind the last box count as dead
      const int lim = a.max_out > 0 ? a.max_out : 0x7fffffff;
      unsigned long long kept = 0;
      int cnt = count;
#pragma unroll
      for (int r = 0; r < 64; ++r) {
        const unsigned long long w = (unsigned long long)(unsigned)__builtin_amdgcn_readlane(olo, r) |
                                     ((unsigned long long)(unsigned)__builtin_amdgcn_readlane(ohi, r) << 32);
        const unsigned long long take = (~(gone >> r) & 1ull) & (unsigned long long)(cnt < lim);   // 0 or 1
        const unsigned long long m = 0ull - take;                                                    // 0 or all ones
        kept |= (1ull << r) & m;
        gone |= w & m;
        cnt += (int)take;
      }
      if ((kept >> lane) & 1) a.out[count + __popcll(kept & ((1ull << lane) - 1))] = (long long)my_idx;
      count = cnt;
      if (lane == 0) {
        kept_s = kept;
        if (a.max_out > 0 && count >= a.max_out) stop = 1;
      }
    }
    __syncthreads();
    const unsigned long long kept = kept_s;
#pragma unroll
    for (int u = 0; u < NMS_SCAN_PT; ++u) {
      const int w = b + wave + u * NMS_SCAN_WAVES;
      const unsigned long long hit = __ballot((cur[u] & kept) != 0);
      if (w < W && lane == 0) dead[w] |= hit;          // (a column block belongs to one wave)
    }
    __syncthreads();
    if (stop) break;
  }
  if (tid == 0) *a.count = count;
}

hipError_t launch_nms(const NmsArgs& a, hipStream_t s) {
  if (a.n < 0 || a.n > NMS_MAX_BOXES) return hipErrorInvalidValue;
  if (a.ws && a.n > 512) {
    const int W = (a.n + 63) / 64;
    hipLaunchKernelGGL(nms_sort_kernel, dim3(1), dim3(NMS_THREADS), 0, s, a);
    hipLaunchKernelGGL(nms_mask_kernel, dim3(W, W), dim3(64), 0, s, a);
    hipLaunchKernelGGL(nms_scan_kernel, dim3(1), dim3(NMS_SCAN_THREADS), 0, s, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(nms_kernel, dim3(1), dim3(NMS_THREADS), 0, s, a);
  return hipGetLastError();
}

// V: the unit a row is copied in (16 bytes when rows and pointers allow it, else one element)
template <class V, class I>
__global__ __launch_bounds__(256) void scatter_rows_kernel(ScatterArgs a, long long row_units) {
  const long long b = blockIdx.y;
  long long m = -1;
  for (long long j = 0; j < a.n; ++j) if ((long long)((const I*)a.idx)[j] == b) m = j;
  const V* src = m >= 0 ? (const V*)a.y + m * row_units : (const V*)a.x + b * row_units;
  V* dst = (V*)a.out + b * row_units;
  for (long long u = (long long)blockIdx.x * 256 + threadIdx.x; u < row_units; u += (long long)gridDim.x * 256) dst[u] = src[u];
}

// rows of a wide table picked by index, copied in 16-byte units by several workgroups per row
template <class I>
__global__ __launch_bounds__(256) void gather_rows16_kernel(GatherArgs a, long long row_units) {
  long long id = (long long)((const I*)a.idx)[blockIdx.y];
  id = id < 0 ? 0 : (id >= a.table_rows ? a.table_rows - 1 : id);
  const uint4* src = (const uint4*)a.table + id * row_units;
  uint4* dst = (uint4*)a.y + (long long)blockIdx.y * row_units;
  for (long long u = (long long)blockIdx.x * 256 + threadIdx.x; u < row_units; u += (long long)gridDim.x * 256) dst[u] = src[u];
}

// nearest-neighbour resize and concat along the last dim: pure copies in units of V
template <class V>
__global__ __launch_bounds__(256) void resize_nearest_kernel(ResizeArgs a) {
  const long long total = a.out[0] * a.out[1] * a.out[2] * a.row_units;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long u = i % a.row_units;
    long long pix = i / a.row_units;
    const long long o2 = pix % a.out[2]; pix /= a.out[2];
    const long long o1 = pix % a.out[1];
    const long long o0 = pix / a.out[1];
    const long long s0 = o0 * a.in[0] / a.out[0], s1 = o1 * a.in[1] / a.out[1], s2 = o2 * a.in[2] / a.out[2];
    ((V*)a.y)[i] = ((const V*)a.x)[((s0 * a.in[1] + s1) * a.in[2] + s2) * a.row_units + u];
  }
}

template <class V>
__global__ __launch_bounds__(256) void concat_last_kernel(ConcatArgs a) {
  const long long row_units = a.units[0] + a.units[1] + a.units[2] + a.units[3];
  const long long total = a.rows * row_units;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long r = i / row_units;
    long long u = i % row_units;
    int k = 0;
    while (k < 3 && u >= a.units[k]) { u -= a.units[k]; ++k; }
    ((V*)a.y)[i] = ((const V*)a.x[k])[r * a.units[k] + u];
  }
}

template <class K, class A>
static hipError_t launch_copy_units(K kernel16, K kernel4, K kernel2, int unit_bytes, long long total, const A& a, hipStream_t s) {
  if (total <= 0) return hipSuccess;
  dim3 grid((unsigned)std::min<long long>((total + 255) / 256, 4096));
  if (unit_bytes == 16) hipLaunchKernelGGL(kernel16, grid, dim3(256), 0, s, a);
  else if (unit_bytes == 4) hipLaunchKernelGGL(kernel4, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(kernel2, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_resize(const Launch& L, const ResizeArgs& a, hipStream_t s) {
  typedef void (*K)(ResizeArgs);
  return launch_copy_units<K>(resize_nearest_kernel<uint4>, resize_nearest_kernel<unsigned>, resize_nearest_kernel<unsigned short>,
                              L.unit_bytes, a.out[0] * a.out[1] * a.out[2] * a.row_units, a, s);
}
hipError_t launch_concat(const Launch& L, const ConcatArgs& a, hipStream_t s) {
  typedef void (*K)(ConcatArgs);
  return launch_copy_units<K>(concat_last_kernel<uint4>, concat_last_kernel<unsigned>, concat_last_kernel<unsigned short>,
                              L.unit_bytes, a.rows * (a.units[0] + a.units[1] + a.units[2] + a.units[3]), a, s);
}

__global__ __launch_bounds__(256) void range_kernel(RangeArgs a) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.n) return;
  const long long v = a.start + i * a.delta;
  if (a.out_i32) ((int*)a.y)[i] = (int)v;
  else ((long long*)a.y)[i] = v;
}
hipError_t launch_range(const RangeArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(range_kernel, dim3((unsigned)((a.n + 255) / 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_kernel(FillArgs a) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.n) return;
  float v = a.value;
  if (a.cols > 0) { const long long r = i / a.cols, c = i - r * a.cols; v = (c == r + a.diag) ? 1.f : 0.f; }
  if (a.dtype == SOD2_BF16_TAG) ((bf16_t*)a.y)[i] = f2bf(v);
  else if (a.dtype == 0) ((float*)a.y)[i] = v;                  // dtype tags: 0 f32, 1 bf16, 2 i64, 3 i32
  else if (a.dtype == 3) ((int*)a.y)[i] = (int)v;
  else ((long long*)a.y)[i] = (long long)v;
}
hipError_t launch_fill(const FillArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((a.n + 255) / 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}

// MaxUnpool: the result is cleared by one kernel and the values are dropped at their positions by a second one on
// the same stream (positions are distinct by contract: the stores of one launch never meet).
template <class T>
__global__ __launch_bounds__(256) void unpool_clear_kernel(UnpoolArgs a) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < a.n_out) ((T*)a.y)[i] = (T)0;
}
template <class T>
__global__ __launch_bounds__(256) void unpool_scatter_kernel(UnpoolArgs a) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.n_in) return;
  const long long at = ((const long long*)a.idx)[i];
  if (at >= 0 && at < a.n_out) ((T*)a.y)[at] = ((const T*)a.x)[i];
}
hipError_t launch_unpool(const Launch& L, const UnpoolArgs& a, hipStream_t s) {
  if (a.n_out <= 0) return hipSuccess;
  const dim3 go((unsigned)((a.n_out + 255) / 256)), gi((unsigned)((a.n_in + 255) / 256));
  if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(unpool_clear_kernel<unsigned short>, go, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(unpool_clear_kernel<unsigned int>, go, dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.n_in <= 0) return e;
  if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(unpool_scatter_kernel<unsigned short>, gi, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(unpool_scatter_kernel<unsigned int>, gi, dim3(256), 0, s, a);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void onehot_kernel(OneHotArgs a) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.n * a.depth) return;
  const long long i = e / a.depth, d = e - i * a.depth;
  long long ix = a.idx_i32 ? (long long)((const int*)a.idx)[i] : ((const long long*)a.idx)[i];
  if (ix < 0) ix += a.depth;
  const float v = ix == d ? a.on : a.off;
  if (a.out_bf16) ((bf16_t*)a.y)[e] = f2bf(v);
  else ((float*)a.y)[e] = v;
}
hipError_t launch_onehot(const OneHotArgs& a, hipStream_t s) {
  const long long total = a.n * a.depth;
  if (total <= 0) return hipSuccess;
  hipLaunchKernelGGL(onehot_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}

// One wave per row.  The entries are taken in the order (value descending, position ascending): round j
// scans the row for the best entry that comes strictly after the one taken in round j - 1, so no
// entry has to be marked; the 64 lanes' candidates are merged with shuffles.  k rounds over a row that
// stays in the caches: meant for the short k of routing and detection heads.
template <bool BF>
__global__ __launch_bounds__(256) void topk_kernel(TopKArgs a) {
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= a.rows) return;
  const bf16_t* xb = (const bf16_t*)a.x + row * a.n;
  const float* xf = (const float*)a.x + row * a.n;
  float last_v = 0.f;
  long long last_i = -1;
  for (long long j = 0; j < a.k; ++j) {
    float best_v = 0.f;
    long long best_i = -1;
    for (long long i = lane; i < a.n; i += 64) {
      const float v = BF ? bf2f(xb[i]) : xf[i];
      const bool after = j == 0 || v < last_v || (v == last_v && i > last_i);
      if (after && (best_i < 0 || v > best_v)) { best_v = v; best_i = i; }     // ascending i: the first of equals stays
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(best_v, off);
      const long long oi = __shfl_xor(best_i, off);
      if (oi >= 0 && (best_i < 0 || ov > best_v || (ov == best_v && oi < best_i))) { best_v = ov; best_i = oi; }
    }
    if (best_i < 0) { best_i = 0; best_v = 0.f; }                // only with NaN entries: stay inside the row
    last_v = best_v;
    last_i = best_i;
    if (lane == 0) {
      const long long o = row * a.k + j;
      if (BF) ((bf16_t*)a.values)[o] = xb[best_i];
      else ((float*)a.values)[o] = best_v;
      if (a.idx_i32) ((int*)a.indices)[o] = (int)best_i;
      else ((long long*)a.indices)[o] = best_i;
    }
  }
}
hipError_t launch_topk(const TopKArgs& a, hipStream_t s) {
  if (a.rows <= 0 || a.k <= 0) return hipSuccess;
  dim3 grid((unsigned)((a.rows + 3) / 4));
  if (a.x_bf16) hipLaunchKernelGGL(topk_kernel<true>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(topk_kernel<false>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_scatter(const Launch& L, const ScatterArgs& a, hipStream_t s) {
  if (a.rows <= 0 || a.cols <= 0) return hipSuccess;
  const long long eb = L.out_dtype == SOD2_BF16_TAG ? 2 : 4, row_bytes = a.cols * eb;
  const bool v16 = row_bytes % 16 == 0 && (((uintptr_t)a.x | (uintptr_t)a.y | (uintptr_t)a.out) & 15) == 0;
  const long long units = v16 ? row_bytes / 16 : a.cols;
  dim3 grid((unsigned)std::min<long long>((units + 255) / 256, 64), (unsigned)a.rows);
  if (v16) {
    if (a.idx_i32) hipLaunchKernelGGL((scatter_rows_kernel<uint4, int>), grid, dim3(256), 0, s, a, units);
    else hipLaunchKernelGGL((scatter_rows_kernel<uint4, long long>), grid, dim3(256), 0, s, a, units);
  } else if (eb == 2) {
    if (a.idx_i32) hipLaunchKernelGGL((scatter_rows_kernel<unsigned short, int>), grid, dim3(256), 0, s, a, units);
    else hipLaunchKernelGGL((scatter_rows_kernel<unsigned short, long long>), grid, dim3(256), 0, s, a, units);
  } else {
    if (a.idx_i32) hipLaunchKernelGGL((scatter_rows_kernel<unsigned, int>), grid, dim3(256), 0, s, a, units);
    else hipLaunchKernelGGL((scatter_rows_kernel<unsigned, long long>), grid, dim3(256), 0, s, a, units);
  }
  return hipGetLastError();
}

hipError_t launch_append(const Launch& L, const AppendArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  dim3 grid((unsigned)a.rows);
  if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(append_kernel<bf16_t>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(append_kernel<float>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_argmax(const Launch& L, const ArgmaxArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  dim3 grid((unsigned)a.rows);
  if (L.in_dtype == SOD2_BF16_TAG && a.cols % 8 == 0 && a.cols >= 2048 && a.x_stride % 8 == 0 && a.x_step % 16 == 0 &&
      ((uintptr_t)a.x & 15) == 0) {
    hipLaunchKernelGGL(argmax_bf16x8_kernel, grid, dim3(1024), 0, s, a);
    return hipGetLastError();
  }
  if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(argmax_kernel<bf16_t>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(argmax_kernel<float>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_eltwise(const Launch& L, const EltArgs& a, hipStream_t s) {
  dim3 grid((unsigned)((a.total + 255) / 256));
  if (L.out_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(eltwise_kernel<bf16_t>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(eltwise_kernel<float>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// host-side launchers
// ---------------------------------------------------------------------------------------------
template <class AL, int WM, int WN, int TM, int TN>
static hipError_t launch_mfma(const AL& al, const GemmArgs& g, hipStream_t s) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  dim3 grid(((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN), g.nb0 * g.nb1);
  hipLaunchKernelGGL((gemm_mfma<AL, WM, WN, TM, TN>), grid, dim3(256), 0, s, al, g);
  return hipGetLastError();
}
template <class AL>
static hipError_t launch_mfma_variant(const AL& al, const GemmArgs& g, int variant, hipStream_t s) {
  switch (variant) {
    case V_FAT: return launch_mfma<AL, 2, 2, 4, 2>(al, g, s);        // 256 x 128
    case V_SKINNY: return launch_mfma<AL, 1, 4, 1, 1>(al, g, s);     // 32 x 128
    case V_SMALL: return launch_mfma<AL, 1, 4, 1, 1>(al, g, s);
    case V_XFAT: return launch_mfma<AL, 2, 2, 4, 2>(al, g, s);
    default: return launch_mfma<AL, 2, 2, 2, 2>(al, g, s);           // 128 x 128
  }
}

hipError_t launch_gemm_dl(const GemmArgs& g, int tile, hipStream_t s);
hipError_t launch_conv_dl(const ConvArgs& c, const GemmArgs& g, int tile, hipStream_t s);

hipError_t launch_gemv(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_ln(const GemmArgs& g, hipStream_t s);

// fp32 contraction with at most 8 rows (the gate networks of the control-flow graphs): one wave per
// output column, the lanes split k in 16-byte chunks of B[n, :], a shuffle tree finishes the sums
template <int MR>
__global__ __launch_bounds__(256) void gemv_f32_kernel(GemmArgs g) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 4 + wave;
  const int b0 = blockIdx.y / g.nb1, b1 = blockIdx.y % g.nb1;
  if (n >= g.N) return;
  const float* A = (const float*)g.A + b0 * g.a_sb0 + b1 * g.a_sb1;
  const float* B = (const float*)g.B + b0 * g.b_sb0 + b1 * g.b_sb1 + (long long)n * g.b_sn;
  float acc[MR];
#pragma unroll
  for (int m = 0; m < MR; ++m) acc[m] = 0.f;
  const int nchunk = g.K >> 2;
  for (int c = lane; c < nchunk; c += 64) {
    const float4 w = *(const float4*)(B + c * 4);
#pragma unroll
    for (int m = 0; m < MR; ++m) {
      if (m < g.M) {
        const float4 a = *(const float4*)(A + (long long)m * g.a_sm + c * 4);
        acc[m] = fmaf(a.x, w.x, fmaf(a.y, w.y, fmaf(a.z, w.z, fmaf(a.w, w.w, acc[m]))));
      }
    }
  }
#pragma unroll
  for (int m = 0; m < MR; ++m) acc[m] = wave_sum(acc[m]);
  if (lane == 0) {
    const float bv = g.bias ? ((const float*)g.bias)[n] : 0.f;
    float* Cp = (float*)g.C + b0 * g.c_sb0 + b1 * g.c_sb1;
    const float* Rp = g.res ? (const float*)g.res + b0 * g.r_sb0 + b1 * g.r_sb1 : nullptr;
#pragma unroll
    for (int m = 0; m < MR; ++m) {
      if (m < g.M) {
        float v = apply_act(acc[m] * g.scale + bv, g.act1);
        if (Rp) v = apply_act(v + Rp[(long long)m * g.r_sm + (long long)n * g.r_sn], g.act2);
        Cp[(long long)m * g.c_sm + (long long)n * g.c_sn] = v;
      }
    }
  }
}

static bool gemv_f32_ok(const Launch& L, const GemmArgs& g) {
  auto al = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  return L.in_dtype != SOD2_BF16_TAG && L.out_dtype != SOD2_BF16_TAG && L.variant == V_GEMV && g.M <= 8 &&
         g.a_sk == 1 && g.b_sk == 1 && g.K % 4 == 0 && g.a_sm % 4 == 0 && g.b_sn % 4 == 0 && g.a_sb0 % 4 == 0 &&
         g.a_sb1 % 4 == 0 && g.b_sb0 % 4 == 0 && g.b_sb1 % 4 == 0 && al(g.A) && al(g.B);
}

hipError_t launch_gemm(const Launch& L, const GemmArgs& g, hipStream_t s) {
  if (g.ln_gamma) return L.in_dtype == SOD2_BF16_TAG ? launch_gemm_ln(g, s) : hipErrorInvalidValue;
  if (gemv_f32_ok(L, g)) {
    dim3 grid((g.N + 3) / 4, g.nb0 * g.nb1);
    if (g.M <= 1) hipLaunchKernelGGL(gemv_f32_kernel<1>, grid, dim3(256), 0, s, g);
    else if (g.M <= 4) hipLaunchKernelGGL(gemv_f32_kernel<4>, grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL(gemv_f32_kernel<8>, grid, dim3(256), 0, s, g);
    return hipGetLastError();
  }
  if (L.variant == V_GEMV && L.in_dtype == SOD2_BF16_TAG && g.a_vec && g.b_mode == 0 && g.M <= 8) return launch_gemv(g, s);
  if (L.variant >= V_DL0 && L.in_dtype == SOD2_BF16_TAG && g.a_vec && g.b_mode == 0)
    return launch_gemm_dl(g, L.variant - V_DL0, s);
  if (L.variant == V_SIMPLE || L.in_dtype != SOD2_BF16_TAG) {
    dim3 grid(((g.M + 63) / 64) * ((g.N + 63) / 64), g.nb0 * g.nb1);
    if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(gemm_simple<bf16_t>, grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL(gemm_simple<float>, grid, dim3(256), 0, s, g);
    return hipGetLastError();
  }
  MatA al{(const bf16_t*)g.A, g.a_sm, g.a_sk, g.M, g.K, g.a_vec};
  return launch_mfma_variant(al, g, L.variant, s);
}

// ---------------------------------------------------------------------------------------------
// Convolution with very few input channels and 64 output channels (the 7x7 / 2 stem on RGB images).
// The implicit-GEMM kernels gather such an operand element by element (k = (kh, kw, c) with c < 8 has
// no 16-byte runs).  Here a workgroup takes 128 consecutive output pixels of one output row, stages
// the KH input rows they touch in LDS once (contiguous in memory: [iw, c] is dense), and reads MFMA
// operands straight from that patch: with k ordered (kh, j = kw * C + c) and j padded from KW * C to 24,
// the 8 consecutive k of a lane are 8 consecutive patch elements starting at stride * C * pixel + 8 r.
// The weights are re-laid to the same padded order in LDS (zeros in the padding, so whatever the patch
// holds there does not count).
constexpr int STEM_BM = 128, STEM_ROW = 1056, STEM_KH = 7, STEM_J = 24, STEM_O = 64, STEM_K = 176, STEM_WROW = 184;
__global__ __launch_bounds__(256) void conv_stem_kernel(ConvArgs c) {
  __shared__ __attribute__((aligned(16))) bf16_t patch[STEM_KH][STEM_ROW];
  __shared__ __attribute__((aligned(16))) bf16_t wt[STEM_O][STEM_WROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles_w = (c.OW + STEM_BM - 1) / STEM_BM;
  int t = blockIdx.x;
  const int ow0 = (t % tiles_w) * STEM_BM; t /= tiles_w;
  const int oh = t % c.OH, nb = t / c.OH;
  const int J = c.KW * c.C, step = c.stride * c.C;
  const bf16_t* w = (const bf16_t*)c.w;
  {
    // one output channel per lane, the kh rows dealt over the 4 waves; fixed trip counts so that all
    // loads of a thread are in flight together
    const int n = tid & 63;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int kh = wave + 4 * kk;
      const bf16_t* wr = w + ((long long)n * c.KH + kh) * J;
      bf16_t v[STEM_J];
#pragma unroll
      for (int j = 0; j < STEM_J; ++j) v[j] = (kh < c.KH && j < J) ? wr[j] : (bf16_t)0;
#pragma unroll
      for (int j = 0; j < STEM_J; ++j) if (kh * STEM_J + j < STEM_K) wt[n][kh * STEM_J + j] = v[j];
    }
  }
  const int need = step * (STEM_BM - 1) + STEM_J + 8;               // patch elements a row of this tile can touch
  const long long first = (long long)(ow0 * c.stride - c.pad) * c.C;  // element offset of patch[.][0] in its input row
  const long long row_len = (long long)c.W * c.C;
#pragma unroll
  for (int kh = 0; kh < STEM_KH; ++kh) {
    const int ih = oh * c.stride - c.pad + kh;
    const bf16_t* xr = (const bf16_t*)c.x + ((long long)nb * c.H + ih) * row_len;
    const bool row_ok = kh < c.KH && ih >= 0 && ih < c.H;
    bf16_t v[(STEM_ROW + 255) / 256];
#pragma unroll
    for (int i = 0; i < (STEM_ROW + 255) / 256; ++i) {
      const int e = tid + 256 * i;
      const long long off = first + e;
      v[i] = (row_ok && e < need && off >= 0 && off < row_len) ? xr[off] : (bf16_t)0;
    }
#pragma unroll
    for (int i = 0; i < (STEM_ROW + 255) / 256; ++i) {
      const int e = tid + 256 * i;
      if (e < need) patch[kh][e] = v[i];
    }
  }
  __syncthreads();
  const int m = wave * 32 + (lane & 31), kg = lane >> 5;
  f32x16_t acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < STEM_K / 16; ++ks) {
    const int q = 2 * ks + kg, kh = q / 3, r8 = (q % 3) * 8;
    V16 af;
    af.u = zero4();
    if (kh < c.KH) {
      const bf16_t* p = &patch[kh][step * m + r8];
#pragma unroll
      for (int e = 0; e < 8; ++e) af.h[e] = p[e];
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      V16 bf;
      bf.u = *(const uint4*)&wt[j * 32 + (lane & 31)][ks * 16 + kg * 8];
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.b, bf.b, acc[j], 0, 0, 0);
    }
  }
  const bf16_t* bias = (const bf16_t*)c.bias;
  bf16_t* y = (bf16_t*)c.y + ((long long)nb * c.OH + oh) * c.OW * STEM_O;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = j * 32 + (lane & 31);
    const float bv = bias ? bf2f(bias[n]) : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int ow = ow0 + wave * 32 + (r >> 2) * 8 + kg * 4 + (r & 3);
      if (ow < c.OW) y[(long long)ow * STEM_O + n] = f2bf(apply_act(acc[j][r] + bv, c.act1));
    }
  }
}

static bool stem_ok(const Launch& L, const ConvArgs& c) {
  return L.in_dtype == SOD2_BF16_TAG && L.variant >= V_DL0 && c.O == STEM_O && c.KH <= STEM_KH && c.KW * c.C <= STEM_J &&
         c.C < 8 && c.stride * c.C * (STEM_BM - 1) + STEM_J + 8 <= STEM_ROW && !c.res && c.act2 == ACT_NONE;
}

hipError_t launch_conv(const Launch& L, const ConvArgs& c, hipStream_t s) {
  if (stem_ok(L, c)) {
    const long long tiles = (long long)c.NB * c.OH * ((c.OW + STEM_BM - 1) / STEM_BM);
    if (tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL(conv_stem_kernel, dim3((unsigned)tiles), dim3(256), 0, s, c);
    return hipGetLastError();
  }
  if (L.variant == V_SIMPLE || L.in_dtype != SOD2_BF16_TAG) {
    long long total = (long long)c.NB * c.OH * c.OW * c.O;
    dim3 grid((unsigned)((total + 255) / 256));
    if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(conv_simple<bf16_t>, grid, dim3(256), 0, s, c);
    else hipLaunchKernelGGL(conv_simple<float>, grid, dim3(256), 0, s, c);
    return hipGetLastError();
  }
  GemmArgs g{};
  g.M = c.NB * c.OH * c.OW; g.N = c.O; g.K = c.KH * c.KW * c.C;
  g.nb0 = g.nb1 = 1;
  g.B = c.w; g.b_sk = 1; g.b_sn = g.K; g.b_mode = (g.K % 8 == 0 && ((uintptr_t)c.w & 15) == 0) ? 0 : 2;
  g.C = c.y; g.c_sm = c.O; g.c_sn = 1;
  g.bias = c.bias; g.res = c.res; g.r_sm = c.O; g.r_sn = 1;
  g.scale = 1.f; g.act1 = c.act1; g.act2 = c.act2;
  g.c_vec = (c.O % 8 == 0) && (((uintptr_t)c.y & 15) == 0) && (!c.bias || ((uintptr_t)c.bias & 15) == 0) &&
            (!c.res || ((uintptr_t)c.res & 15) == 0);
  if (L.variant >= V_DL0 && c.vec && c.C % 64 == 0 && g.b_mode == 0) {
    g.group_m = 8;
    if (c.splits > 1 && c.ws) { g.splits = c.splits; g.ws = c.ws; }
    return launch_conv_dl(c, g, L.variant - V_DL0, s);
  }
  ConvA al{(const bf16_t*)c.x, c.H, c.W, c.C, c.KW, c.stride, c.pad, c.OH, c.OW, g.M, g.K, c.vec};
  return launch_mfma_variant(al, g, L.variant, s);
}

template <class T>
static void launch_row_t(const Launch& L, const RowArgs& a, hipStream_t s) {
  constexpr int VN = Vec<T>::N;
  bool vec = a.cols % VN == 0 && a.cols <= 64 * VN * 4 && a.x_stride % VN == 0 && a.y_stride % VN == 0 &&
             ((uintptr_t)a.x % 16 == 0) && ((uintptr_t)a.y % 16 == 0) &&
             (!L.is_layernorm || (((uintptr_t)a.gamma % 16 == 0) && ((uintptr_t)a.beta % 16 == 0)));
  dim3 grid((unsigned)((a.rows + 3) / 4));
  if (L.is_layernorm) {
    if (vec) hipLaunchKernelGGL((row_kernel<T, 0, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((row_kernel<T, 0, false>), grid, dim3(256), 0, s, a);
  } else {
    if (vec) hipLaunchKernelGGL((row_kernel<T, 1, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((row_kernel<T, 1, false>), grid, dim3(256), 0, s, a);
  }
}
hipError_t launch_row(const Launch& L, const RowArgs& a, hipStream_t s) {
  if (L.in_dtype == SOD2_BF16_TAG) launch_row_t<bf16_t>(L, a, s);
  else launch_row_t<float>(L, a, s);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// GroupNormalization, channels last.  One workgroup per (sample, group): its slab is s positions of cpg
// consecutive channels, `C` elements apart.  Three walks over the slab (mean, centred sum of squares, apply):
// the slab of one group stays in the L2 between them, and the two-pass variance matches the definition.
// A thread handles whole positions (cpg contiguous elements), so the loads of a wave cover runs of cpg elements.
// ---------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void groupnorm_kernel(GroupNormArgs a) {
  __shared__ float red[8];
  const int g = blockIdx.x % a.groups;
  const long long n = blockIdx.x / a.groups;
  const int C = a.groups * a.cpg;
  const T* x = (const T*)a.x + n * a.s * C + (long long)g * a.cpg;
  T* y = (T*)a.y + n * a.s * C + (long long)g * a.cpg;
  const long long total = a.s * a.cpg;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  auto block_sum = [&](float v) {
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
  };
  float sum = 0.f;
  for (long long e = threadIdx.x; e < total; e += 256) sum += to_f<T>(x[(e / a.cpg) * C + e % a.cpg]);
  const float mean = block_sum(sum) / (float)total;
  float ss = 0.f;
  for (long long e = threadIdx.x; e < total; e += 256) {
    const float d = to_f<T>(x[(e / a.cpg) * C + e % a.cpg]) - mean;
    ss += d * d;
  }
  const float rstd = rsqrtf(block_sum(ss) / (float)total + a.eps);
  const T* gam = (const T*)a.gamma + g * a.cpg;
  const T* bet = (const T*)a.beta + g * a.cpg;
  for (long long e = threadIdx.x; e < total; e += 256) {
    const int c = (int)(e % a.cpg);
    const long long at = (e / a.cpg) * C + c;
    y[at] = from_f<T>((to_f<T>(x[at]) - mean) * rstd * to_f<T>(gam[c]) + to_f<T>(bet[c]));
  }
}
hipError_t launch_groupnorm(const Launch& L, const GroupNormArgs& a, hipStream_t s) {
  if (a.n * a.groups <= 0 || a.s <= 0) return hipSuccess;
  dim3 grid((unsigned)(a.n * a.groups));
  if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(groupnorm_kernel<bf16_t>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(groupnorm_kernel<float>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_reduce(const Launch& L, const ReduceArgs& a, hipStream_t s) {
  bool ib = L.in_dtype == SOD2_BF16_TAG, ob = L.out_dtype == SOD2_BF16_TAG;
  if (ib && a.C % 8 == 0 && ((uintptr_t)a.x & 15) == 0 && a.R >= 64) {
    if ((long long)((a.C + 511) / 512) * a.batch >= 16) {
      dim3 wide((a.C + 511) / 512, a.batch);
      if (ob) hipLaunchKernelGGL((reduce_mean_bf16_wide_kernel<bf16_t, 8>), wide, dim3(1024), 0, s, a);
      else hipLaunchKernelGGL((reduce_mean_bf16_wide_kernel<float, 8>), wide, dim3(1024), 0, s, a);
    } else {                                             // few rows of workgroups: narrower ones, more CUs
      dim3 wide((a.C + 127) / 128, a.batch);
      if (ob) hipLaunchKernelGGL((reduce_mean_bf16_wide_kernel<bf16_t, 2>), wide, dim3(1024), 0, s, a);
      else hipLaunchKernelGGL((reduce_mean_bf16_wide_kernel<float, 2>), wide, dim3(1024), 0, s, a);
    }
    return hipGetLastError();
  }
  dim3 grid((a.C + 63) / 64, a.batch);
  if (ib && ob) hipLaunchKernelGGL((reduce_mean_kernel<bf16_t, bf16_t>), grid, dim3(256), 0, s, a);
  else if (ib) hipLaunchKernelGGL((reduce_mean_kernel<bf16_t, float>), grid, dim3(256), 0, s, a);
  else if (ob) hipLaunchKernelGGL((reduce_mean_kernel<float, bf16_t>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((reduce_mean_kernel<float, float>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_pool(const Launch& L, const PoolArgs& p, hipStream_t s) {
  if (L.in_dtype == SOD2_BF16_TAG && p.C % 8 == 0 && (p.k == 2 || p.k == 3) && ((uintptr_t)p.x & 15) == 0 && ((uintptr_t)p.y & 15) == 0) {
    const long long tv = (long long)p.NB * p.OH * p.OW * (p.C / 8);
    if (tv <= 0) return hipSuccess;
    const dim3 gv((unsigned)((tv + 255) / 256));
    if (p.k == 3 && p.avg) hipLaunchKernelGGL((maxpool_bf16x8_kernel<3, true>), gv, dim3(256), 0, s, p);
    else if (p.k == 3) hipLaunchKernelGGL((maxpool_bf16x8_kernel<3, false>), gv, dim3(256), 0, s, p);
    else if (p.avg) hipLaunchKernelGGL((maxpool_bf16x8_kernel<2, true>), gv, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((maxpool_bf16x8_kernel<2, false>), gv, dim3(256), 0, s, p);
    return hipGetLastError();
  }
  long long total = (long long)p.NB * p.OH * p.OW * p.C;
  dim3 grid((unsigned)((total + 255) / 256));
  if (L.in_dtype == SOD2_BF16_TAG) hipLaunchKernelGGL(maxpool_kernel<bf16_t>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(maxpool_kernel<float>, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace sod2
