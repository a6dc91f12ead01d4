// Fused attention for gfx950: O = softmax(scale * Q K^T [+ causal mask]) V per (batch, head), head
// size 64, bf16 operands, fp32 accumulation; scores and probabilities never leave the registers.
//
// Both contractions run on v_mfma_f32_32x32x16_bf16 in the *transposed* form, so that a lane owns one
// query for the whole kernel:
//   S^T[key, query] = sum_d K[key, d] Q[query, d]      A = K tile (LDS, d contiguous), B = Q (registers)
//   O^T[d,   query] = sum_key V[key, d] P[query, key]  A = V^T tile (LDS, keys contiguous), B = P (registers)
// The MFMA result layout puts column (lane & 31) = query in every lane, 16 rows per lane.  Hence the
// softmax statistics of a query are reductions inside a lane plus one exchange with lane ^ 32, the
// rescaling of O is a per-lane scalar, and the probabilities a lane holds after the first
// contraction are exactly the B operand of the second one: the 8 accumulators 8s .. 8s+7 of a
// 32-key block are the keys {16s + 4h + i, 16s + 8 + 4h + i : i < 4} of lane half h.  V is written
// to LDS transposed with the key index permuted the same way (bits 2 and 3 swapped), so one 16-byte
// LDS read yields the matching A operand.
//
// One workgroup = NW waves = NW * 32 queries of one (batch, head); K / V tiles of 64 keys are
// shared through LDS, double buffered, the next two tiles prefetched into registers during the MFMAs.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_common.hpp"

namespace sod2 {

__device__ __forceinline__ int attn_swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }   // 128-byte rows

template <int NW>
__global__ __launch_bounds__(NW * 64) void attention_kernel(AttnArgs a) {
  constexpr int NT = NW * 64, D = 64, BKV = 64;
  constexpr int LPT = BKV * 8 / NT;                      // 16-byte chunks of a K (or V) tile per thread
  __shared__ __attribute__((aligned(16))) bf16_t Ks[2][BKV * D];    // [key][d], chunk-swizzled
  __shared__ __attribute__((aligned(16))) bf16_t Vt[2][D * BKV];    // [d][permuted key], chunk-swizzled

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  // Workgroups are dealt round-robin to the 8 XCDs: keep all query tiles of one (batch, head) on one
  // XCD, so that its K and V are fetched into a single L2 (grid = 8 * ceil(batch / 8) * query tiles)
  const int n_qt = (a.Lq + NW * 32 - 1) / (NW * 32);
  const int slot = blockIdx.x >> 3;
  const int bh = (slot / n_qt) * 8 + (blockIdx.x & 7);
  if (bh >= a.nb0 * a.nb1) return;
  const int b0 = bh / a.nb1, b1 = bh % a.nb1;
  const int q_wg = (slot % n_qt) * (NW * 32);
  const int query = q_wg + wave * 32 + col;
  const int off = a.Lk - a.Lq;                           // causal: query i sees keys <= i + off

  const bf16_t* Qp = (const bf16_t*)a.q + b0 * a.q_sb0 + b1 * a.q_sb1;
  const bf16_t* Kp = (const bf16_t*)a.k + b0 * a.k_sb0 + b1 * a.k_sb1;
  const bf16_t* Vp = (const bf16_t*)a.v + b0 * a.v_sb0 + b1 * a.v_sb1;

  // Q as the B operand of S^T: lane (query, half) holds d = 16 ks + 8 half .. + 7
  V16 qf[4];
  {
    const bf16_t* qr = Qp + (long long)min(query, a.Lq - 1) * a.q_sm;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[ks].u = *(const uint4*)(qr + ks * 16 + half * 8);
  }

  int n_tiles = (a.Lk + BKV - 1) / BKV;
  if (a.causal) {
    const int last_q = min(q_wg + NW * 32, a.Lq) - 1;    // keys beyond last_q + off are masked for everyone here
    n_tiles = min(n_tiles, (last_q + off) / BKV + 1);
  }

  // tile loads.  K: chunk p = tid + i * NT -> key p / 8, d chunk p % 8.  V: a thread takes the same d
  // chunk of LPT consecutive keys, which are LPT consecutive positions of the permuted key order too
  // (LPT is 2 or 4, the permutation moves bits 2 and 3), so the transposed store is one 4- or 8-byte
  // write per d instead of LPT 2-byte writes
  static_assert(LPT == 2 || LPT == 4, "V store packs 2 or 4 keys");
  // two register sets: the tile after next is already on its way while the next one waits for its store
  // (native vector types: with HIP's uint4 class the compiler kept these arrays in scratch memory, every
  //  prefetched tile went global -> registers -> scratch -> registers -> LDS: 17.1 -> 15.2 us per launch)
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 krA[LPT], vrA[LPT], krB[LPT], vrB[LPT];
  const int v_dc = tid & 7, v_key0 = (tid >> 3) * LPT;
  auto gload = [&](int t, u32x4 (&kr)[LPT], u32x4 (&vr)[LPT]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int p = tid + i * NT;
      const int key = min(t * BKV + p / 8, a.Lk - 1);
      kr[i] = *(const u32x4*)(Kp + (long long)key * a.k_sn + (p % 8) * 8);
      const int vkey = min(t * BKV + v_key0 + i, a.Lk - 1);
      vr[i] = *(const u32x4*)(Vp + (long long)vkey * a.v_sn + v_dc * 8);
    }
  };
  auto sstore = [&](int buf, const u32x4 (&kr)[LPT], const u32x4 (&vr)[LPT]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int p = tid + i * NT;
      const int key = p / 8, dc = p % 8;
      *(u32x4*)&Ks[buf][key * D + attn_swz(key, dc) * 8] = kr[i];
    }
    const int kp0 = (v_key0 & ~0xC) | ((v_key0 & 4) << 1) | ((v_key0 & 8) >> 1);   // swap bits 2 and 3
    // element e of a 16-byte chunk: half (e & 1) of its 32-bit word e / 2
    auto elem = [](const u32x4& u, int e) __attribute__((always_inline)) { const uint32_t w = u[e >> 1]; return (e & 1) ? (w >> 16) : (w & 0xffffu); };
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int d = v_dc * 8 + e;
      bf16_t* dst = &Vt[buf][d * BKV + attn_swz(d, kp0 >> 3) * 8 + (kp0 & 7)];
      if (LPT == 4) {
        uint2 w;
        w.x = elem(vr[0], e) | (elem(vr[1], e) << 16);
        w.y = elem(vr[2 % LPT], e) | (elem(vr[3 % LPT], e) << 16);
        *(uint2*)dst = w;
      } else {
        *(uint32_t*)dst = elem(vr[0], e) | (elem(vr[1], e) << 16);
      }
    }
  };

  f32x16_t oacc[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = a.scale * 1.4426950408889634f;        // scores in units of log2 e

  gload(0, krA, vrA);
  sstore(0, krA, vrA);
  if (n_tiles > 1) gload(1, krA, vrA);
  __syncthreads();
  // one key / value tile: `cur` holds tile t + 1 (loaded one step ago), `nxt` receives tile t + 2
  auto step = [&](int t, u32x4 (&kr_cur)[LPT], u32x4 (&vr_cur)[LPT], u32x4 (&kr_nxt)[LPT], u32x4 (&vr_nxt)[LPT]) __attribute__((always_inline)) {
    const int buf = t & 1;
    if (t + 2 < n_tiles) gload(t + 2, kr_nxt, vr_nxt);

    // ---- S^T for the 64 keys of the tile: two 32-key blocks ----
    f32x16_t s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
      const int krow = kb * 32 + col;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        V16 kf;
        kf.u = *(const uint4*)&Ks[buf][krow * D + attn_swz(krow, ks * 2 + half) * 8];
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.b, qf[ks].b, s[kb], 0, 0, 0);
      }
    }
    // ---- mask, running max and sum for this lane's query ----
    const int key_hi = a.causal ? min(a.Lk - 1, query + off) : a.Lk - 1;     // last visible key
    // every key of the tile visible to every query of this wave (the usual case): no compare per score
    const int wave_lo = a.causal ? min(a.Lk - 1, q_wg + wave * 32 + off) : a.Lk - 1;
    // the running maximum is kept on the raw scores (scale > 0), the scale enters with the subtraction:
    // p = 2^(s * sc - max * sc) is one fused multiply-add and one v_exp_f32 per score
    float mx = m_run;
    if (t * BKV + BKV - 1 <= wave_lo) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = t * BKV + kb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          const float v = key <= key_hi ? s[kb][r] : -INFINITY;
          s[kb][r] = v;
          mx = fmaxf(mx, v);
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float msc = mx * sc;
    const float alpha = __builtin_amdgcn_exp2f((m_run - mx) * sc);   // 0 on the first tile (m_run = -inf, mx finite)
    float sum = 0.f;
    V16 pf[2][2];                                        // B operands of O^T: [32-key block][16-key step]
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const uint32_t pb = f2bf2(__builtin_amdgcn_exp2f(fmaf(s[kb][r], sc, -msc)),
                                  __builtin_amdgcn_exp2f(fmaf(s[kb][r + 1], sc, -msc)));
        sum += __uint_as_float(pb << 16) + __uint_as_float(pb & 0xffff0000u);   // normalise by what is actually multiplied
        pf[kb][r >> 3].w[(r & 7) >> 1] = pb;
      }
    sum += __shfl_xor(sum, 32, 64);
    l_run = l_run * alpha + sum;
    m_run = mx;
    if (!__all(alpha == 1.f)) {                          // the maximum of some query of this wave moved
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    // ---- O^T += V^T P ----
#pragma unroll
    for (int db = 0; db < 2; ++db) {
      const int drow = db * 32 + col;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          V16 vf;
          vf.u = *(const uint4*)&Vt[buf][drow * BKV + attn_swz(drow, (kb * 2 + s2) * 2 + half) * 8];
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.b, pf[kb][s2].b, oacc[db], 0, 0, 0);
        }
    }
    if (t + 1 < n_tiles) sstore(buf ^ 1, kr_cur, vr_cur);
    __syncthreads();
  };
  for (int t = 0; t < n_tiles; t += 2) {                 // n_tiles is the same for the whole workgroup
    step(t, krA, vrA, krB, vrB);
    if (t + 1 < n_tiles) step(t + 1, krB, vrB, krA, vrA);
  }

  // ---- O[query, d] = O^T / l : lane (query, half) holds d = 32 db + 8 g + 4 half + i ----
  if (query < a.Lq) {
    const float inv = 1.f / l_run;
    bf16_t* orow = (bf16_t*)a.o + b0 * a.o_sb0 + b1 * a.o_sb1 + (long long)query * a.o_sm;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = f2bf2(oacc[db][g * 4 + 0] * inv, oacc[db][g * 4 + 1] * inv);
        w.y = f2bf2(oacc[db][g * 4 + 2] * inv, oacc[db][g * 4 + 3] * inv);
        *(uint2*)(orow + db * 32 + g * 8 + half * 4) = w;
      }
  }
}

// Few queries against a long key / value cache (the decode step): one workgroup of 16 waves per
// (batch, head, query).  HBM-bound streaming of K and V with plain fp32 FMAs: 8 lanes share a key (16
// bytes of its 64 values each), a thread has 8 keys in flight, so one pass covers 1024 keys and the
// usual cache length costs two memory round trips (scores, values).  Probabilities are kept in LDS,
// hence Lk <= 4096.  With n_new > 0 the kernel also performs the cache append (rule R8).
constexpr int DEC_MAX_KEYS = 4096;
constexpr int DEC_THREADS = 1024, DEC_KG = DEC_THREADS / 8, DEC_U = 8;
__global__ __launch_bounds__(DEC_THREADS) void decode_attention_kernel(AttnArgs a) {
  __shared__ float prob[DEC_MAX_KEYS];
  __shared__ float red[DEC_THREADS / 64][64];
  __shared__ float stat[2 * DEC_THREADS / 64];
  constexpr int NWV = DEC_THREADS / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kg = tid >> 3, dc = tid & 7;
  const int query = blockIdx.x;
  const int b0 = blockIdx.y / a.nb1, b1 = blockIdx.y % a.nb1;
  const bf16_t* Qp = (const bf16_t*)a.q + b0 * a.q_sb0 + b1 * a.q_sb1 + (long long)query * a.q_sm;
  const bf16_t* Kp = (const bf16_t*)a.k + b0 * a.k_sb0 + b1 * a.k_sb1;
  const bf16_t* Vp = (const bf16_t*)a.v + b0 * a.v_sb0 + b1 * a.v_sb1;
  const int Lk = a.Lk + (a.step ? *a.step * a.lk_step : 0);
  const int n_keys = a.causal ? min(Lk, query + (Lk - a.Lq) + 1) : Lk;           // visible keys: 0 .. n_keys-1
  // cache append: the last n_new keys are new.  Everybody reads them from where they were produced; the
  // workgroups of query 0 copy their head's 64 values of every new row into the cache for later calls
  const int past = Lk - a.n_new;
  const bf16_t* NK = a.n_new ? (const bf16_t*)a.new_k + b1 * a.k_sb1 : nullptr;
  const bf16_t* NV = a.n_new ? (const bf16_t*)a.new_v + b1 * a.v_sb1 : nullptr;
  auto krow = [&](int t) { return (NK && t >= past) ? NK + (long long)(t - past) * a.new_k_sn : Kp + (long long)t * a.k_sn; };
  auto vrow = [&](int t) { return (NV && t >= past) ? NV + (long long)(t - past) * a.new_v_sn : Vp + (long long)t * a.v_sn; };
  if (NK && query == 0 && tid < 16 * a.n_new) {
    const int r = tid >> 4, c = tid & 15;
    if (c < 8) *(uint4*)((bf16_t*)Kp + (long long)(past + r) * a.k_sn + c * 8) = *(const uint4*)(NK + (long long)r * a.new_k_sn + c * 8);
    else *(uint4*)((bf16_t*)Vp + (long long)(past + r) * a.v_sn + (c - 8) * 8) = *(const uint4*)(NV + (long long)r * a.new_v_sn + (c - 8) * 8);
  }
  float qf[8];
  {
    V16 q; q.u = *(const uint4*)(Qp + dc * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[e] = bf2f(q.h[e]) * a.scale;
  }
  // scores
  float mx = -INFINITY;
  for (int t0 = kg; t0 < n_keys; t0 += DEC_KG * DEC_U) {
    V16 k[DEC_U];
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) k[u].u = *(const uint4*)(krow(min(t0 + u * DEC_KG, n_keys - 1)) + dc * 8);
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fmaf(qf[e], bf2f(k[u].h[e]), s);
      s = octet_sum(s);                                // the 8 lanes that share the key
      const int t = t0 + u * DEC_KG;
      if (t < n_keys) {
        if (dc == 0) prob[t] = s;
        mx = fmaxf(mx, s);
      }
    }
  }
  mx = wave_max(mx);
  if (lane == 0) stat[wave] = mx;
  __syncthreads();
  mx = stat[0];
#pragma unroll
  for (int w = 1; w < NWV; ++w) mx = fmaxf(mx, stat[w]);
  float sum = 0.f;
  for (int t = tid; t < n_keys; t += DEC_THREADS) {
    const float p = __expf(prob[t] - mx);
    prob[t] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if (lane == 0) stat[NWV + wave] = sum;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int w = 0; w < NWV; ++w) total += stat[NWV + w];
  const float inv = 1.f / total;
  // values
  float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int t0 = kg; t0 < n_keys; t0 += DEC_KG * DEC_U) {
    V16 v[DEC_U];
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) v[u].u = *(const uint4*)(vrow(min(t0 + u * DEC_KG, n_keys - 1)) + dc * 8);
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) {
      const int t = t0 + u * DEC_KG;
      const float p = t < n_keys ? prob[t] : 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = fmaf(p, bf2f(v[u].h[e]), o[e]);
    }
  }
  // the 8 key groups of a wave (lane bits 3..5) first, then the 16 waves through LDS
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    o[e] += __shfl_xor(o[e], 8, 64);
    o[e] += __shfl_xor(o[e], 16, 64);
    o[e] += __shfl_xor(o[e], 32, 64);
  }
  if (lane < 8) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][dc * 8 + e] = o[e];
  }
  __syncthreads();
  if (tid < 64) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) t += red[w][tid];
    bf16_t* orow = (bf16_t*)a.o + b0 * a.o_sb0 + b1 * a.o_sb1 + (long long)query * a.o_sm;
    orow[tid] = f2bf(t * inv);
  }
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t s) {
  if (a.Lq <= 0 || a.Lk <= 0) return hipSuccess;
  const int batch = a.nb0 * a.nb1;
  if (a.n_new > 0 && !(a.Lq <= 4 && a.Lk <= DEC_MAX_KEYS)) return hipErrorInvalidValue;   // only the few-query kernel appends
  if (a.Lq <= 4 && a.Lk <= DEC_MAX_KEYS) {
    hipLaunchKernelGGL(decode_attention_kernel, dim3(a.Lq, batch), dim3(DEC_THREADS), 0, s, a);
    return hipGetLastError();
  }
  // 128 queries per workgroup when that still gives every CU work, else 64
  const int batch8 = (batch + 7) / 8 * 8;
  if ((long long)((a.Lq + 127) / 128) * batch >= 256)
    hipLaunchKernelGGL(attention_kernel<4>, dim3(((a.Lq + 127) / 128) * batch8), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(attention_kernel<2>, dim3(((a.Lq + 63) / 64) * batch8), dim3(128), 0, s, a);
  return hipGetLastError();
}

}  // namespace sod2
