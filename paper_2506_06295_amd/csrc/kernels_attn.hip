// Bidirectional softmax attention of the recomputed query rows over ALL n cached keys and
// values of their sequence, no mask (paper complexity appendix: the 4*r^*n*d term; on refresh
// steps the query set is the whole response or the whole sequence).
//
// Queries arrive compact: sequence b owns rows [b*Mq, (b+1)*Mq) of q and out.
//
//  * k_attn_simple -- any storage type / head width: one wavefront per (query, head), scores
//                     kept in LDS, two passes.  Used for float32 models.
//  * k_attn_mfma   -- bf16, head width 128.  Flash-style online softmax on
//                     v_mfma_f32_16x16x32_bf16.  The score tile is computed transposed
//                     (S^T = K * Q^T) so that each lane ends up holding, for one query, eight
//                     keys of a 32-key block: exactly the B-operand layout of the second
//                     product O^T = V^T * P^T, so probabilities never leave registers.  K rows
//                     are read straight from global memory (64 contiguous bytes per lane);
//                     V tiles are transposed once through LDS.  The four wavefronts of a
//                     workgroup are arranged as QW query groups x KW key ranges: with few
//                     queries (adaptive steps) the key range is split for parallelism and the
//                     partial results are merged through LDS at the end.
#include "common.hpp"

namespace dllmc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

namespace {

template <typename T>
__global__ __launch_bounds__(64) void k_attn_simple(const T* __restrict__ q, int Mq,
                                                    const T* __restrict__ kc,
                                                    const T* __restrict__ vc, int n, int H_q,
                                                    int H_kv, int d_h, T* __restrict__ out) {
  extern __shared__ float sm[];
  float* qs = sm;        // [d_h]
  float* sc = sm + d_h;  // [n]
  const int i = blockIdx.x, a = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x;
  const int d_q = H_q * d_h, d_kv = H_kv * d_h;
  const int kv = a / (H_q / H_kv);
  const T* qr = q + (static_cast<size_t>(b) * Mq + i) * d_q + a * d_h;
  const T* K = kc + static_cast<size_t>(b) * n * d_kv + kv * d_h;
  const T* V = vc + static_cast<size_t>(b) * n * d_kv + kv * d_h;
  const float scale = 1.0f / sqrtf(static_cast<float>(d_h));
  for (int t = lane; t < d_h; t += 64) qs[t] = ldf(qr + t);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < n; j += 64) {
    const T* kr = K + static_cast<size_t>(j) * d_kv;
    float acc = 0.f;
    for (int t = 0; t < d_h; ++t) acc = fmaf(qs[t], ldf(kr + t), acc);
    acc *= scale;
    sc[j] = acc;
    mx = fmaxf(mx, acc);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < n; j += 64) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  __syncthreads();
  T* o = out + (static_cast<size_t>(b) * Mq + i) * d_q + a * d_h;
  for (int t = lane; t < d_h; t += 64) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) acc = fmaf(sc[j], ldf(V + static_cast<size_t>(j) * d_kv + t), acc);
    stf(o + t, acc / sum);
  }
}

constexpr int kDH = 128;     // head width of the MFMA kernel
constexpr int kVtStride = 40;  // 32 keys + 8 pad (bf16 elements) per transposed V row

template <int QW, int KW>
__global__ __launch_bounds__(256) void k_attn_mfma(const bf16_t* __restrict__ q, int Mq,
                                                   const bf16_t* __restrict__ kc,
                                                   const bf16_t* __restrict__ vc, int n, int H_q,
                                                   int H_kv, bf16_t* __restrict__ out) {
  static_assert(QW * KW == 4, "four wavefronts per workgroup");
  constexpr int QT = 16 * QW;  // queries per workgroup
  // V^T tiles during the key loop, reused for the merge buffers afterwards
  constexpr int kVtBytes = KW * kDH * kVtStride * 2;
  constexpr int kMergeBytes = 4 * 16 * (kDH + 2) * 4;
  constexpr int kSmem = kVtBytes > kMergeBytes ? kVtBytes : kMergeBytes;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kSmem];

  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int ln = lane % 16, lg = lane / 16;
  const int qw = wave % QW, kw = wave / QW;
  const int a = blockIdx.y, b = blockIdx.z;
  const int d_q = H_q * kDH, d_kv = H_kv * kDH;
  const int kv = a / (H_q / H_kv);
  const int i0 = blockIdx.x * QT;  // first query of this workgroup inside the sequence

  const bf16_t* K = kc + static_cast<size_t>(b) * n * d_kv + kv * kDH;
  const bf16_t* V = vc + static_cast<size_t>(b) * n * d_kv + kv * kDH;

  // Q fragments (B operand of S^T = K Q^T): lane (n = query ln, g = lg) holds dims 32g+8c..+8
  int qi = i0 + qw * 16 + ln;
  if (qi >= Mq) qi = Mq - 1;  // clamp: padded queries compute a duplicate that is never stored
  const bf16_t* qr = q + (static_cast<size_t>(b) * Mq + qi) * d_q + a * kDH + lg * 32;
  bf16x8 qf[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) qf[c] = *reinterpret_cast<const bf16x8*>(qr + c * 8);

  const float sl2e = 1.4426950408889634f / sqrtf(static_cast<float>(kDH));  // scale * log2(e)
  float m_run = -INFINITY;  // running maximum of the scaled scores (base-2 units), per query
  float l_run = 0.f;        // this lane's share of the running denominator
  f32x4 o_acc[8];           // O^T: dims db*16 + 4*lg + i, query ln
#pragma unroll
  for (int db = 0; db < 8; ++db) o_acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nblk = (n + 31) / 32;
  const int per = (nblk + KW - 1) / KW;  // 32-key blocks per key range (same trip count for all)
  bf16_t* Vt = reinterpret_cast<bf16_t*>(smem) + kw * kDH * kVtStride;
  const int gtid = qw * 64 + lane;  // thread index inside this key range's group

  for (int it = 0; it < per; ++it) {
    const int kb = kw * per + it;
    const int key0 = kb * 32;
    __syncthreads();
    // stage V[key0 .. key0+32) transposed: Vt[dim][key]
    for (int e = gtid; e < 32 * 16; e += 64 * QW) {
      const int key = e / 16, c = e % 16;
      int kr = key0 + key;
      if (kr >= n) kr = n - 1;  // masked below; any finite value will do
      const uint4 raw = *reinterpret_cast<const uint4*>(V + static_cast<size_t>(kr) * d_kv + c * 8);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        Vt[(c * 8 + 2 * j) * kVtStride + key] = static_cast<bf16_t>(w[j] & 0xffffu);
        Vt[(c * 8 + 2 * j + 1) * kVtStride + key] = static_cast<bf16_t>(w[j] >> 16);
      }
    }
    // scores of the two 16-key halves: S^T[key][query]
    f32x4 st[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      int kr = key0 + sb * 16 + ln;
      if (kr >= n) kr = n - 1;
      const bf16_t* kp = K + static_cast<size_t>(kr) * d_kv + lg * 32;
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kp + c * 8);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[c], acc, 0, 0, 0);
      }
      st[sb] = acc;
    }
    // lane holds keys key0 + sb*16 + 4*lg + i of query ln
    float p[8];
    float mx = -INFINITY;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = key0 + sb * 16 + 4 * lg + i;
        const float v = key < n ? st[sb][i] * sl2e : -INFINITY;
        p[sb * 4 + i] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = exp2f(m_run - m_use);  // 0 while nothing has been seen yet
    float psum = 0.f;
    bf16x8 pf;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float e = exp2f(p[t] - m_use);
      psum += e;
      pf[t] = static_cast<__bf16>(e);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      o_acc[db][0] *= alpha;
      o_acc[db][1] *= alpha;
      o_acc[db][2] *= alpha;
      o_acc[db][3] *= alpha;
    }
    __syncthreads();
    // O^T[dim][query] += V^T[dim][key] * P^T[key][query]
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const bf16_t* vr = Vt + (db * 16 + ln) * kVtStride + 4 * lg;
      const uint2 lo = *reinterpret_cast<const uint2*>(vr);
      const uint2 hi = *reinterpret_cast<const uint2*>(vr + 16);
      const uint4 both = make_uint4(lo.x, lo.y, hi.x, hi.y);
      const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
      o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, o_acc[db], 0, 0, 0);
    }
  }

  // merge the KW key ranges and normalise
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  __syncthreads();
  float* mo = reinterpret_cast<float*>(smem);  // [4 waves][16 queries][kDH + 2]: O^T, then m, l
  {
    float* w = mo + (wave * 16 + ln) * (kDH + 2);
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) w[db * 16 + 4 * lg + i] = o_acc[db][i];
    if (lg == 0) {
      w[kDH] = m_run;
      w[kDH + 1] = l_run;
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < QT * kDH; e += 256) {
    const int ql = e / kDH, dim = e % kDH;  // query inside the workgroup tile
    const int qwi = ql / 16, qn = ql % 16;
    const int iq = i0 + ql;
    if (iq >= Mq) continue;
    float M = -INFINITY;
#pragma unroll
    for (int r = 0; r < KW; ++r) M = fmaxf(M, mo[((r * QW + qwi) * 16 + qn) * (kDH + 2) + kDH]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int r = 0; r < KW; ++r) {
      const float* w = mo + ((r * QW + qwi) * 16 + qn) * (kDH + 2);
      const float f = w[kDH] == -INFINITY ? 0.f : exp2f(w[kDH] - M);
      L += w[kDH + 1] * f;
      O += w[dim] * f;
    }
    out[(static_cast<size_t>(b) * Mq + iq) * d_q + a * kDH + dim] = f32_to_bf16(O / L);
  }
}

}  // namespace

bool attention_supported(int dtype, int d_h, int n) {
  if (dtype == 1 && d_h == kDH) return true;
  return static_cast<size_t>(d_h + n) * sizeof(float) <= 60 * 1024;
}

void launch_attention(int dtype, const void* q, int B, int Mq, const void* k_cache,
                      const void* v_cache, int n, int H_q, int H_kv, int d_h, void* out,
                      hipStream_t st) {
  if (B <= 0 || Mq <= 0 || n <= 0) return;
  if (dtype == 1 && d_h == kDH) {
    const bf16_t* qq = static_cast<const bf16_t*>(q);
    const bf16_t* kk = static_cast<const bf16_t*>(k_cache);
    const bf16_t* vv = static_cast<const bf16_t*>(v_cache);
    bf16_t* oo = static_cast<bf16_t*>(out);
    if (static_cast<long>(B) * ((Mq + 63) / 64) * H_q >= 256) {
      hipLaunchKernelGGL((k_attn_mfma<4, 1>), dim3((Mq + 63) / 64, H_q, B), dim3(256), 0, st, qq, Mq,
                         kk, vv, n, H_q, H_kv, oo);
    } else {
      hipLaunchKernelGGL((k_attn_mfma<1, 4>), dim3((Mq + 15) / 16, H_q, B), dim3(256), 0, st, qq, Mq,
                         kk, vv, n, H_q, H_kv, oo);
    }
    return;
  }
  const size_t lds = static_cast<size_t>(d_h + n) * sizeof(float);
  if (dtype == 1)
    hipLaunchKernelGGL(k_attn_simple<bf16_t>, dim3(Mq, H_q, B), dim3(64), lds, st,
                       static_cast<const bf16_t*>(q), Mq, static_cast<const bf16_t*>(k_cache),
                       static_cast<const bf16_t*>(v_cache), n, H_q, H_kv, d_h,
                       static_cast<bf16_t*>(out));
  else
    hipLaunchKernelGGL(k_attn_simple<float>, dim3(Mq, H_q, B), dim3(64), lds, st,
                       static_cast<const float*>(q), Mq, static_cast<const float*>(k_cache),
                       static_cast<const float*>(v_cache), n, H_q, H_kv, d_h,
                       static_cast<float*>(out));
}

}  // namespace dllmc
