// Bidirectional softmax attention of the recomputed query rows over ALL n cached keys and
// values of their sequence, no mask (paper complexity appendix: the 4*r^*n*d term; on refresh
// steps the query set is the whole response or the whole sequence).
//
// Queries arrive compact: sequence b owns rows [b*Mq, (b+1)*Mq) of q and out.
//
//  * k_attn_simple -- any storage type / head width: one wavefront per (query, head), scores
//                     kept in LDS, two passes.  Used for float32 models.
//  * k_attn_mfma / k_attn_walk -- bf16, head width 128.  Flash-style online softmax on
//                     v_mfma_f32_16x16x32_bf16.  The score tile is computed transposed
//                     (S^T = K * Q^T) so that each lane ends up holding, for one query, eight
//                     keys of a 32-key block: exactly the B-operand layout of the second
//                     product O^T = V^T * P^T, so probabilities never leave registers.
//                     V tiles are transposed once per workgroup through LDS and shared by
//                     its four 16-query wavefronts.  With few queries (adaptive steps) the
//                     key range is split over workgroups and k_attn_merge combines the
//                     partial results in key-range order.  k_attn_mfma handles key ranges of
//                     up to three blocks (all of it fetched into registers before the first
//                     use), k_attn_walk longer ones (K and V tiles staged global -> LDS
//                     several blocks ahead).
#include "common.hpp"

namespace dllmc {


namespace {

template <typename T>
__global__ __launch_bounds__(64) void k_attn_simple(const T* __restrict__ q, int Mq,
                                                    const T* __restrict__ kc,
                                                    const T* __restrict__ vc, int n, int H_q,
                                                    int H_kv, int d_h, T* __restrict__ out,
                                                    const int* __restrict__ rmap) {
  extern __shared__ float sm[];
  float* qs = sm;        // [d_h]
  float* sc = sm + d_h;  // [n]
  const int i = blockIdx.x, a = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x;
  const int d_q = H_q * d_h, d_kv = H_kv * d_h;
  const int kv = a / (H_q / H_kv);
  const T* qr = q + (static_cast<size_t>(b) * Mq + i) * d_q + a * d_h;
  // row j of this sequence in the cache tensors (the row map's entry in the paged layout)
  auto crow = [&](int j) { return static_cast<size_t>(rmap ? rmap[b * n + j] : b * n + j); };
  const T* K = kc + kv * d_h;
  const T* V = vc + kv * d_h;
  const float scale = 1.0f / sqrtf(static_cast<float>(d_h));
  for (int t = lane; t < d_h; t += 64) qs[t] = ldf(qr + t);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < n; j += 64) {
    const T* kr = K + crow(j) * d_kv;
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
    for (int j = 0; j < n; ++j) acc = fmaf(sc[j], ldf(V + crow(j) * d_kv + t), acc);
    stf(o + t, acc / sum);
  }
}

constexpr int kDH = 128;       // head width of the MFMA kernel
constexpr int kVtStride = 40;  // 32 keys + 8 pad (bf16 elements) per transposed V row
constexpr int kQT = 64;        // queries per workgroup: four wavefronts x 16
constexpr int kPreload = 3;    // key ranges of up to this many 32-key blocks are fetched whole
constexpr int kMaxKeySplit = 16;

// One 32-key block for a wavefront's 16 queries: scores S^T = K Q^T, running softmax (base 2),
// O^T += V^T P^T.  kf: K fragments (lane: key sb*16 + ln, dims 32c + 8lg .. +8); qf: Q fragments
// (lane: query ln, same dims); vt: the block's V tile transposed, [dim][VS keys] (SWZ: with the
// key pairs of a row permuted, see k_attn_mfma).
template <int VS, bool SWZ>
__device__ __forceinline__ void attn_block(const bf16x8 (&kf)[2][4], const bf16x8 (&qf)[4],
                                           const bf16_t* vt, int key0, int n, int ln, int lg,
                                           float sl2e, float& m_run, float& l_run,
                                           f32x4 (&o_acc)[8]) {
  f32x4 st[2];
#pragma unroll
  for (int sb = 0; sb < 2; ++sb) {
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[sb][c], qf[c], acc, 0, 0, 0);
    st[sb] = acc;
  }
  // lane holds keys key0 + sb*16 + 4*lg + i of query ln
  float p[8];
  float mx = -INFINITY;
  if (key0 + 32 <= n) {  // the whole block lies inside the sequence (wavefront-uniform)
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[sb * 4 + i] = st[sb][i];
        mx = fmaxf(mx, st[sb][i]);
      }
  } else {
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = key0 + sb * 16 + 4 * lg + i;
        const float v = key < n ? st[sb][i] : -INFINITY;
        p[sb * 4 + i] = v;
        mx = fmaxf(mx, v);
      }
  }
  mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  // running maximum of the scaled scores (the scale is positive, so it commutes with the max)
  const float m_new = fmaxf(m_run, mx * sl2e);
  const float m_use = m_new == -INFINITY ? 0.f : m_new;
  // The accumulators are rescaled only in the blocks in which some query's maximum moved
  // (wavefront-uniform test): with alpha == 1 for every lane the multiplications change nothing.
  if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);  // 0 while nothing has been seen yet
    l_run *= alpha;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      o_acc[db][0] *= alpha;
      o_acc[db][1] *= alpha;
      o_acc[db][2] *= alpha;
      o_acc[db][3] *= alpha;
    }
  }
  // probabilities as a bf16 pair (high part + remainder): the second product then carries
  // ~16 bits of each probability instead of 8
  // (the hardware's 2^x as it is: the arguments are <= 0, and results below the normal range, which
  // it flushes to zero, are far below anything a bf16 pair can carry)
  float psum = 0.f;
  bf16x8 pf, pl;
#pragma unroll
  for (int t = 0; t < 8; t += 2) {
    const float e0 = __builtin_amdgcn_exp2f(fmaf(p[t], sl2e, -m_use));
    const float e1 = __builtin_amdgcn_exp2f(fmaf(p[t + 1], sl2e, -m_use));
    psum += e0;
    psum += e1;
    const uint32_t hi = pack_bf16x2(e0, e1);
    reinterpret_cast<uint32_t*>(&pf)[t / 2] = hi;
    reinterpret_cast<uint32_t*>(&pl)[t / 2] =
        pack_bf16x2(e0 - __uint_as_float(hi << 16), e1 - __uint_as_float(hi & 0xffff0000u));
  }
  l_run += psum;
  // O^T[dim][query] += V^T[dim][key] * P^T[key][query]
#pragma unroll
  for (int db = 0; db < 8; ++db) {
    // SWZ: key pair p of the rows of dim block db sits at pair position p ^ 2*db
    const bf16_t* vrow = vt + (db * 16 + ln) * VS;
    const uint2 lo = *reinterpret_cast<const uint2*>(vrow + (SWZ ? (4 * lg) ^ (4 * db) : 4 * lg));
    const uint2 hi =
        *reinterpret_cast<const uint2*>(vrow + (SWZ ? (16 + 4 * lg) ^ (4 * db) : 16 + 4 * lg));
    const uint4 both = make_uint4(lo.x, lo.y, hi.x, hi.y);
    const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
    o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, o_acc[db], 0, 0, 0);
    o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pl, o_acc[db], 0, 0, 0);
  }
}

// End of a key range for query iq (lane's column of O^T): with KS == 1 the normalised output row,
// otherwise the un-normalised partial (O, m, l) of range ks for k_attn_merge.
__device__ __forceinline__ void attn_finish(const f32x4 (&o_acc)[8], float m_run, float l_run, int iq,
                                            int Mq, int b, int a, int ks, int KS, int H_q, int lg,
                                            bf16_t* __restrict__ out, float* __restrict__ part) {
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (iq >= Mq) return;
  const int d_q = H_q * kDH;
  if (KS == 1) {
    const float inv_l = 1.0f / l_run;
    bf16_t* o = out + (static_cast<size_t>(b) * Mq + iq) * d_q + a * kDH;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      uint2 t;
      t.x = static_cast<uint32_t>(f32_to_bf16(o_acc[db][0] * inv_l)) |
            (static_cast<uint32_t>(f32_to_bf16(o_acc[db][1] * inv_l)) << 16);
      t.y = static_cast<uint32_t>(f32_to_bf16(o_acc[db][2] * inv_l)) |
            (static_cast<uint32_t>(f32_to_bf16(o_acc[db][3] * inv_l)) << 16);
      *reinterpret_cast<uint2*>(o + db * 16 + 4 * lg) = t;
    }
  } else {
    // part[((b*Mq + iq)*H_q + a)*KS + ks][kDH + 2]
    float* w = part + ((static_cast<size_t>(b) * Mq + iq) * H_q + a) * KS * (kDH + 2) +
               static_cast<size_t>(ks) * (kDH + 2);
#pragma unroll
    for (int db = 0; db < 8; ++db)
      *reinterpret_cast<float4*>(w + db * 16 + 4 * lg) =
          make_float4(o_acc[db][0], o_acc[db][1], o_acc[db][2], o_acc[db][3]);
    if (lg == 0) {
      w[kDH] = m_run;
      w[kDH + 1] = l_run;
    }
  }
}

// Workgroups are handed to the 8 XCDs round-robin in launch order and each XCD has its own L2.
// The launch is one-dimensional: a "slot" is (query tile, KV head, sequence, key range), and the G
// query heads that share the slot's KV head run back to back on one XCD, so the slot's K and V
// blocks are fetched into that L2 once instead of once per query head (grouped KV heads: 7 x
// fewer fetches for 28 / 4 heads).  Slots beyond the last multiple of 8 are walked in order.
struct AttnWork { int qtile, a, b, ks; };
__device__ __forceinline__ AttnWork attn_work(int qt, int H_q, int H_kv, int KS) {
  const int G = H_q / H_kv;
  const int n_slots = gridDim.x / G;
  const int lin = blockIdx.x;
  const int n8 = n_slots & ~7;
  int slot, j;
  if (lin < n8 * G) {
    const int xcd = lin & 7, idx = lin >> 3;
    slot = (idx / G) * 8 + xcd;
    j = idx % G;
  } else {
    const int rest = lin - n8 * G;
    slot = n8 + rest / G;
    j = rest % G;
  }
  // slot = ((b * KS + ks) * H_kv + kvh) * qt + qtile
  AttnWork w;
  w.qtile = slot % qt;
  const int kvh = (slot / qt) % H_kv;
  const int z = slot / (qt * H_kv);
  w.b = z / KS;
  w.ks = z % KS;
  w.a = kvh * G + j;
  return w;
}

// Workgroup = 4 wavefronts = 4 tiles of 16 queries of one head and one sequence; the slot
// enumerates (sequence, key range).  All four wavefronts use the same 32-key blocks, so a V
// tile is transposed through LDS once per workgroup.  With KS == 1 the normalised output is
// written; otherwise the un-normalised partial (O, m, l) of this key range goes to `part` for
// k_attn_merge.
// k_attn_mfma: key ranges of at most kPreload blocks (the launcher guarantees it: split keys of
// an adaptive step).  Every K fragment and V tile of the range is requested before the first
// one is used, so the range costs one trip to memory instead of one per block.
// V transposition: thread = (key pair kp, 16-byte chunk ch) loads the chunk of keys 2kp and 2kp+1
// (16 consecutive lanes read one key's 256 bytes) and writes, per dim, one 32-bit word holding
// both keys at pair position kp ^ (ch & 14) of the dim's row: the 16 lanes of a key pair then
// hit 16 different banks (lanes along the dims with 16-bit stores spend 7 of 8 LDS cycles on
// bank conflicts), and ch & 14 = 2 * (dim / 16) is the same for all rows of a dim block, so the
// reader undoes it with a constant.
// PAGED: the key rows are looked up in the row map (a compile-time switch: the flat layout's
// code, whose loads must all go out before the first use, stays exactly as it is without it).
template <bool PAGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void k_attn_mfma(
    const bf16_t* __restrict__ q, int Mq, const bf16_t* __restrict__ kc,
    const bf16_t* __restrict__ vc, int n, int H_q, int H_kv, int KS, bf16_t* __restrict__ out,
    float* __restrict__ part, const int* __restrict__ rmap) {
  __shared__ __attribute__((aligned(16))) bf16_t Vt[kPreload][kDH * kVtStride];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;  // scalar
  const int ln = lane % 16, lg = lane / 16;
  const AttnWork wk = attn_work((Mq + kQT - 1) / kQT, H_q, H_kv, KS);
  const int a = wk.a, b = wk.b, ks = wk.ks;
  const int d_q = H_q * kDH, d_kv = H_kv * kDH;
  const int kv = a / (H_q / H_kv);
  const int i0 = wk.qtile * kQT + wave * 16;  // first query of this wavefront

  // key row j of this sequence: cache row b * n + j, or the row map's entry (paged layout)
  const bf16_t* K = kc + kv * kDH;
  const bf16_t* V = vc + kv * kDH;
  const int seq0 = b * n;

  // Q fragments (B operand of S^T = K Q^T): lane (query ln, group lg) holds dims 32c+8lg..+8
  int qi = i0 + ln;
  if (qi >= Mq) qi = Mq - 1;  // padded queries compute a duplicate that is never stored
  const bf16_t* qr = q + (static_cast<size_t>(b) * Mq + qi) * d_q + a * kDH + lg * 8;
  bf16x8 qf[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) qf[c] = *reinterpret_cast<const bf16x8*>(qr + c * 32);

  const float sl2e = 1.4426950408889634f / sqrtf(static_cast<float>(kDH));  // scale * log2(e)
  float m_run = -INFINITY;  // running maximum of the scaled scores (base 2), per query
  float l_run = 0.f;        // this lane's share of the running denominator
  f32x4 o_acc[8];           // O^T: dims db*16 + 4*lg + i, query ln
#pragma unroll
  for (int db = 0; db < 8; ++db) o_acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nblk = (n + 31) / 32;
  const int per = (nblk + KS - 1) / KS;
  const int blk0 = ks * per;
  const int blk1 = min(nblk, blk0 + per);
  const int nb = blk1 - blk0;

  if (nb > 0) {
    const int kp = threadIdx.x / 16, ch = threadIdx.x % 16;
    bf16x8 kall[kPreload][2][4];
    uint4 vall[kPreload][2];
#pragma unroll
    for (int j = 0; j < kPreload; ++j) {
      const int blk = min(blk0 + j, blk1 - 1);  // blocks past the range repeat the last one, unused
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        int kr = blk * 32 + sb * 16 + ln;
        if (kr >= n) kr = n - 1;  // masked in the scores; any finite value will do
        const size_t cr = static_cast<size_t>(PAGED ? rmap[seq0 + kr] : seq0 + kr);
        const bf16_t* kptr = K + cr * d_kv + lg * 8;
#pragma unroll
        for (int c = 0; c < 4; ++c) kall[j][sb][c] = *reinterpret_cast<const bf16x8*>(kptr + c * 32);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        int kr = blk * 32 + 2 * kp + h;
        if (kr >= n) kr = n - 1;
        const size_t cr = static_cast<size_t>(PAGED ? rmap[seq0 + kr] : seq0 + kr);
        vall[j][h] = *reinterpret_cast<const uint4*>(V + cr * d_kv + ch * 8);
      }
    }
#pragma unroll
    for (int j = 0; j < kPreload; ++j) {
      uint32_t* vt32 = reinterpret_cast<uint32_t*>(Vt[j]);
      const uint32_t e0[4] = {vall[j][0].x, vall[j][0].y, vall[j][0].z, vall[j][0].w};
      const uint32_t e1[4] = {vall[j][1].x, vall[j][1].y, vall[j][1].z, vall[j][1].w};
      const int pos = kp ^ (ch & 14);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int dim = ch * 8 + 2 * t;
        vt32[(dim * kVtStride) / 2 + pos] = (e0[t] & 0xffffu) | (e1[t] << 16);
        vt32[((dim + 1) * kVtStride) / 2 + pos] = (e0[t] >> 16) | (e1[t] & 0xffff0000u);
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kPreload; ++j)
      if (j < nb)
        attn_block<kVtStride, true>(kall[j], qf, Vt[j], (blk0 + j) * 32, n, ln, lg, sl2e, m_run, l_run,
                                    o_acc);
  }
  attn_finish(o_acc, m_run, l_run, i0 + ln, Mq, b, a, ks, KS, H_q, lg, out, part);
}

// ---- long key ranges -----------------------------------------------------------------
// k_attn_walk: the same tiling and arithmetic as k_attn_mfma for key ranges of more than kPreload
// blocks (many queries, or long sequences).  A block-by-block walk that fetches one block ahead
// into registers is bound by the memory latency of every block; here the K and V tiles of a
// block go from global memory straight into LDS (global_load_lds: no registers held while they
// are in flight), kWalkStages - 1 blocks ahead.  K fragments are then read from LDS (slot =
// chunk ^ (key % 16), so the 16 keys of a fragment read hit 16 different slots); the V tile is
// read back row-wise and written transposed into Vt as in the other kernel.
constexpr int kWalkStages = 4;
constexpr int kVtStrideW = 36;  // 32 keys + 4 pad: rows of 8 dims apart start 16 banks apart

// (The body is a function of its own with restrict-qualified parameters, inlined into the kernel:
// only then does the compiler keep the global -> LDS loads of the later stages in flight across
// the LDS reads of the landed one; written directly into the kernel it waits for every load in
// flight before each of those reads, and the walk is bound by one memory latency per block.  The
// waits that order the loads against the reads are the explicit ones below.)
template <bool PAGED>
__device__ __forceinline__ void attn_walk_body(const bf16_t* __restrict__ q, int Mq,
                                               const bf16_t* __restrict__ kc,
                                               const bf16_t* __restrict__ vc, int n, int H_q,
                                               int H_kv, int KS, bf16_t* __restrict__ out,
                                               float* __restrict__ part,
                                               const int* __restrict__ rmap) {
  // [stage][K tile, V tile][32 keys][16 slots of 16 bytes], then the transposed V tile.  One LDS
  // object on purpose: with two, the compiler cannot tell reads of the landed stage from the
  // loads in flight into the other stages and waits for all of those before every read.
  constexpr int kTileVecs = kWalkStages * 2 * 32 * 16;
  __shared__ __attribute__((aligned(1024))) uint4 smem[kTileVecs + kDH * kVtStrideW * 2 / 16];
  uint4 (*tiles)[2][32 * 16] = reinterpret_cast<uint4 (*)[2][32 * 16]>(smem);
  bf16_t* Vt = reinterpret_cast<bf16_t*>(smem + kTileVecs);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;  // scalar
  const int ln = lane % 16, lg = lane / 16;
  const AttnWork wk = attn_work((Mq + kQT - 1) / kQT, H_q, H_kv, KS);
  const int a = wk.a, b = wk.b, ks = wk.ks;
  const int d_q = H_q * kDH, d_kv = H_kv * kDH;
  const int kv = a / (H_q / H_kv);
  const int i0 = wk.qtile * kQT + wave * 16;

  const bf16_t* K = kc + kv * kDH;
  const bf16_t* V = vc + kv * kDH;
  const int seq0 = b * n;

  int qi = i0 + ln;
  if (qi >= Mq) qi = Mq - 1;  // padded queries compute a duplicate that is never stored
  const bf16_t* qr = q + (static_cast<size_t>(b) * Mq + qi) * d_q + a * kDH + lg * 8;
  bf16x8 qf[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) qf[c] = *reinterpret_cast<const bf16x8*>(qr + c * 32);

  const float sl2e = 1.4426950408889634f / sqrtf(static_cast<float>(kDH));
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 o_acc[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) o_acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nblk = (n + 31) / 32;
  const int per = (nblk + KS - 1) / KS;
  const int blk0 = ks * per;
  const int blk1 = min(nblk, blk0 + per);
  const int nb = blk1 - blk0;

  if (nb > 0) {
    // loader: a tile is 8 wavefront instructions of 4 keys x 256 bytes; wavefront w issues
    // instructions 2w and 2w+1 of the K and of the V tile.  Lane l: key 4q + l/16, slot l%16.
    // LDS slot l%16 of a key's row holds chunk slot ^ (key % 16) of K (the 16 keys of a
    // fragment read hit 16 slots) and chunk slot ^ (key/2 % 16) of V (so do the 16 key pairs
    // of the transposition)
    int lkey[2], kchunk[2], vchunk[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      lkey[j] = 4 * (2 * wave + j) + lane / 16;
      kchunk[j] = (lane % 16) ^ (lkey[j] % 16);
      vchunk[j] = (lane % 16) ^ ((lkey[j] >> 1) % 16);
    }
    // cache rows of this lane's two keys of a block: the rows themselves, or (paged layout) the
    // row map's entries, looked up one block before the block's loads are issued
    auto rows_of = [&](int blk, int (&cr)[2]) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        int kr = blk * 32 + lkey[j];
        if (kr >= n) kr = n - 1;  // masked in the scores; any finite value will do
        cr[j] = PAGED ? rmap[seq0 + kr] : seq0 + kr;
      }
    };
    auto issue = [&](const int (&cr)[2], int stage) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const size_t row = static_cast<size_t>(cr[j]) * d_kv;
        __builtin_amdgcn_global_load_lds(K + row + kchunk[j] * 8, &tiles[stage][0][(2 * wave + j) * 64],
                                         16, 0, 0);
        __builtin_amdgcn_global_load_lds(V + row + vchunk[j] * 8, &tiles[stage][1][(2 * wave + j) * 64],
                                         16, 0, 0);
      }
    };
    // blocks past the range repeat the last one (never used): the number of loads in flight
    // stays the same in every iteration
    int cr_next[2];
#pragma unroll
    for (int s = 0; s < kWalkStages - 1; ++s) {
      rows_of(min(blk0 + s, blk1 - 1), cr_next);
      issue(cr_next, s);
    }
    rows_of(min(blk0 + kWalkStages - 1, blk1 - 1), cr_next);

    // V transposition: thread = (key pair kp, 16-byte chunk vch); it reads the chunk of keys 2kp
    // and 2kp+1 and writes, per dim, one 32-bit word holding both keys.  Consecutive lanes write
    // consecutive words of a Vt row and the four chunks of a wavefront sit 16 banks apart (row
    // stride 36 elements), so the writes are free of bank conflicts; 16-bit stores with lanes
    // along the dims spend 7 of 8 LDS cycles on conflicts.
    const int kp = threadIdx.x % 16, vch = threadIdx.x / 16;
    uint32_t* vt32 = reinterpret_cast<uint32_t*>(Vt);
    for (int i = 0; i < nb; ++i) {
      const int stage = i % kWalkStages;
      // 4 loads per block and wavefront, kWalkStages - 1 blocks in flight: the oldest has landed
      // (paged layout: the two row-map lookups of the block after those are in flight as well)
      wait_vmcnt<4 * (kWalkStages - 2) + (PAGED ? 2 : 0)>();
      // everybody's loads of block i have landed, and everybody is done with block i - 1: its
      // stage and Vt may be overwritten
      __builtin_amdgcn_s_barrier();
      // The lookups for the block after the one issued now go out first: they are then older
      // than this block's loads, and waiting for them in the next iteration leaves those in flight.
      const int cr_use[2] = {cr_next[0], cr_next[1]};
      rows_of(min(blk0 + i + kWalkStages, blk1 - 1), cr_next);
      issue(cr_use, (i + kWalkStages - 1) % kWalkStages);
      {
        const uint4 r0 = tiles[stage][1][(2 * kp) * 16 + (vch ^ kp)];
        const uint4 r1 = tiles[stage][1][(2 * kp + 1) * 16 + (vch ^ kp)];
        const uint32_t e0[4] = {r0.x, r0.y, r0.z, r0.w}, e1[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int dim = vch * 8 + 2 * j;
          vt32[(dim * kVtStrideW) / 2 + kp] = (e0[j] & 0xffffu) | (e1[j] << 16);
          vt32[((dim + 1) * kVtStrideW) / 2 + kp] = (e0[j] >> 16) | (e1[j] & 0xffff0000u);
        }
      }
      // K fragments of this wavefront: key sb*16 + ln, dims 32c + 8lg .. +8 = chunk 4c + lg
      bf16x8 kf[2][4];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          kf[sb][c] = __builtin_bit_cast(bf16x8, tiles[stage][0][(sb * 16 + ln) * 16 + ((4 * c + lg) ^ ln)]);
      __builtin_amdgcn_s_waitcnt(0xC07F);  // LDS writes of Vt done (lgkmcnt 0); global loads stay in flight
      __builtin_amdgcn_s_barrier();
      attn_block<kVtStrideW, false>(kf, qf, Vt, (blk0 + i) * 32, n, ln, lg, sl2e, m_run, l_run, o_acc);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // the repeated loads past the range, before the LDS goes away
  }
  attn_finish(o_acc, m_run, l_run, i0 + ln, Mq, b, a, ks, KS, H_q, lg, out, part);
}

template <bool PAGED>
__global__ __launch_bounds__(256) void k_attn_walk(const bf16_t* __restrict__ q, int Mq,
                                                   const bf16_t* __restrict__ kc,
                                                   const bf16_t* __restrict__ vc, int n, int H_q,
                                                   int H_kv, int KS, bf16_t* __restrict__ out,
                                                   float* __restrict__ part,
                                                   const int* __restrict__ rmap) {
  attn_walk_body<PAGED>(q, Mq, kc, vc, n, H_q, H_kv, KS, out, part, rmap);
}

// ---- many queries --------------------------------------------------------------------
// k_attn_tile: refresh steps and batched sequences, where a (sequence, head) has hundreds of
// queries and the work is bound by the matrix cores, the LDS and the softmax arithmetic rather
// than by the K/V stream.  Against k_attn_walk: a wavefront owns 32 queries (two 16-query
// column blocks), so every K and V fragment read from LDS feeds two MFMAs; blocks are 64 keys
// (one barrier per 64 keys instead of two per 32); and V is never transposed through LDS: the
// A operand of O^T += V^T P^T (lane: one dim, eight keys) comes straight out of the row-major V
// tile with ds_read_b64_tr_b16.  That instruction works on groups of 16 lanes: lane 4t + q of a
// group passes the address of four consecutive 16-bit elements -- elements 4q .. 4q+3 of row t of
// a 4 x 16 block -- and lane i of the group receives element i of rows 0..3 (layout checked on the
// hardware).  Here a group's rows are the keys 4*lg .. 4*lg+3 of a 16-key sub-block and the 16
// elements a dim block, so lane (ln, lg) gets keys 4*lg .. +3 at dim db*16 + ln: with two such reads
// (sub-blocks 2h and 2h+1) exactly the keys whose probabilities the lane holds after the first
// product.  Two LDS stages of K tile + V tile (64 KB, two workgroups per CU); the tiles arrive by
// global_load_lds with slot = chunk ^ (key % 16) for both, which keeps the K fragment reads (16
// keys, one chunk each) and the transposing reads (16 keys x 32 bytes) spread over all banks.
// Workgroup order of k_attn_tile: a "group" is everything that reads the same K and V rows -- the
// query tiles of all query heads of one KV head, for one sequence and key range.  Groups go to the
// XCDs round-robin and an XCD works through its groups one after the other, so the group's K/V
// blocks are fetched into that XCD's L2 once and then hit by its other workgroups (with the tiles
// of a head dealt over all XCDs, every XCD streams every head's keys: 2.7 GB from beyond L2 for the
// 4608-row refresh, 36 times the K/V cache).  Groups beyond the last multiple of 8 are walked in
// launch order.
__device__ __forceinline__ AttnWork attn_work_tile(int qt, int H_q, int H_kv, int KS) {
  const int G = H_q / H_kv;
  const int W = G * qt;  // workgroups per group
  const int n_groups = gridDim.x / W;
  const int lin = blockIdx.x;
  const int n8 = n_groups & ~7;
  int group, w;
  if (lin < n8 * W) {
    const int xcd = lin & 7, idx = lin >> 3;
    group = (idx / W) * 8 + xcd;
    w = idx % W;
  } else {
    const int rest = lin - n8 * W;
    group = n8 + rest / W;
    w = rest % W;
  }
  // group = (b * KS + ks) * H_kv + kvh;  w = j * qt + qtile
  AttnWork r;
  r.qtile = w % qt;
  const int kvh = group % H_kv;
  const int z = group / H_kv;
  r.b = z / KS;
  r.ks = z % KS;
  r.a = kvh * G + w / qt;
  return r;
}

constexpr int kTQ = 128;  // queries per workgroup
constexpr int kTK = 64;   // keys per block
constexpr float kLazy = 8.0f;
typedef short v4i16_t __attribute__((ext_vector_type(4)));

template <bool PAGED>
__device__ __forceinline__ void attn_tile_body(const bf16_t* __restrict__ q, int Mq,
                                               const bf16_t* __restrict__ kc,
                                               const bf16_t* __restrict__ vc, int n, int H_q,
                                               int H_kv, int KS, bf16_t* __restrict__ out,
                                               float* __restrict__ part,
                                               const int* __restrict__ rmap) {
  // [stage][K tile, V tile][64 keys][16 slots of 16 bytes]
  __shared__ __attribute__((aligned(1024))) uint4 tiles[2][2][kTK * 16];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;  // scalar
  const int ln = lane % 16, lg = lane / 16;
  const AttnWork wk = attn_work_tile((Mq + kTQ - 1) / kTQ, H_q, H_kv, KS);
  const int a = wk.a, b = wk.b, ks = wk.ks;
  const int d_q = H_q * kDH, d_kv = H_kv * kDH;
  const int kv = a / (H_q / H_kv);
  const int i0 = wk.qtile * kTQ + wave * 32;  // first query of this wavefront

  const bf16_t* K = kc + kv * kDH;
  const bf16_t* V = vc + kv * kDH;
  const int seq0 = b * n;

  // Q fragments of the two query blocks: lane (query ln, group lg) holds dims 32c + 8lg .. +8
  bf16x8 qf[2][4];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    int qi = i0 + qb * 16 + ln;
    if (qi >= Mq) qi = Mq - 1;  // padded queries compute a duplicate that is never stored
    const bf16_t* qr = q + (static_cast<size_t>(b) * Mq + qi) * d_q + a * kDH + lg * 8;
#pragma unroll
    for (int c = 0; c < 4; ++c) qf[qb][c] = *reinterpret_cast<const bf16x8*>(qr + c * 32);
  }

  const float sl2e = 1.4426950408889634f / sqrtf(static_cast<float>(kDH));
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
  f32x4 o_acc[2][8];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int db = 0; db < 8; ++db) o_acc[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nblk = (n + kTK - 1) / kTK;
  const int per = (nblk + KS - 1) / KS;
  const int blk0 = ks * per;
  const int blk1 = min(nblk, blk0 + per);
  const int nb = blk1 - blk0;

  if (nb > 0) {
    // loader: a tile is 16 wavefront instructions of 4 keys x 256 bytes; wavefront w issues
    // instructions 4w .. 4w+3 of the K and of the V tile.  Lane l: key 4q + l/16, slot l%16.
    int lkey[4], chunk[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lkey[j] = 4 * (4 * wave + j) + lane / 16;
      chunk[j] = (lane % 16) ^ (lkey[j] % 16);
    }
    auto rows_of = [&](int blk, int (&cr)[4]) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int kr = blk * kTK + lkey[j];
        if (kr >= n) kr = n - 1;  // masked in the scores; any finite value will do
        cr[j] = PAGED ? rmap[seq0 + kr] : seq0 + kr;
      }
    };
    auto issue = [&](const int (&cr)[4], int stage) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const size_t row = static_cast<size_t>(cr[j]) * d_kv;
        __builtin_amdgcn_global_load_lds(K + row + chunk[j] * 8, &tiles[stage][0][(4 * wave + j) * 64], 16,
                                         0, 0);
        __builtin_amdgcn_global_load_lds(V + row + chunk[j] * 8, &tiles[stage][1][(4 * wave + j) * 64], 16,
                                         0, 0);
      }
    };
    // flat layout: a block's rows are 64 rows further on than the previous block's, so the loads
    // take fixed per-lane pointers plus one scalar offset (a block that sticks out of the sequence
    // goes the general way, with its rows clamped)
    const bf16_t* kbase[4];
    const bf16_t* vbase[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const size_t row = static_cast<size_t>(seq0 + blk0 * kTK + lkey[j]) * d_kv;  // may lie past the end: unused then
      kbase[j] = K + row + chunk[j] * 8;
      vbase[j] = V + row + chunk[j] * 8;
    }
    auto issue_block = [&](int blk, const int (&cr)[4], int stage) {
      if (PAGED || (blk + 1) * kTK > n) {
        issue(cr, stage);
      } else {
        const size_t off = static_cast<size_t>(blk - blk0) * kTK * d_kv;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          __builtin_amdgcn_global_load_lds(kbase[j] + off, &tiles[stage][0][(4 * wave + j) * 64], 16, 0, 0);
          __builtin_amdgcn_global_load_lds(vbase[j] + off, &tiles[stage][1][(4 * wave + j) * 64], 16, 0, 0);
        }
      }
    };
    int cr_next[4];
    rows_of(blk0, cr_next);
    issue_block(blk0, cr_next, 0);
    rows_of(min(blk0 + 1, blk1 - 1), cr_next);

    // transposing reads: as lane 4t + q of its group this lane names key row 4*lg + t of a 16-key
    // sub-block and dims 4q .. 4q+3 of a dim block; byte offset inside a V tile for dim block db,
    // sub-block 0 (a sub-block further on is 16 rows = 4096 bytes further)
    const int tt = ln / 4, tq = ln % 4;
    const int krow = 4 * lg + tt;  // = key % 16
    int voff[8];
#pragma unroll
    for (int db = 0; db < 8; ++db)
      voff[db] = (krow * 16 + ((2 * db + tq / 2) ^ krow)) * 16 + (tq % 2) * 8;

    for (int i = 0; i < nb; ++i) {
      const int stage = i & 1;
      // this wavefront's loads of block i have landed and its LDS reads of block i - 1 are
      // complete; behind the barrier that holds for everybody, and the other stage is free
      wait_vmcnt_lds<0>();
      __builtin_amdgcn_s_barrier();
      if (i + 1 < nb) {
        const int cr_use[4] = {cr_next[0], cr_next[1], cr_next[2], cr_next[3]};
        issue_block(blk0 + i + 1, cr_use, stage ^ 1);
        rows_of(min(blk0 + i + 2, blk1 - 1), cr_next);
      }
      const uint4* kt = tiles[stage][0];
      const char* vt = reinterpret_cast<const char*>(tiles[stage][1]);
      const int key0 = (blk0 + i) * kTK;
      // scores S^T = K Q^T: lane holds keys key0 + sb*16 + 4*lg + e of query ln (per query block)
      f32x4 st[4][2];
#pragma unroll
      for (int sb = 0; sb < 4; ++sb) {
        bf16x8 kf[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
          kf[c] = __builtin_bit_cast(bf16x8, kt[(sb * 16 + ln) * 16 + ((4 * c + lg) ^ ln)]);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int c = 0; c < 4; ++c)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[c], qf[qb][c], acc, 0, 0, 0);
          st[sb][qb] = acc;
        }
      }
      // Running softmax (base 2) per query block.  First the maxima of both blocks and the rare
      // rescaling (behind a wavefront-uniform branch), then exponentials and the second product in
      // one straight run of code, so that the MFMAs of one query block can be scheduled under the
      // exponentials of the other.
      if (key0 + kTK > n) {  // wavefront-uniform: the block sticks out of the sequence
#pragma unroll
        for (int sb = 0; sb < 4; ++sb)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (key0 + sb * 16 + 4 * lg + e >= n) st[sb][0][e] = st[sb][1][e] = -INFINITY;
      }
      float m_use[2], m_new[2];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float mx = -INFINITY;
#pragma unroll
        for (int sb = 0; sb < 4; ++sb)
#pragma unroll
          for (int e = 0; e < 4; ++e) mx = fmaxf(mx, st[sb][qb][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // The reference point of the exponentials follows the running maximum lazily: it moves only
        // when the maximum has grown by more than kLazy (base-2 units) since it was last set, so
        // probabilities reach at most 2^kLazy (harmless in float32 sums and in a bf16 pair) and the
        // result is the same quotient.  With 32 queries per wavefront some maximum moves in most
        // blocks; by more than kLazy hardly ever after the first ones.
        const float mb = mx * sl2e;
        m_new[qb] = mb > m_run[qb] + kLazy ? mb : m_run[qb];
        m_use[qb] = m_new[qb] == -INFINITY ? 0.f : m_new[qb];
      }
      // the accumulators are rescaled only in the blocks in which some query's reference moved
      if (__builtin_amdgcn_ballot_w64(m_new[0] != m_run[0] || m_new[1] != m_run[1]) != 0) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          // 1 where nothing moved, 0 while nothing has been seen yet
          const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_use[qb]);
          l_run[qb] *= alpha;
          m_run[qb] = m_new[qb];
#pragma unroll
          for (int db = 0; db < 8; ++db) {
            o_acc[qb][db][0] *= alpha;
            o_acc[qb][db][1] *= alpha;
            o_acc[qb][db][2] *= alpha;
            o_acc[qb][db][3] *= alpha;
          }
        }
      }
      // Probabilities as a bf16 pair (high part + remainder: as single bf16 values they cost 11 % of
      // the step's distance from the float64 evaluation at full depth, more than the 2e-2 budget
      // has left), laid out as the B operand of the second product: MFMA k-slot 8*lg + t of half h is key
      // key0 + (2h + t/4)*16 + 4*lg + t%4.  (The hardware's 2^x as it is: the arguments are <= 0, and
      // results below the normal range, which it flushes to zero, are far below anything a bf16
      // probability can carry.)
      // The exponentials of the block's second 32 keys are dealt out between the MFMAs of its first
      // 32 (eight pieces of four probabilities, one per dim block).  That buys little here: on this
      // chip an MFMA with VALU instructions behind it takes its 16 cycles plus most of theirs
      // (measured: MFMA alone 16.9 cycles, with 4 v_fma 34.6, with 8 43.4 per MFMA at four
      // wavefronts per SIMD), so the block costs about the sum of its matrix and vector cycles and
      // what counts is the number of vector instructions per key.
      bf16x8 pf[2][2], pl[2][2];
      float psum[2] = {0.f, 0.f};
      auto exp_piece = [&](int qb, int sb, int e) {  // probabilities e, e+1 of sub-block sb
        const float e0 = __builtin_amdgcn_exp2f(fmaf(st[sb][qb][e], sl2e, -m_use[qb]));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(st[sb][qb][e + 1], sl2e, -m_use[qb]));
        psum[qb] += e0;
        psum[qb] += e1;
        const uint32_t hi = pack_bf16x2(e0, e1);
        reinterpret_cast<uint32_t*>(&pf[qb][sb / 2])[(sb % 2) * 2 + e / 2] = hi;
        reinterpret_cast<uint32_t*>(&pl[qb][sb / 2])[(sb % 2) * 2 + e / 2] =
            pack_bf16x2(e0 - __uint_as_float(hi << 16), e1 - __uint_as_float(hi & 0xffff0000u));
      };
      // O^T[dim][query] += V^T[dim][key] P^T[key][query] for dim block db and key half h
      auto pv_piece = [&](int db, int h) {
        typedef v4i16_t __attribute__((address_space(3))) * lds_v4;
        const v4i16_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(vt + voff[db] + (2 * h) * 4096));
        const v4i16_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(vt + voff[db] + (2 * h + 1) * 4096));
        typedef short v8i16_t __attribute__((ext_vector_type(8)));
        const v8i16_t both = {r0[0], r0[1], r0[2], r0[3], r1[0], r1[1], r1[2], r1[3]};
        const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          o_acc[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qb][h], o_acc[qb][db], 0, 0, 0);
          o_acc[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pl[qb][h], o_acc[qb][db], 0, 0, 0);
        }
      };
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int e = 0; e < 4; e += 2) exp_piece(qb, sb, e);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int db = 0; db < 8; ++db) {
        pv_piece(db, 0);
        exp_piece(db / 4, 2 + (db / 2) % 2, (db % 2) * 2);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int db = 0; db < 8; ++db) pv_piece(db, 1);
      l_run[0] += psum[0];
      l_run[1] += psum[1];
    }
  }
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
    attn_finish(o_acc[qb], m_run[qb], l_run[qb], i0 + qb * 16 + ln, Mq, b, a, ks, KS, H_q, lg, out, part);
}

template <bool PAGED>
__global__ __launch_bounds__(256, 2) void k_attn_tile(const bf16_t* __restrict__ q, int Mq,
                                                      const bf16_t* __restrict__ kc,
                                                      const bf16_t* __restrict__ vc, int n, int H_q,
                                                      int H_kv, int KS, bf16_t* __restrict__ out,
                                                      float* __restrict__ part,
                                                      const int* __restrict__ rmap) {
  attn_tile_body<PAGED>(q, Mq, kc, vc, n, H_q, H_kv, KS, out, part, rmap);
}

// out[query][head][:] = sum_r O_r 2^(m_r - M) / sum_r l_r 2^(m_r - M), in key-range order.
// One wavefront per (query, head), two dims per lane.
template <int SLOTS>
__global__ __launch_bounds__(64) void k_attn_merge(const float* __restrict__ part, int KS,
                                                   bf16_t* __restrict__ out) {
  const size_t qh = static_cast<size_t>(blockIdx.x);  // (b*Mq + iq)*H_q + a
  const float* w = part + qh * KS * (kDH + 2);
  // All SLOTS >= KS slots are loaded before the first use (slots past KS re-read the last
  // valid one and get weight zero): a loop over the runtime count would wait for each load.
  const int dim = threadIdx.x * 2;
  float mr[SLOTS], lr[SLOTS];
  float2 o[SLOTS];
#pragma unroll
  for (int r = 0; r < SLOTS; ++r) {
    const float* wr = w + min(r, KS - 1) * (kDH + 2);
    mr[r] = wr[kDH];
    lr[r] = wr[kDH + 1];
    o[r] = *reinterpret_cast<const float2*>(wr + dim);
  }
  float M = -INFINITY;
#pragma unroll
  for (int r = 0; r < SLOTS; ++r) M = fmaxf(M, mr[r]);
  float L = 0.f, o0 = 0.f, o1 = 0.f;
#pragma unroll
  for (int r = 0; r < SLOTS; ++r) {
    const float f = (r >= KS || mr[r] == -INFINITY) ? 0.f : exp2f(mr[r] - M);
    L += lr[r] * f;
    o0 += o[r].x * f;
    o1 += o[r].y * f;
  }
  const uint32_t t = static_cast<uint32_t>(f32_to_bf16(o0 / L)) |
                     (static_cast<uint32_t>(f32_to_bf16(o1 / L)) << 16);
  *reinterpret_cast<uint32_t*>(out + qh * kDH + dim) = t;
}

}  // namespace

// Keys are split only while (workgroups without split) * KS stays below 1024, and a workgroup
// covers kQT (query, head) pairs per key range, so this bounds the partial results.
size_t attention_scratch_floats() { return static_cast<size_t>(kQT) * 1024 * (kDH + 2); }

bool attention_supported(int dtype, int d_h, int n) {
  if (dtype == 1 && d_h == kDH) return true;
  return static_cast<size_t>(d_h + n) * sizeof(float) <= 60 * 1024;
}

void launch_attention(int dtype, const void* q, int B, int Mq, const void* k_cache,
                      const void* v_cache, int n, int H_q, int H_kv, int d_h, void* out,
                      float* scratch, hipStream_t st, const int* rmap) {
  if (B <= 0 || Mq <= 0 || n <= 0) return;
  if (dtype == 1 && d_h == kDH) {
    const bf16_t* qq = static_cast<const bf16_t*>(q);
    const bf16_t* kk = static_cast<const bf16_t*>(k_cache);
    const bf16_t* vv = static_cast<const bf16_t*>(v_cache);
    bf16_t* oo = static_cast<bf16_t*>(out);
    if (Mq >= kTQ) {
      // many queries per (sequence, head): 128-query tiles; the keys are split only when the
      // queries alone would leave at least half of the CUs without a workgroup
      const int base128 = B * ((Mq + kTQ - 1) / kTQ) * H_q;
      const int nblk64 = (n + kTK - 1) / kTK;
      int KS = 1;
      if (scratch != nullptr && 2 * base128 <= 256) {
        KS = 256 / base128;
        if (KS > 8) KS = 8;
        if (KS > nblk64 / 2) KS = nblk64 / 2 > 0 ? nblk64 / 2 : 1;
      }
      const dim3 grid(base128 * KS);
      if (rmap)
        hipLaunchKernelGGL(k_attn_tile<true>, grid, dim3(256), 0, st, qq, Mq, kk, vv, n, H_q, H_kv, KS, oo,
                           scratch, rmap);
      else
        hipLaunchKernelGGL(k_attn_tile<false>, grid, dim3(256), 0, st, qq, Mq, kk, vv, n, H_q, H_kv, KS, oo,
                           scratch, rmap);
      if (KS > 1)
        hipLaunchKernelGGL(k_attn_merge<8>, dim3(B * Mq * H_q), dim3(64), 0, st, scratch, KS, oo);
      return;
    }
    const int qt = (Mq + kQT - 1) / kQT;
    const int base = B * qt * H_q;  // workgroups without splitting the keys
    const int nblk = (n + 31) / 32;
    int KS = 1;
    // keys are split only while the queries alone leave CUs without a workgroup (384 workgroups of
    // a 768-row refresh: 54 us split in two with a merge launch, 45 us whole)
    if (scratch != nullptr && base < 256) {
      KS = (512 + base - 1) / base;  // aim for ~512 workgroups
      if (KS > kMaxKeySplit) KS = kMaxKeySplit;
      // ranges of three blocks are fetched whole in one trip; shorter ones only add partial
      // results to merge
      if (KS > (nblk + 2) / 3) KS = (nblk + 2) / 3;
    }
    const dim3 grid(qt * H_q * B * KS);
    const bool whole = (nblk + KS - 1) / KS <= kPreload;
#define DLLMC_ATTN(KERNEL) \
  hipLaunchKernelGGL(KERNEL, grid, dim3(256), 0, st, qq, Mq, kk, vv, n, H_q, H_kv, KS, oo, scratch, rmap)
    if (whole && rmap) DLLMC_ATTN(k_attn_mfma<true>);
    else if (whole) DLLMC_ATTN(k_attn_mfma<false>);
    else if (rmap) DLLMC_ATTN(k_attn_walk<true>);
    else DLLMC_ATTN(k_attn_walk<false>);
#undef DLLMC_ATTN
    if (KS > 8)
      hipLaunchKernelGGL(k_attn_merge<kMaxKeySplit>, dim3(B * Mq * H_q), dim3(64), 0, st, scratch, KS,
                         oo);
    else if (KS > 1)
      hipLaunchKernelGGL(k_attn_merge<8>, dim3(B * Mq * H_q), dim3(64), 0, st, scratch, KS, oo);
    return;
  }
  const size_t lds = static_cast<size_t>(d_h + n) * sizeof(float);
  if (dtype == 1)
    hipLaunchKernelGGL(k_attn_simple<bf16_t>, dim3(Mq, H_q, B), dim3(64), lds, st,
                       static_cast<const bf16_t*>(q), Mq, static_cast<const bf16_t*>(k_cache),
                       static_cast<const bf16_t*>(v_cache), n, H_q, H_kv, d_h,
                       static_cast<bf16_t*>(out), rmap);
  else
    hipLaunchKernelGGL(k_attn_simple<float>, dim3(Mq, H_q, B), dim3(64), lds, st,
                       static_cast<const float*>(q), Mq, static_cast<const float*>(k_cache),
                       static_cast<const float*>(v_cache), n, H_q, H_kv, d_h,
                       static_cast<float*>(out), rmap);
}

}  // namespace dllmc
