// bf16 MFMA scoring kernels for gfx950 (paper Eq. 1, Eq. 2, Eq. 4).
//
// A workgroup (4 waves) owns one KV head's row-chunk (up to 256 query rows = GQA heads x window
// rows, held as MFMA operands in registers for the whole kernel) and one chunk of KC keys.  K tiles
// of TK keys are streamed global -> registers -> LDS (16-byte coalesced loads, double-buffered) and
// shared by all waves, so the GQA heads of a group read K once.  Logits are never stored:
//   pass 1:  S^T = K Q^T  (v_mfma_f32_32x32x16_bf16; a lane owns ONE query row and 16 keys), online
//            softmax statistics per row in the log2 domain:  M = max x,  Z = sum 2^(x-M),
//            E = sum 2^(x-M)(x-M),  x = c2 * (q.k),  c2 = scale * log2(e)
//   pass 2:  S = Q K^T   (a lane owns ONE key and 16 query rows), p = 2^(x - lse2[row]),
//            column sum over the row-chunk's rows, reduced across waves through LDS in a fixed order.
// The scale is applied in fp32 after the MFMA (Q is never re-rounded).
#include "common.h"

#include <type_traits>

namespace skv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float kNegBig = -1.0e30f;

template <int D, int RB, int WR, int WK, int PASS, bool DUMP>
__global__ __launch_bounds__(256, 2) void score_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int64_t ksh, int64_t kst,
    SeqTable seq, int Hq, int G, int w, int causal, float c2, int R, int RC, int KC, int64_t n_chunks,
    float* __restrict__ stats, const float* __restrict__ lse2, float* __restrict__ colsum,
    int64_t total, float* __restrict__ probs) {
  static_assert(WR * WK == 4, "four waves per workgroup");
  static_assert(WK <= 2, "an LDS tile holds two 32-key sub-tiles");
  constexpr int NSUB = 2;                      // 32-key sub-tiles per LDS tile
  constexpr int TK = 32 * NSUB;                // keys per LDS tile
  constexpr int SPW = NSUB / WK;               // sub-tiles per wave
  constexpr int RPC = 32 * RB * WR;            // query rows per workgroup
  constexpr int KS = D / 16;                   // MFMA k-steps
  constexpr int PITCH = D * 2 + 16;            // LDS row pitch in bytes (padding spreads the banks)
  constexpr int SEGS = D / 8;                  // 16-byte pieces per key row
  constexpr int NP = TK * SEGS / 256;          // pieces per thread per tile
  static_assert(TK * SEGS % 256 == 0, "tile pieces divide evenly");

  __shared__ __attribute__((aligned(16))) uint8_t kbuf[2][TK * PITCH];
  __shared__ float cs_lds[PASS == 2 ? 2 : 1][WR][TK];
  __shared__ __attribute__((aligned(16))) float nl_lds[PASS == 2 ? RPC : 4];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wr = wave % WR, wk = wave / WR;
  const int l32 = lane & 31, lh = lane >> 5;

  const int GRC = G * RC;
  const int grc = blockIdx.x % GRC;
  const int64_t chunk = blockIdx.x / GRC;
  const int g = grc / RC, rc = grc % RC;
  int b = 0;
  while (b + 1 < seq.batch && chunk >= seq.chunk_start[b + 1]) ++b;
  const int64_t tok0 = seq.cu[b];
  const int64_t n = seq.cu[b + 1] - tok0;
  const int64_t key0 = (chunk - seq.chunk_start[b]) * (int64_t)KC;
  const int64_t key_end = min(n, key0 + KC);
  const int64_t n_full = causal ? n - w : n;   // keys below n_full are visible to every row
  const int ntiles = (int)((key_end - key0 + TK - 1) / TK);

  // ---- the row-chunk's queries as MFMA operands (registers, whole kernel) ----
  const uint16_t* qg = q + ((int64_t)b * Hq * w + (int64_t)g * R) * D;
  bf16x8 qf[RB][KS];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int grow = min(rc * RPC + (wr * RB + rb) * 32 + l32, R - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[rb][ks] = *reinterpret_cast<const bf16x8*>(qg + (int64_t)grow * D + ks * 16 + 8 * lh);
      // opaque to the compiler from here on: otherwise it re-loads the operands from global memory
      // inside the key loop instead of keeping them in registers
      asm volatile("" : "+v"(qf[rb][ks]));
    }
  }

  const uint16_t* kg = k + (int64_t)g * ksh + tok0 * kst;
  // two K tiles are kept in flight in registers (about two tile-times of HBM latency hidden)
  u32x4 stage[2][NP];
  auto load_tile = [&](auto slot_tag, int64_t t0) {
    constexpr int SLOT = decltype(slot_tag)::value;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int p = tid + 256 * i;
      const int key = p / SEGS, seg = p % SEGS;
      const int64_t j = min(t0 + key, n - 1);
      stage[SLOT][i] = *reinterpret_cast<const u32x4*>(kg + j * kst + seg * 8);
    }
  };
  auto store_tile = [&](auto slot_tag, int buf) {
    constexpr int SLOT = decltype(slot_tag)::value;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int p = tid + 256 * i;
      const int key = p / SEGS, seg = p % SEGS;
      *reinterpret_cast<u32x4*>(&kbuf[buf][key * PITCH + seg * 16]) = stage[SLOT][i];
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

  // pass-1 state: this lane's query row(s)
  float M[RB], Z[RB], E[RB];
  int lim1[RB];   // window index of this lane's row (pass 1, causal limit)
  int rbase[RB];  // first of the 16 rows this lane sees in a row block (pass 2): row = rbase + 8*(i/4) + i%4
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    M[rb] = kNegBig; Z[rb] = 0.f; E[rb] = 0.f;
    lim1[rb] = (rc * RPC + (wr * RB + rb) * 32 + l32) % w;
    rbase[rb] = rc * RPC + (wr * RB + rb) * 32 + 4 * lh;
  }
  if (PASS == 2) {
    // -lse2 of the row-chunk's rows (padded rows get -inf so that they contribute exactly 0)
    for (int r = tid; r < RPC; r += 256) {
      const int r2 = rc * RPC + r;
      nl_lds[r] = r2 < R ? -lse2[(int64_t)b * G * R + (int64_t)g * R + r2] : -INFINITY;
    }
  }

  if (ntiles > 0) load_tile(S0{}, key0);
  if (ntiles > 1) load_tile(S1{}, key0 + TK);
  if (ntiles > 0) store_tile(S0{}, 0);
  __syncthreads();

  // one 32-key sub-tile: MFMA, then the softmax work; MASKED is a compile-time switch so that full
  // tiles carry no masking instructions at all
  auto sub_tile = [&](auto masked_tag, int buf, int sub, int t0i) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    floatx16 acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(
          &kbuf[buf][(sub * 32 + l32) * PITCH + ks * 32 + 16 * lh]);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (PASS == 1) acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][ks], acc[rb], 0, 0, 0);
        else           acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][ks], kf, acc[rb], 0, 0, 0);
      }
    }
    const int ni = (int)n;
    if (PASS == 1) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (MASKED) {
          const int lim = causal ? ni - w + lim1[rb] + 1 : ni;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int j = t0i + sub * 32 + 8 * (i / 4) + 4 * lh + (i % 4);
            if (j >= lim) acc[rb][i] = -INFINITY;
          }
        }
        float tm = fmaxf(fmaxf(acc[rb][0], acc[rb][1]), acc[rb][2]);
#pragma unroll
        for (int i = 3; i < 15; i += 2) tm = fmaxf(fmaxf(tm, acc[rb][i]), acc[rb][i + 1]);
        tm = fmaxf(tm, acc[rb][15]);
        const float Mn = fmaxf(M[rb], tm * c2);
        const float dl = M[rb] - Mn;
        const float f = __builtin_amdgcn_exp2f(dl);
        float z0 = Z[rb] * f, z1 = 0.f;
        float e0 = (E[rb] + dl * Z[rb]) * f, e1 = 0.f;
        const float nm = -Mn;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          float ta = fmaf(acc[rb][i], c2, nm);
          float tb = fmaf(acc[rb][i + 1], c2, nm);
          if (MASKED) { ta = fmaxf(ta, -200.f); tb = fmaxf(tb, -200.f); }   // 2^-200 = 0, and 0 * -200 = 0
          const float pa = __builtin_amdgcn_exp2f(ta);
          const float pb = __builtin_amdgcn_exp2f(tb);
          z0 += pa; z1 += pb;
          e0 = fmaf(pa, ta, e0); e1 = fmaf(pb, tb, e1);
        }
        M[rb] = Mn; Z[rb] = z0 + z1; E[rb] = e0 + e1;
      }
    } else {
      const int j = t0i + sub * 32 + l32;   // this lane's key
      float c0 = 0.f, c1 = 0.f;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const float4 nl4 = *reinterpret_cast<const float4*>(&nl_lds[(wr * RB + rb) * 32 + 8 * q4 + 4 * lh]);
          const float nlv[4] = {nl4.x, nl4.y, nl4.z, nl4.w};
#pragma unroll
          for (int e = 0; e < 4; e += 2) {
            const int i = 4 * q4 + e;
            float pa = __builtin_amdgcn_exp2f(fmaf(acc[rb][i], c2, nlv[e]));
            float pb = __builtin_amdgcn_exp2f(fmaf(acc[rb][i + 1], c2, nlv[e + 1]));
            const int ra = rbase[rb] + 8 * q4 + e, rbw = ra + 1;
            if (MASKED) {
              const int la = causal ? ni - w + (ra % w) + 1 : ni;
              const int lb = causal ? ni - w + (rbw % w) + 1 : ni;
              if (j >= la) pa = 0.f;
              if (j >= lb) pb = 0.f;
            }
            if (DUMP && j < ni) {
              if (ra < R) probs[((int64_t)g * R + ra) * n + j] = pa;
              if (rbw < R) probs[((int64_t)g * R + rbw) * n + j] = pb;
            }
            c0 += pa; c1 += pb;
          }
        }
      }
      float cs = c0 + c1;
      cs += __shfl_xor(cs, 32);
      if (lh == 0) cs_lds[PASS == 2 ? buf : 0][wr][sub * 32 + l32] = cs;
    }
  };

  // tile `it` sits in LDS buffer it&1; its register slot (it&1) is free again and takes tile it+2
  auto tile_step = [&](auto slot_tag, int it) {
    using SLOT = decltype(slot_tag);
    using OTHER = std::integral_constant<int, 1 - SLOT::value>;
    const int64_t t0 = key0 + (int64_t)it * TK;
    const int buf = SLOT::value;
    if (it + 2 < ntiles) load_tile(SLOT{}, t0 + 2 * TK);
    const bool masked = t0 + TK > n_full;
    if (!masked) {
#pragma unroll
      for (int sp = 0; sp < SPW; ++sp)
        sub_tile(std::integral_constant<bool, false>{}, buf, WK == 1 ? sp : wk, (int)t0);
    } else {
#pragma unroll
      for (int sp = 0; sp < SPW; ++sp)
        sub_tile(std::integral_constant<bool, true>{}, buf, WK == 1 ? sp : wk, (int)t0);
    }
    if (it + 1 < ntiles) store_tile(OTHER{}, buf ^ 1);
    __syncthreads();
    if (PASS == 2) {
      if (tid < TK && t0 + tid < key_end) {
        float s = cs_lds[PASS == 2 ? buf : 0][0][tid];
#pragma unroll
        for (int r = 1; r < WR; ++r) s += cs_lds[PASS == 2 ? buf : 0][r][tid];
        colsum[(int64_t)grc * total + tok0 + t0 + tid] = s;
      }
    }
  };
  for (int it = 0; it < ntiles; it += 2) {
    tile_step(S0{}, it);
    if (it + 1 < ntiles) tile_step(S1{}, it + 1);
  }

  if (PASS == 1) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      // the two lane halves hold disjoint key subsets of the same query row
      const float M2 = __shfl_xor(M[rb], 32), Z2 = __shfl_xor(Z[rb], 32), E2 = __shfl_xor(E[rb], 32);
      const float Mn = fmaxf(M[rb], M2);
      const float d1 = M[rb] - Mn, d2 = M2 - Mn;
      const float f1 = __builtin_amdgcn_exp2f(d1), f2 = __builtin_amdgcn_exp2f(d2);
      const float En = (E[rb] + d1 * Z[rb]) * f1 + (E2 + d2 * Z2) * f2;
      const float Zn = Z[rb] * f1 + Z2 * f2;
      if (lh == 0) {
        float* sp = stats + ((((int64_t)grc * n_chunks + chunk) * WK + wk) * 3) * RPC +
                    (wr * RB + rb) * 32 + l32;
        sp[0] = Mn;
        sp[RPC] = Zn;
        sp[2 * RPC] = En;
      }
    }
  }
}

template <int D, int RB, int WR, int WK>
hipError_t launch_cfg(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq, const void* q,
                      const void* k, int64_t ksh, int64_t kst, float c2, float* stats, const float* lse2,
                      float* colsum, int64_t total, float* probs, int pass, hipStream_t st) {
  const int64_t grid = (int64_t)s.n_kv_heads * p.RC * p.n_chunks;
  dim3 g((unsigned)grid), blk(256);
  if (pass == 1)
    hipLaunchKernelGGL((score_mfma_kernel<D, RB, WR, WK, 1, false>), g, blk, 0, st, (const uint16_t*)q,
                       (const uint16_t*)k, ksh, kst, seq, s.n_q_heads, s.n_kv_heads, s.window, s.causal, c2,
                       p.R, p.RC, p.KC, p.n_chunks, stats, lse2, colsum, total, probs);
  else if (probs == nullptr)
    hipLaunchKernelGGL((score_mfma_kernel<D, RB, WR, WK, 2, false>), g, blk, 0, st, (const uint16_t*)q,
                       (const uint16_t*)k, ksh, kst, seq, s.n_q_heads, s.n_kv_heads, s.window, s.causal, c2,
                       p.R, p.RC, p.KC, p.n_chunks, stats, lse2, colsum, total, probs);
  else
    hipLaunchKernelGGL((score_mfma_kernel<D, RB, WR, WK, 2, true>), g, blk, 0, st, (const uint16_t*)q,
                       (const uint16_t*)k, ksh, kst, seq, s.n_q_heads, s.n_kv_heads, s.window, s.causal, c2,
                       p.R, p.RC, p.KC, p.n_chunks, stats, lse2, colsum, total, probs);
  return hipGetLastError();
}

template <int D>
hipError_t launch_d(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq, const void* q,
                    const void* k, int64_t ksh, int64_t kst, float c2, float* stats, const float* lse2,
                    float* colsum, int64_t total, float* probs, int pass, hipStream_t st) {
#define SKV_CFG(rb, wr, wk)                                                                       \
  if (p.RB == rb && p.WR == wr && p.WK == wk)                                                     \
    return launch_cfg<D, rb, wr, wk>(s, p, seq, q, k, ksh, kst, c2, stats, lse2, colsum, total, probs, pass, st)
  SKV_CFG(2, 4, 1);
  SKV_CFG(1, 4, 1);
  SKV_CFG(1, 2, 2);
#undef SKV_CFG
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_score_mfma(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                             const void* q, const void* k, int64_t ksh, int64_t kst, float c2,
                             float* stats, const float* lse2, float* colsum, int64_t total,
                             float* probs, int pass, hipStream_t st) {
  if (p.n_chunks == 0) return hipSuccess;
  if (s.head_dim == 128)
    return launch_d<128>(s, p, seq, q, k, ksh, kst, c2, stats, lse2, colsum, total, probs, pass, st);
  if (s.head_dim == 64)
    return launch_d<64>(s, p, seq, q, k, ksh, kst, c2, stats, lse2, colsum, total, probs, pass, st);
  return hipErrorInvalidValue;
}

}  // namespace skv
