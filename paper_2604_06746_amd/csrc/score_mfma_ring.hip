// bf16 MFMA scoring kernels for gfx950 (paper Eq. 1, Eq. 2, Eq. 4): register-resident queries, keys
// streamed HBM -> LDS by direct-to-LDS loads (no staging registers) through a ring of 32-key tiles.
//
// What shaped it (measured on MI355X): under this mix of MFMA and vector work the chip runs at a
// power-managed ~1.5 GHz and the vector ALU's issue port is the busiest unit (one vector instruction per
// 4 cycles per SIMD, a transcendental ~2.6 of them); a single wave issues only every ~5-6 cycles, so
// the port is fed by several waves per SIMD, and three waves of 64 query rows (168 registers) beat two
// waves of 128 rows (256 registers); a ds_read_b128 stream sustains ~64 B/clk per CU, so each 1 KB
// operand read from LDS must serve at least 2 MFMAs; HBM latency needs ~60 KB of loads in flight per CU.
// Hence:
//   * a wave owns a row-chunk of 64 query rows (2 blocks of 32) or of 32 rows as MFMA
//     operands in registers for the whole kernel, and reads each key operand from LDS once per 32-key tile;
//   * a KV group of 256 rows (GQA 4 x window 64) is four row-chunks of 64 rows = the four waves of a workgroup
//     (128 rows: four row-chunks of 32), which share the LDS tiles, so K crosses HBM -> L2 -> LDS once per pass;
//   * tiles are fetched with global_load_lds_dwordx4 (16 B per lane, lane L lands at base + 16 L), three
//     tiles ahead, into an XOR-swizzled layout that makes the operand reads bank-conflict free;
//   * inside a wave the MFMAs of row block rb+1 are issued under the softmax arithmetic of row block rb.
//
//   pass 1:  S^T = K Q^T   a lane owns ONE query row of each row block and 16 keys: a reference M (the maximum
//            of the chunk's first tile; the running maximum in the rare rerun), Z = sum 2^(x-M),
//            E = sum 2^(x-M)(x-M) per row, x = c2 (q.k), c2 = scale log2(e)
//   pass 2:  S = Q K^T     a lane owns ONE key and 16 rows of each row block; -lse2[row]/c2 rides in
//            one extra MFMA k-step (three bf16 pieces of it against ones on the key side), so
//            p = 2^(c2 acc) needs no per-row constant in registers; the lane sums its key's column.
#include "common.h"

#include <type_traits>

namespace skv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) uint16_t u16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;   // operand of v_mfma_f32_32x32x8_bf16_1k
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr float kNegBig = -1.0e30f;

// x of lane l + x of lane l + 32, in both lanes (the lower half's value first): one vector instruction that swaps
// the halves of two registers, no trip through the LDS crossbar and no wait for it inside the key loop
__device__ __forceinline__ float add_lane_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <bool V> using BoolC = std::integral_constant<bool, V>;
template <int V> using IntC = std::integral_constant<int, V>;
// a ring slot is either a compile-time number (key loop unrolled over the slots) or a run-time one
template <int V> __device__ __forceinline__ constexpr int slot_of(IntC<V>) { return V; }
__device__ __forceinline__ constexpr int slot_of(int v) { return v; }

// round-to-nearest-even bf16 bits of a finite float (or of +-inf)
__device__ inline uint16_t bf16_bits(float x) {
  const uint32_t u = __float_as_uint(x);
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ inline float bf16_value(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// most keys a workgroup may be given (pass 2 keeps one fp32 column sum per key in LDS)
// (one-wave workgroups: 896, so that eight of them -- 16 KB ring + 3.5 KB each -- still share a CU's 160 KB)
template <int NW> constexpr int kKeyCap = NW == 4 ? 2048 : 896;

// Pass 2 with one column-sum plane per QUERY HEAD instead of one per workgroup (the per-head in-degrees of the
// pivot detector's metrics, Eq. 5-6): PPW planes per wave -- 1 when a wave's rows are one head's window, 2 when
// each of its two 32-row blocks is.  Most keys a workgroup may then be given: its LDS holds NW*PPW sums per key for
// all tiles but the chunk's last THREE, whose sums go from the registers straight to global memory (no tile load is
// requested after them any more, so these stores sit behind every load that a wait still counts) -- 20 KB of sums
// beside three 4-wave workgroups' rings, which is what lets a 128K-token layer be ONE round of 768 workgroups with
// 1376 keys each (21 KB already cost the third workgroup per CU).
constexpr int kPlanesDirectTiles = 3;
template <int NW, int PPW> constexpr int kPlanesKeyCap = NW == 4 ? (PPW == 1 ? 1376 : 736) : 1024 / PPW;
// ... of which LDS holds
template <int NW, int PPW> constexpr int kPlanesLdsKeys = kPlanesKeyCap<NW, PPW> - 32 * kPlanesDirectTiles;

// NW = waves per workgroup (row-chunks sharing the key tiles), NBUF = tiles in the LDS ring; PPW > 0 (pass 2):
// planes per wave as above, written to consecutive planes of `colsum`: plane g*RC*PPW + row-chunk*PPW + block.
// NT: the key tiles are fetched with the non-temporal cache policy -- for a K larger than the 256 MB memory-side
// cache, whose lines no later pass would find there anyway (measured: 4-8 % off both passes on a 1.1 GB K,
// ~1 % on 256 MiB, and 3-6 % SLOWER on 64 MiB, where pass 2 and the gather do find pass 1's lines)
template <int D, int NRB, int NW, int NBUF, int PASS, bool DUMP, int PPW = 0, bool NT = false>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 3 : 2) void score_mfma_ring_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int64_t ksh, int64_t kst, int kshare,
    SeqTable seq, int Hq, int G, int w, int causal, float c2, int R, int RC, int KC, int64_t n_chunks,
    float* __restrict__ stats, const float* __restrict__ lse2, float* __restrict__ colsum,
    int64_t total, float* __restrict__ probs) {
  constexpr int KS = D / 16;        // MFMA k-steps over the head dimension
  constexpr int RPC = 32 * NRB;     // query rows per wave
  constexpr int SEGS = D / 8;       // 16-byte pieces per key row
  constexpr int TILE_BYTES = 32 * D * 2;
  constexpr int NINST = 32 * SEGS / 64;   // wave-wide 1 KB load instructions per tile
  constexpr int IPW = NINST / NW;          // ... issued by each wave
  constexpr int PD = NBUF - 1;             // tiles requested ahead of the one being consumed
  static_assert(NINST % NW == 0, "tile loads split evenly over the waves");
  __shared__ __attribute__((aligned(1024))) uint8_t ring[NBUF * TILE_BYTES];
  // pass 2: the workgroup's column sums of its whole key chunk collect in LDS and are written out once at the
  // end, so that the key loop holds no global store (a store between the tile loads would make the
  // s_waitcnt vmcnt(N) below wait for younger loads than it has to).  With several waves, each wave parks
  // its sums of tile s (both lane halves, 64 floats: no cross-lane exchange in the loop) in csbuf[s % 4] and
  // one wave adds them up, halves first, then in wave order, two tiles later: by then
  // every wave has waited for the LDS reads of tile s+1 (LDS operations complete in order, so its older
  // csbuf write is done) and has passed the barrier of tile s+2 -- no extra wait, no extra barrier.
  // Both buffers live in DYNAMIC LDS behind the ring (csout [KCAP] floats, then csbuf [4][NW][64] floats;
  // the launcher passes their size) and are addressed by number, through asm: the ring stays the kernel's only LDS object,
  // whose reads the compiler then never orders behind the tile loads in flight (with the buffers as static
  // arrays, or with their addresses taken, it loses track and waits for ALL tile loads before LDS accesses).
  constexpr bool PLANES = PPW > 0;
  // (with planes: keys per plane in LDS)
  constexpr int KCAP = PASS == 2 ? (PLANES ? kPlanesLdsKeys<NW, (PLANES ? PPW : 1)> : kKeyCap<NW>) : 1;
  static_assert(!PLANES || (PASS == 2 && !DUMP && PPW <= NRB), "per-head planes are a pass-2 output");
  // vector-ALU instructions the scheduler is asked to place after each MFMA of the next row block
  constexpr int VPM = PASS == 1 ? 8 : 4;

  const int lane = threadIdx.x & 63;
  const int l32 = lane & 31, lh = lane >> 5;

  // workgroup -> (KV head g, group of row-chunks, key chunk); wave -> row-chunk inside the group
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // a scalar: addresses built from it stay in SGPRs
  const int rcg = (RC + NW - 1) / NW;
  // groups that share a K head (kshare > 1) get workgroup numbers a multiple of G/kshare apart: with the
  // usual eight KV heads they run on the same XCD at about the same time, and its L2 serves the re-reads
  const int gp = blockIdx.x % G;
  const int g = kshare == 1 ? gp : (gp % (G / kshare)) * kshare + gp / (G / kshare);
  const int64_t t = blockIdx.x / G;
  // a wave beyond the last row-chunk still helps loading tiles and keeps the barriers matched; it
  // computes on a valid chunk (the last one) and simply does not write results
  const int rc_raw = (int)(t % rcg) * NW + wave;
  const bool live = rc_raw < RC;
  const int rc = live ? rc_raw : RC - 1;
  const int64_t chunk = t / rcg;
  const int grc = g * RC + rc;
  const int plane = g * rcg + (int)(t % rcg);   // pass 2: the workgroup's column-sum plane
  int b = 0;
  while (b + 1 < seq.batch && chunk >= seq.chunk_start[b + 1]) ++b;
  const int64_t tok0 = seq.cu[b];
  const int64_t n = seq.cu[b + 1] - tok0;
  const int ni = (int)n;
  const int key0 = (int)((chunk - seq.chunk_start[b]) * (int64_t)KC);
  const int key_end = min(ni, key0 + KC);
  const int n_full = causal ? ni - w : ni;   // keys below n_full are visible to every row
  const int nsub = (key_end - key0 + 31) / 32;

  // ---- the row-chunk's queries as MFMA operands (registers, whole kernel) ----
  const uint16_t* qg = q + ((int64_t)b * Hq * w + (int64_t)g * R) * D;
  bf16x8 qf[NRB][KS];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    const int grow = min(rc * RPC + rb * 32 + l32, R - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[rb][ks] = *reinterpret_cast<const bf16x8*>(qg + (int64_t)grow * D + ks * 16 + 8 * lh);
  }
  // opaque to the compiler from here on, so that it keeps the operands in registers instead of re-loading
  // them inside the key loop (pinned only after ALL loads are in flight: one latency, not one per load)
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[rb][ks]));

  // pass 2: the extra k-step, a v_mfma_f32_32x32x8_bf16_1k (half the operand registers of a 32x32x16 step;
  // lane l holds row/column l%32 and k = 4(l/32)..+3).  Query side: -(lse2[row]/c2) in three
  // bf16 pieces (lane half 0, first three k slots); key side: ones in the same slots.  Padded rows carry -inf,
  // so their p is exactly 0.
  s16x4 qaug[PASS == 2 ? NRB : 1] = {};
  s16x4 kaug = {0, 0, 0, 0};
  if (PASS == 2) {
    if (lh == 0) { kaug[0] = 0x3F80; kaug[1] = 0x3F80; kaug[2] = 0x3F80; }
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const int row = rc * RPC + rb * 32 + l32;
      s16x4 v = {0, 0, 0, 0};
      if (lh == 0) {
        if (row < R) {
          const float lam = -lse2[(int64_t)b * G * R + (int64_t)g * R + row] / c2;
          const uint16_t hi = bf16_bits(lam);
          const float r1 = lam - bf16_value(hi);
          const uint16_t mid = bf16_bits(r1);
          const uint16_t lo = bf16_bits(r1 - bf16_value(mid));
          v[0] = (short)hi; v[1] = (short)mid; v[2] = (short)lo;
        } else {
          v[0] = (short)0xFF80;   // -inf
        }
      }
      qaug[rb] = v;
      asm volatile("" : "+v"(qaug[rb]));
    }
  }

  const uint16_t* kg = k + (int64_t)(g / kshare) * ksh + tok0 * kst;
  // Tile layout in LDS: 16-byte piece (key, seg) sits at unit key*SEGS + (seg ^ swz(key)); any 16
  // consecutive keys at a fixed seg then hit 16 different groups of 4 banks (conflict-free operand reads).
  // Loader: instruction I, lane L writes unit I*64 + L, so it must fetch that unit's (key, seg).
  auto swz = [&](int key) __attribute__((always_inline)) { return SEGS == 16 ? (key & 15) : ((key >> 1) & 7); };
  // per-lane byte offsets of the units this lane fetches, relative to the tile's first key row
  uint32_t voff[IPW];
#pragma unroll
  for (int ii = 0; ii < IPW; ++ii) {
    const int unit = (ii * NW + wave) * 64 + lane;
    const int key = unit / SEGS;
    voff[ii] = (uint32_t)(key * kst + ((unit % SEGS) ^ swz(key)) * 8) * 2u;
  }
  // (where the key loop is unrolled over the NBUF slots the ring slot is a compile-time number, and slot offsets
  // fold into the instructions' immediate offsets instead of costing an address addition per LDS read)
  auto issue_tile = [&](int s_idx, auto slot_tag) __attribute__((always_inline)) {
    const int jbase = key0 + 32 * s_idx;
    uint8_t* slot = ring + slot_of(slot_tag) * TILE_BYTES + wave * 1024;
    const uint8_t* gbase = reinterpret_cast<const uint8_t*>(kg + (int64_t)jbase * kst);   // wave-uniform
    if (jbase + 32 <= ni) {
#pragma unroll
      for (int ii = 0; ii < IPW; ++ii)
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(gbase + voff[ii]), (lds_ptr_t)(slot + ii * NW * 1024), 16, 0, NT ? 2 : 0);
    } else {   // ragged tail: rows past the end re-read the last valid row (their logits are masked)
#pragma unroll
      for (int ii = 0; ii < IPW; ++ii) {
        const int unit = (ii * NW + wave) * 64 + lane;
        const int key0u = unit / SEGS;
        const int seg = (unit % SEGS) ^ swz(key0u);
        const int key = min(key0u, ni - 1 - jbase);
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(gbase + (uint32_t)(key * kst + seg * 8) * 2u),
                                         (lds_ptr_t)(slot + ii * NW * 1024), 16, 0, NT ? 2 : 0);
      }
    }
  };
  // Operands of the tile being consumed.  Plain loads: an asm ds_read whose result is waited for by a later
  // asm statement is NOT safe -- the compiler may copy the "loaded" register in between, before the data has
  // arrived (it did, in a software-pipelined variant of the key loop).
  bf16x8 kf[KS];
  auto read_tile = [&](auto slot_tag) __attribute__((always_inline)) {
    const uint8_t* slot = ring + slot_of(slot_tag) * TILE_BYTES;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int seg = 2 * ks + lh;
      kf[ks] = *reinterpret_cast<const bf16x8*>(slot + (l32 * SEGS + (seg ^ swz(l32))) * 16);
    }
  };

  float M[NRB], Z[NRB], E[NRB];   // pass 1: statistics of this lane's query row in each row block
  int win[NRB];                   // pass 1: window index of that row (causal limit)
  int win2[NRB];                  // pass 2: window index of the first of the 16 rows this lane sees
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    M[rb] = kNegBig; Z[rb] = 0.f; E[rb] = 0.f;
    win[rb] = (rc * RPC + rb * 32 + l32) % w;
    win2[rb] = (rc * RPC + rb * 32) % w + 4 * lh;
  }
  float cs0 = 0.f, cs1 = 0.f;     // pass 2: column sum of this lane's key
  float csp[PPW == 2 ? 2 : 1] = {};   // PPW == 2: the same per 32-row block (cs0 + cs1 of each block)

  auto mfma_block = [&](floatx16& acc, const bf16x8 (&kf)[KS], auto rb_tag) __attribute__((always_inline)) {
    constexpr int rb = decltype(rb_tag)::value;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (PASS == 1) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], acc, 0, 0, 0);
      else           acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][ks], kf[ks], acc, 0, 0, 0);
    }
    if constexpr (PASS == 2) acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(qaug[rb], kaug, acc, 0, 0, 0);
  };

  // softmax arithmetic of one row block against the 32 keys starting at jbase
  // FIXED_REF (pass 1): the row's reference M stays what the chunk's first tile set it to -- no tile maximum, no
  // rescaling of the running sums (a sixth of the vector instructions).  Any reference gives the same
  // statistics as long as nothing overflows; whether something came near that is checked after the loop.
  auto softmax_block = [&](auto masked_tag, floatx16& acc, auto rb_tag, int jbase, auto fixed_tag) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    constexpr int rb = decltype(rb_tag)::value;
    constexpr bool FIXED_REF = decltype(fixed_tag)::value;
    if (PASS == 1) {
      if (MASKED) {
        const int lim = causal ? ni - w + win[rb] + 1 : ni;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = jbase + 8 * (i / 4) + 4 * lh + (i % 4);
          if (j >= lim) acc[i] = -INFINITY;
        }
      }
      if constexpr (FIXED_REF) {
        const float nm = -M[rb];
        float z0 = Z[rb], z1 = 0.f, e0 = E[rb], e1 = 0.f;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          float ta = fmaf(acc[i], c2, nm);
          float tb = fmaf(acc[i + 1], c2, nm);
          if (MASKED) { ta = fmaxf(ta, -200.f); tb = fmaxf(tb, -200.f); }
          const float pa = __builtin_amdgcn_exp2f(ta);
          const float pb = __builtin_amdgcn_exp2f(tb);
          z0 += pa; z1 += pb;
          e0 = fmaf(pa, ta, e0); e1 = fmaf(pb, tb, e1);
        }
        Z[rb] = z0 + z1; E[rb] = e0 + e1;
        return;
      }
      float tm = fmaxf(fmaxf(acc[0], acc[1]), acc[2]);
#pragma unroll
      for (int i = 3; i < 15; i += 2) tm = fmaxf(fmaxf(tm, acc[i]), acc[i + 1]);
      tm = fmaxf(tm, acc[15]);
      const float Mn = fmaxf(M[rb], tm * c2);
      const float dl = M[rb] - Mn;
      const float f = __builtin_amdgcn_exp2f(dl);
      float z0 = Z[rb] * f, z1 = 0.f;
      float e0 = (E[rb] + dl * Z[rb]) * f, e1 = 0.f;
      const float nm = -Mn;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        float ta = fmaf(acc[i], c2, nm);
        float tb = fmaf(acc[i + 1], c2, nm);
        if (MASKED) { ta = fmaxf(ta, -200.f); tb = fmaxf(tb, -200.f); }   // 2^-200 = 0, and 0 * -200 = 0
        const float pa = __builtin_amdgcn_exp2f(ta);
        const float pb = __builtin_amdgcn_exp2f(tb);
        z0 += pa; z1 += pb;
        e0 = fmaf(pa, ta, e0); e1 = fmaf(pb, tb, e1);
      }
      M[rb] = Mn; Z[rb] = z0 + z1; E[rb] = e0 + e1;
    } else {
      const int j = jbase + l32;   // this lane's key
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        float pa = __builtin_amdgcn_exp2f(acc[i] * c2);
        float pb = __builtin_amdgcn_exp2f(acc[i + 1] * c2);
        const int ra = rc * RPC + rb * 32 + 8 * (i / 4) + 4 * lh + (i % 4), rbw = ra + 1;
        if (MASKED) {
          // causal only (keys past the end of the sequence are simply never written), and the window is
          // a multiple of 32 rows here, so a 32-row block never straddles two heads
          const int la = ni - w + win2[rb] + 8 * (i / 4) + (i % 4) + 1;
          if (j >= la) pa = 0.f;
          if (j >= la + 1) pb = 0.f;
        }
        if (DUMP && j < ni) {
          if (ra < R) probs[((int64_t)g * R + ra) * n + j] = pa;
          if (rbw < R) probs[((int64_t)g * R + rbw) * n + j] = pb;
        }
        cs0 += pa; cs1 += pb;
      }
      if constexpr (PPW == 2) { csp[rb] = cs0 + cs1; cs0 = 0.f; cs1 = 0.f; }
    }
  };

  auto interleave_hint = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < KS + (PASS == 2 ? 1 : 0); ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);   // then a group of vector-ALU instructions
      __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);     // and two transcendentals (a class of their own)
    }
  };

  // pass 2, several waves: add up the waves' sums of tile s_idx (see csbuf above for when this is safe).
  // The LDS accesses to csbuf and csout inside the key loop are written as asm: for compiler-generated ones the
  // compiler cannot always rule out that the tile loads in flight (which write LDS too) alias them, and then
  // waits for ALL of those loads (vmcnt 0) in front of the access, which empties the ring every tile.
  // The column-sum buffers never overlap the ring, so no such wait is needed.
  const uint32_t lane_x4_lo = (uint32_t)l32 * 4u, thread_x4 = (uint32_t)threadIdx.x * 4u;
  const uint32_t csout_lds = __builtin_amdgcn_groupstaticsize();   // dynamic LDS starts where the static part ends
  const uint32_t csbuf_lds = csout_lds + (uint32_t)KCAP * 4u;
  // `ring_slot`: s_idx mod 4, a compile-time number where the key loop is unrolled (the slot's offset is then an
  // immediate of the LDS instructions and costs no register), else a run-time one (its scalar part goes through
  // readfirstlane, stays in a scalar register and is added to the lane part at the point of use).
  auto flush_colsum = [&](int s_idx, auto ring_slot) __attribute__((always_inline)) {
    if constexpr (PASS == 2 && NW > 1 && !PLANES) if (wave == (s_idx % NW) && lh == 0) {
      constexpr bool RT = std::is_same<decltype(ring_slot), int>::value;
      uint32_t a = csbuf_lds + lane_x4_lo;
      if constexpr (RT) a = (uint32_t)__builtin_amdgcn_readfirstlane((int)(csbuf_lds + (uint32_t)(ring_slot * NW * 256))) + lane_x4_lo;
      constexpr int OFF = RT ? 0 : slot_of(decltype(ring_slot){}) * NW * 256;
      // all reads AND their wait in ONE asm statement (nothing can get between a read and its wait; one LDS
      // round trip for the lot)
      float lo[NW], hi[NW];
      if constexpr (NW == 4) {
        asm volatile("ds_read_b32 %0, %8 offset:%9\n\tds_read_b32 %1, %8 offset:%9+128\n\t"
                     "ds_read_b32 %2, %8 offset:%9+256\n\tds_read_b32 %3, %8 offset:%9+384\n\t"
                     "ds_read_b32 %4, %8 offset:%9+512\n\tds_read_b32 %5, %8 offset:%9+640\n\t"
                     "ds_read_b32 %6, %8 offset:%9+768\n\tds_read_b32 %7, %8 offset:%9+896\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(lo[0]), "=&v"(hi[0]), "=&v"(lo[1]), "=&v"(hi[1]), "=&v"(lo[2]), "=&v"(hi[2]),
                       "=&v"(lo[NW - 1]), "=&v"(hi[NW - 1])
                     : "v"(a), "n"(OFF));
      } else {
        asm volatile("ds_read_b32 %0, %4 offset:%5\n\tds_read_b32 %1, %4 offset:%5+128\n\t"
                     "ds_read_b32 %2, %4 offset:%5+256\n\tds_read_b32 %3, %4 offset:%5+384\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(lo[0]), "=&v"(hi[0]), "=&v"(lo[NW - 1]), "=&v"(hi[NW - 1])
                     : "v"(a), "n"(OFF));
      }
      // a wave's sum of a key = its lower lane half's + its upper lane half's; then the waves in order
      float cs = lo[0] + hi[0];
#pragma unroll
      for (int wv = 1; wv < NW; ++wv) cs += lo[wv] + hi[wv];
      const uint32_t o = (uint32_t)__builtin_amdgcn_readfirstlane((int)(csout_lds + (uint32_t)(128 * s_idx))) + lane_x4_lo;
      asm volatile("ds_write_b32 %0, %1" : : "v"(o), "v"(cs) : "memory");
    }
  };
  floatx16 acc0, acc1;

  // pass 2: park this tile's column sums.  ONE store in the loop body, outside the masked / unmasked variants
  // of sub_tile: two copies get merged by the compiler into a store that has lost its alias information, and it
  // then waits for every outstanding tile load (which also write LDS) before it.
  auto park_colsum = [&](int jbase, auto ring_slot) __attribute__((always_inline)) {
    if (PASS == 2 && PLANES) {
      // every wave keeps its own sums, one list per head: lane halves added here, no exchange between waves
      constexpr int NP = PLANES ? PPW : 1;
      const uint32_t a0 = csout_lds + (uint32_t)((wave * NP * KCAP + (jbase - key0 + l32)) * 4);
      const bool last = jbase + 32 * kPlanesDirectTiles >= key_end;   // the chunk's last tiles: straight to their planes
#pragma unroll
      for (int sp = 0; sp < NP; ++sp) {
        float cs = PPW == 2 ? csp[sp] : cs0 + cs1;
        cs = add_lane_halves(cs);
        const uint32_t a = a0 + (uint32_t)(sp * KCAP * 4);
        const float val = live ? cs : 0.f;
        if (last) {
          if (lh == 0 && live && jbase + l32 < key_end)
            colsum[((int64_t)g * RC * NP + (int64_t)rc * NP + sp) * total + tok0 + jbase + l32] = val;
        } else if (lh == 0) {
          asm volatile("ds_write_b32 %0, %1" : : "v"(a), "v"(val) : "memory");
        }
      }
      cs0 = 0.f; cs1 = 0.f;
    } else if (PASS == 2) {
      float cs = cs0 + cs1;
      if (NW == 1) {
        cs = add_lane_halves(cs);
        if (lh == 0)
          asm volatile("ds_write_b32 %0, %1" : : "v"(csout_lds + (uint32_t)((jbase - key0 + l32) * 4)), "v"(cs) : "memory");
      } else {
        // both lane halves park their sums: no cross-lane exchange in the key loop
        constexpr bool RT = std::is_same<decltype(ring_slot), int>::value;
        uint32_t a = csbuf_lds + thread_x4;
        if constexpr (RT) a = (uint32_t)__builtin_amdgcn_readfirstlane((int)(csbuf_lds + (uint32_t)(ring_slot * NW * 256))) + thread_x4;
        constexpr int OFF = RT ? 0 : slot_of(decltype(ring_slot){}) * NW * 256;
        asm volatile("ds_write_b32 %0, %1 offset:%2" : : "v"(a), "v"(live ? cs : 0.f), "n"(OFF) : "memory");
      }
      cs0 = 0.f; cs1 = 0.f;
    }
  };
  // my share of tile s has landed when at most the later requests (up to PD-1 tiles) are outstanding; then the
  // barrier: a plain s_barrier, not __syncthreads(), whose fence waits for ALL outstanding loads and would drain
  // the ring.  After it everybody's share of tile s is in LDS (each wave waited for its own loads) and everybody
  // is done reading tile s-1's slot, which the next request overwrites.
  auto tile_ready = [&](int s, auto slot_tag) __attribute__((always_inline)) {
    const int later = min(PD - 1, nsub - 1 - s);
    if (later >= 3) wait_vmcnt<3 * IPW>();
    else if (later == 2) wait_vmcnt<2 * IPW>();
    else if (later == 1) wait_vmcnt<IPW>();
    else wait_vmcnt<0>();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (s + PD < nsub) {
      if constexpr (std::is_same<decltype(slot_tag), int>::value) issue_tile(s + PD, (s + PD) % NBUF);
      else issue_tile(s + PD, IntC<(decltype(slot_tag)::value + PD) % NBUF>{});
    }
  };
  // one tile per step: row block 1's MFMAs run under row block 0's softmax.  While a wave still has MFMAs to
  // issue it runs at a raised priority, and drops back for the trailing softmax, which is vector work only: the
  // SIMD's other waves then get their MFMAs out ahead of it and the matrix pipe idles less (-3.5 % / -5 %).
  auto rest_of_tile = [&](auto masked_tag, int jbase, auto fixed_tag) __attribute__((always_inline)) {
    if constexpr (NRB == 2) {
      __builtin_amdgcn_s_setprio(1);
      mfma_block(acc1, kf, IntC<NRB - 1>{});
      softmax_block(masked_tag, acc0, IntC<0>{}, jbase, fixed_tag);
      interleave_hint();
      __builtin_amdgcn_s_setprio(0);
      softmax_block(masked_tag, acc1, IntC<NRB - 1>{}, jbase, fixed_tag);
    } else {
      softmax_block(masked_tag, acc0, IntC<0>{}, jbase, fixed_tag);
    }
  };
  // fixed_mode: pass 1 with the fixed reference (every tile but the chunk's first, which sets it)
  auto tile_step = [&](int s, auto slot_tag, auto fixed_mode) __attribute__((always_inline)) {
    tile_ready(s, slot_tag);
    read_tile(slot_tag);
    mfma_block(acc0, kf, IntC<0>{});
    // the column sums of tile s-2 are added up under those MFMAs, when the wave has nothing else to issue
    // (parked in step s-2; every wave has since waited for the operand reads of tile s-1 and passed the
    // barrier of tile s)
    if (s >= 2) {
      if constexpr (std::is_same<decltype(slot_tag), int>::value) flush_colsum(s - 2, (s - 2) % 4);
      else flush_colsum(s - 2, IntC<(decltype(slot_tag)::value + 2) % 4>{});
    }
    const int jbase = key0 + 32 * s;
    // pass 1 masks the ragged tail and the causal triangle; pass 2 only the causal triangle
    const bool masked = PASS == 1 ? (jbase + 32 > n_full) : (causal && jbase + 32 > n_full);
    if (!masked) rest_of_tile(BoolC<false>{}, jbase, fixed_mode);
    else         rest_of_tile(BoolC<true>{}, jbase, fixed_mode);
    if constexpr (std::is_same<decltype(slot_tag), int>::value) park_colsum(jbase, s % 4);
    else park_colsum(jbase, slot_tag);
  };
  // the whole key chunk: prologue (request the first PD tiles), then the loop, unrolled over the ring slots
  // (-2 %: a tile's ring slot, and with four slots its column-sum slot (tile mod 4), are compile-time numbers
  // inside a step)
  auto run_chunk = [&](auto fixed_mode) __attribute__((always_inline)) {
    if (0 < PD && 0 < nsub) issue_tile(0, IntC<0>{});
    if (1 < PD && 1 < nsub) issue_tile(1, IntC<1 % NBUF>{});
    if (2 < PD && 2 < nsub) issue_tile(2, IntC<2 % NBUF>{});
    // the first tile on its own (it sets the reference when that is fixed), then groups of NBUF tiles
    if (nsub > 0) tile_step(0, IntC<0>{}, BoolC<false>{});
    for (int s0 = 0; s0 + 1 < nsub; s0 += NBUF) {
      tile_step(s0 + 1, IntC<1 % NBUF>{}, fixed_mode);
      if constexpr (NBUF == 4) {
        if (s0 + 2 < nsub) tile_step(s0 + 2, IntC<2>{}, fixed_mode);
        if (s0 + 3 < nsub) tile_step(s0 + 3, IntC<3>{}, fixed_mode);
      }
      if (s0 + NBUF < nsub) tile_step(s0 + NBUF, IntC<0>{}, fixed_mode);
    }
  };
  static_assert(PD <= 3, "prologue written out for up to three tiles ahead");
  if constexpr (PASS == 1) {
    // Fast run with the fixed reference; then a workgroup-wide vote (every wave has to take part in a rerun:
    // they load the tiles together).  A sum whose exponent shows that some logit lay 2^60 above its row's
    // reference (or that is inf / NaN) sends the workgroup through the chunk again with the running maximum.
    const uint32_t flag_lds = __builtin_amdgcn_groupstaticsize();   // one word of dynamic LDS
    if (threadIdx.x == 0) asm volatile("ds_write_b32 %0, %1" : : "v"(flag_lds), "v"(0) : "memory");
    run_chunk(BoolC<true>{});
    bool suspect = false;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const uint32_t ez = (__float_as_uint(Z[rb]) >> 23) & 0xFFu, ee = (__float_as_uint(E[rb]) >> 23) & 0xFFu;
      suspect = suspect || ez >= 127u + 60u || ee >= 127u + 66u;
    }
    if (nsub > 0) {   // (with no tile there was no barrier either: nothing ran, nothing to vote on)
      if (__builtin_amdgcn_ballot_w64(suspect) != 0 && lane == 0)
        asm volatile("ds_write_b32 %0, %1" : : "v"(flag_lds), "v"(1) : "memory");
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __syncthreads();
      int flag;
      asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(flag) : "v"(flag_lds) : "memory");
      if (__builtin_amdgcn_readfirstlane(flag) != 0) {
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) { M[rb] = kNegBig; Z[rb] = 0.f; E[rb] = 0.f; }
        run_chunk(BoolC<false>{});
      }
    }
  } else {
    run_chunk(BoolC<false>{});
  }
  static_assert(NW == 1 || NBUF == 4, "the parked column sums use the ring slot number as tile mod 4");
  static_assert(NBUF == 2 || NBUF == 4, "key loop unrolled over the ring slots");

  if constexpr (PASS == 2 && PLANES) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
    // plane of (wave, block): g*RC*PPW + (row-chunk)*PPW + block; row-chunks beyond RC do not exist
    constexpr int NP = PLANES ? PPW : 1;
    const int rc0 = (int)(t % rcg) * NW;
    for (int pl = 0; pl < NW * NP; ++pl) {
      if (rc0 + pl / NP >= RC) break;
      float* out = colsum + ((int64_t)g * RC * NP + (int64_t)rc0 * NP + pl) * total + tok0 + key0;
      for (int i = threadIdx.x; i < 32 * (nsub - kPlanesDirectTiles); i += 64 * NW) {   // (the last tiles' sums are there already)
        float v;
        const uint32_t a = csout_lds + (uint32_t)(pl * KCAP + i) * 4u;
        asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a));
        out[i] = v;
      }
    }
  } else if (PASS == 2) {
    if (NW > 1) {
      // the asm LDS writes are unknown to the compiler, so the barriers' own fences do not wait for them
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __syncthreads();
#pragma unroll
      for (int t = 3; t >= 1; --t)
        if (nsub >= t) flush_colsum(nsub - t, (nsub - t) % 4);   // (the oldest of the three may have been added up already)
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
    float* out = colsum + (int64_t)plane * total + tok0 + key0;
    for (int i = threadIdx.x; i < key_end - key0; i += 64 * NW) {
      float v;
      asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(csout_lds + (uint32_t)i * 4u));
      out[i] = v;
    }
  }

  if (PASS == 1) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      // the two lane halves hold disjoint key subsets of the same query row
      const float M2 = __shfl_xor(M[rb], 32), Z2 = __shfl_xor(Z[rb], 32), E2 = __shfl_xor(E[rb], 32);
      const float Mn = fmaxf(M[rb], M2);
      const float d1 = M[rb] - Mn, d2 = M2 - Mn;
      const float f1 = __builtin_amdgcn_exp2f(d1), f2 = __builtin_amdgcn_exp2f(d2);
      const float En = (E[rb] + d1 * Z[rb]) * f1 + (E2 + d2 * Z2) * f2;
      const float Zn = Z[rb] * f1 + Z2 * f2;
      if (live && lh == 0) {
        float* sp = stats + (((int64_t)grc * n_chunks + chunk) * 3) * RPC + rb * 32 + l32;
        sp[0] = Mn;
        sp[RPC] = Zn;
        sp[2 * RPC] = En;
      }
    }
  }
}

template <int D, int NRB, int NW, int NBUF>
hipError_t launch_ring_cfg(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq, const void* q,
                           const void* k, int64_t ksh, int64_t kst, float c2, float* stats,
                           const float* lse2, float* colsum, int64_t total, float* probs, int pass,
                           hipStream_t st) {
  const int64_t grid = (int64_t)s.n_kv_heads * ceil_div(p.RC, NW) * p.grid_chunks;
  dim3 g((unsigned)grid), blk(64 * NW);
  // pass 2: dynamic LDS for the column sums of the key chunk and the waves' parked sums
  const int ppw = pass == 2 && probs == nullptr ? p.planes : 0;
  const unsigned cs_bytes = ppw ? (unsigned)(NW * (NW == 4 ? 1280 : 928) * 4)   // NW * PPW * kPlanesLdsKeys<NW, PPW> * 4 at most
                                : (unsigned)(kKeyCap<NW> * 4 + (NW > 1 ? 4 * NW * 64 * 4 : 0));
  const unsigned dyn = pass == 1 ? 16u : cs_bytes;   // pass 1: the word of the rerun vote
#define SKV_ARGS                                                                                        \
  g, blk, dyn, st, (const uint16_t*)q, (const uint16_t*)k, ksh, kst, p.kshare, seq, s.n_q_heads, s.n_kv_heads, \
      s.window, s.causal, c2, p.R, p.RC, p.KC, p.n_chunks, stats, lse2, colsum, total, probs
  if (pass == 1 && p.stream_k) hipLaunchKernelGGL((score_mfma_ring_kernel<D, NRB, NW, NBUF, 1, false, 0, true>), SKV_ARGS);
  else if (pass == 1) hipLaunchKernelGGL((score_mfma_ring_kernel<D, NRB, NW, NBUF, 1, false>), SKV_ARGS);
  else if (ppw == 1) hipLaunchKernelGGL((score_mfma_ring_kernel<D, NRB, NW, NBUF, 2, false, 1>), SKV_ARGS);
  else if (ppw == 2) {
    if constexpr (NRB == 2) hipLaunchKernelGGL((score_mfma_ring_kernel<D, NRB, NW, NBUF, 2, false, 2>), SKV_ARGS);
    else return hipErrorInvalidValue;
  }
  else if (probs == nullptr && p.stream_k)
    hipLaunchKernelGGL((score_mfma_ring_kernel<D, NRB, NW, NBUF, 2, false, 0, true>), SKV_ARGS);
  else if (probs == nullptr) hipLaunchKernelGGL((score_mfma_ring_kernel<D, NRB, NW, NBUF, 2, false>), SKV_ARGS);
  else hipLaunchKernelGGL((score_mfma_ring_kernel<D, NRB, NW, NBUF, 2, true>), SKV_ARGS);
#undef SKV_ARGS
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_mfma_ring(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                                  const void* q, const void* k, int64_t ksh, int64_t kst, float c2,
                                  float* stats, const float* lse2, float* colsum, int64_t total,
                                  float* probs, int pass, hipStream_t st) {
  if (p.grid_chunks == 0) return hipSuccess;
  // four waves per workgroup (row-chunks of 64 rows for a KV group of more than 128 rows, of 32 rows for 65..128)
  // with a 4-tile ring; up to 64 rows: single-wave workgroups with a 2-tile ring (eight of them share a CU's LDS)
#define SKV_RING(d, nrb, nw, nbuf)                                                                      \
  if (s.head_dim == d && p.RB == nrb && p.NW == nw)                                                      \
    return launch_ring_cfg<d, nrb, nw, nbuf>(s, p, seq, q, k, ksh, kst, c2, stats, lse2, colsum, total, probs, pass, st)
  SKV_RING(128, 2, 4, 4);
  SKV_RING(128, 1, 4, 4);
  SKV_RING(128, 2, 1, 2);
  SKV_RING(128, 1, 1, 2);
  SKV_RING(64, 2, 4, 4);
  SKV_RING(64, 1, 4, 4);
  SKV_RING(64, 2, 1, 2);
  SKV_RING(64, 1, 1, 2);
#undef SKV_RING
  return hipErrorInvalidValue;
}

}  // namespace skv
