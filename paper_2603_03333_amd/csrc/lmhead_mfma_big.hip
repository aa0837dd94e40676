// Eq. (3) l = W h^(i) with a fused per-row argmax on the gfx950 matrix cores, for more than
// 128 masked rows (the MFMA-bound regime: batches of sequences, draft trees).
//
// Same operand roles as the small-row kernel (W rows = MFMA "A" operand, masked rows = "B"
// operand, so a lane owns one masked row and the vocabulary argmax is a per-lane compare),
// but a 256 x 256 output tile per workgroup: at 256 x 128 a CU needs 47 B/clk from L2 to keep
// its matrix cores busy, which the L2 fabric does not deliver to 256 CUs at once (measured:
// 39 % of MFMA peak); 256 x 256 halves that.
//
// Workgroup = 768 threads = 12 wavefronts, three per SIMD:
//   * 8 consumers: wavefront (wv, wm) owns vocabulary rows [64 wv, +64) x masked rows
//     [128 wm, +128) of the tile: 4 x 8 accumulator tiles of v_mfma_f32_16x16x32_bf16 (128 VGPRs; the
//     same flops and the same LDS fragment traffic as 2 x 4 tiles of the 32x32x16 instruction, which this
//     kernel used first, at less power: batched 6.51 -> 6.22 ms on one box);
//   * 4 producers: global -> LDS copies by LDS-DMA, so that a full memory queue stalls a
//     producer and not the MFMA stream.
// k advances in slabs of 64.  LDS holds a ring of three W slabs (two in flight: they come from
// HBM or the memory-side cache) and a ring of two slabs of masked rows (one in flight: they are
// re-read from L2 by every workgroup), 3 x 32 KB + 2 x 32 KB = all of the 160 KB; one workgroup
// barrier per slab: "slab q has landed for everybody, nobody reads slab q-1 any more".  The four
// wavefronts that share a masked row merge their arg max through the 64-bit key in memory.
// W rows are stored in LDS with their 16-byte pieces XOR-swizzled by the row number so that
// the MFMA fragment reads (16 rows each of 4 consecutive pieces) are bank-conflict free; masked rows
// arrive in fragment order from the mask kernel.
//
// Tile order.  Workgroups are persistent; in one "round" the grid covers a block of
// BVc x BMc tiles (BMc <= 16 row tiles wide).  Workgroup ids are dealt round-robin to the 8
// XCDs, each with its own L2, so the 32 workgroups of an XCD take a compact patch of
// sv x sm tiles (sm <= 4): a slab of masked rows is fetched into that L2 once per sv
// workgroups and a slab of W once per sm workgroups.  Rounds sweep the vocabulary first, so
// across the chip W streams from HBM once per sweep of up to 16 row tiles.
#include "kernels.hpp"
#include "mfma_common.hpp"
#include "sampling.hpp"

namespace dm {
namespace {

constexpr int BN = 256;  // vocabulary rows per tile
constexpr int BM = 256;  // masked rows per tile
constexpr int THREADS = 768;
constexpr int kNoiseMinChunks = 16;  // tiles of fewer slabs draw their noise in the epilogue

template <int BK>
struct Cfg {
  static constexpr int PR = BK / 8;                    // 16-byte pieces per W row per slab
  static constexpr int KSTEPS = BK / 32;               // MFMA k-steps (of 32) per slab
  static constexpr int ROW_BYTES = BK * 2;
  static constexpr int W_SLAB = BN * ROW_BYTES;
  static constexpr int A_SLAB = BM * ROW_BYTES;
  static constexpr int W_INSTR = (64 * ROW_BYTES) / 1024;  // W copy instructions per producer per slab
  static constexpr int A_INSTR = KSTEPS * 16 / 4;          // masked-row fragments (16 rows x 32 k) per producer per slab
  // W slabs come from HBM (long latency), masked-row slabs from L2: W gets the deeper ring.
  // 3 x 32 KB + 2 x 32 KB = all 160 KB of the LDS at BK = 64.
  static constexpr int NSW = 3, NSA = 2;
  static constexpr int A_BASE = NSW * W_SLAB;
  static constexpr int LDS_BYTES = NSW * W_SLAB + NSA * A_SLAB;
  static constexpr int SWZ_SHIFT = (BK == 64) ? 1 : 2;     // rows per 256-byte bank period: 2 or 4
};
static_assert(Cfg<64>::LDS_BYTES <= 160 * 1024, "LDS of a gfx950 compute unit");

// How the persistent grid walks the NV x NMB tiles (filled on the host).
struct TileWalk {
  int NV, NMB;      // tiles along the vocabulary / along masked rows
  int BVc, BMc;     // tiles covered by the whole grid in one round
  int nvb, nmb;     // rounds along the vocabulary / along masked rows
  int xcd_aware;    // deal compact sv x sm patches to the XCDs
  int sv, sm, pm;   // patch shape, patches per block row
};

struct TilePos {
  int dv, dm;
  bool active;
};

__device__ __forceinline__ TilePos tile_pos(const TileWalk& w, int g) {
  TilePos p;
  if (w.xcd_aware) {
    const int xcd = g & 7, slot = g >> 3;
    const int pv = xcd / w.pm, pmi = xcd - pv * w.pm;
    const int sl_v = slot / w.sm, sl_m = slot - sl_v * w.sm;
    p.dv = pv * w.sv + sl_v;
    p.dm = pmi * w.sm + sl_m;
  } else {
    p.dv = g / w.BMc;
    p.dm = g - p.dv * w.BMc;
  }
  p.active = p.dv < w.BVc && p.dm < w.BMc;
  return p;
}

// Tile of round `it` for a workgroup at block position p; false if it falls outside the problem.
__device__ __forceinline__ bool tile_of(const TileWalk& w, const TilePos& p, int it, int& tv, int& tm) {
  const int mB = it / w.nvb, vb = it - mB * w.nvb;
  tv = vb * w.BVc + p.dv;
  tm = mB * w.BMc + p.dm;
  return p.active && tv < w.NV && tm < w.NMB;
}

// MODE 0: argmax keys only; MODE 1: debug dump of logits[M, dv1 - dv0]; MODE 2: argmax keys and every
// scaled logit stored in the layout [position][vocabulary row][path] for the distribution-level rule.
// SAMPLE (MODE 0 only): arg max over zscale * logit + Gumbel noise = a draw from Softmax(logit / temperature);
// 1: the noise is drawn in the epilogue (tiles of few slabs), 2: by the copy wavefronts during the tile.
template <int BK, int MODE, int SAMPLE>
__global__ __launch_bounds__(THREADS, 3) void lmhead_mfma_big_kernel(const __bf16* __restrict__ W,
                                                                     const __bf16* __restrict__ A_sw,
                                                                     unsigned long long* __restrict__ keys, int d,
                                                                     int64_t M, int mt_total, int v_lo, int v_hi,
                                                                     TileWalk walk, float* __restrict__ logits,
                                                                     int dv0, int dv1, float scale,
                                                                     LogitStore store, SampleCfg samp) {
  using C = Cfg<BK>;
  constexpr bool DUMP = MODE == 1;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nchunks = d / BK;
  const TilePos pos = tile_pos(walk, (int)blockIdx.x);
  const int nit = walk.nvb * walk.nmb;

  int my_tiles = 0;
  for (int it = 0; it < nit; ++it) {
    int tv, tm;
    my_tiles += tile_of(walk, pos, it, tv, tm) ? 1 : 0;
  }
  const int total = my_tiles * nchunks;
  // k rotation: shared by the workgroups of one XCD (they reuse each other's slabs in L2 only if
  // they want the same slab at about the same time), different between XCDs (so the XCDs do not
  // all pull the same address bits, i.e. the same memory channels, at once)
  const int rot = (int)(((blockIdx.x & 7u) * (unsigned)nchunks) / 8u);

  if (wave >= 8) {
    // ------------------------------------------------------------------ producer
    __builtin_amdgcn_s_setprio(3);
    const int p = wave - 8;
    constexpr int RPI = 64 / C::PR;  // W rows per copy instruction
    const int ld_row = lane / C::PR;
    const int ld_slot = lane % C::PR;
    // Addresses are "uniform 64-bit base + 32-bit lane offset": the lane offsets are fixed for the
    // whole kernel, the bases are scalar arithmetic, so a copy costs the producer no vector ALU work.
    uint32_t woff[C::W_INSTR];
#pragma unroll
    for (int rb = 0; rb < C::W_INSTR; ++rb) {
      const int row = RPI * rb + ld_row;  // row inside this producer's 64
      const int piece = ld_slot ^ ((row >> C::SWZ_SHIFT) & (C::PR - 1));
      woff[rb] = (uint32_t)row * (uint32_t)(2 * d) + (uint32_t)piece * 16u;
    }
    const uint32_t aoff = (uint32_t)lane * 16u;
    const char* Wb = reinterpret_cast<const char*>(W);
    const char* Ab = reinterpret_cast<const char*>(A_sw);
    struct Cursor {
      int it = -1, c = 0, tv = 0, tm = 0;
    };
    Cursor cw, ca;
    cw.c = ca.c = nchunks;
    auto advance = [&](Cursor& cu) {  // returns the k chunk of the cursor's next slab
      if (cu.c == nchunks) {
        cu.c = 0;
        do {
          ++cu.it;
        } while (!tile_of(walk, pos, cu.it, cu.tv, cu.tm) && cu.it < nit);
        if (cu.it >= nit) cu.tv = cu.tm = 0;  // cannot happen (slabs are counted from the same walk); stays in bounds
      }
      int c = cu.c + rot;
      c = c >= nchunks ? c - nchunks : c;
      ++cu.c;
      return c;
    };
    auto issue_w = [&](int q) {
      const int c = advance(cw);
      const int v0 = v_lo + cw.tv * BN + 64 * p;
      unsigned char* stage = lds + (q % C::NSW) * C::W_SLAB;
      const char* wsrc = Wb + ((int64_t)v0 * d + (int64_t)c * BK) * 2;
      if (v0 + 64 <= v_hi) {
#pragma unroll
        for (int rb = 0; rb < C::W_INSTR; ++rb)
          dma_copy16(wsrc, woff[rb], stage + p * (64 * C::ROW_BYTES) + rb * 1024);
      } else {  // last vocabulary tile: rows past the end re-read the last row, masked out later
#pragma unroll
        for (int rb = 0; rb < C::W_INSTR; ++rb) {
          const int row = RPI * rb + ld_row;
          const int vrow = (v0 + row < v_hi) ? v0 + row : v_hi - 1;
          const int piece = ld_slot ^ ((row >> C::SWZ_SHIFT) & (C::PR - 1));
          const __bf16* src = W + (int64_t)vrow * d + c * BK + piece * 8;
          __builtin_amdgcn_global_load_lds(DM_GLOBAL_PTR(src),
                                           DM_LDS_PTR(stage + p * (64 * C::ROW_BYTES) + rb * 1024), 16, 0, 0);
        }
      }
    };
    auto issue_a = [&](int q) {
      const int c = advance(ca);
      unsigned char* stage = lds + C::A_BASE + (q % C::NSA) * C::A_SLAB;
      const char* asrc = Ab + ((int64_t)(c * C::KSTEPS) * mt_total + ca.tm * 16) * 1024;
#pragma unroll
      for (int x = 0; x < C::A_INSTR; ++x) {
        const int f = p + 4 * x;  // fragment index inside the slab: f = s * 16 + mt
        const int s = f >> 4, mt = f & 15;
        dma_copy16(asrc + ((int64_t)s * mt_total + mt) * 1024, aoff, stage + f * 1024);
      }
    };
    // SAMPLE == 2: the copy wavefronts, idle most of the time, also draw the Gumbel noise of the tile
    // the MFMA wavefronts are working on: 256 "items" of 64 lanes x 4 vocabulary rows (one Philox block
    // per lane) per tile, spread over the tile's slabs and left in memory in the order the MFMA
    // wavefronts read them in their epilogue.  (Drawn in the epilogue, the noise also costs the main
    // loop registers it does not have.)  Copy wavefront p makes the 64 items with vocabulary tile w = p:
    // item k = ((wm * 8 + a) * 4 + wv) of MFMA wavefront (wv, wm), masked-row tile a, stored at float4
    // index (4 k + w) * 64 + lane.  Four consecutive items share their 16 masked rows, so the rows'
    // streams are set up once per four.  Items of a tile are made
    // after the barrier of its first slab (the epilogue of the tile before has been read by then) and
    // are complete, by a wait for ALL own memory operations, before the barrier of its last slab.
    constexpr bool prod_noise = SAMPLE == 2;
    Cursor cn;
    cn.c = nchunks;
    int items_done = 0;
    RowRng nrng{0u, 0u, 0u, 0u, false};
    f32x4* const noise_wg = reinterpret_cast<f32x4*>(samp.noise) + (int64_t)blockIdx.x * (BN * BM / 4);
    auto noise_item = [&](int k, int tv, int tm) {
      const int rs = k >> 2, wv_k = k & 3;  // rs = wm * 8 + a
      if ((k & 3) == 0) nrng = make_row_rng(samp, (int64_t)tm * BM + (rs >> 3) * 128 + (rs & 7) * 16 + (lane & 15), M);
      const int v4 = v_lo + tv * BN + 64 * wv_k + 16 * p + 4 * (lane >> 4);
      float g[4] = {0.f, 0.f, 0.f, 0.f};
      if (nrng.on) gumbel4(nrng, (uint32_t)v4, step_now(samp.step, samp.step_dev), g);
      // written once, read once, by this compute unit: streaming, so that it does not displace the W and
      // masked-row slabs the workgroups of the XCD share through L2
      __builtin_nontemporal_store(f32x4{g[0], g[1], g[2], g[3]}, noise_wg + (4 * k + p) * 64 + lane);
    };
    // issue order: W(0) A(0) W(1) | barrier 0 | A(1) W(2) | barrier 1 | A(2) W(3) | ...
    // before barrier q everything but the youngest W slab (q+1, if there is one) has landed
    if (total > 0) {  // a workgroup without tiles has no first slab to look for
      issue_w(0);
      issue_a(0);
    }
    if (total > 1) issue_w(1);
    for (int q = 0; q < total; ++q) {
      // Copies complete in issue order, so "at most the youngest W slab outstanding" means slab q has landed;
      // noise stores in between (which may complete out of order) only make that wait more conservative.
      // Before the barrier of a tile's last slab the noise stores themselves must be complete: wait for all.
      if (q + 1 < total && !(prod_noise && q % nchunks == nchunks - 1)) {
        DM_WAIT_VMCNT(C::W_INSTR);
      } else {
        DM_WAIT_VMCNT(0);
      }
      DM_BARRIER();  // slab q complete for everyone; slab q-1 consumed by everyone
      if (q + 1 < total) issue_a(q + 1);
      if (q + 2 < total) issue_w(q + 2);
      if (prod_noise) {
        (void)advance(cn);         // tile of slab q
        const int sl = cn.c - 1;   // slab q's index inside its tile
        if (sl == 0) items_done = 0;
        if (sl < nchunks - 1) {    // this wavefront's 64 items, evenly over the tile's first nchunks - 1 slabs
          const int target = (64 * (sl + 1) + (nchunks - 2)) / (nchunks - 1);
          for (; items_done < target; ++items_done) noise_item(items_done, cn.tv, cn.tm);
        }
      }
    }
    return;
  }

  // -------------------------------------------------------------------- consumer
  const int wv = wave & 3, wm = wave >> 2;
  const int i16 = lane & 15;  // row inside a 16-row MFMA tile (vocabulary row of W, masked row of the B operand)
  const int kq = lane >> 4;   // which 8 of the 32 k of an MFMA step; in the accumulators: which 4 of the 16 vocabulary rows
  // W fragment of vocabulary tile w (16 rows), k-step s (32 k): piece (4 s + kq) ^ swz = (4 s) ^ (kq ^ swz) of the
  // lane's row (swz depends on i16 only: tiles start at multiples of 16 rows).  Every other term of the address
  // is a multiple of the row size, so the k-step is an XOR on ONE lane offset instead of one precomputed
  // register per k-step.
  static_assert(C::ROW_BYTES == 16 * C::PR && C::W_SLAB % C::ROW_BYTES == 0, "piece index = low bits of the address");
  static_assert(C::PR >= 4, "a k-step of 32 spans four 16-byte pieces");
  const uint32_t wlane = (uint32_t)(wv * (64 * C::ROW_BYTES) + i16 * C::ROW_BYTES +
                                    16 * (kq ^ ((i16 >> C::SWZ_SHIFT) & (C::PR - 1))));

  // acc[a][w][r]: masked row 16 a + i16 of the wavefront's 128, vocabulary row 16 w + 4 kq + r of its 64
  f32x4 acc[8][4];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[a][w][r] = 0.f;

  int it_c = -1, tv_c = 0, tm_c = 0;
  for (int q = 0; q < total; ++q) {
    DM_BARRIER();
    const uint32_t wq = (uint32_t)((q % C::NSW) * C::W_SLAB) + wlane;
    const unsigned char* abase = lds + C::A_BASE + (q % C::NSA) * C::A_SLAB + (8 * wm) * 1024 + lane * 16;
    // Fragments are requested ahead of their use by hand: that of masked-row tile a + 1 before the four MFMAs of
    // tile a, and inside a slab the W fragments of the next k-step one by one behind the last MFMA that reads the
    // register they go to.  Left to itself the compiler requests each fragment right before its use and waits
    // for it on the spot (measured: 6.65 ms at the batched configuration against 5.93 ms with the first kind of
    // request pinned ahead and 5.90 ms with both; two tiles ahead: 5.99 ms; a slab's first requests in the order
    // of their first use: no change, the compiler waits for all of them before the first MFMA either way).
    bf16x8 wf[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) wf[w] = *reinterpret_cast<const bf16x8*>(lds + wq + w * (16 * C::ROW_BYTES));
    bf16x8 af = *reinterpret_cast<const bf16x8*>(abase);
#pragma unroll
    for (int s = 0; s < C::KSTEPS; ++s) {
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        const bool more = a < 7 || s + 1 < C::KSTEPS;  // another masked-row fragment in this slab
        bf16x8 af_next = af;
        if (more) af_next = *reinterpret_cast<const bf16x8*>(abase + (a < 7 ? s * 16 + a + 1 : (s + 1) * 16) * 1024);
        __builtin_amdgcn_sched_barrier(0);  // keeps the request above ahead of the MFMAs below
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          acc[a][w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[w], af, acc[a][w], 0, 0, 0);
          if (a == 7 && s + 1 < C::KSTEPS) {
            __builtin_amdgcn_sched_barrier(0);
            wf[w] = *reinterpret_cast<const bf16x8*>(lds + (wq ^ (uint32_t)(64 * (s + 1))) + w * (16 * C::ROW_BYTES));
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        af = af_next;
      }
    }
    asm volatile("" ::: "memory");

    if ((q % nchunks) != nchunks - 1) continue;

    // ---- tile finished ----
    do {
      ++it_c;
    } while (!tile_of(walk, pos, it_c, tv_c, tm_c) && it_c < nit);
    if (it_c >= nit) tv_c = tm_c = 0;  // cannot happen (slabs are counted from the same walk); stays in bounds
    const int v0 = v_lo + tv_c * BN;
    const int64_t m_first = (int64_t)tm_c * BM + wm * 128;  // first masked row of this wavefront
    // accumulator (a, w, r): v = v0 + 64 wv + 16 w + 4 kq + r,  m = m_first + 16 a + lane % 16
    if (DUMP) {
      const int nv = dv1 - dv0;
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        const int64_t m = m_first + a * 16 + i16;
        const float sc = (store.clean_last && m % store.K == store.K - 1) ? 1.0f : scale;  // clean path: no 1/(1-p)
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int v = v0 + 64 * wv + 16 * w + 4 * kq + r;
            if (m < M && v >= dv0 && v < dv1 && v < v_hi) logits[m * nv + (v - dv0)] = sc * acc[a][w][r];
            acc[a][w][r] = 0.f;
          }
      }
      continue;
    }

    if (MODE == 2) {
      // row m = path m % K of position m / K; stores use a uniform base (first position of this
      // wavefront's 128 rows) plus one 32-bit lane offset
      const int64_t pos0 = m_first / store.K;
      char* lt_base = reinterpret_cast<char*>(store.lt + pos0 * store.V * (int64_t)store.K4);
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        const int64_t m = m_first + a * 16 + i16;
        const int64_t pos = m / store.K;
        const uint32_t lt_off = (uint32_t)(((pos - pos0) * store.V * store.K4 + (m - pos * store.K) + 4 * kq * store.K4) * 4);
        if (m < M) {
#pragma unroll
          for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int vu = v0 + 64 * wv + 16 * w + r;  // + 4 * kq per lane; the base below is uniform over the wavefront
              char* dst = lt_base + (int64_t)vu * store.K4 * 4;
              if (vu + 4 * kq < v_hi) *reinterpret_cast<float*>(dst + lt_off) = scale * acc[a][w][r];
            }
        }
      }
    }

    if (SAMPLE == 0 && v0 + BN <= v_hi) {
      // Plain arg max over a full tile (all but the last vocabulary tile): no bounds checks, the winner is
      // tracked as a 4-bit code and turned into its row once, -0 becomes +0 once (for the comparisons the
      // two are equal; the packed key orders them, and ties must go to the smaller index in every tile).
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        float best = acc[a][0][0];
        int code = 0;
        acc[a][0][0] = 0.f;
#pragma unroll
        for (int c = 1; c < 16; ++c) {  // ascending v for this lane: strict > keeps the smallest index
          const float val = acc[a][c >> 2][c & 3];
          const bool gt = val > best;
          best = gt ? val : best;
          code = gt ? c : code;
          acc[a][c >> 2][c & 3] = 0.f;
        }
        const int v = v0 + 64 * wv + 4 * kq + 16 * (code >> 2) + (code & 3);
        unsigned long long key = pack_key(best + 0.0f, (uint32_t)v);
        unsigned long long other = __shfl_xor(key, 16, 64);
        key = other > key ? other : key;
        other = __shfl_xor(key, 32, 64);
        key = other > key ? other : key;
        const int64_t mrow = m_first + a * 16 + i16;
        if (kq == 0 && mrow < M) atomicMax(&keys[mrow], key);
      }
      continue;
    }

#pragma unroll
    for (int a = 0; a < 8; ++a) {
      float best = -INFINITY;
      uint32_t bv = 0xFFFFFFFFu;
      const int64_t mrow = m_first + a * 16 + i16;
      RowRng rng{0u, 0u, 0u, 0u, false};
      if (SAMPLE == 1) rng = make_row_rng(samp, mrow, M);
      const bool noisy = SAMPLE == 1 ? rng.on : (SAMPLE == 2 && row_draws(samp, mrow, M));
      // SAMPLE == 2: noise made by the copy wavefronts during the tile, items (wm, a, wv), vocabulary tile 0 onwards
      // (a uniform base and one lane offset, opaque so that the 32 addresses are not kept across the tile)
      const char* nz = reinterpret_cast<const char*>(samp.noise) + (int64_t)blockIdx.x * (BN * BM * 4) +
                       ((((wm * 8 + a) * 4 + wv) * 4) * 1024);
      uint32_t nlane = (uint32_t)lane * 16u;
      if (SAMPLE == 2) asm volatile("" : "+v"(nlane));
      // First vocabulary row of this lane in the tile.  When sampling it is made opaque to the compiler
      // for every masked-row tile: otherwise whatever depends on the vocabulary row only (noise
      // counters, the first Philox round) is shared between the tiles, kept in registers across
      // the main loop, and spilled there.
      int vb = v0 + 64 * wv + 4 * kq;
      if (SAMPLE == 1) asm volatile("" : "+v"(vb));
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float g[4] = {0.f, 0.f, 0.f, 0.f};
        if (SAMPLE == 2) {
          const f32x4 g4 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(nz + w * 1024 + nlane));
          g[0] = g4.x;
          g[1] = g4.y;
          g[2] = g4.z;
          g[3] = g4.w;
        } else if (noisy) {
          gumbel4(rng, (uint32_t)(vb + 16 * w), step_now(samp.step, samp.step_dev), g);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {  // ascending v for this lane: strict > keeps the smallest index
          const int v = vb + 16 * w + e;
          const float val = noisy ? fmaf(acc[a][w][e], samp.zscale, g[e]) : acc[a][w][e] + 0.0f;
          if (v < v_hi && (bv == 0xFFFFFFFFu || val > best)) {
            best = val;
            bv = (uint32_t)v;
          }
          acc[a][w][e] = 0.f;
        }
        // the noise of one group of four rows is not computed ahead of the groups before it
        if (SAMPLE == 1) __builtin_amdgcn_sched_barrier(0);
      }
      unsigned long long key = (bv == 0xFFFFFFFFu) ? 0ull : pack_key(best, bv);
      unsigned long long other = __shfl_xor(key, 16, 64);
      key = other > key ? other : key;
      other = __shfl_xor(key, 32, 64);
      key = other > key ? other : key;
      // no LDS left for a reduction over the four wavefronts that share a masked row: each merges its own
      if (kq == 0 && mrow < M && key != 0ull) atomicMax(&keys[mrow], key);
    }
  }
}

int pow2_at_most(int x) {
  int p = 1;
  while (2 * p <= x) p *= 2;
  return p;
}

TileWalk make_walk(int NV, int NMB, int G) {
  TileWalk w{};
  w.NV = NV;
  w.NMB = NMB;
  int bmc = pow2_at_most(NMB < 16 ? NMB : 16);
  if (bmc > G) bmc = pow2_at_most(G);
  w.BMc = bmc;
  w.xcd_aware = 0;
  w.sv = w.sm = w.pm = 1;
  if (G % 8 == 0) {
    const int S = G / 8;
    const int sm = bmc < 4 ? bmc : 4;
    if (S % sm == 0) {
      w.xcd_aware = 1;
      w.sm = sm;
      w.sv = S / sm;
      w.pm = bmc / sm;
      w.BVc = (8 / w.pm) * w.sv;
    }
  }
  if (!w.xcd_aware) w.BVc = G / bmc;
  w.nvb = (NV + w.BVc - 1) / w.BVc;
  w.nmb = (NMB + w.BMc - 1) / w.BMc;
  return w;
}

template <int BK>
hipError_t run_big(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g, int V, int num_cu,
                   float* logits, int v0, int v1, float scale, const LogitStore& store, const SampleCfg& samp,
                   const LaunchSite& at) {
  const bool dump = logits != nullptr;
  const int v_lo = dump ? v0 : 0;
  const int v_hi = dump ? v1 : V;
  if (v_hi <= v_lo) return hipSuccess;
  const int NV = (v_hi - v_lo + BN - 1) / BN;
  const int NMB = (int)(g.M_pad / BM);
  const int64_t ntiles = (int64_t)NV * NMB;
  int G = ntiles < num_cu ? (int)ntiles : num_cu;
  if (G >= 8) G -= G % 8;
  const TileWalk walk = make_walk(NV, NMB, G);
  const dim3 grid((unsigned)G), block(THREADS);
  const int mt_total = (int)(g.M_pad >> 4);  // masked-row tiles of 16
#define DM_LAUNCH(MODE, SAMPLE)                                                                                    \
  launch_at(lmhead_mfma_big_kernel<BK, MODE, SAMPLE>, grid, block, (size_t)Cfg<BK>::LDS_BYTES, at,                  \
            static_cast<const __bf16*>(W), static_cast<const __bf16*>(a_ws), keys, g.d, g.M, mt_total, v_lo, v_hi, \
            walk, logits, v0, v1, scale, store, samp)
  if (dump)
    DM_LAUNCH(1, 0);
  else if (store.lt != nullptr)
    DM_LAUNCH(2, 0);
  else if (samp.seeds != nullptr && samp.noise != nullptr && g.d / BK >= kNoiseMinChunks)
    DM_LAUNCH(0, 2);
  else if (samp.seeds != nullptr)
    DM_LAUNCH(0, 1);
  else
    DM_LAUNCH(0, 0);
#undef DM_LAUNCH
  return hipGetLastError();
}

constexpr int kBigBK = 64;

template <int MODE, int SAMPLE>
hipError_t raise_lds_big() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_mfma_big_kernel<kBigBK, MODE, SAMPLE>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, Cfg<kBigBK>::LDS_BYTES);
}

}  // namespace

hipError_t prepare_lmhead_mfma_big() {
  hipError_t e;
  if ((e = raise_lds_big<0, 0>()) != hipSuccess) return e;
  if ((e = raise_lds_big<0, 1>()) != hipSuccess) return e;
  if ((e = raise_lds_big<0, 2>()) != hipSuccess) return e;
  if ((e = raise_lds_big<1, 0>()) != hipSuccess) return e;
  return raise_lds_big<2, 0>();
}

hipError_t launch_lmhead_mfma_big(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g, int V,
                                  int num_cu, float* logits, int v0, int v1, float scale, const LogitStore& store,
                                  const SampleCfg& samp, const LaunchSite& at) {
  if (g.M_pad % BM != 0) return hipErrorInvalidValue;
  return run_big<kBigBK>(W, a_ws, keys, g, V, num_cu, logits, v0, v1, scale, store, samp, at);
}

}  // namespace dm
