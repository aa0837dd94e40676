// Eq. (3) l = W h^(i) with a fused per-row argmax on the gfx950 matrix cores.
//
// The contraction is C[v, m] = sum_k W[v, k] * a[m, k] with W rows as the MFMA "A" operand
// (index i = vocabulary row) and the masked hidden rows as the "B" operand (index j = masked
// row).  In the accumulator layout of v_mfma_f32_16x16x32_bf16 a lane then owns ONE masked row
// (j = lane % 16) and 4 vocabulary rows per 16 x 16 tile, so the running argmax over the vocabulary
// is a per-lane compare with no cross-lane traffic; lanes meet only once per 256-row vocabulary
// tile.  (The 32x32x16 instruction, which this kernel used first, does the same flops with the
// same fragment traffic at more power: 166.8 -> 160.9 us at 128 rows on one box.)
//
// Workgroup: 512 threads = 8 wavefronts, specialised by role (two per SIMD):
//   * wavefronts 0-3, consumers: wavefront w owns vocabulary rows [64w, 64w+64) of the tile
//     (four 16-row MFMA tiles) against all 32*MT <= 128 masked rows: 4 x 2*MT accumulator tiles.
//     They only read LDS and issue MFMAs.
//   * wavefronts 4-7, producers: they only issue the global -> LDS copies.  Issuing a copy
//     blocks the wavefront while the CU's memory queue is full, which at HBM speed is most
//     of the time; in a separate wavefront that stall overlaps the MFMA work instead of
//     delaying it (measured: 250 us -> 188 us at d=4096, V=128256, 128 rows).
// k advances in slabs of 64 (one 128-byte line of each W row); three slabs live in LDS.
//
// Data movement: both operands go global -> LDS with the LDS-DMA form of global loads (no
// VGPR staging).
//   * W: one DMA instruction moves 8 rows x 128 B; eight consecutive lanes read one full
//     line of a row (coalesced), and the 16-byte piece q of row r is placed at slot
//     q ^ ((r >> 1) & 7) of the row so that the later ds_read_b128 of MFMA fragments (16
//     different rows per piece, 4 pieces) spreads over all LDS banks (measured: 0 bank conflicts).
//   * masked rows: the mask kernel has already laid them out in fragment order, so the copy
//     and the fragment reads are both linear.
// A producer waits for its own DMA of slab q with s_waitcnt vmcnt(n); one s_barrier per slab
// then tells the consumers that slab q is complete and tells the producers that slab q-1 has
// been consumed, so its buffer can take slab q+2.  The compiler does not model LDS-DMA, so
// waits and barriers are explicit and "memory" clobbers keep its LDS reads between them.
//
// Every workgroup walks k in a different rotation: all rows of a slab share the low 13
// address bits (row pitch 2*d bytes), and workgroups marching through k in lockstep would
// all hit the same memory channels at the same time (measured: 4.6 -> 6.1 TB/s for the bare
// access pattern).
//
// Workgroups are persistent and own a contiguous range of ceil(V / grid.x) vocabulary rows
// (walked in tiles of 256, the last one partial), so every CU streams the same number of
// bytes; the slab pipeline runs across tile borders.
#include "kernels.hpp"
#include "mfma_common.hpp"
#include "sampling.hpp"
#include "vote_body.hpp"

namespace dm {
namespace {

constexpr int BN = 256;                 // vocabulary rows per tile
constexpr int BK = 64;                  // k per slab
constexpr int NS = 3;                   // slabs resident in LDS
constexpr int W_SLAB_BYTES = BN * BK * 2;  // 32 KB
constexpr int THREADS = 512;

__host__ __device__ constexpr int slab_bytes(int MT) { return W_SLAB_BYTES + MT * 4 * 1024; }
__host__ __device__ constexpr int lds_bytes(int MT) { return NS * slab_bytes(MT) + 4 * MT * 32 * 8; }

// The W stream is copied with the non-temporal form (dma_copy16_stream): every byte of W is used once
// per call, so its lines should be the first to leave L2, where the masked rows (re-read by every
// workgroup for every vocabulary tile) have to stay.  Without the hint a fifth of the masked-row reads
// missed L2 and the kernel fetched 13 % more than W from memory (measured: 184 us -> 162 us at
// d=4096, V=128256).

// MODE 0: per-row argmax keys only (the verify path of the token-level rules).
// MODE 1: debug dump of scaled logits for vocabulary rows [dv0, dv1) into logits[M, dv1 - dv0].
// MODE 2: argmax keys AND every scaled logit stored for the distribution-level rule, in the
//         layout [position][vocabulary row][path] (store.lt, see LogitStore).
// SAMPLE (MODE 0 only): the per-row arg max runs over zscale * logit + Gumbel noise, i.e. the path token
//         is drawn from Softmax(logit / temperature) instead of being the arg max.
// acc[B / 4][B % 4][e] += g[e]: noise block B of a tile (the lane's 4 consecutive vocabulary rows of vocabulary
// tile B % 4, masked-row tile B / 4) goes to fixed registers, so the block number has to be a constant.
template <int MT, int B>
__device__ __forceinline__ void add_noise_block(f32x4 (&acc)[2 * MT][4], const float (&g)[4]) {
  if constexpr (B / 4 < 2 * MT) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[B / 4][B & 3][e] += g[e];
  }
}

// Sampled tokens: how many of a tile's 8 MT noise blocks are added to the accumulators during the k loop
// instead of being drawn in the epilogue.  Up to 64 rows the MFMA wavefronts wait for data half of every
// slab and take all of them (sampling then costs 2 % instead of 8 %); with more rows they have no such
// slack (measured at 128 rows: 192 us against 188 us) and the epilogue keeps the work.
__host__ __device__ constexpr int noise_blocks_in_loop(int MT) { return MT <= 2 ? 8 * MT : 0; }

template <int MT, int MODE, bool SAMPLE>
__global__ __launch_bounds__(THREADS, 2) void lmhead_mfma_kernel(const __bf16* __restrict__ W,
                                                                 const __bf16* __restrict__ A_sw,
                                                                 unsigned long long* __restrict__ keys, int d,
                                                                 int64_t M, int mt_total /* tiles of 16 rows */, int v_lo, int v_hi,
                                                                 int rows_per_wg, float* __restrict__ logits,
                                                                 int dv0, int dv1, float scale, LogitStore store,
                                                                 VoteFuse fuse, SampleCfg samp) {
  constexpr bool DUMP = MODE == 1;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  constexpr int SLAB = slab_bytes(MT);
  constexpr int LOADS_PER_SLAB = 8 + MT;  // DMA instructions one producer lane issues per slab

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mblk = blockIdx.y;
  const int nchunks = d / BK;

  const int row_begin = v_lo + (int)blockIdx.x * rows_per_wg;
  const int row_end = (row_begin + rows_per_wg < v_hi) ? row_begin + rows_per_wg : v_hi;
  const int my_tiles = (row_begin < row_end) ? (row_end - row_begin + BN - 1) / BN : 0;
  const int total = my_tiles * nchunks;  // slabs this workgroup walks; identical for all its wavefronts
  const int rot = (int)((blockIdx.x * 5u) % (unsigned)nchunks);

  if (wave >= 4) {
    // ------------------------------------------------------------------ producer
    __builtin_amdgcn_s_setprio(3);  // a ready copy instruction goes ahead of the other wavefront's MFMAs
    const int p = wave - 4;
    const int ld_row = lane >> 3;   // row (8*rb + lane/8) of this producer's 64, 16-byte piece lane%8
    const int ld_slot = lane & 7;
    // Addresses are "uniform 64-bit base + 32-bit lane offset": the lane offsets are fixed for the
    // whole kernel, the bases are scalar arithmetic, so a copy costs the producer no vector ALU work.
    uint32_t woff[8];
#pragma unroll
    for (int rb = 0; rb < 8; ++rb) {
      const int row = 8 * rb + ld_row;
      const int piece = ld_slot ^ ((row >> 1) & 7);
      woff[rb] = (uint32_t)row * (uint32_t)(2 * d) + (uint32_t)piece * 16u;
    }
    const uint32_t aoff = (uint32_t)lane * 16u;
    const char* Wb = reinterpret_cast<const char*>(W);
    const char* Ab = reinterpret_cast<const char*>(A_sw);
    auto issue = [&](int q) {
      const int n = q / nchunks;
      int c = q - n * nchunks + rot;
      c = c >= nchunks ? c - nchunks : c;
      const int v0 = row_begin + n * BN + 64 * p;  // first vocabulary row of this producer's 64
      unsigned char* stage = lds + (q % NS) * SLAB;
      const char* wsrc = Wb + ((int64_t)v0 * d + (int64_t)c * BK) * 2;
      if (v0 + 64 <= row_end) {
#pragma unroll
        for (int rb = 0; rb < 8; ++rb) dma_copy16_stream(wsrc, woff[rb], stage + p * 8192 + rb * 1024);
      } else {  // partial tile: rows past the end re-read an own row, masked out later
#pragma unroll
        for (int rb = 0; rb < 8; ++rb) {
          const int row = 8 * rb + ld_row;
          const int vrow = (v0 + row < row_end) ? v0 + row : row_end - 1;
          const int piece = ld_slot ^ ((row >> 1) & 7);
          const __bf16* src = W + (int64_t)vrow * d + c * BK + piece * 8;
          __builtin_amdgcn_global_load_lds(DM_GLOBAL_PTR(src), DM_LDS_PTR(stage + p * 8192 + rb * 1024), 16, 0, 0);
        }
      }
      const char* asrc = Ab + ((int64_t)(c * 2) * mt_total + mblk * (2 * MT)) * 1024;
#pragma unroll
      for (int x = 0; x < MT; ++x) {
        const int f = p + 4 * x;  // fragment index inside the slab: f = s * 2 MT + mt (k-step of 32, tile of 16 rows)
        const int s = f / (2 * MT);
        const int mt = f - s * (2 * MT);
        dma_copy16(asrc + ((int64_t)s * mt_total + mt) * 1024, aoff, stage + W_SLAB_BYTES + f * 1024);
      }
    };
    if (total > 0) issue(0);
    if (total > 1) issue(1);
    for (int q = 0; q < total; ++q) {
      // own DMA of slab q has landed (the slab issued after it may still be in flight)
      if (q + 1 < total) {
        DM_WAIT_VMCNT(LOADS_PER_SLAB);
      } else {
        DM_WAIT_VMCNT(0);
      }
      DM_BARRIER();                     // slab q complete for everyone; slab q-1 consumed by everyone
      if (q + 2 < total) issue(q + 2);  // into the buffer of slab q-1
      const int n = q / nchunks;
      if (MODE != 1 && q - n * nchunks == nchunks - 1) DM_BARRIER();  // pairs with the consumers' tile-end barrier
    }
  } else {
    // -------------------------------------------------------------------- consumer
    const int i16 = lane & 15;  // row inside a 16-row MFMA tile (vocabulary row of W, masked row of the B operand)
    const int kq = lane >> 4;   // which 8 of the 32 k of an MFMA step; in the accumulators: which 4 of a tile's 16 vocabulary rows
    const int swz = (i16 >> 1) & 7;
    constexpr int NA = 2 * MT;  // masked-row tiles of 16

    // acc[a][w][r]: masked row 16 a + i16 of the row block, vocabulary row 16 w + 4 kq + r of the wavefront's 64
    f32x4 acc[NA][4];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[a][w][r] = 0.f;

    // MODE 2: where this lane's masked rows live in the logit store (row m = path m % K of position
    // m / K), as a 32-bit byte offset from the first position of the workgroup's row block, so that a
    // store needs one address register (uniform base + lane offset).  The lane's 4 * kq vocabulary-row
    // offset is folded in.
    uint32_t lt_off[NA];
    bool lt_ok[NA];
    char* lt_base = nullptr;
    if (MODE == 2) {
      const int64_t pos0 = ((int64_t)mblk * MT * 32) / store.K;
      lt_base = reinterpret_cast<char*>(store.lt + pos0 * store.V * (int64_t)store.K4);
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        const int64_t m = (int64_t)mblk * (MT * 32) + a * 16 + i16;
        const int64_t pos = m / store.K;
        lt_ok[a] = m < M;
        lt_off[a] = (uint32_t)(((pos - pos0) * store.V * store.K4 + (m - pos * store.K) + 4 * kq * store.K4) * 4);
      }
    }

    constexpr int NBL = noise_blocks_in_loop(MT);  // SAMPLE: noise blocks 0 .. NBL-1 of a tile are added in the k loop
    static_assert(NBL <= 16, "the switch below has 16 cases");
    static_assert(NBL == 0 || NBL == 4 * NA, "either all blocks of a tile in the k loop or none");
    RowRng rng[NBL > 0 ? NA : 1];                  // the row streams, kept over the k loop only when it draws the noise
    int noise_b = 0;                               // next of them
    const float inv_zscale = SAMPLE ? 1.0f / samp.zscale : 0.f;
    if (SAMPLE && NBL > 0) {
#pragma unroll
      for (int a = 0; a < NA; ++a) rng[a] = make_row_rng(samp, (int64_t)mblk * (MT * 32) + a * 16 + i16, M);
    }

    for (int q = 0; q < total; ++q) {
      DM_BARRIER();
      const unsigned char* stage = lds + (q % NS) * SLAB;
      const unsigned char* wbase = stage + wave * 8192 + i16 * 128;
      const unsigned char* abase = stage + W_SLAB_BYTES + lane * 16;
      // Fragments are requested ahead of their use by hand: that of masked-row tile a + 1 before the four MFMAs
      // of tile a, and the W fragments of the slab's second k-step one by one behind the last MFMA that reads the
      // register they go to (left to itself the compiler requests each fragment right before its use and waits
      // for it on the spot).
      bf16x8 wf[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) wf[w] = *reinterpret_cast<const bf16x8*>(wbase + w * 2048 + 16 * (kq ^ swz));
      bf16x8 af = *reinterpret_cast<const bf16x8*>(abase);
#pragma unroll
      for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          const bool more = a + 1 < NA || s == 0;  // another masked-row fragment in this slab
          bf16x8 af_next = af;
          if (more) af_next = *reinterpret_cast<const bf16x8*>(abase + (a + 1 < NA ? s * NA + a + 1 : (s + 1) * NA) * 1024);
          __builtin_amdgcn_sched_barrier(0);  // keeps the request above ahead of the MFMAs below
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            acc[a][w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[w], af, acc[a][w], 0, 0, 0);
            if (a == NA - 1 && s == 0) {
              __builtin_amdgcn_sched_barrier(0);
              wf[w] = *reinterpret_cast<const bf16x8*>(wbase + w * 2048 + 16 * ((4 + kq) ^ swz));
              __builtin_amdgcn_sched_barrier(0);
            }
          }
          af = af_next;
        }
      }
      asm volatile("" ::: "memory");

      const int n = q / nchunks;
      if constexpr (SAMPLE && NBL > 0) {
        // arg max over zscale * l + g = arg max over l + g / zscale, and l is a sum: noise can be added to the
        // accumulators during the k loop, block by block (4 vocabulary rows of one masked-row tile = one
        // Philox call), evenly over the slabs of the tile, while the wavefront would wait for data anyway
        const int sl = q - n * nchunks;
        const int due = ((sl + 1) * NBL) / nchunks;  // blocks added by the end of this slab; all NBL at the last
        const int vb = row_begin + n * BN + 64 * wave + 4 * kq;
        for (; noise_b < due; ++noise_b) {
          const int a = noise_b >> 2;
          RowRng r = rng[0];
#pragma unroll
          for (int k = 1; k < NA; ++k)
            if (a == k) r = rng[k];
          float g[4] = {0.f, 0.f, 0.f, 0.f};
          if (r.on) {
            gumbel4(r, (uint32_t)(vb + 16 * (noise_b & 3)), step_now(samp.step, samp.step_dev), g);
#pragma unroll
            for (int e = 0; e < 4; ++e) g[e] *= inv_zscale;
          }
          switch (noise_b) {
#define DM_NB(B) case B: add_noise_block<MT, B>(acc, g); break;
            DM_NB(0) DM_NB(1) DM_NB(2) DM_NB(3) DM_NB(4) DM_NB(5) DM_NB(6) DM_NB(7)
            DM_NB(8) DM_NB(9) DM_NB(10) DM_NB(11) DM_NB(12) DM_NB(13) DM_NB(14) DM_NB(15)
#undef DM_NB
            default: break;
          }
        }
        if (sl == nchunks - 1) noise_b = 0;
      }
      if (q - n * nchunks != nchunks - 1) continue;

      // ---- tile finished: accumulator (a, w, r) of lane holds row v, column m ----
      //   v = v0 + 64*wave + 16*w + 4*kq + r,  m = 32*MT*mblk + 16*a + lane%16
      const int v0 = row_begin + n * BN;
      if (DUMP) {
        const int nv = dv1 - dv0;
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          const int64_t m = (int64_t)mblk * (MT * 32) + a * 16 + i16;
          const float sc = (store.clean_last && m % store.K == store.K - 1) ? 1.0f : scale;  // clean path: no 1/(1-p)
#pragma unroll
          for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int v = v0 + 64 * wave + 16 * w + 4 * kq + r;
              if (m < M && v >= dv0 && v < dv1 && v < row_end) logits[m * nv + (v - dv0)] = sc * acc[a][w][r];
              acc[a][w][r] = 0.f;
            }
        }
        continue;
      }

      if (MODE == 2) {
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int vu = v0 + 64 * wave + 16 * w + r;  // + 4 * kq per lane
            char* dst = lt_base + (int64_t)vu * store.K4 * 4;
            const bool v_ok = vu + 4 * kq < row_end;
#pragma unroll
            for (int a = 0; a < NA; ++a)
              if (lt_ok[a] && v_ok) *reinterpret_cast<float*>(dst + lt_off[a]) = scale * acc[a][w][r];
          }
      }

      unsigned long long* red = reinterpret_cast<unsigned long long*>(lds + NS * SLAB);  // [4][MT*32]
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        float best = -INFINITY;
        uint32_t bv = 0xFFFFFFFFu;
        bool noisy = false;
        RowRng ra{0u, 0u, 0u, 0u, false};
        if constexpr (SAMPLE) {
          if constexpr (NBL > 0) {
            noisy = rng[a].on;  // all blocks got their noise in the k loop (as g / zscale, so the expression below holds)
          } else {
            ra = make_row_rng(samp, (int64_t)mblk * (MT * 32) + a * 16 + i16, M);
            noisy = ra.on;
          }
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float g[4] = {0.f, 0.f, 0.f, 0.f};
          if (SAMPLE && NBL == 0 && noisy)
            gumbel4(ra, (uint32_t)(v0 + 64 * wave + 16 * w + 4 * kq), step_now(samp.step, samp.step_dev), g);
#pragma unroll
          for (int e = 0; e < 4; ++e) {  // ascending v for this lane: strict > keeps the smallest index
            const int v = v0 + 64 * wave + 16 * w + 4 * kq + e;
            const float val = noisy ? fmaf(acc[a][w][e], samp.zscale, g[e]) : acc[a][w][e] + 0.0f;
            if (v < row_end && (bv == 0xFFFFFFFFu || val > best)) {
              best = val;
              bv = (uint32_t)v;
            }
            acc[a][w][e] = 0.f;
          }
        }
        unsigned long long key = (bv == 0xFFFFFFFFu) ? 0ull : pack_key(best, bv);
        unsigned long long other = __shfl_xor(key, 16, 64);
        key = other > key ? other : key;
        other = __shfl_xor(key, 32, 64);
        key = other > key ? other : key;
        if (kq == 0) red[wave * (MT * 32) + a * 16 + i16] = key;
      }
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): LDS writes above are done
      DM_BARRIER();
      if (tid < MT * 32) {
        unsigned long long key = red[tid];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
          const unsigned long long other = red[w * (MT * 32) + tid];
          key = other > key ? other : key;
        }
        const int64_t m = (int64_t)mblk * (MT * 32) + tid;
        if (m < M && key != 0ull) atomicMax(&keys[m], key);
      }
    }
  }  // consumer

  // -------------------------------------------------------------------- fused acceptance step
  // Every thread waits until its own argmax merges are done, the workgroup meets, one thread bumps
  // the counter; the workgroup that sees all others done reads the final keys and runs the vote /
  // rule / prefix step.  (The counter starts at 0: the mask kernel of every call resets it, so a
  // launch that did not finish cannot leave later calls without an elected workgroup.)  The merges, the counter and the
  // reads of the keys are all device-scope atomic operations, which are carried out at the memory
  // side, past the per-XCD L2s; that is what makes the keys of other XCDs visible here.  A device
  // scope fence is deliberately not used: it writes back and invalidates the XCD's whole L2, which the
  // workgroups still streaming W depend on for the masked rows (measured: 160 us -> 218 us).
  // The LDS slabs are free by now.
  if (MODE == 0 && fuse.counter != nullptr) {
    asm volatile("" ::: "memory");
    DM_WAIT_VMCNT(0);
    __syncthreads();
    int* flag = reinterpret_cast<int*>(lds);
    if (tid == 0) {
      const unsigned int done = atomicAdd(fuse.counter, 1u);
      *flag = (done == gridDim.x * gridDim.y - 1u) ? 1 : 0;
    }
    __syncthreads();
    const bool last = *flag != 0;
    __syncthreads();  // everyone has read the flag before the scratch below overwrites it
    if (last) {
      for (int b = 0; b < fuse.B; ++b) {
        vote_accept_body<true>(b, tid, THREADS, reinterpret_cast<int32_t*>(lds), keys, fuse.draft_ids, fuse.parent,
                               fuse.T, fuse.K, fuse.Kv, fuse.rule, fuse.out, nullptr, JsGeom{});
        __syncthreads();
      }
    }
  }
}

template <int MT>
hipError_t run(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g, int V, int num_cu,
               float* logits, int v0, int v1, float scale, const LogitStore& store, const VoteFuse& fuse,
               const SampleCfg& samp, const LaunchSite& at) {
  const bool dump = logits != nullptr;
  const int v_lo = dump ? v0 : 0;
  const int v_hi = dump ? v1 : V;
  if (v_hi <= v_lo) return hipSuccess;
  const int mt_total = (int)(g.M_pad >> 5);
  const int mblocks = mt_total / MT;
  // one workgroup per CU (LDS-limited); tiles at least half full
  int cap = num_cu / (mblocks < num_cu ? mblocks : num_cu);
  if (cap < 1) cap = 1;
  int gx = (v_hi - v_lo + BN / 2 - 1) / (BN / 2);
  if (gx > cap) gx = cap;
  int rows_per_wg = (v_hi - v_lo + gx - 1) / gx;
  rows_per_wg = (rows_per_wg + 3) & ~3;  // ranges start at multiples of 4: one Philox call serves 4 rows when sampling
  const dim3 grid((unsigned)gx, (unsigned)mblocks), block(THREADS);
#define DM_LAUNCH(MODE, SAMPLE)                                                                                 \
  launch_at(lmhead_mfma_kernel<MT, MODE, SAMPLE>, grid, block, (size_t)lds_bytes(MT), at,                        \
            static_cast<const __bf16*>(W), static_cast<const __bf16*>(a_ws), keys, g.d, g.M, 2 * mt_total, v_lo, \
            v_hi, rows_per_wg, logits, v0, v1, scale, store, fuse, samp)
  if (dump)
    DM_LAUNCH(1, false);
  else if (store.lt != nullptr)
    DM_LAUNCH(2, false);
  else if (samp.seeds != nullptr)
    DM_LAUNCH(0, true);
  else
    DM_LAUNCH(0, false);
#undef DM_LAUNCH
  return hipGetLastError();
}

template <int MT, int MODE, bool SAMPLE>
hipError_t raise_lds() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_mfma_kernel<MT, MODE, SAMPLE>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(MT));
}

}  // namespace

hipError_t prepare_lmhead_mfma() {
  hipError_t e;
#define DM_RAISE(MT)                                                                                  \
  if ((e = raise_lds<MT, 0, false>()) != hipSuccess || (e = raise_lds<MT, 0, true>()) != hipSuccess || \
      (e = raise_lds<MT, 1, false>()) != hipSuccess || (e = raise_lds<MT, 2, false>()) != hipSuccess)  \
    return e
  DM_RAISE(1);
  DM_RAISE(2);
  DM_RAISE(3);
  DM_RAISE(4);
#undef DM_RAISE
  return hipSuccess;
}

hipError_t launch_lmhead_mfma(const void* W, const void* a_ws, unsigned long long* keys, const RowGeom& g, int V,
                              int num_cu, float* logits, int v0, int v1, float scale, const LogitStore& store,
                              const SampleCfg& samp, const VoteFuse* fuse_in, bool* fused, const LaunchSite& at) {
  // the acceptance step rides along when this is the plain verify path and its scratch fits the slabs
  VoteFuse fuse{};
  const bool can_fuse = fuse_in != nullptr && fuse_in->counter != nullptr && logits == nullptr &&
                        store.lt == nullptr && fuse_in->rule < 2 && fuse_in->B <= 8 &&  // one workgroup does all sequences
                       
                        vote_lds_ints(fuse_in->T, fuse_in->K, fuse_in->rule) * sizeof(int32_t) <= (size_t)lds_bytes(1);
  if (can_fuse) fuse = *fuse_in;
  if (fused) *fused = can_fuse;
  const int mt_total = (int)(g.M_pad >> 5);
  if (mt_total >= 4) {
    if (mt_total % 4 != 0) return hipErrorInvalidValue;
    return run<4>(W, a_ws, keys, g, V, num_cu, logits, v0, v1, scale, store, fuse, samp, at);
  }
  switch (mt_total) {
    case 1: return run<1>(W, a_ws, keys, g, V, num_cu, logits, v0, v1, scale, store, fuse, samp, at);
    case 2: return run<2>(W, a_ws, keys, g, V, num_cu, logits, v0, v1, scale, store, fuse, samp, at);
    case 3: return run<3>(W, a_ws, keys, g, V, num_cu, logits, v0, v1, scale, store, fuse, samp, at);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace dm
