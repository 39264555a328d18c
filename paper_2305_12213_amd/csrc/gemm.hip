// Ragged / grouped GEMMs  C'[i][j] = sum_k A[i][k] * B[j][k]  (both operands k-contiguous).
//   bf16: MFMA 32x32x16 with fp32 accumulators, tiles staged through LDS in 16-byte
//         granules with an XOR swizzle, software-pipelined global loads.
//   fp32: plain FMA tiles (parity path for the fp32 workloads).
// Batch sizes are run-time data: rows, columns and reduction depth are predicated, nothing
// is compiled per size.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "dynb_internal.h"
#include "lds_async.h"

namespace dynb {
namespace {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct GroupView {
  int64_t col0;  // first reduction column of this group
  int depth;     // reduction length
  float* Cf;     // fp32 output base for this group
};

__device__ inline GroupView group_view(const GemmArgs& p, const Segs& s, int g) {
  GroupView v;
  if (p.mode == MODE_WGRAD) {
    v.col0 = s.poff[g];
    v.depth = s.poff[g + 1] - s.poff[g];
    v.Cf = p.Cf + (int64_t)g * p.group_stride;
  } else {
    v.col0 = 0;
    v.depth = p.K;
    v.Cf = p.Cf;
  }
  return v;
}

// Scalar epilogue shared by both kernels (T = storage type of C and mask).
template <typename T, int MODE>
__device__ inline void store_one(const GemmArgs& p, const GroupView& gv, int i, int j, float v) {
  if (MODE == MODE_FWD) {
    if (p.bias) v += p.bias[j];
    if (p.relu) v = fmaxf(v, 0.f);
    if (p.C) ((T*)p.C)[(int64_t)i * p.ldc + j] = (T)v;
    if (p.Cf) p.Cf[(int64_t)i * p.ldcf + j] = v;
  } else if (MODE == MODE_DGRAD) {
    if (p.mask && !((float)((const T*)p.mask)[(int64_t)i * p.ldmask + j] > 0.f)) v = 0.f;
    ((T*)p.C)[(int64_t)i * p.ldc + j] = (T)v;
  } else {
    gv.Cf[(int64_t)j * p.ldcf + i] = v;
  }
}

// ------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------
constexpr int BK = 32;          // reduction elements per stage (two MFMA k-steps)
constexpr int GPR = BK / 8;     // 16-byte granules per tile row

// Workgroup -> tile.  Consecutive workgroup ids are spread round-robin over the 8 XCDs, each
// with its own L2: give every XCD a contiguous chunk of the tile sequence, and walk the tiles
// in bands of 8 tile-rows so that a chunk covers a compact rectangle (few distinct operand
// panels per L2).
__device__ inline void tile_of_block(int pid, int tiles_i, int tiles_j, int& ti, int& tj) {
  const int total = tiles_i * tiles_j;
  const int per = total / 8, extra = total % 8, xcd = pid % 8, local = pid / 8;
  int t = pid;
  if (total >= 16) t = xcd * per + (xcd < extra ? xcd : extra) + local;
  const int band = 8;
  const int bsz = band * tiles_j;
  const int b0 = t / bsz, r = t % bsz;
  const int rows = (tiles_i - b0 * band) < band ? (tiles_i - b0 * band) : band;
  ti = b0 * band + r % rows;
  tj = r / rows;
}

// Staged operand tiles (forward / input gradient): rows of 64 bytes = four 16-byte granules;
// logical granule g of row r sits at physical granule g ^ swizzle_of_row(r).  The LDS has 64
// banks of 4 bytes, so a 16-byte fragment read serves 16 lanes per clock and four consecutive
// rows fill the 256 bytes of one pass over the banks: rows r, r+4, r+8, r+12 need four different
// swizzles (bits 2 and 3 of the row, swapped so that rows r and r+4 differ in the upper bit --
// conflict-free also if the hardware pairs lanes l and l+32, which read granules g and g^1).
__device__ inline int swizzle_of_row(int r) { return (((r >> 2) & 1) << 1) | ((r >> 3) & 1); }

// Position in the stream of 32-deep stages that one workgroup walks: stage `kt` of group `g`.
// FWD/DGRAD have one group; WGRAD has one group per worker, and a workgroup runs through its
// workers back to back so that the load pipeline never drains between them.
struct StageCursor {
  int g, kt;
  int nst, col0, depth;   // of group g: stages, first reduction column, reduction length --
                          // cached here so that the hot loop does no scalar memory loads (their
                          // wait counter is shared with the LDS fragment fetches)
};

// Wait until at most `stages` stages' worth of this wave's LDS-direct copies are pending
// (copies complete in issue order; PER = copies per wave and stage).
template <int PER>
__device__ inline void wait_copies(int stages) {
  static_assert(7 * PER <= 63, "vmcnt range");
  switch (stages) {
    case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER) : "memory"); break;
    case 2: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * PER) : "memory"); break;
    case 3: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * PER) : "memory"); break;
    case 4: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 * PER) : "memory"); break;
    case 5: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(5 * PER) : "memory"); break;
    case 6: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(6 * PER) : "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(7 * PER) : "memory"); break;
  }
}

// LDS patch area of the weight-gradient epilogue; other modes declare nothing (the 256 x 256
// forward kernel uses all 160 KB for its stage ring).
template <int N>
struct PatchArea {
  static __device__ float* get() {
    __shared__ float area[N];
    return area;
  }
};
template <>
struct PatchArea<0> {
  static __device__ float* get() { return nullptr; }
};

// S = number of LDS stage buffers (ring).
// AGG (weight gradient only): the workgroup also accumulates sum_g lam[g] * tile_g in registers
// and writes it to p.agg; it then owns all workers of its tile.
// Weight gradient (RM below): the operands are the row-major tensors themselves, A = dy
// [rows][lda] and B = the layer input [rows][ldb], the reduction runs over their ROWS (worker g
// owns rows [off[g], off[g+1])), and a stage holds 32 rows x BM (BN) features as they lie in
// memory; MFMA operands are fetched with the LDS transpose read (see conv_wgrad.hip for its
// lane layout).  No transposed copies of the activations are needed.
template <int BM, int BN, int WM, int WN, int MODE, bool GATHER, int S, bool AGG = false>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_kernel(GemmArgs p, Segs segs) {
  constexpr bool RM = MODE == MODE_WGRAD;
  constexpr bool WEAVE = !GATHER;   // copies placed between the MFMAs (see the stage pipeline)
  static_assert(!AGG || MODE == MODE_WGRAD, "aggregation belongs to the weight gradient");
  static_assert(!RM || (!GATHER && (BM == 256 || BM == 128) && (BN == 256 || BN == 128)),
                "weight gradient: plain operands, 128 or 256 features per tile side");
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int LA = BM / 16 / NW, LB = BN / 16 / NW;   // 16-row blocks per wave and stage
  constexpr int SPITCH = 36;                            // floats per row of a staged 32x32 tile
  static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0 && GPR == 4 && S >= 2 && S <= 8,
                "tile/waves mismatch");

  __shared__ uint4 sA[S][BM * GPR];
  __shared__ uint4 sB[S][BN * GPR];
  // (128 x 128 aggregating weight gradient: the waves of a tile share one staging area of the
  // whole tile, see store_rows below; otherwise a private 32 x 32 patch per wave)
  constexpr bool ROWS = AGG && BM == 128 && BN == 128 && TM == 1;
  constexpr int RPITCH = BM + 4;                        // floats per row of the shared staging area
  float* const sStage =
      PatchArea<MODE != MODE_WGRAD ? 0 : ROWS ? BN * RPITCH : NW * 32 * SPITCH>::get();

  // groups of this workgroup: [g_lo, g_hi).  A group is a worker, or, when the reduction is
  // split, one chunk of a worker's rows (group id = worker * split + chunk).
  const int split = MODE == MODE_WGRAD && p.split > 1 ? p.split : 1;
  const int n_groups = MODE == MODE_WGRAD ? segs.K * split : 1;
  const int g_lo = MODE == MODE_WGRAD ? blockIdx.y * p.groups_per_block : 0;
  const int g_hi = MODE == MODE_WGRAD
                       ? (g_lo + p.groups_per_block < n_groups ? g_lo + p.groups_per_block : n_groups)
                       : 1;
  int ti, tj;
  tile_of_block(blockIdx.x, (p.M + BM - 1) / BM, (p.N + BN - 1) / BN, ti, tj);
  const int i0 = ti * BM, j0 = tj * BN;
  // (the wave index as a scalar: everything derived from it -- LDS block addresses, which wave
  // sums the bias gradient -- then stays in scalar registers and uniform branches; a wave issues
  // at most one instruction every four clocks, so with two waves per SIMD every instruction
  // saved in the stage loop is time the MFMA pipe does not wait)
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wn = wave / WM;

  auto col0_of = [&](int g) {   // first reduction row of a group (weight gradient)
    if (MODE != MODE_WGRAD) return 0;
    return split > 1 ? segs.off[g / split] + (g % split) * p.chunk : segs.off[g];
  };
  auto depth_of = [&](int g) {
    if (MODE != MODE_WGRAD) return p.K;
    if (split == 1) return segs.off[g + 1] - segs.off[g];
    const int w = g / split, left = segs.off[w + 1] - segs.off[w] - (g % split) * p.chunk;
    return left < 0 ? 0 : (left < p.chunk ? left : p.chunk);
  };
  auto tile_base = [&](int g) -> float* {   // where a group's tile goes
    if (split > 1) return p.partial + (int64_t)g * p.partial_stride;
    return p.Cf + (int64_t)g * p.group_stride;
  };
  // Workgroups walk their groups in different rotations.  In step, every compute unit would
  // finish a worker at the same moment and all 256 tiles (64 MB) would hit the memory system
  // together while the MFMAs wait; rotated, the tile stores of some units overlap the MFMAs of
  // the others.  Position c.g in the walk is group gid(c.g).
  const int rot = (g_hi - g_lo) > 1 ? (int)((blockIdx.x * 7u) % (unsigned)(g_hi - g_lo)) : 0;
  auto gid = [&](int pos) {
    const int r = pos - g_lo + rot, span = g_hi - g_lo;
    return g_lo + (r >= span ? r - span : r);
  };
  auto enter = [&](StageCursor& c) {    // load the cached description of the group at c.g
    c.kt = 0;
    c.depth = c.g < g_hi ? depth_of(gid(c.g)) : 0;
    c.col0 = c.g < g_hi ? col0_of(gid(c.g)) : 0;
    c.nst = (c.depth + BK - 1) / BK;
  };
  auto settle = [&](StageCursor& c) {   // first stage at or after c; skips groups without rows
    while (c.g < g_hi && c.kt >= c.nst) {
      ++c.g;
      enter(c);
    }
  };

  // global -> LDS, asynchronously and without registers: one instruction moves 16 rows x 64
  // bytes; lane l lands at LDS slot l of the block, i.e. row l/4, physical granule l%4, which
  // holds logical granule (l%4) ^ swizzle_of_row(row) (conflict-free 16-byte fragment reads).  Rows
  // past the matrix edge are clamped (their products are never stored).  (Forward and input
  // gradient; the weight gradient's row-major stages are laid out further down.)
  const int lrow = lane >> 2, lgran = (lane & 3) ^ swizzle_of_row(lrow);
  const char* Ab = (const char*)p.A;
  const char* Bb = (const char*)p.B;
  uint32_t offA[LA], offB[LB];
  int gy[GATHER ? LA : 1], gx[GATHER ? LA : 1];   // gather: the row's pixel coordinates
  // gather, cheap addressing: byte offset of (the row's own source pixel, this lane's granule)
  // and one validity bit per tap; a stage then adds one wave-uniform offset per tap
  uint32_t goff[GATHER ? LA : 1], gok[GATHER ? LA : 1];
  const bool gfast = GATHER && p.gather_log2cp >= 0;
#pragma unroll
  for (int u = 0; u < LA; ++u) {
    int i = i0 + (wave + NW * u) * 16 + lrow;
    i = i < p.M ? i : p.M - 1;
    if (GATHER) {
      const int hw = p.row_h * p.row_w;
      const int n = i / hw, rem = i - n * hw;
      gy[u] = rem / p.row_w;
      gx[u] = rem - gy[u] * p.row_w;
      offA[u] = (uint32_t)(n * p.src_h * p.src_w);   // first source pixel of the sample
      const int fwd = p.conv == 1;
      const int py = fwd ? gy[u] * p.stride : gy[u], px = fwd ? gx[u] * p.stride : gx[u];
      goff[u] = (uint32_t)(((int64_t)(offA[u] + py * p.src_w + px) * p.lda + lgran * 8) * 2);
      gok[u] = 0;
      for (int tap = 0; tap < 9; ++tap) {           // (forward: +tap offset, input gradient: -)
        const int dy_ = tap / 3 - 1, dx_ = tap % 3 - 1;
        const int sy = fwd ? py + dy_ : py - dy_, sx = fwd ? px + dx_ : px - dx_;
        if (sy >= 0 && sy < p.src_h && sx >= 0 && sx < p.src_w) gok[u] |= 1u << tap;
      }
    } else {
      offA[u] = (uint32_t)(((int64_t)i * p.lda + lgran * 8) * 2);
    }
  }
#pragma unroll
  for (int u = 0; u < LB; ++u) {
    int j = j0 + (wave + NW * u) * 16 + lrow;
    j = j < p.N ? j : p.N - 1;
    offB[u] = (uint32_t)(((int64_t)j * p.ldb + lgran * 8) * 2);
  }
  const uint32_t ldsA = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)&sA[0][0];
  const uint32_t ldsB = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)&sB[0][0];
  // RM: a copy moves 512/BM (512/BN) whole reduction rows of BM (BN) features; this lane's
  // row within the stage and its byte offset from the stage's first row (0x80000000: past the
  // row pitch -- out of the buffer's range whatever the stage, zeros).  Granule g of reduction row k sits at slot g ^ ((k & 3) << 2): the
  // transpose reads of 4 neighbouring rows and of the two 16-feature halves of a 32-feature
  // block then fall into 8 different 32-byte bank ranges.
  int rkA[RM ? LA : 1], rkB[RM ? LB : 1];
  uint32_t roA[RM ? LA : 1], roB[RM ? LB : 1];
  if constexpr (RM) {
    constexpr int GA = BM / 8, GB = BN / 8;      // granules per reduction row
#pragma unroll
    for (int u = 0; u < LA; ++u) {
      const int k = (wave + NW * u) * (64 / GA) + lane / GA;
      const int f = i0 + (((lane % GA) ^ ((k & 3) << 2)) * 8);
      rkA[u] = k;
      roA[u] = f < p.lda ? (uint32_t)(((int64_t)k * p.lda + f) * 2) : 0x80000000u;
    }
#pragma unroll
    for (int u = 0; u < LB; ++u) {
      const int k = (wave + NW * u) * (64 / GB) + lane / GB;
      const int f = j0 + (((lane % GB) ^ ((k & 3) << 2)) * 8);
      rkB[u] = k;
      roB[u] = f < p.ldb ? (uint32_t)(((int64_t)k * p.ldb + f) * 2) : 0x80000000u;
    }
  }
  // Row pitches in bytes (the launch checks that an operand stays below 4 GiB).  Made opaque to
  // the compiler: it otherwise prefers to re-read lda / ldb from the kernel arguments inside the
  // hot loop when scalar registers run short, and the wait for such a scalar load also waits
  // for every outstanding LDS fragment fetch (they share a counter) -- twice per stage.
  uint32_t pitchA = (uint32_t)(p.lda * 2), pitchB = (uint32_t)(p.ldb * 2);
  asm volatile("" : "+s"(pitchA), "+s"(pitchB));
  // Buffer resources of the two operands (plain and row-major operands; the gathered operand
  // keeps 64-bit addresses).  Plain operands: the whole matrix.  Row-major: the size is set per
  // copy to the end of the worker's rows.
  i32x4 rsA = {0, 0, 0, 0}, rsB = {0, 0, 0, 0};
  if constexpr (!GATHER) {
    rsA = buffer_resource(p.A, RM ? 0u : (uint32_t)((int64_t)p.M * p.lda * 2));
    rsB = buffer_resource(p.B, RM ? 0u : (uint32_t)((int64_t)p.N * p.ldb * 2));
  }
  // One copy of a stage (plain or row-major operands): idx < LA is copy idx of the A operand,
  // else copy idx - LA of the B operand.  The hot loop places these between the MFMAs.
  auto copy_one = [&](int buf, const StageCursor& c, int idx) {
    const int k0 = c.kt * BK;
    const bool isA = idx < LA;
    const int u = isA ? idx : idx - LA;
    const void* src;
    if constexpr (RM) {
      // through a buffer resource that ends with the worker's last row: lanes on rows past it
      // (the last, partly filled stage; every lane once the workgroup is past its last stage)
      // and lanes past the row pitch read zeros by the hardware's range check
      const uint32_t pitch = isA ? pitchA : pitchB;
      i32x4 rs = isA ? rsA : rsB;
      rs[2] = (int)((uint32_t)(c.col0 + c.depth) * pitch);
      const uint32_t dst = isA ? ldsA + (uint32_t)((buf * BM * GPR + (wave + NW * u) * 64) * 16)
                               : ldsB + (uint32_t)((buf * BN * GPR + (wave + NW * u) * 64) * 16);
      async_copy_1k_buffer(rs, (isA ? roA[u] : roB[u]) + (uint32_t)(c.col0 + k0) * pitch, dst);
      return;
    } else if constexpr (!GATHER) {
      // (a workgroup past its last stage keeps copying, see the stage loop: whatever such a
      // copy reads -- the rows again from their start, zeros past the matrix -- is never used)
      const uint32_t dst = isA ? ldsA + (uint32_t)((buf * BM * GPR + (wave + NW * u) * 64) * 16)
                               : ldsB + (uint32_t)((buf * BN * GPR + (wave + NW * u) * 64) * 16);
      async_copy_1k_buffer(isA ? rsA : rsB, (isA ? offA[u] : offB[u]) + (uint32_t)k0 * 2, dst);
      return;
    } else {
      src = (const void*)((isA ? Ab + offA[u] : Bb + offB[u]) + (uint32_t)k0 * 2);
    }
    const uint32_t dst = isA ? ldsA + (uint32_t)((buf * BM * GPR + (wave + NW * u) * 64) * 16)
                             : ldsB + (uint32_t)((buf * BN * GPR + (wave + NW * u) * 64) * 16);
    async_copy_1k(src, dst);
  };

  // All copies of a stage at once (the prologue; every stage of the gathered-operand kernels).
  auto issue = [&](int buf, const StageCursor& c) {
    if constexpr (!GATHER) {
#pragma unroll
      for (int idx = 0; idx < LA + LB; ++idx) copy_one(buf, c, idx);
      return;
    }
    const int k0 = c.kt * BK;
    const uint32_t kbyte = (uint32_t)k0 * 2;
    if (gfast) {
      // the whole stage lies in tap k0 >> log2(cp): one signed byte offset for every row
      const int tap = k0 >> p.gather_log2cp, kc = k0 & (p.cp - 1);
      const int th = (tap * 11) >> 5, tw = tap - 3 * th;          // tap / 3, tap % 3 (tap <= 9)
      const int dpix = (th - 1) * p.src_w + (tw - 1);
      const uint32_t dbyte = (uint32_t)(((p.conv == 1 ? dpix : -dpix) * (int)p.lda + kc) * 2);
#pragma unroll
      for (int u = 0; u < LA; ++u) {
        const void* src = (gok[u] >> tap) & 1u ? (const void*)(Ab + (uint32_t)(goff[u] + dbyte))
                                               : p.zeros;
        async_copy_1k(src, ldsA + (uint32_t)((buf * BM * GPR + (wave + NW * u) * 64) * 16));
      }
    } else {
      const int k = k0 + lgran * 8;
      const int tap = k / p.cp;
      const int ch = k - tap * p.cp;
      const int kh = tap / 3, kw = tap - kh * 3;
      const bool tap_ok = tap < 9;
#pragma unroll
      for (int u = 0; u < LA; ++u) {
        int sy, sx;
        bool ok = tap_ok;
        if (p.conv == 1) {
          sy = gy[u] * p.stride + kh - 1;
          sx = gx[u] * p.stride + kw - 1;
        } else {
          // (stride is 1 or 2: a shift instead of a division in the hot loop)
          const int ty = gy[u] + 1 - kh, tx = gx[u] + 1 - kw, sh = p.stride - 1;
          sy = ty >> sh;
          sx = tx >> sh;
          ok = ok && ty >= 0 && tx >= 0 && (sy << sh) == ty && (sx << sh) == tx;
        }
        ok = ok && sy >= 0 && sy < p.src_h && sx >= 0 && sx < p.src_w;
        const int64_t pix = (int64_t)offA[u] + sy * p.src_w + sx;
        const void* src = ok ? (const void*)(Ab + (pix * p.lda + ch) * 2) : p.zeros;
        async_copy_1k(src, ldsA + (uint32_t)((buf * BM * GPR + (wave + NW * u) * 64) * 16));
      }
    }
#pragma unroll
    for (int u = 0; u < LB; ++u) {
      const void* src = (const void*)(Bb + offB[u] + kbyte);
      async_copy_1k(src, ldsB + (uint32_t)((buf * BN * GPR + (wave + NW * u) * 64) * 16));
    }
  };

  // LDS -> MFMA fragments: lane reads row (lane & 31) of a 32-row block, granule 2*kk + lane/32
  const int frow_a = (wm * (BM / WM) + (lane & 31)) * GPR;
  const int frow_b = (wn * (BN / WN) + (lane & 31)) * GPR;
  const int fsw = swizzle_of_row(lane & 31), fhi = lane >> 5;
  bf16x8 fa[2][TM], fb[2][TN];   // two register sets, alternating per k-step
  // RM: 16 lanes fetch 4 reduction rows x 16 features with two transpose reads (lane r supplies
  // the address of features 4(r%4).. of row r/4 and receives feature r of the 4 rows)
  const int tg = lane >> 4, tr = lane & 15;
  auto tr_off = [&](int feat0, int pitch) {      // this lane's byte offset for the block at feat0
    const int f = feat0 + 16 * (tg & 1) + 4 * (tr & 3);
    return (uint32_t)((8 * (tg >> 1) + (tr >> 2)) * pitch + (((f >> 3) ^ ((tr >> 2) << 2)) * 16) + (f & 7) * 2);
  };
  uint32_t trA[RM ? TM : 1], trB[RM ? TN : 1];
  if constexpr (RM) {
#pragma unroll
    for (int a = 0; a < TM; ++a) trA[a] = tr_off(wm * (BM / WM) + a * 32, BM * 2);
#pragma unroll
    for (int b = 0; b < TN; ++b) trB[b] = tr_off(wn * (BN / WN) + b * 32, BN * 2);
  }
  auto tr_frag = [&](uint32_t addr, int pitch) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(uintptr_t)addr);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(uintptr_t)(addr + 4 * pitch));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };
  // fragment f of k-step kk: f < TM is A fragment f, else B fragment f - TM
  auto frag_one = [&](const uint4* sa, const uint4* sb, int kk, int set, int f) {
    if constexpr (RM) {
      const uint32_t la = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)sa;
      const uint32_t lb = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)sb;
      if (f < TM) fa[set][f] = tr_frag(la + trA[f] + (uint32_t)(kk * 16 * BM * 2), BM * 2);
      else fb[set][f - TM] = tr_frag(lb + trB[f - TM] + (uint32_t)(kk * 16 * BN * 2), BN * 2);
    } else {
      const int g = (kk * 2 + fhi) ^ fsw;
      if (f < TM) fa[set][f] = *(const bf16x8*)&sa[frow_a + f * 32 * GPR + g];
      else fb[set][f - TM] = *(const bf16x8*)&sb[frow_b + (f - TM) * 32 * GPR + g];
    }
  };
  auto lfrag = [&](const uint4* sa, const uint4* sb, int kk, int set) {
#pragma unroll
    for (int f = 0; f < TM + TN; ++f) frag_one(sa, sb, kk, set, f);
  };

  f32x16 agg[AGG ? TM : 1][AGG ? TN : 1];   // weighted sum over the workers (AGG)
  if constexpr (AGG) {
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) agg[a][b][v] = 0.f;
  }
  f32x16 acc[TM][TN];
  auto clear_acc = [&]() {
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  };
  clear_acc();
  // Weight gradient, optional: the bias gradient db_g[i] = sum over worker g's rows of dy[.][i]
  // rides along as one more column of the product -- the waves of one tile column multiply
  // their dy fragments with ones.  Every column of rsum holds the same sums; lanes 0 and
  // 32 (column 0) write them out.
  // The tiles of a tile row all hold these dy fragments: worker g's sums are formed by the tile
  // column g mod (tile columns), so that the extra work is spread over the workgroups instead of
  // making the first tile column the last to finish.
  const int bias_cols = (p.N + BN - 1) / BN;
  auto owns_bias = [&](int g) { return RM && p.bias_grad != nullptr && wn == 0 && g % bias_cols == tj; };
  bool sums_rows = false;           // does this wave sum the rows of the worker being computed?
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 ones_bits = {0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
  f32x16 rsum[TM];   // (unused and optimised away outside the weight gradient)
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) rsum[a][v] = 0.f;
  // writes src (or zeros) as the bias gradient at `dst` (this tile's rows), from column 0
  auto store_row_sums = [&](float* dst, const f32x16 (&src)[TM], bool zeros) {
    if ((lane & 31) != 0) return;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = i0 + wm * (BM / WM) + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
        if (i < p.M) dst[i] = zeros ? 0.f : src[a][v];
      }
  };
  // The MFMA's first operand indexes the 4-consecutive-per-lane dimension of the result.  Weight
  // gradients are stored [j][i] with i contiguous; forward / activation-gradient results are
  // stored [i][j] with j contiguous: feed the operands accordingly.
  auto mma_one = [&](int set, int i) {
    const int a = i / TN, b = i % TN;
    if (MODE == MODE_WGRAD)
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][a], fb[set][b], acc[a][b], 0, 0, 0);
    else
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][b], fa[set][a], acc[a][b], 0, 0, 0);
  };
  auto mma_sums = [&](int set) {
    if constexpr (RM) {
      if (sums_rows) {             // (uniform per wave) the bias gradient: dy against ones
#pragma unroll
        for (int a = 0; a < TM; ++a)
          rsum[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][a], ones, rsum[a], 0, 0, 0);
      }
    }
  };
  auto mma = [&](int set) {
#pragma unroll
    for (int i = 0; i < TM * TN; ++i) mma_one(set, i);
    mma_sums(set);
  };

  // Accumulator element v of lane l sits at (8*(v/4) + 4*(l/32) + v%4, l%32) of its 32x32 tile,
  // first coordinate = the first MFMA operand's row: each lane owns runs of 4 consecutive
  // elements along the output's contiguous dimension.
  const int hi4 = 4 * (lane >> 5), l31 = lane & 31;

  // Weight-gradient tile of worker g -> grads[g].  Each wave passes its 32x32 sub-tiles through
  // a private LDS patch so that one store instruction writes 8 rows x 128 contiguous bytes
  // (whole lines) instead of 32 rows x 32 bytes: these stores are the largest HBM stream of a
  // step.  LDS operations of one wave execute in order, so the patch needs no barrier.
  // The same for the 128 x 128 aggregating kernel, whose matrices are the narrow ones (an output
  // layer of 1000 columns: rows pitched 4000 bytes start on odd 32-byte boundaries, and every
  // 128-byte run of a wave then ends in two partial lines -- the launch takes 120 us at 1000
  // columns and 93 us at 1008).  All waves stage their sub-tiles in one area of the whole tile,
  // and after a barrier each wave writes 16 rows as 2 rows x 512 contiguous bytes per instruction:
  // two partial lines per tile row instead of eight.  The area is next written at the end of the
  // next worker, at least one stage barrier later, by which time every wave has read it.
  auto store_rows = [&](float* Cg, f32x16 (&src)[TM][TN]) {
    if constexpr (ROWS) {
      float* area = sStage;
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 o = {src[0][b][4 * q], src[0][b][4 * q + 1], src[0][b][4 * q + 2], src[0][b][4 * q + 3]};
          *(f32x4*)&area[(wn * (BN / WN) + 32 * b + l31) * RPITCH + wm * 32 + 8 * q + hi4] = o;
        }
      __syncthreads();
      constexpr int RW = BN / NW;                      // rows per wave
      const int r0 = wave * RW + (lane >> 5), c = (lane & 31) * 4;
      const bool col_ok = i0 + c + 3 < p.M;            // (M is a multiple of 4 here)
      f32x4 o[RW / 2];
#pragma unroll
      for (int t = 0; t < RW / 2; ++t) o[t] = *(const f32x4*)&area[(r0 + 2 * t) * RPITCH + c];
#pragma unroll
      for (int t = 0; t < RW / 2; ++t) {
        const int j = j0 + r0 + 2 * t;
        if (col_ok && j < p.N)
          __builtin_nontemporal_store(o[t], (f32x4*)(Cg + (int64_t)j * p.ldcf + i0 + c));
      }
    }
  };
  auto store_tile = [&](float* Cg, f32x16 (&src)[TM][TN]) {
    if constexpr (ROWS) {
      if ((p.ldcf & 3) == 0 && (p.M & 3) == 0 && (((uintptr_t)Cg) & 15) == 0) {   // (uniform)
        store_rows(Cg, src);
        return;
      }
      __syncthreads();   // (other waves may still be reading the shared area of a call that took the path above)
    }
    float* patch = &sStage[wave * 32 * SPITCH];
    const bool vec_ok = (p.ldcf & 3) == 0 && (((uintptr_t)Cg) & 15) == 0;
    const bool interior = vec_ok && i0 + BM <= p.M && j0 + BN <= p.N;   // no edge checks needed
    const int rr = lane >> 3, rc = (lane & 7) * 4;
    const int ib0 = i0 + wm * (BM / WM) + rc, jb0 = j0 + wn * (BN / WN) + rr;
    float* base = Cg + (int64_t)jb0 * p.ldcf + ib0;
    const int64_t row8 = (int64_t)8 * p.ldcf;
    // Sub-tile n = (b, a): b (32-row blocks) outside, a (128-byte column blocks) inside, so the
    // four sub-tiles that complete 512 contiguous bytes of each row are written back to back.
    auto put = [&](int a, int b) {        // accumulators -> patch (j = lane % 32 rows, i columns)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 o = {src[a][b][4 * q], src[a][b][4 * q + 1], src[a][b][4 * q + 2],
                         src[a][b][4 * q + 3]};
        *(f32x4*)&patch[l31 * SPITCH + 8 * q + hi4] = o;
      }
    };
    auto get = [&](f32x4 (&o)[4]) {       // patch -> 8 rows x 128 bytes per instruction
#pragma unroll
      for (int t = 0; t < 4; ++t) o[t] = *(const f32x4*)&patch[(rr + 8 * t) * SPITCH + rc];
    };
    // Software pipeline over the sub-tiles.  LDS operations of one wave execute in order, so
    // sub-tile n+1 may be written to the patch as soon as the reads of sub-tile n are *issued*;
    // its read-back is issued before the global stores of sub-tile n, which therefore wait only
    // for data requested a whole sub-tile earlier.  Without this the tile store is a chain of
    // exposed LDS latencies (one per store instruction).  `checked`: a tile on the matrix edge,
    // one predicate per store.
    auto pipelined = [&](auto checked) {
      f32x4 o[2][4];
      put(0, 0);
      __builtin_amdgcn_wave_barrier();
      get(o[0]);
#pragma unroll
      for (int n = 0; n < TM * TN; ++n) {
        const int a = n % TM, b = n / TM;
        if (n + 1 < TM * TN) {
          __builtin_amdgcn_wave_barrier();
          put((n + 1) % TM, (n + 1) / TM);
          __builtin_amdgcn_wave_barrier();
          get(o[(n + 1) & 1]);
        }
        __builtin_amdgcn_sched_barrier(0);
        float* d = base + (int64_t)(4 * b) * row8 + a * 32;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if constexpr (decltype(checked)::value) {
            if (ib0 + a * 32 + 3 < p.M && jb0 + b * 32 + 8 * t < p.N)
              __builtin_nontemporal_store(o[n & 1][t], (f32x4*)(d + t * row8));
          } else {
            __builtin_nontemporal_store(o[n & 1][t], (f32x4*)(d + t * row8));
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (interior) {
      pipelined(std::false_type{});
      return;
    }
    // (not in the 256 x 128 aggregating kernel, which measurably slows down with the extra code;
    // its edge tiles take the plain loop below)
    if constexpr (!(AGG && BM == 256)) {
      if (vec_ok && (p.M & 3) == 0) {   // a lane's four floats are inside or outside together
        pipelined(std::true_type{});
        return;
      }
    }
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        __builtin_amdgcn_wave_barrier();
        put(a, b);
        __builtin_amdgcn_wave_barrier();
        float* d = base + (int64_t)(4 * b) * row8 + a * 32;
        const int ib = ib0 + a * 32;
        f32x4 o[4];
        get(o);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if (jb0 + b * 32 + 8 * t < p.N) {
            float* dst = d + t * row8;
            if (vec_ok && ib + 3 < p.M) {
              __builtin_nontemporal_store(o[t], (f32x4*)dst);
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (ib + r < p.M) dst[r] = o[t][r];
            }
          }
        }
      }
  };

  // A worker without rows contributes a zero tile (not unrolled: it is rare and tiny).
  auto store_zero = [&](int g) {
    if constexpr (RM) {
      if (owns_bias(g)) store_row_sums(p.bias_grad + (int64_t)g * p.group_stride, rsum, true);
    }
    float* Cg = tile_base(g);
    const bool vec_ok = (p.ldcf & 3) == 0 && (((uintptr_t)Cg) & 15) == 0;
    const int rr = lane >> 3, rc = (lane & 7) * 4;
#pragma unroll 1
    for (int t = 0; t < TM * TN * 4; ++t) {
      const int a = t / (TN * 4), b = (t / 4) % TN;
      const int ib = i0 + wm * (BM / WM) + a * 32 + rc;
      const int j = j0 + wn * (BN / WN) + b * 32 + rr + 8 * (t % 4);
      if (j >= p.N) continue;
      float* dst = Cg + (int64_t)j * p.ldcf + ib;
      if (vec_ok && ib + 3 < p.M) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        __builtin_nontemporal_store(z, (f32x4*)dst);
      } else {
        for (int r = 0; r < 4; ++r)
          if (ib + r < p.M) dst[r] = 0.f;
      }
    }
  };

  // ---- the stage pipeline ----
  // A ring of S stage buffers, each one 32-deep stage (two MFMA k-steps).  Up to S stages are in
  // flight: the barrier of a stage sits right behind the last fragment fetch from its buffer,
  // so the buffer is free from there on and the stage S ahead is issued into it -- it has S-1
  // stages of MFMAs to land, which covers the ~1 us a load takes when every compute unit pulls
  // its operands through L2 at the same time.  Each wave waits only for its own copies of the
  // *next* stage before the barrier (copies complete in order).  Fragments are fetched one
  // k-step ahead into the register set the previous group of MFMAs has released.
  // sched_barrier(0) keeps the compiler's scheduler from gathering the MFMAs behind the waits.
  StageCursor ic;               // next stage to issue
  ic.g = g_lo;
  enter(ic);
  settle(ic);
  StageCursor cc = ic;          // stage being computed
  int stored = g_lo;            // workers whose tile has been written
  if (MODE == MODE_WGRAD)       // workers without rows in front of the first stage: zero gradient
    for (; stored < (cc.g < g_hi ? cc.g : g_hi); ++stored) store_zero(gid(stored));

  int ahead = -1;               // stages issued beyond the one being computed
#pragma unroll
  for (int f = 0; f < S; ++f)
    if (WEAVE || ic.g < g_hi) {
      issue(f, ic);
      ++ic.kt;
      settle(ic);
      ++ahead;
    }
  if (ahead >= 0) {
    wait_copies<LA + LB>(ahead);   // stage 0 has landed
    __syncthreads();
    lfrag(sA[0], sB[0], 0, 0);
  }
  int buf = 0;
  bool pend = false;            // second half of the previous refill still to be issued
  int pbuf = 0;                 // ... into this buffer,
  StageCursor pc = ic;          // ... of this stage
  while (cc.g < g_hi) {
    const int g = cc.g, nst = cc.nst;
    StageCursor ng;                // first stage of the next worker that has rows
    ng.g = g + 1;
    enter(ng);
    settle(ng);
    const bool later = ng.g < g_hi;
    sums_rows = owns_bias(gid(g));
    for (int kt = 0; kt < nst; ++kt) {   // the hot loop: all stages of worker g
      const int nbuf = buf + 1 == S ? 0 : buf + 1;
      if constexpr (WEAVE) {
        // A wave issues in order: copies, fragment fetches and their address arithmetic placed
        // behind a block of MFMAs would leave the matrix pipe idle for as long as they take to
        // issue, and the copies of all four waves would reach the memory pipeline in one burst.
        // They are placed *between* the MFMAs instead (32 clocks each).  First k-step: the
        // fragments of the second k-step, then the second half of the copies that refill the
        // buffer released by the previous stage.  Second k-step (behind the barrier that
        // releases this stage's buffer): the fragments of the next stage's first k-step (of a
        // buffer nobody reads when this is the last stage), then the first half of the copies
        // that refill this buffer.  While a stage is still to be issued, S - 1 stages are in
        // flight beyond this one and the wait is a constant; the last S - 1 stages count down.
        // (weight gradient: all copies of a refill in the second k-step -- the state that
        // carries a half-issued refill into the next iteration costs more scalar instructions
        // per stage than spreading three copies gains)
        constexpr int NM = TM * TN, NF = TM + TN, NC = LA + LB, NC1 = RM ? NC : NC / 2;
        constexpr int NI0 = NF + (NC - NC1), NI1 = NF + NC1;
#pragma unroll
        for (int i = 0; i < NM; ++i) {
          mma_one(0, i);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int it = i * NI0 / NM; it < (i + 1) * NI0 / NM; ++it) {
            if (it < NF) {
              frag_one(sA[buf], sB[buf], 1, 1, it);
            } else if (pend) {
              copy_one(pbuf, pc, NC1 + it - NF);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        mma_sums(0);
        __builtin_amdgcn_sched_barrier(0);
        // (past its last stage a workgroup keeps issuing copies -- weight gradient: a stage of
        // depth 0, all zeros; otherwise the rows from their start again -- so that the number in
        // flight, and with it this wait, is the same constant in every iteration and no branch
        // asks whether stages are left)
        const bool issuing = true;   // (this path: plain and row-major operands)
        if (issuing)
          asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * NC) : "memory");
        else
          wait_copies<NC>(ahead > 0 ? ahead - 1 : 0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NM; ++i) {
          mma_one(1, i);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int it = i * NI1 / NM; it < (i + 1) * NI1 / NM; ++it) {
            if (it < NF) {
              frag_one(sA[nbuf], sB[nbuf], 0, 0, it);
            } else if (issuing) {
              copy_one(buf, ic, it - NF);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        mma_sums(1);
        __builtin_amdgcn_sched_barrier(0);
        pend = issuing;
        pbuf = buf;
        pc = ic;
        if (issuing) {             // (one stage issued, one consumed: `ahead` stays S - 1)
          ++ic.kt;
          settle(ic);
        } else {
          --ahead;
        }
        buf = nbuf;
        continue;
      }
      lfrag(sA[buf], sB[buf], 1, 1);
      mma(0);
      __builtin_amdgcn_sched_barrier(0);
      wait_copies<LA + LB>(ahead > 0 ? ahead - 1 : 0);   // my copies of the next stage landed
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
      if (ic.g < g_hi) {           // refill the buffer this stage has just released
        issue(buf, ic);
        ++ic.kt;
        settle(ic);
        ++ahead;
      }
      if (ahead > 0) lfrag(sA[nbuf], sB[nbuf], 0, 0);
      mma(1);
      __builtin_amdgcn_sched_barrier(0);
      buf = nbuf;
      --ahead;
    }
    if (MODE == MODE_WGRAD) {
      if constexpr (AGG) {
        const float w = p.lam[gid(g)];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b) agg[a][b] += w * acc[a][b];
      }
      store_tile(tile_base(gid(g)), acc);
      clear_acc();
      if constexpr (RM) {
        if (sums_rows) {
          store_row_sums(p.bias_grad + (int64_t)gid(g) * p.group_stride, rsum, false);
#pragma unroll
          for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) rsum[a][v] = 0.f;
        }
      }
      for (stored = g + 1; stored < (later ? ng.g : g_hi); ++stored) store_zero(gid(stored));
    }
    cc = ng;
  }
  // (the copies issued past the end land in this workgroup's LDS: wait for them before the ring
  // is reused by the epilogue or given back)
  if constexpr (WEAVE) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (!RM) __syncthreads();   // ... all waves' copies, before any wave's patch
  }
  if constexpr (ROWS) __syncthreads();   // the last worker's tile has been read out of the shared area
  if constexpr (AGG) store_tile(p.agg, agg);

  if constexpr (MODE != MODE_WGRAD) {
    // Epilogue.  The stage ring is free now (every wave is past the last barrier and its last
    // fragment fetch), so each wave passes its 128-column strip, 32 rows at a time, through a
    // private fp32 patch in LDS: the accumulator layout (4 consecutive columns per lane, 32
    // rows per instruction) becomes 8 consecutive columns per lane, 4 rows per instruction,
    // and bias/ReLU/mask, the bf16 conversion and the global accesses run on whole 128-byte
    // lines.
    constexpr int CW = BN / WN;              // columns of a wave's strip
    constexpr int EP = CW + 4;               // patch row pitch in floats
    static_assert(CW == 128 || CW == 64, "strip width");
    static_assert((size_t)NW * 32 * EP * 4 <= sizeof(sA), "patch must fit in the A ring");
    float* patch = (float*)&sA[0][0] + wave * 32 * EP;
    constexpr int LPR = CW / 8;              // lanes per row in the read-back phase
    constexpr int RPI = 64 / LPR;            // rows per read-back instruction
    const int rrow = lane / LPR, rcol = (lane % LPR) * 8;
    const int jcol = j0 + wn * CW + rcol;    // first of the lane's 8 columns
    const bool col_ok = jcol + 7 < p.N;
    const bool bias_vec = (((uintptr_t)p.bias) & 15) == 0;   // a layer's bias may start anywhere
    float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (MODE == MODE_FWD && p.bias) {
      if (col_ok && bias_vec) {
        const float4 t0 = *(const float4*)&p.bias[jcol], t1 = *(const float4*)&p.bias[jcol + 4];
        bv[0] = t0.x; bv[1] = t0.y; bv[2] = t0.z; bv[3] = t0.w;
        bv[4] = t1.x; bv[5] = t1.y; bv[6] = t1.z; bv[7] = t1.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (jcol + e < p.N) bv[e] = p.bias[jcol + e];
      }
    }
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      // input gradient: the mask and addend rows of this 32-row block are asked for now, all of
      // them at once (rows past the matrix clamped), and travel while the accumulators pass
      // through the patch -- fetched row by row where they are used, every row costs a trip to
      // memory of its own
      bf16x8 mkv[32 / RPI], adv[32 / RPI];
      if (MODE == MODE_DGRAD && col_ok) {
#pragma unroll
        for (int t = 0; t < 32 / RPI; ++t) {
          int i = i0 + wm * (BM / WM) + a * 32 + rrow + RPI * t;
          i = i < p.M ? i : p.M - 1;
          if (p.mask) mkv[t] = *(const bf16x8*)((const bf16*)p.mask + (int64_t)i * p.ldmask + jcol);
          if (p.addend) adv[t] = *(const bf16x8*)((const bf16*)p.addend + (int64_t)i * p.ldadd + jcol);
        }
      }
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 o = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2],
                           acc[a][b][4 * q + 3]};
          *(f32x4*)&patch[l31 * EP + b * 32 + 8 * q + hi4] = o;
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int t = 0; t < 32 / RPI; ++t) {
        const int r = rrow + RPI * t;
        const int i = i0 + wm * (BM / WM) + a * 32 + r;
        const f32x4 lo = *(const f32x4*)&patch[r * EP + rcol];
        const f32x4 hi = *(const f32x4*)&patch[r * EP + rcol + 4];
        if (i >= p.M || jcol >= p.N) continue;
        float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        if (MODE == MODE_FWD) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += bv[e];
          if (p.relu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
          }
        }
        if (col_ok) {
          if (MODE == MODE_DGRAD && p.addend) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = (float)(bf16)v[e] + (float)adv[t][e];
          }
          if (MODE == MODE_DGRAD && p.mask) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (!((float)mkv[t][e] > 0.f)) v[e] = 0.f;
          }
          if (MODE == MODE_FWD && p.Cf) {
            float* dst = p.Cf + (int64_t)i * p.ldcf + jcol;
            *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
            *(float4*)(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
          }
          if (p.C) {
            const bf16x8 o = {(bf16)v[0], (bf16)v[1], (bf16)v[2], (bf16)v[3],
                              (bf16)v[4], (bf16)v[5], (bf16)v[6], (bf16)v[7]};
            *(bf16x8*)((bf16*)p.C + (int64_t)i * p.ldc + jcol) = o;
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int j = jcol + e;
            if (j >= p.N) continue;
            float w = v[e];
            if (MODE == MODE_DGRAD && p.addend)
              w = (float)(bf16)w + (float)((const bf16*)p.addend)[(int64_t)i * p.ldadd + j];
            if (MODE == MODE_DGRAD && p.mask &&
                !((float)((const bf16*)p.mask)[(int64_t)i * p.ldmask + j] > 0.f))
              w = 0.f;
            if (MODE == MODE_FWD && p.Cf) p.Cf[(int64_t)i * p.ldcf + j] = w;
            if (p.C) ((bf16*)p.C)[(int64_t)i * p.ldc + j] = (bf16)w;
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// ------------------------------------------------------------------------------------
// fp32 FMA kernel: 64x64 tile, 16-deep stages, 4x4 outputs per thread
// ------------------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs p, Segs segs) {
  constexpr int TB = 64, TK = 16;
  __shared__ float sA[TK][TB + 4];
  __shared__ float sB[TK][TB + 4];
  const GroupView gv = group_view(p, segs, blockIdx.z);
  const int i0 = blockIdx.x * TB, j0 = blockIdx.y * TB;
  const int tid = threadIdx.x;
  const int lrow = tid >> 2, lk = (tid & 3) * 4;     // loader: one float4 per operand
  const int ti = (tid >> 4) * 4, tj = (tid & 15) * 4;  // compute: 4x4 block
  const float* A = (const float*)p.A + gv.col0;
  const float* B = (const float*)p.B + gv.col0;

  float acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

  // the operands of stage k0 + TK are asked for before stage k0 is computed, so that their
  // trip to memory overlaps the arithmetic instead of preceding it
  auto fetch = [&](int k0, float4& va, float4& vb) {
    va = make_float4(0.f, 0.f, 0.f, 0.f);
    vb = va;
    const int k = k0 + lk;
    if (i0 + lrow < p.M && k < gv.depth) va = *(const float4*)(A + (int64_t)(i0 + lrow) * p.lda + k);
    if (j0 + lrow < p.N && k < gv.depth) vb = *(const float4*)(B + (int64_t)(j0 + lrow) * p.ldb + k);
  };
  float4 va, vb;
  fetch(0, va, vb);
  for (int k0 = 0; k0 < gv.depth; k0 += TK) {
    __syncthreads();
    sA[lk + 0][lrow] = va.x; sA[lk + 1][lrow] = va.y; sA[lk + 2][lrow] = va.z; sA[lk + 3][lrow] = va.w;
    sB[lk + 0][lrow] = vb.x; sB[lk + 1][lrow] = vb.y; sB[lk + 2][lrow] = vb.z; sB[lk + 3][lrow] = vb.w;
    __syncthreads();
    if (k0 + TK < gv.depth) fetch(k0 + TK, va, vb);
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      const float4 a4 = *(const float4*)&sA[kk][ti];
      const float4 b4 = *(const float4*)&sB[kk][tj];
      const float av[4] = {a4.x, a4.y, a4.z, a4.w};
      const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] += av[a] * bv[b];
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int i = i0 + ti + a, j = j0 + tj + b;
      if (i < p.M && j < p.N) store_one<float, MODE>(p, gv, i, j, acc[a][b]);
    }
}

// per-worker weight gradients (no aggregate)
template <int BM, int BN, int WM, int WN, int S>
void launch_bf16_wgrad(GemmArgs a, const Segs& s, hipStream_t st) {
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  // a workgroup streams through several workers; split the workers over more workgroups only
  // when the tiles alone cannot occupy the 256 compute units
  const int n_groups = s.K * (a.split > 1 ? a.split : 1);
  int chunks = (256 + tiles - 1) / tiles;
  if (chunks > n_groups) chunks = n_groups;
  a.groups_per_block = (n_groups + chunks - 1) / chunks;
  const int gy = (n_groups + a.groups_per_block - 1) / a.groups_per_block;
  hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_WGRAD, false, S>), dim3(tiles, gy, 1),
                     dim3(WM * WN * 64), 0, st, a, s);
}

// forward / input gradient
template <int BM, int BN, int WM, int WN, int S>
void launch_bf16_plain(GemmArgs a, const Segs& s, hipStream_t st) {
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  a.groups_per_block = 1;
  dim3 grid(tiles, 1, 1), block(WM * WN * 64);
  if (a.mode == MODE_FWD)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_FWD, false, S>), grid, block, 0, st, a, s);
  else
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_DGRAD, false, S>), grid, block, 0, st, a, s);
}

// Weight gradient with the weighted aggregation folded in: 256 x 128 tiles leave room for a
// second set of accumulators; every workgroup takes all workers of its tile.  A matrix with too
// few such tiles for the 256 compute units takes 128 x 128 tiles.  Eight waves (wave tile
// 64 x 64 / 32 x 64: both accumulator sets within 256 registers, two waves per SIMD) measured
// 5 % and 13 % faster than four: one wave issues MFMAs while the other waits for a copy or a
// store instruction to be accepted.
constexpr int AGG_BM = 256, AGG_BN = 128, AGG_SMALL = 128;
int64_t tiles_of(const GemmArgs& a, int bm, int bn) {
  return (int64_t)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn);
}
void launch_bf16_wgrad_agg(GemmArgs a, const Segs& s, hipStream_t st) {
  a.groups_per_block = s.K;
  if (tiles_of(a, AGG_BM, AGG_BN) >= 256)
    hipLaunchKernelGGL((gemm_bf16_kernel<AGG_BM, AGG_BN, 4, 2, MODE_WGRAD, false, 5, true>),
                       dim3((unsigned)tiles_of(a, AGG_BM, AGG_BN)), dim3(512), 0, st, a, s);
  else
    hipLaunchKernelGGL((gemm_bf16_kernel<AGG_SMALL, AGG_SMALL, 4, 2, MODE_WGRAD, false, 5, true>),
                       dim3((unsigned)tiles_of(a, AGG_SMALL, AGG_SMALL)), dim3(512), 0, st, a, s);
}

// implicit-GEMM convolution (operand A gathered).  The reduction is short (9 x channels), so a
// tile spends much of its time filling and draining the load ring: the rings are kept shallow
// enough (80 KB) for two workgroups per compute unit, whose phases then overlap.  Up to 64
// output channels: 256 x 64 tiles (no half-empty MFMA columns); otherwise 128 x 128.
template <int BM, int BN, int WM, int WN, int S>
void launch_bf16_gather_as(GemmArgs a, const Segs& s, hipStream_t st) {
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  a.groups_per_block = 1;
  dim3 grid(tiles, 1, 1), block(WM * WN * 64);
  if (a.mode == MODE_FWD)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_FWD, true, S>), grid, block, 0, st, a, s);
  else
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_DGRAD, true, S>), grid, block, 0, st, a, s);
}

void launch_bf16_gather(GemmArgs a, const Segs& s, hipStream_t st) {
  a.gather_log2cp = -1;
  const int64_t src_bytes = ((int64_t)((a.M + a.row_h * a.row_w - 1) / (a.row_h * a.row_w)) * a.src_h *
                             a.src_w + 1) * a.lda * 2;
  if (a.cp >= 32 && (a.cp & (a.cp - 1)) == 0 && !(a.conv == 2 && a.stride != 1) &&
      src_bytes < ((int64_t)1 << 31))
    for (int l = 5; l < 31; ++l)
      if ((1 << l) == a.cp) a.gather_log2cp = l;
  if (a.N <= 64)
    launch_bf16_gather_as<256, 64, 4, 1, 4>(a, s, st);
  else
    launch_bf16_gather_as<128, 128, 2, 2, 5>(a, s, st);
}

void launch_f32(const GemmArgs& a, const Segs& s, int groups, hipStream_t st) {
  dim3 grid((a.M + 63) / 64, (a.N + 63) / 64, groups), block(256);
  switch (a.mode) {
    case MODE_FWD:
      hipLaunchKernelGGL(gemm_f32_kernel<MODE_FWD>, grid, block, 0, st, a, s);
      break;
    case MODE_DGRAD:
      hipLaunchKernelGGL(gemm_f32_kernel<MODE_DGRAD>, grid, block, 0, st, a, s);
      break;
    default:
      hipLaunchKernelGGL(gemm_f32_kernel<MODE_WGRAD>, grid, block, 0, st, a, s);
  }
}

}  // namespace

bool gemm_fuses_aggregate(int dtype, const GemmArgs& a, const Segs& s) {
  // enough tiles to occupy the compute units without splitting the workers over workgroups
  return dtype == DYNB_BF16 && a.mode == MODE_WGRAD && !a.conv && a.split <= 1 &&
         tiles_of(a, AGG_SMALL, AGG_SMALL) >= 256 && s.K <= DYNB_MAX_WORKERS;
}

int launch_gemm(int dtype, const GemmArgs& args, const Segs& s, void* stream) {
  GemmArgs a = args;
  a.zeros = device_zero_granule();
  if (!a.zeros) return fail(DYNB_ERR_HIP, "gemm: no address for the zero granule");
  if (a.M <= 0 || a.N <= 0) return DYNB_OK;
  if (a.agg && !gemm_fuses_aggregate(dtype, a, s))
    return fail(DYNB_ERR_UNSUPPORTED, "gemm: this weight gradient cannot fold the aggregation in");
  const int es = dtype == DYNB_BF16 ? 2 : 4;
  const int gran = 16 / es;
  if ((a.lda % gran) || (a.ldb % gran) || ((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15))
    return fail(DYNB_ERR_BADARG, "gemm: operands must have 16-byte aligned rows");
  // the bf16 kernels keep operand byte offsets in 32 bits
  if (dtype == DYNB_BF16 && !a.conv) {
    const int64_t rows_a = a.mode == MODE_WGRAD ? s.off[s.K] : a.M;
    const int64_t rows_b = a.mode == MODE_WGRAD ? s.off[s.K] : a.N;
    const int64_t lim = (int64_t)1 << (a.mode == MODE_WGRAD ? 31 : 32);   // (see async_copy_1k_buffer)
    if (rows_a * a.lda * es >= lim || rows_b * a.ldb * es >= lim)
      return fail(DYNB_ERR_UNSUPPORTED, "gemm: an operand of %d GiB or more (rows * pitch) is not supported",
                  a.mode == MODE_WGRAD ? 2 : 4);
  }
  if (a.bias_grad && (dtype != DYNB_BF16 || a.mode != MODE_WGRAD || a.split > 1))
    return fail(DYNB_ERR_UNSUPPORTED, "gemm: the bias gradient rides along with an unsplit bf16 weight gradient only");
  if (a.addend && (dtype != DYNB_BF16 || a.mode != MODE_DGRAD))
    return fail(DYNB_ERR_UNSUPPORTED, "gemm: an addend belongs to a bf16 input gradient");
  const int groups = a.mode == MODE_WGRAD ? s.K : 1;
  KClass cls = a.mode == MODE_FWD ? KC_GEMM_FWD : a.mode == MODE_DGRAD ? KC_GEMM_DGRAD
                                                                        : KC_GEMM_WGRAD;
  // (the two tile sizes of the bf16 weight gradient are different kernels with different
  // bounds: timed apart, so that a class's average launch is one kernel's)
  if (a.mode == MODE_WGRAD && dtype == DYNB_BF16 && !a.conv) {
    const bool large = a.agg ? tiles_of(a, AGG_BM, AGG_BN) >= 256
                             : (int64_t)((a.M + 255) / 256) * ((a.N + 255) / 256) >= 192;
    if (!large) cls = KC_GEMM_WGRAD_SMALL;
  } else if (dtype == DYNB_BF16 && !a.conv &&
             (int64_t)((a.M + 255) / 256) * ((a.N + 255) / 256) < 192) {
    cls = KC_GEMM_SMALL;
  }
  Timed t(cls, stream, a.alg_flops, a.alg_bytes);
  if (a.conv) {
    if (dtype != DYNB_BF16 || a.mode == MODE_WGRAD || (a.cp & 7) || (a.stride != 1 && a.stride != 2))
      return fail(DYNB_ERR_UNSUPPORTED, "gemm: gathered operand needs bf16, forward/input-gradient mode");
    if (conv_direct_applies(dtype, a)) return launch_conv_direct(a, stream);
    launch_bf16_gather(a, s, (hipStream_t)stream);
  } else if (dtype == DYNB_BF16 && a.agg) {
    launch_bf16_wgrad_agg(a, s, (hipStream_t)stream);
  } else if (dtype == DYNB_BF16) {
    // large tiles have the best LDS-traffic-to-MFMA ratio; small problems need more, smaller
    // tiles to occupy 256 compute units.  Forward / input gradient on 256 x 256 tiles run EIGHT
    // waves (wave tile 128 x 64, at most 256 registers each): two waves per SIMD, so that one
    // can issue MFMAs while the other waits for a copy instruction to be accepted (input
    // gradient 112 -> 102 us, forward 126 -> 124 us per 4096^3 launch against four waves of
    // 128 x 128).  The weight gradient keeps four waves: its 256 accumulators per lane leave no
    // room for a second wave on a SIMD.
    const int64_t big = (int64_t)((a.M + 255) / 256) * ((a.N + 255) / 256);
    const hipStream_t st = (hipStream_t)stream;
    if (a.mode == MODE_WGRAD) {
      if (big >= 192)
        launch_bf16_wgrad<256, 256, 2, 2, 4>(a, s, st);   // 128 + 18 KB of LDS
      else
        launch_bf16_wgrad<128, 128, 2, 2, 8>(a, s, st);
    } else if (big >= 192) {
      launch_bf16_plain<256, 256, 2, 4, 5>(a, s, st);     // all 160 KB of LDS
    } else {
      launch_bf16_plain<128, 128, 2, 2, 8>(a, s, st);
    }
  } else
    launch_f32(a, s, groups, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "gemm launch failed");
}

}  // namespace dynb
