// bf16 MFMA tile GEMM for gfx950 with three fused epilogues.
//
// One kernel body computes C[m][n] = sum_k A[m][k] * B[n][k] for a 256 x 256
// tile per workgroup (both operands K-contiguous, "NT" form).  Four wave64
// wavefronts form a 2 x 2 grid, each owning a 128 x 128 sub-tile as 8 x 8
// MFMA 16x16x32 accumulators (256 accumulator registers per lane).  The
// 16x16x32 shape is chosen over 32x32x16 for energy: with real (random-mantissa)
// operands the chip is power-limited, and an MFMA-only loop sustains about 13 %
// more FLOP/s with the 16 x 16 shape.  Operand panels of 64 K-elements go from
// global memory straight into LDS (global_load ... lds, no staging registers)
// into a double buffer.  LDS rows are 128 bytes whose 16-byte chunks are
// XOR-swizzled with (row / 2) % 8: a 128-bit LDS read is served 16 lanes (16
// rows of one chunk column) per cycle over 64 banks, rows 2 apart share a bank
// window, and the swizzle spreads them over the eight chunk slots, so the
// fragment reads of the MFMA operands are bank-conflict free; the swizzle is
// applied on the global side (each lane picks the chunk whose LDS slot it owns)
// because a direct load writes the wave's 64 x 16 bytes contiguously.
//
// The three uses on the scoring path (Sec. 3: log pi(y_t | ...) needs the
// softmax over the whole vocabulary of the LM-head logits):
//   FWD: A = W (vocabulary rows), B = H (token rows, gathered).  The MFMA result
//        layout keeps 4 rows x 1 column per lane, so putting the vocabulary on
//        the M side makes the max / sum-exp reduction over the vocabulary an
//        in-register reduction with two cross-lane steps.  The fragment rows are
//        permuted so that a lane's accumulators are 8 consecutive vocabulary ids
//        and the stash of exponentials e = exp(z - row offset) is stored as bf16
//        straight from registers.
//   DH : A = stash rows (tokens), B = W^T; each output row is multiplied by its
//        row scale (-g / S) and scattered to its slot.
//   DW : A = stash^T, read from the stash rows themselves (K-major panel, transposing
//        LDS reads), B = (row-scaled H)^T; fp32 read-modify-write of dW.
#include "../../include/mrl.h"
#include "../../include/mrl_diag.h"
#include "mrl_internal.h"

namespace mrl {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NTHREADS = 256;
constexpr int NSTAGE = 2;                          // LDS double buffer of K panels
constexpr int TILE_BYTES = BM * BK * 2;            // one operand panel: 32 KB (256 rows x 128 B)
constexpr int STAGE_BYTES = 2 * TILE_BYTES;        // A + B
constexpr int DHSTAGE_LD = BM + 8;                   // bf16 elements per row of the dH epilogue's staging tile
constexpr int DHSTAGE_BYTES = BN * DHSTAGE_LD * 2;     // 132 KB
constexpr int PIPE_BYTES = NSTAGE * STAGE_BYTES;   // 128 KB
// Direct loads of a slot's 16 (per wave), by the group of the K loop that issues them: the slot is
// released by the barrier in group 5, so its refill starts there and may run on into groups 0 - 4
// of the next panel (it is needed at that panel's barrier).
constexpr int kLoadsInGroup[8] = {4, 0, 0, 0, 0, 4, 4, 4};
constexpr int load_index_base(int g) {      // loads issued before group g, in the order 5, 6, 7, 0, 1, ...
  int n = 0;
  for (int h = 5; h != g; h = (h + 1) & 7) n += kLoadsInGroup[h];
  return n;
}
constexpr int kLoadsCarriedOver = kLoadsInGroup[0] + kLoadsInGroup[1] + kLoadsInGroup[2] + kLoadsInGroup[3] + kLoadsInGroup[4];
static_assert(kLoadsCarriedOver + kLoadsInGroup[5] + kLoadsInGroup[6] + kLoadsInGroup[7] == 16, "a slot takes 16 loads per wave");
constexpr int kDwTailMaxItems = 256;                // K slices of dW tail tiles per launch: one per compute unit
constexpr int ZT_BYTES = BN * 4;                   // forward: the tile's 256 target logits, behind the panels
template <int MODE> constexpr int lds_bytes() {
  return MODE == 0 ? PIPE_BYTES + ZT_BYTES : (DHSTAGE_BYTES > PIPE_BYTES ? DHSTAGE_BYTES : PIPE_BYTES);
}

// s_waitcnt immediates (gfx9 encoding): wait until at most N vector-memory loads are
// outstanding, no wait on the export / LDS counters.
constexpr int waitcnt_vm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

enum { MODE_FWD = 0, MODE_DH = 1, MODE_DW = 2 };
constexpr int NXCD = 8;
template <bool B> struct Flag { static constexpr bool value = B; };

struct Params {
  const uint16_t* A; int64_t lda; int M;
  const uint16_t* B; int64_t ldb; int N;
  int K;
  const int32_t* row_index;   // already offset to the chunk start
  const int64_t* n_scored; int64_t chunk_start; int chunk_rows;
  int sup_m, sup_n;           // super-tile shape of the workgroup -> tile mapping
  // FWD
  const float* zt; float* part_sum; float* part_ez; int64_t part_stride; uint16_t* estash; int64_t lde; int V;
  // DH
  const float* row_scale; void* dH; int dh_f32; int d;
  // DW
  float* dW; int overwrite;
  // DW, K-split tail (see dw_tail_plan): workgroups from main_blocks on take the tiles of the
  // tile rows tail_m0 .. tail_m0 + tail_rows - 1, each cut into tail_split slices of the
  // contraction, and store their accumulators to tail_part instead of dW
  int main_blocks, tail_m0, tail_rows, tail_split; float* tail_part;
  int tail_first[NXCD + 1];   // items tail_first[x] .. tail_first[x + 1] - 1 run on XCD x
};

// Workgroup -> tile mapping.  Workgroups are dealt round-robin to the 8 XCDs, each with its own
// L2 and 32 compute units; sup_m x sup_n consecutive workgroups of one XCD form a super-tile so
// that they share operand panels in that L2 (each A panel is used by sup_n tiles, each B panel by
// sup_m), and super-tiles are numbered N-fastest so that the XCDs walk the same A rows at the same
// time.  The shape is picked per launch from what measurement favours: 8 x 4 when the N extent is
// a multiple of 4 tiles, else 8 x 2.  Two things matter more than the panel-sharing count: the N
// extent must fill whole super-tile columns (6 tiles at d = 1536 and 14 at d = 3584 leave 8 x 4
// with a half-empty last column: dH / dW 11-30 % slower than 8 x 2), and the super-tile size
// must divide the 32 compute units of an XCD, so that the workgroups running on it at any time
// are whole super-tiles (shapes of 24, 28 or 30 tiles lose 5-20 %).
struct SuperTile { int m, n; };
inline SuperTile pick_super_tile(int Nt) {
  if (Nt % 4 == 0) return {8, 4};
  if (Nt == 1) return {16, 1};
  return {8, 2};
}
__host__ __device__ inline int num_blocks(int Mt, int Nt, int sup_m, int sup_n) {
  int s = ((Mt + sup_m - 1) / sup_m) * ((Nt + sup_n - 1) / sup_n);
  return (s + NXCD - 1) / NXCD * NXCD * (sup_m * sup_n);
}
__device__ inline bool tile_coords(int bid, int Mt, int Nt, int sup_m, int sup_n, int& tm, int& tn, int& sm, int& sn) {
  const int sNt = (Nt + sup_n - 1) / sup_n, sMt = (Mt + sup_m - 1) / sup_m;
  const int xcd = bid % NXCD, local = bid / NXCD;
  const int q = local / (sup_m * sup_n), within = local % (sup_m * sup_n);
  const int s = q * NXCD + xcd;
  if (s >= sMt * sNt) return false;
  sm = within % sup_m; sn = within / sup_m;
  tm = (s / sNt) * sup_m + sm;
  tn = (s % sNt) * sup_n + sn;
  return tm < Mt && tn < Nt;
}

// swizzle of the K-major A panel: rows k, k+1, k+2, k+3 and k+8 (or k+16) get distinct values
__device__ inline int kswz(int k) { return (k & 3) | ((((k >> 3) ^ (k >> 4)) & 1) << 2); }

__device__ inline float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// The MFMA is issued through inline assembly with the accumulator tied in place in an
// accumulation register: left to the register allocator, a few of the 64 accumulator tuples
// (which fill the accumulation file completely) end up rotating through copies every iteration.
// The K loop issues the two 32-wide K steps of an accumulator back to back: the second MFMA reads
// as SrcC the register tuple the first one writes as vDst.  That dependent pair with identical
// SrcC / vDst is the case the hardware interlocks by itself (no software wait states required);
// no other instruction touches an accumulator inside the loop.  The first ordinary reads after
// the K loop are fenced by drain_mfma() below.
__device__ __forceinline__ void mfma16(f32x4& c, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
// Wait states between the last MFMAs of the K loop and the first ordinary read of their
// results (the hazard checker of the compiler does not look into inline assembly).
__device__ __forceinline__ void drain_mfma(f32x4 (&r)[8]) {
  asm volatile("s_nop 15\n\ts_nop 15"
               : "+a"(r[0]), "+a"(r[1]), "+a"(r[2]), "+a"(r[3]), "+a"(r[4]), "+a"(r[5]), "+a"(r[6]), "+a"(r[7]));
}

template <int MODE>
__global__ __launch_bounds__(NTHREADS) void gemm_nt_bf16(Params p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // Lane and wave number as the code after the K loop takes them: recomputed there from the
  // execution mask and a scalar, so that nothing lane-dependent has to stay alive (that is, be
  // spilled to scratch memory) across the loop, whose body owns every vector register.  A
  // reload from scratch is a vector-memory load: the wait for it would also wait for every
  // store issued before it, and between the stores of the forward epilogue that costs
  // microseconds each time.
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto lane_now = []() {
    int l = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(l));   // opaque: what is derived from it is computed where it is used, not hoisted
    return l;
  };

  // valid rows of this chunk (device-side, no host sync)
  int64_t nv64 = *p.n_scored - p.chunk_start;
  const int nvalid = nv64 < 0 ? 0 : (nv64 > p.chunk_rows ? p.chunk_rows : (int)nv64);

  int M = p.M, N = p.N, K = p.K;
  if (MODE == MODE_FWD) N = nvalid;
  if (MODE == MODE_DH) M = nvalid;
  if (MODE == MODE_DW) { int kv = (nvalid + 2 * BK - 1) / (2 * BK) * (2 * BK); K = kv < K ? kv : K; }
  if (MODE == MODE_FWD && nvalid == 0) return;
  if (MODE == MODE_DH && nvalid == 0) return;
  if (MODE == MODE_DW && nvalid == 0 && !p.overwrite) return;

  const int Mt = (p.M + BM - 1) / BM, Nt = (p.N + BN - 1) / BN;
  int tm, tn, sm, sn;
  int k_first = 0;                 // first K panel of this workgroup (DW tail slices start later)
  float* tail_out = nullptr;       // DW tail slice: where the accumulators go instead of dW
  if (MODE == MODE_DW && p.tail_split > 0) {
    if ((int)blockIdx.x < p.main_blocks) {
      if (!tile_coords(blockIdx.x, p.tail_m0, Nt, p.sup_m, p.sup_n, tm, tn, sm, sn)) return;
    } else {
      // one XCD takes consecutive items (the host says how many: the XCDs that the whole tiles
      // leave idle earlier take more), i.e. mostly tiles of one slice: they walk the same K range
      // and share its operand panels in that L2
      const int e = blockIdx.x - p.main_blocks;
      const int tiles = p.tail_rows * Nt;
      const int item = p.tail_first[e % NXCD] + e / NXCD;
      if (item >= p.tail_first[e % NXCD + 1]) return;
      const int slice = item / tiles, t = item % tiles;
      sm = t / Nt; sn = t % Nt;
      tm = p.tail_m0 + sm; tn = sn;
      // slices of an even number of panels (the loop body is two panels)
      const int nk_all = K / BK;
      const int per = ((nk_all + p.tail_split - 1) / p.tail_split + 1) & ~1;
      k_first = slice * per;
      const int k_end = k_first + per < nk_all ? k_first + per : nk_all;
      K = k_end > k_first ? (k_end - k_first) * BK : 0;
      tail_out = p.tail_part + (int64_t)item * (BM * BN);
    }
  } else if (!tile_coords(blockIdx.x, Mt, Nt, p.sup_m, p.sup_n, tm, tn, sm, sn)) return;
  const int m0 = tm * BM, n0 = tn * BN;
  if (m0 >= M || n0 >= N) return;

  // ---- global -> LDS: one direct load moves 1 KB, contiguous in LDS.
  // Row-major operands ([row][k], k contiguous): 8 rows x 128 B per load.  Wave w owns row
  // blocks 8w .. 8w+7 of each operand panel; lane l fills LDS chunk (row l/8, slot l%8) and
  // therefore fetches logical chunk slot ^ ((row >> 1) & 7).
  // K-major A operand (DW: A[m][k] = dz[k][m], stored as token rows with the vocabulary
  // contiguous): the panel is 64 k rows x 512 B and a load moves 2 of them; lane l fills chunk
  // slot l%32 of row l/32 and fetches logical chunk slot ^ (h(k) << 1), the swizzle that makes
  // the transposing fragment reads below conflict-free.
  constexpr bool A_KMAJOR = (MODE == MODE_DW);
  // FWD: the 16 rows of A fragment i are not 16 consecutive panel rows but
  //   rho(i, r) = 32*(i/2) + 8*(r/4) + 4*(i%2) + r%4      (within the wave's 128 rows),
  // so that a lane's accumulators (i = 2t, 2t+1; e = 0..3) are 8 consecutive vocabulary ids
  // and the bf16 stash of exponentials can be stored from registers, 16 bytes per lane, without an LDS round
  // trip.  The chunk swizzle of the A panel then takes row bits 1, 3, 4 (the ones that vary
  // inside a fragment) instead of bits 1-3.
  constexpr bool A_PERM = (MODE == MODE_FWD);
  const int64_t a_kstep = A_KMAJOR ? (int64_t)BK * p.lda : BK;   // elements per K panel
  const int lrow = lane >> 3;
  const uint16_t* a_ptr[8];
  const uint16_t* b_ptr[8];
  // Workgroups that share a panel (same sm for A, same sn for B) walk its row blocks in a
  // different cyclic order (rot_a, rot_b), so that they do not all ask the L2 for the same lines
  // at the same moment (1-2 % on the forward and dH launches).
  uint32_t lds_a[8], lds_b[8];                        // LDS offset of load i within the wave's 8 KB
  const float* zt_ptr = nullptr;                      // forward: this lane's entry of the tile's target logits
  {
    const int rot_a = (sn * 8 / p.sup_n) & 7, rot_b = (sm * 8 / p.sup_m) & 7;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int ia = (i + rot_a) & 7, ib = (i + rot_b) & 7;
      lds_a[i] = __builtin_amdgcn_readfirstlane(ia * 1024);
      lds_b[i] = __builtin_amdgcn_readfirstlane(ib * 1024);
      const int r = (wave * 8 + ia) * 8 + lrow;         // row within the 256-row panel
      const int rB = (wave * 8 + ib) * 8 + lrow;
      const int lchunk = (lane & 7) ^ ((rB >> 1) & 7);
      const int lchunk_a = A_PERM ? ((lane & 7) ^ (((r >> 1) & 1) | (((r >> 3) & 3) << 1))) : ((lane & 7) ^ ((r >> 1) & 7));
      int ra = m0 + r; ra = ra < M ? ra : M - 1;
      int rb = n0 + rB; rb = rb < N ? rb : N - 1;
      int64_t rowa = ra, rowb = rb;
      if (A_KMAJOR) {
        const int k = 2 * (wave * 8 + ia) + (lane >> 5);  // k row within the panel
        a_ptr[i] = p.A + ((int64_t)k_first * BK + k) * p.lda + m0 + (((lane & 31) ^ (kswz(k) << 1)) << 3);
      } else {
        a_ptr[i] = p.A + rowa * p.lda + lchunk_a * 8;
      }
      b_ptr[i] = p.B + rowb * p.ldb + lchunk * 8 + (MODE == MODE_DW ? k_first * BK : 0);
    }
    if (MODE == MODE_FWD) {
      int n = n0 + wave * 64 + lane; n = n < N ? n : N - 1;
      zt_ptr = p.zt + n;
    }
  }
  // The direct load is issued through inline assembly on purpose: the compiler's wait-count
  // pass treats a global load that writes LDS as touching both address spaces and then
  // drains every counter to zero before each LDS read, which serialises the pipeline.
  // Issued this way the loads are invisible to that pass; their completion is awaited
  // explicitly below with s_waitcnt vmcnt(0) before the barrier that publishes a panel.
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_base + wave * 8192);

  auto load_lds16 = [](const uint16_t* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(g), "s"(lds_addr) : "memory");
  };
  // loads i0 .. i0+n-1 (of 8) of both operand panels of K panel kt into ring slot `slot`
  auto issue_loads = [&](int kt, int slot, int i0, int n) {
    const uint32_t st = slot * STAGE_BYTES + wave_lds;
    const int koff = kt * BK;
#pragma unroll
    for (int i = i0; i < i0 + n; ++i) {
      load_lds16(a_ptr[i] + kt * a_kstep, st + lds_a[i]);
      load_lds16(b_ptr[i] + koff, st + TILE_BYTES + lds_b[i]);
    }
  };

  // forward: the tile's 256 target logits travel to LDS with the tile's first panel (4 bytes per
  // lane, one direct load per wave) and are published by the same barrier, so that the epilogue
  // starts without a round trip to global memory
  auto issue_zt = [&]() {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 :: "v"(zt_ptr), "s"(__builtin_amdgcn_readfirstlane(lds_base + PIPE_BYTES + wave * 256))
                 : "memory");
  };

  // ---- fragment read offsets.  A 16x16x32 operand fragment: lane -> row (lane & 15),
  // 16-byte K chunk (lane >> 4) of a 32-wide K step.  A 128-bit LDS read is served 16 lanes
  // per cycle over 64 banks; rows 2 apart share a bank window (128-byte rows), the swizzle
  // (row / 2) % 8 spreads the 16 rows of a fragment over distinct banks.
  const int frow = lane & 15, fq = lane >> 4;
  int a_off[2], b_off[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int chunk = ((ks << 2) | fq) ^ ((frow >> 1) & 7);
    if (A_PERM) {
      const int chunk_a = ((ks << 2) | fq) ^ (((frow >> 1) & 1) | ((frow >> 2) << 1));
      a_off[ks] = (wm * 128 + 8 * (frow >> 2) + (frow & 3)) * 128 + (chunk_a << 4);
    } else {
      a_off[ks] = (wm * 128 + frow) * 128 + (chunk << 4);
    }
    b_off[ks] = TILE_BYTES + (wn * 128 + frow) * 128 + (chunk << 4);
  }

  // K-major A panel: the transposing LDS read hands lane (g = lane / 16, s = lane % 16) the four
  // k values kb .. kb+3 of column m = mb + s when lane s points at row kb + s/4, columns
  // mb + 4*(s%4) .. +3.  Two of them (kb = 8g and 8g + 4 within the K step) make the lane's
  // 8-element fragment.  A 64-bit read is served 32 lanes per cycle: 8 rows x 32 bytes, and the
  // swizzle h(k) moves the 32-byte column groups of those rows to distinct bank windows.
  int a_tr_base = 0;
  if (A_KMAJOR) {
    const int k = 8 * fq + (frow >> 2);
    a_tr_base = k * 512 + wm * 256 + (kswz(k) << 5) + ((frow & 2) << 3) + ((frow & 1) << 3);
  }
  auto read_a = [&](int st, int ks, int ib) -> bf16x8 {
    if (A_KMAJOR) {
      typedef short v4i16 __attribute__((ext_vector_type(4)));
      typedef short v8i16 __attribute__((ext_vector_type(8)));
      typedef __attribute__((address_space(3))) v4i16* lds_v4i16;
      unsigned char* q = smem + st + (a_tr_base ^ (ib << 5)) + ks * 16384;
      const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16)q);
      const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16)(q + 2048));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
    return *reinterpret_cast<const bf16x8*>(smem + st + a_off[ks] +
                                            (A_PERM ? (ib >> 1) * 4096 + (ib & 1) * 512 : ib * 2048));
  };

  f32x4 acc[8][8];
  const int nk = K / BK;
  // Software pipeline.  Panel kt+1 is loaded during the MFMAs of panel kt (double buffer).
  // A panel is 8 groups; group g multiplies the A fragments of 16-row block g (both 32-wide
  // K steps) with the panel's 16 B fragments: 16 MFMAs, the two K steps of an accumulator back
  // to back.  Keeping an accumulator for two consecutive MFMAs costs measurably less energy than
  // touching 64 different ones in turn (about 5 % more FLOP/s from an MFMA-only loop at the
  // power limit), which is what bounds these kernels on real data.
  // Registers: the B fragments of a whole panel stay resident, in two sets (this panel / the
  // next one); A fragments sit in a ring of four pairs.  The schedule of reads, barrier and
  // direct loads around the MFMAs is described at `side` below.
  // The loop body (two panels, so that the B sets have fixed registers) is branch-free; loads
  // that would run past the end re-fetch the last panel into a slot nobody reads.
  bf16x8 fbx[2][2][8];   // [set][K step][16-column block]
  bf16x8 fax[4][2];      // [ring slot][K step]
  auto read_b = [&](int st, int ks, int j) -> bf16x8 {
    return *reinterpret_cast<const bf16x8*>(smem + st + b_off[ks] + j * 2048);
  };
  // One load of the K loop: three instructions, what one MFMA leaves room for.  The address
  // arithmetic (panel offset, uniform) is part of the piece, and it separates the write of M0
  // from the load that reads it (one wait state).
  auto load_lds16_at = [](const uint16_t* base, int64_t byte_off, uint32_t lds_addr) {
    uint64_t addr;
    asm volatile("s_mov_b32 m0, %3\n\tv_lshl_add_u64 %0, %1, 0, %2\n\tglobal_load_lds_dwordx4 %0, off"
                 : "=&v"(addr) : "v"(base), "s"(byte_off), "s"(lds_addr) : "memory");
  };
  auto issue_range = [&](int kt, int slot, int j0, int j1) {
#pragma unroll
    for (int j = j0; j < j1; ++j) {
      const uint32_t st = slot * STAGE_BYTES + wave_lds;
      if (j & 1) load_lds16_at(b_ptr[j >> 1], (int64_t)kt * (BK * 2), st + TILE_BYTES + lds_b[j >> 1]);
      else load_lds16_at(a_ptr[j >> 1], (int64_t)kt * a_kstep * 2, st + lds_a[j >> 1]);
    }
  };
  // One panel = 8 groups of 16 MFMAs.  A wave issues in order and the matrix pipe takes a new MFMA
  // only every 16 cycles, so whatever stands between two MFMAs in the instruction stream is free
  // as long as it fits the 12 issue cycles the pipe leaves over - and costs pipe time when it
  // comes as a block after the sixteenth.  The side work of a panel (fragment reads, the barrier,
  // direct loads with their address arithmetic) is therefore cut into pieces of one to four
  // instructions, one piece after an MFMA, in source order (both are volatile assembly or fenced):
  //   group 0      : A fragments of row block 3 (this panel); the last loads of the NEXT panel's slot
  //   groups 1 - 4 : A fragments of row blocks 4 - 7
  //   group 5      : wait for this thread's part of panel kt+1, barrier (every wave has issued its
  //                  last read of this panel's slot by then, so the slot can be refilled; panel
  //                  kt+1 becomes visible); next panel's A block 0, B column blocks 0 - 2; the first
  //                  loads of panel kt+2 into this panel's slot
  //   group 6      : next A block 1, B blocks 3 - 5, loads
  //   group 7      : next A block 2, B blocks 6 - 7, loads   (the rest follows in group 0 of the
  //                  next panel; kLoadsInGroup says how many where)
  // A fragments sit in a ring of four pairs: group g multiplies ring slot g % 4, and the slot a
  // group has just finished with is refilled during the next group.  Four loads per group over
  // four groups measured best: packing them into groups 5 - 7 costs 2 - 4 % (the load path of a
  // compute unit takes about 23 cycles per 1 KB load, four waves issuing one every 16 cycles run
  // its queue full and stall their MFMAs with it), spreading them further leaves the late ones
  // too little time to land.
  auto side = [&](int g, int m, int set, int st_cur, int st_nxt, int kt_nxt, int slot_nxt, int kt_load, int slot_cur) {
    // pieces before the loads: the barrier (group 5) and the fragment reads
    int nr = 2;
    if (g == 0) {
      if (m < 2) fax[3][m] = read_a(st_cur, m, 3);
    } else if (g <= 4) {
      if (m < 2) fax[(g - 1) & 3][m] = read_a(st_cur, m, g + 3);
    } else {
      const int q = g - 5;                          // 0, 1, 2
      if (g == 5 && m == 0) {
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        __syncthreads();
      }
      if (m >= 1 && m < 3) fax[q][m - 1] = read_a(st_nxt, m - 1, q);
      const int nb = q == 2 ? 2 : 3;                // B column blocks read in this group
      if (m >= 3 && m < 3 + 2 * nb) { const int j = 3 * q + (m - 3) / 2, ks = (m - 3) & 1; fbx[set ^ 1][ks][j] = read_b(st_nxt, ks, j); }
      nr = 3 + 2 * nb;
    }
    // this group's share of the 16 loads that fill a slot, spread over the remaining gaps
    const int nl = kLoadsInGroup[g];
    if (nl > 0 && m >= nr) {
      const int room = 16 - nr;
#pragma unroll
      for (int i = 0; i < nl; ++i)
        if (m == nr + i * room / nl) {
          const int l = load_index_base(g) + i;
          if (g >= 5) issue_range(kt_load, slot_cur, l, l + 1);
          else issue_range(kt_nxt, slot_nxt, l, l + 1);
        }
    }
  };
  auto panel = [&](int set, int st_cur, int st_nxt, int kt_nxt, int slot_nxt, int kt_load, int slot_cur) {
#pragma unroll
    for (int g = 0; g < 8; ++g) {
#pragma unroll
      for (int m = 0; m < 16; ++m) {
        mfma16(acc[g][m >> 1], fax[g & 3][m & 1], fbx[set][m & 1][m >> 1]);
        side(g, m, set, st_cur, st_nxt, kt_nxt, slot_nxt, kt_load, slot_cur);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  auto last_k = [&](int k) { return k < nk ? k : nk - 1; };
  // The number of panels is even (the launchers see to it), so that the two-panel body is the
  // only code that touches the accumulators: there is no peeled tail whose different register
  // assignment would make the compiler move accumulators around next to MFMAs it cannot see
  // into.  The last two panels read ahead and load like any other (the panel after the last is
  // a re-fetch of the last one, read into registers nobody uses).
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  if (nk > 0) {
    issue_loads(0, 0, 0, 8);
    if (MODE == MODE_FWD) issue_zt();
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __syncthreads();
    issue_range(last_k(1), 1, 0, 16 - kLoadsCarriedOver);   // the rest comes with the first groups of the first panel
#pragma unroll
    for (int j = 0; j < 8; ++j) { fbx[0][0][j] = read_b(0, 0, j); fbx[0][1][j] = read_b(0, 1, j); }
#pragma unroll
    for (int i = 0; i < 3; ++i) { fax[i][0] = read_a(0, 0, i); fax[i][1] = read_a(0, 1, i); }
    for (int kt = 0; kt < nk; kt += 2) {
      panel(0, 0, STAGE_BYTES, last_k(kt + 1), 1, last_k(kt + 2), 0);
      panel(1, STAGE_BYTES, 0, last_k(kt + 2), 0, last_k(kt + 3), 1);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // no direct load may outlive the wave
    drain_mfma(acc[7]);
  }

  // ---- epilogues.  Accumulator element (i, j, e) of this lane is
  //   row m = m0 + wm*128 + i*16 + 4*(lane>>4) + e      (FWD: the permuted row, see vrow below)
  //   col n = n0 + wn*128 + j*16 + (lane & 15)
  if (MODE == MODE_DH) __syncthreads();   // its staged epilogue reuses the panels' LDS
  const int mrow_base = m0 + wm * 128 + 4 * fq;
  const int ncol_base = n0 + wn * 128 + frow;

  if (MODE == MODE_FWD) {
    const int lane = lane_now(), wave = wave_u;
    const int wm = wave >> 1, wn = wave & 1, frow = lane & 15, fq = lane >> 4;
    const int ncol_base = n0 + wn * 128 + frow;
    // rows = vocabulary ids, cols = token rows of the chunk.  Exponentials are taken relative to
    // the row's offset c2 = z_target * log2(e) + margin (log2 domain), one offset for all
    // vocabulary tiles of a row: e = 2^(z log2(e) - c2), clamped so that neither e nor any sum of
    // it can overflow.  The sums over the wave's 128 vocabulary ids are this tile's partials; e
    // itself, as bf16, is the backward pass's operand (dz = (-g / S)(e - S onehot)).
    constexpr float LOG2E = 1.4426950408889634f;
    const bool full = (m0 + BM <= p.V);
    const int pidx = tm * 2 + wm;
    // vocabulary id of accumulator (i, e) of this lane
    auto vrow = [&](int i, int e) {
      return m0 + wm * 128 + 32 * (i >> 1) + 8 * fq + 4 * (i & 1) + e;
    };
    // The body is instantiated for full / ragged vocabulary tiles and with / without the entropy
    // sums: both conditions are uniform, and left as run-time selects they cost four more
    // instructions per logit (row id, compare, two selects) than the six the work needs
    // (accumulator read, multiply-add, clamp, exponential, add, half a packed conversion).
    auto body = [&](auto full_tile, auto with_ez) {
      constexpr bool kFull = decltype(full_tile)::value, kEz = decltype(with_ez)::value;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int n = ncol_base + j * 16;
        const bool live = n < N;
        const float zt = *reinterpret_cast<const float*>(smem + PIPE_BYTES + (wn * 128 + frow + j * 16) * 4);
        const float c2 = live ? fmaf(zt, LOG2E, kStashMargin2) : 0.f;
        uint16_t* erow = p.estash + (int64_t)n * p.lde + m0 + wm * 128 + 8 * fq;
        float s = 0.f, t = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          // accumulators 2q and 2q+1 hold 8 consecutive vocabulary ids of this lane
          bf16x8 h;
#pragma unroll
          for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              // (read where it is used: left to the compiler, the copies out of the accumulation
              // registers are hoisted to the top of the epilogue and fill the register file)
              float z;
              asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(z) : "a"(acc[2 * q + u][j][e]));
              float w = exp2_fast(fminf(fmaf(z, LOG2E, -c2), kStashClamp2));
              if (!kFull) w = vrow(2 * q + u, e) < p.V ? w : 0.f;
              s += w;
              if (kEz) t = fmaf(w, z, t);     // for the entropy: sum e * z  (H = lse - E_p[z])
              h[4 * u + e] = (__bf16)w;
            }
          if (p.estash != nullptr && live) {
            // 16 bytes per lane, the four lanes of a token row side by side (64 bytes).  Streaming
            // store (non-temporal, device scope): the stash is 5 GB per launch and is next read by
            // the backward launches, so it should not displace operand panels from the L2 and the
            // memory-side cache (2 % of the launch against a plain store).  Written in assembly
            // for its cache policy bits; the two wait states after it are the ones the hardware
            // needs before the data registers of a store wider than 8 bytes may be overwritten
            // (the compiler inserts them for its own stores only).
            asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" :: "v"(erow + 32 * q), "v"(h) : "memory");
          }
        }
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (fq == 0 && live) p.part_sum[(int64_t)pidx * p.part_stride + n] = s;
        if (kEz) {
          t += __shfl_xor(t, 16);
          t += __shfl_xor(t, 32);
          if (fq == 0 && live) p.part_ez[(int64_t)pidx * p.part_stride + n] = t;
        }
        // one column block at a time: interleaving them runs the register allocator out of
        // registers, and its reloads from scratch wait for the stores issued so far
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (full) {
      if (p.part_ez != nullptr) body(Flag<true>{}, Flag<true>{}); else body(Flag<true>{}, Flag<false>{});
    } else {
      if (p.part_ez != nullptr) body(Flag<false>{}, Flag<true>{}); else body(Flag<false>{}, Flag<false>{});
    }
  } else if (MODE == MODE_DH) {
    // rows = token rows of the chunk (scattered to their slots), cols = hidden index; a row
    // of the stash times W is the row's dz W up to its scale -g / S, applied here
    if (p.dh_f32) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int m = mrow_base + i * 16 + e;
          if (m < M) {
            const float sc = p.row_scale[m];
            float* row = reinterpret_cast<float*>(p.dH) + (int64_t)p.row_index[m] * p.d;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const int n = ncol_base + j * 16;
              if (n < p.d) row[n] = sc * acc[i][j][e];
            }
          }
        }
    } else {
      // stage the tile as bf16 in LDS, [token][hidden], then 32 lanes store one 512-byte row segment
      __bf16* st = reinterpret_cast<__bf16*>(smem);
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int m = mrow_base + i * 16 + e;
          const float sc = p.row_scale[m < M ? m : M - 1];
#pragma unroll
          for (int j = 0; j < 8; ++j)
            st[(wm * 128 + i * 16 + 4 * fq + e) * DHSTAGE_LD + wn * 128 + j * 16 + frow] = (__bf16)(sc * acc[i][j][e]);
        }
      __syncthreads();
#pragma unroll 4
      for (int k = 0; k < 32; ++k) {
        const int c = tid + NTHREADS * k;
        const int row = c >> 5, col = c & 31;
        if (m0 + row < M && n0 + col * 8 < p.d) {
          const u32x4 v = *reinterpret_cast<const u32x4*>(smem + row * (DHSTAGE_LD * 2) + col * 16);
          *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.dH) + (int64_t)p.row_index[m0 + row] * p.d + n0 + col * 8) = v;
        }
      }
    }
  } else {
    // rows = vocabulary ids, cols = hidden index; fp32 accumulate into dW.  The old values of
    // one 16-row band are fetched as a batch before any store, so their latencies overlap.
    // A K slice of a tail tile stores its partial tile as it is, [256][256] fp32, to the scratch
    // area instead (dw_tail_reduce adds the slices in their order): the same code with the
    // tile's own origin, row stride and bounds.
    const bool tail = tail_out != nullptr;
    float* const dst = tail ? tail_out : p.dW;
    const int64_t ld = tail ? BN : p.d;
    const int v_org = tail ? m0 : 0, n_org = tail ? n0 : 0;
    const int v_end = tail ? m0 + BM : p.V, n_end = tail ? n0 + BN : p.d;
    const bool overwrite = tail || p.overwrite;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float old[8][4];
      if (!overwrite) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = mrow_base + i * 16 + e;
          const float* row = dst + (int64_t)((v < v_end ? v : v_end - 1) - v_org) * ld - n_org;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int n = ncol_base + j * 16;
            old[j][e] = row[n < n_end ? n : n_end - 1];
          }
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int v = mrow_base + i * 16 + e;
        if (v < v_end) {
          float* row = dst + (int64_t)(v - v_org) * ld - n_org;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int n = ncol_base + j * 16;
            if (n < n_end) row[n] = overwrite ? acc[i][j][e] : old[j][e] + acc[i][j][e];
          }
        }
      }
    }
  }
}

// dW tail.  The workgroup -> tile mapping runs whole super-tile rows of sup_m tile rows; V / 256
// tile rows leave a last, ragged super-tile row (2 tile rows x 16 tiles at V = 151936, d = 4096)
// that keeps an eighth of the compute units busy for the time of a full tile while the others
// idle: 2.3 % of the launch.  Those tiles can be cut into up to 8 slices of the contraction (the
// pass's token rows), work items a fraction of a tile long that fill the compute units the whole
// tiles leave idle at the end.  The slices store their accumulators to a scratch area and
// dw_tail_reduce adds them, slice 0 first, into dW: the result does not depend on execution order.
// Workgroup b runs on XCD b % 8 whatever else is free, so the plan is made per XCD: a model of
// the launch (32 compute units per XCD, whole tiles in id order, then the items) gives the time
// the last item ends for every split and for the unsplit mapping; the best one is taken, and the
// items are dealt to the XCDs as the model placed them.  (Host code that runs once per launch in
// microseconds: not optimised, the optimiser takes very long over its nested constant loops.)
struct DwTailPlan { int m0, rows, split, first[NXCD + 1]; };
__attribute__((optnone, noinline)) DwTailPlan dw_tail_plan(int Mt, int Nt, int sup_m, int sup_n) {
  constexpr int kCus = 32;                       // per XCD
  constexpr double kItemOverhead = 0.02;         // prologue, partial-tile store, reduce: in tile times
  DwTailPlan best = {Mt / sup_m * sup_m, Mt % sup_m, 0, {}};
  const int tiles = best.rows * Nt;
  if (tiles == 0 || best.m0 == 0) return best;
  const int sNt = (Nt + sup_n - 1) / sup_n;
  // tiles per XCD of the first `rows_m` tile rows under the super-tile mapping
  auto tiles_per_xcd = [&](int rows_m, int (&t)[NXCD]) {
    for (int x = 0; x < NXCD; ++x) t[x] = 0;
    const int sMt = (rows_m + sup_m - 1) / sup_m;
    for (int s = 0; s < sMt * sNt; ++s) {
      const int rm = rows_m - (s / sNt) * sup_m, rn = Nt - (s % sNt) * sup_n;
      t[s % NXCD] += (rm < sup_m ? rm : sup_m) * (rn < sup_n ? rn : sup_n);
    }
  };
  int t_all[NXCD], t_main[NXCD];
  tiles_per_xcd(Mt, t_all);
  tiles_per_xcd(best.m0, t_main);
  double unsplit = 0;
  for (int x = 0; x < NXCD; ++x) { const double e = (t_all[x] + kCus - 1) / kCus; unsplit = e > unsplit ? e : unsplit; }
  double best_end = unsplit - kItemOverhead;     // a split has to beat the plain mapping by a margin
  for (int split = 2; split <= 8 && tiles * split <= kDwTailMaxItems; ++split) {
    // free[x][c]: when compute unit c of XCD x has finished its whole tiles
    double free_at[NXCD][kCus];
    for (int x = 0; x < NXCD; ++x)
      for (int c = 0; c < kCus; ++c) free_at[x][c] = t_main[x] / kCus + (c < t_main[x] % kCus ? 1 : 0);
    int count[NXCD] = {};
    double end = 0;
    for (int x = 0; x < NXCD; ++x) for (int c = 0; c < kCus; ++c) end = free_at[x][c] > end ? free_at[x][c] : end;
    for (int i = 0; i < tiles * split; ++i) {
      int bx = 0, bc = 0;
      for (int x = 0; x < NXCD; ++x)
        for (int c = 0; c < kCus; ++c)
          if (free_at[x][c] < free_at[bx][bc]) { bx = x; bc = c; }
      free_at[bx][bc] += 1.0 / split + kItemOverhead;
      end = free_at[bx][bc] > end ? free_at[bx][bc] : end;
      count[bx]++;
    }
    if (end < best_end - 1e-9) {
      best_end = end; best.split = split; best.first[0] = 0;
      for (int x = 0; x < NXCD; ++x) best.first[x + 1] = best.first[x] + count[x];
    }
  }
  return best;
}

__global__ __launch_bounds__(256) void dw_tail_reduce(const float* __restrict__ part, int tiles, int split, int Nt,
                                                      int tail_m0, int V, int d, float* __restrict__ dW,
                                                      int overwrite, const int64_t* __restrict__ n_scored,
                                                      int64_t chunk_start) {
  if (!overwrite && *n_scored - chunk_start <= 0) return;   // the GEMM launch left dW (and part) alone
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int t = (int)(q / (BM * BN)), within = (int)(q % (BM * BN));
  if (t >= tiles) return;
  const int v = (tail_m0 + t / Nt) * BM + within / BN, n = (t % Nt) * BN + within % BN;
  if (v >= V || n >= d) return;
  float s = 0.f;
  for (int k = 0; k < split; ++k) s += part[((int64_t)k * tiles + t) * (BM * BN) + within];
  float* out = dW + (int64_t)v * d + n;
  *out = overwrite ? s : *out + s;
}

template <int MODE>
void launch(Params& p, hipStream_t stream) {
  static LdsLimit lds_limit;
  lds_limit.ensure(reinterpret_cast<const void*>(&gemm_nt_bf16<MODE>), lds_bytes<MODE>());
  const int Mt = (p.M + BM - 1) / BM, Nt = (p.N + BN - 1) / BN;
  const SuperTile st = pick_super_tile(Nt);
  p.sup_m = st.m; p.sup_n = st.n;
  int blocks = num_blocks(Mt, Nt, st.m, st.n);
  DwTailPlan tail = {0, 0, 0, {}};
  if (MODE == MODE_DW && p.tail_part != nullptr) tail = dw_tail_plan(Mt, Nt, st.m, st.n);
  if (tail.split > 0) {
    p.main_blocks = num_blocks(tail.m0, Nt, st.m, st.n);
    p.tail_m0 = tail.m0; p.tail_rows = tail.rows; p.tail_split = tail.split;
    int most = 0;
    for (int x = 0; x < NXCD; ++x) {
      p.tail_first[x] = tail.first[x];
      most = tail.first[x + 1] - tail.first[x] > most ? tail.first[x + 1] - tail.first[x] : most;
    }
    p.tail_first[NXCD] = tail.first[NXCD];
    blocks = p.main_blocks + most * NXCD;
  }
  hipLaunchKernelGGL(gemm_nt_bf16<MODE>, dim3(blocks), dim3(NTHREADS), lds_bytes<MODE>(), stream, p);
  if (tail.split > 0) {
    const int tiles = tail.rows * Nt;
    hipLaunchKernelGGL(dw_tail_reduce, dim3(tiles * (BM * BN / 256)), dim3(256), 0, stream, p.tail_part, tiles,
                       tail.split, Nt, tail.m0, p.V, p.d, p.dW, p.overwrite, p.n_scored, p.chunk_start);
  }
}

}  // namespace

void launch_gemm_fwd_bf16(const void* W, int64_t ldw, const void* Hc, int64_t ldh, int k_len, const float* zt,
                          const int64_t* n_scored, int64_t chunk_start, int chunk_rows,
                          int V, int d, float* part_sum, float* part_ez,
                          int64_t part_stride, void* estash, int64_t lde, hipStream_t stream) {
  Params p = {};
  p.A = static_cast<const uint16_t*>(W); p.lda = ldw; p.M = V;
  p.B = static_cast<const uint16_t*>(Hc); p.ldb = ldh; p.N = chunk_rows;
  p.K = k_len;
  p.n_scored = n_scored; p.chunk_start = chunk_start; p.chunk_rows = chunk_rows;
  p.zt = zt + chunk_start;
  p.part_sum = part_sum; p.part_ez = part_ez; p.part_stride = part_stride;
  p.estash = static_cast<uint16_t*>(estash); p.lde = lde; p.V = V; p.d = d;
  launch<MODE_FWD>(p, stream);
}

void launch_gemm_dh_bf16(const void* E, int64_t lde, const void* Wt, int64_t ldwt,
                         const int32_t* row_index, const float* row_scale, const int64_t* n_scored,
                         int64_t chunk_start, int chunk_rows, int Vp, int d, void* dH, int dh_f32,
                         hipStream_t stream) {
  Params p = {};
  p.A = static_cast<const uint16_t*>(E); p.lda = lde; p.M = chunk_rows;
  p.row_scale = row_scale + chunk_start;
  p.B = static_cast<const uint16_t*>(Wt); p.ldb = ldwt; p.N = d;
  p.K = Vp;
  p.row_index = row_index + chunk_start;
  p.n_scored = n_scored; p.chunk_start = chunk_start; p.chunk_rows = chunk_rows;
  p.dH = dH; p.dh_f32 = dh_f32; p.d = d; p.V = Vp;
  launch<MODE_DH>(p, stream);
}

size_t gemm_dw_tail_bytes() { return (size_t)kDwTailMaxItems * BM * BN * sizeof(float); }

void launch_gemm_dw_bf16(const void* E, int64_t lde, const void* Ht, int64_t ldht,
                         const int64_t* n_scored, int64_t chunk_start, int chunk_rows,
                         int V, int d, float* dW, int overwrite, float* tail_part, hipStream_t stream) {
  Params p = {};
  p.A = static_cast<const uint16_t*>(E); p.lda = lde; p.M = (int)round_up(V, kTile);
  p.B = static_cast<const uint16_t*>(Ht); p.ldb = ldht; p.N = d;
  p.K = chunk_rows;
  p.n_scored = n_scored; p.chunk_start = chunk_start; p.chunk_rows = chunk_rows;
  p.dW = dW; p.overwrite = overwrite; p.V = V; p.d = d;
  p.tail_part = tail_part;
  launch<MODE_DW>(p, stream);
}

}  // namespace mrl

extern "C" int mrl_diag_dw_tail_plan(int32_t V, int32_t d, int32_t* out12) {
  using namespace mrl;
  if (out12 == nullptr) return MRL_ERR_NULL;
  if (V <= 0 || d <= 0) return MRL_ERR_SHAPE;
  const int Mt = (int)(round_up(V, kTile) / BM), Nt = (d + BN - 1) / BN;
  const SuperTile st = pick_super_tile(Nt);
  const DwTailPlan t = dw_tail_plan(Mt, Nt, st.m, st.n);
  out12[0] = t.m0; out12[1] = t.rows; out12[2] = t.split;
  for (int x = 0; x <= NXCD; ++x) out12[3 + x] = t.split > 0 ? t.first[x] : 0;
  return MRL_OK;
}
