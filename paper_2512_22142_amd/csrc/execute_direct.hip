// bf16 sub-GEMM executor, fast path: operand tiles go from global memory
// straight into LDS (no register staging), through a ring of stages.
//
// Same contract as the staged executor (paper Sec. 4.1: a task multiplies its
// rows of A with its columns of B over its chunk of the inner dimension and
// stores an fp32 partial block); used when every chunk length is a multiple of
// the K step and all tile edges / leading dimensions are multiples of 8.
//
// The kernel is a template over its shape (workgroup tile, wave grid, K step,
// ring depth); a wave always owns 32 x 32 MFMA 32x32x16 blocks with fp32
// accumulators in registers.  The two instantiations are at the end of the
// file.
//
// A wave-wide direct load writes 64 consecutive 16-byte LDS slots (lane l ->
// slot l), so the LDS layout is chosen through which global 16 bytes a lane
// fetches:
//   * K-contiguous operand (tile row r, CPR chunks of 8 k per step):
//       slot = r*CPR + (chunk ^ swizzle(r)),  swizzle = (r>>1)&7 for CPR = 8,
//       (r>>2)&3 for CPR = 4;
//     16 consecutive rows at one chunk then cover 16 distinct bank groups, so
//     the 16-byte fragment reads are conflict free.
//   * operand stored with the tile-row index contiguous (read "transposed"):
//     the tile is kept as BK k rows of R/8 chunks,
//       slot = k*(R/8) + (chunk ^ (4*(k & 3)));
//     fragments are gathered with the LDS transpose read (ds_read_b64_tr_b16:
//     within 16 lanes, lane i supplies the address of 4 consecutive elements of
//     k row i/4 and receives column i of the 4 x 16 block), two reads per
//     fragment; the XOR spreads the four k rows of a read over the banks.
//
// Stores: a full sub-tile leaves through a 4 KB row-major image per wave in
// LDS behind the ring, so that every store instruction writes whole 128-byte
// lines (a quarter of the store instructions of the accumulator layout, none
// of them held up by the limit of 63 outstanding operations); outputs that
// are only element-aligned and clipped sub-tiles take 4-byte stores.
//
// Order of accumulation per output element: ascending K steps, inside a step
// ascending 16-element sub-steps, one MFMA each -- a function of the task
// record only (and the same for every shape), hence bitwise reproducible on
// re-issue.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "kernels.h"
#include "tile_store.h"
#include "plan_internal.h"

namespace cleave {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4;

// Shape of the kernel: workgroup tile TM x TN computed by WM x WN waves, BK
// elements of K per step, STAGES ring stages, WGS workgroups per CU.
template <int TM_, int TN_, int WM_, int WN_, int BK_, int STAGES_, int WGS_>
struct Shape {
  static constexpr int TM = TM_, TN = TN_, WM = WM_, WN = WN_, BK = BK_, STAGES = STAGES_, WGS = WGS_;
  static constexpr int NW = WM * WN;            // waves
  static constexpr int NT = NW * 64;            // threads
  static constexpr int WTM = TM / WM, WTN = TN / WN;   // wave tile
  static constexpr int MB = WTM / 32, NB = WTN / 32;   // 32 x 32 MFMA blocks per wave tile
  static constexpr int CPR = BK / 8;            // 16-byte chunks per K-contiguous row and step
  static constexpr int kSub = BK / 16;          // MFMA sub-steps per step
  static constexpr int kATile = TM * BK * 2;    // bytes
  static constexpr int kBTile = TN * BK * 2;
  static constexpr int kStage = kATile + kBTile;
  static constexpr int kLoadsA = kATile / 1024 / NW;   // wave-wide loads per wave and step
  static constexpr int kLoadsB = kBTile / 1024 / NW;
  static constexpr int kLoadsPerStep = kLoadsA + kLoadsB;
  static_assert(kATile % (1024 * NW) == 0 && kBTile % (1024 * NW) == 0, "tile / wave count");
  static_assert(kSub % 2 == 0 && (CPR == 4 || CPR == 8), "BK must be 32 or 64");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0 && STAGES >= 2, "shape");
};

// Waits until at most `n` vector-memory operations of this wave are still in
// flight (loads return in order, so the n youngest) and all of its LDS reads
// have returned, then joins the workgroup barrier.  The wait and the barrier
// sit in one asm statement with a memory clobber: the compiler can neither
// move LDS accesses or direct loads across it nor separate the two, and
// (unlike __syncthreads) it adds no wait for the younger loads.
#define CLEAVE_WAIT_BARRIER(n) \
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(n) : "memory")

template <int V>
using int_c = std::integral_constant<int, V>;

// XOR applied to the chunk index of a K-contiguous row so that 16 consecutive
// rows at one logical chunk fall into 16 different 16-byte bank groups.
template <int CPR>
__device__ __forceinline__ int row_swizzle(int r) {
  return CPR == 4 ? ((r >> 2) & 3) : ((r >> 1) & 7);
}

template <typename S, bool KCONTIG, int R>
struct DirectTile {
  static constexpr int kLoads = R * S::BK * 2 / 1024 / S::NW;
  static constexpr int CH = R / 8;     // chunks per k row (transposed layout)
  uint32_t goff[kLoads];

  __device__ __forceinline__ void init(int64_t row_stride, int64_t k_stride, int r_valid, int wave,
                                       int lane) {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const int slot = (wave + S::NW * i) * 64 + lane;
      if constexpr (KCONTIG) {
        const int r = slot / S::CPR;
        const int c = (slot % S::CPR) ^ row_swizzle<S::CPR>(r);
        goff[i] = static_cast<uint32_t>((min(r, r_valid - 1) * row_stride + c * 8) * 2);
      } else {
        const int k = slot / CH;
        const int c = (slot % CH) ^ (4 * (k & 3));
        goff[i] = static_cast<uint32_t>((k * k_stride + min(c * 8, r_valid - 8)) * 2);
      }
    }
  }

  // gbase: the tile's first row at this step's first k (wave-uniform);
  // lds_tile: LDS byte address of the tile.  The load is issued through inline
  // asm (scalar base + per-lane 32-bit offset, LDS base in M0) for two
  // reasons: no VALU address arithmetic in the K loop, and the compiler does
  // not see an LDS-writing vector-memory operation -- it would otherwise wait
  // for every load in flight before each LDS transpose read.  The statement
  // has no register outputs, so nothing the compiler may spill or reuse is
  // written asynchronously; completion is awaited with CLEAVE_WAIT_BARRIER.
  // M0 is on the clobber list so that the compiler keeps no value of its own
  // in M0 across the statement (it is a reserved register, hence the
  // diagnostic silenced here; nothing needs it preserved).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
  __device__ __forceinline__ void issue(const unsigned char* gbase, uint32_t lds_tile,
                                        int wave) const {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const uint32_t lds = lds_tile + (wave + S::NW * i) * 1024;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(lds), "v"(goff[i]), "s"(gbase)
                   : "memory", "m0");
    }
  }
#pragma clang diagnostic pop
};

template <typename S, bool A_K, bool B_K>
__global__ __launch_bounds__(S::NT, S::WGS) void execute_direct_kernel(ExecuteArgs args) {
  constexpr int TM = S::TM, TN = S::TN, MB = S::MB, NB = S::NB, CPR = S::CPR, kSub = S::kSub;
  constexpr int kStage = S::kStage, kATile = S::kATile, STAGES = S::STAGES, LPS = S::kLoadsPerStep;
  constexpr int kRowBytes = CPR * 16;        // K-contiguous tile row
  constexpr int CHA = TM / 8, CHB = TN / 8;  // chunks per k row, transposed tiles

  extern __shared__ __align__(16) unsigned char smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / S::WN;
  const int wn = wave % S::WN;
  const int l32 = lane & 31;
  const int lh = lane >> 5;

  // Lane-constant fragment addresses (byte offsets inside a stage).
  // K-contiguous: one per sub-step; blocks are 32 rows apart.  Transposed: one
  // per block (the XOR touches the block bits); sub-step and half select the k
  // rows through a constant offset.
  const uint32_t smem_off = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void)smem));
  const int i16 = lane & 15;
  const int kq = i16 >> 2;            // k row (mod 4) this lane addresses in a transpose read
  const int cq = i16 & 3;             // which 4 of the 16 columns
  const int nsub = (lane >> 4) & 1;   // which 16-column half of the 32-wide block
  uint32_t a_addr[A_K ? kSub : MB];
  uint32_t b_addr[B_K ? kSub : NB];
  if constexpr (A_K) {
    const int sw = row_swizzle<CPR>(l32);
#pragma unroll
    for (int ks = 0; ks < kSub; ++ks)
      a_addr[ks] = (wm * S::WTM + l32) * kRowBytes + (((2 * ks + lh) ^ sw) * 16);
  } else {
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int c = wm * (S::WTM / 8) + i * 4 + 2 * nsub + (cq >> 1);
      a_addr[i] = ((8 * lh + kq) * CHA + (c ^ (4 * kq))) * 16 + (cq & 1) * 8;
    }
  }
  if constexpr (B_K) {
    const int sw = row_swizzle<CPR>(l32);
#pragma unroll
    for (int ks = 0; ks < kSub; ++ks)
      b_addr[ks] = kATile + (wn * S::WTN + l32) * kRowBytes + (((2 * ks + lh) ^ sw) * 16);
  } else {
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int c = wn * (S::WTN / 8) + j * 4 + 2 * nsub + (cq >> 1);
      b_addr[j] = kATile + ((8 * lh + kq) * CHB + (c ^ (4 * kq))) * 16 + (cq & 1) * 8;
    }
  }

  // Element strides of the stored operands along (tile row, K).
  const int64_t a_rs = args.transA ? 1 : args.lda;
  const int64_t a_ks = args.transA ? args.lda : 1;
  const int64_t b_rs = args.transB ? args.ldb : 1;
  const int64_t b_ks = args.transB ? 1 : args.ldb;

  // Everything a work item needs, wave-uniform (scalar registers).
  struct ItemCtx {
    const unsigned char* a_ptr;   // first row of the A tile at the chunk's first k
    const unsigned char* b_ptr;
    TileTarget out;               // where this sub-tile's accumulators go
    int steps, m_valid, n_valid;
  };
  // A work item record into scalar registers.  The table is never written by
  // this kernel: read through the constant address space, a wave-uniform
  // address becomes scalar loads whose completion the compiler tracks, even
  // though the kernel also stores to global memory.
  auto load_item = [&](int64_t idx) -> WorkItem {
    typedef const __attribute__((address_space(4))) u32x4* const_words;
    const_words src = (const_words)(args.items + idx);
    uint32_t words[12];
#pragma unroll
    for (int v = 0; v < 3; ++v) {
      const u32x4 q = src[v];
#pragma unroll
      for (int e = 0; e < 4; ++e) words[4 * v + e] = q[e];
    }
    WorkItem w;
    __builtin_memcpy(&w, words, sizeof(w));
    return w;
  };
  auto make_ctx = [&](const WorkItem& w) -> ItemCtx {
    ItemCtx c;
    c.m_valid = static_cast<int>(w.m_valid);
    c.n_valid = static_cast<int>(w.n_valid);
    c.steps = static_cast<int>(w.k_len) / S::BK;
    c.a_ptr = static_cast<const unsigned char*>(args.A) +
              (member_offset(args.a_at, args.batch, w.gemm_id) +
               static_cast<int64_t>(w.m_base) * a_rs + static_cast<int64_t>(w.k0) * a_ks) * 2;
    c.b_ptr = static_cast<const unsigned char*>(args.B) +
              (member_offset(args.b_at, args.batch, w.gemm_id) +
               static_cast<int64_t>(w.n_base) * b_rs + static_cast<int64_t>(w.k0) * b_ks) * 2;
    c.out = tile_target(args, w);
    return c;
  };
  const int64_t a_step = a_ks * S::BK * 2;    // bytes per K step
  const int64_t b_step = b_ks * S::BK * 2;

  DirectTile<S, A_K, TM> ta;
  DirectTile<S, B_K, TN> tb;
  auto issue = [&](const ItemCtx& c, int s, int st) {
    const uint32_t stage = smem_off + st * kStage;
    ta.issue(c.a_ptr + s * a_step, stage, wave);
    tb.issue(c.b_ptr + s * b_step, stage + kATile, wave);
  };
  // Start of a work item: lane offsets for its (possibly clipped) tile, then
  // the first STAGES steps into the ring.
  auto fill_ring = [&](const ItemCtx& c) {
    ta.init(a_rs, a_ks, c.m_valid, wave, lane);
    tb.init(b_rs, b_ks, c.n_valid, wave, lane);
#pragma unroll
    for (int st = 0; st < STAGES; ++st)
      if (st < c.steps) issue(c, st, st);
  };

  // A workgroup walks its work items -- every grid-th one, or a run of its own
  // when the launch comes with a balanced schedule.  The ring runs on across
  // items: when the current item and the next one are both full sub-tiles, the
  // next item's first two K steps are fetched into the ring stages that this
  // item's last two steps free, exactly as this item's own later steps would
  // be, so the next K loop starts without a ring fill and without waiting for
  // this item's stores.  Otherwise (clipped sub-tiles need other lane offsets,
  // one-step items free no stage early) the ring is filled from empty after the
  // item's last step, ahead of its stores.
  static_assert(STAGES == 2, "the hand-over between items is written for a ring of two stages");
  // Store instructions per lane: a full sub-tile whose target takes 16-byte
  // stores goes through the wave's block image in LDS (behind the ring).
  constexpr int kTileStores = MB * staged_stores_per_block_row<NB>();
  constexpr int kHalfStores = kTileStores / 2;
  // "at most n operations outstanding" for n stores issued last: the counter holds 63 at most
  constexpr int kBehindCheck = kHalfStores < 63 ? kHalfStores : 63;
  constexpr int kBehindTile = kTileStores < 63 ? kTileStores : 63;
  static_assert(MB % 2 == 0, "the epilogue stores a sub-tile in two halves of block rows");
  unsigned char* const image = smem + STAGES * kStage + wave * kBlockImageBytes;

  // This workgroup's items: first, first + stride, ... below it_end.
  int64_t it_first = blockIdx.x, it_end = args.n_items, stride = gridDim.x;
  if (args.wg_ranges) {
    it_first = args.wg_ranges[blockIdx.x];
    it_end = args.wg_ranges[blockIdx.x + 1];
    stride = 1;
  }
  if (it_first >= it_end) return;
  ItemCtx c = make_ctx(load_item(it_first));
  fill_ring(c);
  int64_t it_next = it_first + stride;
  // Item records are read two items ahead (scalar loads through the constant
  // address space): the read for the item after next is issued right behind
  // the current item's first barrier, a whole K step before the next wait
  // that covers it.  `last_item` stands in for records past the end.
  const int64_t last_item = it_end - 1;
  ItemCtx nx = make_ctx(load_item(it_next < it_end ? it_next : last_item));
  WorkItem after_next;
  // How the current item's first two steps got into the ring.
  //   kFilled:             ring filled from empty, nothing issued since.
  //   kFilledBehindStores: ring filled from empty, then exactly kTileStores
  //     stores of the previous item: the counter retires in issue order, so the
  //     loads have landed once at most that many operations are outstanding
  //     (or 63, all the counter can hold, if the stores are more than that).
  //   kPrefetched:         fetched during the previous item's last two steps;
  //     step 0 was waited for at that item's last barrier (its first fragments
  //     are already in registers), step 1 between the two halves of its stores.
  enum Entry : int { kFilled = 0, kFilledBehindStores = 1, kPrefetched = 2 };
  int entry = kFilled;
  int phase = 0;   // ring stage that holds the current item's step 0

  f32x16 acc[MB][NB];
  u32x4 fa[2][MB], fb[2][NB];

  // Fragment reads are ordinary (compiler-visible) LDS loads: the compiler
  // tracks their completion, and every address is a lane-constant register
  // plus a compile-time offset (stage, block, sub-step).
  auto tr_read = [&](const unsigned char* p) -> u32x2 {
    return __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)p));
  };
  // Fragments of sub-step KS of the ring stage at byte offset `stage` into
  // register set `buf`.
  auto read_frags = [&](uint32_t stage, auto ks_tag, int buf) {
    constexpr int KS = decltype(ks_tag)::value;
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      if constexpr (A_K) {
        fa[buf][i] = *reinterpret_cast<const u32x4*>(smem + (a_addr[KS] + stage) + i * 32 * kRowBytes);
      } else {
        const unsigned char* p = smem + (a_addr[i] + stage) + KS * (16 * CHA * 16);
        const u32x2 lo = tr_read(p);
        const u32x2 hi = tr_read(p + 4 * CHA * 16);
        fa[buf][i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
      }
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      if constexpr (B_K) {
        fb[buf][j] = *reinterpret_cast<const u32x4*>(smem + (b_addr[KS] + stage) + j * 32 * kRowBytes);
      } else {
        const unsigned char* p = smem + (b_addr[j] + stage) + KS * (16 * CHB * 16);
        const u32x2 lo = tr_read(p);
        const u32x2 hi = tr_read(p + 4 * CHB * 16);
        fb[buf][j] = u32x4{lo[0], lo[1], hi[0], hi[1]};
      }
    }
  };
  // `fresh`: the first product of a work item starts from zero (a constant
  // operand of the instruction: no pass over the accumulators to clear them).
  auto mma = [&](int buf, auto fresh_tag) {
    constexpr bool FRESH = decltype(fresh_tag)::value;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        f32x16 sum = acc[i][j];
        if constexpr (FRESH) sum = f32x16{};
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, fa[buf][i]), __builtin_bit_cast(bf16x8, fb[buf][j]), sum, 0, 0, 0);
      }
  };

  // Instruction order of one sub-step, as a hint to the scheduler: the MFMAs
  // of the current fragments with the LDS reads of the next fragments spread
  // one (or two, for transpose reads) behind each of them, the last two
  // MFMAs without reads.  Measured +2 % over the compiler's own order.
  auto interleave = [&]() {
    constexpr int kReads = (A_K ? MB : 2 * MB) + (B_K ? NB : 2 * NB);
    constexpr int kMfma = MB * NB;
    constexpr int kTail = kMfma > 2 ? 2 : kMfma - 1;             // MFMAs without reads behind them
    constexpr int kPer = (kReads + (kMfma - kTail) - 1) / (kMfma - kTail);
#pragma unroll
    for (int i = 0; i < kMfma; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);         // one MFMA
      if (i < kMfma - kTail) __builtin_amdgcn_sched_group_barrier(0x100, kPer, 0);   // LDS reads
    }
  };

  for (;;) {
    const int steps = c.steps;
    const bool has_next = it_next < it_end;
    const bool interior = c.m_valid == TM && c.n_valid == TN;
    const bool wide = interior && args.out_vec;   // stores of whole lines through the block image
    // hand the ring over without draining it
    const bool cont = has_next && wide && nx.m_valid == TM && nx.n_valid == TN && steps >= 2;

    // Step 0 must have landed.  All earlier fragment reads of this workgroup
    // completed before the previous item's final barrier.
    if (entry != kPrefetched) {
      if (entry == kFilledBehindStores) {
        CLEAVE_WAIT_BARRIER(kBehindTile);
      } else if (steps >= STAGES) {
        CLEAVE_WAIT_BARRIER(LPS);
      } else {
        CLEAVE_WAIT_BARRIER(0);
      }
      read_frags(0u, int_c<0>{}, 0);   // a ring filled from empty starts at stage 0
    }

    // One K step; step s sits in ring stage (s + phase) % 2.  Sub-step j
    // multiplies register set j & 1 while the fragments of sub-step j+1 are
    // fetched into the other set.  The barrier sits before the last sub-step's
    // MFMAs: by then this wave holds all fragments of step s and the step
    // after it has landed (loads return in order), so the stage is refilled
    // with the step after next -- this item's, or the next item's first or
    // second -- and the first fragments of the following step are fetched
    // while the last sub-step multiplies.  MID: a step with at least two more
    // steps of this item behind it and not the item's first -- no case
    // distinctions, the loop body of long chunks.
    auto k_step = [&](auto mid_tag, auto first_tag, int s) {
      constexpr bool MID = decltype(mid_tag)::value;
      constexpr bool FIRST = decltype(first_tag)::value;   // the item's step 0
      const int st = (s + phase) & 1;
      const uint32_t cur = st ? kStage : 0;
      const uint32_t oth = st ? 0 : kStage;
      auto sub = [&](auto j_tag) {
        constexpr int J = decltype(j_tag)::value;
        read_frags(cur, int_c<J + 1>{}, (J + 1) & 1);
        mma(J & 1, std::bool_constant<FIRST && J == 0>{});
        interleave();
      };
      sub(int_c<0>{});
      if constexpr (kSub == 4) {
        sub(int_c<1>{});
        sub(int_c<2>{});
      }
      if constexpr (MID) {
        CLEAVE_WAIT_BARRIER(0);
        issue(c, s + STAGES, st);
        read_frags(oth, int_c<0>{}, 0);
      } else {
        const bool last = s + 1 >= steps;
        if (last && !cont) {
          // no step follows in the ring: nothing to wait for, and no reason to
          // wait for the previous item's stores either
          CLEAVE_WAIT_BARRIER(63);
        } else if (s == 0 && entry == kFilledBehindStores) {
          CLEAVE_WAIT_BARRIER(kBehindTile);
        } else if (s == 0 && entry == kPrefetched) {
          // step 1 was waited for before the second half of the previous item's stores
          CLEAVE_WAIT_BARRIER(kBehindCheck);
        } else {
          CLEAVE_WAIT_BARRIER(0);
        }
        if (s + STAGES < steps) {
          issue(c, s + STAGES, st);
        } else if (cont && s + STAGES - steps < nx.steps) {
          issue(nx, s + STAGES - steps, st);
        }
        if (s == 0) after_next = load_item(it_next + stride < it_end ? it_next + stride : last_item);
        if (!last || cont) read_frags(oth, int_c<0>{}, 0);
      }
      mma((kSub - 1) & 1, std::false_type{});
      interleave();
    };
    k_step(std::false_type{}, std::true_type{}, 0);
    int s = 1;
    for (; s + STAGES < steps; ++s) k_step(std::true_type{}, std::false_type{}, s);
    for (; s < steps; ++s) k_step(std::false_type{}, std::false_type{}, s);

    // Every wave is past the last step's barrier, hence past all of its
    // fragment reads of this item.
    const int row0 = wm * S::WTM + lh * 4;
    const int col0 = wn * S::WTN + l32;
    const TileTarget target = c.out;
    const int m_valid = c.m_valid, n_valid = c.n_valid;
    const bool bf16_out = args.C && args.c_bf16;
    if (cont) {
      // The next item's step 1 went out at the last barrier; wait for it
      // between the two halves of the stores: the first half keeps the memory
      // pipeline busy meanwhile, and the second half then trails the check, so
      // that the next item's first barrier finds at most kBehindCheck
      // operations outstanding without any store having to complete.  The
      // block image is this wave's own: no barrier between the halves.
      store_tile_rows_staged<MB, NB, 0, MB / 2>(acc, target, bf16_out, image, wm * S::WTM, wn * S::WTN, lane);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kBehindCheck) : "memory");
      store_tile_rows_staged<MB, NB, MB / 2, MB>(acc, target, bf16_out, image, wm * S::WTM, wn * S::WTN, lane);
      entry = kPrefetched;
      phase = (phase + steps) & 1;
    } else {
      // The ring is free: the next item's ring fill is issued before this
      // item's stores so that its latency hides behind them.
      if (has_next) fill_ring(nx);
      if (wide) {
        store_tile_rows_staged<MB, NB, 0, MB>(acc, target, bf16_out, image, wm * S::WTM, wn * S::WTN, lane);
      } else {
        store_tile<MB, NB>(acc, target, bf16_out, row0, col0, m_valid, n_valid, interior);
      }
      entry = wide ? kFilledBehindStores : kFilled;
      phase = 0;
    }
    if (!has_next) break;
    c = nx;
    nx = make_ctx(after_next);
    it_next += stride;
  }
}

template <typename S, bool A_K, bool B_K>
hipError_t launch_one(const ExecuteArgs& args, int grid, hipStream_t stream) {
  constexpr size_t lds = S::STAGES * S::kStage + S::NW * kBlockImageBytes;
  hipLaunchKernelGGL((execute_direct_kernel<S, A_K, B_K>), dim3(grid), dim3(S::NT), lds, stream, args);
  return hipGetLastError();
}

template <typename S, bool A_K, bool B_K>
hipError_t configure_one() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(execute_direct_kernel<S, A_K, B_K>),
                             hipFuncAttributeMaxDynamicSharedMemorySize,
                             static_cast<int>(S::STAGES * S::kStage + S::NW * kBlockImageBytes));
}

template <typename S>
hipError_t configure_layouts() {
  hipError_t e = configure_one<S, true, true>();
  if (e == hipSuccess) e = configure_one<S, true, false>();
  if (e == hipSuccess) e = configure_one<S, false, true>();
  if (e == hipSuccess) e = configure_one<S, false, false>();
  return e;
}

// Large class: 256 x 256 tile, 8 waves (2 x 4, each 128 x 64), 64 elements of
// K per step, two 64 KB stages, one workgroup per CU.  Small class: 128 x 128
// tile, 4 waves (each 64 x 64), same K step, two 32 KB stages, two workgroups
// per CU.  Both fetch full 128-byte lines of K-contiguous operands.
#ifndef CLEAVE_DIRECT_SHAPE_LARGE
#define CLEAVE_DIRECT_SHAPE_LARGE Shape<kLargeTileRows, kLargeTileCols, 2, 4, 64, 2, 1>
#endif
using LargeShape = CLEAVE_DIRECT_SHAPE_LARGE;
#ifndef CLEAVE_DIRECT_SHAPE_SMALL
#define CLEAVE_DIRECT_SHAPE_SMALL Shape<kSmallTileRows, kSmallTileCols, 2, 2, 64, 2, 2>
#endif
using SmallShape = CLEAVE_DIRECT_SHAPE_SMALL;
static_assert(LargeShape::TM == kLargeTileRows && LargeShape::TN == kLargeTileCols,
              "the kernel's tile must be the host's sub-tile of the large class");
static_assert(kDirectKStep % LargeShape::BK == 0 && kDirectKStep % SmallShape::BK == 0,
              "the host hands this kernel the work items whose chunk is a multiple of kDirectKStep");

template <typename S>
hipError_t launch_layouts(const ExecuteArgs& args, int grid, hipStream_t stream) {
  const bool a_k = !args.transA;   // A stored M x K: K-contiguous
  const bool b_k = args.transB;    // B stored N x K: K-contiguous
  if (a_k && b_k) return launch_one<S, true, true>(args, grid, stream);
  if (a_k && !b_k) return launch_one<S, true, false>(args, grid, stream);
  if (!a_k && b_k) return launch_one<S, false, true>(args, grid, stream);
  return launch_one<S, false, false>(args, grid, stream);
}

}  // namespace


hipError_t configure_execute_direct_kernels() {
  const hipError_t e = configure_layouts<LargeShape>();
  return e != hipSuccess ? e : configure_layouts<SmallShape>();
}

int direct_workgroups_per_cu(int tile_class) {
  return tile_class == kTileLarge ? LargeShape::WGS : SmallShape::WGS;
}

hipError_t launch_execute_direct(const ExecuteArgs& args, int tile_class, int grid,
                                 hipStream_t stream) {
  return tile_class == kTileLarge ? launch_layouts<LargeShape>(args, grid, stream)
                                  : launch_layouts<SmallShape>(args, grid, stream);
}

}  // namespace cleave
