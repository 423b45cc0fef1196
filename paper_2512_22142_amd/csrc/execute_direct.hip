// bf16 sub-GEMM executor, fast path: operand tiles go from global memory
// straight into LDS (no register staging), through a three-stage ring.
//
// Same contract as the staged executor (paper Sec. 4.1: a task multiplies its
// rows of A with its columns of B over its chunk of the inner dimension and
// stores an fp32 partial block); used when every chunk length is a multiple of
// 32 elements and all tile edges / leading dimensions are multiples of 8.
//
// Workgroup: 4 wave64 (2 x 2), tile 256 x 128, a wave owns 128 x 64 (4 x 2
// MFMA 32x32x16 blocks, 128 accumulator registers); two workgroups share a CU
// so that one's barriers and partial-block stores overlap the other's MFMAs.
//
// K step: 32 elements (64 bytes per K-contiguous row).  A stage holds the A
// tile (16 KB) and the B tile (8 KB); the ring has three stages (72 KB).  A
// wave-wide direct load writes 64 consecutive 16-byte LDS slots (lane l ->
// slot l), so the LDS layout is chosen through which global 16 bytes a lane
// fetches:
//   * K-contiguous operand (row r = tile row, 4 chunks of 8 k per step):
//       slot = r*4 + (chunk ^ ((r >> 2) & 3));
//     16 consecutive rows at one chunk then cover 16 distinct bank groups, so
//     the 16-byte fragment reads are conflict free.
//   * operand stored with the tile-row index contiguous (read "transposed"):
//     the tile is kept as 32 k rows of R/8 chunks,
//       slot = k*(R/8) + (chunk ^ (4*(k & 3)));
//     fragments are gathered with the LDS transpose read (ds_read_b64_tr_b16:
//     within 16 lanes, lane i supplies the address of 4 consecutive elements of
//     k row i/4 and receives column i of the 4 x 16 block), two reads per
//     fragment; the XOR spreads the four k rows of a read over the banks.
//
// Order of accumulation per output element: ascending K steps, inside a step
// ascending 16-element sub-steps, one MFMA each -- a function of the task
// record only, hence bitwise reproducible on re-issue.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "kernels.h"
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
typedef __attribute__((address_space(1))) const void* glb_void;

constexpr int kNT = 256;                 // threads
constexpr int kTM = 256, kTN = 128;      // workgroup tile
constexpr int kWTM = 128, kWTN = 64;     // wave tile
constexpr int kMB = 4, kNB = 2;          // 32 x 32 blocks per wave tile
constexpr int kBK = 32;                  // elements of K per step
constexpr int kATile = kTM * kBK * 2;    // bytes
constexpr int kBTile = kTN * kBK * 2;
constexpr int kStage = kATile + kBTile;
constexpr int kStages = 3;
constexpr int kLoadsA = kATile / 1024 / 4;   // wave-wide loads per wave and step
constexpr int kLoadsB = kBTile / 1024 / 4;
constexpr int kLoadsPerStep = kLoadsA + kLoadsB;

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

template <bool KCONTIG, int R>
struct DirectTile {
  static constexpr int kLoads = R * kBK * 2 / 1024 / 4;
  static constexpr int CH = R / 8;     // chunks per k row (transposed layout)
  uint32_t goff[kLoads];

  __device__ __forceinline__ void init(int64_t row_stride, int64_t k_stride, int r_valid, int wave,
                                       int lane) {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const int slot = (wave + 4 * i) * 64 + lane;
      if constexpr (KCONTIG) {
        const int r = slot >> 2;
        const int c = (slot & 3) ^ ((r >> 2) & 3);
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
  __device__ __forceinline__ void issue(const unsigned char* gbase, uint32_t lds_tile,
                                        int wave) const {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const uint32_t lds = lds_tile + (wave + 4 * i) * 1024;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(lds), "v"(goff[i]), "s"(gbase)
                   : "memory");
    }
  }
};

template <bool A_K, bool B_K>
__global__ __launch_bounds__(kNT, 2) void execute_direct_kernel(ExecuteArgs args) {
  extern __shared__ __align__(16) unsigned char smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1;
  const int wn = wave & 1;
  const int l32 = lane & 31;
  const int lh = lane >> 5;

  // Lane-constant fragment addresses (byte offsets inside a stage).
  // K-contiguous: one per sub-step; blocks are 32 rows = 2048 bytes apart.
  // Transposed: one per block (the XOR touches the block bits); sub-step and
  // half select the k rows through a constant offset.
  const uint32_t smem_off = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void)smem));
  const int i16 = lane & 15;
  const int kq = i16 >> 2;            // k row (mod 4) this lane addresses in a transpose read
  const int cq = i16 & 3;             // which 4 of the 16 columns
  const int nsub = (lane >> 4) & 1;   // which 16-column half of the 32-wide block
  uint32_t a_addr[A_K ? 2 : kMB];
  uint32_t b_addr[B_K ? 2 : kNB];
  if constexpr (A_K) {
    const int sw = (l32 >> 2) & 3;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      a_addr[ks] = (wm * kWTM + l32) * 64 + (((2 * ks + lh) ^ sw) * 16);
  } else {
#pragma unroll
    for (int i = 0; i < kMB; ++i) {
      const int c = wm * (kWTM / 8) + i * 4 + 2 * nsub + (cq >> 1);
      a_addr[i] = ((8 * lh + kq) * (kTM / 8) + (c ^ (4 * kq))) * 16 + (cq & 1) * 8;
    }
  }
  if constexpr (B_K) {
    const int sw = (l32 >> 2) & 3;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      b_addr[ks] = kATile + (wn * kWTN + l32) * 64 + (((2 * ks + lh) ^ sw) * 16);
  } else {
#pragma unroll
    for (int j = 0; j < kNB; ++j) {
      const int c = wn * (kWTN / 8) + j * 4 + 2 * nsub + (cq >> 1);
      b_addr[j] = kATile + ((8 * lh + kq) * (kTN / 8) + (c ^ (4 * kq))) * 16 + (cq & 1) * 8;
    }
  }

  // Element strides of the stored operands along (tile row, K).
  const int64_t a_rs = args.transA ? 1 : args.lda;
  const int64_t a_ks = args.transA ? args.lda : 1;
  const int64_t b_rs = args.transB ? args.ldb : 1;
  const int64_t b_ks = args.transB ? 1 : args.ldb;

  for (int64_t it = blockIdx.x; it < args.n_items; it += gridDim.x) {
    const WorkItem item = args.items[it];
    const cleave_task task = args.tasks[item.task];
    const uint32_t sub_cols = (task.n_len + kTN - 1) / kTN;
    const uint32_t sub_m = item.sub / sub_cols;
    const uint32_t sub_n = item.sub - sub_m * sub_cols;
    const int m_valid = min(static_cast<int>(task.m_len - sub_m * kTM), kTM);
    const int n_valid = min(static_cast<int>(task.n_len - sub_n * kTN), kTN);
    const int64_t m_base = static_cast<int64_t>(task.m0) + static_cast<int64_t>(sub_m) * kTM;
    const int64_t n_base = static_cast<int64_t>(task.n0) + static_cast<int64_t>(sub_n) * kTN;
    const int steps = static_cast<int>(task.k_len) / kBK;

    const unsigned char* a_ptr = static_cast<const unsigned char*>(args.A) +
                                 (m_base * a_rs + static_cast<int64_t>(task.k0) * a_ks) * 2;
    const unsigned char* b_ptr = static_cast<const unsigned char*>(args.B) +
                                 (n_base * b_rs + static_cast<int64_t>(task.k0) * b_ks) * 2;
    const int64_t a_step = a_ks * kBK * 2;    // bytes per K step
    const int64_t b_step = b_ks * kBK * 2;

    DirectTile<A_K, kTM> ta;
    DirectTile<B_K, kTN> tb;
    ta.init(a_rs, a_ks, m_valid, wave, lane);
    tb.init(b_rs, b_ks, n_valid, wave, lane);

    f32x16 acc[kMB][kNB];
#pragma unroll
    for (int i = 0; i < kMB; ++i)
#pragma unroll
      for (int j = 0; j < kNB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4 fa[2][kMB], fb[2][kNB];

    auto issue = [&](int s, int st) {
      const uint32_t stage = smem_off + st * kStage;
      ta.issue(a_ptr + s * a_step, stage, wave);
      tb.issue(b_ptr + s * b_step, stage + kATile, wave);
    };
    // Fragment reads are ordinary (compiler-visible) LDS loads: the compiler
    // tracks their completion, and every address is a lane-constant register
    // plus a compile-time offset (stage, block, sub-step).
    auto tr_read = [&](const unsigned char* p) -> u32x2 {
      return __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)p));
    };
    // Fragments of sub-step KS (0 or 1) of ring stage ST into register set `buf`.
    auto read_frags = [&](auto st, auto ks_tag, int buf) {
      constexpr int ST = decltype(st)::value;
      constexpr int KS = decltype(ks_tag)::value;
#pragma unroll
      for (int i = 0; i < kMB; ++i) {
        if constexpr (A_K) {
          fa[buf][i] = *reinterpret_cast<const u32x4*>(smem + a_addr[KS] + ST * kStage + i * 2048);
        } else {
          const unsigned char* p = smem + a_addr[i] + ST * kStage + KS * (16 * (kTM / 8) * 16);
          const u32x2 lo = tr_read(p);
          const u32x2 hi = tr_read(p + 4 * (kTM / 8) * 16);
          fa[buf][i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
        }
      }
#pragma unroll
      for (int j = 0; j < kNB; ++j) {
        if constexpr (B_K) {
          fb[buf][j] = *reinterpret_cast<const u32x4*>(smem + b_addr[KS] + ST * kStage + j * 2048);
        } else {
          const unsigned char* p = smem + b_addr[j] + ST * kStage + KS * (16 * (kTN / 8) * 16);
          const u32x2 lo = tr_read(p);
          const u32x2 hi = tr_read(p + 4 * (kTN / 8) * 16);
          fb[buf][j] = u32x4{lo[0], lo[1], hi[0], hi[1]};
        }
      }
    };
    auto mma = [&](int buf) {
#pragma unroll
      for (int i = 0; i < kMB; ++i)
#pragma unroll
        for (int j = 0; j < kNB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, fa[buf][i]), __builtin_bit_cast(bf16x8, fb[buf][j]),
              acc[i][j], 0, 0, 0);
    };

    // Prologue.  The previous work item's last fragment reads completed before
    // its final barrier, so the ring can be refilled right away.
    issue(0, 0);
    if (steps > 1) issue(1, 1);
    if (steps > 2) issue(2, 2);
    if (steps > 2) {
      CLEAVE_WAIT_BARRIER(2 * kLoadsPerStep);
    } else if (steps > 1) {
      CLEAVE_WAIT_BARRIER(kLoadsPerStep);
    } else {
      CLEAVE_WAIT_BARRIER(0);
    }
    read_frags(int_c<0>{}, int_c<0>{}, 0);

    // One K step out of ring stage ST.  The barrier sits between the two
    // sub-steps: by then this wave holds all fragments of step s, step s+1 has
    // landed (loads return in order; only step s+2's may still be in flight),
    // so stage ST can be refilled with step s+3 and the first fragments of step
    // s+1 fetched while the second sub-step multiplies.
    auto k_step = [&](auto st, int s) {
      constexpr int ST = decltype(st)::value;
      read_frags(st, int_c<1>{}, 1);
      mma(0);
      if (s + 2 < steps) {
        CLEAVE_WAIT_BARRIER(kLoadsPerStep);
      } else {
        CLEAVE_WAIT_BARRIER(0);
      }
      if (s + 3 < steps) issue(s + 3, ST);
      if (s + 1 < steps) read_frags(int_c<(ST + 1) % kStages>{}, int_c<0>{}, 0);
      mma(1);
    };
    int s = 0;
    for (; s + kStages <= steps; s += kStages) {
      k_step(int_c<0>{}, s);
      k_step(int_c<1>{}, s + 1);
      k_step(int_c<2>{}, s + 2);
    }
    if (s < steps) k_step(int_c<0>{}, s);
    if (s + 1 < steps) k_step(int_c<1>{}, s + 1);

    // Partial block: row-major m_len x n_len at partial_off.  A 32 x 32 MFMA
    // block leaves lane l with column l % 32 and rows 8*q + 4*(l / 32) + r, so
    // half a wave writes one aligned 128-byte run per store.
    const int64_t ldp = task.n_len;
    const int row0 = wm * kWTM + lh * 4;
    const int col0 = wn * kWTN + l32;
    float* tp = args.partials + task.partial_off +
                (static_cast<int64_t>(sub_m) * kTM + row0) * ldp + sub_n * kTN + col0;
    if (m_valid == kTM && n_valid == kTN) {
#pragma unroll
      for (int i = 0; i < kMB; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float* p = tp + static_cast<int64_t>(i * 32 + q * 8 + r) * ldp;
#pragma unroll
            for (int j = 0; j < kNB; ++j) p[j * 32] = acc[i][j][q * 4 + r];
          }
    } else {
#pragma unroll
      for (int i = 0; i < kMB; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int rr = i * 32 + q * 8 + r;
            float* p = tp + static_cast<int64_t>(rr) * ldp;
#pragma unroll
            for (int j = 0; j < kNB; ++j)
              if (row0 + rr < m_valid && col0 + j * 32 < n_valid) p[j * 32] = acc[i][j][q * 4 + r];
          }
    }
  }
}

template <bool A_K, bool B_K>
hipError_t launch_one(const ExecuteArgs& args, int grid, hipStream_t stream) {
  constexpr size_t lds = kStages * kStage;
  auto kern = execute_direct_kernel<A_K, B_K>;
  static thread_local int configured_device = -1;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (configured_device != dev) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    configured_device = dev;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), lds, stream, args);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_execute_direct(const ExecuteArgs& args, int grid, hipStream_t stream) {
  const bool a_k = !args.transA;   // A stored M x K: K-contiguous
  const bool b_k = args.transB;    // B stored N x K: K-contiguous
  if (a_k && b_k) return launch_one<true, true>(args, grid, stream);
  if (a_k && !b_k) return launch_one<true, false>(args, grid, stream);
  if (!a_k && b_k) return launch_one<false, true>(args, grid, stream);
  return launch_one<false, false>(args, grid, stream);
}

}  // namespace cleave
