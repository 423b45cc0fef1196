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
  // lds_tile: byte offset of the tile inside the workgroup's LDS.
  __device__ __forceinline__ void issue(const unsigned char* gbase, unsigned char* lds_tile,
                                        int wave) const {
#pragma unroll
    for (int i = 0; i < kLoads; ++i)
      __builtin_amdgcn_global_load_lds((glb_void)(gbase + goff[i]),
                                       (lds_void)(lds_tile + (wave + 4 * i) * 1024), 16, 0, 0);
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
  // LDS reads per sub-step: one 16-byte read per K-contiguous block, two
  // transpose reads per block otherwise.
  constexpr int kReads = (A_K ? kMB : 2 * kMB) + (B_K ? kNB : 2 * kNB);

  // Lane-constant fragment addresses (byte offsets inside a stage).
  // K-contiguous: one per sub-step; blocks are 32 rows = 2048 bytes apart.
  // Transposed: one per block (the XOR touches the block bits); sub-step and
  // half select the k rows through a constant offset.
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

    auto issue = [&](int s) {
      unsigned char* stage = smem + (s % kStages) * kStage;
      ta.issue(a_ptr + s * a_step, stage, wave);
      tb.issue(b_ptr + s * b_step, stage + kATile, wave);
    };
    // Fragment reads are issued through inline asm so that the compiler does
    // not order them against the in-flight direct loads (it would wait for all
    // of those before every transpose read); their completion is awaited by
    // frag_wait() below, which also ties the registers to the wait.
    auto lds_off = [](const unsigned char* p) -> uint32_t {
      return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void)p));
    };
    auto read_b128 = [&](uint32_t addr) -> u32x4 {
      u32x4 v;
      asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
      return v;
    };
    auto read_tr = [&](uint32_t addr, uint32_t addr_hi) -> u32x4 {
      u32x2 lo, hi;
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(addr));
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(hi) : "v"(addr_hi));
      return u32x4{lo[0], lo[1], hi[0], hi[1]};
    };
    // Fragments of sub-step ks (0 or 1) of the stage into register set `buf`.
    auto read_frags = [&](const unsigned char* stage, int ks, int buf) {
      const uint32_t base = lds_off(stage);
#pragma unroll
      for (int i = 0; i < kMB; ++i) {
        if constexpr (A_K) {
          fa[buf][i] = read_b128(base + a_addr[ks] + i * 2048);
        } else {
          const uint32_t p = base + a_addr[i] + ks * (16 * (kTM / 8) * 16);
          fa[buf][i] = read_tr(p, p + 4 * (kTM / 8) * 16);
        }
      }
#pragma unroll
      for (int j = 0; j < kNB; ++j) {
        if constexpr (B_K) {
          fb[buf][j] = read_b128(base + b_addr[ks] + j * 2048);
        } else {
          const uint32_t p = base + b_addr[j] + ks * (16 * (kTN / 8) * 16);
          fb[buf][j] = read_tr(p, p + 4 * (kTN / 8) * 16);
        }
      }
    };
    // LDS reads return in order: once at most kReads (one sub-step's worth,
    // issued after the set in question) are outstanding, set `buf` is complete.
    // YOUNGER = true: a younger set has been issued since; false: none.
    auto frag_wait = [&](int buf, bool younger) {
      if (younger) {
        asm volatile("s_waitcnt lgkmcnt(%6)"
                     : "+v"(fa[buf][0]), "+v"(fa[buf][1]), "+v"(fa[buf][2]), "+v"(fa[buf][3]),
                       "+v"(fb[buf][0]), "+v"(fb[buf][1])
                     : "n"(kReads));
      } else {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(fa[buf][0]), "+v"(fa[buf][1]), "+v"(fa[buf][2]), "+v"(fa[buf][3]),
                       "+v"(fb[buf][0]), "+v"(fb[buf][1]));
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
    issue(0);
    if (steps > 1) issue(1);
    if (steps > 2) issue(2);
    if (steps > 2) {
      CLEAVE_WAIT_BARRIER(2 * kLoadsPerStep);
    } else if (steps > 1) {
      CLEAVE_WAIT_BARRIER(kLoadsPerStep);
    } else {
      CLEAVE_WAIT_BARRIER(0);
    }
    read_frags(smem, 0, 0);

    for (int s = 0; s < steps; ++s) {
      const unsigned char* cur = smem + (s % kStages) * kStage;
      read_frags(cur, 1, 1);
      frag_wait(0, true);
      mma(0);
      // Step s+1 has landed (loads return in order; only step s+2's may still
      // be in flight), and this wave's reads of stage s are complete.
      if (s + 2 < steps) {
        CLEAVE_WAIT_BARRIER(kLoadsPerStep);
      } else {
        CLEAVE_WAIT_BARRIER(0);
      }
      if (s + 3 < steps) issue(s + 3);            // reuses the stage just read
      if (s + 1 < steps) {
        read_frags(smem + ((s + 1) % kStages) * kStage, 0, 0);
        frag_wait(1, true);
      } else {
        frag_wait(1, false);
      }
      mma(1);
    }

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
