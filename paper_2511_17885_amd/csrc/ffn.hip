// Expert FFNs of Eq.4 as grouped GEMMs on the matrix cores.
//
//   GEMM-1 (per expert e, rows gathered through the permutation):
//       h = silu(X_e W_gate[e]^T) * (X_e W_up[e]^T)      fused SwiGLU epilogue, h stored in dtype
//   GEMM-2:  y = h W_down[e]^T
//
// With FastMMoE switched on an expert sees a few dozen to a few hundred rows, far below the ~315
// rows at which a bf16 expert becomes compute bound on this chip, so the bf16 kernel is built
// around the weight stream:
//  * fmoe_set_weights re-lays the (static) expert weights once into matrix-core operand order:
//    for a column block and a 32-wide k step, the 64 lanes' 16-byte B fragments of
//    v_mfma_f32_16x16x32_bf16 are contiguous (1 KB), gate and up fragments interleaved, k steps
//    consecutive.  A wavefront's whole weight stream for its columns is then one linear run of
//    memory that it loads straight into registers -- no LDS hop, no address arithmetic, perfect
//    coalescing and DRAM page locality -- and every weight byte is fetched by exactly one wavefront
//    per row tile.
//  * a block owns a 128-row tile of one expert and 4 column blocks (one per wavefront); the
//    gathered activation rows are loaded straight from global memory into a 4-stage LDS ring
//    (buffer_load ... lds: no register hop, no LDS store instructions) in a bank-conflict-free
//    swizzled layout; both streams run 3 k-tiles ahead, in a loop whose steady state has no
//    predicated loads so the hardware wait counters can be set exactly.
//  * the ragged per-expert row counts become device-built lists of row tiles (tiles.h); the
//    always-on shared experts are one more dense group in the same lists and the same launch,
//    treated as ONE FFN whose hidden dimension is the concatenation of the N_s experts, so their
//    sum is accumulated in fp32 inside the down projection.
//  * block -> work: workgroups are spread round-robin over the 8 XCDs (each with its own L2), so
//    the linear block id is decoded as (batch of 8 row tiles, column tile, tile within the batch
//    = XCD); all column tiles of one row tile run on one XCD and its activation rows are fetched
//    from HBM once.
// The fp32 storage type (a correctness configuration) uses a plain LDS-tiled kernel on the fp32
// MFMA with the caller's weight layout.

#include <type_traits>

#include "common.h"
#include "tiles.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // one 16-byte chunk

__device__ __forceinline__ float silu_mul(float g, float u) {
  return g * __frcp_rn(1.0f + __expf(-g)) * u;
}
// The same for values that are rounded to bf16 next: the hardware reciprocal (1 ulp of fp32) instead of
// the correctly rounded one, a third of the instructions (1.7 % of the gate/up kernel at 2064 rows per expert).
__device__ __forceinline__ float silu_mul_bf16(float g, float u) {
  return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

// ======================================================================== bf16: weight-stream kernel
constexpr int SBM = 128;        // rows per tile: 8 MFMA row blocks of 16
constexpr int SBK = 64;         // k per tile: two 32-wide MFMA steps; one LDS row = 128 bytes
constexpr int A_STAGES = 4;     // LDS ring of activation k-tiles (weight-stream shape)
constexpr int B_SLOTS = 4;      // register ring of weight k-tiles (weight-stream shape)
// The dense shape of the kernel, for row lists of a few hundred rows per expert and more (where LDS and
// the CU's load path rather than the weight stream hold the weight-stream shape back: it reads every
// activation fragment from LDS once per column block and fetches every activation tile once per four
// column blocks): a workgroup owns 128 rows x 8 column blocks, each wavefront DNCB = 2 column blocks.  A
// wavefront's activation fragments then feed twice as many matrix instructions, which halves the LDS
// reads and the activation fetches per flop.  Two workgroups still share a CU (one hides the other's
// start-up and epilogue), so a wavefront has 256 registers: 128 accumulation registers that the kernel
// names itself and 128 vector registers for a k-step ring of weights, one group of fragments and
// addresses, which is why the wavefront-uniform part of every address is kept in scalar registers.
constexpr int DNCB = 2;         // column blocks per wavefront
constexpr int DA_STAGES = 4;    // LDS ring of activation k tiles (64 wide)
constexpr int DB_SLOTS = 4;     // register ring of weight k steps (32 wide)

struct StreamProblem {
  const bf16_t* A;            // [*, lda]
  int lda;
  const int32_t* map1;        // row -> index (perm_src) or null
  const int32_t* map2;        // index -> token (kept_idx) or null
  int map1_limit;             // clamp for map1 values (exclusive), <= 0: none
  const u32x4_t* Bp;          // packed weights
  long long group_stride;     // 16-byte units between groups
  int nbw;                    // column blocks per group in the packing
  int ks;                     // 32-wide k steps per column block in the packing (K padded to 64)
  bf16_t* C;                  // [*, ldc]
  int ldc;
  int N, K;
  int n_col_tiles;
  int a_group_off;            // shared group g reads A columns from g*a_group_off (elements)
  long long c_group_off;      // and writes C at g*c_group_off (elements)
};

struct StreamArgs {
  StreamProblem p0;           // routed experts
  StreamProblem p1;           // shared group (tile.group == E)
  int E;
  const fmoe_tile* tiles;
  const int32_t* n_tiles;     // device
  int cols;                   // work items per tile entry in this launch (column tiles, or groups of them)
  int cols_entry;             // column tiles per tile entry
};

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding: vmcnt = bits 15:14 | 3:0)
#define FMOE_WAIT_VM(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
__device__ __forceinline__ void wait_vm_upto(int n) {   // n not known at compile time (loop tails)
  switch (n < 0 ? 0 : n) {
    case 0: FMOE_WAIT_VM(0); break;
    case 1: case 2: case 3: FMOE_WAIT_VM(1); break;
    case 4: case 5: case 6: case 7: FMOE_WAIT_VM(4); break;
    case 8: case 9: case 10: case 11: FMOE_WAIT_VM(8); break;
    case 12: case 13: case 14: case 15: FMOE_WAIT_VM(12); break;
    case 16: case 17: case 18: case 19: FMOE_WAIT_VM(16); break;
    default: FMOE_WAIT_VM(20); break;
  }
}
// NRB operand fragments (16 bytes per lane each, 2048 bytes apart) from LDS byte address `addr`,
// valid on return.  Written as one block of machine instructions so that the compiler, which knows
// nothing about the asynchronous global->LDS loads that filled the tile, neither adds waits for them
// here nor touches the destination registers before the LDS counter has drained.
template <int NRB>
__device__ __forceinline__ void lds_read_frags(uint32_t addr, u32x4_t (&f)[NRB]) {
  static_assert(NRB == 2 || NRB == 3 || NRB == 4 || NRB == 6 || NRB == 8, "supported fragment counts");
  if constexpr (NRB == 2) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:2048\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(f[0]), "=&v"(f[1]) : "v"(addr) : "memory");
  } else if constexpr (NRB == 3) {
    asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %3 offset:2048\n\t"
                 "ds_read_b128 %2, %3 offset:4096\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]) : "v"(addr) : "memory");
  } else if constexpr (NRB == 4) {
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:2048\n\t"
                 "ds_read_b128 %2, %4 offset:4096\n\tds_read_b128 %3, %4 offset:6144\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]) : "v"(addr) : "memory");
  } else if constexpr (NRB == 6) {
    asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %6 offset:2048\n\t"
                 "ds_read_b128 %2, %6 offset:4096\n\tds_read_b128 %3, %6 offset:6144\n\t"
                 "ds_read_b128 %4, %6 offset:8192\n\tds_read_b128 %5, %6 offset:10240\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]), "=&v"(f[4]), "=&v"(f[5])
                 : "v"(addr) : "memory");
  } else {
    asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:2048\n\t"
                 "ds_read_b128 %2, %8 offset:4096\n\tds_read_b128 %3, %8 offset:6144\n\t"
                 "ds_read_b128 %4, %8 offset:8192\n\tds_read_b128 %5, %8 offset:10240\n\t"
                 "ds_read_b128 %6, %8 offset:12288\n\tds_read_b128 %7, %8 offset:14336\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]), "=&v"(f[4]), "=&v"(f[5]),
                   "=&v"(f[6]), "=&v"(f[7])
                 : "v"(addr) : "memory");
  }
}
// The same reads without the wait and with a compile-time byte offset OFF on top of the address register
// (one register then serves every stage of the ring): lds_issue_frags_at starts them, lds_settle_frags
// waits for them and is the point from which the compiler may use the registers (they are in/out
// operands of the wait).
template <int NRB, int OFF>
__device__ __forceinline__ void lds_issue_frags_at(uint32_t addr, u32x4_t (&f)[NRB]) {
  static_assert(NRB == 2 || NRB == 3 || NRB == 4, "supported fragment counts");
  static_assert(OFF >= 0 && OFF + (NRB - 1) * 2048 < 65536, "offset field of an LDS instruction");
  if constexpr (NRB == 2) {
    asm volatile("ds_read_b128 %0, %2 offset:%3\n\tds_read_b128 %1, %2 offset:%4"
                 : "=&v"(f[0]), "=&v"(f[1]) : "v"(addr), "n"(OFF), "n"(OFF + 2048) : "memory");
  } else if constexpr (NRB == 3) {
    asm volatile("ds_read_b128 %0, %3 offset:%4\n\tds_read_b128 %1, %3 offset:%5\n\tds_read_b128 %2, %3 offset:%6"
                 : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2])
                 : "v"(addr), "n"(OFF), "n"(OFF + 2048), "n"(OFF + 4096) : "memory");
  } else {
    asm volatile("ds_read_b128 %0, %4 offset:%5\n\tds_read_b128 %1, %4 offset:%6\n\t"
                 "ds_read_b128 %2, %4 offset:%7\n\tds_read_b128 %3, %4 offset:%8"
                 : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3])
                 : "v"(addr), "n"(OFF), "n"(OFF + 2048), "n"(OFF + 4096), "n"(OFF + 6144) : "memory");
  }
}
template <int NRB>
__device__ __forceinline__ void lds_settle_frags(u32x4_t (&f)[NRB]) {
  static_assert(NRB == 2 || NRB == 3 || NRB == 4, "supported fragment counts");
  if constexpr (NRB == 2) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]) : : "memory");
  } else if constexpr (NRB == 3) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]) : : "memory");
  } else {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : : "memory");
  }
}
#define FMOE_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// One (row tile, column tile) work item.  NAB = number of live 32-row bands of the tile (1..4):
// a compile-time constant, so the k loop below is straight-line code with a fixed number of loads,
// LDS reads and matrix instructions per step, and rows past the last live band cost nothing.
//   weights:     register ring of B_SLOTS k-tiles per wavefront (B_SLOTS-1 in flight)
//   activations: LDS ring of A_STAGES k-tiles filled by direct global->LDS loads (no register hop,
//                no LDS store instructions; A_STAGES-1 in flight).  Such a load drops the 64 lanes'
//                16-byte pieces at consecutive LDS addresses, so which (row, k chunk) a lane fetches
//                decides the LDS layout: rows are 128 bytes, and row r keeps its 16-byte chunk c at
//                position c ^ ((r >> 1) & 7), which makes the 16 rows x 16 bytes read for one matrix
//                operand fall on 16 different bank groups without any padding.
// Workgroup barrier without the memory fence of __syncthreads(): a fence would wait for EVERY
// outstanding global->LDS load (they count as stores to LDS), i.e. drain the prefetch ring each
// step.  What the barrier has to order here is covered explicitly: a wavefront waits for its own
// loads of the tile about to be read (FMOE_WAIT_VM) before the barrier, and its LDS reads of the
// previous tile have returned (lds_read_frags) before it.
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {   // f(integral_constant<int, i>) for i in [I, N)
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Byte offsets (into the buffer descriptor over P.A) of the activation rows this lane fetches: rows
// 32*it + 8*wave + lane/8 of the tile, through the two-level gather; rows past the tile reuse its last row.
template <int NAB>
__device__ __forceinline__ void gather_offsets(const StreamProblem& P, const fmoe_tile& tile, uint32_t (&a_src)[NAB]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t a_max_row = 0xffffffffu / ((uint32_t)P.lda * 2u) - 1u;
#pragma unroll
  for (int it = 0; it < NAB; ++it) {
    const int r = 32 * it + 8 * wave + (lane >> 3);
    int src = tile.row0 + (r < tile.rows ? r : tile.rows - 1);
    if (P.map1) {
      src = P.map1[src];
      if (P.map1_limit > 0) src = src < 0 ? 0 : (src >= P.map1_limit ? P.map1_limit - 1 : src);
    }
    if (P.map2) src = P.map2[src];
    src = (uint32_t)src < a_max_row ? src : (int)a_max_row;   // offsets stay below 4 GiB whatever the input
    a_src[it] = (uint32_t)src * (uint32_t)P.lda * 2u;
  }
}

// Epilogue of one 128-row x 4-column-block output tile (column tile nt of the packing): accumulator
// register v of lane l holds row 4*(l/16) + v, column l%16 of a 16x16 block.  The tile is transposed
// through LDS (the activation ring, free once every wavefront has passed the opening barrier) so that
// global memory sees whole 128/256-byte row segments instead of 32-byte pieces.
template <bool SWIGLU, int NAB, int STAGES, typename ACC>
__device__ __forceinline__ void store_tile(const StreamProblem& P, const fmoe_tile& tile, int nt, ACC acc,
                                           bf16_t* As) {   // acc(rb, f): accumulator of row block rb, fragment f
  constexpr int NRB = 2 * NAB;
  constexpr int BC = SWIGLU ? 64 : 128;    // output columns of the block
  constexpr int CS = BC + 8;               // LDS row stride (elements): rows 4 apart land 16 banks apart
  static_assert(SBM * CS <= STAGES * SBM * SBK, "output tile fits in the activation ring");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int N = P.N;
  __syncthreads();   // every wavefront is done with what the ring held
  static_for<0, NRB>([&](auto rbc) {
    constexpr int rb = decltype(rbc)::value;
    const f32x4_t c0 = acc(rbc, std::integral_constant<int, 0>{});
    const f32x4_t c1 = acc(rbc, std::integral_constant<int, 1>{});
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = rb * 16 + 4 * (lane >> 4) + v;
      if (SWIGLU) {
        As[row * CS + wave * 16 + (lane & 15)] = f32_to_bf16(silu_mul_bf16(c0[v], c1[v]));
      } else {
        As[row * CS + wave * 32 + (lane & 15)] = f32_to_bf16(c0[v]);
        As[row * CS + wave * 32 + 16 + (lane & 15)] = f32_to_bf16(c1[v]);
      }
    }
  });
  __syncthreads();
  constexpr int CPR = BC / 8;              // 16-byte chunks per row
  constexpr int RPP = 256 / CPR;           // rows per pass of the block
  const int col = nt * BC + (tid % CPR) * 8;
  const bool vec_ok = ((P.ldc & 7) == 0) && (col + 8 <= N) &&
                      ((reinterpret_cast<uintptr_t>(P.C) & 15) == 0);
#pragma unroll
  for (int r0 = 0; r0 < 32 * NAB; r0 += RPP) {
    const int row = r0 + tid / CPR;
    if (row >= tile.rows || col >= N) continue;
    const bf16_t* src = &As[row * CS + (tid % CPR) * 8];
    bf16_t* dst = P.C + (size_t)(tile.row0 + row) * P.ldc + col;
    if (vec_ok) {
      // streaming store: the next kernel reads the tile, this one never does, and in L2 it would only
      // displace the weights and activation tiles the other workgroups are sharing
      __builtin_nontemporal_store(*reinterpret_cast<const u32x4_t*>(src), reinterpret_cast<u32x4_t*>(dst));
    } else {
      for (int i = 0; i < 8 && col + i < N; ++i) dst[i] = src[i];
    }
  }
}

template <bool SWIGLU, int NAB>
__device__ __forceinline__ void stream_tile(const StreamProblem& P, const fmoe_tile& tile, int group, int nt,
                                            bf16_t* As) {
  constexpr int NRB = 2 * NAB;   // 16-row MFMA blocks computed
  constexpr int PER_STEP = NAB + 4;   // loads a wavefront issues per k step
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = P.K;
  const int NT = (K + SBK - 1) / SBK;

  // this workgroup's weight stream: tile nt of the packing, 16 KB per k tile, 4 KB per wavefront
  // (columns past N are zero in the packing and never stored)
  const u32x4_t* bsrc = P.Bp + (size_t)group * P.group_stride + (size_t)nt * (P.ks / 2) * 1024 + wave * 256 + lane;

  // activation pieces of this lane: rows 32*it + 8*wave + lane/8, LDS position lane%8 of the row,
  // i.e. k chunk (lane%8) ^ ((row >> 1) & 7); rows past the tile reuse its last row
  // (addressed as byte offsets into one buffer descriptor over A: the buffer form of the
  // global->LDS load is an ordinary vector-memory instruction to the compiler, whereas the
  // flat/global form makes it drain every outstanding load whenever it waits for one)
  uint32_t a_src[NAB];
  const __amdgpu_buffer_rsrc_t a_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(P.A), 0, 0xffffffff, 0x00020000);
  const int a_kc = ((lane & 7) ^ ((4 * wave + (lane >> 4)) & 7)) * 8;
  gather_offsets<NAB>(P, tile, a_src);

  f32x4_t acc[NRB][2];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int f = 0; f < 2; ++f) acc[rb][f] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t breg[B_SLOTS][2][2];   // [ring slot][k step][fragment]
  auto loadB = [&](int slot, int t) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int f = 0; f < 2; ++f) breg[slot][s][f] = bsrc[(size_t)t * 1024 + (s * 2 + f) * 64];
  };
  // k past K (ragged last tile): the address is clamped into the row; the packed weights are zero
  // there, so the product vanishes without predicating the load
  auto loadA = [&](int stage, int t) {
    const int k = t * SBK + a_kc;
    const int kk = k < K ? k : K - 8;
#pragma unroll
    for (int it = 0; it < NAB; ++it)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          a_rsrc, FMOE_LPTR(As + stage * (SBM * SBK) + (32 * it + 8 * wave) * SBK), 16,
          a_src[it] + (uint32_t)kk * 2u, 0, 0, 0);
  };
  // LDS byte address of this lane's operand piece in row block 0 of stage 0, for the two 32-wide k steps
  const uint32_t lds0 = (uint32_t)(uintptr_t)FMOE_LPTR(As);
  const uint32_t frag_row = lds0 + (uint32_t)(lane & 15) * (SBK * 2);
  const uint32_t frag_a0 = frag_row + (uint32_t)(((lane >> 4)) ^ ((lane & 15) >> 1)) * 16;
  const uint32_t frag_a1 = frag_row + (uint32_t)(((lane >> 4) + 4) ^ ((lane & 15) >> 1)) * 16;
  // One k step: the products of tile `t_now` (weights in ring slot `slot`, activations in LDS stage
  // `stage`) and, if `issue`, the loads of the tiles A_AHEAD / B_AHEAD steps further on.  The loads
  // are dealt out over the step's groups of matrix instructions instead of being issued in one
  // burst: the four wavefronts leave the barrier together, and 8 loads each at once would queue up
  // at the CU's one address unit for several hundred cycles before any of them could start to
  // multiply.
  constexpr int HB = (NRB > 4) ? NRB / 2 : NRB;   // row blocks whose operands are fetched together
  constexpr int NQ = 2 * (NRB / HB);              // groups per step
  auto step = [&](int slot, int stage, bool issue, int new_slot, int new_stage, int t_a, int t_b) {
    const int ka = t_a * SBK + a_kc;
    const uint32_t a_off = (uint32_t)(ka < K ? ka : K - 8) * 2u;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const bf16x8_t fb0 = __builtin_bit_cast(bf16x8_t, breg[slot][s][0]);
      const bf16x8_t fb1 = __builtin_bit_cast(bf16x8_t, breg[slot][s][1]);
#pragma unroll
      for (int h0 = 0; h0 < NRB; h0 += HB) {
        const int q = s * (NRB / HB) + h0 / HB;
        if (issue) {
#pragma unroll
          for (int i = 0; i < PER_STEP; ++i) {   // load i of the step goes out with group i*NQ/PER_STEP
            if ((i * NQ) / PER_STEP != q) continue;
            if (i < NAB)
              __builtin_amdgcn_raw_ptr_buffer_load_lds(
                  a_rsrc, FMOE_LPTR(As + new_stage * (SBM * SBK) + (32 * i + 8 * wave) * SBK), 16,
                  a_src[i] + a_off, 0, 0, 0);
            else
              breg[new_slot][(i - NAB) >> 1][(i - NAB) & 1] = bsrc[(size_t)t_b * 1024 + (i - NAB) * 64];
          }
        }
        u32x4_t fa[HB];
        lds_read_frags<HB>((s ? frag_a1 : frag_a0) + (uint32_t)stage * (SBM * SBK * 2) + h0 * 2048, fa);
#pragma unroll
        for (int rb = 0; rb < HB; ++rb) {
          const bf16x8_t a8 = __builtin_bit_cast(bf16x8_t, fa[rb]);
          acc[h0 + rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, fb0, acc[h0 + rb][0], 0, 0, 0);
          acc[h0 + rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, fb1, acc[h0 + rb][1], 0, 0, 0);
        }
      }
    }
  };

  // Step t issues the activations of tile t + A_AHEAD and the weights of tile t + B_AHEAD (in an
  // order the compiler may choose, but never across the barrier that opens a step); the prologue
  // replays the steps before 0 the same way.  Loads land in issue order, so "all but the newest
  // (A_AHEAD-1)*PER_STEP loads have landed" implies "tile t's activations are in LDS".
  constexpr int A_AHEAD = A_STAGES - 1, B_AHEAD = B_SLOTS - 1;
  constexpr int NEWER = (A_AHEAD - 1) * PER_STEP;
  constexpr int UNROLL = 4;    // a multiple of both ring sizes: slots and stages are compile-time
  static_assert(UNROLL % A_STAGES == 0 && UNROLL % B_SLOTS == 0, "ring indices must be static");
  static_assert(A_AHEAD <= B_AHEAD, "the prologue below starts with the weights");
  int t = 0;
  if (UNROLL + B_AHEAD <= NT) {
    // the steady loop will run: an unconditional prologue, so that the compiler's own count of the
    // loads in flight at the loop head is exact (a conditional one makes it wait for all of them)
#pragma unroll
    for (int q = -B_AHEAD; q < 0; ++q) {
      if (q + A_AHEAD >= 0) loadA((q + A_AHEAD) % A_STAGES, q + A_AHEAD);
      loadB(q + B_AHEAD, q + B_AHEAD);
      asm volatile("" ::: "memory");   // keeps the steps' loads apart
    }
    for (; t + UNROLL + B_AHEAD <= NT; t += UNROLL) {   // steady state: every load is unconditional
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        FMOE_WAIT_VM(NEWER);
        block_barrier();   // every wavefront's share of tile t+u is in LDS; all are done with tile t+u-1
        step(u % B_SLOTS, u % A_STAGES, true, (u + B_AHEAD) % B_SLOTS, (u + A_AHEAD) % A_STAGES,
             t + u + A_AHEAD, t + u + B_AHEAD);
      }
    }
  } else {
#pragma unroll
    for (int q = -B_AHEAD; q < 0; ++q) {
      if (q + A_AHEAD >= 0 && q + A_AHEAD < NT) loadA((q + A_AHEAD) % A_STAGES, q + A_AHEAD);
      if (q + B_AHEAD < NT) loadB(q + B_AHEAD, q + B_AHEAD);
      asm volatile("" ::: "memory");
    }
  }
  // Tail: 3..6 steps are left after the steady loop (1..6 when it did not run).  Every count gets its
  // own straight-line code, so that which steps still issue loads, and how many loads are newer than
  // the tile a step waits for, are compile-time facts as in the steady state (a loop with run-time
  // conditions around the loads makes the compiler wait for all of them).
  auto tail_step = [&](auto rem_c, auto j_c) {
    constexpr int REM = decltype(rem_c)::value, J = decltype(j_c)::value;
    constexpr int newer = [] {   // loads of the steps after the one that fetched tile J's activations
      int n = 0;
      for (int q = 1; q < A_AHEAD; ++q) {
        const int st = J - A_AHEAD + q;   // issuing step, relative to the first tail step
        n += (st + A_AHEAD < REM ? NAB : 0) + (st + B_AHEAD < REM ? 4 : 0);
      }
      return n;
    }();
    FMOE_WAIT_VM(newer);
    block_barrier();
    constexpr bool more = J + A_AHEAD < REM;   // the rings are equally deep: all of a step's loads or none
    step(J % B_SLOTS, J % A_STAGES, more, (J + B_AHEAD) % B_SLOTS, (J + A_AHEAD) % A_STAGES,
         t + J + A_AHEAD, t + J + B_AHEAD);
  };
  auto tail = [&](auto rem_c) {
    constexpr int REM = decltype(rem_c)::value;
    tail_step(rem_c, std::integral_constant<int, 0>{});
    if constexpr (REM > 1) tail_step(rem_c, std::integral_constant<int, 1>{});
    if constexpr (REM > 2) tail_step(rem_c, std::integral_constant<int, 2>{});
    if constexpr (REM > 3) tail_step(rem_c, std::integral_constant<int, 3>{});
    if constexpr (REM > 4) tail_step(rem_c, std::integral_constant<int, 4>{});
    if constexpr (REM > 5) tail_step(rem_c, std::integral_constant<int, 5>{});
  };
  static_assert(A_AHEAD == B_AHEAD && UNROLL + B_AHEAD == 7, "the tail below covers 1..6 left-over steps");
  switch (NT - t) {   // uniform
    case 1: tail(std::integral_constant<int, 1>{}); break;
    case 2: tail(std::integral_constant<int, 2>{}); break;
    case 3: tail(std::integral_constant<int, 3>{}); break;
    case 4: tail(std::integral_constant<int, 4>{}); break;
    case 5: tail(std::integral_constant<int, 5>{}); break;
    case 6: tail(std::integral_constant<int, 6>{}); break;
    default: break;   // 0: K is a multiple of the steady loop's stride plus its look-ahead
  }

  store_tile<SWIGLU, NAB, A_STAGES>(P, tile, nt, [&](auto rb, auto f) { return acc[rb][f]; }, As);
}

template <bool SWIGLU>
__global__ __launch_bounds__(256, 2) void ffn_stream_kernel(StreamArgs a) {
  __shared__ __align__(16) bf16_t As[A_STAGES * SBM * SBK];

  // One work item per block: item -> (batch of 8 row tiles, column tile, tile within the batch =
  // XCD).  Blocks past the device-side tile count leave at once.
  const int n_tiles = *a.n_tiles;
  const int item = blockIdx.x;
  const int xcd = item & 7;
  const int rr = item >> 3;
  const int batch = rr / a.cols;
  int nt_launch = rr - batch * a.cols;
  int ti;
  if (n_tiles >= FMOE_SEG_MIN_TILES) {
    // long lists: XCD x takes the contiguous eighth [s0, s1) of the list, so that the runs of one
    // group (whose workgroups share weights and activation rows) stay in one L2
    const int s0 = (int)(((long long)n_tiles * xcd) >> 3);
    const int s1 = (int)(((long long)n_tiles * (xcd + 1)) >> 3);
    if (batch >= s1 - s0) return;
    ti = s0 + batch;
  } else {
    // short lists: entries dealt round-robin, which spreads the few long (shared-group) tiles evenly
    ti = batch * 8 + xcd;
    if (ti >= n_tiles) return;
  }
  fmoe_tile tile = a.tiles[ti];
  const bool shared = tile.group >= a.E;
  // field-by-field select keeps the descriptors in scalar registers (indexing the kernel argument
  // dynamically would spill it to scratch memory)
  StreamProblem P;
#define FMOE_SEL(f) P.f = shared ? a.p1.f : a.p0.f
  FMOE_SEL(A); FMOE_SEL(lda); FMOE_SEL(map1); FMOE_SEL(map2); FMOE_SEL(map1_limit); FMOE_SEL(Bp);
  FMOE_SEL(group_stride); FMOE_SEL(nbw); FMOE_SEL(ks); FMOE_SEL(C); FMOE_SEL(ldc); FMOE_SEL(N);
  FMOE_SEL(K); FMOE_SEL(n_col_tiles); FMOE_SEL(a_group_off); FMOE_SEL(c_group_off);
#undef FMOE_SEL
  // column tiles this entry really has
  const int c_eff = (P.n_col_tiles - tile.col0 < a.cols) ? (P.n_col_tiles - tile.col0) : a.cols;
  if (nt_launch >= c_eff) return;
  // A group with several row tiles sits on as many XCDs (consecutive tile indices).  Its blocks are
  // re-dealt column-major: the items, ordered by (column tile, row tile), are cut into runs of C, one
  // run per original row tile, i.e. an XCD gets ALL row tiles of ~C/R column tiles, so each weight
  // column block is fetched by one XCD (two at a run boundary) instead of by all of them (weights
  // outweigh the activation rows, which every XCD then reads).
  // (runs are at most FMOE_TILE_RUN row tiles long; in a long list the whole run sits on this XCD and
  // the re-deal makes it walk the run column-major, about eight row tiles by eight column tiles at a time)
  if (tile.nrt > 1) {
    const int w = tile.rt * c_eff + nt_launch;
    const int r2 = w % tile.nrt;
    nt_launch = w / tile.nrt;
    ti = ti - tile.rt + r2;
    tile = a.tiles[ti];
  }
  const int nt = tile.col0 + nt_launch;
  const int group = shared ? tile.group - a.E : tile.group;
  if (shared) {   // per-shared-expert slices of the hidden buffer / output (down GEMM)
    P.A += (size_t)group * P.a_group_off;
    P.C += (size_t)group * P.c_group_off;
  }
  switch ((tile.rows + 31) >> 5) {   // uniform per block
    case 1: stream_tile<SWIGLU, 1>(P, tile, group, nt, As); break;
    case 2: stream_tile<SWIGLU, 2>(P, tile, group, nt, As); break;
    case 3: stream_tile<SWIGLU, 3>(P, tile, group, nt, As); break;
    default: stream_tile<SWIGLU, 4>(P, tile, group, nt, As); break;
  }
}

// The dense shape keeps its 32 accumulators in accumulation registers that it names itself: accumulator
// IDX is a[4*IDX : 4*IDX+3].  Left to the compiler, the accumulators share the vector register budget
// with everything else and part of them travels through scratch memory; named, they cost the
// allocator nothing, and, being volatile, the instructions keep their place in the step.  The compiler
// does not see what these instructions do, so it is told: dense_claim_acc() lists a0..a127 as written
// (a wavefront is then given them, and the compiler half of its 256 registers), and every matrix
// instruction lists its four registers as destroyed (mfma_at<IDX>), so that the compiler cannot keep a
// value of its own in one of them across the k loop -- it did once: a row index of the epilogue, which
// came back as accumulator bits and sent the output store to a wild address.  On top of that the build
// reads the generated code of the dense kernels from the first to the last line and fails if the
// compiler itself placed anything in an accumulation register, and the parity tests run this shape on
// every size.
template <int IDX>
__device__ __forceinline__ f32x4_t read_acc() {
  float r0, r1, r2, r3;
  asm volatile("v_accvgpr_read_b32 %0, a[%4]\n\tv_accvgpr_read_b32 %1, a[%5]\n\t"
               "v_accvgpr_read_b32 %2, a[%6]\n\tv_accvgpr_read_b32 %3, a[%7]"
               : "=v"(r0), "=v"(r1), "=v"(r2), "=v"(r3)
               : "n"(4 * IDX), "n"(4 * IDX + 1), "n"(4 * IDX + 2), "n"(4 * IDX + 3));
  return f32x4_t{r0, r1, r2, r3};
}
#include "dense_regs.inc"   // dense_claim_acc(): zeroes a0..a127 and lists them as written; mfma_at<IDX>()

// ---- the dense shape: one (row tile, group of DNCB column tiles) work item per workgroup.
// Wavefront w owns column block w of each of the DNCB column tiles nt4 .. nt4+DNCB-1 of the packing (so
// the epilogue of the weight-stream shape serves each of them in turn).  Column tiles at or past
// `ct_limit` do not belong to this work item: their weights are still fetched (clamped into the packing,
// so that every load stays unconditional) but nothing is stored for them.
// The k loop advances in steps of 32: the weights of a step are one register-ring slot (DB_SLOTS slots,
// DB_SLOTS-1 steps in flight), the activations stay in k tiles of 64 in the LDS ring (DA_STAGES tiles,
// DA_STAGES-1 in flight) with one workgroup barrier per tile.  Every step issues its loads
// unconditionally -- past the end of the reduction they fetch the last step / tile again, into slots
// nobody reads -- so the number of loads in flight at every wait is a compile-time constant and there
// is no separate code for the last steps.
// Per step and pair of row blocks a wavefront issues 2 LDS reads for 4*DNCB matrix instructions.
template <bool SWIGLU, int NAB>
__device__ __forceinline__ void dense_tile(const StreamProblem& P, const fmoe_tile& tile, int group, int nt4,
                                           int ct_limit, bf16_t* As) {
  constexpr int NRB = 2 * NAB;
  const int tid = threadIdx.x, lane = tid & 63;
  // the wavefront's number as a scalar: what depends on it alone (LDS destinations of the direct loads,
  // the base of the weight stream) is then computed once per wavefront, not per lane
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = P.K;
  const int NT = (K + SBK - 1) / SBK;
  const int NKS = 2 * NT;
  const int n_pack_tiles = (P.nbw + 3) / 4;

  // weight stream of column tile j: one buffer descriptor over the packed weights, a wavefront-uniform
  // byte offset (scalar) and the lane's 16 bytes (one vector register for all loads); the host refuses
  // this shape when the packed weights of a launch exceed 4 GiB
  const __amdgpu_buffer_rsrc_t b_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4_t*>(P.Bp), 0, 0xffffffff, 0x00020000);
  uint32_t bbase[DNCB];
#pragma unroll
  for (int j = 0; j < DNCB; ++j) {
    int pt = nt4 + j;
    pt = pt < n_pack_tiles ? pt : n_pack_tiles - 1;
    bbase[j] = (uint32_t)(((size_t)group * P.group_stride + (size_t)pt * (P.ks / 2) * 1024 + wave * 256) * 16);
  }
  const uint32_t lane16 = (uint32_t)lane * 16u;
  uint32_t a_src[NAB];
  const __amdgpu_buffer_rsrc_t a_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(P.A), 0, 0xffffffff, 0x00020000);
  const int a_kc = ((lane & 7) ^ ((4 * wave + (lane >> 4)) & 7)) * 8;
  gather_offsets<NAB>(P, tile, a_src);

  dense_claim_acc();   // accumulator (j, rb, f) is number (j*NRB + rb)*2 + f, all zero now

  u32x4_t breg[DB_SLOTS][DNCB][2];   // [ring slot][column tile][fragment]
  // weights of k step ks (clamped to the last one): two fragments per column tile
  auto loadB1 = [&](int slot, int ks, int i) {   // load i of the step's 2*DNCB
    const int kc = ks < NKS ? ks : NKS - 1;
    const uint32_t koff = (uint32_t)(((kc >> 1) * 1024 + (kc & 1) * 128 + (i & 1) * 64) * 16);   // uniform
    breg[slot][i >> 1][i & 1] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, lane16, bbase[i >> 1] + koff, 0);
  };
  // activations of k tile t (clamped to the last one); k past K re-reads the row's last chunk, where
  // the packed weights are zero
  auto loadA1 = [&](int stage, int t, int it) {
    const int tc = t < NT ? t : NT - 1;
    const int k = tc * SBK + a_kc;
    const int kk = k < K ? k : K - 8;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        a_rsrc, FMOE_LPTR(As + stage * (SBM * SBK) + (32 * it + 8 * wave) * SBK), 16,
        a_src[it] + (uint32_t)kk * 2u, 0, 0, 0);
  };
  const uint32_t lds0 = (uint32_t)(uintptr_t)FMOE_LPTR(As);
  const uint32_t frag_row = lds0 + (uint32_t)(lane & 15) * (SBK * 2);
  const uint32_t frag_a0 = frag_row + (uint32_t)(((lane >> 4)) ^ ((lane & 15) >> 1)) * 16;
  const uint32_t frag_a1 = frag_row + (uint32_t)(((lane >> 4) + 4) ^ ((lane & 15) >> 1)) * 16;

  // Row blocks are taken two at a time: the operands of the next pair are requested from LDS before the
  // matrix instructions of the current pair are issued and awaited after them -- also from the first step
  // of a k tile into its second (same tile, no barrier between them) -- so that a wavefront meets the LDS
  // latency once per k tile, behind the barrier that opens it.  Pair number U*NH + h (step U of the round,
  // pair h) alternates between the two operand buffers.
  constexpr int HB = 2;                           // row blocks per pair
  constexpr int NH = NRB / HB;                    // pairs per k step (= NAB)
  constexpr int B_AHEAD = DB_SLOTS - 1, A_AHEAD = DA_STAGES - 1;
  constexpr int UNROLL = 2 * DA_STAGES;           // k steps per round: ring indices are compile-time
  static_assert(UNROLL % DB_SLOTS == 0, "ring indices must be static");
  static_assert((UNROLL * NH) % 2 == 0, "operand buffers alternate consistently from round to round");
  static_assert(2 * A_AHEAD >= B_AHEAD, "a tile's activations are issued before its weights");
  // loads newer than the weights of the step about to run: those of the last B_AHEAD-1 steps, of which
  // every second one also carries a tile of activations
  constexpr int NEWER_EVEN = (B_AHEAD - 1) * 2 * DNCB + ((B_AHEAD - 1) / 2) * NAB;        // before an even step
  constexpr int NEWER_ODD = (B_AHEAD - 1) * 2 * DNCB + (B_AHEAD / 2) * NAB;               // before an odd step

  u32x4_t fa[2][HB];
  // k step `ks` = round base + U (U static): products of the step, loads of the steps further on
  auto kstep = [&](auto uc, int ks) {
    constexpr int U = decltype(uc)::value;
    constexpr int slot = U % DB_SLOTS, s = U & 1, stage = (U >> 1) % DA_STAGES;
    constexpr int new_slot = (U + B_AHEAD) % DB_SLOTS, new_stage = ((U >> 1) + A_AHEAD) % DA_STAGES;
    constexpr int NL = 2 * DNCB + (s == 0 ? NAB : 0);   // loads this step issues
    constexpr int stage_off = stage * (SBM * SBK * 2);
    if constexpr (s == 0) {
      FMOE_WAIT_VM(NEWER_EVEN);
      block_barrier();   // every wavefront's share of the tile is in LDS; all are done with the tile before
    } else {
      FMOE_WAIT_VM(NEWER_ODD);
    }
    // (an odd step's first operands were requested by the step before)
    if constexpr (s == 0) lds_issue_frags_at<HB, stage_off>(frag_a0, fa[(U * NH) & 1]);
    lds_settle_frags<HB>(fa[(U * NH) & 1]);
    static_for<0, NH>([&](auto hc) {
      constexpr int h = decltype(hc)::value;
      constexpr int h0 = h * HB;
      constexpr int cur = (U * NH + h) & 1, nxt = cur ^ 1;
      if constexpr (h + 1 < NH)
        lds_issue_frags_at<HB, stage_off + (h0 + HB) * 2048>(s ? frag_a1 : frag_a0, fa[nxt]);
      else if constexpr (s == 0)
        lds_issue_frags_at<HB, stage_off>(frag_a1, fa[nxt]);   // first pair of the tile's second step
#pragma unroll
      for (int i = 0; i < NL; ++i) {           // load i of the step goes out with pair i*NH/NL
        if ((i * NH) / NL != h) continue;
        if (s == 0 && i < NAB) loadA1(new_stage, (ks >> 1) + A_AHEAD, i);
        else loadB1(new_slot, ks + B_AHEAD, i - (s == 0 ? NAB : 0));
      }
      static_for<0, DNCB>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const bf16x8_t fb0 = __builtin_bit_cast(bf16x8_t, breg[slot][j][0]);
        const bf16x8_t fb1 = __builtin_bit_cast(bf16x8_t, breg[slot][j][1]);
        static_for<0, HB>([&](auto rc) {
          constexpr int rb = decltype(rc)::value;
          const bf16x8_t a8 = __builtin_bit_cast(bf16x8_t, fa[cur][rb]);
          mfma_at<(j * NRB + h0 + rb) * 2>(a8, fb0);
          mfma_at<(j * NRB + h0 + rb) * 2 + 1>(a8, fb1);
        });
      });
      if constexpr (h + 1 < NH) lds_settle_frags<HB>(fa[nxt]);
    });
  };

  // prologue: what the steps before the first would have issued, in their order (activations reach
  // 2*A_AHEAD steps back, weights B_AHEAD)
  static_for<0, 2 * A_AHEAD>([&](auto qc) {
    constexpr int q = decltype(qc)::value - 2 * A_AHEAD;   // step number, negative
    if constexpr ((q + 2 * A_AHEAD) % 2 == 0) {            // an even step: activations of tile q/2 + A_AHEAD
      constexpr int t = q / 2 + A_AHEAD;
#pragma unroll
      for (int it = 0; it < NAB; ++it) loadA1(t % DA_STAGES, t, it);
    }
    if constexpr (q + B_AHEAD >= 0) {
#pragma unroll
      for (int i = 0; i < 2 * DNCB; ++i) loadB1((q + B_AHEAD) % DB_SLOTS, q + B_AHEAD, i);
    }
    asm volatile("" ::: "memory");
  });
  int ks0 = 0;
  for (; ks0 + UNROLL <= NKS; ks0 += UNROLL)
    static_for<0, UNROLL>([&](auto uc) { kstep(uc, ks0 + decltype(uc)::value); });
  switch (NKS - ks0) {   // left-over steps (an even number below UNROLL), uniform
    case 2: static_for<0, 2>([&](auto uc) { kstep(uc, ks0 + decltype(uc)::value); }); break;
    case 4: static_for<0, 4>([&](auto uc) { kstep(uc, ks0 + decltype(uc)::value); }); break;
    case 6: static_for<0, 6>([&](auto uc) { kstep(uc, ks0 + decltype(uc)::value); }); break;
    default: break;
  }
  static_assert(UNROLL == 8, "the switch above covers 2, 4 and 6 left-over steps");
  FMOE_WAIT_VM(0);   // the loads issued past the end have landed before the ring is reused
  // the last matrix instructions have retired before their accumulators are read (24 idle cycles
  // cover the longest read-after-write distance of a 16x16x32 instruction)
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
  static_for<0, DNCB>([&](auto jc) {
    constexpr int j = decltype(jc)::value;
    if (nt4 + j < ct_limit)   // uniform
      store_tile<SWIGLU, NAB, DA_STAGES>(P, tile, nt4 + j, [&](auto rbc, auto fc) {
        return read_acc<(j * NRB + decltype(rbc)::value) * 2 + decltype(fc)::value>();
      }, As);
  });
}

// Work decode as in ffn_stream_kernel, with column tiles taken DNCB at a time (a.cols = such groups per
// tile entry, a.cols_entry = column tiles per tile entry).
template <bool SWIGLU>
__global__ __launch_bounds__(256, 2) void ffn_dense_kernel(StreamArgs a) {
  __shared__ __align__(16) bf16_t As[DA_STAGES * SBM * SBK];
  const int n_tiles = *a.n_tiles;
  const int item = blockIdx.x;
  const int xcd = item & 7;
  const int rr = item >> 3;
  const int batch = rr / a.cols;
  int nt_launch = rr - batch * a.cols;
  int ti;
  if (n_tiles >= FMOE_SEG_MIN_TILES) {
    const int s0 = (int)(((long long)n_tiles * xcd) >> 3);
    const int s1 = (int)(((long long)n_tiles * (xcd + 1)) >> 3);
    if (batch >= s1 - s0) return;
    ti = s0 + batch;
  } else {
    ti = batch * 8 + xcd;
    if (ti >= n_tiles) return;
  }
  fmoe_tile tile = a.tiles[ti];
  const bool shared = tile.group >= a.E;
  StreamProblem P;
#define FMOE_SEL(f) P.f = shared ? a.p1.f : a.p0.f
  FMOE_SEL(A); FMOE_SEL(lda); FMOE_SEL(map1); FMOE_SEL(map2); FMOE_SEL(map1_limit); FMOE_SEL(Bp);
  FMOE_SEL(group_stride); FMOE_SEL(nbw); FMOE_SEL(ks); FMOE_SEL(C); FMOE_SEL(ldc); FMOE_SEL(N);
  FMOE_SEL(K); FMOE_SEL(n_col_tiles); FMOE_SEL(a_group_off); FMOE_SEL(c_group_off);
#undef FMOE_SEL
  // column tiles this entry really has, and groups of DNCB of them
  const int ct_here = (P.n_col_tiles - tile.col0 < a.cols_entry) ? (P.n_col_tiles - tile.col0) : a.cols_entry;
  const int c_eff = (ct_here + DNCB - 1) / DNCB;
  if (nt_launch >= c_eff) return;
  if (tile.nrt > 1) {   // column-major re-deal inside a run of row tiles, as in the weight-stream shape
    const int w = tile.rt * c_eff + nt_launch;
    const int r2 = w % tile.nrt;
    nt_launch = w / tile.nrt;
    ti = ti - tile.rt + r2;
    tile = a.tiles[ti];
  }
  const int nt4 = tile.col0 + nt_launch * DNCB;
  const int ct_limit = tile.col0 + ct_here;
  const int group = shared ? tile.group - a.E : tile.group;
  if (shared) {
    P.A += (size_t)group * P.a_group_off;
    P.C += (size_t)group * P.c_group_off;
  }
  switch ((tile.rows + 31) >> 5) {   // live 32-row bands of the tile, uniform per block
    case 1: dense_tile<SWIGLU, 1>(P, tile, group, nt4, ct_limit, As); break;
    case 2: dense_tile<SWIGLU, 2>(P, tile, group, nt4, ct_limit, As); break;
    case 3: dense_tile<SWIGLU, 3>(P, tile, group, nt4, ct_limit, As); break;
    default: dense_tile<SWIGLU, 4>(P, tile, group, nt4, ct_limit, As); break;
  }
}

// Packing: unit u (16 bytes = 8 consecutive k) -> (group, tile of 4 column blocks, 64-wide k tile,
// column block in the tile = wavefront, 32-wide k step, fragment, lane): the 16 KB a workgroup
// consumes per k tile are contiguous and its whole stream is one linear run of memory.
//   gate/up (PAIR): column block = 16 output features, fragment 0 = gate rows, 1 = up rows
//   down (!PAIR):   column block = 32 output features, fragment f = features 16f..16f+15
// src rows are [group][n][k].
template <bool PAIR>
__global__ void pack_weights_kernel(const bf16_t* __restrict__ src0, const bf16_t* __restrict__ src1,
                                    u32x4_t* __restrict__ dst, int G, int N, int K, int nbw, int ks) {
  const int nbt = (nbw + 3) / 4, NT = ks / 2;
  const size_t total = (size_t)G * nbt * NT * 1024;
  for (size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x; u < total;
       u += (size_t)gridDim.x * blockDim.x) {
    const int lane = (int)(u & 63), f = (int)((u >> 6) & 1), s2 = (int)((u >> 7) & 1), w = (int)((u >> 8) & 3);
    size_t q = u >> 10;
    const int kt = (int)(q % NT);
    q /= NT;
    const int bt = (int)(q % nbt), g = (int)(q / nbt);
    const int b = bt * 4 + w, s = kt * 2 + s2;
    const int n = PAIR ? (b * 16 + (lane & 15)) : (b * 32 + f * 16 + (lane & 15));
    const int k = s * 32 + 8 * (lane >> 4);
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (n < N && k < K) {
      const bf16_t* base = (PAIR && f) ? src1 : src0;
      v = *reinterpret_cast<const u32x4_t*>(base + ((size_t)g * N + n) * K + k);
    }
    dst[u] = v;
  }
}

// ======================================================================== fp32: LDS-tiled kernel
constexpr int BNW = 128;  // weight rows per block: 64 gate + 64 up columns, or 128 down columns

template <typename T> struct Traits;
template <> struct Traits<float> {
  static constexpr int VEC = 4;
  static constexpr int BK = 32;
  static constexpr int LDK = BK + 4;
};

struct GemmProblem {
  const void* A;            // [*, lda]
  int lda;
  const int32_t* map1;      // row -> index (perm_src) or null
  const int32_t* map2;      // index -> token (kept_idx) or null
  int map1_limit;           // clamp for map1 values (exclusive), <= 0: none
  const void* B0;           // [G, N, K] gate / down
  const void* B1;           // [G, N, K] up (SwiGLU only)
  long long group_stride;   // elements between groups (0 for the shared group)
  int ldb;                  // elements between consecutive weight rows
  void* C;                  // [*, ldc]
  int ldc;
  int N, K;
  int n_col_tiles;
  int a_group_off;          // shared group g reads A columns from g*a_group_off (elements)
  long long c_group_off;    // and writes C at g*c_group_off (elements)
};

struct GemmArgs {
  GemmProblem p0;           // routed experts
  GemmProblem p1;           // shared group (tile.group == E)
  int E;
  const fmoe_tile* tiles;
  const int32_t* n_tiles;   // device
  int n_col_tiles_max;
};

template <typename T, bool SWIGLU, int MT>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(GemmArgs a) {
  using TR = Traits<T>;
  constexpr int VEC = TR::VEC, BK = TR::BK, LDK = TR::LDK;
  constexpr int BM = 64 * MT;
  constexpr int CPR = BK / VEC;                 // 16-byte chunks per tile row (8)
  constexpr int A_IT = BM * CPR / 256;          // chunks per thread
  constexpr int B_IT = BNW * CPR / 256;
  __shared__ __align__(16) T As[BM * LDK];
  __shared__ __align__(16) T Bs[BNW * LDK];

  // XCD-aware decode of the linear block id
  const int xcd = blockIdx.x & 7;
  const int rr = blockIdx.x >> 3;
  const int batch = rr / a.n_col_tiles_max;
  const int nt_launch = rr - batch * a.n_col_tiles_max;
  const int ti = batch * 8 + xcd;
  if (ti >= *a.n_tiles) return;
  const fmoe_tile tile = a.tiles[ti];
  const bool shared = tile.group >= a.E;
  // field-by-field select keeps the descriptors in scalar registers (indexing the kernel argument
  // dynamically would spill it to scratch memory)
  GemmProblem P;
#define FMOE_SEL(f) P.f = shared ? a.p1.f : a.p0.f
  FMOE_SEL(A); FMOE_SEL(lda); FMOE_SEL(map1); FMOE_SEL(map2); FMOE_SEL(map1_limit);
  FMOE_SEL(B0); FMOE_SEL(B1); FMOE_SEL(group_stride); FMOE_SEL(ldb);
  FMOE_SEL(C); FMOE_SEL(ldc); FMOE_SEL(N); FMOE_SEL(K); FMOE_SEL(n_col_tiles);
  FMOE_SEL(a_group_off); FMOE_SEL(c_group_off);
#undef FMOE_SEL
  const int nt = tile.col0 + nt_launch;
  if (nt >= P.n_col_tiles) return;
  const int group = shared ? tile.group - a.E : tile.group;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int N = P.N, K = P.K;

  const T* Ag = static_cast<const T*>(P.A) + (shared ? (size_t)group * P.a_group_off : 0);
  const T* B0g = static_cast<const T*>(P.B0) + (size_t)group * P.group_stride;
  const T* B1g = SWIGLU ? static_cast<const T*>(P.B1) + (size_t)group * P.group_stride : nullptr;

  // per-thread chunk sources (fixed over the K loop)
  const T* a_src[A_IT];
  const T* b_src[B_IT];
  int a_lo[A_IT], b_lo[B_IT], a_k[A_IT], b_k[B_IT];
#pragma unroll
  for (int it = 0; it < A_IT; ++it) {
    const int chunk = tid + it * 256;
    const int r = chunk / CPR, kc = (chunk % CPR) * VEC;
    a_lo[it] = r * LDK + kc;
    a_k[it] = kc;
    // rows past the tile reuse its last row: their products land in accumulator rows that are
    // never stored, and the loads stay unconditional (no branches in the pipelined loop)
    int src = tile.row0 + (r < tile.rows ? r : tile.rows - 1);
    if (P.map1) {
      src = P.map1[src];
      if (P.map1_limit > 0) src = src < 0 ? 0 : (src >= P.map1_limit ? P.map1_limit - 1 : src);
    }
    if (P.map2) src = P.map2[src];
    a_src[it] = Ag + (size_t)src * P.lda;
  }
#pragma unroll
  for (int it = 0; it < B_IT; ++it) {
    const int chunk = tid + it * 256;
    const int wr = chunk / CPR, kc = (chunk % CPR) * VEC;
    b_lo[it] = wr * LDK + kc;
    b_k[it] = kc;
    int n;
    const T* base;
    if (SWIGLU) {
      n = nt * 64 + (wr & 63);
      base = (wr < 64) ? B0g : B1g;
    } else {
      n = nt * BNW + wr;
      base = B0g;
    }
    b_src[it] = base + (size_t)(n < N ? n : N - 1) * P.ldb;   // same trick for columns past N
  }
  f32x16_t acc[MT][2];
#pragma unroll
  for (int r = 0; r < MT; ++r)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.0f;

  // which 32-row groups of this wavefront hold any valid row (uniform per wavefront)
  bool live[MT];
#pragma unroll
  for (int r = 0; r < MT; ++r) live[r] = (wm * 32 * MT + 32 * r) < tile.rows;

  u32x4_t ra[A_IT], rb[B_IT];
  const u32x4_t zero4 = {0u, 0u, 0u, 0u};
  // k past K (ragged last k-tile) must contribute zeros: the address is clamped into the row and
  // the loaded value replaced by a select, so the load itself is never predicated
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int k = k0 + a_k[it];
      const int kk = k < K ? k : K - VEC;
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(a_src[it] + kk);
      ra[it] = k < K ? v : zero4;
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int k = k0 + b_k[it];
      const int kk = k < K ? k : K - VEC;
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(b_src[it] + kk);
      rb[it] = k < K ? v : zero4;
    }
  };

  load_tile(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) *reinterpret_cast<u32x4_t*>(&As[a_lo[it]]) = ra[it];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) *reinterpret_cast<u32x4_t*>(&Bs[b_lo[it]]) = rb[it];
    __syncthreads();
    if (k0 + BK < K) load_tile(k0 + BK);   // in flight while the matrix cores work

    const int brow0 = SWIGLU ? (wn * 32 + (lane & 31)) : (wn * 64 + (lane & 31));
    const int brow1 = SWIGLU ? (64 + wn * 32 + (lane & 31)) : (wn * 64 + 32 + (lane & 31));
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 16) {
        const int ko = ks + (lane >> 5) * 8;
        const bf16x8_t fb0 = *reinterpret_cast<const bf16x8_t*>(&Bs[brow0 * LDK + ko]);
        const bf16x8_t fb1 = *reinterpret_cast<const bf16x8_t*>(&Bs[brow1 * LDK + ko]);
#pragma unroll
        for (int r = 0; r < MT; ++r) {
          if (live[r]) {
            const int arow = wm * 32 * MT + 32 * r + (lane & 31);
            const bf16x8_t fa = *reinterpret_cast<const bf16x8_t*>(&As[arow * LDK + ko]);
            acc[r][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb0, acc[r][0], 0, 0, 0);
            acc[r][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb1, acc[r][1], 0, 0, 0);
          }
        }
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 2) {
        const int ko = ks + (lane >> 5);
        const float fb0 = Bs[brow0 * LDK + ko];
        const float fb1 = Bs[brow1 * LDK + ko];
#pragma unroll
        for (int r = 0; r < MT; ++r) {
          if (live[r]) {
            const int arow = wm * 32 * MT + 32 * r + (lane & 31);
            const float fa = As[arow * LDK + ko];
            acc[r][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb0, acc[r][0], 0, 0, 0);
            acc[r][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb1, acc[r][1], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();
  }

  // epilogue: accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
  T* Cg = static_cast<T*>(P.C) + (shared ? (size_t)group * P.c_group_off : 0);
#pragma unroll
  for (int r = 0; r < MT; ++r) {
    if (!live[r]) continue;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wm * 32 * MT + 32 * r + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (row >= tile.rows) continue;
      T* crow = Cg + (size_t)(tile.row0 + row) * P.ldc;
      if (SWIGLU) {
        const int col = nt * 64 + wn * 32 + (lane & 31);
        if (col < N) crow[col] = from_f32<T>(silu_mul(acc[r][0][v], acc[r][1][v]));
      } else {
        const int col = nt * BNW + wn * 64 + (lane & 31);
        if (col < N) crow[col] = from_f32<T>(acc[r][0][v]);
        if (col + 32 < N) crow[col + 32] = from_f32<T>(acc[r][1][v]);
      }
    }
  }
}

__global__ __launch_bounds__(256) void build_tiles_kernel(const int32_t* __restrict__ expert_offsets,
                                                          int E, int row_cap, int n_cap,
                                                          const int32_t* __restrict__ n_dev,
                                                          int n_shared, fmoe_ffn_geom geom,
                                                          fmoe_tile* __restrict__ tiles1,
                                                          fmoe_tile* __restrict__ tiles2,
                                                          int32_t* __restrict__ counts) {
  __shared__ __align__(8) int scratch[513];
  fmoe_build_tiles(expert_offsets, E, row_cap, resolve_count(n_cap, n_dev), n_shared, geom.bm,
                   geom.tile_cap, geom.cols1, geom.scols1, tiles1, tiles2, counts, scratch);
}

inline int ks_steps(int K) { return ((K + SBK - 1) / SBK) * 2; }
// 16-byte units of one packed group: column blocks padded to tiles of four, 128 units per block and k step
inline size_t packed_units(int nbw, int ks) { return (size_t)((nbw + 3) / 4) * 4 * ks * 128; }

}  // namespace

fmoe_ffn_geom fmoe_geom(const fmoe_ctx* ctx, int n_cap) {
  const fmoe_config& c = ctx->cfg;
  fmoe_ffn_geom g;
  g.bm = (c.dtype == FMOE_BF16) ? SBM : 64;
  const int Ft = c.n_shared * c.d_ffn_shared;
  g.cols1 = (c.d_ffn + 63) / 64;           // 64 hidden columns per block
  g.scols1 = (Ft + 63) / 64;
  g.cols2 = (c.d_model + 127) / 128;       // 128 output columns per block
  g.scols2 = c.n_shared > 0 ? g.cols2 : 0;
  const int rep1 = (g.scols1 + g.cols1 - 1) / g.cols1;
  const int rep = rep1 > c.n_shared ? rep1 : (c.n_shared > 1 ? c.n_shared : 1);
  const long long rows = (long long)n_cap * (ctx->kmax > 0 ? ctx->kmax : 1);
  g.tile_cap = (int)(rows / g.bm) + c.n_experts + ((n_cap + g.bm - 1) / g.bm) * rep + 8;
  return g;
}

size_t fmoe_packed_bytes(const fmoe_ctx* ctx, int which) {
  const fmoe_config& c = ctx->cfg;
  if (c.dtype != FMOE_BF16) return 0;
  const size_t Ft = (size_t)c.n_shared * c.d_ffn_shared;
  switch (which) {
    case 0: return (size_t)c.n_experts * packed_units((c.d_ffn + 15) / 16, ks_steps(c.d_model)) * 16;
    case 1: return (size_t)c.n_experts * packed_units((c.d_model + 31) / 32, ks_steps(c.d_ffn)) * 16;
    case 2: return Ft ? packed_units(((int)Ft + 15) / 16, ks_steps(c.d_model)) * 16 : 0;
    case 3: return Ft ? (size_t)c.n_shared * packed_units((c.d_model + 31) / 32, ks_steps(c.d_ffn_shared)) * 16 : 0;
  }
  return 0;
}

int launch_pack_experts(fmoe_ctx* ctx, hipStream_t stream) {
  const fmoe_config& c = ctx->cfg;
  const int d = c.d_model, F = c.d_ffn, E = c.n_experts, Fs = c.d_ffn_shared;
  const int Ft = c.n_shared * Fs;
  auto grid = [](size_t bytes) { size_t b = bytes / 16 / 256 + 1; return (int)(b < 65536 ? b : 65536); };
  hipLaunchKernelGGL(pack_weights_kernel<true>, dim3(grid(fmoe_packed_bytes(ctx, 0))), dim3(256), 0, stream,
                     static_cast<const bf16_t*>(ctx->w_gate), static_cast<const bf16_t*>(ctx->w_up),
                     static_cast<u32x4_t*>(ctx->pk_gate_up), E, F, d, (F + 15) / 16, ks_steps(d));
  hipLaunchKernelGGL(pack_weights_kernel<false>, dim3(grid(fmoe_packed_bytes(ctx, 1))), dim3(256), 0, stream,
                     static_cast<const bf16_t*>(ctx->w_down), static_cast<const bf16_t*>(nullptr),
                     static_cast<u32x4_t*>(ctx->pk_down), E, d, F, (d + 31) / 32, ks_steps(F));
  if (Ft > 0) {
    hipLaunchKernelGGL(pack_weights_kernel<true>, dim3(grid(fmoe_packed_bytes(ctx, 2))), dim3(256), 0, stream,
                       static_cast<const bf16_t*>(ctx->ws_gate), static_cast<const bf16_t*>(ctx->ws_up),
                       static_cast<u32x4_t*>(ctx->pk_sgate_up), 1, Ft, d, (Ft + 15) / 16, ks_steps(d));
    hipLaunchKernelGGL(pack_weights_kernel<false>, dim3(grid(fmoe_packed_bytes(ctx, 3))), dim3(256), 0, stream,
                       static_cast<const bf16_t*>(ctx->ws_down), static_cast<const bf16_t*>(nullptr),
                       static_cast<u32x4_t*>(ctx->pk_sdown), c.n_shared, d, Fs, (d + 31) / 32, ks_steps(Fs));
  }
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

namespace {

int run_ffn_f32(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
                const int32_t* perm_src, void* y, void* y_shared, char* base, const fmoe_ws_layout& L,
                const fmoe_ffn_geom& geo, hipStream_t stream) {
  const fmoe_config& c = ctx->cfg;
  const int d = c.d_model, E = c.n_experts, F = c.d_ffn;
  const int Fs = c.d_ffn_shared, Ft = c.n_shared * Fs;
  int32_t* tile_count = reinterpret_cast<int32_t*>(base + L.tile_count);
  GemmArgs g1{}, g2{};
  g1.E = g2.E = E;
  g1.tiles = reinterpret_cast<fmoe_tile*>(base + L.tiles);
  g2.tiles = reinterpret_cast<fmoe_tile*>(base + L.tiles2);
  g1.n_tiles = tile_count;
  g2.n_tiles = tile_count + 1;
  {
    GemmProblem& p = g1.p0;
    p.A = x; p.lda = d; p.map1 = perm_src; p.map2 = kept_idx; p.map1_limit = n_cap;
    p.B0 = ctx->w_gate; p.B1 = ctx->w_up; p.group_stride = (long long)F * d; p.ldb = d;
    p.C = base + L.h; p.ldc = F; p.N = F; p.K = d; p.n_col_tiles = geo.cols1;
    GemmProblem& q = g1.p1;
    q = p;
    q.map1 = nullptr; q.map1_limit = 0;
    q.B0 = ctx->ws_gate; q.B1 = ctx->ws_up; q.group_stride = 0;
    q.C = base + L.h_shared; q.ldc = Ft; q.N = Ft; q.n_col_tiles = geo.scols1;
    g1.n_col_tiles_max = geo.cols1;
  }
  {
    GemmProblem& p = g2.p0;
    p.A = base + L.h; p.lda = F; p.map1 = nullptr; p.map2 = nullptr; p.map1_limit = 0;
    p.B0 = ctx->w_down; p.B1 = nullptr; p.group_stride = (long long)d * F; p.ldb = F;
    p.C = y; p.ldc = d; p.N = d; p.K = F; p.n_col_tiles = geo.cols2;
    GemmProblem& q = g2.p1;
    q = p;
    q.A = base + L.h_shared; q.lda = Ft; q.a_group_off = Fs;
    q.B0 = ctx->ws_down; q.group_stride = (long long)d * Fs; q.ldb = Fs;
    q.C = y_shared; q.c_group_off = (long long)n_cap * d; q.K = Fs; q.n_col_tiles = geo.scols2;
    g2.n_col_tiles_max = geo.cols2;
  }
  const unsigned batches = (unsigned)((geo.tile_cap + 7) / 8);
  {
    fmoe_prof_scope prof(ctx, SLOT_GEMM1, stream);
    hipLaunchKernelGGL((grouped_gemm_kernel<float, true, 1>), dim3(batches * 8 * g1.n_col_tiles_max),
                       dim3(256), 0, stream, g1);
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_GEMM2, stream);
    hipLaunchKernelGGL((grouped_gemm_kernel<float, false, 1>), dim3(batches * 8 * g2.n_col_tiles_max),
                       dim3(256), 0, stream, g2);
  }
  return FMOE_OK;
}

int run_ffn_bf16(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
                 const int32_t* perm_src, void* y, void* y_shared, char* base, const fmoe_ws_layout& L,
                 const fmoe_ffn_geom& geo, hipStream_t stream) {
  const fmoe_config& c = ctx->cfg;
  const int d = c.d_model, E = c.n_experts, F = c.d_ffn;
  const int Ft = c.n_shared * c.d_ffn_shared;
  // activation rows are addressed with 32-bit byte offsets
  if ((size_t)n_cap * ctx->kmax * F * 2 > 0xffffffffull || (size_t)n_cap * Ft * 2 > 0xffffffffull)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "expert FFN: a hidden buffer of %d rows exceeds 4 GiB", n_cap);
  int32_t* tile_count = reinterpret_cast<int32_t*>(base + L.tile_count);
  StreamArgs g1{}, g2{};
  g1.E = g2.E = E;
  g1.tiles = reinterpret_cast<fmoe_tile*>(base + L.tiles);
  g2.tiles = reinterpret_cast<fmoe_tile*>(base + L.tiles2);
  g1.n_tiles = tile_count;
  g2.n_tiles = tile_count + 1;
  g1.cols = g1.cols_entry = geo.cols1;
  g2.cols = g2.cols_entry = geo.cols2;
  // Shape of the kernel: the dense one when the rows this call can route average FMOE_DENSE_MIN_ROWS per
  // expert or more, else the weight-stream one; fmoe_set_ffn_shape overrides the rule.
  bool dense = (long long)n_cap * ctx->kmax >= (long long)FMOE_DENSE_MIN_ROWS * E;
  if (ctx->ffn_shape == 1) dense = false;
  if (ctx->ffn_shape == 2) dense = true;
  // the dense shape addresses the packed weights with 32-bit byte offsets
  for (int w = 0; w < 4; ++w)
    if (fmoe_packed_bytes(ctx, w) > 0xffffffffull) dense = false;
  if (dense) {
    g1.cols = (geo.cols1 + DNCB - 1) / DNCB;
    g2.cols = (geo.cols2 + DNCB - 1) / DNCB;
  }
  {
    StreamProblem& p = g1.p0;
    p.A = static_cast<const bf16_t*>(x); p.lda = d; p.map1 = perm_src; p.map2 = kept_idx; p.map1_limit = n_cap;
    p.Bp = static_cast<const u32x4_t*>(ctx->pk_gate_up);
    p.nbw = (F + 15) / 16; p.ks = ks_steps(d); p.group_stride = (long long)packed_units(p.nbw, p.ks);
    p.C = reinterpret_cast<bf16_t*>(base + L.h); p.ldc = F; p.N = F; p.K = d; p.n_col_tiles = geo.cols1;
    StreamProblem& q = g1.p1;
    q = p;
    q.map1 = nullptr; q.map1_limit = 0;
    q.Bp = static_cast<const u32x4_t*>(ctx->pk_sgate_up);
    q.nbw = (Ft + 15) / 16; q.group_stride = 0;
    q.C = reinterpret_cast<bf16_t*>(base + L.h_shared); q.ldc = Ft; q.N = Ft; q.n_col_tiles = geo.scols1;
  }
  {
    StreamProblem& p = g2.p0;
    p.A = reinterpret_cast<const bf16_t*>(base + L.h); p.lda = F; p.map1 = nullptr; p.map2 = nullptr; p.map1_limit = 0;
    p.Bp = static_cast<const u32x4_t*>(ctx->pk_down);
    p.nbw = (d + 31) / 32; p.ks = ks_steps(F); p.group_stride = (long long)packed_units(p.nbw, p.ks);
    p.C = static_cast<bf16_t*>(y); p.ldc = d; p.N = d; p.K = F; p.n_col_tiles = geo.cols2;
    StreamProblem& q = g2.p1;
    q = p;
    q.A = reinterpret_cast<const bf16_t*>(base + L.h_shared); q.lda = Ft; q.a_group_off = c.d_ffn_shared;
    q.Bp = static_cast<const u32x4_t*>(ctx->pk_sdown);
    q.ks = ks_steps(c.d_ffn_shared > 0 ? c.d_ffn_shared : 1); q.group_stride = (long long)packed_units(q.nbw, q.ks);
    q.C = static_cast<bf16_t*>(y_shared); q.c_group_off = (long long)n_cap * d; q.K = c.d_ffn_shared;
    q.n_col_tiles = geo.scols2;
  }
  const unsigned batches = (unsigned)((geo.tile_cap + 7) / 8);
  {
    fmoe_prof_scope prof(ctx, dense ? SLOT_GEMM1_DENSE : SLOT_GEMM1, stream);
    const unsigned items = batches * 8 * g1.cols;
    if (dense) hipLaunchKernelGGL((ffn_dense_kernel<true>), dim3(items), dim3(256), 0, stream, g1);
    else hipLaunchKernelGGL((ffn_stream_kernel<true>), dim3(items), dim3(256), 0, stream, g1);
  }
  {
    fmoe_prof_scope prof(ctx, dense ? SLOT_GEMM2_DENSE : SLOT_GEMM2, stream);
    const unsigned items = batches * 8 * g2.cols;
    if (dense) hipLaunchKernelGGL((ffn_dense_kernel<false>), dim3(items), dim3(256), 0, stream, g2);
    else hipLaunchKernelGGL((ffn_stream_kernel<false>), dim3(items), dim3(256), 0, stream, g2);
  }
  return FMOE_OK;
}

}  // namespace

int launch_expert_ffn(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
                      const int32_t* n_dev, const int32_t* expert_offsets, const int32_t* perm_src,
                      void* y, void* y_shared, void* ws, const fmoe_ws_layout& L, bool tiles_ready,
                      hipStream_t stream) {
  const fmoe_config& c = ctx->cfg;
  const bool has_shared = c.n_shared > 0;
  const int row_cap = n_cap * ctx->kmax;
  if (n_cap == 0 || (row_cap == 0 && !has_shared)) return FMOE_OK;
  char* base = static_cast<char*>(ws);
  const fmoe_ffn_geom geo = fmoe_geom(ctx, n_cap);
  if (!tiles_ready) {
    fmoe_prof_scope prof(ctx, SLOT_TILES, stream);
    hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(256), 0, stream, expert_offsets, c.n_experts,
                       row_cap, n_cap, n_dev, c.n_shared, geo,
                       reinterpret_cast<fmoe_tile*>(base + L.tiles),
                       reinterpret_cast<fmoe_tile*>(base + L.tiles2),
                       reinterpret_cast<int32_t*>(base + L.tile_count));
  }
  int rc;
  if (c.dtype == FMOE_BF16)
    rc = run_ffn_bf16(ctx, x, kept_idx, n_cap, perm_src, y, y_shared, base, L, geo, stream);
  else
    rc = run_ffn_f32(ctx, x, kept_idx, n_cap, perm_src, y, y_shared, base, L, geo, stream);
  if (rc != FMOE_OK) return rc;
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}
