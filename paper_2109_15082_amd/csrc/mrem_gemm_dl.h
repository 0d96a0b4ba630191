// Matrix-product kernel with operands moved global -> LDS by the direct-to-LDS load (no
// registers in between) ahead of the MFMAs.  Included by mrem_gemm.hip only.
//
//   C[M,N] = op(A) * op(B)^T with the fused epilogue
//   out = acc * (alpha * col_scale[n]) + beta * (col_vec[n] + row_vec[m]) + bias[n]  (optional GELU, bf16 or fp32 out).
//
// Block tile BM x BN x BK with BK = RB / 2 bf16 values (RB = bytes of k per tile row and stage,
// 64 or 128; int8 codes: RB values), WAVES_M x WAVES_N wavefronts, each owning
// (BM / WAVES_M) x (BN / WAVES_N) of 32 x 32 MFMA tiles.  Every wavefront both fetches and
// multiplies.  All STAGES slots of LDS are kept full: at the one s_barrier per k-step -- taken when
// a wavefront has issued its last fragment reads of stage kt and has seen its own loads of stage
// kt + 1 land (s_waitcnt vmcnt(n)) -- stage kt + 1 is handed over and the slot of stage kt is
// free again, so the loads of stage kt + STAGES go out right behind the barrier.  The MFMAs of the
// last k-substep of a stage are issued after the barrier, over the first fragment reads of the
// next stage; fragments are double-buffered per k-substep.  One direct load moves 1 KiB: lane l
// writes bytes [16 l, 16 l + 16) of the KiB and fetches whichever 16 bytes of the operand belong
// there under the swizzle.
//
// Fragment reads and their waits are inline assembly: the compiler orders a transposing LDS read
// after every direct load in flight (s_waitcnt vmcnt(0)), which would undo the prefetch, so the
// waits are placed by hand (lgkmcnt(0) between k-substeps, tied to the fragment registers).
//
// LDS layouts (rows unpadded, the direct load writes contiguously):
//   k-contiguous operand: tile [ROWS][RB bytes]; 16-byte chunk c of row r sits at slot
//     c ^ ((r >> 1) & 7) (RB = 128) or c ^ ((r >> 2) & 3) (RB = 64): the 16 rows that a group of
//     16 lanes reads fall on 16 distinct 16-byte bank groups of the 64 banks;
//   transposed operand (the contraction index is the slow one in memory): tile [RB / 2][ROWS] bf16;
//     16-byte chunk c of k-row k sits at slot c ^ ((k & 3) << 2) ^ (((k >> 3) & 1) << 1), so the
//     k-rows that one transposing read (ds_read_b64_tr_b16) gathers fall on distinct bank groups.
#pragma once

#include <utility>

namespace mrem {

typedef int i32x2_t __attribute__((ext_vector_type(2)));

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  // s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in
  // bits 15:14; expcnt and lgkmcnt left at "no wait")
  static_assert(N >= 0 && N < 64, "6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x0F70 | ((N >> 4) << 14));
}
template <int LPW, int MAXS>
__device__ __forceinline__ void wait_vmcnt_stages(int s) {
  // at most s * LPW loads may still be in flight, 0 <= s <= MAXS
  if constexpr (MAXS <= 0) { wait_vmcnt<0>(); }
  else {
    if (s >= MAXS) wait_vmcnt<LPW * MAXS>();
    else wait_vmcnt_stages<LPW, MAXS - 1>(s);
  }
}

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int OFF>
__device__ __forceinline__ i32x4_t lds_read_b128(int addr) {
  i32x4_t v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
__device__ __forceinline__ i32x2_t lds_read_tr16_b64(int addr) {
  i32x2_t v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

// One operand (ROWS tile rows) of the product.  T fragments of 32 rows each per wavefront.  KG: wavefront groups
// that share a stage's k-substeps (group g multiplies substeps g, g + KG, ...).
template <bool TR, int ROWS, int RB, int T, int KG = 1>
struct DlOperand {
  static constexpr int KK = RB / 32;               // k-substeps (one MFMA deep) per stage
  static constexpr int KKW = KK / KG;              // ... of them per wavefront
  static constexpr int BYTES = ROWS * RB;          // per stage
  static constexpr int LOADS = BYTES / 1024;       // direct loads (1 KiB each) per stage
  static constexpr int NADDR = TR ? T : KKW;       // per-lane LDS addresses kept in registers (per fragment / per k-substep)
  // byte offset, from the operand's first element of a k-step (row tile0, column k0), of the 16
  // bytes that belong at byte position p of the stage; ld in elements of 2 bytes
  static __device__ __forceinline__ size_t src_offset(int p, int ld) {
    if (TR) {
      const int k = p / (2 * ROWS), slot = (p % (2 * ROWS)) >> 4;
      const int c = slot ^ ((k & 3) << 2) ^ (((k >> 3) & 1) << 1);
      return ((size_t)k * ld + c * 8) * 2;
    }
    const int r = p / RB, slot = (p % RB) >> 4;
    const int c = slot ^ (RB == 128 ? (r >> 1) & 7 : (r >> 2) & 3);
    return ((size_t)r * ld + c * 8) * 2;
  }
  // per-lane byte addresses inside a stage for the fragments of the wavefront whose rows start at row0
  // (kg: this wavefront's group; its j-th substep is kg + KG j)
  static __device__ __forceinline__ void lane_addr(int (&a)[NADDR], int row0, int lane, int kg) {
    if constexpr (TR) {
      // the swizzle term is not additive in the fragment index: one address per fragment
      const int g = lane >> 4, s = lane & 15;
      const int krow = 8 * (g >> 1) + (s >> 2);
#pragma unroll
      for (int i = 0; i < T; ++i) {
        const int col = row0 + 32 * i + 16 * (g & 1) + 4 * (s & 3);
        const int slot = (col >> 3) ^ ((krow & 3) << 2) ^ (((krow >> 3) & 1) << 1);
        a[i] = (krow + 16 * kg) * (2 * ROWS) + slot * 16 + (col & 7) * 2;   // 16 k-rows per substep: the swizzle term is unchanged
      }
    } else {
      const int r = row0 + (lane & 31), x = RB == 128 ? (r >> 1) & 7 : (r >> 2) & 3;
#pragma unroll
      for (int j = 0; j < KKW; ++j) a[j] = r * RB + (((2 * (kg + KG * j) + (lane >> 5)) ^ x) << 4);
    }
  }
  // A fragment in registers: four VGPRs (one 16-byte read), or two pairs (two transposing 8-byte reads;
  // kept as separate asm outputs so that no copy is ever placed between a read and its wait)
  struct FragTr { i32x2_t lo, hi; };
  typedef typename std::conditional<TR, FragTr, i32x4_t>::type frag_t;
  static __device__ __forceinline__ i32x4_t regs(const frag_t& f) {
    if constexpr (TR) return i32x4_t{f.lo[0], f.lo[1], f.hi[0], f.hi[1]};
    else return f;
  }
  // after the wait: ties the registers of f to this point of the instruction stream
  static __device__ __forceinline__ void tie(frag_t (&f)[T]) {
#pragma unroll
    for (int i = 0; i < T; ++i) {
      if constexpr (TR) { asm volatile("" : "+v"(f[i].lo)); asm volatile("" : "+v"(f[i].hi)); }
      else asm volatile("" : "+v"(f[i]));
    }
  }
  // issue the reads of this wavefront's KKI-th k-substep of the stage at byte address `stage` (fragment i: rows + 32 i)
  template <int KKI>
  static __device__ __forceinline__ void read(frag_t (&f)[T], const int (&a)[NADDR], int stage) {
    if constexpr (TR) {
      // k-rows 16 KG KKI (+ 4 for the second half) further down: multiples of 4, the swizzle term is unchanged
      static_for<T>([&](auto i) {
        constexpr int off = KG * KKI * 16 * (2 * ROWS);
        const int addr = a[i.value] + stage;
        f[i.value].lo = lds_read_tr16_b64<off>(addr);
        f[i.value].hi = lds_read_tr16_b64<off + 4 * (2 * ROWS)>(addr);
      });
    } else {
      const int addr = a[KKI] + stage;
      static_for<T>([&](auto i) { f[i.value] = lds_read_b128<i.value * 32 * RB>(addr); });
    }
  }
};

// All LDS reads issued so far have returned; the fragment registers are tied in behind the wait so
// that their MFMAs stay behind it (volatile asm statements keep their order).
template <class OpA, class OpB, int TA, int TB>
__device__ __forceinline__ void wait_frags(typename OpA::frag_t (&a)[TA], typename OpB::frag_t (&b)[TB]) {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  OpA::tie(a);
  OpB::tie(b);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool AT, bool BT, int STAGES, int RB, class TO, bool I8, int MINB, int KG>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KG, MINB) void gemm_dl_k(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B,
                                                                         int ldb, TO* __restrict__ C, int ldc, int M, int N, int K, Epilogue e,
                                                                         int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_dl[];
  constexpr int NW = WAVES_M * WAVES_N * KG;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MT = WM / 32, NT = WN / 32;
  constexpr int BK = RB / 2;  // in 2-byte elements
  typedef DlOperand<AT, BM, RB, MT, KG> OpA;
  typedef DlOperand<BT, BN, RB, NT, KG> OpB;
  constexpr int KK = RB / 32 / KG;  // k-substeps of a stage that this wavefront multiplies
  static_assert((RB / 32) % KG == 0 && MT % KG == 0, "k-substeps and tile rows divide over the wavefront groups");
  constexpr int STAGE_BYTES = OpA::BYTES + OpB::BYTES;
  constexpr int LOADS = OpA::LOADS + OpB::LOADS;
  static_assert(LOADS % NW == 0, "loads of a stage divide evenly over the wavefronts");
  constexpr int LPW = LOADS / NW;  // direct loads per wavefront per stage
  static_assert(LPW * (STAGES - 1) < 64, "loads in flight must fit the 6-bit counter");
  static_assert(!I8 || (!AT && !BT), "int8 operands are read along k only");
  static_assert(STAGES >= 2, "double buffering at least");

  // Tile order: consecutive block ids land on different XCDs (8 of them, each with its own L2), so each XCD
  // gets a contiguous range of tiles, walked in groups of 8 tile rows so that concurrently running blocks
  // share operand panels in that L2.
  const int nblocks = tiles_m * tiles_n;
  int pid = blockIdx.x;
  if ((nblocks & 7) == 0) pid = (pid & 7) * (nblocks >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int group_sz = GROUP * tiles_n;
  const int g = pid / group_sz;
  const int first_m = g * GROUP;
  const int gm = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
  const int tm = first_m + (pid % group_sz) % gm;
  const int tn = (pid % group_sz) / gm;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave / (WAVES_M * WAVES_N), wpos = wave % (WAVES_M * WAVES_N);  // k-group, position in the tile
  const int wm = wpos / WAVES_N, wn = wpos % WAVES_N;

  const int KT = K / BK / (int)gridDim.y;  // gridDim.y > 1: k-slices, added into a zeroed fp32 C
  const int kbase = (int)blockIdx.y * KT * BK;

  // per-lane source addresses of this wavefront's loads for the next stage to fetch
  const unsigned char* src[LPW];
  const size_t adv_a = AT ? (size_t)BK * lda * 2 : RB, adv_b = BT ? (size_t)BK * ldb * 2 : RB;
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int gi = wave * LPW + i;  // load number within the stage: A's loads first, then B's
    if (gi < OpA::LOADS) {
      const unsigned char* base = reinterpret_cast<const unsigned char*>(AT ? A + (size_t)kbase * lda + m0 : A + (size_t)m0 * lda + kbase);
      src[i] = base + OpA::src_offset(gi * 1024 + lane * 16, lda);
    } else {
      const unsigned char* base = reinterpret_cast<const unsigned char*>(BT ? B + (size_t)kbase * ldb + n0 : B + (size_t)n0 * ldb + kbase);
      src[i] = base + OpB::src_offset((gi - OpA::LOADS) * 1024 + lane * 16, ldb);
    }
  }
  auto issue_range = [&](int stage_slot, auto first, auto count) {
    unsigned char* dst = smem_dl + stage_slot * STAGE_BYTES + wave * (LPW * 1024);
#pragma unroll
    for (int i = decltype(first)::value; i < decltype(first)::value + decltype(count)::value; ++i) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src[i],
                                       (__attribute__((address_space(3))) void*)(dst + i * 1024), 16, 0, 0);
      src[i] += (wave * LPW + i < OpA::LOADS) ? adv_a : adv_b;
    }
  };
  auto issue = [&](int stage_slot) { issue_range(stage_slot, std::integral_constant<int, 0>{}, std::integral_constant<int, LPW>{}); };
  // With three or more stages a stage's loads have k-steps to spare, and they go out in KK parts: the first right
  // behind the barrier, the others ahead of the following k-substeps, so the wavefronts of a SIMD do not queue up all
  // their loads at once while the matrix pipe waits.  (With two stages every load is needed one k-step later: all at once.)
  constexpr bool SPREAD = STAGES >= 3 && LPW % KK == 0;
  constexpr int LPP = SPREAD ? LPW / KK : LPW;
  bool pend = false;
  int pslot = 0;

  typedef typename std::conditional<I8, i32x16_t, f32x16_t>::type acc_t;
  acc_t acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  int a_addr[OpA::NADDR], b_addr[OpB::NADDR];
  OpA::lane_addr(a_addr, wm * WM, lane, kg);
  OpB::lane_addr(b_addr, wn * WN, lane, kg);
  const int lds0 = (int)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_dl;

  auto mfmas = [&](const typename OpA::frag_t (&af)[MT], const typename OpB::frag_t (&bf)[NT]) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if constexpr (I8) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(OpA::regs(af[i]), OpB::regs(bf[j]), acc[i][j], 0, 0, 0);
        else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, OpA::regs(af[i])), __builtin_bit_cast(bf16x8_t, OpB::regs(bf[j])), acc[i][j], 0, 0, 0);
      }
  };

  const int pre = KT < STAGES ? KT : STAGES;
  for (int s = 0; s < pre; ++s) issue(s);
  wait_vmcnt_stages<LPW, STAGES - 1>(pre - 1);
  __builtin_amdgcn_s_barrier();  // stage 0 has landed for everybody
  typename OpA::frag_t fa[2][MT];
  typename OpB::frag_t fb[2][NT];
  OpA::template read<0>(fa[0], a_addr, lds0);
  OpB::template read<0>(fb[0], b_addr, lds0 + OpA::BYTES);
  wait_frags<OpA, OpB>(fa[0], fb[0]);
  int slot = 0;
  for (int kt = 0; kt < KT; ++kt) {
    const int stage = lds0 + slot * STAGE_BYTES;
    // k-substeps 0 .. KK-2: fetch the fragments of the next substep, multiply the current one
    static_for<KK - 1>([&](auto kk) {
      constexpr int cur = kk.value & 1, nxt = cur ^ 1;
      if constexpr (SPREAD) {
        if (pend) issue_range(pslot, std::integral_constant<int, (kk.value + 1) * LPP>{}, std::integral_constant<int, LPP>{});
      }
      OpA::template read<kk.value + 1>(fa[nxt], a_addr, stage);
      OpB::template read<kk.value + 1>(fb[nxt], b_addr, stage + OpA::BYTES);
      __builtin_amdgcn_s_setprio(1);
      mfmas(fa[cur], fb[cur]);
      __builtin_amdgcn_s_setprio(0);
      wait_frags<OpA, OpB>(fa[nxt], fb[nxt]);
    });
    constexpr int last = (KK - 1) & 1;  // buffer of the last substep; the first substep of a stage uses buffer 0
    static_assert(KK % 2 == 0, "the fragment buffers alternate an even number of times per stage");
    const int next_slot = slot + 1 == STAGES ? 0 : slot + 1;
    if (kt + 1 < KT) {
      // every fragment read of stage kt has returned (wait_frags above).  Own loads of stage kt + 1 landed?
      const int beyond = KT - kt - 2;  // stages after kt + 1 that exist
      wait_vmcnt_stages<LPW, STAGES - 2>(beyond < STAGES - 2 ? beyond : STAGES - 2);
      __builtin_amdgcn_s_barrier();  // stage kt + 1 has landed for everybody; everybody is done reading stage kt
      pend = kt + STAGES < KT;
      pslot = slot;
      if (pend) issue_range(pslot, std::integral_constant<int, 0>{}, std::integral_constant<int, LPP>{});
      const int nstage = lds0 + next_slot * STAGE_BYTES;
      OpA::template read<0>(fa[last ^ 1], a_addr, nstage);
      OpB::template read<0>(fb[last ^ 1], b_addr, nstage + OpA::BYTES);
    }
    __builtin_amdgcn_s_setprio(1);
    mfmas(fa[last], fb[last]);
    __builtin_amdgcn_s_setprio(0);
    if (kt + 1 < KT) wait_frags<OpA, OpB>(fa[last ^ 1], fb[last ^ 1]);
    slot = next_slot;
  }

  if constexpr (KG > 1) {
    // The KG wavefronts at one tile position hold partial sums over disjoint k-substeps.  Each finalises the MFMA
    // tile rows i with i % KG == kg: it leaves its other tile rows in LDS (the stages are free now) and adds what
    // its partners left for its own rows, in group order (fixed, so results do not depend on timing).
    static_assert(KG == 2, "two groups");
    typedef typename std::conditional<I8, int, float>::type acc_e;
    acc_e* xch = reinterpret_cast<acc_e*>(smem_dl);
    __syncthreads();  // every wavefront is done reading operand stages
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      if (i % KG == kg) continue;
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) xch[(((wpos * MT + i) * NT + j) * 16 + r) * 64 + lane] = acc[i][j][r];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      if (i % KG != kg) continue;
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const acc_e other = xch[(((wpos * MT + i) * NT + j) * 16 + r) * 64 + lane];
          acc[i][j][r] = kg == 0 ? acc[i][j][r] + other : other + acc[i][j][r];  // always group 0's part first
        }
    }
  }

  // epilogue: out = acc * (alpha * col_scale[n]) + beta * (col_vec[n] + row_vec[m]) + bias[n]
  const float alpha = e.alpha ? *e.alpha : 1.f;
  const float beta = (e.beta ? *e.beta : 0.f) + e.beta_alpha * alpha;
  const bool split = gridDim.y > 1, lead = blockIdx.y == 0;
  auto write_out = [&](auto with_row, auto with_gelu, auto with_split) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n = n0 + wn * WN + j * 32 + (lane & 31);
      const float cs = alpha * (e.col_scale ? e.col_scale[n] : 1.f);
      float cb = (e.bias && lead) ? e.bias[n] : 0.f;
      if (e.beta && e.col_vec && lead) cb += beta * e.col_vec[n];
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        if (KG > 1 && i % KG != kg) continue;  // a partner wavefront writes this tile row
        const int mb = m0 + wm * WM + i * 32 + 4 * (lane >> 5);
        TO* __restrict__ out = C + (size_t)mb * ldc + n;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int dm = 8 * (r >> 2) + (r & 3);
          float v = (float)acc[i][j][r] * cs + cb;
          if constexpr (decltype(with_row)::value) v += beta * e.row_vec[mb + dm];
          if constexpr (decltype(with_split)::value) {
            atomicAdd(reinterpret_cast<float*>(out) + (size_t)dm * ldc, v);
          } else {
            if constexpr (decltype(with_gelu)::value) v = gelu_t<TO>(round_to<TO>(v));
            stf(out, (size_t)dm * ldc, v);
          }
        }
      }
    }
  };
  const bool row_term = e.beta && e.row_vec && lead;
  if constexpr (sizeof(TO) == 4) {
    if (split) {
      if (row_term) write_out(std::true_type{}, std::false_type{}, std::true_type{});
      else write_out(std::false_type{}, std::false_type{}, std::true_type{});
      return;
    }
  }
  if (e.gelu) {
    if (row_term) write_out(std::true_type{}, std::true_type{}, std::false_type{});
    else write_out(std::false_type{}, std::true_type{}, std::false_type{});
  } else {
    if (row_term) write_out(std::true_type{}, std::false_type{}, std::false_type{});
    else write_out(std::false_type{}, std::false_type{}, std::false_type{});
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool AT, bool BT, int STAGES, int RB, class TO, bool I8 = false, int MINB = 1, int KG = 1>
static void launch_dl(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                      hipStream_t st, int k_splits = 1) {
  constexpr int NTHREADS = 64 * WAVES_M * WAVES_N * KG;
  constexpr size_t lds = (size_t)STAGES * (BM + BN) * RB;
  static_assert(KG == 1 || (size_t)BM * BN * 4 <= lds, "the partial sums of a k-group fit the stages");
  static std::atomic<int> configured_dev{-1};
  int dev = -1;
  (void)hipGetDevice(&dev);
  if (dev != configured_dev.load()) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dl_k<BM, BN, WAVES_M, WAVES_N, AT, BT, STAGES, RB, TO, I8, MINB, KG>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured_dev.store(dev);
  }
  const int tiles_m = M / BM, tiles_n = N / BN;
  if (tl_launch_events.e0) {
    hipExtLaunchKernelGGL((gemm_dl_k<BM, BN, WAVES_M, WAVES_N, AT, BT, STAGES, RB, TO, I8, MINB, KG>), dim3(tiles_m * tiles_n, k_splits),
                          dim3(NTHREADS), lds, st, tl_launch_events.e0, tl_launch_events.e1, 0, (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (TO*)C, ldc, M, N,
                          K, e, tiles_m, tiles_n);
    return;
  }
  hipLaunchKernelGGL((gemm_dl_k<BM, BN, WAVES_M, WAVES_N, AT, BT, STAGES, RB, TO, I8, MINB, KG>), dim3(tiles_m * tiles_n, k_splits), dim3(NTHREADS),
                     lds, st, (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (TO*)C, ldc, M, N, K, e, tiles_m, tiles_n);
}

}  // namespace mrem
