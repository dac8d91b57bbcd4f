// Kernels, launch tables and the C ABI of the Collage optimizer step for gfx950.
//
// Work decomposition.  A tensor is cut into SLOTS of 16 bytes per stream (8 consecutive bf16 or fp16
// elements, 16 FP8 elements) counted from the 128-byte boundary at or below its first element, so that a
// slot is one 128-bit access per stream whatever the tensor's own alignment and every
// wave's 1 KiB run covers whole cache lines (counting from the 16-byte boundary instead, waves of
// neighbouring workgroups share lines: a set of tensors at odd offsets ran at 5.2 instead of 5.8 TB/s); the slots
// that straddle the ends of the tensor are gathered and scattered element by element (and computed by the same
// vector arithmetic as the others).  A CHUNK is
// kStepBlock*kUnroll consecutive slots of one tensor, done by one workgroup; lane l takes
// slots l, l+kStepBlock, ... so each wave's access is one contiguous 1 KiB run per stream.
// The chunk table {tensor, first slot} and the tensor descriptors live in device memory
// and are wave-uniform, so they arrive through scalar loads into SGPRs; any number of
// tensors of any size is one launch.
//
// Launch shape, from sweeps on MI355X at the 7B-parameter set (9 to 11 concurrent streams
// of 13.5 GB each): one-wave workgroups with one slot per lane, about 10 of them resident per CU,
// and non-temporal loads and stores.  Short-lived single-wave groups keep the set of
// addresses in flight compact, and capping the waves in flight keeps the HBM channels
// from thrashing between too many open rows: 256-thread groups with two slots per lane at
// full occupancy reached 5.5 TB/s, this shape 6.5-6.6 TB/s on the same device in the same run.
// The cap is set by giving every workgroup dynamic LDS it never touches: unlike a waves-per-SIMD
// bound it counts per CU and can sit between multiples of four.  Caps that differ by less than
// 1280 bytes time identically, so the 160 KiB of a CU appear to be handed out in 128 granules of
// 1280 bytes; lds_for_groups() below asks for the largest whole number of granules that still lets
// the wanted number of groups fit (light, 7B set: 8 groups 19.85 ms, 9: 18.76, 10: 18.50, 11: 18.80,
// 12: 18.98, 14: 19.15, 16: 19.52, no cap: 20.32).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/mcf.h"
#include "mcf_host.h"
#include "mcf_math.h"

namespace {

using mcfd::ElemIOT;
using mcfd::P2;
using mcfd::StepScalars;
using mcfd::StepScalarsH;
using mcfd::StepScalarsF8;
using mcfd::StepScalarsT;

// Compile-time tuning knobs of the step kernels (defaults = the measured best, see above).
#ifndef MCF_BLOCK
#define MCF_BLOCK 64                 // threads per workgroup of the step kernels
#endif
#ifndef MCF_UNROLL
#define MCF_UNROLL 1                 // slots per lane
#endif
#ifndef MCF_NT_LOAD
#define MCF_NT_LOAD 1                // non-temporal 128-bit loads
#endif
#ifndef MCF_NT_STORE
#define MCF_NT_STORE 1               // non-temporal 128-bit stores
#endif
#ifndef MCF_REMAP
#define MCF_REMAP 0                  // 1: give each XCD (blocks are dealt round-robin to the 8 XCDs) a contiguous run of chunks
#endif
#ifndef MCF_PERSIST
#define MCF_PERSIST 0                // 1: fixed grid of workgroups that walk the chunk table; 2: MCF_RUN consecutive chunks per workgroup (see adamw_kernel)
#endif
#ifndef MCF_DEPTH
#define MCF_DEPTH 1                  // MCF_PERSIST: chunks whose loads are issued ahead of the one being computed (0 or 1)
#endif
#ifndef MCF_RUN
#define MCF_RUN 4                    // MCF_PERSIST 2: consecutive chunks per workgroup
#endif
#ifndef MCF_WAVES_PER_CU
#define MCF_WAVES_PER_CU 8           // MCF_PERSIST: workgroups of the fixed grid per compute unit
#endif
#ifndef MCF_CHUNK_ALIGN
#define MCF_CHUNK_ALIGN 128          // bytes: a tensor's slots are counted from this address boundary below its first element
#endif
#ifndef MCF_STEP_ATTR
#define MCF_STEP_ATTR                // optional extra attribute of the step kernels (e.g. amdgpu_waves_per_eu)
#endif
// MCF_STEP_LDS, if defined, is the bytes of untouched dynamic LDS per workgroup (= the occupancy cap) of
// every step kernel; by default the cap is per variant, see StepStreams::kLds.
// Dynamic LDS that lets `groups` workgroups share a CU: 128/groups granules, less 256 bytes of room for a
// kernel's own static LDS (the EDQ kernels keep 24 bytes).
constexpr uint32_t lds_for_groups(uint32_t groups) { return (128u / groups) * 1280u - 256u; }
#ifndef MCF_STEP_LDS_EDQ
#define MCF_STEP_LDS_EDQ 0           // 0: per variant (StepStreams::kLdsEdq); else bytes for every EDQ-fused step kernel
#endif
#ifndef MCF_FP32MW_LDS
#define MCF_FP32MW_LDS lds_for_groups(10)   // fp32-master baseline kernel: 9 groups 29.15 ms, 10: 29.14, 11: 29.38, 12: 29.72, 14: 30.40
#endif
#ifndef MCF_FP32MW_STORE
#define MCF_FP32MW_STORE ST_AGENT_NT // StorePolicy of the fp32-master baseline kernel (10 groups: 29.14 ms; ST_AGENT 29.22; ST_NT 29.75)
#endif
#ifndef MCF_COPY_LDS
#define MCF_COPY_LDS 0               // the plain copy (2 streams) is fastest uncapped: 6.66 TB/s against 4.4 TB/s with the cap
#endif
constexpr int kStepBlock = MCF_BLOCK;
constexpr int kUnroll = MCF_UNROLL;
constexpr uint32_t kSlotsPerChunk = kStepBlock * kUnroll;
constexpr int kBlock = 256;          // threads per workgroup of the primitives and reduction tails
constexpr uint64_t kMaxTensorElems = (1ull << 35) - (MCF_CHUNK_ALIGN > 128 ? MCF_CHUNK_ALIGN : 128);   // keeps a tensor's slot count, phase included, below 2^32
constexpr int kMaxStreams = 6;

// Streams of the Collage step, in descriptor order.
enum { S_TH = 0, S_DTH = 1, S_M = 2, S_V = 3, S_G = 4, S_DV = 5 };

struct TensorDesc {
  uint64_t p[kMaxStreams];   // the streams' device addresses, as integers
  uint64_t n;                // elements
  uint32_t phase;            // elements between the MCF_CHUNK_ALIGN-byte boundary below p[0] and p[0]
  uint32_t skewed;           // 1: the streams do not share theta's offset modulo 16 bytes (their 128-bit accesses are unaligned)
};
static_assert(sizeof(TensorDesc) == 64, "descriptor is one 64-byte scalar load");

struct Chunk {
  uint32_t tensor;
  uint32_t slot0;     // first slot of the chunk within its tensor (plan creation refuses a tensor with 2^32 slots or more)
};

struct Slot {       // where one lane's 16 bytes of elements sit
  uint64_t c0;      // aligned coordinate of the first element (multiple of the elements per slot)
  bool any, full;
};

// EB = bytes per element (2: bf16, fp16; 1: FP8); a slot holds 16/EB elements.
template <int EB>
__device__ __forceinline__ Slot classify(const TensorDesc &d, uint64_t slot) {
  constexpr uint64_t kEps = 16 / EB;
  Slot s;
  s.c0 = slot * kEps;
  const uint64_t lo = d.phase, hi = d.phase + d.n;
  s.any = (s.c0 + kEps > lo) && (s.c0 < hi);
  s.full = (s.c0 >= lo) && (s.c0 + kEps <= hi);
  return s;
}

// 128-bit access to the 16 bytes at byte offset `off` of the buffer at p.
// The pointers are device-memory addresses, so the accesses are typed as global (address
// space 1): global_load/global_store instead of the generic flat instructions.
// Slots are cut on theta's 16-byte grid.  A stream whose buffer sits at another offset modulo 16 is
// accessed at addresses that are only element-aligned: the vector type says so (alignment 1), the
// compiler emits the same global_load/store_dwordx4 for it (global memory takes unaligned accesses on
// this target), and the hardware splits an access that straddles a line.  That costs bandwidth on the
// skewed streams only; the alternative, element by element, costs a factor of three on everything.
#define MCF_GLOBAL __attribute__((address_space(1)))
typedef uint32_t u32x4_aligned_t __attribute__((ext_vector_type(4)));
typedef u32x4_aligned_t u32x4_t __attribute__((aligned(1)));
template <class T> __device__ __forceinline__ MCF_GLOBAL T *gptr(uint64_t p) { return (MCF_GLOBAL T *)p; }

__device__ __forceinline__ void load_vec(uint64_t p, uint64_t off, uint32_t (&w)[4]) {
#if MCF_NT_LOAD
  const u32x4_t q = __builtin_nontemporal_load(gptr<const u32x4_t>(p + off));
#else
  const u32x4_t q = *gptr<const u32x4_t>(p + off);
#endif
  w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
}
// How a 128-bit store is marked for the caches.  ST_NT: non-temporal.  ST_AGENT: agent scope -- the data is
// written through to memory instead of waiting in the XCD's L2 for an eviction; ST_AGENT_NT: both.  Measured at the
// 7B set, each kernel at its best cap, same process: light 18.53 ms with ST_NT, 18.17 with ST_AGENT_NT, 17.94 with
// ST_AGENT; plus 23.10 / 22.73 / 22.34; SGD 14.16 / 14.05 / 13.82; the kernels with the fp64 EDQ sums fused in prefer
// ST_AGENT_NT (light 18.70 against 19.23 with ST_AGENT), the ALU-bound FP8 kernels ST_NT (9.80 against 9.99).  In an
// arithmetic-free 5-read/4-write probe every combination of sc0, sc1 and nt on the loads leaves the rate where it is;
// on the stores, any with sc1 gives 6.81-6.83 TB/s against 6.63 for nt alone and 5.7-6.3 for none or sc0.
// That holds where the streams are far larger than the caches.  At small sets the write-through costs: the 64Mi stress
// set (128 MB per stream) takes 0.261 ms with ST_AGENT against 0.241 with ST_NT, the 125M set is level (0.418 / 0.423),
// the 1.3B set (2.6 GB per stream) gains 2.4% like the 7B set.  So the host picks per launch: write-through policies
// from kWriteThroughBytes per stream on, ST_NT below.
enum StorePolicy { ST_NT = 0, ST_AGENT = 1, ST_AGENT_NT = 2, ST_PLAIN = 3 };
constexpr uint64_t kWriteThroughBytes = 512ull << 20;
#ifndef MCF_STORE_POLICY
#define MCF_STORE_POLICY -1          // -1: per kernel (see finish_chunk); else one StorePolicy for every step kernel
#endif

// The scope bits have no builtin, so those stores are written as the instruction.  The s_nop keeps the two wait
// states this target wants between a store of more than 64 bits and a write to its data registers: the compiler's
// hazard pass provides them for instructions it knows and cannot for this one.
template <int POLICY = (MCF_NT_STORE ? ST_NT : ST_PLAIN)>
__device__ __forceinline__ void store_vec(uint64_t p, uint64_t off, const uint32_t (&w)[4]) {
  const u32x4_t q = {w[0], w[1], w[2], w[3]};
  if constexpr (POLICY == ST_AGENT) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p + off), "v"(q) : "memory");
  } else if constexpr (POLICY == ST_AGENT_NT) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p + off), "v"(q) : "memory");
  } else if constexpr (POLICY == ST_NT) {
    __builtin_nontemporal_store(q, gptr<u32x4_t>(p + off));
  } else {
    *gptr<u32x4_t>(p + off) = q;
  }
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4_t load_f4(const MCF_GLOBAL float *p) {
#if MCF_NT_LOAD
  return __builtin_nontemporal_load((const MCF_GLOBAL f32x4_t *)p);
#else
  return *(const MCF_GLOBAL f32x4_t *)p;
#endif
}
template <int POLICY>
__device__ __forceinline__ void store_f4(MCF_GLOBAL float *p, f32x4_t q) {
  const uint64_t at = (uint64_t)p;
  if constexpr (POLICY == ST_AGENT) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(at), "v"(q) : "memory");
  } else if constexpr (POLICY == ST_AGENT_NT) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(at), "v"(q) : "memory");
  } else if constexpr (POLICY == ST_NT) {
    __builtin_nontemporal_store(q, (MCF_GLOBAL f32x4_t *)p);
  } else {
    *(MCF_GLOBAL f32x4_t *)p = q;
  }
}

// One element of EB bytes.
template <int EB> __device__ __forceinline__ uint32_t load_elem(uint64_t p, uint64_t e) {
  if constexpr (EB == 1) return gptr<const uint8_t>(p)[e]; else return gptr<const uint16_t>(p)[e];
}
template <int EB> __device__ __forceinline__ void store_elem(uint64_t p, uint64_t e, uint32_t bits) {
  if constexpr (EB == 1) gptr<uint8_t>(p)[e] = (uint8_t)bits; else gptr<uint16_t>(p)[e] = (uint16_t)bits;
}

// Load the slot of stream `p` as 4 dwords (4/EB elements each); elements outside the tensor read as 0.
template <int EB>
__device__ __forceinline__ void load_slot(uint64_t p, const TensorDesc &d, const Slot &s, uint32_t (&w)[4]) {
  if (s.full) {
    load_vec(p, (s.c0 - d.phase) * EB, w);
  } else {
    // Every element of the slot is loaded without a branch -- those outside the tensor from element 0, which always
    // exists, and then zeroed -- so that all loads of the slot are in flight together (one memory latency, not sixteen).
    constexpr int kPer = 4 / EB;        // elements per dword
    const uint64_t lo = d.phase, hi = d.phase + d.n;
    uint32_t e[16 / EB];
#pragma unroll
    for (int k = 0; k < 16 / EB; ++k) {
      const uint64_t c = s.c0 + k;
      const bool inside = c >= lo && c < hi;
      e[k] = load_elem<EB>(p, inside ? c - lo : 0);
      e[k] = inside ? e[k] : 0u;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      uint32_t word = 0;
#pragma unroll
      for (int j = 0; j < kPer; ++j) word |= e[kPer * k + j] << (8 * EB * j);
      w[k] = word;
    }
  }
}

template <int EB>
__device__ __forceinline__ void store_slot(uint64_t p, const TensorDesc &d, const Slot &s, const uint32_t (&w)[4]) {
  if (s.full) {
    store_vec(p, (s.c0 - d.phase) * EB, w);
  } else {
    constexpr int kPer = 4 / EB;
    const uint64_t lo = d.phase, hi = d.phase + d.n;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
      for (int j = 0; j < kPer; ++j) {
        const uint64_t c = s.c0 + kPer * k + j;
        if (c >= lo && c < hi) store_elem<EB>(p, c - lo, (w[k] >> (8 * EB * j)) & (EB == 1 ? 0xffu : 0xffffu));
      }
    }
  }
}

// ---------------------------------------------------------------- wave and block sums
// Sum over the 64 lanes with DPP row operations, fixed order, result in every lane of
// each 16-lane row; the four row sums are then read with v_readlane and added in order.
template <int CTRL>
__device__ __forceinline__ double dpp_add(double x) {
  const int xl = __double2loint(x), xh = __double2hiint(x);
  const int yl = __builtin_amdgcn_update_dpp(0, xl, CTRL, 0xF, 0xF, false);
  const int yh = __builtin_amdgcn_update_dpp(0, xh, CTRL, 0xF, 0xF, false);
  return x + __hiloint2double(yh, yl);
}

__device__ __forceinline__ double wave_sum(double x) {
  x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);   // row_half_mirror
  x = dpp_add<0x140>(x);   // row_mirror
  const int xl = __double2loint(x), xh = __double2hiint(x);
  double r0 = __hiloint2double(__builtin_amdgcn_readlane(xh, 0), __builtin_amdgcn_readlane(xl, 0));
  double r1 = __hiloint2double(__builtin_amdgcn_readlane(xh, 16), __builtin_amdgcn_readlane(xl, 16));
  double r2 = __hiloint2double(__builtin_amdgcn_readlane(xh, 32), __builtin_amdgcn_readlane(xl, 32));
  double r3 = __hiloint2double(__builtin_amdgcn_readlane(xh, 48), __builtin_amdgcn_readlane(xl, 48));
  return ((r0 + r1) + r2) + r3;
}

// Sum of (a, b, c) over the workgroup; valid in thread 0.  All threads must call.
template <int THREADS = kBlock>
__device__ __forceinline__ void block_sum3(double &a, double &b, double &c) {
  __shared__ double sh[3 * (THREADS / 64)];
  a = wave_sum(a);
  b = wave_sum(b);
  c = wave_sum(c);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sh[3 * wave] = a; sh[3 * wave + 1] = b; sh[3 * wave + 2] = c; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double sa = sh[0], sb = sh[1], sc = sh[2];
    for (int w = 1; w < THREADS / 64; ++w) { sa += sh[3 * w]; sb += sh[3 * w + 1]; sc += sh[3 * w + 2]; }
    a = sa; b = sb; c = sc;
  }
}

// Compile-time loop: f(integral_constant<int, J>) for J = LO .. HI-1.
template <int LO, int HI, class F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (LO < HI) {
    f(std::integral_constant<int, LO>{});
    static_for<LO + 1, HI>(f);
  }
}

// ---------------------------------------------------------------- effective descent quality
// Per-lane totals of Def. 3.3: s1 = sum delta*effective, s2 = sum delta^2, and the number of lost
// updates (Def. 3.2: delta != 0 but the value did not change).  The effective update is taken on
// the value theta+dtheta (Eq. 2 when there is no second component), in fp64 so that "did not
// change" is decided exactly.
struct EdqAcc {
  double s1, s2;
  uint32_t lost;
};

__device__ __forceinline__ void edq_add(EdqAcc &a, float delta, float th0, float dth0, float th1, float dth1) {
  const double d = (double)delta;
  const double eff = ((double)th1 + (double)dth1) - ((double)th0 + (double)dth0);
  a.s1 = __builtin_fma(d, eff, a.s1);
  a.s2 = __builtin_fma(d, d, a.s2);
  a.lost += (d != 0.0 && eff == 0.0) ? 1u : 0u;
}

constexpr int kEdqVals = 3;              // doubles per partial: s1, s2, lost

// One partial per workgroup.  All threads must call.
template <int THREADS>
__device__ __forceinline__ void edq_store_partial(const EdqAcc &a, double *__restrict__ partials, uint64_t index) {
  double s1 = a.s1, s2 = a.s2, lost = (double)a.lost;
  block_sum3<THREADS>(s1, s2, lost);
  if (threadIdx.x == 0) {
    partials[kEdqVals * index] = s1;
    partials[kEdqVals * index + 1] = s2;
    partials[kEdqVals * index + 2] = lost;
  }
}

// ---------------------------------------------------------------- the step kernel
// VARIANT template arguments below carry the variant in the low byte, kGrow2Bit when every Grow
// is to be built on TwoSum (Alg. 3) instead of Fast2Sum, and the component format (mcf_component) in
// bits 12-13, as in the C ABI's variant argument.
constexpr int kGrow2Bit = 0x100;
constexpr int kFmtShift = 12;
constexpr int kHalfBit = MCF_COMPONENT_FP16 << kFmtShift;

// Arithmetic modes of a component format.  Hot: the first pass over a full slot (FAST selects between the two
// bf16 modes); it may give a slot up.  Second: the pass that is right for every slot -- those the first pass
// gave up, those at a tensor's ends, and every slot of a launch whose scalars the first pass cannot take; it
// stores the format's one NaN pattern.  Cold: the mode single operations fall back to (bf16: IEEE divide and root).
template <int FMT, bool FAST> struct ModeOf;
template <bool FAST> struct ModeOf<MCF_COMPONENT_BF16, FAST> {
  using Hot = typename std::conditional<FAST, mcfd::Fast, mcfd::Exact>::type;
  using Second = typename std::conditional<FAST, mcfd::FastSecond, mcfd::Exact>::type;
  using Cold = mcfd::Exact;
};
template <bool FAST> struct ModeOf<MCF_COMPONENT_FP16, FAST> { using Hot = mcfd::HalfHot; using Second = mcfd::HalfCold; using Cold = mcfd::HalfCold; };
template <bool FAST> struct ModeOf<MCF_COMPONENT_FP8_E5M2, FAST> {
  using Hot = mcfd::F8<false, true>; using Second = mcfd::F8<false, false>; using Cold = mcfd::F8<false, false>;
};
template <bool FAST> struct ModeOf<MCF_COMPONENT_FP8_E4M3, FAST> {
  using Hot = mcfd::F8<true, true>; using Second = mcfd::F8<true, false>; using Cold = mcfd::F8<true, false>;
};
template <int VARIANT> struct StepStreams {
  static constexpr int kBase = VARIANT & 0xff;
  static constexpr bool kGrow2 = (VARIANT & kGrow2Bit) != 0;
  static constexpr int kFmt = (VARIANT >> kFmtShift) & 3;
  static constexpr bool kBf16 = kFmt == MCF_COMPONENT_BF16;
  template <bool FAST> using Hot = typename ModeOf<kFmt, FAST>::Hot;
  template <bool FAST> using Second = typename ModeOf<kFmt, FAST>::Second;
  using Cold = typename ModeOf<kFmt, true>::Cold;
  using Scalars = StepScalarsT<typename Cold::S, typename Cold::Rcp>;
  static constexpr int kEB = Cold::kBytes;                 // bytes per element
  static constexpr int kEps = 16 / kEB;                    // elements per slot
  static constexpr bool kDth = kBase != mcfd::V_BF16;      // second component of theta / Kahan variable
  static constexpr bool kDv = kBase == mcfd::V_PLUS;       // second component of v
  static constexpr bool kV = kBase != mcfd::V_SGD;         // second moment
  // Occupancy cap in workgroups per CU, from sweeps of 7..20 at the 7B-parameter set, all settings of a
  // kernel timed in one process on the same arenas (two processes differ by more than two neighbouring caps
  // do: where the allocator puts 80 GB matters at the 1-3% level).  ms per step, best cap first, with the store
  // policy each kernel uses (see StorePolicy):
  //   light 11: 17.96 (10: 18.27, 12: 18.71, 9: 18.95)       Kahan 10: 18.11 (11: 18.22, 9: 18.69, 12: 18.73)
  //   plus  10: 22.34 (9: 22.88, 11: 23.02, 12: 23.54)       plus, fp16 components 10: 22.14 (9: 22.35, 11: 23.10)
  //   plain bf16 12: 14.05 (13: 14.36, 11: 14.50)            SGD 12: 13.82 (11: 14.10, 13: 14.44)
  //   light on TwoSum 12: 18.04 (11: 18.21, 10: 18.69)       plus on TwoSum 12: 23.29 (11: 23.38, 13: 23.48)
  //   light, fp16 components 11: 18.08 (12: 18.39, 10: 18.47)
  // The plain variant and SGD have less memory time per wave to hide their divide and root behind and take
  // more waves.  The optimum moves with a kernel's instruction schedule, so the table is re-measured when the
  // arithmetic or the kernel's structure changes (mcf_set_launch_pacing does that without rebuilding).
  // With the fp64 EDQ sums fused in there is more arithmetic per wave: light 16: 18.65 (13-14: 18.82, 12: 19.40, 18: 19.21);
  // plus 16: 23.40 (14: 23.44, 13: 23.46); Kahan 13: 18.40; plain bf16 18: 14.34 (16: 14.65); SGD 16: 14.22
  // (18: 14.29, 14: 14.67); light on TwoSum 16-18: 19.35; plus on TwoSum 20: 25.42 (18: 25.60); light with fp16
  // components 16: 19.37; plus with fp16 components 14: 23.05.
  // The FP8 kernels move half the bytes with about the same arithmetic (a conversion to and from the
  // 8-bit format around every operation): they are bound by vector-ALU issue and run uncapped (light E5M2,
  // 7B set: 9.80 ms uncapped, 10.06-10.54 at 12 to 14 groups per CU).
#ifdef MCF_STEP_LDS
  static constexpr uint32_t kLds = MCF_STEP_LDS;
#else
  static constexpr int kGroups = (kBase == mcfd::V_BF16 || kBase == mcfd::V_SGD || kGrow2) ? 12 : (kBase == mcfd::V_PLUS || kBase == mcfd::V_KAHAN) ? 10 : 11;
  static constexpr uint32_t kLds = (kEB == 1 || MCF_PERSIST == 1) ? 0 : lds_for_groups(kGroups);
#endif
  static constexpr int kEdqGroups = kBase == mcfd::V_BF16 ? 18 : kBase == mcfd::V_KAHAN ? 13
                                    : kBase == mcfd::V_PLUS ? (kGrow2 ? 20 : kBf16 ? 16 : 14) : 16;
  static constexpr uint32_t kLdsEdq = MCF_STEP_LDS_EDQ ? MCF_STEP_LDS_EDQ : (kEB == 1 || MCF_PERSIST == 1) ? 0 : lds_for_groups(kEdqGroups);
};

// A dword of a stream holds one pair (2-byte elements) or two pairs (1-byte elements).
template <class M, int PAIR> __device__ __forceinline__ typename M::T unpack_pair(uint32_t w) {
  if constexpr (M::kBytes == 1) return M::template unpack<PAIR>(w); else return M::unpack(w);
}
template <class M, int N> __device__ __forceinline__ uint32_t pack_pairs(const typename M::T (&x)[N]) {
  if constexpr (M::kBytes == 1) return M::pack(x[0], x[1]); else return M::pack(x[0]);
}

// One slot, 16 bytes of every stream held as 4 dwords each, through the chain in arithmetic mode M.  Returns
// true when the mode gives the slot up (first-pass modes only): it is then computed again in the variant's
// second mode.  EPS_INSIDE: line 12 with epsilon under the root.  MASKED: bit e of `valid` says whether element e
// of the slot belongs to the tensor; the others were loaded as zeros, are computed along and not stored, and
// must stay out of the EDQ sums.
template <class M, int VARIANT, bool EDQ, bool EPS_INSIDE = false, bool MASKED = false>
__device__ __forceinline__ bool hot_slot(const uint32_t (&in)[kMaxStreams][4], uint32_t (&out)[kMaxStreams][4],
                                         const StepScalarsT<typename M::S, typename M::Rcp> &sc, EdqAcc &acc, uint32_t valid = ~0u) {
  using SS = StepStreams<VARIANT>;
  using T = typename M::T;
  constexpr int kPairs = M::kBytes == 1 ? 2 : 1;
  bool redo = false;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    T th[kPairs], dth[kPairs], m[kPairs], v[kPairs], dv[kPairs];
    static_for<0, kPairs>([&](auto pc) {
      constexpr int P = decltype(pc)::value;
      ElemIOT<T> io;
      io.th = unpack_pair<M, P>(in[S_TH][k]);
      if (SS::kDth) io.dth = unpack_pair<M, P>(in[S_DTH][k]); else io.dth = M::zero();
      io.m = unpack_pair<M, P>(in[S_M][k]);
      if (SS::kV) io.v = unpack_pair<M, P>(in[S_V][k]); else io.v = M::zero();
      io.g = unpack_pair<M, P>(in[S_G][k]);
      if (SS::kDv) io.dv = unpack_pair<M, P>(in[S_DV][k]); else io.dv = M::zero();
      const T th0 = io.th, dth0 = io.dth;
      T delta;
      mcfd::adamw_pair<M, SS::kBase, SS::kGrow2, EPS_INSIDE && SS::kBase != mcfd::V_SGD>(io, sc, delta, redo);
      th[P] = io.th; dth[P] = io.dth; m[P] = io.m; v[P] = io.v; dv[P] = io.dv;
      if (EDQ) {
        const int e = 2 * (kPairs * k + P);          // the pair's first element within the slot
        if (!MASKED || ((valid >> e) & 1u)) edq_add(acc, M::lo(delta), M::lo(th0), M::lo(dth0), M::lo(io.th), M::lo(io.dth));
        if (!MASKED || ((valid >> (e + 1)) & 1u)) edq_add(acc, M::hi(delta), M::hi(th0), M::hi(dth0), M::hi(io.th), M::hi(io.dth));
      }
    });
    out[S_TH][k] = pack_pairs<M>(th);
    if (SS::kDth) out[S_DTH][k] = pack_pairs<M>(dth);
    out[S_M][k] = pack_pairs<M>(m);
    if (SS::kV) out[S_V][k] = pack_pairs<M>(v);
    if (SS::kDv) out[S_DV][k] = pack_pairs<M>(dv);
    if constexpr (M::kFast && M::kNanOnWords) {
      // Any NaN produced or consumed by the chain reaches theta', and a NaN in theta' makes the second component NaN
      // as well (it is computed from theta' - u), so where there is a second component that is the one to look at:
      // it also catches the NaN that inf - inf leaves there when theta' itself is an infinity.  Likewise for (v', dv').
      if (SS::kDth) redo |= M::word_has_nan(out[S_DTH][k]); else redo |= M::word_has_nan(out[S_TH][k]);
      if (SS::kDv) redo |= M::word_has_nan(out[S_DV][k]);
    }
  }
  return redo;
}

// One chunk in flight: where it is and the 16 bytes per stream and slot that its loads bring in.
template <int VARIANT> struct ChunkIn {
  TensorDesc d;                               // wave-uniform (SGPRs)
  uint64_t slot0;
  Slot slot[kUnroll];
  uint32_t in[kUnroll][kMaxStreams][4];
};

// Issues every 128-bit load of chunk `chunk_id` (nothing waits for them here).
template <int VARIANT, bool TABLE>
__device__ __forceinline__ void issue_chunk(uint32_t chunk_id, const TensorDesc *__restrict__ descs, const Chunk *__restrict__ chunks,
                                            const TensorDesc &flat, ChunkIn<VARIANT> &c) {
  using SS = StepStreams<VARIANT>;
  if (TABLE) {
    const Chunk e = chunks[chunk_id];
    c.d = descs[e.tensor];
    c.slot0 = e.slot0;
  } else {
    c.d = flat;
    c.slot0 = (uint64_t)chunk_id * kSlotsPerChunk;
  }
  static_for<0, kUnroll>([&](auto jc) {
    constexpr int j = decltype(jc)::value;
    c.slot[j] = classify<SS::kEB>(c.d, c.slot0 + (uint64_t)j * kStepBlock + threadIdx.x);
    if (c.slot[j].full) {
      const uint64_t e0 = (c.slot[j].c0 - c.d.phase) * SS::kEB;       // byte offset
      load_vec(c.d.p[S_TH], e0, c.in[j][S_TH]);
      if (SS::kDth) load_vec(c.d.p[S_DTH], e0, c.in[j][S_DTH]);
      load_vec(c.d.p[S_M], e0, c.in[j][S_M]);
      if (SS::kV) load_vec(c.d.p[S_V], e0, c.in[j][S_V]);
      load_vec(c.d.p[S_G], e0, c.in[j][S_G]);
      if (SS::kDv) load_vec(c.d.p[S_DV], e0, c.in[j][S_DV]);
    } else if (c.slot[j].any) {
      // a slot that straddles an end of its tensor: its elements one by one, zeros for the rest
      load_slot<SS::kEB>(c.d.p[S_TH], c.d, c.slot[j], c.in[j][S_TH]);
      if (SS::kDth) load_slot<SS::kEB>(c.d.p[S_DTH], c.d, c.slot[j], c.in[j][S_DTH]);
      load_slot<SS::kEB>(c.d.p[S_M], c.d, c.slot[j], c.in[j][S_M]);
      if (SS::kV) load_slot<SS::kEB>(c.d.p[S_V], c.d, c.slot[j], c.in[j][S_V]);
      load_slot<SS::kEB>(c.d.p[S_G], c.d, c.slot[j], c.in[j][S_G]);
      if (SS::kDv) load_slot<SS::kEB>(c.d.p[S_DV], c.d, c.slot[j], c.in[j][S_DV]);
    }
  });
}

// Which elements of a slot belong to the tensor, one bit each.
template <int EB>
__device__ __forceinline__ uint32_t valid_elements(const TensorDesc &d, const Slot &s) {
  uint32_t valid = 0;
#pragma unroll
  for (int k = 0; k < 16 / EB; ++k)
    if (s.c0 + k >= d.phase && s.c0 + k < d.phase + d.n) valid |= 1u << k;
  return valid;
}

// Computes and stores a chunk whose loads were issued by issue_chunk; adds its EDQ terms to acc.
// A full slot takes the first pass; what that pass gives up (bf16: the root met a subnormal operand, or a
// result is NaN; fp16, FP8: a result is NaN) is computed again, still from registers, in the second mode:
// the same vector code with a root that scales tiny operands and a pack that stores the one NaN pattern (an
// all-NaN 7B set costs about twice the ordinary step, not a serial loop).  Slots at a tensor's ends, whose
// elements were gathered one by one, and every slot of a launch the host marked `elementwise` (epsilon under
// the root; an FP8 bias correction with no fp16 reciprocal) go to the second mode directly.
template <int VARIANT, bool FAST, bool EDQ>
__device__ __forceinline__ void finish_chunk(ChunkIn<VARIANT> &c, const typename StepStreams<VARIANT>::Scalars &sc, EdqAcc &acc) {
  using SS = StepStreams<VARIANT>;
  using First = typename SS::template Hot<FAST>;
  using Second = typename SS::template Second<FAST>;
  const TensorDesc &d = c.d;
  // Large sets (sc.write_through): agent scope; with the EDQ sums fused in: agent scope and non-temporal; the
  // ALU-bound FP8 kernels and small sets: non-temporal
  constexpr int kStore = MCF_STORE_POLICY >= 0 ? MCF_STORE_POLICY : SS::kEB == 1 ? ST_NT : EDQ ? ST_AGENT_NT : ST_AGENT;
  const bool skip_first = sc.elementwise != 0;       // uniform over the launch
  static_for<0, kUnroll>([&](auto jc) {
    constexpr int j = decltype(jc)::value;
    const Slot &slot = c.slot[j];
    if (slot.any) {
      uint32_t out[kMaxStreams][4];
      EdqAcc local = {0.0, 0.0, 0u};
      bool again = skip_first || !slot.full;
      if (!again) again = hot_slot<First, VARIANT, EDQ>(c.in[j], out, sc, local);
      if (again) {
        local = {0.0, 0.0, 0u};
        const uint32_t valid = slot.full ? ~0u : valid_elements<SS::kEB>(d, slot);
        if (sc.eps_inside_sqrt) (void)hot_slot<Second, VARIANT, EDQ, true, true>(c.in[j], out, sc, local, valid);
        else (void)hot_slot<Second, VARIANT, EDQ, false, true>(c.in[j], out, sc, local, valid);
      }
      if (slot.full) {
        const uint64_t e0 = (slot.c0 - d.phase) * SS::kEB;
        if (kStore != ST_NT && sc.write_through) {          // uniform over the launch
          store_vec<kStore>(d.p[S_TH], e0, out[S_TH]);
          if (SS::kDth) store_vec<kStore>(d.p[S_DTH], e0, out[S_DTH]);
          store_vec<kStore>(d.p[S_M], e0, out[S_M]);
          if (SS::kV) store_vec<kStore>(d.p[S_V], e0, out[S_V]);
          if (SS::kDv) store_vec<kStore>(d.p[S_DV], e0, out[S_DV]);
        } else {
          store_vec<ST_NT>(d.p[S_TH], e0, out[S_TH]);
          if (SS::kDth) store_vec<ST_NT>(d.p[S_DTH], e0, out[S_DTH]);
          store_vec<ST_NT>(d.p[S_M], e0, out[S_M]);
          if (SS::kV) store_vec<ST_NT>(d.p[S_V], e0, out[S_V]);
          if (SS::kDv) store_vec<ST_NT>(d.p[S_DV], e0, out[S_DV]);
        }
      } else {
        store_slot<SS::kEB>(d.p[S_TH], d, slot, out[S_TH]);
        if (SS::kDth) store_slot<SS::kEB>(d.p[S_DTH], d, slot, out[S_DTH]);
        store_slot<SS::kEB>(d.p[S_M], d, slot, out[S_M]);
        if (SS::kV) store_slot<SS::kEB>(d.p[S_V], d, slot, out[S_V]);
        if (SS::kDv) store_slot<SS::kEB>(d.p[S_DV], d, slot, out[S_DV]);
      }
      if (EDQ) { acc.s1 += local.s1; acc.s2 += local.s2; acc.lost += local.lost; }
    }
  });
}

// The step kernel.  Two work distributions, chosen at compile time (MCF_PERSIST):
//   0  one chunk per single-wave workgroup, the grid covers the chunk table (the default);
//   1  a fixed grid of single-wave workgroups (a few per CU), each walking the chunk table with the grid as
//      its stride and, with MCF_DEPTH 1, issuing the loads of its next chunk before it computes the current
//      one.  The eight XCDs (workgroups are dealt to them round-robin) each take a contiguous eighth of
//      every grid-sized stretch of the table, so a line of the table is fetched by one L2 only.
// Measured on MI355X, same process and arenas (ms per step; the default shape first):
//   7B set, light          19.19 | persistent, k workgroups per CU = 4 / 6 / 8 / 10 / 12 / 16:
//                                  depth 0: 26.6 / 23.4 / 24.2 / 24.9 / 24.9 / 25.4    depth 1: 29.1 / 24.5 / 23.7 / 24.7 / 24.8 / 26.8
//                                  depth 1, two slots per lane: 25.4 / 24.9 / 24.7 / 27.5 / 24.8 / 24.2;  depth 0, four slots: 27.9 ... 24.1
//   7B set, plus           24.00 | 29.4 - 34.4 over the same grid of settings
//   7B set, light FP8 E5M2 10.31 | 12.5 - 18.6      plus FP8 E5M2 14.53 | 16.8 - 24.6
//   64Mi stress set, plus   0.302 | 0.307 - 0.382     GPT-2-125M set, light 0.373 | 0.384 - 0.532
// (that build of the default shape was 3% off its best cap; the comparison does not hinge on it).  The fixed grid loses
// everywhere, by a quarter at the 7B set, and issuing loads a chunk ahead does not help it.  Two reasons.  A static
// stride gives every wave the same amount of work, so the launch ends with its slowest wave (k = 6 and 10, which
// cannot spread evenly over a CU's four SIMDs, stand out), while the hardware dispatcher hands the next chunk
// to whichever CU has room.  And that dispatcher is an in-order ticket counter: the chunks in flight at any
// time are neighbours in every stream, which keeps the DRAM pages in use few; persistent waves drift apart.
// Making the ticket explicit (an atomic counter) would cost 13 million atomics on one address per step to
// rebuild what the hardware does for nothing.
//   2  the middle ground: MCF_RUN consecutive chunks per workgroup, the next chunk's loads issued before the current
//      chunk's arithmetic, the runs still handed out in order by the dispatcher and capped like the default shape.
//      7B set, best cap of 2..12 and none, same process (default shape: light 18.58, plus 23.23, plain bf16 14.28,
//      light FP8 10.06): runs of 2: 19.31 / 24.58 / 14.97 / 10.79; of 4: 20.08 / 25.64 / 15.21 / 10.96; of 8: 22.12 /
//      27.74 / 16.43 / 11.17; of 16: 22.65 / 28.08 / 17.24 / 11.37; runs of 4 without the prefetch 25.99 / 31.94 / 18.57 /
//      12.46.  The longer a wave lives, the worse: one chunk per wave, born and retired in table order, is the shape.
template <int VARIANT, bool FAST, bool EDQ, bool TABLE>
__global__ void __launch_bounds__(kStepBlock) MCF_STEP_ATTR
adamw_kernel(const TensorDesc *__restrict__ descs, const Chunk *__restrict__ chunks, TensorDesc flat,
             typename StepStreams<VARIANT>::Scalars sc, double *__restrict__ partials, uint32_t n_chunks) {
  EdqAcc acc = {0.0, 0.0, 0u};
#if MCF_PERSIST
#if MCF_PERSIST == 2
  // a short run of consecutive chunks per workgroup; the dispatcher still hands the runs out in order
  const uint32_t stride = 1;
  uint32_t chunk_id = blockIdx.x * (uint32_t)MCF_RUN;
  const uint32_t end = n_chunks - chunk_id < (uint32_t)MCF_RUN ? n_chunks : chunk_id + (uint32_t)MCF_RUN;
#else
  const uint32_t stride = gridDim.x, end = n_chunks;
  uint32_t chunk_id = (stride & 7u) ? blockIdx.x : (blockIdx.x & 7u) * (stride >> 3) + (blockIdx.x >> 3);
#endif
  ChunkIn<VARIANT> cur;
  if (chunk_id < end) issue_chunk<VARIANT, TABLE>(chunk_id, descs, chunks, flat, cur);
  while (chunk_id < end) {
    const uint32_t next_id = chunk_id + stride;
#if MCF_DEPTH
    ChunkIn<VARIANT> nxt;
    const bool more = next_id < end && next_id > chunk_id;
    if (more) issue_chunk<VARIANT, TABLE>(next_id, descs, chunks, flat, nxt);
    __builtin_amdgcn_sched_barrier(0);             // the next chunk's loads stay ahead of this chunk's arithmetic
    finish_chunk<VARIANT, FAST, EDQ>(cur, sc, acc);
    if (!more) break;
    cur = nxt;
#else
    finish_chunk<VARIANT, FAST, EDQ>(cur, sc, acc);
    if (!(next_id < end && next_id > chunk_id)) break;
    issue_chunk<VARIANT, TABLE>(next_id, descs, chunks, flat, cur);
#endif
    chunk_id = next_id;
  }
  if (EDQ) edq_store_partial<kStepBlock>(acc, partials, blockIdx.x);
#else
  for (uint32_t i = 0; i < sc.head_sleep; ++i) __builtin_amdgcn_s_sleep(1);
  uint32_t chunk_id = blockIdx.x;
#if MCF_REMAP == 1
  {
    const uint32_t per = gridDim.x / 8;            // the grid is rounded up to a multiple of 8
    chunk_id = (blockIdx.x % 8) * per + blockIdx.x / 8;
    if (chunk_id >= n_chunks) return;
  }
#elif MCF_REMAP == 2
  {
    // within every run of 128 workgroups, XCD x (workgroups are dealt round-robin) takes chunks 16x .. 16x+15:
    // one 128-byte line of the chunk table per XCD instead of every line in all eight L2s
    const uint32_t b = blockIdx.x;
    chunk_id = (b & ~127u) | ((b & 7u) << 4) | ((b >> 3) & 15u);
    if (chunk_id >= n_chunks) return;
  }
#endif
  // Phase 1 issues every 128-bit load of the chunk, phase 2 computes and stores: the stores go to
  // the buffers the loads read, so the compiler would not move a later slot's loads above them.
  ChunkIn<VARIANT> cur;
  issue_chunk<VARIANT, TABLE>(chunk_id, descs, chunks, flat, cur);
  finish_chunk<VARIANT, FAST, EDQ>(cur, sc, acc);
  if (EDQ) edq_store_partial<kStepBlock>(acc, partials, chunk_id);
  for (uint32_t i = 0; i < sc.tail_sleep; ++i) __builtin_amdgcn_s_sleep(1);
#endif
}

// ---------------------------------------------------------------- EDQ reduction tail
constexpr int kStage1Blocks = 1024;

// Stage 1: block b sums partials [b*per, (b+1)*per) in a fixed order -> mid[b].
__global__ void __launch_bounds__(kBlock)
edq_stage1(const double *__restrict__ partials, uint64_t count, uint64_t per, double *__restrict__ mid) {
  const uint64_t lo = (uint64_t)blockIdx.x * per;
  uint64_t hi = lo + per;
  if (hi > count) hi = count;
  double a = 0.0, b = 0.0, c = 0.0;
  for (uint64_t i = lo + threadIdx.x; i < hi; i += kBlock) {
    a += partials[kEdqVals * i];
    b += partials[kEdqVals * i + 1];
    c += partials[kEdqVals * i + 2];
  }
  block_sum3(a, b, c);
  if (threadIdx.x == 0) { mid[kEdqVals * blockIdx.x] = a; mid[kEdqVals * blockIdx.x + 1] = b; mid[kEdqVals * blockIdx.x + 2] = c; }
}

// Stage 2: one block sums mid[0..nmid) and writes {EDQ, S1, S2, lost}.
__global__ void __launch_bounds__(kBlock)
edq_stage2(const double *__restrict__ mid, uint32_t nmid, double *__restrict__ out4) {
  double a = 0.0, b = 0.0, c = 0.0;
  for (uint32_t i = threadIdx.x; i < nmid; i += kBlock) { a += mid[kEdqVals * i]; b += mid[kEdqVals * i + 1]; c += mid[kEdqVals * i + 2]; }
  block_sum3(a, b, c);
  if (threadIdx.x == 0) {
    out4[0] = (b == 0.0) ? 0.0 : a / sqrt(b);
    out4[1] = a;
    out4[2] = b;
    out4[3] = c;
  }
}

// ---------------------------------------------------------------- element-wise primitives
enum PrimOp { P_FAST2SUM, P_TWOSUM, P_GROW, P_ADD, P_SUB, P_MUL, P_DIV, P_SQRT, P_EDQ, P_GROW2, P_TWOPROD, P_SCALING, P_MULX };

struct PrimArgs {
  uint64_t p[kMaxStreams];
  uint64_t n;
  uint32_t phase, skewed;
};

// One pair of elements of one primitive: inputs i[0..3] (and i[4] for EDQ), results (x, y).
template <class M, int OP>
__device__ __forceinline__ void prim_pair(const typename M::T (&i)[5], typename M::T &x, typename M::T &y,
                                          bool &redo, EdqAcc &acc, uint32_t valid2) {
  using O = mcfd::Ops<M>;
  using T = typename M::T;
  const T a = i[0], b = i[1];
  x = M::zero(); y = M::zero();
  if (OP == P_FAST2SUM) O::fast2sum(a, b, x, y);
  if (OP == P_TWOSUM) O::two_sum(a, b, x, y);
  if (OP == P_GROW) O::grow(a, b, i[2], x, y);                            // streams: x, y, a
  if (OP == P_GROW2) O::grow2(a, b, i[2], x, y);
  if (OP == P_TWOPROD) { x = O::mul(a, b); y = O::fms(a, b, x); }         // Alg. 6
  if (OP == P_SCALING) {                                                  // Alg. 7; streams: v, a1, a2
    const T x0 = O::mul(b, a);
    const T e = O::add(O::mul(i[2], a), O::fms(b, a, x0));
    O::fast2sum(x0, e, x, y);
  }
  if (OP == P_MULX) {                                                     // Alg. 8; streams: a1, a2, b1, b2
    const T b1 = i[2], b2 = i[3];
    const T x0 = O::mul(a, b1);
    const T ex = O::fms(a, b1, x0);
    const T cross = O::add(O::mul(a, b2), O::mul(b, b1));
    O::fast2sum(x0, O::add(ex, cross), x, y);
  }
  if (OP == P_ADD) x = O::add(a, b);
  if (OP == P_SUB) x = O::sub(a, b);
  if (OP == P_MUL) x = O::mul(a, b);
  if (OP == P_DIV) {
    if constexpr (M::kGuarded) {
      // the reciprocal route needs |b| zero, infinite, NaN or within [2^-126, 2^126]
      const float alo = __builtin_fabsf(b.lo), ahi = __builtin_fabsf(b.hi);
      redo |= mcfd::is_subnormal(b.lo) | mcfd::is_subnormal(b.hi) | (alo > 0x1p126f && alo < __builtin_inff()) |
              (ahi > 0x1p126f && ahi < __builtin_inff());
    }
    x = O::divg(a, b, redo);
  }
  if (OP == P_SQRT) x = O::sqrt(a, redo);
  if (OP == P_EDQ) {
    // streams: delta, th0, th1, dth0, dth1 (absent second components were loaded as zeros);
    // elements outside the tensor are skipped so that they cannot count as lost updates
    if (valid2 & 1u) edq_add(acc, M::lo(a), M::lo(b), M::lo(i[3]), M::lo(i[2]), M::lo(i[4]));
    if (valid2 & 2u) edq_add(acc, M::hi(a), M::hi(b), M::hi(i[3]), M::hi(i[2]), M::hi(i[4]));
  }
  if (M::kFast && OP != P_EDQ) redo |= M::any_nan(x) | M::any_nan(y);
}

// One slot of a primitive: 4 dwords per stream, 4/M::kBytes elements per dword.
template <class M, int OP>
__device__ __forceinline__ void prim_words(const uint32_t (&in)[kMaxStreams][4], uint32_t (&out)[kMaxStreams][4],
                                           bool &redo, EdqAcc &acc, uint32_t valid) {
  using T = typename M::T;
  constexpr int kPairs = M::kBytes == 1 ? 2 : 1;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    T x[kPairs], y[kPairs];
    static_for<0, kPairs>([&](auto pc) {
      constexpr int P = decltype(pc)::value;
      const T i[5] = {unpack_pair<M, P>(in[0][k]), unpack_pair<M, P>(in[1][k]), unpack_pair<M, P>(in[2][k]),
                      unpack_pair<M, P>(in[3][k]), unpack_pair<M, P>(in[4][k])};
      prim_pair<M, OP>(i, x[P], y[P], redo, acc, (valid >> (2 * (kPairs * k + P))) & 3u);
    });
    out[0][k] = pack_pairs<M>(x);
    out[1][k] = pack_pairs<M>(y);
  }
}

// Stream layout per op (inputs first):   reads            writes
//  FAST2SUM/TWOSUM: p0=a p1=b p2=x p3=y   0,1              out0->p2, out1->p3
//  GROW, GROW2:     p0=x p1=y p2=a p3=x' p4=y'  0,1,2       out0->p3, out1->p4 (may be p0, p1: a lane reads its slot before it writes)
//  TWOPROD:         p0=a p1=b p2=x p3=e   0,1              out0->p2, out1->p3
//  SCALING:         p0=v p1=a1 p2=a2 p3=x p4=e   0,1,2     out0->p3, out1->p4
//  MULX:            p0=a1 p1=a2 p2=b1 p3=b2 p4=x p5=e  0..3  out0->p4, out1->p5
//  ADD..SQRT:       p0=a p1=b p2=out      0,1 (sqrt: 0)    out0->p2
//  EDQ:             p0=delta p1=th0 p2=th1 p3=dth0 p4=dth1  (reads only; partial sums out)
template <int OP, int FMT>
__global__ void __launch_bounds__(kBlock) prim_kernel(PrimArgs a, uint32_t has_d0, uint32_t has_d1, double *__restrict__ partials) {
  using Hot = typename ModeOf<FMT, true>::Hot;
  using Cold = typename ModeOf<FMT, true>::Cold;
  constexpr int EB = Cold::kBytes;
  constexpr int kEps = 16 / EB;
  TensorDesc d;
#pragma unroll
  for (int s = 0; s < kMaxStreams; ++s) d.p[s] = a.p[s];
  d.n = a.n; d.phase = a.phase; d.skewed = a.skewed;
  const Slot s = classify<EB>(d, (uint64_t)blockIdx.x * kBlock + threadIdx.x);
  EdqAcc acc = {0.0, 0.0, 0u};
  if (s.any) {
    uint32_t in[kMaxStreams][4] = {};
    uint32_t out[kMaxStreams][4];
    constexpr int nin = (OP == P_GROW || OP == P_GROW2 || OP == P_SCALING) ? 3 : (OP == P_MULX) ? 4 : (OP == P_SQRT) ? 1 : 2;
    uint32_t valid = 0xffffu;            // which of the slot's elements belong to the tensor
    if (OP == P_EDQ) {
      load_slot<EB>(d.p[0], d, s, in[0]);
      load_slot<EB>(d.p[1], d, s, in[1]);
      load_slot<EB>(d.p[2], d, s, in[2]);
      if (has_d0) load_slot<EB>(d.p[3], d, s, in[3]);
      if (has_d1) load_slot<EB>(d.p[4], d, s, in[4]);
      valid = 0;
      for (int k = 0; k < kEps; ++k)
        if (s.c0 + k >= d.phase && s.c0 + k < d.phase + d.n) valid |= 1u << k;
    } else {
#pragma unroll
      for (int k = 0; k < nin; ++k) load_slot<EB>(d.p[k], d, s, in[k]);
    }
    bool redo = false;
    prim_words<Hot, OP>(in, out, redo, acc, valid);
    if (redo) {
      bool unused = false;
      prim_words<Cold, OP>(in, out, unused, acc, valid);
    }
    if (OP == P_FAST2SUM || OP == P_TWOSUM || OP == P_TWOPROD) { store_slot<EB>(d.p[2], d, s, out[0]); store_slot<EB>(d.p[3], d, s, out[1]); }
    if (OP == P_GROW || OP == P_GROW2) { store_slot<EB>(d.p[3], d, s, out[0]); store_slot<EB>(d.p[4], d, s, out[1]); }
    if (OP == P_SCALING) { store_slot<EB>(d.p[3], d, s, out[0]); store_slot<EB>(d.p[4], d, s, out[1]); }
    if (OP == P_MULX) { store_slot<EB>(d.p[4], d, s, out[0]); store_slot<EB>(d.p[5], d, s, out[1]); }
    if (OP == P_ADD || OP == P_SUB || OP == P_MUL || OP == P_DIV || OP == P_SQRT) store_slot<EB>(d.p[2], d, s, out[0]);
  }
  if (OP == P_EDQ) edq_store_partial<kBlock>(acc, partials, blockIdx.x);
}

// fp32 -> the component format over an array (the rounding inside F).  Two elements per lane.
template <int FMT>
__global__ void __launch_bounds__(kBlock) round_kernel(const float *__restrict__ in, uint64_t out, uint64_t n) {
  using Hot = typename ModeOf<FMT, true>::Hot;
  using Cold = typename ModeOf<FMT, true>::Cold;
  constexpr int EB = Cold::kBytes;
  const uint64_t i = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 2;
  if (i >= n) return;
  const float a = in[i];
  const float b = (i + 1 < n) ? in[i + 1] : 0.f;
  uint32_t lo, hi;
  if constexpr (FMT == MCF_COMPONENT_BF16) {
    if (mcfd::is_nan(a) | mcfd::is_nan(b)) {
      const typename Cold::T r = Cold::round_f32(a, b);
      lo = Cold::bits_lo(r); hi = Cold::bits_hi(r);
    } else {
      const typename Hot::T r = Hot::round_f32(a, b);             // the hardware conversion
      lo = Hot::pack(r) & 0xffffu; hi = Hot::pack(r) >> 16;
    }
  } else {
    const typename Cold::T r = Cold::round_f32(a, b);             // stores the format's one NaN
    lo = Cold::bits_lo(r); hi = Cold::bits_hi(r);
  }
  store_elem<EB>(out, i, lo);
  if (i + 1 < n) store_elem<EB>(out, i + 1, hi);
}

// Plain 128-bit copy in the step kernel's launch shape: the streaming ceiling the step is
// measured against, and the known-size transfer that calibrates the profiler's byte counters.
__global__ void __launch_bounds__(kStepBlock) MCF_STEP_ATTR
copy_kernel(uint64_t dst, uint64_t src, uint64_t nvec) {
  const uint64_t i = (uint64_t)blockIdx.x * kStepBlock + threadIdx.x;
  if (i >= nvec) return;
  uint32_t w[4];
  load_vec(src, 16 * i, w);
  store_vec(dst, 16 * i, w);
}

// The step's memory traffic without its arithmetic: every lane loads one 128-bit vector (VEC of them,
// THREADS * 16 bytes apart) from each of NR buffers and stores NW of them back, write j receiving what read j
// brought in (in place when the caller passes the same buffer for both, as the step does).  The reads that
// have no write are folded in through `mask`, which the host passes as zero: the loads stay, the data
// does not change.  Measures what the memory system gives this mix of streams in a given launch shape.
constexpr int kMaxMix = 8;
struct MixArgs {
  uint64_t rd[kMaxMix], wr[kMaxMix];
  uint64_t nvec;        // 128-bit vectors per buffer
  uint32_t mask;
};

template <int NR, int NW, int THREADS, int VEC, int STORE>
__global__ void __launch_bounds__(THREADS) mix_kernel(MixArgs a) {
  static_assert(NW <= NR && NR <= kMaxMix, "a write needs its read");
  const uint64_t base = (uint64_t)blockIdx.x * (THREADS * VEC) + threadIdx.x;
  uint32_t w[VEC][NR][4];
  static_for<0, VEC>([&](auto vc) {
    constexpr int v = decltype(vc)::value;
    const uint64_t i = base + (uint64_t)v * THREADS;
    if (i < a.nvec) static_for<0, NR>([&](auto rc) { load_vec(a.rd[decltype(rc)::value], 16 * i, w[v][decltype(rc)::value]); });
  });
  static_for<0, VEC>([&](auto vc) {
    constexpr int v = decltype(vc)::value;
    const uint64_t i = base + (uint64_t)v * THREADS;
    if (i < a.nvec) {
      uint32_t extra = 0;
      static_for<NW, NR>([&](auto rc) { constexpr int r = decltype(rc)::value; extra ^= w[v][r][0] ^ w[v][r][1] ^ w[v][r][2] ^ w[v][r][3]; });
      extra &= a.mask;
      static_for<0, NW>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        if (NR > NW) w[v][r][0] ^= extra;
        store_vec<STORE>(a.wr[r], 16 * i, w[v][r]);
      });
      if (NW == 0 && extra == 0x9e3779b9u) store_vec(a.rd[0], 16 * i, w[v][0]);      // never taken: keeps a read-only launch's loads
    }
  });
}

// ---------------------------------------------------------------- option D (fp32 master weights)
struct Fp32Desc {
  uint64_t theta, master, m, v, grad;   // pointers as integers
  uint64_t n;
  uint32_t phase, scalar_only;
  uint64_t pad;
};
static_assert(sizeof(Fp32Desc) == 64, "descriptor is one 64-byte scalar load");

struct Fp32Scalars { float b1, c1, b2, c2, bc1, bc2, e, lam, na; uint32_t write_through; };

__device__ __forceinline__ void fp32mw_elem(float g, float &m, float &v, float &w, const Fp32Scalars &s) {
  const float t1 = s.b1 * m;
  const float t2 = s.c1 * g;
  const float m1 = t1 + t2;
  const float g2 = g * g;
  const float t3 = s.b2 * v;
  const float t4 = s.c2 * g2;
  const float v1 = t3 + t4;
  const float mh = m1 / s.bc1;            // IEEE correctly rounded divide
  const float vh = v1 / s.bc2;
  const float dn = __builtin_sqrtf(vh) + s.e;
  const float q = mh / dn;
  const float dec = s.lam * w;
  const float sum = q + dec;
  const float delta = s.na * sum;
  w = w + delta;
  m = m1;
  v = v1;
}

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__global__ void __launch_bounds__(kStepBlock) MCF_STEP_ATTR
fp32mw_kernel(const Fp32Desc *__restrict__ descs, const Chunk *__restrict__ chunks, Fp32Scalars sc) {
  const Chunk c = chunks[blockIdx.x];
  const Fp32Desc d = descs[c.tensor];
  MCF_GLOBAL uint16_t *theta = gptr<uint16_t>(d.theta);
  const MCF_GLOBAL uint16_t *grad = gptr<const uint16_t>(d.grad);
  MCF_GLOBAL float *master = gptr<float>(d.master);
  MCF_GLOBAL float *mp = gptr<float>(d.m);
  MCF_GLOBAL float *vp = gptr<float>(d.v);
  const uint64_t c_lo = (uint64_t)c.slot0 * 8, c_hi = c_lo + 8ull * kSlotsPerChunk;
  const bool interior = !d.scalar_only && c_lo >= d.phase && c_hi <= d.phase + d.n;      // wave-uniform
  if (interior) {
    // Every access of the wave is one contiguous run: in pass h lane l takes the 4 elements
    // [h*4*kStepBlock + 4l, +4) of the chunk, i.e. 16 bytes of each fp32 buffer and 8 bytes of each
    // bf16 buffer, so a wave reads 1 KiB (fp32) or 512 B (bf16) per instruction with no gaps.
    constexpr int kPasses = 2 * kUnroll;
    u32x2_t gw[kPasses];
    f32x4_t mm[kPasses], vv[kPasses], ww[kPasses];
    static_for<0, kPasses>([&](auto hc) {
      constexpr int h = decltype(hc)::value;
      const uint64_t e0 = (c_lo - d.phase) + (uint64_t)h * 4 * kStepBlock + 4 * threadIdx.x;
#if MCF_NT_LOAD
      gw[h] = __builtin_nontemporal_load((const MCF_GLOBAL u32x2_t *)(grad + e0));
#else
      gw[h] = *(const MCF_GLOBAL u32x2_t *)(grad + e0);
#endif
      mm[h] = load_f4(mp + e0);
      vv[h] = load_f4(vp + e0);
      ww[h] = load_f4(master + e0);
    });
    static_for<0, kPasses>([&](auto hc) {
      constexpr int h = decltype(hc)::value;
      const uint64_t e0 = (c_lo - d.phase) + (uint64_t)h * 4 * kStepBlock + 4 * threadIdx.x;
      const P2 g0 = mcfd::widen2(gw[h].x), g1 = mcfd::widen2(gw[h].y);
      float m[4] = {mm[h].x, mm[h].y, mm[h].z, mm[h].w};
      float v[4] = {vv[h].x, vv[h].y, vv[h].z, vv[h].w};
      float w[4] = {ww[h].x, ww[h].y, ww[h].z, ww[h].w};
      fp32mw_elem(g0.lo, m[0], v[0], w[0], sc);
      fp32mw_elem(g0.hi, m[1], v[1], w[1], sc);
      fp32mw_elem(g1.lo, m[2], v[2], w[2], sc);
      fp32mw_elem(g1.hi, m[3], v[3], w[3], sc);
      const u32x2_t tw = {mcfd::pack2(mcfd::Exact::round_f32(w[0], w[1])), mcfd::pack2(mcfd::Exact::round_f32(w[2], w[3]))};
      const uint64_t theta_at = (uint64_t)(theta + e0);
      if (MCF_FP32MW_STORE != ST_NT && sc.write_through) {       // uniform over the launch
        store_f4<MCF_FP32MW_STORE>(mp + e0, f32x4_t{m[0], m[1], m[2], m[3]});
        store_f4<MCF_FP32MW_STORE>(vp + e0, f32x4_t{v[0], v[1], v[2], v[3]});
        store_f4<MCF_FP32MW_STORE>(master + e0, f32x4_t{w[0], w[1], w[2], w[3]});
        if (MCF_FP32MW_STORE == ST_AGENT) asm volatile("global_store_dwordx2 %0, %1, off sc1" : : "v"(theta_at), "v"(tw) : "memory");
        else asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" : : "v"(theta_at), "v"(tw) : "memory");
      } else {
        store_f4<ST_NT>(mp + e0, f32x4_t{m[0], m[1], m[2], m[3]});
        store_f4<ST_NT>(vp + e0, f32x4_t{v[0], v[1], v[2], v[3]});
        store_f4<ST_NT>(master + e0, f32x4_t{w[0], w[1], w[2], w[3]});
        __builtin_nontemporal_store(tw, (MCF_GLOBAL u32x2_t *)(theta + e0));
      }
    });
    return;
  }
  // Chunks at a tensor's ends, and tensors whose buffers are not mutually aligned: slot by slot,
  // element by element where a slot is not whole.
  TensorDesc t;
  t.n = d.n; t.phase = d.phase; t.skewed = d.scalar_only;
#pragma unroll 1
  for (int j = 0; j < kUnroll; ++j) {
    const Slot s = classify<2>(t, (uint64_t)c.slot0 + (uint64_t)j * kStepBlock + threadIdx.x);
    if (!s.any) continue;
    const uint64_t lo = d.phase, hi = d.phase + d.n;
#pragma unroll 1
    for (int k = 0; k < 8; ++k) {
      const uint64_t cc = s.c0 + k;
      if (cc < lo || cc >= hi) continue;
      const uint64_t e = cc - lo;
      float m = mp[e], v = vp[e], w = master[e];
      fp32mw_elem(mcfd::bitsf((uint32_t)grad[e] << 16), m, v, w, sc);
      mp[e] = m; vp[e] = v; master[e] = w;
      theta[e] = (uint16_t)(mcfd::fbits(mcfd::round_bits(w)) >> 16);
    }
  }
}

// ---------------------------------------------------------------- host side
#define MCF_HIP(call) do { if ((call) != hipSuccess) { (void)hipGetLastError(); return MCF_ERR_HIP; } } while (0)

inline bool misaligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// Where the slots of a set of streams are cut: phase = elements between the `boundary`-byte boundary at or
// below the first stream's pointer and that pointer.  skewed = 1 when some other stream sits at another
// offset modulo 16 bytes (its 128-bit accesses will be unaligned; nothing else depends on it).
inline void phase_of(const uint64_t *ptrs, int count, uint32_t &phase, uint32_t &skewed, uint64_t boundary = 16,
                     uint32_t elem_bytes = 2) {
  phase = (uint32_t)((ptrs[0] & (boundary - 1)) / elem_bytes);
  skewed = 0;
  for (int i = 1; i < count; ++i)
    if ((ptrs[i] & 15) != (ptrs[0] & 15)) skewed = 1;
}

inline uint64_t slots_of(uint64_t n, uint32_t phase, uint32_t elem_bytes = 2) {
  const uint64_t eps = 16 / elem_bytes;
  return (n + phase + eps - 1) / eps;
}

constexpr int kFmtMask = 3 << kFmtShift;
constexpr int kFlagMask = MCF_GROW_TWOSUM | MCF_EPS_INSIDE_SQRT | kFmtMask;
inline int format_of(int variant) { return (variant >> kFmtShift) & 3; }
inline uint32_t elem_bytes_of(int component) { return component >= MCF_COMPONENT_FP8_E5M2 ? 1u : 2u; }

inline bool known_variant(int v) {
  const int base = v & ~kFlagMask;
  if ((v & MCF_EPS_INSIDE_SQRT) && base == MCF_SGD) return false;          // SGD has no epsilon
  if (v & MCF_GROW_TWOSUM) return base == MCF_LIGHT || base == MCF_PLUS;
  return base == MCF_LIGHT || base == MCF_PLUS || base == MCF_BF16 || base == MCF_KAHAN || base == MCF_SGD;
}

int check_tensor(const mcf_tensor &t, int variant) {
  const uintptr_t eb = elem_bytes_of(format_of(variant));
  variant &= ~kFlagMask;
  if (t.n == 0) return MCF_OK;
  const bool need_dth = variant != MCF_BF16, need_dv = variant == MCF_PLUS, need_v = variant != MCF_SGD;
  if (!t.theta || !t.m || !t.grad) return MCF_ERR_NULL;
  if ((need_dth && !t.dtheta) || (need_dv && !t.dv) || (need_v && !t.v)) return MCF_ERR_NULL;
  if (t.n > kMaxTensorElems) return MCF_ERR_SIZE;
  if (misaligned(t.theta, eb) || misaligned(t.m, eb) || misaligned(t.grad, eb) || (need_v && misaligned(t.v, eb)) ||
      (need_dth && misaligned(t.dtheta, eb)) || (need_dv && misaligned(t.dv, eb)))
    return MCF_ERR_ALIGN;
  return MCF_OK;
}

// Streams a variant does not use point at theta (v for dv): they are never accessed and do
// not disturb the alignment class.
void fill_desc(const mcf_tensor &t, int variant, TensorDesc &d) {
  const uint32_t eb = elem_bytes_of(format_of(variant));
  variant &= ~kFlagMask;
  d.p[S_TH] = (uint64_t)(uintptr_t)t.theta;
  d.p[S_DTH] = variant != MCF_BF16 ? (uint64_t)(uintptr_t)t.dtheta : d.p[S_TH];
  d.p[S_M] = (uint64_t)(uintptr_t)t.m;
  d.p[S_V] = variant != MCF_SGD ? (uint64_t)(uintptr_t)t.v : d.p[S_TH];
  d.p[S_G] = (uint64_t)(uintptr_t)t.grad;
  d.p[S_DV] = variant == MCF_PLUS ? (uint64_t)(uintptr_t)t.dv : d.p[S_V];
  d.n = t.n;
  phase_of(d.p, 6, d.phase, d.skewed, MCF_CHUNK_ALIGN, eb);
}

// Order of the chunk table.  A chunk that holds a slot straddling one of its tensor's ends gathers that slot element
// by element and sends it through the second arithmetic pass: its wave lives several times as long as a wave of
// whole slots and moves fewer bytes.  A set with thousands of tiny tensors hands the dispatcher long runs of such
// chunks, and while they fill the CUs little memory traffic flows.  So they are dealt out evenly among the other
// chunks (which keep their order, and with it the neighbourhood of the addresses in flight), leaving the last
// eighth of the table to whole chunks so that the launch does not end on a slow wave.  Chunks are independent:
// the order changes when a chunk runs, never what it computes.
#ifndef MCF_SPREAD_RAGGED
#define MCF_SPREAD_RAGGED 1
#endif
void spread_ragged_chunks(std::vector<Chunk> &chunks, const std::vector<TensorDesc> &descs, uint32_t elem_bytes) {
  if (!MCF_SPREAD_RAGGED) return;
  const uint64_t eps = 16 / elem_bytes;
  auto ragged = [&](const Chunk &c) {
    const TensorDesc &d = descs[c.tensor];
    const uint64_t first = (uint64_t)c.slot0 * eps, last = first + (uint64_t)kSlotsPerChunk * eps;      // elements from the boundary
    const uint64_t end = d.n + d.phase;
    return (first < d.phase && d.phase % eps != 0) || (end > first && end < last && end % eps != 0);
  };
  size_t count = 0;
  for (const Chunk &c : chunks) count += ragged(c) ? 1 : 0;
  if (count == 0 || chunks.size() - count < 8 * count) return;    // nothing to hide, or nothing to hide it behind
  std::vector<Chunk> whole, rag;
  whole.reserve(chunks.size() - count);
  rag.reserve(count);
  for (const Chunk &c : chunks) (ragged(c) ? rag : whole).push_back(c);
  const size_t span = whole.size() - whole.size() / 8, n_rag = rag.size();
  size_t r = 0, out = 0;
  for (size_t w = 0; w < whole.size(); ++w) {
    while (r < n_rag && r * span / n_rag <= w) chunks[out++] = rag[r++];
    chunks[out++] = whole[w];
  }
  while (r < n_rag) chunks[out++] = rag[r++];
}

// Scalars of one step for both formats; fast = the bf16 Fast mode may be used with them.
struct HostScalars {
  StepScalars bf;
  StepScalarsH hf;
  StepScalarsF8 f8;
  bool fast;
};

// Workgroups of a step launch over `n_chunks` chunks (also the number of EDQ partials it writes).
uint32_t step_grid(uint32_t n_chunks) {
#if MCF_PERSIST == 2
  return (n_chunks + (uint32_t)MCF_RUN - 1) / (uint32_t)MCF_RUN;
#elif MCF_PERSIST
  static const uint32_t per_cu = [] {                // MCF_WAVES_PER_CU in the environment overrides the built-in figure (for sweeps)
    const char *e = getenv("MCF_WAVES_PER_CU");
    const int v = e ? atoi(e) : 0;
    return (uint32_t)(v > 0 && v <= 64 ? v : MCF_WAVES_PER_CU);
  }();
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  const uint32_t g = (uint32_t)cus * per_cu;
  return n_chunks < g ? n_chunks : g;
#elif MCF_REMAP == 1
  return (n_chunks + 7) / 8 * 8;
#elif MCF_REMAP == 2
  return (n_chunks + 127) / 128 * 128;
#else
  return n_chunks;
#endif
}

// Launch pacing of the step kernels that mcf_set_launch_pacing() may override (negative: the built-in figures).
std::atomic<int> g_groups_per_cu{-1}, g_head_sleep{-1}, g_tail_sleep{-1};

// Dynamic LDS of a step launch: the variant's built-in cap on the workgroups per CU, unless overridden.
uint32_t step_lds(uint32_t builtin) {
  const int forced = g_groups_per_cu.load(std::memory_order_relaxed);
  if (forced < 0 || MCF_PERSIST == 1) return builtin;
  return forced == 0 ? 0u : lds_for_groups((uint32_t)(forced > 128 ? 128 : forced));
}

template <int VARIANT, bool TABLE>
void launch_step(bool edq, uint32_t blocks, hipStream_t st, const TensorDesc *descs, const Chunk *chunks,
                 const TensorDesc &flat, const HostScalars &hs, double *partials) {
  const dim3 g(step_grid(blocks)), b(kStepBlock);
  using SS = StepStreams<VARIANT>;
  const uint32_t lds = step_lds(SS::kLds), lds_edq = step_lds(SS::kLdsEdq);
  if constexpr (SS::kFmt == MCF_COMPONENT_FP16) {          // one first-pass mode
    if (edq) hipLaunchKernelGGL((adamw_kernel<VARIANT, true, true, TABLE>), g, b, lds_edq, st, descs, chunks, flat, hs.hf, partials, blocks);
    else hipLaunchKernelGGL((adamw_kernel<VARIANT, true, false, TABLE>), g, b, lds, st, descs, chunks, flat, hs.hf, partials, blocks);
  } else if constexpr (!SS::kBf16) {                       // FP8, likewise
    if (edq) hipLaunchKernelGGL((adamw_kernel<VARIANT, true, true, TABLE>), g, b, lds_edq, st, descs, chunks, flat, hs.f8, partials, blocks);
    else hipLaunchKernelGGL((adamw_kernel<VARIANT, true, false, TABLE>), g, b, lds, st, descs, chunks, flat, hs.f8, partials, blocks);
  } else if (hs.fast) {
    if (edq) hipLaunchKernelGGL((adamw_kernel<VARIANT, true, true, TABLE>), g, b, lds_edq, st, descs, chunks, flat, hs.bf, partials, blocks);
    else hipLaunchKernelGGL((adamw_kernel<VARIANT, true, false, TABLE>), g, b, lds, st, descs, chunks, flat, hs.bf, partials, blocks);
  } else {
    if (edq) hipLaunchKernelGGL((adamw_kernel<VARIANT, false, true, TABLE>), g, b, lds_edq, st, descs, chunks, flat, hs.bf, partials, blocks);
    else hipLaunchKernelGGL((adamw_kernel<VARIANT, false, false, TABLE>), g, b, lds, st, descs, chunks, flat, hs.bf, partials, blocks);
  }
}

template <bool TABLE, int FMT>
void launch_format(int variant, bool edq, uint32_t blocks, hipStream_t st, const TensorDesc *descs,
                   const Chunk *chunks, const TensorDesc &flat, const HostScalars &hs, double *partials) {
  constexpr int F = FMT << kFmtShift;
  switch (variant & ~(kFmtMask | MCF_EPS_INSIDE_SQRT)) {       // the epsilon flag travels in the scalars
    case MCF_LIGHT | MCF_GROW_TWOSUM:
      launch_step<mcfd::V_LIGHT | kGrow2Bit | F, TABLE>(edq, blocks, st, descs, chunks, flat, hs, partials); break;
    case MCF_PLUS | MCF_GROW_TWOSUM:
      launch_step<mcfd::V_PLUS | kGrow2Bit | F, TABLE>(edq, blocks, st, descs, chunks, flat, hs, partials); break;
    case MCF_PLUS: launch_step<mcfd::V_PLUS | F, TABLE>(edq, blocks, st, descs, chunks, flat, hs, partials); break;
    case MCF_BF16: launch_step<mcfd::V_BF16 | F, TABLE>(edq, blocks, st, descs, chunks, flat, hs, partials); break;
    case MCF_KAHAN: launch_step<mcfd::V_KAHAN | F, TABLE>(edq, blocks, st, descs, chunks, flat, hs, partials); break;
    case MCF_SGD: launch_step<mcfd::V_SGD | F, TABLE>(edq, blocks, st, descs, chunks, flat, hs, partials); break;
    default: launch_step<mcfd::V_LIGHT | F, TABLE>(edq, blocks, st, descs, chunks, flat, hs, partials); break;
  }
}

template <bool TABLE>
void launch_variant(int variant, bool edq, uint32_t blocks, hipStream_t st, const TensorDesc *descs,
                    const Chunk *chunks, const TensorDesc &flat, const HostScalars &hs, double *partials) {
  switch (format_of(variant)) {
    case MCF_COMPONENT_FP16: launch_format<TABLE, MCF_COMPONENT_FP16>(variant, edq, blocks, st, descs, chunks, flat, hs, partials); break;
    case MCF_COMPONENT_FP8_E5M2: launch_format<TABLE, MCF_COMPONENT_FP8_E5M2>(variant, edq, blocks, st, descs, chunks, flat, hs, partials); break;
    case MCF_COMPONENT_FP8_E4M3: launch_format<TABLE, MCF_COMPONENT_FP8_E4M3>(variant, edq, blocks, st, descs, chunks, flat, hs, partials); break;
    default: launch_format<TABLE, MCF_COMPONENT_BF16>(variant, edq, blocks, st, descs, chunks, flat, hs, partials); break;
  }
}

// Reduce `count` partials (kEdqVals doubles each) to {EDQ, S1, S2, lost}; mid holds kEdqVals*kStage1Blocks doubles.
int launch_edq_tail(const double *partials, uint64_t count, double *mid, double *out3, hipStream_t st) {
  uint64_t per = (count + kStage1Blocks - 1) / kStage1Blocks;
  if (per == 0) per = 1;
  const uint32_t nmid = (uint32_t)((count + per - 1) / per);
  if (nmid) hipLaunchKernelGGL(edq_stage1, dim3(nmid), dim3(kBlock), 0, st, partials, count, per, mid);
  hipLaunchKernelGGL(edq_stage2, dim3(1), dim3(kBlock), 0, st, mid, nmid, out3);
  MCF_HIP(hipGetLastError());
  return MCF_OK;
}

// MCF_FORCE_EXACT=1 in the environment routes every step through the Exact arithmetic mode.
bool force_exact() {
  static const bool v = [] { const char *e = getenv("MCF_FORCE_EXACT"); return e && e[0] == '1'; }();
  return v;
}

HostScalars host_scalars(const mcf_hyper &h, uint64_t step, int variant, uint64_t n_params) {
  HostScalars hs = {};
  const int fmt = format_of(variant);
  if (fmt == MCF_COMPONENT_FP16) {
    mcfh::derive_scalars_fp16(h, step, hs.hf);
    hs.fast = true;
  } else if (fmt != MCF_COMPONENT_BF16) {
    hs.fast = true;
    if (!mcfh::derive_scalars_fp8(h, step, fmt == MCF_COMPONENT_FP8_E4M3, hs.f8)) hs.f8.elementwise = 1u;
  } else {
    hs.fast = mcfh::derive_scalars(h, step, hs.bf) && !force_exact();
  }
  {
    const uint32_t big = n_params * elem_bytes_of(fmt) >= kWriteThroughBytes ? 1u : 0u;
    hs.bf.write_through = hs.hf.write_through = hs.f8.write_through = big;
    const int head = g_head_sleep.load(std::memory_order_relaxed), tail = g_tail_sleep.load(std::memory_order_relaxed);
    hs.bf.head_sleep = hs.hf.head_sleep = hs.f8.head_sleep = (uint32_t)(head > 0 ? head : 0);
    hs.bf.tail_sleep = hs.hf.tail_sleep = hs.f8.tail_sleep = (uint32_t)(tail > 0 ? tail : 0);
  }
  // the printed form of line 12 is compiled into the second arithmetic pass only (SGD has no such line)
  if ((variant & MCF_EPS_INSIDE_SQRT) && (variant & 0xff) != MCF_SGD) {
    hs.bf.eps_inside_sqrt = hs.hf.eps_inside_sqrt = hs.f8.eps_inside_sqrt = 1u;
    hs.bf.elementwise = hs.hf.elementwise = hs.f8.elementwise = 1u;
  }
  return hs;
}

template <int FMT>
int prim_dispatch(int op, const dim3 &g, const dim3 &b, hipStream_t st, const PrimArgs &a) {
  switch (op) {
    case P_FAST2SUM: hipLaunchKernelGGL((prim_kernel<P_FAST2SUM, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_TWOSUM: hipLaunchKernelGGL((prim_kernel<P_TWOSUM, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_GROW: hipLaunchKernelGGL((prim_kernel<P_GROW, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_ADD: hipLaunchKernelGGL((prim_kernel<P_ADD, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_SUB: hipLaunchKernelGGL((prim_kernel<P_SUB, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_MUL: hipLaunchKernelGGL((prim_kernel<P_MUL, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_DIV: hipLaunchKernelGGL((prim_kernel<P_DIV, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_SQRT: hipLaunchKernelGGL((prim_kernel<P_SQRT, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_GROW2: hipLaunchKernelGGL((prim_kernel<P_GROW2, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_TWOPROD: hipLaunchKernelGGL((prim_kernel<P_TWOPROD, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_SCALING: hipLaunchKernelGGL((prim_kernel<P_SCALING, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    case P_MULX: hipLaunchKernelGGL((prim_kernel<P_MULX, FMT>), g, b, 0, st, a, 0u, 0u, nullptr); break;
    default: return MCF_ERR_VARIANT;
  }
  return MCF_OK;
}

int prim_launch(int format, int op, const void *p0, const void *p1, const void *p2, const void *p3, const void *p4,
                       int nptr, uint64_t n, void *stream, const void *p5 = nullptr) {
  const void *ps[6] = {p0, p1, p2, p3, p4, p5};
  const uint32_t eb = elem_bytes_of(format);
  PrimArgs a = {};
  uint64_t al[6];
  int na = 0;
  for (int i = 0; i < nptr; ++i) {
    a.p[i] = (uint64_t)(uintptr_t)ps[i];
    if (ps[i]) {
      if (misaligned(ps[i], eb)) return MCF_ERR_ALIGN;
      al[na++] = a.p[i];
    }
  }
  if (n > kMaxTensorElems) return MCF_ERR_SIZE;
  a.n = n;
  phase_of(al, na, a.phase, a.skewed, 16, eb);
  const uint64_t slots = slots_of(n, a.phase, eb);
  const dim3 g((uint32_t)((slots + kBlock - 1) / kBlock)), b(kBlock);
  hipStream_t st = (hipStream_t)stream;
  int rc;
  switch (format) {
    case MCF_COMPONENT_FP16: rc = prim_dispatch<MCF_COMPONENT_FP16>(op, g, b, st, a); break;
    case MCF_COMPONENT_FP8_E5M2: rc = prim_dispatch<MCF_COMPONENT_FP8_E5M2>(op, g, b, st, a); break;
    case MCF_COMPONENT_FP8_E4M3: rc = prim_dispatch<MCF_COMPONENT_FP8_E4M3>(op, g, b, st, a); break;
    default: rc = prim_dispatch<MCF_COMPONENT_BF16>(op, g, b, st, a); break;
  }
  if (rc != MCF_OK) return rc;
  MCF_HIP(hipGetLastError());
  return MCF_OK;
}

template <int NR, int NW, int THREADS, int STORE>
void launch_mix_vec(uint32_t vec, uint32_t lds, hipStream_t st, const MixArgs &a) {
  const uint64_t per = (uint64_t)THREADS * vec;
  const dim3 g((uint32_t)((a.nvec + per - 1) / per)), b(THREADS);
  switch (vec) {
    case 1: hipLaunchKernelGGL((mix_kernel<NR, NW, THREADS, 1, STORE>), g, b, lds, st, a); break;
    case 2: hipLaunchKernelGGL((mix_kernel<NR, NW, THREADS, 2, STORE>), g, b, lds, st, a); break;
    default: hipLaunchKernelGGL((mix_kernel<NR, NW, THREADS, 4, STORE>), g, b, lds, st, a); break;
  }
}

template <int NR, int NW>
void launch_mix(uint32_t threads, uint32_t vec, uint32_t lds, uint32_t store, hipStream_t st, const MixArgs &a) {
  if (threads == 64) {
    if (store == ST_AGENT) launch_mix_vec<NR, NW, 64, ST_AGENT>(vec, lds, st, a);
    else if (store == ST_AGENT_NT) launch_mix_vec<NR, NW, 64, ST_AGENT_NT>(vec, lds, st, a);
    else launch_mix_vec<NR, NW, 64, ST_NT>(vec, lds, st, a);
  } else {
    if (store == ST_AGENT) launch_mix_vec<NR, NW, 256, ST_AGENT>(vec, lds, st, a);
    else if (store == ST_AGENT_NT) launch_mix_vec<NR, NW, 256, ST_AGENT_NT>(vec, lds, st, a);
    else launch_mix_vec<NR, NW, 256, ST_NT>(vec, lds, st, a);
  }
}

inline bool known_component(int c) { return c >= MCF_COMPONENT_BF16 && c <= MCF_COMPONENT_FP8_E4M3; }

// The stand-alone EDQ reduction (Def. 3.3) over n > 0 elements with `partials` as its scratch memory:
// one partial per workgroup of the first kernel, then the two-kernel tail.
int edq_launch(int component, const void *delta, const void *th0, const void *dth0, const void *th1,
               const void *dth1, uint64_t n, double *partials, hipStream_t st, double *edq_dev) {
  // stream order: delta, th0, th1, dth0, dth1 (absent second components are not read)
  const void *ps[5] = {delta, th0, th1, dth0, dth1};
  const uint32_t eb = elem_bytes_of(component);
  for (int i = 0; i < 5; ++i)
    if (ps[i] && misaligned(ps[i], eb)) return MCF_ERR_ALIGN;
  PrimArgs a = {};
  uint64_t al[5];
  int na = 0;
  for (int i = 0; i < 5; ++i) {
    a.p[i] = (uint64_t)(uintptr_t)ps[i];
    if (ps[i]) al[na++] = a.p[i];
  }
  if (n > kMaxTensorElems) return MCF_ERR_SIZE;
  a.n = n;
  phase_of(al, na, a.phase, a.skewed, 16, eb);
  const uint64_t blocks = (slots_of(n, a.phase, eb) + kBlock - 1) / kBlock;
  const dim3 g((uint32_t)blocks), b(kBlock);
  const uint32_t h0 = dth0 ? 1u : 0u, h1 = dth1 ? 1u : 0u;
  switch (component) {
    case MCF_COMPONENT_FP16: hipLaunchKernelGGL((prim_kernel<P_EDQ, MCF_COMPONENT_FP16>), g, b, 0, st, a, h0, h1, partials); break;
    case MCF_COMPONENT_FP8_E5M2: hipLaunchKernelGGL((prim_kernel<P_EDQ, MCF_COMPONENT_FP8_E5M2>), g, b, 0, st, a, h0, h1, partials); break;
    case MCF_COMPONENT_FP8_E4M3: hipLaunchKernelGGL((prim_kernel<P_EDQ, MCF_COMPONENT_FP8_E4M3>), g, b, 0, st, a, h0, h1, partials); break;
    default: hipLaunchKernelGGL((prim_kernel<P_EDQ, MCF_COMPONENT_BF16>), g, b, 0, st, a, h0, h1, partials); break;
  }
  MCF_HIP(hipGetLastError());
  return launch_edq_tail(partials, blocks, partials + kEdqVals * blocks, edq_dev, st);
}

}  // namespace

// Reduction partials of mcf_edq_noalloc: a fixed array in device memory instead of a buffer somebody
// allocated.  Every GPU the library's code object is loaded on holds its own copy at its own address.
constexpr uint64_t kNoAllocMaxElems = 1ull << 28;
constexpr uint64_t edq_partial_doubles(uint64_t n) {        // for 2-byte elements at the worst phase; 1-byte elements need fewer
  return (uint64_t)kEdqVals * (((n + 7 + 7) / 8 + kBlock - 1) / kBlock + 1 + kStage1Blocks);
}
static __device__ __align__(256) double edq_scratch[edq_partial_doubles(kNoAllocMaxElems)];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double *g_scratch_ptr[kMaxDevices];      // device address of edq_scratch per device, resolved on the first call there

// In host code `edq_scratch` is only a handle for the runtime, not an address a kernel could use: the
// address on the current device comes from hipGetSymbolAddress, once per device.
int scratch_of_current_device(double **out) {
  int dev = -1;
  MCF_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return MCF_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    MCF_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(edq_scratch)));
    if (!p) return MCF_ERR_HIP;
    g_scratch_ptr[dev] = (double *)p;
  }
  *out = g_scratch_ptr[dev];
  return MCF_OK;
}

}  // namespace

struct mcf_plan {
  int device;           // the device that was current at creation: its tables live there
  int variant;
  uint32_t n_tensors;
  uint32_t n_chunks;
  uint64_t n_params;
  // Two descriptor tables in one device allocation; steps read d_descs[cur].  mcf_plan_update fills the
  // other one through its own block of pinned host memory and then makes it current, so it never has to
  // wait for the copy: the pinned block is only written again two updates later, after `staged` of that
  // block (recorded behind its copy) has completed.
  TensorDesc *d_descs[2];
  TensorDesc *h_stage[2];            // pinned host memory, n_tensors descriptors each
  hipEvent_t staged[2];
  bool have_events;
  int cur;
  Chunk *d_chunks;
  double *d_partials;   // kEdqVals*n_chunks doubles, then kEdqVals*kStage1Blocks doubles
  std::vector<uint32_t> phases;      // phase of every non-empty tensor's theta (mcf_plan_update must keep it)
  std::vector<uint64_t> in_n;        // n of every tensor given at creation, empty ones included
};

struct mcf_fp32mw_plan {
  int device;
  uint32_t n_chunks;
  uint64_t n_params;
  Fp32Desc *d_descs;
  Chunk *d_chunks;
};

namespace {
// A plan's tables are memory of one device; a step launched with another device current would hand its kernel
// pointers that device cannot reach.
int on_plan_device(int plan_device) {
  int dev = -1;
  MCF_HIP(hipGetDevice(&dev));
  return dev == plan_device ? MCF_OK : MCF_ERR_HIP;
}
}  // namespace

extern "C" {

const char *mcf_status_string(int status) {
  switch (status) {
    case MCF_OK: return "ok";
    case MCF_ERR_NULL: return "a required pointer is NULL";
    case MCF_ERR_SIZE: return "a size is out of range";
    case MCF_ERR_ALIGN: return "a pointer is not aligned to its element size";
    case MCF_ERR_VARIANT: return "unknown variant or operation code";
    case MCF_ERR_STEP: return "step must be at least 1";
    case MCF_ERR_HYPER: return "hyper-parameter out of range";
    case MCF_ERR_HIP: return "a HIP runtime call failed";
    default: return "unknown status";
  }
}

// The host-side tables are std::vectors: a failed allocation there must not leave through the C boundary.
#define MCF_NO_THROW_BEGIN try {
#define MCF_NO_THROW_END(cleanup) } catch (...) { cleanup; return MCF_ERR_HIP; }

int mcf_plan_create(mcf_plan **out, const mcf_tensor *tensors, uint32_t count, int variant) {
  if (!out) return MCF_ERR_NULL;
  *out = nullptr;
  if (count && !tensors) return MCF_ERR_NULL;
  if (!known_variant(variant)) return MCF_ERR_VARIANT;
  mcf_plan *p = nullptr;
  MCF_NO_THROW_BEGIN
  for (uint32_t i = 0; i < count; ++i) {
    const int rc = check_tensor(tensors[i], variant);
    if (rc != MCF_OK) return rc;
  }
  std::vector<TensorDesc> descs;
  std::vector<Chunk> chunks;
  uint64_t params = 0;
  for (uint32_t i = 0; i < count; ++i) {
    if (tensors[i].n == 0) continue;
    TensorDesc d;
    fill_desc(tensors[i], variant, d);
    const uint64_t slots = slots_of(d.n, d.phase, elem_bytes_of(format_of(variant)));
    const uint64_t nch = (slots + kSlotsPerChunk - 1) / kSlotsPerChunk;
    if (slots > 0xffffffffull || chunks.size() + nch > 0x7fffffffull) return MCF_ERR_SIZE;
    const uint32_t id = (uint32_t)descs.size();
    descs.push_back(d);
    for (uint64_t c = 0; c < nch; ++c) chunks.push_back(Chunk{id, (uint32_t)(c * kSlotsPerChunk)});
    params += d.n;
  }
  spread_ragged_chunks(chunks, descs, elem_bytes_of(format_of(variant)));
  p = new (std::nothrow) mcf_plan();
  if (!p) return MCF_ERR_HIP;
  p->device = -1;
  p->variant = variant;
  p->n_tensors = (uint32_t)descs.size();
  p->n_chunks = (uint32_t)chunks.size();
  p->n_params = params;
  p->d_descs[0] = p->d_descs[1] = nullptr;
  p->h_stage[0] = p->h_stage[1] = nullptr;
  p->have_events = false;
  p->cur = 0;
  p->d_chunks = nullptr;
  p->d_partials = nullptr;
  p->phases.resize(descs.size());
  for (size_t i = 0; i < descs.size(); ++i) p->phases[i] = descs[i].phase;
  p->in_n.resize(count);
  for (uint32_t i = 0; i < count; ++i) p->in_n[i] = tensors[i].n;
  if (p->n_chunks && hipGetDevice(&p->device) != hipSuccess) {       // an empty plan owns nothing on any device
    (void)hipGetLastError();
    mcf_plan_destroy(p);
    return MCF_ERR_HIP;
  }
  if (p->n_chunks) {
    const size_t table = descs.size() * sizeof(TensorDesc);
    bool ok = hipMalloc((void **)&p->d_descs[0], 2 * table) == hipSuccess &&
              hipHostMalloc((void **)&p->h_stage[0], 2 * table, hipHostMallocDefault) == hipSuccess &&
              hipEventCreateWithFlags(&p->staged[0], hipEventDisableTiming) == hipSuccess;
    if (ok) {
      if (hipEventCreateWithFlags(&p->staged[1], hipEventDisableTiming) == hipSuccess) p->have_events = true;
      else { (void)hipEventDestroy(p->staged[0]); ok = false; }
    }
    if (ok) {
      p->d_descs[1] = p->d_descs[0] + descs.size();
      p->h_stage[1] = p->h_stage[0] + descs.size();
    }
    ok = ok && hipMalloc((void **)&p->d_chunks, chunks.size() * sizeof(Chunk)) == hipSuccess &&
         hipMalloc((void **)&p->d_partials, (uint64_t)kEdqVals * ((uint64_t)p->n_chunks + kStage1Blocks) * sizeof(double)) == hipSuccess &&
         hipMemcpy(p->d_descs[0], descs.data(), table, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemcpy(p->d_chunks, chunks.data(), chunks.size() * sizeof(Chunk), hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {
      (void)hipGetLastError();
      mcf_plan_destroy(p);
      return MCF_ERR_HIP;
    }
  }
  *out = p;
  return MCF_OK;
  MCF_NO_THROW_END(mcf_plan_destroy(p))
}

int mcf_plan_destroy(mcf_plan *plan) {
  if (!plan) return MCF_OK;
  int rc = MCF_OK;
  if (plan->have_events) {
    // a copy out of the pinned block may still be queued
    for (hipEvent_t ev : plan->staged) {
      if (hipEventSynchronize(ev) != hipSuccess) rc = MCF_ERR_HIP;
      if (hipEventDestroy(ev) != hipSuccess) rc = MCF_ERR_HIP;
    }
  }
  if (plan->d_descs[0] && hipFree(plan->d_descs[0]) != hipSuccess) rc = MCF_ERR_HIP;
  if (plan->h_stage[0] && hipHostFree(plan->h_stage[0]) != hipSuccess) rc = MCF_ERR_HIP;
  if (plan->d_chunks && hipFree(plan->d_chunks) != hipSuccess) rc = MCF_ERR_HIP;
  if (plan->d_partials && hipFree(plan->d_partials) != hipSuccess) rc = MCF_ERR_HIP;
  if (rc != MCF_OK) (void)hipGetLastError();
  delete plan;
  return rc;
}

uint64_t mcf_plan_params(const mcf_plan *plan) { return plan ? plan->n_params : 0; }

int mcf_plan_update(mcf_plan *plan, const mcf_tensor *tensors, uint32_t count, void *stream) {
  if (!plan) return MCF_ERR_NULL;
  if (count != plan->in_n.size()) return MCF_ERR_SIZE;
  if (count && !tensors) return MCF_ERR_NULL;
  MCF_NO_THROW_BEGIN
  std::vector<TensorDesc> descs;
  descs.reserve(plan->phases.size());
  for (uint32_t i = 0; i < count; ++i) {
    if (tensors[i].n != plan->in_n[i]) return MCF_ERR_SIZE;
    const int rc = check_tensor(tensors[i], plan->variant);
    if (rc != MCF_OK) return rc;
    if (tensors[i].n == 0) continue;
    TensorDesc d;
    fill_desc(tensors[i], plan->variant, d);
    // the chunk table was cut for the old theta's offset within its 128-byte line: the new one must share it
    if (d.phase != plan->phases[descs.size()]) return MCF_ERR_ALIGN;
    descs.push_back(d);
  }
  if (descs.empty()) return MCF_OK;
  const int where = on_plan_device(plan->device);
  if (where != MCF_OK) return where;
  hipStream_t st = (hipStream_t)stream;
  // A captured copy would read the pinned block again at every replay, whatever it holds by then.
  hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
  MCF_HIP(hipStreamIsCapturing(st, &capturing));
  if (capturing != hipStreamCaptureStatusNone) return MCF_ERR_HIP;
  const int nxt = plan->cur ^ 1;
  // The pinned block of table `nxt` was last read by the copy of the update before the previous one;
  // this returns at once unless the host has run two updates ahead of the device.
  MCF_HIP(hipEventSynchronize(plan->staged[nxt]));
  const size_t table = descs.size() * sizeof(TensorDesc);
  memcpy(plan->h_stage[nxt], descs.data(), table);
  // ordered on `stream` behind the steps already enqueued there (they read the other table anyway)
  MCF_HIP(hipMemcpyAsync(plan->d_descs[nxt], plan->h_stage[nxt], table, hipMemcpyHostToDevice, st));
  MCF_HIP(hipEventRecord(plan->staged[nxt], st));
  plan->cur = nxt;
  return MCF_OK;
  MCF_NO_THROW_END((void)0)
}

int mcf_adamw_step(mcf_plan *plan, const mcf_hyper *hyper, uint64_t step, void *stream, double *edq_dev) {
  if (!plan) return MCF_ERR_NULL;
  const int rc = mcfh::check_hyper(hyper, step);
  if (rc != MCF_OK) return rc;
  if (edq_dev && misaligned(edq_dev, 8)) return MCF_ERR_ALIGN;
  const int where = plan->n_chunks ? on_plan_device(plan->device) : MCF_OK;
  if (where != MCF_OK) return where;
  const HostScalars hs = host_scalars(*hyper, step, plan->variant, plan->n_params);
  hipStream_t st = (hipStream_t)stream;
  const TensorDesc none = {};
  if (plan->n_chunks) {
    launch_variant<true>(plan->variant, edq_dev != nullptr, plan->n_chunks, st, plan->d_descs[plan->cur], plan->d_chunks, none, hs,
                         plan->d_partials);
    MCF_HIP(hipGetLastError());
  }
  if (edq_dev) {
    // with no chunks the tail sums nothing and writes zeros
#if MCF_PERSIST
    const uint64_t n_partials = plan->n_chunks ? step_grid(plan->n_chunks) : 0;      // one per workgroup
#else
    const uint64_t n_partials = plan->n_chunks;                                      // one per chunk
#endif
    return launch_edq_tail(plan->d_partials, n_partials, plan->d_partials + (uint64_t)kEdqVals * plan->n_chunks, edq_dev, st);
  }
  return MCF_OK;
}

int mcf_step_scalars(int component, const mcf_hyper *hyper, uint64_t step, uint16_t *out, int *restricted_mode_ok) {
  if (!known_component(component)) return MCF_ERR_VARIANT;
  if (!out) return MCF_ERR_NULL;
  const int rc = mcfh::check_hyper(hyper, step);
  if (rc != MCF_OK) return rc;
  const mcfh::ScalarBits b = component == MCF_COMPONENT_FP16       ? mcfh::scalar_bits_fp16(*hyper, step)
                             : component == MCF_COMPONENT_FP8_E5M2 ? mcfh::scalar_bits_e5m2(*hyper, step)
                             : component == MCF_COMPONENT_FP8_E4M3 ? mcfh::scalar_bits_e4m3(*hyper, step)
                                                                   : mcfh::scalar_bits_bf16(*hyper, step);
  for (int i = 0; i < mcfh::K_COUNT; ++i) out[i] = b.v[i];
  if (restricted_mode_ok) {
    StepScalars unused;
    StepScalarsF8 unused8;
    if (component == MCF_COMPONENT_BF16) *restricted_mode_ok = (mcfh::derive_scalars(*hyper, step, unused) && !force_exact()) ? 1 : 0;
    else if (component == MCF_COMPONENT_FP16) *restricted_mode_ok = 1;
    else *restricted_mode_ok = mcfh::derive_scalars_fp8(*hyper, step, component == MCF_COMPONENT_FP8_E4M3, unused8) ? 1 : 0;
  }
  return MCF_OK;
}

int mcf_adamw_step_flat(void *theta, void *dtheta, void *m, void *v, void *dv,
                        const void *grad, uint64_t n, int variant, const mcf_hyper *hyper,
                        uint64_t step, void *stream) {
  if (!known_variant(variant)) return MCF_ERR_VARIANT;
  const mcf_tensor t = {theta, dtheta, m, v, dv, grad, n};
  int rc = check_tensor(t, variant);
  if (rc != MCF_OK) return rc;
  rc = mcfh::check_hyper(hyper, step);
  if (rc != MCF_OK) return rc;
  if (n == 0) return MCF_OK;
  TensorDesc d;
  fill_desc(t, variant, d);
  const uint64_t nch = (slots_of(d.n, d.phase, elem_bytes_of(format_of(variant))) + kSlotsPerChunk - 1) / kSlotsPerChunk;
  const HostScalars hs = host_scalars(*hyper, step, variant, n);
  launch_variant<false>(variant, false, (uint32_t)nch, (hipStream_t)stream, nullptr, nullptr, d, hs, nullptr);
  MCF_HIP(hipGetLastError());
  return MCF_OK;
}

int mcf_primitive(int component, int which, const void *p0, const void *p1, const void *p2, const void *p3,
                  void *o0, void *o1, uint64_t n, void *stream) {
  static const int ops[7] = {P_FAST2SUM, P_TWOSUM, P_GROW, P_GROW2, P_TWOPROD, P_SCALING, P_MULX};
  static const int nin[7] = {2, 2, 3, 3, 2, 3, 4};
  if (!known_component(component) || which < 0 || which > 6) return MCF_ERR_VARIANT;
  if (n == 0) return MCF_OK;
  const void *ps[6] = {p0, p1, p2, p3, nullptr, nullptr};
  for (int i = 0; i < nin[which]; ++i)
    if (!ps[i]) return MCF_ERR_NULL;
  if (!o0 || !o1) return MCF_ERR_NULL;
  ps[nin[which]] = o0;
  ps[nin[which] + 1] = o1;
  return prim_launch(component, ops[which], ps[0], ps[1], ps[2], ps[3], ps[4], nin[which] + 2, n, stream, ps[5]);
}

int mcf_fast2sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n, void *stream) {
  return mcf_primitive(MCF_COMPONENT_BF16, MCF_PRIM_FAST2SUM, a, b, nullptr, nullptr, x, y, n, stream);
}

int mcf_two_sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n, void *stream) {
  return mcf_primitive(MCF_COMPONENT_BF16, MCF_PRIM_TWOSUM, a, b, nullptr, nullptr, x, y, n, stream);
}

int mcf_grow(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n, void *stream) {
  return mcf_primitive(MCF_COMPONENT_BF16, MCF_PRIM_GROW, x, y, a, nullptr, x, y, n, stream);
}

int mcf_grow_two_sum(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n, void *stream) {
  return mcf_primitive(MCF_COMPONENT_BF16, MCF_PRIM_GROW_TWOSUM, x, y, a, nullptr, x, y, n, stream);
}

int mcf_two_prod_fma(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *e, uint64_t n, void *stream) {
  return mcf_primitive(MCF_COMPONENT_BF16, MCF_PRIM_TWOPROD, a, b, nullptr, nullptr, x, e, n, stream);
}

int mcf_scaling(const uint16_t *v, const uint16_t *a1, const uint16_t *a2, uint16_t *x, uint16_t *e, uint64_t n, void *stream) {
  return mcf_primitive(MCF_COMPONENT_BF16, MCF_PRIM_SCALING, v, a1, a2, nullptr, x, e, n, stream);
}

int mcf_mul(const uint16_t *a1, const uint16_t *a2, const uint16_t *b1, const uint16_t *b2, uint16_t *x, uint16_t *e,
            uint64_t n, void *stream) {
  return mcf_primitive(MCF_COMPONENT_BF16, MCF_PRIM_MUL, a1, a2, b1, b2, x, e, n, stream);
}

int mcf_component_op(int component, int op, const void *a, const void *b, void *out, uint64_t n, void *stream) {
  if (!known_component(component) || op < 0 || op > 4) return MCF_ERR_VARIANT;
  if (n == 0) return MCF_OK;
  if (!a || !out || (op != 4 && !b)) return MCF_ERR_NULL;
  if (op == 4) b = a;
  static const int map[5] = {P_ADD, P_SUB, P_MUL, P_DIV, P_SQRT};
  return prim_launch(component, map[op], a, b, out, nullptr, nullptr, 3, n, stream);
}

int mcf_bf16_op(int op, const uint16_t *a, const uint16_t *b, uint16_t *out, uint64_t n, void *stream) {
  return mcf_component_op(MCF_COMPONENT_BF16, op, a, b, out, n, stream);
}

int mcf_round_f32_to(int component, const float *in, void *out, uint64_t n, void *stream) {
  if (!known_component(component)) return MCF_ERR_VARIANT;
  if (n == 0) return MCF_OK;
  if (!in || !out) return MCF_ERR_NULL;
  if (misaligned(in, 4) || misaligned(out, elem_bytes_of(component))) return MCF_ERR_ALIGN;
  const uint64_t lanes = (n + 1) / 2;
  const uint64_t blocks = (lanes + kBlock - 1) / kBlock;
  if (blocks > 0x7fffffffull) return MCF_ERR_SIZE;
  const dim3 g((uint32_t)blocks), b(kBlock);
  const uint64_t o = (uint64_t)(uintptr_t)out;
  hipStream_t st = (hipStream_t)stream;
  switch (component) {
    case MCF_COMPONENT_FP16: hipLaunchKernelGGL(round_kernel<MCF_COMPONENT_FP16>, g, b, 0, st, in, o, n); break;
    case MCF_COMPONENT_FP8_E5M2: hipLaunchKernelGGL(round_kernel<MCF_COMPONENT_FP8_E5M2>, g, b, 0, st, in, o, n); break;
    case MCF_COMPONENT_FP8_E4M3: hipLaunchKernelGGL(round_kernel<MCF_COMPONENT_FP8_E4M3>, g, b, 0, st, in, o, n); break;
    default: hipLaunchKernelGGL(round_kernel<MCF_COMPONENT_BF16>, g, b, 0, st, in, o, n); break;
  }
  MCF_HIP(hipGetLastError());
  return MCF_OK;
}

int mcf_round_f32(const float *in, uint16_t *out, uint64_t n, void *stream) {
  return mcf_round_f32_to(MCF_COMPONENT_BF16, in, out, n, stream);
}

int mcf_stream_copy(void *dst, const void *src, uint64_t bytes, void *stream) {
  if (bytes == 0) return MCF_OK;
  if (!dst || !src) return MCF_ERR_NULL;
  if (misaligned(dst, 16) || misaligned(src, 16) || (bytes & 15)) return MCF_ERR_ALIGN;
  const uint64_t nvec = bytes / 16;
  const uint64_t blocks = (nvec + kStepBlock - 1) / kStepBlock;
  if (blocks > 0x7fffffffull) return MCF_ERR_SIZE;
  hipLaunchKernelGGL(copy_kernel, dim3((uint32_t)blocks), dim3(kStepBlock), MCF_COPY_LDS, (hipStream_t)stream,
                     (uint64_t)(uintptr_t)dst, (uint64_t)(uintptr_t)src, nvec);
  MCF_HIP(hipGetLastError());
  return MCF_OK;
}

int mcf_set_launch_pacing(int groups_per_cu, int head_sleep, int tail_sleep) {
  if (groups_per_cu > 128 || head_sleep > 4096 || tail_sleep > 4096) return MCF_ERR_SIZE;
  g_groups_per_cu.store(groups_per_cu, std::memory_order_relaxed);
  g_head_sleep.store(head_sleep, std::memory_order_relaxed);
  g_tail_sleep.store(tail_sleep, std::memory_order_relaxed);
  return MCF_OK;
}

int mcf_stream_mix(const void *const *reads, uint32_t n_read, void *const *writes, uint32_t n_write, uint64_t bytes,
                   uint32_t threads, uint32_t vectors_per_lane, uint32_t groups_per_cu, uint32_t store_policy, void *stream) {
  if (bytes == 0) return MCF_OK;
  if (!reads || (n_write && !writes)) return MCF_ERR_NULL;
  if (n_read > (uint32_t)kMaxMix || n_write > n_read) return MCF_ERR_SIZE;
  if ((threads != 64 && threads != 256) || (vectors_per_lane != 1 && vectors_per_lane != 2 && vectors_per_lane != 4) || groups_per_cu > 128 ||
      store_policy > (uint32_t)ST_AGENT_NT)
    return MCF_ERR_VARIANT;
  MixArgs a = {};
  for (uint32_t i = 0; i < n_read; ++i) {
    if (!reads[i]) return MCF_ERR_NULL;
    if (misaligned(reads[i], 16)) return MCF_ERR_ALIGN;
    a.rd[i] = (uint64_t)(uintptr_t)reads[i];
  }
  for (uint32_t i = 0; i < n_write; ++i) {
    if (!writes[i]) return MCF_ERR_NULL;
    if (misaligned(writes[i], 16)) return MCF_ERR_ALIGN;
    a.wr[i] = (uint64_t)(uintptr_t)writes[i];
  }
  if (bytes & 15) return MCF_ERR_ALIGN;
  a.nvec = bytes / 16;
  a.mask = 0;
  if ((a.nvec + (uint64_t)threads * vectors_per_lane - 1) / ((uint64_t)threads * vectors_per_lane) > 0x7fffffffull) return MCF_ERR_SIZE;
  const uint32_t lds = groups_per_cu ? lds_for_groups(groups_per_cu) : 0;
  hipStream_t st = (hipStream_t)stream;
  const uint32_t key = n_read * 16 + n_write;
  switch (key) {
    case 1 * 16 + 1: launch_mix<1, 1>(threads, vectors_per_lane, lds, store_policy, st, a); break;      // a copy
    case 1 * 16 + 0: launch_mix<1, 0>(threads, vectors_per_lane, lds, store_policy, st, a); break;      // read only
    case 4 * 16 + 3: launch_mix<4, 3>(threads, vectors_per_lane, lds, store_policy, st, a); break;      // plain bf16, MCF-SGD
    case 5 * 16 + 4: launch_mix<5, 4>(threads, vectors_per_lane, lds, store_policy, st, a); break;      // light, Kahan
    case 6 * 16 + 5: launch_mix<6, 5>(threads, vectors_per_lane, lds, store_policy, st, a); break;      // plus
    default: return MCF_ERR_VARIANT;
  }
  MCF_HIP(hipGetLastError());
  return MCF_OK;
}

uint64_t mcf_edq_scratch_bytes(uint64_t n) {
  return edq_partial_doubles(n) * sizeof(double);
}

int mcf_edq_component(int component, const void *delta, const void *th0, const void *dth0, const void *th1,
                      const void *dth1, uint64_t n, void *scratch_dev, void *stream, double *edq_dev) {
  if (!known_component(component)) return MCF_ERR_VARIANT;
  if (!edq_dev) return MCF_ERR_NULL;
  if (misaligned(edq_dev, 8)) return MCF_ERR_ALIGN;
  if (n == 0) return launch_edq_tail(nullptr, 0, nullptr, edq_dev, (hipStream_t)stream);
  if (!delta || !th0 || !th1 || !scratch_dev) return MCF_ERR_NULL;
  if (misaligned(scratch_dev, 8)) return MCF_ERR_ALIGN;
  return edq_launch(component, delta, th0, dth0, th1, dth1, n, (double *)scratch_dev, (hipStream_t)stream, edq_dev);
}

int mcf_edq_noalloc(int component, const void *delta, const void *th0, const void *dth0, const void *th1,
                    const void *dth1, uint64_t n, void *stream, double *edq_dev) {
  if (!known_component(component)) return MCF_ERR_VARIANT;
  if (!edq_dev) return MCF_ERR_NULL;
  if (misaligned(edq_dev, 8)) return MCF_ERR_ALIGN;
  if (n > kNoAllocMaxElems) return MCF_ERR_SIZE;
  if (n == 0) return launch_edq_tail(nullptr, 0, nullptr, edq_dev, (hipStream_t)stream);
  if (!delta || !th0 || !th1) return MCF_ERR_NULL;
  double *partials = nullptr;
  const int rc = scratch_of_current_device(&partials);
  if (rc != MCF_OK) return rc;
  // Nothing in the array has to start at zero: the first kernel writes one partial for every one of its
  // workgroups, and the two reduction kernels read exactly those and what they wrote themselves.
  return edq_launch(component, delta, th0, dth0, th1, dth1, n, partials, (hipStream_t)stream, edq_dev);
}

int mcf_edq(const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0, const uint16_t *th1,
            const uint16_t *dth1, uint64_t n, void *scratch_dev, void *stream, double *edq_dev) {
  return mcf_edq_component(MCF_COMPONENT_BF16, delta, th0, dth0, th1, dth1, n, scratch_dev, stream, edq_dev);
}

int mcf_fp32mw_plan_create(mcf_fp32mw_plan **out, const mcf_fp32mw_tensor *tensors, uint32_t count) {
  if (!out) return MCF_ERR_NULL;
  *out = nullptr;
  if (count && !tensors) return MCF_ERR_NULL;
  mcf_fp32mw_plan *p = nullptr;
  MCF_NO_THROW_BEGIN
  std::vector<Fp32Desc> descs;
  std::vector<Chunk> chunks;
  for (uint32_t i = 0; i < count; ++i) {
    const mcf_fp32mw_tensor &t = tensors[i];
    if (t.n == 0) continue;
    if (!t.theta || !t.master || !t.m || !t.v || !t.grad) return MCF_ERR_NULL;
    if (t.n > kMaxTensorElems) return MCF_ERR_SIZE;
    if (misaligned(t.theta, 2) || misaligned(t.grad, 2) || misaligned(t.master, 4) || misaligned(t.m, 4) || misaligned(t.v, 4))
      return MCF_ERR_ALIGN;
  }
  for (uint32_t i = 0; i < count; ++i) {
    const mcf_fp32mw_tensor &t = tensors[i];
    if (t.n == 0) continue;
    Fp32Desc d = {};
    d.theta = (uint64_t)(uintptr_t)t.theta;
    d.master = (uint64_t)(uintptr_t)t.master;
    d.m = (uint64_t)(uintptr_t)t.m;
    d.v = (uint64_t)(uintptr_t)t.v;
    d.grad = (uint64_t)(uintptr_t)t.grad;
    d.n = t.n;
    // 128-bit path: theta and grad share a phase, and each fp32 buffer is 16-byte aligned at the
    // element that sits on theta's 16-byte boundary
    const uint32_t ph = (uint32_t)((d.theta & (MCF_CHUNK_ALIGN - 1)) >> 1);
    bool ok = (d.grad & 15) == (d.theta & 15);
    const uint64_t f32s[3] = {d.master, d.m, d.v};
    for (uint64_t f : f32s) ok = ok && (((f - 4ull * ph) & 15) == 0);
    d.phase = ok ? ph : 0;
    d.scalar_only = ok ? 0 : 1;
    const uint64_t slots = slots_of(d.n, d.phase);
    const uint64_t nch = (slots + kSlotsPerChunk - 1) / kSlotsPerChunk;
    if (slots > 0xffffffffull || chunks.size() + nch > 0x7fffffffull) return MCF_ERR_SIZE;
    const uint32_t id = (uint32_t)descs.size();
    descs.push_back(d);
    for (uint64_t c = 0; c < nch; ++c) chunks.push_back(Chunk{id, (uint32_t)(c * kSlotsPerChunk)});
  }
  p = new (std::nothrow) mcf_fp32mw_plan();
  if (!p) return MCF_ERR_HIP;
  p->d_descs = nullptr;
  p->d_chunks = nullptr;
  p->device = -1;
  if (!chunks.empty() && hipGetDevice(&p->device) != hipSuccess) {
    (void)hipGetLastError();
    mcf_fp32mw_plan_destroy(p);
    return MCF_ERR_HIP;
  }
  p->n_chunks = (uint32_t)chunks.size();
  p->n_params = 0;
  for (const Fp32Desc &d : descs) p->n_params += d.n;
  p->d_descs = nullptr;
  p->d_chunks = nullptr;
  if (p->n_chunks) {
    bool ok = hipMalloc((void **)&p->d_descs, descs.size() * sizeof(Fp32Desc)) == hipSuccess &&
              hipMalloc((void **)&p->d_chunks, chunks.size() * sizeof(Chunk)) == hipSuccess &&
              hipMemcpy(p->d_descs, descs.data(), descs.size() * sizeof(Fp32Desc), hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(p->d_chunks, chunks.data(), chunks.size() * sizeof(Chunk), hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {
      (void)hipGetLastError();
      mcf_fp32mw_plan_destroy(p);
      return MCF_ERR_HIP;
    }
  }
  *out = p;
  return MCF_OK;
  MCF_NO_THROW_END(mcf_fp32mw_plan_destroy(p))
}

int mcf_fp32mw_plan_destroy(mcf_fp32mw_plan *plan) {
  if (!plan) return MCF_OK;
  int rc = MCF_OK;
  if (plan->d_descs && hipFree(plan->d_descs) != hipSuccess) rc = MCF_ERR_HIP;
  if (plan->d_chunks && hipFree(plan->d_chunks) != hipSuccess) rc = MCF_ERR_HIP;
  delete plan;
  return rc;
}

int mcf_fp32mw_step(mcf_fp32mw_plan *plan, const mcf_hyper *hyper, uint64_t step, void *stream) {
  if (!plan) return MCF_ERR_NULL;
  const int rc = mcfh::check_hyper(hyper, step);
  if (rc != MCF_OK) return rc;
  if (!plan->n_chunks) return MCF_OK;
  const int where = on_plan_device(plan->device);
  if (where != MCF_OK) return where;
  const double t = (double)step;
  Fp32Scalars s;
  s.b1 = (float)hyper->beta1;
  s.c1 = (float)(1.0 - hyper->beta1);
  s.b2 = (float)hyper->beta2;
  s.c2 = (float)(1.0 - hyper->beta2);
  s.bc1 = (float)(1.0 - std::pow(hyper->beta1, t));
  s.bc2 = (float)(1.0 - std::pow(hyper->beta2, t));
  s.e = (float)hyper->eps;
  s.lam = (float)hyper->weight_decay;
  s.na = (float)(-hyper->lr);
  s.write_through = plan->n_params * 4 >= kWriteThroughBytes ? 1u : 0u;
  hipLaunchKernelGGL(fp32mw_kernel, dim3(plan->n_chunks), dim3(kStepBlock), step_lds(MCF_FP32MW_LDS), (hipStream_t)stream, plan->d_descs, plan->d_chunks, s);
  MCF_HIP(hipGetLastError());
  return MCF_OK;
}

}  // extern "C"
