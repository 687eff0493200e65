// Expert FFNs of a MoE layer as sparse-sparse matrix multiplications on gfx950.
//
// What is computed: Algorithm 1 and sections 4.2-4.5 of the paper -- C = A x B[:, SEL]
// with A the 2:4-encoded weight (rows = output features), B the token matrix whose
// columns are picked by the selection array, the activation fused into the gate/up
// product and the routing-weight scaling fused into the down product, the
// intermediate kept in the bucketed ("compressed output") layout.
//
// How it is mapped to CDNA4 (this is not the paper's kernel, which was laid out for
// mma.sp / cp.async / ldmatrix):
//   * sparse operand = MFMA A operand of v_smfmac_f32_32x32x32_bf16; tokens are the N
//     dimension; every token row is contiguous along K, so the SEL gather is a set of
//     row-contiguous 16-byte loads (the "transposed packing of B" of section 4.4 is
//     simply the natural layout here);
//   * weights are stored offline in the lane order of the instruction (see
//     ssmm_common.h): a wave fetches an A operand with one coalesced 16-byte-per-lane
//     global load straight into registers -- no LDS, no transposition -- and the index
//     register with one 4-byte-per-lane load (section 4.2: metadata skips the inner
//     tiling step; section 4.4: metadata re-packed for aligned 32-bit access);
//   * only the token tile goes through LDS (shared by the waves of a block), XOR
//     swizzled at 16-byte granularity so that both the row-wise stores and the
//     operand-order reads are conflict free; a ring of stages, one barrier per stage;
//   * A operands of later stages are fetched into registers while the current
//     stage computes (register sets stand in for cp.async groups);
//   * one launch covers all experts: tile -> (expert, row tile, token tile) through an
//     XCD-aware map, token tiles enumerated on the device from expert_offsets, so
//     nothing is padded in memory and ragged tails are masked at the store.
//
// Two kernel families share this mapping: ssmm_kernel (SsmmTile), whose loads and waits the
// compiler schedules -- gathered (N,M,V) formats, layer variants at the large tile shape, token
// matrices of 4 GB and more -- and ssmm_kernel2 (SsmmPipe), the main path, with every
// global-memory instruction and wait placed by hand and resident blocks that walk the tile list.
// In both the MFMAs are asm: NO kernel here may spill (the build checks it) -- the compiler
// stores a spilled accumulator right behind the MFMA that defines it, before it is written.
#include <climits>
#include <cmath>
#include <cstdlib>

#include "ssmm_common.h"

namespace ssmm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kStageK = 64;   // reduction elements per pipeline stage (two MFMA k blocks)
// Consecutive blocks of a launch go round-robin over the accelerator dies (XCDs) of the device, each with
// an L2 of its own; the tile list is dealt to the blocks in this many contiguous shares so that the tiles
// that share operands meet in one L2.  Eight is the MI355X's count; on a device with another count the
// results are the same and only that locality is lost.
constexpr int kXcdGroups = 8;

struct SsmmArgs {
  const uint16_t* act;            // B rows: x [T][K] (gathered through sel) or h [P][K]
  const int32_t* sel;             // token id per bucket position; nullptr: rows are bucket positions
  const bf16x8* a0_vals;          // gate (or down) values, kernel-ready order
  const uint32_t* a0_meta;
  const bf16x8* a1_vals;          // up (gate/up kernel only)
  const uint32_t* a1_meta;
  const uint8_t* a0_vidx;         // (1,2,8) format only: source-row bits of the lane's segments
  const uint8_t* a1_vidx;
  const int32_t* expert_offsets;  // [E_total + 1]; null: one bucket that holds all `pairs` rows (the stand-alone product)
  const float* sel_w;             // routing weight per bucket position (down kernel only)
  uint16_t* out;                  // [P][rows] bf16
  int E_total;
  int rows;                       // output features of one expert (dense rows)
  int row_tiles;                  // 32-row tiles of the stored (compressed) matrix of one expert
  int K;                          // reduction length
  int actfn;                      // SSMM_ACT_*; 0: none.  gate/up kernels: h = act(gate) * up; others: out = act(sum), or sum * routing weight when 0
  int gN, gM;                     // gathered formats: N and M; row_tiles then counts DENSE 32-row tiles
  int vper;                       // compute-skipping kernels: k blocks of 32 per Sub-Row (V / 32)
  int stored_tiles;               // gathered formats: 32-row tiles of the stored matrix of one expert
  int n_tiles_max;                // upper bound on token tiles over all experts
  // split reduction (down projection of small buckets): block (.., split) multiplies stages
  // [split*kper, min(K/64, (split+1)*kper)) and writes unscaled fp32 partial sums
  int ksplit, kper;
  int64_t pairs;                  // P: rows of out / of one partial
  float* out_f32;                 // [ksplit][P][rows] fp32
};

// start of bucket i (i = E_total: the end of the last one)
__device__ inline int bucket_offset(const SsmmArgs& p, int i) {
  return p.expert_offsets ? p.expert_offsets[i] : (i == 0 ? 0 : (int)p.pairs);
}

// c += A(sparse 32x32 tile, 8 kept bf16 per lane) x B(32 x 32 tokens, 16 bf16 per lane).
// Written as asm with the accumulator constrained to the accumulation registers: all 16 x NA x NT
// accumulators of a wave then stay in AGPRs for the whole kernel and the 256 architectural
// VGPRs are left to operands and addresses (the compiler otherwise splits accumulators over
// both files and shuffles them every step).  volatile keeps the MFMAs in source order; loads
// and address arithmetic may still be scheduled around them.  An accumulator is touched again
// only NA*NT instructions later, far beyond the MFMA result latency.
template <int ABID>
__device__ inline void smfmac(f32x16& c, bf16x8 a, bf16x16 b, uint32_t idx) {
  if (ABID == 0)
    asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+a"(c) : "v"(a), "v"(b), "v"(idx));
  else
    asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3 abid:1" : "+a"(c) : "v"(a), "v"(b), "v"(idx));
}
// Same instruction with the accumulator in ordinary vector registers (tiles beyond the 256
// accumulation registers).
template <int ABID>
__device__ inline void smfmac_v(f32x16& c, bf16x8 a, bf16x16 b, uint32_t idx) {
  if (ABID == 0)
    asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+v"(c) : "v"(a), "v"(b), "v"(idx));
  else
    asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3 abid:1" : "+v"(c) : "v"(a), "v"(b), "v"(idx));
}
// The MFMAs are opaque to the compiler's hazard recogniser.  Where ordinary vector instructions
// produce MFMA source registers (the masked operands of the vector-wise format) or overwrite them
// right after, wait states keep the two apart (without them results were wrong on the device).
// Tying the registers to the asm keeps their producers before it and their consumers after it.
__device__ inline void mfma_guard(bf16x8& r, bool last) {
  if (last) asm volatile("s_nop 7" : "+v"(r));
  else asm volatile("" : "+v"(r));
}
// The last MFMA results must have been written before ordinary instructions read the accumulators.
__device__ inline void drain_mfma() { asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : : : "memory"); }

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  // round to nearest even; inputs are finite
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a = (a + 0x7FFFu + ((a >> 16) & 1u)) >> 16;
  b = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  return a | (b << 16);
}

__device__ inline float silu(float g) { return g / (1.0f + __expf(-g)); }
// silu with the hardware exponential and reciprocal (about 1 ulp each, far below the bf16
// rounding of the result); for very negative g the exponential overflows to +inf and the
// reciprocal gives the correct limit 0.
__device__ inline float silu_fast(float g) {
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.44269504088896f));
}
// The activation kinds of the boundary (SSMM_ACT_*), same hardware exponential and reciprocal:
// ReLU; SiLU g*sigmoid(g); tanh-form GELU 0.5 g (1 + tanh(u)) = g*sigmoid(2u), u = sqrt(2/pi) (g + 0.044715 g^3).
__device__ inline float activate(float g, int act) {
  if (act == SSMM_ACT_RELU) return fmaxf(g, 0.0f);
  const float z = act == SSMM_ACT_GELU_TANH ? 1.5957691216057308f * (g + 0.044715f * g * g * g) : g;
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z * -1.44269504088896f));
}
// two floats -> packed bf16, round to nearest even, in one instruction
__device__ inline uint32_t cvt_bf16x2(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16 bytes per lane from global memory straight into LDS (no register staging): lane l of
// the wave lands at LDS byte address lds_wave_base + 16*l; the global address is per lane.
// Written as one asm block so that M0 (the LDS base of the transfer) cannot change between
// its write and its use (the SALU write of M0 needs one wait state before the transfer reads
// it) and so that the compiler neither moves the transfer nor adds waits of its own for it.
// Its completion is implied by the completion of any register load issued after it (loads of
// one wave return in order), which is how the pipeline below awaits it.
__device__ inline void load16_to_lds(const void* src, uint32_t lds_wave_base) {
  asm volatile(
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off"
      :
      : "v"(src), "s"(lds_wave_base)
      : "memory");
}
// The compiler must have waited for the loads that produced these registers before this point.
__device__ inline void require_landed(bf16x8 v0, bf16x8 v1, uint32_t m) {
  asm volatile("" : : "v"(v0), "v"(v1), "v"(m) : "memory");
}
__device__ inline void require_landed(uint32_t m) { asm volatile("" : : "v"(m) : "memory"); }
__device__ inline void block_barrier() { asm volatile("s_barrier" : : : "memory"); }
__device__ inline void pin_order() { asm volatile("" : : : "memory"); }

__device__ inline uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// GATEUP: two weight matrices (gate, up) share the token tile; epilogue silu(g)*u.
// Otherwise one matrix (down); epilogue scales by the routing weight.
// Wave tile: MT row tiles (32 rows each, per matrix) x NT token tiles (32 tokens each).
// Block: WM x WN waves.  DS: register sets of A operands in flight (stages of 64
// reduction elements); the token tile has 2*DS LDS buffers.
//
// Pipeline (the fetch/compute overlap of Algorithm 1, with CDNA4 means).  A stage is 64
// reduction elements = two sparse MFMAs per (A operand, token tile) pair.  The A operands and
// index words of stage s go into register set s % DS, DS-1 steps before they are used; the
// token tile of stage s goes straight into LDS buffer s % (2 DS), 2 DS - 1 steps ahead, so its
// transfer is always older than the A loads of the same stage.  Step s: the compiler's own
// wait for the A registers of stage s (forced before the barrier by require_landed) therefore
// also covers this wave's part of the token tile of stage s; the barrier then makes every
// wave's part visible and tells that everybody has finished stage s-1; the loads of stages
// s+DS-1 (A) and s+2DS-1 (tokens) are issued into what stage s-1 used; stage s is multiplied.
//
// VEC: weights in the (1,2,8)+2:4 format (section 4.1 with N=1, M=2, V=8).  A stored row holds,
// per 8-element segment, the kept Sub-Row of a pair of dense rows.  The sparse MFMA spans four
// segments, so the accumulator cannot be re-targeted between segments the way section 4.3 does
// for V >= k_b; instead every A operand is issued twice, once with the segments of odd source
// rows zeroed (accumulating the even dense rows) and once with the even ones zeroed.  MFMA work
// equals the plain 2:4 case, weight bytes are halved.
//
// GEN: weights in a gathered (N,M,V)+2:4 format (V a multiple of 32 >= the MFMA's k block).  The
// wave's A streams are DENSE row tiles; lane (MFMA row i, half q) fetches its 16 bytes of a k
// block from the stored Sub-Row that holds its dense row there (a byte per dense row and k block,
// read one stage ahead of the operands it addresses), or takes zeros when the row was pruned;
// the index words of the two k blocks of a stage may come from different stored rows and are
// kept apart (the MFMA of k block 0 reads the low half of one, that of k block 1 the high half of
// the other).  MFMA work equals the plain 2:4 case, weight bytes shrink by N/M.
//
// SKIP (with VEC, V a multiple of 32): the compute skipping of sections 4.1 and 4.3 as far as this
// hardware allows it.  A Sub-Row then covers whole k blocks of the MFMA, so every stored operand is
// issued ONCE, into an intermediate accumulator tile (the paper's C_IR), and at the end of every
// V-wide block of the reduction the intermediate sums are moved to the accumulators of the dense rows
// they belong to: register r of a lane holds the same stored row in the intermediate tile and in the
// tiles of its two candidate dense rows, so the move is a selected add per register, by the source-row
// bit of the stored row in that block, and no value changes lanes.  Half the MFMAs of the masked
// scheme, plus two vector instructions and more per accumulator register and block -- measured
// against the masked scheme (bench.py --subrow-ab); it is not what the layer runs by default.
template <bool GATEUP, bool VEC, int MT, int NT, int WM, int WN, int DS, bool GEN = false, bool SKIP = false>
struct SsmmTile {
  static_assert(!(VEC && GEN), "one of the two vector-wise schemes");
  static_assert(!SKIP || VEC, "compute skipping is a way to run the (1,2,V) format");
  static constexpr int DB = 2 * DS;                // token-tile buffers
  static constexpr int NTH = 64 * WM * WN;
  static constexpr int NB = 32 * NT * WN;          // tokens per block tile
  static constexpr int NA = GATEUP ? 2 * MT : MT;  // A streams (stored 32-row tiles) per wave
  static constexpr int NP = VEC ? 2 : 1;           // MFMA passes (accumulators) per A operand
  static constexpr int CH = (NB * 8) / NTH;        // 16-byte chunks of the token tile per thread per stage
  static_assert((NB * 8) % NTH == 0, "token tile must split evenly over the threads");
  static constexpr int kStageBytes = NB * 8 * 16;
  static_assert(DB * kStageBytes <= 160 * 1024, "LDS");
  static_assert(NT <= 4, "load_tasks is spelled out for up to 4 token tiles");

  const char* av[NA];        // wave-uniform address of the next stage of each A stream
  const char* am[NA];        // same for the index words
  const char* ax[NA];        // same for the source-row bits (VEC)
  uint32_t lane16, lane4;    // this lane's byte offset inside an A operand / an index block
  const uint16_t* brow[CH];  // this lane's source of each staged 16-byte chunk, next stage
  uint32_t lds_dst[CH];      // wave-uniform LDS byte address of each staging instruction, buffer 0
  int lds_r[NT];             // 16-byte index of the token row this lane reads, per token tile
  int swz, ph;
  bf16x8 a[DS][NA][2];       // A operands of the stages in flight
  uint32_t idx[DS][NA];
  uint32_t idx1[DS][NA];     // GEN: index word whose high half belongs to the second k block
  const char* adesc[NA];     // GEN: wave-uniform address of the next stage's source bytes of each dense tile
  uint32_t dnext[NA];        // GEN: source bytes of the stage fetched next (low byte: first k block)
  uint32_t lane_i2, half32;  // GEN: 2 * MFMA row of the lane, 32 * its half
  uint32_t vx[DS][NA];       // VEC: 2 bits per k block (bits 0-1: first, bits 8-9: second k block)
  f32x16 acc[NA * NP][NT];   // VEC: accumulator 2x = even dense rows, 2x+1 = odd dense rows of stream x
  f32x16 tmp[SKIP ? NA : 1][NT];   // SKIP: intermediate sums of the stored rows over the current V-wide block
  int vper, ph_shift;              // SKIP: k blocks per Sub-Row (V / 32); 4 * (lane / 32)

  // ---- loads of one stage, as NA + CH separate tasks so that they can be spread between MFMAs
  // (a wave issues in order: a block of address arithmetic and loads in one place would leave
  // its SIMD's MFMA pipe idle meanwhile).  The fences keep every task where the source puts it.
  template <int BUF>
  __device__ inline void issue_b_chunk(int i) {
    load16_to_lds(brow[i], lds_dst[i] + BUF * kStageBytes);
    brow[i] += kStageK;
  }
  // A loads are always issued, so that the number of register loads per step is fixed (the
  // compiler's in-order load counting stays exact); past the last stage the pointers stop
  // advancing and the last stage is simply read again into a set nobody uses.
  template <int SET>
  __device__ inline void issue_a_stream(int x, bool more) {
    pin_order();
    if (GEN) {
      // The source bytes of the NEXT stage are requested first: loads return in order, so waiting
      // for them one step from now leaves this stage's operand loads, which are younger, in flight.
      const uint32_t d0 = dnext[x] & 0xFFu, d1 = (dnext[x] >> 8) & 0xFFu;
      adesc[x] += more ? 64 : 0;
      dnext[x] = *(const uint16_t*)(adesc[x] + lane_i2);
      pin_order();
      const uint32_t l0 = (d0 & 31u) + half32, l1 = (d1 & 31u) + half32;   // lane whose place in the stored tile holds the operand
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      a[SET][x][0] = (d0 & 0x80u) ? zero : *(const bf16x8*)(av[x] + l0 * 16);
      a[SET][x][1] = (d1 & 0x80u) ? zero : *(const bf16x8*)(av[x] + 1024 + l1 * 16);
      idx[SET][x] = (d0 & 0x80u) ? 0u : *(const uint32_t*)(am[x] + l0 * 4);
      idx1[SET][x] = (d1 & 0x80u) ? 0u : *(const uint32_t*)(am[x] + l1 * 4);
      av[x] += more ? 2048 : 0;
      am[x] += more ? 256 : 0;
      pin_order();
      return;
    }
    a[SET][x][0] = *(const bf16x8*)(av[x] + lane16);
    a[SET][x][1] = *(const bf16x8*)(av[x] + 1024 + lane16);
    idx[SET][x] = *(const uint32_t*)(am[x] + lane4);
    if (VEC) vx[SET][x] = *(const uint16_t*)(ax[x] + (lane4 >> 1));
    av[x] += more ? 2048 : 0;
    am[x] += more ? 256 : 0;
    if (VEC) ax[x] += more ? 128 : 0;
    pin_order();
  }
  template <int BUF>
  __device__ inline void issue_b() {
#pragma unroll
    for (int i = 0; i < CH; i++) issue_b_chunk<BUF>(i);
  }
  template <int SET>
  __device__ inline void issue_a(bool more) {
#pragma unroll
    for (int x = 0; x < NA; x++) issue_a_stream<SET>(x, more);
  }
  // the tasks of MFMA group G (of 2 NT groups per step): A streams first, then token-tile chunks
  template <int SET, int BUF, int G>
  __device__ inline void load_tasks(bool more, bool tokens) {
#pragma unroll
    for (int t = 0; t < NA + CH; t++) {
      if (t % (2 * NT) != G) continue;
      if (t < NA) issue_a_stream<SET>(t, more);
      else if (tokens) issue_b_chunk<BUF>(t - NA);
    }
  }
  __device__ inline bf16x16 read_b(const uint4* base, int n, int kb) const {
    union {
      uint4 u[2];
      bf16x16 v;
    } cvt;
    const int c0 = 4 * kb + 2 * ph;
    cvt.u[0] = base[lds_r[n] + (c0 ^ swz)];
    cvt.u[1] = base[lds_r[n] + ((c0 + 1) ^ swz)];
    return cvt.v;
  }
  // VEC: the operand with the segments of the other source row zeroed.  bits: bit 0 = source row
  // of the lane's first four values, bit 1 = of its last four; PASS = the source row wanted.
  template <int PASS>
  __device__ inline bf16x8 masked(bf16x8 v, uint32_t bits) const {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 w = __builtin_bit_cast(u32x4, v);
    const uint32_t m0 = ((bits & 1u) == (uint32_t)PASS) ? 0xFFFFFFFFu : 0u;
    const uint32_t m1 = (((bits >> 1) & 1u) == (uint32_t)PASS) ? 0xFFFFFFFFu : 0u;
    w.x &= m0;
    w.y &= m0;
    w.z &= m1;
    w.w &= m1;
    return __builtin_bit_cast(bf16x8, w);
  }
  // Token tile outermost: the first MFMAs need only the first token operand, and an operand
  // register is free for the next k block as soon as its MFMAs have been issued.
  // SKIP: intermediate sums -> accumulators of the dense rows, by the source-row bits of k block kb of the stage
  template <int SET>
  __device__ inline void merge(int kb) {
#pragma unroll
    for (int x = 0; x < NA; x++) {
      // bit i: MFMA row i of the stored tile came from the odd row of its pair (both lane halves hold it)
      const uint32_t rowbits = (uint32_t)__ballot(((vx[SET][x] >> (8 * kb)) & 1u) != 0);
      // register r of lane (token, half h) is stored row 16 h + r of the tile = MFMA row 8 (r / 4) + 4 h + r % 4
      const uint32_t mine = rowbits >> ph_shift;
#pragma unroll
      for (int n = 0; n < NT; n++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const bool odd = (mine >> (8 * (r / 4) + r % 4)) & 1u;
          const float v = tmp[x][n][r];
          acc[2 * x + 1][n][r] += odd ? v : 0.f;
          acc[2 * x][n][r] += odd ? 0.f : v;
          tmp[x][n][r] = 0.f;
        }
    }
  }
  // SKIP: one MFMA per stored operand and token tile (the compiler's own MFMA: it places the wait
  // states between the matrix pipe and the vector instructions of the merge)
  template <int SET, int BUF>
  __device__ inline void multiply_skip(const uint4* lds, bool more, bool tokens, int s) {
    constexpr int LSET = (SET + DS - 1) % DS, LBUF = (BUF + DB - 1) % DB;
    const uint4* base = lds + BUF * (NB * 8);
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
      bf16x16 bf[NT];
#pragma unroll
      for (int n = 0; n < NT; n++) bf[n] = read_b(base, n, kb);
#pragma unroll
      for (int n = 0; n < NT; n++)
#pragma unroll
        for (int x = 0; x < NA; x++) {
          if (kb == 0) tmp[x][n] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[SET][x][0], bf[n], tmp[x][n], (int)idx[SET][x], 0, 0);
          else tmp[x][n] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[SET][x][1], bf[n], tmp[x][n], (int)idx[SET][x], 0, 1);
        }
      if ((2 * s + kb + 1) % vper == 0) merge<SET>(kb);   // uniform over the wave
      if (kb == 0) {   // this step's loads, in two halves
#pragma unroll
        for (int t = 0; t < NA + CH; t++)
          if (t % 2 == 0) {
            if (t < NA) issue_a_stream<LSET>(t, more);
            else if (tokens) issue_b_chunk<LBUF>(t - NA);
          }
      } else {
#pragma unroll
        for (int t = 0; t < NA + CH; t++)
          if (t % 2 == 1) {
            if (t < NA) issue_a_stream<LSET>(t, more);
            else if (tokens) issue_b_chunk<LBUF>(t - NA);
          }
      }
    }
  }
  template <int SET, int BUF>
  __device__ inline void multiply(const uint4* lds, bool more, bool tokens) {
    constexpr int LSET = (SET + DS - 1) % DS, LBUF = (BUF + DB - 1) % DB;   // where this step's loads go
    const uint4* base = lds + BUF * (NB * 8);
    bf16x16 bf[NT];
#pragma unroll
    for (int n = 0; n < NT; n++) bf[n] = read_b(base, n, 0);
    bf16x8 op[NA * NP];
    if (VEC)   // the previous MFMAs may still be reading the registers the new operands will occupy
#pragma unroll
      for (int x = 0; x < NA; x++) mfma_guard(a[SET][x][0], x == NA - 1);
#pragma unroll
    for (int x = 0; x < NA; x++) {
      if (VEC) {
        op[2 * x] = masked<0>(a[SET][x][0], vx[SET][x]);
        op[2 * x + 1] = masked<1>(a[SET][x][0], vx[SET][x]);
      } else {
        op[x] = a[SET][x][0];
      }
    }
    if (VEC)   // ordinary vector instructions wrote the operands: keep the MFMAs a few cycles away
#pragma unroll
      for (int x = 0; x < NA * NP; x++) mfma_guard(op[x], x == NA * NP - 1);
#pragma unroll
    for (int n = 0; n < NT; n++) {
#pragma unroll
      for (int x = 0; x < NA * NP; x++) smfmac<0>(acc[x][n], op[x], bf[n], idx[SET][x / NP]);
      bf[n] = read_b(base, n, 1);
      if (n == 0) load_tasks<LSET, LBUF, 0>(more, tokens);
      if (n == 1) load_tasks<LSET, LBUF, 1>(more, tokens);
      if (n == 2) load_tasks<LSET, LBUF, 2>(more, tokens);
      if (n == 3) load_tasks<LSET, LBUF, 3>(more, tokens);
    }
    if (VEC)
#pragma unroll
      for (int x = 0; x < NA; x++) mfma_guard(a[SET][x][1], x == NA - 1);
#pragma unroll
    for (int x = 0; x < NA; x++) {
      if (VEC) {
        op[2 * x] = masked<0>(a[SET][x][1], vx[SET][x] >> 8);
        op[2 * x + 1] = masked<1>(a[SET][x][1], vx[SET][x] >> 8);
      } else {
        op[x] = a[SET][x][1];
      }
    }
    if (VEC)
#pragma unroll
      for (int x = 0; x < NA * NP; x++) mfma_guard(op[x], x == NA * NP - 1);
#pragma unroll
    for (int n = 0; n < NT; n++) {
#pragma unroll
      for (int x = 0; x < NA * NP; x++) smfmac<1>(acc[x][n], op[x], bf[n], GEN ? idx1[SET][x / NP] : idx[SET][x / NP]);
      if (n == 0) load_tasks<LSET, LBUF, NT + 0>(more, tokens);
      if (n == 1) load_tasks<LSET, LBUF, NT + 1>(more, tokens);
      if (n == 2) load_tasks<LSET, LBUF, NT + 2>(more, tokens);
      if (n == 3) load_tasks<LSET, LBUF, NT + 3>(more, tokens);
    }
  }
  // one pipeline step; s = stage index, KS = number of stages; U = s % (2 DS)
  template <int U>
  __device__ inline void step(int s, int KS, const uint4* lds) {
    constexpr int SET = U % DS, BUF = U % DB;
#pragma unroll
    for (int x = 0; x < NA; x++) {
      require_landed(a[SET][x][0], a[SET][x][1], idx[SET][x]);
      if (VEC) require_landed(vx[SET][x]);
      if (GEN) require_landed(idx1[SET][x]);
    }
    block_barrier();
    if constexpr (SKIP) multiply_skip<SET, BUF>(lds, s + DS < KS, s + DB - 1 < KS, s);
    else multiply<SET, BUF>(lds, s + DS < KS, s + DB - 1 < KS);
  }
  // the last KS % (2 DS) steps: nested, so that no later step follows a skipped one
  template <int U>
  __device__ inline void tail(int s, int KS, const uint4* lds) {
    if (s < KS) {
      step<U>(s, KS, lds);
      if constexpr (U + 1 < DB) tail<U + 1>(s + 1, KS, lds);
    }
  }
  template <int U>
  __device__ inline void full_trip(int s, int KS, const uint4* lds) {
    step<U>(s + U, KS, lds);
    if constexpr (U + 1 < DB) full_trip<U + 1>(s, KS, lds);
  }
};

// SPLITK: the block multiplies one slice of the reduction and writes unscaled fp32 partial sums
// (single-matrix kernels without activation only)
template <bool GATEUP, bool VEC, int MT, int NT, int WM, int WN, int DS, bool GEN = false, bool ANYACT = false, bool SPLITK = false, bool SKIP = false>
__global__ void __launch_bounds__(64 * WM * WN) ssmm_kernel(const SsmmArgs p) {
  static_assert(!(SPLITK && (GATEUP || ANYACT || VEC)), "partial sums: one matrix, no activation, plain or gathered format");
  using Tile = SsmmTile<GATEUP, VEC, MT, NT, WM, WN, DS, GEN, SKIP>;
  constexpr int NTH = Tile::NTH, NB = Tile::NB, NA = Tile::NA, CH = Tile::CH, NP = Tile::NP;
  __shared__ uint4 lds[Tile::DB * NB * 8];   // token-tile ring

  // ---- block -> (expert, row tile, token tile).  Consecutive blocks go round-robin over the
  // device's XCDs, so each XCD is given a contiguous range of the logical order "expert, then row tile,
  // then token tile": the blocks that run together on an XCD are then all token tiles of a few
  // neighbouring row tiles of one expert, so an A tile is pulled into that XCD's L2 once and
  // shared by all token tiles, and the expert's token tile is shared by the row tiles in flight.
  // The grid is sized for the worst case (every expert with a ragged tile); the XCD ranges are cut
  // from the tiles that exist, so that all eight get an equal share (with the ranges cut from the
  // grid the last XCDs got only blocks without a tile, and the first ones a second round).
  const int MTB = (p.row_tiles + MT * WM - 1) / (MT * WM) * (SPLITK ? p.ksplit : 1);
  // Buckets are looked at 64 at a time, one per lane (their offsets load side by side: one memory
  // latency per 64 buckets instead of one per bucket), tile counts summed by a wave scan; every wave
  // does the same work and arrives at the same, wave-uniform, answer.
  const int ln = threadIdx.x & 63;
  auto scan64 = [&](int base, int& lo, int& tok_tiles, int& tiles) {   // returns the inclusive sum of `tiles` over the lanes
    const int i = base + ln;
    lo = bucket_offset(p, min(i, p.E_total));
    const int hi = bucket_offset(p, min(i + 1, p.E_total));
    tok_tiles = (hi - lo + NB - 1) / NB;
    tiles = i < p.E_total ? tok_tiles * MTB : 0;
    int incl = tiles;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int below = __shfl_up(incl, d, 64);
      if (ln >= d) incl += below;
    }
    return incl;
  };
  int total = 0;
  for (int base = 0; base < p.E_total; base += 64) {
    int lo, tok_tiles, tiles;
    total += __shfl(scan64(base, lo, tok_tiles, tiles), 63, 64);
  }
  total = __builtin_amdgcn_readfirstlane(total);
  constexpr int nx = kXcdGroups;
  const int per_xcd = (total + nx - 1) / nx;
  if ((int)(blockIdx.x / nx) >= per_xcd) return;   // uniform over the block
  const int L = (blockIdx.x % nx) * per_xcd + blockIdx.x / nx;
  int e = -1, row0 = 0, nvalid = 0, mtb = 0, split = 0;
  {
    int carry = 0;   // tiles of the buckets before this round's
    for (int base = 0; base < p.E_total && e < 0; base += 64) {
      int lo, tok_tiles, tiles;
      const int incl = scan64(base, lo, tok_tiles, tiles);
      const int before = carry + incl - tiles;
      const uint64_t hit = __ballot(tiles > 0 && before <= L && L < before + tiles);
      if (hit) {
        const int src = __ffsll((unsigned long long)hit) - 1;
        const int lo_e = __builtin_amdgcn_readfirstlane(__shfl(lo, src, 64));
        const int tt_e = __builtin_amdgcn_readfirstlane(__shfl(tok_tiles, src, 64));
        const int local = L - __builtin_amdgcn_readfirstlane(__shfl(before, src, 64));
        const int hi_e = __builtin_amdgcn_readfirstlane(bucket_offset(p, base + src + 1));
        e = base + src;
        mtb = local / tt_e;
        if (SPLITK) {
          split = mtb % p.ksplit;
          mtb /= p.ksplit;
        }
        row0 = lo_e + (local % tt_e) * NB;
        nvalid = min(NB, hi_e - row0);
      }
      carry += __builtin_amdgcn_readfirstlane(__shfl(incl, 63, 64));
    }
  }
  if (e < 0) return;   // uniform over the block: beyond the last tile

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, lets addresses live in SGPRs
  const int wm = wv % WM, wn = wv / WM;
  const int MTtot = p.row_tiles, KB = p.K / 32;
  const int ks0 = SPLITK ? split * p.kper : 0;                                 // first stage of this block
  const int KS = SPLITK ? min(p.kper, p.K / kStageK - ks0) : p.K / kStageK;    // its number of stages

  Tile t;
  // ---- A streams of this wave: tile tt starts at unit tt*KB; a unit is 1 KB of values,
  // a pair of units shares 256 B of index words
  int tile_id[MT];
#pragma unroll
  for (int i = 0; i < MT; i++) {
    tile_id[i] = (mtb * WM + wm) * MT + i;
    const int64_t tt = (int64_t)e * MTtot + min(tile_id[i], MTtot - 1);   // clamp: loads stay in bounds
    // gathered formats: tt counts dense tiles; the stored Sub-Rows of dense tile d of an expert lie in its stored tile d*N/M
    const int64_t ts = GEN ? (int64_t)e * p.stored_tiles + (int64_t)min(tile_id[i], MTtot - 1) * p.gN / p.gM : tt;
    t.av[i] = (const char*)p.a0_vals + ts * KB * 1024 + (int64_t)ks0 * 2048;
    t.am[i] = (const char*)p.a0_meta + ts * (KB / 2) * 256 + (int64_t)ks0 * 256;
    if (VEC) t.ax[i] = (const char*)p.a0_vidx + tt * (KB / 2) * 128;
    if (GEN) t.adesc[i] = (const char*)p.a0_vidx + tt * (KB / 2) * 64 + (int64_t)ks0 * 64;
    if (GATEUP) {
      t.av[MT + i] = (const char*)p.a1_vals + ts * KB * 1024;
      t.am[MT + i] = (const char*)p.a1_meta + ts * (KB / 2) * 256;
      if (VEC) t.ax[MT + i] = (const char*)p.a1_vidx + tt * (KB / 2) * 128;
      if (GEN) t.adesc[MT + i] = (const char*)p.a1_vidx + tt * (KB / 2) * 64;
    }
  }
  t.lane16 = lane * 16;
  t.lane4 = lane * 4;
  if (GEN) {
    t.lane_i2 = (lane & 31) * 2;
    t.half32 = lane & 32;
#pragma unroll
    for (int x = 0; x < NA; x++) t.dnext[x] = *(const uint16_t*)(t.adesc[x] + t.lane_i2);   // stage 0
  }
  // ---- token rows this thread stages: staging instruction i of wave wv fills the 64 consecutive
  // 16-byte LDS slots starting at i*NTH + wv*64; slot (row r, position q) holds chunk q ^ (r & 7)
#pragma unroll
  for (int i = 0; i < CH; i++) {
    const int slot = i * NTH + wv * 64 + lane, r = slot >> 3, c = (slot & 7) ^ (r & 7);
    const int pos = row0 + min(r, nvalid - 1);   // rows past the ragged end re-read the last valid row
    const int64_t src = p.sel ? p.sel[pos] : pos;
    t.brow[i] = p.act + src * p.K + c * 8 + (int64_t)ks0 * kStageK;
    t.lds_dst[i] = __builtin_amdgcn_readfirstlane(lds_address(lds) + (i * NTH + wv * 64) * 16);
  }
  // ---- operand reads: lane (j, ph) reads 32 consecutive bytes of row j, half ph of the k block
  const int j = lane & 31;
  t.ph = lane >> 5;
#pragma unroll
  for (int n = 0; n < NT; n++) t.lds_r[n] = ((wn * NT + n) * 32 + j) * 8;
  t.swz = j & 7;   // (row & 7) == (j & 7): token tiles start at multiples of 32
#pragma unroll
  for (int x = 0; x < NA * NP; x++)
#pragma unroll
    for (int n = 0; n < NT; n++)
#pragma unroll
      for (int r = 0; r < 16; r++) t.acc[x][n][r] = 0.f;
  if (SKIP) {
    t.vper = p.vper;
    t.ph_shift = 4 * t.ph;
#pragma unroll
    for (int x = 0; x < NA; x++)
#pragma unroll
      for (int n = 0; n < NT; n++)
#pragma unroll
        for (int r = 0; r < 16; r++) t.tmp[x][n][r] = 0.f;
  }

  // ---- prologue: token tiles of the first 2 DS - 1 stages, then A operands of the first DS - 1
  constexpr int DB = Tile::DB;
  t.template issue_b<0>();
  if (KS > 1) t.template issue_b<1>();
  if (KS > 2) t.template issue_b<2>();
  if (DB > 4 && KS > 3) t.template issue_b<3 % DB>();
  if (DB > 4 && KS > 4) t.template issue_b<4 % DB>();
  if (DB > 6 && KS > 5) t.template issue_b<5 % DB>();
  if (DB > 6 && KS > 6) t.template issue_b<6 % DB>();
  t.template issue_a<0>(KS > 1);
  if (DS > 2) t.template issue_a<1 % DS>(KS > 2);
  if (DS > 3) t.template issue_a<2 % DS>(KS > 3);
  // ---- 2 DS steps per trip, so that buffer and register-set numbers are compile-time constants
  int s = 0;
  for (; s + DB <= KS; s += DB) t.template full_trip<0>(s, KS, lds);
  t.template tail<0>(s, KS, lds);
  drain_mfma();
  // whatever reads the sums reads them behind the drain (asm statements keep their order)
  if (!SKIP)
#pragma unroll
    for (int x = 0; x < NA * NP; x++)
#pragma unroll
      for (int n = 0; n < NT; n++) asm volatile("" : "+a"(t.acc[x][n]));

  // ---- epilogue: lane (j, ph) holds, per (stored row tile, token tile), 16 consecutive stored
  // rows 16*ph .. 16*ph+15 of token j.  Plain 2:4: these are 16 consecutive output features (two
  // 16-byte stores).  VEC: stored row r feeds dense rows 2r (even accumulator) and 2r+1 (odd
  // one), i.e. 32 consecutive output features (four 16-byte stores).  Ragged tail masked.
#pragma unroll
  for (int n = 0; n < NT; n++) {
    const int r = (wn * NT + n) * 32 + j;
    if (r >= nvalid) continue;
    const int64_t pos = row0 + r;
    const float scale = (GATEUP || !p.sel_w) ? 1.0f : p.sel_w[pos];
#pragma unroll
    for (int i = 0; i < MT; i++) {
      if (tile_id[i] >= MTtot) continue;
      auto value = [&](int pass, int q) {   // output of stored row q of this lane, dense row 2q+pass (VEC)
        const float g = t.acc[i * NP + pass][n][q];
        if (ANYACT) return GATEUP ? activate(g, p.actfn) * t.acc[(MT + i) * NP + pass][n][q] : activate(g, p.actfn);
        return GATEUP ? silu(g) * t.acc[(MT + i) * NP + pass][n][q] : g * scale;
      };
      if (SPLITK) {   // partial sums of this split, fp32, unscaled
        float4* dst = (float4*)(p.out_f32 + ((int64_t)split * p.pairs + pos) * p.rows + tile_id[i] * 32 + 16 * t.ph);
#pragma unroll
        for (int q = 0; q < 4; q++)
          dst[q] = make_float4(t.acc[i][n][4 * q], t.acc[i][n][4 * q + 1], t.acc[i][n][4 * q + 2], t.acc[i][n][4 * q + 3]);
        continue;
      }
      uint32_t o[8 * NP];
#pragma unroll
      for (int q = 0; q < 8 * NP; q++)
        o[q] = VEC ? pack_bf16x2(value(0, q), value(1, q)) : pack_bf16x2(value(0, 2 * q), value(0, 2 * q + 1));
      uint4* dst = (uint4*)(p.out + pos * p.rows + (tile_id[i] * 32 + 16 * t.ph) * NP);
#pragma unroll
      for (int q = 0; q < 2 * NP; q++) dst[q] = make_uint4(o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Main loop with every global-memory instruction and every wait placed by hand.
//
// Two measured facts of gfx950 shape it (one wave per SIMD, which the 256 accumulators force):
//   * a wave issues in order, a sparse MFMA occupies the matrix pipe for 32 cycles, and every
//     other instruction of the wave takes about 4-5 cycles of issue: more than some three
//     instructions per MFMA on average (a compare-and-branch counts as four) and the matrix pipe
//     starts to idle.  Measured with the memory instructions of a step and no bookkeeping: 21 ns
//     per MFMA; with five scalar instructions per MFMA more: 30 ns.  The loop therefore carries
//     almost no address arithmetic: the A streams are read through fixed scalar bases and ONE
//     vector offset that advances by a stage per step, the token-tile transfers through one scalar
//     base that advances and per-lane offsets that never change, the LDS ring position is a
//     compile-time constant of the unrolled step (immediate offsets of the LDS reads, immediate
//     addend of M0);
//   * the compiler counts outstanding loads only for instructions it emitted itself and cannot
//     see the global->LDS transfers at all, so its own waits cut the prefetch distance.  Here all
//     global loads are asm, the compiler emits no vmcnt wait inside the loop, and the waits are
//     written with exact counts.  A wave issues the same number of global-memory instructions in
//     every step (past the last stage the offsets stop advancing and the last stage is fetched
//     again into registers and LDS buffers nobody reads), which makes the counts constants:
//       step s issues, in this order, the A loads of stage s+DS-1 (LA_N instructions), then the
//       token-tile transfers of stage s+DS-1 (CH instructions);
//       the A operands of stage s are complete when at most CH + (DS-2)*LPS younger ones pend;
//       this wave's part of token-tile stage s+1 is complete when at most (DS-3)*LPS plus the
//       A loads of step s that precede the barrier pend.
// LDS reads stay ordinary loads: the compiler allocates the 8-register B operands and counts
// lgkmcnt exactly (LDS returns in order and nothing else uses that counter in the loop).
//
// Schedule of a step (stage = 64 reduction elements, G = 2 NT groups of NA*NP MFMAs, group =
// (k block, token tile)): the B operand of a group is read from LDS two groups ahead, also across
// the step boundary, so no MFMA waits for an LDS round trip after the barrier; the barrier that
// publishes stage s+1 sits in the middle of step s (at its start when a step has only two
// groups), after it the transfers that overwrite the buffer of stage s-1 are issued; exactly
// one memory instruction follows each MFMA.
//
// An asm load writes its destination long after the compiler believes it has: a destination
// must hold a live value from the load to the wait that covers it, or the compiler hands the
// register to somebody else in between (this is why the last steps' useless fetches are kept
// alive to the final wait).
template <int OFF>
__device__ inline void vm_load16(bf16x8& d, uint32_t voff, const char* base) {
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(d) : "v"(voff), "s"(base), "n"(OFF) : "memory");
}
__device__ inline void vm_load4(uint32_t& d, uint32_t voff, const char* base) {
  asm volatile("global_load_dword %0, %1, %2" : "=v"(d) : "v"(voff), "s"(base) : "memory");
}
__device__ inline void vm_load2(uint32_t& d, uint32_t voff, const char* base) {
  asm volatile("global_load_ushort %0, %1, %2" : "=v"(d) : "v"(voff), "s"(base) : "memory");
}
// 16 bytes per lane from base + voff straight into LDS at lds_wave + ADD + 16*lane (M0 carries the
// LDS address; one wait state between its write and the transfer).
template <int ADD>
__device__ inline void vm_to_lds16(uint32_t voff, const char* base, uint32_t lds_wave) {
  asm volatile(
      "s_add_u32 m0, %2, %3\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(voff), "s"(base), "s"(lds_wave), "n"(ADD)
      : "memory", "scc");
}
template <int N>
__device__ inline void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
constexpr int cmin(int a, int b) { return a < b ? a : b; }

// DS: register sets of A operands = LDS buffers of the token tile = stages in flight + 1.
template <bool GATEUP, bool VEC, int MT, int NT, int WM, int WN, int DS>
struct SsmmPipe {
  static constexpr int NTH = 64 * WM * WN;
  static constexpr int NB = 32 * NT * WN;          // tokens per block tile
  static constexpr int NA = GATEUP ? 2 * MT : MT;  // A streams (stored 32-row tiles) per wave
  static constexpr int NP = VEC ? 2 : 1;           // MFMA passes (accumulators) per A operand
  static constexpr int NM = NA * NP;               // MFMAs per group
  static constexpr int CH = (NB * 8) / NTH;        // token-tile transfers per thread per stage
  static constexpr int G = 2 * NT;                 // groups per step
  static constexpr int LA = 2;                     // groups between the LDS read of a B operand and its use
  static constexpr int GBAR = G >= 4 ? G / 2 : 0;  // group in front of which the barrier sits
  static constexpr int IPS = VEC ? 4 : 3;          // load instructions per A stream and stage
  static constexpr int LA_N = NA * IPS;            // A-side load instructions per step
  static constexpr int LPS = LA_N + CH;            // global-memory instructions per step
  // Where the step's global-memory instructions sit (slot = MFMA number in the step, GI * NM + m,
  // behind which the instruction is issued).  MFMA-bound shapes (TIGHT): one instruction per
  // MFMA -- MFMAs 0 and 1 of a group carry the LDS reads, the others first the A loads, then,
  // not before the barrier, the transfers.  Small token tiles have fewer MFMAs than loads (they
  // are bound by HBM, not by issue): the A loads are spread over the groups in front of the
  // barrier (the first group if the barrier opens the step), the transfers over the rest.
  static constexpr bool TIGHT = NM >= 3 && (LA_N > GBAR * (NM - 2) ? LA_N : GBAR * (NM - 2)) + CH <= G * (NM - 2);
  static constexpr int QB0 = LA_N > GBAR * (NM - 2) ? LA_N : GBAR * (NM - 2);
  static constexpr int SA = (G >= 4 ? GBAR : 1) * NM;   // loose placement: slots of the A loads
  static constexpr int slot_a(int i) { return TIGHT ? (i / (NM - 2)) * NM + 2 + i % (NM - 2) : i * SA / LA_N; }
  static constexpr int slot_b(int j) {
    return TIGHT ? ((QB0 + j) / (NM - 2)) * NM + 2 + (QB0 + j) % (NM - 2) : SA + j * (G * NM - SA) / CH;
  }
  static constexpr int a_before_bar() {
    int c = 0;
    for (int i = 0; i < LA_N; i++) c += slot_a(i) < GBAR * NM ? 1 : 0;
    return c;
  }
  static constexpr int A_BEFORE_BAR = a_before_bar();
  static_assert(slot_b(0) >= GBAR * NM && slot_b(CH - 1) < G * NM && slot_a(LA_N - 1) <= slot_b(0), "placement");
  static constexpr int CNT_A = cmin(63, CH + (DS - 2) * LPS);
  static constexpr int CNT_B = cmin(63, (DS - 3) * LPS + A_BEFORE_BAR);
  static constexpr int CNT_B0 = cmin(63, (DS - 2) * LPS);   // after the prologue: stage 0 of the token tile
  static constexpr int kStageBytes = NB * 128;
  static constexpr int NT_AGPR = cmin(NT, 256 / (16 * NM));   // token tiles whose accumulators fit the accumulation registers
  static constexpr int R = (DS * G) % 4 == 0 ? 4 : 3;         // B operand registers in rotation
  static_assert((NB * 8) % NTH == 0, "token tile must split evenly over the threads");
  static_assert(DS * kStageBytes <= 160 * 1024, "LDS");
  static_assert(DS * kStageBytes <= 65536, "LDS read offsets are 16-bit immediates");
  static_assert((DS * G) % R == 0, "B operand ring positions must repeat with the register sets");
  static_assert(DS >= 3, "pipeline depth");

  const char* av[NA];        // wave-uniform: stage 0 of each A stream (values)
  const char* am[NA];        // index words
  const char* ax[NA];        // source-row bits (VEC)
  uint32_t lane16, lane4, lane2;
  uint32_t va, vm, vxo;      // lane offset + offset of the stage fetched next, per section
  int sa, sb;                // stage the A offsets / the transfer base stand on
  const char* bbase;         // wave-uniform: token matrix + offset of the stage transferred next
  uint32_t vb[CH];           // per lane: offset of its 16-byte piece of each transfer from bbase
  uint32_t dma_w;            // wave-uniform LDS byte address of this wave's slot of transfer 0, buffer 0
  uint32_t rd[4];            // LDS byte offsets in a buffer: this lane's two 16-byte pieces of k block 0, then k block 1
  bf16x8 a[DS][NA][2];
  uint32_t idx[DS][NA];
  uint32_t vx[DS][NA];
  bf16x8 op[2][VEC ? NM : 1];   // VEC: masked operands of the two k blocks of the current stage
  bf16x16 bf[4];
  f32x16 acc[NM][NT];

  // q-th A-side load of a step (stream q / IPS); the offsets move on after the last one
  template <int SET>
  __device__ inline void issue_a_part(int q, int KS) {
    const int x = q / IPS, part = q % IPS;
    if (part == 0) vm_load16<0>(a[SET][x][0], va, av[x]);
    if (part == 1) vm_load16<1024>(a[SET][x][1], va, av[x]);
    if (part == 2) vm_load4(idx[SET][x], vm, am[x]);
    if (VEC && part == 3) vm_load2(vx[SET][x], vxo, ax[x]);
    if (q == LA_N - 1) {
      sa = __builtin_amdgcn_readfirstlane(min(sa + 1, KS - 1));
      va = lane16 + ((uint32_t)sa << 11);
      vm = lane4 + ((uint32_t)sa << 8);
      if (VEC) vxo = lane2 + ((uint32_t)sa << 7);
    }
  }
  // i-th transfer of a step into buffer BUF; the base moves on after the last one
  template <int BUF>
  __device__ inline void issue_b(int i, int KS) {
    if (i == 0) vm_to_lds16<BUF * kStageBytes + 0 * NTH * 16>(vb[0], bbase, dma_w);
    if (i == 1) vm_to_lds16<BUF * kStageBytes + 1 * NTH * 16>(vb[1 % CH], bbase, dma_w);
    if (i == 2) vm_to_lds16<BUF * kStageBytes + 2 * NTH * 16>(vb[2 % CH], bbase, dma_w);
    if (i == 3) vm_to_lds16<BUF * kStageBytes + 3 * NTH * 16>(vb[3 % CH], bbase, dma_w);
    if (i == 4) vm_to_lds16<BUF * kStageBytes + 4 * NTH * 16>(vb[4 % CH], bbase, dma_w);
    if (i == 5) vm_to_lds16<BUF * kStageBytes + 5 * NTH * 16>(vb[5 % CH], bbase, dma_w);
    static_assert(CH <= 6, "issue_b is spelled out for up to 6 transfers");
    if (i == CH - 1) {
      const int more = __builtin_amdgcn_readfirstlane(sb + 1 < KS ? 1 : 0);   // wave-uniform by construction; said so explicitly
      bbase += more * 2 * kStageK;
      sb += more;
    }
  }
  template <int SLOT, int BUF>
  __device__ inline void read_b_half(const char* ldsb, int kb, int n, int half) {
    typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
    const uint4 v = *(const uint4*)(ldsb + rd[2 * kb + half] + (BUF * kStageBytes + n * 4096));
    u32x8 w = __builtin_bit_cast(u32x8, bf[SLOT]);
    if (half == 0) {
      w.s0 = v.x; w.s1 = v.y; w.s2 = v.z; w.s3 = v.w;
    } else {
      w.s4 = v.x; w.s5 = v.y; w.s6 = v.z; w.s7 = v.w;
    }
    bf[SLOT] = __builtin_bit_cast(bf16x16, w);
  }
  template <int PASS>
  __device__ static inline bf16x8 masked(bf16x8 v, uint32_t bits) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 w = __builtin_bit_cast(u32x4, v);
    const uint32_t m0 = ((bits & 1u) == (uint32_t)PASS) ? 0xFFFFFFFFu : 0u;
    const uint32_t m1 = (((bits >> 1) & 1u) == (uint32_t)PASS) ? 0xFFFFFFFFu : 0u;
    w.x &= m0;
    w.y &= m0;
    w.z &= m1;
    w.w &= m1;
    return __builtin_bit_cast(bf16x8, w);
  }
  // MFMAs of token tiles that lie beyond the ragged end of a bucket are not skipped: a test per
  // MFMA costs as much issue time as it saves (measured: equal run times on all layer shapes).
  template <int ABID, int N>
  __device__ inline void multiply(f32x16& c, bf16x8 av_, bf16x16 bv_, uint32_t iv_) {
    if (N < NT_AGPR) smfmac<ABID>(c, av_, bv_, iv_);
    else smfmac_v<ABID>(c, av_, bv_, iv_);
  }
  template <int SET, int GI>
  __device__ inline void group(int KS, const char* ldsb) {
    constexpr int kb = GI / NT, n = GI % NT;
    constexpr int LSET = (SET + DS - 1) % DS;   // register set and LDS buffer this step fetches into
    constexpr int NEXT = (SET + 1) % DS;
    if (GI == GBAR) {
      wait_vm<CNT_B>();
      block_barrier();
    }
#pragma unroll
    for (int m = 0; m < NM; m++) {
      if (VEC) multiply<kb, n>(acc[m][n], op[kb][m], bf[(SET * G + GI) % R], idx[SET][m / NP]);
      else multiply<kb, n>(acc[m][n], a[SET][m][kb], bf[(SET * G + GI) % R], idx[SET][m]);
      constexpr int GL = GI + LA;
      if (m < 2) {   // halves of the B operand of the group after next
        if (GL < G) read_b_half<(SET * G + GL) % R, SET>(ldsb, GL / NT, GL % NT, m);
        else read_b_half<(SET * G + GL) % R, NEXT>(ldsb, (GL - G) / NT, (GL - G) % NT, m);
      }
#pragma unroll
      for (int i = 0; i < LA_N; i++)
        if (slot_a(i) == GI * NM + m) issue_a_part<LSET>(i, KS);
#pragma unroll
      for (int i = 0; i < CH; i++)
        if (slot_b(i) == GI * NM + m) issue_b<LSET>(i, KS);
    }
  }
  template <int SET, int GI>
  __device__ inline void groups(int KS, const char* ldsb) {
    group<SET, GI>(KS, ldsb);
    if constexpr (GI + 1 < G) groups<SET, GI + 1>(KS, ldsb);
  }
  // one pipeline step; KS = number of stages, SET = stage index % DS
  template <int SET>
  __device__ inline void step(int KS, const char* ldsb) {
    wait_vm<CNT_A>();
#pragma unroll
    for (int x = 0; x < NA; x++) {   // everything below sees the registers as written here, after the wait
      asm volatile("" : "+v"(a[SET][x][0]), "+v"(a[SET][x][1]), "+v"(idx[SET][x]));
      if (VEC) asm volatile("" : "+v"(vx[SET][x]));
    }
    if (VEC) {
      // the last MFMAs of the previous step may still be reading the operand registers
#pragma unroll
      for (int k = 0; k < 2; k++)
#pragma unroll
        for (int m = 0; m < NM; m++) mfma_guard(op[k][m], k == 1 && m == NM - 1);
#pragma unroll
      for (int k = 0; k < 2; k++)
#pragma unroll
        for (int x = 0; x < NA; x++) {
          op[k][2 * x] = masked<0>(a[SET][x][k], vx[SET][x] >> (8 * k));
          op[k][2 * x + 1] = masked<1>(a[SET][x][k], vx[SET][x] >> (8 * k));
        }
      // ordinary vector instructions wrote the operands: keep the MFMAs a few cycles away
#pragma unroll
      for (int k = 0; k < 2; k++)
#pragma unroll
        for (int m = 0; m < NM; m++) mfma_guard(op[k][m], k == 1 && m == NM - 1);
    }
    groups<SET, 0>(KS, ldsb);
  }
  // the steps before the first: stage V+DS-1 of the A streams and of the token tile
  template <int V>
  __device__ inline void prologue(int KS) {
    constexpr int SET = V + DS - 1;
#pragma unroll
    for (int q = 0; q < LA_N; q++) issue_a_part<SET>(q, KS);
#pragma unroll
    for (int i = 0; i < CH; i++) issue_b<SET>(i, KS);
    if constexpr (V + 1 < 0) prologue<V + 1>(KS);
  }
  template <int U>
  __device__ inline void tail(int s, int KS, const char* ldsb) {
    if (s < KS) {
      step<U>(KS, ldsb);
      if constexpr (U + 1 < DS) tail<U + 1>(s + 1, KS, ldsb);
    }
  }
  template <int U>
  __device__ inline void full_trip(int KS, const char* ldsb) {
    step<U>(KS, ldsb);
    if constexpr (U + 1 < DS) full_trip<U + 1>(KS, ldsb);
  }
  __device__ inline void loop(int KS, const char* ldsb) {
    int s = 0;
    for (; s + DS <= KS; s += DS) full_trip<0>(KS, ldsb);
    tail<0>(s, KS, ldsb);
  }
  // first DS-1 stages of a tile; the A bases, the transfer base and vb stand on its stage 0
  __device__ inline void start(int KS) {
    // opaque to the compiler, or it computes the offsets of all the prologue's stages once per
    // kernel and keeps them in (spills them from) registers across the multiplications
    asm volatile("" : "+v"(lane16), "+v"(lane4), "+v"(lane2));
    sa = sb = 0;
    va = lane16;
    vm = lane4;
    vxo = lane2;
    prologue<-(DS - 1)>(KS);
  }
  // The lane's offsets into the A streams, from the lane number, as they stand after start(): computed again
  // behind the epilogue so that they hold no registers while it runs.
  __device__ inline void refresh_offsets(int lane) {
    lane16 = lane * 16;
    lane4 = lane * 4;
    lane2 = lane * 2;
    asm volatile("" : "+v"(lane16), "+v"(lane4), "+v"(lane2));
    va = lane16 + ((uint32_t)sa << 11);
    vm = lane4 + ((uint32_t)sa << 8);
    if (VEC) vxo = lane2 + ((uint32_t)sa << 7);
  }
  // Cleared while the first stages are on their way: one dense MFMA 0 x 0 + 0 per accumulator tile
  // (output-only for the compiler: no zero tile to keep in, or spill from, registers).
  __device__ inline void clear() {
    float z = 0.f;
    asm volatile("s_nop 4" : "+v"(z));   // the operand register is written by a vector instruction just before
#pragma unroll
    for (int x = 0; x < NM; x++)
#pragma unroll
      for (int n = 0; n < NT; n++) {
        if (n < NT_AGPR) asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %1, 0" : "=a"(acc[x][n]) : "v"(z));
        else asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %1, 0" : "=v"(acc[x][n]) : "v"(z));
      }
    // the sparse MFMAs that accumulate into these tiles come hundreds of cycles later (waits, barrier,
    // LDS reads); drain the pipe all the same
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" : : : "memory");
  }
  // all steps of a tile; on return every load and transfer has landed, every MFMA has retired and
  // every wave of the block has left the LDS buffers
  __device__ inline void mainloop(int KS, const char* ldsb) {
    wait_vm<CNT_B0>();             // this wave's part of stage 0 of the token tile (memory instructions issued since only make the wait stricter)
    block_barrier();
    read_b_half<0, 0>(ldsb, 0, 0, 0);
    read_b_half<0, 0>(ldsb, 0, 0, 1);
    read_b_half<1, 0>(ldsb, 1 / NT, 1 % NT, 0);
    read_b_half<1, 0>(ldsb, 1 / NT, 1 % NT, 1);
    loop(KS, ldsb);
    wait_vm<0>();                  // re-fetched stages must not land in the LDS of a later tile
#pragma unroll
    for (int d = 0; d < DS; d++)
#pragma unroll
      for (int x = 0; x < NA; x++) {
        asm volatile("" : : "v"(a[d][x][0]), "v"(a[d][x][1]), "v"(idx[d][x]));
        if (VEC) asm volatile("" : : "v"(vx[d][x]));
      }
    drain_mfma();
    block_barrier();
  }
};

constexpr int kMaxBuckets = 512;   // experts (routed + shared) one launch can serve: size of the bucket table in LDS

// 4 bytes per lane from base + voff straight into LDS at lds_wave + ADD + 4*lane
__device__ inline void vm_to_lds4(uint32_t voff, const char* base, uint32_t lds_wave) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dword %0, %1"
      :
      : "v"(voff), "s"(base), "s"(lds_wave)
      : "memory");
}

// OCC: waves per SIMD the register budget is set for (2 for the small, HBM-bound tiles)
// SPLITK: the block multiplies one slice of the reduction and writes fp32 partial sums (down projection only)
//
// A block walks tiles L, L + slots, ... of its XCD's share of the tile list (slots = blocks per
// XCD).  The first stages of a tile are requested before the epilogue of the tile before it runs,
// so that their latency and the tile's address set-up hide under the epilogue's arithmetic.
// Between the multiplications nothing waits for global memory: the bucket table sits in LDS, and
// the token rows (and routing weights) of the next tile are transferred into LDS while the
// current tile is multiplied.
// ANYACT: the epilogue applies the activation kind of the call (gate/up: act(gate) * up; one matrix:
// act(sum), no scaling) instead of the kernel's usual one (SiLU * up; sum * routing weight)
template <bool GATEUP, bool VEC, int MT, int NT, int WM, int WN, int DS, int OCC, bool SPLITK, bool ANYACT = false>
__global__ void __launch_bounds__(64 * WM * WN, OCC) ssmm_kernel2(const SsmmArgs p) {
  static_assert(!(GATEUP && SPLITK), "the gate/up epilogue needs whole sums");
  static_assert(!(ANYACT && SPLITK), "partial sums carry no activation");
  using Pipe = SsmmPipe<GATEUP, VEC, MT, NT, WM, WN, DS>;
  constexpr int NTH = Pipe::NTH, NB = Pipe::NB, CH = Pipe::CH, NP = Pipe::NP;
  constexpr int NBW = (NB + 63) / 64;      // waves that fetch routing weights
  __shared__ uint4 lds[DS * NB * 8];       // token-tile ring
  __shared__ int32_t side_sel[CH * NTH];   // token row of every 16-byte slot this block stages, for the tile after the current one
  __shared__ float side_w[2][NBW * 64];    // routing weights of the tile's rows (two tiles alive: the one multiplied, the one before it)
  __shared__ int32_t tab_cum[kMaxBuckets + 1], tab_off[kMaxBuckets + 1];   // tiles in front of each bucket; bucket offsets

  // tile -> (expert, row tile, token tile): see ssmm_kernel.  The number of tiles is known only
  // here; each XCD gets an equal share of it.  Order inside an expert: row tile, then split of the
  // reduction, then token tile, so that the token tiles that share weights run side by side on
  // one XCD.
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wv % WM, wn = wv / WM;
  const int MTB = (p.row_tiles + MT * WM - 1) / (MT * WM) * (SPLITK ? p.ksplit : 1);
  // Tile table, built by the first wave: 64 buckets per round, their offsets loaded side by side
  // (one memory latency per round instead of one per bucket), tile counts summed by a wave scan.
  if (wv == 0) {
    int carry = 0;
    for (int base = 0; base <= p.E_total; base += 64) {
      const int i = base + lane;
      const int lo = bucket_offset(p, min(i, p.E_total));
      const int hi = bucket_offset(p, min(i + 1, p.E_total));
      const int tiles = i < p.E_total ? (hi - lo + NB - 1) / NB * MTB : 0;
      int incl = tiles;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int below = __shfl_up(incl, d, 64);
        if (lane >= d) incl += below;
      }
      if (i <= p.E_total) {
        tab_cum[i] = carry + incl - tiles;
        tab_off[i] = lo;
      }
      carry += __shfl(incl, 63, 64);
    }
  }
  __syncthreads();
  const int total = __builtin_amdgcn_readfirstlane(tab_cum[p.E_total]);
  constexpr int nx = kXcdGroups;
  const int per_xcd = (total + nx - 1) / nx;
  const int xcd = blockIdx.x % nx, nslots = gridDim.x / nx;
  struct Where {
    int row0, nvalid, mtb, split, e;
  };
  // ln: the lane number, computed again (two instructions) in front of every phase between two
  // multiplications, so that neither it nor what the tile look-up, the row requests, the address
  // set-up and the epilogue derive from it lives in (and spills from) registers across them
  auto lane_again = [] {
    uint32_t ones = ~0u;
    asm volatile("" : "+s"(ones));
    return (int)__builtin_amdgcn_mbcnt_hi(ones, __builtin_amdgcn_mbcnt_lo(ones, 0u));
  };
  int ln = lane;
  // the bucket of tile L = number of buckets i >= 1 with tab_cum[i] <= L (one bucket per lane and round)
  auto locate = [&](int li, Where& w) -> bool {
    const int L = li < per_xcd ? xcd * per_xcd + li : total;
    if (L >= total) return false;   // beyond the last tile (uniform over the block)
    int e = 0;
    for (int base = 0; base < p.E_total; base += 64) {
      const int i = base + ln + 1;
      const bool le = i <= p.E_total && tab_cum[min(i, p.E_total)] <= L;
      e += __popcll(__ballot(le));
    }
    e = __builtin_amdgcn_readfirstlane(e);
    const int before = __builtin_amdgcn_readfirstlane(tab_cum[e]);
    const int lo = __builtin_amdgcn_readfirstlane(tab_off[e]), hi = __builtin_amdgcn_readfirstlane(tab_off[e + 1]);
    const int tiles = (hi - lo + NB - 1) / NB;
    const int local = L - before;
    w.e = e;
    w.mtb = local / tiles;
    w.split = 0;
    if (SPLITK) {
      w.split = w.mtb % p.ksplit;
      w.mtb /= p.ksplit;
    }
    w.row0 = lo + (local % tiles) * NB;
    w.nvalid = min(NB, hi - w.row0);
    return true;
  };

  const int MTtot = p.row_tiles, KB = p.K / 32;
  // Every tile walks the reduction from stage 0: the token tiles of one expert that share a row
  // tile run side by side on one XCD and find each other's weights in its L2 only while they
  // stay at the same stage (starting each at a stage of its own was measured: 1.5x slower).

  Pipe t;
  t.lane16 = lane * 16;
  t.lane4 = lane * 4;
  t.lane2 = lane * 2;
  t.dma_w = __builtin_amdgcn_readfirstlane(lds_address(lds) + wv * 1024);
  // operand reads: lane (j, ph) reads pieces 2ph, 2ph+1 (k block 0) and 4+2ph, 5+2ph (k block 1)
  // of row j of each of its token tiles
  auto operand_offsets = [&](int l) {
    const int j = l & 31, ph = l >> 5, swz = j & 7;   // (row & 7) == (j & 7): token tiles start at multiples of 32
    const uint32_t rowb = (uint32_t)((wn * NT * 32 + j) * 128);
    t.rd[0] = rowb + (((2 * ph) ^ swz) << 4);
    t.rd[1] = rowb + (((2 * ph + 1) ^ swz) << 4);
    t.rd[2] = rowb + (((4 + 2 * ph) ^ swz) << 4);
    t.rd[3] = rowb + (((5 + 2 * ph) ^ swz) << 4);
  };
  operand_offsets(lane);

  const uint32_t sel_w0 = __builtin_amdgcn_readfirstlane(lds_address(side_sel) + wv * 256);
  const uint32_t w_w0 = __builtin_amdgcn_readfirstlane(lds_address(side_w) + wv * 256);
  // Token rows this thread stages: transfer i of wave wv fills the 64 consecutive 16-byte LDS
  // slots starting at i*NTH + wv*64; slot (row r, position q) holds piece q ^ (r & 7) of the row.
  // Rows past the ragged end re-read the last valid row.  The row ids (through SEL) and the
  // routing weights of tile w go global -> LDS without passing registers; they have landed when
  // the multiplication that follows has ended.
  auto request_rows = [&](const Where& w, int parity) {
    if (p.sel) {
#pragma unroll
      for (int i = 0; i < CH; i++) {
        const int slot = i * NTH + wv * 64 + ln, r = slot >> 3;
        const int pos = w.row0 + min(r, w.nvalid - 1);
        vm_to_lds4((uint32_t)pos * 4u, (const char*)p.sel, sel_w0 + i * NTH * 4);
      }
    }
    if (!GATEUP && p.sel_w && wv < NBW) {
      const int pos = w.row0 + min(wv * 64 + ln, w.nvalid - 1);
      vm_to_lds4((uint32_t)pos * 4u, (const char*)p.sel_w, w_w0 + parity * (NBW * 256));
    }
  };
  auto rows_of = [&](const Where& w, int (&src)[CH]) {
#pragma unroll
    for (int i = 0; i < CH; i++) {
      const int slot = i * NTH + wv * 64 + ln, r = slot >> 3;
      src[i] = p.sel ? side_sel[slot] : w.row0 + min(r, w.nvalid - 1);
    }
  };

  Where cur = {}, prev = {};
  // per-lane offsets of the token-tile transfers of tile cur (rel: counted from the tile's first row)
  auto transfer_offsets = [&](bool rel) {
    int src[CH];
    rows_of(cur, src);
#pragma unroll
    for (int i = 0; i < CH; i++) {
      const int slot = i * NTH + wv * 64 + ln, r = slot >> 3, c = (slot & 7) ^ (r & 7);
      const int row = rel ? min(r, cur.nvalid - 1) : src[i];
      t.vb[i] = (uint32_t)(((int64_t)row * p.K + c * 8) * 2);
    }
#pragma unroll
    for (int i = 0; i < CH; i++) asm volatile("" : "+v"(t.vb[i]));   // as computed here, not carried over from the first time
  };
  int parity = 0;   // of the tile the accumulators belong to when the epilogue runs
  // epilogue of the tile whose sums the accumulators hold: see ssmm_kernel
  auto epilogue = [&]() {
    const int j = ln & 31, ph = ln >> 5;
#pragma unroll
    for (int n = 0; n < NT; n++) {
      const int r = (wn * NT + n) * 32 + j;
      if (r >= prev.nvalid) continue;
      const int64_t pos = prev.row0 + r;
      const float scale = (GATEUP || !p.sel_w) ? 1.0f : side_w[parity][r];
#pragma unroll
      for (int i = 0; i < MT; i++) {
        const int tile = (prev.mtb * WM + wm) * MT + i;
        if (tile >= MTtot) continue;
        auto value = [&](int pass, int q) {
          const float g = t.acc[i * NP + pass][n][q];
          if (ANYACT) return GATEUP ? activate(g, p.actfn) * t.acc[(MT + i) * NP + pass][n][q] : activate(g, p.actfn);
          return GATEUP ? silu_fast(g) * t.acc[(MT + i) * NP + pass][n][q] : g * scale;
        };
        if (SPLITK) {   // partial sums of this split, fp32, unscaled, same feature order
          float4* dst = (float4*)(p.out_f32 + ((int64_t)prev.split * p.pairs + pos) * p.rows + (tile * 32 + 16 * ph) * NP);
#pragma unroll
          for (int q = 0; q < 4 * NP; q++) {
            if (VEC)
              dst[q] = make_float4(t.acc[i * NP][n][2 * q], t.acc[i * NP + 1][n][2 * q], t.acc[i * NP][n][2 * q + 1],
                                   t.acc[i * NP + 1][n][2 * q + 1]);
            else
              dst[q] = make_float4(t.acc[i][n][4 * q], t.acc[i][n][4 * q + 1], t.acc[i][n][4 * q + 2], t.acc[i][n][4 * q + 3]);
          }
          continue;
        }
        uint4* dst = (uint4*)(p.out + pos * p.rows + (tile * 32 + 16 * ph) * NP);
#pragma unroll
        for (int half = 0; half < NP; half++) {   // 32 bytes at a time (registers)
          uint32_t o[8];
#pragma unroll
          for (int q = 0; q < 8; q++) {
            const int qq = half * 8 + q;
            o[q] = VEC ? cvt_bf16x2(value(0, qq), value(1, qq)) : cvt_bf16x2(value(0, 2 * qq), value(0, 2 * qq + 1));
          }
          dst[2 * half] = make_uint4(o[0], o[1], o[2], o[3]);
          dst[2 * half + 1] = make_uint4(o[4], o[5], o[6], o[7]);
          if (VEC) __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };

  int li = blockIdx.x / nx;
  bool have_cur = locate(li, cur), have_prev = false;
  if (!have_cur) return;
  request_rows(cur, 1);
  wait_vm<0>();
  block_barrier();      // the routing weights are read by other waves than the one that fetched them
  int KS = 0;
  for (;;) {
    // Order: aim the streams at the tile and request its first stages; epilogue of the tile
    // multiplied before (hides their latency); request the rows of the tile after; clear; multiply.
    // Nothing is in flight here: the multiplication ended with every load landed.  Said once more
    // for the build's check of the assembly, which follows every path through the loop without
    // correlating its branches (the pass that only runs the last epilogue requests no stages).
    wait_vm<0>();
    ln = lane_again();
    if (have_cur) {
      const int ks0 = SPLITK ? cur.split * p.kper : 0;                       // first stage of this tile
      KS = SPLITK ? min(p.kper, p.K / kStageK - ks0) : p.K / kStageK;        // its number of stages
      asm volatile("" : "+s"(KS));   // per tile: nothing derived from it is carried (spilled) across the multiplication
#pragma unroll
      for (int i = 0; i < MT; i++) {
        const int tile = (cur.mtb * WM + wm) * MT + i;
        const int64_t tt = (int64_t)cur.e * MTtot + min(tile, MTtot - 1);   // clamp: loads stay in bounds
        t.av[i] = (const char*)p.a0_vals + tt * KB * 1024 + (int64_t)ks0 * 2048;
        t.am[i] = (const char*)p.a0_meta + tt * (KB / 2) * 256 + (int64_t)ks0 * 256;
        if (VEC) t.ax[i] = (const char*)p.a0_vidx + tt * (KB / 2) * 128 + (int64_t)ks0 * 128;
        if (GATEUP) {
          t.av[MT + i] = (const char*)p.a1_vals + tt * KB * 1024;
          t.am[MT + i] = (const char*)p.a1_meta + tt * (KB / 2) * 256;
          if (VEC) t.ax[MT + i] = (const char*)p.a1_vidx + tt * (KB / 2) * 128;
        }
      }
      // 32-bit per-lane offsets.  Rows gathered through SEL: from the start of the token matrix
      // (the host has checked that it is smaller than 4 GB).  Consecutive rows: from the tile's
      // first row, which goes into the scalar base, so the matrix may have any size.
      // (Plain 2:4 single-matrix kernels only: the others have no register to spare for it.)
      constexpr bool REL = !GATEUP && !VEC;
      const bool rel = REL && !p.sel;
      t.bbase = (const char*)p.act + (int64_t)ks0 * (2 * kStageK) + (rel ? (int64_t)cur.row0 * p.K * 2 : 0);
      transfer_offsets(rel);
      t.start(KS);
    }
    ln = lane_again();
    if (have_prev) epilogue();
    if (!have_cur) break;
    ln = lane_again();
    // The kernels with the fewest registers to spare (vector-wise format on 160-token tiles, 512 x 128 tiles) compute the
    // per-lane offsets once more, so that they occupy no registers while the epilogue runs (the row ids
    // are still in LDS: the rows of the tile after cur are requested below).
    if constexpr ((VEC && NT == 5) || (!GATEUP && !VEC && MT == 4 && NT == 4)) {
      transfer_offsets((!GATEUP && !VEC) && !p.sel);
      operand_offsets(ln);
      t.refresh_offsets(ln);
    }
    Where next = {};
    li += nslots;
    const bool have_next = locate(li, next);
    parity ^= 1;          // now the parity of cur
    block_barrier();      // every wave has read the routing weights of the tile before cur
    if (have_next) request_rows(next, parity ^ 1);

    t.clear();
    t.mainloop(KS, (const char*)lds);

    prev = cur;
    have_prev = true;
    cur = next;
    have_cur = have_next;
  }
}

// y[t] = sum over slots, in slot order, of yp[inv[t][slot]]; fp32 adds, bf16 out.
// One thread per (token, 8 consecutive features).
__global__ void __launch_bounds__(256) combine_kernel(const uint16_t* __restrict__ yp, const int32_t* __restrict__ inv,
                                                      int T, int H, int slots, uint16_t* __restrict__ y) {
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int hc = H / 8;
  if (tid >= (int64_t)T * hc) return;
  const int t = (int)(tid / hc), c = (int)(tid % hc);
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  // eight slots at a time: first their positions, then their rows (all loads of a group in flight
  // together), then the adds in slot order
  for (int j0 = 0; j0 < slots; j0 += 8) {
    const int nj = min(8, slots - j0);
    int64_t pos[8];
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) pos[u] = u < nj ? inv[(int64_t)t * slots + j0 + u] : 0;
#pragma unroll
    for (int u = 0; u < 8; u++)
      if (u < nj) v[u] = *(const uint4*)(yp + pos[u] * H + c * 8);
#pragma unroll
    for (int u = 0; u < 8; u++) {
      if (u >= nj) break;
      const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int q = 0; q < 4; q++) {
        s[2 * q] += __uint_as_float(w[q] << 16);
        s[2 * q + 1] += __uint_as_float(w[q] & 0xFFFF0000u);
      }
    }
  }
  *(uint4*)(y + (int64_t)t * H + c * 8) =
      make_uint4(pack_bf16x2(s[0], s[1]), pack_bf16x2(s[2], s[3]), pack_bf16x2(s[4], s[5]), pack_bf16x2(s[6], s[7]));
}

// Same sum when the down projection was split along its reduction:
// y[t] = sum over slots of sel_w[pos] * (sum over splits, in split order, of part[split][pos]).
__global__ void __launch_bounds__(256) combine_split_kernel(const float* __restrict__ part, const int32_t* __restrict__ inv,
                                                            const float* __restrict__ sel_w, int T, int H, int slots,
                                                            int ksplit, int64_t P, uint16_t* __restrict__ y) {
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int hc = H / 8;
  if (tid >= (int64_t)T * hc) return;
  const int t = (int)(tid / hc), c = (int)(tid % hc);
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int jj = 0; jj < slots; jj++) {
    const int64_t pos = inv[(int64_t)t * slots + jj];
    const float w = sel_w[pos];
    float a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int k = 0; k < ksplit; k++) {
      const float4* src = (const float4*)(part + ((int64_t)k * P + pos) * H + c * 8);
      const float4 v0 = src[0], v1 = src[1];
      a[0] += v0.x; a[1] += v0.y; a[2] += v0.z; a[3] += v0.w;
      a[4] += v1.x; a[5] += v1.y; a[6] += v1.z; a[7] += v1.w;
    }
#pragma unroll
    for (int q = 0; q < 8; q++) s[q] += w * a[q];
  }
  *(uint4*)(y + (int64_t)t * H + c * 8) =
      make_uint4(cvt_bf16x2(s[0], s[1]), cvt_bf16x2(s[2], s[3]), cvt_bf16x2(s[4], s[5]), cvt_bf16x2(s[6], s[7]));
}

inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

// Tuning overrides of the tile and split rules below.  The library as built for use has none: every
// knob reads as unset and the rules alone decide, so what a call computes depends on its arguments
// only.  A build with -DSSMM_TUNING (sweeps on the device, never the shipped library) reads them from
// the environment at every call.
constexpr int kUnset = INT32_MIN;
inline int knob(const char* name) {
#ifdef SSMM_TUNING
  const char* v = getenv(name);
  return v ? atoi(v) : kUnset;
#else
  (void)name;
  return kUnset;
#endif
}

// Compute units of the current device, asked for once per device.
struct DeviceShape {
  int cus;
};
inline int device_shape(DeviceShape* out) {
  constexpr int kMaxDevices = 64;
  static int known[kMaxDevices];   // 0: not asked yet
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SSMM_EHIP;
  int cus = __atomic_load_n(&known[dev], __ATOMIC_ACQUIRE);
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return SSMM_EHIP;
    __atomic_store_n(&known[dev], cus, __ATOMIC_RELEASE);
  }
  out->cus = cus;
  return SSMM_OK;
}
// Compute units the tile and split rules reckon with: those of the current device; where none is
// visible (size queries on a host without a GPU) those of the MI355X.
inline int compute_units() {
  DeviceShape d;
  return device_shape(&d) == SSMM_OK ? d.cus : 256;
}


// Tile shape by the mean bucket size: 2 = large buckets (MFMA-bound: 128/160-token tiles, 256 or
// 512 rows per block), 1 = 128-token tiles with few rows per block (HBM-bound: the tile is wide
// enough that most experts need one, so their weights are streamed once, and narrow in rows so
// that there are many blocks), 0 = 32-token tiles (a handful of tokens per expert).
inline int tile_shape(int64_t P, int E_total) {
  const int64_t mean = P / E_total;
  return mean >= 192 ? 2 : mean > 20 ? 1 : 0;
}
// Splits of the down projection's reduction.  Small buckets give the down kernel few blocks
// (rows / 256 row tiles x one token tile per expert that has tokens); splitting the reduction
// gives every CU a block to stream weights with.  Measured on the Mixtral-shaped layer at 16 and
// 256 tokens: two splits (256 blocks) are best, more only add partial-sum traffic.  At least 8
// stages per split.
inline int down_splits(int shape, int64_t P, int H, int F, int E_total, ssmm_format f, int tile_tokens = 0) {
  if (shape == 2) return 1;
  const int64_t rc = compressed_rows(f, H);
  const int rows_per_block = 2 * 4 * 32 / (is_vectorwise(f) ? 2 : 1);   // stored rows: MT x 4 waves x 32
  const int NB = tile_tokens ? tile_tokens : shape == 1 ? 128 : 32;
  const int64_t active = P < E_total ? P : E_total;                  // experts that can have tokens
  const int64_t tiles = (P / active + NB - 1) / NB;                  // token tiles of an average expert
  const int64_t blocks = (rc + rows_per_block - 1) / rows_per_block * active * tiles;
  int S = (int)((compute_units() + blocks / 2) / blocks);
  S = S < 1 ? 1 : S > 8 ? 8 : S;
  const int KS = F / kStageK;
  while (S > 1 && KS / S < 8) S--;
  return S;
}

// Blocks the down projection's 512-row x 160-token tiles give for large buckets (a bucket somewhat
// above the mean decides the token tiles per expert).
inline int64_t tall_down_blocks(int64_t P, int H, int E_total, ssmm_format f) {
  const int64_t active = P < E_total ? P : E_total;
  if (active < 1) return 0;
  const double est = (double)(P / active) + 2.0 * sqrt((double)(P / active));
  return (compressed_rows(f, H) / 32 + 15) / 16 * active * (int64_t)ceil(est / 160.0);
}
// Large buckets, but so few of those blocks that half the CUs or more would stay without one: the
// reduction is split (2 to 4 slices of at least 8 stages) so that the blocks fill the chip once.
// Each block is bound by the latency of its own chain of stages there, not by the MFMAs, so the
// shorter chains pay for the fp32 partial sums (measured on the Mixtral shape: down projection
// 24 % faster at 768 tokens, 20 % at 1024).  Returns the number of slices (1: no split).
inline int tall_down_splits(int64_t P, int H, int F, int E_total, ssmm_format f) {
  if (tile_shape(P, E_total) != 2 || is_vectorwise(f) || gathered_format(f)) return 1;
  const int64_t blocks = tall_down_blocks(P, H, E_total, f);
  if (blocks < 1 || blocks > compute_units() / 2) return 1;
  int S = (int)(compute_units() / blocks);
  S = S > 4 ? 4 : S;
  const int KS = F / kStageK;
  while (S > 1 && KS / S < 8) S--;
  return S;
}

template <bool GATEUP, bool VEC, int MT, int NT, int WM, int WN, int DS, bool GEN = false, bool ANYACT = false, bool SPLITK = false, bool SKIP = false>
int launch_ssmm(SsmmArgs a, int64_t P, hipStream_t s) {
  constexpr int NB = 32 * NT * WN;
  DeviceShape dev;
  if (int st = device_shape(&dev)) return st;
  if (!SPLITK) a.ksplit = 1;
  a.pairs = P;
  const int MTB = (a.row_tiles + MT * WM - 1) / (MT * WM) * a.ksplit;
  a.n_tiles_max = (int)((P + NB - 1) / NB) + a.E_total;   // every expert adds at most one ragged tile
  int64_t grid = (int64_t)MTB * a.n_tiles_max;
  grid = (grid + kXcdGroups - 1) / kXcdGroups * kXcdGroups;
  auto kern = ssmm_kernel<GATEUP, VEC, MT, NT, WM, WN, DS, GEN, ANYACT, SPLITK, SKIP>;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * WM * WN), 0, s, a);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  return SSMM_OK;
}

// Blocks a launch of the hand-scheduled kernels gets: one resident set (OCC per compute unit) when the
// tile list may be longer than that, else one block per possible tile.
inline int64_t resident_grid(int64_t tiles_bound, int occ, const DeviceShape& dev) {
  int64_t grid = (tiles_bound + kXcdGroups - 1) / kXcdGroups * kXcdGroups;
  const int64_t resident = (int64_t)dev.cus * occ / kXcdGroups * kXcdGroups;
  const int persistent = knob("SSMM_PERSISTENT");   // 0: one block per tile
  if (persistent != 0 && grid > resident) grid = resident;
  if (const int want = knob("SSMM_GRID"); want > 0 && want % kXcdGroups == 0 && grid > want) grid = want;   // smaller resident set
  return grid;
}

template <bool GATEUP, bool VEC, int MT, int NT, int WM, int WN, int DS, int OCC = 1, bool SPLITK = false, bool ANYACT = false>
int launch_ssmm2(SsmmArgs a, int64_t P, hipStream_t s) {
  constexpr int NB = 32 * NT * WN;
  DeviceShape dev;
  if (int st = device_shape(&dev)) return st;
  if (!SPLITK) a.ksplit = 1;
  a.pairs = P;
  const int MTB = (a.row_tiles + MT * WM - 1) / (MT * WM) * a.ksplit;
  a.n_tiles_max = (int)((P + NB - 1) / NB) + a.E_total;   // every expert adds at most one ragged tile
  const int64_t bound = (int64_t)MTB * a.n_tiles_max;
  const int64_t grid = resident_grid(bound, OCC, dev);
  auto kern = ssmm_kernel2<GATEUP, VEC, MT, NT, WM, WN, DS, OCC, SPLITK, ANYACT>;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * WM * WN), 0, s, a);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  return SSMM_OK;
}

// Gathered format -> plain 2:4 operand order (the kernel-ready form of the pruned DENSE matrix:
// pruned rows become zero operands).  Large buckets are compute-bound, where the Sub-Row level saves
// nothing (the MFMA count is that of plain 2:4 either way) and the gather costs address-path time:
// there the layer expands the three weight tensors once per call into its workspace (a streaming
// pass over the weights) and multiplies with the hand-scheduled plain kernels.
// One thread per (expert, dense row tile, k block, lane).
__global__ void __launch_bounds__(256) expand_gathered_kernel(const uint4* __restrict__ vals, const uint16_t* __restrict__ meta,
                                                              const uint8_t* __restrict__ desc, int64_t total, int dense_tiles,
                                                              int stored_tiles, int KB, int N, int M,
                                                              uint4* __restrict__ out_vals, uint16_t* __restrict__ out_meta) {
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const int lane = (int)(tid & 63);
  const int64_t unit = tid >> 6;                 // (expert, dense tile, k block)
  const int kb = (int)(unit % KB);
  const int64_t et = unit / KB;                  // expert * dense_tiles + dense tile
  const int rt = (int)(et % dense_tiles);
  const int64_t e = et / dense_tiles;
  const uint8_t d = desc[((et * (KB / 2) + kb / 2) * 32 + (lane & 31)) * 2 + (kb & 1)];
  uint4 v = make_uint4(0, 0, 0, 0);
  uint16_t m = 0;
  if (!(d & 0x80)) {
    const int64_t ts = e * stored_tiles + (int64_t)rt * N / M;
    const int src = (d & 31) + (lane & 32);
    v = vals[(ts * KB + kb) * 64 + src];
    m = meta[(((ts * (KB / 2) + kb / 2) * 64 + src) << 1) + (kb & 1)];
  }
  out_vals[unit * 64 + lane] = v;
  out_meta[(((et * (KB / 2) + kb / 2) * 64 + lane) << 1) + (kb & 1)] = m;
}

// bytes of the plain kernel-ready form of E matrices rows x K
inline size_t plain_tiled_bytes(int E, int64_t rows, int64_t K) {
  return align256((size_t)E * (tiled_values_bytes(rows, K) + tiled_meta_bytes(rows, K)));
}
inline int launch_expand_gathered(const void* tiled, int E, int64_t rows, int64_t K, ssmm_format f, void* dst, hipStream_t s) {
  const int64_t rc = compressed_rows(f, rows);
  const char* base = (const char*)tiled;
  const uint4* vals = (const uint4*)base;
  const uint16_t* meta = (const uint16_t*)(base + E * tiled_values_bytes(rc, K));
  const uint8_t* desc = (const uint8_t*)(base + E * (tiled_values_bytes(rc, K) + tiled_meta_bytes(rc, K)));
  uint4* ov = (uint4*)dst;
  uint16_t* om = (uint16_t*)((char*)dst + E * tiled_values_bytes(rows, K));
  const int64_t total = (int64_t)E * (rows / 32) * (K / 32) * 64;
  hipLaunchKernelGGL(expand_gathered_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, vals, meta, desc, total,
                     (int)(rows / 32), (int)(rc / 32), (int)(K / 32), f.N, f.M, ov, om);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  return SSMM_OK;
}
// the layer expands gathered weights when its buckets are large: a mean of 256 pairs per expert and
// more (measured on the Mixtral shape, (4,8,32): the pass costs what the gathering kernels lose at 900 tokens)
inline bool expands_weights(ssmm_format f, int64_t P, int E_total) {
  return gathered_format(f) && tile_shape(P, E_total) == 2 && P / E_total >= 256 && knob("SSMM_NO_EXPAND") == kUnset;
}

// What one call of the layer launches, decided on the host from its shapes alone (the bucket sizes
// stay on the device, so the rules work with a bucket "somewhat above the mean").  The workspace
// size and the call itself both read this plan, so they cannot disagree.
#ifndef SKIP_NT
#define SKIP_NT 2   // token tiles of 32 per wave on the compute-skipping kernels (their accumulators live in vector registers)
#endif
enum DownKernel { kDownSmall, kDownMedium, kDownMedium5, kDownHalf, kDownTall, kDownTall4 };
struct FfnPlan {
  int64_t P;
  bool expanded;         // gathered format multiplied as plain 2:4 operands expanded into the workspace
  bool gen, vec;         // format class the kernels see: gathered / (1,2,V) masked / neither (plain 2:4)
  bool skip;             // (1,2,V), V % 32 == 0, on the compute-skipping kernels (tuning knob; the masked ones are the default)
  int shape;             // tile class by mean bucket size (tile_shape), lowered for small gathered buckets
  int gen_first_shape;   // gathered formats: tile class of the first product
  int pipe, pipe_down;   // 2: hand-scheduled kernels, 1: compiler-scheduled ones
  int gshape;            // first product on the hand-scheduled kernels: tile class
  bool wide5;            //   ... and 160 instead of 128 tokens at the widest class
  bool gu_nt2;           //   ... or 64 tokens, for buckets that fit them
  bool vec_gu5, vec_down5;   // (1,2,V) on the hand-scheduled kernels: 160- instead of 128-token tiles for the first product / the down projection
  int down_kernel;       // DownKernel (hand-scheduled kernels, plain 2:4)
  int splits, kper;      // slices of the down projection's reduction (1: whole sums), stages per slice
  size_t yp_off, extra_off, bytes;   // workspace: h at 0, yp, partial sums / expanded weights
};

// Expected number of NB-token tiles of a bucket: its size taken as normal around `mean` with variance `mean`
// (balanced routing; the host never sees the real sizes): the sum over j of P(size > j NB).
inline double expected_tiles(double mean, int NB) {
  const double sd = sqrt(mean > 1.0 ? mean : 1.0);
  // every term more than six standard deviations below the mean is 1, every one as far above it 0
  const double first = floor((mean - 6.0 * sd) / NB);
  double sum = first > 0.0 ? first : 0.0;
  for (double j = sum; j * NB < mean + 6.0 * sd; j += 1.0) sum += 0.5 * erfc((j * NB - mean) / (sd * 1.4142135623730951));
  return sum;
}
// Time of a launch whose equal tiles the resident blocks take in rounds, in units of one round: a last round
// that is not full costs a full round unless it holds very few tiles (measured on the Mixtral shape, (1,2,8):
// 0.04 of a round of tiles cost half a round, 0.125 a whole one).
inline double rounds_cost(double tiles, int slots) {
  const double r = tiles / slots, whole = floor(r), part = r - whole;
  return whole + (part <= 0.01 ? 0.0 : fmin(1.0, 0.4 + 5.0 * part));
}

inline FfnPlan plan_ffn(int T, int H, int F, int E_total, int slots, ssmm_format f) {
  FfnPlan pl = {};
  const int64_t P = pl.P = (int64_t)T * slots;
  pl.expanded = expands_weights(f, P, E_total);
  const ssmm_format fk = pl.expanded ? ssmm_format{1, 1, 0} : f;   // what the kernels multiply
  pl.gen = gathered_format(fk);
  pl.vec = is_vectorwise(fk) && !pl.gen;
  int shape = tile_shape(P, E_total);
  if (const int want = knob("SSMM_TILE_SHAPE"); want >= 0 && want <= 2) shape = want;
  pl.pipe = 2;
  if (const int want = knob("SSMM_PIPE"); want != kUnset) pl.pipe = want;   // 1: compiler-scheduled loop
  pl.pipe_down = pl.pipe;
  // the hand-scheduled kernels address the token matrix with 32-bit offsets
  if ((int64_t)T * H * 2 >= (int64_t)1 << 32) pl.pipe = 1;
  // plain 2:4: h is read in consecutive rows and the offsets count from a tile's first row
  if (P * F * 2 >= (int64_t)1 << 32 && (is_vectorwise(fk) || (int64_t)256 * F * 2 >= (int64_t)1 << 32)) pl.pipe_down = 1;
  if (pl.gen) pl.pipe = pl.pipe_down = 1;
  pl.skip = pl.vec && fk.V % 32 == 0 && knob("SSMM_SUBROW_SKIP") == 1;
  if (pl.skip) pl.pipe = pl.pipe_down = 1;   // built on the compiler-scheduled kernels
  // Gathered formats, up to 64 pairs per expert: the down projection (reduction split, many blocks)
  // is faster on 32-token tiles than on 64-token ones (measured); the first product only while one
  // 32-token tile holds a bucket somewhat above the mean -- a second tile streams the weights again.
  pl.gen_first_shape = shape;
  if (pl.gen && shape == 1 && P / E_total <= 64) {
    const double mean = (double)(P / E_total);
    shape = 0;
    pl.gen_first_shape = mean + 2.0 * sqrt(mean) <= 32.0 ? 0 : 1;
  }
  pl.shape = shape;
  const int64_t active = P < E_total ? (P > 0 ? P : 1) : E_total;   // experts that can have tokens
  const double est = (double)(P / active) + 2.0 * sqrt((double)(P / active));   // a bucket somewhat above the mean

  // ---- first product on the hand-scheduled kernels.  The widest tile (256 output features x 128
  // tokens per block) also wins for small buckets, as long as it gives every CU a block: the weights
  // stream once per expert whatever the tile, and the wide tile needs half the blocks and transfers
  // per byte (measured on the Mixtral shape from 8 to 512 tokens: equal at 16 tokens, 8 % faster at
  // 256, 21 % at 512).  (1,2,V): the narrow tiles stay ahead below 20 pairs per expert (measured);
  // F = 1408: half a tile of overhang costs what the wide tile gains.
  pl.gshape = shape;
  {
    const int64_t wide_blocks = (F + 255) / 256 * active * ((P / active + 127) / 128);
    const int64_t wide_rows = (F + 255) / 256 * 256;   // rows the wide tiles stream (the last tile may hang over)
    if (!pl.vec && wide_blocks >= compute_units() * 25 / 32 && (wide_rows - F) * 32 <= F) pl.gshape = 2;   // 200 blocks on 256 CUs
    if (const int want = knob("SSMM_GU_SHAPE"); want >= 0 && want <= 2) pl.gshape = want;
    // 128- or 160-token tiles for the wide shape: the 160-token tile reuses every weight operand
    // five times instead of four (measured 3-11 % faster per token from 512 to 8192 tokens on the
    // Mixtral shape) but pads more; it is taken when a bucket of mean + 2 sqrt(mean) pairs pads to
    // at most 10 % more tokens with it.
    const double pad4 = ceil(est / 128.0) * 128.0, pad5 = ceil(est / 160.0) * 160.0;
    pl.wide5 = pad5 <= 1.1 * pad4;
    if (const int want = knob("SSMM_GU_NT5"); want != kUnset) pl.wide5 = want == 1;
    // ... and 64-token tiles while a bucket somewhat above the mean fits one: the weights stream once either way
    // and half the token-tile transfers and MFMAs go (measured: Qwen-shaped layer, 256 tokens, 0.234 -> 0.219 ms;
    // Mixtral shape, 128 tokens, 0.191 -> 0.187; equal at 16 to 64 tokens, where the weight stream alone counts)
    pl.gu_nt2 = !pl.vec && pl.gshape == 2 && !pl.wide5 && est <= 64.0;
    if (const int want = knob("SSMM_GU_NT2"); want != kUnset) pl.gu_nt2 = !pl.vec && pl.gshape == 2 && !pl.wide5 && want == 1;
    // (1,2,V): the same choice, on the expected tile counts and with 5 % (measured on the Mixtral shape, (1,2,8),
    // first product: 15 % faster at 512 tokens, 6 % at 1024, 4.5 % at 8192, equal at 4096 -- and 5 % slower at
    // 2048, where 4.5 tiles of 128 stand against 4 of 160; DeepSeek-shaped with two shared experts, 2048 tokens:
    // 12 % slower, the routed buckets of 192 pad to 320)
    const double mean = (double)P / (double)active;
    pl.vec_gu5 = pl.vec && pl.gshape >= 1 && expected_tiles(mean, 160) * 160.0 <= 1.05 * expected_tiles(mean, 128) * 128.0;
    if (const int want = knob("SSMM_VEC_GU_NT5"); want != kUnset) pl.vec_gu5 = pl.vec && pl.gshape >= 1 && want == 1;
  }

  // ---- down projection
  const int KS = F / kStageK;
  int splits = 1;
  pl.down_kernel = shape == 2 ? kDownTall : shape == 1 ? kDownMedium : kDownSmall;
  if (pl.pipe_down != 1) {
    auto forced_splits = [&](int v) {   // tuning knob: 1..8, small and medium buckets only
      const int want = knob("SSMM_DOWN_SPLITS");
      return want >= 1 && want <= 8 && shape < 2 ? want : v;
    };
    splits = forced_splits(down_splits(shape, P, H, F, E_total, fk));
    if (!pl.vec) {
      int dshape = shape;
      if (knob("SSMM_DOWN_SHAPE") == 1 && shape == 2) dshape = 1;   // the medium tile (unsplit) where the large one was chosen
      // large buckets, but so few of them that 512-row tiles would leave CUs without a block: half-height
      // tiles (measured on the Mixtral shape: 5-6 % at 768 and 1024 tokens) ...
      bool half_height = dshape == 2 && tall_down_blocks(P, H, E_total, fk) <= compute_units() * 5 / 8;   // 160 blocks on 256 CUs
      if (const int want = knob("SSMM_DOWN_HALF"); want != kUnset) half_height = dshape == 2 && want == 1;
      // ... or, with fewer still, the tall tile with its reduction in 2 to 4 slices
      int tall_splits = dshape == 2 && !pl.expanded ? tall_down_splits(P, H, F, E_total, fk) : 1;
      if (knob("SSMM_DOWN_TALLSPLIT") == 0) tall_splits = 1;
      // medium buckets that one 160-token tile holds but a 128-token tile does not (a second,
      // nearly empty tile would stream the expert's weights again)
      bool medium5 = dshape == 1 && ceil(est / 160.0) < ceil(est / 128.0);
      if (const int want = knob("SSMM_DOWN_NT5"); want != kUnset) medium5 = dshape == 1 && want == 1;
      if (medium5) {
        pl.down_kernel = kDownMedium5;
        splits = forced_splits(down_splits(shape, P, H, F, E_total, fk, 160));
      } else if (tall_splits > 1) {
        pl.down_kernel = kDownTall;
        splits = tall_splits;
      } else if (half_height) {
        pl.down_kernel = kDownHalf;
        splits = 1;
      } else {
        pl.down_kernel = dshape == 2 ? kDownTall : dshape == 1 ? kDownMedium : kDownSmall;
        if (dshape == 2) {
          splits = 1;
          // 512 rows x 160 or 128 tokens per block, by the rounds the resident blocks need (the 160-token tile
          // takes 5/4 of the time of the 128-token one): measured on the Mixtral shape, the down projection is a
          // staircase in the token count -- 0.26 ms up to 2304 tokens (256 tiles of 160: one round), 0.47-0.51 from
          // 2560 to 4608 (two), 0.73-0.81 from 5120 to 7168 (three) -- and the other width often needs a round less
          const double mean = (double)P / (double)active, blocks = (double)active * ((H + 511) / 512);
          const int cus = compute_units();
          // (long reductions only: with 22 or 40 stages per tile -- DeepSeek-, Qwen-shaped -- a tile's time hardly
          // depends on its width, the 160-token tiles are fewer, and they were 3-10 % faster at every token count)
          bool tall4 = KS >= 128 && 4.0 * rounds_cost(blocks * expected_tiles(mean, 128), cus) < 5.0 * rounds_cost(blocks * expected_tiles(mean, 160), cus);
          if (const int want = knob("SSMM_DOWN_TALL_NT4"); want != kUnset) tall4 = want == 1;
          if (tall4) pl.down_kernel = kDownTall4;
        }
      }
    } else if (shape == 2) {
      splits = 1;
      // (1,2,V), large buckets: 512 dense rows x 128 or 160 tokens per block.  The 160-token tile takes 5/4 of
      // the time of a 128-token one; what decides is the number of rounds the resident blocks need (measured on
      // the Mixtral shape, (1,2,8): 4096 tokens, 544 tiles of 128 = 3 rounds against 448 of 160 = 2: 0.55 -> 0.47 ms;
      // 2048 tokens 0.35 -> 0.25 ms; 1024 and 6000 tokens the other way round, 0.18 / 0.20 and 0.63 / 0.72 ms)
      const double mean = (double)P / (double)active, blocks = (double)active * ((H + 511) / 512);
      const int cus = compute_units();
      // (short reductions -- 22 or 40 stages per tile on the DeepSeek- and Qwen-shaped layers: a tile's time hardly
      // depends on its width there, so the width that pads less)
      pl.vec_down5 = KS >= 128 ? 5.0 * rounds_cost(blocks * expected_tiles(mean, 160), cus) <= 4.0 * rounds_cost(blocks * expected_tiles(mean, 128), cus)
                               : expected_tiles(mean, 160) * 160.0 <= 1.05 * expected_tiles(mean, 128) * 128.0;
      if (const int want = knob("SSMM_VEC_DOWN_NT5"); want != kUnset) pl.vec_down5 = want == 1;
    }
  } else if (pl.gen && shape < 2 && P * F * 2 < (int64_t)1 << 32) {
    // small buckets: few rows per block and the reduction split, so that every CU has blocks to
    // stream weights with (the partial sums go the way of the hand-scheduled kernels' split)
    const int rows_per_block = shape == 1 ? 256 : 128, NBg = shape == 1 ? 64 : 32;
    const int64_t blocks = (H + rows_per_block - 1) / rows_per_block * active * ((P / active + NBg - 1) / NBg);
    splits = (int)((4 * compute_units() + blocks / 2) / blocks);   // measured on the Mixtral shape at 16 and 256 tokens: four and two splits
    splits = splits < 1 ? 1 : splits > 8 ? 8 : splits;
    if (const int want = knob("SSMM_DOWN_SPLITS"); want >= 1 && want <= 8) splits = want;
    while (splits > 1 && KS / splits < 8) splits--;
  }
  pl.kper = (KS + splits - 1) / splits;
  pl.splits = (KS + pl.kper - 1) / pl.kper;   // no empty slice

  // ---- workspace: h [P][F] bf16, yp [P][H] bf16, then the fp32 partial sums of a split down projection
  // or (gathered formats with large buckets) the three weight tensors in plain 2:4 operand order
  const size_t part = pl.splits > 1 ? align256((size_t)pl.splits * P * H * 4) : 0;
  const size_t expanded = pl.expanded ? 2 * plain_tiled_bytes(E_total, F, H) + plain_tiled_bytes(E_total, H, F) : 0;
  pl.yp_off = align256((size_t)P * F * 2);
  pl.extra_off = pl.yp_off + align256((size_t)P * H * 2);
  pl.bytes = pl.extra_off + (part > expanded ? part : expanded) + 256;
  return pl;
}

}  // namespace ssmm

using namespace ssmm;

extern "C" size_t ssmm_ffn_workspace_bytes(int T, int H, int F, int E_total, int slots, ssmm_format f) {
  if (T < 0 || H < 1 || F < 1 || slots < 1 || E_total < 1) return 0;
  return plan_ffn(T, H, F, E_total, slots, f).bytes;
}

extern "C" int ssmm_expand_tiled_weights(const void* tiled, int E, int64_t rows, int64_t K, ssmm_format f, void* tiled_plain,
                                         void* stream) {
  if (E < 0 || rows < 1 || K < 1) return SSMM_EINVAL;
  int st = check_format(f, rows, K);
  if (st) return st;
  if (!gathered_format(f)) return SSMM_ESHAPE;
  const ssmm_format plain = {1, 1, 0};
  if (!can_tile(f, rows, K) || !can_tile(plain, rows, K)) return SSMM_ESHAPE;
  if ((int64_t)E * (rows / 32) * (K / 32) * 64 / 256 >= INT32_MAX) return SSMM_ESHAPE;   // one launch
  if (E == 0) return SSMM_OK;
  if (!tiled || !tiled_plain) return SSMM_EINVAL;
  return launch_expand_gathered(tiled, E, rows, K, f, tiled_plain, (hipStream_t)stream);
}

extern "C" int ssmm_expert_ffn_timed(const uint16_t* x, int T, int H, int F, int E_total, ssmm_format f,
                                     const void* wg_tiled, const void* wu_tiled, const void* wd_tiled,
                                     const int32_t* expert_offsets, const int32_t* sel, const float* sel_w,
                                     const int32_t* inv, int slots, uint16_t* y, void* workspace,
                                     size_t workspace_bytes, void* stream, void* const* events) {
  return ssmm_expert_ffn_variant(x, T, H, F, E_total, f, SSMM_ACT_SILU, 1, wg_tiled, wu_tiled, wd_tiled, expert_offsets, sel,
                                 sel_w, inv, slots, y, workspace, workspace_bytes, stream, events);
}

extern "C" int ssmm_expert_ffn_variant(const uint16_t* x, int T, int H, int F, int E_total, ssmm_format f, int activation,
                                       int gated, const void* wg_tiled, const void* wu_tiled, const void* wd_tiled,
                                       const int32_t* expert_offsets, const int32_t* sel, const float* sel_w,
                                       const int32_t* inv, int slots, uint16_t* y, void* workspace,
                                       size_t workspace_bytes, void* stream, void* const* events) {
  if (T < 0 || H < 1 || F < 1 || E_total < 1 || slots < 1) return SSMM_EINVAL;
  if (activation != SSMM_ACT_SILU && activation != SSMM_ACT_GELU_TANH && activation != SSMM_ACT_RELU) return SSMM_EINVAL;
  if (!gated) wu_tiled = wg_tiled;   // never read; keeps the pointer checks below in one form
  int st = check_format(f, F, H);
  if (st) return st;
  st = check_format(f, H, F);
  if (st) return st;
  if (!can_tile(f, F, H) || !can_tile(f, H, F)) return SSMM_ESHAPE;
  if ((int64_t)T * slots > INT32_MAX || E_total > kMaxBuckets) return SSMM_ESHAPE;
  if (T == 0) return SSMM_OK;
  if (!x || !wg_tiled || !wu_tiled || !wd_tiled || !expert_offsets || !sel || !sel_w || !inv || !y || !workspace)
    return SSMM_EINVAL;
  const FfnPlan pl = plan_ffn(T, H, F, E_total, slots, f);
  if (workspace_bytes < pl.bytes) return SSMM_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  auto mark = [&](int i) { return events ? hipEventRecord((hipEvent_t)events[i], s) == hipSuccess : true; };
  const int64_t P = pl.P;
  char* const ws = (char*)workspace;
  uint16_t* h = (uint16_t*)ws;
  uint16_t* yp = (uint16_t*)(ws + pl.yp_off);

  if (pl.expanded) {   // gathered format, large buckets: multiply in plain 2:4 operand order
    char* xb = ws + pl.extra_off;
    const size_t szg = plain_tiled_bytes(E_total, F, H);
    st = launch_expand_gathered(wg_tiled, E_total, F, H, f, xb, s);
    if (st) return st;
    if (gated) {
      st = launch_expand_gathered(wu_tiled, E_total, F, H, f, xb + szg, s);
      if (st) return st;
    }
    st = launch_expand_gathered(wd_tiled, E_total, H, F, f, xb + 2 * szg, s);
    if (st) return st;
    wg_tiled = xb;
    wu_tiled = gated ? xb + szg : xb;
    wd_tiled = xb + 2 * szg;
    f.N = f.M = 1;
    f.V = 0;
  }
  // sections of a kernel-ready weight buffer: values, index words, (vector-wise only) source-row bits
  const bool gen = pl.gen;   // operands gathered lane by lane (compiler-scheduled kernels)
  const bool vec = pl.vec;   // (1,2,V): operands multiplied twice, masked
  auto bind = [&](const void* tiled, int64_t w_rows, int64_t w_K, const bf16x8*& vals, const uint32_t*& meta,
                  const uint8_t*& vidx, SsmmArgs& a) {
    const int64_t rc = compressed_rows(f, w_rows);
    const char* base = (const char*)tiled;
    vals = (const bf16x8*)base;
    meta = (const uint32_t*)(base + E_total * tiled_values_bytes(rc, w_K));
    vidx = is_vectorwise(f) ? (const uint8_t*)(base + E_total * (tiled_values_bytes(rc, w_K) + tiled_meta_bytes(rc, w_K)))
                            : nullptr;
    a.row_tiles = (int)((gen ? w_rows : rc) / 32);
    a.stored_tiles = (int)(rc / 32);
    a.gN = f.N;
    a.gM = f.M;
  };
  SsmmArgs g = {};
  g.act = x;
  g.sel = sel;
  bind(wg_tiled, F, H, g.a0_vals, g.a0_meta, g.a0_vidx, g);
  bind(wu_tiled, F, H, g.a1_vals, g.a1_meta, g.a1_vidx, g);
  g.expert_offsets = expert_offsets;
  g.sel_w = nullptr;
  g.out = h;
  g.E_total = E_total;
  g.rows = F;
  g.K = H;
  g.actfn = activation;
  g.vper = f.V / 32;

  SsmmArgs d = {};
  d.act = h;
  d.sel = nullptr;
  bind(wd_tiled, H, F, d.a0_vals, d.a0_meta, d.a0_vidx, d);
  d.expert_offsets = expert_offsets;
  d.sel_w = sel_w;
  d.out = yp;
  d.E_total = E_total;
  d.rows = H;
  d.K = F;
  d.vper = f.V / 32;
  d.kper = pl.kper;
  d.ksplit = pl.splits;
  d.out_f32 = (float*)(ws + pl.extra_off);

  // Template arguments of the launches: gate/up?, vector-wise?, stored row tiles per wave and matrix,
  // token tiles per wave, waves along rows, waves along tokens, stages in flight + 1, waves per SIMD
  // (hand-scheduled kernels), split reduction?, activation kind from the call?.
  // Large buckets amortise weight traffic over 128 (160) tokens; small ones keep the token tile
  // narrow so no MFMA work is spent on padding, give up the one-memory-instruction-per-MFMA placement
  // (they are bound by HBM) and run two waves per SIMD.
  const int shape = pl.shape, gfs = pl.gen_first_shape, pipe = pl.pipe;
  const bool variant = activation != SSMM_ACT_SILU || !gated;   // kernels whose epilogue takes the activation kind from the call
  if (!mark(0)) return SSMM_EHIP;
  // First product.  Usual layer (SiLU, gated): hand-scheduled kernels; gathered formats and token
  // matrices of 4 GB and more: compiler-scheduled ones.  Another activation kind or no gate
  // ("variant"): kernels whose epilogue takes the kind from the call -- hand-scheduled for the
  // small and medium tile shapes, compiler-scheduled where the generic epilogue does not fit
  // the register budget of the hand-scheduled form (every kernel here must compile without
  // spills: the build checks it).
  if (!variant && pl.skip) {
    st = shape >= 1 ? launch_ssmm<true, true, 1, SKIP_NT, 4, 1, 3, false, false, false, true>(g, P, s)
                    : launch_ssmm<true, true, 1, 1, 4, 1, 3, false, false, false, true>(g, P, s);
  } else if (!variant) {
    if (gen)
      // One stored row tile per wave and matrix at every shape.  Large buckets: the gather needs
      // the registers.  Small and medium ones: two blocks then fit a CU, which doubles the weight
      // bytes in flight (measured on the Mixtral shape, (4,8,32): first product 0.148 -> 0.118 ms
      // at 16 tokens, 0.31 -> 0.20 ms at 256).
      st = gfs == 2   ? launch_ssmm<true, false, 1, 4, 4, 1, 3, true>(g, P, s)
           : gfs == 1 ? launch_ssmm<true, false, 1, 2, 4, 1, 3, true>(g, P, s)
                      : launch_ssmm<true, false, 1, 1, 4, 1, 3, true>(g, P, s);
    else if (pipe != 1 && !vec)
      st = pl.gshape == 2 && pl.wide5 ? launch_ssmm2<true, false, 2, 5, 4, 1, 3>(g, P, s)
           : pl.gshape == 2 && pl.gu_nt2 ? launch_ssmm2<true, false, 2, 2, 4, 1, 4>(g, P, s)
           : pl.gshape == 2           ? launch_ssmm2<true, false, 2, 4, 4, 1, 4>(g, P, s)
           : pl.gshape == 1           ? launch_ssmm2<true, false, 1, 4, 4, 1, 4>(g, P, s)
                                      : launch_ssmm2<true, false, 1, 1, 4, 1, 4, 2>(g, P, s);
    else if (pipe != 1)
      st = pl.gshape >= 1 ? (pl.vec_gu5 ? launch_ssmm2<true, true, 1, 5, 4, 1, 3>(g, P, s) : launch_ssmm2<true, true, 1, 4, 4, 1, 4>(g, P, s))
                          : launch_ssmm2<true, true, 1, 1, 4, 1, 4>(g, P, s);
    else if (!vec)   // fall-back kernels: 128-, 64- and 32-token tiles
      st = shape == 2   ? launch_ssmm<true, false, 2, 4, 4, 1, 3>(g, P, s)
           : shape == 1 ? launch_ssmm<true, false, 2, 2, 4, 1, 3>(g, P, s)
                        : launch_ssmm<true, false, 2, 1, 4, 1, 3>(g, P, s);
    else
      st = shape == 2   ? launch_ssmm<true, true, 1, 4, 4, 1, 3>(g, P, s)
           : shape == 1 ? launch_ssmm<true, true, 1, 2, 4, 1, 3>(g, P, s)
                        : launch_ssmm<true, true, 1, 1, 4, 1, 3>(g, P, s);
  } else if (gated) {
    if (gen)
      st = gfs >= 1 ? launch_ssmm<true, false, 1, 2, 4, 1, 3, true, true>(g, P, s)
                    : launch_ssmm<true, false, 1, 1, 4, 1, 3, true, true>(g, P, s);
    else if (pipe != 1 && !vec && shape < 2)
      st = shape == 1 ? launch_ssmm2<true, false, 1, 4, 4, 1, 4, 1, false, true>(g, P, s)
                      : launch_ssmm2<true, false, 1, 1, 4, 1, 4, 2, false, true>(g, P, s);
    else if (pipe != 1 && vec && shape == 0)
      st = launch_ssmm2<true, true, 1, 1, 4, 1, 4, 1, false, true>(g, P, s);
    else if (!vec)
      st = shape >= 1 ? launch_ssmm<true, false, 2, 2, 4, 1, 3, false, true>(g, P, s)
                      : launch_ssmm<true, false, 2, 1, 4, 1, 3, false, true>(g, P, s);
    else
      st = shape >= 1 ? launch_ssmm<true, true, 1, 2, 4, 1, 3, false, true>(g, P, s)
                      : launch_ssmm<true, true, 1, 1, 4, 1, 3, false, true>(g, P, s);
  } else {
    // one weight matrix, activation in the epilogue: the single-matrix kernels (those of the
    // down projection, unsplit) with the token rows gathered through SEL
    if (gen)
      st = gfs >= 1 ? launch_ssmm<false, false, 2, 2, 4, 1, 3, true, true>(g, P, s)
                    : launch_ssmm<false, false, 1, 1, 4, 1, 3, true, true>(g, P, s);
    else if (pipe != 1 && !vec && shape < 2)
      st = shape == 1 ? launch_ssmm2<false, false, 2, 4, 4, 1, 4, 1, false, true>(g, P, s)
                      : launch_ssmm2<false, false, 2, 1, 4, 1, 4, 2, false, true>(g, P, s);
    else if (pipe != 1 && vec && shape < 2)
      st = shape == 1 ? launch_ssmm2<false, true, 1, 4, 4, 1, 4, 1, false, true>(g, P, s)
                      : launch_ssmm2<false, true, 1, 1, 4, 1, 4, 2, false, true>(g, P, s);
    else if (!vec)
      st = shape >= 1 ? launch_ssmm<false, false, 4, 2, 4, 1, 3, false, true>(g, P, s)
                      : launch_ssmm<false, false, 2, 1, 4, 1, 3, false, true>(g, P, s);
    else
      st = shape >= 1 ? launch_ssmm<false, true, 2, 2, 4, 1, 3, false, true>(g, P, s)
                      : launch_ssmm<false, true, 1, 1, 4, 1, 3, false, true>(g, P, s);
  }
  if (st) return st;
  if (!mark(1)) return SSMM_EHIP;
  // Down projection; with pl.splits > 1 the kernels write fp32 partial sums of the slices
  const bool split = pl.splits > 1;
  if (pl.pipe_down != 1 && !vec) {
    switch (pl.down_kernel) {
      case kDownMedium5:
        st = split ? launch_ssmm2<false, false, 2, 5, 4, 1, 3, 1, true>(d, P, s) : launch_ssmm2<false, false, 2, 5, 4, 1, 3>(d, P, s);
        break;
      case kDownHalf:
        st = launch_ssmm2<false, false, 2, 5, 4, 1, 3>(d, P, s);
        break;
      case kDownTall:
        st = split ? launch_ssmm2<false, false, 4, 5, 4, 1, 3, 1, true>(d, P, s) : launch_ssmm2<false, false, 4, 5, 4, 1, 3>(d, P, s);
        break;
      case kDownTall4:
        st = launch_ssmm2<false, false, 4, 4, 4, 1, 3>(d, P, s);
        break;
      case kDownMedium:
        st = split ? launch_ssmm2<false, false, 2, 4, 4, 1, 4, 1, true>(d, P, s) : launch_ssmm2<false, false, 2, 4, 4, 1, 4>(d, P, s);
        break;
      default:
        st = split ? launch_ssmm2<false, false, 2, 1, 4, 1, 4, 2, true>(d, P, s) : launch_ssmm2<false, false, 2, 1, 4, 1, 4, 2>(d, P, s);
    }
  } else if (pl.pipe_down != 1) {
    st = shape == 2   ? (pl.vec_down5 ? launch_ssmm2<false, true, 2, 5, 4, 1, 3>(d, P, s) : launch_ssmm2<false, true, 2, 4, 4, 1, 4>(d, P, s))
         : shape == 1 ? (split ? launch_ssmm2<false, true, 1, 4, 4, 1, 4, 1, true>(d, P, s)
                               : launch_ssmm2<false, true, 1, 4, 4, 1, 4>(d, P, s))
                      : (split ? launch_ssmm2<false, true, 1, 1, 4, 1, 4, 2, true>(d, P, s)
                               : launch_ssmm2<false, true, 1, 1, 4, 1, 4, 2>(d, P, s));
  } else if (pl.skip) {
    st = shape >= 1 ? launch_ssmm<false, true, 2, SKIP_NT, 4, 1, 3, false, false, false, true>(d, P, s)
                    : launch_ssmm<false, true, 1, 1, 4, 1, 3, false, false, false, true>(d, P, s);
  } else if (gen) {
    if (split)
      st = shape == 1 ? launch_ssmm<false, false, 2, 2, 4, 1, 3, true, false, true>(d, P, s)
                      : launch_ssmm<false, false, 1, 1, 4, 1, 3, true, false, true>(d, P, s);
    else
      st = shape == 2   ? launch_ssmm<false, false, 2, 4, 4, 1, 3, true>(d, P, s)
           : shape == 1 ? launch_ssmm<false, false, 2, 2, 4, 1, 3, true>(d, P, s)
                        : launch_ssmm<false, false, 1, 1, 4, 1, 3, true>(d, P, s);
  } else if (!vec) {
    st = shape == 2   ? launch_ssmm<false, false, 4, 4, 4, 1, 3>(d, P, s)
         : shape == 1 ? launch_ssmm<false, false, 4, 2, 4, 1, 3>(d, P, s)
                      : launch_ssmm<false, false, 2, 1, 4, 1, 3>(d, P, s);
  } else {
    st = shape == 2   ? launch_ssmm<false, true, 2, 4, 4, 1, 3>(d, P, s)
         : shape == 1 ? launch_ssmm<false, true, 2, 2, 4, 1, 3>(d, P, s)
                      : launch_ssmm<false, true, 1, 1, 4, 1, 3>(d, P, s);
  }
  if (st) return st;
  if (!mark(2)) return SSMM_EHIP;
  const int64_t total = (int64_t)T * (H / 8);
  if (split)
    hipLaunchKernelGGL(combine_split_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       (const float*)d.out_f32, inv, sel_w, T, H, slots, pl.splits, P, y);
  else
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const uint16_t*)yp, inv,
                       T, H, slots, y);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  if (!mark(3)) return SSMM_EHIP;
  return SSMM_OK;
}

extern "C" int ssmm_expert_ffn(const uint16_t* x, int T, int H, int F, int E_total, ssmm_format f,
                               const void* wg_tiled, const void* wu_tiled, const void* wd_tiled,
                               const int32_t* expert_offsets, const int32_t* sel, const float* sel_w,
                               const int32_t* inv, int slots, uint16_t* y, void* workspace,
                               size_t workspace_bytes, void* stream) {
  return ssmm_expert_ffn_timed(x, T, H, F, E_total, f, wg_tiled, wu_tiled, wd_tiled, expert_offsets, sel, sel_w, inv,
                               slots, y, workspace, workspace_bytes, stream, nullptr);
}

namespace ssmm {
// c[pos][r] = sum over the slices of the reduction, in slice order, of part[slice][pos][r]; bf16 out.
// One thread per 8 consecutive output features.
__global__ void __launch_bounds__(256) reduce_split_kernel(const float* __restrict__ part, int64_t n, int rows, int ksplit,
                                                           uint16_t* __restrict__ c) {
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = n * (rows / 8);
  if (tid >= total) return;
  float a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int k = 0; k < ksplit; k++) {
    const float4* src = (const float4*)(part + ((int64_t)k * n * rows + tid * 8));
    const float4 v0 = src[0], v1 = src[1];
    a[0] += v0.x; a[1] += v0.y; a[2] += v0.z; a[3] += v0.w;
    a[4] += v1.x; a[5] += v1.y; a[6] += v1.z; a[7] += v1.w;
  }
  *(uint4*)(c + tid * 8) = make_uint4(cvt_bf16x2(a[0], a[1]), cvt_bf16x2(a[2], a[3]), cvt_bf16x2(a[4], a[5]), cvt_bf16x2(a[6], a[7]));
}

// Slices of the reduction of the stand-alone product: up to as many as it takes for the blocks to
// fill the chip once (at most 8, at least 8 stages each), while the partial sums cost less than the
// shorter chains save.  Few selected columns and few rows give few
// tiles, each with the whole reduction as one chain of dependent stages (about 0.6 us per stage):
// (256 x 16384) x 256 columns ran 0.15 ms in two blocks.  Formats on the hand-scheduled kernels only.
inline int matmul_splits(int64_t rows, int64_t K, int n, ssmm_format f) {
  if (gathered_format(f) || n < 1) return 1;
  const bool vec = is_vectorwise(f);
  const int shape = tile_shape(n, 1);
  if (vec && shape == 2) return 1;   // no split instance of that kernel
  const int64_t rc = compressed_rows(f, rows);
  const int rows_per_block = (shape == 2 ? 512 : 256) / (vec ? 2 : 1);            // stored rows
  const int NB = shape == 2 ? 160 : shape == 1 ? 128 : 32;
  const int64_t blocks = (rc + rows_per_block - 1) / rows_per_block * ((n + NB - 1) / NB);
  int most = (int)(compute_units() / blocks);
  most = most < 1 ? 1 : most > 8 ? 8 : most;
  const int KS = (int)(K / kStageK);
  // a slice costs its chain of stages; the partial sums are written and read once at about 4 TB/s,
  // and the pass that adds them is one more launch (microseconds; measured crossovers on the shape grid)
  int best = 1;
  double best_us = KS * 0.6;
  for (int S = 2; S <= most && KS / S >= 8; S++) {
    const double us = (double)((KS + S - 1) / S) * 0.6 + 4.0 + (double)S * n * rows * 8.0 / 4.0e6;
    if (us < best_us) {
      best_us = us;
      best = S;
    }
  }
  return best;
}
}  // namespace ssmm

extern "C" size_t ssmm_matmul_workspace_bytes(int64_t rows, int64_t K, int n, ssmm_format f) {
  if (rows < 1 || K < 1 || n < 0 || check_format(f, rows, K) != SSMM_OK || !can_tile(f, rows, K)) return 256;
  const int S = matmul_splits(rows, K, n, f);
  return 256 + (S > 1 ? align256((size_t)S * n * rows * 4) : 0);
}

extern "C" int ssmm_matmul(const void* a_tiled, int64_t rows, int64_t K, ssmm_format f, const uint16_t* b, int64_t n_b,
                           const int32_t* sel, int n, uint16_t* c, void* workspace, size_t workspace_bytes,
                           void* stream) {
  if (n < 0 || n_b < 0) return SSMM_EINVAL;
  int st = check_format(f, rows, K);
  if (st) return st;
  if (!can_tile(f, rows, K)) return SSMM_ESHAPE;
  if (rows > INT32_MAX || K > INT32_MAX) return SSMM_ESHAPE;
  if (n_b * K * 2 >= (int64_t)1 << 32) return SSMM_ESHAPE;   // the kernels address B with 32-bit offsets
  if (!sel && n > n_b) return SSMM_EINVAL;
  if (n == 0) return SSMM_OK;
  if (!a_tiled || !b || !c || !workspace) return SSMM_EINVAL;
  if (workspace_bytes < ssmm_matmul_workspace_bytes(rows, K, n, f)) return SSMM_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const bool gen = gathered_format(f);
  const bool vec = is_vectorwise(f) && !gen;
  const int64_t rc = compressed_rows(f, rows);
  const char* base = (const char*)a_tiled;
  SsmmArgs d = {};
  d.act = b;
  d.sel = sel;
  d.a0_vals = (const bf16x8*)base;
  d.a0_meta = (const uint32_t*)(base + tiled_values_bytes(rc, K));
  d.a0_vidx = is_vectorwise(f) ? (const uint8_t*)(base + tiled_values_bytes(rc, K) + tiled_meta_bytes(rc, K)) : nullptr;
  d.row_tiles = (int)((gen ? rows : rc) / 32);
  d.stored_tiles = (int)(rc / 32);
  d.gN = f.N;
  d.gM = f.M;
  d.expert_offsets = nullptr;   // one bucket: all n selected columns
  d.sel_w = nullptr;   // no scaling
  d.out = c;
  d.E_total = 1;
  d.rows = (int)rows;
  d.K = (int)K;
  // same tile shapes as the down projection of the expert FFN (one "expert" with n tokens)
  const int shape = tile_shape(n, 1);
  int splits = matmul_splits(rows, K, n, f);
  if (knob("SSMM_MATMUL_SPLITS") == 1) splits = 1;   // tuning knob: no split
  if (splits > 1) {
    const int KS = (int)(K / kStageK);
    d.kper = (KS + splits - 1) / splits;
    d.ksplit = splits = (KS + d.kper - 1) / d.kper;   // no empty slice
    d.out_f32 = (float*)((char*)workspace + 256);
  }
  if (gen)
    st = shape == 2   ? launch_ssmm<false, false, 2, 4, 4, 1, 3, true>(d, n, s)
         : shape == 1 ? launch_ssmm<false, false, 2, 2, 4, 1, 3, true>(d, n, s)
                      : launch_ssmm<false, false, 1, 1, 4, 1, 3, true>(d, n, s);
  else if (splits > 1 && !vec)
    st = shape == 2   ? launch_ssmm2<false, false, 4, 5, 4, 1, 3, 1, true>(d, n, s)
         : shape == 1 ? launch_ssmm2<false, false, 2, 4, 4, 1, 4, 1, true>(d, n, s)
                      : launch_ssmm2<false, false, 2, 1, 4, 1, 4, 2, true>(d, n, s);
  else if (splits > 1)
    st = shape == 1 ? launch_ssmm2<false, true, 1, 4, 4, 1, 4, 1, true>(d, n, s)
                    : launch_ssmm2<false, true, 1, 1, 4, 1, 4, 2, true>(d, n, s);
  else if (!vec)
    st = shape == 2   ? launch_ssmm2<false, false, 4, 5, 4, 1, 3>(d, n, s)
         : shape == 1 ? launch_ssmm2<false, false, 2, 4, 4, 1, 4>(d, n, s)
                      : launch_ssmm2<false, false, 2, 1, 4, 1, 4, 2>(d, n, s);
  else
    st = shape == 2   ? launch_ssmm2<false, true, 2, 4, 4, 1, 4>(d, n, s)
         : shape == 1 ? launch_ssmm2<false, true, 1, 4, 4, 1, 4>(d, n, s)
                      : launch_ssmm2<false, true, 1, 1, 4, 1, 4, 2>(d, n, s);
  if (st) return st;
  if (splits > 1) {
    const int64_t total = (int64_t)n * (rows / 8);
    hipLaunchKernelGGL(reduce_split_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const float*)d.out_f32,
                       (int64_t)n, (int)rows, splits, c);
    SSMM_RETURN_IF_LAUNCH_FAILED();
  }
  return SSMM_OK;
}
