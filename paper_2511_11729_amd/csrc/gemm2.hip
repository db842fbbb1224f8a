// Weight GEMM of the finetune unit (see gemm2.h for the operand layouts).
//
// Workgroup tile (64 FM) x 256, K step 32, FOUR waves -- one per SIMD, each with the whole register file: a wave owns
// a (32 FM) x 128 block of the tile = FM x 4 accumulators of v_mfma_f32_32x32x16 (256 accumulator registers at FM = 4).
// What this shape buys on gfx950, measured:
//   * operand bytes per flop through L2 and through LDS fall with the tile edge: a CU pulls no more than ~22-41 B/clk
//     from L2 and LDS serves 128 B/clk, and 64 x 64 wave tiles (two waves per SIMD) need all of the latter at the full
//     MFMA rate.  128 x 128 per wave needs half;
//   * operands go from global memory straight into LDS (global_load_lds, 16 B per lane, no register staging); the
//     rows of a stage are XOR-swizzled in 16-byte chunks on the way in (each lane picks the global chunk that belongs
//     in its LDS slot), which makes the 32-row fragment reads conflict free;
//   * four LDS stages: while stage s is multiplied, s+1 has landed and s+2, s+3 are in flight;
//   * one wave per SIMD has nobody to hide its waits, so the K loop is software pipelined by hand: the fragments of
//     the next half step are read while the MFMAs of this one issue, and the eight loads a wave owes per stage are
//     dealt out between MFMAs (sched_group_barrier pins that order).  The loop runs within 14 % of the MFMA issue
//     bound in cycles; what it delivers is then set by the clock the chip grants under that load (1.5-1.6 GHz).
// FM = 2 (128-row tiles) doubles the tile count for outputs that would not fill the chip with 256-row tiles.
#include "gemm2.h"

#include <algorithm>

#include "ctx.h"
#include "device_utils.h"

namespace harli {
namespace {

constexpr int BN = kG2TileN, BK = kG2StepK, NT = 256;
// LDS stages: four (128 KiB at 256-row tiles).  Six stages at 128-row tiles (144 KiB) were measured and changed nothing:
// those tiles are not short of loads in flight.
template <int FM>
constexpr int stages() { return 4; }
constexpr int BSZ = BN * BK * 2;  // 16 KiB: one stage of the weight-side tile

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define G2_WAITV(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
#define G2_SB0() __builtin_amdgcn_sched_barrier(0)
#define G2_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// One 32-row slab of a wave's block (the four accumulators c0..c3 side by side, 128 columns) to its destinations.
template <bool HALF, int EPI>
__device__ __forceinline__ void g2_store_slab(const f32x16& c0, const f32x16& c1, const f32x16& c2, const f32x16& c3, char* ebuf,
                                              const Gemm2Args& a, const Gemm2Out& out, int tn, int wn, int lane, int mrow0,
                                              bool& clamped) {
  constexpr int ER = (128 + 8) * 4;
  // a lane of accumulator j holds rows 8 (v/4) + 4 (lane/32) + v%4 of column lane%32 of that 32 x 32 block
  const int col_l = lane & 31, rgrp = (lane >> 5) * 4;
  auto pack8 = [&](const float* v) {
    if (HALF) {
#pragma unroll
      for (int e = 0; e < 8; ++e) clamped = clamped || !(fabsf(v[e]) <= 65504.f);
      return make_uint4(pack_h2(v[0], v[1]), pack_h2(v[2], v[3]), pack_h2(v[4], v[5]), pack_h2(v[6], v[7]));
    }
    return make_uint4(pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7]));
  };
  auto unpack = [](const uint4& wv, float* v) {
    if (HALF) unpack8h(wv, v);
    else unpack8(wv, v);
  };
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        *reinterpret_cast<float*>(ebuf + (8 * (v >> 2) + rgrp + (v & 3)) * ER + (j * 32 + col_l) * 4) = (j == 0 ? c0 : j == 1 ? c1 : j == 2 ? c2 : c3)[v] * a.alpha;
    __builtin_amdgcn_wave_barrier();
        if (EPI == GEMM2_EPI_GATEUP) {
      // staged columns [0,32) gate, [32,64) up of output columns 0..31 of this wave's 64; [64,96), [96,128) of 32..63
      const int c8 = (lane & 7) * 8;                              // 8 output columns of the 64
      const int n8 = (tn - out.tile0) * 128 + wn * 64 + c8;       // column in a, u, m
      const int sc = (c8 >> 5) * 64 + (c8 & 31);                  // staged column of the gate values
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int row = it * 8 + (lane >> 3), m = mrow0 + row;
        const float4 g0 = *reinterpret_cast<const float4*>(ebuf + row * ER + sc * 4);
        const float4 g1 = *reinterpret_cast<const float4*>(ebuf + row * ER + sc * 4 + 16);
        const float4 u0 = *reinterpret_cast<const float4*>(ebuf + row * ER + (sc + 32) * 4);
        const float4 u1 = *reinterpret_cast<const float4*>(ebuf + row * ER + (sc + 32) * 4 + 16);
        if (m >= a.M || n8 >= out.N) continue;
        const float gx[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        const float ux[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
        const uint4 gp = pack8(gx), up = pack8(ux);
        float av[8], uv[8], mv[8];
        unpack(gp, av);  // the rounded values, as the backward pass will read them
        unpack(up, uv);
#pragma unroll
        for (int e = 0; e < 8; ++e) mv[e] = av[e] / (1.f + __expf(-av[e])) * uv[e];
        *reinterpret_cast<uint4*>(out.Cb + (long long)m * out.ldcb + n8) = gp;
        *reinterpret_cast<uint4*>(a.o1 + (long long)m * a.lde + n8) = up;
        *reinterpret_cast<uint4*>(a.o0 + (long long)m * a.lde + n8) = pack8(mv);
      }
    } else if (EPI == GEMM2_EPI_SWIGLU_BWD || EPI == GEMM2_EPI_NONE) {
      // 16-bit outputs only: eight columns (16 bytes) per lane, four rows per pass
      const int c8 = (lane & 15) * 8, n8 = (tn - out.tile0) * BN + wn * 128 + c8;
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int row = it * 4 + (lane >> 4), m = mrow0 + row;
        const float4 lo = *reinterpret_cast<const float4*>(ebuf + row * ER + c8 * 4);
        const float4 hi = *reinterpret_cast<const float4*>(ebuf + row * ER + c8 * 4 + 16);
        if (m >= a.M || n8 >= out.N) continue;
        const float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        if (EPI == GEMM2_EPI_SWIGLU_BWD) {
          float av[8], uv[8], oa[8], ou[8];
          unpack(*reinterpret_cast<const uint4*>(a.e0 + (long long)m * a.lde + n8), av);
          unpack(*reinterpret_cast<const uint4*>(a.e1 + (long long)m * a.lde + n8), uv);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float sg = 1.f / (1.f + __expf(-av[e]));
            oa[e] = x[e] * uv[e] * sg * (1.f + av[e] * (1.f - sg));
            ou[e] = x[e] * av[e] * sg;
          }
          *reinterpret_cast<uint4*>(a.o0 + (long long)m * a.lde + n8) = pack8(oa);
          *reinterpret_cast<uint4*>(a.o1 + (long long)m * a.lde + n8) = pack8(ou);
        } else {
          *reinterpret_cast<uint4*>(out.Cb + (long long)m * out.ldcb + n8) = pack8(x);
        }
      }
    } else {
      // fp32 output (+ residual, + optional 16-bit copy): four columns per lane, two rows per pass
      const int c4 = (lane & 31) * 4, n = (tn - out.tile0) * BN + wn * 128 + c4;
      const bool nvec = n + 3 < out.N;
#pragma unroll
      for (int half8 = 0; half8 < 2; ++half8) {
        float4 rv[8];
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int m = mrow0 + (half8 * 8 + it) * 2 + (lane >> 5);
          rv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
          if (out.res && nvec && m < a.M) rv[it] = *reinterpret_cast<const float4*>(out.res + (long long)m * out.ldcf + n);
        }
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int row = (half8 * 8 + it) * 2 + (lane >> 5), m = mrow0 + row;
          float4 o = *reinterpret_cast<const float4*>(ebuf + row * ER + c4 * 4);
          if (m >= a.M || n >= out.N) continue;
          if (nvec) {
            o.x += rv[it].x, o.y += rv[it].y, o.z += rv[it].z, o.w += rv[it].w;
            *reinterpret_cast<float4*>(out.Cf + (long long)m * out.ldcf + n) = o;
            if (out.Cb) {
              const float ov[4] = {o.x, o.y, o.z, o.w};
              if (HALF) clamped = clamped || !(fabsf(ov[0]) <= 65504.f) || !(fabsf(ov[1]) <= 65504.f) || !(fabsf(ov[2]) <= 65504.f) || !(fabsf(ov[3]) <= 65504.f);
              *reinterpret_cast<uint2*>(out.Cb + (long long)m * out.ldcb + n) =
                  HALF ? make_uint2(pack_h2(o.x, o.y), pack_h2(o.z, o.w)) : make_uint2(pack_bf2(o.x, o.y), pack_bf2(o.z, o.w));
            }
          } else {  // the last columns of a matrix whose width is not a multiple of four
            const float ov[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < out.N) {
                float x = ov[e];
                if (out.res) x += out.res[(long long)m * out.ldcf + n + e];
                out.Cf[(long long)m * out.ldcf + n + e] = x;
                if (out.Cb) out.Cb[(long long)m * out.ldcb + n + e] = HALF ? f2h(x) : f2bf(x);
              }
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }

template <int FM, bool HALF, int EPI>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(1, 1)))
k_gemm2(Gemm2Args a, int tiles_total, int chunk, int GM, int GN, const uint4* zero16) {
  constexpr int BM = 64 * FM, ASZ = BM * BK * 2, STG = ASZ + BSZ, NS = stages<FM>();
  constexpr int LOADS = FM + 4;  // direct-to-LDS loads a wave issues per stage
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;  // 2 x 2 waves of (32 FM) x 128
  // XCD-aware tile order (workgroup w runs on XCD w % 8): every XCD walks blocks of GM x GN tiles, so the workgroups
  // that share an L2 share operand panels.
  const int w = blockIdx.x;
  const int slot = (w & 7) * chunk + (w >> 3);
  if (slot >= tiles_total) return;
  const int nbn = (a.tiles_n + GN - 1) / GN;
  const int blk = slot / (GM * GN), within = slot - blk * (GM * GN);
  const int bm = blk / nbn, bn = blk - bm * nbn;
  const int tm = bm * GM + within / GN, tn = bn * GN + within % GN;
  const int m0 = tm * BM;
  if (m0 >= a.M || tn >= a.tiles_n) return;

  f32x16 acc[FM][4];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // ---- stage bookkeeping (uniform): the segments that cover this tile, 32 k at a time -------------------------------
  int n_stage = 0;
  for (int s = 0; s < a.nseg; ++s)
    if (tn >= a.seg[s].tile0 && tn < a.seg[s].tile1) n_stage += (a.seg[s].K + BK - 1) / BK;
  const int n_step = (n_stage + NS - 1) / NS * NS;  // the loop body covers NS stages; stages past the end multiply zeros

  // Loads: instruction j of a wave fills 16 rows of a stage; lane -> row lane/4, LDS slot lane%4, which receives the
  // global chunk slot ^ ((row/2)%4).  They are buffer loads (buffer_load_dwordx4 ... lds): the operand is described by
  // a resource in scalar registers, a lane contributes a 32-bit byte offset that stays the same for a whole segment,
  // and the walk along K is one scalar offset per load -- no per-lane 64-bit address arithmetic in the loop, and an
  // instruction that the wave issues faster than a global load with 64-bit addresses (measured: +8-11 % on the whole
  // kernel with nothing else changed).  What must read as zero is out of the resource's range, which the hardware
  // answers with zeros: rows past M lie behind num_records = M * lda, and lanes whose k is past the segment, stages
  // past the end and the absent half of a pair get the offset kOut (>= any num_records; the scalar offsets stay
  // below 2^31, so the sum cannot wrap back into range).
  const int drow = lane >> 2, dchunk = (lane & 3) ^ ((lane >> 3) & 3);
  constexpr unsigned kOut = 0x80000000u;
  constexpr int kRsrcFlags = 0x00020000;  // raw buffer of dwords
  const unsigned voffB = (unsigned)(drow * BK + dchunk * 8) * 2u;  // a lane's place inside a 16-row group of the weight side
  unsigned voffA[FM];                                             // and inside the activation operand: (row, chunk)
  __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(zero16), 0, 0, kRsrcFlags), rsB = rsA, rsB2 = rsA;
  unsigned soffA = 0, soffB[4] = {0u, 0u, 0u, 0u};
  bool pairseg = false;
  int seg = -1, k0 = 0, Kseg = 0, issued = 0;
  bool valid = n_stage > 0;

  // (macros rather than lambdas: arrays captured by reference were left in scratch memory by the compiler)
#define G2_OPEN_SEG()                                                                                                  \
  do {                                                                                                                 \
    for (++seg; seg < a.nseg; ++seg)                                                                                   \
      if (tn >= a.seg[seg].tile0 && tn < a.seg[seg].tile1 && a.seg[seg].K > 0) break;                                 \
    if (seg < a.nseg) {                                                                                                \
      const Gemm2Seg& sg = a.seg[seg];                                                                                 \
      Kseg = sg.K;                                                                                                     \
      k0 = 0;                                                                                                          \
      const unsigned ks_n = (unsigned)((sg.K + BK - 1) / BK);                                                          \
      const unsigned lda2 = (unsigned)sg.lda * 2u;                                                                     \
      rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(sg.A), 0, (int)((unsigned)a.M * lda2), kRsrcFlags); \
      soffA = 0;                                                                                                       \
      _Pragma("unroll") for (int j = 0; j < FM; ++j)                                                                   \
        voffA[j] = (unsigned)(m0 + (wave * FM + j) * 16 + drow) * lda2 + (unsigned)dchunk * 16u;                       \
      pairseg = sg.pair != 0;                                                                                          \
      const int bbytes = (int)((unsigned)((sg.rows + BN - 1) / BN) * ks_n * (unsigned)(BN * BK * 2));                  \
      rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(sg.B ? sg.B : sg.A), 0, sg.B ? bbytes : 0, kRsrcFlags);   \
      /* groups 2, 3 of a wave: the second matrix of a pair, else the same operand */                                  \
      {                                                                                                                \
        const unsigned short* b2 = pairseg ? sg.B2 : sg.B;                                                             \
        rsB2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(b2 ? b2 : sg.A), 0, b2 ? bbytes : 0, kRsrcFlags); \
      }                                                                                                                \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                                  \
        const int g16 = wave * 4 + j; /* 16-row group of the tile's weight side */                                     \
        /* row of the operand this group starts at; in a pair, groups with g16 & 2 (that is, j & 2) come from B2 */    \
        const unsigned brow = pairseg ? 128u * (unsigned)(tn - sg.tile0) + 32u * (unsigned)(g16 >> 2) + 16u * (unsigned)(g16 & 1) \
                                      : 256u * (unsigned)(tn - sg.tile0) + 16u * (unsigned)g16;                        \
        soffB[j] = ((brow >> 8) * ks_n * (unsigned)BN + (brow & 255u)) * (unsigned)(BK * 2);                           \
      }                                                                                                                \
    }                                                                                                                  \
  } while (0)
  // moves the cursor to the stage after the one just issued
#define G2_ADVANCE()                                                                                                   \
  do {                                                                                                                 \
    ++issued;                                                                                                          \
    valid = issued < n_stage;                                                                                          \
    if (valid) {                                                                                                       \
      k0 += BK;                                                                                                        \
      if (k0 >= Kseg) {                                                                                                \
        G2_OPEN_SEG();                                                                                                 \
      } else {                                                                                                         \
        soffA += BK * 2;                                                                                               \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) soffB[j] += BN * BK * 2;                                         \
      }                                                                                                                \
    }                                                                                                                  \
  } while (0)
#define G2_BL(rs, voff, soff, sp) \
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)(sp), 16, (int)(voff), (int)(soff), 0, 0)
#define G2_ISSUE(buf)                                                                                                  \
  do {                                                                                                                 \
    char* SA = smem + (buf) * STG;                                                                                     \
    char* SB = SA + ASZ;                                                                                               \
    const bool kok = valid && (k0 + dchunk * 8 < Kseg);                                                                \
    _Pragma("unroll") for (int j = 0; j < FM; ++j) G2_BL(rsA, kok ? voffA[j] : kOut, soffA, SA + (wave * FM + j) * 1024); \
    const unsigned vb = valid ? voffB : kOut;                                                                          \
    G2_BL(rsB, vb, soffB[0], SB + (wave * 4 + 0) * 1024);                                                              \
    G2_BL(rsB, vb, soffB[1], SB + (wave * 4 + 1) * 1024);                                                              \
    G2_BL(rsB2, vb, soffB[2], SB + (wave * 4 + 2) * 1024);                                                             \
    G2_BL(rsB2, vb, soffB[3], SB + (wave * 4 + 3) * 1024);                                                             \
  } while (0)

  // fragment reads: row lane%32, 16-byte chunk 2 sub + lane/32, swizzled like the loads
  const int sw = ((lane & 31) >> 1) & 3;
  const int fo0 = (lane & 31) * 64 + ((lane >> 5) ^ sw) * 16;
  const int fo1 = fo0 ^ 32;
  const int aoff = wm * (FM * 32) * 64, boff = ASZ + wn * 128 * 64;
  u32x4 fa0[FM], fb0[4], fa1[FM], fb1[4];
#define G2_RD(FA, FB, buf, sub)                                                                                        \
  do {                                                                                                                 \
    const char* sa_ = smem + (buf) * STG + aoff + ((sub) ? fo1 : fo0);                                                 \
    const char* sb_ = smem + (buf) * STG + boff + ((sub) ? fo1 : fo0);                                                 \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) FA[i] = *reinterpret_cast<const u32x4*>(sa_ + i * 2048);            \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) FB[j] = *reinterpret_cast<const u32x4*>(sb_ + j * 2048);             \
  } while (0)
#define G2_MM(FA, FB)                                                                                                  \
  do {                                                                                                                 \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)                       \
        acc[i][j] = HALF ? __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, FA[i]),                    \
                                                                  __builtin_bit_cast(f16x8, FB[j]), acc[i][j], 0, 0, 0) \
                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, FA[i]),                  \
                                                                   __builtin_bit_cast(bf16x8, FB[j]), acc[i][j], 0, 0, 0); \
  } while (0)
  // issue order of a half step: the FM + 4 fragment reads ride on the first MFMAs, then one load per MFMA
  constexpr int kRd = (FM + 4) / 2;             // MFMAs that carry the fragment reads (two reads each)
  constexpr int kRest = 4 * FM - kRd;           // MFMAs left in the half step
  constexpr int kLd = LOADS < kRest ? LOADS : kRest;  // loads that get an MFMA of their own
#define G2_PIPE_RD()                                                                                                   \
  do {                                                                                                                 \
    _Pragma("unroll") for (int q = 0; q < kRd; ++q) { G2_SGB(0x008, 1); G2_SGB(0x100, 2); }                            \
  } while (0)
#define G2_PIPE1()                                                                                                     \
  do {                                                                                                                 \
    G2_PIPE_RD();                                                                                                      \
    G2_SGB(0x008, kRest);                                                                                              \
  } while (0)
#define G2_PIPE2()                                                                                                     \
  do {                                                                                                                 \
    G2_PIPE_RD();                                                                                                      \
    _Pragma("unroll") for (int q = 0; q < kLd; ++q) { G2_SGB(0x008, 1); G2_SGB(0x020, 1); }                            \
    if (LOADS > kLd) G2_SGB(0x020, LOADS - kLd);                                                                       \
    if (kRest > kLd) G2_SGB(0x008, kRest - kLd);                                                                       \
  } while (0)
#define G2_STEP(cur, nxt, dma)                                                                                         \
  do {                                                                                                                 \
    G2_RD(fa1, fb1, cur, 1);                                                                                           \
    G2_MM(fa0, fb0);                                                                                                   \
    G2_PIPE1();                                                                                                        \
    G2_SB0();                                                                                                          \
    G2_ADVANCE();                                                                                                      \
    G2_WAITV((NS - 3) * LOADS); /* all but the NS - 3 newest stages in flight have landed: stage `nxt` is in LDS */   \
    __builtin_amdgcn_s_barrier();                                                                                      \
    G2_SB0();                                                                                                          \
    G2_RD(fa0, fb0, nxt, 0);                                                                                           \
    G2_ISSUE(dma);                                                                                                     \
    G2_MM(fa1, fb1);                                                                                                   \
    G2_PIPE2();                                                                                                        \
    G2_SB0();                                                                                                          \
  } while (0)

  const bool probe = a.clk != nullptr && blockIdx.x == 0;
  long long c_start = 0, w_start = 0;
  if (probe) c_start = clock64(), w_start = wall_clock64();
  if (n_stage > 0) {
    G2_OPEN_SEG();
    G2_ISSUE(0);
    G2_ADVANCE();
    G2_ISSUE(1);
    G2_ADVANCE();
    G2_ISSUE(2);
    if constexpr (NS == 6) {
      G2_ADVANCE();
      G2_ISSUE(3);
      G2_ADVANCE();
      G2_ISSUE(4);
    }
    G2_WAITV((NS - 2) * LOADS);
    __builtin_amdgcn_s_barrier();
    G2_RD(fa0, fb0, 0, 0);
    G2_SB0();
    for (int st = 0; st < n_step; st += NS) {
      if constexpr (NS == 4) {
        G2_STEP(0, 1, 3);
        G2_STEP(1, 2, 0);
        G2_STEP(2, 3, 1);
        G2_STEP(3, 0, 2);
      } else {
        G2_STEP(0, 1, 5);
        G2_STEP(1, 2, 0);
        G2_STEP(2, 3, 1);
        G2_STEP(3, 4, 2);
        G2_STEP(4, 5, 3);
        G2_STEP(5, 0, 4);
      }
    }
    G2_WAITV(0);
  }
  if (probe && tid == 0) a.clk[0] = clock64() - c_start, a.clk[1] = wall_clock64() - w_start;
  __syncthreads();  // every wave is done with the stage buffers: the epilogue reuses them
#undef G2_OPEN_SEG
#undef G2_ADVANCE
#undef G2_ISSUE
#undef G2_BL
#undef G2_RD
#undef G2_MM
#undef G2_PIPE_RD
#undef G2_PIPE1
#undef G2_PIPE2
#undef G2_STEP

  // ---- epilogue ---------------------------------------------------------------------------------------------------
  // Output block of this tile and its first column inside the block.
  Gemm2Out out = a.out[0];
  if (a.nout > 1 && tn >= a.out[1].tile0) out = a.out[1];
  if (a.nout > 2 && tn >= a.out[2].tile0) out = a.out[2];
  constexpr int ER = (128 + 8) * 4;  // staged row in bytes; 4 rows further = 32 banks further
  static_assert(4 * 32 * ER <= NS * STG, "epilogue staging must fit the stage buffers");
  char* ebuf = smem + wave * (32 * ER);
  bool clamped = false;
  const int mrow_w = m0 + wm * (FM * 32);
  g2_store_slab<HALF, EPI>(acc[0][0], acc[0][1], acc[0][2], acc[0][3], ebuf, a, out, tn, wn, lane, mrow_w, clamped);
  g2_store_slab<HALF, EPI>(acc[1][0], acc[1][1], acc[1][2], acc[1][3], ebuf, a, out, tn, wn, lane, mrow_w + 32, clamped);
  if constexpr (FM == 4) {
    g2_store_slab<HALF, EPI>(acc[2][0], acc[2][1], acc[2][2], acc[2][3], ebuf, a, out, tn, wn, lane, mrow_w + 64, clamped);
    g2_store_slab<HALF, EPI>(acc[3][0], acc[3][1], acc[3][2], acc[3][3], ebuf, a, out, tn, wn, lane, mrow_w + 96, clamped);
  }
  if (clamped && a.overflow_flag) atomicOr(a.overflow_flag, 8);
}

// ---- blocked copies ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_block_jobs(BlockJobs jobs) {
  const BlockJob jb = jobs.j[blockIdx.y];
  const long long N = jb.transpose ? jb.C : jb.R, K = jb.transpose ? jb.R : jb.C;
  const long long ks_n = (K + BK - 1) / BK;
  const long long total = (long long)blocked_elems(N, K) / 8;  // 16-byte chunks of the destination
  bool over = false;
  for (long long ci = (long long)blockIdx.x * 256 + threadIdx.x; ci < total; ci += (long long)gridDim.x * 256) {
    const long long e0 = ci * 8;  // first element of the chunk: ((tile * ks_n + ks) * 256 + row) * 32 + kk
    const int kk = (int)(e0 & 31), row = (int)((e0 >> 5) & 255);
    const long long tk = e0 >> 13, ks = tk % ks_n, tile = tk / ks_n;
    const long long n = tile * BN + row, k = ks * BK + kk;
    unsigned short v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      v[e] = 0;
      if (n < N && k + e < K) {
        const long long si = jb.transpose ? (k + e) * jb.C + n : n * jb.C + k + e;
        if (jb.src_f32 == 2) {  // already in the compute element: bits as they are
          v[e] = static_cast<const unsigned short*>(jb.src)[si];
        } else {
          const float f = jb.src_f32 ? static_cast<const float*>(jb.src)[si] : bf2f(static_cast<const unsigned short*>(jb.src)[si]);
          v[e] = jobs.half ? f2h(f) : f2bf(f);
          over = over || (jobs.half && !(fabsf(f) <= 65504.f));
        }
      }
    }
    *reinterpret_cast<uint4*>(jb.dst + e0) = make_uint4(v[0] | (unsigned)v[1] << 16, v[2] | (unsigned)v[3] << 16, v[4] | (unsigned)v[5] << 16,
                                                        v[6] | (unsigned)v[7] << 16);
  }
  if (over && jobs.flag) atomicOr(jobs.flag, 8);
}

template <int FM>
constexpr int lds_bytes() { return stages<FM>() * (64 * FM * BK * 2 + BSZ); }

int g_force_fm = 0;  // measurement hook: 2 or 4 fixes the tile height

}  // namespace

void gemm2_force_tile_rows(int rows) { g_force_fm = rows == 256 ? 4 : rows == 128 ? 2 : 0; }

void gemm2_block_jobs(const BlockJobs& jobs, hipStream_t st) {
  if (jobs.n < 1) return;
  hipLaunchKernelGGL(k_block_jobs, dim3(256, jobs.n), dim3(256), 0, st, jobs);
}

// Grid of a launch: the XCD-aware tile order of the kernel and its cost in rounds of tiles over n_cu compute units.
Gemm2Plan gemm2_plan(int M, int tiles_n, int FM, int n_cu) {
  Gemm2Plan p{};
  const int BM = 64 * FM, tiles_m = (M + BM - 1) / BM;
  // The 32 workgroups an XCD runs at a time form one GM x GN block of tiles about 1024 x 2048 outputs large, so that
  // they share GM + GN operand panels in its L2.
  p.GM = std::min(FM == 2 ? 8 : 4, tiles_m);
  p.GN = std::min(FM == 2 ? 4 : 8, tiles_n);
  p.total = ((tiles_m + p.GM - 1) / p.GM) * ((tiles_n + p.GN - 1) / p.GN) * p.GM * p.GN;  // whole blocks: slots past the matrix return at once
  p.chunk = (p.total + 7) / 8;
  p.grid = p.chunk * 8;
  p.rounds = (tiles_m * tiles_n + n_cu - 1) / n_cu;
  return p;
}

harli_status gemm2_launch(const Gemm2Args& a, hipStream_t st) {
  if (a.M < 1 || a.nseg < 1 || a.nseg > kGemm2MaxSeg || a.nout < 1 || a.nout > kGemm2MaxOut || a.tiles_n < 1)
    return fail(HARLI_ERR_INVALID, "gemm2: bad shape M %d nseg %d nout %d tiles %d", a.M, a.nseg, a.nout, a.tiles_n);
  for (int s = 0; s < a.nseg; ++s) {
    const Gemm2Seg& g = a.seg[s];
    if (!g.A || g.K < 8 || (g.K & 7) || (g.lda & 7) || ((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15) || ((uintptr_t)g.B2 & 15) ||
        g.tile0 < 0 || g.tile1 > a.tiles_n || g.tile0 >= g.tile1 || (g.pair ? (!g.B && !g.B2) : (!g.B || g.B2)))
      return fail(HARLI_ERR_INVALID, "gemm2: segment %d needs K %% 8 == 0, 16-byte aligned operands and a tile range inside the output (K %d lda %lld tiles %d..%d)",
                  s, g.K, g.lda, g.tile0, g.tile1);
  }
  const bool f32out = a.out[0].Cf != nullptr;
  for (int s = 0; s < a.nseg; ++s) {
    // the kernel addresses row tiles of the weight operands from the tile range alone: the range must stay inside them
    const Gemm2Seg& g = a.seg[s];
    const int row_tiles = (g.rows + BN - 1) / BN, span = g.tile1 - g.tile0;
    if (g.rows < 1 || (g.pair ? (span + 1) / 2 : span) > row_tiles)
      return fail(HARLI_ERR_INVALID, "gemm2: segment %d: a weight operand of %d rows cannot cover output tiles %d..%d", s, g.rows, g.tile0, g.tile1);
    // the kernel addresses both operands with 32-bit byte offsets below 2^31
    if (((long long)a.M + 255) * g.lda * 2 >= (1ll << 31) || (long long)blocked_elems(g.rows, g.K) * 2 >= (1ll << 31))
      return fail(HARLI_ERR_INVALID, "gemm2: segment %d: an operand of 2 GiB or more (M %d, lda %lld, %d weight rows, K %d)", s, a.M, g.lda, g.rows, g.K);
  }
  for (int o = 0; o < a.nout; ++o) {
    const Gemm2Out& q = a.out[o];
    if ((q.Cf != nullptr) != f32out) return fail(HARLI_ERR_INVALID, "gemm2: the output blocks of a launch are all fp32 or all 16-bit");
    const int t_end = o + 1 < a.nout ? a.out[o + 1].tile0 : a.tiles_n;
    const int width = a.epi == GEMM2_EPI_GATEUP ? 128 : BN;  // columns of the block per tile
    if (q.tile0 < 0 || q.tile0 >= t_end || (o == 0 && q.tile0 != 0) || q.N < 1 || q.N > (t_end - q.tile0) * width)
      return fail(HARLI_ERR_INVALID, "gemm2: output block %d (tiles %d..%d) cannot hold %d columns", o, q.tile0, t_end, q.N);
    if (a.epi == GEMM2_EPI_NONE && !q.Cb && !q.Cf) return fail(HARLI_ERR_INVALID, "gemm2: output block %d has no destination", o);
    if (q.res && !q.Cf) return fail(HARLI_ERR_INVALID, "gemm2: a residual needs the fp32 output");
    if (q.Cb && !q.Cf && ((q.ldcb & 7) || (q.N & 7) || ((uintptr_t)q.Cb & 15)))
      return fail(HARLI_ERR_INVALID, "gemm2: a 16-bit output needs N and its row stride to be multiples of 8");
    if (q.Cf && ((q.ldcf & 3) || ((uintptr_t)q.Cf & 15) || ((uintptr_t)q.res & 15) || (q.Cb && ((q.ldcb & 3) || ((uintptr_t)q.Cb & 7)))))
      return fail(HARLI_ERR_INVALID, "gemm2: an fp32 output needs a row stride that is a multiple of 4 and aligned pointers");
  }
  if (a.epi != GEMM2_EPI_NONE) {
    const bool gu = a.epi == GEMM2_EPI_GATEUP;
    if ((a.epi != GEMM2_EPI_GATEUP && a.epi != GEMM2_EPI_SWIGLU_BWD) || a.nout != 1 || a.out[0].Cf || (a.out[0].N & 7) || (a.lde & 7) ||
        !a.o0 || !a.o1 || (gu ? (!a.out[0].Cb) : (!a.e0 || !a.e1 || a.out[0].Cb)) ||
        (((uintptr_t)a.e0 | (uintptr_t)a.e1 | (uintptr_t)a.o0 | (uintptr_t)a.o1) & 15))
      return fail(HARLI_ERR_INVALID, "gemm2: fused SwiGLU epilogue %d needs one block, N and lde %% 8 == 0 and its own aligned outputs", a.epi);
    for (int s = 0; s < a.nseg; ++s)
      if ((a.seg[s].pair != 0) != gu) return fail(HARLI_ERR_INVALID, "gemm2: interleaved pairs go with the gate/up epilogue and only with it");
  }
  static bool attr_set = false;
  static uint4* zero16 = nullptr;  // 256 zero bytes in device memory, kept for the life of the process
  if (!attr_set) {
    HARLI_HIP(hipMalloc(reinterpret_cast<void**>(&zero16), 256));
    HARLI_HIP(hipMemset(zero16, 0, 256));
#define G2_ATTR(F_, H_, E_) \
  HARLI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm2<F_, H_, E_>), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes<F_>()))
#define G2_ATTR4(F_, H_) \
  G2_ATTR(F_, H_, GEMM2_EPI_NONE); G2_ATTR(F_, H_, GEMM2_EPI_F32); G2_ATTR(F_, H_, GEMM2_EPI_SWIGLU_BWD); G2_ATTR(F_, H_, GEMM2_EPI_GATEUP)
    G2_ATTR4(2, true); G2_ATTR4(4, true); G2_ATTR4(2, false); G2_ATTR4(4, false);
#undef G2_ATTR4
#undef G2_ATTR
    attr_set = true;
  }
  int n_cu = a.n_cu > 0 ? a.n_cu : cu_stream_count(st);
  if (n_cu < 1) {
    n_cu = 256;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
  }
  const Gemm2Plan p4 = gemm2_plan(a.M, a.tiles_n, 4, n_cu), p2 = gemm2_plan(a.M, a.tiles_n, 2, n_cu);
  // Tile height: rounds of workgroups over the compute units of the stream, a 128-row tile costed at 0.55 of a 256-row
  // one (it moves 3/4 of the operand bytes for half the flops).
  int FM = (a.M > 128 && p4.rounds <= 0.55 * p2.rounds) ? 4 : 2;
  if (g_force_fm == 2 || g_force_fm == 4) FM = g_force_fm;
  const Gemm2Plan& pl = FM == 4 ? p4 : p2;
  const int GM = pl.GM, GN = pl.GN, total = pl.total, chunk = pl.chunk, grid = pl.grid;
#define G2_LAUNCH(F_, H_, E_) \
  hipLaunchKernelGGL((k_gemm2<F_, H_, E_>), dim3(grid), dim3(NT), lds_bytes<F_>(), st, a, total, chunk, GM, GN, zero16)
#define G2_PICK(F_)                                                                    \
  do {                                                                                 \
    if (a.half) {                                                                      \
      if (a.epi == GEMM2_EPI_GATEUP) G2_LAUNCH(F_, true, GEMM2_EPI_GATEUP);            \
      else if (a.epi == GEMM2_EPI_SWIGLU_BWD) G2_LAUNCH(F_, true, GEMM2_EPI_SWIGLU_BWD); \
      else if (f32out) G2_LAUNCH(F_, true, GEMM2_EPI_F32);                             \
      else G2_LAUNCH(F_, true, GEMM2_EPI_NONE);                                        \
    } else {                                                                           \
      if (a.epi == GEMM2_EPI_GATEUP) G2_LAUNCH(F_, false, GEMM2_EPI_GATEUP);           \
      else if (a.epi == GEMM2_EPI_SWIGLU_BWD) G2_LAUNCH(F_, false, GEMM2_EPI_SWIGLU_BWD); \
      else if (f32out) G2_LAUNCH(F_, false, GEMM2_EPI_F32);                            \
      else G2_LAUNCH(F_, false, GEMM2_EPI_NONE);                                       \
    }                                                                                  \
  } while (0)
  // flops asked for: 2 M K per valid output column a segment reaches (an interleaved pair fills both halves of a tile)
  double flops = 0;
  for (int s = 0; s < a.nseg; ++s) {
    long long cols = 0;
    for (int o = 0; o < a.nout; ++o) {
      const int T0 = a.out[o].tile0, T1 = o + 1 < a.nout ? a.out[o + 1].tile0 : a.tiles_n;
      const int lo = std::max(a.seg[s].tile0, T0), hi = std::min(a.seg[s].tile1, T1);
      if (hi <= lo) continue;
      const long long width = a.epi == GEMM2_EPI_GATEUP ? 128 : BN;
      const long long c0 = (long long)(lo - T0) * width, c1 = std::min<long long>((long long)(hi - T0) * width, a.out[o].N);
      if (c1 > c0) cols += (c1 - c0) * (a.epi == GEMM2_EPI_GATEUP ? ((a.seg[s].B != nullptr) + (a.seg[s].B2 != nullptr)) : 1);
    }
    flops += 2.0 * a.M * (double)cols * a.seg[s].K;
  }
  GemmTimer timer;
  HARLI_HIP(timer.begin(flops, st));
  if (FM == 4) G2_PICK(4);
  else G2_PICK(2);
#undef G2_PICK
#undef G2_LAUNCH
  HARLI_HIP(timer.end(st));
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}

}  // namespace harli
