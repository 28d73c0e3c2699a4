// libccoll_szx: SZx block compression, decompression and the fused reduce step of C-Coll
// (arXiv 2304.03890) as HIP kernels for gfx950, behind the C ABI of include/ccoll_szx.h.
//
// Mapping to the hardware
//   * one wavefront per 5120-element chunk (Sec. III-E.2), 8 blocks (1024 elements) at a time: half a DPP
//     row (8 lanes) per 128-element block, 16 consecutive elements per lane, so a lane moves 64 contiguous
//     bytes as four 16-byte accesses and every block-wide reduction or scan is three DPP steps.  Wavefronts
//     are independent of each other inside a chunk: no barrier, every SIMD gets the same load;
//   * the chunk payload is assembled in the wavefront's own piece of LDS and leaves as 16-byte stores; what
//     outgrows that piece moves on to a per-wavefront spill slot in global memory while the chunk is coded;
//   * the wavefronts of a workgroup take consecutive chunks (a group).  Groups are handed out by a ticket
//     counter; their byte offsets come from a single-pass decoupled look-back scan over the group sizes.  A
//     payload is placed one turn after it was coded, when the groups in front have announced their sizes:
//     meanwhile it stays in LDS (a wavefront has two stages and uses them in turns); block bodies are ORed into
//     the zeroed stage as whole aligned words, gathered four elements at a time in registers;
//   * the reduce step (Sec. III-A.2, Eq. 2) is the coder with another source of elements: the local floats plus
//     the incoming chunk, decoded out of a window that shares the stage with the bodies being coded;
//   * the decompressor needs no scan between workgroups: one small kernel turns the stream's front index into
//     chunk offsets, then every wavefront decodes a chunk out of a sliding window of its payload in LDS and
//     writes whole 64-byte lines with streaming stores.
// No MFMA: the path is a streaming codec bound by instruction issue and HBM, not by a contraction.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <string.h>
#include <math.h>
#include <new>
#include <mutex>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/ccoll_szx.h"

#ifndef CCOLL_RED_OCC
#define CCOLL_RED_OCC 3
#endif

namespace {

typedef uint32_t u32;
typedef uint64_t u64;
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int kBlock = CCOLL_BLOCK_ELEMS;            // 128
constexpr int kChunk = CCOLL_CHUNK_ELEMS;            // 5120
constexpr int kBpc = kChunk / kBlock;                // 40 blocks per chunk
constexpr int kE = 16;                               // elements per lane
constexpr int kGrp = kBlock / kE;                    // 8 lanes per block
constexpr u32 kHeader = 32;
constexpr u32 kMaxPayload = 8 + 4 * 40 + 2 * 40 + 40 + 40 * (32 + 512);   // 22048
constexpr int kUnit = 8 * kBlock;                    // elements a wavefront handles per step: 8 blocks
constexpr int kUnits = kChunk / kUnit;               // 5

// ---- look-back status words: [63:62] flag, [61:36] launch epoch, [35:0] byte count -------------
constexpr u64 kFlagA = 1ull << 62;                   // this chunk's own size is known
constexpr u64 kFlagP = 2ull << 62;                   // inclusive prefix is known
constexpr u64 kFlagMask = 3ull << 62;
constexpr int kEpochShift = 36;
constexpr u64 kEpochMask = ((1ull << 26) - 1) << kEpochShift;
constexpr u64 kValueMask = (1ull << kEpochShift) - 1;
constexpr u32 kSpinLimit = 1u << 22;                 // polls before a scan wait gives up (seconds)

struct Workspace {            // lives in device memory, one per context
  u64 total;                  // stream bytes written by the call in flight
  u64 err;                    // (epoch << 8) | (code << 4) | detail of the call in flight
  u64 abort;                  // epoch of a call whose scan wait timed out
  u64 ticket[2];              // groups of chunks handed out: launches use the two counters in turns, and every
                              // launch zeroes the one the next launch will use (whatever way it ends itself)
  u64 idx_bad;                // epoch of a ccoll_szx_index call that found its stream malformed
  u64 pad[2];
};

struct Params {
  const void* in;             // compress: floats; decompress: stream
  void* out;                  // compress: stream; decompress: floats
  const float* local;         // reduce step: local floats
  const void* cin;            // reduce step: incoming stream
  u64 n;                      // elements of the whole stream
  u64 in_bytes;               // decompress / reduce: bytes available in the incoming stream
  u64 out_cap;                // compress / reduce: capacity of the output stream
  u64 first, count;           // decompress: element range
  u32 nchunks;                // chunks of the whole stream
  u32 c0, c1;                 // chunk range [c0, c1) handled by this launch
  float eb;
  int e_eb;                   // floor(log2(eb))
  u32 eb_bits;
  u32 epoch;
  u32 aligned16;              // float pointers are 16-byte aligned
  Workspace* ws;
  u64* stat;                  // look-back status of the outgoing stream, one word per chunk
  u64* offs;                  // byte offset of every chunk of the incoming stream (from k_index_scan)
  u64* result;                // {bytes, status} for the caller, or null
  u32 no_total;               // k_publish: the call reports no byte count
  u32 ticket_sel;             // which of the two ticket counters this launch draws from
  u32 spin_limit;             // polls after which a scan wait gives up
  u32 scan_epoch;             // tag of the look-back status words: the call's epoch, or, for the pieces of a stream that
                              // is compressed piece by piece, the epoch of the call that began the stream
  u32 scan_chunks;            // incoming stream: index entries to walk (all, or those that have arrived of an open stream)
  u32 open_stream;            // incoming stream: still being written (the header's total is not final)
  unsigned long long* progress;  // compress: {chunks coded, stream bytes final} of the launch, or null
  u32 idx_epoch;              // decompress with kept chunk offsets: the epoch of the ccoll_szx_index call that made them
  u32 index_call;             // k_index_scan runs for ccoll_szx_index: a malformed stream is also noted in ws->idx_bad
  unsigned char* spill;       // per-wavefront slots for payloads whose place in the stream is not known yet
};


// Parameters that the kernels need once per turn or less (the scan words, the output, capacities, epochs) are read
// from the kernel argument segment where they are used, by a scalar load the compiler may not hoist or keep: held
// in registers for the whole kernel they would push the coder's hot loop, which is short of scalar registers, into
// spilling them through vector registers and scratch memory.  Every kernel that uses these helpers takes the
// Params block as its first argument.
template <u32 OFF>
__device__ __forceinline__ u32 karg32() {
  u32 v;
  asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(__builtin_amdgcn_kernarg_segment_ptr()), "n"(OFF));
  return v;
}
template <u32 OFF>
__device__ __forceinline__ u64 karg64() {
  u64 v;
  asm volatile("s_load_dwordx2 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(__builtin_amdgcn_kernarg_segment_ptr()), "n"(OFF));
  return v;
}
#define KARG32(field) karg32<(u32)offsetof(Params, field)>()
#define KARG64(field) karg64<(u32)offsetof(Params, field)>()
#define KARGP(type, field) ((type)karg64<(u32)offsetof(Params, field)>())

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ u32 dpp0(u32 v) {   // lanes without a source read 0
  return (u32)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114;
constexpr int kQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kHalfMirror = 0x141;   // lane i <- lane 7-i inside each half row

// Reductions over the 8 lanes of a block: every lane gets the result.
__device__ __forceinline__ u32 grp_max_u32(u32 v) {
  v = max(v, dpp0<kQuadXor1>(v)); v = max(v, dpp0<kQuadXor2>(v)); v = max(v, dpp0<kHalfMirror>(v));
  return v;
}
__device__ __forceinline__ int grp_max_i32(int v) {
  v = max(v, (int)dpp0<kQuadXor1>((u32)v)); v = max(v, (int)dpp0<kQuadXor2>((u32)v)); v = max(v, (int)dpp0<kHalfMirror>((u32)v));
  return v;
}
__device__ __forceinline__ int grp_min_i32(int v) {
  v = min(v, (int)dpp0<kQuadXor1>((u32)v)); v = min(v, (int)dpp0<kQuadXor2>((u32)v)); v = min(v, (int)dpp0<kHalfMirror>((u32)v));
  return v;
}
__device__ __forceinline__ u32 grp_or_u32(u32 v) {
  v |= dpp0<kQuadXor1>(v); v |= dpp0<kQuadXor2>(v); v |= dpp0<kHalfMirror>(v);
  return v;
}
// Lane masks that stop a row shift at the boundary between the two blocks of a DPP row.
struct GrpMasks { u32 m1, m2, m4; };
__device__ __forceinline__ GrpMasks grp_masks() {
  const u32 l = threadIdx.x & 7u;
  GrpMasks m; m.m1 = l >= 1 ? ~0u : 0u; m.m2 = l >= 2 ? ~0u : 0u; m.m4 = l >= 4 ? ~0u : 0u;
  return m;
}
// value of the lane to the left inside the block, 0 for the block's first lane
__device__ __forceinline__ u32 grp_left(u32 v, const GrpMasks& m) { return dpp0<kRowShr1>(v) & m.m1; }
// inclusive sum over the 8 lanes of a block
__device__ __forceinline__ u32 grp_scan_add(u32 v, const GrpMasks& m) {
  v += dpp0<kRowShr1>(v) & m.m1; v += dpp0<kRowShr2>(v) & m.m2; v += dpp0<kRowShr4>(v) & m.m4;
  return v;
}
// inclusive sum over the wavefront: Hillis-Steele inside each row, then the row totals
__device__ __forceinline__ u32 wave_scan_add(u32 v) {
  v += dpp0<kRowShr1>(v); v += dpp0<kRowShr2>(v); v += dpp0<kRowShr4>(v); v += dpp0<0x118>(v);
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return v;
}
__device__ __forceinline__ u64 wave_sum_u64(u64 v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ u32 f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(u32 u) { return __uint_as_float(u); }
__device__ __forceinline__ u32 bswap32(u32 v) { return __builtin_amdgcn_perm(0u, v, 0x00010203u); }
__device__ __forceinline__ u32 pad4(u32 v) { return (v + 3u) & ~3u; }

// Selection by a lane mask (all ones / all zeros) that the compiler cannot see through: it stays a bit operation.
// A select would become v_cndmask_b32 in its short encoding, which this device issues six times slower than
// other vector instructions (measured: 23 cycles per wavefront instruction against 3 to 4).
__device__ __forceinline__ u32 lane_mask(bool c) { u32 m = c ? ~0u : 0u; asm("" : "+v"(m)); return m; }
__device__ __forceinline__ u32 sel_mask(u32 m, u32 a, u32 b) {      // m ? a : b bit by bit, as one v_bitop3_b32 (the fast class)
  u32 r;
  asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0xca" : "=v"(r) : "v"(m), "v"(a), "v"(b));
  return r;
}

__device__ __forceinline__ void lds_store16(unsigned char* p, u32 v) { unsigned short s = (unsigned short)v; __builtin_memcpy(p, &s, 2); }
__device__ __forceinline__ void lds_store32(unsigned char* p, u32 v) { __builtin_memcpy(p, &v, 4); }
__device__ __forceinline__ u32 lds_load32(const unsigned char* p) { u32 v; __builtin_memcpy(&v, p, 4); return v; }
// The 4 bytes at any byte address of LDS, from the two aligned words that hold them: an unaligned LDS
// access is replayed lane by lane, two aligned words cost one ds_read2_b32.
__device__ __forceinline__ u32 lds_load32_any(const unsigned char* base, u32 addr) {
  const u32* q = (const u32*)(base + (addr & ~3u));
  return __builtin_amdgcn_alignbyte(q[1], q[0], addr);
}
__device__ __forceinline__ u32 lds_load16(const unsigned char* p) { unsigned short s; __builtin_memcpy(&s, p, 2); return s; }
// OR into an aligned LDS word.  Only the wavefront that owns the word touches it; LDS executes a wavefront's
// operations in order, so later reads of the word by the same wavefront see the result.
__device__ __forceinline__ void lds_or32(u32* p, u32 v) { __hip_atomic_fetch_or(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT); }

// Device-scope relaxed atomics: they bypass the per-XCD L2, so workgroups on different XCDs see each
// other's words without any cache write-back or invalidate.
__device__ __forceinline__ u64 ld_dev(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(u64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// detail: which check failed (1 header, 2 index entry, 3 range base, 4 bounds, 5 index sum, 6 chunk
// metadata, 7 block body, 8 scan wait); reported on stderr by ccoll_wait when CCOLL_DEBUG is set.
__device__ __forceinline__ void raise_error(const Params& P, int code, u32 detail = 0) {
  // codes are negative; keep the most severe (most negative) one of this epoch
  (void)P;
  Workspace* ws = KARGP(Workspace*, ws);
  const u32 epoch = KARG32(epoch);
  u64 word = ((u64)epoch << 8) | ((u64)(u32)(-code) << 4) | (u64)(detail & 15u);
  __hip_atomic_fetch_max(&ws->err, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (KARG32(index_call)) __hip_atomic_fetch_max(&ws->idx_bad, (u64)epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- decoupled look-back over the sizes of the outgoing chunks (first wavefront, all 64 lanes) ----
__device__ __forceinline__ void publish_size(u64* stat, u32 c, u64 mine, u32 epoch) {
  if ((threadIdx.x & 63u) == 0) st_dev(stat + c, (c == 0 ? kFlagP : kFlagA) | ((u64)epoch << kEpochShift) | mine);
}
// Exclusive prefix of the sizes of entries [0, c) of the scan; waits (bounded) for entries that have not been
// announced yet.  Returns true: known (and published for the entries behind), false: the wait was abandoned
// (error raised).  Four windows of 64 status words are fetched per round trip.
__device__ __forceinline__ bool lookback(u64* stat, u32 c, u64 mine, const Params& P, u64& excl_out) {
  const u32 lane = threadIdx.x & 63u;
  const u64 tag = (u64)KARG32(scan_epoch) << kEpochShift;
  u64 excl = 0;
  if (c > 0) {
    long long look = (long long)c - 1;
    u32 polls = 0;
    bool done = false;
    while (!done) {
      u64 s[4];
      while (true) {
        bool ready = true;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const long long j = look - 64 * q - (long long)lane;
          s[q] = (j >= 0) ? ld_dev(stat + j) : (kFlagP | tag);
          ready = ready && ((s[q] & kEpochMask) == tag) && ((s[q] & kFlagMask) != 0);
        }
        if (__ballot(!ready) == 0) break;
        ++polls;
        const u32 spin_limit = KARG32(spin_limit);
        if ((polls & 63u) == 0 || polls >= spin_limit) {
          Workspace* ws = KARGP(Workspace*, ws);
          const u64 epoch = KARG32(epoch);
          const bool stop = polls >= spin_limit || ld_dev(&ws->abort) == epoch;
          if (stop) {                                   // uniform: every lane reads the same words
            if (lane == 0) { st_dev(&ws->abort, epoch); raise_error(P, CCOLL_ETIMEDOUT, 8); }
            excl_out = 0;
            return false;
          }
        }
        __builtin_amdgcn_s_sleep(2);
      }
      // Sizes in front of the nearest full prefix are group sizes (< 2^20 each, at most 256 per round trip): they are
      // added up in 32 bits, per lane over the four windows and then over the wavefront with one DPP scan; the
      // prefix itself (36 bits) is read from its lane.
      u32 part = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (!done) {
          const u64 pmask = __ballot((s[q] & kFlagMask) == kFlagP);
          const u64 v = s[q] & kValueMask;
          if (pmask) {
            const int first = __ffsll((long long)pmask) - 1;     // nearest predecessor with a full prefix
            excl += ((u64)(u32)__builtin_amdgcn_readlane((int)(u32)(v >> 32), first) << 32) |
                    (u64)(u32)__builtin_amdgcn_readlane((int)(u32)v, first);
            if ((int)lane < first) part += (u32)v;
            done = true;
          } else {
            part += (u32)v;
          }
        }
      }
      excl += (u64)(u32)__builtin_amdgcn_readlane((int)wave_scan_add(part), 63);
      look -= 256;
    }
    if (lane == 0) st_dev(stat + c, kFlagP | tag | (excl + mine));
  }
  excl_out = excl;
  return true;
}

// ---------------------------------------------------------------------------------------------
// block classification (every lane of the block computes the same result)
//   type 0: constant, 1: non-constant with m mantissa bits, 2: raw
// ---------------------------------------------------------------------------------------------
struct RowClass { u32 type; float mu; u32 m; };

__device__ __forceinline__ RowClass classify_row(const u32 (&xb)[kE], float eb, int e_eb) {
  // min / max under the total order of the bit patterns, plus NaN / Inf detection, from three
  // integer reductions: signed max, signed min, unsigned max.
  int smax = (int)xb[0], smin = (int)xb[0]; u32 umax = xb[0];
#pragma unroll
  for (int k = 1; k < kE; ++k) { smax = max(smax, (int)xb[k]); smin = min(smin, (int)xb[k]); umax = max(umax, xb[k]); }
  smax = grp_max_i32(smax); smin = grp_min_i32(smin); umax = grp_max_u32(umax);
  // largest value: the signed maximum if it is not negative, else (all negative) the signed minimum; smallest
  // value: the unsigned maximum if it has the sign bit, else the signed minimum.  Selected under sign masks.
  const u32 mxb = sel_mask((u32)(smax >> 31), (u32)smin, (u32)smax);
  const u32 mnb = sel_mask((u32)((int)umax >> 31), umax, (u32)smin);
  const bool nonfinite = (smax >= 0x7f800000) || (umax >= 0xff800000u);
  const float mx = u2f(mxb), mn = u2f(mnb);
  const float d = __fsub_rn(mx, mn);
  const float r = __fmul_rn(0.5f, d);
  const float mu = __fadd_rn(mn, r);
  const bool dfinite = f2u(d) < 0x7f800000u;
  RowClass rc; rc.mu = mu; rc.m = 0; rc.type = 2;
  if (nonfinite || !dfinite) { rc.mu = 0.0f; return rc; }
  const double deb = (double)eb;
  const bool c1 = fabs((double)mx - (double)mu) <= deb;
  const bool c2 = fabs((double)mn - (double)mu) <= deb;
  if (r <= eb && c1 && c2) { rc.type = 0; return rc; }
  const u32 va = f2u(__fsub_rn(mx, mu)) & 0x7fffffffu, vb = f2u(__fsub_rn(mn, mu)) & 0x7fffffffu;
  const u32 vmaxb = max(va, vb);
  const int e_v = (int)max(vmaxb >> 23, 1u) - 127;
  const u32 amax = max(mxb & 0x7fffffffu, mnb & 0x7fffffffu);
  const int e_M = (int)max(amax >> 23, 1u) - 127;
  int m = e_v - e_eb; m = m < 0 ? 0 : (m > 23 ? 23 : m);
  // raw: bound below 4 ulp of the largest magnitude, 16 or more mantissa bits to keep, or a value in the top
  // binade (the rounded centred value plus the median could reach 2^128 and decode as Inf)
  if (e_eb < e_M - 21 || m >= 16 || e_M >= 127) { rc.mu = 0.0f; return rc; }
  rc.type = 1; rc.m = (u32)m;
  return rc;
}

// ---------------------------------------------------------------------------------------------
// Encoder, in the phases the persistent loop interleaves.
// ---------------------------------------------------------------------------------------------
struct EncRegs {       // what a lane keeps between sizing its elements and writing their bytes
  u32 t[kE];           // the coded words
  u32 lc;              // the lane's 32 bits of lead codes: an element emits nb - code bytes
  u32 cc;              // lean path: the bytes each element emits, 2 bits each
  u32 nb;              // bytes per element of the lane's block (2, 3, or 4 for raw)
  int nv;              // elements of the lane that exist
  u32 len, incl;       // bytes emitted by the lane, inclusive scan of it over the block
  u32 nlead;
  bool active;
  bool anyraw;         // wave-uniform: some block of this wavefront is raw
};

// Sum of the sixteen 2-bit fields of x.
__device__ __forceinline__ u32 sum_fields2(u32 x) {
  x = (x & 0x33333333u) + ((x >> 2) & 0x33333333u);
  x = (x + (x >> 4)) & 0x0f0f0f0fu;
  return __builtin_amdgcn_sad_u8(x, 0u, 0u);
}

// Transform and code the lane's elements.  MAYRAW = false is the lean path for wavefronts without a raw
// block: 2 or 3 bytes per element, so the byte counts fit 2-bit fields (r.cc) like the lead codes.
template <bool FULL, bool MAYRAW>
__device__ __forceinline__ void enc_code(const u32 (&xb)[kE], int nv, const RowClass& rc, const GrpMasks& gm, EncRegs& r) {
  const bool raw = MAYRAW && rc.type == 2;
  const u32 m = rc.m;
  const u32 nb = raw ? 4u : (m >= 8 ? 3u : 2u);
  const u32 half = raw ? 0u : (1u << (22 - m));
  const u32 sh = raw ? 0u : (23 - m);
  const float mu = rc.mu;
  const u32 rawm = MAYRAW ? lane_mask(raw) : 0u;
#pragma unroll
  for (int k = 0; k < kE; ++k) {
    const float v = __fsub_rn(u2f(xb[k]), mu);
    const u32 src = MAYRAW ? sel_mask(rawm, xb[k], f2u(v)) : f2u(v);
    r.t[k] = (src + half) >> sh;
  }
  u32 prev = grp_left(r.t[kE - 1], gm);         // last element of the lane to the left, 0 at the block start
  u32 lc = 0;
  if (MAYRAW) {
    const u32 s1 = raw ? 0u : 1u;
    const u32 kk = raw ? 39u : 38u;
    u32 len = 0;
#pragma unroll
    for (int k = 0; k < kE; ++k) {
      const u32 d = r.t[k] ^ prev;
      const u32 y = (d << s1) | 1u;
      u32 c = (kk - (u32)__builtin_clz(y)) >> 3;             // bytes that differ from the predecessor
      u32 L = nb - c;
      if (!FULL && k >= nv) { c = 0; L = 0; }
      lc |= L << (2 * k);
      len += c;
      prev = r.t[k];
    }
    r.len = len; r.cc = 0;
  } else {
    // equal leading bytes = (8 nb - significant bits of the difference) / 8, from one count of leading zeros
    const u32 kz = 8u * nb - 31u;
#pragma unroll
    for (int k = 0; k < kE; ++k) {
      const u32 d = r.t[k] ^ prev;
      const u32 z = (u32)__builtin_clz((d << 1) | 1u);       // 31 - significant bits of d
      lc |= ((z + kz) >> 3) << (2 * k);
      prev = r.t[k];
    }
    u32 nbrep = nb * 0x55555555u;
    if (!FULL) {
      const u32 valid = nv >= kE ? ~0u : ((1u << (2 * nv)) - 1u);
      lc &= valid; nbrep &= valid;
    }
    r.cc = nbrep - lc;                                       // field by field: a lead code never exceeds nb
    r.len = sum_fields2(r.cc);
  }
  r.lc = lc; r.nb = nb; r.nv = nv;
}

// ---------------------------------------------------------------------------------------------
// Decoder.
// ---------------------------------------------------------------------------------------------
// What a block's lanes need to decode it.
struct BlockInfo { u32 rq, bs, boff; };

// Decodes the lane's 16 elements of its block into xo (bit patterns); bi.rq == 0 means a constant block
// (or one that does not exist).  Returns a block-uniform flag: the block body is malformed.
// All reads stay inside the stage (bi.boff + bi.bs is inside the payload, and a lane reads at most
// 8 lanes x 64 bytes past the lead codes).  MAYRAW = false is the lean path for wavefronts without a raw
// block: at most 3 bytes per element, so every mask is a 32-bit shift.
// KEEPMASK: what a lane remembers per element for the second pass is the mask of the bits it has decided so
// far (one OR per element, 16 more live registers of full width) instead of their count (a max per element and
// a shift in the second pass): faster where registers are plentiful (decompress), slower in the reduce step.
template <bool FULL, bool MAYRAW, bool KEEPMASK>
__device__ __forceinline__ u32 dec_rows_impl(int nv, int blen, const unsigned char* st, const BlockInfo& bi, float mu,
                                             const GrpMasks& gm, u32 (&xo)[kE]) {
  const int l8 = threadIdx.x & 7;
  const u32 rq = bi.rq;
  u32 rowbad = 0;
  if (rq == 0) {
#pragma unroll
    for (int k = 0; k < kE; ++k) xo[k] = f2u(mu);
  } else {
    const bool raw = MAYRAW && rq == 32;
    const u32 nb8 = raw ? 32u : (((rq + 7u) >> 3) << 3);
    const u32 sh = raw ? 0u : 32u - rq;
    const u32 boff = bi.boff, bs = bi.bs;
    const u32 nlead = FULL ? 32u : (u32)((blen + 3) >> 2);
    u32 lead = lds_load32_any(st, boff + 4u * (u32)l8);
    if (!FULL) lead &= nv >= kE ? ~0u : ((1u << (2 * nv)) - 1u);    // codes of elements that exist
    // a lead code of 3 with 2-byte elements is the one code that cannot occur
    if (nb8 == 16u && (lead & (lead >> 1) & 0x55555555u) != 0u) rowbad = 1;
    u32 t[kE], c8[kE]; u32 prev = 0, cmax = 0;                       // c8 / cmax: bit count, or mask if KEEPMASK
    if (!MAYRAW) {
      // Lean path: 2 or 3 bytes per element, so the bytes each element stores fit 2-bit fields like the
      // lead codes: cc = nb - lead, field by field (a code above nb has been flagged; the fields stay 0..3).
      const u32 nb = nb8 >> 3;
      u32 nbrep = nb * 0x55555555u;
      if (!FULL) nbrep &= nv >= kE ? ~0u : ((1u << (2 * nv)) - 1u);
      const u32 cc = nbrep - lead;
      const u32 len = sum_fields2(cc);
      const u32 incl = grp_scan_add(len, gm);
      if (l8 == kGrp - 1 && nlead + incl != bs) rowbad = 1;
      // a: the byte address just past the element's stored bytes, minus 4: the 4-byte word that ends there
      // holds the element's stored bytes last, i.e. in its top bytes; byte-swapped they are the low bytes, in
      // the right order, and whatever lies above them is masked away.  All 16 words are requested before the
      // first one is used: the addresses depend on the lead codes only.
      u32 a = boff + nlead - 4u + (incl - len);
      u32 wlo[kE], whi[kE], sel[kE];
#pragma unroll
      for (int k = 0; k < kE; ++k) {
        a += (cc >> (2 * k)) & 3u;
        const u32* q = (const u32*)(st + (a & ~3u));
        wlo[k] = q[0]; whi[k] = q[1]; sel[k] = a;
      }
#pragma unroll
      for (int k = 0; k < kE; ++k) {
        const u32 c = ((cc >> (2 * k)) & 3u) << 3;                    // bits this element stores
        const u32 be = bswap32(__builtin_amdgcn_alignbyte(whi[k], wlo[k], sel[k]));
        const u32 mask = ~(~0u << c);
        prev = (mask & be) | (~mask & prev);
        t[k] = prev;
        cmax = KEEPMASK ? (cmax | mask) : max(cmax, c);
        c8[k] = cmax;                                                 // bits already decided
      }
    } else {
    u32 len8 = 0;
#pragma unroll
    for (int k = 0; k < kE; ++k) {
      const u32 L = (lead >> (2 * k)) & 3u;
      u32 c = nb8 - 8u * L;                                         // bits this element stores
      if (!FULL && k >= nv) c = 0;
      len8 += c;
    }
    const u32 incl8 = grp_scan_add(len8, gm);
    if (l8 == kGrp - 1 && 8u * nlead + incl8 != 8u * bs) rowbad = 1;
    u32 q8 = 8u * (boff + nlead - 4u) + (incl8 - len8);
    u32 wlo[kE], whi[kE], sel[kE];
#pragma unroll
    for (int k = 0; k < kE; ++k) {
      const u32 L = (lead >> (2 * k)) & 3u;
      u32 c = nb8 - 8u * L;
      if (!FULL && k >= nv) c = 0;
      q8 += c;
      const u32 a = q8 >> 3;
      const u32* q = (const u32*)(st + (a & ~3u));
      wlo[k] = q[0]; whi[k] = q[1]; sel[k] = a;
    }
#pragma unroll
    for (int k = 0; k < kE; ++k) {
      const u32 L = (lead >> (2 * k)) & 3u;
      u32 c = nb8 - 8u * L;
      if (!FULL && k >= nv) c = 0;
      const u32 be = bswap32(__builtin_amdgcn_alignbyte(whi[k], wlo[k], sel[k]));
      const u32 mask = (u32)((1ull << c) - 1ull);
      prev = (mask & be) | (~mask & prev);
      t[k] = prev;
      cmax = KEEPMASK ? (cmax | mask) : max(cmax, c);
      c8[k] = cmax;                                                 // bits already decided
    }
    }
    // what the lane passes on: V = its last element, N = mask of the bits it decided itself.
    // Inclusive scan over the block of the composition "take my bits where I decided, else the left one's".
    u32 N = KEEPMASK ? cmax : (MAYRAW ? (u32)((1ull << cmax) - 1ull) : ~(~0u << cmax)), V = prev;
    {
      u32 Vp = dpp0<kRowShr1>(V) & gm.m1, Np = dpp0<kRowShr1>(N) & gm.m1; V |= Vp & ~N; N |= Np;
      Vp = dpp0<kRowShr2>(V) & gm.m2; Np = dpp0<kRowShr2>(N) & gm.m2; V |= Vp & ~N; N |= Np;
      Vp = dpp0<kRowShr4>(V) & gm.m4; Np = dpp0<kRowShr4>(N) & gm.m4; V |= Vp & ~N; N |= Np;
    }
    const u32 tin = grp_left(V, gm);                                // 0 at the block start
    const u32 rawm = MAYRAW ? lane_mask(raw) : 0u;
#pragma unroll
    for (int k = 0; k < kE; ++k) {
      const u32 own = KEEPMASK ? c8[k] : (MAYRAW ? (u32)((1ull << c8[k]) - 1ull) : ~(~0u << c8[k]));
      const u32 tt = (own & t[k]) | (~own & tin);
      xo[k] = MAYRAW ? sel_mask(rawm, tt, f2u(__fadd_rn(u2f(tt << sh), mu))) : f2u(__fadd_rn(u2f(tt << sh), mu));
    }
  }
  return grp_or_u32(rowbad);
}
template <bool FULL, bool KEEPMASK = false>
__device__ __forceinline__ u32 dec_rows(int nv, int blen, const unsigned char* st, const BlockInfo& bi, float mu,
                                        const GrpMasks& gm, u32 (&xo)[kE]) {
  if (__ballot(bi.rq == 32) != 0) return dec_rows_impl<FULL, true, KEEPMASK>(nv, blen, st, bi, mu, gm, xo);
  return dec_rows_impl<FULL, false, KEEPMASK>(nv, blen, st, bi, mu, gm, xo);
}

// ---------------------------------------------------------------------------------------------
// geometry, loads, stores
// ---------------------------------------------------------------------------------------------
// 4 x 4 transposition of 16-byte vectors inside every group of four lanes: on entry lane r of a quad holds
// its own 16 elements as vectors x[4j .. 4j+3]; on return x[4i .. 4i+3] is vector r of lane i of the quad.
// A wavefront memory instruction then touches, per quad, 64 contiguous bytes (the 16 elements of one lane)
// instead of four separate 16-byte pieces: whole 64-byte lines per instruction, which is what the memory
// system wants (16 bytes per lane at a 64-byte stride ran at two thirds of the speed).  Two butterfly
// stages of DPP moves and selects.  All four lanes of a quad must be active.
// One butterfly stage for a pair of vectors (lo, hi) between a lane and its partner (the lane CTRL away): the
// lanes with `first` set keep lo and hand over hi, the others keep hi and hand over lo, so one value per dword
// crosses (one DPP move); the three selections are bit operations under a lane mask.
template <int CTRL>
__device__ __forceinline__ void butterfly(u32 first, u32 (&lo)[4], u32 (&hi)[4]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const u32 send = sel_mask(first, hi[d], lo[d]);
    const u32 got = (u32)__builtin_amdgcn_update_dpp(0, (int)send, CTRL, 0xf, 0xf, true);
    const u32 nlo = sel_mask(first, lo[d], got), nhi = sel_mask(first, got, hi[d]);
    lo[d] = nlo; hi[d] = nhi;
  }
}

__device__ __forceinline__ void quad_transpose(u32 (&x)[kE]) {
  const u32 even = lane_mask((threadIdx.x & 1u) == 0), low2 = lane_mask((threadIdx.x & 2u) == 0);
  u32 v[4][4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int d = 0; d < 4; ++d) v[j][d] = x[4 * j + d];
  // stage 1, partner lane ^ 1: even lanes end up with (own 2m, partner's 2m), odd lanes with (partner's 2m+1, own 2m+1)
  butterfly<kQuadXor1>(even, v[0], v[1]);
  butterfly<kQuadXor1>(even, v[2], v[3]);
  // stage 2, partner lane ^ 2, on the vector pairs (b, 2 + b)
  butterfly<kQuadXor2>(low2, v[0], v[2]);
  butterfly<kQuadXor2>(low2, v[1], v[3]);
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int d = 0; d < 4; ++d) x[4 * j + d] = v[j][d];
}

// Writes the decoded elements of the lane's quad that fall into [lo, hi) to out[e - lo].  xt: the quad's
// elements after quad_transpose (vector i = elements qe0 + 16 i + 4 r .. + 3 for lane r of the quad, qe0 the
// quad's first element).  Elements at or past `hi` do not exist or are not wanted.
__device__ __forceinline__ void store_quad(float* out, const u32 (&xt)[kE], u64 qe0, u64 lo, u64 hi, bool aligned16) {
  const u32 r = threadIdx.x & 3u;
  if (aligned16 && qe0 >= lo && qe0 + 4 * kE <= hi) {
    // streaming stores: the output is not read again by this kernel, and keeping it out of the way of the
    // payload reads in L2 is worth a fifth of the kernel's time
    v4u* q = (v4u*)(out + (qe0 - lo)) + r;
#pragma unroll
    for (int i = 0; i < kE / 4; ++i) {
      v4u a; a.x = xt[4 * i]; a.y = xt[4 * i + 1]; a.z = xt[4 * i + 2]; a.w = xt[4 * i + 3];
      __builtin_nontemporal_store(a, q + 4 * i);
    }
  } else {
#pragma unroll
    for (int i = 0; i < kE / 4; ++i)
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const u64 e = qe0 + (u64)(16 * i + 4 * (int)r + d);
        if (e >= lo && e < hi) ((u32*)out)[e - lo] = xt[4 * i + d];
      }
  }
}

// {bytes, status} of the call for a caller that wants them in device memory (one thread, launched
// behind the work on the same stream).
__global__ void k_publish(Params P) {
  const u64 e = ld_dev(&P.ws->err);
  const bool mine = (e >> 8) == (u64)P.epoch;
  P.result[0] = P.no_total ? 0ull : ld_dev(&P.ws->total);
  P.result[1] = (u64)(mine ? -(long long)((e >> 4) & 0xfu) : 0ll);
}

// ---------------------------------------------------------------------------------------------
// compress
// ---------------------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------------------
// incoming streams: header checks and chunk offsets
// ---------------------------------------------------------------------------------------------
// Header checks shared by decompress and reduce (one thread).
__device__ __forceinline__ bool header_ok(const unsigned char* s, const Params& P) {
  const u32* h = (const u32*)s;
  if (h[0] != 0x31585343u) return false;
  if (h[1] != ((u32)kBlock | ((u32)kChunk << 16))) return false;
  const u64 n = (u64)h[2] | ((u64)h[3] << 32);
  if (n != P.n) return false;
  const u32 eb = h[4];
  if (eb == 0 || eb >= 0x7f800000u) return false;       // must be finite and > 0
  if (h[5] != P.nchunks) return false;
  const u64 total = (u64)h[6] | ((u64)h[7] << 32);
  const u64 front = kHeader + 4ull * P.nchunks;
  if (!P.open_stream && (total < front || total > P.in_bytes)) return false;
  return true;
}

// n == 0: only the header.  With an incoming stream (reduce step) that one must be a bare header too.
__global__ void k_empty_stream(Params P) {
  if (threadIdx.x == 0) {
    bool ok = true;
    if (P.cin) {
      const u32* hc = (const u32*)P.cin;
      ok = header_ok((const unsigned char*)P.cin, P) && hc[6] == kHeader && hc[7] == 0;
    }
    u32* h = (u32*)P.out;
    h[0] = 0x31585343u; h[1] = (u32)kBlock | ((u32)kChunk << 16);
    h[2] = 0; h[3] = 0; h[4] = P.eb_bits; h[5] = 0; h[6] = kHeader; h[7] = 0;
    st_dev(&P.ws->total, (u64)kHeader);
    if (!ok) raise_error(P, CCOLL_ECORRUPT, 1);
  }
}

// A stream that is compressed piece by piece (Sec. III-E.2): the header goes first, with a total of 0 that the last
// piece replaces, so that a receiver can check what has arrived of the stream before all of it exists.
__global__ void k_begin_stream(Params P) {
  if (threadIdx.x == 0) {
    u32* h = (u32*)P.out;
    h[0] = 0x31585343u; h[1] = (u32)kBlock | ((u32)kChunk << 16);
    h[2] = (u32)P.n; h[3] = (u32)(P.n >> 32); h[4] = P.eb_bits; h[5] = P.nchunks; h[6] = 0; h[7] = 0;
    st_dev(&P.ws->total, (u64)kHeader);
  }
}

// What a transport would send of a stream that is still being written: the front index entries of chunks
// [from.chunks, upto.chunks), the payload bytes [from.bytes, upto.bytes) and, once the last chunk is among them,
// the header; copied to the same offsets of dst.  from / upto: {chunks coded, stream bytes final} as a compress
// call leaves them; from == null: the start of the stream.
__global__ void __launch_bounds__(256) k_forward(unsigned char* dst, const unsigned char* src, u32 nchunks,
                                                 const unsigned long long* from, const unsigned long long* upto) {
  const u64 front = kHeader + 4ull * nchunks;
  const u64 c_lo = from ? from[0] : 0ull, b_lo = from ? from[1] : front;
  const u64 c_hi = upto[0], b_hi = upto[1];
  const u64 tid = (u64)blockIdx.x * blockDim.x + threadIdx.x, nth = (u64)gridDim.x * blockDim.x;
  if (c_hi < c_lo || b_hi < b_lo || b_lo < front || c_hi > nchunks) return;      // not a pair of progress words of one stream
  const u32* s32 = (const u32*)src; u32* d32 = (u32*)dst;
  for (u64 i = kHeader / 4 + c_lo + tid; i < kHeader / 4 + c_hi; i += nth) d32[i] = s32[i];
  // payload: whole 16-byte vectors where source and destination (same offset in both) are aligned, words at the ends
  const u64 w_lo = b_lo / 4, w_hi = b_hi / 4;
  const bool al = ((((uintptr_t)src) | ((uintptr_t)dst)) & 15u) == 0;
  u64 v_lo = (w_lo + 3) & ~3ull, v_hi = w_hi & ~3ull;
  if (!al || v_lo > v_hi) { v_lo = w_hi; v_hi = w_hi; }
  for (u64 i = w_lo + tid; i < (v_lo < w_hi ? v_lo : w_hi); i += nth) d32[i] = s32[i];
  for (u64 i = v_lo / 4 + tid; i < v_hi / 4; i += nth) ((uint4*)dst)[i] = ((const uint4*)src)[i];
  for (u64 i = v_hi + tid; i < w_hi; i += nth) d32[i] = s32[i];
  if (c_hi == nchunks && tid < kHeader / 4) d32[tid] = s32[tid];
  else if (c_lo == 0 && tid < kHeader / 4) d32[tid] = s32[tid];                    // the open header travels with the first piece
}

// n == 0: the stream must be a bare header.
__global__ void k_check_empty(Params P) {
  if (threadIdx.x == 0) {
    const u32* h = (const u32*)P.in;
    const bool ok = header_ok((const unsigned char*)P.in, P) && h[6] == kHeader && h[7] == 0;
    if (!ok) raise_error(P, CCOLL_ECORRUPT, 1);
  }
}

// Incoming stream: header and front index checked once, and the chunk-start pointers of
// Sec. III-E.2 (exclusive prefix of the chunk sizes) written to P.offs.  One workgroup per tile of 8192
// entries (the index is 4 bytes per 20 KB of data): it first adds up all entries in front of its tile
// straight from L2, then scans its tile, each thread fetching 8 consecutive entries as two 16-byte loads;
// the prefixes go through LDS so that the 64-bit offsets leave as coalesced stores.
constexpr u32 kScanTile = 8192;
__global__ void __launch_bounds__(1024) k_index_scan(Params P) {
  __shared__ u64 wtot[16];
  __shared__ u64 wbase[16];
  __shared__ u32 rel[1024 * 9];                        // 8 per thread, padded against bank conflicts
  const unsigned char* s = (const unsigned char*)(P.cin ? P.cin : P.in);
  const u32* ci = (const u32*)(s + kHeader);
  const u32 tid = threadIdx.x, lane = tid & 63u, wv = tid >> 6;
  const u32 n = P.scan_chunks, nall = P.nchunks;       // entries walked (those that have arrived), entries of the stream
  const u32 nlast = (u32)((P.n - (u64)(nall ? nall - 1 : 0) * kChunk + kBlock - 1) / kBlock);   // blocks of the last chunk
  const bool al16 = (((uintptr_t)ci) & 15u) == 0;
  const u32 tile = blockIdx.x * kScanTile;
  u32 why = 0;
  // the tile's own entries are requested first: they come back while the entries in front are added up
  const u32 a = tile + tid * 8u;
  u32 v[8];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const u32 c = a + 4u * q;
    if (al16 && c + 4u <= n) {
      const uint4 x = *(const uint4*)(ci + c);
      v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) v[4 * q + j] = (c + j < n) ? ci[c + j] : 0u;
    }
  }
  // sum of the entries in front of the tile (entries are validated by the workgroup that owns them; here
  // they are only kept from overflowing the sum)
  u64 before = 0;
  for (u32 c0 = 0; c0 < tile; c0 += 8u * 4096u) {          // 8 loads in flight per thread: one round trip per 32,768 entries
    uint4 x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u32 c = c0 + 4096u * (u32)i + 4u * tid;
      x[i] = make_uint4(0, 0, 0, 0);
      if (c < tile) {
        if (al16) x[i] = *(const uint4*)(ci + c);
        else { x[i].x = ci[c]; x[i].y = ci[c + 1]; x[i].z = ci[c + 2]; x[i].w = ci[c + 3]; }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      before += x[i].x <= kMaxPayload ? x[i].x : 0u; before += x[i].y <= kMaxPayload ? x[i].y : 0u;
      before += x[i].z <= kMaxPayload ? x[i].z : 0u; before += x[i].w <= kMaxPayload ? x[i].w : 0u;
    }
  }
  before = wave_sum_u64(before);
  if (lane == 0) wbase[wv] = before;
  u32 local = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const u32 c = a + i;
    if (c < n) {
      const u32 nbc = (c + 1 == nall) ? nlast : (u32)kBpc;
      if ((v[i] & 3u) || v[i] < 8u + 4u * nbc || v[i] > kMaxPayload) { why = 2; v[i] = 0; }
    }
    rel[tid * 9 + i] = local;                         // prefix inside the thread; valid sizes are < 2^15
    local += v[i];
  }
  // exclusive scan of the per-thread sums over the workgroup
  u32 incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) { const u32 up = __shfl_up(incl, o); if (lane >= (u32)o) incl += up; }
  if (lane == 63) wtot[wv] = incl;
  __syncthreads();
  u32 base = 0;
  for (u32 i = 0; i < wv; ++i) base += (u32)wtot[i];
  u64 carry = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) carry += wbase[i];
  const u32 excl = base + incl - local;               // inside the tile: < 8192 * 22048 < 2^28
#pragma unroll
  for (int i = 0; i < 8; ++i) rel[tid * 9 + i] += excl;
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const u32 e = j * 1024u + tid;
    if (tile + e < n) P.offs[tile + e] = carry + rel[(e >> 3) * 9 + (e & 7u)];
  }
  if (tid == 1023 && tile + kScanTile >= n) {         // the workgroup of the last tile: the sizes must add up to the header's total
    const u64 front = kHeader + 4ull * nall;
    const u64 total = (u64)((const u32*)s)[6] | ((u64)((const u32*)s)[7] << 32);
    const u64 sum = front + carry + excl + local;
    if (!why && (P.open_stream ? sum > P.in_bytes : sum != total)) why = 5;
  }
  if (tid == 0 && blockIdx.x == 0 && !header_ok(s, P)) why = 1;
  if (why) raise_error(P, CCOLL_ECORRUPT, why);
}

// ---------------------------------------------------------------------------------------------
// decompress
// ---------------------------------------------------------------------------------------------
// Where an incoming chunk's payload is and whether it may be read at all (k_index_scan reports what is
// wrong with the index; this only keeps every read inside the stream).
struct InChunk { const unsigned char* src; u32 size; bool ok; };
// vzero: a zero the compiler cannot see through, so that these loads go through the vector memory path:
// scalar loads share their counter with LDS reads, and a look-ahead load would stall the decode.
__device__ __forceinline__ InChunk locate_chunk(const unsigned char* s, u32 c, const Params& P, u32 vzero) {
  const u64 front = kHeader + 4ull * P.nchunks;
  const u64 ofs = P.offs[c + vzero];
  const u32 sz = ((const u32*)(s + kHeader))[c + vzero];
  InChunk r;
  r.ok = !(sz & 3u) && sz <= kMaxPayload && !(ofs & 3ull) && ofs <= P.in_bytes && front + ofs + sz <= P.in_bytes;
  r.size = r.ok ? sz : 0u;
  r.src = s + front + (r.ok ? ofs : 0ull);
  return r;
}


// ---- one wavefront per chunk ---------------------------------------------------------------------
// A wavefront decodes a chunk by itself, 8 blocks (1024 elements, 16 per lane) at a time, out of a window
// of the payload that it keeps in its own piece of LDS: no barrier anywhere, every SIMD gets the same
// load, and the memory round trips of one wavefront (chunk start, payload) hide behind the decoding of
// the others on its SIMD.
constexpr u32 kMaxBody = 32 + 4 * kBlock;            // 544: lead codes + 4 bytes per element
constexpr u32 kWinPad = 16;                          // the decoder reads up to 3 bytes in front of a body
constexpr u32 kWin = 9632;                           // payload bytes a wavefront holds at a time (>= 8 * 544 + 3)
constexpr u32 kRegion = kWinPad + kWin + 576;        // + what a malformed body may be read past its start
constexpr int kDecWaves = 4;                         // wavefronts (= chunks) per workgroup
static_assert(kRegion % 16 == 0 && kWin % 16 == 0 && kWin >= 8 * kMaxBody + 3, "window geometry");

// Payload bytes [from, from + len) -> st[0, len): len and from are multiples of 4, st is 16-byte aligned.
// All loads are issued before the first LDS write so that they share one round trip.
__device__ __forceinline__ void fetch_window(const unsigned char* src, u32 from, u32 len, unsigned char* st) {
  const u32 lane = threadIdx.x & 63u;
  const unsigned char* g = src + from;
  const u32 n16 = len >> 4;
  constexpr int kBatch = 4;                              // 4 KB per round trip
  for (u32 j0 = 0; j0 < n16; j0 += 64u * kBatch) {
    uint4 v[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const u32 j = j0 + lane + 64u * (u32)i;
      v[i] = make_uint4(0, 0, 0, 0);
      if (j < n16) __builtin_memcpy(&v[i], g + 16u * j, 16);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const u32 j = j0 + lane + 64u * (u32)i;
      if (j < n16) *(uint4*)(st + 16u * j) = v[i];
    }
  }
  const u32 rest = (len >> 2) & 3u;
  if (lane < rest) ((u32*)(st + 16u * n16))[lane] = ((const u32*)(g + 16u * n16))[lane];
}

// Per-block metadata of a chunk, lane j = block j (lanes >= nbc hold zeros).
struct ChunkMeta {
  u32 rq, bs, boff, end; float mu;
  u32 packed;                                          // rq | bs << 6 | boff << 16: one word to hand to the block's lanes
};
// What lane `b` holds of a chunk's metadata, for the lanes of block b: two cross-lane reads (ds_bpermute is the most
// expensive instruction of the decoder: 24 cycles per wavefront) instead of four.
__device__ __forceinline__ void block_info(const ChunkMeta& m, int b, u32 wbase, BlockInfo& bi, float& mu) {
  const u32 w = (u32)__shfl((int)m.packed, b);
  bi.rq = w & 63u; bi.bs = (w >> 6) & 1023u; bi.boff = (w >> 16) - wbase;
  mu = __shfl(m.mu, b);
}

// Parses the metadata at the start of a payload (in `st`).  Returns false (wave-uniform) if malformed.
__device__ __forceinline__ bool parse_meta(const unsigned char* st, u32 payload, int nbc, ChunkMeta& m) {
  const u32 lane = threadIdx.x & 63u;
  bool bad = payload < 8u + 4u * (u32)nbc;
  const u64 bitmap = bad ? 0ull : ((u64)((const u32*)st)[0] | ((u64)((const u32*)st)[1] << 32));
  if (nbc < 64 && (bitmap >> nbc) != 0) bad = true;
  const u32 k = (u32)__popcll(bitmap);
  const u32 meta = pad4(8u + 4u * (u32)nbc + 3u * k);
  if (meta > payload) bad = true;
  const bool in = (int)lane < nbc && !bad;
  const bool nonconst = in && ((bitmap >> lane) & 1ull);
  const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(bitmap >> 32), __builtin_amdgcn_mbcnt_lo((u32)bitmap, 0u));   // set bits below the lane's
  u32 bs = 0, rq = 0;
  if (nonconst) {
    bs = lds_load16(st + 8 + 4 * nbc + 2 * rank);
    rq = st[8 + 4 * nbc + 2 * k + rank];
    if (!((rq >= 9 && rq <= 24) || rq == 32) || bs > kMaxBody) bad = true;
  }
  m.mu = in ? ((const float*)(st + 8))[lane] : 0.0f;
  if (__ballot(bad) != 0) { bs = 0; bad = true; }        // keep the sums below small whatever the stream says
  const u32 sc = wave_scan_add(bs);
  const u32 bodies = (u32)__builtin_amdgcn_readlane((int)sc, 63);
  if (pad4(meta + bodies) != payload) bad = true;
  m.rq = bad ? 0u : rq; m.bs = bs; m.end = meta + sc; m.boff = meta + sc - bs;
  m.packed = m.rq | (m.bs << 6) | (m.boff << 16);      // rq <= 32, bs <= 544, boff <= 22048
  return !bad;
}

template <bool FULL>
__device__ __forceinline__ void decompress_chunk(u32 c, const Params& P, const unsigned char* src, u32 payload,
                                                 unsigned char* st) {
  const u32 lane = threadIdx.x & 63u, l8 = lane & 7u;
  const u64 cbeg = (u64)c * kChunk;
  const int clen = FULL ? kChunk : (int)(P.n - cbeg);
  const int nbc = FULL ? kBpc : (clen + kBlock - 1) / kBlock;
  const u64 lo = P.first, hi = P.first + P.count;
  const GrpMasks gm = grp_masks();
  unsigned char* w = st + kWinPad;
  u32 wbase = 0, wend = payload < kWin ? payload : kWin;
  fetch_window(src, 0, wend, w);
  ChunkMeta m;
  if (!parse_meta(w, payload, nbc, m)) { if (lane == 0) raise_error(P, CCOLL_ECORRUPT, 6); return; }
  u32 anybad = 0;
#pragma unroll 1
  for (int u = 0; u < kUnits; ++u) {
    if (!FULL && 8 * u >= nbc) break;
    const u64 ubeg = cbeg + (u64)u * kUnit;
    if (ubeg >= hi || ubeg + kUnit <= lo) continue;                    // nothing of it is wanted
    const int last = FULL ? 8 * u + 7 : (8 * u + 7 < nbc ? 8 * u + 7 : nbc - 1);
    const u32 ustart = (u32)__builtin_amdgcn_readlane((int)m.boff, 8 * u);
    const u32 uend = (u32)__builtin_amdgcn_readlane((int)m.end, last);
    if (ustart < wbase || uend > wend) {                               // slide the window to this unit's bodies
      wbase = ustart & ~3u;
      const u32 len = payload - wbase < kWin ? payload - wbase : kWin;
      wend = wbase + len;
      fetch_window(src, wbase, len, w);
    }
    const int b = 8 * u + (int)(lane >> 3);
    BlockInfo bi; float mu;
    block_info(m, b, wbase, bi, mu);
    int blen = kBlock, nv = kE;
    if (!FULL) {
      blen = clen - b * kBlock; blen = blen < 0 ? 0 : (blen > kBlock ? kBlock : blen);
      nv = blen - (int)l8 * kE; nv = nv < 0 ? 0 : (nv > kE ? kE : nv);
      if (blen == 0) bi.rq = 0;
    }
    u32 xo[kE];
    const u32 rowbad = dec_rows<FULL, true>(nv, blen, w, bi, mu, gm, xo);
    anybad |= rowbad;
    quad_transpose(xo);
    const u64 vend = P.n < hi ? P.n : hi;                              // elements past the end of the data do not exist
    if (!rowbad) store_quad((float*)P.out, xo, ubeg + (u64)(lane & ~3u) * kE, lo, vend, P.aligned16 != 0);
  }
  if (__ballot(anybad != 0) != 0 && lane == 0) raise_error(P, CCOLL_ECORRUPT, 7);
}

// Four independent wavefronts per workgroup, one chunk each; the chunk starts come from k_index_scan.
__global__ void __launch_bounds__(64 * kDecWaves) __attribute__((amdgpu_waves_per_eu(4, 4))) k_decompress(Params P) {
  __shared__ __align__(16) unsigned char lds[kDecWaves][kRegion];
  const unsigned char* s = (const unsigned char*)P.in;
  const u32 wv = threadIdx.x >> 6;
  const u32 nfull = (u32)(P.n / kChunk);
  const u32 c = P.c0 + blockIdx.x * kDecWaves + wv;
  if (c >= P.c1) return;
  if (P.idx_epoch && ld_dev(&P.ws->idx_bad) == (u64)P.idx_epoch) {     // the kept offsets come from a stream that failed its checks
    if ((threadIdx.x & 63u) == 0) raise_error(P, CCOLL_ECORRUPT, 2);
    return;
  }
  const InChunk cur = locate_chunk(s, c, P, 0u);
  if (!cur.ok) { if ((threadIdx.x & 63u) == 0) raise_error(P, CCOLL_ECORRUPT, 4); return; }
  if (c < nfull) decompress_chunk<true>(c, P, cur.src, cur.size, lds[wv]);
  else decompress_chunk<false>(c, P, cur.src, cur.size, lds[wv]);
}

// Many ranges of one stream in one launch (the receivers' parts of a scattered or broadcast stream, Sec. IV-C):
// a workgroup looks up which range it works for in a small table that travels with the kernel arguments.
constexpr int kMaxRanges = CCOLL_MAX_RANGES_PER_LAUNCH;
struct RangeTable {
  u64 first[kMaxRanges], count[kMaxRanges];
  float* out[kMaxRanges];
  u32 wg_end[kMaxRanges];                            // workgroups of ranges 0..r, running total
  u32 nranges;
};
__global__ void __launch_bounds__(64 * kDecWaves) __attribute__((amdgpu_waves_per_eu(4, 4))) k_decompress_ranges(Params P, RangeTable T) {
  __shared__ __align__(16) unsigned char lds[kDecWaves][kRegion];
  const unsigned char* s = (const unsigned char*)P.in;
  const u32 wv = threadIdx.x >> 6;
  u32 lo = 0, hi = T.nranges - 1u;                   // first range whose running total exceeds the workgroup's number
  while (lo < hi) { const u32 mid = (lo + hi) >> 1; if (blockIdx.x >= T.wg_end[mid]) lo = mid + 1u; else hi = mid; }
  const u32 r = lo, wg0 = r ? T.wg_end[r - 1u] : 0u;
  Params Q = P;
  Q.first = T.first[r]; Q.count = T.count[r]; Q.out = T.out[r];
  Q.aligned16 = (((uintptr_t)T.out[r]) & 15u) == 0;
  const u32 c1 = (u32)((Q.first + Q.count + kChunk - 1) / kChunk);
  const u32 c = (u32)(Q.first / kChunk) + (blockIdx.x - wg0) * kDecWaves + wv;
  if (c >= c1) return;
  const InChunk cur = locate_chunk(s, c, Q, 0u);
  if (!cur.ok) { if ((threadIdx.x & 63u) == 0) raise_error(Q, CCOLL_ECORRUPT, 4); return; }
  if (c < (u32)(Q.n / kChunk)) decompress_chunk<true>(c, Q, cur.src, cur.size, lds[wv]);
  else decompress_chunk<false>(c, Q, cur.src, cur.size, lds[wv]);
}

// ---------------------------------------------------------------------------------------------
// compress and reduce step: one wavefront per chunk
// ---------------------------------------------------------------------------------------------
// A wavefront codes a chunk by itself, 8 blocks (1024 elements, 16 per lane) at a time, and assembles the
// payload in its own piece of LDS; no barrier inside a chunk.  The wavefronts of a workgroup take
// consecutive chunks (a "group"): groups are handed out in order by a ticket counter and their sizes go
// through the look-back scan as one entry, so a scan wait only ever concerns groups that are already
// running and nothing depends on which workgroups are resident together.
// The reduce step (Sec. III-A.2, Eq. 2) is the same kernel with another source of elements: the local
// floats plus the incoming chunk decoded out of a sliding window, so the sums never leave the registers.
constexpr u32 kMetaMax = 8 + 4 * kBpc + 3 * kBpc;    // 288
template <u32 CAP>
struct __align__(16) EncWaveLds {
  u32 meta[kMetaMax / 4];                            // bitmap, mu[], then bsize[], reqlen[]
  unsigned char body[CAP + 16];                      // block bodies, back to back
  u32 tmp[kBpc];                                     // body bytes | reqlen << 16 per block
};

// The lane's 16 floats of unit u of chunk c (bit patterns).  Slots past the end of a partial block repeat
// the block's first element; lanes without a block get zeros.
template <bool FULL>
__device__ __forceinline__ void load_unit(const float* base, u64 n, u32 c, int u, bool aligned16, u32 (&xb)[kE], int& nv, int& blen) {
  const u32 lane = threadIdx.x & 63u;
  const u64 e0 = (u64)c * kChunk + (u64)u * kUnit + (u64)lane * kE;
  if (FULL) {
    nv = kE; blen = kBlock;
    if (aligned16) {
      const uint4* q = (const uint4*)(base + e0);
#pragma unroll
      for (int i = 0; i < kE / 4; ++i) {
        const uint4 a = q[i];
        xb[4 * i] = a.x; xb[4 * i + 1] = a.y; xb[4 * i + 2] = a.z; xb[4 * i + 3] = a.w;
      }
    } else {
      const u32* p = (const u32*)base + e0;
#pragma unroll
      for (int k = 0; k < kE; ++k) xb[k] = p[k];
    }
  } else {
    const u64 blk0 = e0 - (u64)(lane & 7u) * kE;
    long long bl = (long long)n - (long long)blk0; bl = bl < 0 ? 0 : (bl > kBlock ? kBlock : bl);
    blen = (int)bl;
    int v = blen - (int)(lane & 7u) * kE; nv = v < 0 ? 0 : (v > kE ? kE : v);
    const u32* p = (const u32*)base;
    const u32 fill = blen > 0 ? p[blk0] : 0u;
#pragma unroll
    for (int k = 0; k < kE; ++k) xb[k] = k < nv ? p[e0 + k] : fill;
  }
}

// Source of the elements to code.  load() starts the memory reads of a unit (it may run one unit ahead),
// finish() turns what was read into the values to code.
struct SrcPlain {                                     // compress: the floats themselves
  static constexpr bool kPrefetch = true;             // a unit's floats are requested while the one before is coded
  const float* in; bool al;
  __device__ __forceinline__ void begin_chunk(u32, const Params&, unsigned char*) {}
  template <bool FULL>
  __device__ __forceinline__ void load(const Params& P, u32 c, int u, u32 (&xb)[kE], int& nv, int& blen) const {
    load_unit<FULL>(in, P.n, c, u, al, xb, nv, blen);
  }
  __device__ __forceinline__ bool needs_room(const Params&, u32, int, u32) { return false; }
  __device__ __forceinline__ void fetch(const Params&, u32, int, u32) {}
  template <bool FULL>
  __device__ __forceinline__ void finish(const Params&, u32, int, u32 (&)[kE], int, int, const GrpMasks&) {}
  __device__ __forceinline__ void make_room(u32) {}
  __device__ __forceinline__ void end_chunk() {}
};

// The reduce step keeps its window of the incoming payload inside the LDS stage it is coding into: the coded
// bodies grow from the front of the stage, the window sits at its end and holds the bodies of the units that
// are still to be decoded.  (A window of its own next to two stages per wavefront does not fit a compute unit's
// LDS at three wavefronts per SIMD.)  Where the coded bodies reach the window, its front is given up (zeroed:
// bodies are ORed into zeros); as a rule that front has been decoded by then.  If bodies that are still needed
// are lost that way, or did not fit in the first place, they are fetched again behind the coded bodies.
template <int OP, u32 CAP>
struct SrcReduce {                                    // reduce step: local floats (+, max, min) the incoming chunk, decoded
  static constexpr bool kPrefetch = false;            // registers are short: the decoder needs them
  static constexpr u32 kEnd = CAP + 16u;              // size of a stage's body area
  const float* local; bool al;
  const unsigned char* s;                             // incoming stream
  unsigned char* stage;                               // body area of the stage being coded into (16-byte aligned)
  const unsigned char* src; u32 payload; bool good;
  u32 wbase, wlen, wpos;                              // payload bytes [wbase, wbase + wlen) are at stage[wpos ...); wlen = 0: no window
  ChunkMeta m;
  // bytes between the coded bodies (the writer touches up to 16 bytes past its last body) and the end of the stage
  static __device__ __forceinline__ u32 room_behind(u32 fill) {
    const u32 used = ((fill + 31u) & ~15u) + 16u;
    return used < kEnd ? kEnd - used : 0u;
  }
  __device__ __forceinline__ void zero_window() {
    const u32 lane = threadIdx.x & 63u;
    for (u32 j = (wpos >> 4) + lane; j < kEnd / 16u; j += 64u) *(uint4*)(stage + 16u * j) = make_uint4(0, 0, 0, 0);
    wlen = 0;
  }
  // Window <- payload bytes from `from` on, as many as fit between the coded bodies (`fill` bytes) and the end.
  __device__ __forceinline__ void fetch_from(u32 from, u32 fill) {
    if (wlen) zero_window();
    const u32 room = room_behind(fill);
    u32 len = payload - from; len = len < room ? len : room;
    wpos = kEnd - ((len + 15u) & ~15u);
    fetch_window(src, from, len, stage + wpos);
    wbase = from; wlen = len;
  }
  __device__ __forceinline__ void begin_chunk(u32 c, const Params& P, unsigned char* stage_body) {
    const u32 lane = threadIdx.x & 63u;
    stage = stage_body;
    const InChunk cur = locate_chunk(s, c, P, 0u);
    good = cur.ok; src = cur.src; payload = cur.size; wbase = 0; wlen = 0; wpos = kEnd;
    m.rq = 0; m.bs = 0; m.boff = 0; m.end = 0; m.mu = 0.0f; m.packed = 0;
    if (!good) { if (lane == 0) raise_error(P, CCOLL_ECORRUPT, 4); return; }
    fetch_from(0, 0);
    const u64 cbeg = (u64)c * kChunk;
    const int nbc = P.n - cbeg >= (u64)kChunk ? kBpc : (int)((P.n - cbeg + kBlock - 1) / kBlock);
    good = parse_meta(stage + wpos, payload, nbc, m);
    if (!good && lane == 0) raise_error(P, CCOLL_ECORRUPT, 6);
  }
  template <bool FULL>
  __device__ __forceinline__ void load(const Params& P, u32 c, int u, u32 (&xb)[kE], int& nv, int& blen) const {
    load_unit<FULL>(KARGP(const float*, local), FULL ? 0ull : KARG64(n), c, u, al, xb, nv, blen);
  }
  // bodies of unit u of the incoming chunk: payload bytes [ustart, uend)
  __device__ __forceinline__ void unit_span(const Params& P, u32 c, int u, u32& ustart, u32& uend) const {
    const u64 left = P.n - (u64)c * kChunk;
    const int nbc = left >= (u64)kChunk ? kBpc : (int)((left + kBlock - 1) / kBlock);
    const int last = 8 * u + 7 < nbc ? 8 * u + 7 : nbc - 1;
    ustart = (u32)__builtin_amdgcn_readlane((int)m.boff, 8 * u);
    uend = (u32)__builtin_amdgcn_readlane((int)m.end, last);
  }
  // True: unit u is not in the window and there is no room for its bodies behind the `fill` coded bytes: the
  // caller moves the coded bytes on to the spill slot first.
  __device__ __forceinline__ bool needs_room(const Params& P, u32 c, int u, u32 fill) {
    if (!good) return false;
    u32 ustart, uend; unit_span(P, c, u, ustart, uend);
    if (ustart >= wbase && uend <= wbase + wlen) return false;
    return uend - (ustart & ~3u) > room_behind(fill);
  }
  // Brings unit u's bodies into the window if they are not there.
  __device__ __forceinline__ void fetch(const Params& P, u32 c, int u, u32 fill) {
    if (!good) return;
    u32 ustart, uend; unit_span(P, c, u, ustart, uend);
    if (ustart >= wbase && uend <= wbase + wlen) return;
    fetch_from(ustart & ~3u, fill);
  }
  // The coder is about to write up to byte `upto` of the stage: the front of the window that is in its way is
  // given up.  As a rule that front holds the metadata and the bodies of units that have been decoded already,
  // and the rest of the window stays in use.
  __device__ __forceinline__ void make_room(u32 upto) {
    if (wlen && upto + 16u > wpos) {
      const u32 lane = threadIdx.x & 63u;
      u32 z = (upto + 31u) & ~15u; z = z < kEnd ? z : kEnd;
      for (u32 j = (wpos >> 4) + lane; j < (z >> 4); j += 64u) *(uint4*)(stage + 16u * j) = make_uint4(0, 0, 0, 0);
      const u32 d = z - wpos;
      if (d >= wlen) wlen = 0;
      else { wbase += d; wlen -= d; wpos = z; }
    }
  }
  __device__ __forceinline__ void end_chunk() { if (wlen) zero_window(); }
  // xb: local floats in, sums out (Eq. 2: one float32 round-to-nearest add per element).  If the incoming
  // chunk cannot be read, 0 stands in for it so that the outgoing stream is still well formed; the error
  // has been raised.
  template <bool FULL>
  __device__ __forceinline__ void finish(const Params& P, u32 c, int u, u32 (&xb)[kE], int nv, int blen, const GrpMasks& gm) {
    const u32 lane = threadIdx.x & 63u;
    const int b = 8 * u + (int)(lane >> 3);
    BlockInfo bi; bi.rq = 0; bi.bs = 0; bi.boff = 0;
    float mu = 0.0f;
    const unsigned char* win = stage + wpos;
    if (good) {
      block_info(m, b, wbase, bi, mu);
      if (!FULL && blen == 0) bi.rq = 0;
    }
    u32 xo[kE];
    const u32 rowbad = dec_rows<FULL>(nv, blen, win, bi, mu, gm, xo);
    if (__ballot(rowbad != 0) != 0 && lane == 0) raise_error(P, CCOLL_ECORRUPT, 7);
    const bool use = good && !rowbad;
    if (OP == CCOLL_OP_SUM) {
      if (__ballot(!use) == 0) {
#pragma unroll
        for (int k = 0; k < kE; ++k) xb[k] = f2u(__fadd_rn(u2f(xb[k]), u2f(xo[k])));
      } else {
        const u32 um = lane_mask(use);
#pragma unroll
        for (int k = 0; k < kE; ++k) xb[k] = f2u(__fadd_rn(u2f(xb[k]), u2f(xo[k] & um)));
      }
    } else if (use) {
      // Max / Min (Sec. III-B) under the total order of the bit patterns: key = bits with the sign bit set for
      // non-negative values and all bits flipped for negative ones; the larger / smaller key wins.
      const bool take_max = OP == CCOLL_OP_MAX;
#pragma unroll
      for (int k = 0; k < kE; ++k) {
        const u32 a = xb[k], b = xo[k];
        const u32 ka = a ^ (((u32)((int)a >> 31)) | 0x80000000u), kb = b ^ (((u32)((int)b >> 31)) | 0x80000000u);
        xb[k] = ((ka > kb) == take_max) ? a : b;
      }
    }
    if (!FULL) {
      // slots past the end of the block must repeat a valid element of the block
      const u32 first = __shfl(xb[0], (int)(lane & ~7u));
#pragma unroll
      for (int k = 0; k < kE; ++k) if (k >= nv) xb[k] = first;
    }
  }
};

// Lead codes and differing bytes of the lane's elements into the block's body, for a wavefront with a raw block
// (an element emits up to 4 bytes).  The scheme of write_body_or below with one change: v_alignbyte shifts by 0 to 3
// bytes, so an element's c <= 4 bytes enter the string in two pushes, min(c, 2) bytes of t and the c - min(c, 2)
// bytes above them.  Four elements are at most 16 bytes: four registers, five words touched.  (Byte stores under
// predicates, the first version, cost four times the instructions.)
template <bool FULL>
__device__ __forceinline__ void write_body_or4(const EncRegs& r, u32* body32, u32 off) {
  const u32 l8 = threadIdx.x & 7u;
  {
    const u32 q = off + 4u * l8;
    const u32 sel = __builtin_amdgcn_alignbyte(0x00070605u, 0x04030201u, ~q);     // bytes 4-a, 5-a, 6-a, 7-a
    u32* w = body32 + (q >> 2);
    if (FULL || 4u * l8 < r.nlead) {
      lds_or32(w, __builtin_amdgcn_perm(r.lc, 0u, sel));
      lds_or32(w + 1, __builtin_amdgcn_perm(0u, r.lc, sel));
    }
  }
  u32 p = off + r.nlead + (r.incl - r.len);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    u32 a3 = 0, a2 = 0, a1 = 0, a0 = 0, bytes = 0;
#pragma unroll
    for (int e = 3; e >= 0; --e) {
      const int k = 4 * g + e;
      u32 c = r.nb - ((r.lc >> (2 * k)) & 3u);
      if (!FULL && k >= r.nv) c = 0;
      const u32 c1 = c < 2u ? c : 2u, c2 = c - c1;
      const u32 t = r.t[k], th = t >> (8u * c1);
      bytes += c;
      // pushes number 2 (3 - e) + 1 and + 2: the string holds at most 2 (pushes so far) bytes, so the low registers
      // only take part from the push on that can reach them
      const int n1 = 2 * (3 - e) + 1, n2 = n1 + 1;
      if (n1 >= 7) a0 = __builtin_amdgcn_alignbyte(a1, a0, c1);
      if (n1 >= 5) a1 = __builtin_amdgcn_alignbyte(a2, a1, c1);
      if (n1 >= 3) a2 = __builtin_amdgcn_alignbyte(a3, a2, c1);
      a3 = __builtin_amdgcn_alignbyte(t, a3, c1);
      if (n2 >= 7) a0 = __builtin_amdgcn_alignbyte(a1, a0, c2);
      if (n2 >= 5) a1 = __builtin_amdgcn_alignbyte(a2, a1, c2);
      if (n2 >= 3) a2 = __builtin_amdgcn_alignbyte(a3, a2, c2);
      a3 = __builtin_amdgcn_alignbyte(th, a3, c2);
    }
    const u32 sel = __builtin_amdgcn_alignbyte(0x00000102u, 0x03040506u, ~p);    // bytes a+3, a+2, a+1, a with a = p & 3
    u32* w = body32 + (p >> 2);
    lds_or32(w, __builtin_amdgcn_perm(0u, a3, sel));
    lds_or32(w + 1, __builtin_amdgcn_perm(a3, a2, sel));
    lds_or32(w + 2, __builtin_amdgcn_perm(a2, a1, sel));
    lds_or32(w + 3, __builtin_amdgcn_perm(a1, a0, sel));
    lds_or32(w + 4, __builtin_amdgcn_perm(a0, 0u, sel));
    p += bytes;
  }
}

// The same for blocks without raw elements (at most 3 bytes per element), without any predication: the stage
// is all zeros where nothing has been written yet, and a lane ORs whole aligned words into it.
//   * A lane's elements go four at a time.  The up to 12 bytes of four elements are first gathered in three
//     registers as a byte-reversed string: elements are pushed last to first, a push is {t, A} >> 8c (the low c
//     bytes of t are exactly the bytes to emit, least significant first, and v_alignbyte takes c from the two
//     low bits of its operand, so c = 0 needs no special case).  After the four pushes the reversed string
//     sits at the top of the three registers, zeros below.
//   * One v_perm per output word then reverses the bytes back and shifts the string to the byte position
//     (p & 3) of its place in the stage; four words at most are touched, and words or bytes that belong to a
//     neighbour (the lane before, the next group, the next block) receive zeros.
// `off`: byte offset of the block's body in the stage; body32: the stage as words (16-byte aligned).
template <bool FULL, bool NB2>
__device__ __forceinline__ void write_body_or(const EncRegs& r, u32* body32, u32 off) {
  const u32 l8 = threadIdx.x & 7u;
  {
    // the lane's four bytes of lead codes at byte offset q: word 0 gets lc << 8a, word 1 gets lc >> (32 - 8a), a = q & 3
    const u32 q = off + 4u * l8;
    const u32 sel = __builtin_amdgcn_alignbyte(0x00070605u, 0x04030201u, ~q);     // bytes 4-a, 5-a, 6-a, 7-a
    u32* w = body32 + (q >> 2);
    if (FULL || 4u * l8 < r.nlead) {
      lds_or32(w, __builtin_amdgcn_perm(r.lc, 0u, sel));
      lds_or32(w + 1, __builtin_amdgcn_perm(0u, r.lc, sel));
    }
  }
  const u32 cc = r.cc;
  // bytes of each group of four elements, and their running sums, one per byte
  const u32 pr = (cc & 0x33333333u) + ((cc >> 2) & 0x33333333u);
  const u32 gs = (pr + (pr >> 4)) & 0x0f0f0f0fu;
  u32 run = gs + (gs << 8); run += run << 16;
  const u32 p0 = off + r.nlead + (r.incl - r.len);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const u32 c0 = cc >> (8 * g), c1 = cc >> (8 * g + 2), c2 = cc >> (8 * g + 4), c3 = cc >> (8 * g + 6);
    const u32 p = g == 0 ? p0 : p0 + ((run >> (8 * (g - 1))) & 0xffu);
    const u32 sel = __builtin_amdgcn_alignbyte(0x00000102u, 0x03040506u, ~p);    // bytes a+3, a+2, a+1, a with a = p & 3
    u32* w = body32 + (p >> 2);
    if (NB2) {
      // at most 2 bytes per element: 8 bytes per group, two registers, three words
      u32 a1 = __builtin_amdgcn_alignbyte(r.t[4 * g + 3], 0u, c3);
      a1 = __builtin_amdgcn_alignbyte(r.t[4 * g + 2], a1, c2);
      u32 a0 = __builtin_amdgcn_alignbyte(a1, 0u, c1);
      a1 = __builtin_amdgcn_alignbyte(r.t[4 * g + 1], a1, c1);
      a0 = __builtin_amdgcn_alignbyte(a1, a0, c0);
      a1 = __builtin_amdgcn_alignbyte(r.t[4 * g], a1, c0);
      lds_or32(w, __builtin_amdgcn_perm(0u, a1, sel));
      lds_or32(w + 1, __builtin_amdgcn_perm(a1, a0, sel));
      lds_or32(w + 2, __builtin_amdgcn_perm(a0, 0u, sel));
    } else {
      u32 a2 = __builtin_amdgcn_alignbyte(r.t[4 * g + 3], 0u, c3);
      u32 a1 = __builtin_amdgcn_alignbyte(a2, 0u, c2);
      a2 = __builtin_amdgcn_alignbyte(r.t[4 * g + 2], a2, c2);
      u32 a0 = __builtin_amdgcn_alignbyte(a1, 0u, c1);
      a1 = __builtin_amdgcn_alignbyte(a2, a1, c1);
      a2 = __builtin_amdgcn_alignbyte(r.t[4 * g + 1], a2, c1);
      a0 = __builtin_amdgcn_alignbyte(a1, a0, c0);
      a1 = __builtin_amdgcn_alignbyte(a2, a1, c0);
      a2 = __builtin_amdgcn_alignbyte(r.t[4 * g], a2, c0);
      lds_or32(w, __builtin_amdgcn_perm(0u, a2, sel));
      lds_or32(w + 1, __builtin_amdgcn_perm(a2, a1, sel));
      lds_or32(w + 2, __builtin_amdgcn_perm(a1, a0, sel));
      lds_or32(w + 3, __builtin_amdgcn_perm(a0, 0u, sel));
    }
  }
}

// ZERO: the LDS bytes are set to zero behind the copy (a stage must be all zeros before bodies are ORed into it).
// Four vectors per lane are read before the first one is stored, so that a payload of up to 4 KB costs one
// LDS round trip.
// The stores to the outgoing stream are ordinary ones: streaming (non-temporal) stores gain 1.6 % in the coder, but
// the stream then bypasses the memory-side cache, and a decoder that reads it next on the same device loses 15 %.
template <bool ZERO>
__device__ __forceinline__ void copy_out(unsigned char* dst, unsigned char* src, u32 n) {
  const u32 lane = threadIdx.x & 63u;
  const u32 n16 = n >> 4;
  constexpr int kBatch = 4;
  for (u32 j0 = 0; j0 < n16; j0 += 64u * kBatch) {
    uint4 v[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const u32 j = j0 + lane + 64u * (u32)i;
      v[i] = make_uint4(0, 0, 0, 0);
      if (j < n16) v[i] = *(const uint4*)(src + 16u * j);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const u32 j = j0 + lane + 64u * (u32)i;
      if (j < n16) {
        if (ZERO) *(uint4*)(src + 16u * j) = make_uint4(0, 0, 0, 0);
        __builtin_memcpy(dst + 16u * j, &v[i], 16);
      }
    }
  }
  const u32 rest = (n >> 2) & 3u;
  if (lane < rest) {
    ((u32*)(dst + 16u * n16))[lane] = ((const u32*)(src + 16u * n16))[lane];
    if (ZERO) ((u32*)(src + 16u * n16))[lane] = 0u;
  }
}

// n bytes (a multiple of 4) between global addresses: src 16-byte aligned, dst 4-byte aligned.
__device__ __forceinline__ void copy_gg(unsigned char* dst, const unsigned char* src, u32 n) {
  const u32 lane = threadIdx.x & 63u;
  const u32 n16 = n >> 4;
  constexpr int kBatch = 4;
  for (u32 j0 = 0; j0 < n16; j0 += 64u * kBatch) {
    uint4 v[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const u32 j = j0 + lane + 64u * (u32)i;
      v[i] = make_uint4(0, 0, 0, 0);
      if (j < n16) v[i] = *(const uint4*)(src + 16u * j);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const u32 j = j0 + lane + 64u * (u32)i;
      if (j < n16) __builtin_memcpy(dst + 16u * j, &v[i], 16);
    }
  }
  const u32 rest = (n >> 2) & 3u;
  if (lane < rest) ((u32*)(dst + 16u * n16))[lane] = ((const u32*)(src + 16u * n16))[lane];
}

// One unit of a chunk: classify its 8 blocks, code the elements, append the bodies to the chunk's body
// bytes (bodybase so far), mu and sizes to the metadata.  The bodies are assembled in the wavefront's LDS
// stage; when a unit does not fit behind what is staged, the staged bytes (all but the last < 16) move on to
// the wavefront's spill slot and the stage starts over: `flushed` counts the body bytes already in the slot.
// Returns the body bytes of the unit.
// The staged body bytes (all but the last < 16) move on to the wavefront's spill slot; the stage starts over.
template <u32 CAP>
__device__ __forceinline__ void flush_stage(EncWaveLds<CAP>& L, u32 bodybase, u32& flushed, unsigned char* slot) {
  const u32 lane = threadIdx.x & 63u;
  const u32 fill = bodybase - flushed, n = fill & ~15u;
  copy_out<true>(slot + kMetaMax + flushed, L.body, n);
  unsigned char keep = 0;
  if (lane < fill - n) { keep = L.body[n + lane]; L.body[n + lane] = 0; }
  if (lane < fill - n) L.body[lane] = keep;
  flushed += n;
}

// Where the bodies of a unit's blocks go: scans of the emitted bytes over the block and of the body sizes over the
// wavefront, room made in the stage, mu and sizes noted for the chunk's metadata.  len: bytes the lane emits
// (0 if its block is not active); v: body bytes of the block at its last lane, else 0.
struct UnitPos { u32 incl, nlead, start, total; };
template <bool FULL, u32 CAP, class Src>
__device__ __forceinline__ UnitPos place_unit(u32 len, bool active, int blen, int blk, int nbc, const RowClass& rc,
                                              const GrpMasks& gm, EncWaveLds<CAP>& L, u32 bodybase, u32& flushed,
                                              unsigned char* slot, Src& src) {
  const u32 l8 = threadIdx.x & 7u;
  UnitPos o;
  o.incl = grp_scan_add(len, gm);
  o.nlead = FULL ? 32u : (u32)((blen + 3) >> 2);
  const u32 v = (l8 == kGrp - 1 && active) ? o.nlead + o.incl : 0u;       // the block's body bytes, at its last lane
  const u32 sc = wave_scan_add(v);
  o.total = (u32)__builtin_amdgcn_readlane((int)sc, 63);
  if (bodybase - flushed + o.total > CAP) flush_stage<CAP>(L, bodybase, flushed, slot);   // make room: at most 15 + 8 * 544 bytes are needed
  src.make_room(bodybase - flushed + o.total);                            // a window of the source in the way is given up
  o.start = bodybase - flushed + sc - v;                                  // in the stage; the same for all lanes of a block
  if (l8 == kGrp - 1 && blk < nbc) {
    L.meta[2 + blk] = f2u(rc.mu);
    L.tmp[blk] = v | ((rc.type == 0 ? 0u : (rc.type == 2 ? 32u : 9u + rc.m)) << 16);
  }
  return o;
}

template <bool FULL, u32 CAP, class Src>
__device__ __forceinline__ u32 encode_unit(const u32 (&xb)[kE], int nv, int blen, int blk, int nbc, const Params& P,
                                           const GrpMasks& gm, EncWaveLds<CAP>& L, u32 bodybase, u32& flushed, unsigned char* slot,
                                           Src& src) {
  const bool exists = FULL || blen > 0;
  const RowClass rc = classify_row(xb, P.eb, P.e_eb);
  const bool active = exists && rc.type != 0;
  const bool anyraw = __ballot(rc.type == 2) != 0;
  EncRegs r;
  r.active = active; r.anyraw = anyraw;
  if (anyraw) enc_code<FULL, true>(xb, nv, rc, gm, r);
  else enc_code<FULL, false>(xb, nv, rc, gm, r);
  if (!active) r.len = 0;
  const UnitPos o = place_unit<FULL, CAP>(r.len, active, blen, blk, nbc, rc, gm, L, bodybase, flushed, slot, src);
  r.incl = o.incl; r.nlead = o.nlead;
  if (active) {
    if (anyraw) write_body_or4<FULL>(r, (u32*)L.body, o.start);
    else if (__ballot(r.nb != 2u) == 0) write_body_or<FULL, true>(r, (u32*)L.body, o.start);     // active lanes only
    else write_body_or<FULL, false>(r, (u32*)L.body, o.start);
  }
  return o.total;
}

// A coded chunk: payload bytes, metadata bytes, body bytes, and how many of the body bytes are in the spill
// slot already (a multiple of 16); the rest is in the LDS stage.
struct ChunkOut { u32 payload, meta_len, bodies, flushed; };

// Chunk c into the wavefront's LDS (and, if it outgrows the stage, its spill slot).
// xa / nv / blen: the floats of the chunk's first unit if `preloaded` (requested by the previous turn), else they are
// loaded here.  `turn` is called between the units (the work a wavefront does for its workgroup while it codes) and
// names, in front of the last unit, the chunk the wavefront codes next: a source that requests its elements a unit
// ahead then requests that chunk's first unit, so that the turn after this one starts without a memory round trip
// (on return `preloaded` says whether xa holds it).
template <bool FULL, u32 CAP, class Src, class Turn>
__device__ __forceinline__ ChunkOut encode_chunk(Src& src, u32 c, const Params& P, const GrpMasks& gm, EncWaveLds<CAP>& L,
                                                 unsigned char* slot, u32 (&xa)[kE], int& nv, int& blen, bool& preloaded,
                                                 Turn& turn) {
  const u32 lane = threadIdx.x & 63u;
  const int nbc = FULL ? kBpc : (int)((P.n - (u64)c * kChunk + kBlock - 1) / kBlock);
  const int nunits = FULL ? kUnits : (nbc + 7) / 8;
  src.begin_chunk(c, P, L.body);
  if (!(Src::kPrefetch && preloaded)) src.template load<FULL>(P, c, 0, xa, nv, blen);
  preloaded = false;
  u32 bodybase = 0, flushed = 0;
#pragma unroll 1
  for (int u = 0; u < nunits; ++u) {
    const int blk = 8 * u + (int)(lane >> 3);
    if (Src::kPrefetch) {
      // A wavefront that is behind the others of its SIMD in its chunk goes first: the wavefronts of a turn reach
      // the turn's barrier together instead of one after the other (the issue arbiter otherwise prefers the oldest
      // one, and the last one of a SIMD codes alone, at two thirds of the issue rate).  Measured: 3 % for
      // compress; the reduce step, which does not request its floats a unit ahead, is better off staggered.
      if (u == 0) __builtin_amdgcn_s_setprio(3);
      else if (u == 1) __builtin_amdgcn_s_setprio(2);
      else if (u == 2) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
    }
    if (Src::kPrefetch) {
      // The floats of the next unit are requested now and taken over behind the coding of this one.  In front of the
      // chunk's last unit the request is for the first unit of the chunk the wavefront codes next (if that is a whole
      // chunk; else this chunk's first unit once more, unused: every pass requests and takes over the same way).
      u32 xn[kE]; int nvn = 0, blenn = 0;
      u32 cl = c; int ul = u + 1;
      if (u + 1 == nunits) {
        ul = 0;
        if (FULL) {
          const u32 cn = turn.next_chunk();
          if (cn != ~0u) { cl = cn; preloaded = true; }
        }
      }
      src.template load<FULL>(P, cl, ul, xn, nvn, blenn);
      src.template finish<FULL>(P, c, u, xa, nv, blen, gm);
      bodybase += encode_unit<FULL, CAP>(xa, nv, blen, blk, nbc, P, gm, L, bodybase, flushed, slot, src);
#pragma unroll
      for (int k = 0; k < kE; ++k) xa[k] = xn[k];
      nv = nvn; blen = blenn;
    } else {
      if (u > 0) src.template load<FULL>(P, c, u, xa, nv, blen);
      if (src.needs_room(P, c, u, bodybase - flushed)) flush_stage<CAP>(L, bodybase, flushed, slot);
      src.fetch(P, c, u, bodybase - flushed);
      src.template finish<FULL>(P, c, u, xa, nv, blen, gm);
      bodybase += encode_unit<FULL, CAP>(xa, nv, blen, blk, nbc, P, gm, L, bodybase, flushed, slot, src);
    }
    turn.between_units(u);
  }
  turn.after_units(nunits);
  src.end_chunk();
  if (Src::kPrefetch) __builtin_amdgcn_s_setprio(0);
  // metadata: lane j = block j
  const u32 tv = (int)lane < nbc ? L.tmp[lane] : 0u;
  const u32 rq = tv >> 16, bs = tv & 0xffffu;
  const u64 bitmap = __ballot(rq != 0);
  const u32 k = (u32)__popcll(bitmap);
  const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(bitmap >> 32), __builtin_amdgcn_mbcnt_lo((u32)bitmap, 0u));
  const u32 meta_raw = 8u + 4u * (u32)nbc + 3u * k;
  ChunkOut o;
  o.meta_len = pad4(meta_raw); o.bodies = bodybase; o.payload = o.meta_len + pad4(bodybase); o.flushed = flushed;
  unsigned char* m8 = (unsigned char*)L.meta;
  if (lane == 0) {
    L.meta[0] = (u32)bitmap; L.meta[1] = (u32)(bitmap >> 32);
    for (u32 i = meta_raw; i < o.meta_len; ++i) m8[i] = 0;            // the stage's body bytes behind the last body are zeros already
  }
  if (rq != 0) {
    lds_store16(m8 + 8 + 4 * nbc + 2 * rank, bs);
    m8[8 + 4 * nbc + 2 * k + rank] = (unsigned char)rq;
  }
  return o;
}

// Header of the stream: written by the wavefront that places the last chunk.
__device__ __forceinline__ void write_header(const Params& P, u64 total) {
  u32* h = KARGP(u32*, out);
  h[0] = 0x31585343u;               // 'C','S','X','1'
  h[1] = (u32)kBlock | ((u32)kChunk << 16);
  h[2] = (u32)P.n; h[3] = (u32)(P.n >> 32);
  h[4] = KARG32(eb_bits); h[5] = KARG32(nchunks);
  h[6] = (u32)total; h[7] = (u32)(total >> 32);
  st_dev(&KARGP(Workspace*, ws)->total, total);
}

// The payload of chunk c, still in LDS stage L (and, what had outgrown it, in the spill slot), goes to its place.
template <u32 CAP>
__device__ __forceinline__ void place_staged(u32 c, const ChunkOut& o, u64 off, const unsigned char* slot, const Params& P,
                                             EncWaveLds<CAP>& L) {
  const u32 lane = threadIdx.x & 63u;
  const u32 nchunks = KARG32(nchunks), c1 = KARG32(c1);
  const u64 front = kHeader + 4ull * nchunks;
  const bool fits = front + off + o.payload <= KARG64(out_cap);
  if (lane == 0) {
    if (!fits) raise_error(P, CCOLL_ENOSPC);
    if (c + 1 == nchunks) write_header(P, front + off + o.payload);
    else if (c + 1 == c1) st_dev(&KARGP(Workspace*, ws)->total, front + off + o.payload);      // a piece of a stream: bytes so far
    unsigned long long* progress = KARGP(unsigned long long*, progress);
    if (c + 1 == c1 && progress) { progress[0] = c1; progress[1] = front + off + o.payload; }
  }
  if (!fits) return;
  unsigned char* dst = KARGP(unsigned char*, out) + front + off;
  copy_out<false>(dst, (unsigned char*)L.meta, o.meta_len);
  if (o.flushed) copy_gg(dst + o.meta_len, slot + kMetaMax, o.flushed);
  copy_out<true>(dst + o.meta_len + o.flushed, L.body, pad4(o.bodies) - o.flushed);
}

template <int NW>
struct GroupLds {
  u32 size[3][NW];                                   // payload bytes of the group's chunks, by turn mod 3: a turn's sizes are
                                                     // still read (offsets of parked payloads) during the next turn
  u64 pbase[2];                                      // byte offset of the parked group's first payload
  u32 pres[2];                                       // look-back result for it (1 known, 0 abandoned)
  unsigned long long nextq[2];                       // by turn mod 2: (turn << 32) | the workgroup's group of the turn after
  u32 first;                                         // the workgroup's first group
};

// What a wavefront does for its workgroup while it codes its chunk of the turn (called by encode_chunk between the
// units).  The first wavefront hands on the ticket of the workgroup's next group as soon as it is there (after its
// first unit), so that every wavefront knows in front of its last unit which chunk it codes next, and walks the
// look-back scan for the group of the turn before when its own chunk is coded: by then the groups in front have,
// as a rule, announced their sizes.  (Walking the scan earlier, between the units, was slower: 0.145 ms against
// 0.141 ms on the 512^3 field; more of the walks then have to wait.)
template <int NW>
struct TurnWork {
  GroupLds<NW>& g; const Params& P;
  u32 wv, turn, ngroups, nfull;
  bool pend; u32 pq;                                 // the group of the turn before waits for its place
  u32 tnext;                                         // thread 0: the group drawn for the turn after this one (ngroups: none)
  bool handed;
  __device__ __forceinline__ void hand_on_ticket() {
    if (threadIdx.x == 0)
      __hip_atomic_store(&g.nextq[turn & 1u], ((unsigned long long)turn << 32) | tnext, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    handed = true;
  }
  __device__ __forceinline__ void between_units(int u) {
    if (wv == 0 && u == 0) hand_on_ticket();
  }
  __device__ __forceinline__ void after_units(int) {
    if (wv != 0) return;
    if (!handed) hand_on_ticket();                   // a chunk without units cannot occur; kept for safety
    if (pend) {
      const u32 lane = threadIdx.x & 63u, par = turn & 1u, tp = (turn + 2u) % 3u;
      u32 ptot = 0;
#pragma unroll
      for (int j = 0; j < NW; ++j) ptot += g.size[tp][j];
      u64 pb = 0;
      const bool pr = lookback(KARGP(u64*, stat), pq, ptot, P, pb);
      if (lane == 0) { g.pres[par] = pr ? 1u : 0u; g.pbase[par] = pb; }
    }
  }
  // The chunk this wavefront codes in the next turn if that is a whole chunk, else ~0.  The ticket has as a rule
  // been handed on long ago; the wait is bounded, and giving up only costs the early request of the floats.
  __device__ __forceinline__ u32 next_chunk() {
    unsigned long long w = 0;
    bool have = false;
    for (int tries = 0; tries < 64 && !have; ++tries) {
      w = __hip_atomic_load(&g.nextq[turn & 1u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      have = (u32)(w >> 32) == turn;
      if (!have) __builtin_amdgcn_s_sleep(1);
    }
    if (!have) return ~0u;
    const u32 qn = (u32)w;
    if (qn >= ngroups) return ~0u;
    const u32 cn = qn * NW + wv;
    return (cn < nfull && cn < KARG32(c1)) ? cn : ~0u;
  }
};

// Per turn a workgroup codes one group of NW chunks.  When a group has just been coded, the groups in front
// of it are as a rule still being coded and its place in the stream is not known, so a payload is never
// placed in the turn it is coded in, but one turn later: by then the groups in front have announced their
// sizes, the walk through the scan returns at once, and coding never waits for a slower workgroup.
// Meanwhile the payload stays where it is: a wavefront has two LDS stages and uses them in turns.
// One barrier per turn.  slot_bytes: size of a spill slot; every wavefront has two, used in turns.
template <int NW, u32 CAP, class Src>
__device__ __forceinline__ void encode_groups(Src& src, const Params& P, GroupLds<NW>& g, EncWaveLds<CAP>* Ls, u32 slot_bytes) {
  const u32 lane = threadIdx.x & 63u, wv = (u32)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // a scalar
  const u32 nfull = (u32)(P.n / kChunk);
  const u32 g0 = KARG32(c0) / NW;                             // the launch codes chunks [c0, c1): groups [g0, ngroups)
  const u32 ngroups = (KARG32(c1) + NW - 1) / NW;
  const GrpMasks gm = grp_masks();
  // two spill slots per wavefront, used in turns: one may still hold the parked payload of the previous turn
  // while the chunk being coded outgrows the LDS stage into the other
  const u64 slot0 = ((u64)blockIdx.x * NW + wv) * 2u * slot_bytes;          // + the spill area's base (a parameter read where used)

  // bodies are ORed into the stages: they start as zeros, and every copy out of a stage leaves zeros behind
#pragma unroll
  for (int i = 0; i < 2; ++i)
    for (u32 j = lane; j < (CAP + 16u) / 16u; j += 64u) *(uint4*)(Ls[i].body + 16u * j) = make_uint4(0, 0, 0, 0);
  if (threadIdx.x == 0) {
    Workspace* ws = KARGP(Workspace*, ws);
    const u32 sel = KARG32(ticket_sel);
    if (blockIdx.x == 0) st_dev(&ws->ticket[sel ^ 1u], 0ull);                 // for the next launch on the stream
    const u64 t = (u64)g0 + __hip_atomic_fetch_add(&ws->ticket[sel], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    g.first = t < (u64)ngroups ? (u32)t : ngroups;
    g.nextq[0] = ~0ull; g.nextq[1] = ~0ull;
  }
  // Workgroups that start together stay in step for many turns (their turns take the same time), and the memory
  // system then sees the whole device ask at once and pause at once.  A launch that is long enough to gain from it
  // (four turns per workgroup or more) spreads the starts over about 6 us, 16 steps of 0.4 us by workgroup number.
  // Measured on the 512^3 field: 1.5 % for compress; the reduce step's three workgroups per compute unit are out
  // of step anyway.
  if (Src::kPrefetch && ngroups - g0 >= 4u * gridDim.x)
    for (u32 i = 0; i < 2u * (blockIdx.x & 15u); ++i) __builtin_amdgcn_s_sleep(8);
  __syncthreads();
  u32 q = g.first;
  bool pend = false, phave = false, dead = false;
  u32 pq = 0, pc = 0;
  ChunkOut po; po.payload = 0; po.meta_len = 0; po.bodies = 0; po.flushed = 0;
  u32 xa[kE]; int nv = 0, blen = 0; bool preloaded = false;    // the first unit of the next chunk, requested a turn ahead
  u32 turn = 0;
  for (; q < ngroups; ++turn) {
    const u32 par = turn & 1u, ts = turn % 3u, tp = (turn + 2u) % 3u;   // tp: the previous turn's sizes
    unsigned char* slots = KARGP(unsigned char*, spill) + slot0;
    unsigned char* slot = slots + par * slot_bytes;           // this turn's
    unsigned char* pslot = slots + (par ^ 1u) * slot_bytes;   // the previous turn's
    EncWaveLds<CAP>& L = Ls[par];
    EncWaveLds<CAP>& Lp = Ls[par ^ 1u];                       // where the previous turn's payload is
    TurnWork<NW> tw{g, P, wv, turn, ngroups, nfull, pend, pq, 0u, false};
    // the next group is asked for now; the first wavefront hands it on while it codes
    if (threadIdx.x == 0) {
      const u64 t = (u64)g0 + __hip_atomic_fetch_add(&KARGP(Workspace*, ws)->ticket[KARG32(ticket_sel)], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      tw.tnext = t < (u64)ngroups ? (u32)t : ngroups;
    }
    const u32 c = q * NW + wv;
    const bool have = c < KARG32(c1);
    ChunkOut o; o.payload = 0; o.meta_len = 0; o.bodies = 0; o.flushed = 0;
    if (have) {
      if (c < nfull) o = encode_chunk<true, CAP>(src, c, P, gm, L, slot, xa, nv, blen, preloaded, tw);
      else { preloaded = false; o = encode_chunk<false, CAP>(src, c, P, gm, L, slot, xa, nv, blen, preloaded, tw); }
    } else preloaded = false;
    if (lane == 0) {
      g.size[ts][wv] = o.payload;
      if (have) ((u32*)(KARGP(unsigned char*, out) + kHeader))[c] = o.payload;       // the front index entry (Sec. III-E.2)
    }
    __syncthreads();
    if (wv == 0) {                                            // announce this group's size
      u32 gtot = 0;
#pragma unroll
      for (int j = 0; j < NW; ++j) gtot += g.size[ts][j];
      publish_size(KARGP(u64*, stat), q, gtot, KARG32(scan_epoch));
    }
    if (pend) {
      if (g.pres[par] == 0) { dead = true; break; }           // the scan wait was abandoned: error raised, everyone leaves
      if (phave) {
        u64 off = g.pbase[par];
        for (u32 j = 0; j < wv; ++j) off += g.size[tp][j];
        place_staged<CAP>(pc, po, off, pslot, P, Lp);
      }
    }
    pend = true; phave = have; pq = q; pc = c; po = o;
    q = (u32)g.nextq[par];
  }
  if (pend && !dead) {                                        // the last group of this workgroup is still parked
    const u32 par = turn & 1u, tp = (turn + 2u) % 3u;
    if (wv == 0) {
      u32 ptot = 0;
#pragma unroll
      for (int j = 0; j < NW; ++j) ptot += g.size[tp][j];
      u64 pb = 0;
      const bool pr = lookback(KARGP(u64*, stat), pq, ptot, P, pb);
      if (lane == 0) { g.pres[par] = pr ? 1u : 0u; g.pbase[par] = pb; }
    }
    __syncthreads();
    if (g.pres[par] == 1 && phave) {
      u64 off = g.pbase[par];
      for (u32 j = 0; j < wv; ++j) off += g.size[tp][j];
      place_staged<CAP>(pc, po, off, KARGP(unsigned char*, spill) + slot0 + (par ^ 1u) * slot_bytes, P, Ls[par ^ 1u]);
    }
  }
}

// compress: 12 wavefronts per workgroup, one workgroup per compute unit (3 wavefronts per SIMD: no register
// spills, and 13 KB of LDS per wavefront for its two stages)
constexpr int kEncWaves = 12;
constexpr u32 kEncCap = 6240;                        // body bytes a wavefront stages at a time; what outgrows them goes to the spill slot
constexpr u32 kSpillSlot = 22272;                    // >= kMetaMax + 40 * 544 + 16, a multiple of 256: a whole payload
static_assert(CCOLL_PIECE_CHUNKS == kEncWaves, "a piece of a stream ends where a group of chunks ends");
struct __align__(16) CompressSmem { EncWaveLds<kEncCap> wave[kEncWaves][2]; GroupLds<kEncWaves> g; };

__global__ void __launch_bounds__(64 * kEncWaves) __attribute__((amdgpu_waves_per_eu(3, 3))) k_compress(Params P) {
  __shared__ CompressSmem sm;
  SrcPlain src; src.in = (const float*)P.in; src.al = P.aligned16 != 0;
  encode_groups<kEncWaves, kEncCap>(src, P, sm.g, sm.wave[__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))], kSpillSlot);
}

// reduce step: 4 wavefronts per workgroup, three workgroups per compute unit; two stages per wavefront like
// compress, the window of the incoming payload lives in the stage being coded into
constexpr int kRedWaves = 4;
constexpr u32 kRedCap = 6240;
struct __align__(16) ReduceSmem {
  EncWaveLds<kRedCap> wave[kRedWaves][2];
  GroupLds<kRedWaves> g;
};
static_assert(kMetaMax + kBpc * kMaxBody + 16 <= kSpillSlot && kRedCap >= 8 * kMaxBody + 64, "spill slot, stage");

template <int OP>
__device__ __forceinline__ void reduce_step_body(const Params& P, ReduceSmem& sm) {
  const u32 wv = (u32)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  SrcReduce<OP, kRedCap> src; src.local = P.local; src.al = P.aligned16 != 0; src.s = (const unsigned char*)P.cin;
  src.stage = nullptr; src.src = nullptr; src.payload = 0; src.wbase = 0; src.wlen = 0; src.wpos = 0; src.good = false;
  encode_groups<kRedWaves, kRedCap>(src, P, sm.g, sm.wave[wv], kSpillSlot);
}
// one kernel per reduction, so that the sum carries nothing of the others
__global__ void __launch_bounds__(64 * kRedWaves) __attribute__((amdgpu_waves_per_eu(CCOLL_RED_OCC, CCOLL_RED_OCC))) k_reduce_step(Params P) {
  __shared__ ReduceSmem sm;
  reduce_step_body<CCOLL_OP_SUM>(P, sm);
}
__global__ void __launch_bounds__(64 * kRedWaves) __attribute__((amdgpu_waves_per_eu(CCOLL_RED_OCC, CCOLL_RED_OCC))) k_reduce_step_max(Params P) {
  __shared__ ReduceSmem sm;
  reduce_step_body<CCOLL_OP_MAX>(P, sm);
}
__global__ void __launch_bounds__(64 * kRedWaves) __attribute__((amdgpu_waves_per_eu(CCOLL_RED_OCC, CCOLL_RED_OCC))) k_reduce_step_min(Params P) {
  __shared__ ReduceSmem sm;
  reduce_step_body<CCOLL_OP_MIN>(P, sm);
}

// ---------------------------------------------------------------------------------------------
// scratch of the entry point that allocates nothing (ccoll_szx_decompress_static)
// ---------------------------------------------------------------------------------------------
// What ccoll_szx_decompress keeps in the context's device allocations -- the result / error words and the
// chunk-start offsets that k_index_scan hands to k_decompress -- in a static device array, so that a caller
// under stream capture or in a loop that must not allocate can decode without a context.  Every device
// that runs the library holds its own copy until the process ends.
constexpr size_t kStaticMaxElems = CCOLL_STATIC_MAX_ELEMS;
constexpr size_t kStaticMaxChunks = (kStaticMaxElems + kChunk - 1) / kChunk;
struct StaticScratch {
  Workspace ws;
  u64 offs[kStaticMaxChunks + 1];
};

// The words of the last call are cleared by a kernel, not by a memset, so that the sequence can be captured
// into a graph and replayed.
__global__ void k_static_fail(Params P) {
  if (threadIdx.x == 0) raise_error(P, CCOLL_ECORRUPT, 1);
}
__global__ void k_static_begin(Workspace* ws) {
  if (threadIdx.x == 0) { st_dev(&ws->total, 0ull); st_dev(&ws->err, 0ull); st_dev(&ws->abort, 0ull); }
}

}  // namespace

// file scope: host code takes its device address with hipGetSymbolAddress, never by its name
static __device__ __align__(256) unsigned char scratch[(sizeof(StaticScratch) + 255) / 256 * 256];

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct ccoll_ctx {
  int device;
  hipStream_t stream;
  Workspace* ws;          // device
  u64* stat;              // device, cap_chunks status words
  u64* offs;              // device, cap_chunks chunk offsets of the incoming stream
  size_t cap_chunks;
  u32 epoch;
  u64* host_ws;           // pinned copy of the workspace words
  u32 last_epoch;         // epoch of the last call that kept its result in the context
  u32 waited_epoch;       // calls up to this epoch have been reported by ccoll_wait
  u64 own_slot;           // bit i: the call of epoch (epoch - i) keeps its result in the context (not in a caller's slot)
  u32 idx_epoch;          // epoch of the ccoll_szx_index call whose offsets are kept
  size_t spill_waves;     // wavefronts the spill area has slots for
  bool pipe_open;         // a stream is being compressed piece by piece (ccoll_szx_compress_begin)
  size_t pipe_n, pipe_cap, pipe_next; void* pipe_out; float pipe_eb; u32 pipe_epoch;
  bool last_total;        // that call reports a byte count
  int grid_compress, grid_decompress, grid_reduce;   // workgroups that are resident at once
  u32 ticket_sel;         // ticket counter of the next ticketed launch (0 / 1); the other one is being zeroed by the last
  u32 spin_limit;         // polls after which a scan wait gives up (ccoll_set_scan_wait)
  const void* idx_ptr;    // the stream whose chunk offsets are in `offs` (ccoll_szx_index), or null
  size_t idx_bytes, idx_n;
  unsigned char* spill;   // device, one slot per wavefront of the widest ticketed launch
  hipEvent_t ev_start, ev_stop;   // if set: recorded around the next coding / decoding kernel (ccoll_time_next_kernel)
};

namespace {

bool eb_valid(float eb) { return isfinite(eb) && eb > 0.0f; }

// With CCOLL_DEBUG set in the environment, a failing HIP call is reported on stderr.
bool hip_ok(hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  if (getenv("CCOLL_DEBUG")) fprintf(stderr, "libccoll_szx: %s failed: %s\n", what, hipGetErrorString(e));
  return false;
}
#define HIP_OK(call) hip_ok((call), #call)

// Launch of a call's coding / decoding kernel.  If the caller has armed a pair of events, they take the start and
// the end of this dispatch itself (the dispatch packet's own time stamps: no marker packets around it).
template <class K, class... Args>
void launch_main(ccoll_ctx* c, K kernel, dim3 grid, dim3 block, Args... args) {
  if (c->ev_start || c->ev_stop) {
    hipExtLaunchKernelGGL(kernel, grid, block, 0, c->stream, c->ev_start, c->ev_stop, 0, args...);
    c->ev_start = nullptr; c->ev_stop = nullptr;
  } else {
    hipLaunchKernelGGL(kernel, grid, block, 0, c->stream, args...);
  }
}

int reset_workspace(ccoll_ctx* c) {
  if (!HIP_OK(hipMemsetAsync(c->ws, 0, sizeof(Workspace), c->stream))) return CCOLL_EHIP;
  if (c->stat && !HIP_OK(hipMemsetAsync(c->stat, 0, c->cap_chunks * sizeof(u64), c->stream))) return CCOLL_EHIP;
  c->epoch = 0; c->waited_epoch = 0; c->last_epoch = 0; c->own_slot = 0; c->idx_ptr = nullptr; c->pipe_open = false;
  c->ticket_sel = 0;
  return CCOLL_OK;
}

struct DeviceGuard {
  int prev = -1; bool ok = true;
  explicit DeviceGuard(int dev) { if (!HIP_OK(hipGetDevice(&prev)) || !HIP_OK(hipSetDevice(dev))) ok = false; }
  ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

int prepare(ccoll_ctx* c, size_t n, Params& P) {
  const size_t nchunks = (n + kChunk - 1) / kChunk;
  if (nchunks > c->cap_chunks) return CCOLL_EINVAL;
  if (c->epoch >= (1u << 26) - 2) { int rc = reset_workspace(c); if (rc) return rc; }
  memset(&P, 0, sizeof(P));
  P.n = n; P.nchunks = (u32)nchunks; P.c0 = 0; P.c1 = (u32)nchunks;
  P.epoch = ++c->epoch;
  P.scan_epoch = P.epoch; P.scan_chunks = P.nchunks;
  c->own_slot <<= 1;
  P.ws = c->ws; P.stat = c->stat; P.offs = c->offs;
  P.spin_limit = c->spin_limit;
  P.result = nullptr;
  return CCOLL_OK;
}

// Behind the work: hand {bytes, status} to the caller's device words, or remember which call the
// context's own words belong to.
int after_launch(ccoll_ctx* c, Params& P, unsigned long long* d_result, bool reports_total) {
  if (d_result) {
    P.result = (u64*)d_result; P.no_total = reports_total ? 0u : 1u;
    hipLaunchKernelGGL(k_publish, dim3(1), dim3(1), 0, c->stream, P);
  } else {
    c->last_epoch = P.epoch; c->last_total = reports_total; c->own_slot |= 1ull;
  }
  if (!HIP_OK(hipGetLastError())) { (void)reset_workspace(c); return CCOLL_EHIP; }
  return CCOLL_OK;
}

// Workgroups that fill the device once, by the occupancy calculator (the ticketed kernels do not depend on it).
template <typename K>
int occupancy_grid(ccoll_ctx* c, K kernel, int threads) {
  int per_cu = 0, cus = 0;
  if (!HIP_OK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0))) return 0;
  if (!HIP_OK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device))) return 0;
  if (getenv("CCOLL_DEBUG")) fprintf(stderr, "libccoll_szx: %d workgroups of %d threads per CU, %d CUs\n", per_cu, threads, cus);
  return per_cu * cus;
}

u32 grid_for(int resident, u32 nwork) { return nwork < (u32)resident ? nwork : (u32)resident; }

}  // namespace

extern "C" {

size_t ccoll_szx_max_compressed_bytes(size_t n) {
  const size_t nchunks = (n + kChunk - 1) / kChunk;
  return kHeader + nchunks * (size_t)(kMaxPayload + 4);
}

int ccoll_create(ccoll_ctx** out, int device, void* hip_stream) {
  if (!out) return CCOLL_EINVAL;
  *out = nullptr;
  DeviceGuard g(device);
  if (!g.ok) return CCOLL_EHIP;
  ccoll_ctx* c = new (std::nothrow) ccoll_ctx();
  if (!c) return CCOLL_EHIP;
  c->device = device; c->stream = (hipStream_t)hip_stream; c->stat = nullptr; c->cap_chunks = 0;
  c->ws = nullptr; c->spill = nullptr; c->spin_limit = kSpinLimit; c->idx_ptr = nullptr; c->idx_bytes = 0; c->idx_n = 0; c->host_ws = nullptr; c->offs = nullptr; c->last_epoch = 0; c->last_total = false; c->waited_epoch = 0; c->own_slot = 0; c->idx_epoch = 0; c->spill_waves = 0; c->pipe_open = false; c->ev_start = nullptr; c->ev_stop = nullptr;
  if (!HIP_OK(hipMalloc((void**)&c->ws, sizeof(Workspace))) ||
      !HIP_OK(hipHostMalloc((void**)&c->host_ws, sizeof(Workspace), hipHostMallocDefault))) {
    ccoll_destroy(c); return CCOLL_EHIP;
  }
  // The persistent kernels wait on each other's chunks, so a launch never has more workgroups than
  // the device keeps resident at once.
  c->grid_compress = occupancy_grid(c, k_compress, 64 * kEncWaves);
  c->grid_reduce = occupancy_grid(c, k_reduce_step, 64 * kRedWaves);
  c->grid_decompress = 1;
  if (c->grid_compress <= 0 || c->grid_reduce <= 0 || c->grid_decompress <= 0) { ccoll_destroy(c); return CCOLL_EHIP; }
  if (reset_workspace(c) != CCOLL_OK || !HIP_OK(hipStreamSynchronize(c->stream))) { ccoll_destroy(c); return CCOLL_EHIP; }
  const int rc = ccoll_reserve(c, (size_t)1 << 20);
  if (rc != CCOLL_OK) { ccoll_destroy(c); return rc; }
  *out = c;
  return CCOLL_OK;
}

int ccoll_reserve(ccoll_ctx* c, size_t max_n) {
  if (!c || max_n > ((size_t)1 << 31)) return CCOLL_EINVAL;
  const size_t need = (max_n + kChunk - 1) / kChunk + 1;
  if (need <= c->cap_chunks) return CCOLL_OK;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  if (!HIP_OK(hipStreamSynchronize(c->stream))) return CCOLL_EHIP;
  c->idx_ptr = nullptr;
  {
    // Spill slots (two whole payloads per wavefront, for chunks that outgrow their LDS stage): one pair for
    // every wavefront of the widest launch these sizes can lead to, at most the resident ones.
    const size_t gc = (need + kEncWaves - 1) / kEncWaves, gr = (need + kRedWaves - 1) / kRedWaves;
    const size_t wc = (gc < (size_t)c->grid_compress ? gc : (size_t)c->grid_compress) * kEncWaves;
    const size_t wr = (gr < (size_t)c->grid_reduce ? gr : (size_t)c->grid_reduce) * kRedWaves;
    const size_t waves = wc > wr ? wc : wr;
    if (waves > c->spill_waves) {
      if (c->spill) { (void)hipFree(c->spill); c->spill = nullptr; c->spill_waves = 0; }
      if (!HIP_OK(hipMalloc((void**)&c->spill, waves * 2 * kSpillSlot))) return CCOLL_EHIP;
      c->spill_waves = waves;
    }
  }
  if (c->stat) { (void)hipFree(c->stat); c->stat = nullptr; c->cap_chunks = 0; }
  if (c->offs) { (void)hipFree(c->offs); c->offs = nullptr; }
  if (!HIP_OK(hipMalloc((void**)&c->stat, need * sizeof(u64))) ||
      !HIP_OK(hipMalloc((void**)&c->offs, need * sizeof(u64)))) return CCOLL_EHIP;
  c->cap_chunks = need;
  int rc = reset_workspace(c);
  if (rc) return rc;
  return HIP_OK(hipStreamSynchronize(c->stream)) ? CCOLL_OK : CCOLL_EHIP;
}

int ccoll_time_next_kernel(ccoll_ctx* c, void* start_event, void* stop_event) {
  if (!c) return CCOLL_EINVAL;
  c->ev_start = (hipEvent_t)start_event; c->ev_stop = (hipEvent_t)stop_event;
  return CCOLL_OK;
}

int ccoll_set_scan_wait(ccoll_ctx* c, unsigned int polls) {
  if (!c) return CCOLL_EINVAL;
  c->spin_limit = polls ? polls : kSpinLimit;
  return CCOLL_OK;
}

void ccoll_destroy(ccoll_ctx* c) {
  if (!c) return;
  DeviceGuard g(c->device);
  if (c->stream) (void)hipStreamSynchronize(c->stream); else (void)hipDeviceSynchronize();
  if (c->stat) (void)hipFree(c->stat);
  if (c->offs) (void)hipFree(c->offs);
  if (c->ws) (void)hipFree(c->ws);
  if (c->spill) (void)hipFree(c->spill);
  if (c->host_ws) (void)hipHostFree(c->host_ws);
  delete c;
}

int ccoll_szx_compress_async(ccoll_ctx* c, const float* d_in, size_t n, float abs_eb, void* d_out, size_t out_cap,
                             unsigned long long* d_result) {
  if (!c || !d_out || (!d_in && n) || !eb_valid(abs_eb) || n > ((size_t)1 << 31)) return CCOLL_EINVAL;
  if (((uintptr_t)d_in & 3) || ((uintptr_t)d_out & 3)) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  if (out_cap < kHeader + 4ull * P.nchunks) return CCOLL_ENOSPC;
  c->pipe_open = false;                        // the scan words are about to belong to this stream
  P.in = d_in; P.out = d_out; P.out_cap = out_cap;
  P.eb = abs_eb; P.e_eb = ilogbf(abs_eb); memcpy(&P.eb_bits, &abs_eb, 4);
  P.aligned16 = (((uintptr_t)d_in & 15) == 0);
  if (n == 0) hipLaunchKernelGGL(k_empty_stream, dim3(1), dim3(64), 0, c->stream, P);
  else {
    const u32 ngroups = (P.nchunks + kEncWaves - 1) / kEncWaves;
    const u32 grid = grid_for(c->grid_compress, ngroups);
    P.ticket_sel = c->ticket_sel; c->ticket_sel ^= 1u; P.spill = c->spill;
    launch_main(c, k_compress, dim3(grid), dim3(64 * kEncWaves), P);
  }
  return after_launch(c, P, d_result, true);
}

int ccoll_szx_decompress_range_async(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, size_t first,
                                     size_t count, float* d_out, unsigned long long* d_result) {
  if (!c || !d_in || (!d_out && count) || n > ((size_t)1 << 31)) return CCOLL_EINVAL;
  if (((uintptr_t)d_in & 3) || ((uintptr_t)d_out & 3) || (first % kBlock)) return CCOLL_EINVAL;
  if (first > n || count > n - first) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  if (in_bytes < kHeader + 4ull * P.nchunks) return CCOLL_ECORRUPT;
  P.in = d_in; P.in_bytes = in_bytes; P.out = d_out; P.first = first; P.count = count;
  P.aligned16 = (((uintptr_t)d_out & 15) == 0);
  if (n == 0) {
    hipLaunchKernelGGL(k_check_empty, dim3(1), dim3(64), 0, c->stream, P);
    return after_launch(c, P, d_result, false);
  }
  if (count == 0) { P.c0 = 0; P.c1 = 1; }      // still validates the header, the index and the first chunk
  else { P.c0 = (u32)(first / kChunk); P.c1 = (u32)((first + count + kChunk - 1) / kChunk); }
  c->idx_ptr = nullptr;                        // the offsets in the context are about to be this stream's
  hipLaunchKernelGGL(k_index_scan, dim3((P.nchunks + kScanTile - 1) / kScanTile), dim3(1024), 0, c->stream, P);
  {
    u32 grid = (P.c1 - P.c0 + kDecWaves - 1) / kDecWaves;
    launch_main(c, k_decompress, dim3(grid), dim3(64 * kDecWaves), P);
  }
  return after_launch(c, P, d_result, false);
}

int ccoll_szx_index_async(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, unsigned long long* d_result) {
  if (!c || !d_in || n > ((size_t)1 << 31) || ((uintptr_t)d_in & 3)) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  if (in_bytes < kHeader + 4ull * P.nchunks) return CCOLL_ECORRUPT;
  P.in = d_in; P.in_bytes = in_bytes; P.index_call = 1;
  c->idx_ptr = nullptr;
  if (n == 0) hipLaunchKernelGGL(k_check_empty, dim3(1), dim3(64), 0, c->stream, P);
  else hipLaunchKernelGGL(k_index_scan, dim3((P.nchunks + kScanTile - 1) / kScanTile), dim3(1024), 0, c->stream, P);
  rc = after_launch(c, P, d_result, false);
  if (rc == CCOLL_OK) { c->idx_ptr = d_in; c->idx_bytes = in_bytes; c->idx_n = n; c->idx_epoch = P.epoch; }
  return rc;
}

int ccoll_szx_decompress_range_indexed_async(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, size_t first,
                                             size_t count, float* d_out, unsigned long long* d_result) {
  if (!c || !d_in || (!d_out && count) || n > ((size_t)1 << 31)) return CCOLL_EINVAL;
  if (((uintptr_t)d_out & 3) || (first % kBlock)) return CCOLL_EINVAL;
  if (first > n || count > n - first) return CCOLL_EINVAL;
  if (c->idx_ptr != d_in || c->idx_bytes != in_bytes || c->idx_n != n) return CCOLL_EINVAL;   // not the indexed stream
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  P.in = d_in; P.in_bytes = in_bytes; P.out = d_out; P.first = first; P.count = count;
  P.aligned16 = (((uintptr_t)d_out & 15) == 0);
  P.idx_epoch = c->idx_epoch;                  // an enqueue-only index call may still turn out to have failed
  if (n == 0 || count == 0) return after_launch(c, P, d_result, false);
  P.c0 = (u32)(first / kChunk); P.c1 = (u32)((first + count + kChunk - 1) / kChunk);
  launch_main(c, k_decompress, dim3((P.c1 - P.c0 + kDecWaves - 1) / kDecWaves), dim3(64 * kDecWaves), P);
  return after_launch(c, P, d_result, false);
}

int ccoll_szx_compress_begin(ccoll_ctx* c, size_t n, float abs_eb, void* d_out, size_t out_cap) {
  if (!c || !d_out || !eb_valid(abs_eb) || n == 0 || n > ((size_t)1 << 31) || ((uintptr_t)d_out & 3)) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  if (out_cap < kHeader + 4ull * P.nchunks) return CCOLL_ENOSPC;
  P.out = d_out; P.out_cap = out_cap; memcpy(&P.eb_bits, &abs_eb, 4);
  hipLaunchKernelGGL(k_begin_stream, dim3(1), dim3(64), 0, c->stream, P);
  rc = after_launch(c, P, nullptr, true);
  if (rc) return rc;
  c->pipe_open = true; c->pipe_n = n; c->pipe_cap = out_cap; c->pipe_next = 0; c->pipe_out = d_out; c->pipe_eb = abs_eb;
  c->pipe_epoch = P.epoch;
  return CCOLL_OK;
}

int ccoll_szx_compress_chunks_async(ccoll_ctx* c, const float* d_in, size_t chunk_first, size_t chunk_end,
                                    unsigned long long* d_progress, unsigned long long* d_result) {
  if (!c || !d_in || !c->pipe_open || ((uintptr_t)d_in & 3) || ((uintptr_t)d_progress & 7)) return CCOLL_EINVAL;
  const size_t nchunks = (c->pipe_n + kChunk - 1) / kChunk;
  if (chunk_first != c->pipe_next || chunk_end <= chunk_first || chunk_end > nchunks) return CCOLL_EINVAL;
  if (chunk_end != nchunks && chunk_end % CCOLL_PIECE_CHUNKS) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, c->pipe_n, P);
  if (rc) return rc;
  P.in = d_in; P.out = c->pipe_out; P.out_cap = c->pipe_cap;
  const float eb = c->pipe_eb;
  P.eb = eb; P.e_eb = ilogbf(eb); memcpy(&P.eb_bits, &eb, 4);
  P.aligned16 = (((uintptr_t)d_in & 15) == 0);
  P.c0 = (u32)chunk_first; P.c1 = (u32)chunk_end;
  P.scan_epoch = c->pipe_epoch;                // the scan goes on where the piece before stopped
  P.progress = d_progress;
  const u32 ngroups = (u32)((chunk_end + kEncWaves - 1) / kEncWaves - chunk_first / kEncWaves);
  const u32 grid = grid_for(c->grid_compress, ngroups);
  P.ticket_sel = c->ticket_sel; c->ticket_sel ^= 1u; P.spill = c->spill;
  launch_main(c, k_compress, dim3(grid), dim3(64 * kEncWaves), P);
  rc = after_launch(c, P, d_result, true);
  if (rc) { c->pipe_open = false; return rc; }
  c->pipe_next = chunk_end;
  if (chunk_end == nchunks) c->pipe_open = false;
  return CCOLL_OK;
}

int ccoll_szx_decompress_chunks_async(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, size_t chunk_first,
                                      size_t chunk_end, float* d_out, unsigned long long* d_result) {
  if (!c || !d_in || !d_out || n == 0 || n > ((size_t)1 << 31)) return CCOLL_EINVAL;
  if (((uintptr_t)d_in & 3) || ((uintptr_t)d_out & 3)) return CCOLL_EINVAL;
  const size_t nchunks = (n + kChunk - 1) / kChunk;
  if (chunk_first >= chunk_end || chunk_end > nchunks) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  if (in_bytes < kHeader + 4ull * P.nchunks) return CCOLL_ECORRUPT;
  P.in = d_in; P.in_bytes = in_bytes; P.out = d_out;
  P.first = chunk_first * (size_t)kChunk;
  P.count = (chunk_end * (size_t)kChunk < n ? chunk_end * (size_t)kChunk : n) - P.first;
  P.aligned16 = (((uintptr_t)d_out & 15) == 0);
  P.c0 = (u32)chunk_first; P.c1 = (u32)chunk_end;
  P.scan_chunks = (u32)chunk_end; P.open_stream = 1;       // only what has arrived is checked; the total may not be final
  c->idx_ptr = nullptr;
  hipLaunchKernelGGL(k_index_scan, dim3((P.scan_chunks + kScanTile - 1) / kScanTile), dim3(1024), 0, c->stream, P);
  launch_main(c, k_decompress, dim3((P.c1 - P.c0 + kDecWaves - 1) / kDecWaves), dim3(64 * kDecWaves), P);
  return after_launch(c, P, d_result, false);
}

int ccoll_szx_forward_async(int device, void* hip_stream, void* d_dst, const void* d_src, size_t n,
                            const unsigned long long* d_from, const unsigned long long* d_upto) {
  if (!d_dst || !d_src || !d_upto || n == 0 || n > ((size_t)1 << 31)) return CCOLL_EINVAL;
  if (((uintptr_t)d_dst & 3) || ((uintptr_t)d_src & 3) || ((uintptr_t)d_from & 7) || ((uintptr_t)d_upto & 7)) return CCOLL_EINVAL;
  DeviceGuard g(device);
  if (!g.ok) return CCOLL_EHIP;
  const u32 nchunks = (u32)((n + kChunk - 1) / kChunk);
  hipLaunchKernelGGL(k_forward, dim3(512), dim3(256), 0, (hipStream_t)hip_stream, (unsigned char*)d_dst,
                     (const unsigned char*)d_src, nchunks, d_from, d_upto);
  return HIP_OK(hipGetLastError()) ? CCOLL_OK : CCOLL_EHIP;
}

int ccoll_szx_decompress_ranges_async(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, size_t nranges,
                                      const size_t* first, const size_t* count, float* const* d_out,
                                      unsigned long long* d_result) {
  if (!c || !d_in || n > ((size_t)1 << 31) || ((uintptr_t)d_in & 3)) return CCOLL_EINVAL;
  if (nranges && (!first || !count || !d_out)) return CCOLL_EINVAL;
  for (size_t r = 0; r < nranges; ++r) {
    if ((!d_out[r] && count[r]) || ((uintptr_t)d_out[r] & 3) || (first[r] % kBlock)) return CCOLL_EINVAL;
    if (first[r] > n || count[r] > n - first[r]) return CCOLL_EINVAL;
  }
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  if (in_bytes < kHeader + 4ull * P.nchunks) return CCOLL_ECORRUPT;
  P.in = d_in; P.in_bytes = in_bytes;
  if (n == 0) {
    hipLaunchKernelGGL(k_check_empty, dim3(1), dim3(64), 0, c->stream, P);
    return after_launch(c, P, d_result, false);
  }
  c->idx_ptr = nullptr;                        // the offsets in the context are about to be this stream's
  hipLaunchKernelGGL(k_index_scan, dim3((P.nchunks + kScanTile - 1) / kScanTile), dim3(1024), 0, c->stream, P);
  for (size_t r0 = 0; r0 < nranges; r0 += kMaxRanges) {      // up to 64 ranges per launch: the table is a kernel argument
    RangeTable T;
    memset(&T, 0, sizeof(T));
    u32 wgs = 0, k = 0;
    for (size_t r = r0; r < nranges && k < (u32)kMaxRanges; ++r, ++k) {
      T.first[k] = first[r]; T.count[k] = count[r]; T.out[k] = d_out[r];
      if (count[r]) {
        const u64 c0 = first[r] / kChunk, c1 = (first[r] + count[r] + kChunk - 1) / kChunk;
        wgs += (u32)((c1 - c0 + kDecWaves - 1) / kDecWaves);
      }
      T.wg_end[k] = wgs;
    }
    T.nranges = k;
    if (wgs) launch_main(c, k_decompress_ranges, dim3(wgs), dim3(64 * kDecWaves), P, T);
  }
  return after_launch(c, P, d_result, false);
}

int ccoll_szx_decompress_async(ccoll_ctx* c, const void* d_in, size_t in_bytes, float* d_out, size_t n,
                               unsigned long long* d_result) {
  return ccoll_szx_decompress_range_async(c, d_in, in_bytes, n, 0, n, d_out, d_result);
}

int ccoll_reduce_step_op_async(ccoll_ctx* c, int op, const float* d_local, size_t n, const void* d_cin, size_t cin_bytes,
                               float abs_eb, void* d_cout, size_t cout_cap, unsigned long long* d_result) {
  if (op != CCOLL_OP_SUM && op != CCOLL_OP_MAX && op != CCOLL_OP_MIN) return CCOLL_EINVAL;
  if (!c || !d_cin || !d_cout || (!d_local && n) || !eb_valid(abs_eb) || n > ((size_t)1 << 31)) return CCOLL_EINVAL;
  if (((uintptr_t)d_local & 3) || ((uintptr_t)d_cin & 3) || ((uintptr_t)d_cout & 3)) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  Params P;
  int rc = prepare(c, n, P);
  if (rc) return rc;
  if (cin_bytes < kHeader + 4ull * P.nchunks) return CCOLL_ECORRUPT;
  if (cout_cap < kHeader + 4ull * P.nchunks) return CCOLL_ENOSPC;
  c->pipe_open = false;
  P.local = d_local; P.cin = d_cin; P.in_bytes = cin_bytes; P.out = d_cout; P.out_cap = cout_cap;
  P.eb = abs_eb; P.e_eb = ilogbf(abs_eb); memcpy(&P.eb_bits, &abs_eb, 4);
  P.aligned16 = (((uintptr_t)d_local & 15) == 0);
  if (n == 0) hipLaunchKernelGGL(k_empty_stream, dim3(1), dim3(64), 0, c->stream, P);
  else {
    c->idx_ptr = nullptr;
    hipLaunchKernelGGL(k_index_scan, dim3((P.nchunks + kScanTile - 1) / kScanTile), dim3(1024), 0, c->stream, P);
    const u32 ngroups = (P.nchunks + kRedWaves - 1) / kRedWaves;
    const u32 grid = grid_for(c->grid_reduce, ngroups);
    P.ticket_sel = c->ticket_sel; c->ticket_sel ^= 1u; P.spill = c->spill;
    if (op == CCOLL_OP_MAX) launch_main(c, k_reduce_step_max, dim3(grid), dim3(64 * kRedWaves), P);
    else if (op == CCOLL_OP_MIN) launch_main(c, k_reduce_step_min, dim3(grid), dim3(64 * kRedWaves), P);
    else launch_main(c, k_reduce_step, dim3(grid), dim3(64 * kRedWaves), P);
  }
  return after_launch(c, P, d_result, true);
}

int ccoll_reduce_step_async(ccoll_ctx* c, const float* d_local, size_t n, const void* d_cin, size_t cin_bytes,
                            float abs_eb, void* d_cout, size_t cout_cap, unsigned long long* d_result) {
  return ccoll_reduce_step_op_async(c, CCOLL_OP_SUM, d_local, n, d_cin, cin_bytes, abs_eb, d_cout, cout_cap, d_result);
}

// Address of the static scratch array on `device`, resolved once per device with that device current (every
// device has its own copy at its own address).  Host code never uses the array's name as an address.
static int static_scratch(int device, StaticScratch** out) {
  constexpr int kMaxDevices = 64;
  static StaticScratch* ptrs[kMaxDevices];
  static std::mutex lock;
  if (device < 0 || device >= kMaxDevices) return CCOLL_EINVAL;
  std::lock_guard<std::mutex> hold(lock);
  if (!ptrs[device]) {
    void* p = nullptr;
    if (!HIP_OK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) || !p) return CCOLL_EHIP;
    ptrs[device] = (StaticScratch*)p;
  }
  *out = ptrs[device];
  return CCOLL_OK;
}

int ccoll_szx_decompress_static(int device, void* hip_stream, const void* d_in, size_t in_bytes, float* d_out, size_t n,
                                unsigned long long* d_result) {
  if (!d_in || (!d_out && n) || !d_result) return CCOLL_EINVAL;
  if (n > kStaticMaxElems) return CCOLL_EINVAL;                 // larger streams need a context (ccoll_szx_decompress)
  if (((uintptr_t)d_in & 3) || ((uintptr_t)d_out & 3) || ((uintptr_t)d_result & 7)) return CCOLL_EINVAL;
  DeviceGuard g(device);
  if (!g.ok) return CCOLL_EHIP;
  StaticScratch* sc = nullptr;
  int rc = static_scratch(device, &sc);
  if (rc) return rc;
  hipStream_t stream = (hipStream_t)hip_stream;
  Params P;
  memset(&P, 0, sizeof(P));
  P.n = n; P.nchunks = (u32)((n + kChunk - 1) / kChunk); P.c0 = 0; P.c1 = P.nchunks;
  P.epoch = 1; P.scan_epoch = 1; P.scan_chunks = P.nchunks;     // the words are cleared per call, not tagged
  P.ws = &sc->ws; P.offs = sc->offs; P.spin_limit = kSpinLimit;
  P.in = d_in; P.in_bytes = in_bytes; P.out = d_out; P.first = 0; P.count = n;
  P.aligned16 = (((uintptr_t)d_out & 15) == 0);
  P.result = (u64*)d_result; P.no_total = 1;
  hipLaunchKernelGGL(k_static_begin, dim3(1), dim3(64), 0, stream, &sc->ws);
  if (in_bytes < kHeader + 4ull * P.nchunks) {
    // too short to hold the header and the front index: reported through d_result like every stream error
    hipLaunchKernelGGL(k_static_fail, dim3(1), dim3(64), 0, stream, P);
  } else if (n == 0) {
    hipLaunchKernelGGL(k_check_empty, dim3(1), dim3(64), 0, stream, P);
  } else {
    hipLaunchKernelGGL(k_index_scan, dim3((P.nchunks + kScanTile - 1) / kScanTile), dim3(1024), 0, stream, P);
    hipLaunchKernelGGL(k_decompress, dim3((P.nchunks + kDecWaves - 1) / kDecWaves), dim3(64 * kDecWaves), 0, stream, P);
  }
  hipLaunchKernelGGL(k_publish, dim3(1), dim3(1), 0, stream, P);
  return HIP_OK(hipGetLastError()) ? CCOLL_OK : CCOLL_EHIP;
}

int ccoll_wait(ccoll_ctx* c, size_t* bytes) {
  if (!c) return CCOLL_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return CCOLL_EHIP;
  if (!HIP_OK(hipMemcpyAsync(c->host_ws, c->ws, sizeof(Workspace), hipMemcpyDeviceToHost, c->stream)) ||
      !HIP_OK(hipStreamSynchronize(c->stream))) {
    (void)reset_workspace(c);
    return CCOLL_EHIP;
  }
  const Workspace* h = (const Workspace*)c->host_ws;
  // The error word keeps the latest failing call (and its most severe code): it is reported if that call was
  // enqueued since the previous wait, so that an earlier failure is not hidden by later calls that went well.
  const u64 eep = h->err >> 8, age = (u64)c->epoch - eep;
  const bool mine = eep > (u64)c->waited_epoch && eep <= (u64)c->epoch && (age >= 64 || ((c->own_slot >> age) & 1ull));
  const int status = mine ? -(int)((h->err >> 4) & 0xfu) : 0;
  c->waited_epoch = c->epoch;
  if (bytes) *bytes = c->last_total ? (size_t)h->total : 0;
  if (status && getenv("CCOLL_DEBUG"))
    fprintf(stderr, "libccoll_szx: device status %d (check %u)\n", status, (unsigned)(h->err & 0xfu));
  if (status == CCOLL_ETIMEDOUT) (void)reset_workspace(c);    // leave no stale scan state behind
  return status;
}

int ccoll_szx_compress(ccoll_ctx* c, const float* d_in, size_t n, float abs_eb, void* d_out, size_t out_cap,
                       size_t* out_bytes) {
  if (!out_bytes) return CCOLL_EINVAL;
  *out_bytes = 0;
  int rc = ccoll_szx_compress_async(c, d_in, n, abs_eb, d_out, out_cap, nullptr);
  if (rc) return rc;
  return ccoll_wait(c, out_bytes);
}

int ccoll_szx_decompress(ccoll_ctx* c, const void* d_in, size_t in_bytes, float* d_out, size_t n) {
  int rc = ccoll_szx_decompress_async(c, d_in, in_bytes, d_out, n, nullptr);
  if (rc) return rc;
  return ccoll_wait(c, nullptr);
}

int ccoll_szx_decompress_range(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, size_t first, size_t count,
                               float* d_out) {
  int rc = ccoll_szx_decompress_range_async(c, d_in, in_bytes, n, first, count, d_out, nullptr);
  if (rc) return rc;
  return ccoll_wait(c, nullptr);
}

int ccoll_szx_decompress_ranges(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, size_t nranges,
                                const size_t* first, const size_t* count, float* const* d_out) {
  int rc = ccoll_szx_decompress_ranges_async(c, d_in, in_bytes, n, nranges, first, count, d_out, nullptr);
  if (rc) return rc;
  return ccoll_wait(c, nullptr);
}

int ccoll_szx_index(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n) {
  int rc = ccoll_szx_index_async(c, d_in, in_bytes, n, nullptr);
  if (rc) return rc;
  rc = ccoll_wait(c, nullptr);
  if (rc) c->idx_ptr = nullptr;
  return rc;
}

int ccoll_szx_decompress_range_indexed(ccoll_ctx* c, const void* d_in, size_t in_bytes, size_t n, size_t first,
                                       size_t count, float* d_out) {
  int rc = ccoll_szx_decompress_range_indexed_async(c, d_in, in_bytes, n, first, count, d_out, nullptr);
  if (rc) return rc;
  return ccoll_wait(c, nullptr);
}

int ccoll_reduce_step_op(ccoll_ctx* c, int op, const float* d_local, size_t n, const void* d_cin, size_t cin_bytes,
                         float abs_eb, void* d_cout, size_t cout_cap, size_t* cout_bytes) {
  if (!cout_bytes) return CCOLL_EINVAL;
  *cout_bytes = 0;
  int rc = ccoll_reduce_step_op_async(c, op, d_local, n, d_cin, cin_bytes, abs_eb, d_cout, cout_cap, nullptr);
  if (rc) return rc;
  return ccoll_wait(c, cout_bytes);
}

int ccoll_reduce_step(ccoll_ctx* c, const float* d_local, size_t n, const void* d_cin, size_t cin_bytes, float abs_eb,
                      void* d_cout, size_t cout_cap, size_t* cout_bytes) {
  return ccoll_reduce_step_op(c, CCOLL_OP_SUM, d_local, n, d_cin, cin_bytes, abs_eb, d_cout, cout_cap, cout_bytes);
}


const char* ccoll_strerror(int code) {
  switch (code) {
    case CCOLL_OK: return "ok";
    case CCOLL_EINVAL: return "invalid argument";
    case CCOLL_ENOSPC: return "output capacity too small";
    case CCOLL_ECORRUPT: return "corrupt compressed stream";
    case CCOLL_EHIP: return "HIP runtime error";
    case CCOLL_ETIMEDOUT: return "scan wait timed out (the device made no progress on the launch)";
    default: return "unknown error";
  }
}

}  // extern "C"
